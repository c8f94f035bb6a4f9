"""MI355X-native batch-1 LLaMA decode/prefill hot path behind a C ABI.

``binding`` wraps the HIP library (``csrc/``); ``workloads`` draws the seeded
synthetic inputs.  Nothing is loaded at import time.
"""
