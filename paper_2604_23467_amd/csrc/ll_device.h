// Device-side types and wave-level helpers shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef _Float16 half_t;
typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

// Per-step dynamic values.  They live in device memory so that one captured
// graph serves every position: kernels read them, the last kernel of a step
// advances them (the paper keeps these on the host, Sec. III-A "dynamic
// operations"; here they never leave the GPU).
struct DevState {
  int32_t pos;         // cached positions = position of the token fed next
  int32_t next_token;  // token the next decode step feeds
  int32_t n_prompt;    // prompt length of the prefill in flight
  int32_t steps;       // tokens produced since reset (index into the host ring)
  int32_t fault;       // set by a kernel whose bounded wait for another workgroup ran out: the step reports token -1
  int32_t pad[11];
};

#define LL_WAVE 64
#define LL_WG 256

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over aligned groups of N lanes (N = 8 or 16) with DPP only: two quad
// permutes, then a mirror inside each half row, then a mirror of the row.
template <int N>
__device__ __forceinline__ float group_sum(float v) {
  v += dpp_mov<0xB1>(v);   // quad_perm [1,0,3,2]
  v += dpp_mov<0x4E>(v);   // quad_perm [2,3,0,1]
  v += dpp_mov<0x141>(v);  // row_half_mirror
  if (N == 16) v += dpp_mov<0x140>(v);  // row_mirror
  return v;
}

// Sum over the 64 lanes of a wave; the result is wave-uniform.
__device__ __forceinline__ float wave_sum(float v) {
  v = group_sum<16>(v);
  int b = __builtin_bit_cast(int, v);
  float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

// Pointers that were themselves loaded from memory (e.g. a per-layer pointer
// table) are "generic" to the compiler, which then emits FLAT loads; those count
// against the LDS counter as well, so every LDS wait and every workgroup
// barrier would also wait for weight loads still in flight.  All device
// buffers here live in global memory: say so.
#define LL_GLOBAL __attribute__((address_space(1)))
template <class T>
__device__ __forceinline__ const LL_GLOBAL T* as_global(const T* p) {
  return (const LL_GLOBAL T*)p;
}
template <class T>
__device__ __forceinline__ LL_GLOBAL T* as_global(T* p) {
  return (LL_GLOBAL T*)p;
}

// Device-scope accesses for data that one workgroup writes and another reads INSIDE one launch.
// The 8 XCDs have private L2s: relaxed device-scope atomic stores go through to memory and
// device-scope atomic loads do not stop at a stale line, so they are coherent across the L2s on
// their own.  Ordering comes from completion: a producer drains its vector-memory counter before
// it signals.  No release / acquire fences: a device-scope release writes back the whole L2.
__device__ __forceinline__ float ld_dev(const float* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev(float* p, float v) {
  __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev_i(int* p, int v) {
  __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ int ld_dev_i(const int* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev_h(half_t* p, float v) {
  const half_t h = (half_t)v;
  __hip_atomic_store(as_global(reinterpret_cast<unsigned short*>(p)), __builtin_bit_cast(unsigned short, h),
                     __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float2 ld_dev2(const float* p) {
  const unsigned long long u = __hip_atomic_load(as_global(reinterpret_cast<const unsigned long long*>(p)),
                                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return make_float2(__builtin_bit_cast(float, (unsigned)(u & 0xffffffffu)),
                     __builtin_bit_cast(float, (unsigned)(u >> 32)));
}
struct U64x2 { unsigned long long v[2]; };
__device__ __forceinline__ h8 ld_dev_h8(const half_t* p) {   // 16 bytes as two 8-byte device-scope loads
  const LL_GLOBAL unsigned long long* q = as_global(reinterpret_cast<const unsigned long long*>(p));
  U64x2 t;
  t.v[0] = __hip_atomic_load(q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  t.v[1] = __hip_atomic_load(q + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  return __builtin_bit_cast(h8, t);
}

__device__ __forceinline__ unsigned ld_dev_u(const unsigned* p) {
  return __hip_atomic_load(as_global(p), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_dev_u(unsigned* p, unsigned v) {
  __hip_atomic_store(as_global(p), v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// 16-byte streaming load of weights that are read exactly once per step.
__device__ __forceinline__ h8 load_stream(const half_t* p) {
  return __builtin_nontemporal_load(as_global(reinterpret_cast<const h8*>(p)));
}
// s_waitcnt vmcnt(N) (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the export and LDS counters
// left at "no wait")
template <int N>
__device__ __forceinline__ void wait_vm_at_most() {
  __builtin_amdgcn_s_waitcnt((N & 15) | 0x70 | 0xF00 | ((N >> 4) << 14));
}

// s_waitcnt lgkmcnt(N): at most N LDS operations of this wave still outstanding (they complete in order);
// the vector-memory and export counters left at "no wait"
template <int N>
__device__ __forceinline__ void wait_lgkm_at_most() {
  static_assert(N >= 0 && N < 16, "lgkmcnt is a 4-bit counter");
  __builtin_amdgcn_s_waitcnt(0xC00F | 0x70 | (N << 8));
}

// plain 16-byte load from global memory
__device__ __forceinline__ h8 load_h8(const half_t* p) {
  return *as_global(reinterpret_cast<const h8*>(p));
}

__device__ __forceinline__ float dot8(h8 w, f4 x0, f4 x1, float acc) {
  acc += (float)w[0] * x0[0];
  acc += (float)w[1] * x0[1];
  acc += (float)w[2] * x0[2];
  acc += (float)w[3] * x0[3];
  acc += (float)w[4] * x1[0];
  acc += (float)w[5] * x1[1];
  acc += (float)w[6] * x1[2];
  acc += (float)w[7] * x1[3];
  return acc;
}

// "Fragment-major" layout of an fp16 activation matrix of 16*TB token rows that feeds the
// short-prompt kernels' MFMA B operand: the 16 bytes lane (16 g + r) needs for K step s and
// token block t (token 16 t + r, k = 32 s + 8 g .. + 8) are stored at lane-consecutive
// addresses, so a wave's fragment is one contiguous 1 KB load.  Offset in halves of element
// (tok, k); tb = 0 selects plain row-major with row length K.
__host__ __device__ __forceinline__ size_t act_offset(int tok, int k, int K, int tb) {
  if (tb == 0) return (size_t)tok * K + k;
  return ((size_t)((k >> 5) * tb + (tok >> 4)) * 64 + ((k >> 3) & 3) * 16 + (tok & 15)) * 8 + (k & 7);
}

// Where the prefill projection GEMM leaves its output: the K loop of all 256-column tiles is cut
// into runs of `quota` 64-wide slabs, one run per workgroup (see prefill_gemm.h), and every run
// stores its part of a tile's product into a slice of its own.  Column tile nt (counted over
// the concatenated outputs of the GEMM's matrices) owns slabs nt * nslabs .. + nslabs - 1 of
// that sequence, so its product is the sum of the slices 0 .. slice_count - 1.
struct SliceMap {
  int nslabs;             // 64-wide K slabs per tile
  int quota;              // slabs per workgroup
  int ntiles;             // 256-column tiles per matrix
  int N;                  // columns per matrix
  size_t slice_floats;    // floats per slice ([rows][ldc])
};

__host__ __device__ __forceinline__ int slice_count(const SliceMap& m, int col) {
  const int z = col / m.N;
  const int u0 = (z * m.ntiles + ((col - z * m.N) >> 8)) * m.nslabs;
  return (u0 + m.nslabs - 1) / m.quota - u0 / m.quota + 1;
}
