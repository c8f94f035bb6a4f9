"""Host logic of the prefill GEMM's work distribution (no GPU): the plan the library computes
must cover every K slab of every column tile exactly once, give every piece of a tile a slice
of its own, and agree with the slice counts the consuming kernels use."""
import pytest

from paper_2604_23467_amd import binding

SHAPES = [(4096, 4096, 3), (4096, 4096, 1), (11008, 4096, 2), (4096, 11008, 1),      # LLaMA-2-7B projections
          (256, 256, 3), (688, 256, 2), (256, 688, 1),                                  # tiny configuration
          (4224, 4224, 3), (1000, 520, 1), (32, 64, 1), (300, 8, 2), (5120, 13824, 1)]
CUS = 256


def walk(plan, N, K, nmat):
    """Pieces (tile, slice, first slab, count) in the order the kernel's workgroups take them."""
    s_real = -(-K // 64)
    tiles = -(-N // 256) * nmat
    S, q = plan["tile_slabs"], plan["quota"]
    total = tiles * S
    pieces = []
    for run in range(plan["runs"]):
        u, u_end = run * q, min(run * q + q, total)
        assert u < u_end, "a run without work"
        while u < u_end:
            tile = u // S
            sl0 = u - tile * S
            span = min(S - sl0, u_end - u)
            u += span
            cnt = min(span, s_real - sl0)
            assert cnt >= 1, "empty piece"
            pieces.append((tile, run - (tile * S) // q, sl0, cnt))
    assert plan["runs"] * q >= total
    return pieces


@pytest.mark.parametrize("rows", [64, 128, 256, 512, 1024])
@pytest.mark.parametrize("shape", SHAPES)
def test_runs_cover_every_slab_once_and_slices_match(shape, rows):
    N, K, nmat = shape
    plan = binding.ll_dbg_gemm_plan(N, K, nmat, rows)
    assert plan["row_tile"] * plan["row_tiles"] == rows
    whole_tiles = plan["quota"] == plan["tile_slabs"]         # one workgroup per tile, no slices to add
    assert plan["runs"] * plan["row_tiles"] <= CUS or whole_tiles     # whoever splits stays within one round
    s_real = -(-K // 64)
    assert plan["tile_slabs"] >= s_real
    ntiles = -(-N // 256)
    by_tile = {}
    for tile, sl, first, cnt in walk(plan, N, K, nmat):
        by_tile.setdefault(tile, []).append((sl, first, cnt))
    assert sorted(by_tile) == list(range(ntiles * nmat))
    for tile, ps in by_tile.items():
        covered = sorted(s for _, first, cnt in ps for s in range(first, first + cnt))
        assert covered == list(range(s_real)), (tile, ps)
        assert sorted(sl for sl, _, _ in ps) == list(range(len(ps))), (tile, ps)
        assert len(ps) <= plan["max_slices"]
        z, nt = divmod(tile, ntiles)
        for col in (z * N + nt * 256, z * N + min(nt * 256 + 255, N - 1)):
            assert binding.ll_dbg_gemm_slice_count(N, K, nmat, rows, col) == len(ps)


def test_plan_keeps_the_chip_busy_at_the_7b_shapes():
    """Every 7B projection gets at least half of the CUs at every bucket (the O projection's K loop
    is too short for more: a run keeps 8 slabs), and tile counts that do not divide over the CUs
    are dealt across tile borders instead of leaving a round part empty."""
    for rows in (64, 128, 256, 512, 1024):
        for N, K, nmat in SHAPES[:4]:
            p = binding.ll_dbg_gemm_plan(N, K, nmat, rows)
            assert p["runs"] * p["row_tiles"] >= 128, (rows, N, K, p)
    p = binding.ll_dbg_gemm_plan(11008, 4096, 2, 512)       # 344 tiles on 256 CUs
    assert p["runs"] * p["row_tiles"] == 256 and p["quota"] > p["tile_slabs"]


def test_row_tiles_of_the_residual_projections_at_128_rows():
    """One matrix of d_model columns (O, down) has few column tiles: at 65..128 rows it runs as two 64-row
    tiles per column tile, everything else at 128 rows as one tile of 128; the slices a consumer adds up
    stay within what the plan reports either way."""
    d, F = 4096, 11008
    for N, K, nmat, bm, tiles in ((d, d, 1, 64, 2), (d, F, 1, 64, 2), (d, d, 3, 128, 1), (F, d, 2, 128, 1)):
        p = binding.ll_dbg_gemm_plan(N, K, nmat, 128)
        assert (p["row_tile"], p["row_tiles"]) == (bm, tiles), (N, K, nmat, p)
        assert p["runs"] * p["row_tiles"] <= 256
    for N, K, nmat in ((d, d, 1), (d, F, 1)):
        assert binding.ll_dbg_gemm_plan(N, K, nmat, 256)["row_tile"] == 128
        assert binding.ll_dbg_gemm_plan(N, K, nmat, 64)["row_tile"] == 64


def test_plan_rejects_bad_arguments():
    for bad in ((0, 64, 1, 64), (64, 0, 1, 64), (64, 64, 4, 64), (64, 64, 1, 100)):
        with pytest.raises(binding.LLError) as e:
            binding.ll_dbg_gemm_plan(*bad)
        assert e.value.code == binding.LL_E_BAD_ARG
    with pytest.raises(binding.LLError):
        binding.ll_dbg_gemm_slice_count(64, 64, 1, 64, 64)


def test_plan_invariants_on_random_shapes():
    """The same coverage property on 300 seeded random shapes (N, K multiples of 8, as the library
    requires of d_model and ffn_hidden)."""
    import numpy as np
    rng = np.random.default_rng(2024)
    for _ in range(300):
        N = int(rng.integers(1, 3000)) * 8
        K = int(rng.integers(1, 2500)) * 8
        nmat = int(rng.integers(1, 4))
        rows = int(rng.choice([64, 128, 256, 512, 1024]))
        plan = binding.ll_dbg_gemm_plan(N, K, nmat, rows)
        s_real = -(-K // 64)
        seen = {}
        for tile, sl, first, cnt in walk(plan, N, K, nmat):
            seen.setdefault(tile, []).append((sl, first, cnt))
        assert len(seen) == -(-N // 256) * nmat
        for tile, ps in seen.items():
            assert sorted(s for _, first, cnt in ps for s in range(first, first + cnt)) == list(range(s_real)), (N, K, nmat, rows, tile)
            assert sorted(sl for sl, _, _ in ps) == list(range(len(ps)))
            assert len(ps) <= plan["max_slices"]
