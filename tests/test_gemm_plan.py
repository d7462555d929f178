"""Host logic of the matrix-core GEMM launch policy (no GPU): invariants over a sweep of problem shapes.

The policy picks a workgroup tile (rows x columns) and a number of splits along k.  Whatever it picks must be a shape
the kernels can run correctly: the tile is one of the compiled ones, every split owns at least one 64-deep slice (an
empty split would leave its partial-sum slab unwritten), the slabs fit the scratch area, and epilogues that need the
whole sum (SiLU(gate)*up, LM head) are never split."""
import itertools

import pytest

from paper_2509_24007_amd import sdlm

SLAB_FLOATS = 16 << 20
STORE, RESID, SWIGLU, LMHEAD = 0, 1, 2, 3


def slices_per_split(k, splits):
    s = k // 64
    return (s + splits - 1) // splits


@pytest.mark.parametrize("epi", [STORE, RESID, SWIGLU, LMHEAD])
def test_policy_invariants(epi):
    rows_list = [1, 5, 8, 31, 32, 33, 48, 64, 65, 100, 144, 160, 192, 256, 323, 384, 512, 960, 2048, 4096]
    n_list = [128, 130, 512, 1088, 2048, 2560, 3584, 4608, 5120, 7168, 8960, 18944, 27648, 151936]
    k_list = [64, 128, 192, 1536, 2048, 2688, 3584, 5120, 8960, 18944, 27648]
    seen = set()
    for rows, n, k in itertools.product(rows_list, n_list, k_list):
        for min_rows in {0, rows, max(1, rows // 2), max(1, (rows * 5) // 8)}:
            tr, tc, sp = sdlm.gemm_plan(epi, rows, min_rows, n, k)
            seen.add((tr, tc))
            assert tr in (32, 64, 128, 192) and tc in (128, 256, 512), (rows, n, k, tr, tc)
            assert tr != 192 or (epi == SWIGLU and tc == 256)                 # the 192-row tile exists for gate/up only
            assert tc >= 256 or epi in (STORE, RESID)                          # the narrow tile has only the plain epilogues
            if tc == 512:
                # the eight-wavefront tile: 128 rows, never split, only where the four-wavefront launch would have put more
                # workgroups on the chip than it has compute units; not compiled for the plain-store and LM-head epilogues
                assert tr == 128 and sp == 1 and epi in (RESID, SWIGLU)
                col_blocks4 = -(-n // 128) if epi == SWIGLU else -(-n // 256)
                sure_row_blocks = max(1, min(-(-rows // 128), -(-min_rows // 128))) if min_rows > 0 else -(-rows // 128)
                assert col_blocks4 * sure_row_blocks > 256, (rows, min_rows, n, k)
            if rows <= 32:
                assert tr == 32
            assert sp >= 1
            if epi in (SWIGLU, LMHEAD):
                assert sp == 1
            per = slices_per_split(k, sp)
            assert (sp - 1) * per < k // 64 <= sp * per, f"empty or missing split: rows={rows} n={n} k={k} splits={sp}"
            if sp > 1:
                assert sp * rows * n <= SLAB_FLOATS, (rows, n, k, sp)
                assert sp <= 16
    if epi in (STORE, RESID):
        assert (128, 128) in seen and (128, 256) in seen and (32, 128) in seen      # the sweep reaches both widths


def test_policy_on_the_benchmark_shapes():
    # the 7B shape at 323 typical rows (capacity 512, 320 certain): one workgroup per compute unit for the long-k
    # projection, few splits for the short-k ones, the 192-row tile only for the 32B gate/up
    assert sdlm.gemm_plan(RESID, 512, 320, 3584, 18944) == (128, 256, 6)
    tr, tc, sp = sdlm.gemm_plan(RESID, 512, 320, 3584, 3584)
    assert sp <= 3
    tr, tc, sp = sdlm.gemm_plan(STORE, 512, 320, 4608, 3584)
    assert sp <= 3
    assert sdlm.gemm_plan(SWIGLU, 512, 320, 18944, 3584) == (128, 512, 1)             # 444 workgroups of four wavefronts: eight instead
    assert sdlm.gemm_plan(SWIGLU, 256, 160, 27648, 5120) == (192, 256, 1)
    assert sdlm.gemm_plan(SWIGLU, 256, 144, 11008, 2048)[0] == 128               # too few column blocks for the tall tile
    assert sdlm.gemm_plan(LMHEAD, 256, 256, 151936, 3584) == (128, 256, 1)
    # a 4096-row prefill pass of the 7B shape: unsplit everywhere; the residual projections and gate/up take the wide tile
    assert sdlm.gemm_plan(RESID, 4096, 4096, 3584, 18944) == (128, 512, 1)
    assert sdlm.gemm_plan(SWIGLU, 4096, 4096, 18944, 3584) == (128, 512, 1)
    assert sdlm.gemm_plan(STORE, 4096, 4096, 4608, 3584) == (128, 256, 1)


def test_plan_rejects_bad_arguments():
    with pytest.raises(sdlm.SdlmError):
        sdlm.gemm_plan(0, 0, 0, 128, 128)
    with pytest.raises(sdlm.SdlmError):
        sdlm.gemm_plan(0, 8, 0, 128, 100)
    with pytest.raises(sdlm.SdlmError):
        sdlm.gemm_plan(7, 8, 0, 128, 128)
