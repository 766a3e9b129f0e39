"""The launch plan the host derives from a shape (lsr_head_plan): documented values for the benchmark
shapes and the invariants the kernels rely on, over a few thousand random shapes.  No GPU needed."""
import ctypes

import numpy as np
import pytest

import paper_2603_25011_amd as lsr
from paper_2603_25011_amd import binding


@pytest.fixture(scope="module", autouse=True)
def lib():
    import os
    if not os.path.exists(lsr.library_path()):
        from paper_2603_25011_amd import build
        build.build()
    return lsr.load_library()


def test_plans_of_the_benchmark_shapes():
    p = lsr.lsr_head_plan(64, 512, 1024, 250002, lsr.LSR_BF16)          # C5
    assert p == {"fwd_tiles_per_chunk": 4, "fwd_chunks": 32, "fwd_segment_rows": 32, "fwd_resident_workgroups": 0,
                 "sort_segments": 64, "sort_segment_len": 3968, "sort_places_through_lds": 1,
                 "dh_chunks": 8, "dh_chunk_len": 31251, "dh_buckets_per_wave": 2, "dw_tile_rows": 64,
                 "dw_sequences_per_launch": 64, "dh_slices_owned_by_xcd": 0, "dw_lds_tile_passes": 4}
    p = lsr.lsr_head_plan(16, 256, 768, 250002, lsr.LSR_BF16)           # C4: longer buckets, one per wave
    assert (p["dh_chunks"], p["dh_buckets_per_wave"], p["dw_tile_rows"]) == (8, 1, 64)
    # a small batch: dH slices owned by XCDs; S = 256: the LDS-tile dW kernel with two copy passes per tile
    assert (p["dh_slices_owned_by_xcd"], p["dw_lds_tile_passes"]) == (1, 2)
    p = lsr.lsr_head_plan(256, 32, 768, 30522, lsr.LSR_BF16)            # C3: one pass over a 30k vocabulary, 16-row dW tiles
    assert (p["dh_chunks"], p["dh_buckets_per_wave"], p["dw_tile_rows"]) == (1, 1, 16)
    # short sequences: 8-row segments; a shallow grid: resident workgroups over one-tile units
    assert (p["fwd_tiles_per_chunk"], p["fwd_chunks"], p["fwd_segment_rows"], p["fwd_resident_workgroups"]) == (1, 32, 8, 1)
    assert (p["dh_slices_owned_by_xcd"], p["dw_lds_tile_passes"]) == (0, 0)      # S below the LDS-tile kernel's range
    p = lsr.lsr_head_plan(128, 8192, 768, 30522, lsr.LSR_BF16)          # long sequences: short buckets, direct placement
    assert (p["dh_buckets_per_wave"], p["sort_places_through_lds"], p["dh_chunks"]) == (8, 0, 1)
    assert p["dw_lds_tile_passes"] == 0                                 # a sequence's slice does not fit an LDS tile
    # the LDS-tile dW kernel needs a workgroup per CU: 1024 vocabulary rows x 64 columns each
    assert lsr.lsr_head_plan(32, 256, 128, 30522, lsr.LSR_BF16)["dw_lds_tile_passes"] == 0      # 30 x 2 workgroups
    assert lsr.lsr_head_plan(32, 256, 768, 30522, lsr.LSR_BF16)["dw_lds_tile_passes"] == 2      # 30 x 12
    assert lsr.lsr_head_plan(32, 256, 768, 30522, lsr.LSR_F32)["dw_lds_tile_passes"] == 0       # bfloat16 only
    assert lsr.lsr_head_plan(32, 513, 768, 30522, lsr.LSR_BF16)["dw_lds_tile_passes"] == 0
    assert lsr.lsr_head_plan(32, 127, 768, 30522, lsr.LSR_BF16)["dw_lds_tile_passes"] == 0
    assert lsr.lsr_head_plan(17, 128, 768, 30522, lsr.LSR_BF16)["dh_slices_owned_by_xcd"] == 0
    p = lsr.lsr_head_plan(256, 512, 768, 250002, lsr.LSR_BF16)          # a batch whose H slice is 4x L2: four dW launches
    assert (p["dw_sequences_per_launch"], p["dw_tile_rows"]) == (64, 64)
    p = lsr.lsr_head_plan(3, 40, 200, 900, lsr.LSR_BF16)                # D not a multiple of 64: whole-row kernels
    assert (p["dh_buckets_per_wave"], p["dw_tile_rows"], p["dh_chunks"]) == (0, 0, 1)


def test_plan_invariants_on_random_shapes():
    rng = np.random.default_rng(11)
    for _ in range(3000):
        B = int(rng.choice([1, 2, 7, 16, 64, 192, 193, 256, 384, 385, 1000, 6144]))
        S = int(rng.choice([1, 5, 32, 33, 512, 1024, 1025, 4096, 8192]))
        D = int(rng.choice([8, 64, 72, 128, 768, 1024, 4096]))
        V = int(rng.choice([1, 63, 512, 4097, 30522, 32769, 65536, 250002, 1000003]))
        if B * V >= 2 ** 31 or B * S >= 2 ** 31:
            continue
        for dt, esize in ((lsr.LSR_BF16, 2), (lsr.LSR_F32, 4)):
            p = lsr.lsr_head_plan(B, S, D, V, dt)
            n_seg, seg_len = p["sort_segments"], p["sort_segment_len"]
            assert n_seg >= 1 and seg_len % 64 == 0 and n_seg * seg_len >= V and (n_seg - 1) * seg_len < V
            assert n_seg == 1 or n_seg * S <= V + S              # count table stays within about B*V ints
            if S <= 1024:
                assert seg_len <= 4096 and p["sort_places_through_lds"] == 1
            else:
                assert p["sort_places_through_lds"] == 0
            c, clen = p["dh_chunks"], p["dh_chunk_len"]
            assert 1 <= c <= 64 and c * clen >= V and (c - 1) * clen < V
            if D % 64 != 0:
                assert c == 1 and p["dh_buckets_per_wave"] == 0 and p["dw_tile_rows"] == 0
            else:
                assert p["dh_buckets_per_wave"] in ((1, 2, 4) if dt == lsr.LSR_F32 else (1, 2, 4, 8))
                assert c == 1 or c <= V * esize // (32 * S)      # re-reading dH stays below a quarter of the gathers
                assert c == 1 or clen * 64 * esize <= (4 << 20) or c == 64 or c == V * esize // (32 * S)
                rows, nb = p["dw_tile_rows"], p["dw_sequences_per_launch"]
                assert 1 <= nb <= B and (B + nb - 1) // nb <= 16
                assert rows in (0, 16, 32, 64) and nb * rows * 8 <= 48 * 1024
                assert (rows == 0) == (nb * 16 * 8 > 48 * 1024)
                # several launches only where rows of H are reused often, and few enough that re-reading dW stays small
                assert nb == B or (V >= 16 * S and (B + nb - 1) // nb <= min(16, 1 + B * esize // 32))
            seg = p["fwd_segment_rows"]
            assert seg == (8 if S <= 64 else 32)
            segs = B * ((S + seg - 1) // seg)
            tiles_max = (segs * seg + 255) // 256
            assert p["fwd_tiles_per_chunk"] >= 1 and p["fwd_chunks"] <= B
            assert (p["fwd_chunks"] - 1) * p["fwd_tiles_per_chunk"] < tiles_max <= p["fwd_chunks"] * p["fwd_tiles_per_chunk"]
            # forward workspace: O(B*S) tables, plus one (max, position) slot per chunk and vocabulary entry
            # where a chunk boundary can fall inside a sequence (bf16 path, S above one block)
            fw = lsr.lsr_head_workspace_bytes(B, S, D, V, dt, False)
            tables = 4 * B + 4 * B * S + 4 * (B + 1) + 4 * segs + 8 * seg * segs
            parts = 8 * p["fwd_chunks"] * V if (dt == lsr.LSR_BF16 and S > seg and p["fwd_chunks"] > 1) else 0
            assert tables + parts <= fw <= tables + parts + 8 * 256
            # the backward workspace holds what the plan implies
            # (the sorted (v, g) lists are followed by 256 entries of slack that the dH gather may read, never write)
            need = 8 * (B * V + 256) + 4 * B * n_seg * S + 4 * B * (S + 1) + (4 * B * S * (c + 1) if c > 1 else 0)
            if S <= 8192 and B <= 6144:
                ws = lsr.lsr_head_workspace_bytes(B, S, D, V, dt, True)
                assert need <= ws <= need + 4 * 256


def test_plan_argument_errors(lib):
    out = (ctypes.c_int32 * 16)()
    d = binding._desc(2, 16, 64, 1000, lsr.LSR_BF16)
    assert lib.lsr_head_plan(ctypes.byref(d), None) == 1
    bad = binding._desc(2, 16, 60, 1000, lsr.LSR_BF16)
    assert lib.lsr_head_plan(ctypes.byref(bad), out) == 2
    assert lib.lsr_head_plan(None, out) == 1
