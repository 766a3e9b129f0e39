"""Parity of the HIP path against the fp64 oracle, element by element, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2603_25011_amd import binding as lsr
from paper_2603_25011_amd import inputs as wl
from paper_2603_25011_amd.harness import DeviceHead
from tests import parity

pytestmark = pytest.mark.gpu


def run_case(inp, mask=None, want_index=True, check_bwd=True):
    head = DeviceHead(inp, mask=mask, want_index=want_index)
    head.poison_outputs()
    head.forward()
    torch.cuda.synchronize()
    Y = head.Y.cpu().numpy()
    I = head.I.cpu().numpy() if want_index else None
    _, _, _, stats = parity.compare_forward(inp, Y, I, mask=mask)
    m = inp.mask if mask is None else mask
    empty = ~(m != 0).any(axis=1)
    assert np.all(Y[empty] == 0.0)
    assert np.all(Y >= 0.0)
    if want_index:
        assert np.all(I[empty] == 0)
    if check_bwd and head.has_backward and want_index:
        head.backward()
        torch.cuda.synchronize()
        dH, dW, db = head.dH.cpu().numpy(), head.dW.cpu().numpy(), head.db.cpu().numpy()
        stats.update(parity.compare_backward(inp, I, dH, dW, db, mask=mask))
        # positions that cannot be selected receive exactly zero
        assert np.all(dH[m == 0] == 0.0)
        # same call again: owner-computes sums are bit-reproducible
        head.backward()
        torch.cuda.synchronize()
        assert torch.equal(head.dH.cpu(), torch.from_numpy(dH))
        assert torch.equal(head.dW.cpu(), torch.from_numpy(dW))
        assert torch.equal(head.db.cpu(), torch.from_numpy(db))
    return stats


def test_c1_tiny_fp32_forward_backward():
    print(run_case(wl.make_inputs(wl.WORKLOADS["c1_tiny_f32"])))


@pytest.mark.parametrize("B,S,D,V,len_lo", [
    (20, 32, 128, 700, 1),      # one 32-row block per sequence, short last tile, ragged V
    (7, 48, 64, 300, 5),        # one or two blocks per sequence
    (5, 100, 192, 513, 3),      # up to four blocks per sequence
    (3, 300, 256, 1000, 200),   # sequences that straddle tiles
    (2, 129, 200, 260, 1),      # K tail (D not a multiple of 64): register-staged loader
    (4, 1, 64, 257, 1),         # S = 1: a plain linear layer
    (9, 700, 64, 96, 1),        # long sequences, single narrow vocabulary tile, one K slab
    (300, 20, 64, 520, 1),      # more sequences than the planning pass scans at once; several row groups
    (40, 260, 128, 300, 100),   # several row groups of several tiles each
    (1, 8, 8, 1, 1),            # smallest legal D, one vocabulary entry
    (2, 16, 128, 70000, 1),     # vocabulary wide enough that the dH gather runs in three vocabulary chunks
    (48, 200, 64, 70000, 1),    # enough workgroups per CU that the row-group cuts are nudged to whole tiles
    (2, 1024, 64, 300, 900),    # longest sequences whose bucket sort still places through LDS
    (2, 1100, 64, 300, 900),    # just beyond: direct placement
    (3, 40, 64, 9000, 1),       # several sort segments per sequence, the last one short
    (260, 256, 64, 4100, 60),   # a batch whose H slice exceeds L2: the dW gather runs in three launches of 87 sequences
    (2, 130, 128, 132000, 40),  # LDS-tile dW kernel: S just above one copy pass, ragged last vocabulary tile; dH slices dealt over XCDs
    (3, 128, 576, 30000, 1),    # LDS-tile dW kernel, one pass; nine column slices: eight owned by XCDs, one shared
    (2, 512, 64, 262200, 300),  # LDS-tile dW kernel at its longest sequence (four passes), one column slice
    (17, 300, 128, 131100, 50), # LDS-tile dW kernel, three passes, S not a multiple of 128; slice-major dH
])
def test_small_bf16_shapes(B, S, D, V, len_lo):
    inp = wl.make_custom(B, S, D, V, seed=B * 1000 + S, len_lo=len_lo)
    print(run_case(inp))


@pytest.mark.parametrize("B,S,D,V", [
    (450, 12, 64, 700),       # more than 384 sequences, D a multiple of 64: whole-row dW kernel beside the sliced dH gather
    (500, 9, 128, 333),
    (3000, 4, 64, 130),       # batches in the thousands (the 48 KiB staging tile of dW is two rows wide)
    (6144, 2, 64, 40),        # the largest batch the backward takes
])
def test_large_batches_whole_row_dw_beside_sliced_dh(B, S, D, V):
    from paper_2603_25011_amd import binding as b
    plan = b.lsr_head_plan(B, S, D, V, b.LSR_BF16)
    assert plan["dw_tile_rows"] == 0 and plan["dh_buckets_per_wave"] > 0
    inp = wl.make_custom(B, S, D, V, seed=B + S, len_lo=1)
    print(run_case(inp))


def test_forward_beyond_the_backward_length_limit():
    # S above 8192 is forward-only
    inp = wl.make_custom(2, 9000, 64, 40, seed=31, len_lo=8000, backward=False)
    print(run_case(inp, check_bwd=False))


def test_fp32_small_shapes():
    print(run_case(wl.make_custom(3, 20, 72, 333, dtype="f32", seed=5, w_std=0.05)))
    # D a multiple of 64 and a vocabulary of three dH chunks
    print(run_case(wl.make_custom(3, 20, 64, 40000, dtype="f32", seed=6, w_std=0.05)))
    # two buckets per wave in the dH gather (about 70 entries per bucket expected)
    print(run_case(wl.make_custom(3, 20, 64, 1000, dtype="f32", seed=8, w_std=0.05)))
    # dW in two launches of 100 sequences (the second adds to the first)
    print(run_case(wl.make_custom(200, 128, 64, 2100, dtype="f32", seed=9, w_std=0.05)))
    # a batch above 192: dW from 16-row tiles whose columns are compacted to the non-zero gradients
    print(run_case(wl.make_custom(200, 6, 64, 100, dtype="f32", seed=7, w_std=0.05)))


def test_scattered_mask_and_empty_rows():
    inp = wl.make_custom(6, 150, 128, 600, seed=77)
    rng = np.random.default_rng(3)
    mask = wl.scattered_mask(rng, 6, 150, keep=0.4)
    mask[2, :] = 0
    mask[4, :] = 0
    mask[4, 149] = 1
    print(run_case(inp, mask=mask))
    inp2 = wl.make_custom(40, 30, 64, 300, seed=78)
    mask2 = wl.scattered_mask(rng, 40, 30, keep=0.3)
    mask2[0, :] = 0
    mask2[39, :] = 0
    print(run_case(inp2, mask=mask2))


def test_forced_exact_ties_pick_lowest_position():
    inp = wl.make_custom(2, 40, 64, 500, seed=9, len_lo=40)
    for arr in (inp.H, inp.H_bits):
        arr[0, 33] = arr[0, 2]
        arr[0, 17] = arr[0, 2]
        arr[1, 39] = arr[1, 0]
    head = DeviceHead(inp)
    head.forward()
    torch.cuda.synchronize()
    I = head.I.cpu().numpy()
    assert not np.any((I[0] == 33) | (I[0] == 17)) and not np.any(I[1] == 39)
    parity.compare_forward(inp, head.Y.cpu().numpy(), I)
    inp = wl.make_custom(1, 600, 64, 300, seed=10, len_lo=600)
    for arr in (inp.H, inp.H_bits):
        arr[0, 599] = arr[0, 100]          # twins in different chunks and different waves
        arr[0, 300] = arr[0, 100]
        arr[0, 200] = arr[0, 7]
    head = DeviceHead(inp)
    head.forward()
    torch.cuda.synchronize()
    I = head.I.cpu().numpy()
    assert not np.any((I == 599) | (I == 300) | (I == 200))
    parity.compare_forward(inp, head.Y.cpu().numpy(), I)


def test_forward_without_index_output():
    inp = wl.make_custom(3, 300, 128, 700, seed=12, len_lo=10)
    print(run_case(inp, want_index=False))
    inp = wl.make_custom(12, 32, 128, 700, seed=13)
    print(run_case(inp, want_index=False))


def test_backward_output_subsets():
    inp = wl.make_custom(4, 64, 128, 520, seed=21)
    head = DeviceHead(inp)
    head.forward()
    head.backward()
    torch.cuda.synchronize()
    ref = (head.dH.clone(), head.dW.clone(), head.db.clone())
    from paper_2603_25011_amd import binding as b
    shape = (head.B, head.S, head.D, head.V, head.dt)
    for keep in ((1, 0, 0), (0, 1, 0), (0, 0, 1), (0, 1, 1)):
        head.poison_outputs()
        head.forward()
        b.lsr_head_backward(*shape, head.H, head.W, head.dY, head.Y, head.I,
                            head.dH if keep[0] else None, head.dW if keep[1] else None,
                            head.db if keep[2] else None, head.ws_bwd)
        torch.cuda.synchronize()
        for k, out, r in zip(keep, (head.dH, head.dW, head.db), ref):
            if k:
                assert torch.equal(out, r)
            else:
                assert torch.isnan(out).all()


def test_c2_document_encoding_forward_full():
    inp = wl.make_inputs(wl.WORKLOADS["c2_doc_fwd"])
    print(run_case(inp, check_bwd=False))


def test_c3_query_encoding_forward_backward_full():
    inp = wl.make_inputs(wl.WORKLOADS["c3_query_fwdbwd"])
    print(run_case(inp))


def test_autograd_wrapper_matches_direct_calls():
    from paper_2603_25011_amd.autograd import lsr_head
    inp = wl.make_custom(5, 70, 128, 640, seed=41, len_lo=3)
    head = DeviceHead(inp)
    head.forward()
    head.backward()
    torch.cuda.synchronize()
    H = head.H.clone().requires_grad_(True)
    W = head.W.clone().requires_grad_(True)
    bias = head.bias.clone().requires_grad_(True)
    Y, I = lsr_head(H, W, bias, head.mask)
    assert torch.equal(Y, head.Y) and torch.equal(I, head.I)
    Y.backward(head.dY)
    torch.cuda.synchronize()
    # the wrapper's own outputs against the oracle; dH and dW arrive in the parameters' dtype (bf16), so
    # they are held to the oracle within one bf16 rounding step instead of the fp32 bound
    I_np = I.cpu().numpy()
    print(parity.compare_forward(inp, Y.detach().cpu().numpy(), I_np)[3])
    print(parity.compare_backward(inp, I_np, H.grad.float().cpu().numpy(), W.grad.float().cpu().numpy(),
                                  bias.grad.cpu().numpy(), bf16_grads=True))
    # same kernels, same order of the float32 sums; the library rounds to the parameter dtype as torch does
    assert torch.equal(H.grad, head.dH.to(torch.bfloat16))
    assert torch.equal(W.grad, head.dW.to(torch.bfloat16))
    assert torch.equal(bias.grad, head.db)
    # only the bias needs a gradient: the other outputs are skipped
    H2, W2, b2 = head.H.clone(), head.W.clone(), head.bias.clone().requires_grad_(True)
    Y2, _ = lsr_head(H2, W2, b2, head.mask)
    Y2.backward(head.dY)
    assert torch.equal(b2.grad, head.db)


def test_random_shapes_and_masks():
    """Two dozen seeded random problems: odd sizes, D from the smallest legal value up, masks of any
    density with empty sequences mixed in, both loaders (D a multiple of 64 or not)."""
    rng = np.random.default_rng(20260325)
    for case in range(24):
        B = int(rng.integers(1, 41))
        S = int(rng.integers(1, 301))
        D = int(rng.choice([8, 16, 24, 64, 72, 128, 192, 200, 256]))
        V = int(rng.integers(1, 1501))
        keep = float(rng.choice([0.05, 0.3, 0.7, 1.0]))
        inp = wl.make_custom(B, S, D, V, seed=5000 + case)
        mask = wl.scattered_mask(rng, B, S, keep=keep)
        if B > 2 and case % 3 == 0:
            mask[int(rng.integers(0, B)), :] = 0
        print(f"case {case}: B={B} S={S} D={D} V={V} keep={keep}", flush=True)
        run_case(inp, mask=mask)


def test_random_shapes_batched_long_and_wide():
    """A dozen seeded problems from the corners the first set does not reach: batches of several
    hundred short sequences (16-row dW tiles, compacted), sequences beyond 1024 positions (direct
    bucket placement, eight buckets per wave), vocabularies of tens of thousands (chunked dH)."""
    rng = np.random.default_rng(20260326)
    for case in range(12):
        kind = case % 3
        if kind == 0:
            B, S, V = int(rng.integers(150, 420)), int(rng.integers(1, 40)), int(rng.integers(1, 2500))
        elif kind == 1:
            B, S, V = int(rng.integers(1, 6)), int(rng.integers(300, 1300)), int(rng.integers(1, 1200))
        else:
            B, S, V = int(rng.integers(1, 5)), int(rng.integers(1, 60)), int(rng.integers(33000, 90000))
        D = int(rng.choice([64, 128])) if kind == 2 else int(rng.choice([8, 24, 64, 128, 192, 200, 256, 320]))
        keep = float(rng.choice([0.02, 0.3, 0.7, 1.0]))
        inp = wl.make_custom(B, S, D, V, seed=7000 + case)
        mask = wl.scattered_mask(rng, B, S, keep=keep)
        print(f"case {case}: B={B} S={S} D={D} V={V} keep={keep}", flush=True)
        run_case(inp, mask=mask)


@pytest.mark.parametrize("B,S,D,V", [
    (5, 70, 128, 900),          # sliced gathers
    (3, 200, 128, 131100),      # LDS-tile dW kernel: the tile copy brings masked rows into LDS
    (4, 50, 72, 300),           # whole-row kernels, register-staged forward loader
])
def test_masked_positions_may_hold_anything(B, S, D, V):
    """Hidden states at masked positions are never multiplied, in the forward or in the backward: with
    NaN and infinities written there every output is bit-identical to the run on the clean input."""
    inp = wl.make_custom(B, S, D, V, seed=77 + B, len_lo=3)
    rng = np.random.default_rng(B)
    mask = wl.scattered_mask(rng, B, S, keep=0.6)
    clean = DeviceHead(inp, mask=mask)
    clean.poison_outputs()
    clean.forward()
    clean.backward()
    torch.cuda.synchronize()
    ref = [t.clone() for t in (clean.Y, clean.I, clean.dH, clean.dW, clean.db)]
    dirty = DeviceHead(inp, mask=mask)
    junk = torch.tensor([float("nan"), float("inf"), -float("inf")], device=dirty.dev)
    pick = torch.randint(0, 3, (B, S, D), device=dirty.dev, generator=torch.Generator(device=dirty.dev).manual_seed(3))
    masked = (dirty.mask == 0).view(B, S, 1).expand(B, S, D)
    dirty.H = torch.where(masked, junk[pick].to(dirty.H.dtype), dirty.H).contiguous()
    dirty.poison_outputs()
    dirty.forward()
    dirty.backward()
    torch.cuda.synchronize()
    for name, got, want in zip(("Y", "I", "dH", "dW", "db"), (dirty.Y, dirty.I, dirty.dH, dirty.dW, dirty.db), ref):
        assert torch.equal(got, want), name
    parity.compare_forward(inp, dirty.Y.cpu().numpy(), dirty.I.cpu().numpy(), mask=mask)


def test_random_shapes_lds_tile_dw():
    """Seeded problems in the range of the LDS-tile dW kernel (128 <= S <= 512, at least 256 workgroups of 1024
    vocabulary rows x 64 columns): few sequences against vocabularies wide enough for that, scattered masks
    with empty sequences, gradients from dense to 2 % non-zero (pairs without gradient read the tile's row
    of zeros; all-zero groups are skipped), D from one column slice to sixteen."""
    from paper_2603_25011_amd import binding as b
    rng = np.random.default_rng(20260327)
    for case in range(8):
        D = int(rng.choice([64, 128, 192, 256, 512, 1024]))
        B = int(rng.integers(1, 5))
        S = int(rng.integers(128, 513)) if case else 512
        V = (256 * 1024 * 64) // D - int(rng.integers(0, 1024)) + (1024 if case % 2 else 3000)
        V = max(V, (255 * 1024 * 64) // D + 1025)             # at least 256 vocabulary tiles x slices
        plan = b.lsr_head_plan(B, S, D, V, b.LSR_BF16)
        assert plan["dw_lds_tile_passes"] == (S + 127) // 128, plan
        keep = float(rng.choice([0.3, 0.7, 1.0]))
        density = float(rng.choice([0.02, 0.3, 1.0]))
        inp = wl.make_custom(B, S, D, V, seed=9000 + case)
        inp.dY[...] = inp.dY * (rng.random(inp.dY.shape) < density)
        mask = wl.scattered_mask(rng, B, S, keep=keep)
        if B > 2 and case % 3 == 0:
            mask[int(rng.integers(0, B)), :] = 0
        print(f"case {case}: B={B} S={S} D={D} V={V} keep={keep} gradient density={density}", flush=True)
        run_case(inp, mask=mask)


@pytest.mark.parametrize("B,S,D,V,len_lo", [
    (5, 70, 128, 640, 3),          # one launch each
    (2, 16, 128, 70000, 1),        # dH over three vocabulary chunks: float32 partial sums staged in the workspace
    (260, 256, 64, 4100, 60),      # dW over three launches of sequences: staged likewise
    (3, 40, 200, 900, 1),          # D not a multiple of 64: whole-row kernels
    (450, 12, 64, 700, 1),         # whole-row dW beside sliced dH
    (3, 200, 128, 131100, 20),     # LDS-tile dW kernel (dW requested) and the sliced gather (db alone)
])
def test_bf16_gradient_outputs_and_accumulation(B, S, D, V, len_lo):
    """lsr_head_backward_ex: bfloat16 dH / dW (compared with the oracle within one bf16 step), and
    accumulation into the caller's buffers for float32 and bfloat16 outputs."""
    from oracle import lsr_head_oracle as orc
    inp = wl.make_custom(B, S, D, V, seed=900 + B, len_lo=len_lo)
    head = DeviceHead(inp)
    head.forward()
    head.backward()
    torch.cuda.synchronize()
    shape = (head.B, head.S, head.D, head.V, head.dt)
    dev = head.dev
    I = head.I.cpu().numpy()
    parity.compare_forward(inp, head.Y.cpu().numpy(), I)
    dH_ref, dW_ref, db_ref, _, _ = orc.backward(inp.H, inp.W, inp.bias, inp.mask, inp.dY, I_override=I)
    f32 = (head.dH.clone(), head.dW.clone(), head.db.clone())

    def run(grad_dtype, accumulate, dH, dW, db):
        ws = torch.empty(lsr.lsr_head_backward_ex_workspace_bytes(*shape, grad_dtype, accumulate), dtype=torch.uint8, device=dev)
        lsr.lsr_head_backward_ex(*shape, head.H, head.W, head.dY, head.Y, head.I, dH, dW, db, grad_dtype, accumulate, ws)
        torch.cuda.synchronize()

    # float32, overwrite: the same launches as lsr_head_backward
    out = [torch.full_like(t, float("nan")) for t in f32]
    run(lsr.LSR_F32, False, *out)
    for a, b_ in zip(out, f32):
        assert torch.equal(a, b_)
    # bfloat16, overwrite
    dH16 = torch.full((B, S, D), float("nan"), dtype=torch.bfloat16, device=dev)
    dW16 = torch.full((V, D), float("nan"), dtype=torch.bfloat16, device=dev)
    db32 = torch.full((V,), float("nan"), device=dev)
    run(lsr.LSR_BF16, False, dH16, dW16, db32)
    parity.check_close_bf16("dH bf16", dH16.float().cpu().numpy(), dH_ref)
    parity.check_close_bf16("dW bf16", dW16.float().cpu().numpy(), dW_ref)
    assert torch.equal(db32, f32[2])
    # one rounding of the float32 result, exactly
    assert torch.equal(dH16, f32[0].to(torch.bfloat16)) and torch.equal(dW16, f32[1].to(torch.bfloat16))
    # float32, accumulate into buffers that already hold something
    g = torch.Generator(device=dev)
    g.manual_seed(5)
    base = [torch.randn(t.shape, device=dev, generator=g) for t in f32]
    out = [t.clone() for t in base]
    run(lsr.LSR_F32, True, *out)
    for name, a, b0, ref in zip(("dH", "dW", "db"), out, base, (dH_ref, dW_ref, db_ref)):
        parity.check_close(name + " accumulated", a.cpu().numpy(), b0.cpu().numpy().astype(np.float64) + ref)
    # bfloat16, accumulate
    b16 = [base[0].to(torch.bfloat16), base[1].to(torch.bfloat16)]
    dH16, dW16, db32 = b16[0].clone(), b16[1].clone(), base[2].clone()
    run(lsr.LSR_BF16, True, dH16, dW16, db32)
    parity.check_close_bf16("dH bf16 accumulated", dH16.float().cpu().numpy(), b16[0].float().cpu().numpy().astype(np.float64) + dH_ref)
    parity.check_close_bf16("dW bf16 accumulated", dW16.float().cpu().numpy(), b16[1].float().cpu().numpy().astype(np.float64) + dW_ref)
    parity.check_close("db accumulated", db32.cpu().numpy(), base[2].cpu().numpy().astype(np.float64) + db_ref)
    # subsets of outputs
    dW16b = torch.full((V, D), float("nan"), dtype=torch.bfloat16, device=dev)
    run(lsr.LSR_BF16, False, None, dW16b, None)
    assert torch.equal(dW16b, f32[1].to(torch.bfloat16))
    db_only = torch.full((V,), float("nan"), device=dev)
    run(lsr.LSR_F32, False, None, None, db_only)
    assert torch.equal(db_only, f32[2])


def test_two_host_threads_on_two_streams():
    """Two host threads call forward + backward concurrently, each on its own stream, buffers and small
    problem (small problems fork the dW gather onto the library's shared auxiliary stream).  Every call
    of both threads must match the oracle."""
    import threading
    inps = [wl.make_custom(6, 70, 128, 900, seed=101, len_lo=3), wl.make_custom(9, 33, 64, 1500, seed=102, len_lo=1)]
    errors = []
    results = [[], []]

    def worker(k):
        try:
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                head = DeviceHead(inps[k])
                for it in range(20):
                    head.poison_outputs()
                    head.forward()
                    head.backward()
                    stream.synchronize()
                    results[k].append(tuple(t.cpu().numpy().copy() for t in (head.Y, head.I, head.dH, head.dW, head.db)))
        except Exception as exc:          # surfaced in the main thread
            errors.append((k, repr(exc)))

    threads = [threading.Thread(target=worker, args=(k,)) for k in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for k, inp in enumerate(inps):
        assert len(results[k]) == 20
        Y, I, dH, dW, db = results[k][0]
        parity.compare_forward(inp, Y, I)
        parity.compare_backward(inp, I, dH, dW, db)
        for other in results[k][1:]:      # deterministic kernels: every later call is bit-identical to the checked one
            for a, b_ in zip(results[k][0], other):
                assert np.array_equal(a, b_)


def test_mfma_probe_reports_a_plausible_rate():
    from paper_2603_25011_amd import binding as b
    sink = torch.zeros(1, dtype=torch.float32, device="cuda:0")
    tf = b.lsr_mfma_peak_probe(20000, 2, sink)
    print(f"register-only bf16 MFMA rate: {tf:.0f} TFLOP/s")
    assert 800.0 < tf < 2600.0          # between a third of and just above the nominal 2.5 PFLOP/s
    assert float(sink.item()) == 0.0    # nothing is ever stored
