"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before touching a device."""
import ctypes
import os
import re

import pytest

import paper_2603_25011_amd as lsr
from paper_2603_25011_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADERS = [os.path.join(ROOT, "include", n) for n in sorted(os.listdir(os.path.join(ROOT, "include"))) if n.endswith(".h")]


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(lsr.library_path()):
        from paper_2603_25011_amd import build
        build.build()
    return lsr.load_library()


def declared_symbols():
    names = set()
    for h in HEADERS:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names |= set(re.findall(r"\b(lsr_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert {"lsr_head_forward", "lsr_head_backward", "lsr_head_workspace_bytes", "lsr_status_string",
            "lsr_head_forward_profiled", "lsr_head_backward_profiled", "lsr_mfma_peak_probe"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/*.h but not exported"


def test_status_strings(lib):
    seen = {lsr.lsr_status_string(i) for i in range(8)}
    assert len(seen) == 8 and lsr.lsr_status_string(0) == "ok"
    assert lsr.lsr_status_string(99) == "unknown status"


def test_workspace_sizes_scale_as_documented(lib):
    f = lsr.lsr_head_workspace_bytes
    # forward: O(B*S) tables + 8 bytes per vocabulary entry and chunk of tiles (never more chunks than
    # sequences); backward: O(B*V); nothing proportional to B*S*V
    fw = f(64, 512, 1024, 250002, lsr.LSR_BF16, False)
    bw = f(64, 512, 1024, 250002, lsr.LSR_BF16, True)
    assert 4 * 64 * 512 <= fw <= 16 * 64 * 512 + 16384 + 8 * 250002 * (64 * 512 // 1024 + 1)
    assert fw < 8 * 64 * 250002                           # below the size of the outputs Y and I
    long_s = f(128, 8192, 768, 30522, lsr.LSR_BF16, False)
    assert long_s <= 16 * 128 * 8192 + 8 * 128 * 30522 + 16384
    assert 8 * 64 * 250002 <= bw <= 16 * 64 * 250002
    assert bw < 64 * 512 * 250002 // 8
    # long sequences do not blow up the backward count table
    big_s = f(128, 8192, 768, 30522, lsr.LSR_BF16, True)
    assert big_s <= 16 * 128 * 30522 + 8 * 128 * 8192 + 8192
    assert f(0, 1, 8, 1, lsr.LSR_BF16, False) == 0        # invalid shape
    assert f(1, 1, 12, 1, lsr.LSR_BF16, False) == 0       # D not a multiple of 8
    assert f(1, 1, 8, 1, 7, False) == 0                   # unknown dtype


def _fwd(shape, ptrs, ws=(4096, 1 << 30)):
    return binding.lsr_head_forward(*shape, *ptrs, ws, stream=0)


def test_forward_argument_errors_come_before_any_device_work(lib):
    shape = (2, 16, 64, 1000, lsr.LSR_F32)
    good = [4096] * 6                                     # fake, aligned, never dereferenced
    with pytest.raises(lsr.LsrError) as e:
        _fwd(shape, [None] + good[1:])
    assert e.value.status == 1
    with pytest.raises(lsr.LsrError) as e:
        _fwd((2, 16, 60, 1000, lsr.LSR_F32), good)
    assert e.value.status == 2
    with pytest.raises(lsr.LsrError) as e:
        _fwd((2, 16, 64, 1000, 5), good)
    assert e.value.status == 3
    for bad in ((70000, 16, 64, 1000, lsr.LSR_BF16),        # B above 65535
                (2, 40000, 64, 1000, lsr.LSR_BF16),         # S above 32768
                (2, 16, 8200, 1000, lsr.LSR_BF16),          # D above 8192
                (40000, 16, 64, 60000, lsr.LSR_BF16)):      # B*V at or above 2^31
        with pytest.raises(lsr.LsrError) as e:
            _fwd(bad, good)
        assert e.value.status == 2, bad
    with pytest.raises(lsr.LsrError) as e:
        _fwd(shape, [4100] + good[1:])
    assert e.value.status == 4
    with pytest.raises(lsr.LsrError) as e:
        _fwd(shape, good, ws=(4096, 16))
    assert e.value.status == 5
    with pytest.raises(lsr.LsrError) as e:
        _fwd(shape, good, ws=(None, 0))
    assert e.value.status == 5


def test_backward_argument_errors(lib):
    shape = (2, 16, 64, 1000, lsr.LSR_BF16)
    good = [4096] * 8
    with pytest.raises(lsr.LsrError) as e:
        binding.lsr_head_backward(*shape, *([4096, 4096, None] + good[3:]), (4096, 1 << 30), stream=0)
    assert e.value.status == 1
    with pytest.raises(lsr.LsrError) as e:
        binding.lsr_head_backward(*shape, *good, (4096, 8), stream=0)
    assert e.value.status == 5
    with pytest.raises(lsr.LsrError) as e:
        binding.lsr_head_backward(2, 40000, 64, 1000, lsr.LSR_BF16, *good, (4096, 1 << 30), stream=0)
    assert e.value.status == 2


def test_backward_options(lib):
    shape = (2, 16, 64, 70000, lsr.LSR_BF16)
    base = binding.lsr_head_workspace_bytes(*shape, True)
    assert binding.lsr_head_backward_ex_workspace_bytes(*shape, lsr.LSR_F32, False) == base
    assert binding.lsr_head_backward_ex_workspace_bytes(*shape, lsr.LSR_F32, True) == base
    # bfloat16 dH over several vocabulary chunks keeps float32 partial sums: B*S*D*4 more
    staged = binding.lsr_head_backward_ex_workspace_bytes(*shape, lsr.LSR_BF16, False)
    assert base + 2 * 16 * 64 * 4 <= staged <= base + 2 * 16 * 64 * 4 + 256
    # bfloat16 gradients need bfloat16 parameters; unknown dtypes are refused
    assert binding.lsr_head_backward_ex_workspace_bytes(2, 16, 64, 1000, lsr.LSR_F32, lsr.LSR_BF16, False) == 0
    assert binding.lsr_head_backward_ex_workspace_bytes(*shape, 9, False) == 0
    good = [4096] * 8
    with pytest.raises(lsr.LsrError) as e:
        binding.lsr_head_backward_ex(2, 16, 64, 1000, lsr.LSR_F32, *good, lsr.LSR_BF16, False, (4096, 1 << 30), stream=0)
    assert e.value.status == 3
    with pytest.raises(lsr.LsrError) as e:
        binding.lsr_head_backward_ex(*shape, *good, lsr.LSR_BF16, False, (4096, base), stream=0)
    assert e.value.status == 5          # the staged variant needs the larger workspace


def test_profiled_variants_need_a_host_array(lib):
    d = binding._desc(2, 16, 64, 1000, 0)
    rc = lib.lsr_head_forward_profiled(ctypes.byref(d), 4096, 4096, 4096, 4096, 4096, None, 4096, 1 << 30, None, None)
    assert rc == 1


def test_probe_argument_errors(lib):
    out = ctypes.c_double(0.0)
    assert lib.lsr_mfma_peak_probe(1000, 1, None, ctypes.byref(out), None) == 1
    assert lib.lsr_mfma_peak_probe(1000, 1, 4096, None, None) == 1
    assert lib.lsr_mfma_peak_probe(0, 1, 4096, ctypes.byref(out), None) == 2
    assert lib.lsr_mfma_peak_probe(1000, 65, 4096, ctypes.byref(out), None) == 2


def test_without_a_gfx950_device_calls_fail_loudly(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(lsr.LsrError) as e:
        _fwd((2, 16, 64, 1000, lsr.LSR_F32), [4096] * 6)
    assert e.value.status == 6
