"""The projection entry point that allocates nothing (`pat_op_gemm_static`: partial sums of a K split
across workgroups in an array inside the library's code object) against `pat_op_gemm` with a caller's
scratch buffer: same kernels, same summation order, so the results must be bit-identical.  Two calls in
a row, the second with a smaller input, so that what the first call left in the shared array would show
if the second read any of it."""
import ctypes

import numpy as np
import pytest
import torch

import pat_inputs as pi
from gpu_util import DEV

pytestmark = pytest.mark.gpu


def _case(pat, n, k, b, mode, seed):
    lib = pat.load_library()
    idx = torch.arange(n * k, dtype=torch.int64, device=DEV)
    w = pi.normal_bf16(pi.stream_key(0x57A7, seed), idx, 0.05).view(n, k)
    wp = pat.pat_op_pack_weight(w[: n // 2], w[n // 2:]) if mode == 2 else pat.pat_op_pack_weight(w)
    x = torch.randn(b, k, device=DEV, generator=torch.Generator(device=DEV).manual_seed(seed))
    hi, lo = pat.pat_op_pack_act(x)
    need = lib.pat_op_gemm_scratch_bytes(n, k, b)
    assert 0 < need <= (32 << 20), f"shape ({n}, {k}, {b}) does not use the scratch buffer ({need} bytes): pick another"
    outs = []
    for fn in (pat.pat_op_gemm, pat.pat_op_gemm_static):
        if mode == 2:
            nb = lib.pat_op_packed_act_bytes(b, n // 2)
            yh = torch.zeros(nb, dtype=torch.uint8, device=DEV); yl = torch.zeros_like(yh)
            fn(wp, n, k, hi, lo, b, None, mode=2, y_hi=yh, y_lo=yl)
            outs.append(torch.cat([yh, yl]).cpu().numpy())
        else:
            y = torch.full((b, n), 0.25, device=DEV)
            fn(wp, n, k, hi, lo, b, y, mode=mode)
            outs.append(y.cpu().numpy().view(np.uint32))
    return outs


def test_static_scratch_matches_caller_scratch_on_two_calls_in_a_row():
    import paper_2605_23945_amd as pat
    # first call: 8 K slices of partial sums (8 MiB); second call: a smaller projection and batch whose partial
    # sums cover only the start of what the first call wrote
    big = _case(pat, 4096, 4096, 64, 1, 1)
    assert np.array_equal(big[0], big[1])
    small = _case(pat, 1024, 2048, 40, 0, 2)
    assert np.array_equal(small[0], small[1])
    swi = _case(pat, 2 * 352, 4096, 50, 2, 3)                     # gate/up interleave with the SwiGLU epilogue
    assert np.array_equal(swi[0], swi[1])
    again = _case(pat, 4096, 4096, 64, 1, 1)                      # and the first shape once more over the leftovers
    assert np.array_equal(again[1], big[1])


def test_static_scratch_rejects_what_does_not_fit_and_needs_none_for_small_batches():
    import paper_2605_23945_amd as pat
    lib = pat.load_library()
    # a shape whose partial sums exceed the array: refused before anything is enqueued
    n, k, b = 22016, 4096, 256
    assert lib.pat_op_gemm_scratch_bytes(n, k, b) > (32 << 20)
    dummy = torch.zeros(64, dtype=torch.uint8, device=DEV)
    rc = lib.pat_op_gemm_static(dummy.data_ptr(), n, k, dummy.data_ptr(), dummy.data_ptr(), b, dummy.data_ptr(), n,
                                None, None, 0, None)
    assert rc == pat.binding.PAT_ENOMEM
    # live batch <= 32: one workgroup walks all of K, no partial sums at all; the entry point still works
    w = pi.normal_bf16(pi.stream_key(0x57A7, 9), torch.arange(256 * 512, dtype=torch.int64, device=DEV), 0.05).view(256, 512)
    wp = pat.pat_op_pack_weight(w)
    x = torch.randn(5, 512, device=DEV, generator=torch.Generator(device=DEV).manual_seed(4))
    hi, lo = pat.pat_op_pack_act(x)
    y0 = torch.empty(5, 256, device=DEV); y1 = torch.empty(5, 256, device=DEV)
    pat.pat_op_gemm(wp, 256, 512, hi, lo, 5, y0, mode=0)
    pat.pat_op_gemm_static(wp, 256, 512, hi, lo, 5, y1, mode=0)
    assert torch.equal(y0, y1)
