"""Kernel-level parity: single operators of the HIP library, called through the C ABI,
against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

import pat_inputs as pi
from gpu_util import DEV, widen
from oracle import bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def pat():
    import paper_2605_23945_amd as p
    p.load_library()
    return p


def _w(n, k, tid, std=0.02):
    idx = torch.arange(n * k, dtype=torch.int64)
    return pi.normal_bf16(pi.stream_key(0xABCD, tid), idx, std).view(n, k)


def _x(b, k, seed):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(b, k, generator=g, dtype=torch.float32)


def test_generator_same_bytes_on_cpu_and_gpu():
    s = pi.CONFIGS["tiny_tp1"]["shard"]
    a, b = pi.layer_weights(s, 1, device="cpu"), pi.layer_weights(s, 1, device=DEV)
    for k in a:
        assert torch.equal(a[k], b[k].cpu()), k
    ka, va = pi.kv_prefix(s, 3, 0, 50, device="cpu")
    kb, vb = pi.kv_prefix(s, 3, 0, 50, device=DEV)
    assert torch.equal(ka, kb.cpu()) and torch.equal(va, vb.cpu())


def test_weight_packing_and_mfma_layout_exact(pat):
    """One-hot activations make y[b, :] a column of W: exact, so any slip in the packed
    layouts or in the matrix-core lane mapping shows as a wrong or misplaced value."""
    n, k = 80, 96
    w = _w(n, k, 1, std=1.0)
    wp = pat.pat_op_pack_weight(w.to(DEV))
    cols = [0, 1, 7, 8, 31, 32, 33, 63, 64, 95, 40, 17, 90, 5, 77, 50, 3]      # 17 rows: two batch tiles
    x = torch.zeros(len(cols), k)
    for b, c in enumerate(cols):
        x[b, c] = 1.0
    hi, lo = pat.pat_op_pack_act(x.to(DEV))
    y = torch.full((len(cols), n), 7.0, device=DEV)
    pat.pat_op_gemm(wp, n, k, hi, lo, len(cols), y, mode=0)
    ref = w.float()[:, cols].T
    assert torch.equal(y.cpu(), ref)


@pytest.mark.parametrize("n,k,b", [(256, 1024, 1), (256, 1024, 5), (1040, 352, 16), (512, 2752, 17), (96, 4096, 33),
                                   (64, 256, 100), (48, 64, 256), (4096, 4096, 8), (16, 32, 3),
                                   (4096, 1024, 200), (528, 2752, 130), (1024, 4096, 40), (256, 8192, 30),
                                   (4096, 4096, 256), (2048, 11008, 96), (8192, 512, 192), (16384, 1024, 255), (4096, 4096, 177),
                                   (34000, 512, 250), (4112, 1024, 65), (22016, 1024, 129),
                                   (4096, 4096, 1), (4096, 11008, 2), (1040, 352, 2), (2064, 4096, 2), (16, 32, 1), (48, 64, 2),
                                   (8192, 28672, 1)])
def test_gemm_store_and_accumulate_vs_oracle(pat, orc, n, k, b):
    w, x = _w(n, k, 2 + n + k), _x(b, k, n + b)
    wp = pat.pat_op_pack_weight(w.to(DEV))
    hi, lo = pat.pat_op_pack_act(x.to(DEV))
    y = torch.empty(b, n, device=DEV)
    pat.pat_op_gemm(wp, n, k, hi, lo, b, y, mode=0)
    y0 = _x(b, n, 99)
    y1 = y0.to(DEV)
    pat.pat_op_gemm(wp, n, k, hi, lo, b, y1, mode=1)
    rows = sorted(set([0, b - 1, b // 2, min(b - 1, 15), min(b - 1, 16)]))
    wb = bits(w)
    for r in rows:
        ref = orc.matvec(wb, x[r].double().numpy())
        scale = float(np.sqrt(np.mean(ref * ref)))
        assert np.max(np.abs(y[r].cpu().double().numpy() - ref)) <= 1e-4 * scale
        assert np.max(np.abs(y1[r].cpu().double().numpy() - (ref + y0[r].double().numpy()))) <= 1e-4 * scale + 1e-6


@pytest.mark.parametrize("f,k,b", [(64, 256, 3), (352, 512, 16), (1024, 256, 40), (512, 2048, 70), (64, 4096, 9),
                                   (2752, 1024, 256), (1376, 4096, 150), (352, 512, 2), (64, 4096, 1)])
def test_gemm_swiglu_epilogue_vs_oracle(pat, orc, f, k, b):
    wg, wu, x = _w(f, k, 11, 0.05), _w(f, k, 12, 0.05), _x(b, k, 5)
    wp = pat.pat_op_pack_weight(wg.to(DEV), wu.to(DEV))
    hi, lo = pat.pat_op_pack_act(x.to(DEV))
    nbytes = pat.load_library().pat_op_packed_act_bytes(b, f)
    yh = torch.zeros(nbytes, dtype=torch.uint8, device=DEV); yl = torch.zeros_like(yh)
    pat.pat_op_gemm(wp, 2 * f, k, hi, lo, b, None, mode=2, y_hi=yh, y_lo=yl)
    got = pat.unpack_act(yh, yl, b, f)
    for r in sorted(set([0, b - 1, b // 2])):
        g = orc.matvec(bits(wg), x[r].double().numpy()); u = orc.matvec(bits(wu), x[r].double().numpy())
        ref = np.array([orc.silu(float(a)) for a in g]) * u
        scale = float(np.sqrt(np.mean(ref * ref)))
        assert np.max(np.abs(got[r] - ref)) <= 1e-4 * scale


def test_pack_act_split_is_fp32_class(pat):
    x = _x(19, 160, 3) * 100.0
    hi, lo = pat.pat_op_pack_act(x.to(DEV))
    got = pat.unpack_act(hi, lo, 19, 160)
    rel = np.abs(got - x.double().numpy()) / np.abs(x.double().numpy())
    assert rel.max() <= 2.0 ** -16


@pytest.mark.parametrize("b,h", [(1, 256), (7, 4096), (20, 5120), (3, 10240), (2, 8192)])
def test_rmsnorm_pack_vs_oracle(pat, orc, b, h):
    x = _x(b, h, 17) * 3.0
    g = pi.normal_bf16(pi.stream_key(1, 2), torch.arange(h, dtype=torch.int64), 0.02, 1.0)
    hi, lo = pat.pat_op_rmsnorm_pack(x.to(DEV), g.to(DEV), 1e-6)
    got = pat.unpack_act(hi, lo, b, h)
    for r in range(b):
        ref = orc.rmsnorm(x[r].double().numpy(), bits(g), 1e-6)
        assert np.max(np.abs(got[r] - ref)) <= 3e-5 * np.max(np.abs(ref))


def test_argmax_bit_exact(pat, orc):
    g = torch.Generator().manual_seed(5)
    n = 8000
    rows = [torch.randn(n, generator=g) for _ in range(6)]
    rows[1][[4000, 17, 7999]] = 9.0                 # ties: lowest index wins
    rows[2][:] = float("-inf")                      # nothing finite
    rows[3][100] = float("nan"); rows[3][200] = 50.0
    rows[4][:] = float("nan")
    rows[5][[7999]] = float("inf")
    x = torch.stack(rows)
    idx, val = pat.pat_op_argmax(x.to(DEV), base=16000)
    ref = [16000 + orc.argmax_f32(r.numpy()) for r in rows]
    assert idx.cpu().tolist() == ref
    assert ref[1] == 16017 and ref[2] == 16000 and ref[3] == 16200 and ref[4] == 16000
    # ragged widths
    for n in (16, 1024, 1040, 32000):
        x = torch.randn(3, n, generator=g)
        idx, _ = pat.pat_op_argmax(x.to(DEV))
        assert idx.cpu().tolist() == [orc.argmax_f32(r.numpy()) for r in x]


@pytest.mark.parametrize("fused", [False, True])
@pytest.mark.parametrize("n,k,b", [(256, 1024, 1), (1040, 4096, 16), (512, 5120, 7), (96, 8192, 3), (2048, 256, 16), (4096, 4096, 2),
                                   (8000, 4096, 5), (1040, 4096, 17), (512, 2752, 32), (4096, 11008, 20)])
def test_gemm_with_folded_rmsnorm_vs_oracle(pat, orc, n, k, b, fused):
    """The projection of the small-batch step: the operand is x * gains (packed by the producer of x), the rows' sums
    of squares arrive as per-16-column partial sums (what the producing projection writes) and the result is scaled
    by 1 / rms.  Both kernels that do this: the streaming kernel (up to 32 rows) and the fused layer kernel's
    projection phase (up to 16).  Rows past the live batch are padding and must not leak into any result (NaN here)."""
    if fused and b > 16:
        pytest.skip("the fused layer kernel takes at most 16 rows")
    R = (b + 15) // 16 * 16
    w, x = _w(n, k, 7 + n + k), _x(b, k, 3 * n + b) * 3.0
    g = pi.normal_bf16(pi.stream_key(1, 3), torch.arange(k, dtype=torch.int64), 0.02, 1.0)
    xr = torch.full((R, k), float("nan"))
    xr[:b] = x
    stats = (xr.view(R, k // 16, 16) ** 2).sum(-1).T.contiguous()             # [k / 16, R]
    wp = pat.pat_op_pack_weight(w.to(DEV))
    hi, lo = pat.pat_op_pack_act_gain(xr.to(DEV), g.to(DEV))
    y = pat.pat_op_gemm_norm(wp, n, k, hi, lo, stats.to(DEV), 1e-6, b, fused=fused).cpu().double().numpy()
    assert np.all(np.isfinite(y))
    for r in sorted(set([0, b - 1, b // 2, min(b - 1, 15), min(b - 1, 16)])):
        ref = orc.matvec(bits(w), orc.rmsnorm(x[r].double().numpy(), bits(g), 1e-6))
        scale = float(np.sqrt(np.mean(ref * ref)))
        assert np.max(np.abs(y[r] - ref)) <= 1e-4 * scale
    # one part per row (as after the embedding) gives the same 1/rms up to the summation order
    y1 = pat.pat_op_gemm_norm(wp, n, k, hi, lo, torch.nan_to_num((xr ** 2).sum(-1), nan=0.0).to(DEV), 1e-6, b, fused=fused)
    assert np.max(np.abs(y1.cpu().double().numpy() - y)) <= 1e-5 * float(np.sqrt(np.mean(y * y)))


def test_embed_stats_rows_sums_and_packed_operand(pat):
    s = pi.CONFIGS["tiny_tp1"]["shard"]
    table = pi.embedding_table(s, device=DEV)
    g = pi.layer_weights(s, 0, device=DEV)["g1"]
    tok = torch.tensor([5, 0, 1023, 77, 5], dtype=torch.int32, device=DEV)
    x, stats, hi, lo = pat.pat_op_embed_stats(table, tok, g)
    ref = table[tok.long()].float()
    assert torch.equal(x[:5], ref)
    assert torch.allclose(stats[:5], (ref.double() ** 2).sum(-1).float(), rtol=1e-6)
    got = pat.unpack_act(hi, lo, 16, s.hidden)[:5]
    want = (ref.double() * g.double()[None, :]).cpu().numpy()
    assert np.max(np.abs(got - want) / np.maximum(np.abs(want), 1e-30)) <= 2.0 ** -16
    hi2, lo2 = pat.pat_op_pack_act_gain(x[:5].contiguous(), g)                 # the stand-alone packing agrees bit for bit
    assert np.array_equal(pat.unpack_act(hi2, lo2, 5, s.hidden), got)


@pytest.mark.parametrize("n,k,b", [(4096, 11008, 20), (4096, 4096, 32), (4096, 4096, 16),
                                   (4096, 11008, 200), (4096, 4096, 64), (12288, 4096, 256), (2048, 8192, 130)])
def test_projection_is_bitwise_repeatable(pat, n, k, b):
    """One tile per workgroup, two batch tiles: the case in which a read of a matrix-instruction result that the compiler
    had moved behind a branch returned a stale element in about one call out of five.  Above 32 rows: K split across
    workgroups, the slices' partial sums added in slice order by a second kernel.  Every sum has a fixed order, so
    repeated calls must agree bit for bit."""
    w, x = _w(n, k, 5 + n + k).to(DEV), _x(b, k, 2 * n + b).to(DEV) * 3.0
    wp = pat.pat_op_pack_weight(w)
    hi, lo = pat.pat_op_pack_act(x)
    y0 = torch.empty(b, n, device=DEV)
    pat.pat_op_gemm(wp, n, k, hi, lo, b, y0, mode=0)
    for _ in range(60):
        y = torch.empty(b, n, device=DEV)
        pat.pat_op_gemm(wp, n, k, hi, lo, b, y, mode=0)
        assert torch.equal(y, y0)


def test_device_barrier_probe_runs_and_its_bounded_wait_ends(pat):
    """The fused layer kernel's device-wide barrier on its own: it completes among resident workgroups, and with a
    spin limit of zero every workgroup still exits (the call reports the state error instead of hanging)."""
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    for n_wg in (1, 7, min(64, n_cu), n_cu):
        us = pat.pat_op_barrier_probe(n_wg, iters=50)
        assert 0.0 < us < 200.0, (n_wg, us)
    with pytest.raises(pat.PatError) as e:
        pat.pat_op_barrier_probe(n_cu, iters=4, max_spin=0)        # the host forces the time-out; the kernel ends by itself
    assert e.value.code == -3
    with pytest.raises(pat.PatError) as e:
        pat.pat_op_barrier_probe(n_cu + 1, iters=4)                # more workgroups than are resident at once: refused
    assert e.value.code == -1
    assert pat.pat_op_barrier_probe(n_cu, iters=20) > 0.0          # and the next call starts from clean words
