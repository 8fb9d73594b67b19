"""ctypes binding of libpat_decode.so: same names as include/pat_decode.h.

Argument marshalling only.  torch supplies device memory (the three arenas, the
staging tensors) and the stream; every step of the decode path runs in the
library's HIP kernels.  There is no fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("PAT_DECODE_LIB", os.path.join(_HERE, "libpat_decode.so"))   # override: A/B of two builds

PAT_OK, PAT_EINVAL, PAT_ENOMEM, PAT_ESTATE, PAT_EHIP = 0, -1, -2, -3, -4


class PatError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"pat error {code}: {msg}")
        self.code = code


class pat_cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab",
                                         "tp_degree", "tp_rank")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float),
                ("max_batch", C.c_int32), ("max_seq_len", C.c_int32), ("page_tokens", C.c_int32),
                ("kv_token_budget", C.c_int64), ("eos_token", C.c_int32), ("qk_norm", C.c_int32)]


class pat_mem_req(C.Structure):
    _fields_ = [("weights_bytes", C.c_int64), ("kv_bytes", C.c_int64), ("work_bytes", C.c_int64),
                ("n_pages", C.c_int32), ("max_pages_per_seq", C.c_int32)]


class pat_buffers(C.Structure):
    _fields_ = [("weights", C.c_void_p), ("kv", C.c_void_p), ("work", C.c_void_p)]


class pat_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g1", "wqkv", "wo", "g2", "wg", "wu", "wd", "gq", "gk")]


class pat_final_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("embed", "gf", "wlm")]


class pat_step_report(C.Structure):
    _fields_ = [("live_batch", C.c_int32), ("n_finished", C.c_int32), ("sum_context", C.c_int64),
                ("free_pages", C.c_int32), ("step_index", C.c_int32)]


class pat_grid_row(C.Structure):
    _fields_ = [("tp_degree", C.c_int32), ("batch", C.c_int32), ("kv_len", C.c_int32), ("skipped", C.c_int32),
                ("sum_context", C.c_int64), ("mean_us", C.c_double), ("min_us", C.c_double), ("std_us", C.c_double),
                ("tokens_per_s", C.c_double), ("algo_bytes", C.c_double), ("hbm_frac", C.c_double)]


class pat_prefill_row(C.Structure):
    _fields_ = [("tp_degree", C.c_int32), ("batch", C.c_int32), ("length", C.c_int32), ("latency_us", C.c_double)]


class pat_plan_point(C.Structure):
    _fields_ = [("tp_degree", C.c_int32), ("batch", C.c_int32), ("kv_len", C.c_int32), ("reserved", C.c_int32)]


class pat_switch_input(C.Structure):
    _fields_ = [("tp", C.c_int32), ("tp_list", C.POINTER(C.c_int32)), ("n_tp", C.c_int32), ("n_gpus", C.c_int32),
                ("group_batch", C.POINTER(C.c_int32)), ("group_context", C.POINTER(C.c_double)), ("n_groups", C.c_int32),
                ("l_max", C.c_int32), ("l_gen", C.c_int32), ("lengths", C.POINTER(C.c_int32)), ("n_lengths", C.c_int32),
                ("n_layers", C.c_int32), ("hidden", C.c_int32), ("bytes_per_elem", C.c_int32),
                ("net_bytes_per_s", C.c_double), ("fixed_us", C.POINTER(C.c_double)),
                ("prefill", C.POINTER(pat_prefill_row)), ("n_prefill", C.c_int32)]


class pat_switch_decision(C.Structure):
    _fields_ = [("do_switch", C.c_int32), ("tp_new", C.c_int32), ("t_cur_us", C.c_double), ("t_best_us", C.c_double),
                ("t_rem_us", C.POINTER(C.c_double)), ("t_switch_us", C.POINTER(C.c_double)),
                ("t_total_us", C.POINTER(C.c_double))]


EXPORTS = ["pat_decode_query", "pat_decode_init", "pat_load_layer", "pat_load_layer_from_full", "pat_load_final", "pat_decode_admit",
           "pat_kv_write", "pat_kv_read", "pat_kv_extract", "pat_kv_inject", "pat_prefill", "pat_decode_step", "pat_kv_compact", "pat_get_state", "pat_get_pages",
           "pat_profile_grid", "pat_profile_prefill", "pat_decode_reset", "pat_step_algo_bytes", "pat_timing_enable", "pat_timing_read", "pat_timing_fused_trace",
           "pat_decode_destroy", "pat_last_error", "pat_op_packed_weight_bytes", "pat_op_pack_weight",
           "pat_op_packed_act_bytes", "pat_op_pack_act", "pat_op_gemm", "pat_op_gemm_static", "pat_op_gemm_scratch_bytes", "pat_op_gemm_plan", "pat_op_rmsnorm_pack", "pat_op_embed_stats", "pat_op_pack_act_gain", "pat_op_gemm_norm", "pat_decode_uses_fused_kernel", "pat_op_barrier_probe", "pat_op_argmax",
           "pat_predictor_fit", "pat_predictor_destroy", "pat_predictor_line", "pat_predictor_query", "pat_switch_decide",
           "pat_kv_move_seconds", "pat_rms_length", "pat_profile_plan"]

_lib = None


def load_library() -> C.CDLL:
    """dlopen the in-tree library; raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise FileNotFoundError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
    lib = C.CDLL(LIB_PATH)
    i32p, vp = C.POINTER(C.c_int32), C.c_void_p
    lib.pat_decode_query.argtypes = [C.POINTER(pat_cfg), C.POINTER(pat_mem_req)]
    lib.pat_decode_init.argtypes = [C.POINTER(pat_cfg), C.POINTER(pat_buffers), vp, C.POINTER(vp)]
    lib.pat_load_layer.argtypes = [vp, C.c_int32, C.POINTER(pat_layer_weights)]
    lib.pat_load_layer_from_full.argtypes = [vp, C.c_int32, C.POINTER(pat_layer_weights)]
    lib.pat_load_final.argtypes = [vp, C.POINTER(pat_final_weights)]
    lib.pat_decode_admit.argtypes = [vp, C.c_int32, i32p, i32p, i32p, i32p]
    lib.pat_kv_write.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32]
    lib.pat_kv_read.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32]
    lib.pat_kv_extract.argtypes = [vp, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, C.c_int64, C.POINTER(C.c_int64)]
    lib.pat_kv_inject.argtypes = [vp, C.c_int32, i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, vp, C.c_int32, C.c_int32, C.c_int64]
    lib.pat_prefill.argtypes = [vp, C.c_int32, i32p, i32p, C.c_int64]
    lib.pat_decode_step.argtypes = [vp, C.POINTER(pat_step_report), vp, vp]
    lib.pat_kv_compact.argtypes = [vp, i32p]
    lib.pat_get_state.argtypes = [vp, i32p] + [i32p] * 6
    lib.pat_get_pages.argtypes = [vp, i32p, i32p, i32p]
    lib.pat_profile_grid.argtypes = [vp, i32p, C.c_int32, i32p, C.c_int32, C.c_int64, C.c_int32, C.c_int32, C.c_int32,
                                     C.c_uint64, C.POINTER(pat_grid_row), i32p]
    lib.pat_profile_prefill.argtypes = [vp, i32p, C.c_int32, i32p, C.c_int32, C.c_int64, C.c_int32, C.c_uint64, C.POINTER(pat_prefill_row)]
    lib.pat_decode_reset.argtypes = [vp]
    lib.pat_step_algo_bytes.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.pat_timing_enable.argtypes = [vp, C.c_int32]
    lib.pat_timing_read.argtypes = [vp, C.c_int32, C.POINTER(C.c_double), C.POINTER(C.c_int64), C.c_int32]
    lib.pat_timing_fused_trace.argtypes = [vp, vp]
    lib.pat_decode_destroy.argtypes = [vp]
    lib.pat_last_error.argtypes = [vp]
    lib.pat_last_error.restype = C.c_char_p
    lib.pat_op_packed_weight_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.pat_op_packed_weight_bytes.restype = C.c_int64
    lib.pat_op_packed_act_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.pat_op_packed_act_bytes.restype = C.c_int64
    lib.pat_op_pack_weight.argtypes = [vp, vp, C.c_int32, C.c_int32, vp, vp]
    lib.pat_op_pack_act.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, vp]
    lib.pat_op_gemm.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32, vp, C.c_int32, vp, vp, C.c_int32, vp, vp]
    lib.pat_op_gemm_static.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, C.c_int32, vp, C.c_int32, vp, vp, C.c_int32, vp]
    lib.pat_op_gemm_scratch_bytes.argtypes = [C.c_int32, C.c_int32, C.c_int32]
    lib.pat_op_gemm_scratch_bytes.restype = C.c_int64
    lib.pat_op_gemm_plan.argtypes = [C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_int32)]
    lib.pat_op_gemm_plan.restype = C.c_int
    lib.pat_op_rmsnorm_pack.argtypes = [vp, vp, C.c_int32, C.c_int32, C.c_float, vp, vp, vp]
    lib.pat_op_argmax.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, vp, vp, vp]
    lib.pat_op_barrier_probe.argtypes = [vp, C.c_int32, C.c_int32, C.c_int32, C.POINTER(C.c_double), vp]
    lib.pat_op_embed_stats.argtypes = [vp, C.c_int32, vp, vp, C.c_int32, vp, vp, vp, vp, vp]
    lib.pat_op_pack_act_gain.argtypes = [vp, vp, C.c_int32, C.c_int32, vp, vp, vp]
    lib.pat_op_gemm_norm.argtypes = [vp, C.c_int32, C.c_int32, vp, vp, vp, C.c_int32, C.c_float, C.c_int32, vp, C.c_int32, C.c_int32, vp]
    lib.pat_decode_uses_fused_kernel.argtypes = [vp]
    dp = C.POINTER(C.c_double)
    lib.pat_predictor_fit.argtypes = [C.POINTER(pat_grid_row), C.c_int32, C.POINTER(vp)]
    lib.pat_predictor_destroy.argtypes = [vp]
    lib.pat_predictor_destroy.restype = None
    lib.pat_predictor_line.argtypes = [vp, C.c_int32, C.c_int32, dp, dp]
    lib.pat_predictor_query.argtypes = [vp, C.c_int32, C.c_int32, C.c_double, dp]
    lib.pat_switch_decide.argtypes = [vp, C.POINTER(pat_switch_input), C.POINTER(pat_switch_decision)]
    lib.pat_kv_move_seconds.argtypes = [i32p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_double]
    lib.pat_kv_move_seconds.restype = C.c_double
    lib.pat_rms_length.argtypes = [i32p, C.c_int32]
    lib.pat_rms_length.restype = C.c_double
    lib.pat_profile_plan.argtypes = [C.c_int32, C.c_int64, C.c_int64, C.POINTER(pat_plan_point), C.POINTER(C.c_int32)]
    _lib = lib
    return lib


def make_cfg(shard, max_batch, max_seq_len, kv_token_budget, page_tokens=64, eos_token=-1) -> pat_cfg:
    """pat_cfg from a pat_inputs.ShardShape-like object (fields model.*, tp, rank)."""
    m = shard.model
    return pat_cfg(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab, shard.tp, shard.rank,
                   m.rms_eps, m.rope_base, max_batch, max_seq_len, page_tokens, kv_token_budget, eos_token,
                   1 if getattr(m, "qk_norm", False) else 0)


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else C.c_void_p(0)


class Decoder:
    """Owns the arenas (torch uint8 tensors on the current device) and a pat_ctx."""

    def __init__(self, cfg: pat_cfg, device="cuda:0"):
        import torch
        self.lib = load_library()
        self.cfg = cfg
        self.req = pat_mem_req()
        rc = self.lib.pat_decode_query(C.byref(cfg), C.byref(self.req))
        if rc:
            raise PatError(rc, "pat_decode_query rejected the configuration")
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        alloc = lambda n: torch.empty(int(n) + 256, dtype=torch.uint8, device=self.device)
        self._w, self._kv, self._work = alloc(self.req.weights_bytes), alloc(self.req.kv_bytes), alloc(self.req.work_bytes)
        al = lambda t: (t.data_ptr() + 255) // 256 * 256
        self._bufs = pat_buffers(al(self._w), al(self._kv), al(self._work))
        self.ctx = C.c_void_p()
        rc = self.lib.pat_decode_init(C.byref(cfg), C.byref(self._bufs), _stream(), C.byref(self.ctx))
        if rc:
            raise PatError(rc, "pat_decode_init failed")
        tp = cfg.tp_degree
        self.hq, self.hkv = cfg.n_q_heads // tp, max(1, cfg.n_kv_heads // tp)
        self.vs, self.d = cfg.vocab // tp, cfg.head_dim

    def _chk(self, rc):
        if rc:
            raise PatError(rc, self.lib.pat_last_error(self.ctx).decode())

    def close(self):
        if self.ctx:
            self.lib.pat_decode_destroy(self.ctx)
            self.ctx = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- same names as the C ABI ---------------------------------------------------
    def pat_load_layer(self, layer, w: dict):
        lw = pat_layer_weights(*[_ptr(w.get(k)) for k in ("g1", "wqkv", "wo", "g2", "wg", "wu", "wd", "gq", "gk")])
        self._chk(self.lib.pat_load_layer(self.ctx, layer, C.byref(lw)))

    def pat_load_layer_from_full(self, layer, w: dict):
        """w: the UNSHARDED layer's tensors (same keys as pat_load_layer)."""
        lw = pat_layer_weights(*[_ptr(w.get(k)) for k in ("g1", "wqkv", "wo", "g2", "wg", "wu", "wd", "gq", "gk")])
        self._chk(self.lib.pat_load_layer_from_full(self.ctx, layer, C.byref(lw)))

    def pat_load_final(self, w: dict):
        fw = pat_final_weights(_ptr(w["embed"]), _ptr(w["gf"]), _ptr(w["wlm"]))
        self._chk(self.lib.pat_load_final(self.ctx, C.byref(fw)))

    def pat_decode_admit(self, seq_id, token, kv_len, target):
        a, ap = _i32(seq_id); b, bp = _i32(token); c, cp = _i32(kv_len); d, dp = _i32(target)
        self._chk(self.lib.pat_decode_admit(self.ctx, len(a), ap, bp, cp, dp))

    def pat_kv_write(self, slot, layer, k, v):
        assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
        self._chk(self.lib.pat_kv_write(self.ctx, slot, layer, _ptr(k), _ptr(v), k.shape[0]))

    def pat_kv_read(self, slot, layer, n_tokens):
        import torch
        k = torch.empty((n_tokens, self.hkv, self.d), dtype=torch.bfloat16, device=self.device)
        v = torch.empty_like(k)
        self._chk(self.lib.pat_kv_read(self.ctx, slot, layer, _ptr(k), _ptr(v), n_tokens))
        return k, v

    def pat_kv_extract(self, slots, layer0=0, n_layers=None, head0=0, n_heads=None, buf=None):
        """Returns (buf, T): buf a bf16 tensor [n_layers, 2, n_heads, T, d] on the device."""
        import torch
        n_layers = self.cfg.n_layers - layer0 if n_layers is None else n_layers
        n_heads = self.hkv - head0 if n_heads is None else n_heads
        if buf is None:
            st = self.pat_get_state()
            t = int(sum(int(st["kv_len"][s]) for s in slots if 0 <= s < st["live"]))     # the library rejects the rest
            buf = torch.empty((n_layers, 2, n_heads, t, self.d), dtype=torch.bfloat16, device=self.device)
        t_sel = C.c_int64()
        sl, slp = _i32(slots)
        self._chk(self.lib.pat_kv_extract(self.ctx, len(sl), slp, layer0, n_layers, head0, n_heads, _ptr(buf),
                                          buf.numel() * 2, C.byref(t_sel)))
        return buf, t_sel.value

    def pat_kv_inject(self, slots, buf, layer0=0, pool_head0=0, n_heads=None, buf_head0=0):
        """buf: bf16 tensor [n_layers, 2, buf_heads, T, d] (contiguous) on the device."""
        n_layers, _, buf_heads, t, _ = buf.shape
        n_heads = min(self.hkv - pool_head0, buf_heads - buf_head0) if n_heads is None else n_heads
        sl, slp = _i32(slots)
        self._chk(self.lib.pat_kv_inject(self.ctx, len(sl), slp, layer0, n_layers, pool_head0, n_heads,
                                         _ptr(buf), buf_heads, buf_head0, t))

    def pat_prefill(self, slots, tokens):
        """tokens: flat int32 array, the slots' token ids at positions 0 .. kv_len - 1, slot after slot."""
        sl, slp = _i32(slots); tk, tkp = _i32(tokens)
        self._chk(self.lib.pat_prefill(self.ctx, len(sl), slp, tkp, len(tk)))

    def pat_decode_step(self, report=True, next_tok=None, logits=None):
        rep = pat_step_report()
        self._chk(self.lib.pat_decode_step(self.ctx, C.byref(rep) if report else None, _ptr(next_tok), _ptr(logits)))
        return rep if report else None

    def pat_kv_compact(self) -> int:
        n = C.c_int32()
        self._chk(self.lib.pat_kv_compact(self.ctx, C.byref(n)))
        return n.value

    def pat_get_state(self) -> dict:
        mb = self.cfg.max_batch
        live = C.c_int32()
        arrs = {k: np.zeros(mb, np.int32) for k in ("seq_id", "token", "kv_len", "gen", "target", "fin")}
        ps = [a.ctypes.data_as(C.POINTER(C.c_int32)) for a in arrs.values()]
        self._chk(self.lib.pat_get_state(self.ctx, C.byref(live), *ps))
        return {k: v[:live.value].copy() for k, v in arrs.items()} | {"live": live.value}

    def pat_get_pages(self):
        live = self.pat_get_state()["live"]
        pt = np.zeros((max(live, 1), self.req.max_pages_per_seq), np.int32)
        fl = np.zeros(self.req.n_pages, np.int32)
        nf = C.c_int32()
        self._chk(self.lib.pat_get_pages(self.ctx, pt.ctypes.data_as(C.POINTER(C.c_int32)),
                                         fl.ctypes.data_as(C.POINTER(C.c_int32)), C.byref(nf)))
        return pt[:live], fl[:nf.value].copy()

    def pat_profile_grid(self, batches, kv_lens, t_cap, steps=60, warmup=3, reps=5, seed=1):
        b, bp = _i32(batches); l, lp = _i32(kv_lens)
        rows = (pat_grid_row * (len(b) * len(l)))()
        n = C.c_int32(len(b) * len(l))
        self._chk(self.lib.pat_profile_grid(self.ctx, bp, len(b), lp, len(l), t_cap, steps, warmup, reps, seed, rows,
                                            C.byref(n)))
        return [{f: getattr(rows[i], f) for f, _ in pat_grid_row._fields_} for i in range(n.value)]

    def pat_profile_prefill(self, batches, lengths, t_cap, reps=2, seed=1):
        """Returns the ctypes array of pat_prefill_row (what pat_switch_decide takes) and the same rows as dicts."""
        b, bp = _i32(batches); l, lp = _i32(lengths)
        rows = (pat_prefill_row * (len(b) * len(l)))()
        self._chk(self.lib.pat_profile_prefill(self.ctx, bp, len(b), lp, len(l), t_cap, reps, seed, rows))
        return rows, [{f: getattr(rows[i], f) for f, _ in pat_prefill_row._fields_} for i in range(len(rows))]

    def pat_decode_reset(self):
        self._chk(self.lib.pat_decode_reset(self.ctx))

    def pat_step_algo_bytes(self):
        w, k = C.c_double(), C.c_double()
        self._chk(self.lib.pat_step_algo_bytes(self.ctx, C.byref(w), C.byref(k)))
        return w.value, k.value

    def pat_timing_enable(self, on: bool):
        self._chk(self.lib.pat_timing_enable(self.ctx, int(on)))

    def pat_decode_uses_fused_kernel(self) -> bool:
        return bool(self.lib.pat_decode_uses_fused_kernel(self.ctx))

    def pat_timing_fused_trace(self, trace):
        """trace: int64 device tensor of 256 x 16 words (or None to switch the stamps off)."""
        self._chk(self.lib.pat_timing_fused_trace(self.ctx, _ptr(trace)))

    def pat_timing_read(self, klass, reset=True):
        ms, n = C.c_double(), C.c_int64()
        self._chk(self.lib.pat_timing_read(self.ctx, klass, C.byref(ms), C.byref(n), int(reset)))
        return ms.value, n.value


# ---- single operators ------------------------------------------------------------------

def pat_op_pack_weight(w, w2=None):
    """torch bf16 [n, k] (and optionally a second one to interleave) -> packed uint8 tensor."""
    import torch
    lib = load_library()
    n, k = w.shape
    rows = 2 * n if w2 is not None else n
    out = torch.empty(lib.pat_op_packed_weight_bytes(rows, k), dtype=torch.uint8, device=w.device)
    rc = lib.pat_op_pack_weight(_ptr(w.contiguous()), _ptr(w2.contiguous() if w2 is not None else None), n, k, _ptr(out), _stream())
    if rc:
        raise PatError(rc, "pat_op_pack_weight")
    return out


def pat_op_pack_act(x):
    import torch
    lib = load_library()
    b, k = x.shape
    nbytes = lib.pat_op_packed_act_bytes(b, k)
    hi = torch.empty(nbytes, dtype=torch.uint8, device=x.device); lo = torch.empty_like(hi)
    rc = lib.pat_op_pack_act(_ptr(x.contiguous()), b, k, _ptr(hi), _ptr(lo), _stream())
    if rc:
        raise PatError(rc, "pat_op_pack_act")
    return hi, lo


def pat_op_gemm(w_packed, n, k, xhi, xlo, b, y=None, mode=0, y_hi=None, y_lo=None):
    import torch
    lib = load_library()
    nbytes = lib.pat_op_gemm_scratch_bytes(n, k, b)
    scratch = torch.empty(nbytes, dtype=torch.uint8, device=w_packed.device) if nbytes > 0 else None
    rc = lib.pat_op_gemm(_ptr(w_packed), n, k, _ptr(xhi), _ptr(xlo), b, _ptr(y), (y.stride(0) if y is not None else 0),
                         _ptr(y_hi), _ptr(y_lo), mode, _ptr(scratch), _stream())
    if rc:
        raise PatError(rc, "pat_op_gemm")


def pat_op_gemm_static(w_packed, n, k, xhi, xlo, b, y=None, mode=0, y_hi=None, y_lo=None):
    """pat_op_gemm with the library's own static scratch: no allocation on this path, torch's included."""
    rc = load_library().pat_op_gemm_static(_ptr(w_packed), n, k, _ptr(xhi), _ptr(xlo), b, _ptr(y),
                                           (y.stride(0) if y is not None else 0), _ptr(y_hi), _ptr(y_lo), mode, _stream())
    if rc:
        raise PatError(rc, "pat_op_gemm_static" + (": the K-slice partial sums exceed PAT_STATIC_SCRATCH_BYTES" if rc == PAT_ENOMEM else ""))


def pat_op_rmsnorm_pack(x, g, eps):
    import torch
    lib = load_library()
    b, h = x.shape
    nbytes = lib.pat_op_packed_act_bytes(b, h)
    hi = torch.empty(nbytes, dtype=torch.uint8, device=x.device); lo = torch.empty_like(hi)
    rc = lib.pat_op_rmsnorm_pack(_ptr(x.contiguous()), _ptr(g), b, h, eps, _ptr(hi), _ptr(lo), _stream())
    if rc:
        raise PatError(rc, "pat_op_rmsnorm_pack")
    return hi, lo


def pat_op_embed_stats(table, tok, g):
    """table bf16 [vocab, h], tok int32 [b <= 32], g bf16 [h] (device) -> (x fp32 [R, h] with rows >= b unset,
    stats fp32 [R], packed x * g (hi, lo)); R = 16 * ceil(b / 16)."""
    import torch
    lib = load_library()
    b, h = tok.shape[0], table.shape[1]
    R = (b + 15) // 16 * 16
    x = torch.zeros(R, h, dtype=torch.float32, device=table.device)
    stats = torch.zeros(R, dtype=torch.float32, device=table.device)
    nbytes = lib.pat_op_packed_act_bytes(R, h)
    hi = torch.zeros(nbytes, dtype=torch.uint8, device=table.device); lo = torch.zeros_like(hi)
    rc = lib.pat_op_embed_stats(_ptr(table), h, _ptr(tok), _ptr(g), b, _ptr(x), _ptr(stats), _ptr(hi), _ptr(lo), _stream())
    if rc:
        raise PatError(rc, "pat_op_embed_stats")
    return x, stats, hi, lo


def pat_op_pack_act_gain(x, g):
    """x fp32 [b, k], g bf16 [k] -> packed split-bf16 of x * g (hi, lo)."""
    import torch
    lib = load_library()
    b, k = x.shape
    nbytes = lib.pat_op_packed_act_bytes(b, k)
    hi = torch.zeros(nbytes, dtype=torch.uint8, device=x.device); lo = torch.zeros_like(hi)
    rc = lib.pat_op_pack_act_gain(_ptr(x.contiguous()), _ptr(g), b, k, _ptr(hi), _ptr(lo), _stream())
    if rc:
        raise PatError(rc, "pat_op_pack_act_gain")
    return hi, lo


def pat_op_gemm_norm(w_packed, n, k, xg_hi, xg_lo, stats, eps, b, fused=False):
    """y [b, n] = RMSNorm(x; g, eps) W^T from the packed x * g and stats fp32 [n_parts, R] partial sums of squares of x
    (R = 16 * ceil(b / 16)); fused: through the fused layer kernel's projection phase instead of the streaming kernel."""
    import torch
    R = (b + 15) // 16 * 16
    assert stats.is_contiguous() and stats.numel() % R == 0
    y = torch.empty(b, n, dtype=torch.float32, device=stats.device)
    rc = load_library().pat_op_gemm_norm(_ptr(w_packed), n, k, _ptr(xg_hi), _ptr(xg_lo), _ptr(stats), stats.numel() // R, eps, b,
                                         _ptr(y), n, int(bool(fused)), _stream())
    if rc:
        raise PatError(rc, "pat_op_gemm_norm")
    return y


def pat_op_argmax(logits, base=0):
    import torch
    lib = load_library()
    b, n = logits.shape
    idx = torch.empty(b, dtype=torch.int32, device=logits.device)
    val = torch.empty(b, dtype=torch.float32, device=logits.device)
    rc = lib.pat_op_argmax(_ptr(logits.contiguous()), b, n, base, _ptr(idx), _ptr(val), _stream())
    if rc:
        raise PatError(rc, "pat_op_argmax")
    return idx, val


PAT_BARRIER_PROBE_BYTES = 16384


def pat_op_barrier_probe(n_workgroups, iters=200, max_spin=1 << 22, device="cuda:0"):
    """Mean microseconds per device-wide barrier among n_workgroups resident workgroups."""
    import torch
    lib = load_library()
    scratch = torch.empty(PAT_BARRIER_PROBE_BYTES, dtype=torch.uint8, device=device)
    us = C.c_double(0.0)
    rc = lib.pat_op_barrier_probe(_ptr(scratch), int(n_workgroups), int(iters), int(max_spin), C.byref(us), _stream())
    if rc:
        raise PatError(rc, "pat_op_barrier_probe")
    return us.value


def unpack_act(hi, lo, b, k):
    """Inverse of the packed activation layout (test helper: pure index arithmetic on the host).

    Returns float64 numpy [b, k] = hi + lo.
    """
    import torch
    KS = k // 32
    bt = (b + 15) // 16
    def one(t):
        a = t.view(torch.bfloat16).float().cpu().numpy().reshape(bt, KS, 4, 16, 8)   # [tile, ks, g, r, j]
        return a.transpose(0, 3, 1, 2, 4).reshape(bt * 16, k)[:b].astype(np.float64)
    return one(hi) + one(lo)


class Predictor:
    """Latency predictor fitted to grid rows (include/pat_switch.h); argument marshalling only.

    rows: a ctypes array of pat_grid_row (as pat_profile_grid returns) or an iterable of
    (tp, batch, sum_context, mean_us) tuples of measured points."""

    def __init__(self, rows):
        self._lib = load_library()
        if not (isinstance(rows, C.Array) and rows._type_ is pat_grid_row):
            rows = list(rows)
            arr = (pat_grid_row * len(rows))()
            for r, (tp, b, t, us) in zip(arr, rows):
                r.tp_degree, r.batch, r.sum_context, r.mean_us, r.skipped = int(tp), int(b), int(t), float(us), 0
            rows = arr
        self._h = C.c_void_p()
        rc = self._lib.pat_predictor_fit(rows, len(rows), C.byref(self._h))
        if rc:
            raise PatError(rc, "pat_predictor_fit")

    def close(self):
        if self._h:
            self._lib.pat_predictor_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def pat_predictor_line(self, tp, batch):
        a, b = C.c_double(), C.c_double()
        rc = self._lib.pat_predictor_line(self._h, tp, batch, C.byref(a), C.byref(b))
        if rc:
            raise PatError(rc, "pat_predictor_line")
        return a.value, b.value

    def pat_predictor_query(self, tp, batch, sum_context):
        out = C.c_double()
        rc = self._lib.pat_predictor_query(self._h, tp, batch, float(sum_context), C.byref(out))
        if rc:
            raise PatError(rc, "pat_predictor_query")
        return out.value

    def pat_switch_decide(self, tp, tp_list, groups, l_max, l_gen, lengths, model, fixed_us, net_bytes_per_s, n_gpus,
                          prefill=None):
        """groups: [(batch, context tokens)] per DP group; model = (n_layers, hidden, bytes per element);
        fixed_us: {(tp_from, tp_to): microseconds}; prefill: [(tp, batch, length, microseconds)] or None.
        Returns (do_switch, tp_new, t_cur_us, t_best_us, [(tp, t_rem, t_switch, t_total)])."""
        n = len(tp_list)
        inp = pat_switch_input()
        tpl = (C.c_int32 * n)(*tp_list)
        gb = (C.c_int32 * len(groups))(*[int(g[0]) for g in groups])
        gc = (C.c_double * len(groups))(*[float(g[1]) for g in groups])
        ln = (C.c_int32 * max(1, len(lengths)))(*[int(x) for x in lengths])
        fx = (C.c_double * (n * n))(*[float(fixed_us.get((a, b), 0.0)) for a in tp_list for b in tp_list])
        inp.tp, inp.tp_list, inp.n_tp, inp.n_gpus = tp, tpl, n, n_gpus
        inp.group_batch, inp.group_context, inp.n_groups = gb, gc, len(groups)
        inp.l_max, inp.l_gen, inp.lengths, inp.n_lengths = l_max, l_gen, ln, len(lengths)
        inp.n_layers, inp.hidden, inp.bytes_per_elem = model
        inp.net_bytes_per_s, inp.fixed_us = float(net_bytes_per_s), fx
        if prefill:
            pf = (pat_prefill_row * len(prefill))()
            for r, (ptp, pb, pl, pus) in zip(pf, prefill):
                r.tp_degree, r.batch, r.length, r.latency_us = int(ptp), int(pb), int(pl), float(pus)
            inp.prefill, inp.n_prefill = pf, len(prefill)
        rem, sw, tot = (C.c_double * n)(), (C.c_double * n)(), (C.c_double * n)()
        out = pat_switch_decision()
        out.t_rem_us, out.t_switch_us, out.t_total_us = rem, sw, tot
        rc = self._lib.pat_switch_decide(self._h, C.byref(inp), C.byref(out))
        if rc:
            raise PatError(rc, "pat_switch_decide")
        return bool(out.do_switch), out.tp_new, out.t_cur_us, out.t_best_us, [(tp_list[j], rem[j], sw[j], tot[j]) for j in range(n)]


def pat_kv_move_seconds(lengths, n_layers, hidden, bytes_per_elem, tp_src, net_bytes_per_s):
    ln = (C.c_int32 * max(1, len(lengths)))(*[int(x) for x in lengths])
    return load_library().pat_kv_move_seconds(ln, len(lengths), n_layers, hidden, bytes_per_elem, tp_src, float(net_bytes_per_s))


def pat_rms_length(lengths):
    ln = (C.c_int32 * len(lengths))(*[int(x) for x in lengths])
    return load_library().pat_rms_length(ln, len(lengths))


def pat_profile_plan(n_gpus, t_cap, l_max, capacity=None):
    """The offline profiler's sampling plan as a list of (tp_degree, batch, kv_len)."""
    lib = load_library()
    n = C.c_int32(0)
    rc = lib.pat_profile_plan(int(n_gpus), int(t_cap), int(l_max), None, C.byref(n))
    if rc != 0:
        raise PatError(rc, "pat_profile_plan: bad arguments")
    cap = n.value if capacity is None else int(capacity)
    pts = (pat_plan_point * max(1, cap))()
    n = C.c_int32(cap)
    rc = lib.pat_profile_plan(int(n_gpus), int(t_cap), int(l_max), pts, C.byref(n))
    if rc != 0:
        raise PatError(rc, "pat_profile_plan: %d points do not fit a capacity of %d" % (n.value, cap))
    return [(pts[i].tp_degree, pts[i].batch, pts[i].kv_len) for i in range(n.value)]
