"""ctypes front end of the CPU oracle (TEST INFRASTRUCTURE, not product code).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
It marshals numpy arrays into `pat_oracle.c`; the only logic here is the loop
"for each sequence, for each layer" that strings the C sub-layer calls into a
decode step, in the order the step is defined.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pat_oracle.c")


def build(force: bool = False) -> None:
    """Compile the float64 oracle and its float32 twin with gcc."""
    for real, name in (("double", "libpat_oracle_f64.so"), ("float", "libpat_oracle_f32.so")):
        out = os.path.join(_HERE, name)
        if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(_SRC):
            subprocess.check_call(
                ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-fno-fast-math",
                 "-ffp-contract=off", f"-DORC_REAL={real}", _SRC, "-o", out, "-lm"])


_u16p = C.POINTER(C.c_uint16)
_i32p = C.POINTER(C.c_int32)


def _p(a, ct):
    return a.ctypes.data_as(ct)


class Oracle:
    """One precision of the oracle ("f64" is the reference, "f32" its twin)."""

    def __init__(self, precision: str = "f64"):
        build()
        self.lib = C.CDLL(os.path.join(_HERE, f"libpat_oracle_{precision}.so"))
        self.real = np.float64 if precision == "f64" else np.float32
        self._rp = C.POINTER(C.c_double if precision == "f64" else C.c_float)
        creal = C.c_double if precision == "f64" else C.c_float
        L = self.lib
        assert L.orc_real_bytes() == np.dtype(self.real).itemsize
        L.orc_bf16_to_real.restype = creal
        L.orc_bf16_to_real.argtypes = [C.c_uint16]
        L.orc_real_to_bf16.restype = C.c_uint16
        L.orc_real_to_bf16.argtypes = [creal]
        L.orc_silu.restype = creal
        L.orc_silu.argtypes = [creal]
        for name in ("orc_embed", "orc_rmsnorm", "orc_matvec", "orc_rope", "orc_softmax", "orc_attend",
                     "orc_attn_sublayer", "orc_ffn_sublayer", "orc_layer", "orc_logits"):
            getattr(L, name).restype = None

    # -- helpers ------------------------------------------------------------
    def _r(self, a):
        a = np.ascontiguousarray(a, dtype=self.real)
        return a, _p(a, self._rp)

    @staticmethod
    def _b(a):
        a = np.ascontiguousarray(a)
        assert a.dtype == np.uint16, a.dtype
        return a, _p(a, _u16p)

    # -- scalar / elementwise -------------------------------------------------
    def bf16_to_real(self, bits: int) -> float:
        return float(self.lib.orc_bf16_to_real(int(bits)))

    def real_to_bf16(self, v: float) -> int:
        return int(self.lib.orc_real_to_bf16(v))

    def silu(self, z: float) -> float:
        return float(self.lib.orc_silu(z))

    # -- operators ------------------------------------------------------------
    def embed(self, row_bits):
        row, rp = self._b(row_bits)
        x = np.empty(row.shape[0], self.real)
        self.lib.orc_embed(rp, C.c_int(row.shape[0]), _p(x, self._rp))
        return x

    def rmsnorm(self, x, g_bits, eps):
        x, xp = self._r(x)
        g, gp = self._b(g_bits)
        out = np.empty_like(x)
        self.lib.orc_rmsnorm(xp, gp, C.c_int(x.shape[0]), C.c_double(eps), _p(out, self._rp))
        return out

    def matvec(self, w_bits, x):
        w, wp = self._b(w_bits)
        x, xp = self._r(x)
        n, k = w.shape
        assert x.shape == (k,)
        y = np.empty(n, self.real)
        self.lib.orc_matvec(wp, C.c_int(n), C.c_int(k), C.c_int(k), xp, _p(y, self._rp))
        return y

    def rope(self, v, pos, base):
        v, vp = self._r(np.array(v, dtype=self.real, copy=True))
        self.lib.orc_rope(vp, C.c_int(v.shape[0]), C.c_int(pos), C.c_double(base))
        return v

    def softmax(self, s):
        s, sp = self._r(np.array(s, dtype=self.real, copy=True))
        self.lib.orc_softmax(sp, C.c_int(s.shape[0]))
        return s

    def attend(self, q, k_bits, v_bits):
        """q [d]; k_bits, v_bits [n, d] uint16 -> (o [d], p [n])."""
        q, qp = self._r(q)
        k, kp = self._b(k_bits)
        v, vp = self._b(v_bits)
        n, d = k.shape
        o = np.empty(d, self.real)
        p = np.empty(n, self.real)
        self.lib.orc_attend(qp, kp, vp, C.c_int(n), C.c_int(d), C.c_int(d), _p(o, self._rp), _p(p, self._rp))
        return o, p

    def attn_sublayer(self, shp, w, x, kc, vc, L):
        """shp = (H, hq, hkv, d, eps, rope_base); kc, vc uint16 [cap, hkv, d], modified at L."""
        H, hq, hkv, d, eps, base = shp
        x, xp = self._r(x)
        assert kc.flags.c_contiguous and vc.flags.c_contiguous and kc.shape[0] > L
        g1, g1p = self._b(w["g1"]); wqkv, wqp = self._b(w["wqkv"]); wo, wop = self._b(w["wo"])
        assert wqkv.shape == ((hq + 2 * hkv) * d, H) and wo.shape == (H, hq * d)
        delta = np.empty(H, self.real)
        gq = gk = None
        if "gq" in w:                                    # model family with per-head q/k normalisation
            (gqa, gq), (gka, gk) = self._b(w["gq"]), self._b(w["gk"])
            assert gqa.shape == (d,) and gka.shape == (d,)
        self.lib.orc_attn_sublayer_qkn(C.c_int(H), C.c_int(hq), C.c_int(hkv), C.c_int(d), C.c_double(eps),
                                       C.c_double(base), g1p, wqp, wop, gq, gk, xp, _p(kc, _u16p), _p(vc, _u16p),
                                       C.c_int(L), _p(delta, self._rp))
        return delta

    def ffn_sublayer(self, H, F, eps, w, x):
        x, xp = self._r(x)
        g2, g2p = self._b(w["g2"]); wg, wgp = self._b(w["wg"]); wu, wup = self._b(w["wu"]); wd, wdp = self._b(w["wd"])
        assert wg.shape == (F, H) and wu.shape == (F, H) and wd.shape == (H, F)
        delta = np.empty(H, self.real)
        self.lib.orc_ffn_sublayer(C.c_int(H), C.c_int(F), C.c_double(eps), g2p, wgp, wup, wdp, xp,
                                  _p(delta, self._rp))
        return delta

    def layer(self, shp, F, w, x, kc, vc, L):
        """x (modified in place, must be a contiguous `real` array) through one layer."""
        H, hq, hkv, d, eps, base = shp
        assert x.dtype == self.real and x.flags.c_contiguous
        g1, g1p = self._b(w["g1"]); wqkv, wqp = self._b(w["wqkv"]); wo, wop = self._b(w["wo"])
        g2, g2p = self._b(w["g2"]); wg, wgp = self._b(w["wg"]); wu, wup = self._b(w["wu"]); wd, wdp = self._b(w["wd"])
        assert kc.flags.c_contiguous and vc.flags.c_contiguous and kc.shape[0] > L
        gq = gk = None
        if "gq" in w:                                    # model family with per-head q/k normalisation
            (gqa, gq), (gka, gk) = self._b(w["gq"]), self._b(w["gk"])
            assert gqa.shape == (d,) and gka.shape == (d,)
        self.lib.orc_layer_qkn(C.c_int(H), C.c_int(hq), C.c_int(hkv), C.c_int(d), C.c_int(F), C.c_double(eps),
                               C.c_double(base), g1p, wqp, wop, g2p, wgp, wup, wdp, gq, gk, _p(x, self._rp),
                               _p(kc, _u16p), _p(vc, _u16p), C.c_int(L))

    def logits(self, H, eps, w, x):
        x, xp = self._r(x)
        gf, gfp = self._b(w["gf"]); wlm, wlp = self._b(w["wlm"])
        out = np.empty(wlm.shape[0], self.real)
        self.lib.orc_logits(C.c_int(H), C.c_int(wlm.shape[0]), C.c_double(eps), gfp, wlp, xp, _p(out, self._rp))
        return out

    def argmax(self, v) -> int:
        v, vp = self._r(v)
        return int(self.lib.orc_argmax(vp, C.c_int(v.shape[0])))

    def argmax_f32(self, v) -> int:
        v = np.ascontiguousarray(v, dtype=np.float32)
        return int(self.lib.orc_argmax_f32(_p(v, C.POINTER(C.c_float)), C.c_int(v.shape[0])))

    def finish(self, tok, gen, kv_len, target, eos=-1):
        """gen and kv_len (int32 arrays) are advanced in place; returns (fin, n_finished)."""
        B = len(tok)
        tok = np.ascontiguousarray(tok, np.int32); target = np.ascontiguousarray(target, np.int32)
        assert gen.dtype == np.int32 and kv_len.dtype == np.int32
        fin = np.zeros(B, np.int32)
        nf = self.lib.orc_finish(C.c_int(B), _p(tok, _i32p), _p(gen, _i32p), _p(kv_len, _i32p),
                                 _p(target, _i32p), C.c_int(eos), _p(fin, _i32p))
        return fin, int(nf)

    def compact_map(self, fin):
        fin = np.ascontiguousarray(fin, np.int32)
        m = np.empty(len(fin), np.int32)
        nb = self.lib.orc_compact_map(C.c_int(len(fin)), _p(fin, _i32p), _p(m, _i32p))
        return m, int(nb)


def bits(t):
    """torch bf16 tensor (CPU) -> numpy uint16 bit patterns, same shape."""
    import torch
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


class OracleDecoder:
    """A live batch decoded by the oracle, one sequence at a time.

    State per sequence: last token, kv_len, gen, target, seq_id and a contiguous
    bf16 cache [n_layers][cap, hkv, d] (K and V).  `layer_w(l)` / `final_w` give
    uint16 weight dicts; `embed_row(tok)` gives one embedding row's bits.
    """

    def __init__(self, oracle: Oracle, dims, layer_w, final_w, embed_row, vocab0=0, eos=-1):
        # dims = (n_layers, H, hq, hkv, d, F, eps, rope_base)
        self.o, self.dims = oracle, dims
        self.layer_w, self.final_w, self.embed_row = layer_w, final_w, embed_row
        self.vocab0, self.eos = vocab0, eos
        self.seq_id = np.zeros(0, np.int32); self.tok = np.zeros(0, np.int32)
        self.kv_len = np.zeros(0, np.int32); self.gen = np.zeros(0, np.int32)
        self.target = np.zeros(0, np.int32); self.fin = np.zeros(0, np.int32)
        self.kc, self.vc = [], []      # per sequence: list over layers of [cap, hkv, d] uint16

    def admit(self, seq_id, tok, kv_len, target, k_bits, v_bits, cap_extra):
        """k_bits / v_bits: list over layers of uint16 [kv_len, hkv, d] for this one sequence."""
        NL, H, hq, hkv, d = self.dims[:5]
        cap = int(kv_len) + int(cap_extra)
        kc, vc = [], []
        for l in range(NL):
            a = np.zeros((cap, hkv, d), np.uint16); b = np.zeros((cap, hkv, d), np.uint16)
            a[:kv_len] = k_bits[l]; b[:kv_len] = v_bits[l]
            kc.append(a); vc.append(b)
        self.kc.append(kc); self.vc.append(vc)
        self.seq_id = np.append(self.seq_id, np.int32(seq_id)); self.tok = np.append(self.tok, np.int32(tok))
        self.kv_len = np.append(self.kv_len, np.int32(kv_len)); self.gen = np.append(self.gen, np.int32(0))
        self.target = np.append(self.target, np.int32(target)); self.fin = np.append(self.fin, np.int32(0))

    def step(self):
        """One decode step over every live slot.  Returns (logits [B, Vs] real, next tokens)."""
        NL, H, hq, hkv, d, F, eps, base = self.dims
        o = self.o
        B = len(self.tok)
        logits, nxt = [], np.zeros(B, np.int32)
        xs = [o.embed(self.embed_row(int(self.tok[i]))) for i in range(B)]
        for l in range(NL):
            w = self.layer_w(l)
            for i in range(B):
                o.layer((H, hq, hkv, d, eps, base), F, w, xs[i], self.kc[i][l], self.vc[i][l], int(self.kv_len[i]))
        fw = self.final_w
        for i in range(B):
            lg = o.logits(H, eps, fw, xs[i])
            logits.append(lg)
            nxt[i] = self.vocab0 + o.argmax(lg)
        self.tok = nxt.copy()
        self.fin, nf = o.finish(self.tok, self.gen, self.kv_len, self.target, self.eos)
        return np.stack(logits) if B else np.zeros((0, 0)), nxt, nf

    def compact(self):
        m, nb = self.o.compact_map(self.fin)
        keep = [j for j in range(len(m)) if m[j] >= 0]
        for name in ("seq_id", "tok", "kv_len", "gen", "target", "fin"):
            setattr(self, name, getattr(self, name)[keep].copy())
        self.kc = [self.kc[j] for j in keep]; self.vc = [self.vc[j] for j in keep]
        return nb


def kv_extract(od: OracleDecoder, slots, layer0, n_layers, head0, n_heads):
    """Valid K/V of the chosen live slots as one buffer [layer][K|V][head][token][d] (uint16 bf16 bits),
    the tokens of the slots back to back in the order given: the send buffer of the paper's KV
    migration (Sec. 4.2, "All-Gather and Slice": only valid states of unfinished samples move, as
    plain copies).  Written out element by element."""
    d = od.dims[4]
    t_sel = int(sum(int(od.kv_len[s]) for s in slots))
    out = np.zeros((n_layers, 2, n_heads, t_sel, d), np.uint16)
    for l in range(n_layers):
        for h in range(n_heads):
            t = 0
            for s in slots:
                for tok in range(int(od.kv_len[s])):
                    out[l, 0, h, t] = od.kc[s][layer0 + l][tok, head0 + h]
                    out[l, 1, h, t] = od.vc[s][layer0 + l][tok, head0 + h]
                    t += 1
    return out


def prefill(od: OracleDecoder, slot, tokens):
    """Rebuild the K/V states of one live slot from its token ids (the recomputation way of restoring
    a sample after a switch, Sec. 4.2: the token sequence is all that moves, a prefill pass builds
    the states).  Causal attention written out as what it means: the token at position t is embedded
    and taken through every layer with the cache holding positions 0 .. t-1, which appends its own
    K/V at position t.  Overwrites positions 0 .. kv_len-1 of the slot's cache in every layer; the
    slot's other state is untouched."""
    NL, H, hq, hkv, d, F, eps, base = od.dims
    L = int(od.kv_len[slot])
    assert len(tokens) == L
    for t in range(L):
        x = od.o.embed(od.embed_row(int(tokens[t])))
        for l in range(NL):
            od.o.layer((H, hq, hkv, d, eps, base), F, od.layer_w(l), x, od.kc[slot][l], od.vc[slot][l], t)
