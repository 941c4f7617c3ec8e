"""ctypes wrapper around the CPU oracle (oracle/sfo.c).  Test infrastructure only: imported by
tests/, by __graft_entry__.smoke() and by bench.py's cpu_baseline leg -- never by the product.

All arrays are numpy: weights float32, activations / caches / logits float64, integers int32.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

MASK_CAUSAL, MASK_BIDIR = 0, 1
DRAFT_TWO_STAGE = 16   # OR-ed into draft_step's mask_mode: context attention and slot attention kept apart

_f = C.POINTER(C.c_float)
_d = C.POINTER(C.c_double)
_i = C.POINTER(C.c_int32)


class Cfg(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] + \
               [("rope_theta", C.c_double), ("rms_eps", C.c_double), ("round_bf16", C.c_int32)]


class TargetW(C.Structure):
    _fields_ = [("embed", _f), ("lm_head", _f), ("final_norm", _f),
                ("attn_norm", C.POINTER(_f)), ("wqkv", C.POINTER(_f)), ("wo", C.POINTER(_f)),
                ("ffn_norm", C.POINTER(_f)), ("w_gate", C.POINTER(_f)), ("w_up", C.POINTER(_f)),
                ("w_down", C.POINTER(_f))]


class DraftW(C.Structure):
    _fields_ = [(n, _f) for n in
                ("group_norm", "w_ds", "pos_norm", "w_pos", "b_pos", "attn_norm", "wqkv", "wo",
                 "ffn_norm", "w_gate", "w_up", "w_down", "out_norm", "sa_norm", "sa_wqkv", "sa_wo")]


class State(C.Structure):
    _fields_ = [("B", C.c_int32), ("cap", C.c_int32), ("q_max", C.c_int32),
                ("tk", _d), ("tv", _d), ("dk", _d), ("dv", _d),
                ("kv_len", _i), ("pending", _i), ("hooks", _d), ("n_new", _i), ("cu_new", _i)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(_build.build())
        _lib.sfo_round_bf16.restype = C.c_double
        _lib.sfo_round_bf16.argtypes = [C.c_double]
        _lib.sfo_argmax.restype = C.c_int32
    return _lib


def _fp(a):
    assert a.dtype == np.float32 and a.flags.c_contiguous
    return a.ctypes.data_as(_f)


def _dp(a):
    assert a.dtype == np.float64 and a.flags.c_contiguous
    return a.ctypes.data_as(_d)


def _ip(a):
    assert a.dtype == np.int32 and a.flags.c_contiguous
    return a.ctypes.data_as(_i)


def _c64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def _c32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


# ---- primitives ------------------------------------------------------------------------------
def round_bf16(x):
    x = np.asarray(x, dtype=np.float64)
    out = np.empty_like(x)
    flat, o = x.reshape(-1), out.reshape(-1)
    f = lib().sfo_round_bf16
    for j in range(flat.size):
        o[j] = f(float(flat[j]))
    return out


def rmsnorm(x, g, eps=1e-6):
    x, g = _c64(x), _c32(g)
    M, d = x.reshape(-1, x.shape[-1]).shape
    y = np.empty_like(x)
    lib().sfo_rmsnorm(_dp(x), _fp(g), M, d, C.c_double(eps), _dp(y))
    return y


def group_rmsnorm(x, g, eps=1e-6):
    x, g = _c64(x), _c32(g)
    ng, d = x.shape[-2:]
    M = x.size // (ng * d)
    y = np.empty_like(x)
    lib().sfo_group_rmsnorm(_dp(x), _fp(g), M, ng, d, C.c_double(eps), _dp(y))
    return y


def linear(x, w, bias=None):
    x, w = _c64(x), _c32(w)
    M, K = x.reshape(-1, x.shape[-1]).shape
    N = w.shape[0]
    assert w.shape == (N, K)
    y = np.empty(x.shape[:-1] + (N,), dtype=np.float64)
    b = _fp(_c32(bias)) if bias is not None else None
    lib().sfo_linear(_dp(x), _fp(w), b, M, K, N, _dp(y))
    return y


def norm_linear(x, g, w, eps=1e-6, round_bf16=False):
    """RMSNorm(x; g) . w^T as the decoder layers' norm + linear pairs compute it."""
    x, g, w = _c64(x), _c32(g), _c32(w)
    M, K = x.shape
    N = w.shape[0]
    assert w.shape == (N, K) and g.shape == (K,)
    y = np.empty((M, N))
    lib().sfo_norm_linear(_dp(x), _fp(g), _fp(w), M, K, N, C.c_double(eps), int(bool(round_bf16)), _dp(y))
    return y


def rope(x, pos, theta=10000.0):
    x = _c64(x).copy()
    pos = np.ascontiguousarray(pos, dtype=np.int32)
    M, H, hd = x.shape
    assert pos.shape == (M,)
    lib().sfo_rope(_dp(x), _ip(pos), M, H, hd, C.c_double(theta))
    return x


def silu_mul(gate, up):
    gate, up = _c64(gate), _c64(up)
    y = np.empty_like(gate)
    lib().sfo_silu_mul(_dp(gate), _dp(up), C.c_long(gate.size), _dp(y))
    return y


def attention(q, kc, vc, lens, mode):
    """q [B,nq,Hq,hd]; kc, vc [B,Hkv,cap,hd]; lens [B]  ->  out [B,nq,Hq,hd]"""
    q, kc, vc = _c64(q), _c64(kc), _c64(vc)
    lens = np.ascontiguousarray(lens, dtype=np.int32)
    B, nq, Hq, hd = q.shape
    _, Hkv, cap, _ = kc.shape
    assert kc.shape == vc.shape == (B, Hkv, cap, hd) and Hq % Hkv == 0
    assert int(lens.max(initial=0)) + nq <= cap
    out = np.empty_like(q)
    lib().sfo_attention(_dp(q), _dp(kc), _dp(vc), _ip(lens), B, nq, Hq, Hkv, hd, cap, int(mode), _dp(out))
    return out


def argmax(x):
    x = _c64(x)
    return int(lib().sfo_argmax(_dp(x), x.size))


# ---- the model -------------------------------------------------------------------------------
class Oracle:
    """Holds weights + decoding state and runs the three steps of one speculative step.

    cfg: dict with n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_theta,
         rms_eps.  tw / dw: dicts of float32 numpy arrays with the key names of sfo.h (tw lists
         hold one array per layer).  The draft block uses the same widths as the target.
    """

    def __init__(self, cfg, tw, dw, B, cap, q_max, round_bf16=False):
        self.cfg_d = dict(cfg)
        L = cfg["n_layers"]
        self.B, self.cap, self.q_max, self.L = B, cap, q_max, L
        self.d, self.V = cfg["d_model"], cfg["vocab"]
        self.Hkv, self.hd = cfg["n_kv_heads"], cfg["head_dim"]

        def mk(n_layers):
            return Cfg(n_layers, cfg["d_model"], cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"],
                       cfg["d_ffn"], cfg["vocab"], cfg.get("rope_theta", 10000.0),
                       cfg.get("rms_eps", 1e-6), int(bool(round_bf16)))
        self.cfg_t, self.cfg_dr = mk(L), mk(1)
        self._keep = []
        self.tw = TargetW()
        for name in ("embed", "lm_head", "final_norm"):
            a = _c32(tw[name]); self._keep.append(a); setattr(self.tw, name, _fp(a))
        for name in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
            arrs = [_c32(a) for a in tw[name]]
            assert len(arrs) == L
            self._keep.append(arrs)
            parr = (_f * L)(*[_fp(a) for a in arrs]); self._keep.append(parr)
            setattr(self.tw, name, parr)
        self.lm_head = _c32(tw["lm_head"]); self._keep.append(self.lm_head)
        self.dw = None
        if dw is not None:
            self.dw = DraftW()
            for name, _t in DraftW._fields_:
                if name.startswith("sa_") and name not in dw:      # two-stage wiring not used
                    continue
                a = _c32(dw[name]); self._keep.append(a); setattr(self.dw, name, _fp(a))
        shp = (B, self.Hkv, cap, self.hd)
        self.tk = np.zeros((L,) + shp); self.tv = np.zeros((L,) + shp)
        self.dk = np.zeros(shp); self.dv = np.zeros(shp)
        self.kv_len = np.zeros(B, np.int32); self.pending = np.zeros(B, np.int32)
        self.hooks = np.zeros((B, q_max, 4, self.d))
        self.n_new = np.zeros(B, np.int32); self.cu_new = np.zeros(B + 1, np.int32)
        self.st = State(B, cap, q_max, _dp(self.tk), _dp(self.tv), _dp(self.dk), _dp(self.dv),
                        _ip(self.kv_len), _ip(self.pending), _dp(self.hooks), _ip(self.n_new),
                        _ip(self.cu_new))

    def verify_step(self, k, draft):
        draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(self.B, k)
        logits = np.empty((self.B, k + 1, self.V))
        rc = lib().sfo_verify_step(C.byref(self.cfg_t), C.byref(self.tw), C.byref(self.st), k,
                                   _ip(draft), _dp(logits))
        if rc != 0:
            raise ValueError("sfo_verify_step: capacity or argument error")
        return logits

    def draft_step(self, k, mask_mode=MASK_BIDIR, want_logits=False):
        draft = np.zeros((self.B, k), np.int32)
        lg = np.empty((self.B, k, self.V)) if want_logits else None
        rc = lib().sfo_draft_step(C.byref(self.cfg_dr), C.byref(self.dw), _fp(self.lm_head),
                                  C.byref(self.st), k, int(mask_mode), _ip(draft),
                                  _dp(lg) if want_logits else None)
        if rc != 0:
            raise ValueError("sfo_draft_step: capacity or argument error")
        return (draft, lg) if want_logits else draft

    def accept_commit(self, k, draft, logits, force_len=None):
        draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(self.B, k)
        logits = _c64(logits)
        assert logits.shape == (self.B, k + 1, self.V)
        acc = np.zeros(self.B, np.int32)
        out = np.zeros((self.B, k + 1), np.int32)
        fl = None
        if force_len is not None:
            fl_a = np.ascontiguousarray(force_len, dtype=np.int32)
            fl = _ip(fl_a)
        rc = lib().sfo_accept_commit(C.byref(self.st), k, self.V, _ip(draft), _dp(logits), fl,
                                     _ip(acc), _ip(out))
        if rc != 0:
            raise ValueError("sfo_accept_commit: argument error")
        return acc, out

    def prefill(self, prompts):
        """Run the target causally over every prompt in one block (a verify pass whose block is
        the whole prompt), commit all of it and set the pending token to the target's choice
        after the last prompt token.  n_new = prompt length, so the next draft_step fills the
        draft cache from the hooked states of every prompt position.  Returns the first emitted
        token of every sequence."""
        lens = np.array([len(p) for p in prompts], np.int32)
        P = int(lens.max())
        assert P <= self.q_max and len(prompts) == self.B
        toks = np.zeros((self.B, P), np.int32)
        for b, p in enumerate(prompts):
            toks[b, :len(p)] = p
        self.kv_len[:] = 0
        self.pending[:] = toks[:, 0]
        logits = self.verify_step(P - 1, toks[:, 1:])
        self.accept_commit(P - 1, toks[:, 1:], logits, force_len=lens)
        return self.pending.copy()

    def snapshot(self):
        return {n: getattr(self, n).copy() for n in
                ("tk", "tv", "dk", "dv", "kv_len", "pending", "hooks", "n_new", "cu_new")}

    def restore(self, snap):
        for n, a in snap.items():
            getattr(self, n)[...] = a


def ncores():
    return len(os.sched_getaffinity(0))
