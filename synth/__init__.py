"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU library's tests / bench.

Holds no arithmetic of the method: only shapes, random weights, random prompts, random caches.
Everything is drawn from numpy's counter-based Philox generator keyed by (seed, stream id), so a
tensor's values depend only on its own stream, never on what was drawn before it.

The models are random-init stand-ins for the decoder families the paper evaluates (Experiment,
"Base LLM"): weights i.i.d. N(0, 0.02^2), norm gains 1, prompts uniform random token ids.
"""
from dataclasses import dataclass, asdict

import numpy as np


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    dtype: str  # "bf16" | "f32"
    rope_theta: float = 10000.0
    rms_eps: float = 1e-6

    def cfg(self):
        d = asdict(self)
        d.pop("name")
        return d

    def scaled(self, **kw):
        d = asdict(self)
        d.update(kw)
        return ModelShape(**d)


@dataclass(frozen=True)
class Workload:
    name: str
    model: ModelShape
    batch: int
    prefix_lo: int
    prefix_hi: int  # inclusive; == prefix_lo for a fixed prefix
    k: int
    steps: int
    seed: int


TINY = ModelShape("tiny-f32", 2, 256, 4, 4, 64, 1024, 1024, "f32")
M1B = ModelShape("1b-bf16", 16, 2048, 32, 8, 64, 8192, 32000, "bf16")
M8B = ModelShape("8b-bf16", 32, 4096, 32, 8, 128, 14336, 128256, "bf16")
M14B = ModelShape("14b-bf16", 40, 5120, 40, 8, 128, 13824, 152064, "bf16")

# index i = the i-th configuration of the baseline list (0-based)
WORKLOADS = [
    Workload("tiny-f32-b4-p64-k4", TINY, 4, 64, 64, 4, 16, 203401),
    Workload("1b-bf16-b32-p512-k4", M1B, 32, 512, 512, 4, 128, 203402),
    Workload("8b-bf16-b64-p256..2048-k4", M8B, 64, 256, 2048, 4, 64, 203403),
    Workload("8b-bf16-b256-p1024-ksweep", M8B, 256, 1024, 1024, 4, 32, 203404),
    Workload("14b-bf16-b128-p1024..4096-k4", M14B, 128, 1024, 4096, 4, 32, 203405),
]


def rng(seed, stream):
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def to_bf16_values(a):
    """Round float32 values to the nearest bf16-representable float32 (ties to even)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(a.shape)


def bf16_bits(a):
    """uint16 bit patterns of bf16-representable float32 values (for upload as torch.bfloat16)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> 16).astype(np.uint16).reshape(a.shape)


def _normal(seed, stream, shape, std, dtype):
    a = (rng(seed, stream).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)
    return to_bf16_values(a) if dtype == "bf16" else a


def target_weights(m: ModelShape, seed, std=0.02):
    """Dict of float32 arrays; linear weights are [out_features, in_features]."""
    d, hd, F, V, L = m.d_model, m.head_dim, m.d_ffn, m.vocab, m.n_layers
    nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * hd
    w = {"embed": _normal(seed, 1, (V, d), std, m.dtype),
         "lm_head": _normal(seed, 2, (V, d), std, m.dtype),
         "final_norm": np.ones(d, np.float32)}
    for name in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate", "w_up", "w_down"):
        w[name] = []
    for l in range(L):
        s = 100 + 10 * l
        w["attn_norm"].append(np.ones(d, np.float32))
        w["wqkv"].append(_normal(seed, s + 1, (nqkv, d), std, m.dtype))
        w["wo"].append(_normal(seed, s + 2, (d, m.n_q_heads * hd), std, m.dtype))
        w["ffn_norm"].append(np.ones(d, np.float32))
        w["w_gate"].append(_normal(seed, s + 3, (F, d), std, m.dtype))
        w["w_up"].append(_normal(seed, s + 4, (F, d), std, m.dtype))
        w["w_down"].append(_normal(seed, s + 5, (d, F), std, m.dtype))
    return w


def draft_weights(m: ModelShape, k_max, seed, std=0.02):
    d, hd, F = m.d_model, m.head_dim, m.d_ffn
    nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * hd
    s = 50000
    return {
        "group_norm": np.ones((4, d), np.float32),
        "w_ds": _normal(seed, s + 1, (d, 4 * d), std, m.dtype),
        "pos_norm": np.ones(d, np.float32),
        "w_pos": _normal(seed, s + 2, (k_max * d, d), std, m.dtype),
        "b_pos": _normal(seed, s + 3, (k_max * d,), std, m.dtype),
        "attn_norm": np.ones(d, np.float32),
        "wqkv": _normal(seed, s + 4, (nqkv, d), std, m.dtype),
        "wo": _normal(seed, s + 5, (d, m.n_q_heads * hd), std, m.dtype),
        "ffn_norm": np.ones(d, np.float32),
        "w_gate": _normal(seed, s + 6, (F, d), std, m.dtype),
        "w_up": _normal(seed, s + 7, (F, d), std, m.dtype),
        "w_down": _normal(seed, s + 8, (d, F), std, m.dtype),
        "out_norm": np.ones(d, np.float32),
        # the slot attention's own parameter set (two-stage wiring of the draft block)
        "sa_norm": np.ones(d, np.float32),
        "sa_wqkv": _normal(seed, s + 9, (nqkv, d), std, m.dtype),
        "sa_wo": _normal(seed, s + 10, (d, m.n_q_heads * hd), std, m.dtype),
    }


def prefix_lengths(B, lo, hi, seed):
    """One inclusive-uniform draw per sequence."""
    if lo == hi:
        return np.full(B, lo, np.int32)
    return rng(seed, 900).integers(lo, hi + 1, size=B).astype(np.int32)


def prompts(lens, vocab, seed):
    g = rng(seed, 901)
    return [g.integers(0, vocab, size=int(n)).astype(np.int32) for n in lens]


def random_qkv(seed, B, nq, Hq, Hkv, hd, cap, dtype, k_std=1.0):
    """Random attention operands: q [B,nq,Hq,hd], k/v caches [B,Hkv,cap,hd] (every slot filled,
    so reads of dead slots show up)."""
    q = _normal(seed, 11, (B, nq, Hq, hd), 1.0, dtype)
    kc = _normal(seed, 12, (B, Hkv, cap, hd), k_std, dtype)
    vc = _normal(seed, 13, (B, Hkv, cap, hd), 1.0, dtype)
    return q, kc, vc


def kv_capacity(max_prefix, steps, k, align=64):
    need = int(max_prefix) + (steps + 1) * (k + 1)
    return (need + align - 1) // align * align


def device_weights(m: ModelShape, k_max, seed, two_stage=False, std=0.02, device="cuda"):
    """The same recipe drawn with torch's generator directly on `device` (for models too large to draw
    on the host in reasonable time): N(0, std^2) matrices in the model dtype, norm gains 1.  Returns
    (target dict, draft dict) of torch tensors in the layout the GPU engine binds: gate and up stacked as
    w_gate_up = [gate; up].  host_weights() turns them into the oracle's numpy dicts."""
    import torch
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    dt = torch.bfloat16 if m.dtype == "bf16" else torch.float32

    def rnd(*shape):
        return (torch.randn(*shape, generator=g, device=device, dtype=torch.float32) * std).to(dt)

    def ones(*shape):
        return torch.ones(*shape, device=device, dtype=dt)
    d, hd, F, V, L = m.d_model, m.head_dim, m.d_ffn, m.vocab, m.n_layers
    nqkv = (m.n_q_heads + 2 * m.n_kv_heads) * hd
    tw = {"embed": rnd(V, d), "lm_head": rnd(V, d), "final_norm": ones(d),
          "attn_norm": [ones(d) for _ in range(L)], "wqkv": [rnd(nqkv, d) for _ in range(L)],
          "wo": [rnd(d, m.n_q_heads * hd) for _ in range(L)], "ffn_norm": [ones(d) for _ in range(L)],
          "w_gate_up": [rnd(2 * F, d) for _ in range(L)], "w_down": [rnd(d, F) for _ in range(L)]}
    dw = {"group_norm": ones(4, d), "w_ds": rnd(d, 4 * d), "pos_norm": ones(d), "w_pos": rnd(max(k_max, 1) * d, d),
          "b_pos": rnd(max(k_max, 1) * d), "attn_norm": ones(d), "wqkv": rnd(nqkv, d), "wo": rnd(d, m.n_q_heads * hd),
          "ffn_norm": ones(d), "w_gate_up": rnd(2 * F, d), "w_down": rnd(d, F), "out_norm": ones(d)}
    if two_stage:      # the slot attention's own parameter set
        dw.update({"sa_norm": ones(d), "sa_wqkv": rnd(nqkv, d), "sa_wo": rnd(d, m.n_q_heads * hd)})
    return tw, dw


def host_weights(tw, dw=None):
    """device_weights() dicts -> float32 numpy dicts with the oracle's key names (w_gate / w_up apart)."""
    def h(t):
        return t.detach().float().cpu().numpy()

    def conv(w, per_layer):
        out = {}
        for n, v in w.items():
            if n == "w_gate_up":
                halves = [h(x) for x in v] if per_layer else h(v)
                if per_layer:
                    out["w_gate"] = [np.ascontiguousarray(x[:x.shape[0] // 2]) for x in halves]
                    out["w_up"] = [np.ascontiguousarray(x[x.shape[0] // 2:]) for x in halves]
                else:
                    out["w_gate"] = np.ascontiguousarray(halves[:halves.shape[0] // 2])
                    out["w_up"] = np.ascontiguousarray(halves[halves.shape[0] // 2:])
            else:
                out[n] = [h(x) for x in v] if isinstance(v, list) else h(v)
        return out
    return conv(tw, True), (conv(dw, False) if dw is not None else None)
