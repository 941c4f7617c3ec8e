"""Device-buffer owner for libspecformer: allocates weights, caches, state and workspace as PyTorch
tensors and hands their pointers to the C ABI.  Method names mirror the C entry points; no step
of the path is computed here (torch is used for memory, streams and host<->device copies only).
"""
import ctypes as C

import numpy as np
import torch

from . import binding as sfb


def _ptr(t):
    return C.c_void_p(t.data_ptr()) if t is not None else None


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


class Engine:
    def __init__(self, cfg, B, cap, max_k, device="cuda:0", share_caches=None):
        """cfg: dict(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, dtype
        ('bf16'|'f32'), rope_theta, rms_eps).  share_caches: another engine of the same shape, batch and
        capacity whose K/V cache buffers this one works on instead of allocating its own."""
        self.lib = sfb.lib()
        self.cfg = dict(cfg)
        self.B, self.cap, self.max_k = int(B), int(cap), int(max_k)
        self.dev = torch.device(device)
        self.dtype_id = sfb.SF_BF16 if cfg["dtype"] == "bf16" else sfb.SF_F32
        self.tdtype = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        self.L, self.d, self.V = cfg["n_layers"], cfg["d_model"], cfg["vocab"]
        self.Hq, self.Hkv, self.hd, self.F = cfg["n_q_heads"], cfg["n_kv_heads"], cfg["head_dim"], cfg["d_ffn"]

        def mk(n_layers):
            return sfb.ModelCfg(n_layers, self.d, self.Hq, self.Hkv, self.hd, self.F, self.V,
                                float(cfg.get("rope_theta", 10000.0)), float(cfg.get("rms_eps", 1e-6)),
                                self.dtype_id)
        self._tc, self._dc = mk(self.L), mk(1)
        self.ctx = C.c_void_p()
        sfb.check(self.lib.sf_create(C.byref(self._tc), C.byref(self._dc), self.B, self.max_k, C.byref(self.ctx)),
                  "sf_create")
        es = 2 if self.dtype_id == sfb.SF_BF16 else 4
        tb = self.lib.sf_kv_cache_bytes(self.ctx, 0, self.B, self.cap)
        db = self.lib.sf_kv_cache_bytes(self.ctx, 1, self.B, self.cap)
        assert tb and db
        z = lambda nbytes: torch.zeros(nbytes // es, dtype=self.tdtype, device=self.dev)
        if share_caches is not None:
            o = share_caches
            assert (o.B, o.cap, o.cfg) == (self.B, self.cap, self.cfg) and o.tk.numel() * es == tb
            self.tk, self.tv, self.dk, self.dv = o.tk, o.tv, o.dk, o.dv
        else:
            self.tk, self.tv, self.dk, self.dv = z(tb), z(tb), z(db), z(db)
        self.layer_elems = db // es
        i32 = dict(dtype=torch.int32, device=self.dev)
        self.kv_len = torch.zeros(self.B, **i32)
        self.pending = torch.zeros(self.B, **i32)
        self.n_new = torch.zeros(self.B, **i32)
        self.cu_new = torch.zeros(self.B + 1, **i32)
        self.hooks = torch.zeros(self.B, self.max_k + 1, 4, self.d, dtype=self.tdtype, device=self.dev)
        wb = self.lib.sf_workspace_bytes(self.ctx, self.B, self.max_k, self.cap)
        assert wb
        self.workspace = torch.zeros(wb + 256, dtype=torch.uint8, device=self.dev)
        off = (-self.workspace.data_ptr()) % 256
        self._ws_ptr = self.workspace.data_ptr() + off
        self.st = sfb.State(self.B, self.cap, _ptr(self.tk), _ptr(self.tv), _ptr(self.dk), _ptr(self.dv),
                            _ptr(self.kv_len), _ptr(self.pending), _ptr(self.hooks), _ptr(self.n_new),
                            _ptr(self.cu_new), C.c_void_p(self._ws_ptr), wb)
        self.len_upper = 0          # host-side upper bound of max_b kv_len[b]
        self._pinned = False
        self._keep = []

    def close(self):
        if self.ctx:
            self.lib.sf_destroy(self.ctx)
            self.ctx = C.c_void_p()

    # ---- weights -----------------------------------------------------------------------------
    def _up(self, a):
        if isinstance(a, torch.Tensor):
            t = a.to(device=self.dev, dtype=self.tdtype).contiguous()
        else:
            t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev).to(self.tdtype).contiguous()
        self._keep.append(t)
        return t

    def sf_pack_weight(self, w, glu=False, gain=None):
        """row-major device tensor [N,K] -> packed device buffer (kept alive by the engine); gain: the
        device gain vector [K] of the RMSNorm in front of the layer, folded into the columns (bf16)."""
        N, K = w.shape
        nb = self.lib.sf_packed_weight_bytes(self.ctx, N, K)
        es = 2 if self.dtype_id == sfb.SF_BF16 else 4
        out = torch.empty(nb // es, dtype=self.tdtype, device=self.dev)
        sfb.check(self.lib.sf_pack_weight(self.ctx, _ptr(w), _ptr(out), N, K, int(glu), _ptr(gain), _stream()),
                  "sf_pack_weight")
        self._keep.append(out)
        return out

    def _lin(self, a, glu=False, gain=None):
        """upload + pack one linear weight (with the gains of its norm, if any); the row-major copy is dropped."""
        t = self._up(a)
        self._keep.pop()
        p = self.sf_pack_weight(t, glu, gain)
        torch.cuda.current_stream().synchronize()
        return p

    def bind(self, tw, dw=None):
        """tw / dw: dicts of arrays (numpy float32 or torch) named as in the C structs; a dict that
        has separate w_gate / w_up gets them stacked into w_gate_up = [gate; up]."""
        self._keep = []
        L = self.L

        # norm gains go up first: a layer that consumes a norm's output is packed with that norm's gain
        # vector folded into its columns (bf16; the fp32 pack ignores it)
        def gate_up(w, gain, l=None):
            if "w_gate_up" in w:
                return self._lin(w["w_gate_up"] if l is None else w["w_gate_up"][l], glu=True, gain=gain)
            g, u = (w["w_gate"], w["w_up"]) if l is None else (w["w_gate"][l], w["w_up"][l])
            g, u = (torch.as_tensor(np.asarray(g)) if not isinstance(g, torch.Tensor) else g,
                    torch.as_tensor(np.asarray(u)) if not isinstance(u, torch.Tensor) else u)
            return self._lin(torch.cat([g, u], 0), glu=True, gain=gain)
        T = sfb.TargetWeights()
        self.w = {}
        for n in ("embed", "lm_head", "final_norm"):
            self.w[n] = self._lin(tw[n]) if n == "lm_head" else self._up(tw[n])
            setattr(T, n, self.w[n].data_ptr())
        for n in ("attn_norm", "ffn_norm"):
            self.w[n] = [self._up(tw[n][l]) for l in range(L)]
        self.w["wqkv"] = [self._lin(tw["wqkv"][l], gain=self.w["attn_norm"][l]) for l in range(L)]
        for n in ("wo", "w_down"):
            self.w[n] = [self._lin(tw[n][l]) for l in range(L)]
        self.w["w_gate_up"] = [gate_up(tw, self.w["ffn_norm"][l], l) for l in range(L)]
        for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down"):
            arr = (C.c_void_p * L)(*[t.data_ptr() for t in self.w[n]])
            self._keep.append(arr)
            setattr(T, n, arr)
        D = None
        if dw is not None:
            D = sfb.DraftWeights()
            self.wd = {}
            folded = {"wqkv": "attn_norm", "w_gate_up": "ffn_norm", "sa_wqkv": "sa_norm"}
            names = [n for n, _ in sfb.DraftWeights._fields_]
            for n in [x for x in names if x not in folded] + [x for x in names if x in folded]:
                if n.startswith("sa_") and n not in dw:        # two-stage wiring not used: NULL
                    continue
                if n == "w_gate_up":
                    self.wd[n] = gate_up(dw, self.wd[folded[n]])
                elif n in folded:
                    self.wd[n] = self._lin(dw[n], gain=self.wd[folded[n]])
                elif n in ("w_ds", "w_pos", "wo", "w_down", "sa_wo"):
                    self.wd[n] = self._lin(dw[n])
                else:
                    self.wd[n] = self._up(dw[n])
                setattr(D, n, self.wd[n].data_ptr())
        self._T, self._D = T, D
        sfb.check(self.lib.sf_bind(self.ctx, C.byref(T), C.byref(D) if D is not None else None), "sf_bind")

    def bind_shared(self, other, with_draft=False):
        """Bind the weights that another engine has already uploaded and packed (no copy): the target's
        only (a plain-decoding engine next to a speculative one), or the draft block's too."""
        self.w, self._T, self._D = other.w, other._T, (other._D if with_draft else None)
        self._keep = other._keep
        sfb.check(self.lib.sf_bind(self.ctx, C.byref(self._T), C.byref(self._D) if self._D is not None else None),
                  "sf_bind")

    # ---- the three steps ---------------------------------------------------------------------
    def sf_draft_step(self, k, mask=sfb.SF_MASK_BIDIR, draft_out=None, logits_out=None):
        out = draft_out if draft_out is not None else torch.empty(self.B, max(k, 0), dtype=torch.int32, device=self.dev)
        sfb.check(self.lib.sf_draft_step(self.ctx, C.byref(self.st), k, mask, self.len_upper, _ptr(out),
                                         _ptr(logits_out), _stream()), "sf_draft_step", self.ctx)
        return out

    def sf_verify_step(self, k, draft, logits_out=None, ids_out=None, logits=True):
        """-> (logits [B,k+1,V] float32 or None, target_ids [B,k+1] int32).  logits=False asks for the
        target's choices only: the logits are then not stored at all (bf16 mode)."""
        lg = logits_out
        if lg is None and logits:
            lg = torch.empty(self.B, k + 1, self.V, dtype=torch.float32, device=self.dev)
        ids = ids_out if ids_out is not None else torch.empty(self.B, k + 1, dtype=torch.int32, device=self.dev)
        sfb.check(self.lib.sf_verify_step(self.ctx, C.byref(self.st), k, _ptr(draft) if k > 0 else None,
                                          self.len_upper, _ptr(lg), _ptr(ids), _stream()), "sf_verify_step", self.ctx)
        return lg, ids

    def sf_accept_commit(self, k, draft, target_ids, force_len=None, accept_out=None, tokens_out=None):
        acc = accept_out if accept_out is not None else torch.empty(self.B, dtype=torch.int32, device=self.dev)
        out = tokens_out if tokens_out is not None else \
            torch.empty(self.B, k + 1, dtype=torch.int32, device=self.dev)
        sfb.check(self.lib.sf_accept_commit(self.ctx, C.byref(self.st), k, _ptr(draft) if k > 0 else None,
                                            _ptr(target_ids), _ptr(force_len), _ptr(acc), _ptr(out), _stream()),
                  "sf_accept_commit", self.ctx)
        if not self._pinned:
            self.len_upper = min(self.len_upper + k + 1, self.cap)
        return acc, out

    def sf_check_state(self):
        """-> SF_DEVERR_* bits the device collected since the last check (0 = none); waits for the stream."""
        flags = C.c_int32(0)
        st = self.lib.sf_check_state(self.ctx, C.byref(self.st), C.byref(flags), _stream())
        if st not in (sfb.SF_OK, sfb.SF_ECAPACITY):
            sfb.check(st, "sf_check_state", self.ctx)
        return flags.value

    def sf_op_accept(self, k, draft, target_ids, force_len=None):
        """The acceptance rule alone on this engine's state arrays (no call-order check)."""
        acc = torch.empty(self.B, dtype=torch.int32, device=self.dev)
        out = torch.empty(self.B, k + 1, dtype=torch.int32, device=self.dev)
        sfb.check(self.lib.sf_op_accept(self.ctx, self.B, k, _ptr(draft) if k > 0 else None, _ptr(target_ids),
                                        _ptr(force_len), _ptr(acc), _ptr(out), _ptr(self.kv_len), _ptr(self.pending),
                                        _ptr(self.n_new), _ptr(self.cu_new), _stream()), "sf_op_accept", self.ctx)
        return acc, out

    def sf_tune_linear(self, tile=0, split_k=0):
        sfb.check(self.lib.sf_tune_linear(self.ctx, tile, split_k), "sf_tune_linear")

    def sf_tune_attention(self, chunk_tiles=0):
        sfb.check(self.lib.sf_tune_attention(self.ctx, chunk_tiles), "sf_tune_attention")

    def sf_profile_begin(self):
        sfb.check(self.lib.sf_profile_begin(self.ctx), "sf_profile_begin")

    def sf_profile_end(self):
        """-> {class name: (total ms, launches)}; waits for the profiled work."""
        n = len(sfb.KERNEL_CLASSES)
        ms, cnt = (C.c_double * n)(), (C.c_int32 * n)()
        sfb.check(self.lib.sf_profile_end(self.ctx, ms, cnt, n), "sf_profile_end")
        return {name: (ms[i], cnt[i]) for i, name in enumerate(sfb.KERNEL_CLASSES)}

    def pin_len_upper(self, pinned=True):
        """Pin the host-side length bound to its maximum, so that every launch grid is the same
        from step to step (what a captured HIP graph needs); unpin to track the lengths again."""
        self._pinned = pinned
        if pinned:
            self.len_upper = self.cap - (self.max_k + 1)

    # ---- state helpers (plumbing) ------------------------------------------------------------
    def set_state(self, kv_len=None, pending=None, n_new=None):
        if kv_len is not None:
            self.kv_len.copy_(torch.as_tensor(np.asarray(kv_len, dtype=np.int32)))
            self.len_upper = int(np.max(kv_len))
        if pending is not None:
            self.pending.copy_(torch.as_tensor(np.asarray(pending, dtype=np.int32)))
        if n_new is not None:
            self.n_new.copy_(torch.as_tensor(np.asarray(n_new, dtype=np.int32)))

    def layer_cache(self, which, layer=0):
        """Flat view of one layer's slab of 'tk' | 'tv' | 'dk' | 'dv'."""
        buf = getattr(self, which)
        return buf[layer * self.layer_elems:(layer + 1) * self.layer_elems]

    def sf_kv_import(self, plain, which, layer=0):
        """plain: array [B,Hkv,cap,hd] -> tiled slab of cache `which` ('tk','tv','dk','dv')."""
        t = self._as_dev(plain).reshape(self.B, self.Hkv, self.cap, self.hd).contiguous()
        sfb.check(self.lib.sf_kv_import(self.ctx, _ptr(t), _ptr(self.layer_cache(which, layer)),
                                        int(which[1] == "v"), self.B, self.cap, _stream()), "sf_kv_import")
        torch.cuda.current_stream().synchronize()

    def sf_kv_export(self, which, layer=0):
        out = torch.empty(self.B, self.Hkv, self.cap, self.hd, dtype=self.tdtype, device=self.dev)
        sfb.check(self.lib.sf_kv_export(self.ctx, _ptr(self.layer_cache(which, layer)), _ptr(out),
                                        int(which[1] == "v"), self.B, self.cap, _stream()), "sf_kv_export")
        return out

    def _as_dev(self, a):
        if isinstance(a, torch.Tensor):
            return a.to(device=self.dev, dtype=self.tdtype)
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev).to(self.tdtype)

    # ---- single operations -------------------------------------------------------------------
    def sf_op_attention(self, q, kc, vc, kv_len, n_q, mask, len_upper=None):
        """q [B,n_q,Hq,hd] device tensor; kc/vc tiled slabs; kv_len int32 device [B]."""
        B = q.shape[0]
        slab = self.Hkv * self.cap * self.hd
        if (tuple(q.shape) != (B, n_q, self.Hq, self.hd) or kv_len.numel() != B or kv_len.dtype != torch.int32
                or kc.numel() < B * slab or vc.numel() < B * slab):
            raise ValueError("sf_op_attention: q must be [B,n_q,Hq,hd], kv_len int32 [B], caches at least B slabs")
        if len_upper is None:
            len_upper = int(kv_len.max().item())
        need = self.lib.sf_attention_workspace_bytes(self.ctx, B, n_q, len_upper)
        ws = torch.empty(need + 256, dtype=torch.uint8, device=self.dev)
        p = ws.data_ptr() + (-ws.data_ptr()) % 256
        out = torch.empty_like(q)
        sfb.check(self.lib.sf_op_attention(self.ctx, _ptr(q), _ptr(kc), _ptr(vc), _ptr(kv_len), B, n_q, self.cap,
                                           mask, len_upper, _ptr(out), C.c_void_p(p), need, _stream()),
                  "sf_op_attention", self.ctx)
        self._keep_ws = ws
        return out

    def linear_workspace(self, M):
        """(pointer, bytes) of a zero-filled split-K workspace, cached per engine."""
        nb = self.lib.sf_linear_workspace_bytes(self.ctx, M)
        if nb == 0:
            return None, 0
        if getattr(self, "_lin_ws", None) is None or self._lin_ws.numel() < nb + 256:
            self._lin_ws = torch.zeros(nb + 256, dtype=torch.uint8, device=self.dev)
        p = self._lin_ws.data_ptr() + (-self._lin_ws.data_ptr()) % 256
        return C.c_void_p(p), nb

    def sf_op_linear(self, x, w, bias=None, residual=None, out_f32=False, y=None, packed=None):
        """w: row-major [N,K] device tensor (packed here) unless `packed` = (buffer, N) is given."""
        M, K = x.shape
        if packed is None:
            N = w.shape[0]
            w = self.sf_pack_weight(w)
            self._keep.pop()
        else:
            w, N = packed
        if y is None:
            y = torch.empty(M, N, dtype=torch.float32 if out_f32 else self.tdtype, device=self.dev)
        wsp, nb = self.linear_workspace(M)
        sfb.check(self.lib.sf_op_linear(self.ctx, _ptr(x), _ptr(w), _ptr(bias), _ptr(residual), _ptr(y), M, N, K,
                                        int(out_f32), wsp, nb, _stream()), "sf_op_linear", self.ctx)
        return y

    def sf_op_rmsnorm_linear(self, x, gain, w, out_f32=False, packed=None):
        """RMSNorm(x; gain) . w^T in one kernel (bf16).  w: row-major [N,K] device tensor, packed here with
        the gains folded in, unless `packed` = (buffer packed that way, N) is given."""
        M, K = x.shape
        if packed is None:
            N = w.shape[0]
            w = self.sf_pack_weight(w, gain=gain)
            self._keep.pop()
        else:
            w, N = packed
        y = torch.empty(M, N, dtype=torch.float32 if out_f32 else self.tdtype, device=self.dev)
        wsp, nb = self.linear_workspace(M)
        sfb.check(self.lib.sf_op_rmsnorm_linear(self.ctx, _ptr(x), _ptr(w), _ptr(y), M, N, K, int(out_f32), wsp, nb,
                                                _stream()), "sf_op_rmsnorm_linear", self.ctx)
        return y

    def sf_op_linear_swiglu(self, x, w_gate_up):
        """x [M,K]; w_gate_up row-major [2F,K] device tensor (packed here) -> act [M,F]."""
        M, K = x.shape
        F = w_gate_up.shape[0] // 2
        pk = self.sf_pack_weight(w_gate_up, glu=True)
        self._keep.pop()
        act = torch.empty(M, F, dtype=self.tdtype, device=self.dev)
        if self.dtype_id == sfb.SF_BF16:
            wsp, nb = self.linear_workspace(M)
        else:
            nb = M * 2 * F * 4 + 256
            self._gu_ws = torch.empty(nb + 256, dtype=torch.uint8, device=self.dev)
            wsp = C.c_void_p(self._gu_ws.data_ptr() + (-self._gu_ws.data_ptr()) % 256)
        sfb.check(self.lib.sf_op_linear_swiglu(self.ctx, _ptr(x), _ptr(pk), _ptr(act), M, F, K, wsp, nb, _stream()),
                  "sf_op_linear_swiglu", self.ctx)
        self._pk_keep = pk
        return act

    def sf_op_linear_argmax(self, x, w=None, packed=None, want_logits=False):
        """ids [M] = argmax over the columns of x . w^T, as the LM head runs (+ the logits when asked for)."""
        M, K = x.shape
        if packed is None:
            N = w.shape[0]
            w = self.sf_pack_weight(w)
            self._keep.pop()
        else:
            w, N = packed
        nb = self.lib.sf_linear_argmax_workspace_bytes(self.ctx, M, N)
        ws = torch.zeros(nb + 256, dtype=torch.uint8, device=self.dev)
        p = ws.data_ptr() + (-ws.data_ptr()) % 256
        ids = torch.empty(M, dtype=torch.int32, device=self.dev)
        lg = torch.empty(M, N, dtype=torch.float32, device=self.dev) if want_logits else None
        sfb.check(self.lib.sf_op_linear_argmax(self.ctx, _ptr(x), _ptr(w), M, N, K, _ptr(ids), _ptr(lg),
                                               C.c_void_p(p), nb, _stream()), "sf_op_linear_argmax", self.ctx)
        self._keep_ws = (ws, w)
        return (ids, lg) if want_logits else ids

    def sf_op_rmsnorm(self, x, gain, n_gain=1):
        M, d = x.shape
        y = torch.empty_like(x)
        sfb.check(self.lib.sf_op_rmsnorm(self.ctx, _ptr(x), _ptr(gain), _ptr(y), M, d, n_gain, _stream()),
                  "sf_op_rmsnorm")
        return y

    def sf_op_rope_kv_append(self, qkv, kv_len, n_q, kc, vc):
        B = kv_len.shape[0]
        q_out = torch.empty(B * n_q, self.Hq * self.hd, dtype=self.tdtype, device=self.dev)
        nb = B * n_q * (self.hd // 2) * 8
        ws = torch.empty(nb, dtype=torch.uint8, device=self.dev)
        sfb.check(self.lib.sf_op_rope_kv_append(self.ctx, _ptr(qkv), _ptr(kv_len), B, n_q, self.cap, _ptr(q_out),
                                                _ptr(kc), _ptr(vc), _ptr(ws), nb, _stream()),
                  "sf_op_rope_kv_append")
        self._keep_ws = ws
        return q_out

    def sf_op_rope_attention(self, qkv, kv_len, n_q, kc, vc, mask, len_upper=None):
        """Rotate + append + attend in one kernel (bf16).  qkv [B*n_q,(Hq+2Hkv)*hd]; returns [B,n_q,Hq,hd]."""
        B = kv_len.shape[0]
        slab = self.Hkv * self.cap * self.hd
        if (qkv.numel() != B * n_q * (self.Hq + 2 * self.Hkv) * self.hd or kv_len.dtype != torch.int32
                or kc.numel() < B * slab or vc.numel() < B * slab):
            raise ValueError("sf_op_rope_attention: qkv must be [B*n_q,(Hq+2Hkv)*hd], kv_len int32 [B], "
                             "caches at least B slabs")
        if len_upper is None:
            len_upper = int(kv_len.max().item())
        need = self.lib.sf_rope_attention_workspace_bytes(self.ctx, B, n_q, len_upper)
        ws = torch.empty(need + 256, dtype=torch.uint8, device=self.dev)
        p = ws.data_ptr() + (-ws.data_ptr()) % 256
        out = torch.empty(B, n_q, self.Hq, self.hd, dtype=self.tdtype, device=self.dev)
        sfb.check(self.lib.sf_op_rope_attention(self.ctx, _ptr(qkv), _ptr(kv_len), B, n_q, self.cap, mask, len_upper,
                                                _ptr(kc), _ptr(vc), _ptr(out), C.c_void_p(p), need, _stream()),
                  "sf_op_rope_attention", self.ctx)
        self._keep_ws = ws
        return out

    def sf_op_silu_mul(self, gu):
        M, F2 = gu.shape
        act = torch.empty(M, F2 // 2, dtype=self.tdtype, device=self.dev)
        sfb.check(self.lib.sf_op_silu_mul(self.ctx, _ptr(gu), _ptr(act), M, F2 // 2, _stream()), "sf_op_silu_mul")
        return act

    def sf_op_argmax(self, logits):
        M, V = logits.shape
        nb = self.lib.sf_argmax_workspace_bytes(M)
        ws = torch.empty(nb + 256, dtype=torch.uint8, device=self.dev)
        p = ws.data_ptr() + (-ws.data_ptr()) % 256
        ids = torch.empty(M, dtype=torch.int32, device=self.dev)
        sfb.check(self.lib.sf_op_argmax(self.ctx, _ptr(logits), M, V, _ptr(ids), C.c_void_p(p), nb, _stream()),
                  "sf_op_argmax")
        self._keep_ws = ws
        return ids

    def sf_op_argmax_noalloc(self, logits, ids):
        """ids (preallocated int32 [M]) = row arg-max of logits; nothing is allocated on the way."""
        M, V = logits.shape
        sfb.check(self.lib.sf_op_argmax_noalloc(self.ctx, _ptr(logits), M, V, _ptr(ids), _stream()),
                  "sf_op_argmax_noalloc", self.ctx)
        return ids

    # ---- prefill: chunked verify with forced acceptance --------------------------------------
    def prefill(self, prompts, block=None):
        """Feeds every prompt through sf_verify_step in blocks of `block` tokens (default max_k+1) with forced
        commits, right-aligned so that all sequences finish with the last block, and runs sf_draft_step after
        every block so the draft cache follows.  A block longer than max_k+1 runs on a helper engine created
        for that block length (same weights, same caches); its final lengths, pending tokens and newest hooked
        rows are then handed to this engine.  Returns the first emitted token of every sequence (device)."""
        q = self.max_k + 1 if block is None else int(block)
        if q <= self.max_k + 1:
            return _prefill_blocks(self, prompts, q, self.max_k)
        helper = Engine(self.cfg, self.B, self.cap, q - 1, device=self.dev, share_caches=self)
        helper.bind_shared(self, with_draft=self._D is not None)
        first = _prefill_blocks(helper, prompts, q, max(self.max_k, 1))
        # hand-over: committed lengths, pending tokens, and every sequence's newest committed row of hooks
        self.kv_len.copy_(helper.kv_len)
        self.pending.copy_(helper.pending)
        last = (helper.n_new.to(torch.int64) - 1).clamp_(min=0)
        rows = helper.hooks[torch.arange(self.B, device=self.dev), last]          # [B, 4, d]
        self.hooks.zero_()
        self.hooks[:, 0] = rows
        self.n_new.copy_((helper.n_new > 0).to(torch.int32))
        self.len_upper = helper.len_upper
        torch.cuda.current_stream().synchronize()
        helper.close()
        return first


def _prefill_blocks(eng, prompts, q, k_draft):
    """Chunked prefill on `eng` in blocks of q <= eng.max_k + 1 prompt tokens (see Engine.prefill)."""
    k = q - 1
    lens = np.array([len(p) for p in prompts], np.int64)
    nblk = (lens + q - 1) // q
    total = int(nblk.max())
    eng.set_state(kv_len=np.zeros(eng.B, np.int32), pending=np.zeros(eng.B, np.int32),
                  n_new=np.zeros(eng.B, np.int32))
    done = np.zeros(eng.B, np.int64)
    for step in range(total):
        toks = np.zeros((eng.B, q), np.int32)
        force = np.zeros(eng.B, np.int32)
        nxt = np.zeros(eng.B, np.int32)
        for b, p in enumerate(prompts):
            if step < total - nblk[b]:
                continue                      # this sequence starts later
            first = lens[b] - (nblk[b] - 1) * q if done[b] == 0 else q   # short block first
            seg = p[done[b]:done[b] + first]
            toks[b, :len(seg)] = seg
            force[b] = len(seg)
            done[b] += len(seg)
            nxt[b] = p[done[b]] if done[b] < lens[b] else -1
        eng.pending.copy_(torch.from_numpy(toks[:, 0].copy()))
        draft = torch.from_numpy(toks[:, 1:].copy()).to(eng.dev)
        fl = torch.from_numpy(force).to(eng.dev)
        _, ids = eng.sf_verify_step(k, draft, logits=False)
        eng.sf_accept_commit(k, draft, ids, force_len=fl)
        eng.len_upper = int(done.max())
        if step < total - 1:
            # pending of a finished block is the next prompt token, not the target's choice
            pend = eng.pending.cpu().numpy()
            pend[nxt >= 0] = nxt[nxt >= 0]
            eng.pending.copy_(torch.from_numpy(pend))
        if k_draft > 0 and eng._D is not None:
            eng.sf_draft_step(k_draft)
    return eng.pending.clone()
