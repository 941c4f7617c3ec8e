"""ctypes mirror of include/specformer.h and include/specformer_aux.h.  Argument marshalling only."""
import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
# SF_LIB in the environment names a library built elsewhere (the host-sanitizer run of the ABI tests)
LIB_PATH = os.environ.get("SF_LIB") or os.path.join(HERE, "libspecformer.so")

SF_OK, SF_EINVAL, SF_ECAPACITY, SF_ESTATE, SF_EHIP, SF_EUNSUPPORTED = range(6)
SF_BF16, SF_F32 = 0, 1
SF_MASK_CAUSAL, SF_MASK_BIDIR = 0, 1
SF_DRAFT_TWO_STAGE = 16   # OR-ed into sf_draft_step's mask
KERNEL_CLASSES = ["linear", "attention", "attention_combine", "rmsnorm", "rope_kv_append", "silu_mul",
                  "embed_hook", "argmax", "accept"]

EXPORTS = [
    "sf_create", "sf_destroy", "sf_workspace_bytes", "sf_kv_cache_bytes", "sf_bind", "sf_draft_step",
    "sf_verify_step", "sf_accept_commit", "sf_check_state", "sf_kv_import", "sf_kv_export", "sf_attention_workspace_bytes",
    "sf_op_attention", "sf_packed_weight_bytes", "sf_pack_weight", "sf_linear_workspace_bytes", "sf_op_linear",
    "sf_op_rmsnorm_linear", "sf_op_linear_swiglu", "sf_linear_argmax_workspace_bytes", "sf_op_linear_argmax",
    "sf_op_rmsnorm", "sf_op_rope_kv_append", "sf_rope_attention_workspace_bytes", "sf_op_rope_attention",
    "sf_op_silu_mul", "sf_argmax_workspace_bytes", "sf_op_argmax", "sf_op_argmax_noalloc", "sf_op_accept", "sf_strerror",
    "sf_last_hip_error", "sf_version",
    # include/specformer_aux.h
    "sf_tune_linear", "sf_linear_num_tiles", "sf_linear_config", "sf_tune_attention", "sf_calib_copy",
    "sf_profile_begin", "sf_profile_end",
]

vp, i32, sz = C.c_void_p, C.c_int32, C.c_size_t


class ModelCfg(C.Structure):
    _fields_ = [(n, i32) for n in ("n_layers", "d_model", "n_q_heads", "n_kv_heads", "head_dim", "d_ffn", "vocab")] \
        + [("rope_theta", C.c_float), ("rms_eps", C.c_float), ("dtype", i32)]


class TargetWeights(C.Structure):
    _fields_ = [("embed", vp), ("lm_head", vp), ("final_norm", vp)] + \
        [(n, C.POINTER(vp)) for n in ("attn_norm", "wqkv", "wo", "ffn_norm", "w_gate_up", "w_down")]


class DraftWeights(C.Structure):
    _fields_ = [(n, vp) for n in ("group_norm", "w_ds", "pos_norm", "w_pos", "b_pos", "attn_norm", "wqkv", "wo",
                                  "ffn_norm", "w_gate_up", "w_down", "out_norm", "sa_norm", "sa_wqkv", "sa_wo")]


class State(C.Structure):
    _fields_ = [("B", i32), ("cap", i32), ("tk", vp), ("tv", vp), ("dk", vp), ("dv", vp), ("kv_len", vp),
                ("pending", vp), ("hooks", vp), ("n_new", vp), ("cu_new", vp), ("workspace", vp),
                ("workspace_bytes", sz)]


class SfError(RuntimeError):
    def __init__(self, status, what, hip_err=0):
        self.status, self.hip_err = status, hip_err
        extra = f", hipError_t {hip_err}" if hip_err else ""
        super().__init__(f"{what}: {lib().sf_strerror(status).decode()} (status {status}{extra})")


_lib = None


def lib():
    """Load the HIP library; there is no fallback path."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_20340_amd.build` "
                           "(or __graft_entry__.build()); there is no CPU fallback")
    # PyTorch owns the device memory this library works on, and it bundles its own HIP runtime:
    # load it first so that both sides share ONE libamdhip64 (two runtimes in a process do not
    # see each other's allocations or streams).
    import torch  # noqa: F401
    L = C.CDLL(LIB_PATH)
    P = C.POINTER
    L.sf_create.argtypes = [P(ModelCfg), P(ModelCfg), i32, i32, P(vp)]
    L.sf_destroy.argtypes = [vp]
    L.sf_workspace_bytes.argtypes = [vp, i32, i32, i32]
    L.sf_workspace_bytes.restype = sz
    L.sf_kv_cache_bytes.argtypes = [vp, i32, i32, i32]
    L.sf_kv_cache_bytes.restype = sz
    L.sf_bind.argtypes = [vp, P(TargetWeights), P(DraftWeights)]
    L.sf_draft_step.argtypes = [vp, P(State), i32, i32, i32, vp, vp, vp]
    L.sf_verify_step.argtypes = [vp, P(State), i32, vp, i32, vp, vp, vp]
    L.sf_accept_commit.argtypes = [vp, P(State), i32, vp, vp, vp, vp, vp, vp]
    L.sf_check_state.argtypes = [vp, P(State), P(i32), vp]
    L.sf_op_accept.argtypes = [vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
    L.sf_linear_argmax_workspace_bytes.argtypes = [vp, i32, i32]
    L.sf_linear_argmax_workspace_bytes.restype = sz
    L.sf_op_linear_argmax.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, sz, vp]
    L.sf_kv_import.argtypes = [vp, vp, vp, i32, i32, i32, vp]
    L.sf_kv_export.argtypes = [vp, vp, vp, i32, i32, i32, vp]
    L.sf_attention_workspace_bytes.argtypes = [vp, i32, i32, i32]
    L.sf_attention_workspace_bytes.restype = sz
    L.sf_op_attention.argtypes = [vp, vp, vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    L.sf_op_linear.argtypes = [vp, vp, vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    L.sf_op_rmsnorm_linear.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, sz, vp]
    L.sf_packed_weight_bytes.argtypes = [vp, i32, i32]
    L.sf_packed_weight_bytes.restype = sz
    L.sf_pack_weight.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp]
    L.sf_op_linear_swiglu.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp, sz, vp]
    L.sf_linear_workspace_bytes.argtypes = [vp, i32]
    L.sf_linear_workspace_bytes.restype = sz
    L.sf_tune_linear.argtypes = [vp, i32, i32]
    L.sf_linear_num_tiles.argtypes = []
    L.sf_linear_num_tiles.restype = i32
    L.sf_linear_config.argtypes = [i32, i32, i32, i32, C.c_size_t, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32)]
    L.sf_tune_attention.argtypes = [vp, i32]
    L.sf_op_rmsnorm.argtypes = [vp, vp, vp, vp, i32, i32, i32, vp]
    L.sf_op_rope_kv_append.argtypes = [vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.sf_rope_attention_workspace_bytes.argtypes = [vp, i32, i32, i32]
    L.sf_rope_attention_workspace_bytes.restype = sz
    L.sf_op_rope_attention.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.sf_op_silu_mul.argtypes = [vp, vp, vp, i32, i32, vp]
    L.sf_argmax_workspace_bytes.argtypes = [i32]
    L.sf_argmax_workspace_bytes.restype = sz
    L.sf_op_argmax.argtypes = [vp, vp, i32, i32, vp, vp, sz, vp]
    L.sf_op_argmax_noalloc.argtypes = [vp, vp, i32, i32, vp, vp]
    L.sf_calib_copy.argtypes = [vp, vp, sz, vp]
    L.sf_profile_begin.argtypes = [vp]
    L.sf_profile_end.argtypes = [vp, P(C.c_double), P(i32), i32]
    L.sf_strerror.argtypes = [i32]
    L.sf_strerror.restype = C.c_char_p
    L.sf_last_hip_error.argtypes = [vp]
    L.sf_version.restype = C.c_char_p
    for name in EXPORTS:
        f = getattr(L, name)
        if f.restype is C.c_int:  # status-returning entry points
            f.restype = i32
    _lib = L
    return L


def check(status, what, ctx=None):
    if status != SF_OK:
        raise SfError(status, what, lib().sf_last_hip_error(ctx) if ctx is not None and status == SF_EHIP else 0)
