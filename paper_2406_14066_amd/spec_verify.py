"""Thin ctypes binding of ``libspec_verify.so`` (the C ABI in ``include/spec_verify.h``).

Argument marshalling only: tensors are passed as raw device pointers, the
stream as the raw ``hipStream_t`` of torch's current stream; every step of the
path runs in the library's kernels.  There is no CPU fallback: if the library
has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspec_verify.so")

K_MAX = 8
BLOCK_SIZE = 16
NUM_COUNTERS = 8

SPEC_OK, SPEC_EINVAL, SPEC_EUNSUPPORTED, SPEC_EWORKSPACE, SPEC_EHIP = 0, -1, -2, -3, -4
SPEC_F32, SPEC_BF16 = 0, 1
KV_TOKEN_MAJOR, KV_MFMA = 0, 1
ACCEPT_SAMPLE, ACCEPT_GREEDY, ACCEPT_POINT_DRAFT = 0, 1, 2   # spec_accept_mode

COUNTER_NAMES = ("proposed", "accepted", "attempted", "emitted", "near_tie", "requests", "input_errors", "abandoned")


class AttnArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32),
        ("block_size", C.c_int32), ("num_blocks", C.c_int32), ("max_blocks_per_req", C.c_int32),
        ("T", C.c_int32), ("qkv_dtype", C.c_int32), ("kv_layout", C.c_int32),
        ("q", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
        ("block_table", C.c_void_p), ("kv_len", C.c_void_p), ("cu_q_len", C.c_void_p),
        ("softmax_scale", C.c_float),
        ("out", C.c_void_p),
        ("host_kv_len", C.c_void_p), ("host_cu_q_len", C.c_void_p),
        ("max_kv_len", C.c_int32), ("validate", C.c_int32),
        ("host_block_table", C.c_void_p), ("error_count", C.c_void_p),
    ]


class RejectArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("V", C.c_int32), ("T", C.c_int32),
        ("target_logits", C.c_void_p), ("draft_logits", C.c_void_p),
        ("draft_tokens", C.c_void_p), ("cu_q_len", C.c_void_p), ("host_cu_q_len", C.c_void_p),
        ("philox_seed", C.c_uint64), ("philox_step", C.c_uint64),
        ("accepted_len", C.c_void_p), ("next_token", C.c_void_p), ("out_tokens", C.c_void_p),
        ("counters", C.c_void_p), ("debug_u_ratio", C.c_void_p),
        ("accept_mode", C.c_int32),
        ("kv_len", C.c_void_p), ("new_kv_len", C.c_void_p), ("draft_next_len", C.c_void_p),
        ("philox_step_device", C.c_void_p), ("validate", C.c_int32), ("host_draft_tokens", C.c_void_p),
    ]


class KvAppendArgs(C.Structure):
    _fields_ = [
        ("B", C.c_int32), ("Hkv", C.c_int32), ("d", C.c_int32), ("num_blocks", C.c_int32),
        ("max_blocks_per_req", C.c_int32), ("T", C.c_int32), ("dtype", C.c_int32), ("kv_layout", C.c_int32),
        ("new_k", C.c_void_p), ("new_v", C.c_void_p), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
        ("block_table", C.c_void_p), ("kv_len", C.c_void_p), ("cu_q_len", C.c_void_p),
        ("host_kv_len", C.c_void_p), ("host_cu_q_len", C.c_void_p),
        ("error_count", C.c_void_p),
    ]


class PlanInfo(C.Structure):
    _fields_ = [
        ("attn_path", C.c_int32), ("row_tiles", C.c_int32), ("row_groups", C.c_int32),
        ("chunk_tokens", C.c_int32), ("max_chunks", C.c_int32), ("launches", C.c_int32),
        ("early_stop", C.c_int32), ("stat_segments", C.c_int32), ("race_segments", C.c_int32),
        ("attn_blocks", C.c_int32), ("reject_blocks", C.c_int32), ("reserved", C.c_int32),
        ("workspace_bytes", C.c_uint64),
    ]

    def as_dict(self):
        return {f: getattr(self, f) for f, _ in self._fields_ if f != "reserved"}


PATH_NONE, PATH_MFMA, PATH_GENERIC = 0, 1, 2


EXPORTS = (
    "spec_verify_workspace_bytes", "spec_verify_attn", "spec_reject_sample", "spec_verify_step",
    "spec_verify_step_static", "spec_verify_plan", "spec_verify_reload_env",
    "spec_validate_attn", "spec_validate_reject", "spec_kv_repack_mfma", "spec_kv_append", "spec_status_string",
    "spec_verify_version", "spec_profile_begin", "spec_profile_end",
    "spec_expected_generated_len", "spec_predict_latency", "spec_fit_latency",
    "spec_acceptance_update", "spec_acceptance_rate", "spec_argmax_goodput",
)
NUM_KERNELS = 5
KERNEL_NAMES = ("step", "attn", "attn_generic", "attn_combine", "reject")

_lib = None


class SpecVerifyError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (where, status_string(status), status))


def lib():
    """Loads the HIP library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libspec_verify.so is missing: build it first (python -c 'import __graft_entry__ as g; g.build()'). "
                "There is no fallback path.")
        L = C.CDLL(LIB_PATH)
        L.spec_verify_workspace_bytes.argtypes = [C.POINTER(AttnArgs), C.POINTER(RejectArgs)]
        L.spec_verify_workspace_bytes.restype = C.c_size_t
        L.spec_verify_attn.argtypes = [C.POINTER(AttnArgs), C.c_void_p, C.c_size_t, C.c_void_p]
        L.spec_verify_attn.restype = C.c_int
        L.spec_reject_sample.argtypes = [C.POINTER(RejectArgs), C.c_void_p, C.c_size_t, C.c_void_p]
        L.spec_reject_sample.restype = C.c_int
        L.spec_verify_step.argtypes = [C.POINTER(AttnArgs), C.POINTER(RejectArgs), C.c_void_p, C.c_size_t, C.c_void_p]
        L.spec_verify_step.restype = C.c_int
        L.spec_verify_step_static.argtypes = [C.POINTER(AttnArgs), C.POINTER(RejectArgs), C.c_void_p]
        L.spec_verify_step_static.restype = C.c_int
        L.spec_verify_plan.argtypes = [C.POINTER(AttnArgs), C.POINTER(RejectArgs), C.POINTER(PlanInfo)]
        L.spec_verify_plan.restype = C.c_int
        L.spec_verify_reload_env.argtypes = []
        L.spec_verify_reload_env.restype = None
        L.spec_validate_attn.argtypes = [C.POINTER(AttnArgs)]
        L.spec_validate_attn.restype = C.c_int
        L.spec_validate_reject.argtypes = [C.POINTER(RejectArgs)]
        L.spec_validate_reject.restype = C.c_int
        L.spec_kv_repack_mfma.argtypes = [C.c_void_p] * 4 + [C.c_int32] * 3 + [C.c_void_p]
        L.spec_kv_repack_mfma.restype = C.c_int
        L.spec_status_string.argtypes = [C.c_int]
        L.spec_status_string.restype = C.c_char_p
        L.spec_profile_begin.argtypes = [C.c_int32]
        L.spec_profile_begin.restype = C.c_int
        L.spec_profile_end.argtypes = [C.c_void_p, C.c_void_p]
        L.spec_profile_end.restype = C.c_int
        L.spec_verify_version.argtypes = []
        L.spec_verify_version.restype = C.c_int32
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().spec_status_string(int(status)).decode()


def _check(status: int, where: str):
    if status != SPEC_OK:
        raise SpecVerifyError(status, where)


def _dev_ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _host_i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a), dtype=np.int32)


def _stream_handle(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def make_attn_args(q, k_cache, v_cache, block_table, kv_len, cu_q_len, out, host_kv_len, host_cu_q_len,
                   *, Hkv: int, kv_layout: int = KV_TOKEN_MAJOR, softmax_scale: float = 0.0,
                   block_size: int = BLOCK_SIZE, max_kv_len: int = 0, validate: int = 0, host_block_table=None,
                   error_count=None):
    """Builds the argument struct from device tensors (torch) and host arrays (numpy).
    Returns (struct, keepalive) -- keep `keepalive` referenced while the struct is in use."""
    import torch
    T, Hq, d = q.shape
    if q.dtype == torch.float32:
        dtype = SPEC_F32
    elif q.dtype == torch.bfloat16:
        dtype = SPEC_BF16
    else:
        raise TypeError("q must be float32 or bfloat16")
    hk = _host_i32(host_kv_len) if host_kv_len is not None else None
    hc = _host_i32(host_cu_q_len)
    hb = _host_i32(host_block_table) if host_block_table is not None else None
    a = AttnArgs()
    a.B = hc.shape[0] - 1
    a.Hq, a.Hkv, a.d = Hq, Hkv, d
    a.block_size = block_size
    a.num_blocks = k_cache.shape[0]
    a.max_blocks_per_req = block_table.shape[1]
    a.T = T
    a.qkv_dtype = dtype
    a.kv_layout = kv_layout
    a.q, a.k_cache, a.v_cache = q.data_ptr(), k_cache.data_ptr(), v_cache.data_ptr()
    a.block_table, a.kv_len, a.cu_q_len = block_table.data_ptr(), kv_len.data_ptr(), cu_q_len.data_ptr()
    a.softmax_scale = softmax_scale
    a.out = out.data_ptr()
    a.host_kv_len = hk.ctypes.data if hk is not None else None
    a.host_cu_q_len = hc.ctypes.data
    a.max_kv_len = max_kv_len
    a.validate = validate
    a.host_block_table = hb.ctypes.data if hb is not None else None
    a.error_count = _dev_ptr(error_count)
    return a, (hk, hc, hb, q, k_cache, v_cache, block_table, kv_len, cu_q_len, out, error_count)


def make_reject_args(target_logits, draft_logits, draft_tokens, cu_q_len, host_cu_q_len, accepted_len, next_token,
                     counters, *, philox_seed: int, philox_step: int, out_tokens=None, debug_u_ratio=None,
                     accept_mode: int = 0, kv_len=None, new_kv_len=None, draft_next_len=None,
                     philox_step_device=None, validate: int = 0, host_draft_tokens=None):
    hc = _host_i32(host_cu_q_len)
    hd = _host_i32(host_draft_tokens) if host_draft_tokens is not None else None
    r = RejectArgs()
    r.B = hc.shape[0] - 1
    r.T, r.V = target_logits.shape
    r.target_logits = target_logits.data_ptr()
    r.draft_logits = _dev_ptr(draft_logits) if (r.T > r.B and accept_mode == ACCEPT_SAMPLE) else None
    r.draft_tokens = _dev_ptr(draft_tokens) if r.T > r.B else None
    r.cu_q_len = cu_q_len.data_ptr()
    r.host_cu_q_len = hc.ctypes.data
    r.philox_seed = philox_seed
    r.philox_step = philox_step
    r.accepted_len = accepted_len.data_ptr()
    r.next_token = next_token.data_ptr()
    r.out_tokens = _dev_ptr(out_tokens)
    r.counters = counters.data_ptr()
    r.debug_u_ratio = _dev_ptr(debug_u_ratio)
    r.accept_mode = accept_mode
    r.kv_len = _dev_ptr(kv_len)
    r.new_kv_len = _dev_ptr(new_kv_len)
    r.draft_next_len = _dev_ptr(draft_next_len)
    r.philox_step_device = _dev_ptr(philox_step_device)
    r.validate = validate
    r.host_draft_tokens = hd.ctypes.data if hd is not None else None
    return r, (hc, hd, philox_step_device, target_logits, draft_logits, draft_tokens, cu_q_len, accepted_len, next_token, counters,
               out_tokens, debug_u_ratio, kv_len, new_kv_len, draft_next_len)


def spec_verify_workspace_bytes(attn: Optional[AttnArgs], reject: Optional[RejectArgs]) -> int:
    n = lib().spec_verify_workspace_bytes(C.byref(attn) if attn is not None else None,
                                          C.byref(reject) if reject is not None else None)
    if n == 0:
        raise SpecVerifyError(SPEC_EINVAL, "spec_verify_workspace_bytes")
    return int(n)


def spec_verify_plan(attn: Optional[AttnArgs], reject: Optional[RejectArgs]) -> dict:
    """How the library would run this step: which attention kernel, the split, the launches."""
    info = PlanInfo()
    _check(lib().spec_verify_plan(C.byref(attn) if attn is not None else None,
                                  C.byref(reject) if reject is not None else None, C.byref(info)), "spec_verify_plan")
    return info.as_dict()


def reload_env() -> None:
    """Re-reads the SPEC_VERIFY_* tuning switches (the library reads them once, at its first call)."""
    lib().spec_verify_reload_env()


def spec_validate_attn(attn: AttnArgs) -> int:
    return int(lib().spec_validate_attn(C.byref(attn)))


def spec_validate_reject(reject: RejectArgs) -> int:
    return int(lib().spec_validate_reject(C.byref(reject)))


def spec_verify_attn(attn: AttnArgs, workspace, stream=None) -> None:
    _check(lib().spec_verify_attn(C.byref(attn), workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                  _stream_handle(stream)), "spec_verify_attn")


def spec_reject_sample(reject: RejectArgs, workspace, stream=None) -> None:
    _check(lib().spec_reject_sample(C.byref(reject), workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream_handle(stream)),
           "spec_reject_sample")


def spec_verify_step(attn: AttnArgs, reject: RejectArgs, workspace, stream=None) -> None:
    _check(lib().spec_verify_step(C.byref(attn), C.byref(reject), workspace.data_ptr(),
                                  workspace.numel() * workspace.element_size(), _stream_handle(stream)),
           "spec_verify_step")


STATIC_SCRATCH_BYTES = 16 << 20


def spec_verify_step_static(attn: AttnArgs, reject: RejectArgs, stream=None) -> None:
    """The step on the library's own per-GPU scratch array (no workspace argument, no allocation)."""
    _check(lib().spec_verify_step_static(C.byref(attn), C.byref(reject), _stream_handle(stream)),
           "spec_verify_step_static")


def spec_kv_repack_mfma(src_k, src_v, dst_k, dst_v, stream=None) -> None:
    nb, Hkv, bs, d = src_k.shape
    assert bs == BLOCK_SIZE and src_k.element_size() == 2
    _check(lib().spec_kv_repack_mfma(src_k.data_ptr(), src_v.data_ptr(), dst_k.data_ptr(), dst_v.data_ptr(),
                                     nb, Hkv, d, _stream_handle(stream)), "spec_kv_repack_mfma")


def make_kv_append_args(new_k, new_v, k_cache, v_cache, block_table, kv_len, cu_q_len, host_kv_len, host_cu_q_len, *,
                        kv_layout: int = KV_TOKEN_MAJOR, error_count=None):
    """The argument struct of `spec_kv_append` for tensors that stay where they are (a decode loop
    appends from the same buffers every step).  Returns (args, keepalive)."""
    hk, hc = _host_i32(host_kv_len), _host_i32(host_cu_q_len)
    a = KvAppendArgs()
    a.T, a.Hkv, a.d = new_k.shape
    a.B = hk.shape[0]
    a.num_blocks = k_cache.shape[0]
    a.max_blocks_per_req = block_table.shape[1]
    a.dtype = SPEC_F32 if new_k.element_size() == 4 else SPEC_BF16
    a.kv_layout = kv_layout
    a.new_k, a.new_v = new_k.data_ptr(), new_v.data_ptr()
    a.k_cache, a.v_cache = k_cache.data_ptr(), v_cache.data_ptr()
    a.block_table, a.kv_len, a.cu_q_len = block_table.data_ptr(), kv_len.data_ptr(), cu_q_len.data_ptr()
    a.host_kv_len, a.host_cu_q_len = hk.ctypes.data, hc.ctypes.data
    a.error_count = _dev_ptr(error_count)
    return a, (hk, hc, new_k, new_v, k_cache, v_cache, block_table, kv_len, cu_q_len, error_count)


def spec_kv_append_args(args, stream=None) -> None:
    """`spec_kv_append` on a struct made by `make_kv_append_args`."""
    fn = lib().spec_kv_append
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p, C.c_void_p]
    _check(fn(C.addressof(args), _stream_handle(stream)), "spec_kv_append")


def spec_kv_append(new_k, new_v, k_cache, v_cache, block_table, kv_len, cu_q_len, host_kv_len, host_cu_q_len, *,
                   kv_layout: int = KV_TOKEN_MAJOR, stream=None, error_count=None) -> None:
    """Writes this step's K/V rows [T,Hkv,d] into the paged caches [nb,Hkv,16,d] in place."""
    a, _keep = make_kv_append_args(new_k, new_v, k_cache, v_cache, block_table, kv_len, cu_q_len, host_kv_len,
                                   host_cu_q_len, kv_layout=kv_layout, error_count=error_count)
    spec_kv_append_args(a, stream)


def spec_profile_begin(max_launches: int) -> None:
    _check(lib().spec_profile_begin(int(max_launches)), "spec_profile_begin")


def spec_profile_end():
    """Returns {kernel name: (total ms, launches)}."""
    ms = (C.c_float * NUM_KERNELS)()
    n = (C.c_int32 * NUM_KERNELS)()
    _check(lib().spec_profile_end(ms, n), "spec_profile_end")
    return {KERNEL_NAMES[i]: (float(ms[i]), int(n[i])) for i in range(NUM_KERNELS)}


def spec_verify_version() -> int:
    return int(lib().spec_verify_version())


def alloc_workspace(nbytes: int, device="cuda"):
    """A 256-byte aligned device buffer (torch's allocator aligns to 512)."""
    import torch
    return torch.empty(max(nbytes, 256), dtype=torch.uint8, device=device)


# ---------------------------------------------------------------------------
# Host-side speculation control (no GPU work): thin wrappers, marshalling only.
# ---------------------------------------------------------------------------
class LatencyModel(C.Structure):
    """Eq. 3 of the paper: seconds = c_context * N_context + c_batched * N_batched + c_fixed."""
    _fields_ = [("c_context", C.c_double), ("c_batched", C.c_double), ("c_fixed", C.c_double)]


class AcceptanceTracker(C.Structure):
    _fields_ = [("accepted_weighted", C.c_double), ("attempted_weighted", C.c_double)]

    def update(self, accepted: int, attempted: int, decay: float = 0.9) -> None:
        _host_fn("spec_acceptance_update", None, [C.c_void_p, C.c_int64, C.c_int64, C.c_double])(
            C.addressof(self), int(accepted), int(attempted), float(decay))

    def rate(self, prior: float = 0.7) -> float:
        return float(_host_fn("spec_acceptance_rate", C.c_double, [C.c_void_p, C.c_double])(
            C.addressof(self), float(prior)))


class GoodputArgs(C.Structure):
    _fields_ = [("B", C.c_int32), ("max_k", C.c_int32), ("context_len", C.c_void_p), ("alpha", C.c_void_p),
                ("alpha_per_request", C.c_int32), ("target", LatencyModel), ("draft_is_model", C.c_int32),
                ("draft", LatencyModel), ("draft_fixed_seconds", C.c_double), ("free_kv_tokens", C.c_int64)]


def _host_fn(name, restype, argtypes):
    fn = getattr(lib(), name)
    fn.restype = restype
    fn.argtypes = argtypes
    return fn


def expected_generated_len(alpha: float, k: int) -> float:
    return float(_host_fn("spec_expected_generated_len", C.c_double, [C.c_double, C.c_int32])(alpha, k))


def fit_latency(n_context, n_batched, seconds) -> LatencyModel:
    nc = np.ascontiguousarray(n_context, dtype=np.float64)
    nb = np.ascontiguousarray(n_batched, dtype=np.float64)
    t = np.ascontiguousarray(seconds, dtype=np.float64)
    m = LatencyModel()
    _check(_host_fn("spec_fit_latency", C.c_int, [C.c_void_p] * 3 + [C.c_int32, C.c_void_p])(
        nc.ctypes.data, nb.ctypes.data, t.ctypes.data, len(t), C.addressof(m)), "spec_fit_latency")
    return m


def predict_latency(model: LatencyModel, n_context: float, n_batched: float) -> float:
    return float(_host_fn("spec_predict_latency", C.c_double, [C.c_void_p, C.c_double, C.c_double])(
        C.addressof(model), n_context, n_batched))


def argmax_goodput(context_len, alpha, max_k: int, target: LatencyModel, draft: Optional[LatencyModel] = None,
                   draft_fixed_seconds: float = 0.0, free_kv_tokens: int = -1):
    """Returns (best k, goodput per k in tokens/s)."""
    ctx = np.ascontiguousarray(context_len, dtype=np.int32)
    al = np.ascontiguousarray(np.atleast_1d(alpha), dtype=np.float64)
    a = GoodputArgs()
    a.B, a.max_k = len(ctx), max_k
    a.context_len, a.alpha = ctx.ctypes.data, al.ctypes.data
    a.alpha_per_request = 1 if (len(al) == len(ctx) and len(ctx) > 1) else 0
    a.target = target
    a.draft_is_model = 1 if draft is not None else 0
    if draft is not None:
        a.draft = draft
    a.draft_fixed_seconds = draft_fixed_seconds
    a.free_kv_tokens = free_kv_tokens
    curve = np.zeros(max_k + 1, dtype=np.float64)
    k = int(_host_fn("spec_argmax_goodput", C.c_int32, [C.c_void_p, C.c_void_p])(C.addressof(a), curve.ctypes.data))
    return k, curve
