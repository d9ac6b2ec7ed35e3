"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol the header declares, and validates arguments before launching anything."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2406_14066_amd import spec_verify as sv

ROOT = os.path.abspath(os.path.join(os.path.dirname(__file__), ".."))
HEADER = os.path.join(ROOT, "include", "spec_verify.h")


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spec_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(sv.EXPORTS)
    lib = C.CDLL(sv.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_version_and_status_strings():
    assert sv.spec_verify_version() >= 100
    seen = {sv.status_string(s) for s in (0, -1, -2, -3, -4)}
    assert len(seen) == 5 and "ok" in seen
    assert "unknown" in sv.status_string(-99)


FAKE = 0x1000  # non-null, 16-byte aligned, never dereferenced: validation is host-only


def _attn(B=2, Hq=4, Hkv=2, d=128, kv_len=(40, 20), q_len=(3, 2), max_blocks=4, dtype=sv.SPEC_BF16,
          layout=sv.KV_MFMA):
    hk = np.asarray(kv_len, dtype=np.int32)
    hc = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    a = sv.AttnArgs()
    a.B, a.Hq, a.Hkv, a.d = B, Hq, Hkv, d
    a.block_size, a.num_blocks, a.max_blocks_per_req = 16, 16, max_blocks
    a.T = int(hc[-1])
    a.qkv_dtype, a.kv_layout = dtype, layout
    for f in ("q", "k_cache", "v_cache", "block_table", "kv_len", "cu_q_len", "out"):
        setattr(a, f, FAKE)
    a.host_kv_len = hk.ctypes.data
    a.host_cu_q_len = hc.ctypes.data
    a._keep = (hk, hc)
    return a


def _reject(B=2, V=32, q_len=(3, 2)):
    hc = np.concatenate([[0], np.cumsum(q_len)]).astype(np.int32)
    r = sv.RejectArgs()
    r.B, r.V, r.T = B, V, int(hc[-1])
    for f in ("target_logits", "draft_logits", "draft_tokens", "cu_q_len", "accepted_len", "next_token", "counters"):
        setattr(r, f, FAKE)
    r.host_cu_q_len = hc.ctypes.data
    r._keep = (hc,)
    return r


def test_validate_attn_accepts_good_arguments():
    assert sv.spec_validate_attn(_attn()) == sv.SPEC_OK
    assert sv.spec_validate_attn(_attn(dtype=sv.SPEC_F32, layout=sv.KV_TOKEN_MAJOR, d=64)) == sv.SPEC_OK


@pytest.mark.parametrize("mutate,status", [
    (lambda a: setattr(a, "q", None), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "out", None), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "host_kv_len", None), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "Hkv", 3), sv.SPEC_EINVAL),             # Hq % Hkv != 0
    (lambda a: setattr(a, "T", 6), sv.SPEC_EINVAL),               # != cu_q_len[B]
    (lambda a: setattr(a, "max_blocks_per_req", 2), sv.SPEC_EINVAL),  # 40 tokens need 3 pages
    (lambda a: setattr(a, "softmax_scale", -1.0), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "k_cache", FAKE + 16), sv.SPEC_EINVAL),     # pools, q and out: 32-byte aligned
    (lambda a: setattr(a, "out", FAKE + 4), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "qkv_dtype", 5), sv.SPEC_EINVAL),
    (lambda a: setattr(a, "block_size", 32), sv.SPEC_EUNSUPPORTED),
    (lambda a: setattr(a, "d", 96), sv.SPEC_EUNSUPPORTED),
    (lambda a: setattr(a, "qkv_dtype", sv.SPEC_F32), sv.SPEC_EUNSUPPORTED),  # fp32 in the bf16-only layout
])
def test_validate_attn_rejects(mutate, status):
    a = _attn()
    mutate(a)
    assert sv.spec_validate_attn(a) == status
    # the launching entry point reports the same status without touching the GPU
    assert sv.lib().spec_verify_attn(C.byref(a), FAKE, 1 << 30, None) == status


def test_validate_attn_per_request_limits():
    assert sv.spec_validate_attn(_attn(kv_len=(40, 1), q_len=(3, 2))) == sv.SPEC_EINVAL      # kv_len < q_len
    assert sv.spec_validate_attn(_attn(kv_len=(40, 20), q_len=(10, 2))) == sv.SPEC_EINVAL    # k_b > K_MAX
    assert sv.spec_validate_attn(_attn(kv_len=(40, 20), q_len=(9, 1))) == sv.SPEC_OK


def test_validate_reject():
    assert sv.spec_validate_reject(_reject()) == sv.SPEC_OK
    r = _reject()
    r.counters = None
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL
    r = _reject()
    r.draft_logits = None
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL
    r = _reject(q_len=(1, 1))       # k = 0 everywhere: no draft rows needed
    r.draft_logits = None
    r.draft_tokens = None
    assert sv.spec_validate_reject(r) == sv.SPEC_OK
    assert sv.spec_validate_reject(_reject(V=30)) == sv.SPEC_EUNSUPPORTED
    assert sv.spec_validate_reject(_reject(q_len=(10, 2))) == sv.SPEC_EINVAL
    r = _reject()
    r.target_logits = FAKE + 4
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL


def test_workspace_query_and_workspace_errors():
    a, r = _attn(), _reject()
    na = sv.spec_verify_workspace_bytes(a, None)
    nr = sv.spec_verify_workspace_bytes(None, r)
    nb = sv.spec_verify_workspace_bytes(a, r)
    assert na > 0 and nr > 0 and nb == na + nr and na % 256 == 0 and nr % 256 == 0
    L = sv.lib()
    assert L.spec_verify_attn(C.byref(a), None, na, None) == sv.SPEC_EWORKSPACE
    assert L.spec_verify_attn(C.byref(a), FAKE, na - 1, None) == sv.SPEC_EWORKSPACE
    assert L.spec_verify_attn(C.byref(a), FAKE + 8, na, None) == sv.SPEC_EWORKSPACE      # misaligned
    assert L.spec_reject_sample(C.byref(r), FAKE, nr - 1, None) == sv.SPEC_EWORKSPACE
    assert L.spec_verify_step(C.byref(a), C.byref(r), FAKE, nb - 1, None) == sv.SPEC_EWORKSPACE
    bad = _attn()
    bad.q = None
    with pytest.raises(sv.SpecVerifyError):
        sv.spec_verify_workspace_bytes(bad, None)
    # step: the two halves must describe the same batch
    r3 = _reject(B=2, q_len=(2, 2))
    assert L.spec_verify_step(C.byref(a), C.byref(r3), FAKE, 1 << 30, None) == sv.SPEC_EINVAL


def test_repack_validation():
    L = sv.lib()
    assert L.spec_kv_repack_mfma(None, FAKE, FAKE + 256, FAKE + 512, 1, 1, 128, None) == sv.SPEC_EINVAL
    assert L.spec_kv_repack_mfma(FAKE, FAKE + 256, FAKE, FAKE + 512, 1, 1, 128, None) == sv.SPEC_EINVAL   # aliasing
    assert L.spec_kv_repack_mfma(FAKE, FAKE + 256, FAKE + 512, FAKE + 768, 1, 1, 96, None) == sv.SPEC_EUNSUPPORTED


def test_product_never_touches_the_oracle():
    pkg = os.path.join(ROOT, "paper_2406_14066_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text and "spec_oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2406_14066_amd" not in text and "spec_verify.h" not in text, f


def test_accept_mode_validation():
    """Modes without a draft distribution take a NULL draft_logits; an unknown mode is refused."""
    cu = np.array([0, 3, 5], dtype=np.int32)
    FAKE = 0x1000
    def args(mode, draft_logits):
        r = sv.RejectArgs()
        r.B, r.V, r.T = 2, 64, 5
        r.target_logits = FAKE
        r.draft_logits = draft_logits
        r.draft_tokens = FAKE
        r.cu_q_len = FAKE
        r.host_cu_q_len = cu.ctypes.data
        r.accepted_len = FAKE
        r.next_token = FAKE
        r.counters = FAKE
        r.accept_mode = mode
        return r
    assert sv.spec_validate_reject(args(sv.ACCEPT_SAMPLE, FAKE)) == sv.SPEC_OK
    assert sv.spec_validate_reject(args(sv.ACCEPT_SAMPLE, None)) == sv.SPEC_EINVAL
    assert sv.spec_validate_reject(args(sv.ACCEPT_GREEDY, None)) == sv.SPEC_OK
    assert sv.spec_validate_reject(args(sv.ACCEPT_POINT_DRAFT, None)) == sv.SPEC_OK
    assert sv.spec_validate_reject(args(3, FAKE)) == sv.SPEC_EINVAL
    assert sv.spec_validate_reject(args(-1, FAKE)) == sv.SPEC_EINVAL
    # fewer logit rows get a statistics pass without a draft distribution: the workspace is smaller
    assert (sv.spec_verify_workspace_bytes(None, args(sv.ACCEPT_GREEDY, None))
            <= sv.spec_verify_workspace_bytes(None, args(sv.ACCEPT_SAMPLE, FAKE)))


def test_kv_append_validation():
    import ctypes as C
    hk = np.array([20, 40], dtype=np.int32)
    hc = np.array([0, 3, 5], dtype=np.int32)
    FAKE = 0x1000
    def args(**kw):
        a = sv.KvAppendArgs()
        a.B, a.Hkv, a.d, a.num_blocks, a.max_blocks_per_req, a.T = 2, 2, 128, 8, 3, 5
        a.dtype, a.kv_layout = sv.SPEC_BF16, sv.KV_MFMA
        for f in ("new_k", "new_v", "k_cache", "v_cache", "block_table", "kv_len", "cu_q_len"):
            setattr(a, f, FAKE)
        a.host_kv_len, a.host_cu_q_len = hk.ctypes.data, hc.ctypes.data
        for k, v in kw.items():
            setattr(a, k, v)
        return a
    fn = sv.lib().spec_kv_append
    fn.restype = C.c_int
    fn.argtypes = [C.c_void_p, C.c_void_p]
    assert fn(None, None) == sv.SPEC_EINVAL
    assert fn(C.addressof(args(new_k=None)), None) == sv.SPEC_EINVAL
    assert fn(C.addressof(args(max_blocks_per_req=2)), None) == sv.SPEC_EINVAL     # 40 tokens need 3 pages
    assert fn(C.addressof(args(dtype=sv.SPEC_F32)), None) == sv.SPEC_EUNSUPPORTED        # tiles are bf16 only
    assert fn(C.addressof(args(d=96)), None) == sv.SPEC_EUNSUPPORTED
    assert fn(C.addressof(args(T=6)), None) == sv.SPEC_EINVAL
    bad_len = np.array([2, 40], dtype=np.int32)                                    # kv_len < q_len
    assert fn(C.addressof(args(host_kv_len=bad_len.ctypes.data)), None) == sv.SPEC_EINVAL


def test_bookkeeping_outputs_need_kv_len():
    cu = np.array([0, 3, 5], dtype=np.int32)
    FAKE = 0x1000
    r = sv.RejectArgs()
    r.B, r.V, r.T = 2, 64, 5
    for f in ("target_logits", "draft_logits", "draft_tokens", "cu_q_len", "accepted_len", "next_token", "counters"):
        setattr(r, f, FAKE)
    r.host_cu_q_len = cu.ctypes.data
    r.new_kv_len = FAKE
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL
    r.kv_len = FAKE
    assert sv.spec_validate_reject(r) == sv.SPEC_OK


def test_static_scratch_entry_refuses_what_does_not_fit():
    """spec_verify_step_static sizes the step on the host first: a step whose workspace exceeds the
    library's scratch array is refused before anything touches the GPU, and argument errors come
    back as from spec_verify_step."""
    L = sv.lib()
    # fp32 takes the generic kernel: one partial per (row, head, 256-token chunk)
    q_len = (9,) * 12
    a = _attn(B=12, Hq=32, Hkv=8, d=128, kv_len=(8000,) * 12, q_len=q_len, max_blocks=500,
              dtype=sv.SPEC_F32, layout=sv.KV_TOKEN_MAJOR)
    r = _reject(B=12, V=32, q_len=q_len)
    assert sv.spec_verify_workspace_bytes(a, r) > sv.STATIC_SCRATCH_BYTES
    assert L.spec_verify_step_static(C.byref(a), C.byref(r), None) == sv.SPEC_EWORKSPACE
    bad = _attn()
    bad.q = None
    assert L.spec_verify_step_static(C.byref(bad), C.byref(_reject()), None) == sv.SPEC_EINVAL
    assert L.spec_verify_step_static(C.byref(_attn()), C.byref(_reject(B=2, q_len=(2, 2))), None) == sv.SPEC_EINVAL


# --------------------------------------------------------------------------
# length buckets, host copies checked on request, plan query, tuning switches
# --------------------------------------------------------------------------
def test_validate_flag_checks_the_host_copies():
    a = _attn(kv_len=(40, 20), max_blocks=4)
    table = np.array([[0, 1, 2, 9], [3, 4, 9, 9]], dtype=np.int32)       # entries past the pages in use are not looked at
    a.host_block_table = table.ctypes.data
    a.validate = 1
    assert sv.spec_validate_attn(a) == sv.SPEC_OK
    table[0, 2] = 16                                                        # num_blocks is 16: out of range
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL
    assert sv.lib().spec_verify_attn(C.byref(a), FAKE, 1 << 30, None) == sv.SPEC_EINVAL
    table[0, 2] = -1
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL
    a.validate = 0                                                          # not asked for: not looked at
    assert sv.spec_validate_attn(a) == sv.SPEC_OK
    a.validate = 2
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL

    r = _reject(V=32, q_len=(3, 2))
    tok = np.array([1, 31, 0], dtype=np.int32)
    r.host_draft_tokens = tok.ctypes.data
    r.validate = 1
    assert sv.spec_validate_reject(r) == sv.SPEC_OK
    tok[1] = 32
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL
    assert sv.lib().spec_reject_sample(C.byref(r), FAKE, 1 << 30, None) == sv.SPEC_EINVAL
    tok[1] = -3
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL
    r.philox_step_device = FAKE + 4                                         # must be 8-byte aligned
    r.validate = 0
    assert sv.spec_validate_reject(r) == sv.SPEC_EINVAL


def test_length_bucket_arguments():
    a = _attn(kv_len=(40, 20), max_blocks=4)
    a.max_kv_len = 64
    assert sv.spec_validate_attn(a) == sv.SPEC_OK
    a.max_kv_len = 65                      # 5 pages do not fit a block-table row of 4
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL
    a.max_kv_len = 32                      # a host length above the bucket
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL
    a.max_kv_len = -1
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL
    a.max_kv_len = 64
    a.host_kv_len = None                   # with a bucket the host lengths are optional
    assert sv.spec_validate_attn(a) == sv.SPEC_OK
    a.max_kv_len = 0
    assert sv.spec_validate_attn(a) == sv.SPEC_EINVAL


def test_bucket_plan_does_not_depend_on_the_lengths():
    """Under a length bucket the split, the grid and the workspace depend on the bound only, so a
    launch captured for one set of lengths stays valid for another."""
    q_len = (3,) * 6
    plans = []
    for lens in [(100,) * 6, (5, 900, 64, 65, 1000, 3), None]:
        a = _attn(B=6, Hq=8, Hkv=2, kv_len=lens or (1,) * 6, q_len=q_len, max_blocks=64)
        a.max_kv_len = 1024
        if lens is None:
            a.host_kv_len = None
        r = _reject(B=6, V=4096, q_len=q_len)
        plans.append(sv.spec_verify_plan(a, r))
    assert plans[0] == plans[1] == plans[2]
    assert plans[0]["attn_path"] == sv.PATH_MFMA
    assert plans[0]["chunk_tokens"] * plans[0]["max_chunks"] >= 1024
    # without a bucket the plan follows the host lengths
    a = _attn(B=6, Hq=8, Hkv=2, kv_len=(100,) * 6, q_len=q_len, max_blocks=64)
    exact = sv.spec_verify_plan(a, _reject(B=6, V=4096, q_len=q_len))
    assert exact["chunk_tokens"] * exact["max_chunks"] < 1024


@pytest.mark.parametrize("Hq,Hkv,k,path,tiles,groups", [
    (32, 32, 8, sv.PATH_MFMA, 1, 1),     # 9 rows per KV head
    (64, 8, 2, sv.PATH_MFMA, 2, 1),      # 24 rows
    (32, 8, 8, sv.PATH_MFMA, 3, 1),      # 36 rows
    (64, 8, 5, sv.PATH_MFMA, 3, 1),      # 48 rows
    (64, 8, 6, sv.PATH_MFMA, 2, 2),      # 56 rows: two wave groups of two tiles
    (64, 8, 7, sv.PATH_MFMA, 2, 2),      # 64 rows
    (64, 8, 8, sv.PATH_MFMA, 3, 2),      # 72 rows
    (16, 1, 6, sv.PATH_MFMA, 2, 4),      # 112 rows: four wave groups
    (16, 1, 8, sv.PATH_MFMA, 3, 4),      # 144 rows: the widest group at the longest draft
    (16, 1, 3, sv.PATH_MFMA, 2, 2),      # 64 rows
])
def test_every_supported_row_count_takes_the_matrix_path(Hq, Hkv, k, path, tiles, groups):
    B = 4
    a = _attn(B=B, Hq=Hq, Hkv=Hkv, kv_len=(300,) * B, q_len=(k + 1,) * B, max_blocks=32)
    info = sv.spec_verify_plan(a, None)
    assert (info["attn_path"], info["row_tiles"], info["row_groups"]) == (path, tiles, groups), info
    assert info["launches"] == 1
    # token-major bf16 pages take the same path with the same split of the rows (V transposed through LDS);
    # fp32 takes the generic kernels; d = 64 takes the matrix path like d = 128
    tm = sv.spec_verify_plan(_attn(B=B, Hq=Hq, Hkv=Hkv, kv_len=(300,) * B, q_len=(k + 1,) * B, max_blocks=32,
                                   layout=sv.KV_TOKEN_MAJOR), None)
    assert (tm["attn_path"], tm["row_tiles"], tm["row_groups"], tm["launches"]) == (path, tiles, groups, 1), tm
    assert sv.spec_verify_plan(_attn(B=B, Hq=Hq, Hkv=Hkv, kv_len=(300,) * B, q_len=(k + 1,) * B, max_blocks=32,
                                     dtype=sv.SPEC_F32, layout=sv.KV_TOKEN_MAJOR), None)["attn_path"] == sv.PATH_GENERIC
    d64 = sv.spec_verify_plan(_attn(B=B, Hq=Hq, Hkv=Hkv, d=64, kv_len=(300,) * B, q_len=(k + 1,) * B, max_blocks=32), None)
    assert (d64["attn_path"], d64["row_tiles"], d64["row_groups"]) == (path, tiles, groups), d64
    d64tm = sv.spec_verify_plan(_attn(B=B, Hq=Hq, Hkv=Hkv, d=64, kv_len=(300,) * B, q_len=(k + 1,) * B, max_blocks=32,
                                      layout=sv.KV_TOKEN_MAJOR), None)
    assert (d64tm["attn_path"], d64tm["row_tiles"], d64tm["row_groups"]) == (path, tiles, groups), d64tm


def test_tuning_switches_are_read_once_and_on_reload(monkeypatch):
    a = _attn(B=4, Hq=8, Hkv=2, kv_len=(300,) * 4, q_len=(3,) * 4, max_blocks=32)
    assert sv.spec_verify_plan(a, None)["attn_path"] == sv.PATH_MFMA
    monkeypatch.setenv("SPEC_VERIFY_FORCE_GENERIC", "1")
    assert sv.spec_verify_plan(a, None)["attn_path"] == sv.PATH_MFMA        # not re-read on the call path
    sv.reload_env()
    try:
        assert sv.spec_verify_plan(a, None)["attn_path"] == sv.PATH_GENERIC
    finally:
        monkeypatch.undo()
        sv.reload_env()
    assert sv.spec_verify_plan(a, None)["attn_path"] == sv.PATH_MFMA


@pytest.mark.parametrize("B,Hq,Hkv,length,most_chunks", [
    (1, 64, 8, 2749, 8),      # a launch bound by latencies: few chunks, however many compute units are idle
    (1, 64, 8, 172, 1),       # ... and none below 256 tokens
    (4, 64, 8, 204, 1),
    (1, 32, 32, 2048, 8),
    (1, 32, 8, 32768, 32),    # long enough for chunks of 1024 tokens: split as far as the compute units ask
])
def test_small_launches_are_split_sparingly(B, Hq, Hkv, length, most_chunks):
    a = _attn(B=B, Hq=Hq, Hkv=Hkv, kv_len=(length,) * B, q_len=(3,) * B, max_blocks=(length + 15) // 16)
    plan = sv.spec_verify_plan(a, None)
    assert plan["attn_path"] == sv.PATH_MFMA
    assert plan["max_chunks"] <= most_chunks, plan
    assert plan["chunk_tokens"] >= 256 and plan["chunk_tokens"] * plan["max_chunks"] >= length, plan
    if most_chunks > 8:
        assert plan["max_chunks"] > 8 and plan["chunk_tokens"] >= 1024, plan


def test_split_requests_get_whole_rows_of_eight_attention_items():
    """With split requests every chunk index has its items padded to whole rows of 8 blocks (one per XCD),
    so that all chunks of a (request, KV head) run on the same XCD; unsplit requests need no padding."""
    long = _attn(B=3, Hq=32, Hkv=4, kv_len=(20000, 17000, 23000), q_len=(5, 5, 5), max_blocks=1500)
    plan = sv.spec_verify_plan(long, None)
    assert plan["max_chunks"] > 1 and plan["attn_blocks"] == 16 * plan["max_chunks"], plan      # 12 units -> 16 items per row
    short = _attn(B=3, Hq=32, Hkv=4, kv_len=(200, 170, 230), q_len=(5, 5, 5), max_blocks=16)
    plan = sv.spec_verify_plan(short, None)
    assert plan["max_chunks"] == 1 and plan["attn_blocks"] == 12, plan


def test_plan_is_reused_for_an_unchanged_shape_and_follows_a_changed_one():
    q_len = (3,) * 6
    a = _attn(B=6, Hq=8, Hkv=2, kv_len=(100, 200, 300, 400, 500, 600), q_len=q_len, max_blocks=64)
    r = _reject(B=6, V=4096, q_len=q_len)
    first = sv.spec_verify_plan(a, r)
    assert sv.spec_verify_plan(a, r) == first
    hk = np.array([100, 200, 300, 400, 500, 1000], dtype=np.int32)        # same buffer shape, one longer request
    a.host_kv_len = hk.ctypes.data
    longer = sv.spec_verify_plan(a, r)
    assert longer["chunk_tokens"] * longer["max_chunks"] >= 1000 > first["chunk_tokens"] * first["max_chunks"]
    bad = np.array([100, 200, 300, 400, 500, 2], dtype=np.int32)          # kv_len < q_len: the cached plan must not hide it
    a.host_kv_len = bad.ctypes.data
    assert sv.lib().spec_verify_step(C.byref(a), C.byref(r), FAKE, 1 << 30, None) == sv.SPEC_EINVAL
