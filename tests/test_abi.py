"""The C-ABI library loads without a GPU and exports every symbol the header declares;
argument checks that launch nothing run here too."""
import ctypes as C
import os
import re

from paper_2502_02789_amd import binding as sp

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "specprefill.h")).read()
    return re.findall(r"^SP_API\s+[\w\s\*]+?\b(sp_\w+)\s*\(", text, flags=re.M)


def test_every_declared_symbol_is_exported():
    names = _declared()
    assert set(names) == set(sp.EXPORTS) and len(names) == len(sp.EXPORTS)
    lib = C.CDLL(sp.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_probe_library_exports_what_its_header_declares():
    from paper_2502_02789_amd import probe
    text = open(os.path.join(ROOT, "include", "sp_probe.h")).read()
    names = re.findall(r"^SP_PROBE_API\s+[\w\s\*]+?\b(sp_\w+)\s*\(", text, flags=re.M)
    assert set(names) == set(probe.EXPORTS) and len(names) == len(probe.EXPORTS)
    lib = C.CDLL(probe.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    lib = probe.load_library()
    assert lib.sp_probe_read(None, 1, 16, 1, None, None) == -1          # argument checks need no GPU
    assert lib.sp_probe_tiled(None, 1, 32768, 8, 128, 1024, 128, None, None) == -1
    assert lib.sp_probe_tiled_default_policy(None, 1, 32768, 8, 128, 1024, 128, None, None) == -1


def test_struct_layouts_match_the_header_field_order():
    text = open(os.path.join(ROOT, "include", "specprefill.h")).read()
    for cname, cls in (("sp_score_args", sp.ScoreArgs), ("sp_pool_select_args", sp.PoolSelectArgs),
                       ("sp_gather_args", sp.GatherArgs)):
        body = re.search(r"typedef struct \{([^}]*)\}\s*" + cname + ";", text).group(1)
        body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
        fields = [re.search(r"(\w+)\s*$", decl.strip()).group(1) for decl in body.split(";") if decl.strip()]
        assert fields == [f[0] for f in cls._fields_], cname


def test_version_and_messages():
    assert sp.sp_version() >= 100
    for code in range(0, -8, -1):
        assert sp.strerror(code) and sp.strerror(code) != "unknown status"
    assert sp.strerror(-99) == "unknown status"


def test_host_side_argument_checks_need_no_gpu():
    lib = sp.load_library()
    assert lib.sp_score(None, None) == sp.SP_ENULL
    assert lib.sp_score(C.byref(sp.ScoreArgs()), None) == sp.SP_EINVAL
    assert lib.sp_score_workspace_bytes(C.byref(sp.ScoreArgs())) == 0
    assert lib.sp_pool_select(None, None) == sp.SP_ENULL
    assert lib.sp_pool_select(C.byref(sp.PoolSelectArgs()), None) == sp.SP_EINVAL
    assert lib.sp_gather(None, None) == sp.SP_ENULL
    a = sp.ScoreArgs()
    a.B, a.N, a.L, a.H, a.H_kv, a.d, a.T = 1, 8, 32, 32, 8, 128, 32768
    assert lib.sp_score_workspace_bytes(C.byref(a)) > 0
    assert lib.sp_score(C.byref(a), None) == sp.SP_ENULL


def _fake_score_args():
    """A fully populated sp_score_args whose device pointers are made-up, aligned addresses: good
    enough for every host-side check (which come before any launch), never dereferenced."""
    a = sp.ScoreArgs()
    a.B, a.N, a.L, a.H, a.H_kv, a.d, a.T = 1, 8, 2, 32, 8, 128, 4096
    arr = (C.c_void_p * 2)(0x7000_0000_0000, 0x7000_1000_0000)
    a._keepalive = arr
    a.k_layers = C.cast(arr, C.POINTER(C.c_void_p))
    a.d_q, a.d_cu_seqlens, a.d_scores = 0x7000_2000_0000, 0x7000_2100_0000, 0x7000_2200_0000
    a.k_token_stride, a.k_head_stride = 1024, 128
    a.scale, a.layer_reduce = 0.088, sp.SP_LAYER_MAX
    return a


def test_nan_arguments_are_refused_before_anything_is_launched():
    lib = sp.load_library()
    nan = float("nan")
    a = _fake_score_args()
    assert lib.sp_score(C.byref(a), None) == sp.SP_EWORKSPACE          # everything else is acceptable
    a.scale = nan
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    assert lib.sp_score_general(C.byref(a), None) == sp.SP_EINVAL
    a = _fake_score_args()
    a.rope_theta = nan
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    a = _fake_score_args()
    a.scale = float("inf")
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    s = sp.PoolSelectArgs()
    s.B, s.T, s.chunk, s.pool_window, s.keep_rate, s.kept_capacity = 1, 4096, 32, 13, 0.1, 4096
    s.d_cu_seqlens, s.d_scores, s.d_kept_idx, s.d_cu_keep = 0x7000_0000_0000, 0x7000_1000_0000, 0x7000_2000_0000, 0x7000_3000_0000
    assert lib.sp_pool_select(C.byref(s), None) == sp.SP_EWORKSPACE
    for bad in (nan, 0.0, -0.5, 1.5, float("inf")):
        s.keep_rate = bad
        assert lib.sp_pool_select(C.byref(s), None) == sp.SP_EINVAL, bad
        assert lib.sp_pool_select_workspace_bytes(C.byref(s)) == 0, bad
    assert sp.sp_keep_upper_bound([10], 4, nan) == -1


def test_keep_upper_bound_follows_the_chunk_ratio_rule():
    assert sp.sp_keep_upper_bound([1024], 32, 0.25) == 256
    assert sp.sp_keep_upper_bound([8192], 32, 0.1) == 26 * 32
    assert sp.sp_keep_upper_bound([32768], 32, 0.1) == 103 * 32
    assert sp.sp_keep_upper_bound([131072], 64, 0.05) == 103 * 64
    assert sp.sp_keep_upper_bound([10], 1, 0.3) == 3
    assert sp.sp_keep_upper_bound([10, 0, 5], 4, 1.0) == 15
    assert sp.sp_keep_upper_bound([10], 0, 0.3) == -1
    assert sp.sp_keep_upper_bound([10], 4, 0.0) == -1


def test_rules_of_the_later_fields_need_no_gpu():
    """max_seqlen, k_dtype and d_k_scale: what the header promises about them is checked on the host."""
    lib = sp.load_library()
    a = _fake_score_args()
    a.max_seqlen = -1
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    a = _fake_score_args()
    a.k_dtype = 7
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    assert lib.sp_score_workspace_bytes(C.byref(a)) == 0
    a = _fake_score_args()
    a.d_k_scale = 0x7000_3000_0000                      # scales with a bf16 cache
    assert lib.sp_score(C.byref(a), None) == sp.SP_EINVAL
    a = _fake_score_args()
    a.k_dtype = sp.SP_K_FP8_E4M3
    a.d_k_scale = 0x7000_3000_0000
    assert lib.sp_score(C.byref(a), None) == sp.SP_EWORKSPACE          # acceptable apart from the workspace
    a.k_token_stride = 1032                             # a multiple of 8, not of 16
    assert lib.sp_score(C.byref(a), None) == sp.SP_EALIGN
    a.k_token_stride = 1024
    a.rope_theta, a.d_q_pos = 10000.0, 0x7000_4000_0000
    assert lib.sp_score(C.byref(a), None) == sp.SP_EUNSUPPORTED
    # the workspace query follows the kernels the fields select
    b = _fake_score_args()
    b.B, b.N, b.T = 64, 1, 4096 * 64
    without = lib.sp_score_workspace_bytes(C.byref(b))
    b.max_seqlen = 4096
    with_promise = lib.sp_score_workspace_bytes(C.byref(b))
    assert 0 < with_promise < without                   # no kept-logits buffer once the batch kernel applies
