"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes the workspace, and turns bad arguments into error codes before anything
is enqueued (dry-run contexts never touch a device)."""
import ctypes as C
import os
import re

import pytest

from paper_2511_14510_amd import binding as Q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(Q.LIB_PATH):
        from paper_2511_14510_amd import build
        build.build()
    return Q.load()


def _declared(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return set(re.findall(r"\b(qsac_[a-z_]+)\s*\(", text))


def test_exports_every_declared_symbol(lib):
    declared = _declared("qsac.h")
    assert declared == set(Q.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    # the measurement aids live in a library of their own and are not part of the product library
    calib = Q.load_calib()
    assert _declared("qsac_calib.h") == set(Q.CALIB_EXPORTS)
    for name in Q.CALIB_EXPORTS:
        assert hasattr(calib, name), name
        assert not hasattr(lib, name), name


def test_struct_sizes_match_the_header(lib):
    # a mismatch between the ctypes mirror and the C structs would corrupt every call
    src = r'''
    #include "qsac.h"
    #include <stdio.h>
    int main(void){ printf("%zu %zu %zu %zu %zu\n", sizeof(qsac_config), sizeof(qsac_ws_layout), sizeof(qsac_step_args), sizeof(qsac_stats), sizeof(qsac_dev_params)); return 0; }
    '''
    import subprocess, tempfile
    with tempfile.TemporaryDirectory() as d:
        open(os.path.join(d, "s.c"), "w").write(src)
        subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", os.path.join(d, "s"), os.path.join(d, "s.c")])
        sizes = [int(x) for x in subprocess.check_output([os.path.join(d, "s")]).split()]
    assert sizes == [C.sizeof(Q.qsac_config), C.sizeof(Q.qsac_ws_layout), C.sizeof(Q.qsac_step_args), C.sizeof(Q.qsac_stats),
                     C.sizeof(Q.qsac_dev_params)]


def test_workspace_size_and_layout(lib):
    cfg = Q.make_config(8, 32, 8, 32768, 2048, Q.QSAC_BF16)
    n = Q.qsac_workspace_bytes(cfg)
    L = Q.qsac_workspace_layout(cfg)
    assert n == L.total and n > 64 * 32768 * 4
    assert L.n_pad == 32768 and L.words == 1024 and L.max_splits == 32
    offs = [getattr(L, f) for f, _ in Q.qsac_ws_layout._fields_[:17]]
    assert offs == sorted(offs) and all(o % 256 == 0 for o in offs)
    cfg = Q.make_config(1, 8, 2, 5000, 100, Q.QSAC_F16)
    assert Q.qsac_workspace_layout(cfg).n_pad == 8192


@pytest.mark.parametrize("kw,code", [
    (dict(D=64), Q.QSAC_EINVAL),
    (dict(dtype=7), Q.QSAC_EINVAL),
    (dict(Hq=9), Q.QSAC_EINVAL),          # 9 % 2 != 0
    (dict(Hq=18), Q.QSAC_ERANGE),         # G = 9 > 8
    (dict(B=0), Q.QSAC_ERANGE),
    (dict(N=0), Q.QSAC_ERANGE),
    (dict(N=(1 << 20) + 1), Q.QSAC_ERANGE),
    (dict(k_max=0), Q.QSAC_ERANGE),
    (dict(k_max=4097), Q.QSAC_ERANGE),    # k_max > N
    (dict(Hkv=65, Hq=65), Q.QSAC_ERANGE),
    (dict(flags=1 << 20), Q.QSAC_EINVAL),
    (dict(importance=[1, 1, 1, 0, 1, 1, 1, 1]), Q.QSAC_EINVAL),
    (dict(flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_PUSH_HOLD), Q.QSAC_EINVAL),                         # hold without push mode
    (dict(flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_PUSH_FILL | Q.QSAC_FLAG_FILL_KERNEL), Q.QSAC_EINVAL),  # two ways to fill
    (dict(flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_PUSH_FILL, push_threads=65), Q.QSAC_ERANGE),
    (dict(flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_PUSH_FILL, push_wait_us=-1), Q.QSAC_ERANGE),
    (dict(flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_STAGGER), Q.QSAC_EINVAL),                           # a batch of one has no halves
    (dict(B=2, flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_STAGGER | Q.QSAC_FLAG_FILL_KERNEL), Q.QSAC_EINVAL),
    (dict(B=2, flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_STAGGER | Q.QSAC_FLAG_PUSH_FILL), Q.QSAC_EINVAL),
    (dict(B=2, flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_STAGGER | Q.QSAC_FLAG_PROFILE), Q.QSAC_EINVAL),
    (dict(B=4097, flags=Q.QSAC_FLAG_DRY_RUN | Q.QSAC_FLAG_STAGGER), Q.QSAC_EINVAL),                   # more than 8192 pairs
])
def test_bad_configs_are_rejected(lib, kw, code):
    a = dict(B=1, Hq=8, Hkv=2, N=4096, k_max=256, dtype=Q.QSAC_F16, flags=Q.QSAC_FLAG_DRY_RUN, importance=None, D=128,
             push_threads=0, push_wait_us=0)
    a.update(kw)
    cfg = Q.make_config(a["B"], a["Hq"], a["Hkv"], a["N"], a["k_max"], a["dtype"], a["flags"], a["importance"],
                        push_threads=a["push_threads"], push_wait_us=a["push_wait_us"])
    cfg.head_dim = a["D"]
    assert Q.qsac_workspace_bytes(cfg) == 0
    ctx = C.c_void_p()
    assert lib.qsac_init(C.byref(cfg), C.byref(ctx)) == code
    assert not ctx.value


def test_staggered_schedule_needs_a_second_stream(lib):
    """Checked by qsac_init before it touches a device (the workspace size does not depend on streams)."""
    cfg = Q.make_config(2, 8, 2, 4096, 256, Q.QSAC_F16, Q.QSAC_FLAG_STAGGER, None)
    assert Q.qsac_workspace_bytes(cfg) > 0
    ctx = C.c_void_p()
    assert lib.qsac_init(C.byref(cfg), C.byref(ctx)) == Q.QSAC_EINVAL and not ctx.value


def test_workspace_checks_without_dry_run(lib):
    cfg = Q.make_config(1, 8, 2, 4096, 256, Q.QSAC_F16)
    ctx = C.c_void_p()
    assert lib.qsac_init(C.byref(cfg), C.byref(ctx)) == Q.QSAC_EWORKSPACE     # no workspace
    cfg.workspace, cfg.workspace_bytes = 0x1000100, 16                          # too small
    assert lib.qsac_init(C.byref(cfg), C.byref(ctx)) == Q.QSAC_EWORKSPACE
    cfg.workspace, cfg.workspace_bytes = 0x1000010, 1 << 30                     # misaligned
    assert lib.qsac_init(C.byref(cfg), C.byref(ctx)) == Q.QSAC_EWORKSPACE
    assert lib.qsac_init(None, C.byref(ctx)) == Q.QSAC_ENULL
    assert lib.qsac_init(C.byref(cfg), None) == Q.QSAC_ENULL


def _args(**over):
    a = Q.qsac_step_args()
    for f, _ in Q.qsac_step_args._fields_:
        if f not in ("tau", "n_tau", "k", "V_res", "res_slot", "n_res", "K_app", "V_app", "n_app", "dev_params"):
            setattr(a, f, 0x10000)
    tau = (C.c_float * 2)(0.9, 0.8)
    a._keep = tau
    a.tau, a.n_tau, a.k = C.cast(tau, C.POINTER(C.c_float)), 1, 256
    for key, v in over.items():
        setattr(a, key, v)
    return a


def test_step_validation_on_a_dry_run_context(lib):
    cfg = Q.make_config(1, 8, 2, 4096, 256, Q.QSAC_F16, Q.QSAC_FLAG_DRY_RUN)
    ctx = Q.qsac_init(cfg)
    step = lambda a: lib.qsac_step(ctx, C.byref(a))
    assert lib.qsac_step(ctx, None) == Q.QSAC_ENULL
    assert lib.qsac_step(None, C.byref(_args())) == Q.QSAC_ESTATE
    for f in ("q", "K_dev", "K_src", "V_src", "K_slots", "V_slots", "slot_idx", "prev_q", "out", "topk_idx",
              "hit_mask", "reuse_flags"):
        assert step(_args(**{f: None})) == Q.QSAC_ENULL, f
    assert step(_args(tau=C.POINTER(C.c_float)())) == Q.QSAC_ENULL
    assert step(_args(sim=None)) == Q.QSAC_OK                      # sim is optional
    Q.qsac_reset(ctx)
    assert step(_args(n_tau=3)) == Q.QSAC_EINVAL                   # neither 1 nor n_kv_heads
    assert step(_args(n_tau=2)) == Q.QSAC_OK
    nan = (C.c_float * 1)(float("nan"))
    assert step(_args(tau=C.cast(nan, C.POINTER(C.c_float)))) == Q.QSAC_EINVAL
    assert step(_args(k=0)) == Q.QSAC_ERANGE
    assert step(_args(k=257)) == Q.QSAC_ERANGE
    assert step(_args(q=0x10008)) == Q.QSAC_EALIGN
    rs = (C.c_int8 * 2)(0, -1)
    rsp = C.cast(rs, C.POINTER(C.c_int8))
    assert step(_args(res_slot=rsp, n_res=1)) == Q.QSAC_ENULL      # resident heads without a resident V
    assert step(_args(res_slot=rsp, n_res=1, V_res=0x20000)) == Q.QSAC_OK
    assert step(_args(res_slot=rsp, n_res=0, V_res=0x20000)) == Q.QSAC_ERANGE
    assert step(_args(res_slot=rsp, n_res=3, V_res=0x20000)) == Q.QSAC_ERANGE
    bad = (C.c_int8 * 2)(1, -1)
    assert step(_args(res_slot=C.cast(bad, C.POINTER(C.c_int8)), n_res=1, V_res=0x20000)) == Q.QSAC_ERANGE
    assert step(_args(n_app=1, K_app=0x30000, V_app=0x40000)) == Q.QSAC_ERANGE   # no append capacity configured
    assert step(_args(k=128)) == Q.QSAC_ESTATE                     # k changed without a reset
    Q.qsac_reset(ctx)
    assert step(_args(k=128)) == Q.QSAC_OK
    # per-step scalars in device memory: tau may then be absent; the block must be aligned
    assert step(_args(k=128, dev_params=0x50000, tau=C.POINTER(C.c_float)(), n_tau=0)) == Q.QSAC_OK
    assert step(_args(k=128, dev_params=0x50004)) == Q.QSAC_EALIGN
    st = Q.qsac_get_stats(ctx)
    assert st["steps"] == 2 and st["bytes_filled_host"] == 0 and st["bytes_filled_dev"] == 0   # failed calls do not count
    # a graph needs a context that runs on a device
    g = C.c_void_p()
    assert lib.qsac_graph_capture(ctx, C.byref(_args(k=128, dev_params=0x50000)), C.byref(g)) == Q.QSAC_ESTATE
    assert lib.qsac_graph_capture(ctx, C.byref(_args(k=128)), None) == Q.QSAC_ENULL
    assert lib.qsac_graph_launch(None) == Q.QSAC_ESTATE and lib.qsac_graph_free(None) == Q.QSAC_ESTATE
    st = Q.qsac_get_stats(ctx)
    assert st["steps"] == 2 and st["reuse_heads"] == 0
    Q.qsac_free(ctx)
    assert lib.qsac_free(None) == Q.QSAC_ESTATE
    assert lib.qsac_reset(None) == Q.QSAC_ESTATE


def test_strerror_and_stage_names(lib):
    for code in range(0, -8, -1):
        assert Q.qsac_strerror(code) != "unknown error"
    assert Q.qsac_strerror(-99) == "unknown error"
    n = lib.qsac_num_stages()
    assert n == 6 and lib.qsac_stage_name(n) is None
    assert [lib.qsac_stage_name(i) for i in range(n)] == [b"gate", b"score", b"select", b"fill", b"attn", b"combine"]


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2511_14510_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no other implementation", "")


def test_adaptive_thresholds_match_the_oracle_and_the_closed_forms(lib, oracle):
    import numpy as np
    rng = np.random.default_rng(0)
    for eta, p in ((0.8, 3.0), (0.5, 2.0), (-0.25, 1.0), (1.0, 3.0), (-1.0, 2.0)):
        s = np.concatenate([[0.0, 1.0, 0.5], rng.uniform(0, 1, 20)]).astype(np.float32)
        got = Q.qsac_adaptive_thresholds(list(s), eta, p)
        want = [oracle.adaptive_tau(float(x), float(np.float32(eta)), float(np.float32(p))) for x in s]
        assert np.allclose(got, want, rtol=0, atol=6e-8)
        assert got[1] == pytest.approx(eta, abs=6e-8) and got[0] == pytest.approx(-1.0, abs=6e-8)
    # the hand-derived fixture values
    gold = os.path.join(ROOT, "tests", "golden", "eq345_thresholds.txt")
    for line in open(gold):
        line = line.strip()
        if line and not line.startswith("#"):
            s_i, eta, p, want = [float(x) for x in line.split(";")[:4]]
            assert Q.qsac_adaptive_thresholds([s_i], eta, p)[0] == pytest.approx(want, abs=1e-6)
    for bad in (dict(importance=[1.5], eta=0.8, p=3), dict(importance=[0.5], eta=1.5, p=3),
                dict(importance=[0.5], eta=0.8, p=0), dict(importance=[-0.1], eta=0.8, p=3)):
        with pytest.raises(Q.QsacError):
            Q.qsac_adaptive_thresholds(**bad)


def test_reuse_difficulty_matches_the_oracle(lib, oracle):
    tau, sim = [0.8, 0.5, -0.2], [0.9, 0.6, 0.95]
    got = Q.qsac_reuse_difficulty(tau, sim, 0.1)
    import numpy as np
    f = lambda x: float(np.float32(x))
    want = [oracle.reuse_difficulty(f(t), f(s), f(0.1)) for t, s in zip(tau, sim)]
    assert np.allclose(got, want, atol=6e-8)
    with pytest.raises(Q.QsacError):
        Q.qsac_reuse_difficulty(tau, sim, 0.0)


def test_sink_recent_and_append_validation(lib):
    cfg = Q.make_config(1, 8, 2, 4096, 256, Q.QSAC_F16, Q.QSAC_FLAG_DRY_RUN, n_sink=4, n_recent=64, append_capacity=32)
    assert Q.qsac_workspace_layout(cfg).max_splits == (256 + 32 + 63) // 64
    ctx = Q.qsac_init(cfg)
    step = lambda a: lib.qsac_step(ctx, C.byref(a))
    assert step(_args(k=67)) == Q.QSAC_ERANGE                      # no room for the 68 persistent tokens
    assert step(_args(k=68)) == Q.QSAC_OK
    Q.qsac_reset(ctx)
    assert step(_args(n_app=33, K_app=0x30000, V_app=0x40000)) == Q.QSAC_ERANGE
    assert step(_args(n_app=5, K_app=None, V_app=0x40000)) == Q.QSAC_ENULL
    assert step(_args(n_app=5, K_app=0x30008, V_app=0x40000)) == Q.QSAC_EALIGN
    assert step(_args(n_app=32, K_app=0x30000, V_app=0x40000)) == Q.QSAC_OK
    Q.qsac_free(ctx)
    for kw in (dict(n_sink=-1), dict(n_sink=200, n_recent=100), dict(append_capacity=-5)):
        bad = Q.make_config(1, 8, 2, 4096, 256, Q.QSAC_F16, Q.QSAC_FLAG_DRY_RUN, **kw)
        assert Q.qsac_workspace_bytes(bad) == 0


def test_calibration_entry_points_validate_before_touching_a_device():
    # NULL and misaligned arguments are turned down on the host; nothing is launched
    lib = Q.load_calib()
    assert lib.qsac_calibration_copy(None, None, 256, None) == Q.QSAC_ENULL
    assert lib.qsac_calibration_read(None, 256, None, None) == Q.QSAC_ENULL
    assert lib.qsac_calibration_copy(4096, 8192, 24, None) == Q.QSAC_EALIGN      # size not a multiple of 16
    assert lib.qsac_calibration_read(4096 + 8, 256, 4096, None) == Q.QSAC_EALIGN  # source not 16-byte aligned
    assert lib.qsac_calibration_read(4096, 0, 4096, None) == Q.QSAC_OK           # nothing to read: no launch
