"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest

from paper_2512_17570_amd import gs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "gs.h")

FAKE = 0x10000          # non-null, 16-byte aligned; never dereferenced by a rejected call
# distinct, far-apart fake arrays (p, m, v, w, two gradient buffers, staged sum): a valid call must not alias
FP, FM, FV, FW, FG0, FG1, FACC = (FAKE + i * (1 << 24) for i in range(1, 8))
GOOD_HP = gs.HParams(step=3)


def declared_functions():
    src = open(HEADER).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    names = re.findall(r"\b(gs_[a-z0-9_]+)\s*\(", src)
    return sorted(set(names))


def test_header_symbols_all_exported():
    names = declared_functions()
    assert {"gs_grad_sqnorm", "gs_accum_adamw", "gs_stream_layer_step", "gs_sqnorm_workspace_bytes",
            "gs_stream_ctx_create_inplace", "gs_stream_ctx_create", "gs_stream_ctx_destroy", "gs_stream_ctx_sync", "gs_pinned_alloc",
            "gs_pinned_free", "gs_strerror", "gs_last_hip_error", "gs_grad_accum_sqnorm", "gs_adamw_from_acc",
            "gs_cu_stream_create", "gs_cu_stream_destroy", "gs_accum_adamw_oop", "gs_accum_adamw_spec",
            "gs_clip_coefficient", "gs_sqnorm_workspace_bytes_for", "gs_accum_add", "gs_acc_sqnorm",
            "gs_tier_ctx_create", "gs_tier_ctx_destroy", "gs_tier_ctx_sync", "gs_tier_ctx_error", "gs_tier_layer_step",
            "gs_stream_layer_step_range", "gs_tier_layer_step_range"} <= set(names)
    lib = ctypes.CDLL(gs.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in gs.h but not exported"


def test_binding_has_same_names():
    for n in declared_functions():
        assert hasattr(gs, n), n


def test_hparams_struct_layout_matches_header():
    assert ctypes.sizeof(gs.gs_adamw_hparams) == 28
    assert gs.gs_adamw_hparams.step.offset == 24
    assert gs.GS_MAX_K == int(re.search(r"#define\s+GS_MAX_K\s+(\d+)", open(HEADER).read()).group(1))


def test_strerror_and_workspace():
    assert gs.gs_strerror(gs.GS_OK) == "ok"
    for s in (gs.GS_ERR_INVALID_ARG, gs.GS_ERR_WORKSPACE, gs.GS_ERR_HIP, gs.GS_ERR_NOMEM):
        assert gs.gs_strerror(s) not in ("ok", "unknown status")
    assert gs.gs_strerror(-99) == "unknown status"
    assert gs.gs_sqnorm_workspace_bytes() >= 8 * 1024
    assert gs.gs_sqnorm_workspace_bytes() % 8 == 0


def _adamw(**kw):
    a = dict(p=FP, m=FM, v=FV, w_bf16=FW, grads=[FG0, FG1], begin=0, end=100, hp=GOOD_HP,
             d_sqnorm=None, stream=0, check=False)
    a.update(kw)
    return gs.gs_accum_adamw(**a)


@pytest.mark.parametrize("kw", [
    dict(p=None), dict(m=None), dict(v=None), dict(w_bf16=None),
    dict(p=FP + 4), dict(w_bf16=FW + 2), dict(m=FM + 8),
    dict(grads=None, k=2), dict(grads=[FAKE], k=0), dict(grads=[FAKE] * 33),
    dict(grads=[FAKE, None]), dict(grads=[FAKE, FAKE + 2]),
    dict(begin=-1), dict(begin=10, end=9),
    dict(hp=None),
    dict(hp=gs.HParams(step=0)), dict(hp=gs.HParams(step=-5)),
    dict(hp=gs.HParams(lr=-1.0, step=1)), dict(hp=gs.HParams(lr=float("nan"), step=1)),
    dict(hp=gs.HParams(beta1=1.0, step=1)), dict(hp=gs.HParams(beta1=-0.1, step=1)),
    dict(hp=gs.HParams(beta2=1.0, step=1)), dict(hp=gs.HParams(beta2=float("inf"), step=1)),
    dict(hp=gs.HParams(eps=-1e-8, step=1)), dict(hp=gs.HParams(weight_decay=-0.1, step=1)),
    dict(hp=gs.HParams(max_grad_norm=float("nan"), step=1)),
    dict(d_sqnorm=FAKE + 4),
])
def test_accum_adamw_rejects(kw):
    assert _adamw(**kw) == gs.GS_ERR_INVALID_ARG


def test_baseline_arguments_of_the_rejection_tests_are_valid():
    """The calls the rejection tests start from pass every check: without a GPU they get as far as
    the launch and come back as GS_ERR_HIP, so each rejection above is caused by the one argument
    that test changed."""
    assert _adamw() == gs.GS_ERR_HIP
    assert _sqnorm() == gs.GS_ERR_HIP
    assert gs.gs_last_hip_error() != ""


def test_accum_adamw_empty_range_is_ok_without_gpu():
    assert _adamw(begin=50, end=50) == gs.GS_OK
    assert _adamw(begin=0, end=0) == gs.GS_OK


def _sqnorm(**kw):
    a = dict(grads=[FAKE], begin=0, end=100, d_sqnorm=FAKE, d_workspace=FAKE,
             workspace_bytes=gs.gs_sqnorm_workspace_bytes(), accumulate=False, stream=0, check=False)
    a.update(kw)
    return gs.gs_grad_sqnorm(**a)


@pytest.mark.parametrize("kw,want", [
    (dict(grads=None, k=1), gs.GS_ERR_INVALID_ARG),
    (dict(grads=[FAKE] * 40), gs.GS_ERR_INVALID_ARG),
    (dict(grads=[FAKE + 6]), gs.GS_ERR_INVALID_ARG),
    (dict(begin=-3), gs.GS_ERR_INVALID_ARG),
    (dict(begin=5, end=4), gs.GS_ERR_INVALID_ARG),
    (dict(d_sqnorm=None), gs.GS_ERR_INVALID_ARG),
    (dict(d_sqnorm=FAKE + 4), gs.GS_ERR_INVALID_ARG),
    (dict(d_workspace=None), gs.GS_ERR_WORKSPACE),
    (dict(workspace_bytes=16), gs.GS_ERR_WORKSPACE),
    (dict(d_workspace=FAKE + 4), gs.GS_ERR_WORKSPACE),
])
def test_grad_sqnorm_rejects(kw, want):
    assert _sqnorm(**kw) == want


def test_grad_sqnorm_empty_accumulate_is_noop():
    assert _sqnorm(begin=7, end=7, accumulate=True) == gs.GS_OK


def test_grad_sqnorm_noalloc_rejects_without_gpu():
    ok = dict(grads=[FAKE], begin=0, end=100, d_sqnorm=FAKE, accumulate=False, stream=0, check=False)
    for kw, want in ((dict(grads=None, k=1), gs.GS_ERR_INVALID_ARG), (dict(grads=[FAKE] * 33), gs.GS_ERR_INVALID_ARG),
                     (dict(grads=[FAKE + 6]), gs.GS_ERR_INVALID_ARG), (dict(begin=-3), gs.GS_ERR_INVALID_ARG),
                     (dict(begin=5, end=4), gs.GS_ERR_INVALID_ARG), (dict(d_sqnorm=None), gs.GS_ERR_INVALID_ARG),
                     (dict(d_sqnorm=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(end=gs.GS_NOALLOC_MAX_ELEMS + 1), gs.GS_ERR_TOO_LARGE),
                     (dict(begin=7, end=8 + gs.GS_NOALLOC_MAX_ELEMS), gs.GS_ERR_TOO_LARGE)):
        assert gs.gs_grad_sqnorm_noalloc(**{**ok, **kw}) == want, kw
    assert gs.gs_grad_sqnorm_noalloc(**{**ok, "begin": 7, "end": 7, "accumulate": True}) == gs.GS_OK
    assert gs.gs_strerror(gs.GS_ERR_TOO_LARGE) not in ("ok", "unknown status")
    hdr = open(HEADER).read()
    assert gs.GS_NOALLOC_MAX_ELEMS == 1 << int(re.search(r"#define\s+GS_NOALLOC_MAX_ELEMS\s+\(\(int64_t\)1\s*<<\s*(\d+)\)", hdr).group(1))
    assert gs.GS_ERR_TOO_LARGE == int(re.search(r"GS_ERR_TOO_LARGE\s*=\s*(-\d+)", hdr).group(1))


def test_stream_api_rejects_without_gpu():
    st, ctx = gs.gs_stream_ctx_create_inplace(-1, check=False)
    assert st == gs.GS_ERR_INVALID_ARG and not ctx
    for chunk, slots in ((0, 2), (1024, 1), (1024, 65), ((1 << 34) + 1, 2)):
        st, ctx = gs.gs_stream_ctx_create(chunk, slots, check=False)
        assert st == gs.GS_ERR_INVALID_ARG and not ctx
    assert gs.gs_stream_ctx_sync(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_stream_ctx_destroy(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_stream_layer_step(None, FAKE, FAKE, FAKE, FAKE, [FAKE], 10, GOOD_HP, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_pinned_alloc(0) is None
    gs.gs_pinned_free(None)


def test_tier_api_rejects_without_gpu():
    for chunk, slots, cus in ((0, 2, 0), (1024, 1, 0), (1024, 65, 0), (-5, 3, 0), ((1 << 34) + 1, 2, 0), (1024, 2, -1)):
        st, ctx = gs.gs_tier_ctx_create(chunk, slots, cus, check=False)
        assert st == gs.GS_ERR_INVALID_ARG and not ctx
    assert gs.gs_tier_ctx_sync(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_tier_ctx_destroy(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_tier_ctx_error(None) == ""
    assert gs.gs_tier_layer_step(None, FAKE, FAKE, FAKE, 4, (3, 4, 5), (0, 0, 0), FAKE, [FAKE], 10, GOOD_HP,
                                 check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_strerror(gs.GS_ERR_IO) == "file read or write failed"
    assert gs.gs_tier_layer_step_range(None, FAKE, FAKE, FAKE, 4, (3, 4, 5), (0, 0, 0), FAKE, [FAKE], 10, 0, 10, GOOD_HP,
                                       check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_stream_layer_step_range(None, FAKE, FAKE, FAKE, FAKE, [FAKE], 0, 10, GOOD_HP,
                                         check=False) == gs.GS_ERR_INVALID_ARG


def test_accum_add_rejects_without_gpu():
    ws = gs.gs_sqnorm_workspace_bytes()
    ok = dict(acc_f32=FAKE, grad_bf16=FAKE, first=True, begin=0, end=64, d_sqnorm=FAKE, d_workspace=FAKE,
              workspace_bytes=ws, stream=0, check=False)
    for kw, want in ((dict(acc_f32=None), gs.GS_ERR_INVALID_ARG), (dict(acc_f32=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(grad_bf16=None), gs.GS_ERR_INVALID_ARG), (dict(grad_bf16=FAKE + 2), gs.GS_ERR_INVALID_ARG),
                     (dict(begin=9, end=3), gs.GS_ERR_INVALID_ARG), (dict(begin=-1), gs.GS_ERR_INVALID_ARG),
                     (dict(d_sqnorm=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(workspace_bytes=8), gs.GS_ERR_WORKSPACE), (dict(d_workspace=None), gs.GS_ERR_WORKSPACE)):
        assert gs.gs_accum_add(**{**ok, **kw}) == want
    # an empty range launches nothing: with no norm, or with a norm that is only added to
    assert gs.gs_accum_add(**{**ok, "begin": 5, "end": 5, "d_sqnorm": None, "d_workspace": None}) == gs.GS_OK
    assert gs.gs_accum_add(**{**ok, "begin": 5, "end": 5, "accumulate": True}) == gs.GS_OK


def test_acc_sqnorm_rejects_without_gpu():
    ws = gs.gs_sqnorm_workspace_bytes()
    ok = dict(acc_f32=FAKE, begin=0, end=64, d_sqnorm=FAKE, d_workspace=FAKE, workspace_bytes=ws, stream=0, check=False)
    for kw, want in ((dict(acc_f32=None), gs.GS_ERR_INVALID_ARG), (dict(acc_f32=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(begin=9, end=3), gs.GS_ERR_INVALID_ARG), (dict(begin=-1), gs.GS_ERR_INVALID_ARG),
                     (dict(d_sqnorm=None), gs.GS_ERR_INVALID_ARG), (dict(d_sqnorm=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(workspace_bytes=8), gs.GS_ERR_WORKSPACE), (dict(d_workspace=None), gs.GS_ERR_WORKSPACE)):
        assert gs.gs_acc_sqnorm(**{**ok, **kw}) == want
    assert gs.gs_acc_sqnorm(**{**ok, "begin": 5, "end": 5, "accumulate": True}) == gs.GS_OK


def test_staged_variant_rejects_without_gpu():
    ws = gs.gs_sqnorm_workspace_bytes()
    ok = dict(grads=[FAKE], begin=0, end=64, acc_f32=FAKE, d_sqnorm=FAKE, d_workspace=FAKE, workspace_bytes=ws,
              stream=0, check=False)
    for kw, want in ((dict(acc_f32=None), gs.GS_ERR_INVALID_ARG), (dict(acc_f32=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(grads=[FAKE] * 33), gs.GS_ERR_INVALID_ARG), (dict(begin=9, end=3), gs.GS_ERR_INVALID_ARG),
                     (dict(workspace_bytes=8), gs.GS_ERR_WORKSPACE), (dict(d_sqnorm=None), gs.GS_ERR_INVALID_ARG)):
        assert gs.gs_grad_accum_sqnorm(**{**ok, **kw}) == want
    assert gs.gs_grad_accum_sqnorm(**{**ok, "begin": 5, "end": 5, "accumulate": True}) == gs.GS_OK
    ok2 = dict(p=FP, m=FM, v=FV, w_bf16=FW, acc_f32=FACC, begin=0, end=64, hp=GOOD_HP, d_sqnorm=None,
               stream=0, check=False)
    for kw in (dict(acc_f32=None), dict(acc_f32=FACC + 8), dict(p=None), dict(hp=gs.HParams(step=0)),
               dict(begin=-1), dict(d_sqnorm=FAKE + 4)):
        assert gs.gs_adamw_from_acc(**{**ok2, **kw}) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_adamw_from_acc(**{**ok2, "begin": 7, "end": 7}) == gs.GS_OK


def test_speculative_and_oop_reject_without_gpu():
    ws = gs.gs_sqnorm_workspace_bytes()
    PO, MO, VO = (FACC + i * (1 << 24) for i in range(1, 4))
    oop = dict(p=FP, m=FM, v=FV, p_out=PO, m_out=MO, v_out=VO, w_bf16=FW, grads=[FG0], begin=0, end=64,
               hp=GOOD_HP, d_sqnorm=None, stream=0, check=False)
    assert gs.gs_accum_adamw_oop(**{**oop, "begin": 4, "end": 4}) == gs.GS_OK
    for kw in (dict(p_out=None), dict(m_out=FM + 4), dict(p_out=FP + 64),       # partial overlap with p
               dict(v_out=FV - 128), dict(grads=[FG0] * 33), dict(hp=None), dict(begin=5, end=1)):
        assert gs.gs_accum_adamw_oop(**{**oop, **kw}) == gs.GS_ERR_INVALID_ARG, kw
    assert gs.gs_accum_adamw_oop(**{**oop, "p_out": FP, "m_out": FM, "v_out": FV, "begin": 9, "end": 9}) == gs.GS_OK
    spec = dict(p=FP, m=FM, v=FV, p_out=PO, m_out=MO, v_out=VO, w_bf16=FW, grads=[FG0], begin=0, end=64,
                hp=GOOD_HP, d_sqnorm=FAKE, d_workspace=FAKE, workspace_bytes=ws, stream=0, check=False)
    for kw, want in ((dict(d_sqnorm=None), gs.GS_ERR_INVALID_ARG), (dict(d_sqnorm=FAKE + 4), gs.GS_ERR_INVALID_ARG),
                     (dict(d_workspace=None), gs.GS_ERR_WORKSPACE), (dict(workspace_bytes=64), gs.GS_ERR_WORKSPACE),
                     (dict(p_out=FP + 16), gs.GS_ERR_INVALID_ARG), (dict(v=None), gs.GS_ERR_INVALID_ARG)):
        assert gs.gs_accum_adamw_spec(**{**spec, **kw}) == want, kw
    assert gs.gs_accum_adamw_spec(**{**spec, "begin": 3, "end": 3, "accumulate": True}) == gs.GS_OK


def test_overlapping_inputs_and_outputs_are_rejected():
    """An output may be exactly its own input; any other overlap between an output and an input, or
    between two outputs, over the bytes of [begin,end) is refused before anything is enqueued."""
    n = 1000
    A, B, C, W, G, X = (FAKE + i * (1 << 20) for i in range(6))
    oop = dict(p=A, m=B, v=C, p_out=A, m_out=B, v_out=C, w_bf16=W, grads=[G], begin=0, end=n, hp=GOOD_HP,
               d_sqnorm=None, stream=0, check=False)
    ok_empty = {**oop, "begin": 5, "end": 5}
    assert gs.gs_accum_adamw_oop(**ok_empty) == gs.GS_OK
    bad = [dict(p_out=B),                     # p_out over m (an input that is not its own)
           dict(m_out=A, p_out=X),            # m_out over p
           dict(v_out=A + 64, p_out=X),       # v_out partly over p
           dict(w_bf16=A),                    # w over p
           dict(w_bf16=C + 2 * n),            # w over the upper half of v's bytes
           dict(p_out=X, m_out=X),            # two outputs on one array
           dict(p_out=X, w_bf16=X + 16),      # w inside p_out
           dict(grads=[A]),                   # a gradient buffer that is also a state being written
           dict(grads=[G, W]),                # a gradient buffer that is also w
           dict(p_out=G)]                     # p_out over a gradient buffer
    for kw in bad:
        assert gs.gs_accum_adamw_oop(**{**oop, **kw}) == gs.GS_ERR_INVALID_ARG, kw
        assert gs.gs_accum_adamw_oop(**{**oop, **kw, "begin": 5, "end": 5}) in (gs.GS_OK, gs.GS_ERR_INVALID_ARG)
    # ranges that do not touch each other are fine even when the arrays as a whole would overlap
    assert gs.gs_accum_adamw(p=A, m=A + 4 * n, v=A + 8 * n, w_bf16=A + 12 * n, grads=[G], begin=0, end=0, hp=GOOD_HP,
                             d_sqnorm=None, stream=0, check=False) == gs.GS_OK
    # in place through the plain entry point, and the staged one with acc over a state
    assert _adamw(p=A, m=B, v=C, w_bf16=W, grads=[G, G + (1 << 19)], begin=3, end=3) == gs.GS_OK
    assert _adamw(p=A, m=A, v=C, w_bf16=W, grads=[G], end=n) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_adamw_from_acc(p=A, m=B, v=C, w_bf16=W, acc_f32=B, begin=0, end=n, hp=GOOD_HP, d_sqnorm=None, stream=0,
                                check=False) == gs.GS_ERR_INVALID_ARG


def test_host_clip_coefficient_matches_oracle():
    from oracle import gs_oracle as O
    for S, mx in ((0.0, 1.0), (0.25, 1.0), (1.0, 1.0), (4.0, 1.0), (3221.8, 1.0), (1e12, 0.5), (7.0, 0.0), (7.0, -1.0),
                  (float("inf"), 1.0), (float("nan"), 1.0), (1e-30, 1e-3), (0.99999, 1.0), (1.00001, 1.0)):
        assert gs.gs_clip_coefficient(S, mx) == O.clip_coef(S, mx), (S, mx)


def test_workspace_size_for_range():
    base = gs.gs_sqnorm_workspace_bytes()
    assert gs.gs_sqnorm_workspace_bytes_for(0) == base and gs.gs_sqnorm_workspace_bytes_for(-5) == base
    assert gs.gs_sqnorm_workspace_bytes_for(1 << 20) == base
    big = gs.gs_sqnorm_workspace_bytes_for(805_412_864)
    assert big > base and big % 8 == 0 and 805_412_864 // 32 <= big <= 805_412_864 // 32 + 4096    # a double per 256 elements
    assert gs.gs_sqnorm_workspace_bytes_for(1 << 34) > big


def test_cu_stream_rejects_without_gpu():
    st, s = gs.gs_cu_stream_create(0, check=False)
    assert st == gs.GS_ERR_INVALID_ARG and not s
    st, s = gs.gs_cu_stream_create(-4, check=False)
    assert st == gs.GS_ERR_INVALID_ARG and not s
    assert gs.gs_cu_stream_destroy(None, check=False) == gs.GS_ERR_INVALID_ARG


def test_defer_api_rejects_without_gpu():
    for layers, cus in ((0, 0), (-3, 0), (65537, 0), (4, -1)):
        st, ctx = gs.gs_defer_ctx_create(layers, cus, check=False)
        assert st == gs.GS_ERR_INVALID_ARG and not ctx
    assert gs.gs_defer_ctx_sync(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_defer_ctx_destroy(None, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_defer_wait_layer(None, 0, 0, check=False) == gs.GS_ERR_INVALID_ARG
    assert gs.gs_defer_layer_done(None, 0) == -1
    assert gs.gs_defer_layer_step(None, 0, FP, FM, FV, FW, [FG0], 0, 10, GOOD_HP, producer_stream=0,
                                  check=False) == gs.GS_ERR_INVALID_ARG


def test_error_raises_through_binding():
    with pytest.raises(gs.GsError) as ei:
        _adamw(begin=3, end=2, check=True)
    assert ei.value.status == gs.GS_ERR_INVALID_ARG


def test_header_is_plain_c_and_cxx(tmp_path):
    """include/gs.h must be usable from a C99 translation unit (and from C++) on its own."""
    import subprocess
    c = tmp_path / "use_gs.c"
    c.write_text('#include "gs.h"\n'
                 'int probe(void) { gs_adamw_hparams hp = {1e-4f, 0.9f, 0.999f, 1e-8f, 0.01f, 1.0f, 1};\n'
                 '  const char *(*f)(gs_status) = gs_strerror; (void)f;\n'
                 '  return (int)sizeof(hp) + (int)GS_MAX_K + (int)GS_ERR_NOMEM; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", inc, "-fsyntax-only", str(c)], check=True)
    cxx = tmp_path / "use_gs.cpp"
    cxx.write_text(c.read_text())
    subprocess.run(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-I", inc, "-fsyntax-only", str(cxx)], check=True)
