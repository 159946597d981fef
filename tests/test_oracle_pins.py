"""Pins for the CPU oracle: it is checked against things other than itself --
closed forms, torch's own AdamW / clip_grad_norm_ / bf16 cast (library routines evaluated in
fp64 or bit-exactly), an independently written brute-force loop, and invariants the paper
states (element-wise => any partition gives the same result, Sec. 2.2 / Sec. 4.4 / Sec. 6.5;
gradients of all micro-batches are summed in full precision, Sec. 2.1).
"""
import math
import struct

import numpy as np
import pytest
import torch

from oracle import gs_oracle as O
from paper_2512_17570_amd import inputs as I


# ----------------------------------------------------------------------------- helpers
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Decode bf16 bit patterns with torch's own bf16 type (library decode, not the oracle's)."""
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16)
    return t.to(torch.float64).numpy()


def rand_case(n, k, seed, sigma=1e-3, outlier_frac=0.0):
    p, m, v = I.make_states(n, seed)
    g = I.make_grads(n, k, sigma, seed, outlier_frac=outlier_frac)
    return (p.numpy().copy(), m.numpy().copy(), v.numpy().copy(), [I.bf16_bits(x).copy() for x in g])


def ulp_diff_f32(a: np.ndarray, b: np.ndarray) -> np.ndarray:
    """Distance in units of fp32 representable values (monotone integer mapping)."""
    def key(x):
        i = x.astype(np.float32).view(np.int32).astype(np.int64)
        return np.where(i < 0, -(i & 0x7FFFFFFF), i)
    return np.abs(key(a) - key(b))


def f64_to_f32_ulps(truth: np.ndarray, got: np.ndarray, scale=None) -> np.ndarray:
    """|got - truth| in units of the fp32 spacing at truth (or at `scale` where that is larger:
    p' = p*decay - step is a difference, so its rounding error is set by the larger operand)."""
    t32 = truth.astype(np.float32)
    if scale is not None:      # scale = old p: operands of the difference are ~|p| and ~|p' - p|
        t32 = np.maximum(np.abs(t32), np.maximum(np.abs(scale), np.abs(truth - scale)).astype(np.float32))
    spacing = np.spacing(np.abs(t32)).astype(np.float64)
    return np.abs(got.astype(np.float64) - truth) / spacing


# ----------------------------------------------------------------------------- a6: bf16 RNE
def f32_from_bits(u):
    return struct.unpack("<f", struct.pack("<I", u))[0]


@pytest.mark.parametrize("bits,expect", [
    (0x3F800000, 0x3F80),            # 1.0 exact
    (0x3F808000, 0x3F80),            # tie, kept lsb even  -> stays
    (0x3F818000, 0x3F82),            # tie, kept lsb odd   -> rounds up to even
    (0x3F808001, 0x3F81),            # just above tie      -> up
    (0x3F807FFF, 0x3F80),            # just below tie      -> down
    (0x3F7F8000, 0x3F80),            # tie that carries into the exponent (0x3F7F odd)
    (0x00000000, 0x0000),            # +0
    (0x80000000, 0x8000),            # -0
    (0x7F800000, 0x7F80),            # +Inf
    (0xFF800000, 0xFF80),            # -Inf
    (0x7F7FFFFF, 0x7F80),            # largest finite fp32 rounds to +Inf
    (0x7F7F7FFF, 0x7F7F),            # just below the tie under bf16 max stays finite
    (0x00008000, 0x0000),            # subnormal tie to even (0)
    (0x00018000, 0x0002),            # subnormal tie to even (up)
    (0xBF818000, 0xBF82),            # negative tie
])
def test_bf16_rne_hand_cases(bits, expect):
    assert O.f32_to_bf16(f32_from_bits(bits)) == expect


def test_bf16_nan_stays_nan():
    for bits in (0x7FC00000, 0x7F800001, 0xFFC12345, 0x7F80FFFF):
        h = O.f32_to_bf16(np.array([bits], dtype=np.uint32).view(np.float32)[0])
        assert (h & 0x7F80) == 0x7F80 and (h & 0x007F) != 0, hex(h)


def test_bf16_rne_matches_torch_cast():
    rng = np.random.default_rng(1)
    bits = rng.integers(0, 2**32, size=200_000, dtype=np.uint64).astype(np.uint32)
    x = bits.view(np.float32)
    x = x[np.isfinite(x)]
    want = I.bf16_bits(torch.from_numpy(x.copy()).to(torch.bfloat16))
    got = np.array([O.f32_to_bf16(val) for val in x[:50_000]], dtype=np.uint16)
    assert np.array_equal(got, want[:50_000])


def test_bf16_decode_matches_torch():
    bits = np.arange(0, 65536, dtype=np.uint32).astype(np.uint16)
    want = bf16_bits_to_f64(bits)
    got = np.array([O.bf16_to_f32(int(b)) for b in bits], dtype=np.float64)
    fin = np.isfinite(want)
    assert np.array_equal(got[fin], want[fin])
    assert np.array_equal(np.isnan(got), np.isnan(want))


# ----------------------------------------------------------------------------- a2: squared norm
def test_sqnorm_all_ones_exact():
    n, k = 1000, 5
    ones = np.full(n, 0x3F80, dtype=np.uint16)
    assert O.grad_sqnorm([ones] * k) == float(k * k * n)


def test_sqnorm_power_of_two_pattern_exact():
    # g_0 = +2^-3 everywhere, g_1 alternates +-2^-4  => a alternates 3/16, 1/16
    n = 4096
    g0 = np.full(n, 0x3E00, dtype=np.uint16)                    # 0.125
    g1 = np.where(np.arange(n) % 2 == 0, 0x3D80, 0xBD80).astype(np.uint16)   # +-0.0625
    want = (n // 2) * ((3 / 16) ** 2 + (1 / 16) ** 2)
    assert O.grad_sqnorm([g0, g1]) == want


def test_sqnorm_range_and_additivity():
    _, _, _, g = rand_case(5000, 3, seed=3)
    full = O.grad_sqnorm(g)
    parts = O.grad_sqnorm(g, 0, 1237) + O.grad_sqnorm(g, 1237, 5000)
    assert math.isclose(full, parts, rel_tol=1e-14)
    assert O.grad_sqnorm(g, 17, 17) == 0.0


def test_sqnorm_matches_numpy_dot_of_sum():
    _, _, _, g = rand_case(100_000, 8, seed=4)
    a = np.zeros(100_000)
    for b in g:
        a += bf16_bits_to_f64(b)          # exact in fp64; fp32 sum of 8 bf16 values rounds at most 2^-24 rel.
    want = float(np.dot(a, a))
    assert math.isclose(O.grad_sqnorm(g), want, rel_tol=1e-6)


def test_sqnorm_statistics_of_workload0():
    # E[S] = n k sigma^2 for the small GPT workload's distribution (sanity of scale, not of bits)
    n, k, sigma = 1 << 20, 4, 1e-3
    _, _, _, g = rand_case(n, k, seed=0, sigma=sigma)
    S = O.grad_sqnorm(g)
    assert abs(S / (n * k * sigma ** 2) - 1.0) < 0.02


# ----------------------------------------------------------------------------- a3: clip coefficient
def test_clip_coef_against_torch_clip_grad_norm():
    for scale in (0.01, 0.5, 3.0, 250.0):
        gvec = torch.linspace(-1, 1, 101, dtype=torch.float64) * scale
        prm = torch.nn.Parameter(torch.zeros(101, dtype=torch.float64))
        prm.grad = gvec.clone()
        torch.nn.utils.clip_grad_norm_([prm], max_norm=1.0)
        ratio = (prm.grad / gvec)[gvec != 0]
        S = float((gvec * gvec).sum())
        c = O.clip_coef(S, 1.0)
        assert abs(c - float(ratio[0])) <= 2e-7 * max(1.0, abs(c))
        assert c <= 1.0


def test_clip_coef_disabled_and_edges():
    assert O.clip_coef(1e12, 0.0) == 1.0
    assert O.clip_coef(1e12, -1.0) == 1.0
    assert O.clip_coef(0.0, 1.0) == 1.0
    assert O.clip_coef(float("inf"), 1.0) == 0.0
    assert O.clip_coef(float("nan"), 1.0) == 1.0
    # norm exactly 2*max_norm -> c = 1/(2+1e-6) in fp32
    c = O.clip_coef(4.0, 1.0)
    assert c == np.float32(1.0) / (np.float32(2.0) + np.float32(1e-6))


# ----------------------------------------------------------------------------- a4-a6: element update
def test_first_step_zero_moments_closed_form():
    """t=1, m=v=0, no clipping:  p' = p(1-lr wd) - lr g/(|g|+eps); m' = (1-b1) g; v' = (1-b2) g^2."""
    n, k = 4096, 3
    p, _, _, g = rand_case(n, k, seed=5)
    m = np.zeros(n, np.float32); v = np.zeros(n, np.float32); w = np.zeros(n, np.uint16)
    hp = O.HParams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.1, max_grad_norm=0.0, step=1)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    lr, wd, eps = map(lambda x: float(np.float32(x)), (hp.lr, hp.weight_decay, hp.eps))
    b1, b2 = float(np.float32(hp.beta1)), float(np.float32(hp.beta2))
    want_p = p.astype(np.float64) * (1 - lr * wd) - lr * gs / (np.abs(gs) + eps)
    want_m = (1 - b1) * gs
    want_v = (1 - b2) * gs * gs
    tp, tm, tv = O.accum_adamw_f64(p, m, v, g, hp)
    assert np.allclose(tp, want_p, rtol=1e-11, atol=0)
    assert np.allclose(tm, want_m, rtol=1e-12, atol=0)
    assert np.allclose(tv, want_v, rtol=1e-12, atol=0)
    p2 = p.copy()
    O.accum_adamw(p2, m, v, w, g, hp, 1.0)
    # |update| = lr(1 +- tiny): sign(g) recovered
    nz = np.abs(gs) > 1e-4
    assert np.allclose((p.astype(np.float64) * (1 - lr * wd) - p2)[nz], lr * np.sign(gs)[nz], rtol=2e-3)
    assert f64_to_f32_ulps(want_p, p2, scale=p).max() <= 2.0
    assert f64_to_f32_ulps(want_m, m).max() <= 2.0
    assert f64_to_f32_ulps(want_v, v).max() <= 2.0


def _torch_adamw_f64(p, m, v, gsum, hp, nsteps=1):
    """torch.optim.AdamW in fp64, state preset so that its next step is step hp.step."""
    prm = torch.nn.Parameter(torch.from_numpy(p.astype(np.float64)))
    f = lambda x: float(np.float32(x))
    opt = torch.optim.AdamW([prm], lr=f(hp.lr), betas=(f(hp.beta1), f(hp.beta2)), eps=f(hp.eps),
                            weight_decay=f(hp.weight_decay), foreach=False)
    opt.state[prm] = {"step": torch.tensor(float(hp.step - 1)),
                      "exp_avg": torch.from_numpy(m.astype(np.float64)),
                      "exp_avg_sq": torch.from_numpy(v.astype(np.float64))}
    for _ in range(nsteps):
        prm.grad = torch.from_numpy(gsum.copy())
        opt.step()
    st = opt.state[prm]
    return prm.detach().numpy(), st["exp_avg"].numpy(), st["exp_avg_sq"].numpy()


@pytest.mark.parametrize("step", [1, 2, 10, 100, 5000])
def test_truth_matches_torch_adamw_fp64(step):
    n, k = 3000, 4
    p, m, v, g = rand_case(n, k, seed=6 + step)
    hp = O.HParams(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.01, max_grad_norm=0.0, step=step)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    wp, wm, wv = _torch_adamw_f64(p, m, v, gs, hp)
    tp, tm, tv = O.accum_adamw_f64(p, m, v, g, hp)
    assert np.allclose(tp, wp, rtol=1e-12, atol=1e-18)
    assert np.allclose(tm, wm, rtol=1e-12, atol=1e-18)
    assert np.allclose(tv, wv, rtol=1e-12, atol=1e-24)


@pytest.mark.parametrize("step", [1, 10, 100])
def test_fp32_oracle_within_ulps_of_torch_fp64(step):
    n, k = 20000, 8
    p, m, v, g = rand_case(n, k, seed=20 + step)
    hp = O.HParams(step=step, max_grad_norm=0.0)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    wp, wm, wv = _torch_adamw_f64(p, m, v, gs, hp)
    w = np.zeros(n, np.uint16)
    p0, m0 = p.copy(), m.copy()
    O.accum_adamw(p, m, v, w, g, hp, 1.0)
    # fp32 evaluation of ~10 roundings: a few ulp of the result, or 1e-6 relative
    for got, want, sc in ((p, wp, p0), (m, wm, m0), (v, wv, None)):
        ul = f64_to_f32_ulps(want, got, sc)
        rel = np.abs(got - want) / np.maximum(np.abs(want), 1e-30)
        assert np.all((ul <= 4.0) | (rel <= 1e-6)), (ul.max(), rel.max())


def test_clipped_step_matches_torch_clip_then_adamw():
    n, k = 5000, 4
    p, m, v, g = rand_case(n, k, seed=31, sigma=1e-2)
    hp = O.HParams(step=7, max_grad_norm=0.5)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    prm = torch.nn.Parameter(torch.zeros(n, dtype=torch.float64))
    prm.grad = torch.from_numpy(gs.copy())
    total = torch.nn.utils.clip_grad_norm_([prm], max_norm=float(np.float32(0.5)))
    assert float(total) > 0.5                     # clipping is active in this case
    wp, wm, wv = _torch_adamw_f64(p, m, v, prm.grad.numpy(), hp)
    S = O.grad_sqnorm(g)
    assert math.isclose(S, float(total) ** 2, rel_tol=1e-6)
    tp, tm, tv = O.accum_adamw_f64(p, m, v, g, hp, sqnorm_total=S)
    assert np.allclose(tp, wp, rtol=1e-9, atol=1e-15)
    assert np.allclose(tm, wm, rtol=1e-9, atol=1e-15)
    w = np.zeros(n, np.uint16)
    p0, m0 = p.copy(), m.copy()
    O.accum_adamw(p, m, v, w, g, hp, O.clip_coef(S, hp.max_grad_norm))
    for got, want, sc in ((p, wp, p0), (m, wm, m0), (v, wv, None)):
        ul = f64_to_f32_ulps(want, got, sc)
        rel = np.abs(got - want) / np.maximum(np.abs(want), 1e-30)
        assert np.all((ul <= 4.0) | (rel <= 1e-6)), (ul.max(), rel.max())


def test_multi_step_trajectory_matches_torch_fp64():
    n, k = 2000, 2
    p, m, v, g = rand_case(n, k, seed=40)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    hp0 = O.HParams(step=3, max_grad_norm=0.0)
    wp, wm, wv = _torch_adamw_f64(p, m, v, gs, hp0, nsteps=5)
    w = np.zeros(n, np.uint16)
    for s in range(5):
        O.accum_adamw(p, m, v, w, g, O.HParams(step=3 + s, max_grad_norm=0.0), 1.0)
    assert np.allclose(p, wp, rtol=2e-6, atol=1e-9)
    assert np.allclose(m, wm, rtol=2e-6, atol=1e-9)
    assert np.allclose(v, wv, rtol=2e-6, atol=1e-15)


def test_brute_force_small_n_independent_loop():
    """n <= 64, pure-Python doubles, a different grouping: p - lr*(mhat/(sqrt(vhat)+eps) + wd*p)."""
    n, k = 61, 5
    p, m, v, g = rand_case(n, k, seed=50, sigma=3e-3)
    hp = O.HParams(lr=2e-3, beta1=0.8, beta2=0.99, eps=1e-6, weight_decay=0.05, max_grad_norm=0.01, step=4)
    lr, b1, b2, eps, wd, mx = (float(np.float32(x)) for x in
                               (hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, hp.max_grad_norm))
    gdec = [bf16_bits_to_f64(b) for b in g]
    acc = [sum(float(gdec[j][i]) for j in range(k)) for i in range(n)]
    S = math.fsum(a * a for a in acc)
    norm = math.sqrt(S)
    assert norm > mx
    c = min(1.0, mx / (norm + 1e-6))
    exp_p, exp_m, exp_v = [], [], []
    for i in range(n):
        gi = acc[i] * c
        mi = float(m[i]) + (1 - b1) * (gi - float(m[i]))
        vi = b2 * float(v[i]) + (1 - b2) * gi * gi
        mhat = mi / (1 - b1 ** hp.step)
        vhat = vi / (1 - b2 ** hp.step)
        pi = float(p[i])
        exp_p.append(pi - lr * (mhat / (math.sqrt(vhat) + eps) + wd * pi))
        exp_m.append(mi); exp_v.append(vi)
    exp_p, exp_m, exp_v = map(np.array, (exp_p, exp_m, exp_v))
    assert math.isclose(O.grad_sqnorm(g), S, rel_tol=1e-6)
    tp, tm, tv = O.accum_adamw_f64(p, m, v, g, hp, sqnorm_total=S)
    assert np.allclose(tp, exp_p, rtol=1e-12) and np.allclose(tm, exp_m, rtol=1e-12) and np.allclose(tv, exp_v, rtol=1e-12)
    w = np.zeros(n, np.uint16)
    p0, m0 = p.copy(), m.copy()
    O.accum_adamw(p, m, v, w, g, hp, O.clip_coef(O.grad_sqnorm(g), hp.max_grad_norm))
    for got, want, sc in ((p, exp_p, p0), (m, exp_m, m0), (v, exp_v, None)):
        ul = f64_to_f32_ulps(want, got, sc)
        rel = np.abs(got - want) / np.maximum(np.abs(want), 1e-30)
        assert np.all((ul <= 4.0) | (rel <= 1e-6)), (ul.max(), rel.max())
    # a6: w is the RNE bf16 of the new master weight (torch's cast as the independent rounding)
    assert np.array_equal(w, I.bf16_bits(torch.from_numpy(p.copy()).to(torch.bfloat16)))


# ----------------------------------------------------------------------------- a1: accumulation
def test_k_buffers_equal_one_step_on_their_sum():
    """Small integers x 2^-10 so that the sum of k buffers is itself a bf16 value."""
    n, k = 3001, 6
    rng = np.random.default_rng(7)
    ints = rng.integers(-10, 11, size=(k, n))               # |sum| <= 60 < 2^8: exact in bf16
    gk = [I.bf16_bits(torch.from_numpy(ints[j] * 2.0 ** -10).to(torch.bfloat16)) for j in range(k)]
    g1 = [I.bf16_bits(torch.from_numpy(ints.sum(0) * 2.0 ** -10).to(torch.bfloat16))]
    assert np.array_equal(bf16_bits_to_f64(g1[0]), ints.sum(0) * 2.0 ** -10)
    p, m, v, _ = rand_case(n, 1, seed=8)
    hp = O.HParams(step=12, max_grad_norm=0.0)
    pa, ma, va, wa = p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)
    pb, mb, vb, wb = p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)
    O.accum_adamw(pa, ma, va, wa, gk, hp, 1.0)
    O.accum_adamw(pb, mb, vb, wb, g1, hp, 1.0)
    assert np.array_equal(pa, pb) and np.array_equal(ma, mb) and np.array_equal(va, vb) and np.array_equal(wa, wb)
    assert O.grad_sqnorm(gk) == O.grad_sqnorm(g1)


def test_accumulate_matches_sequential_float32_adds_and_exact_sum():
    """a1 on its own: equal to numpy float32 adds in the same order (library arithmetic), and to
    the exact (fp64) sum whenever that sum is representable in fp32."""
    n, k = 10_000, 7
    _, _, _, g = rand_case(n, k, seed=70, sigma=1e-2)
    want = np.zeros(n, np.float32)
    for b in g:
        want = (want + bf16_bits_to_f64(b).astype(np.float32)).astype(np.float32)
    got = O.accumulate(g)
    assert np.array_equal(got, want)
    exact = sum(bf16_bits_to_f64(b) for b in g)
    assert np.allclose(got, exact, rtol=4e-7, atol=0)
    rep = exact.astype(np.float32).astype(np.float64) == exact
    assert rep.sum() > n // 4 and np.array_equal(got[rep].astype(np.float64), exact[rep])
    part = O.accumulate(g, 100, 200)
    assert np.array_equal(part[100:200], want[100:200]) and not part[:100].any() and not part[200:].any()
    assert math.isclose(float(np.dot(got.astype(np.float64), got.astype(np.float64))), O.grad_sqnorm(g), rel_tol=1e-12)


def test_accum_add_one_micro_batch_at_a_time():
    """As-you-go accumulation: each call equals a numpy float32 add of the widened buffer
    (library arithmetic); k calls in order reproduce the k-way sum; the returned value is the
    squared norm of the updated range; `first` ignores what the buffer held; elements outside
    the range are untouched."""
    n, k = 5_000, 5
    _, _, _, g = rand_case(n, k, seed=71, sigma=1e-2)
    acc = np.full(n, np.float32(np.nan))            # garbage that `first` must ignore
    want = np.zeros(n, np.float32)
    for j, b in enumerate(g):
        S = O.accum_add(acc, b, first=(j == 0))
        want = (want + bf16_bits_to_f64(b).astype(np.float32)).astype(np.float32)
        assert np.array_equal(acc, want)
        assert math.isclose(S, float(np.dot(want.astype(np.float64), want.astype(np.float64))), rel_tol=1e-12)
    assert np.array_equal(acc, O.accumulate(g))
    # a range: only [lo,hi) moves, and the returned norm covers only that range
    before = acc.copy()
    S = O.accum_add(acc, g[0], first=False, begin=123, end=457)
    assert np.array_equal(acc[:123], before[:123]) and np.array_equal(acc[457:], before[457:])
    mid = (before[123:457] + bf16_bits_to_f64(g[0][123:457]).astype(np.float32)).astype(np.float32)
    assert np.array_equal(acc[123:457], mid)
    assert math.isclose(S, float(np.dot(mid.astype(np.float64), mid.astype(np.float64))), rel_tol=1e-12)
    # -0 inputs: +0 + (-0) is +0, so the buffer never holds a negative zero after `first`
    z = np.zeros(4, np.float32)
    O.accum_add(z, np.full(4, 0x8000, np.uint16), first=True)
    assert not np.signbit(z).any()
    assert O.accum_add(z, np.zeros(4, np.uint16), first=True, begin=2, end=2) == 0.0


def test_acc_sqnorm_of_a_finished_buffer():
    """Norm of an fp32 buffer: numpy's fp64 dot (library routine), the closed form of a constant
    buffer, additivity over ranges, and agreement with the norm computed from the k bf16 buffers."""
    n, k = 20_000, 3
    _, _, _, g = rand_case(n, k, seed=72, sigma=1e-2)
    acc = O.accumulate(g)
    a64 = acc.astype(np.float64)
    assert math.isclose(O.acc_sqnorm(acc), float(np.dot(a64, a64)), rel_tol=1e-13)
    assert math.isclose(O.acc_sqnorm(acc), O.grad_sqnorm(g), rel_tol=1e-13)
    assert math.isclose(O.acc_sqnorm(acc, 0, 777) + O.acc_sqnorm(acc, 777, n), O.acc_sqnorm(acc), rel_tol=1e-13)
    assert O.acc_sqnorm(acc, 5, 5) == 0.0
    assert O.acc_sqnorm(np.full(4096, np.float32(-0.25))) == 4096 * 0.0625
    assert math.isclose(O.acc_sqnorm(acc, 123, 124), float(a64[123] ** 2), rel_tol=1e-15)


def test_sum_not_mean():
    n = 256
    one = np.full(n, 0x3C00, dtype=np.uint16)       # 2^-7
    hp = O.HParams(step=1, max_grad_norm=0.0, weight_decay=0.0)
    z = lambda: np.zeros(n, np.float32)
    m4, m1 = z(), z()
    O.accum_adamw(z(), m4, z(), np.zeros(n, np.uint16), [one] * 4, hp, 1.0)
    O.accum_adamw(z(), m1, z(), np.zeros(n, np.uint16), [one], hp, 1.0)
    assert np.allclose(m4, 4 * m1, rtol=1e-6)


# ----------------------------------------------------------------------------- a7: split == full
@pytest.mark.parametrize("n", [64, 1000, 4099])
def test_split_equals_full_bitwise(n):
    k = 3
    p, m, v, g = rand_case(n, k, seed=9)
    hp = O.HParams(step=10)
    c = O.clip_coef(O.grad_sqnorm(g), hp.max_grad_norm)
    full = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    O.accum_adamw(*full, g, hp, c)
    for s in sorted({0, 1, 7, 8, 9, n // 2 - 1, n // 2 + 1, n - 1, n, int(0.4 * n)}):
        part = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
        O.accum_adamw(*part, g, hp, c, 0, s)
        O.accum_adamw(*part, g, hp, c, s, n)
        for a, b in zip(full, part):
            assert np.array_equal(a, b), s


def test_range_leaves_outside_untouched():
    n = 500
    p, m, v, g = rand_case(n, 2, seed=10)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    w = np.full(n, 0xABCD, np.uint16)
    O.accum_adamw(p, m, v, w, g, O.HParams(step=2), 1.0, 100, 200)
    for a, b in ((p, p0), (m, m0), (v, v0)):
        assert np.array_equal(a[:100], b[:100]) and np.array_equal(a[200:], b[200:])
        assert not np.array_equal(a[100:200], b[100:200])
    assert np.all(w[:100] == 0xABCD) and np.all(w[200:] == 0xABCD)


# ----------------------------------------------------------------------------- special hyper-parameters
def test_lr_zero_keeps_p_but_moments_advance():
    n = 777
    p, m, v, g = rand_case(n, 2, seed=11)
    p0, m0, v0 = p.copy(), m.copy(), v.copy()
    O.accum_adamw(p, m, v, np.zeros(n, np.uint16), g, O.HParams(lr=0.0, weight_decay=0.0, step=3, max_grad_norm=0.0), 1.0)
    assert np.array_equal(p, p0)
    assert not np.array_equal(m, m0) and not np.array_equal(v, v0)


def test_zero_betas_reduce_to_sign_like_update_for_every_t():
    n = 512
    p, m, v, g = rand_case(n, 2, seed=12)
    gs = sum(bf16_bits_to_f64(b) for b in g)
    for t in (1, 5, 1000):
        hp = O.HParams(lr=1e-3, beta1=0.0, beta2=0.0, eps=1e-8, weight_decay=0.02, max_grad_norm=0.0, step=t)
        lr, wd, eps = (float(np.float32(x)) for x in (hp.lr, hp.weight_decay, hp.eps))
        want = p.astype(np.float64) * (1 - lr * wd) - lr * gs / (np.abs(gs) + eps)
        tp, _, _ = O.accum_adamw_f64(p, m, v, g, hp)
        assert np.allclose(tp, want, rtol=1e-11)


def test_clip_inactive_equals_unclipped_and_power_of_two_clip():
    n, k = 1024, 2
    p, m, v, _ = rand_case(n, k, seed=13)
    # all-equal gradients 2^-4 each, k=2: a = 2^-3, norm = sqrt(n)*2^-3 = 4  (n = 1024)
    g = [np.full(n, 0x3D80, np.uint16)] * k
    S = O.grad_sqnorm(g)
    assert S == 16.0
    # inactive: max_norm well above the norm
    hp_hi = O.HParams(step=5, max_grad_norm=8.0)
    a = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    b = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    O.accum_adamw(*a, g, hp_hi, O.clip_coef(S, 8.0))
    O.accum_adamw(*b, g, O.HParams(step=5, max_grad_norm=0.0), 1.0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)
    # active with max_norm = 2 -> c = 2/(4+1e-6) ~ 0.5: equals an unclipped step on half gradients
    # up to the 1e-6 in the denominator (relative 2.5e-7 on g)
    c = O.clip_coef(S, 2.0)
    assert abs(c - 0.5) < 2e-7
    half = [np.full(n, 0x3D00, np.uint16)] * k           # 2^-5 each
    tp_c, tm_c, tv_c = O.accum_adamw_f64(p, m, v, g, O.HParams(step=5, max_grad_norm=2.0), sqnorm_total=S)
    tp_h, tm_h, tv_h = O.accum_adamw_f64(p, m, v, half, O.HParams(step=5, max_grad_norm=0.0))
    assert np.allclose(tm_c, tm_h, rtol=1e-6) and np.allclose(tv_c, tv_h, rtol=1e-6)
    assert np.allclose(tp_c, tp_h, rtol=1e-6, atol=1e-9)


# ----------------------------------------------------------------------------- resume
def test_step_dump_reload_step_equals_two_steps():
    n = 999
    p, m, v, g = rand_case(n, 3, seed=14)
    a = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    O.accum_adamw(*a, g, O.HParams(step=1), 1.0)
    dumped = [x.tobytes() for x in a[:3]]
    O.accum_adamw(*a, g, O.HParams(step=2), 1.0)
    b = [np.frombuffer(d, dtype=np.float32).copy() for d in dumped] + [np.zeros(n, np.uint16)]
    O.accum_adamw(*b, g, O.HParams(step=2), 1.0)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


def test_fp32_oracle_meets_stated_tolerance_of_fp64_wherever_the_update_does_not_cancel():
    """4 fp32 ulp or 1e-6 relative to the fp64 evaluation, asserted on every element whose final add
    does not cancel (89-100 % of them on these distributions); the operand-aware bound only
    on the rest.  Three value regimes: the small layer, hard clipping with outliers, k = 16."""
    from tolerances import f64_truth_check
    for n, k, sigma, frac, step in ((300_007, 4, 1e-3, 0.0, 10), (200_003, 8, 1e-3, 1e-3, 100), (150_001, 16, 5e-4, 0.0, 100)):
        p, m, v, g = rand_case(n, k, seed=77 + k, sigma=sigma, outlier_frac=frac)
        hp = O.HParams(1e-4, 0.9, 0.999, 1e-8, 0.01, 1.0, step)
        S = O.grad_sqnorm(g)
        tp, tm, tv = O.accum_adamw_f64(p, m, v, g, hp, S)
        op, om, ov, w = p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)
        O.accum_adamw(op, om, ov, w, g, hp, O.clip_coef(S, hp.max_grad_norm))
        shares = [f64_truth_check(got, tr, old, nm)[0] for nm, got, tr, old in
                  (("p", op, tp, p), ("m", om, tm, m), ("v", ov, tv, v))]
        assert min(shares) > 0.85 and shares[2] == 1.0         # v' never cancels: both terms are >= 0
