"""Property tests of the oracle (hypothesis): invariants that hold for any shape, any partition and
any value pattern, special bit patterns included.  They complement the fixed pins: a mistake that
only shows for an odd length, a range of one element or a particular mix of special values is what
these are for."""
import math

import numpy as np
from hypothesis import given, settings
from hypothesis import strategies as st

from oracle import gs_oracle as O

SPECIAL_BF16 = [0x0000, 0x8000, 0x3F80, 0xBF80, 0x0001, 0x8001, 0x7F7F, 0xFF7F, 0x0080, 0x3C00]
bf16_finite = st.one_of(st.sampled_from(SPECIAL_BF16),
                        st.integers(0, 0xFFFF).filter(lambda u: (u & 0x7F80) != 0x7F80))     # no Inf / NaN


@st.composite
def layer(draw, max_n=97, max_k=5):
    n = draw(st.integers(1, max_n))
    k = draw(st.integers(1, max_k))
    seed = draw(st.integers(0, 2**31 - 1))
    rng = np.random.default_rng(seed)
    g = [np.array(draw(st.lists(bf16_finite, min_size=n, max_size=n)), np.uint16) if j == 0
         else (rng.standard_normal(n) * 1e-2).astype(np.float32).view(np.uint32).__rshift__(16).astype(np.uint16)
         for j in range(k)]
    p = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v = ((rng.standard_normal(n) * 1e-3) ** 2).astype(np.float32)
    cuts = sorted(set(draw(st.lists(st.integers(0, n), max_size=4)) + [0, n]))
    return n, k, p, m, v, g, cuts


HP = O.HParams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0, step=3)


@settings(max_examples=60, deadline=None)
@given(layer())
def test_any_partition_of_the_range_gives_the_same_bits(case):
    n, k, p, m, v, g, cuts = case
    c = O.clip_coef(O.grad_sqnorm(g), HP.max_grad_norm)
    full = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    O.accum_adamw(*full, g, HP, c)
    part = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    for lo, hi in reversed(list(zip(cuts[:-1], cuts[1:]))):       # pieces in reverse order
        O.accum_adamw(*part, g, HP, c, lo, hi)
    for a, b in zip(full, part):
        assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a,
                              b.view(np.uint32) if b.dtype == np.float32 else b)


@settings(max_examples=60, deadline=None)
@given(layer())
def test_norm_is_additive_and_matches_the_buffer_routes(case):
    n, k, p, m, v, g, cuts = case
    S = O.grad_sqnorm(g)
    pieces = sum(O.grad_sqnorm(g, lo, hi) for lo, hi in zip(cuts[:-1], cuts[1:]))
    assert math.isclose(S, pieces, rel_tol=1e-12, abs_tol=1e-300)
    acc = O.accumulate(g)
    assert math.isclose(S, O.acc_sqnorm(acc), rel_tol=1e-12, abs_tol=1e-300)
    buf = np.full(n, np.float32(np.nan))
    last = 0.0
    for j, b in enumerate(g):
        last = O.accum_add(buf, b, first=(j == 0))
    assert np.array_equal(buf.view(np.uint32), acc.view(np.uint32))
    assert math.isclose(S, last, rel_tol=1e-12, abs_tol=1e-300)
    # exact cross-check in fp64: every bf16 value and every fp32 partial sum is an fp64 number
    ref = np.zeros(n, np.float32)
    for b in g:
        ref = (ref + (b.astype(np.uint32) << 16).view(np.float32)).astype(np.float32)
    assert math.isclose(S, float(np.dot(ref.astype(np.float64), ref.astype(np.float64))), rel_tol=1e-12, abs_tol=1e-300)


@settings(max_examples=60, deadline=None)
@given(layer(max_k=3), st.one_of(st.just(0.0), st.floats(2.0 ** -20, 10.0, width=32)))
def test_emitted_weight_is_the_rounded_master_weight_and_clip_never_amplifies(case, max_norm):
    n, k, p, m, v, g, _ = case
    S = O.grad_sqnorm(g)
    c = O.clip_coef(S, max_norm)
    assert 0.0 <= c <= 1.0
    if max_norm > 0.0 and math.sqrt(S) > 0:
        assert c * math.sqrt(S) <= max_norm * (1 + 1e-6)          # the clipped norm respects the bound
    st_ = [p.copy(), m.copy(), v.copy(), np.zeros(n, np.uint16)]
    O.accum_adamw(*st_, g, HP, c)
    for i in range(n):
        assert int(st_[3][i]) == O.f32_to_bf16(st_[0][i])
    assert np.all(st_[2] >= 0.0)                                   # the variance stays non-negative
