"""GPU parity at the full workload sizes, in the launch configuration bench.py times.

The resident workloads are compared with the oracle over their WHOLE range: h=4096 in one piece,
the headline h=8192 layer and both halves of the h=12288 split step in 2^26-element chunks on the
host's threads (norm first, from the oracle's own sum; then every element of p, m, v, w).  The
widened entry points, the GPT-30B-shaped layer and the host-resident workloads run on the full
range and are compared with the oracle on sampled windows (head, tail, windows at random unaligned
offsets, windows straddling split and chunk boundaries), plus properties that hold at any size:
split == full and streamed == resident bit for bit, w == bf16_rne(p'), additivity of the norm, and
the norm against a torch evaluation of its definition.
"""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import (DEV, O, assert_bf16_close, assert_f32_close, assert_w_is_rne_of_p, f64_truth_check, gs, np_bf16,
                      np_f32, ohp)
from paper_2512_17570_amd import inputs as I

pytestmark = pytest.mark.gpu


def hp_of(wl):
    return gs.HParams(wl.lr, wl.beta1, wl.beta2, wl.eps, wl.weight_decay, wl.max_grad_norm, wl.step)


def windows(n, count, width, seed, extra=()):
    rng = np.random.default_rng(seed)
    ws = [(0, min(n, width)), (max(0, n - width), n)]
    for _ in range(count):
        lo = int(rng.integers(0, n - width))
        ws.append((lo, lo + width + int(rng.integers(0, 9))))
    for c in extra:
        ws.append((max(0, c - width // 2), min(n, c + width // 2 + 3)))
    return ws


def grab(tensors, lo, hi):
    return [np_f32(t[lo:hi]) for t in tensors]


def torch_sqnorm(grads, chunk=1 << 26):
    """The definition with torch primitives: fp32 sum over j (ascending), squares summed in fp64."""
    n = grads[0].numel()
    tot = 0.0
    for lo in range(0, n, chunk):
        hi = min(n, lo + chunk)
        acc = torch.zeros(hi - lo, dtype=torch.float32, device=grads[0].device)
        for g in grads:
            acc += g[lo:hi].float()
        tot += float(acc.double().square().sum().item())
    return tot


def check_windows(wins, before, after, grads, hp, c, tag):
    """before/after: dicts lo -> (p,m,v[,w]) numpy windows; oracle applied to `before`."""
    worst = 0
    for (lo, hi) in wins:
        p, m, v = (a.copy() for a in before[lo])
        g = [np_bf16(x[lo:hi]) for x in grads]
        w = np.zeros(hi - lo, np.uint16)
        O.accum_adamw(p, m, v, w, g, ohp(hp), c)
        gp, gm, gv, gw = after[lo]
        worst = max(worst, assert_f32_close(gp, p, f"{tag}.p[{lo}:{hi}]"), assert_f32_close(gm, m, f"{tag}.m[{lo}:{hi}]"),
                    assert_f32_close(gv, v, f"{tag}.v[{lo}:{hi}]"))
        assert_bf16_close(gw, w, f"{tag}.w[{lo}:{hi}]")
    return worst


def whole_range_oracle_compare(tag, orig, result, w, grads, hp, S_gpu, chunk=1 << 26, threads=16, layer_is_part=False):
    """Oracle over every element of [0,n), chunk by chunk on `threads` host threads: the squared
    norm from the oracle's own sums (held against the GPU's), the clip coefficient from it, then
    the step on host copies of the ORIGINAL states, compared element by element with the GPU's
    p, m, v (4 ulp or 1e-6) and w (1 bf16 ulp).  layer_is_part: S_gpu is the norm over more than
    this layer (several layers clipped together), so the oracle's sum over this layer cannot be
    held against it and the clip coefficient is taken from S_gpu.  `result` tensors may live on the
    host (states stepped in pinned memory).  Returns (oracle S, c, worst ulp seen)."""
    n = grads[0].numel()
    cuts = list(range(0, n, chunk)) + [n]
    host_g = []
    S_o = 0.0
    with ThreadPoolExecutor(threads) as ex:
        for lo, hi in zip(cuts[:-1], cuts[1:]):
            hg = [np_bf16(g[lo:hi]) for g in grads]
            host_g.append(hg)
            b = [(hi - lo) * i // threads for i in range(threads + 1)]
            S_o += sum(ex.map(lambda i: O.grad_sqnorm(hg, b[i], b[i + 1]), range(threads)))
        if layer_is_part:
            assert 0.0 < S_o < S_gpu
            c = O.clip_coef(S_gpu, hp.max_grad_norm)
        else:
            assert abs(S_gpu - S_o) <= 1e-5 * S_o, (S_gpu, S_o)
            c = O.clip_coef(S_o, hp.max_grad_norm)
            assert c == O.clip_coef(S_gpu, hp.max_grad_norm)      # both sides clip with the same fp32 coefficient
        print(f"[{tag}] oracle norm over {n} elements done: S={S_o:.9e} (GPU {S_gpu:.9e}) c={c:.6f}", flush=True)
        worst = 0
        for ci, (lo, hi) in enumerate(zip(cuts[:-1], cuts[1:])):
            hg = host_g[ci]
            h_p, h_m, h_v = (np_f32(t[lo:hi]) for t in orig)
            h_w = np.zeros(hi - lo, np.uint16)
            b = [(hi - lo) * i // threads for i in range(threads + 1)]
            list(ex.map(lambda i: O.accum_adamw(h_p, h_m, h_v, h_w, hg, ohp(hp), c, b[i], b[i + 1]), range(threads)))
            for want, t, nm in ((h_p, result[0], "p"), (h_m, result[1], "m"), (h_v, result[2], "v")):
                got = np_f32(t[lo:hi])
                if not np.array_equal(got.view(np.uint32), want.view(np.uint32)):     # fast path: same bits
                    worst = max(worst, assert_f32_close(got, want, f"{tag}.{nm}[{lo}:{hi}]"))
            gw = np_bf16(w[lo:hi])
            if not np.array_equal(gw, h_w):
                assert_bf16_close(gw, h_w, f"{tag}.w[{lo}:{hi}]")
            host_g[ci] = None
            if ci % 4 == 3 or hi == n:
                print(f"[{tag}] oracle step compared through element {hi} of {n}", flush=True)
    return S_o, c, worst


@pytest.mark.timeout(900)
def test_h8192_k16_whole_layer_against_the_oracle():
    """The headline workload in the configuration bench.py times (norm, then the fused step over
    the whole layer: 3.1 M workgroups), every one of its 805 412 864 elements against the oracle."""
    wl = I.WORKLOADS["gpt65b_layer_h8192_k16"]
    n, k = wl.n, wl.k
    print(f"[h8192 whole] n={n} k={k}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    orig = (p.clone(), m.clone(), v.clone())
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    hp = hp_of(wl)
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)
    torch.cuda.synchronize()
    S_o, c, worst = whole_range_oracle_compare("h8192 whole", orig, (p, m, v), w, grads, hp, float(sq.item()))
    assert c < 1.0
    assert_w_is_rne_of_p(p, w, 0, n)
    print(f"[h8192 whole] every element within tolerance, worst ulp {worst}", flush=True)


@pytest.mark.timeout(1200)
def test_h12288_k8_both_halves_of_the_split_against_the_oracle():
    """The split step as bench.py times it -- immediate part [0,s) and deferred part [s,n) as two
    calls on two streams, s = 724 839 628 unaligned -- with all 1 812 099 072 elements of both
    halves against the oracle."""
    wl = I.WORKLOADS["gpt175b_layer_h12288_k8_split"]
    n, k = wl.n, wl.k
    s_pt = int(wl.extra["immediate_frac"] * n)
    print(f"[h12288 whole] n={n} k={k} split at {s_pt}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    orig = (p.clone(), m.clone(), v.clone())
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    hp = hp_of(wl)
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    cur = torch.cuda.current_stream()
    sa.wait_stream(cur); sb.wait_stream(cur)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, s_pt, hp, sq, stream=sa)      # immediate part
    gs.gs_accum_adamw(p, m, v, w, grads, s_pt, n, hp, sq, stream=sb)      # deferred part, other stream
    torch.cuda.synchronize()
    S_o, c, worst = whole_range_oracle_compare("h12288 whole", orig, (p, m, v), w, grads, hp, float(sq.item()))
    assert_w_is_rne_of_p(p, w, 0, n)
    print(f"[h12288 whole] both halves within tolerance, worst ulp {worst}", flush=True)


def test_h4096_k8_full_oracle_with_clipping():
    wl = I.WORKLOADS["gpt_h4096_k8"]
    n, k = wl.n, wl.k
    print(f"[h4096] n={n} k={k}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    h_p, h_m, h_v = np_f32(p), np_f32(m), np_f32(v)
    h_g = [np_bf16(g) for g in grads]
    hp = hp_of(wl)
    nn = 1 << 25
    o_p, o_m, o_v = h_p[:nn].copy(), h_m[:nn].copy(), h_v[:nn].copy()      # originals, for the fp64 evaluation below
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)
    torch.cuda.synchronize()
    S = float(sq.item())
    T = 16
    bounds = [n * i // T for i in range(T + 1)]
    with ThreadPoolExecutor(T) as ex:
        So = sum(ex.map(lambda i: O.grad_sqnorm(h_g, bounds[i], bounds[i + 1]), range(T)))
        assert abs(S - So) <= 1e-5 * So
        assert 100 < np.sqrt(So) < 170              # outliers x100 on 0.1 % of entries: ||g|| ~ 133
        c = O.clip_coef(So, hp.max_grad_norm)
        assert c < 0.01
        h_w = np.zeros(n, np.uint16)
        list(ex.map(lambda i: O.accum_adamw(h_p, h_m, h_v, h_w, h_g, ohp(hp), c, bounds[i], bounds[i + 1]), range(T)))
    up = assert_f32_close(np_f32(p), h_p, "h4096.p")
    um = assert_f32_close(np_f32(m), h_m, "h4096.m")
    uv = assert_f32_close(np_f32(v), h_v, "h4096.v")
    uw = assert_bf16_close(np_bf16(w), h_w, "h4096.w")
    assert_w_is_rne_of_p(p, w, 0, n)
    print(f"[h4096] S={S:.6e} oracle={So:.6e} c={c:.4e} max ulp p/m/v/w={up, um, uv, uw}", flush=True)
    # GPU against the fp64 evaluation of the same formulas, with clipping active, on the first 2^25
    # elements: the stated tolerance wherever the final add does not cancel, the operand-aware bound elsewhere
    tp, tm, tv = O.accum_adamw_f64(o_p, o_m, o_v, [g[:nn] for g in h_g], ohp(hp), So)
    for nm, t, truth, old in (("p", p, tp, o_p), ("m", m, tm, o_m), ("v", v, tv, o_v)):
        share, worst_rel, worst_sp = f64_truth_check(np_f32(t[:nn]), truth, old, f"h4096 vs fp64 {nm}")
        print(f"[h4096] {nm} vs fp64: {100 * share:.2f} % of elements judged by 4 ulp / 1e-6 (worst rel {worst_rel:.2e}); "
              f"worst error {worst_sp:.2f} spacings of the larger operand", flush=True)


@pytest.mark.parametrize("name", ["gpt65b_layer_h8192_k16", "gpt30b_layer_h7168_k16"])
def test_resident_layer_sampled(name):
    wl = I.WORKLOADS[name]
    n, k = wl.n, wl.k
    print(f"[{name}] n={n} k={k}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    hp = hp_of(wl)
    wins = windows(n, 40, 6000, seed=1)
    before = {lo: grab((p, m, v), lo, hi) for lo, hi in wins}
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)
    torch.cuda.synchronize()
    S = float(sq.item())
    # norm: the definition in torch primitives, additivity, oracle on windows
    St = torch_sqnorm(grads)
    assert abs(S - St) <= 1e-5 * St and abs(S - St) <= 1e-11 * St
    assert abs(np.sqrt(S) / np.sqrt(n * k * wl.grad_sigma ** 2) - 1) < 0.01      # n k sigma^2 (3221.7 at h = 8192)
    part = torch.zeros(1, dtype=torch.float64, device=DEV)
    cuts = [0, 12345, n // 3 + 1, n // 2 + 7, n - 5, n]
    for a, b in zip(cuts[:-1], cuts[1:]):
        gs.gs_grad_sqnorm(grads, a, b, part, ws, accumulate=(a > 0))
    torch.cuda.synchronize()
    assert abs(float(part.item()) - S) <= 1e-12 * S
    one = torch.zeros(1, dtype=torch.float64, device=DEV)
    for lo, hi in wins[:6]:
        gs.gs_grad_sqnorm(grads, lo, hi, one, ws)
        torch.cuda.synchronize()
        want = O.grad_sqnorm([np_bf16(g[lo:hi]) for g in grads])
        assert abs(float(one.item()) - want) <= 1e-12 * want
    # step on sampled windows
    c = O.clip_coef(S, hp.max_grad_norm)
    after = {lo: grab((p, m, v), lo, hi) + [np_bf16(w[lo:hi])] for lo, hi in wins}
    worst = check_windows(wins, before, after, grads, hp, c, "h8192")
    assert_w_is_rne_of_p(p, w, 0, n)
    print(f"[{name}] S={S:.6e} torch={St:.6e} c={c:.5f} worst ulp on {len(wins)} windows={worst}", flush=True)


@pytest.mark.timeout(600)
def test_h8192_k16_staged_and_speculative_at_full_size():
    """The widened entry points at the headline size, in the shapes bench.py times (large
    workspace): staged two-pass == fused bit for bit; speculative pass == oracle with c = 1 on
    sampled windows, inputs untouched, its norm equal to gs_grad_sqnorm's; k calls of gs_accum_add
    leave the staged buffer bit for bit."""
    wl = I.WORKLOADS["gpt65b_layer_h8192_k16"]
    n, k = wl.n, wl.k
    print(f"[h8192 staged/spec] n={n} k={k}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    p0, m0, v0 = p.clone(), m.clone(), v.clone()
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    sq2 = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    big = torch.empty(gs.gs_sqnorm_workspace_bytes_for(n), dtype=torch.uint8, device=DEV)
    hp = hp_of(wl)
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)                    # fused reference
    torch.cuda.synchronize()
    S = float(sq.item())
    # speculative pass from the untouched originals
    wins = windows(n, 16, 5000, seed=3)
    before = {lo: grab((p0, m0, v0), lo, hi) for lo, hi in wins}
    po, mo, vo = torch.empty_like(p0), torch.empty_like(m0), torch.empty_like(v0)
    w_s = torch.zeros_like(w)
    gs.gs_accum_adamw_spec(p0, m0, v0, po, mo, vo, w_s, grads, 0, n, hp, sq2, big)
    torch.cuda.synchronize()
    assert abs(float(sq2.item()) - S) <= 1e-12 * S
    after = {lo: grab((po, mo, vo), lo, hi) + [np_bf16(w_s[lo:hi])] for lo, hi in wins}
    check_windows(wins, before, after, grads, hp, 1.0, "spec")
    for lo, hi in wins[:4]:
        for a, b in zip(grab((p0, m0, v0), lo, hi), before[lo]):
            assert np.array_equal(a, b)                                   # inputs untouched
    assert gs.gs_clip_coefficient(S, hp.max_grad_norm) < 1.0              # the guess fails on this workload
    del po, mo, vo, w_s
    # staged two-pass on the originals, in place: must equal the fused result bit for bit
    acc = torch.empty(n, dtype=torch.float32, device=DEV)
    w2 = torch.zeros_like(w)
    gs.gs_grad_accum_sqnorm(grads, 0, n, acc, sq2, big)
    gs.gs_adamw_from_acc(p0, m0, v0, w2, acc, 0, n, hp, sq)               # same norm scalar as the fused run
    torch.cuda.synchronize()
    assert abs(float(sq2.item()) - S) <= 1e-12 * S
    for a, b, nm in ((p, p0, "p"), (m, m0, "m"), (v, v0, "v"), (w, w2, "w")):
        assert torch.equal(a, b), f"staged != fused in {nm}"
    lo, hi = wins[3]
    assert np.array_equal(np_f32(acc[lo:hi]), O.accumulate([np_bf16(g[lo:hi]) for g in grads]))
    # accumulate as you go, one call per micro-batch, the last with the norm: the same buffer bit for bit
    acc2 = torch.full((n,), float("nan"), dtype=torch.float32, device=DEV)
    for j in range(k):
        last = j == k - 1
        gs.gs_accum_add(acc2, grads[j], j == 0, 0, n, sq2 if last else None, big if last else None)
    torch.cuda.synchronize()
    assert torch.equal(acc, acc2), "k calls of gs_accum_add != k-way sum"
    assert abs(float(sq2.item()) - S) <= 1e-12 * S
    print(f"[h8192 staged/spec] S={S:.6e}; staged == fused bitwise; spec windows ok; as-you-go == staged", flush=True)


@pytest.mark.timeout(600)
def test_h12288_k8_split_equals_full_and_sampled():
    wl = I.WORKLOADS["gpt175b_layer_h12288_k8_split"]
    n, k = wl.n, wl.k
    s_pt = int(wl.extra["immediate_frac"] * n)
    assert s_pt == 724_839_628
    print(f"[h12288] n={n} k={k} split at {s_pt}", flush=True)
    p, m, v, grads = I.make_workload_tensors(wl, DEV)
    w = torch.zeros(n, dtype=torch.bfloat16, device=DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    hp = hp_of(wl)
    wins = windows(n, 24, 6000, seed=2, extra=(s_pt,))
    before = {lo: grab((p, m, v), lo, hi) for lo, hi in wins}
    p2, m2, v2, w2 = p.clone(), m.clone(), v.clone(), torch.zeros_like(w)
    gs.gs_grad_sqnorm(grads, 0, n, sq, ws)
    gs.gs_accum_adamw(p, m, v, w, grads, 0, n, hp, sq)                      # full
    sa, sb = torch.cuda.Stream(), torch.cuda.Stream()
    cur = torch.cuda.current_stream()
    sa.wait_stream(cur); sb.wait_stream(cur)
    gs.gs_accum_adamw(p2, m2, v2, w2, grads, 0, s_pt, hp, sq, stream=sa)    # immediate part
    gs.gs_accum_adamw(p2, m2, v2, w2, grads, s_pt, n, hp, sq, stream=sb)    # deferred part, other stream
    torch.cuda.synchronize()
    for a, b, nm in ((p, p2, "p"), (m, m2, "m"), (v, v2, "v"), (w, w2, "w")):
        assert torch.equal(a, b), f"split != full in {nm}"
    del p2, m2, v2, w2
    S = float(sq.item())
    St = torch_sqnorm(grads)
    assert abs(S - St) <= 1e-5 * St
    c = O.clip_coef(S, hp.max_grad_norm)
    after = {lo: grab((p, m, v), lo, hi) + [np_bf16(w[lo:hi])] for lo, hi in wins}
    worst = check_windows(wins, before, after, grads, hp, c, "h12288")
    assert_w_is_rne_of_p(p, w, 0, n)
    print(f"[h12288] S={S:.6e} c={c:.5f} worst ulp={worst}; split == full bitwise", flush=True)


@pytest.mark.timeout(900)
@pytest.mark.parametrize("mode", ["staged", "inplace"])
def test_streamed_8_layers_h8192_equals_resident(mode):
    wl = I.WORKLOADS["gpt65b_8layers_streamed_k8"]
    nl, k, chunk = I.layer_numel(wl.h), wl.k, wl.extra["chunk_elems"]
    layers = wl.layers
    bufs = None
    while layers > 0:
        bufs = gs.pinned_f32_set(layers * nl, 3)
        if bufs is not None:
            break
        layers -= 1
    assert layers >= 1, "could not pin host memory for one layer"
    n = layers * nl
    print(f"[streamed {mode}] layers={layers} n={n} k={k} chunk={chunk} pinned={12 * n / 1e9:.1f} GB", flush=True)
    (hp_t, hp_p), (hm_t, hm_p), (hv_t, hv_p) = bufs
    try:
        hp = hp_of(wl)
        sq = torch.zeros(1, dtype=torch.float64, device=DEV)
        ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
        grads_l, w_l, ref = [], [], []
        for L in range(layers):
            pd, md, vd = I.make_states(nl, wl.seed + L, DEV)
            for dst, src in ((hp_t, pd), (hm_t, md), (hv_t, vd)):
                dst[L * nl:(L + 1) * nl].copy_(src)
            g = I.make_grads(nl, k, wl.grad_sigma, wl.seed + L, DEV)
            grads_l.append(g)
            w_l.append(torch.zeros(nl, dtype=torch.bfloat16, device=DEV))
            if L == 0 and mode == "staged":
                orig0 = (pd.clone(), md.clone(), vd.clone())             # for the whole-layer oracle pass below
            ref.append((pd, md, vd, torch.zeros(nl, dtype=torch.bfloat16, device=DEV)))
            gs.gs_grad_sqnorm(g, 0, nl, sq, ws, accumulate=(L > 0))       # global norm over all layers
        torch.cuda.synchronize()
        print(f"[streamed] inputs ready, ||g||={np.sqrt(float(sq.item())):.3f}", flush=True)
        # a window that straddles a chunk boundary inside layer 0 and the ragged tail chunk of the last layer
        wins = [(chunk - 3000, chunk + 3001), (nl - 4000, nl)]
        before0 = {lo: [hp_t[lo:hi].numpy().copy(), hm_t[lo:hi].numpy().copy(), hv_t[lo:hi].numpy().copy()] for lo, hi in wins}
        if mode == "staged":
            ctx = gs.gs_stream_ctx_create(chunk, 3)        # 2^26-element chunks through three HBM slots, as bench.py times
        else:
            ctx = gs.gs_stream_ctx_create_inplace(16)      # 16 of the CUs carry the full link rate
        for L in range(layers):
            o = L * nl * 4
            gs.gs_stream_layer_step(ctx, hp_p + o, hm_p + o, hv_p + o, w_l[L], grads_l[L], nl, hp, sq)
        gs.gs_stream_ctx_sync(ctx)
        gs.gs_stream_ctx_destroy(ctx)
        print("[streamed] streamed pass done", flush=True)
        # resident path on device copies, then compare bit for bit layer by layer
        for L in range(layers):
            pd, md, vd, wd = ref[L]
            gs.gs_accum_adamw(pd, md, vd, wd, grads_l[L], 0, nl, hp, sq)
            torch.cuda.synchronize()
            for host, devt, nm in ((hp_t, pd, "p"), (hm_t, md, "m"), (hv_t, vd, "v")):
                for lo in range(0, nl, chunk):
                    hi = min(nl, lo + chunk)
                    up = host[L * nl + lo:L * nl + hi].to(DEV)
                    assert torch.equal(up, devt[lo:hi]), f"layer {L} {nm}[{lo}:{hi}] streamed != resident"
            assert torch.equal(w_l[L], wd), f"layer {L} w streamed != resident"
            ref[L] = None
            del pd, md, vd, wd
            print(f"[streamed] layer {L} == resident", flush=True)
        # oracle on the sampled windows of layer 0
        c = O.clip_coef(float(sq.item()), hp.max_grad_norm)
        after0 = {lo: [hp_t[lo:hi].numpy().copy(), hm_t[lo:hi].numpy().copy(), hv_t[lo:hi].numpy().copy(), np_bf16(w_l[0][lo:hi])]
                  for lo, hi in wins}
        check_windows(wins, before0, after0, grads_l[0], hp, c, "streamed")
        if mode == "staged":
            # and every element of layer 0 as the 2^26-element chunk pipeline left it in host memory
            _, _, worst = whole_range_oracle_compare("streamed layer 0", orig0, (hp_t[:nl], hm_t[:nl], hv_t[:nl]), w_l[0],
                                                     grads_l[0], hp, float(sq.item()), layer_is_part=layers > 1)
            print(f"[streamed] layer 0: all {nl} elements against the oracle, worst ulp {worst}", flush=True)
    finally:
        del hp_t, hm_t, hv_t
        for t, ptr in bufs:
            gs.gs_pinned_free(ptr)


@pytest.mark.timeout(900)
def test_tiered_one_layer_h8192_equals_resident(tmp_path):
    """One GPT-65B-shaped layer with half of its states in pinned host memory and half in files
    (the tiered workload's split and chunk size): bit for bit the resident result, and the oracle
    on windows at the head, across the host/file boundary, across a file-chunk boundary and at the
    ragged tail."""
    import os
    wl = I.WORKLOADS["gpt65b_2layers_tiered_k8"]
    nl, k, chunk, x = I.layer_numel(wl.h), wl.k, wl.extra["chunk_elems"], wl.extra["host_share"]
    n_host = int(round(x * nl))
    hp = hp_of(wl)
    pd, md, vd = I.make_states(nl, wl.seed, DEV)
    grads = I.make_grads(nl, k, wl.grad_sigma, wl.seed, DEV)
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    gs.gs_grad_sqnorm(grads, 0, nl, sq, ws)
    bufs = gs.pinned_f32_set(n_host, 3)
    assert bufs is not None, "could not pin the host share"
    fds, paths = [], []
    try:
        for name, (t, _), src in zip("pmv", bufs, (pd, md, vd)):
            t.copy_(src[:n_host])
            path = str(tmp_path / f"{name}.bin")
            src[n_host:].cpu().numpy().tofile(path)
            paths.append(path)
            fds.append(os.open(path, os.O_RDWR))
        print(f"[tiered] n={nl} n_host={n_host} file bytes={12 * (nl - n_host) / 1e9:.1f} GB chunk={chunk}", flush=True)
        wins = [(0, 4000), (n_host - 3000, n_host + 3001), (n_host + chunk - 3000, n_host + chunk + 3001), (nl - 4000, nl)]
        before = {lo: grab((pd, md, vd), lo, hi) for lo, hi in wins}
        w = torch.zeros(nl, dtype=torch.bfloat16, device=DEV)
        ctx = gs.gs_tier_ctx_create(chunk, 3, 16)
        gs.gs_tier_layer_step(ctx, bufs[0][1], bufs[1][1], bufs[2][1], n_host, fds, (0, 0, 0), w, grads, nl, hp, sq)
        gs.gs_tier_ctx_sync(ctx)
        assert gs.gs_tier_ctx_error(ctx) == ""
        gs.gs_tier_ctx_destroy(ctx)
        print("[tiered] tiered pass done", flush=True)
        wd = torch.zeros(nl, dtype=torch.bfloat16, device=DEV)
        gs.gs_accum_adamw(pd, md, vd, wd, grads, 0, nl, hp, sq)
        torch.cuda.synchronize()
        assert torch.equal(w, wd)
        for (t, _), path, ref, nm in zip(bufs, paths, (pd, md, vd), "pmv"):
            assert torch.equal(t.to(DEV), ref[:n_host]), f"{nm}: host share != resident"
            tail = np.memmap(path, dtype=np.float32, mode="r")
            assert tail.shape[0] == nl - n_host
            for lo in range(0, nl - n_host, 1 << 26):
                hi = min(nl - n_host, lo + (1 << 26))
                up = torch.from_numpy(np.array(tail[lo:hi])).to(DEV)
                assert torch.equal(up, ref[n_host + lo:n_host + hi]), f"{nm}: file share [{lo}:{hi}) != resident"
            del tail
        c = O.clip_coef(float(sq.item()), hp.max_grad_norm)
        after = {lo: grab((pd, md, vd), lo, hi) + [np_bf16(wd[lo:hi])] for lo, hi in wins}
        check_windows(wins, before, after, grads, hp, c, "tiered")
    finally:
        for fd in fds:
            os.close(fd)
        for p_ in paths:
            if os.path.exists(p_):
                os.unlink(p_)
        for _, ptr in bufs:
            gs.gs_pinned_free(ptr)


@pytest.mark.timeout(600)
def test_element_indices_beyond_2_to_31():
    """Arrays longer than 2^31 elements: a window straddling index 2^31 is stepped as a range of
    its own and as part of the whole [0,N) range (N/512 = 4.2 M workgroups; the norm folds more
    tiles than its fixed workspace has partials), and checked against the oracle.  Everything
    outside the window is zero, where the step leaves zeros and the norm adds nothing."""
    N = (1 << 31) + 4096 + 5
    lo, hi = (1 << 31) - 3001, N
    k = 2
    hp = gs.HParams(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, max_grad_norm=1.0, step=7)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(4242)
    p = torch.zeros(N, dtype=torch.float32, device=DEV)
    m = torch.zeros(N, dtype=torch.float32, device=DEV)
    v = torch.zeros(N, dtype=torch.float32, device=DEV)
    w = torch.zeros(N, dtype=torch.bfloat16, device=DEV)
    grads = [torch.zeros(N, dtype=torch.bfloat16, device=DEV) for _ in range(k)]
    wn = hi - lo
    p[lo:hi] = torch.randn(wn, generator=gen, device=DEV) * 0.02
    m[lo:hi] = torch.randn(wn, generator=gen, device=DEV) * 1e-3
    v[lo:hi] = (torch.randn(wn, generator=gen, device=DEV) * 1e-3) ** 2
    for g in grads:
        g[lo:hi] = (torch.randn(wn, generator=gen, device=DEV) * 1e-2).to(torch.bfloat16)
    h_p, h_m, h_v = (np_f32(t[lo:hi]) for t in (p, m, v))
    h_g = [np_bf16(g[lo:hi]) for g in grads]
    sq = torch.zeros(1, dtype=torch.float64, device=DEV)
    ws = torch.empty(gs.gs_sqnorm_workspace_bytes(), dtype=torch.uint8, device=DEV)
    S_o = O.grad_sqnorm(h_g)
    # the norm: window alone, whole range, and whole range staged (large and minimum workspace)
    gs.gs_grad_sqnorm(grads, lo, hi, sq, ws)
    torch.cuda.synchronize()
    assert abs(float(sq.item()) - S_o) <= 1e-12 * S_o
    gs.gs_grad_sqnorm(grads, 0, N, sq, ws)
    torch.cuda.synchronize()
    assert abs(float(sq.item()) - S_o) <= 1e-12 * S_o
    acc = torch.full((N,), 3.0, dtype=torch.float32, device=DEV)
    gs.gs_grad_accum_sqnorm(grads, 0, N, acc, sq, ws)
    torch.cuda.synchronize()
    assert abs(float(sq.item()) - S_o) <= 1e-12 * S_o
    assert np.array_equal(np_f32(acc[lo:hi]), O.accumulate(h_g)) and float(acc[:lo].abs().max().item()) == 0.0
    # accumulate as you go over the whole range
    acc.fill_(5.0)
    gs.gs_accum_add(acc, grads[0], True, 0, N)
    gs.gs_accum_add(acc, grads[1], False, 0, N, sq, ws)
    torch.cuda.synchronize()
    assert abs(float(sq.item()) - S_o) <= 1e-12 * S_o
    assert np.array_equal(np_f32(acc[lo:hi]), O.accumulate(h_g)) and float(acc[:lo].abs().max().item()) == 0.0
    del acc
    c = O.clip_coef(S_o, hp.max_grad_norm)
    o_p, o_m, o_v, o_w = h_p.copy(), h_m.copy(), h_v.copy(), np.zeros(wn, np.uint16)
    O.accum_adamw(o_p, o_m, o_v, o_w, h_g, ohp(hp), c)
    # the step over the window as a range of its own (out of place, so the inputs survive)
    po, mo, vo = (torch.zeros(N, dtype=torch.float32, device=DEV) for _ in range(3))
    gs.gs_accum_adamw_oop(p, m, v, po, mo, vo, w, grads, lo, hi, hp, sq)
    torch.cuda.synchronize()
    for got, want, nm in ((po, o_p, "p"), (mo, o_m, "m"), (vo, o_v, "v")):
        assert_f32_close(np_f32(got[lo:hi]), want, f"2^31 window {nm}")
        assert float(got[:lo].abs().max().item()) == 0.0
    assert_bf16_close(np_bf16(w[lo:hi]), o_w, "2^31 window w")
    del po, mo, vo
    # and as part of the whole range, in place
    w.zero_()
    gs.gs_accum_adamw(p, m, v, w, grads, 0, N, hp, sq)
    torch.cuda.synchronize()
    for got, want, nm in ((p, o_p, "p"), (m, o_m, "m"), (v, o_v, "v")):
        assert_f32_close(np_f32(got[lo:hi]), want, f"whole range {nm}")
        assert float(got[:lo].abs().max().item()) == 0.0, f"{nm}: zeros outside the window moved"
    assert_bf16_close(np_bf16(w[lo:hi]), o_w, "whole range w")
    assert int(torch.count_nonzero(w[:lo].view(torch.int16)).item()) == 0
    print(f"[2^31] N={N} window=[{lo},{hi}) S={S_o:.6e} c={c:.5f}", flush=True)
