"""Pins of the CPU oracle against things other than itself: published known-answer vectors,
hand-worked traces, closed forms, special cases that reduce to a library routine, invariants
stated by the paper's lemmas, and brute force on tiny inputs.  No GPU needed."""
import math

import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as O

EMPTY_P = 1e-12      # floor(p * 2^32) = 0: the subset is empty, i.e. no averaging ever happens


# --------------------------------------------------------------------------------------------
# subset generator
# --------------------------------------------------------------------------------------------
def test_philox_known_answers(golden_dir):
    rows = [l.split() for l in (golden_dir / "philox4x32_10_kat.txt").read_text().splitlines()
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        vals = [int(x, 16) for x in r]
        assert O.philox4x32_10(vals[0:4], vals[4:6]) == tuple(vals[6:10])


def test_threshold_edges():
    assert O.threshold(1.0) == 2 ** 32
    assert O.threshold(0.5) == 2 ** 31
    assert O.threshold(0.05) == math.floor(0.05 * 2 ** 32)
    assert O.threshold(EMPTY_P) == 0
    assert O.subset(3, 7, 5000, EMPTY_P).size == 0
    assert np.array_equal(O.subset(3, 7, 5000, 1.0), np.arange(5000, dtype=np.uint64))


def test_membership_uses_the_stated_counter_layout():
    """member(mu) must be lane mu&3 of philox(counter=(lo(mu>>2), hi(mu>>2), lo(s), hi(s)), key=seed)."""
    seed, s = 0x1234_5678_9ABC_DEF0, (5 << 32) | 17
    for mu in [0, 1, 2, 3, 4, 1023, (1 << 34) + 6, (1 << 40) + 3]:
        g = mu >> 2
        x = O.philox4x32_10((g & 0xFFFFFFFF, g >> 32, s & 0xFFFFFFFF, s >> 32), (seed & 0xFFFFFFFF, seed >> 32))
        for p in (0.01, 0.3, 0.9):
            assert O.member(seed, s, mu, p) == (x[mu & 3] < math.floor(p * 2 ** 32))


def test_subset_list_is_the_predicate_brute_force():
    n, p, seed, s = 1 << 14, 0.05, 11, 3
    want = np.array([mu for mu in range(n) if O.member(seed, s, mu, p)], dtype=np.uint64)
    got = O.subset(seed, s, n, p)
    assert np.array_equal(got, want)
    assert np.all(np.diff(got.astype(np.int64)) > 0)
    # a slice of the stage sees the same global subset
    lo, ln = 4099, 3001
    assert np.array_equal(O.subset(seed, s, ln, p, mu0=lo), want[(want >= lo) & (want < lo + ln)])


def test_subset_statistics():
    n, p = 200_000, 0.05
    sets = [O.subset(0, t, n, p) for t in range(1, 41)]
    sigma = math.sqrt(n * p * (1 - p))
    for S in sets:
        assert abs(S.size - n * p) < 5 * sigma                      # |S| ~ Binomial(n, p)
    assert not np.array_equal(sets[0], sets[1])                         # redrawn every step
    assert not np.array_equal(O.subset(1, 1, n, p), sets[0])            # depends on the seed
    assert np.array_equal(O.subset(0, 1, n, p), sets[0])                # pure function of (seed, t)
    # every coordinate is included with frequency ~ p: chi-square-like bound on the histogram
    hits = np.zeros(n, dtype=np.int64)
    for S in sets:
        hits[S.astype(np.int64)] += 1
    assert abs(hits.mean() - 40 * p) < 5 * math.sqrt(40 * p * (1 - p) / n)
    # inclusion is independent between neighbours inside one Philox block (lanes 0..3)
    a = np.zeros(n, dtype=bool); a[sets[0].astype(np.int64)] = True
    both = np.count_nonzero(a[0::4] & a[1::4])
    assert abs(both - (n / 4) * p * p) < 6 * math.sqrt((n / 4) * p * p)


def test_block_granule_variant_keeps_the_marginal_probability():
    """Variant (not the paper's sampling): aligned blocks of 32 coordinates drawn as a whole.  Every
    coordinate is still selected with probability p; blocks are all-or-nothing; block b uses the
    generator exactly as coordinate b does in the per-coordinate scheme."""
    n, p, seed, s = 64_000, 0.1, 7, 4
    S = O.subset(seed, s, n, p, granule=32)
    a = np.zeros(n, dtype=bool); a[S.astype(np.int64)] = True
    blocks = a.reshape(-1, 32)
    assert np.all(blocks.all(axis=1) | ~blocks.any(axis=1))
    per_coord = O.subset(seed, s, n // 32, p)                     # "coordinates" = block numbers
    assert np.array_equal(np.flatnonzero(blocks[:, 0]).astype(np.uint64), per_coord)
    hits = np.zeros(n // 32)
    for t in range(1, 201):
        b = np.zeros(n, dtype=bool); b[O.subset(seed, t, n, p, granule=32).astype(np.int64)] = True
        hits += b[::32]
    assert abs(hits.mean() / 200 - p) < 5 * math.sqrt(p * (1 - p) / (200 * n / 32))
    # the averaging itself is unchanged: subset coordinates take the mean (tau = 0)
    R, lr = 3, O.f32(0.25)
    w0 = np.stack([si.stage_weights(n, seed=60 + i) for i in range(R)])
    orc = O.Oracle(n, R, delay=0, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0,
                   subset_granule=32)
    orc.set_w(w0)
    g = np.stack(si.replica_grads(n, R, 1, seed=9))
    what = (w0.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
    want = what.copy()
    S1 = O.subset(seed, 1, n, p, granule=32).astype(np.int64)
    want[:, S1] = what[:, S1].astype(np.float64).mean(axis=0).astype(np.float32)
    orc.step(1, list(g), lr)
    assert np.array_equal(np.stack([orc.w(i) for i in range(R)]), want)


def test_stratified_variant_has_exact_size_and_the_marginal_probability():
    """Variant (not the paper's independent draws): one coordinate out of every aligned block of
    B = round(1/p).  Exact size, offsets written out from the generator word of block b, every
    offset equally likely, and the averaging itself unchanged."""
    assert [O.block_size(p) for p in (1.0, 0.6, 0.5, 0.4, 0.3, 0.05, 0.01, 1e-3)] == [1, 2, 2, 3, 3, 20, 100, 1000]   # nearest, halves up
    seed, s, p = 21, 6, 0.05
    B = 20
    for n in (20 * 500, 20 * 500 + 7):
        S = O.subset(seed, s, n, p, stratified=True).astype(np.int64)
        full = n // B
        assert np.array_equal(S[:full] // B, np.arange(full))            # exactly one per full block
        assert S.size in (full, full + (1 if n % B else 0))              # the cut block may or may not reach its member
        for b in (0, 1, 2, 3, 4, 77, full - 1):                          # offset = floor(X_b B / 2^32)
            g = b >> 2
            x = O.philox4x32_10((g, 0, s, 0), (seed, 0))
            assert S[b] - b * B == (x[b & 3] * B) >> 32
        lo, ln = 4099, 3001                                              # a slice sees the same global subset
        assert np.array_equal(O.subset(seed, s, ln, p, mu0=lo, stratified=True).astype(np.int64), S[(S >= lo) & (S < lo + ln)])
    assert np.array_equal(O.subset(3, 9, 777, 1.0, stratified=True), np.arange(777, dtype=np.uint64))   # B = 1: everything
    # offsets are uniform over the block: chi-square over 20 cells, 40 steps x 5000 blocks
    n = B * 5000
    cells = np.zeros(B)
    for t in range(1, 41):
        cells += np.bincount(O.subset(seed, t, n, p, stratified=True).astype(np.int64) % B, minlength=B)
    expect = 40 * 5000 / B
    chi2 = float(np.sum((cells - expect) ** 2 / expect))
    assert chi2 < 60.0                                                   # 19 degrees of freedom: P(chi2 > 60) ~ 4e-6
    assert not np.array_equal(O.subset(seed, 1, n, p, stratified=True), O.subset(seed, 2, n, p, stratified=True))
    # subset coordinates take the mean (tau = 0), the rest keep the local step
    R, lr, n = 3, O.f32(0.25), 10_007
    w0 = np.stack([si.stage_weights(n, seed=70 + i) for i in range(R)])
    orc = O.Oracle(n, R, delay=0, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0,
                   subset_kind=O.SUBSET_STRATIFIED)
    orc.set_w(w0)
    g = np.stack(si.replica_grads(n, R, 1, seed=10))
    what = (w0.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
    want = what.copy()
    S1 = O.subset(seed, 1, n, p, stratified=True).astype(np.int64)
    want[:, S1] = what[:, S1].astype(np.float64).mean(axis=0).astype(np.float32)
    orc.step(1, list(g), lr)
    assert np.array_equal(np.stack([orc.w(i) for i in range(R)]), want)


# --------------------------------------------------------------------------------------------
# bf16 helpers against a library conversion
# --------------------------------------------------------------------------------------------
def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4000).astype(np.float32) * np.float32(0.02),
                        np.array([0.0, -0.0, 1.0, -1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40],
                                 dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([O.double_to_bf16(float(v)) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)
    assert np.array_equal(si.to_bf16_bits(x), want)
    back = np.array([O.bf16_to_float(int(h)) for h in want[:100]], dtype=np.float32)
    assert np.array_equal(back, si.bf16_bits_to_f32(want[:100]))
    # ties go to even: 1 + 2^-8 is halfway between 1 and 1 + 2^-7
    assert O.double_to_bf16(1.0 + 2.0 ** -8) == 0x3F80
    assert O.double_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82
    # one rounding, not two: just above the tie must round up even if fp32 would land on the tie
    assert O.double_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81


def test_e4m3_rounding_matches_library():
    rng = np.random.default_rng(6)
    x = np.concatenate([rng.standard_normal(3000).astype(np.float32) * np.float32(0.02),
                        rng.standard_normal(1000).astype(np.float32),
                        rng.uniform(-440, 440, 500).astype(np.float32),
                        np.array([0.0, 2.0 ** -9, 2.0 ** -10, 3 * 2.0 ** -10, 2.0 ** -6, 0.0175, 448.0, 1.0625, 1.1875],
                                 dtype=np.float32)])
    want = torch.from_numpy(x).to(torch.float8_e4m3fn).to(torch.float32).numpy()
    got = np.array([O.quantize_e4m3(float(v)) for v in x], dtype=np.float32)
    assert np.array_equal(got, want)
    assert O.quantize_e4m3(1000.0) == 448.0 and O.quantize_e4m3(-1e9) == -448.0        # saturating
    assert O.quantize_message(0.3, O.MSG_F32) == float(np.float32(0.3))
    assert O.quantize_message(0.3, O.MSG_BF16) == O.bf16_to_float(O.double_to_bf16(float(np.float32(0.3))))


def test_quantised_message_only_touches_the_average():
    """Compression experiment: the average is formed from quantised values; everything a replica
    knows locally (its own old value in the staleness term) stays exact."""
    n, R, tau, lr, lam = 1200, 3, 1, O.f32(0.125), O.f32(0.5)
    w0 = si.stage_weights(n, seed=40)
    for msg, quant in ((O.MSG_BF16, lambda a: si.bf16_bits_to_f32(si.to_bf16_bits(a))),
                       (O.MSG_E4M3, lambda a: torch.from_numpy(a).to(torch.float8_e4m3fn).to(torch.float32).numpy())):
        orc = O.Oracle(n, R, delay=tau, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0, msg_dtype=msg)
        orc.set_w(w0)
        cur, whats, d = np.stack([w0] * R), {}, np.zeros((R, n), np.float32)
        for t in range(1, 5):
            g = np.stack(si.replica_grads(n, R, t, seed=40))
            what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
            whats[t] = what
            want = what.copy()
            if t > tau:
                old = whats[t - tau]
                abar = np.stack([quant(np.ascontiguousarray(old[i])) for i in range(R)]).astype(np.float64).mean(axis=0).astype(np.float32)
                d = ((1 - lam) * d.astype(np.float64) + lam * (what.astype(np.float64) - old.astype(np.float64))).astype(np.float32)
                want = (abar.astype(np.float64)[None, :] + d.astype(np.float64)).astype(np.float32)
            orc.step(t, list(g), lr, lam=lam)
            cur = np.stack([orc.w(i) for i in range(R)])
            assert np.array_equal(cur, want), (msg, t)


# --------------------------------------------------------------------------------------------
# local step alone == a stand-alone optimizer run (library routine)
# --------------------------------------------------------------------------------------------
def _torch_run(make_opt, w0, grads_per_step):
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = make_opt([p])
    for g in grads_per_step:
        p.grad = torch.from_numpy(g.copy())
        opt.step()
    return p.detach().numpy()


@pytest.mark.parametrize("name", ["sgd", "sgd_momentum", "adamw", "nadamw"])
def test_local_step_equals_library_optimizer(name):
    n, R, steps, lr = 3000, 2, 12, 3e-3
    w0 = si.stage_weights(n, seed=1)
    grads = [si.replica_grads(n, R, t, seed=1) for t in range(1, steps + 1)]
    b1, b2, eps = O.f32(0.9), O.f32(0.999), O.f32(1e-8)
    if name == "sgd":
        kw = dict(optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
        mk = lambda ps: torch.optim.SGD(ps, lr=O.f32(lr), foreach=False)
    elif name == "sgd_momentum":
        kw = dict(optimizer=O.OPT_SGD, beta1=0.9, weight_decay=0.0)
        mk = lambda ps: torch.optim.SGD(ps, lr=O.f32(lr), momentum=b1, foreach=False)
    elif name == "adamw":
        kw = dict(optimizer=O.OPT_ADAMW, weight_decay=0.01)
        mk = lambda ps: torch.optim.AdamW(ps, lr=O.f32(lr), betas=(b1, b2), eps=eps,
                                          weight_decay=O.f32(0.01), foreach=False)
    else:
        kw = dict(optimizer=O.OPT_NADAMW, weight_decay=0.01)
        mk = lambda ps: torch.optim.NAdam(ps, lr=O.f32(lr), betas=(b1, b2), eps=eps,
                                          weight_decay=O.f32(0.01), decoupled_weight_decay=True,
                                          momentum_decay=0.004, foreach=False)
    orc = O.Oracle(n, R, delay=1, fraction=EMPTY_P, **kw)       # empty subset: averaging never acts
    orc.set_w(w0)
    for t in range(1, steps + 1):
        orc.step(t, grads[t - 1], lr)
    for i in range(R):
        want = _torch_run(mk, w0, [g[i] for g in grads])
        got = orc.w(i)
        scale = np.maximum(np.abs(want), np.sqrt(np.mean(want ** 2)))
        assert np.max(np.abs(got - want) / scale) < 2e-6
        assert np.array_equal(orc.fwd(i), got)                 # look-ahead off: fwd is w
        assert not np.any(orc.d(i))


@pytest.mark.parametrize("name", ["adamw", "nadamw"])
def test_replicas_of_unequal_speed_each_follow_their_own_optimizer_run(name):
    """Heterogeneous set-up: a replica that steps in only some ticks is, with averaging off, a
    stand-alone library optimizer run over just the gradients of its own steps (own step count in
    the bias corrections, own momentum schedule), and an idle tick leaves it untouched."""
    n, R, ticks, lr = 2000, 3, 12, 3e-3
    b1, b2, eps = O.f32(0.9), O.f32(0.999), O.f32(1e-8)
    w0 = si.stage_weights(n, seed=4)
    grads = [si.replica_grads(n, R, t, seed=4) for t in range(1, ticks + 1)]
    masks = [0b111, 0b110, 0b100, 0b111, 0b010, 0b100, 0b101, 0b110, 0b100, 0b000, 0b011, 0b100]
    if name == "adamw":
        kw = dict(optimizer=O.OPT_ADAMW, weight_decay=0.01)
        mk = lambda ps: torch.optim.AdamW(ps, lr=O.f32(lr), betas=(b1, b2), eps=eps, weight_decay=O.f32(0.01), foreach=False)
    else:
        kw = dict(optimizer=O.OPT_NADAMW, weight_decay=0.01)
        mk = lambda ps: torch.optim.NAdam(ps, lr=O.f32(lr), betas=(b1, b2), eps=eps, weight_decay=O.f32(0.01),
                                          decoupled_weight_decay=True, momentum_decay=0.004, foreach=False)
    orc = O.Oracle(n, R, delay=1, fraction=EMPTY_P, **kw)
    orc.set_w(w0)
    for t in range(1, ticks + 1):
        before = [(orc.w(i).copy(), orc.m(i).copy(), orc.v(i).copy()) for i in range(R)]
        g = [grads[t - 1][i] if (masks[t - 1] >> i) & 1 else None for i in range(R)]
        orc.step_masked(t, g, lr, 0.5, masks[t - 1])
        for i in range(R):
            if not (masks[t - 1] >> i) & 1:
                assert all(np.array_equal(a, b) for a, b in zip(before[i], (orc.w(i), orc.m(i), orc.v(i))))
    for i in range(R):
        own = [grads[t][i] for t in range(ticks) if (masks[t] >> i) & 1]
        want = _torch_run(mk, w0, own)
        scale = np.maximum(np.abs(want), np.sqrt(np.mean(want ** 2)))
        assert np.max(np.abs(orc.w(i) - want) / scale) < 2e-6, i


def test_all_replicas_active_is_the_ordinary_step_and_idle_ones_still_average():
    n, R, lr = 5000, 3, O.f32(0.25)
    for opt in (O.OPT_ADAMW, O.OPT_NADAMW):
        a = O.Oracle(n, R, delay=1, fraction=0.2, seed=3, optimizer=opt, lookahead=True, gamma=0.9)
        b = O.Oracle(n, R, delay=1, fraction=0.2, seed=3, optimizer=opt, lookahead=True, gamma=0.9)
        w0 = si.stage_weights(n, seed=5)
        a.set_w(w0); b.set_w(w0)
        for t in range(1, 7):
            g = si.replica_grads(n, R, t, seed=5)
            a.step(t, g, 1e-3, 0.5)
            b.step_masked(t, g, 1e-3, 0.5, 0b111)
        for i in range(R):
            for name in ("w", "m", "v", "d", "fwd"):
                assert np.array_equal(getattr(a, name)(i), getattr(b, name)(i)), (opt, name, i)
    # tau = 0, p = 1, plain SGD: everybody ends on the mean of the w^, and an idle replica's w^ is its old w
    w0 = np.stack([si.stage_weights(n, seed=80 + i) for i in range(R)])
    orc = O.Oracle(n, R, delay=0, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0, lookahead=True, gamma=0.5)
    orc.set_w(w0)
    g = np.stack(si.replica_grads(n, R, 1, seed=6))
    orc.step_masked(1, [g[0], None, g[2]], lr, 0.5, 0b101)
    what = w0.astype(np.float64) - lr * g.astype(np.float64) * np.array([1.0, 0.0, 1.0])[:, None]
    what = what.astype(np.float32)
    mean = what.astype(np.float64).mean(axis=0).astype(np.float32)
    for i in range(R):
        assert np.array_equal(orc.w(i), mean)
        delta = what[i].astype(np.float64) - w0[i].astype(np.float64)          # the optimizer's displacement: 0 when idle
        assert np.array_equal(orc.fwd(i), (mean.astype(np.float64) + 0.5 * delta).astype(np.float32))


def test_sgd_decoupled_weight_decay_hand_trace(golden_dir):
    """SGD (plain and heavy-ball) with weight_decay != 0 against a hand-worked dyadic trace: the decay
    multiplies the weights and never enters the momentum."""
    rows = [l.split() for l in (golden_dir / "sgd_decoupled_decay_trace.txt").read_text().splitlines()
            if l.strip() and not l.startswith("#")]
    for beta in (0.5, 0.0):
        orc = O.Oracle(1, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=beta, weight_decay=0.25)
        orc.set_w(np.array([1.0], np.float32))
        mine = [r for r in rows if float(r[0]) == beta]
        assert len(mine) == 2
        for r in mine:
            t, g, m, w = int(r[1]), float(r[2]), float(r[3]), float(r[4])
            orc.step(t, [np.array([g], np.float32)], 0.5)
            assert orc.w(0)[0] == w and orc.m(0)[0] == m, (beta, t, orc.w(0)[0], orc.m(0)[0])


def test_sgd_decoupled_weight_decay_closed_form_and_library():
    """One plain step is w (1 - lr wd) - lr g element-wise; many heavy-ball steps equal the library's
    SGD (no decay of its own) run on weights that are shrunk by (1 - lr wd) before every step."""
    n, lr, wd, b1, steps = 2000, 3e-3, 0.05, 0.9, 10
    lr32, wd32, b132 = O.f32(lr), O.f32(wd), O.f32(b1)
    w0 = si.stage_weights(n, seed=6)
    grads = [si.replica_grads(n, 1, t, seed=6)[0] for t in range(1, steps + 1)]
    one = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=wd)
    one.set_w(w0); one.step(1, [grads[0]], lr)
    want = w0.astype(np.float64) * (1.0 - lr32 * wd32) - lr32 * grads[0].astype(np.float64)
    assert np.array_equal(one.w(0), want.astype(np.float32))
    assert not np.array_equal(one.w(0), (w0.astype(np.float64) - lr32 * grads[0].astype(np.float64)).astype(np.float32))
    orc = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=b1, weight_decay=wd)
    orc.set_w(w0)
    p = torch.nn.Parameter(torch.from_numpy(w0.astype(np.float64)))
    opt = torch.optim.SGD([p], lr=lr32, momentum=b132, foreach=False)
    for t in range(1, steps + 1):
        orc.step(t, [grads[t - 1]], lr)
        with torch.no_grad():
            p.mul_(1.0 - lr32 * wd32)
        p.grad = torch.from_numpy(grads[t - 1].astype(np.float64))
        opt.step()
    want = p.detach().numpy()
    scale = np.maximum(np.abs(want), np.sqrt(np.mean(want ** 2)))
    assert np.max(np.abs(orc.w(0) - want) / scale) < 1e-6
    nodecay = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=b1, weight_decay=0.0)
    nodecay.set_w(w0)
    for t in range(1, steps + 1):
        nodecay.step(t, [grads[t - 1]], lr)
    assert np.max(np.abs(nodecay.w(0) - want) / scale) > 1e-4          # the decay term is not a no-op here


def test_stateless_lookahead_bf16_branch_rounds_once_to_nearest_even():
    """out = w + gamma (w - w_prev) in bf16: on inputs whose exact result fits fp32 (12-bit integers
    times 2^-10, gamma = 0.5) the library's fp32 -> bf16 cast is the one correct rounding, ties
    included; on general inputs the result is the bf16 nearest to the fp64 value."""
    rng = np.random.default_rng(12)
    k1 = rng.integers(-4095, 4096, 5000); k2 = rng.integers(-4095, 4096, 5000)
    w = (k1 * 2.0 ** -10).astype(np.float32); wp = (k2 * 2.0 ** -10).astype(np.float32)
    exact = (3 * k1 - k2) * 2.0 ** -11                                  # 1.5 w - 0.5 w_prev, a 15-bit integer / 2^11
    assert np.array_equal(exact.astype(np.float32).astype(np.float64), exact)
    want = torch.from_numpy(exact.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = O.lookahead(w, wp, 0.5, bf16=True)
    assert np.array_equal(got, want)
    ties = np.abs(exact) * 2.0 ** 11 >= 512                              # more than 8 significant bits: rounding happened
    assert ties.sum() > 1000
    # general inputs: nearest bf16 to the fp64 value (|error| <= half a bf16 ulp) and the fp32 branch agrees
    w = si.stage_weights(4000, seed=3); wp = si.stage_weights(4000, seed=4)
    g = O.f32(0.9)
    x = w.astype(np.float64) + g * (w.astype(np.float64) - wp.astype(np.float64))
    got = si.bf16_bits_to_f32(O.lookahead(w, wp, g, bf16=True)).astype(np.float64)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(x))) - 7)
    assert np.all(np.abs(got - x) <= 0.5 * ulp)
    assert np.array_equal(O.lookahead(w, wp, g), x.astype(np.float32))


def test_first_adamw_step_closed_form():
    """From zero moments, one AdamW step is w(1 - lr wd) - lr g / (|g| + eps)."""
    n, lr, wd, eps = 1000, O.f32(1e-3), O.f32(0.01), O.f32(1e-8)
    w0 = si.stage_weights(n, seed=2)
    g = si.replica_grads(n, 1, 1, seed=2)[0]
    orc = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_ADAMW, weight_decay=0.01)
    orc.set_w(w0)
    orc.step(1, [g], 1e-3)
    w64, g64 = w0.astype(np.float64), g.astype(np.float64)
    want = w64 * (1 - lr * wd) - lr * g64 / (np.abs(g64) + eps)
    assert np.max(np.abs(orc.w(0) - want)) < 1e-7 * 0.02


def test_grad_scale_and_bf16_grads():
    n = 512
    w0 = si.stage_weights(n, seed=3)
    g = si.replica_grads(n, 1, 1, seed=3)[0]
    a = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    a.set_w(w0); a.step(1, [g * np.float32(0.5)], 0.25)
    b = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    b.set_w(w0); b.step(1, [g], 0.25, grad_scale=0.5)
    assert np.array_equal(a.w(0), b.w(0))
    gb = si.to_bf16_bits(g)
    c = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0, grad_bf16=True)
    c.set_w(w0); c.step(1, [gb], 0.25)
    e = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    e.set_w(w0); e.step(1, [si.bf16_bits_to_f32(gb)], 0.25)
    assert np.array_equal(c.w(0), e.w(0))


def test_per_replica_scale_and_gradient_norm():
    """Clipping support: a per-replica factor equals pre-scaled gradients; the squared norm is the
    plain sum of squares."""
    n, R = 700, 3
    w0 = si.stage_weights(n, seed=50)
    g = si.replica_grads(n, R, 1, seed=50)
    scales = np.array([0.5, 0.25, 2.0], dtype=np.float32)           # dyadic: pre-scaling is exact
    a = O.Oracle(n, R, fraction=EMPTY_P, optimizer=O.OPT_ADAMW)
    b = O.Oracle(n, R, fraction=EMPTY_P, optimizer=O.OPT_ADAMW)
    a.set_w(w0); b.set_w(w0)
    a.step(1, g, 1e-3, replica_scale=scales)
    b.step(1, [g[i] * scales[i] for i in range(R)], 1e-3)
    for i in range(R):
        assert np.array_equal(a.w(i), b.w(i)) and np.array_equal(a.v(i), b.v(i))
    assert abs(O.grad_sqnorm(g[0]) - float(np.sum(g[0].astype(np.float64) ** 2))) < 1e-12 * O.grad_sqnorm(g[0])
    gb = si.to_bf16_bits(g[1])
    assert abs(O.grad_sqnorm(gb) - float(np.sum(si.bf16_bits_to_f32(gb).astype(np.float64) ** 2))) < 1e-12 * O.grad_sqnorm(gb)


# --------------------------------------------------------------------------------------------
# synchronous special cases of the averaging (tau = 0)
# --------------------------------------------------------------------------------------------
def test_full_subset_no_delay_is_dense_averaging_and_large_batch_sgd():
    """p = 1, tau = 0: every replica ends on the mean of the local results; with plain SGD from a
    common start that is one SGD step on the mean gradient (synchronous data parallelism)."""
    n, R, lr = 2048, 4, O.f32(0.5)
    w0 = si.stage_weights(n, seed=4)
    orc = O.Oracle(n, R, delay=0, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    orc.set_w(w0)
    w = w0.astype(np.float64)
    for t in range(1, 4):
        g = si.replica_grads(n, R, t, seed=4)
        orc.step(t, g, lr)
        w = w - lr * np.mean(np.stack(g).astype(np.float64), axis=0)
        for i in range(R):
            assert np.max(np.abs(orc.w(i) - w)) < 2e-8      # a few fp32 roundings of values ~0.05
            assert np.array_equal(orc.w(i), orc.w(0))
            assert not np.any(orc.d(i))          # staleness is zero, so the EMA stays zero
    assert orc.consensus_error() == 0.0


def test_no_delay_is_sparta():
    """tau = 0, any p: subset coordinates take the current mean, the others keep the local result."""
    n, R, p, lr, seed = 5000, 3, 0.2, O.f32(0.25), 21
    w0 = np.stack([si.stage_weights(n, seed=10 + i) for i in range(R)])     # replicas already apart
    orc = O.Oracle(n, R, delay=0, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    orc.set_w(w0)
    cur = w0.copy()
    for t in range(1, 4):
        g = np.stack(si.replica_grads(n, R, t, seed=6))
        what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
        S = O.subset(seed, t, n, p).astype(np.int64)
        want = what.copy()
        want[:, S] = np.mean(what[:, S].astype(np.float64), axis=0).astype(np.float32)
        orc.step(t, list(g), lr)
        got = np.stack([orc.w(i) for i in range(R)])
        assert np.array_equal(got, want)
        assert not any(np.any(orc.d(i)) for i in range(R))
        cur = got


def test_sparse_average_shrinks_consensus_error_as_the_lemma_says():
    """After a synchronous sparse average the consensus error is exactly the part carried by the
    coordinates that were not selected, which is (1 - p) of the error before, on expectation."""
    n, R, p, seed = 400_000, 4, 0.1, 5
    w = np.stack([si.stage_weights(n, seed=30 + i) for i in range(R)])
    orc = O.Oracle(n, R, delay=0, fraction=p, seed=seed, optimizer=O.OPT_SGD)
    orc.set_w(w)
    before = orc.consensus_error()
    orc.sparse_average(1)
    after = orc.consensus_error()
    keep = np.ones(n, dtype=bool)
    keep[O.subset(seed, 1, n, p).astype(np.int64)] = False
    w64 = w.astype(np.float64)
    carried = np.sum((w64[:, keep] - w64[:, keep].mean(axis=0)) ** 2)
    assert abs(after - carried) < 1e-6 * carried       # fp32 rounding of the mean only
    assert abs(after / before - (1 - p)) < 0.01


# --------------------------------------------------------------------------------------------
# delayed averaging with EMA correction
# --------------------------------------------------------------------------------------------
def _read_trace(golden_dir):
    rows, extra = [], []
    for l in (golden_dir / "ema_trace_two_replicas.txt").read_text().splitlines():
        if not l.strip() or l.startswith("#"):
            continue
        f = l.split()
        (extra if f[0] in ("none", "diff") else rows).append(f)
    return rows, extra


def _trace_oracle(**kw):
    # look-ahead with gamma = 1: fwd = w + (w^ - w_before), so the local step's result w^ (which the
    # oracle does not hand out) is fwd - w + w_before, exactly, in these dyadic numbers
    orc = O.Oracle(1, 2, delay=1, avg_interval=1, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0,
                   weight_decay=0.0, lookahead=True, gamma=1.0, **kw)
    orc.set_w(np.array([1.0], dtype=np.float32))
    return orc


def test_hand_worked_ema_trace(golden_dir):
    rows, extra = _read_trace(golden_dir)
    orc = _trace_oracle(correction=O.CORR_EMA)
    none = _trace_oracle(correction=O.CORR_NONE)
    diff = _trace_oracle(correction=O.CORR_EMA)
    for r in rows:
        t = int(r[0]); g0, g1, wh0, wh1, w0, w1, d0, d1 = map(float, r[1:])
        grads = [np.array([g0], np.float32), np.array([g1], np.float32)]
        before = (float(orc.w(0)[0]), float(orc.w(1)[0]))
        orc.step(t, grads, 0.5, lam=0.5)
        # the local step's result (what is sent, and what enters the EMA): first line of the
        # asynchronous sparse averaging equation
        assert tuple(float(orc.fwd(i)[0]) - float(orc.w(i)[0]) + before[i] for i in (0, 1)) == (wh0, wh1)
        assert (orc.w(0)[0], orc.w(1)[0]) == (w0, w1)
        assert (orc.d(0)[0], orc.d(1)[0]) == (d0, d1)
        none.step(t, grads, 0.5, lam=0.5)
        for e in extra:
            if e[0] == "none" and int(e[1]) == t:
                assert (none.w(0)[0], none.w(1)[0]) == (float(e[2]), float(e[3]))
        if t <= 2:
            diff.step(t, grads, 0.5, lam=1.0)
            for e in extra:
                if e[0] == "diff" and int(e[1]) == t:
                    assert (diff.w(0)[0], diff.w(1)[0]) == (float(e[2]), float(e[3]))
    # consensus identity of the EMA theorem's proof: w_i - mean w = d_i - mean d on received coordinates
    w = np.array([orc.w(0)[0], orc.w(1)[0]]); d = np.array([orc.d(0)[0], orc.d(1)[0]])
    assert np.array_equal(w - w.mean(), d - d.mean())


def test_nothing_is_received_before_anything_was_sent():
    n, R, tau, K = 600, 3, 2, 2
    w0 = si.stage_weights(n, seed=7)
    orc = O.Oracle(n, R, delay=tau, avg_interval=K, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    ref = O.Oracle(n, R, delay=tau, avg_interval=K, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    orc.set_w(w0); ref.set_w(w0)
    for t in range(1, tau * K + K + 2):
        g = si.replica_grads(n, R, t, seed=7)
        orc.step(t, g, 0.1); ref.step(t, g, 0.1)
        same = all(np.array_equal(orc.w(i), ref.w(i)) for i in range(R))
        # first receive happens at the first averaging step t with t - tau*K >= 1, i.e. t = tau*K + K
        assert same == (t < tau * K + K)


def test_interval_and_delay_in_rounds():
    """K = 2, tau = 1: odd steps are purely local; at t = 4 the mean sent at t = 2 arrives."""
    n, R, p, seed, lr, lam = 800, 2, 0.5, 9, O.f32(0.125), O.f32(0.25)
    w0 = si.stage_weights(n, seed=8)
    orc = O.Oracle(n, R, delay=1, avg_interval=2, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    orc.set_w(w0)
    cur = np.stack([w0] * R)
    whats = {}
    for t in range(1, 5):
        g = np.stack(si.replica_grads(n, R, t, seed=8))
        what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
        whats[t] = what
        want = what.copy()
        if t == 4:
            S = O.subset(seed, 2, n, p).astype(np.int64)
            abar = whats[2][:, S].astype(np.float64).mean(axis=0).astype(np.float32)
            d = (lam * (what[:, S].astype(np.float64) - whats[2][:, S].astype(np.float64))).astype(np.float32)
            want[:, S] = (abar.astype(np.float64) + d.astype(np.float64)).astype(np.float32)
        orc.step(t, list(g), lr, lam=lam)
        got = np.stack([orc.w(i) for i in range(R)])
        assert np.array_equal(got, want), t
        cur = got


def test_lambda_one_leaves_the_replica_mean_untouched():
    """lambda = 1 ("difference only"): w_i[S] = abar_old + w^_i^t - w^_i^old, whose replica mean is
    the current mean of the local results: the sparse step moves no mass."""
    n, R, tau, p = 3000, 4, 2, 0.3
    w0 = si.stage_weights(n, seed=12)
    a = O.Oracle(n, R, delay=tau, fraction=p, seed=1, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    b = O.Oracle(n, R, delay=tau, fraction=EMPTY_P, seed=1, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0)
    a.set_w(w0); b.set_w(w0)
    for t in range(1, 9):
        g = si.replica_grads(n, R, t, seed=12)
        a.step(t, g, 0.05, lam=1.0); b.step(t, g, 0.05, lam=1.0)
        ma = np.mean(np.stack([a.w(i) for i in range(R)]).astype(np.float64), axis=0)
        mb = np.mean(np.stack([b.w(i) for i in range(R)]).astype(np.float64), axis=0)
        assert np.max(np.abs(ma - mb)) < 2e-8


def test_consensus_identity_on_received_subset():
    n, R, tau, p, seed = 4000, 5, 3, 0.25, 77
    w0 = si.stage_weights(n, seed=13)
    orc = O.Oracle(n, R, delay=tau, fraction=p, seed=seed, optimizer=O.OPT_ADAMW)
    orc.set_w(w0)
    for t in range(1, 11):
        orc.step(t, si.replica_grads(n, R, t, seed=13), 1e-3, lam=0.5)
        if t > tau:
            S = O.subset(seed, t - tau, n, p).astype(np.int64)
            w = np.stack([orc.w(i)[S] for i in range(R)]).astype(np.float64)
            d = np.stack([orc.d(i)[S] for i in range(R)]).astype(np.float64)
            assert np.max(np.abs((w - w.mean(0)) - (d - d.mean(0)))) < 5e-9


def test_identical_replicas_stay_identical():
    n, R = 1000, 3
    w0 = si.stage_weights(n, seed=14)
    orc = O.Oracle(n, R, delay=2, fraction=0.3, seed=4, optimizer=O.OPT_ADAMW)
    orc.set_w(w0)
    for t in range(1, 8):
        g = si.replica_grads(n, 1, t, seed=14)[0]
        orc.step(t, [g] * R, 1e-3)
        for i in range(1, R):
            assert np.array_equal(orc.w(i), orc.w(0)) and np.array_equal(orc.d(i), orc.d(0))
    assert np.any(orc.d(0))


def test_ema_closed_form_under_constant_staleness():
    """If the local weights advance by the same c between send and receive on every visit, the EMA
    after n visits is c (1 - (1 - lambda)^n)."""
    c, lam = 0.25, 0.5
    orc = O.Oracle(1, 1, delay=1, fraction=1.0, optimizer=O.OPT_SGD)
    for t in range(1, 9):
        orc.w(0)[0] = np.float32(1.0 + c * t) if t == 1 else np.float32(orc.w(0)[0])
        if t > 1:
            # replace the averaged value by "previous local value + c": local progress of exactly c
            orc.w(0)[0] = np.float32(prev_local + c)
        prev_local = float(orc.w(0)[0])
        orc.sparse_average(t, lam=lam)
        visits = t - 1
        assert orc.d(0)[0] == c * (1 - (1 - lam) ** visits)
        if visits:
            assert orc.w(0)[0] == np.float32((prev_local - c) + orc.d(0)[0])     # old mean + EMA


def test_no_correction_is_plain_delayed_averaging():
    n, R, tau, p, seed, lr = 1500, 3, 2, 0.4, 15, O.f32(0.125)
    w0 = si.stage_weights(n, seed=15)
    orc = O.Oracle(n, R, delay=tau, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0,
                   correction=O.CORR_NONE)
    orc.set_w(w0)
    cur, whats = np.stack([w0] * R), {}
    for t in range(1, 7):
        g = np.stack(si.replica_grads(n, R, t, seed=15))
        what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
        whats[t] = what
        want = what.copy()
        if t > tau:
            S = O.subset(seed, t - tau, n, p).astype(np.int64)
            want[:, S] = whats[t - tau][:, S].astype(np.float64).mean(axis=0).astype(np.float32)
        orc.step(t, list(g), lr)
        cur = np.stack([orc.w(i) for i in range(R)])
        assert np.array_equal(cur, want)
        assert not any(np.any(orc.d(i)) for i in range(R))


def test_eager_mode_is_fresh_own_plus_stale_others():
    """Eager-DiLoCo special case (all parameters, d_i = (1/m)(w^_i^t - w^_i^{t-tau})): every replica
    ends on the average in which its own contribution is fresh and the others' are tau rounds old."""
    n, R, tau, lr = 700, 4, 2, O.f32(0.125)
    w0 = si.stage_weights(n, seed=18)
    orc = O.Oracle(n, R, delay=tau, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0,
                   correction=O.CORR_EAGER)
    orc.set_w(w0)
    cur, whats = np.stack([w0] * R), {}
    for t in range(1, 7):
        g = np.stack(si.replica_grads(n, R, t, seed=18))
        what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
        whats[t] = what
        orc.step(t, list(g), lr)
        got = np.stack([orc.w(i) for i in range(R)])
        if t > tau:
            old = whats[t - tau].astype(np.float64)
            want = (old.sum(axis=0)[None, :] - old + what.astype(np.float64)) / R
            assert np.max(np.abs(got - want)) < 2e-8
        else:
            assert np.array_equal(got, what)
        cur = got


def test_delay_can_change_at_run_time():
    """A late average: with the delay lowered from 3 to 1 for one step, that step receives what was
    sent one round ago; raised back, it receives the three-round-old average again."""
    n, R, p, seed, lr = 900, 2, 0.5, 31, O.f32(0.125)
    w0 = si.stage_weights(n, seed=19)
    orc = O.Oracle(n, R, delay=3, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0,
                   correction=O.CORR_NONE)
    orc.set_w(w0)
    cur, whats = np.stack([w0] * R), {}
    delays = {1: 3, 2: 3, 3: 3, 4: 3, 5: 1, 6: 3, 7: 0, 8: 2}
    for t in range(1, 9):
        orc.set_delay(delays[t])
        g = np.stack(si.replica_grads(n, R, t, seed=19))
        what = (cur.astype(np.float64) - lr * g.astype(np.float64)).astype(np.float32)
        whats[t] = what
        want = what.copy()
        s_ = t - delays[t]
        if s_ >= 1:
            S = O.subset(seed, s_, n, p).astype(np.int64)
            want[:, S] = whats[s_][:, S].astype(np.float64).mean(axis=0).astype(np.float32)
        orc.step(t, list(g), lr)
        cur = np.stack([orc.w(i) for i in range(R)])
        assert np.array_equal(cur, want), t
    with pytest.raises(ValueError):
        orc.set_delay(4)


def test_ema_variance_diagnostic():
    n, R = 3000, 5
    orc = O.Oracle(n, R, delay=1, fraction=0.5, seed=2, optimizer=O.OPT_ADAMW)
    orc.set_w(si.stage_weights(n, seed=20))
    for t in range(1, 6):
        orc.step(t, si.replica_grads(n, R, t, seed=20), 1e-3)
    d = np.stack([orc.d(i) for i in range(R)]).astype(np.float64)
    var = d.var(axis=0)                                   # population variance over the replicas
    mean_, max_ = orc.ema_variance()
    assert abs(mean_ - var.mean()) < 1e-12 * var.mean() + 1e-30 and abs(max_ - var.max()) < 1e-12 * var.max()
    w = np.stack([orc.w(i) for i in range(R)]).astype(np.float64)
    assert abs(orc.consensus_error() - np.sum((w - w.mean(axis=0)) ** 2)) < 1e-10 * orc.consensus_error()


# --------------------------------------------------------------------------------------------
# look-ahead
# --------------------------------------------------------------------------------------------
def test_lookahead_scalars():
    # w_old = 1, g = 0.5, lr = 0.5 -> w^ = 0.75, displacement -0.25; gamma = 0.5 -> fwd = 0.625
    orc = O.Oracle(1, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0, lookahead=True, gamma=0.5)
    orc.set_w(np.array([1.0], np.float32))
    orc.step(1, [np.array([0.5], np.float32)], 0.5)
    assert orc.w(0)[0] == 0.75 and orc.fwd(0)[0] == 0.625
    # on a received coordinate only the optimizer's displacement is extrapolated, not the averaging jump:
    # second step of the hand-worked trace: w = 0.875, displacement 0.5 - 0.75 = -0.25 -> fwd = 0.75
    tr = O.Oracle(1, 2, delay=1, fraction=1.0, optimizer=O.OPT_SGD, beta1=0.0, weight_decay=0.0, lookahead=True, gamma=0.5)
    tr.set_w(np.array([1.0], np.float32))
    tr.step(1, [np.array([0.5], np.float32), np.array([-0.5], np.float32)], 0.5)
    tr.step(2, [np.array([0.5], np.float32), np.array([0.5], np.float32)], 0.5)
    assert tr.w(0)[0] == 0.875 and tr.fwd(0)[0] == 0.75
    # gamma = 0 and look-ahead off both give fwd = w
    z = O.Oracle(4, 1, fraction=EMPTY_P, optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.0)
    z.set_w(si.stage_weights(4, seed=1)); z.step(1, si.replica_grads(4, 1, 1), 1e-3)
    assert np.array_equal(z.fwd(0), z.w(0))
    # stateless two-point form
    out = O.lookahead(np.array([0.75], np.float32), np.array([1.0], np.float32), 0.5)
    assert out[0] == 0.625


def test_explicit_lookahead_is_nesterov_momentum():
    """Heavy-ball SGD whose gradient is taken at fwd = w + gamma (w^ - w_prev) is textbook Nesterov
    momentum  v <- mu v - lr grad f(w + mu v),  w <- w + v  (here f(w) = w^2 / 2, grad f = identity)."""
    mu, lr, steps = 0.5, 0.25, 12
    w0 = np.array([1.0, -2.0, 0.5], dtype=np.float32)
    orc = O.Oracle(3, 1, fraction=EMPTY_P, optimizer=O.OPT_SGD, beta1=mu, weight_decay=0.0, lookahead=True, gamma=mu)
    orc.set_w(w0)
    w, v = w0.astype(np.float64), np.zeros(3)
    point = w0.copy()                                   # first gradient is taken at w0 (v = 0)
    for t in range(1, steps + 1):
        orc.step(t, [point.copy()], lr)                 # grad f at the look-ahead point
        point = orc.fwd(0).copy()
        v = mu * v - lr * (w + mu * v)
        w = w + v
        assert np.max(np.abs(orc.w(0) - w)) < 1e-6
        assert np.max(np.abs(orc.fwd(0) - (w + mu * v))) < 1e-6


def test_bf16_forward_copy():
    n = 2000
    w0 = si.stage_weights(n, seed=16)
    a = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.9, fwd_bf16=True)
    b = O.Oracle(n, 1, fraction=EMPTY_P, optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.9)
    a.set_w(w0); b.set_w(w0)
    g = si.replica_grads(n, 1, 1, seed=16)
    a.step(1, g, 1e-3); b.step(1, g, 1e-3)
    assert np.array_equal(a.w(0), b.w(0))
    f = a.fwd(0)
    assert np.array_equal(si.bf16_bits_to_f32(si.to_bf16_bits(f)), f)       # representable in bf16
    assert np.max(np.abs(f - b.fwd(0)) / np.abs(b.fwd(0))) <= 2.0 ** -8     # within half a bf16 ulp


def test_step_order_is_enforced():
    orc = O.Oracle(4, 1)
    with pytest.raises(ValueError):
        orc.step(2, si.replica_grads(4, 1, 1), 1e-3)


def test_oracle_is_clean_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Host-side check of the checker itself: every mode on small ragged sizes, no out-of-bounds
    access, no undefined behaviour, no leak."""
    import os
    import subprocess
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    exe = tmp_path / "drive"
    subprocess.run(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
                    "-I", str(root / "oracle"), "-o", str(exe), str(root / "tests" / "oracle_sanitizer_driver.c"), "-lm"], check=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1", OMP_NUM_THREADS="2")
    out = subprocess.run([str(exe)], capture_output=True, text=True, env=env)
    if out.returncode != 0 and "AddressSanitizer" in out.stderr and "runtime does not come first" in out.stderr:
        pytest.skip("the sanitizer runtime cannot start in this environment")
    assert out.returncode == 0, out.stderr[-2000:]
    assert len(out.stdout.splitlines()) == 30
