"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element, on the same
seeded inputs.  Bar: subset indices bit-exact; fp32 values within 1e-6 relative, bf16 outputs
within 1e-2 relative, both measured against max(|ref|, rms(ref))."""
import numpy as np
import pytest
import torch

import synth_inputs as si
from oracle import oracle as O

pytestmark = pytest.mark.gpu

TOL_F32 = 1e-6
TOL_BF16 = 1e-2
EMPTY_P = 1e-12

# memory layout of the EMA vectors: one array per replica, or replicas interleaved per coordinate;
# tests that do not name one run with the interleaved layout (the benchmark's)
PER_REPLICA, INTERLEAVED = 0, 1
both_layouts = pytest.mark.parametrize("d_layout", [pytest.param(PER_REPLICA, id="d_per_replica"),
                                                    pytest.param(INTERLEAVED, id="d_interleaved")])


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    got = got.astype(np.float64); ref = ref.astype(np.float64)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref ** 2)))
    if rms == 0.0:
        return 0.0 if not np.any(got) else float("inf")
    return float(np.max(np.abs(got - ref) / np.maximum(np.abs(ref), rms)))


def make_pair(am, n, R, w0=None, fwd_bf16=False, grad_bf16=False, force_fwd=False, **kw):
    """A GPU stage and an oracle with the same configuration and starting weights.  kw holds the
    configuration fields that carry the same name (and the same enum values) on both sides."""
    if w0 is None:
        w0 = si.stage_weights(n, kw.get("seed", 0))
    kw = dict(kw)
    d_layout = kw.pop("d_layout", INTERLEAVED)          # a layout changes no value: the oracle has none
    cfg = am.make_config(n, R, fwd_dtype=am.BF16 if fwd_bf16 else am.F32,
                         grad_dtype=am.BF16 if grad_bf16 else am.F32, d_layout=d_layout, **kw)
    with_fwd = bool(kw.get("lookahead", False)) or fwd_bf16 or force_fwd
    st = am.init_state(cfg, torch.from_numpy(np.ascontiguousarray(w0)).cuda(), with_fwd=with_fwd)
    orc = O.Oracle(n, R, fwd_bf16=fwd_bf16, grad_bf16=grad_bf16, **kw)
    orc.set_w(w0)
    return st, orc


def grads_for(n, R, t, seed, bf16):
    g = si.replica_grads(n, R, t, seed)
    if bf16:
        g = [si.to_bf16_bits(x) for x in g]
        dev = [torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16) for x in g]
    else:
        dev = [torch.from_numpy(x).cuda() for x in g]
    return g, dev


def compare(st, orc, where=""):
    R = orc.R
    worst = {}
    for i in range(R):
        for name in ("w", "m", "v", "d"):
            ts = getattr(st, name)
            if ts is None:
                continue
            e = rel_err(ts[i].cpu().numpy(), getattr(orc, name)(i))
            worst[name] = max(worst.get(name, 0.0), e)
            assert e < TOL_F32, f"{where} {name}[{i}] rel err {e:.3e}"
        if st.fwd is not None:
            bf = st.fwd[i].dtype == torch.bfloat16
            got = st.fwd[i].float().cpu().numpy()
            e = rel_err(got, orc.fwd(i))
            worst["fwd"] = max(worst.get("fwd", 0.0), e)
            assert e < (TOL_BF16 if bf else TOL_F32), f"{where} fwd[{i}] rel err {e:.3e}"
            if bf:
                fresh = not st.cfg.lookahead and not getattr(st, "fwd_is_stale", False)     # fwd = bf16(w) right after a fused step
                check_bf16_rounded_once(got, orc.fwd(i), st.w[i].cpu().numpy() if fresh else None, f"{where} fwd[{i}]")
    assert st.read_flags() == 0
    return worst


def check_bf16_rounded_once(got, ref, w_gpu, where):
    """bf16 outputs are the ONE rounding of the fp64 value.  They can differ from the oracle's only
    where the fp32 quantities behind them already differ in their last bit (the refined square root
    and quotient are not correctly rounded), which moves a bf16 result with probability 2^-16 each:
    so almost every element is bit-equal, no element is more than one bf16 step off, and without
    look-ahead the output is exactly the bf16 rounding of the GPU's own fp32 weights."""
    if got.size == 0:
        return
    diff = got != ref
    assert diff.mean() <= 1e-3, f"{where}: {int(diff.sum())} of {got.size} bf16 values differ from the oracle's"
    if diff.any():
        step = np.abs(ref[diff]).astype(np.float64) * 2.0 ** -7      # at most one step of 8 significant bits
        assert np.all(np.abs(got[diff].astype(np.float64) - ref[diff]) <= step), where
    if w_gpu is not None:
        assert np.array_equal(got, si.bf16_bits_to_f32(si.to_bf16_bits(w_gpu))), where


def run_steps(am, n, R, steps, lr=3e-4, lam=0.5, grad_scale=1.0, check_every=1, **kw):
    print(f"case n={n} R={R} steps={steps} {kw}", flush=True)
    st, orc = make_pair(am, n, R, **kw)
    bf = kw.get("grad_bf16", False)
    for t in range(1, steps + 1):
        g, gd = grads_for(n, R, t, kw.get("seed", 0), bf)
        st.step(t, gd, lr, lam, grad_scale)
        orc.step(t, g, lr, lam, grad_scale)
        if t % check_every == 0 or t == steps:
            worst = compare(st, orc, f"n={n} R={R} t={t} {kw}")
    print("  worst rel err at last step:", {k: f"{v:.1e}" for k, v in worst.items()}, flush=True)
    return st, orc


# --------------------------------------------------------------------------------------------
# subset indices: bit exact
# --------------------------------------------------------------------------------------------
@pytest.mark.parametrize("n,p,seed", [
    (1, 1.0, 0), (3, 0.5, 1), (255, 0.3, 2), (256, 0.05, 3), (257, 0.05, 3), (100_003, 0.05, 0),
    (131_072 * 3 + 5, 0.01, 7), (1_048_576, 0.05, 0), (2_000_000, 0.10, 0xDEADBEEF12345678),
    (70_001, 1.0, 5), (70_001, EMPTY_P, 5),
])
def test_subset_indices_bit_exact(amlib, n, p, seed):
    am = amlib
    cfg = am.make_config(n, 1, fraction=p, seed=seed, optimizer=am.OPT_SGD, beta1=0.0, correction=am.CORR_NONE)
    st = am.init_state(cfg, torch.zeros(n))
    for t in (0, 1, 2, 1000, (1 << 32) + 5):
        idx, k = st.subset_indices(t)
        want = O.subset(seed, t, n, p)
        assert k == want.size
        assert np.array_equal(idx.cpu().numpy().astype(np.uint64), want), (n, p, seed, t)
    # truncated output keeps the ascending prefix and still reports the full count
    idx, k = st.subset_indices(1, capacity=10)
    want = O.subset(seed, 1, n, p)
    assert k == want.size and np.array_equal(idx.cpu().numpy().astype(np.uint64), want[:10])


def test_subset_indices_beyond_2_to_30(amlib):
    """n > 2^30: every index produced satisfies the oracle's predicate, and windows of the stage
    match the oracle's enumeration exactly."""
    am = amlib
    n, p, seed, t = (1 << 30) + 12_345, 2e-4, 9, 3
    cfg = am.make_config(n, 1, fraction=p, seed=seed, optimizer=am.OPT_SGD, beta1=0.0, correction=am.CORR_NONE)
    st = am.init_state(cfg, None)
    idx, k = st.subset_indices(t, capacity=400_000)
    got = idx.cpu().numpy().astype(np.uint64)
    assert k == got.size and np.all(np.diff(got.astype(np.int64)) > 0) and got[-1] < n
    rng = np.random.default_rng(0)
    for mu in rng.choice(got, 300, replace=False):
        assert O.member(seed, t, int(mu), p)
    for lo in (0, (1 << 30) - 70_000, n - 200_000, 536_870_912 - 1000):
        ln = min(200_000, n - lo)
        want = O.subset(seed, t, ln, p, mu0=lo)
        assert np.array_equal(got[(got >= lo) & (got < lo + ln)], want)
    assert abs(k - n * p) < 6 * (n * p) ** 0.5


# --------------------------------------------------------------------------------------------
# fused step
# --------------------------------------------------------------------------------------------
@both_layouts
def test_config_tiny(amlib, d_layout):
    """1,048,576 fp32 params, R=4, staleness 1, 5 % per step, Adam-style state, 10 steps, seed 0."""
    st, orc = run_steps(amlib, 1_048_576, 4, 10, delay=1, fraction=0.05, seed=0, optimizer=O.OPT_ADAMW, d_layout=d_layout)
    assert any(np.any(orc.d(i)) for i in range(4))           # the EMA path did real work


@pytest.mark.parametrize("n", [1, 2, 3, 4, 5, 255, 256, 257, 1023, 4099, 131_072 + 7, 3 * 131_072 + 1])
@both_layouts
def test_ragged_sizes(amlib, n, d_layout):
    run_steps(amlib, n, 3, 5, delay=1, fraction=0.3, seed=n, optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.9, d_layout=d_layout)


@both_layouts
@pytest.mark.parametrize("R", [1, 2, 3, 4, 5, 7, 8, 9, 12, 16, 17, 24, 31, 32])
def test_replica_counts(amlib, R, d_layout):
    run_steps(amlib, 10_007, R, 6, delay=2, fraction=0.2, seed=R, optimizer=O.OPT_ADAMW, d_layout=d_layout)


@both_layouts
@pytest.mark.parametrize("R", [9, 16, 20, 32])
def test_more_than_one_block_of_replicas_without_delay(amlib, R, d_layout):
    """tau = 0 with more than 8 replicas: one workgroup walks all the blocks of its tile."""
    run_steps(amlib, 20_011, R, 5, delay=0, fraction=0.2, seed=R, optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.9,
              d_layout=d_layout)
    run_steps(amlib, 5_003, R, 4, delay=0, avg_interval=2, fraction=1.0, seed=R, optimizer=O.OPT_SGD, beta1=0.9,
              d_layout=d_layout)


@pytest.mark.parametrize("tau,K", [(0, 1), (0, 3), (1, 1), (1, 2), (3, 1), (2, 3), (7, 1)])
@both_layouts
def test_delay_and_interval(amlib, tau, K, d_layout):
    run_steps(amlib, 20_011, 4, 3 * (tau + 1) * K + 2, delay=tau, avg_interval=K, fraction=0.25, seed=5,
              optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.5, d_layout=d_layout)


@pytest.mark.parametrize("p", [EMPTY_P, 0.01, 0.05, 0.5, 1.0])
@both_layouts
def test_fractions(amlib, p, d_layout):
    run_steps(amlib, 50_021, 4, 6, delay=1, fraction=p, seed=3, optimizer=O.OPT_ADAMW, d_layout=d_layout)
    run_steps(amlib, 50_021, 8, 4, delay=1, fraction=p, seed=4, optimizer=O.OPT_ADAMW, d_layout=d_layout)


@pytest.mark.parametrize("opt,b1", [(O.OPT_SGD, 0.0), (O.OPT_SGD, 0.9), (O.OPT_ADAMW, 0.9), (O.OPT_ADAMW, 0.99),
                                    (O.OPT_NADAMW, 0.99)])
@pytest.mark.parametrize("corr", [O.CORR_NONE, O.CORR_EMA])
@both_layouts
def test_optimizers_and_corrections(amlib, opt, b1, corr, d_layout):
    run_steps(amlib, 30_011, 3, 8, lr=1e-3, delay=2, fraction=0.2, seed=11, optimizer=opt, beta1=b1,
              correction=corr, lookahead=True, gamma=0.9, weight_decay=0.01, d_layout=d_layout)


def test_block_granule_variant(amlib):
    """Variant sampling: aligned blocks of 32 coordinates drawn as a whole (indices and values)."""
    am = amlib
    n, p, seed = 300_007, 0.07, 5
    st, orc = run_steps(am, n, 4, 8, delay=2, fraction=p, seed=seed, subset_granule=32, lookahead=True, gamma=0.9)
    for t in (1, 5, (1 << 33) + 2):
        idx, k = st.subset_indices(t)
        want = O.subset(seed, t, n, p, granule=32)
        assert k == want.size and np.array_equal(idx.cpu().numpy().astype(np.uint64), want)
    run_steps(am, 1000, 3, 6, delay=0, fraction=0.3, seed=2, subset_granule=32)
    run_steps(am, 4099, 8, 6, delay=1, fraction=1.0, seed=2, subset_granule=32)

@pytest.mark.parametrize("p", [0.05, 0.3, 0.6, 1.0 / 256, 1.0 / 1000, 1.0])
def test_stratified_variant(amlib, p):
    """Variant sampling: exactly one coordinate of every aligned block of round(1/p) (indices bit-exact,
    state to the fp32 bar); block lengths below, at and above the tile length, and a cut last block."""
    am = amlib
    n, seed = 300_007, 5
    st, orc = run_steps(am, n, 4, 8, delay=2, fraction=p, seed=seed, subset_kind=am.SUBSET_STRATIFIED,
                        lookahead=True, gamma=0.9)
    B = O.block_size(p)
    for t in (1, 5, (1 << 33) + 2):
        idx, k = st.subset_indices(t)
        want = O.subset(seed, t, n, p, stratified=True)
        assert k == want.size and np.array_equal(idx.cpu().numpy().astype(np.uint64), want)
        assert n // B <= k <= n // B + 1
    run_steps(am, 1000, 3, 6, delay=0, fraction=p, seed=2, subset_kind=am.SUBSET_STRATIFIED)
    run_steps(am, 4099, 8, 6, delay=1, fraction=p, seed=2, subset_kind=am.SUBSET_STRATIFIED, correction=am.CORR_NONE)


def test_stratified_variant_sparse_average_entry(amlib):
    am = amlib
    n, R, p = 77_003, 4, 0.05
    st, orc = make_pair(am, n, R, delay=1, fraction=p, seed=8, subset_kind=am.SUBSET_STRATIFIED)
    rng = np.random.default_rng(5)
    for t in range(1, 6):
        w = [(orc.w(i) + rng.normal(0, 1e-3, n).astype(np.float32)) for i in range(R)]
        for i in range(R):
            orc.w(i)[:] = w[i]
            st.w[i].copy_(torch.from_numpy(w[i]))
        st.sparse_average(t, 0.5); orc.sparse_average(t, 0.5)
    compare(st, orc, "stratified sparse_average")



@pytest.mark.parametrize("msg", [O.MSG_BF16, O.MSG_E4M3])
@pytest.mark.parametrize("tau", [0, 2])
def test_quantised_exchange(amlib, msg, tau):
    run_steps(amlib, 60_013, 4, 3 * (tau + 1) + 2, delay=tau, fraction=0.2, seed=14, msg_dtype=msg, lookahead=True, gamma=0.9)


@pytest.mark.parametrize("bf16", [False, True])
def test_clipping_by_each_replica_s_own_norm(amlib, bf16):
    """Global-norm clipping at 1 without leaving the device: squared norms from am_grad_sqnorm, factors
    min(1, 1/norm) formed on the device, applied per replica by am_step_scaled."""
    n, R = 90_001, 4
    st, orc = make_pair(amlib, n, R, delay=1, fraction=0.1, seed=33, grad_bf16=bf16, lookahead=True, gamma=0.9)
    for t in range(1, 6):
        g, gd = grads_for(n, R, t, 33, bf16)
        g = [x * (np.float32(40.0 * (i + 1)) if not bf16 else 1) for i, x in enumerate(g)]      # norms around 1
        if not bf16:
            gd = [torch.from_numpy(x).cuda() for x in g]
        sq = st.grad_sqnorm(gd)
        want = np.array([O.grad_sqnorm(x) for x in g])
        assert np.max(np.abs(sq.cpu().numpy() - want) / want) < 1e-12
        scale = torch.clamp(1.0 / sq.sqrt(), max=1.0).to(torch.float32)
        st.step_scaled(t, gd, 1e-3, 0.5, 1.0, scale)
        orc.step(t, g, 1e-3, 0.5, 1.0, replica_scale=scale.cpu().numpy())
        compare(st, orc, f"clipping t={t}")
    assert bf16 or float(scale.min()) < 1.0                      # clipping was active


def test_eager_correction_mode(amlib):
    run_steps(amlib, 25_013, 4, 9, delay=2, fraction=1.0, seed=4, correction=O.CORR_EAGER)
    run_steps(amlib, 25_013, 3, 9, delay=1, avg_interval=2, fraction=0.3, seed=4, correction=O.CORR_EAGER,
              lookahead=True, gamma=0.9)


def test_delay_changed_at_run_time(amlib):
    """Late and early averages: the delay in force changes from step to step within the ring's depth."""
    n, R = 33_333, 4
    st, orc = make_pair(amlib, n, R, delay=3, fraction=0.2, seed=6, lookahead=True, gamma=0.9)
    delays = [3, 3, 3, 3, 1, 3, 0, 2, 2, 3, 0, 0, 1, 3]
    for t, tau in enumerate(delays, start=1):
        st.set_delay(tau); orc.set_delay(tau)
        g, gd = grads_for(n, R, t, 6, False)
        st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
        compare(st, orc, f"t={t} tau={tau}")
    with pytest.raises(amlib.AsyncMeshError):
        st.set_delay(4)


@pytest.mark.parametrize("n,R", [(123_457, 5), (1003, 1), (70_001, 2), (70_002, 3), (33_333, 12), (33_331, 20), (10_007, 32)])
@both_layouts
def test_diagnostics(amlib, n, R, d_layout):
    st, orc = make_pair(amlib, n, R, delay=1, fraction=0.3, seed=12, d_layout=d_layout)
    for t in range(1, 6):
        g, gd = grads_for(n, R, t, 12, False)
        st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
    cons, vmean, vmax = st.diagnostics()
    ovm, ovx = orc.ema_variance()
    assert abs(cons - orc.consensus_error()) <= 1e-9 * orc.consensus_error()
    assert abs(vmean - ovm) <= 1e-9 * ovm and abs(vmax - ovx) <= 1e-9 * ovx
    assert st.diagnostics() == (cons, vmean, vmax)                 # fixed reduction order
    if R == 1:
        assert (cons, vmean, vmax) == (0.0, 0.0, 0.0)              # one replica: nothing to disagree with


def test_diagnostics_without_a_correction_vector(amlib):
    st2, orc2 = make_pair(amlib, 1000, 2, delay=1, fraction=0.3, seed=12, correction=O.CORR_NONE)
    assert st2.diagnostics() == (0.0, 0.0, 0.0)                    # identical replicas, no correction vector


def test_lambda_and_grad_scale(amlib):
    run_steps(amlib, 12_345, 4, 6, lam=1.0, grad_scale=0.25, delay=1, fraction=0.3, seed=2)
    run_steps(amlib, 12_345, 4, 6, lam=0.01, delay=1, fraction=0.3, seed=2)
    run_steps(amlib, 12_345, 4, 6, lam=0.0, delay=1, fraction=0.3, seed=2)


@pytest.mark.parametrize("fwd_bf16,grad_bf16,look", [(True, True, True), (True, False, False), (False, True, True),
                                                     (False, False, False)])
@both_layouts
def test_dtypes(amlib, fwd_bf16, grad_bf16, look, d_layout):
    run_steps(amlib, 40_009, 4, 6, delay=1, fraction=0.1, seed=8, fwd_bf16=fwd_bf16, grad_bf16=grad_bf16,
              lookahead=look, gamma=0.9, force_fwd=True, d_layout=d_layout)


@both_layouts
def test_config_small_model_stage(amlib, d_layout):
    """12 d^2 = 7,077,888 params (d=768), R=4, staleness 2, 10 %, look-ahead on, 100 steps."""
    run_steps(amlib, 7_077_888, 4, 100, check_every=25, delay=2, fraction=0.10, seed=0,
              optimizer=O.OPT_ADAMW, lookahead=True, gamma=0.9, d_layout=d_layout)


@both_layouts
def test_config_bf16_stage_reduced(amlib, d_layout):
    """bf16 gradients and forward weights over fp32 masters, R=16, staleness 8, 1 % (the large
    configuration's settings on a stage the oracle finishes in seconds)."""
    run_steps(amlib, 1_000_003, 16, 12, check_every=4, delay=8, fraction=0.01, seed=0, fwd_bf16=True,
              grad_bf16=True, d_layout=d_layout)


def test_wide_dynamic_range(amlib):
    """Gradients over 24 decades (second moments down into the fp32 subnormals), weights over 8: the
    refined square root / quotient and the fp64 accumulations must still land on the oracle's values."""
    n, R, seed = 65_537, 3, 77
    rng = np.random.default_rng(seed)
    w0 = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 2, n)).astype(np.float32)
    st, orc = make_pair(amlib, n, R, w0=w0, delay=1, fraction=0.3, seed=seed, lookahead=True, gamma=0.9)
    for t in range(1, 7):
        g = [(rng.standard_normal(n) * 10.0 ** rng.uniform(-21, 3, n)).astype(np.float32) for _ in range(R)]
        if t == 3:
            g[0][::7] = 0.0                                     # exact zeros: v stays where it decays to
        gd = [torch.from_numpy(x).cuda() for x in g]
        st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
        for i in range(R):
            for name in ("w", "m", "v", "d", "fwd"):
                got = getattr(st, name)[i].cpu().numpy(); ref = getattr(orc, name)(i)
                assert np.all(np.isfinite(got)) and np.all(np.isfinite(ref))
                # element-wise relative error with a floor of one fp32 subnormal step
                err = np.abs(got.astype(np.float64) - ref.astype(np.float64)) / (np.abs(ref.astype(np.float64)) + 1.5e-45)
                if name in ("m", "v"):
                    assert np.max(err) < 1e-6, (t, i, name, float(np.max(err)))
                else:
                    assert rel_err(got, ref) < TOL_F32, (t, i, name)


def test_replicas_apart_from_the_start(amlib):
    n, R = 9_001, 4
    w0 = np.stack([si.stage_weights(n, 40 + i) for i in range(R)])
    st, orc = make_pair(amlib, n, R, w0=w0, delay=1, fraction=0.5, seed=1)
    for t in range(1, 6):
        g, gd = grads_for(n, R, t, 1, False)
        st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
    compare(st, orc)


# --------------------------------------------------------------------------------------------
# full-size stage, sampled: the 125M-parameter configuration in the benchmark's launch shape
# --------------------------------------------------------------------------------------------
def _free_hbm() -> int:
    """Free device memory after giving back what earlier tests left in torch's caching allocator."""
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    return torch.cuda.mem_get_info()[0]


def _tiled_dev(pool_dev, n, offset):
    reps = (n + offset) // pool_dev.numel() + 2
    return pool_dev.repeat(reps)[offset:offset + n].clone()


def _full_size_case(am, n, R, tau, p, steps, windows, bf16=False, lookahead=True, seed=0, optimizer=O.OPT_ADAMW,
                    beta1=0.9, d_layout=INTERLEAVED, whole_subset=False):
    """Run `steps` fused steps of a full-size stage in the launch shape the benchmark times and compare
    windows of it with oracle instances that evaluate just those coordinate ranges (exact: the
    method is coordinate-wise given (seed, step, global coordinate)).  windows = "all": consecutive
    windows that cover every coordinate of the stage, replayed one after the other once the GPU is done."""
    pool_n = 1 << 20
    w_pool = si.stage_weights(pool_n, seed)
    cfg = am.make_config(n, R, delay=tau, fraction=p, seed=seed, lookahead=lookahead, gamma=0.9,
                         optimizer=optimizer, beta1=beta1, d_layout=d_layout,
                         fwd_dtype=am.BF16 if bf16 else am.F32, grad_dtype=am.BF16 if bf16 else am.F32)
    st = am.init_state(cfg, _tiled_dev(torch.from_numpy(w_pool).cuda(), n, 0))
    sweep = windows == "all"
    if sweep:
        ln = 3_000_017                                   # not a multiple of the tile: window edges fall inside tiles
        windows = [(lo, min(ln, n - lo)) for lo in range(0, n, ln)]

    def make_oracle(lo, ln):
        orc = O.Oracle(ln, R, delay=tau, fraction=p, seed=seed, lookahead=lookahead, gamma=0.9, mu0=lo,
                       optimizer=optimizer, beta1=beta1, fwd_bf16=bf16, grad_bf16=bf16)
        orc.set_w(si.tiled(w_pool, ln, lo))
        return orc

    def step_inputs(t):
        pools = si.replica_grads(pool_n, R, t, seed)
        if bf16:
            pools = [si.to_bf16_bits(x) for x in pools]
        return pools, [(7919 * (i + 1) * t) % pool_n for i in range(R)]

    def check_window(lo, ln, orc):
        for i in range(R):
            for name in ("w", "m", "v", "d", "fwd"):
                if getattr(st, name) is None:
                    continue
                got = getattr(st, name)[i][lo:lo + ln].float().cpu().numpy()
                ref = getattr(orc, name)(i)
                e = rel_err(got, ref)
                tol = TOL_BF16 if (bf16 and name == "fwd") else TOL_F32
                assert e < tol, f"window {lo} {name}[{i}] rel err {e:.3e}"
                if bf16 and name == "fwd":
                    check_bf16_rounded_once(got, ref, None if lookahead else st.w[i][lo:lo + ln].cpu().numpy(),
                                            f"window {lo} fwd[{i}]")

    oracles = [] if sweep else [make_oracle(lo, ln) for lo, ln in windows]
    inputs = {}
    for t in range(1, steps + 1):
        print(f"  full-size n={n} R={R} step {t}", flush=True)
        pools, offs = step_inputs(t)
        if sweep:
            inputs[t] = (pools, offs)
        gd = []
        for i in range(R):
            dev = torch.from_numpy(pools[i].view(np.int16) if bf16 else pools[i]).cuda()
            g = _tiled_dev(dev, n, offs[i])
            gd.append(g.view(torch.bfloat16) if bf16 else g)
        st.step(t, gd, 3e-4, 0.5)
        for (lo, ln), orc in zip(windows, oracles):
            orc.step(t, [si.tiled(pools[i], ln, lo + offs[i]) for i in range(R)], 3e-4, 0.5)
        torch.cuda.synchronize()
        del gd
    assert st.read_flags() == 0
    if sweep:
        any_d = False
        for k, (lo, ln) in enumerate(windows):
            if k % 8 == 0:
                print(f"  oracle window {k + 1} of {len(windows)}", flush=True)
            orc = make_oracle(lo, ln)
            for t in range(1, steps + 1):
                pools, offs = inputs[t]
                orc.step(t, [si.tiled(pools[i], ln, lo + offs[i]) for i in range(R)], 3e-4, 0.5)
            check_window(lo, ln, orc)
            any_d = any_d or any(np.any(orc.d(i)) for i in range(R))
            orc.close()
        assert any_d
    else:
        for (lo, ln), orc in zip(windows, oracles):
            check_window(lo, ln, orc)
            assert any(np.any(orc.d(i)) for i in range(R))
    # the subset of one step: against the oracle's enumeration, whole or on the windows, and against Binomial(n, p)
    idx, k = st.subset_indices(3, capacity=int(n * p * 1.05) + 1000)
    got = idx.cpu().numpy().astype(np.uint64)
    assert abs(k - n * p) < 6 * (n * p * (1 - p)) ** 0.5
    if whole_subset:
        assert np.array_equal(got, O.subset(seed, 3, n, p))
    else:
        for lo, ln in windows[:: max(1, len(windows) // 4)]:
            assert np.array_equal(got[(got >= lo) & (got < lo + ln)], O.subset(seed, 3, ln, p, mu0=lo))


def test_full_size_stage_every_coordinate(amlib):
    """125,829,120 fp32 params, R=8, staleness 4, 5 %: the benchmark's workload and layout, every
    element of w, m, v, d, fwd of every replica against the oracle, and the whole index list of one subset."""
    _full_size_case(amlib, 125_829_120, 8, 4, 0.05, 7, "all", whole_subset=True)


def test_full_size_stage_on_sampled_windows_with_per_replica_d(amlib):
    """The same workload with one EMA array per replica, on windows."""
    n = 125_829_120
    _full_size_case(amlib, n, 8, 4, 0.05, 7,
                    [(0, 70_000), (131_072 * 211 - 3_000, 70_000), (62_914_560 - 5, 40_000), (n - 70_001, 70_001)],
                    d_layout=PER_REPLICA)


def test_full_size_bf16_stage_every_coordinate(amlib):
    """Same stage with bf16 gradients / forward weights over fp32 masters, R=16, staleness 8, 1 %:
    every element against the oracle."""
    _full_size_case(amlib, 125_829_120, 16, 8, 0.01, 11, "all", bf16=True, lookahead=False)


def test_full_size_1b_stage_on_sampled_windows(amlib):
    """10^9 fp32 params on one stage, R=8, staleness 4, 10 %, look-ahead + EMA (needs ~215 GB of HBM)."""
    n = 1_000_000_000
    if _free_hbm() < 230e9:
        pytest.skip("not enough free HBM for the 1B-parameter stage")
    _full_size_case(amlib, n, 8, 4, 0.10, 6, [(0, 40_000), (2 ** 29 - 20_000, 40_000), (n - 40_003, 40_003)])


def test_largest_stage_the_library_accepts(amlib):
    """n just under 2^32 - 2^20 (the documented limit): 64-bit addressing, 16.7 M tiles, windows at the
    start, across 2^31 and at the very end (ragged tail).  Plain SGD, two replicas (about 120 GB)."""
    n = (1 << 32) - (1 << 20) - 5
    if _free_hbm() < 140e9:
        pytest.skip("not enough free HBM for the largest stage")
    _full_size_case(amlib, n, 2, 1, 0.002, 3, [(0, 30_000), ((1 << 31) - 15_000, 30_000), (n - 30_001, 30_001)],
                    lookahead=False, optimizer=O.OPT_SGD, beta1=0.0)
    with pytest.raises(amlib.AsyncMeshError):
        amlib.workspace_bytes(amlib.make_config(n + 5, 2))


# --------------------------------------------------------------------------------------------
# stand-alone entry points
# --------------------------------------------------------------------------------------------
def run_average(am, n, R, steps, seed=17, lam=0.5, **kw):
    """am_sparse_average on weights the caller steps itself (here: a seeded perturbation between the
    calls), every element of w and d against the oracle after every call."""
    print(f"case sparse_average n={n} R={R} steps={steps} {kw}", flush=True)
    w0 = np.stack([si.stage_weights(n, 100 + i) for i in range(R)])
    st, orc = make_pair(am, n, R, w0=w0, seed=seed, optimizer=O.OPT_SGD, beta1=0.0, **kw)
    for t in range(1, steps + 1):
        bump = si.replica_grads(n, R, t, seed)
        for i in range(R):
            orc.w(i)[:] += bump[i]
            st.w[i] += torch.from_numpy(bump[i]).cuda()
        st.sparse_average(t, lam)
        orc.sparse_average(t, lam)
        for i in range(R):
            assert rel_err(st.w[i].cpu().numpy(), orc.w(i)) < TOL_F32, (t, i)
            if st.d is not None:
                assert rel_err(st.d[i].cpu().numpy(), orc.d(i)) < TOL_F32, (t, i)
    assert st.read_flags() == 0
    return st, orc


@pytest.mark.parametrize("n,R,tau,K,p,corr", [
    (1, 1, 0, 1, 1.0, O.CORR_EMA), (257, 2, 1, 1, 0.5, O.CORR_EMA), (10_007, 3, 0, 1, 0.2, O.CORR_EMA),
    (10_007, 4, 2, 1, 0.05, O.CORR_EMA), (10_007, 5, 1, 2, 0.3, O.CORR_NONE), (131_072 + 9, 8, 3, 1, 0.05, O.CORR_EMA),
    (50_000, 16, 1, 1, 1.0, O.CORR_EMA), (50_000, 32, 2, 1, 0.01, O.CORR_EMA), (50_000, 7, 1, 1, EMPTY_P, O.CORR_EMA),
    (1, 1, 1, 1, 1.0, O.CORR_EMA), (1003, 1, 2, 1, 0.3, O.CORR_EMA), (1003, 8, 2, 1, 0.3, O.CORR_EMA),
    (40_001, 12, 1, 3, 0.3, O.CORR_EMA), (40_001, 20, 3, 1, 0.1, O.CORR_NONE), (40_001, 9, 0, 2, 0.1, O.CORR_EMA),
    (20_001, 32, 0, 1, 0.2, O.CORR_EMA), (20_001, 16, 0, 1, 1.0, O.CORR_NONE), (20_003, 6, 0, 1, 0.05, O.CORR_EMA),
])
@both_layouts
def test_sparse_average_alone(amlib, n, R, tau, K, p, corr, d_layout):
    """The caller runs its own optimizer.  With tau > 0 this is the kernel that keeps a block's replicas
    side by side in registers; with tau = 0 the fused kernel without its optimizer pass."""
    run_average(amlib, n, R, 3 * (tau + 1) * K + 2, delay=tau, avg_interval=K, fraction=p, correction=corr, d_layout=d_layout)


@pytest.mark.parametrize("msg", [O.MSG_BF16, O.MSG_E4M3])
@both_layouts
def test_sparse_average_quantised_exchange(amlib, msg, d_layout):
    """The mean takes the rounded messages, a replica's own staleness term its exact value."""
    run_average(amlib, 30_011, 5, 8, delay=2, fraction=0.2, msg_dtype=msg, d_layout=d_layout)
    run_average(amlib, 30_011, 11, 5, delay=1, fraction=0.2, msg_dtype=msg, d_layout=d_layout)
    run_average(amlib, 30_011, 11, 4, delay=0, fraction=0.2, msg_dtype=msg, d_layout=d_layout)


@both_layouts
def test_sparse_average_eager_correction(amlib, d_layout):
    run_average(amlib, 25_013, 4, 9, delay=2, fraction=1.0, correction=O.CORR_EAGER, d_layout=d_layout)
    run_average(amlib, 25_013, 3, 9, delay=1, avg_interval=2, fraction=0.3, correction=O.CORR_EAGER, d_layout=d_layout)


def test_sparse_average_delay_changed_at_run_time(amlib):
    am = amlib
    n, R = 60_003, 6
    w0 = np.stack([si.stage_weights(n, 100 + i) for i in range(R)])
    st, orc = make_pair(am, n, R, w0=w0, delay=3, fraction=0.1, seed=29, optimizer=O.OPT_SGD, beta1=0.0)
    for t in range(1, 16):
        if t == 6:
            st.set_delay(1); orc.set_delay(1)
        if t == 11:
            st.set_delay(3); orc.set_delay(3)
        bump = si.replica_grads(n, R, t, 29)
        for i in range(R):
            orc.w(i)[:] += bump[i]
            st.w[i] += torch.from_numpy(bump[i]).cuda()
        st.sparse_average(t, 0.5); orc.sparse_average(t, 0.5)
        for i in range(R):
            assert rel_err(st.w[i].cpu().numpy(), orc.w(i)) < TOL_F32, (t, i)
            assert rel_err(st.d[i].cpu().numpy(), orc.d(i)) < TOL_F32, (t, i)


@both_layouts
def test_sparse_average_ring_slot_overflow(amlib, d_layout):
    """The averaging-only kernel leaves the tiles past a too small slot out at send and receive alike,
    as the fused one does: the tiles before the first dropped one follow the method, those after
    the last are never averaged, the flag is raised."""
    am = amlib
    n, R, tau, p, seed, steps, cap, rb = 100_003, 4, 1, 0.2, 19, 6, 700, 4
    w0 = np.stack([si.stage_weights(n, 100 + i) for i in range(R)])
    cfg = am.make_config(n, R, delay=tau, fraction=p, seed=seed, optimizer=am.OPT_SGD, beta1=0.0, d_layout=d_layout, ring_cap_lines=cap)
    st = am.init_state(cfg, torch.from_numpy(w0).cuda())
    full = O.Oracle(n, R, delay=tau, fraction=p, seed=seed, optimizer=O.OPT_SGD, beta1=0.0); full.set_w(w0)
    never = O.Oracle(n, R, delay=tau, fraction=EMPTY_P, seed=seed, optimizer=O.OPT_SGD, beta1=0.0); never.set_w(w0)
    first_dropped = []
    for t in range(1, steps + 1):
        bump = si.replica_grads(n, R, t, seed)
        for i in range(R):
            full.w(i)[:] += bump[i]; never.w(i)[:] += bump[i]
            st.w[i] += torch.from_numpy(bump[i]).cuda()
        st.sparse_average(t, 0.5); full.sparse_average(t, 0.5); never.sparse_average(t, 0.5)
        counts = np.bincount((O.subset(seed, t, n, p) // 256).astype(np.int64), minlength=-(-n // 256))
        lines = -(-counts * rb // 32)
        start = np.cumsum(lines) - lines
        assert (start + lines > cap).any()
        first_dropped.append(int(np.argmax(start + lines > cap)))
    lo, hi = min(first_dropped) * 256, (max(first_dropped) + 1) * 256
    assert 0 < lo <= hi < n - 10_000
    for i in range(R):
        for name in ("w", "d"):
            got = getattr(st, name)[i].cpu().numpy()
            assert rel_err(got[:lo], getattr(full, name)(i)[:lo]) < TOL_F32, (name, i, "kept tiles")
            assert rel_err(got[hi:], getattr(never, name)(i)[hi:]) < TOL_F32, (name, i, "dropped tiles")
    assert st.read_flags() & 1
    with pytest.raises(am.AsyncMeshError) as e:
        st.sparse_average(steps + 1, 0.5)
    assert e.value.status == -6


def test_fused_steps_and_stand_alone_averaging_interleaved(amlib):
    """am_step and am_sparse_average share the ring, the step counter and the subset offsets."""
    n, R, tau = 70_003, 4, 1
    st, orc = make_pair(amlib, n, R, delay=tau, fraction=0.1, seed=23)
    for t in range(1, 10):
        if t % 3 == 0:
            st.sparse_average(t, 0.5); orc.sparse_average(t, 0.5)
        else:
            g, gd = grads_for(n, R, t, 23, False)
            st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
        for i in range(R):
            assert rel_err(st.w[i].cpu().numpy(), orc.w(i)) < TOL_F32, (t, i)
            assert rel_err(st.d[i].cpu().numpy(), orc.d(i)) < TOL_F32, (t, i)
    assert st.read_flags() == 0


@pytest.mark.parametrize("n", [1, 5, 1000, 1_000_003])
@pytest.mark.parametrize("bf16", [False, True])
def test_lookahead_alone(amlib, n, bf16):
    """The stateless look-ahead has no approximate step: its output is the oracle's bit for bit, in
    fp32 and in bf16 (ONE rounding of the fp64 value)."""
    am = amlib
    w = si.stage_weights(n, 1); wp = si.stage_weights(n, 2)
    out = am.lookahead(torch.from_numpy(w).cuda(), torch.from_numpy(wp).cuda(), 0.9, am.BF16 if bf16 else am.F32)
    if bf16:
        got = out.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got, O.lookahead(w, wp, O.f32(0.9), bf16=True))
    else:
        assert np.array_equal(out.cpu().numpy(), O.lookahead(w, wp, O.f32(0.9)))


def test_lookahead_alone_rounds_to_bf16_once(amlib):
    """Values a hair above or below a bf16 tie, where rounding to fp32 first lands ON the tie and a
    second rounding then goes the wrong way: w = a bf16 tie (9 significant bits), w_prev one fp32 step
    away, gamma = 2^-10, so that w + gamma (w - w_prev) = tie +- 2^-10 fp32 steps."""
    am = amlib
    rng = np.random.default_rng(3)
    k = rng.integers(128, 256, 20_000) * 2 + 1                       # odd 9-bit integers: halfway between two bf16 values
    e = rng.integers(-20, 10, 20_000)
    w = (k * 2.0 ** (e - 8.0)).astype(np.float32) * rng.choice([-1.0, 1.0], 20_000).astype(np.float32)
    away = rng.choice([np.float32(np.inf), np.float32(-np.inf)], 20_000)
    wp = np.nextafter(w, away).astype(np.float32)
    g = 2.0 ** -10
    out = am.lookahead(torch.from_numpy(w).cuda(), torch.from_numpy(wp).cuda(), g, am.BF16)
    got = out.view(torch.int16).cpu().numpy().view(np.uint16)
    want = O.lookahead(w, wp, g, bf16=True)
    assert np.array_equal(got, want)
    twice = si.to_bf16_bits((w.astype(np.float64) + g * (w.astype(np.float64) - wp.astype(np.float64))).astype(np.float32))
    assert (twice != want).mean() > 0.2                                # rounding twice would have been caught


# --------------------------------------------------------------------------------------------
# API behaviour on the device
# --------------------------------------------------------------------------------------------
def test_step_order_and_argument_errors(amlib):
    am = amlib
    n, R = 1000, 2
    st = am.init_state(am.make_config(n, R, delay=1, fraction=0.1), torch.zeros(n))
    g = [torch.zeros(n, device="cuda") for _ in range(R)]
    with pytest.raises(am.AsyncMeshError) as e:
        st.step(2, g, 1e-3)
    assert e.value.status == -4
    st.step(1, g, 1e-3)
    with pytest.raises(am.AsyncMeshError) as e:
        st.step(1, g, 1e-3)
    assert e.value.status == -4
    with pytest.raises(am.AsyncMeshError) as e:
        st.step(2, [g[0], torch.zeros(n + 1, device="cuda")[1:]], 1e-3)       # misaligned gradient pointer
    assert e.value.status == -2
    with pytest.raises(ValueError):
        st.step(2, [g[0], g[1][1:]], 1e-3)                      # too short: refused by the binding, before any launch
    with pytest.raises(am.AsyncMeshError) as e:
        st.step(2, g, 1e-3, lambda_t=1.5)
    assert e.value.status == -1
    st.step(2, g, 1e-3)                                         # failed calls left the state untouched
    cap, slots = st.ring_info()
    assert slots == 2 and 4 * 32 <= cap <= 4 * 256 * 2       # 4 tiles of two interleaved replicas, between 1 and 16 lines each


def test_runs_on_the_stream_given_at_init(amlib):
    """All work goes to the stream that was current at init_state (here a side stream)."""
    n, R = 50_021, 4
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        st, orc = make_pair(amlib, n, R, delay=1, fraction=0.1, seed=9, lookahead=True, gamma=0.9)
        for t in range(1, 6):
            g, gd = grads_for(n, R, t, 9, False)
            st.step(t, gd, 1e-3, 0.5); orc.step(t, g, 1e-3, 0.5)
        side.synchronize()
        compare(st, orc, "side stream")


def test_two_states_do_not_interfere(amlib):
    n, R = 30_011, 3
    a, oa = make_pair(amlib, n, R, delay=1, fraction=0.2, seed=1)
    b, ob = make_pair(amlib, n + 77, R + 1, delay=2, fraction=0.05, seed=2, lookahead=True, gamma=0.5)
    for t in range(1, 7):
        ga, gda = grads_for(n, R, t, 1, False)
        gb, gdb = grads_for(n + 77, R + 1, t, 2, False)
        a.step(t, gda, 1e-3, 0.5); b.step(t, gdb, 2e-3, 0.25)
        oa.step(t, ga, 1e-3, 0.5); ob.step(t, gb, 2e-3, 0.25)
    compare(a, oa, "state a"); compare(b, ob, "state b")


@pytest.mark.parametrize("speeds,opt,bf16", [
    ([2, 1, 2, 3], O.OPT_ADAMW, False), ([5, 3, 1, 11], O.OPT_NADAMW, False), ([1, 2, 1, 2, 1, 2, 1, 2, 2, 1], O.OPT_ADAMW, True),
    ([3, 1], O.OPT_SGD, False),
])
def test_replicas_of_unequal_speed(amlib, speeds, opt, bf16):
    """Heterogeneous set-up: ticks in which only some replicas make a local step, the averaging
    interval equal to the round length."""
    am = amlib
    n, R, K, seed = 40_009, len(speeds), max(speeds), 41
    kw = dict(delay=1, avg_interval=K, fraction=0.2, seed=seed, optimizer=opt, lookahead=(opt == O.OPT_ADAMW), gamma=0.9)
    st, orc = make_pair(am, n, R, grad_bf16=bf16, fwd_bf16=bf16, **kw)
    for t in range(1, 3 * K + 2):
        mask = am.active_mask(t, speeds)
        g, gd = grads_for(n, R, t, seed, bf16)
        g = [x if (mask >> i) & 1 else None for i, x in enumerate(g)]
        gd = [x if (mask >> i) & 1 else None for i, x in enumerate(gd)]
        st.step_masked(t, gd, 1e-3, 0.5, mask)
        orc.step_masked(t, g, 1e-3, 0.5, mask)
        if t % K <= 1:
            compare(st, orc, f"speeds={speeds} t={t}")
    assert any(np.any(orc.d(i)) for i in range(R))
    with pytest.raises(am.AsyncMeshError):
        st.step_masked(3 * K + 2, gd, 1e-3, 0.5, 1 << R)               # names a replica that does not exist


def test_idle_replica_ignores_its_gradient_pointer_and_scale(amlib):
    am = amlib
    n, R, seed = 20_011, 3, 47
    st, orc = make_pair(am, n, R, delay=1, fraction=0.3, seed=seed, lookahead=True, gamma=0.9)
    scale = np.array([0.5, np.nan, 2.0], dtype=np.float32)
    scale_dev = torch.from_numpy(scale).cuda()
    for t in range(1, 5):
        g, gd = grads_for(n, R, t, seed, False)
        mask = 0b101 if t != 3 else 0b111
        sc = scale if t != 3 else np.array([0.5, 1.5, 2.0], dtype=np.float32)
        scale_dev.copy_(torch.from_numpy(sc))
        if t != 3:
            g[1], gd[1] = None, None
        st.step_masked(t, gd, 1e-3, 0.5, mask, grad_scale=0.75, replica_scale=scale_dev)
        orc.step_masked(t, g, 1e-3, 0.5, mask, grad_scale=0.75, replica_scale=sc)
        compare(st, orc, f"t={t}")


def test_all_active_ticks_are_ordinary_steps(amlib):
    am = amlib
    n, R, seed = 30_011, 3, 43
    kw = dict(delay=1, fraction=0.2, seed=seed, optimizer=O.OPT_NADAMW)
    a, _ = make_pair(am, n, R, **kw)
    b, _ = make_pair(am, n, R, **kw)
    for t in range(1, 6):
        _, gd = grads_for(n, R, t, seed, False)
        a.step(t, gd, 1e-3, 0.5)
        b.step_masked(t, gd, 1e-3, 0.5, 0b111)
    torch.cuda.synchronize()
    for name in ("w", "m", "v", "d"):
        for i in range(R):
            assert torch.equal(getattr(a, name)[i], getattr(b, name)[i]), (name, i)


def test_a_thousand_steps_stay_within_the_bar(amlib):
    """Rounding must not random-walk: the tiny configuration (1,048,576 x 4, delay 1, 5 %) with
    look-ahead for 1000 steps, eight gradient sets cycled, schedules of the paper's set-up."""
    am = amlib
    n, R, seed, steps = 1_048_576, 4, 0, 1000
    st, orc = make_pair(am, n, R, delay=1, fraction=0.05, seed=seed, lookahead=True, gamma=0.9)
    pool = [grads_for(n, R, 100 + k, seed, False) for k in range(8)]
    worst = {}
    for t in range(1, steps + 1):
        g, gd = pool[t % 8]
        lr = am.learning_rate(t, steps, warmup=100)
        lam = am.ema_lambda(t, steps, hold=300)
        st.step(t, gd, lr, lam); orc.step(t, g, lr, lam)
        if t % 250 == 0:
            worst = compare(st, orc, f"t={t}")
            print(f"  t={t}", {k: f"{v:.1e}" for k, v in worst.items()}, flush=True)
    assert max(worst.values()) < TOL_F32


@pytest.mark.parametrize("case", range(128))
def test_random_configurations(amlib, case):
    """Seeded random draws over the whole configuration space (sizes, replicas, delay, interval,
    fraction, optimizer, correction, message precision, sampling rule, dtypes, idle replicas)."""
    am = amlib
    rng = np.random.default_rng(1000 + case)
    n = int(rng.choice([1, 7, 255, 256, 257, 1023, int(rng.integers(1, 200_000)), int(rng.integers(1, 200_000))]))
    R = int(rng.integers(1, 13)) if rng.integers(0, 4) else int(rng.integers(13, 33))
    tau, K = int(rng.integers(0, 4)), int(rng.integers(1, 4))
    p = float(rng.choice([0.003, 0.05, 0.3, 0.9, 1.0]))
    opt = int(rng.choice([O.OPT_SGD, O.OPT_ADAMW, O.OPT_NADAMW]))
    rule = int(rng.integers(0, 3))                       # 0 independent, 1 whole lines, 2 stratified
    bf16 = bool(rng.integers(0, 2))
    kw = dict(delay=tau, avg_interval=K, fraction=p, seed=int(rng.integers(0, 2 ** 62)), optimizer=opt,
              beta1=float(rng.choice([0.0, 0.9])) if opt == O.OPT_SGD else 0.9,
              lookahead=bool(rng.integers(0, 2)) and opt != O.OPT_NADAMW, gamma=0.9,
              correction=int(rng.choice([O.CORR_NONE, O.CORR_EMA, O.CORR_EAGER])),
              msg_dtype=int(rng.choice([O.MSG_F32, O.MSG_BF16, O.MSG_E4M3])),
              subset_granule=32 if rule == 1 else 1,
              subset_kind=am.SUBSET_STRATIFIED if rule == 2 else am.SUBSET_BERNOULLI,
              d_layout=int(rng.integers(0, 2)))
    print(f"case {case}: n={n} R={R} bf16={bf16} {kw}", flush=True)
    st, orc = make_pair(am, n, R, grad_bf16=bf16, fwd_bf16=bf16, **kw)
    if st.fwd is not None:                       # am_sparse_average leaves fwd alone; the oracle's starts at zero
        for f in st.fwd:
            f.zero_()
    masked = bool(rng.integers(0, 2))
    for t in range(1, (tau + 2) * K + 3):
        g, gd = grads_for(n, R, t, case, bf16)
        lam, lr = float(rng.choice([0.0, 0.01, 0.5, 1.0])), float(rng.choice([1e-4, 3e-3]))
        if masked:
            mask = int(rng.integers(0, 1 << R))
            st.step_masked(t, gd, lr, lam, mask, grad_scale=0.5)
            orc.step_masked(t, g, lr, lam, mask, grad_scale=0.5)
        elif rng.integers(0, 4) == 0:
            st.sparse_average(t, lam); orc.sparse_average(t, lam)
            st.fwd_is_stale = True                  # am_sparse_average leaves fwd alone
        else:
            st.step(t, gd, lr, lam); orc.step(t, g, lr, lam)
            st.fwd_is_stale = False
        compare(st, orc, f"case {case} t={t}")


@both_layouts
@pytest.mark.parametrize("opt,K", [(O.OPT_NADAMW, 1), (O.OPT_ADAMW, 2)])
def test_checkpoint_and_resume(amlib, opt, K, d_layout):
    """A run that is checkpointed after step 5 and resumed on other memory continues bit for bit as
    the uninterrupted run does (and both agree with the oracle)."""
    am = amlib
    n, R, tau, seed, total = 60_017, 4, 2, 31, 13
    kw = dict(delay=tau, avg_interval=K, fraction=0.1, seed=seed, optimizer=opt, lookahead=(opt != O.OPT_NADAMW), gamma=0.9,
              d_layout=d_layout)
    a, orc = make_pair(am, n, R, **kw)
    saved = None
    mask_at = lambda t: 0b1111 if (t % 2 or opt != O.OPT_NADAMW) else 0b1011    # NADAMW case: replica 2 idles in even ticks
    for t in range(1, total + 1):
        g, gd = grads_for(n, R, t, seed, False)
        a.step_masked(t, gd, 1e-3, 0.5, mask_at(t)); orc.step_masked(t, g, 1e-3, 0.5, mask_at(t))
        if t == 3:
            a.set_delay(1); orc.set_delay(1)
        if t == 5:
            torch.cuda.synchronize()
            clone = lambda ts: None if ts is None else [x.clone() for x in ts]
            saved = (a.export_state(), clone(a.w), clone(a.m), clone(a.v), clone(a.d_storage), clone(a.fwd), a.workspace.clone())
    compare(a, orc, "uninterrupted")
    snap, w, m, v, d, fwd, ws = saved
    assert snap.last_t == 5 and snap.delay_now == 1
    b = am.Stage.resume(a.cfg, snap, w, m, v, d, fwd, ws)
    with pytest.raises(am.AsyncMeshError):
        b.step(5, grads_for(n, R, 5, seed, False)[1], 1e-3, 0.5)           # the step counter came back too
    assert list(snap.opt_steps[:R]) == ([5, 5, 3, 5] if opt == O.OPT_NADAMW else [5] * R)
    for t in range(6, total + 1):
        b.step_masked(t, grads_for(n, R, t, seed, False)[1], 1e-3, 0.5, mask_at(t))
    torch.cuda.synchronize()
    for name in ("w", "m", "v", "d", "fwd"):
        if getattr(a, name) is not None:
            for i in range(R):
                assert torch.equal(getattr(a, name)[i], getattr(b, name)[i]), (name, i)
    other = am.make_config(n, R, **dict(kw, seed=seed + 1))
    with pytest.raises(am.AsyncMeshError):
        am.Stage.resume(other, snap, w, m, v, d, fwd, ws)


def test_kernel_profiling_hooks(amlib):
    am = amlib
    n, R = 200_000, 2
    st = am.init_state(am.make_config(n, R, delay=1, fraction=0.1), torch.zeros(n))
    g = [torch.zeros(n, device="cuda") for _ in range(R)]
    st.set_profiling(True)
    for t in range(1, 6):
        st.step(t, g, 1e-3)
    ms, k = st.get_profile()
    assert k == 5 and 0.0 < ms < 1000.0
    st.set_profiling(False)
    st.step(6, g, 1e-3)
    assert st.get_profile()[1] == 0


def test_ring_slot_overflow_drops_whole_tiles_and_is_loud(amlib):
    """A caller-named slot size (ring_cap_lines) that is too small: the tiles past the capacity are
    left out of the round at send and at receive alike (they evolve as if never averaged), the
    tiles before it follow the method exactly, the sticky flag is raised, and once it has been
    read as set the next step is refused."""
    am = amlib
    n, R, tau, p, seed, steps, cap = 100_003, 4, 1, 0.2, 19, 6, 700
    rb = 4
    w0 = si.stage_weights(n, seed)
    cfg = am.make_config(n, R, delay=tau, fraction=p, seed=seed, lookahead=True, gamma=0.9, d_layout=INTERLEAVED,
                         ring_cap_lines=cap)
    st = am.init_state(cfg, torch.from_numpy(w0).cuda())
    assert st.ring_info()[0] == cap * 32
    full = O.Oracle(n, R, delay=tau, fraction=p, seed=seed, lookahead=True, gamma=0.9); full.set_w(w0)
    never = O.Oracle(n, R, delay=tau, fraction=EMPTY_P, seed=seed, lookahead=True, gamma=0.9); never.set_w(w0)
    first_dropped = []
    for t in range(1, steps + 1):
        g, gd = grads_for(n, R, t, seed, False)
        st.step(t, gd, 1e-3, 0.5); full.step(t, g, 1e-3, 0.5); never.step(t, g, 1e-3, 0.5)
        counts = np.bincount((O.subset(seed, t, n, p) // 256).astype(np.int64), minlength=-(-n // 256))
        lines = -(-counts * rb // 32)
        start = np.cumsum(lines) - lines
        first_dropped.append(int(np.argmax(start + lines > cap)))
        assert (start + lines > cap).any()
    lo, hi = min(first_dropped) * 256, (max(first_dropped) + 1) * 256
    assert 0 < lo <= hi < n - 10_000
    for i in range(R):
        for name in ("w", "m", "v", "d", "fwd"):
            got = getattr(st, name)[i].cpu().numpy()
            assert rel_err(got[:lo], getattr(full, name)(i)[:lo]) < TOL_F32, (name, i, "kept tiles")
            assert rel_err(got[hi:], getattr(never, name)(i)[hi:]) < TOL_F32, (name, i, "dropped tiles")
    assert not np.any(st.d[0].cpu().numpy()[hi:]) and np.any(st.d[0].cpu().numpy()[:lo])
    assert st.read_flags() & 1
    with pytest.raises(am.AsyncMeshError) as e:
        st.step(steps + 1, grads_for(n, R, steps + 1, seed, False)[1], 1e-3, 0.5)
    assert e.value.status == -6
    with pytest.raises(am.AsyncMeshError) as e:
        st.sparse_average(steps + 1, 0.5)
    assert e.value.status == -6


def test_profiling_pool_is_bounded(amlib):
    """More launches than the event pool holds: the later ones run untimed, nothing grows."""
    am = amlib
    n, R = 4096, 1
    st = am.init_state(am.make_config(n, R, fraction=0.1, optimizer=am.OPT_SGD, beta1=0.0, correction=am.CORR_NONE), torch.zeros(n))
    g = [torch.zeros(n, device="cuda")]
    st.set_profiling(True)
    for t in range(1, 4200):
        st.step(t, g, 1e-3)
    times = st.get_profile_times()
    assert len(times) == 4096 and all(x > 0 for x in times)
    st.step(4200, g, 1e-3)
    assert len(st.get_profile_times()) == 1
