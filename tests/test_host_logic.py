"""The library's host-side arithmetic (ring slot capacity, workspace layout, which slot a step writes
and reads, replica blocks) driven directly on the CPU: csrc/am_host_logic.h holds no HIP, so a plain
g++ build of a small driver exposes it to ctypes."""
import ctypes as C
import math
import random
import subprocess
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


@pytest.fixture(scope="module")
def hl(tmp_path_factory):
    so = tmp_path_factory.mktemp("hostlogic") / "libhostlogic.so"
    subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Wextra", "-Werror", "-fPIC", "-shared", "-o", str(so),
                    str(ROOT / "tests" / "host_logic_driver.cpp")], check=True)
    L = C.CDLL(str(so))
    L.hl_threshold.argtypes = [C.c_double]; L.hl_threshold.restype = C.c_uint64
    L.hl_stratified_block.argtypes = [C.c_double]; L.hl_stratified_block.restype = C.c_uint64
    L.hl_blocks.argtypes = [C.c_uint32] + [C.POINTER(C.c_uint32)] * 3
    L.hl_capacity.argtypes = [C.c_uint64, C.c_double, C.c_uint32, C.c_int, C.c_uint64]; L.hl_capacity.restype = C.c_uint64
    L.hl_layout.argtypes = [C.c_void_p, C.POINTER(C.c_uint64)]
    L.hl_plan_round.argtypes = [C.c_uint64] * 4 + [C.POINTER(C.c_uint64)]
    return L


def _config(**kw):
    """am_config as the binding lays it out (the ABI test checks that layout against the C compiler's)."""
    from paper_2601_22442_amd.binding import Config
    base = dict(n=1000, replicas=2, delay=0, avg_interval=1, optimizer=1, fraction=0.05, seed=0, beta1=0.9, beta2=0.999,
                eps=1e-8, weight_decay=0.01, gamma=0.0, lookahead=0, correction=1, fwd_dtype=0, grad_dtype=0,
                momentum_decay=0.004, subset_granule=1, msg_dtype=0, subset_kind=0, d_layout=0, ring_cap_lines=0)
    base.update(kw)
    return Config(**base)


def test_threshold_and_blocks(hl, amlib):
    assert hl.hl_threshold(0.0) == 0 and hl.hl_threshold(1.0) == 1 << 32 and hl.hl_threshold(0.5) == 1 << 31
    assert hl.hl_threshold(0.05) == math.floor(0.05 * 2 ** 32)
    assert hl.hl_stratified_block(0.05) == 20 and hl.hl_stratified_block(1.0) == 1 and hl.hl_stratified_block(0.3) == 3
    for R in range(1, 33):
        rb, sh, nb = C.c_uint32(), C.c_uint32(), C.c_uint32()
        hl.hl_blocks(R, C.byref(rb), C.byref(sh), C.byref(nb))
        want_rb = min(8, 1 << (R - 1).bit_length())
        assert (rb.value, 1 << sh.value, nb.value) == (want_rb, want_rb, -(-R // want_rb)), R
        assert nb.value * rb.value >= R > (nb.value - 1) * rb.value


@pytest.mark.parametrize("p,rb", [(0.05, 8), (0.05, 1), (0.01, 8), (0.10, 8), (0.3, 4), (0.001, 2), (0.9, 8)])
def test_slot_capacity_is_mean_plus_twelve_sigma_of_the_exact_line_count(hl, p, rb):
    """A tile of 256 coordinates owns ceil(X rb / 32) lines, X ~ Binomial(256, p): exact moments by summation."""
    ntiles = 491_520
    pmf = [math.comb(256, k) * p ** k * (1 - p) ** (256 - k) for k in range(257)]
    lines = [-(-k * rb // 32) for k in range(257)]
    mean = sum(a * b for a, b in zip(pmf, lines))
    var = sum(a * b * b for a, b in zip(pmf, lines)) - mean ** 2
    want = math.ceil(ntiles * mean + 12 * math.sqrt(ntiles * var)) + 64
    got = hl.hl_capacity(ntiles, p, rb, 0, 0)
    assert abs(got - min(want, ntiles * 8 * rb)) <= 1
    # the margin is real: at least ten standard deviations above the mean, never more than every line
    assert got <= ntiles * 8 * rb
    if got < ntiles * 8 * rb:
        assert got >= ntiles * mean + 10 * math.sqrt(ntiles * var)


def test_slot_capacity_special_cases(hl):
    assert hl.hl_capacity(100, 1.0, 8, 0, 0) == 100 * 64                # everything selected: 256 * 8 / 32 lines a tile
    assert hl.hl_capacity(100, 1.0, 1, 0, 0) == 100 * 8
    assert hl.hl_capacity(1000, 0.05, 8, 0, 20) == 1000 * 4              # stratified, B = 20: at most 14 members -> 4 lines
    assert hl.hl_capacity(1000, 1 / 256, 8, 0, 256) == 1000              # B = 256: at most 2 members -> one line
    assert hl.hl_capacity(1000, 1.0, 4, 0, 1) == 1000 * 32               # B = 1: every coordinate
    # whole lines of 32 coordinates drawn: Binomial(8, p) x rb lines a tile
    ntiles, p, rb = 100_000, 0.07, 8
    want = math.ceil(ntiles * 8 * p * rb + 12 * math.sqrt(ntiles * 8 * p * (1 - p)) * rb) + 64
    assert abs(hl.hl_capacity(ntiles, p, rb, 1, 0) - want) <= 1
    assert hl.hl_capacity(1, 0.5, 8, 0, 0) == 64                         # tiny stage: the margin saturates at every line


def test_workspace_regions_do_not_overlap_and_match_the_library(hl, amlib):
    am = amlib
    rng = random.Random(5)
    for _ in range(60):
        n = rng.choice([1, 255, 256, 257, 131_072, 131_073, rng.randrange(1, 50_000_000)])
        R = rng.randrange(1, 33)
        cfg = _config(n=n, replicas=R, delay=rng.randrange(0, 9), fraction=rng.choice([1e-6, 0.01, 0.05, 0.5, 1.0]),
                      subset_kind=rng.randrange(0, 2), ring_cap_lines=rng.choice([0, 0, 17, 10 ** 12]))
        out = (C.c_uint64 * 13)()
        hl.hl_layout(C.byref(cfg), out)
        ntiles, nsb, slots, cap, off_flags, off_reduce, off_next, off_meta, meta_stride, off_ring, ring_stride, total, sb_off = out
        assert ntiles == -(-n // 256) and nsb == -(-ntiles // 512) and slots == cfg.delay + 1
        rb = min(8, 1 << (R - 1).bit_length()); nblocks = -(-R // rb)
        if cfg.ring_cap_lines:
            assert cap == min(cfg.ring_cap_lines, ntiles * 8 * rb)
        regions = [(off_flags, 256), (off_reduce, 32 * 1024 * 8), (off_next, ntiles * 4)]
        for s in range(slots + 1):
            base = off_meta + s * meta_stride
            regions += [(base, ntiles * 4), (base + sb_off, (nsb + 1) * 4)]
        for s in range(slots):
            regions.append((off_ring + s * ring_stride, cap * 128 * nblocks))
        regions.sort()
        for (a, la), (b, _) in zip(regions, regions[1:]):
            assert a + la <= b, (a, la, b)
        assert regions[-1][0] + regions[-1][1] <= total
        assert all(a % 256 == 0 for a, _ in regions)
        assert am.workspace_bytes(cfg) == total                           # the library uses this very arithmetic


def test_ring_slots_hold_what_a_step_expects_under_any_delay_sequence(hl):
    """Model: a slot holds the round that last wrote it.  Whatever the interval, the ring depth and
    the delays in force from step to step (am_set_delay), a receive must find, in the slot it reads,
    exactly the round sent tau rounds earlier, and nothing is received before anything was sent."""
    rng = random.Random(11)
    for _ in range(200):
        K, delay = rng.randrange(1, 6), rng.randrange(0, 7)
        depth = delay + 1
        held = {}
        out = (C.c_uint64 * 6)()
        for t in range(1, 12 * K * depth + 3):
            tau = rng.randrange(0, depth)
            hl.hl_plan_round(K, depth, tau, t, out)
            send, recv, same, slot_s, slot_r, step_r = out
            if t % K:
                assert not send and not recv
                continue
            assert send and slot_s == (t // K) % depth
            if recv:
                assert step_r == t - tau * K and step_r >= 1 and bool(same) == (tau == 0)
                if same:
                    assert slot_r == slot_s
                else:
                    assert held[slot_r] == step_r, (K, delay, tau, t)      # still there: not yet overwritten
            else:
                assert t - tau * K < 1
            held[slot_s] = t                                              # the send of this step lands after the receive


def test_static_scratch_limit_is_stated_consistently():
    """The header, and the entry point's refusal, speak of 2^27 coordinates."""
    text = (ROOT / "include" / "asyncmesh.h").read_text()
    assert "n <= 2^27 = 134,217,728" in text
    src = (ROOT / "paper_2601_22442_amd" / "csrc" / "asyncmesh.hip").read_text()
    assert "kStaticMaxN = 1ull << 27" in src
