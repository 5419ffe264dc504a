"""Host-only checks of the C-ABI library: it loads, exports every symbol the header declares, and
rejects bad arguments before any device work.  No GPU needed (no compute call is made)."""
import ctypes as C
import math
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent


def _declared_symbols():
    text = (ROOT / "include" / "asyncmesh.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(am_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(amlib):
    names = _declared_symbols()
    assert {"am_init_state", "am_step", "am_sparse_average", "am_lookahead", "am_subset_indices",
            "am_workspace_bytes", "am_destroy"} <= set(names)
    raw = C.CDLL(str(ROOT / "paper_2601_22442_amd" / "libasyncmesh.so"))
    for name in names:
        assert hasattr(raw, name), name
    from paper_2601_22442_amd import binding
    assert sorted(binding.EXPORTS) == names


def test_config_struct_matches_header_layout(amlib):
    from paper_2601_22442_amd.binding import Config
    assert C.sizeof(Config) == 112
    assert Config.fraction.offset == 24 and Config.seed.offset == 32
    assert Config.beta1.offset == 40 and Config.gamma.offset == 56
    assert Config.grad_dtype.offset == 72 and Config.momentum_decay.offset == 80 and Config.subset_granule.offset == 88
    assert Config.msg_dtype.offset == 92 and Config.subset_kind.offset == 96
    assert Config.d_layout.offset == 100 and Config.ring_cap_lines.offset == 104


def test_workspace_bytes_and_capacity_formula(amlib):
    """A ring slot keeps the replicas of a block side by side: per block, a tile of 256 coordinates owns
    ceil(X rb / 32) whole 128-byte lines, X ~ Binomial(256, p); room for the expected total plus 12
    standard deviations."""
    am = amlib
    n, R, tau, p = 125_829_120, 8, 4, 0.05
    ntiles = n // 256
    pmf = [math.comb(256, k) * p ** k * (1 - p) ** (256 - k) for k in range(257)]
    lines = [(k * 8 + 31) // 32 for k in range(257)]
    mean = sum(a * b for a, b in zip(pmf, lines))
    var = sum(a * b * b for a, b in zip(pmf, lines)) - mean ** 2
    cap_lines = math.ceil(ntiles * mean + 12 * math.sqrt(ntiles * var)) + 64
    ring = (tau + 1) * cap_lines * 32 * 4
    b = am.workspace_bytes(am.make_config(n, R, delay=tau, fraction=p))
    tables = (tau + 2) * ntiles * 4 + ntiles * 4                  # per slot (and one spare): 4 bytes per tile; next step's sizes
    assert ring + tables <= b < ring + tables + (1 << 20)
    assert 3.5 < mean < 3.7                                        # 12.8 values of 8 replicas: about 3.6 lines a tile
    # 16 replicas = two blocks of 8, each with its own lines
    b16 = am.workspace_bytes(am.make_config(n, 16, delay=tau, fraction=p))
    assert 2 * ring + tables <= b16 < 2 * ring + tables + (1 << 20)
    # stratified variant: a tile meets at most floor(255/20) + 2 = 14 blocks -> ceil(14 * 8 / 32) = 4 lines, no margin needed
    bs = am.workspace_bytes(am.make_config(n, R, delay=tau, fraction=p, subset_kind=am.SUBSET_STRATIFIED))
    ring_s = (tau + 1) * ntiles * 4 * 32 * 4
    assert ring_s <= bs < ring_s + (64 << 20)
    full = am.workspace_bytes(am.make_config(1000, 2, delay=0, fraction=1.0))
    assert full >= 4 * 256 * 2 * 4                                 # p = 1: every tile owns all its lines
    # a caller-named slot size is taken as given (and clipped to what p = 1 would need)
    small = am.workspace_bytes(am.make_config(n, R, delay=tau, fraction=p, ring_cap_lines=1000))
    assert small < b and (tau + 1) * 1000 * 128 + tables <= small < (tau + 1) * 1000 * 128 + tables + (1 << 20)
    assert am.workspace_bytes(am.make_config(1000, 2, fraction=0.1, ring_cap_lines=10 ** 9)) == \
        am.workspace_bytes(am.make_config(1000, 2, fraction=1.0))


def test_d_layout_info(amlib):
    am = amlib
    assert am.d_layout_info(am.make_config(1000, 8)) == (1, 8, 1000)
    assert am.d_layout_info(am.make_config(1000, 8, d_layout=am.D_INTERLEAVED)) == (8, 1, 1024 * 8)
    assert am.d_layout_info(am.make_config(1000, 3, d_layout=am.D_INTERLEAVED)) == (4, 1, 1024 * 4)
    assert am.d_layout_info(am.make_config(256, 1, d_layout=am.D_INTERLEAVED)) == (1, 1, 256)
    assert am.d_layout_info(am.make_config(257, 20, d_layout=am.D_INTERLEAVED)) == (8, 3, 512 * 8)
    assert am.d_layout_info(am.make_config(5, 32, d_layout=am.D_INTERLEAVED)) == (8, 4, 256 * 8)


@pytest.mark.parametrize("kw,needle", [
    (dict(n=0), "n="), (dict(n=2 ** 32), "n="), (dict(replicas=0), "replicas"), (dict(replicas=33), "replicas"),
    (dict(avg_interval=0), "avg_interval"), (dict(fraction=0.0), "fraction"), (dict(fraction=1.5), "fraction"),
    (dict(optimizer=7), "optimizer"), (dict(correction=5), "correction"), (dict(beta1=1.0), "beta1"),
    (dict(fwd_dtype=3), "dtype"), (dict(subset_granule=16), "granule"),
    (dict(subset_kind=2), "subset_kind"), (dict(subset_kind=1, subset_granule=32), "stratified"),
    (dict(subset_kind=1, fraction=1e-10), "block"), (dict(d_layout=2), "d_layout"),
])
def test_bad_configs_are_rejected(amlib, kw, needle):
    am = amlib
    base = dict(n=1000, replicas=2)
    base.update(kw)
    with pytest.raises(am.AsyncMeshError) as e:
        am.workspace_bytes(am.make_config(**base))
    assert e.value.status == -1 and needle in str(e.value)


def test_init_rejects_bad_buffers_before_touching_the_device(amlib):
    am = amlib
    from paper_2601_22442_amd import binding as B
    cfg = am.make_config(1000, 2, delay=1, fraction=0.1)
    h = C.c_void_p(None)

    def table(vals):
        return C.cast((C.c_void_p * len(vals))(*vals), C.POINTER(C.c_void_p))

    good = table([0x10000, 0x20000])
    bufs = B.Buffers(w=good, m=good, v=good, d=good, workspace=0x100000, workspace_bytes=16)
    assert B.lib.am_init_state(C.byref(cfg), C.byref(bufs), None, C.byref(h)) == -3        # workspace too small
    assert b"workspace" in B.lib.am_last_error()
    bufs = B.Buffers(w=table([0x10000, 0x20004]), m=good, v=good, d=good, workspace=0x100000, workspace_bytes=1 << 30)
    assert B.lib.am_init_state(C.byref(cfg), C.byref(bufs), None, C.byref(h)) == -2        # misaligned w[1]
    bufs = B.Buffers(w=good, m=good, v=good, workspace=0x100000, workspace_bytes=1 << 30)
    assert B.lib.am_init_state(C.byref(cfg), C.byref(bufs), None, C.byref(h)) == -1        # EMA needs d
    cfg2 = am.make_config(1000, 2, lookahead=True, gamma=0.5)
    bufs = B.Buffers(w=good, m=good, v=good, d=good, workspace=0x100000, workspace_bytes=1 << 30)
    assert B.lib.am_init_state(C.byref(cfg2), C.byref(bufs), None, C.byref(h)) == -1       # look-ahead needs fwd
    assert B.lib.am_step(None, 1, None, 0.1, 0.5, 1.0) == -1
    assert B.lib.am_lookahead(None, 0, None, None, 4, 0.5, None) == -1
    assert B.lib.am_destroy(None) == 0


def test_schedules_of_the_paper_s_setup(amlib):
    am = amlib
    T = 30_000
    assert am.ema_lambda(1, T) == 0.5 and am.ema_lambda(1000, T) == 0.5
    assert abs(am.ema_lambda(T, T) - 0.01) < 1e-15
    assert abs(am.ema_lambda((1000 + T) // 2, T) - 0.255) < 1e-12             # cosine midpoint
    lam = [am.ema_lambda(t, T) for t in range(1, T + 1)]
    assert all(a >= b for a, b in zip(lam, lam[1:])) and 0.01 <= min(lam)
    assert am.learning_rate(0, T) == 1e-7 and abs(am.learning_rate(3000, T) - 3e-4) < 1e-18
    assert abs(am.learning_rate(1500, T) - (1e-7 + 3e-4) / 2) < 1e-15
    assert abs(am.learning_rate(T, T) - 3e-5) < 1e-18
    lr = [am.learning_rate(t, T) for t in range(3000, T + 1)]
    assert all(a >= b for a, b in zip(lr, lr[1:]))


def test_snapshot_record_layout_and_checks(amlib):
    """am_resume_state looks at the record before it looks at the device."""
    am = amlib
    from paper_2601_22442_amd import binding as B
    assert C.sizeof(B.Snapshot) == 40 + 2 * 8 * 32 and B.Snapshot.delay_now.offset == 32 and B.Snapshot.opt_steps.offset == 40
    cfg = am.make_config(1000, 2, delay=1, fraction=0.1)
    h = C.c_void_p(None)
    bufs = B.Buffers()
    assert B.lib.am_export_state(None, C.byref(B.Snapshot())) == -1
    snap = B.Snapshot(magic=123)
    assert B.lib.am_resume_state(C.byref(cfg), C.byref(bufs), None, C.byref(snap), C.byref(h)) == -1
    assert "layout" in B.lib.am_last_error().decode()
    snap = B.Snapshot(magic=0x414D534E41503033, config_digest=1)
    assert B.lib.am_resume_state(C.byref(cfg), C.byref(bufs), None, C.byref(snap), C.byref(h)) == -1
    assert "different config" in B.lib.am_last_error().decode()
    assert B.lib.am_resume_state(C.byref(cfg), C.byref(bufs), None, None, C.byref(h)) == -1
    assert not h.value


def test_active_mask_schedule_of_the_heterogeneous_setup():
    """Replica i steps speeds[i] times per round of max(speeds) ticks, the fastest in every tick."""
    from paper_2601_22442_amd.schedules import active_mask
    for speeds in ([1, 1, 1, 1], [2, 1, 2, 3], [5, 3, 1, 11], [10, 8, 1, 21]):
        K = max(speeds)
        counts = [0] * len(speeds)
        for t in range(1, 3 * K + 1):
            m = active_mask(t, speeds)
            assert m & (1 << speeds.index(K))
            for i in range(len(speeds)):
                counts[i] += (m >> i) & 1
            if t % K == 0:
                assert counts == [s * (t // K) for s in speeds]
    assert [active_mask(t, [1, 3]) for t in (1, 2, 3, 4)] == [0b10, 0b10, 0b11, 0b10]
    with pytest.raises(ValueError):
        active_mask(1, [0, 2])


def test_no_fallback_without_the_library(tmp_path):
    """In a tree where nothing is built the builder imports, and the first use of the binding fails loudly."""
    import shutil
    import subprocess
    import sys
    pkg = tmp_path / "paper_2601_22442_amd"
    pkg.mkdir()
    for f in ("__init__.py", "binding.py", "schedules.py", "build.py"):
        shutil.copy(ROOT / "paper_2601_22442_amd" / f, pkg / f)
    code = ("import paper_2601_22442_amd as am; from paper_2601_22442_amd.build import LIB; assert not LIB.exists()\n"
            "assert am.active_mask(1, [1, 2]) == 2\n"
            "try:\n    am.make_config(10, 2)\nexcept ImportError as e:\n    assert 'no fallback' in str(e); print('refused')\n")
    out = subprocess.run([sys.executable, "-c", code], cwd=tmp_path, capture_output=True, text=True)
    assert out.returncode == 0 and "refused" in out.stdout, out.stderr


def test_header_is_plain_c_and_the_binding_mirrors_its_layout(amlib, tmp_path):
    """A C11 program that includes the header, links the library, prints the layout the C compiler
    gives the structs and makes two host-only calls."""
    import subprocess
    from paper_2601_22442_amd import binding as B
    src = tmp_path / "abi.c"
    src.write_text(r"""
#include <stddef.h>
#include <stdio.h>
#include "asyncmesh.h"
int main(void) {
    printf("%zu %zu %zu %zu %zu\n", sizeof(am_config), offsetof(am_config, fraction), offsetof(am_config, momentum_decay),
           offsetof(am_config, ring_cap_lines), sizeof(am_buffers));
    printf("%zu %zu %zu\n", sizeof(am_snapshot), offsetof(am_snapshot, opt_steps), offsetof(am_snapshot, mu_product));
    am_config c = {0};
    c.n = 125829120u; c.replicas = 8; c.delay = 4; c.avg_interval = 1; c.optimizer = AM_OPT_ADAMW; c.fraction = 0.05;
    c.beta1 = 0.9f; c.beta2 = 0.999f; c.eps = 1e-8f; c.correction = AM_CORR_EMA;
    uint64_t bytes = 0;
    am_status s = am_workspace_bytes(&c, &bytes);
    printf("%d %llu\n", (int)s, (unsigned long long)bytes);
    c.replicas = 99;
    s = am_workspace_bytes(&c, &bytes);
    printf("%d %s\n", (int)s, am_last_error());
    return 0;
}
""")
    exe = tmp_path / "abi"
    lib_dir = ROOT / "paper_2601_22442_amd"
    subprocess.run(["gcc", "-std=c11", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", str(ROOT / "include"), "-o", str(exe), str(src),
                    "-L", str(lib_dir), "-lasyncmesh", f"-Wl,-rpath,{lib_dir}"], check=True)
    out = subprocess.run([str(exe)], capture_output=True, text=True, check=True).stdout.splitlines()
    assert out[0].split() == [str(C.sizeof(B.Config)), str(B.Config.fraction.offset), str(B.Config.momentum_decay.offset),
                              str(B.Config.ring_cap_lines.offset), str(C.sizeof(B.Buffers))]
    assert out[1].split() == [str(C.sizeof(B.Snapshot)), str(B.Snapshot.opt_steps.offset), str(B.Snapshot.mu_product.offset)]
    status, nbytes = out[2].split()
    assert status == "0" and int(nbytes) == am_bytes(amlib)
    assert out[3].startswith("-1 ") and "replicas" in out[3]


def am_bytes(am):
    return am.workspace_bytes(am.make_config(125_829_120, 8, delay=4, fraction=0.05))


def test_library_carries_the_digest_of_its_sources(amlib):
    """am_version() ends with a digest of the source files the library was built from; the test
    fixture has already refused a library whose digest is not that of the files in the tree."""
    from paper_2601_22442_amd.build import source_hash
    v = amlib.version()
    assert v.startswith("asyncmesh-gfx950 ") and v.endswith("src:" + source_hash())
    from paper_2601_22442_amd.build import check_library_is_current
    with pytest.raises(RuntimeError):
        check_library_is_current("asyncmesh-gfx950 0.2 src:0123456789abcdef")


def test_binding_refuses_wrong_gradients_before_any_launch(amlib):
    """The C side sees raw pointers only, so the binding checks count, dtype, size, device and
    contiguity of the gradients (no GPU needed: the checks run on meta-data alone)."""
    import torch
    am = amlib
    from paper_2601_22442_amd import binding as B

    class FakeStage(B.Stage):
        def __init__(self, cfg):
            self.cfg, self.device = cfg, torch.device("cpu")
            self.n, self.R = int(cfg.n), int(cfg.replicas)
            self._handle = C.c_void_p(None)

    st = FakeStage(am.make_config(100, 2))
    ok = [torch.zeros(100) for _ in range(2)]
    for bad in ([ok[0]], [ok[0], torch.zeros(99)], [ok[0], torch.zeros(100, dtype=torch.bfloat16)],
                [ok[0], torch.zeros(200)[::2]], [ok[0], None]):
        with pytest.raises(ValueError):
            st._check_grads(bad)
    st16 = FakeStage(am.make_config(100, 2, grad_dtype=am.BF16))
    with pytest.raises(ValueError):
        st16._check_grads(ok)
    with pytest.raises(ValueError):
        B._check_tensors("w", ok, 2, 101, torch.float32, torch.device("cpu"))
