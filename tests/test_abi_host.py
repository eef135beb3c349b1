"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, rejects invalid arguments before touching the device, and its host-only
planner (Eq. 9, Eq. 10) reproduces the paper's worked numbers."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    return binding


def declared_functions():
    text = open(os.path.join(ROOT, "include", "cocodc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cocodc_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(B):
    names = declared_functions()
    assert len(names) >= 14 and "cocodc_sync_step" in names
    lib = C.CDLL(B.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(B.EXPORTS) == names


def test_header_is_plain_c():
    """The boundary is a C ABI: the header compiles as C99 without warnings, and a C program that
    uses its types links against the library."""
    import subprocess, tempfile
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    inc = os.path.join(root, "include")
    r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                        os.path.join(inc, "cocodc.h")], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    src = r"""
#include "cocodc.h"
#include <stdio.h>
int main(void) {
  cocodc_fragment_t f = {0, 16};
  cocodc_hparams_t hp = {5, 100, 0.5, 0.7, 0.9, 1, 1, 0, 2, 0, 1.0, 0, 0};
  int64_t N = 0, h = 0;
  (void)f; (void)hp;
  if (cocodc_sync_plan(4, 100, 0.4, 1.0, 5.0, &N, &h) != COCODC_OK) return 2;
  printf("%lld %lld %zu %s\n", (long long)N, (long long)h, cocodc_workspace_bytes(4, 1u << 20),
         cocodc_status_string(COCODC_ERR_ALIAS));
  return 0;
}
"""
    lib = os.path.join(root, "paper_2504_17672_amd", "libcocodc.so")
    with tempfile.TemporaryDirectory() as d:
        c = os.path.join(d, "t.c")
        open(c, "w").write(src)
        exe = os.path.join(d, "t")
        r = subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-I", inc, c, lib, "-Wl,-rpath," + os.path.dirname(lib),
                            "-Wl,-rpath,/opt/rocm/lib", "-o", exe], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr
        r = subprocess.run([exe], capture_output=True, text=True)
        assert r.returncode == 0, (r.stdout, r.stderr)
        N, h, ws, name = r.stdout.split()
        assert (int(N), int(h)) == (8, 12) and int(ws) > 0 and name == "COCODC_ERR_ALIAS"


def test_workspace_size(B):
    assert B.cocodc_workspace_bytes(0, 100) == 0
    assert B.cocodc_workspace_bytes(B.COCODC_MAX_FRAGMENTS + 1, 100) == 0
    a = B.cocodc_workspace_bytes(4, 1 << 20)
    b = B.cocodc_workspace_bytes(4, 1 << 30)
    assert 0 < a < b and a % 256 == 0
    # 32 bytes of partial sums per tile of 4096 elements (16 KiB of one buffer): 0.2 %, far below 1 %
    assert b < 0.01 * 4 * (1 << 30)


def test_planner_golden_and_ranges(B):
    rows = [ln.split() for ln in open(os.path.join(GOLDEN, "planner_worked_example.txt"))
            if ln.strip() and not ln.startswith("#")]
    for K, H, gamma, Tc, Ts, N, h in rows:
        assert B.cocodc_sync_plan(int(K), int(H), float(gamma), float(Tc), float(Ts)) == (0, int(N), int(h))
    assert B.cocodc_sync_plan(4, 100, 0.4, 1.0, 50.0) == (0, 4, 25)
    assert B.cocodc_sync_plan(4, 100, 1.0, 2.0, 1.0) == (0, 200, 0)
    assert B.cocodc_sync_plan(0, 100, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_sync_plan(4, 100, 1.5, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_sync_plan(4, 100, float("nan"), 1.0, 5.0)[0] == B.COCODC_ERR_NONFINITE


def test_planner_agrees_with_oracle_on_a_grid(B, ref):
    for K in (1, 4, 12):
        for H in (1, 50, 100, 1000):
            for gamma in (0.1, 0.4, 1.0):
                for ratio in (0.5, 1.0, 5.0, 37.0):
                    assert B.cocodc_sync_plan(K, H, gamma, 1.0, ratio) == ref.sync_plan(K, H, gamma, 1.0, ratio)


def test_status_strings(B):
    assert B.cocodc_status_string(0) == "COCODC_OK"
    assert B.cocodc_status_string(B.COCODC_ERR_ALIAS) == "COCODC_ERR_ALIAS"
    assert B.cocodc_status_string(-99) == "COCODC_ERR_UNKNOWN"


def test_invalid_arguments_are_rejected_before_any_device_work(B):
    """Fake (never dereferenced) device addresses: every call below must fail validation."""
    n = 4096
    nb = 4 * n
    base = 0x10000000
    tm, ts, tg, m, dg, pg = (base + i * 0x100000 for i in range(6))
    R, sel, nsel, sums, ws = (base + 0x1000000 + i * 0x100000 for i in range(5))
    wsb = B.cocodc_workspace_bytes(2, n)
    frags = [(0, 2048), (2048, 2048)]
    hp = B.hparams(5, 100)
    I_p, t_b = [1, 1], [0, 0]

    def step(**kw):
        a = dict(frags=frags, n=n, tm=tm, ts=ts, tg=tg, m=m, dg=dg, pg=pg, I_p=I_p, t_b=t_b, budget=1, hp=hp,
                 R=R, sel=sel, nsel=nsel, sums=sums, ws=ws, wsb=wsb, K=None)
        a.update(kw)
        return B.cocodc_sync_step(a["frags"], a["n"], a["tm"], a["ts"], a["tg"], a["m"], a["dg"], a["pg"],
                                  a["I_p"], a["t_b"], 10, a["budget"], a["hp"], a["R"], a["sel"], a["nsel"],
                                  a["sums"], a["ws"], a["wsb"], stream=0, K=a["K"])
    assert step(tm=None) == B.COCODC_ERR_NULL
    assert step(R=None) == B.COCODC_ERR_NULL
    assert step(I_p=None) == B.COCODC_ERR_NULL
    assert step(hp=None) == B.COCODC_ERR_NULL
    assert step(frags=None, K=2) == B.COCODC_ERR_NULL
    assert step(ws=None) == B.COCODC_ERR_NULL
    assert step(tg=tg + 1) == B.COCODC_ERR_ALIGN
    assert step(R=R + 4) == B.COCODC_ERR_ALIGN
    assert step(ws=ws + 16) == B.COCODC_ERR_ALIGN
    assert step(K=0) == B.COCODC_ERR_RANGE
    assert step(K=B.COCODC_MAX_FRAGMENTS + 1) == B.COCODC_ERR_RANGE
    assert step(frags=[(0, 2048), (2047, 2049)]) == B.COCODC_ERR_RANGE
    assert step(frags=[(0, 2048), (2048, 2049)]) == B.COCODC_ERR_RANGE
    assert step(frags=[(2 ** 63, 2 ** 63), (0, 1)]) == B.COCODC_ERR_RANGE
    assert step(budget=-1) == B.COCODC_ERR_RANGE
    assert step(n=(1 << 44) + 4, wsb=1 << 62) == B.COCODC_ERR_RANGE
    for bad in (dict(tau=-1), dict(H=0), dict(nesterov=2), dict(drift_sign=0), dict(score_src=2),
                dict(norm_kind=3), dict(merge_mode=3), dict(delta_src=2), dict(pg_format=2), dict(pg_format=-1)):
        kw = dict(tau=5, H=100)
        kw.update(bad)
        assert step(hp=B.hparams(**kw)) == B.COCODC_ERR_RANGE, bad
    for bad in (dict(lam=float("inf")), dict(eta=float("nan")), dict(mu=float("-inf")), dict(alpha=float("nan"))):
        assert step(hp=B.hparams(5, 100, **bad)) == B.COCODC_ERR_NONFINITE, bad
    assert step(wsb=wsb - 1) == B.COCODC_ERR_WORKSPACE
    assert step(tm=tg) == B.COCODC_ERR_ALIAS
    assert step(pg=dg + nb // 2) == B.COCODC_ERR_ALIAS
    assert step(sums=R) == B.COCODC_ERR_ALIAS

    # the entry point without a workspace: same checks, and a size limit instead of a workspace size
    def noalloc(**kw):
        a = dict(frags=frags, n=n, tm=tm, budget=1, hp=hp, R=R, K=None)
        a.update(kw)
        return B.cocodc_sync_step_noalloc(a["frags"], a["n"], a["tm"], ts, tg, m, dg, pg, I_p, t_b, 10, a["budget"],
                                          a["hp"], a["R"], sel, nsel, sums, stream=0, K=a["K"])
    assert noalloc(tm=None) == B.COCODC_ERR_NULL
    assert noalloc(R=R + 4) == B.COCODC_ERR_ALIGN
    assert noalloc(budget=-1) == B.COCODC_ERR_RANGE
    assert noalloc(hp=B.hparams(5, 0)) == B.COCODC_ERR_RANGE
    assert noalloc(frags=[(0, 2048), (2047, 2049)]) == B.COCODC_ERR_RANGE
    assert noalloc(tm=tg) == B.COCODC_ERR_ALIAS
    big = 1 << 34
    assert B.cocodc_workspace_bytes(2, big) > B.COCODC_NOALLOC_SCRATCH_BYTES
    assert noalloc(frags=[(0, big // 2), (big // 2, big // 2)], n=big) in (B.COCODC_ERR_WORKSPACE, B.COCODC_ERR_ALIAS)
    assert B.cocodc_sync_step_noalloc([(0, big)], big, base, base + (1 << 40), base + (2 << 40), base + (3 << 40),
                                      base + (4 << 40), None, [1], [0], 10, 1, hp, base + (5 << 40),
                                      base + (5 << 40) + 4096, base + (5 << 40) + 8192, None, stream=0) \
        == B.COCODC_ERR_WORKSPACE

    def event(mask, **kw):
        a = dict(tm=tm, R=R, ws=ws, wsb=wsb, frags=frags)
        a.update(kw)
        return B.cocodc_sync_event(a["frags"], n, mask, a["tm"], ts, tg, m, dg, pg, I_p, t_b, 10, 1, hp, a["R"], sel,
                                   nsel, sums, a["ws"], a["wsb"], stream=0)
    assert event(None) == B.COCODC_ERR_NULL
    assert event([1, 0], tm=None) == B.COCODC_ERR_NULL
    assert event([1, 0], R=R + 4) == B.COCODC_ERR_ALIGN
    assert event([0, 0], frags=[(0, 2048), (2047, 2049)]) == B.COCODC_ERR_RANGE   # checked whatever the mask says
    assert event([1, 1], wsb=wsb - 1) == B.COCODC_ERR_WORKSPACE
    assert step(ws=tm) == B.COCODC_ERR_ALIAS

    assert B.cocodc_pseudograd_bf16(frags, n, tg, tm, pg, None, ws, wsb, stream=0, pg_format=2) == B.COCODC_ERR_RANGE
    assert B.cocodc_pseudograd_bf16(frags, n, tg, tm, None, None, ws, wsb, stream=0, pg_format=1) == B.COCODC_ERR_NULL
    assert B.cocodc_pseudograd(frags, n, tg, tm, None, None, ws, wsb, stream=0) == B.COCODC_ERR_NULL
    assert B.cocodc_pseudograd(frags, n, tg, tm, tm, None, ws, wsb, stream=0) == B.COCODC_ERR_ALIAS
    assert B.cocodc_outer_nesterov(frags, n, tg, m, tg, hp, ws, wsb, stream=0) == B.COCODC_ERR_ALIAS
    assert B.cocodc_outer_nesterov(frags, n, tg, m, dg, None, ws, wsb, stream=0) == B.COCODC_ERR_NULL
    assert B.cocodc_delay_compensate(frags, n, tm, ts, tm, hp, ws, wsb, stream=0) == B.COCODC_ERR_ALIAS
    assert B.cocodc_delay_compensate(frags, n, tm, ts, tg, hp, ws, 8, stream=0) == B.COCODC_ERR_WORKSPACE
    assert B.cocodc_delay_compensate(frags, n, tm, ts, tg, B.hparams(5, 100, delta_src=1), ws, wsb,
                                     stream=0) == B.COCODC_ERR_RANGE  # needs the previous global state
    assert B.cocodc_fragment_scores(frags, n, dg, I_p, 3, R, None, ws, wsb, stream=0) == B.COCODC_ERR_RANGE
    assert B.cocodc_fragment_scores(frags, n, dg, None, 2, R, None, ws, wsb, stream=0) == B.COCODC_ERR_NULL
    assert B.cocodc_select_fragments(2, R, t_b, 10, 0, 1, sel, nsel, ws, wsb, stream=0) == B.COCODC_ERR_RANGE
    assert B.cocodc_select_fragments(2, R, t_b, 10, 100, -1, sel, nsel, ws, wsb, stream=0) == B.COCODC_ERR_RANGE
    assert B.cocodc_select_fragments(2, R, None, 10, 100, 1, sel, nsel, ws, wsb, stream=0) == B.COCODC_ERR_NULL
    assert B.cocodc_select_fragments(2, R, t_b, 10, 100, 1, R, nsel, ws, wsb, stream=0) == B.COCODC_ERR_ALIAS


def test_loop_create_checks_its_table(B):
    hp = B.hparams(5, 100)
    ok = [(0, 10, 0), (10, 10, 1), (30, 5, 0)]
    rc, loop = B.cocodc_loop_create_segmented(ok, 2, 40, hp, 0.4, 1.0, 5.0)
    assert rc == 0 and B.cocodc_loop_plan(loop) == (0, 8, 12)
    B.cocodc_loop_destroy(loop)
    assert B.cocodc_loop_create_segmented([(0, 10, 0), (5, 10, 1)], 2, 40, hp, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create_segmented([(0, 10, 2)], 2, 40, hp, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create_segmented([(35, 10, 0)], 2, 40, hp, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create_segmented(None, 2, 40, hp, 0.4, 1.0, 5.0, S=3)[0] == B.COCODC_ERR_NULL
    assert B.cocodc_loop_create_segmented(ok, 0, 40, hp, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create_segmented(ok, 2, 40, None, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_NULL
    assert B.cocodc_loop_create_segmented(ok, 2, 40, hp, 0.0, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create([(0, 10), (5, 10)], 20, hp, 0.4, 1.0, 5.0)[0] == B.COCODC_ERR_RANGE
    assert B.cocodc_loop_create(None, 20, hp, 0.4, 1.0, 5.0, K=2)[0] == B.COCODC_ERR_NULL


def test_loop_step_rejects_bad_buffers_before_any_device_work(B):
    """Fake (never dereferenced) device addresses: cocodc_loop_step checks every pointer of its buffer
    struct, their alignment and overlap, the workspace size and the step number before it enqueues
    anything, and a rejected step leaves the schedule as it was."""
    import ctypes as C
    n, K = 4096, 2
    frags = [(0, 2048), (2048, 2048)]
    rc, loop = B.cocodc_loop_create(frags, n, B.hparams(2, 10), 1.0, 1.0, 5.0)
    assert rc == 0
    base = 0x20000000
    addr = dict(theta_m=base, theta_m_send=base + 0x100000, theta_g=base + 0x200000, momentum=base + 0x300000,
                delta_g=base + 0x400000, delta_m_out=base + 0x500000, R=base + 0x600000, sel=base + 0x700000,
                n_sel=base + 0x800000, workspace=base + 0x900000)
    wsb = B.cocodc_workspace_bytes(K, n)

    def step(t=5, wsb=wsb, **kw):
        a = dict(addr)
        a.update(kw)
        buf = B.cocodc_loop_buffers_t(a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                                      a["delta_m_out"], a["R"], a["sel"], a["n_sel"], a["workspace"], wsb)
        return B.cocodc_loop_step(loop, t, buf, stream=0)[0]
    try:
        for name in addr:
            assert step(**{name: None}) == B.COCODC_ERR_NULL, name
        assert step(theta_g=addr["theta_g"] + 2) == B.COCODC_ERR_ALIGN
        assert step(R=addr["R"] + 4) == B.COCODC_ERR_ALIGN
        assert step(workspace=addr["workspace"] + 64) == B.COCODC_ERR_ALIGN
        assert step(wsb=wsb - 1) == B.COCODC_ERR_WORKSPACE
        assert step(delta_m_out=addr["theta_m"]) == B.COCODC_ERR_ALIAS
        assert step(momentum=addr["theta_g"] + 4 * n - 16) == B.COCODC_ERR_ALIAS
        assert step(delta_m_out=addr["delta_g"] + 16) == B.COCODC_ERR_ALIAS      # only the exact in-place buffer is allowed
        assert step(t=0) == B.COCODC_ERR_RANGE and step(t=-3) == B.COCODC_ERR_RANGE
        assert B.cocodc_loop_state(loop) == (0, [0, 0], [0, 0], [-1, -1])
        assert B.cocodc_loop_last_sent(loop) == (0, -1, -1)
        assert B.cocodc_loop_due(loop, 100) == (0, [])
        assert step(t=3) == 0          # h = 5: neither an arrival nor a decision at step 3, nothing is enqueued
        assert step(t=3) == B.COCODC_ERR_RANGE and step(t=2) == B.COCODC_ERR_RANGE   # steps never go back
    finally:
        B.cocodc_loop_destroy(loop)


def test_bf16_entry_points_reject_bad_arguments_before_any_device_work(B):
    """Fake (never dereferenced) device addresses through the 16-bit fused step on segments, the 16-bit event
    and the 16-bit loop step."""
    n, K = 4096, 2
    base = 0x30000000
    tm, ts, tg, m, dg, pg = (base + i * 0x100000 for i in range(6))
    R, sel, nsel, sums, ws = (base + 0x1000000 + i * 0x100000 for i in range(5))
    frags = [(0, 2048), (2048, 2048)]
    segs = [(0, 1000, 0), (1000, 1048, 1), (2048, 2048, 0)]
    hp = B.hparams(5, 100, pg_format=B.COCODC_PG_F16)
    I_p, t_b = [1, 1], [0, 0]
    wss = B.cocodc_workspace_bytes_segmented(len(segs), K, n)

    def seg(**kw):
        a = dict(segs=segs, tm=tm, pg=pg, hp=hp, R=R, ws=ws, wsb=wss, I_p=I_p, budget=1)
        a.update(kw)
        return B.cocodc_sync_step_bf16_segmented(a["segs"], K, n, a["tm"], ts, tg, m, dg, a["pg"], a["I_p"], t_b, 10,
                                                 a["budget"], a["hp"], a["R"], sel, nsel, sums, a["ws"], a["wsb"],
                                                 stream=0)
    assert seg(tm=None) == B.COCODC_ERR_NULL and seg(I_p=None) == B.COCODC_ERR_NULL and seg(hp=None) == B.COCODC_ERR_NULL
    assert seg(tm=tm + 1) == B.COCODC_ERR_ALIGN and seg(R=R + 4) == B.COCODC_ERR_ALIGN
    assert seg(segs=[(0, 1000, 0), (999, 10, 1)]) == B.COCODC_ERR_RANGE
    assert seg(segs=[(0, 1000, 2)]) == B.COCODC_ERR_RANGE
    assert seg(budget=-1) == B.COCODC_ERR_RANGE
    assert seg(hp=B.hparams(5, 100, pg_format=2)) == B.COCODC_ERR_RANGE
    assert seg(wsb=wss - 1) == B.COCODC_ERR_WORKSPACE
    assert seg(pg=tm) == B.COCODC_ERR_ALIAS
    assert seg(pg=dg) == B.COCODC_ERR_ALIAS          # a 16-bit pseudo-gradient cannot share the fp32 average's buffer
    assert seg(ws=tm) == B.COCODC_ERR_ALIAS

    wsb = B.cocodc_workspace_bytes(K, n)

    def event(mask, **kw):
        a = dict(tm=tm, R=R, ws=ws, wsb=wsb, frags=frags, pg=pg)
        a.update(kw)
        return B.cocodc_sync_event_bf16(a["frags"], n, mask, a["tm"], ts, tg, m, dg, a["pg"], I_p, t_b, 10, 1, hp,
                                        a["R"], sel, nsel, sums, a["ws"], a["wsb"], stream=0)
    assert event(None) == B.COCODC_ERR_NULL
    assert event([1, 0], tm=None) == B.COCODC_ERR_NULL
    assert event([1, 0], R=R + 4) == B.COCODC_ERR_ALIGN
    assert event([4, 0]) == B.COCODC_ERR_RANGE
    assert event([0, 0], frags=[(0, 2048), (2047, 2049)]) == B.COCODC_ERR_RANGE
    assert event([1, 1], wsb=wsb - 1) == B.COCODC_ERR_WORKSPACE
    assert event([1, 2], pg=ts) == B.COCODC_ERR_ALIAS

    rc, loop = B.cocodc_loop_create(frags, n, B.hparams(2, 10), 1.0, 1.0, 5.0)
    assert rc == 0
    addr = dict(theta_m=tm, theta_m_send=ts, theta_g=tg, momentum=m, delta_g=dg, delta_m_out=pg, R=R, sel=sel,
                n_sel=nsel, workspace=ws)

    def step(t=5, wsb=wsb, **kw):
        a = dict(addr)
        a.update(kw)
        buf = B.cocodc_loop_buffers_t(a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                                      a["delta_m_out"], a["R"], a["sel"], a["n_sel"], a["workspace"], wsb)
        return B.cocodc_loop_step_bf16(loop, t, buf, stream=0)[0]
    try:
        for name in addr:
            assert step(**{name: None}) == B.COCODC_ERR_NULL, name
        assert step(theta_m=tm + 1) == B.COCODC_ERR_ALIGN and step(theta_g=tg + 2) == B.COCODC_ERR_ALIGN
        assert step(wsb=wsb - 1) == B.COCODC_ERR_WORKSPACE
        assert step(delta_m_out=dg) == B.COCODC_ERR_ALIAS       # no in-place exchange buffer in 16 bits
        assert step(theta_m_send=tm + 2 * n - 2) == B.COCODC_ERR_ALIAS
        assert step(t=0) == B.COCODC_ERR_RANGE
        assert B.cocodc_loop_state(loop) == (0, [0, 0], [0, 0], [-1, -1])
        assert step(t=3) == 0 and step(t=3) == B.COCODC_ERR_RANGE
    finally:
        B.cocodc_loop_destroy(loop)


def test_segmented_event_rejects_bad_arguments_before_any_device_work(B):
    n, K = 4096, 2
    base = 0x40000000
    tm, ts, tg, m, dg, pg = (base + i * 0x100000 for i in range(6))
    R, sel, nsel, sums, ws = (base + 0x1000000 + i * 0x100000 for i in range(5))
    segs = [(0, 1000, 0), (1000, 1048, 1), (2048, 2048, 0)]
    hp = B.hparams(5, 100)
    I_p, t_b = [1, 1], [0, 0]
    wss = B.cocodc_workspace_bytes_segmented(len(segs), K, n)

    def event(mask, **kw):
        a = dict(segs=segs, tm=tm, R=R, ws=ws, wsb=wss, pg=pg, K=K)
        a.update(kw)
        return B.cocodc_sync_event_segmented(a["segs"], a["K"], n, mask, a["tm"], ts, tg, m, dg, a["pg"], I_p, t_b, 10,
                                             1, hp, a["R"], sel, nsel, sums, a["ws"], a["wsb"], stream=0)
    assert event(None) == B.COCODC_ERR_NULL
    assert event([1, 0], tm=None) == B.COCODC_ERR_NULL
    assert event([1, 0], R=R + 4) == B.COCODC_ERR_ALIGN
    assert event([1, 8]) == B.COCODC_ERR_RANGE
    assert event([0, 0], segs=[(0, 1000, 0), (999, 10, 1)]) == B.COCODC_ERR_RANGE   # checked whatever the mask says
    assert event([1, 0], segs=[(0, 1000, 2)]) == B.COCODC_ERR_RANGE
    assert event([1, 1], wsb=wss - 1) == B.COCODC_ERR_WORKSPACE
    assert event([1, 2], pg=tm) == B.COCODC_ERR_ALIAS

    def event16(mask, **kw):
        a = dict(segs=segs, tm=tm, R=R, wsb=wss, pg=pg)
        a.update(kw)
        return B.cocodc_sync_event_bf16_segmented(a["segs"], K, n, mask, a["tm"], ts, tg, m, dg, a["pg"], I_p, t_b, 10,
                                                  1, hp, a["R"], sel, nsel, sums, ws, a["wsb"], stream=0)
    assert event16(None) == B.COCODC_ERR_NULL
    assert event16([1, 0], tm=tm + 1) == B.COCODC_ERR_ALIGN
    assert event16([1, 8]) == B.COCODC_ERR_RANGE
    assert event16([1, 0], segs=[(0, 1000, 0), (999, 10, 1)]) == B.COCODC_ERR_RANGE
    assert event16([1, 1], wsb=wss - 1) == B.COCODC_ERR_WORKSPACE
    assert event16([1, 2], pg=dg) == B.COCODC_ERR_ALIAS
