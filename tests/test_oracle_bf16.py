"""Pins of the oracle's bf16 variant (local parameters kept in bfloat16, Sec. 4.1): the
rounding primitive against torch's float32 -> bfloat16 conversion and against exact rational
arithmetic, and the bf16 fused step against the pinned fp32 step on the widened inputs.
CPU only."""
import math
from fractions import Fraction

import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth


def bf16_bits(t32):
    """torch's own float32 -> bfloat16 conversion, as raw bit patterns."""
    return t32.to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def test_widen_and_round_are_inverse_on_every_pattern(ref):
    for b in range(0, 65536, 1):
        x = ref.widen_bf16(b)
        if math.isnan(x):
            assert ref.round_bf16(x) == 0x7FC0
        else:
            assert ref.round_bf16(x) == b


def test_rounding_matches_torch_on_float32_values(ref):
    g = torch.Generator().manual_seed(5)
    vals = torch.cat([
        torch.empty(20000).normal_(0, 0.02, generator=g), torch.empty(20000).normal_(0, 1e-3, generator=g),
        torch.empty(2000).normal_(0, 1e30, generator=g), torch.empty(2000).normal_(0, 1e-39, generator=g),
        torch.tensor([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895e38, 3.4e38, float("inf"), float("-inf"),
                      1e-45, -1e-40, 9.2e-41, 4.6e-41])])
    want = bf16_bits(vals)
    got = np.array([ref.round_bf16(float(v)) for v in vals.numpy()], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_rounding_of_doubles_is_nearest_ties_to_even(ref):
    rng = np.random.default_rng(7)
    xs = list(rng.normal(0, 0.02, 3000)) + list(rng.normal(0, 1e-39, 300)) + [1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8,
                                                                          1 + 2.0 ** -8 + 2.0 ** -50,
                                                                          1 + 2.0 ** -8 - 2.0 ** -50]
    for x in xs:
        b = ref.round_bf16(float(x))
        r = Fraction(ref.widen_bf16(b))
        # neighbours on the bf16 grid
        up = ref.widen_bf16(b + 1) if (b & 0x7FFF) < 0x7F7F else None
        dn = ref.widen_bf16(b - 1) if (b & 0x7FFF) > 0 else ref.widen_bf16(b ^ 0x8000 | 1)
        err = abs(Fraction(float(x)) - r)
        for nb in (up, dn):
            if nb is None or math.isinf(nb):
                continue
            e2 = abs(Fraction(float(x)) - Fraction(nb))
            assert err <= e2
            if err == e2:
                assert b % 2 == 0  # a tie goes to the even pattern


def _bf16_state(wl, seed, amplified=False):
    st = {k: v.numpy() for k, v in synth.make_state(wl, "cpu", seed=seed, amplified=amplified).items()}
    for k in ("theta_m", "theta_m_send"):
        st[k] = bf16_bits(torch.from_numpy(st[k])).copy()
    return st


def _widen(u16):
    return torch.from_numpy(u16.view(np.int16)).view(torch.bfloat16).float().numpy()


def test_bf16_step_is_the_fp32_step_on_widened_inputs_rounded_once(ref):
    for amplified, tau, H in ((False, 5, 100), (True, 2, 1)):
        wl = synth.Workload("b", (3000, 1999, 0, 777), tau=tau, H=H, budget=2)
        bk = synth.bookkeeping(wl, "mixed")
        hp = ref.hparams(tau, H)
        a = _bf16_state(wl, 11, amplified)
        w = {k: (v.copy() if v.dtype == np.float32 else _widen(v)) for k, v in a.items()}
        pg = np.zeros(wl.n_total, np.uint16)
        oa = ref.sync_step_bf16(wl.frags, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                                pg, bk.I_p, bk.t_b, bk.t_g, 2, hp, shadow=True)
        pg32 = np.zeros(wl.n_total, np.float32)
        tm_before, tg_before = w["theta_m"].copy(), w["theta_g"].copy()
        ow = ref.sync_step(wl.frags, w["theta_m"], w["theta_m_send"], w["theta_g"], w["momentum"], w["delta_g"],
                           pg32, bk.I_p, bk.t_b, bk.t_g, 2, hp, shadow=True)
        assert oa["rc"] == 0 and ow["rc"] == 0
        assert np.array_equal(a["theta_g"], w["theta_g"]) and np.array_equal(a["momentum"], w["momentum"])
        assert np.array_equal(oa["theta_m64"], ow["theta_m64"])
        assert np.array_equal(oa["R"], ow["R"]) and np.array_equal(oa["sums"], ow["sums"])
        assert oa["sel"].tolist() == ow["sel"].tolist()
        want_tm = np.array([ref.round_bf16(v) for v in ow["theta_m64"]], dtype=np.uint16)
        assert np.array_equal(a["theta_m"], want_tm)
        diff = tg_before.astype(np.float64) - tm_before.astype(np.float64)
        want_pg = np.array([ref.round_bf16(v) for v in diff], dtype=np.uint16)
        assert np.array_equal(pg, want_pg)
        # the rounded result is within half a bf16 step of the fp64 value
        rel = np.abs(_widen(a["theta_m"]).astype(np.float64) - ow["theta_m64"]) / np.maximum(np.abs(ow["theta_m64"]), 1e-30)
        assert rel.max() <= 2.0 ** -8


def test_bf16_pseudograd_records_the_send_time_parameters(ref):
    wl = synth.Workload("b", (500, 300), tau=5, H=100)
    a = _bf16_state(wl, 12)
    pg = np.zeros(800, np.uint16)
    send = np.zeros(800, np.uint16)
    assert ref.pseudograd_bf16([(100, 600)], a["theta_g"], a["theta_m"], pg, send) == 0
    assert np.array_equal(send[100:700], a["theta_m"][100:700]) and not send[:100].any() and not send[700:].any()
    for i in (100, 333, 699):
        exact = Fraction(float(a["theta_g"][i])) - Fraction(ref.widen_bf16(int(a["theta_m"][i])))
        assert pg[i] == ref.round_bf16(float(exact))  # the difference is exact in fp64 here
    assert not pg[:100].any() and not pg[700:].any()


# ------------------------------------------------------------------ IEEE binary16 pseudo-gradient
def test_f16_widen_and_round_are_inverse_on_every_pattern_and_agree_with_numpy(ref):
    for b in range(65536):
        x = ref.widen_f16(b)
        want = float(np.array([b], np.uint16).view(np.float16)[0])
        if math.isnan(want):
            assert math.isnan(x) and ref.round_f16(x) == 0x7E00
        else:
            assert x == want and ref.round_f16(x) == b


F16_TRAPS = [65504.0, 65519.999, 65520.0, 65520.0001, -65520.0, 65536.0, 1e6, -1e300, 2.0 ** -24, 2.0 ** -25,
             2.0 ** -25 * (1 + 2.0 ** -30), 2.0 ** -25 * (1 - 2.0 ** -30), 3 * 2.0 ** -25, 2.0 ** -14, 2.0 ** -14 - 2.0 ** -25,
             1 + 2.0 ** -11, 1 + 2.0 ** -11 + 2.0 ** -40, 1 + 2.0 ** -11 - 2.0 ** -40, 1 + 3 * 2.0 ** -11,
             # a double that rounds to a binary32 lying exactly on a binary16 tie (rounding twice would go wrong)
             1 + 2.0 ** -11 + 2.0 ** -30, 1 + 3 * 2.0 ** -11 - 2.0 ** -30, -(2 + 2.0 ** -10 + 2.0 ** -29),
             0.0, -0.0, 1e-320, -4e-46, float("inf"), float("-inf")]


def _f16_samples():
    rng = np.random.default_rng(11)
    return np.concatenate([rng.normal(0, 1, 20000), rng.normal(0, 0.02, 20000), rng.normal(0, 1e-5, 10000),
                           rng.normal(0, 1e-7, 5000), rng.normal(0, 3e4, 5000), np.array(F16_TRAPS)])


def test_f16_rounding_matches_numpy_from_float64_and_torch_from_float32(ref):
    """numpy converts a double to binary16 in one rounding.  torch's CPU conversion of a double goes
    through binary32 (it rounds the traps below twice and gets them wrong), so torch is only asked
    about values that are binary32 numbers to begin with, where one rounding is all there is."""
    xs = _f16_samples()
    got = np.array([ref.round_f16(float(x)) for x in xs], np.uint16)
    with np.errstate(over="ignore"):
        want_np = xs.astype(np.float16).view(np.uint16)
    assert np.array_equal(got, want_np)
    with np.errstate(over="ignore"):
        x32 = xs.astype(np.float32)
    got32 = np.array([ref.round_f16(float(x)) for x in x32], np.uint16)
    want_t = torch.from_numpy(x32).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got32, want_t)


def test_f16_rounding_is_nearest_ties_to_even_in_exact_arithmetic(ref):
    xs = list(_f16_samples()[::23]) + F16_TRAPS
    for x in xs:
        x = float(x)
        if math.isinf(x) or abs(x) >= 65520.0:
            assert ref.round_f16(x) == (0xFC00 if x < 0 else 0x7C00)
            continue
        b = ref.round_f16(x)
        assert (b & 0x7C00) != 0x7C00                       # finite
        r = Fraction(ref.widen_f16(b))
        err = abs(Fraction(x) - r)
        mag = b & 0x7FFF
        nbs = []
        if mag < 0x7BFF:
            nbs.append(Fraction(ref.widen_f16(b + 1)))
        else:
            nbs.append(Fraction(65536) * (-1 if b & 0x8000 else 1))   # the value the next pattern would have
        nbs.append(Fraction(ref.widen_f16(b - 1)) if mag > 0 else Fraction(ref.widen_f16((b ^ 0x8000) | 1)))
        for nb in nbs:
            e2 = abs(Fraction(x) - nb)
            assert err <= e2, (x, hex(b))
            if err == e2:
                assert b % 2 == 0, (x, hex(b))              # a tie goes to the even pattern


def test_f16_pseudograd_in_the_bf16_calls(ref):
    """pg_format 1 changes the format of the outgoing pseudo-gradient and nothing else."""
    wl = synth.Workload("h", (3000, 1999, 0, 777), tau=2, H=1, budget=2)
    bk = synth.bookkeeping(wl, "mixed")
    a = _bf16_state(wl, 13, amplified=True)
    b = {k: v.copy() for k, v in a.items()}
    tg0, tm0 = a["theta_g"].copy(), a["theta_m"].copy()
    pg_a, pg_b = np.zeros(wl.n_total, np.uint16), np.zeros(wl.n_total, np.uint16)
    oa = ref.sync_step_bf16(wl.frags, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"], pg_a,
                            bk.I_p, bk.t_b, bk.t_g, 2, ref.hparams(2, 1, pg_format=0))
    ob = ref.sync_step_bf16(wl.frags, b["theta_m"], b["theta_m_send"], b["theta_g"], b["momentum"], b["delta_g"], pg_b,
                            bk.I_p, bk.t_b, bk.t_g, 2, ref.hparams(2, 1, pg_format=1))
    assert oa["rc"] == 0 and ob["rc"] == 0
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(oa["R"], ob["R"]) and oa["sel"].tolist() == ob["sel"].tolist()
    diff = tg0.astype(np.float64) - _widen(tm0).astype(np.float64)      # exact in fp64
    with np.errstate(over="ignore"):
        want = diff.astype(np.float16).view(np.uint16)
    assert np.array_equal(pg_b, want)
    assert not np.array_equal(pg_a, pg_b)
    # the single-step call
    pg_c, send = np.zeros(wl.n_total, np.uint16), np.zeros(wl.n_total, np.uint16)
    assert ref.pseudograd_bf16(wl.frags, tg0, tm0, pg_c, send, pg_format=1) == 0
    assert np.array_equal(pg_c, want) and np.array_equal(send, tm0)
    assert ref.pseudograd_bf16(wl.frags, tg0, tm0, pg_c, send, pg_format=2) < 0
    assert ref.sync_step_bf16(wl.frags, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                              pg_a, bk.I_p, bk.t_b, bk.t_g, 2, ref.hparams(2, 1, pg_format=3))["rc"] < 0


# ------------------------------------------------------------------ 16-bit parameters on strided shards, events
def _run_bf16_seg(ref, segs, K, st, hp, I_p, t_b, budget=2):
    pg = np.full(st["theta_m"].size, 0x7FC0, np.uint16)
    out = ref.sync_step_bf16_segmented(segs, K, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                       st["delta_g"], pg, I_p, t_b, 100, budget, hp)
    assert out["rc"] == 0
    return out, pg


def test_bf16_segmented_step_against_the_contiguous_and_the_fp32_segmented_steps(ref):
    """(a) one segment per fragment, and a fragment cut into adjacent pieces, are the contiguous 16-bit step
    bit for bit; (b) on strided shards (Sec. 4.1) it is the fp32 segmented step on the widened inputs with
    the local parameters and the pseudo-gradient rounded once: the two already pinned functions fix it."""
    wl = synth.Workload("b", (3000, 1999, 0, 777), tau=5, H=100, budget=2)
    bk = synth.bookkeeping(wl, "mixed")
    for pg_format in (0, 1):
        hp = ref.hparams(5, 100, pg_format=pg_format)
        a = _bf16_state(wl, 21)
        b = {k: v.copy() for k, v in a.items()}
        c = {k: v.copy() for k, v in a.items()}
        pg_a = np.full(wl.n_total, 0x7FC0, np.uint16)
        oa = ref.sync_step_bf16(wl.frags, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                                pg_a, bk.I_p, bk.t_b, 100, 2, hp)
        ob, pg_b = _run_bf16_seg(ref, [(o, l, p) for p, (o, l) in enumerate(wl.frags)], wl.K, b, hp, bk.I_p, bk.t_b)
        cut = []
        for p, (o, l) in enumerate(wl.frags):
            cut += [(o, l // 3, p), (o + l // 3, l - l // 3, p)]
        oc, pg_c = _run_bf16_seg(ref, cut, wl.K, c, hp, bk.I_p, bk.t_b)
        for other, o2, pg2 in ((b, ob, pg_b), (c, oc, pg_c)):
            for k in a:
                assert np.array_equal(a[k], other[k]), k
            assert np.array_equal(pg_a, pg2)
            assert np.array_equal(oa["R"], o2["R"]) and np.array_equal(oa["sums"], o2["sums"])
            assert oa["sel"].tolist() == o2["sel"].tolist()

        # (b) 12 layers of unequal size in K = 4 strided shards, with a gap that nobody owns
        sizes = [300, 170, 411, 96, 250, 333, 128, 77, 205, 190, 64, 501]
        offs = np.concatenate(([40], 40 + np.cumsum(sizes)[:-1]))
        segs = [(int(offs[j]), sizes[j], j % 4) for j in range(12)]
        n = 40 + sum(sizes) + 25
        wl2 = synth.Workload("b2", (n,), tau=5, H=100)
        s16 = _bf16_state(wl2, 22)
        w = {k: (v.copy() if v.dtype == np.float32 else _widen(v)) for k, v in s16.items()}
        before = {k: v.copy() for k, v in s16.items()}
        I_p, t_b = [3, 5, 2, 7], [90, 95, 97, 60]
        o16, pg16 = _run_bf16_seg(ref, segs, 4, s16, hp, I_p, t_b)
        pg32 = np.zeros(n, np.float32)
        o32 = ref.sync_step_segmented(segs, 4, w["theta_m"], w["theta_m_send"], w["theta_g"], w["momentum"],
                                      w["delta_g"], pg32, I_p, t_b, 100, 2, hp, shadow=True)
        assert o32["rc"] == 0
        assert np.array_equal(s16["theta_g"], w["theta_g"]) and np.array_equal(s16["momentum"], w["momentum"])
        assert np.array_equal(o16["R"], o32["R"]) and np.array_equal(o16["sums"], o32["sums"])
        assert o16["sel"].tolist() == o32["sel"].tolist()
        rnd = ref.round_f16 if pg_format else ref.round_bf16
        owned = np.zeros(n, bool)
        for o, l, _ in segs:
            owned[o:o + l] = True
        want_tm = np.array([ref.round_bf16(v) for v in o32["theta_m64"]], dtype=np.uint16)
        assert np.array_equal(s16["theta_m"][owned], want_tm[owned])
        diff = before["theta_g"].astype(np.float64) - _widen(before["theta_m"]).astype(np.float64)
        want_pg = np.array([rnd(v) for v in diff], dtype=np.uint16)
        assert np.array_equal(pg16[owned], want_pg[owned])
        # what no shard owns is left alone
        assert np.array_equal(s16["theta_m"][~owned], before["theta_m"][~owned])
        assert (pg16[~owned] == 0x7FC0).all()
        for k in ("theta_g", "momentum", "delta_g", "theta_m_send"):
            assert np.array_equal(s16[k][~owned], before[k][~owned])


@pytest.mark.parametrize("mask", [(1, 1, 1, 1, 1), (0, 1, 0, 2, 1), (0, 0, 0, 0, 0), (1, 2, 2, 0, 2), (3, 0, 1, 0, 0)])
def test_bf16_event_is_the_bf16_step_on_the_arrived_fragments_then_selection(ref, mask):
    """The 16-bit event == the 16-bit step restricted to the arrived fragments (everything else untouched),
    then Alg. 2 over old and new scores with the fragments in flight struck out of the priority order."""
    frags = [(3, 700), (703, 0), (710, 1), (800, 4100), (5000, 333)]
    K, n = len(frags), 5400
    wl = synth.Workload("e", (n,), tau=2, H=3)
    hp = ref.hparams(2, 3, lam=0.5, pg_format=1)
    I_p = [4, 9, 2, 6, 3]
    t_b = [90, 99, 40, 95, 97]
    R_old = np.array([0.25, np.inf, 7.0, 0.5, 0.125])
    a = _bf16_state(wl, 31, amplified=True)
    b = {k: v.copy() for k, v in a.items()}
    orig = {k: v.copy() for k, v in a.items()}
    pg_a = np.full(n, 0x7E00, np.uint16)
    pg_b = pg_a.copy()
    sums_a = np.full((K, 4), -3.0)
    R_a = R_old.copy()
    out = ref.sync_event_bf16(frags, mask, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"],
                              pg_a, I_p, t_b, 100, 2, hp, R_a, sums=sums_a)
    assert out["rc"] == 0
    arrived = [q for q in range(K) if mask[q] & 1]
    R_b = R_old.copy()
    sums_b = np.full((K, 4), -3.0)
    if arrived:
        sub = ref.sync_step_bf16([frags[q] for q in arrived], b["theta_m"], b["theta_m_send"], b["theta_g"],
                                 b["momentum"], b["delta_g"], pg_b, [I_p[q] for q in arrived],
                                 [t_b[q] for q in arrived], 100, 0, hp)
        assert sub["rc"] == 0
        for j, q in enumerate(arrived):
            R_b[q] = sub["R"][j]
            sums_b[q] = sub["sums"][j]
    rc, order = ref.select_fragments(R_b, t_b, 100, hp.H, K)
    assert rc == 0
    want = [q for q in order.tolist() if not mask[q] & 2][:2]
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(pg_a, pg_b)
    assert np.array_equal(R_a, R_b) and np.array_equal(sums_a, sums_b)
    assert out["sel"].tolist() == want
    if arrived:
        assert not np.array_equal(a["theta_m"], orig["theta_m"])
    else:
        for k in a:
            assert np.array_equal(a[k], orig[k])
    assert ref.sync_event_bf16(frags, [4, 0, 0, 0, 0], a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"],
                               a["delta_g"], pg_a, I_p, t_b, 100, 2, hp, R_a)["rc"] < 0


@pytest.mark.parametrize("mask", [(1, 1, 1, 1), (0, 1, 2, 1), (0, 0, 0, 0), (3, 2, 0, 1)])
def test_bf16_segmented_event_is_the_bf16_segmented_step_on_the_arrived_shards_then_selection(ref, mask):
    """The 16-bit event on strided shards == the (pinned) 16-bit segmented step on the arrived shards alone, then
    Alg. 2 with the shards in flight struck out; with one segment per fragment it is the contiguous 16-bit event."""
    sizes = [300, 170, 411, 96, 250, 333, 128, 77, 205, 190, 64, 501]
    offs = np.concatenate(([7], 7 + np.cumsum(sizes)[:-1]))
    segs = [(int(offs[j]), sizes[j], j % 4) for j in range(12)]
    K, n = 4, 7 + sum(sizes) + 9
    wl = synth.Workload("e", (n,), tau=2, H=3)
    hp = ref.hparams(2, 3, lam=0.5, pg_format=1)
    I_p, t_b = [4, 9, 2, 6], [90, 99, 40, 97]
    R_old = np.array([0.25, np.inf, 7.0, 0.5])
    a = _bf16_state(wl, 51, amplified=True)
    b = {k: v.copy() for k, v in a.items()}
    pg_a = np.full(n, 0x7E00, np.uint16)
    pg_b = pg_a.copy()
    sums_a, R_a = np.full((K, 4), -3.0), R_old.copy()
    out = ref.sync_event_bf16_segmented(segs, K, mask, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"],
                                        a["delta_g"], pg_a, I_p, t_b, 100, 2, hp, R_a, sums=sums_a)
    assert out["rc"] == 0
    arrived = [q for q in range(K) if mask[q] & 1]
    R_b, sums_b = R_old.copy(), np.full((K, 4), -3.0)
    if arrived:
        sub = [(o, l, arrived.index(f)) for o, l, f in segs if f in arrived]
        so = ref.sync_step_bf16_segmented(sub, len(arrived), b["theta_m"], b["theta_m_send"], b["theta_g"], b["momentum"],
                                          b["delta_g"], pg_b, [I_p[q] for q in arrived], [t_b[q] for q in arrived],
                                          100, 0, hp)
        assert so["rc"] == 0
        for j, q in enumerate(arrived):
            R_b[q], sums_b[q] = so["R"][j], so["sums"][j]
    rc, order = ref.select_fragments(R_b, t_b, 100, hp.H, K)
    assert rc == 0
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(pg_a, pg_b) and np.array_equal(R_a, R_b) and np.array_equal(sums_a, sums_b)
    assert out["sel"].tolist() == [q for q in order.tolist() if not mask[q] & 2][:2]
    frags = [(5, 700), (705, 0), (710, 1), (800, 900)]
    c = _bf16_state(wl, 52)
    d = {k: v.copy() for k, v in c.items()}
    R_c, R_d = R_old.copy(), R_old.copy()
    pg_c, pg_d = np.zeros(n, np.uint16), np.zeros(n, np.uint16)
    oc = ref.sync_event_bf16(frags, mask, c["theta_m"], c["theta_m_send"], c["theta_g"], c["momentum"], c["delta_g"],
                             pg_c, I_p, t_b, 100, 3, hp, R_c)
    od = ref.sync_event_bf16_segmented([(o, l, p) for p, (o, l) in enumerate(frags)], K, mask, d["theta_m"],
                                       d["theta_m_send"], d["theta_g"], d["momentum"], d["delta_g"], pg_d, I_p, t_b,
                                       100, 3, hp, R_d)
    assert oc["rc"] == 0 and od["rc"] == 0 and oc["sel"].tolist() == od["sel"].tolist()
    for k in c:
        assert np.array_equal(c[k], d[k]), k
    assert np.array_equal(pg_c, pg_d) and np.array_equal(R_c, R_d)
