"""Pins of the oracle's bf16 variant (local parameters kept in bfloat16, Sec. 4.1): the
rounding primitive against torch's float32 -> bfloat16 conversion and against exact rational
arithmetic, and the bf16 fused step against the pinned fp32 step on the widened inputs.
CPU only."""
import math
from fractions import Fraction

import numpy as np
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
