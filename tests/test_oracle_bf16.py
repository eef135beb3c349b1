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
