"""Pins of the oracle's segmented (strided-shard, Sec. 4.1) functions: they must reduce to the
contiguous ones where a fragment is one piece, must not care how a contiguous run is cut into
adjacent pieces, and must agree with library norms over the concatenated pieces.  CPU only."""
import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth


def _state(n, seed, amplified=False):
    wl = synth.Workload("s", (n,), tau=5, H=100)
    return {k: v.numpy() for k, v in synth.make_state(wl, "cpu", seed=seed, amplified=amplified).items()}


def _run(ref, fn, table, K, st, hp, I_p, t_b, budget=2, **kw):
    a = {k: v.copy() for k, v in st.items()}
    pg = np.full(a["theta_m"].size, 555.0, np.float32)
    if fn == "seg":
        out = ref.sync_step_segmented(table, K, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"],
                                      a["delta_g"], pg, I_p, t_b, 1000, budget, hp, **kw)
    else:
        out = ref.sync_step(table, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"], a["delta_g"], pg,
                            I_p, t_b, 1000, budget, hp, **kw)
    assert out["rc"] == 0
    return a, pg, out


def test_one_segment_per_fragment_is_the_contiguous_step(ref):
    st = _state(5000, 1)
    frags = [(0, 1000), (1500, 2001), (3600, 1400)]
    segs = [(o, l, p) for p, (o, l) in enumerate(frags)]
    hp = ref.hparams(5, 100)
    a, pga, oa = _run(ref, "frag", frags, 3, st, hp, [3, 5, 7], [990, 990, 990])
    b, pgb, ob = _run(ref, "seg", segs, 3, st, hp, [3, 5, 7], [990, 990, 990])
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(pga, pgb) and np.array_equal(oa["R"], ob["R"]) and np.array_equal(oa["sums"], ob["sums"])
    assert oa["sel"].tolist() == ob["sel"].tolist()


def test_cutting_a_run_into_adjacent_pieces_changes_nothing(ref):
    st = _state(6000, 2, amplified=True)
    frags = [(0, 2500), (2500, 3500)]
    segs = [(0, 1, 0), (1, 999, 0), (1000, 0, 0), (1000, 1500, 0), (2500, 3, 1), (2503, 3000, 1), (5503, 497, 1)]
    hp = ref.hparams(2, 1)
    a, pga, oa = _run(ref, "frag", frags, 2, st, hp, [3, 5], [990, 990])
    b, pgb, ob = _run(ref, "seg", segs, 2, st, hp, [3, 5], [990, 990])
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(oa["sums"], ob["sums"]) and np.array_equal(oa["R"], ob["R"])


def test_strided_shards_score_the_union_of_their_layers(ref):
    segs, n = synth.strided_segments(12, 16, 40, 4)
    assert len(segs) == 13 and {f for _, _, f in segs} == {0, 1, 2, 3}
    assert [f for _, _, f in segs[1:]] == [0, 1, 2, 3] * 3  # layer l belongs to shard l mod 4
    st = _state(n, 3)
    I_p = [2, 3, 5, 7]
    for kind in (2, 1):
        rc, R, S = ref.fragment_scores_segmented(segs, 4, st["delta_g"], I_p, kind)
        assert rc == 0
        for p in range(4):
            cat = torch.cat([torch.from_numpy(st["delta_g"][o:o + l]) for o, l, f in segs if f == p])
            norm = torch.linalg.vector_norm(cat, ord=kind, dtype=torch.float64).item()
            assert abs(R[p] * I_p[p] - norm) <= 1e-12 * norm
    hp = ref.hparams(5, 100)
    b, pg, ob = _run(ref, "seg", segs, 4, st, hp, I_p, [990] * 4, shadow=True)
    rc, R, S = ref.fragment_scores_segmented(segs, 4, st["delta_g"], I_p, 2)
    assert np.array_equal(ob["R"], R) and np.array_equal(ob["sums"][:, 0], S)
    # element-wise results do not depend on the grouping: same as one contiguous fragment
    a, pga, oa = _run(ref, "frag", [(0, n)], 1, st, hp, [1], [990], budget=1)
    for k in a:
        assert np.array_equal(a[k], b[k])
    assert np.array_equal(pg, pga)


def test_listing_order_only_reorders_the_sum(ref):
    st = _state(4000, 4)
    segs = [(0, 1000, 0), (1000, 1000, 1), (2000, 1000, 0), (3000, 1000, 1)]
    swapped = [segs[2], segs[1], segs[0], segs[3]]
    rc, R1, S1 = ref.fragment_scores_segmented(segs, 2, st["delta_g"], [1, 1], 2)
    rc, R2, S2 = ref.fragment_scores_segmented(swapped, 2, st["delta_g"], [1, 1], 2)
    assert abs(S1[0] - S2[0]) <= 1e-13 * S1[0] and S1[1] == S2[1]


def test_untouched_elements_empty_fragments_and_errors(ref):
    st = _state(3000, 5)
    segs = [(10, 500, 2), (700, 300, 0)]  # fragment 1 has no segment
    hp = ref.hparams(5, 100)
    b, pg, ob = _run(ref, "seg", segs, 3, st, hp, [1, 1, 0], [990] * 3, budget=3)
    mask = np.zeros(3000, bool)
    mask[10:510] = True
    mask[700:1000] = True
    for k in st:
        assert np.array_equal(b[k][~mask], st[k][~mask])
    assert np.all(pg[~mask] == 555.0)
    assert ob["R"][1] == 0.0 and np.isposinf(ob["R"][2]) and ob["sums"][1].tolist() == [0, 0, 0, 0]
    assert ob["sel"].tolist() == [2, 0, 1]
    x = st["delta_g"]
    assert ref.fragment_scores_segmented([(0, 10, 0), (5, 10, 1)], 2, x, [1, 1])[0] == -3  # overlap
    assert ref.fragment_scores_segmented([(0, 10, 2)], 2, x, [1, 1])[0] == -3            # fragment id
    assert ref.fragment_scores_segmented([(2995, 10, 0)], 1, x, [1])[0] == -3            # out of range


# ------------------------------------------------------------------ one loop event on strided shards
@pytest.mark.parametrize("mask", [(1, 1, 1, 1), (0, 1, 2, 1), (0, 0, 0, 0), (3, 2, 0, 1), (2, 2, 2, 2)])
def test_segmented_event_is_the_segmented_step_on_the_arrived_shards_then_selection(ref, mask):
    """The event on strided shards == the (pinned) segmented step on the arrived shards alone, everything else
    untouched, then Alg. 2 over old and new scores with the shards in flight struck out; and with one segment
    per fragment it is the contiguous event bit for bit."""
    sizes = [300, 170, 411, 96, 250, 333, 128, 77, 205, 190, 64, 501]
    offs = np.concatenate(([7], 7 + np.cumsum(sizes)[:-1]))
    segs = [(int(offs[j]), sizes[j], j % 4) for j in range(12)]
    K, n = 4, 7 + sum(sizes) + 9
    hp = ref.hparams(2, 3, lam=0.5)
    I_p, t_b = [4, 9, 2, 6], [90, 99, 40, 97]
    R_old = np.array([0.25, np.inf, 7.0, 0.5])
    a = _state(n, 41, amplified=True)
    b = {k: v.copy() for k, v in a.items()}
    orig = {k: v.copy() for k, v in a.items()}
    pg_a = np.full(n, 555.0, np.float32)
    pg_b = pg_a.copy()
    sums_a = np.full((K, 4), -3.0)
    R_a = R_old.copy()
    out = ref.sync_event_segmented(segs, K, mask, a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"],
                                   a["delta_g"], pg_a, I_p, t_b, 100, 2, hp, R_a, sums=sums_a)
    assert out["rc"] == 0
    arrived = [q for q in range(K) if mask[q] & 1]
    R_b, sums_b = R_old.copy(), np.full((K, 4), -3.0)
    if arrived:
        sub = [(o, l, arrived.index(f)) for o, l, f in segs if f in arrived]
        so = ref.sync_step_segmented(sub, len(arrived), b["theta_m"], b["theta_m_send"], b["theta_g"], b["momentum"],
                                     b["delta_g"], pg_b, [I_p[q] for q in arrived], [t_b[q] for q in arrived], 100, 0, hp)
        assert so["rc"] == 0
        for j, q in enumerate(arrived):
            R_b[q], sums_b[q] = so["R"][j], so["sums"][j]
    rc, order = ref.select_fragments(R_b, t_b, 100, hp.H, K)
    assert rc == 0
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert np.array_equal(pg_a, pg_b)
    assert np.array_equal(R_a, R_b) and np.array_equal(sums_a, sums_b)
    assert out["sel"].tolist() == [q for q in order.tolist() if not mask[q] & 2][:2]
    if not arrived:
        for k in a:
            assert np.array_equal(a[k], orig[k])
    # one segment per fragment: the contiguous event
    frags = [(5, 700), (705, 0), (710, 1), (800, 900)]
    c = _state(n, 42)
    d = {k: v.copy() for k, v in c.items()}
    R_c, R_d = R_old.copy(), R_old.copy()
    pg_c, pg_d = np.zeros(n, np.float32), np.zeros(n, np.float32)
    oc = ref.sync_event(frags, mask, c["theta_m"], c["theta_m_send"], c["theta_g"], c["momentum"], c["delta_g"], pg_c,
                        I_p, t_b, 100, 3, hp, R_c)
    od = ref.sync_event_segmented([(o, l, p) for p, (o, l) in enumerate(frags)], K, mask, d["theta_m"],
                                  d["theta_m_send"], d["theta_g"], d["momentum"], d["delta_g"], pg_d, I_p, t_b, 100, 3,
                                  hp, R_d)
    assert oc["rc"] == 0 and od["rc"] == 0 and oc["sel"].tolist() == od["sel"].tolist()
    for k in c:
        assert np.array_equal(c[k], d[k]), k
    assert np.array_equal(pg_c, pg_d) and np.array_equal(R_c, R_d)
    assert ref.sync_event_segmented(segs, K, [4, 0, 0, 0], a["theta_m"], a["theta_m_send"], a["theta_g"], a["momentum"],
                                    a["delta_g"], pg_a, I_p, t_b, 100, 2, hp, R_a)["rc"] < 0
