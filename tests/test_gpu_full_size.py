"""Full-size parity of the fused step on the 1.3B and 7B fragment sets, in the buffer layout
and launch configuration that bench.py times.

The CPU oracle cannot sweep 6.6e9 parameters in a test, so:
  * three whole fragments (the large fragment 0, a middle one, the last one) go through the
    oracle element by element, with the same bar as the small tests;
  * every fragment's score is compared with torch.linalg.vector_norm in fp64 (a library
    routine) and the selection with the oracle's Algorithm 2 run on those scores;
  * every 61st element of every buffer is compared with the update written out in torch
    fp64 operations (not the oracle: a property check that no region of the buffers was
    skipped or written twice);
  * the inputs the step must not modify are checksummed before and after.
"""
import numpy as np
import pytest
import torch

from paper_2504_17672_amd import synth

import parity_util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_2504_17672_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return binding


def _torch_expected(x, wl):
    """The update of one element written with torch fp64 operations."""
    tm, ts, tg, m, dg = (x[k].double() for k in ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g"))
    m1 = wl.mu * m + dg
    G = (tg - wl.eta * (dg + wl.mu * m1)).float()
    d = ts - tm
    Gd = G.double()
    tm1 = Gd + d + wl.lam * d * d * (Gd - ts) / (wl.tau * wl.H)
    return dict(theta_m=tm1.float(), theta_g=G, momentum=m1.float(), pg=(x["theta_g"] - x["theta_m"]))


def _checksum(t):
    return t.view(torch.int32).sum(dtype=torch.int64).item()


@pytest.mark.parametrize("name,sample_frags", [("1.3B", (0, 11, 23)), ("7B", (0, 13, 31))])
def test_full_size_sampled(B, ref, name, sample_frags):
    wl = synth.WORKLOADS[name]
    n, K = wl.n_total, wl.K
    torch.cuda.empty_cache()
    free, _ = torch.cuda.mem_get_info()
    # what bench.py does by default, leaving a fifth of the memory for this test's own temporaries
    arena, carved, stride, _ = B.tuned_spaced_buffers(n, wl.frags, "cuda", max_arena_bytes=int(free * 0.8))
    print(f"case {name} full size K={K} n={n} layout=tuned stride={stride / 2**30:.0f} GiB", flush=True)
    names = ("theta_m", "theta_m_send", "theta_g", "momentum", "delta_g", "pg")
    bufs = dict(zip(names, carved))
    st = synth.make_state(wl, "cuda", seed=0, buffers=bufs)
    pg = bufs["pg"]
    pg.fill_(555.0)
    bk = synth.bookkeeping(wl)
    ghp, rhp = B.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu), ref.hparams(wl.tau, wl.H, wl.lam, wl.eta, wl.mu)
    ws = B.new_workspace(K, n)

    n_rounds = 2 if wl.n_syncs > 1 else 1
    for rnd in range(n_rounds):
        if rnd > 0:
            synth.next_sync_inputs(wl, st, 0, rnd)
        print(f"   sync {rnd + 1}: staging samples", flush=True)
        host = {p: U.host_copy(st, *(wl.frags[p][0], wl.frags[p][0] + wl.frags[p][1])) for p in sample_frags}
        idx = torch.arange(0, n, 61, device="cuda")
        want = _torch_expected({k: st[k][idx] for k in st}, wl)
        norms = [torch.linalg.vector_norm(st["delta_g"][o:o + l], ord=2, dtype=torch.float64).item()
                 for o, l in wl.frags]
        before = {k: _checksum(st[k]) for k in ("theta_m_send", "delta_g")}

        out = U.gpu_outputs(K)
        rc = B.cocodc_sync_step(wl.frags, n, st["theta_m"], st["theta_m_send"], st["theta_g"], st["momentum"],
                                st["delta_g"], pg, bk.I_p, bk.t_b, bk.t_g, wl.budget, ghp, out["R"], out["sel"],
                                out["n_sel"], out["sums"], ws)
        assert rc == 0
        torch.cuda.synchronize()
        print("   GPU step done; checking", flush=True)

        # inputs untouched
        for k, v in before.items():
            assert _checksum(st[k]) == v, k
        # every 61st element against the torch fp64 formula
        got = dict(theta_m=st["theta_m"][idx], theta_g=st["theta_g"][idx], momentum=st["momentum"][idx], pg=pg[idx])
        assert torch.equal(got["pg"], want["pg"])
        for k in ("theta_m", "theta_g", "momentum"):
            assert torch.allclose(got[k], want[k], rtol=1e-5, atol=1e-9), k
            frac_equal = (got[k] == want[k]).double().mean().item()
            assert frac_equal > 0.999, (k, frac_equal)
        # every fragment's score against the library norm; selection from those scores
        Rg = out["R"].cpu().numpy()
        Rt = np.array([nv / i for nv, i in zip(norms, bk.I_p)])
        assert U.rel_err(Rg, Rt) <= 1e-9
        rc, want_sel = ref.select_fragments(Rg, bk.t_b, bk.t_g, wl.H, wl.budget)
        n_sel = int(out["n_sel"].item())
        assert n_sel == min(wl.budget, K)
        sel = out["sel"][:n_sel].cpu().tolist()
        assert sel == want_sel.tolist()
        # whole fragments through the oracle
        for p in sample_frags:
            off, ln = wl.frags[p]
            h = host[p]
            one = synth.Bookkeeping(t_g=bk.t_g, t_b=[bk.t_b[p]], I_p=[bk.I_p[p]])
            ro = U.run_ref_fused(ref, [(0, ln)], h, one, 1, rhp)
            gstate = {k: st[k][off:off + ln] for k in ("theta_m", "theta_g", "momentum")}
            gout = dict(pg=pg[off:off + ln], R=out["R"][p:p + 1], sums=out["sums"][p:p + 1])
            obs = U.compare_fused(gstate, gout, h, ro, [(0, ln)])
            print(f"   fragment {p} ({ln} params) observed",
                  {a: (f"{b:.3g}" if isinstance(b, float) else b) for a, b in obs.items()}, flush=True)
            del ro, h
        host.clear()
        bk = synth.advance_bookkeeping(wl, bk, sel)
