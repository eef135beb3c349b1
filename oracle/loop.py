"""CPU definition of the adaptive-transmission loop of the paper's Sec. 3.2 around the oracle's
single steps.  TEST INFRASTRUCTURE ONLY (see oracle/cocodc_ref.h).

One worker, inner steps t = 1, 2, ...; all buffers are host numpy arrays.  Per step, after the
worker's local update:
  1. every fragment whose all-reduce was launched tau (or more) steps ago completes: the fused
     oracle step on that fragment alone, with I_p = t_p - t_{p,b} (Eq. 11), taken as 1 when it
     would be 0; then t_{p,b} <- t (Sec. 3.2 defines t_{p,b} as the step at which the
     fragment's previous synchronisation completed);
  2. every h steps (Eq. 10; h = floor(H/N), at least 1, N from Eq. 9) the next fragment is
     chosen by Algorithm 2 with t_g = t among the fragments that are not in flight; its
     pseudo-gradient is written to the send buffer and its parameters are recorded.
All t_{p,b} start at 0 and all R_p at +infinity (never-synchronised fragments go first).
Readings where the paper is silent: a fragment in flight is not eligible; h = 0 is taken as 1;
receives happen before the send decision of the same step, in ascending fragment index.
When a fragment is sent again at the very step its previous synchronisation completed (possible
when a decision step coincides with an arrival), Eq. 11 as printed has I_p = t_p - t_{p,b} = 0.
Sec. 3.2 keeps R_p = infinity for fragments that have not yet completed a synchronisation, so a
fragment that has completed one must get a finite score: the interval is taken as one step.

Fragments may be strided shards (Sec. 4.1: shard k = layers k, k + K, ... of a layer-ordered buffer):
pass segs = [(offset, length, fragment), ...] and K instead of frags.  A shard's pieces are walked in
the order listed; everything else is the same loop.

half=True: the local parameters, their send-time record and the send buffer hold 16-bit patterns
(uint16 arrays: bf16 parameters as in the mixed-precision training of Sec. 4.1, pseudo-gradient in
hp.pg_format); the loop is the same, built on the 16-bit single steps.
"""
import numpy as np

from . import (pseudograd, pseudograd_bf16, select_fragments, sync_plan, sync_step, sync_step_bf16,
               sync_step_bf16_segmented, sync_step_segmented)


class RefLoop:
    # The interval of Eq. 11 never counts as less than this many steps (see the module text).
    min_interval = 1

    def __init__(self, frags, hp, gamma, T_c, T_s, segs=None, K=None, half=False):
        self.half = bool(half)
        if segs is None:
            self.frags = [(int(o), int(l)) for o, l in frags]
            self.K = len(self.frags)
            self.pieces = None
        else:
            assert frags is None and K is not None
            self.frags = None
            self.K = int(K)
            self.pieces = [[(int(o), int(l)) for o, l, f in segs if int(f) == p] for p in range(self.K)]
        self.hp = hp
        self.gamma, self.T_c, self.T_s = float(gamma), float(T_c), float(T_s)
        self.t_b = [0] * self.K
        self.I_p = [0] * self.K
        self.in_flight = [-1] * self.K
        self.R = np.full(self.K, np.inf)
        self._replan()

    def _replan(self):
        rc, N, h = sync_plan(self.K, self.hp.H, self.gamma, self.T_c, self.T_s)
        assert rc == 0
        self.N, self.h = N, max(1, h)

    def observe(self, T_c_sample, T_s_sample, beta):
        self.T_c = (1.0 - beta) * self.T_c + beta * T_c_sample
        self.T_s = (1.0 - beta) * self.T_s + beta * T_s_sample
        self._replan()

    def due(self, t):
        return [p for p in range(self.K) if self.in_flight[p] >= 0 and self.in_flight[p] + self.hp.tau <= t]

    def step(self, t, theta_m, theta_m_send, theta_g, momentum, delta_g, delta_m_out):
        received = []
        for p in self.due(t):
            I = max(self.min_interval, self.in_flight[p] - self.t_b[p])
            one, many = (sync_step_bf16, sync_step_bf16_segmented) if self.half else (sync_step, sync_step_segmented)
            if self.pieces is None:
                out = one([self.frags[p]], theta_m, theta_m_send, theta_g, momentum, delta_g, None,
                          [I], [self.t_b[p]], t, 0, self.hp)
            else:   # the shard alone, as the one fragment of a segmented step
                out = many([(o, l, 0) for o, l in self.pieces[p]], 1, theta_m, theta_m_send, theta_g,
                           momentum, delta_g, None, [I], [self.t_b[p]], t, 0, self.hp)
            assert out["rc"] == 0
            self.R[p] = out["R"][0]
            self.I_p[p] = I
            self.t_b[p] = t
            self.in_flight[p] = -1
            received.append(p)
        sent = -1
        if t % self.h == 0:
            rc, order = select_fragments(self.R, self.t_b, t, self.hp.H, self.K)
            assert rc == 0
            for q in order.tolist():
                if self.in_flight[q] < 0:
                    sent = q
                    break
            if sent >= 0:
                where = [self.frags[sent]] if self.pieces is None else self.pieces[sent]
                if where and self.half:
                    assert pseudograd_bf16(where, theta_g, theta_m, delta_m_out, theta_m_send, self.hp.pg_format) == 0
                elif where:
                    assert pseudograd(where, theta_g, theta_m, delta_m_out, theta_m_send) == 0
                self.in_flight[sent] = t
        return received, sent
