"""Two-stream schedule of one CO2 worker on one GPU.

CO2 (Algorithm 1; Section 3.1 and Fig. 1) lets the all-reduce launched after
round t and the outer update that consumes the previous one run beside the next
round's local steps.  On one GPU the all-reduce's result is K device buffers, and
what can legally overlap follows from the data flow of Algorithm 1: m_t and
x_{t+1,0} depend only on x_{t,0}, m_{t-1} and round t-1's pseudo-gradients, all
of which exist when round t's inner loop STARTS (that is the one-round
staleness).  So during round t

  main stream : tau fused AdamW steps on the local parameters; the first reads
                its input from the anchor x_{t,0} and leaves ||x_{t,1}-x_{t,0}||_s
                (next round's Eq. 3 denominator), the last also forms this
                round's pseudo-gradient x_{t,0} - x_{t,tau};
  side stream : co2_outer_step in split form (params = NULL): Lambda_t, m_t and
                the next anchor x_{t+1,0} into a second anchor buffer;

and at the round boundary each stream waits on the other's event.  The fused
form of co2_outer_step cannot run beside the inner loop, because it writes the
parameters the next local step reads.

This module only sequences launches, streams and events; all arithmetic is in
the kernels of libco2.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List

import torch

from . import binding as co2


@dataclass
class AdamWConfig:
    lr: float = 3e-4
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.1


class CO2Worker:
    """State of one worker and the per-round schedule (overlapped or serial).

    Buffers (all flat fp32 of n elements unless noted):
      params, exp_avg, exp_avg_sq  -- local parameters and AdamW moments
      anchor[2]                    -- x_{t,0} / x_{t+1,0}, ping-pong
      momentum                     -- outer momentum m
      own[2]                       -- this worker's pseudo-gradient of the previous /
                                      current round, ping-pong
      peers[K-1]                   -- the other workers' pseudo-gradients (arrive
                                      through the all-reduce; filled by the caller)
      step_sq[2] (fp64[S]), fsn[2] (fp32[S]) -- first-inner-step norms, ping-pong
    """

    def __init__(self, table: co2.SegmentTable, K: int, tau: int, alpha: float, beta: float,
                 clip_phi: float, penalty_c: float, adamw: AdamWConfig, device,
                 params_init: torch.Tensor, buffer_set: bool = False, extra_bytes=()):
        """buffer_set: take all flat buffers from ONE co2.BufferSet (the layout the sweep and
        the AdamW step run fastest on) instead of separate allocations; `extra_bytes` then
        asks for further buffers in the same set for the caller (e.g. its gradient buffers),
        handed back as uint8 views in `self.extra`."""
        self.table, self.K, self.tau = table, K, tau
        self.alpha, self.beta, self.phi, self.c = alpha, beta, clip_phi, penalty_c
        self.hp = adamw
        n, S = table.n, table.S
        self.n, self.S = n, S
        f32 = dict(dtype=torch.float32, device=device)
        self.extra, self._set = [], None
        if buffer_set:
            count = 8 + (K - 1)
            self._set = co2.BufferSet([4 * n] * count + [int(b) for b in extra_bytes], 0, device)
            flat = [v.view(torch.float32) for v in self._set.views[:count]]
            self.extra = list(self._set.views[count:])
            for t in flat[1:3] + flat[5:]:
                t.zero_()
            self.params, self.exp_avg, self.exp_avg_sq = flat[0], flat[1], flat[2]
            self.anchor = [flat[3], flat[4]]
            self.momentum = flat[5]                                # m_0 = 0
            self.own = [flat[6], flat[7]]
            self.peers = flat[8:]
            self.params.copy_(params_init)
            self.anchor[0].copy_(params_init)
        else:
            self.params = params_init.clone()
            self.exp_avg = torch.zeros(n, **f32)
            self.exp_avg_sq = torch.zeros(n, **f32)
            self.anchor = [params_init.clone(), torch.empty(n, **f32)]
            self.momentum = torch.zeros(n, **f32)                      # m_0 = 0
            self.own = [torch.zeros(n, **f32), torch.zeros(n, **f32)]
            self.peers = [torch.zeros(n, **f32) for _ in range(K - 1)]
        self.step_sq = [torch.zeros(S, dtype=torch.float64, device=device) for _ in range(2)]
        self.fsn = [torch.zeros(S, **f32) for _ in range(2)]
        self.lam = torch.ones(S, **f32)
        wsb = co2.workspace_bytes(n, S, K)
        self.ws_main = torch.empty(wsb, dtype=torch.uint8, device=device)
        self.ws_side = torch.empty(wsb, dtype=torch.uint8, device=device)
        self.main = torch.cuda.current_stream(device)
        self.side = torch.cuda.Stream(device=device)               # default priority
        self.ev_main = torch.cuda.Event()
        self.ev_side = torch.cuda.Event()
        self.t = 0            # outer round index
        self.adam_k = 0       # AdamW step count (bias correction)
        # Resident-wavefront cap of the side-stream sweep while it shares the GPU with
        # the AdamW steps (co2_params.sweep_waves_per_cu; 0 = the sweep's stand-alone default)
        self.side_waves = 0
        # Optional stand-in for what produces the gradient of a local step (forward and
        # backward pass): called as inner_compute(k) before local step k, on the main stream.
        self.inner_compute = None
        # The last local step of a round forms the pseudo-gradient x_{t,0} - x_{t,tau}; x_{t,tau}
        # itself is read by nothing afterwards (the next round's first step starts from the new
        # anchor).  With this set the last step does not store it (4 bytes per parameter less);
        # `params` then holds x_{t,tau-1} after a round (x_{t,0} itself is anchor[t % 2] if tau = 1).
        self.skip_last_param_store = False

    def close(self):
        """Frees a buffer set taken at construction (all work on the buffers has completed)."""
        if self._set is not None:
            for name in ("params", "exp_avg", "exp_avg_sq", "anchor", "momentum", "own", "peers", "extra"):
                setattr(self, name, None)
            self._set.close()
            self._set = None

    # ------------------------------------------------------------------ pieces
    def _inner_loop(self, grads: List[torch.Tensor], stream):
        """tau local steps of round t on `stream`."""
        t, hp = self.t, self.hp
        a_cur = self.anchor[t % 2]
        for k in range(self.tau):
            self.adam_k += 1
            first, last = k == 0, k == self.tau - 1
            if self.inner_compute is not None:
                self.inner_compute(k)
            co2.co2_inner_adamw(
                self.n, a_cur if first else self.params,
                None if (last and self.skip_last_param_store) else self.params, grads[k], self.exp_avg,
                self.exp_avg_sq, hp.lr, hp.beta1, hp.beta2, hp.eps, hp.weight_decay, self.adam_k,
                anchor=a_cur if last else None, delta_out=self.own[t % 2] if last else None,
                table=self.table if first else None,
                step_sq_out=self.step_sq[t % 2] if first else None,
                workspace=self.ws_main if first else None, stream=stream)
            if first:
                co2.co2_sqrt_to_f32(self.step_sq[t % 2], self.fsn[t % 2], self.S, stream=stream)

    def _outer_update(self, stream, carried: bool):
        """Lambda_t, m_t and x_{t+1,0} (split form) on `stream`."""
        t = self.t
        flags = co2.CO2_FLAG_CARRIED_NORMS if (carried and t >= 1) else 0
        p = co2.make_params(self.table, self.K, self.alpha, self.beta, self.phi, self.c, self.tau,
                            t, flags, sweep_waves_per_cu=self.side_waves if stream is self.side else 0)
        deltas = [self.own[(t - 1) % 2]] + self.peers          # round t-1's pseudo-gradients
        co2.co2_outer_step(p, None, self.anchor[t % 2], self.anchor[(t + 1) % 2], self.momentum,
                           deltas, None, self.fsn[(t - 1) % 2] if t >= 1 else None, self.lam,
                           self.ws_side, stream=stream)

    # ------------------------------------------------------------------ rounds
    def round_overlapped(self, grads: List[torch.Tensor], carried: bool = True):
        """Round t with the outer update on the side stream beside the inner loop."""
        # the side stream needs the previous round's pseudo-gradient and step norms
        self.ev_main.record(self.main)
        self.side.wait_event(self.ev_main)
        self._outer_update(self.side, carried)
        self.ev_side.record(self.side)
        self._inner_loop(grads, self.main)
        # boundary: the next round starts from the anchor the side stream wrote
        self.main.wait_event(self.ev_side)
        self.t += 1

    def round_serial(self, grads: List[torch.Tensor], carried: bool = True):
        """The same round with every launch on the main stream, inner loop first."""
        self._inner_loop(grads, self.main)
        self._outer_update(self.main, carried)
        self.t += 1
