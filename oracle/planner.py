"""CPU model of the budget-aware residency planner: TEST INFRASTRUCTURE, not a product path.

Only tests/ may import this module.  It follows Sec. 4.3 ("Budget-Aware Residency Planner")
and Alg. 2 of the paper in the paper's notation:

  tau_eff  = (B_rem / B_act) * tau_fwd            batch-normalised effective latency
  tau_load = sum_i tau_load_layer^(i)             per-layer materialization times, summed
  rho      = tau_eff / tau_load                   (+inf for zero load)
  rho > 1 and B_act < B_rem  -> next reclamation step
  rho < theta (0.9)          -> reverse one reclamation step
  otherwise                  -> keep
  the planner runs every CI (16) decoding iterations, only with B_act > 0, and ends at B_rem = 0.

Reclamation has two stages: first every uncompressed-resident layer becomes pageable (its
tensors stay in compressed GPU memory), then tensor-level offloading: a step moves up to
ceil(AG * L_r) GPU-backed down-projection tensors to the host, and once no down-projection
tensor is GPU-backed, up to ceil(AG * L_r / 2) fused gate/up tensors.  Every tensor of a step
goes to the layer with the smallest CPU-assigned volume, ties to the larger layer index, and
inside the layer to the largest expert index.  Restoration undoes the steps in reverse order.

Readings where the paper is silent: layers are converted one per step, largest index first;
a step that finds fewer tensors than its size takes what is left; volumes are counted in
down-projection tensors (a fused tensor counts 2, Sec. 4.2: sigma_1 = 2 sigma_2).
"""
from __future__ import annotations

import math

KEEP, RECLAIM, RESTORE, SKIP, DONE = 0, 1, -1, 2, 3
DOWN, FUSED = 2, 1


class Planner:
    def __init__(self, n_layers: int, L_r: int, theta: float = 0.9, AG: float = 0.25, CI: int = 16,
                 uncompressed_layers=()):
        self.N, self.L_r, self.theta, self.AG, self.CI = n_layers, L_r, theta, AG, CI
        self.uncompressed = set(uncompressed_layers)          # U_r; the rest is P_r
        self.on_host = set()                                  # (layer, expert, type)
        self.volume = [0] * n_layers                          # CPU-assigned volume per layer
        self.history = []                                     # reclamation steps, for restoration
        self.iteration = 0
        self.done = False

    # ------------------------------------------------------------------ control signals
    @staticmethod
    def rho(B_rem, B_act, tau_fwd, tau_load_layer):
        tau_eff = (B_rem / B_act) * tau_fwd
        tau_load = sum(tau_load_layer)
        return math.inf if tau_load == 0 else tau_eff / tau_load

    # ------------------------------------------------------------------ residency steps
    def cpu_volume(self, layer):
        return self.volume[layer]

    def _move(self, t, to_host):
        layer, _, d = t
        (self.on_host.add if to_host else self.on_host.discard)(t)
        self.volume[layer] += (1 if d == DOWN else 2) * (1 if to_host else -1)

    def _pick(self, d):
        """The next tensor of type d to offload, or None."""
        best = None
        for layer in range(self.N):
            if layer in self.uncompressed:
                continue
            experts = [e for e in range(self.L_r) if (layer, e, d) not in self.on_host]
            if not experts:
                continue
            key = (self.cpu_volume(layer), -layer)
            if best is None or key < best[0]:
                best = (key, (layer, max(experts), d))
        return None if best is None else best[1]

    def reclaim(self):
        if self.uncompressed:
            layer = max(self.uncompressed)
            self.uncompressed.discard(layer)
            self.history.append(("layer", layer))
            return [("layer", layer)]
        d = DOWN if self._pick(DOWN) is not None else FUSED
        size = math.ceil(self.AG * self.L_r) if d == DOWN else math.ceil(self.AG * self.L_r / 2)
        moved = []
        for _ in range(size):
            t = self._pick(d)
            if t is None:
                break
            self._move(t, True)
            moved.append(t)
        if moved:
            self.history.append(("tensors", moved))
        return moved

    def restore(self):
        if not self.history:
            return []
        kind, what = self.history.pop()
        if kind == "layer":
            self.uncompressed.add(what)
            return [("layer", what)]
        for t in what:
            self._move(t, False)
        return list(reversed(what))

    # ------------------------------------------------------------------ Alg. 2
    def tick(self, B_rem, B_act, tau_fwd, tau_load_layer):
        """One decoding iteration.  Returns (action, rho, changed)."""
        if self.done or B_rem == 0:
            self.done = True
            return DONE, math.nan, []
        self.iteration += 1
        if self.iteration % self.CI != 0 or B_act == 0:
            return SKIP, math.nan, []
        r = self.rho(B_rem, B_act, tau_fwd, tau_load_layer)
        if r > 1 and B_act < B_rem:
            changed = self.reclaim()
            return (RECLAIM if changed else KEEP), r, changed
        if r < self.theta:
            changed = self.restore()
            return (RESTORE if changed else KEEP), r, changed
        return KEEP, r, []


def balanced_split(beta_gpu: float, beta_cpu: float, L_r: int):
    """Sec. 4.2 "Memory hierarchy model": the CPU share that equalises the two backends' times is
    x_bw = beta_cpu / (beta_gpu + beta_cpu); a layer's BF16 volume is 3 L_r down-projection
    tensors (sigma_1 = 2 sigma_2), so the target is 3 L_r x_bw down tensors, rounded upward.
    Returns (x_bw, n_down, n_fused, x_realised).  Reading for x_bw > 1/3, which the paper says
    does not occur in its deployments: all L_r down tensors, then fused tensors (2 units each),
    rounded upward again."""
    x_bw = beta_cpu / (beta_gpu + beta_cpu)
    units = math.ceil(3 * L_r * x_bw - 1e-12)
    n_down = min(units, L_r)
    n_fused = min(L_r, math.ceil((units - n_down) / 2))
    return x_bw, n_down, n_fused, (n_down + 2 * n_fused) / (3 * L_r)
