"""Hierarchical Roofline Model for the MoE layer (host arithmetic only, no GPU work).

The paper extends the roofline model with the bandwidth BETWEEN two memory levels
(its section 3): a task executed on level i (the GPU) whose data comes from level j
(host memory) is bounded by three roofs,

    P = min(P_peak^i, B_peak^i * I^i, B_peak^{j,i} * I^j)                    (Eq. 7)

where I^i and I^j are the operational intensities with respect to the bytes touched in
each level.  The two turning points (Eqs. 9, 10), the balance point (Eq. 11) and the
per-layer latency model T = max(comm, T_cpu, T_gpu) of its section 4.2 follow from that.
This module states those formulas for the layer this library computes (FLOPs
6*R*h1*h2 + 2*T*h1*n_e; weights 3*n_e*h1*h2*dt) and searches the policy (batch size N,
micro-batch size mu, resident weight fraction r_w) the way the paper's optimiser does, for
the part of the system that exists here: there is no CPU task, so T_cpu = 0.

Symbols follow the paper's notation table: h1, h2 model and expert hidden sizes, n_e
experts, k experts per token, dt bytes per element, N tokens per pass (batch), mu
tokens per kernel execution (micro-batch), r_w fraction of the weights kept on the GPU,
p_g, b_g GPU FLOP/s and memory bandwidth, b_cg host-to-GPU bandwidth, m_g GPU memory.
"""
from __future__ import annotations

import dataclasses
import math
from typing import Dict, Iterable, Optional, Tuple


@dataclasses.dataclass(frozen=True)
class Hardware:
    p_g: float                      # GPU FLOP/s
    b_g: float                      # GPU memory bytes/s
    b_cg: float                     # host -> GPU bytes/s
    m_g: float = 288e9              # GPU memory bytes
    p_c: float = 0.0                # host FLOP/s   (only used by the turning point P1)
    b_c: float = 0.0                # host memory bytes/s
    m_c: float = math.inf           # host memory bytes (bounds the batch size in the policy search)


# Published peaks of one MI355X, and its profiled rates (section 4.2 of the paper feeds its model with profiled peak
# performance and bandwidths).  The profiled rates come from `python bench.py --rate-probes`, three probes that are none
# of the layer runs the model is compared with: a dense bf16 product of 2048 x 8192 x 32768 through the library's paged
# linear map (1290 TFLOP/s), a kernel of nothing but loads over 4 GiB of device memory (6.15 TB/s), one pinned-host to
# device copy of 1 GiB (57.3 GB/s).
MI355X_PEAK = Hardware(p_g=2.5e15, b_g=8.0e12, b_cg=64e9)
MI355X_PROBED = Hardware(p_g=1.29e15, b_g=6.15e12, b_cg=57.3e9)


@dataclasses.dataclass(frozen=True)
class Layer:
    h1: int
    h2: int
    n_e: int
    k: int
    dt: int = 2                     # bytes per element of weights and activations

    @property
    def weight_bytes(self) -> float:
        return 3.0 * self.n_e * self.h1 * self.h2 * self.dt

    def flops(self, tokens: int) -> float:
        """Expert FFN (three products per routed row) plus the router."""
        return 6.0 * tokens * self.k * self.h1 * self.h2 + 2.0 * tokens * self.h1 * self.n_e

    def gpu_bytes(self, mu: int) -> float:
        """Algorithmic GPU-memory traffic of one kernel execution on mu tokens: the weights of the experts
        that receive rows, once, plus the activations (x, permuted rows, h written and read, expert
        outputs written and read, y)."""
        R = mu * self.k
        touched = self.n_e * (1.0 - (1.0 - 1.0 / self.n_e) ** R)          # expected experts with at least one row
        weights = 3.0 * touched * self.h1 * self.h2 * self.dt
        acts = (2 * mu * self.h1 * self.dt + 2 * R * self.h1 * self.dt + 2 * R * self.h2 * self.dt
                + 2 * 4 * R * self.h1 + 4 * mu * self.h1)
        return weights + acts

    def workspace_bytes(self, mu: int) -> float:
        R = mu * self.k
        return R * self.h1 * self.dt + R * self.h2 * self.dt + 4.0 * R * self.h1 + 4.0 * mu * self.h1 + 40.0 * R


def attainable(p_peak: float, b_peak: float, intensity: float) -> float:
    """Single-level roofline (Eq. 8): min(P_peak, B_peak * I)."""
    return min(p_peak, b_peak * intensity)


def attainable_hrm(p_peak_i: float, b_peak_i: float, i_i: float, b_ji: float, i_j: float) -> float:
    """Three roofs of a task on level i that fetches its data from level j (Eq. 7)."""
    return min(p_peak_i, b_peak_i * i_i, b_ji * i_j)


def turning_point_p1(hw: Hardware) -> float:
    """Eq. 9 solved for the intensity (with respect to the data on the host): below it the link roof
    B^{j,i} * I lies under what the host itself attains, min(P^j, B^j * I), so moving the data to the GPU
    does not pay.  With b_cg < b_c the two meet on the host's compute roof, at I = p_c / b_cg."""
    if hw.b_cg >= hw.b_c:
        return 0.0 if hw.b_c > 0 else math.inf
    return hw.p_c / hw.b_cg


def turning_point_p2(hw: Hardware, i_gpu: float) -> float:
    """Eq. 10: the intensity (with respect to the host data) below which the task is bound by the
    host-to-GPU bandwidth; i_gpu is its intensity with respect to GPU memory."""
    return attainable(hw.p_g, hw.b_g, i_gpu) / hw.b_cg


def balance_intensity(hw: Hardware, i_gpu: float) -> float:
    """Eq. 11: the host-data intensity at which the link roof equals the GPU memory roof."""
    return hw.b_g * i_gpu / hw.b_cg


def layer_latency(layer: Layer, hw: Hardware, N: int, mu: int, r_w: float, hidden_from_host: bool = True) -> Dict[str, float]:
    """Per-layer latency of one pass of N tokens in micro-batches of mu (section 4.2):
    T = max(comm, T_gpu), comm = the bytes that go from the host to the GPU for the layer / b_cg, i.e. the
    non-resident weights (1 - r_w) * weight bytes and, with hidden_from_host, the hidden state of every
    token (h1 * dt bytes: in the paper's pipeline it comes back from the attention on the host), and
    T_gpu = sum over micro-batches of max(FLOPs / p_g, GPU bytes / b_g)."""
    n_full, rest = divmod(N, mu)
    t_gpu = 0.0
    for tokens, count in ((mu, n_full), (rest, 1 if rest else 0)):
        if count:
            t_gpu += count * max(layer.flops(tokens) / hw.p_g, layer.gpu_bytes(tokens) / hw.b_g)
    comm = ((1.0 - r_w) * layer.weight_bytes + (N * layer.h1 * layer.dt if hidden_from_host else 0.0)) / hw.b_cg
    t = max(comm, t_gpu)
    flops = layer.flops(N)
    i_link = flops / ((1.0 - r_w) * layer.weight_bytes) if r_w < 1.0 else math.inf
    return {"T": t, "comm": comm, "T_gpu": t_gpu, "tokens_per_s": N / t, "flops_per_s": flops / t,
            "bound": "link" if comm >= t_gpu else "gpu", "I_link": i_link,
            "I_gpu": layer.flops(mu) / layer.gpu_bytes(mu)}


def crossover_micro_batch(layer: Layer, hw: Hardware) -> int:
    """Smallest micro-batch for which one kernel execution is compute bound on the GPU
    (FLOPs / p_g >= GPU bytes / b_g): the ridge of Eq. 8 expressed in tokens."""
    lo, hi = 1, 1 << 24
    while lo < hi:
        mid = (lo + hi) // 2
        if layer.flops(mid) / hw.p_g >= layer.gpu_bytes(mid) / hw.b_g:
            hi = mid
        else:
            lo = mid + 1
    return lo


def best_policy(layer: Layer, hw: Hardware, batch_sizes, micro_batches: Iterable[int], n_layers: int = 1,
                r_w_steps: int = 20, host_bytes_per_token: float = 0.0) -> Tuple[Optional[Dict[str, float]], Dict[str, float]]:
    """Exhaustive search over the policy (N, mu, r_w) - the two integers and the weight fraction of the paper's
    section 4.2 that exist for this layer - for the highest throughput N / T, T = layer_latency(N, mu, r_w), under
      GPU memory:  n_layers * r_w * weights + 2 * (1 - r_w) * weights (the double buffer) + workspace(mu) <= m_g
      host memory: n_layers * (1 - r_w) * weights + N * host_bytes_per_token <= m_c
    (host_bytes_per_token: what a token keeps in host memory over all layers, e.g. its KV cache and hidden states; the
    attention side is not part of this library, so it is a parameter).  batch_sizes: an int or the candidate values of N.
    Among policies of equal throughput the smallest N, then the smallest r_w wins (less latency, less GPU memory).
    Returns (policy or None, its latency record)."""
    Ns = [batch_sizes] if isinstance(batch_sizes, int) else sorted(batch_sizes)
    mus = sorted(micro_batches)
    best, best_rec = None, {}
    for N in Ns:
        for mu in mus:
            if mu > N:
                continue
            for step in range(r_w_steps + 1):
                r_w = step / r_w_steps
                need = (n_layers * r_w + 2.0 * (1.0 - r_w)) * layer.weight_bytes + layer.workspace_bytes(mu)
                host = n_layers * (1.0 - r_w) * layer.weight_bytes + N * host_bytes_per_token
                if need > hw.m_g or host > hw.m_c:
                    continue
                rec = layer_latency(layer, hw, N, mu, r_w)
                if best is None or rec["tokens_per_s"] > best_rec["tokens_per_s"] * (1.0 + 1e-12):
                    best, best_rec = {"N": N, "mu": mu, "r_w": r_w, "gpu_bytes_needed": need, "host_bytes_needed": host}, rec
    return best, best_rec


MIXTRAL_8X7B = Layer(h1=4096, h2=14336, n_e=8, k=2)
MIXTRAL_8X22B = Layer(h1=6144, h2=16384, n_e=8, k=2)
DBRX = Layer(h1=6144, h2=10752, n_e=16, k=4)


if __name__ == "__main__":
    hw = MI355X_PROBED
    for name, layer in (("Mixtral-8x7B", MIXTRAL_8X7B), ("Mixtral-8x22B", MIXTRAL_8X22B), ("DBRX", DBRX)):
        mu_star = crossover_micro_batch(layer, hw)
        print(f"{name}: weights {layer.weight_bytes / 2**30:.2f} GiB/layer, compute bound from mu = {mu_star} tokens; "
              f"P2 at I_link = {turning_point_p2(hw, layer.flops(mu_star) / layer.gpu_bytes(mu_star)):.0f} FLOP/B")
        for N, mu, r_w in ((256, 256, 1.0), (4096, 4096, 1.0), (16384, 4096, 0.0), (16384, 4096, 0.5), (16384, 4096, 0.8)):
            r = layer_latency(layer, hw, N, mu, r_w)
            print(f"   N={N:6d} mu={mu:5d} r_w={r_w:.1f}: T={r['T'] * 1e3:8.3f} ms ({r['bound']:4s} bound)  "
                  f"{r['tokens_per_s'] / 1e6:6.3f} M tokens/s  I_link={r['I_link']:.0f}")
