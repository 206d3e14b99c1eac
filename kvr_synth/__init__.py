"""Seeded synthetic inputs for the KVReviver decode hot path.

This module only manufactures *inputs* (keys, values, queries, needle
positions, workload sizes).  It contains none of the method's arithmetic: no
hashing into the sketch, no median, no softmax, no selection.  Both the CPU
oracle's tests and the HIP path's tests / benchmark draw their inputs from
here, so the two sides see the same bytes.

Generator: counter based.  Every tensor element has a 64-bit counter
``key(tensor, layer, sequence, head) + flat_index``; the counter goes through a
SplitMix64-style finaliser built only from wrapping integer multiplies, xors and
shifts (bit-identical on CPU and GPU torch), and the top 16 bits index a table
of standard-normal quantiles that is always built on the CPU and quantised to
multiples of 2**-12 so that it does not depend on a libm's last bit.  Any
row of any unit can therefore be regenerated alone, on either device.

The workloads mimic the *shape* of what the paper evaluates on (Experiments,
Setup: ~2k-token summarisation inputs and up-to-32k needle-in-a-haystack /
long-document inputs): iid N(0,1) keys and values (the distribution the paper's
Mathematical Analysis assumes), a few outlier channels, and a handful of
"needle" keys aligned with the query direction.  None of the paper's datasets
is used or reproduced.
"""
from __future__ import annotations

import functools
import math
from dataclasses import dataclass

import numpy as np
import torch

BASE_SEED = 251217917
_M64 = (1 << 64) - 1

# tensor ids that key the counter streams
_T_K, _T_V, _T_Q, _T_U, _T_NEEDLE, _T_SCORE = 1, 2, 3, 4, 5, 6


@dataclass(frozen=True)
class Workload:
    """One synthetic configuration (shapes only; all data comes from the seed)."""
    name: str
    cfg_id: int
    layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    context: int          # N: tokens present before the first decode step
    dtype: str            # "f32" | "bf16": storage type of K, V, q and the sketch
    budget: float         # fraction of the full KV bytes that may stay resident
    r: int                # sketch rows
    needles: int
    outlier_channels: int
    steps: int
    needle_spread: bool = False   # True: needles at evenly spaced positions

    # -- sizes derived from the budget (Parameter Settings appendix: the
    #    best split found is Vague 0.1 / Candidate 0.45 / Recent 0.45) --------
    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def budget_tokens(self) -> int:          # M
        return int(math.floor(self.budget * self.context + 1e-9))

    @property
    def w(self) -> int:                       # slots per sketch row
        return max(1, (self.budget_tokens // 10) // self.r)

    @property
    def sketch_slots(self) -> int:            # S = r*w
        return self.r * self.w

    @property
    def n_retained(self) -> int:              # R
        return self.budget_tokens - self.sketch_slots

    @property
    def n_recent(self) -> int:                # R_r
        return self.n_retained // 2

    @property
    def n_candidate(self) -> int:             # C
        return self.n_retained - self.n_recent

    @property
    def n_vague0(self) -> int:                # a at step 0
        return self.context - self.n_retained

    @property
    def units_per_layer(self) -> int:
        return self.batch * self.n_kv_heads

    @property
    def torch_dtype(self) -> torch.dtype:
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS = {
    "c1": Workload("c1", 1, 1, 1, 1, 1, 128, 2048, "f32", 0.10, 3, 4, 0, 1),
    "c2": Workload("c2", 2, 1, 8, 32, 8, 128, 2048, "bf16", 0.10, 3, 16, 4, 128),
    "c3": Workload("c3", 3, 36, 1, 32, 8, 128, 32768, "bf16", 0.25, 3, 64, 4, 256),
    "c4": Workload("c4", 4, 36, 16, 32, 8, 128, 32768, "bf16", 0.25, 3, 64, 4, 128),
    "c5": Workload("c5", 5, 36, 4, 32, 8, 128, 131072, "bf16", 0.25, 4, 64, 4, 64,
                   needle_spread=True),
}


def layer_budgets(wl: Workload, ratios):
    """Non-uniform memory budgets across layers (the paper derives the allocation
    ratio of a layer from the Fisher information of its key and value weights;
    here the ratios are an input).  Returns one Workload per layer with
    budget_l = wl.budget * ratios[l] / mean(ratios), so that the total over the
    layers stays wl.budget * layers (up to the per-layer rounding to tokens).
    Everything else (shapes, seeds, data) is the layer's own as before."""
    import dataclasses
    ratios = [float(x) for x in ratios]
    if len(ratios) != wl.layers or min(ratios) <= 0:
        raise ValueError("one positive ratio per layer")
    mean = sum(ratios) / len(ratios)
    out = []
    for x in ratios:
        b = wl.budget * x / mean
        if not (0.0 < b <= 1.0):
            raise ValueError(f"layer budget {b} outside (0, 1]")
        out.append(dataclasses.replace(wl, budget=b))
    return out


def small_workload(name="tiny", *, layers=1, batch=2, n_q_heads=4, n_kv_heads=2,
                   context=300, dtype="bf16", budget=0.25, r=3, needles=3,
                   outlier_channels=2, steps=4, cfg_id=99, needle_spread=False):
    """A free-form small workload for tests (same recipe, other sizes)."""
    return Workload(name, cfg_id, layers, batch, n_q_heads, n_kv_heads, 128, context,
                    dtype, budget, r, needles, outlier_channels, steps, needle_spread)


# ---------------------------------------------------------------------------
# counter-based generator
# ---------------------------------------------------------------------------
def _s64(x: int) -> int:
    """Python int (mod 2**64) -> the same bits as a signed int64 value."""
    x &= _M64
    return x - (1 << 64) if x >= (1 << 63) else x


def _mix_py(x: int) -> int:
    x = (x + 0x9E3779B97F4A7C15) & _M64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _M64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _M64
    return x ^ (x >> 31)


def stream_key(seed: int, *ids: int) -> int:
    """64-bit key of one counter stream (pure Python integer arithmetic)."""
    k = _mix_py(seed)
    for i in ids:
        k = _mix_py(k ^ _mix_py((int(i) + 0x632BE59BD9B4E019) & _M64))
    return k


def _lsr(z: torch.Tensor, k: int) -> torch.Tensor:
    return (z >> k) & ((1 << (64 - k)) - 1)


def _mix_torch(x: torch.Tensor) -> torch.Tensor:
    """SplitMix64-style finaliser on int64 tensors (wrapping arithmetic)."""
    z = x + _s64(0x9E3779B97F4A7C15)
    z = (z ^ _lsr(z, 30)) * _s64(0xBF58476D1CE4E5B9)
    z = (z ^ _lsr(z, 27)) * _s64(0x94D049BB133111EB)
    return z ^ _lsr(z, 31)


_TABLE_CPU = None
_TABLE_DEV = {}


def normal_table(device="cpu") -> torch.Tensor:
    """65536 standard-normal quantiles, float32, multiples of 2**-12 (built on CPU)."""
    global _TABLE_CPU
    if _TABLE_CPU is None:
        u = (torch.arange(65536, dtype=torch.float64) + 0.5) / 65536.0
        z = torch.special.ndtri(u)
        _TABLE_CPU = (torch.round(z * 4096.0) / 4096.0).to(torch.float32)
    dev = torch.device(device)
    if dev.type == "cpu":
        return _TABLE_CPU
    key = str(dev)
    if key not in _TABLE_DEV:
        _TABLE_DEV[key] = _TABLE_CPU.to(dev)
    return _TABLE_DEV[key]


def normals(keys, count: int, offset: int = 0, device="cpu") -> torch.Tensor:
    """float32 [len(keys), count] of N(0,1) draws; row i uses stream keys[i],
    counters offset .. offset+count-1."""
    dev = torch.device(device)
    kt = torch.tensor([_s64(k) for k in keys], dtype=torch.int64, device=dev).view(-1, 1)
    ctr = torch.arange(offset, offset + count, dtype=torch.int64, device=dev).view(1, -1)
    z = _mix_torch(kt + ctr)
    idx = _lsr(z, 48)
    return normal_table(dev)[idx]


def uniforms(keys, count: int, offset: int = 0, device="cpu") -> torch.Tensor:
    """float32 [len(keys), count] in [0,1): 24 random bits / 2**24 (exact)."""
    dev = torch.device(device)
    kt = torch.tensor([_s64(k) for k in keys], dtype=torch.int64, device=dev).view(-1, 1)
    ctr = torch.arange(offset, offset + count, dtype=torch.int64, device=dev).view(1, -1)
    z = _mix_torch(kt + ctr)
    return _lsr(z, 40).to(torch.float32) * (1.0 / 16777216.0)


# ---------------------------------------------------------------------------
# per-unit small quantities (always computed on the CPU, float64)
# ---------------------------------------------------------------------------
@functools.lru_cache(maxsize=None)
def topic_direction(wl: Workload, layer: int, b: int, h: int) -> np.ndarray:
    """Unit vector u of the (layer, sequence, kv head) unit, float64 [D]."""
    g = normals([stream_key(BASE_SEED, wl.cfg_id, _T_U, layer, b, h)], wl.head_dim)
    u = g[0].double().numpy()
    return u / np.linalg.norm(u)


def needle_positions(wl: Workload, b: int) -> np.ndarray:
    """Sorted needle positions of sequence b (the same for all layers and heads).
    Drawn outside the step-0 Recent window unless the workload spreads them."""
    if wl.needles == 0:
        return np.zeros(0, dtype=np.int64)
    if wl.needle_spread:
        i = np.arange(wl.needles, dtype=np.float64)
        return np.floor((i + 0.5) * wl.context / wl.needles).astype(np.int64)
    hi = max(wl.needles, wl.context - wl.n_recent)
    rng = np.random.Generator(np.random.Philox(key=[BASE_SEED + wl.cfg_id, b]))
    return np.sort(rng.choice(hi, size=wl.needles, replace=False)).astype(np.int64)


def outlier_channels(wl: Workload, layer: int, h: int) -> np.ndarray:
    if wl.outlier_channels == 0:
        return np.zeros(0, dtype=np.int64)
    rng = np.random.Generator(np.random.Philox(key=[BASE_SEED + 7919 * wl.cfg_id, layer * 4096 + h]))
    return np.sort(rng.choice(wl.head_dim, size=wl.outlier_channels, replace=False)).astype(np.int64)


def needle_keys(wl: Workload, layer: int, b: int, h: int) -> np.ndarray:
    """float64 [needles, D]: sqrt(D) * (0.9 u + sqrt(0.19) n), n a unit vector
    orthogonal to u, so cos(key, u) = 0.9."""
    D = wl.head_dim
    u = topic_direction(wl, layer, b, h)
    if wl.needles == 0:
        return np.zeros((0, D))
    g = normals([stream_key(BASE_SEED, wl.cfg_id, _T_NEEDLE, layer, b, h)], wl.needles * D)
    n = g[0].double().numpy().reshape(wl.needles, D)
    n = n - np.outer(n @ u, u)
    n = n / np.linalg.norm(n, axis=1, keepdims=True)
    return math.sqrt(D) * (0.9 * u[None, :] + math.sqrt(0.19) * n)


# ---------------------------------------------------------------------------
# bulk tensors
# ---------------------------------------------------------------------------
def _kv_rows(wl: Workload, layer: int, units, pos0: int, pos1: int, device):
    """K, V float32 [len(units), pos1-pos0, D] before the storage cast."""
    D = wl.head_dim
    n = pos1 - pos0
    kk = [stream_key(BASE_SEED, wl.cfg_id, _T_K, layer, b, h) for (b, h) in units]
    vk = [stream_key(BASE_SEED, wl.cfg_id, _T_V, layer, b, h) for (b, h) in units]
    K = normals(kk, n * D, pos0 * D, device).view(len(units), n, D)
    V = normals(vk, n * D, pos0 * D, device).view(len(units), n, D)
    for i, (b, h) in enumerate(units):
        oc = outlier_channels(wl, layer, h)
        if len(oc):
            oct_ = torch.as_tensor(oc, device=K.device)
            K[i, :, oct_] *= 8.0
            V[i, :, oct_] *= 8.0
        npos = needle_positions(wl, b)
        sel = [(j, int(p)) for j, p in enumerate(npos) if pos0 <= p < pos1]
        if sel:
            nk = needle_keys(wl, layer, b, h)
            rows = torch.as_tensor([p - pos0 for _, p in sel], device=K.device)
            vals = torch.as_tensor(nk[[j for j, _ in sel]], dtype=torch.float32, device=K.device)
            K[i, rows] = vals
    return K, V


def kv_unit(wl: Workload, layer: int, b: int, h: int, pos0: int = 0, pos1: int | None = None,
            device="cpu"):
    """K, V of one (layer, sequence, kv head) unit, rows pos0..pos1-1, storage dtype."""
    if pos1 is None:
        pos1 = wl.context
    K, V = _kv_rows(wl, layer, [(b, h)], pos0, pos1, device)
    return K[0].to(wl.torch_dtype), V[0].to(wl.torch_dtype)


def kv_layer(wl: Workload, layer: int, pos0: int = 0, pos1: int | None = None, device="cpu"):
    """K, V [B, Hkv, pos1-pos0, D] of a whole layer, storage dtype."""
    if pos1 is None:
        pos1 = wl.context
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    K, V = _kv_rows(wl, layer, units, pos0, pos1, device)
    shp = (wl.batch, wl.n_kv_heads, pos1 - pos0, wl.head_dim)
    return K.view(shp).to(wl.torch_dtype), V.view(shp).to(wl.torch_dtype)


def new_tokens(wl: Workload, layer: int, step: int, device="cpu"):
    """k, v [B, Hkv, D] of the token generated at decode step `step`
    (position context+step of every unit's stream)."""
    K, V = kv_layer(wl, layer, wl.context + step, wl.context + step + 1, device)
    return K[:, :, 0].contiguous(), V[:, :, 0].contiguous()


def queries(wl: Workload, layer: int, step: int, device="cpu") -> torch.Tensor:
    """q [B, Hq, D] for decode step `step`: sqrt(D) * normalize(u + 0.3 eps); the
    fp32 single-head workload (no noise term needed) uses q = sqrt(D) u at step 0.
    Float arithmetic here runs on the CPU; the result is then moved."""
    D = wl.head_dim
    G = wl.group
    out = np.zeros((wl.batch, wl.n_q_heads, D))
    for b in range(wl.batch):
        keys = [stream_key(BASE_SEED, wl.cfg_id, _T_Q, layer, b, hq) for hq in range(wl.n_q_heads)]
        eps = normals(keys, D, step * D).double().numpy()
        for hq in range(wl.n_q_heads):
            u = topic_direction(wl, layer, b, hq // G)
            if wl.name == "c1" and step == 0:
                x = u
            else:
                x = u + 0.3 * eps[hq]
                x = x / np.linalg.norm(x)
            out[b, hq] = math.sqrt(D) * x
    return torch.as_tensor(out, dtype=torch.float32).to(wl.torch_dtype).to(device)


def queries_many(wl: Workload, layer: int, step0: int, nsteps: int, device="cpu") -> torch.Tensor:
    """q [nsteps, B, Hq, D], same values as stacking queries(step0..step0+nsteps-1)
    when run on the CPU; on a GPU the normalisation runs there (benchmark use:
    last-bit differences from the CPU version are possible)."""
    D = wl.head_dim
    G = wl.group
    dev = torch.device(device)
    keys = [stream_key(BASE_SEED, wl.cfg_id, _T_Q, layer, b, hq)
            for b in range(wl.batch) for hq in range(wl.n_q_heads)]
    eps = normals(keys, nsteps * D, step0 * D, dev).view(wl.batch, wl.n_q_heads, nsteps, D)
    u = np.stack([np.stack([topic_direction(wl, layer, b, hq // G) for hq in range(wl.n_q_heads)])
                  for b in range(wl.batch)])
    ut = torch.as_tensor(u, dtype=torch.float64, device=dev).unsqueeze(2)
    x = ut + 0.3 * eps.double()
    x = x / torch.linalg.vector_norm(x, dim=-1, keepdim=True)
    q = (math.sqrt(D) * x).to(torch.float32).to(wl.torch_dtype)
    return q.permute(2, 0, 1, 3).contiguous()


def positive_scores(wl: Workload, layer: int, b: int, h: int, n: int, device="cpu") -> torch.Tensor:
    """float32 [n] of strictly positive pseudo "cumulative scores" (uniform draws
    on a 2**-24 grid plus 2**-24): an input for selection tests that need scores
    but no attention pass; ties occur on purpose."""
    k = stream_key(BASE_SEED, wl.cfg_id, _T_SCORE, layer, b, h)
    return uniforms([k], n, 0, device)[0] + (1.0 / 16777216.0)
