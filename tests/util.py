"""Test helpers: move data between the oracle's numpy world and device tensors,
and build oracle states from the synthetic workloads.  No method arithmetic."""
import math

import numpy as np
import torch

import kvr_synth as S
from oracle import kvr_oracle as O


def storage_name(dtype):
    return "f32" if dtype == torch.float32 else "bf16"


def to_np(t: torch.Tensor) -> np.ndarray:
    """Device/any tensor -> float64 numpy (exact for f32 and bf16)."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def to_dev(x: np.ndarray, dtype, device="cuda") -> torch.Tensor:
    """float64 numpy holding storage-representable values -> device tensor."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float64)).to(dtype)
    return t.to(device).contiguous()


def rand_storage(rng, shape, dtype, scale=1.0):
    """Random values representable in the storage type, as float64 numpy."""
    x = rng.standard_normal(shape) * scale
    return O.to_storage(x, storage_name(dtype))


def oracle_units_from_workload(wl: S.Workload, layer: int, units, *, acc_dtype=np.float32,
                               compress=True, extra_tokens=None):
    """For each (b, h) in units: the oracle state after the prompt (dense scores
    from the step-0 queries, partition, bulk insert, compaction to R+1 slots).
    Returns list of UnitState."""
    params = O.hash_params_from_seed(S.BASE_SEED + layer, wl.r)
    scale = 1.0 / math.sqrt(wl.head_dim)
    q0 = S.queries(wl, layer, 0)
    G = wl.group
    extra = wl.steps if extra_tokens is None else extra_tokens
    out = []
    for (b, h) in units:
        K, V = S.kv_unit(wl, layer, b, h)
        K, V = to_np(K), to_np(V)
        q = to_np(q0[b, h * G:(h + 1) * G])
        st = O.dense_prefill_state(K, V, q, scale, wl.r, wl.w, params, wl.dtype,
                                   n_recent=wl.n_recent, k_candidate=wl.n_candidate,
                                   n_cap=wl.context + extra, acc_dtype=acc_dtype)
        if compress:
            st.compress()
            st = O.compact(st, wl.n_retained + 1)
        out.append(st)
    return out


def layer_state_from_oracle(kvr, LayerState, desc, states, B, Hkv, *, vague_cap, evict_cap=8, slack=0, side=None):
    """Upload a list of oracle UnitStates (unit-major, B*Hkv of them) into a
    LayerState on the GPU."""
    s0 = states[0]
    ret_cap = len(s0.ret_pos)
    n_cap = len(s0.scores)
    ls = LayerState(desc, n_recent=s0.n_recent, k_candidate=s0.k_candidate, ret_cap=ret_cap,
                    vague_cap=vague_cap, n_cap=n_cap, evict_cap=evict_cap, slack=slack, side=side)
    ls.r_size = int(s0.r_size)
    dt = ls.dtype
    D = desc.head_dim

    def stack(f, shape):
        return np.stack([f(s) for s in states]).reshape((B, Hkv) + shape)

    ls.k_ret.copy_(to_dev(stack(lambda s: s.K_ret, (ret_cap, D)), dt))
    ls.v_ret.copy_(to_dev(stack(lambda s: s.V_ret, (ret_cap, D)), dt))
    ls.ret_pos.copy_(torch.as_tensor(stack(lambda s: s.ret_pos, (ret_cap,)).astype(np.int32)).cuda())
    ls.scores.copy_(torch.as_tensor(stack(lambda s: s.scores, (n_cap,))).cuda())
    ls.sketch_k.copy_(to_dev(stack(lambda s: s.SK, s0.SK.shape), dt))
    ls.sketch_v.copy_(to_dev(stack(lambda s: s.SV, s0.SV.shape), dt))
    vp = np.zeros((B * Hkv, vague_cap), dtype=np.int32)
    nv = np.zeros(B * Hkv, dtype=np.int32)
    for u, s in enumerate(states):
        nv[u] = len(s.vague_pos)
        vp[u, :nv[u]] = s.vague_pos
    ls.vague_pos.copy_(torch.as_tensor(vp.reshape(B, Hkv, vague_cap)).cuda())
    ls.n_vague.copy_(torch.as_tensor(nv.reshape(B, Hkv)).cuda())
    nctx = np.array([states[b * Hkv].n_ctx for b in range(B)], dtype=np.int32)
    ls.n_ctx.copy_(torch.as_tensor(nctx).cuda())
    return ls
