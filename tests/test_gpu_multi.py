"""GPU parity of kvr_attend_multi (several query tokens per sequence over one
rebuilt cache, each seeing the positions up to its own) against the oracle.
bf16 storage: max |out - oracle| <= 2e-2, cumulative scores within 2e-5 per
query of the call."""
import numpy as np
import pytest
import torch

import kvr_synth as S
from oracle import kvr_oracle as O
from tests import util as U
from tests.test_gpu_parity import TOL_OUT_BF16, say

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def kvr():
    from paper_2512_17917_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def LayerState():
    from paper_2512_17917_amd.state import LayerState as LS
    return LS


def run_multi_case(kvr, LayerState, wl, layer, n_q, accumulate=True):
    """The state after the prompt plus n_q appended tokens (pushed into free retained
    slots, nothing evicted in between: Slack >= n_q), then n_q queries at once."""
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, extra_tokens=n_q + 2)
    G = wl.group
    ret_cap = wl.n_retained + n_q + 1
    for u, st in enumerate(states):
        O.compact(st, ret_cap)
    for t in range(n_q):
        kn, vn = S.new_tokens(wl, layer, t)
        for u, (b, h) in enumerate(units):
            states[u].append(U.to_np(kn[b, h]), U.to_np(vn[b, h]))
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype,
                      hash_params=states[0].params)
    ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads,
                                   vague_cap=wl.n_vague0 + 3)
    q = torch.stack([S.queries(wl, layer, t + 1) for t in range(n_q)], dim=1).contiguous()     # [B, n_q, Hq, D]
    out = ls.attend_multi(q.cuda(), n_q, accumulate_scores=accumulate)
    torch.cuda.synchronize()
    og = out.cpu().double().numpy()
    worst = 0.0
    for u, (b, h) in enumerate(units):
        st = states[u]
        qq = U.to_np(q[b, :, h * G:(h + 1) * G])                                              # [n_q, G, D]
        q_pos = np.arange(st.n_ctx - n_q, st.n_ctx)
        o_ref, sc_ref, _ = O.attend_multi(qq, q_pos, st.K_ret, st.V_ret, st.ret_pos, st.SK, st.SV, st.params,
                                          st.vague_pos, st.n_ctx, d.softmax_scale,
                                          scores=st.scores if accumulate else None, storage=wl.dtype)
        err = np.abs(og[b, :, h * G:(h + 1) * G] - o_ref).max()
        worst = max(worst, err)
        assert err <= TOL_OUT_BF16, f"unit {(b, h)}: max abs error {err}"
        got = ls.scores[b, h].cpu().double().numpy()
        want = (sc_ref if accumulate else st.scores).astype(np.float64)
        assert np.abs(got - want).max() <= 2e-5 * n_q
    return worst


@pytest.mark.parametrize("n_q,heads", [(4, (8, 2)), (2, (8, 2)), (1, (8, 2)), (4, (4, 2)), (8, (4, 2)), (16, (2, 2)),
                                       (4, (2, 2))])
def test_attend_multi_follows_the_oracle(kvr, LayerState, n_q, heads):
    say("attend multi", n_q, heads)
    hq, hkv = heads
    wl = S.small_workload(f"mq{n_q}", batch=2, n_q_heads=hq, n_kv_heads=hkv, context=900, budget=0.25, r=3,
                          steps=n_q + 1, cfg_id=90)
    run_multi_case(kvr, LayerState, wl, 0, n_q)


def test_attend_multi_short_vague_list(kvr, LayerState):
    """Fewer than 64 Vague tokens: the list is not worth staging the sketch through LDS for; the dense kernel
    rebuilds its tiles from sketch rows gathered out of memory."""
    say("attend multi, short Vague list")
    wl = S.small_workload("mqshort", batch=1, n_q_heads=8, n_kv_heads=2, context=300, budget=0.9, r=3, steps=5,
                          cfg_id=87)
    assert wl.n_vague0 + 3 < 64
    run_multi_case(kvr, LayerState, wl, 0, 4)


def test_attend_multi_ragged_device_counts(kvr):
    """The Vague list of every unit has its own length on the device: empty, one token, around a tile
    boundary, around a workgroup's share, full, negative and oversized (clamped).  Reference: float64 dense
    causal attention over kvr_reconstruct's output (which test_gpu_parity ties to the oracle bit for bit)."""
    say("attend multi, ragged device counts")
    rng = np.random.default_rng(77)
    B, Hq, Hkv, r, w, D, n_q = 5, 4, 2, 3, 40, 128, 4
    G = Hq // Hkv
    ret_cap, vague_cap = 70, 900
    counts = np.array([[0, 1], [15, 16], [17, 255], [257, 900], [-3, 5000]], dtype=np.int32)
    dt = torch.bfloat16
    d = kvr.make_desc(B, Hq, Hkv, r, w, dt, seed=31)
    dev = "cuda"
    n_ctx_val = ret_cap + vague_cap
    q = torch.randn(B, n_q, Hq, D, device=dev).to(dt)
    k_ret = torch.randn(B, Hkv, ret_cap, D, device=dev).to(dt)
    v_ret = torch.randn(B, Hkv, ret_cap, D, device=dev).to(dt)
    sk = (3 * torch.randn(B, Hkv, r, w, D, device=dev)).to(dt)
    sv = (3 * torch.randn(B, Hkv, r, w, D, device=dev)).to(dt)
    ret_pos = torch.empty(B, Hkv, ret_cap, dtype=torch.int32, device=dev)
    vague_pos = torch.empty(B, Hkv, vague_cap, dtype=torch.int32, device=dev)
    for b in range(B):
        for h in range(Hkv):
            perm = torch.as_tensor(rng.permutation(n_ctx_val).astype(np.int32))
            ret_pos[b, h] = perm[:ret_cap].to(dev)
            vague_pos[b, h] = perm[ret_cap:].to(dev)
    ret_pos[1, 0, 5:9] = -1                                              # a few empty slots
    n_vague = torch.as_tensor(counts).to(dev)
    n_ctx = torch.full((B,), n_ctx_val, dtype=torch.int32, device=dev)
    scores = torch.rand(B, Hkv, n_ctx_val, device=dev)
    scores0 = scores.clone()
    out = torch.full((B, n_q, Hq, D), 9.0, dtype=torch.float32, device=dev)
    ws = torch.empty(kvr.kvr_attend_multi_workspace_size(d, n_q, ret_cap, vague_cap), dtype=torch.uint8, device=dev)
    kvr.kvr_attend_multi(d, q, n_q, n_ctx, k_ret, v_ret, ret_pos, ret_cap, sk, sv, vague_pos, n_vague, vague_cap,
                         out, scores, n_ctx_val, ws)
    kh = torch.zeros(B, Hkv, vague_cap, D, dtype=dt, device=dev)
    vh = torch.zeros_like(kh)
    kvr.kvr_reconstruct(d, sk, sv, vague_pos, n_vague, vague_cap, kh, vh)
    torch.cuda.synchronize()
    nv = n_vague.clamp(0, vague_cap)
    live = torch.arange(vague_cap, device=dev).view(1, 1, -1) < nv.unsqueeze(-1)
    pos_all = torch.cat([ret_pos, torch.where(live, vague_pos, torch.full_like(vague_pos, -1))], dim=2).long()
    Kall = torch.cat([k_ret, kh], dim=2).double()
    Vall = torch.cat([v_ret, vh], dim=2).double()
    inc = torch.zeros(B, Hkv, pos_all.shape[2], dtype=torch.float64, device=dev)
    for t in range(n_q):
        qf = q[:, t].double().view(B, Hkv, G, D)
        logit = torch.einsum("bhgd,bhnd->bhgn", qf, Kall) * d.softmax_scale
        seen = (pos_all >= 0) & (pos_all <= n_ctx_val - n_q + t)
        logit = logit.masked_fill(~seen.unsqueeze(2), float("-inf"))
        pr = torch.softmax(logit, dim=-1)
        ref = torch.einsum("bhgn,bhnd->bhgd", pr, Vall).reshape(B, Hq, D)
        err = (out[:, t].double() - ref).abs().max().item()
        assert err <= 3e-5 * ref.abs().max().item(), (t, err)
        inc += pr.sum(dim=2)
    got = (scores.double() - scores0.double()).gather(2, pos_all.clamp(min=0))
    got = torch.where(pos_all >= 0, got, torch.zeros_like(got))
    assert (got - inc).abs().max().item() <= 2e-5 * n_q
    # positions that are in neither set keep their scores
    touched = torch.zeros(B, Hkv, n_ctx_val + 1, dtype=torch.bool, device=dev)
    touched.scatter_(2, torch.where(pos_all >= 0, pos_all, torch.full_like(pos_all, n_ctx_val)), True)
    assert bool(((scores == scores0) | touched[:, :, :n_ctx_val]).all())


def test_attend_multi_even_rows_and_no_scores(kvr, LayerState):
    say("attend multi r=4, scores off")
    wl = S.small_workload("mq4r", batch=1, n_q_heads=8, n_kv_heads=2, context=700, budget=0.3, r=4, steps=5,
                          cfg_id=89)
    run_multi_case(kvr, LayerState, wl, 1, 4, accumulate=False)


def test_attend_multi_one_query_equals_attend_decode(kvr, LayerState):
    """n_q = 1 is the decode case, computed by another route (rebuilt tokens through
    memory, other kernels): the two entry points must agree to float32 rounding."""
    say("attend multi vs attend decode")
    wl = S.small_workload("mq1", batch=2, n_q_heads=8, n_kv_heads=2, context=1100, budget=0.25, r=3, steps=2,
                          cfg_id=88)
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, 0, units, extra_tokens=3)
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype,
                      hash_params=states[0].params)
    q = S.queries(wl, 0, 1)
    outs, scs = [], []
    for multi in (False, True):
        ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads,
                                       vague_cap=wl.n_vague0 + 3)
        if multi:
            o = ls.attend_multi(q.unsqueeze(1).contiguous().cuda(), 1)[:, 0]
        else:
            o = ls.attend(q.cuda())
        torch.cuda.synchronize()
        outs.append(o.cpu().double().numpy().copy())
        scs.append(ls.scores.cpu().double().numpy().copy())
    big = np.abs(outs[0]).max()
    assert np.abs(outs[0] - outs[1]).max() <= 2e-5 * big
    assert np.abs(scs[0] - scs[1]).max() <= 2e-6


def test_attend_multi_argument_errors(kvr):
    d = kvr.make_desc(1, 8, 2, 3, 5, torch.bfloat16, seed=1)
    with pytest.raises(kvr.KvrError):
        kvr.kvr_attend_multi_workspace_size(d, 3, 10, 10)            # 3 * 4 columns: unsupported
    with pytest.raises(kvr.KvrError):
        kvr.kvr_attend_multi_workspace_size(d, 8, 10, 10)            # 32 columns
    df = kvr.make_desc(1, 8, 2, 3, 5, torch.float32, seed=1)
    with pytest.raises(kvr.KvrError):
        kvr.kvr_attend_multi_workspace_size(df, 1, 10, 10)           # f32 storage
    assert kvr.kvr_attend_multi_workspace_size(d, 4, 10, 10) > 0
