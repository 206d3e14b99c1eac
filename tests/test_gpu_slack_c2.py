"""GPU parity for two things the other step tests do not reach:

  * Slack > 0 (Algorithm 3, first branch): several tokens leave a unit in one
    kvr_step_update call -- append, in-kernel selection of s + 1 tokens, and the
    insert of a list in which tokens share sketch slots, all in one launch --
    against the oracle's UnitState.compress(slack), bit for bit.
  * the second named workload (one Llama-3-8B-shaped layer, batch 8, context 2048,
    10 % budget, x8 outlier channels, 16 needles): all 64 units through prompt
    compression and decode steps on the GPU's own keys, values, sketch and index
    lists.

Tolerances as everywhere: integers and everything stored bit-exact, out within
2e-2 (bf16 storage), scores within 2e-5 per call.
"""
import numpy as np
import pytest
import torch

import kvr_synth as S
from oracle import kvr_oracle as O
from tests import util as U

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]


@pytest.fixture(scope="module")
def kvr():
    from paper_2512_17917_amd import binding
    binding.lib()
    return binding


@pytest.fixture(scope="module")
def LayerState():
    from paper_2512_17917_amd.state import LayerState as LS
    return LS


def say(*a):
    print("[case]", *a, flush=True)


def shared_slot_pairs(params, w, positions):
    """Number of (row, pair of listed tokens) that fall into one sketch slot."""
    n = 0
    for i, prm in enumerate(params):
        b = [O.bucket_of(prm, int(J), w) for J in positions]
        n += sum(1 for x in range(len(b)) for y in range(x) if b[x] == b[y])
    return n


def compare_unit_state(ls, b, h, st, tag):
    assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos), (tag, "ret_pos")
    nv = int(ls.n_vague[b, h])
    assert nv == len(st.vague_pos), (tag, "n_vague", nv, len(st.vague_pos))
    assert np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), np.asarray(st.vague_pos, dtype=np.int64)), (tag, "vague_pos")
    assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK), (tag, "sketch_k")
    assert np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV), (tag, "sketch_v")
    used = st.ret_pos >= 0
    assert np.array_equal(U.to_np(ls.k_ret[b, h])[used], st.K_ret[used]), (tag, "k_ret")
    assert np.array_equal(U.to_np(ls.v_ret[b, h])[used], st.V_ret[used]), (tag, "v_ret")


# ----------------------------------------------------------------------------- Slack
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("slack,context,nsteps", [(3, 700, 9), (7, 700, 17), (63, 600, 65)])
def test_slack_steps_follow_the_oracle(kvr, LayerState, slack, context, nsteps, fused):
    """Decode steps with Slack = s: most steps evict nothing, every (s + 1)-th step
    evicts s + 1 tokens per unit at once.  Before every step the float state
    (scores) comes from the oracle; keys, values, sketch and index lists stay the
    GPU's own from the first step on."""
    say("slack", slack, "fused" if fused else "three calls")
    wl = S.small_workload("slack%d" % slack, batch=2, n_q_heads=8, n_kv_heads=2, context=context, budget=0.25, r=3,
                          steps=nsteps, cfg_id=90)
    layer = 0
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, compress=False, extra_tokens=nsteps + 2)
    for i, st in enumerate(states):
        st.compress(slack)
        states[i] = O.compact(st, wl.n_retained + slack + 1)
    params = states[0].params
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    G, scale = wl.group, d.softmax_scale
    vague_cap = wl.n_vague0 + nsteps + 2
    ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads, vague_cap=vague_cap,
                                   evict_cap=max(8, slack + 1), slack=slack)
    assert ls.ret_cap == wl.n_retained + slack + 1 and ls.r_size == states[0].r_size == wl.n_recent
    pops = shared = 0
    for t in range(nsteps):
        # float state from the oracle; everything else stays the GPU's own
        sc = np.stack([s.scores for s in states]).reshape(wl.batch, wl.n_kv_heads, -1)
        ls.scores.copy_(torch.as_tensor(sc).cuda())
        kn, vn = S.new_tokens(wl, layer, t)
        q = S.queries(wl, layer, t + 1)
        out = ls.decode_step(kn.cuda(), vn.cuda(), q.cuda(), fused=fused, check=True)
        torch.cuda.synchronize()
        og = out.cpu().double().numpy()
        ne = ls.n_evict.cpu().numpy().reshape(-1)
        es = ls.evict_slot.cpu().numpy().reshape(len(units), -1)
        ep = ls.evict_pos.cpu().numpy().reshape(len(units), -1)
        worst = 0.0
        for u, (b, h) in enumerate(units):
            st = states[u]
            o_ref, (ws_, wp_), _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]), U.to_np(q[b, h * G:(h + 1) * G]),
                                                  scale, slack=slack)
            want = slack + 1 if (t + 1) % (slack + 1) == 0 else 0
            assert ne[u] == len(ws_) == want, (t, u, ne[u], len(ws_), want)
            assert np.array_equal(es[u, :want], ws_) and np.array_equal(ep[u, :want], wp_)
            assert ls.r_size == st.r_size
            compare_unit_state(ls, b, h, st, (t, u))
            err = np.abs(og[b, h * G:(h + 1) * G] - o_ref).max()
            worst = max(worst, err)
            assert err <= 2e-2, (t, u, err)
            assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max() <= 2e-5
            if want:
                pops += 1
                shared += shared_slot_pairs(params, wl.w, wp_)
        if (t + 1) % (slack + 1) == 0:
            say("slack", slack, "step", t, "evicted", slack + 1, "per unit; max |out - oracle| =", worst)
    assert pops >= len(units)
    assert shared > 0, "no two tokens of one bulk pop shared a sketch slot: the case does not test what it is for"


def test_step_update_with_an_empty_recent_window(kvr, LayerState):
    """n_recent = 0: the token that was just appended is a Candidate like any other and may
    be the one that leaves.  Fused call = the three separate calls = the oracle."""
    say("step update, n_recent = 0")
    rng = np.random.default_rng(7)
    B, Hkv, D, r, w, k_cand, n0 = 1, 3, 128, 3, 5, 20, 40
    dtype = torch.bfloat16
    params = O.hash_params_from_seed(77, r)
    d = kvr.make_desc(B, Hkv, Hkv, r, w, dtype, hash_params=params)
    results = []
    for fused in (True, False):
        states = []
        for h in range(Hkv):
            st = O.UnitState(k_cand + 1, n0 + 4, r, w, D, params, "bf16", n_recent=0, k_candidate=k_cand,
                             acc_dtype=np.float32)
            rs = np.random.default_rng(100 + h)
            for p in range(k_cand):                       # k_cand raw tokens at scattered positions
                st.K_ret[p] = U.rand_storage(rs, (D,), dtype)
                st.V_ret[p] = U.rand_storage(rs, (D,), dtype)
            st.ret_pos[:k_cand] = rs.choice(n0, size=k_cand, replace=False)
            st.vague_pos = [int(p) for p in range(n0) if p not in set(st.ret_pos.tolist())]
            st.n_ctx = n0
            st.scores[:n0] = rs.random(n0).astype(np.float32) + 0.5
            # unit 0: the new token will score lowest (0) and leaves at once; unit 1: it outranks
            # everything; unit 2: it ties with the lowest candidate (the later position leaves)
            st.scores[n0] = [0.0, 9.0, float(st.scores[st.ret_pos[:k_cand]].min())][h]
            states.append(st)
        ls = U.layer_state_from_oracle(kvr, LayerState, d, states, B, Hkv, vague_cap=n0 + 4)
        ls.r_size = 0
        ls.n_recent = 0
        kn = torch.as_tensor(U.rand_storage(rng, (B, Hkv, D), dtype)).to(dtype)
        vn = torch.as_tensor(U.rand_storage(rng, (B, Hkv, D), dtype)).to(dtype)
        ls.n_ctx += 1
        if fused:
            ls.step_update(kn.cuda(), vn.cuda())
        else:
            ls.append(kn.cuda(), vn.cuda())
            ls.select()
            ls.encode()
        torch.cuda.synchronize()
        left = []
        for h, st in enumerate(states):
            st.append(U.to_np(kn[0, h]), U.to_np(vn[0, h]))
            st.r_size = 0
            ev_s, ev_p = st.compress()
            assert int(ls.n_evict[0, h]) == len(ev_s) == 1
            assert int(ls.evict_slot[0, h, 0]) == ev_s[0] and int(ls.evict_pos[0, h, 0]) == ev_p[0]
            compare_unit_state(ls, 0, h, st, ("n_recent=0", fused, h))
            left.append(int(ev_p[0]))
        results.append(left)
    assert results[0] == results[1]
    assert results[0][0] == n0 and results[0][1] != n0 and results[0][2] == n0


# ----------------------------------------------------------------------------- workload c2
def test_c2_all_units_follow_the_oracle(kvr, LayerState):
    """The Llama-3-8B-shaped layer as named: batch 8, 32 q / 8 kv heads, context 2048, bf16,
    10 % budget (186 retained tokens, a 3 x 6 sketch that holds 1862 tokens: the worst-conditioned
    case, 310 tokens per slot), x8 outlier channels, 16 needles.  All 64 units: prompt compression
    by the library (selection fed with the oracle's prompt scores so that the partition is
    comparable bit for bit), then decode steps through the fused update on the GPU's own state."""
    wl = S.WORKLOADS["c2"]
    layer, nsteps = 0, 6
    B, Hkv, G, N = wl.batch, wl.n_kv_heads, wl.group, wl.context
    units = [(b, h) for b in range(B) for h in range(Hkv)]
    say("c2: oracle prompt states of", len(units), "units")
    dense = U.oracle_units_from_workload(wl, layer, units, compress=False, extra_tokens=nsteps + 2)
    params = dense[0].params
    d = kvr.make_desc(B, wl.n_q_heads, Hkv, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    assert (wl.r, wl.w, wl.n_retained, wl.n_vague0) == (3, 6, 186, 1862)
    scale = d.softmax_scale
    K, V = S.kv_layer(wl, layer)
    q0 = S.queries(wl, layer, 0)
    sc0 = np.stack([s.scores[:N] for s in dense]).reshape(B, Hkv, N)
    ls, _ = LayerState.from_prefill(d, K.cuda(), V.cuda(), q0.cuda(), n_recent=wl.n_recent,
                                    k_candidate=wl.n_candidate, max_new_tokens=nsteps + 2,
                                    init_scores=torch.as_tensor(sc0).cuda())
    torch.cuda.synchronize()
    states = []
    for u, (b, h) in enumerate(units):
        st = dense[u]
        st.compress()
        st = O.compact(st, wl.n_retained + 1)
        compare_unit_state(ls, b, h, st, ("c2 prompt", u))
        states.append(st)
    say("c2: prompt partition and sketch of all units bit-exact")
    for t in range(nsteps):
        sc = np.stack([s.scores for s in states]).reshape(B, Hkv, -1)
        ls.scores.copy_(torch.as_tensor(sc).cuda())            # the float state; the rest is the GPU's own
        kn, vn = S.new_tokens(wl, layer, t)
        q = S.queries(wl, layer, t + 1)
        out = ls.decode_step(kn.cuda(), vn.cuda(), q.cuda(), check=True)
        torch.cuda.synchronize()
        og = out.cpu().double().numpy()
        worst_o = worst_s = 0.0
        big = 0.0
        for u, (b, h) in enumerate(units):
            st = states[u]
            o_ref, (ws_, wp_), _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]), U.to_np(q[b, h * G:(h + 1) * G]),
                                                  scale)
            assert int(ls.n_evict[b, h]) == len(ws_) == 1
            assert int(ls.evict_slot[b, h, 0]) == ws_[0] and int(ls.evict_pos[b, h, 0]) == wp_[0]
            compare_unit_state(ls, b, h, st, ("c2 step", t, u))
            worst_o = max(worst_o, np.abs(og[b, h * G:(h + 1) * G] - o_ref).max())
            big = max(big, np.abs(o_ref).max())
            worst_s = max(worst_s, np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max())
        say("c2 step", t, ": max |out - oracle| =", worst_o, "(max |out| =", big, ") max |score - oracle| =", worst_s)
        assert worst_o <= 2e-2 and worst_s <= 2e-5


# ----------------------------------------------------------------------------- entirely on its own state
@pytest.mark.parametrize("name,nsteps", [("c1", 32), ("tiny_bf16", 64)])
def test_many_steps_entirely_on_the_gpus_own_state(kvr, LayerState, name, nsteps):
    """After the prompt nothing is re-loaded from the oracle, not even the float scores: the library
    runs nsteps decode steps on what it computed itself, the oracle runs beside it, and every step's
    eviction, the whole integer state and the sketch must still agree bit for bit, outputs and scores
    within tolerance.  (The other step tests re-load the scores so that one step's float rounding
    cannot decide a later step's integer choice; on these seeded inputs it never does.)"""
    if name == "c1":
        wl = S.WORKLOADS["c1"]
    else:
        wl = S.small_workload(batch=2, n_q_heads=8, n_kv_heads=2, context=700, budget=0.25, r=3, steps=nsteps)
    say("own state", name, nsteps, "steps")
    layer = 0
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, extra_tokens=nsteps + 2)
    params = states[0].params
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    G, scale = wl.group, d.softmax_scale
    ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads,
                                   vague_cap=wl.n_vague0 + nsteps + 2)
    worst_o = worst_s = 0.0
    for t in range(nsteps):
        kn, vn = S.new_tokens(wl, layer, t)
        q = S.queries(wl, layer, t + 1)
        out = ls.decode_step(kn.cuda(), vn.cuda(), q.cuda(), check=True)
        torch.cuda.synchronize()
        og = out.cpu().double().numpy()
        for u, (b, h) in enumerate(units):
            st = states[u]
            o_ref, (ws_, wp_), _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]), U.to_np(q[b, h * G:(h + 1) * G]),
                                                  scale)
            assert int(ls.n_evict[b, h]) == 1 and int(ls.evict_pos[b, h, 0]) == int(wp_[0]), (t, u)
            if t % 8 == 7 or t == nsteps - 1:
                compare_unit_state(ls, b, h, st, ("own state", t, u))
            err = np.abs(og[b, h * G:(h + 1) * G] - o_ref).max()
            if wl.torch_dtype == torch.float32:
                err = err / max(np.abs(o_ref).max(), 1e-30)
            worst_o = max(worst_o, err)
            worst_s = max(worst_s, np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max())
    say("own state", name, ": max out error", worst_o, "max score error", worst_s)
    assert worst_o <= (1e-5 if wl.torch_dtype == torch.float32 else 2e-2)
    assert worst_s <= 2e-5
