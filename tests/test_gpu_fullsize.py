"""Parity at the benchmark's full size and launch configuration (workload c4: one
layer, 16 sequences x 8 kv heads, 32768-token prompt, fused update call, retained
and sketch kernels side by side).

The oracle needs seconds per unit at this size, so it follows a few sampled
units exactly; every other unit is covered by properties that hold at any
size: the partition of positions, the evicted token being a lowest-score
candidate, and the attention output against the library's own dense path over
kvr_reconstruct's output (which the sampled units tie to the oracle)."""
import numpy as np
import pytest
import torch

import kvr_synth as S
from oracle import kvr_oracle as O
from tests import util as U

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(600)]

SAMPLED = [(0, 0), (6, 3), (15, 7)]
NSTEPS = 2


def say(*a):
    print("[case]", *a, flush=True)


def upload_unit(ls, b, h, st):
    dt = ls.dtype
    ls.k_ret[b, h].copy_(U.to_dev(st.K_ret, dt))
    ls.v_ret[b, h].copy_(U.to_dev(st.V_ret, dt))
    ls.ret_pos[b, h].copy_(torch.as_tensor(st.ret_pos.astype(np.int32)).cuda())
    ls.scores[b, h].copy_(torch.as_tensor(st.scores.astype(np.float32)).cuda())
    ls.sketch_k[b, h].copy_(U.to_dev(st.SK, dt))
    ls.sketch_v[b, h].copy_(U.to_dev(st.SV, dt))
    nv = len(st.vague_pos)
    ls.vague_pos[b, h, :nv].copy_(torch.as_tensor(np.asarray(st.vague_pos, dtype=np.int32)).cuda())
    ls.n_vague[b, h] = nv


def test_c4_layer_in_bench_configuration():
    from paper_2512_17917_amd import binding as kvr
    from paper_2512_17917_amd.state import LayerState

    wl = S.WORKLOADS["c4"]
    layer = 0
    dev = torch.device("cuda:0")
    B, Hkv, Hq, D, G, N = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.group, wl.context
    R = wl.n_retained
    say("full size: oracle prompt state of", SAMPLED)
    states = U.oracle_units_from_workload(wl, layer, SAMPLED, extra_tokens=NSTEPS)
    params = states[0].params
    assert kvr.kvr_hash_params_from_seed(S.BASE_SEED + layer, wl.r) == params
    d = kvr.make_desc(B, Hq, Hkv, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    scale = d.softmax_scale

    say("full size: prompt compression on the GPU, all", B * Hkv, "units")
    Kf, Vf = S.kv_layer(wl, layer, device=dev)
    qall = S.queries_many(wl, layer, 0, NSTEPS + 1, device=dev)
    ls, _ = LayerState.from_prefill(d, Kf, Vf, qall[0].contiguous(), n_recent=wl.n_recent,
                                    k_candidate=wl.n_candidate, max_new_tokens=NSTEPS, side=kvr.SideStream(dev))
    torch.cuda.synchronize()
    del Kf, Vf
    assert ls.ret_cap == R + 1 and int(ls.n_evict.min()) == int(ls.n_evict.max()) == wl.n_vague0
    # the GPU's own prompt state of the sampled units.  Its selection ran on its own
    # float32 scores, so two tokens whose scores tie to the last bits may swap sides
    # of the Candidate boundary; everything else must be the oracle's partition.
    for (b, h), st in zip(SAMPLED, states):
        assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores).max() <= 2e-5
        mine = set(ls.ret_pos[b, h].cpu().numpy().tolist()) - {-1}
        theirs = set(st.ret_pos.tolist()) - {-1}
        assert len(mine) == len(theirs) == R
        swapped = mine ^ theirs
        say("full size: unit", (b, h), "prompt partition differs from the oracle's in", len(swapped), "positions")
        assert len(swapped) <= 8
        if swapped:
            sc = st.scores[sorted(swapped)]
            assert sc.max() - sc.min() <= 1e-6 * max(sc.max(), 1e-30) + 1e-9

    kn_all, vn_all = S.kv_layer(wl, layer, N, N + NSTEPS, device=dev)          # [B, Hkv, T, D]
    for t in range(NSTEPS):
        say("full size: decode step", t)
        # the sampled units start from the oracle's prompt state; from then on they keep their own
        # keys, values, sketch and lists, and only the float scores are re-loaded from the oracle
        for (b, h), st in zip(SAMPLED, states):
            if t == 0:
                upload_unit(ls, b, h, st)
            else:
                ls.scores[b, h].copy_(torch.as_tensor(st.scores.astype(np.float32)).cuda())
        kn, vn = kn_all[:, :, t].contiguous(), vn_all[:, :, t].contiguous()
        q = qall[t + 1].contiguous()
        scores_before = ls.scores.clone()
        ret_before = ls.ret_pos.clone()
        nv_before = ls.n_vague.clone()
        out = ls.decode_step(kn, vn, q).clone()                # fused update, as the benchmark runs it
        torch.cuda.synchronize()
        n_ctx = N + t + 1
        assert int(ls.n_ctx.min()) == int(ls.n_ctx.max()) == n_ctx

        # ---- sampled units against the oracle --------------------------------
        for (b, h), st in zip(SAMPLED, states):
            o_ref, (ws_, wp_), _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]),
                                                  U.to_np(q[b, h * G:(h + 1) * G]), scale)
            assert int(ls.n_evict[b, h]) == len(ws_) == 1
            assert ls.evict_slot[b, h, 0].item() == ws_[0] and ls.evict_pos[b, h, 0].item() == wp_[0]
            assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
            nv = int(ls.n_vague[b, h])
            assert nv == len(st.vague_pos)
            assert np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
            assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK)
            assert np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
            assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret)
            assert np.array_equal(U.to_np(ls.v_ret[b, h]), st.V_ret)
            og = out[b, h * G:(h + 1) * G].cpu().double().numpy()
            assert np.abs(og - o_ref).max() <= 2e-2
            assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max() <= 2e-5

        # ---- every unit: bookkeeping properties ------------------------------
        assert int(ls.n_evict.min()) == int(ls.n_evict.max()) == 1
        assert torch.equal(ls.n_vague, nv_before + 1)
        cnt = torch.zeros(B, Hkv, n_ctx + 1, dtype=torch.int32, device=dev)
        rp = ls.ret_pos.long()
        cnt.scatter_add_(2, torch.where(rp >= 0, rp, torch.full_like(rp, n_ctx)),
                         torch.ones_like(rp, dtype=torch.int32))
        nv = int(ls.n_vague.max())
        vp = ls.vague_pos[:, :, :nv].long()
        live = torch.arange(nv, device=dev).view(1, 1, nv) < ls.n_vague.unsqueeze(-1)
        cnt.scatter_add_(2, torch.where(live, vp, torch.full_like(vp, n_ctx)), torch.ones_like(vp, dtype=torch.int32))
        assert bool((cnt[:, :, :n_ctx] == 1).all()), "retained + Vague positions are not a partition of the context"
        # the evicted token: outside the Recent window, and no candidate scored lower
        ep = ls.evict_pos[:, :, 0].long()
        assert bool((ep < n_ctx - wl.n_recent).all()) and bool((ep >= 0).all())
        was = ret_before.long()
        cand = (was >= 0) & (was < n_ctx - wl.n_recent)
        sc_slot = scores_before.gather(2, was.clamp(min=0))
        lowest = torch.where(cand, sc_slot, torch.full_like(sc_slot, float("inf"))).amin(dim=2)
        assert torch.equal(scores_before.gather(2, ep.unsqueeze(-1)).squeeze(-1), lowest)
        # the evicted slot was released (or reused by nothing): its position left the retained set
        assert bool((ls.ret_pos.gather(2, ls.evict_slot[:, :, :1].long()).squeeze(-1) == -1).all())

        # ---- every unit: attention output against dense attention over the
        #      library's reconstruction (tied to the oracle on the sampled units)
        kh = torch.zeros(B, Hkv, nv, D, dtype=ls.dtype, device=dev)
        vh = torch.zeros_like(kh)
        kvr.kvr_reconstruct(d, ls.sketch_k, ls.sketch_v, ls.vague_pos[:, :, :nv].contiguous(), ls.n_vague, nv, kh, vh)
        torch.cuda.synchronize()
        for (b, h), st in zip(SAMPLED, states):
            Kq, Vq = O.query(st.SK, st.SV, params, list(st.vague_pos), storage="bf16")
            assert np.array_equal(U.to_np(kh[b, h, :len(st.vague_pos)]), Kq)
            assert np.array_equal(U.to_np(vh[b, h, :len(st.vague_pos)]), Vq)
        Kall = torch.cat([ls.k_ret, kh], dim=2).double()
        Vall = torch.cat([ls.v_ret, vh], dim=2).double()
        valid = torch.cat([ls.ret_pos >= 0, live], dim=2)                                  # [B, Hkv, n]
        qf = q.double().view(B, Hkv, G, D)
        logit = torch.einsum("bhgd,bhnd->bhgn", qf, Kall) * scale
        logit = logit.masked_fill(~valid.unsqueeze(2), float("-inf"))
        ref = torch.einsum("bhgn,bhnd->bhgd", torch.softmax(logit, dim=-1), Vall).reshape(B, Hq, D)
        err = (out.double() - ref).abs().max().item()
        big = ref.abs().max().item()
        say("full size: max |out - dense over reconstruction| =", err, " max |out| =", big)
        assert err <= 2e-5 * big
        del Kall, Vall, logit, kh, vh

    # ---- swap loop (Algorithm 3) at this size: the natural state after two steps,
    #      then with a few Vague scores of the sampled units raised so that they swap
    say("full size: swap loop")
    MAXSW = 4
    rng = np.random.default_rng(4)
    for (b, h), st in zip(SAMPLED, states):
        cand = [int(p) for p in st.ret_pos if 0 <= p < st.n_ctx - st.n_recent]
        top = float(st.scores[cand].max())
        for n, i in enumerate(rng.choice(len(st.vague_pos), size=3, replace=False)):
            st.scores[st.vague_pos[i]] = np.float32(top * (2 + n // 2))
        upload_unit(ls, b, h, st)
    n_sw = torch.full((B, Hkv), -1, dtype=torch.int32, device=dev)
    log = torch.full((B, Hkv, MAXSW, 2), -1, dtype=torch.int32, device=dev)
    sk_before = ls.sketch_k.clone()
    ls.swap_back(1.1, MAXSW, n_sw, log)
    torch.cuda.synchronize()
    for (b, h), st in zip(SAMPLED, states):
        done = st.swap_back(1.1, MAXSW)
        assert len(done) >= 3 and int(n_sw[b, h]) == len(done)
        assert [tuple(x) for x in log[b, h, :len(done)].cpu().tolist()] == done
        assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
        nv = int(ls.n_vague[b, h])
        assert np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
        assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK) and np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
        assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret) and np.array_equal(U.to_np(ls.v_ret[b, h]), st.V_ret)
    # every unit: counts in range, still a partition, and where the loop stopped by
    # itself its exit condition holds: min Candidate score * 1.1 >= max Vague score (float32)
    assert int(n_sw.min()) >= 0 and int(n_sw.max()) <= MAXSW
    n_ctx = N + NSTEPS
    cnt = torch.zeros(B, Hkv, n_ctx + 1, dtype=torch.int32, device=dev)
    rp = ls.ret_pos.long()
    cnt.scatter_add_(2, torch.where(rp >= 0, rp, torch.full_like(rp, n_ctx)), torch.ones_like(rp, dtype=torch.int32))
    nv = int(ls.n_vague.max())
    vp = ls.vague_pos[:, :, :nv].long()
    live = torch.arange(nv, device=dev).view(1, 1, nv) < ls.n_vague.unsqueeze(-1)
    cnt.scatter_add_(2, torch.where(live, vp, torch.full_like(vp, n_ctx)), torch.ones_like(vp, dtype=torch.int32))
    assert bool((cnt[:, :, :n_ctx] == 1).all())
    cand = (rp >= 0) & (rp < n_ctx - wl.n_recent)
    sc_c = ls.scores.gather(2, rp.clamp(min=0))
    cmin = torch.where(cand, sc_c, torch.full_like(sc_c, float("inf"))).amin(dim=2)
    sc_v = ls.scores.gather(2, vp)
    vmax = torch.where(live, sc_v, torch.full_like(sc_v, float("-inf"))).amax(dim=2)
    stopped = n_sw < MAXSW
    assert bool(((cmin * torch.tensor(1.1, dtype=torch.float32, device=dev) >= vmax) | ~stopped).all())
    untouched = n_sw == 0
    assert bool((ls.sketch_k == sk_before)[untouched].all())
    say("full size: swaps per unit: min", int(n_sw.min()), "max", int(n_sw.max()), "mean", float(n_sw.float().mean()))

    # ---- several queries at once (kvr_attend_multi) on this state: the four newest tokens are the
    #      queries' own positions.  Sampled units against the oracle; every unit against dense causal
    #      attention over the library's reconstruction.
    say("full size: attend_multi, 4 queries")
    NQ = 4
    qm = S.queries_many(wl, layer, 10, NQ, device=dev).transpose(0, 1).contiguous()        # [B, NQ, Hq, D]
    scores_before = ls.scores.clone()
    outm = ls.attend_multi(qm, NQ).clone()
    torch.cuda.synchronize()
    q_pos = np.arange(n_ctx - NQ, n_ctx)
    for (b, h), st in zip(SAMPLED, states):
        qq = U.to_np(qm[b, :, h * G:(h + 1) * G])
        o_ref, sc_ref, _ = O.attend_multi(qq, q_pos, st.K_ret, st.V_ret, st.ret_pos, st.SK, st.SV, params,
                                          st.vague_pos, st.n_ctx, scale, scores=st.scores, storage="bf16")
        assert np.abs(outm[b, :, h * G:(h + 1) * G].cpu().double().numpy() - o_ref).max() <= 2e-2
        assert np.abs(ls.scores[b, h].cpu().double().numpy() - sc_ref.astype(np.float64)).max() <= 2e-5 * NQ
    nv = int(ls.n_vague.max())
    kh = torch.zeros(B, Hkv, nv, D, dtype=ls.dtype, device=dev)
    vh = torch.zeros_like(kh)
    kvr.kvr_reconstruct(d, ls.sketch_k, ls.sketch_v, ls.vague_pos[:, :, :nv].contiguous(), ls.n_vague, nv, kh, vh)
    live = torch.arange(nv, device=dev).view(1, 1, nv) < ls.n_vague.unsqueeze(-1)
    pos_all = torch.cat([ls.ret_pos, torch.where(live, ls.vague_pos[:, :, :nv], torch.full_like(ls.vague_pos[:, :, :nv], -1))],
                        dim=2).long()                                                          # [B, Hkv, n]
    Kall = torch.cat([ls.k_ret, kh], dim=2).double()
    Vall = torch.cat([ls.v_ret, vh], dim=2).double()
    inc = torch.zeros(B, Hkv, pos_all.shape[2], dtype=torch.float64, device=dev)
    worst = 0.0
    for t in range(NQ):
        qf = qm[:, t].double().view(B, Hkv, G, D)
        logit = torch.einsum("bhgd,bhnd->bhgn", qf, Kall) * scale
        seen = (pos_all >= 0) & (pos_all <= n_ctx - NQ + t)
        logit = logit.masked_fill(~seen.unsqueeze(2), float("-inf"))
        pr = torch.softmax(logit, dim=-1)
        ref = torch.einsum("bhgn,bhnd->bhgd", pr, Vall).reshape(B, Hq, D)
        worst = max(worst, ((outm[:, t].double() - ref).abs().max() / ref.abs().max()).item())
        inc += pr.sum(dim=2)
    say("full size: attend_multi max relative |out - dense over reconstruction| =", worst)
    assert worst <= 3e-5
    got_inc = (ls.scores.double() - scores_before.double()).gather(2, pos_all.clamp(min=0))
    got_inc = torch.where(pos_all >= 0, got_inc, torch.zeros_like(got_inc))
    assert (got_inc - inc).abs().max().item() <= 2e-5 * NQ


def upload_scores(ls, b, h, st):
    ls.scores[b, h].copy_(torch.as_tensor(st.scores.astype(np.float32)).cuda())


@pytest.mark.parametrize("name,layer,sampled", [("c3", 0, [(0, 1), (0, 6)]), ("c3", 35, [(0, 0), (0, 5)]),
                                                ("c5", 0, [(0, 2), (3, 5)]), ("c5", 35, [(1, 2), (2, 7)])])
def test_other_workloads_sampled(name, layer, sampled):
    """The first and the last layer of the batch-1 32k workload (few units: the kernels run back
    to back, the Vague list is cut into many short workgroups) and of the 131k / r = 4 workload
    (general staged kernel, 16-channel chunks, mean-of-middle-two median, selection with keys
    re-read from memory) at full shape: prompt compression and two decode steps.  Two sampled units
    per layer (two heads; two sequences where the batch has them) against the oracle -- from the
    first step on they run on the GPU's own keys, values, sketch and lists, only the float scores
    are re-loaded from the oracle -- and all units by bookkeeping."""
    from paper_2512_17917_amd import binding as kvr
    from paper_2512_17917_amd.state import LayerState

    NST = 2
    wl = S.WORKLOADS[name]
    dev = torch.device("cuda:0")
    B, Hkv, Hq, D, G, N = wl.batch, wl.n_kv_heads, wl.n_q_heads, wl.head_dim, wl.group, wl.context
    say("full size", name, "layer", layer, ": oracle prompt state of", sampled)
    states = U.oracle_units_from_workload(wl, layer, sampled, extra_tokens=NST)
    params = states[0].params
    d = kvr.make_desc(B, Hq, Hkv, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    say("full size", name, ": prompt compression on the GPU")
    Kf, Vf = S.kv_layer(wl, layer, device=dev)
    qall = S.queries_many(wl, layer, 0, NST + 1, device=dev)
    ls, _ = LayerState.from_prefill(d, Kf, Vf, qall[0].contiguous(), n_recent=wl.n_recent,
                                    k_candidate=wl.n_candidate, max_new_tokens=NST, side=kvr.SideStream(dev))
    torch.cuda.synchronize()
    del Kf, Vf
    assert int(ls.n_evict.min()) == int(ls.n_evict.max()) == wl.n_vague0
    for (b, h), st in zip(sampled, states):
        assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores).max() <= 2e-5
        mine = set(ls.ret_pos[b, h].cpu().numpy().tolist()) - {-1}
        theirs = set(st.ret_pos.tolist()) - {-1}
        say("full size", name, "unit", (b, h), ": prompt partition differs from the oracle's in", len(mine ^ theirs),
            "positions")
        assert len(mine) == len(theirs) == wl.n_retained and len(mine ^ theirs) <= 8
        upload_unit(ls, b, h, st)
    kn_all, vn_all = S.kv_layer(wl, layer, N, N + NST, device=dev)
    for t in range(NST):
        kn, vn = kn_all[:, :, t].contiguous(), vn_all[:, :, t].contiguous()
        q = qall[t + 1].contiguous()
        if t > 0:
            for (b, h), st in zip(sampled, states):
                upload_scores(ls, b, h, st)
        say("full size", name, ": decode step", t)
        out = ls.decode_step(kn, vn, q, check=True).clone()
        torch.cuda.synchronize()
        for (b, h), st in zip(sampled, states):
            o_ref, (ws_, wp_), _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]), U.to_np(q[b, h * G:(h + 1) * G]),
                                                  d.softmax_scale)
            assert int(ls.n_evict[b, h]) == len(ws_) == 1
            assert ls.evict_slot[b, h, 0].item() == ws_[0] and ls.evict_pos[b, h, 0].item() == wp_[0]
            assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
            nv = int(ls.n_vague[b, h])
            assert nv == len(st.vague_pos) and np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
            assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK) and np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
            assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret) and np.array_equal(U.to_np(ls.v_ret[b, h]), st.V_ret)
            err = np.abs(out[b, h * G:(h + 1) * G].cpu().double().numpy() - o_ref).max()
            say("full size", name, "layer", layer, "step", t, "unit", (b, h), "max |out - oracle| =", err)
            assert err <= 2e-2
            assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max() <= 2e-5
        # every unit: one eviction, still a partition of the context
        n_ctx = N + t + 1
        assert int(ls.n_evict.min()) == int(ls.n_evict.max()) == 1
        cnt = torch.zeros(B, Hkv, n_ctx + 1, dtype=torch.int32, device=dev)
        rp = ls.ret_pos.long()
        cnt.scatter_add_(2, torch.where(rp >= 0, rp, torch.full_like(rp, n_ctx)), torch.ones_like(rp, dtype=torch.int32))
        nv = int(ls.n_vague.max())
        vp = ls.vague_pos[:, :, :nv].long()
        live = torch.arange(nv, device=dev).view(1, 1, nv) < ls.n_vague.unsqueeze(-1)
        cnt.scatter_add_(2, torch.where(live, vp, torch.full_like(vp, n_ctx)), torch.ones_like(vp, dtype=torch.int32))
        assert bool((cnt[:, :, :n_ctx] == 1).all())
        assert bool(torch.isfinite(out).all())
