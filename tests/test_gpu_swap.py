"""GPU parity of kvr_swap_back (swap loop of Algorithm 3) against the CPU oracle.
Everything it produces is an index, a stored value or a count, so everything
must match bit for bit: which tokens are exchanged and in which order, the
sketch after delete + insert, the estimate written into the Candidate's slot,
ret_pos, vague_pos and the swap count.  One decode-step test checks the
attention output after swaps within the usual float tolerance."""
import numpy as np
import pytest
import torch

import kvr_synth as S
from oracle import kvr_oracle as O
from tests import util as U
from tests.test_gpu_parity import check_out, say

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


def doctor_scores(states, rng):
    """Give the units different swap workloads: unit 0 untouched (its Vague scores
    are below every Candidate's: no swap), the others get some Vague scores
    raised above Candidate scores, with exact ties among them and among the
    lowest Candidates."""
    for u, st in enumerate(states):
        if u == 0:
            continue
        cand = [int(p) for p in st.ret_pos if 0 <= p < st.n_ctx - st.n_recent]
        top = float(max(st.scores[cand]))
        vp = st.vague_pos
        picks = rng.choice(len(vp), size=min(2 + 2 * u, len(vp)), replace=False)
        for n, i in enumerate(picks):
            # pairs of equal scores above the Candidates' range; later units get more of them
            st.scores[vp[i]] = np.float32(top * (2.0 + (n // 2)))
        low = sorted(cand, key=lambda p: float(st.scores[p]))[:3]
        st.scores[low] = st.scores[low[0]]                    # three-way tie for the Candidate minimum


def run_swap_case(kvr, LayerState, wl, layer, rate, max_swaps, rng, sign_mask=2, median_mode=0, vague_cap=None):
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, extra_tokens=4)
    for st in states:
        st.sign_mask = sign_mask
        st.median_mode = "lower" if median_mode else "midmean"
    if sign_mask != 2:
        # the prompt was inserted with the default sign setting: rebuild the sketches
        for st in states:
            vp = st.vague_pos
            K, V = S.kv_unit(wl, layer, *units[states.index(st)])
            K, V = U.to_np(K), U.to_np(V)
            st.SK, st.SV = O.sketch_zeros(wl.r, wl.w, wl.head_dim)
            st.SK, st.SV = O.insert(st.SK, st.SV, st.params, vp, K[vp], V[vp], storage=wl.dtype,
                                    acc_dtype=np.float32, sign_mask=sign_mask)
    doctor_scores(states, rng)
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype,
                      hash_params=states[0].params, sign_mask=sign_mask, median_mode=median_mode)
    ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads,
                                   vague_cap=vague_cap or wl.n_vague0 + 4)
    n_sw = torch.full((wl.batch, wl.n_kv_heads), -7, dtype=torch.int32, device="cuda")
    log = torch.full((wl.batch, wl.n_kv_heads, max(max_swaps, 1), 2), -1, dtype=torch.int32, device="cuda")
    ls.swap_back(rate, max_swaps, n_sw, log)
    torch.cuda.synchronize()
    n_sw, log = n_sw.cpu().numpy().reshape(-1), log.cpu().numpy().reshape(len(units), -1, 2)
    total = 0
    for u, (b, h) in enumerate(units):
        st = states[u]
        done = st.swap_back(rate, max_swaps)
        total += len(done)
        assert n_sw[u] == len(done), (u, n_sw[u], len(done))
        assert [tuple(x) for x in log[u, :len(done)].tolist()] == done
        assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
        nv = int(ls.n_vague[b, h])
        assert nv == len(st.vague_pos) and np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
        assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK) and np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
        assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret) and np.array_equal(U.to_np(ls.v_ret[b, h]), st.V_ret)
    return total, n_sw


@pytest.mark.parametrize("max_swaps", [0, 1, 16])
def test_swap_back_bf16_r3(kvr, LayerState, max_swaps):
    say("swap bf16 r3", max_swaps)
    wl = S.small_workload("swp", batch=2, n_q_heads=8, n_kv_heads=2, context=700, budget=0.25, r=3, steps=2,
                          cfg_id=96)
    total, n_sw = run_swap_case(kvr, LayerState, wl, 0, 1.1, max_swaps, np.random.default_rng(5))
    assert n_sw[0] == 0
    if max_swaps == 1:
        assert list(n_sw[1:]) == [1, 1, 1]
    if max_swaps == 16:
        assert total >= 9 and len(set(n_sw.tolist())) >= 3       # units did different numbers of swaps


def test_swap_back_keys_from_memory_and_more_swaps_than_one_scan(kvr, LayerState):
    """A Vague list capacity beyond what the kernel keeps in registers (26 keys per
    thread) takes the path that re-reads keys from memory; 40 allowed swaps need
    more than one scan (a scan serves 16)."""
    say("swap, memory path / several scans")
    rng = np.random.default_rng(8)
    wl = S.small_workload("swpm", batch=1, n_q_heads=4, n_kv_heads=2, context=1200, budget=0.25, r=3, steps=2,
                          cfg_id=87)
    total, _ = run_swap_case(kvr, LayerState, wl, 0, 1.1, 8, rng, vague_cap=27000)
    assert total >= 2

    def many(states, rng_):
        for st in states:
            cand = [int(p) for p in st.ret_pos if 0 <= p < st.n_ctx - st.n_recent]
            top = float(max(st.scores[cand]))
            for n, i in enumerate(rng_.choice(len(st.vague_pos), size=30, replace=False)):
                st.scores[st.vague_pos[i]] = np.float32(top * (2.0 + n))
    global doctor_scores
    saved = doctor_scores
    doctor_scores = many
    try:
        total, n_sw = run_swap_case(kvr, LayerState, wl, 0, 1.1, 40, rng)
    finally:
        doctor_scores = saved
    assert n_sw.min() >= 30 and n_sw.max() <= 40


def test_swap_back_f32_and_even_rows_and_signed_keys(kvr, LayerState):
    say("swap f32 / r4 / sign_mask 3")
    rng = np.random.default_rng(6)
    wl = S.small_workload("swpf", batch=1, n_q_heads=2, n_kv_heads=2, context=500, budget=0.3, r=3, steps=2,
                          cfg_id=95, dtype="f32")
    total, _ = run_swap_case(kvr, LayerState, wl, 0, 1.0, 8, rng)
    assert total >= 2
    wl4 = S.small_workload("swp4", batch=1, n_q_heads=4, n_kv_heads=2, context=900, budget=0.3, r=4, steps=2,
                           cfg_id=94)
    for mode in (0, 1):
        total, _ = run_swap_case(kvr, LayerState, wl4, 1, 1.5, 8, rng, median_mode=mode)
        assert total >= 2
    total, _ = run_swap_case(kvr, LayerState, wl4, 2, 1.1, 8, rng, sign_mask=3)
    assert total >= 2


def test_decode_steps_with_swaps_follow_the_oracle(kvr, LayerState):
    """append -> select -> insert -> swap loop -> attend, three steps; the state is
    reloaded from the oracle before every step."""
    say("decode steps with swaps")
    wl = S.small_workload("swpd", batch=2, n_q_heads=8, n_kv_heads=2, context=700, budget=0.25, r=3, steps=4,
                          cfg_id=93)
    layer, nsteps = 0, 3
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, extra_tokens=nsteps + 2)
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype,
                      hash_params=states[0].params)
    G, scale = wl.group, d.softmax_scale
    swaps_seen = 0
    for t in range(nsteps):
        ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads,
                                       vague_cap=wl.n_vague0 + nsteps + 2)
        kn, vn = S.new_tokens(wl, layer, t)
        q = S.queries(wl, layer, t + 1)
        out = ls.decode_step(kn.cuda(), vn.cuda(), q.cuda(), replace_rate=1.1, max_swaps=4)
        torch.cuda.synchronize()
        og = out.cpu().double().numpy()
        for u, (b, h) in enumerate(units):
            st = states[u]
            before = list(st.vague_pos)
            o_ref, _, _ = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]), U.to_np(q[b, h * G:(h + 1) * G]),
                                         scale, replace_rate=1.1, max_swaps=4)
            swaps_seen += len(set(before) - set(st.vague_pos))
            assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
            nv = int(ls.n_vague[b, h])
            assert nv == len(st.vague_pos) and np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
            assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK) and np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
            assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret)
            check_out(og[b, h * G:(h + 1) * G], o_ref, wl.torch_dtype)
            assert np.abs(ls.scores[b, h].cpu().double().numpy() - st.scores.astype(np.float64)).max() <= 2e-5
    assert swaps_seen > 0, "the workload never swapped: the test does not exercise the loop"
