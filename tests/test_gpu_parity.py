"""GPU parity: every entry point of libkvr against the CPU oracle on the same
seeded inputs.  Bucket indices, signs, selected indices, the stored sketch and
reconstructed tokens must match bit for bit; attention outputs and scores
within the stated float tolerances:
  bf16 storage: max |out_gpu - out_oracle| <= 2e-2
  f32 storage:  max |out_gpu - out_oracle| / max |out_oracle| <= 1e-5
Scores (float32 accumulators of probabilities): max abs difference <= 2e-5
(bf16) / 1e-5 (f32) per call.
"""
import math

import numpy as np
import pytest
import torch

import kvr_synth as S
from oracle import kvr_oracle as O
from tests import util as U

pytestmark = pytest.mark.gpu

TOL_OUT_BF16 = 2e-2
TOL_OUT_F32_REL = 1e-5


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


def check_out(out_gpu, out_ref, dtype):
    if dtype == torch.float32:
        err = np.abs(out_gpu - out_ref).max() / max(np.abs(out_ref).max(), 1e-30)
        assert err <= TOL_OUT_F32_REL, f"relative error {err}"
    else:
        err = np.abs(out_gpu - out_ref).max()
        assert err <= TOL_OUT_BF16, f"max abs error {err}"
    return err


# ----------------------------------------------------------------------------- reconstruct
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("r,w,mode,mask", [(3, 37, 0, 2), (1, 5, 0, 2), (2, 9, 0, 2), (2, 9, 1, 3),
                                           (4, 21, 0, 2), (4, 21, 1, 2), (5, 11, 0, 1), (8, 6, 0, 2),
                                           (6, 7, 1, 0), (3, 1, 0, 2), (4, 13, 0, 3), (4, 13, 1, 1),
                                           (3, 17, 0, 3), (3, 9, 0, 0)])
def test_reconstruct_bit_exact(kvr, dtype, r, w, mode, mask):
    say("reconstruct", dtype, r, w, mode, mask)
    rng = np.random.default_rng(100 + r * 7 + w)
    B, Hkv, cap, D = 2, 3, 301, 128
    d = kvr.make_desc(B, Hkv * 2, Hkv, r, w, dtype, seed=900 + r, sign_mask=mask, median_mode=mode)
    params = kvr.desc_hash_params(d)
    SK = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 3.0)
    SV = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 3.0)
    pos = rng.integers(0, 200000, size=(B, Hkv, cap)).astype(np.int32)
    count = np.array([[301, 0, 64], [1, 300, 17]], dtype=np.int32)
    k_out = torch.full((B, Hkv, cap, D), 7.0, dtype=dtype, device="cuda")
    v_out = torch.full((B, Hkv, cap, D), 7.0, dtype=dtype, device="cuda")
    kvr.kvr_reconstruct(d, U.to_dev(SK, dtype), U.to_dev(SV, dtype), torch.as_tensor(pos).cuda(),
                        torch.as_tensor(count).cuda(), cap, k_out, v_out)
    torch.cuda.synchronize()
    kg, vg = U.to_np(k_out), U.to_np(v_out)
    st = U.storage_name(dtype)
    for b in range(B):
        for h in range(Hkv):
            n = count[b, h]
            kr, vr = O.query(SK[b, h], SV[b, h], params, pos[b, h, :n], storage=st,
                             median_mode="lower" if mode else "midmean", sign_mask=mask)
            assert np.array_equal(kg[b, h, :n], kr), (b, h)
            assert np.array_equal(vg[b, h, :n], vr), (b, h)
            assert (kg[b, h, n:] == 7.0).all() and (vg[b, h, n:] == 7.0).all()   # rows beyond count untouched


@pytest.mark.parametrize("w,mask,B,Hkv", [(50, 2, 1, 3), (341, 3, 2, 8), (273, 0, 1, 1), (9, 1, 3, 5)])
def test_reconstruct_long_lists_through_lds(kvr, w, mask, B, Hkv):
    """bf16, three rows, a list of 4096 tokens or more: the sketch is copied into LDS chunk by chunk
    and every (unit, tensor, half row, token slice) has a workgroup of its own.  Several token tiles
    per workgroup, several slices per unit, unit counts that are no multiple of 8, a ragged last
    tile, an empty unit, every sign setting, the widest sketch the route takes (3 w = 1023 rows).
    Bit for bit against the oracle; rows beyond a unit's count stay untouched."""
    dtype = torch.bfloat16
    say("reconstruct through LDS", w, mask, B, Hkv)
    rng = np.random.default_rng(300 + w)
    cap, D = 6200, 128
    d = kvr.make_desc(B, Hkv, Hkv, 3, w, dtype, seed=910 + w, sign_mask=mask)
    params = kvr.desc_hash_params(d)
    SK = U.rand_storage(rng, (B, Hkv, 3, w, D), dtype, 3.0)
    SV = U.rand_storage(rng, (B, Hkv, 3, w, D), dtype, 3.0)
    pos = rng.integers(0, 2000000, size=(B, Hkv, cap)).astype(np.int32)
    pool = [6200, 4097, 0, 2049, 1, 6137, 64, 5000]
    count = np.array([pool[i % len(pool)] for i in range(B * Hkv)], dtype=np.int32).reshape(B, Hkv)
    k_out = torch.full((B, Hkv, cap, D), 7.0, dtype=dtype, device="cuda")
    v_out = torch.full((B, Hkv, cap, D), 7.0, dtype=dtype, device="cuda")
    kvr.kvr_reconstruct(d, U.to_dev(SK, dtype), U.to_dev(SV, dtype), torch.as_tensor(pos).cuda(),
                        torch.as_tensor(count).cuda(), cap, k_out, v_out)
    torch.cuda.synchronize()
    kg, vg = U.to_np(k_out), U.to_np(v_out)
    for b in range(B):
        for h in range(Hkv):
            n = count[b, h]
            kr, vr = O.query(SK[b, h], SV[b, h], params, pos[b, h, :n], storage="bf16", sign_mask=mask)
            assert np.array_equal(kg[b, h, :n], kr), (b, h)
            assert np.array_equal(vg[b, h, :n], vr), (b, h)
            assert (kg[b, h, n:] == 7.0).all() and (vg[b, h, n:] == 7.0).all()


# ----------------------------------------------------------------------------- encode
def run_encode_case(kvr, dtype, r, w, cap, counts, src_rows, mask, seed, preload=True, bad_slot=False):
    rng = np.random.default_rng(seed)
    B, Hkv = counts.shape
    D = 128
    d = kvr.make_desc(B, Hkv, Hkv, r, w, dtype, seed=seed, sign_mask=mask)
    params = kvr.desc_hash_params(d)
    st = U.storage_name(dtype)
    Ksrc = U.rand_storage(rng, (B, Hkv, src_rows, D), dtype)
    Vsrc = U.rand_storage(rng, (B, Hkv, src_rows, D), dtype)
    if preload:
        SK0 = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 5.0)
        SV0 = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 5.0)
    else:
        SK0 = np.zeros((B, Hkv, r, w, D))
        SV0 = np.zeros((B, Hkv, r, w, D))
    slot = rng.integers(0, src_rows, size=(B, Hkv, cap)).astype(np.int32)
    pos = np.stack([rng.choice(1 << 20, size=cap, replace=False) for _ in range(B * Hkv)]).reshape(B, Hkv, cap).astype(np.int32)
    if bad_slot:
        slot[0, 0, 1] = -5
        slot[0, 0, 2] = src_rows
    sk = U.to_dev(SK0, dtype)
    sv = U.to_dev(SV0, dtype)
    ob = torch.full((B, Hkv, cap, r), -9, dtype=torch.int32, device="cuda")
    osg = torch.full((B, Hkv, cap), 255, dtype=torch.uint8, device="cuda")
    ws = kvr.alloc_workspace(d, kvr.KVR_OP_ENCODE, cap)
    kvr.kvr_encode(d, U.to_dev(Ksrc, dtype), U.to_dev(Vsrc, dtype), src_rows, torch.as_tensor(slot).cuda(),
                   torch.as_tensor(pos).cuda(), torch.as_tensor(counts.astype(np.int32)).cuda(), cap, sk, sv,
                   ob, osg, ws)
    torch.cuda.synchronize()
    skg, svg = U.to_np(sk), U.to_np(sv)
    obg, osgg = ob.cpu().numpy(), osg.cpu().numpy()
    for b in range(B):
        for h in range(Hkv):
            n = max(0, min(int(counts[b, h]), cap))
            ok = [e for e in range(n) if 0 <= slot[b, h, e] < src_rows]
            SKr, SVr = O.insert(SK0[b, h], SV0[b, h], params, pos[b, h, ok], Ksrc[b, h][slot[b, h, ok]],
                                Vsrc[b, h][slot[b, h, ok]], storage=st, acc_dtype=np.float32, sign_mask=mask)
            assert np.array_equal(skg[b, h], SKr), ("sketch_k", b, h)
            assert np.array_equal(svg[b, h], SVr), ("sketch_v", b, h)
            for e in range(n):
                J = int(pos[b, h, e])
                assert obg[b, h, e].tolist() == [O.bucket_of(params[i], J, w) for i in range(r)]
                bits = sum((1 << i) for i in range(r) if O.sign_of(params[i], J) < 0)
                assert osgg[b, h, e] == bits
            assert (obg[b, h, n:] == -9).all() and (osgg[b, h, n:] == 255).all()


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_encode_small_path_bit_exact(kvr, dtype):
    say("encode small", dtype)
    # heavy collisions (w = 2) so that several listed tokens share a slot and the
    # "one rounding per slot per call" rule matters
    run_encode_case(kvr, dtype, 3, 2, 8, np.array([[8, 1, 0], [5, -3, 99]]), 20, 2, 11)
    run_encode_case(kvr, dtype, 4, 13, 64, np.array([[64, 33]]), 70, 3, 12, bad_slot=True)
    run_encode_case(kvr, dtype, 1, 1, 7, np.array([[7]]), 9, 0, 13, preload=False)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_encode_bulk_path_bit_exact(kvr, dtype):
    say("encode bulk", dtype)
    run_encode_case(kvr, dtype, 3, 29, 700, np.array([[700, 65, 0], [1, 333, 699]]), 512, 2, 21)
    run_encode_case(kvr, dtype, 4, 3, 300, np.array([[300, 250]]), 300, 2, 22, bad_slot=True)
    run_encode_case(kvr, dtype, 2, 257, 129, np.array([[129]]), 64, 1, 23, preload=False)


def test_encode_is_deterministic_and_linear_on_exact_data(kvr):
    say("encode determinism")
    rng = np.random.default_rng(5)
    B, Hkv, r, w, cap, D = 1, 2, 3, 17, 400, 128
    dtype = torch.float32
    d = kvr.make_desc(B, Hkv, Hkv, r, w, dtype, seed=3)
    K = rng.integers(-8, 9, size=(B, Hkv, cap, D)).astype(np.float64)
    V = rng.integers(-8, 9, size=(B, Hkv, cap, D)).astype(np.float64)
    slot = np.tile(np.arange(cap, dtype=np.int32), (B, Hkv, 1))
    pos = rng.permutation(100000)[:B * Hkv * cap].reshape(B, Hkv, cap).astype(np.int32)
    ws = kvr.alloc_workspace(d, kvr.KVR_OP_ENCODE, cap)

    def run(count, kscale=1.0):
        sk = torch.zeros(B, Hkv, r, w, D, device="cuda")
        sv = torch.zeros(B, Hkv, r, w, D, device="cuda")
        kvr.kvr_encode(d, U.to_dev(K * kscale, dtype), U.to_dev(V * kscale, dtype), cap,
                       torch.as_tensor(slot).cuda(), torch.as_tensor(pos).cuda(),
                       torch.full((B, Hkv), count, dtype=torch.int32, device="cuda"), cap, sk, sv, None, None, ws)
        torch.cuda.synchronize()
        return sk.cpu(), sv.cpu()

    a1, b1 = run(cap)
    a2, b2 = run(cap)
    assert torch.equal(a1, a2) and torch.equal(b1, b2)
    a3, b3 = run(cap, 3.0)
    assert torch.equal(a3, 3 * a1) and torch.equal(b3, 3 * b1)
    # mass conservation of the unsigned keys in every row
    for i in range(r):
        assert torch.equal(a1[:, :, i].sum(dim=2).double(), torch.as_tensor(K.sum(axis=2)))


# ----------------------------------------------------------------------------- select
def run_select_case(kvr, rng, B, Hkv, ret_cap, n_cap, n_ctx, n_recent, k_cand, evict_cap, vague_cap, fill, nv0,
                    score_levels=None):
    d = kvr.make_desc(B, Hkv, Hkv, 3, 4, torch.bfloat16, seed=1)
    ret_pos = np.full((B, Hkv, ret_cap), -1, dtype=np.int32)
    scores = np.zeros((B, Hkv, n_cap), dtype=np.float32)
    for b in range(B):
        for h in range(Hkv):
            nfill = min(fill, n_ctx[b])
            p = rng.choice(n_ctx[b], size=nfill, replace=False)
            ret_pos[b, h, rng.choice(ret_cap, size=nfill, replace=False)] = p
            if score_levels:
                scores[b, h] = rng.integers(0, score_levels, size=n_cap) / 16.0 - 1.0
            else:
                scores[b, h] = rng.standard_normal(n_cap).astype(np.float32)
    scores[0, 0, ::7] = -0.0
    rp = torch.as_tensor(ret_pos).cuda()
    es = torch.full((B, Hkv, evict_cap), -7, dtype=torch.int32, device="cuda")
    ep = torch.full((B, Hkv, evict_cap), -7, dtype=torch.int32, device="cuda")
    ne = torch.full((B, Hkv), -99, dtype=torch.int32, device="cuda")
    vp = torch.full((B, Hkv, vague_cap), -7, dtype=torch.int32, device="cuda")
    nv = torch.full((B, Hkv), nv0, dtype=torch.int32, device="cuda")
    kvr.kvr_select(d, torch.as_tensor(scores).cuda(), n_cap, rp, ret_cap,
                   torch.as_tensor(np.array(n_ctx, dtype=np.int32)).cuda(), n_recent, k_cand, es, ep, ne,
                   evict_cap, vp, nv, vague_cap)
    torch.cuda.synchronize()
    rpg, esg, epg, neg, vpg, nvg = (x.cpu().numpy() for x in (rp, es, ep, ne, vp, nv))
    for b in range(B):
        for h in range(Hkv):
            ws_, wp_ = O.select(scores[b, h], ret_pos[b, h], n_ctx[b], n_recent, k_cand)
            n = len(ws_)
            if n > evict_cap or nv0 + n > vague_cap:
                assert neg[b, h] == -n
                assert np.array_equal(rpg[b, h], ret_pos[b, h]) and nvg[b, h] == nv0
                continue
            assert neg[b, h] == n, (b, h, neg[b, h], n)
            assert np.array_equal(esg[b, h, :n], ws_) and np.array_equal(epg[b, h, :n], wp_)
            assert (esg[b, h, n:] == -7).all()
            want_rp = ret_pos[b, h].copy()
            want_rp[ws_] = -1
            assert np.array_equal(rpg[b, h], want_rp)
            assert nvg[b, h] == nv0 + n
            assert np.array_equal(vpg[b, h, nv0:nv0 + n], wp_) and (vpg[b, h, :nv0] == -7).all()


def test_select_bit_exact(kvr):
    rng = np.random.default_rng(31)
    say("select steady state")
    run_select_case(kvr, rng, 2, 3, 187, 2200, [2049, 2100], 93, 93, 8, 2000, 187, 1862)
    say("select bulk with ties")
    run_select_case(kvr, rng, 2, 2, 3000, 3100, [3000, 2500], 500, 700, 3000, 3000, 3000, 0, score_levels=40)
    say("select k = 0, nothing recent")
    run_select_case(kvr, rng, 1, 2, 1500, 1500, [1500], 0, 0, 1500, 1500, 1200, 3)
    say("select nothing to evict")
    run_select_case(kvr, rng, 1, 2, 64, 300, [300], 10, 1000, 4, 100, 60, 0)
    say("select everything recent")
    run_select_case(kvr, rng, 1, 1, 64, 300, [300], 1000, 5, 4, 100, 60, 0)
    say("select overflow of evict_cap")
    run_select_case(kvr, rng, 1, 2, 200, 400, [400], 20, 30, 4, 1000, 200, 0)
    say("select overflow of vague_cap")
    run_select_case(kvr, rng, 1, 2, 200, 400, [400], 20, 30, 200, 60, 200, 50)
    say("select ragged tail, 1025 slots")
    run_select_case(kvr, rng, 1, 1, 1025, 5000, [5000], 100, 400, 1025, 2000, 1025, 0, score_levels=8)
    say("select 9000 slots (32 keys per thread in registers), ties")
    run_select_case(kvr, rng, 1, 2, 9000, 9100, [9050], 700, 2500, 9000, 9000, 8800, 5, score_levels=300)
    say("select 9000 slots, a handful of evictions")
    run_select_case(kvr, rng, 1, 1, 9000, 9100, [9050], 700, 8095, 16, 9000, 8800, 5)
    say("select 33000 slots (keys re-read from memory in every pass), ties")
    run_select_case(kvr, rng, 1, 1, 33000, 33100, [33000], 3000, 9000, 33000, 33000, 32500, 0, score_levels=500)


# ----------------------------------------------------------------------------- append
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_append(kvr, dtype):
    say("append", dtype)
    rng = np.random.default_rng(41)
    B, Hkv, cap, D = 2, 3, 300, 128
    d = kvr.make_desc(B, Hkv, Hkv, 3, 4, dtype, seed=1)
    k_ret = U.rand_storage(rng, (B, Hkv, cap, D), dtype)
    v_ret = U.rand_storage(rng, (B, Hkv, cap, D), dtype)
    ret_pos = rng.permutation(B * Hkv * cap).reshape(B, Hkv, cap).astype(np.int32)
    free = {(0, 0): [299], (0, 1): [0, 5], (0, 2): [257, 256], (1, 0): [], (1, 1): [128], (1, 2): [64, 63, 299]}
    for (b, h), fs in free.items():
        for f in fs:
            ret_pos[b, h, f] = -1
    kn, vn = U.rand_storage(rng, (B, Hkv, D), dtype), U.rand_storage(rng, (B, Hkv, D), dtype)
    kr, vr, rp = U.to_dev(k_ret, dtype), U.to_dev(v_ret, dtype), torch.as_tensor(ret_pos).cuda()
    osl = torch.full((B, Hkv), -5, dtype=torch.int32, device="cuda")
    n_ctx = torch.tensor([1000, 2000], dtype=torch.int32, device="cuda")
    kvr.kvr_append(d, U.to_dev(kn, dtype), U.to_dev(vn, dtype), n_ctx, kr, vr, rp, cap, osl)
    torch.cuda.synchronize()
    krg, vrg, rpg, oslg = U.to_np(kr), U.to_np(vr), rp.cpu().numpy(), osl.cpu().numpy()
    for (b, h), fs in free.items():
        wk, wv, wp = k_ret[b, h].copy(), v_ret[b, h].copy(), ret_pos[b, h].copy()
        if fs:
            s = min(fs)
            wk[s], wv[s], wp[s] = kn[b, h], vn[b, h], [999, 1999][b]
            assert oslg[b, h] == s
        else:
            assert oslg[b, h] == -1
        assert np.array_equal(krg[b, h], wk) and np.array_equal(vrg[b, h], wv) and np.array_equal(rpg[b, h], wp)


# ----------------------------------------------------------------------------- attend
def run_attend_case(kvr, rng, dtype, B, Hq, Hkv, r, w, ret_cap, n_vagues, vague_cap, mask=2, mode=0,
                    free_frac=0.1, with_scores=True, identity=False, kscale=1.0, side=None, keep=None,
                    check_units=None):
    """side: a binding.SideStream lent to the call (None: the kernels run back to back).
    keep: a list that receives (out, scores) of the call as CPU tensors.
    check_units: the (b, h) units the oracle is run for (None: all of them)."""
    D = 128
    G = Hq // Hkv
    d = kvr.make_desc(B, Hq, Hkv, r, w, dtype, seed=77, sign_mask=mask, median_mode=mode)
    params = kvr.desc_hash_params(d)
    st = U.storage_name(dtype)
    n_cap = ret_cap + vague_cap + 5
    K = U.rand_storage(rng, (B, Hkv, ret_cap, D), dtype, kscale)
    V = U.rand_storage(rng, (B, Hkv, ret_cap, D), dtype)
    SK = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 2.0 * kscale)
    SV = U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 2.0)
    q = U.rand_storage(rng, (B, Hq, D), dtype)
    scores0 = rng.random((B, Hkv, n_cap)).astype(np.float32)
    ret_pos = np.full((B, Hkv, ret_cap), -1, dtype=np.int32)
    vague_pos = np.zeros((B, Hkv, max(vague_cap, 1)), dtype=np.int32)
    nv = np.array(n_vagues, dtype=np.int32).reshape(B, Hkv)
    for b in range(B):
        for h in range(Hkv):
            n_used = ret_cap if identity else int(round(ret_cap * (1 - free_frac)))
            perm = rng.permutation(ret_cap + vague_cap)
            slots = np.arange(ret_cap) if identity else rng.choice(ret_cap, size=n_used, replace=False)
            ret_pos[b, h, slots] = np.arange(ret_cap) if identity else perm[:n_used]
            n = min(max(int(nv[b, h]), 0), vague_cap)
            vague_pos[b, h, :n] = perm[ret_cap:ret_cap + n] if not identity else ret_cap + np.arange(n)
    out = torch.full((B, Hq, D), 9.0, dtype=torch.float32, device="cuda")
    sc = torch.as_tensor(scores0).cuda() if with_scores else None
    ws = kvr.alloc_workspace(d, kvr.KVR_OP_ATTEND, ret_cap, vague_cap)
    kvr.kvr_attend_decode(
        d, U.to_dev(q, dtype), U.to_dev(K, dtype), U.to_dev(V, dtype),
        None if identity else torch.as_tensor(ret_pos).cuda(), ret_cap,
        U.to_dev(SK, dtype) if vague_cap else None, U.to_dev(SV, dtype) if vague_cap else None,
        torch.as_tensor(vague_pos).cuda() if vague_cap else None,
        torch.as_tensor(nv).cuda() if vague_cap else None, vague_cap, out, sc, n_cap, ws,
        side.opts() if side is not None else None)
    torch.cuda.synchronize()
    og = out.cpu().double().numpy()
    if keep is not None:
        keep.append((out.cpu().clone(), sc.cpu().clone() if sc is not None else None))
    worst = 0.0
    assert np.isfinite(og).all()
    for b in range(B):
        for h in range(Hkv):
            if check_units is not None and (b, h) not in check_units:
                continue
            n = min(max(int(nv[b, h]), 0), vague_cap)
            vp = vague_pos[b, h, :n].tolist()
            used = ret_pos[b, h] >= 0
            allpos = np.concatenate([ret_pos[b, h][used], np.array(vp, dtype=np.int64)])
            if len(allpos) == 0:
                assert (og[b, h * G:(h + 1) * G] == 0).all()
                continue
            # the oracle rebuilds KV indexed by position; remap positions to 0..n-1
            order = np.argsort(allpos)
            rank = {int(p): i for i, p in enumerate(allpos[order])}
            rp2 = np.array([rank[int(p)] if p >= 0 else -1 for p in ret_pos[b, h]], dtype=np.int64)
            # hashing uses the true positions, so query first with them
            Kh, Vh = O.query(SK[b, h], SV[b, h], params, vp, storage=st,
                             median_mode="lower" if mode else "midmean", sign_mask=mask)
            Kall = np.zeros((len(allpos), D))
            Vall = np.zeros((len(allpos), D))
            for s_ in range(ret_cap):
                if rp2[s_] >= 0:
                    Kall[rp2[s_]], Vall[rp2[s_]] = K[b, h, s_], V[b, h, s_]
            for t, p in enumerate(vp):
                Kall[rank[p]], Vall[rank[p]] = Kh[t], Vh[t]
            o_ref, p_ref = O.attention(q[b, h * G:(h + 1) * G], Kall, Vall, d.softmax_scale)
            worst = max(worst, check_out(og[b, h * G:(h + 1) * G], o_ref, dtype))
            if with_scores:
                inc = np.zeros(n_cap)
                inc[allpos[order]] = p_ref.sum(axis=0)
                want = scores0[b, h].astype(np.float64) + inc
                got = sc[b, h].cpu().double().numpy()
                tol = 1e-5 if dtype == torch.float32 else 2e-5
                assert np.abs(got - want).max() <= tol + 1e-6 * np.abs(want).max(), np.abs(got - want).max()
    return worst


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_attend_general(kvr, dtype):
    rng = np.random.default_rng(51)
    say("attend G=4 r=3", dtype)
    run_attend_case(kvr, rng, dtype, 2, 8, 2, 3, 6, 187, [1862, 1000, 0, 1863], 1900)
    say("attend G=1 r=3 single unit", dtype)
    run_attend_case(kvr, rng, dtype, 1, 1, 1, 3, 6, 187, [1862], 1862)
    say("attend G=2 r=4 midmean", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 2, 4, 9, 70, [333, 64], 400)
    say("attend G=8 r=4 lower, keys signed too", dtype)
    run_attend_case(kvr, rng, dtype, 1, 8, 1, 4, 9, 130, [257], 300, mask=3, mode=1)
    say("attend G=4 r=5 (run-time row count)", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 1, 5, 7, 65, [100], 128)
    say("attend r=1, r=2", dtype)
    run_attend_case(kvr, rng, dtype, 1, 2, 1, 1, 7, 65, [100], 128)
    run_attend_case(kvr, rng, dtype, 1, 2, 1, 2, 7, 65, [100], 128)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_attend_edges(kvr, dtype):
    rng = np.random.default_rng(52)
    say("attend full budget = dense attention (no sketch, identity slots)", dtype)
    run_attend_case(kvr, rng, dtype, 2, 8, 2, 3, 6, 700, [0, 0, 0, 0], 0, identity=True)
    say("attend no retained token", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 1, 3, 6, 5, [200], 256, free_frac=1.0)
    say("attend nothing at all", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 1, 3, 6, 5, [0], 16, free_frac=1.0)
    say("attend without score accumulation", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 1, 3, 6, 100, [150], 150, with_scores=False)
    say("attend peaked softmax (large key scale)", dtype)
    run_attend_case(kvr, rng, dtype, 1, 4, 1, 3, 6, 100, [300], 300, kscale=6.0)
    say("attend negative / oversized device count is clamped", dtype)
    run_attend_case(kvr, rng, dtype, 1, 8, 2, 3, 6, 50, [-4, 9999], 120)


def test_attend_staged_channel_chunks(kvr):
    """bf16, r in {3, 4}, G <= 4 takes the LDS-staged kernel; the width of a
    sketch row decides how many channels fit per phase (64 / 32 / 16 / 8).  Several
    workgroups per unit, ragged last round, more than one 64-token round per wave."""
    rng = np.random.default_rng(55)
    dtype = torch.bfloat16
    for (G, r, w, nv, cap, mode) in [(4, 3, 273, [5000, 4097], 5200, 0),      # 64 channels per phase
                                     (4, 3, 400, [700, 1], 800, 0),           # 32
                                     (2, 4, 500, [600, 333], 640, 0),         # 16, midmean
                                     (2, 4, 500, [600, 333], 640, 1),         # 16, lower
                                     (1, 3, 2000, [300, 64], 320, 0),         # 8
                                     (4, 4, 30, [900, 65], 1000, 0)]:         # 64, r = 4
        say("attend staged", G, r, w, nv, mode)
        run_attend_case(kvr, rng, dtype, 1, 2 * G, 2, r, w, 130, nv, cap, mode=mode)
    say("attend staged, many units (XCD mapping), 3 rounds per wave")
    run_attend_case(kvr, rng, dtype, 3, 12, 3, 3, 50, 70, [4000, 3999, 1, 0, 64, 65, 2500, 4100, 128], 4100)


@pytest.mark.parametrize("G,mode", [(1, 0), (2, 1), (4, 0)])
def test_attend_four_rows_many_rounds(kvr, G, mode):
    """Four sketch rows with so many units that the plan gives every unit one workgroup: a wave of the
    four-row staged kernel then takes up to 13 rounds of 64 tokens.  Units with shorter lists exercise the
    round counts in between, a ragged last round, one token and none.  Both median rules."""
    B, Hkv, cap = 32, 8, 6656
    lens = {(0, 0): 6656, (0, 1): 6593, (5, 3): 5000, (17, 6): 3300, (31, 7): 1, (31, 6): 0, (12, 0): 4161}
    nv = [lens.get((u // Hkv, u % Hkv), 6656 - 64 * (u % 7)) for u in range(B * Hkv)]
    rng = np.random.default_rng(61 + G)
    say("attend four rows, up to 13 rounds per wave", G, mode)
    run_attend_case(kvr, rng, torch.bfloat16, B, Hkv * G, Hkv, 4, 64, 70, nv, cap, mode=mode,
                    check_units=set(lens))


@pytest.mark.parametrize("G", [1, 2, 4])
def test_attend_side_by_side(kvr, G):
    """Enough units and Vague tokens that the staged kernel fills the chip more than twice over: with a
    second stream lent to the call the retained-slot kernel runs next to it, in its register-capped form.
    Both ways against the oracle, and against each other bit for bit (the same kernels compute the same
    sums in the same order; only where they run differs)."""
    B, Hkv = 16, 8
    nv = [9300 - 7 * (i % 5) for i in range(B * Hkv)]
    side = kvr.SideStream()
    got = []
    for sd in (side, None):
        say("attend side by side" if sd else "attend back to back", G)
        rng = np.random.default_rng(59 + G)
        run_attend_case(kvr, rng, torch.bfloat16, B, Hkv * G, Hkv, 3, 60, 150, nv, 9400, side=sd, keep=got)
    assert torch.equal(got[0][0], got[1][0]) and torch.equal(got[0][1], got[1][1])
    # the lent handles serve any number of calls in a row (and small calls, which do not fork)
    rng = np.random.default_rng(3)
    run_attend_case(kvr, rng, torch.bfloat16, 1, 4, 1, 3, 6, 100, [150], 150, side=side)
    run_attend_case(kvr, rng, torch.float32, 1, 4, 1, 3, 6, 100, [150], 150, side=side)


def test_attend_eight_heads_per_kv_head(kvr):
    """bf16, r = 3, G = 8: the Vague list goes through the streaming LDS-staged kernel (the one of
    kvr_attend_multi, one query, 8 columns): several workgroups per unit, ragged tiles, empty and clamped
    lists, with and without score accumulation."""
    rng = np.random.default_rng(58)
    dtype = torch.bfloat16
    for (w, nv, cap, ret, sc) in [(40, [900, 64, 0, 257], 900, 70, True),
                                  (273, [1500, 1499], 1500, 130, True),
                                  (7, [300, -2, 5000, 17], 400, 20, False)]:
        say("attend G=8 streamed", w, nv)
        B = len(nv)
        run_attend_case(kvr, rng, dtype, B, 8, 1, 3, w, ret, nv, cap, with_scores=sc)


def test_attend_staged64_shapes(kvr):
    """bf16, r = 3, 64-channel chunks: the specialised staged kernel.  Group sizes 1, 2, 4; widths from a few
    slots to the widest sketch that still fits LDS; 1 to 6 rounds of 64 tokens per wave; lists that end inside
    a round, inside a quad and inside a pair; units with nothing in the list."""
    rng = np.random.default_rng(56)
    dtype = torch.bfloat16
    for (G, w, nv, cap, ret) in [(1, 100, [300, 64, 1], 320, 40),
                                 (2, 320, [1000, 999, 2], 1024, 70),        # widest: 3 * 320 rows of 128 B
                                 (4, 7, [3070, 3071, 3072], 3072, 20),      # 6 rounds per wave, one workgroup
                                 (4, 273, [130, 0, 67], 200, 130),          # few tokens: most waves idle
                                 (2, 33, [5000, 4999, 63], 6000, 65)]:
        say("attend staged64", G, w, nv)
        B = len(nv)
        run_attend_case(kvr, rng, dtype, B, G, 1, 3, w, ret, nv, cap)


def test_full_budget_matches_library_sdpa(kvr):
    """n_vague = 0 must be textbook softmax(qK^T/sqrt(d))V: checked against
    torch's SDPA on the CPU in float64 (not the oracle)."""
    say("attend vs torch SDPA")
    rng = np.random.default_rng(53)
    B, Hq, Hkv, N, D = 2, 8, 2, 900, 128
    dtype = torch.bfloat16
    d = kvr.make_desc(B, Hq, Hkv, 3, 4, dtype, seed=1)
    K, V = U.rand_storage(rng, (B, Hkv, N, D), dtype), U.rand_storage(rng, (B, Hkv, N, D), dtype)
    q = U.rand_storage(rng, (B, Hq, D), dtype)
    out = torch.zeros(B, Hq, D, device="cuda")
    ws = kvr.alloc_workspace(d, kvr.KVR_OP_ATTEND, N)
    kvr.kvr_attend_decode(d, U.to_dev(q, dtype), U.to_dev(K, dtype), U.to_dev(V, dtype), None, N, None, None,
                          None, None, 0, out, None, N, ws)
    torch.cuda.synchronize()
    G = Hq // Hkv
    Kx = torch.as_tensor(K).repeat_interleave(G, dim=1)
    Vx = torch.as_tensor(V).repeat_interleave(G, dim=1)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.as_tensor(q).unsqueeze(2), Kx, Vx)[:, :, 0]
    assert (out.cpu().double() - ref).abs().max() <= TOL_OUT_BF16 * 1e-2


def test_fused_equals_dense_over_kvr_reconstruct(kvr):
    """The fused kernel must equal dense attention over [retained, kvr_reconstruct output]
    (both computed by the library)."""
    say("attend fused vs reconstruct + dense")
    rng = np.random.default_rng(54)
    B, Hq, Hkv, r, w, R, A, D = 1, 8, 2, 3, 11, 60, 500, 128
    dtype = torch.bfloat16
    d = kvr.make_desc(B, Hq, Hkv, r, w, dtype, seed=5)
    K, V = U.to_dev(U.rand_storage(rng, (B, Hkv, R, D), dtype), dtype), U.to_dev(U.rand_storage(rng, (B, Hkv, R, D), dtype), dtype)
    SK, SV = U.to_dev(U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 2.0), dtype), U.to_dev(U.rand_storage(rng, (B, Hkv, r, w, D), dtype, 2.0), dtype)
    q = U.to_dev(U.rand_storage(rng, (B, Hq, D), dtype), dtype)
    rp = torch.arange(R, dtype=torch.int32, device="cuda").expand(B, Hkv, R).contiguous()
    vp = (R + torch.arange(A, dtype=torch.int32, device="cuda")).expand(B, Hkv, A).contiguous()
    nv = torch.full((B, Hkv), A, dtype=torch.int32, device="cuda")
    out1 = torch.zeros(B, Hq, D, device="cuda")
    ws = kvr.alloc_workspace(d, kvr.KVR_OP_ATTEND, R + A, 0)
    ws1 = kvr.alloc_workspace(d, kvr.KVR_OP_ATTEND, R, A)
    kvr.kvr_attend_decode(d, q, K, V, rp, R, SK, SV, vp, nv, A, out1, None, R + A, ws1)
    kh, vh = torch.zeros(B, Hkv, A, D, dtype=dtype, device="cuda"), torch.zeros(B, Hkv, A, D, dtype=dtype, device="cuda")
    kvr.kvr_reconstruct(d, SK, SV, vp, nv, A, kh, vh)
    Kc, Vc = torch.cat([K, kh], dim=2).contiguous(), torch.cat([V, vh], dim=2).contiguous()
    out2 = torch.zeros(B, Hq, D, device="cuda")
    kvr.kvr_attend_decode(d, q, Kc, Vc, None, R + A, None, None, None, None, 0, out2, None, R + A, ws)
    torch.cuda.synchronize()
    assert (out1 - out2).abs().max().item() <= 1e-4


# ----------------------------------------------------------------------------- whole steps
@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("name", ["c1", "tiny_bf16", "tiny_r4"])
def test_decode_steps_follow_the_oracle(kvr, LayerState, name, fused):
    """Several decode steps.  Before every step the GPU state is loaded from the
    oracle's state; after it, indices and sketch must match bit for bit, floats
    within tolerance.  (Feeding each step from the oracle keeps one step's float
    rounding from deciding the next step's integer choices.)  fused: append, select
    and encode through kvr_step_update instead of the three separate calls."""
    if name == "c1":
        wl = S.WORKLOADS["c1"]
        nsteps = 3
    elif name == "tiny_bf16":
        wl = S.small_workload(batch=2, n_q_heads=8, n_kv_heads=2, context=700, budget=0.25, r=3, steps=4)
        nsteps = 4
    else:
        wl = S.small_workload("tiny4", batch=1, n_q_heads=4, n_kv_heads=2, context=900, budget=0.3, r=4, steps=3,
                              cfg_id=98)
        nsteps = 3
    say("decode steps", name)
    run_decode_steps(kvr, LayerState, wl, 0, nsteps, fused)


def run_decode_steps(kvr, LayerState, wl, layer, nsteps, fused):
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    states = U.oracle_units_from_workload(wl, layer, units, extra_tokens=nsteps + 2)
    params = states[0].params
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    G = wl.group
    scale = d.softmax_scale
    vague_cap = wl.n_vague0 + nsteps + 2
    for t in range(nsteps):
        ls = U.layer_state_from_oracle(kvr, LayerState, d, states, wl.batch, wl.n_kv_heads, vague_cap=vague_cap)
        kn, vn = S.new_tokens(wl, layer, t)
        q = S.queries(wl, layer, t + 1)
        out = ls.decode_step(kn.cuda(), vn.cuda(), q.cuda(), fused=fused)
        torch.cuda.synchronize()
        og = out.cpu().double().numpy()
        ne = ls.n_evict.cpu().numpy().reshape(-1)
        es = ls.evict_slot.cpu().numpy().reshape(len(units), -1)
        ep = ls.evict_pos.cpu().numpy().reshape(len(units), -1)
        skg = U.to_np(ls.sketch_k).reshape((len(units),) + states[0].SK.shape)
        svg = U.to_np(ls.sketch_v).reshape((len(units),) + states[0].SV.shape)
        rpg = ls.ret_pos.cpu().numpy().reshape(len(units), -1)
        scg = ls.scores.cpu().numpy().reshape(len(units), -1)
        nvg = ls.n_vague.cpu().numpy().reshape(-1)
        vpg = ls.vague_pos.cpu().numpy().reshape(len(units), -1)
        for u, (b, h) in enumerate(units):
            st = states[u]
            o_ref, (ws_, wp_), p = st.decode_step(U.to_np(kn[b, h]), U.to_np(vn[b, h]),
                                                  U.to_np(q[b, h * G:(h + 1) * G]), scale)
            assert ne[u] == len(ws_) == 1
            assert np.array_equal(es[u, :1], ws_) and np.array_equal(ep[u, :1], wp_)
            assert np.array_equal(rpg[u], st.ret_pos)
            assert nvg[u] == len(st.vague_pos) and np.array_equal(vpg[u, :nvg[u]], st.vague_pos)
            assert np.array_equal(skg[u], st.SK) and np.array_equal(svg[u], st.SV)
            check_out(og[b, h * G:(h + 1) * G], o_ref, wl.torch_dtype)
            assert np.abs(scg[u].astype(np.float64) - st.scores.astype(np.float64)).max() <= 2e-5


def test_prefill_compress_follows_the_oracle(kvr, LayerState):
    """from_prefill (dense scores -> select -> bulk encode -> compaction) against
    the oracle's prompt handling.  The oracle's initial scores are fed to the GPU
    selection (after checking the GPU's own dense scores against them), so the
    partition is comparable bit for bit."""
    say("prefill compress")
    wl = S.small_workload("pre", batch=2, n_q_heads=8, n_kv_heads=2, context=1500, budget=0.2, r=3, steps=2,
                          cfg_id=97)
    layer = 1
    units = [(b, h) for b in range(wl.batch) for h in range(wl.n_kv_heads)]
    dense = U.oracle_units_from_workload(wl, layer, units, compress=False, extra_tokens=4)
    params = dense[0].params
    d = kvr.make_desc(wl.batch, wl.n_q_heads, wl.n_kv_heads, wl.r, wl.w, wl.torch_dtype, hash_params=params)
    K, V = S.kv_layer(wl, layer)
    q0 = S.queries(wl, layer, 0)
    N = wl.context
    # (a) the library's own dense pass gives the same scores within tolerance
    ls0, _ = LayerState.from_prefill(d, K.cuda(), V.cuda(), q0.cuda(), n_recent=wl.n_recent,
                                     k_candidate=wl.n_candidate, max_new_tokens=4)
    # (b) partition + sketch with the oracle's scores as input
    sc0 = np.stack([s.scores[:N] for s in dense]).reshape(wl.batch, wl.n_kv_heads, N)
    ls, info = LayerState.from_prefill(d, K.cuda(), V.cuda(), q0.cuda(), n_recent=wl.n_recent,
                                       k_candidate=wl.n_candidate, max_new_tokens=4,
                                       init_scores=torch.as_tensor(sc0).cuda())
    torch.cuda.synchronize()
    for u, (b, h) in enumerate(units):
        st = dense[u]
        st.compress()
        st = O.compact(st, wl.n_retained + 1)
        assert np.array_equal(ls.ret_pos[b, h].cpu().numpy(), st.ret_pos)
        assert np.array_equal(U.to_np(ls.k_ret[b, h]), st.K_ret) and np.array_equal(U.to_np(ls.v_ret[b, h]), st.V_ret)
        nv = int(ls.n_vague[b, h])
        assert nv == len(st.vague_pos) == wl.n_vague0
        assert np.array_equal(ls.vague_pos[b, h, :nv].cpu().numpy(), st.vague_pos)
        assert np.array_equal(U.to_np(ls.sketch_k[b, h]), st.SK) and np.array_equal(U.to_np(ls.sketch_v[b, h]), st.SV)
        # dense-pass scores of run (a): all positions still in its retained set or list
        got = ls0.scores[b, h, :N].cpu().double().numpy()
        assert np.abs(got - sc0[b, h]).max() <= 2e-5
