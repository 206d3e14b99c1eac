"""kvr_attend_decode_static (the entry point for callers that cannot allocate: its
scratch memory is a fixed array inside the library) against kvr_attend_decode with a
caller workspace, through the C ABI: same inputs, outputs and scores must agree bit
for bit (the same kernels run, only the workspace address differs).  Two calls in a
row, the second with a smaller input, so that whatever the first call left in the
shared array is there when the second runs."""
import ctypes as C

import numpy as np
import pytest
import torch

from tests import util as U

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(300)]


def _case(kvr, rng, B, Hq, Hkv, r, w, ret_cap, vague_cap, dtype):
    D = 128
    d = kvr.make_desc(B, Hq, Hkv, r, w, dtype, seed=4242)
    n_cap = ret_cap + vague_cap + 3
    t = lambda shape, scale=1.0: U.to_dev(U.rand_storage(rng, shape, dtype, scale), dtype)
    K, V = t((B, Hkv, ret_cap, D)), t((B, Hkv, ret_cap, D))
    SK, SV = t((B, Hkv, r, w, D), 2.0), t((B, Hkv, r, w, D), 2.0)
    q = t((B, Hq, D))
    ret_pos = np.full((B, Hkv, ret_cap), -1, dtype=np.int32)
    vague_pos = np.zeros((B, Hkv, vague_cap), dtype=np.int32)
    nv = np.zeros((B, Hkv), dtype=np.int32)
    for b in range(B):
        for h in range(Hkv):
            perm = rng.permutation(ret_cap + vague_cap)
            n_used = ret_cap - int(rng.integers(0, 5))
            ret_pos[b, h, rng.choice(ret_cap, size=n_used, replace=False)] = perm[:n_used]
            nv[b, h] = vague_cap - int(rng.integers(0, 70))
            vague_pos[b, h, :nv[b, h]] = perm[ret_cap:ret_cap + nv[b, h]]
    scores0 = torch.as_tensor(rng.random((B, Hkv, n_cap)).astype(np.float32)).cuda()
    return dict(d=d, q=q, K=K, V=V, rp=torch.as_tensor(ret_pos).cuda(), ret_cap=ret_cap, SK=SK, SV=SV,
                vp=torch.as_tensor(vague_pos).cuda(), nv=torch.as_tensor(nv).cuda(), vague_cap=vague_cap,
                scores0=scores0, n_cap=n_cap, B=B, Hq=Hq)


def _raw_args(c, out, scores):
    p = lambda x: C.c_void_p(x.data_ptr())
    return [C.byref(c["d"]), p(c["q"]), p(c["K"]), p(c["V"]), p(c["rp"]), c["ret_cap"], p(c["SK"]), p(c["SV"]),
            p(c["vp"]), p(c["nv"]), c["vague_cap"], p(out), p(scores), c["n_cap"]]


def _run_both(kvr, c, side=None):
    """Both entry points through the raw C ABI on the current torch stream."""
    L = kvr.lib()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    opts = C.byref(side.opts()) if side is not None else None
    out_a = torch.full((c["B"], c["Hq"], 128), 7.0, dtype=torch.float32, device="cuda")
    out_b = torch.full_like(out_a, -7.0)
    sc_a, sc_b = c["scores0"].clone(), c["scores0"].clone()
    need = kvr.kvr_workspace_size(c["d"], kvr.KVR_OP_ATTEND, c["ret_cap"], c["vague_cap"])
    assert need <= kvr.KVR_STATIC_SCRATCH_BYTES
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    rc = L.kvr_attend_decode(*_raw_args(c, out_a, sc_a), C.c_void_p(ws.data_ptr()), C.c_size_t(ws.numel()), opts, stream)
    assert rc == kvr.KVR_OK, rc
    rc = L.kvr_attend_decode_static(*_raw_args(c, out_b, sc_b), opts, stream)
    assert rc == kvr.KVR_OK, (rc, L.kvr_last_hip_error())
    torch.cuda.synchronize()
    assert torch.isfinite(out_a).all()
    assert torch.equal(out_a, out_b), float((out_a - out_b).abs().max())
    assert torch.equal(sc_a, sc_b)
    assert not torch.equal(sc_a, c["scores0"])


def test_static_scratch_entry_point_matches_the_workspace_one():
    from paper_2512_17917_amd import binding as kvr
    kvr.lib()
    rng = np.random.default_rng(2024)
    print("[case] static scratch: staged path, 12 units, then a smaller call", flush=True)
    big = _case(kvr, rng, 3, 16, 4, 3, 60, 300, 5000, torch.bfloat16)       # staged kernel, several workgroups per unit
    small = _case(kvr, rng, 1, 4, 1, 3, 6, 70, 400, torch.bfloat16)
    _run_both(kvr, big)
    _run_both(kvr, small)
    print("[case] static scratch: f32 storage (generic kernel), then side by side with a lent stream", flush=True)
    _run_both(kvr, _case(kvr, rng, 1, 2, 2, 4, 9, 50, 200, torch.float32))
    side = kvr.SideStream()
    _run_both(kvr, _case(kvr, rng, 16, 8, 8, 3, 60, 150, 9400, torch.bfloat16), side=side)
    _run_both(kvr, small, side=side)


def test_static_scratch_refuses_what_does_not_fit():
    from paper_2512_17917_amd import binding as kvr
    L = kvr.lib()
    d = kvr.make_desc(64, 32, 8, 3, 273, kvr.KVR_BF16, seed=1)            # four times the largest named workload
    need = kvr.kvr_workspace_size(d, kvr.KVR_OP_ATTEND, 7400, 25600)
    assert need > kvr.KVR_STATIC_SCRATCH_BYTES
    p = C.c_void_p(0x10000)                                              # never dereferenced: refused before any launch
    rc = L.kvr_attend_decode_static(C.byref(d), p, p, p, p, 7400, p, p, p, p, 25600, p, p, 40000, None, None)
    assert rc == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
