"""CPU-only checks of the C ABI: the library loads, exports what include/kvr.h
declares, its pure-host functions agree with the oracle, and every argument
error is reported before anything touches a GPU."""
import ctypes as C
import os
import re

import pytest

from oracle import kvr_oracle as O
from paper_2512_17917_amd import binding as kvr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "kvr.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(kvr_[a-z_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(kvr.EXPORTS)
    L = kvr.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert kvr.kvr_version().startswith("kvr")


def test_desc_layout_matches_header():
    # 9 int32 + 1 float = 40 bytes, then 8 x 4 uint64
    assert C.sizeof(kvr.kvr_desc) == 40 + 8 * 4 * 8
    assert kvr.kvr_desc.hash_params.offset == 40
    assert C.sizeof(kvr.kvr_attend_opts) == 5 * C.sizeof(C.c_void_p)


def test_recent_size_follows_the_oracle_queue():
    """kvr_recent_size against the oracle's Recent queue over a run of pushes."""
    import numpy as np
    for budget, slack in [(5, 0), (5, 3), (1, 7), (0, 2)]:
        st = O.UnitState(64, 64, 1, 1, 128, O.hash_params_from_seed(1, 1), "f32", n_recent=budget, k_candidate=64)
        r = 0
        for t in range(30):
            st.append(np.zeros(128), np.zeros(128))
            st.compress(slack)                       # k_candidate is large: nothing reaches the sketch
            r = kvr.kvr_recent_size(r + 1, budget, slack)
            assert r == st.r_size


def test_host_hash_matches_oracle():
    for seed, r, w in [(0, 1, 1), (2512, 3, 273), (17917, 4, 819), (5, 8, 65536)]:
        params = kvr.kvr_hash_params_from_seed(seed, r)
        assert params == O.hash_params_from_seed(seed, r)
        d = kvr.make_desc(1, 4, 1, r, w, kvr.KVR_BF16, seed=seed)
        for J in [0, 1, 2, 63, 64, 4095, 32767, 131071, 2 ** 31 - 1]:
            b, s = kvr.kvr_hash_host(d, J)
            assert b == [O.bucket_of(params[i], J, w) for i in range(r)]
            assert s == [O.sign_of(params[i], J) for i in range(r)]
            assert all(0 <= x < w for x in b)
    # arbitrary tables (not from the LCG), including wrap-around
    hp = [(0xFFFFFFFFFFFFFFFF, 0xFFFFFFFF00000000, 1 << 63, 1 << 63)]
    d = kvr.make_desc(1, 1, 1, 1, 7, kvr.KVR_F32, hash_params=hp)
    for J in [0, 1, 2, 3, 1000]:
        b, s = kvr.kvr_hash_host(d, J)
        assert b == [O.bucket_of(hp[0], J, 7)] and s == [O.sign_of(hp[0], J)]


def test_workspace_sizes():
    d = kvr.make_desc(16, 32, 8, 3, 273, kvr.KVR_BF16, seed=1)
    assert kvr.kvr_workspace_size(d, kvr.KVR_OP_SELECT, 10000) == 0
    assert kvr.kvr_workspace_size(d, kvr.KVR_OP_RECONSTRUCT, 10000) == 0
    assert kvr.kvr_workspace_size(d, kvr.KVR_OP_ENCODE, 8) == 0
    big = kvr.kvr_workspace_size(d, kvr.KVR_OP_ENCODE, 30000)
    assert big >= 16 * 8 * 3 * 2 * 30000 * 4
    a1 = kvr.kvr_workspace_size(d, kvr.KVR_OP_ATTEND, 200, 800)
    a2 = kvr.kvr_workspace_size(d, kvr.KVR_OP_ATTEND, 7400, 25600)
    assert 0 < a1 < a2
    assert a2 >= 16 * 8 * 33000 * 4 * 4           # the spilled logits
    with pytest.raises(kvr.KvrError):
        kvr.kvr_workspace_size(d, 99, 10)
    with pytest.raises(kvr.KvrError):
        kvr.kvr_workspace_size(d, kvr.KVR_OP_ATTEND, -1, 0)


def bad_descs():
    base = dict(batch=2, n_q_heads=8, n_kv_heads=2, r=3, w=10, dtype=kvr.KVR_BF16)
    out = []
    for k, v, code in [("batch", 0, kvr.KVR_ERR_INVALID_ARG), ("r", 0, kvr.KVR_ERR_INVALID_ARG),
                       ("r", 9, kvr.KVR_ERR_INVALID_ARG), ("w", 0, kvr.KVR_ERR_INVALID_ARG),
                       ("w", 70000, kvr.KVR_ERR_INVALID_ARG), ("n_q_heads", 6, kvr.KVR_ERR_UNSUPPORTED),
                       ("n_q_heads", 7, kvr.KVR_ERR_UNSUPPORTED)]:
        kw = dict(base)
        kw[k] = v
        out.append((kvr.make_desc(kw["batch"], kw["n_q_heads"], kw["n_kv_heads"], kw["r"] if 1 <= kw["r"] <= 8 else 1,
                                  kw["w"], kw["dtype"], seed=1), k, v, code))
        if k == "r":
            out[-1][0].r = v
    d = kvr.make_desc(2, 8, 2, 3, 10, kvr.KVR_BF16, seed=1)
    d.head_dim = 64
    out.append((d, "head_dim", 64, kvr.KVR_ERR_UNSUPPORTED))
    d = kvr.make_desc(2, 8, 2, 3, 10, kvr.KVR_BF16, seed=1)
    d.dtype = 5
    out.append((d, "dtype", 5, kvr.KVR_ERR_INVALID_ARG))
    d = kvr.make_desc(2, 8, 2, 3, 10, kvr.KVR_BF16, seed=1)
    d.sign_mask = 4
    out.append((d, "sign_mask", 4, kvr.KVR_ERR_INVALID_ARG))
    return out


def test_bad_descriptors_are_rejected_without_a_gpu():
    L = kvr.lib()
    sz = C.c_size_t(0)
    for d, k, v, code in bad_descs():
        assert L.kvr_workspace_size(C.byref(d), kvr.KVR_OP_ATTEND, 100, 0, C.byref(sz)) == code, (k, v)
        # a compute entry point with otherwise plausible (fake, never dereferenced) pointers
        p = 0x10000
        assert L.kvr_reconstruct(C.byref(d), p, p, p, p, 4, p, p, None) == code, (k, v)
    assert L.kvr_workspace_size(None, kvr.KVR_OP_ATTEND, 100, 0, C.byref(sz)) == kvr.KVR_ERR_INVALID_ARG


def test_bad_arguments_are_rejected_without_a_gpu():
    L = kvr.lib()
    d = kvr.make_desc(2, 8, 2, 3, 10, kvr.KVR_BF16, seed=1)
    dp = C.byref(d)
    p, odd = 0x10000, 0x10008                     # fake device addresses; never dereferenced
    E = kvr.KVR_ERR_INVALID_ARG
    # reconstruct
    assert L.kvr_reconstruct(dp, None, p, p, p, 4, p, p, None) == E
    assert L.kvr_reconstruct(dp, odd, p, p, p, 4, p, p, None) == E
    assert L.kvr_reconstruct(dp, p, p, p, p, -1, p, p, None) == E
    # encode
    assert L.kvr_encode(dp, p, p, 0, p, p, p, 4, p, p, None, None, None, 0, None) == E
    assert L.kvr_encode(dp, p, None, 8, p, p, p, 4, p, p, None, None, None, 0, None) == E
    assert L.kvr_encode(dp, p, p, 8, p, p, p, 1000, p, p, None, None, None, 0, None) == E      # bulk needs ws
    assert L.kvr_encode(dp, p, p, 8, p, p, p, 1000, p, p, None, None, p, 16, None) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    # select
    assert L.kvr_select(dp, None, 100, p, 10, p, 2, 3, p, p, p, 4, p, p, 50, None, 0, None) == E
    assert L.kvr_select(dp, p, 100, p, 10, p, -1, 3, p, p, p, 4, p, p, 50, None, 0, None) == E
    assert L.kvr_select(dp, p, 100, p, 10, p, 2, 3, p, p, p, 0, p, p, 50, None, 0, None) == E
    assert L.kvr_select(dp, p, 100, p, 10, p, 2, 3, p, p, p, 4, p, None, 50, None, 0, None) == E  # pair
    # append
    assert L.kvr_append(dp, p, p, p, p, p, None, 10, None, None) == E
    assert L.kvr_append(dp, p, p, p, p, p, p, 0, None, None) == E
    # step_update
    ok_args = [dp, p, p, p, p, p, p, 100, p, 1000, 10, 20, p, p, p, 8, p, p, 500, p, p, None]
    bad = list(ok_args); bad[1] = None
    assert L.kvr_step_update(*bad) == E
    bad = list(ok_args); bad[16] = None          # vague_pos without n_vague
    assert L.kvr_step_update(*bad) == E
    bad = list(ok_args); bad[7] = 40000          # more slots than the fused kernel takes
    assert L.kvr_step_update(*bad) == kvr.KVR_ERR_UNSUPPORTED
    bad = list(ok_args); bad[15] = 65
    assert L.kvr_step_update(*bad) == kvr.KVR_ERR_UNSUPPORTED
    # attend
    assert L.kvr_attend_decode(dp, None, p, p, p, 10, p, p, p, p, 20, p, p, 100, p, 1 << 30, None, None) == E
    assert L.kvr_attend_decode(dp, p, p, p, p, 10, p, p, p, None, 20, p, p, 100, p, 1 << 30, None, None) == E
    assert L.kvr_attend_decode(dp, p, p, p, p, 10, None, None, p, p, 20, p, p, 100, p, 1 << 30, None, None) == E
    assert L.kvr_attend_decode(dp, p, p, p, p, 10, p, p, p, p, 20, p, p, 100, None, 0, None, None) == E
    assert L.kvr_attend_decode(dp, p, p, p, p, 10, p, p, p, p, 20, p, p, 100, p, 64, None, None) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    assert L.kvr_attend_decode(dp, p, p, p, p, 10, p, p, p, p, 20, p, p, 0, p, 1 << 30, None, None) == E
    # attend options: a side stream comes with both of its events or not at all, the two timing
    # events come as a pair, and the side stream is not the call's own stream
    def attend_with(opts, stream=None):
        return L.kvr_attend_decode(dp, p, p, p, p, 10, p, p, p, p, 20, p, p, 100, p, 64, C.byref(opts), stream)
    h = 0x20000                                   # fake handles; never used: the workspace check fails first
    assert attend_with(kvr.kvr_attend_opts(h, h, h, None, None)) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    assert attend_with(kvr.kvr_attend_opts(None, None, None, h, h)) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    assert attend_with(kvr.kvr_attend_opts(None, None, None, None, None)) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    assert attend_with(kvr.kvr_attend_opts(h, None, h, None, None)) == E
    assert attend_with(kvr.kvr_attend_opts(h, h, None, None, None)) == E
    assert attend_with(kvr.kvr_attend_opts(None, h, h, None, None)) == E
    assert attend_with(kvr.kvr_attend_opts(None, None, None, h, None)) == E
    assert attend_with(kvr.kvr_attend_opts(None, None, None, None, h)) == E
    assert attend_with(kvr.kvr_attend_opts(h, h, h, None, None), stream=h) == E
    # the static-scratch entry point: same checks, and a call that needs more than the fixed array is refused
    assert L.kvr_attend_decode_static(dp, None, p, p, p, 10, p, p, p, p, 20, p, p, 100, None, None) == E
    assert L.kvr_attend_decode_static(dp, p, p, p, p, 10, p, p, p, p, 20, p, p, 0, None, None) == E
    dbig = kvr.make_desc(64, 32, 8, 3, 273, kvr.KVR_BF16, seed=1)
    assert kvr.kvr_workspace_size(dbig, kvr.KVR_OP_ATTEND, 7400, 25600) > kvr.KVR_STATIC_SCRATCH_BYTES
    assert L.kvr_attend_decode_static(C.byref(dbig), p, p, p, p, 7400, p, p, p, p, 25600, p, p, 40000, None,
                                      None) == kvr.KVR_ERR_WORKSPACE_TOO_SMALL
    # Recent queue size after a push (Algorithm 3, first branch)
    assert L.kvr_recent_size(6, 5, 0) == 5 and L.kvr_recent_size(5, 5, 0) == 5 and L.kvr_recent_size(3, 5, 0) == 3
    assert L.kvr_recent_size(8, 5, 3) == 8 and L.kvr_recent_size(9, 5, 3) == 5 and L.kvr_recent_size(40, 5, 3) == 5
    assert L.kvr_recent_size(2 ** 31 - 1, 2 ** 31 - 1, 2 ** 31 - 1) == 2 ** 31 - 1
    assert L.kvr_recent_size(-1, 5, 0) == E and L.kvr_recent_size(5, -1, 0) == E and L.kvr_recent_size(5, 5, -1) == E
    # hash helpers
    assert L.kvr_hash_params_from_seed(1, 0, None) == E
    assert L.kvr_hash_host(dp, -1, None, None) == E
    assert L.kvr_last_hip_error() == 0


def test_binding_refuses_host_tensors():
    import torch
    d = kvr.make_desc(1, 1, 1, 3, 4, kvr.KVR_F32, seed=1)
    x = torch.zeros(1, 1, 3, 4, 128)
    with pytest.raises(ValueError):
        kvr.kvr_reconstruct(d, x, x, torch.zeros(1, 1, 2, dtype=torch.int32),
                            torch.zeros(1, 1, dtype=torch.int32), 2, torch.zeros(1, 1, 2, 128),
                            torch.zeros(1, 1, 2, 128))
