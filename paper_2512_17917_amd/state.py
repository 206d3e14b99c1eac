"""Device buffers of one attention layer and the call sequence of a decode step.

Plumbing only (allocation, slicing, one gather that compacts the prompt's kept
rows): every arithmetic step is a call into libkvr through `binding`.
"""
from __future__ import annotations

import torch

from . import binding as kvr


class LayerState:
    """All per-unit buffers of one layer, unit-major [B, Hkv, ...]."""

    def __init__(self, desc, *, n_recent, k_candidate, ret_cap, vague_cap, n_cap, evict_cap=8,
                 device="cuda", ws_attend=None, ws_encode=None, n_ctx=None, slack=0, side=None):
        """n_recent, k_candidate: R.budget and C.budget of Algorithm 3; slack: its Slack (the
        Recent queue may outgrow its budget by that many tokens before slack + 1 of them leave at
        once; needs ret_cap >= n_recent + k_candidate + slack + 1 and evict_cap >= slack + 1);
        side: a binding.SideStream lent to every attend call (None: kernels back to back)."""
        self.desc = desc
        self.n_recent, self.k_candidate = int(n_recent), int(k_candidate)
        self.slack = int(slack)
        self.side = side
        # R.size after the last update; the queue itself is "the r_size newest positions"
        self.r_size = self.n_recent
        self.ret_cap, self.vague_cap, self.n_cap, self.evict_cap = int(ret_cap), int(vague_cap), int(n_cap), int(evict_cap)
        B, Hkv, Hq, D = desc.batch, desc.n_kv_heads, desc.n_q_heads, desc.head_dim
        dt = torch.float32 if desc.dtype == kvr.KVR_F32 else torch.bfloat16
        dev = torch.device(device)
        self.device, self.dtype = dev, dt
        self.k_ret = torch.zeros(B, Hkv, self.ret_cap, D, dtype=dt, device=dev)
        self.v_ret = torch.zeros(B, Hkv, self.ret_cap, D, dtype=dt, device=dev)
        self.ret_pos = torch.full((B, Hkv, self.ret_cap), -1, dtype=torch.int32, device=dev)
        self.scores = torch.zeros(B, Hkv, self.n_cap, dtype=torch.float32, device=dev)
        self.sketch_k = torch.zeros(B, Hkv, desc.r, desc.w, D, dtype=dt, device=dev)
        self.sketch_v = torch.zeros(B, Hkv, desc.r, desc.w, D, dtype=dt, device=dev)
        self.vague_pos = torch.zeros(B, Hkv, self.vague_cap, dtype=torch.int32, device=dev)
        self.n_vague = torch.zeros(B, Hkv, dtype=torch.int32, device=dev)
        self.evict_slot = torch.zeros(B, Hkv, self.evict_cap, dtype=torch.int32, device=dev)
        self.evict_pos = torch.zeros(B, Hkv, self.evict_cap, dtype=torch.int32, device=dev)
        self.n_evict = torch.zeros(B, Hkv, dtype=torch.int32, device=dev)
        # several layers may share one n_ctx tensor and one workspace (calls on one
        # stream are ordered, and no workspace content outlives a call)
        self.n_ctx = torch.zeros(B, dtype=torch.int32, device=dev) if n_ctx is None else n_ctx
        self.out = torch.zeros(B, Hq, D, dtype=torch.float32, device=dev)
        self.ws_attend = ws_attend if ws_attend is not None else kvr.alloc_workspace(
            desc, kvr.KVR_OP_ATTEND, self.ret_cap, self.vague_cap, dev)
        self.ws_encode = ws_encode if ws_encode is not None else kvr.alloc_workspace(
            desc, kvr.KVR_OP_ENCODE, self.evict_cap, 0, dev)

    # -- the four calls of a decode step, on this layer's buffers ---------------
    def append(self, k_new, v_new):
        kvr.kvr_append(self.desc, k_new, v_new, self.n_ctx, self.k_ret, self.v_ret, self.ret_pos,
                       self.ret_cap)

    def select(self):
        kvr.kvr_select(self.desc, self.scores, self.n_cap, self.ret_pos, self.ret_cap, self.n_ctx,
                       self.r_size, self.k_candidate, self.evict_slot, self.evict_pos, self.n_evict,
                       self.evict_cap, self.vague_pos, self.n_vague, self.vague_cap)

    def encode(self):
        kvr.kvr_encode(self.desc, self.k_ret, self.v_ret, self.ret_cap, self.evict_slot, self.evict_pos,
                       self.n_evict, self.evict_cap, self.sketch_k, self.sketch_v, None, None,
                       self.ws_encode)

    def attend(self, q, accumulate_scores=True, opts=None):
        kvr.kvr_attend_decode(self.desc, q, self.k_ret, self.v_ret, self.ret_pos, self.ret_cap,
                              self.sketch_k, self.sketch_v, self.vague_pos, self.n_vague, self.vague_cap,
                              self.out, self.scores if accumulate_scores else None, self.n_cap,
                              self.ws_attend, self.side.opts() if self.side is not None and opts is None else opts)
        return self.out

    def attend_multi(self, q, n_q, accumulate_scores=True, ws=None):
        """n_q query tokens per sequence (q [B, n_q, Hq, D]) at the n_q newest
        positions, over one rebuilt cache.  Returns out [B, n_q, Hq, D] float32."""
        if ws is None:
            n = kvr.kvr_attend_multi_workspace_size(self.desc, n_q, self.ret_cap, self.vague_cap)
            ws = torch.empty(max(n, 256), dtype=torch.uint8, device=self.device)
        B, Hq, D = self.desc.batch, self.desc.n_q_heads, self.desc.head_dim
        out = torch.zeros(B, n_q, Hq, D, dtype=torch.float32, device=self.device)
        kvr.kvr_attend_multi(self.desc, q, n_q, self.n_ctx, self.k_ret, self.v_ret, self.ret_pos, self.ret_cap,
                             self.sketch_k, self.sketch_v, self.vague_pos, self.n_vague, self.vague_cap, out,
                             self.scores if accumulate_scores else None, self.n_cap, ws)
        return out

    def step_update(self, k_new, v_new):
        """append + select + encode in one launch (decode steady state)."""
        kvr.kvr_step_update(self.desc, k_new, v_new, self.n_ctx, self.k_ret, self.v_ret, self.ret_pos,
                            self.ret_cap, self.scores, self.n_cap, self.r_size, self.k_candidate,
                            self.evict_slot, self.evict_pos, self.n_evict, self.evict_cap, self.vague_pos,
                            self.n_vague, self.vague_cap, self.sketch_k, self.sketch_v)

    def swap_back(self, replace_rate=1.1, max_swaps=4, n_swapped=None, swap_log=None):
        """The swap loop of Algorithm 3 on this layer's buffers."""
        kvr.kvr_swap_back(self.desc, self.scores, self.n_cap, self.k_ret, self.v_ret, self.ret_pos,
                          self.ret_cap, self.n_ctx, self.r_size, replace_rate, max_swaps, self.sketch_k,
                          self.sketch_v, self.vague_pos, self.n_vague, self.vague_cap, n_swapped, swap_log)

    def check_evictions(self):
        """Synchronises and raises if the last update of some unit could not evict what it had to
        (n_evict < 0: evict_cap or vague_cap too small; the unit then kept everything and its
        retained slots fill up)."""
        worst = int(self.n_evict.min().item())
        if worst < 0:
            raise RuntimeError(f"a unit needed {-worst} evictions but evict_cap = {self.evict_cap}, "
                               f"vague_cap = {self.vague_cap}: nothing was evicted there")

    def decode_step(self, k_new, v_new, q, *, bump_n_ctx=True, fused=None, replace_rate=None, max_swaps=4,
                    check=False, opts=None):
        """append -> select -> encode -> (swap loop, if replace_rate is given) ->
        attend.  n_ctx counts the new token from here on; pass bump_n_ctx=False when
        several layers share one n_ctx tensor that the caller advances once per
        step.  fused: use kvr_step_update for the first three (default: whenever its
        size limits allow).  check: synchronise after the update and raise if a unit
        could not evict (see check_evictions)."""
        if bump_n_ctx:
            self.n_ctx += 1
        # Algorithm 3, first branch: does the Recent queue hand its overhang on to the Candidates?
        self.r_size = kvr.kvr_recent_size(self.r_size + 1, self.n_recent, self.slack)
        if fused is None:
            fused = self.ret_cap <= 32768 and self.evict_cap <= 64
        if fused:
            self.step_update(k_new, v_new)
        else:
            self.append(k_new, v_new)
            self.select()
            self.encode()
        if check:
            self.check_evictions()
        if replace_rate is not None and max_swaps > 0:
            self.swap_back(replace_rate, max_swaps)
        return self.attend(q, opts=opts)

    # -- building the state from a prompt ---------------------------------------
    @classmethod
    def from_prefill(cls, desc, K, V, q0, *, n_recent, k_candidate, max_new_tokens, evict_cap=None,
                     init_scores=None, ws_attend=None, ws_encode=None, n_ctx=None, timers=None, slack=0,
                     side=None):
        """Compress a prompt's KV cache K, V [B, Hkv, N, D]: cumulative scores are
        initialised with one dense attention pass of q0 (or taken from
        init_scores [B, Hkv, N]), the Recent and Candidate parts are kept raw and
        compacted into ret_cap = n_recent + k_candidate + 1 slots, everything else
        goes into the sketch.  Returns (state, info)."""
        B, Hkv, N, D = K.shape
        dev = K.device
        R = n_recent + k_candidate
        ret_cap = R + slack + 1
        n_cap = N + max_new_tokens
        n_vague0 = max(N - R, 0)
        vague_cap = n_vague0 + max_new_tokens
        if evict_cap is None:
            evict_cap = max(8, slack + 1)
        st = cls(desc, n_recent=n_recent, k_candidate=k_candidate, ret_cap=ret_cap, vague_cap=vague_cap,
                 n_cap=n_cap, evict_cap=evict_cap, device=dev, ws_attend=ws_attend, ws_encode=ws_encode,
                 n_ctx=n_ctx, slack=slack, side=side)
        st.n_ctx.fill_(N)
        # the whole prompt was pushed into the Recent queue
        st.r_size = kvr.kvr_recent_size(N, n_recent, slack)
        # 1. cumulative scores of the prompt
        if init_scores is not None:
            st.scores[:, :, :N] = init_scores
        else:
            ws = kvr.alloc_workspace(desc, kvr.KVR_OP_ATTEND, N, 0, dev)
            kvr.kvr_attend_decode(desc, q0, K, V, None, N, None, None, None, None, 0, st.out, st.scores,
                                  n_cap, ws)
            del ws
        # 2. partition: every prompt token sits in "slot = position" of the full cache
        full_pos = torch.arange(N, dtype=torch.int32, device=dev).expand(B, Hkv, N).contiguous()
        ev_cap = max(n_vague0, 1)
        ev_slot = torch.zeros(B, Hkv, ev_cap, dtype=torch.int32, device=dev)
        ev_pos = torch.zeros(B, Hkv, ev_cap, dtype=torch.int32, device=dev)
        ws = kvr.alloc_workspace(desc, kvr.KVR_OP_ENCODE, ev_cap, 0, dev)
        if timers is not None:       # (start, stop) torch events around select + bulk encode
            timers[0].record()
        kvr.kvr_select(desc, st.scores, n_cap, full_pos, N, st.n_ctx, st.r_size, k_candidate,
                       ev_slot, ev_pos, st.n_evict, ev_cap, st.vague_pos, st.n_vague, vague_cap)
        # 3. bulk insert of the evicted tokens
        kvr.kvr_encode(desc, K, V, N, ev_slot, ev_pos, st.n_evict, ev_cap, st.sketch_k, st.sketch_v,
                       None, None, ws)
        if timers is not None:
            timers[1].record()
        del ws
        # 4. compact the kept rows (ascending slot order) into the small slot array
        R = min(st.r_size + k_candidate, N)
        kept_first = torch.sort((full_pos < 0).to(torch.int8), dim=2, stable=True).indices[:, :, :R]
        n_kept = (full_pos >= 0).sum(dim=2)
        st.k_ret[:, :, :R] = K.gather(2, kept_first.unsqueeze(-1).expand(-1, -1, -1, D))
        st.v_ret[:, :, :R] = V.gather(2, kept_first.unsqueeze(-1).expand(-1, -1, -1, D))
        rp = full_pos.gather(2, kept_first)
        rp = torch.where(torch.arange(R, device=dev).view(1, 1, R) < n_kept.unsqueeze(-1), rp,
                         torch.full_like(rp, -1))
        st.ret_pos[:, :, :R] = rp
        info = {"evict_slot": ev_slot, "evict_pos": ev_pos, "n_evict": st.n_evict.clone()}
        return st, info
