"""CPU oracle for the KVReviver decode hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, deliberately unoptimised implementation of what the paper
defines, one (layer, sequence, kv-head) unit at a time, written from the
paper's Algorithm section (Vague Sketch: Algorithms 1 and 2; Recent and
Candidate: Algorithms 3 and 4, the swap loop of Algorithm 3 included; Overview:
accumulation of attention scores).
It shares no code with the HIP library and never imports it.  Only tests, the
smoke check and the benchmark's CPU-baseline leg may import this file; the
product path must never call it.

Floating point: float64 throughout, except where a value is *stored* -- the
sketch, K, V and q live in a storage type ("f32" or "bf16") and scores live in
float32, because those are the formats of the buffers the method keeps.  Stored
values are held here as float64 arrays whose entries are exactly representable
in the storage type.  Rounding to storage is round-to-nearest-even, done once
per sketch slot per insert call (after all of that call's contributions have
been added to the slot's previous content, in the order the call lists them).
`acc_dtype=np.float32` makes the insert accumulate in float32 in that same
order: the sum that decides the stored bf16/f32 code is then taken in the
precision the kernel uses, so stored sketches can be compared bit for bit.

Readings of points the paper leaves open (hash family, sign function, median
for an even number of rows, tie-breaks, scope of one sketch) are stated at the
functions that take them.

Pins: every function here is checked in tests/test_oracle_pins.py against
closed forms, invariants, library routines, brute force or a figure the paper
prints; none is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

MASK64 = (1 << 64) - 1
LCG_MUL = 6364136223846793005      # Knuth's MMIX linear congruential constants
LCG_INC = 1442695040888963407


# ---------------------------------------------------------------------------
# hash and sign functions (Vague Sketch: "r distinct hash functions h_1..h_r"
# and the random +-1 coefficients g_i; the paper names no family)
# ---------------------------------------------------------------------------
def hash_params_from_seed(seed: int, r: int):
    """r rows of (a, b, c, d): a 64-bit LCG started at `seed` is stepped once per
    drawn word, rows in order, words in the order a, b, c, d; a and c are then
    forced odd."""
    x = seed & MASK64
    rows = []
    for _ in range(r):
        words = []
        for _ in range(4):
            x = (x * LCG_MUL + LCG_INC) & MASK64
            words.append(x)
        a, b, c, d = words
        rows.append((a | 1, b, c | 1, d))
    return rows


def bucket_of(row_params, J: int, w: int) -> int:
    """h_i(J): multiply-add on 64 bits, keep the high 32 bits, scale to [0, w)."""
    a, b, _, _ = row_params
    u = (a * J + b) & MASK64
    return ((u >> 32) * w) >> 32


def sign_of(row_params, J: int) -> int:
    """g_i(J) in {+1, -1}: top bit of a second multiply-add."""
    _, _, c, d = row_params
    s = (c * J + d) & MASK64
    return -1 if (s >> 63) else 1


# ---------------------------------------------------------------------------
# storage rounding
# ---------------------------------------------------------------------------
def to_storage(x, storage: str) -> np.ndarray:
    """Round to the storage type (nearest, ties to even); result as float64.
    float32 input is rounded from float32, float64 input directly from float64
    (a single rounding in both cases)."""
    x = np.asarray(x)
    if storage == "f64":
        return x.astype(np.float64)
    if storage == "f32":
        return x.astype(np.float32).astype(np.float64)
    if storage != "bf16":
        raise ValueError(storage)
    if x.dtype == np.float32:
        b = x.copy().view(np.uint32)
        lsb = (b >> np.uint32(16)) & np.uint32(1)
        b = (b + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
        return b.view(np.float32).astype(np.float64)
    x = x.astype(np.float64)
    ax = np.abs(x)
    if np.any((ax != 0) & ((ax < 2.0 ** -100) | ~(ax < 2.0 ** 100))):
        raise ValueError("oracle bf16 rounding handles 0 and 2^-100 <= |x| < 2^100 only")
    b = x.copy().view(np.uint64)
    lsb = (b >> np.uint64(45)) & np.uint64(1)
    b = (b + np.uint64((1 << 44) - 1) + lsb) & np.uint64(MASK64 ^ ((1 << 45) - 1))
    return b.view(np.float64)


# ---------------------------------------------------------------------------
# Algorithm 1: insert tokens into the Vague sketch
# ---------------------------------------------------------------------------
def sketch_zeros(r: int, w: int, D: int):
    """All slots start at zero (Vague Sketch, first paragraph)."""
    return np.zeros((r, w, D)), np.zeros((r, w, D))


def insert(SK, SV, params, tok_pos, K_tok, V_tok, *, storage="f64",
           acc_dtype=np.float64, sign_mask=2, coef=None):
    """V.Insert for a batch of tokens, in list order.

    For each token with index J and each row i:
        SK[i][h_i(J)] += key,   SV[i][h_i(J)] += value * g_i(J)
    Keys are not signed (sign_mask bit 0 clear) and values are (bit 1 set), as
    in Algorithm 1; the other settings of sign_mask exist for experiments.
    coef (optional, +1 or -1 per listed token) turns an entry into V.Delete of
    Algorithm 3's swap loop: the same slots, the contribution subtracted.
    Returns new (SK, SV); slots that receive nothing keep their content.
    """
    r, w, _ = SK.shape
    SK = SK.copy()
    SV = SV.copy()
    acc_k, acc_v = {}, {}
    for n, J in enumerate(tok_pos):
        J = int(J)
        cf = 1 if coef is None else int(coef[n])
        if cf not in (1, -1):
            raise ValueError("coef entries are +1 (insert) or -1 (delete)")
        for i in range(r):
            s = bucket_of(params[i], J, w)
            g = sign_of(params[i], J)
            key = (i, s)
            if key not in acc_k:
                acc_k[key] = SK[i, s].astype(acc_dtype)
                acc_v[key] = SV[i, s].astype(acc_dtype)
            gk = cf * (g if (sign_mask & 1) else 1)
            gv = cf * (g if (sign_mask & 2) else 1)
            acc_k[key] = acc_k[key] + acc_dtype(gk) * np.asarray(K_tok[n]).astype(acc_dtype)
            acc_v[key] = acc_v[key] + acc_dtype(gv) * np.asarray(V_tok[n]).astype(acc_dtype)
    for (i, s), v in acc_k.items():
        SK[i, s] = to_storage(v, storage)
    for (i, s), v in acc_v.items():
        SV[i, s] = to_storage(v, storage)
    return SK, SV


# ---------------------------------------------------------------------------
# Algorithm 2: query tokens from the Vague sketch
# ---------------------------------------------------------------------------
def median_rows(res, median_mode="midmean", storage="f64"):
    """Element-wise median over axis 1 of res [n, r, D].  Odd r: the middle order
    statistic.  Even r (the paper fixes r = 3 and never meets this): "midmean" =
    mean of the two middle order statistics, rounded to storage; "lower" = the
    lower of the two."""
    r = res.shape[1]
    srt = np.sort(res, axis=1)
    if r % 2 == 1:
        return srt[:, r // 2]
    lo, hi = srt[:, r // 2 - 1], srt[:, r // 2]
    if median_mode == "lower":
        return lo
    return to_storage(0.5 * (lo + hi), storage)


def query(SK, SV, params, tok_pos, *, storage="f64", median_mode="midmean", sign_mask=2):
    """V.Query for a batch of token indices: per row i collect
    <SK[i][h_i(J)], SV[i][h_i(J)] * g_i(J)>, return the element-wise median over
    the r rows.  Returns (K_hat, V_hat), float64 [n, D]."""
    r, w, D = SK.shape
    n = len(tok_pos)
    res_k = np.zeros((n, r, D))
    res_v = np.zeros((n, r, D))
    for t, J in enumerate(tok_pos):
        J = int(J)
        for i in range(r):
            s = bucket_of(params[i], J, w)
            g = sign_of(params[i], J)
            res_k[t, i] = SK[i, s] * (g if (sign_mask & 1) else 1)
            res_v[t, i] = SV[i, s] * (g if (sign_mask & 2) else 1)
    if n == 0:
        return np.zeros((0, D)), np.zeros((0, D))
    return (median_rows(res_k, median_mode, storage),
            median_rows(res_v, median_mode, storage))


# ---------------------------------------------------------------------------
# Recent / Candidate / Vague partition (Algorithm 3 without the swap loop)
# ---------------------------------------------------------------------------
def select(scores, ret_pos, n_ctx: int, n_recent: int, k_candidate: int):
    """Which retained tokens move to the Vague part.

    ret_pos[s] is the position of the token held in retained slot s (-1: empty).
    Recent = the n_recent newest positions (>= n_ctx - n_recent).  Of the other
    retained tokens the k_candidate with the highest cumulative score stay as
    Candidate; the rest are popped (lowest scores first in the paper's heap; the
    set is what matters) and returned.  Ties: the earlier position ranks higher.
    Returns (evict_slots, evict_pos), both in ascending slot order.
    """
    recent_from = n_ctx - n_recent
    elig = [s for s in range(len(ret_pos)) if 0 <= ret_pos[s] < recent_from]
    order = sorted(elig, key=lambda s: (-float(scores[ret_pos[s]]), int(ret_pos[s])))
    keep = set(order[:max(0, k_candidate)])
    ev = [s for s in elig if s not in keep]
    return (np.array(ev, dtype=np.int64),
            np.array([ret_pos[s] for s in ev], dtype=np.int64))


# ---------------------------------------------------------------------------
# Algorithm 3, swap loop: a Vague token that has become important enough
# changes places with the least important Candidate token
# ---------------------------------------------------------------------------
def swap_pick(scores, ret_pos, vague_pos, n_ctx: int, n_recent: int, replace_rate):
    """One evaluation of the loop condition
        C.Min_Score() * ReplaceRate < V.Max_Score().
    Candidate = retained tokens that are not Recent (position < n_ctx - n_recent).
    C.Min: lowest cumulative score, ties: the later position (the order in which
    `select` would pop them).  V.Max: highest cumulative score among the Vague
    tokens, ties: the earlier position.  The product and the comparison are taken
    in float32, the type the scores are kept in.  Returns (slot of the Candidate
    minimum, index into vague_pos of the Vague maximum) or None when the condition
    does not hold (or either part is empty)."""
    recent_from = n_ctx - n_recent
    cand = [s for s in range(len(ret_pos)) if 0 <= ret_pos[s] < recent_from]
    if not cand or len(vague_pos) == 0:
        return None
    s_min = min(cand, key=lambda s: (float(scores[ret_pos[s]]), -int(ret_pos[s])))
    i_max = min(range(len(vague_pos)),
                key=lambda i: (-float(scores[vague_pos[i]]), int(vague_pos[i])))
    lhs = np.float32(scores[ret_pos[s_min]]) * np.float32(replace_rate)
    if not (np.float32(lhs) < np.float32(scores[vague_pos[i_max]])):
        return None
    return s_min, i_max


def swap_once(SK, SV, params, K_ret, V_ret, ret_pos, vague_pos, s_min: int, i_max: int, *,
              storage="f64", acc_dtype=np.float64, median_mode="midmean", sign_mask=2):
    """The body of the swap loop for the chosen pair (Algorithm 3, second loop):
    query the Vague token J, delete that estimate from the sketch, insert the
    popped Candidate, push the estimate into the Candidate part.
    J = vague_pos[i_max]; the popped Candidate sits in retained slot s_min.
    V.Delete subtracts the queried estimate tmp from exactly the slots that an
    insert of J adds to (with the same signs); Delete and Insert form one sketch
    update in that order (a slot that both touch is rounded to storage once).
    The Candidate's slot then holds tmp at position J, and J's entry of the Vague
    index list is overwritten with the popped token's position.
    Returns new (SK, SV); K_ret, V_ret, ret_pos, vague_pos are modified in place."""
    J = int(vague_pos[i_max])
    pc = int(ret_pos[s_min])
    k_hat, v_hat = query(SK, SV, params, [J], storage=storage, median_mode=median_mode,
                         sign_mask=sign_mask)
    SK, SV = insert(SK, SV, params, [J, pc],
                    [k_hat[0], np.array(K_ret[s_min], copy=True)],
                    [v_hat[0], np.array(V_ret[s_min], copy=True)],
                    storage=storage, acc_dtype=acc_dtype, sign_mask=sign_mask, coef=[-1, 1])
    K_ret[s_min] = k_hat[0]
    V_ret[s_min] = v_hat[0]
    ret_pos[s_min] = J
    vague_pos[i_max] = pc
    return SK, SV


# ---------------------------------------------------------------------------
# Algorithm 4 (rebuild the KV cache) and the attention that follows it
# ---------------------------------------------------------------------------
def revive(K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx: int, *,
           storage="f64", median_mode="midmean", sign_mask=2):
    """KV[p] for every position p < n_ctx: V.Query(p) if p is in the Vague part,
    else the raw token from its retained slot.  Returns K*, V* [n_ctx, D]."""
    D = SK.shape[2]
    K = np.zeros((n_ctx, D))
    V = np.zeros((n_ctx, D))
    seen = np.zeros(n_ctx, dtype=bool)
    kq, vq = query(SK, SV, params, vague_pos, storage=storage,
                   median_mode=median_mode, sign_mask=sign_mask)
    for t, p in enumerate(vague_pos):
        K[p], V[p] = kq[t], vq[t]
        seen[p] = True
    for s, p in enumerate(ret_pos):
        if p >= 0:
            if seen[p]:
                raise ValueError(f"position {p} is in two parts")
            K[p], V[p] = K_ret[s], V_ret[s]
            seen[p] = True
    if not seen.all():
        raise ValueError("some position below n_ctx is in no part")
    return K, V


def attention(q, K, V, scale: float):
    """p = softmax(q K^T * scale) row-wise, o = p V.  q [G, D]; returns (o [G, D],
    p [G, n])."""
    logits = (np.asarray(q, dtype=np.float64) @ K.T) * scale
    logits = logits - logits.max(axis=1, keepdims=True)
    e = np.exp(logits)
    p = e / e.sum(axis=1, keepdims=True)
    return p @ V, p


def attend_decode(q, K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx, scale, *,
                  scores=None, storage="f64", median_mode="midmean", sign_mask=2):
    """Calculation phase of one unit: rebuild, attend with the G query heads of
    this kv head, and add each token's probability (summed over the G heads)
    to its cumulative score.  Returns (out [G, D] float64, new scores float32 or
    None, p [G, n_ctx])."""
    K, V = revive(K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx,
                  storage=storage, median_mode=median_mode, sign_mask=sign_mask)
    out, p = attention(q, K, V, scale)
    new_scores = None
    if scores is not None:
        new_scores = np.array(scores, dtype=np.float32, copy=True)
        inc = p.sum(axis=0)
        new_scores[:n_ctx] = (new_scores[:n_ctx].astype(np.float64) + inc).astype(np.float32)
    return out, new_scores, p


def attend_multi(q, q_pos, K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx, scale, *,
                 scores=None, storage="f64", median_mode="midmean", sign_mask=2):
    """Calculation phase for several query tokens at once (a chunk of prompt or
    of drafted tokens): the cache is rebuilt once (Algorithm 4), then query t,
    which sits at position q_pos[t], attends over the positions <= q_pos[t]
    (a token does not see later tokens), with the G query heads of this kv head.
    Every token's cumulative score grows by its probability summed over the
    queries and heads.  q [Tq, G, D].  Returns (out [Tq, G, D] float64, new scores
    float32 or None, p [Tq, G, n_ctx] with zeros at the positions a query does not
    see)."""
    K, V = revive(K_ret, V_ret, ret_pos, SK, SV, params, vague_pos, n_ctx,
                  storage=storage, median_mode=median_mode, sign_mask=sign_mask)
    q = np.asarray(q, dtype=np.float64)
    Tq, G, D = q.shape
    out = np.zeros((Tq, G, D))
    p_all = np.zeros((Tq, G, n_ctx))
    for t in range(Tq):
        n_vis = int(q_pos[t]) + 1
        if not (1 <= n_vis <= n_ctx):
            raise ValueError("query position outside the context")
        o, p = attention(q[t], K[:n_vis], V[:n_vis], scale)
        out[t] = o
        p_all[t, :, :n_vis] = p
    new_scores = None
    if scores is not None:
        new_scores = np.array(scores, dtype=np.float32, copy=True)
        inc = p_all.sum(axis=(0, 1))
        new_scores[:n_ctx] = (new_scores[:n_ctx].astype(np.float64) + inc).astype(np.float32)
    return out, new_scores, p_all


# ---------------------------------------------------------------------------
# one unit's whole state and one decode step
# ---------------------------------------------------------------------------
class UnitState:
    """Storage of one (layer, sequence, kv head): retained slots, sketch, scores,
    Vague index list."""

    def __init__(self, ret_cap, n_cap, r, w, D, params, storage, *, n_recent, k_candidate,
                 median_mode="midmean", sign_mask=2, acc_dtype=np.float64):
        self.K_ret = np.zeros((ret_cap, D))
        self.V_ret = np.zeros((ret_cap, D))
        self.ret_pos = np.full(ret_cap, -1, dtype=np.int64)
        self.scores = np.zeros(n_cap, dtype=np.float32)
        self.SK, self.SV = sketch_zeros(r, w, D)
        self.vague_pos = []
        self.n_ctx = 0
        self.r_size = 0              # R.size: the Recent queue holds the r_size newest positions
        self.params = params
        self.storage = storage
        self.n_recent = n_recent
        self.k_candidate = k_candidate
        self.median_mode = median_mode
        self.sign_mask = sign_mask
        self.acc_dtype = acc_dtype

    def free_slots(self):
        return [s for s in range(len(self.ret_pos)) if self.ret_pos[s] < 0]

    def append(self, k, v, slot=None):
        """Push the newly generated token into the Recent part (a free slot)."""
        if slot is None:
            slot = self.free_slots()[0]
        if self.ret_pos[slot] >= 0:
            raise ValueError("slot in use")
        self.K_ret[slot] = k
        self.V_ret[slot] = v
        self.ret_pos[slot] = self.n_ctx
        self.n_ctx += 1
        self.r_size += 1             # R.Push(T)
        return slot

    def compress(self, slack=0):
        """Algorithm 3 without the swap loop, after the push of the new token.  The
        Recent part is a queue over the r_size newest positions; n_recent is its
        budget.  First branch: only when the queue has outgrown its budget by more
        than `slack` do its oldest (size - budget) tokens leave it for the Candidate
        part, all at once.  Then, as long as the Candidate part is over its budget,
        its lowest-score token moves into the sketch (one insert call in ascending
        slot order: a slot shared by several of them is rounded once).
        slack = 0: one token in, one token out per step."""
        if self.r_size > self.n_recent + slack:
            self.r_size = self.n_recent
        ev_slots, ev_pos = select(self.scores, self.ret_pos, self.n_ctx,
                                  self.r_size, self.k_candidate)
        if len(ev_slots):
            self.SK, self.SV = insert(self.SK, self.SV, self.params, ev_pos,
                                      self.K_ret[ev_slots], self.V_ret[ev_slots],
                                      storage=self.storage, acc_dtype=self.acc_dtype,
                                      sign_mask=self.sign_mask)
            for s in ev_slots:
                self.ret_pos[s] = -1
            self.vague_pos.extend(int(p) for p in ev_pos)
        return ev_slots, ev_pos

    def swap_back(self, replace_rate, max_swaps):
        """The swap loop of Algorithm 3, at most max_swaps rounds.  Returns the
        list of (Vague position brought back, Candidate position sent out)."""
        done = []
        for _ in range(max_swaps):
            pick = swap_pick(self.scores, self.ret_pos, self.vague_pos, self.n_ctx,
                             self.r_size, replace_rate)
            if pick is None:
                break
            s_min, i_max = pick
            done.append((int(self.vague_pos[i_max]), int(self.ret_pos[s_min])))
            self.SK, self.SV = swap_once(
                self.SK, self.SV, self.params, self.K_ret, self.V_ret, self.ret_pos,
                self.vague_pos, s_min, i_max, storage=self.storage, acc_dtype=self.acc_dtype,
                median_mode=self.median_mode, sign_mask=self.sign_mask)
        return done

    def attend(self, q, scale):
        out, self.scores, p = attend_decode(
            q, self.K_ret, self.V_ret, self.ret_pos, self.SK, self.SV, self.params,
            self.vague_pos, self.n_ctx, scale, scores=self.scores, storage=self.storage,
            median_mode=self.median_mode, sign_mask=self.sign_mask)
        return out, p

    def decode_step(self, k_new, v_new, q, scale, *, replace_rate=None, max_swaps=0, slack=0):
        """append -> select -> insert -> (swap loop, if replace_rate is given) ->
        rebuild + attend + accumulate scores."""
        self.append(k_new, v_new)
        ev = self.compress(slack)
        if replace_rate is not None and max_swaps > 0:
            self.swap_back(replace_rate, max_swaps)
        out, p = self.attend(q, scale)
        return out, ev, p


def dense_prefill_state(K, V, q0, scale, r, w, params, storage, *, n_recent, k_candidate,
                        ret_cap=None, n_cap=None, **kw) -> UnitState:
    """State right after the prompt: all N tokens held raw, cumulative scores
    initialised with one dense attention pass of q0 (a stand-in for the scores a
    real prefill would have accumulated), nothing compressed yet."""
    N, D = K.shape
    st = UnitState(ret_cap or N, n_cap or N, r, w, D, params, storage,
                   n_recent=n_recent, k_candidate=k_candidate, **kw)
    st.K_ret[:N] = K
    st.V_ret[:N] = V
    st.ret_pos[:N] = np.arange(N)
    st.n_ctx = N
    st.r_size = N                    # every prompt token was pushed into the Recent queue
    _, p = attention(q0, st.K_ret[:N], st.V_ret[:N], scale)
    st.scores[:N] = p.sum(axis=0).astype(np.float32)
    return st


def compact(st: UnitState, ret_cap: int) -> UnitState:
    """Move the occupied retained slots, in ascending slot order, to the front of
    a smaller slot array (bookkeeping only; no arithmetic)."""
    used = [s for s in range(len(st.ret_pos)) if st.ret_pos[s] >= 0]
    if len(used) > ret_cap:
        raise ValueError("retained tokens exceed the new capacity")
    D = st.K_ret.shape[1]
    K = np.zeros((ret_cap, D))
    V = np.zeros((ret_cap, D))
    rp = np.full(ret_cap, -1, dtype=np.int64)
    K[:len(used)] = st.K_ret[used]
    V[:len(used)] = st.V_ret[used]
    rp[:len(used)] = st.ret_pos[used]
    st.K_ret, st.V_ret, st.ret_pos = K, V, rp
    return st
