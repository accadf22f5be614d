"""CPU oracle for the FreeKV retrieval-decode step.  TEST INFRASTRUCTURE ONLY.

A plain, slow, obviously-correct NumPy statement of what one decode step of one
(layer, request) computes, written from the paper:

  * decode attention and the GQA head mapping        -- Sec. 2.1
  * budget B with S sink and W window tokens kept    -- Sec. 2.1
  * min-max page summaries, page attention weights,
    softmax -> group mean pooling, top-k pages       -- Sec. 3.2 "Group-consistent selection"
  * reuse of the previous step's selection           -- Sec. 3.2 "Speculative retrieval"
  * cosine test, group mean, head-wise correction    -- Sec. 3.1 (definition of C_i), Sec. 3.3
  * which selected pages must be recalled            -- Sec. 4.1 (GPU cache of selected pages)
  * the alternative group poolings of the selection
    (Max/Mean over Q, QK, S) and of the correction    -- App. B.2, App. B.3

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
module.  It shares no code with the HIP path and never calls it.

Precision.  Attention and the cosine test are fp64.  The page score decides an
integer result (which pages are picked), so it is computed in the precision the
kernel uses and in ONE written-down order, all of it IEEE fp32/fp64 operations
that any conforming machine reproduces bit for bit:

  a. products q_c * s_c are exact in fp32 (fp16 and bf16 inputs), s_c being
     kmax_c if q_c >= 0 else kmin_c;
  b. the 128 products are summed in fp32 as 16 chunks of 8 consecutive
     channels (left to right inside a chunk), the 16 chunk sums then combined
     by a balanced binary tree over adjacent pairs;
  c. one fp32 multiply by fl32(1/sqrt(d));
  d. subtract the per-head maximum over the candidate pages (fp32);
  e. exp via exp_spec below (fp32 multiply, rint, exact subtract, degree-6
     Horner with separate fp32 multiply and add, ldexp);
  f. E = rint(e * 2^31) as an integer; the softmax denominator Z is the integer
     sum of E (no rounding, so no summation order);
  g. pooled score = fl32( (sum_g fp64(E_g)/fp64(Z_g), g ascending) / fp64(G) );
  h. top-k by (score descending, page id ascending); ids emitted ascending.

Inputs are float32 arrays whose values are exactly representable in the storage
type (fp16 or bf16); the oracle itself never rounds to a storage type.

Readings of points the paper leaves open are listed in the design notes; the
ones that matter here: the page weight is the channel-wise upper bound
sum_c max(q_c*kmax_c, q_c*kmin_c) (the min-max summaries of Sec. 3.2), scaled
by 1/sqrt(d); only candidate pages (not sink, window or the open page) enter the
softmax; sink and window are whole pages; the appended token is attended; the
first step corrects every head; correction is strict (C < tau) on the fp64
group mean; an uncorrected head attends with the reused pages.
"""
from __future__ import annotations

import dataclasses

import numpy as np

F32 = np.float32
F64 = np.float64

LOG2E_F32 = F32(1.4426950408889634)
# fl32((ln 2)^i / i!), i = 0..6
_LN2 = 0.6931471805599453
EXP_COEF = tuple(F32(_LN2 ** i / float(np.prod(np.arange(1, i + 1)) if i else 1.0)) for i in range(7))
TWO31_F32 = F32(2147483648.0)


# --------------------------------------------------------------------------
# Sec. 2.1: dense decode attention (the definition everything reduces to)
# --------------------------------------------------------------------------
def dense_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray) -> np.ndarray:
    """o_h = softmax(q_h K_m^T / sqrt(d)) V_m with m = h // G  (Sec. 2.1).

    q [n_q, d]; K, V [L, n_kv, d]; returns [n_q, d] in fp64.
    """
    n_q, d = q.shape
    n_kv = K.shape[1]
    G = n_q // n_kv
    out = np.zeros((n_q, d), dtype=F64)
    for h in range(n_q):
        m = h // G
        s = K[:, m, :].astype(F64) @ q[h].astype(F64) / np.sqrt(F64(d))
        w = np.exp(s - s.max())
        w /= w.sum()
        out[h] = w @ V[:, m, :].astype(F64)
    return out


# --------------------------------------------------------------------------
# Sec. 3.2: page summaries and page attention weights
# --------------------------------------------------------------------------
def page_summaries(K: np.ndarray, page_size: int):
    """Channel-wise max and min of the keys of each page (min-max pooling, Sec. 3.2).

    K [L, n_kv, d] -> kmax, kmin [ceil(L/p), n_kv, d].  A partial last page is
    summarised over the tokens it holds.
    """
    L = K.shape[0]
    n_page = (L + page_size - 1) // page_size
    kmax = np.empty((n_page,) + K.shape[1:], dtype=F32)
    kmin = np.empty_like(kmax)
    for j in range(n_page):
        blk = K[j * page_size:min((j + 1) * page_size, L)]
        kmax[j] = blk.max(axis=0)
        kmin[j] = blk.min(axis=0)
    return kmax, kmin


def _canonical_sum128(t: np.ndarray) -> np.ndarray:
    """fp32 sum over the last axis (128 terms) in the written-down order (b)."""
    assert t.dtype == F32 and t.shape[-1] == 128
    c = t.reshape(t.shape[:-1] + (16, 8))
    s = c[..., 0]
    for u in range(1, 8):
        s = s + c[..., u]
    while s.shape[-1] > 1:
        s = s[..., 0::2] + s[..., 1::2]
    return s[..., 0]


def page_weights(q: np.ndarray, kmax: np.ndarray, kmin: np.ndarray) -> np.ndarray:
    """P^h_j for every head h and page j (steps a-c).  q [n_q, d]; kmax/kmin [n_page, n_kv, d] -> [n_q, n_page] fp32."""
    n_q, d = q.shape
    n_kv = kmax.shape[1]
    G = n_q // n_kv
    q = q.astype(F32)
    scale = F32(1.0 / np.sqrt(F64(d)))
    P = np.empty((n_q, kmax.shape[0]), dtype=F32)
    for h in range(n_q):
        m = h // G
        s = np.where(q[h] >= 0, kmax[:, m, :], kmin[:, m, :]).astype(F32)
        P[h] = _canonical_sum128(q[h][None, :] * s) * scale
    return P


def exp_spec(x: np.ndarray) -> np.ndarray:
    """The fp32 exponential of step (e), for x <= 0."""
    x = np.asarray(x, dtype=F32)
    t = x * LOG2E_F32
    n = np.rint(t)
    f = t - n
    p = np.full_like(f, EXP_COEF[6])
    for i in range(5, -1, -1):
        p = p * f
        p = p + EXP_COEF[i]
    e = np.ldexp(p, n.astype(np.int32)).astype(F32)
    return np.where(t < F32(-64.0), F32(0.0), e)


SELECT_POOLINGS = ("MeanS", "MaxS", "MeanQK", "MaxQK", "MeanQ", "MaxQ")
CORR_POOLINGS = ("mean", "max", "min")


def pool_queries(q: np.ndarray, G: int, pooling: str) -> np.ndarray:
    """Group-pooled query vectors (App. B.2, variants "Q"): [n_q, d] -> [n_kv, d] fp32.

    MeanQ: channel-wise fp32 sum over the group in head order, divided by fl32(G);
    MaxQ: channel-wise maximum.
    """
    n_q, d = q.shape
    n_kv = n_q // G
    q = q.astype(F32)
    out = np.empty((n_kv, d), dtype=F32)
    for m in range(n_kv):
        acc = q[m * G].copy()
        for g in range(1, G):
            acc = (acc + q[m * G + g]) if pooling == "MeanQ" else np.maximum(acc, q[m * G + g])
        out[m] = acc / F32(G) if pooling == "MeanQ" else acc
    return out


def pooled_scores(P: np.ndarray, G: int, pooling: str = "MeanS") -> np.ndarray:
    """Group-consistent page scores: P [n_q, n_cand] -> [n_kv, n_cand] fp32.

    MeanS (the method, Sec. 3.2): score_{m,j} = (1/G) sum_g softmax_j(P^{mG+g}), steps d-g.
    Alternatives of App. B.2: MaxS (maximum over the group of the softmax values), MeanQK / MaxQK
    (mean / maximum over the group of the weights themselves: fp32 sum in head order divided by
    fl32(G), or the maximum), and MeanQ / MaxQ, where P already holds one row per KV head
    (weights of the pooled query) and is the score.
    """
    assert pooling in SELECT_POOLINGS
    if pooling in ("MeanQ", "MaxQ"):
        return P.astype(F32)
    n_q, n_cand = P.shape
    n_kv = n_q // G
    if n_cand == 0:
        return np.zeros((n_kv, 0), dtype=F32)
    score = np.empty((n_kv, n_cand), dtype=F32)
    if pooling in ("MeanQK", "MaxQK"):
        for m in range(n_kv):
            acc = P[m * G].astype(F32)
            for g in range(1, G):
                acc = (acc + P[m * G + g]) if pooling == "MeanQK" else np.maximum(acc, P[m * G + g])
            score[m] = acc / F32(G) if pooling == "MeanQK" else acc
        return score
    M = P.max(axis=1, keepdims=True)
    e = exp_spec(P - M)
    E = np.rint(e * TWO31_F32).astype(np.uint64)
    Z = E.sum(axis=1)
    for m in range(n_kv):
        acc = None
        for g in range(G):
            h = m * G + g
            s_g = E[h].astype(F64) / F64(Z[h])
            if acc is None:
                acc = s_g if pooling == "MaxS" else np.zeros(n_cand, dtype=F64) + s_g
            else:
                acc = np.maximum(acc, s_g) if pooling == "MaxS" else acc + s_g
        score[m] = acc.astype(F32) if pooling == "MaxS" else (acc / F64(G)).astype(F32)
    return score


def topk_pages(score: np.ndarray, k: int) -> np.ndarray:
    """The k highest-scoring positions, ties to the lower position, returned ascending (step h)."""
    n = score.shape[0]
    k = min(k, n)
    order = np.lexsort((np.arange(n), -score.astype(F64)))
    return np.sort(order[:k]).astype(np.int32)


# --------------------------------------------------------------------------
# Sec. 3.1 / 3.3: query similarity and the correction test
# --------------------------------------------------------------------------
def query_cosine(q: np.ndarray, q_prev: np.ndarray) -> np.ndarray:
    """C = <q, q_prev> / (|q| |q_prev|) per head (Sec. 3.1), fp64; 0 when a norm is 0."""
    a = q.astype(F64)
    b = q_prev.astype(F64)
    dot = np.zeros(a.shape[0], dtype=F64)
    na = np.zeros(a.shape[0], dtype=F64)
    nb = np.zeros(a.shape[0], dtype=F64)
    for c in range(a.shape[1]):          # channels in order, all heads at once
        dot = dot + a[:, c] * b[:, c]
        na = na + a[:, c] * a[:, c]
        nb = nb + b[:, c] * b[:, c]
    den = np.sqrt(na * nb)
    C = np.where(den > 0, dot / np.where(den > 0, den, 1.0), 0.0)
    return C


def correction_flags(C: np.ndarray, G: int, tau: float, pooling: str = "mean") -> np.ndarray:
    """A KV head is corrected iff the group-pooled C is strictly below tau (Sec. 3.3).

    pooling "mean" is the method; "max" is the alternative of App. B.3 taken literally (the largest
    similarity of the group); "min" corrects as soon as any head of the group is below tau.
    """
    assert pooling in CORR_POOLINGS
    n_kv = C.shape[0] // G
    flags = np.zeros(n_kv, dtype=np.uint8)
    for m in range(n_kv):
        acc = F64(C[m * G])
        for g in range(1, G):
            c = F64(C[m * G + g])
            acc = acc + c if pooling == "mean" else (max(acc, c) if pooling == "max" else min(acc, c))
        pooled = acc / F64(G) if pooling == "mean" else acc
        flags[m] = 1 if pooled < F64(F32(tau)) else 0
    return flags


# --------------------------------------------------------------------------
# geometry of the budget (Sec. 2.1: B, S, W)
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class Geometry:
    L: int
    n_full: int     # full pages
    r: int          # tokens in the open page
    n_sink: int     # sink pages
    n_win: int      # window pages (full pages just before the open page)
    cand_lo: int    # first candidate page
    n_cand: int     # candidate pages [cand_lo, cand_lo + n_cand)
    k_eff: int      # pages picked per KV head


def geometry(L: int, p: int, budget: int, sink: int, window: int) -> Geometry:
    n_full, r = divmod(L, p)
    n_sink = min(sink // p, n_full)
    n_win = min(window // p, n_full - n_sink)
    n_cand = n_full - n_sink - n_win
    k = (budget - sink - window) // p
    return Geometry(L, n_full, r, n_sink, n_win, n_sink, n_cand, min(k, n_cand))


# --------------------------------------------------------------------------
# the stateful step
# --------------------------------------------------------------------------
class FreeKVOracle:
    """State of one (layer, request) and the decode step on it."""

    def __init__(self, n_q: int, n_kv: int, d: int, p: int, budget: int, sink: int,
                 window: int, tau: float, max_ctx: int, select_pooling: str = "MeanS",
                 corr_pooling: str = "mean"):
        assert n_q % n_kv == 0 and budget % p == 0 and sink % p == 0 and window % p == 0
        self.n_q, self.n_kv, self.d, self.p = n_q, n_kv, d, p
        self.G = n_q // n_kv
        self.budget, self.sink, self.window, self.tau = budget, sink, window, tau
        self.k = (budget - sink - window) // p
        self.max_ctx = max_ctx
        self.select_pooling, self.corr_pooling = select_pooling, corr_pooling
        max_pages = (max_ctx + p - 1) // p
        self.K = np.zeros((max_ctx, n_kv, d), dtype=F32)
        self.V = np.zeros((max_ctx, n_kv, d), dtype=F32)
        self.kmax = np.zeros((max_pages, n_kv, d), dtype=F32)
        self.kmin = np.zeros((max_pages, n_kv, d), dtype=F32)
        self.L = 0
        self.q_prev = None
        self.active = np.full((n_kv, self.k), -1, dtype=np.int32)
        self.resident = [set() for _ in range(n_kv)]

    # -- data plane ---------------------------------------------------------
    def append(self, k_new: np.ndarray, v_new: np.ndarray) -> None:
        """Store one token and fold its key into the open page's summary (Sec. 3.2)."""
        t = self.L
        assert t < self.max_ctx
        self.K[t] = k_new
        self.V[t] = v_new
        j, pos = divmod(t, self.p)
        if pos == 0:
            self.kmax[j] = k_new
            self.kmin[j] = k_new
        else:
            self.kmax[j] = np.maximum(self.kmax[j], k_new)
            self.kmin[j] = np.minimum(self.kmin[j], k_new)
        self.L = t + 1

    def load_prefix(self, K: np.ndarray, V: np.ndarray) -> None:
        for t in range(K.shape[0]):
            self.append(K[t], V[t])

    def load_prefix_bulk(self, K: np.ndarray, V: np.ndarray) -> None:
        """Same state as load_prefix, built with page_summaries (for long prefixes)."""
        assert self.L == 0
        n = K.shape[0]
        self.K[:n] = K
        self.V[:n] = V
        kmax, kmin = page_summaries(K, self.p)
        self.kmax[:kmax.shape[0]] = kmax
        self.kmin[:kmin.shape[0]] = kmin
        self.L = n

    def geom(self) -> Geometry:
        return geometry(self.L, self.p, self.budget, self.sink, self.window)

    # -- selection (Sec. 3.2) ------------------------------------------------
    def select(self, q: np.ndarray):
        """Sel(q): page ids per KV head [n_kv, k] (ascending, -1 padded), with the weights and scores it used."""
        g = self.geom()
        lo, hi = g.cand_lo, g.cand_lo + g.n_cand
        if self.select_pooling in ("MeanQ", "MaxQ"):
            q = pool_queries(q, self.G, self.select_pooling)      # one pooled query per KV head
        P = page_weights(q, self.kmax[lo:hi], self.kmin[lo:hi])
        score = pooled_scores(P, self.G, self.select_pooling)
        ids = np.full((self.n_kv, self.k), -1, dtype=np.int32)
        for m in range(self.n_kv):
            top = topk_pages(score[m], g.k_eff)
            ids[m, :top.shape[0]] = top + lo
        return ids, P, score

    # -- attention over sink + chosen pages + window + open page (Sec. 2.1) ---
    def attended_tokens(self, page_ids: np.ndarray) -> np.ndarray:
        g = self.geom()
        p = self.p
        pages = list(range(g.n_sink))
        pages += [int(j) for j in page_ids if j >= 0]
        pages += list(range(g.n_full - g.n_win, g.n_full))
        assert len(set(pages)) == len(pages), "a chosen page lies inside sink or window"
        tok = [np.arange(j * p, (j + 1) * p) for j in pages]
        if g.r:
            tok.append(np.arange(g.n_full * p, g.L))
        return np.concatenate(tok) if tok else np.zeros(0, dtype=np.int64)

    def attend(self, q: np.ndarray, ids: np.ndarray) -> np.ndarray:
        """ids [n_kv, k]; returns [n_q, d] fp64."""
        out = np.zeros((self.n_q, self.d), dtype=F64)
        for m in range(self.n_kv):
            tok = self.attended_tokens(ids[m])
            Ks = self.K[tok, m, :].astype(F64)
            Vs = self.V[tok, m, :].astype(F64)
            for gq in range(self.G):
                h = m * self.G + gq
                s = Ks @ q[h].astype(F64) / np.sqrt(F64(self.d))
                w = np.exp(s - s.max())
                w /= w.sum()
                out[h] = w @ Vs
        return out

    # -- the pages a head attends, laid out token-major with all heads side by side (Sec. 4.2) --
    def export_nhd(self, ids: np.ndarray, n_slots: int):
        """The NHD-layout GPU pool of the paper's hybrid layouts, for the page lists `ids` [n_kv, k]:
        pool [n_slots, 2 (K, V), p, n_kv, d] and slot_pages [n_kv, n_slots].  Slot s of head m holds the
        s-th page of m's attend list -- sink pages, then the k chosen pages in the order of `ids` (an
        unused entry leaves its slot empty), then the window pages, then the open page; an empty slot
        has page -1 and zeros, and so have the tokens of the open page that do not exist yet."""
        g = self.geom()
        p = self.p
        pool = np.zeros((n_slots, 2, p, self.n_kv, self.d), dtype=F32)
        slot_pages = np.full((self.n_kv, n_slots), -1, dtype=np.int32)
        for m in range(self.n_kv):
            pages = list(range(g.n_sink)) + [int(j) for j in ids[m]] + list(range(g.n_full - g.n_win, g.n_full))
            if g.r:
                pages.append(g.n_full)
            assert len(pages) <= n_slots
            for s, page in enumerate(pages):
                if page < 0:
                    continue
                n_tok = min(p, self.L - page * p)
                slot_pages[m, s] = page
                pool[s, 0, :n_tok, m, :] = self.K[page * p:page * p + n_tok, m, :]
                pool[s, 1, :n_tok, m, :] = self.V[page * p:page * p + n_tok, m, :]
        return pool, slot_pages

    # -- one decode step -------------------------------------------------------
    def step(self, q: np.ndarray, k_new: np.ndarray, v_new: np.ndarray) -> dict:
        self.append(k_new, v_new)
        new_ids, P, score = self.select(q)
        if self.q_prev is None:
            C = np.zeros(self.n_q, dtype=F64)
            flags = np.ones(self.n_kv, dtype=np.uint8)
        else:
            C = query_cosine(q, self.q_prev)
            flags = correction_flags(C, self.G, self.tau, self.corr_pooling)
        used = np.where(flags[:, None] != 0, new_ids, self.active)
        out = self.attend(q, used)
        # pages of Sel(q_i) not in the GPU cache of selected pages: those of the
        # previous selection are there, every other one has to be recalled.
        miss = []
        for m in range(self.n_kv):
            new_set = {int(j) for j in new_ids[m] if j >= 0}
            miss.append(sorted(new_set - self.resident[m]))
            self.resident[m] = new_set
        self.active = new_ids
        self.q_prev = np.array(q, dtype=F32, copy=True)
        return dict(out=out, new_ids=new_ids, used_ids=used, flags=flags, cosine=C,
                    P=P, score=score, miss=miss, geom=self.geom())
