"""Do the oracle's pins have teeth?  Each case plants one plausible mistake in the oracle (a swapped
operand, a dropped factor, a wrong comparison, a wrong index, another summation order) and asserts
that at least one pin of tests/test_oracle_pins.py then fails.  CPU only; the mistakes live for the
duration of one test."""
import numpy as np
import pytest

import test_oracle_pins as pins
from oracle import freekv_oracle as O

F32, F64 = np.float32, np.float64


def _pin_calls():
    """Every pin as a zero-argument callable, parametrised ones expanded."""
    calls = []
    for name in sorted(dir(pins)):
        fn = getattr(pins, name)
        if not name.startswith("test_") or not callable(fn):
            continue
        marks = [m for m in getattr(fn, "pytestmark", []) if m.name == "parametrize"]
        if not marks:
            calls.append((name, _call_page_set_pin if name == PAGE_SET_PIN else fn))
            continue
        argnames = [a.strip() for a in marks[0].args[0].split(",")]
        for values in marks[0].args[1]:
            values = values if isinstance(values, (tuple, list)) else (values,)
            calls.append((f"{name}{list(values)}", lambda fn=fn, kw=dict(zip(argnames, values)): fn(**kw)))
    return calls


def _first_failing_pin():
    for name, call in _pin_calls():
        try:
            call()
        except Exception:                 # noqa: BLE001 - any failure of a pin counts
            return name
    return None


def _all_failing_pins():
    failing = []
    for name, call in _pin_calls():
        try:
            call()
        except Exception:                 # noqa: BLE001
            failing.append(name)
    return failing


PAGE_SET_PIN = "test_selected_page_set_equals_the_plain_fp64_definition_except_at_near_ties"


def test_the_pins_pass_on_the_oracle_as_it_is():
    assert _first_failing_pin() is None


# ---- the mistakes -------------------------------------------------------------------
def _weights_swapped(q, kmax, kmin):
    return _orig["page_weights"](q, kmin, kmax)


def _weights_unscaled(q, kmax, kmin):
    return _orig["page_weights"](q, kmax, kmin) * F32(np.sqrt(128.0))


def _weights_head_modulo(q, kmax, kmin):
    n_kv = kmax.shape[1]
    perm = [(h % n_kv) * (q.shape[0] // n_kv) + h // n_kv for h in range(q.shape[0])]
    return _orig["page_weights"](q[perm], kmax, kmin)


def _sum_sequential(t):
    s = t[..., 0]
    for c in range(1, 128):
        s = s + t[..., c]
    return s


def _exp_degree5(x):
    x = np.asarray(x, dtype=F32)
    t = x * O.LOG2E_F32
    n = np.rint(t)
    f = t - n
    p = np.full_like(f, O.EXP_COEF[5])
    for i in range(4, -1, -1):
        p = p * f
        p = p + O.EXP_COEF[i]
    e = np.ldexp(p, n.astype(np.int32)).astype(F32)
    return np.where(t < F32(-64.0), F32(0.0), e)


def _pooled_softmax_of_mean(P, G, pooling="MeanS"):
    if pooling != "MeanS":
        return _orig["pooled_scores"](P, G, pooling)
    mean = P.reshape(-1, G, P.shape[1]).astype(F64).mean(axis=1)
    e = np.exp(mean - mean.max(axis=1, keepdims=True))
    return (e / e.sum(axis=1, keepdims=True)).astype(F32)


def _pooled_max_for_mean(P, G, pooling="MeanS"):
    return _orig["pooled_scores"](P, G, "MaxS" if pooling == "MeanS" else pooling)


def _topk_ties_to_higher(score, k):
    n = score.shape[0]
    order = np.lexsort((-np.arange(n), -score.astype(F64)))
    return np.sort(order[:min(k, n)]).astype(np.int32)


def _topk_lowest(score, k):
    return _orig["topk_pages"](-score, k)


def _flags_not_strict(C, G, tau, pooling="mean"):
    f = _orig["correction_flags"](C, G, tau, pooling)
    pooled = C.reshape(-1, G).mean(axis=1)
    return np.where(pooled == F64(F32(tau)), 1, f).astype(np.uint8)


def _flags_any_head(C, G, tau, pooling="mean"):
    return _orig["correction_flags"](C, G, tau, "min" if pooling == "mean" else pooling)


def _cosine_one_norm(q, q_prev):
    a, b = q.astype(F64), q_prev.astype(F64)
    return (a * b).sum(axis=1) / np.maximum((a * a).sum(axis=1), 1e-300)


def _summaries_swapped(K, page_size):
    kmax, kmin = _orig["page_summaries"](K, page_size)
    return kmin, kmax


def _summaries_drop_last_token(K, page_size):
    kmax, kmin = _orig["page_summaries"](K, page_size)
    if K.shape[0] % page_size == 0 and K.shape[0] >= page_size:
        blk = K[-page_size:-1]
        kmax[-1], kmin[-1] = blk.max(axis=0), blk.min(axis=0)
    return kmax, kmin


def _dense_unscaled(q, K, V):
    return _orig["dense_attention"](q * F32(np.sqrt(128.0)), K, V)


def _dense_head_modulo(q, K, V):
    n_q, n_kv = q.shape[0], K.shape[1]
    out = np.zeros((n_q, q.shape[1]), dtype=F64)
    for h in range(n_q):
        out[h] = _orig["dense_attention"](q[h:h + 1], K[:, h % n_kv:h % n_kv + 1], V[:, h % n_kv:h % n_kv + 1])[0]
    return out


def _geometry_window_one_short(L, p, budget, sink, window):
    g = _orig["geometry"](L, p, budget, sink, window)
    if g.n_win == 0:
        return g
    return O.Geometry(g.L, g.n_full, g.r, g.n_sink, g.n_win - 1, g.cand_lo, g.n_cand + 1, min((budget - sink - window) // p, g.n_cand + 1))


def _pool_queries_wrong_divisor(q, G, pooling):
    out = _orig["pool_queries"](q, G, pooling)
    return out * F32(G) / F32(q.shape[0]) if pooling == "MeanQ" else out


MODULE_MISTAKES = {
    "kmax and kmin swapped in the page weight": ("page_weights", _weights_swapped),
    "page weight without 1/sqrt(d)": ("page_weights", _weights_unscaled),
    "page weight with KV head h % n_kv": ("page_weights", _weights_head_modulo),
    "128-term sum in plain sequential order": ("_canonical_sum128", _sum_sequential),
    "exponential polynomial one degree short": ("exp_spec", _exp_degree5),
    "softmax of the mean instead of mean of the softmax": ("pooled_scores", _pooled_softmax_of_mean),
    "max over the group where the method takes the mean": ("pooled_scores", _pooled_max_for_mean),
    "top-k ties to the higher page id": ("topk_pages", _topk_ties_to_higher),
    "top-k of the lowest scores": ("topk_pages", _topk_lowest),
    "correction test with <= instead of <": ("correction_flags", _flags_not_strict),
    "correction as soon as any head is below tau": ("correction_flags", _flags_any_head),
    "cosine normalised by one norm only": ("query_cosine", _cosine_one_norm),
    "page maxima and minima swapped": ("page_summaries", _summaries_swapped),
    "summary of a full page misses its last token": ("page_summaries", _summaries_drop_last_token),
    "dense attention without 1/sqrt(d)": ("dense_attention", _dense_unscaled),
    "dense attention with KV head h % n_kv": ("dense_attention", _dense_head_modulo),
    "window one page short": ("geometry", _geometry_window_one_short),
    "mean query divided by n_q instead of G": ("pool_queries", _pool_queries_wrong_divisor),
}
_orig = {name: getattr(O, name) for name, _ in MODULE_MISTAKES.values()}
_orig["exp_spec"] = O.exp_spec


@pytest.mark.parametrize("mistake", sorted(MODULE_MISTAKES))
def test_a_planted_mistake_in_a_function_fails_a_pin(mistake, monkeypatch):
    name, wrong = MODULE_MISTAKES[mistake]
    monkeypatch.setattr(O, name, wrong)
    assert _first_failing_pin() is not None, f"no pin noticed: {mistake}"


# ---- mistakes in the stateful step --------------------------------------------------
def _step_commits_flagged_heads_only(self, q, k_new, v_new):
    before = self.active.copy()
    res = _orig_step(self, q, k_new, v_new)
    self.active = np.where(res["flags"][:, None] != 0, res["new_ids"], before)
    return res


def _step_never_reuses(self, q, k_new, v_new):
    res = _orig_step(self, q, k_new, v_new)
    res["out"] = self.attend(q, res["new_ids"])
    res["used_ids"] = res["new_ids"]
    return res


def _attended_without_open_page(self, page_ids):
    tok = _orig_attended(self, page_ids)
    g = self.geom()
    return tok[tok < g.n_full * self.p] if g.r else tok


def _export_nhd_kv_swapped(self, ids, n_slots):
    pool, pages = _orig_export(self, ids, n_slots)
    return pool[:, ::-1].copy(), pages


def _exp_cut_off_too_early(x):
    x = np.asarray(x, dtype=F32)
    e = _orig["exp_spec"](x)
    return np.where(x * O.LOG2E_F32 < F32(-20.0), F32(0.0), e)


def test_an_early_exponential_cut_off_changes_the_picked_page_set(monkeypatch):
    """The cut-off of the exponential moved from t < -64 to t < -20: in a peaked softmax the k-th best page
    lies below it, the tail ties at zero and the picked SET departs from the plain fp64 definition."""
    monkeypatch.setattr(O, "exp_spec", _exp_cut_off_too_early)
    with pytest.raises(AssertionError):
        _call_page_set_pin()


def _call_page_set_pin():
    class _NoCapture:                      # stands in for pytest's capsys fixture
        def disabled(self):
            import contextlib
            return contextlib.nullcontext()
    getattr(pins, PAGE_SET_PIN)(_NoCapture())


def _select_softmax_over_every_page(self, q):
    """Sel(q) with the softmax normalised over ALL full pages (sink and window included) instead of the
    candidate pages only; the top-k still runs over the candidates."""
    g = self.geom()
    lo, hi = g.cand_lo, g.cand_lo + g.n_cand
    P_all = O.page_weights(q, self.kmax[:g.n_full], self.kmin[:g.n_full])
    score = O.pooled_scores(P_all, self.G, self.select_pooling)[:, lo:hi]
    ids = np.full((self.n_kv, self.k), -1, dtype=np.int32)
    for m in range(self.n_kv):
        top = O.topk_pages(score[m], g.k_eff)
        ids[m, :top.shape[0]] = top + lo
    return ids, P_all[:, lo:hi], score


def test_softmax_over_sink_and_window_pages_is_caught_by_the_page_set_pin_alone(monkeypatch):
    """A mistake in WHICH pages enter the softmax moves every head's normaliser by its own amount, which
    re-weights the heads inside the group mean: value-level pins on pooled_scores cannot see it (the function
    is handed the wrong rows but computes them correctly); only the comparison of the picked set with the
    plain definition does."""
    monkeypatch.setattr(O.FreeKVOracle, "select", _select_softmax_over_every_page)
    assert _all_failing_pins() == [PAGE_SET_PIN]


_orig_step, _orig_attended, _orig_export = O.FreeKVOracle.step, O.FreeKVOracle.attended_tokens, O.FreeKVOracle.export_nhd
METHOD_MISTAKES = {
    "only corrected heads commit their new selection": ("step", _step_commits_flagged_heads_only),
    "every head attends with the fresh selection (no reuse)": ("step", _step_never_reuses),
    "the open page is not attended": ("attended_tokens", _attended_without_open_page),
    "K and V swapped in the NHD pool": ("export_nhd", _export_nhd_kv_swapped),
}


@pytest.mark.parametrize("mistake", sorted(METHOD_MISTAKES))
def test_a_planted_mistake_in_the_step_fails_a_pin(mistake, monkeypatch):
    name, wrong = METHOD_MISTAKES[mistake]
    monkeypatch.setattr(O.FreeKVOracle, name, wrong)
    assert _first_failing_pin() is not None, f"no pin noticed: {mistake}"
