"""The selection kernel on hand-made group scores (Sec. 3.3, "TopK"), checked against the
definition itself: the M largest scores, ties to the lower index, indices ascending.

The parity tests proper compare whole predict+select calls with the CPU oracle; here the
score arrays are written directly so that each one drives the kernel down a particular
path: how many scores share the threshold's histogram bin (a handful, exactly as many as
the in-wave list holds, one more, nearly all), after which level the threshold is settled,
both register-slot instantiations, sizes that are not a multiple of four, infinities.
Needs an MI355X: run with  -m gpu."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2511_11907_amd as kv  # noqa: E402

import gpu_harness as H  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert "gfx950" in kv.kvs_version()


def _select(gs: np.ndarray, M: int) -> np.ndarray:
    """gs [P, NG] fp32 -> idx [P, M] through kvs_select_topk (the kernel builds its own histogram)."""
    P, NG = gs.shape
    G = 4
    p = kv.Params(P, 4, 1, 128, 32, NG * G, G, M, kv.KVS_BF16, kv.KVS_BF16)
    d_gs = torch.from_numpy(np.ascontiguousarray(gs)).to(H.DEV).view(P, 1, NG)
    guard = 64
    buf = torch.full((P * M + guard,), -7, dtype=torch.int32, device=H.DEV)
    idx = buf[: P * M].view(P, 1, M)
    kv.kvs_select_topk(p, d_gs, idx, None)
    torch.cuda.synchronize()
    assert bool((buf[P * M:] == -7).all()), "wrote past idx"
    return idx.cpu().numpy().reshape(P, M)


def _by_definition(gs: np.ndarray, M: int) -> np.ndarray:
    # -0.0 and +0.0 are equal scores: compare as numbers, ties by index (stable sort)
    order = np.argsort(-(gs.astype(np.float64) + 0.0), axis=1, kind="stable")[:, :M]
    return np.sort(order, axis=1).astype(np.int32)


def _check(gs, M, what):
    got = _select(gs, M)
    want = _by_definition(gs, M)
    assert np.array_equal(got, want), f"{what}: {np.count_nonzero(got != want)} of {got.size} indices differ"


RNG = np.random.default_rng(20251127)


@pytest.mark.parametrize("NG,M", [(8192, 820), (8192, 1), (8192, 8191), (8192, 8192), (4096, 410), (1000, 77),
                                  (999, 500), (7, 3), (1, 1), (16384, 1638), (32768, 3277), (30001, 12345), (8193, 820), (12001, 4000), (16385, 1638),
                                  (8193, 2000), (20000, 50)])
def test_random_scores(NG, M):
    gs = (RNG.standard_normal((5, NG)) * 20.0).astype(np.float32)
    _check(gs, M, f"normal NG={NG} M={M}")
    # heavy-tailed and one-sided
    _check(np.exp(RNG.standard_normal((3, NG)) * 3.0).astype(np.float32), M, f"lognormal NG={NG} M={M}")
    _check((-np.abs(RNG.standard_normal((3, NG)))).astype(np.float32), M, f"negative NG={NG} M={M}")


@pytest.mark.parametrize("NG", [8192, 16384])
@pytest.mark.parametrize("n_equal", [2, 63, 64, 65, 1023, 1024, 1025, 3000])
def test_threshold_inside_a_run_of_equal_scores(NG, n_equal):
    """`n_equal` scores share the threshold value, scattered over the array; M is chosen so
    that only some of them are selected (the first ones by index).  1024 is the number of keys
    the in-wave list holds: one more takes the path where all waves run the levels."""
    gs = (RNG.standard_normal((4, NG)) * 20.0).astype(np.float32)
    T = np.float32(13.25)
    n_above = int((gs[0] > T).sum())
    for p in range(4):
        where = RNG.choice(NG, size=n_equal, replace=False)
        gs[p, where] = T
    for take in (1, n_equal // 2, n_equal - 1, n_equal):
        if take < 1:
            continue
        # the same M for all problems: the count of larger scores differs per problem, so some
        # problems cut the run of equal scores and some do not - the definition decides
        M = n_above + take
        if 1 <= M <= NG:
            _check(gs, M, f"{n_equal} equal scores, NG={NG}, M={M}")


@pytest.mark.parametrize("NG", [4096, 8192, 32768])
def test_few_distinct_values(NG):
    """Scores quantised to a handful of values: every histogram bin in use holds hundreds or
    thousands of equal keys."""
    for step in (16.0, 4.0, 1.0):
        gs = (np.floor(RNG.standard_normal((3, NG)) * 20.0 / step) * step).astype(np.float32)
        for M in (1, NG // 10, NG // 2, NG - 1):
            _check(gs, M, f"quantised step={step} NG={NG} M={M}")
    _check(np.full((2, NG), 3.5, dtype=np.float32), NG // 3, "all equal")
    _check(np.zeros((2, NG), dtype=np.float32) * np.float32(-1.0), 5, "all negative zero")


def test_close_scores_settled_at_every_level():
    """Scores that differ only in their lowest mantissa bits share the first-level bin and
    most of the 20 bits below it: the threshold is settled at the last level, or earlier
    when the bin found holds a single key."""
    NG = 8192
    base = np.float32(1.0)
    ulp = np.spacing(base)
    for spread in (1, 16, 300, 5000, 70000, 1 << 20):
        k = RNG.integers(0, spread + 1, size=(4, NG))
        gs = (base + k * ulp).astype(np.float32)
        for M in (1, 100, 820, 4000):
            _check(gs, M, f"spread {spread} ulps, M={M}")


def test_infinities_and_mixed_signs():
    NG = 8192
    gs = (RNG.standard_normal((4, NG)) * 5.0).astype(np.float32)
    gs[:, RNG.choice(NG, 300, replace=False)] = -np.inf       # masked groups
    gs[:, RNG.choice(NG, 7, replace=False)] = np.inf
    gs[:, RNG.choice(NG, 50, replace=False)] = 0.0
    gs[:, RNG.choice(NG, 50, replace=False)] = -0.0
    for M in (1, 7, 8, 820, NG - 300, NG - 299, NG):
        _check(gs, M, f"infinities M={M}")


def _select_with_workspace(gs: np.ndarray, M: int, ws, p):
    P, NG = gs.shape
    d_gs = torch.from_numpy(np.ascontiguousarray(gs)).to(H.DEV).view(P, 1, NG)
    idx = torch.full((P, 1, M), -7, dtype=torch.int32, device=H.DEV)
    kv.kvs_select_topk(p, d_gs, idx, ws)
    torch.cuda.synchronize()
    return idx.cpu().numpy().reshape(P, M)


@pytest.mark.parametrize("NG,M", [(8192, 820), (16384, 2048), (1000, 77)])
def test_workspace_whose_histogram_is_not_of_these_scores(NG, M):
    """kvs_select_topk with a workspace whose histogram area does not belong to the scores:
    all zero (the scores came from elsewhere, or from kvs_predict_scores called without a
    workspace), and then holding another call's left-over counts.  The selection must notice
    (the histogram does not count NG scores), build its own, be exact, and leave the counters
    zero."""
    P, G = 3, 4
    p = kv.Params(P, 4, 1, 128, 32, NG * G, G, M, kv.KVS_BF16, kv.KVS_BF16)
    gs = (RNG.standard_normal((P, NG)) * 20.0).astype(np.float32)
    want = _by_definition(gs, M)
    ws = H.workspace(p)
    got = _select_with_workspace(gs, M, ws, p)
    assert np.array_equal(got, want), "zeroed histogram"
    # counters of a prediction that was never consumed: the histograms of other scores, twice
    L_q = torch.randn((P, 4, 128), device=H.DEV).to(torch.bfloat16)
    klr = torch.randn((P, 1, NG * G, 32), device=H.DEV).to(torch.bfloat16)
    A = torch.randn((1, 128, 32), device=H.DEV)
    other = torch.empty((P, 1, NG), dtype=torch.float32, device=H.DEV)
    kv.kvs_predict_scores(p, L_q, klr, A, other, ws)
    kv.kvs_predict_scores(p, L_q, klr, A, other, ws)
    got = _select_with_workspace(gs, M, ws, p)
    assert np.array_equal(got, want), "histogram holding 2 x NG foreign counts"
    # ... and that call left the counters zero: the paired calls work again and are exact
    kv.kvs_predict_scores(p, L_q, klr, A, other, ws)
    idx = torch.empty((P, 1, M), dtype=torch.int32, device=H.DEV)
    kv.kvs_select_topk(p, other, idx, ws)
    torch.cuda.synchronize()
    assert np.array_equal(idx.cpu().numpy().reshape(P, M), _by_definition(other.cpu().numpy().reshape(P, NG), M))


def test_scores_predicted_without_a_workspace_then_selected_with_one():
    """The pattern the header warns about: kvs_predict_scores(workspace = NULL) followed by
    kvs_select_topk(workspace): must equal the oracle's selection."""
    import oracle
    from workloads import PRESETS, make_layer
    cfg = PRESETS["c2"].replace(name="c2s", batch=2, ctx_len=4096, n_select=103)
    L = make_layer(cfg)
    sh = H.orc_shape(cfg)
    klr = oracle.build_metadata(sh, L.K, L.A)
    ref = oracle.predict_select(sh, L.q, klr, L.A)
    p = H.kv_params(cfg)
    ws = H.workspace(p)
    gs = torch.empty(p.sets + (cfg.n_groups,), dtype=torch.float32, device=H.DEV)
    idx = torch.full(p.sets + (cfg.n_select,), -1, dtype=torch.int32, device=H.DEV)
    kv.kvs_predict_scores(p, H.to_dev(L.q), H.to_dev(klr), H.to_dev(L.A), gs, None)
    kv.kvs_select_topk(p, gs, idx, ws)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    for b in range(cfg.batch):
        for k in range(cfg.n_kv_heads):
            if H.check_index_margin(idx_h[b, k], ref["gs"][b, k], ref["boundary"][b, k], f"b={b} k={k}"):
                assert np.array_equal(idx_h[b, k], ref["idx"][b, k])
