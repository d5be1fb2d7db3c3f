"""The 36-layer stack workload (batch 16, 16K context, 5 % budget) as a whole: every layer
resident in HBM with its own adapter, K_lr, selection and output; one decode step = 36
layer-steps sharing one workspace.  Checked per layer against the CPU oracle on sampled
(sequence, KV head) problems - index margin rule and attention tolerance - first launched
eagerly, then replayed from one captured HIP graph of all 36 layer-steps.
Needs an MI355X: run with  -m gpu."""
import time

import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import paper_2511_11907_amd as kv  # noqa: E402
from workloads import PRESETS, make_layer  # noqa: E402

import gpu_harness as H  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert "gfx950" in kv.kvs_version()


def _samples(layer: int, cfg):
    """Three (b, k) problems per layer, walking over all sequences and KV heads."""
    return [((layer * 3 + j * 5) % cfg.batch, (layer + 3 * j) % cfg.n_kv_heads) for j in range(3)]


def test_c5_whole_stack_eager_and_graph():
    cfg = PRESETS["c5"]
    p = H.kv_params(cfg)
    B, Hk, N, r, M, qpk = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.rank, cfg.n_select, cfg.q_per_kv
    sh1 = H.orc_shape(cfg, batch=1, n_kv_heads=1, n_q_heads=qpk, n_threads=1)
    ws = H.workspace(p)
    layers, refs = [], []
    t0 = time.time()
    for l in range(cfg.layers):
        L = make_layer(cfg, layer=l, workers=16)
        D = H.DeviceLayer(L)
        klr = torch.empty((B, Hk, N, r), dtype=torch.bfloat16, device=H.DEV)
        kv.kvs_build_metadata(p, D.K, D.A, klr)
        per = {}
        for (b, k) in _samples(l, cfg):
            K1, V1 = L.K[b:b + 1, k:k + 1].copy(), L.V[b:b + 1, k:k + 1].copy()
            q1, A1 = L.q[b:b + 1, k * qpk:(k + 1) * qpk].copy(), L.A[k:k + 1].copy()
            klr1, exact1 = oracle.build_metadata(sh1, K1, A1, want_exact=True)
            absdot = np.abs(H.storage_to_f32(K1)).astype(np.float64)[0, 0] @ np.abs(A1[0]).astype(np.float64)
            torch.cuda.synchronize()
            H.compare_metadata(H.to_host_storage(klr[b, k]), klr1[0, 0], exact1[0, 0], absdot, cfg.head_dim, "bf16")
            klr[b, k].copy_(H.to_dev(klr1[0, 0]))      # both sides score the oracle's metadata
            ref = oracle.predict_select(sh1, q1, klr1, A1)
            per[(b, k)] = (K1, V1, q1, ref)
        D.klr = klr
        D.idx = torch.full((B, Hk, M), -1, dtype=torch.int32, device=H.DEV)
        D.out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=torch.bfloat16, device=H.DEV)
        layers.append(D)
        refs.append(per)
        del L
        if l % 6 == 5:
            print(f"[stack] {l + 1} layers resident, {time.time() - t0:.0f} s", flush=True)

    def run_stack():
        for D in layers:
            kv.kvs_decode_step(p, D.q, D.klr, D.A, D.K, D.V, D.idx, None, D.out, ws)

    def check(tag):
        worst, exact, n = 0.0, 0, 0
        for l, (D, per) in enumerate(zip(layers, refs)):
            idx_h, out_h = D.idx.cpu().numpy(), H.out_values(D.out)
            assert np.all(np.diff(idx_h, axis=-1) > 0) and idx_h.min() >= 0 and idx_h.max() < cfg.n_groups, (tag, l)
            assert np.isfinite(out_h).all(), (tag, l)
            for (b, k), (K1, V1, q1, ref) in per.items():
                n += 1
                if H.check_index_margin(idx_h[b, k], ref["gs"][0, 0], ref["boundary"][0, 0], f"{tag} layer {l} b={b} k={k}"):
                    np.testing.assert_array_equal(idx_h[b, k], ref["idx"][0, 0])
                    exact += 1
                out_ref = oracle.sparse_attn(sh1, q1, K1, V1, idx_h[b:b + 1, k:k + 1])
                err = H.attn_error(out_h[b:b + 1, k * qpk:(k + 1) * qpk], out_ref)
                assert err <= H.ATTN_TOL["bf16"], (tag, l, b, k, err)
                worst = max(worst, err)
        print(f"[stack] {tag}: {n} sampled problems over {len(layers)} layers, {exact} by exact set equality, "
              f"worst attention err {worst:.3g}", flush=True)
        return [(D.idx.clone(), D.out.clone()) for D in layers]

    run_stack()
    torch.cuda.synchronize()
    eager = check("eager")

    # the same step as one captured graph of all 36 layer-steps, replayed twice with the
    # outputs cleared in between: every replay must reproduce the eager results bit for bit
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run_stack()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        run_stack()
    for rep in range(2):
        for D in layers:
            D.idx.fill_(-1)
            D.out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        if rep == 0:
            check("graph replay")
        for (idx_e, out_e), D in zip(eager, layers):
            assert torch.equal(idx_e, D.idx) and torch.equal(out_e.view(torch.int16), D.out.view(torch.int16)), \
                f"graph replay {rep} differs from the eager step"
