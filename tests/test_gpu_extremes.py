"""GPU parity at the edges of the supported shapes, and correctness of the step when it is
replayed from a captured graph."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11907_amd as kv
import gpu_harness as H
from workloads import PRESETS, Config, make_layer

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU (run them with -m gpu on a GPU box)")
    kv.load_library()


def _say(name, stats):
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in stats.items()), flush=True)


EXTREMES = [
    # a context of one single group: one score, one selected group, G attended tokens
    Config("one_group", 1, 2, 8, 2, 128, 4, 32, 4, 1, "bf16", 32, 0.1, 0),
    # the largest number of groups a problem may have (32768), token-level selection (G = 1)
    Config("max_groups", 1, 1, 4, 1, 64, 32768, 16, 1, 3277, "bf16", 16, 0.1, 8),
    # the same with every group selected: the attention is dense over 32768 tokens in 256 splits
    Config("max_groups_all", 1, 1, 2, 1, 64, 32768, 16, 1, 32768, "f32", 16, 0.1, 8),
    # many small problems: 4096 (sequence, kv head) pairs
    Config("many_problems", 1, 512, 8, 8, 64, 64, 16, 4, 3, "bf16", 16, 0.1, 2),
    # widest group and widest rank with the narrowest head
    Config("g16_r64_d64", 1, 2, 8, 1, 64, 2048, 64, 16, 128, "f32", 32, 0.1, 8),
]


@pytest.mark.parametrize("cfg", EXTREMES, ids=[c.name for c in EXTREMES])
def test_extreme_shapes(cfg):
    stats = H.run_and_compare(cfg)
    _say(cfg.name, stats)


def test_group_count_above_the_limit_is_refused():
    p = H.kv_params(Config("too_many", 1, 1, 4, 1, 64, 65536, 16, 1, 10, "bf16", 16, 0.1, 0))
    assert kv.kvs_check_params(p) == 4


@pytest.mark.parametrize("mode", ["per_head", "joint_fp8"])
def test_step_replayed_from_a_graph_matches_eager_every_time(mode):
    """The three (four) launches of a step captured into one graph; replays are interleaved
    with eager work on other inputs and synchronisations, and every replay must reproduce
    the eager result bit for bit (the workspace counters are reset by fill kernels inside
    the kernels themselves, never by memset nodes)."""
    joint = mode == "joint_fp8"
    cfg = PRESETS["c2j" if joint else "c2"].replace(name="graph", batch=2, ctx_len=4096, n_select=103)
    meta = dict(meta_dtype="fp8", meta_scale=0.125) if joint else {}
    p, sh = H.kv_params(cfg, **meta), H.orc_shape(cfg, **meta)
    layers = [make_layer(cfg, layer=i) for i in range(2)]
    dev = []
    for L in layers:
        klr = oracle.build_metadata(sh, L.K, L.A)
        dev.append({k: H.to_dev(v) for k, v in dict(q=L.q, K=L.K, V=L.V, A=L.A, klr=klr).items()})
    ws = H.workspace(p)
    shape_idx, shape_out = p.sets + (cfg.n_select,), (cfg.batch, cfg.n_q_heads, cfg.head_dim)

    def eager(d):
        idx = torch.full(shape_idx, -1, dtype=torch.int32, device=H.DEV)
        out = torch.full(shape_out, float("nan"), dtype=d["q"].dtype, device=H.DEV)
        kv.kvs_decode_step(p, d["q"], d["klr"], d["A"], d["K"], d["V"], idx, None, out, ws)
        torch.cuda.synchronize()
        return idx.clone(), out.clone()

    want = [eager(d) for d in dev]
    # capture the step on static buffers (layer 0's inputs)
    s_idx = torch.full(shape_idx, -1, dtype=torch.int32, device=H.DEV)
    s_out = torch.full(shape_out, float("nan"), dtype=dev[0]["q"].dtype, device=H.DEV)
    d0 = dev[0]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        kv.kvs_decode_step(p, d0["q"], d0["klr"], d0["A"], d0["K"], d0["V"], s_idx, None, s_out, ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        kv.kvs_decode_step(p, d0["q"], d0["klr"], d0["A"], d0["K"], d0["V"], s_idx, None, s_out, ws)
    for r in range(4):
        s_idx.fill_(-1)
        s_out.fill_(float("nan"))
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(s_idx, want[0][0]), f"replay {r}: selection differs"
        assert torch.equal(s_out.view(torch.int16), want[0][1].view(torch.int16)), f"replay {r}: output differs"
        # eager work of the program's own on the same workspace between replays
        i1, o1 = eager(dev[1])
        assert torch.equal(i1, want[1][0]) and torch.equal(o1.view(torch.int16), want[1][1].view(torch.int16))
    # and the eager result is the oracle's
    ref = oracle.predict_select(sh, layers[0].q, H.to_host_storage(dev[0]["klr"]), layers[0].A)
    flat = lambda a: a.reshape((-1,) + a.shape[len(p.sets):])
    for i, (ig, gr, bd) in enumerate(zip(flat(want[0][0].cpu().numpy()), flat(ref["gs"]), flat(ref["boundary"]))):
        H.check_index_margin(ig, gr, bd, f"graph set {i}")


def test_non_finite_metadata_still_gives_a_well_formed_selection():
    """Infinities and NaNs are outside the contract, but whatever comes out must still be M
    distinct in-range group indices in ascending order (all index arithmetic is integer
    work on the scores' bit patterns), and nothing may be written outside the outputs."""
    cfg = PRESETS["c2"].replace(name="nonfinite", batch=2, ctx_len=4096, n_select=103)
    L = make_layer(cfg)
    p, sh = H.kv_params(cfg), H.orc_shape(cfg)
    klr = oracle.build_metadata(sh, L.K, L.A)
    g = np.random.default_rng(0)
    flat = klr.reshape(-1)
    where = g.choice(flat.size, 600, replace=False)
    flat[where[:200]] = 0x7F80      # +inf (bf16 bits)
    flat[where[200:400]] = 0xFF80   # -inf
    flat[where[400:]] = 0x7FC0      # NaN
    D = H.DeviceLayer(L)
    ws = H.workspace(p)
    guard = 64
    idx = torch.full((cfg.batch * cfg.n_kv_heads * cfg.n_select + 2 * guard,), -7, dtype=torch.int32, device=H.DEV)
    view = idx[guard:-guard].view(cfg.batch, cfg.n_kv_heads, cfg.n_select)
    out = torch.zeros((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=D.q.dtype, device=H.DEV)
    for _ in range(2):      # twice: the counters must come back to zero even then
        kv.kvs_decode_step(p, D.q, H.to_dev(klr), D.A, D.K, D.V, view, None, out, ws)
        torch.cuda.synchronize()
        got = view.cpu().numpy()
        assert got.min() >= 0 and got.max() < cfg.n_groups
        assert np.all(np.diff(got, axis=-1) > 0)
        assert torch.all(idx[:guard] == -7) and torch.all(idx[-guard:] == -7)
    # and the workspace still serves a clean problem afterwards
    klr_ok = oracle.build_metadata(sh, L.K, L.A)
    kv.kvs_decode_step(p, D.q, H.to_dev(klr_ok), D.A, D.K, D.V, view, None, out, ws)
    torch.cuda.synchronize()
    ref = oracle.predict_select(sh, L.q, klr_ok, L.A)
    for i, (ig, gr, bd) in enumerate(zip(view.cpu().numpy().reshape(-1, cfg.n_select),
                                         ref["gs"].reshape(-1, cfg.n_groups), ref["boundary"].reshape(-1, 2))):
        H.check_index_margin(ig, gr, bd, f"after non-finite, set {i}")
