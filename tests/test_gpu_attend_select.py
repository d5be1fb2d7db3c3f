"""kvs_attend_select_next (the attention of one layer and the selection for the next layer in
one launch, the pipelined form of Sec. 3.3 / 3.4) against the separate calls and the CPU
oracle: the next layer's indices must equal kvs_select_topk's and the outputs
kvs_sparse_decode_attn's bit for bit (same routines, same split plan), with and without the
score histograms handed over by kvs_predict_scores; a pipelined loop over layers must
reproduce the serial steps; the workspace's counters are left zero.  Needs an MI355X:
run with  -m gpu."""
import ctypes

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


def _bits(t):
    return t.view(torch.int16) if t.dtype == torch.bfloat16 else t


class Layer:
    def __init__(self, cfg, seq_offset=0, adapter_from=None):
        self.cfg = cfg
        self.L = make_layer(cfg, workers=16, seq_offset=seq_offset, adapter_from=adapter_from)
        self.D = H.DeviceLayer(self.L)
        self.sh = H.orc_shape(cfg, n_threads=16)
        self.klr = oracle.build_metadata(self.sh, self.L.K, self.L.A)   # (the shape says which head mode)
        self.klr_dev = H.to_dev(self.klr)


def _bufs(cfg, p, like):
    return (torch.full(p.sets + (cfg.n_select,), -1, dtype=torch.int32, device=H.DEV),
            torch.full(p.sets + (cfg.n_groups,), float("nan"), dtype=torch.float32, device=H.DEV),
            torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=like.dtype, device=H.DEV))


def _c2(**kw):
    base = dict(name="c2a", batch=1, ctx_len=4096, n_select=103)
    base.update(kw)
    return PRESETS["c2"].replace(**base)


def _c4(**kw):
    base = dict(name="c4a", batch=1, ctx_len=16384, n_select=256)
    base.update(kw)
    return PRESETS["c4"].replace(**base)


SHAPES = [
    _c2(),                                                      # 8 sets, 1024 groups
    _c2(n_kv_heads=1, n_q_heads=4),                             # one set
    _c2(ctx_len=4004, n_select=77),                             # ragged: 1001 groups
    _c2(ctx_len=2048, n_select=512),                            # everything selected
    _c2(batch=24, ctx_len=1024, n_select=26),                   # 192 sets (no histogram hand-over), unsplit attention
    _c2(batch=2, ctx_len=32768, n_select=820),                  # 8192 groups: 16 keys per lane
    _c2(n_q_heads=28, n_kv_heads=4, ctx_len=8192, n_select=205),   # seven query heads per KV head
    _c2(n_q_heads=24, n_kv_heads=8, ctx_len=8192, n_select=205),   # three
    _c4(),                                                      # r = 64, G = 8
    _c4(batch=2, ctx_len=65536, n_select=2048),                 # interleaved attention splits
    _c4(ctx_len=131072, n_select=1638),                         # 16384 groups: 32 keys per lane
    PRESETS["c2j"].replace(name="c2ja", batch=2, ctx_len=4096, n_select=103),   # joint-head mode: one set per sequence
]


@pytest.mark.parametrize("cfg", SHAPES, ids=[f"{c.name}_b{c.batch}_q{c.n_q_heads}_h{c.n_kv_heads}_N{c.ctx_len}_M{c.n_select}" for c in SHAPES])
def test_one_launch_equals_the_two_calls_and_the_oracle(cfg):
    cur = Layer(cfg)
    nxt = Layer(cfg, seq_offset=1, adapter_from=cur.L.A)
    p = H.kv_params(cfg)
    ws = H.workspace(p)
    # this layer's selection, and the reference results of the separate calls
    idx, gs, out_ref = _bufs(cfg, p, cur.D.q)
    kv.kvs_predict_select(p, cur.D.q, cur.klr_dev, cur.D.A, idx, None, ws)
    kv.kvs_sparse_decode_attn(p, cur.D.q, cur.D.K, cur.D.V, idx, out_ref, ws)
    idx_ref, gs_next, _ = _bufs(cfg, p, cur.D.q)
    kv.kvs_predict_scores(p, nxt.D.q, nxt.klr_dev, nxt.D.A, gs_next, ws)
    kv.kvs_select_topk(p, gs_next, idx_ref, ws)
    torch.cuda.synchronize()
    # the same with the one launch, histograms handed over by kvs_predict_scores
    idx_new, gs2, out = _bufs(cfg, p, cur.D.q)
    kv.kvs_predict_scores(p, nxt.D.q, nxt.klr_dev, nxt.D.A, gs2, ws)
    kv.kvs_attend_select_next(p, cur.D.q, cur.D.K, cur.D.V, idx, out, gs2, idx_new, ws)
    torch.cuda.synchronize()
    assert torch.equal(gs2, gs_next)
    assert torch.equal(idx_new, idx_ref), "the next layer's selection differs"
    assert torch.equal(_bits(out), _bits(out_ref)), "the attention output differs"
    # scores that did not come through this workspace (no histogram there): still exact
    idx_new2, _, out2 = _bufs(cfg, p, cur.D.q)
    kv.kvs_attend_select_next(p, cur.D.q, cur.D.K, cur.D.V, idx, out2, gs_next, idx_new2, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx_new2, idx_ref) and torch.equal(_bits(out2), _bits(out_ref))
    # counters and histograms are left zero
    P = cfg.batch * cfg.n_kv_heads
    n_sets = int(np.prod(p.sets))
    zero_words = (-(-((3 * P + 4) * 4) // 256) * 256 + -(-(n_sets * 4096 * 4) // 256) * 256) // 4
    assert zero_words * 4 <= kv.kvs_workspace_bytes(p)
    assert int(ws.view(torch.int32)[:zero_words].abs().max()) == 0, "the launch left counters behind"
    # the oracle's bar on the launch itself
    ref = oracle.predict_select(nxt.sh, nxt.L.q, nxt.klr, nxt.L.A)
    got = idx_new.cpu().numpy().reshape(ref["gs"].shape[:-1] + (cfg.n_select,))
    for s in np.ndindex(*ref["gs"].shape[:-1]):
        H.check_index_margin(got[s], ref["gs"][s], ref["boundary"][s], f"set {s}")
    idx_h = idx.cpu().numpy()
    err = H.attn_error(H.out_values(out), oracle.sparse_attn(cur.sh, cur.L.q, cur.L.K, cur.L.V, idx_h))
    assert err <= H.ATTN_TOL["bf16"], err


def test_a_pipelined_loop_over_layers_reproduces_the_serial_steps():
    """Five layers of the c2 shape at 8K tokens: serial kvs_decode_step per layer against the
    pipelined issue order (prediction of layer l+1, then attention of layer l together with
    the selection of layer l+1), one workspace, indices and outputs of every layer equal."""
    cfg = _c2(batch=2, ctx_len=8192, n_select=205)
    layers = []
    for i in range(5):
        layers.append(Layer(cfg, seq_offset=i))
    p = H.kv_params(cfg)
    ws = H.workspace(p)
    serial = []
    for l in layers:
        idx, _, out = _bufs(cfg, p, l.D.q)
        kv.kvs_decode_step(p, l.D.q, l.klr_dev, l.D.A, l.D.K, l.D.V, idx, None, out, ws)
        serial.append((idx, out))
    torch.cuda.synchronize()
    bufs = [_bufs(cfg, p, l.D.q) for l in layers]
    # prologue: the first layer's selection by the ordinary calls
    l0 = layers[0]
    kv.kvs_predict_select(p, l0.D.q, l0.klr_dev, l0.D.A, bufs[0][0], None, ws)
    for i, l in enumerate(layers):
        if i + 1 < len(layers):
            n = layers[i + 1]
            kv.kvs_predict_scores(p, n.D.q, n.klr_dev, n.D.A, bufs[i + 1][1], ws)
            kv.kvs_attend_select_next(p, l.D.q, l.D.K, l.D.V, bufs[i][0], bufs[i][2], bufs[i + 1][1], bufs[i + 1][0], ws)
        else:
            kv.kvs_sparse_decode_attn(p, l.D.q, l.D.K, l.D.V, bufs[i][0], bufs[i][2], ws)
    torch.cuda.synchronize()
    for i in range(len(layers)):
        assert torch.equal(bufs[i][0], serial[i][0]), f"layer {i}: selection"
        assert torch.equal(_bits(bufs[i][2]), _bits(serial[i][1])), f"layer {i}: output"


def test_layouts_outside_its_set_are_refused():
    cfg = PRESETS["c1"]          # fp32, d = 64: the vector-ALU attention
    p = H.kv_params(cfg)
    lib = kv.load_library()
    x = torch.empty(64, dtype=torch.float32, device=H.DEV)
    a = ctypes.c_void_p(x.data_ptr())
    ws = H.workspace(p)
    st = lib.kvs_attend_select_next(ctypes.byref(p._c()), a, a, a, a, a, a, a,
                                    ctypes.c_void_p(ws.data_ptr()), ws.numel() * 4, None)
    assert st == 4     # KVS_ERR_UNSUPPORTED
    st = lib.kvs_attend_select_next(ctypes.byref(p._c()), a, a, a, a, a, None, a,
                                    ctypes.c_void_p(ws.data_ptr()), ws.numel() * 4, None)
    assert st == 1     # KVS_ERR_NULL


@pytest.mark.parametrize("cfg,cap", [(_c2(ctx_len=8192, n_select=205), 4), (_c4(), 8),
                                     (_c4(batch=2, ctx_len=65536, n_select=2048), 8),
                                     (PRESETS["c2j"].replace(name="c2ja", batch=2, ctx_len=4096, n_select=103), 4)],
                         ids=["r32_G4", "r64_G8", "r64_G8_interleaved", "joint"])
def test_with_the_rolling_buffer_it_equals_the_rolling_buffer_attention_and_the_selection(cfg, cap):
    """kvs_attend_select_next_rb for every fill of the buffer: outputs equal
    kvs_sparse_decode_attn_rb's and the next layer's indices kvs_select_topk's, bit for bit;
    with an empty buffer it is kvs_attend_select_next."""
    cur = Layer(cfg)
    nxt = Layer(cfg, seq_offset=1, adapter_from=cur.L.A)
    p = H.kv_params(cfg)
    ws = H.workspace(p)
    rng = np.random.default_rng(5)
    shape = (cfg.batch, cfg.n_kv_heads, cap, cfg.head_dim)
    rbK = (rng.standard_normal(shape) * 0.7).astype(np.float32)
    rbV = rng.standard_normal(shape).astype(np.float32)
    drK = torch.from_numpy(rbK).to(H.DEV).to(cur.D.K.dtype)
    drV = torch.from_numpy(rbV).to(H.DEV).to(cur.D.K.dtype)
    idx, _, _ = _bufs(cfg, p, cur.D.q)
    kv.kvs_predict_select(p, cur.D.q, cur.klr_dev, cur.D.A, idx, None, ws)
    idx_ref, gs_next, _ = _bufs(cfg, p, cur.D.q)
    kv.kvs_predict_scores(p, nxt.D.q, nxt.klr_dev, nxt.D.A, gs_next, ws)
    kv.kvs_select_topk(p, gs_next, idx_ref, ws)
    for rb_len in sorted({0, 1, cap - 1, cap}):
        _, _, out_ref = _bufs(cfg, p, cur.D.q)
        kv.kvs_sparse_decode_attn_rb(p, cur.D.q, cur.D.K, cur.D.V, idx, drK, drV, rb_len, out_ref, ws)
        idx_new, gs2, out = _bufs(cfg, p, cur.D.q)
        kv.kvs_predict_scores(p, nxt.D.q, nxt.klr_dev, nxt.D.A, gs2, ws)
        kv.kvs_attend_select_next_rb(p, cur.D.q, cur.D.K, cur.D.V, idx, drK, drV, rb_len, out, gs2, idx_new, ws)
        torch.cuda.synchronize()
        assert torch.equal(idx_new, idx_ref), f"rb_len={rb_len}: selection"
        assert torch.equal(_bits(out), _bits(out_ref)), f"rb_len={rb_len}: output"
        if rb_len == 0:
            _, _, out0 = _bufs(cfg, p, cur.D.q)
            idx0 = torch.full_like(idx_new, -1)
            kv.kvs_attend_select_next(p, cur.D.q, cur.D.K, cur.D.V, idx, out0, gs_next, idx0, ws)
            torch.cuda.synchronize()
            assert torch.equal(idx0, idx_ref) and torch.equal(_bits(out0), _bits(out_ref))
    assert not torch.isnan(out.float()).any()


@pytest.mark.parametrize("name", ["c3", "c4"])
def test_at_the_benchmark_sizes_it_equals_the_separate_calls(name):
    """The launch configuration bench.py times (c3: 64 problems of 8192 groups, unsplit
    interleaving off; c4: 32 problems of 16384 groups, interleaved splits): outputs and the
    selection equal the separate kernels' bit for bit.  (The separate kernels are compared
    with the oracle at these sizes in test_gpu_parity.py; one layer's inputs serve as both
    the attended and the next layer here.)"""
    cfg = PRESETS[name]
    L = make_layer(cfg, workers=16)
    D = H.DeviceLayer(L)
    p = H.kv_params(cfg)
    ws = H.workspace(p)
    klr = torch.empty(p.sets + (cfg.ctx_len, cfg.rank), dtype=torch.bfloat16, device=H.DEV)
    kv.kvs_build_metadata(p, D.K, D.A, klr)
    idx, gs, out_ref = _bufs(cfg, p, D.q)
    kv.kvs_predict_select(p, D.q, klr, D.A, idx, gs, ws)
    kv.kvs_sparse_decode_attn(p, D.q, D.K, D.V, idx, out_ref, ws)
    idx_new, gs2, out = _bufs(cfg, p, D.q)
    kv.kvs_predict_scores(p, D.q, klr, D.A, gs2, ws)
    kv.kvs_attend_select_next(p, D.q, D.K, D.V, idx, out, gs2, idx_new, ws)
    torch.cuda.synchronize()
    assert torch.equal(gs2, gs)
    assert torch.equal(idx_new, idx), "selection"
    assert torch.equal(_bits(out), _bits(out_ref)), "output"
    assert int((idx_new[..., 1:] <= idx_new[..., :-1]).sum()) == 0      # ascending, distinct
