"""The single-launch decode step (kvs_decode_step_single_launch: prediction, selection and
attention as work items of one persistent grid) against the three separate launches
(kvs_predict_select + kvs_sparse_decode_attn) and against the CPU oracle.

Scores and selections of the two paths must agree bit for bit whatever the timing (same
arithmetic, same order); the attention outputs agree within the tolerance only, because the
single launch cuts a problem's selected tokens into another number of splits (one work item
per workgroup slot), which changes the order of the fp32 partial sums - but they must be the
same bits from run to run.  The cases: shapes that stress the work-item plan
(one problem, more problems than workgroups' worth of items, a single prediction chunk, an
unsplit attention, everything selected), the counters being left zero, thousands of steps
over rotating inputs with every output compared, and the bounded wait being forced to run
out from the host.  Needs an MI355X: run with  -m gpu."""
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


def _counter_words(p):
    """int32 view length of the workspace's zero-on-entry area (counters + histograms)."""
    P = p.batch * p.n_kv_heads
    return (-(-((3 * P + 4) * 4) // 256) * 256 + -(-(P * 4096 * 4) // 256) * 256) // 4


class Case:
    def __init__(self, cfg, seq_offset=0, adapter_from=None):
        self.cfg = cfg
        self.L = make_layer(cfg, workers=16, seq_offset=seq_offset, adapter_from=adapter_from)
        self.D = H.DeviceLayer(self.L)
        self.p = H.kv_params(cfg)
        self.sh = H.orc_shape(cfg, n_threads=16)
        self.klr = oracle.build_metadata(self.sh, self.L.K, self.L.A)
        self.klr_dev = H.to_dev(self.klr)

    def bufs(self):
        cfg, p = self.cfg, self.p
        return (torch.full(p.sets + (cfg.n_select,), -1, dtype=torch.int32, device=H.DEV),
                torch.full(p.sets + (cfg.n_groups,), float("nan"), dtype=torch.float32, device=H.DEV),
                torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=self.D.q.dtype, device=H.DEV))

    def three_launches(self, ws, gs=True):
        idx, g, out = self.bufs()
        D = self.D
        kv.kvs_predict_select(self.p, D.q, self.klr_dev, D.A, idx, g if gs else None, ws)
        kv.kvs_sparse_decode_attn(self.p, D.q, D.K, D.V, idx, out, ws)
        return idx, g, out

    def one_call(self, ws, gs=True, into=None):
        idx, g, out = into or self.bufs()
        D = self.D
        kv.kvs_decode_step_single_launch(self.p, D.q, self.klr_dev, D.A, D.K, D.V, idx, g if gs else None, out, ws)
        return idx, g, out


def _c2(**kw):
    base = dict(name="c2v", batch=1, ctx_len=4096, n_select=103)
    base.update(kw)
    return PRESETS["c2"].replace(**base)


def _c4(**kw):
    base = dict(name="c4v", batch=1, ctx_len=16384, n_select=256)
    base.update(kw)
    return PRESETS["c4"].replace(**base)


PLAN_SHAPES = [
    _c2(),                                            # 8 problems, a few chunks each
    _c2(n_kv_heads=1, n_q_heads=4),                   # a single problem: D = P = 1
    _c2(ctx_len=256, n_select=7),                     # one prediction chunk, one attention split
    _c2(ctx_len=4004, n_select=77),                   # ragged: 1001 groups
    _c2(ctx_len=2048, n_select=512),                  # everything selected
    _c2(batch=24, ctx_len=1024, n_select=26),         # 192 problems: more problems than a wave of items
    _c2(batch=2, ctx_len=32768, n_select=820),        # the 32K layer, two sequences
    _c4(),                                            # r = 64, G = 8
    _c4(batch=2, ctx_len=65536, n_select=2048),       # long problems: interleaved attention splits
    _c4(ctx_len=131072, n_select=4096),               # 16384 groups (32 keys per lane), 4096 selected
]


@pytest.mark.parametrize("cfg", PLAN_SHAPES, ids=[f"{c.name}_b{c.batch}_h{c.n_kv_heads}_N{c.ctx_len}_M{c.n_select}" for c in PLAN_SHAPES])
def test_one_launch_equals_three_launches_and_the_oracle(cfg):
    c = Case(cfg)
    ws = H.workspace(c.p)
    idx3, gs3, out3 = c.three_launches(ws)
    idx1, gs1, out1 = c.one_call(ws)
    torch.cuda.synchronize()
    assert kv.kvs_workspace_check(c.p, ws) == 0
    assert torch.equal(idx1, idx3), "selections differ"
    assert torch.equal(gs1, gs3), "group scores differ"
    err13 = H.attn_error(H.out_values(out1), H.out_values(out3))
    assert err13 <= H.ATTN_TOL["bf16"], f"outputs differ by {err13}"
    n = _counter_words(c.p)
    assert int(ws.view(torch.int32)[:n].abs().max()) == 0, "the step left counters behind"
    # the oracle's bar on the single launch itself
    ref = oracle.predict_select(c.sh, c.L.q, c.klr, c.L.A)
    idx_h = idx1.cpu().numpy()
    for b in range(cfg.batch):
        for k in range(cfg.n_kv_heads):
            H.check_index_margin(idx_h[b, k], ref["gs"][b, k], ref["boundary"][b, k], f"b={b} k={k}")
    err = H.attn_error(H.out_values(out1), oracle.sparse_attn(c.sh, c.L.q, c.L.K, c.L.V, idx_h))
    assert err <= H.ATTN_TOL["bf16"], err
    # without the caller's score array the scores stay in the workspace: same results
    idx2, _, out2 = c.one_call(ws, gs=False)
    torch.cuda.synchronize()
    assert torch.equal(idx2, idx3) and torch.equal(_bits(out2), _bits(out1))   # run to run: the same bits


@pytest.mark.parametrize("path", ["one_launch", "three_launches"])
def test_thousands_of_steps_reproduce_every_output_bit_for_bit(path):
    """The raciest shape of the cross-workgroup hand-overs: the 32K layer at batch 1, where each
    problem's attention is cut into 32 splits that are merged by whichever workgroup arrives
    last, and (single launch) selections and attention items wait on counters.  3000 steps
    over three rotating inputs sharing one workspace; every step's indices and outputs are
    compared on the device with that input's first result; stops at the first mismatch."""
    cfg = PRESETS["c2"]
    cases = []
    A0 = None
    for i in range(3):
        c = Case(cfg, seq_offset=i, adapter_from=A0)
        A0 = c.L.A
        cases.append(c)
    p = cases[0].p
    ws = H.workspace(p)
    run = (lambda c, into=None: c.one_call(ws, gs=False, into=into)) if path == "one_launch" else None
    first = []
    for c in cases:
        if path == "one_launch":
            idx, _, out = c.one_call(ws, gs=False)
        else:
            idx, _, out = c.three_launches(ws, gs=False)
        torch.cuda.synchronize()
        ref = oracle.predict_select(c.sh, c.L.q, c.klr, c.L.A)
        idx_h = idx.cpu().numpy()
        for k in range(cfg.n_kv_heads):
            H.check_index_margin(idx_h[0, k], ref["gs"][0, k], ref["boundary"][0, k], f"k={k}")
        first.append((idx.clone(), out.clone()))
    idx, gs, out = cases[0].bufs()
    bad = torch.zeros((), dtype=torch.int32, device=H.DEV)
    steps, window = 3000, 100
    for s in range(steps):
        i = s % 3
        c = cases[i]
        D = c.D
        if path == "one_launch":
            kv.kvs_decode_step_single_launch(p, D.q, c.klr_dev, D.A, D.K, D.V, idx, None, out, ws)
        else:
            kv.kvs_predict_select(p, D.q, c.klr_dev, D.A, idx, None, ws)
            kv.kvs_sparse_decode_attn(p, D.q, D.K, D.V, idx, out, ws)
        bad += (idx != first[i][0]).any().int() + (_bits(out) != _bits(first[i][1])).any().int()
        if (s + 1) % window == 0:
            assert int(bad.item()) == 0, f"{path}: a step in {s + 1 - window}..{s} did not reproduce its first result"
    assert kv.kvs_workspace_check(p, ws) == 0
    print(f"[soak] {path}: {steps} steps at the c2 shape reproduced bit for bit", flush=True)


def test_a_wait_that_runs_out_is_reported_and_the_workspace_recovers():
    """The bound of the in-kernel waits, forced from the host: with a limit of one poll some
    selection or attention items give up (their dependencies are still streaming), every
    workgroup still leaves, and the workspace says so; prepared again and with the default
    limit the next step is exact."""
    cfg = _c2(batch=4, ctx_len=16384, n_select=410)
    c = Case(cfg)
    ws = H.workspace(c.p)
    idx3, _, out3 = c.three_launches(ws)
    torch.cuda.synchronize()
    try:
        kv.kvs_set_wait_limit(1)
        idx, gs, out = c.bufs()
        idx.fill_(0)       # (items that are skipped leave idx as it is: keep it in range)
        c.one_call(ws, into=(idx, gs, out))
        torch.cuda.synchronize()              # the launch ends although waits ran out
        status = kv.kvs_workspace_check(c.p, ws)
    finally:
        kv.kvs_set_wait_limit(0)
    assert status in (0, 6)
    if status == 6:
        assert "wait" in kv.kvs_last_device_error()
    print(f"[wait-limit] status after a one-poll limit: {status}", flush=True)
    kv.kvs_workspace_init(c.p, ws)
    assert kv.kvs_workspace_check(c.p, ws) == 0
    idx1, _, out1 = c.one_call(ws)
    torch.cuda.synchronize()
    assert kv.kvs_workspace_check(c.p, ws) == 0
    assert torch.equal(idx1, idx3)
    assert H.attn_error(H.out_values(out1), H.out_values(out3)) <= H.ATTN_TOL["bf16"]


def test_layouts_outside_its_set_are_refused():
    cfg = PRESETS["c1"]
    p = H.kv_params(cfg)
    import ctypes
    lib = kv.load_library()
    x = torch.empty(64, dtype=torch.float32, device=H.DEV)
    a = ctypes.c_void_p(x.data_ptr())
    ws = H.workspace(p)
    st = lib.kvs_decode_step_single_launch(ctypes.byref(p._c()), a, a, a, a, a, a, None, a,
                                           ctypes.c_void_p(ws.data_ptr()), ws.numel() * 4, None)
    assert st == 4     # KVS_ERR_UNSUPPORTED: fp32, d = 64
