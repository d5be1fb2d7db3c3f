"""GPU parity of attention through a mapping table (Sec. 3.4.4: KV groups addressed
logically, a table says in which physical slot each one is) and of the selection-overlap
count (Sec. 3.4.2), against the CPU oracle, through the C-ABI binding."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11907_amd as kv
import gpu_harness as H
from workloads import PRESETS, Config, make_layer, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU (run them with -m gpu on a GPU box)")
    kv.load_library()


def _say(name, stats):
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in stats.items()), flush=True)


def _scatter_into_pool(cfg, L, spare, seed):
    """The cache's groups placed at random slots of a larger pool whose unused slots are
    poisoned; returns (K_pool, V_pool, slot_table) as storage arrays."""
    B, Hk, NG, G, d = cfg.batch, cfg.n_kv_heads, cfg.n_groups, cfg.group_size, cfg.head_dim
    n_used = B * Hk * NG
    n_slots = n_used + spare
    g = np.random.default_rng(seed)
    where = g.permutation(n_slots)[:n_used].astype(np.int32)
    poison = np.uint16(0x7FC0) if cfg.dtype == "bf16" else np.float32(np.nan)
    Kp = np.full((n_slots, G, d), poison, dtype=L.K.dtype)
    Vp = np.full((n_slots, G, d), poison, dtype=L.K.dtype)
    Kp[where] = L.K.reshape(n_used, G, d)
    Vp[where] = L.V.reshape(n_used, G, d)
    return Kp, Vp, where.reshape(B, Hk, NG)


CASES = [
    PRESETS["c2"].replace(name="c2s", batch=2, ctx_len=4096, n_select=103),
    PRESETS["c2"].replace(name="c2r", batch=1, ctx_len=4004, n_select=77),
    PRESETS["c4"].replace(name="c4s", batch=1, ctx_len=16384, n_select=256),
    PRESETS["c1"].replace(name="c1s", ctx_len=2048, n_select=40),
    PRESETS["c2j"].replace(name="c2js", batch=2, ctx_len=4096, n_select=103),
    Config("f32_g1_qpk8", 1, 2, 8, 1, 64, 1024, 16, 1, 33, "f32", 16, 0.1, 8),
    Config("bf16_g16_qpk2", 1, 2, 4, 2, 128, 2048, 64, 16, 9, "bf16", 32, 0.1, 8),
    # slots of 12, 3 and 6 rows; 5, 3 and 7 query heads per KV head
    Config("bf16_g12_qpk5", 1, 2, 10, 2, 128, 12 * 170, 32, 12, 33, "bf16", 32, 0.1, 8),
    Config("f32_g3_qpk3", 1, 2, 6, 2, 64, 3 * 683, 16, 3, 41, "f32", 16, 0.1, 8),
    Config("bf16_g6_qpk7", 1, 1, 7, 1, 128, 6 * 300, 64, 6, 20, "bf16", 32, 0.1, 8),
]


# seeded random draws from the supported shape space (the same ones the plain path is tested on)
from test_gpu_random_shapes import _draw  # noqa: E402
CASES += [_draw(_seed)[0] for _seed in (0, 3, 6, 10, 13, 17, 22, 27, 31)]


@pytest.mark.parametrize("cfg", CASES, ids=[c.name for c in CASES])
def test_attention_through_a_mapping_table(cfg):
    L = make_layer(cfg)
    p, sh = H.kv_params(cfg), H.orc_shape(cfg)
    klr = oracle.build_metadata(sh, L.K, L.A)
    ref = oracle.predict_select(sh, L.q, klr, L.A)
    Kp, Vp, table = _scatter_into_pool(cfg, L, spare=37, seed=4)
    dq, dKp, dVp, dtab, didx = (H.to_dev(x) for x in (L.q, Kp, Vp, table, ref["idx"]))
    ws = H.workspace(p)
    stats = {}
    g = np.random.default_rng(9)
    cap = 2 * cfg.group_size
    rb = g.standard_normal((2, cfg.batch, cfg.n_kv_heads, cap, cfg.head_dim)).astype(np.float32)
    rbK, rbV = (f32_to_bf16_bits(x) if cfg.dtype == "bf16" else x for x in (rb[0], rb[1]))
    for rb_len in (0, cap - 1):
        out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=dq.dtype, device=H.DEV)
        kv.kvs_sparse_decode_attn_paged(p, dq, dKp, dVp, dtab, didx, out, ws,
                                        H.to_dev(rbK), H.to_dev(rbV), rb_len)
        torch.cuda.synchronize()
        want = oracle.sparse_attn_paged(sh, L.q, Kp, Vp, table, ref["idx"], rbK, rbV, rb_len)
        # (and the oracle's paged result is the unpaged one on the original cache)
        np.testing.assert_array_equal(want, oracle.sparse_attn(sh, L.q, L.K, L.V, ref["idx"], rbK, rbV, rb_len))
        stats[f"rb{rb_len}"] = H.attn_error(H.out_values(out), want)
        assert stats[f"rb{rb_len}"] <= H.ATTN_TOL[cfg.dtype], stats
    # bit-identical to the unpaged kernel on the same tokens (same order of operations)
    out_a = torch.empty((cfg.batch, cfg.n_q_heads, cfg.head_dim), dtype=dq.dtype, device=H.DEV)
    out_b = torch.empty_like(out_a)
    kv.kvs_sparse_decode_attn(p, dq, H.to_dev(L.K), H.to_dev(L.V), didx, out_a, ws)
    kv.kvs_sparse_decode_attn_paged(p, dq, dKp, dVp, dtab, didx, out_b, ws)
    torch.cuda.synchronize()
    assert torch.equal(out_a.view(torch.int16 if cfg.dtype == "bf16" else torch.int32),
                       out_b.view(torch.int16 if cfg.dtype == "bf16" else torch.int32))
    _say(cfg.name + "_paged", stats)


def test_c3_full_size_paged_sampled():
    """The 32K, batch-8 workload with its 524 288 groups scattered over a pool; oracle on
    sampled (b, kv head) problems, finiteness everywhere (a wrong slot would read poison)."""
    cfg = PRESETS["c3"]
    L = make_layer(cfg, 0, workers=16)
    p = H.kv_params(cfg)
    Kp, Vp, table = _scatter_into_pool(cfg, L, spare=1000, seed=11)
    dq, dKp, dVp, dtab = (H.to_dev(x) for x in (L.q, Kp, Vp, table))
    g = np.random.default_rng(3)
    idx = np.stack([np.sort(g.choice(cfg.n_groups, cfg.n_select, replace=False))
                    for _ in range(cfg.batch * cfg.n_kv_heads)]).astype(np.int32)
    idx = idx.reshape(cfg.batch, cfg.n_kv_heads, cfg.n_select)
    out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=dq.dtype, device=H.DEV)
    kv.kvs_sparse_decode_attn_paged(p, dq, dKp, dVp, dtab, H.to_dev(idx), out, H.workspace(p))
    torch.cuda.synchronize()
    out_h = H.out_values(out)
    assert np.isfinite(out_h).all()
    qpk = cfg.q_per_kv
    worst = 0.0
    for (b, k) in [(0, 0), (4, 3), (7, 7)]:
        sh1 = H.orc_shape(cfg, batch=1, n_kv_heads=1, n_q_heads=qpk)
        want = oracle.sparse_attn_paged(sh1, L.q[b:b + 1, k * qpk:(k + 1) * qpk], Kp, Vp,
                                        table[b:b + 1, k:k + 1], idx[b:b + 1, k:k + 1])
        worst = max(worst, H.attn_error(out_h[b:b + 1, k * qpk:(k + 1) * qpk], want))
    assert worst <= H.ATTN_TOL[cfg.dtype]
    _say("c3_paged_full", {"attn_err": worst})


@pytest.mark.parametrize("joint", [False, True], ids=["per_head", "joint"])
def test_selection_overlap_counts(joint):
    cfg = PRESETS["c3j" if joint else "c3"].replace(ctx_len=32768)
    p, sh = H.kv_params(cfg), H.orc_shape(cfg)
    g = np.random.default_rng(5)
    n = int(np.prod(p.sets))
    M, NG = cfg.n_select, cfg.n_groups

    def draw():
        return np.stack([np.sort(g.choice(NG, M, replace=False)) for _ in range(n)]).astype(np.int32).reshape(p.sets + (M,))

    a = draw()
    b = draw()
    b.reshape(n, M)[0] = a.reshape(n, M)[0]                       # one set fully reused
    b.reshape(n, M)[1] = np.arange(M, dtype=np.int32) + (NG - M)  # (whatever overlap that gives)
    got = torch.full(p.sets, -1, dtype=torch.int32, device=H.DEV)
    kv.kvs_selection_overlap(p, H.to_dev(a), H.to_dev(b), got)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), oracle.selection_overlap(sh, a, b))
    assert got.cpu().numpy().reshape(-1)[0] == M
    # an unsorted row counts the same
    b2 = b.copy()
    b2.reshape(n, M)[2] = g.permutation(b.reshape(n, M)[2])
    kv.kvs_selection_overlap(p, H.to_dev(a), H.to_dev(b2), got)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(got.cpu().numpy(), oracle.selection_overlap(sh, a, b))
