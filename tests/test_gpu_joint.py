"""GPU parity of the joint-head mode (Sec. 3.2 design (b): one adapter over the flattened
keys, one K_lr row per token, scores summed over all query heads by Eq. 1, one selection
per sequence) against the CPU oracle, through the C-ABI binding."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11907_amd as kv
import gpu_harness as H
from workloads import PRESETS, Config, make_layer, storage_to_f32

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU (run them with -m gpu on a GPU box)")
    kv.load_library()


def _say(name, stats):
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in stats.items()), flush=True)


def _variant(name, dtype, Hq, Hk, d, r, G, N, M, B=2):
    return Config(name, 1, B, Hq, Hk, d, N, r, G, M, dtype, min(r, 32), 0.1, 8, joint=True)


CASES = {
    "c1j": PRESETS["c1j"],
    # scaled versions of the large workloads: several tiles, ragged tails
    "c2j_small": PRESETS["c2j"].replace(name="c2js", batch=2, ctx_len=4096, n_select=103),
    "c2j_ragged": PRESETS["c2j"].replace(name="c2jr", batch=3, ctx_len=4004, n_select=77),
    "c4j_small": PRESETS["c4j"].replace(name="c4js", batch=1, ctx_len=16384, n_select=256),
    # layouts: rank above the head dimension (only legal here), one KV head, 8 heads per KV
    # head, every group size class, fp32 and bf16
    "bf16_d64_r128_g2": _variant("bf16_d64_r128_g2", "bf16", 8, 4, 64, 128, 2, 1536, 50),
    "bf16_d128_r16_g16_hk1": _variant("bf16_d128_r16_g16_hk1", "bf16", 8, 1, 128, 16, 16, 2048, 9),
    "f32_d64_r32_g1": _variant("f32_d64_r32_g1", "f32", 4, 4, 64, 32, 1, 1024, 64),
    "f32_d128_r64_g8": _variant("f32_d128_r64_g8", "f32", 16, 8, 128, 64, 8, 2048, 17, B=1),
}


@pytest.mark.parametrize("name", sorted(CASES))
def test_joint_mode_matches_the_oracle(name):
    stats = H.run_and_compare(CASES[name])
    _say(name, stats)


def test_joint_mean_reduce():
    _say("c2js_mean", H.run_and_compare(CASES["c2j_small"], reduce=kv.KVS_REDUCE_MEAN, check_meta=False))


def test_one_kv_head_gives_the_same_bits_in_both_modes():
    """With a single KV head the two designs are the same computation; the kernels differ
    only in where the query is projected, so the selections must be identical and the
    scores equal to fp32 rounding of the projection."""
    cfg = _variant("hk1", "bf16", 4, 1, 128, 32, 4, 4096, 100)
    L = make_layer(cfg)
    D = H.DeviceLayer(L)
    pj, ps = H.kv_params(cfg), H.kv_params(cfg, head_mode=kv.KVS_HEADS_SEPARATE)
    klr_j = torch.empty((cfg.batch, cfg.ctx_len, cfg.rank), dtype=D.K.dtype, device=H.DEV)
    klr_s = torch.empty((cfg.batch, 1, cfg.ctx_len, cfg.rank), dtype=D.K.dtype, device=H.DEV)
    kv.kvs_build_metadata(pj, D.K, D.A, klr_j)
    kv.kvs_build_metadata(ps, D.K, D.A, klr_s)
    assert torch.equal(klr_j, klr_s[:, 0])
    ij = torch.empty((cfg.batch, cfg.n_select), dtype=torch.int32, device=H.DEV)
    is_ = torch.empty((cfg.batch, 1, cfg.n_select), dtype=torch.int32, device=H.DEV)
    gj = torch.empty((cfg.batch, cfg.n_groups), dtype=torch.float32, device=H.DEV)
    gs = torch.empty((cfg.batch, 1, cfg.n_groups), dtype=torch.float32, device=H.DEV)
    kv.kvs_predict_select(pj, D.q, klr_j, D.A, ij, gj, H.workspace(pj))
    kv.kvs_predict_select(ps, D.q, klr_s, D.A, is_, gs, H.workspace(ps))
    torch.cuda.synchronize()
    rel = float((gj - gs[:, 0]).abs().max() / gs.abs().max())
    assert rel <= 1e-5, rel
    same = float((ij == is_[:, 0]).float().mean())
    assert same >= 0.99, same     # a score pair closer than the rounding may swap


def test_joint_split_calls_match_the_fused_call_and_need_the_workspace():
    cfg = CASES["c2j_small"]
    L = make_layer(cfg)
    D = H.DeviceLayer(L)
    p = H.kv_params(cfg)
    sh = H.orc_shape(cfg)
    klr = H.to_dev(oracle.build_metadata(sh, L.K, L.A))
    ws = H.workspace(p)
    B, M, NG = cfg.batch, cfg.n_select, cfg.n_groups
    idx_a = torch.full((B, M), -1, dtype=torch.int32, device=H.DEV)
    gs_a = torch.full((B, NG), float("nan"), dtype=torch.float32, device=H.DEV)
    kv.kvs_predict_select(p, D.q, klr, D.A, idx_a, gs_a, ws)
    idx_b, gs_b = torch.full_like(idx_a, -1), torch.full_like(gs_a, float("nan"))
    kv.kvs_predict_scores(p, D.q, klr, D.A, gs_b, ws)
    kv.kvs_select_topk(p, gs_b, idx_b, ws)
    idx_c = torch.full_like(idx_a, -1)
    kv.kvs_select_topk(p, gs_b, idx_c, None)          # builds its own histogram
    torch.cuda.synchronize()
    assert torch.equal(gs_a, gs_b) and torch.equal(idx_a, idx_b) and torch.equal(idx_a, idx_c)
    with pytest.raises(kv.KvsError) as e:
        kv.kvs_predict_scores(p, D.q, klr, D.A, gs_b, None)
    assert e.value.status == 5
    # repeated whole steps are bit-identical and leave the workspace reusable
    out0 = None
    for _ in range(20):
        idx = torch.full_like(idx_a, -1)
        out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=D.q.dtype, device=H.DEV)
        kv.kvs_decode_step(p, D.q, klr, D.A, D.K, D.V, idx, None, out, ws)
        torch.cuda.synchronize()
        assert torch.equal(idx, idx_a)
        out0 = out if out0 is None else out0
        assert torch.equal(out.view(torch.int16), out0.view(torch.int16))


def _full_size_sampled_joint(cfg: Config, seqs):
    """GPU on the whole batch at the real size; oracle on the sampled sequences, whose
    oracle-built metadata rows replace the GPU-built ones so both sides score the same K_lr."""
    L = make_layer(cfg, 0, workers=16)
    D = H.DeviceLayer(L)
    p = H.kv_params(cfg)
    B, Hk, N, r, M = cfg.batch, cfg.n_kv_heads, cfg.ctx_len, cfg.rank, cfg.n_select
    klr = torch.empty((B, N, r), dtype=D.K.dtype, device=H.DEV)
    kv.kvs_build_metadata(p, D.K, D.A, klr)
    torch.cuda.synchronize()
    sh1 = H.orc_shape(cfg, batch=1)
    sub = {}
    for b in seqs:
        print(f"[joint full] {cfg.name}: oracle metadata of sequence {b}", flush=True)
        klr1, exact1 = oracle.build_metadata(sh1, L.K[b:b + 1], L.A, want_exact=True)
        absdot = np.einsum("knd,kdr->nr", np.abs(storage_to_f32(L.K[b])).astype(np.float64),
                           np.abs(L.A).astype(np.float64))
        frac = H.compare_metadata(H.to_host_storage(klr[b]), klr1[0], exact1[0], absdot,
                                  Hk * cfg.head_dim, cfg.dtype)
        klr[b].copy_(H.to_dev(klr1[0]))
        sub[b] = (klr1, frac)
    ws = H.workspace(p)
    idx = torch.full((B, M), -1, dtype=torch.int32, device=H.DEV)
    out = torch.full((B, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=D.q.dtype, device=H.DEV)
    kv.kvs_decode_step(p, D.q, klr, D.A, D.K, D.V, idx, None, out, ws)
    torch.cuda.synchronize()
    idx_h, out_h = idx.cpu().numpy(), H.out_values(out)
    assert np.all(np.diff(idx_h, axis=-1) > 0) and idx_h.min() >= 0 and idx_h.max() < cfg.n_groups
    assert np.isfinite(out_h).all()
    worst = 0.0
    for b, (klr1, frac) in sub.items():
        ref = oracle.predict_select(sh1, L.q[b:b + 1], klr1, L.A)
        H.check_index_margin(idx_h[b], ref["gs"][0], ref["boundary"][0], f"{cfg.name} b={b}")
        out_ref = oracle.sparse_attn(sh1, L.q[b:b + 1], L.K[b:b + 1], L.V[b:b + 1], idx_h[b:b + 1])
        err = H.attn_error(out_h[b:b + 1], out_ref)
        assert err <= H.ATTN_TOL[cfg.dtype], (cfg.name, b, err)
        worst = max(worst, err)
    _say(cfg.name + "_full", {"attn_err": worst, "meta_mismatch": max(f for _, f in sub.values())})


def test_c2j_full_size_sampled():
    _full_size_sampled_joint(PRESETS["c2j"], [0])


def test_c3j_full_size_sampled():
    _full_size_sampled_joint(PRESETS["c3j"], [2, 7])


def test_c4j_full_size_sampled():
    _full_size_sampled_joint(PRESETS["c4j"], [3])
