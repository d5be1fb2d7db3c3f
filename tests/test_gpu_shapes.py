"""Parity of the HIP path against the CPU oracle at the head geometries of the paper's
evaluated models and at group sizes that are not powers of two.

Head geometry (Sec. 4.1): LLaMA3-3B 24 query / 8 KV heads, LLaMA3-8B and Qwen3-4B/8B 32/8,
Qwen3-14B and InternVL3-14B 40/8, Qwen2.5-VL-7B 28/4, Qwen2.5-VL-3B 16/2, all with a head
dimension of 128.  Group sizes: the parameter solver walks G upwards from 1 (App. A.4)
with M*G held near 400 (App. A.2), and the appendix's rolling-buffer table goes to G = 12.
Needs an MI355X: run with  -m gpu."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import oracle  # noqa: E402
import paper_2511_11907_amd as kv  # noqa: E402
from workloads import PRESETS, Config, f32_to_bf16_bits, make_layer, storage_to_f32  # noqa: E402

import gpu_harness as H  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert "gfx950" in kv.kvs_version()


def _say(name, stats):
    print(f"[shapes] {name}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in stats.items()), flush=True)


def _cfg(name, dtype, Hq, Hk, d, r, G, NG, M, B=2, joint=False):
    return Config(name, 1, B, Hq, Hk, d, NG * G, r, G, M, dtype, min(r, 32), 0.1, 8, joint=joint)


# ---- the evaluated models' head geometry, M*G about 400 tokens -------------------------------
MODELS = [
    _cfg("llama3_3b_24q8kv_g4", "bf16", 24, 8, 128, 32, 4, 1024, 100, B=1),
    _cfg("qwen3_14b_40q8kv_g8", "bf16", 40, 8, 128, 32, 8, 512, 50, B=1),
    _cfg("qwen3_14b_40q8kv_g12", "bf16", 40, 8, 128, 32, 12, 341, 33, B=1),
    _cfg("qwen25vl_7b_28q4kv_g4", "bf16", 28, 4, 128, 16, 4, 1001, 100),
    _cfg("qwen25vl_3b_16q2kv_g2", "bf16", 16, 2, 128, 16, 2, 2048, 200),
    _cfg("six_heads_per_kv_f32_d64", "f32", 12, 2, 64, 16, 2, 700, 60),
    _cfg("three_heads_per_kv_f32", "f32", 6, 2, 128, 64, 4, 515, 31),
    _cfg("five_heads_per_kv_f32_d64", "f32", 5, 1, 64, 32, 8, 300, 17),
    _cfg("seven_heads_per_kv_f32", "f32", 14, 2, 128, 128, 1, 1024, 90),
]


@pytest.mark.parametrize("cfg", MODELS, ids=[c.name for c in MODELS])
def test_model_head_geometries(cfg):
    _say(cfg.name, H.run_and_compare(cfg))


@pytest.mark.parametrize("cfg", [MODELS[0], MODELS[2], MODELS[3]], ids=lambda c: c.name + "_joint")
def test_model_head_geometries_joint_head(cfg):
    """The same layers under the joint-head design: one adapter over H_kv*d = 1024 (512)
    flattened key values, rank 32 (compression ratio 32 resp. 16)."""
    j = cfg.replace(name=cfg.name + "_joint", joint=True, rank=32, planted_rank=32)
    _say(j.name, H.run_and_compare(j))


# ---- group sizes off the powers of two, in every row-width class of the metadata --------------
# (rows per 1 KiB load: bf16 r=16 32, r=32 16, r=64 8, r=128 4; fp32 r=16 16, r=64 4, r=128 2)
GROUPS = [
    _cfg("bf16_r32_g3", "bf16", 8, 2, 128, 32, 3, 683, 41),
    _cfg("bf16_r32_g12", "bf16", 8, 2, 128, 32, 12, 341, 33),
    _cfg("bf16_r32_g11", "bf16", 8, 2, 128, 32, 11, 187, 20),
    _cfg("bf16_r32_g13", "bf16", 4, 2, 128, 32, 13, 158, 12),
    _cfg("bf16_r32_g15", "bf16", 4, 2, 64, 32, 15, 137, 10),
    _cfg("bf16_r64_g6", "bf16", 8, 2, 128, 64, 6, 500, 37),
    _cfg("bf16_r128_g5", "bf16", 8, 2, 128, 128, 5, 411, 40),
    _cfg("bf16_r16_g7", "bf16", 4, 2, 64, 16, 7, 293, 29),
    _cfg("bf16_r16_g10", "bf16", 4, 2, 64, 16, 10, 205, 9),
    _cfg("f32_r64_g12", "f32", 2, 2, 128, 64, 12, 171, 17),
    _cfg("f32_r128_g3", "f32", 4, 2, 128, 128, 3, 343, 33),
    _cfg("f32_r16_g9", "f32", 8, 2, 64, 16, 9, 228, 19),
    _cfg("f32_r32_g14", "f32", 8, 1, 64, 32, 14, 147, 5),
    # a single group, one fewer than all, and all of them
    _cfg("bf16_r32_g12_one_group", "bf16", 8, 2, 128, 32, 12, 1, 1),
    _cfg("bf16_r32_g6_all_but_one", "bf16", 8, 2, 128, 32, 6, 100, 99),
    _cfg("f32_r16_g5_every_group", "f32", 4, 2, 64, 16, 5, 77, 77),
]


@pytest.mark.parametrize("cfg", GROUPS, ids=[c.name for c in GROUPS])
def test_group_sizes_off_the_powers_of_two(cfg):
    _say(cfg.name, H.run_and_compare(cfg))


@pytest.mark.parametrize("cfg", [GROUPS[1], GROUPS[6], GROUPS[9]], ids=lambda c: c.name + "_mean")
def test_mean_reduce_over_padded_groups(cfg):
    """The empty row slots of a padded group must count as 0 in the sum and not at all in the
    divisor."""
    _say(cfg.name + "_mean", H.run_and_compare(cfg, reduce=kv.KVS_REDUCE_MEAN, check_meta=False))


@pytest.mark.parametrize("cfg,scale", [(GROUPS[1], 0.125), (GROUPS[5], 0.0), (GROUPS[7], 0.25)],
                         ids=lambda x: x.name + "_fp8" if isinstance(x, Config) else None)
def test_eight_bit_metadata_with_padded_groups(cfg, scale):
    """8-bit rows are half as wide: 32, 16 and 64 rows per load for these three."""
    _say(cfg.name + "_fp8", H.run_and_compare(cfg, meta="fp8", meta_scale=scale))


@pytest.mark.parametrize("cfg", [GROUPS[1], GROUPS[5], GROUPS[11]], ids=lambda c: c.name + "_joint")
def test_joint_head_with_padded_groups(cfg):
    j = cfg.replace(name=cfg.name + "_joint", joint=True)
    _say(j.name, H.run_and_compare(j))


def test_all_negative_scores_with_padded_groups():
    """An empty slot must never win a max: with every token score negative the group score
    is still the largest real member (an empty slot scored 0 would beat them all)."""
    cfg = GROUPS[1]
    L = make_layer(cfg)
    p, sh = H.kv_params(cfg), H.orc_shape(cfg)
    klr = oracle.build_metadata(sh, L.K, L.A)
    ref = oracle.predict_select(sh, L.q, klr, L.A)
    # scores are linear in the metadata rows: negating the rows that score above zero leaves
    # no positive score
    vals = storage_to_f32(klr).copy()
    vals[ref["s"] > 0] *= -1.0
    klr2 = f32_to_bf16_bits(vals)
    ref2 = oracle.predict_select(sh, L.q, klr2, L.A)
    assert ref2["s"].max() <= 0.0 and ref2["gs"].max() <= 0.0
    idx = torch.full(p.sets + (cfg.n_select,), -1, dtype=torch.int32, device=H.DEV)
    gs = torch.full(p.sets + (cfg.n_groups,), float("nan"), dtype=torch.float32, device=H.DEV)
    kv.kvs_predict_select(p, H.to_dev(L.q), H.to_dev(klr2), H.to_dev(L.A), idx, gs, H.workspace(p))
    torch.cuda.synchronize()
    gs_h, idx_h = gs.cpu().numpy().astype(np.float64), idx.cpu().numpy()
    assert gs_h.max() <= 0.0
    assert np.abs(gs_h - ref2["gs"]).max() / np.abs(ref2["gs"]).max() <= H.GS_TOL
    for b in range(cfg.batch):
        for k in range(cfg.n_kv_heads):
            H.check_index_margin(idx_h[b, k], ref2["gs"][b, k], ref2["boundary"][b, k], f"negative b={b} k={k}")


def test_one_problem_cut_into_the_maximum_number_of_splits():
    """A single (sequence, KV head) problem with 32 768 selected tokens: 256 attention
    workgroups, i.e. as many splits as the merge can hold (four per lane of the wave that
    weighs them, sixteen loops of the batched partial loads)."""
    cfg = _cfg("one_problem_256_splits", "bf16", 4, 1, 128, 64, 8, 8192, 4096, B=1)
    _say(cfg.name, H.run_and_compare(cfg, check_meta=False))
    # the same through the vector-ALU kernel (two heads per KV head)
    cfg2 = _cfg("one_problem_valu", "bf16", 2, 1, 128, 64, 8, 8192, 4096, B=1)
    _say(cfg2.name, H.run_and_compare(cfg2, check_meta=False))


def test_more_problems_than_workgroups_one_split_each():
    """More (sequence, KV head) problems than the attention launch has workgroups to hand
    out: every problem is one split of several workgroup steps and writes its result
    itself, without partial results or an arrival counter.  Also split counts that make
    the final merge take its partial results in rounds of 4, 8, 16 and 32, the last with a
    remainder."""
    cfg = _cfg("320_problems_matrix_core", "bf16", 32, 8, 128, 32, 4, 512, 128, B=40)
    _say(cfg.name, H.run_and_compare(cfg, check_meta=False))
    cfg2 = _cfg("576_problems_valu_f32", "f32", 16, 8, 64, 16, 4, 256, 96, B=72)
    _say(cfg2.name, H.run_and_compare(cfg2, check_meta=False))
    for name, B, Hk, NG, M in (("3_splits", 11, 8, 1024, 96), ("6_splits", 5, 8, 1024, 192),
                               ("12_splits", 11, 2, 2048, 400), ("20_splits", 13, 1, 2048, 700),
                               ("39_splits", 3, 2, 4096, 1400)):
        c = _cfg(name, "bf16", 4 * Hk, Hk, 128, 32, 4, NG, M, B=B)
        _say(c.name, H.run_and_compare(c, check_meta=False))


# ---- the paper's operating point at full context length, oracle on sampled problems ------------
def test_qwen3_14b_layer_32k_g12_full_size_sampled():
    """40 query / 8 KV heads, 32 760 tokens, G = 12, M = 33 (M*G = 396), batch 4."""
    cfg = PRESETS["c3"].replace(name="q14b_g12", batch=4, n_q_heads=40, ctx_len=12 * 2730,
                                group_size=12, n_select=33)
    H.full_size_sampled(cfg, samples=[(0, 0), (3, 7)])


def test_llama3_3b_layer_32k_g4_full_size_sampled():
    """24 query / 8 KV heads, 32 768 tokens, G = 4, M = 100, batch 8."""
    cfg = PRESETS["c3"].replace(name="l3b_g4", n_q_heads=24, n_select=100)
    H.full_size_sampled(cfg, samples=[(1, 2), (7, 5)])
