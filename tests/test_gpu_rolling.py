"""GPU parity of the rolling buffer (Sec. 3.4.1: newest tokens outside the cache, never
scored, always attended), of caches with spare row capacity, and of the incremental
update when a group completes, against the CPU oracle, through the C-ABI binding."""
import numpy as np
import pytest
import torch

import oracle
import paper_2511_11907_amd as kv
import gpu_harness as H
from workloads import PRESETS, Config, make_layer, storage_to_f32, f32_to_bf16_bits

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.fail("these tests need the GPU (run them with -m gpu on a GPU box)")
    kv.load_library()


def _say(name, stats):
    print(f"[parity] {name}: " + ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}"
                                           for k, v in stats.items()), flush=True)


def _store(x, dtype):
    return f32_to_bf16_bits(x) if dtype == "bf16" else np.ascontiguousarray(x, np.float32)


def _buffer(cfg, cap, seed):
    g = np.random.default_rng(seed)
    shape = (cfg.batch, cfg.n_kv_heads, cap, cfg.head_dim)
    return (_store(g.standard_normal(shape).astype(np.float32), cfg.dtype),
            _store(g.standard_normal(shape).astype(np.float32), cfg.dtype))


def _pad_rows(x, rows, fill):
    """[..., N, c] storage array -> [..., rows, c] with the extra rows filled (poisoned)."""
    out = np.empty(x.shape[:-2] + (rows, x.shape[-1]), dtype=x.dtype)
    out[..., :x.shape[-2], :] = x
    out[..., x.shape[-2]:, :] = fill
    return out


def _poison(dtype):
    return np.uint16(0x7FC0) if dtype == "bf16" else np.float32(np.nan)   # NaN in either format


CASES = [
    # (config, spare rows, buffer capacity)
    (PRESETS["c2"].replace(name="c2s", batch=2, ctx_len=4096, n_select=103), 0, 4),
    (PRESETS["c2"].replace(name="c2r", batch=1, ctx_len=4004, n_select=77), 12, 8),
    (PRESETS["c4"].replace(name="c4s", batch=1, ctx_len=16384, n_select=256), 8, 8),
    (PRESETS["c1"].replace(name="c1cap", ctx_len=2048, n_select=40), 64, 16),
    (PRESETS["c2j"].replace(name="c2js", batch=2, ctx_len=4096, n_select=103), 4, 4),
    (Config("f32_g1_qpk8", 1, 2, 8, 1, 64, 1024, 16, 1, 33, "f32", 16, 0.1, 8), 3, 5),
    (Config("bf16_g16_qpk2", 1, 2, 4, 2, 128, 2048, 64, 16, 9, "bf16", 32, 0.1, 8), 16, 16),
    # group sizes and head ratios off the powers of two (App. A.4 searches G in steps of one;
    # Qwen3-14B has 5 query heads per KV head, LLaMA3-3B 3, Qwen2.5-VL-7B 7)
    (Config("bf16_g12_qpk5", 1, 2, 10, 2, 128, 12 * 170, 32, 12, 33, "bf16", 32, 0.1, 8), 24, 12),
    (Config("f32_g3_qpk3", 1, 2, 6, 2, 64, 3 * 683, 16, 3, 41, "f32", 16, 0.1, 8), 5, 3),
    (Config("bf16_g6_qpk7", 1, 1, 7, 1, 128, 6 * 300, 64, 6, 20, "bf16", 32, 0.1, 8), 0, 7),
]


# seeded random draws from the supported shape space (the same ones the plain path is tested on)
from test_gpu_random_shapes import _draw  # noqa: E402
for _seed in (2, 5, 7, 13, 18, 21, 26, 30):
    _c = _draw(_seed)[0]
    CASES.append((_c, (3 * _seed) % 17, _c.group_size + _seed % 5))


@pytest.mark.parametrize("cfg,spare,cap", CASES, ids=[c[0].name for c in CASES])
def test_attention_with_rolling_buffer_and_spare_capacity(cfg, spare, cap):
    L = make_layer(cfg)
    rows = cfg.ctx_len + spare
    p = H.kv_params(cfg, ctx_capacity=rows if spare else 0)
    sh = H.orc_shape(cfg, ctx_capacity=rows if spare else 0)
    Kp, Vp = _pad_rows(L.K, rows, _poison(cfg.dtype)), _pad_rows(L.V, rows, _poison(cfg.dtype))
    klr = oracle.build_metadata(sh, Kp, L.A)
    klr[..., cfg.ctx_len:, :] = _poison(cfg.dtype)
    ref = oracle.predict_select(sh, L.q, klr, L.A)
    dK, dV, dq, dA, dklr = (H.to_dev(x) for x in (Kp, Vp, L.q, L.A, klr))
    rbK, rbV = _buffer(cfg, cap, 3)
    drK, drV = H.to_dev(rbK), H.to_dev(rbV)
    ws = H.workspace(p)
    M = cfg.n_select
    stats = {}
    for rb_len in sorted({0, 1, cap - 1, cap}):
        # poison the rows of the buffer that are not valid
        drK[:] = H.to_dev(rbK)
        drV[:] = H.to_dev(rbV)
        drK[:, :, rb_len:] = float("nan")
        drV[:, :, rb_len:] = float("nan")
        out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=dq.dtype, device=H.DEV)
        kv.kvs_sparse_decode_attn_rb(p, dq, dK, dV, H.to_dev(ref["idx"]), drK, drV, rb_len, out, ws)
        torch.cuda.synchronize()
        want = oracle.sparse_attn(sh, L.q, Kp, Vp, ref["idx"], rbK, rbV, rb_len)
        stats[f"rb{rb_len}"] = H.attn_error(H.out_values(out), want)
        assert stats[f"rb{rb_len}"] <= H.ATTN_TOL[cfg.dtype], stats
    # the whole step on the padded cache: same selection as the oracle's rule allows
    idx = torch.full(p.sets + (M,), -1, dtype=torch.int32, device=H.DEV)
    out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=dq.dtype, device=H.DEV)
    drK[:] = H.to_dev(rbK)
    drV[:] = H.to_dev(rbV)
    kv.kvs_decode_step_rb(p, dq, dklr, dA, dK, dV, drK, drV, cap, idx, None, out, ws)
    torch.cuda.synchronize()
    idx_h = idx.cpu().numpy()
    flat = lambda a: a.reshape((-1,) + a.shape[len(p.sets):])
    for i, (ig, gr, bd) in enumerate(zip(flat(idx_h), flat(ref["gs"]), flat(ref["boundary"]))):
        H.check_index_margin(ig, gr, bd, f"{cfg.name} set {i}")
    want = oracle.sparse_attn(sh, L.q, Kp, Vp, idx_h, rbK, rbV, cap)
    stats["step"] = H.attn_error(H.out_values(out), want)
    assert stats["step"] <= H.ATTN_TOL[cfg.dtype], stats
    _say(cfg.name, stats)


@pytest.mark.parametrize("shape", ["g4_qpk4", "g12_qpk5"])
@pytest.mark.parametrize("joint", [False, True], ids=["per_head", "joint"])
def test_decode_loop_appends_groups_and_matches_the_oracle_every_step(joint, shape):
    """A decode loop over 3 G + 2 tokens: each new token enters the rolling buffer and is
    attended at once; when the buffer holds a group it is appended to the cache (rows and
    metadata) and takes part in the prediction from then on."""
    base = PRESETS["c2j" if joint else "c2"]
    if shape == "g12_qpk5":                               # the Qwen3-14B head geometry at G = 12
        base = base.replace(n_q_heads=40, group_size=12)
    G = base.group_size
    N0, steps = 2048 // G * G, 3 * G + 2
    cap_rows = N0 + 4 * G
    cfg = base.replace(name="loop", batch=2, ctx_len=cap_rows, n_select=52)
    L = make_layer(cfg)                                   # rows beyond N0 are the tokens to come
    hK, hV = L.K.copy(), L.V.copy()
    poison = _poison(cfg.dtype)
    hK[:, :, N0:] = poison
    hV[:, :, N0:] = poison
    dK, dV, dq, dA = (H.to_dev(x) for x in (hK, hV, L.q, L.A))
    sh0 = H.orc_shape(cfg, ctx_len=N0, ctx_capacity=cap_rows)
    hklr = oracle.build_metadata(sh0, hK, L.A)
    hklr[..., N0:, :] = poison
    dklr = H.to_dev(hklr)
    rbK = np.full((cfg.batch, cfg.n_kv_heads, G, cfg.head_dim), poison, dtype=hK.dtype)
    rbV = rbK.copy()
    drK, drV = H.to_dev(rbK), H.to_dev(rbV)
    N, rb_len, worst, appended = N0, 0, 0.0, 0
    p0 = H.kv_params(cfg, ctx_len=cap_rows)               # largest params the loop will use
    ws = H.workspace(p0)
    for t in range(steps):
        # the new token's K, V (taken from the generated layer) enter the buffer
        rbK[:, :, rb_len] = L.K[:, :, N + rb_len]
        rbV[:, :, rb_len] = L.V[:, :, N + rb_len]
        drK[:, :, rb_len] = H.to_dev(np.ascontiguousarray(L.K[:, :, N + rb_len]))
        drV[:, :, rb_len] = H.to_dev(np.ascontiguousarray(L.V[:, :, N + rb_len]))
        rb_len += 1
        p = H.kv_params(cfg, ctx_len=N, ctx_capacity=cap_rows)
        sh = H.orc_shape(cfg, ctx_len=N, ctx_capacity=cap_rows)
        idx = torch.full(p.sets + (cfg.n_select,), -1, dtype=torch.int32, device=H.DEV)
        out = torch.full((cfg.batch, cfg.n_q_heads, cfg.head_dim), float("nan"), dtype=dq.dtype, device=H.DEV)
        print(f"[loop] step {t}: N={N} rb_len={rb_len}", flush=True)
        kv.kvs_decode_step_rb(p, dq, dklr, dA, dK, dV, drK, drV, rb_len, idx, None, out, ws)
        torch.cuda.synchronize()
        ref = oracle.predict_select(sh, L.q, hklr, L.A)
        idx_h = idx.cpu().numpy()
        flat = lambda a: a.reshape((-1,) + a.shape[len(p.sets):])
        for i, (ig, gr, bd) in enumerate(zip(flat(idx_h), flat(ref["gs"]), flat(ref["boundary"]))):
            H.check_index_margin(ig, gr, bd, f"loop step {t} set {i}")
        want = oracle.sparse_attn(sh, L.q, hK, hV, idx_h, rbK, rbV, rb_len)
        err = H.attn_error(H.out_values(out), want)
        assert err <= H.ATTN_TOL[cfg.dtype], (t, err)
        worst = max(worst, err)
        if rb_len == G:                                   # the group is complete: offload it
            kv.kvs_append_group(p, drK, drV, dK, dV, dA, dklr)
            torch.cuda.synchronize()
            hK[:, :, N:N + G] = rbK
            hV[:, :, N:N + G] = rbV
            assert np.array_equal(H.to_host_storage(dK), hK) and np.array_equal(H.to_host_storage(dV), hV)
            exact = np.zeros(hklr.shape, np.float64)
            oracle.build_metadata_rows(sh, hK, L.A, hklr, N, G, exact)
            got = H.to_host_storage(dklr)
            new = np.s_[..., N:N + G, :]
            absdot = np.einsum("bknd,kdr->bnr" if joint else "bknd,kdr->bknr",
                               np.abs(storage_to_f32(hK[:, :, N:N + G])).astype(np.float64),
                               np.abs(L.A).astype(np.float64))
            H.compare_metadata(got[new], hklr[new], exact[new], absdot,
                               cfg.head_dim * (cfg.n_kv_heads if joint else 1), cfg.dtype)
            old = np.s_[..., :N, :]
            assert np.array_equal(got[old], hklr[old])    # earlier rows untouched
            dklr[new] = H.to_dev(np.ascontiguousarray(hklr[new]))   # both sides score the same rows
            N, rb_len, appended = N + G, 0, appended + 1
            rbK[:], rbV[:] = poison, poison
            drK[:] = float("nan")
            drV[:] = float("nan")
    assert appended == 3 and N == N0 + 3 * G and rb_len == 2
    _say(f"decode_loop_{shape}_" + ("joint" if joint else "per_head"),
         {"worst_attn_err": worst, "appended": appended})
