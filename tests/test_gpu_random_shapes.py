"""Parity of the HIP path against the CPU oracle on seeded random draws from the supported
shape space (head ratio, head dimension, rank, group size, group count, budget, batch,
head mode, storage types, reduce).  Needs an MI355X: run with  -m gpu."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

import paper_2511_11907_amd as kv  # noqa: E402
from workloads import Config  # noqa: E402

import gpu_harness as H  # noqa: E402


@pytest.fixture(scope="module", autouse=True)
def _need_gpu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    assert "gfx950" in kv.kvs_version()


def _draw(seed: int):
    g = np.random.default_rng(1000 + seed)
    dtype = "bf16" if g.random() < 0.7 else "f32"
    d = int(g.choice([64, 128], p=[0.3, 0.7]))
    Hk = int(g.integers(1, 4))
    qpk = int(g.integers(1, 9))
    joint = bool(g.random() < 0.25)
    ranks = [r for r in (16, 32, 64, 128) if r <= (Hk * d if joint else d)]
    r = int(g.choice(ranks))
    G = int(g.integers(1, 17))
    NG = int(g.integers(1, 700))
    M = int(g.integers(1, NG + 1)) if g.random() < 0.8 else NG
    B = int(g.integers(1, 4))
    meta = str(g.choice(["same", "same", "fp8", "f32" if dtype == "bf16" else "bf16"]))
    reduce = int(g.random() < 0.25)
    cfg = Config(f"rand{seed}_{dtype}_d{d}_{Hk * qpk}q{Hk}kv_r{r}_g{G}_ng{NG}_m{M}_b{B}" + ("_joint" if joint else ""),
                 1, B, Hk * qpk, Hk, d, NG * G, r, G, M, dtype, min(r, 32), 0.1, 8, joint=joint)
    return cfg, (None if meta == "same" else meta), reduce


@pytest.mark.parametrize("seed", range(32))
def test_random_shape(seed):
    cfg, meta, reduce = _draw(seed)
    scale = 0.125 if meta == "fp8" else 0.0
    stats = H.run_and_compare(cfg, reduce=reduce, meta=meta, meta_scale=scale, check_meta=(reduce == 0))
    print(f"[random] {cfg.name} meta={meta or cfg.dtype} reduce={reduce}: " +
          ", ".join(f"{k}={v:.3g}" if isinstance(v, float) else f"{k}={v}" for k, v in stats.items()), flush=True)
