"""Workload shapes and seeded input generators (no method arithmetic here)."""
from __future__ import annotations

import dataclasses
from concurrent.futures import ThreadPoolExecutor

import numpy as np


@dataclasses.dataclass(frozen=True)
class MoeConfig:
    """One MoE-FFN problem instance: one GPU's expert-parallel share.

    T tokens, H hidden, I per-expert intermediate, E global experts of which
    this device owns ids ``expert_base .. expert_base+E_local-1``, top-k ``k``.
    ``dtype`` is "f32" or "bf16" (storage type of x, weights, outputs; router
    logits are always fp32).  ``skew`` adds the Zipf-like per-expert bias.
    """

    name: str
    T: int
    H: int
    I: int
    E: int
    E_local: int
    expert_base: int
    k: int
    dtype: str
    seed: int
    skew: bool = False

    @property
    def R_max(self) -> int:
        return self.T * min(self.k, self.E_local)


CONFIGS = {
    # tiny fp32 forward
    "c1": MoeConfig("c1", 256, 256, 128, 8, 8, 0, 2, "f32", 1001),
    # mid-size bf16 forward
    "c2": MoeConfig("c2", 4096, 2048, 1408, 16, 16, 0, 4, "bf16", 1002),
    # DeepSeek-V3-shaped EP=8 share (experts 0..31 of 256), bf16
    "c3": MoeConfig("c3", 8192, 7168, 2048, 256, 32, 0, 8, "bf16", 1003),
    # skewed-load variant of c3
    "c4": MoeConfig("c4", 8192, 7168, 2048, 256, 32, 0, 8, "bf16", 1004, skew=True),
    # forward + backward at c3 shapes (adds dY)
    "c5": MoeConfig("c5", 8192, 7168, 2048, 256, 32, 0, 8, "bf16", 1005),
}


def bf16_round(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to the nearest bf16 (ties to even); result stays fp32.

    Storage conversion only: the returned fp32 array holds values that are
    exactly representable in bf16, so a later cast to bf16 is lossless.
    """
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = (u + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


_TENSOR_IDS = {"x": 0, "logits": 1, "w_gate_up": 2, "w_down": 3, "dy": 4, "ranks": 5, "mb_x": 6, "mb_y": 7}


def _normal(seed: int, tensor: str, shape, scale: float, bf16: bool) -> np.ndarray:
    """N(0, scale^2) fp32 tensor; leading axis drawn as independent sub-streams.

    Each slice along axis 0 (in blocks) has its own child seed, so the values do
    not depend on how many threads draw them.
    """
    shape = tuple(int(s) for s in shape)
    out = np.empty(shape, dtype=np.float32)
    n0 = shape[0]
    per = int(np.prod(shape[1:])) if len(shape) > 1 else 1
    # blocks of about 16M elements along axis 0
    rows_per_block = max(1, min(n0, (1 << 24) // max(per, 1)))
    n_blocks = (n0 + rows_per_block - 1) // rows_per_block
    children = np.random.SeedSequence([seed, _TENSOR_IDS[tensor]]).spawn(n_blocks)

    def draw(b: int) -> None:
        lo = b * rows_per_block
        hi = min(n0, lo + rows_per_block)
        g = np.random.Generator(np.random.PCG64(children[b]))
        blk = out[lo:hi]
        g.standard_normal(out=blk.reshape(-1), dtype=np.float32)
        if scale != 1.0:
            blk *= np.float32(scale)
        if bf16:
            blk[...] = bf16_round(blk)

    if n_blocks == 1:
        draw(0)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(draw, range(n_blocks)))
    return out


def expert_bias(cfg: MoeConfig) -> np.ndarray:
    """Additive router bias b_e = 2.0*log(1/rank_e^1.2) for the skewed workload.

    rank_e in 1..E is a seeded permutation of the experts.  The logarithm is
    taken base 10 (b_e = -2.4*log10(rank_e)): with that reading and this seed
    the hottest local expert of workload c4 gets about 11x the mean rows and 9
    of the 32 local experts get none, which is the load shape the workload is
    meant to have; the natural logarithm would leave 24+ of them empty.
    Returns zeros for unskewed workloads.
    """
    if not cfg.skew:
        return np.zeros(cfg.E, dtype=np.float32)
    g = np.random.Generator(np.random.PCG64(np.random.SeedSequence([cfg.seed, _TENSOR_IDS["ranks"]])))
    rank = g.permutation(cfg.E) + 1
    return (2.0 * np.log10(1.0 / rank.astype(np.float64) ** 1.2)).astype(np.float32)


def make_inputs(cfg: MoeConfig, with_dy: bool = False) -> dict:
    """Draw all inputs of one workload as fp32 numpy arrays.

    For bf16 workloads x, the weights and dY hold bf16-representable values
    (rounded to nearest even), so uploading them as bf16 is exact and the fp64
    oracle sees precisely the numbers the device sees.  Logits stay fp32.
    """
    bf = cfg.dtype == "bf16"
    T, H, I, E, El = cfg.T, cfg.H, cfg.I, cfg.E, cfg.E_local
    inp = {
        "x": _normal(cfg.seed, "x", (T, H), 1.0, bf),
        "logits": _normal(cfg.seed, "logits", (T, E), 1.0, False),
        "w_gate_up": _normal(cfg.seed, "w_gate_up", (El, H, 2 * I), 1.0 / np.sqrt(H), bf),
        "w_down": _normal(cfg.seed, "w_down", (El, I, H), 1.0 / np.sqrt(I), bf),
    }
    if cfg.skew:
        inp["logits"] = (inp["logits"] + expert_bias(cfg)[None, :]).astype(np.float32)
    if with_dy:
        inp["dy"] = _normal(cfg.seed, "dy", (T, H), 1.0, bf)
    return inp


def realised_local_counts(cfg: MoeConfig, logits: np.ndarray) -> np.ndarray:
    """Rows per local expert for a logits draw (diagnostic for the skew recipe).

    Uses a plain partial sort; ties are irrelevant for a histogram diagnostic.
    """
    top = np.argpartition(-logits, cfg.k - 1, axis=1)[:, : cfg.k]
    cnt = np.bincount(top.reshape(-1), minlength=cfg.E)
    return cnt[cfg.expert_base : cfg.expert_base + cfg.E_local]


def make_microbench_inputs(M: int, N: int = 2048, seed: int = 2006) -> dict:
    """Inputs of the SwiGLU + Add operator pair (the paper's Section 6): X [M, 2N] and
    Y [M, N], standard normal, stored as bf16-representable fp32."""
    return dict(x=_normal(seed, "mb_x", (M, 2 * N), 1.0, True), y=_normal(seed, "mb_y", (M, N), 1.0, True))
