"""Seeded synthetic inputs shaped like MMDiT joint-attention layers, and per-head plans.

This module only *draws inputs*: it holds none of the operator's arithmetic and is
the one piece both the GPU library's callers and the CPU oracle's callers share.

The real workloads of the paper (Sec. 4.1: SD3 / FLUX.1-dev activations on MS-COCO
captions; Sec. 4.5: 4096+512 and 16384+512 tokens) are not available offline; the
generators below take only their shapes and the structure Sec. 3.1 describes: an
image-image block that is local around the diagonal, heads that differ from global
to very local, and an arbitrary text block.

Layout everywhere: [B, H, N, D], N = n_text + n_img, text tokens first, image token
(y, x) of a Gy x Gx latent grid at index n_text + y*Gx + x (a video latent adds a leading
frame axis: (f, y, x) at n_text + (f*Gy + y)*Gx + x).
"""
from dataclasses import dataclass, field
import math

import numpy as np
import torch

FULL, ARROW, CACHE = 0, 1, 2


@dataclass
class Workload:
    name: str
    B: int
    H: int
    D: int
    n_text: int
    n_img: int
    head_plan: np.ndarray
    window: np.ndarray
    seed: int
    positional: bool = True
    grid: tuple = None          # latent grid (Gy, Gx) or (frames, Gy, Gx); None: the most nearly square Gy x Gx
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def N(self) -> int:
        return self.n_text + self.n_img

    @property
    def scale(self) -> float:
        return 1.0 / math.sqrt(self.D)


def default_grid(n_img: int) -> tuple:
    """The most nearly square (Gy, Gx) with Gy * Gx = n_img and Gy <= Gx."""
    gy = int(math.isqrt(n_img))
    while n_img % gy:
        gy -= 1
    return (gy, n_img // gy)


def positional_term(n_img: int, D: int, amplitude: float = 1.5, grid: tuple = None) -> np.ndarray:
    """Smooth sinusoidal term [n_img, D] shared by every head and batch entry.

    Per grid axis of extent G, frequencies run from a period of 2 tokens to a period of 2G tokens;
    the features alternate sin/cos of each axis coordinate, so that q.k between two image tokens peaks
    when they are close on the grid.  With k axes the first (D // 2k) * 2k features carry the term, the
    rest stay zero.
    """
    grid = tuple(int(g) for g in (grid if grid is not None else default_grid(n_img)))
    k = len(grid)
    assert k in (2, 3) and int(np.prod(grid)) == n_img and D >= 2 * k
    nk = D // (2 * k)
    kk = np.arange(nk, dtype=np.float64)
    coords = np.stack(np.meshgrid(*[np.arange(g, dtype=np.float64) for g in grid], indexing="ij"), axis=-1)
    coords = coords.reshape(n_img, k)                      # row-major flattening: the last axis moves fastest
    pos = np.zeros((n_img, D), dtype=np.float64)
    for ax, G in enumerate(grid):
        omega = np.pi / np.power(float(max(G, 2)), kk / max(nk - 1, 1))
        c = coords[:, ax:ax + 1]
        pos[:, 2 * ax:2 * k * nk:2 * k] = np.sin(omega * c)
        pos[:, 2 * ax + 1:2 * k * nk:2 * k] = np.cos(omega * c)
    return (amplitude * pos).astype(np.float32)


def _normal(seed, stream, shape) -> np.ndarray:
    # Philox is counter based: (seed, stream) names an independent sequence.
    g = np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))
    return g.standard_normal(size=shape, dtype=np.float32)


def make_qkv(wl: Workload, step: int = 0, dtype=torch.bfloat16):
    """Q, K, V = N(0,1) (+ the positional term on image tokens), rounded to `dtype`."""
    shape = (wl.B, wl.H, wl.N, wl.D)
    outs = []
    pos = positional_term(wl.n_img, wl.D, grid=wl.grid) if (wl.positional and wl.n_img > 0) else None
    for t in range(3):
        a = _normal(wl.seed, 16 * step + t, shape)
        if pos is not None:
            a[:, :, wl.n_text:, :] += pos
        outs.append(torch.from_numpy(a).to(dtype))
    return tuple(outs)


def make_cache(wl: Workload, step: int = 0, dtype=torch.bfloat16):
    """A stand-in previous-step output buffer: N(0,1) drawn from its own stream."""
    a = _normal(wl.seed + 1, 16 * step + 7, (wl.B, wl.H, wl.N, wl.D))
    return torch.from_numpy(a).to(dtype)


def shuffled_plan(H, counts, seed):
    """counts: list of (mode, window, how_many); positions shuffled by `seed`."""
    modes, wins = [], []
    for mode, w, c in counts:
        modes += [mode] * c
        wins += [w] * c
    assert len(modes) == H
    perm = np.random.Generator(np.random.PCG64(seed)).permutation(H)
    return (np.asarray(modes, dtype=np.int32)[perm].copy(),
            np.asarray(wins, dtype=np.int32)[perm].copy())


def tiny() -> Workload:
    hp = np.array([FULL, ARROW, ARROW, CACHE], dtype=np.int32)
    win = np.array([0, 8, 16, 0], dtype=np.int32)
    return Workload("tiny", 1, 4, 64, 16, 64, hp, win, seed=0, positional=False,
                    notes="B=1 H=4 D=64 n_text=16 n_img=64 (8x8); plain N(0,1)")


def sd3_1k() -> Workload:
    hp, win = shuffled_plan(24, [(FULL, 0, 8), (ARROW, 256, 3), (ARROW, 512, 3), (ARROW, 1024, 2),
                                 (CACHE, 0, 8)], seed=2)
    return Workload("sd3_1k", 2, 24, 64, 333, 4096, hp, win, seed=2,
                    notes="SD3-medium-like 1024^2 layer, CFG pair")


def flux_1k() -> Workload:
    hp, win = shuffled_plan(24, [(FULL, 0, 6), (ARROW, 128, 3), (ARROW, 256, 3), (ARROW, 512, 3),
                                 (ARROW, 1024, 3), (CACHE, 0, 6)], seed=3)
    return Workload("flux_1k", 1, 24, 128, 512, 4096, hp, win, seed=3,
                    notes="FLUX-like 1024^2 layer")


def flux_2k_mixed() -> Workload:
    # 5 full, 13 arrow (4 x w512, 4 x w1024, 5 x w2048), 6 cache: about 68 % fewer
    # attention FLOPs than dense, the reduction the paper reports for FLUX at 2K.
    hp, win = shuffled_plan(24, [(FULL, 0, 5), (ARROW, 512, 4), (ARROW, 1024, 4), (ARROW, 2048, 5),
                                 (CACHE, 0, 6)], seed=4)
    return Workload("flux_2k_mixed", 1, 24, 128, 512, 16384, hp, win, seed=4,
                    notes="FLUX-like 2048^2 layer, mixed plan (~68 % FLOP reduction)")


def flux_2k_full() -> Workload:
    wl = flux_2k_mixed()
    wl.name = "flux_2k_full"
    wl.head_plan = np.zeros(24, dtype=np.int32)
    wl.window = np.zeros(24, dtype=np.int32)
    wl.notes = "FLUX-like 2048^2 layer, every head full (dense baseline)"
    return wl


def flux_2k_single_mode(mode: int, w: int = 0) -> Workload:
    wl = flux_2k_mixed()
    wl.name = f"flux_2k_mode{mode}_w{w}"
    wl.head_plan = np.full(24, mode, dtype=np.int32)
    wl.window = np.full(24, w, dtype=np.int32)
    return wl


def sd3_2k() -> Workload:
    """SD3-like 2048^2 layer: the 1K layer's heads and text length on a 128 x 128 latent."""
    hp, win = shuffled_plan(24, [(FULL, 0, 8), (ARROW, 512, 3), (ARROW, 1024, 3), (ARROW, 2048, 2),
                                 (CACHE, 0, 8)], seed=6)
    return Workload("sd3_2k", 2, 24, 64, 333, 16384, hp, win, seed=6,
                    notes="SD3-medium-like 2048^2 layer, CFG pair")


def flux_1k_text(n_text: int) -> Workload:
    """The FLUX-like 1024^2 layer with another prompt length (77, 154 and 256 are common encoder limits)."""
    wl = flux_1k()
    wl.name = f"flux_1k_text{n_text}"
    wl.n_text = int(n_text)
    wl.seed = 30 + int(n_text)
    return wl


def video_like() -> Workload:
    """A video MMDiT layer (Sec. 2.1 names CogVideoX, HunyuanVideo and Mochi-1 as MMDiT models): a latent of
    13 frames of 30 x 52 tokens flattened frame by frame, 256 text tokens, 24 heads of 128.  Windows are a
    fraction of a frame, one frame and two frames (a frame is 1560 tokens)."""
    hp, win = shuffled_plan(24, [(FULL, 0, 4), (ARROW, 520, 5), (ARROW, 1560, 5), (ARROW, 3120, 4),
                                 (CACHE, 0, 6)], seed=7)
    return Workload("video_like", 1, 24, 128, 256, 13 * 30 * 52, hp, win, seed=7, grid=(13, 30, 52),
                    notes="video MMDiT-like layer, 13 x 30 x 52 latent")


def schedule_plans(layers: int, steps: int, H: int = 24, seed: int = 5):
    """Per-(layer, step, head) plan: step 0 all full, cache only after step 0.

    Later steps draw 5 full / 13 arrow (w in {512, 1024, 2048}) / 6 cache per layer,
    positions and windows seeded by (seed, layer, step).
    Returns (head_plan[L,T,H], window[L,T,H]) int32.
    """
    hp = np.zeros((layers, steps, H), dtype=np.int32)
    win = np.zeros((layers, steps, H), dtype=np.int32)
    for l in range(layers):
        for t in range(1, steps):
            g = np.random.Generator(np.random.Philox(key=[seed, l * 4096 + t]))
            modes = np.array([FULL] * 5 + [ARROW] * 13 + [CACHE] * 6, dtype=np.int32)
            ws = g.choice(np.array([512, 1024, 2048], dtype=np.int32), size=H)
            perm = g.permutation(H)
            hp[l, t] = modes[perm]
            win[l, t] = np.where(hp[l, t] == ARROW, ws, 0)
    return hp, win


CONFIGS = {
    "tiny": tiny, "sd3_1k": sd3_1k, "flux_1k": flux_1k,
    "flux_2k_mixed": flux_2k_mixed, "flux_2k_full": flux_2k_full,
    "sd3_2k": sd3_2k, "video_like": video_like,
    "flux_1k_text77": lambda: flux_1k_text(77), "flux_1k_text154": lambda: flux_1k_text(154),
    "flux_1k_text256": lambda: flux_1k_text(256),
}


def config(name: str) -> Workload:
    return CONFIGS[name]()
