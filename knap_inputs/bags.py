"""Seeded generators of sequence-length bags.

Two families:

* the five benchmark bags (tiny, mixed-resolution image, image+video, skewed,
  post-Ulysses share), which stand in for the paper's mixed-resolution and
  joint image-video simulator workloads (Sec. 4.1, Table 1);
* the paper's own data-code streams ``g{G}b{B}i{R}f{F}s{S}`` (Sec. 4.1), used
  to rebuild the per-GPU length lists behind Table 1.

Only lengths are produced here; no cost model and no assignment logic.
"""
from __future__ import annotations

import re
from dataclasses import dataclass, field
from typing import List, Sequence

import numpy as np

CONFIG_NAMES = (
    "tiny",            # configs[0]
    "mixed_res_image",  # configs[1]
    "image_video",     # configs[2]
    "skewed",          # configs[3]
    "post_ulysses",    # configs[4]
)

BASE_SEED = 20250806

# image token counts for 256^2, 512^2, 768^2, 1024^2 and 768x1344 pixels at a
# spatial compression of 16 per side (patching included)
IMAGE_TOKENS = (256, 1024, 2304, 4096, 4032)
# 480x832 video: 30x52 tokens per latent frame, (F-1)/4+1 latent frames
VIDEO_FRAMES = (17, 33, 61)
VIDEO_TOKENS_PER_LATENT_FRAME = 30 * 52


@dataclass
class BagSpec:
    name: str
    seq_lens: List[int]
    H: int
    d: int
    seed: int
    k_outlier_prob: float = 0.0   # each k entry independently scaled by k_outlier_scale
    k_outlier_scale: float = 1.0
    notes: str = ""
    extra: dict = field(default_factory=dict)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    @property
    def sum_l2(self) -> int:
        return int(sum(int(l) * int(l) for l in self.seq_lens))


def cu_seqlens_of(seq_lens: Sequence[int]) -> np.ndarray:
    """Prefix sums of the lengths, int32, cu[0] = 0."""
    cu = np.zeros(len(seq_lens) + 1, dtype=np.int64)
    np.cumsum(np.asarray(seq_lens, dtype=np.int64), out=cu[1:])
    if cu[-1] >= 2**31:
        raise ValueError("total tokens exceed int32")
    return cu.astype(np.int32)


def _length_rng(seed: int) -> np.random.Generator:
    # sub-stream 0 of the seed = lengths; sub-stream 1.. = tensor values (tensors.py)
    return np.random.Generator(np.random.Philox(np.random.SeedSequence([seed, 0])))


def _image_sample(rng: np.random.Generator, text_lo: int = 16, text_hi: int = 512) -> int:
    text = int(rng.integers(text_lo, text_hi + 1))
    img = int(IMAGE_TOKENS[int(rng.integers(0, len(IMAGE_TOKENS)))])
    return text + img


def _video_sample(rng: np.random.Generator) -> int:
    frames = int(VIDEO_FRAMES[int(rng.integers(0, len(VIDEO_FRAMES)))])
    latent = (frames - 1) // 4 + 1
    text = int(rng.integers(64, 512 + 1))
    return text + latent * VIDEO_TOKENS_PER_LATENT_FRAME


def _fill(rng: np.random.Generator, target: int, draw) -> List[int]:
    """Add samples until the total is within [0.95, 1.05] of target.

    A drawn sample that would overshoot 1.05*target is redrawn (at most 64
    times in a row); the bag is closed once 0.95*target is reached.
    """
    lens: List[int] = []
    total = 0
    while total < 0.95 * target:
        for _ in range(64):
            l = draw(rng)
            if total + l <= 1.05 * target:
                lens.append(l)
                total += l
                break
        else:
            break
    return lens


def config_bag(index: int, seed_offset: int = 0, long_position: str = "first") -> BagSpec:
    """The bag of benchmark configuration ``index`` (0..4).

    ``seed_offset`` selects an alternative draw; ``long_position`` ("first",
    "middle", "last") moves the long sequence of the skewed bag.
    """
    seed = BASE_SEED + index + 1000 * seed_offset
    rng = _length_rng(seed)
    if index == 0:
        return BagSpec("tiny", [37, 128, 200, 311], H=2, d=64, seed=seed)
    if index == 1:
        lens = _fill(rng, 32768, _image_sample)
        return BagSpec("mixed_res_image", lens, H=24, d=128, seed=seed)
    if index == 2:
        def draw(r):
            return _image_sample(r) if r.random() < 0.5 else _video_sample(r)
        lens = _fill(rng, 65536, draw)
        return BagSpec("image_video", lens, H=24, d=128, seed=seed)
    if index == 3:
        short = [int(x) for x in rng.integers(200, 401, size=200)]
        if long_position == "first":
            lens = [65536] + short
        elif long_position == "last":
            lens = short + [65536]
        elif long_position == "middle":
            lens = short[:100] + [65536] + short[100:]
        else:
            raise ValueError(long_position)
        return BagSpec("skewed", lens, H=24, d=128, seed=seed,
                       k_outlier_prob=0.01, k_outlier_scale=8.0)
    if index == 4:
        return BagSpec("post_ulysses", [131072, 32768, 8192, 8192, 8192, 8192], H=3, d=128, seed=seed)
    raise IndexError(index)


# --------------------------------------------------------------------------
# The paper's data codes (Sec. 4.1): g{G}b{B}i{R}f{F}s{S}
# --------------------------------------------------------------------------

_CODE_RE = re.compile(r"^g(\d+)b(\d+)i(\d+)f(\d+)s(\d+)$")


def parse_data_code(code: str) -> dict:
    m = _CODE_RE.match(code.strip())
    if not m:
        raise ValueError(f"bad data code {code!r}")
    g, b, r, f, s = (int(x) for x in m.groups())
    return {"gpus": g, "batch": b, "res": r, "frames": f, "smooth": s}


def data_code_lengths(code: str, rng: np.random.Generator | None = None) -> List[List[int]]:
    """Per-GPU lists of sequence lengths for one data code.

    Visual tokens = (R/16)^2 x F' with F' = F when S = 0 (sparse key frames) and
    F/3.4 when S = 1 (a clip with temporal compression; 17 frames -> 5, 85 -> 25).
    With ``rng`` None the deterministic mean stream is returned: 196 text tokens
    and no aspect jitter.  Otherwise text ~ U{0..392} per sample and one aspect
    multiplier U[0.96, 1.04] per batch (per GPU).
    """
    c = parse_data_code(code)
    spatial = (c["res"] // 16) ** 2
    frames = c["frames"] if c["smooth"] == 0 else int(round(c["frames"] / 3.4))
    out: List[List[int]] = []
    for _ in range(c["gpus"]):
        if rng is None:
            out.append([196 + spatial * frames] * c["batch"])
        else:
            mult = float(rng.uniform(0.96, 1.04))
            vis = int(round(spatial * mult)) * frames
            out.append([int(rng.integers(0, 393)) + vis for _ in range(c["batch"])])
    return out


TABLE1_WORKLOADS = {
    "low_res": ["g32b32i256f1s0"],
    "mixed_res": ["g16b4i256f1s0", "g4b5i512f1s0", "g4b5i1024f1s0", "g8b1i2048f1s0"],
    "joint": ["g8b4i256f1s0", "g2b5i512f1s0", "g2b5i1024f1s0", "g4b1i2048f1s0",
              "g1b10i256f4s0", "g3b1i512f4s0", "g8b2i256f85s1", "g4b1i512f85s1"],
}


def table1_streams(workload: str, seed: int | None = None) -> List[List[int]]:
    """Per-GPU sequence lengths of one Table 1 workload on 32 GPUs (rank order)."""
    rng = None if seed is None else np.random.Generator(np.random.Philox(seed))
    per_gpu: List[List[int]] = []
    for code in TABLE1_WORKLOADS[workload]:
        per_gpu.extend(data_code_lengths(code, rng))
    return per_gpu
