"""Seeded synthetic inputs shaped like the paper's student/teacher workloads.

This module only draws random numbers and lays them out; it contains none of the
method's arithmetic (no softmax, no KL, no gradient).  Both the CPU oracle's tests
and the GPU path's tests/benchmark take their inputs from here, so that the two
sides see bit-identical bf16 values.

Shapes follow the paper's setup: Qwen3-like hidden sizes and a 151,936-entry
vocabulary (base models paragraph of the experimental setup), responses up to
8,192 tokens (OPD hyper-parameter table), candidate windows {64..2048} (training
details).  The datasets and checkpoints themselves are not used: every tensor is
i.i.d. normal, rounded to bf16.
"""
from __future__ import annotations

import dataclasses
import zlib

import numpy as np
import torch

SEED = 20260528

MODE_PREFIX_ONLY = 0
MODE_PREFIX_AND_FULL = 1


@dataclasses.dataclass
class Workload:
    """Shape and ragged structure of one configuration (no tensors)."""
    name: str
    V: int
    H_s: int            # 0 for the logits-given workload
    H_t: int
    offsets: np.ndarray  # int64 [B+1]
    window: np.ndarray   # int32 [B]
    mode: int = MODE_PREFIX_ONLY

    @property
    def B(self) -> int:
        return int(self.window.shape[0])

    @property
    def T(self) -> int:
        return int(self.offsets[-1])


def _rng(*key) -> np.random.Generator:
    h = zlib.crc32(repr(key).encode())
    return np.random.Generator(np.random.Philox(key=[SEED, h]))


def _offsets(lens) -> np.ndarray:
    off = np.zeros(len(lens) + 1, dtype=np.int64)
    off[1:] = np.cumsum(np.asarray(lens, dtype=np.int64))
    return off


def _adjust_to_total(lens: np.ndarray, total: int, lo: int, hi: int) -> np.ndarray:
    """Deterministically nudge lengths so they sum to `total`, staying in [lo, hi]."""
    lens = lens.astype(np.int64).copy()
    while lens.sum() > total:
        cand = np.where(lens > lo)[0]
        i = cand[np.argmax(lens[cand])]
        lens[i] -= min(int(lens.sum() - total), int(lens[i] - lo))
    while lens.sum() < total:
        cand = np.where(lens < hi)[0]
        i = cand[np.argmin(lens[cand])]
        lens[i] += min(int(total - lens.sum()), int(hi - lens[i]))
    return lens


def workload(name: str) -> Workload:
    """The five benchmark configurations plus a few small ragged test shapes."""
    if name == "tiny":
        return Workload("tiny", 4096, 256, 384, _offsets([96, 128]),
                        np.array([64, 128], np.int32))
    if name == "tiny_probe":
        w = workload("tiny")
        return dataclasses.replace(w, name="tiny_probe", mode=MODE_PREFIX_AND_FULL)
    if name == "logits_given":
        g = _rng("cfg2")
        lens = g.integers(256, 2048, size=32, endpoint=True)
        lens = _adjust_to_total(lens, 32768, 256, 2048)
        win = np.array([g.integers(64, l, endpoint=True) for l in lens], np.int32)
        return Workload("logits_given", 151936, 0, 0, _offsets(lens), win)
    if name == "strong_to_weak":
        g = _rng("cfg3")
        lens = g.integers(1024, 8192, size=64, endpoint=True)
        return Workload("strong_to_weak", 151936, 2048, 4096, _offsets(lens),
                        np.full(64, 1024, np.int32))
    if name == "same_family":
        g = _rng("cfg4")
        lens = g.integers(512, 4096, size=128, endpoint=True)
        win = g.choice(np.array([256, 512, 1024, 2048]), size=128)
        win = np.minimum(win, lens).astype(np.int32)
        return Workload("same_family", 151936, 2560, 4096, _offsets(lens), win)
    if name == "probe_alignment":
        g = _rng("cfg5")
        lens = g.integers(8192, 16384, size=16, endpoint=True)
        return Workload("probe_alignment", 151936, 2048, 4096, _offsets(lens),
                        np.full(16, 2048, np.int32), MODE_PREFIX_AND_FULL)
    # small ragged shapes for parity tests: several tiles plus ragged tails, an
    # empty rollout, a zero window and a window longer than its rollout
    if name == "ragged_small":
        return Workload("ragged_small", 1000 * 8, 192, 320,
                        _offsets([37, 0, 301, 5, 129, 64]),
                        np.array([64, 16, 200, 0, 4096, 64], np.int32),
                        MODE_PREFIX_AND_FULL)
    if name == "ragged_mid":
        g = _rng("ragged_mid")
        lens = g.integers(1, 700, size=9, endpoint=True)
        win = g.integers(0, 800, size=9, endpoint=True).astype(np.int32)
        return Workload("ragged_mid", 128 * 93 + 8, 512, 640, _offsets(lens), win,
                        MODE_PREFIX_AND_FULL)
    raise KeyError(name)


WORKLOADS = ("tiny", "logits_given", "strong_to_weak", "same_family", "probe_alignment")


# ---------------------------------------------------------------------------
# tensors
# ---------------------------------------------------------------------------

def _torch_gen(device, *key) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((SEED << 20) ^ zlib.crc32(repr(key).encode()))
    return g


def normal_bf16(shape, std: float, key, device="cpu", row_shift=None,
                chunk_rows: int = 8192) -> torch.Tensor:
    """bf16 tensor of N(0, std^2) draws (fp32 draws rounded to nearest-even bf16).

    `row_shift` (fp32 [rows]) is added per row before rounding.  Generated in row
    chunks so the fp32 temporary stays small.  The same key and device type always
    give the same bits.
    """
    rows, cols = int(shape[0]), int(shape[1])
    out = torch.empty((rows, cols), dtype=torch.bfloat16, device=device)
    g = _torch_gen(device, key)
    for r0 in range(0, rows, chunk_rows):
        r1 = min(rows, r0 + chunk_rows)
        x = torch.randn((r1 - r0, cols), generator=g, device=device, dtype=torch.float32)
        x.mul_(std)
        if row_shift is not None:
            x.add_(row_shift[r0:r1].to(device=device, dtype=torch.float32)[:, None])
        out[r0:r1] = x.to(torch.bfloat16)
    return out


def uniform_ids(T: int, V: int, key, device="cpu") -> torch.Tensor:
    g = _torch_gen("cpu", key)
    ids = torch.randint(0, V, (T,), generator=g, dtype=torch.int32)
    return ids.to(device)


def hidden_problem(w: Workload, device="cpu") -> dict:
    """Hidden states ~N(0,1) and LM-head weights ~N(0,0.02^2), bf16; uniform ids."""
    return {
        "h_s": normal_bf16((w.T, w.H_s), 1.0, (w.name, "h_s"), device),
        "h_t": normal_bf16((w.T, w.H_t), 1.0, (w.name, "h_t"), device),
        "W_s": normal_bf16((w.V, w.H_s), 0.02, (w.name, "W_s"), device),
        "W_t": normal_bf16((w.V, w.H_t), 0.02, (w.name, "W_t"), device),
        "ids": uniform_ids(w.T, w.V, (w.name, "ids"), device),
    }


def peaked_problem(w: Workload, device="cpu", logit_std: float = 4.0, teacher_noise: float = 0.3) -> dict:
    """A same-family pair with peaked distributions, the regime of trained language models
    rather than of random initialisation: student logits ~N(0, logit_std^2) (a handful of
    entries carry most of the mass), the teacher a perturbed copy of the student (its first H_s
    hidden columns are h_s + noise and W_s + noise, any further columns small noise; needs
    H_t >= H_s), so that the KL is of order one and z_s - z_t is small against the spread of the
    logits.  The rows of W grow with the entry index, so the largest logits tend to sit late in
    the vocabulary and references taken from its first entries lie far below the row maximum."""
    assert w.H_t >= w.H_s
    sd = logit_std / float(w.H_s) ** 0.5
    h_s = normal_bf16((w.T, w.H_s), 1.0, (w.name, "pk_h_s"), device)
    W_s = normal_bf16((w.V, w.H_s), sd, (w.name, "pk_W_s"), device)
    W_s.mul_(torch.linspace(0.5, 1.5, w.V, device=device, dtype=torch.float32)[:, None].to(torch.bfloat16))
    h_t = normal_bf16((w.T, w.H_t), 1.0, (w.name, "pk_nh"), device)
    h_t.mul_(teacher_noise)
    h_t[:, :w.H_s] += h_s
    W_t = normal_bf16((w.V, w.H_t), teacher_noise * sd, (w.name, "pk_nW"), device)
    W_t[:, :w.H_s] += W_s
    return {"h_s": h_s, "h_t": h_t, "W_s": W_s, "W_t": W_t,
            "ids": uniform_ids(w.T, w.V, (w.name, "ids"), device)}


def logits_problem(w: Workload, device="cpu", T: int | None = None) -> dict:
    """Student logits ~N(0,2^2); teacher logits ~N(0,2^2) + per-row shift ~N(0,1)."""
    T = w.T if T is None else T
    shift = torch.randn((T,), generator=_torch_gen("cpu", (w.name, "shift")),
                        dtype=torch.float32)
    return {
        "z_s": normal_bf16((T, w.V), 2.0, (w.name, "z_s"), device),
        "z_t": normal_bf16((T, w.V), 2.0, (w.name, "z_t"), device, row_shift=shift),
        "ids": uniform_ids(T, w.V, (w.name, "ids"), device),
    }


def to_f64(t: torch.Tensor) -> np.ndarray:
    """Exact widening of a (bf16/fp32) tensor to a host float64 array."""
    return t.detach().to("cpu").to(torch.float64).numpy()


def sample_rows(w: Workload, k: int, computed_only: bool = True) -> np.ndarray:
    """Seeded sample of packed row indices for spot checks at sizes the oracle cannot
    sweep: always the first row, each rollout's last admitted row, the first
    non-admitted row and the last row, then uniform draws."""
    lens = np.diff(w.offsets)
    n = np.minimum(w.window.astype(np.int64), lens)
    must, pool = [], []
    for i in range(w.B):
        o, l, ni = int(w.offsets[i]), int(lens[i]), int(n[i])
        hi = l if (w.mode == MODE_PREFIX_AND_FULL or not computed_only) else ni
        if hi > 0:
            must += [o, o + hi - 1]
            if ni > 0:
                must.append(o + ni - 1)
            if ni < hi:
                must.append(o + ni)
            pool.append(np.arange(o, o + hi, dtype=np.int64))
    pool = np.concatenate(pool) if pool else np.zeros(0, np.int64)
    must = np.unique(np.asarray(must, dtype=np.int64))[:k]
    g = _rng(w.name, "sample", k)
    extra = g.choice(pool, size=min(len(pool), max(0, k - len(must))), replace=False)
    return np.unique(np.concatenate([must, extra]))[:k]
