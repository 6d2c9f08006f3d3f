"""Seeded synthetic stand-ins for the paper's datasets (Table II shapes).

Nothing here is real ISOLET / MNIST / UCIHAR / CHB-MIT data: every matrix is drawn
from ``numpy.random.default_rng`` with a key derived from ``(seed, config, stream,
chunk)``, so any row range of any config can be regenerated without producing the
rows before it.  Rows come in fixed blocks of ``CHUNK`` rows; row ``r`` of a split
always lives in block ``r // CHUNK`` at offset ``r % CHUNK``.

Only inputs are produced: features, labels, the item (ID) table, the level (value)
table, the tie-break vector and the per-feature quantiser range ``lo`` / ``scale``.
The hypervector tables are handed over bit-packed, LSB first: dimension ``d`` is bit
``d & 31`` of 32-bit word ``d >> 5`` and the pad bits of the last word are zero.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional, Tuple

import numpy as np

CHUNK = 65536  # rows per independently seeded block

# name, D, F, L, C, feature dtype, n_train, n_test, mode, epochs, lr
CONFIGS = {
    1: dict(name="tiny-classical", D=1024, F=100, L=16, C=5, dtype="f32",
            n_train=2000, n_test=500, mode="classical", epochs=1, lr=1.0),
    2: dict(name="isolet-shape-classical", D=10000, F=617, L=64, C=26, dtype="f32",
            n_train=6238, n_test=1559, mode="classical", epochs=1, lr=1.0),
    3: dict(name="mnist-shape-classical", D=10000, F=784, L=256, C=10, dtype="u8",
            n_train=60000, n_test=10000, mode="classical", epochs=1, lr=1.0),
    4: dict(name="ucihar-shape-online", D=10000, F=561, L=100, C=6, dtype="f32",
            n_train=7352, n_test=2947, mode="online", epochs=3, lr=1.0),
    5: dict(name="chbmit-shape-classical", D=10000, F=342, L=64, C=2, dtype="f32",
            n_train=5_000_000, n_test=5_000_000, mode="classical", epochs=1, lr=1.0),
    # not one of the five benchmark configurations: the fourth small dataset of Table II
    # (31 features, 5 classes, about 80k samples), the small-F end of the evaluation
    6: dict(name="pamap-shape-classical", D=10000, F=31, L=64, C=5, dtype="f32",
            n_train=64000, n_test=16000, mode="classical", epochs=1, lr=1.0),
}


def pack_bits_lsb(bits: np.ndarray) -> np.ndarray:
    """{0,1} bytes ``[..., D]`` -> little-endian u32 words ``[..., ceil(D/32)]``, pad 0."""
    bits = np.ascontiguousarray(bits, dtype=np.uint8)
    D = bits.shape[-1]
    W = (D + 31) // 32
    padded = np.zeros(bits.shape[:-1] + (W * 32,), dtype=np.uint8)
    padded[..., :D] = bits
    by = np.packbits(padded, axis=-1, bitorder="little")
    return np.ascontiguousarray(by).view("<u4").reshape(bits.shape[:-1] + (W,))


def _rng(seed: int, cfg: int, stream: int, chunk: int = 0) -> np.random.Generator:
    return np.random.default_rng([int(seed), int(cfg), int(stream), int(chunk)])


def _level_bits(rng: np.random.Generator, D: int, L: int) -> np.ndarray:
    """Linear-scaling level table: level 0 random, each next level flips
    ``D // (2 (L-1))`` positions never flipped before (consecutive slices of one
    random permutation of the dimensions)."""
    b = D // (2 * (L - 1)) if L > 1 else 0
    lv = np.empty((L, D), dtype=np.uint8)
    lv[0] = rng.integers(0, 2, size=D, dtype=np.uint8)
    perm = rng.permutation(D)
    for k in range(1, L):
        lv[k] = lv[k - 1]
        lv[k, perm[(k - 1) * b:k * b]] ^= 1
    return lv


def _blob_masks(rng: np.random.Generator, C: int, side: int, cover: float) -> np.ndarray:
    """One fixed blob-shaped pixel mask per class covering ``cover`` of the grid."""
    masks = np.zeros((C, side * side), dtype=bool)
    for c in range(C):
        g = rng.standard_normal((side, side))
        for _ in range(3):  # cheap 3x3 box blur, three passes
            p = np.pad(g, 1, mode="edge")
            g = sum(p[i:i + side, j:j + side] for i in range(3) for j in range(3)) / 9.0
        thr = np.quantile(g, 1.0 - cover)
        masks[c] = (g > thr).ravel()
    return masks


@dataclass
class Workload:
    cfg: int
    seed: int
    name: str
    D: int
    F: int
    L: int
    C: int
    dtype: str            # "f32" or "u8"
    n_train: int
    n_test: int
    mode: str             # "classical" or "online"
    epochs: int
    lr: float
    item: np.ndarray      # u32 [F][W]
    level: np.ndarray     # u32 [L][W]
    tie: np.ndarray       # u32 [W]
    lo: Optional[np.ndarray]     # f32 [F] (None for u8 features)
    scale: Optional[np.ndarray]  # f32 [F] = float32(L / (hi - lo))
    params: dict = field(default_factory=dict, repr=False)

    @property
    def W(self) -> int:
        return (self.D + 31) // 32

    # ------------------------------------------------------------------ rows
    def _block(self, split: int, chunk: int, upto: int = CHUNK) -> Tuple[np.ndarray, np.ndarray]:
        """First ``upto`` rows of block ``chunk``.  Labels, feature noise and (config 3)
        pixel values each have a generator of their own, and every draw fills rows in
        order, so a shorter prefix is bit-identical to the start of a longer one."""
        r_lab = _rng(self.seed, self.cfg, 10 + split, 3 * chunk)
        r_x = _rng(self.seed, self.cfg, 10 + split, 3 * chunk + 1)
        r_v = _rng(self.seed, self.cfg, 10 + split, 3 * chunk + 2)
        p = self.params
        n = upto
        if self.cfg == 5:
            y = np.zeros(CHUNK, dtype=np.int32)
            n_runs = max(1, int(round(CHUNK * 0.01 / 90.0)))
            starts = r_lab.integers(0, CHUNK - 120, size=n_runs)
            lens = r_lab.integers(60, 121, size=n_runs)
            for s, ln in zip(starts, lens):
                y[s:s + ln] = 1
            y = y[:n]
            mu = np.repeat(p["mu_ch"], 19)[None, :] + 0.5 * y[:, None]
            x = np.exp(mu + 0.5 * r_x.standard_normal((n, self.F))).astype(np.float32)
            return x, y
        y = r_lab.integers(0, self.C, size=CHUNK).astype(np.int32)[:n]
        if self.cfg == 3:
            on = p["masks"][y]                                   # [n][F] bool
            keep = r_x.random((n, self.F)) < np.where(on, 0.9, 0.01)
            val = r_v.integers(64, 256, size=(n, self.F))
            x = np.where(keep, val, 0).astype(np.uint8)
            return x, y
        x = p["means"][y] + p["sigma"] * r_x.standard_normal((n, self.F))
        x = np.clip(x, p["clip"][0], p["clip"][1]).astype(np.float32)
        return x, y

    def rows(self, split: str, start: int, count: int) -> Tuple[np.ndarray, np.ndarray]:
        """Rows ``[start, start+count)`` of ``split`` ("train" or "test").
        Config 5 searches the windows it trained on: both splits are the same rows."""
        total = self.n_train if split == "train" else self.n_test
        if start < 0 or count < 0 or start + count > total:
            raise ValueError("row range outside the split")
        s = 0 if (split == "train" or self.cfg == 5) else 1
        xs, ys = [], []
        r = start
        while r < start + count:
            ch, off = divmod(r, CHUNK)
            take = min(CHUNK - off, start + count - r)
            x, y = self._block(s, ch, off + take)
            xs.append(x[off:off + take])
            ys.append(y[off:off + take])
            r += take
        if not xs:
            dt = np.float32 if self.dtype == "f32" else np.uint8
            return np.zeros((0, self.F), dtype=dt), np.zeros(0, dtype=np.int32)
        return np.ascontiguousarray(np.concatenate(xs)), np.ascontiguousarray(np.concatenate(ys))

    def train(self, count: Optional[int] = None, start: int = 0):
        return self.rows("train", start, self.n_train - start if count is None else count)

    def test(self, count: Optional[int] = None, start: int = 0):
        return self.rows("test", start, self.n_test - start if count is None else count)


def make_workload(cfg: int, seed: int = 0, **override) -> Workload:
    """Tables and class parameters of config ``cfg`` (1..6); rows are drawn lazily.

    Draw order: item table, level-0 vector, flip permutation, tie vector (stream 0);
    then the class parameters (stream 1); labels and features come per block.
    ``override`` may replace D, F, L, C, n_train, n_test for scaled-down test cases."""
    c = dict(CONFIGS[cfg])
    c.update(override)
    D, F, L, C = c["D"], c["F"], c["L"], c["C"]
    rt = _rng(seed, cfg, 0)
    item = pack_bits_lsb(rt.integers(0, 2, size=(F, D), dtype=np.uint8))
    level = pack_bits_lsb(_level_bits(rt, D, L))
    tie = pack_bits_lsb(rt.integers(0, 2, size=D, dtype=np.uint8))

    rp = _rng(seed, cfg, 1)
    params: dict = {}
    lo = hi = None
    if cfg == 1:
        params = dict(means=rp.uniform(0.2, 0.8, size=(C, F)), sigma=0.1, clip=(0.0, 1.0))
        lo, hi = np.zeros(F), np.ones(F)
    elif cfg in (2, 4, 6):
        params = dict(means=rp.uniform(-0.5, 0.5, size=(C, F)), sigma=0.25, clip=(-1.0, 1.0))
        lo, hi = -np.ones(F), np.ones(F)
    elif cfg == 3:
        side = int(round(F ** 0.5))
        if side * side != F:
            raise ValueError("config 3 needs a square feature grid")
        params = dict(masks=_blob_masks(rp, C, side, 0.20))
    elif cfg == 5:
        if F % 19 != 0:
            raise ValueError("config 5 needs F = channels x 19")
        mu_ch = rp.uniform(-0.5, 0.5, size=F // 19)
        params = dict(mu_ch=mu_ch)
        lo = np.zeros(F)
        # fixed upper edge: the 99.9th percentile of the negative-class lognormal
        hi = np.repeat(np.exp(mu_ch + 3.0902 * 0.5), 19)
    else:
        raise ValueError("config must be 1..6")
    lo32 = scale32 = None
    if c["dtype"] == "f32":
        lo32 = lo.astype(np.float32)
        scale32 = (L / (hi - lo)).astype(np.float32)
    return Workload(cfg=cfg, seed=seed, name=c["name"], D=D, F=F, L=L, C=C, dtype=c["dtype"],
                    n_train=c["n_train"], n_test=c["n_test"], mode=c["mode"],
                    epochs=c["epochs"], lr=c["lr"], item=item, level=level, tie=tie,
                    lo=lo32, scale=scale32, params=params)
