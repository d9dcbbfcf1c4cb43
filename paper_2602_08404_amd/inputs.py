"""Seeded synthetic inputs for the TEAM MoE-layer hot path.

This module only *draws numbers*: Gaussian hidden states, Gaussian weights, the
row normalisation applied to hidden states before an MoE layer, rounding to
bfloat16 storage, and the activated-expert masks the workloads use.  It holds
none of the layer's arithmetic (no router, no top-k, no expert FFN, no combine)
so that both the HIP path and the CPU oracle can be fed from it without sharing
any code of the method.

Shapes follow the model the paper evaluates (Section "Experiments", setup: SDAR
30B-A3B with 128 experts, 8 experts per token, 48 layers, blocks of 32 tokens,
4 speculative branches); the paper's own benchmarks and weights are not used,
every tensor here is synthetic.

Reproducibility: every tensor is drawn from a counter-based Philox stream keyed
by ``(seed, tag, layer, sub)`` so any slice (one expert of one layer) can be
regenerated on its own, in any order, on any number of threads.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, replace
from typing import Dict, Optional

import numpy as np

# tensor tags of the Philox key
TAG_X_BASE, TAG_X_NOISE, TAG_W_ROUTER, TAG_W_GATE, TAG_W_UP, TAG_W_DOWN, TAG_MASK, TAG_PERM, TAG_CLASS, TAG_STATE, TAG_CONF = range(1, 12)

WEIGHT_STD = 0.02          # "weights ~ N(0, 0.02)" read as standard deviation 0.02
RMS_EPS = 1e-6


@dataclass(frozen=True)
class MoEShape:
    """Sizes of one MoE layer call. dtype is the storage type of x, weights and y."""
    name: str
    T: int          # tokens in the call
    H: int          # hidden size
    E: int          # number of experts
    k: int          # experts per token
    I: int          # expert SwiGLU intermediate size
    dtype: str      # "f32" | "bf16"
    renormalize: int = 1
    normed_x: bool = True

    @property
    def bytes_per_expert(self) -> int:
        return 3 * self.H * self.I * (4 if self.dtype == "f32" else 2)


# The five workload shapes (one entry per benchmark configuration).
CFG1 = MoEShape("cfg1_tiny_f32", T=8, H=256, E=16, k=2, I=128, dtype="f32", normed_x=False)
CFG2 = MoEShape("cfg2_30b_a3b_block32", T=32, H=2048, E=128, k=8, I=768, dtype="bf16")
CFG3 = MoEShape("cfg3_speculative_4x32", T=128, H=2048, E=128, k=8, I=768, dtype="bf16")
CFG4 = MoEShape("cfg4_stack48_block32", T=32, H=2048, E=128, k=8, I=768, dtype="bf16")
CFG5 = MoEShape("cfg5_fine_grained_256", T=256, H=2048, E=256, k=8, I=512, dtype="bf16")
CONFIGS = {c.name: c for c in (CFG1, CFG2, CFG3, CFG4, CFG5)}


def scaled(shape: MoEShape, **kw) -> MoEShape:
    """A copy of a shape with some sizes replaced (reduced test cases)."""
    return replace(shape, **kw)


# --------------------------------------------------------------------------- rng
def _stream(seed: int, tag: int, layer: int = 0, sub: int = 0) -> np.random.Generator:
    key = np.array([np.uint64(seed), (np.uint64(tag) << np.uint64(48)) | (np.uint64(layer) << np.uint64(24))
                    | np.uint64(sub)], dtype=np.uint64)
    return np.random.Generator(np.random.Philox(key=key))


def normal(seed: int, tag: int, layer: int, sub: int, n: int, std: float = 1.0) -> np.ndarray:
    """n fp32 draws of N(0, std^2) from stream (seed, tag, layer, sub)."""
    a = _stream(seed, tag, layer, sub).standard_normal(n, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


# --------------------------------------------------------------------------- bf16 storage
def bf16_round(a: np.ndarray) -> np.ndarray:
    """fp32 -> bfloat16 bit patterns (uint16), round to nearest even. Finite inputs only."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    r = (u + (np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1)))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_widen(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> the exactly equal fp32 values."""
    out = np.zeros(bits.shape, np.uint32)
    out.view(np.uint16).reshape(bits.shape + (2,))[..., 1] = bits      # little-endian: high half-word
    return out.view(np.float32)


def store(a: np.ndarray, dtype: str) -> np.ndarray:
    """Round fp32 draws to the storage dtype: float32 array for "f32", uint16 bit patterns for "bf16"."""
    return np.ascontiguousarray(a, dtype=np.float32) if dtype == "f32" else bf16_round(a)


def as_f32(stored: np.ndarray) -> np.ndarray:
    """Exact fp32 view of a stored tensor (what the CPU oracle consumes)."""
    return bf16_widen(stored) if stored.dtype == np.uint16 else np.asarray(stored, dtype=np.float32)


# --------------------------------------------------------------------------- 8-bit weight storage
def e4m3_values() -> np.ndarray:
    """The 256 fp32 values of the OCP 8-bit floating-point format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
    bits; exponent field 0 holds the subnormals m/8 * 2^-6; there are no infinities; 0x7f and 0xff are NaN; largest
    finite magnitude 448), indexed by the code."""
    code = np.arange(256)
    e, m = (code >> 3) & 15, code & 7
    mag = np.where(e == 0, m / 8.0 * 2.0 ** -6, (1.0 + m / 8.0) * 2.0 ** (e.astype(np.float64) - 7))
    mag = np.where((e == 15) & (m == 7), np.nan, mag)
    return np.where(code >= 128, -mag, mag).astype(np.float32)


def _e4m3_codes(v: np.ndarray) -> np.ndarray:
    """Finite fp32 values -> codes of the nearest E4M3 values (ties to the even code, magnitudes above 448 saturate)."""
    u = np.ascontiguousarray(v, dtype=np.float32).view(np.uint32)
    mag = u & np.uint32(0x7FFFFFFF)
    # normal range (>= 2^-6): keep 3 mantissa bits, round to nearest even on the 20 dropped bits -> exponent(8) | mantissa(3),
    # saturate at the code of 448, then re-bias the exponent from 127 to 7
    r = (mag + (np.uint32(0x7FFFF) + ((mag >> np.uint32(20)) & np.uint32(1)))) >> np.uint32(20)
    r = np.minimum(r, np.uint32(0x7E + ((127 - 7) << 3)))
    r -= np.uint32((127 - 7) << 3)                          # wraps for values below the normal range: replaced next
    # below 2^-6 the format has the fixed step 2^-9: the code is the number of steps (8 steps = 2^-6 = code 0x08, the first normal)
    small = mag < np.uint32(0x3C800000)                     # 0x3C800000 = 2^-6
    if small.any():
        r[small] = np.rint(mag.view(np.float32)[small] * np.float32(512.0)).astype(np.uint32)
    code = r.astype(np.uint8)
    code |= ((u >> np.uint32(24)) & np.uint32(0x80)).astype(np.uint8)
    return code


def _over_slices(fn, n: int) -> None:
    """fn(i) for i in range(n) on worker threads (NumPy releases the interpreter lock inside its loops)."""
    workers = min(16, os.cpu_count() or 1)
    if n > 1 and workers > 1:
        with ThreadPoolExecutor(workers) as ex:
            list(ex.map(fn, range(n)))
    else:
        for i in range(n):
            fn(i)


def quantize_rows_e4m3(w: np.ndarray):
    """fp32 matrix [..., R, C] -> (codes uint8 [..., R, C], scale fp32 [..., R]): every row is stored as E4M3 codes times one
    scale per row.  scale = max|row| / 448 rounded to 8 significant bits (so that code value x scale is exact in fp32; 1 for an
    all-zero row); code = E4M3 value nearest to w / scale (ties to the even code, magnitudes above 448 saturate)."""
    w = np.ascontiguousarray(w, dtype=np.float32)
    w3 = w.reshape((-1,) + w.shape[-2:])
    code = np.empty(w3.shape, np.uint8)
    scale = np.empty(w3.shape[:2], np.float32)

    def one(i):
        amax = np.abs(w3[i]).max(axis=-1)
        scale[i] = bf16_widen(bf16_round(np.where(amax > 0, amax / np.float32(448.0), np.float32(1.0)).astype(np.float32)))
        code[i] = _e4m3_codes(w3[i] / scale[i][:, None])

    _over_slices(one, w3.shape[0])
    return code.reshape(w.shape), scale.reshape(w.shape[:-1])


def dequantize_rows_e4m3(code: np.ndarray, scale: np.ndarray) -> np.ndarray:
    """The fp32 weights that (code, scale) stand for: value of the code times the row's scale (exact in fp32)."""
    code = np.ascontiguousarray(code)
    c3 = code.reshape((-1,) + code.shape[-2:])
    s2 = np.ascontiguousarray(scale, dtype=np.float32).reshape(c3.shape[:2])
    out = np.empty(c3.shape, np.float32)
    table = e4m3_values()

    def one(i):
        np.multiply(table[c3[i]], s2[i][:, None], out=out[i])

    _over_slices(one, c3.shape[0])
    return out.reshape(code.shape)


# --------------------------------------------------------------------------- hidden states
def rms_normalise(x: np.ndarray) -> np.ndarray:
    """Unit-gain RMS normalisation of each row, fp32 (the pre-MoE norm of the model; input recipe only)."""
    x = x.astype(np.float32)
    ms = np.mean(x.astype(np.float64) ** 2, axis=1, keepdims=True)
    return (x / np.sqrt(ms + RMS_EPS)).astype(np.float32)


def make_x(shape: MoEShape, seed: int = 0, layer: int = 0, step: int = 0, kind: str = "iid",
           noise_std: float = 0.0) -> np.ndarray:
    """Hidden states [T,H] in storage dtype.

    kind="iid":        rows ~ N(0,1) (RMS-normalised when shape.normed_x).
    kind="candidates": T = C*32 rows; a shared 32-row base ~N(0,1) plus per-candidate noise of std
                       ``noise_std`` (speculative branches whose hidden states are highly similar;
                       Section "Speculative Exploration for Hot Tokens").
    kind="structured": every row = one vector shared by the block (per layer) + per-row, per-step noise of std ``noise_std``:
                       masked positions of a block have highly similar hidden states (Section "Spatial Consistency"; two
                       rows have cosine similarity 1 / (1 + noise_std^2), 0.86 at 0.40).
    kind="drift":      base ~N(0,1) for the layer plus per-step noise of std ``noise_std`` (hidden states of
                       the same block at successive denoising steps; Section "Temporal Consistency").
    kind="branches":   T = 4*32 rows: a 32-row base branch and the three extra branches of Section "Aligned Token
                       Candidates in SEH" as they look where rows do not depend on each other yet (token embeddings):
                       branch 1 replaces the row of the first candidate position, branch 2 that of the second, branch 3
                       both (with the same two new rows); every other row repeats the base branch bit for bit.
                       34 distinct rows out of 128.
    """
    T, H = shape.T, shape.H
    if kind == "iid":
        x = normal(seed, TAG_X_BASE, layer, step, T * H).reshape(T, H)
    elif kind == "candidates":
        L = 32
        assert T % L == 0
        base = normal(seed, TAG_X_BASE, layer, 0, L * H).reshape(L, H)
        parts = [base + normal(seed, TAG_X_NOISE, layer, c, L * H, noise_std).reshape(L, H) for c in range(T // L)]
        x = np.concatenate(parts, axis=0)
    elif kind == "branches":
        L = 32
        assert T == 4 * L
        base = normal(seed, TAG_X_BASE, layer, 0, L * H).reshape(L, H)
        new_rows = normal(seed, TAG_X_NOISE, layer, step, 2 * H).reshape(2, H)
        p1, p2 = (int(v) for v in _stream(seed, TAG_X_NOISE, layer, 1000 + step).permutation(L)[:2])
        b1, b2, b3 = base.copy(), base.copy(), base.copy()
        b1[p1] = new_rows[0]
        b2[p2] = new_rows[1]
        b3[p1], b3[p2] = new_rows[0], new_rows[1]
        x = np.concatenate([base, b1, b2, b3], axis=0)
    elif kind == "structured":
        shared = normal(seed, TAG_X_BASE, layer, 0, H).reshape(1, H)
        x = shared + normal(seed, TAG_X_NOISE, layer, step, T * H, noise_std).reshape(T, H)
    elif kind == "drift":
        base = normal(seed, TAG_X_BASE, layer, 0, T * H).reshape(T, H)
        x = base + normal(seed, TAG_X_NOISE, layer, step, T * H, noise_std).reshape(T, H)
    else:
        raise ValueError(kind)
    if shape.normed_x:
        x = rms_normalise(x)
    return store(x, shape.dtype)


# --------------------------------------------------------------------------- weights
def _expert_matrix(seed: int, tag: int, layer: int, e: int, n: int, dtype: str) -> np.ndarray:
    return store(normal(seed, tag, layer, e + 1, n, WEIGHT_STD), dtype)


def make_router(shape: MoEShape, seed: int = 0, layer: int = 0) -> np.ndarray:
    return store(normal(seed, TAG_W_ROUTER, layer, 0, shape.E * shape.H, WEIGHT_STD), shape.dtype).reshape(shape.E, shape.H)


def make_expert(shape: MoEShape, e: int, seed: int = 0, layer: int = 0) -> Dict[str, np.ndarray]:
    """Weights of one expert: gate [I,H], up [I,H], down [H,I] (out-features major, reduction dim contiguous)."""
    H, I = shape.H, shape.I
    return {
        "gate": _expert_matrix(seed, TAG_W_GATE, layer, e, I * H, shape.dtype).reshape(I, H),
        "up": _expert_matrix(seed, TAG_W_UP, layer, e, I * H, shape.dtype).reshape(I, H),
        "down": _expert_matrix(seed, TAG_W_DOWN, layer, e, H * I, shape.dtype).reshape(H, I),
    }


def make_weights(shape: MoEShape, seed: int = 0, layer: int = 0, threads: Optional[int] = None) -> Dict[str, np.ndarray]:
    """All weights of one layer: router [E,H], gate/up [E,I,H], down [E,H,I] in storage dtype."""
    E, H, I = shape.E, shape.H, shape.I
    np_dt = np.float32 if shape.dtype == "f32" else np.uint16
    out = {"router": make_router(shape, seed, layer),
           "gate": np.empty((E, I, H), np_dt), "up": np.empty((E, I, H), np_dt), "down": np.empty((E, H, I), np_dt)}

    def fill(e):
        w = make_expert(shape, e, seed, layer)
        out["gate"][e], out["up"][e], out["down"][e] = w["gate"], w["up"], w["down"]

    threads = threads or min(16, os.cpu_count() or 1)
    if threads > 1 and E > 1:
        with ThreadPoolExecutor(threads) as ex:
            list(ex.map(fill, range(E)))
    else:
        for e in range(E):
            fill(e)
    return out


# --------------------------------------------------------------------------- activated-expert sets
def random_mask(E: int, M: int, seed: int = 0, layer: int = 0) -> np.ndarray:
    """Byte mask [E] with exactly M ones at seeded random positions."""
    perm = _stream(seed, TAG_MASK, layer, M).permutation(E)
    m = np.zeros(E, np.uint8)
    m[perm[:M]] = 1
    return m


def activated_set_by_summed_probability(logits: np.ndarray, M: int) -> np.ndarray:
    """Workload recipe for the activated-expert set of a call: the M experts with the largest router
    probability summed over all tokens of the call (ties to the lower id).  ``logits`` [T,E] are handed in by
    the caller (the oracle's in the tests); this is how the *input* mask is drawn, not a step of the layer."""
    z = logits.astype(np.float64)
    z = z - z.max(axis=1, keepdims=True)
    p = np.exp(z)
    p /= p.sum(axis=1, keepdims=True)
    score = p.sum(axis=0)
    order = np.lexsort((np.arange(score.size), -score))
    m = np.zeros(score.size, np.uint8)
    m[order[:M]] = 1
    return m


def token_permutation(T: int, seed: int = 0) -> np.ndarray:
    return _stream(seed, TAG_PERM, 0, T).permutation(T)


def token_classes(T: int, n_first: int, seed: int = 0, layer: int = 0) -> np.ndarray:
    """Byte vector [T] with exactly n_first ones at seeded random positions: the tokens of a denoising step that
    take part in the first routing round (newly accepted and hot tokens); the zeros are the cold tokens."""
    perm = _stream(seed, TAG_CLASS, layer, n_first).permutation(T)
    c = np.zeros(T, np.uint8)
    c[perm[:n_first]] = 1
    return c


def block_states(n_blocks: int, block_len: int, n_decoded: int, n_new: int, seed: int = 0) -> np.ndarray:
    """Byte vector [n_blocks*block_len]: per block a decoded prefix of about n_decoded positions (near-autoregressive
    acceptance: a contiguous prefix plus one or two stray positions further right), n_new of the decoded positions marked
    newly accepted (2), the rest decoded earlier (1), everything else masked (0)."""
    out = np.zeros(n_blocks * block_len, np.uint8)
    for b in range(n_blocks):
        r = _stream(seed, TAG_STATE, b, n_decoded)
        pre = max(0, min(block_len, n_decoded - 2 + int(r.integers(0, 3))))
        dec = set(range(pre))
        for _ in range(min(2, max(0, n_decoded - pre))):
            dec.add(int(r.integers(pre, block_len)))
        dec = sorted(dec)
        new = set(r.permutation(len(dec))[:min(n_new, len(dec))].tolist())
        for i, p in enumerate(dec):
            out[b * block_len + p] = 2 if i in new else 1
    return out


def confidences(n: int, seed: int = 0) -> np.ndarray:
    """fp32 [n] confidences in (0, 1), skewed towards small values the way re-masked attempts are."""
    u = _stream(seed, TAG_CONF, 0, n).random(n)
    return (u ** 2).astype(np.float32)
