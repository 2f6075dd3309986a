"""Seeded synthetic inputs shaped like the paper's workloads.

This module only draws numbers: it holds none of the method's arithmetic (no rounding to a
format, no classification, no matrix product) and is the one piece shared by the CPU oracle's
tests and the GPU library's tests and benchmark.  Everything is generated on the host with
``numpy.random.default_rng`` in fp64 and cast once to fp32.

The distributions stand in for the tensors the paper monitors (activations, weights and
activation gradients of ResNet / BERT / LSTM / CVAE training, Sec. IV-B and Sec. V), whose
datasets are not available here: "log2|x| ~ D" means draw L ~ D, a random sign s, and set
x = s * 2^L, with exact zeros placed by an independent Bernoulli mask.
"""
from __future__ import annotations

import numpy as np

# The six format variants of the study: (e, m, denormals kept?)  (Sec. III-A, Table I; Sec. V-C)
FORMATS = {
    "1/5/10/d": (5, 10, True), "1/5/10/n": (5, 10, False),
    "1/6/9/d": (6, 9, True), "1/6/9/n": (6, 9, False),
    "1/8/7/d": (8, 7, True), "1/8/7/n": (8, 7, False),
}
DEFAULT_EXP_LO = -48


def _rng(*key) -> np.random.Generator:
    return np.random.default_rng([int(k) for k in key])


def _cast32(x: np.ndarray) -> np.ndarray:
    with np.errstate(over="ignore", under="ignore"):
        return x.astype(np.float32)


def log2_normal(n, mean: float, sigma: float, zero_frac: float, rng: np.random.Generator,
                chunk: int = 1 << 24) -> np.ndarray:
    """x = +-2^L with L ~ Normal(mean, sigma^2); a fraction zero_frac of exact +0."""
    shape = (n,) if np.isscalar(n) else tuple(n)
    total = int(np.prod(shape))
    out = np.empty(total, dtype=np.float32)
    for s in range(0, total, chunk):
        c = min(chunk, total - s)
        L = rng.normal(mean, sigma, c)
        sign = np.where(rng.random(c) < 0.5, -1.0, 1.0)
        v = sign * np.exp2(L)
        if zero_frac > 0:
            v[rng.random(c) < zero_frac] = 0.0
        out[s:s + c] = _cast32(v)
    return out.reshape(shape)


def _student_chunk(args):
    seed_key, idx, count, center, scale, dof, zero_frac = args
    rng = _rng(*seed_key, idx)
    L = center + scale * rng.standard_t(dof, count)
    sign = np.where(rng.random(count) < 0.5, -1.0, 1.0)
    with np.errstate(over="ignore", under="ignore"):
        v = sign * np.exp2(L)
    if zero_frac > 0:
        v[rng.random(count) < zero_frac] = 0.0
    return _cast32(v)


def log2_student_t(n: int, center: float, scale: float, dof: float, zero_frac: float,
                   seed_key=(5,), chunk: int = 1 << 22, workers: int = 0) -> np.ndarray:
    """x = +-2^L with L = center + scale*T, T ~ Student-t(dof); no clipping, so the fp32 cast
    produces a few infinities, fp32 denormals and extra zeros on purpose.  The tensor is drawn in
    chunks of 2^22, chunk i from its own generator seeded (seed_key, i), so the result does not
    depend on how many threads draw it."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    n = int(n)
    out = np.empty(n, dtype=np.float32)
    jobs = [(tuple(seed_key), i, min(chunk, n - s), center, scale, dof, zero_frac)
            for i, s in enumerate(range(0, n, chunk))]
    if workers <= 0:
        workers = min(16, os.cpu_count() or 1)
    with ThreadPoolExecutor(max_workers=workers) as pool:
        for i, part in enumerate(pool.map(_student_chunk, jobs)):
            out[i * chunk:i * chunk + part.size] = part
    return out


# --------------------------------------------------------------------------------------
# The five benchmark configurations
# --------------------------------------------------------------------------------------

def config1(seed: int = 0) -> dict:
    """2^20 values with log2|x| ~ N(-14, 6^2), 1 % zeros; 256^3 GEMM operands N(0,1)*2^-10."""
    rng = _rng(seed)
    x = log2_normal(1 << 20, -14.0, 6.0, 0.01, rng)
    A = _cast32(rng.standard_normal((256, 256)) * 2.0 ** -10)
    B = _cast32(rng.standard_normal((256, 256)) * 2.0 ** -10)
    return {"x": x, "A": A, "B": B}


MLP_SIZES = (784, 1024, 1024, 10)
MLP_BATCH = 256
LOSS_SCALE = 1024.0


def config2(seed: int = 2) -> dict:
    """3-layer MLP 784-1024-1024-10, batch 256: Kaiming-normal fp32 master weights [out, in],
    inputs U[0,1), integer labels."""
    rng = _rng(seed, 0)
    X = _cast32(rng.random((MLP_BATCH, MLP_SIZES[0])))
    W = []
    for l in range(3):
        fan_in, fan_out = MLP_SIZES[l], MLP_SIZES[l + 1]
        W.append(_cast32(rng.standard_normal((fan_out, fan_in)) * np.sqrt(2.0 / fan_in)))
    labels = rng.integers(0, MLP_SIZES[-1], MLP_BATCH)
    return {"X": X, "W": W, "labels": labels, "loss_scale": LOSS_SCALE}


CONV_SHAPE = dict(batch=64, cin=256, cout=256, h=14, w=14, k=3)   # GEMM M=12544 N=256 K=2304


def config3(seed: int = 3, batch: int = CONV_SHAPE["batch"]) -> dict:
    """3x3 conv 256->256 at 14x14 as an im2col GEMM.  X = relu(N(0,1)) in NCHW, W ~ N(0, 2/2304)
    as [cout, cin*9], dY with log2|g| ~ N(-20, 5^2) as [batch*196, cout]."""
    s = CONV_SHAPE
    rng = _rng(seed, 0)
    X = _cast32(np.maximum(rng.standard_normal((batch, s["cin"], s["h"], s["w"])), 0.0))
    K = s["cin"] * s["k"] * s["k"]
    W = _cast32(rng.standard_normal((s["cout"], K)) * np.sqrt(2.0 / K))
    dY = log2_normal((batch * s["h"] * s["w"], s["cout"]), -20.0, 5.0, 0.0, rng)
    return {"X": X, "W": W, "dY": dY}


def im2col_3x3(X: np.ndarray) -> np.ndarray:
    """[N, C, H, W] -> [N*H*W, C*9] patches of a 3x3, pad 1, stride 1 convolution (pure data
    movement; column order c*9 + ky*3 + kx, matching torch.nn.functional.unfold)."""
    n, c, h, w = X.shape
    P = np.zeros((n, c, h + 2, w + 2), dtype=X.dtype)
    P[:, :, 1:-1, 1:-1] = X
    cols = np.empty((n, h, w, c, 3, 3), dtype=X.dtype)
    for ky in range(3):
        for kx in range(3):
            cols[:, :, :, :, ky, kx] = P[:, :, ky:ky + h, kx:kx + w].transpose(0, 2, 3, 1)
    return cols.reshape(n * h * w, c * 9)


BERT_TOKENS = 4096
BERT_LAYERS = (("qkv", 1024, 3072), ("attn_out", 1024, 1024), ("ffn1", 1024, 4096), ("ffn2", 4096, 1024))


def config4(seed: int = 4, tokens: int = BERT_TOKENS) -> dict:
    """BERT-Large-shaped encoder-layer GEMMs: weights N(0, 0.02^2) [out, in], activations N(0,1)
    [tokens, in], output gradients log2|g| ~ N(-24, 6^2) [tokens, out]."""
    layers = []
    for idx, (name, fin, fout) in enumerate(BERT_LAYERS):
        rng = _rng(seed, idx)
        layers.append({
            "name": name,
            "X": _cast32(rng.standard_normal((tokens, fin))),
            "W": _cast32(rng.standard_normal((fout, fin)) * 0.02),
            "dY": log2_normal((tokens, fout), -24.0, 6.0, 0.0, rng),
        })
    return {"layers": layers}


def config5(seed: int = 5, n: int = 1 << 28) -> np.ndarray:
    """Heavy-tailed gradient tensor: log2|x| = -18 + 8*T, T ~ Student-t(3), 2 % zeros."""
    return log2_student_t(n, -18.0, 8.0, 3.0, 0.02, seed_key=(seed,))


def special_values() -> np.ndarray:
    """fp32 inputs every kernel must treat exactly: signed zeros, infinities, NaNs with
    payloads, fp32 denormals, extreme normals."""
    bits = np.array([
        0x00000000, 0x80000000, 0x7F800000, 0xFF800000, 0x7FC00000, 0xFFC00000, 0x7F800001,
        0xFFFFFFFF, 0x7FA00000, 0x00000001, 0x80000001, 0x007FFFFF, 0x807FFFFF, 0x00400000,
        0x00800000, 0x80800000, 0x7F7FFFFF, 0xFF7FFFFF, 0x3F800000, 0xBF800000, 0x00008000,
        0x00010000, 0x00018000, 0x00008001, 0x007F8000, 0x007F0000, 0x7F7F8000, 0x7F7F7FFF,
    ], dtype=np.uint32)
    return bits.view(np.float32)


def random_bits(n: int, seed: int) -> np.ndarray:
    """Uniformly random fp32 bit patterns (all exponents, NaNs and denormals included)."""
    return _rng(seed, 99).integers(0, 1 << 32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
