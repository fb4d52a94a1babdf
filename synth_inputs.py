"""Seeded synthetic inputs shared by the tests, the bench and the smoke check.

This module only makes numbers.  It holds none of the method's arithmetic (no
matrix product, no activation, no softmax, no gradient), so both the CPU oracle
and the HIP path can be fed from it without sharing any code of their own.

The generator is counter based: element `i` of tensor `t` under seed `s` is a
pure function of (s, t, i).  Any slice of any tensor can therefore be produced
on its own (a chunk of a 9,000,000-pattern epoch, one sampled row) and on any
device, and the integer part is bit-identical everywhere because it is done in
wrapping 64-bit integer arithmetic.

The inputs stand in for the paper's training data (20x20 grey-scale character
images, 3203 classes, about 9 million patterns; section 6.1), which is not
available: only the shapes are kept.  Values are X ~ N(0,1),
W ~ N(0, 1/fan_in) (variance), labels uniform, GEMM entries uniform[-1,1].
"""
from __future__ import annotations

import math
from dataclasses import dataclass

import torch

# tensor ids (the `t` of the counter)
T_X, T_W1, T_W2, T_B1, T_B2, T_LABELS, T_A, T_B, T_C, T_TARGETS = range(1, 11)

_MASK63 = 0x7FFFFFFFFFFFFFFF


def _i64(v: int) -> int:
    """Python int -> the int64 with the same low 64 bits."""
    v &= 0xFFFFFFFFFFFFFFFF
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLDEN = _i64(0x9E3779B97F4A7C15)
_M1 = _i64(0xBF58476D1CE4E5B9)
_M2 = _i64(0x94D049BB133111EB)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of int64 lanes."""
    return (x >> s) & (_MASK63 >> (s - 1))


def _mix(z: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 lanes (wrapping multiply)."""
    z = (z ^ _lsr(z, 30)) * _M1
    z = (z ^ _lsr(z, 27)) * _M2
    return z ^ _lsr(z, 31)


def _bits(seed: int, tensor_id: int, idx: torch.Tensor, stream: int) -> torch.Tensor:
    """64 hashed bits per counter value; `stream` separates the draws one element needs."""
    key = _i64((seed * 0xD1342543DE82EF95 + tensor_id * 0xA0761D6478BD642F + stream * 0xE7037ED1A0B428DB))
    return _mix(_mix(idx * _GOLDEN + key))


def _unit(bits: torch.Tensor) -> torch.Tensor:
    """Top 53 bits -> float64 in (0, 1)."""
    return (_lsr(bits, 11).to(torch.float64) + 0.5) * (1.0 / 9007199254740992.0)


def _index(start: int, count: int, device) -> torch.Tensor:
    return torch.arange(start, start + count, dtype=torch.int64, device=device)


_CHUNK = 1 << 24


def _chunks(start, count):
    done = 0
    while done < count:
        n = min(_CHUNK, count - done)
        yield start + done, done, n
        done += n


def uniform(seed: int, tensor_id: int, count: int, lo: float = -1.0, hi: float = 1.0, *, start: int = 0,
            device="cpu", dtype=torch.float32) -> torch.Tensor:
    """`count` values uniform in (lo, hi), elements start..start+count-1 of the tensor's stream."""
    out = torch.empty(count, dtype=dtype, device=device)
    for s, o, n in _chunks(start, count):
        u = _unit(_bits(seed, tensor_id, _index(s, n, device), 0))
        out[o:o + n] = (lo + (hi - lo) * u).to(dtype)
    return out


def normal(seed: int, tensor_id: int, count: int, std: float = 1.0, *, start: int = 0, device="cpu",
           dtype=torch.float32) -> torch.Tensor:
    """`count` values ~ N(0, std^2) by Box-Muller in float64, then rounded to `dtype`."""
    out = torch.empty(count, dtype=dtype, device=device)
    for s, o, n in _chunks(start, count):
        idx = _index(s, n, device)
        u1 = _unit(_bits(seed, tensor_id, idx, 0))
        u2 = _unit(_bits(seed, tensor_id, idx, 1))
        z = torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
        out[o:o + n] = (std * z).to(dtype)
    return out


def integers(seed: int, tensor_id: int, count: int, lo: int, hi: int, *, start: int = 0, device="cpu",
             dtype=torch.int32) -> torch.Tensor:
    """`count` integers uniform in [lo, hi)."""
    out = torch.empty(count, dtype=dtype, device=device)
    for s, o, n in _chunks(start, count):
        u = _unit(_bits(seed, tensor_id, _index(s, n, device), 0))
        v = torch.clamp((u * (hi - lo)).floor().to(torch.int64), max=hi - lo - 1) + lo
        out[o:o + n] = v.to(dtype)
    return out


# ---------------------------------------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------------------------------------

@dataclass(frozen=True)
class MlpShape:
    n_in: int
    n_hid: int
    n_out: int
    biases: bool = False


MLP_SMALL = MlpShape(64, 32, 10, biases=True)      # the small case: batch 256, seed 0
MLP_JOCR = MlpShape(400, 480, 3203, biases=False)  # the paper's 400-480-3203 network (section 6.1)


def mlp_weights(shape: MlpShape, seed: int, device="cpu"):
    """W1[n_in x n_hid] ~ N(0,1/n_in), W2[n_hid x n_out] ~ N(0,1/n_hid) (variances); biases zero or None."""
    W1 = normal(seed, T_W1, shape.n_in * shape.n_hid, 1.0 / math.sqrt(shape.n_in), device=device)
    W2 = normal(seed, T_W2, shape.n_hid * shape.n_out, 1.0 / math.sqrt(shape.n_hid), device=device)
    W1 = W1.reshape(shape.n_in, shape.n_hid)
    W2 = W2.reshape(shape.n_hid, shape.n_out)
    if shape.biases:
        b1 = torch.zeros(shape.n_hid, dtype=torch.float32, device=device)
        b2 = torch.zeros(shape.n_out, dtype=torch.float32, device=device)
    else:
        b1 = b2 = None
    return W1, W2, b1, b2


def mlp_patterns(shape: MlpShape, seed: int, first: int, count: int, device="cpu"):
    """Patterns first..first+count-1 of the seed's pattern stream: X[count x n_in] ~ N(0,1), labels[count]."""
    X = normal(seed, T_X, count * shape.n_in, 1.0, start=first * shape.n_in, device=device)
    labels = integers(seed, T_LABELS, count, 0, shape.n_out, start=first, device=device)
    return X.reshape(count, shape.n_in), labels


def mlp_targets(shape: MlpShape, seed: int, first: int, count: int, device="cpu"):
    """Dense target matrix T[count x n_out] for the squared-error form: +0.9 for the pattern's class, -0.9
    elsewhere (targets inside the range of tanh), plus uniform(-0.05, 0.05) noise so no two columns coincide."""
    _, labels = mlp_patterns(shape, seed, first, count, device=device)
    T = uniform(seed, T_TARGETS, count * shape.n_out, -0.05, 0.05, start=first * shape.n_out, device=device)
    T = T.reshape(count, shape.n_out) - 0.9
    T[torch.arange(count, device=device), labels.long()] += 1.8
    return T


def random_biases(shape: MlpShape, seed: int, std: float = 0.1, device="cpu"):
    """Non-zero biases for tests that must see the bias terms act."""
    return (normal(seed, T_B1, shape.n_hid, std, device=device),
            normal(seed, T_B2, shape.n_out, std, device=device))


def gemm_operands(seed: int, rows_a: int, cols_a: int, rows_b: int, cols_b: int, m: int, n: int,
                  lda: int | None = None, ldb: int | None = None, ldc: int | None = None, device="cpu"):
    """A, B, C with entries uniform[-1,1], stored row-major with the given leading dimensions.

    A is rows_a x cols_a as stored (before op()), B rows_b x cols_b, C m x n.  Padding columns
    (ld > cols) are filled from the same stream, so reading them by mistake changes results.
    """
    lda = lda or cols_a
    ldb = ldb or cols_b
    ldc = ldc or n
    A = uniform(seed, T_A, rows_a * lda, device=device).reshape(rows_a, lda)
    B = uniform(seed, T_B, rows_b * ldb, device=device).reshape(rows_b, ldb)
    C = uniform(seed, T_C, m * ldc, device=device).reshape(m, ldc)
    return A, B, C


def small_integers(seed: int, tensor_id: int, rows: int, cols: int, bound: int = 8, even: bool = False,
                   device="cpu") -> torch.Tensor:
    """Integer-valued fp32 matrix with entries in [-bound, bound]; `even` doubles them (exact halves)."""
    v = integers(seed, tensor_id, rows * cols, -bound, bound + 1, device=device, dtype=torch.int64)
    if even:
        v = v * 2
    return v.to(torch.float32).reshape(rows, cols)
