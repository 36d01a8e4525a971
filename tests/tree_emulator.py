"""CPU emulation of the reduction trees the RMSNorm kernels document, operation by operation in
float32 (numpy), so that "the tree is fixed by the shape" is a checked fact: the GPU's output must
equal these bits, at every CU width.  Test infrastructure: shares no code with the HIP path and
is no oracle (the oracle is the plain definition in double).

Tree of a row's sum of squares:
  workgroup per row, T threads: thread t owns the 8-element chunks t, t+T, ... and adds the
    squares of its elements in ascending index order by fused multiply-add; the 64 lanes of a wave
    are combined by the butterfly with partner distances 32, 16, 8, 4, 2, 1; wave partials are
    added in wave order;
  wave per row (from 512 rows, rows of at most 4096 columns): lane l owns chunks l, l+64, ...;
    same in-lane order, same butterfly, no third stage.
Then rstd = 1 / sqrt(ss / cols + eps) and y = bf16(x * rstd * gamma), every operation rounded to
float32 once, the result to bf16 by round-to-nearest-even.
"""
import numpy as np

f32 = np.float32


def _bf16_to_f32(bits):
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def _f32_to_bf16(x):
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    return ((u + 0x7fff + ((u >> 16) & 1)) >> 16).astype(np.uint16)


def _fma(a, b, c):
    # a, b carry 8 significant bits (bf16): the product is exact in double, and so is the sum with a
    # float32 unless the exponents lie more than 29 binary orders apart; one rounding to float32
    return (a.astype(np.float64) * b.astype(np.float64) + c.astype(np.float64)).astype(np.float32)


def _butterfly(v):
    """v: [..., 64] float32 -> the value every lane ends with."""
    lanes = np.arange(64)
    for d in (32, 16, 8, 4, 2, 1):
        v = (v + v[..., lanes ^ d]).astype(np.float32)
    return v[..., 0]


def norm_threads(cols):
    chunks, t = cols // 8, 64
    while t < 256 and t < chunks:
        t *= 2
    while cols > 64 * t and t < 512:
        t *= 2
    return t


def rmsnorm_bits(x_bits, gamma_bits, eps, threads=None):
    """x_bits [rows, cols] uint16, gamma_bits [cols] uint16 -> uint16 bits the kernel must produce."""
    x = _bf16_to_f32(x_bits)
    g = _bf16_to_f32(gamma_bits)
    rows, cols = x.shape
    nch = cols // 8
    by_wave = threads is None and rows >= 512 and cols <= 4096
    T = 64 if by_wave else (threads or norm_threads(cols))
    per = 8 if not by_wave else (2 if cols <= 1024 else (4 if cols <= 2048 else 8))
    ss = np.zeros((rows, T), dtype=np.float32)          # one partial per thread
    for j in range(per):
        c = np.arange(T) + j * T
        live = c < nch
        idx = np.where(live, c, 0)
        for e in range(8):                               # elements of a chunk in ascending order
            v = x[:, idx * 8 + e]
            ss = np.where(live[None, :], _fma(v, v, ss), ss)
    waves = _butterfly(ss.reshape(rows, T // 64, 64))    # [rows, waves]
    tot = waves[:, 0]
    for w in range(1, T // 64):
        tot = (tot + waves[:, w]).astype(np.float32)
    mean = (tot / f32(cols)).astype(np.float32)
    rstd = (f32(1.0) / np.sqrt((mean + f32(eps)).astype(np.float32)).astype(np.float32)).astype(np.float32)
    y = ((x * rstd[:, None]).astype(np.float32) * g[None, :]).astype(np.float32)
    return _f32_to_bf16(y)
