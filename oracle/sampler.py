"""Log-softmax, Gumbel-max sampling and the recorded behaviour log-prob.

One decode step draws y_t ~ mu(. | x, y_<t) (Sec. 2.1 eq. 1) and records log mu(y_t | .) so the
trainer can form the truncated importance weight min(c, pi/mu) (Sec. 2.1, IS equation).  mu is
softmax(logits / T): the distribution actually sampled.

Sampling is Gumbel-max: argmax_i (z_i + g_i), g_i = -log(-log u_i), which is an exact draw from
softmax(z).  Because a float decides an integer here, the decision is specified in float32,
operation by operation, so that any implementation following the same order gets the same token:

  u_i  = (2 * (bits_i >> 9) + 1) * 2^-24          (exact in float32, strictly inside (0, 1))
  z_i  = logits_i * inv_T                         (one float32 multiply; inv_T = float32(1) / float32(T))
  g_i  = -LOG(-LOG(u_i))                          (LOG below; negations are exact)
  y_i  = z_i + g_i                                (one float32 add)
  tok  = lowest i attaining max_i y_i

LOG(x), x a positive normal float32, uses float32 multiplies and adds only (no fused multiply-add):
  e = exponent(x) - 127, m = mantissa(x) in [1, 2); if bits(m) > 0x3FB504F3: m = m * 0.5, e = e + 1
  f = m - 1
  p = C8; for j = 7..0: p = p * f + Cj            (each * and + rounded separately)
  f2 = f * f;  r = (f2 * f) * p;  r = r + (-0.5) * f2;  r = r + float(e) * LN2_LO;  r = r + f
  LOG = float(e) * LN2_HI + r
"""
import numpy as np

from .philox import sampler_bits

_C = [np.uint32(b).view(np.float32) for b in (
    0x3EAAAAAA, 0xBE7FFFFE, 0x3E4CCEAD, 0xBE2AADA5, 0x3E11E90D,
    0xBDFE7A63, 0x3DEF5141, 0xBDEB1ADE, 0x3D8EC753)]
_LN2_HI = np.uint32(0x3F317200).view(np.float32)
_LN2_LO = np.uint32(0x35BFBE8E).view(np.float32)
_F = np.float32


def log_f32(x: np.ndarray) -> np.ndarray:
    """The specified float32 logarithm (see module docstring); x positive normal float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    e = (bits >> np.uint32(23)).astype(np.int32) - 127
    mb = (bits & np.uint32(0x007FFFFF)) | np.uint32(0x3F800000)
    big = mb > np.uint32(0x3FB504F3)
    m = mb.view(np.float32)
    m = np.where(big, m * _F(0.5), m).astype(np.float32)
    e = e + big.astype(np.int32)
    f = m - _F(1.0)
    p = np.full_like(f, _C[8])
    for j in range(7, -1, -1):
        p = p * f
        p = p + _C[j]
    f2 = f * f
    r = (f2 * f) * p
    r = r + _F(-0.5) * f2
    ef = e.astype(np.float32)
    r = r + ef * _LN2_LO
    r = r + f
    return ef * _LN2_HI + r


def uniform_from_bits(bits: np.ndarray) -> np.ndarray:
    k = (np.asarray(bits, dtype=np.uint32) >> np.uint32(9)).astype(np.float32)
    return (k * _F(2.0) + _F(1.0)) * _F(2.0 ** -24)


def gumbel_from_bits(bits: np.ndarray) -> np.ndarray:
    return -log_f32(-log_f32(uniform_from_bits(bits)))


def log_softmax(z: np.ndarray) -> np.ndarray:
    """log softmax over the last axis, float64, max subtracted first."""
    z = np.asarray(z, dtype=np.float64)
    m = z.max(axis=-1, keepdims=True)
    return z - (m + np.log(np.exp(z - m).sum(axis=-1, keepdims=True)))


def sample_row(logits_f32: np.ndarray, temperature: float, seed: int, seq_id: int, position: int,
               forced: int = -1):
    """One row of the sampler: returns (token, logprob of that token under softmax(logits/T)).
    `forced` >= 0 replaces the drawn token (teacher forcing); its log-prob is still recorded."""
    logits_f32 = np.ascontiguousarray(logits_f32, dtype=np.float32)
    inv_t = _F(1.0) / _F(temperature)
    z = logits_f32 * inv_t
    if forced >= 0:
        tok = int(forced)
    else:
        g = gumbel_from_bits(sampler_bits(seed, seq_id, position, z.shape[0]))
        tok = int(np.argmax(z + g))          # numpy's argmax returns the lowest index on ties
    return tok, float(log_softmax(z)[tok])
