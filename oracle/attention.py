"""CPU oracle of single-token decode attention over the particle caches (TEST INFRASTRUCTURE, not the product).

Not part of the paper's method: it is what a decoder computes with the cache that the reorder step of Alg. 1 /
App. C maintains, written out from the textbook definition (scaled dot-product attention with grouped query heads),
in fp64 with plain numpy.  Shares no code with the HIP library.

For row r, KV head h and each of the G = Hq / Hkv query heads g of its group:
    s_j = scale * <q[r, h*G+g, :], K[r, h, j, :]>,  j < len
    p   = softmax_j(s)
    out[r, h*G+g, :] = sum_j p_j V[r, h, j, :]
"""
import numpy as np


def bf16_bits_to_f64(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def decode_attention(q_bits, k_bits, v_bits, length, scale):
    """q_bits: uint16 [R, Hq, D] bf16 bit patterns; k_bits, v_bits: uint16 [R, Hkv, S, D]; returns float64 [R, Hq, D]."""
    q = bf16_bits_to_f64(q_bits)
    K = bf16_bits_to_f64(k_bits[:, :, :length, :])
    V = bf16_bits_to_f64(v_bits[:, :, :length, :])
    R, Hq, D = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    assert G * Hkv == Hq
    out = np.empty((R, Hq, D), np.float64)
    for r in range(R):
        for hq in range(Hq):
            h = hq // G
            s = scale * (K[r, h] @ q[r, hq])                     # [len]
            s = s - s.max()
            p = np.exp(s)
            p = p / p.sum()
            out[r, hq] = p @ V[r, h]
    return out
