"""Storage-format encoders used only by the synthetic input generators.

These turn float32 draws into the raw bytes the batch is stored in (bf16 bit
patterns, OCP fp8 E4M3FN codes with per-page scales).  Nothing here is attention
arithmetic; decoding the bytes back to numbers is done separately, and
independently, by each consumer of the batch.
"""
import numpy as np

BF16_NAN = np.uint16(0x7FC0)
FP8_NAN = np.uint8(0x7F)
FP8_MAX = 448.0


def f32_to_bf16_bits(x):
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.array(x, dtype=np.float32, order="C", copy=True).view(np.uint32)
    bias = u >> np.uint32(16)
    bias &= np.uint32(1)
    bias += np.uint32(0x7FFF)
    u += bias
    u >>= np.uint32(16)
    return u.astype(np.uint16)


def bf16_bits_to_f32(b):
    """Exact widening of bfloat16 bit patterns to float32 (generator-side helper)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f32_to_e4m3fn(x):
    """Encode float32 as OCP FP8 E4M3FN (bias 7, max 448, no inf), nearest-even, saturating.

    Finite inputs only (the generators never produce NaN for valid tokens).
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    sign = ((bits >> np.uint32(24)) & np.uint32(0x80)).astype(np.uint8)
    a = np.minimum(np.abs(x), np.float32(FP8_MAX))
    # normal binades: round the float32 significand to 3 fraction bits, ties to even
    u = a.view(np.uint32).copy()
    lsb = (u >> np.uint32(20)) & np.uint32(1)
    u += np.uint32(0x7FFFF)
    u += lsb
    u &= np.uint32(0xFFF00000)
    expo = (u >> np.uint32(23)).astype(np.int32) - 127 + 7          # biased e4m3 exponent
    code_n = ((expo << 3) | ((u >> np.uint32(20)) & np.uint32(7)).astype(np.int32))
    # subnormal binade (|x| < 2^-6): multiples of 2^-9, ties to even via the add-magic-constant trick
    magic = np.float32(2.0 ** 14)                                      # ulp(2^14) = 2^-9 in float32
    sub = ((a + magic) - magic) * np.float32(512.0)                   # 0..8 (8 = smallest normal, code 0x08)
    code_s = sub.astype(np.int32)
    code = np.where(a < np.float32(2.0 ** -6), code_s, code_n)
    return (code.astype(np.uint8) | sign).astype(np.uint8)


def quantize_per_page_head(x, head_axis_size):
    """Quantise a float32 pool x[pages, Hkv, ...] to e4m3 with one float32 scale per (page, head).

    scale = amax/448 (1 if the page is all zero); returns (codes uint8 same shape, scale[pages,Hkv] f32).
    """
    pages = x.shape[0]
    assert x.shape[1] == head_axis_size
    flat = x.reshape(pages, head_axis_size, -1)
    amax = np.max(np.abs(flat), axis=2)
    scale = np.where(amax > 0, amax / np.float32(FP8_MAX), np.float32(1.0)).astype(np.float32)
    codes = f32_to_e4m3fn(flat / scale[:, :, None]).reshape(x.shape)
    return codes, scale
