// Device-side number formats, counter-based random fields and rounding for the ELMO head.
//
// Everything here is written for gfx950 only.  The rules implemented are the paper's:
//   * formats: Section 3 "Floating-point formats" (BF16; FP8 E4M3 as used in Algorithm 1,
//     i.e. the OCP flavour: bias 7, largest finite 448, no infinities);
//   * stochastic rounding: Section 3, Eq. (1);
//   * the FP32 update arithmetic and Kahan compensation: Algorithm 1 (fuse_update) and the
//     three-line recurrence of Section 3.
// Where the paper is silent the choices are: Philox4x32-10 as the counter-based generator, one
// 16-bit field per weight element, add-and-truncate on the magnitude, clipping of finite
// overflow to the largest finite value, sign kept when a value rounds to zero.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elmo {

enum : int { FMT_BF16 = 0, FMT_E4M3 = 1 };

// ---------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11).  ctr = (c0..c3), key = (k0, k1).
// ---------------------------------------------------------------------------------------------
struct U4 { uint32_t x, y, z, w; };

// a ^ b ^ c: one v_bitop3_b32 on the device (the compiler otherwise emits two 2-input XORs)
__host__ __device__ inline uint32_t xor3(uint32_t a, uint32_t b, uint32_t c) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
#else
  return a ^ b ^ c;
#endif
}

__host__ __device__ inline U4 philox4x32_10(U4 c, uint32_t k0, uint32_t k1) {
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint64_t p0 = (uint64_t)0xD2511F53u * c.x;
    const uint64_t p1 = (uint64_t)0xCD9E8D57u * c.z;
    U4 n;
    n.x = xor3((uint32_t)(p1 >> 32), c.y, k0);
    n.y = (uint32_t)p1;
    n.z = xor3((uint32_t)(p0 >> 32), c.w, k1);
    n.w = (uint32_t)p0;
    c = n;
    k0 += 0x9E3779B9u;
    k1 += 0xBB67AE85u;
  }
  return c;
}

// The eight 16-bit rounding fields of the block of elements [8*blk, 8*blk+8).
// Field f (element 8*blk+f) is bits [16*(f&1), 16*(f&1)+16) of word f>>1.
__host__ __device__ inline U4 sr_block(uint64_t blk, uint64_t seed, uint64_t step) {
  U4 c;
  c.x = (uint32_t)blk;
  c.y = (uint32_t)(blk >> 32);
  c.z = (uint32_t)step;
  c.w = (uint32_t)(step >> 32);
  return philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
}

__host__ __device__ inline uint32_t sr_field(const U4& b, int f) {
  const uint32_t w = (f >> 1) == 0 ? b.x : (f >> 1) == 1 ? b.y : (f >> 1) == 2 ? b.z : b.w;
  return (f & 1) ? (w >> 16) : (w & 0xFFFFu);
}

// ---------------------------------------------------------------------------------------------
// Classifier dropout (appendix "Low-Memory Dropout for Classifier"): the keep mask is a pure
// function of (seed, step, element), so every kernel that touches a weight tile regenerates it
// and no masked copy of W exists.  One Philox block per 16 consecutive elements, one byte each:
// counter = (block, step | 2^63) -- the top bit separates this stream from the rounding fields,
// whose steps stay below 2^63 -- and element e is kept iff byte e % 16 of the block is >= thresh
// (byte b = bits [8 (b % 4), +8) of word b / 4), i.e. dropped with probability thresh / 256.
// ---------------------------------------------------------------------------------------------
struct DropArgs {
  uint32_t thresh;      // 1..255 (kernels built without dropout ignore the struct)
  float scale;          // 256 / (256 - thresh), applied to FP32 results, never to stored weights
};

__host__ __device__ inline U4 drop_block(uint64_t blk, uint64_t seed, uint64_t step) {
  U4 c;
  c.x = (uint32_t)blk;
  c.y = (uint32_t)(blk >> 32);
  c.z = (uint32_t)step;
  c.w = (uint32_t)(step >> 32) | 0x80000000u;
  return philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
}

// 0xFF in every byte of r that is >= thresh (unsigned), 0x00 elsewhere.  tb = thresh * 0x01010101.
// The low seven bits are compared by a borrow-free subtraction per byte, the top bits decide first.
__host__ __device__ inline uint32_t keep_bytes(uint32_t r, uint32_t tb) {
  const uint32_t s = ((r & 0x7F7F7F7Fu) | 0x80808080u) - (tb & 0x7F7F7F7Fu);   // bit 7: low bits of r >= low bits of thresh
  const uint32_t ge = ((r & ~tb) | (~(r ^ tb) & s)) & 0x80808080u;
  return ge | (ge - (ge >> 7));
}

// ---------------------------------------------------------------------------------------------
// Bit casts and decoding
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t f2u(float f) { return __float_as_uint(f); }
__device__ inline float u2f(uint32_t u) { return __uint_as_float(u); }

__device__ inline float bf16_decode(uint32_t bits16) { return u2f(bits16 << 16); }

// E4M3 (OCP) byte -> FP32, exact.  gfx950's conversion instruction implements the OCP format.
__device__ inline float e4m3_decode(uint32_t code) {
  return __builtin_amdgcn_cvt_f32_fp8((int)code, 0);
}

// ---------------------------------------------------------------------------------------------
// FP32 -> BF16.  ADD = 0x7FFF + lsb gives round-to-nearest-even; ADD = r (16-bit field) gives
// Eq. (1): the 16 dropped bits carry into the kept ones with probability dropped / 2^16.
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t bf16_finish(uint32_t bits, uint32_t mag, uint32_t q) {
  q = q > 0x7F7Fu ? 0x7F7Fu : q;                 // finite overflow (and inf) clips
  q = mag > 0x7F800000u ? 0x7FC0u : q;           // NaN stays NaN
  return ((bits >> 16) & 0x8000u) | q;
}
__device__ inline uint32_t bf16_rne(float t) {
  const uint32_t bits = f2u(t), mag = bits & 0x7FFFFFFFu;
  const uint32_t q = (mag + 0x7FFFu + ((mag >> 16) & 1u)) >> 16;
  return bf16_finish(bits, mag, q);
}
__device__ inline uint32_t bf16_sr(float t, uint32_t r16) {
  const uint32_t bits = f2u(t), mag = bits & 0x7FFFFFFFu;
  return bf16_finish(bits, mag, (mag + r16) >> 16);
}

// ---------------------------------------------------------------------------------------------
// FP32 -> E4M3.  From 2^-6 upwards 20 bits of the FP32 magnitude are dropped; below, the grid is
// uniform with spacing 2^-9 and |t| * 2^9 is rounded as a fixed-point number.
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t e4m3_finish(uint32_t bits, uint32_t mag, uint32_t code) {
  code = code > 0x7Eu ? 0x7Eu : code;            // clip to 448
  code = mag > 0x7F800000u ? 0x7Fu : code;       // NaN
  return ((bits >> 24) & 0x80u) | code;
}
__device__ inline uint32_t e4m3_rne(float t) {
  const uint32_t bits = f2u(t), mag = bits & 0x7FFFFFFFu;
  uint32_t code;
  if (mag >= 0x3C800000u) {                      // |t| >= 2^-6
    code = ((mag + 0x7FFFFu + ((mag >> 20) & 1u)) >> 20) - 960u;
  } else {
    code = (uint32_t)__builtin_rintf(u2f(mag) * 512.0f);   // ties to even; 8 = first normal code
  }
  return e4m3_finish(bits, mag, code);
}
// Stochastic rounding to E4M3 on gfx950's conversion unit.  v_cvt_sr_fp8_f32 adds the top bits of
// its 32-bit random operand to the dropped bits of the magnitude and truncates; with the 16-bit
// field in the upper half of that operand this is the add-and-truncate rule above (the 16 most
// significant dropped bits decide), in the subnormal range too.  The instruction turns finite
// overflow into NaN, so the clipping to +-448 is done first; NaN is passed through unclipped.
// `old`/`byte` select the destination byte of a packed result (the other bytes are kept).
__device__ inline uint32_t e4m3_sr_pack(float t, uint32_t rand_hi16, uint32_t old, int byte) {
  float tc = __builtin_amdgcn_fmed3f(t, -448.0f, 448.0f);
  tc = (t != t) ? t : tc;
  switch (byte) {
    case 0: return (uint32_t)__builtin_amdgcn_cvt_sr_fp8_f32(tc, rand_hi16, (int)old, 0);
    case 1: return (uint32_t)__builtin_amdgcn_cvt_sr_fp8_f32(tc, rand_hi16, (int)old, 1);
    case 2: return (uint32_t)__builtin_amdgcn_cvt_sr_fp8_f32(tc, rand_hi16, (int)old, 2);
    default: return (uint32_t)__builtin_amdgcn_cvt_sr_fp8_f32(tc, rand_hi16, (int)old, 3);
  }
}
// (for a NaN input the instruction returns a NaN code whose sign bit need not be the input's)
__device__ inline uint32_t e4m3_sr(float t, uint32_t r16) {
  const uint32_t q = e4m3_sr_pack(t, r16 << 16, 0u, 0) & 0xFFu;
  return (t != t) ? (((f2u(t) >> 24) & 0x80u) | 0x7Fu) : q;
}

__device__ inline float e4m3_decode_byte(uint32_t packed, int byte) {
  switch (byte) {
    case 0: return __builtin_amdgcn_cvt_f32_fp8((int)packed, 0);
    case 1: return __builtin_amdgcn_cvt_f32_fp8((int)packed, 1);
    case 2: return __builtin_amdgcn_cvt_f32_fp8((int)packed, 2);
    default: return __builtin_amdgcn_cvt_f32_fp8((int)packed, 3);
  }
}

// ---------------------------------------------------------------------------------------------
// FP32 -> a simulated format with E exponent and M mantissa bits, result as FP32 (the bit-width
// study of Section 4.3).  IEEE pattern: bias 2^(E-1)-1, top exponent code reserved, gradual
// underflow; overflow and infinities clip to the largest finite value, NaN passes through.
// 2 <= E <= 8, 1 <= M <= 22.  r16 < 0: round to nearest even; otherwise the 16-bit field of Eq. (1).
// ---------------------------------------------------------------------------------------------
__device__ inline float round_em(float t, int E, int M, int r16) {
  const uint32_t bits = f2u(t), mag = bits & 0x7FFFFFFFu;
  if (mag > 0x7F800000u) return t;
  const int emax = (1 << (E - 1)) - 1, emin = 2 - (1 << (E - 1));
  const uint32_t top = ((uint32_t)(emax + 127) << 23) | (((1u << M) - 1u) << (23 - M));   // (2 - 2^-M) 2^emax
  const int drop = 23 - M;
  uint32_t q;
  if (E == 8 || mag >= ((uint32_t)(emin + 127) << 23)) {
    // normal range of the format (for E = 8 also FP32's own subnormals, whose encoding is linear)
    const uint32_t frac = mag & ((1u << drop) - 1u);
    uint32_t up;
    if (r16 < 0) {
      const uint32_t half = 1u << (drop - 1);
      up = frac > half || (frac == half && ((mag >> drop) & 1u));
    } else {
      const uint32_t f16 = drop >= 16 ? frac >> (drop - 16) : frac << (16 - drop);
      up = (f16 + (uint32_t)r16) >> 16;
    }
    q = ((mag >> drop) + up) << drop;
  } else {
    // below the smallest normal: uniform grid of spacing 2^(emin - M); |t| / spacing as fixed point
    const float pos = u2f(mag) * u2f((uint32_t)(M - emin + 127) << 23);      // exact power-of-two scaling
    float lo = __builtin_floorf(pos);
    const float frac = pos - lo;                                             // exact
    if (r16 < 0) lo = __builtin_rintf(pos);
    else lo += (__builtin_floorf(frac * 65536.0f) + (float)r16 >= 65536.0f) ? 1.0f : 0.0f;
    q = f2u(lo * u2f((uint32_t)(emin - M + 127) << 23));
  }
  q = q > top ? top : q;
  return u2f((bits & 0x80000000u) | q);
}

template <int FMT> __device__ inline uint32_t quant_rne(float t) {
  return FMT == FMT_BF16 ? bf16_rne(t) : e4m3_rne(t);
}
template <int FMT> __device__ inline uint32_t quant_sr(float t, uint32_t r16) {
  return FMT == FMT_BF16 ? bf16_sr(t, r16) : e4m3_sr(t, r16);
}
template <int FMT> __device__ inline float decode(uint32_t bits) {
  return FMT == FMT_BF16 ? bf16_decode(bits) : e4m3_decode(bits);
}

// ---------------------------------------------------------------------------------------------
// One element of the fused update (Algorithm 1, fuse_update; Kahan recurrence of Section 3 with
// s = w, v = -lr*g).  Every FP32 operation is rounded once (no fused multiply-add).
//   plain : t = w - lr*g                    w' = Q(t)
//   Kahan : y = -(lr*g) - c;  t = w + y     w' = Q(t);  c' = RNE_BF16((w' - w) - y)
// ---------------------------------------------------------------------------------------------
// Weight decay (wd != 0; the classifier's WD of the paper's hyper-parameter table, read as the L2
// term of plain SGD): g <- g + wd*w, two more rounded operations, before the lines above.
template <int FMT, bool SR, bool KAHAN>
__device__ inline void update_element(uint32_t& wbits, uint32_t& cbits, float g, float lr, float wd, uint32_t r16) {
  const float w = decode<FMT>(wbits);
  if (wd != 0.0f) g = __fadd_rn(g, __fmul_rn(wd, w));
  const float u = __fmul_rn(lr, g);
  float t, y = 0.0f;
  if (KAHAN) {
    y = __fsub_rn(-u, bf16_decode(cbits));
    t = __fadd_rn(w, y);
  } else {
    t = __fsub_rn(w, u);
  }
  const uint32_t q = SR ? quant_sr<FMT>(t, r16) : quant_rne<FMT>(t);
  if (KAHAN) {
    const float wn = decode<FMT>(q);
    cbits = bf16_rne(__fsub_rn(__fsub_rn(wn, w), y));
  }
  wbits = q;
}

}  // namespace elmo
