// LDS tile staging and MFMA fragment access shared by the head's three matrix products
// (Algorithm 1: logits, input gradient, weight gradient).  gfx950 only, 64-wide wavefronts,
// 256-thread workgroups arranged as 2 x 2 waves.
//
// LDS tile layout: ROWS rows of ROWB bytes (ROWB = 128 or 256).  Rows are cut into 16-byte
// chunks and the low three bits of the chunk index are XORed with (row & 7), so that eight
// consecutive rows at the same logical chunk cover all 32 banks exactly once, both for the
// 16-byte fragment reads of K-contiguous operands and for the transposing reads.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elmo {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x2 __attribute__((ext_vector_type(2)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int kThreads = 256;

#define ELMO_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

template <int ROWB> __device__ inline int tile_off(int r, int c) {
  return r * ROWB + ((c ^ (r & 7)) << 4);
}

// Workgroups are dealt round-robin to the 8 XCDs (each with its own L2).  This maps the hardware
// id to a logical id such that consecutive logical ids run on the same XCD, so that tiles which
// share an operand (given consecutive logical ids) share that XCD's L2.
__device__ inline int xcd_logical_id(int wg, int nwg) {
  const int per = nwg >> 3;
  return wg < (per << 3) ? (wg & 7) * per + (wg >> 3) : wg;
}

// Global -> registers -> LDS copy of a ROWS x ROWB-byte slab of a row-major matrix.
// Rows at or beyond rows_valid read as zero (ragged last chunk / padded batch).
template <int ROWS, int ROWB> struct TileLoader {
  static constexpr int CPR = ROWB / 16;
  static constexpr int N = ROWS * CPR / kThreads;
  static_assert(ROWS * CPR % kThreads == 0, "tile must split evenly over the workgroup");
  u32x4 v[N];   // native vectors: plain loads/stores the optimiser keeps in registers
  __device__ inline void load(const char* __restrict__ g, size_t stride, int rows_valid, int tid) {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int id = it * kThreads + tid;
      const int r = id / CPR, c = id % CPR;
      if (r < rows_valid) v[it] = *reinterpret_cast<const u32x4*>(g + (size_t)r * stride + c * 16);
      else v[it] = u32x4{0u, 0u, 0u, 0u};
    }
  }
  // Branch-free variant: rows at or beyond rows_valid (>= 1) re-read the last valid row.  For
  // operands whose out-of-range rows only feed outputs that are masked later.
  __device__ inline void load_clamped(const char* __restrict__ g, size_t stride, int rows_valid, int tid) {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int id = it * kThreads + tid;
      const int r = min(id / CPR, rows_valid - 1), c = id % CPR;
      v[it] = *reinterpret_cast<const u32x4*>(g + (size_t)r * stride + c * 16);
    }
  }
  __device__ inline void store(char* lds, int tid) const {
#pragma unroll
    for (int it = 0; it < N; ++it) {
      const int id = it * kThreads + tid;
      const int r = id / CPR, c = id % CPR;
      *reinterpret_cast<u32x4*>(lds + tile_off<ROWB>(r, c)) = v[it];
    }
  }
};

// ---------------------------------------------------------------------------------------------
// K-contiguous operands (rows of 128 bytes = one K slab).
// BF16, v_mfma_f32_32x32x16_bf16: lane i holds row i%32, K elements 8*(i/32) .. +7 of the step.
// ---------------------------------------------------------------------------------------------
__device__ inline bf16x8 frag_bf16(const char* lds, int row0, int kstep, int lane) {
  const int r = row0 + (lane & 31);
  return *reinterpret_cast<const bf16x8*>(lds + tile_off<128>(r, 2 * kstep + (lane >> 5)));
}
// FP8, v_mfma_f32_32x32x64_f8f6f4: lane i holds row i%32, K bytes 32*(i/32) .. +31 of the step.
__device__ inline i32x8 frag_fp8(const char* lds, int row0, int kstep, int lane) {
  const int r = row0 + (lane & 31);
  const int c = 4 * kstep + 2 * (lane >> 5);
  const i32x4 lo = *reinterpret_cast<const i32x4*>(lds + tile_off<128>(r, c));
  const i32x4 hi = *reinterpret_cast<const i32x4*>(lds + tile_off<128>(r, c + 1));
  i32x8 o;
  o[0] = lo[0]; o[1] = lo[1]; o[2] = lo[2]; o[3] = lo[3];
  o[4] = hi[0]; o[5] = hi[1]; o[6] = hi[2]; o[7] = hi[3];
  return o;
}

// ---------------------------------------------------------------------------------------------
// K-major operands (tile rows are K, the M or N index is contiguous): transposing LDS reads.
// ds_read_b64_tr_b16: within each group of 16 lanes, lane q supplies the address of 4 elements
// (row q/4 of a 4 x 16 block, columns 4*(q%4)..+3) and receives column q of that block, rows 0..3.
// ds_read_b64_tr_b8: lane q supplies 8 bytes (row q/2 of an 8 x 16 block, columns 8*(q%2)..+7) and
// receives column q, rows 0..7.
// Fragment for v_mfma_f32_32x32x16_bf16 at K rows k0 .. k0+15 of the tile and columns col0..+31:
// lane i -> column col0 + i%32, K rows k0 + 8*(i/32) .. +7.
// ---------------------------------------------------------------------------------------------
template <int ROWB> __device__ inline bf16x8 frag_tr_bf16(const char* lds, int k0, int col0, int lane) {
  const int g = lane >> 4, q = lane & 15;
  const int col = col0 + 16 * (g & 1) + 4 * (q & 3);     // element column of this lane's 8 bytes
  const int kr = k0 + 8 * (g >> 1) + (q >> 2);
  const int c = col >> 3, h = (col & 4) << 1;            // 16-byte chunk, byte offset inside it
  const s16x4 a = __builtin_amdgcn_ds_read_tr16_b64_v4i16(ELMO_LDS_PTR(s16x4, lds + tile_off<ROWB>(kr, c) + h));
  const s16x4 b = __builtin_amdgcn_ds_read_tr16_b64_v4i16(ELMO_LDS_PTR(s16x4, lds + tile_off<ROWB>(kr + 4, c) + h));
  union { s16x4 s[2]; bf16x8 v; } u;
  u.s[0] = a; u.s[1] = b;
  return u.v;
}
// Same fragment from an FP8 (E4M3) tile; the eight values are widened to BF16 (exact).
template <int ROWB> __device__ inline bf16x8 frag_tr_fp8(const char* lds, int k0, int col0, int lane) {
  const int g = lane >> 4, q = lane & 15;
  const int col = col0 + 16 * (g & 1) + 8 * (q & 1);     // byte column of this lane's 8 bytes
  const int kr = k0 + 8 * (g >> 1) + (q >> 1);
  const i32x2 w = __builtin_amdgcn_ds_read_tr8_b64_v2i32(ELMO_LDS_PTR(i32x2, lds + tile_off<ROWB>(kr, col >> 4) + (col & 8)));
  union { bf16x2 p[4]; bf16x8 v; } u;
  u.p[0] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)w[0], 1.0f, false);
  u.p[1] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)w[0], 1.0f, true);
  u.p[2] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)w[1], 1.0f, false);
  u.p[3] = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((unsigned)w[1], 1.0f, true);
  return u.v;
}

// Accumulator element v (0..15) of a 32x32 MFMA tile sits at row 8*(v/4) + 4*(lane/32) + v%4,
// column lane%32.
__device__ inline int acc_row(int v, int lane) { return 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3); }

}  // namespace elmo
