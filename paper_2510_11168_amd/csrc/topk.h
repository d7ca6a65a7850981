// Top-k scoring over all labels (the top_k of the paper's P@k definition) for gfx950.
//
// The [B, L] score matrix is never formed.  A workgroup owns 64 query rows and one contiguous
// segment of the labels; it walks the segment in 128-label tiles, computes the tile's logits on
// the matrix cores exactly as the training step does (E4M3 x E4M3 or BF16 x BF16, FP32
// accumulation), and keeps per row a sorted list of the k best (score, id) seen so far in LDS.
// Only scores above the row's current k-th best take the insertion path.  A second kernel merges
// the per-segment lists of a row.  Order: score descending, label id ascending on ties.
#pragma once
#include <limits.h>

#include <algorithm>
#include <cstdio>

#include "kernels.h"

namespace elmo {

constexpr int kTopkMaxK = 128;
constexpr int kTopkRows = 64;                       // query rows per workgroup
constexpr int kTopkZP = 132;                        // floats per staged row
constexpr int kTopkLP = 129;                        // list pitch (odd: one row per thread, no bank clash)
constexpr int kTopkStage = 49152;                   // operand double buffer (2 x (8 + 16) KiB); aliases the stage
constexpr int kTopkSmem = kTopkStage + 2 * kTopkRows * kTopkLP * 4 + kTopkRows * 16;
static_assert(kTopkRows * kTopkZP * 4 <= kTopkStage, "staged tile must fit the operand buffers");

// Label segments per 64-row group: enough workgroups to fill the chip, at most 64 lists to merge.
inline int topk_segments(int tiles_b) { return std::max(1, std::min(64, 512 / tiles_b)); }

// Bytes of per-segment partial lists for any batch of at most Bp_max rows.
inline size_t topk_scratch_bytes(int Bp_max, int64_t /*chunk*/) {
  const int tb_max = (Bp_max + kTopkRows - 1) / kTopkRows;
  size_t lists = 0;
  for (int tb = 1; tb <= tb_max; ++tb) lists = std::max(lists, (size_t)tb * kTopkRows * topk_segments(tb));
  return lists * kTopkMaxK * 8;
}

template <bool FP8>
__global__ void __launch_bounds__(kThreads, 1)
k_topk_chunk(const char* __restrict__ Xa, int a_rows, const char* __restrict__ W, int64_t L, int d, int k, int P,
             int tiles_per_seg, float* __restrict__ part_sc, int* __restrict__ part_id) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* zs = reinterpret_cast<float*>(smem);
  float* lsc = reinterpret_cast<float*>(smem + kTopkStage);
  int* lid = reinterpret_cast<int*>(smem + kTopkStage + kTopkRows * kTopkLP * 4);
  uint32_t* hit = reinterpret_cast<uint32_t*>(smem + kTopkStage + 2 * kTopkRows * kTopkLP * 4);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  const int seg = blockIdx.x % P, bt = blockIdx.x / P;
  const int b0 = bt * kTopkRows;
  const int tiles_l = (int)((L + 127) >> 7);
  const int t0 = seg * tiles_per_seg, t1 = min(t0 + tiles_per_seg, tiles_l);
  const size_t rowb = (size_t)d * (FP8 ? 1 : 2);
  const int nk = (int)(rowb >> 7);

  for (int i = tid; i < kTopkRows * kTopkLP; i += kThreads) { lsc[i] = -INFINITY; lid[i] = INT_MAX; }
  __syncthreads();

  TileLoader<128, 128> lw;
  TileLoader<64, 128> lx;
  const char* gx = Xa + (size_t)b0 * rowb;
  const int vx = a_rows - b0;
  for (int t = t0; t < t1; ++t) {
    const int64_t l0 = (int64_t)t << 7;
    const char* gw = W + (size_t)l0 * rowb;
    const int vw = (int)min<int64_t>(128, L - l0);
    f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][v] = 0.0f;
    lw.load(gw, rowb, vw, tid);
    lx.load(gx, rowb, vx, tid);
    lw.store(smem, tid);
    lx.store(smem + 16384, tid);
    __syncthreads();
    for (int ks = 0; ks < nk; ++ks) {
      const char* sw = smem + (ks & 1) * 24576;
      const char* sx = sw + 16384;
      if (ks + 1 < nk) {
        lw.load(gw + (size_t)(ks + 1) * 128, rowb, vw, tid);
        lx.load(gx + (size_t)(ks + 1) * 128, rowb, vx, tid);
      }
      if (FP8) {
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
          const i32x8 b = frag_fp8(sx, wn * 32, kk, lane);
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const i32x8 a = frag_fp8(sw, wm * 64 + 32 * i, kk, lane);
            acc[i] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[i], 0, 0, 0, 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
          const bf16x8 b = frag_bf16(sx, wn * 32, kk, lane);
#pragma unroll
          for (int i = 0; i < 2; ++i) {
            const bf16x8 a = frag_bf16(sw, wm * 64 + 32 * i, kk, lane);
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
          }
        }
      }
      if (ks + 1 < nk) {
        char* dw = smem + ((ks + 1) & 1) * 24576;
        lw.store(dw, tid);
        lx.store(dw + 16384, tid);
      }
      __syncthreads();
    }
    // stage Z[b][l] (aliases the operand buffers; every wave is past its last fragment read)
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int b = wn * 32 + (lane & 31);
        const int l = wm * 64 + 32 * i + 8 * q + 4 * (lane >> 5);
        f32x4 z;
        z[0] = acc[i][4 * q]; z[1] = acc[i][4 * q + 1]; z[2] = acc[i][4 * q + 2]; z[3] = acc[i][4 * q + 3];
        *reinterpret_cast<f32x4*>(zs + b * kTopkZP + l) = z;
      }
    __syncthreads();
    {  // pre-filter: which of this row-quarter's 32 scores beat the row's current k-th best
      const int r = tid >> 2, q = tid & 3;
      const float tau = lsc[r * kTopkLP + k - 1];
      uint32_t m = 0;
#pragma unroll 8
      for (int e = 0; e < 32; ++e) {
        const int l = 32 * q + e;
        if (l < vw && zs[r * kTopkZP + l] > tau) m |= 1u << e;
      }
      hit[r * 4 + q] = m;
    }
    __syncthreads();
    if (tid < kTopkRows && b0 + tid < a_rows) {   // one thread per row drains its hits in label order
      const int r = tid;
      float* sc = lsc + r * kTopkLP;
      int* id = lid + r * kTopkLP;
      for (int q = 0; q < 4; ++q) {
        uint32_t m = hit[r * 4 + q];
        while (m) {
          const int e = __ffs(m) - 1;
          m &= m - 1;
          const float z = zs[r * kTopkZP + 32 * q + e];
          if (z > sc[k - 1]) {
            int i = k - 1;
            while (i > 0 && sc[i - 1] < z) { sc[i] = sc[i - 1]; id[i] = id[i - 1]; --i; }
            sc[i] = z;
            id[i] = (int)l0 + 32 * q + e;
          }
        }
      }
    }
    __syncthreads();
  }
  for (int i = tid; i < kTopkRows * k; i += kThreads) {
    const int r = i / k, c = i % k;
    const size_t o = ((size_t)(b0 + r) * P + seg) * kTopkMaxK + c;
    part_sc[o] = lsc[r * kTopkLP + c];
    part_id[o] = lid[r * kTopkLP + c];
  }
}

// Merge the P per-segment lists of one row: bitonic sort of P*k (padded to a power of two) pairs
// by (score descending, id ascending), first k written out.
__global__ void __launch_bounds__(kThreads) k_topk_merge(const float* __restrict__ part_sc, const int* __restrict__ part_id,
                                                         int P, int k, int N2, int* __restrict__ idx_out,
                                                         float* __restrict__ score_out) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* sc = reinterpret_cast<float*>(smem);
  int* id = reinterpret_cast<int*>(smem + (size_t)N2 * 4);
  const int b = blockIdx.x, tid = threadIdx.x;
  const int items = P * k;
  for (int i = tid; i < N2; i += kThreads) {
    if (i < items) {
      const size_t o = ((size_t)b * P + i / k) * kTopkMaxK + i % k;
      sc[i] = part_sc[o];
      id[i] = part_id[o];
    } else {
      sc[i] = -INFINITY;
      id[i] = INT_MAX;
    }
  }
  __syncthreads();
  for (int size = 2; size <= N2; size <<= 1) {
    for (int stride = size >> 1; stride > 0; stride >>= 1) {
      for (int i = tid; i < (N2 >> 1); i += kThreads) {
        const int lo = 2 * i - (i & (stride - 1));       // index with the `stride` bit clear
        const int hi = lo + stride;
        const bool desc = (lo & size) == 0;              // direction of this bitonic block
        const float a = sc[lo], c = sc[hi];
        const int ia = id[lo], ic = id[hi];
        const bool a_first = a > c || (a == c && ia < ic);   // a belongs before c in the final order
        if (a_first != desc) { sc[lo] = c; sc[hi] = a; id[lo] = ic; id[hi] = ia; }
      }
      __syncthreads();
    }
  }
  for (int i = tid; i < k; i += kThreads) {
    if (idx_out) idx_out[(size_t)b * k + i] = id[i];
    if (score_out) score_out[(size_t)b * k + i] = sc[i];
  }
}

inline int topk_run(hipStream_t st, bool fp8, const char* Xa, int a_rows, const char* W, int64_t L, int d, int64_t /*chunk*/,
                    int B, int Bp, int k, char* scratch, int* idx_out, float* score_out, char* err, size_t errsz) {
  const int tiles_b = (B + kTopkRows - 1) / kTopkRows;
  const int tiles_l = (int)((L + 127) / 128);
  int P = topk_segments(tiles_b);
  P = std::min(P, tiles_l);
  const int tps = (tiles_l + P - 1) / P;
  P = (tiles_l + tps - 1) / tps;
  float* part_sc = reinterpret_cast<float*>(scratch);
  int* part_id = reinterpret_cast<int*>(scratch + (size_t)tiles_b * kTopkRows * P * kTopkMaxK * 4);
  if ((size_t)tiles_b * kTopkRows * P * kTopkMaxK * 8 > topk_scratch_bytes(Bp, 0)) {
    snprintf(err, errsz, "top-k scratch plan exceeded");
    return -3;
  }
  if (fp8) k_topk_chunk<true><<<tiles_b * P, kThreads, kTopkSmem, st>>>(Xa, a_rows, W, L, d, k, P, tps, part_sc, part_id);
  else k_topk_chunk<false><<<tiles_b * P, kThreads, kTopkSmem, st>>>(Xa, a_rows, W, L, d, k, P, tps, part_sc, part_id);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) { snprintf(err, errsz, "launch of k_topk_chunk failed: %s", hipGetErrorString(e)); return -3; }
  int N2 = 2;
  while (N2 < P * k) N2 <<= 1;
  k_topk_merge<<<B, kThreads, (size_t)N2 * 8, st>>>(part_sc, part_id, P, k, N2, idx_out, score_out);
  e = hipGetLastError();
  if (e != hipSuccess) { snprintf(err, errsz, "launch of k_topk_merge failed: %s", hipGetErrorString(e)); return -3; }
  return 0;
}

}  // namespace elmo
