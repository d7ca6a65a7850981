// Top-k scoring over all labels (the top_k of the paper's P@k definition) for gfx950.
//
// The [B, L] score matrix is never formed.  Main path: the labels are visited in levels of
// geometrically growing size (the first 1024, then each level takes the labels seen so far from
// N to 4 N).  A level computes its logits tile by tile on the matrix cores exactly as the
// training step does (E4M3 x E4M3 or BF16 x BF16, FP32 accumulation) and appends every score that
// beats the row's threshold -- the k-th best score over all earlier levels -- to the row's
// candidate list; a select kernel then sorts the candidates, keeps the k best and raises the
// threshold.  A later label that merely ties the threshold can never enter the top k (same score,
// larger id), so the comparison is strict and the result exact.  With thresholds from a quarter
// of the labels a level is expected to append about 3 x k scores per row (scores in no particular
// order along the label axis); the lists hold 4096.  Every append is an atomic addition on the
// row's counter, and those cost more than anything else besides the product: with levels growing
// 17-fold (about 16 x k appends per row and level, 3600 per row in all at 3 M labels and k = 100) the two middle
// levels took up to five times their product's time; growing 4-fold (1500 appends per row in all,
// and selects over 400 instead of 1700 candidates) measured 9 % faster end to end, 3-fold the same,
// 2-fold slower again (more launches).  In the large levels a pass is rare (a few per row and
// million labels), so the filter first takes one wave-wide vote per sample on the largest of a
// lane's four scores and skips the four compares when no lane passes (13 % end to end).
// A row whose list overflows (scores rising steeply with
// the label id) is flagged and recomputed by the fallback path below, which has no capacity
// limit: 64 query rows per workgroup walk a label segment keeping a sorted k-list in LDS, and a
// merge kernel joins the segments.  Order: score descending, label id ascending on ties.
//
// k above 128: the result is produced in pages of 128 entries.  Every page is one more sweep over
// the labels that only admits (score, id) pairs strictly after the last entry of the page before
// it in that order (the row's cursor), so page p holds entries 128 p .. 128 p + 127 of the full
// ranking exactly.  Costs one pass over W per 128 entries; k <= 128 (evaluation uses k <= 100) is
// a single sweep with no cursor.
#pragma once
#include <limits.h>

#include <algorithm>
#include <cstdio>

#include "kernels.h"

namespace elmo {

constexpr int kTopkMaxK = 128;                     // entries selected per sweep (one page)
constexpr int kTopkCand = 4096;                    // candidate list length per row (main path)
constexpr int kTopkCntStride = 32;                 // ints between two rows' candidate counters: one 128-byte line each, so that the
                                                   // atomic additions of different rows do not queue up on the same few lines
constexpr int kTopkGrowth = 4;                     // labels seen after a level / labels seen before it
constexpr int kTopkLevel0 = 1024;                  // labels of the first level
constexpr int kTopkRows = 64;                       // query rows per workgroup
constexpr int kTopkZP = 132;                        // floats per staged row
constexpr int kTopkLP = 129;                        // list pitch (odd: one row per thread, no bank clash)
constexpr int kTopkStage = 49152;                   // operand double buffer (2 x (8 + 16) KiB); aliases the stage
constexpr int kTopkSmem = kTopkStage + 2 * kTopkRows * kTopkLP * 4 + kTopkRows * 16;
static_assert(kTopkRows * kTopkZP * 4 <= kTopkStage, "staged tile must fit the operand buffers");

// Label segments per 64-row group: enough workgroups to fill the chip, at most 64 lists to merge.
inline int topk_segments(int tiles_b) { return std::max(1, std::min(64, 512 / tiles_b)); }

// Main-path scratch: thresholds, counters, overflow flags and candidate lists per (padded) row.
inline size_t topk_main_rows(int Bp_max) { return (size_t)(Bp_max + 255) / 256 * 256; }
inline size_t topk_main_bytes(int Bp_max) { return topk_main_rows(Bp_max) * (24 + (size_t)kTopkCntStride * 4 + (size_t)kTopkCand * 8) + 1024; }

// (score, id) strictly after the cursor (cs, ci) in the order score descending, id ascending.
__device__ inline bool topk_after(float z, int l, float cs, int ci) { return z < cs || (z == cs && l > ci); }

// Bytes of per-segment partial lists for any batch of at most Bp_max rows, plus the main path's.
inline size_t topk_scratch_bytes(int Bp_max, int64_t /*chunk*/) {
  const int tb_max = (Bp_max + kTopkRows - 1) / kTopkRows;
  size_t lists = 0;
  for (int tb = 1; tb <= tb_max; ++tb) lists = std::max(lists, (size_t)tb * kTopkRows * topk_segments(tb));
  return lists * kTopkMaxK * 8 + topk_main_bytes(Bp_max);
}

template <bool FP8>
__global__ void __launch_bounds__(kThreads, 1)
k_topk_chunk(const char* __restrict__ Xa, int a_rows, const char* __restrict__ W, int64_t L, int d, int k, int P,
             int tiles_per_seg, float* __restrict__ part_sc, int* __restrict__ part_id, const int* __restrict__ only_rows,
             int B, const float* __restrict__ cur_sc, const int* __restrict__ cur_id) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  if (only_rows) {   // fallback use: nothing to do unless one of this group's rows is flagged
    const int r = (blockIdx.x / P) * kTopkRows + (threadIdx.x & 63);
    if (!__syncthreads_or(r < B && only_rows[r] != 0)) return;
  }
  float* zs = reinterpret_cast<float*>(smem);
  float* lsc = reinterpret_cast<float*>(smem + kTopkStage);
  int* lid = reinterpret_cast<int*>(smem + kTopkStage + kTopkRows * kTopkLP * 4);
  uint32_t* hit = reinterpret_cast<uint32_t*>(smem + kTopkStage + 2 * kTopkRows * kTopkLP * 4);
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
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
      const bool paged = cur_sc != nullptr && b0 + r < B;
      const float cs = paged ? cur_sc[b0 + r] : INFINITY;
      const int ci = paged ? cur_id[b0 + r] : -1;
      uint32_t m = 0;
#pragma unroll 8
      for (int e = 0; e < 32; ++e) {
        const int l = 32 * q + e;
        const float z = zs[r * kTopkZP + l];
        if (l < vw && z > tau && (!paged || topk_after(z, (int)l0 + l, cs, ci))) m |= 1u << e;
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

// In-LDS bitonic sort of N2 (a power of two) pairs by (score descending, id ascending).
__device__ inline void bitonic_sort_pairs(float* sc, int* id, int N2, int tid) {
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
}

// Merge the P per-segment lists of one row: bitonic sort of P*k (padded to a power of two) pairs
// by (score descending, id ascending), first k written out.
// Output row pitch out_ld, first column out_off (the page); next_sc / next_id receive the row's new cursor.
__global__ void __launch_bounds__(kThreads) k_topk_merge(const float* __restrict__ part_sc, const int* __restrict__ part_id,
                                                         int P, int k, int N2, int* __restrict__ idx_out,
                                                         float* __restrict__ score_out, const int* __restrict__ only_rows,
                                                         int out_ld, int out_off, float* __restrict__ next_sc,
                                                         int* __restrict__ next_id) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  float* sc = reinterpret_cast<float*>(smem);
  int* id = reinterpret_cast<int*>(smem + (size_t)N2 * 4);
  const int b = blockIdx.x, tid = threadIdx.x;
  if (only_rows && only_rows[b] == 0) return;
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
  bitonic_sort_pairs(sc, id, N2, tid);
  for (int i = tid; i < k; i += kThreads) {
    if (idx_out) idx_out[(size_t)b * out_ld + out_off + i] = id[i];
    if (score_out) score_out[(size_t)b * out_ld + out_off + i] = sc[i];
  }
  if (tid == 0 && next_sc) { next_sc[b] = sc[k - 1]; next_id[b] = id[k - 1]; }
}

// ---------------------------------------------------------------------------------------------
// Main path: threshold filter fused into the logits tile, and the per-row select.
// ---------------------------------------------------------------------------------------------
// cnt0: candidates per row that the first level writes without counting (all of its labels).
// Rows at or beyond B (padding up to whole 256-row tiles) get an infinite threshold: they never emit.
__global__ void __launch_bounds__(kThreads) k_topk_init(float* __restrict__ tau, int* __restrict__ cnt, int* __restrict__ ovf, int rows,
                                                        int B, int cnt0) {
  const int i = blockIdx.x * kThreads + threadIdx.x;
  if (i < rows) { tau[i] = i < B ? -INFINITY : INFINITY; cnt[(size_t)i * kTopkCntStride] = cnt0; ovf[i] = 0; }
}

// Logits of labels [l_begin, l_begin + n) for all rows, 256 x 256 tiles as in the training step.
// The first level has no threshold yet and at most kTopkCand labels: label l of the level goes to
// slot l of every row, no counting (scores that could never be selected, NaN or -inf, are stored
// as empty slots).
template <bool FP8>
__global__ void __launch_bounds__(kGemmThreads, 1)
k_topk_first(const char* __restrict__ Xa, int a_rows, const char* __restrict__ Wl, int n, int l_begin, int d, int Bp, int B,
             float* __restrict__ cand_sc, int* __restrict__ cand_id, const float* __restrict__ cur_sc, const int* __restrict__ cur_id) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
  const int tiles_b = (Bp + 255) >> 8;
  const int wg = xcd_logical_id(blockIdx.x, gridDim.x);
  const int lt = wg / tiles_b, bt = wg % tiles_b;
  const int b0 = bt << 8, l0 = lt << 8;
  const size_t rowb = (size_t)d * (FP8 ? 1 : 2);
  // cursors of the tile's rows (pages after the first), else +inf / -1: in LDS behind the ring,
  // loaded before the product (the K loop's barriers publish them)
  float* cs_s = reinterpret_cast<float*>(smem + logits_mask_offset<256>());
  int* ci_s = reinterpret_cast<int*>(cs_s + 256);
  const bool paged = cur_sc != nullptr;
  for (int i = tid; i < 256; i += kGemmThreads) {
    cs_s[i] = paged && b0 + i < B ? cur_sc[b0 + i] : INFINITY;
    ci_s[i] = paged && b0 + i < B ? cur_id[b0 + i] : -1;
  }
  f32x16 acc[2][4];
  logits_tile_product<FP8, 256, 4>(Xa + (size_t)b0 * rowb, a_rows - b0, Wl + (size_t)l0 * rowb, n - l0, rowb, smem, wave, lane, acc);
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int b = wm * 64 + 32 * i + acc_row(v, lane);
      const int row = b0 + b;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int l = l0 + wn * 128 + 32 * j + (lane & 31);
        const float z = acc[i][j][v];
        if (l < n && row < B) {
          const bool live = z > -INFINITY && (!paged || topk_after(z, l_begin + l, cs_s[b], ci_s[b]));
          cand_sc[(size_t)row * kTopkCand + l] = live ? z : -INFINITY;
          cand_id[(size_t)row * kTopkCand + l] = live ? l_begin + l : INT_MAX;
        }
      }
    }
}

// The levels after the first: one workgroup per CU walks the tiles w, w + gridDim, ... of the level
// and keeps the ring of K slabs running from one tile into the next, so a tile's first slabs are
// on their way while the tile before it is being filtered (a workgroup per tile pays the first
// slab's round trip, a third of a tile's K loop at d = 768, and the launch of the next workgroup
// between any two tiles of a CU).  The thresholds (and cursors) of a tile's 256 rows are fetched
// by asynchronous loads into one of two LDS buffers behind the ring a tile ahead; the two-stage
// ring waits for all of a wave's loads at every slab, so they need no accounting of their own.
// DENSE: for the small early levels, where a large share of the scores still passes (several per
// row among a wave's 128 labels): the 32 lanes of a half wave hold 4 x 32 labels of one row per
// accumulator index (i, v); the half's first lane reserves the slots of all of the half's passes
// with one atomic addition, the sixteen additions of one i are issued before the first result is
// waited for, and the slots are handed out by position in the vote masks.  With one addition per
// passing score these levels took four times their product's time; in the large levels, where a
// wave rarely sees two passes of one row, the plain form is the faster one.
// Large levels, appends: a row's counter is shared by every workgroup that holds one of the row's
// tiles, on all XCDs, so an append is a device-scope atomic addition carried out at the memory
// side, and the wave waits a memory round trip for its slot before it can go on.  A workgroup
// therefore keeps one batch tile for all of its label tiles (the grid is a multiple of the number
// of batch tiles) and collects its passes in LDS lists of kTopkLdsCap entries per row (LDS
// atomics); at its end it reserves each row's slots with one global addition and copies the
// entries.  A row whose LDS list is full appends directly as before.
constexpr int kTopkLdsCap = 8;
constexpr int kTopkSide = 3 * 256 * 4;                // [thresholds | cursor scores | cursor ids] of a tile's 256 rows
constexpr int kTopkRunSmem = kWideRingBytes + 2 * kTopkSide + 256 * 4 + 256 * kTopkLdsCap * 8;   // ring, two side buffers, LDS lists
static_assert(kTopkRunSmem <= 160 * 1024, "LDS plan of the persistent filter");
template <bool FP8, bool DENSE>
__global__ void __launch_bounds__(kGemmThreads, 1)
k_topk_filter_run(const char* __restrict__ Xa, int a_rows, const char* __restrict__ Wl, int n, int l_begin, int d, int Bp,
                  const float* __restrict__ tau, int* __restrict__ cnt, int* __restrict__ ovf, float* __restrict__ cand_sc,
                  int* __restrict__ cand_id, const float* __restrict__ cur_sc, const int* __restrict__ cur_id) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
  const int tiles_b = (Bp + 255) >> 8, ntiles = ((n + 255) >> 8) * tiles_b;
  const int G = (int)gridDim.x, w0 = xcd_logical_id((int)blockIdx.x, (int)gridDim.x);   // consecutive w0 share an XCD (and a label tile)
  if (w0 >= ntiles) return;
  const int mine = (ntiles - w0 + G - 1) / G;                          // this workgroup's tiles: w0, w0 + G, ...
  const bool agg = !DENSE && G % tiles_b == 0;                         // one batch tile for all of them: passes collect in LDS
  const size_t rowb = (size_t)d * (FP8 ? 1 : 2);
  const int nk = (int)(rowb >> 7);
  const bool paged = cur_sc != nullptr;
  constexpr int kSide = kTopkSide;
  char* side = smem + kWideRingBytes;                                  // behind the ring
  auto tile_of = [&](int t, int& b0, int& l0) {
    const int wg = w0 + t * G;
    l0 = (wg / tiles_b) << 8;
    b0 = (wg % tiles_b) << 8;
  };
  char* lists = side + 2 * kSide;                                      // [256 rows][kTopkLdsCap] (score, id) pairs, then 256 counters
  if (agg) {
    for (int i = tid; i < 256; i += kGemmThreads) reinterpret_cast<int*>(lists + 256 * kTopkLdsCap * 8)[i] = 0;
    barrier_lds();
  }
  auto dma_rows = [&](const void* src, char* dst) {                    // 256 consecutive 4-byte values -> LDS, issued by one wave
    const char* g = reinterpret_cast<const char*>(src);
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)g), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uintptr_t)g >> 32));
    asm volatile("" : "+s"(lo), "+s"(hi));
    g = reinterpret_cast<const char*>(((uintptr_t)hi << 32) | lo);
    const uint32_t d32 = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)dst);
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(d32), "v"((uint32_t)(lane * 16)), "s"(g) : "memory", "m0");
  };
  auto fetch_side = [&](int t) {
    if (wave != 0 || t >= mine) return;
    int b0, l0;
    tile_of(t, b0, l0);
    char* dst = side + (t & 1) * kSide;
    dma_rows(tau + b0, dst);
    if (paged) {
      dma_rows(cur_sc + b0, dst + 1024);
      dma_rows(cur_id + b0, dst + 2048);
    }
  };
  f32x16 acc[2][4];
  auto filter = [&](int t) {
    int b0, l0;
    tile_of(t, b0, l0);
    const float* tau_s = reinterpret_cast<const float*>(side + (t & 1) * kSide);
    const float* cs_s = tau_s + 256;
    const int* ci_s = reinterpret_cast<const int*>(cs_s + 256);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int b = wm * 64 + 32 * i + acc_row(v, lane);
        const float th = tau_s[b];
        // passes are rare in these levels (a few per row and million labels): one vote on the largest of the
        // lane's four scores of this sample skips the rest for the whole wave nine times out of ten
        const float zmax = fmaxf(fmaxf(acc[i][0][v], acc[i][1][v]), fmaxf(acc[i][2][v], acc[i][3][v]));
        if (__builtin_amdgcn_ballot_w64(zmax > th) == 0ull) continue;
        // everything the rare branch needs is formed inside it, from an opaque copy of the lane index: nothing of it
        // is held in registers through the product
        int ln = lane;
        asm volatile("" : "+v"(ln));
        const int bb = wm * 64 + 32 * i + acc_row(v, ln);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int l = l0 + wn * 128 + 32 * j + (ln & 31);
          const float z = acc[i][j][v];
          if (l < n && z > th && (!paged || topk_after(z, l_begin + l, cs_s[bb], ci_s[bb]))) {
            const int row = b0 + bb;
            if (agg) {
              const int ls = atomicAdd(reinterpret_cast<int*>(lists + 256 * kTopkLdsCap * 8) + bb, 1);
              if (ls < kTopkLdsCap) {
                *reinterpret_cast<int2*>(lists + (bb * kTopkLdsCap + ls) * 8) = make_int2(__float_as_int(z), l_begin + l);
                continue;
              }
            }
            const int slot = atomicAdd(&cnt[(size_t)row * kTopkCntStride], 1);
            if (slot < kTopkCand) {
              cand_sc[(size_t)row * kTopkCand + slot] = z;
              cand_id[(size_t)row * kTopkCand + slot] = l_begin + l;
            } else {
              ovf[row] = 1;
            }
          }
        }
      }
  };
  auto filter_dense = [&](int t) {
    int b0, l0;
    tile_of(t, b0, l0);
    const float* tau_s = reinterpret_cast<const float*>(side + (t & 1) * kSide);
    const float* cs_s = tau_s + 256;
    const int* ci_s = reinterpret_cast<const int*>(cs_s + 256);
    const int half = lane >> 5;
    const uint32_t below = (1u << (lane & 31)) - 1u;
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      uint32_t pbits[4] = {0u, 0u, 0u, 0u};                              // bit v of pbits[j]: acc[i][j][v] passes
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int b = wm * 64 + 32 * i + acc_row(v, lane);
        const float th = tau_s[b];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int l = l0 + wn * 128 + 32 * j + (lane & 31);
          const float z = acc[i][j][v];
          const bool pass = l < n && z > th && (!paged || topk_after(z, l_begin + l, cs_s[b], ci_s[b]));
          pbits[j] |= (uint32_t)pass << v;
        }
      }
      const uint32_t anyj = pbits[0] | pbits[1] | pbits[2] | pbits[3];
      if (__builtin_amdgcn_ballot_w64(anyj != 0u) == 0ull) continue;
      int base[16];
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        base[v] = 0;
        if (__builtin_amdgcn_ballot_w64((anyj >> v) & 1u) == 0ull) continue;
        uint32_t tot = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint64_t bal = __builtin_amdgcn_ballot_w64((pbits[j] >> v) & 1u);
          tot += __builtin_popcount(half ? (uint32_t)(bal >> 32) : (uint32_t)bal);
        }
        if ((lane & 31) == 0 && tot != 0u)
          base[v] = atomicAdd(&cnt[(size_t)(b0 + wm * 64 + 32 * i + acc_row(v, lane)) * kTopkCntStride], (int)tot);
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) asm volatile("" : "+v"(pbits[j]));      // the votes are taken again below rather than kept over the additions
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        if (__builtin_amdgcn_ballot_w64((anyj >> v) & 1u) == 0ull) continue;
        const int base_lo = __builtin_amdgcn_readlane(base[v], 0), base_hi = __builtin_amdgcn_readlane(base[v], 32);
        int run = half ? base_hi : base_lo;
        const int row = b0 + wm * 64 + 32 * i + acc_row(v, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const bool pass = (pbits[j] >> v) & 1u;
          const uint64_t bal = __builtin_amdgcn_ballot_w64(pass);
          const uint32_t mine_m = half ? (uint32_t)(bal >> 32) : (uint32_t)bal;
          if (pass) {
            const int slot = run + __builtin_popcount(mine_m & below);
            if (slot < kTopkCand) {
              cand_sc[(size_t)row * kTopkCand + slot] = acc[i][j][v];
              cand_id[(size_t)row * kTopkCand + slot] = l_begin + l0 + wn * 128 + 32 * j + (lane & 31);
            } else {
              ovf[row] = 1;
            }
          }
          run += __builtin_popcount(mine_m);
        }
      }
    }
  };
  fetch_side(0);
  ring_stream_pp<256, 128, 256, 128, 2, kGemmWaves, true>(
      Xa, rowb, 8, Wl, rowb, 8, mine * nk, smem, wave, lane,
      [&](int ks, size_t& off_a, int& va, size_t& off_b, int& vb) {
        const int t = ks / nk, sl = ks - t * nk;
        int b0, l0;
        tile_of(t, b0, l0);
        off_a = (size_t)b0 * rowb + (size_t)sl * 128; va = a_rows - b0;
        off_b = (size_t)l0 * rowb + (size_t)sl * 128; vb = n - l0;
      },
      [&](const char* sa, const char* sb, int q0, int q1, int ks) {
        const int t = ks / nk, sl = ks - t * nk;
        if (q0 == 0 && sl == 0) {
          zero_acc(acc);
          fetch_side(t + 1);
        }
        logits_slab_product<FP8, 4>(sa, sb, q0 >> 1, wm, wn, lane, acc);
        if (q1 == 4 && sl == nk - 1) { if constexpr (DENSE) filter_dense(t); else filter(t); }
      });
  if (agg) {
    barrier_lds();                                                     // every wave's LDS appends are in
    int b0, l0;
    tile_of(0, b0, l0);
    for (int r = tid; r < 256; r += kGemmThreads) {
      const int c = min(reinterpret_cast<const int*>(lists + 256 * kTopkLdsCap * 8)[r], kTopkLdsCap);
      if (c == 0) continue;
      const int row = b0 + r;
      const int base = atomicAdd(&cnt[(size_t)row * kTopkCntStride], c);
      for (int e = 0; e < c; ++e) {
        const int2 en = *reinterpret_cast<const int2*>(lists + (r * kTopkLdsCap + e) * 8);
        if (base + e < kTopkCand) {
          cand_sc[(size_t)row * kTopkCand + base + e] = __int_as_float(en.x);
          cand_id[(size_t)row * kTopkCand + base + e] = en.y;
        } else {
          ovf[row] = 1;
        }
      }
    }
  }
}

// Per row: sort the candidates, keep the k best at the front of the list, raise the threshold.
__global__ void __launch_bounds__(kThreads) k_topk_select(float* __restrict__ tau, int* __restrict__ cnt, float* __restrict__ cand_sc,
                                                          int* __restrict__ cand_id, int k, int* __restrict__ idx_out,
                                                          float* __restrict__ score_out, int out_ld, int out_off,
                                                          float* __restrict__ next_sc, int* __restrict__ next_id) {
  __shared__ float sc[kTopkCand];
  __shared__ int id[kTopkCand];
  const int b = blockIdx.x, tid = threadIdx.x;
  const int m = min(cnt[(size_t)b * kTopkCntStride], kTopkCand);
  int N2 = 2;
  while (N2 < max(m, k)) N2 <<= 1;                   // the first k sorted slots are read below even when fewer candidates exist
  for (int i = tid; i < N2; i += kThreads) {
    sc[i] = i < m ? cand_sc[(size_t)b * kTopkCand + i] : -INFINITY;
    id[i] = i < m ? cand_id[(size_t)b * kTopkCand + i] : INT_MAX;
  }
  __syncthreads();
  bitonic_sort_pairs(sc, id, N2, tid);
  const int keep = min(m, k);
  for (int i = tid; i < keep; i += kThreads) {
    cand_sc[(size_t)b * kTopkCand + i] = sc[i];
    cand_id[(size_t)b * kTopkCand + i] = id[i];
  }
  if (tid == 0) {
    cnt[(size_t)b * kTopkCntStride] = keep;
    tau[b] = m >= k ? sc[k - 1] : -INFINITY;
  }
  if (idx_out || score_out)
    for (int i = tid; i < k; i += kThreads) {
      if (idx_out) idx_out[(size_t)b * out_ld + out_off + i] = id[i];
      if (score_out) score_out[(size_t)b * out_ld + out_off + i] = sc[i];
    }
  if (tid == 0 && next_sc) { next_sc[b] = sc[k - 1]; next_id[b] = id[k - 1]; }
}

// ---------------------------------------------------------------------------------------------
// P@k numerators: per position j the number of rows whose j-th prediction is a true label, then
// the running sum over positions.  Integer counts: the result does not depend on the order of the
// atomic additions.
// ---------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(kThreads) k_hits_at(const int* __restrict__ idx, int B, int k, const int* __restrict__ indptr,
                                                      const int* __restrict__ indices, unsigned long long* __restrict__ hits) {
  const int t = blockIdx.x * kThreads + threadIdx.x;
  if (t >= B * k) return;
  const int b = t / k, j = t - b * k;
  const int l = idx[t];
  int lo = indptr[b], hi = indptr[b + 1];          // binary search in the row's ascending ids
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (indices[mid] < l) lo = mid + 1; else hi = mid;
  }
  if (lo < indptr[b + 1] && indices[lo] == l) atomicAdd(&hits[j], 1ull);
}
__global__ void __launch_bounds__(kThreads) k_hits_scan(unsigned long long* __restrict__ hits, int k) {
  if (threadIdx.x == 0) {
    unsigned long long run = 0;
    for (int j = 0; j < k; ++j) { run += hits[j]; hits[j] = run; }
  }
}

inline int topk_launch_error(const char* what, char* err, size_t errsz) {
  const hipError_t e = hipGetLastError();
  if (e == hipSuccess) return 0;
  snprintf(err, errsz, "launch of %s failed: %s", what, hipGetErrorString(e));
  return -3;
}

inline int topk_run(hipStream_t st, bool fp8, const char* Xa, int a_rows, const char* W, int64_t L, int d, int64_t /*chunk*/,
                    int B, int Bp, int k_total, char* scratch, int* idx_out, float* score_out, char* err, size_t errsz) {
  const size_t rows = topk_main_rows(Bp);
  float* tau = reinterpret_cast<float*>(scratch);
  int* ovf = reinterpret_cast<int*>(scratch + rows * 4);
  float* cursor_sc[2] = {reinterpret_cast<float*>(scratch + rows * 8), reinterpret_cast<float*>(scratch + rows * 12)};
  int* cursor_id[2] = {reinterpret_cast<int*>(scratch + rows * 16), reinterpret_cast<int*>(scratch + rows * 20)};
  int* cnt = reinterpret_cast<int*>(scratch + rows * 24);                    // one counter per 128-byte line
  const size_t lists0 = rows * (24 + (size_t)kTopkCntStride * 4);
  float* cand_sc = reinterpret_cast<float*>(scratch + lists0);
  int* cand_id = reinterpret_cast<int*>(scratch + lists0 + rows * (size_t)kTopkCand * 4);
  char* fb_scratch = scratch + topk_main_bytes(Bp);
  const size_t rowb = (size_t)d * (fp8 ? 1 : 2);
  static_assert(kTopkLevel0 <= kTopkCand, "the first level writes one slot per label");
  const int tiles_b256 = (Bp + 255) / 256;
  // fallback geometry (rows whose candidate list overflowed)
  const int tiles_b = (B + kTopkRows - 1) / kTopkRows;
  const int tiles_l = (int)((L + 127) / 128);
  int P = topk_segments(tiles_b);
  P = std::min(P, tiles_l);
  const int tps = (tiles_l + P - 1) / P;
  P = (tiles_l + tps - 1) / tps;
  float* part_sc = reinterpret_cast<float*>(fb_scratch);
  int* part_id = reinterpret_cast<int*>(fb_scratch + (size_t)tiles_b * kTopkRows * P * kTopkMaxK * 4);
  if ((size_t)tiles_b * kTopkRows * P * kTopkMaxK * 8 + topk_main_bytes(Bp) > topk_scratch_bytes(Bp, 0)) {
    snprintf(err, errsz, "top-k scratch plan exceeded");
    return -3;
  }
  // one sweep over the labels per page of kTopkMaxK entries; pages after the first admit only what
  // lies strictly after the row's cursor (the last entry of the page before)
  for (int page = 0, off = 0; off < k_total; ++page, off += kTopkMaxK) {
    const int k = std::min(kTopkMaxK, k_total - off);
    const float* cs = page ? cursor_sc[page & 1] : nullptr;
    const int* ci = page ? cursor_id[page & 1] : nullptr;
    const bool more = off + k < k_total;
    float* ns = more ? cursor_sc[(page + 1) & 1] : nullptr;
    int* ni = more ? cursor_id[(page + 1) & 1] : nullptr;
    // ---- main path
    k_topk_init<<<(int)((rows + kThreads - 1) / kThreads), kThreads, 0, st>>>(tau, cnt, ovf, (int)rows, B,
                                                                               (int)std::min<int64_t>(L, kTopkLevel0));
    if (int rc = topk_launch_error("k_topk_init", err, errsz)) return rc;
    for (int64_t begin = 0, end = std::min<int64_t>(L, kTopkLevel0); begin < L; begin = end, end = std::min<int64_t>(L, end * kTopkGrowth)) {
      const int n = (int)(end - begin);
      const int grid = (n + 255) / 256 * tiles_b256;
      const char* Wl = W + (size_t)begin * rowb;
      const bool first = begin == 0;
      // persistent levels: at most one workgroup per CU, a multiple of the batch tiles when there are enough of them
      const int run_grid = grid <= 256 ? grid : (tiles_b256 <= 256 ? 256 - 256 % tiles_b256 : 256);
#define ELMO_TOPK_FIRST(F) \
  k_topk_first<F><<<grid, kGemmThreads, logits_smem<256>(), st>>>(Xa, a_rows, Wl, n, (int)begin, d, Bp, B, cand_sc, cand_id, cs, ci)
#define ELMO_TOPK_FILTER_RUN(F, DE) \
  k_topk_filter_run<F, DE><<<run_grid, kGemmThreads, kTopkRunSmem, st>>>(Xa, a_rows, Wl, n, (int)begin, d, Bp, tau, cnt, ovf, cand_sc, cand_id, cs, ci)
      // expected passes per row among a wave's 128 labels of this level: k (growth - 1) 128 / n
      const bool dense = (int64_t)k * (kTopkGrowth - 1) * 128 >= n;
      if (fp8 && first) ELMO_TOPK_FIRST(true);
      else if (first) ELMO_TOPK_FIRST(false);
      else if (fp8 && dense) ELMO_TOPK_FILTER_RUN(true, true);
      else if (fp8) ELMO_TOPK_FILTER_RUN(true, false);
      else if (dense) ELMO_TOPK_FILTER_RUN(false, true);
      else ELMO_TOPK_FILTER_RUN(false, false);
#undef ELMO_TOPK_FIRST
#undef ELMO_TOPK_FILTER_RUN
      if (int rc = topk_launch_error("top-k level kernel", err, errsz)) return rc;
      const bool last = end == L;
      k_topk_select<<<B, kThreads, 0, st>>>(tau, cnt, cand_sc, cand_id, k, last ? idx_out : nullptr, last ? score_out : nullptr,
                                            k_total, off, last ? ns : nullptr, last ? ni : nullptr);
      if (int rc = topk_launch_error("k_topk_select", err, errsz)) return rc;
    }
    // ---- fallback for rows whose candidate list overflowed (does nothing when no row is flagged)
    if (fp8) k_topk_chunk<true><<<tiles_b * P, kThreads, kTopkSmem, st>>>(Xa, a_rows, W, L, d, k, P, tps, part_sc, part_id, ovf, B, cs, ci);
    else k_topk_chunk<false><<<tiles_b * P, kThreads, kTopkSmem, st>>>(Xa, a_rows, W, L, d, k, P, tps, part_sc, part_id, ovf, B, cs, ci);
    if (int rc = topk_launch_error("k_topk_chunk", err, errsz)) return rc;
    int N2 = 2;
    while (N2 < P * k) N2 <<= 1;
    k_topk_merge<<<B, kThreads, (size_t)N2 * 8, st>>>(part_sc, part_id, P, k, N2, idx_out, score_out, ovf, k_total, off, ns, ni);
    if (int rc = topk_launch_error("k_topk_merge", err, errsz)) return rc;
  }
  return 0;
}

}  // namespace elmo
