// HIP kernels of the ELMO head step for gfx950 (Algorithm 1 of the paper, one label chunk at a
// time): logits + sigmoid-BCE gradient epilogue, input-gradient product, fused weight-gradient +
// SGD + Kahan + stochastic-rounding update, and the small per-step helpers around them.
#pragma once
#include "numerics.h"
#include "tiles.h"

namespace elmo {

// ---------------------------------------------------------------------------------------------
// Small helpers
// ---------------------------------------------------------------------------------------------
__device__ inline uint32_t pack2_bf16(float a, float b) {   // hardware round-to-nearest-even
  bf16x2 v;
  v[0] = (__bf16)a;
  v[1] = (__bf16)b;
  return __builtin_bit_cast(uint32_t, v);
}
// sigmoid on the transcendental unit: v_exp_f32 and v_rcp_f32 (about 1 ulp each), five instructions.
// The result is rounded to BF16 right away, so the last FP32 bits only matter next to a BF16 tie.
__device__ inline float sigmoidf_fast(float z) {
  return __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.44269504088896341f * z));
}
__device__ inline float softplusf_fast(float z) { return fmaxf(z, 0.0f) + __logf(1.0f + __expf(-fabsf(z))); }

template <int NW> __device__ inline float block_sum(float v, float* red /*>= NW floats of LDS*/) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_down(v, o, 64);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  if (lane == 0) red[w] = v;
  __syncthreads();
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < NW; ++i) s += red[i];
  return s;
}

__global__ void __launch_bounds__(kThreads) k_fill_u32(uint32_t* __restrict__ p, size_t n, uint32_t v) {
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads) p[i] = v;
}

// Step set-up of the inputs (Algorithm 1: "X.t().to(float8_e4m3fn)"): the E4M3 cast Xq [Bp, d]
// used by the logits product and the transposed BF16 copy XT [d, Bp] used by the weight-gradient
// product; rows B..Bp-1 are zero padding.  Either output may be absent.
__global__ void __launch_bounds__(kThreads) k_prep_x(const uint16_t* __restrict__ X, int B, int Bp, int d,
                                                     uint8_t* __restrict__ Xq, uint16_t* __restrict__ XT) {
  const size_t n = (size_t)Bp * d;
  for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads) {
    const int b = (int)(i / d), j = (int)(i % d);
    const uint32_t bits = b < B ? X[i] : 0u;
    if (Xq) Xq[i] = (uint8_t)e4m3_rne(bf16_decode(bits));
    if (XT) XT[(size_t)j * Bp + b] = (uint16_t)bits;
  }
}

// k_prep_x plus the clearing of the step's scratch (input-gradient partial sums, bin counters,
// validation flag) in one launch: the small heads are bound by the number of launches.
__global__ void __launch_bounds__(kThreads) k_step_setup(const uint16_t* __restrict__ X, int B, int Bp, int d,
                                                         uint8_t* __restrict__ Xq, uint16_t* __restrict__ XT,
                                                         uint32_t* __restrict__ dx_words, size_t n_dx, uint32_t* __restrict__ cnt,
                                                         size_t n_cnt, uint32_t* __restrict__ flag) {
  const size_t n = (size_t)Bp * d, stride = (size_t)gridDim.x * kThreads, t0 = (size_t)blockIdx.x * kThreads + threadIdx.x;
  for (size_t i = t0; i < n; i += stride) {
    const int b = (int)(i / d), j = (int)(i % d);
    const uint32_t bits = b < B ? X[i] : 0u;
    if (Xq) Xq[i] = (uint8_t)e4m3_rne(bf16_decode(bits));
    XT[(size_t)j * Bp + b] = (uint16_t)bits;
  }
  for (size_t i = t0; i < n_dx; i += stride) dx_words[i] = 0u;
  for (size_t i = t0; i < n_cnt; i += stride) cnt[i] = 0u;
  if (flag && t0 == 0) *flag = 0u;
}

// ---------------------------------------------------------------------------------------------
// Per-batch label index: the positives (CSR by sample) regrouped by 128-label tile, so that the
// logits epilogue of a tile finds its few positives with two loads (Algorithm 1 filters the
// COO pairs of each chunk; here the filter is a counting sort done once per step).
// ---------------------------------------------------------------------------------------------
// Eight lanes share a sample row (its positives are few, and one lane per row would walk them as a
// chain of dependent loads).  Label ids sorted by falling frequency put most positives of a batch
// into the first few bins; atomics on one address serialise in L2, so every workgroup first counts
// the bins below kHotBins in LDS and touches each of those global counters once.
constexpr int kRowLanes = 8;
constexpr int kHotBins = 2048;                                   // labels 0 .. 262143
__global__ void __launch_bounds__(kThreads) k_label_hist(const int* __restrict__ indptr, const int* __restrict__ indices,
                                                         int B, int64_t L, int64_t nnz, int* __restrict__ cnt,
                                                         int* __restrict__ bad) {
  __shared__ int hot[kHotBins];
  for (int i = threadIdx.x; i < kHotBins; i += kThreads) hot[i] = 0;
  __syncthreads();
  const int t = blockIdx.x * kThreads + threadIdx.x;
  const int b = t / kRowLanes, sub = t % kRowLanes;
  if (b < B) {
    const int p0 = indptr[b], p1 = indptr[b + 1];
    if (p0 < 0 || p1 < p0 || p1 > nnz) {
      if (bad && sub == 0) atomicOr(bad, 1);
    } else {
      for (int p = p0 + sub; p < p1; p += kRowLanes) {
        const int l = indices[p];
        const bool in_range = l >= 0 && l < L;
        if (bad && (!in_range || (p > p0 && l <= indices[p - 1]))) atomicOr(bad, 2);   // out of range, or not strictly ascending
        if (in_range) {
          const int bin = l >> 7;
          if (bin < kHotBins) atomicAdd(&hot[bin], 1);
          else atomicAdd(&cnt[bin], 1);
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kHotBins; i += kThreads) {
    const int c = hot[i];
    if (c) atomicAdd(&cnt[i], c);
  }
}
// Exclusive scan of cnt[0..nb) into ptr[0..nb] (ptr[nb] = total) and cur[0..nb) = ptr.  One
// workgroup; the bins pass through LDS in segments so that global memory is read and written in
// whole lines (a thread's run of consecutive bins would otherwise touch 64 lines per load), every
// thread sums a run of a segment, the 1024 run totals are scanned in LDS.
constexpr int kScanRun = 15, kScanSeg = kScanRun * 1024;
__global__ void __launch_bounds__(1024) k_label_scan(const int* __restrict__ cnt, int nb, int* __restrict__ ptr, int* __restrict__ cur) {
  __shared__ int seg[kScanSeg];
  __shared__ int part[1024];
  const int tid = threadIdx.x;
  int carry = 0;
  for (int base = 0; base < nb; base += kScanSeg) {
    const int m = min(kScanSeg, nb - base);
    for (int i = tid; i < m; i += 1024) seg[i] = cnt[base + i];
    __syncthreads();
    const int i0 = min(tid * kScanRun, m), i1 = min(i0 + kScanRun, m);
    int sum = 0;
    for (int i = i0; i < i1; ++i) sum += seg[i];
    part[tid] = sum;
    __syncthreads();
    for (int o = 1; o < 1024; o <<= 1) {
      const int t = tid >= o ? part[tid - o] : 0;
      __syncthreads();
      part[tid] += t;
      __syncthreads();
    }
    int run = carry + part[tid] - sum;               // exclusive prefix of this thread's run
    for (int i = i0; i < i1; ++i) {
      const int v = seg[i];
      seg[i] = run;
      run += v;
    }
    carry += part[1023];
    __syncthreads();
    for (int i = tid; i < m; i += 1024) {
      const int v = seg[i];
      ptr[base + i] = v;
      cur[base + i] = v;
    }
    __syncthreads();
  }
  if (tid == 0) ptr[nb] = carry;
}
// Positives into their bins.  For the bins below kHotBins a workgroup ranks its positives in LDS,
// reserves one range per bin with a single global atomic and then writes; a thread keeps up to
// four such positives in registers between the two phases, anything beyond goes the direct way.
__global__ void __launch_bounds__(kThreads) k_label_scatter(const int* __restrict__ indptr, const int* __restrict__ indices,
                                                            int B, int64_t L, int64_t nnz, int* __restrict__ cur,
                                                            int2* __restrict__ pos) {
  __shared__ int hot[kHotBins];
  for (int i = threadIdx.x; i < kHotBins; i += kThreads) hot[i] = 0;
  __syncthreads();
  const int t = blockIdx.x * kThreads + threadIdx.x;
  const int b = t / kRowLanes, sub = t % kRowLanes;
  int lab[4] = {-1, -1, -1, -1}, rank[4] = {0, 0, 0, 0};
  if (b < B) {
    const int p0 = indptr[b], p1 = indptr[b + 1];
    if (!(p0 < 0 || p1 < p0 || p1 > nnz)) {
      int kept = 0;
      for (int p = p0 + sub; p < p1; p += kRowLanes) {
        const int l = indices[p];
        if (l < 0 || l >= L) continue;
        const int bin = l >> 7;
        if (bin < kHotBins && kept < 4) {
          const int r = atomicAdd(&hot[bin], 1);
#pragma unroll
          for (int k = 0; k < 4; ++k)
            if (k == kept) { lab[k] = l; rank[k] = r; }
          ++kept;
        } else {
          const int slot = atomicAdd(&cur[bin], 1);
          if (slot < nnz) pos[slot] = make_int2(l, b);
        }
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kHotBins; i += kThreads) {
    const int c = hot[i];
    hot[i] = c ? atomicAdd(&cur[i], c) : 0;          // first slot of this workgroup's range in bin i
  }
  __syncthreads();
#pragma unroll
  for (int k = 0; k < 4; ++k)
    if (lab[k] >= 0) {
      const int slot = hot[lab[k] >> 7] + rank[k];
      if (slot < nnz) pos[slot] = make_int2(lab[k], b);
    }
}

// ---------------------------------------------------------------------------------------------
// The three matrix products share one shape: 512-thread workgroups (8 waves as 4 x 2, each wave a
// 64 x 128 block of 32x32 MFMA tiles) computing a 256 x 256 output tile, operands streamed by
// asynchronous global->LDS loads through a ring of LDS stages (tiles.h, ring_pipeline_pp).  One
// workgroup per CU.  On this part the matrix cores and the L2->LDS fill do not overlap for free:
// a tile of this size halves the fill traffic per flop of a 256 x 128 tile, and the ping-pong
// issue order of the ring hides most of what is left.
// ---------------------------------------------------------------------------------------------
// How the input-gradient product splits a slab's loads between the early and the late waves
// (tiles.h, ring_stream_pp): uneven = three quarters early; late issue after this many quarters of
// the slab's MFMAs (issuing after one or three quarters was never better than after two).  The
// update product uses the paced ring instead (ring_pipeline_paced).
constexpr bool kDxUneven = true;
constexpr int kDxLateAfter = 2;
constexpr int kGemmThreads = 512;
constexpr int kGemmWaves = 8;
constexpr int kStages = 3;                                       // ring depth of the small-batch kernel
constexpr int kWideRingBytes = 2 * (256 + 256) * 128;            // K-contiguous operands, 128-byte slabs, 2 stages

// Register fragments of one step of a product: FM x FN blocks of 32 x 32 outputs.
template <int FM, int FN> struct FragBF16 { bf16x8 a[FM], b[FN]; };
template <int FM, int FN> struct FragFP8 { i32x8 a[FM], b[FN]; };

template <int FN> __device__ inline void zero_acc(f32x16 (&acc)[2][FN]) {
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;
}

// Classifier dropout on a weight slab that has landed in LDS (appendix "Low-Memory Dropout for
// Classifier": mask after the load, before the product).  The slab is ROWS weight rows of ROWB
// bytes of consecutive columns in the tile_off<ROWB> layout; blk0 is the mask block of its first
// 16 elements and blk_stride the mask blocks per weight row (d / 16).  Every thread draws whole
// mask blocks and zeroes the dropped elements in place.
template <int ROWS, int ROWB, bool FP8>
__device__ __forceinline__ void drop_slab(char* tile, uint64_t blk0, uint32_t blk_stride, uint64_t seed, uint64_t step,
                                          uint32_t thresh, int tid) {
  constexpr int UPR = ROWB / (FP8 ? 16 : 32);                  // mask blocks per slab row
  static_assert((ROWS * UPR) % kGemmThreads == 0, "slab size");
  const uint32_t tb = thresh * 0x01010101u;
#pragma unroll
  for (int u0 = 0; u0 < ROWS * UPR; u0 += kGemmThreads) {
    const int u = u0 + tid, r = u / UPR, k = u % UPR;
    const U4 rb = drop_block(blk0 + (uint64_t)r * blk_stride + k, seed, step);
    if (FP8) {
      u32x4* p = reinterpret_cast<u32x4*>(tile + tile_off<ROWB>(r, k));
      u32x4 w = *p;
      w[0] &= keep_bytes(rb.x, tb);
      w[1] &= keep_bytes(rb.y, tb);
      w[2] &= keep_bytes(rb.z, tb);
      w[3] &= keep_bytes(rb.w, tb);
      *p = w;
    } else {
      // byte mask -> one 16-bit mask per element (v_perm_b32 doubles each byte)
      u32x4* p0 = reinterpret_cast<u32x4*>(tile + tile_off<ROWB>(r, 2 * k));
      u32x4* p1 = reinterpret_cast<u32x4*>(tile + tile_off<ROWB>(r, 2 * k + 1));
      u32x4 a = *p0, b = *p1;
      uint32_t m = keep_bytes(rb.x, tb);
      a[0] &= __builtin_amdgcn_perm(m, m, 0x01010000u);
      a[1] &= __builtin_amdgcn_perm(m, m, 0x03030202u);
      m = keep_bytes(rb.y, tb);
      a[2] &= __builtin_amdgcn_perm(m, m, 0x01010000u);
      a[3] &= __builtin_amdgcn_perm(m, m, 0x03030202u);
      m = keep_bytes(rb.z, tb);
      b[0] &= __builtin_amdgcn_perm(m, m, 0x01010000u);
      b[1] &= __builtin_amdgcn_perm(m, m, 0x03030202u);
      m = keep_bytes(rb.w, tb);
      b[2] &= __builtin_amdgcn_perm(m, m, 0x01010000u);
      b[3] &= __builtin_amdgcn_perm(m, m, 0x03030202u);
      *p0 = a;
      *p1 = b;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Logits + fused epilogue (Algorithm 1: matmul_fp8, sigmoid_, "-= 1" at the positives).
// One workgroup computes a 256 (samples) x 256 (labels) tile of Z = Xq W_c^T with FP32
// accumulation over the full embedding width, then G = sigmoid(Z) - Y, and stores G^T[l][b] as
// BF16 (labels x batch, the layout the paper's logits buffer has).  Z never reaches memory.
// FP8: both operands E4M3, v_mfma_f32_32x32x64_f8f6f4.  BF16: v_mfma_f32_32x32x16_bf16.
// The positives of the tile's two 128-label bins are turned into a bit mask in LDS before the K
// loop; afterwards every wave finishes its accumulators in registers (sigmoid, minus the mask
// bit, BF16), transposes its block through a private LDS area and stores 128-byte segments of
// G^T rows, without a workgroup barrier.
// Rows of G^T between n and the next multiple of 128 are written as zeros (the input-gradient
// product reads whole 64-label slabs).
// ---------------------------------------------------------------------------------------------
// TB x TB output tiles: TB = 256, or 128 for padded batches of at most 128 rows, where half of a
// 256-row tile would be padding and the kernel is bound by the stream of W: 128 x 128 tiles need
// 66 KiB of LDS, so two workgroups share a CU and one's epilogue overlaps the other's loads.
constexpr int kGtPitch = 136;                                                        // bytes per staged G^T row segment of 64 samples (odd multiple of 8)
template <int TB> constexpr int logits_ring_bytes() { return 2 * (TB + TB) * 128; }
template <int TB> constexpr int logits_stage_bytes() { return TB * (TB / 64) * kGtPitch; }   // 8 waves x (their label rows) x pitch
template <int TB> constexpr int logits_mask_offset() {                              // positives mask: behind ring and G^T stages
  return logits_stage_bytes<TB>() > logits_ring_bytes<TB>() ? logits_stage_bytes<TB>() : logits_ring_bytes<TB>();
}
template <int TB> constexpr int logits_smem() { return logits_mask_offset<TB>() + TB * (TB / 32) * 4 + 32; }

// One half (0 or 1) of the product of a 128-byte K slab of the logits tile: A = TB sample rows,
// B = TB label rows, K-contiguous in LDS.  Wave (wm, wn) owns samples 64 wm .. +63 and labels
// 32 FN wn .. +32 FN - 1; acc[i][j] is its 32 x 32 block (i, j).
template <bool FP8, int FN>
__device__ __forceinline__ void logits_slab_product(const char* sa, const char* sb, int half, int wm, int wn, int lane,
                                                    f32x16 (&acc)[2][FN]) {
  if (FP8) {
    i32x8 a[2], b[FN];
#pragma unroll
    for (int i = 0; i < 2; ++i) a[i] = frag_fp8(sa, wm * 64 + 32 * i, half, lane);
#pragma unroll
    for (int j = 0; j < FN; ++j) b[j] = frag_fp8(sb, wn * 32 * FN + 32 * j, half, lane);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a[i], b[j], acc[i][j], 0, 0, 0, 0, 0, 0);
  } else {
#pragma unroll
    for (int kk = 2 * half; kk < 2 * half + 2; ++kk) {
      bf16x8 a[2], b[FN];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = frag_bf16(sa, wm * 64 + 32 * i, kk, lane);
#pragma unroll
      for (int j = 0; j < FN; ++j) b[j] = frag_bf16(sb, wn * 32 * FN + 32 * j, kk, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  }
}

// Z tile = Xa[TB rows] . Wc[TB rows]^T over the full embedding width (rowb bytes per row), FP32
// accumulators.  Waves as (8 / WGN) x WGN with WGN = 2 (TB = 256, 64 x 128 per wave) or 4
// (TB = 128, 64 x 32 per wave).
template <bool FP8, int TB, int FN, class Prep = NoPrep>
__device__ __forceinline__ void logits_tile_product(const char* __restrict__ Xa, int a_valid, const char* __restrict__ Wc, int w_valid,
                                                    size_t rowb, char* smem, int wave, int lane, f32x16 (&acc)[2][FN],
                                                    Prep&& prep = Prep{}) {
  constexpr int WGN = TB / 32 / FN;
  static_assert(WGN == (TB == 256 ? 2 : 4), "wave layout");
  const int wm = wave / WGN, wn = wave % WGN;
  zero_acc(acc);
  ring_pipeline_pp<TB, 128, TB, 128, 2, kGemmWaves, true>(
      Xa, rowb, a_valid, 0, 128, 8, Wc, rowb, w_valid, 0, 128, 8, (int)(rowb >> 7), smem, wave, lane,
      [&](const char* sa, const char* sb, int q0, int) { logits_slab_product<FP8, FN>(sa, sb, q0 >> 1, wm, wn, lane, acc); },
      static_cast<Prep&&>(prep));
}

// DROP: the W slabs are masked in LDS as they land (drop_slab) and Z is scaled by 1 / (1 - p);
// elem0 = flat index of the chunk's first weight element.
template <bool FP8, bool LOSS, int TB, bool DROP>
__global__ void __launch_bounds__(kGemmThreads, TB == 256 ? 1 : 2)
k_logits(const char* __restrict__ Xa, int a_rows, const char* __restrict__ Wc, int n, int d, int Bp, int B,
         uint16_t* __restrict__ Gt, const int* __restrict__ binptr, const int2* __restrict__ pos, int tile0,
         float* __restrict__ loss_slots, uint64_t seed, uint64_t step, uint64_t elem0, DropArgs dr) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int WGN = TB == 256 ? 2 : 4, FN = TB / 32 / WGN;   // waves along the labels, 32-label blocks per wave
  constexpr int MW = TB / 32;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave / WGN, wn = wave % WGN;
  const int tiles_b = (Bp + TB - 1) / TB;
  const int wg = xcd_logical_id(blockIdx.x, gridDim.x);
  const int lt = wg / tiles_b, bt = wg % tiles_b;
  const int b0 = bt * TB, l0 = lt * TB;
  const size_t rowb = (size_t)d * (FP8 ? 1 : 2);

  uint32_t* ym = reinterpret_cast<uint32_t*>(smem + logits_mask_offset<TB>());   // [TB labels][MW] bits over the samples
  float* red = reinterpret_cast<float*>(smem + logits_mask_offset<TB>() + TB * MW * 4);
  const int rows_out = min(TB, ((n - l0 + 127) >> 7) << 7);              // rows of G^T this tile writes
  const int gt0 = tile0 + lt * (TB / 128);                               // first of the tile's one or two bins

  // ---- positives of this tile's bins that fall into this batch tile -> bit mask.  The mask lives
  // behind the ring, so it is built first: its loads overlap the first slabs' way in, and the K
  // loop's barriers publish it.
  for (int i = tid; i < TB * MW; i += kGemmThreads) ym[i] = 0u;
  barrier_lds();
  {
    const int p0 = binptr[gt0], p1 = binptr[gt0 + (rows_out >> 7)];
    for (int p = p0 + tid; p < p1; p += kGemmThreads) {
      const int2 e = pos[p];
      const int lr_ = e.x - (gt0 << 7), br = e.y - b0;
      if (br >= 0 && br < TB && lr_ >= 0 && lr_ < TB) atomicOr(&ym[lr_ * MW + (br >> 5)], 1u << (br & 31));
    }
  }
  barrier_lds();

  f32x16 acc[2][FN];
  if constexpr (DROP) {
    const uint64_t blk_tile = (elem0 + (uint64_t)l0 * d) >> 4;     // mask block of the tile's first element
    logits_tile_product<FP8, TB, FN>(Xa + (size_t)b0 * rowb, a_rows - b0, Wc + (size_t)l0 * rowb, n - l0, rowb, smem, wave, lane, acc,
                                     [&](char* sb, int ks) {
                                       drop_slab<TB, 128, FP8>(sb, blk_tile + (uint64_t)ks * (FP8 ? 8 : 4), (uint32_t)d >> 4, seed,
                                                               step, dr.thresh, tid);
                                     });
  } else {
    logits_tile_product<FP8, TB, FN>(Xa + (size_t)b0 * rowb, a_rows - b0, Wc + (size_t)l0 * rowb, n - l0, rowb, smem, wave, lane, acc);
  }


  // ---- G = sigmoid(Z) - Y in registers, BF16, transposed through LDS, stored as row segments.
  // Each wave finishes its own 64-sample x (32 FN)-label block on its own: it stages the block in
  // a private LDS area ((32 FN) rows of 128 bytes, 4 samples = 8 bytes per write) and stores
  // 128-byte segments of G^T rows (8 lanes each).  No workgroup barrier: one wave's stores overlap
  // another's arithmetic, and this phase is bound by the vector ALU (two transcendental
  // instructions per value).
  // Positives are a handful per sample among millions of labels: a 32 x 32 block whose mask words
  // are all zero, in a tile without ragged rows, takes the short form (sigmoid only); the wave
  // votes, so the choice is uniform.
  constexpr int WROWS = 32 * FN;
  char* gts = smem + wave * (WROWS * kGtPitch);
  float loss = 0.0f;
  const bool tile_full = n - l0 >= TB;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int lw = 32 * j + (lane & 31), l = wn * WROWS + lw;
      const bool row_ok = l0 + l < n;
      const uint32_t ybits = (ym[l * MW + 2 * wm + i] >> (4 * (lane >> 5))) & 0x0F0F0F0Fu;
      const bool plain = !LOSS && tile_full && __builtin_amdgcn_ballot_w64(ybits != 0u) == 0ull;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int bw = 32 * i + 8 * q + 4 * (lane >> 5), b = wm * 64 + bw;
        float g[4];
        if (plain) {
#pragma unroll
          for (int e = 0; e < 4; ++e) g[e] = sigmoidf_fast(DROP ? acc[i][j][4 * q + e] * dr.scale : acc[i][j][4 * q + e]);
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float z = DROP ? acc[i][j][4 * q + e] * dr.scale : acc[i][j][4 * q + e];
            const float y = (float)((ybits >> (8 * q + e)) & 1u);
            g[e] = row_ok ? sigmoidf_fast(z) - y : 0.0f;
            if (LOSS) loss += (row_ok && b0 + b + e < B) ? softplusf_fast(z) - y * z : 0.0f;
          }
        }
        uint2 o;
        o.x = pack2_bf16(g[0], g[1]);
        o.y = pack2_bf16(g[2], g[3]);
        *reinterpret_cast<uint2*>(gts + lw * kGtPitch + bw * 2) = o;
      }
    }
  __builtin_amdgcn_s_waitcnt(0xC07F);              // this wave's LDS writes have completed (its lanes read each other's)
  asm volatile("" ::: "memory");
  if (b0 + wm * 64 < Bp) {
#pragma unroll
    for (int it = 0; it < WROWS * 8 / 64; ++it) {
      const int id = it * 64 + lane, r = id >> 3, sgm = id & 7;
      const int row = wn * WROWS + r;
      if (row < rows_out) {
        const uint2 lo = *reinterpret_cast<const uint2*>(gts + r * kGtPitch + sgm * 16);
        const uint2 hi = *reinterpret_cast<const uint2*>(gts + r * kGtPitch + sgm * 16 + 8);
        // streaming store: G^T is written once here and read by other kernels later (measured 157 -> 150 us
        // per chunk against a plain store; the same hint on the weight stores of the update kernels and on
        // the asynchronous loads changed nothing or made them slower)
        __builtin_nontemporal_store(u32x4{lo.x, lo.y, hi.x, hi.y}, reinterpret_cast<u32x4*>(Gt + (size_t)(l0 + row) * Bp + b0 + wm * 64 + sgm * 8));
      }
    }
  }
  if (LOSS) {
    const float s = block_sum<kGemmWaves>(loss, red);
    if (tid == 0) {
      loss_slots[(size_t)gt0 * tiles_b + bt] = s;                        // both bins' loss in the first bin's slot
      if (rows_out > 128) loss_slots[(size_t)(gt0 + 1) * tiles_b + bt] = 0.0f;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Input gradient (Algorithm 1: X_gradient += large_k_matmul(logits, W_i)), dX += G W_c with the
// weights as they are before this step's update.  The contraction runs over the labels; both
// operands are stored label-major, so fragments come from transposing LDS reads and E4M3
// weights are widened to BF16 in registers (no up-cast copy of W in memory).
// Workgroup = 256 samples x 256 embedding columns x one slice s of the chunk's labels; the FP32
// partial goes to dXacc[s] (owned by exactly this workgroup, so plain read-modify-write).
// Label rows beyond n inside the last 64-label slab are harmless: G^T holds zeros there and the
// weight rows are re-reads of row n-1.  Columns beyond d in the last column tile re-read the
// row's last 16 bytes and are not stored.
// ---------------------------------------------------------------------------------------------
// dst[32 x 32 block, row pitch d] += one 32x32 accumulator tile.  All sixteen loads are issued
// before the first store, so the read-modify-write costs one memory round trip, not sixteen.
__device__ inline void add_acc_to_global(float* __restrict__ dst, int d, int lane, const f32x16& acc) {
  float old[16];
#pragma unroll
  for (int v = 0; v < 16; ++v) old[v] = dst[(size_t)acc_row(v, lane) * d + (lane & 31)];
#pragma unroll
  for (int v = 0; v < 16; ++v) dst[(size_t)acc_row(v, lane) * d + (lane & 31)] = old[v] + acc[v];
}

// ring stage: [G^T slab 64 labels x 256 samples (512-byte rows) | W slab 64 labels x 256 columns]
template <bool FP8> constexpr int dx_stages() { return FP8 ? 3 : 2; }
template <bool FP8> constexpr int dx_smem_bytes() { return dx_stages<FP8>() * (64 * 512 + 64 * (FP8 ? 256 : 512)); }

template <bool FP8, bool DROP>
__global__ void __launch_bounds__(kGemmThreads, 1)
k_dx(const char* __restrict__ Gt, const char* __restrict__ Wc, float* __restrict__ dXacc, int n, int d, int Bp,
     int Bp256, int S, uint64_t seed, uint64_t step, uint64_t elem0, DropArgs dr) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int ESZ = FP8 ? 1 : 2, WROWB = 256 * ESZ;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), wm = wave >> 1, wn = wave & 1;
  const int tiles_b = Bp256 >> 8, tiles_j = (d + 255) >> 8;
  const int wg = xcd_logical_id(blockIdx.x, gridDim.x);
  const int jt = wg % tiles_j, bt = (wg / tiles_j) % tiles_b, s = wg / (tiles_j * tiles_b);
  const int b0 = bt << 8, j0 = jt << 8;
  const int ksteps = (n + 63) >> 6, per = (ksteps + S - 1) / S;
  const int ks0 = s * per, ks1 = min(ks0 + per, ksteps);
  if (ks0 >= ks1) return;
  const size_t strideA = (size_t)Bp * 2, strideB = (size_t)d * ESZ;

  f32x16 acc[2][4];
  zero_acc(acc);
  auto product = [&](const char* sa, const char* sb, int q0, int q1) {
#pragma unroll
    for (int kk = q0; kk < q1; ++kk) {
      bf16x8 a[2], b[4];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = frag_tr_bf16<512>(sa, 16 * kk, wm * 64 + 32 * i, lane);
#pragma unroll
      for (int j = 0; j < 4; ++j)
        b[j] = FP8 ? frag_tr_fp8<WROWB>(sb, 16 * kk, wn * 128 + 32 * j, lane)
                   : frag_tr_bf16<WROWB>(sb, 16 * kk, wn * 128 + 32 * j, lane);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };
  const char* ga = Gt + (size_t)ks0 * 64 * strideA + (size_t)b0 * 2;
  const char* gb = Wc + (size_t)ks0 * 64 * strideB + (size_t)j0 * ESZ;
  const int va0 = (ksteps - ks0) * 64;                 // zero rows of G^T past n are real
  const int chunks_b = min(256, d - j0) * ESZ / 16;
  if constexpr (DROP) {
    // the same masked weights as in the logits product (appendix "Low-Memory Dropout for Classifier")
    const uint64_t blk_first = (elem0 + (uint64_t)ks0 * 64 * d + j0) >> 4;
    ring_pipeline_pp<64, 512, 64, WROWB, dx_stages<FP8>(), kGemmWaves, kDxUneven, kDxLateAfter>(
        ga, strideA, va0, 64, 64 * strideA, 32, gb, strideB, n - ks0 * 64, 64, 64 * strideB, chunks_b, ks1 - ks0, smem, wave, lane,
        product, [&](char* sb, int ks) {
          drop_slab<64, WROWB, FP8>(sb, blk_first + (uint64_t)ks * 4 * d, (uint32_t)d >> 4, seed, step, dr.thresh, tid);
        });
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] *= dr.scale;
  } else {
    ring_pipeline_pp<64, 512, 64, WROWB, dx_stages<FP8>(), kGemmWaves, kDxUneven, kDxLateAfter>(
        ga, strideA, va0, 64, 64 * strideA, 32, gb, strideB, n - ks0 * 64, 64, 64 * strideB, chunks_b, ks1 - ks0, smem, wave, lane,
        product);
  }
  float* out = dXacc + (size_t)s * Bp256 * d;
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = j0 + wn * 128 + 32 * j;
      if (col < d) add_acc_to_global(out + (size_t)(b0 + wm * 64 + 32 * i) * d + col, d, lane, acc[i][j]);
    }
}

// dX_out = BF16(sum over label slices of the FP32 partials); loss_out = sum of the tile losses.
__global__ void __launch_bounds__(kThreads) k_finalize(const float* __restrict__ dXacc, int S, int Bp256, int B, int d,
                                                       uint16_t* __restrict__ dX_out, const float* __restrict__ loss_slots,
                                                       int nslots, float* __restrict__ loss_out) {
  __shared__ float red[4];
  if (dX_out) {
    const size_t n = (size_t)B * d, plane = (size_t)Bp256 * d;
    for (size_t i = (size_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (size_t)gridDim.x * kThreads) {
      float s = 0.0f;
      for (int k = 0; k < S; ++k) s += dXacc[k * plane + i];
      dX_out[i] = (uint16_t)bf16_rne(s);
    }
  }
  if (loss_out && blockIdx.x == 0) {
    float s = 0.0f;
    for (int i = threadIdx.x; i < nslots; i += kThreads) s += loss_slots[i];
    const float t = block_sum<4>(s, red);
    if (threadIdx.x == 0) *loss_out = t;
  }
}

// ---------------------------------------------------------------------------------------------
// Fused weight gradient + SGD + (Kahan) + rounding, in place (Algorithm 1, fuse_update).
// One workgroup owns a 256 (labels) x 256 (columns) tile of W_c: grad = G^T X accumulated in FP32
// over the whole batch on the BF16 matrix cores, then per element the FP32 update of
// numerics.h, rounded stochastically (Eq. 1) or to nearest, written back in the storage format.
// The weight gradient only ever exists as MFMA accumulators and one LDS tile (staged in two
// halves of 128 columns).
// ---------------------------------------------------------------------------------------------
constexpr int kGPitch = 132;                                     // floats per staged gradient row of 128 columns
constexpr int kUpdateEpiBytes = kGemmWaves * 32 * kGPitch * 4;   // one 32 x 128 FP32 half-block per wave
constexpr int kUpdateSmem = kUpdateEpiBytes > kWideRingBytes ? kUpdateEpiBytes : kWideRingBytes;

// Sixteen consecutive elements of one weight row: storage bits in, storage bits out.
// E4M3: w[0..3] hold 4 codes each; BF16: w[0..7] hold 2 patterns each.  c[0..7]: BF16 compensation.
// WD = false ignores wd (the two extra operations of the decay are not even selected away).
template <int FMT, bool SR, bool KAHAN, bool WD>
__device__ inline void update16_wd(uint32_t (&w)[8], uint32_t (&c)[8], const float (&g)[16], float lr, float wd_, const U4 (&rb)[2]) {
  const float wd = WD ? wd_ : 0.0f;
  const uint32_t rw[8] = {rb[0].x, rb[0].y, rb[0].z, rb[0].w, rb[1].x, rb[1].y, rb[1].z, rb[1].w};
  if (FMT == FMT_E4M3) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      // four codes at a time: the packed conversion decodes two E4M3 bytes per instruction (exact)
      const f32x2 wlo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w[q], 1.0f, false);
      const f32x2 whi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w[q], 1.0f, true);
      const float wv[4] = {wlo[0], wlo[1], whi[0], whi[1]};
      uint32_t out = 0u;
      float y[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int i = 4 * q + e;
        const float gi = wd != 0.0f ? __fadd_rn(g[i], __fmul_rn(wd, wv[e])) : g[i];   // L2 weight decay as a gradient term
        const float u = __fmul_rn(lr, gi);
        float t;
        y[e] = 0.0f;
        if (KAHAN) {
          const float cv = u2f((i & 1) ? (c[i >> 1] & 0xFFFF0000u) : (c[i >> 1] << 16));
          y[e] = __fsub_rn(-u, cv);
          t = __fadd_rn(wv[e], y[e]);
        } else {
          t = __fsub_rn(wv[e], u);
        }
        if (SR) {
          const uint32_t rnd = (i & 1) ? (rw[i >> 1] & 0xFFFF0000u) : (rw[i >> 1] << 16);
          out = e4m3_sr_pack(t, rnd, out, e);
        } else {
          out |= e4m3_rne(t) << (8 * e);
        }
      }
      w[q] = out;
      if (KAHAN) {
        const f32x2 nlo = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(out, 1.0f, false);
        const f32x2 nhi = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(out, 1.0f, true);
        c[2 * q] = pack2_bf16(__fsub_rn(__fsub_rn(nlo[0], wv[0]), y[0]), __fsub_rn(__fsub_rn(nlo[1], wv[1]), y[1]));   // hardware round-to-nearest-even
        c[2 * q + 1] = pack2_bf16(__fsub_rn(__fsub_rn(nhi[0], wv[2]), y[2]), __fsub_rn(__fsub_rn(nhi[1], wv[3]), y[3]));
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      uint32_t wb = (w[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu;
      uint32_t cb = KAHAN ? (c[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu : 0u;
      const uint32_t r16 = SR ? ((rw[i >> 1] >> ((i & 1) * 16)) & 0xFFFFu) : 0u;
      update_element<FMT, SR, KAHAN>(wb, cb, g[i], lr, wd, r16);
      w[i >> 1] = (i & 1) ? (w[i >> 1] & 0x0000FFFFu) | (wb << 16) : (w[i >> 1] & 0xFFFF0000u) | wb;
      if (KAHAN) c[i >> 1] = (i & 1) ? (c[i >> 1] & 0x0000FFFFu) | (cb << 16) : (c[i >> 1] & 0xFFFF0000u) | cb;
    }
  }
}

// DROP: the weight gradient is that of the masked model: zero where the step's mask drops the
// element, scaled by 1 / (1 - p) elsewhere.
// WD: the update includes the weight-decay term (a template parameter because this phase is bound
// by the vector ALU: the common wd = 0 case should not compute the term and select it away).
template <int FMT, bool SR, bool KAHAN, bool DROP, bool WD>
__global__ void __launch_bounds__(kGemmThreads, 1)
k_update(const char* __restrict__ Gt, const char* __restrict__ XT, char* __restrict__ Wc, uint16_t* __restrict__ Cc,
         int n, int d, int Bp, float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0, DropArgs dr) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  constexpr int ESZ = FMT == FMT_E4M3 ? 1 : 2;
  constexpr int WQ = FMT == FMT_E4M3 ? 1 : 2;       // 16-byte loads per 16 weights
  // (the wave index is left a vector value here: with a scalar one, as in the other two products,
  // this kernel's K loop measured 9 % slower, 66.4 k against 60.4 k clocks per tile)
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  const int tiles_j = (d + 255) >> 8;
  const int wg = xcd_logical_id(blockIdx.x, gridDim.x);
  const int lt = wg / tiles_j, jt = wg % tiles_j;
  const int l0 = lt << 8, j0 = jt << 8;
  const size_t stride = (size_t)Bp * 2;
  // Every wave finishes its own 64 (labels) x 128 (columns) block of the tile on its own, in two
  // halves of 32 labels: per half the lane handles 4 passes x 16 consecutive columns of one row
  // (row = 8 pass + lane / 8; eight lanes cover the 128 columns of a row, i.e. whole 128-byte
  // lines of E4M3 weights -- halves of 64 columns measured 3.5 % slower for E4M3 with
  // compensation and 7 % faster for BF16).  The first half's weights (and compensation) are fetched before
  // the product, the second half's pass by pass while the first is being updated, so the
  // read-modify-write does not wait on memory.  A wave whose columns lie beyond d (the last
  // column tile of a d = 128 (mod 256) head) has nothing to update.
  const int wl0 = l0 + wm * 64, wj0 = j0 + wn * 128;
  const bool has_cols = wj0 < d;
  const int urow = lane >> 3, useg = lane & 7;
  u32x4 wreg[4][WQ];
  u32x4 creg[4][2];
  auto fetch = [&](int it, int half) {
    const int l = min(wl0 + 32 * half + it * 8 + urow, n - 1);
    const size_t eoff = (size_t)l * d + wj0 + useg * 16;
#pragma unroll
    for (int q = 0; q < WQ; ++q) wreg[it][q] = *reinterpret_cast<const u32x4*>(Wc + eoff * ESZ + 16 * q);
    if (KAHAN) {
      creg[it][0] = *reinterpret_cast<const u32x4*>(Cc + eoff);
      creg[it][1] = *reinterpret_cast<const u32x4*>(Cc + eoff + 8);
    }
  };
  if (has_cols) {   // passes 0 and 1 of the first half before the product, passes 2 and 3 right after it
#pragma unroll
    for (int it = 0; it < 2; ++it) fetch(it, 0);
  }

  f32x16 acc[2][4];
  zero_acc(acc);
  // K loop over the batch in slabs of 64 samples
  ring_pipeline_paced<256, 128, 256, 128, kGemmWaves, 4, 6, 8, FragBF16<2, 4>>(
      Gt + (size_t)l0 * stride, stride, n - l0, 0, 128, 8, XT + (size_t)j0 * stride, stride, d - j0, 0, 128, 8, Bp >> 6, smem, wave,
      lane,
      [&](FragBF16<2, 4>& f, const char* sa, const char* sb, int kk) {
#pragma unroll
        for (int i = 0; i < 2; ++i) f.a[i] = frag_bf16(sa, wm * 64 + 32 * i, kk, lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) f.b[j] = frag_bf16(sb, wn * 128 + 32 * j, kk, lane);
      },
      [&](const FragBF16<2, 4>& f, int i) {
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[i], f.b[j], acc[i][j], 0, 0, 0);
      });
  if (!has_cols) return;                             // after the ring's last barrier: no barrier follows
#pragma unroll
  for (int it = 2; it < 4; ++it) fetch(it, 0);

  // This wave's LDS area: a 32 x 128 FP32 half-block, [label][column], turns the MFMA layout into
  // 16 consecutive columns per lane.  Nothing below synchronises the workgroup.
  float* gs = reinterpret_cast<float*>(smem) + wave * (32 * kGPitch);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    asm volatile("" ::: "memory");
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) gs[acc_row(v, lane) * kGPitch + 32 * j + (lane & 31)] = acc[h][j][v];
    __builtin_amdgcn_s_waitcnt(0xC07F);              // the wave's own LDS writes (its lanes read each other's)
    asm volatile("" ::: "memory");

    // ---- per-element update
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      const int row = it * 8 + urow;
      const int l = wl0 + 32 * h + row;
      uint32_t w[8], c[8];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        w[q] = wreg[it][0][q];
        if (WQ == 2) w[4 + q] = wreg[it][WQ - 1][q];
        if (KAHAN) { c[q] = creg[it][0][q]; c[4 + q] = creg[it][1][q]; }
      }
      float g[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 t = *reinterpret_cast<const f32x4*>(gs + row * kGPitch + useg * 16 + 4 * q);
        g[4 * q] = t[0]; g[4 * q + 1] = t[1]; g[4 * q + 2] = t[2]; g[4 * q + 3] = t[3];
      }
      if (h == 0) fetch(it, 1);
      if (l >= n) continue;
      const size_t eoff = (size_t)l * d + wj0 + useg * 16;
      if (DROP) {
        const U4 mb = drop_block((elem0 + eoff) >> 4, seed, step);
        const uint32_t tb = dr.thresh * 0x01010101u;
        const uint32_t km[4] = {keep_bytes(mb.x, tb), keep_bytes(mb.y, tb), keep_bytes(mb.z, tb), keep_bytes(mb.w, tb)};
#pragma unroll
        for (int i = 0; i < 16; ++i) g[i] = ((km[i >> 2] >> (8 * (i & 3))) & 1u) ? g[i] * dr.scale : 0.0f;
      }
      U4 rb[2];
      if (SR) {
        const uint64_t blk = (elem0 + eoff) >> 3;
        rb[0] = sr_block(blk, seed, step);
        rb[1] = sr_block(blk + 1, seed, step);
      }
      update16_wd<FMT, SR, KAHAN, WD>(w, c, g, lr, wd, rb);
      char* wp = Wc + eoff * ESZ;
      *reinterpret_cast<u32x4*>(wp) = u32x4{w[0], w[1], w[2], w[3]};
      if (WQ == 2) *reinterpret_cast<u32x4*>(wp + 16) = u32x4{w[4], w[5], w[6], w[7]};
      if (KAHAN) {
        *reinterpret_cast<u32x4*>(Cc + eoff) = u32x4{c[0], c[1], c[2], c[3]};
        *reinterpret_cast<u32x4*>(Cc + eoff + 8) = u32x4{c[4], c[5], c[6], c[7]};
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Small batches (padded batch <= 128): input gradient and fused update in ONE pass over the
// weights.  At small batch the step is bound by memory traffic, and running the two products as
// separate kernels reads every weight twice; here a workgroup streams tiles of 32 labels x 256
// columns of W_c (and of the compensation) exactly once, and from each tile, while it sits in LDS,
// forms both  dX[:, cols] += G W_tile  (old weights, transposing reads)  and  grad = G^T X[:, cols]
// followed by the same per-element update as k_update.  Workgroup (g, c) owns column block c
// (256 columns) and the g-th contiguous range of label tiles of the chunk; its 128 x 256 slice of
// dX stays in registers over all its tiles and is added to dXacc[g] at the end (one owner).
// The X operand of the gradient product lives in registers for the whole kernel.
// Stage of the 3-deep ring: [W 32 x 256 el | G^T 32 x 256 B | comp 32 x 512 B].
// ---------------------------------------------------------------------------------------------
template <int FMT, bool KAHAN> constexpr int dxu_stage_bytes() {
  return 32 * 256 * (FMT == FMT_E4M3 ? 1 : 2) + 32 * 256 + (KAHAN ? 32 * 512 : 0);
}
constexpr int kDxuGsBytes = 32 * 260 * 4;
// With dropout one more W tile: the masked copy the input-gradient product reads (the update
// needs the stored weights, so the tile cannot be masked in place).
template <int FMT, bool KAHAN, bool DROP = false> constexpr int dxu_smem_bytes() {
  return kStages * dxu_stage_bytes<FMT, KAHAN>() + kDxuGsBytes + (DROP ? 32 * 256 * (FMT == FMT_E4M3 ? 1 : 2) : 0);
}

// The body is a separate inlined function with restrict-qualified parameters on purpose: inlining
// it tags every LDS access inside with alias information, without which the compiler puts a full
// vmcnt(0) wait in front of the transposing LDS reads (it cannot tell them from the asynchronous
// loads still in flight for later stages) and the ring stops prefetching.  The waits that are
// needed are the explicit ones below.
template <int FMT, bool SR, bool KAHAN, bool DX, bool WD, bool DROP>
__device__ __forceinline__ void dx_update_body(const char* __restrict__ Gt, const char* __restrict__ XT, char* __restrict__ Wc,
                                               uint16_t* __restrict__ Cc, float* __restrict__ dXacc, int n, int d, int Bp,
                                               float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0, int tiles_per_group,
                                               DropArgs dr, char* smem) {
  constexpr int ESZ = FMT == FMT_E4M3 ? 1 : 2;
  constexpr int WROWB = 256 * ESZ;
  constexpr int WBYTES = 32 * WROWB, GBYTES = 32 * 256, SBYTES = dxu_stage_bytes<FMT, KAHAN>();
  constexpr int LPS = WROWB / 256 + 1 + (KAHAN ? 2 : 0);     // asynchronous loads per wave and tile
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int C = d >> 8;
  const int wg = xcd_logical_id(blockIdx.x, gridDim.x);
  const int g = wg / C, c = wg % C;
  const int ntiles = (n + 31) >> 5;
  const int t0 = g * tiles_per_group, t1 = min(t0 + tiles_per_group, ntiles);
  if (t0 >= t1) return;
  const int j0 = c << 8;
  const size_t gstride = (size_t)Bp * 2;
  const int KS = Bp >> 4;                                   // k16 steps over the batch: 4 or 8
  char* ring = smem;
  float* gs = reinterpret_cast<float*>(smem + kStages * SBYTES);
  char* wmk = smem + kStages * SBYTES + kDxuGsBytes;          // DROP: masked copy of the current W tile

  // X^T fragments of this wave's 32 columns (B operand of grad = G^T X), resident for the kernel
  bf16x8 xt[8];
#pragma unroll
  for (int ks = 0; ks < 8; ++ks) {
    const int b = min(16 * ks + 8 * (lane >> 5), Bp - 8);
    xt[ks] = *reinterpret_cast<const bf16x8*>(XT + ((size_t)(j0 + 32 * wave + (lane & 31)) * Bp + b) * 2);
  }
  const int bt = wave & 3, jh = wave >> 2;                  // dX block of this wave: rows 32*bt.., columns 128*jh..
  f32x16 dxa[4];
#pragma unroll
  for (int t = 0; t < 4; ++t)
#pragma unroll
    for (int v = 0; v < 16; ++v) dxa[t][v] = 0.0f;

  auto issue = [&](int t) {
    char* st = ring + (t % kStages) * SBYTES;
    const int l0 = t << 5, valid = n - l0;
    dma_tile<32, WROWB, kGemmWaves>(Wc + ((size_t)l0 * d + j0) * ESZ, (size_t)d * ESZ, valid, st, wave, lane);
    // rows of G^T past n exist and hold zeros (written by the logits kernel): no clamping, so they add nothing to dX
    dma_tile<32, 256, kGemmWaves>(Gt + (size_t)l0 * gstride, gstride, 32, st + WBYTES, wave, lane, Bp >> 3);
    if (KAHAN)
      dma_tile<32, 512, kGemmWaves>(reinterpret_cast<const char*>(Cc) + ((size_t)l0 * d + j0) * 2, (size_t)d * 2, valid,
                                    st + WBYTES + GBYTES, wave, lane);
  };
  issue(t0);
  if (t0 + 1 < t1) issue(t0 + 1);
  for (int t = t0; t < t1; ++t) {
    // Tile t has landed once only younger operations are outstanding: tile t+1's loads and the
    // stores of tile t-1's update (vector loads and stores retire in issue order on gfx9-family
    // parts and share vmcnt).  Every wave issues NSTORE stores per full tile; the only tile that
    // can be ragged is the last one of the chunk, after which nothing is waited for.
    constexpr int NSTORE = ESZ + (KAHAN ? 2 : 0);
    if (t + 1 >= t1) wait_vmcnt<0>();
    else if (t == t0) wait_vmcnt<LPS>();
    else wait_vmcnt<LPS + NSTORE>();
    barrier_nofence();
    if (t + 2 < t1) issue(t + 2);
    const char* ws = ring + (t % kStages) * SBYTES;
    const char* gsl = ws + WBYTES;
    const char* cs = gsl + GBYTES;
    const int l0 = t << 5;
    const int l = tid >> 4, seg = tid & 15;                 // this thread's part of the tile: one label row, 16 consecutive columns
    const size_t eoff = (size_t)(l0 + l) * d + j0 + seg * 16;
    uint32_t w[8], km[4];
    auto load_w = [&]() {
      if (FMT == FMT_E4M3) {
        const u32x4 t4 = *reinterpret_cast<const u32x4*>(ws + tile_off<WROWB>(l, seg));
        w[0] = t4[0]; w[1] = t4[1]; w[2] = t4[2]; w[3] = t4[3];
      } else {
        const u32x4 ta = *reinterpret_cast<const u32x4*>(ws + tile_off<WROWB>(l, 2 * seg));
        const u32x4 tb = *reinterpret_cast<const u32x4*>(ws + tile_off<WROWB>(l, 2 * seg + 1));
        w[0] = ta[0]; w[1] = ta[1]; w[2] = ta[2]; w[3] = ta[3]; w[4] = tb[0]; w[5] = tb[1]; w[6] = tb[2]; w[7] = tb[3];
      }
    };
    if (DROP) {
      // the step's keep mask of these 16 elements (appendix "Low-Memory Dropout for Classifier"):
      // the input-gradient product reads a masked copy, the update below masks the gradient
      load_w();
      const U4 mb = drop_block((elem0 + eoff) >> 4, seed, step);
      const uint32_t tb = dr.thresh * 0x01010101u;
      km[0] = keep_bytes(mb.x, tb); km[1] = keep_bytes(mb.y, tb); km[2] = keep_bytes(mb.z, tb); km[3] = keep_bytes(mb.w, tb);
      if (DX) {
        if (FMT == FMT_E4M3) {
          *reinterpret_cast<u32x4*>(wmk + tile_off<WROWB>(l, seg)) = u32x4{w[0] & km[0], w[1] & km[1], w[2] & km[2], w[3] & km[3]};
        } else {
          u32x4 a, b;
#pragma unroll
          for (int q = 0; q < 2; ++q) {
            a[2 * q] = w[2 * q] & __builtin_amdgcn_perm(km[q], km[q], 0x01010000u);
            a[2 * q + 1] = w[2 * q + 1] & __builtin_amdgcn_perm(km[q], km[q], 0x03030202u);
            b[2 * q] = w[4 + 2 * q] & __builtin_amdgcn_perm(km[2 + q], km[2 + q], 0x01010000u);
            b[2 * q + 1] = w[5 + 2 * q] & __builtin_amdgcn_perm(km[2 + q], km[2 + q], 0x03030202u);
          }
          *reinterpret_cast<u32x4*>(wmk + tile_off<WROWB>(l, 2 * seg)) = a;
          *reinterpret_cast<u32x4*>(wmk + tile_off<WROWB>(l, 2 * seg + 1)) = b;
        }
        barrier_lds();
      }
    }
    const char* wdx = DROP ? wmk : ws;                      // what the input-gradient product reads

    // grad[32 labels x 32 columns of this wave] = G^T X
    f32x16 wa;
#pragma unroll
    for (int v = 0; v < 16; ++v) wa[v] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
      if (ks < KS) wa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag_bf16<256>(gsl, 0, ks, lane), xt[ks], wa, 0, 0, 0);
    // dX[32 samples x 128 columns of this wave] += G W_tile (weights as stored before the update)
    if (DX) {
#pragma unroll
      for (int kk = 0; kk < 2; ++kk) {
        const bf16x8 a = frag_tr_bf16<256>(gsl, 16 * kk, 32 * bt, lane);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const bf16x8 b = FMT == FMT_E4M3 ? frag_tr_fp8<WROWB>(wdx, 16 * kk, 128 * jh + 32 * q, lane)
                                           : frag_tr_bf16<WROWB>(wdx, 16 * kk, 128 * jh + 32 * q, lane);
          dxa[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, dxa[q], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int v = 0; v < 16; ++v) gs[acc_row(v, lane) * 260 + 32 * wave + (lane & 31)] = wa[v];
    barrier_lds();

    // per-element update
    if (l0 + l < n) {
      uint32_t cc[8];
      if (!DROP) load_w();
      if (KAHAN) {
        const u32x4 ta = *reinterpret_cast<const u32x4*>(cs + tile_off<512>(l, 2 * seg));
        const u32x4 tb = *reinterpret_cast<const u32x4*>(cs + tile_off<512>(l, 2 * seg + 1));
        cc[0] = ta[0]; cc[1] = ta[1]; cc[2] = ta[2]; cc[3] = ta[3]; cc[4] = tb[0]; cc[5] = tb[1]; cc[6] = tb[2]; cc[7] = tb[3];
      }
      float gr[16];
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 t4 = *reinterpret_cast<const f32x4*>(gs + l * 260 + seg * 16 + 4 * q);
        gr[4 * q] = t4[0]; gr[4 * q + 1] = t4[1]; gr[4 * q + 2] = t4[2]; gr[4 * q + 3] = t4[3];
      }
      if (DROP) {
#pragma unroll
        for (int i = 0; i < 16; ++i) gr[i] = ((km[i >> 2] >> (8 * (i & 3))) & 1u) ? gr[i] * dr.scale : 0.0f;
      }
      U4 rb[2];
      if (SR) {
        const uint64_t blk = (elem0 + eoff) >> 3;
        rb[0] = sr_block(blk, seed, step);
        rb[1] = sr_block(blk + 1, seed, step);
      }
      update16_wd<FMT, SR, KAHAN, WD>(w, cc, gr, lr, wd, rb);
      char* wp = Wc + eoff * ESZ;
      *reinterpret_cast<u32x4*>(wp) = u32x4{w[0], w[1], w[2], w[3]};
      if (ESZ == 2) *reinterpret_cast<u32x4*>(wp + 16) = u32x4{w[4], w[5], w[6], w[7]};
      if (KAHAN) {
        *reinterpret_cast<u32x4*>(Cc + eoff) = u32x4{cc[0], cc[1], cc[2], cc[3]};
        *reinterpret_cast<u32x4*>(Cc + eoff + 8) = u32x4{cc[4], cc[5], cc[6], cc[7]};
      }
    }
  }
  if (DX) {
    float* out = dXacc + (size_t)g * 128 * d;
    if (DROP) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int v = 0; v < 16; ++v) dxa[q][v] *= dr.scale;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
      add_acc_to_global(out + (size_t)(32 * bt) * d + j0 + 128 * jh + 32 * q, d, lane, dxa[q]);
  }
}

template <int FMT, bool SR, bool KAHAN, bool DX, bool WD, bool DROP>
__global__ void __launch_bounds__(kGemmThreads, 1)
k_dx_update(const char* __restrict__ Gt, const char* __restrict__ XT, char* __restrict__ Wc, uint16_t* __restrict__ Cc,
            float* __restrict__ dXacc, int n, int d, int Bp, float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0,
            int tiles_per_group, DropArgs dr) {
  extern __shared__ __attribute__((aligned(16))) char smem[];
  dx_update_body<FMT, SR, KAHAN, DX, WD, DROP>(Gt, XT, Wc, Cc, dXacc, n, d, Bp, lr, wd, seed, step, elem0, tiles_per_group, dr, smem);
}

// ---------------------------------------------------------------------------------------------
// Stand-alone quantiser (round to nearest even or stochastic rounding with the step's fields).
// ---------------------------------------------------------------------------------------------
template <int FMT, bool SR>
__global__ void __launch_bounds__(kThreads) k_quantize(const float* __restrict__ src, int64_t n, uint64_t seed, uint64_t step,
                                                       uint64_t first, void* __restrict__ dst) {
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
    const float t = src[i];
    uint32_t q;
    if (SR) {
      const uint64_t e = first + (uint64_t)i;
      const U4 rb = sr_block(e >> 3, seed, step);
      q = quant_sr<FMT>(t, sr_field(rb, (int)(e & 7)));
    } else {
      q = quant_rne<FMT>(t);
    }
    if (FMT == FMT_E4M3) reinterpret_cast<uint8_t*>(dst)[i] = (uint8_t)q;
    else reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)q;
  }
}

// Simulated (E, M) format: dst[i] = FP32 value of src[i] rounded to that format.
template <bool SR>
__global__ void __launch_bounds__(kThreads) k_quantize_em(const float* __restrict__ src, int64_t n, int E, int M, uint64_t seed,
                                                          uint64_t step, uint64_t first, float* __restrict__ dst) {
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int64_t)gridDim.x * kThreads) {
    int r16 = -1;
    if (SR) {
      const uint64_t e = first + (uint64_t)i;
      r16 = (int)sr_field(sr_block(e >> 3, seed, step), (int)(e & 7));
    }
    dst[i] = round_em(src[i], E, M, r16);
  }
}

// ---------------------------------------------------------------------------------------------
// AdamW with Kahan-compensated BF16 parameters (Section 4.1: Kahan summation for the encoder's
// parameters).  Elementwise, 8 elements per thread and pass; FP32 arithmetic, every operation
// rounded once; the moments are BF16 (stored round-to-nearest-even) or FP32.
//   m' = b1 m + o1 g;  v' = b2 v + (o2 g) g;  r = (m'/bc1) / (sqrt(v'/bc2) + eps) [+ wd p];  u = lr r
//   y = -u - c;  s = p + y;  p' = RNE_BF16(s);  c' = RNE_BF16((p' - p) - y)
// ---------------------------------------------------------------------------------------------
struct AdamArgs { float lr, b1, o1, b2, o2, bc1, bc2, eps, wd; };

__device__ inline void adamw_element(uint32_t& pb, uint32_t& cb, float& m, float& v, uint32_t gb, const AdamArgs& a) {
  const float p = bf16_decode(pb), c = bf16_decode(cb), g = bf16_decode(gb);
  m = __fadd_rn(__fmul_rn(a.b1, m), __fmul_rn(a.o1, g));
  v = __fadd_rn(__fmul_rn(a.b2, v), __fmul_rn(__fmul_rn(a.o2, g), g));
  const float mh = __fdiv_rn(m, a.bc1), vh = __fdiv_rn(v, a.bc2);
  float r = __fdiv_rn(mh, __fadd_rn(sqrtf(vh), a.eps));      // sqrtf and '/' are correctly rounded (the __fsqrt_rn intrinsic is not)
  if (a.wd != 0.0f) r = __fadd_rn(r, __fmul_rn(a.wd, p));
  const float u = __fmul_rn(a.lr, r);
  const float y = __fsub_rn(-u, c);
  const uint32_t q = bf16_rne(__fadd_rn(p, y));
  cb = bf16_rne(__fsub_rn(__fsub_rn(bf16_decode(q), p), y));
  pb = q;
}

template <bool STATE_BF16>
__global__ void __launch_bounds__(kThreads) k_kahan_adamw(uint16_t* __restrict__ P, uint16_t* __restrict__ C, void* __restrict__ Mv,
                                                          void* __restrict__ Vv, const uint16_t* __restrict__ G, int64_t n,
                                                          AdamArgs a) {
  const int64_t groups = n >> 3;
  for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < groups; i += (int64_t)gridDim.x * kThreads) {
    u32x4 p4 = reinterpret_cast<const u32x4*>(P)[i], c4 = reinterpret_cast<const u32x4*>(C)[i];
    const u32x4 g4 = reinterpret_cast<const u32x4*>(G)[i];
    float m[8], v[8];
    if (STATE_BF16) {
      const u32x4 m4 = reinterpret_cast<const u32x4*>(Mv)[i], v4 = reinterpret_cast<const u32x4*>(Vv)[i];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        m[e] = bf16_decode((m4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
        v[e] = bf16_decode((v4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu);
      }
    } else {
      const f32x4 ma = reinterpret_cast<const f32x4*>(Mv)[2 * i], mb = reinterpret_cast<const f32x4*>(Mv)[2 * i + 1];
      const f32x4 va = reinterpret_cast<const f32x4*>(Vv)[2 * i], vb = reinterpret_cast<const f32x4*>(Vv)[2 * i + 1];
#pragma unroll
      for (int e = 0; e < 4; ++e) { m[e] = ma[e]; m[4 + e] = mb[e]; v[e] = va[e]; v[4 + e] = vb[e]; }
    }
    uint32_t pn[8], cn[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pn[e] = (p4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
      cn[e] = (c4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu;
      adamw_element(pn[e], cn[e], m[e], v[e], (g4[e >> 1] >> (16 * (e & 1))) & 0xFFFFu, a);
    }
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      p4[q] = pn[2 * q] | (pn[2 * q + 1] << 16);
      c4[q] = cn[2 * q] | (cn[2 * q + 1] << 16);
    }
    reinterpret_cast<u32x4*>(P)[i] = p4;
    reinterpret_cast<u32x4*>(C)[i] = c4;
    if (STATE_BF16) {
      u32x4 m4, v4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        m4[q] = bf16_rne(m[2 * q]) | (bf16_rne(m[2 * q + 1]) << 16);
        v4[q] = bf16_rne(v[2 * q]) | (bf16_rne(v[2 * q + 1]) << 16);
      }
      reinterpret_cast<u32x4*>(Mv)[i] = m4;
      reinterpret_cast<u32x4*>(Vv)[i] = v4;
    } else {
      reinterpret_cast<f32x4*>(Mv)[2 * i] = f32x4{m[0], m[1], m[2], m[3]};
      reinterpret_cast<f32x4*>(Mv)[2 * i + 1] = f32x4{m[4], m[5], m[6], m[7]};
      reinterpret_cast<f32x4*>(Vv)[2 * i] = f32x4{v[0], v[1], v[2], v[3]};
      reinterpret_cast<f32x4*>(Vv)[2 * i + 1] = f32x4{v[4], v[5], v[6], v[7]};
    }
  }
  // the last n % 8 elements, one thread each
  const int64_t tail = (groups << 3) + (int64_t)blockIdx.x * kThreads + threadIdx.x;
  if (tail < n) {
    uint32_t pb = P[tail], cb = C[tail];
    float m = STATE_BF16 ? bf16_decode(reinterpret_cast<uint16_t*>(Mv)[tail]) : reinterpret_cast<float*>(Mv)[tail];
    float v = STATE_BF16 ? bf16_decode(reinterpret_cast<uint16_t*>(Vv)[tail]) : reinterpret_cast<float*>(Vv)[tail];
    adamw_element(pb, cb, m, v, G[tail], a);
    P[tail] = (uint16_t)pb;
    C[tail] = (uint16_t)cb;
    if (STATE_BF16) {
      reinterpret_cast<uint16_t*>(Mv)[tail] = (uint16_t)bf16_rne(m);
      reinterpret_cast<uint16_t*>(Vv)[tail] = (uint16_t)bf16_rne(v);
    } else {
      reinterpret_cast<float*>(Mv)[tail] = m;
      reinterpret_cast<float*>(Vv)[tail] = v;
    }
  }
}

}  // namespace elmo
