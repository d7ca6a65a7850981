// C ABI of the ELMO classifier-head library (see include/elmo_head.h) and its chunk scheduler.
#include "../../include/elmo_head.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.h"
#include "topk.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
  return code;
}

#define ELMO_HIP(call)                                                                       \
  do {                                                                                       \
    hipError_t e_ = (call);                                                                  \
    if (e_ != hipSuccess) return fail(-3, "%s failed: %s", #call, hipGetErrorString(e_));    \
  } while (0)

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }
inline int round_up(int x, int m) { return (x + m - 1) / m * m; }

// Workspace plan: byte offsets of every region (Section 4.2/4.4: only one chunk's logit-gradient
// buffer is ever alive; everything else is O(max_B * d) or O(L / 128) integers).
struct Plan {
  int64_t L; int d; int fmt; int64_t chunk; int maxB; int64_t max_nnz; uint32_t flags;
  int64_t kahan_rows;                   // leading label rows that carry compensation (0 without ELMO_KAHAN)
  float weight_decay;                   // L2 term of the update, 0 = none
  uint32_t drop_thresh;                 // classifier dropout: weights dropped with probability drop_thresh / 256, 0 = none
  int Bp_max, tiles_b_max, ntiles;      // padded batch, batch tiles, 128-label tiles of the whole head
  int dx_rows;                          // rows of FP32 input-gradient partials (slices x padded batch)
  size_t off_xq, off_xt, off_g, off_dx, off_loss, off_cnt, off_ptr, off_cur, off_pos, off_flag, off_topk, total;
  size_t W_bytes, comp_bytes;
};

int make_plan(int64_t L, int d, int fmt, int64_t chunk, int maxB, int64_t max_nnz, uint32_t flags, int64_t kahan_rows, Plan& p) {
  if (L < 1) return fail(-1, "L must be >= 1 (got %lld)", (long long)L);
  if (L > (int64_t)1 << 31) return fail(-1, "L must fit 31 bits (got %lld)", (long long)L);
  if (d < 128 || d % 128 != 0) return fail(-1, "d must be a positive multiple of 128 (got %d)", d);
  if (d > (1 << 20)) return fail(-1, "d must be at most 2^20 (got %d)", d);   // tile loads use 24-bit x 24-bit row offsets
  if (chunk < 1) return fail(-1, "chunk must be >= 1 (got %lld)", (long long)chunk);
  if (chunk > ((int64_t)1 << 30)) return fail(-1, "chunk too large (got %lld)", (long long)chunk);
  // The kernels work on whole 128-label tiles: a pass takes the next multiple of 128 labels.  The
  // results do not depend on the chunk size (every label's quantities depend on its own weight row
  // only), so the rounding only shows in the workspace size.
  chunk = (chunk + 127) / 128 * 128;
  if (maxB < 1 || maxB > 65536) return fail(-1, "max_B must be in [1, 65536] (got %d)", maxB);
  if (max_nnz < 1 || max_nnz > ((int64_t)1 << 30)) return fail(-1, "max_nnz must be in [1, 2^30] (got %lld)", (long long)max_nnz);
  if (fmt != ELMO_BF16 && fmt != ELMO_FP8_E4M3) return fail(-2, "unsupported weight_dtype %d", fmt);
  if (flags & ~(uint32_t)(ELMO_SR | ELMO_KAHAN | ELMO_VALIDATE)) return fail(-2, "unknown flag bits 0x%x", flags);
  if (kahan_rows < 0 || kahan_rows > L) return fail(-1, "kahan_rows must be in [0, L] (got %lld)", (long long)kahan_rows);
  if (!(flags & ELMO_KAHAN) && kahan_rows != 0) return fail(-1, "kahan_rows = %lld without ELMO_KAHAN", (long long)kahan_rows);
  if (kahan_rows != 0 && kahan_rows != L && kahan_rows % 128 != 0)
    return fail(-1, "kahan_rows must be 0 (all labels), L, or a multiple of 128 (got %lld)", (long long)kahan_rows);
  p.L = L; p.d = d; p.fmt = fmt; p.chunk = chunk; p.maxB = maxB; p.max_nnz = max_nnz; p.flags = flags;
  p.kahan_rows = (flags & ELMO_KAHAN) ? (kahan_rows ? kahan_rows : L) : 0;
  p.weight_decay = 0.0f;
  p.drop_thresh = 0;
  p.Bp_max = round_up(maxB, 64);
  p.tiles_b_max = (p.Bp_max + 255) / 256;      // 256-sample tiles of the matrix products
  p.ntiles = (int)((L + 127) / 128);
  const int tiles_j = (d + 255) / 256;           // 256-column tiles of the input-gradient product
  // slices x padded batch of the input-gradient partials: about one workgroup per CU
  p.dx_rows = std::min(65536 / tiles_j + 256 * p.tiles_b_max + 256, 64 * 256 * p.tiles_b_max);
  if (d % 256 == 0) p.dx_rows = std::max(p.dx_rows, std::max(1, 256 / (d / 256)) * 128);   // small-batch path: one 128-row slice per label group
  const int64_t chunk_eff = std::min<int64_t>(chunk, (L + 127) / 128 * 128);
  size_t o = 0;
  p.off_xq = o;  o += align256(fmt == ELMO_FP8_E4M3 ? (size_t)p.Bp_max * d : 0);
  p.off_xt = o;  o += align256((size_t)d * p.Bp_max * 2);
  p.off_g = o;   o += align256((size_t)chunk_eff * p.Bp_max * 2 + 4096);   // + slack: the last rows are read 512 bytes wide
  p.off_dx = o;  o += align256((size_t)p.dx_rows * d * 4);
  p.off_loss = o; o += align256((size_t)p.ntiles * p.tiles_b_max * 4);
  p.off_cnt = o; o += align256((size_t)(p.ntiles + 1) * 4);
  p.off_ptr = o; o += align256((size_t)(p.ntiles + 1) * 4);
  p.off_cur = o; o += align256((size_t)(p.ntiles + 1) * 4);
  p.off_pos = o; o += align256((size_t)max_nnz * 8);
  p.off_flag = o; o += 256;
  p.off_topk = o; o += align256(elmo::topk_scratch_bytes(p.Bp_max, chunk_eff));
  p.total = o;
  p.W_bytes = (size_t)L * d * (fmt == ELMO_FP8_E4M3 ? 1 : 2);
  p.comp_bytes = (size_t)p.kahan_rows * d * 2;
  return 0;
}

int check_launch(const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return fail(-3, "launch of %s failed: %s", what, hipGetErrorString(e));
  return 0;
}

}  // namespace

// Optional per-kernel-class timing: one event at every boundary between kernel classes of a
// step; a span is charged to the class launched after its first event.
enum { CLS_SETUP = 0, CLS_LOGITS, CLS_DX, CLS_UPDATE, CLS_FINAL, CLS_TOPK, CLS_END, CLS_COUNT = CLS_END };
struct Profiler {
  bool on = false;
  std::vector<hipEvent_t> ev;
  std::vector<int> cls;       // class of the span that starts at ev[i]; CLS_END closes a call
  size_t used = 0;
  void mark(hipStream_t st, int c) {
    if (!on) return;
    if (used == ev.size()) {
      hipEvent_t e;
      if (hipEventCreate(&e) != hipSuccess) { on = false; return; }
      ev.push_back(e);
      cls.push_back(c);
    }
    cls[used] = c;
    if (hipEventRecord(ev[used], st) != hipSuccess) { on = false; return; }
    ++used;
  }
};

struct elmo_head {
  Plan p;
  char* W; char* comp; char* ws;
  bool validated_step_pending;
  Profiler prof;
};

extern "C" {

const char* elmo_last_error(void) { return g_err; }

size_t elmo_logit_buffer_bytes(int64_t batch, int64_t labels) {
  return (batch < 0 || labels < 0) ? 0 : (size_t)batch * (size_t)labels * 2;
}

int elmo_head_sizes(int64_t L, int32_t d, int weight_dtype, int64_t chunk, int32_t max_B, int64_t max_nnz,
                    uint32_t flags, int64_t kahan_rows, size_t* W_bytes, size_t* comp_bytes, size_t* workspace_bytes) {
  Plan p;
  const int rc = make_plan(L, d, weight_dtype, chunk, max_B, max_nnz, flags, kahan_rows, p);
  if (rc) return rc;
  if (W_bytes) *W_bytes = p.W_bytes;
  if (comp_bytes) *comp_bytes = p.comp_bytes;
  if (workspace_bytes) *workspace_bytes = p.total;
  return 0;
}

int elmo_head_create(int64_t L, int32_t d, int weight_dtype, int64_t chunk, const elmo_head_opts* opts,
                     elmo_head_t** out) {
  if (!opts || !out) return fail(-1, "opts and out must not be NULL");
  Plan p;
  const int rc = make_plan(L, d, weight_dtype, chunk, opts->max_B, opts->max_nnz, opts->flags, opts->kahan_rows, p);
  if (rc) return rc;
  if (!(opts->weight_decay >= 0.0f) || opts->weight_decay > 1.0f) return fail(-1, "weight_decay must be in [0, 1] (got %g)", (double)opts->weight_decay);
  p.weight_decay = opts->weight_decay;
  if (!(opts->dropout_p >= 0.0f) || opts->dropout_p > 255.0f / 256.0f)
    return fail(-1, "dropout_p must be in [0, 255/256] (got %g)", (double)opts->dropout_p);
  p.drop_thresh = (uint32_t)lrintf(opts->dropout_p * 256.0f);
  if (!opts->W || opts->W_bytes < p.W_bytes) return fail(-1, "W buffer missing or smaller than %zu bytes", p.W_bytes);
  if ((opts->flags & ELMO_KAHAN) && (!opts->comp || opts->comp_bytes < p.comp_bytes))
    return fail(-1, "ELMO_KAHAN needs a compensation buffer of %zu bytes", p.comp_bytes);
  if (!opts->workspace || opts->workspace_bytes < p.total) return fail(-1, "workspace missing or smaller than %zu bytes", p.total);
  if (((uintptr_t)opts->W | (uintptr_t)opts->workspace | (uintptr_t)opts->comp) & 255)
    return fail(-1, "W, comp and workspace must be 256-byte aligned");
  elmo_head* h = new (std::nothrow) elmo_head;
  if (!h) return fail(-3, "out of host memory");
  h->p = p;
  h->W = (char*)opts->W;
  h->comp = (opts->flags & ELMO_KAHAN) ? (char*)opts->comp : nullptr;
  h->ws = (char*)opts->workspace;
  h->validated_step_pending = false;
  *out = h;
  return 0;
}

int elmo_head_destroy(elmo_head_t* h) {
  if (!h) return fail(-1, "NULL head");
  for (hipEvent_t e : h->prof.ev) (void)hipEventDestroy(e);
  delete h;
  return 0;
}

int elmo_head_profile(elmo_head_t* h, int enable) {
  if (!h) return fail(-1, "NULL head");
  h->prof.on = enable != 0;
  h->prof.used = 0;
  return 0;
}

int elmo_head_profile_read(elmo_head_t* h, double ms[6], int64_t launches[6]) {
  if (!h || !ms || !launches) return fail(-1, "NULL argument");
  Profiler& pr = h->prof;
  for (int i = 0; i < CLS_COUNT; ++i) { ms[i] = 0.0; launches[i] = 0; }
  if (pr.used) ELMO_HIP(hipEventSynchronize(pr.ev[pr.used - 1]));
  for (size_t i = 0; i + 1 < pr.used; ++i) {
    if (pr.cls[i] == CLS_END) continue;
    float t = 0.0f;
    ELMO_HIP(hipEventElapsedTime(&t, pr.ev[i], pr.ev[i + 1]));
    ms[pr.cls[i]] += t;
    launches[pr.cls[i]] += 1;
  }
  pr.used = 0;
  return 0;
}

void elmo_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]) {
  elmo::U4 c{ctr[0], ctr[1], ctr[2], ctr[3]};
  c = elmo::philox4x32_10(c, key[0], key[1]);
  out[0] = c.x; out[1] = c.y; out[2] = c.z; out[3] = c.w;
}

uint32_t elmo_dropout_keep16(uint64_t seed, uint64_t step, uint64_t block, uint32_t threshold) {
  const elmo::U4 b = elmo::drop_block(block, seed, step);
  const uint32_t tb = (threshold & 0xFFu) * 0x01010101u;
  const uint32_t w[4] = {b.x, b.y, b.z, b.w};
  uint32_t bits = 0;
  for (int i = 0; i < 16; ++i) bits |= ((elmo::keep_bytes(w[i >> 2], tb) >> (8 * (i & 3))) & 1u) << i;
  return bits;
}

int elmo_quantize(const float* src, int64_t n, int dtype, int mode, uint64_t seed, uint64_t step,
                  uint64_t first_elem, void* dst, void* hip_stream) {
  if (n < 0 || (n > 0 && (!src || !dst))) return fail(-1, "bad src/dst/n");
  if (dtype != ELMO_BF16 && dtype != ELMO_FP8_E4M3) return fail(-2, "unsupported dtype %d", dtype);
  if (mode != 0 && mode != 1) return fail(-1, "mode must be 0 (nearest) or 1 (stochastic)");
  if (n == 0) return 0;
  hipStream_t st = (hipStream_t)hip_stream;
  const int grid = (int)std::min<int64_t>((n + elmo::kThreads - 1) / elmo::kThreads, 256 * 16);
  if (dtype == ELMO_BF16) {
    if (mode) elmo::k_quantize<elmo::FMT_BF16, true><<<grid, elmo::kThreads, 0, st>>>(src, n, seed, step, first_elem, dst);
    else elmo::k_quantize<elmo::FMT_BF16, false><<<grid, elmo::kThreads, 0, st>>>(src, n, seed, step, first_elem, dst);
  } else {
    if (mode) elmo::k_quantize<elmo::FMT_E4M3, true><<<grid, elmo::kThreads, 0, st>>>(src, n, seed, step, first_elem, dst);
    else elmo::k_quantize<elmo::FMT_E4M3, false><<<grid, elmo::kThreads, 0, st>>>(src, n, seed, step, first_elem, dst);
  }
  return check_launch("k_quantize");
}

}  // extern "C"

namespace {

int poll_validation(elmo_head* h) {
  if (!(h->p.flags & ELMO_VALIDATE) || !h->validated_step_pending) return 0;
  int flag = 0;
  ELMO_HIP(hipMemcpy(&flag, h->ws + h->p.off_flag, sizeof flag, hipMemcpyDeviceToHost));
  h->validated_step_pending = false;
  if (flag) return fail(-4, "the previous step found invalid label data (code %d: 1 = bad indptr, 2 = id out of range or not ascending)", flag);
  return 0;
}

template <bool FP8, bool LOSS, int TB, bool DROP>
void launch_logits_tb(hipStream_t st, int grid, const char* Xa, int a_rows, const char* Wc, int n, int d, int Bp, int B,
                      uint16_t* Gt, const int* binptr, const int2* pos, int tile0, float* loss_slots, uint64_t seed, uint64_t step,
                      uint64_t elem0, elmo::DropArgs dr) {
  elmo::k_logits<FP8, LOSS, TB, DROP><<<grid, elmo::kGemmThreads, elmo::logits_smem<TB>(), st>>>(
      Xa, a_rows, Wc, n, d, Bp, B, Gt, binptr, pos, tile0, loss_slots, seed, step, elem0, dr);
}
// tb = rows of the batch tile (256, or 128 when the whole padded batch fits in 128 rows)
template <bool FP8, bool LOSS>
void launch_logits(hipStream_t st, int tb, int grid, const char* Xa, int a_rows, const char* Wc, int n, int d, int Bp, int B,
                   uint16_t* Gt, const int* binptr, const int2* pos, int tile0, float* loss_slots, uint64_t seed, uint64_t step,
                   uint64_t elem0, elmo::DropArgs dr) {
#define ELMO_LOGITS(TB_, DR_) \
  launch_logits_tb<FP8, LOSS, TB_, DR_>(st, grid, Xa, a_rows, Wc, n, d, Bp, B, Gt, binptr, pos, tile0, loss_slots, seed, step, elem0, dr)
  if (tb == 128) { if (dr.thresh) ELMO_LOGITS(128, true); else ELMO_LOGITS(128, false); }
  else { if (dr.thresh) ELMO_LOGITS(256, true); else ELMO_LOGITS(256, false); }
#undef ELMO_LOGITS
}

template <int FMT>
void launch_update(hipStream_t st, int grid, bool sr, bool kahan, const char* Gt, const char* XT, char* Wc, uint16_t* Cc,
                   int n, int d, int Bp, float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0, elmo::DropArgs dr) {
#define ELMO_UPD2(SR_, KA_, DR_, WD_) \
  elmo::k_update<FMT, SR_, KA_, DR_, WD_><<<grid, elmo::kGemmThreads, elmo::kUpdateSmem, st>>>(Gt, XT, Wc, Cc, n, d, Bp, lr, wd, seed, step, elem0, dr)
#define ELMO_UPD(SR_, KA_)                                               \
  do {                                                                   \
    if (dr.thresh) { if (wd != 0.0f) ELMO_UPD2(SR_, KA_, true, true); else ELMO_UPD2(SR_, KA_, true, false); }   \
    else { if (wd != 0.0f) ELMO_UPD2(SR_, KA_, false, true); else ELMO_UPD2(SR_, KA_, false, false); }           \
  } while (0)
  if (sr && kahan) ELMO_UPD(true, true);
  else if (sr) ELMO_UPD(true, false);
  else if (kahan) ELMO_UPD(false, true);
  else ELMO_UPD(false, false);
#undef ELMO_UPD2
#undef ELMO_UPD
}

// Small-batch fused input gradient + update.  Returns the launch's dynamic LDS size through the
// template so that the attribute call and the launch agree.
template <int FMT, bool SR, bool KAHAN, bool DX, bool WD, bool DROP>
int launch_dx_update_one(hipStream_t st, int grid, const char* Gt, const char* XT, char* Wc, uint16_t* Cc, float* dXacc, int n,
                         int d, int Bp, float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0, int tpg, elmo::DropArgs dr) {
  constexpr int smem = elmo::dxu_smem_bytes<FMT, KAHAN, DROP>();
  if constexpr (smem > 160 * 1024) {
    return fail(-3, "internal: no single-pass kernel for this mode");      // the caller takes the separate kernels instead
  } else {
    // once per process and instantiation, safe against two host threads stepping two heads
    static std::once_flag once;
    static hipError_t attr_rc = hipSuccess;
    std::call_once(once, [] {
      attr_rc = hipFuncSetAttribute(reinterpret_cast<const void*>(&elmo::k_dx_update<FMT, SR, KAHAN, DX, WD, DROP>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    });
    if (attr_rc != hipSuccess) return fail(-3, "hipFuncSetAttribute(k_dx_update) failed: %s", hipGetErrorString(attr_rc));
    elmo::k_dx_update<FMT, SR, KAHAN, DX, WD, DROP><<<grid, elmo::kGemmThreads, smem, st>>>(Gt, XT, Wc, Cc, dXacc, n, d, Bp, lr, wd, seed,
                                                                                            step, elem0, tpg, dr);
    return 0;
  }
}
template <int FMT>
int launch_dx_update(hipStream_t st, int grid, bool sr, bool kahan, bool dx, const char* Gt, const char* XT, char* Wc, uint16_t* Cc,
                     float* dXacc, int n, int d, int Bp, float lr, float wd, uint64_t seed, uint64_t step, uint64_t elem0, int tpg,
                     elmo::DropArgs dr) {
#define ELMO_DXU3(SR_, KA_, DX_, WD_) \
  return dr.thresh ? launch_dx_update_one<FMT, SR_, KA_, DX_, WD_, true>(st, grid, Gt, XT, Wc, Cc, dXacc, n, d, Bp, lr, wd, seed, step, elem0, tpg, dr) \
                   : launch_dx_update_one<FMT, SR_, KA_, DX_, WD_, false>(st, grid, Gt, XT, Wc, Cc, dXacc, n, d, Bp, lr, wd, seed, step, elem0, tpg, dr)
#define ELMO_DXU(SR_, KA_, DX_)                 \
  do {                                          \
    if (wd != 0.0f) ELMO_DXU3(SR_, KA_, DX_, true); \
    ELMO_DXU3(SR_, KA_, DX_, false);            \
  } while (0)
  if (sr && kahan && dx) ELMO_DXU(true, true, true);
  if (sr && kahan) ELMO_DXU(true, true, false);
  if (sr && dx) ELMO_DXU(true, false, true);
  if (sr) ELMO_DXU(true, false, false);
  if (kahan && dx) ELMO_DXU(false, true, true);
  if (kahan) ELMO_DXU(false, true, false);
  if (dx) ELMO_DXU(false, false, true);
  ELMO_DXU(false, false, false);
#undef ELMO_DXU
#undef ELMO_DXU3
}

// Opt in to more than 64 KiB of dynamic LDS for the tile kernels: once per process, whichever
// host thread comes first (std::call_once below); every caller sees the same outcome.
int raise_lds_limits_once() {
#define ELMO_ATTR(k, bytes) ELMO_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(&k), hipFuncAttributeMaxDynamicSharedMemorySize, bytes))
#define ELMO_ATTR_LOGITS(F, LO) \
  ELMO_ATTR((elmo::k_logits<F, LO, 256, false>), elmo::logits_smem<256>()); ELMO_ATTR((elmo::k_logits<F, LO, 256, true>), elmo::logits_smem<256>()); \
  ELMO_ATTR((elmo::k_logits<F, LO, 128, false>), elmo::logits_smem<128>()); ELMO_ATTR((elmo::k_logits<F, LO, 128, true>), elmo::logits_smem<128>())
  ELMO_ATTR_LOGITS(true, true);
  ELMO_ATTR_LOGITS(true, false);
  ELMO_ATTR_LOGITS(false, true);
  ELMO_ATTR_LOGITS(false, false);
#undef ELMO_ATTR_LOGITS
#define ELMO_ATTR_UPDATE(F, SR_, KA_)                                                                                                        \
  ELMO_ATTR((elmo::k_update<F, SR_, KA_, false, false>), elmo::kUpdateSmem); ELMO_ATTR((elmo::k_update<F, SR_, KA_, true, false>), elmo::kUpdateSmem); \
  ELMO_ATTR((elmo::k_update<F, SR_, KA_, false, true>), elmo::kUpdateSmem); ELMO_ATTR((elmo::k_update<F, SR_, KA_, true, true>), elmo::kUpdateSmem)
  ELMO_ATTR_UPDATE(elmo::FMT_BF16, true, true);
  ELMO_ATTR_UPDATE(elmo::FMT_BF16, true, false);
  ELMO_ATTR_UPDATE(elmo::FMT_BF16, false, true);
  ELMO_ATTR_UPDATE(elmo::FMT_BF16, false, false);
  ELMO_ATTR_UPDATE(elmo::FMT_E4M3, true, true);
  ELMO_ATTR_UPDATE(elmo::FMT_E4M3, true, false);
  ELMO_ATTR_UPDATE(elmo::FMT_E4M3, false, true);
  ELMO_ATTR_UPDATE(elmo::FMT_E4M3, false, false);
#undef ELMO_ATTR_UPDATE
  ELMO_ATTR((elmo::k_dx<true, false>), elmo::dx_smem_bytes<true>());
  ELMO_ATTR((elmo::k_dx<true, true>), elmo::dx_smem_bytes<true>());
  ELMO_ATTR((elmo::k_dx<false, false>), elmo::dx_smem_bytes<false>());
  ELMO_ATTR((elmo::k_dx<false, true>), elmo::dx_smem_bytes<false>());
  ELMO_ATTR((elmo::k_topk_first<true>), elmo::logits_smem<256>());
  ELMO_ATTR((elmo::k_topk_first<false>), elmo::logits_smem<256>());
  ELMO_ATTR((elmo::k_topk_filter_run<true, true>), elmo::kTopkRunSmem);
  ELMO_ATTR((elmo::k_topk_filter_run<true, false>), elmo::kTopkRunSmem);
  ELMO_ATTR((elmo::k_topk_filter_run<false, true>), elmo::kTopkRunSmem);
  ELMO_ATTR((elmo::k_topk_filter_run<false, false>), elmo::kTopkRunSmem);
  ELMO_ATTR((elmo::k_topk_chunk<true>), elmo::kTopkSmem);
  ELMO_ATTR((elmo::k_topk_chunk<false>), elmo::kTopkSmem);
#undef ELMO_ATTR
  return 0;
}
int raise_lds_limits() {
  static std::once_flag once;
  static int rc = 0;
  static char text[sizeof g_err];
  std::call_once(once, [] {
    rc = raise_lds_limits_once();
    if (rc) memcpy(text, g_err, sizeof text);      // the error text is thread-local: keep it for later callers
  });
  if (rc) memcpy(g_err, text, sizeof g_err);
  return rc;
}

}  // namespace

extern "C" int elmo_head_step(elmo_head_t* h, const void* X, int32_t B, const int32_t* indptr, const int32_t* indices,
                              int64_t nnz, float lr, uint64_t seed, uint64_t step, void* dX_out, float* loss_out,
                              void* hip_stream) {
  if (!h) return fail(-1, "NULL head");
  const Plan& p = h->p;
  if (!X || !indptr) return fail(-1, "X and indptr must not be NULL");
  if (B < 1 || B > p.maxB) return fail(-1, "B = %d outside [1, max_B = %d]", B, p.maxB);
  if (nnz < 0 || nnz > p.max_nnz) return fail(-1, "nnz = %lld outside [0, max_nnz = %lld]", (long long)nnz, (long long)p.max_nnz);
  if (nnz > 0 && !indices) return fail(-1, "indices must not be NULL when nnz > 0");
  if (p.drop_thresh && (step >> 63)) return fail(-1, "with dropout the step counter must stay below 2^63");
  if (int rc = poll_validation(h)) return rc;
  if (int rc = raise_lds_limits()) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool fp8 = p.fmt == ELMO_FP8_E4M3;
  const elmo::DropArgs dr{p.drop_thresh, 256.0f / (256.0f - (float)p.drop_thresh)};
  const int d = p.d, Bp = round_up(B, 64), Bp256 = round_up(Bp, 256);
  const int tiles_b = Bp256 / 256, tiles_j = (d + 255) / 256;   // 256 x 256 tiles of the matrix products

  uint8_t* Xq = fp8 ? (uint8_t*)(h->ws + p.off_xq) : nullptr;
  uint16_t* XT = (uint16_t*)(h->ws + p.off_xt);
  uint16_t* Gt = (uint16_t*)(h->ws + p.off_g);
  float* dXacc = (float*)(h->ws + p.off_dx);
  float* loss_slots = (float*)(h->ws + p.off_loss);
  int* cnt = (int*)(h->ws + p.off_cnt);
  int* ptr = (int*)(h->ws + p.off_ptr);
  int* cur = (int*)(h->ws + p.off_cur);
  int2* pos = (int2*)(h->ws + p.off_pos);
  int* flag = (p.flags & ELMO_VALIDATE) ? (int*)(h->ws + p.off_flag) : nullptr;

  // Small batches are bound by memory traffic: input gradient and update share one pass over W
  // With dropout that kernel keeps a masked copy of the W tile in LDS, which does not fit next to
  // BF16 weights with compensation: that one mode takes the separate kernels.
  const bool small_batch = Bp <= 128 && d % 256 == 0 && !(p.drop_thresh && !fp8 && (p.flags & ELMO_KAHAN));
  const int col_blocks = d / 256, label_groups = small_batch ? std::max(1, 256 / col_blocks) : 0;   // widths above 65536: one group
  // label slices of the input-gradient product: at most one 512-thread workgroup per CU, so the
  // whole grid is resident at once (256 CUs) and no second, nearly empty round of workgroups runs
  int S = std::max(1, 256 / (tiles_b * tiles_j));
  S = std::min(S, p.dx_rows / Bp256);
  S = std::max(1, std::min(S, 64));
  const int dx_slices = small_batch ? label_groups : S;
  const int dx_plane_rows = small_batch ? 128 : Bp256;

  Profiler& prof = h->prof;
  prof.mark(st, CLS_SETUP);
  // ---- step set-up: inputs, zeroed partial sums, label index
  {
    const size_t n = (size_t)Bp * d;
    const size_t n_dx = dX_out ? (size_t)dx_slices * dx_plane_rows * d : 0;
    const size_t work = std::max(n, n_dx);
    elmo::k_step_setup<<<(int)std::min<size_t>((work + 255) / 256, 4096), elmo::kThreads, 0, st>>>(
        (const uint16_t*)X, B, Bp, d, Xq, XT, (uint32_t*)dXacc, n_dx, (uint32_t*)cnt, (size_t)p.ntiles + 1, (uint32_t*)flag);
    if (int rc = check_launch("k_step_setup")) return rc;
    const int row_grid = (B * elmo::kRowLanes + elmo::kThreads - 1) / elmo::kThreads;
    elmo::k_label_hist<<<row_grid, elmo::kThreads, 0, st>>>(indptr, indices, B, p.L, nnz, cnt, flag);
    if (int rc = check_launch("k_label_hist")) return rc;
    elmo::k_label_scan<<<1, 1024, 0, st>>>(cnt, p.ntiles, ptr, cur);
    if (int rc = check_launch("k_label_scan")) return rc;
    elmo::k_label_scatter<<<row_grid, elmo::kThreads, 0, st>>>(indptr, indices, B, p.L, nnz, cur, pos);
    if (int rc = check_launch("k_label_scatter")) return rc;
    if (flag) h->validated_step_pending = true;
  }

  // ---- chunk schedule (Section 4.2): forward, backward and update of one label chunk at a time
  const size_t esz = fp8 ? 1 : 2;
  const char* Xa = fp8 ? (const char*)Xq : (const char*)X;
  const int a_rows = fp8 ? Bp : B;
  for (int64_t c0 = 0; c0 < p.L; c0 += p.chunk) {
    const int n = (int)std::min<int64_t>(p.chunk, p.L - c0);
    char* Wc = h->W + (size_t)c0 * d * esz;
    uint16_t* Cc = h->comp ? (uint16_t*)h->comp + (size_t)c0 * d : nullptr;
    const int tile0 = (int)(c0 / 128);
    prof.mark(st, CLS_LOGITS);
    {
      const int tb = Bp <= 128 ? 128 : 256;        // the logits kernel's tile is tb samples x tb labels
      const int grid = ((n + tb - 1) / tb) * ((Bp + tb - 1) / tb);
      const uint64_t celem0 = (uint64_t)c0 * (uint64_t)d;
      if (fp8) {
        if (loss_out) launch_logits<true, true>(st, tb, grid, Xa, a_rows, Wc, n, d, Bp, B, Gt, ptr, pos, tile0, loss_slots, seed, step, celem0, dr);
        else launch_logits<true, false>(st, tb, grid, Xa, a_rows, Wc, n, d, Bp, B, Gt, ptr, pos, tile0, loss_slots, seed, step, celem0, dr);
      } else {
        if (loss_out) launch_logits<false, true>(st, tb, grid, Xa, a_rows, Wc, n, d, Bp, B, Gt, ptr, pos, tile0, loss_slots, seed, step, celem0, dr);
        else launch_logits<false, false>(st, tb, grid, Xa, a_rows, Wc, n, d, Bp, B, Gt, ptr, pos, tile0, loss_slots, seed, step, celem0, dr);
      }
      if (int rc = check_launch("k_logits")) return rc;
    }
    // Update of the chunk in at most two parts: labels below kahan_rows carry compensation
    // (Kahan summation for head labels), the others are updated without it.
    const bool sr = p.flags & ELMO_SR;
    const int n_head = (int)std::max<int64_t>(0, std::min<int64_t>(n, p.kahan_rows - c0));
    if (small_batch) {
      prof.mark(st, CLS_UPDATE);
      for (int part = 0; part < 2; ++part) {
        const int l_off = part ? n_head : 0, n_part = part ? n - n_head : n_head;   // n_head is a multiple of 32 or all of n
        if (n_part == 0) continue;
        const bool kahan = part == 0;
        const int ntiles32 = (n_part + 31) / 32, tpg = (ntiles32 + label_groups - 1) / label_groups;
        const int groups_used = (ntiles32 + tpg - 1) / tpg;
        const uint64_t elem0 = (uint64_t)(c0 + l_off) * (uint64_t)d;
        const char* Gp = (const char*)(Gt + (size_t)l_off * Bp);
        char* Wp = Wc + (size_t)l_off * d * esz;
        uint16_t* Cp = kahan ? Cc + (size_t)l_off * d : nullptr;
        int rc;
        if (fp8) rc = launch_dx_update<elmo::FMT_E4M3>(st, groups_used * col_blocks, sr, kahan, dX_out != nullptr, Gp, (const char*)XT, Wp, Cp, dXacc, n_part, d, Bp, lr, p.weight_decay, seed, step, elem0, tpg, dr);
        else rc = launch_dx_update<elmo::FMT_BF16>(st, groups_used * col_blocks, sr, kahan, dX_out != nullptr, Gp, (const char*)XT, Wp, Cp, dXacc, n_part, d, Bp, lr, p.weight_decay, seed, step, elem0, tpg, dr);
        if (rc) return rc;
        if (int rc2 = check_launch("k_dx_update")) return rc2;
      }
      continue;
    }
    if (dX_out) {
      prof.mark(st, CLS_DX);
      const int grid = tiles_b * tiles_j * S;
      const uint64_t celem0 = (uint64_t)c0 * (uint64_t)d;
#define ELMO_DX(F, DR_) \
  elmo::k_dx<F, DR_><<<grid, elmo::kGemmThreads, elmo::dx_smem_bytes<F>(), st>>>((const char*)Gt, Wc, dXacc, n, d, Bp, Bp256, S, seed, step, celem0, dr)
      if (fp8) { if (dr.thresh) ELMO_DX(true, true); else ELMO_DX(true, false); }
      else { if (dr.thresh) ELMO_DX(false, true); else ELMO_DX(false, false); }
#undef ELMO_DX
      if (int rc = check_launch("k_dx")) return rc;
    }
    prof.mark(st, CLS_UPDATE);
    for (int part = 0; part < 2; ++part) {
      const int l_off = part ? n_head : 0, n_part = part ? n - n_head : n_head;
      if (n_part == 0) continue;
      const bool kahan = part == 0;
      const int grid = ((n_part + 255) / 256) * tiles_j;
      const uint64_t elem0 = (uint64_t)(c0 + l_off) * (uint64_t)d;
      const char* Gp = (const char*)(Gt + (size_t)l_off * Bp);
      char* Wp = Wc + (size_t)l_off * d * esz;
      uint16_t* Cp = kahan ? Cc + (size_t)l_off * d : nullptr;
      if (fp8) launch_update<elmo::FMT_E4M3>(st, grid, sr, kahan, Gp, (const char*)XT, Wp, Cp, n_part, d, Bp, lr, p.weight_decay, seed, step, elem0, dr);
      else launch_update<elmo::FMT_BF16>(st, grid, sr, kahan, Gp, (const char*)XT, Wp, Cp, n_part, d, Bp, lr, p.weight_decay, seed, step, elem0, dr);
      if (int rc = check_launch("k_update")) return rc;
    }
  }

  prof.mark(st, CLS_FINAL);
  if (dX_out || loss_out) {
    const size_t n = (size_t)B * d;
    const int grid = dX_out ? (int)std::min<size_t>((n + 255) / 256, 4096) : 1;
    elmo::k_finalize<<<grid, elmo::kThreads, 0, st>>>(dXacc, dx_slices, dx_plane_rows, B, d, (uint16_t*)dX_out, loss_slots,
                                                     p.ntiles * tiles_b, loss_out);
    if (int rc = check_launch("k_finalize")) return rc;
  }
  prof.mark(st, CLS_END);
  return 0;
}

extern "C" int elmo_head_topk(elmo_head_t* h, const void* X, int32_t B, int32_t k, int32_t* idx_out, float* score_out,
                              void* hip_stream) {
  if (!h) return fail(-1, "NULL head");
  const Plan& p = h->p;
  if (!X) return fail(-1, "X must not be NULL");
  if (B < 1 || B > p.maxB) return fail(-1, "B = %d outside [1, max_B = %d]", B, p.maxB);
  if (k < 1 || k > p.L) return fail(-1, "k = %d outside [1, L = %lld]", k, (long long)p.L);
  if (int rc = poll_validation(h)) return rc;
  if (int rc = raise_lds_limits()) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  const bool fp8 = p.fmt == ELMO_FP8_E4M3;
  const int d = p.d, Bp = round_up(B, 64);
  uint8_t* Xq = fp8 ? (uint8_t*)(h->ws + p.off_xq) : nullptr;
  uint16_t* XT = (uint16_t*)(h->ws + p.off_xt);
  {
    const size_t n = (size_t)Bp * d;
    elmo::k_prep_x<<<(int)std::min<size_t>((n + 255) / 256, 4096), elmo::kThreads, 0, st>>>((const uint16_t*)X, B, Bp, d, Xq, XT);
    if (int rc = check_launch("k_prep_x")) return rc;
  }
  const char* Xa = fp8 ? (const char*)Xq : (const char*)X;
  const int a_rows = fp8 ? Bp : B;
  h->prof.mark(st, CLS_TOPK);
  const int rc = elmo::topk_run(st, fp8, Xa, a_rows, h->W, p.L, d, p.chunk, B, Bp, k, h->ws + p.off_topk, idx_out, score_out, g_err,
                                sizeof g_err);
  h->prof.mark(st, CLS_END);
  return rc;
}

// ---------------------------------------------------------------------------------------------
// Top-k without a head, a workspace or any allocation: the scratch of the top-k kernels (thresholds,
// counters, candidate lists, per-segment lists of the overflow path) and the E4M3 copy of X live
// in a file-scope device array.  Every GPU the library runs on holds its own copy of that array at
// its own address until the process ends; the address is looked up once per device.
// ---------------------------------------------------------------------------------------------
namespace {
constexpr int kStaticMaxB = 128;                                  // queries per call
constexpr int kStaticMaxD = 4096;                                 // embedding width
constexpr size_t kStaticXqBytes = (size_t)kStaticMaxB * kStaticMaxD;
constexpr size_t kStaticBytes = (size_t)18 << 20;                 // 0.5 MiB staged inputs + 16.1 MiB top-k scratch for 128 rows
constexpr int kStaticMaxDevices = 64;
std::mutex g_static_mu;
char* g_static_ptr[kStaticMaxDevices] = {};
}  // namespace

static __device__ __align__(256) unsigned char scratch[kStaticBytes];

namespace {
// Device address of `scratch` on the current device.  In host code the array's name is only a
// stand-in for the symbol, never a device address: the address comes from the runtime, per device.
int static_scratch(char** out) {
  int dev = -1;
  ELMO_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kStaticMaxDevices) return fail(-3, "device ordinal %d outside [0, %d)", dev, kStaticMaxDevices);
  std::lock_guard<std::mutex> lock(g_static_mu);
  if (!g_static_ptr[dev]) {
    void* p = nullptr;
    ELMO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
    if (!p) return fail(-3, "hipGetSymbolAddress returned a null address");
    g_static_ptr[dev] = (char*)p;
  }
  *out = g_static_ptr[dev];
  return 0;
}
}  // namespace

extern "C" int elmo_topk_static(const void* W, int64_t L, int32_t d, int weight_dtype, const void* X, int32_t B, int32_t k,
                                int32_t* idx_out, float* score_out, void* hip_stream) {
  if (!W || !X) return fail(-1, "W and X must not be NULL");
  if (L < 1 || L > (int64_t)1 << 31) return fail(-1, "L must be in [1, 2^31] (got %lld)", (long long)L);
  if (d < 128 || d % 128 != 0 || d > kStaticMaxD) return fail(-1, "d must be a multiple of 128 in [128, %d] (got %d)", kStaticMaxD, d);
  if (weight_dtype != ELMO_BF16 && weight_dtype != ELMO_FP8_E4M3) return fail(-2, "unsupported weight_dtype %d", weight_dtype);
  if (B < 1 || B > kStaticMaxB) return fail(-1, "B = %d outside [1, %d]: the static scratch holds the lists of %d queries", B, kStaticMaxB, kStaticMaxB);
  if (k < 1 || k > L) return fail(-1, "k = %d outside [1, L = %lld]", k, (long long)L);
  if (((uintptr_t)W | (uintptr_t)X) & 15) return fail(-1, "W and X must be 16-byte aligned");
  const bool fp8 = weight_dtype == ELMO_FP8_E4M3;
  const int Bp = round_up(B, 64);
  if (kStaticXqBytes + elmo::topk_scratch_bytes(Bp, 0) > kStaticBytes) return fail(-3, "internal: static scratch plan exceeded");
  if (int rc = raise_lds_limits()) return rc;
  char* base = nullptr;
  if (int rc = static_scratch(&base)) return rc;
  hipStream_t st = (hipStream_t)hip_stream;
  uint8_t* Xq = (uint8_t*)base;
  if (fp8) {   // E4M3 copy of X, rows B..Bp-1 zero (the BF16 product reads X itself and clamps its rows)
    const size_t n = (size_t)Bp * d;
    elmo::k_prep_x<<<(int)std::min<size_t>((n + 255) / 256, 4096), elmo::kThreads, 0, st>>>((const uint16_t*)X, B, Bp, d, Xq, nullptr);
    if (int rc = check_launch("k_prep_x")) return rc;
  }
  // every call starts from the scratch the last call left: topk_run re-initialises the thresholds,
  // counters and overflow flags of all rows itself, and reads candidate slots only below the counters
  return elmo::topk_run(st, fp8, fp8 ? (const char*)Xq : (const char*)X, fp8 ? Bp : B, (const char*)W, L, d, 0, B, Bp, k,
                        base + kStaticXqBytes, idx_out, score_out, g_err, sizeof g_err);
}

extern "C" int elmo_precision_hits(const int32_t* idx, int32_t B, int32_t k, const int32_t* indptr, const int32_t* indices,
                                   int64_t* hits_out, void* hip_stream) {
  if (!idx || !indptr || !hits_out) return fail(-1, "idx, indptr and hits_out must not be NULL");
  if (B < 1) return fail(-1, "B must be >= 1 (got %d)", B);
  if (k < 1 || k > (1 << 20)) return fail(-1, "k = %d outside [1, 2^20]", k);
  if ((int64_t)B * k > INT32_MAX) return fail(-1, "B * k = %lld does not fit 31 bits", (long long)B * k);
  hipStream_t st = (hipStream_t)hip_stream;
  unsigned long long* hits = reinterpret_cast<unsigned long long*>(hits_out);
  elmo::k_fill_u32<<<1, elmo::kThreads, 0, st>>>((uint32_t*)hits, (size_t)k * 2, 0u);
  if (int rc = check_launch("k_fill_u32")) return rc;
  const int64_t n = (int64_t)B * k;
  elmo::k_hits_at<<<(int)((n + elmo::kThreads - 1) / elmo::kThreads), elmo::kThreads, 0, st>>>(idx, B, k, indptr, indices, hits);
  if (int rc = check_launch("k_hits_at")) return rc;
  elmo::k_hits_scan<<<1, elmo::kThreads, 0, st>>>(hits, k);
  return check_launch("k_hits_scan");
}

extern "C" int elmo_quantize_em(const float* src, int64_t n, int exp_bits, int man_bits, int mode, uint64_t seed, uint64_t step,
                                uint64_t first_elem, float* dst, void* hip_stream) {
  if (n < 0 || (n > 0 && (!src || !dst))) return fail(-1, "bad src/dst/n");
  if (exp_bits < 2 || exp_bits > 8 || man_bits < 1 || man_bits > 22)
    return fail(-2, "unsupported format E%dM%d (2 <= E <= 8, 1 <= M <= 22)", exp_bits, man_bits);
  if (mode != 0 && mode != 1) return fail(-1, "mode must be 0 (nearest) or 1 (stochastic)");
  if (n == 0) return 0;
  hipStream_t st = (hipStream_t)hip_stream;
  const int grid = (int)std::min<int64_t>((n + elmo::kThreads - 1) / elmo::kThreads, 256 * 16);
  if (mode) elmo::k_quantize_em<true><<<grid, elmo::kThreads, 0, st>>>(src, n, exp_bits, man_bits, seed, step, first_elem, dst);
  else elmo::k_quantize_em<false><<<grid, elmo::kThreads, 0, st>>>(src, n, exp_bits, man_bits, seed, step, first_elem, dst);
  return check_launch("k_quantize_em");
}

extern "C" int elmo_kahan_adamw(void* param, void* comp, void* m, void* v, const void* grad, int64_t n, int state_dtype, float lr,
                                double beta1, double beta2, float eps, float weight_decay, int64_t t, void* hip_stream) {
  if (n < 0 || (n > 0 && (!param || !comp || !m || !v || !grad))) return fail(-1, "bad buffers / n");
  if (state_dtype != ELMO_BF16 && state_dtype != ELMO_FP32) return fail(-2, "state_dtype must be ELMO_BF16 or ELMO_FP32 (got %d)", state_dtype);
  if (!(beta1 >= 0.0 && beta1 < 1.0) || !(beta2 >= 0.0 && beta2 < 1.0)) return fail(-1, "betas must be in [0, 1)");
  if (t < 1) return fail(-1, "the step count t starts at 1 (got %lld)", (long long)t);
  if (!(eps >= 0.0f) || !(weight_decay >= 0.0f)) return fail(-1, "eps and weight_decay must be >= 0");
  if (((uintptr_t)param | (uintptr_t)comp | (uintptr_t)m | (uintptr_t)v | (uintptr_t)grad) & 15)
    return fail(-1, "all buffers must be 16-byte aligned");
  if (n == 0) return 0;
  elmo::AdamArgs a;
  a.lr = lr;
  a.b1 = (float)beta1; a.o1 = (float)(1.0 - beta1); a.bc1 = (float)(1.0 - std::pow(beta1, (double)t));
  a.b2 = (float)beta2; a.o2 = (float)(1.0 - beta2); a.bc2 = (float)(1.0 - std::pow(beta2, (double)t));
  a.eps = eps; a.wd = weight_decay;
  hipStream_t st = (hipStream_t)hip_stream;
  const int64_t work = std::max<int64_t>(n >> 3, 8);
  const int grid = (int)std::min<int64_t>((work + elmo::kThreads - 1) / elmo::kThreads, 256 * 16);
  if (state_dtype == ELMO_BF16)
    elmo::k_kahan_adamw<true><<<grid, elmo::kThreads, 0, st>>>((uint16_t*)param, (uint16_t*)comp, m, v, (const uint16_t*)grad, n, a);
  else
    elmo::k_kahan_adamw<false><<<grid, elmo::kThreads, 0, st>>>((uint16_t*)param, (uint16_t*)comp, m, v, (const uint16_t*)grad, n, a);
  return check_launch("k_kahan_adamw");
}
