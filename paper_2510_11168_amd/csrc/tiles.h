// LDS tile staging and MFMA fragment access shared by the head's three matrix products
// (Algorithm 1: logits, input gradient, weight gradient).  gfx950 only, 64-wide wavefronts,
// matrix-product workgroups of 512 threads arranged as 4 x 2 waves, each wave owning 64 x 128 outputs.
//
// LDS tile layout: ROWS rows of ROWB bytes (ROWB = 64, 128, 256 or 512), cut into 16-byte chunks whose
// index is XORed with a key derived from the row.  gfx950's LDS has 64 banks of 4 bytes (256 bytes
// per clock); a 16-byte-per-lane read is served 16 lanes at a time, so 16 lanes must touch 16
// different 16-byte bank groups.  The keys below make that true for the K-contiguous fragment
// reads (16 consecutive rows, same logical chunk) and for the transposing reads (4 rows x 32
// bytes, or 8 rows x 16 bytes), measured at 214 of 256 bytes/clock/CU against 117 for a plain
// (row & 7) key.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace elmo {

typedef float f32x2 __attribute__((ext_vector_type(2)));
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

template <int ROWB> __device__ inline int swz_key(int r) {
  // 256- and 512-byte rows (the K-major tiles read by the transposing loads): pairs of chunks move
  // together.  512-byte rows: four consecutive rows go to four different 64-byte quarters of the
  // 256-byte bank period, which is what one pass of ds_read_b64_tr_b16 (4 rows x 64 B) touches;
  // with the (r & 7) << 1 key of the 256-byte rows that read ran into two-way conflicts (a third
  // of the LDS cycles of the input-gradient kernel by the SQ_LDS_BANK_CONFLICT counter).  The
  // 256-byte rows keep their key: ds_read_b64_tr_b8 (8 rows x 32 B) is conflict-free with it, and
  // the single-pass small-batch kernel measured 4 % slower with the other one.
  return ROWB == 64 ? (r >> 2) & 3 : ROWB == 128 ? (r >> 1) & 7 : ROWB == 256 ? (r & 7) << 1 : ((r & 3) << 2) | (((r >> 2) & 1) << 1);
}
template <int ROWB> __device__ inline int tile_off(int r, int c) {
  return r * ROWB + ((c ^ swz_key<ROWB>(r)) << 4);
}

#define ELMO_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// s_waitcnt vmcnt(N) with the other counters left alone (gfx9 encoding: vmcnt = imm[15:14]:imm[3:0]).
template <int N> __device__ inline void wait_vmcnt() {
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0F70);
}
// Workgroup barrier without a memory fence: the caller has already waited for exactly the
// asynchronous loads it depends on.  The empty asm statements keep the compiler from moving LDS
// accesses across it.
__device__ inline void barrier_nofence() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Same, after this wave's own LDS writes have completed (lgkmcnt(0)): orders ds_write -> barrier ->
// ds_read without the fence of __syncthreads(), which would also drain the asynchronous loads.
__device__ inline void barrier_lds() {
  __builtin_amdgcn_s_waitcnt(0xC07F);   // lgkmcnt(0), vmcnt and expcnt untouched
  barrier_nofence();
}

// Asynchronous global -> LDS copy of a ROWS x ROWB-byte slab (no registers in between): one
// global_load_lds_dwordx4 moves 64 lanes x 16 bytes into 1 KiB of consecutive LDS, i.e. 1024/ROWB
// whole tile rows; each lane fetches the global chunk that belongs at its swizzled position.
// Rows at or beyond rows_valid (>= 1) re-read the last valid row.  Issues ROWS*ROWB/4096 loads per
// wave; completion is tracked by vmcnt in issue order.
// I0, I1: only loads I0 .. I1-1 of the wave's NI loads (default: all), for callers that pace them.
template <int ROWS, int ROWB, int NW, int I0 = 0, int I1 = 1 << 20>
__device__ inline void dma_tile(const char* __restrict__ g, size_t stride, int rows_valid, char* lds_tile, int wave, int lane,
                                int chunks_valid = 1 << 20) {
  constexpr int RPI = 1024 / ROWB, CPR = ROWB / 16, NI = ROWS / RPI / NW;
  static_assert(ROWS % (RPI * NW) == 0 && NI >= 1, "tile must split evenly over the waves");
  // The slab pointer is wave-uniform.  Passing it through an empty asm statement as a scalar
  // register pair keeps the compiler from folding it into per-lane 64-bit addresses that it then
  // hoists out of the K loop (two registers per load, kept alive for the whole kernel).
  {
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)g), hi = __builtin_amdgcn_readfirstlane((uint32_t)((uintptr_t)g >> 32));
    asm volatile("" : "+s"(lo), "+s"(hi));
    g = reinterpret_cast<const char*>(((uintptr_t)hi << 32) | lo);
  }
#pragma unroll
  for (int i = (I0 > 0 ? I0 : 0); i < (I1 < NI ? I1 : NI); ++i) {
    const int rbase = (wave * NI + i) * RPI;
    const int r = rbase + lane / CPR;
    const int c = min((lane % CPR) ^ swz_key<ROWB>(r), chunks_valid - 1);   // chunks past a short row re-read its last one
    const int rc = min(r, rows_valid - 1);
    // 32-bit lane offset on top of the (wave-uniform) slab pointer: the load then takes the
    // scalar-base + vector-offset form and needs no 64-bit address arithmetic per lane
    const uint32_t off = __umul24((uint32_t)rc, (uint32_t)stride) + (uint32_t)(c * 16);
    // The load is written as an assembly statement (M0 = LDS address of lane 0's 16 bytes, lane i
    // lands 16 i bytes further; scalar base + 32-bit lane offset).  Issued through the builtin, the
    // compiler books it as an access that may touch both memory and LDS, and while one is in
    // flight it turns every wait for LDS fragment reads into lgkmcnt(0) -- which also waits for
    // the reads of the next step issued just before -- and puts vmcnt(0) in front of LDS reads it
    // cannot tell from the load's destination.  Completion is tracked by the explicit vmcnt
    // waits of the rings (loads complete in issue order; the compiler's own vmcnt waits only
    // become stricter by loads it does not know of).
    // (the low 32 bits of a generic pointer into LDS are the LDS byte address)
    const uint32_t dst = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lds_tile + (uint32_t)(rbase * ROWB));
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(off), "s"(g) : "memory", "m0");
  }
}
template <int ROWS, int ROWB, int NW> constexpr int dma_loads_per_wave() { return ROWS * ROWB / 1024 / NW; }

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

// Software pipeline over K slabs with a ring of NST LDS stages (stage = [A tile | B tile]) filled
// by asynchronous global->LDS loads that run NST-1 slabs ahead of the matrix cores.  Per slab:
// wait until at most the younger slabs' loads are outstanding (vmcnt counts in issue order), one
// barrier, refill the stage that was consumed one step earlier, then the slab's products.
//
// Ping-pong issue order.  The product of one slab is split in two parts (by default its two
// halves), mma(stageA, stageB, 0, LATE_AFTER) and mma(stageA, stageB, LATE_AFTER, 4), in units of
// quarters of the slab.  A wave that issues an asynchronous
// load is held until the memory pipeline accepts it, i.e. roughly for as long as the data takes
// to move; with every wave issuing at the same point the load and MFMA phases add up instead of
// overlapping.  Here waves 0..NW/2-1 issue right after the barrier (the whole A slab and the first
// half of the B slab), waves NW/2..NW-1 between the two parts (the second half of the B slab);
// with UNEVEN = false both groups issue an equal share of both slabs.
// Waves w and w + 4 share a SIMD, so one wave of each SIMD computes while its partner is held.
// Measured on the BF16 main loop alone: all waves issuing together 1.33 PFLOP/s, equal shares
// early/late 1.34-1.6, this 3:1 split 1.42-1.44 at the same clocks as 1.31 for equal shares.
// chunks_a / chunks_b: valid 16-byte chunks per row (short rows re-read their last chunk).
//
// ring_stream_pp is the general form: src(ks, off_a, va, off_b, vb) names slab ks of each operand
// (byte offset from ga / gb and number of valid rows), so a workgroup can run the ring across the
// output tiles it owns without draining it; mma(stageA, stageB, q0, q1, ks).  The base pointers are
// restrict-qualified parameters on purpose: inlining then tags every LDS access inside with alias
// information, without which the compiler puts a vmcnt(0) in front of LDS reads it cannot tell
// from the asynchronous loads still in flight.
// prep(stageB, ks), if given, is run by every wave on the landed B slab before the product (it may
// rewrite the slab in LDS); a barrier follows it.
struct NoPrep {};
// LATE_AFTER (1..3): the product of a slab is four quarters, mma(stageA, stageB, q0, q1, ks) runs
// quarters [q0, q1); the late waves issue after LATE_AFTER of them (2 = between the two halves).
template <int AROWS, int AROWB, int BROWS, int BROWB, int NST, int NW, bool UNEVEN, int LATE_AFTER = 2, class Src, class Mma,
          class Prep = NoPrep>
__device__ inline void ring_stream_pp(const char* __restrict__ ga, size_t stride_a, int chunks_a, const char* __restrict__ gb,
                                      size_t stride_b, int chunks_b, int nk, char* smem, int wave, int lane, Src&& src, Mma&& mma,
                                      Prep&& prep = Prep{}) {
  constexpr bool HAS_PREP = !std::is_same<std::remove_cv_t<std::remove_reference_t<Prep>>, NoPrep>::value;
  constexpr int ABYTES = AROWS * AROWB, SBYTES = ABYTES + BROWS * BROWB, NH = NW / 2, BH = BROWS / 2;
  constexpr int LPS_ALL = dma_loads_per_wave<AROWS, AROWB, NW>() + dma_loads_per_wave<BROWS, BROWB, NW>();
  constexpr int LPS_LATE = UNEVEN ? dma_loads_per_wave<BH, BROWB, NH>() : LPS_ALL;
  constexpr int LPS_EARLY = UNEVEN ? dma_loads_per_wave<AROWS, AROWB, NH>() + LPS_LATE : LPS_ALL;
  static_assert(NST >= 2 && NST <= 3 && (NST - 2) * LPS_EARLY <= 63, "ring depth");
  const bool late = wave >= NH;
  auto issue = [&](int ks) {
    char* st = smem + (ks % NST) * SBYTES;
    size_t off_a, off_b;
    int va, vb;
    src(ks, off_a, va, off_b, vb);
    if (!UNEVEN) {
      dma_tile<AROWS, AROWB, NW>(ga + off_a, stride_a, va, st, wave, lane, chunks_a);
      dma_tile<BROWS, BROWB, NW>(gb + off_b, stride_b, vb, st + ABYTES, wave, lane, chunks_b);
    } else if (!late) {
      dma_tile<AROWS, AROWB, NH>(ga + off_a, stride_a, va, st, wave, lane, chunks_a);
      dma_tile<BH, BROWB, NH>(gb + off_b, stride_b, vb, st + ABYTES, wave, lane, chunks_b);
    } else {
      // rows BH.. of the B slab; a slab with fewer valid rows re-reads its last valid row
      dma_tile<BH, BROWB, NH>(gb + off_b + (size_t)min(BH, vb - 1) * stride_b, stride_b, max(vb - BH, 1),
                              st + ABYTES + BH * BROWB, wave - NH, lane, chunks_b);
    }
  };
  for (int s = 0; s < NST - 1; ++s)
    if (s < nk) issue(s);
  for (int ks = 0; ks < nk; ++ks) {
    if (NST == 2 || ks + 1 >= nk) wait_vmcnt<0>();
    else if (late) wait_vmcnt<LPS_LATE>();
    else wait_vmcnt<LPS_EARLY>();
    barrier_nofence();
    const bool more = ks + NST - 1 < nk;
    if (more && !late) issue(ks + NST - 1);
    char* st = smem + (ks % NST) * SBYTES;
    if constexpr (HAS_PREP) {
      prep(st + ABYTES, ks);
      barrier_lds();
    }
    __builtin_amdgcn_sched_barrier(0);
    mma(st, st + ABYTES, 0, LATE_AFTER, ks);
    __builtin_amdgcn_sched_barrier(0);
    if (more && late) issue(ks + NST - 1);
    __builtin_amdgcn_sched_barrier(0);
    mma(st, st + ABYTES, LATE_AFTER, 4, ks);
  }
  barrier_nofence();   // every wave is done with the ring: the caller may reuse the memory
}

// One output tile: slab ks of an operand starts at g + ks*adv and has v0 - ks*dv valid rows.
template <int AROWS, int AROWB, int BROWS, int BROWB, int NST, int NW, bool UNEVEN, int LATE_AFTER = 2, class Mma, class Prep = NoPrep>
__device__ inline void ring_pipeline_pp(const char* __restrict__ ga, size_t stride_a, int va0, int dva, size_t adv_a, int chunks_a,
                                        const char* __restrict__ gb, size_t stride_b, int vb0, int dvb, size_t adv_b, int chunks_b,
                                        int nk, char* smem, int wave, int lane, Mma&& mma, Prep&& prep = Prep{}) {
  ring_stream_pp<AROWS, AROWB, BROWS, BROWB, NST, NW, UNEVEN, LATE_AFTER>(
      ga, stride_a, chunks_a, gb, stride_b, chunks_b, nk, smem, wave, lane,
      [&](int ks, size_t& off_a, int& va, size_t& off_b, int& vb) {
        off_a = (size_t)ks * adv_a; va = va0 - ks * dva;
        off_b = (size_t)ks * adv_b; vb = vb0 - ks * dvb;
      },
      [&](const char* sa, const char* sb, int q0, int q1, int) { mma(sa, sb, q0, q1); }, static_cast<Prep&&>(prep));
}

// Software-pipelined, paced form of the two-stage ring for one output tile.  The product of a slab
// is KSTEPS fragment steps; ld(f, stageA, stageB, kk) reads the fragments of step kk into registers
// and mm(f, h) issues half h (0 / 1) of that step's MFMAs.  Two fragment sets alternate: the LDS
// reads of step kk + 1 are issued before the MFMAs of step kk, and the last step of a slab is
// multiplied after the next slab's barrier, behind the first fragment reads of that slab, so a
// wave meets one wait per slab (the barrier) instead of an LDS round trip with idle matrix cores
// at every half slab (what the compiler makes of ring_pipeline_pp: read, wait, 8 MFMAs per step).
// Every wave issues its equal share of the next slab's asynchronous loads in four quarters,
// between the MFMA groups of the first two steps after the barrier, instead of half of the waves
// issuing everything at once.  Fragments of the stage being left are all in registers
// (lgkmcnt(0)) before a wave arrives at the barrier that lets other waves overwrite that stage.
// NRD / NMM: LDS reads per ld() and MFMAs per step; the scheduler is told to issue a step's reads
// ahead of the MFMAs they overlap with (it otherwise sinks them behind the MFMAs to save registers).
// Measured on the update product (per chunk of the 3M-label FP8 head, B = 1024): 282 us with
// ring_pipeline_pp, 274 us software-pipelined with the early / late split, 267 us paced.  What
// bounds the loop is the round trip of a slab's loads (about 3 k clocks for 64 KiB whether or not
// the lines are already in L2; the same loop without MFMAs and fragment reads takes 0.8 of the
// full loop's time, without loads 0.65), and 160 KiB of LDS do not hold a third 64 KiB stage.
template <int NRD, int NMM> __device__ __forceinline__ void sched_reads_then_mfma() {
  __builtin_amdgcn_sched_group_barrier(0x100, NRD, 0);
  __builtin_amdgcn_sched_group_barrier(0x008, NMM, 0);
}
template <int AROWS, int AROWB, int BROWS, int BROWB, int NW, int KSTEPS, int NRD, int NMM, class F, class Ld, class Mm>
__device__ inline void ring_pipeline_paced(const char* __restrict__ ga, size_t stride_a, int va0, int dva, size_t adv_a, int chunks_a,
                                           const char* __restrict__ gb, size_t stride_b, int vb0, int dvb, size_t adv_b, int chunks_b,
                                           int nk, char* smem, int wave, int lane, Ld&& ld, Mm&& mm) {
  static_assert(KSTEPS >= 2 && KSTEPS % 2 == 0, "fragment steps come in pairs");
  constexpr int ABYTES = AROWS * AROWB, SBYTES = ABYTES + BROWS * BROWB;
  constexpr int NA = dma_loads_per_wave<AROWS, AROWB, NW>(), NB = dma_loads_per_wave<BROWS, BROWB, NW>();
  static_assert(NA % 2 == 0 && NB % 2 == 0, "loads are issued in four quarters");
  auto issue_a = [&](int ks, auto half) {
    constexpr int H = decltype(half)::value;
    dma_tile<AROWS, AROWB, NW, H * NA / 2, (H + 1) * NA / 2>(ga + (size_t)ks * adv_a, stride_a, va0 - ks * dva, smem + (ks & 1) * SBYTES, wave, lane, chunks_a);
  };
  auto issue_b = [&](int ks, auto half) {
    constexpr int H = decltype(half)::value;
    dma_tile<BROWS, BROWB, NW, H * NB / 2, (H + 1) * NB / 2>(gb + (size_t)ks * adv_b, stride_b, vb0 - ks * dvb, smem + (ks & 1) * SBYTES + ABYTES, wave, lane, chunks_b);
  };
  using H0 = std::integral_constant<int, 0>;
  using H1 = std::integral_constant<int, 1>;
  issue_a(0, H0{}); issue_a(0, H1{}); issue_b(0, H0{}); issue_b(0, H1{});
  F f0, f1;
  for (int ks = 0; ks < nk; ++ks) {
    wait_vmcnt<0>();
    barrier_nofence();
    const bool more = ks + 1 < nk;
    const char* sa = smem + (ks & 1) * SBYTES;
    const char* sb = sa + ABYTES;
    __builtin_amdgcn_sched_barrier(0);
    ld(f0, sa, sb, 0);
    if (ks > 0) {                          // last step of the slab before, behind this slab's first reads
      mm(f1, 0);
      sched_reads_then_mfma<NRD, NMM / 2>();
      __builtin_amdgcn_sched_barrier(0);
      if (more) issue_a(ks + 1, H0{});
      __builtin_amdgcn_sched_barrier(0);
      mm(f1, 1);
      __builtin_amdgcn_sched_barrier(0);
      if (more) issue_a(ks + 1, H1{});
    } else if (more) {
      issue_a(ks + 1, H0{});
      issue_a(ks + 1, H1{});
    }
    __builtin_amdgcn_sched_barrier(0);
    ld(f1, sa, sb, 1);
    mm(f0, 0);
    sched_reads_then_mfma<NRD, NMM / 2>();
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue_b(ks + 1, H0{});
    __builtin_amdgcn_sched_barrier(0);
    mm(f0, 1);
    __builtin_amdgcn_sched_barrier(0);
    if (more) issue_b(ks + 1, H1{});
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int kk = 2; kk < KSTEPS; kk += 2) {
      ld(f0, sa, sb, kk);
      mm(f1, 0); mm(f1, 1);
      sched_reads_then_mfma<NRD, NMM>();
      __builtin_amdgcn_sched_barrier(0);
      ld(f1, sa, sb, kk + 1);
      mm(f0, 0); mm(f0, 1);
      sched_reads_then_mfma<NRD, NMM>();
      __builtin_amdgcn_sched_barrier(0);
    }
    __builtin_amdgcn_s_waitcnt(0xC07F);    // lgkmcnt(0): every fragment of this stage is in registers
  }
  mm(f1, 0); mm(f1, 1);
  barrier_nofence();   // every wave is done with the ring: the caller may reuse the memory
}

// ---------------------------------------------------------------------------------------------
// K-contiguous operands (rows of ROWB bytes = one K slab).
// BF16, v_mfma_f32_32x32x16_bf16: lane i holds row i%32, K elements 8*(i/32) .. +7 of the step.
// ---------------------------------------------------------------------------------------------
template <int ROWB = 128> __device__ inline bf16x8 frag_bf16(const char* lds, int row0, int kstep, int lane) {
  const int r = row0 + (lane & 31);
  return *reinterpret_cast<const bf16x8*>(lds + tile_off<ROWB>(r, 2 * kstep + (lane >> 5)));
}
// FP8, v_mfma_f32_32x32x64_f8f6f4: lane i holds row i%32, K bytes 32*(i/32) .. +31 of the step.
template <int ROWB = 128> __device__ inline i32x8 frag_fp8(const char* lds, int row0, int kstep, int lane) {
  const int r = row0 + (lane & 31);
  const int c = 4 * kstep + 2 * (lane >> 5);
  const i32x4 lo = *reinterpret_cast<const i32x4*>(lds + tile_off<ROWB>(r, c));
  const i32x4 hi = *reinterpret_cast<const i32x4*>(lds + tile_off<ROWB>(r, c + 1));
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
