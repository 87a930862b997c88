// Replica-batched ("grouped") bf16 GEMM on the gfx950 matrix cores.
//
//   C[g][m][n] = sum_k A[g][m][k] * B[g][n][k],   g = replica
//
// covers the contractions of one local step (Alg. 1 of the paper, "compute the local batch
// gradient"): forward  a W^T, backward-data  delta W, weight gradient  delta^T a, and the extra
// contraction  a Gbar^T  of the inner-product statistics.  Either operand may be stored
// k-contiguous (memory [row][k]) or row-contiguous (memory [k][row]).
//
// Data path (no operand ever passes through vector registers on its way to LDS):
//   * global -> LDS with `buffer_load_dwordx4 ... lds` (16 bytes per lane, written by the
//     memory pipeline at M0 + 16*lane), NS stage buffers in a ring; out-of-range chunks come
//     back as zeros through the buffer descriptor's range check, so ragged m / n / k need no
//     branches.  A stage's loads are spread over the MFMA groups of the previous stage so that
//     a wavefront never sits in the memory-issue queue while the matrix pipe idles.
//   * k-contiguous tiles are kept as [row][BK] with the 16-byte chunk index XOR-swizzled by the
//     row (the permutation is applied on the global-address side, since the LDS side of a
//     direct load is linear in the lane id); an MFMA fragment is one ds_read_b128.
//   * row-contiguous tiles are kept as [k][rows] and read with ds_read_b64_tr_b16, the LDS
//     transpose read: inside each group of 16 lanes, lane i receives element (i % 4) of the
//     8-byte vectors addressed by lanes i/4, i/4 + 4, i/4 + 8, i/4 + 12 -- i.e. four
//     consecutive k for its own row when lane j addresses (k = j / 4, rows 4 (j % 4) ..+3).
//   * one s_barrier per k-tile; s_waitcnt vmcnt(n) lets the younger stages stay in flight.
//
// Tiling: BM x BN x BK block tile, WM x WN wavefronts of 64 lanes, each a grid of 32x32x16
// bf16 MFMAs with fp32 accumulators.  Work-group ids are remapped so that each XCD (ids are
// dealt round-robin to the 8 XCDs) works on a contiguous range of tiles and its L2 sees one
// replica's operands at a time.
#include <mutex>
#include "abs_internal.h"
#include "device_utils.h"

namespace absk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef __attribute__((address_space(3))) void lds_void;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

namespace {

// Epilogue outputs and the elementwise operand are touched once per launch: non-temporal accesses
// keep them from displacing the operand tiles that other work-groups of the launch re-read from L2.
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 ld_once(const bf16_t *p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_once(bf16_t *p, uint4 v) {
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ void st_once(bf16_t *p, uint2 v) {
  const u32x2_t w = {v.x, v.y};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x2_t *>(p));
}
__device__ __forceinline__ float4 ld_once(const float *p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_once(float *p, float4 v) {
  const f32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t *>(p));
}

constexpr uint32_t OOB = 0x80000000u;   // byte offset beyond any operand (operands are < 2 GiB)

template <int N> __device__ __forceinline__ void wait_vmcnt() {
  // s_waitcnt immediate on gfx9: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[5:4] at [15:14]
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// ---- one operand's stage: addressing of the direct loads and of the fragment reads ---------
// ROWS = tile extent along m (or n); TRANS = memory is [k][row].
template <int ROWS, int BK, bool TRANS, int NW>
struct Operand {
  static constexpr int ELEMS = ROWS * BK;                 // bf16 elements per stage
  static constexpr int NI = ELEMS / 8 / 64 / NW;          // load instructions per wave per stage
  static_assert(ELEMS % (8 * 64 * NW) == 0 && NI >= 1, "tile too small for the wave count");
  static constexpr int CPR = BK / 8;                      // k-contiguous: chunks per row
  static constexpr int SWS = CPR >= 8 ? 1 : 2;
  static constexpr int CH = ROWS / 8;                     // row-contiguous: chunks per k-row
  static_assert(!TRANS || CH >= 8, "transposed tiles need at least 64 rows");

  uint32_t voff[NI];     // per-lane byte offset of its chunk at k0 = 0 (OOB if the row is outside)
  int kofs[NI];          // k (relative to k0) of the chunk, for the ragged last k-tile

  __device__ __forceinline__ void init(int wave, int lane, int row0, int rows, int ld) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int c = (wave * NI + i) * 64 + lane;          // linear 16-byte chunk index in the stage
      if (!TRANS) {
        const int row = c / CPR, kc = (c % CPR) ^ ((row >> SWS) & (CPR - 1));
        kofs[i] = kc * 8;
        voff[i] = (row0 + row < rows) ? (uint32_t)((row0 + row) * ld + kc * 8) * 2u : OOB;
      } else {
        const int kq = c / CH, ch = (c % CH) ^ ((4 * (kq & 3)) & (CH - 1));
        kofs[i] = kq;
        voff[i] = (row0 + ch * 8 < rows) ? (uint32_t)(kq * ld + row0 + ch * 8) * 2u : OOB;
      }
    }
  }
  // byte offset added for k-tile kt (scalar)
  static __device__ __forceinline__ uint32_t soff(int kt, int ld) {
    return TRANS ? (uint32_t)kt * BK * ld * 2u : (uint32_t)kt * BK * 2u;
  }
  // i is a compile-time constant after unrolling (voff / kofs live in registers)
  __device__ __forceinline__ void load(int i, __amdgpu_buffer_rsrc_t rsrc, bf16_t *stage, int wave, int kt,
                                       int K, int ld, bool full) const {
    uint32_t v = voff[i];
    if (!full && kt * BK + kofs[i] >= K) v = OOB;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void *)(stage + (wave * NI + i) * 512), 16, v,
                                             soff(kt, ld), 0, 0);
  }
};

// fragment of rows [r0, r0+32) for k-step kk of a stage
template <int ROWS, int BK, bool TRANS>
struct Frag {
  static constexpr int CPR = BK / 8, SWS = CPR >= 8 ? 1 : 2, CH = ROWS / 8;
  int base, swz;         // !TRANS: element offset of the row, and its swizzle
  int tbase[2];          // TRANS: element offsets for the two transpose reads at kk = 0
  __device__ __forceinline__ void init(int r0, int lane) {
    if (!TRANS) {
      const int r = r0 + (lane & 31);
      base = r * BK;
      swz = (r >> SWS) & (CPR - 1);
    } else {
      const int i16 = lane & 15, g16 = lane >> 4;
      const int rr = r0 + (g16 & 1) * 16 + 4 * (i16 & 3);     // first of this lane's 4 rows
      const int kq = (g16 >> 1) * 8 + (i16 >> 2);             // k within the 16-wide step
      // the chunk swizzle 4*(k&3) does not depend on kk (16 | step) nor on the +4 of the 2nd read.
      // A 32-lane half of the read covers 4 values of k x 4 chunks (16 bytes each, two lanes per
      // chunk): XOR-ing k&3 into chunk bits 2..3 spreads these 16 chunks over all 64 banks.
      const int ch = (rr >> 3) ^ ((4 * (kq & 3)) & (CH - 1));
      tbase[0] = kq * ROWS + ch * 8 + (rr & 7);
      tbase[1] = tbase[0] + 4 * ROWS;
    }
  }
  __device__ __forceinline__ bf16x8 read(const bf16_t *stage, int kk) const {
    if (!TRANS) {
      const int kc = kk * 2 + (threadIdx.x >> 5 & 1);
      return *reinterpret_cast<const bf16x8 *>(stage + base + ((kc ^ swz) << 3));
    } else {
      // Issued as inline assembly: through the builtin the compiler cannot tell that this read
      // does not alias the direct-to-LDS loads in flight (they fill the other stage buffer) and
      // puts s_waitcnt vmcnt(0) in front of every group of reads, which serialises the pipeline.
      // The price is that the compiler no longer counts these reads in lgkmcnt: the main loop
      // waits for them itself (wait_frags) before the MFMAs that use them.
      const uint32_t a0 = (uint32_t)(uintptr_t)(lds_void *)(stage + tbase[0] + kk * 16 * ROWS);
      const uint32_t a1 = (uint32_t)(uintptr_t)(lds_void *)(stage + tbase[1] + kk * 16 * ROWS);
      s16x4 lo, hi;
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(lo) : "v"(a0) : "memory");
      asm volatile("ds_read_b64_tr_b16 %0, %1" : "=v"(hi) : "v"(a1) : "memory");
      const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
      return __builtin_bit_cast(bf16x8, v);
    }
  }
};

// Wait until at most N LDS operations of this wave are outstanding, and make the fragments that
// the following MFMAs read depend on that wait (needed where fragment reads are inline assembly).
template <int N, int MI, int NI>
__device__ __forceinline__ void wait_frags(bf16x8 (&a)[MI], bf16x8 (&b)[NI]) {
  static_assert(N >= 0 && N <= 15, "lgkmcnt range");
  __builtin_amdgcn_s_waitcnt(0xC07F | (N << 8));          // vmcnt, expcnt: no wait; lgkmcnt = N
#pragma unroll
  for (int i = 0; i < MI; ++i) asm volatile("" : "+v"(a[i]));
#pragma unroll
  for (int j = 0; j < NI; ++j) asm volatile("" : "+v"(b[j]));
}

// ---- the kernel --------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, int NS, bool AT, bool BT, int EPI, int ACT>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_bf16_kernel(const GemmP pin, const int tilesM, const int tilesN, const int nblk, const int chunk) {
  constexpr int NW = WM * WN, NT = NW * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr bool IS_WGRAD = EPI == EPI_WGRAD || EPI == EPI_WGRAD_UPD;   // _UPD: ACT carries the optimizer
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int STAGE = (BM + BN) * BK;                 // bf16 elements per stage
  constexpr int NPART = BK / 16;                        // MFMA groups per k-tile
  static_assert(TM % 32 == 0 && TN % 32 == 0 && BK % 16 == 0 && NS >= 2, "tile shape");
  typedef Operand<BM, BK, AT, NW> OpA;
  typedef Operand<BN, BK, BT, NW> OpB;
  constexpr int NL = OpA::NI + OpB::NI;                 // load instructions per wave per stage
  static_assert((NS - 2) * NL <= 63, "vmcnt range");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);

  // XCD-aware remap of the flat work-group id
  const int bid = blockIdx.x;
  const int lb = (bid & 7) * chunk + (bid >> 3);
  if (lb >= nblk) return;
  const int per_g = tilesM * tilesN;
  const int vg = lb / per_g;                      // group, or (group, k-slice) pair of a split reduction
  const int t = lb - vg * per_g;
  const int ksplit = (EPI == EPI_WGRAD && pin.ksplit > 1) ? pin.ksplit : 1;   // (no split with the step fused)
  const int gv = vg / ksplit, ksl = vg - gv * ksplit;
  const int g = pin.gperm ? pin.gperm[gv] : gv;   // position in the launch order -> group
  const int tm = t / tilesN, tn = t - tm * tilesN;
  const int m0 = tm * BM, n0 = tn * BN;
  GemmP p = pin;
  if (p.rows) {                                   // ragged groups: this group's own extent
    const int r = p.rows[g];
    if (p.rows_is_k) { p.Kd = r; p.alpha = 1.0f / (float)r; } else p.Md = r;
    if (m0 >= p.Md) return;                       // uniform over the block, before any barrier
  }
  long long kofsA = 0, kofsB = 0;                 // element offsets of this block's k-slice
  if (EPI == EPI_WGRAD && ksplit > 1) {
    const int k0 = ksl * p.kchunk;
    int kd = p.Kd - k0;
    kd = kd < 0 ? 0 : (kd > p.kchunk ? p.kchunk : kd);
    p.Kd = kd;                                    // an empty slice runs no k-tile and writes zeros
    kofsA = AT ? (long long)k0 * p.lda : k0;
    kofsB = BT ? (long long)k0 * p.ldb : k0;
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave / WN, wn = wave % WN;

  const bf16_t *A = static_cast<const bf16_t *>(p.A) + (long long)g * p.sAg + kofsA;
  const bf16_t *B = static_cast<const bf16_t *>(p.B) + (long long)g * p.sBg + kofsB;
  // range = the operand's extent in memory: rows*ld (k-contiguous) or K*ld (row-contiguous)
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t *>(A), 0, (int)((long long)(AT ? p.Kd : p.Md) * p.lda * 2), 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<bf16_t *>(B), 0, (int)((long long)(BT ? p.Kd : p.Nd) * p.ldb * 2), 0x00020000);

  OpA oa;
  OpB ob;
  oa.init(wave, lane, m0, p.Md, p.lda);
  ob.init(wave, lane, n0, p.Nd, p.ldb);

  // issue the loads of stage-slot `buf` for k-tile kt whose index l satisfies l % NPART == part
  auto issue = [&](int kt, int buf, int part) {
    bf16_t *sa = smem + buf * STAGE, *sb = sa + BM * BK;
    const bool full = (kt + 1) * BK <= p.Kd;
#pragma unroll
    for (int l = 0; l < NL; ++l) {
      if (l % NPART != part) continue;
      if (l < OpA::NI) oa.load(l, ra, sa, wave, kt, p.Kd, p.lda, full);
      else ob.load(l - OpA::NI, rb, sb, wave, kt, p.Kd, p.ldb, full);
    }
  };

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  Frag<BM, BK, AT> fa[MI];
  Frag<BN, BK, BT> fb[NI];
#pragma unroll
  for (int i = 0; i < MI; ++i) fa[i].init(wm * TM + i * 32, lane);
#pragma unroll
  for (int j = 0; j < NI; ++j) fb[j].init(wn * TN + j * 32, lane);

  // Fused optimizer step (EPI_WGRAD_UPD): the epilogue walks this wave's slices (32 rows x TN columns) in batches of
  // UHB 16-byte chunks per lane, and the loads of batch k + 1 (parameters and optimizer state) are issued before
  // batch k is processed, so that a wave always has a batch of loads in flight while it computes and stores.
  // (Four chunks for the 128 x 128 and 64 x 256 tiles: config 3 at b = 64 2.4 % faster than with two, b = 256
  // unchanged; the 256 x 256 tile has no registers to spare for more than two.)
  constexpr bool UPD = EPI == EPI_WGRAD_UPD;
  constexpr int UFCPR = TN / 4;                             // float4 chunks per slice row
  constexpr int UFIT = 32 * UFCPR / 64;                     // chunks per lane per slice
  constexpr int UHBW = ((BM == 128 && BN == 128) || BM == 64) ? 4 : 2;
  constexpr int UHB = UFIT < UHBW ? UFIT : UHBW;
  constexpr int UBPS = UFIT / UHB;
  static_assert(!UPD || UFIT % UHB == 0, "chunk batches");
  // The 128 x 128 and 64 x 256 tiles (short batches: a launch is all epilogue) issue the first batch before the operand loads of
  // the reduction, so that its latency passes behind the main loop; being older than every operand load, these
  // loads do not disturb the counting of the main loop's waits (loads return in order).
  constexpr bool UPD_EARLY = UPD && ((BM == 128 && BN == 128) || BM == 64);
  float4 xq[2][UPD ? UHB : 1], vq[2][UPD ? UHB : 1], mq[2][UPD ? UHB : 1];
  const long long ugoff = UPD ? (long long)g * p.sCg : 0;
  auto upd_where = [&](int bi, int u, int &m, int &n, int &row, int &cc) {
    const int c = ((bi % UBPS) * UHB + u) * 64 + lane;
    row = c / UFCPR; cc = c % UFCPR;
    m = m0 + wm * TM + (bi / UBPS) * 32 + row;
    n = n0 + wn * TN + cc * 4;
  };
  auto upd_prefetch = [&](int bi) {
    if constexpr (UPD) {
#pragma unroll
      for (int u = 0; u < UHB; ++u) {
        int m, n, row, cc;
        upd_where(bi, u, m, n, row, cc);
        xq[bi & 1][u] = vq[bi & 1][u] = mq[bi & 1][u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (m < p.Md && n < p.Nd) {                          // Nd is a multiple of 4 (checked by the launcher)
          const long long o = ugoff + (long long)m * p.ldc + n;
          xq[bi & 1][u] = ld_once(p.upd_x + o);
          if (ACT != OPT_SGD) vq[bi & 1][u] = ld_once(p.upd_v + o);       // (the optimizer travels in the activation slot)
          if (ACT == OPT_ADAMW) mq[bi & 1][u] = ld_once(p.upd_m + o);
        }
      }
    }
  };
  if constexpr (UPD_EARLY) upd_prefetch(0);

  const int KT = (p.Kd + BK - 1) / BK;
#pragma unroll
  for (int s = 0; s < NS - 1; ++s) {
    if (s < KT) {
#pragma unroll
      for (int q = 0; q < NPART; ++q) issue(s, s, q);
    }
  }

  for (int kt = 0; kt < KT; ++kt) {
    // k-tile kt has landed once only the loads of the younger in-flight stages are outstanding
    if (kt + NS - 1 <= KT) wait_vmcnt<(NS - 2) * NL>(); else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();      // all waves' loads of kt visible; everyone is done with kt-1
    const bool more = kt + NS - 1 < KT;
    const bf16_t *S = smem + (kt % NS) * STAGE;
    // fragments are double-buffered in registers: the LDS reads of MFMA group kk+1 and this
    // group's share of the next stage's global loads are issued before the MFMAs of group kk,
    // which then run as one raised-priority cluster
    bf16x8 af[2][MI], bfr[2][NI];
    // transpose reads (untracked by the compiler's lgkmcnt accounting) go first, so that the
    // newest outstanding reads are always the ones the compiler counts
    if (BT && !AT) {
#pragma unroll
      for (int j = 0; j < NI; ++j) bfr[0][j] = fb[j].read(S + BM * BK, 0);
    }
#pragma unroll
    for (int i = 0; i < MI; ++i) af[0][i] = fa[i].read(S, 0);
    if (!(BT && !AT)) {
#pragma unroll
      for (int j = 0; j < NI; ++j) bfr[0][j] = fb[j].read(S + BM * BK, 0);
    }
#pragma unroll
    for (int kk = 0; kk < NPART; ++kk) {
      const int cur = kk & 1, nxt = cur ^ 1;
      if (kk + 1 < NPART) {
        if (BT && !AT) {
#pragma unroll
          for (int j = 0; j < NI; ++j) bfr[nxt][j] = fb[j].read(S + BM * BK, kk + 1);
        }
#pragma unroll
        for (int i = 0; i < MI; ++i) af[nxt][i] = fa[i].read(S, kk + 1);
        if (!(BT && !AT)) {
#pragma unroll
          for (int j = 0; j < NI; ++j) bfr[nxt][j] = fb[j].read(S + BM * BK, kk + 1);
        }
      }
      if (more) issue(kt + NS - 1, (kt + NS - 1) % NS, kk);
      if (AT || BT) {
        // LDS reads issued per MFMA group (transpose reads count two per fragment); the reads of
        // group kk + 1, if any, are the newest ones and may stay outstanding
        constexpr int RD = (AT ? 2 : 1) * MI + (BT ? 2 : 1) * NI;
        if (kk + 1 < NPART) wait_frags<RD>(af[cur], bfr[cur]); else wait_frags<0>(af[cur], bfr[cur]);
      }
      __builtin_amdgcn_sched_barrier(0);
      __builtin_amdgcn_s_setprio(1);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          // operands swapped: the accumulator tile is C^T, so a lane owns one row m of C and
          // groups of four consecutive columns n (see the epilogue)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[cur][j], af[cur][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_s_setprio(0);
      __builtin_amdgcn_sched_barrier(0);
    }
  }

  // ---- epilogue.  With the operands swapped in the MFMA, accumulator element r = 4q + e of tile
  // (i, j) belongs to   row  m = wm*TM + 32 i + lane % 32,
  //                     col  n = wn*TN + 32 j + 8 q + 4 (lane / 32) + e      (tile-relative),
  // i.e. a lane holds four consecutive columns per q.  bf16 outputs and the elementwise operand E
  // go through a per-wave LDS staging slice of 32 rows x TN columns, so that every global access
  // of the epilogue is a 16-byte vector, 8 lanes to a 128-byte row segment.
  const int lcol = lane & 31, lhalf = lane >> 5;
  const float *bias = p.bias ? p.bias + (long long)g * p.sBiasg : nullptr;
  constexpr int SLD = TN + 8;                               // staging row stride (elements)
  bf16_t *stg = smem + wave * (32 * SLD);
  constexpr int CPRW = TN / 8;                              // 16-byte chunks per staged row
  constexpr int SIT = 32 * CPRW / 64;                       // chunks per lane per slice
  static_assert(32 * CPRW % 64 == 0, "staging slice");
  const int nw0 = n0 + wn * TN;                             // first column of this wave
  const bool nfull = n0 + BN <= p.Nd;                       // no ragged columns in this tile (uniform)
  // this lane's 4-column groups of the bias vector, loaded once for all row slices
  float bv[NI][4][4];
  if (EPI == EPI_FWD_ACT || EPI == EPI_IPDOT || EPI == EPI_LOGITS) {
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nw0 + j * 32 + q * 8 + lhalf * 4;
        if (bias && nfull) {
          const float4 b4 = *reinterpret_cast<const float4 *>(bias + n);
          bv[j][q][0] = b4.x; bv[j][q][1] = b4.y; bv[j][q][2] = b4.z; bv[j][q][3] = b4.w;
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e) bv[j][q][e] = (bias && n + e < p.Nd) ? bias[n + e] : 0.0f;
        }
      }
  }

  // rows [mrow0, mrow0+32) x this wave's TN columns of a bf16 matrix: global -> registers (so the
  // next slice can be in flight while the current one is processed), registers -> staging
  auto load_slice = [&](const bf16_t *src, int ld, int mrow0, int ncols, uint4 (&r)[SIT]) {
#pragma unroll
    for (int it = 0; it < SIT; ++it) {
      const int c = it * 64 + lane, row = c / CPRW, cc = c % CPRW;
      r[it] = make_uint4(0, 0, 0, 0);
      if (mrow0 + row < p.Md && nw0 + cc * 8 < ncols)
        r[it] = ld_once(src + (long long)(mrow0 + row) * ld + nw0 + cc * 8);
    }
  };
  auto put_slice = [&](const uint4 (&r)[SIT]) {
#pragma unroll
    for (int it = 0; it < SIT; ++it) {
      const int c = it * 64 + lane, row = c / CPRW, cc = c % CPRW;
      *reinterpret_cast<uint4 *>(stg + row * SLD + cc * 8) = r[it];
    }
  };
  uint4 ereg[2][SIT];
  const bf16_t *Eg = p.E ? static_cast<const bf16_t *>(p.E) + (long long)g * p.sEg : nullptr;
  constexpr bool USES_E = EPI == EPI_IPDOT || (EPI == EPI_BWD && ACT != ACT_NONE);
  if (USES_E) load_slice(Eg, p.lde, m0 + wm * TM, p.Nd, ereg[0]);
  // staging -> global
  auto stage_out = [&](bf16_t *dst, int ld, int mrow0, int ncols) {
#pragma unroll
    for (int it = 0; it < SIT; ++it) {
      const int c = it * 64 + lane, row = c / CPRW, cc = c % CPRW;
      const uint4 v = *reinterpret_cast<const uint4 *>(stg + row * SLD + cc * 8);
      if (mrow0 + row < p.Md && nw0 + cc * 8 < ncols)
        st_once(dst + (long long)(mrow0 + row) * ld + nw0 + cc * 8, v);
    }
  };
  auto piece = [&](int j, int q) -> bf16_t * { return stg + lcol * SLD + j * 32 + q * 8 + lhalf * 4; };

  if (EPI == EPI_FWD_ACT || EPI == EPI_BWD || EPI == EPI_IPDOT) __syncthreads();   // stages are dead
  static_assert(32 * (TN / 4) % 64 == 0, "fp32 staging slice");

  float *red = reinterpret_cast<float *>(smem + NW * 32 * SLD);   // [WN][BM] row partials of the waves
  // add the WN waves' row partials in wave order and write part[g][tn][m]
  auto finish_rows = [&]() {
    __syncthreads();
    float *part = p.part + (long long)g * p.sPartg + (long long)tn * p.sPartTile;
    for (int r = tid; r < BM; r += NT) {
      float v = 0.0f;
#pragma unroll
      for (int w = 0; w < WN; ++w) v += red[w * BM + r];
      if (m0 + r < p.Md) part[m0 + r] = v;
    }
  };
  // squares of the four bf16 values packed in pk
  auto sq4 = [](uint2 pk) -> float {
    const float a = __uint_as_float(pk.x << 16), b = __uint_as_float(pk.x & 0xffff0000u);
    const float c = __uint_as_float(pk.y << 16), d = __uint_as_float(pk.y & 0xffff0000u);
    return fmaf(a, a, fmaf(b, b, fmaf(c, c, d * d)));
  };

  if (EPI == EPI_IPDOT) {
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int mrow0 = m0 + wm * TM + i * 32;
      if (i + 1 < MI) load_slice(Eg, p.lde, mrow0 + 32, p.Nd, ereg[(i + 1) & 1]);
      put_slice(ereg[i & 1]);
      float rs = 0.0f;
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const uint2 ev = *reinterpret_cast<const uint2 *>(piece(j, q));
          const float e4[4] = {__uint_as_float(ev.x << 16), __uint_as_float(ev.x & 0xffff0000u),
                               __uint_as_float(ev.y << 16), __uint_as_float(ev.y & 0xffff0000u)};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            rs = fmaf(e4[e], acc[i][j][4 * q + e] + bv[j][q][e], rs);   // E is zero outside the matrix
          }
        }
      rs += __shfl_xor(rs, 32, 64);                               // the two column halves of the row
      if (lhalf == 0) red[wn * BM + wm * TM + i * 32 + lcol] = rs;
    }
    finish_rows();
    return;
  }

  if (EPI == EPI_FWD_ACT) {
    bf16_t *C = static_cast<bf16_t *>(p.C) + (long long)g * p.sCg;
    bf16_t *C2 = p.C2 ? static_cast<bf16_t *>(p.C2) + (long long)g * p.sC2g : nullptr;
    const int ncols = p.pad_to_ld ? p.ldc : p.Nd;           // pad columns are written as zeros
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int mrow0 = m0 + wm * TM + i * 32;
      uint2 dpk[NI][4];
      float rs = 0.0f;
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float a4[4], d4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            // columns beyond Nd: accumulator and bias are both zero there (operand rows past the
            // matrix read as zeros), so phi(0) = 0 is what the pad columns of C receive
            act_fwd<ACT>(acc[i][j][4 * q + e] + bv[j][q][e], a4[e], d4[e]);
          }
          uint2 apk;
          apk.x = pack2bf(a4[0], a4[1]); apk.y = pack2bf(a4[2], a4[3]);
          dpk[j][q].x = pack2bf(d4[0], d4[1]); dpk[j][q].y = pack2bf(d4[2], d4[3]);
          *reinterpret_cast<uint2 *>(piece(j, q)) = apk;
          rs += sq4(apk);
        }
      if (p.part) {
        rs += __shfl_xor(rs, 32, 64);
        if (lhalf == 0) red[wn * BM + wm * TM + i * 32 + lcol] = rs;
      }
      stage_out(C, p.ldc, mrow0, ncols);
      if (ACT == ACT_GELU && C2) {
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) *reinterpret_cast<uint2 *>(piece(j, q)) = dpk[j][q];
        stage_out(C2, p.ldc2, mrow0, ncols);
      }
    }
    if (p.part) finish_rows();
    return;
  }

  if (EPI == EPI_BWD) {
    bf16_t *C = static_cast<bf16_t *>(p.C) + (long long)g * p.sCg;
    const int ncols = p.pad_to_ld ? p.ldc : p.Nd;
    static_assert(TN % 64 == 0 || TN == 32, "column sums: lanes map to columns");
    float cs[(TN + 63) / 64];                            // column sums over this wave's rows, one column per lane
#pragma unroll
    for (int c = 0; c < (TN + 63) / 64; ++c) cs[c] = 0.0f;
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      const int mrow0 = m0 + wm * TM + i * 32;
      if (ACT != ACT_NONE) {
        if (i + 1 < MI) load_slice(Eg, p.lde, mrow0 + 32, p.Nd, ereg[(i + 1) & 1]);
        put_slice(ereg[i & 1]);
      }
      float rs = 0.0f;
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          float e4[4] = {1.0f, 1.0f, 1.0f, 1.0f};
          if (ACT != ACT_NONE) {
            const uint2 ev = *reinterpret_cast<const uint2 *>(piece(j, q));
            e4[0] = __uint_as_float(ev.x << 16); e4[1] = __uint_as_float(ev.x & 0xffff0000u);
            e4[2] = __uint_as_float(ev.y << 16); e4[3] = __uint_as_float(ev.y & 0xffff0000u);
          }
          float o4[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float v = acc[i][j][4 * q + e];
            o4[e] = (ACT == ACT_RELU) ? (e4[e] > 0.0f ? v : 0.0f) : (ACT == ACT_GELU ? v * e4[e] : v);
            if (!nfull && nw0 + j * 32 + q * 8 + lhalf * 4 + e >= p.Nd) o4[e] = 0.0f;
          }
          uint2 opk;
          opk.x = pack2bf(o4[0], o4[1]); opk.y = pack2bf(o4[2], o4[3]);
          *reinterpret_cast<uint2 *>(piece(j, q)) = opk;      // each lane overwrites the piece it read
          rs += sq4(opk);
        }
      if (p.part) {
        rs += __shfl_xor(rs, 32, 64);
        if (lhalf == 0) red[wn * BM + wm * TM + i * 32 + lcol] = rs;
      }
      stage_out(C, p.ldc, mrow0, ncols);
      if (p.cpart) {
        // bias-gradient partials: a lane adds its column of the staged slice, rows in order (rows
        // past the batch were computed from zero operands and hold zeros)
#pragma unroll
        for (int c = 0; c < (TN + 63) / 64; ++c) {
          const int col = c * 64 + lane;
          if (col < TN) {
#pragma unroll
            for (int r = 0; r < 32; ++r) cs[c] += bf2f(stg[r * SLD + col]);
          }
        }
      }
    }
    if (p.cpart) {
      float *cp = p.cpart + (long long)g * p.sCpartg + (long long)(tm * WM + wm) * p.Nd;
#pragma unroll
      for (int c = 0; c < (TN + 63) / 64; ++c) {
        const int n = nw0 + c * 64 + lane;
        if (c * 64 + lane < TN && n < p.Nd) cp[n] = cs[c];
      }
    }
    if (p.part) finish_rows();
    return;
  }

  // fp32 outputs (weight gradient, logits).  A lane holds one row and groups of four columns, so
  // direct stores would scatter 16-byte pieces over 32 rows per instruction; instead each wave
  // passes its 32 x TN slice through an fp32 staging area in LDS and writes whole row segments
  // (16 lanes x 16 bytes = 256 contiguous bytes per row).
  constexpr int FLD = TN + 4;                               // staging row stride (floats)
  constexpr int FCPR = TN / 4;                              // float4 chunks per staged row
  constexpr int FIT = 32 * FCPR / 64;                       // chunks per lane per slice
  float *stf = reinterpret_cast<float *>(smem) + wave * (32 * FLD);
  float *Cg = static_cast<float *>(p.C) + (long long)g * p.sCg;
  bf16_t *C2g = (IS_WGRAD && p.C2) ? static_cast<bf16_t *>(p.C2) + (long long)g * p.sC2g : nullptr;
  bool accumulate = EPI == EPI_WGRAD && p.accumulate;        // micro-batch accumulation: C += alpha * acc
  if (EPI == EPI_WGRAD && ksplit > 1) {                      // raw partial product of this k-slice
    Cg = p.kpart + ((long long)g * ksplit + ksl) * p.Md * p.Nd;
    p.ldc = p.Nd; p.alpha = 1.0f;
    C2g = nullptr; accumulate = false;
  }
  const bool vec_ok = (p.ldc & 3) == 0 && (!C2g || (p.ldc2 & 3) == 0);
  __syncthreads();                                          // stages are dead
  if constexpr (EPI == EPI_WGRAD_UPD) {
    // The optimizer step in place of the gradient store: a lane's staged float4 holds four consecutive entries
    // of one row of Gbar_l; the parameters, their state and their bf16 shadow sit at the same offsets.
    const long long goff = (long long)g * p.sCg;
    float *X = p.upd_x + goff;                               // (loaded through upd_prefetch, stored through these)
    float *V = p.upd_v ? p.upd_v + goff : nullptr;
    float *Mo = p.upd_m ? p.upd_m + goff : nullptr;
    bf16_t *__restrict__ SH = p.upd_shadow ? p.upd_shadow + goff : nullptr;
    OptHyper h = {p.upd_lr, p.upd_momentum, p.upd_beta1, p.upd_beta2, p.upd_eps, p.upd_wd, p.upd_c1, p.upd_c2};
    if (p.upd_scal) { h.lr = p.upd_scal[0]; h.c1 = p.upd_scal[1]; h.c2 = p.upd_scal[2]; }     // uniform loads
    constexpr int opt = ACT;                                 // the optimizer travels in the activation slot
    float sq = 0.0f;
    constexpr int HB = UHB, BPS = UBPS, NBATCH = MI * BPS;
    auto &where = upd_where;
    auto &prefetch = upd_prefetch;
    if constexpr (!UPD_EARLY) prefetch(0);
#pragma unroll
    for (int bi = 0; bi < NBATCH; ++bi) {
      if (bi % BPS == 0) {                                   // a new slice: accumulators -> staging
        const int i = bi / BPS;
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const float4 o = make_float4(acc[i][j][4 * q] * p.alpha, acc[i][j][4 * q + 1] * p.alpha,
                                         acc[i][j][4 * q + 2] * p.alpha, acc[i][j][4 * q + 3] * p.alpha);
            *reinterpret_cast<float4 *>(stf + lcol * FLD + j * 32 + q * 8 + lhalf * 4) = o;
          }
      }
      if (bi + 1 < NBATCH) prefetch(bi + 1);
#pragma unroll
      for (int u = 0; u < HB; ++u) {
        int m, n, row, cc;
        where(bi, u, m, n, row, cc);
        if (m >= p.Md || n >= p.Nd) continue;
        const long long o = (long long)m * p.ldc + n;
        const float4 gv = *reinterpret_cast<const float4 *>(stf + row * FLD + cc * 4);
        const float gs[4] = {gv.x, gv.y, gv.z, gv.w};
        float xs[4] = {xq[bi & 1][u].x, xq[bi & 1][u].y, xq[bi & 1][u].z, xq[bi & 1][u].w};
        float vs[4] = {vq[bi & 1][u].x, vq[bi & 1][u].y, vq[bi & 1][u].z, vq[bi & 1][u].w};
        float ms[4] = {mq[bi & 1][u].x, mq[bi & 1][u].y, mq[bi & 1][u].z, mq[bi & 1][u].w};
#pragma unroll
        for (int e = 0; e < 4; ++e) opt_step_elem<opt>(xs[e], gs[e], vs[e], ms[e], h);
        sq = fmaf(gs[0], gs[0], fmaf(gs[1], gs[1], fmaf(gs[2], gs[2], fmaf(gs[3], gs[3], sq))));
        st_once(X + o, make_float4(xs[0], xs[1], xs[2], xs[3]));
        if (opt != OPT_SGD) st_once(V + o, make_float4(vs[0], vs[1], vs[2], vs[3]));
        if (opt == OPT_ADAMW) st_once(Mo + o, make_float4(ms[0], ms[1], ms[2], ms[3]));
        if (SH) {
          uint2 w;
          w.x = pack2bf(xs[0], xs[1]); w.y = pack2bf(xs[2], xs[3]);
          st_once(SH + o, w);
        }
        if (C2g) {
          uint2 w;
          w.x = pack2bf(gs[0], gs[1]); w.y = pack2bf(gs[2], gs[3]);
          st_once(C2g + (long long)m * p.ldc2 + n, w);
        }
      }
    }
    sq = wave_sum(sq);
    if (lane == 0) p.upd_sq[(long long)g * p.upd_sSqg + p.upd_slot0 + (long long)t * NW + wave] = sq;
    return;
  }
#pragma unroll
  for (int i = 0; i < MI; ++i) {
    const int mrow0 = m0 + wm * TM + i * 32;
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float4 o;
        if (IS_WGRAD) {
          o = make_float4(acc[i][j][4 * q] * p.alpha, acc[i][j][4 * q + 1] * p.alpha, acc[i][j][4 * q + 2] * p.alpha,
                          acc[i][j][4 * q + 3] * p.alpha);
        } else {
          o = make_float4(acc[i][j][4 * q] + bv[j][q][0], acc[i][j][4 * q + 1] + bv[j][q][1],
                          acc[i][j][4 * q + 2] + bv[j][q][2], acc[i][j][4 * q + 3] + bv[j][q][3]);
        }
        *reinterpret_cast<float4 *>(stf + lcol * FLD + j * 32 + q * 8 + lhalf * 4) = o;
      }
#pragma unroll
    for (int it = 0; it < FIT; ++it) {
      const int c = it * 64 + lane, row = c / FCPR, cc = c % FCPR;
      const int m = mrow0 + row, n = nw0 + cc * 4;
      if (m >= p.Md || n >= p.Nd) continue;
      float4 v = *reinterpret_cast<const float4 *>(stf + row * FLD + cc * 4);
      float *crow = Cg + (long long)m * p.ldc + n;
      if (n + 4 <= p.Nd && vec_ok) {
        if (accumulate) {
          const float4 old = *reinterpret_cast<const float4 *>(crow);
          v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
        }
        st_once(crow, v);
        if (C2g) {
          uint2 o;
          o.x = pack2bf(v.x, v.y); o.y = pack2bf(v.z, v.w);
          st_once(C2g + (long long)m * p.ldc2 + n, o);
        }
      } else {
        const float v4[4] = {v.x, v.y, v.z, v.w};
        for (int e = 0; e < 4; ++e) {
          if (n + e >= p.Nd) break;
          const float r = accumulate ? v4[e] + crow[e] : v4[e];
          crow[e] = r;
          if (C2g) C2g[(long long)m * p.ldc2 + n + e] = f2bf(r);
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN, int NS, bool AT, bool BT, int EPI, int ACT>
hipError_t launch_cfg(const GemmP &p, hipStream_t s) {
  constexpr int NT = WM * WN * 64;
  constexpr size_t tile_bytes = (size_t)NS * (BM + BN) * BK * sizeof(bf16_t);
  constexpr size_t epi_bf16 = (size_t)WM * WN * 32 * (BN / WN + 8) * sizeof(bf16_t) + (size_t)WN * BM * sizeof(float);
  constexpr size_t epi_f32 = (size_t)WM * WN * 32 * (BN / WN + 4) * sizeof(float);
  constexpr size_t epi_bytes = epi_bf16 > epi_f32 ? epi_bf16 : epi_f32;
  constexpr size_t lds = tile_bytes > epi_bytes ? tile_bytes : epi_bytes;
  static_assert(lds <= 160 * 1024, "LDS budget");
  auto kern = gemm_bf16_kernel<BM, BN, BK, WM, WN, NS, AT, BT, EPI, ACT>;
  // once per kernel variant, also when several host threads (each with a context of its own) launch it first together
  static std::once_flag attr_once;
  static hipError_t attr_err = hipSuccess;
  std::call_once(attr_once, [&] {
    attr_err = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  });
  if (attr_err != hipSuccess) return attr_err;
  const int tilesM = (p.Md + BM - 1) / BM, tilesN = (p.Nd + BN - 1) / BN;
  const long long nblk = (long long)tilesM * tilesN * p.groups * ((EPI == EPI_WGRAD && p.ksplit > 1) ? p.ksplit : 1);
  if (nblk <= 0) return hipSuccess;
  if (nblk > 0x3fffffff) return hipErrorInvalidValue;
  const int chunk = (int)((nblk + 7) / 8);
  hipLaunchKernelGGL(kern, dim3(chunk * 8), dim3(NT), lds, s, p, tilesM, tilesN, (int)nblk, chunk);
  return hipGetLastError();
}

// Tile shape by problem size: the large shape when both output extents fill it,
// otherwise a 128x128 (or 128x64 for narrow outputs, 64x128 for outputs of at most 64 rows) tile.
template <bool AT, bool BT, int EPI, int ACT>
hipError_t launch_shape(const GemmP &p, hipStream_t s) {
  constexpr bool IS_WGRAD = EPI == EPI_WGRAD || EPI == EPI_WGRAD_UPD;
  switch (IS_WGRAD ? gemm_bf16_wgrad_shape(p.Md, p.Nd, p.Kd, p.groups, p.upd_x != nullptr) : gemm_bf16_tile_shape(p.Md, p.Nd, p.groups)) {
    case 0: return launch_cfg<128, 64, 64, 4, 1, 3, AT, BT, EPI, ACT>(p, s);
    case 3:
      if constexpr (IS_WGRAD) return launch_cfg<64, 256, 32, 1, 4, 2, AT, BT, EPI, ACT>(p, s);
      else return hipErrorInvalidValue;
    case 2: return launch_cfg<256, 256, 64, 2, 4, 2, AT, BT, EPI, ACT>(p, s);
    case 4:
      if constexpr (!IS_WGRAD) return launch_cfg<64, 128, 64, 2, 2, 6, AT, BT, EPI, ACT>(p, s);
      else return hipErrorInvalidValue;
    default: {
      // Two stages (64 KB) let two work-groups share a CU; a deeper ring keeps one work-group fed through a long
      // reduction.  Two when the reduction is short or the launch has more blocks than CUs (measured: 2048-wide
      // layers at b = 256, 512 blocks: 43 against 62 us; 1024 blocks of a 100-wide output: 145 against 163 us;
      // 256 blocks: the deeper ring wins); four stages (128 KB, still one work-group per CU, three k-tiles in
      // flight: such launches are bound by the latency of their operand stream) otherwise.
      const long long nblk = (long long)((p.Md + 127) / 128) * ((p.Nd + 127) / 128) * p.groups *
                             ((EPI == EPI_WGRAD && p.ksplit > 1) ? p.ksplit : 1);
      if (p.Kd <= 1024 || nblk > 256) return launch_cfg<128, 128, 64, 2, 2, 2, AT, BT, EPI, ACT>(p, s);
      return launch_cfg<128, 128, 64, 2, 2, 4, AT, BT, EPI, ACT>(p, s);
    }
  }
}

template <bool AT, bool BT, int EPI>
hipError_t launch_act(const GemmP &p, hipStream_t s) {
  if constexpr (EPI == EPI_WGRAD_UPD) {          // the optimizer is a compile-time constant of the fused epilogue
    switch (p.upd_opt) {
      case OPT_SGD: return launch_shape<AT, BT, EPI, OPT_SGD>(p, s);
      case OPT_SHB: return launch_shape<AT, BT, EPI, OPT_SHB>(p, s);
      case OPT_ADAMW: return launch_shape<AT, BT, EPI, OPT_ADAMW>(p, s);
      case OPT_ADAGRAD: return launch_shape<AT, BT, EPI, OPT_ADAGRAD>(p, s);
      default: return hipErrorInvalidValue;
    }
  }
  if constexpr (EPI == EPI_FWD_ACT || EPI == EPI_BWD) {
    switch (p.act) {
      case ACT_RELU: return launch_shape<AT, BT, EPI, ACT_RELU>(p, s);
      case ACT_GELU: return launch_shape<AT, BT, EPI, ACT_GELU>(p, s);
      default: return launch_shape<AT, BT, EPI, ACT_NONE>(p, s);
    }
  }
  return launch_shape<AT, BT, EPI, ACT_NONE>(p, s);
}

}  // namespace

int gemm_bf16_tile_shape(int Md, int Nd, int groups) {
  if (Nd <= 64) return 0;
  // up to 64 rows (the first local batch sizes): the launch streams its B operand (the weights) once and is bound by
  // that stream; a 64-row tile leaves LDS for a ring of six stages, five k-tiles of B in flight per work-group
  // (config 3 at b = 64 against the 128 x 128 tile with four stages: forward 4.1 -> 4.3 TB/s of weight bytes,
  // backward-data 4.5 -> 5.0-5.1, the step 1.17 -> 1.155 ms)
  if (Md <= 64) return 4;
  if (Md >= 1024 && Nd >= 1024) return 2;
  // mid-sized outputs: the large tile only if it still gives every CU a work-group and its last row of tiles is
  // not mostly padding (measured on 2048-wide layers, 16 groups: b = 384 and 512 faster with 256 x 256 tiles,
  // b = 256 with two 128 x 128 work-groups per CU)
  if (Md >= 256 && Nd >= 512) {
    const long long tm = (Md + 255) / 256;
    const long long tiles = tm * ((Nd + 255) / 256) * groups;
    if (tiles >= 256 && 10LL * Md >= 7LL * tm * 256) return 2;
  }
  return 1;
}

// Weight gradients reduce over the local batch (Kd = b).  While the batch is short the launch is all epilogue
// (one or a few k-tiles, then 4 to 20 bytes of stores and loads per output entry): a 64 x 256 x 32 tile with two
// 20 KB stages lets several work-groups share a CU, which keeps far more memory requests in flight than one
// 256 x 256 work-group does; its four wavefronts sit side by side, so a work-group touches 1 KB of consecutive
// bytes in each of its 64 rows (measured against a 128 x 128 tile, 512 bytes in each of 128 rows, on config 3 at
// b = 64: 2 to 2.5 % faster with the optimizer step in the epilogue, equal at b = 256).
int gemm_bf16_wgrad_shape(int Md, int Nd, int Kd, int groups, int fused) {
  int sh = gemm_bf16_tile_shape(Md, Nd, groups);
  if (sh == 4) sh = 1;                       // (the short-batch tile of the other contractions)
  if (sh != 0 && Kd <= 256) return 3;        // (measured on config 3: at b = 384 and above the large tiles are faster)
  // with the optimizer step in the epilogue a medium batch is still mostly epilogue: two or three 128 x 128
  // work-groups per CU stream it better than one 256 x 256 work-group (config 3: b = 384 1.92 -> 1.87 ms per step,
  // b = 512 2.02 -> 2.00; from b = 768 on the large tile wins)
  if (fused && sh == 2 && Kd <= 512) return 1;
  return sh;
}

int gemm_bf16_upd_slots(int Md, int Nd, int Kd, int groups) {   // (always with the step in the epilogue)
  const int bm[4] = {128, 128, 256, 64}, bn[4] = {64, 128, 256, 256}, nw[4] = {4, 4, 8, 4};
  const int sh = gemm_bf16_wgrad_shape(Md, Nd, Kd, groups, 1);
  return ((Md + bm[sh] - 1) / bm[sh]) * ((Nd + bn[sh] - 1) / bn[sh]) * nw[sh];
}

int gemm_bf16_row_parts(int Md, int Nd, int groups) {
  const int bn[5] = {64, 128, 256, 0, 128};
  const int sh = gemm_bf16_tile_shape(Md, Nd, groups);
  return (Nd + bn[sh] - 1) / bn[sh];
}

int gemm_bf16_col_parts(int Md, int Nd, int groups) {
  const int bm[5] = {128, 128, 256, 0, 64}, wm[5] = {4, 2, 2, 0, 2};
  const int sh = gemm_bf16_tile_shape(Md, Nd, groups);
  return (Md + bm[sh] - 1) / bm[sh] * wm[sh];
}

void gemm_bf16_col_part_shape(int shape, int *tile_m, int *parts_per_tile) {
  const int bm[5] = {128, 128, 256, 0, 64}, wm[5] = {4, 2, 2, 0, 2};
  *tile_m = bm[shape];
  *parts_per_tile = wm[shape];
}

int gemm_bf16_ipdot_parts(int Nd) {
  if (Nd <= 64) return 1;
  // upper bound over the tile shapes launch_shape may pick (128-wide tiles)
  return (Nd + 127) / 128;
}

hipError_t launch_gemm_bf16(const GemmP &p, int epi, hipStream_t s) {
  // operand checks the kernels rely on: 16-byte aligned rows, operands below 2 GiB per replica
  if ((p.lda & 7) || (p.ldb & 7)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(p.A) & 15) || (reinterpret_cast<uintptr_t>(p.B) & 15)) return hipErrorInvalidValue;
  if ((p.sAg & 7) || (p.sBg & 7)) return hipErrorInvalidValue;
  if (!p.a_trans && (p.Kd > p.lda)) return hipErrorInvalidValue;
  if (!p.b_trans && (p.Kd > p.ldb)) return hipErrorInvalidValue;
  if (p.a_trans && (p.Md > p.lda)) return hipErrorInvalidValue;
  if (p.b_trans && (p.Nd > p.ldb)) return hipErrorInvalidValue;
  const long long abytes = (long long)(p.a_trans ? p.Kd : p.Md) * p.lda * 2;
  const long long bbytes = (long long)(p.b_trans ? p.Kd : p.Nd) * p.ldb * 2;
  if (abytes >= (1LL << 31) || bbytes >= (1LL << 31)) return hipErrorInvalidValue;
  if (p.ksplit > 1 && (epi != EPI_WGRAD || !p.kpart || p.kchunk <= 0 || (p.kchunk & 63) ||
                       (long long)p.kchunk * p.ksplit < p.Kd || (p.Nd & 3)))
    return hipErrorInvalidValue;
  if (p.upd_x && (epi != EPI_WGRAD || p.ksplit > 1 || p.accumulate || !p.upd_sq || (p.ldc & 3) || (p.Nd & 3) ||
                  (p.sCg & 3) || (reinterpret_cast<uintptr_t>(p.upd_x) & 15) || (p.C2 && ((p.ldc2 & 3) || p.ldc2 != p.ldc)) ||
                  (p.upd_opt != OPT_SGD && !p.upd_v) || (p.upd_opt == OPT_ADAMW && !p.upd_m)))
    return hipErrorInvalidValue;
  if (!p.a_trans && !p.b_trans) {
    if (epi == EPI_FWD_ACT) return launch_act<false, false, EPI_FWD_ACT>(p, s);
    if (epi == EPI_LOGITS) return launch_act<false, false, EPI_LOGITS>(p, s);
    if (epi == EPI_IPDOT) return launch_act<false, false, EPI_IPDOT>(p, s);
  } else if (!p.a_trans && p.b_trans) {
    if (epi == EPI_BWD) return launch_act<false, true, EPI_BWD>(p, s);
  } else if (p.a_trans && p.b_trans) {
    if (epi == EPI_WGRAD) return p.upd_x ? launch_act<true, true, EPI_WGRAD_UPD>(p, s) : launch_act<true, true, EPI_WGRAD>(p, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace absk
