// Replica-batched ("grouped") bf16 GEMM on the gfx950 matrix cores.
//
//   C[g][m][n] = sum_k A[g][m][k] * B[g][n][k],   g = replica
//
// covers the three contractions of one local step (Alg. 1 of the paper, "compute the local
// batch gradient"): forward  a W^T, backward-data  delta W, weight gradient  delta^T a, and
// the extra contraction  a Gbar^T  of the inner-product statistics.  Either operand may be
// stored k-contiguous ([row][k]) or row-contiguous ([k][row]); the latter is transposed in
// registers (8x8 / 8x4 bf16 blocks, v_perm) on its way into LDS, so LDS always holds
// k-contiguous tiles and every MFMA operand fragment is one 16-byte LDS read.
//
// Tiling: BM x BN x BK block tile, WM x WN wavefronts of 64 lanes, each computing a
// (BM/WM) x (BN/WN) sub-tile as a grid of 32x32x16 bf16 MFMAs with fp32 accumulators.
// Global -> registers -> LDS with two LDS buffers: the loads of tile k+1 are issued before
// the MFMAs of tile k and written to the other buffer afterwards (one barrier per k-tile).
// Work-group ids are remapped so that each XCD (ids are dealt round-robin to the 8 XCDs)
// works on a contiguous range of tiles and its L2 sees a few row-blocks of A and one
// replica's B at a time.
#include "abs_internal.h"
#include "device_utils.h"

namespace absk {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

namespace {

constexpr int LPAD = 8;  // bf16 elements of padding per LDS row (16 bytes)

// ---- global -> register staging ---------------------------------------------------------
// k-contiguous operand tile [ROWS x BK]: 16-byte chunks, thread t takes chunks t, t+NT, ...
template <int ROWS, int BK, int NT>
struct StageK {
  static constexpr int CPR = BK / 8;                 // chunks per row
  static constexpr int N = (ROWS * CPR) / NT;        // chunks per thread
  static_assert((ROWS * CPR) % NT == 0, "tile/threads mismatch");
  uint4 r[N];
  __device__ __forceinline__ void load(const bf16_t *base, int ld, int row0, int rows, int k0,
                                       int K, int tid) {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = tid + i * NT;
      const int row = row0 + c / CPR, k = k0 + (c % CPR) * 8;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (row < rows && k < K) v = *reinterpret_cast<const uint4 *>(base + (long long)row * ld + k);
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_t *lds, int tid) const {
#pragma unroll
    for (int i = 0; i < N; ++i) {
      const int c = tid + i * NT;
      *reinterpret_cast<uint4 *>(lds + (c / CPR) * (BK + LPAD) + (c % CPR) * 8) = r[i];
    }
  }
};

// row-contiguous operand (memory [k][row]): thread takes 8 k-rows x NV rows-of-the-tile,
// transposes them in registers and writes NV 16-byte LDS chunks.
template <int ROWS, int BK, int NT>
struct StageT {
  static constexpr int PER = (ROWS * BK) / (8 * NT);   // tile rows per thread (times 8 k)
  static constexpr int NV = PER >= 8 ? 8 : PER;        // rows per block: 8 (16 B), 4 or 2
  static constexpr int NB = PER / NV;                  // blocks per thread
  static_assert(PER == 2 || PER == 4 || PER % 8 == 0, "unsupported tile/threads ratio");
  static constexpr int KC = BK / 8;                    // k-chunks per tile
  static constexpr int NW = NV / 2;                    // 32-bit words per loaded vector
  uint32_t r[NB][8][NW];
  __device__ __forceinline__ void load(const bf16_t *base, int ld, int row0, int rows, int k0,
                                       int K, int tid) {
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
      const int blk = tid + bi * NT;
      const int kc = blk % KC, nb = blk / KC;
      const int row = row0 + nb * NV;                  // first tile row (memory column)
      const bool rin = row < rows;                     // ld is a multiple of 8: whole vector in
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int k = k0 + kc * 8 + j;
        const bf16_t *src = base + (long long)k * ld + row;
        const bool in = rin && k < K;
        if constexpr (NV == 8) {
          uint4 v = make_uint4(0, 0, 0, 0);
          if (in) v = *reinterpret_cast<const uint4 *>(src);
          r[bi][j][0] = v.x; r[bi][j][1] = v.y; r[bi][j][2] = v.z; r[bi][j][3] = v.w;
        } else if constexpr (NV == 4) {
          uint2 v = make_uint2(0, 0);
          if (in) v = *reinterpret_cast<const uint2 *>(src);
          r[bi][j][0] = v.x; r[bi][j][1] = v.y;
        } else {
          uint32_t v = 0;
          if (in) v = *reinterpret_cast<const uint32_t *>(src);
          r[bi][j][0] = v;
        }
      }
    }
  }
  __device__ __forceinline__ void store(bf16_t *lds, int tid) const {
#pragma unroll
    for (int bi = 0; bi < NB; ++bi) {
      const int blk = tid + bi * NT;
      const int kc = blk % KC, nb = blk / KC;
#pragma unroll
      for (int n = 0; n < NV; ++n) {
        // column n of the 8 x NV block: element k of it sits in half (n&1) of r[.][k][n/2]
        const uint32_t sel = (n & 1) ? 0x07060302u : 0x05040100u;
        uint4 o;
        o.x = __builtin_amdgcn_perm(r[bi][1][n / 2], r[bi][0][n / 2], sel);
        o.y = __builtin_amdgcn_perm(r[bi][3][n / 2], r[bi][2][n / 2], sel);
        o.z = __builtin_amdgcn_perm(r[bi][5][n / 2], r[bi][4][n / 2], sel);
        o.w = __builtin_amdgcn_perm(r[bi][7][n / 2], r[bi][6][n / 2], sel);
        *reinterpret_cast<uint4 *>(lds + (nb * NV + n) * (BK + LPAD) + kc * 8) = o;
      }
    }
  }
};

template <bool TRANS, int ROWS, int BK, int NT> struct StageSel { typedef StageK<ROWS, BK, NT> type; };
template <int ROWS, int BK, int NT> struct StageSel<true, ROWS, BK, NT> { typedef StageT<ROWS, BK, NT> type; };

// ---- the kernel --------------------------------------------------------------------------
template <int BM, int BN, int BK, int WM, int WN, bool AT, bool BT, int EPI, int ACT>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_bf16_kernel(const GemmP p, const int tilesM, const int tilesN, const int nblk, const int chunk) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;
  constexpr int MI = TM / 32, NI = TN / 32;
  constexpr int LS = BK + LPAD;
  constexpr int TILE = (BM + BN) * LS;                  // bf16 elements per LDS buffer
  static_assert(TM % 32 == 0 && TN % 32 == 0 && BK % 16 == 0, "tile shape");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t *smem = reinterpret_cast<bf16_t *>(smem_raw);

  // XCD-aware remap of the flat work-group id
  const int bid = blockIdx.x;
  const int lb = (bid & 7) * chunk + (bid >> 3);
  if (lb >= nblk) return;
  const int per_g = tilesM * tilesN;
  const int g = lb / per_g;
  const int t = lb - g * per_g;
  const int tm = t / tilesN, tn = t - tm * tilesN;
  const int m0 = tm * BM, n0 = tn * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

  const bf16_t *A = static_cast<const bf16_t *>(p.A) + (long long)g * p.sAg;
  const bf16_t *B = static_cast<const bf16_t *>(p.B) + (long long)g * p.sBg;

  typename StageSel<AT, BM, BK, NT>::type sa;
  typename StageSel<BT, BN, BK, NT>::type sb;

  f32x16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const int KT = (p.Kd + BK - 1) / BK;
  sa.load(A, p.lda, m0, p.Md, 0, p.Kd, tid);
  sb.load(B, p.ldb, n0, p.Nd, 0, p.Kd, tid);
  sa.store(smem, tid);
  sb.store(smem + BM * LS, tid);
  __syncthreads();

  const int lrow = lane & 31, lk = (lane >> 5) * 8;
  for (int kt = 0; kt < KT; ++kt) {
    const bf16_t *As = smem + (kt & 1) * TILE;
    const bf16_t *Bs = As + BM * LS;
    if (kt + 1 < KT) {
      sa.load(A, p.lda, m0, p.Md, (kt + 1) * BK, p.Kd, tid);
      sb.load(B, p.ldb, n0, p.Nd, (kt + 1) * BK, p.Kd, tid);
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i)
        af[i] = *reinterpret_cast<const bf16x8 *>(As + (wm * TM + i * 32 + lrow) * LS + kk * 16 + lk);
#pragma unroll
      for (int j = 0; j < NI; ++j)
        bfr[j] = *reinterpret_cast<const bf16x8 *>(Bs + (wn * TN + j * 32 + lrow) * LS + kk * 16 + lk);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      bf16_t *nx = smem + ((kt + 1) & 1) * TILE;
      sa.store(nx, tid);
      sb.store(nx + BM * LS, tid);
    }
    __syncthreads();
  }

  // ---- epilogue.  Accumulator element r of a 32x32 tile: column = lane % 32,
  //      row = 8 * (r / 4) + 4 * (lane / 32) + r % 4.
  const int lcol = lane & 31, lhalf = lane >> 5;
  const float *bias = p.bias ? p.bias + (long long)g * p.sBiasg : nullptr;

  if (EPI == EPI_IPDOT) {
    const bf16_t *E = static_cast<const bf16_t *>(p.E) + (long long)g * p.sEg;
    float *red = reinterpret_cast<float *>(smem_raw);     // [WN][BM] row partials (tiles are dead)
#pragma unroll
    for (int i = 0; i < MI; ++i) {
      float rs[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) rs[r] = 0.0f;
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int n = n0 + wn * TN + j * 32 + lcol;
        const float bv = (bias && n < p.Nd) ? bias[n] : 0.0f;
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = m0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
          float e = 0.0f;
          if (m < p.Md && n < p.Nd) e = bf2f(E[(long long)m * p.lde + n]);
          rs[r] = fmaf(e, acc[i][j][r] + bv, rs[r]);
        }
      }
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float v = rs[r];
#pragma unroll
        for (int o = 16; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);   // over the 32 columns
        if (lcol == 0) red[wn * BM + wm * TM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3)] = v;
      }
    }
    __syncthreads();
    float *part = p.part + (long long)g * p.sPartg + (long long)tn * p.sPartTile;
    for (int r = tid; r < BM; r += NT) {
      float v = 0.0f;
#pragma unroll
      for (int w = 0; w < WN; ++w) v += red[w * BM + r];
      if (m0 + r < p.Md) part[m0 + r] = v;
    }
    return;
  }

#pragma unroll
  for (int i = 0; i < MI; ++i) {
#pragma unroll
    for (int j = 0; j < NI; ++j) {
      const int n = n0 + wn * TN + j * 32 + lcol;
      const bool nin = n < p.Nd;
      const float bv = (bias && nin) ? bias[n] : 0.0f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * TM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        if (m >= p.Md) continue;
        const float v = acc[i][j][r];
        if (EPI == EPI_FWD_ACT) {
          if (n < p.ldc && (nin || p.pad_to_ld)) {
            float a = 0.0f, d = 0.0f;
            if (nin) act_fwd<ACT>(v + bv, a, d);
            static_cast<bf16_t *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = f2bf(a);
            if (ACT == ACT_GELU && p.C2)
              static_cast<bf16_t *>(p.C2)[(long long)g * p.sC2g + (long long)m * p.ldc2 + n] = f2bf(d);
          }
        } else if (EPI == EPI_LOGITS) {
          if (nin) static_cast<float *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = v + bv;
        } else if (EPI == EPI_BWD) {
          if (n < p.ldc && (nin || p.pad_to_ld)) {
            float o = 0.0f;
            if (nin) {
              const float e = bf2f(static_cast<const bf16_t *>(p.E)[(long long)g * p.sEg + (long long)m * p.lde + n]);
              o = (ACT == ACT_RELU) ? (e > 0.0f ? v : 0.0f) : (ACT == ACT_GELU ? v * e : v);
            }
            static_cast<bf16_t *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = f2bf(o);
          }
        } else if (EPI == EPI_WGRAD) {
          if (nin) {
            const float o = v * p.alpha;
            static_cast<float *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = o;
            if (p.C2) static_cast<bf16_t *>(p.C2)[(long long)g * p.sC2g + (long long)m * p.ldc2 + n] = f2bf(o);
          }
        }
      }
    }
  }
}

template <int BM, int BN, int BK, int WM, int WN, bool AT, bool BT, int EPI, int ACT>
hipError_t launch_cfg(const GemmP &p, hipStream_t s) {
  constexpr int NT = WM * WN * 64;
  constexpr size_t tile_bytes = 2ull * (BM + BN) * (BK + LPAD) * sizeof(bf16_t);
  constexpr size_t red_bytes = (size_t)WN * BM * sizeof(float);
  constexpr size_t lds = tile_bytes > red_bytes ? tile_bytes : red_bytes;
  auto kern = gemm_bf16_kernel<BM, BN, BK, WM, WN, AT, BT, EPI, ACT>;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_set = true;
  }
  const int tilesM = (p.Md + BM - 1) / BM, tilesN = (p.Nd + BN - 1) / BN;
  const long long nblk = (long long)tilesM * tilesN * p.groups;
  if (nblk <= 0) return hipSuccess;
  if (nblk > 0x3fffffff) return hipErrorInvalidValue;
  const int chunk = (int)((nblk + 7) / 8);
  hipLaunchKernelGGL(kern, dim3(chunk * 8), dim3(NT), lds, s, p, tilesM, tilesN, (int)nblk, chunk);
  return hipGetLastError();
}

// Tile shape by problem size: the large shape when both output extents fill it,
// otherwise a 128x128 (or 128x64 for narrow outputs) tile.
template <bool AT, bool BT, int EPI, int ACT>
hipError_t launch_shape(const GemmP &p, hipStream_t s) {
  switch (gemm_bf16_tile_shape(p.Md, p.Nd)) {
    case 0: return launch_cfg<128, 64, 64, 4, 1, AT, BT, EPI, ACT>(p, s);
    case 2: return launch_cfg<256, 256, 64, 2, 4, AT, BT, EPI, ACT>(p, s);
    default: return launch_cfg<128, 128, 64, 2, 2, AT, BT, EPI, ACT>(p, s);
  }
}

template <bool AT, bool BT, int EPI>
hipError_t launch_act(const GemmP &p, hipStream_t s) {
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

int gemm_bf16_tile_shape(int Md, int Nd) {
  if (Nd <= 64) return 0;
  if (Md >= 1024 && Nd >= 1024) return 2;
  return 1;
}

int gemm_bf16_ipdot_parts(int Nd) {
  if (Nd <= 64) return 1;
  // upper bound over the tile shapes launch_shape may pick (128-wide tiles)
  return (Nd + 127) / 128;
}

hipError_t launch_gemm_bf16(const GemmP &p, int epi, hipStream_t s) {
  // operand checks the kernels rely on: 16-byte aligned rows
  if ((p.lda & 7) || (p.ldb & 7)) return hipErrorInvalidValue;
  if ((reinterpret_cast<uintptr_t>(p.A) & 15) || (reinterpret_cast<uintptr_t>(p.B) & 15)) return hipErrorInvalidValue;
  if ((p.sAg & 7) || (p.sBg & 7)) return hipErrorInvalidValue;
  if (!p.a_trans && (p.Kd > p.lda)) return hipErrorInvalidValue;
  if (!p.b_trans && (p.Kd > p.ldb)) return hipErrorInvalidValue;
  if (p.a_trans && (p.Md > p.lda)) return hipErrorInvalidValue;
  if (p.b_trans && (p.Nd > p.ldb)) return hipErrorInvalidValue;
  if (!p.a_trans && !p.b_trans) {
    if (epi == EPI_FWD_ACT) return launch_act<false, false, EPI_FWD_ACT>(p, s);
    if (epi == EPI_LOGITS) return launch_act<false, false, EPI_LOGITS>(p, s);
    if (epi == EPI_IPDOT) return launch_act<false, false, EPI_IPDOT>(p, s);
  } else if (!p.a_trans && p.b_trans) {
    if (epi == EPI_BWD) return launch_act<false, true, EPI_BWD>(p, s);
  } else if (p.a_trans && p.b_trans) {
    if (epi == EPI_WGRAD) return launch_act<true, true, EPI_WGRAD>(p, s);
  }
  return hipErrorInvalidValue;
}

}  // namespace absk
