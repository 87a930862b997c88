// Replica-batched fp32 GEMM (plain vector ALU, LDS-tiled) for the fp32 precision mode:
//   C[g][m][n] = sum_k A[g][m][k] * B[g][n][k]
// with the same operand-layout flags and epilogues as the bf16 matrix-core family.  The fp32
// mode serves small, latency-bound problems (logistic regression), so this kernel favours
// generality (arbitrary strides and extents) over peak rate: TS x TS block tile (64, or 32 when
// the output has few tiles, so that more work-groups share the latency-bound walk over k),
// k-step 32, 256 threads, (TS/16)^2 outputs per thread; the next k-step's operands are fetched
// into registers while the current one is multiplied.
#include "abs_internal.h"
#include "device_utils.h"

namespace absk {
namespace {

template <int EPI, int ACT, int TS>
__global__ void __launch_bounds__(256) gemm_f32_kernel(const GemmP pin) {
  constexpr int BK = 32, PT = TS * BK / 256;     // k-step, elements per thread and operand
  constexpr int R = TS / 16;                     // outputs per thread and dimension
  __shared__ float As[BK][TS + 4];
  __shared__ float Bs[BK][TS + 4];
  // blockIdx.z = group, or (group, k-slice) of a weight gradient whose reduction is split
  const int ksplit = (EPI == EPI_WGRAD && pin.ksplit > 1) ? pin.ksplit : 1;
  const int g = blockIdx.z / ksplit, ksl = blockIdx.z - g * ksplit;
  const int m0 = blockIdx.y * TS, n0 = blockIdx.x * TS;
  GemmP p = pin;
  if (p.rows) {                                   // ragged groups: this group's own extent
    const int r = p.rows[g];
    if (p.rows_is_k) { p.Kd = r; p.alpha = 1.0f / (float)r; } else p.Md = r;
    if (m0 >= p.Md) return;                       // uniform over the block, before any barrier
  }
  int kbeg = 0;
  if (ksplit > 1) {                               // this block's slice; an empty one writes zeros
    kbeg = ksl * p.kchunk;
    const int kend = kbeg + p.kchunk;
    if (kend < p.Kd) p.Kd = kend;
    if (kbeg > p.Kd) kbeg = p.Kd;
  }
  const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
  const float *A = static_cast<const float *>(p.A) + (long long)g * p.sAg;
  const float *B = static_cast<const float *>(p.B) + (long long)g * p.sBg;
  float acc[R][R];
#pragma unroll
  for (int i = 0; i < R; ++i)
#pragma unroll
    for (int j = 0; j < R; ++j) acc[i][j] = 0.0f;

  float ra[PT], rb[PT];
  auto fetch = [&](int k0) {
#pragma unroll
    for (int e = 0; e < PT; ++e) {
      const int id = tid + e * 256;
      int kk, rr;
      if (!p.a_trans) { kk = id & (BK - 1); rr = id / BK; } else { rr = id % TS; kk = id / TS; }
      const int m = m0 + rr, k = k0 + kk;
      ra[e] = 0.0f;
      if (m < p.Md && k < p.Kd) ra[e] = p.a_trans ? A[(long long)k * p.lda + m] : A[(long long)m * p.lda + k];
      if (!p.b_trans) { kk = id & (BK - 1); rr = id / BK; } else { rr = id % TS; kk = id / TS; }
      const int n = n0 + rr, kb = k0 + kk;
      rb[e] = 0.0f;
      if (n < p.Nd && kb < p.Kd) rb[e] = p.b_trans ? B[(long long)kb * p.ldb + n] : B[(long long)n * p.ldb + kb];
    }
  };
  if (kbeg < p.Kd) fetch(kbeg);
  for (int k0 = kbeg; k0 < p.Kd; k0 += BK) {
#pragma unroll
    for (int e = 0; e < PT; ++e) {
      const int id = tid + e * 256;
      int kk, rr;
      if (!p.a_trans) { kk = id & (BK - 1); rr = id / BK; } else { rr = id % TS; kk = id / TS; }
      As[kk][rr] = ra[e];
      if (!p.b_trans) { kk = id & (BK - 1); rr = id / BK; } else { rr = id % TS; kk = id / TS; }
      Bs[kk][rr] = rb[e];
    }
    __syncthreads();
    if (k0 + BK < p.Kd) fetch(k0 + BK);
#pragma unroll
    for (int kk = 0; kk < BK; ++kk) {
      float a[R], b[R];
#pragma unroll
      for (int i = 0; i < R; ++i) a[i] = As[kk][ty * R + i];
#pragma unroll
      for (int j = 0; j < R; ++j) b[j] = Bs[kk][tx * R + j];
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

  const float *bias = p.bias ? p.bias + (long long)g * p.sBiasg : nullptr;
#pragma unroll
  for (int i = 0; i < R; ++i) {
    const int m = m0 + ty * R + i;
    if (m >= p.Md) continue;
#pragma unroll
    for (int j = 0; j < R; ++j) {
      const int n = n0 + tx * R + j;
      const bool nin = n < p.Nd;
      const float v = acc[i][j];
      const float bv = (bias && nin) ? bias[n] : 0.0f;
      if (EPI == EPI_FWD_ACT) {
        if (n < p.ldc && (nin || p.pad_to_ld)) {
          float a = 0.0f, d = 0.0f;
          if (nin) act_fwd<ACT>(v + bv, a, d);
          static_cast<float *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = a;
          if (ACT == ACT_GELU && p.C2)
            static_cast<float *>(p.C2)[(long long)g * p.sC2g + (long long)m * p.ldc2 + n] = d;
        }
      } else if (EPI == EPI_LOGITS) {
        if (nin) static_cast<float *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = v + bv;
      } else if (EPI == EPI_BWD) {
        if (n < p.ldc && (nin || p.pad_to_ld)) {
          float o = 0.0f;
          if (nin) {
            float e = 1.0f;
            if (ACT != ACT_NONE) e = static_cast<const float *>(p.E)[(long long)g * p.sEg + (long long)m * p.lde + n];
            o = (ACT == ACT_RELU) ? (e > 0.0f ? v : 0.0f) : (ACT == ACT_GELU ? v * e : v);
          }
          static_cast<float *>(p.C)[(long long)g * p.sCg + (long long)m * p.ldc + n] = o;
        }
      } else if (EPI == EPI_WGRAD) {
        if (nin && ksplit > 1) {                  // raw partial product of this k-slice, packed Md x Nd
          p.kpart[((long long)g * ksplit + ksl) * p.Md * p.Nd + (long long)m * p.Nd + n] = v;
        } else if (nin) {
          float *o = static_cast<float *>(p.C) + (long long)g * p.sCg + (long long)m * p.ldc + n;
          *o = p.accumulate ? fmaf(v, p.alpha, *o) : v * p.alpha;
        }
      }
    }
  }
}

template <int EPI, int ACT>
hipError_t launch1(const GemmP &p, hipStream_t s) {
  const int ks = (EPI == EPI_WGRAD && p.ksplit > 1) ? p.ksplit : 1;
  if (ks > 1 && (!p.kpart || p.kchunk <= 0 || (p.kchunk & 31) || (long long)p.kchunk * ks < p.Kd)) return hipErrorInvalidValue;
  // 32 x 32 tiles while 64 x 64 ones would leave most CUs without a work-group
  const long long blocks64 = (long long)((p.Nd + 63) / 64) * ((p.Md + 63) / 64) * p.groups * ks;
  const int ts = blocks64 < 128 ? 32 : 64;
  const dim3 grid((p.Nd + ts - 1) / ts, (p.Md + ts - 1) / ts, p.groups * ks);
  if (grid.y > 65535 || grid.z > 65535) return hipErrorInvalidValue;
  if (ts == 32) hipLaunchKernelGGL((gemm_f32_kernel<EPI, ACT, 32>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((gemm_f32_kernel<EPI, ACT, 64>), grid, dim3(256), 0, s, p);
  return hipGetLastError();
}
template <int EPI>
hipError_t launch_act(const GemmP &p, hipStream_t s) {
  if constexpr (EPI == EPI_FWD_ACT || EPI == EPI_BWD) {
    if (p.act == ACT_RELU) return launch1<EPI, ACT_RELU>(p, s);
    if (p.act == ACT_GELU) return launch1<EPI, ACT_GELU>(p, s);
  }
  return launch1<EPI, ACT_NONE>(p, s);
}

}  // namespace

hipError_t launch_gemm_f32(const GemmP &p, int epi, hipStream_t s) {
  if (p.Md <= 0 || p.Nd <= 0 || p.groups <= 0) return hipSuccess;
  switch (epi) {
    case EPI_FWD_ACT: return launch_act<EPI_FWD_ACT>(p, s);
    case EPI_LOGITS: return launch_act<EPI_LOGITS>(p, s);
    case EPI_BWD: return launch_act<EPI_BWD>(p, s);
    case EPI_WGRAD: return launch_act<EPI_WGRAD>(p, s);
    default: return hipErrorInvalidValue;
  }
}

}  // namespace absk
