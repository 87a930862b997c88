// Inner products q_i = <g_i, gbar> of the inner-product test (named at the end of Sec. 4.1) for short
// local batches, without touching the batch gradient.
//
// The per-sample gradient of layer l is the outer product delta_i^l a_i^{l-1 T} (plus delta_i^l for the
// bias), so
//     <g_i, g_j> = sum_l (delta_i^l . delta_j^l) (a_i^{l-1} . a_j^{l-1} + [bias])
// and q_i = (1/b) sum_j <g_i, g_j>: two b x b Gram matrices per layer, multiplied entry by entry and summed
// along j.  The contraction Gbar_l a_i that the long-batch path uses reads every parameter once per step
// (2 bytes each, and 2 more to write the bf16 copy of Gbar it reads); the Gram form reads only the b rows of
// activations and backprop signals, b (in + out) entries per layer.  Its arithmetic grows with b^2 instead of
// b, so the host takes it for short batches only.
//
//   gram_partial_kernel : partial Gram matrices X X^T over slices of the feature dimension, MFMA
//                         (v_mfma_f32_32x32x16_bf16) with both operands read straight from memory: a lane's
//                         fragment is 8 consecutive features of one row, which is how the rows lie in memory
//   gram_finish_kernel  : adds the slices in order, multiplies the two matrices of each layer, adds the layers
//                         and the row, divides by b
#include "abs_internal.h"
#include "device_utils.h"

namespace absk {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int GT = 64;            // output tile: GT x GT entries of a Gram matrix per work-group
constexpr int GCH = 32;           // features per wave and loop trip (two MFMA k-steps)
constexpr int RLD = GT + 4;       // row stride of the work-group's reduction buffer (floats)

// 8 consecutive features k .. k+7 of row `row` (zeros outside the matrix)
__device__ __forceinline__ bf16x8 load_frag(const bf16_t *X, int ld, int row, int nrows, int k, int K) {
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (row < nrows && k < K) {
    v = *reinterpret_cast<const uint4 *>(X + (long long)row * ld + k);   // k + 8 <= ld: ld is a multiple of 8
    if (k + 8 > K) {                                                    // ragged last chunk: columns >= K may hold anything
      uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int e = 0; e < 8; ++e)
        if (k + e >= K) w[e >> 1] &= (e & 1) ? 0x0000ffffu : 0xffff0000u;
      v = make_uint4(w[0], w[1], w[2], w[3]);
    }
  }
  return __builtin_bit_cast(bf16x8, v);
}

__global__ void __launch_bounds__(256) gram_partial_kernel(const GramP p) {
  __shared__ float red[GT * RLD];
  const int nT = p.bp / GT, nP = nT * (nT + 1) / 2;
  int id = blockIdx.x;
  // a Gram matrix is symmetric: only tiles on and above the diagonal are computed, (ti, tj) with ti <= tj
  int ti = 0, tj = id % nP; id /= nP;
  while (tj >= nT - ti) { tj -= nT - ti; ++ti; }
  tj += ti;
  const int sl = id % p.S; id /= p.S;
  const int mat = id % p.n;
  const int g = id / p.n;
  const int nrows = p.rows ? p.rows[g] : p.b;
  // uniform over the block, before any barrier: tiles outside this group's batch and empty slices are never read
  if (tj * GT >= nrows || sl >= p.nsl[mat]) return;          // (ti <= tj)
  const int K = p.K[mat], ld = p.ld[mat];
  const bf16_t *X = p.X[mat] + (long long)g * p.sXg[mat];
  const int kbeg = sl * p.kslice[mat];
  const int kend = kbeg + p.kslice[mat] < K ? kbeg + p.kslice[mat] : K;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lrow = lane & 31, lk = (lane >> 5) * 8;
  const bool diag = ti == tj;

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  // The four waves take the slice's chunks of GCH features in turn, GD chunks per trip: all loads of a trip are
  // issued before its first MFMA (a slice is a few chunks per wave, so the launch is bound by load latency).
  // A chunk never crosses the slice end (slices are multiples of GCH long); chunks past it read as zeros.
  constexpr int GD = 2;
  for (int k0 = kbeg + wave * GCH; k0 < kend; k0 += GD * 4 * GCH) {
    bf16x8 fi[GD][2][2], fj[GD][2][2];
#pragma unroll
    for (int d = 0; d < GD; ++d)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int h = 0; h < 2; ++h) {
          const int k = k0 + d * 4 * GCH + kk * 16 + lk;
          fi[d][kk][h] = load_frag(X, ld, ti * GT + h * 32 + lrow, nrows, k, kend);
          fj[d][kk][h] = diag ? fi[d][kk][h] : load_frag(X, ld, tj * GT + h * 32 + lrow, nrows, k, kend);
        }
#pragma unroll
    for (int d = 0; d < GD; ++d)
#pragma unroll
      for (int kk = 0; kk < 2; ++kk)
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            // first operand: the columns.  A lane then owns row 32 i + lane % 32 of the tile and, per q, the four
            // consecutive columns 32 j + 8 q + 4 (lane / 32) .. + 3 in accumulator elements 4 q .. 4 q + 3.
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fj[d][kk][j], fi[d][kk][i], acc[i][j], 0, 0, 0);
  }

  // add the four waves' tiles in wave order
  const int lhalf = lane >> 5;
  for (int w = 0; w < 4; ++w) {
    if (wave == w) {
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float4 *dst = reinterpret_cast<float4 *>(red + (i * 32 + lrow) * RLD + j * 32 + q * 8 + lhalf * 4);
            float4 v = make_float4(acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            if (w > 0) { const float4 o = *dst; v.x += o.x; v.y += o.y; v.z += o.z; v.w += o.w; }
            *dst = v;
          }
    }
    __syncthreads();
  }
  float *mat0 = p.part + (((long long)g * p.n + mat) * p.S + sl) * p.bp * p.bp;
  float *out = mat0 + (long long)(ti * GT) * p.bp + tj * GT;
  for (int c = tid; c < GT * GT / 4; c += 256) {
    const int r = c / (GT / 4), cc = c % (GT / 4);
    *reinterpret_cast<float4 *>(out + (long long)r * p.bp + cc * 4) = *reinterpret_cast<const float4 *>(red + r * RLD + cc * 4);
  }
  if (!diag) {                                    // the mirror tile (tj, ti) is the transpose
    float *outT = mat0 + (long long)(tj * GT) * p.bp + ti * GT;
    for (int c = tid; c < GT * GT / 4; c += 256) {
      const int r = c / (GT / 4), cc = c % (GT / 4);
      const float4 v = make_float4(red[(cc * 4) * RLD + r], red[(cc * 4 + 1) * RLD + r], red[(cc * 4 + 2) * RLD + r],
                                   red[(cc * 4 + 3) * RLD + r]);
      *reinterpret_cast<float4 *>(outT + (long long)r * p.bp + cc * 4) = v;
    }
  }
}

constexpr int GSMAX = 8;          // most slices per matrix (the finish kernel keeps one load per slice in flight)

// one wavefront per sample: q[g][i] = (1 / b_g) sum_l sum_j Kd_l[i][j] (Ka_l[i][j] + add)
__global__ void __launch_bounds__(256) gram_finish_kernel(const GramP p, const float add, float *q, const long long sQg) {
  const int lane = threadIdx.x & 63;
  const int i = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int g = blockIdx.y;
  const int nrows = p.rows ? p.rows[g] : p.b;
  if (i >= nrows) return;
  const long long tile = (long long)p.bp * p.bp;
  const int L = p.n / 2;
  float s = 0.0f;
  // two layers per trip, every slice of their four matrices loaded before the first addition: the kernel is a
  // chain of dependent memory latencies otherwise
  for (int l = 0; l < L; l += 2) {
    for (int j = lane; j < nrows; j += 64) {
      float v[4][GSMAX];
#pragma unroll
      for (int m = 0; m < 4; ++m) {
        const int mat = 2 * l + m;
        const float *pm = p.part + ((long long)g * p.n + mat) * p.S * tile + (long long)i * p.bp + j;
        const int ns = mat < p.n ? p.nsl[mat] : 0;
#pragma unroll
        for (int t = 0; t < GSMAX; ++t) v[m][t] = t < ns ? pm[t * tile] : 0.0f;
      }
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        float ka = add, kd = 0.0f;                   // slices in order (absent ones add zero)
#pragma unroll
        for (int t = 0; t < GSMAX; ++t) { ka += v[2 * h][t]; kd += v[2 * h + 1][t]; }
        s = fmaf(kd, ka, s);                         // an absent second layer has kd = 0
      }
    }
  }
  s = wave_sum(s);
  if (lane == 0) q[(long long)g * sQg + i] = s / (float)nrows;
}

}  // namespace

long long gram_ip_scratch_floats(int n, int groups) {
  return (long long)groups * n * GRAM_SLICE_ELEMS;
}

hipError_t launch_gram_ip(GramP p, int has_bias, float *q, long long sQg, hipStream_t s) {
  if (p.n < 2 || p.n > 2 * GramP::MAXL || (p.n & 1) || p.b < 1 || p.groups < 1 || !p.part || !q) return hipErrorInvalidValue;
  p.bp = (p.b + GT - 1) / GT * GT;
  const long long tile = (long long)p.bp * p.bp;
  if (tile > GRAM_SLICE_ELEMS) return hipErrorInvalidValue;
  int kmax = 0;
  for (int m = 0; m < p.n; ++m) {
    // operand checks the kernel relies on: whole 16-byte chunks inside every row
    if (!p.X[m] || p.K[m] < 1 || p.K[m] > p.ld[m] || (p.ld[m] & 7) || (p.sXg[m] & 7) ||
        (reinterpret_cast<uintptr_t>(p.X[m]) & 15))
      return hipErrorInvalidValue;
    kmax = p.K[m] > kmax ? p.K[m] : kmax;
  }
  // Slices of the feature dimension: enough work-groups to fill the chip about once (three fit a CU), no more,
  // since every slice writes and the finish reads a partial matrix (measured on config 3, 16 workers: b = 64 best
  // with 6 slices, b = 128 with 2); at most GSMAX, what the scratch holds, and 4 x GCH features each (a chunk per wave).
  const int nT = p.bp / GT, nP = nT * (nT + 1) / 2;
  int S = (int)(768 / ((long long)p.groups * p.n * nP));
  const int sfit = (int)(GRAM_SLICE_ELEMS / tile);
  S = S > sfit ? sfit : S;
  S = S > GSMAX ? GSMAX : S;
  const int smax = (kmax + 4 * GCH - 1) / (4 * GCH);
  S = S > smax ? smax : S;
  p.S = S < 1 ? 1 : S;
  for (int m = 0; m < p.n; ++m) {
    const int per = (p.K[m] + p.S - 1) / p.S;
    p.kslice[m] = (per + 4 * GCH - 1) / (4 * GCH) * (4 * GCH);
    p.nsl[m] = (p.K[m] + p.kslice[m] - 1) / p.kslice[m];
  }
  const long long blocks = (long long)p.groups * p.n * p.S * nP;
  if (blocks > 0x7fffffff) return hipErrorInvalidValue;
  hipLaunchKernelGGL(gram_partial_kernel, dim3((unsigned)blocks), dim3(256), 0, s, p);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(gram_finish_kernel, dim3((p.b + 3) / 4, p.groups), dim3(256), 0, s, p, has_bias ? 1.0f : 0.0f, q, sQg);
  return hipGetLastError();
}

}  // namespace absk
