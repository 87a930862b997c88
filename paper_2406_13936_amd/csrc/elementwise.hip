// Bandwidth-bound kernels of the local step: batch gather, softmax cross-entropy head,
// row / column reductions, the test statistics, the fused optimizer update, the replica
// average.  All reductions run in a fixed order (no floating-point atomics), so a step is
// bit-reproducible.  Wavefronts are 64 lanes; rows are read with 16-byte loads.
#include "abs_internal.h"
#include "device_utils.h"

namespace absk {
namespace {

// Streaming accesses: data that is touched once per launch is read and written with the
// non-temporal hint so that it does not displace the caches' contents (measured on MI355X:
// +7 % on a plain copy, +8 % on the update's three-read / three-write pattern).
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float4 ld_stream(const float4 *p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(float4 *p, float4 v) {
  const f32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<f32x4_t *>(p));
}
__device__ __forceinline__ uint4 ld_stream(const uint4 *p) {
  const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
  return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st_stream(uint4 *p, uint4 v) {
  const u32x4_t w = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x4_t *>(p));
}
__device__ __forceinline__ void st_stream(uint2 *p, uint2 v) {
  const u32x2_t w = {v.x, v.y};
  __builtin_nontemporal_store(w, reinterpret_cast<u32x2_t *>(p));
}

template <class T> struct Vec;                      // 16-byte vector of T
template <> struct Vec<float> {
  enum { N = 4 };
  static __device__ __forceinline__ void load(const float *p, float (&o)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Vec<bf16_t> {
  enum { N = 8 };
  static __device__ __forceinline__ void unpack(uint4 v, float (&o)[8]) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      o[2 * i] = __uint_as_float(w[i] << 16);
      o[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
  static __device__ __forceinline__ void load(const bf16_t *p, float (&o)[8]) {
    unpack(*reinterpret_cast<const uint4 *>(p), o);
  }
  static __device__ __forceinline__ void load_stream(const bf16_t *p, float (&o)[8]) {
    unpack(ld_stream(reinterpret_cast<const uint4 *>(p)), o);
  }
};

__global__ void convert_kernel(const float *__restrict__ src, bf16_t *__restrict__ dst, long long n) {
  long long i = (blockIdx.x * (long long)blockDim.x + threadIdx.x) * 4;
  const long long stride = (long long)gridDim.x * blockDim.x * 4;
  for (; i + 3 < n; i += stride) {
    const float4 v = *reinterpret_cast<const float4 *>(src + i);
    uint2 o;
    o.x = pack2bf(v.x, v.y);
    o.y = pack2bf(v.z, v.w);
    *reinterpret_cast<uint2 *>(dst + i) = o;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0)
    for (long long j = n & ~3LL; j < n; ++j) dst[j] = f2bf(src[j]);
}

// One wavefront per gathered row.  Source rows have d elements (row stride d); the
// destination row stride is ldo >= d (multiple of 8), pad columns are written as zeros.
// Indices outside [0, N) are clamped into the range (the kernels never read out of bounds).
template <class T>
__global__ void gather_kernel(const T *__restrict__ X, int d, int N, const int32_t *__restrict__ idx, int ldi, int b,
                              T *__restrict__ A0, long long sAg, int ldo, float *__restrict__ an0,
                              long long sNg, const int *__restrict__ rows) {
  const int g = blockIdx.y;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= (rows ? rows[g] : b)) return;
  const int lane = threadIdx.x & 63;
  const int32_t id = min(max(idx[(long long)g * ldi + i], 0), N - 1);
  const long long src = (long long)id * d;
  T *dst = A0 + (long long)g * sAg + (long long)i * ldo;
  float s = 0.0f;
  constexpr int V = Vec<T>::N;
  if ((d % V) == 0) {
    for (int c = lane * V; c < d; c += 64 * V) {
      const uint4 raw = *reinterpret_cast<const uint4 *>(X + src + c);
      float f[V];
      Vec<T>::load(X + src + c, f);
#pragma unroll
      for (int k = 0; k < V; ++k) s = fmaf(f[k], f[k], s);
      *reinterpret_cast<uint4 *>(dst + c) = raw;
    }
  } else {
    for (int c = lane; c < d; c += 64) {
      const T raw = X[src + c];
      const float f = Elem<T>::ld(&raw);
      s = fmaf(f, f, s);
      dst[c] = raw;
    }
  }
  for (int c = d + lane; c < ldo; c += 64) Elem<T>::st(dst + c, 0.0f);
  s = wave_sum(s);
  if (lane == 0) an0[(long long)g * sNg + i] = s;
}

// LPR lanes per row of logits: a whole wavefront, or 16 lanes (four rows per wavefront) for at most 16
// classes.  The butterflies stay inside a row's lanes (xor distances below LPR).
template <class T, int LPR>
__global__ void softmax_ce_kernel(const float *__restrict__ Z, long long sZg, int ldz, int K,
                                  const int32_t *__restrict__ y, int N, const int32_t *__restrict__ idx, int ldi,
                                  int b, T *__restrict__ D, long long sDg, int ldd,
                                  float *__restrict__ dn, float *__restrict__ loss, long long sNg,
                                  const int *__restrict__ rows) {
  const int g = blockIdx.y;
  const int i = (blockIdx.x * blockDim.x + threadIdx.x) / LPR;
  if (i >= (rows ? rows[g] : b)) return;          // uniform over a row's lanes
  const int lane = threadIdx.x & (LPR - 1);
  const float *z = Z + (long long)g * sZg + (long long)i * ldz;
  const int label = min(max(y[min(max(idx[(long long)g * ldi + i], 0), N - 1)], 0), K - 1);
  float mx = -INFINITY;
  for (int c = lane; c < K; c += LPR) mx = fmaxf(mx, z[c]);
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float se = 0.0f;
  for (int c = lane; c < K; c += LPR) se += expf(z[c] - mx);
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
  const float inv = 1.0f / se;
  T *drow = D + (long long)g * sDg + (long long)i * ldd;
  float sq = 0.0f;
  for (int c = lane; c < ldd; c += LPR) {
    float dv = 0.0f;
    if (c < K) dv = expf(z[c] - mx) * inv - (c == label ? 1.0f : 0.0f);
    const float st = Elem<T>::rnd(dv);
    Elem<T>::st(drow + c, dv);
    sq = fmaf(st, st, sq);
  }
#pragma unroll
  for (int o = LPR / 2; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  if (lane == 0) {
    dn[(long long)g * sNg + i] = sq;
    loss[(long long)g * sNg + i] = -(z[label] - mx - logf(se));
  }
}

// The same head for 17 .. 128 (padded) classes: 32 lanes per row (two rows per wavefront), four consecutive
// classes per lane, so the logits are read once as 16-byte vectors, every exponential is taken once and the
// signal leaves as 8-byte (bf16) or 16-byte (fp32) vectors.
template <class T>
__global__ void __launch_bounds__(256) softmax_ce_vec_kernel(const float *__restrict__ Z, long long sZg, int ldz, int K,
                                                             const int32_t *__restrict__ y, int N,
                                                             const int32_t *__restrict__ idx, int ldi, int b,
                                                             T *__restrict__ D, long long sDg, int ldd,
                                                             float *__restrict__ dn, float *__restrict__ loss,
                                                             long long sNg, const int *__restrict__ rows) {
  const int g = blockIdx.y;
  const int i = (blockIdx.x * 256 + threadIdx.x) >> 5;
  if (i >= (rows ? rows[g] : b)) return;          // uniform over a row's 32 lanes
  const int lane = threadIdx.x & 31, c0 = 4 * lane;
  const float *z = Z + (long long)g * sZg + (long long)i * ldz;
  const int label = min(max(y[min(max(idx[(long long)g * ldi + i], 0), N - 1)], 0), K - 1);
  float zv[4] = {-INFINITY, -INFINITY, -INFINITY, -INFINITY};
  if (c0 < ldz) {                                  // ldz is a multiple of 4: the whole vector lies inside the row
    const float4 v = *reinterpret_cast<const float4 *>(z + c0);
    zv[0] = v.x; zv[1] = v.y; zv[2] = v.z; zv[3] = v.w;
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) if (c0 + e >= K) zv[e] = -INFINITY;
  float mx = fmaxf(fmaxf(zv[0], zv[1]), fmaxf(zv[2], zv[3]));
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
  float ev[4];
#pragma unroll
  for (int e = 0; e < 4; ++e) ev[e] = c0 + e < K ? expf(zv[e] - mx) : 0.0f;
  float se = ((ev[0] + ev[1]) + ev[2]) + ev[3];
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) se += __shfl_xor(se, o, 64);
  const float inv = 1.0f / se;
  float dv[4], sq = 0.0f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    dv[e] = c0 + e < K ? ev[e] * inv - (c0 + e == label ? 1.0f : 0.0f) : 0.0f;
    const float st = Elem<T>::rnd(dv[e]);
    sq = fmaf(st, st, sq);
  }
  if (c0 < ldd) {                                  // ldd is a multiple of 4 as well; pad columns receive zeros
    T *drow = D + (long long)g * sDg + (long long)i * ldd + c0;
    if (sizeof(T) == 2) {
      uint2 o;
      o.x = pack2bf(dv[0], dv[1]); o.y = pack2bf(dv[2], dv[3]);
      *reinterpret_cast<uint2 *>(drow) = o;
    } else {
      *reinterpret_cast<float4 *>(drow) = make_float4(dv[0], dv[1], dv[2], dv[3]);
    }
  }
#pragma unroll
  for (int o = 16; o > 0; o >>= 1) sq += __shfl_xor(sq, o, 64);
  if (lane == 0) {
    dn[(long long)g * sNg + i] = sq;
    loss[(long long)g * sNg + i] = -(z[label] - mx - logf(se));
  }
}

template <class T>
__global__ void row_sqnorm_kernel(const T *__restrict__ X, long long sXg, int ld, int cols, int b,
                                  float *__restrict__ out, long long sOg, const int *__restrict__ rows) {
  const int g = blockIdx.y;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= (rows ? rows[g] : b)) return;
  const int lane = threadIdx.x & 63;
  const T *row = X + (long long)g * sXg + (long long)i * ld;
  constexpr int V = Vec<T>::N;
  float s = 0.0f;
  const int cv = cols / V * V;
  for (int c = lane * V; c < cv; c += 64 * V) {
    float f[V];
    Vec<T>::load(row + c, f);
#pragma unroll
    for (int k = 0; k < V; ++k) s = fmaf(f[k], f[k], s);
  }
  for (int c = cv + lane; c < cols; c += 64) {
    const float f = Elem<T>::ld(row + c);
    s = fmaf(f, f, s);
  }
  s = wave_sum(s);
  if (lane == 0) out[(long long)g * sOg + i] = s;
}

// Column sums in two fixed-order stages.  Stage 1: a block owns CL columns x COLSUM_ROWS rows
// (256 / CL row-lanes striding over them, added in lane order) and writes one partial per column;
// stage 2 adds the partials of all row-blocks in index order and scales.  CL = 64, or 16 for narrow
// matrices (the signals of a small last layer), where more row-lanes shorten each lane's serial walk.
template <class T, int CL>
__global__ void __launch_bounds__(256) col_sum_stage1(const T *__restrict__ X, long long sXg, int ld, int cols,
                                                      int b, float *__restrict__ part, int nsplit,
                                                      const int *__restrict__ rows) {
  constexpr int RL = 256 / CL;
  __shared__ float red[RL][CL];
  const int g = blockIdx.z, rs = blockIdx.y;
  const int cl = threadIdx.x % CL, rl = threadIdx.x / CL;
  const int c = blockIdx.x * CL + cl;
  const int r0 = rs * COLSUM_ROWS, r1 = min(rows ? rows[g] : b, r0 + COLSUM_ROWS);
  float s = 0.0f;
  if (c < cols) {
    const T *p = X + (long long)g * sXg + c;
    for (int i = r0 + rl; i < r1; i += RL) s += Elem<T>::ld(p + (long long)i * ld);
  }
  red[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && c < cols) {
    float t = red[0][cl];
#pragma unroll
    for (int k = 1; k < RL; ++k) t += red[k][cl];
    part[((long long)g * nsplit + rs) * cols + c] = t;
  }
}
// Stage 2: a block owns 64 columns; its four row-lanes add the partials r = lane, lane + 4, ... in that
// order and the four sums are combined in lane order.
__global__ void __launch_bounds__(256) col_sum_stage2(const float *__restrict__ part, int cols, int nsplit,
                                                      float alpha, float *__restrict__ out, long long sOg,
                                                      const int *__restrict__ rows, int tile_m, int parts_per_tile,
                                                      int accumulate) {
  __shared__ float red[4][64];
  const int g = blockIdx.y, cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int c = blockIdx.x * 64 + cl;
  int ns = nsplit;
  if (rows) {
    alpha = 1.0f / (float)rows[g];
    if (tile_m > 0) ns = (rows[g] + tile_m - 1) / tile_m * parts_per_tile;   // only these were written
  }
  float s = 0.0f;
  if (c < cols) {
    const float *p = part + (long long)g * nsplit * cols + c;
    for (int r = rl; r < ns; r += 4) s += p[(long long)r * cols];
  }
  red[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && c < cols) {
    const float t = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
    float *o = out + (long long)g * sOg + c;
    *o = accumulate ? fmaf(alpha, t, *o) : alpha * t;
  }
}

__global__ void __launch_bounds__(256) col_sum_stage2_many(const ColFinishMany p) {
  __shared__ float red[4][64];
  const int l = blockIdx.z, g = blockIdx.y, cl = threadIdx.x & 63, rl = threadIdx.x >> 6;
  const int cols = p.cols[l];
  if (blockIdx.x * 64 >= cols) return;             // uniform over the block
  const int c = blockIdx.x * 64 + cl;
  int ns = p.nsplit[l];
  float alpha = p.alpha;
  if (p.rows) {
    alpha = 1.0f / (float)p.rows[g];
    if (p.tile_m[l] > 0) ns = (p.rows[g] + p.tile_m[l] - 1) / p.tile_m[l] * p.parts_per_tile[l];
  }
  float s = 0.0f;
  if (c < cols) {
    const float *q = p.part[l] + (long long)g * p.nsplit[l] * cols + c;
    for (int r = rl; r < ns; r += 4) s += q[(long long)r * cols];
  }
  red[rl][cl] = s;
  __syncthreads();
  if (rl == 0 && c < cols) {
    const float t = ((red[0][cl] + red[1][cl]) + red[2][cl]) + red[3][cl];
    float *o = p.out + (long long)g * p.sOg + p.out_off[l] + c;
    *o = p.accumulate ? fmaf(alpha, t, *o) : alpha * t;
  }
}

__global__ void rowdot_f32_kernel(const float *__restrict__ D, long long sDg, int ldd,
                                  const float *__restrict__ U, long long sUg, int ldu, int cols,
                                  int b, float *__restrict__ q, long long sQg, int accumulate,
                                  const int *__restrict__ rows) {
  const int g = blockIdx.y;
  const int i = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
  if (i >= (rows ? rows[g] : b)) return;
  const int lane = threadIdx.x & 63;
  const float *d = D + (long long)g * sDg + (long long)i * ldd;
  const float *u = U + (long long)g * sUg + (long long)i * ldu;
  float s = 0.0f;
  for (int c = lane; c < cols; c += 64) s = fmaf(d[c], u[c], s);
  s = wave_sum(s);
  if (lane == 0) {
    float *o = q + (long long)g * sQg + i;
    *o = accumulate ? *o + s : s;
  }
}

// ---- statistics ---------------------------------------------------------------------------
// Stage 1a (grid: PBLK x groups): per-sample squared gradient norms
//   n_i = sum_l ||delta_i^l||^2 (||a_i^{l-1}||^2 + [bias])   and   q_i = sum_l sum_parts ...
// with block partial sums of n_i, q_i, q_i^2 and the loss, in double.
// s = (((s0 + base[0]) + base[stride]) + base[2 stride]) + ... over n entries: the additions keep their order, the
// loads go out eight at a time (one at a time, n dependent round trips to memory dominate the kernel).
__device__ __forceinline__ float sum_strided(float s0, const float *__restrict__ base, int n, long long stride) {
  float s = s0;
  int k = 0;
  for (; k + 8 <= n; k += 8) {
    float v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = base[(long long)(k + u) * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) s += v[u];
  }
  if (k + 4 <= n) {
    float v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = base[(long long)(k + u) * stride];
#pragma unroll
    for (int u = 0; u < 4; ++u) s += v[u];
    k += 4;
  }
  for (; k < n; ++k) s += base[(long long)k * stride];
  return s;
}

// Blocks 0 .. nb-1 of a group share its samples (block j owns samples 256 j + t, then strides of 256 nb);
// the launch uses nb = min(PBLK, ceil(b / 256)) blocks and stage 2 takes the other partials as zero.
__device__ __forceinline__ void stats_samples_block(const StatsP &p, int g, int blk, int nb, double *red) {
  double s1 = 0.0, s3 = 0.0, s4 = 0.0, sl = 0.0;
  const float hb = p.has_bias ? 1.0f : 0.0f;
  const int bg = p.rows ? p.rows[g] : p.b;
  for (int i = blk * 256 + threadIdx.x; i < bg; i += 256 * nb) {
    const long long o = (long long)g * p.sNg + i;
    if (p.do_n) {
      float n = 0.0f;
      for (int l = 0; l < p.L; ++l) {
        const float a = sum_strided(0.0f, p.an[l] + (long long)g * p.an_sg[l] + i, p.an_parts[l], p.sNg);
        const float d = sum_strided(0.0f, p.dn[l] + (long long)g * p.dn_sg[l] + i, p.dn_parts[l], p.sNg);
        n = fmaf(d, a + hb, n);
      }
      if (p.n_out) p.n_out[o] = n;
      s1 += (double)n;
      sl += (double)p.loss[o];
    }
    if (p.do_q) {
      float q = 0.0f;
      for (int l = 0; l < p.L; ++l) {
        q = sum_strided(q, p.qpart[l] + (long long)g * p.sQg[l] + i, p.nparts[l], p.sQpart[l]);
      }
      if (p.q_out) p.q_out[o] = q;
      s4 += (double)q;
      s3 += (double)q * (double)q;
    }
  }
  double *out = p.partials + ((long long)g * 5) * STATS_PBLK + blk;
  double r;
  r = block_sum<4>(s1, red); if (threadIdx.x == 0) out[0 * STATS_PBLK] = r;
  r = block_sum<4>(s3, red); if (threadIdx.x == 0) out[2 * STATS_PBLK] = r;
  r = block_sum<4>(s4, red); if (threadIdx.x == 0) out[3 * STATS_PBLK] = r;
  r = block_sum<4>(sl, red); if (threadIdx.x == 0) out[4 * STATS_PBLK] = r;
}
__device__ __forceinline__ void stats_gradsq_parts_block(const float *__restrict__ sq_wave, long long per_group,
                                                         long long stride, double *__restrict__ partials, int g, int blk,
                                                         double *red) {
  const float *p = sq_wave + (long long)g * (stride ? stride : per_group);
  double s = 0.0;
  for (long long i = blk * 256LL + threadIdx.x; i < per_group; i += 256LL * STATS_PBLK) s += (double)p[i];
  const double r = block_sum<4>(s, red);
  if (threadIdx.x == 0) partials[((long long)g * 5 + 1) * STATS_PBLK + blk] = r;
}
// grid (nb_samples + nb_parts) x groups: the first nb_samples blocks of a group take the per-sample sums,
// the other PBLK blocks (present when the update kernel left per-wavefront partials) the ||gbar||^2 partials.
__global__ void __launch_bounds__(256) stats_samples_kernel(const StatsP p, int nb_samples) {
  __shared__ double red[4];
  const int g = blockIdx.y, blk = blockIdx.x;
  if (blk < nb_samples) stats_samples_block(p, g, blk, nb_samples, red);
  else stats_gradsq_parts_block(p.sq_wave, p.n_sq_wave, p.sq_stride, p.partials, g, blk - nb_samples, red);
}

// Stage 1b (grid: PBLK x groups): ||gbar||^2 over the padded gradient vector.
__global__ void __launch_bounds__(256) stats_gradsq_kernel(const float *__restrict__ grad, long long Ppad,
                                                           double *__restrict__ partials) {
  __shared__ double red[4];
  const int g = blockIdx.y;
  const float4 *p4 = reinterpret_cast<const float4 *>(grad + (long long)g * Ppad);
  const long long n4 = Ppad / 4;
  double s = 0.0;
  for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n4; i += 256LL * STATS_PBLK) {
    const float4 v = ld_stream(p4 + i);
    const float t = fmaf(v.x, v.x, fmaf(v.y, v.y, fmaf(v.z, v.z, v.w * v.w)));
    s += (double)t;
  }
  const double r = block_sum<4>(s, red);
  if (threadIdx.x == 0) partials[((long long)g * 5 + 1) * STATS_PBLK + blockIdx.x] = r;
}

// Stage 2 (grid: groups): add the PBLK partials of each of the five sums in index order.
// sel / acc: bit k set = sum k is produced by this launch / is added to the stored value.
// nb_samples: how many partials of the per-sample sums (all but k = 1) this step wrote; the rest count as zero.
__global__ void __launch_bounds__(256) stats_final_kernel(const double *__restrict__ partials,
                                                          double *__restrict__ stats, double *__restrict__ stats_host,
                                                          int sel, int acc, int nb_samples, double ticket) {
  __shared__ double red[4];
  const int g = blockIdx.x;
  static_assert(STATS_PBLK == 256, "one partial per thread");
  for (int k = 0; k < 5; ++k) {
    if (!((sel >> k) & 1)) continue;
    const bool live = k == 1 || (int)threadIdx.x < nb_samples;
    const double v = live ? partials[((long long)g * 5 + k) * STATS_PBLK + threadIdx.x] : 0.0;
    const double r = block_sum<4>(v, red);
    if (threadIdx.x == 0) {
      const double v = ((acc >> k) & 1) ? stats[g * 8 + k] + r : r;
      stats[g * 8 + k] = v;
      if (stats_host) stats_host[g * 8 + k] = v;
    }
  }
  if (stats_host && threadIdx.x == 0) {
    __threadfence_system();                       // the sums above reach host memory before the ticket does
    *reinterpret_cast<volatile double *>(stats_host + g * 8 + 7) = ticket;
  }
}

// ---- optimizer update ------------------------------------------------------------------------
// With SQ the kernel also leaves, per wavefront (256 consecutive parameters), the sum of the squared
// gradient entries it read: ||gbar||^2 then costs no second pass over the gradient.  (SQ launches use
// a grid that covers the data in one pass, and n is a multiple of 256, so wavefronts are whole.)
template <int OPT, bool SHADOW, bool SQ>
__global__ void __launch_bounds__(256) update_kernel(const UpdateP pin) {
  UpdateP p = pin;
  if (p.scal) { p.lr = p.scal[0]; p.c1 = p.scal[1]; p.c2 = p.scal[2]; }     // uniform loads
  const OptHyper h = {p.lr, p.momentum, p.beta1, p.beta2, p.eps, p.wd, p.c1, p.c2};
  const long long n4 = p.n / 4;
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n4; i += stride) {
    float4 x = ld_stream(reinterpret_cast<const float4 *>(p.x) + i);
    const float4 g = ld_stream(reinterpret_cast<const float4 *>(p.g) + i);
    if (SQ) {
      const float t = wave_sum(fmaf(g.x, g.x, fmaf(g.y, g.y, fmaf(g.z, g.z, g.w * g.w))));
      if ((threadIdx.x & 63) == 0) p.sq_wave[i >> 6] = t;
    }
    float xs[4] = {x.x, x.y, x.z, x.w};
    const float gs[4] = {g.x, g.y, g.z, g.w};
    float vs[4] = {0.f, 0.f, 0.f, 0.f}, ms[4] = {0.f, 0.f, 0.f, 0.f};
    if (OPT != OPT_SGD) {
      const float4 v = ld_stream(reinterpret_cast<const float4 *>(p.v) + i);
      vs[0] = v.x; vs[1] = v.y; vs[2] = v.z; vs[3] = v.w;
    }
    if (OPT == OPT_ADAMW) {
      const float4 m = ld_stream(reinterpret_cast<const float4 *>(p.m) + i);
      ms[0] = m.x; ms[1] = m.y; ms[2] = m.z; ms[3] = m.w;
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) opt_step_elem<OPT>(xs[k], gs[k], vs[k], ms[k], h);
    if (OPT != OPT_SGD) st_stream(reinterpret_cast<float4 *>(p.v) + i, make_float4(vs[0], vs[1], vs[2], vs[3]));
    if (OPT == OPT_ADAMW) st_stream(reinterpret_cast<float4 *>(p.m) + i, make_float4(ms[0], ms[1], ms[2], ms[3]));
    st_stream(reinterpret_cast<float4 *>(p.x) + i, make_float4(xs[0], xs[1], xs[2], xs[3]));
    if (SHADOW) {
      uint2 o;
      o.x = pack2bf(xs[0], xs[1]);
      o.y = pack2bf(xs[2], xs[3]);
      st_stream(reinterpret_cast<uint2 *>(p.shadow) + i, o);
    }
  }
}

// The step of the bias vectors alone, for steps whose weights were updated inside the weight-gradient epilogue.
// grid (ceil(max width / 256), groups, layers); one bias per thread; each block also leaves the sum of its
// squared gradient entries in sq[g * sSqg + slot0 + (layer * gridDim.x + blockIdx.x)] (their share of ||gbar||^2).
template <int OPT>
__global__ void __launch_bounds__(256) update_bias_kernel(const BiasUpdateP p) {
  __shared__ double red[4];
  const int l = blockIdx.z, g = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
  OptHyper h = {p.lr, p.momentum, p.beta1, p.beta2, p.eps, p.wd, p.c1, p.c2};
  if (p.scal) { h.lr = p.scal[0]; h.c1 = p.scal[1]; h.c2 = p.scal[2]; }
  float gg = 0.0f;
  if (j < p.width[l]) {
    const long long o = (long long)g * p.stride + p.off[l] + j;
    const float gr = p.g[o];
    float x = p.x[o], v = OPT != OPT_SGD ? p.v[o] : 0.0f, m = OPT == OPT_ADAMW ? p.m[o] : 0.0f;
    opt_step_elem<OPT>(x, gr, v, m, h);
    p.x[o] = x;
    if (OPT != OPT_SGD) p.v[o] = v;
    if (OPT == OPT_ADAMW) p.m[o] = m;
    if (p.shadow) p.shadow[o] = f2bf(x);
    gg = gr * gr;
  }
  const double r = block_sum<4>((double)gg, red);
  if (threadIdx.x == 0) p.sq[(long long)g * p.sSqg + p.slot0 + l * gridDim.x + blockIdx.x] = (float)r;
}

// ---- replica average ------------------------------------------------------------------------
// Thread owns 4 consecutive parameters: reads them from all replicas (in replica order), divides
// once, writes the mean back to every replica (and the bf16 shadow if there is one).
template <bool SHADOW>
__global__ void __launch_bounds__(256) average_f32_kernel(float *__restrict__ x, bf16_t *__restrict__ shadow,
                                                          int groups, long long Ppad) {
  const long long n4 = Ppad / 4;
  const long long stride = (long long)gridDim.x * 256;
  const float Mf = (float)groups;
  for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n4; i += stride) {
    float4 s = ld_stream(reinterpret_cast<const float4 *>(x) + i);
    for (int g = 1; g < groups; ++g) {
      const float4 v = ld_stream(reinterpret_cast<const float4 *>(x + (long long)g * Ppad) + i);
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    s.x /= Mf; s.y /= Mf; s.z /= Mf; s.w /= Mf;
    uint2 o;
    if (SHADOW) { o.x = pack2bf(s.x, s.y); o.y = pack2bf(s.z, s.w); }
    for (int g = 0; g < groups; ++g) {
      st_stream(reinterpret_cast<float4 *>(x + (long long)g * Ppad) + i, s);
      if (SHADOW) st_stream(reinterpret_cast<uint2 *>(shadow + (long long)g * Ppad) + i, o);
    }
  }
}

__global__ void __launch_bounds__(256) average_bf16_kernel(bf16_t *__restrict__ x, int groups, long long n) {
  const long long n8 = n / 8;
  const long long stride = (long long)gridDim.x * 256;
  const float Mf = (float)groups;
  for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n8; i += stride) {
    float s[8];
    Vec<bf16_t>::load_stream(x + i * 8, s);
    for (int g = 1; g < groups; ++g) {
      float v[8];
      Vec<bf16_t>::load_stream(x + (long long)g * n + i * 8, v);
#pragma unroll
      for (int k = 0; k < 8; ++k) s[k] += v[k];
    }
    uint4 o;
    o.x = pack2bf(s[0] / Mf, s[1] / Mf);
    o.y = pack2bf(s[2] / Mf, s[3] / Mf);
    o.z = pack2bf(s[4] / Mf, s[5] / Mf);
    o.w = pack2bf(s[6] / Mf, s[7] / Mf);
    for (int g = 0; g < groups; ++g) st_stream(reinterpret_cast<uint4 *>(x + (long long)g * n + i * 8), o);
  }
}

// Two-pass form of the same averages for blocks far beyond the caches: the first kernel only reads
// (all replicas, same order of additions, same division) and leaves the mean in a buffer of one replica's
// size, the second only writes (its one read, the mean, comes from the caches).  HBM serves a pure read
// stream and a pure write stream faster than their mixture, which more than pays for the extra buffer.
// A block reads U * 4 KB of consecutive bytes from every replica: U independent vectors per thread keep more
// loads in flight (U = 4: the read pass of a 32-way average 3 % faster than with one vector per thread).
template <int U>
__global__ void __launch_bounds__(256) average_f32_reduce_kernel(const float *__restrict__ x, float *__restrict__ mean,
                                                                 int groups, long long Ppad) {
  const long long n4 = Ppad / 4;
  const long long base = (long long)blockIdx.x * (256 * U) + threadIdx.x;
  const float Mf = (float)groups;
  float4 s[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long i = base + u * 256;
    s[u] = i < n4 ? ld_stream(reinterpret_cast<const float4 *>(x) + i) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  for (int g = 1; g < groups; ++g) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = base + u * 256;
      if (i < n4) {
        const float4 v = ld_stream(reinterpret_cast<const float4 *>(x + (long long)g * Ppad) + i);
        s[u].x += v.x; s[u].y += v.y; s[u].z += v.z; s[u].w += v.w;
      }
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long i = base + u * 256;
    if (i < n4) reinterpret_cast<float4 *>(mean)[i] = make_float4(s[u].x / Mf, s[u].y / Mf, s[u].z / Mf, s[u].w / Mf);
  }
}
template <bool SHADOW>
__global__ void __launch_bounds__(256) average_f32_spread_kernel(const float *__restrict__ mean, float *__restrict__ x,
                                                                 bf16_t *__restrict__ shadow, int groups, long long Ppad) {
  const long long i = blockIdx.x * 256LL + threadIdx.x;
  if (i >= Ppad / 4) return;
  const float4 s = reinterpret_cast<const float4 *>(mean)[i];
  uint2 o;
  if (SHADOW) { o.x = pack2bf(s.x, s.y); o.y = pack2bf(s.z, s.w); }
  for (int g = 0; g < groups; ++g) {
    st_stream(reinterpret_cast<float4 *>(x + (long long)g * Ppad) + i, s);
    if (SHADOW) st_stream(reinterpret_cast<uint2 *>(shadow + (long long)g * Ppad) + i, o);
  }
}
template <int U>
__global__ void __launch_bounds__(256) average_bf16_reduce_kernel(const bf16_t *__restrict__ x, bf16_t *__restrict__ mean,
                                                                  int groups, long long n) {
  const long long n8 = n / 8;
  const long long base = (long long)blockIdx.x * (256 * U) + threadIdx.x;
  const float Mf = (float)groups;
  float s[U][8];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long i = base + u * 256;
    if (i < n8) Vec<bf16_t>::load_stream(x + i * 8, s[u]);
  }
  for (int g = 1; g < groups; ++g) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const long long i = base + u * 256;
      if (i < n8) {
        float v[8];
        Vec<bf16_t>::load_stream(x + (long long)g * n + i * 8, v);
#pragma unroll
        for (int k = 0; k < 8; ++k) s[u][k] += v[k];
      }
    }
  }
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const long long i = base + u * 256;
    if (i < n8) {
      uint4 o;
      o.x = pack2bf(s[u][0] / Mf, s[u][1] / Mf);
      o.y = pack2bf(s[u][2] / Mf, s[u][3] / Mf);
      o.z = pack2bf(s[u][4] / Mf, s[u][5] / Mf);
      o.w = pack2bf(s[u][6] / Mf, s[u][7] / Mf);
      reinterpret_cast<uint4 *>(mean)[i] = o;
    }
  }
}
__global__ void __launch_bounds__(256) average_bf16_spread_kernel(const bf16_t *__restrict__ mean, bf16_t *__restrict__ x,
                                                                  int groups, long long n) {
  const long long i = blockIdx.x * 256LL + threadIdx.x;
  if (i >= n / 8) return;
  const uint4 o = reinterpret_cast<const uint4 *>(mean)[i];
  for (int g = 0; g < groups; ++g) st_stream(reinterpret_cast<uint4 *>(x + (long long)g * n + i * 8), o);
}

// sum_m ||g^m||^2 and ||mean_m g^m||^2 over the padded gradient block (Alg. 2 statistics).
// Stage 1 (data-sized grid): a thread owns four consecutive parameters, reads them from every worker's
// gradient (in worker order) and adds its two contributions; one pair of partials per block.
// Stage 2 (one block): the block partials are added in index order.
__global__ void __launch_bounds__(256) cross_worker_kernel(const float *__restrict__ grad, int groups,
                                                           long long Ppad, double *__restrict__ partials, int nblocks) {
  __shared__ double red[4];
  const long long n4 = Ppad / 4;
  const long long i = blockIdx.x * 256LL + threadIdx.x;
  double ss = 0.0, sm = 0.0;
  if (i < n4) {
    double sx = 0.0, sy = 0.0, sz = 0.0, sw = 0.0;
    for (int g = 0; g < groups; ++g) {
      const float4 v = ld_stream(reinterpret_cast<const float4 *>(grad + (long long)g * Ppad) + i);
      const double x = v.x, y = v.y, z = v.z, w = v.w;
      sx += x; sy += y; sz += z; sw += w;
      ss += x * x + y * y + z * z + w * w;
    }
    const double inv = 1.0 / (double)groups;
    sx *= inv; sy *= inv; sz *= inv; sw *= inv;
    sm = sx * sx + sy * sy + sz * sz + sw * sw;
  }
  double r = block_sum<4>(ss, red);
  if (threadIdx.x == 0) partials[blockIdx.x] = r;
  r = block_sum<4>(sm, red);
  if (threadIdx.x == 0) partials[nblocks + blockIdx.x] = r;
}
__global__ void __launch_bounds__(256) cross_worker_final_kernel(const double *__restrict__ partials, int nblocks,
                                                                 double *__restrict__ out) {
  __shared__ double red[4];
  for (int k = 0; k < 2; ++k) {
    double s = 0.0;
    for (int i = threadIdx.x; i < nblocks; i += 256) s += partials[(long long)k * nblocks + i];
    const double r = block_sum<4>(s, red);
    if (threadIdx.x == 0) out[k] = r;
  }
}

// Plain copy of n16 16-byte vectors, one per thread: the known-traffic reference that hardware
// counters are scaled by.
__global__ void __launch_bounds__(256) copy_probe_kernel(const uint4 *__restrict__ src, uint4 *__restrict__ dst,
                                                         long long n16) {
  const long long i = blockIdx.x * 256LL + threadIdx.x;
  if (i < n16) dst[i] = src[i];
}

// blockIdx.z = layer; the layers of a step share one launch
// OPT < 0: store the finished gradient; OPT >= 0: apply that optimizer's step to the parameters instead.
template <int OPT>
__global__ void __launch_bounds__(256) splitk_finish_kernel(const SplitKFinishMany p) {
  __shared__ double red[4];
  const int l = blockIdx.z, g = blockIdx.y;
  const long long mn = p.mn[l];
  const long long i = blockIdx.x * 256LL + threadIdx.x;          // float4 index inside the group's layer
  if (blockIdx.x * 1024LL >= mn) return;                         // uniform over the block
  const bool live = i * 4 < mn;
  float gg = 0.0f;
  if (live) {
    const int ksplit = p.ksplit[l];
    const float alpha = p.rows ? 1.0f / (float)p.rows[g] : p.alpha;
    const float *q = p.kpart[l] + (long long)g * ksplit * mn + i * 4;
    float4 s = ld_stream(reinterpret_cast<const float4 *>(q));
    for (int sp = 1; sp < ksplit; ++sp) {
      const float4 v = ld_stream(reinterpret_cast<const float4 *>(q + (long long)sp * mn));
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    s.x *= alpha; s.y *= alpha; s.z *= alpha; s.w *= alpha;
    const long long o = (long long)g * p.sCg + p.c_off[l] + i * 4;
    if (OPT < 0) {
      float4 *c = reinterpret_cast<float4 *>(p.C + o);
      if (p.accumulate) { const float4 old = *c; s.x += old.x; s.y += old.y; s.z += old.z; s.w += old.w; }
      *c = s;
    } else {
      OptHyper h = {p.upd_lr, p.upd_momentum, p.upd_beta1, p.upd_beta2, p.upd_eps, p.upd_wd, p.upd_c1, p.upd_c2};
      if (p.upd_scal) { h.lr = p.upd_scal[0]; h.c1 = p.upd_scal[1]; h.c2 = p.upd_scal[2]; }
      const float4 x4 = ld_stream(reinterpret_cast<const float4 *>(p.upd_x + o));
      float xs[4] = {x4.x, x4.y, x4.z, x4.w}, vs[4] = {0.f, 0.f, 0.f, 0.f}, ms[4] = {0.f, 0.f, 0.f, 0.f};
      const float gs[4] = {s.x, s.y, s.z, s.w};
      if (OPT != OPT_SGD) {
        const float4 v4 = ld_stream(reinterpret_cast<const float4 *>(p.upd_v + o));
        vs[0] = v4.x; vs[1] = v4.y; vs[2] = v4.z; vs[3] = v4.w;
      }
      if (OPT == OPT_ADAMW) {
        const float4 m4 = ld_stream(reinterpret_cast<const float4 *>(p.upd_m + o));
        ms[0] = m4.x; ms[1] = m4.y; ms[2] = m4.z; ms[3] = m4.w;
      }
#pragma unroll
      for (int k = 0; k < 4; ++k) opt_step_elem<(OPT < 0 ? 0 : OPT)>(xs[k], gs[k], vs[k], ms[k], h);
      st_stream(reinterpret_cast<float4 *>(p.upd_x + o), make_float4(xs[0], xs[1], xs[2], xs[3]));
      if (OPT != OPT_SGD) st_stream(reinterpret_cast<float4 *>(p.upd_v + o), make_float4(vs[0], vs[1], vs[2], vs[3]));
      if (OPT == OPT_ADAMW) st_stream(reinterpret_cast<float4 *>(p.upd_m + o), make_float4(ms[0], ms[1], ms[2], ms[3]));
      if (p.upd_shadow) {
        uint2 w;
        w.x = pack2bf(xs[0], xs[1]); w.y = pack2bf(xs[2], xs[3]);
        st_stream(reinterpret_cast<uint2 *>(p.upd_shadow + o), w);
      }
      gg = fmaf(s.x, s.x, fmaf(s.y, s.y, fmaf(s.z, s.z, s.w * s.w)));
    }
    if (p.C2) {
      uint2 w;
      w.x = pack2bf(s.x, s.y); w.y = pack2bf(s.z, s.w);
      reinterpret_cast<uint2 *>(p.C2 + (long long)g * p.sC2g + p.c_off[l])[i] = w;
    }
  }
  if (OPT >= 0) {
    const double r = block_sum<4>((double)gg, red);
    if (threadIdx.x == 0) p.upd_sq[(long long)g * p.upd_sSqg + p.upd_slot0[l] + blockIdx.x] = (float)r;
  }
}

__global__ void __launch_bounds__(256) stage_step_inputs_kernel(const int32_t *__restrict__ src, int32_t *__restrict__ dst,
                                                                long long n, float lr, float c1, float c2,
                                                                float *__restrict__ scal) {
  const long long stride = (long long)gridDim.x * 256;
  for (long long i = blockIdx.x * 256LL + threadIdx.x; i < n; i += stride) dst[i] = src[i];
  if (blockIdx.x == 0 && threadIdx.x == 0) { scal[0] = lr; scal[1] = c1; scal[2] = c2; }
}

struct IntsArg { int v[SET_INTS_MAX]; };
__global__ void set_ints_kernel(const IntsArg a, int n, int *__restrict__ dst) {
  if ((int)threadIdx.x < n) dst[threadIdx.x] = a.v[threadIdx.x];
}

__global__ void fill_zero_kernel(uint4 *p, long long n16) {
  const long long stride = (long long)gridDim.x * blockDim.x;
  for (long long i = blockIdx.x * (long long)blockDim.x + threadIdx.x; i < n16; i += stride)
    p[i] = make_uint4(0, 0, 0, 0);
}

inline int grid_for(long long work_items, int per_block, int max_blocks) {
  long long b = (work_items + per_block - 1) / per_block;
  if (b < 1) b = 1;
  if (b > max_blocks) b = max_blocks;
  return (int)b;
}

}  // namespace

hipError_t launch_convert_f32_to_bf16(const float *src, bf16_t *dst, long long n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(convert_kernel, dim3(grid_for(n / 4, 256, 1 << 30)), dim3(256), 0, s, src, dst, n);
  return hipGetLastError();
}

hipError_t launch_gather_rows(int is_bf16, const void *X, int d, int N, const int32_t *idx, int ldi, int groups, int b,
                              void *A0, long long sA0g, int ldo, float *an0, long long sNg, const int *rows,
                              hipStream_t s) {
  const dim3 grid((b + 3) / 4, groups), blk(256);
  if (is_bf16)
    hipLaunchKernelGGL(gather_kernel<bf16_t>, grid, blk, 0, s, static_cast<const bf16_t *>(X), d, N, idx, ldi, b,
                       static_cast<bf16_t *>(A0), sA0g, ldo, an0, sNg, rows);
  else
    hipLaunchKernelGGL(gather_kernel<float>, grid, blk, 0, s, static_cast<const float *>(X), d, N, idx, ldi, b,
                       static_cast<float *>(A0), sA0g, ldo, an0, sNg, rows);
  return hipGetLastError();
}

hipError_t launch_softmax_ce(int is_bf16, const float *Z, long long sZg, int ldz, int K, const int32_t *y,
                             int N, const int32_t *idx, int ldi, int groups, int b, void *D, long long sDg, int ldd,
                             float *dn, float *loss, long long sNg, const int *rows, hipStream_t s) {
  const dim3 blk(256);
  if (ldd <= 16) {
    const dim3 grid((b + 15) / 16, groups);
    if (is_bf16)
      hipLaunchKernelGGL((softmax_ce_kernel<bf16_t, 16>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                         static_cast<bf16_t *>(D), sDg, ldd, dn, loss, sNg, rows);
    else
      hipLaunchKernelGGL((softmax_ce_kernel<float, 16>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                         static_cast<float *>(D), sDg, ldd, dn, loss, sNg, rows);
    return hipGetLastError();
  }
  if (ldd <= 128 && (ldd & 3) == 0 && (ldz & 3) == 0 && ldz >= ldd && (sZg & 3) == 0 && (sDg & 3) == 0) {
    const dim3 grid((b + 7) / 8, groups);
    if (is_bf16)
      hipLaunchKernelGGL((softmax_ce_vec_kernel<bf16_t>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                         static_cast<bf16_t *>(D), sDg, ldd, dn, loss, sNg, rows);
    else
      hipLaunchKernelGGL((softmax_ce_vec_kernel<float>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                         static_cast<float *>(D), sDg, ldd, dn, loss, sNg, rows);
    return hipGetLastError();
  }
  const dim3 grid((b + 3) / 4, groups);
  if (is_bf16)
    hipLaunchKernelGGL((softmax_ce_kernel<bf16_t, 64>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                       static_cast<bf16_t *>(D), sDg, ldd, dn, loss, sNg, rows);
  else
    hipLaunchKernelGGL((softmax_ce_kernel<float, 64>), grid, blk, 0, s, Z, sZg, ldz, K, y, N, idx, ldi, b,
                       static_cast<float *>(D), sDg, ldd, dn, loss, sNg, rows);
  return hipGetLastError();
}

hipError_t launch_row_sqnorm(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups, int b,
                             float *out, long long sOg, const int *rows, hipStream_t s) {
  const dim3 grid((b + 3) / 4, groups), blk(256);
  if (is_bf16)
    hipLaunchKernelGGL(row_sqnorm_kernel<bf16_t>, grid, blk, 0, s, static_cast<const bf16_t *>(X), sXg, ld,
                       cols, b, out, sOg, rows);
  else
    hipLaunchKernelGGL(row_sqnorm_kernel<float>, grid, blk, 0, s, static_cast<const float *>(X), sXg, ld,
                       cols, b, out, sOg, rows);
  return hipGetLastError();
}

static void launch_col_sum_stage1(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups, int b,
                                  float *scratch, int nsplit, const int *rows, hipStream_t s) {
  const dim3 blk(256);
  if (cols <= 16) {
    const dim3 grid((cols + 15) / 16, nsplit, groups);
    if (is_bf16)
      hipLaunchKernelGGL((col_sum_stage1<bf16_t, 16>), grid, blk, 0, s, static_cast<const bf16_t *>(X), sXg, ld, cols, b,
                         scratch, nsplit, rows);
    else
      hipLaunchKernelGGL((col_sum_stage1<float, 16>), grid, blk, 0, s, static_cast<const float *>(X), sXg, ld, cols, b,
                         scratch, nsplit, rows);
    return;
  }
  const dim3 grid((cols + 63) / 64, nsplit, groups);
  if (is_bf16)
    hipLaunchKernelGGL((col_sum_stage1<bf16_t, 64>), grid, blk, 0, s, static_cast<const bf16_t *>(X), sXg, ld, cols, b,
                       scratch, nsplit, rows);
  else
    hipLaunchKernelGGL((col_sum_stage1<float, 64>), grid, blk, 0, s, static_cast<const float *>(X), sXg, ld, cols, b,
                       scratch, nsplit, rows);
}

hipError_t launch_col_sum(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups, int b,
                          float alpha, float *out, long long sOg, float *scratch, const int *rows, int accumulate,
                          hipStream_t s) {
  const int nsplit = (b + COLSUM_ROWS - 1) / COLSUM_ROWS;
  launch_col_sum_stage1(is_bf16, X, sXg, ld, cols, groups, b, scratch, nsplit, rows, s);
  // stage 1 writes every partial (zeros past a group's rows), so stage 2 adds all of them
  hipLaunchKernelGGL(col_sum_stage2, dim3((cols + 63) / 64, groups), dim3(256), 0, s, scratch, cols, nsplit,
                     alpha, out, sOg, rows, 0, 0, accumulate);
  return hipGetLastError();
}

hipError_t launch_col_sum_partials(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups, int b,
                                   float *scratch, const int *rows, hipStream_t s) {
  const int nsplit = (b + COLSUM_ROWS - 1) / COLSUM_ROWS;
  launch_col_sum_stage1(is_bf16, X, sXg, ld, cols, groups, b, scratch, nsplit, rows, s);
  return hipGetLastError();
}

hipError_t launch_col_sum_finish_many(const ColFinishMany &p, int groups, hipStream_t s) {
  if (p.n < 1 || p.n > ColFinishMany::MAXN) return hipErrorInvalidValue;
  int mx = 0;
  for (int l = 0; l < p.n; ++l) mx = p.cols[l] > mx ? p.cols[l] : mx;
  hipLaunchKernelGGL(col_sum_stage2_many, dim3((mx + 63) / 64, groups, p.n), dim3(256), 0, s, p);
  return hipGetLastError();
}

hipError_t launch_rowdot_f32(const float *D, long long sDg, int ldd, const float *U, long long sUg, int ldu,
                             int cols, int groups, int b, float *q, long long sQg, int accumulate,
                             const int *rows, hipStream_t s) {
  hipLaunchKernelGGL(rowdot_f32_kernel, dim3((b + 3) / 4, groups), dim3(256), 0, s, D, sDg, ldd, U, sUg, ldu,
                     cols, b, q, sQg, accumulate, rows);
  return hipGetLastError();
}

hipError_t launch_stats(const StatsP &p, hipStream_t s) {
  if (p.do_q && !p.want_ip) return hipErrorInvalidValue;
  int sel = 0, acc = 0;
  if (p.do_n) { sel |= 1 | 16; if (p.acc_n) acc |= 1 | 16; }
  if (p.do_q) { sel |= 4 | 8; if (p.acc_q) acc |= 4 | 8; }
  if (p.grad && p.sq_wave) return hipErrorInvalidValue;
  if (p.grad || p.sq_wave) sel |= 2;
  if (!sel && !p.stats_host) return hipSuccess;       // (with a mirror the final kernel still delivers the ticket)
  int nb_samples = 0;
  if (p.do_n || p.do_q) {
    nb_samples = (p.b + 255) / 256;
    nb_samples = nb_samples < 1 ? 1 : (nb_samples > STATS_PBLK ? STATS_PBLK : nb_samples);
  }
  const int nb_parts = p.sq_wave ? STATS_PBLK : 0;
  if (nb_samples + nb_parts > 0)
    hipLaunchKernelGGL(stats_samples_kernel, dim3(nb_samples + nb_parts, p.groups), dim3(256), 0, s, p, nb_samples);
  if (p.grad)
    hipLaunchKernelGGL(stats_gradsq_kernel, dim3(STATS_PBLK, p.groups), dim3(256), 0, s, p.grad, p.Ppad,
                       p.partials);
  hipLaunchKernelGGL(stats_final_kernel, dim3(p.groups), dim3(256), 0, s, p.partials, p.stats, p.stats_host, sel, acc,
                     nb_samples, p.ticket);
  return hipGetLastError();
}

hipError_t launch_update(const UpdateP &p, hipStream_t s) {
  // one 16-byte vector per thread and a grid as large as the data: measured fastest on MI355X
  const dim3 grid(grid_for(p.n / 4, 256, 1 << 30)), blk(256);
  const bool sh = p.shadow != nullptr, sq = p.sq_wave != nullptr;
  if (sq && (p.n & 255)) return hipErrorInvalidValue;
#define ABS_UPD(O)                                                                  \
  do {                                                                              \
    if (sh && sq) hipLaunchKernelGGL((update_kernel<O, true, true>), grid, blk, 0, s, p);        \
    else if (sh) hipLaunchKernelGGL((update_kernel<O, true, false>), grid, blk, 0, s, p);        \
    else if (sq) hipLaunchKernelGGL((update_kernel<O, false, true>), grid, blk, 0, s, p);        \
    else hipLaunchKernelGGL((update_kernel<O, false, false>), grid, blk, 0, s, p);               \
  } while (0)
  if (p.opt == OPT_SGD) ABS_UPD(OPT_SGD);
  else if (p.opt == OPT_SHB) ABS_UPD(OPT_SHB);
  else if (p.opt == OPT_ADAGRAD) ABS_UPD(OPT_ADAGRAD);
  else ABS_UPD(OPT_ADAMW);
#undef ABS_UPD
  return hipGetLastError();
}

int update_bias_slots(const BiasUpdateP &p) {
  int mx = 0;
  for (int l = 0; l < p.n; ++l) mx = p.width[l] > mx ? p.width[l] : mx;
  return p.n * ((mx + 255) / 256);
}

hipError_t launch_update_bias(const BiasUpdateP &p, int groups, hipStream_t s) {
  if (p.n < 1 || p.n > BiasUpdateP::MAXN) return hipErrorInvalidValue;
  int mx = 0;
  for (int l = 0; l < p.n; ++l) mx = p.width[l] > mx ? p.width[l] : mx;
  const dim3 grid((mx + 255) / 256, groups, p.n), blk(256);
  if (p.opt == OPT_SGD) hipLaunchKernelGGL(update_bias_kernel<OPT_SGD>, grid, blk, 0, s, p);
  else if (p.opt == OPT_SHB) hipLaunchKernelGGL(update_bias_kernel<OPT_SHB>, grid, blk, 0, s, p);
  else if (p.opt == OPT_ADAGRAD) hipLaunchKernelGGL(update_bias_kernel<OPT_ADAGRAD>, grid, blk, 0, s, p);
  else hipLaunchKernelGGL(update_bias_kernel<OPT_ADAMW>, grid, blk, 0, s, p);
  return hipGetLastError();
}

// Blocks of at least this many elements over all replicas take the two-pass form when the caller brings a buffer.
static constexpr long long AVERAGE_TWO_PASS_MIN = 32LL << 20;

hipError_t launch_average_f32(float *x, bf16_t *shadow, float *mean, int groups, long long Ppad, hipStream_t s) {
  const dim3 grid(grid_for(Ppad / 4, 256, 1 << 30)), blk(256);
  if (mean && groups > 1 && (long long)groups * Ppad >= AVERAGE_TWO_PASS_MIN) {
    const dim3 rgrid(grid_for((Ppad / 4 + 3) / 4, 256, 1 << 30));
    hipLaunchKernelGGL(average_f32_reduce_kernel<4>, rgrid, blk, 0, s, x, mean, groups, Ppad);
    if (shadow) hipLaunchKernelGGL(average_f32_spread_kernel<true>, grid, blk, 0, s, mean, x, shadow, groups, Ppad);
    else hipLaunchKernelGGL(average_f32_spread_kernel<false>, grid, blk, 0, s, mean, x, shadow, groups, Ppad);
    return hipGetLastError();
  }
  if (shadow) hipLaunchKernelGGL(average_f32_kernel<true>, grid, blk, 0, s, x, shadow, groups, Ppad);
  else hipLaunchKernelGGL(average_f32_kernel<false>, grid, blk, 0, s, x, shadow, groups, Ppad);
  return hipGetLastError();
}

hipError_t launch_average_bf16(bf16_t *x, bf16_t *mean, int groups, long long n, hipStream_t s) {
  const dim3 grid(grid_for(n / 8, 256, 1 << 30)), blk(256);
  if (mean && groups > 1 && (long long)groups * n >= AVERAGE_TWO_PASS_MIN) {
    const dim3 rgrid(grid_for((n / 8 + 3) / 4, 256, 1 << 30));
    hipLaunchKernelGGL(average_bf16_reduce_kernel<4>, rgrid, blk, 0, s, x, mean, groups, n);
    hipLaunchKernelGGL(average_bf16_spread_kernel, grid, blk, 0, s, mean, x, groups, n);
    return hipGetLastError();
  }
  hipLaunchKernelGGL(average_bf16_kernel, grid, blk, 0, s, x, groups, n);
  return hipGetLastError();
}

hipError_t launch_cross_worker(const float *g, int groups, long long Ppad, double *partials, double *out,
                               hipStream_t s) {
  const int nblocks = cross_worker_blocks(Ppad);
  hipLaunchKernelGGL(cross_worker_kernel, dim3(nblocks), dim3(256), 0, s, g, groups, Ppad, partials, nblocks);
  hipLaunchKernelGGL(cross_worker_final_kernel, dim3(1), dim3(256), 0, s, partials, nblocks, out);
  return hipGetLastError();
}

int cross_worker_blocks(long long Ppad) { return (int)((Ppad / 4 + 255) / 256); }

hipError_t launch_copy_probe(const void *src, void *dst, long long bytes, hipStream_t s) {
  const long long n16 = bytes / 16;
  if (n16 <= 0) return hipSuccess;
  hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)((n16 + 255) / 256)), dim3(256), 0, s,
                     static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n16);
  return hipGetLastError();
}

hipError_t launch_splitk_finish(const SplitKFinishMany &p, int groups, hipStream_t s) {
  if (p.n < 1 || p.n > SplitKFinishMany::MAXN) return hipErrorInvalidValue;
  long long mx = 0;
  for (int l = 0; l < p.n; ++l) {
    if ((p.mn[l] & 3) || (p.c_off[l] & 3) || p.ksplit[l] < 1 || !p.kpart[l]) return hipErrorInvalidValue;
    mx = p.mn[l] > mx ? p.mn[l] : mx;
  }
  const dim3 grid((unsigned)((mx / 4 + 255) / 256), groups, p.n), blk(256);
  if (!p.upd_x) {
    hipLaunchKernelGGL(splitk_finish_kernel<-1>, grid, blk, 0, s, p);
    return hipGetLastError();
  }
  if (p.accumulate || !p.upd_sq || (p.upd_opt != OPT_SGD && !p.upd_v) || (p.upd_opt == OPT_ADAMW && !p.upd_m))
    return hipErrorInvalidValue;
  if (p.upd_opt == OPT_SGD) hipLaunchKernelGGL(splitk_finish_kernel<OPT_SGD>, grid, blk, 0, s, p);
  else if (p.upd_opt == OPT_SHB) hipLaunchKernelGGL(splitk_finish_kernel<OPT_SHB>, grid, blk, 0, s, p);
  else if (p.upd_opt == OPT_ADAGRAD) hipLaunchKernelGGL(splitk_finish_kernel<OPT_ADAGRAD>, grid, blk, 0, s, p);
  else hipLaunchKernelGGL(splitk_finish_kernel<OPT_ADAMW>, grid, blk, 0, s, p);
  return hipGetLastError();
}

hipError_t launch_stage_step_inputs(const int32_t *idx_src, int32_t *idx_dst, long long n, float lr, float c1, float c2,
                                    float *scal, hipStream_t s) {
  hipLaunchKernelGGL(stage_step_inputs_kernel, dim3(grid_for(n, 256, 1024)), dim3(256), 0, s, idx_src, idx_dst, n, lr, c1,
                     c2, scal);
  return hipGetLastError();
}

hipError_t launch_set_ints(const int *v_host, int n, int *dst, hipStream_t s) {
  for (int o = 0; o < n; o += SET_INTS_MAX) {
    IntsArg a;
    const int m = n - o < SET_INTS_MAX ? n - o : SET_INTS_MAX;
    for (int i = 0; i < SET_INTS_MAX; ++i) a.v[i] = i < m ? v_host[o + i] : 0;
    hipLaunchKernelGGL(set_ints_kernel, dim3(1), dim3(SET_INTS_MAX), 0, s, a, m, dst + o);
  }
  return hipGetLastError();
}

// x[g * stride + i] = 0 for i in [from, to) and every group g (a short range: padding behind the data)
__global__ void __launch_bounds__(256) zero_range_kernel(float *__restrict__ x, long long stride, long long from, long long to) {
  float *p = x + (long long)blockIdx.x * stride;
  for (long long i = from + threadIdx.x; i < to; i += 256) p[i] = 0.0f;
}

hipError_t launch_zero_range(float *x, long long stride, long long from, long long to, int groups, hipStream_t s) {
  if (to <= from || groups <= 0) return hipSuccess;
  hipLaunchKernelGGL(zero_range_kernel, dim3(groups), dim3(256), 0, s, x, stride, from, to);
  return hipGetLastError();
}

hipError_t launch_fill_zero(void *p, long long bytes, hipStream_t s) {
  if (bytes <= 0) return hipSuccess;
  hipLaunchKernelGGL(fill_zero_kernel, dim3(grid_for(bytes / 16, 256, 4096)), dim3(256), 0, s,
                     static_cast<uint4 *>(p), bytes / 16);
  return hipGetLastError();
}

}  // namespace absk
