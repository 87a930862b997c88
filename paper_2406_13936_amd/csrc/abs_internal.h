// Internal declarations shared by the translation units of the library
// (host launchers only; kernels stay private to their .hip file).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace absk {

typedef uint16_t bf16_t;   // raw bfloat16 bits in memory

enum { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };
enum { OPT_SGD = 0, OPT_SHB = 1, OPT_ADAMW = 2, OPT_ADAGRAD = 3 };

// Epilogues of the grouped GEMM  C[g][m][n] = sum_k A[g][m][k] * B[g][n][k].
enum {
  EPI_FWD_ACT = 0,  // C = bf16/f32 phi(acc + bias[n]); C2 = phi'(acc + bias[n]) if C2 != null
  EPI_LOGITS = 1,   // C(f32) = acc + bias[n]
  EPI_BWD = 2,      // C = acc * E[m][n]   (act == RELU: E > 0 ? 1 : 0 ; GELU: E itself)
  EPI_WGRAD = 3,    // C(f32) = alpha * acc ; C2(bf16) = same, rounded, if C2 != null
  EPI_IPDOT = 4,    // part[tile_n][m] = sum_{n in tile} E[m][n] * (acc + bias[n])
  EPI_WGRAD_UPD = 5 // internal to the bf16 family: EPI_WGRAD with the optimizer step in the epilogue (GemmP::upd_x)
};

struct GemmP {
  const void *A, *B;           // operands (bf16 bits or float, by kernel family)
  long long sAg, sBg;          // group (replica) strides in elements
  int lda, ldb;                // leading dimensions in elements
  int a_trans, b_trans;        // 0: memory is [row][k] (k contiguous); 1: memory is [k][row]
  int Md, Nd, Kd, groups;
  void *C;  long long sCg;  int ldc;     // main output
  void *C2; long long sC2g; int ldc2;    // optional second output
  const float *bias; long long sBiasg;   // per-column vector (may be null)
  const void *E; long long sEg; int lde; // elementwise operand of the epilogue
  float *part; long long sPartg; long long sPartTile; // row partials: part[g][tile_n][m]
                               //   EPI_IPDOT: the row dots; EPI_FWD_ACT / EPI_BWD (bf16 family, optional):
                               //   sum over the tile's columns of the squared stored outputs
  float *cpart; long long sCpartg;   // EPI_BWD (bf16 family, optional): column partials
                               //   cpart[g][tile_m * WM + wave_m][n] = sum over the wave's rows of the stored outputs
  float alpha;
  int act;
  int pad_to_ld;               // also write zeros to columns [Nd, ldc) of C (and C2)
  // Ragged groups (optional): rows[g] (device) replaces Md (rows_is_k == 0) or Kd (rows_is_k == 1,
  // where alpha becomes 1 / rows[g]) for group g; Md / Kd then hold the largest count and size the
  // grid.  Memory beyond a group's own rows is neither read nor written.
  const int *rows;
  int rows_is_k;
  // Optional (device, bf16 family): the order in which the launch walks the groups.  Work-group ids are dealt
  // to the XCDs in contiguous ranges of groups, so with ragged groups the host orders them such that every
  // XCD gets about the same number of rows.
  const int *gperm;
  int accumulate;              // EPI_WGRAD: C = alpha * acc + C  (micro-batch accumulation)
  // Split reduction (EPI_WGRAD of the bf16 family, optional): ksplit > 1 cuts k into ksplit slices of
  // kchunk elements; slice sp of group g writes its raw partial product to
  // kpart[(g * ksplit + sp) * Md * Nd] (row-major, ld = Nd) and C / C2 are left to launch_splitk_finish.
  int ksplit, kchunk;
  float *kpart;
  // Optimizer step inside the epilogue (EPI_WGRAD of the bf16 family, optional: upd_x != null; needs ksplit <= 1,
  // accumulate == 0 and ldc, the layer offsets and the group stride multiples of 4).  The finished gradient entry
  // g = alpha * acc is not stored in C; instead the parameter at the same offset of upd_x (and its state in
  // upd_v / upd_m, its bf16 shadow in upd_shadow; all laid out like C: group stride sCg, leading dimension ldc)
  // takes its step.  C2 (the bf16 copy of the gradient) is still written.  Every wavefront leaves the sum of its
  // squared gradient entries in upd_sq[g * upd_sSqg + upd_slot0 + tile * waves + wave] (tile = tm * tilesN + tn):
  // the layer's share of ||gbar||^2, added up later in index order.
  float *upd_x, *upd_v, *upd_m;
  bf16_t *upd_shadow;
  int upd_opt;
  float upd_lr, upd_momentum, upd_beta1, upd_beta2, upd_eps, upd_wd, upd_c1, upd_c2;
  const float *upd_scal;       // optional (device): {lr, c1, c2} read from memory (replayable launches)
  float *upd_sq; long long upd_sSqg; int upd_slot0;
};

// bf16 MFMA family (gemm_bf16.hip).  Returns the number of column partials that
// EPI_IPDOT writes per row (tiles along n) for the tile shape it picks.
hipError_t launch_gemm_bf16(const GemmP &p, int epi, hipStream_t s);
int gemm_bf16_ipdot_parts(int Nd);
// Exact number of row partials (tiles along n) and of column-partial rows (tiles along m times
// wave rows) that the bf16 family writes for an Md x Nd output.
int gemm_bf16_row_parts(int Md, int Nd, int groups);
int gemm_bf16_col_parts(int Md, int Nd, int groups);
// Tile shape the bf16 family uses for an Md x Nd output over `groups` replicas: 0 = 128x64, 1 = 128x128, 2 = 256x256,
// 4 = 64x128 with a six-stage ring (outputs of at most 64 rows; 3 is a weight-gradient shape, see below).
int gemm_bf16_tile_shape(int Md, int Nd, int groups);
// Tile shape of an EPI_WGRAD launch whose reduction runs over Kd samples: as above, or 3 = 64x256 with a k-step of
// 32 and several work-groups per CU while the batch is short and the launch is bound by its epilogue's memory traffic;
// fused != 0: the launch carries the optimizer step in its epilogue (GemmP::upd_x), which keeps medium batches on
// 128x128 tiles.
int gemm_bf16_wgrad_shape(int Md, int Nd, int Kd, int groups, int fused);
// Number of upd_sq slots an EPI_WGRAD launch with an in-epilogue optimizer step writes per group.
int gemm_bf16_upd_slots(int Md, int Nd, int Kd, int groups);
// fp32 SIMT family (gemm_f32.hip); EPI_IPDOT is not offered (U is materialised instead).
hipError_t launch_gemm_f32(const GemmP &p, int epi, hipStream_t s);

// ---- gram_ip.hip -----------------------------------------------------------
// q[g][i] = (1 / b_g) sum_l sum_j (D_l D_l^T)[i][j] ((A_l A_l^T)[i][j] + [has_bias]),  i, j < b_g: the inner products
// <g_i, gbar> of a short batch from the Gram matrices of the layer inputs A_l = a^{l-1} and backprop signals
// D_l = delta^l (bf16, rows = samples, K[.] features at leading dimension ld[.], a multiple of 8).  Matrices come
// in pairs: X[2 l] = A_l, X[2 l + 1] = D_l.  part: scratch of gram_ip_scratch_floats(n, groups) floats.  The
// launcher fills in the slicing fields.  b <= GRAM_MAX_B.
enum { GRAM_MAX_B = 256, GRAM_SLICE_ELEMS = 2 * GRAM_MAX_B * GRAM_MAX_B };
struct GramP {
  enum { MAXL = 16 };
  int n;                                   // matrices (two per layer)
  const bf16_t *X[2 * MAXL];
  long long sXg[2 * MAXL];                 // group strides in elements
  int ld[2 * MAXL], K[2 * MAXL];
  int b, groups;
  const int *rows;                         // optional per-group sample counts (device) replacing b
  float *part;                             // [g][matrix][slice][bp][bp] partial Gram matrices
  int bp, S, kslice[2 * MAXL], nsl[2 * MAXL];   // set by the launcher: padded b, slices, features per slice, slices in use
};
long long gram_ip_scratch_floats(int n, int groups);
hipError_t launch_gram_ip(GramP p, int has_bias, float *q, long long sQg, hipStream_t s);

// ---- elementwise.hip -------------------------------------------------------
// T = activation element type: 0 float, 1 bf16
hipError_t launch_convert_f32_to_bf16(const float *src, bf16_t *dst, long long n, hipStream_t s);
// A0[g][i][:] = X[idx[g][i]][:]  and  an0[g][i] = ||row||^2
// Every launcher below takes `rows` (device, may be null): per-group row counts that replace b
// (then b is the largest count and sizes the grid).  `ldi` is the row stride of idx.
hipError_t launch_gather_rows(int is_bf16, const void *X, int d, int N, const int32_t *idx, int ldi, int groups,
                              int b, void *A0, long long sA0g, int ldo, float *an0, long long sNg,
                              const int *rows, hipStream_t s);
// softmax cross-entropy head: delta = p - e_y (stored in T, pad columns zeroed),
// dn[g][i] = ||stored delta_i||^2, loss[g][i] = f_i
hipError_t launch_softmax_ce(int is_bf16, const float *Z, long long sZg, int ldz, int K,
                             const int32_t *y, int N, const int32_t *idx, int ldi, int groups, int b,
                             void *D, long long sDg, int ldd, float *dn, float *loss,
                             long long sNg, const int *rows, hipStream_t s);
// out[g][i] = sum_j X[g][i][j]^2
hipError_t launch_row_sqnorm(int is_bf16, const void *X, long long sXg, int ld, int cols,
                             int groups, int b, float *out, long long sOg, const int *rows, hipStream_t s);
// out[g][j] = alpha * sum_i X[g][i][j]   (bias gradients); scratch: groups * ceil(b / COLSUM_ROWS)
// * cols floats of partial sums
enum { COLSUM_ROWS = 128 };
hipError_t launch_col_sum(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups,
                          int b, float alpha, float *out, long long sOg, float *scratch, const int *rows,
                          int accumulate, hipStream_t s);
// First stage of launch_col_sum alone (partials into scratch, nsplit = ceil(b / COLSUM_ROWS) rows per group).
hipError_t launch_col_sum_partials(int is_bf16, const void *X, long long sXg, int ld, int cols, int groups, int b,
                                   float *scratch, const int *rows, hipStream_t s);
// Second stage alone, for several layers in one launch (the bias gradients of a whole step):
// out[g][out_off_l + j] = alpha * sum_r part_l[g][r][j], r < nsplit_l (partials from a GEMM epilogue or from
// launch_col_sum_partials).  With rows: alpha = 1 / rows[g] and, where tile_m_l > 0, only the first
// ceil(rows[g] / tile_m_l) * parts_per_tile_l partials of group g exist.
struct ColFinishMany {
  enum { MAXN = 16 };
  int n;                         // layers
  const float *part[MAXN];       // partials [groups][nsplit][cols]
  int cols[MAXN], nsplit[MAXN], tile_m[MAXN], parts_per_tile[MAXN];
  long long out_off[MAXN];       // offset of the layer's sums inside a group's output vector
  float alpha;
  float *out; long long sOg;
  const int *rows;
  int accumulate;
};
hipError_t launch_col_sum_finish_many(const ColFinishMany &p, int groups, hipStream_t s);
// q[g][i] += sum_j D[g][i][j] * U[g][i][j]  (fp32 path of the inner products)
hipError_t launch_rowdot_f32(const float *D, long long sDg, int ldd, const float *U,
                             long long sUg, int ldu, int cols, int groups, int b, float *q,
                             long long sQg, int accumulate, const int *rows, hipStream_t s);

struct StatsP {
  int L, has_bias, groups, b, want_ip;
  const float *an[16];      // layer-input squared norms as an_parts[l] partial vectors:
  const float *dn[16];      //   an[l][g * an_sg[l] + part * sNg + i]; likewise the backprop-signal norms
  int an_parts[16], dn_parts[16];
  long long an_sg[16], dn_sg[16];
  long long sNg;
  const float *qpart[16];   // per layer: [g][part][i]
  int nparts[16];
  long long sQg[16], sQpart[16];
  const float *loss;        // [g][i]
  float *n_out, *q_out;     // [g][i] (stride sNg)
  const float *grad;        // [g][Ppad]
  long long Ppad;
  double *partials;         // scratch: [groups][5][PBLK]
  double *stats;            // out: [groups][8] = S1, S2, S3, S4, loss, 0,0,0
  double ticket;            // with stats_host: written to stats_host[g * 8 + 7] after group g's sums have been
                            //   made visible to the host (a host that polls that word needs no stream synchronisation)
  double *stats_host;       // optional mirror in device-visible pinned host memory (same layout): the host then
                            //   needs a stream synchronisation only, no copy
  const float *sq_wave;     // alternative source of S2 (grad must be null): per-wavefront sums of g^2 left by the
  long long n_sq_wave;      //   update kernel, n_sq_wave per group (one per 256 consecutive parameters)
  long long sq_stride;      //   distance between two groups' sums (0: n_sq_wave)
  const int *rows;          // optional per-group sample counts (device) replacing b
  // which sums this launch produces: S1 and the loss (do_n), S3 and S4 (do_q; needs want_ip),
  // S2 (grad != null); acc_n / acc_q add to the stored sums instead of replacing them
  int do_n, do_q, acc_n, acc_q;
};
enum { STATS_PBLK = 256 };
hipError_t launch_stats(const StatsP &p, hipStream_t s);

struct UpdateP {
  float *x; const float *g; float *v; float *m; bf16_t *shadow;
  long long n;              // total elements (groups * Ppad)
  float *sq_wave;           // optional: sq_wave[i / 256] = sum of g^2 over parameters [256 i', 256 i' + 256)
  int opt; float lr, momentum, beta1, beta2, eps, wd, c1, c2;  // c = 1/(1-beta^t)
  const float *scal;        // optional (device): {lr, c1, c2} read from memory instead of the fields above, so
                            //   that a captured launch can be replayed with new values
};
hipError_t launch_update(const UpdateP &p, hipStream_t s);
// The optimizer step of the bias vectors alone (layers l < n: width[l] entries at offset off[l] of every group's
// vector of `stride` elements), with per-block sums of their squared gradient entries into sq.
struct BiasUpdateP {
  enum { MAXN = 16 };
  int n;
  int width[MAXN];
  long long off[MAXN];
  long long stride;
  float *x; const float *g; float *v; float *m; bf16_t *shadow;
  int opt; float lr, momentum, beta1, beta2, eps, wd, c1, c2;
  const float *scal;
  float *sq; long long sSqg; int slot0;
};
int update_bias_slots(const BiasUpdateP &p);
hipError_t launch_update_bias(const BiasUpdateP &p, int groups, hipStream_t s);
hipError_t launch_average_f32(float *x, bf16_t *shadow, float *mean, int groups, long long Ppad, hipStream_t s);
hipError_t launch_average_bf16(bf16_t *x, bf16_t *mean, int groups, long long n, hipStream_t s);
// cross-worker statistics: out[0] = sum_m ||g^m||^2, out[1] = ||mean_m g^m||^2;
// partials: 2 * cross_worker_blocks(Ppad) doubles of scratch
int cross_worker_blocks(long long Ppad);
hipError_t launch_cross_worker(const float *g, int groups, long long Ppad, double *partials,
                               double *out, hipStream_t s);
hipError_t launch_fill_zero(void *p, long long bytes, hipStream_t s);
hipError_t launch_zero_range(float *x, long long stride, long long from, long long to, int groups, hipStream_t s);
// Finish of split reductions, the layers of a step in one launch: for layer l and group g
//   C[g][c_off_l + e] = alpha * sum_sp kpart_l[(g * ksplit_l + sp) * mn_l + e]  (+ the old value if accumulate),
// slices added in order; C2 (bf16, may be null) gets the rounded result at the same offsets; rows (may be null):
// alpha = 1 / rows[g].  mn_l and c_off_l are multiples of 4.
struct SplitKFinishMany {
  enum { MAXN = 16 };
  int n;
  const float *kpart[MAXN];
  int ksplit[MAXN];
  long long mn[MAXN], c_off[MAXN];
  float alpha;
  const int *rows;
  float *C; long long sCg;
  bf16_t *C2; long long sC2g;
  int accumulate;
  // Optional (upd_x != null, accumulate == 0): the optimizer step in place of the store to C, as in the
  // weight-gradient epilogue (GemmP::upd_*): parameters, state and shadow at upd_* + g * sCg + c_off_l + e; block j of
  // layer l leaves the sum of its squared gradient entries in upd_sq[g * upd_sSqg + upd_slot0[l] + j]
  // (launch_splitk_finish_slots(mn_l) blocks per layer).
  float *upd_x, *upd_v, *upd_m;
  bf16_t *upd_shadow;
  int upd_opt;
  float upd_lr, upd_momentum, upd_beta1, upd_beta2, upd_eps, upd_wd, upd_c1, upd_c2;
  const float *upd_scal;
  float *upd_sq; long long upd_sSqg; int upd_slot0[MAXN];
};
hipError_t launch_splitk_finish(const SplitKFinishMany &p, int groups, hipStream_t s);
inline int splitk_finish_slots(long long mn) { return (int)((mn / 4 + 255) / 256); }
// Inputs of a replayed step: idx_dst[0..n) = idx_src[0..n), scal[0..3) = {lr, c1, c2}
hipError_t launch_stage_step_inputs(const int32_t *idx_src, int32_t *idx_dst, long long n, float lr, float c1, float c2,
                                    float *scal, hipStream_t s);
// dst[0..n) = v[0..n): the values travel as kernel arguments, so the host array may be reused at once
enum { SET_INTS_MAX = 64 };
hipError_t launch_set_ints(const int *v_host, int n, int *dst, hipStream_t s);
// tile extent along m and column partials per tile of the bf16 family's tile shape `shape`
void gemm_bf16_col_part_shape(int shape, int *tile_m, int *parts_per_tile);
hipError_t launch_copy_probe(const void *src, void *dst, long long bytes, hipStream_t s);

}  // namespace absk
