// C ABI of the library (declared in include/abs.h): context, workspace plan, the call
// sequence of one local step, host-side tests and the batch-size rule.
#include <algorithm>
#include <atomic>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "../../include/abs.h"
#include "abs_internal.h"

using namespace absk;

namespace {

thread_local std::string g_err;

constexpr int MAXL = 16;
constexpr int GRAM_IP_DEFAULT_B = 256;   // largest local batch that takes the Gram form of the inner products by default

inline long long rup(long long v, long long a) { return (v + a - 1) / a * a; }

struct Plan {
  int L = 0;
  bool bf16 = false, gelu = false, want_ip = false;
  int esz = 4;                       // bytes per activation element
  std::vector<int> dims, ld;         // ld[l]: row stride of layer-l activations / signals
  std::vector<long long> offW, offB; // internal (padded) parameter offsets
  std::vector<long long> extW, extB; // packed external offsets
  long long P = 0, Ppad = 0;
  int M = 0, cap = 0;
  int qparts[MAXL] = {0};
  size_t colpart_per = 0;              // floats of column-partial scratch per replica (fp32 mode: one piece for all layers)
  size_t o_colpart_l[MAXL + 1] = {0};  // bf16 mode: one piece per layer, so that one launch can finish all bias gradients
  size_t colpart_l_per[MAXL + 1] = {0};
  int rparts[MAXL + 1] = {0};          // partial vectors kept for the row norms of width dims[l]
  // byte offsets into the workspace
  size_t o_xm = 0, o_xs = 0, o_grad = 0, o_gradbf = 0, o_v = 0, o_m = 0, o_Xbf = 0;
  size_t o_A[MAXL] = {0}, o_Dact[MAXL] = {0}, o_Dl[MAXL + 1] = {0};
  size_t o_Z = 0, o_U = 0, o_gram = 0, o_an[MAXL] = {0}, o_dn[MAXL + 1] = {0}, o_loss = 0, o_nout = 0, o_qout = 0;
  size_t o_qpart[MAXL] = {0}, o_partials = 0, o_stats = 0, o_cw = 0, o_colpart = 0, o_rows = 0, o_sqwave = 0, o_idx = 0, o_scal = 0, o_mean = 0;
  size_t o_kpart_l[MAXL + 1] = {0};    // per layer: partial products of a split weight-gradient reduction
  size_t kpart_floats_l[MAXL + 1] = {0};
  size_t total = 0;
};

abs_status fail(abs_status st, const std::string &msg) {
  g_err = msg;
  return st;
}

abs_status check_cfg(const abs_config *c) {
  if (!c || !c->dims) return fail(ABS_EINVAL, "config or dims is NULL");
  if (c->n_layers < 1 || c->n_layers > MAXL) return fail(ABS_EINVAL, "n_layers must be in [1,16]");
  for (int l = 0; l <= c->n_layers; ++l)
    if (c->dims[l] < 1) return fail(ABS_EINVAL, "layer width < 1");
  if (c->dims[c->n_layers] < 2) return fail(ABS_EINVAL, "need at least 2 classes");
  if (c->M < 1) return fail(ABS_EINVAL, "M < 1");
  if (c->b_cap < 2) return fail(ABS_EINVAL, "b_cap < 2");
  if (c->act < ABS_ACT_NONE || c->act > ABS_ACT_GELU) return fail(ABS_EINVAL, "unknown activation");
  if (c->opt < ABS_OPT_SGD || c->opt > ABS_OPT_ADAGRAD) return fail(ABS_EINVAL, "unknown optimizer");
  if (c->prec != ABS_PREC_F32 && c->prec != ABS_PREC_BF16) return fail(ABS_EINVAL, "unknown precision");
  if (!(c->stats_mask & ABS_STATS_NORM)) return fail(ABS_EINVAL, "stats_mask needs ABS_STATS_NORM");
  if (c->prec == ABS_PREC_BF16)
    for (int l = 0; l < c->n_layers; ++l)
      if (c->dims[l] % 8) return fail(ABS_EUNSUPPORTED, "bf16 mode needs dims[0..L-1] to be multiples of 8");
  if ((long long)c->M * c->b_cap > (1LL << 30)) return fail(ABS_EUNSUPPORTED, "M * b_cap too large");
  return ABS_OK;
}

void make_plan(const abs_config *c, long long N, Plan &pl) {
  pl.L = c->n_layers;
  pl.bf16 = c->prec == ABS_PREC_BF16;
  pl.gelu = c->act == ABS_ACT_GELU;
  pl.want_ip = (c->stats_mask & ABS_STATS_IP) != 0;
  pl.esz = pl.bf16 ? 2 : 4;
  pl.M = c->M;
  pl.cap = c->b_cap;
  pl.dims.assign(c->dims, c->dims + pl.L + 1);
  pl.ld.resize(pl.L + 1);
  for (int l = 0; l <= pl.L; ++l) pl.ld[l] = (int)rup(pl.dims[l], 8);
  pl.offW.assign(pl.L + 1, 0); pl.offB.assign(pl.L + 1, 0);
  pl.extW.assign(pl.L + 1, 0); pl.extB.assign(pl.L + 1, 0);
  long long o = 0, e = 0;
  for (int l = 1; l <= pl.L; ++l) {
    const long long w = (long long)pl.dims[l] * pl.dims[l - 1];
    pl.offW[l] = o; o = rup(o + w, 64);
    pl.extW[l] = e; e += w;
    if (c->has_bias) {
      pl.offB[l] = o; o = rup(o + pl.dims[l], 64);
      pl.extB[l] = e; e += pl.dims[l];
    }
  }
  pl.P = e;
  pl.Ppad = rup(o, 256);
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t r = off; off = (size_t)rup((long long)(off + bytes), 256); return r; };
  const size_t MP = (size_t)pl.M * pl.Ppad;
  pl.o_xm = take(MP * 4);
  if (pl.bf16) pl.o_xs = take(MP * 2);
  pl.o_grad = take(MP * 4);
  if (pl.bf16 && pl.want_ip) pl.o_gradbf = take(MP * 2);
  if (c->opt != ABS_OPT_SGD) pl.o_v = take(MP * 4);
  if (c->opt == ABS_OPT_ADAMW) pl.o_m = take(MP * 4);
  if (pl.bf16) pl.o_Xbf = take((size_t)N * pl.dims[0] * 2);
  const size_t MB = (size_t)pl.M * pl.cap;
  for (int l = 0; l < pl.L; ++l) pl.o_A[l] = take(MB * pl.ld[l] * pl.esz);
  if (pl.gelu)
    for (int l = 1; l < pl.L; ++l) pl.o_Dact[l] = take(MB * pl.ld[l] * pl.esz);
  for (int l = 1; l <= pl.L; ++l) pl.o_Dl[l] = take(MB * pl.ld[l] * pl.esz);
  pl.o_Z = take(MB * pl.ld[pl.L] * 4);
  if (!pl.bf16 && pl.want_ip) {
    int mx = 0;
    for (int l = 1; l <= pl.L; ++l) mx = pl.ld[l] > mx ? pl.ld[l] : mx;
    pl.o_U = take(MB * mx * 4);
  }
  for (int l = 0; l <= pl.L; ++l)
    pl.rparts[l] = (pl.bf16 && l >= 1 && l < pl.L) ? gemm_bf16_ipdot_parts(pl.dims[l]) : 1;
  for (int l = 0; l < pl.L; ++l) pl.o_an[l] = take(MB * 4 * pl.rparts[l]);
  for (int l = 1; l <= pl.L; ++l) pl.o_dn[l] = take(MB * 4 * pl.rparts[l]);
  pl.o_loss = take(MB * 4);
  pl.o_nout = take(MB * 4);
  pl.o_qout = take(MB * 4);
  if (pl.want_ip) {
    for (int l = 1; l <= pl.L; ++l) {
      pl.qparts[l - 1] = pl.bf16 ? gemm_bf16_ipdot_parts(pl.dims[l]) : (l == 1 ? 1 : 0);
      if (pl.qparts[l - 1]) pl.o_qpart[l - 1] = take(MB * 4 * pl.qparts[l - 1]);
    }
    // partial Gram matrices of the short-batch form of the inner products
    if (pl.bf16) pl.o_gram = take((size_t)gram_ip_scratch_floats(2 * pl.L, pl.M) * 4);
  }
  if (c->has_bias && !pl.bf16) {
    int mx = 0;
    for (int l = 1; l <= pl.L; ++l) mx = pl.dims[l] > mx ? pl.dims[l] : mx;
    pl.colpart_per = (size_t)((pl.cap + COLSUM_ROWS - 1) / COLSUM_ROWS) * mx;      // standalone column sums
    pl.o_colpart = take((size_t)pl.M * pl.colpart_per * 4);
  }
  if (c->has_bias && pl.bf16) {
    for (int l = 1; l <= pl.L; ++l) {
      // layers below L: partials from the backward epilogue, at most ceil(b / 128) * 4 rows for any tile shape the
      // GEMM may pick (128-row tiles of 4 wave rows; the other shapes write fewer); layer L: the standalone sums
      const size_t rows = l < pl.L ? (size_t)((pl.cap + 127) / 128 * 4) : (size_t)((pl.cap + COLSUM_ROWS - 1) / COLSUM_ROWS);
      pl.colpart_l_per[l] = rows * pl.dims[l];
      pl.o_colpart_l[l] = take((size_t)pl.M * pl.colpart_l_per[l] * 4);
    }
  }
  pl.o_partials = take((size_t)pl.M * 5 * STATS_PBLK * 8);
  pl.o_stats = take((size_t)pl.M * 8 * 8);
  pl.o_rows = take((size_t)2 * pl.M * sizeof(int));          // per-group row counts, then the launch order
  pl.o_sqwave = take((size_t)pl.M * (pl.Ppad / 256) * sizeof(float));
  for (int l = 1; l <= pl.L; ++l) {
    // one piece per layer, so that one launch can finish the split reductions of all layers.  bf16: a split is
    // only taken when the un-split launch has at most 256 tiles, and never makes more than 512 (tile, slice) pairs
    // of at most 128 x 128 or 256 x 256 outputs each; fp32: at most 8 slices of launches of fewer than 256 tiles
    // of 64 x 64
    const size_t full = (size_t)8 * pl.M * pl.dims[l] * pl.dims[l - 1];
    pl.kpart_floats_l[l] = std::min(full, pl.bf16 ? (size_t)512 * 65536 : (size_t)8 * 256 * 4096);
    pl.o_kpart_l[l] = take(pl.kpart_floats_l[l] * sizeof(float));
  }
  pl.o_cw = take((2 * (size_t)cross_worker_blocks(pl.Ppad) + 8) * 8);
  pl.o_idx = take((size_t)pl.M * pl.cap * sizeof(int32_t));      // inputs of replayed (graph) steps
  pl.o_scal = take(256);
  pl.o_mean = take((size_t)pl.Ppad * sizeof(float));          // the mean between the two passes of a large average
  pl.total = off;
}

// Number of slices for the reduction of a weight-gradient launch with `tiles` output tiles of shape `shape`
// and `KT` k-tiles of 64, from a small cost model in microseconds fitted to measured launches (256..1024-wide
// layers, b = 256..4096): a 128-wide tile takes 0.9 us per k-tile alone on a CU and 1.1 us when two work-groups
// share it (launches of more than 256 blocks), a 256 x 256 tile 2.0 us; the partial products are written and
// read once (8 bytes per slice and output at about 4.5 TB/s) and the finishing launch costs 10 us inside a
// step (a dependent launch more on the stream).  The split
// pays for few tiles and long reductions only: at b <= 1024 the un-split launch wins for every layer measured.
int choose_ksplit(int shape, long long tiles, int KT, double outputs, size_t kpart_floats) {
  if (tiles < 1 || tiles > 256) return 1;
  int best = 1;
  double best_cost = 0.0;
  for (int S = 1; S <= 8; ++S) {
    if (S > 1 && ((double)S * outputs > (double)kpart_floats || (KT + S - 1) / S < 4)) break;
    const long long blocks = tiles * S;
    const int kt = (KT + S - 1) / S;
    double cost;
    if (shape == 2) cost = (double)((blocks + 255) / 256) * kt * 2.0;
    else if (blocks <= 256) cost = kt * 0.9;
    else cost = (double)((blocks + 511) / 512) * kt * 1.1;
    if (S > 1) cost += 10.0 + (double)S * outputs * 8.0 / 4.5e6;
    if (S == 1 || cost < best_cost) { best = S; best_cost = cost; }
  }
  return best;
}

}  // namespace

// Event-timed launch classes (abs_profile_*): one entry per kernel symbol of interest.
enum {
  T_GATHER = 0, T_SOFTMAX, T_ROWNORM, T_COLSUM, T_STATS, T_UPDATE, T_AVERAGE, T_ROWDOT, T_GRAM,
  T_GEMM0,                       // + epi * 5 + tile shape (bf16) ; fp32 family uses shape 1
  T_GEMM_KINDS = 5 * 5, T_LAYERS = 17,   // GEMM classes are resolved per layer
  T_COUNT = T_GEMM0 + T_GEMM_KINDS * T_LAYERS
};
static const char *const kTagNames[T_GEMM0 + T_GEMM_KINDS] = {
  "gather_rows", "softmax_ce", "row_sqnorm", "col_sum", "stats", "update", "average", "rowdot", "gram_ip",
  "gemm_fwd_128x64", "gemm_fwd_128x128", "gemm_fwd_256x256", "gemm_fwd_64x256", "gemm_fwd_64x128",
  "gemm_logits_128x64", "gemm_logits_128x128", "gemm_logits_256x256", "gemm_logits_64x256", "gemm_logits_64x128",
  "gemm_bwd_128x64", "gemm_bwd_128x128", "gemm_bwd_256x256", "gemm_bwd_64x256", "gemm_bwd_64x128",
  "gemm_wgrad_128x64", "gemm_wgrad_128x128", "gemm_wgrad_256x256", "gemm_wgrad_64x256", "gemm_wgrad_64x128",
  "gemm_ipdot_128x64", "gemm_ipdot_128x128", "gemm_ipdot_256x256", "gemm_ipdot_64x256", "gemm_ipdot_64x128"};

struct ProfRec { int tag; hipEvent_t e0, e1; double flops, bytes; };

struct abs_ctx {
  bool prof_on = false;            // launches are being bracketed right now
  bool prof_enabled = false;       // abs_profile_enable(1) is in force (abs_profile_pause toggles prof_on under it)
  std::vector<ProfRec> prof_recs;      // event pool, reused
  size_t prof_used = 0;
  double prof_ms[T_COUNT] = {0}, prof_flops[T_COUNT] = {0}, prof_bytes[T_COUNT] = {0};
  long long prof_calls[T_COUNT] = {0};
  Plan pl;
  abs_config cfg;
  hipStream_t stream = nullptr;
  unsigned char *ws = nullptr;
  const float *X = nullptr;
  const int32_t *y = nullptr;
  long long N = 0;
  double *host_stats = nullptr;     // pinned, M*8 + 8 doubles
  double *host_stats_dev = nullptr; // the same memory as the device sees it (the statistics kernel writes there)
  double ticket = 0.0;              // number of the last statistics launch that mirrors its sums (exact in a double)
  bool ticket_live = false;         // that launch carried the ticket as a kernel argument (not a replayed graph)
  long long t = 0;                  // local steps taken (Adam bias correction)
  long long n_rounds = 0;           // Alg. 1's k: communication rounds completed (model averages)
  long long n_samples = 0;          // Alg. 1's B: samples processed, summed over workers and local steps
  int last_b = 0;                 // largest local batch size of the last step
  std::vector<int> last_bm;       // per worker
  int last_ps = -1;               // per-sample outputs stored (accumulated steps; -1: all of them)
  bool last_ragged = false;
  bool have_stats = false;
  int gram_ip_max_b = GRAM_IP_DEFAULT_B;   // abs_set_gram_ip_max_batch: batches up to this size take the Gram form of <g_i, gbar>
  bool fused_update = true;       // abs_set_fused_update: apply the optimizer step inside the weight-gradient epilogue (bf16 mode)
  bool last_fused = false;        // the last step did so: the fp32 gradient of its weights is not stored (materialize_grad)
  // captured steps (abs_local_step_graphed): one executable graph per batch size, a few kept
  struct GraphSlot { int b; hipGraphExec_t exec; long long last_use; bool fused; };   // fused: the captured step took its update in the weight-gradient epilogue
  std::vector<GraphSlot> graphs;
  std::vector<int> graph_warm;      // batch sizes that ran once eagerly (kernel attributes are set)
  std::string err;

  template <class T> T *at(size_t off) const { return reinterpret_cast<T *>(ws + off); }

  abs_ctx() = default;
  abs_ctx(const abs_ctx &) = delete;
  abs_ctx &operator=(const abs_ctx &) = delete;
  ~abs_ctx() {                      // the library owns the pinned mirror, the event pool and the graphs
    if (host_stats) (void)hipHostFree(host_stats);
    for (ProfRec &r : prof_recs) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
    for (auto &g : graphs) (void)hipGraphExecDestroy(g.exec);
  }
};

namespace {

abs_status cfail(abs_ctx *c, abs_status st, const std::string &msg) {
  if (c) c->err = msg;
  g_err = msg;
  return st;
}

#define HIPCHK(ctx, call)                                                                       \
  do {                                                                                          \
    hipError_t e_ = (call);                                                                     \
    if (e_ != hipSuccess)                                                                       \
      return cfail(ctx, ABS_EHIP, std::string(#call) + ": " + hipGetErrorString(e_));           \
  } while (0)

// external packed vector <-> internal padded layout
void to_internal(const Plan &pl, bool has_bias, const float *ext, float *in /*Ppad, zeroed*/) {
  for (int l = 1; l <= pl.L; ++l) {
    const long long w = (long long)pl.dims[l] * pl.dims[l - 1];
    std::memcpy(in + pl.offW[l], ext + pl.extW[l], w * sizeof(float));
    if (has_bias) std::memcpy(in + pl.offB[l], ext + pl.extB[l], pl.dims[l] * sizeof(float));
  }
}
void to_external(const Plan &pl, bool has_bias, const float *in, float *ext) {
  for (int l = 1; l <= pl.L; ++l) {
    const long long w = (long long)pl.dims[l] * pl.dims[l - 1];
    std::memcpy(ext + pl.extW[l], in + pl.offW[l], w * sizeof(float));
    if (has_bias) std::memcpy(ext + pl.extB[l], in + pl.offB[l], pl.dims[l] * sizeof(float));
  }
}

// Optional event bracket around one launch (profiling on: two hipEventRecord calls).
struct ProfScope {
  abs_ctx *c; ProfRec *r = nullptr;
  ProfScope(abs_ctx *ctx, int tag, double flops, double bytes) : c(ctx) {
    if (!c->prof_on) return;
    if (c->prof_used == c->prof_recs.size()) {
      ProfRec n{};
      if (hipEventCreate(&n.e0) != hipSuccess) return;
      if (hipEventCreate(&n.e1) != hipSuccess) { (void)hipEventDestroy(n.e0); return; }
      c->prof_recs.push_back(n);
    }
    r = &c->prof_recs[c->prof_used++];
    r->tag = tag; r->flops = flops; r->bytes = bytes;
    (void)hipEventRecord(r->e0, c->stream);
  }
  ~ProfScope() { if (r) (void)hipEventRecord(r->e1, c->stream); }
};

hipError_t gemm(abs_ctx *c, const GemmP &p, int epi, int layer) {
  int shape = !c->pl.bf16 ? 1 : (epi == EPI_WGRAD ? gemm_bf16_wgrad_shape(p.Md, p.Nd, p.Kd, p.groups, p.upd_x != nullptr)
                                                   : gemm_bf16_tile_shape(p.Md, p.Nd, p.groups));
  // algorithmic bytes of the launch: both operands once, the outputs once, the epilogue's elementwise operand once
  const double e = c->pl.esz, mn = (double)p.Md * p.Nd;
  double bytes = ((double)p.Md + p.Nd) * p.Kd * e;
  if (epi == EPI_FWD_ACT) bytes += mn * e * (p.C2 ? 2 : 1);
  else if (epi == EPI_LOGITS) bytes += mn * 4;
  else if (epi == EPI_BWD) bytes += mn * e * (p.act != ABS_ACT_NONE ? 2 : 1);
  else if (epi == EPI_IPDOT) bytes += mn * e;
  else if (p.upd_x) bytes += mn * (8 + (p.upd_v ? 8 : 0) + (p.upd_m ? 8 : 0) + (p.upd_shadow ? 2 : 0) + (p.C2 ? 2 : 0));
  else bytes += mn * (4 + (p.C2 ? 2 : 0) + (p.accumulate ? 4 : 0));
  ProfScope ps(c, T_GEMM0 + (epi * 5 + shape) * T_LAYERS + layer, 2.0 * p.Md * p.Nd * p.Kd * p.groups, bytes * p.groups);
  return c->pl.bf16 ? launch_gemm_bf16(p, epi, c->stream) : launch_gemm_f32(p, epi, c->stream);
}

void fill_result(abs_test_result &r, int b, const double *st) {
  std::memset(&r, 0, sizeof(r));
  r.b = b;
  r.sum_sq = st[0];
  r.gbar_sq = st[1];
  r.sum_q2 = st[2];
  r.sum_q = st[3];
  r.loss_sum = st[4];
}

// ratio and its ceiling; a zero batch gradient leaves the batch size unchanged
void ceil_ratio(double num, double den, int b, double &ratio, long long &T) {
  if (!(den > 0.0)) { ratio = (double)b; T = b; return; }
  ratio = num / den;
  const double c = std::ceil(ratio);
  T = c > 9.0e18 ? (long long)9e18 : (c < -9.0e18 ? (long long)-9e18 : (long long)c);
}

abs_status read_stats(abs_ctx *c) {
  if (!c->have_stats) return cfail(c, ABS_ESTATE, "no local step has been taken yet");
  if (!c->host_stats_dev)
    HIPCHK(c, hipMemcpyAsync(c->host_stats, c->at<double>(c->pl.o_stats), (size_t)c->pl.M * 8 * sizeof(double),
                             hipMemcpyDeviceToHost, c->stream));
  if (c->host_stats_dev && c->ticket_live) {
    // The final statistics kernel writes its launch number behind each worker's sums in the pinned mirror: poll
    // for it (a stream synchronisation costs tens of microseconds of wake-up latency, which is a third of a step of
    // the small configurations).  Bounded: after 20 ms the stream synchronisation below takes over.
    const volatile double *h = c->host_stats;
    const auto t0 = std::chrono::steady_clock::now();
    for (unsigned spin = 0;; ++spin) {
      bool done = true;
      for (int m = 0; m < c->pl.M && done; ++m) done = h[m * 8 + 7] == c->ticket;
      if (done) { std::atomic_thread_fence(std::memory_order_acquire); return ABS_OK; }
      if ((spin & 63) == 63 && std::chrono::steady_clock::now() - t0 > std::chrono::milliseconds(20)) break;
      __builtin_ia32_pause();
    }
  }
  HIPCHK(c, hipStreamSynchronize(c->stream));      // the statistics kernel has written the pinned mirror itself
  return ABS_OK;
}

// No exception leaves the library: host allocations (vectors, strings) are the only throwing operations.
abs_status on_exception() noexcept {
  try { throw; }
  catch (const std::bad_alloc &) {
    try { g_err = "out of host memory"; } catch (...) {}
    return ABS_ENOMEM;
  }
  catch (...) {
    try { g_err = "internal error"; } catch (...) {}
    return ABS_EHIP;
  }
}

}  // namespace

extern "C" {

const char *abs_last_error(const abs_ctx *ctx) { return ctx ? ctx->err.c_str() : g_err.c_str(); }

abs_status abs_lr_linear_scaling(double lr_ref, int64_t b, int64_t b_ref, double *lr) try {
  if (!lr) return fail(ABS_EINVAL, "lr is NULL");
  if (b < 1 || b_ref < 1) return fail(ABS_EINVAL, "batch sizes must be positive");
  *lr = lr_ref * (double)b / (double)b_ref;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_lr_schedule(long long step, long long total_steps, long long warmup_steps, double peak, double floor,
                           double *lr) try {
  if (!lr) return fail(ABS_EINVAL, "lr is NULL");
  if (step < 0 || total_steps < 1 || warmup_steps < 0 || warmup_steps > total_steps)
    return fail(ABS_EINVAL, "need 0 <= step, 0 <= warmup_steps <= total_steps, total_steps >= 1");
  const double kPi = 3.14159265358979323846;
  if (step < warmup_steps) *lr = peak * (double)(step + 1) / (double)warmup_steps;
  else if (step >= total_steps) *lr = floor;
  else {
    const long long span = total_steps - warmup_steps > 1 ? total_steps - warmup_steps : 1;
    *lr = floor + 0.5 * (peak - floor) * (1.0 + std::cos(kPi * (double)(step - warmup_steps) / (double)span));
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_n_params(const abs_config *cfg, int64_t *n) try {
  if (!n) return fail(ABS_EINVAL, "n is NULL");
  abs_status st = check_cfg(cfg);
  if (st != ABS_OK) return st;
  Plan pl;
  make_plan(cfg, 0, pl);
  *n = pl.P;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_workspace_bytes(const abs_config *cfg, int64_t N, size_t *bytes) try {
  if (!bytes) return fail(ABS_EINVAL, "bytes is NULL");
  if (N < 1) return fail(ABS_EINVAL, "N < 1");
  abs_status st = check_cfg(cfg);
  if (st != ABS_OK) return st;
  Plan pl;
  make_plan(cfg, N, pl);
  *bytes = pl.total;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_init_replicas(const abs_config *cfg, const float *x0_host, const float *X_dev,
                             const int32_t *y_dev, int64_t N, abs_ctx **out) try {
  if (!out || !x0_host || !X_dev || !y_dev) return fail(ABS_EINVAL, "NULL argument");
  if (N < 1 || N > 0x7fffffffLL) return fail(ABS_EINVAL, "N out of range");
  abs_status st = check_cfg(cfg);
  if (st != ABS_OK) return st;
  if (!cfg->workspace || (reinterpret_cast<uintptr_t>(cfg->workspace) & 255))
    return fail(ABS_EINVAL, "workspace must be a 256-byte aligned device pointer");
  if ((reinterpret_cast<uintptr_t>(X_dev) & 15)) return fail(ABS_EINVAL, "X_dev must be 16-byte aligned");
  std::unique_ptr<abs_ctx> owner(new (std::nothrow) abs_ctx());
  abs_ctx *c = owner.get();
  if (!c) return fail(ABS_ENOMEM, "host allocation failed");
  make_plan(cfg, N, c->pl);
  if (cfg->workspace_bytes < c->pl.total) return fail(ABS_ENOMEM, "workspace too small (see abs_workspace_bytes)");
  c->cfg = *cfg;
  c->cfg.dims = c->pl.dims.data();
  c->stream = static_cast<hipStream_t>(cfg->hip_stream);
  c->ws = static_cast<unsigned char *>(cfg->workspace);
  c->X = X_dev; c->y = y_dev; c->N = N;
  const Plan &pl = c->pl;
  auto bail = [&](const std::string &m) { g_err = m; return ABS_EHIP; };      // `owner` frees what was acquired
  hipError_t e = hipHostMalloc(reinterpret_cast<void **>(&c->host_stats), ((size_t)pl.M * 8 + 8) * sizeof(double), hipHostMallocMapped);
  if (e != hipSuccess) { c->host_stats = nullptr; return bail(std::string("hipHostMalloc: ") + hipGetErrorString(e)); }
  std::memset(c->host_stats, 0, ((size_t)pl.M * 8 + 8) * sizeof(double));
  void *hs_dev = nullptr;
  if (hipHostGetDevicePointer(&hs_dev, c->host_stats, 0) == hipSuccess) c->host_stats_dev = static_cast<double *>(hs_dev);
  else (void)hipGetLastError();                   // no mapping: read_stats copies instead
  // zero parameters, gradient and optimizer state (including their padding)
  const size_t MP = (size_t)pl.M * pl.Ppad;
  if ((e = launch_fill_zero(c->at<void>(pl.o_xm), MP * 4, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  if ((e = launch_fill_zero(c->at<void>(pl.o_grad), MP * 4, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  if (pl.bf16 && pl.want_ip)
    if ((e = launch_fill_zero(c->at<void>(pl.o_gradbf), MP * 2, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  if (cfg->opt != ABS_OPT_SGD)
    if ((e = launch_fill_zero(c->at<void>(pl.o_v), MP * 4, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  if (cfg->opt == ABS_OPT_ADAMW)
    if ((e = launch_fill_zero(c->at<void>(pl.o_m), MP * 4, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  std::vector<float> in(pl.Ppad, 0.0f);
  to_internal(pl, cfg->has_bias != 0, x0_host, in.data());
  for (int m = 0; m < pl.M; ++m)
    if ((e = hipMemcpy(c->at<float>(pl.o_xm) + (size_t)m * pl.Ppad, in.data(), pl.Ppad * sizeof(float), hipMemcpyHostToDevice)) != hipSuccess)
      return bail(std::string("hipMemcpy x0: ") + hipGetErrorString(e));
  if (pl.bf16) {
    if ((e = launch_convert_f32_to_bf16(c->at<float>(pl.o_xm), c->at<bf16_t>(pl.o_xs), (long long)MP, c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
    if ((e = launch_convert_f32_to_bf16(X_dev, c->at<bf16_t>(pl.o_Xbf), (long long)N * pl.dims[0], c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  }
  if ((e = hipStreamSynchronize(c->stream)) != hipSuccess) return bail(hipGetErrorString(e));
  *out = owner.release();
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_destroy(abs_ctx *c) try {
  if (!c) return ABS_OK;
  (void)hipStreamSynchronize(c->stream);
  delete c;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_profile_enable(abs_ctx *c, int on) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  c->prof_on = c->prof_enabled = on != 0;
  c->prof_used = 0;
  for (int t = 0; t < T_COUNT; ++t) { c->prof_ms[t] = c->prof_flops[t] = c->prof_bytes[t] = 0.0; c->prof_calls[t] = 0; }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_profile_pause(abs_ctx *c, int paused) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  c->prof_on = c->prof_enabled && paused == 0;   // no synchronisation, totals and pending records are kept
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_profile_read(abs_ctx *c, int max_entries, abs_profile_entry *out, int *n_entries) try {
  if (!c || !out || !n_entries) return fail(ABS_EINVAL, "NULL argument");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  for (size_t i = 0; i < c->prof_used; ++i) {
    ProfRec &r = c->prof_recs[i];
    float ms = 0.0f;
    HIPCHK(c, hipEventElapsedTime(&ms, r.e0, r.e1));
    c->prof_ms[r.tag] += ms; c->prof_flops[r.tag] += r.flops; c->prof_bytes[r.tag] += r.bytes;
    c->prof_calls[r.tag] += 1;
  }
  c->prof_used = 0;
  int n = 0;
  for (int t = 0; t < T_COUNT && n < max_entries; ++t) {
    if (!c->prof_calls[t]) continue;
    abs_profile_entry e;
    std::memset(&e, 0, sizeof(e));
    if (t < T_GEMM0) std::strncpy(e.name, kTagNames[t], sizeof(e.name) - 1);
    else std::snprintf(e.name, sizeof(e.name), "%s_L%d", kTagNames[T_GEMM0 + (t - T_GEMM0) / T_LAYERS], (t - T_GEMM0) % T_LAYERS);
    e.calls = c->prof_calls[t]; e.total_ms = c->prof_ms[t]; e.flops = c->prof_flops[t]; e.bytes = c->prof_bytes[t];
    out[n++] = e;
  }
  *n_entries = n;
  return ABS_OK;
} catch (...) { return on_exception(); }

// One local step.  b is the largest local batch size; with b_host (M entries, each in [2, b]) the
// workers' batches are ragged: worker m uses the first b_host[m] entries of row m of idx (row
// stride ldi) and every kernel takes its group's own row count from the device copy `rows`.
// Host-side record of the step just enqueued (what the tests and getters refer to).
static void note_step(abs_ctx *c, int b, const int *b_host) {
  c->last_b = b;
  c->last_bm.assign(c->pl.M, b);
  if (b_host) c->last_bm.assign(b_host, b_host + c->pl.M);
  c->last_ragged = b_host != nullptr;
  c->last_ps = -1;
  c->have_stats = true;
  for (int m = 0; m < c->pl.M; ++m) c->n_samples += c->last_bm[m];      // Alg. 1: B <- B + sum_m b^m
}

// Which parts of the step one call of local_step_impl runs.  A plain step runs all of them once;
// a step accumulated over micro-batches runs the passes once per micro-batch for the gradient,
// S1 and the loss, and (for the inner products, which need the batch gradient of the whole batch)
// a second time per micro-batch, before the single update.
struct StepPhase {
  bool passes = true;    // gather, forward, loss head, backward-data
  bool wgrad = true;     // batch gradient
  bool nstats = true;    // S1 and the loss sum
  bool s2 = true;        // ||gbar||^2
  bool ip = true;        // inner products, S3, S4 (when the statistics mask asks for them)
  bool update = true;
  bool acc_grad = false, acc_n = false, acc_q = false;   // add to what earlier micro-batches left
  int b_total = 0;       // divisor of the batch gradient (0: this call's b)
  float c1 = 1.0f, c2 = 1.0f;   // Adam bias corrections 1 / (1 - beta^t) of this step (set by the caller)
  const float *scal = nullptr;  // device {lr, c1, c2} for replayable launches (then lr / c1 / c2 here are unused)
  long long ps_off = 0;  // offset of this call's samples in the per-sample outputs (-1: not stored)
  bool whole_launches = false;  // take the split decisions of a step with the update in the epilogue (materialize_grad)
};

static abs_status local_step_impl(abs_ctx *c, const int32_t *idx_dev, int ldi, int b, const int *b_host, float lr,
                                  const StepPhase &ph = StepPhase()) {
  const Plan &pl = c->pl;
  const int L = pl.L, M = pl.M, isb = pl.bf16 ? 1 : 0;
  const int *rows = nullptr, *gperm = nullptr;
  if (b_host) {
    // row counts, and an order of the groups in which each of the 8 XCDs (which take contiguous ranges of
    // that order) gets about the same number of rows: sort by size, deal in snake order
    std::vector<int> both(2 * (size_t)M);
    std::copy(b_host, b_host + M, both.begin());
    std::vector<int> order(M);
    for (int m = 0; m < M; ++m) order[m] = m;
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return b_host[x] > b_host[y]; });
    std::vector<std::vector<int>> deal(8);
    for (int i = 0; i < M; ++i) {
      const int r = i / 8, j = i % 8;
      deal[(r & 1) ? 7 - j : j].push_back(order[i]);
    }
    int pos = 0;
    for (int x = 0; x < 8; ++x) for (int gidx : deal[x]) both[M + pos++] = gidx;
    int *rows_dev = c->at<int>(pl.o_rows);
    HIPCHK(c, launch_set_ints(both.data(), 2 * M, rows_dev, c->stream));
    rows = rows_dev;
    if (M >= 8) gperm = rows_dev + M;
  }
  int an_parts[MAXL + 1], dn_parts[MAXL + 2];
  for (int l = 0; l <= MAXL; ++l) an_parts[l] = dn_parts[l] = 1;
  dn_parts[MAXL + 1] = 1;
  const long long cap = pl.cap;
  hipStream_t s = c->stream;
  const bool hb = c->cfg.has_bias != 0;
  float *xm = c->at<float>(pl.o_xm);
  float *grad = c->at<float>(pl.o_grad);
  const void *wts = pl.bf16 ? static_cast<const void *>(c->at<bf16_t>(pl.o_xs)) : static_cast<const void *>(xm);
  auto wptr = [&](int l) -> const void * {
    return static_cast<const unsigned char *>(wts) + (size_t)pl.offW[l] * pl.esz;
  };
  auto act_ptr = [&](size_t off) -> void * { return c->ws + off; };

  const bool want_parts = ph.nstats;      // row-norm partials feed S1 only
  ColFinishMany cf;                       // bias-gradient partials of the layers, finished together (bf16 mode)
  std::memset(&cf, 0, sizeof(cf));
  double cf_bytes = 0.0;
  SplitKFinishMany kf;                    // split weight-gradient reductions, finished together
  std::memset(&kf, 0, sizeof(kf));
  double kf_bytes = 0.0;
  const float inv_b = 1.0f / (float)(ph.b_total > 0 ? ph.b_total : b);
  if (ph.passes) {
    // batch gather (Alg. 1: "sample the local batch")
    const void *Xsrc = pl.bf16 ? static_cast<const void *>(c->at<bf16_t>(pl.o_Xbf)) : static_cast<const void *>(c->X);
    { ProfScope ps_(c, T_GATHER, 0.0, 2.0 * M * b * pl.dims[0] * pl.esz);
    HIPCHK(c, launch_gather_rows(isb, Xsrc, pl.dims[0], (int)c->N, idx_dev, ldi, M, b, act_ptr(pl.o_A[0]), cap * pl.ld[0],
                                 pl.ld[0], c->at<float>(pl.o_an[0]), cap, rows, s)); }

    // forward
    for (int l = 1; l <= L; ++l) {
      GemmP p;
      std::memset(&p, 0, sizeof(p));
      p.A = act_ptr(pl.o_A[l - 1]); p.sAg = cap * pl.ld[l - 1]; p.lda = pl.ld[l - 1];
      p.B = wptr(l); p.sBg = pl.Ppad; p.ldb = pl.dims[l - 1];
      p.Md = b; p.Nd = pl.dims[l]; p.Kd = pl.dims[l - 1]; p.groups = M; p.rows = rows; p.gperm = gperm;
      if (hb) { p.bias = xm + pl.offB[l]; p.sBiasg = pl.Ppad; }
      p.act = c->cfg.act;
      if (l < L) {
        p.C = act_ptr(pl.o_A[l]); p.sCg = cap * pl.ld[l]; p.ldc = pl.ld[l]; p.pad_to_ld = 1;
        if (pl.gelu) { p.C2 = act_ptr(pl.o_Dact[l]); p.sC2g = cap * pl.ld[l]; p.ldc2 = pl.ld[l]; }
        if (pl.bf16) {
          // ||a_i^l||^2 as per-tile partials out of the GEMM epilogue (summed by the statistics kernel)
          an_parts[l] = gemm_bf16_row_parts(b, pl.dims[l], M);
          if (an_parts[l] > pl.rparts[l]) return cfail(c, ABS_ENOMEM, "row-partial scratch too small for this tile shape");
          if (want_parts) { p.part = c->at<float>(pl.o_an[l]); p.sPartg = cap * pl.rparts[l]; p.sPartTile = cap; }
          HIPCHK(c, gemm(c, p, EPI_FWD_ACT, l));
        } else {
          HIPCHK(c, gemm(c, p, EPI_FWD_ACT, l));
          if (!want_parts) continue;
          ProfScope ps_(c, T_ROWNORM, 0.0, 1.0 * M * b * pl.ld[l] * pl.esz);
          HIPCHK(c, launch_row_sqnorm(isb, p.C, p.sCg, pl.ld[l], pl.ld[l], M, b, c->at<float>(pl.o_an[l]), cap, rows, s));
        }
      } else {
        p.C = c->at<float>(pl.o_Z); p.sCg = cap * pl.ld[L]; p.ldc = pl.ld[L];
        HIPCHK(c, gemm(c, p, EPI_LOGITS, l));
      }
    }
    // loss head: per-sample backprop signal of the last layer
    { ProfScope ps_(c, T_SOFTMAX, 0.0, 1.0 * M * b * pl.ld[L] * (4 + pl.esz));
    HIPCHK(c, launch_softmax_ce(isb, c->at<float>(pl.o_Z), cap * pl.ld[L], pl.ld[L], pl.dims[L], c->y, (int)c->N, idx_dev, ldi, M, b,
                                act_ptr(pl.o_Dl[L]), cap * pl.ld[L], pl.ld[L], c->at<float>(pl.o_dn[L]),
                                c->at<float>(pl.o_loss), cap, rows, s)); }
    // backward-data
    for (int l = L; l >= 2; --l) {
      GemmP p;
      std::memset(&p, 0, sizeof(p));
      p.A = act_ptr(pl.o_Dl[l]); p.sAg = cap * pl.ld[l]; p.lda = pl.ld[l];
      p.B = wptr(l); p.sBg = pl.Ppad; p.ldb = pl.dims[l - 1]; p.b_trans = 1;
      p.Md = b; p.Nd = pl.dims[l - 1]; p.Kd = pl.dims[l]; p.groups = M; p.rows = rows; p.gperm = gperm;
      p.C = act_ptr(pl.o_Dl[l - 1]); p.sCg = cap * pl.ld[l - 1]; p.ldc = pl.ld[l - 1]; p.pad_to_ld = 1;
      p.act = c->cfg.act;
      p.E = pl.gelu ? act_ptr(pl.o_Dact[l - 1]) : act_ptr(pl.o_A[l - 1]);
      p.sEg = cap * pl.ld[l - 1]; p.lde = pl.ld[l - 1];
      if (pl.bf16) {
        // ||delta_i^{l-1}||^2 and (with biases) the column sums of delta^{l-1} as epilogue partials
        dn_parts[l - 1] = gemm_bf16_row_parts(b, pl.dims[l - 1], M);
        if (dn_parts[l - 1] > pl.rparts[l - 1]) return cfail(c, ABS_ENOMEM, "row-partial scratch too small for this tile shape");
        if (want_parts) { p.part = c->at<float>(pl.o_dn[l - 1]); p.sPartg = cap * pl.rparts[l - 1]; p.sPartTile = cap; }
        if (hb && ph.wgrad) {
          p.cpart = c->at<float>(pl.o_colpart_l[l - 1]);
          p.sCpartg = (long long)gemm_bf16_col_parts(b, pl.dims[l - 1], M) * pl.dims[l - 1];
          if ((size_t)p.sCpartg > pl.colpart_l_per[l - 1]) return cfail(c, ABS_ENOMEM, "column-partial scratch too small for this tile shape");
          // the partials are added up for all layers at once after the weight gradients
          const int e = cf.n++;
          cf.part[e] = p.cpart; cf.cols[e] = pl.dims[l - 1]; cf.nsplit[e] = gemm_bf16_col_parts(b, pl.dims[l - 1], M);
          gemm_bf16_col_part_shape(gemm_bf16_tile_shape(b, pl.dims[l - 1], M), &cf.tile_m[e], &cf.parts_per_tile[e]);
          cf.out_off[e] = pl.offB[l - 1];
          cf_bytes += 4.0 * M * cf.nsplit[e] * cf.cols[e];
        }
        HIPCHK(c, gemm(c, p, EPI_BWD, l));
      } else {
        HIPCHK(c, gemm(c, p, EPI_BWD, l));
        if (!want_parts) continue;
        ProfScope ps_(c, T_ROWNORM, 0.0, 1.0 * M * b * pl.ld[l - 1] * pl.esz);
        HIPCHK(c, launch_row_sqnorm(isb, p.C, p.sCg, pl.ld[l - 1], pl.ld[l - 1], M, b, c->at<float>(pl.o_dn[l - 1]), cap, rows, s));
      }
    }
  }   // passes
  // Number of slices of layer l's weight-gradient reduction (bf16 mode): few output tiles and a long reduction
  // (small layers, or any layer while b is the long side) are cut into slices so that the launch fills the chip;
  // the slices are added in order afterwards.
  const bool want_fused = c->fused_update && pl.bf16 && ph.wgrad && ph.update && ph.s2 && !ph.acc_grad;
  auto bf16_ksplit = [&](int l) -> int {
    const int Md = pl.dims[l], Nd = pl.dims[l - 1];
    if (!pl.bf16 || (Nd & 3)) return 1;
    const int sh = gemm_bf16_wgrad_shape(Md, Nd, b, M, want_fused);
    if (sh == 3) return 1;                      // short batches: never split
    const int te = sh == 2 ? 256 : 128, tn_e = sh == 0 ? 64 : te;
    const long long tiles = (long long)((Md + te - 1) / te) * ((Nd + tn_e - 1) / tn_e) * M;
    // with the optimizer step in the epilogue a launch that gives every CU a work-group stays whole (measured on the
    // 100 x 2048 layer of config 3 at b = 8192: 256 tiles un-split take as long as the split launch and its finish)
    if ((want_fused || ph.whole_launches) && tiles >= 256) return 1;
    return choose_ksplit(sh, tiles, (b + 63) / 64, (double)M * Md * Nd, pl.kpart_floats_l[l]);
  };
  // The optimizer step moves into the weight-gradient epilogue when the caller asked for it and this call both
  // finishes the gradient and updates, no reduction is split and the per-wavefront sums of squares fit their scratch.
  bool fused = want_fused;
  if (fused) {
    long long slots = 0;
    for (int l = 1; l <= L; ++l) {
      if (pl.dims[l - 1] & 3) fused = false;
      // a layer whose reduction is split takes its step in the launch that adds the slices
      slots += bf16_ksplit(l) > 1 ? splitk_finish_slots((long long)pl.dims[l] * pl.dims[l - 1])
                                  : gemm_bf16_upd_slots(pl.dims[l], pl.dims[l - 1], b, M);
    }
    if (hb) { int mx = 0; for (int l = 1; l <= L; ++l) mx = std::max(mx, pl.dims[l]); slots += (long long)L * ((mx + 255) / 256); }
    if (slots > pl.Ppad / 256) fused = false;
  }
  int fused_slots = 0;
  // Short batches take the inner products <g_i, gbar> from the Gram matrices of activations and backprop signals:
  // the bf16 copy of Gbar is then neither written nor read.  Only a call that runs the whole step can do so (an
  // accumulated step needs the products between samples of different micro-batches).
  const bool use_gram = pl.bf16 && pl.want_ip && ph.ip && ph.passes && ph.wgrad && !ph.acc_grad && !ph.acc_q &&
                        ph.b_total == 0 && b <= c->gram_ip_max_b && b <= GRAM_MAX_B;
  // local batch gradient, eq. (batch_grad): Gbar_l = delta^T a / b, betabar_l = mean_i delta_i
  if (ph.wgrad) {
    for (int l = 1; l <= L; ++l) {
      GemmP p;
      std::memset(&p, 0, sizeof(p));
      p.A = act_ptr(pl.o_Dl[l]); p.sAg = cap * pl.ld[l]; p.lda = pl.ld[l]; p.a_trans = 1;
      p.B = act_ptr(pl.o_A[l - 1]); p.sBg = cap * pl.ld[l - 1]; p.ldb = pl.ld[l - 1]; p.b_trans = 1;
      p.Md = pl.dims[l]; p.Nd = pl.dims[l - 1]; p.Kd = b; p.groups = M; p.rows = rows; p.gperm = gperm; p.rows_is_k = 1;
      p.C = grad + pl.offW[l]; p.sCg = pl.Ppad; p.ldc = pl.dims[l - 1];
      p.alpha = inv_b; p.accumulate = ph.acc_grad ? 1 : 0;
      if (pl.bf16 && pl.want_ip && !use_gram) { p.C2 = c->at<bf16_t>(pl.o_gradbf) + pl.offW[l]; p.sC2g = pl.Ppad; p.ldc2 = pl.dims[l - 1]; }
      if (!pl.bf16 && p.ldc == p.Nd && (((long long)p.Md * p.Nd) & 3) == 0) {
        // fp32 mode (small problems): a block walks its reduction 32 samples at a time, about 2.7 us a step, so
        // a long batch over few 64 x 64 output tiles is cut into up to 8 slices (finish launch: about 8 us)
        const long long blocks = (long long)((p.Md + 63) / 64) * ((p.Nd + 63) / 64) * M;
        const int KT = (b + 31) / 32;
        int best = 1;
        double best_cost = KT * 2.7;
        for (int S = 2; S <= 8 && blocks < 256; ++S) {
          if (blocks * S > 1024 || (size_t)S * M * p.Md * p.Nd > pl.kpart_floats_l[l]) break;
          const double cost = ((KT + S - 1) / S) * 2.7 + 8.0;
          if (cost < best_cost) { best = S; best_cost = cost; }
        }
        if (best > 1) {
          p.ksplit = best;
          p.kchunk = ((KT + best - 1) / best) * 32;
          p.kpart = c->at<float>(pl.o_kpart_l[l]);
        }
      }
      if (bf16_ksplit(l) > 1) {
        const int KT = (b + 63) / 64, S = bf16_ksplit(l);
        p.ksplit = S;
        p.kchunk = ((KT + S - 1) / S) * 64;
        p.kpart = c->at<float>(pl.o_kpart_l[l]);
      }
      if (fused && p.ksplit <= 1) {
        // the optimizer step replaces the gradient store (the fp32 gradient of the weights is never written)
        p.upd_x = xm + pl.offW[l];
        p.upd_v = c->cfg.opt != ABS_OPT_SGD ? c->at<float>(pl.o_v) + pl.offW[l] : nullptr;
        p.upd_m = c->cfg.opt == ABS_OPT_ADAMW ? c->at<float>(pl.o_m) + pl.offW[l] : nullptr;
        p.upd_shadow = c->at<bf16_t>(pl.o_xs) + pl.offW[l];
        p.upd_opt = c->cfg.opt; p.upd_lr = lr; p.upd_momentum = c->cfg.momentum; p.upd_beta1 = c->cfg.beta1;
        p.upd_beta2 = c->cfg.beta2; p.upd_eps = c->cfg.eps; p.upd_wd = c->cfg.weight_decay;
        p.upd_c1 = ph.c1; p.upd_c2 = ph.c2; p.upd_scal = ph.scal;
        p.upd_sq = c->at<float>(pl.o_sqwave); p.upd_sSqg = pl.Ppad / 256; p.upd_slot0 = fused_slots;
        fused_slots += gemm_bf16_upd_slots(p.Md, p.Nd, b, M);
      }
      HIPCHK(c, gemm(c, p, EPI_WGRAD, l));
      if (p.ksplit > 1) {                    // its slices are added up after the loop, with those of the other layers
        const int e = kf.n++;
        kf.kpart[e] = p.kpart; kf.ksplit[e] = p.ksplit; kf.mn[e] = (long long)p.Md * p.Nd; kf.c_off[e] = pl.offW[l];
        kf_bytes += (4.0 * p.ksplit + 6.0) * M * p.Md * p.Nd;
        if (fused) { kf.upd_slot0[e] = fused_slots; fused_slots += splitk_finish_slots(kf.mn[e]); }
      }
      if (hb && !pl.bf16) {
        ProfScope ps_(c, T_COLSUM, 0.0, 1.0 * M * b * pl.ld[l] * pl.esz);
        HIPCHK(c, launch_col_sum(isb, p.A, p.sAg, pl.ld[l], pl.dims[l], M, b, inv_b, grad + pl.offB[l], pl.Ppad,
                                 c->at<float>(pl.o_colpart), rows, ph.acc_grad ? 1 : 0, s));
      }
      if (hb && pl.bf16 && l == L) {      // bf16 mode: layers below L got their partials from the backward epilogue
        ProfScope ps_(c, T_COLSUM, 0.0, 1.0 * M * b * pl.ld[l] * pl.esz);
        float *scr = c->at<float>(pl.o_colpart_l[L]);
        const int e = cf.n++;
        cf.part[e] = scr; cf.cols[e] = pl.dims[L]; cf.nsplit[e] = (b + COLSUM_ROWS - 1) / COLSUM_ROWS;
        cf.tile_m[e] = 0; cf.parts_per_tile[e] = 0; cf.out_off[e] = pl.offB[L];
        if ((size_t)cf.nsplit[e] * cf.cols[e] > pl.colpart_l_per[L]) return cfail(c, ABS_ENOMEM, "column-sum scratch too small");
        cf_bytes += 4.0 * M * cf.nsplit[e] * cf.cols[e];
        HIPCHK(c, launch_col_sum_partials(isb, p.A, p.sAg, pl.ld[l], pl.dims[l], M, b, scr, rows, s));
      }
    }
    if (kf.n > 0) {                        // all split reductions of the step in one launch
      ProfScope ps_(c, T_COLSUM, 0.0, kf_bytes);
      kf.alpha = inv_b; kf.rows = rows; kf.C = grad; kf.sCg = pl.Ppad;
      kf.C2 = (pl.bf16 && pl.want_ip && !use_gram) ? c->at<bf16_t>(pl.o_gradbf) : nullptr; kf.sC2g = pl.Ppad;
      kf.accumulate = ph.acc_grad ? 1 : 0;
      if (fused) {
        kf.upd_x = xm;
        kf.upd_v = c->cfg.opt != ABS_OPT_SGD ? c->at<float>(pl.o_v) : nullptr;
        kf.upd_m = c->cfg.opt == ABS_OPT_ADAMW ? c->at<float>(pl.o_m) : nullptr;
        kf.upd_shadow = c->at<bf16_t>(pl.o_xs);
        kf.upd_opt = c->cfg.opt; kf.upd_lr = lr; kf.upd_momentum = c->cfg.momentum; kf.upd_beta1 = c->cfg.beta1;
        kf.upd_beta2 = c->cfg.beta2; kf.upd_eps = c->cfg.eps; kf.upd_wd = c->cfg.weight_decay;
        kf.upd_c1 = ph.c1; kf.upd_c2 = ph.c2; kf.upd_scal = ph.scal;
        kf.upd_sq = c->at<float>(pl.o_sqwave); kf.upd_sSqg = pl.Ppad / 256;
      }
      HIPCHK(c, launch_splitk_finish(kf, M, s));
    }
    if (cf.n > 0) {                        // all bias gradients of the step in one launch
      ProfScope ps_(c, T_COLSUM, 0.0, cf_bytes);
      cf.alpha = inv_b; cf.out = grad; cf.sOg = pl.Ppad; cf.rows = rows; cf.accumulate = ph.acc_grad ? 1 : 0;
      HIPCHK(c, launch_col_sum_finish_many(cf, M, s));
    }
  }
  // inner products <g_i, gbar>
  StatsP sp;
  std::memset(&sp, 0, sizeof(sp));
  const bool do_ip = pl.want_ip && ph.ip;
  if (do_ip && use_gram) {
    GramP gp;
    std::memset(&gp, 0, sizeof(gp));
    gp.n = 2 * L; gp.b = b; gp.groups = M; gp.rows = rows;
    gp.part = c->at<float>(pl.o_gram);
    double bytes = 0.0;
    for (int l = 1; l <= L; ++l) {
      const int a = 2 * (l - 1), d = a + 1;
      gp.X[a] = static_cast<const bf16_t *>(act_ptr(pl.o_A[l - 1])); gp.sXg[a] = cap * pl.ld[l - 1]; gp.ld[a] = pl.ld[l - 1]; gp.K[a] = pl.dims[l - 1];
      gp.X[d] = static_cast<const bf16_t *>(act_ptr(pl.o_Dl[l])); gp.sXg[d] = cap * pl.ld[l]; gp.ld[d] = pl.ld[l]; gp.K[d] = pl.dims[l];
      bytes += 2.0 * M * b * (pl.dims[l - 1] + pl.dims[l]);
    }
    float *q = c->at<float>(pl.o_qpart[0]);
    { ProfScope ps_(c, T_GRAM, 2.0 * M * b * b * (bytes / (2.0 * M * b)), bytes);
      HIPCHK(c, launch_gram_ip(gp, hb ? 1 : 0, q, cap * pl.qparts[0], s)); }
    for (int l = 1; l <= L; ++l) {          // one finished vector: it takes the place of the first layer's partials
      sp.qpart[l - 1] = q; sp.nparts[l - 1] = (l == 1) ? 1 : 0; sp.sQg[l - 1] = cap * pl.qparts[0]; sp.sQpart[l - 1] = cap;
    }
  } else if (do_ip) {
    for (int l = 1; l <= L; ++l) {
      GemmP p;
      std::memset(&p, 0, sizeof(p));
      p.A = act_ptr(pl.o_A[l - 1]); p.sAg = cap * pl.ld[l - 1]; p.lda = pl.ld[l - 1];
      p.Md = b; p.Nd = pl.dims[l]; p.Kd = pl.dims[l - 1]; p.groups = M; p.rows = rows; p.gperm = gperm;
      p.ldb = pl.dims[l - 1]; p.sBg = pl.Ppad;
      if (hb) { p.bias = grad + pl.offB[l]; p.sBiasg = pl.Ppad; }
      if (pl.bf16) {
        p.B = c->at<bf16_t>(pl.o_gradbf) + pl.offW[l];
        p.E = act_ptr(pl.o_Dl[l]); p.sEg = cap * pl.ld[l]; p.lde = pl.ld[l];
        p.part = c->at<float>(pl.o_qpart[l - 1]);
        p.sPartg = cap * pl.qparts[l - 1]; p.sPartTile = cap;
        HIPCHK(c, gemm(c, p, EPI_IPDOT, l));
        sp.qpart[l - 1] = p.part; sp.nparts[l - 1] = gemm_bf16_row_parts(b, pl.dims[l], M);
        if (sp.nparts[l - 1] > pl.qparts[l - 1]) return cfail(c, ABS_ENOMEM, "inner-product scratch too small for this tile shape");
        sp.sQg[l - 1] = p.sPartg; sp.sQpart[l - 1] = cap;
      } else {
        p.B = grad + pl.offW[l];
        float *U = c->at<float>(pl.o_U);
        p.C = U; p.sCg = cap * pl.ld[l]; p.ldc = pl.ld[l];
        HIPCHK(c, gemm(c, p, EPI_LOGITS, l));
        float *q = c->at<float>(pl.o_qpart[0]);
        { ProfScope ps_(c, T_ROWDOT, 0.0, 2.0 * M * b * pl.ld[l] * 4);
  HIPCHK(c, launch_rowdot_f32(static_cast<const float *>(act_ptr(pl.o_Dl[l])), cap * pl.ld[l], pl.ld[l], U,
                                    cap * pl.ld[l], pl.ld[l], pl.dims[l], M, b, q, cap, l > 1, rows, s)); }
        sp.qpart[l - 1] = q; sp.nparts[l - 1] = (l == 1) ? 1 : 0; sp.sQg[l - 1] = cap; sp.sQpart[l - 1] = cap;
      }
    }
  }
  // statistics
  sp.L = L; sp.has_bias = hb ? 1 : 0; sp.groups = M; sp.b = b; sp.want_ip = pl.want_ip ? 1 : 0; sp.rows = rows;
  sp.do_n = ph.nstats ? 1 : 0; sp.do_q = do_ip ? 1 : 0; sp.acc_n = ph.acc_n ? 1 : 0; sp.acc_q = ph.acc_q ? 1 : 0;
  for (int l = 0; l < L; ++l) {
    sp.an[l] = c->at<float>(pl.o_an[l]); sp.dn[l] = c->at<float>(pl.o_dn[l + 1]);
    sp.an_parts[l] = an_parts[l]; sp.an_sg[l] = cap * pl.rparts[l];
    sp.dn_parts[l] = dn_parts[l + 1]; sp.dn_sg[l] = cap * pl.rparts[l + 1];
  }
  sp.sNg = cap;
  sp.loss = c->at<float>(pl.o_loss);
  if (ph.ps_off >= 0) { sp.n_out = c->at<float>(pl.o_nout) + ph.ps_off; sp.q_out = c->at<float>(pl.o_qout) + ph.ps_off; }
  sp.Ppad = pl.Ppad;
  sp.partials = c->at<double>(pl.o_partials); sp.stats = c->at<double>(pl.o_stats);
  sp.stats_host = c->host_stats_dev;
  if (sp.stats_host) { c->ticket += 1.0; sp.ticket = c->ticket; c->ticket_live = true; }
  // When this call both finishes the gradient and updates, the update kernel gathers ||gbar||^2 on
  // its way through the gradient (none of the statistics depends on the parameters, so the update
  // may run first); otherwise a separate pass over the gradient does.
  const bool s2_in_update = ph.s2 && ph.update;
  sp.grad = (ph.s2 && !s2_in_update) ? grad : nullptr;
  if (fused) {
    // the weights have taken their step in the epilogues; the biases take theirs here, and ||gbar||^2 is the sum
    // of the slots the epilogues and this launch left
    if (hb) {
      BiasUpdateP bu;
      std::memset(&bu, 0, sizeof(bu));
      bu.n = L;
      for (int l = 1; l <= L; ++l) { bu.width[l - 1] = pl.dims[l]; bu.off[l - 1] = pl.offB[l]; }
      bu.stride = pl.Ppad;
      bu.x = xm; bu.g = grad;
      bu.v = c->cfg.opt != ABS_OPT_SGD ? c->at<float>(pl.o_v) : nullptr;
      bu.m = c->cfg.opt == ABS_OPT_ADAMW ? c->at<float>(pl.o_m) : nullptr;
      bu.shadow = c->at<bf16_t>(pl.o_xs);
      bu.opt = c->cfg.opt; bu.lr = lr; bu.momentum = c->cfg.momentum; bu.beta1 = c->cfg.beta1; bu.beta2 = c->cfg.beta2;
      bu.eps = c->cfg.eps; bu.wd = c->cfg.weight_decay; bu.c1 = ph.c1; bu.c2 = ph.c2; bu.scal = ph.scal;
      bu.sq = c->at<float>(pl.o_sqwave); bu.sSqg = pl.Ppad / 256; bu.slot0 = fused_slots;
      fused_slots += update_bias_slots(bu);
      ProfScope ps_(c, T_UPDATE, 0.0, 0.0);
      HIPCHK(c, launch_update_bias(bu, M, s));
    }
    sp.sq_wave = c->at<float>(pl.o_sqwave); sp.n_sq_wave = fused_slots;
    sp.sq_stride = pl.Ppad / 256;
    ProfScope ps_(c, T_STATS, 0.0, 4.0 * M * fused_slots);
    HIPCHK(c, launch_stats(sp, s));
    note_step(c, ph.b_total > 0 ? ph.b_total : b, b_host);
    c->last_fused = true;
    return ABS_OK;
  }
  c->last_fused = false;
  if (!s2_in_update) {
    ProfScope ps_(c, T_STATS, 0.0, ph.s2 ? 4.0 * M * pl.Ppad : 0.0);
    HIPCHK(c, launch_stats(sp, s));
  }
  if (!ph.update) return ABS_OK;
  // optimizer update (Alg. 1: "local SGD step ... or other inner optimizers")
  UpdateP up;
  std::memset(&up, 0, sizeof(up));
  up.x = xm; up.g = grad;
  up.v = c->cfg.opt != ABS_OPT_SGD ? c->at<float>(pl.o_v) : nullptr;
  up.m = c->cfg.opt == ABS_OPT_ADAMW ? c->at<float>(pl.o_m) : nullptr;
  up.shadow = pl.bf16 ? c->at<bf16_t>(pl.o_xs) : nullptr;
  up.n = (long long)M * pl.Ppad;
  up.opt = c->cfg.opt; up.lr = lr; up.momentum = c->cfg.momentum;
  up.beta1 = c->cfg.beta1; up.beta2 = c->cfg.beta2; up.eps = c->cfg.eps; up.wd = c->cfg.weight_decay;
  up.c1 = ph.c1; up.c2 = ph.c2; up.scal = ph.scal;
  if (s2_in_update) up.sq_wave = c->at<float>(pl.o_sqwave);
  { ProfScope ps_(c, T_UPDATE, 0.0, 1.0 * M * pl.P * (c->cfg.opt == ABS_OPT_SGD ? 12 : c->cfg.opt == ABS_OPT_ADAMW ? 28 : 20) + (pl.bf16 ? 2.0 * M * pl.P : 0.0));
  HIPCHK(c, launch_update(up, s)); }
  if (s2_in_update) {
    sp.sq_wave = up.sq_wave; sp.n_sq_wave = pl.Ppad / 256;
    ProfScope ps_(c, T_STATS, 0.0, 4.0 * M * (pl.Ppad / 256));
    HIPCHK(c, launch_stats(sp, s));
  }
  note_step(c, ph.b_total > 0 ? ph.b_total : b, b_host);
  return ABS_OK;
}

// A step that failed before its update was enqueued has not advanced the optimizer.
static abs_status settle_update(abs_ctx *c, abs_status st) {
  if (st != ABS_OK) c->t -= 1;
  return st;
}

// Captured steps record which form of the update and of the inner products they took: a change of either setting
// discards them (the next graphed step captures again).
static void drop_graphs(abs_ctx *c) {
  if (c->graphs.empty()) return;
  (void)hipStreamSynchronize(c->stream);          // one of them may still be running
  for (auto &g : c->graphs) (void)hipGraphExecDestroy(g.exec);
  c->graphs.clear();
}

// After a step that took the optimizer step inside the weight-gradient epilogue the fp32 gradient of the weights was
// never stored.  The layer inputs and backprop signals of that step are still in the workspace (only the next step
// overwrites them), so the gradient is formed on demand: the same contractions with the plain epilogue, cut into the
// same launches, give the very entries the epilogue applied.  Bias gradients were stored by the step itself.
static abs_status materialize_grad(abs_ctx *c) {
  if (!c->last_fused) return ABS_OK;
  StepPhase ph;
  ph.passes = ph.nstats = ph.s2 = ph.ip = ph.update = false;
  ph.whole_launches = true;
  ph.ps_off = -1;
  abs_status st = local_step_impl(c, nullptr, c->last_b, c->last_b, c->last_ragged ? c->last_bm.data() : nullptr, 0.0f, ph);
  if (st != ABS_OK) return st;
  c->last_fused = false;
  return ABS_OK;
}

// One more optimizer step is about to be taken: advance the counter and return Adam's bias corrections.
static void next_update(abs_ctx *c, StepPhase &ph) {
  c->t += 1;
  if (c->cfg.opt == ABS_OPT_ADAMW) {
    ph.c1 = (float)(1.0 / (1.0 - std::pow((double)c->cfg.beta1, (double)c->t)));
    ph.c2 = (float)(1.0 / (1.0 - std::pow((double)c->cfg.beta2, (double)c->t)));
  }
}

abs_status abs_local_step(abs_ctx *c, const int32_t *idx_dev, int b, float lr) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (!idx_dev) return cfail(c, ABS_EINVAL, "idx_dev is NULL");
  if (b < 2 || b > c->pl.cap) return cfail(c, ABS_EINVAL, "b must be in [2, b_cap]");
  if (!(lr == lr)) return cfail(c, ABS_EINVAL, "lr is NaN");
  StepPhase ph;
  next_update(c, ph);
  return settle_update(c, local_step_impl(c, idx_dev, b, b, nullptr, lr, ph));
} catch (...) { return on_exception(); }

abs_status abs_local_step_graphed(abs_ctx *c, const int32_t *idx_dev, int b, float lr) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (!idx_dev) return cfail(c, ABS_EINVAL, "idx_dev is NULL");
  if (b < 2 || b > c->pl.cap) return cfail(c, ABS_EINVAL, "b must be in [2, b_cap]");
  if (!(lr == lr)) return cfail(c, ABS_EINVAL, "lr is NaN");
  // event brackets cannot be captured, nor can work on the legacy default stream: run such steps directly
  if (c->prof_on || c->stream == nullptr) return abs_local_step(c, idx_dev, b, lr);
  const Plan &pl = c->pl;
  StepPhase ph;
  next_update(c, ph);
  int32_t *idx_in = c->at<int32_t>(pl.o_idx);
  float *scal = c->at<float>(pl.o_scal);
  ph.scal = scal;
  // the only launch whose arguments change from step to step: it carries them into fixed device locations
  {
    hipError_t e = launch_stage_step_inputs(idx_dev, idx_in, (long long)pl.M * b, lr, ph.c1, ph.c2, scal, c->stream);
    if (e != hipSuccess) return settle_update(c, cfail(c, ABS_EHIP, std::string("launch_stage_step_inputs: ") + hipGetErrorString(e)));
  }
  abs_ctx::GraphSlot *slot = nullptr;
  for (auto &g : c->graphs) if (g.b == b) slot = &g;
  if (!slot) {
    bool warm = false;
    for (int w : c->graph_warm) warm = warm || w == b;
    if (!warm) {
      // first step at this batch size: run it directly, which also sets the attributes of every kernel
      // variant this size uses (not something to do inside a capture)
      c->graph_warm.push_back(b);
      return settle_update(c, local_step_impl(c, idx_in, b, b, nullptr, lr, ph));
    }
    hipGraph_t graph = nullptr;
    {
      hipError_t eb = hipStreamBeginCapture(c->stream, hipStreamCaptureModeThreadLocal);
      if (eb != hipSuccess) return settle_update(c, cfail(c, ABS_EHIP, std::string("hipStreamBeginCapture: ") + hipGetErrorString(eb)));
    }
    const long long samples_before = c->n_samples;     // the captured pass only records launches: it is not a step
    abs_status st = local_step_impl(c, idx_in, b, b, nullptr, lr, ph);
    hipError_t e = hipStreamEndCapture(c->stream, &graph);
    c->n_samples = samples_before;
    if (st != ABS_OK) { if (graph) (void)hipGraphDestroy(graph); return settle_update(c, st); }
    if (e != hipSuccess || !graph) return settle_update(c, cfail(c, ABS_EHIP, std::string("hipStreamEndCapture: ") + hipGetErrorString(e)));
    hipGraphExec_t exec = nullptr;
    e = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    (void)hipGraphDestroy(graph);
    if (e != hipSuccess) return settle_update(c, cfail(c, ABS_EHIP, std::string("hipGraphInstantiate: ") + hipGetErrorString(e)));
    if (c->graphs.size() >= 8) {                                  // keep a few sizes: drop the least recently used
      size_t old = 0;
      for (size_t i = 1; i < c->graphs.size(); ++i) if (c->graphs[i].last_use < c->graphs[old].last_use) old = i;
      (void)hipGraphExecDestroy(c->graphs[old].exec);
      c->graphs.erase(c->graphs.begin() + old);
    }
    c->graphs.push_back({b, exec, 0, c->last_fused});    // (set by the capturing pass)
    slot = &c->graphs.back();
  }
  slot->last_use = c->t;
  c->ticket_live = false;             // a replayed launch carries the ticket of its capture: synchronise instead
  {
    hipError_t el = hipGraphLaunch(slot->exec, c->stream);
    if (el != hipSuccess) return settle_update(c, cfail(c, ABS_EHIP, std::string("hipGraphLaunch: ") + hipGetErrorString(el)));
  }
  c->last_fused = slot->fused;        // whether the replayed step left its fp32 gradient unstored
  note_step(c, b, nullptr);
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_graph_count(const abs_ctx *c, int *n) try {
  if (!c || !n) return fail(ABS_EINVAL, "NULL argument");
  *n = (int)c->graphs.size();
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_local_step_accumulated(abs_ctx *c, const int32_t *idx_dev, int b, int micro_b, float lr) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (!idx_dev) return cfail(c, ABS_EINVAL, "idx_dev is NULL");
  if (!(lr == lr)) return cfail(c, ABS_EINVAL, "lr is NaN");
  const int cap = c->pl.cap;
  if (micro_b < 2 || micro_b > cap) return cfail(c, ABS_EINVAL, "micro_b must be in [2, b_cap]");
  if (b < 2) return cfail(c, ABS_EINVAL, "b must be at least 2");
  if (b % micro_b == 1) return cfail(c, ABS_EINVAL, "the last micro-batch would hold a single sample");
  const int nmb = (b + micro_b - 1) / micro_b;
  // pass 1: batch gradient, S1 and the loss, micro-batch by micro-batch; S2 once the gradient is whole
  for (int j = 0; j < nmb; ++j) {
    const int off = j * micro_b, mb = b - off < micro_b ? b - off : micro_b;
    StepPhase ph;
    ph.ip = false; ph.update = false;
    ph.s2 = j == nmb - 1;
    ph.acc_grad = ph.acc_n = j > 0;
    ph.b_total = b;
    ph.ps_off = off + mb <= cap ? off : -1;
    abs_status st = local_step_impl(c, idx_dev + off, b, mb, nullptr, lr, ph);
    if (st != ABS_OK) return st;
  }
  // pass 2: <g_i, gbar> needs the gradient of the whole batch, so the passes run once more
  if (c->pl.want_ip) {
    for (int j = 0; j < nmb; ++j) {
      const int off = j * micro_b, mb = b - off < micro_b ? b - off : micro_b;
      StepPhase ph;
      ph.wgrad = ph.nstats = ph.s2 = ph.update = false;
      ph.acc_q = j > 0;
      ph.b_total = b;
      ph.ps_off = off + mb <= cap ? off : -1;
      abs_status st = local_step_impl(c, idx_dev + off, b, mb, nullptr, lr, ph);
      if (st != ABS_OK) return st;
    }
  }
  StepPhase up;
  up.passes = up.wgrad = up.nstats = up.s2 = up.ip = false;
  up.b_total = b;
  next_update(c, up);
  abs_status st = settle_update(c, local_step_impl(c, idx_dev, b, micro_b, nullptr, lr, up));
  if (st != ABS_OK) return st;
  c->last_ps = 0;
  for (int j = 0; j < nmb; ++j) {
    const int off = j * micro_b, mb = b - off < micro_b ? b - off : micro_b;
    if (off + mb <= cap) c->last_ps = off + mb;
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_local_step_ragged(abs_ctx *c, const int32_t *idx_dev, int ldi, const int *b_host, float lr) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (!idx_dev || !b_host) return cfail(c, ABS_EINVAL, "idx_dev or b_host is NULL");
  if (!(lr == lr)) return cfail(c, ABS_EINVAL, "lr is NaN");
  int bmax = 0;
  for (int m = 0; m < c->pl.M; ++m) {
    if (b_host[m] < 2 || b_host[m] > c->pl.cap) return cfail(c, ABS_EINVAL, "every b[m] must be in [2, b_cap]");
    if (b_host[m] > bmax) bmax = b_host[m];
  }
  if (ldi < bmax) return cfail(c, ABS_EINVAL, "ldi must be >= max_m b[m]");
  StepPhase ph;
  next_update(c, ph);
  return settle_update(c, local_step_impl(c, idx_dev, ldi, bmax, b_host, lr, ph));
} catch (...) { return on_exception(); }

static abs_status norm_test_impl(abs_ctx *c, const double *eta_m, double eta_all, int64_t n_total,
                                 abs_test_result *out) {
  if (!c || !out) return fail(ABS_EINVAL, "NULL argument");
  for (int m = 0; m < c->pl.M; ++m) {
    const double eta = eta_m ? eta_m[m] : eta_all;
    if (!(eta > 0.0 && eta < 1.0)) return cfail(c, ABS_EINVAL, "eta must be in (0,1)");
  }
  abs_status st = read_stats(c);
  if (st != ABS_OK) return st;
  if (n_total != 0 && (n_total < 2 || n_total < c->last_b)) return cfail(c, ABS_EINVAL, "n_total must be >= max(2, b)");
  for (int m = 0; m < c->pl.M; ++m) {
    const int b = c->last_bm[m];
    const double eta = eta_m ? eta_m[m] : eta_all;
    // finite-population factor of Sec. 4.1 (1 when sampling with replacement / n unknown)
    const double fpc = n_total > 0 ? (double)(n_total - b) / (double)(n_total - 1) : 1.0;
    abs_test_result r;
    fill_result(r, b, c->host_stats + m * 8);
    r.var = fpc * (r.sum_sq - (double)b * r.gbar_sq) / (double)(b - 1);
    r.lhs = r.var / (double)b;
    r.rhs = eta * eta * r.gbar_sq;
    ceil_ratio(r.var, eta * eta * r.gbar_sq, b, r.ratio, r.T);
    r.pass = (r.lhs <= r.rhs) ? 1 : 0;
    out[m] = r;
  }
  return ABS_OK;
}

abs_status abs_norm_test(abs_ctx *c, double eta, abs_test_result *out) try {
  return norm_test_impl(c, nullptr, eta, 0, out);
} catch (...) { return on_exception(); }

abs_status abs_norm_test_per_worker(abs_ctx *c, const double *eta, abs_test_result *out) try {
  if (!eta) return c ? cfail(c, ABS_EINVAL, "eta is NULL") : fail(ABS_EINVAL, "NULL argument");
  return norm_test_impl(c, eta, 0.0, 0, out);
} catch (...) { return on_exception(); }

abs_status abs_norm_test_fpc(abs_ctx *c, double eta, int64_t n_total, abs_test_result *out) try {
  if (n_total < 2) return c ? cfail(c, ABS_EINVAL, "n_total must be >= max(2, b)") : fail(ABS_EINVAL, "NULL argument");
  return norm_test_impl(c, nullptr, eta, n_total, out);
} catch (...) { return on_exception(); }

abs_status abs_inner_product_test(abs_ctx *c, double theta, double nu, abs_test_result *out) try {
  if (!c || !out) return fail(ABS_EINVAL, "NULL argument");
  if (!(theta > 0.0)) return cfail(c, ABS_EINVAL, "theta must be positive");
  if (!c->pl.want_ip) return cfail(c, ABS_ESTATE, "stats_mask lacks ABS_STATS_IP");
  abs_status st = read_stats(c);
  if (st != ABS_OK) return st;
  for (int m = 0; m < c->pl.M; ++m) {
    const int b = c->last_bm[m];
    abs_test_result r;
    fill_result(r, b, c->host_stats + m * 8);
    const double S1 = r.sum_sq, S2 = r.gbar_sq, S3 = r.sum_q2, S4 = r.sum_q;
    r.var = (S3 - S4 * S4 / (double)b) / (double)(b - 1);
    r.var_perp = S2 > 0.0 ? (S1 - S3 / S2) / (double)(b - 1) : 0.0;
    r.lhs = r.var / (double)b;
    r.rhs = theta * theta * S2 * S2;
    ceil_ratio(r.var, r.rhs, b, r.ratio, r.T);
    r.pass = (r.lhs <= r.rhs) ? 1 : 0;
    if (nu > 0.0) {
      double ro; long long To;
      ceil_ratio(r.var_perp, nu * nu * S2, b, ro, To);
      if (To > r.T) r.T = To;
      if (ro > r.ratio) r.ratio = ro;
      if (!(r.var_perp / (double)b <= nu * nu * S2)) r.pass = 0;
    }
    out[m] = r;
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_cross_worker_test(abs_ctx *c, double eta, abs_test_result *out) try {
  if (!c || !out) return fail(ABS_EINVAL, "NULL argument");
  if (!(eta > 0.0 && eta < 1.0)) return cfail(c, ABS_EINVAL, "eta must be in (0,1)");
  if (c->pl.M < 2) return cfail(c, ABS_EINVAL, "the cross-worker estimator needs M >= 2");
  if (!c->have_stats) return cfail(c, ABS_ESTATE, "no local step has been taken yet");
  if (c->last_ragged) return cfail(c, ABS_ESTATE, "the cross-worker estimator needs equal local batch sizes");
  { abs_status ms = materialize_grad(c); if (ms != ABS_OK) return ms; }
  const Plan &pl = c->pl;
  double *cw = c->at<double>(pl.o_cw);
  HIPCHK(c, launch_cross_worker(c->at<float>(pl.o_grad), pl.M, pl.Ppad, cw + 8, cw, c->stream));
  double *h = c->host_stats + (size_t)pl.M * 8;
  HIPCHK(c, hipMemcpyAsync(h, cw, 2 * sizeof(double), hipMemcpyDeviceToHost, c->stream));
  HIPCHK(c, hipStreamSynchronize(c->stream));
  abs_test_result r;
  std::memset(&r, 0, sizeof(r));
  const int b = c->last_b, M = pl.M;
  r.b = b; r.sum_sq = h[0]; r.gbar_sq = h[1];
  r.var = (double)b * (h[0] - (double)M * h[1]) / (double)(M - 1);
  r.lhs = r.var / ((double)b * M);
  r.rhs = eta * eta * r.gbar_sq;
  ceil_ratio(r.var, (double)M * eta * eta * r.gbar_sq, b, r.ratio, r.T);
  r.pass = (r.lhs <= r.rhs) ? 1 : 0;
  *out = r;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_next_batch_size(const abs_test_result *res, int M, const int *b_cur, int b_cap, int sync_max,
                               int *b_next) try {
  if (!res || !b_cur || !b_next) return fail(ABS_EINVAL, "NULL argument");
  if (M < 1 || b_cap < 1) return fail(ABS_EINVAL, "M or b_cap out of range");
  long long mx = 0;
  std::vector<long long> nx(M);
  for (int m = 0; m < M; ++m) {
    nx[m] = res[m].T > b_cur[m] ? res[m].T : b_cur[m];
    if (nx[m] > mx) mx = nx[m];
  }
  for (int m = 0; m < M; ++m) {
    long long v = sync_max ? mx : nx[m];
    b_next[m] = (int)(v > b_cap ? b_cap : v);
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_average_replicas(abs_ctx *c) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  const Plan &pl = c->pl;
  {
    ProfScope ps_(c, T_AVERAGE, 0.0, (double)pl.M * pl.P * (pl.bf16 ? 10.0 : 8.0));
    HIPCHK(c, launch_average_f32(c->at<float>(pl.o_xm), pl.bf16 ? c->at<bf16_t>(pl.o_xs) : nullptr, c->at<float>(pl.o_mean), pl.M, pl.Ppad,
                                 c->stream));
  }
  c->n_rounds += 1;                  // Alg. 1: k <- k + 1
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_set_fused_update(abs_ctx *c, int on) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (on && !c->pl.bf16) return cfail(c, ABS_EUNSUPPORTED, "the fused update needs ABS_PREC_BF16");
  if (c->fused_update != (on != 0)) drop_graphs(c);      // captured steps recorded the other form
  c->fused_update = on != 0;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_set_gram_ip_max_batch(abs_ctx *c, int b_max) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (b_max < 0 || b_max > GRAM_MAX_B) return cfail(c, ABS_EINVAL, "b_max must be in [0, 256]");
  if (c->gram_ip_max_b != b_max) drop_graphs(c);         // captured steps recorded the other form
  c->gram_ip_max_b = b_max;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_get_counters(const abs_ctx *c, long long *rounds, long long *local_steps, long long *samples) try {
  if (!c) return fail(ABS_EINVAL, "ctx is NULL");
  if (rounds) *rounds = c->n_rounds;
  if (local_steps) *local_steps = c->t;
  if (samples) *samples = c->n_samples;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_get_opt_state(abs_ctx *c, int m, int which, float *out_host) try {
  if (!c || !out_host) return fail(ABS_EINVAL, "NULL argument");
  if (m < 0 || m >= c->pl.M) return cfail(c, ABS_EINVAL, "replica index out of range");
  const bool has_v = c->cfg.opt != ABS_OPT_SGD, has_m = c->cfg.opt == ABS_OPT_ADAMW;
  if (!((which == 0 && has_v) || (which == 1 && has_m)))
    return cfail(c, ABS_EINVAL, "this optimizer keeps no such state vector");
  std::vector<float> in(c->pl.Ppad);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(in.data(), c->at<float>(which == 0 ? c->pl.o_v : c->pl.o_m) + (size_t)m * c->pl.Ppad,
                      c->pl.Ppad * sizeof(float), hipMemcpyDeviceToHost));
  to_external(c->pl, c->cfg.has_bias != 0, in.data(), out_host);
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_get_params(abs_ctx *c, int m, float *out_host) try {
  if (!c || !out_host) return fail(ABS_EINVAL, "NULL argument");
  if (m < 0 || m >= c->pl.M) return cfail(c, ABS_EINVAL, "replica index out of range");
  std::vector<float> in(c->pl.Ppad);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(in.data(), c->at<float>(c->pl.o_xm) + (size_t)m * c->pl.Ppad, c->pl.Ppad * sizeof(float), hipMemcpyDeviceToHost));
  to_external(c->pl, c->cfg.has_bias != 0, in.data(), out_host);
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_get_grad(abs_ctx *c, int m, float *out_host) try {
  if (!c || !out_host) return fail(ABS_EINVAL, "NULL argument");
  if (m < 0 || m >= c->pl.M) return cfail(c, ABS_EINVAL, "replica index out of range");
  if (!c->have_stats) return cfail(c, ABS_ESTATE, "no local step has been taken yet");
  { abs_status ms = materialize_grad(c); if (ms != ABS_OK) return ms; }
  std::vector<float> in(c->pl.Ppad);
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(in.data(), c->at<float>(c->pl.o_grad) + (size_t)m * c->pl.Ppad, c->pl.Ppad * sizeof(float), hipMemcpyDeviceToHost));
  to_external(c->pl, c->cfg.has_bias != 0, in.data(), out_host);
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_set_params(abs_ctx *c, int m, const float *in_host) try {
  if (!c || !in_host) return fail(ABS_EINVAL, "NULL argument");
  if (m < 0 || m >= c->pl.M) return cfail(c, ABS_EINVAL, "replica index out of range");
  const Plan &pl = c->pl;
  std::vector<float> in(pl.Ppad, 0.0f);
  to_internal(pl, c->cfg.has_bias != 0, in_host, in.data());
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(c->at<float>(pl.o_xm) + (size_t)m * pl.Ppad, in.data(), pl.Ppad * sizeof(float), hipMemcpyHostToDevice));
  if (pl.bf16) {
    HIPCHK(c, launch_convert_f32_to_bf16(c->at<float>(pl.o_xm) + (size_t)m * pl.Ppad, c->at<bf16_t>(pl.o_xs) + (size_t)m * pl.Ppad, pl.Ppad, c->stream));
    HIPCHK(c, hipStreamSynchronize(c->stream));
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_get_per_sample(abs_ctx *c, int m, float *n_host, float *q_host) try {
  if (!c || !n_host) return fail(ABS_EINVAL, "NULL argument");
  if (m < 0 || m >= c->pl.M) return cfail(c, ABS_EINVAL, "replica index out of range");
  if (!c->have_stats) return cfail(c, ABS_ESTATE, "no local step has been taken yet");
  if (q_host && !c->pl.want_ip) return cfail(c, ABS_ESTATE, "stats_mask lacks ABS_STATS_IP");
  HIPCHK(c, hipStreamSynchronize(c->stream));
  HIPCHK(c, hipMemcpy(n_host, c->at<float>(c->pl.o_nout) + (size_t)m * c->pl.cap, (size_t)(c->last_ps >= 0 ? c->last_ps : c->last_bm[m]) * sizeof(float), hipMemcpyDeviceToHost));
  if (q_host)
    HIPCHK(c, hipMemcpy(q_host, c->at<float>(c->pl.o_qout) + (size_t)m * c->pl.cap, (size_t)(c->last_ps >= 0 ? c->last_ps : c->last_bm[m]) * sizeof(float), hipMemcpyDeviceToHost));
  return ABS_OK;
} catch (...) { return on_exception(); }

// ---- statistics and averaging alone ---------------------------------------------------------

static abs_status ls_plan(int L, const int *in_dims, const int *out_dims, int M, int b, std::vector<size_t> &off,
                          std::vector<long long> &woff, long long &Wtot, size_t &total) {
  if (L < 1 || L > MAXL || !in_dims || !out_dims) return fail(ABS_EINVAL, "bad layer list");
  if (M < 1 || b < 2) return fail(ABS_EINVAL, "M < 1 or b < 2");
  woff.assign(L, 0);
  Wtot = 0;
  for (int l = 0; l < L; ++l) {
    if (in_dims[l] < 8 || out_dims[l] < 8 || (in_dims[l] % 8) || (out_dims[l] % 8))
      return fail(ABS_EUNSUPPORTED, "layer widths must be multiples of 8");
    woff[l] = Wtot;
    Wtot += (long long)in_dims[l] * out_dims[l];
  }
  Wtot = rup(Wtot, 256);
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t r = o; o = (size_t)rup((long long)(o + bytes), 256); return r; };
  off.clear();
  off.push_back(take((size_t)M * Wtot * 4));                 // 0: grad f32
  off.push_back(take((size_t)M * Wtot * 2));                 // 1: grad bf16
  off.push_back(take((size_t)M * b * 4 * L));                // 2: an
  off.push_back(take((size_t)M * b * 4 * L));                // 3: dn
  off.push_back(take((size_t)M * b * 4));                    // 4: loss (zeros)
  off.push_back(take((size_t)M * b * 4));                    // 5: n_out
  off.push_back(take((size_t)M * b * 4));                    // 6: q_out
  off.push_back(take((size_t)M * 5 * STATS_PBLK * 8));       // 7: partials
  off.push_back(take((size_t)M * 8 * 8));                    // 8: stats
  for (int l = 0; l < L; ++l) off.push_back(take((size_t)M * b * 4 * gemm_bf16_ipdot_parts(out_dims[l])));  // 9+l
  total = o;
  return ABS_OK;
}

abs_status abs_layer_stats_workspace_bytes(int L, const int *in_dims, const int *out_dims, int M, int b,
                                           size_t *bytes) try {
  if (!bytes) return fail(ABS_EINVAL, "bytes is NULL");
  std::vector<size_t> off; std::vector<long long> woff; long long Wtot; size_t total;
  abs_status st = ls_plan(L, in_dims, out_dims, M, b, off, woff, Wtot, total);
  if (st != ABS_OK) return st;
  *bytes = total;
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_layer_stats(int L, const int *in_dims, const int *out_dims, int M, int b, const void *const *a_dev,
                           const void *const *delta_dev, void *workspace, size_t workspace_bytes, void *hip_stream,
                           abs_test_result *out, float *n_out_dev, float *q_out_dev, float *gbar_out_dev) try {
  if (!a_dev || !delta_dev || !workspace || !out) return fail(ABS_EINVAL, "NULL argument");
  std::vector<size_t> off; std::vector<long long> woff; long long Wtot; size_t total;
  abs_status st = ls_plan(L, in_dims, out_dims, M, b, off, woff, Wtot, total);
  if (st != ABS_OK) return st;
  if (workspace_bytes < total) return fail(ABS_ENOMEM, "workspace too small");
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(ABS_EINVAL, "workspace must be 256-byte aligned");
  for (int l = 0; l < L; ++l)
    if (!a_dev[l] || !delta_dev[l] || (reinterpret_cast<uintptr_t>(a_dev[l]) & 15) || (reinterpret_cast<uintptr_t>(delta_dev[l]) & 15))
      return fail(ABS_EINVAL, "layer pointers must be non-NULL and 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  unsigned char *ws = static_cast<unsigned char *>(workspace);
  float *grad = reinterpret_cast<float *>(ws + off[0]);
  bf16_t *gradbf = reinterpret_cast<bf16_t *>(ws + off[1]);
  float *an = reinterpret_cast<float *>(ws + off[2]);
  float *dn = reinterpret_cast<float *>(ws + off[3]);
  float *loss = reinterpret_cast<float *>(ws + off[4]);
  abs_ctx *nc = nullptr;
  HIPCHK(nc, launch_fill_zero(loss, (long long)M * b * 4, s));
  {
    // the weight gradients overwrite every entry of their layers; only the padding behind the last layer,
    // which the ||gbar||^2 pass reads too, has to be cleared
    long long Wsum = 0;
    for (int l = 0; l < L; ++l) Wsum += (long long)in_dims[l] * out_dims[l];
    HIPCHK(nc, launch_zero_range(grad, Wtot, Wsum, Wtot, M, s));
  }
  StatsP sp;
  std::memset(&sp, 0, sizeof(sp));
  const float inv_b = 1.0f / (float)b;
  for (int l = 0; l < L; ++l) {
    const long long sa = (long long)b * in_dims[l], sd = (long long)b * out_dims[l];
    HIPCHK(nc, launch_row_sqnorm(1, a_dev[l], sa, in_dims[l], in_dims[l], M, b, an + (size_t)l * M * b, b, nullptr, s));
    HIPCHK(nc, launch_row_sqnorm(1, delta_dev[l], sd, out_dims[l], out_dims[l], M, b, dn + (size_t)l * M * b, b, nullptr, s));
    GemmP p;
    std::memset(&p, 0, sizeof(p));
    p.A = delta_dev[l]; p.sAg = sd; p.lda = out_dims[l]; p.a_trans = 1;
    p.B = a_dev[l]; p.sBg = sa; p.ldb = in_dims[l]; p.b_trans = 1;
    p.Md = out_dims[l]; p.Nd = in_dims[l]; p.Kd = b; p.groups = M;
    p.C = grad + woff[l]; p.sCg = Wtot; p.ldc = in_dims[l];
    p.C2 = gradbf + woff[l]; p.sC2g = Wtot; p.ldc2 = in_dims[l];
    p.alpha = inv_b;
    HIPCHK(nc, launch_gemm_bf16(p, EPI_WGRAD, s));
  }
  for (int l = 0; l < L; ++l) {
    const long long sa = (long long)b * in_dims[l], sd = (long long)b * out_dims[l];
    const int np = gemm_bf16_ipdot_parts(out_dims[l]);
    GemmP p;
    std::memset(&p, 0, sizeof(p));
    p.A = a_dev[l]; p.sAg = sa; p.lda = in_dims[l];
    p.B = gradbf + woff[l]; p.sBg = Wtot; p.ldb = in_dims[l];
    p.Md = b; p.Nd = out_dims[l]; p.Kd = in_dims[l]; p.groups = M;
    p.E = delta_dev[l]; p.sEg = sd; p.lde = out_dims[l];
    p.part = reinterpret_cast<float *>(ws + off[9 + l]); p.sPartg = (long long)b * np; p.sPartTile = b;
    HIPCHK(nc, launch_gemm_bf16(p, EPI_IPDOT, s));
    sp.qpart[l] = p.part; sp.nparts[l] = gemm_bf16_row_parts(b, out_dims[l], M); sp.sQg[l] = p.sPartg; sp.sQpart[l] = b;
    sp.an[l] = an + (size_t)l * M * b; sp.dn[l] = dn + (size_t)l * M * b;
    sp.an_parts[l] = sp.dn_parts[l] = 1; sp.an_sg[l] = sp.dn_sg[l] = b;
  }
  sp.L = L; sp.has_bias = 0; sp.groups = M; sp.b = b; sp.want_ip = 1; sp.sNg = b;
  sp.do_n = sp.do_q = 1;
  sp.loss = loss;
  sp.n_out = n_out_dev ? n_out_dev : reinterpret_cast<float *>(ws + off[5]);
  sp.q_out = q_out_dev ? q_out_dev : reinterpret_cast<float *>(ws + off[6]);
  sp.grad = grad; sp.Ppad = Wtot;
  sp.partials = reinterpret_cast<double *>(ws + off[7]);
  sp.stats = reinterpret_cast<double *>(ws + off[8]);
  HIPCHK(nc, launch_stats(sp, s));
  if (gbar_out_dev) {
    long long Wsum = 0;
    for (int l = 0; l < L; ++l) Wsum += (long long)in_dims[l] * out_dims[l];
    for (int m = 0; m < M; ++m)
      HIPCHK(nc, hipMemcpyAsync(gbar_out_dev + (size_t)m * Wsum, grad + (size_t)m * Wtot, Wsum * sizeof(float), hipMemcpyDeviceToDevice, s));
  }
  std::vector<double> h((size_t)M * 8);
  HIPCHK(nc, hipMemcpyAsync(h.data(), sp.stats, h.size() * sizeof(double), hipMemcpyDeviceToHost, s));
  HIPCHK(nc, hipStreamSynchronize(s));
  for (int m = 0; m < M; ++m) {
    abs_test_result r;
    fill_result(r, b, h.data() + (size_t)m * 8);
    r.var = (r.sum_sq - (double)b * r.gbar_sq) / (double)(b - 1);
    out[m] = r;
  }
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_copy_probe(const void *src_dev, void *dst_dev, int64_t bytes, void *hip_stream) try {
  if (!src_dev || !dst_dev) return fail(ABS_EINVAL, "NULL argument");
  if (bytes < 16 || (bytes % 16) || ((reinterpret_cast<uintptr_t>(src_dev) | reinterpret_cast<uintptr_t>(dst_dev)) & 15))
    return fail(ABS_EINVAL, "bytes must be a positive multiple of 16 and the pointers 16-byte aligned");
  abs_ctx *nc = nullptr;
  HIPCHK(nc, launch_copy_probe(src_dev, dst_dev, bytes, static_cast<hipStream_t>(hip_stream)));
  return ABS_OK;
} catch (...) { return on_exception(); }

// ---- the mean buffer of abs_average_bf16_static -----------------------------------------------
// Device memory that belongs to the library's code object: every GPU the library runs on holds its own copy
// at its own address until the process ends.  Host code never uses the array's name as an address; it asks the
// runtime for the address once per device and passes that pointer to the kernels.
constexpr long long AVG_STATIC_ELEMS = 16LL << 20;            // bf16 values: 32 MiB
static __device__ __align__(256) unsigned char g_avg_mean[AVG_STATIC_ELEMS * 2];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_avg_mu;
void *g_avg_mean_ptr[MAX_DEVICES] = {nullptr};

// Address of the current device's copy of g_avg_mean (resolved on the first call on that device).
abs_status avg_static_ptr(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(ABS_EHIP, std::string("hipGetDevice: ") + hipGetErrorString(e));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(ABS_EUNSUPPORTED, "device ordinal beyond the static-scratch table");
  std::lock_guard<std::mutex> lk(g_avg_mu);
  if (!g_avg_mean_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_avg_mean));
    if (e != hipSuccess || !ptr) return fail(ABS_EHIP, std::string("hipGetSymbolAddress: ") + hipGetErrorString(e));
    g_avg_mean_ptr[dev] = ptr;
  }
  *out = g_avg_mean_ptr[dev];
  return ABS_OK;
}
}  // namespace

abs_status abs_average_bf16_static(void *params_dev, int M, int64_t n, void *hip_stream) try {
  if (!params_dev) return fail(ABS_EINVAL, "params_dev is NULL");
  if (M < 1 || n < 8 || (n % 8)) return fail(ABS_EINVAL, "M < 1 or n not a positive multiple of 8");
  if (n > AVG_STATIC_ELEMS) return fail(ABS_EINVAL, "n exceeds the static mean buffer (16 Mi bf16 values per replica)");
  if (reinterpret_cast<uintptr_t>(params_dev) & 15) return fail(ABS_EINVAL, "params_dev must be 16-byte aligned");
  void *mean = nullptr;
  abs_status st = avg_static_ptr(&mean);
  if (st != ABS_OK) return st;
  abs_ctx *nc = nullptr;
  // the first pass writes mean[0, n) before the second reads it: nothing of the last call's contents is used
  HIPCHK(nc, launch_average_bf16(static_cast<bf16_t *>(params_dev), static_cast<bf16_t *>(mean), M, n,
                                 static_cast<hipStream_t>(hip_stream)));
  return ABS_OK;
} catch (...) { return on_exception(); }

abs_status abs_average_bf16(void *params_dev, int M, int64_t n, void *scratch_dev, void *hip_stream) try {
  if (!params_dev) return fail(ABS_EINVAL, "params_dev is NULL");
  if (M < 1 || n < 8 || (n % 8)) return fail(ABS_EINVAL, "M < 1 or n not a positive multiple of 8");
  if ((reinterpret_cast<uintptr_t>(params_dev) | reinterpret_cast<uintptr_t>(scratch_dev)) & 15)
    return fail(ABS_EINVAL, "params_dev and scratch_dev must be 16-byte aligned");
  abs_ctx *nc = nullptr;
  HIPCHK(nc, launch_average_bf16(static_cast<bf16_t *>(params_dev), static_cast<bf16_t *>(scratch_dev), M, n,
                                 static_cast<hipStream_t>(hip_stream)));
  return ABS_OK;
} catch (...) { return on_exception(); }

}  // extern "C"
