// Host side of the Accordion hot-path library: configuration checks, workspace layout,
// tile tables, the step state machine and the kernel launches.  The C ABI is declared and
// documented in include/accordion.h.
#include "../../include/accordion.h"

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "acc_common.h"
#include "acc_powersgd.h"
#include "acc_regime.h"
#include "acc_topk.h"
#include "acc_batch.h"

using namespace acc;

namespace {

thread_local char g_init_error[256] = "no error";

inline int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }

struct Region { int64_t off = 0, bytes = 0; };

// Everything that follows from the configuration alone (no GPU needed).
struct Plan {
  std::vector<LayerDev> layers;
  std::vector<FlatTile> ftiles;
  std::vector<MatTile> mtiles, qmtiles;
  std::vector<QTile> qtiles;
  std::vector<PTile> ptiles;
  std::vector<int32_t> vectiles;
  std::vector<int32_t> matlayers;
  int32_t rmax = 0;
  int64_t N = 0, e_stride = 0;
  int64_t q_total = 0;   // floats of Q in the caller's layout (rows of rmax floats)
  int64_t q_dev = 0;     // floats of Q on the device: every row padded to kMaxRank floats
  int64_t p_total = 0, ppart_stride = 0, qpart_stride = 0, vec_total = 0;
  int64_t pay_stride = 0, q_stride = 0;
  int64_t n_t2slots = 0;    // TopK: slots of level-2 counts per worker (one per kT2Group tiles of a layer)
  bool pick3_big = false;   // TopK: some layer has more quarters than the small last pick kernel takes
  // workspace regions
  Region r_layers, r_ftiles, r_mtiles, r_qmtiles, r_qtiles, r_ptiles, r_vectiles, r_matlayers;
  Region r_level, r_norm_old, r_norm_prev, r_norm_curr, r_has_old, r_rank_used, r_words;
  Region r_A, r_e, r_norm_part, r_norm_part_m, r_afresh, r_sq_part, r_bstate;
  int64_t n_model = 0;   // elements that belong to a layer
  Region r_Q, r_Phat, r_Pwork, r_Ppart, r_Qpart, r_vecmean, r_pending;
  Region r_hist1, r_t2, r_qlist, r_sel, r_hist2m, r_lflag, r_b1hist, r_guess, r_qinfo, r_candval, r_candidx, r_gtq, r_eqq, r_gtpre, r_eqpre, r_payidx, r_payval, r_overlap, r_tpending;
  int64_t total_bytes = 0;
};

int fail(char* buf, int code, const char* msg) {
  std::snprintf(buf, 256, "%s", msg);
  return code;
}

int make_plan(const acc_config* c, Plan& p, char* err) {
  if (!c) return fail(err, ACC_EINVAL, "config is NULL");
  if (c->method != ACC_POWERSGD && c->method != ACC_TOPK && c->method != ACC_BATCH)
    return fail(err, ACC_EINVAL, "unknown method");
  if (c->n_layers <= 0 || c->n_layers > (1 << 20)) return fail(err, ACC_EINVAL, "n_layers out of range");
  if (!c->layers) return fail(err, ACC_EINVAL, "layers is NULL");
  if (c->n_workers < 1 || c->n_workers > ACC_MAX_WORKERS) return fail(err, ACC_EINVAL, "n_workers out of range");
  if (c->n_params <= 0 || c->n_params > (int64_t(1) << 40)) return fail(err, ACC_EINVAL, "n_params out of range");
  if (!(c->eta >= 0.0f) || !std::isfinite(c->eta)) return fail(err, ACC_EINVAL, "eta must be finite and >= 0");
  if (c->initial_level != 0 && c->initial_level != 1) return fail(err, ACC_EINVAL, "initial_level must be 0 or 1");
  if (c->detector != ACC_DETECT_NORM && c->detector != ACC_DETECT_MSDR) return fail(err, ACC_EINVAL, "unknown detector");
  if (c->detector == ACC_DETECT_MSDR && c->method == ACC_BATCH)
    return fail(err, ACC_EINVAL, "the MSDR detector is not available in batch-size mode");
  if (c->detector == ACC_DETECT_MSDR && !(c->eta < 1.0f)) return fail(err, ACC_EINVAL, "MSDR detector: eta must be below 1");
  if (c->method == ACC_POWERSGD) {
    if (c->rank_crit < 1 || c->rank_crit > ACC_MAX_RANK || c->rank_noncrit < 1 || c->rank_noncrit > ACC_MAX_RANK)
      return fail(err, ACC_EINVAL, "rank out of [1, ACC_MAX_RANK]");
  } else if (c->method == ACC_BATCH) {
    if (c->batch_multiplier < 1 || c->batch_multiplier > ACC_MAX_BATCH_MULTIPLIER)
      return fail(err, ACC_EINVAL, "batch_multiplier out of [1, ACC_MAX_BATCH_MULTIPLIER]");
    if (c->batch_monotone != 0 && c->batch_monotone != 1) return fail(err, ACC_EINVAL, "batch_monotone must be 0 or 1");
  } else {
    if (c->k_den < 1 || c->k_num_crit < 1 || c->k_num_noncrit < 1 || c->k_num_crit > c->k_den ||
        c->k_num_noncrit > c->k_den)
      return fail(err, ACC_EINVAL, "k fraction out of (0, 1]");
  }
  const int nl = c->n_layers;
  // layers: positive shapes, inside the flat buffer, pairwise disjoint
  std::vector<std::pair<int64_t, int64_t>> spans;
  spans.reserve(nl);
  for (int i = 0; i < nl; ++i) {
    const acc_layer& l = c->layers[i];
    if (l.rows < 1 || l.cols < 1) return fail(err, ACC_EINVAL, "layer with rows < 1 or cols < 1");
    if (l.is_matrix != 0 && l.is_matrix != 1) return fail(err, ACC_EINVAL, "is_matrix must be 0 or 1");
    const int64_t n = (int64_t)l.rows * l.cols;
    if (n >= (int64_t(1) << 31)) return fail(err, ACC_EINVAL, "layer has 2^31 or more elements");
    if (l.offset < 0 || l.offset + n > c->n_params) return fail(err, ACC_EINVAL, "layer outside [0, n_params)");
    spans.emplace_back(l.offset, l.offset + n);
  }
  std::sort(spans.begin(), spans.end());
  for (size_t i = 1; i < spans.size(); ++i)
    if (spans[i].first < spans[i - 1].second) return fail(err, ACC_EINVAL, "layers overlap");

  p.N = c->n_params;
  p.e_stride = align_up(p.N, 64);
  p.rmax = (c->method == ACC_POWERSGD) ? std::max(c->rank_crit, c->rank_noncrit) : 0;
  p.layers.resize(nl);
  int64_t ntile = 0;
  for (int i = 0; i < nl; ++i) {
    const acc_layer& l = c->layers[i];
    LayerDev& d = p.layers[i];
    std::memset(&d, 0, sizeof(d));
    const int64_t n = (int64_t)l.rows * l.cols;
    d.offset = l.offset;
    d.rows = l.rows;
    d.cols = l.cols;
    d.is_matrix = (c->method == ACC_POWERSGD && l.is_matrix) ? 1 : 0;
    d.vec4 = (l.offset % 4 == 0 && l.cols % 4 == 0) ? 1 : 0;
    d.tile0 = (int32_t)ntile;
    d.ntiles = (int32_t)((n + kTile - 1) / kTile);
    d.qoff = 4 * (int64_t)d.tile0 + i;
    for (int t = 0; t < d.ntiles; ++t) {
      FlatTile ft;
      ft.layer = i;
      ft.start = t * kTile;
      ft.count = (int32_t)std::min<int64_t>(kTile, n - (int64_t)t * kTile);
      ft.qslot0 = (int32_t)(d.qoff + 4 * (int64_t)t);
      p.ftiles.push_back(ft);
    }
    ntile += d.ntiles;
    if (4 * (int64_t)d.ntiles > kLdsQuarters) p.pick3_big = true;
    d.t2slot0 = (int32_t)p.n_t2slots;
    p.n_t2slots += (d.ntiles + kT2Group - 1) / kT2Group;
    p.n_model += n;
    if (ntile > (int64_t(1) << 30)) return fail(err, ACC_EINVAL, "too many tiles");
    if (c->method == ACC_POWERSGD) {
      if (d.is_matrix) {
        const int cap = std::min(l.rows, l.cols);
        d.rank[0] = std::max(1, std::min(c->rank_noncrit, cap));
        d.rank[1] = std::max(1, std::min(c->rank_crit, cap));
        d.n_colchunks = (l.cols + kMatCols - 1) / kMatCols;
        d.mt0 = (int32_t)p.mtiles.size();
        const int n_rb = (l.rows + kMatRows - 1) / kMatRows;
        d.n_rowblocks = (l.rows + kQRows - 1) / kQRows;
        d.q_off = p.q_dev;
        p.q_total += (int64_t)l.cols * p.rmax;
        p.q_dev += (int64_t)l.cols * kMaxRank;
        d.p_off = p.p_total;
        p.p_total += (int64_t)l.rows * p.rmax;
        d.ppart_off = p.ppart_stride;
        p.ppart_stride += (int64_t)d.n_colchunks * l.rows * p.rmax;
        d.qpart_off = p.qpart_stride;
        p.qpart_stride += (int64_t)d.n_rowblocks * l.cols * p.rmax;
        p.matlayers.push_back(i);
        for (int rb = 0; rb < d.n_rowblocks; ++rb)
          for (int cc = 0; cc < d.n_colchunks; ++cc) p.qmtiles.push_back(MatTile{i, rb * kQRows, cc * kMatCols, 0});
        for (int rb = 0; rb < n_rb; ++rb)
          for (int cc = 0; cc < d.n_colchunks; ++cc) {
            MatTile mt;
            mt.layer = i;
            mt.row0 = rb * kMatRows;
            mt.col0 = cc * kMatCols;
            mt.pad = 0;
            p.mtiles.push_back(mt);
          }
        for (int r0 = 0; r0 < l.rows; r0 += kPmeanRows) p.ptiles.push_back(PTile{i, r0});
        for (int cc = 0; cc < d.n_colchunks; ++cc) {
          QTile qt;
          qt.layer = i;
          qt.col0 = cc * kMatCols;
          p.qtiles.push_back(qt);
        }
      } else {
        d.vec_off = p.vec_total;
        p.vec_total += n;
        for (int t = 0; t < d.ntiles; ++t) p.vectiles.push_back(d.tile0 + t);
      }
    } else if (c->method == ACC_TOPK) {
      auto kof = [&](int num) {
        const int64_t k = ((int64_t)n * num + c->k_den - 1) / c->k_den;
        return (int32_t)std::max<int64_t>(1, std::min<int64_t>(n, k));
      };
      d.k[0] = kof(c->k_num_noncrit);
      d.k[1] = kof(c->k_num_crit);
      d.pay_off = p.pay_stride;
      p.pay_stride += std::max(d.k[0], d.k[1]);
    }
  }
  p.q_stride = 4 * ntile + nl;

  // workspace layout, 256-byte aligned regions
  int64_t off = 0;
  auto reg = [&](Region& r, int64_t bytes) {
    r.off = off;
    r.bytes = bytes;
    off = align_up(off + std::max<int64_t>(bytes, 0), 256);
  };
  const int64_t W = c->n_workers;
  reg(p.r_layers, (int64_t)sizeof(LayerDev) * nl);
  reg(p.r_ftiles, (int64_t)sizeof(FlatTile) * (int64_t)p.ftiles.size());
  reg(p.r_mtiles, (int64_t)sizeof(MatTile) * (int64_t)p.mtiles.size());
  reg(p.r_qmtiles, (int64_t)sizeof(MatTile) * (int64_t)p.qmtiles.size());
  reg(p.r_qtiles, (int64_t)sizeof(QTile) * (int64_t)p.qtiles.size());
  reg(p.r_ptiles, (int64_t)sizeof(PTile) * (int64_t)p.ptiles.size());
  reg(p.r_vectiles, 4 * (int64_t)p.vectiles.size());
  reg(p.r_matlayers, 4 * (int64_t)p.matlayers.size());
  reg(p.r_level, 4 * (int64_t)nl);
  reg(p.r_norm_old, 4 * (int64_t)nl);
  reg(p.r_norm_prev, 4 * (int64_t)nl);
  reg(p.r_norm_curr, 4 * (int64_t)nl);
  reg(p.r_has_old, 4 * (int64_t)nl);
  reg(p.r_rank_used, 4 * (int64_t)nl);
  reg(p.r_words, 8 * 6);
  reg(p.r_A, 4 * p.e_stride);
  reg(p.r_e, 4 * p.e_stride * W);
  reg(p.r_norm_part, 8 * ntile);
  reg(p.r_norm_part_m, 8 * (int64_t)p.mtiles.size());
  reg(p.r_afresh, 4);
  reg(p.r_sq_part, c->detector == ACC_DETECT_MSDR ? 8 * ntile : 0);
  reg(p.r_bstate, 4 * 8);
  if (c->method == ACC_POWERSGD) {
    reg(p.r_Q, 4 * p.q_dev);
    reg(p.r_Phat, 4 * p.p_total);
    reg(p.r_Pwork, 8 * p.p_total);
    reg(p.r_Ppart, 8 * p.ppart_stride * W);
    reg(p.r_Qpart, 8 * p.qpart_stride * W);
    reg(p.r_vecmean, 4 * p.vec_total);
    reg(p.r_pending, 4);
  } else if (c->method == ACC_TOPK) {
    reg(p.r_hist1, 4 * (int64_t)kHistBins * nl * W);
    reg(p.r_t2, 4 * (int64_t)kSub2 * p.n_t2slots * W);
    reg(p.r_qlist, 4 * (int64_t)kQListCap * p.q_stride * W);
    reg(p.r_sel, (int64_t)sizeof(SelState) * nl * W);
    reg(p.r_hist2m, 4 * (int64_t)kL2Bins * nl * W);
    reg(p.r_lflag, 4 * (int64_t)nl);
    reg(p.r_b1hist, 8 * 2 * (int64_t)nl * W);
    reg(p.r_guess, 4 * 2 * (int64_t)nl * W);
    reg(p.r_qinfo, (int64_t)sizeof(uint4) * p.q_stride * W);
    reg(p.r_candval, 4 * (int64_t)kCandCap * p.q_stride * W);
    reg(p.r_candidx, 2 * (int64_t)kCandCap * p.q_stride * W);
    reg(p.r_gtq, 4 * p.q_stride * W);
    reg(p.r_eqq, 4 * p.q_stride * W);
    reg(p.r_gtpre, 4 * p.q_stride * W);
    reg(p.r_eqpre, 4 * p.q_stride * W);
    reg(p.r_payidx, 4 * p.pay_stride * W);
    reg(p.r_payval, 4 * p.pay_stride * W);
    reg(p.r_overlap, 8 * (int64_t)nl);
    reg(p.r_tpending, 4);
  }
  p.total_bytes = off;
  return ACC_OK;
}

}  // namespace

// Plain streaming copy used to calibrate hardware counters and to measure the copy bandwidth
// the memory system reaches: 256 threads, four 16-byte groups per thread, loads before stores.
constexpr int kProbeQuadsPerThread = 4;
__global__ __launch_bounds__(256) void probe_copy_kernel(float4* __restrict__ dst, const float4* __restrict__ src,
                                                         int64_t nquads) {
  const int64_t base = (int64_t)blockIdx.x * (256 * kProbeQuadsPerThread) + threadIdx.x;
  float4 v[kProbeQuadsPerThread];
#pragma unroll
  for (int i = 0; i < kProbeQuadsPerThread; ++i) {
    const int64_t q = base + (int64_t)i * 256;
    if (q < nquads) v[i] = src[q];
  }
#pragma unroll
  for (int i = 0; i < kProbeQuadsPerThread; ++i) {
    const int64_t q = base + (int64_t)i * 256;
    if (q < nquads) dst[q] = v[i];
  }
}

// ---- the workspace of callers that cannot allocate (accordion_init_static) ----------------------
// One array per GPU (every device that loads the library holds its own copy until the process
// ends).  Host code never uses the array's name as an address: the device address is taken once
// per device with hipGetSymbolAddress, that device being current, and kept.
static __device__ __align__(256) unsigned char scratch[ACC_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
struct StaticSlot {
  void* ptr = nullptr;         // device address of `scratch` on this device
  acc_ctx* owner = nullptr;    // the context that uses it now (the last one created on it)
};
StaticSlot g_static[kMaxDevices];
std::mutex g_static_mutex;
}  // namespace

enum Stage {
  ST_psgd_ef_p_kernel = 0, ST_psgd_orth_kernel, ST_psgd_q_kernel, ST_psgd_qmean_kernel,
  ST_psgd_decomp_kernel, ST_psgd_residual_kernel, ST_topk_ef_hist_kernel, ST_topk_pick12_kernel,
  ST_topk_count3_kernel, ST_topk_pick3_kernel,
  ST_topk_compact_kernel, ST_topk_compact_mean_kernel, ST_topk_sparse_mean_kernel,
  ST_norm_partial_kernel, ST_regime_decide_kernel, ST_recount_words_kernel, ST_zero_accum_kernel,
  ST_psgd_decomp_update_kernel, ST_topk_compact_update_kernel, ST_topk_sparse_update_kernel,
  ST_batch_micro_kernel, ST_batch_micro_update_kernel, ST_batch_decide_kernel,
  ST_topk_overlap_kernel, ST_zero_u64_kernel, ST_msdr_sq_kernel, ST_msdr_decide_kernel,
  ST_psgd_clear_pending_kernel, ST_topk_residual_kernel, ST_topk_clear_pending_kernel,
  ST_topk_pick3_big_kernel, ST_psgd_pmean_kernel, ST_norm_refresh_kernel,
  ST_COUNT
};
static_assert(ST_COUNT <= ACC_N_STAGES, "more stages than the header announces");
static const char* const kStageNames[ST_COUNT] = {
  "psgd_ef_p_kernel", "psgd_orth_kernel", "psgd_q_kernel", "psgd_qmean_kernel",
  "psgd_decomp_kernel", "psgd_residual_kernel", "topk_ef_hist_kernel", "topk_pick12_kernel",
  "topk_count3_kernel", "topk_pick3_kernel",
  "topk_compact_kernel", "topk_compact_mean_kernel", "topk_sparse_mean_kernel",
  "norm_partial_kernel", "regime_decide_kernel", "recount_words_kernel", "zero_accum_kernel",
  "psgd_decomp_update_kernel", "topk_compact_update_kernel", "topk_sparse_update_kernel",
  "batch_micro_kernel", "batch_micro_update_kernel", "batch_decide_kernel",
  "topk_overlap_kernel", "zero_u64_kernel", "msdr_sq_kernel", "msdr_decide_kernel",
  "psgd_clear_pending_kernel", "topk_residual_kernel", "topk_clear_pending_kernel",
  "topk_pick3_big_kernel", "psgd_pmean_kernel", "norm_refresh_kernel"};

struct EventPair { hipEvent_t a, b; int stage; };

struct acc_ctx {
  // per-kernel timing
  int profiling = 0;               // 0 off, 1 every kernel, 2 only the fused error-feedback pass, 3 every fourth launch of it
  uint32_t prof_tick = 0;          // launches of that pass seen in mode 3
  std::vector<EventPair> pending, spare;
  double stage_ms[ST_COUNT] = {0};
  long long stage_n[ST_COUNT] = {0};
  acc_config cfg;
  std::vector<acc_layer> layers;
  Plan plan;
  Ws ws;
  char* base = nullptr;
  hipStream_t stream = nullptr;
  int static_dev = -1;             // >= 0: the workspace is the library's static array of that device
  // step state machine
  bool in_step = false;
  uint32_t step_id = 2;            // number of the current step (the device keeps 0 for "never")
  uint32_t p0_mask = 0, p1_mask = 0;
  bool agg0 = false, agg1 = false;
  GradPtrs grads;
  char err[256];
};

namespace {

#define ACC_HIP(ctx, call)                                                              \
  do {                                                                                  \
    hipError_t e_ = (call);                                                             \
    if (e_ != hipSuccess) {                                                             \
      std::snprintf((ctx)->err, 256, "%s failed: %s", #call, hipGetErrorString(e_));    \
      return ACC_EHIP;                                                                  \
    }                                                                                   \
  } while (0)

template <class T>
T* at(acc_ctx* c, const Region& r) { return reinterpret_cast<T*>(c->base + r.off); }

uint32_t all_workers_mask(const acc_ctx* c) {
  return c->cfg.n_workers == 32 ? 0xffffffffu : ((1u << c->cfg.n_workers) - 1u);
}

int check_launch(acc_ctx* c, const char* what) {
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) {
    std::snprintf(c->err, 256, "launch of %s failed: %s", what, hipGetErrorString(e));
    return ACC_EHIP;
  }
  return ACC_OK;
}

// A context on the library's static workspace is usable only while it is the last one created on
// that device's array (a later accordion_init_static cleared and re-planned the memory).
int check_owner(acc_ctx* c) {
  if (c->static_dev < 0) return ACC_OK;
  std::lock_guard<std::mutex> lock(g_static_mutex);
  if (g_static[c->static_dev].owner == c) return ACC_OK;
  return fail(c->err, ACC_ESTATE, "the static workspace of this context was taken over by a later accordion_init_static");
}

#define ACC_USABLE(c)                          \
  do {                                         \
    if (!(c)) return ACC_EINVAL;               \
    const int rc_owner_ = check_owner(c);      \
    if (rc_owner_ != ACC_OK) return rc_owner_; \
  } while (0)

// Fold the finished event pairs into the per-stage totals (synchronises the stream).
int drain_profile(acc_ctx* c) {
  if (c->pending.empty()) return ACC_OK;
  if (hipStreamSynchronize(c->stream) != hipSuccess) return fail(c->err, ACC_EHIP, "hipStreamSynchronize failed");
  for (EventPair& p : c->pending) {
    float ms = 0.f;
    if (hipEventElapsedTime(&ms, p.a, p.b) == hipSuccess) {
      c->stage_ms[p.stage] += ms;
      c->stage_n[p.stage] += 1;
    }
    c->spare.push_back(p);
  }
  c->pending.clear();
  return ACC_OK;
}

bool prof_begin(acc_ctx* c, int stage, EventPair& p) {
  if (!c->profiling) return false;
  if (c->profiling >= 2 && stage != ST_topk_ef_hist_kernel && stage != ST_psgd_ef_p_kernel &&
      stage != ST_batch_micro_kernel && stage != ST_batch_micro_update_kernel)
    return false;
  if (c->profiling == 3 && (c->prof_tick++ & 3u) != 0u) return false;
  if (c->pending.size() >= 8192) drain_profile(c);
  if (!c->spare.empty()) {
    p = c->spare.back();
    c->spare.pop_back();
  } else {
    if (hipEventCreate(&p.a) != hipSuccess) return false;
    if (hipEventCreate(&p.b) != hipSuccess) { (void)hipEventDestroy(p.a); return false; }
  }
  p.stage = stage;
  return true;
}

void prof_end(acc_ctx* c, EventPair& p) { c->pending.push_back(p); }

#define ACC_LAUNCH(ctx, name, grid, block, ...)                              \
  do {                                                                       \
    EventPair ep_;                                                           \
    const bool prof_ = prof_begin(ctx, ST_##name, ep_);                      \
    if (prof_) {                                                             \
      /* the two events take the dispatch's own begin and end timestamps */  \
      hipExtLaunchKernelGGL(name, grid, block, 0, (ctx)->stream, ep_.a, ep_.b, 0, __VA_ARGS__); \
      prof_end(ctx, ep_);                                                    \
    } else {                                                                 \
      hipLaunchKernelGGL(name, grid, block, 0, (ctx)->stream, __VA_ARGS__);  \
    }                                                                        \
    int rc_ = check_launch(ctx, #name);                                      \
    if (rc_ != ACC_OK) return rc_;                                           \
  } while (0)

// --- launches of each stage for workers [w0, w0 + nw) ------------------------------------

// TopK selection of workers [w0, w0 + nw): the fused error-feedback pass, then the per-layer decisions
// (level-1/2 bins, re-staging after a missed guess, level-3/4 counts, threshold and prefixes).
int launch_topk_select(acc_ctx* c, int w0, int nw) {
  const Ws& ws = c->ws;
  ACC_LAUNCH(c, topk_ef_hist_kernel, dim3(ws.n_ftiles, nw), dim3(256), ws, c->grads, w0);
  ACC_LAUNCH(c, topk_pick12_kernel, dim3(ws.L, nw), dim3(kPickThreads), ws, w0);
  ACC_LAUNCH(c, topk_count3_kernel, dim3((ws.n_ftiles + kCountTiles - 1) / kCountTiles, nw), dim3(256), ws, w0);
  ACC_LAUNCH(c, topk_pick3_kernel, dim3(ws.L, nw), dim3(kPickThreads), ws, w0, c->step_id);
  if (c->plan.pick3_big) ACC_LAUNCH(c, topk_pick3_big_kernel, dim3(ws.L, nw), dim3(kPickThreads), ws, w0, c->step_id);
  return ACC_OK;
}

// The MSDR detector also needs the squared norm of worker 0's raw gradient of every step.
int launch_detector_feed(acc_ctx* c, int w0) {
  const Ws& ws = c->ws;
  if (c->cfg.detector == ACC_DETECT_MSDR && w0 == 0)
    ACC_LAUNCH(c, msdr_sq_kernel, dim3(ws.n_ftiles), dim3(256), ws, c->grads.p[0]);
  return ACC_OK;
}

int launch_phase0(acc_ctx* c, int w0, int nw) {
  const Ws& ws = c->ws;
  {
    const int rc = launch_detector_feed(c, w0);
    if (rc != ACC_OK) return rc;
  }
  if (c->cfg.method == ACC_POWERSGD) {
    const int gx = ws.n_mtiles + (w0 == 0 ? ws.n_vectiles : 0);
    if (gx > 0) ACC_LAUNCH(c, psgd_ef_p_kernel, dim3(gx, nw), dim3(256), ws, c->grads, w0);
  } else {
    const int rc = launch_topk_select(c, w0, nw);
    if (rc != ACC_OK) return rc;
    ACC_LAUNCH(c, topk_compact_kernel, dim3(ws.n_ftiles, nw), dim3(256), ws, w0);
  }
  return ACC_OK;
}

int launch_agg0(acc_ctx* c) {
  const Ws& ws = c->ws;
  if (c->cfg.method == ACC_POWERSGD) {
    if (ws.n_ptiles > 0) ACC_LAUNCH(c, psgd_pmean_kernel, dim3(ws.n_ptiles), dim3(256), ws);
    const int gx = ws.n_mat + ws.n_vectiles;
    if (gx > 0) ACC_LAUNCH(c, psgd_orth_kernel, dim3(gx), dim3(kOrthThreads), ws, c->grads);
  }
  return ACC_OK;
}

int launch_phase1(acc_ctx* c, int w0, int nw) {
  const Ws& ws = c->ws;
  if (ws.n_qmtiles > 0) ACC_LAUNCH(c, psgd_q_kernel, dim3(ws.n_qmtiles, nw), dim3(256), ws, w0);
  return ACC_OK;
}

int launch_agg1(acc_ctx* c) {
  const Ws& ws = c->ws;
  if (ws.n_qtiles > 0) ACC_LAUNCH(c, psgd_qmean_kernel, dim3(ws.n_qtiles), dim3(256), ws);
  return ACC_OK;
}

bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Weights and velocity are read and written by every step, like the error memory.  Where both
// fit the last-level cache together they are accessed plainly (ResNet-18 shapes at W = 1: the
// fused TopK update is 11 us faster); where they do not, streaming them keeps the error memory
// resident for the next pass (W = 4: 2 us).
int32_t stream_wv(const acc_ctx* c) {
  const int64_t resident = 4 * c->plan.e_stride * (int64_t)c->cfg.n_workers + 8 * c->plan.N;
  return resident > (192ll << 20) ? 1 : 0;
}

Sink sink_out(float* out) { return Sink{out, nullptr, nullptr, 0.f, 0.f, 0.f, 0}; }

// sink.wt != nullptr: the optimizer step consumes the averaged gradient instead of a store.
int launch_decompress(acc_ctx* c, const Sink& sink) {
  const Ws& ws = c->ws;
  if (c->cfg.method == ACC_POWERSGD) {
    const dim3 grid(ws.n_mtiles + ws.n_vectiles);
    if (sink.wt) ACC_LAUNCH(c, psgd_decomp_update_kernel, grid, dim3(256), ws, sink);
    else ACC_LAUNCH(c, psgd_decomp_kernel, grid, dim3(256), ws, sink);
  } else {
    if (sink.wt) ACC_LAUNCH(c, topk_sparse_update_kernel, dim3(ws.n_ftiles), dim3(256), ws, sink);
    else ACC_LAUNCH(c, topk_sparse_mean_kernel, dim3(ws.n_ftiles), dim3(256), ws, sink);
  }
  return ACC_OK;
}

const char* const kBatchCallByCall =
    "batch-size mode has no call-by-call sequence: use accordion_step_all / accordion_step_all_update";

// One micro-step of the batch-size mode for all workers (c->grads is set).
int launch_batch_micro(acc_ctx* c, const Sink& sink) {
  const Ws& ws = c->ws;
  const uint32_t parity = c->step_id & 1u;
  if (sink.wt) ACC_LAUNCH(c, batch_micro_update_kernel, dim3(ws.n_ftiles), dim3(256), ws, c->grads, sink, parity);
  else ACC_LAUNCH(c, batch_micro_kernel, dim3(ws.n_ftiles), dim3(256), ws, c->grads, sink, parity);
  return ACC_OK;
}

int launch_topk_compact_mean(acc_ctx* c, const Sink& sink) {
  const Ws& ws = c->ws;
  if (sink.wt) ACC_LAUNCH(c, topk_compact_update_kernel, dim3(ws.n_ftiles * kMeanSplit), dim3(kMeanWaves * kWave), ws, sink);
  else ACC_LAUNCH(c, topk_compact_mean_kernel, dim3(ws.n_ftiles * kMeanSplit), dim3(kMeanWaves * kWave), ws, sink);
  return ACC_OK;
}

// Arguments of the optimizer step: finite hyper-parameters, two distinct aligned device buffers.
int check_sgd(acc_ctx* c, const float* w, const float* v, float lr, float mu, float wd) {
  if (!w || !v) return fail(c->err, ACC_EINVAL, "weights_dev or velocity_dev is NULL");
  if (misaligned(w) || misaligned(v)) return fail(c->err, ACC_EINVAL, "weights_dev / velocity_dev is not 16-byte aligned");
  if (w == v) return fail(c->err, ACC_EINVAL, "weights_dev and velocity_dev are the same buffer");
  if (!(std::isfinite(lr) && std::isfinite(mu) && std::isfinite(wd)) || lr < 0.f || mu < 0.f || wd < 0.f)
    return fail(c->err, ACC_EINVAL, "lr, momentum and weight_decay must be finite and not negative");
  return ACC_OK;
}

// Make the error memory explicit: e_w = Delta_w - D for the workers whose residual is pending.
int materialise(acc_ctx* c) {
  const Ws& ws = c->ws;
  if (c->cfg.method == ACC_TOPK) {
    ACC_LAUNCH(c, topk_residual_kernel, dim3(ws.n_ftiles, ws.W), dim3(256), ws);
    ACC_LAUNCH(c, topk_clear_pending_kernel, dim3(1), dim3(64), ws);
    return ACC_OK;
  }
  if (c->cfg.method != ACC_POWERSGD) return ACC_OK;
  if (ws.n_mtiles > 0) ACC_LAUNCH(c, psgd_residual_kernel, dim3(ws.n_mtiles, ws.W), dim3(256), ws);
  ACC_LAUNCH(c, psgd_clear_pending_kernel, dim3(1), dim3(64), ws);
  return ACC_OK;
}

void end_step(acc_ctx* c) {
  c->in_step = false;
  c->step_id += 1;
  c->p0_mask = c->p1_mask = 0;
  c->agg0 = c->agg1 = false;
}

// Q between the caller's layout (every matrix layer's cols x rmax block, layers in order) and the
// device layout (rows padded to kMaxRank floats, so that a row is one aligned 16-byte load).
int copy_q(acc_ctx* c, float* host, bool to_host) {
  const Plan& p = c->plan;
  if (p.q_dev == 0) return ACC_OK;
  std::vector<float> dev((size_t)p.q_dev, 0.f);
  if (to_host) ACC_HIP(c, hipMemcpy(dev.data(), c->ws.Q, 4 * dev.size(), hipMemcpyDeviceToHost));
  size_t hp = 0;
  for (const int li : p.matlayers) {
    const LayerDev& L = p.layers[(size_t)li];
    for (int j = 0; j < L.cols; ++j)
      for (int k = 0; k < p.rmax; ++k) {
        float& d = dev[(size_t)L.q_off + (size_t)j * kMaxRank + k];
        if (to_host) host[hp] = d; else d = host[hp];
        ++hp;
      }
  }
  if (!to_host) ACC_HIP(c, hipMemcpy(c->ws.Q, dev.data(), 4 * dev.size(), hipMemcpyHostToDevice));
  return ACC_OK;
}

size_t state_bytes_of(const acc_ctx* c) {
  const Plan& p = c->plan;
  const size_t L = (size_t)c->cfg.n_layers;
  return 4 * ((size_t)p.N * (size_t)(c->cfg.n_workers + 1) + (size_t)p.q_total + 3 * L +
              (c->cfg.method == ACC_BATCH ? 1u : 0u));
}

}  // namespace

extern "C" {

int32_t accordion_workspace_bytes(const acc_config* cfg, size_t* out_bytes) {
  if (!out_bytes) return fail(g_init_error, ACC_EINVAL, "out_bytes is NULL");
  Plan p;
  const int rc = make_plan(cfg, p, g_init_error);
  if (rc != ACC_OK) return rc;
  *out_bytes = (size_t)p.total_bytes;
  return ACC_OK;
}

static int32_t init_common(const acc_config* cfg, void* workspace_dev, size_t workspace_bytes,
                           const float* q_init_host, void* hip_stream, acc_ctx** out, const char* too_small) {
  if (!out) return fail(g_init_error, ACC_EINVAL, "out is NULL");
  *out = nullptr;
  acc_ctx* c = new (std::nothrow) acc_ctx();
  if (!c) return fail(g_init_error, ACC_ENOSPACE, "out of host memory");
  auto bail = [&](int rc, const char* msg) {
    if (msg) std::snprintf(g_init_error, 256, "%s", msg);
    else std::snprintf(g_init_error, 256, "%s", c->err);
    delete c;
    return rc;
  };
  int rc = make_plan(cfg, c->plan, g_init_error);
  if (rc != ACC_OK) { delete c; return rc; }
  if (!workspace_dev) return bail(ACC_EINVAL, "workspace is NULL");
  if ((reinterpret_cast<uintptr_t>(workspace_dev) & 255u) != 0) return bail(ACC_EINVAL, "workspace is not 256-byte aligned");
  if (workspace_bytes < (size_t)c->plan.total_bytes) return bail(ACC_ENOSPACE, too_small);
  if (cfg->method == ACC_POWERSGD && c->plan.q_total > 0 && !q_init_host)
    return bail(ACC_EINVAL, "q_init_host is NULL");
  c->cfg = *cfg;
  c->layers.assign(cfg->layers, cfg->layers + cfg->n_layers);
  c->cfg.layers = c->layers.data();
  c->base = static_cast<char*>(workspace_dev);
  c->stream = static_cast<hipStream_t>(hip_stream);
  std::snprintf(c->err, 256, "no error");
  std::memset(&c->grads, 0, sizeof(c->grads));
  Plan& p = c->plan;

  Ws& ws = c->ws;
  std::memset(&ws, 0, sizeof(ws));
  ws.layers = at<LayerDev>(c, p.r_layers);
  ws.ftiles = at<FlatTile>(c, p.r_ftiles);
  ws.mtiles = at<MatTile>(c, p.r_mtiles);
  ws.qmtiles = at<MatTile>(c, p.r_qmtiles);
  ws.qtiles = at<QTile>(c, p.r_qtiles);
  ws.ptiles = at<PTile>(c, p.r_ptiles);
  ws.vectiles = at<int32_t>(c, p.r_vectiles);
  ws.matlayers = at<int32_t>(c, p.r_matlayers);
  ws.level = at<int32_t>(c, p.r_level);
  ws.norm_old = at<float>(c, p.r_norm_old);
  ws.norm_prev = at<float>(c, p.r_norm_prev);
  ws.norm_curr = at<float>(c, p.r_norm_curr);
  ws.has_old = at<int32_t>(c, p.r_has_old);
  ws.rank_used = at<int32_t>(c, p.r_rank_used);
  ws.words = at<unsigned long long>(c, p.r_words);
  ws.stats = ws.words + 4;
  ws.A = at<float>(c, p.r_A);
  ws.e = at<float>(c, p.r_e);
  ws.e_stride = p.e_stride;
  ws.norm_part = at<double>(c, p.r_norm_part);
  ws.norm_part_m = at<double>(c, p.r_norm_part_m);
  ws.a_fresh = at<uint32_t>(c, p.r_afresh);
  ws.sq_part = p.r_sq_part.bytes > 0 ? at<double>(c, p.r_sq_part) : nullptr;
  if (cfg->method == ACC_POWERSGD) {
    ws.Q = at<float>(c, p.r_Q);
    ws.Phat = at<float>(c, p.r_Phat);
    ws.Pwork = at<double>(c, p.r_Pwork);
    ws.Ppart = at<double>(c, p.r_Ppart);
    ws.ppart_stride = p.ppart_stride;
    ws.Qpart = at<double>(c, p.r_Qpart);
    ws.qpart_stride = p.qpart_stride;
    ws.vecmean = at<float>(c, p.r_vecmean);
    ws.pending = at<uint32_t>(c, p.r_pending);
  } else if (cfg->method == ACC_TOPK) {
    ws.hist1 = at<uint32_t>(c, p.r_hist1);
    ws.t2 = at<uint32_t>(c, p.r_t2);
    ws.qlist = at<uint32_t>(c, p.r_qlist);
    ws.sel = at<SelState>(c, p.r_sel);
    ws.hist2m = at<uint32_t>(c, p.r_hist2m);
    ws.lflag = at<uint32_t>(c, p.r_lflag);
    ws.b1hist = at<uint2>(c, p.r_b1hist);
    ws.guess = at<uint32_t>(c, p.r_guess);
    ws.qinfo = at<uint4>(c, p.r_qinfo);
    ws.cand_val = at<uint32_t>(c, p.r_candval);
    ws.cand_idx = at<uint16_t>(c, p.r_candidx);
    ws.gtq = at<uint32_t>(c, p.r_gtq);
    ws.eqq = at<uint32_t>(c, p.r_eqq);
    ws.gtpre = at<uint32_t>(c, p.r_gtpre);
    ws.eqpre = at<uint32_t>(c, p.r_eqpre);
    ws.pay_idx = at<int32_t>(c, p.r_payidx);
    ws.pay_val = at<float>(c, p.r_payval);
    ws.pay_stride = p.pay_stride;
    ws.overlap = at<unsigned long long>(c, p.r_overlap);
    ws.tpending = at<uint32_t>(c, p.r_tpending);
  }
  ws.bstate = at<uint32_t>(c, p.r_bstate);
  ws.bmult = cfg->method == ACC_BATCH ? cfg->batch_multiplier : 1;
  ws.bmono = cfg->method == ACC_BATCH ? cfg->batch_monotone : 0;
  ws.n_model = p.n_model;
  ws.q_stride = p.q_stride;
  ws.n_qslots = p.q_stride * cfg->n_workers;
  ws.N = p.N;
  ws.W = cfg->n_workers;
  ws.L = cfg->n_layers;
  ws.rmax = p.rmax;
  ws.n_ftiles = (int32_t)p.ftiles.size();
  ws.n_t2slots = (int32_t)p.n_t2slots;
  ws.n_mtiles = (int32_t)p.mtiles.size();
  ws.n_qmtiles = (int32_t)p.qmtiles.size();
  ws.n_qtiles = (int32_t)p.qtiles.size();
  ws.n_ptiles = (int32_t)p.ptiles.size();
  ws.n_vectiles = (int32_t)p.vectiles.size();
  ws.n_mat = (int32_t)p.matlayers.size();
  ws.eta = cfg->eta;

  const int nl_ = cfg->n_layers;
  auto init_dev = [&]() -> int {
    ACC_HIP(c, hipMemsetAsync(c->base, 0, (size_t)p.total_bytes, c->stream));
    ACC_HIP(c, hipStreamSynchronize(c->stream));
    auto up = [&](const Region& r, const void* src) -> hipError_t {
      if (r.bytes == 0) return hipSuccess;
      return hipMemcpy(c->base + r.off, src, (size_t)r.bytes, hipMemcpyHostToDevice);
    };
    ACC_HIP(c, up(p.r_layers, p.layers.data()));
    ACC_HIP(c, up(p.r_ftiles, p.ftiles.data()));
    ACC_HIP(c, up(p.r_mtiles, p.mtiles.data()));
    ACC_HIP(c, up(p.r_qmtiles, p.qmtiles.data()));
    ACC_HIP(c, up(p.r_qtiles, p.qtiles.data()));
    ACC_HIP(c, up(p.r_ptiles, p.ptiles.data()));
    ACC_HIP(c, up(p.r_vectiles, p.vectiles.data()));
    ACC_HIP(c, up(p.r_matlayers, p.matlayers.data()));
    std::vector<int32_t> lv((size_t)cfg->n_layers, cfg->initial_level);
    ACC_HIP(c, up(p.r_level, lv.data()));
    if (cfg->method == ACC_POWERSGD && p.q_total > 0) {
      const int rq = copy_q(c, const_cast<float*>(q_init_host), false);
      if (rq != ACC_OK) return rq;
    }
    if (cfg->method == ACC_TOPK) {
      std::vector<uint32_t> none((size_t)2 * nl_ * cfg->n_workers, kNoGuess);
      ACC_HIP(c, up(p.r_guess, none.data()));
    }
    ACC_LAUNCH(c, recount_words_kernel, dim3(1), dim3(256), c->ws, (int)cfg->method, -1);
    ACC_HIP(c, hipStreamSynchronize(c->stream));
    return ACC_OK;
  };
  rc = init_dev();
  if (rc != ACC_OK) return bail(rc, nullptr);
  *out = c;
  return ACC_OK;
}

int32_t accordion_init(const acc_config* cfg, void* workspace_dev, size_t workspace_bytes,
                       const float* q_init_host, void* hip_stream, acc_ctx** out) {
  return init_common(cfg, workspace_dev, workspace_bytes, q_init_host, hip_stream, out, "workspace too small");
}

int32_t accordion_init_static(const acc_config* cfg, const float* q_init_host, void* hip_stream, acc_ctx** out) {
  if (!out) return fail(g_init_error, ACC_EINVAL, "out is NULL");
  *out = nullptr;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
    return fail(g_init_error, ACC_EHIP, "hipGetDevice failed (or a device number beyond the library's table)");
  std::lock_guard<std::mutex> lock(g_static_mutex);
  StaticSlot& slot = g_static[dev];
  if (!slot.ptr) {
    void* p = nullptr;
    const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !p) {
      std::snprintf(g_init_error, 256, "hipGetSymbolAddress(scratch) failed: %s", hipGetErrorString(e));
      return ACC_EHIP;
    }
    slot.ptr = p;
  }
  const int32_t rc = init_common(cfg, slot.ptr, (size_t)ACC_STATIC_WORKSPACE_BYTES, q_init_host, hip_stream, out,
                                 "configuration needs more than ACC_STATIC_WORKSPACE_BYTES of workspace: "
                                 "use accordion_init with a caller-owned workspace");
  if (rc != ACC_OK) return rc;
  (*out)->static_dev = dev;
  slot.owner = *out;                                       // an earlier context on this array is now stale
  return ACC_OK;
}

int32_t accordion_destroy(acc_ctx* ctx) {
  if (!ctx) return ACC_EINVAL;
  if (ctx->static_dev >= 0) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static[ctx->static_dev].owner == ctx) g_static[ctx->static_dev].owner = nullptr;
  }
  (void)drain_profile(ctx);
  for (EventPair& p : ctx->spare) {
    (void)hipEventDestroy(p.a);
    (void)hipEventDestroy(p.b);
  }
  delete ctx;
  return ACC_OK;
}

const char* accordion_last_error(const acc_ctx* ctx) { return ctx ? ctx->err : g_init_error; }

int32_t accordion_compress_step(acc_ctx* c, int32_t worker, const float* grad_dev, int32_t phase) {
  ACC_USABLE(c);
  if (c->cfg.method == ACC_BATCH) return fail(c->err, ACC_EINVAL, kBatchCallByCall);
  if (worker < 0 || worker >= c->cfg.n_workers) return fail(c->err, ACC_EINVAL, "worker out of range");
  const uint32_t bit = 1u << worker;
  if (phase == 0) {
    if (!grad_dev) return fail(c->err, ACC_EINVAL, "grad_dev is NULL");
    if (misaligned(grad_dev)) return fail(c->err, ACC_EINVAL, "grad_dev is not 16-byte aligned");
    if (c->agg0) return fail(c->err, ACC_ESTATE, "phase 0 after aggregate(0); finish the step with decompress first");
    if (c->p0_mask & bit) return fail(c->err, ACC_ESTATE, "worker already compressed in this step");
    c->grads.p[worker] = grad_dev;
    const int rc = launch_phase0(c, worker, 1);
    if (rc != ACC_OK) return rc;
    c->in_step = true;
    c->p0_mask |= bit;
    return ACC_OK;
  }
  if (phase == 1) {
    if (c->cfg.method != ACC_POWERSGD) return fail(c->err, ACC_EINVAL, "phase 1 exists for PowerSGD only");
    if (!c->agg0 || c->agg1) return fail(c->err, ACC_ESTATE, "phase 1 needs aggregate(0) first and comes before aggregate(1)");
    if (c->p1_mask & bit) return fail(c->err, ACC_ESTATE, "worker already did phase 1 in this step");
    const int rc = launch_phase1(c, worker, 1);
    if (rc != ACC_OK) return rc;
    c->p1_mask |= bit;
    return ACC_OK;
  }
  return fail(c->err, ACC_EINVAL, "phase must be 0 or 1");
}

int32_t accordion_aggregate(acc_ctx* c, int32_t phase) {
  ACC_USABLE(c);
  if (c->cfg.method == ACC_BATCH) return fail(c->err, ACC_EINVAL, kBatchCallByCall);
  if (phase == 0) {
    if (c->agg0) return fail(c->err, ACC_ESTATE, "aggregate(0) already done");
    if (c->p0_mask != all_workers_mask(c)) return fail(c->err, ACC_ESTATE, "aggregate(0) needs phase 0 of every worker");
    const int rc = launch_agg0(c);
    if (rc != ACC_OK) return rc;
    c->agg0 = true;
    return ACC_OK;
  }
  if (phase == 1) {
    if (c->cfg.method != ACC_POWERSGD) return fail(c->err, ACC_EINVAL, "phase 1 exists for PowerSGD only");
    if (!c->agg0 || c->agg1) return fail(c->err, ACC_ESTATE, "aggregate(1) out of order");
    if (c->p1_mask != all_workers_mask(c)) return fail(c->err, ACC_ESTATE, "aggregate(1) needs phase 1 of every worker");
    const int rc = launch_agg1(c);
    if (rc != ACC_OK) return rc;
    c->agg1 = true;
    return ACC_OK;
  }
  return fail(c->err, ACC_EINVAL, "phase must be 0 or 1");
}

static int32_t decompress_into(acc_ctx* c, const Sink& sink) {
  if (c->cfg.method == ACC_BATCH) return fail(c->err, ACC_EINVAL, kBatchCallByCall);
  if (c->cfg.method == ACC_POWERSGD ? !c->agg1 : !c->agg0)
    return fail(c->err, ACC_ESTATE, "decompress before the aggregation of this step is complete");
  const int rc = launch_decompress(c, sink);
  if (rc != ACC_OK) return rc;
  end_step(c);
  return ACC_OK;
}

int32_t accordion_decompress(acc_ctx* c, float* out_dev) {
  ACC_USABLE(c);
  if (!out_dev) return fail(c->err, ACC_EINVAL, "out_dev is NULL");
  if (misaligned(out_dev)) return fail(c->err, ACC_EINVAL, "out_dev is not 16-byte aligned");
  return decompress_into(c, sink_out(out_dev));
}

int32_t accordion_decompress_update(acc_ctx* c, float* weights_dev, float* velocity_dev, float lr,
                                    float momentum, float weight_decay) {
  ACC_USABLE(c);
  const int rc = check_sgd(c, weights_dev, velocity_dev, lr, momentum, weight_decay);
  if (rc != ACC_OK) return rc;
  return decompress_into(c, Sink{nullptr, weights_dev, velocity_dev, lr, momentum, weight_decay, stream_wv(c)});
}

static int32_t step_all_into(acc_ctx* c, const float* const* grads_host_array, const Sink& sink) {
  if (!grads_host_array) return fail(c->err, ACC_EINVAL, "grads_host_array is NULL");
  if (c->in_step) return fail(c->err, ACC_ESTATE, "a call-by-call step is in flight");
  const int W = c->cfg.n_workers;
  for (int w = 0; w < W; ++w) {
    if (!grads_host_array[w]) return fail(c->err, ACC_EINVAL, "a gradient pointer is NULL");
    if (misaligned(grads_host_array[w])) return fail(c->err, ACC_EINVAL, "a gradient pointer is not 16-byte aligned");
  }
  for (int w = 0; w < W; ++w) c->grads.p[w] = grads_host_array[w];
  int rc;
  if (c->cfg.method == ACC_BATCH) {
    rc = launch_batch_micro(c, sink);
  } else if (c->cfg.method == ACC_POWERSGD) {
    rc = launch_phase0(c, 0, W);
    if (rc == ACC_OK) rc = launch_agg0(c);
    if (rc == ACC_OK) rc = launch_phase1(c, 0, W);
    if (rc == ACC_OK) rc = launch_agg1(c);
    if (rc == ACC_OK) rc = launch_decompress(c, sink);
  } else {
    // the compaction of all workers and the mean of their kept values share one pass over Delta
    rc = launch_detector_feed(c, 0);
    if (rc == ACC_OK) rc = launch_topk_select(c, 0, W);
    if (rc == ACC_OK) rc = launch_topk_compact_mean(c, sink);
  }
  end_step(c);
  return rc;
}

int32_t accordion_step_all(acc_ctx* c, const float* const* grads_host_array, float* out_dev) {
  ACC_USABLE(c);
  if (!out_dev) return fail(c->err, ACC_EINVAL, "out_dev is NULL");
  if (misaligned(out_dev)) return fail(c->err, ACC_EINVAL, "out_dev is not 16-byte aligned");
  return step_all_into(c, grads_host_array, sink_out(out_dev));
}

int32_t accordion_step_all_update(acc_ctx* c, const float* const* grads_host_array, float* weights_dev,
                                  float* velocity_dev, float lr, float momentum, float weight_decay) {
  ACC_USABLE(c);
  const int rc = check_sgd(c, weights_dev, velocity_dev, lr, momentum, weight_decay);
  if (rc != ACC_OK) return rc;
  return step_all_into(c, grads_host_array, Sink{nullptr, weights_dev, velocity_dev, lr, momentum, weight_decay, stream_wv(c)});
}

int32_t accordion_set_stream(acc_ctx* c, void* hip_stream) {
  ACC_USABLE(c);
  if (c->in_step) return fail(c->err, ACC_ESTATE, "set_stream inside a step");
  const int rc = drain_profile(c);                           // pending timing events belong to the old stream
  if (rc != ACC_OK) return rc;
  c->stream = static_cast<hipStream_t>(hip_stream);
  return ACC_OK;
}

int32_t accordion_detect_regime(acc_ctx* c, float lr_curr, float lr_next) {
  ACC_USABLE(c);
  if (c->in_step) return fail(c->err, ACC_ESTATE, "detect_regime inside a step");
  const Ws& ws = c->ws;
  if (c->cfg.method == ACC_BATCH) {
    ACC_LAUNCH(c, norm_partial_kernel, dim3(ws.n_ftiles), dim3(256), ws);
    ACC_LAUNCH(c, batch_decide_kernel, dim3(1), dim3(256), ws, lr_curr, lr_next);
    return ACC_OK;
  }
  // the sums of squares of A are kept per tile by the pass that adds the gradient; "A <- 0" is a
  // flag that the counting kernel sets once every layer has been decided
  if (c->cfg.detector == ACC_DETECT_MSDR) ACC_LAUNCH(c, msdr_decide_kernel, dim3(ws.L), dim3(64), ws);
  else ACC_LAUNCH(c, regime_decide_kernel, dim3(ws.L), dim3(64), ws, lr_curr, lr_next);
  ACC_LAUNCH(c, recount_words_kernel, dim3(1), dim3(256), ws, (int)c->cfg.method, 1);
  return ACC_OK;
}

int32_t accordion_flush(acc_ctx* c) {
  ACC_USABLE(c);
  if (c->in_step) return fail(c->err, ACC_ESTATE, "flush inside a step");
  return materialise(c);
}

int32_t accordion_reset_accumulator(acc_ctx* c) {
  ACC_USABLE(c);
  if (c->in_step) return fail(c->err, ACC_ESTATE, "reset_accumulator inside a step");
  ACC_LAUNCH(c, zero_accum_kernel, dim3(c->ws.n_ftiles), dim3(256), c->ws, c->cfg.method == ACC_BATCH ? 1 : 0);
  return ACC_OK;
}

int32_t accordion_get_levels(acc_ctx* c, int32_t* levels_host) {
  ACC_USABLE(c);
  if (!levels_host) return fail(c->err, ACC_EINVAL, "levels_host is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  ACC_HIP(c, hipMemcpy(levels_host, c->ws.level, 4 * (size_t)c->cfg.n_layers, hipMemcpyDeviceToHost));
  return ACC_OK;
}

int32_t accordion_get_norms(acc_ctx* c, float* old_host, float* curr_host) {
  ACC_USABLE(c);
  if (!old_host || !curr_host) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  ACC_HIP(c, hipMemcpy(old_host, c->ws.norm_prev, 4 * (size_t)c->cfg.n_layers, hipMemcpyDeviceToHost));
  ACC_HIP(c, hipMemcpy(curr_host, c->ws.norm_curr, 4 * (size_t)c->cfg.n_layers, hipMemcpyDeviceToHost));
  return ACC_OK;
}

int32_t accordion_get_payload(acc_ctx* c, int32_t worker, int32_t layer, int32_t* idx_host,
                              float* val_host, int64_t capacity, int64_t* count_out) {
  ACC_USABLE(c);
  if (c->cfg.method != ACC_TOPK) return fail(c->err, ACC_EINVAL, "payloads exist for TopK only");
  if (worker < 0 || worker >= c->cfg.n_workers) return fail(c->err, ACC_EINVAL, "worker out of range");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(c->err, ACC_EINVAL, "layer out of range");
  if (!count_out) return fail(c->err, ACC_EINVAL, "count_out is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  SelState s;
  ACC_HIP(c, hipMemcpy(&s, c->ws.sel + (size_t)worker * c->cfg.n_layers + layer, sizeof(s), hipMemcpyDeviceToHost));
  const LayerDev& L = c->plan.layers[layer];
  const int64_t k = std::min<int64_t>(s.k, std::max(L.k[0], L.k[1]));
  *count_out = k;
  if (capacity < k) return fail(c->err, ACC_ENOSPACE, "payload buffers too small");
  if (k == 0) return ACC_OK;
  if (!idx_host || !val_host) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  const size_t o = (size_t)worker * c->plan.pay_stride + L.pay_off;
  ACC_HIP(c, hipMemcpy(val_host, c->ws.pay_val + o, 4 * (size_t)k, hipMemcpyDeviceToHost));
  const uint32_t n = (uint32_t)L.rows * (uint32_t)L.cols;
  const uint32_t nholes = n - (uint32_t)k;
  if (!payload_has_holes(n, (uint32_t)k)) {
    ACC_HIP(c, hipMemcpy(idx_host, c->ws.pay_idx + o, 4 * (size_t)k, hipMemcpyDeviceToHost));
    return ACC_OK;
  }
  // values + holes: the kept indices are the complement of the (ascending) hole list
  std::vector<int32_t> holes(nholes);
  if (nholes > 0)
    ACC_HIP(c, hipMemcpy(holes.data(), c->ws.pay_idx + o, 4 * (size_t)nholes, hipMemcpyDeviceToHost));
  int64_t out_pos = 0;
  uint32_t h = 0;
  for (uint32_t i = 0; i < n; ++i) {
    if (h < nholes && holes[h] == (int32_t)i) { ++h; continue; }
    if (out_pos < k) idx_host[out_pos] = (int32_t)i;
    ++out_pos;
  }
  if (out_pos != k || h != nholes) return fail(c->err, ACC_EHIP, "hole list of the payload is inconsistent");
  return ACC_OK;
}

int32_t accordion_payload_format(const acc_config* cfg, int32_t layer, int32_t level, int32_t* format,
                                 int64_t* kept, int64_t* words) {
  if (!cfg || !format || !kept || !words) return fail(g_init_error, ACC_EINVAL, "NULL argument");
  Plan p;
  const int rc = make_plan(cfg, p, g_init_error);
  if (rc != ACC_OK) return rc;
  if (cfg->method != ACC_TOPK) return fail(g_init_error, ACC_EINVAL, "payload formats exist for TopK only");
  if (layer < 0 || layer >= cfg->n_layers) return fail(g_init_error, ACC_EINVAL, "layer out of range");
  if (level != 0 && level != 1) return fail(g_init_error, ACC_EINVAL, "level must be 0 or 1");
  const LayerDev& L = p.layers[layer];
  const uint32_t n = (uint32_t)L.rows * (uint32_t)L.cols, k = (uint32_t)L.k[level];
  const bool holes = payload_has_holes(n, k);
  *format = holes ? ACC_PAYLOAD_VALUES_HOLES : ACC_PAYLOAD_INDEX_VALUE;
  *kept = k;
  *words = holes ? (int64_t)n : 2 * (int64_t)k;
  return ACC_OK;
}

int32_t accordion_get_factors(acc_ctx* c, int32_t layer, float* p_hat_host, float* q_host, int32_t* rank_out) {
  ACC_USABLE(c);
  if (c->cfg.method != ACC_POWERSGD) return fail(c->err, ACC_EINVAL, "factors exist for PowerSGD only");
  if (layer < 0 || layer >= c->cfg.n_layers) return fail(c->err, ACC_EINVAL, "layer out of range");
  const LayerDev& L = c->plan.layers[layer];
  if (!L.is_matrix) return fail(c->err, ACC_EINVAL, "layer is not a matrix");
  if (!p_hat_host || !q_host || !rank_out) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  int32_t r = 0;
  ACC_HIP(c, hipMemcpy(&r, c->ws.rank_used + layer, 4, hipMemcpyDeviceToHost));
  r = std::max(0, std::min(r, c->plan.rmax));
  *rank_out = r;
  const int rmax = c->plan.rmax;
  std::vector<float> tp((size_t)L.rows * rmax), tq((size_t)L.cols * kMaxRank);
  ACC_HIP(c, hipMemcpy(tp.data(), c->ws.Phat + L.p_off, 4 * tp.size(), hipMemcpyDeviceToHost));
  ACC_HIP(c, hipMemcpy(tq.data(), c->ws.Q + L.q_off, 4 * tq.size(), hipMemcpyDeviceToHost));
  for (int i = 0; i < L.rows; ++i)
    for (int k = 0; k < r; ++k) p_hat_host[(size_t)i * r + k] = tp[(size_t)i * rmax + k];
  for (int j = 0; j < L.cols; ++j)
    for (int k = 0; k < r; ++k) q_host[(size_t)j * r + k] = tq[(size_t)j * kMaxRank + k];
  return ACC_OK;
}

int32_t accordion_payload_words(acc_ctx* c, int64_t* last_step, int64_t* cumulative) {
  ACC_USABLE(c);
  if (!last_step || !cumulative) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  unsigned long long w[3] = {0, 0, 0};
  ACC_HIP(c, hipMemcpy(w, c->ws.words, sizeof(w), hipMemcpyDeviceToHost));
  *last_step = (int64_t)w[1];
  *cumulative = (int64_t)w[2];
  return ACC_OK;
}

int32_t accordion_topk_stats(acc_ctx* c, int64_t* restaged_layers, int64_t* swept_layers) {
  ACC_USABLE(c);
  if (c->cfg.method != ACC_TOPK) return fail(c->err, ACC_EINVAL, "TopK statistics exist for TopK only");
  if (!restaged_layers || !swept_layers) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  unsigned long long s[2] = {0, 0};
  ACC_HIP(c, hipMemcpy(s, c->ws.stats, sizeof(s), hipMemcpyDeviceToHost));
  *restaged_layers = (int64_t)s[0];
  *swept_layers = (int64_t)s[1];
  return ACC_OK;
}

int32_t accordion_topk_overlap(acc_ctx* c, int32_t worker_a, int32_t worker_b, int64_t* common_host,
                               int64_t* kept_host) {
  ACC_USABLE(c);
  if (c->cfg.method != ACC_TOPK) return fail(c->err, ACC_EINVAL, "overlaps exist for TopK only");
  if (worker_a < 0 || worker_a >= c->cfg.n_workers || worker_b < 0 || worker_b >= c->cfg.n_workers)
    return fail(c->err, ACC_EINVAL, "worker out of range");
  if (!common_host || !kept_host) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  if (c->in_step) return fail(c->err, ACC_ESTATE, "overlap inside a step");
  if (c->step_id == 2) return fail(c->err, ACC_ESTATE, "no step has run yet: there are no payloads");
  const Ws& ws = c->ws;
  const int L = ws.L;
  ACC_LAUNCH(c, zero_u64_kernel, dim3((L + 255) / 256), dim3(256), ws.overlap, L);
  ACC_LAUNCH(c, topk_overlap_kernel, dim3(ws.n_ftiles), dim3(256), ws, (int)worker_a, (int)worker_b, ws.overlap);
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  std::vector<unsigned long long> cnt((size_t)L);
  std::vector<SelState> sel((size_t)L);
  ACC_HIP(c, hipMemcpy(cnt.data(), ws.overlap, 8 * (size_t)L, hipMemcpyDeviceToHost));
  ACC_HIP(c, hipMemcpy(sel.data(), ws.sel + (size_t)worker_a * L, sizeof(SelState) * (size_t)L, hipMemcpyDeviceToHost));
  for (int i = 0; i < L; ++i) {
    common_host[i] = (int64_t)cnt[(size_t)i];
    kept_host[i] = (int64_t)sel[(size_t)i].k;
  }
  return ACC_OK;
}

int32_t accordion_batch_status(acc_ctx* c, int32_t* level, int32_t* pending_micro_steps,
                               int32_t* last_batch_micro_steps, int64_t* exchanges, int64_t* micro_steps) {
  ACC_USABLE(c);
  if (c->cfg.method != ACC_BATCH) return fail(c->err, ACC_EINVAL, "batch status exists for the batch-size mode only");
  if (!level || !pending_micro_steps || !last_batch_micro_steps || !exchanges || !micro_steps)
    return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  uint32_t slot[4] = {0, 0, 0, 0};
  unsigned long long s[2] = {0, 0};
  ACC_HIP(c, hipMemcpy(slot, c->ws.bstate + 4 * (c->step_id & 1u), sizeof(slot), hipMemcpyDeviceToHost));
  ACC_HIP(c, hipMemcpy(s, c->ws.stats, sizeof(s), hipMemcpyDeviceToHost));
  ACC_HIP(c, hipMemcpy(level, c->ws.level, 4, hipMemcpyDeviceToHost));
  *pending_micro_steps = (int32_t)slot[0];
  *last_batch_micro_steps = (int32_t)slot[1];
  *exchanges = (int64_t)s[0];
  *micro_steps = (int64_t)s[1];
  return ACC_OK;
}

int32_t accordion_state_bytes(const acc_ctx* c, size_t* out_bytes) {
  if (!c || !out_bytes) return ACC_EINVAL;
  *out_bytes = state_bytes_of(c);
  return ACC_OK;
}

static int32_t state_copy(acc_ctx* c, char* host, bool to_host) {
  const Plan& p = c->plan;
  const size_t N4 = 4 * (size_t)p.N, L4 = 4 * (size_t)c->cfg.n_layers;
  auto cp = [&](void* dev, size_t bytes) -> hipError_t {
    if (bytes == 0) return hipSuccess;
    hipError_t e = to_host ? hipMemcpy(host, dev, bytes, hipMemcpyDeviceToHost)
                           : hipMemcpy(dev, host, bytes, hipMemcpyHostToDevice);
    host += bytes;
    return e;
  };
  for (int w = 0; w < c->cfg.n_workers; ++w) ACC_HIP(c, cp(c->ws.e + (size_t)w * p.e_stride, N4));
  uint32_t fresh = 0;                                        // the window has just restarted: A counts as zero
  if (to_host) ACC_HIP(c, hipMemcpy(&fresh, c->ws.a_fresh, 4, hipMemcpyDeviceToHost));
  if (fresh) {
    std::memset(host, 0, N4);
    host += N4;
  } else {
    ACC_HIP(c, cp(c->ws.A, N4));
  }
  if (c->cfg.method == ACC_POWERSGD) {
    const int rq = copy_q(c, reinterpret_cast<float*>(host), to_host);
    if (rq != ACC_OK) return rq;
    host += 4 * (size_t)p.q_total;
  }
  // batch-size mode: micro-steps summed so far, in the slot the next micro-step reads
  if (c->cfg.method == ACC_BATCH) ACC_HIP(c, cp(c->ws.bstate + 4 * (c->step_id & 1u), 4));
  ACC_HIP(c, cp(c->ws.norm_old, L4));
  ACC_HIP(c, cp(c->ws.has_old, L4));
  ACC_HIP(c, cp(c->ws.level, L4));
  return ACC_OK;
}

int32_t accordion_get_state(acc_ctx* c, void* state_host, size_t bytes) {
  ACC_USABLE(c);
  if (!state_host) return fail(c->err, ACC_EINVAL, "state_host is NULL");
  if (c->in_step) return fail(c->err, ACC_ESTATE, "get_state inside a step");
  if (bytes < state_bytes_of(c)) return fail(c->err, ACC_ENOSPACE, "state buffer too small");
  const int rc = materialise(c);
  if (rc != ACC_OK) return rc;
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  return state_copy(c, static_cast<char*>(state_host), true);
}

int32_t accordion_set_state(acc_ctx* c, const void* state_host, size_t bytes) {
  ACC_USABLE(c);
  if (!state_host) return fail(c->err, ACC_EINVAL, "state_host is NULL");
  if (c->in_step) return fail(c->err, ACC_ESTATE, "set_state inside a step");
  if (bytes < state_bytes_of(c)) return fail(c->err, ACC_ENOSPACE, "state buffer too small");
  // levels must be 0 or 1: they index the per-layer rank / k tables in the kernels
  const size_t L = (size_t)c->cfg.n_layers;
  const int32_t* lv = reinterpret_cast<const int32_t*>(static_cast<const char*>(state_host) + state_bytes_of(c) - 4 * L);
  for (size_t i = 0; i < L; ++i)
    if (lv[i] != 0 && lv[i] != 1) return fail(c->err, ACC_EINVAL, "state holds a level other than 0 or 1");
  if (c->cfg.method == ACC_BATCH) {
    for (size_t i = 1; i < L; ++i)
      if (lv[i] != lv[0]) return fail(c->err, ACC_EINVAL, "batch-size mode has one level for the whole model");
    const int32_t* jp = reinterpret_cast<const int32_t*>(reinterpret_cast<const char*>(lv) - 8 * L - 4);
    if (*jp < 0 || *jp >= c->cfg.batch_multiplier)
      return fail(c->err, ACC_EINVAL, "state holds a micro-step count outside [0, batch_multiplier)");
  }
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  const int32_t rc = state_copy(c, const_cast<char*>(static_cast<const char*>(state_host)), false);
  if (rc != ACC_OK) return rc;
  if (c->cfg.method == ACC_POWERSGD)                         // the memory just written is explicit
    ACC_LAUNCH(c, psgd_clear_pending_kernel, dim3(1), dim3(64), c->ws);
  if (c->cfg.method == ACC_TOPK) ACC_LAUNCH(c, topk_clear_pending_kernel, dim3(1), dim3(64), c->ws);
  if (c->plan.r_sq_part.bytes > 0) {                         // the MSDR window restarts with the import
    const int n8 = (int)(c->plan.r_sq_part.bytes / 8);
    ACC_LAUNCH(c, zero_u64_kernel, dim3((n8 + 255) / 256), dim3(256),
               reinterpret_cast<unsigned long long*>(c->ws.sq_part), n8);
  }
  // the imported A: its sums of squares per tile, and it is not "fresh"
  if (c->cfg.method != ACC_BATCH)
    ACC_LAUNCH(c, norm_refresh_kernel, dim3(c->ws.n_ftiles + c->ws.n_mtiles), dim3(256), c->ws);
  ACC_LAUNCH(c, recount_words_kernel, dim3(1), dim3(256), c->ws, (int)c->cfg.method, c->cfg.method != ACC_BATCH ? 0 : -1);
  ACC_HIP(c, hipStreamSynchronize(c->stream));
  return ACC_OK;
}

int32_t accordion_set_profiling(acc_ctx* c, int32_t enable) {
  if (!c) return ACC_EINVAL;
  const int rc = drain_profile(c);
  if (rc != ACC_OK) return rc;
  if (enable && !c->profiling) {
    for (int i = 0; i < ST_COUNT; ++i) { c->stage_ms[i] = 0.0; c->stage_n[i] = 0; }
  }
  c->profiling = (enable == 2 || enable == 3) ? enable : (enable != 0 ? 1 : 0);
  c->prof_tick = 0;
  return ACC_OK;
}

int32_t accordion_get_profile(acc_ctx* c, int32_t stage, double* total_ms, int64_t* launches) {
  if (!c) return ACC_EINVAL;
  if (stage < 0 || stage >= ST_COUNT) return fail(c->err, ACC_EINVAL, "stage out of range");
  if (!total_ms || !launches) return fail(c->err, ACC_EINVAL, "host pointer is NULL");
  const int rc = drain_profile(c);
  if (rc != ACC_OK) return rc;
  *total_ms = c->stage_ms[stage];
  *launches = c->stage_n[stage];
  return ACC_OK;
}

const char* accordion_stage_name(int32_t stage) {
  return (stage >= 0 && stage < ST_COUNT) ? kStageNames[stage] : nullptr;
}

int32_t accordion_probe_copy(float* dst_dev, const float* src_dev, int64_t n, void* hip_stream) {
  if (!dst_dev || !src_dev) return fail(g_init_error, ACC_EINVAL, "probe_copy: pointer is NULL");
  if (misaligned(dst_dev) || misaligned(src_dev)) return fail(g_init_error, ACC_EINVAL, "probe_copy: pointer is not 16-byte aligned");
  if (n <= 0 || n % 4 != 0 || n > (int64_t(1) << 36)) return fail(g_init_error, ACC_EINVAL, "probe_copy: n must be a positive multiple of 4");
  const int64_t nquads = n / 4;
  const int64_t per_block = 256 * kProbeQuadsPerThread;
  const int64_t blocks = (nquads + per_block - 1) / per_block;
  if (blocks > (int64_t(1) << 31) - 1) return fail(g_init_error, ACC_EINVAL, "probe_copy: n too large");
  hipLaunchKernelGGL(probe_copy_kernel, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(hip_stream),
                     reinterpret_cast<float4*>(dst_dev), reinterpret_cast<const float4*>(src_dev), nquads);
  if (hipGetLastError() != hipSuccess) return fail(g_init_error, ACC_EHIP, "probe_copy: launch failed");
  return ACC_OK;
}

}  // extern "C"
