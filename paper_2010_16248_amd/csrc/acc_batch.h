// Batch-size mode of Accordion (Section 3 "Distributed SGD with adaptive batch size"; Section
// 4.2: the same algorithm on the gradient of the whole model; Section 5.1 "Hyperparameters":
// learning rate scaled with the batch; Appendix A "Additional Details for Batch Size experiment":
// the large batch is several backward passes summed before one exchange, and it only grows).
//
// One launch per micro-step (one backward pass of every worker on B_low samples):
//   A += g_0;   S_w = g_w (first micro-step of a batch) or S_w + g_w;
//   batch complete (1 micro-step inside a critical regime, `mult` outside):
//     D = (S_0 + S_1 + ... + S_{W-1}) / (W * micro-steps), stored or consumed by the optimizer step
//     with the learning rate lr * micro-steps; the sums need not be written then.
// The number of micro-steps summed so far lives on the device in two slots used alternately
// (slot = micro-step parity), so that the one thread that advances it never races with the
// workgroups that read it.
#pragma once
#include "acc_common.h"

namespace acc {

constexpr int kBatchWorkers = 4;   // workers whose loads are in flight together
// The gradients stream in (read once), so that the running sums, the accumulator and, in the
// small-batch regime, the averaged gradient stay in the caches from one micro-step to the next:
// 118 -> 95 us per micro-step on ResNet-18 shapes, W = 4.  Streaming the rest as well brings
// nothing in the large-batch regime and costs 3 us in the small-batch one.
constexpr bool kBatchStreamG = true;
constexpr bool kBatchStream = false;

// Slot layout (uint32 x 4): [0] micro-steps summed before this micro-step, [1] micro-steps of the
// batch the previous micro-step completed (0: none), [2], [3] spare.
__device__ __forceinline__ const uint32_t* batch_slot(const Ws& ws, uint32_t parity) {
  return ws.bstate + 4 * (parity & 1u);
}

template <bool AL, bool UPD>
__device__ __forceinline__ void batch_tile(const Ws& ws, const GradPtrs& gp, const Sink& sink,
                                           const TileGeom& tg, uint32_t j, bool exch) {
  const int W = ws.W;
  const int64_t e_stride = ws.e_stride;
  float* const S = ws.e;
  float* const A = ws.A;
  const float denom = (float)((uint32_t)W * (j + 1u));
  const float lr_eff = sink.lr * (float)(j + 1u);
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int q = threadIdx.x; q < tg.nquads; q += kFlatThreads) {
    float4 a = ldq<AL, kBatchStream>(A, tg.a0, tg.lo, tg.hi, q, true);
    float4 wq = zero4, vq = zero4;
    if (UPD && exch) {
      wq = ldq<AL, kBatchStream>(sink.wt, tg.a0, tg.lo, tg.hi, q, true);
      vq = ldq<AL, kBatchStream>(sink.vel, tg.a0, tg.lo, tg.hi, q, true);
    }
    float4 acc = zero4;
    for (int wb = 0; wb < W; wb += kBatchWorkers) {
      float4 g[kBatchWorkers], s[kBatchWorkers];
#pragma unroll
      for (int u = 0; u < kBatchWorkers; ++u) {
        const int w = min(wb + u, W - 1);                  // clamped: the loads go out unconditionally
        g[u] = ldq<AL, kBatchStreamG>(gp.p[w], tg.a0, tg.lo, tg.hi, q, true);
        s[u] = (j > 0u) ? ldq<AL>(S + (int64_t)w * e_stride, tg.a0, tg.lo, tg.hi, q, true) : zero4;
      }
#pragma unroll
      for (int u = 0; u < kBatchWorkers; ++u) {
        const int w = wb + u;
        if (w < W) {                                       // workgroup-uniform
          if (w == 0) a = make_float4(a.x + g[u].x, a.y + g[u].y, a.z + g[u].z, a.w + g[u].w);
          float4 t = g[u];
          if (j > 0u) t = make_float4(s[u].x + t.x, s[u].y + t.y, s[u].z + t.z, s[u].w + t.w);
          if (exch) {
            acc = (w == 0) ? t : make_float4(acc.x + t.x, acc.y + t.y, acc.z + t.z, acc.w + t.w);
          } else {
            stq<AL>(S + (int64_t)w * e_stride, tg.a0, tg.lo, tg.hi, q, t);
          }
        }
      }
    }
    stq<AL, kBatchStream>(A, tg.a0, tg.lo, tg.hi, q, a);
    if (exch) {
      const float4 d = make_float4(acc.x / denom, acc.y / denom, acc.z / denom, acc.w / denom);
      if (UPD) {
        nesterov(d.x, wq.x, vq.x, lr_eff, sink.mu, sink.wd);
        nesterov(d.y, wq.y, vq.y, lr_eff, sink.mu, sink.wd);
        nesterov(d.z, wq.z, vq.z, lr_eff, sink.mu, sink.wd);
        nesterov(d.w, wq.w, vq.w, lr_eff, sink.mu, sink.wd);
        stq<AL, kBatchStream>(sink.wt, tg.a0, tg.lo, tg.hi, q, wq);
        stq<AL, kBatchStream>(sink.vel, tg.a0, tg.lo, tg.hi, q, vq);
      } else {
        stq<AL, kBatchStream>(sink.out, tg.a0, tg.lo, tg.hi, q, d);
      }
    }
  }
}

template <bool UPD>
__device__ __forceinline__ void batch_micro_body(const Ws& ws, const GradPtrs& gp, const Sink& sink,
                                                 uint32_t parity) {
  const uint32_t j = batch_slot(ws, parity)[0];
  const uint32_t target = (ws.level[0] == 1) ? 1u : (uint32_t)ws.bmult;
  const bool exch = j + 1u >= target;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t* next = ws.bstate + 4 * ((parity + 1u) & 1u);
    next[0] = exch ? 0u : j + 1u;
    next[1] = exch ? j + 1u : 0u;
    const unsigned long long sent = exch ? (unsigned long long)ws.n_model : 0ull;
    ws.words[1] = sent;
    ws.words[2] += sent;
    ws.stats[0] += exch ? 1ull : 0ull;                     // exchanges
    ws.stats[1] += 1ull;                                   // micro-steps
  }
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  if (tg.aligned) batch_tile<true, UPD>(ws, gp, sink, tg, j, exch);
  else batch_tile<false, UPD>(ws, gp, sink, tg, j, exch);
}

__global__ __launch_bounds__(256) void batch_micro_kernel(const Ws ws, const GradPtrs gp, const Sink sink,
                                                          uint32_t parity) {
  batch_micro_body<false>(ws, gp, sink, parity);
}

__global__ __launch_bounds__(256) void batch_micro_update_kernel(const Ws ws, const GradPtrs gp,
                                                                 const Sink sink, uint32_t parity) {
  batch_micro_body<true>(ws, gp, sink, parity);
}

// One workgroup: c = sqrt(sum of all tile partials) (the norm of the whole model's accumulated
// gradient), Algorithm 1 once, "the batch only grows" if asked for; the decision is written to
// every layer's entry so that the per-layer read-backs show it.
__global__ __launch_bounds__(256) void batch_decide_kernel(const Ws ws, float lr_curr, float lr_next) {
  __shared__ double red[4];
  __shared__ int s_level;
  __shared__ float s_old, s_c;
  const int tid = threadIdx.x;
  double s = 0.0;
  for (int t = tid; t < ws.n_ftiles; t += 256) s += ws.norm_part[t];
  s = wave_sum_f64(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    const float c = (float)sqrt((red[0] + red[1]) + (red[2] + red[3]));
    const float old = ws.norm_old[0];
    const bool has_old = ws.has_old[0] != 0;
    bool crit;
    if (lr_next < lr_curr) crit = true;
    else if (!has_old) crit = true;
    else if (old == 0.0f) crit = true;
    else crit = (fabsf(old - c) / old) >= ws.eta;
    int level = crit ? 1 : 0;
    if (ws.bmono != 0 && ws.level[0] == 0) level = 0;
    s_level = level;
    s_old = old;
    s_c = c;
  }
  __syncthreads();
  for (int li = tid; li < ws.L; li += 256) {
    ws.level[li] = s_level;
    ws.norm_prev[li] = s_old;
    ws.norm_curr[li] = s_c;
    ws.norm_old[li] = s_c;
    ws.has_old[li] = 1;
  }
}

}  // namespace acc
