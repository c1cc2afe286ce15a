// Accumulated-gradient norms and the per-layer critical-regime decision (Section 4.2,
// Algorithm 1 of the paper), entirely on the device.
#pragma once
#include "acc_common.h"

namespace acc {

// The norm of the accumulated gradient costs no pass of its own for TopK and PowerSGD: the pass
// that adds worker 0's gradient to A has every element of A in registers and leaves the sum of
// their squares per tile (fp64; each fp32 square is exact there) in norm_part / norm_part_m, and
// "A <- 0" at the end of a window is a flag (a_fresh) that makes the next such pass store the
// gradient instead of adding it.  A window end is then the decision kernel alone.  (The
// batch-size mode keeps the separate pass below.)
// After an import of A (accordion_set_state): the per-tile sums of squares of the imported A.
// Workgroups 0 .. n_ftiles-1 take the flat tiles, the rest the matrix tiles (PowerSGD).
__global__ __launch_bounds__(256) void norm_refresh_kernel(const Ws ws) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  double s = 0.0;
  if ((int)blockIdx.x < ws.n_ftiles) {
    const FlatTile ft = ws.ftiles[blockIdx.x];
    const LayerDev& L = ws.layers[ft.layer];
    const TileGeom tg = tile_geom(L, ft);
    for (int q = tid; q < tg.nquads; q += kFlatThreads) s += sq4(ld_quad(ws.A, tg.a0 + 4 * (int64_t)q, tg.lo, tg.hi));
    s = block_sum4_d(s, red);
    if (tid == 0) ws.norm_part[blockIdx.x] = s;
  } else {
    const int mt = (int)blockIdx.x - ws.n_ftiles;
    const MatTile t = ws.mtiles[mt];
    const LayerDev& L = ws.layers[t.layer];
    const int rows = min(kMatRows, L.rows - t.row0), cols = min(kMatCols, L.cols - t.col0);
    for (int x = tid; x < rows * cols; x += kFlatThreads) {
      const float a = ws.A[L.offset + (int64_t)(t.row0 + x / cols) * L.cols + t.col0 + x % cols];
      s += (double)a * (double)a;
    }
    s = block_sum4_d(s, red);
    if (tid == 0) ws.norm_part_m[mt] = s;
  }
}

// Batch-size mode.  Per flat tile: sum of squares of A in fp64, then A <- 0.
__global__ __launch_bounds__(256) void norm_partial_kernel(const Ws ws) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  double s = 0.0;
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int q = tid; q < tg.nquads; q += kFlatThreads) {
    const int64_t base = tg.a0 + 4 * (int64_t)q;
    const float4 a = ld_quad(ws.A, base, tg.lo, tg.hi);   // outside the tile: 0
    s += (double)a.x * (double)a.x;
    s += (double)a.y * (double)a.y;
    s += (double)a.z * (double)a.z;
    s += (double)a.w * (double)a.w;
    st_quad(ws.A, base, tg.lo, tg.hi, zero);
  }
  s = wave_sum_f64(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) ws.norm_part[blockIdx.x] = (red[0] + red[1]) + (red[2] + red[3]);
}

// The accumulation window restarts without a decision.  zero_a (batch-size mode): A is cleared
// here; otherwise the restart is the a_fresh flag.
__global__ __launch_bounds__(256) void zero_accum_kernel(const Ws ws, int zero_a) {
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const float4 zero = make_float4(0.f, 0.f, 0.f, 0.f);
  if (zero_a) {
    for (int q = threadIdx.x; q < tg.nquads; q += kFlatThreads)
      st_quad(ws.A, tg.a0 + 4 * (int64_t)q, tg.lo, tg.hi, zero);
  } else if (blockIdx.x == 0 && threadIdx.x == 0) {
    *ws.a_fresh = 1u;
  }
  if (threadIdx.x == 0) {                                   // the MSDR detector's window sums too
    if (ws.sq_part) ws.sq_part[blockIdx.x] = 0.0;
    if (blockIdx.x == 0) ws.words[3] = 0ull;
  }
}

// Sum of the layer's per-tile sums of squares of A (0 when the window has just restarted), the same
// value in every lane of the wave.  batch: the partials are those of norm_partial_kernel.
__device__ __forceinline__ double layer_sumsq(const Ws& ws, const LayerDev& L, int lane) {
  if (*ws.a_fresh != 0u) return 0.0;
  double s = 0.0;
  if (L.is_matrix) {
    const int nmt = L.n_colchunks * ((L.rows + kMatRows - 1) / kMatRows);
    for (int t = lane; t < nmt; t += kWave) s += ws.norm_part_m[L.mt0 + t];
  } else {
    for (int t = lane; t < L.ntiles; t += kWave) s += ws.norm_part[L.tile0 + t];
  }
  return wave_sum_f64(s);
}

// One wave per layer: c = sqrt(sum of the layer's tile partials), then Algorithm 1 in fp32:
// critical <=> lr_next < lr_curr, or no previous norm, or previous norm 0,
//              or |old - c| / old >= eta.   level <- critical; old <- c.
__global__ __launch_bounds__(64) void regime_decide_kernel(const Ws ws, float lr_curr, float lr_next) {
  const int li = blockIdx.x;
  const int lane = threadIdx.x;
  const LayerDev& L = ws.layers[li];
  const double s = layer_sumsq(ws, L, lane);
  if (lane == 0) {
    const float c = (float)sqrt(s);
    const float old = ws.norm_old[li];
    const bool has_old = ws.has_old[li] != 0;
    bool crit;
    if (lr_next < lr_curr) crit = true;
    else if (!has_old) crit = true;
    else if (old == 0.0f) crit = true;
    else crit = (fabsf(old - c) / old) >= ws.eta;
    ws.level[li] = crit ? 1 : 0;
    ws.norm_prev[li] = old;
    ws.norm_curr[li] = c;
    ws.norm_old[li] = c;
    ws.has_old[li] = 1;
  }
}

// ---- comparison detector: mean to standard deviation ratio (Section 5.6) -----------------------

// Per flat tile: sq_part[tile] += sum of squares of worker 0's gradient (fp64; one workgroup owns
// a tile, the order inside is fixed: the running sums are reproducible).  Block 0 counts the step.
__global__ __launch_bounds__(256) void msdr_sq_kernel(const Ws ws, const float* __restrict__ g0) {
  __shared__ double red[4];
  const int tid = threadIdx.x;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  double s = 0.0;
  for (int q = tid; q < tg.nquads; q += kFlatThreads) {
    const float4 a = ld_quad(g0, tg.a0 + 4 * (int64_t)q, tg.lo, tg.hi);
    s += (double)a.x * (double)a.x;
    s += (double)a.y * (double)a.y;
    s += (double)a.z * (double)a.z;
    s += (double)a.w * (double)a.w;
  }
  s = wave_sum_f64(s);
  if ((tid & 63) == 0) red[tid >> 6] = s;
  __syncthreads();
  if (tid == 0) {
    ws.sq_part[blockIdx.x] += (red[0] + red[1]) + (red[2] + red[3]);
    if (blockIdx.x == 0) ws.words[3] += 1ull;               // steps in the window
  }
}

// One wave per layer, after norm_partial_kernel: with a = sum of the layer's tile partials of
// ||A||^2, q = sum of its sq_part and T steps,  m = sqrt( (a / T^2) / (q / T - a / T^2) )  (+inf
// when the gradients did not vary).  First window: m becomes the reference.  Later: once
// m <= (1 - eta) * reference the layer moves to the accurate level (1) for good and m becomes
// the reference.  norm_curr = m, norm_old = reference.  The window's sums are cleared.
__global__ __launch_bounds__(64) void msdr_decide_kernel(const Ws ws) {
  const int li = blockIdx.x;
  const int lane = threadIdx.x;
  const LayerDev& L = ws.layers[li];
  const double a = layer_sumsq(ws, L, lane);
  double q = 0.0;
  for (int t = lane; t < L.ntiles; t += kWave) {
    q += ws.sq_part[L.tile0 + t];
    ws.sq_part[L.tile0 + t] = 0.0;
  }
  q = wave_sum_f64(q);
  if (lane == 0) {
    const unsigned long long steps = ws.words[3];
    const double T = steps ? (double)steps : 1.0;
    const double mu2 = a / (T * T);
    const double var = q / T - mu2;
    const float m = var <= 0.0 ? __builtin_inff() : (float)sqrt(mu2 / var);
    const float ref = ws.norm_old[li];
    ws.norm_prev[li] = ref;
    ws.norm_curr[li] = m;
    if (ws.has_old[li] == 0) {
      ws.norm_old[li] = m;
      ws.has_old[li] = 1;
    } else if (m <= (1.0f - ws.eta) * ref) {
      ws.level[li] = 1;
      ws.norm_old[li] = m;
    }
  }
}

// Floats one worker sends per step at the current levels (the paper's "Data Sent" unit).
// fresh: 0 / 1 = what the a_fresh flag becomes (1 after a decision: the window restarts; 0 after an
// import of A); -1 leaves it.
__global__ __launch_bounds__(256) void recount_words_kernel(const Ws ws, int method, int fresh) {
  __shared__ unsigned long long red[256];
  if (threadIdx.x == 0) ws.words[3] = 0ull;                 // a new detection window starts
  if (threadIdx.x == 0 && fresh >= 0) *ws.a_fresh = (uint32_t)fresh;
  if (method == 2) {                        // batch-size mode: an exchange is the dense model
    if (threadIdx.x == 0) ws.words[0] = (unsigned long long)ws.n_model;
    return;
  }
  unsigned long long s = 0;
  for (int li = threadIdx.x; li < ws.L; li += 256) {
    const LayerDev& L = ws.layers[li];
    const int lv = ws.level[li];
    if (method == 0) {
      if (L.is_matrix) s += (unsigned long long)L.rank[lv] * (unsigned long long)(L.rows + L.cols);
      else s += (unsigned long long)L.rows * (unsigned long long)L.cols;
    } else {
      s += 2ull * (unsigned long long)L.k[lv];
    }
  }
  red[threadIdx.x] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    unsigned long long t = 0;
    for (int i = 0; i < 256; ++i) t += red[i];
    ws.words[0] = t;
  }
}

}  // namespace acc
