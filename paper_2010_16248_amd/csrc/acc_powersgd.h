// PowerSGD kernels: error-feedback add fused with P = Delta Q, mean + Gram-Schmidt,
// Q = Delta^T P^, mean of Q, decompress + residual.  All products are HBM-bound at rank <= 4
// (2r flop per 4-byte element), so the kernels stream the matrix once per pass with 16-byte
// accesses and keep the thin factor in registers; no MFMA.
//
// The residual e_w = Delta_w - P^ Q~^T of a step is not written by that step: the error memory
// keeps Delta_w, and the next step's first pass forms e_w on the fly from the previous factors
// (which are still in place: Q~ is the warm start, P^ is overwritten only later in the step)
// before it adds the new gradient.  That saves one read and one write of the matrix per worker
// and step.  psgd_residual_kernel makes the memory explicit when somebody wants to look at it.
//
// Matrix tile: 64 rows x 256 columns, one workgroup of 4 waves.  A lane owns 4 columns
// (vec4 layers: 4 adjacent columns, one 16-byte access per row; other layers: columns
// lane, lane+64, lane+128, lane+192, 4-byte accesses).  A wave owns rows wave, wave+4, ...
#pragma once
#include "acc_common.h"

namespace acc {

template <bool V4>
__device__ __forceinline__ void lane_cols(int col0, int lane, int cols, int (&col)[4], bool (&cm)[4]) {
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    col[v] = V4 ? col0 + lane * 4 + v : col0 + lane + 64 * v;
    cm[v] = col[v] < cols;
  }
}

// Streaming access for what a step touches once, so that Delta stays in the caches between the
// passes (first pass 119 -> 110 us on ResNet-18 shapes, W = 4).
constexpr bool kPsgdStreamG = true;     // gradients: read once per step
constexpr bool kPsgdStreamA = true;     // accumulator: read and written once per step
constexpr bool kPsgdStreamOut = true;   // averaged gradient: written once, read by nobody here

// STREAM: streaming (non-temporal) access on the 16-byte path, for data touched once per step.
template <bool V4, bool STREAM = false>
__device__ __forceinline__ void load_row(const float* __restrict__ p, int64_t rowbase,
                                         const int (&col)[4], const bool (&cm)[4], float (&d)[4]) {
  if (V4) {
    if (cm[0]) {
      const float4 t = STREAM ? ld16_stream(p + rowbase + col[0])
                              : *reinterpret_cast<const float4*>(p + rowbase + col[0]);
      d[0] = t.x; d[1] = t.y; d[2] = t.z; d[3] = t.w;
    } else {
      d[0] = d[1] = d[2] = d[3] = 0.f;
    }
  } else {
#pragma unroll
    for (int v = 0; v < 4; ++v) d[v] = cm[v] ? p[rowbase + col[v]] : 0.f;
  }
}

template <bool V4, bool STREAM = false>
__device__ __forceinline__ void store_row(float* __restrict__ p, int64_t rowbase,
                                          const int (&col)[4], const bool (&cm)[4],
                                          const float (&d)[4]) {
  if (V4) {
    if (cm[0]) {
      if (STREAM) st16_stream(p + rowbase + col[0], make_float4(d[0], d[1], d[2], d[3]));
      else *reinterpret_cast<float4*>(p + rowbase + col[0]) = make_float4(d[0], d[1], d[2], d[3]);
    }
  } else {
#pragma unroll
    for (int v = 0; v < 4; ++v)
      if (cm[v]) p[rowbase + col[v]] = d[v];
  }
}

// The rows of Q (kMaxRank floats each on the device, zero beyond rmax) of the four columns a lane
// owns: one aligned 16-byte load per row.  (Sixteen single-word loads at a 64-byte stride between
// lanes kept the texture path busy for longer than the rows of the tile themselves.)
__device__ __forceinline__ void load_q_rows(const Ws& ws, const LayerDev& L, const int (&col)[4],
                                            const bool (&cm)[4], float (&q)[4][kMaxRank]) {
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
    if (cm[v]) t = *reinterpret_cast<const float4*>(ws.Q + L.q_off + (int64_t)col[v] * kMaxRank);
    q[v][0] = t.x; q[v][1] = t.y; q[v][2] = t.z; q[v][3] = t.w;
  }
}

// ---- phase 0: Delta = g + e (in place of e), A += g (worker 0), P partial = Delta Q ---------

// One entry of P^ Q~^T: sum_k p[k] q[k] over all kMaxRank columns, where the caller has set p[k]
// to 0 beyond the rank in use (a product with 0 leaves the sum as it is).  Every kernel that
// needs an entry of D forms it with this one expression, so that they agree bit for bit.
__device__ __forceinline__ float low_rank_entry(const float (&p)[kMaxRank], const float (&q)[kMaxRank]) {
  float s = p[0] * q[0];
  s = fmaf(p[1], q[1], s);
  s = fmaf(p[2], q[2], s);
  s = fmaf(p[3], q[3], s);
  return s;
}

// rp > 0: the memory still holds the previous step's Delta; its residual is Delta - P^ Q~^T with
// the previous P^ (rows in ws.Phat) and Q~ (= the warm start, first rp columns).
template <int R, bool V4>
__device__ void ef_p_tile(const Ws& ws, const LayerDev& L, const MatTile& t, const float* __restrict__ g,
                          float* __restrict__ e, float* __restrict__ A, double* __restrict__ ppart, int rp,
                          float (*ps)[kMaxRank], bool a_fresh, double* red4) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int col[4]; bool cm[4];
  lane_cols<V4>(t.col0, lane, L.cols, col, cm);
  if (rp > 0) {
    // the previous P^ rows of the tile (zero-padded) go to LDS with one load per thread, requested
    // together with Q's rows, so that the row loop waits for no load of theirs
    const int pr = threadIdx.x >> 2, pk = threadIdx.x & 3;
    const int i = t.row0 + pr;
    ps[pr][pk] = (i < L.rows && pk < rp) ? ws.Phat[L.p_off + (int64_t)i * ws.rmax + pk] : 0.f;
  }
  float q[4][kMaxRank];
  load_q_rows(ws, L, col, cm, q);

  if (rp > 0) __syncthreads();                             // uniform over the workgroup
  const int row_end = min(t.row0 + kMatRows, L.rows);
  const int chunk = t.col0 / kMatCols;
  constexpr int B = 2;   // rows in flight per wave (one row is as fast; more rows cost registers and occupancy)
  double a_sq = 0.0;     // worker 0: the lane's share of the tile's sum of squares of A
  for (int i0 = t.row0 + wave; i0 < row_end; i0 += 4 * B) {
    float gd[B][4], ed[B][4], ad[B][4];
    double part[R >= 3 ? 1 : B][R];                          // a row that does not exist contributes zeros
#pragma unroll
    for (int b = 0; b < (R >= 3 ? 1 : B); ++b)
#pragma unroll
      for (int k = 0; k < R; ++k) part[b][k] = 0.0;
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int i = i0 + 4 * b;
      if (i < row_end) {
        const int64_t rb = L.offset + (int64_t)i * L.cols;
        load_row<V4, kPsgdStreamG>(g, rb, col, cm, gd[b]);
        load_row<V4>(e, rb, col, cm, ed[b]);
        if (A && !a_fresh) load_row<V4, kPsgdStreamA>(A, rb, col, cm, ad[b]);
        else ad[b][0] = ad[b][1] = ad[b][2] = ad[b][3] = 0.f;
      }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int i = i0 + 4 * b;
      if (i < row_end) {                       // wave-uniform
        const int64_t rb = L.offset + (int64_t)i * L.cols;
        if (rp > 0) {                          // wave-uniform: the pending residual first
          float pp[kMaxRank];
#pragma unroll
          for (int k = 0; k < kMaxRank; ++k) pp[k] = ps[i - t.row0][k];
#pragma unroll
          for (int v = 0; v < 4; ++v) ed[b][v] = ed[b][v] - low_rank_entry(pp, q[v]);
        }
        float d[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) d[v] = gd[b][v] + ed[b][v];
        store_row<V4>(e, rb, col, cm, d);
        if (A) {
#pragma unroll
          for (int v = 0; v < 4; ++v) ad[b][v] += gd[b][v];
          store_row<V4, kPsgdStreamA>(A, rb, col, cm, ad[b]);
#pragma unroll
          for (int v = 0; v < 4; ++v) a_sq += (double)ad[b][v] * (double)ad[b][v];   // masked columns hold zeros
        }
        // the lane's share of the chunk's share of P_w's row, in fp64: products of fp32 values are
        // exact there, the sums carry an error far below the fp32 rounding of the stored P_w
        double dd[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) dd[v] = (double)d[v];
#pragma unroll
        for (int k = 0; k < R; ++k) {
          double s = dd[0] * (double)q[0][k];
          s = fma(dd[1], (double)q[1][k], s);
          s = fma(dd[2], (double)q[2][k], s);
          s = fma(dd[3], (double)q[3][k], s);
          part[R >= 3 ? 0 : b][k] = s;
        }
        if constexpr (R >= 3) {
          // Three or four values per row: folded row by row (as many instructions as folding both
          // rows together, half the registers).  The lower 32 lanes end with columns 0 and 1 of
          // P (even / odd rows of 16 lanes), the upper 32 with columns 2 and 3.
          const double y02 = fold32_d(part[0][0], part[0][2]);
          const double y13 = fold32_d(part[0][1], R > 3 ? part[0][R - 1] : 0.0);
          const double y = row_sum_d(fold16_d(y02, y13));
          const int kcol = 2 * (lane >> 5) + ((lane >> 4) & 1);
          if ((lane & 15) == 0 && kcol < R)
            ppart[L.ppart_off + ((int64_t)chunk * L.rows + i) * ws.rmax + kcol] = y;
        }
      }
    }
    if constexpr (R <= 2) {
      // One or two values per row: both rows' values are folded over the wave together (the upper
      // 32 lanes keep the second row, the odd rows of 16 lanes the second column of P), so that
      // the lane exchanges of a full butterfly per value (27 instructions each in fp64) shrink
      // to about 20 for all of them.
      const int hb = lane >> 5, rp16 = (lane >> 4) & 1;     // which row of the pair / which column
      const int i_mine = i0 + 4 * hb;
      double* dst = ppart + L.ppart_off + ((int64_t)chunk * L.rows + i_mine) * ws.rmax;
      const bool writer = (lane & 15) == 0 && i_mine < row_end;
      if constexpr (R == 1) {
        double y = fold32_d(part[0][0], part[1][0]);
        y = row_sum_d(y);
        y = fold16_d(y, y);                                  // both rows of 16 lanes of a half
        if (writer && rp16 == 0) dst[0] = y;
      } else {
        const double y0 = fold32_d(part[0][0], part[1][0]), y1 = fold32_d(part[0][1], part[1][1]);
        const double y = row_sum_d(fold16_d(y0, y1));       // even rows of 16 lanes: column 0, odd rows: column 1
        if (writer) dst[rp16] = y;
      }
    }
  }
  if (A) {                                                 // uniform over the workgroup
    const double tsum = block_sum4_d(a_sq, red4);
    if (threadIdx.x == 0) ws.norm_part_m[blockIdx.x] = tsum;
  }
}

// *ws.pending: bit w set = worker w's memory holds the previous Delta (see the top of this file).
// The mask lives on the device (set by the decompress pass, cleared when the residual is written
// out), so a captured graph of a step stays valid whatever happens between its replays.
__global__ __launch_bounds__(256) void psgd_ef_p_kernel(const Ws ws, const GradPtrs gp, int w0) {
  __shared__ float ps[kMatRows][kMaxRank];
  __shared__ double red4[4];
  const uint32_t pending = *ws.pending;
  const int w = w0 + blockIdx.y;
  const float* __restrict__ g = gp.p[w];
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  float* __restrict__ A = (w == 0) ? ws.A : nullptr;
  // the accumulation window has just restarted: A counts as zero and is not read
  const bool a_fresh = A && *ws.a_fresh != 0u;             // uniform over the workgroup
  if ((int)blockIdx.x >= ws.n_mtiles) {
    // 1-D layers: only the accumulation A += g of worker 0 happens here (and the tile's sum of squares)
    if (w != 0) return;
    const int tile_id = ws.vectiles[blockIdx.x - ws.n_mtiles];
    const FlatTile ft = ws.ftiles[tile_id];
    const LayerDev& L = ws.layers[ft.layer];
    const TileGeom tg = tile_geom(L, ft);
    double a_sq = 0.0;
    for (int q = threadIdx.x; q < tg.nquads; q += kFlatThreads) {
      const int64_t base = tg.a0 + 4 * (int64_t)q;
      float4 a = a_fresh ? make_float4(0.f, 0.f, 0.f, 0.f) : ld_quad(ws.A, base, tg.lo, tg.hi);
      const float4 gv = ld_quad(g, base, tg.lo, tg.hi);
      a.x += gv.x; a.y += gv.y; a.z += gv.z; a.w += gv.w;
      st_quad(ws.A, base, tg.lo, tg.hi, a);
      a_sq += sq4(a);                                        // elements outside the tile were loaded as zeros
    }
    a_sq = block_sum4_d(a_sq, red4);
    if (threadIdx.x == 0) ws.norm_part[tile_id] = a_sq;
    return;
  }
  const MatTile t = ws.mtiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = L.rank[ws.level[t.layer]];
  const int rp = ((pending >> w) & 1u) ? ws.rank_used[t.layer] : 0;   // rank of the previous step's factors
  double* ppart = ws.Ppart + (int64_t)w * ws.ppart_stride;
  if (L.vec4) {
    switch (r) {
      case 1: ef_p_tile<1, true>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      case 2: ef_p_tile<2, true>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      case 3: ef_p_tile<3, true>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      default: ef_p_tile<4, true>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
    }
  } else {
    switch (r) {
      case 1: ef_p_tile<1, false>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      case 2: ef_p_tile<2, false>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      case 3: ef_p_tile<3, false>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
      default: ef_p_tile<4, false>(ws, L, t, g, e, A, ppart, rp, ps, a_fresh, red4); break;
    }
  }
}

// ---- aggregate 0: P_bar = mean over workers (and column chunks), Gram-Schmidt -----------
//
// Precision.  Gram-Schmidt carries an error of its input into column k multiplied by the
// condition number of P_bar, and P_bar = Delta_bar Q is as badly conditioned as the warm start Q
// happens to be (a 2 x 2 Q with condition 2000 occurs among random starts).  So the whole chain
// that leads to P^ runs in fp64 and rounds to fp32 exactly where the method stores an fp32
// quantity: the products Delta Q are accumulated in fp64 per 256-column chunk (first pass), a
// worker's chunks are summed in fp64 and rounded (P_w), the workers' P_w are summed in fp64,
// divided by W and rounded (P_bar), the projections and norms of Gram-Schmidt are fp64 and the
// finished column is rounded (P^).  The passes over Delta are bound by memory either way.

constexpr int kOrthThreads = 1024;
constexpr int kOrthWaves = kOrthThreads / kWave;

// P_bar[i][k] = fl32( (sum_w fl32(sum_c partial[w][c][i][k])) / W ), chunks in index order.
// One workgroup per 16 rows of a layer; thread = (share, row, column of P), four shares per entry:
// share s sums the workers s, s + 4, ... (each worker's chunks in fp64, rounded to the fp32 value
// P_w), then the four shares are added in order.  Many small workgroups: the partial sums of a
// layer (1.2 MB for the largest ResNet-18 layer at four workers) are read by many compute units
// at once, and a thread waits for few dependent batches of loads.
constexpr int kPmeanRows = 16;
constexpr int kPmeanLoads = 8;   // partial sums a thread has in flight

__global__ __launch_bounds__(256) void psgd_pmean_kernel(const Ws ws) {
  __shared__ double share_sum[4][kPmeanRows * 4];
  const PTile t = ws.ptiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = L.rank[ws.level[t.layer]];
  const int share = threadIdx.x >> 6, slot = threadIdx.x & 63;
  const int i = t.row0 + (slot >> 2), k = slot & 3;
  const bool live = i < L.rows && k < r;
  double total = 0.0;
  if (live) {
    const int nc = L.n_colchunks;
    const int64_t cstride = (int64_t)L.rows * ws.rmax;
    const double* base = ws.Ppart + L.ppart_off + (int64_t)i * ws.rmax + k;
    for (int w = share; w < ws.W; w += 4) {
      const double* src = base + (int64_t)w * ws.ppart_stride;
      double s = 0.0;
      for (int c0 = 0; c0 < nc; c0 += kPmeanLoads) {
        double v[kPmeanLoads];
#pragma unroll
        for (int u = 0; u < kPmeanLoads; ++u) v[u] = src[(int64_t)min(c0 + u, nc - 1) * cstride];
#pragma unroll
        for (int u = 0; u < kPmeanLoads; ++u) s += (c0 + u < nc) ? v[u] : 0.0;
      }
      total += (double)(float)s;                            // P_w is an fp32 quantity
    }
  }
  share_sum[share][slot] = total;
  __syncthreads();
  if (share == 0 && live) {
    const double sum = ((share_sum[0][slot] + share_sum[1][slot]) + share_sum[2][slot]) + share_sum[3][slot];
    ws.Phat[L.p_off + (int64_t)i * ws.rmax + k] = (float)(sum / (double)ws.W);
  }
}

// Sum over the threads of the orthogonalisation workgroup, same value for every thread.  `slot`
// alternates between calls so that one barrier per call is enough.
// Only the first nwaves waves of the workgroup are still running (the others have left).
__device__ __forceinline__ double block_sum_orth(double v, double (*red)[kOrthWaves], int& slot, int nwaves) {
  v = wave_sum_d(v);
  if (nwaves == 1) return v;
  const int wave = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) red[slot][wave] = v;
  __syncthreads();
  double r = 0.0;
  for (int i = 0; i < nwaves; ++i) r += red[slot][i];
  slot ^= 1;
  return r;
}

// Modified Gram-Schmidt over the r columns of P_bar (in ws.Phat, fp32), in column order, in
// fp64; a column of zero length stays zero; P^ (fp32) replaces P_bar.  Layers of up to
// kOrthThreads rows live in registers, one row per thread; taller ones in an fp64 copy in
// global memory (each thread only ever touches its own rows).
template <int R>
__device__ void orth_layer(const Ws& ws, const LayerDev& L, double (*red)[kOrthWaves]) {
  const int n = L.rows;
  const int tid = threadIdx.x;
  float* ph = ws.Phat + L.p_off;
  int slot = 0;
  if (n <= kOrthThreads) {
    const int nwaves = (n + kWave - 1) / kWave;
    if (tid >= nwaves * kWave) return;                       // whole waves
    const bool holder = tid < n;
    double v[R];
#pragma unroll
    for (int k = 0; k < R; ++k) v[k] = holder ? (double)ph[(int64_t)tid * ws.rmax + k] : 0.0;
#pragma unroll
    for (int k = 0; k < R; ++k) {
#pragma unroll
      for (int j = 0; j < R; ++j) {
        if (j < k) {
          const double d = block_sum_orth(v[j] * v[k], red, slot, nwaves);
          v[k] = fma(-d, v[j], v[k]);
        }
      }
      const double nn = block_sum_orth(v[k] * v[k], red, slot, nwaves);
      const double nrm = sqrt(nn);
      v[k] = (nrm > 0.0) ? v[k] / nrm : 0.0;
    }
    if (holder) {
#pragma unroll
      for (int k = 0; k < R; ++k) ph[(int64_t)tid * ws.rmax + k] = (float)v[k];
    }
  } else {
    double* pw = ws.Pwork + L.p_off;
    for (int i = tid; i < n; i += kOrthThreads)
#pragma unroll
      for (int k = 0; k < R; ++k) pw[(int64_t)i * ws.rmax + k] = (double)ph[(int64_t)i * ws.rmax + k];
    for (int k = 0; k < R; ++k) {
      for (int j = 0; j < k; ++j) {
        double d = 0.0;
        for (int i = tid; i < n; i += kOrthThreads)
          d = fma(pw[(int64_t)i * ws.rmax + j], pw[(int64_t)i * ws.rmax + k], d);
        d = block_sum_orth(d, red, slot, kOrthWaves);
        for (int i = tid; i < n; i += kOrthThreads)
          pw[(int64_t)i * ws.rmax + k] = fma(-d, pw[(int64_t)i * ws.rmax + j], pw[(int64_t)i * ws.rmax + k]);
      }
      double nn = 0.0;
      for (int i = tid; i < n; i += kOrthThreads) {
        const double x = pw[(int64_t)i * ws.rmax + k];
        nn = fma(x, x, nn);
      }
      nn = block_sum_orth(nn, red, slot, kOrthWaves);
      const double nrm = sqrt(nn);
      for (int i = tid; i < n; i += kOrthThreads) {
        const double x = (nrm > 0.0) ? pw[(int64_t)i * ws.rmax + k] / nrm : 0.0;
        pw[(int64_t)i * ws.rmax + k] = x;
        ph[(int64_t)i * ws.rmax + k] = (float)x;
      }
    }
  }
}

__global__ __launch_bounds__(kOrthThreads) void psgd_orth_kernel(const Ws ws, const GradPtrs gp) {
  __shared__ double red[2][kOrthWaves];
  // worker 0's first pass has added its gradient to A: the window is no longer fresh
  if (blockIdx.x == 0 && threadIdx.x == 0) *ws.a_fresh = 0u;
  if ((int)blockIdx.x >= ws.n_mat) {
    // 1-D layers are sent raw: mean over workers in worker order
    const FlatTile ft = ws.ftiles[ws.vectiles[blockIdx.x - ws.n_mat]];
    const LayerDev& L = ws.layers[ft.layer];
    for (int i = threadIdx.x; i < ft.count; i += kOrthThreads) {
      const int64_t a = L.offset + ft.start + i;
      double s = (double)gp.p[0][a];
      for (int w = 1; w < ws.W; ++w) s += (double)gp.p[w][a];
      ws.vecmean[L.vec_off + ft.start + i] = (float)(s / (double)ws.W);
    }
    return;
  }
  const int li = ws.matlayers[blockIdx.x];
  const LayerDev& L = ws.layers[li];
  const int r = L.rank[ws.level[li]];
  if (threadIdx.x == 0) ws.rank_used[li] = r;
  switch (r) {
    case 1: orth_layer<1>(ws, L, red); break;
    case 2: orth_layer<2>(ws, L, red); break;
    case 3: orth_layer<3>(ws, L, red); break;
    default: orth_layer<4>(ws, L, red); break;
  }
}

// ---- phase 1: Q partial = Delta^T P^ over one 64-row block -----------------------------------
//
// fp64 accumulation here too: where the memory dominates gradient + memory, Delta^T p^_k cancels
// to a small fraction of its terms for the columns of P^ that the new gradient determines, and an
// fp32 sum would lose those columns of Q (the oracle's contraction is fp64, rounded once).

// Tile: kQRows rows x 256 columns, one workgroup of 4 waves; a wave owns rows wave, wave + 4, ...
// and keeps the sums of its four columns per lane in registers; the four waves' sums meet in LDS.
template <int R, bool V4>
__device__ void q_tile(const Ws& ws, const LayerDev& L, const MatTile& t, const float* __restrict__ e,
                       double* __restrict__ qpart, double (*red)[16][64], float (*ps)[kMaxRank]) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int col[4]; bool cm[4];
  lane_cols<V4>(t.col0, lane, L.cols, col, cm);
  // the tile's rows of P^ go to LDS
  for (int s = threadIdx.x; s < kQRows * kMaxRank; s += 256) {
    const int pr = s >> 2, pk = s & 3;
    const int i = t.row0 + pr;
    ps[pr][pk] = (i < L.rows && pk < R) ? ws.Phat[L.p_off + (int64_t)i * ws.rmax + pk] : 0.f;
  }
  __syncthreads();
  double acc[4][R];
#pragma unroll
  for (int v = 0; v < 4; ++v)
#pragma unroll
    for (int k = 0; k < R; ++k) acc[v][k] = 0.0;
  const int row_end = min(t.row0 + kQRows, L.rows);
  constexpr int B = 4;   // rows in flight per wave (2 and 8 are no faster)
  for (int i0 = t.row0 + wave; i0 < row_end; i0 += 4 * B) {
    float d[B][4];
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int i = i0 + 4 * b;
      if (i < row_end) load_row<V4>(e, L.offset + (int64_t)i * L.cols, col, cm, d[b]);
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int i = i0 + 4 * b;
      if (i < row_end) {                                     // wave-uniform
        double p[R], dd[4];
#pragma unroll
        for (int k = 0; k < R; ++k) p[k] = (double)ps[i - t.row0][k];
#pragma unroll
        for (int v = 0; v < 4; ++v) dd[v] = (double)d[b][v];
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
          for (int k = 0; k < R; ++k) acc[v][k] = fma(dd[v], p[k], acc[v][k]);
      }
    }
  }
  // the four waves' sums, in the fixed order (wave 0 + wave 2) + (wave 1 + wave 3)
  if (wave >= 2) {
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int k = 0; k < R; ++k) red[wave - 2][v * R + k][lane] = acc[v][k];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int k = 0; k < R; ++k) acc[v][k] += red[wave][v * R + k][lane];
  }
  __syncthreads();
  if (wave < 2) {
#pragma unroll
    for (int v = 0; v < 4; ++v)
#pragma unroll
      for (int k = 0; k < R; ++k) red[wave][v * R + k][lane] = acc[v][k];
  }
  __syncthreads();
  // thread (wave, lane) finishes column slot v = wave of that lane
  {
    const int v = wave;
    const int cv = V4 ? t.col0 + lane * 4 + v : t.col0 + lane + 64 * v;
    if (cv < L.cols) {
      const int rb = t.row0 / kQRows;
      double* dst = qpart + L.qpart_off + ((int64_t)rb * L.cols + cv) * ws.rmax;
#pragma unroll
      for (int k = 0; k < R; ++k) {
        const int s = v * R + k;
        dst[k] = red[0][s][lane] + red[1][s][lane];
      }
    }
  }
}

__global__ __launch_bounds__(256) void psgd_q_kernel(const Ws ws, int w0) {
  __shared__ double red[2][16][64];
  __shared__ float ps[kQRows][kMaxRank];
  const int w = w0 + blockIdx.y;
  const MatTile t = ws.qmtiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = L.rank[ws.level[t.layer]];
  const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  double* qpart = ws.Qpart + (int64_t)w * ws.qpart_stride;
  if (L.vec4) {
    switch (r) {
      case 1: q_tile<1, true>(ws, L, t, e, qpart, red, ps); break;
      case 2: q_tile<2, true>(ws, L, t, e, qpart, red, ps); break;
      case 3: q_tile<3, true>(ws, L, t, e, qpart, red, ps); break;
      default: q_tile<4, true>(ws, L, t, e, qpart, red, ps); break;
    }
  } else {
    switch (r) {
      case 1: q_tile<1, false>(ws, L, t, e, qpart, red, ps); break;
      case 2: q_tile<2, false>(ws, L, t, e, qpart, red, ps); break;
      case 3: q_tile<3, false>(ws, L, t, e, qpart, red, ps); break;
      default: q_tile<4, false>(ws, L, t, e, qpart, red, ps); break;
    }
  }
}

// ---- aggregate 1: Q_bar = mean over workers of (sum over row blocks) -------------------------

// Q_bar[c][k] = fl32( (sum_w fl32(sum_rb partial[w][rb][c][k])) / W ), row blocks and workers in
// index order; the partial sums of one worker are independent loads, issued eight at a time
// (unconditionally, from clamped addresses, so that all eight are in flight together).
template <int R, int U = 8>
__device__ __forceinline__ void qmean_col(const Ws& ws, const LayerDev& L, int c) {
  const double* base = ws.Qpart + L.qpart_off + (int64_t)c * ws.rmax;
  const int64_t pstride = (int64_t)L.cols * ws.rmax;
  const int nb = L.n_rowblocks;
  double total[R];
#pragma unroll
  for (int k = 0; k < R; ++k) total[k] = 0.0;
  for (int w = 0; w < ws.W; ++w) {
    const double* src = base + (int64_t)w * ws.qpart_stride;
    double s[R];
#pragma unroll
    for (int k = 0; k < R; ++k) s[k] = 0.0;
    for (int b0 = 0; b0 < nb; b0 += U) {
      double v[U][R];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const double* q = src + (int64_t)min(b0 + u, nb - 1) * pstride;
#pragma unroll
        for (int k = 0; k < R; ++k) v[u][k] = q[k];
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
#pragma unroll
        for (int k = 0; k < R; ++k) s[k] += (b0 + u < nb) ? v[u][k] : 0.0;
    }
#pragma unroll
    for (int k = 0; k < R; ++k) total[k] += (double)(float)s[k];   // Q_w is an fp32 quantity
  }
  float* dst = ws.Q + L.q_off + (int64_t)c * kMaxRank;    // rows of Q are kMaxRank floats apart
#pragma unroll
  for (int k = 0; k < R; ++k) dst[k] = (float)(total[k] / (double)ws.W);
}

__global__ __launch_bounds__(256) void psgd_qmean_kernel(const Ws ws) {
  const QTile t = ws.qtiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = L.rank[ws.level[t.layer]];
  const int c = t.col0 + threadIdx.x;
  if (c >= L.cols) return;
  switch (r) {
    case 1: qmean_col<1>(ws, L, c); break;
    case 2: qmean_col<2>(ws, L, c); break;
    case 3: qmean_col<3>(ws, L, c); break;
    default: qmean_col<4>(ws, L, c); break;
  }
}

// ---- decompress: D = P^ Q_bar^T (the residual stays implicit) ----------------------------------

// MODE 0: writes D of the tile to sink.out.  MODE 1: e = Delta - D in place.  MODE 2: D drives the
// optimizer step on sink.wt / sink.vel and is not stored.
template <int MODE, bool V4>
__device__ void decomp_tile(const Ws& ws, const LayerDev& L, const MatTile& t, float* __restrict__ e,
                            const Sink& sink, int r, float (*ps)[kMaxRank]) {
  constexpr bool RESIDUAL = MODE == 1;
  constexpr bool UPD = MODE == 2;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int col[4]; bool cm[4];
  lane_cols<V4>(t.col0, lane, L.cols, col, cm);
  const int row_end = min(t.row0 + kMatRows, L.rows);
  const float* __restrict__ ph = ws.Phat + L.p_off;
  // the tile's 64 rows of P^ (zero-padded to four columns) go to LDS with one load per thread,
  // requested together with Q's rows: the row loop then waits for no global load of its own
  {
    const int pr = threadIdx.x >> 2, pk = threadIdx.x & 3;
    const int i = t.row0 + pr;
    ps[pr][pk] = (i < row_end && pk < r) ? ph[(int64_t)i * ws.rmax + pk] : 0.f;
  }
  float q[4][kMaxRank];
  load_q_rows(ws, L, col, cm, q);
  __syncthreads();
  constexpr int B = 4;
  // Weights and velocity are read and written by every step, so they are accessed like the error
  // memory, not streamed like the gradients: where they fit the caches next to it (VGG-19 shapes,
  // W = 1) the fused update is 17 us faster that way, elsewhere it makes no difference.
  constexpr bool NT = false;
  for (int i0 = t.row0 + wave; i0 < row_end; i0 += 4 * B) {
    float d[B][4], vv[UPD ? B : 1][4];
    if (RESIDUAL || UPD) {
#pragma unroll
      for (int b = 0; b < B; ++b) {
        const int i = i0 + 4 * b;
        if (i < row_end) {
          const int64_t rb = L.offset + (int64_t)i * L.cols;
          load_row<V4, UPD && NT>(UPD ? sink.wt : e, rb, col, cm, d[b]);   // weights, velocity: once per step
          if (UPD) load_row<V4, NT>(sink.vel, rb, col, cm, vv[UPD ? b : 0]);
        }
      }
    }
#pragma unroll
    for (int b = 0; b < B; ++b) {
      const int i = i0 + 4 * b;
      if (i < row_end) {
        const int64_t rb = L.offset + (int64_t)i * L.cols;
        float p[kMaxRank];
#pragma unroll
        for (int k = 0; k < kMaxRank; ++k) p[k] = ps[i - t.row0][k];
        float D[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) D[v] = low_rank_entry(p, q[v]);
        if (RESIDUAL) {
          float res[4];
#pragma unroll
          for (int v = 0; v < 4; ++v) res[v] = d[b][v] - D[v];
          store_row<V4>(e, rb, col, cm, res);
        } else if (UPD) {
#pragma unroll
          for (int v = 0; v < 4; ++v) nesterov(D[v], d[b][v], vv[UPD ? b : 0][v], sink.lr, sink.mu, sink.wd);
          store_row<V4, NT>(sink.wt, rb, col, cm, d[b]);
          store_row<V4, NT>(sink.vel, rb, col, cm, vv[UPD ? b : 0]);
        } else {
          store_row<V4, kPsgdStreamOut>(sink.out, rb, col, cm, D);
        }
      }
    }
  }
}

// The averaged decompressed gradient: D on matrix layers, the plain mean on 1-D layers (which keep
// no memory: their e is cleared for every worker).
template <bool UPD>
__device__ __forceinline__ void decomp_body(const Ws& ws, const Sink& sink) {
  __shared__ float ps[kMatRows][kMaxRank];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *ws.pending = ws.W == 32 ? 0xffffffffu : ((1u << ws.W) - 1u);   // every e_w now holds Delta_w
    ws.words[1] = ws.words[0];
    ws.words[2] += ws.words[0];
  }
  if ((int)blockIdx.x >= ws.n_mtiles) {
    const FlatTile ft = ws.ftiles[ws.vectiles[blockIdx.x - ws.n_mtiles]];
    const LayerDev& L = ws.layers[ft.layer];
    for (int i = threadIdx.x; i < ft.count; i += kFlatThreads) {
      const int64_t a = L.offset + ft.start + i;
      for (int w = 0; w < ws.W; ++w) ws.e[(int64_t)w * ws.e_stride + a] = 0.f;
      const float d = ws.vecmean[L.vec_off + ft.start + i];
      if (UPD) {
        float wv = sink.wt[a], vv = sink.vel[a];
        nesterov(d, wv, vv, sink.lr, sink.mu, sink.wd);
        sink.wt[a] = wv;
        sink.vel[a] = vv;
      } else {
        sink.out[a] = d;
      }
    }
    return;
  }
  const MatTile t = ws.mtiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = ws.rank_used[t.layer];                     // written by the orthogonalisation of this step
  if (L.vec4) decomp_tile<UPD ? 2 : 0, true>(ws, L, t, nullptr, sink, r, ps);
  else decomp_tile<UPD ? 2 : 0, false>(ws, L, t, nullptr, sink, r, ps);
}

__global__ __launch_bounds__(256) void psgd_decomp_kernel(const Ws ws, const Sink sink) {
  decomp_body<false>(ws, sink);
}

// The same pass with the optimizer step in place of the store of D.
__global__ __launch_bounds__(256) void psgd_decomp_update_kernel(const Ws ws, const Sink sink) {
  decomp_body<true>(ws, sink);
}

// e_w = Delta_w - D for the workers whose bit is set in *ws.pending, in place; the caller clears
// the mask with psgd_clear_pending_kernel afterwards.
__global__ __launch_bounds__(256) void psgd_residual_kernel(const Ws ws) {
  const uint32_t pending = *ws.pending;
  const int w = blockIdx.y;
  if (((pending >> w) & 1u) == 0u) return;
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  const MatTile t = ws.mtiles[blockIdx.x];
  const LayerDev& L = ws.layers[t.layer];
  const int r = ws.rank_used[t.layer];
  const Sink none = {nullptr, nullptr, nullptr, 0.f, 0.f, 0.f};
  __shared__ float ps[kMatRows][kMaxRank];
  if (L.vec4) decomp_tile<1, true>(ws, L, t, e, none, r, ps);
  else decomp_tile<1, false>(ws, L, t, e, none, r, ps);
}

__global__ void psgd_clear_pending_kernel(const Ws ws) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *ws.pending = 0u;
}

}  // namespace acc
