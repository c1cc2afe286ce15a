// TopK kernels: exact per-layer selection of the k entries with the largest |Delta|
// (ties: lower flat index) by a three-level radix select on the 31 magnitude bits
// (11 + 11 + 9).  Every kernel is tile-parallel (one workgroup per 8192-element tile and
// worker).  The per-(worker, layer) decisions (which bin holds the k-th largest) are
// recomputed by every workgroup of the layer from the layer's global histogram at the start
// of the next kernel: that costs an 8 KB L2 read per workgroup and needs neither an extra
// launch nor a device-scope fence (which on this multi-die part writes back the whole L2).
//
//   A  topk_ef_hist      Delta = g + e (in place), A += g (worker 0), level-1 histogram
//                        (key bits 30..20) per (worker, layer)
//   B  topk_cand         [bin b1 of the k-th largest]  count of entries above b1 per tile;
//                        entries in b1 (candidates) go to the tile's segment as (key, index);
//                        level-2 histogram of the candidates (bits 19..9)
//   C  topk_level3       [bin b2]  candidates above b2 counted per tile; level-3 histogram
//                        (bits 8..0) of those in b2
//   D  topk_count        [threshold key T, tie quota]  per tile: candidates above T and
//                        candidates equal to T
//   E  topk_compact      [sums over the preceding tiles]  ordered compaction of the selected
//                        entries into the payload (index ascending), zeroing them in e
//   K6 topk_sparse_mean  dense mean of the W payloads
//
// Cross-workgroup combination is by integer atomics and fixed-order sums only, so every
// output is bit-reproducible.  A wave quarter's segment holds kSubCap candidates; if a quarter
// has more (huge tie classes: zeros, constants) the layer falls back to re-reading Delta in C
// and D.
#pragma once
#include "acc_common.h"

namespace acc {

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS histogram add with a fast path for a wave whose valid lanes all hit one bin.
__device__ __forceinline__ void hist_add(uint32_t* hist, bool valid, uint32_t bin, int lane) {
  const uint32_t b = valid ? bin : 0xffffffffu;
  const uint32_t fb = (uint32_t)__builtin_amdgcn_readfirstlane((int)b);
  const uint64_t act = __ballot(valid);
  const uint64_t same = __ballot(valid && b == fb);
  if (act != 0 && same == act) {
    if (lane == (int)__builtin_ctzll(act)) atomicAdd(&hist[fb], (uint32_t)__popcll(act));
  } else if (valid) {
    atomicAdd(&hist[bin], 1u);
  }
}

__device__ __forceinline__ void hist_flush(const uint32_t* hist, uint32_t* gh, int nbins) {
  for (int b = threadIdx.x; b < nbins; b += kFlatThreads) {
    const uint32_t h = hist[b];
    if (h) atomicAdd(&gh[b], h);
  }
}

// Copies a layer's global histogram into LDS, zero-padded to kHistBins.  Ends with a barrier.
__device__ __forceinline__ void hist_load(uint32_t* hist, const uint32_t* gh, int nbins) {
  for (int b = threadIdx.x; b < kHistBins; b += kFlatThreads) hist[b] = (b < nbins) ? gh[b] : 0u;
  __syncthreads();
}

__device__ __forceinline__ void hist_clear_global(uint32_t* gh, int nbins) {
  for (int b = threadIdx.x; b < nbins; b += kFlatThreads) gh[b] = 0u;
}

// hist: kHistBins counts in LDS.  Finds the largest bin b with count(bins >= b) >= k.
// Result in out[0..2] (LDS, zeroed by the caller before a barrier): bin, entries above the
// bin, entries in the bin.  256 threads; two barriers; every thread calls it.
__device__ __forceinline__ void pick_bin(const uint32_t* hist, uint32_t k, uint32_t* out,
                                         uint32_t* scratch) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  uint32_t h[8];
  uint32_t part = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) { h[i] = hist[tid * 8 + i]; part += h[i]; }
  const uint32_t suf = wave_incl_suffix_u32(part, lane);
  if (lane == 0) scratch[wave] = suf;            // wave total
  __syncthreads();
  uint32_t run = suf - part;                     // entries in bins of later threads of my wave
  for (int v = wave + 1; v < 4; ++v) run += scratch[v];
#pragma unroll
  for (int i = 7; i >= 0; --i) {
    if (run < k && run + h[i] >= k) {
      out[0] = (uint32_t)(tid * 8 + i);
      out[1] = run;
      out[2] = h[i];
    }
    run += h[i];
  }
  __syncthreads();
}

__device__ __forceinline__ uint32_t block_sum_u32(uint32_t v, uint32_t* red) {
  v = wave_sum_u32(v);
  __syncthreads();
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return red[0] + red[1] + red[2] + red[3];
}

// ---- A ----------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void topk_ef_hist_kernel(const Ws ws, const GradPtrs gp, int w0) {
  __shared__ uint32_t hist[kHistBins];
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const float* __restrict__ g = gp.p[w];
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  float* __restrict__ A = (w == 0) ? ws.A : nullptr;
  for (int b = tid; b < kHistBins; b += kFlatThreads) hist[b] = 0;
  __syncthreads();
#pragma unroll 3
  for (int j = 0; j < kQuadIters; ++j) {
    const int q = j * kFlatThreads + tid;
    const bool qa = q < tg.nquads;
    const int64_t base = tg.a0 + 4 * (int64_t)q;
    float4 d = make_float4(0.f, 0.f, 0.f, 0.f);
    if (qa) {
      const float4 gv = ld_quad(g, base, tg.lo, tg.hi);
      const float4 ev = ld_quad(e, base, tg.lo, tg.hi);
      d = make_float4(gv.x + ev.x, gv.y + ev.y, gv.z + ev.z, gv.w + ev.w);
      st_quad(e, base, tg.lo, tg.hi, d);
      if (A) {
        float4 a = ld_quad(A, base, tg.lo, tg.hi);
        a.x += gv.x; a.y += gv.y; a.z += gv.z; a.w += gv.w;
        st_quad(A, base, tg.lo, tg.hi, a);
      }
    }
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool valid = qa && (base + c >= tg.lo) && (base + c < tg.hi);
      hist_add(hist, valid, key_of(comp(d, c)) >> 20, lane);
    }
  }
  __syncthreads();
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  uint32_t* gh = ws.hist1 + wl * kHistBins;
  hist_flush(hist, gh, kHistBins);
  if (ft.start == 0 && tid == 0) ws.sel[wl].mode = 0;    // B raises it on segment overflow
}

// ---- wave quarters ------------------------------------------------------------------------------
// In kernels B..E wave v of the workgroup owns the contiguous quarter [v*qw, (v+1)*qw) of the
// tile's 16-byte groups, so every count, candidate list and running offset is wave-local
// (scalar registers, no barriers, no atomics) and index order is (wave, iteration, lane,
// component).

struct WaveSpan { int qbeg, qend; };

__device__ __forceinline__ WaveSpan wave_span(const TileGeom& tg, int wave) {
  const int qw = (tg.nquads + 3) >> 2;
  WaveSpan s;
  s.qbeg = wave * qw;
  s.qend = min(s.qbeg + qw, tg.nquads);
  return s;
}

__device__ __forceinline__ float4 ld_span(const float* __restrict__ e, const TileGeom& tg,
                                          const WaveSpan& sp, int q) {
  if (q < sp.qend) return ld_quad(e, tg.a0 + 4 * (int64_t)q, tg.lo, tg.hi);
  return make_float4(0.f, 0.f, 0.f, 0.f);
}

// Candidates (entries in level-1 bin b1) of my wave's quarter: from the quarter's segment, or,
// after a segment overflow, re-read from Delta.  f(key, valid) is called by all 64 lanes
// together (valid marks the lanes that hold a candidate).
template <class F>
__device__ __forceinline__ void for_wave_candidates(const Ws& ws, const LayerDev& L, const TileGeom& tg,
                                                    int w, int tile_id, int wave, int lane, uint32_t mode,
                                                    uint32_t b1, F f) {
  if (mode == 0) {
    const int64_t slot4 = ((int64_t)w * ws.n_ftiles + tile_id) * 4 + wave;
    const uint32_t cn = min(ws.cand_n[slot4], (uint32_t)kSubCap);
    const uint2* seg = ws.cand + slot4 * kSubCap;
    for (uint32_t i0 = 0; i0 < cn; i0 += kWave) {          // cn is wave-uniform
      const uint32_t i = i0 + lane;
      const bool valid = i < cn;
      const uint32_t key = valid ? seg[i].x : 0u;
      f(key, valid);
    }
  } else {
    const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
    const WaveSpan sp = wave_span(tg, wave);
    for (int q0 = sp.qbeg; q0 < sp.qend; q0 += kWave) {
      const int q = q0 + lane;
      const int64_t base = tg.a0 + 4 * (int64_t)q;
      const float4 d = ld_span(e, tg, sp, q);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool valid = (q < sp.qend) && (base + c >= tg.lo) && (base + c < tg.hi);
        const uint32_t key = key_of(comp(d, c));
        f(key, valid && (key >> 20) == b1);
      }
    }
  }
}

// ---- B ----------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void topk_cand_kernel(const Ws ws, int w0) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t out[3], scratch[4];
  __shared__ uint2 stage[4][kSubCap];
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const WaveSpan span = wave_span(tg, wave);
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  SelState* sp = ws.sel + wl;
  const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  const int64_t slot4 = ((int64_t)w * ws.n_ftiles + blockIdx.x) * 4 + wave;
  // the first data is requested before the bin search so that the two latencies overlap
  float4 cur = ld_span(e, tg, span, span.qbeg + lane);
  // the bin that holds the k-th largest key of this (worker, layer)
  if (tid < 3) out[tid] = 0;
  hist_load(hist, ws.hist1 + wl * kHistBins, kHistBins);
  const uint32_t k = (uint32_t)L.k[ws.level[ft.layer]];
  pick_bin(hist, k, out, scratch);
  const uint32_t b1 = out[0];
  if (ft.start == 0 && tid == 0) {
    sp->b1 = out[0]; sp->above1 = out[1]; sp->c1 = out[2]; sp->k = k;
  }
  for (int b = tid; b < kHistBins; b += kFlatThreads) hist[b] = 0;
  __syncthreads();
  uint32_t n_gt = 0, n_c = 0;                              // wave-uniform
  for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
    const int q = q0 + lane;
    const float4 nxt = ld_span(e, tg, span, q + kWave);
    const int64_t base = tg.a0 + 4 * (int64_t)q;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const bool valid = (q < span.qend) && (base + c >= tg.lo) && (base + c < tg.hi);
      const uint32_t key = key_of(comp(cur, c));
      const uint32_t bin = key >> 20;
      n_gt += (uint32_t)__popcll(__ballot(valid && bin > b1));
      const bool cand = valid && bin == b1;
      const uint64_t m = __ballot(cand);
      if (m != 0) {
        const uint32_t pos = n_c + lanes_below(m, lane);
        if (cand && pos < (uint32_t)kSubCap)
          stage[wave][pos] = make_uint2(key, (uint32_t)(base + c - L.offset));
        n_c += (uint32_t)__popcll(m);
      }
    }
    cur = nxt;
  }
  if (lane == 0) {
    ws.gt4[slot4] = n_gt;
    ws.cand_n[slot4] = n_c;
    if (n_c > (uint32_t)kSubCap) sp->mode = 1;             // segment overflow: re-read path
  }
  __syncthreads();                                         // staged candidates are visible
  if (n_c <= (uint32_t)kSubCap) {
    // level-2 histogram and the segment from the compacted list (coalesced stores)
    uint2* seg = ws.cand + slot4 * kSubCap;
    for (uint32_t i = lane; i < n_c; i += kWave) {
      const uint2 c = stage[wave][i];
      atomicAdd(&hist[(c.x >> 9) & 0x7ffu], 1u);
      seg[i] = c;
    }
  } else {
    // more candidates than slots (huge tie class): the histogram still has to count them all
    for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
      const int q = q0 + lane;
      const int64_t base = tg.a0 + 4 * (int64_t)q;
      const float4 d = ld_span(e, tg, span, q);
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool valid = (q < span.qend) && (base + c >= tg.lo) && (base + c < tg.hi);
        const uint32_t key = key_of(comp(d, c));
        hist_add(hist, valid && (key >> 20) == b1, (key >> 9) & 0x7ffu, lane);
      }
    }
  }
  __syncthreads();
  hist_flush(hist, ws.hist2 + wl * kHistBins, kHistBins);
}

// ---- C ----------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void topk_level3_kernel(const Ws ws, int w0) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t out[3], scratch[4];
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  SelState* sp = ws.sel + wl;
  const uint32_t b1 = sp->b1, mode = sp->mode;
  // level-2 bin of the k-th largest: k - above1 are still needed from bin b1
  if (tid < 3) out[tid] = 0;
  hist_load(hist, ws.hist2 + wl * kHistBins, kHistBins);
  pick_bin(hist, sp->k - sp->above1, out, scratch);
  const uint32_t b2 = out[0];
  if (ft.start == 0) {
    if (tid == 0) { sp->b2 = out[0]; sp->above2 = out[1]; }
    hist_clear_global(ws.hist1 + wl * kHistBins, kHistBins);   // every reader of hist1 is done
  }
  for (int b = tid; b < 512; b += kFlatThreads) hist[b] = 0;
  __syncthreads();
  uint32_t n_gt = 0;
  for_wave_candidates(ws, L, tg, w, blockIdx.x, wave, lane, mode, b1, [&](uint32_t key, bool valid) {
    const uint32_t bb = (key >> 9) & 0x7ffu;
    n_gt += (uint32_t)__popcll(__ballot(valid && bb > b2));
    if (valid && bb == b2) atomicAdd(&hist[key & 0x1ffu], 1u);
  });
  const int64_t slot4 = ((int64_t)w * ws.n_ftiles + blockIdx.x) * 4 + wave;
  if (lane == 0) ws.gt4[slot4] += n_gt;
  __syncthreads();
  hist_flush(hist, ws.hist3 + wl * 512, 512);
}

// ---- D ----------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void topk_count_kernel(const Ws ws, int w0) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t out[3], scratch[4], tot[2][4];
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  SelState* sp = ws.sel + wl;
  const uint32_t b1 = sp->b1, b2 = sp->b2, mode = sp->mode;
  // exact threshold: k - above1 - above2 are still needed from bin (b1, b2)
  if (tid < 3) out[tid] = 0;
  hist_load(hist, ws.hist3 + wl * 512, 512);
  const uint32_t k2 = sp->k - sp->above1 - sp->above2;
  pick_bin(hist, k2, out, scratch);
  const uint32_t T = (b1 << 20) | (b2 << 9) | out[0];
  if (ft.start == 0) {
    if (tid == 0) {
      sp->T = T;
      sp->ktie = k2 - out[1];                              // 1 <= ktie <= entries equal to T
      sp->alleq = (k2 - out[1] == out[2]) ? 1u : 0u;
    }
    hist_clear_global(ws.hist2 + wl * kHistBins, kHistBins);
  }
  uint32_t n_gt = 0, n_eq = 0;
  for_wave_candidates(ws, L, tg, w, blockIdx.x, wave, lane, mode, b1, [&](uint32_t key, bool valid) {
    const bool in_b2 = valid && ((key >> 9) & 0x7ffu) == b2;   // bins above b2 were counted in C
    n_gt += (uint32_t)__popcll(__ballot(in_b2 && key > T));
    n_eq += (uint32_t)__popcll(__ballot(in_b2 && key == T));
  });
  const int64_t slot4 = ((int64_t)w * ws.n_ftiles + blockIdx.x) * 4 + wave;
  if (lane == 0) {
    const uint32_t g = ws.gt4[slot4] + n_gt;
    ws.gt4[slot4] = g;
    ws.eq4[slot4] = n_eq;
    tot[0][wave] = g;
    tot[1][wave] = n_eq;
  }
  __syncthreads();
  if (tid == 0) {
    const int64_t tslot = (int64_t)w * ws.tile_stride + L.toff + (ft.start >> kTileShift);
    ws.gt_cnt[tslot] = tot[0][0] + tot[0][1] + tot[0][2] + tot[0][3];
    ws.eq_cnt[tslot] = tot[1][0] + tot[1][1] + tot[1][2] + tot[1][3];
  }
}

// ---- E ----------------------------------------------------------------------------------------

__global__ __launch_bounds__(256) void topk_compact_kernel(const Ws ws, int w0) {
  __shared__ uint32_t red[4];
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const WaveSpan span = wave_span(tg, wave);
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  const SelState* sp = ws.sel + wl;
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  float4 cur = ld_span(e, tg, span, span.qbeg + lane);
  const uint32_t T = sp->T, ktie = sp->ktie, alleq = sp->alleq, kk = sp->k;
  // ties and selected entries before my wave's quarter.  The tie quota is used up in index
  // order, so everything before a point took min(ktie, ties before that point) ties in total.
  const int my_t = ft.start >> kTileShift;
  const int64_t tbase = (int64_t)w * ws.tile_stride + L.toff;
  uint32_t s_eq = 0, s_gt = 0;
  for (int t = tid; t < my_t; t += kFlatThreads) {
    s_eq += ws.eq_cnt[tbase + t];
    s_gt += ws.gt_cnt[tbase + t];
  }
  const uint32_t eq_base = block_sum_u32(s_eq, red);
  const uint32_t gt_base = block_sum_u32(s_gt, red);
  if (tid == 0) {
    ws.sel_off[tbase + my_t] = gt_base + min(ktie, eq_base);   // read by the payload mean
    if (my_t == L.ntiles - 1) ws.sel_off[tbase + L.ntiles] = kk;
  }
  if (ft.start == 0) hist_clear_global(ws.hist3 + wl * 512, 512);
  const int64_t slot4 = ((int64_t)w * ws.n_ftiles + blockIdx.x) * 4;
  uint32_t eq_run = eq_base, gt_before = gt_base;
  for (int v = 0; v < wave; ++v) { eq_run += ws.eq4[slot4 + v]; gt_before += ws.gt4[slot4 + v]; }
  uint32_t pos_run = gt_before + min(ktie, eq_run);

  int32_t* pidx = ws.pay_idx + (int64_t)w * ws.pay_stride + L.pay_off;
  float* pval = ws.pay_val + (int64_t)w * ws.pay_stride + L.pay_off;
  for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
    const int q = q0 + lane;
    const float4 nxt = ld_span(e, tg, span, q + kWave);
    const int64_t base = tg.a0 + 4 * (int64_t)q;
    bool sel[4];
    uint32_t key[4];
    bool valid[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      valid[c] = (q < span.qend) && (base + c >= tg.lo) && (base + c < tg.hi);
      key[c] = key_of(comp(cur, c));
    }
    if (alleq) {
#pragma unroll
      for (int c = 0; c < 4; ++c) sel[c] = valid[c] && key[c] >= T;
    } else {
      uint32_t below = 0, total = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint64_t m = __ballot(valid[c] && key[c] == T);
        below += lanes_below(m, lane);
        total += (uint32_t)__popcll(m);
      }
      uint32_t rank = eq_run + below;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool iseq = valid[c] && key[c] == T;
        sel[c] = valid[c] && (key[c] > T || (iseq && rank < ktie));
        rank += iseq ? 1u : 0u;
      }
      eq_run += total;
    }
    uint32_t below = 0, total = 0;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint64_t m = __ballot(sel[c]);
      below += lanes_below(m, lane);
      total += (uint32_t)__popcll(m);
    }
    if (total != 0) {
      uint32_t pos = pos_run + below;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        if (sel[c]) {
          if (pos < kk) {                          // always true for consistent state
            pidx[pos] = (int32_t)(base + c - L.offset);
            pval[pos] = comp(cur, c);
          }
          e[base + c] = 0.f;
          ++pos;
        }
      }
      pos_run += total;
    }
    cur = nxt;
  }
}

// ---- K6: dense mean of the W payloads --------------------------------------------------------

__global__ __launch_bounds__(256) void topk_sparse_mean_kernel(const Ws ws, float* __restrict__ out) {
  __shared__ float acc[kTile];
  const int tid = threadIdx.x;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  if (blockIdx.x == 0 && tid == 0) {
    ws.words[1] = ws.words[0];
    ws.words[2] += ws.words[0];
  }
  for (int i = tid; i < kTile; i += kFlatThreads) acc[i] = 0.f;
  __syncthreads();
  const int tl = ft.start >> kTileShift;
  for (int w = 0; w < ws.W; ++w) {
    const int64_t tslot = (int64_t)w * ws.tile_stride + L.toff + tl;
    const uint32_t lo = ws.sel_off[tslot], hi = ws.sel_off[tslot + 1];
    const int32_t* pidx = ws.pay_idx + (int64_t)w * ws.pay_stride + L.pay_off;
    const float* pval = ws.pay_val + (int64_t)w * ws.pay_stride + L.pay_off;
    const uint32_t kk = ws.sel[(int64_t)w * ws.L + ft.layer].k;
    for (uint32_t p = lo + tid; p < hi && p < kk; p += kFlatThreads) {
      const int32_t i = pidx[p] - ft.start;
      if (i >= 0 && i < ft.count) acc[i] += pval[p];   // indices are unique within a worker
    }
    __syncthreads();                             // workers are added in order
  }
  const float fw = (float)ws.W;
  for (int q = tid; q < tg.nquads; q += kFlatThreads) {
    const int64_t base = tg.a0 + 4 * (int64_t)q;
    float4 v;
    const int64_t i0 = base - tg.lo;
    v.x = (i0 + 0 >= 0 && i0 + 0 < ft.count) ? acc[i0 + 0] / fw : 0.f;
    v.y = (i0 + 1 >= 0 && i0 + 1 < ft.count) ? acc[i0 + 1] / fw : 0.f;
    v.z = (i0 + 2 >= 0 && i0 + 2 < ft.count) ? acc[i0 + 2] / fw : 0.f;
    v.w = (i0 + 3 >= 0 && i0 + 3 < ft.count) ? acc[i0 + 3] / fw : 0.f;
    st_quad(out, base, tg.lo, tg.hi, v);
  }
}

}  // namespace acc
