// Shared device-side definitions of the Accordion hot-path kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace acc {

constexpr int kWave = 64;
constexpr int kFlatThreads = 256;        // workgroup of every flat-tile kernel
constexpr int kTile = 8192;              // elements per flat tile (power of two)
constexpr int kTileShift = 13;
constexpr int kQuadIters = (kTile / 4 + 1 + kFlatThreads - 1) / kFlatThreads;  // 9
constexpr int kMatRows = 64;             // matrix tile: 64 rows x 256 columns
constexpr int kMatCols = 256;
constexpr int kHistBins = 2048;          // 11 key bits per radix level
constexpr int kSubCap = 256;             // candidate slots per wave quarter of a flat tile (TopK)
constexpr int kSegCap = 4 * kSubCap;    // candidate slots per flat tile
constexpr int kMaxW = 32;
constexpr int kMaxRank = 4;

// One layer as the kernels see it.  Built on the host at init, read-only afterwards.
struct LayerDev {
  int64_t offset;        // first element in the flat buffers
  int32_t rows, cols;
  int32_t is_matrix;     // 1: PowerSGD compresses it
  int32_t vec4;          // 1: every row start is 16-byte aligned and cols % 4 == 0
  int32_t rank[2];       // effective rank at level 0 (non-critical) / 1 (critical)
  int32_t k[2];          // TopK kept count at level 0 / 1
  int32_t n_colchunks;   // ceil(cols / kMatCols)
  int32_t n_rowblocks;   // ceil(rows / kMatRows)
  int32_t tile0;         // first flat tile of the layer
  int32_t ntiles;        // number of flat tiles
  int32_t toff;          // slot of tile 0 in the per-worker tile arrays (tile0 + layer index)
  int32_t pad0;
  int64_t q_off;         // into Q      (cols * rmax floats)
  int64_t p_off;         // into Phat   (rows * rmax floats)
  int64_t ppart_off;     // into one worker's P partials (n_colchunks * rows * rmax)
  int64_t qpart_off;     // into one worker's Q partials (n_rowblocks * cols * rmax)
  int64_t pay_off;       // into one worker's payload arrays (entries)
  int64_t vec_off;       // into the 1-D mean buffer (PowerSGD, 1-D layers)
};

struct FlatTile { int32_t layer, start, count, pad; };
struct MatTile { int32_t layer, row0, col0, pad; };
struct QTile { int32_t layer, col0; };

// Per (worker, layer) state of the TopK selection of the current step.
struct SelState {
  uint32_t b1;        // level-1 bin (key bits 30..20) that holds the k-th largest key
  uint32_t above1;    // entries in bins above b1 (all selected)
  uint32_t c1;        // entries in bin b1 (candidates)
  uint32_t mode;      // 0: candidates are in the tiles' segments; 1: a segment overflowed,
                      //    candidates are re-read from Delta
  uint32_t b2;        // level-2 bin (key bits 19..9) within b1
  uint32_t above2;    // candidates in level-2 bins above b2
  uint32_t T;         // exact threshold key (the k-th largest)
  uint32_t ktie;      // how many entries with key == T are selected (lowest indices first)
  uint32_t alleq;     // 1: every entry with key == T is selected
  uint32_t k;         // kept count used by this step
  uint32_t pad[2];
};

struct GradPtrs { const float* p[kMaxW]; };

// Everything the kernels need, passed by value.
struct Ws {
  const LayerDev* layers;
  int32_t* level;              // per layer, 1 = critical
  float* norm_old;             // per layer
  float* norm_prev;            // old norm the last decision used
  float* norm_curr;
  int32_t* has_old;
  int32_t* rank_used;          // per layer, rank of the last PowerSGD step
  unsigned long long* words;   // [0] per step at current levels, [1] last step, [2] cumulative
  float* A;                    // accumulated gradient, N
  float* e;                    // W x e_stride error memory (holds Delta during a step)
  int64_t e_stride;
  double* norm_part;           // per flat tile
  const FlatTile* ftiles;
  const MatTile* mtiles;
  const QTile* qtiles;
  const int32_t* vectiles;     // flat-tile ids of 1-D layers (PowerSGD)
  const int32_t* matlayers;    // layer ids of matrix layers (PowerSGD)
  // PowerSGD
  float* Q;
  float* Phat;
  float* Ppart;  int64_t ppart_stride;
  float* Qpart;  int64_t qpart_stride;
  float* vecmean;
  // TopK
  uint32_t* hist1;             // W x L x kHistBins, zero between steps
  uint32_t* hist2;             // W x L x kHistBins, zero between steps
  uint32_t* hist3;             // W x L x 512, zero between steps
  SelState* sel;               // W x L
  uint2* cand;                 // W x n_ftiles x 4 x kSubCap candidate slots (key, layer-local index)
  uint32_t* cand_n;            // W x n_ftiles x 4 candidates found per wave quarter
  uint32_t* gt4;               // W x n_ftiles x 4 entries above the threshold per wave quarter
  uint32_t* eq4;               // W x n_ftiles x 4 entries equal to the threshold per wave quarter
  uint32_t* gt_cnt;            // W x tile_stride, per tile
  uint32_t* eq_cnt;            // W x tile_stride, per tile
  uint32_t* sel_off;           // W x tile_stride, payload position of a tile's first entry
  int64_t tile_stride;
  int32_t* pay_idx;  float* pay_val;  int64_t pay_stride;
  int64_t N;
  int32_t W, L, rmax;
  int32_t n_ftiles, n_mtiles, n_qtiles, n_vectiles, n_mat;
  float eta;
};

// ---- wave64 helpers ---------------------------------------------------------------

template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __builtin_bit_cast(
      float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum over the 64 lanes, same value (bit for bit) returned to every lane.
// All 64 lanes must be active.  Order: quads, 8, 16 by DPP, then the four rows.
__device__ __forceinline__ float wave_sum(float v) {
  v += dpp_f<0xB1>(v);    // quad_perm [1,0,3,2]
  v += dpp_f<0x4E>(v);    // quad_perm [2,3,0,1]
  v += dpp_f<0x141>(v);   // row_half_mirror
  v += dpp_f<0x140>(v);   // row_mirror
  const int b = __builtin_bit_cast(int, v);
  const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
  const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
  const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
  const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
  return (r0 + r1) + (r2 + r3);
}

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) v += __shfl_xor(v, d, kWave);
  return v;
}

__device__ __forceinline__ uint32_t wave_sum_u32(uint32_t v) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) v += (uint32_t)__shfl_xor((int)v, d, kWave);
  return v;
}

// Inclusive prefix sum over lanes 0..lane.
__device__ __forceinline__ uint32_t wave_incl_scan_u32(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint32_t y = (uint32_t)__shfl_up((int)v, d, kWave);
    if (lane >= d) v += y;
  }
  return v;
}

// Inclusive suffix sum over lanes lane..63.
__device__ __forceinline__ uint32_t wave_incl_suffix_u32(uint32_t v, int lane) {
#pragma unroll
  for (int d = 1; d < kWave; d <<= 1) {
    uint32_t y = (uint32_t)__shfl_down((int)v, d, kWave);
    if (lane + d < kWave) v += y;
  }
  return v;
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, int lane) {
  return (uint32_t)__popcll(mask & ((1ull << lane) - 1ull));
}

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

// ---- masked 16-byte access on a flat buffer ---------------------------------------
// base is a multiple of 4 (elements) and the buffer is 16-byte aligned; elements outside
// [lo, hi) are neither read nor written.

__device__ __forceinline__ float4 ld_quad(const float* __restrict__ p, int64_t base, int64_t lo,
                                          int64_t hi) {
  if (base >= lo && base + 4 <= hi) return *reinterpret_cast<const float4*>(p + base);
  float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
  if (base + 0 >= lo && base + 0 < hi) v.x = p[base + 0];
  if (base + 1 >= lo && base + 1 < hi) v.y = p[base + 1];
  if (base + 2 >= lo && base + 2 < hi) v.z = p[base + 2];
  if (base + 3 >= lo && base + 3 < hi) v.w = p[base + 3];
  return v;
}

__device__ __forceinline__ void st_quad(float* __restrict__ p, int64_t base, int64_t lo, int64_t hi,
                                        float4 v) {
  if (base >= lo && base + 4 <= hi) {
    *reinterpret_cast<float4*>(p + base) = v;
    return;
  }
  if (base + 0 >= lo && base + 0 < hi) p[base + 0] = v.x;
  if (base + 1 >= lo && base + 1 < hi) p[base + 1] = v.y;
  if (base + 2 >= lo && base + 2 < hi) p[base + 2] = v.z;
  if (base + 3 >= lo && base + 3 < hi) p[base + 3] = v.w;
}

__device__ __forceinline__ float comp(const float4& v, int c) {
  return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

// Geometry of one flat tile in absolute element indices.
struct TileGeom {
  int64_t lo, hi;   // the tile's elements: [lo, hi)
  int64_t a0;       // lo rounded down to a multiple of 4
  int32_t nquads;   // 16-byte groups that intersect [lo, hi)
};

__device__ __forceinline__ TileGeom tile_geom(const LayerDev& L, const FlatTile& t) {
  TileGeom g;
  g.lo = L.offset + t.start;
  g.hi = g.lo + t.count;
  g.a0 = g.lo & ~int64_t(3);
  g.nquads = (int32_t)((g.hi - g.a0 + 3) >> 2);
  return g;
}

}  // namespace acc
