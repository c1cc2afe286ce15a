// Shared device-side definitions of the Accordion hot-path kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace acc {

constexpr int kWave = 64;
constexpr int kFlatThreads = 256;        // workgroup of every flat-tile kernel
constexpr int kTile = 8192;              // elements per flat tile (power of two)
constexpr int kTileShift = 13;
constexpr int kT2Group = 16;             // TopK: consecutive tiles of a layer that add their level-2 counts into one slot
constexpr int kQuadIters = (kTile / 4 + 1 + kFlatThreads - 1) / kFlatThreads;  // 9
constexpr int kMatRows = 64;             // matrix tile: 64 rows x 256 columns
constexpr int kMatCols = 256;
constexpr int kQRows = 128;              // rows of a tile of the right product Q = Delta^T P^ (64: 5 us slower on
                                         // ResNet-18 shapes, twice the partial sums; 256: too few workgroups at W = 1)
constexpr int kHistBins = 2048;          // 11 key bits per radix level
// a wave quarter has at most ceil((kTile / 4 + 1) / 4) 16-byte groups: iterations of 64 lanes
constexpr int kSpanIters = ((kTile / 4 + 1 + 3) / 4 + kWave - 1) / kWave;   // 9
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
  int32_t n_rowblocks;   // ceil(rows / kQRows)
  int32_t tile0;         // first flat tile of the layer
  int32_t ntiles;        // number of flat tiles
  int32_t t2slot0;       // TopK: the layer's first slot in a worker's level-2 count array (one slot per kT2Group tiles)
  int32_t mt0;           // PowerSGD matrix layer: its first 64 x 256 matrix tile (it has n_colchunks * ceil(rows / 64))
  int64_t qoff;          // slot of the layer's first wave quarter in the per-worker quarter arrays
                         // (4 * tile0 + layer index: one spare slot per layer for the totals)
  int64_t q_off;         // into Q      (cols rows of kMaxRank floats, zero beyond rmax)
  int64_t p_off;         // into Phat   (rows * rmax floats)
  int64_t ppart_off;     // into one worker's P partials (n_colchunks * rows * rmax doubles)
  int64_t qpart_off;     // into one worker's Q partials (n_rowblocks * cols * rmax doubles)
  int64_t pay_off;       // into one worker's payload arrays (entries)
  int64_t vec_off;       // into the 1-D mean buffer (PowerSGD, 1-D layers)
};

// qslot0: slot of the tile's first wave quarter in a worker's per-quarter arrays (the layer's qoff +
// 4 * tile within the layer), so that a kernel can request them before it has the layer's entry.
struct FlatTile { int32_t layer, start, count, qslot0; };
struct MatTile { int32_t layer, row0, col0, pad; };
struct QTile { int32_t layer, col0; };
struct PTile { int32_t layer, row0; };   // a block of rows of a matrix layer's P (PowerSGD, mean over workers)

// Per (worker, layer) state of the TopK selection of the current step.
struct SelState {
  uint32_t b1;        // level-1 bin (key bits 30..20) that holds the k-th largest key
  uint32_t need2;     // entries still to be taken from bin b1
  uint32_t mode;      // 0: b1 is one of the guessed bins (or decided); 1: the guess missed
  uint32_t side;      // which of the guessed bins b1 is (0: the lowest)
  uint32_t b2;        // level-2 bin (key bits 19..14) within b1
  uint32_t need3;     // entries still to be taken from bin (b1, b2)
  uint32_t zeros;     // exact zeros of the layer (filled in when b1 == 0)
  uint32_t bin0;      // entries of level-1 bin 0 (exact zeros and the smallest denormals) in this step's Delta
  uint32_t k;         // kept count used by this step
  uint32_t T;         // exact threshold key (the k-th largest)
  uint32_t ktie;      // how many entries with key == T are selected (lowest indices first)
  uint32_t alleq;     // 1: every entry with key == T is selected
  uint32_t fresh_nnz; // entries outside bin 0 in the last step whose threshold lay in bin 0 (everything
                      //   non-zero was kept then, so these were the gradient's own); 0: no such step yet.
                      //   Only steers the next guess.
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
  unsigned long long* words;   // [0] per step at current levels, [1] last step, [2] cumulative,
                               // [3] steps in the current detection window (MSDR detector)
  unsigned long long* stats;   // TopK diagnostics: [0] (worker, layer) pairs re-staged, [1] decided by sweeps
  float* A;                    // accumulated gradient, N
  float* e;                    // W x e_stride error memory (holds Delta during a step)
  int64_t e_stride;
  double* norm_part;           // per flat tile: sum of squares of A (kept up to date by the pass that adds the gradient)
  double* norm_part_m;         // PowerSGD: the same per 64 x 256 matrix tile
  uint32_t* a_fresh;           // one word: nonzero = the accumulation window has just restarted: A counts as zero
                               //   (the next pass over it stores the gradient instead of adding it)
  double* sq_part;             // per flat tile: sum over the window of ||g_0||^2 (MSDR detector)
  const FlatTile* ftiles;
  const MatTile* mtiles;
  const MatTile* qmtiles;      // kQRows x 256 tiles of the matrix layers (right product)
  const QTile* qtiles;
  const int32_t* vectiles;     // flat-tile ids of 1-D layers (PowerSGD)
  const int32_t* matlayers;    // layer ids of matrix layers (PowerSGD)
  // PowerSGD
  float* Q;
  float* Phat;
  double* Ppart; int64_t ppart_stride;   // per worker and 256-column chunk: that chunk's share of P_w, fp64
  double* Pwork;               // p_total doubles: working columns of the orthogonalisation of tall layers
  const PTile* ptiles;         // row blocks of the matrix layers (mean of P)
  double* Qpart; int64_t qpart_stride;   // per worker and 64-row block: that block's share of Q_w, fp64
  float* vecmean;
  uint32_t* pending;           // one word: workers whose e still holds Delta (residual not formed yet)
  // TopK
  uint32_t* hist1;             // W x L x kHistBins, zero between steps
  uint32_t* t2;                // W x n_t2slots x 640: level-2 counts of the ten guessed bins, summed over kT2Group tiles
  uint32_t* qlist;             // W x q_stride x kQListCap: per quarter, its keys in bin (b1, b2)
  SelState* sel;               // W x L
  uint32_t* hist2m;            // W x L x 64: level-2 counts of b1 of a layer whose guess missed
  uint32_t* lflag;             // L: nonzero = this step's compaction of the layer reads Delta (some worker's guess
                               //   missed, or the guess was a band), not the candidate lists
  uint2* b1hist;               // W x L x 2 (level): {b1 | (last move + 64) << 16 | steps at rest << 24, step number} of the last step at this level
  uint32_t* guess;             // W x L x 2 (level): lowest guessed level-1 bin | number of bins << 16, or a special value
  uint4* qinfo;                // W x q_stride: per wave quarter {entries above what is listed (one-bin and band
                               //   lists), listed entries, 0, exact zeros (one-bin and zero-guess lists)}
  uint32_t* cand_val;          // W x q_stride x kCandCap: per wave quarter, the values of its candidates (or keys of one bin)
  uint16_t* cand_idx;          // W x q_stride x kCandCap: ... and their offsets inside the quarter
  uint32_t* gtq;               // W x q_stride entries above the threshold per quarter
  uint32_t* eqq;               // W x q_stride keys in bin (b1, b2) / entries equal to the threshold per quarter
  uint32_t* gtpre;             // W x q_stride exclusive prefix of gtq within the layer (+ total)
  uint32_t* eqpre;             // W x q_stride exclusive prefix of eqq within the layer (+ total)
  int64_t q_stride;
  int64_t n_qslots;            // W * q_stride: all quarter slots (the stride between the chunks of a candidate list)
  int32_t* pay_idx;  float* pay_val;  int64_t pay_stride;
  unsigned long long* overlap; // L per-layer counters of the overlap read-back
  uint32_t* tpending;          // one word: workers whose e still holds Delta with the kept entries in it
  // batch-size mode
  uint32_t* bstate;            // two slots of four words, used alternately (micro-step parity)
  int32_t bmult, bmono;        // micro-steps per large batch; 1: the batch only grows
  int64_t n_model;             // elements that belong to a layer
  int64_t N;
  int32_t W, L, rmax;
  int32_t n_ftiles, n_mtiles, n_qmtiles, n_qtiles, n_vectiles, n_mat, n_ptiles;
  int32_t n_t2slots;           // TopK: slots of t2 per worker
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

template <int CTRL>
__device__ __forceinline__ double dpp_d(double v) {
  const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), CTRL, 0xf, 0xf, false);
  const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), CTRL, 0xf, 0xf, false);
  return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double readlane_d(double v, int l) {
  return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), l),
                          __builtin_amdgcn_readlane(__double2loint(v), l));
}

// fp64 sum over the 64 lanes in the order of wave_sum (lane exchanges through DPP moves, no LDS
// traffic), same value returned to every lane.  All 64 lanes must be active.
__device__ __forceinline__ double wave_sum_d(double v) {
  v += dpp_d<0xB1>(v);
  v += dpp_d<0x4E>(v);
  v += dpp_d<0x141>(v);
  v += dpp_d<0x140>(v);
  return (readlane_d(v, 0) + readlane_d(v, 16)) + (readlane_d(v, 32) + readlane_d(v, 48));
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

// Lane mask of a predicate, taken straight from the compare (no round trip through a register
// holding 0 / 1).
__device__ __forceinline__ uint64_t ballot64(bool p) { return __builtin_amdgcn_ballot_w64(p); }

// Number of set bits of mask in the lanes below the calling lane.
__device__ __forceinline__ uint32_t lanes_below(uint64_t mask, int /*lane*/) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// The calling lane's bit of a wave-uniform lane mask, as a predicate (the mask itself becomes the
// condition of the instruction that uses it; no per-lane shift).
__device__ __forceinline__ bool lane_bit(uint64_t mask) { return __builtin_amdgcn_inverse_ballot_w64(mask); }

// A wave-uniform value, moved to a scalar register.
__device__ __forceinline__ uint32_t rfl(uint32_t v) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)v); }

// Keeps a lane mask in scalar registers across a join of control flow (otherwise the compiler
// carries the predicate behind it per lane, as a 0 / 1 vector value it has to compare again).
__device__ __forceinline__ uint64_t scalar_mask(uint64_t mask) {
  asm volatile("" : "+s"(mask));
  return mask;
}

__device__ __forceinline__ uint32_t key_of(float v) { return __float_as_uint(v) & 0x7fffffffu; }

__device__ __forceinline__ double sq4(const float4& a) {
  double s = (double)a.x * (double)a.x;
  s += (double)a.y * (double)a.y;
  s += (double)a.z * (double)a.z;
  s += (double)a.w * (double)a.w;
  return s;
}

// Sum over the workgroup's four waves of one fp64 value per lane; the result is valid in thread 0.
// Every thread calls it (one barrier).
__device__ __forceinline__ double block_sum4_d(double s, double* red4) {
  s = wave_sum_d(s);
  if ((threadIdx.x & 63) == 0) red4[threadIdx.x >> 6] = s;
  __syncthreads();
  return (red4[0] + red4[1]) + (red4[2] + red4[3]);
}

// Folding sums of two values over the wave (gfx950 lane swaps): the result holds, in the lower 32
// lanes (fold32) / the even rows of 16 lanes (fold16), the sum of a over the two halves that are
// folded together, and in the upper 32 lanes / the odd rows the same sum of b.  All lanes active.
typedef unsigned int u2v __attribute__((ext_vector_type(2)));
__device__ __forceinline__ double fold32_d(double a, double b) {
  const u2v lo = __builtin_amdgcn_permlane32_swap((unsigned)__double2loint(a), (unsigned)__double2loint(b), false, false);
  const u2v hi = __builtin_amdgcn_permlane32_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(b), false, false);
  return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
__device__ __forceinline__ double fold16_d(double a, double b) {
  const u2v lo = __builtin_amdgcn_permlane16_swap((unsigned)__double2loint(a), (unsigned)__double2loint(b), false, false);
  const u2v hi = __builtin_amdgcn_permlane16_swap((unsigned)__double2hiint(a), (unsigned)__double2hiint(b), false, false);
  return __hiloint2double((int)hi[0], (int)lo[0]) + __hiloint2double((int)hi[1], (int)lo[1]);
}
// Sum over each row of 16 lanes, returned to all its lanes.
__device__ __forceinline__ double row_sum_d(double v) {
  v += dpp_d<0xB1>(v);
  v += dpp_d<0x4E>(v);
  v += dpp_d<0x141>(v);
  v += dpp_d<0x140>(v);
  return v;
}

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

// Streaming ("non-temporal") 16-byte access: for data that this step reads or writes once and no
// later kernel of the step touches (the gradients coming in, the averaged gradient and the payload
// going out), so that it does not push the error memory out of the caches or sit there dirty
// until the kernel ends.
typedef float f4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 ld16_stream(const float* p) {
  const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st16_stream(float* p, const float4& v) {
  f4v t;
  t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
  __builtin_nontemporal_store(t, reinterpret_cast<f4v*>(p));
}

// Access to 16-byte group q of a tile.  AL (a workgroup-uniform property of the tile): the tile
// starts on a 16-byte boundary and holds a whole number of groups, so no element needs a mask.
// STREAM: non-temporal access on the mask-free path (the masked path is rare and stays plain).
template <bool AL, bool STREAM = false>
__device__ __forceinline__ float4 ldq(const float* __restrict__ p, int64_t a0, int64_t lo, int64_t hi,
                                      int q, bool in) {
  if (!in) return make_float4(0.f, 0.f, 0.f, 0.f);
  if (AL) return STREAM ? ld16_stream(p + a0 + 4 * (int64_t)q) : *reinterpret_cast<const float4*>(p + a0 + 4 * (int64_t)q);
  return ld_quad(p, a0 + 4 * (int64_t)q, lo, hi);
}

// Group q of a tile with AL, loaded whatever lane asks: the caller has clamped q into the tile
// (0 <= q < nquads) and masks what it does with the value.  Costs an integer min / max where
// the predicated load costs four moves of zeros and a branch around the load.
template <bool STREAM = false>
__device__ __forceinline__ float4 ldq_clamped(const float* __restrict__ p, int64_t a0, int q) {
  return STREAM ? ld16_stream(p + a0 + 4 * (int64_t)q) : *reinterpret_cast<const float4*>(p + a0 + 4 * (int64_t)q);
}

template <bool AL, bool STREAM = false>
__device__ __forceinline__ void stq(float* __restrict__ p, int64_t a0, int64_t lo, int64_t hi, int q,
                                    float4 v) {
  if (AL) {
    if (STREAM) st16_stream(p + a0 + 4 * (int64_t)q, v);
    else *reinterpret_cast<float4*>(p + a0 + 4 * (int64_t)q) = v;
  } else {
    st_quad(p, a0 + 4 * (int64_t)q, lo, hi, v);
  }
}

// ---- where the averaged decompressed gradient goes -------------------------------------------
// Either it is written to `out`, or it is consumed on the spot by SGD with Nesterov momentum
// (Appendix A, table "Hyperparameters"; update rule of Section 3) on the weights `wt` and the
// velocity `vel`, and never stored.
struct Sink {
  float* out;
  float* wt;
  float* vel;
  float lr, mu, wd;
  int32_t stream_wv;   // TopK: weights and velocity are accessed with streaming loads / stores
};

// d' = d + wd w (if wd != 0);  v = mu v + d';  w = w - lr (d' + mu v).  Every product and every sum
// is rounded on its own (the library is built with floating-point contraction off), so that the
// result has one definite value.
__device__ __forceinline__ void nesterov(float d, float& w, float& v, float lr, float mu, float wd) {
  if (wd != 0.f) d = d + wd * w;
  v = mu * v + d;
  const float look = d + mu * v;
  w = w - lr * look;
}

__device__ __forceinline__ void nesterov4(const float4& d, float4& w, float4& v, const Sink& s) {
  nesterov(d.x, w.x, v.x, s.lr, s.mu, s.wd);
  nesterov(d.y, w.y, v.y, s.lr, s.mu, s.wd);
  nesterov(d.z, w.z, v.z, s.lr, s.mu, s.wd);
  nesterov(d.w, w.w, v.w, s.lr, s.mu, s.wd);
}

__device__ __forceinline__ float comp(const float4& v, int c) {
  return c == 0 ? v.x : (c == 1 ? v.y : (c == 2 ? v.z : v.w));
}

// Geometry of one flat tile in absolute element indices.
struct TileGeom {
  int64_t lo, hi;   // the tile's elements: [lo, hi)
  int64_t a0;       // lo rounded down to a multiple of 4
  int32_t nquads;   // 16-byte groups that intersect [lo, hi)
  bool aligned;     // lo and hi are multiples of 4: every group is whole
};

__device__ __forceinline__ TileGeom tile_geom(const LayerDev& L, const FlatTile& t) {
  TileGeom g;
  g.lo = L.offset + t.start;
  g.hi = g.lo + t.count;
  g.a0 = g.lo & ~int64_t(3);
  g.nquads = (int32_t)((g.hi - g.a0 + 3) >> 2);
  g.aligned = ((g.lo | g.hi) & 3) == 0;
  return g;
}

}  // namespace acc
