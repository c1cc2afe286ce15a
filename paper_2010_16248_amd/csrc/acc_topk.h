// TopK kernels: exact per-layer selection of the k entries with the largest |Delta|
// (ties: lower flat index) by a radix select on the 31 magnitude bits, organised so that Delta
// is streamed once per step, when it is formed; the passes after that work on lists of CANDIDATES
// that pass leaves.  Key bits: level 1 = 30..20 (2048 bins), level 2 = 19..14 (64), level 3 =
// 13..6 (256), level 4 = 5..0 (64).
//
//   A   topk_ef_hist   Delta = g + e (in place; the entries the previous step kept are dropped
//                      from e first), A += g (worker 0) with its sum of squares, level-1 histogram
//                      per (worker, layer).  The level-1 bin b1 that will hold the k-th largest key
//                      is not known yet, so the pass works on a GUESS (from the previous steps at
//                      this level): every entry at or above the lowest guessed bin goes into its
//                      wave quarter's candidate list as (offset, value), and the tile's level-2
//                      counts of the kGuessBins guessed bins are written.
//   P12 topk_pick12    one workgroup per (worker, layer): b1 from the histogram; if it is one
//                      of the guessed bins, b2 from the sum of the tiles' level-2 counts.
//   C3  topk_count3    one workgroup per tile: per quarter the candidates above cell (b1, b2); the
//                      keys inside the cell go to a short list per quarter.  A layer whose guess
//                      missed is staged again here, from Delta (the keys of b1 only).
//   P3  topk_pick3     per (worker, layer): levels 3 and 4 on the lists, threshold key T and tie
//                      quota; the listed keys are added to their quarters' counts; exclusive
//                      prefix over the quarters = payload position of every quarter; the next
//                      step's guess.
//                      Layers of a single tile, which skip the passes before, are decided here
//                      completely, from Delta, by their own workgroups.
//                      A layer whose guess missed (first step, shifted distribution) or whose
//                      short lists overflowed (huge tie class) is decided here by sweeps of one
//                      workgroup (correct, slow).
//   E   topk_compact   ordered compaction of the selected entries into the payload (index
//                      ascending).  The batched form loops over the workers, forms the dense mean
//                      of the kept values and leaves e as it is (Delta: the next pass A drops the
//                      kept entries); it reads the candidate lists, or Delta where they cannot
//                      serve (a layer with a missed guess, the holes layout or a band guess; a
//                      worker's quarter whose list overflowed or that keeps exact zeros).
//                      The call-by-call form reads Delta and zeroes the kept entries in e.
//   K6  topk_sparse_mean  dense mean of the W payloads (call-by-call path).
//
// The guess only decides which path is taken, never the result.  Cross-workgroup combination
// is by integer atomics and fixed-order sums only, so every output is bit-reproducible.
#pragma once
#include "acc_common.h"

namespace acc {

constexpr uint32_t kNoGuess = 0xffffffffu;
// Guess "the threshold lies in bin 0" (exact zeros and the smallest denormals: sparse gradients of
// which more is kept than is non-zero).  The first pass then lists every non-zero entry as a
// candidate and counts the exact zeros.
constexpr uint32_t kGuessZero = 0xfffffffeu;
constexpr int kPickThreads = 1024;
constexpr int kPickWaves = kPickThreads / kWave;
static_assert(kHistBins == 2 * kPickThreads, "the pick kernels load two histogram bins per thread");
constexpr int kQListCap = 16;            // keys of bin (b1, b2) listed per wave quarter
constexpr int kL2Bins = 64;              // level 2: key bits 19..14
// A guess names kGuessBins adjacent level-1 bins, lo .. lo + kGuessBins - 1 (lo >= 1): the first
// pass lists every entry of bin lo and above as a candidate and counts the level-2 bins of the
// guessed ones.  Bins above the threshold cost no candidates (their entries are kept anyway), so the
// guess always reaches far up; what varies is how far below the expected bin it starts: one bin
// while the threshold rests (no move for two steps in a row), three while it moves -- after a level
// switch the error memory adapts for ten steps or so, during which the threshold moves by one to
// three bins per step (an eighth of an octave each), not quite steadily, and a sparse layer's can
// jump four bins up out of rest.  A deeper start costs more candidates (under error feedback the
// entries pile up just below the threshold: 22 % of them lie within one and a half bins below it
// at K = 10 %, 30 % within three and a half), a missed guess a second read of Delta and a slow
// decision for that layer.
constexpr int kGuessBins = 10, kGuessCalmBelow = 1, kGuessMovingBelow = 3, kGuessRestSteps = 2;
constexpr int kSub2 = kGuessBins * kL2Bins;  // a tile's level-2 counts of the guessed bins
// Where a large part is kept (more than a sixth: the paper's own levels of 25 % and 99 %) the
// entries above the threshold are too many to list: the guess is then a BAND of kBandBins bins, the
// first pass lists the keys inside the band only and counts the entries above it, and the
// compaction reads Delta.  A guess of fewer than kGuessBins bins means exactly that.
constexpr int kBandBins = 8, kBandKeepDiv = 6;
__device__ __forceinline__ int guess_bins_for(uint32_t k, uint32_t n) {
  return (uint64_t)k * kBandKeepDiv > (uint64_t)n ? kBandBins : kGuessBins;
}
__device__ __forceinline__ uint32_t make_guess(int lo, int nb) {
  return (uint32_t)max(1, min(kHistBins - nb, lo)) | ((uint32_t)nb << 16);
}
__device__ __forceinline__ uint32_t guess_lo(uint32_t g) { return g & 0xffffu; }
__device__ __forceinline__ uint32_t guess_nb(uint32_t g) { return g >> 16; }
__device__ __forceinline__ uint32_t bin2_of(uint32_t key) { return (key >> 14) & 0x3fu; }
__device__ __forceinline__ uint32_t bin3_of(uint32_t key) { return (key >> 6) & 0xffu; }
__device__ __forceinline__ uint32_t bin4_of(uint32_t key) { return key & 0x3fu; }

// A load the compiler leaves where it is written.  Plain loads are moved down to their first use,
// behind every branch and every wait on the way: the loads of a quarter's record and list, written
// at the top of the counting kernel, were issued after its chain of seven dependent scalar loads
// instead of beside it, and the first pass read its flags, its level and its guess one after the
// other before it requested any data.  A relaxed atomic load of wavefront scope is the same instruction as a
// plain load and is not moved.
__device__ __forceinline__ uint32_t ld_here(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WAVEFRONT);
}

__device__ __forceinline__ uint32_t ld_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// LDS histogram add.  Keys of bin 0 (the exact zeros -- the one tie class that is common in real
// gradients -- and the smallest denormals) are left out: their number is the layer's size minus
// the other bins.
__device__ __forceinline__ void hist_add(uint32_t* hist, bool valid_not_bin0, uint32_t bin) {
  if (valid_not_bin0) atomicAdd(&hist[bin], 1u);
}

// hist: kHistBins counts in LDS.  Finds the largest bin b with count(bins >= b) >= k.
// Result in out[0..2] (LDS): bin, entries above the bin, entries in the bin.  Every thread of
// the workgroup calls it (two barriers); threads 0..255 own eight bins each.
__device__ __forceinline__ void pick_bin(const uint32_t* hist, uint32_t k, uint32_t* out,
                                         uint32_t* scratch) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const bool owner = tid < 256;
  uint32_t h[8];
  uint32_t part = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) { h[i] = owner ? hist[tid * 8 + i] : 0u; part += h[i]; }
  const uint32_t suf = wave_incl_suffix_u32(part, lane);
  if (owner && lane == 0) scratch[wave] = suf;   // wave total
  if (tid < 3) out[tid] = 0;
  __syncthreads();
  if (owner) {
    uint32_t run = suf - part;                   // entries in bins of later threads of my wave
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
  }
  __syncthreads();
}

// ---- wave quarters --------------------------------------------------------------------------
// Wave v of a 256-thread workgroup owns the contiguous quarter [v*qw, (v+1)*qw) of the tile's
// 16-byte groups, so every count, staged list and running offset is wave-local (scalar
// registers, no barriers, no atomics) and index order is (wave, iteration, lane, component).

struct WaveSpan { int qbeg, qend; };

__device__ __forceinline__ WaveSpan wave_span(const TileGeom& tg, int wave) {
  const int qw = (tg.nquads + 3) >> 2;
  WaveSpan s;
  s.qbeg = wave * qw;
  s.qend = min(s.qbeg + qw, tg.nquads);
  return s;
}

// What is accessed with streaming loads / stores (measured on ResNet-18 shapes, W = 4: the fused
// error-feedback pass drops from 123 to 103 us when the gradients stream in, because the error
// memory then stays in the caches for the compaction).
constexpr bool kStreamG = true;      // gradients: read once per step
constexpr bool kStreamA = true;      // accumulator: read and written once per step
constexpr bool kStreamOut = true;    // averaged gradient: written once, read by nobody here
// Delta stays plain: streaming its store in the first pass changes nothing, and streaming its load
// in the compaction (which then writes the same lines) costs 30 us.

template <bool AL, bool STREAM = false>
__device__ __forceinline__ float4 ld_span(const float* __restrict__ p, const TileGeom& tg,
                                          const WaveSpan& sp, int q) {
  return ldq<AL, STREAM>(p, tg.a0, tg.lo, tg.hi, q, q < sp.qend);
}

// Is element c of group q (which lies in the wave's span iff in_span) an element of the tile?
template <bool AL>
__device__ __forceinline__ bool elem_valid(const TileGeom& tg, int q, int c, bool in_span) {
  if (AL) return in_span;
  const int64_t i = tg.a0 + 4 * (int64_t)q + c;
  return in_span && i >= tg.lo && i < tg.hi;
}

// Lane mask of elem_valid for component c; for an aligned tile it is the span mask m_span.
template <bool AL>
__device__ __forceinline__ uint64_t valid_mask(const TileGeom& tg, int q, int c, bool in_span, uint64_t m_span) {
  if (AL) return m_span;
  return ballot64(elem_valid<AL>(tg, q, c, in_span));
}

// Slot of quarter `wave` of tile `tl` of a layer in the per-worker quarter arrays.
__device__ __forceinline__ int64_t quarter_slot(const Ws& ws, const LayerDev& L, int w, int tl, int wave) {
  return (int64_t)w * ws.q_stride + L.qoff + 4 * (int64_t)tl + wave;
}

// ---- candidate lists ---------------------------------------------------------------------------
// Pass A leaves, per wave quarter, the list of its CANDIDATES: every entry whose level-1 bin is at
// or above the lowest guessed bin, as (offset inside the quarter, value), in index order.  When the
// guess holds, the kept entries are among them, and the passes after it -- the counting kernel, the
// compaction and the mean -- read these 6 bytes per candidate (under error feedback, which piles
// the entries up just below the threshold, 17 to 27 % of the entries at K = 10 % and 8 to 18 % at
// K = 1 %) instead of Delta once more.  A wave collects its candidates in LDS
// and writes them out, consecutive lanes to consecutive addresses, whenever another iteration
// (up to 256 entries) might not fit.  A quarter with more than kCandCap candidates keeps the
// first kCandCap and its full count: whoever reads the list sees the overflow and goes back to
// Delta (and the layer is compacted from Delta).
// The passes that stage ONE bin (bin 0 on a guess, or the bin of a missed guess) use the same
// lists for that bin's keys (no offsets; zeros counted apart).
constexpr int kCandCap = 1024;                   // candidates of a wave quarter kept in device memory
constexpr int kCandLds = 512;                    // a wave's list in LDS
constexpr int kCandLdsSlots = kCandLds + kWave;  // + one slot per lane that takes the writes of unselected elements

struct CandList { uint32_t* val; uint16_t* idx; uint4* qi; };   // qi: the workgroup's four quarter records

// n_lds: entries in the LDS list; n_out: entries already written out (both wave-uniform);
// v_hi, v_nz: per lane, summed over the wave when the quarter is finished.
struct StageCounts { uint32_t n_lds, n_out, v_hi, v_nz; };

// Layout of the lists in device memory: 64-entry chunks, chunk-major -- chunk c of quarter slot q
// is entries (c * n_slots + q) * 64 ... + 63, n_slots = all quarter slots of all workers.  The first
// chunks of all quarters are one dense region, the second chunks the next, and so on: a list
// uses as many chunks as it has entries, so what is touched is dense (a fixed 4 KB slot per quarter
// of which the first KB is used puts all the traffic on a few memory channels: 10 us per step on
// ResNet-18 shapes).
__device__ __forceinline__ int64_t cand_at(const Ws& ws, int64_t qslot, uint32_t chunk, int lane) {
  return ((int64_t)chunk * ws.n_qslots + qslot) * kWave + lane;
}

// Writes the whole 64-entry chunks of the wave's LDS list out (final: the rest too) and moves what
// is left to the front of the list; n_out stays a multiple of 64 until the final call, so every
// store instruction writes one chunk, consecutive lanes to consecutive addresses.
__device__ __forceinline__ void cand_write_out(const Ws& ws, int64_t qslot, const CandList& cl, StageCounts& c,
                                               int lane, bool final) {
  __builtin_amdgcn_wave_barrier();                          // the list is complete (LDS is in order per wave)
  const uint32_t n_full = final ? c.n_lds : (c.n_lds & ~(uint32_t)(kWave - 1));
  for (uint32_t t0 = 0u; t0 < n_full; t0 += kWave) {
    // the last chunk is written whole as well (its tail is whatever the LDS list holds there, and is
    // never read): a store that fills only part of a 64-byte line is a read-modify-write in memory
    const uint32_t t = t0 + lane, chunk = (c.n_out + t0) >> 6;
    if (chunk < (uint32_t)(kCandCap / kWave)) {
      // plain stores: the counting kernel and the compaction read the lists within microseconds
      // (streaming stores here cost the compaction 6 us on ResNet-18 shapes)
      const int64_t a = cand_at(ws, qslot, chunk, lane);
      ws.cand_val[a] = cl.val[t];
      ws.cand_idx[a] = cl.idx[t];
    }
  }
  const uint32_t rest = c.n_lds - n_full;                   // < 64 unless final (then 0)
  uint32_t rv = 0u;
  uint16_t ri = 0;
  if ((uint32_t)lane < rest) { rv = cl.val[n_full + lane]; ri = cl.idx[n_full + lane]; }
  __builtin_amdgcn_wave_barrier();
  if ((uint32_t)lane < rest) { cl.val[lane] = rv; cl.idx[lane] = ri; }
  __builtin_amdgcn_wave_barrier();
  c.n_out += n_full;
  c.n_lds = rest;
}

// Room for one more group of four elements per lane?  Called after every group (wave-uniform).
__device__ __forceinline__ void cand_make_room(const Ws& ws, int64_t qslot, const CandList& cl, StageCounts& c,
                                               int lane) {
  if (c.n_lds > (uint32_t)(kCandLds - 4 * kWave)) cand_write_out(ws, qslot, cl, c, lane, false);
}

// Pass A, one group: the candidates among the four elements of every lane (bins glo and up;
// glo >= 1, so a candidate is never an exact zero, and zeros are not counted: should the
// threshold turn out to lie in bin 0 the guess has missed and the staging after a miss counts
// them).  BAND: only the bins glo .. glo + gnb - 1 are listed, what lies above is counted.
// mv: lane masks of the valid elements
// per component.  i_rel: offset of the lane's first element inside the quarter.  The level-2 counts of
// the kGuessBins guessed bins go to sub2.  Every ballot is taken from a single compare and
// combined with the other masks in scalar registers; the list is in index order.
// ZERO (the guess is bin 0, glo = 0, gnb = 1): every non-zero entry is a candidate, the exact
// zeros are counted, and the level-2 counts are those of the non-zero keys of bin 0.
template <bool MASKED, bool BAND, bool ZERO = false>
__device__ __forceinline__ void stage_candidates(const CandList& cl, uint32_t* sub2, StageCounts& c,
                                                 uint64_t mv0, uint64_t mv1, uint64_t mv2, uint64_t mv3,
                                                 const float4& d, uint32_t glo, uint32_t gnb, uint32_t i_rel,
                                                 int lane) {
  uint32_t key[4], rel[4];
  uint64_t m[4];
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    key[x] = key_of(comp(d, x));
    rel[x] = (key[x] >> 20) - glo;
    const uint64_t mvx = (x == 0 ? mv0 : x == 1 ? mv1 : x == 2 ? mv2 : mv3);
    if (ZERO) {
      m[x] = ballot64(key[x] != 0u);
      c.v_nz += (key[x] == 0u && (!MASKED || lane_bit(mvx))) ? 1u : 0u;
    } else if (BAND) {
      // inside the band: listed; above it: counted (a bin below glo wraps to a huge rel)
      m[x] = ballot64(rel[x] < gnb);
      const bool above = (int32_t)rel[x] >= (int32_t)gnb;
      c.v_hi += (above && (!MASKED || lane_bit(mvx))) ? 1u : 0u;
    } else {
      m[x] = ballot64((int32_t)rel[x] >= 0);
    }
    if (MASKED) m[x] &= mvx;
  }
  if ((m[0] | m[1] | m[2] | m[3]) == 0) return;              // wave-uniform
  uint32_t place = c.n_lds, total = 0u;
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    place = __builtin_amdgcn_mbcnt_hi((uint32_t)(m[x] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m[x], place));
    total += (uint32_t)__popcll(m[x]);
  }
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    const bool sel = lane_bit(m[x]);
    const uint32_t slot = sel ? place : (uint32_t)(kCandLds + lane);
    cl.val[slot] = __float_as_uint(comp(d, x));
    cl.idx[slot] = (uint16_t)(i_rel + x);
    if (sel && rel[x] < gnb) atomicAdd(&sub2[rel[x] * kL2Bins + bin2_of(key[x])], 1u);
    place += sel ? 1u : 0u;
  }
  c.n_lds += total;
}

// The passes that stage one bin: the keys of bin b1 alone, exact zeros left out and counted, the
// entries of the bins above counted.  The caller makes room after every group.
__device__ __forceinline__ void stage_one_bin(const CandList& cl, uint32_t* sub2, StageCounts& c, uint64_t mv,
                                              bool valid, uint32_t key, uint32_t b1, int lane) {
  const uint32_t bin = key >> 20;
  c.v_nz += (valid && key == 0u) ? 1u : 0u;
  c.v_hi += (valid && bin > b1) ? 1u : 0u;
  const uint64_t m = ballot64(bin == b1) & ballot64(key != 0u) & mv;
  if (m != 0) {
    if (valid && bin == b1 && key != 0u) {
      cl.val[c.n_lds + lanes_below(m, lane)] = key;
      atomicAdd(&sub2[bin2_of(key)], 1u);
    }
    c.n_lds += (uint32_t)__popcll(m);
  }
}

// qinfo of the quarter: {entries above the staged bin (one-bin lists; 0 for candidate lists, which
// hold those entries), staged entries (the full count, also beyond kCandCap), 0, exact zeros
// (one-bin lists)}.  Returns the number of exact zeros (the same value in every lane).  The record
// goes to LDS; after a barrier qinfo_flush writes the tile's four records as one 64-byte line.
__device__ __forceinline__ uint32_t stage_finish(const Ws& ws, int64_t qslot, const CandList& cl, StageCounts& c,
                                                 int wave, int lane) {
  cand_write_out(ws, qslot, cl, c, lane, true);
  const uint32_t n_hi = wave_sum_u32(c.v_hi), nz = wave_sum_u32(c.v_nz);
  if (lane == 0) cl.qi[wave] = make_uint4(n_hi, c.n_out, 0u, nz);
  return nz;
}

__device__ __forceinline__ void qinfo_flush(const Ws& ws, int64_t qslot_tile, const CandList& cl) {
  if (threadIdx.x < 4) ws.qinfo[qslot_tile + threadIdx.x] = cl.qi[threadIdx.x];
}

// What every group of a quarter needs from the selection of its (worker, layer): t_all = T when
// every entry equal to T is selected, else T + 1; ties: the quarter holds entries equal to T of
// which only some are selected (then t_all = T + 1).  Both are wave-uniform.
struct SelCommon { uint32_t t_all; bool ties; };
struct SelTies { uint32_t T, ktie; };

__device__ __forceinline__ SelCommon sel_common(uint32_t T, uint32_t alleq, uint32_t eq_here) {
  SelCommon c;
  c.t_all = alleq ? T : T + 1u;
  c.ties = eq_here != 0u && alleq == 0u;
  return c;
}

// Which of the four elements a lane holds of one group are selected, as lane masks per component:
// the keys >= t_all and, where ties matter, the entries equal to T within the tie quota ktie,
// counted in index order over the layer: eq_run is the number of entries equal to T before this
// group (advanced here).  mv: lane masks of the valid elements per component; tie(): T and ktie,
// fetched only when needed.
template <class TieF>
__device__ __forceinline__ void group_select(const SelCommon& sc, TieF tie, uint32_t& eq_run,
                                             const uint32_t (&key)[4], const uint64_t (&mv)[4], int lane,
                                             uint64_t (&msel)[4]) {
#pragma unroll
  for (int c = 0; c < 4; ++c) msel[c] = ballot64(key[c] >= sc.t_all) & mv[c];
  if (sc.ties) {                                            // wave-uniform
    const SelTies t = tie();
    uint64_t meq[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) meq[c] = ballot64(key[c] == t.T) & mv[c];
    if ((meq[0] | meq[1] | meq[2] | meq[3]) != 0) {
      // the tie quota is used up in index order
      uint32_t rank = eq_run;
      uint32_t total = 0;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        rank += lanes_below(meq[c], lane);
        total += (uint32_t)__popcll(meq[c]);
      }
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const bool iseq = lane_bit(meq[c]);
        msel[c] |= ballot64(iseq && rank < t.ktie);
        rank += iseq ? 1u : 0u;
      }
      eq_run += total;
    }
  }
#pragma unroll
  for (int c = 0; c < 4; ++c) msel[c] = scalar_mask(msel[c]);
}

// The selection of the previous step as the next pass over Delta needs it to zero the kept
// entries (the residual is not written by the compaction of the batched path: see tpending).
struct PrevSel { uint32_t T, ktie, eq_run; SelCommon sc; };

__device__ __forceinline__ PrevSel load_prev_sel(const Ws& ws, int64_t wl, int64_t qslot) {
  const SelState* sp = ws.sel + wl;
  PrevSel p;
  // wave-uniform values: into scalar registers, whatever kind of load fetched them
  p.T = rfl(ld_here(&sp->T)); p.ktie = rfl(ld_here(&sp->ktie));
  p.eq_run = rfl(ld_here(ws.eqpre + qslot));
  p.sc = sel_common(p.T, rfl(ld_here(&sp->alleq)), rfl(ld_here(ws.eqpre + qslot + 1)) - p.eq_run);   // the layer's last slot: the total
  return p;
}

// d with the entries the previous step kept set to zero (q: the group, qa: inside the wave's span).
template <bool AL>
__device__ __forceinline__ float4 drop_kept(const TileGeom& tg, int q, bool qa, uint64_t m_span, PrevSel& ps,
                                            float4 d, int lane) {
  uint32_t key[4];
  uint64_t mv[4], msel[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    mv[c] = valid_mask<AL>(tg, q, c, qa, m_span);
    key[c] = key_of(comp(d, c));
  }
  group_select(ps.sc, [&]() { SelTies t; t.T = ps.T; t.ktie = ps.ktie; return t; }, ps.eq_run, key, mv, lane, msel);
  if (lane_bit(msel[0])) d.x = 0.f;
  if (lane_bit(msel[1])) d.y = 0.f;
  if (lane_bit(msel[2])) d.z = 0.f;
  if (lane_bit(msel[3])) d.w = 0.f;
  return d;
}

// ---- A ----------------------------------------------------------------------------------------

// SELECT = false (layers of a single tile, which the pick kernel decides from Delta itself):
// only the error-feedback add and the accumulation.  ZB: the guess is kGuessZero.
template <bool AL, bool SELECT, bool ZB>
__device__ __forceinline__ void ef_hist_tile(const Ws& ws, const GradPtrs& gp, int w, int tile_id,
                                             const FlatTile& ft, const LayerDev& L, const TileGeom& tg,
                                             uint32_t* hist, const CandList& cl, uint32_t* sub2, double* red4, uint32_t guess,
                                             bool window_fresh, uint32_t pending) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const WaveSpan span = wave_span(tg, wave);
  const float* __restrict__ g = gp.p[w];
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  float* __restrict__ A = (w == 0) ? ws.A : nullptr;
  // the accumulation window has just restarted: A counts as zero and is not read
  const bool a_fresh = A && window_fresh;                  // uniform over the workgroup
  double a_sq = 0.0;                                       // worker 0: the lane's share of the tile's sum of squares of A
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  uint32_t glo = 0x7ffffff0u, gnb = 0u;                    // no bin matches without a guess
  if (SELECT && !ZB && guess != kNoGuess) { glo = guess_lo(guess); gnb = guess_nb(guess); }
  const bool band = gnb != 0u && gnb < (uint32_t)kGuessBins;   // uniform over the workgroup
  // two groups per lane are requested before anything else
  constexpr int U = 2;   // (one group is as fast where the memory fits the caches, three or four are no faster anywhere)
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  float4 gc[U], ec[U], ac[U];
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const int q = span.qbeg + u * kWave + lane;
    gc[u] = ld_span<AL, kStreamG>(g, tg, span, q);
    ec[u] = ld_span<AL>(e, tg, span, q);
    ac[u] = (A && !a_fresh) ? ld_span<AL, kStreamA>(A, tg, span, q) : zero4;
  }
  // the batched path leaves Delta of the previous step in e: its kept entries are dropped here.
  // The previous selection is requested whether or not it is needed, so that its loads do not
  // wait for the load of the mask.
  PrevSel ps = load_prev_sel(ws, wl, quarter_slot(ws, L, w, ft.start >> kTileShift, wave));
  const bool pend = ((pending >> w) & 1u) != 0u;           // uniform over the workgroup
  if (SELECT) {
    for (int b = tid; b < kHistBins; b += kFlatThreads) hist[b] = 0;
    for (int b = tid; b < kSub2; b += kFlatThreads) sub2[b] = 0;
    __syncthreads();
  }
  StageCounts cnt = {0u, 0u, 0u, 0u};
  const int64_t qslot_mine = quarter_slot(ws, L, w, ft.start >> kTileShift, wave);
  for (int q0 = span.qbeg; q0 < span.qend; q0 += U * kWave) {
    float4 gn[U], en[U], an[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int q = q0 + (U + u) * kWave + lane;
      gn[u] = ld_span<AL, kStreamG>(g, tg, span, q);
      en[u] = ld_span<AL>(e, tg, span, q);
      an[u] = (A && !a_fresh) ? ld_span<AL, kStreamA>(A, tg, span, q) : zero4;
    }
    const bool full = q0 + U * kWave <= span.qend;          // wave-uniform
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int q = q0 + u * kWave + lane;
      const bool qa = q < span.qend;
      if (pend) ec[u] = drop_kept<AL>(tg, q, qa, ballot64(qa), ps, ec[u], lane);
      const float4 d = make_float4(gc[u].x + ec[u].x, gc[u].y + ec[u].y, gc[u].z + ec[u].z, gc[u].w + ec[u].w);
      if (qa) {
        stq<AL>(e, tg.a0, tg.lo, tg.hi, q, d);
        if (A) {
          const float4 a = make_float4(ac[u].x + gc[u].x, ac[u].y + gc[u].y, ac[u].z + gc[u].z, ac[u].w + gc[u].w);
          stq<AL, kStreamA>(A, tg.a0, tg.lo, tg.hi, q, a);
          a_sq += sq4(a);                                    // elements outside the tile were loaded as zeros
        }
      }
      if (SELECT) {
        const uint32_t i_rel = 4u * (uint32_t)(q - span.qbeg);
        if (AL && full) {
          // every lane of both groups is inside the span: no masks
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const uint32_t key = key_of(comp(d, c));
            hist_add(hist, (key >> 20) != 0u, key >> 20);
          }
          if (ZB) {
            stage_candidates<false, false, true>(cl, sub2, cnt, 0ull, 0ull, 0ull, 0ull, d, 0u, 1u, i_rel, lane);
          } else {
            if (band) stage_candidates<false, true>(cl, sub2, cnt, 0ull, 0ull, 0ull, 0ull, d, glo, gnb, i_rel, lane);
            else stage_candidates<false, false>(cl, sub2, cnt, 0ull, 0ull, 0ull, 0ull, d, glo, gnb, i_rel, lane);
          }
        } else {
          const uint64_t m_span = ballot64(qa);
          uint64_t mv[4];
#pragma unroll
          for (int c = 0; c < 4; ++c) {
            const bool valid = elem_valid<AL>(tg, q, c, qa);
            mv[c] = valid_mask<AL>(tg, q, c, qa, m_span);
            const uint32_t key = key_of(comp(d, c));
            hist_add(hist, valid && (key >> 20) != 0u, key >> 20);
          }
          if (ZB) {
            stage_candidates<true, false, true>(cl, sub2, cnt, mv[0], mv[1], mv[2], mv[3], d, 0u, 1u, i_rel, lane);
          } else {
            if (band) stage_candidates<true, true>(cl, sub2, cnt, mv[0], mv[1], mv[2], mv[3], d, glo, gnb, i_rel, lane);
            else stage_candidates<true, false>(cl, sub2, cnt, mv[0], mv[1], mv[2], mv[3], d, glo, gnb, i_rel, lane);
          }
        }
        cand_make_room(ws, qslot_mine, cl, cnt, lane);
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) { gc[u] = gn[u]; ec[u] = en[u]; ac[u] = an[u]; }
  }
  if (A) {                                                 // uniform over the workgroup
    const double t = block_sum4_d(a_sq, red4);
    if (tid == 0) ws.norm_part[tile_id] = t;
    __syncthreads();
  }
  if (SELECT) {
    stage_finish(ws, qslot_mine, cl, cnt, wave, lane);
    __syncthreads();
    qinfo_flush(ws, qslot_mine - wave, cl);
    uint32_t* gh = ws.hist1 + wl * kHistBins;                // bin 0 stays empty: the pick kernel derives it
    for (int b = tid; b < kHistBins; b += kFlatThreads) {
      const uint32_t h = hist[b];
      if (h) atomicAdd(&gh[b], h);
    }
    // the tile's level-2 counts are added to the slot its group of kT2Group tiles shares (integer
    // atomics; the pick kernel reads and clears the slots): one compute unit works on a whole
    // layer there, and a slot per tile is 2 MB to read for a layer of 22 M entries
    const int slot = L.t2slot0 + (ft.start >> kTileShift) / kT2Group;
    for (int b = tid; b < kSub2; b += kFlatThreads)
      if (sub2[b] != 0u) atomicAdd(&ws.t2[((int64_t)w * ws.n_t2slots + slot) * kSub2 + b], sub2[b]);
  }
}

__global__ __launch_bounds__(256) void topk_ef_hist_kernel(const Ws ws, const GradPtrs gp, int w0) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t cand_val[4][kCandLdsSlots];
  __shared__ uint16_t cand_idx[4][kCandLdsSlots];
  __shared__ uint32_t sub2[kSub2];
  __shared__ double red4[4];
  __shared__ uint4 qi[4];
  const int w = w0 + blockIdx.y;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  // Everything else the tile depends on is requested together, as soon as its layer is known: the
  // flags, the layer's level and the guesses of both levels (one of them is the one to use).
  const uint32_t* gp2 = ws.guess + ((int64_t)w * ws.L + ft.layer) * 2;
  const uint32_t guess0 = ld_here(gp2), guess1 = ld_here(gp2 + 1);
  const uint32_t lvl = ld_here(reinterpret_cast<const uint32_t*>(ws.level + ft.layer));
  const uint32_t fresh_w = ld_here(ws.a_fresh), pend_w = ld_here(ws.tpending);
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  const int lw = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const CandList cl = {cand_val[lw], cand_idx[lw], qi};
  // the layer's "compact from Delta" flag of the last step is cleared before this step's
  // decision kernels (which set it) run
  if (w == 0 && ft.start == 0 && threadIdx.x == 0) ws.lflag[ft.layer] = 0u;
  const bool fresh = rfl(fresh_w) != 0u;
  const uint32_t pending = rfl(pend_w);
  if (L.ntiles == 1) {
    if (tg.aligned) ef_hist_tile<true, false, false>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, kNoGuess, fresh, pending);
    else ef_hist_tile<false, false, false>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, kNoGuess, fresh, pending);
  } else {
    const uint32_t guess = rfl(rfl(lvl) != 0u ? guess1 : guess0);
    if (guess == kGuessZero) {                               // uniform over the workgroup
      if (tg.aligned) ef_hist_tile<true, true, true>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, guess, fresh, pending);
      else ef_hist_tile<false, true, true>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, guess, fresh, pending);
    } else {
      if (tg.aligned) ef_hist_tile<true, true, false>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, guess, fresh, pending);
      else ef_hist_tile<false, true, false>(ws, gp, w, blockIdx.x, ft, L, tg, hist, cl, sub2, red4, guess, fresh, pending);
    }
  }
}

// ---- B: re-stage the keys of b1 for a layer whose guess missed -----------------------------------
// Run by the counting kernel's workgroup of the tile (the per-layer kernel after it then works from
// these lists).

template <bool AL>
__device__ __forceinline__ void restage_tile(const Ws& ws, int w, const FlatTile& ft,
                                             const LayerDev& L, const TileGeom& tg, uint32_t b1, const CandList& cl,
                                             uint32_t* sub2) {
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const WaveSpan span = wave_span(tg, wave);
  const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  if (tid < kL2Bins) sub2[tid] = 0;
  __syncthreads();
  StageCounts cnt = {0u, 0u, 0u, 0u};
  const int64_t qslot = quarter_slot(ws, L, w, ft.start >> kTileShift, wave);
  float4 cur = ld_span<AL>(e, tg, span, span.qbeg + lane);
  for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
    const int q = q0 + lane;
    const float4 nxt = ld_span<AL>(e, tg, span, q + kWave);
    const bool qa = q < span.qend;
    const uint64_t m_span = ballot64(qa);
#pragma unroll
    for (int c = 0; c < 4; ++c)
      stage_one_bin(cl, sub2, cnt, valid_mask<AL>(tg, q, c, qa, m_span), elem_valid<AL>(tg, q, c, qa),
                    key_of(comp(cur, c)), b1, lane);
    cand_make_room(ws, qslot, cl, cnt, lane);
    cur = nxt;
  }
  const uint32_t nz = stage_finish(ws, qslot, cl, cnt, wave, lane);
  const int64_t wl = (int64_t)w * ws.L + ft.layer;
  if (lane == 0 && nz) atomicAdd(&ws.sel[wl].zeros, nz);
  __syncthreads();
  qinfo_flush(ws, qslot - wave, cl);
  // the tile's level-2 counts of b1 go straight into the layer's (cleared by the pick kernel)
  if (tid < kL2Bins && sub2[tid]) atomicAdd(&ws.hist2m[wl * kL2Bins + tid], sub2[tid]);
}

// ---- the per-layer decisions ---------------------------------------------------------------------

// The first kEagerChunks 64-entry chunks of a quarter's list are requested together with its
// counts (the slot always exists; what lies past the count is ignored later), the rest once the
// count is there and only as far as it reaches: a quarter lists 60 to 500 candidates on Gaussian
// or Laplacian gradients at K = 1 % to 10 %, and chunks requested for nothing are read from memory
// all the same (eight early chunks were 0.8 GB per step on the LSTM set at K = 1 %).
constexpr int kEagerChunks = 2;
struct QuarterHead {
  uint4 info;                      // see stage_finish
  uint32_t chunk[kEagerChunks];    // the calling lane's entries of the first chunks
};

__device__ __forceinline__ QuarterHead load_quarter_head(const Ws& ws, int64_t qslot, int lane) {
  QuarterHead h;
  const uint32_t* qi = reinterpret_cast<const uint32_t*>(ws.qinfo + qslot);
  h.info = make_uint4(ld_here(qi), ld_here(qi + 1), ld_here(qi + 2), ld_here(qi + 3));
#pragma unroll
  for (int ch = 0; ch < kEagerChunks; ++ch) h.chunk[ch] = ld_here(ws.cand_val + cand_at(ws, qslot, (uint32_t)ch, lane));
  return h;
}

// Calls f(key, valid) with all 64 lanes for every key of bin b1 (zeros excluded) of one quarter
// and returns the quarter's number of entries in bins above b1: from the quarter's list (the
// candidates of pass A, or the keys of b1 alone with the entries above counted in info.x), or --
// when the quarter has more entries than its list holds -- from Delta itself.
// tl: tile within the layer, wave: quarter within the tile.
template <class F>
__device__ __forceinline__ uint32_t for_quarter_keys(const Ws& ws, const LayerDev& L, int w, int tl, int wave,
                                                     int64_t qslot, const QuarterHead& h, uint32_t b1, int lane,
                                                     F f) {
  const uint32_t n = rfl(h.info.y);
  if (n <= (uint32_t)kCandCap) {
    uint32_t above = rfl(h.info.x);
    auto visit = [&](uint32_t raw, uint32_t t) {
      const uint32_t key = raw & 0x7fffffffu;
      const uint32_t bin = key >> 20;
      const uint64_t mvalid = ballot64(t < n);
      above += (uint32_t)__popcll(ballot64(bin > b1) & mvalid);
      f(key, t < n && bin == b1);
    };
#pragma unroll
    for (int ch = 0; ch < kEagerChunks; ++ch)
      if (n > (uint32_t)(ch * kWave)) visit(h.chunk[ch], (uint32_t)(ch * kWave + lane));   // uniform condition
    constexpr int U = 4;
    for (uint32_t t0 = kEagerChunks * kWave; t0 < n; t0 += U * kWave) {
      uint32_t raw[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        raw[u] = 0u;
        if (n > t0 + u * kWave) raw[u] = ws.cand_val[cand_at(ws, qslot, t0 / kWave + u, lane)];   // uniform condition
      }
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (n > t0 + u * kWave) visit(raw[u], t0 + u * kWave + lane);                         // uniform condition
    }
    return above;
  }
  FlatTile ft;
  ft.layer = 0;
  ft.start = tl << kTileShift;
  ft.count = (int32_t)min((int64_t)kTile, (int64_t)L.rows * L.cols - ft.start);
  ft.qslot0 = 0;
  const TileGeom tg = tile_geom(L, ft);
  const WaveSpan sp = wave_span(tg, wave);
  const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  uint32_t above = 0;
  for (int q0 = sp.qbeg; q0 < sp.qend; q0 += kWave) {
    const int qq = q0 + lane;
    const float4 d = ld_span<false>(e, tg, sp, qq);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const uint32_t key = key_of(comp(d, c));
      const bool valid = elem_valid<false>(tg, qq, c, qq < sp.qend);
      above += (uint32_t)__popcll(ballot64(valid && (key >> 20) > b1));
      f(key, valid && key != 0u && (key >> 20) == b1);
    }
  }
  return above;
}

// A layer of a single tile, decided by one workgroup from Delta: the keys go to LDS, three
// histogram levels (11 + 11 + 9 bits) give the threshold, and the counts of its four quarters
// give their payload positions.
__device__ __forceinline__ void pick_small_layer(const Ws& ws, const LayerDev& L, int w, int li, uint32_t k,
                                                 uint32_t* hist, uint32_t* skeys, uint32_t* out,
                                                 uint32_t* scratch, uint32_t* qcnt) {
  const int tid = threadIdx.x;
  FlatTile ft;
  ft.layer = li;
  ft.start = 0;
  ft.count = L.rows * L.cols;
  ft.qslot0 = 0;
  const TileGeom tg = tile_geom(L, ft);
  const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  const int count = ft.count;
  const int head = (int)(tg.lo - tg.a0);                   // elements of the first group before the tile
  for (int q = tid; q < tg.nquads; q += kPickThreads) {
    const float4 d = ld_quad(e, tg.a0 + 4 * (int64_t)q, tg.lo, tg.hi);
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int i = 4 * q + c - head;
      if (i >= 0 && i < count) skeys[i] = key_of(comp(d, c));
    }
  }
  for (int b = tid; b < kHistBins; b += kPickThreads) hist[b] = 0u;
  if (tid < 8) qcnt[tid] = 0u;
  __syncthreads();
  for (int i = tid; i < count; i += kPickThreads) atomicAdd(&hist[skeys[i] >> 20], 1u);
  __syncthreads();
  pick_bin(hist, k, out, scratch);
  const uint32_t b1 = out[0], need2 = k - out[1];
  __syncthreads();
  for (int b = tid; b < kHistBins; b += kPickThreads) hist[b] = 0u;
  __syncthreads();
  for (int i = tid; i < count; i += kPickThreads) {
    const uint32_t key = skeys[i];
    if ((key >> 20) == b1) atomicAdd(&hist[(key >> 9) & 0x7ffu], 1u);
  }
  __syncthreads();
  pick_bin(hist, need2, out, scratch);
  const uint32_t b12 = (b1 << 11) | out[0], need3 = need2 - out[1];
  __syncthreads();
  for (int b = tid; b < kHistBins; b += kPickThreads) hist[b] = 0u;
  __syncthreads();
  for (int i = tid; i < count; i += kPickThreads) {
    const uint32_t key = skeys[i];
    if ((key >> 9) == b12) atomicAdd(&hist[key & 0x1ffu], 1u);
  }
  __syncthreads();
  pick_bin(hist, need3, out, scratch);
  const uint32_t T = (b12 << 9) | out[0];
  const uint32_t ktie = need3 - out[1];
  const uint32_t alleq = (ktie == out[2]) ? 1u : 0u;
  // counts of the four wave quarters the compaction kernel will use
  const int qw = (tg.nquads + 3) >> 2;
  for (int i = tid; i < count; i += kPickThreads) {
    const uint32_t key = skeys[i];
    if (key >= T) atomicAdd(&qcnt[(key > T ? 0 : 4) + ((i + head) >> 2) / qw], 1u);
  }
  __syncthreads();
  if (tid == 0) {
    const int64_t qbase = (int64_t)w * ws.q_stride + L.qoff;
    uint32_t g = 0, q = 0;
    for (int v = 0; v < 4; ++v) {
      ws.gtpre[qbase + v] = g;
      ws.eqpre[qbase + v] = q;
      g += qcnt[v];
      q += qcnt[4 + v];
    }
    ws.gtpre[qbase + 4] = g;
    ws.eqpre[qbase + 4] = q;
    SelState* sp = ws.sel + (int64_t)w * ws.L + li;
    sp->mode = 0u; sp->k = k; sp->T = T; sp->ktie = ktie; sp->alleq = alleq;
  }
}

__global__ __launch_bounds__(kPickThreads) void topk_pick12_kernel(const Ws ws, int w0) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t out[3], scratch[4];
  const int li = blockIdx.x;
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int64_t wl = (int64_t)w * ws.L + li;
  // Requested together, before anything is known (every address follows from the workgroup's
  // index): the layer's entry, its level, the guesses of both levels and the layer's level-1
  // histogram (cleared for the next step).  The tiles' level-2 counts of ALL guessed bins follow
  // as soon as the entry says where they are.
  const LayerDev* Lp = ws.layers + li;
  const uint32_t l_ntiles = ld_here(reinterpret_cast<const uint32_t*>(&Lp->ntiles));
  const uint32_t l_t2slot0 = ld_here(reinterpret_cast<const uint32_t*>(&Lp->t2slot0));
  const uint32_t l_k0 = ld_here(reinterpret_cast<const uint32_t*>(&Lp->k[0]));
  const uint32_t l_k1 = ld_here(reinterpret_cast<const uint32_t*>(&Lp->k[1]));
  const uint32_t l_rows = ld_here(reinterpret_cast<const uint32_t*>(&Lp->rows));
  const uint32_t l_cols = ld_here(reinterpret_cast<const uint32_t*>(&Lp->cols));
  const uint32_t lvl_v = ld_here(reinterpret_cast<const uint32_t*>(ws.level + li));
  const uint32_t guess0 = ld_here(ws.guess + wl * 2), guess1 = ld_here(ws.guess + wl * 2 + 1);
  uint32_t* gh = ws.hist1 + wl * kHistBins;
  uint32_t h0 = ld_here(gh + tid), h1 = ld_here(gh + tid + kPickThreads);
  const int L_ntiles = (int)rfl(l_ntiles), L_t2slot0 = (int)rfl(l_t2slot0);
  const uint32_t n_layer = rfl(l_rows) * rfl(l_cols);
  const int lv = (int)rfl(lvl_v);
  const uint32_t k = rfl(lv ? l_k1 : l_k0), k_other = rfl(lv ? l_k0 : l_k1);
  // worker 0's first pass has added its gradient to A: the window is no longer fresh
  if (w == 0 && li == 0 && tid == 0) *ws.a_fresh = 0u;
  if (L_ntiles == 1) return;                               // decided by the last pick kernel, from Delta
  SelState* sp = ws.sel + wl;
  __shared__ uint32_t sub[kSub2];
  __shared__ uint32_t nb0;
  // a thread sums four adjacent counts (one 16-byte load) of every kStripes-th slot
  constexpr int kCols4 = kSub2 / 4;
  constexpr int kStripes = kPickThreads / kCols4;           // slots summed side by side
  static_assert(kSub2 % 4 == 0 && kStripes >= 1, "four counts per load");
  const int col4 = tid % kCols4, stripe = tid / kCols4;
  uint4* t2 = reinterpret_cast<uint4*>(ws.t2 + ((int64_t)w * ws.n_t2slots + L_t2slot0) * kSub2) + col4;
  const int nslots = (L_ntiles + kT2Group - 1) / kT2Group;
  uint4 s2 = make_uint4(0u, 0u, 0u, 0u);
  constexpr int kT2Loads = 8;                               // independent loads in flight
  for (int sl0 = (stripe < kStripes ? stripe : nslots); sl0 < nslots; sl0 += kT2Loads * kStripes) {
    uint4 v[kT2Loads];
#pragma unroll
    for (int u = 0; u < kT2Loads; ++u) v[u] = t2[(int64_t)min(sl0 + u * kStripes, nslots - 1) * kCols4];
#pragma unroll
    for (int u = 0; u < kT2Loads; ++u) {
      const int sl = sl0 + u * kStripes;
      if (sl < nslots) {
        s2.x += v[u].x; s2.y += v[u].y; s2.z += v[u].z; s2.w += v[u].w;
        t2[(int64_t)sl * kCols4] = make_uint4(0u, 0u, 0u, 0u);   // cleared for the next step
      }
    }
  }
  const uint32_t guess = rfl(lv ? guess1 : guess0);
  gh[tid] = 0u;
  gh[tid + kPickThreads] = 0u;
  hist[tid] = h0;
  hist[tid + kPickThreads] = h1;
  if (tid < kSub2) sub[tid] = 0u;
  if (tid == 0) nb0 = 0u;
  __syncthreads();
  if (s2.x) atomicAdd(&sub[4 * col4 + 0], s2.x);
  if (s2.y) atomicAdd(&sub[4 * col4 + 1], s2.y);
  if (s2.z) atomicAdd(&sub[4 * col4 + 2], s2.z);
  if (s2.w) atomicAdd(&sub[4 * col4 + 3], s2.w);
  {
    // bin 0 (exact zeros and the smallest denormals) was not histogrammed: the rest of the layer
    const uint32_t part = wave_sum_u32(h0 + h1 - (tid == 0 ? h0 : 0u));
    if (lane == 0 && part) atomicAdd(&nb0, part);
  }
  __syncthreads();
  if (tid == 0) hist[0] = n_layer - nb0;
  __syncthreads();
  pick_bin(hist, k, out, scratch);
  const uint32_t b1 = out[0], need2 = k - out[1];
  // The other level's guess, from the same histogram: the bin its k-th largest key would lie in
  // in this step's Delta.  It serves the first step after a level switch, when the level's own
  // history is stale (or missing); after that the threshold is followed as usual.
  if (k_other != k) {                                      // uniform over the workgroup
    __syncthreads();                                       // everybody has read out[]
    pick_bin(hist, k_other, out, scratch);
    if (tid == 0) {
      const uint32_t bo = out[0];
      // (the memory will adapt to the new level for some steps: a wide guess)
      ws.guess[wl * 2 + (1 - lv)] = (bo == 0u) ? kGuessZero
          : make_guess((int)bo - kGuessMovingBelow, guess_bins_for(k_other, n_layer));
    }
    __syncthreads();
  }
  const bool guessed = guess != kNoGuess && guess != kGuessZero;
  const uint32_t glo = guessed ? guess_lo(guess) : 0u;     // the bins pass A counted: glo .. glo + nb - 1
  const bool hit = guessed && b1 >= glo && b1 - glo < guess_nb(guess);
  // bin 0 guessed and found: pass A listed every non-zero entry and counted the zeros (mode 2)
  const bool zhit = guess == kGuessZero && b1 == 0u;
  const uint32_t side = hit ? b1 - glo : 0u;
  if (tid == 0) {
    sp->b1 = b1; sp->need2 = need2; sp->k = k; sp->side = side; sp->zeros = 0u; sp->bin0 = hist[0];
    sp->mode = hit ? 0u : (zhit ? 2u : 1u);
    // the candidate lists of this layer cannot serve the compaction (a miss, or a band, which does
    // not list what lies above it): it reads Delta instead.  (Bin 0 guessed and found: the lists
    // hold every non-zero entry; the quarters that keep exact zeros go back to Delta one by one.)
    if ((!hit && !zhit) || (guessed && guess_nb(guess) < (uint32_t)kGuessBins))
      atomicOr(&ws.lflag[li], 1u);                         // cleared by the next step's first pass
    if (!hit && !zhit) atomicAdd(&ws.stats[0], 1ull);      // layers re-staged (diagnostic counter)
  }
  if (zhit) {
    // level-2 counts of the non-zero keys of bin 0 (summed over the tiles above); the rest of
    // bin 0 are exact zeros, which belong to level-2 bin 0
    __shared__ uint32_t zeros_s;
    if (tid == 0) {
      uint32_t nnz0 = 0;
      for (int b = 0; b < kL2Bins; ++b) nnz0 += sub[b];
      zeros_s = hist[0] - min(nnz0, hist[0]);
      sp->zeros = zeros_s;
    }
    __syncthreads();
    for (int b = tid; b < kHistBins; b += kPickThreads)
      hist[b] = (b < kL2Bins) ? sub[b] + (b == 0 ? zeros_s : 0u) : 0u;
    __syncthreads();
    pick_bin(hist, need2, out, scratch);
    if (tid == 0) {
      sp->b2 = out[0];
      sp->need3 = need2 - out[1];
    }
    return;
  }
  if (!hit) {
    // its keys get staged tile by tile, with their level-2 counts added up here
    if (tid < kL2Bins) ws.hist2m[wl * kL2Bins + tid] = 0u;
    return;
  }
  __syncthreads();
  // level 2: the summed counts of bin b1 (a threshold in bin 0 never gets here)
  for (int b = tid; b < kHistBins; b += kPickThreads) hist[b] = (b < kL2Bins) ? sub[side * kL2Bins + b] : 0u;
  __syncthreads();
  pick_bin(hist, need2, out, scratch);
  if (tid == 0) {
    sp->b2 = out[0];
    sp->need3 = need2 - out[1];                            // still needed from bin (b1, b2)
  }
}

// A workgroup takes kCountTiles consecutive tiles, a wave one quarter of each; everything the tiles
// need is requested before the first of them is looked at.  (Two tiles per workgroup are no faster
// than one, on 100 000 tiles as on 5 000.)
constexpr int kCountTiles = 1;

struct CountLds {
  // The staging lists of a missed layer's tile (values, then offsets), used by that rare path only.
  static constexpr int kListWords = 4 * kCandLdsSlots;
  static constexpr int kRareWords = kListWords + kListWords / 2;
  uint32_t* rare;
  uint32_t* sub2;
  uint4* qi;
};

struct CountTile { FlatTile ft; int64_t qslot; QuarterHead qh; uint32_t b1, b2, mode; int ntiles; };

__device__ __forceinline__ void count3_tile(const Ws& ws, int w, const CountTile& t, const CountLds& lds,
                                            int wave, int lane) {
  const FlatTile& ft = t.ft;
  if (t.ntiles == 1) return;                               // decided by the last pick kernel
  const LayerDev& L = ws.layers[ft.layer];
  const int tl = ft.start >> kTileShift;
  const uint32_t b1 = t.b1, b2 = t.b2;
  if (t.mode == 1u) {                                      // uniform over the workgroup
    // The guess missed: nothing useful was staged.  This tile's keys of b1 are staged now (one
    // more read of Delta) with their level-2 counts; the layer's pick kernel takes it from there.
    const TileGeom tg = tile_geom(L, ft);
    const CandList cl = {lds.rare + wave * kCandLdsSlots,
                         reinterpret_cast<uint16_t*>(lds.rare + CountLds::kListWords) + wave * kCandLdsSlots, lds.qi};
    if (tg.aligned) restage_tile<true>(ws, w, ft, L, tg, b1, cl, lds.sub2);
    else restage_tile<false>(ws, w, ft, L, tg, b1, cl, lds.sub2);
    __syncthreads();                                       // the block of LDS may serve the next tile
    return;
  }
  uint32_t* list = ws.qlist + t.qslot * kQListCap;
  uint32_t n_gt = 0, n_in = 0;                             // wave-uniform
  const uint32_t above = for_quarter_keys(ws, L, w, tl, wave, t.qslot, t.qh, b1, lane, [&](uint32_t key, bool valid) {
    const uint32_t bb = bin2_of(key);
    const uint64_t mv = ballot64(valid);
    n_gt += (uint32_t)__popcll(ballot64(bb > b2) & mv);
    const uint64_t m2 = ballot64(bb == b2) & mv;
    if (m2 != 0) {
      const uint32_t pos = n_in + lanes_below(m2, lane);
      if (valid && bb == b2 && pos < (uint32_t)kQListCap) list[pos] = key;
      n_in += (uint32_t)__popcll(m2);
    }
  });
  if (lane == 0) { ws.gtq[t.qslot] = above + n_gt; ws.eqq[t.qslot] = n_in; }
}

__global__ __launch_bounds__(256) void topk_count3_kernel(const Ws ws, int w0) {
  __shared__ __attribute__((aligned(16))) uint32_t rare[CountLds::kRareWords];
  __shared__ uint32_t sub2[kL2Bins];
  __shared__ uint4 qi[4];
  const CountLds lds = {rare, sub2, qi};
  const int w = w0 + blockIdx.y;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int tile0 = (int)blockIdx.x * kCountTiles;
  CountTile t[kCountTiles];
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u) t[u].ft = ws.ftiles[min(tile0 + u, ws.n_ftiles - 1)];
  // the lists are requested before the layers' entries and their states have arrived
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u) {
    t[u].qslot = (int64_t)w * ws.q_stride + t[u].ft.qslot0 + wave;
    t[u].qh = load_quarter_head(ws, t[u].qslot, lane);
  }
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u) {
    const SelState* sp = ws.sel + (int64_t)w * ws.L + t[u].ft.layer;
    t[u].b1 = rfl(ld_here(&sp->b1)); t[u].b2 = rfl(ld_here(&sp->b2)); t[u].mode = rfl(ld_here(&sp->mode));
    t[u].ntiles = (int)rfl(ld_here(reinterpret_cast<const uint32_t*>(&ws.layers[t[u].ft.layer].ntiles)));
  }
#pragma unroll
  for (int u = 0; u < kCountTiles; ++u)
    if (tile0 + u < ws.n_ftiles) count3_tile(ws, w, t[u], lds, wave, lane);   // uniform over the workgroup
}

// Two sizes of the last pick kernel: kLdsList keys of bin (b1, b2) of a layer gathered in LDS
// (packed), kLdsQuarters quarters of a layer whose counts are kept in LDS.  The small one (60 KB
// of LDS) takes the layers up to 6.3 M entries; the layers beyond that go to the big one (152 KB,
// one workgroup per compute unit; launched only for models that have such a layer), which
// serves up to 25 M entries from LDS.  Larger layers, or more keys around the threshold, work
// from device memory (slower, same results).
constexpr int kLdsList = 10240, kLdsQuarters = 3072;
constexpr int kLdsListBig = 24576, kLdsQuartersBig = 12288;
static_assert(2 * kLdsQuarters <= kLdsList && 2 * kLdsQuartersBig <= kLdsListBig,
              "the prefixes of a layer are staged in the key list");

template <int kLdsList, int kLdsQuarters, bool BIG>
__device__ __forceinline__ void pick3_body(const Ws& ws, int w0, uint32_t step_id) {
  __shared__ uint32_t hist[kHistBins];
  __shared__ uint32_t llist[kLdsList];
  // per quarter (2048 entries): entries above T | listed keys equal to T << 12 | exact zeros << 17
  __shared__ uint32_t lcnt[kLdsQuarters];
  __shared__ uint32_t out[3], scratch[4];
  __shared__ uint32_t wsum[2][kPickWaves];
  __shared__ uint32_t flag, lcount;
  const int li = blockIdx.x;
  const int w = w0 + blockIdx.y;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const LayerDev& L = ws.layers[li];
  if (L.ntiles == 1) {
    // A layer of a single tile needs none of the passes in between: its workgroup, idle otherwise,
    // decides it here from Delta (in the first pick kernel, where this used to happen, these layers
    // were the ones that kernel waited for: 3 us of every step).
    static_assert(kLdsList >= kTile && 2 * kPickWaves >= 8, "the key list holds a tile's keys");
    if (!BIG) pick_small_layer(ws, L, w, li, (uint32_t)L.k[ws.level[li]], hist, llist, out, scratch, &wsum[0][0]);
    return;
  }
  const int nq = 4 * L.ntiles;
  if (BIG != (nq > acc::kLdsQuarters)) return;             // the other instantiation's layer
  const int64_t wl = (int64_t)w * ws.L + li;
  SelState* sp = ws.sel + wl;
  const int lv = ws.level[li];
  const int64_t qbase = (int64_t)w * ws.q_stride + L.qoff;
  // gtq: per quarter, the entries above bin (b1, b2); eqq: the number of keys inside (b1, b2), of
  // which the first kQListCap are listed.  Thread t owns a contiguous chunk of quarters.
  uint32_t* gtq = ws.gtq + qbase;
  uint32_t* eqq = ws.eqq + qbase;
  const uint32_t* nlist = eqq;                             // until the counts are final
  const uint4* qlist4 = reinterpret_cast<const uint4*>(ws.qlist + qbase * kQListCap);
  const int chunk = (nq + kPickThreads - 1) / kPickThreads;
  const int q_lo = min(tid * chunk, nq), q_hi = min(q_lo + chunk, nq);
  if (tid == 0) { flag = 0u; lcount = 0u; }
  // requested now, used by thread 0 at the very end (the guess for the next step)
  const uint2 prev_hist = ws.b1hist[wl * 2 + lv];
  const uint32_t b1 = sp->b1, zeros = sp->zeros, mode = sp->mode;
  uint32_t b2 = sp->b2;
  uint32_t need = sp->need3;
  __syncthreads();
  if (mode == 1u) {                                        // uniform over the workgroup
    // The guess missed: the counting kernel's workgroups have staged the keys of b1 tile by tile
    // and summed their level-2 counts.  b2 comes from those; what the quarter lists would have
    // given is taken by sweeps over the staged keys (one workgroup for the whole layer: slower
    // than the listed path, and rare).
    for (int b = tid; b < kHistBins; b += kPickThreads) {
      uint32_t h = (b < kL2Bins) ? ws.hist2m[wl * kL2Bins + b] : 0u;
      if (b == 0 && b1 == 0u) h += zeros;                    // exact zeros: level-2 bin 0 of bin 0
      hist[b] = h;
    }
    __syncthreads();
    const uint32_t need2 = sp->need2;
    pick_bin(hist, need2, out, scratch);
    b2 = out[0];
    need = need2 - out[1];
    if (tid == 0) { flag = 1u; sp->b2 = b2; sp->need3 = need; }
    __syncthreads();                                       // everybody has read out[]
  }
  const bool zero_bin = (b1 == 0u && b2 == 0u);            // bin (b1, b2) holds the exact zeros
  // Gather the listed keys of the whole layer in LDS, packed as (quarter << 14 | low 14 key
  // bits): the upper 17 key bits are those of (b1, b2).  A quarter's count and its list slot are
  // requested together.
  const bool packable = nq <= (1 << 18);
  // A layer of at most kLdsQuarters quarters has its per-quarter counts summed up in LDS (a
  // quarter holds 2048 entries: 16 bits per count), which saves the round trips of global atomics
  // and of reading them back.
  const bool lds_q = nq <= kLdsQuarters;
  // the exact zeros of a quarter count as equal to T when T turns out to be 0, which can only
  // happen in the zero bin
  const uint4* qinfo = ws.qinfo + qbase;
  // Every lane of a wave calls this together (valid: the lane has a quarter): the wave's keys get
  // one stretch of the list, reserved with one atomic per wave -- an atomic per quarter on the one
  // counter costs 20 cycles each, one after the other (10 us for a layer of 2.4 M entries).
  auto take_quarter = [&](int q, bool valid, uint32_t n, uint32_t g0, uint32_t zq,
                          const uint4 (&k4)[kQListCap / 4]) {
    if (valid && lds_q) lcnt[q] = g0 | (zq << 17);
    const bool over = valid && (n > (uint32_t)kQListCap || !packable);
    if (over) flag = 1u;                                   // a list overflowed: the sweeps decide
    const uint32_t ne = (valid && !over) ? n : 0u;
    const uint32_t incl = wave_incl_scan_u32(ne, lane);
    const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, kWave - 1);
    if (total == 0u) return;                               // wave-uniform
    uint32_t base = 0u;
    if (lane == kWave - 1) base = atomicAdd(&lcount, total);
    base = (uint32_t)__builtin_amdgcn_readlane((int)base, kWave - 1);
    const uint32_t pos = base + incl - ne;
    if (ne != 0u && pos + ne <= (uint32_t)kLdsList) {
#pragma unroll
      for (int i = 0; i < kQListCap; ++i) {
        const uint4& v = k4[i / 4];
        const uint32_t key = (i % 4 == 0) ? v.x : (i % 4 == 1) ? v.y : (i % 4 == 2) ? v.z : v.w;
        if ((uint32_t)i < ne) llist[pos + i] = ((uint32_t)q << 14) | (key & 0x3fffu);
      }
    }
  };
  // Consecutive threads take consecutive quarters (whole cache lines per request: with a chunk of
  // quarters per thread the one compute unit that works on a large layer spends its time on
  // requests, 388 lines per wave and round instead of 40), four rounds requested together, from
  // clamped indices, so that every lane runs every round.  Of a quarter's list the first four keys
  // come with its count; the rest only when the count reaches them.
  constexpr int G = 4;
  for (int q0 = (mode == 1u ? nq : 0); q0 < nq; q0 += G * kPickThreads) {
    uint32_t n[G], g0[G], zq[G];
    uint4 k4[G][kQListCap / 4];
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int q = min(q0 + u * kPickThreads + tid, nq - 1);
      n[u] = eqq[q];
      g0[u] = gtq[q];
      zq[u] = zero_bin ? qinfo[q].w : 0u;
      k4[u][0] = qlist4[(int64_t)q * (kQListCap / 4)];
    }
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int qv = q0 + u * kPickThreads + tid, q = min(qv, nq - 1);
#pragma unroll
      for (int i = 1; i < kQListCap / 4; ++i)
        k4[u][i] = (n[u] > (uint32_t)(4 * i) && n[u] <= (uint32_t)kQListCap) ? qlist4[(int64_t)q * (kQListCap / 4) + i]
                                                                            : make_uint4(0u, 0u, 0u, 0u);
    }
#pragma unroll
    for (int u = 0; u < G; ++u) {
      const int qv = q0 + u * kPickThreads + tid;
      if (q0 + u * kPickThreads < nq)                       // uniform over the workgroup
        take_quarter(min(qv, nq - 1), qv < nq, n[u], g0[u], zq[u], k4[u]);
    }
  }
  __syncthreads();
  const uint32_t ln = lcount;
  const bool listed = flag == 0u;                          // every quarter's list is complete
  const bool in_lds = ln <= (uint32_t)kLdsList;            // ... and all of them fit in LDS
  auto clear_hist = [&]() {
    __syncthreads();
    for (int b = tid; b < kHistBins; b += kPickThreads) hist[b] = 0u;
    __syncthreads();
  };
  // f(low 14 key bits, quarter) for every listed key of the layer: from LDS, or -- a very large
  // layer -- from the quarters' lists again (each thread its own quarters)
  auto for_listed = [&](auto f) {
    if (in_lds) {
      for (uint32_t i = tid; i < ln; i += kPickThreads) f(llist[i] & 0x3fffu, (int)(llist[i] >> 14));
    } else {
      const uint32_t* ql = ws.qlist + qbase * kQListCap;
      for (int q = q_lo; q < q_hi; ++q) {
        const uint32_t n = min(ld_agent(&nlist[q]), (uint32_t)kQListCap);
        for (uint32_t i = 0; i < n; ++i) f(ql[(int64_t)q * kQListCap + i] & 0x3fffu, q);
      }
    }
  };
  uint32_t T, ktie, alleq;
  if (listed) {
    // level 3: key bits 13..6
    clear_hist();
    for_listed([&](uint32_t low, int) { atomicAdd(&hist[low >> 6], 1u); });
    if (zero_bin && tid == 0) atomicAdd(&hist[0], zeros);
    __syncthreads();
    pick_bin(hist, need, out, scratch);
    const uint32_t b3 = out[0];
    need -= out[1];
    // level 4: key bits 5..0
    clear_hist();
    for_listed([&](uint32_t low, int) { if ((low >> 6) == b3) atomicAdd(&hist[low & 0x3fu], 1u); });
    if (zero_bin && b3 == 0u && tid == 0) atomicAdd(&hist[0], zeros);
    __syncthreads();
    pick_bin(hist, need, out, scratch);
    T = (b1 << 20) | (b2 << 14) | (b3 << 6) | out[0];
    ktie = need - out[1];                                  // 1 <= ktie <= entries equal to T
    alleq = (ktie == out[2]) ? 1u : 0u;
    // per quarter: the listed keys above T and equal to T
    const uint32_t t_low = T & 0x3fffu;
    if (in_lds && lds_q) {
      for_listed([&](uint32_t low, int q) {
        if (low > t_low) atomicAdd(&lcnt[q], 1u);
        else if (low == t_low) atomicAdd(&lcnt[q], 1u << 12);
      });
    } else if (in_lds) {
      for (int q = q_lo; q < q_hi; ++q) eqq[q] = 0u;
      __syncthreads();
      for_listed([&](uint32_t low, int q) {
        if (low > t_low) atomicAdd(&gtq[q], 1u);
        else if (low == t_low) atomicAdd(&eqq[q], 1u);
      });
    } else {
      uint32_t g = 0, e = 0;
      auto close = [&](int q) { gtq[q] = ld_agent(&gtq[q]) + g; eqq[q] = e; g = 0; e = 0; };
      // the keys come quarter by quarter (the thread's own quarters, ascending)
      for (int q = q_lo; q < q_hi; ++q) {
        const uint32_t n = min(ld_agent(&nlist[q]), (uint32_t)kQListCap);
        const uint32_t* ql = ws.qlist + (qbase + q) * kQListCap;
        for (uint32_t i = 0; i < n; ++i) {
          const uint32_t low = ql[i] & 0x3fffu;
          g += (low > t_low) ? 1u : 0u;
          e += (low == t_low) ? 1u : 0u;
        }
        close(q);
      }
    }
  } else {
    // layers whose tie class sent them to the sweeps (diagnostic counter; a missed guess is counted apart)
    if (tid == 0 && mode != 1u) atomicAdd(&ws.stats[1], 1ull);
    // Slow path (some quarter holds more keys of bin (b1, b2) than its list, i.e. a large tie
    // class; or the guess missed): sweeps of the workgroup over the keys of bin b1 of the whole layer.
    auto sweep = [&](auto per_key, auto per_quarter) {
      for (int q = wave; q < nq; q += kPickWaves) {
        const QuarterHead qh = load_quarter_head(ws, qbase + q, lane);
        const uint32_t above = for_quarter_keys(ws, L, w, q >> 2, q & 3, qbase + q, qh, b1, lane, per_key);
        per_quarter(q, above);
      }
    };
    auto nothing = [](int, uint32_t) {};
    clear_hist();
    sweep([&](uint32_t key, bool valid) { if (valid && bin2_of(key) == b2) atomicAdd(&hist[bin3_of(key)], 1u); },
          nothing);
    if (zero_bin && tid == 0) atomicAdd(&hist[0], zeros);
    __syncthreads();
    pick_bin(hist, need, out, scratch);
    const uint32_t b3 = out[0];
    need -= out[1];
    clear_hist();
    const uint32_t hi3 = (b1 << 14) | (b2 << 8) | b3;      // key >> 6 of the keys of (b1, b2, b3)
    sweep([&](uint32_t key, bool valid) { if (valid && (key >> 6) == hi3) atomicAdd(&hist[bin4_of(key)], 1u); },
          nothing);
    if (zero_bin && b3 == 0u && tid == 0) atomicAdd(&hist[0], zeros);
    __syncthreads();
    pick_bin(hist, need, out, scratch);
    T = (hi3 << 6) | out[0];
    ktie = need - out[1];
    alleq = (ktie == out[2]) ? 1u : 0u;
    uint32_t n_gt = 0, n_eq = 0;
    sweep([&](uint32_t key, bool valid) {
            const uint64_t mv = ballot64(valid);
            n_gt += (uint32_t)__popcll(ballot64(key > T) & mv);
            n_eq += (uint32_t)__popcll(ballot64(key == T) & mv);
          },
          [&](int q, uint32_t above) {
            if (lane == 0) { gtq[q] = above + n_gt; eqq[q] = n_eq; }
            n_gt = 0; n_eq = 0;
          });
  }
  __syncthreads();

  // exclusive prefix over the quarters of the layer (entries above T; entries equal to T, the
  // exact zeros, counted apart, included when T is 0)
  {
    const bool from_lds = listed && in_lds && lds_q;         // uniform over the workgroup
    auto quarter_counts = [&](int q, uint32_t& g, uint32_t& e) {
      if (from_lds) {
        const uint32_t v = lcnt[q];
        g = v & 0xfffu;
        e = ((v >> 12) & 0x1fu) + (T == 0u ? v >> 17 : 0u);
      } else {
        g = ld_agent(&gtq[q]);
        e = ld_agent(&eqq[q]);
        if (T == 0u) e += qinfo[q].w;
      }
    };
    uint32_t s_gt = 0, s_eq = 0;
    for (int q = q_lo; q < q_hi; ++q) {
      uint32_t g, e;
      quarter_counts(q, g, e);
      s_gt += g;
      s_eq += e;
    }
    const uint32_t i_gt = wave_incl_scan_u32(s_gt, lane), i_eq = wave_incl_scan_u32(s_eq, lane);
    if (lane == kWave - 1) { wsum[0][wave] = i_gt; wsum[1][wave] = i_eq; }
    __syncthreads();
    uint32_t o_gt = i_gt - s_gt, o_eq = i_eq - s_eq;
    for (int v = 0; v < wave; ++v) { o_gt += wsum[0][v]; o_eq += wsum[1][v]; }
    uint32_t* gtpre = ws.gtpre + qbase;
    uint32_t* eqpre = ws.eqpre + qbase;
    if (chunk == 1) {
      if (q_lo < q_hi) { gtpre[q_lo] = o_gt; eqpre[q_lo] = o_eq; }
      o_gt += s_gt;
      o_eq += s_eq;
    } else if (from_lds) {
      // the prefixes go through LDS (the key list is no longer needed; 2 nq <= its size) and out
      // with consecutive threads on consecutive quarters: a chunk per thread would be one cache
      // line per lane and store
      __syncthreads();                                      // nobody reads the key list any more
      for (int q = q_lo; q < q_hi; ++q) {
        uint32_t g, e;
        quarter_counts(q, g, e);
        llist[q] = o_gt;
        llist[nq + q] = o_eq;
        o_gt += g;
        o_eq += e;
      }
      __syncthreads();
      for (int q = tid; q < nq; q += kPickThreads) {
        gtpre[q] = llist[q];
        eqpre[q] = llist[nq + q];
      }
    } else {
      for (int q = q_lo; q < q_hi; ++q) {
        uint32_t g, e;
        quarter_counts(q, g, e);
        gtpre[q] = o_gt;
        eqpre[q] = o_eq;
        o_gt += g;
        o_eq += e;
      }
    }
    if (tid == kPickThreads - 1) { gtpre[nq] = o_gt; eqpre[nq] = o_eq; }   // totals: o_gt + ktie == k
  }
  if (tid == 0) {
    sp->T = T; sp->ktie = ktie; sp->alleq = alleq; sp->mode = 0u;
    // Next step's guess at this level, from the bin this step ended in and the last two moves.
    // b1hist: (b1 | (last move + 64) << 16 | steps at rest << 24, step)
    const uint2 prev = prev_hist;
    const bool consecutive = prev.y + 1u == step_id;
    int v = consecutive ? (int)b1 - (int)(prev.x & 0xffffu) : 0;
    v = max(-64, min(64, v));
    // steps in a row without a move (two equal steps right after a level switch are no rest yet)
    const int rest = (consecutive && v == 0) ? min(15, (int)(prev.x >> 24) + 1) : 0;
    ws.b1hist[wl * 2 + lv] = make_uint2(b1 | ((uint32_t)(v + 64) << 16) | ((uint32_t)rest << 24), step_id);
    // A move down is followed at once (the guess must start below the threshold); a move up only
    // with a lag of two bins: the guess reaches four to six bins above its centre anyway, and a
    // jump up is often followed by smaller steps.
    int centre = (int)b1 + (v < 0 ? v : max(0, v - 2));
    const uint32_t n_layer = (uint32_t)L.rows * (uint32_t)L.cols, k_now = (uint32_t)L.k[lv];
    if (guess_bins_for(k_now, n_layer) < kGuessBins) {
      // A level that keeps a large part empties the memory in one step: on the first step after
      // a switch to it the threshold is that of gradient plus a full memory, from the second on that
      // of the gradient alone, octaves below.  So the step after a switch is guessed where the
      // threshold was the last time this level ran, and a jump of many bins is not taken for a drift.
      const int remembered = (int)(prev.x & 0xffffu);
      if (!consecutive && remembered != 0 && remembered < (int)b1) centre = remembered;
      else if (consecutive && abs(v) > 6) centre = (int)b1;
    }
    // how far below the centre the guess starts: one bin at rest, two while the move is steady (it
    // changed by at most one bin from the step before), three otherwise (the first steps at a level)
    const int pv = consecutive ? (int)((prev.x >> 16) & 0xffu) - 64 : 0;
    const bool steady = consecutive && abs(v - pv) <= 1;
    const int below = rest >= kGuessRestSteps ? kGuessCalmBelow : (steady ? kGuessMovingBelow - 1 : kGuessMovingBelow);
    // A sparse layer of which more is kept than the gradient brings in: once the memory has been
    // emptied down to less than k non-zero entries the threshold drops to zero.  This step leaves
    // nnz - k of its non-zero entries behind and the next gradient adds about as many as it did
    // the last time everything non-zero was kept.
    const uint32_t nnz = n_layer - min(sp->bin0, n_layer);
    uint32_t fresh = sp->fresh_nnz;
    if (b1 == 0u && nnz != 0u) { fresh = nnz; sp->fresh_nnz = nnz; }
    const bool runs_dry = fresh != 0u && (uint64_t)(nnz - min(k_now, nnz)) + fresh <= (uint64_t)k_now;
    ws.guess[wl * 2 + lv] = (b1 == 0u || runs_dry) ? kGuessZero
        : make_guess(centre - below, guess_bins_for(k_now, n_layer));
  }
}

__global__ __launch_bounds__(kPickThreads) void topk_pick3_kernel(const Ws ws, int w0, uint32_t step_id) {
  pick3_body<kLdsList, kLdsQuarters, false>(ws, w0, step_id);
}

// The layers of more than kLdsQuarters quarters.
__global__ __launch_bounds__(kPickThreads) void topk_pick3_big_kernel(const Ws ws, int w0, uint32_t step_id) {
  pick3_body<kLdsListBig, kLdsQuartersBig, true>(ws, w0, step_id);
}

// ---- E ----------------------------------------------------------------------------------------

// Payload format of a layer of n entries that keeps k (static per level): more than half kept =>
// the values go out dense-in-order and the indices name the n - k holes (none if k = n).
__device__ __host__ __forceinline__ bool payload_has_holes(uint32_t n, uint32_t k) { return 2ull * k > n; }

// What a wave needs to know about one worker's selection in its quarter.
struct QuarterSel {
  uint32_t T, ktie, k;
  uint32_t t_all;                    // see SelCommon
  uint32_t flags;                    // bit 0: ties matter in this quarter (see SelCommon); bit 1: the
                                     // layer keeps more than half: payload = the k values in index
                                     // order + the nholes = n - k indices of the dropped entries
                                     // (else: payload = (index, value) of the kept entries)
  uint32_t nholes;
  uint32_t gt_before, eq_before;     // selected-above-T and equal-to-T entries in the quarters before
};

__device__ __forceinline__ QuarterSel load_quarter_sel(const Ws& ws, int w, int layer, int64_t qslot_local) {
  const SelState* sp = ws.sel + (int64_t)w * ws.L + layer;
  const int64_t qs = (int64_t)w * ws.q_stride + qslot_local;
  QuarterSel s;
  s.T = sp->T; s.ktie = sp->ktie; s.k = sp->k;
  const uint32_t n_layer = (uint32_t)ws.layers[layer].rows * (uint32_t)ws.layers[layer].cols;
  s.nholes = n_layer - min(s.k, n_layer);
  s.gt_before = ws.gtpre[qs];
  s.eq_before = ws.eqpre[qs];
  const SelCommon sc = sel_common(s.T, sp->alleq, ws.eqpre[qs + 1] - s.eq_before);   // last slot: the total
  s.t_all = sc.t_all;
  s.flags = (sc.ties ? 1u : 0u) | (payload_has_holes(n_layer, s.k) ? 2u : 0u);
  return s;
}

// The part of it every group uses (wave-uniform) ...
struct GroupSel { uint32_t t_all, k, flags; };
// ... and the part only groups with ties or layers with a hole list use.
struct GroupRare { uint32_t T, ktie, nholes; };

constexpr int kGroupList = 4 * kWave;   // payload entries one group of a wave can produce
// A wave's staging list in LDS: kStgStride indices, then kStgStride values.  Slots kGroupList and up
// take the writes of the lanes' unselected elements (one slot per lane, never read), so that the
// staging needs no branches.
constexpr int kStgStride = kGroupList + kWave;
constexpr int kStgWords = 2 * kStgStride;

// Running state of the ordered compaction of one worker's quarter.
struct CompactRun { uint32_t eq_run, pos_run; };

// The compaction of the call-by-call path (one worker per grid row; the batched path has its own,
// compact_mean_tile below).  One group of four elements per lane: which are selected, their
// payload entries, the zeros in e.  The payload entries of the group are first put in order into
// the wave's list in LDS, then written out by consecutive lanes to consecutive addresses: stores
// of single words scattered over the lanes of four instructions cost a quarter of this kernel's
// time.  HOLES: the layer keeps more than half of its entries (the
// values go out dense, the indices name the dropped entries).  Everything per element is kept
// free of branches.
// The second half of compact_group: the selection is known (msel: lane masks of the selected
// elements per component, below: selected elements of the group in the lanes before this one,
// total: in all lanes); mv: lane masks of the valid elements.
template <bool AL, bool HOLES, class RareF>
__device__ __forceinline__ void compact_selected(const TileGeom& tg, int64_t layer_offset, const GroupSel& gs,
                                                 RareF rare, CompactRun& run, float* __restrict__ e,
                                                 int32_t* __restrict__ pidx, float* __restrict__ pval, int q,
                                                 const float4& cur, int lane, uint32_t* stg,
                                                 const uint64_t (&msel)[4], const uint64_t (&mv)[4],
                                                 uint32_t below, uint32_t total) {
  const int32_t i0 = (int32_t)(tg.a0 + 4 * (int64_t)q - layer_offset);
  bool sel[4];
  uint32_t place[4];                                        // of element c in the group's list, if selected
  uint32_t local = below;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    sel[c] = lane_bit(msel[c]);
    place[c] = local;
    local += sel[c] ? 1u : 0u;
  }
  uint32_t nholes = 0u;
  if (HOLES) nholes = rare().nholes;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    const uint32_t slot = sel[c] ? place[c] : (uint32_t)(kGroupList + lane);
    if (!HOLES) stg[slot] = (uint32_t)(i0 + c);
    stg[kStgStride + slot] = __float_as_uint(comp(cur, c));
    if (HOLES && lane_bit(mv[c] & ~msel[c])) {
      // dropped entry number (index - kept before it) of the layer
      const uint32_t hp = (uint32_t)(i0 + c) - (run.pos_run + place[c]);
      if (hp < nholes) pidx[hp] = i0 + c;                   // always true for consistent state
    }
  }
  __builtin_amdgcn_wave_barrier();                          // the list is complete (LDS is in order per wave)
  auto flush = [&](uint32_t t) {
    const uint32_t ix = HOLES ? 0u : stg[t];
    const uint32_t vb = stg[kStgStride + t];
    const uint32_t pos = run.pos_run + t;
    if (t < total && pos < gs.k) {                          // pos < k: always true for consistent state
      // streaming stores: nothing in this step reads the payload again.  The byte offset is a
      // 32-bit value (the payload of a worker is far below 4 GiB).
      const uint32_t boff = pos << 2;
      if (!HOLES) __builtin_nontemporal_store((int32_t)ix, (int32_t*)((char*)pidx + boff));
      __builtin_nontemporal_store(__uint_as_float(vb), (float*)((char*)pval + boff));
    }
  };
  flush((uint32_t)lane);                                    // total <= 256: four rounds at most, mostly one
  if (total > (uint32_t)kWave) {
#pragma unroll 1
    for (uint32_t t0 = kWave; t0 < total; t0 += kWave) flush(t0 + lane);
  }
  __builtin_amdgcn_wave_barrier();
  // the residual: zeros where entries were kept
  if (sel[0] || sel[1] || sel[2] || sel[3]) {
    float4 z = cur;
    if (sel[0]) z.x = 0.f;
    if (sel[1]) z.y = 0.f;
    if (sel[2]) z.z = 0.f;
    if (sel[3]) z.w = 0.f;
    stq<AL>(e, tg.a0, tg.lo, tg.hi, q, z);
  }
  run.pos_run += total;
}

// The selection is taken before the two payload layouts part ways, so that every compare sits next
// to its ballot (a predicate that crosses a branch is carried as a 0 / 1 value per lane and
// compared again) and only lane masks in scalar registers cross.
template <bool AL, class RareF>
__device__ __forceinline__ void compact_group(const TileGeom& tg, const WaveSpan& span, int64_t layer_offset,
                                              const GroupSel& gs, RareF rare, CompactRun& run,
                                              float* __restrict__ e, int32_t* __restrict__ pidx,
                                              float* __restrict__ pval, int q, uint64_t m_span,
                                              const float4& cur, int lane, uint32_t* stg) {
  const bool qa = lane_bit(m_span);                         // m_span: the lanes whose group q is in the span
  uint64_t mv[4], msel[4];
  uint32_t key[4];
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    mv[c] = valid_mask<AL>(tg, q, c, qa, m_span);
    key[c] = key_of(comp(cur, c));
  }
  SelCommon sc;
  sc.t_all = gs.t_all;
  sc.ties = (gs.flags & 1u) != 0u;
  group_select(sc, [&]() { const GroupRare r = rare(); SelTies t; t.T = r.T; t.ktie = r.ktie; return t; },
               run.eq_run, key, mv, lane, msel);
  uint32_t below = 0, total = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    below = __builtin_amdgcn_mbcnt_hi((uint32_t)(msel[c] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)msel[c], below));
    total += (uint32_t)__popcll(msel[c]);
  }
  if ((gs.flags & 2u) != 0u) {                              // wave-uniform
    uint64_t mvs[4];
#pragma unroll
    for (int c = 0; c < 4; ++c) mvs[c] = scalar_mask(mv[c]);
    compact_selected<AL, true>(tg, layer_offset, gs, rare, run, e, pidx, pval, q, cur, lane, stg, msel, mvs, below, total);
  } else if (total != 0u) {
    compact_selected<AL, false>(tg, layer_offset, gs, rare, run, e, pidx, pval, q, cur, lane, stg, msel, mv, below, total);
  }
}

// One worker per grid row; the mean is taken later from the payloads.
template <bool AL>
__device__ __forceinline__ void compact_tile(const Ws& ws, int w, const FlatTile& ft, const LayerDev& L,
                                             const TileGeom& tg, uint32_t* stg) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const WaveSpan span = wave_span(tg, wave);
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  float4 cur = ld_span<AL>(e, tg, span, span.qbeg + lane);
  float4 nxt = ld_span<AL>(e, tg, span, span.qbeg + kWave + lane);
  const QuarterSel qs = load_quarter_sel(ws, w, ft.layer, L.qoff + 4 * (int64_t)(ft.start >> kTileShift) + wave);
  // wave-uniform values: into scalar registers, whatever kind of load fetched them
  CompactRun run;
  run.eq_run = rfl(qs.eq_before);
  run.pos_run = rfl(qs.gt_before + min(qs.ktie, qs.eq_before));
  GroupSel gs;
  gs.t_all = rfl(qs.t_all); gs.k = rfl(qs.k); gs.flags = rfl(qs.flags);
  auto rare = [&]() { GroupRare r; r.T = rfl(qs.T); r.ktie = rfl(qs.ktie); r.nholes = rfl(qs.nholes); return r; };
  int32_t* pidx = ws.pay_idx + (int64_t)w * ws.pay_stride + L.pay_off;
  float* pval = ws.pay_val + (int64_t)w * ws.pay_stride + L.pay_off;
  const int64_t layer_offset = L.offset;                   // by value: nothing is re-read inside the loop
  for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
    const int q = q0 + lane;
    const float4 nn = ld_span<AL>(e, tg, span, q + 2 * kWave);
    compact_group<AL>(tg, span, layer_offset, gs, rare, run, e, pidx, pval, q,
                      scalar_mask(ballot64(q < span.qend)), cur, lane, stg);
    cur = nxt;
    nxt = nn;
  }
}

__global__ __launch_bounds__(256) void topk_compact_kernel(const Ws ws, int w0) {
  const int w = w0 + blockIdx.y;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    atomicAnd(ws.tpending, ~(1u << w));                    // this path writes the residual itself
  }
  __shared__ uint32_t stage[4][kStgWords];
  uint32_t* stg = stage[__builtin_amdgcn_readfirstlane(threadIdx.x >> 6)];
  if (tg.aligned) compact_tile<true>(ws, w, ft, L, tg, stg);
  else compact_tile<false>(ws, w, ft, L, tg, stg);
}

// All workers in worker order, and the dense mean of the kept values: out[i] = (sum over the
// workers that kept i, from +0, of their value) / W.  A wave takes its quarter in chunks of
// kChunkGroups groups and, inside a chunk, worker by worker: the sums of a chunk live in registers,
// a worker's selection state is fetched and its payload entries are written once per chunk (the
// entries of a chunk are listed in LDS first), and the group a worker has just used is
// requested for the next worker at once, so that it has the rest of the chunk's work to arrive
// (the compiler waits for all requests at the top of a worker's turn).  The running compaction
// state of every worker is kept in one lane each.
constexpr int kChunkGroups = 4;
constexpr int kChunkCap = 2 * kGroupList;          // listed entries at which a wave writes its list out early
constexpr int kChunkStride = kChunkCap + kWave;    // + one slot per lane for the unselected elements
constexpr int kChunkWords = 2 * kChunkStride;      // indices, then values

// UPD: the mean is not written out but drives the optimizer step on the weights and the velocity
// (requested group by group once the chunk's sums are complete: requested earlier they cost
// 32 registers across the last worker's turn and two waves of occupancy).
// HOLES: the layer keeps more than half of its entries (static per level, the same for every worker).
template <bool AL, bool UPD, bool HOLES>
__device__ __forceinline__ void compact_mean_tile(const Ws& ws, const FlatTile& ft, const LayerDev& L,
                                                  const TileGeom& tg, const Sink sink, uint32_t* stg, int wave) {
  constexpr int G = kChunkGroups;
  const int lane = threadIdx.x & 63;
  const WaveSpan span = wave_span(tg, wave);
  const int n = (span.qend - span.qbeg + kWave - 1) / kWave;   // groups of the quarter, wave-uniform
  if (n <= 0) return;
  const int64_t qslot_local = L.qoff + 4 * (int64_t)(ft.start >> kTileShift) + wave;
  const int W = ws.W;
  // everything the loop needs from the layer and the workspace, by value (a reference into global
  // memory would be re-read after every store, and that wait would drain the loads in flight)
  const int64_t layer_offset = L.offset, pay_off = L.pay_off, e_stride = ws.e_stride, pay_stride = ws.pay_stride;
  const float* const e_base = ws.e;
  int32_t* const pay_idx = ws.pay_idx;
  float* const pay_val = ws.pay_val;
  // lane w holds worker w's selection state for this quarter
  QuarterSel mine = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
  if (lane < W) mine = load_quarter_sel(ws, lane, ft.layer, qslot_local);
  uint32_t eq_run_v = mine.eq_before;
  uint32_t pos_run_v = mine.gt_before + min(mine.ktie, mine.eq_before);
  const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
  // group j of chunk c of the worker whose memory is e (past the end of the quarter an aligned
  // tile re-reads its last group: nobody looks at it).  q_end: the end of the span, or its begin
  // for a request that nobody will look at (every lane then asks for the same 16 bytes, or for
  // nothing)
  auto load_group = [&](const float* __restrict__ e, int c, int j, int q_end) {
    const int q = span.qbeg + (c * G + j) * kWave + lane;
    if (AL) return ldq_clamped(e, tg.a0, min(q, max(q_end - 1, span.qbeg)));
    return ldq<AL>(e, tg.a0, tg.lo, tg.hi, q, q < q_end);
  };
  const float fw = (float)W;
  // x / W and x * (1 / W) are the same real number when W is a power of two, so both round alike
  const bool pow2 = (W & (W - 1)) == 0;
  const float rw = 1.0f / fw;
  const int n_chunks = (n + G - 1) / G;
  float4 cur[G];
#pragma unroll
  for (int j = 0; j < G; ++j) cur[j] = load_group(e_base, 0, j, span.qend);
  for (int c = 0; c < n_chunks; ++c) {
    uint64_t m_span[G];                                      // the same for every worker
#pragma unroll
    for (int j = 0; j < G; ++j)
      m_span[j] = scalar_mask(ballot64(span.qbeg + (c * G + j) * kWave + lane < span.qend));
    const int32_t i0_chunk = (int32_t)(tg.a0 + 4 * (int64_t)(span.qbeg + c * G * kWave + lane) - layer_offset);
    float4 acc[G], wq[G], vq[G];
#pragma unroll
    for (int j = 0; j < G; ++j) acc[j] = wq[j] = vq[j] = zero4;
    for (int w = 0; w < W; ++w) {
      // what the registers of a used group are loaded with: the same chunk of the next worker,
      // after the last worker the next chunk of the first
      // (after the last worker of the last chunk there is nothing to request, but a request behind
      // a branch would make every wait for a group wait for all requests: see load_group)
      const bool last_w = w + 1 == W;
      const float* __restrict__ e_next = e_base + (int64_t)(last_w ? 0 : w + 1) * e_stride;
      const int c_next = last_w ? min(c + 1, n_chunks - 1) : c;
      const int q_end_next = (last_w && c + 1 == n_chunks) ? span.qbeg : span.qend;
      SelCommon sc;
      sc.t_all = (uint32_t)__builtin_amdgcn_readlane((int)mine.t_all, w);
      const uint32_t k = (uint32_t)__builtin_amdgcn_readlane((int)mine.k, w);
      const uint32_t flags = (uint32_t)__builtin_amdgcn_readlane((int)mine.flags, w);
      sc.ties = (flags & 1u) != 0u;
      uint32_t eq_run = (uint32_t)__builtin_amdgcn_readlane((int)eq_run_v, w);
      uint32_t pos_run = (uint32_t)__builtin_amdgcn_readlane((int)pos_run_v, w);
      auto rare = [&]() {
        GroupRare r;
        r.T = (uint32_t)__builtin_amdgcn_readlane((int)mine.T, w);
        r.ktie = (uint32_t)__builtin_amdgcn_readlane((int)mine.ktie, w);
        r.nholes = (uint32_t)__builtin_amdgcn_readlane((int)mine.nholes, w);
        return r;
      };
      int32_t* __restrict__ pidx = pay_idx + (int64_t)w * pay_stride + pay_off;
      float* __restrict__ pval = pay_val + (int64_t)w * pay_stride + pay_off;
      uint32_t cnt = 0u;                                     // entries in the wave's list
      // the list goes out by consecutive lanes to consecutive addresses, as streaming stores (nothing
      // in this step reads the payload again); the byte offset is a 32-bit value (the payload of a
      // worker is far below 4 GiB)
      auto write_list = [&]() {
        __builtin_amdgcn_wave_barrier();                     // the list is complete (LDS is in order per wave)
#pragma unroll 1
        for (uint32_t t0 = 0u; t0 < cnt; t0 += kWave) {
          const uint32_t t = t0 + lane;
          const uint32_t ix = HOLES ? 0u : stg[t];
          const uint32_t vb = stg[kChunkStride + t];
          const uint32_t pos = pos_run + t;
          if (t < cnt && pos < k) {                          // pos < k: always true for consistent state
            const uint32_t boff = pos << 2;
            if (!HOLES) __builtin_nontemporal_store((int32_t)ix, (int32_t*)((char*)pidx + boff));
            __builtin_nontemporal_store(__uint_as_float(vb), (float*)((char*)pval + boff));
          }
        }
        __builtin_amdgcn_wave_barrier();
        pos_run += cnt;
        cnt = 0u;
      };
      // a worker whose layout differs from the layer's (never, for consistent state) is left out
      const bool layout_ok = ((flags & 2u) != 0u) == HOLES;
#pragma unroll
      for (int j = 0; j < G; ++j) {
        if (c * G + j < n && layout_ok) {                    // wave-uniform
          const int q = span.qbeg + (c * G + j) * kWave + lane;
          const float4 d = cur[j];
          const bool qa = lane_bit(m_span[j]);
          uint64_t mv[4], msel[4];
          uint32_t key[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            mv[x] = valid_mask<AL>(tg, q, x, qa, m_span[j]);
            key[x] = key_of(comp(d, x));
          }
          group_select(sc, [&]() { const GroupRare r = rare(); SelTies t; t.T = r.T; t.ktie = r.ktie; return t; },
                       eq_run, key, mv, lane, msel);
          uint32_t below = 0u, total = 0u;
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            below = __builtin_amdgcn_mbcnt_hi((uint32_t)(msel[x] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)msel[x], below));
            total += (uint32_t)__popcll(msel[x]);
          }
          if (HOLES || total != 0u) {                        // wave-uniform
            // the index of the lane's first element in the layer; hidden from the optimizer, which
            // would otherwise keep the indices of all elements of a chunk in registers across the loop
            // over the workers (sixteen registers, and one wave less per SIMD)
            int32_t i0 = i0_chunk + 4 * j * kWave;
            asm volatile("" : "+v"(i0));
            uint32_t nholes = 0u;
            if (HOLES) nholes = rare().nholes;
            uint32_t place = cnt + below;                    // of the lane's next selected element in the list
#pragma unroll
            for (int x = 0; x < 4; ++x) {
              const bool sel = lane_bit(msel[x]);
              const uint32_t slot = sel ? place : (uint32_t)(kChunkCap + lane);
              if (!HOLES) stg[slot] = (uint32_t)(i0 + x);
              stg[kChunkStride + slot] = __float_as_uint(comp(d, x));
              if (HOLES && lane_bit(scalar_mask(mv[x]) & ~msel[x])) {
                // dropped entry number (index - kept before it) of the layer
                const uint32_t hp = (uint32_t)(i0 + x) - (pos_run + place);
                if (hp < nholes) pidx[hp] = i0 + x;           // always true for consistent state
              }
              place += sel ? 1u : 0u;
              // acc is never -0, so adding +0 changes nothing
              if (x == 0) acc[j].x += sel ? d.x : 0.f;
              if (x == 1) acc[j].y += sel ? d.y : 0.f;
              if (x == 2) acc[j].z += sel ? d.z : 0.f;
              if (x == 3) acc[j].w += sel ? d.w : 0.f;
            }
            cnt += total;
          }
        }
        // the registers of the group are free: request what they hold next
        cur[j] = load_group(e_next, c_next, j, q_end_next);
        if (j + 1 < G && cnt > (uint32_t)(kChunkCap - kGroupList)) write_list();   // room for one more group
      }
      write_list();
      if (lane == w) { eq_run_v = eq_run; pos_run_v = pos_run; }
    }
#pragma unroll
    for (int j = 0; j < G; ++j) {
      const int q = span.qbeg + (c * G + j) * kWave + lane;
      if (UPD) {                                           // the group's weights and velocity
        if (sink.stream_wv) {                               // uniform: see stream_wv() on the host side
          wq[j] = ld_span<AL, true>(sink.wt, tg, span, q);
          vq[j] = ld_span<AL, true>(sink.vel, tg, span, q);
        } else {
          wq[j] = ld_span<AL>(sink.wt, tg, span, q);
          vq[j] = ld_span<AL>(sink.vel, tg, span, q);
        }
      }
      if (q < span.qend) {
        const float4 a = acc[j];
        const float4 v = pow2 ? make_float4(a.x * rw, a.y * rw, a.z * rw, a.w * rw)
                              : make_float4(a.x / fw, a.y / fw, a.z / fw, a.w / fw);
        if (UPD) {
          nesterov4(v, wq[j], vq[j], sink);
          if (sink.stream_wv) {
            stq<AL, true>(sink.wt, tg.a0, tg.lo, tg.hi, q, wq[j]);
            stq<AL, true>(sink.vel, tg.a0, tg.lo, tg.hi, q, vq[j]);
          } else {
            stq<AL>(sink.wt, tg.a0, tg.lo, tg.hi, q, wq[j]);
            stq<AL>(sink.vel, tg.a0, tg.lo, tg.hi, q, vq[j]);
          }
        } else {
          stq<AL, kStreamOut>(sink.out, tg.a0, tg.lo, tg.hi, q, v);
        }
      }
    }
  }
}

// The same pass from the candidate lists of pass A instead of Delta: for a layer whose guess held
// for every worker, whose lists are complete and which keeps at most half of its entries, a wave
// reads the (offset, value) candidates of its quarter worker by worker (6 bytes per candidate),
// picks the selected ones with the same rule (key >= t_all, or equal to T within the tie quota,
// in index order), writes them to the payload at consecutive positions (the selected lanes of one
// instruction write consecutive words) and adds the values into the quarter's dense sums in
// LDS, workers in order from +0; the sums, divided by W, go out as the quarter's part of the
// averaged gradient.  acc: the wave's kQuarterFloats floats of LDS.
constexpr int kGatherChunks = 4;                            // 64-entry chunks of a candidate list requested together (2 to 8: within 2 us)
constexpr int kQuarterGroups = (kTile / 4 + 1 + 3) / 4;     // 513: 16-byte groups of a wave quarter at most
constexpr int kQuarterFloats = 4 * kQuarterGroups + 12;     // rounded up to whole 64-byte rows
constexpr int kPayRing = 128;                               // a wave's payload ring in LDS: entries (indices, then values)

template <bool AL, bool UPD>
__device__ __forceinline__ void gather_mean_tile(const Ws& ws, const FlatTile& ft, const LayerDev& L,
                                                 const TileGeom& tg, const Sink sink, float* acc, uint32_t* ring,
                                                 int wave) {
  const int lane = threadIdx.x & 63;
  const WaveSpan span = wave_span(tg, wave);
  const int ng = span.qend - span.qbeg;                    // groups of the quarter, wave-uniform
  if (ng <= 0) return;
  int32_t* const ring_idx = reinterpret_cast<int32_t*>(ring);
  float* const ring_val = reinterpret_cast<float*>(ring + kPayRing);
  const int64_t qslot_local = L.qoff + 4 * (int64_t)(ft.start >> kTileShift) + wave;
  const int W = ws.W;
  const int64_t pay_off = L.pay_off, pay_stride = ws.pay_stride, q_stride = ws.q_stride;
  int32_t* const pay_idx = ws.pay_idx;
  float* const pay_val = ws.pay_val;
  const uint32_t* const cand_val = ws.cand_val;
  const uint16_t* const cand_idx = ws.cand_idx;
  // lane w holds worker w's selection state and candidate count for this quarter
  QuarterSel mine = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
  uint32_t n_mine = 0u;
  if (lane < W) {
    mine = load_quarter_sel(ws, lane, ft.layer, qslot_local);
    n_mine = ws.qinfo[(int64_t)lane * q_stride + qslot_local].y;   // beyond kCandCap: the list is incomplete
  }
  // A batch = up to kGatherChunks 64-entry chunks of one worker's list, requested together; the next
  // batch (the rest of this worker's list, else the head of the next worker's) is requested before
  // the current one is processed, whether or not anybody will look at it, so that a batch has the
  // processing of the one before it to arrive.
  constexpr int U = kGatherChunks;
  auto load_batch = [&](int w, uint32_t t0, uint32_t (&v)[U], uint32_t (&ix)[U]) {
    const int64_t qslot = (int64_t)w * q_stride + qslot_local;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t a = cand_at(ws, qslot, min(t0 / kWave + u, (uint32_t)(kCandCap / kWave - 1)), lane);
      v[u] = cand_val[a];
      ix[u] = cand_idx[a];
    }
  };
  uint32_t cv[U], ci[U];
  load_batch(0, 0u, cv, ci);
  float4* acc4 = reinterpret_cast<float4*>(acc);
  for (int g = lane; g < ng; g += kWave) acc4[g] = make_float4(0.f, 0.f, 0.f, 0.f);
  __builtin_amdgcn_wave_barrier();
  // index of the quarter's first element in the layer
  const int32_t i_quarter = (int32_t)(tg.a0 + 4 * (int64_t)span.qbeg - L.offset);
  for (int w = 0; w < W; ++w) {
    const uint32_t n_listed = (uint32_t)__builtin_amdgcn_readlane((int)n_mine, w);
    const uint32_t t_all = (uint32_t)__builtin_amdgcn_readlane((int)mine.t_all, w);
    const uint32_t k = (uint32_t)__builtin_amdgcn_readlane((int)mine.k, w);
    const bool ties = ((uint32_t)__builtin_amdgcn_readlane((int)mine.flags, w) & 1u) != 0u;
    const uint32_t T = (uint32_t)__builtin_amdgcn_readlane((int)mine.T, w);
    const uint32_t ktie = (uint32_t)__builtin_amdgcn_readlane((int)mine.ktie, w);
    uint32_t eq_run = (uint32_t)__builtin_amdgcn_readlane((int)mine.eq_before, w);
    uint32_t pos_run = (uint32_t)__builtin_amdgcn_readlane((int)mine.gt_before, w) + min(ktie, eq_run);
    int32_t* __restrict__ pidx = pay_idx + (int64_t)w * pay_stride + pay_off;
    float* __restrict__ pval = pay_val + (int64_t)w * pay_stride + pay_off;
    // This worker's list cannot serve this quarter -- it overflowed, or the threshold is zero and
    // some of the quarter's exact zeros, which no list holds, are kept (the tie quota is not used
    // up before it): the quarter is taken from Delta, group by group, with the same selection rule.
    const bool from_delta = n_listed > (uint32_t)kCandCap || (T == 0u && ties && eq_run < ktie);   // wave-uniform
    const uint32_t n = from_delta ? 0u : n_listed;
    if (from_delta) {
      const float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
      const SelCommon sc = {t_all, ties};
      for (int g0 = 0; g0 < ng; g0 += kWave) {
        const int q = span.qbeg + g0 + lane;
        const bool qa = q < span.qend;
        const float4 d = ld_span<AL>(e, tg, span, q);
        const uint64_t m_span = ballot64(qa);
        uint32_t key[4];
        uint64_t mv[4], msel[4];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          mv[c] = valid_mask<AL>(tg, q, c, qa, m_span);
          key[c] = key_of(comp(d, c));
        }
        group_select(sc, [&]() { SelTies t; t.T = T; t.ktie = ktie; return t; }, eq_run, key, mv, lane, msel);
        // Payload positions in index order: lane by lane, component by component.  The entries
        // pass through a ring in LDS (slot = position mod kPayRing), half a wave at a time -- 128
        // entries at most --, and leave it through consecutive lanes at consecutive positions.
        uint32_t pos = pos_run, total = 0u, total_lo = 0u;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
          pos += lanes_below(msel[c], lane);
          total += (uint32_t)__popcll(msel[c]);
          total_lo += (uint32_t)__popcll(msel[c] & 0xffffffffull);
        }
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          const uint32_t h_lo = pos_run + (half ? total_lo : 0u), h_hi = pos_run + (half ? total : total_lo);
          if (h_hi == h_lo) continue;                        // wave-uniform
          if ((lane >> 5) == half) {
            uint32_t p = pos;
#pragma unroll
            for (int c = 0; c < 4; ++c) {
              if (lane_bit(msel[c])) {
                const int32_t off = 4 * (g0 + lane) + c;     // offset in the quarter
                ring_idx[p & (kPayRing - 1)] = i_quarter + off;
                ring_val[p & (kPayRing - 1)] = comp(d, c);
                acc[off] += comp(d, c);
                ++p;
              }
            }
          }
          __builtin_amdgcn_wave_barrier();
          for (uint32_t j0 = h_lo; j0 < h_hi; j0 += kWave) {
            const uint32_t j = j0 + lane;
            if (j < h_hi && j < k) {                         // < k: always true for consistent state
              __builtin_nontemporal_store(ring_idx[j & (kPayRing - 1)], pidx + j);
              __builtin_nontemporal_store(ring_val[j & (kPayRing - 1)], pval + j);
            }
          }
          __builtin_amdgcn_wave_barrier();
        }
        pos_run += total;
      }
    }
    for (uint32_t t0 = 0u; t0 < n || t0 == 0u; t0 += U * kWave) {
      uint32_t nv[U], ni[U];
      const bool more = t0 + U * kWave < n;
      load_batch(more ? w : min(w + 1, W - 1), more ? t0 + U * kWave : 0u, nv, ni);
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const uint32_t t = t0 + u * kWave + lane;
        if (t0 + u * kWave < n) {                            // wave-uniform
          const uint32_t key = cv[u] & 0x7fffffffu;
          const uint64_t mvalid = ballot64(t < n);
          uint64_t msel = ballot64(key >= t_all) & mvalid;
          if (ties) {                                        // wave-uniform
            const uint64_t meq = ballot64(key == T) & mvalid;
            if (meq != 0) {
              const uint32_t rank = eq_run + lanes_below(meq, lane);
              msel |= ballot64(rank < ktie) & meq;
              eq_run += (uint32_t)__popcll(meq);
            }
          }
          msel = scalar_mask(msel);
          if (lane_bit(msel)) {
            const uint32_t pos = pos_run + lanes_below(msel, lane);
            if (pos < k) {                                   // always true for consistent state
              const uint32_t boff = pos << 2;
              __builtin_nontemporal_store(i_quarter + (int32_t)ci[u], (int32_t*)((char*)pidx + boff));
              __builtin_nontemporal_store(__uint_as_float(cv[u]), (float*)((char*)pval + boff));
            }
            // offsets are unique within a worker's list, and a wave's LDS operations keep their order
            acc[ci[u]] += __uint_as_float(cv[u]);
          }
          pos_run += (uint32_t)__popcll(msel);
        }
      }
#pragma unroll
      for (int u = 0; u < U; ++u) { cv[u] = nv[u]; ci[u] = ni[u]; }
    }
  }
  __builtin_amdgcn_wave_barrier();
  const float fw = (float)W;
  const bool pow2 = (W & (W - 1)) == 0;                     // then x / W and x * (1 / W) round alike
  const float rw = 1.0f / fw;
  for (int g0 = 0; g0 < ng; g0 += kWave) {
    const int g = g0 + lane;
    const int q = span.qbeg + g;
    float4 wq = make_float4(0.f, 0.f, 0.f, 0.f), vq = wq;
    if (UPD) {
      if (sink.stream_wv) {                                 // uniform: see stream_wv() on the host side
        wq = ld_span<AL, true>(sink.wt, tg, span, q);
        vq = ld_span<AL, true>(sink.vel, tg, span, q);
      } else {
        wq = ld_span<AL>(sink.wt, tg, span, q);
        vq = ld_span<AL>(sink.vel, tg, span, q);
      }
    }
    if (g < ng) {
      const float4 a = acc4[g];
      const float4 v = pow2 ? make_float4(a.x * rw, a.y * rw, a.z * rw, a.w * rw)
                            : make_float4(a.x / fw, a.y / fw, a.z / fw, a.w / fw);
      if (UPD) {
        nesterov4(v, wq, vq, sink);
        if (sink.stream_wv) {
          stq<AL, true>(sink.wt, tg.a0, tg.lo, tg.hi, q, wq);
          stq<AL, true>(sink.vel, tg.a0, tg.lo, tg.hi, q, vq);
        } else {
          stq<AL>(sink.wt, tg.a0, tg.lo, tg.hi, q, wq);
          stq<AL>(sink.vel, tg.a0, tg.lo, tg.hi, q, vq);
        }
      } else {
        stq<AL, kStreamOut>(sink.out, tg.a0, tg.lo, tg.hi, q, v);
      }
    }
  }
}

// The waves of this pass are independent of each other (one quarter of a tile each), so the
// workgroup can be smaller than a tile: kMeanWaves quarters per workgroup (two: 1 us faster than
// four on ResNet-18 shapes, the same as one).
constexpr int kMeanWaves = 2;
constexpr int kMeanSplit = 4 / kMeanWaves;                  // workgroups per tile
constexpr int kMeanLdsWords = kQuarterFloats + 2 * kPayRing > kChunkWords ? kQuarterFloats + 2 * kPayRing : kChunkWords;

template <bool UPD>
__device__ __forceinline__ void compact_mean_body(const Ws& ws, const Sink& sink) {
  const FlatTile ft = ws.ftiles[blockIdx.x / kMeanSplit];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    ws.words[1] = ws.words[0];
    ws.words[2] += ws.words[0];
  }
  // every e_w keeps Delta_w: the kept entries are dropped by the next pass over it
  if (blockIdx.x == 0 && threadIdx.x == 0) *ws.tpending = ws.W == 32 ? 0xffffffffu : ((1u << ws.W) - 1u);
  // a wave's LDS: the staging list of the pass over Delta, or the dense sums of the pass over the lists
  __shared__ __attribute__((aligned(16))) uint32_t stage[kMeanWaves][kMeanLdsWords];
  const int lw = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  uint32_t* stg = stage[lw];
  const int wave = (int)(blockIdx.x % kMeanSplit) * kMeanWaves + lw;   // the quarter of the tile
  // the payload layout of the layer at its level (k is the same for every worker)
  const uint32_t n_layer = (uint32_t)L.rows * (uint32_t)L.cols;
  const bool holes = payload_has_holes(n_layer, min(rfl(ws.sel[ft.layer].k), n_layer));
  if (holes) {
    if (tg.aligned) compact_mean_tile<true, UPD, true>(ws, ft, L, tg, sink, stg, wave);
    else compact_mean_tile<false, UPD, true>(ws, ft, L, tg, sink, stg, wave);
  } else if (L.ntiles > 1 && rfl(ws.lflag[ft.layer]) == 0u) {
    // every worker's guess held and every list is complete: the candidates serve
    if (tg.aligned) gather_mean_tile<true, UPD>(ws, ft, L, tg, sink, reinterpret_cast<float*>(stg), stg + kQuarterFloats, wave);
    else gather_mean_tile<false, UPD>(ws, ft, L, tg, sink, reinterpret_cast<float*>(stg), stg + kQuarterFloats, wave);
  } else {
    if (tg.aligned) compact_mean_tile<true, UPD, false>(ws, ft, L, tg, sink, stg, wave);
    else compact_mean_tile<false, UPD, false>(ws, ft, L, tg, sink, stg, wave);
  }
}

__global__ __launch_bounds__(kMeanWaves * kWave) void topk_compact_mean_kernel(const Ws ws, const Sink sink) {
  compact_mean_body<false>(ws, sink);
}

// The same pass with the optimizer step in place of the store of the mean.
__global__ __launch_bounds__(kMeanWaves * kWave) void topk_compact_update_kernel(const Ws ws, const Sink sink) {
  compact_mean_body<true>(ws, sink);
}

// ---- K6: dense mean of the W payloads (call-by-call path) ----------------------------------------

template <bool UPD>
__device__ __forceinline__ void sparse_mean_body(const Ws& ws, const Sink& sink) {
  __shared__ float acc[kTile];
  __shared__ uint16_t hole[kTile];                         // tile-local offsets of the dropped entries
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
    // payload positions of the tile's first quarter and of the next tile's first quarter
    const int64_t qs = (int64_t)w * ws.q_stride + L.qoff + 4 * (int64_t)tl;
    const SelState* sp = ws.sel + (int64_t)w * ws.L + ft.layer;
    const uint32_t ktie = sp->ktie, kk = sp->k;
    const uint32_t lo = ws.gtpre[qs] + min(ktie, ws.eqpre[qs]);
    const uint32_t hi = ws.gtpre[qs + 4] + min(ktie, ws.eqpre[qs + 4]);
    const int32_t* pidx = ws.pay_idx + (int64_t)w * ws.pay_stride + L.pay_off;
    const float* pval = ws.pay_val + (int64_t)w * ws.pay_stride + L.pay_off;
    const uint32_t n_layer = (uint32_t)L.rows * (uint32_t)L.cols;
    const uint32_t nholes = n_layer - min(kk, n_layer);
    if (!payload_has_holes(n_layer, kk)) {
      for (uint32_t p = lo + tid; p < hi && p < kk; p += kFlatThreads) {
        const int32_t i = pidx[p] - ft.start;
        if (i >= 0 && i < ft.count) acc[i] += pval[p];   // indices are unique within a worker
      }
    } else {
      // values in index order + hole list: the tile's entries are kept entries lo .. hi-1 and
      // holes (start - lo) .. (start + count - hi) - 1; entry i of the tile is kept entry
      // lo + i - (holes of the tile before i)
      const uint32_t h0 = (uint32_t)ft.start - lo;
      const uint32_t nh = nholes ? min((uint32_t)ft.count - (hi - lo), (uint32_t)kTile) : 0u;
      for (uint32_t t = tid; t < nh; t += kFlatThreads) {
        const uint32_t hp = min(h0 + t, nholes - 1u);
        hole[t] = (uint16_t)min((uint32_t)max(pidx[hp] - ft.start, 0), (uint32_t)(kTile - 1));
      }
      __syncthreads();
      for (int i = tid; i < ft.count; i += kFlatThreads) {
        uint32_t a = 0, b = nh;                              // first hole >= i
        while (a < b) {
          const uint32_t m = (a + b) >> 1;
          if ((int)hole[m] < i) a = m + 1; else b = m;
        }
        const bool is_hole = a < nh && (int)hole[a] == i;
        const uint32_t p = lo + (uint32_t)i - a;
        if (!is_hole && p < kk) acc[i] += pval[p];
      }
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
    if (UPD) {
      float4 wq = ld_quad(sink.wt, base, tg.lo, tg.hi);
      float4 vq = ld_quad(sink.vel, base, tg.lo, tg.hi);
      nesterov4(v, wq, vq, sink);
      st_quad(sink.wt, base, tg.lo, tg.hi, wq);
      st_quad(sink.vel, base, tg.lo, tg.hi, vq);
    } else {
      st_quad(sink.out, base, tg.lo, tg.hi, v);
    }
  }
}

__global__ __launch_bounds__(256) void topk_sparse_mean_kernel(const Ws ws, const Sink sink) {
  sparse_mean_body<false>(ws, sink);
}

__global__ __launch_bounds__(256) void topk_sparse_update_kernel(const Ws ws, const Sink sink) {
  sparse_mean_body<true>(ws, sink);
}

// ---- the residual written out on demand --------------------------------------------------------
// e_w = Delta_w with the kept entries zeroed, for the workers whose bit is set in *ws.tpending
// (accordion_flush / accordion_get_state); the caller clears the mask afterwards.
template <bool AL>
__device__ __forceinline__ void residual_tile(const Ws& ws, int w, const FlatTile& ft, const LayerDev& L,
                                              const TileGeom& tg) {
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const WaveSpan span = wave_span(tg, wave);
  float* __restrict__ e = ws.e + (int64_t)w * ws.e_stride;
  PrevSel ps = load_prev_sel(ws, (int64_t)w * ws.L + ft.layer, quarter_slot(ws, L, w, ft.start >> kTileShift, wave));
  for (int q0 = span.qbeg; q0 < span.qend; q0 += kWave) {
    const int q = q0 + lane;
    const bool qa = q < span.qend;
    const float4 d = ld_span<AL>(e, tg, span, q);
    const float4 z = drop_kept<AL>(tg, q, qa, ballot64(qa), ps, d, lane);
    if (qa && (z.x != d.x || z.y != d.y || z.z != d.z || z.w != d.w)) stq<AL>(e, tg.a0, tg.lo, tg.hi, q, z);
  }
}

__global__ __launch_bounds__(256) void topk_residual_kernel(const Ws ws) {
  const int w = blockIdx.y;
  if (((*ws.tpending >> w) & 1u) == 0u) return;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  const TileGeom tg = tile_geom(L, ft);
  if (tg.aligned) residual_tile<true>(ws, w, ft, L, tg);
  else residual_tile<false>(ws, w, ft, L, tg);
}

__global__ void topk_clear_pending_kernel(const Ws ws) {
  if (blockIdx.x == 0 && threadIdx.x == 0) *ws.tpending = 0u;
}

// ---- overlap of two workers' kept sets (Section 4.3) ---------------------------------------------
// Per layer, the number of coordinates both workers kept in the last step.  One workgroup per flat
// tile: worker a's index list of the tile (kept entries, or the holes when the layer keeps more than
// half) is marked in an LDS bit set, worker b's list is tested against it; for hole lists
// |kept_a & kept_b| = count - |holes_a| - |holes_b| + |holes_a & holes_b|.  Integer atomics on the
// per-layer counters (which the caller has cleared): the result does not depend on their order.
__global__ __launch_bounds__(256) void topk_overlap_kernel(const Ws ws, int wa, int wb,
                                                           unsigned long long* __restrict__ common) {
  __shared__ uint32_t bits[kTile / 32];
  __shared__ uint32_t hits;
  const int tid = threadIdx.x;
  const FlatTile ft = ws.ftiles[blockIdx.x];
  const LayerDev& L = ws.layers[ft.layer];
  for (int i = tid; i < kTile / 32; i += kFlatThreads) bits[i] = 0u;
  if (tid == 0) hits = 0u;
  __syncthreads();
  const int tl = ft.start >> kTileShift;
  const uint32_t n_layer = (uint32_t)L.rows * (uint32_t)L.cols;
  uint32_t listed[2];
  bool holes = false;
  for (int side = 0; side < 2; ++side) {
    const int w = side == 0 ? wa : wb;
    const int64_t qs = (int64_t)w * ws.q_stride + L.qoff + 4 * (int64_t)tl;
    const SelState* sp = ws.sel + (int64_t)w * ws.L + ft.layer;
    const uint32_t ktie = sp->ktie, kk = sp->k;
    const uint32_t lo = ws.gtpre[qs] + min(ktie, ws.eqpre[qs]);
    const uint32_t hi = ws.gtpre[qs + 4] + min(ktie, ws.eqpre[qs + 4]);
    const int32_t* pidx = ws.pay_idx + (int64_t)w * ws.pay_stride + L.pay_off;
    holes = payload_has_holes(n_layer, kk);
    uint32_t p0 = lo, p1 = min(hi, kk);
    if (holes) {                                             // the tile's part of the hole list
      const uint32_t nholes = n_layer - min(kk, n_layer);
      p0 = min((uint32_t)ft.start - lo, nholes);
      p1 = min((uint32_t)(ft.start + ft.count) - hi, nholes);
    }
    listed[side] = p1 > p0 ? p1 - p0 : 0u;
    uint32_t mine = 0;
    for (uint32_t p = p0 + tid; p < p1; p += kFlatThreads) {
      const int32_t i = pidx[p] - ft.start;
      if (i >= 0 && i < ft.count) {
        if (side == 0) atomicOr(&bits[i >> 5], 1u << (i & 31));
        else mine += (bits[i >> 5] >> (i & 31)) & 1u;
      }
    }
    if (side == 1) {
      mine = wave_sum_u32(mine);
      if ((tid & 63) == 0 && mine) atomicAdd(&hits, mine);
    }
    __syncthreads();
  }
  if (tid == 0) {
    const uint32_t both = holes ? (uint32_t)ft.count - listed[0] - listed[1] + hits : hits;
    if (both) atomicAdd(&common[ft.layer], (unsigned long long)both);
  }
}

__global__ __launch_bounds__(256) void zero_u64_kernel(unsigned long long* __restrict__ p, int n) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0ull;
}

}  // namespace acc
