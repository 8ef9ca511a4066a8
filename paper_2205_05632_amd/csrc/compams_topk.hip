// Top-k with error feedback (Definition 1 inside the worker lines of Algorithm 2) for gfx950.
//
// Per worker row:  x = e + g is stored in place of e, the k coordinates of largest magnitude key
// (fp32 pattern without the sign; ties to the lower coordinate) are written out as ascending
// (coordinate, value) lists and their residual entries are set to zero.
//
// The k-th largest key is found by a three-level radix select (12 + 10 + 9 key bits).  The level-0
// histogram is built by the same pass that forms x.  Everything after it works on a candidate list
// (all entries whose level-0 bucket is at least the threshold bucket), which is written
//   * by the first pass itself when the previous step's threshold bucket is carried over as a guess
//     and turns out to be low enough (no second read of the row), or
//   * by one more read of the row once the exact bucket is known, or
//   * not at all when it would not fit (rows dominated by equal keys): then every later pass reads
//     the row itself.
// All three routes give the same result; the guess only decides how many bytes move.
//
// Ordering: a candidate list is a set of per-chunk segments.  Each segment is in ascending coordinate
// order; segments are placed by an integer atomic cursor, so their physical order varies from run to
// run, but nothing that is output depends on it.  No floating-point atomics are used anywhere.

#include <cstdlib>
#include "compams_device.h"
#include "compams_internal.h"

namespace compams {
namespace {

// ---------------------------------------------------------------------------------------------
// First pass: x = e + g -> e, level-0 histogram, optional candidate emission with a guessed bucket.
// Grid (groups_per_row, n); each wavefront walks chunks wave, wave + stride, ...
// ---------------------------------------------------------------------------------------------
struct Quad {
  uint32_t key[4];
  bool ok[4];
};

__device__ __forceinline__ void hist4(uint32_t* lh, const Quad& q, uint32_t& zeros) {
  // Zero keys (frequent in sparse gradients) would serialise on one LDS word: count them by ballot.
  uint32_t z = 0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const bool isz = q.ok[s] && q.key[s] == 0;
    const uint64_t bz = ballot64(isz);
    if (bz) z += popc64(bz);
    if (q.ok[s] && q.key[s] != 0) atomicAdd(&lh[q.key[s] >> kL0Shift], 1u);
  }
  zeros += z;
}

// Number of flagged entries of one round, and this lane's position among them in (lane, slot) order.
struct RoundRank {
  uint32_t total;
  uint32_t below;
};
__device__ __forceinline__ RoundRank rank_round(const bool flag[4]) {
  const uint64_t b0 = ballot64(flag[0]), b1 = ballot64(flag[1]), b2 = ballot64(flag[2]), b3 = ballot64(flag[3]);
  RoundRank rr;
  rr.total = popc64(b0) + popc64(b1) + popc64(b2) + popc64(b3);
  rr.below = rr.total ? count_below(b0) + count_below(b1) + count_below(b2) + count_below(b3) : 0;
  return rr;
}

// Candidate entries of the chunk a wavefront is walking are first staged in LDS (kStage entries per
// wavefront) so that the chunk's segment can be allocated with one atomic once its size is known and
// then written with coalesced stores.  A chunk with more candidates than that is re-read instead.
constexpr int kStage = 512;

__device__ __forceinline__ void stage_round(uint2* stage, uint32_t& n, uint32_t j, const uint32_t bits[4],
                                            const bool flag[4]) {
  const RoundRank rr = rank_round(flag);
  if (rr.total == 0) return;
  uint32_t pos = n + rr.below;
#pragma unroll
  for (int s = 0; s < 4; ++s)
    if (flag[s]) {
      if (pos < static_cast<uint32_t>(kStage)) stage[pos] = make_uint2(j + s, bits[s]);
      ++pos;
    }
  n += rr.total;
}

// Allocate the chunk's segment and write it: from the staging area if everything fitted there, else by
// reading the chunk's (already stored) corrected gradients again.
__device__ __forceinline__ void flush_chunk(const uint2* stage, uint32_t cnt, const float* __restrict__ er, uint32_t d,
                                            uint32_t c, uint32_t thr_bucket, TopkRow* rowp, uint2* candr,
                                            uint32_t cap, uint2* descr) {
  const uint32_t lane = lane_id();
  uint32_t off = 0;
  if (cnt) {
    if (lane == 0) off = atomicAdd(&rowp->cursor, cnt);
    off = first_lane(off);
    if (off + cnt <= cap) {  // otherwise the row's list has overflowed and will not be used
      if (cnt <= static_cast<uint32_t>(kStage)) {
        for (uint32_t q = lane; q < cnt; q += 64) candr[off + q] = stage[q];
      } else {
        uint32_t at = off;
        for (int r = 0; r < kRounds; ++r) {
          const uint32_t j = c * kChunk + r * 256 + lane * 4;
          float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
          if (j < d) x = *reinterpret_cast<const float4*>(er + j);
          const uint32_t bits[4] = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z),
                                    __float_as_uint(x.w)};
          bool flag[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) flag[s] = j + s < d && (key_of_bits(bits[s]) >> kL0Shift) >= thr_bucket;
          const RoundRank rr = rank_round(flag);
          uint32_t pos = at + rr.below;
#pragma unroll
          for (int s = 0; s < 4; ++s)
            if (flag[s]) {
              if (pos < off + cnt) candr[pos] = make_uint2(j + s, bits[s]);
              ++pos;
            }
          at += rr.total;
        }
      }
    }
  }
  if (lane == 0) descr[c] = make_uint2(off, cnt);
}

typedef float f4v __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float* p) {
  const f4v v = __builtin_nontemporal_load(reinterpret_cast<const f4v*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void store_stream(float* p, const float4& x) {
  f4v v;
  v.x = x.x; v.y = x.y; v.z = x.z; v.w = x.w;
  __builtin_nontemporal_store(v, reinterpret_cast<f4v*>(p));
}

constexpr int kBatch = 4;  // rounds whose loads are issued together

template <bool PRED, bool FULL>
__device__ __forceinline__ void pass_a_chunk(const float* __restrict__ gr, float* __restrict__ er, uint32_t d,
                                             uint32_t c, uint32_t* lh, uint32_t& zeros, bool pred, uint32_t bg,
                                             TopkRow* rowp, uint2* candr, uint32_t cap, uint2* descr, uint2* stage, uint32_t dbg) {
  const uint32_t lane = lane_id();
  const uint32_t base = c * kChunk + lane * 4;
  uint32_t cnt = 0;
#pragma unroll 1
  for (int r0 = 0; r0 < kRounds; r0 += kBatch) {
    float4 gv[kBatch], ev[kBatch];
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t j = base + (r0 + u) * 256;
      gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      ev[u] = gv[u];
      if (FULL || j < d) {
        gv[u] = load_stream(gr + j);
        ev[u] = load_stream(er + j);
      }
    }
#pragma unroll
    for (int u = 0; u < kBatch; ++u) {
      const uint32_t j = base + (r0 + u) * 256;
      const bool in = FULL || j < d;
      float4 x = make_float4(ev[u].x + gv[u].x, ev[u].y + gv[u].y, ev[u].z + gv[u].z, ev[u].w + gv[u].w);
      Quad q;
      q.ok[0] = in; q.ok[1] = FULL || j + 1 < d; q.ok[2] = FULL || j + 2 < d; q.ok[3] = FULL || j + 3 < d;
      if (!FULL) {  // columns >= d keep what they held
        if (!q.ok[1]) x.y = ev[u].y;
        if (!q.ok[2]) x.z = ev[u].z;
        if (!q.ok[3]) x.w = ev[u].w;
      }
      if (in) store_stream(er + j, x);
      const uint32_t bits[4] = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z),
                                __float_as_uint(x.w)};
#pragma unroll
      for (int s = 0; s < 4; ++s) q.key[s] = key_of_bits(bits[s]);
      if (!(dbg & 1)) hist4(lh, q, zeros);
      if constexpr (PRED) {
        if (pred && !(dbg & 2)) {
          bool flag[4];
#pragma unroll
          for (int s = 0; s < 4; ++s) flag[s] = q.ok[s] && (q.key[s] >> kL0Shift) >= bg;
          stage_round(stage, cnt, j, bits, flag);
        }
      }
    }
  }
  if constexpr (PRED)
    if (pred) flush_chunk(stage, cnt, er, d, c, bg, rowp, candr, cap, descr);
}

template <bool PRED>
__global__ __launch_bounds__(kWG) void k_topk_pass_a(const float* __restrict__ g, float* __restrict__ e,
                                                      Geometry geo, TopkWorkspace ws, TopkOptions opt) {
  __shared__ uint32_t lh[kNB0];
  __shared__ uint2 stage_all[PRED ? kWaves * kStage : 1];
  const uint32_t row = blockIdx.y;
  for (int b = threadIdx.x; b < kNB0; b += kWG) lh[b] = 0;
  __syncthreads();
  const float* gr = g + static_cast<int64_t>(row) * geo.ld;
  float* er = e + static_cast<int64_t>(row) * geo.ld;
  TopkRow* rowp = ws.rows + row;
  bool pred = false;
  uint32_t bg = 0;
  if (PRED) {
    pred = rowp->pred_valid != 0;
    bg = rowp->b_guess;
  }
  uint2* candr = ws.cand + static_cast<size_t>(row) * opt.cap;
  uint2* descr = ws.desc + static_cast<size_t>(row) * geo.num_chunks;
  const uint32_t wave = threadIdx.x >> 6;
  uint2* stage = stage_all + (PRED ? wave * kStage : 0);
  const uint32_t stride = gridDim.x * kWaves;
  uint32_t zeros = 0;
  for (uint32_t c = blockIdx.x * kWaves + wave; c < geo.num_chunks; c += stride) {
    if ((c + 1) * static_cast<uint64_t>(kChunk) <= geo.d)
      pass_a_chunk<PRED, true>(gr, er, geo.d, c, lh, zeros, pred, bg, rowp, candr, opt.cap, descr, stage, opt.dbg);
    else
      pass_a_chunk<PRED, false>(gr, er, geo.d, c, lh, zeros, pred, bg, rowp, candr, opt.cap, descr, stage, opt.dbg);
  }
  if (zeros && lane_id() == 0) atomicAdd(&lh[0], zeros);
  __syncthreads();
  uint32_t* gh = ws.hist0 + static_cast<size_t>(row) * kNB0;
  for (int b = threadIdx.x; b < kNB0; b += kWG) {
    const uint32_t h = lh[b];
    if (h) atomicAdd(&gh[b], h);
  }
}

// ---------------------------------------------------------------------------------------------
// Finding the bucket in which a suffix count crosses `need`, by one workgroup of kWG threads.
// h: NB bucket counts in LDS.  Returns (wave-uniformly, through LDS) the largest s with
// sum_{b >= s} h[b] >= need, and the count strictly above it.  Requires 1 <= need <= sum h.
// ---------------------------------------------------------------------------------------------
template <int NB>
__device__ void find_crossing(const uint32_t* h, uint32_t need, uint32_t* suf /* kWG + 1 */, uint32_t* out2) {
  constexpr int PER = NB / kWG;
  static_assert(NB % kWG == 0, "buckets per thread");
  const int t = threadIdx.x;
  uint32_t part = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) part += h[t * PER + i];
  suf[t] = part;
  if (t == 0) { suf[kWG] = 0; out2[0] = 0; out2[1] = 0; }
  __syncthreads();
  // inclusive suffix sums by doubling
  for (int s = 1; s < kWG; s <<= 1) {
    const uint32_t add = (t + s < kWG) ? suf[t + s] : 0;
    __syncthreads();
    suf[t] += add;
    __syncthreads();
  }
  if (suf[t] >= need && suf[t + 1] < need) {
    uint32_t acc = suf[t + 1];
    for (int i = PER - 1; i >= 0; --i) {
      const uint32_t hb = h[t * PER + i];
      if (acc + hb >= need) {
        out2[0] = t * PER + i;
        out2[1] = acc;
        break;
      }
      acc += hb;
    }
  }
  __syncthreads();
}

// Level 0: one workgroup per row.
__global__ __launch_bounds__(kWG) void k_topk_resolve0(Geometry geo, TopkWorkspace ws, TopkOptions opt) {
  __shared__ uint32_t h[kNB0];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  const uint32_t row = blockIdx.x;
  uint32_t* gh = ws.hist0 + static_cast<size_t>(row) * kNB0;
  for (int b = threadIdx.x; b < kNB0; b += kWG) {
    h[b] = gh[b];
    gh[b] = 0;  // ready for the next step
  }
  __syncthreads();
  find_crossing<kNB0>(h, geo.k, suf, out2);
  if (threadIdx.x == 0) {
    TopkRow* rp = ws.rows + row;
    const uint32_t bstar = out2[0], above = out2[1];
    const uint32_t total = above + h[bstar];  // entries with bucket >= bstar
    const bool pred_ok = opt.first_pass_emits && rp->pred_valid && bstar >= rp->b_guess && rp->cursor <= opt.cap &&
                         !opt.force_dense;
    uint32_t mode, n_src, reads;
    if (pred_ok) { mode = kModeCand; n_src = rp->cursor; reads = 0; }
    else if (total <= opt.cap && !opt.force_dense) { mode = kModeNeedB; n_src = total; reads = 1; }
    else { mode = kModeDense; n_src = 0; reads = 4; }
    rp->mode = mode;
    rp->n_src = n_src;
    rp->cursor = 0;
    rp->bstar = bstar;
    rp->need = geo.k - above;
    // Guess for the next step: one bucket below this step's threshold bucket if the list that guess would
    // have produced now fits with room to spare, else the bucket itself, else no guess.
    uint32_t valid = 0, guess = 0;
    if (opt.predict && !opt.force_dense) {
      const uint32_t below = bstar ? h[bstar - 1] : 0;
      if (bstar && total + below <= opt.cap / 2) { valid = 1; guess = bstar - 1; }
      else if (total <= opt.cap / 2) { valid = 1; guess = bstar; }
    }
    rp->pred_valid = valid;
    rp->b_guess = guess;
    uint32_t* cn = ws.counters + row * 4;
    cn[0] = reads;
    cn[1] = n_src;
  }
}

// Second dense pass (rows in kModeNeedB only): candidate list = entries with level-0 bucket >= bstar.
__global__ __launch_bounds__(kWG) void k_topk_pass_b(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                      TopkOptions opt) {
  __shared__ uint2 stage_all[kWaves * kStage];
  const uint32_t row = blockIdx.y;
  TopkRow* rowp = ws.rows + row;
  if (rowp->mode != kModeNeedB) return;
  const uint32_t bstar = rowp->bstar;
  const float* er = e + static_cast<int64_t>(row) * geo.ld;
  uint2* candr = ws.cand + static_cast<size_t>(row) * opt.cap;
  uint2* descr = ws.desc + static_cast<size_t>(row) * geo.num_chunks;
  const uint32_t wave = threadIdx.x >> 6, lane = lane_id();
  uint2* stage = stage_all + wave * kStage;
  const uint32_t stride = gridDim.x * kWaves;
  for (uint32_t c = blockIdx.x * kWaves + wave; c < geo.num_chunks; c += stride) {
    const uint32_t base = c * kChunk + lane * 4;
    uint32_t cnt = 0;
#pragma unroll 4
    for (int r = 0; r < kRounds; ++r) {
      const uint32_t j = base + r * 256;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < geo.d) x = *reinterpret_cast<const float4*>(er + j);
      const uint32_t bits[4] = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z),
                                __float_as_uint(x.w)};
      bool flag[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) flag[s] = j + s < geo.d && (key_of_bits(bits[s]) >> kL0Shift) >= bstar;
      stage_round(stage, cnt, j, bits, flag);
    }
    // fits by construction: the level-0 histogram counted exactly these entries
    flush_chunk(stage, cnt, er, geo.d, c, bstar, rowp, candr, opt.cap, descr);
  }
}

// ---------------------------------------------------------------------------------------------
// Levels 1 and 2: histogram of the next key bits over the entries that match the prefix so far.
// LEVEL 1: match (key >> 19) == bstar, bin = (key >> 9) & 1023.  LEVEL 2: match (key >> 9) == prefix1,
// bin = key & 511.  Source: the candidate list (linear sweep) or the row itself.
// ---------------------------------------------------------------------------------------------
template <int LEVEL>
__global__ __launch_bounds__(kWG) void k_topk_hist(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                    TopkOptions opt) {
  constexpr int NB = LEVEL == 1 ? kNB1 : kNB2;
  __shared__ uint32_t lh[NB];
  const uint32_t row = blockIdx.y;
  const TopkRow* rowp = ws.rows + row;
  const uint32_t mode = rowp->mode;
  const uint32_t want = LEVEL == 1 ? rowp->bstar : rowp->prefix1;
  for (int b = threadIdx.x; b < NB; b += kWG) lh[b] = 0;
  __syncthreads();
  auto visit = [&](uint32_t bits, bool ok) {
    const uint32_t key = key_of_bits(bits);
    if (LEVEL == 1) {
      if (ok && (key >> kL0Shift) == want) atomicAdd(&lh[(key >> kL1Shift) & (kNB1 - 1)], 1u);
    } else {
      if (ok && (key >> kL1Shift) == want) atomicAdd(&lh[key & (kNB2 - 1)], 1u);
    }
  };
  if (mode == kModeDense) {
    const float* er = e + static_cast<int64_t>(row) * geo.ld;
    const uint32_t step = gridDim.x * kWG * 4;
    for (uint32_t j = (blockIdx.x * kWG + threadIdx.x) * 4; j < geo.d; j += step) {
      const float4 x = *reinterpret_cast<const float4*>(er + j);
      visit(__float_as_uint(x.x), true);
      visit(__float_as_uint(x.y), j + 1 < geo.d);
      visit(__float_as_uint(x.z), j + 2 < geo.d);
      visit(__float_as_uint(x.w), j + 3 < geo.d);
    }
  } else {
    const uint2* candr = ws.cand + static_cast<size_t>(row) * opt.cap;
    const uint32_t n_src = rowp->n_src;
    const uint32_t step = gridDim.x * kWG;
    for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < n_src; q += step) visit(candr[q].y, true);
  }
  __syncthreads();
  uint32_t* gh = (LEVEL == 1 ? ws.hist1 : ws.hist2) + static_cast<size_t>(row) * NB;
  for (int b = threadIdx.x; b < NB; b += kWG) {
    const uint32_t h = lh[b];
    if (h) atomicAdd(&gh[b], h);
  }
}

template <int LEVEL>
__global__ __launch_bounds__(kWG) void k_topk_resolve(Geometry geo, TopkWorkspace ws) {
  constexpr int NB = LEVEL == 1 ? kNB1 : kNB2;
  __shared__ uint32_t h[NB];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  const uint32_t row = blockIdx.x;
  TopkRow* rp = ws.rows + row;
  uint32_t* gh = (LEVEL == 1 ? ws.hist1 : ws.hist2) + static_cast<size_t>(row) * NB;
  for (int b = threadIdx.x; b < NB; b += kWG) {
    h[b] = gh[b];
    gh[b] = 0;
  }
  __syncthreads();
  const uint32_t need = rp->need;
  find_crossing<NB>(h, need, suf, out2);
  if (threadIdx.x == 0) {
    const uint32_t s = out2[0], above = out2[1];
    if (LEVEL == 1) {
      rp->prefix1 = (rp->bstar << (kL0Shift - kL1Shift)) | s;
      rp->need = need - above;
    } else {
      const uint32_t tau = (rp->prefix1 << kL1Shift) | s;
      const uint32_t r = need - above, ties = h[s];
      rp->tau = tau;
      rp->r = r;
      rp->ties = ties;
      rp->take_all_ties = (r == ties);
      ws.tau[row] = tau;
      uint32_t* cn = ws.counters + row * 4;
      cn[2] = ties;
      cn[3] = r;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Chunk-ordered sweeps.  A wavefront visits a chunk's entries round by round; within a round the
// order (lane, slot) is ascending coordinate order, in both sources.
// ---------------------------------------------------------------------------------------------
struct Entry4 {
  uint32_t j[4];
  uint32_t bits[4];
  bool ok[4];
};

// f(const Entry4&, int slots) is called wave-uniformly once per round.
template <typename F>
__device__ __forceinline__ void for_each_round(uint32_t mode, const float* __restrict__ er, uint32_t d, uint32_t c,
                                               const uint2* __restrict__ candr, const uint2* __restrict__ descr,
                                               uint32_t cap, F&& f) {
  const uint32_t lane = lane_id();
  if (mode == kModeDense) {
    const uint32_t base = c * kChunk + lane * 4;
    for (int r = 0; r < kRounds; ++r) {
      const uint32_t j = base + r * 256;
      if (c * kChunk + r * 256 >= d) break;  // wave-uniform
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < d) x = *reinterpret_cast<const float4*>(er + j);
      Entry4 en;
      en.bits[0] = __float_as_uint(x.x); en.bits[1] = __float_as_uint(x.y);
      en.bits[2] = __float_as_uint(x.z); en.bits[3] = __float_as_uint(x.w);
#pragma unroll
      for (int s = 0; s < 4; ++s) { en.j[s] = j + s; en.ok[s] = j + s < d; }
      f(en, 4);
    }
  } else {
    const uint2 ds = descr[c];
    const uint32_t off = first_lane(ds.x);
    uint32_t cnt = first_lane(ds.y);
    if (off > cap) cnt = 0;                      // segments always lie inside the list; never read outside it
    else if (cnt > cap - off) cnt = cap - off;
    for (uint32_t t = 0; t < cnt; t += 64) {
      Entry4 en;
      const uint32_t q = t + lane;
      en.ok[0] = q < cnt;
      uint2 cv = make_uint2(0, 0);
      if (en.ok[0]) cv = candr[off + q];
      en.j[0] = cv.x; en.bits[0] = cv.y;
#pragma unroll
      for (int s = 1; s < 4; ++s) { en.j[s] = 0; en.bits[s] = 0; en.ok[s] = false; }
      f(en, 1);
    }
  }
}

// Per chunk: how many keys lie above tau and how many equal it.
__global__ __launch_bounds__(kWG) void k_topk_count(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                     TopkOptions opt) {
  const uint32_t row = blockIdx.y;
  const TopkRow* rowp = ws.rows + row;
  const uint32_t mode = rowp->mode, tau = rowp->tau;
  const float* er = e + static_cast<int64_t>(row) * geo.ld;
  const uint2* candr = ws.cand + static_cast<size_t>(row) * opt.cap;
  const uint2* descr = ws.desc + static_cast<size_t>(row) * geo.num_chunks;
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t stride = gridDim.x * kWaves;
  for (uint32_t c = blockIdx.x * kWaves + wave; c < geo.num_chunks; c += stride) {
    uint32_t gt = 0, eq = 0;
    for_each_round(mode, er, geo.d, c, candr, descr, opt.cap, [&](const Entry4& en, int slots) {
      for (int s = 0; s < slots; ++s) {
        const uint32_t key = key_of_bits(en.bits[s]);
        gt += popc64(ballot64(en.ok[s] && key > tau));
        eq += popc64(ballot64(en.ok[s] && key == tau));
      }
    });
    if (lane_id() == 0) {
      ws.cnt_gt[static_cast<size_t>(row) * geo.num_chunks + c] = gt;
      ws.cnt_eq[static_cast<size_t>(row) * geo.num_chunks + c] = eq;
    }
  }
}

// Per row: exclusive prefix over chunks of the selected counts, and of the tie counts.
constexpr int kScanWG = 1024;
__global__ __launch_bounds__(kScanWG) void k_topk_scan(Geometry geo, TopkWorkspace ws) {
  __shared__ uint32_t scratch[kScanWG / 64 + 1];
  const uint32_t row = blockIdx.x;
  TopkRow* rp = ws.rows + row;
  const uint32_t r = rp->r;
  const size_t rb = static_cast<size_t>(row) * geo.num_chunks;
  uint32_t* sel_off = ws.sel_off + static_cast<size_t>(row) * (geo.num_chunks + 1);
  uint32_t eq_carry = 0, sel_carry = 0;
  for (uint32_t c0 = 0; c0 < geo.num_chunks; c0 += kScanWG) {
    const uint32_t c = c0 + threadIdx.x;
    const bool in = c < geo.num_chunks;
    const uint32_t eq = in ? ws.cnt_eq[rb + c] : 0;
    const uint32_t gt = in ? ws.cnt_gt[rb + c] : 0;
    uint32_t eq_total, sel_total;
    const uint32_t eq_before = eq_carry + block_excl_scan<kScanWG>(eq, scratch, &eq_total);
    // ties are taken in coordinate order until r of them are in
    const uint32_t room = r > eq_before ? r - eq_before : 0;
    const uint32_t take = eq < room ? eq : room;
    const uint32_t sel_before = sel_carry + block_excl_scan<kScanWG>(gt + take, scratch, &sel_total);
    if (in) {
      ws.eq_before[rb + c] = eq_before;
      sel_off[c] = sel_before;
    }
    eq_carry += eq_total;
    sel_carry += sel_total;
  }
  if (threadIdx.x == 0) {
    sel_off[geo.num_chunks] = sel_carry;  // == k
    rp->cursor = 0;                       // the list has been counted; the next first pass allocates from 0
  }
}

// Per chunk: write the selected (coordinate, value) pairs at their final ascending positions and clear
// their residual entries (the worker's error update of Algorithm 2 for the kept coordinates).
__global__ __launch_bounds__(kWG) void k_topk_emit(float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                    TopkOptions opt) {
  const uint32_t row = blockIdx.y;
  const TopkRow* rowp = ws.rows + row;
  const uint32_t mode = rowp->mode, tau = rowp->tau, r = rowp->r;
  const bool all_ties = rowp->take_all_ties != 0;
  float* er = e + static_cast<int64_t>(row) * geo.ld;
  const uint2* candr = ws.cand + static_cast<size_t>(row) * opt.cap;
  const uint2* descr = ws.desc + static_cast<size_t>(row) * geo.num_chunks;
  int32_t* idx = ws.idx + static_cast<size_t>(row) * geo.k;
  float* val = ws.val + static_cast<size_t>(row) * geo.k;
  const size_t rb = static_cast<size_t>(row) * geo.num_chunks;
  const uint32_t* sel_off = ws.sel_off + static_cast<size_t>(row) * (geo.num_chunks + 1);
  const uint32_t wave = threadIdx.x >> 6;
  const uint32_t stride = gridDim.x * kWaves;
  for (uint32_t c = blockIdx.x * kWaves + wave; c < geo.num_chunks; c += stride) {
    uint32_t at = sel_off[c];
    if (sel_off[c + 1] == at) continue;  // nothing selected in this chunk (wave-uniform)
    uint32_t eq_seen = ws.eq_before[rb + c];
    for_each_round(mode, er, geo.d, c, candr, descr, opt.cap, [&](const Entry4& en, int slots) {
      bool sel[4] = {false, false, false, false};
      if (all_ties) {
        for (int s = 0; s < slots; ++s) sel[s] = en.ok[s] && key_of_bits(en.bits[s]) >= tau;
      } else {
        uint64_t be[4];
        uint32_t below = 0, total = 0;
        for (int s = 0; s < slots; ++s) {
          be[s] = ballot64(en.ok[s] && key_of_bits(en.bits[s]) == tau);
          below += count_below(be[s]);
          total += popc64(be[s]);
        }
        uint32_t rank = eq_seen + below;  // ties before this lane's first slot, in coordinate order
        for (int s = 0; s < slots; ++s) {
          const uint32_t key = key_of_bits(en.bits[s]);
          const bool is_eq = en.ok[s] && key == tau;
          sel[s] = en.ok[s] && (key > tau || (is_eq && rank < r));
          rank += is_eq;
        }
        eq_seen += total;
      }
      uint64_t bs[4];
      uint32_t below = 0, total = 0;
      for (int s = 0; s < slots; ++s) {
        bs[s] = ballot64(sel[s]);
        below += count_below(bs[s]);
        total += popc64(bs[s]);
      }
      uint32_t pos = at + below;
      for (int s = 0; s < slots; ++s)
        if (sel[s]) {
          if (pos < geo.k && en.j[s] < geo.d) {  // always true when the counts are consistent
            idx[pos] = static_cast<int32_t>(en.j[s]);
            val[pos] = __uint_as_float(en.bits[s]);
            if (!(opt.dbg & 8)) er[en.j[s]] = 0.0f;
          }
          ++pos;
        }
      at += total;
    });
  }
}

// ---------------------------------------------------------------------------------------------
// Server lines of Algorithm 2 for sparse messages: worker-ordered sum of the selected values, divided
// by n, then the AMSGrad moment and parameter update.  One workgroup per chunk of coordinates; the
// chunk's averaged gradient lives in LDS.  Workers are added one after the other (a barrier between
// them), and one worker's coordinates are distinct, so no atomics are needed and the fp32 sum has
// exactly the order i = 0 .. n-1.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void ams_update(float gb, float& th, float& mm, float& vv, float& vh, const AmsParams& p) {
  const float mj = p.beta1 * mm + p.one_minus_beta1 * gb;
  const float vj = p.beta2 * vv + p.one_minus_beta2 * (gb * gb);
  const float vhj = (vh < vj) ? vj : vh;
  const float den = p.eps_out ? sqrtf(vhj) + p.eps : sqrtf(vhj + p.eps);
  mm = mj;
  vv = vj;
  vh = vhj;
  th = th - p.lr * (mj / den);
}

__global__ __launch_bounds__(kWG) void k_topk_amsgrad(float* __restrict__ theta, float* __restrict__ m,
                                                       float* __restrict__ v, float* __restrict__ vhat, Geometry geo,
                                                       TopkWorkspace ws, AmsParams p) {
  __shared__ float gs[kChunk];
  const uint32_t c = blockIdx.x;
  const uint32_t base = c * kChunk;
  for (int t = threadIdx.x; t < kChunk; t += kWG) gs[t] = 0.0f;
  __syncthreads();
  for (uint32_t i = 0; i < geo.n; ++i) {
    const uint32_t* so = ws.sel_off + static_cast<size_t>(i) * (geo.num_chunks + 1) + c;
    const uint32_t lo = so[0], hi = so[1];
    const int32_t* idx = ws.idx + static_cast<size_t>(i) * geo.k;
    const float* val = ws.val + static_cast<size_t>(i) * geo.k;
    for (uint32_t q = lo + threadIdx.x; q < hi && q < geo.k; q += kWG) {
      const uint32_t j = static_cast<uint32_t>(idx[q]) - base;
      if (j < static_cast<uint32_t>(kChunk)) gs[j] = gs[j] + val[q];
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < kChunk / (kWG * 4); ++r) {
    const uint32_t t = r * kWG * 4 + threadIdx.x * 4;
    const uint32_t j = base + t;
    if (j + 3 < geo.d) {
      float4 th = *reinterpret_cast<float4*>(theta + j), mm = *reinterpret_cast<float4*>(m + j);
      float4 vv = *reinterpret_cast<float4*>(v + j), vh = *reinterpret_cast<float4*>(vhat + j);
      const float4 s = *reinterpret_cast<const float4*>(gs + t);
      ams_update(s.x / p.nf, th.x, mm.x, vv.x, vh.x, p);
      ams_update(s.y / p.nf, th.y, mm.y, vv.y, vh.y, p);
      ams_update(s.z / p.nf, th.z, mm.z, vv.z, vh.z, p);
      ams_update(s.w / p.nf, th.w, mm.w, vv.w, vh.w, p);
      *reinterpret_cast<float4*>(theta + j) = th;
      *reinterpret_cast<float4*>(m + j) = mm;
      *reinterpret_cast<float4*>(v + j) = vv;
      *reinterpret_cast<float4*>(vhat + j) = vh;
    } else {
      for (uint32_t s = 0; s < 4 && j + s < geo.d; ++s) {
        float th = theta[j + s], mm = m[j + s], vv = v[j + s], vh = vhat[j + s];
        ams_update(gs[t + s] / p.nf, th, mm, vv, vh, p);
        theta[j + s] = th; m[j + s] = mm; v[j + s] = vv; vhat[j + s] = vh;
      }
    }
  }
}

}  // namespace

#define COMPAMS_CHECK_LAUNCH()                    \
  do {                                            \
    hipError_t err__ = hipGetLastError();         \
    if (err__ != hipSuccess) return err__;        \
  } while (0)

hipError_t topk_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt_in, const AmsParams& ap,
                     const float* g, float* e, float* theta, float* m, float* v, float* vhat,
                     bool first_pass_may_predict, hipStream_t stream, Launcher* L) {
  TopkOptions opt = opt_in;
  opt.first_pass_emits = first_pass_may_predict ? 1u : 0u;
  const uint32_t G = groups_per_row(geo.n, geo.num_chunks);
  uint32_t GA = G;
  if (getenv("COMPAMS_TUNE_GA")) GA = atoi(getenv("COMPAMS_TUNE_GA"));
  if (getenv("COMPAMS_TUNE_DBG")) opt.dbg = atoi(getenv("COMPAMS_TUNE_DBG"));
  const dim3 grid_rows(G, geo.n), wg(kWG), grid_a(GA, geo.n);
  {
    ScopedSlot s(L, kSlotPassA, stream);
    if (first_pass_may_predict)
      hipLaunchKernelGGL(k_topk_pass_a<true>, grid_a, wg, 0, stream, g, e, geo, ws, opt);
    else
      hipLaunchKernelGGL(k_topk_pass_a<false>, grid_a, wg, 0, stream, g, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotResolve0, stream);
    hipLaunchKernelGGL(k_topk_resolve0, dim3(geo.n), wg, 0, stream, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotPassB, stream);
    hipLaunchKernelGGL(k_topk_pass_b, grid_rows, wg, 0, stream, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  // sweeps over the (short) candidate lists use fewer, fully occupied workgroups per row
  const dim3 grid_hist(G, geo.n);
  {
    ScopedSlot s(L, kSlotHist1, stream);
    hipLaunchKernelGGL(k_topk_hist<1>, grid_hist, wg, 0, stream, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotResolve1, stream);
    hipLaunchKernelGGL(k_topk_resolve<1>, dim3(geo.n), wg, 0, stream, geo, ws);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotHist2, stream);
    hipLaunchKernelGGL(k_topk_hist<2>, grid_hist, wg, 0, stream, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotResolve2, stream);
    hipLaunchKernelGGL(k_topk_resolve<2>, dim3(geo.n), wg, 0, stream, geo, ws);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotCount, stream);
    hipLaunchKernelGGL(k_topk_count, grid_rows, wg, 0, stream, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotScan, stream);
    hipLaunchKernelGGL(k_topk_scan, dim3(geo.n), dim3(kScanWG), 0, stream, geo, ws);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotEmit, stream);
    hipLaunchKernelGGL(k_topk_emit, grid_rows, wg, 0, stream, e, geo, ws, opt);
  }
  COMPAMS_CHECK_LAUNCH();
  {
    ScopedSlot s(L, kSlotTopkAms, stream);
    hipLaunchKernelGGL(k_topk_amsgrad, dim3(geo.num_chunks), wg, 0, stream, theta, m, v, vhat, geo, ws, ap);
  }
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

}  // namespace compams
