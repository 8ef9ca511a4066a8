// Top-k with error feedback (Definition 1 inside the worker lines of Algorithm 2) and the server
// lines for sparse messages, for gfx950.
//
// Per worker row:  x = e + g is stored in place of e, the k coordinates of largest magnitude key
// (fp32 pattern without the sign; ties to the lower coordinate) are written out as ascending
// (coordinate, value) lists, and the residual at those coordinates becomes zero.
//
// Kernels of a step.  In the steady state three of them do the work (first pass, band, final); the four
// general ones in between return at once for every row whose threshold the band kernel has found:
//   first pass     x = e + g -> e as a grid of short workgroups, one chunk each.  When the previous step's
//                  threshold bucket is carried over as a guess, the same pass writes the candidate list: the
//                  entries at or above the guessed bucket, a segment per chunk.  When the last two thresholds
//                  also give a band of keys in which this step's threshold is expected, the candidates are the
//                  entries from the band's first key upwards (it lies at or above the guessed bucket), and the
//                  pass counts per chunk the entries above the band, lists the entries inside it (a segment per
//                  chunk again) and adds them to the row's histogram of 2048 buckets across the band.
//   band           if the threshold key does lie in the band (decided exactly from the counts): per chunk the
//                  entries kept for certain, their prefixes inside blocks of chunks and the block totals; the
//                  few entries of the threshold's bucket are ranked by the last workgroup of the row, which
//                  gives tau, the ties to keep (by coordinate) and the next step's guess and band.
//   The general route (12 + 10 + 9 key bits and a zero sign bit), for every other row:
//   level 0        histogram of the 12-bit threshold buckets, from the candidate list when the guess held (the
//                  list then holds at least k entries), else from the row itself; for a listed row also the
//                  level-1 histograms of the three buckets from the guess upwards, among which the threshold
//                  is expected.  The last workgroup of a row to finish finds the threshold bucket, checks the
//                  guess, resolves level 1 if it can, and sets the next step's guess.
//   level 1        only for rows that level 0 could not resolve: one more read of the row that writes the
//                  candidate list with the exact bucket and builds the level-1 histogram (10 bits), or a
//                  sweep of the list; rows that would not fit a list are histogrammed from the row itself.
//   level 2        histogram of the last 9 key bits over the matching candidates; yields the k-th largest
//                  key tau and how many keys equal to tau are taken; sets the next step's band.
//   count          per chunk: keys above tau and keys equal to tau, with prefixes inside contiguous blocks of
//                  chunks and the totals of every block.
//   final          per chunk of coordinates: the position of each worker's entries in its list follows from
//                  the block totals and prefixes; the selected entries are written there, then added in
//                  worker order into an LDS tile of the averaged gradient, then AMSGrad.
// With top-k inside every block (one selection problem per worker and block) the same launches go over all
// problems at once through tables of workgroup slots; problems of at most 1024 coordinates are solved by one
// wavefront inside the first pass.
// Zeroing the residual at the selected coordinates is not done by scattered stores: the next step's
// first pass treats the coordinates in the previous lists as zero while it forms x (and a small kernel
// applies the zeros when the caller asks for e).
//
// All routes give the same result; the guess only decides how many bytes move.  A candidate list is a
// set of per-chunk segments, each in ascending coordinate order, placed by integer atomic cursors (a row's
// list is kept as eight runs with a cursor each, chunk c appending to run c % 8): their physical order
// varies from run to run but nothing that is output depends on it.  No floating-point atomics are used
// anywhere.

#include "compams_device.h"
#include "compams_internal.h"

namespace compams {
namespace {

struct Quad {
  uint32_t key[4];
  bool ok[4];
};

template <bool FULL>
__device__ __forceinline__ void hist4(uint32_t* lh, const Quad& q, uint32_t& zeros) {
  if (FULL) {
    // common case: no zero key in the whole round -> four unconditional LDS adds
    const uint32_t kmin = min(min(q.key[0], q.key[1]), min(q.key[2], q.key[3]));
    if (ballot64(kmin == 0) == 0) {
#pragma unroll
      for (int s = 0; s < 4; ++s) atomicAdd(&lh[q.key[s] >> kL0Shift], 1u);
      return;
    }
  }
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

__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
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

// Allocating a chunk's segment of the candidate list takes an atomic with return.  It is split in two so
// that a caller can put other work between the request and the first use of its result.
__device__ __forceinline__ uint32_t segment_request(TopkRow* rowp, uint32_t cnt) {
  uint32_t raw = 0;
  if (cnt && lane_id() == 0) raw = atomicAdd(&rowp->cursor, cnt);
  return raw;  // meaningful in lane 0 only; nobody has looked at it yet
}

// Write the chunk's segment: from the staging area if everything fitted there, else by reading the chunk's
// (already stored) corrected gradients again.
__device__ __forceinline__ void segment_write(uint32_t raw, const uint2* stage, uint32_t cnt,
                                              const float* __restrict__ er, uint32_t d, uint32_t c,
                                              uint32_t thr_bucket, uint2* candr, uint32_t cap, uint2* descr) {
  const uint32_t lane = lane_id();
  uint32_t off = 0;
  if (cnt) {
    off = first_lane(raw);
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

__device__ __forceinline__ void flush_chunk(const uint2* stage, uint32_t cnt, const float* __restrict__ er, uint32_t d,
                                            uint32_t c, uint32_t thr_bucket, TopkRow* rowp, uint2* candr,
                                            uint32_t cap, uint2* descr) {
  const uint32_t raw = segment_request(rowp, cnt);
  segment_write(raw, stage, cnt, er, d, c, thr_bucket, candr, cap, descr);
}

// ---------------------------------------------------------------------------------------------
// "Last workgroup of the row": every workgroup of a row takes a ticket when it has finished; the one
// that draws the last ticket continues with the row-wide step.  No workgroup ever waits for another.
//
// Everything the last workgroup reads from the others travels through device-scope atomics (adds,
// stores) and is read back with device-scope atomic loads: those are performed at the level of the
// memory hierarchy that all compute units share, so no cache write-back or invalidation is needed
// (a full device-scope fence would write back and invalidate the whole L2 of the die at every call).
// Ordering: each wavefront waits until its own atomics have been acknowledged, the workgroup barrier
// collects all wavefronts, and only then is the ticket drawn.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ bool last_group_of_row(uint32_t* ticket, uint32_t groups, uint32_t* sh_flag) {
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");  // this wavefront's atomics have been performed
  __syncthreads();
  if (threadIdx.x == 0) {
    const uint32_t t = __hip_atomic_fetch_add(ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    const bool last = (t + 1 == groups);
    if (last) __hip_atomic_store(ticket, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // ready for the next launch
    *sh_flag = last ? 1u : 0u;
  }
  __syncthreads();
  return *sh_flag != 0;
}

__device__ __forceinline__ uint32_t load_agent(const uint32_t* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Many device-scope loads in flight at once.  The compiler waits for each atomic load before it issues the
// next, which turns a row-wide step of a few thousand words into a chain of memory round trips; buffer loads
// with the same cache policy (served by the level all compute units share) are ordinary loads to it and
// overlap.  A view covers `words` 32-bit words from p; reads beyond it return 0.
struct AgentView {
  __amdgpu_buffer_rsrc_t rsrc;
};
__device__ __forceinline__ AgentView agent_view(const uint32_t* p, uint32_t words) {
  AgentView v;
  v.rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<uint32_t*>(p), 0, words * 4u, 0x00020000);
  return v;
}
__device__ __forceinline__ uint32_t load_agent(const AgentView& v, uint32_t word) {
  return __builtin_amdgcn_raw_buffer_load_b32(v.rsrc, word * 4u, 0, /*device-scope policy*/ 16);
}

// ---------------------------------------------------------------------------------------------
// Finding the bucket in which a suffix count crosses `need`, by one workgroup of kWG threads.
// h: NB bucket counts in LDS.  Returns through out2 the largest s with sum_{b >= s} h[b] >= need and the
// count strictly above it.  Requires 1 <= need <= sum h.
// ---------------------------------------------------------------------------------------------
template <int NB, int NT = kWG>
__device__ void find_crossing(const uint32_t* h, uint32_t need, uint32_t* suf /* NT + 1 */, uint32_t* out2) {
  constexpr int PER = NB / NT;
  static_assert(NB % NT == 0 && NT % 64 == 0, "buckets per thread, whole wavefronts");
  const int t = threadIdx.x;
  const uint32_t lane = lane_id(), wave = t >> 6;
  uint32_t part = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) part += h[t * PER + i];
  // inclusive suffix sum over the threads: inside the wavefront by shuffles, across wavefronts through LDS
  uint32_t s = part;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const uint32_t up = __shfl_down(s, o, 64);
    if (lane + o < 64) s += up;
  }
  __syncthreads();  // everybody has read h and whatever suf / out2 held before
  if (lane == 0) suf[wave] = s;  // the wavefront's total
  if (t == 0) { out2[0] = 0; out2[1] = 0; }
  __syncthreads();
  uint32_t higher = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w)
    if (static_cast<uint32_t>(w) > wave) higher += suf[w];
  s += higher;                       // entries in this thread's buckets and all buckets above them
  const uint32_t above_mine = s - part;  // entries in the buckets above this thread's
  if (s >= need && above_mine < need) {  // exactly one thread when 1 <= need <= sum h
    uint32_t acc = above_mine;
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

// Copy a row's global histogram into LDS and clear it for the next step.
template <int NB, int NT = kWG>
__device__ __forceinline__ void take_hist(uint32_t* gh, uint32_t* h) {
  static_assert(NB % NT == 0, "buckets per thread");
  constexpr int PER = NB / NT;
  const AgentView view = agent_view(gh, NB);
  uint32_t x[PER];
#pragma unroll
  for (int i = 0; i < PER; ++i) x[i] = load_agent(view, i * NT + threadIdx.x);
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    h[i * NT + threadIdx.x] = x[i];
    gh[i * NT + threadIdx.x] = 0;
  }
  __syncthreads();
}

// bstar and need are passed in (not re-read from the control block): the caller may have written them a
// moment ago, and a line of the control block read earlier by this compute unit may still sit in its L1.
template <int NT = kWG>
__device__ __forceinline__ void resolve_level1(TopkRow* rp, uint32_t bstar, uint32_t need, const uint32_t* h,
                                               uint32_t* suf, uint32_t* out2) {
  find_crossing<kNB1, NT>(h, need, suf, out2);
  if (threadIdx.x == 0) {
    rp->prefix1 = (bstar << (kL0Shift - kL1Shift)) | out2[0];
    rp->need = need - out2[1];
    rp->level1_done = 1;
  }
}

__device__ __forceinline__ void emit_chunk(uint32_t mode, const float* __restrict__ er, uint32_t d, uint32_t c,
                                           const uint2* __restrict__ candr, uint2 ds,
                                           uint32_t cap, uint32_t tau, uint32_t r, bool all_ties, uint32_t eq_seen,
                                           uint32_t at, int32_t* __restrict__ idx, float* __restrict__ val, uint32_t k,
                                           uint32_t coord_base, bool by_coord = false, uint32_t tie_last = 0);

// A micro problem (top-k inside a block of at most kMicroCoords coordinates) from end to end by one wavefront:
// x = e + g with the pending zeros honoured, stored in place of e; the k-th largest key by a bit-by-bit search
// over the keys, which stay in registers (31 steps of ballots: the largest t with at least k keys >= t); the
// selected entries in coordinate order into the problem's part of the worker's list (ties as everywhere: in
// coordinate order until r are in); and the records the last kernel reads (it finds the list written).
// bm: 32 words of LDS of this wavefront (PEND only).  No barrier: other wavefronts of the workgroup do other
// problems.
constexpr int kMicroRounds = static_cast<int>(kMicroCoords / 256);

template <bool PEND>
__device__ __forceinline__ void micro_problem(const float* __restrict__ g, float* __restrict__ e, const Seg& sg,
                                              uint32_t seg, const TopkWorkspace& ws, uint32_t* bm) {
  const uint32_t lane = lane_id();
  const float* gr = g + sg.elem_off;
  float* er = e + sg.elem_off;
  const uint32_t d = sg.d, k = sg.k;
  int32_t* idx = ws.idx + sg.list_base;
  float* val = ws.val + sg.list_base;
  if constexpr (PEND) {
    if (lane < kMicroCoords / 32) bm[lane] = 0;
    const uint32_t* so = ws.sel_off + sg.seloff_base;
    const uint32_t lo = so[0];
    const uint32_t hi = so[1] < k ? so[1] : k;
    for (uint32_t q = lo + lane; q < hi; q += 64) {
      const uint32_t jl = static_cast<uint32_t>(idx[q]) - sg.coord_base;
      if (jl < kMicroCoords) atomicOr(&bm[jl >> 5], 1u << (jl & 31u));
    }
  }
  uint32_t key[kMicroRounds * 4];
  uint32_t okm = 0;  // bit 4r + s: this lane's slot s of round r is a coordinate of the problem
#pragma unroll
  for (int r = 0; r < kMicroRounds; ++r) {
    const uint32_t j = r * 256 + lane * 4;
#pragma unroll
    for (int s = 0; s < 4; ++s) key[4 * r + s] = 0;
    if (j < d) {
      const float4 gv = *reinterpret_cast<const float4*>(gr + j);
      const float4 e_in = *reinterpret_cast<const float4*>(er + j);
      float4 ev = e_in;
      if constexpr (PEND) {
        const uint32_t nib = (bm[r * 8 + (lane >> 3)] >> ((lane & 7u) * 4u)) & 15u;
        if (nib & 1u) ev.x = 0.0f;
        if (nib & 2u) ev.y = 0.0f;
        if (nib & 4u) ev.z = 0.0f;
        if (nib & 8u) ev.w = 0.0f;
      }
      float4 x = make_float4(ev.x + gv.x, ev.y + gv.y, ev.z + gv.z, ev.w + gv.w);
      const bool ok1 = j + 1 < d, ok2 = j + 2 < d, ok3 = j + 3 < d;
      if (!ok1) x.y = e_in.y;  // columns >= d keep what they held
      if (!ok2) x.z = e_in.z;
      if (!ok3) x.w = e_in.w;
      *reinterpret_cast<float4*>(er + j) = x;
      key[4 * r + 0] = key_of_bits(__float_as_uint(x.x));
      key[4 * r + 1] = ok1 ? key_of_bits(__float_as_uint(x.y)) : 0u;
      key[4 * r + 2] = ok2 ? key_of_bits(__float_as_uint(x.z)) : 0u;
      key[4 * r + 3] = ok3 ? key_of_bits(__float_as_uint(x.w)) : 0u;
      okm |= (1u | (ok1 ? 2u : 0u) | (ok2 ? 4u : 0u) | (ok3 ? 8u : 0u)) << (4 * r);
    }
  }
  const int rounds = static_cast<int>((d + 255) / 256);  // wave-uniform; keys of later rounds are 0 and not looked at
  uint32_t tau = 0;
  for (int bit = 30; bit >= 0; --bit) {
    const uint32_t t = tau | (1u << bit);  // t >= 1: a slot outside the problem (key 0) never counts
    uint32_t cnt = 0;
#pragma unroll
    for (int r = 0; r < kMicroRounds; ++r)
      if (r < rounds) {
#pragma unroll
        for (int s = 0; s < 4; ++s) cnt += popc64(ballot64(key[4 * r + s] >= t));
      }
    if (cnt >= k) tau = t;
  }
  uint32_t gt = 0, ties = 0;
#pragma unroll
  for (int r = 0; r < kMicroRounds; ++r)
    if (r < rounds) {
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const bool ok = (okm >> (4 * r + s)) & 1u;
        gt += popc64(ballot64(ok && key[4 * r + s] > tau));
        ties += popc64(ballot64(ok && key[4 * r + s] == tau));
      }
    }
  const uint32_t r_take = k - gt;  // 1 <= r_take <= ties
  if (lane == 0) {
    TopkRow* rowp = ws.rows + seg;
    rowp->mode = kModeDense;
    rowp->n_src = 0;
    rowp->cursor = 0;
    rowp->cursor_band = 0;
    rowp->pred_valid = 0;
    rowp->band_valid = 0;
    rowp->fast = 0;
    rowp->b_guess = 0;
    rowp->level1_done = 1;
    rowp->tau = tau;
    rowp->r = r_take;
    rowp->ties = ties;
    ws.tau[seg] = tau;
    ws.count_gt[seg] = gt;
    uint32_t* cn = ws.counters + seg * kCountersPerRow;
    cn[0] = 0;
    cn[1] = 0;
    cn[2] = ties;
    cn[3] = r_take;
    cn[4] = 0;
    cn[5] = 1;
    ws.chunk_rec[sg.chunk_base] = make_uint4(gt, ties, 0u, 0u);  // one chunk, nothing before it
    ws.blk[static_cast<size_t>(seg) * kMaxCountBlocks] = make_uint2(gt, ties);
  }
  // the values come back from where this wavefront has just stored them
  emit_chunk(kModeDense, er, d, 0u, nullptr, make_uint2(0u, 0u), 0u, tau, r_take, r_take == ties, 0u, 0u, idx, val, k,
             sg.coord_base);
}

// ---------------------------------------------------------------------------------------------
// Which selection problem a workgroup works on.  UNI: one problem per worker row, all of one shape, grid
// (groups, rows): everything follows from the block indices.  Otherwise the launch is flat and tables say
// which segment (a block of a worker's row) and which of its workgroups this is; geo and opt are then
// narrowed to the segment's own shape.
// ---------------------------------------------------------------------------------------------
enum : int { kClassFirst = 0, kClassSweep = 1, kClassCount = 2, kClassLevel0 = 3 };

struct SegCtx {
  uint32_t seg;     // index into the per-problem tables (control blocks, histograms, thresholds)
  uint32_t group;   // this workgroup's index among the `groups` that share the problem
  uint32_t groups;
  int64_t elem_off;
  uint32_t coord_base;
  size_t chunk_base, seloff_base, cand_base, list_base, band_base;
  uint32_t cursor_set;  // see Seg
};

// The context of workgroup `group` of segment `seg` in a flat launch.
__device__ __forceinline__ SegCtx seg_ctx_of(uint32_t seg, uint32_t group, uint32_t groups, const Seg& sg, Geometry& geo,
                                             TopkOptions& opt) {
  SegCtx c;
  c.seg = seg;
  c.group = group;
  c.groups = groups;
  c.elem_off = sg.elem_off;
  c.coord_base = sg.coord_base;
  c.chunk_base = sg.chunk_base;
  c.seloff_base = sg.seloff_base;
  c.cand_base = sg.cand_base;
  c.list_base = sg.list_base;
  c.band_base = sg.band_base;
  c.cursor_set = sg.cursor_set;
  geo.d = sg.d;
  geo.k = sg.k;
  geo.num_chunks = sg.num_chunks;
  geo.count_cpw = sg.count_cpw;
  opt.cap = opt.cap < sg.cap ? opt.cap : sg.cap;
  opt.band_cap = opt.band_cap < sg.band_cap ? opt.band_cap : sg.band_cap;
  return c;
}

template <bool UNI, int CLASS>
__device__ __forceinline__ SegCtx seg_ctx(Geometry& geo, TopkOptions& opt, const TopkWorkspace& ws) {
  if (UNI) {
    SegCtx c;
    c.seg = blockIdx.y;
    c.group = blockIdx.x;
    c.groups = gridDim.x;
    c.elem_off = static_cast<int64_t>(c.seg) * geo.ld;
    c.coord_base = 0;
    c.chunk_base = static_cast<size_t>(c.seg) * geo.num_chunks;
    c.seloff_base = static_cast<size_t>(c.seg) * (geo.num_chunks + 1);
    c.cand_base = static_cast<size_t>(c.seg) * opt.cap;
    c.list_base = static_cast<size_t>(c.seg) * geo.k;
    c.band_base = static_cast<size_t>(c.seg) * opt.band_cap;
    c.cursor_set = geo.num_chunks >= kSubListMinChunks ? c.seg : kNoCursorSet;  // short rows keep one run
    return c;
  }
  // (the records come through the vector path: through the scalar one the first pass was 1-2 % slower)
  const WgSlot slot = (CLASS == kClassFirst ? ws.map_first
                       : CLASS == kClassLevel0 ? ws.map_level0
                       : CLASS == kClassSweep ? ws.map_sweep : ws.map_count)[blockIdx.x];
  const Seg sg = ws.segs[slot.seg];
  return seg_ctx_of(slot.seg, slot.group,
                    CLASS == kClassFirst ? sg.groups_first
                    : CLASS == kClassLevel0 ? sg.groups_level0
                    : CLASS == kClassSweep ? sg.groups_sweep : sg.count_blocks,
                    sg, geo, opt);
}

// The runs of a problem's candidate list (one, or kSubLists for a row of the one-selection-per-row form).
struct ListRuns {
  uint32_t lists, pitch;  // run s starts at entry s * pitch
  uint32_t n[kSubLists];
  uint32_t total;
  bool fits;              // no run has outgrown its share of the capacity
};

// As the first pass left them: from the cursors.
__device__ __forceinline__ ListRuns runs_from_cursors(const TopkWorkspace& ws, const TopkRow* rowp, uint32_t cursor_set,
                                                      uint32_t cap) {
  ListRuns L;
  L.total = 0;
  L.fits = true;
  if (cursor_set != kNoCursorSet) {  // uniform
    L.lists = kSubLists;
    L.pitch = cap / kSubLists;
    const uint32_t* cur = ws.xcur + static_cast<size_t>(cursor_set) * kSubLists * kCursorPitch;
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s) {
      L.n[s] = cur[s * kCursorPitch];
      L.total += L.n[s];
      L.fits = L.fits && L.n[s] <= L.pitch;
    }
  } else {
    L.lists = 1;
    L.pitch = 0;
    L.n[0] = rowp->cursor;
#pragma unroll
    for (uint32_t s = 1; s < kSubLists; ++s) L.n[s] = 0;
    L.total = L.n[0];
    L.fits = L.n[0] <= cap;
  }
  return L;
}

// As level 0 recorded them for the later sweeps.
__device__ __forceinline__ ListRuns runs_of_row(const TopkRow* rowp, uint32_t cap) {
  ListRuns L;
  L.lists = rowp->n_lists;
  L.pitch = cap / kSubLists;
  L.total = 0;
  L.fits = true;
#pragma unroll
  for (uint32_t s = 0; s < kSubLists; ++s) {
    L.n[s] = s < L.lists ? rowp->n_sub[s] : 0u;
    L.total += L.n[s];
  }
  return L;
}

// A sweep over a problem's candidate list by `threads` threads, of which the caller is number `first`: visit(bits)
// for the entries first, first + threads, ... of every run.  The loads of a trip are requested together -- four
// entries of a list kept as one run, one entry of each of the kSubLists runs otherwise -- because a thread's trips
// are a chain of round trips (run after run, the sweep of level 2 took 10.4 us instead of 7).
template <typename F>
__device__ __forceinline__ void sweep_list(const uint2* __restrict__ candr, const ListRuns& R, uint32_t first,
                                           uint32_t threads, F&& visit) {
  if (R.lists == 1) {  // uniform
    const uint32_t len = R.n[0];
    for (uint32_t q = first; q < len; q += 4 * threads) {
      uint32_t bits[4];
      bool ok[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        ok[w] = q + w * threads < len;
        bits[w] = ok[w] ? candr[q + w * threads].y : 0u;
      }
#pragma unroll
      for (int w = 0; w < 4; ++w)
        if (ok[w]) visit(bits[w]);
    }
    return;
  }
  uint32_t longest = 0;
#pragma unroll
  for (uint32_t s = 0; s < kSubLists; ++s) longest = R.n[s] > longest ? R.n[s] : longest;
  for (uint32_t q = first; q < longest; q += threads) {
    uint32_t bits[kSubLists];
    bool ok[kSubLists];
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s) {
      ok[s] = q < R.n[s];
      bits[s] = ok[s] ? candr[static_cast<size_t>(s) * R.pitch + q].y : 0u;
    }
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s)
      if (ok[s]) visit(bits[s]);
  }
}

// ---------------------------------------------------------------------------------------------
// One selection per row, first pass without histograms.  A workgroup takes ONE chunk and ends; wavefront w takes
// rounds 4w .. 4w+3 of it.  Measured on MI355X with plain streaming kernels of the same traffic (read g, read e,
// write e, 2.1 GB): a grid of such short workgroups, handed out in order, streams at 6.1-6.4 TB/s, while
// workgroups that each walk many chunks stay at 5.4-5.7 TB/s whatever their number, occupancy or prefetch depth.
// A short-lived workgroup cannot afford a 4096-bin histogram in LDS (to clear and to flush), so this pass has
// none: x = e + g (pending zeros honoured) is stored, and when the row carries a guess for the threshold bucket
// the entries at or above it are staged per wavefront in coordinate order, the chunk's segment of the candidate
// list is allocated with one atomic for the whole workgroup, and the four quarters are written behind one
// another.  The level-0 histogram is taken afterwards, from the candidate list (k_topk_level0).
// ---------------------------------------------------------------------------------------------
constexpr int kLeanRounds = kRounds / kWaves;  // rounds of a chunk per wavefront
constexpr int kStageQ = 512;                   // staged candidates per wavefront (of at most 1024 coordinates)

// UNI: grid (chunks, rows).  Otherwise (top-k inside every block) the launch is flat over map_first: a workgroup
// per chunk of every segment in address order, and at the end the workgroups whose wavefronts take one micro
// problem each; coordinates below are the segment's own, the lists hold coordinates of the worker's row.
template <bool PEND, bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_lean(const float* __restrict__ g, float* __restrict__ e, Geometry geo,
                                                    TopkWorkspace ws, TopkOptions opt, uint32_t use_guess) {
  __shared__ uint2 stage_all[kWaves * kStageQ];
  __shared__ uint32_t bm_all[PEND ? kWaves * 32 : 1];
  __shared__ uint32_t sh_cnt[kWaves], sh_above[kWaves], sh_from[kWaves], sh_off, sh_boff;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  if constexpr (!UNI) {
    const WgSlot slot = ws.map_first[blockIdx.x];
    if (slot.seg & kMicroFlag) {  // workgroup-uniform: up to four micro problems, one per wavefront
      if (wave < slot.group) {
        const uint32_t seg = ws.micro_list[(slot.seg & ~kMicroFlag) + wave];
        const Seg sg = ws.segs[seg];
        micro_problem<PEND>(g, e, sg, seg, ws, bm_all + (PEND ? wave * 32 : 0));
      }
      return;
    }
  }
  const SegCtx sc = seg_ctx<UNI, kClassFirst>(geo, opt, ws);
  const uint32_t c = sc.group, row = sc.seg;
  const float* gr = g + sc.elem_off;
  float* er = e + sc.elem_off;
  TopkRow* rowp = ws.rows + row;
  const uint32_t d = geo.d;
  const uint32_t q0 = c * kChunk + wave * (kLeanRounds * 256);  // first coordinate of this wavefront's quarter
  const bool full = (c + 1) * static_cast<uint64_t>(kChunk) <= d;
  // The chunk's loads go out before anything else is asked for: nothing below decides their addresses.
  float4 gv[kLeanRounds], ev[kLeanRounds];
#pragma unroll
  for (int u = 0; u < kLeanRounds; ++u) {
    const uint32_t j = q0 + u * 256 + lane * 4;
    gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
    ev[u] = gv[u];
    if (full || j < d) {
      gv[u] = load_stream4(gr + j);
      ev[u] = load_stream4(er + j);
    }
  }
  // What this pass reads of the row's control block and of the previous step's list offsets was written by earlier
  // launches and is the same for the whole workgroup: it comes through the scalar path, whose answers do not
  // queue behind the chunk's loads (vector loads return in order) - the first eight words of the control block
  // with one load, the list offsets with it, and only then is any of it looked at (one round trip, not one per
  // condition).
  static_assert(offsetof(TopkRow, pred_valid) == 0 && offsetof(TopkRow, b_guess) == 4 &&
                offsetof(TopkRow, band_valid) == 16 && offsetof(TopkRow, band_lo) == 20 &&
                offsetof(TopkRow, band_hi) == 24 && offsetof(TopkRow, band_mul) == 28 &&
                offsetof(TopkRow, cursor) == 8 && offsetof(TopkRow, cursor_band) == 12,
                "words read below; the two cursors form one 64-bit word");
  const U32x8 rw = table_u32x8(reinterpret_cast<const uint32_t*>(rowp));
  uint32_t prev_lo = 0, prev_hi = 0;
  if constexpr (PEND) {
    const uint32_t* prev_off = ws.sel_off + sc.seloff_base;
    prev_lo = table_u32(prev_off, c);
    prev_hi = table_u32(prev_off, c + 1);
  }
  const bool pred = use_guess && rw[0] != 0;  // workgroup-uniform
  const uint32_t bg = rw[1];
  // the band [blo, bhi) of keys: empty (no key is >= 0xffffffff) unless the row carries one
  const bool banded = pred && opt.band && rw[4] != 0;
  const uint32_t blo = banded ? rw[5] : 0xffffffffu;
  const uint32_t bhi = banded ? rw[6] : 0xffffffffu;
  const uint32_t bmul = banded ? rw[7] : 0u;
  // Candidates: every key at or above cand_lo - the guessed bucket's first key, or, with a band (which starts at or
  // above that), the band's first key: the threshold is expected inside the band, so that nothing below it is needed
  // (a list of at least k entries that holds every key from some key upwards holds the k largest, wherever that
  // key lies inside a bucket; a shorter one sends the row to the kernels that read it again).
  const uint32_t cand_lo = banded ? blo : bg << kL0Shift;
  uint32_t* bh = ws.bhist + static_cast<size_t>(row) * kBandBuckets;
  uint32_t* bm = bm_all + (PEND ? wave * 32 : 0);
  if constexpr (PEND) {
    // the quarter's coordinates that were selected in the previous step: their residual counts as zero
    if (lane < 32) bm[lane] = 0;
    const int32_t* prev_idx = ws.idx + sc.list_base;
    const uint32_t lo = prev_lo;
    const uint32_t hi = prev_hi < geo.k ? prev_hi : geo.k;
    // 256 entries of the chunk's slice per trip, requested together (a chunk that holds entries at all holds
    // 80 to 150 of a worker's: one round trip instead of two or three in a row)
    for (uint32_t q = lo + lane; q < hi; q += 256) {
      uint32_t jv[4];
#pragma unroll
      for (int w = 0; w < 4; ++w) jv[w] = q + 64 * w < hi ? static_cast<uint32_t>(prev_idx[q + 64 * w]) : 0xffffffffu;
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const uint32_t jl = jv[w] - sc.coord_base - q0;
        if (q + 64 * w < hi && jl < static_cast<uint32_t>(kLeanRounds * 256)) atomicOr(&bm[jl >> 5], 1u << (jl & 31u));
      }
    }
  }
  uint2* stage = stage_all + wave * kStageQ;
  uint32_t cnt = 0;
  uint32_t n_above = 0, n_from = 0;  // this lane's entries at or above the band's upper end / its lower end
#pragma unroll
  for (int u = 0; u < kLeanRounds; ++u) {
    const uint32_t j = q0 + u * 256 + lane * 4;
    const bool ok[4] = {full || j < d, full || j + 1 < d, full || j + 2 < d, full || j + 3 < d};
    float4 en = ev[u];
    if constexpr (PEND) {
      const uint32_t nib = (bm[u * 8 + (lane >> 3)] >> ((lane & 7u) * 4u)) & 15u;
      if (nib & 1u) en.x = 0.0f;
      if (nib & 2u) en.y = 0.0f;
      if (nib & 4u) en.z = 0.0f;
      if (nib & 8u) en.w = 0.0f;
    }
    float4 x = make_float4(en.x + gv[u].x, en.y + gv[u].y, en.z + gv[u].z, en.w + gv[u].w);
    if (!full) {  // columns >= d keep what they held
      if (!ok[1]) x.y = ev[u].y;
      if (!ok[2]) x.z = ev[u].z;
      if (!ok[3]) x.w = ev[u].w;
    }
    if (ok[0]) store_stream4(er + j, x);
    if (pred) {
      const uint32_t bits[4] = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z), __float_as_uint(x.w)};
      bool flag[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint32_t key = key_of_bits(bits[s]);
        flag[s] = ok[s] && key >= cand_lo;
        n_above += (ok[s] && key >= bhi) ? 1u : 0u;
        n_from += (ok[s] && key >= blo) ? 1u : 0u;
      }
      const RoundRank rr = rank_round(flag);
      if (rr.total) {
        uint32_t pos = cnt + rr.below;
#pragma unroll
        for (int s = 0; s < 4; ++s)
          if (flag[s]) {
            if (pos < static_cast<uint32_t>(kStageQ)) stage[pos] = make_uint2(j + s, bits[s]);
            ++pos;
          }
        cnt += rr.total;
      }
    }
  }
  if (!pred) return;  // workgroup-uniform
  // the chunk's segments of the candidate list and of the band list: one allocation for the four quarters
  const uint32_t above_w = banded ? wave_sum(n_above) : 0u;
  const uint32_t band_w = banded ? wave_sum(n_from) - above_w : 0u;  // this quarter's entries inside the band
  if (lane == 0) { sh_cnt[wave] = cnt; sh_above[wave] = above_w; sh_from[wave] = band_w; }
  __syncthreads();
  uint32_t before = 0, total = 0, bbefore = 0, btotal = 0, atotal = 0;
#pragma unroll
  for (int w = 0; w < kWaves; ++w) {
    const uint32_t t = sh_cnt[w], tb = sh_from[w];
    before += static_cast<uint32_t>(w) < wave ? t : 0u;
    bbefore += static_cast<uint32_t>(w) < wave ? tb : 0u;
    total += t;
    btotal += tb;
    atotal += sh_above[w];
  }
  // the run this chunk appends to, its share of the capacities and its cursors (candidates in the low half of a
  // 64-bit word, band entries in the high half: one atomic advances both)
  const bool runs = sc.cursor_set != kNoCursorSet;  // workgroup-uniform
  const uint32_t run = runs ? c % kSubLists : 0u;
  const uint32_t run_cap = runs ? opt.cap / kSubLists : opt.cap;
  const uint32_t run_base = run * run_cap;
  const uint32_t brun_cap = runs ? opt.band_cap / kSubLists : opt.band_cap;
  const uint32_t brun_base = run * brun_cap;
  if (threadIdx.x == 0) {
    uint32_t* cur =
        runs ? ws.xcur + (static_cast<size_t>(sc.cursor_set) * kSubLists + run) * kCursorPitch : &rowp->cursor;
    const unsigned long long add = static_cast<unsigned long long>(total) | (static_cast<unsigned long long>(btotal) << 32);
    const unsigned long long old = add ? atomicAdd(reinterpret_cast<unsigned long long*>(cur), add) : 0ull;
    const uint32_t off = static_cast<uint32_t>(old), boff = static_cast<uint32_t>(old >> 32);
    sh_off = off;
    sh_boff = boff;
    ws.desc[sc.chunk_base + c] = make_uint2(run_base + off, total);
    ws.desc2[sc.chunk_base + c] = make_uint2(brun_base + boff, atotal | (btotal << 13));
    if (atotal) atomicAdd(runs ? cur + kCursorAboveWord : &rowp->above, atotal);  // nobody waits for it
  }
  __syncthreads();
  const uint32_t off = sh_off, boff = sh_boff;
  if (off + total > run_cap) return;  // the list has overflowed and will not be used (nor will the band)
  const bool band_fits = boff + btotal <= brun_cap;  // else the band has overflowed and will not be used
  uint2* dst = ws.cand + sc.cand_base + run_base + off + before;
  uint2* bdst = ws.band + sc.band_base + brun_base + boff + bbefore;
  uint32_t bat = 0;  // band entries of this quarter written so far
  if (cnt <= static_cast<uint32_t>(kStageQ)) {
    for (uint32_t q0s = 0; q0s < cnt; q0s += 64) {
      const uint32_t q = q0s + lane;
      uint2 en = make_uint2(0u, 0u);
      if (q < cnt) {
        en = stage[q];
        dst[q] = en;
      }
      if (band_w && band_fits) {  // wave-uniform
        const uint32_t key = key_of_bits(en.y);
        const bool inb = q < cnt && key >= blo && key < bhi;
        const uint64_t bb = ballot64(inb);
        if (inb) {
          bdst[bat + count_below(bb)] = en;
          atomicAdd(&bh[band_bucket(key - blo, bmul)], 1u);  // the row's bucket histogram; nobody waits for it
        }
        bat += popc64(bb);
      }
    }
  } else {
    // more candidates than the staging area holds: the quarter's (already stored) values are read again
    uint32_t at = 0;
    for (int u = 0; u < kLeanRounds; ++u) {
      const uint32_t j = q0 + u * 256 + lane * 4;
      float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
      if (j < d) x = *reinterpret_cast<const float4*>(er + j);
      const uint32_t bits[4] = {__float_as_uint(x.x), __float_as_uint(x.y), __float_as_uint(x.z), __float_as_uint(x.w)};
      bool flag[4], inb[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint32_t key = key_of_bits(bits[s]);
        flag[s] = j + s < d && key >= cand_lo;
        inb[s] = j + s < d && key >= blo && key < bhi;
      }
      const RoundRank rr = rank_round(flag);
      uint32_t pos = at + rr.below;
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (flag[s]) {
          if (pos < cnt) dst[pos] = make_uint2(j + s, bits[s]);
          ++pos;
        }
      at += rr.total;
      if (band_w && band_fits) {  // wave-uniform
        const RoundRank br = rank_round(inb);
        uint32_t bpos = bat + br.below;
#pragma unroll
        for (int s = 0; s < 4; ++s)
          if (inb[s]) {
            if (bpos < band_w) {
              bdst[bpos] = make_uint2(j + s, bits[s]);
              atomicAdd(&bh[band_bucket(key_of_bits(bits[s]) - blo, bmul)], 1u);
            }
            ++bpos;
          }
        bat += br.total;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// The window of keys in which the next step's threshold is expected, from this step's threshold key `tau` and the
// one before (0: none).  The keys of positive floats order as the floats do, so the window is set in float
// arithmetic.  Training thresholds drift smoothly while the residuals build up (+34 %, +17 %, +10 %, +7.5 % ... over
// the first steps of the ResNet-18-shaped workload, +2 % at step ten): with d1 the last relative change and d0 the
// one before, a drift that is dying down (same sign, |d1| < |d0|) is taken to go on doing so, next = d1 * d1 / d0
// (not below d1 / 4), and to be off by at most half of what that took away from d1; any other pair of changes is
// extrapolated flat, next = d1, unsure by 0.4 |d1| + |d1 - d0|.  The centre is tau (1 + next), the half-width
// 0.4 % + unsure + `noise`, an allowance for the scatter of the k-th largest of a sample from step to step.  With B entries found in a window
// of relative width w around the threshold, one entry more or fewer above a level moves the k-th largest key by
// w / B of its value and the count above a level scatters by about sqrt(k): k_topk_band passes 8 w sqrt(k) / B
// (the extrapolation more than doubles the scatter, and three times the result is allowed for); where no window
// has been looked at yet, 1.5 / sqrt(k) stands in (as if a fourteenth of the kept entries lay within one per
// cent of the threshold).  It only decides which route the next step takes, never a result.  guess_valid / guess:
// the bucket guess the next first pass will use; the window must lie at or above it so that every band entry is
// also a candidate.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ float default_band_noise(uint32_t k) { return 1.5f / sqrtf(static_cast<float>(k)); }

__device__ __forceinline__ bool normal_key(uint32_t key) { return key >= 0x00800000u && key < 0x7f000000u; }

__device__ __forceinline__ void set_next_band(TopkRow* rowp, uint32_t tau, uint32_t tau_prev, uint32_t tau_prev2,
                                              uint32_t guess_valid, uint32_t guess, float noise,
                                              const TopkOptions& opt) {
  uint32_t valid = 0, lo = 0, hi = 0;
  if (guess_valid && opt.band && opt.band_cap && normal_key(tau)) {
    const float t1 = __uint_as_float(tau);
    float d1 = 0.0f;  // the last relative change of the threshold
    if (normal_key(tau_prev)) d1 = fminf(fmaxf(t1 / __uint_as_float(tau_prev), 0.5f), 2.0f) - 1.0f;
    float next = d1, unsure = 0.4f * fabsf(d1);  // the change expected next, and how far off that may be
    if (normal_key(tau_prev) && normal_key(tau_prev2)) {
      const float d0 = fminf(fmaxf(__uint_as_float(tau_prev) / __uint_as_float(tau_prev2), 0.5f), 2.0f) - 1.0f;
      if (d0 * d1 > 0.0f && fabsf(d1) < fabsf(d0)) {  // a drift that is dying down: let it go on doing so
        next = d1 * fmaxf(d1 / d0, 0.25f);
        unsure = 0.5f * fabsf(d1 - next);
      } else {
        unsure += fabsf(d1 - d0);
      }
    }
    const float delta = fminf(0.004f + unsure + fminf(fmaxf(noise, 0.0005f), 0.25f), 0.25f);
    const float centre = t1 * (1.0f + next);
    const float flo = centre * (1.0f - delta), fhi = centre * (1.0f + delta);
    lo = __float_as_uint(flo);
    hi = __float_as_uint(fhi);
    const uint32_t floor_key = guess << kL0Shift;
    if (lo < floor_key) lo = floor_key;
    valid = (hi < 0x7f800000u && hi > lo && lo >= 0x00800000u) ? 1u : 0u;
  }
  rowp->band_valid = valid;
  rowp->band_lo = lo;
  rowp->band_hi = hi;
  rowp->band_mul = valid ? band_multiplier_dev(hi - lo) : 0u;
}

// The runs of a problem's band list, from the high halves of the cursors the first pass advanced.
__device__ __forceinline__ ListRuns band_runs_from_cursors(const TopkWorkspace& ws, const TopkRow* rowp,
                                                           uint32_t cursor_set, uint32_t cap) {
  ListRuns L;
  L.total = 0;
  L.fits = true;
  if (cursor_set != kNoCursorSet) {  // uniform
    L.lists = kSubLists;
    L.pitch = cap / kSubLists;
    const uint32_t* cur = ws.xcur + static_cast<size_t>(cursor_set) * kSubLists * kCursorPitch;
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s) {
      L.n[s] = cur[s * kCursorPitch + 1];
      L.total += L.n[s];
      L.fits = L.fits && L.n[s] <= L.pitch;
    }
  } else {
    L.lists = 1;
    L.pitch = 0;
    L.n[0] = rowp->cursor_band;
#pragma unroll
    for (uint32_t s = 1; s < kSubLists; ++s) L.n[s] = 0;
    L.total = L.n[0];
    L.fits = L.n[0] <= cap;
  }
  return L;
}

// ---------------------------------------------------------------------------------------------
// The selection in one launch, for problems whose threshold key falls inside the band the first pass was given.
// Same geometry as the counting kernel: a workgroup owns a contiguous block of geo.count_cpw chunks.
//   1. Every workgroup of a problem reads the problem's bucket histogram of band entries (kBandBuckets counts,
//      added up by the first pass) and the count A of entries at or above the band, and finds by itself the
//      bucket that holds the k-th largest key: it exists iff A < k <= A + (entries in the band); both lists must
//      have fitted and the bucket must hold at most kBoundaryCap entries.  Otherwise the problem is left to the
//      general kernels that follow.  All workgroups of a problem read the same data and decide alike.
//   2. Per chunk: kept for certain = entries at or above the band + band entries in a bucket above the threshold's;
//      the workgroup leaves these counts with their prefixes inside the block, and the block's total, in the
//      tables the last kernel reads (the "equal to tau" columns stay 0).  Band entries in the threshold's bucket
//      are gathered in a small array of the problem.
//   3. The last workgroup of the problem to finish ranks the gathered entries by (key descending, coordinate
//      ascending): the first k - (entries above the bucket) of them are kept, the last of those holds tau;
//      an entry anywhere is kept iff key > tau, or key == tau and coordinate <= tie_last.  The coordinates of
//      the kept ones, ascending, let the last kernel add them to the positions of the chunks after them.
//      It also sets the guess and the band for the next step and clears the histogram.
// ---------------------------------------------------------------------------------------------
template <bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_band(Geometry geo, TopkWorkspace ws, TopkOptions opt, uint32_t use_guess) {
  __shared__ uint32_t lh[kBandBuckets];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  __shared__ uint32_t l_gt[kMaxCountCpw];
  __shared__ uint32_t scratch[kWG / 64 + 1];
  __shared__ uint32_t sh_flag;
  __shared__ uint2 b_en[kBoundaryCap];
  __shared__ uint32_t b_rank[kBoundaryCap];
  const SegCtx sc = seg_ctx<UNI, kClassCount>(geo, opt, ws);
  const uint32_t row = sc.seg, t = threadIdx.x;
  const uint32_t cpw = geo.count_cpw, nc = geo.num_chunks, k = geo.k;
  const uint32_t start = sc.group * cpw;
  if (start >= nc) return;  // uniform; the grid has exactly the blocks that exist
  const uint32_t end = start + cpw < nc ? start + cpw : nc;
  TopkRow* rowp = ws.rows + row;
  uint32_t* bh = ws.bhist + static_cast<size_t>(row) * kBandBuckets;
  const uint32_t wave = uniform_u32(t >> 6), lane = lane_id();
  constexpr int kGroup = 8;  // chunks a wavefront takes at a time: descriptors with one load, entries together
  // Everything that can be asked for before anything is known goes out together (a workgroup's work is a chain
  // of round trips otherwise): the control block and the cursors, the bucket histogram, the counts above the
  // band, the first descriptors.
  const uint2* d2 = ws.desc2 + sc.chunk_base;
  const uint32_t c_first = start + wave * kGroup;
  uint2 ds = make_uint2(0, 0);
  if (lane < kGroup && c_first + lane < end) ds = d2[c_first + lane];
  uint32_t x[kBandBuckets / kWG];
#pragma unroll
  for (uint32_t i = 0; i < kBandBuckets / kWG; ++i) x[i] = bh[i * kWG + t];
  uint32_t total_above = rowp->above;
  if (sc.cursor_set != kNoCursorSet) {
    total_above = 0;
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s)
      total_above += ws.xcur[(static_cast<size_t>(sc.cursor_set) * kSubLists + s) * kCursorPitch + kCursorAboveWord];
  }
  const uint32_t blo = rowp->band_lo, bhi = rowp->band_hi, bmul = rowp->band_mul, bg = rowp->b_guess;
  const uint32_t tau_before = rowp->tau, tau_before2 = rowp->tau_prev;  // the last two threshold keys (asked for
                                                                       // here: the last workgroup needs them)
  const ListRuns cand = runs_from_cursors(ws, rowp, sc.cursor_set, opt.cap);
  const ListRuns band = band_runs_from_cursors(ws, rowp, sc.cursor_set, opt.band_cap);
  // all of it was written by earlier launches: the same for every workgroup of the problem
  const bool banded = use_guess && opt.band && !opt.force_dense && rowp->pred_valid != 0 && rowp->band_valid != 0;
  if (!(banded && cand.fits && band.fits && bhi > blo)) {
    // Not this route.  The first pass may still have counted (lists that did not fit): one workgroup clears the
    // problem's histogram and counters; nobody of this launch makes use of them.
    if (sc.group == 0) {
      if (banded)
        for (uint32_t b = t; b < kBandBuckets; b += kWG) bh[b] = 0;
      if (t == 0) {
        rowp->fast = 0;
        rowp->above = 0;
        if (sc.cursor_set != kNoCursorSet)
          for (uint32_t s = 0; s < kSubLists; ++s)
            ws.xcur[(static_cast<size_t>(sc.cursor_set) * kSubLists + s) * kCursorPitch + kCursorAboveWord] = 0;
        uint32_t* cn = ws.counters + row * kCountersPerRow;
        cn[4] = 0;
        cn[5] = !banded ? 1u : (!cand.fits ? 2u : 3u);  // no band was set; the candidate list / the band list overflowed
        ws.flags[0] = 1;  // work for the general kernels
      }
    }
    return;
  }
  // the band entries of this wavefront's first chunks: requested before the histogram is looked at
  const uint2* bandr = ws.band + sc.band_base;
  uint32_t off[kGroup], cnt[kGroup];
  uint2 a[kGroup];
  auto request = [&](const uint2& d) {
    uint32_t cnt_l = (d.y >> 13) & 0x1fffu;
    if (d.x > opt.band_cap) cnt_l = 0;  // segments always lie inside the list; never read outside it
    else if (cnt_l > opt.band_cap - d.x) cnt_l = opt.band_cap - d.x;
#pragma unroll
    for (int u = 0; u < kGroup; ++u) {
      off[u] = __builtin_amdgcn_readlane(d.x, u);
      cnt[u] = __builtin_amdgcn_readlane(cnt_l, u);
      a[u] = lane < cnt[u] ? bandr[off[u] + lane] : make_uint2(0, 0);
    }
  };
  request(ds);
  // ---- 1. the bucket of the threshold key ----
#pragma unroll
  for (uint32_t i = 0; i < kBandBuckets / kWG; ++i) lh[i * kWG + t] = x[i];
  __syncthreads();
  bool inside = total_above < k && k - total_above <= band.total;  // uniform
  const uint32_t miss = total_above >= k ? 4u : (inside ? 6u : 5u);  // the threshold lies above / below the band; or (6) ...
  uint32_t bstar = 0, need = 0;
  if (inside) {
    find_crossing<kBandBuckets>(lh, k - total_above, suf, out2);
    bstar = out2[0];
    need = k - total_above - out2[1];       // how many entries of bucket bstar are kept: 1 <= need <= lh[bstar]
    inside = lh[bstar] <= kBoundaryCap;
  }
  const uint32_t n_boundary = inside ? lh[bstar] : 0u;
  // ---- 2. per chunk: entries kept for certain; the threshold bucket's entries are gathered ----
  if (inside) {
    uint2* bnd = ws.bnd + static_cast<size_t>(row) * kBoundaryCap;
    for (uint32_t c0 = c_first; c0 < end; c0 += kWaves * kGroup) {
      if (c0 != c_first) {  // wave-uniform
        ds = make_uint2(0, 0);
        if (lane < kGroup && c0 + lane < end) ds = d2[c0 + lane];
        request(ds);
      }
      uint32_t gt[kGroup];  // wave-uniform
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        gt[u] = 0;
        for (uint32_t q = 0; q < cnt[u]; q += 64) {  // one trip unless the chunk holds more than 64 band entries
          const uint2 en = q == 0 ? a[u] : (q + lane < cnt[u] ? bandr[off[u] + q + lane] : make_uint2(0, 0));
          const bool ok = q + lane < cnt[u];
          const uint32_t bucket = band_bucket(key_of_bits(en.y) - blo, bmul);
          gt[u] += popc64(ballot64(ok && bucket > bstar));
          if (ok && bucket == bstar) {
            const uint32_t slot = atomicAdd(&rowp->bnd_n, 1u);
            if (slot < kBoundaryCap) {  // always: the histogram counted these entries
              __hip_atomic_store(&bnd[slot].x, en.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              __hip_atomic_store(&bnd[slot].y, en.y, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
          }
        }
      }
      uint32_t mine = 0;
#pragma unroll
      for (int u = 0; u < kGroup; ++u)
        if (lane == static_cast<uint32_t>(u)) mine = gt[u];
      if (lane < kGroup && c0 + lane < end) l_gt[c0 - start + lane] = (ds.y & 0x1fffu) + mine;
    }
    __syncthreads();
    // exclusive prefixes within the block: thread t takes `per` consecutive chunks
    const uint32_t len = end - start;
    const uint32_t per = (cpw + kWG - 1) / kWG;  // <= kMaxCountCpw / kWG
    const uint32_t first = t * per;
    uint32_t sum_gt = 0;
    for (uint32_t i = 0; i < per; ++i)
      if (first + i < len) sum_gt += l_gt[first + i];
    uint32_t tot_gt;
    uint32_t pre_gt = block_excl_scan<kWG>(sum_gt, scratch, &tot_gt);
    uint4* rec = ws.chunk_rec + sc.chunk_base + start;
    for (uint32_t i = 0; i < per; ++i)
      if (first + i < len) {
        const uint32_t g = l_gt[first + i];
        rec[first + i] = make_uint4(g, 0u, pre_gt, 0u);
        pre_gt += g;
      }
    if (t == 0) {  // (device-scope stores: the problem's last workgroup adds the blocks' totals up)
      uint2* tot = ws.blk + static_cast<size_t>(row) * kMaxCountBlocks + sc.group;
      __hip_atomic_store(&tot->x, tot_gt, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(&tot->y, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
  }
  // ---- 3. the problem-wide part, by whichever of its workgroups finishes last ----
  if (!last_group_of_row(&rowp->ticket_band, sc.groups, &sh_flag)) return;
  for (uint32_t b = t; b < kBandBuckets; b += kWG) bh[b] = 0;  // every workgroup has read it
  uint32_t n_kept = 0;
  if (inside) {
    // the gathered entries (written by other workgroups with device-scope stores: read at that scope)
    const uint2* bnd = ws.bnd + static_cast<size_t>(row) * kBoundaryCap;
    const AgentView view = agent_view(reinterpret_cast<const uint32_t*>(bnd), 2 * kBoundaryCap);
    // ... and with the same round trip the blocks' totals, for their prefix sums: the last kernel then needs one
    // number per worker and chunk instead of a sum over all the blocks before the chunk's
    static_assert(kMaxCountBlocks <= kWG, "a thread per count block");
    const AgentView totals = agent_view(reinterpret_cast<const uint32_t*>(ws.blk + static_cast<size_t>(row) * kMaxCountBlocks),
                                        2 * kMaxCountBlocks);
    const uint32_t my_total = t < sc.groups ? load_agent(totals, 2 * t) : 0u;
    if (t < kBoundaryCap) {
      uint2 en = make_uint2(0xffffffffu, 0u);
      if (t < n_boundary) en = make_uint2(load_agent(view, 2 * t), load_agent(view, 2 * t + 1));
      b_en[t] = en;
    }
    {
      uint32_t all;
      const uint32_t before = block_excl_scan<kWG>(my_total, scratch, &all);  // (ends with a barrier of its own)
      if (t < sc.groups) ws.blk_prefix[static_cast<size_t>(row) * kMaxCountBlocks + t] = make_uint2(before, 0u);
    }
    __syncthreads();
    // rank by (key descending, coordinate ascending): coordinates are distinct, so ranks are
    bool kept = false;
    uint32_t my_key = 0, my_coord = 0xffffffffu;
    if (t < n_boundary) {
      my_key = key_of_bits(b_en[t].y);
      my_coord = b_en[t].x;
      uint32_t rank = 0;
      for (uint32_t q = 0; q < n_boundary; ++q) {
        const uint32_t kq = key_of_bits(b_en[q].y), cq = b_en[q].x;
        rank += (kq > my_key || (kq == my_key && cq < my_coord)) ? 1u : 0u;
      }
      kept = rank < need;
      if (rank == need - 1) { out2[0] = my_key; out2[1] = my_coord; }  // the last kept one: tau and the last tie taken
    }
    __syncthreads();
    const uint32_t tau = out2[0], last_coord = out2[1];
    // ties, and the kept entries' coordinates in ascending order
    if (t < kBoundaryCap) b_rank[t] = 0xffffffffu;
    __syncthreads();
    uint32_t is_tie = 0;
    if (t < n_boundary) {
      is_tie = my_key == tau ? 1u : 0u;
      if (kept) {
        uint32_t pos = 0;
        for (uint32_t q = 0; q < n_boundary; ++q) {
          const uint32_t kq = key_of_bits(b_en[q].y), cq = b_en[q].x;
          const bool kept_q = kq > tau || (kq == tau && cq <= last_coord);
          pos += (kept_q && cq < my_coord) ? 1u : 0u;
        }
        b_rank[pos] = my_coord;
      }
    }
    __syncthreads();
    static_assert(kBoundaryCap <= 64, "the first wavefront holds all of it");
    if (wave == 0) {
      const uint32_t ties = popc64(ballot64(is_tie != 0));
      const uint32_t ties_in = popc64(ballot64(is_tie != 0 && my_coord <= last_coord));
      if (lane == 0) { suf[0] = ties; suf[1] = ties_in; }
    }
    __syncthreads();
    const uint32_t n_ties = suf[0];
    n_kept = need;
    uint32_t* sel = ws.bnd_sel + static_cast<size_t>(row) * kBoundaryCap;
    if (t < kBoundaryCap) sel[t] = b_rank[t];
    if (t == 0) {
      // ties kept: those at coordinates <= last_coord; all of them if the last tie is kept
      const uint32_t ties_kept = suf[1], ties_after = n_ties - ties_kept;
      const uint32_t tau_prev = tau_before;
      rowp->fast = 1;
      rowp->level1_done = 1;
      rowp->mode = kModeCand;
      rowp->n_src = cand.total;
      rowp->tau_prev = tau_prev;
      rowp->tau = tau;
      rowp->r = ties_kept;
      rowp->ties = n_ties;
      rowp->tie_last = ties_after ? last_coord : 0xffffffffu;
      rowp->bnd_kept = n_kept;
      ws.tau[row] = tau;
      ws.count_gt[row] = k - ties_kept;
      uint32_t* cn = ws.counters + row * kCountersPerRow;
      cn[0] = 0;
      cn[1] = cand.total;
      cn[2] = n_ties;
      cn[3] = ties_kept;
      cn[4] = band.total;
      cn[5] = 0;
      // Guess for the next step, as the general route sets it but from what is known here: the candidate list held
      // cand.total entries at or above bucket bg, so that many bound the entries from any bucket >= bg upwards;
      // of the bucket below bg nothing is known, and it is taken to hold at most as many again.
      const uint32_t b0 = tau >> kL0Shift;  // >= bg
      uint32_t valid = 0, guess = 0;
      if (opt.predict) {
        const uint32_t bound = b0 > bg ? cand.total : 2u * cand.total;  // entries from bucket b0 - 1 upwards
        if (b0 && bound <= opt.cap / 2) { valid = 1; guess = b0 - 1; }
        else if (cand.total <= opt.cap / 2) { valid = 1; guess = b0; }
      }
      rowp->pred_valid = valid;
      rowp->b_guess = guess;
      const float width = (__uint_as_float(bhi) - __uint_as_float(blo)) / __uint_as_float(tau);  // band keys are normal floats
      const float noise = 8.0f * width * sqrtf(static_cast<float>(k)) / static_cast<float>(band.total);
      set_next_band(rowp, tau, tau_prev, tau_before2, valid, guess, noise, opt);
    }
  } else if (t == 0) {
    rowp->fast = 0;
    uint32_t* cn = ws.counters + row * kCountersPerRow;
    cn[4] = 0;
    cn[5] = miss;  // (6): ... its bucket holds more entries than are ranked here
    ws.flags[0] = 1;  // work for the general kernels
  }
  if (t == 0) {
    rowp->above = 0;
    rowp->bnd_n = 0;
    if (inside) {  // the cursors go back to zero for the next step (else the general kernels still read them)
      rowp->cursor = 0;
      rowp->cursor_band = 0;
    }
    if (sc.cursor_set != kNoCursorSet) {
      for (uint32_t s = 0; s < kSubLists; ++s) {
        uint32_t* cur = ws.xcur + (static_cast<size_t>(sc.cursor_set) * kSubLists + s) * kCursorPitch;
        if (inside) { cur[0] = 0; cur[1] = 0; }
        cur[kCursorAboveWord] = 0;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Level 0 after the lean first pass.  A row whose guess held (its candidate list holds at least k entries and
// did not overflow) gets the histogram of threshold buckets from the list -- every key at or above the guessed
// bucket is in it, so the k-th largest key of the list is the row's -- together with the level-1 histograms of
// the three buckets from the guess upwards.  Any other row (no guess yet, the guess was too high, the list
// overflowed) gets its histogram from the stored values themselves, one more read of the row.  The last
// workgroup of the row finds the threshold bucket, decides the route of the remaining kernels and leaves the
// guess for the next step.
// ---------------------------------------------------------------------------------------------
template <bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_level0(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                      TopkOptions opt, uint32_t use_guess) {
  if (table_u32(ws.flags, 0) == 0) return;  // every problem of this step was selected by k_topk_band
  __shared__ uint32_t lh[kNB0];
  __shared__ uint32_t lh1[kTracked * kNB1];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  __shared__ uint32_t sh_flag, sh_l1, sh_bstar, sh_need;
  const SegCtx sc = seg_ctx<UNI, kClassLevel0>(geo, opt, ws);
  const uint32_t row = sc.seg;
  TopkRow* rowp = ws.rows + row;
  if (rowp->fast) return;  // the threshold was found in the band (k_topk_band); same for the whole row
  const uint32_t bg = rowp->b_guess;
  const ListRuns runs = runs_from_cursors(ws, rowp, sc.cursor_set, opt.cap);  // written by the previous launch
  const bool listed = use_guess && rowp->pred_valid != 0 && runs.total >= geo.k && runs.fits && !opt.force_dense;
  for (int b = threadIdx.x; b < kNB0; b += kWG) lh[b] = 0;
  for (uint32_t b = threadIdx.x; b < kTracked * kNB1; b += kWG) lh1[b] = 0;
  __syncthreads();
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  if (listed) {
    sweep_list(ws.cand + sc.cand_base, runs, sc.group * kWG + threadIdx.x, sc.groups * kWG, [&](uint32_t bits) {
      const uint32_t key = key_of_bits(bits);
      const uint32_t bucket = key >> kL0Shift;
      atomicAdd(&lh[bucket], 1u);
      const uint32_t rel = bucket - bg;
      if (rel < kTracked) atomicAdd(&lh1[rel * kNB1 + ((key >> kL1Shift) & (kNB1 - 1))], 1u);
    });
  } else {
    const float* er = e + sc.elem_off;
    uint32_t zeros = 0;
    const uint32_t stride = sc.groups * kWaves;
    for (uint32_t c = sc.group * kWaves + wave; c < geo.num_chunks; c += stride) {
      const uint32_t base = c * kChunk + lane * 4;
#pragma unroll 4
      for (int r = 0; r < kRounds; ++r) {
        const uint32_t j = base + r * 256;
        if (c * kChunk + r * 256 >= geo.d) break;  // wave-uniform
        float4 x = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < geo.d) x = *reinterpret_cast<const float4*>(er + j);
        Quad q;
        q.key[0] = key_of_bits(__float_as_uint(x.x)); q.key[1] = key_of_bits(__float_as_uint(x.y));
        q.key[2] = key_of_bits(__float_as_uint(x.z)); q.key[3] = key_of_bits(__float_as_uint(x.w));
#pragma unroll
        for (int s = 0; s < 4; ++s) q.ok[s] = j + s < geo.d;
        hist4<false>(lh, q, zeros);
      }
    }
    if (zeros && lane == 0) atomicAdd(&lh[0], zeros);
  }
  __syncthreads();
  uint32_t* gh = ws.hist0 + static_cast<size_t>(row) * kNB0;
  for (int b = threadIdx.x; b < kNB0; b += kWG) {
    const uint32_t h = lh[b];
    if (h) atomicAdd(&gh[b], h);
  }
  uint32_t* gh1 = ws.hist1x + static_cast<size_t>(row) * kTracked * kNB1;
  if (listed)
    for (uint32_t b = threadIdx.x; b < kTracked * kNB1; b += kWG) {
      const uint32_t h = lh1[b];
      if (h) atomicAdd(&gh1[b], h);
    }
  // ---- row-wide part, by whichever workgroup of the row finishes last ----
  if (!last_group_of_row(&rowp->ticket[0], sc.groups, &sh_flag)) return;
  take_hist<kNB0>(gh, lh);
  find_crossing<kNB0>(lh, geo.k, suf, out2);
  if (threadIdx.x == 0) {
    const uint32_t bstar = out2[0], above = out2[1];
    const uint32_t total = above + lh[bstar];  // entries with bucket >= bstar
    uint32_t mode, n_src, reads;
    if (listed) { mode = kModeCand; n_src = runs.total; reads = 0; }  // bstar >= bg: the list holds the k largest keys
    else if (total <= opt.cap && !opt.force_dense) { mode = kModeNeedB; n_src = total; reads = 1; }
    else { mode = kModeDense; n_src = 0; reads = 4; }
    rowp->mode = mode;
    rowp->n_src = n_src;
    // the list's runs for the sweeps that follow: as the first pass left them, or the one run that the second
    // read of the row is about to write; the cursors go back to zero for that read and for the next step
    rowp->n_lists = listed ? runs.lists : 1u;
#pragma unroll
    for (uint32_t s = 0; s < kSubLists; ++s) rowp->n_sub[s] = listed ? runs.n[s] : (s == 0 ? n_src : 0u);
    rowp->cursor = 0;
    rowp->cursor_band = 0;
    if (sc.cursor_set != kNoCursorSet) {
#pragma unroll
      for (uint32_t s = 0; s < kSubLists; ++s) {
        uint32_t* cur = ws.xcur + (static_cast<size_t>(sc.cursor_set) * kSubLists + s) * kCursorPitch;
        cur[0] = 0;
        cur[1] = 0;
      }
    }
    rowp->bstar = bstar;
    rowp->need = geo.k - above;
    rowp->level1_done = 0;
    // Guess for the next step: one bucket below this step's threshold bucket if the list that guess would
    // have produced now fits with room to spare, else the bucket itself, else no guess.  From a list, nothing
    // is known about the buckets below the guess it was made with: the bucket below is then taken to hold at
    // most as many entries as all the buckets above it together.
    uint32_t valid = 0, guess = 0;
    if (opt.predict && !opt.force_dense) {
      const uint32_t below = bstar ? ((listed && bstar == bg) ? total : lh[bstar - 1]) : 0;
      if (bstar && total + below <= opt.cap / 2) { valid = 1; guess = bstar - 1; }
      else if (total <= opt.cap / 2) { valid = 1; guess = bstar; }
    }
    rowp->pred_valid = valid;
    rowp->b_guess = guess;
    uint32_t* cn = ws.counters + row * kCountersPerRow;
    cn[0] = reads;
    cn[1] = n_src;
    sh_l1 = (listed && bstar - bg < kTracked) ? 1u + (bstar - bg) : 0u;
    sh_bstar = bstar;
    sh_need = geo.k - above;
  }
  __syncthreads();
  if (listed) {
    const uint32_t which = sh_l1;  // 0: level 1 not available; 1 + t: histogram of bucket guess + t
    if (which) {
      const AgentView view = agent_view(gh1 + (which - 1) * kNB1, kNB1);
      uint32_t x[kNB1 / kWG];
#pragma unroll
      for (int i = 0; i < kNB1 / kWG; ++i) x[i] = load_agent(view, i * kWG + threadIdx.x);
#pragma unroll
      for (int i = 0; i < kNB1 / kWG; ++i) lh[i * kWG + threadIdx.x] = x[i];
    }
    for (uint32_t b = threadIdx.x; b < kTracked * kNB1; b += kWG) gh1[b] = 0;
    __syncthreads();
    if (which) resolve_level1(rowp, sh_bstar, sh_need, lh, suf, out2);
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel 2: level 1 for rows that could not resolve it in the first pass.
//   kModeNeedB: one more read of the row; writes the candidate list (bucket >= bstar) and the histogram.
//   kModeCand : the list exists (the threshold bucket was above the tracked ones): sweep it.
//   kModeDense: no list: histogram from the row itself.
// ---------------------------------------------------------------------------------------------
template <bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_level1(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                      TopkOptions opt) {
  if (table_u32(ws.flags, 0) == 0) return;  // every problem of this step was selected by k_topk_band
  __shared__ uint32_t lh[kNB1];
  __shared__ uint2 stage_all[kWaves * kStage];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  __shared__ uint32_t sh_flag;
  const SegCtx sc = seg_ctx<UNI, kClassSweep>(geo, opt, ws);
  const uint32_t row = sc.seg;
  TopkRow* rowp = ws.rows + row;
  if (rowp->fast || rowp->level1_done) return;
  const uint32_t mode = rowp->mode, bstar = rowp->bstar, need = rowp->need;
  for (int b = threadIdx.x; b < kNB1; b += kWG) lh[b] = 0;
  __syncthreads();
  const float* er = e + sc.elem_off;
  uint2* candr = ws.cand + sc.cand_base;
  auto visit = [&](uint32_t bits, bool ok) {
    const uint32_t key = key_of_bits(bits);
    if (ok && (key >> kL0Shift) == bstar) atomicAdd(&lh[(key >> kL1Shift) & (kNB1 - 1)], 1u);
  };
  if (mode == kModeNeedB) {
    uint2* descr = ws.desc + sc.chunk_base;
    const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
    uint2* stage = stage_all + wave * kStage;
    const uint32_t stride = sc.groups * kWaves;
    for (uint32_t c = sc.group * kWaves + wave; c < geo.num_chunks; c += stride) {
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
        for (int s = 0; s < 4; ++s) {
          flag[s] = j + s < geo.d && (key_of_bits(bits[s]) >> kL0Shift) >= bstar;
          visit(bits[s], j + s < geo.d);
        }
        stage_round(stage, cnt, j, bits, flag);
      }
      // fits by construction: the level-0 histogram counted exactly these entries
      flush_chunk(stage, cnt, er, geo.d, c, bstar, rowp, candr, opt.cap, descr);
    }
  } else if (mode == kModeCand) {
    const ListRuns runs = runs_of_row(rowp, opt.cap);
    sweep_list(candr, runs, sc.group * kWG + threadIdx.x, sc.groups * kWG, [&](uint32_t bits) { visit(bits, true); });
  } else {
    const uint32_t step = sc.groups * kWG * 4;
    for (uint32_t j = (sc.group * kWG + threadIdx.x) * 4; j < geo.d; j += step) {
      const float4 x = *reinterpret_cast<const float4*>(er + j);
      visit(__float_as_uint(x.x), true);
      visit(__float_as_uint(x.y), j + 1 < geo.d);
      visit(__float_as_uint(x.z), j + 2 < geo.d);
      visit(__float_as_uint(x.w), j + 3 < geo.d);
    }
  }
  __syncthreads();
  uint32_t* gh = ws.hist1 + static_cast<size_t>(row) * kNB1;
  for (int b = threadIdx.x; b < kNB1; b += kWG) {
    const uint32_t h = lh[b];
    if (h) atomicAdd(&gh[b], h);
  }
  if (!last_group_of_row(&rowp->ticket[1], sc.groups, &sh_flag)) return;
  take_hist<kNB1>(gh, lh);
  resolve_level1(rowp, bstar, need, lh, suf, out2);
}

// ---------------------------------------------------------------------------------------------
// Kernel 3: level 2 (last 9 key bits) over the entries that match bits 30..9 of the threshold key.
// ---------------------------------------------------------------------------------------------
template <bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_level2(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                      TopkOptions opt) {
  if (table_u32(ws.flags, 0) == 0) return;  // every problem of this step was selected by k_topk_band
  __shared__ uint32_t lh[kNB2];
  __shared__ uint32_t suf[kWG + 1];
  __shared__ uint32_t out2[2];
  __shared__ uint32_t sh_flag;
  const SegCtx sc = seg_ctx<UNI, kClassSweep>(geo, opt, ws);
  const uint32_t row = sc.seg;
  TopkRow* rowp = ws.rows + row;
  if (rowp->fast) return;
  const uint32_t mode = rowp->mode, want = rowp->prefix1, need = rowp->need;
  for (int b = threadIdx.x; b < kNB2; b += kWG) lh[b] = 0;
  __syncthreads();
  auto visit = [&](uint32_t bits, bool ok) {
    const uint32_t key = key_of_bits(bits);
    if (ok && (key >> kL1Shift) == want) atomicAdd(&lh[key & (kNB2 - 1)], 1u);
  };
  if (mode == kModeDense) {
    const float* er = e + sc.elem_off;
    const uint32_t step = sc.groups * kWG * 4;
    for (uint32_t j = (sc.group * kWG + threadIdx.x) * 4; j < geo.d; j += step) {
      const float4 x = *reinterpret_cast<const float4*>(er + j);
      visit(__float_as_uint(x.x), true);
      visit(__float_as_uint(x.y), j + 1 < geo.d);
      visit(__float_as_uint(x.z), j + 2 < geo.d);
      visit(__float_as_uint(x.w), j + 3 < geo.d);
    }
  } else {
    const uint2* candr = ws.cand + sc.cand_base;
    const ListRuns runs = runs_of_row(rowp, opt.cap);
    sweep_list(candr, runs, sc.group * kWG + threadIdx.x, sc.groups * kWG, [&](uint32_t bits) { visit(bits, true); });
  }
  __syncthreads();
  uint32_t* gh = ws.hist2 + static_cast<size_t>(row) * kNB2;
  for (int b = threadIdx.x; b < kNB2; b += kWG) {
    const uint32_t h = lh[b];
    if (h) atomicAdd(&gh[b], h);
  }
  if (!last_group_of_row(&rowp->ticket[2], sc.groups, &sh_flag)) return;
  take_hist<kNB2>(gh, lh);
  find_crossing<kNB2>(lh, need, suf, out2);
  if (threadIdx.x == 0) {
    const uint32_t s = out2[0], above = out2[1];
    const uint32_t tau = (want << kL1Shift) | s;
    const uint32_t r = need - above, ties = lh[s];
    const uint32_t tau_prev = rowp->tau, tau_prev2 = rowp->tau_prev;
    rowp->tau_prev = tau_prev;
    rowp->tau = tau;
    rowp->r = r;
    rowp->ties = ties;
    ws.tau[row] = tau;
    ws.count_gt[row] = geo.k - r;
    uint32_t* cn = ws.counters + row * kCountersPerRow;
    cn[2] = ties;
    cn[3] = r;
    cn[4] = 0;
    // the guess was set when the threshold bucket was found (first kernel of this route, an earlier launch)
    set_next_band(rowp, tau, tau_prev, tau_prev2, rowp->pred_valid, rowp->b_guess, default_band_noise(geo.k), opt);
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
                                               const uint2* __restrict__ candr, uint2 ds, uint32_t cap, F&& f) {
  // ds: the chunk's segment of the candidate list (offset, count), the same in every lane; not looked at without a list
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
    const uint32_t off = first_lane(ds.x);
    uint32_t cnt = first_lane(ds.y);
    if (off > cap) cnt = 0;                      // segments always lie inside the list; never read outside it
    else if (cnt > cap - off) cnt = cap - off;
    constexpr int kAhead = 4;  // loads in flight per trip (long segments would otherwise be a chain of round trips)
    for (uint32_t t = 0; t < cnt; t += 64 * kAhead) {
      uint2 cv[kAhead];
#pragma unroll
      for (int w = 0; w < kAhead; ++w) {
        const uint32_t q = t + w * 64 + lane;
        cv[w] = q < cnt ? candr[off + q] : make_uint2(0, 0);
      }
#pragma unroll
      for (int w = 0; w < kAhead; ++w) {
        if (t + w * 64 >= cnt) break;  // wave-uniform
        Entry4 en;
        en.ok[0] = t + w * 64 + lane < cnt;
        en.j[0] = cv[w].x; en.bits[0] = cv[w].y;
#pragma unroll
        for (int s = 1; s < 4; ++s) { en.j[s] = 0; en.bits[s] = 0; en.ok[s] = false; }
        f(en, 1);
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Kernel 4: per chunk, how many keys lie above tau and how many equal it.  A workgroup owns a contiguous
// block of geo.count_cpw chunks; it leaves, per chunk, the two counts and their exclusive prefixes within
// the block, and per block the two totals.  The last kernel turns these into positions in the worker's
// list (a sum over at most kMaxCountBlocks block totals), so no workgroup waits for or follows another.
// ---------------------------------------------------------------------------------------------
template <bool UNI>
__global__ __launch_bounds__(kWG) void k_topk_count(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                     TopkOptions opt) {
  if (table_u32(ws.flags, 0) == 0) return;  // every problem of this step was selected by k_topk_band
  __shared__ uint32_t l_gt[kMaxCountCpw], l_eq[kMaxCountCpw];
  __shared__ uint32_t scratch[kWG / 64 + 1];
  const SegCtx sc = seg_ctx<UNI, kClassCount>(geo, opt, ws);
  const uint32_t row = sc.seg;
  const uint32_t cpw = geo.count_cpw;
  const uint32_t start = sc.group * cpw;
  if (start >= geo.num_chunks) return;  // uniform; the grid has exactly the blocks that exist
  const uint32_t end = start + cpw < geo.num_chunks ? start + cpw : geo.num_chunks;
  const TopkRow* rowp = ws.rows + row;
  if (rowp->fast) return;
  const uint32_t mode = rowp->mode, tau = rowp->tau;
  const float* er = e + sc.elem_off;
  const uint2* candr = ws.cand + sc.cand_base;
  const uint2* descr = ws.desc + sc.chunk_base;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  if (mode == kModeDense) {
    for (uint32_t c = start + wave; c < end; c += kWaves) {
      uint32_t gt = 0, eq = 0;
      for_each_round(mode, er, geo.d, c, candr, make_uint2(0u, 0u), opt.cap, [&](const Entry4& en, int slots) {
        for (int s = 0; s < slots; ++s) {
          const uint32_t key = key_of_bits(en.bits[s]);
          gt += popc64(ballot64(en.ok[s] && key > tau));
          eq += popc64(ballot64(en.ok[s] && key == tau));
        }
      });
      if (lane == 0) { l_gt[c - start] = gt; l_eq[c - start] = eq; }
    }
  } else {
    // A wavefront takes kGroup consecutive chunks at a time: their descriptors come with one load, the first
    // 128 entries of every segment with independent loads (two round trips for the whole group).
    constexpr int kGroup = 8;
    for (uint32_t c0 = start + wave * kGroup; c0 < end; c0 += kWaves * kGroup) {
      uint2 ds = make_uint2(0, 0);
      if (lane < kGroup && c0 + lane < end) ds = descr[c0 + lane];
      if (ds.x > opt.cap) ds.y = 0;  // segments always lie inside the list; never read outside it
      else if (ds.y > opt.cap - ds.x) ds.y = opt.cap - ds.x;
      uint32_t off[kGroup], cnt[kGroup];
      uint2 a[kGroup], b[kGroup];
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        off[u] = __builtin_amdgcn_readlane(ds.x, u);
        cnt[u] = __builtin_amdgcn_readlane(ds.y, u);
        a[u] = lane < cnt[u] ? candr[off[u] + lane] : make_uint2(0, 0);
        b[u] = lane + 64 < cnt[u] ? candr[off[u] + lane + 64] : make_uint2(0, 0);
      }
      uint32_t gt[kGroup], eq[kGroup];  // wave-uniform
      uint32_t longest = 0;
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const uint32_t ka = key_of_bits(a[u].y), kb = key_of_bits(b[u].y);
        gt[u] = popc64(ballot64(lane < cnt[u] && ka > tau)) + popc64(ballot64(lane + 64 < cnt[u] && kb > tau));
        eq[u] = popc64(ballot64(lane < cnt[u] && ka == tau)) + popc64(ballot64(lane + 64 < cnt[u] && kb == tau));
        longest = cnt[u] > longest ? cnt[u] : longest;
      }
      // long segments: the next 128 entries of every segment of the group per trip, all loads in flight together
      // (a trip per segment instead would make a group of long segments a chain of several dozen round trips)
      for (uint32_t t = 128; t < longest; t += 128) {
        uint32_t ka[kGroup], kb[kGroup];
#pragma unroll
        for (int u = 0; u < kGroup; ++u) {
          ka[u] = kb[u] = 0;
          if (t < cnt[u]) {  // wave-uniform
            if (t + lane < cnt[u]) ka[u] = key_of_bits(candr[off[u] + t + lane].y);
            if (t + 64 + lane < cnt[u]) kb[u] = key_of_bits(candr[off[u] + t + 64 + lane].y);
          }
        }
#pragma unroll
        for (int u = 0; u < kGroup; ++u)
          if (t < cnt[u]) {
            const bool oa = t + lane < cnt[u], ob = t + 64 + lane < cnt[u];
            gt[u] += popc64(ballot64(oa && ka[u] > tau)) + popc64(ballot64(ob && kb[u] > tau));
            eq[u] += popc64(ballot64(oa && ka[u] == tau)) + popc64(ballot64(ob && kb[u] == tau));
          }
      }
      uint32_t my_gt = 0, my_eq = 0;
#pragma unroll
      for (int u = 0; u < kGroup; ++u)
        if (lane == static_cast<uint32_t>(u)) { my_gt = gt[u]; my_eq = eq[u]; }
      if (lane < kGroup && c0 + lane < end) { l_gt[c0 - start + lane] = my_gt; l_eq[c0 - start + lane] = my_eq; }
    }
  }
  __syncthreads();
  // exclusive prefixes within the block: thread t takes `per` consecutive chunks
  const uint32_t len = end - start;
  const uint32_t per = (cpw + kWG - 1) / kWG;  // <= kMaxCountCpw / kWG
  const uint32_t first = threadIdx.x * per;
  uint32_t sum_gt = 0, sum_eq = 0;
  for (uint32_t i = 0; i < per; ++i)
    if (first + i < len) { sum_gt += l_gt[first + i]; sum_eq += l_eq[first + i]; }
  uint32_t tot_gt, tot_eq;
  uint32_t pre_gt = block_excl_scan<kWG>(sum_gt, scratch, &tot_gt);
  uint32_t pre_eq = block_excl_scan<kWG>(sum_eq, scratch, &tot_eq);
  uint4* rec = ws.chunk_rec + sc.chunk_base + start;
  for (uint32_t i = 0; i < per; ++i)
    if (first + i < len) {
      const uint32_t gt = l_gt[first + i], eq = l_eq[first + i];
      rec[first + i] = make_uint4(gt, eq, pre_gt, pre_eq);
      pre_gt += gt;
      pre_eq += eq;
    }
  if (threadIdx.x == 0) ws.blk[static_cast<size_t>(row) * kMaxCountBlocks + sc.group] = make_uint2(tot_gt, tot_eq);
}

// ---------------------------------------------------------------------------------------------
// Kernel 5: per chunk of coordinates.  Workers are taken in tiles of kTileWorkers.
//   Phase 1: a wavefront finds where its workers' entries of this chunk go in the workers' lists (entries
//            above the threshold in earlier chunks, plus the ties taken there: in coordinate order until r
//            are in) and writes the selected (coordinate, value) pairs there.
//   Phase 2: the chunk's entries are added into an LDS tile of the summed gradient, one worker after
//            the other (a barrier between them): the fp32 sum has exactly the order i = 0 .. n-1, and
//            one worker's coordinates are distinct, so no atomics are needed.
//   Phase 3: gbar = sum / n and the AMSGrad moment and parameter update (server lines of Algorithm 2).
// ---------------------------------------------------------------------------------------------
// One wavefront writes the selected entries of chunk c of one selection problem to their places in the list:
// `at` is where the chunk's slice starts, eq_seen how many keys equal to tau lie in earlier chunks (ties are
// taken in coordinate order until r are in).  Coordinates are written relative to the worker's row
// (coord_base = the problem's first coordinate there).  by_coord: the ties to keep are given as "up to and
// including coordinate tie_last of the problem" (k_topk_band) instead of through r and eq_seen.
__device__ __forceinline__ void emit_chunk(uint32_t mode, const float* __restrict__ er, uint32_t d, uint32_t c,
                                           const uint2* __restrict__ candr, uint2 ds,
                                           uint32_t cap, uint32_t tau, uint32_t r, bool all_ties, uint32_t eq_seen,
                                           uint32_t at, int32_t* __restrict__ idx, float* __restrict__ val, uint32_t k,
                                           uint32_t coord_base, bool by_coord, uint32_t tie_last) {
  for_each_round(mode, er, d, c, candr, ds, cap, [&](const Entry4& en, int slots) {
    bool sel[4] = {false, false, false, false};
    if (by_coord) {
      for (int s = 0; s < slots; ++s) {
        const uint32_t key = key_of_bits(en.bits[s]);
        sel[s] = en.ok[s] && (key > tau || (key == tau && en.j[s] <= tie_last));
      }
    } else if (all_ties) {
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
        if (pos < k) {  // always true when the counts are consistent
          idx[pos] = static_cast<int32_t>(coord_base + en.j[s]);
          val[pos] = __uint_as_float(en.bits[s]);
        }
        ++pos;
      }
    at += total;
  });
}

constexpr int kPerWave = 4;                       // workers per wavefront and tile
constexpr int kTileWorkers = kWaves * kPerWave;

// ROLE: kWholeStep runs all phases; kWorkerHalf stops after phase 1 (the workers' lines of Algorithm 2: the
// lists are the messages); kServerHalf starts at phase 2 from lists that were put into the workspace (the
// server's lines; where a chunk's slice of each list starts was found by k_topk_list_offsets).
// (eight wavefronts per SIMD: the streaming phase needs the occupancy more than phase 1 needs registers)
enum : int { kWholeStep = 0, kWorkerHalf = 1, kServerHalf = 2 };

// UNI: one selection problem per worker over its whole row, one workgroup per chunk of the row.  !UNI (whole step
// only): top-k inside every block; a workgroup takes one chunk of one block (flat launch over map_final) and goes
// through the workers' segments of that block, which lie a fixed stride apart in every table.
struct FinalCtx {
  uint32_t c;                     // chunk of the problem
  uint32_t base;                  // first coordinate of the chunk, in coordinates of the worker's row
  uint32_t coord_base, d_loc;     // the problem covers coordinates coord_base .. coord_base + d_loc of the row
  uint32_t k_loc, num_chunks, count_cpw, cap;
  bool micro;                     // the list entries are there already (written by the first pass)
  uint32_t row0, row_stride;      // control block of worker i: row0 + i * row_stride
  size_t chunk0, chunk_stride, seloff0, seloff_stride, cand0, cand_stride, list0, list_stride;
};

template <bool UNI>
__device__ __forceinline__ FinalCtx final_ctx(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt,
                                              const TopkFlat& flat) {
  FinalCtx f;
  if (UNI) {
    f.c = blockIdx.x;
    f.base = f.c * kChunk;
    f.coord_base = 0; f.d_loc = geo.d; f.k_loc = geo.k; f.num_chunks = geo.num_chunks; f.count_cpw = geo.count_cpw;
    f.cap = opt.cap;
    f.micro = false;
    f.row0 = 0; f.row_stride = 1;
    f.chunk0 = 0; f.chunk_stride = geo.num_chunks;
    f.seloff0 = 0; f.seloff_stride = geo.num_chunks + 1;
    f.cand0 = 0; f.cand_stride = opt.cap;
    f.list0 = 0; f.list_stride = geo.k;
  } else {
    const WgSlot slot = ws.map_final[blockIdx.x];
    const Seg sg = ws.segs[slot.seg];  // worker 0's segment of the block
    f.c = slot.group;
    f.coord_base = sg.coord_base;
    f.base = sg.coord_base + f.c * kChunk;
    f.d_loc = sg.d; f.k_loc = sg.k; f.num_chunks = sg.num_chunks; f.count_cpw = sg.count_cpw;
    f.cap = opt.cap < sg.cap ? opt.cap : sg.cap;
    f.micro = sg.micro != 0;
    f.row0 = slot.seg; f.row_stride = flat.blocks;
    f.chunk0 = sg.chunk_base; f.chunk_stride = flat.chunk_stride;
    f.seloff0 = sg.seloff_base; f.seloff_stride = flat.seloff_stride;
    f.cand0 = sg.cand_base; f.cand_stride = flat.cand_stride;
    f.list0 = sg.list_base; f.list_stride = geo.k;  // a worker's list holds the lists of all its blocks
  }
  return f;
}

// NC: how many of theta, m, v, vhat (in that order) are read and written with ordinary accesses, the others with
// streaming ones (a template parameter: as a run-time choice between otherwise identical branches the compiler
// merges them and drops the hint).
template <int ROLE, bool UNI, int NC>
__global__ __launch_bounds__(kWG) __attribute__((amdgpu_waves_per_eu((UNI && NC == 4) ? 8 : 7, 8))) void k_topk_final(
    float* __restrict__ theta, float* __restrict__ m, float* __restrict__ v, float* __restrict__ vhat,
    const float* __restrict__ e, Geometry geo, TopkWorkspace ws, TopkOptions opt, AmsParams p, TopkFlat flat) {
  static_assert(UNI || ROLE == kWholeStep, "the halves of a step work on whole rows");
  __shared__ float gs[kChunk];
  __shared__ uint32_t sh_lo[kTileWorkers], sh_hi[kTileWorkers], sh_eqb[kTileWorkers];
  const FinalCtx f = final_ctx<UNI>(geo, ws, opt, flat);
  const uint32_t c = f.c;
  const uint32_t base = f.base;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();  // the wavefront's number: a scalar
  if (ROLE != kWorkerHalf)
    for (int t = threadIdx.x; t < kChunk; t += kWG) gs[t] = 0.0f;
  if (ROLE != kServerHalf && blockIdx.x == 0 && threadIdx.x == 0) ws.flags[0] = 0;  // the general kernels have run
  if (ROLE != kServerHalf && c == 0)  // the next step's first pass allocates its candidate lists from the start
    for (uint32_t i = threadIdx.x; i < geo.n; i += kWG) {
      ws.rows[f.row0 + i * f.row_stride].cursor = 0;
      ws.rows[f.row0 + i * f.row_stride].cursor_band = 0;
    }
  const uint32_t my_block = c / f.count_cpw;  // count blocks before this chunk's
  // State that comes from HBM (not all of it kept in the memory-side cache): the first quarter of the chunk's is
  // requested here, before the look-ups of phases 1 and 2, and travels while they run (16 more registers: seven
  // wavefronts per SIMD; measured on the final kernel: GPT-2, nothing cached, 727 -> 650-710 us; ResNet-50, two
  // arrays cached, 139 -> 137; two quarters, at five wavefronts, are slower again; with all four arrays cached the
  // request gains nothing and the kernel keeps its eight wavefronts).
  constexpr int kEarly = (ROLE != kWorkerHalf && UNI && NC < 4) ? 1 : 0;  // (the per-block form has no registers to spare)
  const uint32_t d_end = f.coord_base + f.d_loc;  // the chunk's coordinates end here at the latest
  float4 th0[kEarly > 0 ? kEarly : 1], mm0[kEarly > 0 ? kEarly : 1], vv0[kEarly > 0 ? kEarly : 1];
#pragma unroll
  for (int r = 0; r < kEarly; ++r) {
    const uint32_t j = base + r * kWG * 4 + threadIdx.x * 4;
    th0[r] = mm0[r] = vv0[r] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (j + 3 < d_end) {
      th0[r] = load_state4<(NC > 0)>(theta + j); mm0[r] = load_state4<(NC > 1)>(m + j);
      vv0[r] = load_state4<(NC > 2)>(v + j);  // (vhat follows in phase 3: a fourth early load would be spilled)
    }
  }

  for (uint32_t i0 = 0; i0 < geo.n; i0 += kTileWorkers) {
    if (ROLE == kServerHalf) {
      if (threadIdx.x < kTileWorkers && i0 + threadIdx.x < geo.n) {
        const uint32_t* so = ws.sel_off_srv + static_cast<size_t>(i0 + threadIdx.x) * (geo.num_chunks + 1) + c;
        sh_lo[threadIdx.x] = so[0];
        sh_hi[threadIdx.x] = so[1];
      }
    } else {
    // ---- phase 1a: positions, for this wavefront's workers of the tile (all loads issued together) ----
    {
      uint4 rec[kPerWave];
      uint2 part[kPerWave];
      uint32_t r_[kPerWave];
      uint32_t fast_mask = 0;  // wave-uniform: bit u = worker u of this wavefront was selected by k_topk_band
      // Nothing is looked at before everything has been asked for (a sum inside the loop that loads, a value moved
      // to a scalar register where it is loaded, or a branch around a worker's loads makes every worker a round
      // trip of its own): the chunk's record and the first 128 block totals of each worker as vector loads, r and
      // the route through the scalar path.  A worker beyond the last reads worker i0's tables and is ignored.
      uint2 pre[kPerWave];
      uint32_t fast_[kPerWave];
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const uint32_t i = i0 + wave + u * kWaves;
        const uint32_t is = i < geo.n ? i : i0;
        const uint32_t rowi = f.row0 + is * f.row_stride;
        rec[u] = ws.chunk_rec[f.chunk0 + is * f.chunk_stride + c];
        // a problem selected by k_topk_band has the sum over the blocks before the chunk's ready (the same in
        // every lane); for any other the blocks' totals are added up below
        pre[u] = make_uint2(0, 0);
        if (my_block) pre[u] = ws.blk_prefix[static_cast<size_t>(rowi) * kMaxCountBlocks + my_block];
        const uint32_t* rw = reinterpret_cast<const uint32_t*>(ws.rows + rowi);
        r_[u] = table_u32(rw, offsetof(TopkRow, r) / 4);
        fast_[u] = table_u32(rw, offsetof(TopkRow, fast) / 4);
      }
      bool sums = false;  // wave-uniform: some worker of this wavefront needs its totals added up
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const bool there = i0 + wave + u * kWaves < geo.n;  // wave-uniform
        fast_mask |= (there && fast_[u] ? 1u : 0u) << u;
        sums = sums || (there && !fast_[u] && my_block != 0);
        part[u] = pre[u];
        if (!there) { rec[u] = make_uint4(0, 0, 0, 0); part[u] = make_uint2(0, 0); r_[u] = 0; }
      }
      if (sums) {  // the general kernels' problems (the rare route: worker after worker, few registers)
#pragma unroll
        for (int u = 0; u < kPerWave; ++u) {
          const uint32_t i = i0 + wave + u * kWaves;
          if (i < geo.n && !((fast_mask >> u) & 1u)) {  // wave-uniform
            const uint2* blk = ws.blk + static_cast<size_t>(f.row0 + i * f.row_stride) * kMaxCountBlocks;
            uint2 sum = make_uint2(0, 0);
            for (uint32_t b = lane; b < my_block; b += 64) {
              const uint2 t = blk[b];
              sum.x += t.x;
              sum.y += t.y;
            }
            part[u] = make_uint2(wave_sum(sum.x), wave_sum(sum.y));
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const uint32_t i = i0 + wave + u * kWaves;
        if (i >= geo.n) continue;  // wave-uniform
        const uint32_t gt_before = part[u].x + rec[u].z;
        const uint32_t eq_before = part[u].y + rec[u].w;
        const uint32_t r = ((fast_mask >> u) & 1u) ? 0u : r_[u];  // that route does not use the "equal to tau" columns
        const uint32_t taken_before = eq_before < r ? eq_before : r;  // ties go in coordinate order until r are in
        const uint32_t quota = r - taken_before;
        const uint32_t take_here = rec[u].y < quota ? rec[u].y : quota;
        const uint32_t at = gt_before + taken_before;
        const uint32_t hi = at + rec[u].x + take_here;
        if (lane == 0) {
          sh_lo[i - i0] = at;
          sh_hi[i - i0] = hi;
          sh_eqb[i - i0] = eq_before;
        }
      }
      // A row selected by k_topk_band: the kept entries of the threshold's bucket are not in the tables above.
      // Their coordinates (ascending, 0xffffffff beyond the last) come with one load per lane; those before the
      // chunk move its slice of the list up, those inside lengthen it.
      if (fast_mask) {  // wave-uniform
        static_assert(kBoundaryCap == 64, "one entry per lane");
        uint32_t a[kPerWave];
#pragma unroll
        for (int u = 0; u < kPerWave; ++u) {
          const uint32_t i = i0 + wave + u * kWaves;
          a[u] = 0xffffffffu;
          if ((fast_mask >> u) & 1u)
            a[u] = ws.bnd_sel[static_cast<size_t>(f.row0 + i * f.row_stride) * kBoundaryCap + lane];
        }
        const uint32_t lo_c = c * kChunk, hi_c = lo_c + kChunk;  // coordinates of the problem
#pragma unroll
        for (int u = 0; u < kPerWave; ++u) {
          const uint32_t i = i0 + wave + u * kWaves;
          if (!((fast_mask >> u) & 1u)) continue;
          const uint32_t before = popc64(ballot64(a[u] < lo_c));
          const uint32_t here = popc64(ballot64(a[u] >= lo_c && a[u] < hi_c));
          if (lane == 0) {
            sh_lo[i - i0] += before;
            sh_hi[i - i0] += before + here;
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kPerWave; ++u) {
        const uint32_t i = i0 + wave + u * kWaves;
        if (i >= geo.n) continue;  // wave-uniform
        if (lane == 0) {
          uint32_t* so = ws.sel_off + f.seloff0 + i * f.seloff_stride;
          so[c] = sh_lo[i - i0];  // the next step's first pass finds this chunk's slice of the list here
          if (c + 1 == f.num_chunks) so[c + 1] = sh_hi[i - i0];
        }
      }
    }
    // ---- phase 1b: write the selected entries (positions come back from LDS: written by this wavefront) ----
    // What a worker's turn needs of its control block and the chunk's segment descriptor is the same in every lane
    // and was written by earlier launches: it comes through the scalar path, all of it with one round trip, and the
    // next worker's is asked for before this worker's entries are (a turn was a chain of three round trips).
    {
      struct Turn { uint32_t mode, tau, r, ties, fast, tie_last, off, cnt; };
      auto fetch = [&](uint32_t i) {
        Turn w{kModeDense, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
        if (i < geo.n && i < i0 + kTileWorkers) {  // wave-uniform
          const uint32_t* rw = reinterpret_cast<const uint32_t*>(ws.rows + f.row0 + i * f.row_stride);
          w.mode = table_u32(rw, offsetof(TopkRow, mode) / 4);
          w.tau = table_u32(rw, offsetof(TopkRow, tau) / 4);
          w.r = table_u32(rw, offsetof(TopkRow, r) / 4);
          w.ties = table_u32(rw, offsetof(TopkRow, ties) / 4);
          w.fast = table_u32(rw, offsetof(TopkRow, fast) / 4);
          w.tie_last = table_u32(rw, offsetof(TopkRow, tie_last) / 4);
          const uint32_t* dw = reinterpret_cast<const uint32_t*>(ws.desc + f.chunk0 + i * f.chunk_stride + c);
          w.off = table_u32(dw, 0);
          w.cnt = table_u32(dw, 1);
        }
        return w;
      };
      Turn next = fetch(i0 + wave);
#pragma unroll 1
      for (uint32_t i = i0 + wave; i < geo.n && i < i0 + kTileWorkers; i += kWaves) {
        const Turn w = next;
        next = fetch(i + kWaves);
        const uint32_t at = sh_lo[i - i0];
        const uint32_t hi = sh_hi[i - i0];
        if (hi == at || f.micro) continue;  // nothing of this worker in the chunk, or written already (wave-uniform)
        const float* er = e + static_cast<int64_t>(i) * geo.ld + f.coord_base;
        const uint2* candr = ws.cand + f.cand0 + i * f.cand_stride;
        int32_t* idx = ws.idx + f.list0 + i * f.list_stride;
        float* val = ws.val + f.list0 + i * f.list_stride;
        emit_chunk(w.mode, er, f.d_loc, c, candr, make_uint2(w.off, w.cnt), f.cap, w.tau, w.r, w.r == w.ties,
                   sh_eqb[i - i0], at, idx, val, f.k_loc, f.coord_base, w.fast != 0, w.tie_last);
      }
    }
    }  // ROLE != kServerHalf
    if (ROLE == kWorkerHalf) continue;
    __syncthreads();  // the chunk's list entries and their positions are visible to the whole workgroup

    // ---- phase 2 ----
    // Workers are taken in groups of kGroup: every thread first requests its entry of each worker's chunk
    // segment (independent loads, one round trip for the whole group), then the entries are added one worker
    // after the other.
    constexpr int kGroup = 8;
    const uint32_t i_end = i0 + kTileWorkers < geo.n ? i0 + kTileWorkers : geo.n;
    for (uint32_t g0 = i0; g0 < i_end; g0 += kGroup) {
      uint32_t lo[kGroup], hi[kGroup], jl[kGroup];
      float vl[kGroup];
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const uint32_t i = g0 + u;
        lo[u] = hi[u] = 0;
        jl[u] = 0xffffffffu;
        vl[u] = 0.0f;
        if (i < i_end) {
          lo[u] = sh_lo[i - i0];
          hi[u] = sh_hi[i - i0] < f.k_loc ? sh_hi[i - i0] : f.k_loc;
          const uint32_t q = lo[u] + threadIdx.x;
          if (q < hi[u]) {
            jl[u] = static_cast<uint32_t>(ws.idx[f.list0 + i * f.list_stride + q]) - base;
            vl[u] = ws.val[f.list0 + i * f.list_stride + q];
          }
        }
      }
#pragma unroll
      for (int u = 0; u < kGroup; ++u) {
        const uint32_t i = g0 + u;
        if (i < i_end && hi[u] > lo[u]) {  // the same in every thread of the workgroup: a worker without entries in
                                           // the chunk (every worker, in more than half of the chunks) adds nothing
                                           // and needs no barrier
          if (jl[u] < static_cast<uint32_t>(kChunk)) gs[jl[u]] = gs[jl[u]] + vl[u];
          // segments longer than a workgroup: four entries per thread and trip, loads in flight together
          for (uint32_t q = lo[u] + kWG + threadIdx.x; q < hi[u]; q += 4 * kWG) {
            uint32_t jj[4];
            float vv[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) {
              const uint32_t qq = q + w * kWG;
              jj[w] = 0xffffffffu;
              vv[w] = 0.0f;
              if (qq < hi[u]) {
                jj[w] = static_cast<uint32_t>(ws.idx[f.list0 + i * f.list_stride + qq]) - base;
                vv[w] = ws.val[f.list0 + i * f.list_stride + qq];
              }
            }
#pragma unroll
            for (int w = 0; w < 4; ++w)
              if (jj[w] < static_cast<uint32_t>(kChunk)) gs[jj[w]] = gs[jj[w]] + vv[w];
          }
          __syncthreads();
        }
      }
    }
  }

  if (ROLE == kWorkerHalf) return;
#pragma unroll
  for (int r = 0; r < kChunk / (kWG * 4); ++r) {
    const uint32_t t = r * kWG * 4 + threadIdx.x * 4;
    const uint32_t j = base + t;
    if (j + 3 < d_end) {
      float4 th, mm, vv, vh;
      if (r < kEarly) {
        th = th0[r]; mm = mm0[r]; vv = vv0[r];
        vh = load_state4<(NC > 3)>(vhat + j);
      } else {
        th = load_state4<(NC > 0)>(theta + j); mm = load_state4<(NC > 1)>(m + j);
        vv = load_state4<(NC > 2)>(v + j); vh = load_state4<(NC > 3)>(vhat + j);
      }
      const float4 s = *reinterpret_cast<const float4*>(gs + t);
      ams_update(s.x / p.nf, th.x, mm.x, vv.x, vh.x, p);
      ams_update(s.y / p.nf, th.y, mm.y, vv.y, vh.y, p);
      ams_update(s.z / p.nf, th.z, mm.z, vv.z, vh.z, p);
      ams_update(s.w / p.nf, th.w, mm.w, vv.w, vh.w, p);
      store_state4<(NC > 0)>(theta + j, th);
      store_state4<(NC > 1)>(m + j, mm);
      store_state4<(NC > 2)>(v + j, vv);
      store_state4<(NC > 3)>(vhat + j, vh);
    } else {
      for (uint32_t s = 0; s < 4 && j + s < d_end; ++s) {
        float th = theta[j + s], mm = m[j + s], vv = v[j + s], vh = vhat[j + s];
        ams_update(gs[t + s] / p.nf, th, mm, vv, vh, p);
        theta[j + s] = th; m[j + s] = mm; v[j + s] = vv; vhat[j + s] = vh;
      }
    }
  }
}

// Top-k inside every block: the workers' last lines on their own.  A wavefront takes one chunk of one segment,
// finds where its slice of the list starts (as phase 1 of the kernel above does for a worker's row) and writes
// the selected entries there, with coordinates of the worker's whole row.  Flat launch over map_emit.
__global__ __launch_bounds__(kWG) void k_topk_emit(const float* __restrict__ e, Geometry geo, TopkWorkspace ws,
                                                    TopkOptions opt) {
  if (blockIdx.x == 0 && threadIdx.x == 0) ws.flags[0] = 0;  // the general kernels have run
  const WgSlot slot = ws.map_emit[blockIdx.x];
  const Seg sg = ws.segs[slot.seg];
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  const uint32_t c = slot.group + wave;
  if (c >= sg.num_chunks) return;  // wave-uniform; no barrier in this kernel
  TopkRow* rowp = ws.rows + slot.seg;
  if (c == 0 && lane == 0) {  // the next step's first pass allocates its list from the start
    rowp->cursor = 0;
    rowp->cursor_band = 0;
  }
  const uint32_t cap = opt.cap < sg.cap ? opt.cap : sg.cap;
  const uint32_t r = rowp->r, tau = rowp->tau, mode = rowp->mode;
  const uint4 rec = ws.chunk_rec[sg.chunk_base + c];
  const uint2* blk = ws.blk + static_cast<size_t>(slot.seg) * kMaxCountBlocks;
  const uint32_t my_block = c / sg.count_cpw;
  uint2 part = make_uint2(0, 0);
  for (uint32_t b = lane; b < my_block; b += 64) {
    const uint2 t = blk[b];
    part.x += t.x;
    part.y += t.y;
  }
  const bool all_ties = rowp->r == rowp->ties;
  const bool fast = uniform_u32(rowp->fast) != 0;
  uint32_t gt_before = wave_sum(part.x) + rec.z;
  const uint32_t eq_before = wave_sum(part.y) + rec.w;
  uint32_t gt_here = rec.x;
  uint32_t r_pos = r;
  if (fast) {  // selected by k_topk_band: see the last kernel
    const uint32_t a = ws.bnd_sel[static_cast<size_t>(slot.seg) * kBoundaryCap + lane];
    const uint32_t lo_c = c * kChunk, hi_c = lo_c + kChunk;
    gt_before += popc64(ballot64(a < lo_c));
    gt_here += popc64(ballot64(a >= lo_c && a < hi_c));
    r_pos = 0;
  }
  const uint32_t taken_before = eq_before < r_pos ? eq_before : r_pos;
  const uint32_t quota = r_pos - taken_before;
  const uint32_t take_here = rec.y < quota ? rec.y : quota;
  const uint32_t at = gt_before + taken_before;
  const uint32_t hi = at + gt_here + take_here;
  if (lane == 0) {
    uint32_t* so = ws.sel_off + sg.seloff_base;
    so[c] = at;
    if (c + 1 == sg.num_chunks) so[c + 1] = hi;
  }
  if (hi == at || sg.micro) return;  // a micro problem's entries were written by the first pass
  emit_chunk(mode, e + sg.elem_off, sg.d, c, ws.cand + sg.cand_base, ws.desc[sg.chunk_base + c], cap, tau, r, all_ties,
             eq_before, at, ws.idx + sg.list_base, ws.val + sg.list_base, sg.k, sg.coord_base, fast, rowp->tie_last);
  (void)geo;
}

// Where each chunk's slice of a worker's ascending coordinate list starts: sel_off[c] = number of listed
// coordinates below c * kChunk, for c = 0 .. num_chunks.  The thread of entry q fills the chunks between its
// predecessor's chunk (exclusive) and its own (inclusive); the last entry also fills the rest up to num_chunks.
__global__ __launch_bounds__(kWG) void k_topk_list_offsets(Geometry geo, TopkWorkspace ws) {
  const uint32_t row = blockIdx.y;
  const int32_t* idx = ws.idx + static_cast<size_t>(row) * geo.k;
  uint32_t* so = ws.sel_off_srv + static_cast<size_t>(row) * (geo.num_chunks + 1);
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < geo.k; q += step) {
    uint32_t cur = static_cast<uint32_t>(idx[q]) / kChunk;
    if (cur >= geo.num_chunks) cur = geo.num_chunks - 1;  // a coordinate beyond d (flagged by the unpacking)
    uint32_t from = 0;
    if (q) {
      uint32_t prev = static_cast<uint32_t>(idx[q - 1]) / kChunk;
      if (prev >= geo.num_chunks) prev = geo.num_chunks - 1;
      from = prev + 1;
    }
    for (uint32_t c = from; c <= cur; ++c) so[c] = q;
    if (q + 1 == geo.k)
      for (uint32_t c = cur + 1; c <= geo.num_chunks; ++c) so[c] = geo.k;
  }
}

// The residual at the coordinates selected in the last step becomes zero (the worker's error update of
// Algorithm 2 for the kept coordinates), applied on request.
__global__ __launch_bounds__(kWG) void k_topk_apply_clear(float* __restrict__ e, Geometry geo, TopkWorkspace ws) {
  const uint32_t row = blockIdx.y;
  float* er = e + static_cast<int64_t>(row) * geo.ld;
  const int32_t* idx = ws.idx + static_cast<size_t>(row) * geo.k;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < geo.k; q += step) {
    const uint32_t j = static_cast<uint32_t>(idx[q]);
    if (j < geo.d) er[j] = 0.0f;
  }
}

}  // namespace

#define COMPAMS_CHECK_LAUNCH()                    \
  do {                                            \
    hipError_t err__ = hipGetLastError();         \
    if (err__ != hipSuccess) return err__;        \
  } while (0)

hipError_t topk_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                     const float* g, float* e, float* theta, float* m, float* v, float* vhat,
                     bool first_pass_may_predict, bool clear_pending, bool workers_only, hipStream_t stream,
                     Launcher* L) {
  const int role = workers_only ? kWorkerHalf : kWholeStep;
  const uint32_t G = groups_per_row(geo.n, geo.num_chunks);
  const dim3 grid_rows(G, geo.n), wg(kWG);
  const uint32_t use_guess = first_pass_may_predict ? 1u : 0u;
  const dim3 grid_chunks(geo.num_chunks, geo.n);
  if (clear_pending)
    launch(L, kSlotPassA, k_topk_lean<true, true>, grid_chunks, wg, stream, g, e, geo, ws, opt, use_guess);
  else
    launch(L, kSlotPassA, k_topk_lean<false, true>, grid_chunks, wg, stream, g, e, geo, ws, opt, use_guess);
  COMPAMS_CHECK_LAUNCH();
  // the selection in one launch for the rows whose threshold lies in the band; it clears the rows' "fast" mark
  // otherwise, so it runs in every step (about a microsecond when it has nothing to do)
  const uint32_t count_blocks = (geo.num_chunks + geo.count_cpw - 1) / geo.count_cpw;  // <= kMaxCountBlocks
  launch(L, kSlotBand, k_topk_band<true>, dim3(count_blocks, geo.n), wg, stream, geo, ws, opt, use_guess);
  COMPAMS_CHECK_LAUNCH();
  {
    // about two workgroups per compute unit over all rows: each clears and flushes a whole histogram, and the
    // lists are short (measured on the headline workload: 37 us with 128 workgroups per row, 23 us with 32)
    uint32_t g0 = (512 + geo.n - 1) / geo.n;
    g0 = g0 > G ? G : g0;
    launch(L, kSlotLevel0, k_topk_level0<true>, dim3(g0, geo.n), wg, stream, e, geo, ws, opt, use_guess);
  }
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotLevel1, k_topk_level1<true>, grid_rows, wg, stream, e, geo, ws, opt);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotLevel2, k_topk_level2<true>, grid_rows, wg, stream, e, geo, ws, opt);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotCount, k_topk_count<true>, dim3(count_blocks, geo.n), wg, stream, e, geo, ws, opt);
  COMPAMS_CHECK_LAUNCH();
  const dim3 grid_f(geo.num_chunks);
  const TopkFlat none{};
#define COMPAMS_FINAL_WHOLE_ROW(NC) k_topk_final<kWholeStep, true, NC>
  if (role == kWorkerHalf)
    launch(L, kSlotTopkFinal, k_topk_final<kWorkerHalf, true, 0>, grid_f, wg, stream, theta, m, v, vhat, e, geo, ws, opt,
           ap, none);
  else
    COMPAMS_LAUNCH_BY_CACHED(ap.cached_arrays, L, kSlotTopkFinal, COMPAMS_FINAL_WHOLE_ROW, grid_f, wg, stream, theta, m, v,
                             vhat, e, geo, ws, opt, ap, none);
#undef COMPAMS_FINAL_WHOLE_ROW
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

// Top-k inside every block: the same kernels over segments (flat launches), then the lists are complete and
// the server's lines run from them.
hipError_t topk_blocks_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                            const TopkFlat& flat, const float* g, float* e, float* theta, float* m, float* v,
                            float* vhat, bool first_pass_may_predict, bool clear_pending, bool workers_only,
                            hipStream_t stream, Launcher* L) {
  const dim3 wg(kWG);
  const uint32_t use_guess = first_pass_may_predict ? 1u : 0u;
  if (clear_pending)
    launch(L, kSlotPassA, k_topk_lean<true, false>, dim3(flat.wg_first), wg, stream, g, e, geo, ws, opt, use_guess);
  else
    launch(L, kSlotPassA, k_topk_lean<false, false>, dim3(flat.wg_first), wg, stream, g, e, geo, ws, opt, use_guess);
  COMPAMS_CHECK_LAUNCH();
  if (flat.wg_count) {
    launch(L, kSlotBand, k_topk_band<false>, dim3(flat.wg_count), wg, stream, geo, ws, opt, use_guess);
    COMPAMS_CHECK_LAUNCH();
  }
  if (flat.wg_level0) {
    launch(L, kSlotLevel0, k_topk_level0<false>, dim3(flat.wg_level0), wg, stream, e, geo, ws, opt, use_guess);
    COMPAMS_CHECK_LAUNCH();
  }
  if (flat.wg_sweep) {  // none if every block is a micro problem
    launch(L, kSlotLevel1, k_topk_level1<false>, dim3(flat.wg_sweep), wg, stream, e, geo, ws, opt);
    COMPAMS_CHECK_LAUNCH();
    launch(L, kSlotLevel2, k_topk_level2<false>, dim3(flat.wg_sweep), wg, stream, e, geo, ws, opt);
    COMPAMS_CHECK_LAUNCH();
    launch(L, kSlotCount, k_topk_count<false>, dim3(flat.wg_count), wg, stream, e, geo, ws, opt);
    COMPAMS_CHECK_LAUNCH();
  }
  if (workers_only) {
    launch(L, kSlotTopkEmit, k_topk_emit, dim3(flat.wg_emit), wg, stream, e, geo, ws, opt);
  } else {
    const float* residuals = e;
    const dim3 grid_f(flat.wg_final);
#define COMPAMS_FINAL_BLOCKS(NC) k_topk_final<kWholeStep, false, NC>
    COMPAMS_LAUNCH_BY_CACHED(ap.cached_arrays, L, kSlotTopkFinal, COMPAMS_FINAL_BLOCKS, grid_f, wg, stream, theta, m, v, vhat,
                             residuals, geo, ws, opt, ap, flat);
#undef COMPAMS_FINAL_BLOCKS
  }
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

// The server's lines from lists that sit in the workspace (idx, val: n ascending lists of k entries).
hipError_t topk_server_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                            float* theta, float* m, float* v, float* vhat, hipStream_t stream, Launcher* L) {
  uint32_t groups = (geo.k + kWG * 4 - 1) / (kWG * 4);
  if (groups > 256) groups = 256;
  launch(L, kSlotTopkOffsets, k_topk_list_offsets, dim3(groups, geo.n), dim3(kWG), stream, geo, ws);
  COMPAMS_CHECK_LAUNCH();
  const float* no_e = nullptr;
  const dim3 grid_f(geo.num_chunks), wg(kWG);
  const TopkFlat none{};
#define COMPAMS_FINAL_SERVER(NC) k_topk_final<kServerHalf, true, NC>
  COMPAMS_LAUNCH_BY_CACHED(ap.cached_arrays, L, kSlotTopkFinal, COMPAMS_FINAL_SERVER, grid_f, wg, stream, theta, m, v, vhat,
                           no_e, geo, ws, opt, ap, none);
#undef COMPAMS_FINAL_SERVER
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t topk_apply_clear(const Geometry& geo, const TopkWorkspace& ws, float* e, hipStream_t stream) {
  uint32_t blocks = (geo.k + kWG - 1) / kWG;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(k_topk_apply_clear, dim3(blocks, geo.n), dim3(kWG), 0, stream, e, geo, ws);
  return hipGetLastError();
}

}  // namespace compams
