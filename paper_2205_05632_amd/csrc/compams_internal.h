// Internal declarations shared by the kernel files and the C-ABI host code of libcompams.
// Nothing here is part of the public interface (include/compams.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace compams {

// ---------------------------------------------------------------------------------------------
// Geometry shared by all kernels.
//
// A row (one worker's d coordinates) is cut into chunks of kChunk consecutive coordinates, a chunk into
// kRounds rounds of 256 coordinates; in a round lane l of a wavefront holds the four coordinates
// base + 256*round + 4*l + {0,1,2,3}, so that a wave's 128-bit accesses cover 1 KiB of contiguous memory and
// (round, lane, slot) order is ascending coordinate order.  The dense passes give a chunk to a workgroup
// (a quarter of its rounds to each wavefront), the sweeps over stored rows and lists a chunk to a wavefront.
// ---------------------------------------------------------------------------------------------
constexpr int kWG = 256;                 // threads per workgroup = 4 wavefronts
constexpr int kWaves = kWG / 64;
constexpr int kChunk = 4096;             // coordinates per chunk
constexpr int kRounds = kChunk / 256;    // rounds per chunk

// Radix levels over the 31-bit magnitude key (fp32 bit pattern without the sign):
// level 0 = bits 30..19 (the exponent and 4 mantissa bits), level 1 = bits 18..9, level 2 = bits 8..0.
constexpr int kL0Shift = 19;
constexpr int kNB0 = 1 << 12;
constexpr int kL1Shift = 9;
constexpr int kNB1 = 1 << 10;
constexpr int kNB2 = 1 << 9;
// The level-0 kernel keeps level-1 histograms of this many buckets, starting at the guessed one: the guess is one
// below the last threshold bucket, so a threshold that moved by one bucket either way still resolves there.
constexpr uint32_t kTracked = 3;
// Top-k inside every block: a block of at most this many coordinates (a bias, a norm weight) is one wavefront's
// work from reading g to writing its part of the list; it takes no part in histograms, sweeps or counting.
constexpr uint32_t kMicroCoords = 1024;
constexpr uint32_t kMicroFlag = 0x80000000u;  // WgSlot.seg of a first-pass workgroup that takes micro problems

// The counting kernel splits a row's chunks into at most kMaxCountBlocks contiguous blocks of count_cpw chunks
// (a multiple of 32: four wavefronts, eight chunks at a time).  d < 2^31 gives at most 2^19 chunks.
constexpr uint32_t kMaxCountBlocks = 256;
constexpr uint32_t kMaxCountCpw = 2048;
inline uint32_t count_chunks_per_block(uint32_t num_chunks) {
  const uint32_t m = (num_chunks + 32 * kMaxCountBlocks - 1) / (32 * kMaxCountBlocks);
  return 32 * (m ? m : 1);
}

// The candidate list of a selection problem is kept as kSubLists runs, chunk c of the problem appending to run
// c % kSubLists, each run with a cursor in a 128-byte line of its own.  Atomics to one address are performed one
// after the other (about 3 ns apart on MI355X); a chunk's allocation every 8 ns through a single cursor queued long
// enough to cost the first pass 9 of 352 us, and cursors that share a line were little better.
constexpr uint32_t kSubLists = 8;
constexpr uint32_t kCursorPitch = 32;  // words between the cursors of a problem
// A problem (row or block) of fewer chunks than this keeps its list as one run: its allocations are few, and
// with a handful of chunks the runs would be of very different lengths and an eighth of the capacity each
// would overflow for nothing.
constexpr uint32_t kSubListMinChunks = 64;
constexpr uint32_t kNoCursorSet = 0xffffffffu;

constexpr uint32_t kCountersPerRow = 8;  // == COMPAMS_COUNTERS_PER_ROW of the public header

constexpr int kWireTile = 256;  // coordinate gaps per tile of a top-k message (one width per tile)

// Where a row's selection reads its elements from after level 0.
enum : uint32_t {
  kModeCand = 0,   // candidate list written by the first pass (threshold bucket was predicted)
  kModeNeedB = 1,  // candidate list written by a second dense pass that knows the exact level-0 bucket
  kModeDense = 2   // no candidate list (it would not fit): every later pass reads the whole row
};

// The band: a window of magnitude keys [band_lo, band_hi) in which the next step's threshold key is expected,
// set from the last two thresholds, cut into kBandBuckets buckets of equal width (band_bucket below).  The first pass counts, per
// chunk, the entries at or above band_hi, copies the entries inside the window to a short list of their own (a
// segment per chunk) and adds them to the row's bucket histogram.  If the threshold does fall inside (checked
// exactly), one launch finishes the selection from the short list alone (k_topk_band).
constexpr uint32_t kBandBuckets = 2048;
constexpr uint32_t kBandMaxEntries = 1u << 20;  // capacity of a band list at most
constexpr uint32_t kBoundaryCap = 64;      // entries in the bucket that holds the threshold key; more: general route
constexpr uint32_t kCursorAboveWord = 2;   // word of a run's cursor line that counts the run's entries above the band

// Per-row control block of the top-k selection (device memory, written by single workgroups).
struct TopkRow {
  uint32_t pred_valid;  // the next first pass may emit candidates with level-0 bucket >= b_guess
  uint32_t b_guess;
  uint32_t cursor;      // candidate entries allocated so far in this step (a list kept as one run) ...
  uint32_t cursor_band; // ... and band entries: the two are advanced together as one 64-bit word
  uint32_t band_valid;  // the next first pass may also fill the band list and the bucket histogram
  uint32_t band_lo, band_hi;  // keys; band_lo >= b_guess << kL0Shift, band_hi > band_lo
  uint32_t band_mul;    // bucket of a key inside the band: see band_bucket()
  uint32_t fast;        // this step's threshold was found in the band: the general kernels skip the problem
  uint32_t mode;        // kMode*
  uint32_t n_src;       // entries in the candidate list (kModeCand / kModeNeedB)
  uint32_t bstar;       // level-0 bucket that holds the k-th largest key
  uint32_t need;        // keys still to be taken inside the current prefix
  uint32_t prefix1;     // bits 30..9 of the k-th largest key (after level 1)
  uint32_t tau;         // the k-th largest key
  uint32_t r;           // how many keys equal to tau are selected
  uint32_t ties;        // how many keys equal tau
  uint32_t level1_done;    // bits 30..9 of the threshold key are known (prefix1 / need are valid)
  uint32_t ticket[4];      // "last workgroup of the row" counters of kernels 1..4; zero between launches
  uint32_t n_lists;        // runs of the candidate list: kSubLists (run s from entry s * (capacity / kSubLists) on), or 1
  uint32_t n_sub[kSubLists];  // entries of each run (n_src in all)
  uint32_t tie_last;       // fast: ties are taken up to and including this coordinate (of the problem)
  uint32_t tau_prev;       // the threshold key of the step before (0: none)
  uint32_t above;          // entries at or above band_hi (a list kept as one run; else in the runs' cursor lines)
  uint32_t bnd_n;          // entries of the threshold's bucket gathered so far (k_topk_band); zero between launches
  uint32_t bnd_kept;       // fast: how many of them are kept; their coordinates, ascending, are in bnd_sel
  uint32_t ticket_band;    // "last workgroup" counter of k_topk_band; zero between launches
  uint32_t pad[27];
};
static_assert(sizeof(TopkRow) == 256, "TopkRow layout");

// Bucket of a key inside a band of `span` keys starting at lo: floor(rel * kBandBuckets / span) for rel = key - lo,
// computed as the high word of rel * mul with mul = floor(2^32 * kBandBuckets / span); a band of at most kBandBuckets
// keys (mul = 0) has a bucket per key.  Non-decreasing in the key and always below kBandBuckets.
inline uint32_t band_multiplier(uint32_t span) {
  return span > kBandBuckets ? static_cast<uint32_t>((static_cast<uint64_t>(kBandBuckets) << 32) / span) : 0u;
}
__device__ __forceinline__ uint32_t band_multiplier_dev(uint32_t span) {
  return span > kBandBuckets ? static_cast<uint32_t>((static_cast<uint64_t>(kBandBuckets) << 32) / span) : 0u;
}
__device__ __forceinline__ uint32_t band_bucket(uint32_t rel, uint32_t mul) { return mul ? __umulhi(rel, mul) : rel; }

// One selection problem: a worker's whole row (top-k over the flattened gradient) or one block of a worker's
// row (top-k inside every block).  Index fields count entries of the respective workspace tables.
struct Seg {
  int64_t elem_off;      // first element, relative to the start of g and of e
  uint64_t chunk_base;   // first entry in the per-chunk tables (segment descriptors, count records)
  uint64_t seloff_base;  // first entry in sel_off (a segment has one entry more than it has chunks)
  uint64_t cand_base;    // first entry of the segment's candidate list
  uint64_t list_base;    // first entry of the segment's slice of the worker's (coordinate, value) list
  uint64_t band_base;    // first entry of the segment's band list
  uint32_t d, k;         // length, and how many coordinates are kept
  uint32_t num_chunks;
  uint32_t cap;          // capacity of the candidate list
  uint32_t band_cap;     // capacity of the band list
  uint32_t coord_base;   // coordinate of the first element within the worker's row
  uint32_t count_cpw;    // chunks per block of the counting kernel
  uint32_t groups_first, groups_sweep, count_blocks;  // workgroups the kernel classes give this segment (first pass:
                                                      // one per chunk)
  uint32_t micro;        // at most kMicroCoords coordinates: one wavefront of the first pass does the whole selection
  uint32_t groups_level0;
  uint32_t cursor_set;   // which set of kSubLists cursors the problem's list uses, or kNoCursorSet: one run, rowp->cursor
};
static_assert(sizeof(Seg) % 8 == 0, "Seg layout");

// Which segment, and which of its workgroups, a workgroup of a flat launch is.
struct WgSlot {
  uint32_t seg, group;
};

struct TopkOptions {
  uint32_t cap;            // candidate entries per row
  uint32_t predict;        // 1: carry the threshold bucket over to the next step's first pass
  uint32_t force_dense;    // 1: never build a candidate list (test / ablation)
  uint32_t band;           // 1: also carry a window for the threshold key itself over (k_topk_band)
  uint32_t band_cap;       // band entries per row
};

struct TopkWorkspace {
  TopkRow* rows;        // n
  uint32_t* counters;   // n * COMPAMS_COUNTERS_PER_ROW
  uint32_t* hist0;      // n * kNB0
  uint32_t* hist1;      // n * kNB1
  uint32_t* hist1x;     // n * kTracked * kNB1 : level-1 histograms of the tracked buckets
  uint32_t* hist2;      // n * kNB2
  uint32_t* xcur;       // sets of kSubLists cursors, kCursorPitch words apart: one set per row, or per segment of at
                        // least kSubListMinChunks chunks
  uint4* chunk_rec;     // n * num_chunks : keys above tau, keys equal to tau, and the exclusive prefixes of both
                        //                  within the chunk's count block
  uint2* blk;           // n * kMaxCountBlocks : the two totals of every count block
  uint2* blk_prefix;    // n * kMaxCountBlocks : for a problem selected by k_topk_band, the totals of the blocks
                        // before each block (the sums the last kernel would otherwise form per chunk)
  uint32_t* sel_off;    // n * (num_chunks + 1) : where each chunk's slice of the worker's list starts
  uint32_t* count_gt;   // n : selected entries whose key lies strictly above the threshold key
  uint32_t* wire_total;    // n : words of the gap stream of the message being packed or unpacked
  uint32_t* wire_tile_off; // n * ceil(k / kWireTile) : where each tile of gaps starts in its stream
  uint32_t* wire_tile_sum; // n * ceil(k / kWireTile) : coordinates before each tile, while unpacking
  uint2* desc;          // n * num_chunks : (offset, count) of the chunk's segment in the candidate list
  uint2* desc2;         // n * num_chunks : offset of the chunk's segment in the band list; entries at or above the
                        //                  band | entries in the band << 13 | kBandChunkOverflow
  uint2* band;          // n * band_cap   : (coordinate, fp32 bits) of the entries inside the band
  uint32_t* bhist;      // n * kBandBuckets : how many band entries fall into each bucket; zero between steps
  uint2* bnd;           // n * kBoundaryCap : the entries of the bucket that holds the threshold key
  uint32_t* bnd_sel;    // n * kBoundaryCap : coordinates of the kept ones among them, ascending
  uint32_t* flags;      // [0]: some problem of this step was left to the general kernels (set by k_topk_band, cleared
                        //      by the step's last kernel): the general kernels return at once otherwise
  uint2* cand;          // n * cap_alloc  : (coordinate, fp32 bits)
  int32_t* idx;         // n * k
  float* val;           // n * k
  uint32_t* tau;        // n
  // top-k inside every block only: the segments and, per kernel class, the workgroups of a flat launch
  const Seg* segs;
  const WgSlot* map_first;   // first pass: .group = chunk of the segment (or a workgroup of micro problems, see below)
  const WgSlot* map_level0;
  const WgSlot* map_sweep;
  const WgSlot* map_count;
  const WgSlot* map_emit;   // .group = first chunk of the four that the workgroup's wavefronts take
  const uint32_t* micro_list;  // segments that are micro problems; a first-pass workgroup with kMicroFlag takes
                               // .group (<= 4) of them, from entry (.seg without the flag) on, one per wavefront
  const WgSlot* map_final;  // .seg = block (worker 0's segment of it), .group = chunk of the block
  uint32_t* sel_off_srv;    // n * (chunks of a whole row + 1) : list offsets per chunk of coordinates, for the
                            //                                   server's lines run from lists
};

struct BlocksignWorkspace {
  uint32_t* offsets;    // M + 1 block offsets
  uint32_t* chunk_block; // num_chunks : index of the block that holds the chunk's first coordinate
  uint64_t* acc;        // n * M * acc_replicas * kLimbs : exact sums of |x| (32-bit digits carried in 64-bit words);
                        // the sum of a (row, block) is the sum of its replicas
  uint32_t acc_replicas;
  uint32_t* special;    // n * M : bit 0 = an infinity was seen, bit 1 = a NaN was seen
  float* scales;        // n * M
  uint32_t* bits;       // n * words
};
constexpr int kLimbs = 10;  // 10 digits of 32 bits cover 2^-149 .. 2^171

struct AmsParams {
  float beta1, beta2, one_minus_beta1, one_minus_beta2, eps, lr, nf;
  int eps_out;  // 1: epsilon outside the square root
  int cached_arrays;  // how many of theta, m, v, vhat (in that order) fit the memory-side cache together from one
                      // step to the next: those are read and written with ordinary accesses, the others with
                      // streaming ones (measured, final kernel of the top-k step: ResNet-18, 4 x 45 MB, all four
                      // cached 70 against 87 us; ResNet-50, 4 x 102 MB, none 174, one 147, two 144, three 175 us;
                      // GPT-2, 4 x 498 MB, none is best)
};

// The memory-side cache holds 256 MB; what the first pass streams through in between costs some of it.
inline int cached_state_arrays(int64_t d) {
  const int64_t budget = int64_t(212) << 20, each = d * 4;
  const int64_t fit = budget / each;
  return fit > 4 ? 4 : static_cast<int>(fit);
}

// Moment and parameter lines of Algorithm 2 for one coordinate: every product, sum, square root and
// quotient is a separately rounded fp32 operation (the library is built without contraction).
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

struct Geometry {
  uint32_t n;
  uint32_t d;
  int64_t ld;
  uint32_t num_chunks;
  uint32_t k;
  uint32_t num_blocks;
  uint32_t words;  // ceil(d / 32)
  uint32_t count_cpw;  // top-k: chunks per block of the counting kernel
};

// Kernel slots for optional timing.
enum KernelSlot {
  kSlotPassA = 0, kSlotBand, kSlotLevel0, kSlotLevel1, kSlotLevel2, kSlotCount, kSlotTopkFinal, kSlotTopkEmit, kSlotTopkOffsets,
  kSlotBsPass1, kSlotBsFinal, kSlotBsPass2, kSlotBsAms,
  kSlotNoneAms, kSlotWireEncode, kSlotWireDecode, kNumSlots
};

struct Launcher;  // host-side helper that brackets launches with events (compams_api.hip)

// Host-side launch entry points, one per compressor (defined next to their kernels).
hipError_t topk_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                     const float* g, float* e, float* theta, float* m, float* v, float* vhat,
                     bool first_pass_may_predict, bool clear_pending, bool workers_only, hipStream_t stream,
                     Launcher* L);
// Sizes of the flat launches of top-k inside every block.
struct TopkFlat {
  uint32_t wg_first, wg_level0, wg_sweep, wg_count, wg_emit, wg_final;
  // from worker i's segment of a block to worker i + 1's: segment index, chunk tables, list offsets, candidates
  uint32_t blocks, chunk_stride, seloff_stride;
  uint64_t cand_stride, band_stride;
};
hipError_t topk_blocks_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                            const TopkFlat& flat, const float* g, float* e, float* theta, float* m, float* v,
                            float* vhat, bool first_pass_may_predict, bool clear_pending, bool workers_only,
                            hipStream_t stream, Launcher* L);
hipError_t topk_server_step(const Geometry& geo, const TopkWorkspace& ws, const TopkOptions& opt, const AmsParams& ap,
                            float* theta, float* m, float* v, float* vhat, hipStream_t stream, Launcher* L);
hipError_t topk_apply_clear(const Geometry& geo, const TopkWorkspace& ws, float* e, hipStream_t stream);
hipError_t blocksign_step(const Geometry& geo, const BlocksignWorkspace& ws, const AmsParams& ap, const float* g,
                          float* e, float* theta, float* m, float* v, float* vhat, bool residual_pending,
                          bool workers_only, hipStream_t stream, Launcher* L);
hipError_t blocksign_server_step(const Geometry& geo, const BlocksignWorkspace& ws, const AmsParams& ap, float* theta,
                                 float* m, float* v, float* vhat, hipStream_t stream, Launcher* L);
hipError_t blocksign_apply_residual(const Geometry& geo, const BlocksignWorkspace& ws, float* e, hipStream_t stream);
hipError_t none_step(const Geometry& geo, const AmsParams& ap, const float* g, float* theta, float* m, float* v,
                     float* vhat, hipStream_t stream, Launcher* L);
hipError_t wire_encode_topk(const Geometry& geo, const TopkWorkspace& ws, uint32_t* messages, int64_t stride,
                            uint32_t* words_out, hipStream_t stream, Launcher* L);
hipError_t wire_decode_topk(const Geometry& geo, const TopkWorkspace& ws, const uint32_t* messages, int64_t stride,
                            const uint32_t* words, int32_t* idx_out, float* val_out, uint32_t* status,
                            hipStream_t stream, Launcher* L);
hipError_t wire_encode_blocksign(const Geometry& geo, const BlocksignWorkspace& ws, uint32_t* messages, int64_t stride,
                                 uint32_t* words_out, hipStream_t stream, Launcher* L);
hipError_t wire_decode_blocksign(const Geometry& geo, const uint32_t* messages, int64_t stride, const uint32_t* words,
                                 uint32_t* bits_out, float* scales_out, uint32_t* status, hipStream_t stream,
                                 Launcher* L);
hipError_t fill_u32(uint32_t* p, size_t count, uint32_t value, hipStream_t stream);
hipError_t fill_rows_f32(float* p, uint32_t n, int64_t ld, uint32_t d, float value, hipStream_t stream);
hipError_t copy_u32(uint32_t* dst, const uint32_t* src, size_t count, hipStream_t stream);
hipError_t stream_copy(void* dst, const void* src, size_t bytes, hipStream_t stream);
hipError_t inplace_probe(float* const* arrays, int n_arrays, size_t count, int cached_arrays, hipStream_t stream);

// Launch with optional timing: when the slot is being timed, the launch is bracketed by a pair of events on
// the same stream.  (Events attached to the dispatch itself give the same durations but slow the step down
// by more than the bracketing does; measured on MI355X.)
void launcher_begin(Launcher* L, int slot, hipStream_t stream);
void launcher_end(Launcher* L, int slot, hipStream_t stream);

template <typename... KArgs, typename... Args>
inline void launch(Launcher* L, int slot, void (*kernel)(KArgs...), const dim3& grid, const dim3& block,
                   hipStream_t stream, Args... args) {
  if (L) launcher_begin(L, slot, stream);
  hipLaunchKernelGGL(kernel, grid, block, 0, stream, static_cast<KArgs>(args)...);
  if (L) launcher_end(L, slot, stream);
}

// A kernel template over the number of cached state arrays (0..4), picked at run time.
#define COMPAMS_LAUNCH_BY_CACHED(nc, L, slot, KERNEL, ...)                      \
  do {                                                                          \
    switch (nc) {                                                               \
      case 0: launch(L, slot, KERNEL(0), __VA_ARGS__); break;                   \
      case 1: launch(L, slot, KERNEL(1), __VA_ARGS__); break;                   \
      case 2: launch(L, slot, KERNEL(2), __VA_ARGS__); break;                   \
      case 3: launch(L, slot, KERNEL(3), __VA_ARGS__); break;                   \
      default: launch(L, slot, KERNEL(4), __VA_ARGS__); break;                  \
    }                                                                           \
  } while (0)

// How many workgroups per row the streaming kernels use: enough to keep 256 compute units busy
// with several workgroups each, whatever n is.
inline uint32_t groups_per_row(uint32_t n, uint32_t num_chunks) {
  const uint32_t target = 256 * 8;  // workgroups in flight over the whole grid
  uint32_t g = (target + n - 1) / n;
  const uint32_t max_g = (num_chunks + kWaves - 1) / kWaves;  // one chunk per wavefront at least
  if (g > max_g) g = max_g;
  if (g < 1) g = 1;
  return g;
}


}  // namespace compams
