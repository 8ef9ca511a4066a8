// Host side of libcompams: the C ABI declared in include/compams.h.
// Validates arguments, lays out the caller's workspace, and enqueues the kernels of one step.

#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "../../include/compams.h"
#include "compams_internal.h"

namespace compams {

struct Launcher {
  struct Pair { hipEvent_t a, b; };
  std::vector<Pair> pending[kNumSlots];
  std::vector<Pair> pool;
  double total_ms[kNumSlots];
  int64_t launches[kNumSlots];
  uint32_t mask;  // slots that are bracketed
  bool failed;
  Launcher() : mask(0), failed(false) {
    for (int i = 0; i < kNumSlots; ++i) { total_ms[i] = 0.0; launches[i] = 0; }
  }
};

void launcher_begin(Launcher* L, int slot, hipStream_t stream) {
  if (!(L->mask & (1u << slot))) return;
  Launcher::Pair p;
  if (!L->pool.empty()) {
    p = L->pool.back();
    L->pool.pop_back();
  } else if (hipEventCreate(&p.a) != hipSuccess || hipEventCreate(&p.b) != hipSuccess) {
    L->failed = true;
    return;
  }
  if (hipEventRecord(p.a, stream) != hipSuccess) L->failed = true;
  L->pending[slot].push_back(p);
}

void launcher_end(Launcher* L, int slot, hipStream_t stream) {
  if (!(L->mask & (1u << slot)) || L->pending[slot].empty()) return;
  if (hipEventRecord(L->pending[slot].back().b, stream) != hipSuccess) L->failed = true;
}

namespace {

const char* const kSlotNames[kNumSlots] = {
    "topk_pass_a", "topk_band", "topk_level0", "topk_level1", "topk_level2", "topk_count", "topk_final", "topk_emit", "topk_offsets",
    "bs_pass1", "bs_finalize", "bs_pass2", "bs_amsgrad", "none_amsgrad", "wire_encode", "wire_decode"};

static_assert(kCountersPerRow == COMPAMS_COUNTERS_PER_ROW, "the kernels' stride of the counters is the header's");

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

struct Layout {
  size_t total;
  // top-k
  size_t rows, flags, counters, hist0, hist1, hist1x, hist2, bhist, xcur, chunk_rec, blk, blk_prefix, sel_off, desc, desc2, bnd, bnd_sel, cand, band,
      idx, val, tau, count_gt, wire_total, wire_tile_off, wire_tile_sum, sel_off_srv, segs, map_first, map_level0, map_sweep,
      map_count, map_emit, map_final, micro_list;
  // block-sign
  size_t offsets, chunk_block, acc, special, scales, bits;
  uint32_t acc_replicas;
  uint32_t cap_alloc, band_alloc, num_chunks, words;
  // top-k inside every block
  uint64_t k_total;
  size_t num_micro;  // selection problems taken by single wavefronts (top-k per block)
  TopkFlat flat;
};

bool blocks_valid(const compams_config* c) {
  const int64_t* o = c->block_offsets;
  if (c->num_blocks < 1 || c->num_blocks > c->d || !o || o[0] != 0 || o[c->num_blocks] != c->d) return false;
  for (int64_t b = 0; b < c->num_blocks; ++b)
    if (o[b + 1] <= o[b]) return false;
  return true;
}

bool basic_valid(const compams_config* c) {
  if (!c) return false;
  if (c->n < 1 || c->n > 65535 || c->d < 1 || c->d >= (int64_t(1) << 31)) return false;  // n is a grid dimension
  if (c->compressor != COMPAMS_NONE && c->compressor != COMPAMS_TOPK && c->compressor != COMPAMS_BLOCKSIGN &&
      c->compressor != COMPAMS_TOPK_BLOCKS)
    return false;
  if (c->compressor == COMPAMS_TOPK && (c->k < 1 || c->k > c->d)) return false;
  if (c->compressor == COMPAMS_BLOCKSIGN && (c->num_blocks < 1 || c->num_blocks > c->d)) return false;
  if (c->compressor == COMPAMS_TOPK_BLOCKS) {  // its workspace depends on the blocks: they are checked here already
    if (!blocks_valid(c) || !c->block_k) return false;
    for (int64_t b = 0; b < c->num_blocks; ++b)
      if (c->block_k[b] < 1 || c->block_k[b] > c->block_offsets[b + 1] - c->block_offsets[b]) return false;
  }
  return true;
}

// Top-k inside every block: the shape of one block's selection problem and how many workgroups it gets.
struct BlockShape {
  uint32_t off, d, k, nc, cap, band_cap, cpw, groups_first, groups_level0, groups_sweep, count_blocks, emit_slots, micro;
};

// Entries of a problem's band list: the window around the expected threshold holds a fraction of k.
uint32_t band_capacity(uint64_t k, uint32_t cap) {
  uint64_t want = k + 4096;
  if (want > kBandMaxEntries) want = kBandMaxEntries;
  return want > cap ? cap : static_cast<uint32_t>(want);
}

std::vector<BlockShape> block_shapes(const compams_config* c) {
  const size_t M = static_cast<size_t>(c->num_blocks);
  std::vector<BlockShape> v(M);
  uint64_t chunks_per_worker = 0;
  for (size_t b = 0; b < M; ++b) {
    BlockShape& s = v[b];
    s.off = static_cast<uint32_t>(c->block_offsets[b]);
    s.d = static_cast<uint32_t>(c->block_offsets[b + 1] - c->block_offsets[b]);
    s.k = static_cast<uint32_t>(c->block_k[b]);
    s.nc = (s.d + kChunk - 1) / kChunk;
    const uint64_t cap = 8ull * s.k + 8192;
    s.cap = cap > s.d ? s.d : static_cast<uint32_t>(cap);
    s.cpw = count_chunks_per_block(s.nc);
    s.micro = s.d <= kMicroCoords ? 1u : 0u;
    s.band_cap = s.micro ? 0u : band_capacity(s.k, s.cap);
    s.count_blocks = (s.nc + s.cpw - 1) / s.cpw;
    s.emit_slots = (s.nc + kWaves - 1) / kWaves;
    chunks_per_worker += s.nc;
  }
  // the first pass takes a workgroup per chunk; about 512 workgroups find the threshold buckets and 2048 make the
  // sweeps over all workers, at least one per problem
  const uint64_t all = chunks_per_worker * static_cast<uint64_t>(c->n);
  const uint32_t per_level0 = static_cast<uint32_t>(std::max<uint64_t>(8, (all + 511) / 512));
  const uint32_t per_sweep = static_cast<uint32_t>(std::max<uint64_t>(4, (all + 2047) / 2048));
  for (BlockShape& s : v) {
    const uint32_t most = (s.nc + kWaves - 1) / kWaves;  // one chunk per wavefront at least
    s.groups_first = s.nc;
    s.groups_level0 = std::max<uint32_t>(1, std::min<uint32_t>(most, (s.nc + per_level0 / 2) / per_level0));
    s.groups_sweep = std::max<uint32_t>(1, std::min<uint32_t>(most, (s.nc + per_sweep / 2) / per_sweep));
    // a micro problem is a wavefront of a shared workgroup of the first pass instead
    if (s.micro) s.groups_first = s.groups_level0 = s.groups_sweep = s.count_blocks = 0;
  }
  return v;
}

Layout make_layout(const compams_config* c) {
  Layout L;
  std::memset(&L, 0, sizeof L);
  const size_t n = static_cast<size_t>(c->n), d = static_cast<size_t>(c->d);
  L.num_chunks = static_cast<uint32_t>((d + kChunk - 1) / kChunk);
  L.words = static_cast<uint32_t>((d + 31) / 32);
  const size_t nc = L.num_chunks;
  size_t at = 0;
  auto take = [&](size_t bytes) { const size_t o = at; at = align_up(at + bytes, 256); return o; };
  if (c->compressor == COMPAMS_TOPK) {
    const size_t k = static_cast<size_t>(c->k);
    size_t cap = 8 * k + 65536;
    if (cap > d) cap = d;
    L.cap_alloc = static_cast<uint32_t>(cap);
    L.band_alloc = band_capacity(k, L.cap_alloc);
    L.rows = take(n * sizeof(TopkRow));
    L.flags = take(64);
    L.counters = take(n * COMPAMS_COUNTERS_PER_ROW * 4);
    L.hist0 = take(n * kNB0 * 4);
    L.hist1 = take(n * kNB1 * 4);
    L.hist1x = take(n * kTracked * kNB1 * 4);
    L.hist2 = take(n * kNB2 * 4);
    L.bhist = take(n * kBandBuckets * 4);
    L.xcur = take(n * kSubLists * kCursorPitch * 4);
    L.chunk_rec = take(n * nc * 16);
    L.blk = take(n * kMaxCountBlocks * 8);
    L.blk_prefix = take(n * kMaxCountBlocks * 8);
    L.sel_off = take(n * (nc + 1) * 4);
    L.desc = take(n * nc * 8);
    L.desc2 = take(n * nc * 8);
    L.bnd = take(n * kBoundaryCap * 8);
    L.bnd_sel = take(n * kBoundaryCap * 4);
    L.cand = take(n * cap * 8);
    L.band = take(n * static_cast<size_t>(L.band_alloc) * 8);
    L.idx = take(n * k * 4);
    L.val = take(n * k * 4);
    L.tau = take(n * 4);
    L.count_gt = take(n * 4);
    L.wire_total = take(n * 4);
    L.wire_tile_off = take(n * ((k + kWireTile - 1) / kWireTile) * 4);
    L.wire_tile_sum = take(n * ((k + kWireTile - 1) / kWireTile) * 4);
    L.sel_off_srv = take(n * (nc + 1) * 4);
  } else if (c->compressor == COMPAMS_TOPK_BLOCKS) {
    const std::vector<BlockShape> shapes = block_shapes(c);
    const size_t M = shapes.size(), S = n * M;
    size_t k = 0, chunks = 0, caps = 0, bcaps = 0, wg_first = 0, wg_level0 = 0, wg_sweep = 0, wg_count = 0, wg_emit = 0, micro = 0,
           big = 0;
    uint32_t cap_max = 0, band_max = 0;
    for (const BlockShape& b : shapes) {
      k += b.k; chunks += b.nc; caps += b.cap; cap_max = std::max(cap_max, b.cap);
      bcaps += b.band_cap; band_max = std::max(band_max, b.band_cap);
      wg_first += b.groups_first; wg_level0 += b.groups_level0; wg_sweep += b.groups_sweep; wg_count += b.count_blocks; wg_emit += b.emit_slots;
      micro += b.micro;
      big += b.nc >= kSubListMinChunks ? 1 : 0;  // blocks whose candidate lists are kept as several runs
    }
    L.k_total = k;
    L.cap_alloc = cap_max;
    L.band_alloc = band_max;
    L.num_micro = n * micro;
    L.flat.wg_first = static_cast<uint32_t>(n * wg_first + (n * micro + kWaves - 1) / kWaves);
    L.flat.wg_level0 = static_cast<uint32_t>(n * wg_level0);
    L.flat.wg_sweep = static_cast<uint32_t>(n * wg_sweep);
    L.flat.wg_count = static_cast<uint32_t>(n * wg_count);
    L.flat.wg_emit = static_cast<uint32_t>(n * wg_emit);
    L.flat.wg_final = static_cast<uint32_t>(chunks);
    L.flat.band_stride = bcaps;
    L.flat.blocks = static_cast<uint32_t>(M);
    L.flat.chunk_stride = static_cast<uint32_t>(chunks);
    L.flat.seloff_stride = static_cast<uint32_t>(chunks + M);
    L.flat.cand_stride = caps;
    L.rows = take(S * sizeof(TopkRow));
    L.flags = take(64);
    L.counters = take(S * COMPAMS_COUNTERS_PER_ROW * 4);
    L.hist0 = take(S * kNB0 * 4);
    L.hist1 = take(S * kNB1 * 4);
    L.hist1x = take(S * kTracked * kNB1 * 4);
    L.hist2 = take(S * kNB2 * 4);
    L.bhist = take(S * kBandBuckets * 4);
    L.xcur = take(n * big * kSubLists * kCursorPitch * 4);
    L.chunk_rec = take(n * chunks * 16);
    L.blk = take(S * kMaxCountBlocks * 8);
    L.blk_prefix = take(S * kMaxCountBlocks * 8);
    L.sel_off = take(n * (chunks + M) * 4);
    L.desc = take(n * chunks * 8);
    L.desc2 = take(n * chunks * 8);
    L.bnd = take(S * kBoundaryCap * 8);
    L.bnd_sel = take(S * kBoundaryCap * 4);
    L.cand = take(n * caps * 8);
    L.band = take(n * bcaps * 8);
    L.idx = take(n * k * 4);
    L.val = take(n * k * 4);
    L.tau = take(S * 4);
    L.count_gt = take(S * 4);
    L.wire_total = take(n * 4);
    L.wire_tile_off = take(n * ((k + kWireTile - 1) / kWireTile) * 4);
    L.wire_tile_sum = take(n * ((k + kWireTile - 1) / kWireTile) * 4);
    L.sel_off_srv = take(n * (nc + 1) * 4);
    L.segs = take(S * sizeof(Seg));
    L.map_first = take(L.flat.wg_first * sizeof(WgSlot));
    L.map_level0 = take(L.flat.wg_level0 * sizeof(WgSlot));
    L.map_sweep = take(L.flat.wg_sweep * sizeof(WgSlot));
    L.map_count = take(L.flat.wg_count * sizeof(WgSlot));
    L.map_emit = take(L.flat.wg_emit * sizeof(WgSlot));
    L.map_final = take(L.flat.wg_final * sizeof(WgSlot));
    L.micro_list = take(L.num_micro * 4);
  } else if (c->compressor == COMPAMS_BLOCKSIGN) {
    const size_t M = static_cast<size_t>(c->num_blocks);
    L.offsets = take((M + 1) * 4);
    L.chunk_block = take(nc * 4);
    // sets of digits per (row, block): as many as a block has chunks on average, at most 32 (one for the layout
    // "block = chunk")
    L.acc_replicas = static_cast<uint32_t>(std::min<size_t>(32, std::max<size_t>(1, nc / M)));
    L.acc = take(n * M * L.acc_replicas * kLimbs * 8);
    L.special = take(n * M * 4);
    L.scales = take(n * M * 4);
    L.bits = take(n * static_cast<size_t>(L.words) * 4);
  }
  L.total = at ? at : 256;
  return L;
}

}  // namespace
}  // namespace compams

using namespace compams;

// Largest message of one worker in 32-bit words (k: entries of a worker's list).
static size_t wire_capacity_words(int compressor, size_t k, size_t d, size_t num_blocks) {
  if (compressor == COMPAMS_TOPK || compressor == COMPAMS_TOPK_BLOCKS) {
    const size_t tiles = (k + kWireTile - 1) / kWireTile;  // header, a width byte per tile, at most 31 bits per gap
    return 3 + (tiles + 3) / 4 + 2 * k;
  }
  if (compressor == COMPAMS_BLOCKSIGN) return 3 + (d + 31) / 32 + num_blocks;
  return 0;
}

static size_t ctx_wire_capacity(const compams_config& c) {  // a context's configuration holds the list length in k
  return wire_capacity_words(c.compressor, static_cast<size_t>(c.k), static_cast<size_t>(c.d),
                             static_cast<size_t>(c.num_blocks));
}

static bool is_topk(int compressor) { return compressor == COMPAMS_TOPK || compressor == COMPAMS_TOPK_BLOCKS; }

struct compams_ctx {
  compams_config cfg;
  int cached_override = -1;  // COMPAMS_OPT_CACHED_ARRAYS: -1 = the library picks by size
  Layout lay;
  Geometry geo;
  TopkWorkspace tk;
  TopkOptions tkopt;
  BlocksignWorkspace bs;
  int device;
  int64_t steps;
  bool clear_pending;      // the last step's residual update is still to be applied: top-k: e holds x at the
                           // selected coordinates; block-sign (general layouts): e holds x everywhere
  hipStream_t last_stream; // stream of the last call that enqueued work of this context
  bool enqueued;           // last_stream is meaningful: some call has enqueued work there
  hipEvent_t order_event;  // made at init (no timing): orders a new stream behind last_stream, device-side
  bool failed;             // a step's launches failed half-way: e and the workspace are in no defined state
  bool profiling;
  Launcher launcher;
};

// One context is a single sequence of steps: each reads what the one before left in theta, m, v, vhat, e and the
// workspace.  When a call arrives on another stream than the previous one, the new stream is made to wait (on the
// device; the host does not) for everything the context has enqueued so far.
static bool is_capturing(hipStream_t stream) {
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(stream, &st) != hipSuccess) {
    (void)hipGetLastError();  // e.g. the null stream while another stream is being captured: not capturing itself
    return false;
  }
  return st == hipStreamCaptureStatusActive;
}

// A stream that is being captured into a graph runs nothing now: no event is recorded for it and it does not
// become the context's last stream (whoever replays the graph orders the replays).
static hipError_t order_after_last(compams_ctx* ctx, hipStream_t stream) {
  if (!ctx->enqueued || ctx->last_stream == stream || is_capturing(stream)) return hipSuccess;
  hipError_t err = hipEventRecord(ctx->order_event, ctx->last_stream);
  if (err == hipSuccess) err = hipStreamWaitEvent(stream, ctx->order_event, 0);
  return err;
}

static void free_ctx(compams_ctx* ctx) {
  if (ctx->order_event) (void)hipEventDestroy(ctx->order_event);
  Launcher& L = ctx->launcher;
  for (int s = 0; s < kNumSlots; ++s)
    for (const Launcher::Pair& p : L.pending[s]) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  for (const Launcher::Pair& p : L.pool) { (void)hipEventDestroy(p.a); (void)hipEventDestroy(p.b); }
  delete ctx;
}

static void note_enqueued(compams_ctx* ctx, hipStream_t stream) {
  if (is_capturing(stream)) return;
  ctx->last_stream = stream;
  ctx->enqueued = true;
}

// Top-k leaves the zeroing of the residual at the selected coordinates to the next step's first pass.
// Before anybody else looks at e, the zeros are written for real (on the stream of the last step).
static hipError_t settle_residuals(compams_ctx* ctx) {
  if (!ctx->clear_pending) return hipSuccess;
  if (ctx->failed) return hipErrorInvalidValue;  // the lists or scales it would apply were never completed
  hipError_t err = hipSuccess;
  if (is_topk(ctx->cfg.compressor)) err = topk_apply_clear(ctx->geo, ctx->tk, ctx->cfg.e, ctx->last_stream);
  else if (ctx->cfg.compressor == COMPAMS_BLOCKSIGN)
    err = blocksign_apply_residual(ctx->geo, ctx->bs, ctx->cfg.e, ctx->last_stream);
  if (err == hipSuccess) ctx->clear_pending = false;
  return err;
}

// Points a context's top-k tables into a workspace laid out by make_layout (one selection per row: no segment
// tables), with the default options.
static void bind_topk_workspace(compams_ctx* ctx, char* w) {
  const Layout& lay = ctx->lay;
  TopkWorkspace& t = ctx->tk;
  t.rows = reinterpret_cast<TopkRow*>(w + lay.rows);
  t.counters = reinterpret_cast<uint32_t*>(w + lay.counters);
  t.hist0 = reinterpret_cast<uint32_t*>(w + lay.hist0);
  t.hist1 = reinterpret_cast<uint32_t*>(w + lay.hist1);
  t.hist1x = reinterpret_cast<uint32_t*>(w + lay.hist1x);
  t.hist2 = reinterpret_cast<uint32_t*>(w + lay.hist2);
  t.xcur = reinterpret_cast<uint32_t*>(w + lay.xcur);
  t.chunk_rec = reinterpret_cast<uint4*>(w + lay.chunk_rec);
  t.blk = reinterpret_cast<uint2*>(w + lay.blk);
  t.blk_prefix = reinterpret_cast<uint2*>(w + lay.blk_prefix);
  t.sel_off = reinterpret_cast<uint32_t*>(w + lay.sel_off);
  t.count_gt = reinterpret_cast<uint32_t*>(w + lay.count_gt);
  t.wire_total = reinterpret_cast<uint32_t*>(w + lay.wire_total);
  t.wire_tile_off = reinterpret_cast<uint32_t*>(w + lay.wire_tile_off);
  t.wire_tile_sum = reinterpret_cast<uint32_t*>(w + lay.wire_tile_sum);
  t.desc = reinterpret_cast<uint2*>(w + lay.desc);
  t.desc2 = reinterpret_cast<uint2*>(w + lay.desc2);
  t.cand = reinterpret_cast<uint2*>(w + lay.cand);
  t.band = reinterpret_cast<uint2*>(w + lay.band);
  t.bhist = reinterpret_cast<uint32_t*>(w + lay.bhist);
  t.bnd = reinterpret_cast<uint2*>(w + lay.bnd);
  t.bnd_sel = reinterpret_cast<uint32_t*>(w + lay.bnd_sel);
  t.flags = reinterpret_cast<uint32_t*>(w + lay.flags);
  t.idx = reinterpret_cast<int32_t*>(w + lay.idx);
  t.val = reinterpret_cast<float*>(w + lay.val);
  t.tau = reinterpret_cast<uint32_t*>(w + lay.tau);
  t.sel_off_srv = reinterpret_cast<uint32_t*>(w + lay.sel_off_srv);
  t.segs = nullptr;
  t.map_first = t.map_level0 = t.map_sweep = t.map_count = t.map_emit = t.map_final = nullptr;
  t.micro_list = nullptr;
  ctx->tkopt.cap = lay.cap_alloc;
  ctx->tkopt.predict = 1;
  ctx->tkopt.force_dense = 0;
  ctx->tkopt.band = 1;
  ctx->tkopt.band_cap = lay.band_alloc;
}

// The shape of the launches, from a validated configuration and its layout.
static void set_geometry(compams_ctx* ctx) {
  const compams_config& c = ctx->cfg;
  Geometry& geo = ctx->geo;
  geo.n = static_cast<uint32_t>(c.n);
  geo.d = static_cast<uint32_t>(c.d);
  geo.ld = c.ld;
  geo.num_chunks = ctx->lay.num_chunks;
  geo.k = is_topk(c.compressor) ? static_cast<uint32_t>(c.k) : 0;
  geo.num_blocks = c.compressor == COMPAMS_BLOCKSIGN ? static_cast<uint32_t>(c.num_blocks) : 0;
  geo.words = ctx->lay.words;
  geo.count_cpw = count_chunks_per_block(ctx->lay.num_chunks);
}

// What compams_init checks of a configuration before it looks at the workspace.
static int check_config(const compams_config* cfg) {
  if (!basic_valid(cfg)) return COMPAMS_INVALID_ARG;
  if (cfg->ld < cfg->d) return COMPAMS_INVALID_ARG;
  if (cfg->ld % 4 != 0) return COMPAMS_BAD_ALIGNMENT;
  if (cfg->eps_mode != COMPAMS_EPS_IN_SQRT && cfg->eps_mode != COMPAMS_EPS_OUT_SQRT) return COMPAMS_INVALID_ARG;
  if (!cfg->theta || !cfg->m || !cfg->v || !cfg->vhat) return COMPAMS_INVALID_ARG;
  if (cfg->compressor != COMPAMS_NONE && !cfg->e) return COMPAMS_INVALID_ARG;
  auto misaligned = [](const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) != 0; };
  if (misaligned(cfg->theta, 16) || misaligned(cfg->m, 16) || misaligned(cfg->v, 16) || misaligned(cfg->vhat, 16) ||
      (cfg->e && misaligned(cfg->e, 16)))
    return COMPAMS_BAD_ALIGNMENT;
  if (cfg->compressor == COMPAMS_BLOCKSIGN && !blocks_valid(cfg)) return COMPAMS_INVALID_ARG;
  if (cfg->compressor == COMPAMS_TOPK_BLOCKS)
    for (int64_t b = 0; b < cfg->num_blocks; ++b)
      if (cfg->block_offsets[b] % 4 != 0) return COMPAMS_BAD_ALIGNMENT;  // every block starts on 16 bytes
  return COMPAMS_OK;
}

extern "C" {

size_t compams_workspace_size(const compams_config* cfg) {
  if (!basic_valid(cfg)) return 0;
  try {
    return make_layout(cfg).total;
  } catch (...) {
    return 0;
  }
}

int compams_init(const compams_config* cfg, compams_ctx** out) {
  if (!out) return COMPAMS_INVALID_ARG;
  if (const int bad = check_config(cfg)) return bad;
  if (!cfg->workspace) return COMPAMS_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(cfg->workspace) % 256 != 0) return COMPAMS_BAD_ALIGNMENT;
  Layout lay;
  try {
    lay = make_layout(cfg);
  } catch (...) {
    return COMPAMS_HIP_ERROR;
  }
  if (cfg->workspace_bytes < lay.total) return COMPAMS_WORKSPACE_TOO_SMALL;

  compams_ctx* ctx = new (std::nothrow) compams_ctx();
  if (!ctx) return COMPAMS_HIP_ERROR;
  ctx->cfg = *cfg;
  ctx->cfg.block_offsets = nullptr;  // the host arrays are the caller's; device copies are made below
  ctx->cfg.block_k = nullptr;
  if (cfg->compressor == COMPAMS_TOPK_BLOCKS) ctx->cfg.k = static_cast<int64_t>(lay.k_total);
  ctx->lay = lay;
  ctx->steps = 0;
  ctx->clear_pending = false;
  ctx->last_stream = nullptr;
  ctx->enqueued = false;
  ctx->failed = false;
  ctx->profiling = false;
  ctx->order_event = nullptr;
  if (hipGetDevice(&ctx->device) != hipSuccess ||
      hipEventCreateWithFlags(&ctx->order_event, hipEventDisableTiming) != hipSuccess) {
    free_ctx(ctx);
    return COMPAMS_HIP_ERROR;
  }
  set_geometry(ctx);
  const Geometry& geo = ctx->geo;
  char* w = static_cast<char*>(cfg->workspace);
  hipStream_t s0 = nullptr;
  hipError_t err = hipSuccess;
  auto ok = [&](hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; };

  if (is_topk(cfg->compressor)) {
    bind_topk_workspace(ctx, w);
    TopkWorkspace& t = ctx->tk;
    // control blocks, counters, histograms and chunk tables start at zero; lists need no initial value
    ok(fill_u32(reinterpret_cast<uint32_t*>(w), lay.cand / 4, 0u, s0));
    ok(fill_u32(reinterpret_cast<uint32_t*>(w + lay.idx), (lay.total - lay.idx) / 4, 0u, s0));
    if (cfg->compressor == COMPAMS_TOPK_BLOCKS) {
      // the segments (worker-major: worker i, block b is segment i * M + b) and the workgroups of the flat launches
      std::vector<Seg> segs;
      std::vector<WgSlot> m_first, m_level0, m_sweep, m_count, m_emit, m_final;
      std::vector<uint32_t> micro;
      try {
        const std::vector<BlockShape> shapes = block_shapes(cfg);
        const size_t M = shapes.size();
        uint64_t chunks = 0, caps = 0, bcaps = 0;
        for (const BlockShape& b : shapes) { chunks += b.nc; caps += b.cap; bcaps += b.band_cap; }
        uint32_t cursor_sets = 0;
        segs.resize(static_cast<size_t>(cfg->n) * M);
        for (int64_t i = 0; i < cfg->n; ++i) {
          uint64_t c_at = 0, cap_at = 0, k_at = 0, band_at = 0;
          for (size_t b = 0; b < M; ++b) {
            const BlockShape& sh = shapes[b];
            const uint32_t si = static_cast<uint32_t>(static_cast<size_t>(i) * M + b);
            Seg& sg = segs[si];
            std::memset(&sg, 0, sizeof sg);
            sg.elem_off = i * cfg->ld + sh.off;
            sg.chunk_base = static_cast<uint64_t>(i) * chunks + c_at;
            sg.seloff_base = static_cast<uint64_t>(i) * (chunks + M) + c_at + b;
            sg.cand_base = static_cast<uint64_t>(i) * caps + cap_at;
            sg.list_base = static_cast<uint64_t>(i) * lay.k_total + k_at;
            sg.band_base = static_cast<uint64_t>(i) * bcaps + band_at;
            sg.d = sh.d; sg.k = sh.k; sg.num_chunks = sh.nc; sg.cap = sh.cap; sg.coord_base = sh.off;
            sg.band_cap = sh.band_cap;
            sg.count_cpw = sh.cpw;
            sg.groups_first = sh.groups_first; sg.groups_sweep = sh.groups_sweep; sg.count_blocks = sh.count_blocks;
            sg.micro = sh.micro;
            sg.groups_level0 = sh.groups_level0;
            sg.cursor_set = sh.nc >= kSubListMinChunks ? cursor_sets++ : kNoCursorSet;
            if (sh.micro) micro.push_back(si);
            for (uint32_t q = 0; q < sh.groups_first; ++q) m_first.push_back(WgSlot{si, q});  // in address order
            for (uint32_t q = 0; q < sh.groups_level0; ++q) m_level0.push_back(WgSlot{si, q});
            for (uint32_t q = 0; q < sh.groups_sweep; ++q) m_sweep.push_back(WgSlot{si, q});
            for (uint32_t q = 0; q < sh.count_blocks; ++q) m_count.push_back(WgSlot{si, q});
            for (uint32_t q = 0; q < sh.emit_slots; ++q) m_emit.push_back(WgSlot{si, q * static_cast<uint32_t>(kWaves)});
            if (i == 0)
              for (uint32_t q = 0; q < sh.nc; ++q) m_final.push_back(WgSlot{si, q});
            c_at += sh.nc; cap_at += sh.cap; k_at += sh.k; band_at += sh.band_cap;
          }
        }
        // and last of all the workgroups whose wavefronts take one micro problem each
        for (size_t q = 0; q < micro.size(); q += kWaves)
          m_first.push_back(WgSlot{kMicroFlag | static_cast<uint32_t>(q),
                                   static_cast<uint32_t>(std::min<size_t>(kWaves, micro.size() - q))});
      } catch (...) { free_ctx(ctx); return COMPAMS_HIP_ERROR; }
      ok(hipStreamSynchronize(s0));
      ok(hipMemcpy(w + lay.segs, segs.data(), segs.size() * sizeof(Seg), hipMemcpyHostToDevice));
      ok(hipMemcpy(w + lay.map_first, m_first.data(), m_first.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      if (!m_level0.empty())
        ok(hipMemcpy(w + lay.map_level0, m_level0.data(), m_level0.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      ok(hipMemcpy(w + lay.map_sweep, m_sweep.data(), m_sweep.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      ok(hipMemcpy(w + lay.map_count, m_count.data(), m_count.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      ok(hipMemcpy(w + lay.map_emit, m_emit.data(), m_emit.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      ok(hipMemcpy(w + lay.map_final, m_final.data(), m_final.size() * sizeof(WgSlot), hipMemcpyHostToDevice));
      if (!micro.empty()) ok(hipMemcpy(w + lay.micro_list, micro.data(), micro.size() * 4, hipMemcpyHostToDevice));
      if (m_first.size() != lay.flat.wg_first || m_level0.size() != lay.flat.wg_level0 || m_sweep.size() != lay.flat.wg_sweep || m_count.size() != lay.flat.wg_count ||
          m_emit.size() != lay.flat.wg_emit || m_final.size() != lay.flat.wg_final || micro.size() != lay.num_micro)
        ok(hipErrorInvalidValue);  // the tables and the launch sizes come from the same shapes
      t.segs = reinterpret_cast<const Seg*>(w + lay.segs);
      t.map_first = reinterpret_cast<const WgSlot*>(w + lay.map_first);
      t.map_level0 = reinterpret_cast<const WgSlot*>(w + lay.map_level0);
      t.map_sweep = reinterpret_cast<const WgSlot*>(w + lay.map_sweep);
      t.map_count = reinterpret_cast<const WgSlot*>(w + lay.map_count);
      t.map_emit = reinterpret_cast<const WgSlot*>(w + lay.map_emit);
      t.map_final = reinterpret_cast<const WgSlot*>(w + lay.map_final);
      t.micro_list = reinterpret_cast<const uint32_t*>(w + lay.micro_list);
    }
  } else if (cfg->compressor == COMPAMS_BLOCKSIGN) {
    BlocksignWorkspace& b = ctx->bs;
    b.offsets = reinterpret_cast<uint32_t*>(w + lay.offsets);
    b.chunk_block = reinterpret_cast<uint32_t*>(w + lay.chunk_block);
    b.acc = reinterpret_cast<uint64_t*>(w + lay.acc);
    b.acc_replicas = lay.acc_replicas;
    b.special = reinterpret_cast<uint32_t*>(w + lay.special);
    b.scales = reinterpret_cast<float*>(w + lay.scales);
    b.bits = reinterpret_cast<uint32_t*>(w + lay.bits);
    std::vector<uint32_t> off32, cb;
    try {
      off32.resize(static_cast<size_t>(cfg->num_blocks) + 1);
      cb.resize(lay.num_chunks);
    } catch (...) { free_ctx(ctx); return COMPAMS_HIP_ERROR; }
    for (int64_t i = 0; i <= cfg->num_blocks; ++i) off32[static_cast<size_t>(i)] = static_cast<uint32_t>(cfg->block_offsets[i]);
    uint32_t blk = 0;
    for (uint32_t c = 0; c < lay.num_chunks; ++c) {
      const uint32_t j = c * static_cast<uint32_t>(kChunk);
      while (off32[blk + 1] <= j) ++blk;
      cb[c] = blk;
    }
    ok(fill_u32(reinterpret_cast<uint32_t*>(w), lay.total / 4, 0u, s0));
    ok(hipStreamSynchronize(s0));
    ok(hipMemcpy(b.offsets, off32.data(), off32.size() * 4, hipMemcpyHostToDevice));
    ok(hipMemcpy(b.chunk_block, cb.data(), cb.size() * 4, hipMemcpyHostToDevice));
  }
  if (!(cfg->flags & COMPAMS_KEEP_STATE)) {
    if (cfg->e) ok(fill_rows_f32(cfg->e, geo.n, geo.ld, geo.d, 0.0f, s0));
    ok(fill_rows_f32(cfg->m, 1, 0, geo.d, 0.0f, s0));
    ok(fill_rows_f32(cfg->v, 1, 0, geo.d, 0.0f, s0));
    ok(fill_rows_f32(cfg->vhat, 1, 0, geo.d, 0.0f, s0));
  }
  ok(hipStreamSynchronize(s0));
  if (err != hipSuccess) { free_ctx(ctx); return COMPAMS_HIP_ERROR; }
  *out = ctx;
  return COMPAMS_OK;
}

static AmsParams ams_params(const compams_config& c, float lr, int cached_override) {
  AmsParams ap;
  ap.beta1 = c.beta1;
  ap.beta2 = c.beta2;
  ap.one_minus_beta1 = 1.0f - c.beta1;
  ap.one_minus_beta2 = 1.0f - c.beta2;
  ap.eps = c.eps;
  ap.lr = lr;
  ap.nf = static_cast<float>(c.n);
  ap.eps_out = c.eps_mode == COMPAMS_EPS_OUT_SQRT;
  ap.cached_arrays = cached_override >= 0 ? cached_override : cached_state_arrays(c.d);
  return ap;
}

// A call that enqueues work of the context: not after a failed step, and on the device the context was made on.
static int usable(const compams_ctx* ctx) {
  if (ctx->failed) return COMPAMS_BAD_STATE;
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return COMPAMS_HIP_ERROR;
  return dev == ctx->device ? COMPAMS_OK : COMPAMS_BAD_STATE;
}

// The whole step, or only the workers' lines of it.
static int step_impl(compams_ctx* ctx, const float* g, float lr, bool workers_only, void* hip_stream) {
  if (!ctx || !g) return COMPAMS_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(g) % 16 != 0) return COMPAMS_BAD_ALIGNMENT;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const compams_config& c = ctx->cfg;
  if (workers_only && c.compressor == COMPAMS_NONE) return COMPAMS_BAD_STATE;  // the message is g itself
  if (const int bad = usable(ctx)) return bad;
  if (order_after_last(ctx, stream) != hipSuccess) return COMPAMS_HIP_ERROR;  // nothing of the step is enqueued yet
  const AmsParams ap = ams_params(c, lr, ctx->cached_override);
  Launcher* L = ctx->profiling ? &ctx->launcher : nullptr;
  hipError_t err;
  try {
    if (is_topk(c.compressor)) {
      const bool may_predict = ctx->steps > 0 && ctx->tkopt.predict && !ctx->tkopt.force_dense;
      if (c.compressor == COMPAMS_TOPK)
        err = topk_step(ctx->geo, ctx->tk, ctx->tkopt, ap, g, c.e, c.theta, c.m, c.v, c.vhat, may_predict,
                        ctx->clear_pending, workers_only, stream, L);
      else
        err = topk_blocks_step(ctx->geo, ctx->tk, ctx->tkopt, ap, ctx->lay.flat, g, c.e, c.theta, c.m, c.v, c.vhat,
                               may_predict, ctx->clear_pending, workers_only, stream, L);
    } else if (c.compressor == COMPAMS_BLOCKSIGN) {
      err = blocksign_step(ctx->geo, ctx->bs, ap, g, c.e, c.theta, c.m, c.v, c.vhat, ctx->clear_pending, workers_only,
                           stream, L);
    } else {
      err = none_step(ctx->geo, ap, g, c.theta, c.m, c.v, c.vhat, stream, L);
    }
  } catch (...) {
    err = hipErrorUnknown;
  }
  note_enqueued(ctx, stream);  // whatever was launched before a failure sits on this stream
  if (err != hipSuccess || (L && L->failed)) {
    // some of the step's kernels may run, others not: nothing that later calls could build on
    if (err != hipSuccess) ctx->failed = true;
    return COMPAMS_HIP_ERROR;
  }
  // every kernel of the step is enqueued: the error line it leaves to the next first pass is pending from now on
  if (c.compressor != COMPAMS_NONE) ctx->clear_pending = true;
  ++ctx->steps;
  return COMPAMS_OK;
}

int compams_step(compams_ctx* ctx, const float* g, float lr, void* hip_stream) {
  return step_impl(ctx, g, lr, false, hip_stream);
}

int compams_worker_step(compams_ctx* ctx, const float* g, void* hip_stream) {
  return step_impl(ctx, g, 0.0f, true, hip_stream);
}

int compams_server_step(compams_ctx* ctx, const uint32_t* messages, int64_t stride_words, const uint32_t* words,
                        float lr, uint32_t* status_out, void* hip_stream) {
  if (!ctx || !messages || !status_out) return COMPAMS_INVALID_ARG;
  const compams_config& c = ctx->cfg;
  if (c.compressor == COMPAMS_NONE) return COMPAMS_BAD_STATE;
  if (stride_words < static_cast<int64_t>(ctx_wire_capacity(c))) return COMPAMS_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(messages) % 4 != 0 || reinterpret_cast<uintptr_t>(status_out) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(words) % 4 != 0)
    return COMPAMS_BAD_ALIGNMENT;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (const int bad = usable(ctx)) return bad;
  // The messages are unpacked into the workspace arrays that a pending residual update of this context still
  // needs (the last lists, the last scales): apply it first, on the stream of the step that left it; then this
  // call's stream is ordered behind that one on the device.
  if (settle_residuals(ctx) != hipSuccess) return COMPAMS_HIP_ERROR;
  if (order_after_last(ctx, stream) != hipSuccess) return COMPAMS_HIP_ERROR;
  const AmsParams ap = ams_params(c, lr, ctx->cached_override);
  Launcher* L = ctx->profiling ? &ctx->launcher : nullptr;
  hipError_t err;
  try {
    if (is_topk(c.compressor)) {
      err = wire_decode_topk(ctx->geo, ctx->tk, messages, stride_words, words, ctx->tk.idx, ctx->tk.val, status_out,
                             stream, L);
      if (err == hipSuccess)
        err = topk_server_step(ctx->geo, ctx->tk, ctx->tkopt, ap, c.theta, c.m, c.v, c.vhat, stream, L);
    } else {
      err = wire_decode_blocksign(ctx->geo, messages, stride_words, words, ctx->bs.bits, ctx->bs.scales, status_out,
                                  stream, L);
      if (err == hipSuccess) err = blocksign_server_step(ctx->geo, ctx->bs, ap, c.theta, c.m, c.v, c.vhat, stream, L);
    }
  } catch (...) {
    err = hipErrorUnknown;
  }
  note_enqueued(ctx, stream);
  if (err != hipSuccess) ctx->failed = true;  // theta, m, v, vhat may be half updated
  return err == hipSuccess && !(L && L->failed) ? COMPAMS_OK : COMPAMS_HIP_ERROR;
}

int compams_state(compams_ctx* ctx, int which, const void** dev_ptr, int64_t* count) {
  if (!ctx || !dev_ptr || !count) return COMPAMS_INVALID_ARG;
  const compams_config& c = ctx->cfg;
  const int64_t n = c.n, d = c.d;
  const void* p = nullptr;
  int64_t cnt = 0;
  const bool tk = is_topk(c.compressor), bs = c.compressor == COMPAMS_BLOCKSIGN;
  const int64_t problems = c.compressor == COMPAMS_TOPK_BLOCKS ? n * c.num_blocks : n;  // selection problems
  switch (which) {
    case COMPAMS_STATE_THETA: p = c.theta; cnt = d; break;
    case COMPAMS_STATE_M: p = c.m; cnt = d; break;
    case COMPAMS_STATE_V: p = c.v; cnt = d; break;
    case COMPAMS_STATE_VHAT: p = c.vhat; cnt = d; break;
    case COMPAMS_STATE_E:
      if (!c.e) return COMPAMS_BAD_STATE;
      if (settle_residuals(ctx) != hipSuccess) return COMPAMS_HIP_ERROR;
      p = c.e; cnt = n * c.ld; break;
    case COMPAMS_STATE_LAST_IDX:
      if (!tk) return COMPAMS_BAD_STATE;
      p = ctx->tk.idx; cnt = n * c.k; break;
    case COMPAMS_STATE_LAST_VAL:
      if (!tk) return COMPAMS_BAD_STATE;
      p = ctx->tk.val; cnt = n * c.k; break;
    case COMPAMS_STATE_LAST_THRESHOLD:
      if (!tk) return COMPAMS_BAD_STATE;
      p = ctx->tk.tau; cnt = problems; break;
    case COMPAMS_STATE_LAST_COUNT_GT:
      if (!tk) return COMPAMS_BAD_STATE;
      p = ctx->tk.count_gt; cnt = problems; break;
    case COMPAMS_STATE_COUNTERS:
      if (!tk) return COMPAMS_BAD_STATE;
      p = ctx->tk.counters; cnt = problems * COMPAMS_COUNTERS_PER_ROW; break;
    case COMPAMS_STATE_LAST_SIGNBITS:
      if (!bs) return COMPAMS_BAD_STATE;
      p = ctx->bs.bits; cnt = n * static_cast<int64_t>(ctx->geo.words); break;
    case COMPAMS_STATE_LAST_SCALES:
      if (!bs) return COMPAMS_BAD_STATE;
      p = ctx->bs.scales; cnt = n * c.num_blocks; break;
    case COMPAMS_STATE_PENDING:  // no pointer: the answer is the count
      p = nullptr; cnt = ctx->clear_pending ? 1 : 0; break;
    default: return COMPAMS_INVALID_ARG;
  }
  *dev_ptr = p;
  *count = cnt;
  return COMPAMS_OK;
}

int compams_set_option(compams_ctx* ctx, int option, int64_t value) {
  if (!ctx) return COMPAMS_INVALID_ARG;
  if (option == COMPAMS_OPT_CACHED_ARRAYS) {  // every compressor
    if (value < -1 || value > 4) return COMPAMS_INVALID_ARG;
    ctx->cached_override = static_cast<int>(value);
    return COMPAMS_OK;
  }
  if (!is_topk(ctx->cfg.compressor)) return COMPAMS_BAD_STATE;
  switch (option) {
    case COMPAMS_OPT_CANDIDATE_CAP:
      if (value < 0 || value > static_cast<int64_t>(ctx->lay.cap_alloc)) return COMPAMS_INVALID_ARG;
      ctx->tkopt.cap = static_cast<uint32_t>(value);
      return COMPAMS_OK;
    case COMPAMS_OPT_PREDICT:
      ctx->tkopt.predict = value ? 1u : 0u;
      return COMPAMS_OK;
    case COMPAMS_OPT_FORCE_DENSE:
      ctx->tkopt.force_dense = value ? 1u : 0u;
      return COMPAMS_OK;
    case COMPAMS_OPT_BAND:
      ctx->tkopt.band = value ? 1u : 0u;
      return COMPAMS_OK;
    default: return COMPAMS_INVALID_ARG;
  }
}

int compams_profile_enable(compams_ctx* ctx, int enable) {
  if (!ctx) return COMPAMS_INVALID_ARG;
  if (enable < 0 || enable > 2) return COMPAMS_INVALID_ARG;
  ctx->profiling = enable != 0;
  // 1: every kernel; 2: only the kernel that moves most of the bytes (the first pass of each compressor)
  ctx->launcher.mask = enable == 1 ? 0xffffffffu
                                   : (1u << kSlotPassA) | (1u << kSlotBsPass1) | (1u << kSlotNoneAms);
  return COMPAMS_OK;
}

int compams_profile_read(compams_ctx* ctx, int cap, const char** names, double* ms, int64_t* launches, int* count) {
  if (!ctx || !count || cap < 0 || (cap > 0 && (!names || !ms || !launches))) return COMPAMS_INVALID_ARG;
  Launcher& L = ctx->launcher;
  bool bad = false;
  for (int s = 0; s < kNumSlots; ++s) {
    for (const Launcher::Pair& p : L.pending[s]) {
      float t = 0.0f;
      if (hipEventSynchronize(p.b) != hipSuccess || hipEventElapsedTime(&t, p.a, p.b) != hipSuccess) bad = true;
      else { L.total_ms[s] += t; ++L.launches[s]; }
      try { L.pool.push_back(p); } catch (...) { bad = true; }
    }
    L.pending[s].clear();
  }
  int outn = 0;
  for (int s = 0; s < kNumSlots; ++s) {
    if (L.launches[s] == 0) continue;
    if (outn < cap) { names[outn] = kSlotNames[s]; ms[outn] = L.total_ms[s]; launches[outn] = L.launches[s]; }
    ++outn;
  }
  for (int s = 0; s < kNumSlots; ++s) { L.total_ms[s] = 0.0; L.launches[s] = 0; }
  L.failed = false;
  *count = outn;
  return bad ? COMPAMS_HIP_ERROR : COMPAMS_OK;
}

int compams_destroy(compams_ctx* ctx) {
  if (!ctx) return COMPAMS_INVALID_ARG;
  int status = COMPAMS_OK;
  if (ctx->clear_pending && !ctx->failed) {  // hand e back to the caller in its settled form
    if (settle_residuals(ctx) != hipSuccess || hipStreamSynchronize(ctx->last_stream) != hipSuccess)
      status = COMPAMS_HIP_ERROR;
  }
  free_ctx(ctx);
  return status;
}

const char* compams_strerror(int status) {
  switch (status) {
    case COMPAMS_OK: return "ok";
    case COMPAMS_INVALID_ARG: return "invalid argument";
    case COMPAMS_BAD_ALIGNMENT: return "pointer or row stride not aligned";
    case COMPAMS_WORKSPACE_TOO_SMALL: return "workspace too small";
    case COMPAMS_HIP_ERROR: return "HIP runtime error";
    case COMPAMS_BAD_STATE: return "call does not apply to this context (compressor, device, or a step that failed)";
    default: return "unknown status";
  }
}

size_t compams_wire_capacity(const compams_config* cfg) {
  if (!basic_valid(cfg)) return 0;
  size_t k = static_cast<size_t>(cfg->k);
  if (cfg->compressor == COMPAMS_TOPK_BLOCKS) {
    k = 0;
    for (int64_t b = 0; b < cfg->num_blocks; ++b) k += static_cast<size_t>(cfg->block_k[b]);
  }
  return wire_capacity_words(cfg->compressor, k, static_cast<size_t>(cfg->d), static_cast<size_t>(cfg->num_blocks));
}

int compams_encode(compams_ctx* ctx, uint32_t* messages, int64_t stride_words, uint32_t* words_out, void* hip_stream) {
  if (!ctx || !messages || !words_out) return COMPAMS_INVALID_ARG;
  const compams_config& c = ctx->cfg;
  if (c.compressor == COMPAMS_NONE || ctx->steps == 0) return COMPAMS_BAD_STATE;
  if (stride_words < static_cast<int64_t>(ctx_wire_capacity(c))) return COMPAMS_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(messages) % 4 != 0 || reinterpret_cast<uintptr_t>(words_out) % 4 != 0)
    return COMPAMS_BAD_ALIGNMENT;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (const int bad = usable(ctx)) return bad;
  if (order_after_last(ctx, stream) != hipSuccess) return COMPAMS_HIP_ERROR;
  Launcher* L = ctx->profiling ? &ctx->launcher : nullptr;
  hipError_t err;
  try {
    err = is_topk(c.compressor)
              ? wire_encode_topk(ctx->geo, ctx->tk, messages, stride_words, words_out, stream, L)
              : wire_encode_blocksign(ctx->geo, ctx->bs, messages, stride_words, words_out, stream, L);
  } catch (...) {
    err = hipErrorUnknown;
  }
  note_enqueued(ctx, stream);
  return err == hipSuccess && !(L && L->failed) ? COMPAMS_OK : COMPAMS_HIP_ERROR;
}

int compams_decode(compams_ctx* ctx, const uint32_t* messages, int64_t stride_words, const uint32_t* words,
                   void* out_a, void* out_b, uint32_t* status_out, void* hip_stream) {
  if (!ctx || !messages || !out_a || !out_b || !status_out) return COMPAMS_INVALID_ARG;
  const compams_config& c = ctx->cfg;
  if (c.compressor == COMPAMS_NONE) return COMPAMS_BAD_STATE;
  if (stride_words < static_cast<int64_t>(ctx_wire_capacity(c))) return COMPAMS_INVALID_ARG;
  if (reinterpret_cast<uintptr_t>(messages) % 4 != 0 || reinterpret_cast<uintptr_t>(out_a) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(out_b) % 4 != 0 || reinterpret_cast<uintptr_t>(status_out) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(words) % 4 != 0)
    return COMPAMS_BAD_ALIGNMENT;
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  if (const int bad = usable(ctx)) return bad;
  if (order_after_last(ctx, stream) != hipSuccess) return COMPAMS_HIP_ERROR;
  Launcher* L = ctx->profiling ? &ctx->launcher : nullptr;
  hipError_t err;
  try {
    err = is_topk(c.compressor)
              ? wire_decode_topk(ctx->geo, ctx->tk, messages, stride_words, words, static_cast<int32_t*>(out_a),
                                 static_cast<float*>(out_b), status_out, stream, L)
              : wire_decode_blocksign(ctx->geo, messages, stride_words, words, static_cast<uint32_t*>(out_a),
                                      static_cast<float*>(out_b), status_out, stream, L);
  } catch (...) {
    err = hipErrorUnknown;
  }
  note_enqueued(ctx, stream);
  return err == hipSuccess && !(L && L->failed) ? COMPAMS_OK : COMPAMS_HIP_ERROR;
}

int compams_copy(void* dst, const void* src, size_t bytes, void* hip_stream) {
  if (!dst || !src) return COMPAMS_INVALID_ARG;
  if (bytes % 16 != 0 || reinterpret_cast<uintptr_t>(dst) % 16 != 0 || reinterpret_cast<uintptr_t>(src) % 16 != 0)
    return COMPAMS_BAD_ALIGNMENT;
  return stream_copy(dst, src, bytes, static_cast<hipStream_t>(hip_stream)) == hipSuccess ? COMPAMS_OK
                                                                                            : COMPAMS_HIP_ERROR;
}

int compams_cached_state_arrays(int64_t d) { return d < 1 ? COMPAMS_INVALID_ARG : cached_state_arrays(d); }

int compams_inplace_probe(float* const* arrays, int n_arrays, size_t count, int cached_arrays, void* hip_stream) {
  if (!arrays || n_arrays < 1 || n_arrays > 4 || count > (static_cast<size_t>(1) << 40) || cached_arrays < 0 ||
      cached_arrays > 4)
    return COMPAMS_INVALID_ARG;
  for (int a = 0; a < n_arrays; ++a)
    if (!arrays[a]) return COMPAMS_INVALID_ARG;
  if (count % 4 != 0) return COMPAMS_BAD_ALIGNMENT;
  for (int a = 0; a < n_arrays; ++a)
    if (reinterpret_cast<uintptr_t>(arrays[a]) % 16 != 0) return COMPAMS_BAD_ALIGNMENT;
  return inplace_probe(arrays, n_arrays, count, cached_arrays, static_cast<hipStream_t>(hip_stream)) == hipSuccess
             ? COMPAMS_OK
             : COMPAMS_HIP_ERROR;
}

// ---- One whole step without a workspace argument -----------------------------------------------------------
// For callers that cannot hand over (or allocate) a workspace: the tables of the top-k selection live in a
// device array that is part of the library's code object.  Every device the library runs on holds its own copy
// at its own address until the process ends; the host-side name below is only a handle for hipGetSymbolAddress.
__attribute__((used)) static __device__ __align__(256) unsigned char scratch[COMPAMS_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices];  // device address of `scratch` per device, once looked up

// The address of this device's copy of the array (the device must be current).
hipError_t scratch_of_current_device(char** out) {
  int dev = -1;
  hipError_t err = hipGetDevice(&dev);
  if (err != hipSuccess) return err;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (err != hipSuccess) return err;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = static_cast<char*>(g_scratch_ptr[dev]);
  return hipSuccess;
}
}  // namespace

int compams_step_static(const compams_config* cfg, const float* g, float lr, int32_t* idx_out, float* val_out,
                        void* hip_stream) {
  if (!cfg || !g) return COMPAMS_INVALID_ARG;
  if (const int bad = check_config(cfg)) return bad;
  if (cfg->compressor != COMPAMS_TOPK) return COMPAMS_BAD_STATE;  // the other compressors' tables come from the host
  if (reinterpret_cast<uintptr_t>(g) % 16 != 0 || reinterpret_cast<uintptr_t>(idx_out) % 4 != 0 ||
      reinterpret_cast<uintptr_t>(val_out) % 4 != 0)
    return COMPAMS_BAD_ALIGNMENT;
  compams_ctx ctx;  // lives for this call only; nothing in it owns memory
  try {
    ctx.lay = make_layout(cfg);
  } catch (...) {
    return COMPAMS_HIP_ERROR;
  }
  if (ctx.lay.total > static_cast<size_t>(COMPAMS_STATIC_SCRATCH_BYTES)) return COMPAMS_WORKSPACE_TOO_SMALL;
  char* w = nullptr;
  if (scratch_of_current_device(&w) != hipSuccess) return COMPAMS_HIP_ERROR;
  ctx.cfg = *cfg;
  ctx.cfg.workspace = w;
  ctx.cfg.workspace_bytes = COMPAMS_STATIC_SCRATCH_BYTES;
  set_geometry(&ctx);
  bind_topk_workspace(&ctx, w);
  hipStream_t stream = static_cast<hipStream_t>(hip_stream);
  const Layout& lay = ctx.lay;
  const AmsParams ap = ams_params(ctx.cfg, lr, -1);
  hipError_t err = hipSuccess;
  auto ok = [&](hipError_t e) { if (err == hipSuccess && e != hipSuccess) err = e; };
  // the array keeps what the last call left: control blocks, counters, histograms and chunk tables start at zero
  // (fill kernels, so that the call can be recorded into a graph); lists need no initial value
  ok(fill_u32(reinterpret_cast<uint32_t*>(w), lay.cand / 4, 0u, stream));
  ok(fill_u32(reinterpret_cast<uint32_t*>(w + lay.idx), (lay.total - lay.idx) / 4, 0u, stream));
  if (!(cfg->flags & COMPAMS_KEEP_STATE)) {
    ok(fill_rows_f32(cfg->e, ctx.geo.n, ctx.geo.ld, ctx.geo.d, 0.0f, stream));
    ok(fill_rows_f32(cfg->m, 1, 0, ctx.geo.d, 0.0f, stream));
    ok(fill_rows_f32(cfg->v, 1, 0, ctx.geo.d, 0.0f, stream));
    ok(fill_rows_f32(cfg->vhat, 1, 0, ctx.geo.d, 0.0f, stream));
  }
  if (err == hipSuccess) {
    try {
      // no guess is carried over and no error line is pending on entry; the one this step leaves is applied at once
      err = topk_step(ctx.geo, ctx.tk, ctx.tkopt, ap, g, cfg->e, cfg->theta, cfg->m, cfg->v, cfg->vhat, false, false,
                      false, stream, nullptr);
    } catch (...) {
      err = hipErrorUnknown;
    }
  }
  if (err == hipSuccess) err = topk_apply_clear(ctx.geo, ctx.tk, cfg->e, stream);
  const size_t nk = static_cast<size_t>(cfg->n) * static_cast<size_t>(cfg->k);
  if (err == hipSuccess && idx_out)
    err = copy_u32(reinterpret_cast<uint32_t*>(idx_out), reinterpret_cast<const uint32_t*>(ctx.tk.idx), nk, stream);
  if (err == hipSuccess && val_out)
    err = copy_u32(reinterpret_cast<uint32_t*>(val_out), reinterpret_cast<const uint32_t*>(ctx.tk.val), nk, stream);
  return err == hipSuccess ? COMPAMS_OK : COMPAMS_HIP_ERROR;
}

}  // extern "C"
