// The workers' messages as they would go on the wire (the send line among the worker lines of Algorithm 2),
// and back.  One message per worker, a sequence of 32-bit words:
//
//   top-k      [1, k, 256,  width words,  gap stream,  k value words]
//              gap_0 = idx_0, gap_q = idx_q - idx_{q-1} - 1.  The gaps are taken in tiles of 256 (the last one
//              may be shorter); tile t has its own width b_t = number of bits of its largest gap (at least 1),
//              kept as byte (t mod 4) of width word t div 4 (unused bytes 0).  In the stream the tiles follow
//              one another, each starting on a word boundary: gap i of a tile occupies the tile's bits
//              i*b_t .. i*b_t + b_t - 1, least significant bit first; bit u of a tile is bit (u mod 32) of its
//              word u div 32; unused bits of a tile's last word are 0.
//   block-sign [2, d, M,  ceil(d/32) sign words,  M scale words]
//
// A wavefront owns a tile.  Packing: the tile's gaps are staged in LDS and every stream word is written by one
// lane, which gathers the (at most 32) gaps that overlap it: no atomics touch the message.  Where a tile starts
// in the stream, and the coordinate before its first entry when unpacking, come from prefix sums over the
// tiles of a row (one workgroup per row).  A message that is not well formed never makes a kernel read outside
// [message, message + stride): counts come from the configuration and widths are clamped to 1 .. 31.

#include "compams_device.h"
#include "compams_internal.h"

namespace compams {
namespace {

static_assert(kWireTile == 256, "a wavefront takes a tile as four gaps per lane");

__device__ __forceinline__ uint32_t gap_of(const int32_t* idx, uint32_t q) {
  const uint32_t cur = static_cast<uint32_t>(idx[q]);
  return q == 0 ? cur : cur - static_cast<uint32_t>(idx[q - 1]) - 1u;
}

__device__ __forceinline__ uint32_t width_of(uint32_t widest) {  // coordinates are below 2^31: at most 31
  return widest ? 32u - static_cast<uint32_t>(__clz(widest)) : 1u;
}

__device__ __forceinline__ uint32_t clamp_width(uint32_t b) { return b < 1u ? 1u : (b > 31u ? 31u : b); }

__device__ __forceinline__ uint32_t tile_count(uint32_t k, uint32_t t) {
  const uint32_t left = k - t * kWireTile;
  return left < kWireTile ? left : kWireTile;
}

__device__ __forceinline__ uint32_t tile_words(uint32_t cnt, uint32_t b) { return (cnt * b + 31u) >> 5; }

__device__ __forceinline__ uint32_t width_byte(const uint32_t* msg, uint32_t t) {
  return (msg[3 + (t >> 2)] >> (8u * (t & 3u))) & 0xffu;
}

__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    const uint32_t o = __shfl_xor(v, s, 64);
    v = o > v ? o : v;
  }
  return v;
}

// Widths of the tiles (into the message) and the words each tile will take (into tile_off, to be scanned).
__global__ __launch_bounds__(kWG) void k_wire_tile_width(const int32_t* __restrict__ idx_all, uint32_t k,
                                                          uint32_t tiles, uint32_t* __restrict__ messages,
                                                          int64_t stride, uint32_t* __restrict__ tile_off) {
  __shared__ uint32_t sb[kWaves];
  const uint32_t row = blockIdx.y, wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t t = blockIdx.x * kWaves + wave;
  const int32_t* idx = idx_all + static_cast<size_t>(row) * k;
  uint32_t b = 0;  // tiles beyond the last one leave a zero byte
  if (t < tiles) {
    const uint32_t cnt = tile_count(k, t);
    uint32_t mx = 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const uint32_t i = lane + 64u * s;
      if (i < cnt) {
        const uint32_t g = gap_of(idx, t * kWireTile + i);
        mx = g > mx ? g : mx;
      }
    }
    b = width_of(wave_max(mx));
    if (lane == 0) tile_off[static_cast<size_t>(row) * tiles + t] = tile_words(cnt, b);
  }
  if (lane == 0) sb[wave] = b;
  __syncthreads();
  if (threadIdx.x == 0)
    messages[static_cast<int64_t>(row) * stride + 3 + blockIdx.x] = sb[0] | (sb[1] << 8) | (sb[2] << 16) | (sb[3] << 24);
}

// In place: per-tile amounts -> what lies before each tile; totals[row] (if given) gets the row's sum.
// One workgroup per row.
__global__ __launch_bounds__(kWG) void k_wire_tile_scan(uint32_t* __restrict__ tiles, uint32_t tiles_per_row,
                                                         uint32_t* __restrict__ totals) {
  __shared__ uint32_t scratch[kWG / 64 + 1];
  uint32_t* t = tiles + static_cast<size_t>(blockIdx.x) * tiles_per_row;
  uint32_t carry = 0;
  for (uint32_t base = 0; base < tiles_per_row; base += kWG) {
    const uint32_t i = base + threadIdx.x;
    const uint32_t v = i < tiles_per_row ? t[i] : 0u;
    uint32_t total;
    const uint32_t before = block_excl_scan<kWG>(v, scratch, &total);
    if (i < tiles_per_row) t[i] = carry + before;
    carry += total;
  }
  if (totals && threadIdx.x == 0) totals[blockIdx.x] = carry;
}

__global__ __launch_bounds__(kWG) void k_wire_pack_topk(const int32_t* __restrict__ idx_all,
                                                         const float* __restrict__ val_all, uint32_t k,
                                                         uint32_t tiles, const uint32_t* __restrict__ tile_off,
                                                         const uint32_t* __restrict__ totals,
                                                         uint32_t* __restrict__ messages, int64_t stride,
                                                         uint32_t* __restrict__ words_out) {
  __shared__ uint32_t sg[kWaves][kWireTile];
  const uint32_t row = blockIdx.y, wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t t = blockIdx.x * kWaves + wave;
  const int32_t* idx = idx_all + static_cast<size_t>(row) * k;
  const float* val = val_all + static_cast<size_t>(row) * k;
  uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  const uint32_t width_words = (tiles + 3u) >> 2;
  const uint32_t stream_total = totals[row];
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    msg[0] = 1u;
    msg[1] = k;
    msg[2] = kWireTile;
    words_out[row] = 3u + width_words + stream_total + k;
  }
  const bool live = t < tiles;
  const uint32_t cnt = live ? tile_count(k, t) : 0u;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t i = lane + 64u * s;
    sg[wave][i] = i < cnt ? gap_of(idx, t * kWireTile + i) : 0u;
  }
  __syncthreads();
  if (live) {
    const uint32_t b = width_byte(msg, t);  // written by the width kernel: 1 .. 31
    uint32_t* stream = msg + 3 + width_words + tile_off[static_cast<size_t>(row) * tiles + t];
    const uint32_t nw = tile_words(cnt, b);
    for (uint32_t w = lane; w < nw; w += 64) {
      const uint32_t lo = w * 32u;
      const uint32_t q0 = lo / b;
      uint32_t q1 = (lo + 31u) / b;
      if (q1 > cnt - 1u) q1 = cnt - 1u;
      uint32_t word = 0;
      for (uint32_t q = q0; q <= q1; ++q) {
        const uint32_t g = sg[wave][q];
        const int32_t sh = static_cast<int32_t>(q * b) - static_cast<int32_t>(lo);
        word |= sh >= 0 ? (g << sh) : (g >> (-sh));  // |sh| <= 31
      }
      stream[w] = word;
    }
  }
  uint32_t* values = msg + 3 + width_words + stream_total;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < k; q += step) values[q] = __float_as_uint(val[q]);
}

// Gap i of a tile whose stream starts at `tile` and has nw words (i < cnt, so the field lies inside them).
__device__ __forceinline__ uint32_t field_of(const uint32_t* __restrict__ tile, uint32_t nw, uint32_t i, uint32_t b) {
  const uint32_t pos = i * b;
  const uint32_t w = pos >> 5, sh = pos & 31u;
  uint64_t two = tile[w];
  if (w + 1 < nw) two |= static_cast<uint64_t>(tile[w + 1]) << 32;
  return static_cast<uint32_t>(two >> sh) & ((1u << b) - 1u);
}

// status[row]: 0 well formed; bit 0: not a message of this kind and size, or a width outside 1 .. 31; bit 1 (set
// while unpacking): length differs; bit 2 (set while unpacking): a coordinate at or beyond d.
// Also leaves the words each tile takes (from the clamped widths) in tile_off, to be scanned.
__global__ __launch_bounds__(kWG) void k_wire_check_topk(const uint32_t* __restrict__ messages, int64_t stride,
                                                          uint32_t k, uint32_t tiles,
                                                          uint32_t* __restrict__ tile_off,
                                                          uint32_t* __restrict__ status) {
  __shared__ uint32_t st;
  const uint32_t row = blockIdx.x;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  if (threadIdx.x == 0) st = (msg[0] != 1u || msg[1] != k || msg[2] != kWireTile) ? 1u : 0u;
  __syncthreads();
  bool bad = false;
  for (uint32_t t = threadIdx.x; t < tiles; t += kWG) {
    const uint32_t b = width_byte(msg, t);
    bad |= b < 1u || b > 31u;
    tile_off[static_cast<size_t>(row) * tiles + t] = tile_words(tile_count(k, t), clamp_width(b));
  }
  if (bad) atomicOr(&st, 1u);
  __syncthreads();
  if (threadIdx.x == 0) status[row] = st;
}

// The gaps of a lane's four consecutive entries of tile t (zero beyond the tile) and their number.
struct LaneGaps {
  uint32_t gap[4];
  uint32_t n;
};
__device__ __forceinline__ LaneGaps lane_gaps(const uint32_t* __restrict__ msg, uint32_t k, uint32_t tiles, uint32_t t,
                                              const uint32_t* __restrict__ tile_off_row) {
  const uint32_t lane = lane_id();
  const uint32_t cnt = tile_count(k, t);
  const uint32_t b = clamp_width(width_byte(msg, t));
  const uint32_t* tile = msg + 3 + ((tiles + 3u) >> 2) + tile_off_row[t];
  const uint32_t nw = tile_words(cnt, b);
  LaneGaps g;
  g.n = 0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t i = lane * 4u + s;
    g.gap[s] = 0;
    if (i < cnt) {
      g.gap[s] = field_of(tile, nw, i, b);
      g.n = s + 1;
    }
  }
  return g;
}

__device__ __forceinline__ uint32_t wave_total(uint32_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) v += __shfl_xor(v, s, 64);
  return v;
}

// Coordinates covered by each tile (sum of gap + 1), to be scanned into the coordinate before each tile.
__global__ __launch_bounds__(kWG) void k_wire_tile_sums(const uint32_t* __restrict__ messages, int64_t stride,
                                                         uint32_t k, uint32_t tiles,
                                                         const uint32_t* __restrict__ tile_off,
                                                         uint32_t* __restrict__ tile_sum) {
  const uint32_t row = blockIdx.y, wave = threadIdx.x >> 6;
  const uint32_t t = blockIdx.x * kWaves + wave;
  if (t >= tiles) return;  // wave-uniform; no barrier below
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  const LaneGaps g = lane_gaps(msg, k, tiles, t, tile_off + static_cast<size_t>(row) * tiles);
  uint32_t sum = g.n;
#pragma unroll
  for (int s = 0; s < 4; ++s) sum += g.gap[s];
  sum = wave_total(sum);
  if (lane_id() == 0) tile_sum[static_cast<size_t>(row) * tiles + t] = sum;
}

__global__ __launch_bounds__(kWG) void k_wire_unpack_topk(const uint32_t* __restrict__ messages, int64_t stride,
                                                           const uint32_t* __restrict__ words, uint32_t k,
                                                           uint32_t d, uint32_t tiles,
                                                           const uint32_t* __restrict__ tile_off,
                                                           const uint32_t* __restrict__ totals,
                                                           const uint32_t* __restrict__ tile_sum,
                                                           int32_t* __restrict__ idx_out, float* __restrict__ val_out,
                                                           uint32_t* __restrict__ status) {
  const uint32_t row = blockIdx.y, wave = threadIdx.x >> 6, lane = lane_id();
  const uint32_t t = blockIdx.x * kWaves + wave;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  const uint32_t width_words = (tiles + 3u) >> 2;
  const uint32_t stream_total = totals[row];
  if (blockIdx.x == 0 && threadIdx.x == 0 && words && words[row] != 3u + width_words + stream_total + k)
    atomicOr(&status[row], 2u);
  if (t < tiles) {  // wave-uniform
    const LaneGaps g = lane_gaps(msg, k, tiles, t, tile_off + static_cast<size_t>(row) * tiles);
    uint32_t mine = g.n;
#pragma unroll
    for (int s = 0; s < 4; ++s) mine += g.gap[s];
    // coordinates before this lane's first entry: those before the tile + those of the lanes below
    uint32_t pos = tile_sum[static_cast<size_t>(row) * tiles + t] + wave_incl_scan(mine) - mine;
    int32_t* idx = idx_out + static_cast<size_t>(row) * k + t * kWireTile + lane * 4u;
    bool beyond = false;
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (static_cast<uint32_t>(s) < g.n) {
        const uint32_t j = pos + g.gap[s];
        beyond |= j >= d;
        idx[s] = static_cast<int32_t>(j);
        pos = j + 1u;
      }
    if (beyond) atomicOr(&status[row], 4u);
  }
  const uint32_t* values = msg + 3 + width_words + stream_total;
  float* val = val_out + static_cast<size_t>(row) * k;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < k; q += step) val[q] = __uint_as_float(values[q]);
}

__global__ __launch_bounds__(kWG) void k_wire_pack_blocksign(const uint32_t* __restrict__ bits_all,
                                                              const float* __restrict__ scales_all, uint32_t d,
                                                              uint32_t words, uint32_t M,
                                                              uint32_t* __restrict__ messages, int64_t stride,
                                                              uint32_t* __restrict__ words_out) {
  const uint32_t row = blockIdx.y;
  uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    msg[0] = 2u;
    msg[1] = d;
    msg[2] = M;
    words_out[row] = 3u + words + M;
  }
  const uint32_t* bits = bits_all + static_cast<size_t>(row) * words;
  const float* mu = scales_all + static_cast<size_t>(row) * M;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t w = blockIdx.x * kWG + threadIdx.x; w < words; w += step) msg[3 + w] = bits[w];
  for (uint32_t b = blockIdx.x * kWG + threadIdx.x; b < M; b += step) msg[3 + words + b] = __float_as_uint(mu[b]);
}

__global__ __launch_bounds__(kWG) void k_wire_unpack_blocksign(const uint32_t* __restrict__ messages, int64_t stride,
                                                                const uint32_t* __restrict__ words_in, uint32_t d,
                                                                uint32_t words, uint32_t M,
                                                                uint32_t* __restrict__ bits_out,
                                                                float* __restrict__ scales_out,
                                                                uint32_t* __restrict__ status) {
  const uint32_t row = blockIdx.y;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    uint32_t st = 0;
    if (msg[0] != 2u || msg[1] != d || msg[2] != M) st |= 1u;
    else if (words_in && words_in[row] != 3u + words + M) st |= 2u;
    status[row] = st;
  }
  uint32_t* bits = bits_out + static_cast<size_t>(row) * words;
  float* mu = scales_out + static_cast<size_t>(row) * M;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t w = blockIdx.x * kWG + threadIdx.x; w < words; w += step) bits[w] = msg[3 + w];
  for (uint32_t b = blockIdx.x * kWG + threadIdx.x; b < M; b += step) mu[b] = __uint_as_float(msg[3 + words + b]);
}

#define COMPAMS_CHECK_LAUNCH()                    \
  do {                                            \
    hipError_t err__ = hipGetLastError();         \
    if (err__ != hipSuccess) return err__;        \
  } while (0)

uint32_t copy_groups(uint32_t n, uint64_t items) {
  uint64_t g = (items + kWG * 8 - 1) / (kWG * 8);  // eight items per thread
  const uint64_t most = (256 * 8 + n - 1) / n;
  if (g > most) g = most;
  return g < 1 ? 1u : static_cast<uint32_t>(g);
}

}  // namespace

hipError_t wire_encode_topk(const Geometry& geo, const TopkWorkspace& ws, uint32_t* messages, int64_t stride,
                            uint32_t* words_out, hipStream_t stream, Launcher* L) {
  const uint32_t tiles = (geo.k + kWireTile - 1) / kWireTile;
  const dim3 grid((tiles + kWaves - 1) / kWaves, geo.n), wg(kWG);
  launch(L, kSlotWireEncode, k_wire_tile_width, grid, wg, stream, ws.idx, geo.k, tiles, messages, stride,
         ws.wire_tile_off);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireEncode, k_wire_tile_scan, dim3(geo.n), wg, stream, ws.wire_tile_off, tiles, ws.wire_total);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireEncode, k_wire_pack_topk, grid, wg, stream, ws.idx, ws.val, geo.k, tiles, ws.wire_tile_off,
         ws.wire_total, messages, stride, words_out);
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t wire_decode_topk(const Geometry& geo, const TopkWorkspace& ws, const uint32_t* messages, int64_t stride,
                            const uint32_t* words, int32_t* idx_out, float* val_out, uint32_t* status,
                            hipStream_t stream, Launcher* L) {
  const uint32_t tiles = (geo.k + kWireTile - 1) / kWireTile;
  const dim3 grid((tiles + kWaves - 1) / kWaves, geo.n), wg(kWG);
  uint32_t* none = nullptr;
  launch(L, kSlotWireDecode, k_wire_check_topk, dim3(geo.n), wg, stream, messages, stride, geo.k, tiles,
         ws.wire_tile_off, status);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_tile_scan, dim3(geo.n), wg, stream, ws.wire_tile_off, tiles, ws.wire_total);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_tile_sums, grid, wg, stream, messages, stride, geo.k, tiles, ws.wire_tile_off,
         ws.wire_tile_sum);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_tile_scan, dim3(geo.n), wg, stream, ws.wire_tile_sum, tiles, none);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_unpack_topk, grid, wg, stream, messages, stride, words, geo.k, geo.d, tiles,
         ws.wire_tile_off, ws.wire_total, ws.wire_tile_sum, idx_out, val_out, status);
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t wire_encode_blocksign(const Geometry& geo, const BlocksignWorkspace& ws, uint32_t* messages, int64_t stride,
                                 uint32_t* words_out, hipStream_t stream, Launcher* L) {
  const dim3 grid(copy_groups(geo.n, geo.words), geo.n), wg(kWG);
  launch(L, kSlotWireEncode, k_wire_pack_blocksign, grid, wg, stream, ws.bits, ws.scales, geo.d, geo.words,
         geo.num_blocks, messages, stride, words_out);
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t wire_decode_blocksign(const Geometry& geo, const uint32_t* messages, int64_t stride, const uint32_t* words,
                                 uint32_t* bits_out, float* scales_out, uint32_t* status, hipStream_t stream,
                                 Launcher* L) {
  const dim3 grid(copy_groups(geo.n, geo.words), geo.n), wg(kWG);
  launch(L, kSlotWireDecode, k_wire_unpack_blocksign, grid, wg, stream, messages, stride, words, geo.d, geo.words,
         geo.num_blocks, bits_out, scales_out, status);
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

}  // namespace compams
