// The workers' messages as they would go on the wire ("send the compressed gradient to the server" in the
// worker lines of Algorithm 2), and back.  One message per worker, a sequence of 32-bit words:
//
//   top-k      [1, k, b,  gap stream of ceil(k*b/32) words,  k value words]
//              gap_0 = idx_0, gap_q = idx_q - idx_{q-1} - 1; b = number of bits of the largest gap (at least 1);
//              gap q occupies stream bits q*b .. q*b+b-1, least significant bit first; stream bit t is
//              bit (t mod 32) of stream word t div 32; unused bits of the last stream word are 0.
//   block-sign [2, d, M,  ceil(d/32) sign words,  M scale words]
//
// Packing: every stream word is owned by one thread, which gathers the (at most 32) gaps that overlap it, so
// no atomics touch the message.  Unpacking turns gaps back into coordinates with a two-level prefix sum over
// tiles of 4096 entries.  A message that is not well formed never makes a kernel read outside
// [message, message + stride): the entry count and the sizes come from the configuration, not from the words.

#include "compams_device.h"
#include "compams_internal.h"

namespace compams {
namespace {

constexpr int kWirePer = kWireTile / kWG;  // entries per thread in a tile

__device__ __forceinline__ uint32_t gap_of(const int32_t* idx, uint32_t q) {
  const uint32_t cur = static_cast<uint32_t>(idx[q]);
  return q == 0 ? cur : cur - static_cast<uint32_t>(idx[q - 1]) - 1u;
}

__device__ __forceinline__ uint32_t width_of(uint32_t widest) {  // coordinates are below 2^31: at most 31
  return widest ? 32u - static_cast<uint32_t>(__clz(widest)) : 1u;
}

__device__ __forceinline__ uint32_t clamp_width(uint32_t b) { return b < 1u ? 1u : (b > 31u ? 31u : b); }

__device__ __forceinline__ uint32_t stream_words(uint32_t k, uint32_t b) {
  return static_cast<uint32_t>((static_cast<uint64_t>(k) * b + 31u) >> 5);
}

__global__ __launch_bounds__(kWG) void k_wire_gap_max(const int32_t* __restrict__ idx_all, uint32_t k,
                                                       uint32_t* __restrict__ wmax) {
  const uint32_t row = blockIdx.y;
  const int32_t* idx = idx_all + static_cast<size_t>(row) * k;
  uint32_t mx = 0;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < k; q += step) {
    const uint32_t g = gap_of(idx, q);
    mx = g > mx ? g : mx;
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    const uint32_t o = __shfl_xor(mx, s, 64);
    mx = o > mx ? o : mx;
  }
  // one atomic per workgroup: atomics on one word are served one after the other
  __shared__ uint32_t part[kWG / 64];
  if (lane_id() == 0) part[threadIdx.x >> 6] = mx;
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int w = 1; w < kWG / 64; ++w) mx = part[w] > mx ? part[w] : mx;
    if (mx) atomicMax(&wmax[row], mx);
  }
}

__global__ __launch_bounds__(kWG) void k_wire_pack_topk(const int32_t* __restrict__ idx_all,
                                                         const float* __restrict__ val_all, uint32_t k,
                                                         const uint32_t* __restrict__ wmax,
                                                         uint32_t* __restrict__ messages, int64_t stride,
                                                         uint32_t* __restrict__ words_out) {
  const uint32_t row = blockIdx.y;
  const int32_t* idx = idx_all + static_cast<size_t>(row) * k;
  const float* val = val_all + static_cast<size_t>(row) * k;
  const uint32_t b = width_of(wmax[row]);
  const uint32_t P = stream_words(k, b);
  uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    msg[0] = 1u;
    msg[1] = k;
    msg[2] = b;
    words_out[row] = 3u + P + k;
  }
  uint32_t* stream = msg + 3;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t w = blockIdx.x * kWG + threadIdx.x; w < P; w += step) {
    const uint64_t lo = static_cast<uint64_t>(w) * 32u;
    const uint32_t q0 = static_cast<uint32_t>(lo / b);
    uint64_t q1 = (lo + 31u) / b;
    if (q1 > k - 1u) q1 = k - 1u;
    uint32_t word = 0;
    for (uint32_t q = q0; q <= static_cast<uint32_t>(q1); ++q) {
      const uint32_t g = gap_of(idx, q);
      const int64_t sh = static_cast<int64_t>(static_cast<uint64_t>(q) * b) - static_cast<int64_t>(lo);
      word |= sh >= 0 ? (g << sh) : (g >> (-sh));  // |sh| <= 31
    }
    stream[w] = word;
  }
  uint32_t* values = stream + P;
  for (uint32_t q = blockIdx.x * kWG + threadIdx.x; q < k; q += step) values[q] = __float_as_uint(val[q]);
}

// Gap q of a stream of P words (q < k, so the field lies inside the stream).
__device__ __forceinline__ uint32_t field_of(const uint32_t* __restrict__ stream, uint32_t P, uint32_t q, uint32_t b) {
  const uint64_t pos = static_cast<uint64_t>(q) * b;
  const uint32_t w = static_cast<uint32_t>(pos >> 5), sh = static_cast<uint32_t>(pos & 31u);
  uint64_t two = stream[w];
  if (w + 1 < P) two |= static_cast<uint64_t>(stream[w + 1]) << 32;
  return static_cast<uint32_t>(two >> sh) & ((1u << b) - 1u);
}

// status[row]: 0 well formed; bit 0: not a message of this kind and size; bit 1: length differs; bit 2 (set
// while unpacking): a coordinate at or beyond d.
__global__ void k_wire_check_topk(const uint32_t* __restrict__ messages, int64_t stride,
                                  const uint32_t* __restrict__ words, uint32_t n, uint32_t k,
                                  uint32_t* __restrict__ status) {
  const uint32_t row = blockIdx.x * blockDim.x + threadIdx.x;
  if (row >= n) return;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  uint32_t st = 0;
  const uint32_t b = msg[2];
  if (msg[0] != 1u || msg[1] != k || b < 1u || b > 31u) st |= 1u;
  else if (words && words[row] != 3u + stream_words(k, b) + k) st |= 2u;
  status[row] = st;
}

__global__ __launch_bounds__(kWG) void k_wire_tile_sums(const uint32_t* __restrict__ messages, int64_t stride,
                                                         uint32_t k, uint32_t tiles_per_row,
                                                         uint32_t* __restrict__ tiles) {
  __shared__ uint32_t scratch[kWG / 64 + 1];
  const uint32_t row = blockIdx.y, t = blockIdx.x;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  const uint32_t b = clamp_width(msg[2]);
  const uint32_t P = stream_words(k, b);
  const uint32_t first = t * kWireTile + threadIdx.x * kWirePer;
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < kWirePer; ++i)
    if (first + i < k) sum += field_of(msg + 3, P, first + i, b) + 1u;
  uint32_t total;
  (void)block_excl_scan<kWG>(sum, scratch, &total);
  if (threadIdx.x == 0) tiles[static_cast<size_t>(row) * tiles_per_row + t] = total;
}

// In place: tile totals -> what lies before each tile.  One workgroup per row.
__global__ __launch_bounds__(kWG) void k_wire_tile_scan(uint32_t* __restrict__ tiles, uint32_t tiles_per_row) {
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
}

__global__ __launch_bounds__(kWG) void k_wire_unpack_topk(const uint32_t* __restrict__ messages, int64_t stride,
                                                           uint32_t k, uint32_t d, uint32_t tiles_per_row,
                                                           const uint32_t* __restrict__ tiles,
                                                           int32_t* __restrict__ idx_out, float* __restrict__ val_out,
                                                           uint32_t* __restrict__ status) {
  __shared__ uint32_t scratch[kWG / 64 + 1];
  const uint32_t row = blockIdx.y, t = blockIdx.x;
  const uint32_t* msg = messages + static_cast<int64_t>(row) * stride;
  const uint32_t b = clamp_width(msg[2]);
  const uint32_t P = stream_words(k, b);
  const uint32_t first = t * kWireTile + threadIdx.x * kWirePer;
  uint32_t gap[kWirePer];
  uint32_t sum = 0;
#pragma unroll
  for (int i = 0; i < kWirePer; ++i) {
    gap[i] = 0;
    if (first + i < k) {
      gap[i] = field_of(msg + 3, P, first + i, b);
      sum += gap[i] + 1u;
    }
  }
  uint32_t total;
  uint32_t pos = tiles[static_cast<size_t>(row) * tiles_per_row + t] + block_excl_scan<kWG>(sum, scratch, &total);
  int32_t* idx = idx_out + static_cast<size_t>(row) * k;
  bool beyond = false;
#pragma unroll
  for (int i = 0; i < kWirePer; ++i)
    if (first + i < k) {
      const uint32_t j = pos + gap[i];  // coordinates before this entry + its gap
      beyond |= j >= d;
      idx[first + i] = static_cast<int32_t>(j);
      pos = j + 1u;
    }
  if (beyond) atomicOr(&status[row], 4u);
  const uint32_t* values = msg + 3 + P;
  float* val = val_out + static_cast<size_t>(row) * k;
  for (uint32_t q = t * kWireTile + threadIdx.x; q < (t + 1) * kWireTile && q < k; q += kWG)
    val[q] = __uint_as_float(values[q]);
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
  hipError_t err = fill_u32(ws.wire_max, geo.n, 0u, stream);
  if (err != hipSuccess) return err;
  const dim3 grid(copy_groups(geo.n, geo.k), geo.n), wg(kWG);
  launch(L, kSlotWireEncode, k_wire_gap_max, grid, wg, stream, ws.idx, geo.k, ws.wire_max);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireEncode, k_wire_pack_topk, grid, wg, stream, ws.idx, ws.val, geo.k, ws.wire_max, messages, stride,
         words_out);
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t wire_decode_topk(const Geometry& geo, const TopkWorkspace& ws, const uint32_t* messages, int64_t stride,
                            const uint32_t* words, int32_t* idx_out, float* val_out, uint32_t* status,
                            hipStream_t stream, Launcher* L) {
  const uint32_t tiles = (geo.k + kWireTile - 1) / kWireTile;
  const dim3 wg(kWG), grid(tiles, geo.n);
  launch(L, kSlotWireDecode, k_wire_check_topk, dim3((geo.n + kWG - 1) / kWG), wg, stream, messages, stride, words,
         geo.n, geo.k, status);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_tile_sums, grid, wg, stream, messages, stride, geo.k, tiles, ws.wire_tiles);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_tile_scan, dim3(geo.n), wg, stream, ws.wire_tiles, tiles);
  COMPAMS_CHECK_LAUNCH();
  launch(L, kSlotWireDecode, k_wire_unpack_topk, grid, wg, stream, messages, stride, geo.k, geo.d, tiles,
         ws.wire_tiles, idx_out, val_out, status);
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
