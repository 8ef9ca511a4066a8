// Block-Sign with error feedback (Definition 2 inside the worker lines of Algorithm 2) for gfx950, and
// the server lines for sign/scale messages.
//
// Per worker row and block B:  mu = ||x_B||_1 / d_B with x = e + g, message = (one sign bit per
// coordinate, mu), residual e = x - sign(x) * mu, where sign(x) = -1 iff x < 0.
//
// The block L1 norm is accumulated EXACTLY, so that the scale does not depend on how the sum was
// split over lanes, wavefronts and workgroups: every |x| is a 24-bit integer times a power of two;
// it is added into a fixed-point number whose 32-bit digits are carried in 64-bit words (room for
// 2^32 additions before a digit could overflow).  Integer addition commutes, so integer atomics leave
// the result unique.  Inside a lane the additions run in fp64 over windows of exponents narrow enough that
// no addition rounds.  The sum is rounded once to double, divided by d_B in double and rounded to fp32.
//
// Pass 1 forms x (stored in place of e), its sign words and the sums, a small kernel turns sums into
// scales, and the server kernel adds the n workers' +-mu in worker order before the AMSGrad update.  The
// residual e = x - sign(x) * mu is applied by the next step's pass 1 as it reads e (or by the stand-alone
// residual kernel when e is asked for).

#include <type_traits>

#include "compams_device.h"
#include "compams_internal.h"

namespace compams {
namespace {

// |x| = mant * 2^(sh - 149), mant < 2^24, sh in [0, 253]; digit w = sh / 32 gets the low 32 bits of
// mant << (sh % 32), digit w + 1 the rest.
struct Fixed {
  uint32_t w;
  uint32_t lo;
  uint32_t hi;
  uint32_t special;  // 1: infinity, 2: NaN
};

__device__ __forceinline__ Fixed to_fixed(uint32_t bits) {
  const uint32_t key = bits & 0x7fffffffu;
  const uint32_t ex = key >> 23, frac = key & 0x7fffffu;
  Fixed f;
  const bool nonfinite = ex == 255u;
  const uint32_t mant = nonfinite ? 0u : (ex ? (frac | 0x800000u) : frac);
  const uint32_t sh = ex ? ex - 1 : 0;
  const uint64_t val = static_cast<uint64_t>(mant) << (sh & 31u);
  f.w = nonfinite ? 0u : sh >> 5;
  f.lo = static_cast<uint32_t>(val);
  f.hi = static_cast<uint32_t>(val >> 32);
  f.special = nonfinite ? (frac ? 2u : 1u) : 0u;
  return f;
}

__device__ __forceinline__ uint64_t wave_sum_u64(uint64_t v) {
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    const uint32_t lo = __shfl_xor(static_cast<uint32_t>(v), s, 64);
    const uint32_t hi = __shfl_xor(static_cast<uint32_t>(v >> 32), s, 64);
    v += (static_cast<uint64_t>(hi) << 32) | lo;
  }
  return v;
}

__device__ __forceinline__ void atomic_add_u64(uint64_t* p, uint64_t v) {
  atomicAdd(reinterpret_cast<unsigned long long*>(p), static_cast<unsigned long long>(v));
}

// Register accumulator of a lane: an fp64 sum over a window of kWinSpan binary exponents, placed by the
// wavefront (wave-uniform) so that it ends at the largest magnitude of the coordinates it is about to add.
// Every |x| in the window is an integer below 2^(24 + kWinSpan - 1) = 2^45 times the window's quantum
// 2^(lowest exponent - 150), so the fp64 sum of up to kWinAdds = 2^8 of them (a lane adds 16) is below 2^53
// quanta: every addition is exact and their order does not matter.  The sum then becomes an integer again, is
// added over the wavefront and goes to the global digits.  Entries below the window (more than 2^21 below the
// largest magnitude: rare) and non-finite ones go straight to the global digits and flags.
// "Exponent" here is the effective one: max(biased exponent, 1), so that subnormals share the quantum of
// the smallest normal numbers; |x| = mantissa * 2^(exponent - 150).
// (One window of 22 exponents replaced two of 17: per entry one compare, one select, one conversion and one
// addition instead of twice that and a second range test.)
constexpr uint32_t kWinSpan = 22;
constexpr uint32_t kWinAdds = 256;
static_assert(24 + kWinSpan - 1 + 8 <= 53, "a window's sum must stay an exact integer in fp64");

struct WaveAcc {
  double sum;       // sum of the window
  uint32_t eh;      // window: exponents eh .. eh + kWinSpan - 1
  uint32_t klo;     // magnitude keys klo .. klo + kspan - 1 lie in the window (eh == 1: from key 0, the
  uint32_t kspan;   // subnormals and zero included)
};

__device__ __forceinline__ void acc_reset(WaveAcc& A) {
  A.sum = 0.0; A.eh = 1; A.klo = 0; A.kspan = 0;
}

// Places the window so that it ends `headroom` exponents above the largest finite magnitude key kmax_key
// seen so far (wave-uniform).  Its top exponent is at most 254: infinities and NaNs are never inside.
__device__ __forceinline__ void acc_place(WaveAcc& A, uint32_t kmax_key, uint32_t headroom) {
  uint32_t top = kmax_key >> 23;
  top = top ? top : 1u;
  top = top + headroom > 254u ? 254u : top + headroom;
  A.eh = top >= kWinSpan ? top - (kWinSpan - 1u) : 1u;
  A.klo = A.eh == 1u ? 0u : A.eh << 23;
  A.kspan = ((A.eh + kWinSpan) << 23) - A.klo;
}

// The window's sum as an integer number of quanta 2^(e_low - 150), added over the wavefront and then, by
// lane 0, into the digits: bit position e_low - 1 above 2^-149, i.e. digit (e_low - 1) / 32 and up.
// In line: once per wavefront, and a call would pass its arguments through scratch memory.
__device__ __forceinline__ void window_to_digits(double sum, uint32_t e_low, uint64_t* digits) {
  const uint64_t mine = static_cast<uint64_t>(ldexp(sum, 150 - static_cast<int>(e_low)));  // exact, below 2^53
  const uint64_t all = wave_sum_u64(mine);                                                 // below 2^59
  if (lane_id() == 0 && all) {
    const uint32_t sh = e_low - 1u, w = sh >> 5, s = sh & 31u;
    const uint64_t low = all << s, high = s ? all >> (64u - s) : 0ull;
    const uint64_t d0 = low & 0xffffffffull, d1 = low >> 32;
    if (d0) atomic_add_u64(digits + w, d0);
    if (d1) atomic_add_u64(digits + w + 1, d1);
    if (high) atomic_add_u64(digits + w + 2, high);  // w <= 7: still inside the kLimbs digits
  }
}

// One entry straight into the global digits (or the flags for non-finite values).  Out of line: rare.
__device__ __noinline__ void add_direct(uint32_t bits, uint64_t* digits, uint32_t* special) {
  const Fixed f = to_fixed(bits);
  if (f.special) atomicOr(special, f.special);
  else {
    if (f.lo) atomic_add_u64(digits + f.w, f.lo);
    if (f.hi) atomic_add_u64(digits + f.w + 1, f.hi);
  }
}

// Adds the four entries of a lane's quad.  Branch-free for entries inside the window; everything else
// leaves through one wave-uniform branch.
__device__ __forceinline__ void acc_add4(WaveAcc& A, const uint32_t bits[4], const bool ok[4], uint64_t* digits,
                                         uint32_t* special) {
  bool rare[4];
  bool any = false;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    const uint32_t key = bits[s] & 0x7fffffffu;
    const bool in = ok[s] && key - A.klo < A.kspan;  // unsigned: false below the window
    uint32_t ksel = in ? key : 0u;
    asm volatile("" : "+v"(ksel));  // select the 32-bit key, then convert (not: convert, then select both halves)
    A.sum += static_cast<double>(__uint_as_float(ksel));  // |x|, exactly
    rare[s] = ok[s] && !in && key != 0u;
    any |= rare[s];
  }
  if (ballot64(any) != 0) {
#pragma unroll
    for (int s = 0; s < 4; ++s)
      if (rare[s]) add_direct(bits[s], digits, special);
  }
}

// Largest b with off[b] <= j, starting the walk at hint (off[hint] <= j must hold).
__device__ __forceinline__ uint32_t block_of(const uint32_t* __restrict__ off, uint32_t hint, uint32_t j) {
  uint32_t b = hint;
  while (off[b + 1] <= j) ++b;
  return b;
}

// ---------------------------------------------------------------------------------------------
// Exact rounding of a fixed-point sum to double (nearest, ties to even).
// The value is (w2:w1:w0 as a 192-bit integer) * 2^lsb_exp; extra_sticky says that non-zero bits exist
// below bit 0 (they can only matter as a sticky bit).
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ double fixed192_to_double(uint64_t w0, uint64_t w1, uint64_t w2, int lsb_exp,
                                                     bool extra_sticky) {
  int top;
  if (w2) top = 128 + 63 - __clzll(static_cast<long long>(w2));
  else if (w1) top = 64 + 63 - __clzll(static_cast<long long>(w1));
  else if (w0) top = 63 - __clzll(static_cast<long long>(w0));
  else return 0.0;
  if (top <= 52) return ldexp(static_cast<double>(w0), lsb_exp);  // fits a double exactly (extra_sticky is then false)
  const int sh = top - 52;  // bits dropped: 1 .. 139
  auto word = [&](int i) -> uint64_t { return i == 0 ? w0 : (i == 1 ? w1 : (i == 2 ? w2 : 0ull)); };
  const int wi = sh >> 6, bi = sh & 63;
  uint64_t kept = bi ? ((word(wi) >> bi) | (word(wi + 1) << (64 - bi))) : word(wi);
  const int gp = sh - 1, gw = gp >> 6, gb = gp & 63;
  const bool guard = ((word(gw) >> gb) & 1ull) != 0;
  bool sticky = extra_sticky || (word(gw) & ((1ull << gb) - 1ull)) != 0;
  if (gw >= 1) sticky = sticky || w0 != 0;
  if (gw >= 2) sticky = sticky || w1 != 0;
  if (guard && (sticky || (kept & 1ull))) ++kept;  // may reach 2^53: still exact
  return ldexp(static_cast<double>(kept), lsb_exp + sh);
}

// ---------------------------------------------------------------------------------------------
// Pass 1: x = e + g -> e, the sign words of x and the exact block sums.
// ---------------------------------------------------------------------------------------------
constexpr int kBsBatch = 4;
constexpr int kQuarter = kRounds / kWaves;  // rounds of a chunk per wavefront when a workgroup takes one chunk
static_assert(kQuarter == kBsBatch, "a wavefront's quarter of a chunk is one batch of loads");
static_assert(kQuarter * 4 <= static_cast<int>(kWinAdds), "additions per lane into one window");

struct BsBatch {
  float4 g[kBsBatch], e[kBsBatch];
};

template <bool FULL>
__device__ __forceinline__ void bs_load_batch_t(BsBatch& B, const float* __restrict__ gr, const float* __restrict__ er,
                                                uint32_t c, int r0, uint32_t d) {
  const uint32_t lane = lane_id();
#pragma unroll
  for (int u = 0; u < kBsBatch; ++u) {
    const uint32_t j = c * kChunk + (r0 + u) * 256 + lane * 4;
    if (FULL) {
      B.g[u] = load_stream4(gr + j);
      B.e[u] = load_stream4(er + j);
    } else {
      B.g[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      B.e[u] = B.g[u];
      if (j < d) {
        B.g[u] = load_stream4(gr + j);
        B.e[u] = load_stream4(er + j);
      }
    }
  }
}


// One round (256 coordinates from j0 on) that straddles block boundaries.  The blocks that meet the round are
// the same for every lane, so they are gone through one after the other (from block b, the block of the round's
// first coordinate, on): the block's previous mean is taken off the residuals of its coordinates (PEND), and
// after x has been formed and stored the magnitudes of its coordinates are summed in a register window and go
// to its digits like any other partial sum.  A block with at most 8 coordinates in the round adds them one by
// one instead (a layout of one-coordinate blocks would otherwise make 256 trips through the wavefront-wide
// sum).  Rare -- a few rounds per row in layouts worth the name -- and out of line.
template <bool PEND>
__device__ __noinline__ void straddling_round(float4 g4, float4 e4, uint32_t j0, uint32_t d, uint32_t b,
                                              const uint32_t* __restrict__ off, const float* __restrict__ mur,
                                              float* __restrict__ er, uint32_t* __restrict__ bitr, uint32_t words,
                                              uint64_t* accr, size_t blk_digits, uint32_t replica, uint32_t* specr) {
  const uint32_t lane = lane_id();
  const uint32_t j = j0 + lane * 4;
  const uint32_t j_end = j0 + 256 < d ? j0 + 256 : d;
  const bool ok[4] = {j < d, j + 1 < d, j + 2 < d, j + 3 < d};
  float ev[4] = {e4.x, e4.y, e4.z, e4.w};
  const float gv[4] = {g4.x, g4.y, g4.z, g4.w};
  if (PEND) {
    for (uint32_t bb = b; table_u32(off, bb) < j_end; ++bb) {  // wave-uniform
      const uint32_t lo = table_u32(off, bb), hi = table_u32(off, bb + 1);
      const float mu = table_f32(mur, bb);
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (ok[s] && j + s >= lo && j + s < hi) ev[s] = ev[s] - (ev[s] < 0.0f ? -mu : mu);
    }
  }
  float xv[4];
  uint32_t nib = 0;
#pragma unroll
  for (int s = 0; s < 4; ++s) {
    xv[s] = ok[s] ? ev[s] + gv[s] : ev[s];  // columns at and beyond d keep their contents
    nib |= (ok[s] && xv[s] < 0.0f ? 1u : 0u) << s;
  }
  if (ok[0]) store_stream4(er + j, make_float4(xv[0], xv[1], xv[2], xv[3]));
  const uint32_t word = or_over_8_lanes(nib << ((lane & 7u) * 4u));
  const uint32_t widx = (j0 >> 5) + (lane >> 3);
  if ((lane & 7u) == 0 && widx < words) bitr[widx] = word;
  const uint32_t bits[4] = {__float_as_uint(xv[0]), __float_as_uint(xv[1]), __float_as_uint(xv[2]),
                            __float_as_uint(xv[3])};
  for (uint32_t bb = b; table_u32(off, bb) < j_end; ++bb) {  // wave-uniform
    const uint32_t lo = table_u32(off, bb), hi = table_u32(off, bb + 1);
    bool in[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) in[s] = ok[s] && j + s >= lo && j + s < hi;
    uint64_t* dg = accr + static_cast<size_t>(bb) * blk_digits;
    const uint32_t first = lo > j0 ? lo : j0, last = hi < j_end ? hi : j_end;
    if (last - first <= 8) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (in[s]) add_direct(bits[s], dg, specr + bb);
    } else {
      uint32_t kmax = 0;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint32_t key = bits[s] & 0x7fffffffu;
        if (in[s] && key < 0x7f800000u && key > kmax) kmax = key;
      }
#pragma unroll
      for (int s = 32; s >= 1; s >>= 1) {
        const uint32_t o = __shfl_xor(kmax, s, 64);
        kmax = o > kmax ? o : kmax;
      }
      WaveAcc A;
      acc_reset(A);
      acc_place(A, uniform_u32(kmax), 0);
      acc_add4(A, bits, in, dg + static_cast<size_t>(replica) * kLimbs, specr + bb);
      window_to_digits(A.sum, A.eh, dg + static_cast<size_t>(replica) * kLimbs);
    }
  }
}

// ---------------------------------------------------------------------------------------------
// First pass for general block layouts as a grid of short workgroups: a workgroup takes ONE chunk and ends,
// wavefront w takes rounds 4w .. 4w+3 of it (plain streaming kernels of this shape move the same traffic at
// 6.1-6.4 TB/s on MI355X, workgroups that walk many chunks at 5.4-5.7 TB/s).  A quarter that lies inside one
// block -- all but a few per row -- is summed in a register window placed by the quarter's own largest
// magnitude and goes to the block's digits with at most three atomics per wavefront; a quarter that straddles
// block boundaries goes out of line through the blocks it meets.  The pending residual update of the previous
// step is applied to e as it is read.
// ---------------------------------------------------------------------------------------------
template <bool PEND>
__global__ __launch_bounds__(kWG) void k_bs_lean(const float* __restrict__ g, float* __restrict__ e, Geometry geo,
                                                  BlocksignWorkspace ws) {
  const uint32_t c = blockIdx.x, row = blockIdx.y;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  const float* gr = g + static_cast<int64_t>(row) * geo.ld;
  float* er = e + static_cast<int64_t>(row) * geo.ld;
  const uint32_t* __restrict__ off = ws.offsets;
  const float* mur = ws.scales + static_cast<size_t>(row) * geo.num_blocks;  // previous step's means (PEND)
  uint32_t* bitr = ws.bits + static_cast<size_t>(row) * geo.words;
  const size_t blk_digits = static_cast<size_t>(ws.acc_replicas) * kLimbs;  // digits of one (row, block): all replicas
  uint64_t* accr = ws.acc + static_cast<size_t>(row) * geo.num_blocks * blk_digits;
  uint32_t* specr = ws.special + static_cast<size_t>(row) * geo.num_blocks;
  const uint32_t d = geo.d;
  const uint32_t q0 = c * kChunk + wave * (kQuarter * 256);  // first coordinate of this wavefront's quarter
  if (q0 >= d) return;                                       // wave-uniform; no barrier in this kernel
  const bool full = (c + 1) * static_cast<uint64_t>(kChunk) <= d;
  BsBatch cur;
  if (full) bs_load_batch_t<true>(cur, gr, er, c, wave * kQuarter, d);
  else bs_load_batch_t<false>(cur, gr, er, c, wave * kQuarter, d);
  uint32_t b = table_u32(ws.chunk_block, c);
  while (table_u32(off, b + 1) <= q0) ++b;  // block of the quarter's first coordinate
  const uint32_t q_end = q0 + kQuarter * 256 < d ? q0 + kQuarter * 256 : d;
  if (table_u32(off, b + 1) < q_end) {  // the quarter straddles block boundaries (a scalar condition)
#pragma unroll  // (a run-time index into the batch would put it into scratch memory)
    for (int u = 0; u < kQuarter; ++u) {
      const uint32_t j0 = q0 + u * 256;
      if (j0 >= d) break;
      while (table_u32(off, b + 1) <= j0) ++b;
      straddling_round<PEND>(cur.g[u], cur.e[u], j0, d, b, off, mur, er, bitr, geo.words, accr, blk_digits,
                             c % ws.acc_replicas, specr);
    }
    return;
  }
  const float mu_b = PEND ? table_f32(mur, b) : 0.0f;
  uint32_t bits[kQuarter][4];
  uint32_t kmax = 0;
#pragma unroll
  for (int u = 0; u < kQuarter; ++u) {
    const uint32_t j0 = q0 + u * 256;
    const uint32_t j = j0 + lane * 4;
    const bool ok[4] = {full || j < d, full || j + 1 < d, full || j + 2 < d, full || j + 3 < d};
    float ev[4] = {cur.e[u].x, cur.e[u].y, cur.e[u].z, cur.e[u].w};
    const float gv[4] = {cur.g[u].x, cur.g[u].y, cur.g[u].z, cur.g[u].w};
    if (PEND) {
#pragma unroll
      for (int s = 0; s < 4; ++s)
        if (ok[s]) ev[s] = ev[s] - (ev[s] < 0.0f ? -mu_b : mu_b);
    }
    float xv[4];
    uint32_t nib = 0;
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      xv[s] = ok[s] ? ev[s] + gv[s] : ev[s];  // columns at and beyond d keep their contents
      nib |= (ok[s] && xv[s] < 0.0f ? 1u : 0u) << s;
    }
    if (ok[0]) store_stream4(er + j, make_float4(xv[0], xv[1], xv[2], xv[3]));
    if (full || j0 < d) {  // wave-uniform
      const uint32_t word = or_over_8_lanes(nib << ((lane & 7u) * 4u));
      const uint32_t widx = (j0 >> 5) + (lane >> 3);
      if ((lane & 7u) == 0 && (full || widx < geo.words)) bitr[widx] = word;
    }
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      bits[u][s] = ok[s] ? __float_as_uint(xv[s]) : 0u;  // a coordinate beyond d adds nothing
      const uint32_t key = bits[u][s] & 0x7fffffffu;
      if (key < 0x7f800000u && key > kmax) kmax = key;
    }
  }
#pragma unroll
  for (int s = 32; s >= 1; s >>= 1) {
    const uint32_t o = __shfl_xor(kmax, s, 64);
    kmax = o > kmax ? o : kmax;
  }
  // the window ends at the quarter's largest magnitude: 16 additions per lane, exact
  WaveAcc A;
  acc_reset(A);
  acc_place(A, uniform_u32(kmax), 0);
  // a large block receives the sums of thousands of wavefronts: they go to one of several sets of digits, chosen
  // by the chunk (atomics to one address are performed one after the other), which the finalize kernel adds up
  uint64_t* dg = accr + static_cast<size_t>(b) * blk_digits + static_cast<size_t>(c % ws.acc_replicas) * kLimbs;
  const bool all[4] = {true, true, true, true};
#pragma unroll
  for (int u = 0; u < kQuarter; ++u) acc_add4(A, bits[u], all, dg, specr + b);
  window_to_digits(A.sum, A.eh, dg);
}

// ---------------------------------------------------------------------------------------------
// Scales: per (row, block) add up the sets of digits (a thread when there is one set, else a wavefront with a
// lane per set), normalise them, round the sum to double (nearest, ties to even), divide by the block length,
// round to fp32.  Clears the digits for the next step.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWG) void k_bs_finalize(Geometry geo, BlocksignWorkspace ws) {
  const size_t total = static_cast<size_t>(geo.n) * geo.num_blocks;
  const uint32_t R = ws.acc_replicas;  // sets of digits per (row, block)
  size_t t;
  uint64_t word[kLimbs];
  if (R == 1) {  // a thread per (row, block)
    t = static_cast<size_t>(blockIdx.x) * kWG + threadIdx.x;
    if (t >= total) return;
    uint64_t* dg = ws.acc + t * kLimbs;
#pragma unroll
    for (int i = 0; i < kLimbs; ++i) {
      word[i] = dg[i];
      dg[i] = 0;
    }
  } else {  // a wavefront per (row, block): lane r brings replica r, the sums are taken over the wavefront
    t = static_cast<size_t>(blockIdx.x) * kWaves + (threadIdx.x >> 6);
    if (t >= total) return;
    const uint32_t lane = lane_id();
    uint64_t* dg = ws.acc + (t * R + lane) * kLimbs;
#pragma unroll
    for (int i = 0; i < kLimbs; ++i) {
      uint64_t mine = 0;
      if (lane < R) {
        mine = dg[i];
        dg[i] = 0;
      }
      word[i] = wave_sum_u64(mine);  // every digit word is far below 2^53 (see window_to_digits): no wrap
    }
    if (lane != 0) return;
  }
  const uint32_t b = static_cast<uint32_t>(t % geo.num_blocks);
  uint32_t digit[kLimbs + 1];
  uint64_t carry = 0;
#pragma unroll
  for (int i = 0; i < kLimbs; ++i) {
    const uint64_t v = word[i] + carry;
    digit[i] = static_cast<uint32_t>(v);
    carry = v >> 32;
  }
  digit[kLimbs] = static_cast<uint32_t>(carry);
  const uint32_t sp = ws.special[t];
  ws.special[t] = 0;
  const double len = static_cast<double>(ws.offsets[b + 1] - ws.offsets[b]);
  double sum;
  if (sp & 2u) sum = __longlong_as_double(0x7ff8000000000000ll);
  else if (sp & 1u) sum = __longlong_as_double(0x7ff0000000000000ll);
  else {
    // the four highest non-zero digits carry every bit a double can hold; the rest is a sticky bit
    int top = 0;
#pragma unroll
    for (int i = 1; i <= kLimbs; ++i)
      if (digit[i]) top = i;
    const int low = top >= 3 ? top - 3 : 0;
    uint32_t q[4] = {0, 0, 0, 0};
    bool below = false;
#pragma unroll
    for (int i = 0; i <= kLimbs; ++i) {
      if (i >= low && i < low + 4) q[i - low] = digit[i];
      else if (i < low && digit[i]) below = true;
    }
    const uint64_t w0 = (static_cast<uint64_t>(q[1]) << 32) | q[0], w1 = (static_cast<uint64_t>(q[3]) << 32) | q[2];
    sum = fixed192_to_double(w0, w1, 0, 32 * low - 149, below);
  }
  ws.scales[t] = static_cast<float>(sum / len);
}

// ---------------------------------------------------------------------------------------------
// The residual  e = x - sign(x) * mu  on its own (and the sign words once more): when the caller asks for e
// while the update is still pending.  One wavefront per chunk.  Eight lanes (32 coordinates) share one word
// of the bit map.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWG) void k_bs_pass2(float* __restrict__ e, Geometry geo, BlocksignWorkspace ws) {
  const uint32_t row = blockIdx.y;
  float* er = e + static_cast<int64_t>(row) * geo.ld;
  const uint32_t* __restrict__ off = ws.offsets;
  const float* __restrict__ mur = ws.scales + static_cast<size_t>(row) * geo.num_blocks;
  uint32_t* bitr = ws.bits + static_cast<size_t>(row) * geo.words;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  const uint32_t stride = gridDim.x * kWaves;
  const uint32_t d = geo.d;
  for (uint32_t c = blockIdx.x * kWaves + wave; c < geo.num_chunks; c += stride) {
    uint32_t b = ws.chunk_block[c];
#pragma unroll 1
    for (int r0 = 0; r0 < kRounds; r0 += kBsBatch) {
      if (c * kChunk + r0 * 256 >= d) break;  // wave-uniform
      float4 xb[kBsBatch];
#pragma unroll
      for (int u = 0; u < kBsBatch; ++u) {
        const uint32_t j = c * kChunk + (r0 + u) * 256 + lane * 4;
        xb[u] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (j < d) xb[u] = load_stream4(er + j);
      }
#pragma unroll
      for (int u = 0; u < kBsBatch; ++u) {
        const uint32_t j0 = c * kChunk + (r0 + u) * 256;
        if (j0 >= d) break;
        const uint32_t j = j0 + lane * 4;
        const bool in = j < d;
        const bool ok[4] = {in, j + 1 < d, j + 2 < d, j + 3 < d};
        while (off[b + 1] <= j0) ++b;
        const uint32_t j_end = (j0 + 256 < d) ? j0 + 256 : d;
        float mu[4];
        if (off[b + 1] >= j_end) {
          const float m0 = mur[b];
          mu[0] = mu[1] = mu[2] = mu[3] = m0;
        } else {
#pragma unroll
          for (int s = 0; s < 4; ++s) mu[s] = ok[s] ? mur[block_of(off, b, j + s)] : 0.0f;
        }
        float xv[4] = {xb[u].x, xb[u].y, xb[u].z, xb[u].w};
        uint32_t nib = 0;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const bool neg = ok[s] && xv[s] < 0.0f;
          nib |= (neg ? 1u : 0u) << s;
          if (ok[s]) xv[s] = xv[s] - (neg ? -mu[s] : mu[s]);
        }
        if (in) store_stream4(er + j, make_float4(xv[0], xv[1], xv[2], xv[3]));
        const uint32_t word = or_over_8_lanes(nib << ((lane & 7u) * 4u));
        const uint32_t widx = (j0 >> 5) + (lane >> 3);
        if ((lane & 7u) == 0 && widx < geo.words) bitr[widx] = word;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Server lines for sign/scale messages: gbar_j = (sum_i s_ij * mu_i,b(j)) / n in worker order, then
// AMSGrad.  A workgroup per chunk of coordinates, each of its wavefronts a share of KQ rounds.
// ---------------------------------------------------------------------------------------------
constexpr int kBsWorkers = 8;  // workers whose sign words and scales are requested together (rounds that meet block ends)

// Wavefronts per chunk.  With the whole state cached a wavefront takes two rounds and asks for everything it
// needs at once; with state that streams from HBM four rounds, the next one's state requested while one is
// updated (ResNet-18 shape, all cached: 61 against 66 us; GPT-2 shape, all streamed: 666 against 685 us).
constexpr int bs_server_split(int cached_arrays) { return cached_arrays == 4 ? 8 : 4; }

// Sums of a share of KQ rounds that lies inside block b and inside the row: sum[r][s] for the lane's four
// coordinates of round r.  A worker's sign words of the share are KQ * 8 consecutive words, which a group of
// lanes requests once, several workers per load; a round then takes its word out of the holder's register.
// (Asked for round by round, 32 bytes at a time with the state's traffic in between, the lines were fetched
// 3.4 times over.)  One scale per worker serves all rounds.  Worker order, as everywhere.
template <int KQ>
__device__ __forceinline__ void bs_share_sums(float (&sum)[KQ][4], const Geometry& geo, const BlocksignWorkspace& ws,
                                              uint32_t b, uint32_t q0, uint32_t lane) {
  constexpr int kShareWords = KQ * 8;           // sign words of one worker for the share
  constexpr int kPerLoad = 64 / kShareWords;    // workers whose words one load of the wavefront brings in
  constexpr int kTrip = KQ == 2 ? 16 : 8;       // workers per trip: kTrip / kPerLoad loads, kTrip scales
  static_assert(kShareWords * kPerLoad == 64 && kTrip % kPerLoad == 0, "lanes of a load: worker by word");
#pragma unroll
  for (int r = 0; r < KQ; ++r)
#pragma unroll
    for (int s = 0; s < 4; ++s) sum[r][s] = 0.0f;
  const uint32_t qw = (q0 >> 5) + (lane % kShareWords), sub = lane / kShareWords;
  const uint32_t sh = (lane & 7u) * 4u, src = lane >> 3;
  for (uint32_t i0 = 0; i0 < geo.n; i0 += kTrip) {
    uint32_t w[kTrip / kPerLoad];
#pragma unroll
    for (int u = 0; u < kTrip / kPerLoad; ++u) {
      const uint32_t i = i0 + kPerLoad * u + sub;
      w[u] = i < geo.n ? ws.bits[static_cast<size_t>(i) * geo.words + qw] : 0u;
    }
    float mu[kTrip];
#pragma unroll
    for (int u = 0; u < kTrip; ++u)
      mu[u] = i0 + u < geo.n ? table_f32(ws.scales + static_cast<size_t>(i0 + u) * geo.num_blocks, b) : 0.0f;
#pragma unroll
    for (int u = 0; u < kTrip; ++u) {
      if (i0 + u < geo.n) {  // wave-uniform
        if ((u & 1) == 0) __builtin_amdgcn_sched_barrier(0);  // (else the words of all workers are taken at once: 82 registers)
#pragma unroll
        for (int r = 0; r < KQ; ++r) {
          const uint32_t word =
              __shfl(w[u / kPerLoad], static_cast<int>((u % kPerLoad) * kShareWords + r * 8 + src), 64);
          const uint32_t nib = (word >> sh) & 15u;
#pragma unroll
          for (int s = 0; s < 4; ++s) sum[r][s] = sum[r][s] + (((nib >> s) & 1u) ? -mu[u] : mu[u]);
        }
      }
    }
  }
}

template <int NC>  // how many of theta, m, v, vhat are cached, the others streamed (see the top-k final kernel)
__global__ __launch_bounds__(bs_server_split(NC) * 64) __attribute__((amdgpu_waves_per_eu(7, 8))) void k_bs_amsgrad(
    float* __restrict__ theta, float* __restrict__ m, float* __restrict__ v, float* __restrict__ vhat, Geometry geo,
    BlocksignWorkspace ws, AmsParams p) {
  const uint32_t* __restrict__ off = ws.offsets;
  const uint32_t wave = uniform_u32(threadIdx.x >> 6), lane = lane_id();
  const uint32_t d = geo.d;
  // (chunk, block and block end are scalars and come through scalar loads: a look-up through the vector path
  // would wait for the state loads issued just before it, a second round trip per round)
  const uint32_t c = blockIdx.x, part = wave;
  if (c >= geo.num_chunks) return;
  uint32_t b = table_u32(ws.chunk_block, c);
  constexpr int kQ = kRounds / bs_server_split(NC);  // rounds of a wavefront's share of the chunk
  const uint32_t q0 = c * kChunk + part * (kQ * 256);
  if (q0 >= d) return;
  while (table_u32(off, b + 1) <= q0) ++b;  // block of the share's first coordinate
  if (q0 + kQ * 256 <= d && table_u32(off, b + 1) >= q0 + kQ * 256) {
    // the whole share lies inside one block (all but a few per row in layouts worth the name)
    const uint32_t j = q0 + lane * 4;
    float sum[kQ][4];
    if constexpr (kQ == 2) {  // the state of both rounds and the sign words are requested together
      float4 th[kQ], mm[kQ], vv[kQ], vh[kQ];
#pragma unroll
      for (int r = 0; r < kQ; ++r) {
        th[r] = load_state4<(NC > 0)>(theta + j + r * 256); mm[r] = load_state4<(NC > 1)>(m + j + r * 256);
        vv[r] = load_state4<(NC > 2)>(v + j + r * 256); vh[r] = load_state4<(NC > 3)>(vhat + j + r * 256);
      }
      bs_share_sums<kQ>(sum, geo, ws, b, q0, lane);
#pragma unroll
      for (int r = 0; r < kQ; ++r) {
        const uint32_t jr = j + r * 256;
        ams_update(sum[r][0] / p.nf, th[r].x, mm[r].x, vv[r].x, vh[r].x, p);
        ams_update(sum[r][1] / p.nf, th[r].y, mm[r].y, vv[r].y, vh[r].y, p);
        ams_update(sum[r][2] / p.nf, th[r].z, mm[r].z, vv[r].z, vh[r].z, p);
        ams_update(sum[r][3] / p.nf, th[r].w, mm[r].w, vv[r].w, vh[r].w, p);
        store_state4<(NC > 0)>(theta + jr, th[r]);
        store_state4<(NC > 1)>(m + jr, mm[r]);
        store_state4<(NC > 2)>(v + jr, vv[r]);
        store_state4<(NC > 3)>(vhat + jr, vh[r]);
      }
    } else {  // the first round's state with the sign words, each next round's while one is updated
      float4 th = load_state4<(NC > 0)>(theta + j), mm = load_state4<(NC > 1)>(m + j);
      float4 vv = load_state4<(NC > 2)>(v + j), vh = load_state4<(NC > 3)>(vhat + j);
      bs_share_sums<kQ>(sum, geo, ws, b, q0, lane);
#pragma unroll
      for (int r = 0; r < kQ; ++r) {
        __builtin_amdgcn_sched_barrier(0);  // (else all rounds' loads are moved up front: 82 registers)
        const uint32_t jr = j + r * 256;
        float4 th2 = th, mm2 = mm, vv2 = vv, vh2 = vh;
        if (r + 1 < kQ) {
          th2 = load_state4<(NC > 0)>(theta + jr + 256); mm2 = load_state4<(NC > 1)>(m + jr + 256);
          vv2 = load_state4<(NC > 2)>(v + jr + 256); vh2 = load_state4<(NC > 3)>(vhat + jr + 256);
        }
        ams_update(sum[r][0] / p.nf, th.x, mm.x, vv.x, vh.x, p);
        ams_update(sum[r][1] / p.nf, th.y, mm.y, vv.y, vh.y, p);
        ams_update(sum[r][2] / p.nf, th.z, mm.z, vv.z, vh.z, p);
        ams_update(sum[r][3] / p.nf, th.w, mm.w, vv.w, vh.w, p);
        store_state4<(NC > 0)>(theta + jr, th);
        store_state4<(NC > 1)>(m + jr, mm);
        store_state4<(NC > 2)>(v + jr, vv);
        store_state4<(NC > 3)>(vhat + jr, vh);
        th = th2; mm = mm2; vv = vv2; vh = vh2;
      }
    }
    return;
  }
  // a share that meets block ends or the row's end: round by round, the sign words and scales of a round
  // requested after its state
  for (int r = part * kQ; r < static_cast<int>(part + 1) * kQ; ++r) {
    const uint32_t j0 = c * kChunk + r * 256;
    if (j0 >= d) break;
    const uint32_t j = j0 + lane * 4;
    const bool ok[4] = {j < d, j + 1 < d, j + 2 < d, j + 3 < d};
    // the optimizer state of this round is requested first; the sign/scale loop runs while it travels
    float4 th = make_float4(0.f, 0.f, 0.f, 0.f), mm = th, vv = th, vh = th;
    if (ok[3]) {
      th = load_state4<(NC > 0)>(theta + j); mm = load_state4<(NC > 1)>(m + j);
      vv = load_state4<(NC > 2)>(v + j); vh = load_state4<(NC > 3)>(vhat + j);
    }
    while (table_u32(off, b + 1) <= j0) ++b;
    const uint32_t j_end = (j0 + 256 < d) ? j0 + 256 : d;
    const bool uniform = table_u32(off, b + 1) >= j_end;
    uint32_t bb[4] = {b, b, b, b};
    if (!uniform) {
#pragma unroll
      for (int s = 0; s < 4; ++s) bb[s] = ok[s] ? block_of(off, b, j + s) : b;
    }
    float sum[4] = {0.f, 0.f, 0.f, 0.f};
    const uint32_t widx = j >> 5, sh = j & 31u;
    if (uniform) {
      for (uint32_t i0 = 0; i0 < geo.n; i0 += kBsWorkers) {
        uint32_t word[kBsWorkers];
        float mu[kBsWorkers];
#pragma unroll
        for (int u = 0; u < kBsWorkers; ++u) {
          const uint32_t i = i0 + u;
          word[u] = 0;
          mu[u] = 0.0f;
          if (i < geo.n) {
            if (ok[0]) word[u] = ws.bits[static_cast<size_t>(i) * geo.words + widx];
            mu[u] = table_f32(ws.scales + static_cast<size_t>(i) * geo.num_blocks, b);
          }
        }
#pragma unroll
        for (int u = 0; u < kBsWorkers; ++u) {
          if (i0 + u < geo.n) {  // wave-uniform
            const uint32_t nib = (word[u] >> sh) & 15u;
#pragma unroll
            for (int s = 0; s < 4; ++s) sum[s] = sum[s] + (((nib >> s) & 1u) ? -mu[u] : mu[u]);
          }
        }
      }
    } else {
      for (uint32_t i = 0; i < geo.n; ++i) {
        const uint32_t word = ok[0] ? ws.bits[static_cast<size_t>(i) * geo.words + widx] : 0u;
        const float* mur = ws.scales + static_cast<size_t>(i) * geo.num_blocks;
        const uint32_t nib = (word >> sh) & 15u;
#pragma unroll
        for (int s = 0; s < 4; ++s) {
          const float mu = mur[bb[s]];
          sum[s] = sum[s] + (((nib >> s) & 1u) ? -mu : mu);
        }
      }
    }
    if (ok[3]) {
      ams_update(sum[0] / p.nf, th.x, mm.x, vv.x, vh.x, p);
      ams_update(sum[1] / p.nf, th.y, mm.y, vv.y, vh.y, p);
      ams_update(sum[2] / p.nf, th.z, mm.z, vv.z, vh.z, p);
      ams_update(sum[3] / p.nf, th.w, mm.w, vv.w, vh.w, p);
      store_state4<(NC > 0)>(theta + j, th);
      store_state4<(NC > 1)>(m + j, mm);
      store_state4<(NC > 2)>(v + j, vv);
      store_state4<(NC > 3)>(vhat + j, vh);
    } else {
      for (int s = 0; s < 4; ++s)
        if (ok[s]) {
          float t1 = theta[j + s], m1 = m[j + s], v1 = v[j + s], h1 = vhat[j + s];
          ams_update(sum[s] / p.nf, t1, m1, v1, h1, p);
          theta[j + s] = t1; m[j + s] = m1; v[j + s] = v1; vhat[j + s] = h1;
        }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// C = identity (full-precision distributed AMSGrad): gbar = mean of the n gradients in worker order.
// ---------------------------------------------------------------------------------------------
template <int NC>  // how many of theta, m, v, vhat are cached (the others are streamed)
__global__ __launch_bounds__(kWG) void k_none_amsgrad(const float* __restrict__ g, float* __restrict__ theta,
                                                       float* __restrict__ m, float* __restrict__ v,
                                                       float* __restrict__ vhat, Geometry geo, AmsParams p) {
  const uint32_t j = (blockIdx.x * kWG + threadIdx.x) * 4;
  if (j >= geo.d) return;
  const bool whole = j + 3 < geo.d;
  // the optimizer state is requested first; the workers' gradients follow eight rows at a time, loads together
  float4 th = make_float4(0.f, 0.f, 0.f, 0.f), mm = th, vv = th, vh = th;
  if (whole) {
    th = load_state4<(NC > 0)>(theta + j); mm = load_state4<(NC > 1)>(m + j);
    vv = load_state4<(NC > 2)>(v + j); vh = load_state4<(NC > 3)>(vhat + j);
  }
  float sum[4] = {0.f, 0.f, 0.f, 0.f};
  constexpr int kRows = 8;
  for (uint32_t i0 = 0; i0 < geo.n; i0 += kRows) {
    float4 gv[kRows];
#pragma unroll
    for (int u = 0; u < kRows; ++u) {
      gv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
      if (i0 + u < geo.n) gv[u] = load_stream4(g + static_cast<int64_t>(i0 + u) * geo.ld + j);  // uniform condition
    }
#pragma unroll
    for (int u = 0; u < kRows; ++u)
      if (i0 + u < geo.n) {
        // x = e + g with e identically zero
        sum[0] = sum[0] + (0.0f + gv[u].x); sum[1] = sum[1] + (0.0f + gv[u].y);
        sum[2] = sum[2] + (0.0f + gv[u].z); sum[3] = sum[3] + (0.0f + gv[u].w);
      }
  }
  if (whole) {
    ams_update(sum[0] / p.nf, th.x, mm.x, vv.x, vh.x, p);
    ams_update(sum[1] / p.nf, th.y, mm.y, vv.y, vh.y, p);
    ams_update(sum[2] / p.nf, th.z, mm.z, vv.z, vh.z, p);
    ams_update(sum[3] / p.nf, th.w, mm.w, vv.w, vh.w, p);
    store_state4<(NC > 0)>(theta + j, th);
    store_state4<(NC > 1)>(m + j, mm);
    store_state4<(NC > 2)>(v + j, vv);
    store_state4<(NC > 3)>(vhat + j, vh);
  } else {
    for (uint32_t s = 0; s < 4 && j + s < geo.d; ++s) {
      float th = theta[j + s], mm = m[j + s], vv = v[j + s], vh = vhat[j + s];
      ams_update(sum[s] / p.nf, th, mm, vv, vh, p);
      theta[j + s] = th; m[j + s] = mm; v[j + s] = vv; vhat[j + s] = vh;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Utility kernels.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kWG) void k_fill_u32(uint32_t* p, size_t count, uint32_t value) {
  const size_t step = static_cast<size_t>(gridDim.x) * kWG;
  for (size_t i = static_cast<size_t>(blockIdx.x) * kWG + threadIdx.x; i < count; i += step) p[i] = value;
}

__global__ __launch_bounds__(kWG) void k_copy_u32(uint32_t* __restrict__ dst, const uint32_t* __restrict__ src, size_t count) {
  const size_t step = static_cast<size_t>(gridDim.x) * kWG;
  for (size_t i = static_cast<size_t>(blockIdx.x) * kWG + threadIdx.x; i < count; i += step) dst[i] = src[i];
}

__global__ __launch_bounds__(kWG) void k_fill_rows(float* p, int64_t ld, uint32_t d, float value) {
  float* r = p + static_cast<int64_t>(blockIdx.y) * ld;
  const uint32_t step = gridDim.x * kWG;
  for (uint32_t j = blockIdx.x * kWG + threadIdx.x; j < d; j += step) r[j] = value;
}

// Streaming (non-temporal) accesses and short workgroups (4 KiB each, handed out in order), as in the step's dense
// kernels: the shape that streams fastest on this part.
__global__ __launch_bounds__(kWG) void k_copy16(float* __restrict__ dst, const float* __restrict__ src, size_t count) {
  const size_t step = static_cast<size_t>(gridDim.x) * kWG;
  for (size_t i = static_cast<size_t>(blockIdx.x) * kWG + threadIdx.x; i < count; i += step)
    store_stream4(dst + 4 * i, load_stream4(src + 4 * i));
}

// The access pattern of the server's lines of Algorithm 2 with nothing else around it: A separately allocated
// arrays (the pointers beyond the A-th are not looked at), a workgroup per 4096 elements that takes that stretch of
// every array, 16 bytes per lane and access, every element read, increased by one and written back.  All of a
// lane's loads are requested before the first is used (nothing else needs the registers here: the most this
// pattern can have in flight).  NC as in the kernels that apply those lines.
template <int A, int NC>
__global__ __launch_bounds__(kWG) void k_inplace_probe(float* a0, float* a1, float* a2, float* a3, size_t count) {
  constexpr int kR = kChunk / (kWG * 4);
  float4 x[kR][4];
  const size_t j0 = static_cast<size_t>(blockIdx.x) * kChunk + threadIdx.x * 4;
#pragma unroll
  for (int r = 0; r < kR; ++r) {
    const size_t j = j0 + r * kWG * 4;
    if (j + 3 < count) {
      x[r][0] = load_state4<(NC > 0)>(a0 + j);
      if (A > 1) x[r][1] = load_state4<(NC > 1)>(a1 + j);
      if (A > 2) x[r][2] = load_state4<(NC > 2)>(a2 + j);
      if (A > 3) x[r][3] = load_state4<(NC > 3)>(a3 + j);
    }
  }
#pragma unroll
  for (int r = 0; r < kR; ++r) {
    const size_t j = j0 + r * kWG * 4;
    if (j + 3 < count) {
#pragma unroll
      for (int a = 0; a < A; ++a) {
        x[r][a].x += 1.0f; x[r][a].y += 1.0f; x[r][a].z += 1.0f; x[r][a].w += 1.0f;
      }
      store_state4<(NC > 0)>(a0 + j, x[r][0]);
      if (A > 1) store_state4<(NC > 1)>(a1 + j, x[r][1]);
      if (A > 2) store_state4<(NC > 2)>(a2 + j, x[r][2]);
      if (A > 3) store_state4<(NC > 3)>(a3 + j, x[r][3]);
    }
  }
}

}  // namespace

#define COMPAMS_CHECK_LAUNCH()                    \
  do {                                            \
    hipError_t err__ = hipGetLastError();         \
    if (err__ != hipSuccess) return err__;        \
  } while (0)

hipError_t blocksign_step(const Geometry& geo, const BlocksignWorkspace& ws, const AmsParams& ap, const float* g,
                          float* e, float* theta, float* m, float* v, float* vhat, bool residual_pending,
                          bool workers_only, hipStream_t stream, Launcher* L) {
  const dim3 grid_chunks(geo.num_chunks, geo.n), wg(kWG);
  if (residual_pending) launch(L, kSlotBsPass1, k_bs_lean<true>, grid_chunks, wg, stream, g, e, geo, ws);
  else launch(L, kSlotBsPass1, k_bs_lean<false>, grid_chunks, wg, stream, g, e, geo, ws);
  COMPAMS_CHECK_LAUNCH();
  const size_t total = static_cast<size_t>(geo.n) * geo.num_blocks;
  const size_t per_group = ws.acc_replicas == 1 ? kWG : kWaves;  // (row, block) pairs per workgroup
  launch(L, kSlotBsFinal, k_bs_finalize, dim3(static_cast<uint32_t>((total + per_group - 1) / per_group)), wg, stream,
         geo, ws);
  COMPAMS_CHECK_LAUNCH();
  // The residual e = x - sign(x) * mu is left to the next step's first pass (or to blocksign_apply_residual when
  // e is asked for).
  if (workers_only) return hipSuccess;
  return blocksign_server_step(geo, ws, ap, theta, m, v, vhat, stream, L);
}

// The server's lines from the sign words and scales that sit in the workspace.
hipError_t blocksign_server_step(const Geometry& geo, const BlocksignWorkspace& ws, const AmsParams& ap, float* theta,
                                 float* m, float* v, float* vhat, hipStream_t stream, Launcher* L) {
  const dim3 grid(geo.num_chunks), wg(bs_server_split(ap.cached_arrays) * 64);  // a workgroup per chunk
#define COMPAMS_BS_AMSGRAD(NC) k_bs_amsgrad<NC>
  COMPAMS_LAUNCH_BY_CACHED(ap.cached_arrays, L, kSlotBsAms, COMPAMS_BS_AMSGRAD, grid, wg, stream, theta, m, v, vhat, geo, ws,
                           ap);
#undef COMPAMS_BS_AMSGRAD
  COMPAMS_CHECK_LAUNCH();
  return hipSuccess;
}

hipError_t blocksign_apply_residual(const Geometry& geo, const BlocksignWorkspace& ws, float* e, hipStream_t stream) {
  const uint32_t G = groups_per_row(geo.n, geo.num_chunks);
  hipLaunchKernelGGL(k_bs_pass2, dim3(G * 2, geo.n), dim3(kWG), 0, stream, e, geo, ws);
  return hipGetLastError();
}

hipError_t none_step(const Geometry& geo, const AmsParams& ap, const float* g, float* theta, float* m, float* v,
                     float* vhat, hipStream_t stream, Launcher* L) {
  const uint32_t quads = (geo.d + 3) / 4;
  const dim3 grid((quads + kWG - 1) / kWG), wg(kWG);
#define COMPAMS_NONE_AMSGRAD(NC) k_none_amsgrad<NC>
  COMPAMS_LAUNCH_BY_CACHED(ap.cached_arrays, L, kSlotNoneAms, COMPAMS_NONE_AMSGRAD, grid, wg, stream, g, theta, m, v, vhat,
                           geo, ap);
#undef COMPAMS_NONE_AMSGRAD
  return hipGetLastError();
}

hipError_t fill_u32(uint32_t* p, size_t count, uint32_t value, hipStream_t stream) {
  if (!count) return hipSuccess;
  size_t blocks = (count + kWG - 1) / kWG;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_fill_u32, dim3(static_cast<uint32_t>(blocks)), dim3(kWG), 0, stream, p, count, value);
  return hipGetLastError();
}

hipError_t copy_u32(uint32_t* dst, const uint32_t* src, size_t count, hipStream_t stream) {
  if (!count) return hipSuccess;
  size_t blocks = (count + kWG - 1) / kWG;
  if (blocks > 4096) blocks = 4096;
  hipLaunchKernelGGL(k_copy_u32, dim3(static_cast<uint32_t>(blocks)), dim3(kWG), 0, stream, dst, src, count);
  return hipGetLastError();
}

hipError_t fill_rows_f32(float* p, uint32_t n, int64_t ld, uint32_t d, float value, hipStream_t stream) {
  uint32_t blocks = (d + kWG - 1) / kWG;
  if (blocks > 2048) blocks = 2048;
  hipLaunchKernelGGL(k_fill_rows, dim3(blocks, n), dim3(kWG), 0, stream, p, ld, d, value);
  return hipGetLastError();
}

hipError_t stream_copy(void* dst, const void* src, size_t bytes, hipStream_t stream) {
  const size_t count = bytes / 16;
  if (!count) return hipSuccess;
  size_t blocks = (count + kWG - 1) / kWG;  // one quad per thread up to 32 GiB, a stride loop beyond
  if (blocks > 0x7fffffffu) blocks = 0x7fffffffu;
  hipLaunchKernelGGL(k_copy16, dim3(static_cast<uint32_t>(blocks)), dim3(kWG), 0, stream,
                     static_cast<float*>(dst), static_cast<const float*>(src), count);
  return hipGetLastError();
}

template <int A>
static void launch_inplace_probe(int cached, dim3 grid, hipStream_t stream, float* const* a, size_t count) {
  float* const last = a[A - 1];
  float* const a1 = A > 1 ? a[1] : last;
  float* const a2 = A > 2 ? a[2] : last;
  float* const a3 = A > 3 ? a[3] : last;
  switch (cached) {
    case 0: hipLaunchKernelGGL((k_inplace_probe<A, 0>), grid, dim3(kWG), 0, stream, a[0], a1, a2, a3, count); break;
    case 1: hipLaunchKernelGGL((k_inplace_probe<A, 1>), grid, dim3(kWG), 0, stream, a[0], a1, a2, a3, count); break;
    case 2: hipLaunchKernelGGL((k_inplace_probe<A, 2>), grid, dim3(kWG), 0, stream, a[0], a1, a2, a3, count); break;
    case 3: hipLaunchKernelGGL((k_inplace_probe<A, 3>), grid, dim3(kWG), 0, stream, a[0], a1, a2, a3, count); break;
    default: hipLaunchKernelGGL((k_inplace_probe<A, 4>), grid, dim3(kWG), 0, stream, a[0], a1, a2, a3, count); break;
  }
}

hipError_t inplace_probe(float* const* arrays, int n_arrays, size_t count, int cached_arrays, hipStream_t stream) {
  if (!count) return hipSuccess;
  const dim3 grid(static_cast<uint32_t>((count + kChunk - 1) / kChunk));
  switch (n_arrays) {
    case 1: launch_inplace_probe<1>(cached_arrays, grid, stream, arrays, count); break;
    case 2: launch_inplace_probe<2>(cached_arrays, grid, stream, arrays, count); break;
    case 3: launch_inplace_probe<3>(cached_arrays, grid, stream, arrays, count); break;
    default: launch_inplace_probe<4>(cached_arrays, grid, stream, arrays, count); break;
  }
  return hipGetLastError();
}

}  // namespace compams
