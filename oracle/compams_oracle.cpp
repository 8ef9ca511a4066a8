// compams_oracle.cpp -- TEST INFRASTRUCTURE, not the product.
//
// Plain, slow, single-threaded CPU statement of one COMP-AMS iteration
// (Algorithm 2 of the paper: error-feedback compression on each of n workers,
// worker-ordered average, AMSGrad update at the server), with the two
// compressors of Definition 1 (Top-k) and Definition 2 (Block-Sign).
//
// It exists so that tests, the smoke check and the benchmark's cpu_baseline leg
// have something to compare the GPU library against.  It shares no code, header,
// table or helper with the GPU library and neither includes the other.  Nothing
// here is blocked, fused or reordered: every function walks the definition it
// cites so that it can be checked against the paper by eye.
//
// Readings where the paper is silent (each is pinned by a CPU test):
//   * magnitude order = unsigned order of (bits(x) & 0x7fffffff); ties go to the
//     lower index (Definition 1 does not say which of several equal |x_i| wins).
//   * sign(x) = -1 iff x < 0, else +1 (Definition 2 leaves sign(0) open; a
//     ternary code would not be a 1-bit code).
//   * ||x_B||_1 is the exact real sum of the fp32 values |x_j|, rounded once to
//     double; the block scale is (float)(that / (double)d_B).
//   * the average is a left-to-right fp32 sum over workers 0..n-1 divided by
//     (float)n; all other arithmetic is fp32, one rounding per operation, no
//     fused multiply-add (build with -ffp-contract=off).
//   * epsilon sits inside the square root as in Algorithms 1 and 2; the outside
//     form is available as a switch.
//
//   * the wire format of a message is this library's own (the paper only fixes 32 bits per transmitted
//     float); it is stated at the encode functions below and in the public header.
//
// Parity pins: every exported function is pinned by tests/test_oracle_*.py
// (brute-force sort, math.fsum, closed forms, Lemma 5 telescoping, the identity
// special cases that reduce Algorithm 2 to Algorithm 1, a hand-derived d=8 case).

#include <algorithm>
#include <cmath>
#include <cstdint>
#include <cstring>
#include <limits>
#include <new>
#include <vector>

namespace {

enum { C_NONE = 0, C_TOPK = 1, C_BLOCKSIGN = 2, C_TOPK_BLOCKS = 3 };
enum { EPS_IN_SQRT = 0, EPS_OUT_SQRT = 1 };

inline uint32_t bits_of(float x) {
  uint32_t u;
  std::memcpy(&u, &x, sizeof u);
  return u;
}

// Magnitude key: for finite values and infinities the unsigned order of this key
// is the order of |x|; +0 and -0 share key 0.
inline uint32_t key_of(float x) { return bits_of(x) & 0x7fffffffu; }

// (key descending, index ascending): the total order that makes "the k largest
// magnitudes" of Definition 1 a unique set.
struct BeforeInTopkOrder {
  const float* x;
  bool operator()(int32_t a, int32_t b) const {
    const uint32_t ka = key_of(x[a]), kb = key_of(x[b]);
    if (ka != kb) return ka > kb;
    return a < b;
  }
};

// Definition 1: S = the first k indices in the order above.  out_idx gets S sorted
// ascending.  Uses a selection routine; the brute-force twin below uses a full sort.
void topk_select(const float* x, int64_t d, int64_t k, int32_t* out_idx) {
  std::vector<int32_t> perm(static_cast<size_t>(d));
  for (int64_t j = 0; j < d; ++j) perm[static_cast<size_t>(j)] = static_cast<int32_t>(j);
  BeforeInTopkOrder before{x};
  if (k < d) std::nth_element(perm.begin(), perm.begin() + k, perm.end(), before);
  std::sort(perm.begin(), perm.begin() + k);
  std::copy(perm.begin(), perm.begin() + k, out_idx);
}

void topk_select_fullsort(const float* x, int64_t d, int64_t k, int32_t* out_idx) {
  std::vector<int32_t> perm(static_cast<size_t>(d));
  for (int64_t j = 0; j < d; ++j) perm[static_cast<size_t>(j)] = static_cast<int32_t>(j);
  std::sort(perm.begin(), perm.end(), BeforeInTopkOrder{x});
  std::sort(perm.begin(), perm.begin() + k);
  std::copy(perm.begin(), perm.begin() + k, out_idx);
}

// Exact accumulator for sums of fp32 magnitudes: a 384-bit unsigned fixed-point
// integer whose unit is 2^-149 (the smallest fp32 subnormal).  One fp32 value is a
// 24-bit integer shifted by at most 253 bits; 2^31 of them stay below 2^309.
struct ExactSum {
  static const int LIMBS = 6;
  uint64_t limb[LIMBS];
  bool saw_nan, saw_inf;
  ExactSum() : saw_nan(false), saw_inf(false) {
    for (int i = 0; i < LIMBS; ++i) limb[i] = 0;
  }
  void add_abs(float x) {
    const uint32_t k = key_of(x);
    const uint32_t expo = k >> 23;
    const uint32_t frac = k & 0x7fffffu;
    if (expo == 255) {
      if (frac) saw_nan = true; else saw_inf = true;
      return;
    }
    // |x| = mant * 2^(shift-149) with an integer mant < 2^24
    const uint64_t mant = expo ? (frac | 0x800000u) : frac;
    const int shift = expo ? static_cast<int>(expo) - 1 : 0;
    const int w = shift / 64, o = shift % 64;
    uint64_t lo = mant << o;
    uint64_t hi = o ? (mant >> (64 - o)) : 0;
    int i = w;
    uint64_t carry = 0;
    uint64_t t = limb[i] + lo;
    carry = t < lo;
    limb[i] = t;
    ++i;
    uint64_t add = hi + carry;  // hi < 2^24, cannot wrap
    while (add && i < LIMBS) {
      t = limb[i] + add;
      add = t < add;
      limb[i] = t;
      ++i;
    }
  }
  // The sum rounded once (to nearest, ties to even) to double.
  double to_double() const {
    if (saw_nan) return std::numeric_limits<double>::quiet_NaN();
    if (saw_inf) return std::numeric_limits<double>::infinity();
    int top = -1;  // position of the highest set bit
    for (int i = LIMBS - 1; i >= 0 && top < 0; --i)
      if (limb[i]) {
        int b = 63;
        while (!((limb[i] >> b) & 1)) --b;
        top = i * 64 + b;
      }
    if (top < 0) return 0.0;
    if (top <= 52) return std::ldexp(static_cast<double>(limb[0]), -149);  // fits exactly
    const int low = top - 52;  // lowest kept bit
    uint64_t kept = 0;
    for (int p = top; p >= low; --p) kept = (kept << 1) | bit(p);
    const int guard = bit(low - 1);
    bool sticky = false;
    for (int p = low - 2; p >= 0 && !sticky; --p) sticky = bit(p);
    if (guard && (sticky || (kept & 1))) ++kept;  // may become 2^53: still exact in double
    return std::ldexp(static_cast<double>(kept), low - 149);
  }
  int bit(int p) const { return static_cast<int>((limb[p / 64] >> (p % 64)) & 1); }
};

// Definition 2, one block: ||x_B||_1 / d_B.
float block_l1_mean(const float* x, int64_t len) {
  ExactSum s;
  for (int64_t j = 0; j < len; ++j) s.add_abs(x[j]);
  return static_cast<float>(s.to_double() / static_cast<double>(len));
}

struct Oracle {
  int n;
  int64_t d;
  int compressor;
  int64_t k;
  int64_t M;
  std::vector<int64_t> off;  // M+1 block offsets
  std::vector<int64_t> kb;   // top-k per block: how many coordinates each block keeps
  float beta1, beta2, eps;
  int eps_mode;
  int64_t t;  // iterations done
  std::vector<float> theta, m, v, vhat;  // d
  std::vector<float> e;                  // n*d, worker-major
  // what the workers "sent" in the last iteration
  std::vector<float> ctil;         // n*d dense form of C(g+e)
  std::vector<int32_t> last_idx;   // n*k ascending per worker (top-k)
  std::vector<float> last_val;     // n*k
  std::vector<uint32_t> last_bits; // n*ceil(d/32) (block-sign), bit j&31 of word j>>5 = (x_j < 0)
  std::vector<float> last_mu;      // n*M
  std::vector<float> gbar;         // d
  std::vector<float> x;            // d scratch: corrected gradient of the current worker
};

void worker_topk(Oracle& o, int i) {
  const int64_t d = o.d, k = o.k;
  float* e = &o.e[static_cast<size_t>(i) * d];
  float* c = &o.ctil[static_cast<size_t>(i) * d];
  int32_t* idx = &o.last_idx[static_cast<size_t>(i) * k];
  float* val = &o.last_val[static_cast<size_t>(i) * k];
  topk_select(o.x.data(), d, k, idx);
  // C(x)_j = x_j on S, 0 elsewhere; e_{t+1} = x - C(x)  (Alg. 2, the two worker lines)
  for (int64_t j = 0; j < d; ++j) { c[j] = 0.0f; e[j] = o.x[j]; }
  for (int64_t q = 0; q < k; ++q) {
    const int32_t j = idx[q];
    val[q] = o.x[j];
    c[j] = o.x[j];
    e[j] = 0.0f;
  }
}

// Definition 1 applied to every block on its own: block b keeps its kb[b] largest magnitudes.  The worker's list
// holds the kept coordinates of block 0, then of block 1, ...: ascending over the whole row.
void worker_topk_blocks(Oracle& o, int i) {
  const int64_t d = o.d, k = o.k;
  float* e = &o.e[static_cast<size_t>(i) * d];
  float* c = &o.ctil[static_cast<size_t>(i) * d];
  int32_t* idx = &o.last_idx[static_cast<size_t>(i) * k];
  float* val = &o.last_val[static_cast<size_t>(i) * k];
  for (int64_t j = 0; j < d; ++j) { c[j] = 0.0f; e[j] = o.x[j]; }
  int64_t at = 0;
  for (int64_t b = 0; b < o.M; ++b) {
    const int64_t lo = o.off[b], len = o.off[b + 1] - lo;
    topk_select(o.x.data() + lo, len, o.kb[b], idx + at);
    for (int64_t q = 0; q < o.kb[b]; ++q) {
      const int32_t j = static_cast<int32_t>(lo) + idx[at + q];
      idx[at + q] = j;
      val[at + q] = o.x[j];
      c[j] = o.x[j];
      e[j] = 0.0f;
    }
    at += o.kb[b];
  }
}

void worker_blocksign(Oracle& o, int i) {
  const int64_t d = o.d;
  const int64_t words = (d + 31) / 32;
  float* e = &o.e[static_cast<size_t>(i) * d];
  float* c = &o.ctil[static_cast<size_t>(i) * d];
  uint32_t* bits = &o.last_bits[static_cast<size_t>(i) * words];
  float* mu = &o.last_mu[static_cast<size_t>(i) * o.M];
  for (int64_t w = 0; w < words; ++w) bits[w] = 0;
  for (int64_t b = 0; b < o.M; ++b) {
    const int64_t lo = o.off[b], hi = o.off[b + 1];
    mu[b] = block_l1_mean(o.x.data() + lo, hi - lo);
    for (int64_t j = lo; j < hi; ++j) {
      const bool neg = o.x[j] < 0.0f;
      if (neg) bits[j >> 5] |= (1u << (j & 31));
      c[j] = neg ? -mu[b] : mu[b];
      e[j] = o.x[j] - c[j];
    }
  }
}

void worker_identity(Oracle& o, int i) {
  const int64_t d = o.d;
  float* e = &o.e[static_cast<size_t>(i) * d];
  float* c = &o.ctil[static_cast<size_t>(i) * d];
  for (int64_t j = 0; j < d; ++j) { c[j] = o.x[j]; e[j] = o.x[j] - c[j]; }
}

void step(Oracle& o, const float* g, float lr) {
  const int64_t d = o.d;
  for (int i = 0; i < o.n; ++i) {
    const float* gi = g + static_cast<size_t>(i) * d;
    const float* ei = &o.e[static_cast<size_t>(i) * d];
    for (int64_t j = 0; j < d; ++j) o.x[j] = ei[j] + gi[j];  // corrected gradient
    if (o.compressor == C_TOPK) worker_topk(o, i);
    else if (o.compressor == C_TOPK_BLOCKS) worker_topk_blocks(o, i);
    else if (o.compressor == C_BLOCKSIGN) worker_blocksign(o, i);
    else worker_identity(o, i);
  }
  const float one_minus_b1 = 1.0f - o.beta1;
  const float one_minus_b2 = 1.0f - o.beta2;
  const float nf = static_cast<float>(o.n);
  for (int64_t j = 0; j < d; ++j) {
    float s = 0.0f;
    for (int i = 0; i < o.n; ++i) s = s + o.ctil[static_cast<size_t>(i) * d + j];
    const float gb = s / nf;
    o.gbar[j] = gb;
    const float mj = o.beta1 * o.m[j] + one_minus_b1 * gb;
    const float vj = o.beta2 * o.v[j] + one_minus_b2 * (gb * gb);
    const float vh = std::max(o.vhat[j], vj);
    const float den = (o.eps_mode == EPS_IN_SQRT) ? std::sqrt(vh + o.eps) : std::sqrt(vh) + o.eps;
    o.m[j] = mj;
    o.v[j] = vj;
    o.vhat[j] = vh;
    o.theta[j] = o.theta[j] - lr * (mj / den);
  }
  ++o.t;
}

}  // namespace

extern "C" {

void* oracle_compams_create(int n, int64_t d, int compressor, int64_t k, int64_t num_blocks,
                            const int64_t* block_offsets, float beta1, float beta2, float eps,
                            int eps_mode, const float* theta0) {
  if (n < 1 || d < 1 || d >= (int64_t(1) << 31)) return nullptr;
  if (compressor == C_TOPK && (k < 1 || k > d)) return nullptr;
  if (compressor == C_BLOCKSIGN) {
    if (num_blocks < 1 || !block_offsets || block_offsets[0] != 0 || block_offsets[num_blocks] != d)
      return nullptr;
    for (int64_t b = 0; b < num_blocks; ++b)
      if (block_offsets[b + 1] <= block_offsets[b]) return nullptr;
  }
  Oracle* o = new (std::nothrow) Oracle();
  if (!o) return nullptr;
  o->n = n; o->d = d; o->compressor = compressor;
  o->k = (compressor == C_TOPK) ? k : 0;
  o->M = (compressor == C_BLOCKSIGN) ? num_blocks : 0;
  if (o->M) o->off.assign(block_offsets, block_offsets + num_blocks + 1);
  o->beta1 = beta1; o->beta2 = beta2; o->eps = eps; o->eps_mode = eps_mode; o->t = 0;
  const size_t sd = static_cast<size_t>(d), sn = static_cast<size_t>(n);
  o->theta.assign(theta0, theta0 + d);
  o->m.assign(sd, 0.0f); o->v.assign(sd, 0.0f); o->vhat.assign(sd, 0.0f);
  o->e.assign(sn * sd, 0.0f);
  o->ctil.assign(sn * sd, 0.0f);
  o->gbar.assign(sd, 0.0f);
  o->x.assign(sd, 0.0f);
  o->last_idx.assign(sn * static_cast<size_t>(o->k), 0);
  o->last_val.assign(sn * static_cast<size_t>(o->k), 0.0f);
  if (o->M) {
    o->last_bits.assign(sn * static_cast<size_t>((d + 31) / 32), 0u);
    o->last_mu.assign(sn * static_cast<size_t>(o->M), 0.0f);
  }
  return o;
}

// Top-k per block: block b = [block_offsets[b], block_offsets[b+1]) keeps block_k[b] coordinates (1 .. its size).
void* oracle_compams_create_topk_blocks(int n, int64_t d, int64_t num_blocks, const int64_t* block_offsets,
                                        const int64_t* block_k, float beta1, float beta2, float eps, int eps_mode,
                                        const float* theta0) {
  if (num_blocks < 1 || !block_offsets || !block_k) return nullptr;
  int64_t total = 0;
  for (int64_t b = 0; b < num_blocks; ++b) {
    const int64_t len = block_offsets[b + 1] - block_offsets[b];
    if (len < 1 || block_k[b] < 1 || block_k[b] > len) return nullptr;
    total += block_k[b];
  }
  // created as a block layout (validates the offsets), then turned into the per-block top-k
  Oracle* o = static_cast<Oracle*>(oracle_compams_create(n, d, C_BLOCKSIGN, 0, num_blocks, block_offsets, beta1, beta2,
                                                          eps, eps_mode, theta0));
  if (!o) return nullptr;
  o->compressor = C_TOPK_BLOCKS;
  o->k = total;
  o->kb.assign(block_k, block_k + num_blocks);
  o->last_idx.assign(static_cast<size_t>(n) * static_cast<size_t>(total), 0);
  o->last_val.assign(static_cast<size_t>(n) * static_cast<size_t>(total), 0.0f);
  o->last_bits.clear();
  o->last_mu.clear();
  return o;
}

void oracle_compams_destroy(void* h) { delete static_cast<Oracle*>(h); }

// g: host, n*d floats, worker-major, dense (row stride d).
void oracle_compams_step(void* h, const float* g, float lr) { step(*static_cast<Oracle*>(h), g, lr); }

// Overwrite the whole state (resume / tests).  Any pointer may be null = keep.
void oracle_compams_set_state(void* h, const float* theta, const float* m, const float* v,
                              const float* vhat, const float* e) {
  Oracle& o = *static_cast<Oracle*>(h);
  if (theta) o.theta.assign(theta, theta + o.d);
  if (m) o.m.assign(m, m + o.d);
  if (v) o.v.assign(v, v + o.d);
  if (vhat) o.vhat.assign(vhat, vhat + o.d);
  if (e) o.e.assign(e, e + static_cast<size_t>(o.n) * o.d);
}

enum { Q_THETA = 0, Q_M, Q_V, Q_VHAT, Q_E, Q_IDX, Q_VAL, Q_BITS, Q_MU, Q_GBAR, Q_CTIL };

// Borrowed host pointer to a state or last-message array; count in elements.
const void* oracle_compams_get(void* h, int which, int64_t* count) {
  Oracle& o = *static_cast<Oracle*>(h);
  const void* p = nullptr; size_t c = 0;
  switch (which) {
    case Q_THETA: p = o.theta.data(); c = o.theta.size(); break;
    case Q_M: p = o.m.data(); c = o.m.size(); break;
    case Q_V: p = o.v.data(); c = o.v.size(); break;
    case Q_VHAT: p = o.vhat.data(); c = o.vhat.size(); break;
    case Q_E: p = o.e.data(); c = o.e.size(); break;
    case Q_IDX: p = o.last_idx.data(); c = o.last_idx.size(); break;
    case Q_VAL: p = o.last_val.data(); c = o.last_val.size(); break;
    case Q_BITS: p = o.last_bits.data(); c = o.last_bits.size(); break;
    case Q_MU: p = o.last_mu.data(); c = o.last_mu.size(); break;
    case Q_GBAR: p = o.gbar.data(); c = o.gbar.size(); break;
    case Q_CTIL: p = o.ctil.data(); c = o.ctil.size(); break;
    default: break;
  }
  if (count) *count = static_cast<int64_t>(c);
  return p;
}

// Stand-alone pieces, exported so that tests can pin each one separately.
void oracle_topk_select(const float* x, int64_t d, int64_t k, int32_t* out_idx) { topk_select(x, d, k, out_idx); }
void oracle_topk_select_fullsort(const float* x, int64_t d, int64_t k, int32_t* out_idx) { topk_select_fullsort(x, d, k, out_idx); }
float oracle_block_l1_mean(const float* x, int64_t len) { return block_l1_mean(x, len); }
double oracle_exact_abs_sum(const float* x, int64_t len) {
  ExactSum s;
  for (int64_t j = 0; j < len; ++j) s.add_abs(x[j]);
  return s.to_double();
}

// ---------------------------------------------------------------------------------------------
// Wire format of one worker's message (what the send line among the worker lines of Algorithm 2 puts on the
// wire), as a sequence of 32-bit words.  The paper fixes only the
// accounting (32 bits per transmitted float, experiments section); the layout is this library's own and
// is stated in full in the public header.  Written here bit by bit, straight from that statement.
//
//   top-k      [1, k, 256,  width words,  gap stream,  k value words]
//              gap_0 = idx_0, gap_q = idx_q - idx_{q-1} - 1.  The gaps are taken in tiles of 256 (the last one
//              may be shorter); tile t has its own width b_t = number of bits of its largest gap (at least 1),
//              kept as byte (t mod 4) of width word t div 4 (unused bytes 0).  In the stream the tiles follow
//              one another, each starting on a word boundary: gap i of a tile occupies the tile's bits
//              i*b_t .. i*b_t + b_t - 1, least significant bit first; bit u of a tile is bit (u mod 32) of its
//              word u div 32; unused bits of a tile's last word are 0.
//   block-sign [2, d, M,  ceil(d/32) sign words,  M scale words]
// ---------------------------------------------------------------------------------------------
constexpr int64_t kWireTileGaps = 256;

int64_t oracle_wire_encode_topk(int64_t k, const int32_t* idx, const float* val, uint32_t* out) {
  std::vector<uint32_t> gap(static_cast<size_t>(k));
  for (int64_t q = 0; q < k; ++q)
    gap[q] = q == 0 ? static_cast<uint32_t>(idx[0])
                    : static_cast<uint32_t>(idx[q]) - static_cast<uint32_t>(idx[q - 1]) - 1u;
  const int64_t tiles = (k + kWireTileGaps - 1) / kWireTileGaps;
  const int64_t width_words = (tiles + 3) / 4;
  out[0] = 1u; out[1] = static_cast<uint32_t>(k); out[2] = static_cast<uint32_t>(kWireTileGaps);
  uint32_t* widths = out + 3;
  for (int64_t w = 0; w < width_words; ++w) widths[w] = 0;
  uint32_t* stream = widths + width_words;
  int64_t at = 0;  // words of the stream written so far
  for (int64_t t = 0; t < tiles; ++t) {
    const int64_t first = t * kWireTileGaps;
    const int64_t cnt = std::min<int64_t>(kWireTileGaps, k - first);
    uint32_t widest = 0;
    for (int64_t i = 0; i < cnt; ++i) widest = std::max(widest, gap[first + i]);
    uint32_t b = 1;
    while (b < 32 && (widest >> b) != 0) ++b;
    widths[t / 4] |= b << (8 * (t % 4));
    const int64_t tile_words = (cnt * b + 31) / 32;
    for (int64_t w = 0; w < tile_words; ++w) stream[at + w] = 0;
    for (int64_t i = 0; i < cnt; ++i)
      for (uint32_t u = 0; u < b; ++u)
        if ((gap[first + i] >> u) & 1u) {
          const int64_t pos = i * b + u;
          stream[at + pos / 32] |= 1u << (pos % 32);
        }
    at += tile_words;
  }
  uint32_t* values = stream + at;
  for (int64_t q = 0; q < k; ++q) std::memcpy(&values[q], &val[q], 4);
  return 3 + width_words + at + k;
}

// Returns 0, or a negative number if the words are not a top-k message of k entries below d.
int64_t oracle_wire_decode_topk(const uint32_t* msg, int64_t nwords, int64_t k, int64_t d, int32_t* idx, float* val) {
  if (nwords < 3 || msg[0] != 1u || msg[1] != static_cast<uint32_t>(k) ||
      msg[2] != static_cast<uint32_t>(kWireTileGaps))
    return -1;
  const int64_t tiles = (k + kWireTileGaps - 1) / kWireTileGaps;
  const int64_t width_words = (tiles + 3) / 4;
  if (nwords < 3 + width_words) return -3;
  const uint32_t* widths = msg + 3;
  int64_t stream_words = 0;
  for (int64_t t = 0; t < tiles; ++t) {
    const uint32_t b = (widths[t / 4] >> (8 * (t % 4))) & 0xffu;
    if (b < 1 || b > 31) return -2;
    const int64_t cnt = std::min<int64_t>(kWireTileGaps, k - t * kWireTileGaps);
    stream_words += (cnt * b + 31) / 32;
  }
  if (nwords != 3 + width_words + stream_words + k) return -3;
  const uint32_t* stream = widths + width_words;
  int64_t at = 0, prev = -1;
  for (int64_t t = 0; t < tiles; ++t) {
    const uint32_t b = (widths[t / 4] >> (8 * (t % 4))) & 0xffu;
    const int64_t first = t * kWireTileGaps;
    const int64_t cnt = std::min<int64_t>(kWireTileGaps, k - first);
    for (int64_t i = 0; i < cnt; ++i) {
      uint32_t gap = 0;
      for (uint32_t u = 0; u < b; ++u) {
        const int64_t pos = i * b + u;
        gap |= ((stream[at + pos / 32] >> (pos % 32)) & 1u) << u;
      }
      const int64_t j = prev + 1 + static_cast<int64_t>(gap);
      if (j >= d) return -4;
      idx[first + i] = static_cast<int32_t>(j);
      prev = j;
    }
    at += (cnt * b + 31) / 32;
  }
  const uint32_t* values = stream + at;
  for (int64_t q = 0; q < k; ++q) std::memcpy(&val[q], &values[q], 4);
  return 0;
}

int64_t oracle_wire_encode_blocksign(int64_t d, int64_t M, const uint32_t* bits, const float* mu, uint32_t* out) {
  const int64_t words = (d + 31) / 32;
  out[0] = 2u; out[1] = static_cast<uint32_t>(d); out[2] = static_cast<uint32_t>(M);
  for (int64_t w = 0; w < words; ++w) out[3 + w] = bits[w];
  for (int64_t b = 0; b < M; ++b) std::memcpy(&out[3 + words + b], &mu[b], 4);
  return 3 + words + M;
}

int64_t oracle_wire_decode_blocksign(const uint32_t* msg, int64_t nwords, int64_t d, int64_t M, uint32_t* bits,
                                     float* mu) {
  const int64_t words = (d + 31) / 32;
  if (nwords != 3 + words + M || msg[0] != 2u || msg[1] != static_cast<uint32_t>(d) ||
      msg[2] != static_cast<uint32_t>(M))
    return -1;
  for (int64_t w = 0; w < words; ++w) bits[w] = msg[3 + w];
  for (int64_t b = 0; b < M; ++b) std::memcpy(&mu[b], &msg[3 + words + b], 4);
  return 0;
}

}  // extern "C"
