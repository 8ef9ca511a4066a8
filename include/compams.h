/* compams.h -- C ABI of the COMP-AMS optimizer step for MI355X (gfx950).
 *
 * One call of compams_step() is one iteration of the paper's Algorithm 2
 * (the distributed method with error feedback): every one of n workers adds its
 * error accumulator to its gradient, compresses the sum, keeps what the
 * compressor dropped as the new error, and the server averages the n compressed
 * gradients and applies an AMSGrad update (Algorithm 1's moment and parameter
 * lines).  The n workers are the rows of an n x ld fp32 buffer in one GPU's
 * memory; nothing is sent anywhere.
 *
 * Conventions that hold for every entry point
 *   - Pointers marked DEVICE are HIP device pointers on the device that was
 *     current when compams_init() ran; pointers marked HOST are ordinary host
 *     memory.  The library never allocates or frees device memory: all device
 *     buffers, the workspace included, belong to the caller and are borrowed
 *     until compams_destroy().
 *   - Every function returns COMPAMS_OK (0) or a negative compams_status; it
 *     never throws, aborts or prints.  Out-parameters are untouched on error.
 *   - compams_step() only enqueues work on the given stream; it does not
 *     synchronise with the host and takes no data-dependent decision on the
 *     host.  One context may be driven by one host thread at a time.
 *   - A context is one sequence of steps.  Calls that enqueue work (the step
 *     calls, compams_encode, compams_decode) may come on different streams: a
 *     call on another stream than the previous one first makes its stream wait,
 *     on the device, for everything the context has enqueued so far (an event
 *     made at compams_init; the host does not wait).  Ordering the caller's own
 *     work (filling g, reading state) against those streams stays the caller's,
 *     and so does the order of graph replays: a stream under capture runs
 *     nothing and takes no part in this.
 *   - The device that was current at compams_init() must be current at every
 *     later call on the context (COMPAMS_BAD_STATE otherwise).
 */
#ifndef COMPAMS_H
#define COMPAMS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct compams_ctx compams_ctx; /* opaque; host memory owned by the library */

/* The compressor C of Assumption 1. */
enum {
  COMPAMS_NONE = 0,     /* C(x) = x (q = 0): full-precision distributed AMSGrad (Algorithm 1, which has no residual);
                           e is neither read nor written and stays zero, also for an infinite gradient entry,
                           where the error line of Algorithm 2 taken literally (Inf - Inf) would leave a NaN */
  COMPAMS_TOPK = 1,     /* Definition 1: keep the k coordinates of largest magnitude per worker */
  COMPAMS_BLOCKSIGN = 2, /* Definition 2: per block, sign(x) times the block's mean absolute value */
  COMPAMS_TOPK_BLOCKS = 3 /* Definition 1 applied to every block on its own: block b keeps its block_k[b] coordinates
                             of largest magnitude per worker (the usual per-layer top-k).  Block offsets must be
                             multiples of 4.  Workspace grows with n * num_blocks (about 35 KB each): meant for
                             layer-sized blocks */
};

/* Where epsilon sits in the parameter line of Algorithms 1 and 2. */
enum {
  COMPAMS_EPS_IN_SQRT = 0, /* theta -= lr * m / sqrt(vhat + eps)   (as printed in the paper) */
  COMPAMS_EPS_OUT_SQRT = 1 /* theta -= lr * m / (sqrt(vhat) + eps) */
};

enum {
  COMPAMS_KEEP_STATE = 1 /* compams_init() leaves e, m, v, vhat as the caller filled them (resume) */
};

enum {
  COMPAMS_OK = 0,
  COMPAMS_INVALID_ARG = -1,         /* null pointer, size out of range, bad enum, offsets not ascending */
  COMPAMS_BAD_ALIGNMENT = -2,       /* a device pointer is not 16-byte aligned, or ld is not a multiple of 4 */
  COMPAMS_WORKSPACE_TOO_SMALL = -3, /* workspace_bytes < compams_workspace_size() */
  COMPAMS_HIP_ERROR = -4,           /* a HIP runtime call failed */
  COMPAMS_BAD_STATE = -5            /* the call does not apply to this context: wrong compressor for the query,
                                       another device is current, or an earlier step failed with COMPAMS_HIP_ERROR
                                       half-way (the context can then only be destroyed) */
};

typedef struct compams_config {
  int32_t n;          /* number of workers (rows), 1 <= n <= 65535 */
  int64_t d;          /* coordinates per worker, 1 <= d < 2^31 */
  int64_t ld;         /* row stride of g and e in elements: ld >= d and ld % 4 == 0; a multiple of 1024 (rows that
                         start on 4 KiB boundaries) streams about 8 % faster than an odd stride */
  int32_t compressor; /* COMPAMS_NONE / COMPAMS_TOPK / COMPAMS_BLOCKSIGN / COMPAMS_TOPK_BLOCKS */
  int64_t k;          /* top-k: 1 <= k <= d, per worker over the whole flattened row; else ignored */
  int64_t num_blocks; /* block-sign, top-k per block: number of blocks M >= 1; else ignored */
  const int64_t* block_offsets; /* HOST, block-sign, top-k per block: M+1 strictly ascending offsets, [0] = 0,
                                   [M] = d; copied */
  float beta1, beta2, eps;      /* the paper's defaults are 0.9, 0.999, 1e-8 (Section 5.1) */
  int32_t eps_mode;             /* COMPAMS_EPS_* */
  int32_t flags;                /* bit set of COMPAMS_KEEP_STATE */
  /* DEVICE buffers, 16-byte aligned, borrowed for the life of the context */
  float* theta; /* d: the parameter, theta_1 on entry to the first step */
  float* m;     /* d: first moment  */
  float* v;     /* d: second moment */
  float* vhat;  /* d: running maximum of v */
  float* e;     /* n * ld: error accumulators, row i = worker i; columns >= d are never touched.  Between steps
                   the contents are the library's: see compams_step() */
  void* workspace;        /* DEVICE scratch of at least compams_workspace_size() bytes, 256-byte aligned */
  size_t workspace_bytes;
  const int64_t* block_k; /* HOST, top-k per block: M counts, 1 <= block_k[b] <= size of block b; copied; else
                             ignored (may be NULL).  The workers' lists then hold sum(block_k) entries: the kept
                             coordinates of block 0, of block 1, ...: ascending over the whole row */
} compams_config;

/* Bytes of device workspace this configuration needs (0 on an invalid configuration).
 * Host-only; reads n, d, compressor, k, num_blocks (and block_offsets, block_k for top-k per block).
 * The workspace holds what the workers "send" in Algorithm 2 (the kept coordinates and values of Definition 1,
 * the sign words and block means of Definition 2) and the tables of the selection; the paper's own state
 * (theta, m, v, vhat, e_i: Algorithm 2's input and initialisation lines) is never kept there. */
size_t compams_workspace_size(const compams_config* cfg);

/* Validates cfg, copies it, lays out the workspace, uploads the block offsets and, unless
 * COMPAMS_KEEP_STATE is set, zeroes e, m, v and vhat (the initialisation line of Algorithm 2).
 * Blocks until that set-up work has finished.  *out receives the context. */
int compams_init(const compams_config* cfg, compams_ctx** out);

/* One iteration of Algorithm 2 with learning rate lr (eta_t).
 *   g: DEVICE, n * ld floats, row i = worker i's stochastic gradient; read-only; may be reused by the
 *      caller once the stream has passed the step.
 *   hip_stream: a hipStream_t (NULL = the default stream).  All kernels of the step are enqueued there.
 * Top-k ties are broken towards the larger |x| and then the lower index, with |x| ordered by the fp32
 * bit pattern without its sign bit; the selected indices come out ascending per worker.  Block-sign
 * uses sign(x) = -1 iff x < 0 and the exactly summed block L1 norm.  The average adds the workers'
 * compressed gradients in the order 0..n-1 in fp32 and divides by n.
 * The error line of Algorithm 2 (e <- x - C(x)) may be left pending when the step returns: e then still
 * holds the corrected gradient x where the update has not been applied (top-k: at the selected
 * coordinates; block-sign: everywhere), and the next step applies it while it reads e.
 * compams_state(COMPAMS_STATE_E) and compams_destroy() apply what is pending first (one kernel on the last
 * step's stream); do not read or write the e buffer between steps by any other route.  Every other result
 * of the step is final when the stream has passed it.
 * Stream capture: the call only enqueues kernel launches on hip_stream (no allocation, no synchronisation, no
 * memset or copy node; profiling must be off), so it may be recorded into a HIP graph.  Which kernels are
 * enqueued depends on the context's state at that moment (the first step of a context differs from the later
 * ones; a pending error line is applied by the step that follows): record a step after at least one step has
 * run, replay it with new gradients copied into the same g, and record it again after a call that applies
 * the pending error line (compams_state(COMPAMS_STATE_E), compams_server_step) if replays are to follow. */
int compams_step(compams_ctx* ctx, const float* g, float lr, void* hip_stream);

/* What compams_state() can hand out.  Counts are in elements of the listed type.
 * 0..4 are the state of Algorithm 2: its parameter theta_t, the moments m_t, v_t and the running maximum vhat_t
 * of its server lines, and the workers' error accumulators e_{t,i} (all zero after the initialisation line,
 * theta_1 the caller's).  5..8 are what the workers sent in the last step (the send line of Algorithm 2, in the
 * form of Definition 1 or Definition 2).  The rest describes how the last selection went. */
enum {
  COMPAMS_STATE_THETA = 0,          /* float[d] */
  COMPAMS_STATE_M = 1,              /* float[d] */
  COMPAMS_STATE_V = 2,              /* float[d] */
  COMPAMS_STATE_VHAT = 3,           /* float[d] */
  COMPAMS_STATE_E = 4,              /* float[n*ld]; asking for it applies a pending residual update first */
  COMPAMS_STATE_LAST_IDX = 5,       /* top-k: int32[n*k], worker i's selected coordinates, ascending */
  COMPAMS_STATE_LAST_VAL = 6,       /* top-k: float[n*k], the corrected gradient at those coordinates */
  COMPAMS_STATE_LAST_SIGNBITS = 7,  /* block-sign: uint32[n*ceil(d/32)], bit (j&31) of word j>>5 = (x_j < 0) */
  COMPAMS_STATE_LAST_SCALES = 8,    /* block-sign: float[n*M], the block means of |x| */
  COMPAMS_STATE_LAST_THRESHOLD = 9, /* top-k: uint32[n], magnitude key of the k-th largest entry (top-k per block:
                                       uint32[n*M], worker-major; likewise the count and the counters below) */
  COMPAMS_STATE_COUNTERS = 10,      /* uint32[n*COMPAMS_COUNTERS_PER_ROW], see below */
  COMPAMS_STATE_LAST_COUNT_GT = 11, /* top-k: uint32[n], selected entries strictly above the threshold key (the
                                       other k - that many are ties, taken in coordinate order) */
  COMPAMS_STATE_PENDING = 12        /* a host-side answer, no pointer: *dev_ptr = NULL and *count = 1 if the error
                                       line of the last step is still pending (see compams_step), else 0.  A step
                                       recorded into a HIP graph while the answer was 1 must be replayed only while
                                       it is 1 (and the other way round) */
};

/* Per-worker counters of the last step (top-k), for tests and profiling reports. */
enum {
  COMPAMS_CNT_DENSE_READS = 0, /* how many times the step read the whole row of corrected gradients back
                                  (0: candidates came out of the first pass; 1: the candidate list had to be made
                                  from the stored row; 4: no candidate list) */
  COMPAMS_CNT_CANDIDATES = 1,  /* entries in the candidate list, 0 if none was used */
  COMPAMS_CNT_TIES = 2,        /* coordinates whose key equals the threshold key */
  COMPAMS_CNT_TIES_TAKEN = 3,  /* how many of those were selected */
  COMPAMS_CNT_BAND = 4,        /* entries in the band list if the threshold key was found there (the selection then
                                  took a single launch), else 0 */
  COMPAMS_CNT_BAND_MISS = 5,   /* why not: 0 = it was; 1 = the step had no window to offer (first steps, options, blocks of
                                  at most 1024 coordinates); 2 = the candidate list did not fit; 3 = the band list did
                                  not fit; 4 / 5 = the threshold key lay above / below the window; 6 = its bucket held
                                  more than 64 entries (many equal or nearly equal magnitudes) */
  COMPAMS_COUNTERS_PER_ROW = 8 /* 6, 7 are reserved and read 0 */
};

/* Borrowed DEVICE pointer to a state tensor or to what the workers "sent" in the last step, valid until
 * the next compams_step() on the context changes it.  Reading it is the caller's business (ordered after
 * the step on the step's stream). */
int compams_state(compams_ctx* ctx, int which, const void** dev_ptr, int64_t* count);

/* Knobs.  None of them changes any result; they decide which route the top-k selection takes, or how memory is
 * accessed, and exist for tests of the rarely taken routes and for ablation measurements.  Options 0..3 are for the
 * top-k compressors only (COMPAMS_BAD_STATE otherwise). */
enum {
  COMPAMS_OPT_CANDIDATE_CAP = 0, /* candidate-list capacity per worker, 0 .. the capacity the workspace was sized
                                    for (min(d, 8k + 65536)); a list that would not fit is not built.  Rows of 64
                                    chunks (262144 coordinates) and more keep the list as eight runs of an eighth
                                    of the capacity each, filled by every eighth chunk of the row: a run that would
                                    not fit counts as a list that would not fit */
  COMPAMS_OPT_PREDICT = 1,       /* 1 (default): the first pass of a step already writes the candidate list, using
                                    the previous step's threshold bucket as a guess that is verified afterwards */
  COMPAMS_OPT_FORCE_DENSE = 2,   /* 1: never build a candidate list; every selection pass reads the whole row */
  COMPAMS_OPT_BAND = 3,          /* 1 (default): the first pass also gets a window of keys around the threshold
                                    expected from the last two steps, counts what lies above it and lists what lies
                                    inside; when the threshold does fall inside (verified exactly), one launch
                                    finishes the selection from that short list */
  COMPAMS_OPT_CACHED_ARRAYS = 4  /* every compressor: how many of theta, m, v, vhat (in that order) the server's
                                    lines read and write with ordinary accesses, the others with streaming ones:
                                    0..4, or -1 (default) for compams_cached_state_arrays(d) */
};
int compams_set_option(compams_ctx* ctx, int option, int64_t value);

/* Optional per-kernel timing.  enable = 1: compams_step() brackets every kernel with HIP events on the
 * step's stream (about 3 us per kernel of extra time); enable = 2: only the kernel that moves most of the
 * step's bytes is bracketed; enable = 0: off.  compams_profile_read() waits for the recorded events, then
 * fills names[i] (static strings), ms[i] (total milliseconds since the last reset) and launches[i] for up to
 * cap kernels, returns how many kernels there are through *count, and resets the totals. */
int compams_profile_enable(compams_ctx* ctx, int enable);
int compams_profile_read(compams_ctx* ctx, int cap, const char** names, double* ms, int64_t* launches, int* count);

/* Ends the sequence of steps: applies a pending error line (so that e holds e_{t+1,i} of Algorithm 2, as
 * compams_state(COMPAMS_STATE_E) would), waits for it, and frees the context (host memory and HIP events only;
 * device buffers stay the caller's). */
int compams_destroy(compams_ctx* ctx);

/* Static description of a status code. */
const char* compams_strerror(int status);

/* ---- The workers' messages on the wire ------------------------------------------------------------------
 * What a worker sends to the server in its send line of Algorithm 2, as one contiguous sequence of 32-bit
 * little-endian words per worker.  The paper fixes only the accounting (experiments section: 32 bits per
 * transmitted float); the layout below is this library's.
 *
 *   top-k (Definition 1)       [1, k, 256,  width words,  gap stream,  k value words]
 *       The kept coordinates are ascending; gap_0 = idx_0 and gap_q = idx_q - idx_{q-1} - 1.  The gaps are
 *       taken in tiles of 256 (the last tile may be shorter).  Tile t has its own width b_t (1..31), the number
 *       of bits of its largest gap (1 if all its gaps are 0), kept as byte (t mod 4) of width word t div 4;
 *       there are ceil(ceil(k/256)/4) width words and their unused bytes are 0.  In the stream the tiles follow
 *       one another, each starting on a word boundary and taking ceil(count_t * b_t / 32) words: gap i of a
 *       tile occupies the tile's bits i*b_t .. i*b_t+b_t-1, least significant bit first; bit u of a tile is bit
 *       (u mod 32) of its word u div 32; the unused high bits of a tile's last word are 0.  The values are the
 *       fp32 patterns of the corrected gradient at the kept coordinates, in the same order.
 *   block-sign (Definition 2)  [2, d, M,  ceil(d/32) sign words,  M scale words]
 *       Bit (j mod 32) of sign word j div 32 is 1 iff x_j < 0 (unused bits 0); scale b is the fp32 mean of
 *       |x| over block b.
 *
 * Bits per worker and step: 32 * (message length in words).  For comparison the paper counts 32*d bits for an
 * uncompressed gradient; a top-k message is between 32*k (its values alone) and about 64*k bits.
 *
 * compams_wire_capacity: the largest message (in words) a worker of this configuration can produce; pure,
 *   host only; 0 for an invalid configuration or COMPAMS_NONE (nothing is compressed: the message would be
 *   the gradient row itself).
 * compams_encode: packs the n messages of the last step.  messages: DEVICE, n * stride_words words, worker
 *   i's message starts at messages + i * stride_words (stride_words >= capacity); words_out: DEVICE, n
 *   words, receives each message's length.  Enqueued on hip_stream (the step's stream, or one ordered after
 *   it).  COMPAMS_BAD_STATE before the first step or for COMPAMS_NONE.
 * compams_decode: the inverse, for n messages laid out the same way.  words: DEVICE, the n lengths, or NULL
 *   (then lengths are not checked).  top-k: out_a = int32[n*k] coordinates, out_b = float[n*k] values;
 *   block-sign: out_a = uint32[n*ceil(d/32)] sign words, out_b = float[n*M] scales (all DEVICE, caller-owned).
 *   status_out: DEVICE, n words: 0 if message i was well formed, else bit 0 = not a message of this kind and
 *   size or a tile width outside 1..31, bit 1 = length differs from `words`, bit 2 = a coordinate at or
 *   beyond d.  Malformed input never makes the library read outside [message, message + stride_words); the
 *   outputs for such a message are unspecified.  Uses the context's workspace: not concurrent with
 *   compams_step or another decode on the same context. */
size_t compams_wire_capacity(const compams_config* cfg);
int compams_encode(compams_ctx* ctx, uint32_t* messages, int64_t stride_words, uint32_t* words_out, void* hip_stream);
int compams_decode(compams_ctx* ctx, const uint32_t* messages, int64_t stride_words, const uint32_t* words,
                   void* out_a, void* out_b, uint32_t* status_out, void* hip_stream);

/* ---- The two halves of a step ---------------------------------------------------------------------------
 * Algorithm 2 as printed has the workers and the server on different machines.  compams_step() runs both
 * halves on one device; these two calls run them apart, with the packed messages in between.
 *
 * compams_worker_step: the workers' lines for the context's n rows: x = e + g, the compressor, the error
 *   update (possibly left pending, see compams_step).  Leaves the messages in the workspace (compams_state
 *   LAST_*, compams_encode).  Neither reads nor writes theta, m, v, vhat.  COMPAMS_BAD_STATE for COMPAMS_NONE
 *   (nothing is compressed: the message is the gradient row itself).
 * compams_server_step: the server's lines from n packed messages (laid out as for compams_decode; message i
 *   is worker i in the fixed order of the average): unpacks them into the workspace, adds them in that order,
 *   divides by n and applies the AMSGrad lines with learning rate lr.  Reads no gradient; touches e only to
 *   apply a residual update of this same context that is still pending (on the stream of the step that left
 *   it; this call's stream then waits for that one on the device).  status_out: as for compams_decode; a
 *   message that is not well formed still contributes whatever it unpacks to (never read out of bounds), so
 *   check status_out.
 * compams_worker_step + compams_encode on one context followed by compams_server_step on a context of the
 * same configuration gives, bit for bit, the state that compams_step gives. */
int compams_worker_step(compams_ctx* ctx, const float* g, void* hip_stream);
int compams_server_step(compams_ctx* ctx, const uint32_t* messages, int64_t stride_words, const uint32_t* words,
                        float lr, uint32_t* status_out, void* hip_stream);

/* A plain streaming copy of `bytes` bytes (multiple of 16, both pointers DEVICE and 16-byte aligned) with
 * the same launch style as the step's dense kernels: the measured bandwidth ceiling that reports set
 * beside the step's figures, and the known-size kernel that hardware counters are calibrated against. */
int compams_copy(void* dst, const void* src, size_t bytes, void* hip_stream);

/* How many of theta, m, v, vhat (in that order) the kernels that apply the server's lines of Algorithm 2 read and
 * write with ordinary accesses for a problem of d coordinates, so that they stay in the memory-side cache from
 * one step to the next; the others are streamed past it.  As many as fit a fixed share of that cache together:
 * 0..4 (4 for every small d).  Pure, host-only; COMPAMS_INVALID_ARG for d < 1. */
int compams_cached_state_arrays(int64_t d);

/* A second measured ceiling, for the server's lines of Algorithm 2 (theta, m, v, vhat each read once and
 * written once, in place): n_arrays (1..4) separately allocated fp32 arrays of `count` elements each are
 * updated in place, x += 1, by a workgroup per 4096 elements that takes that stretch of every array, 16 bytes
 * per lane and access - the access pattern of those lines without their arithmetic and without the look-ups
 * that precede them.  What the box gives this pattern bounds the kernels that apply those lines.
 *   arrays: HOST array of n_arrays DEVICE pointers (16-byte aligned, distinct, count elements each, modified).
 *   count: multiple of 4.  cached_arrays (0..4): the first that many arrays are accessed with ordinary loads
 *   and stores, the others with non-temporal ones (see compams_cached_state_arrays).
 * Only enqueues on hip_stream.  COMPAMS_INVALID_ARG / COMPAMS_BAD_ALIGNMENT as for compams_copy. */
int compams_inplace_probe(float* const* arrays, int n_arrays, size_t count, int cached_arrays, void* hip_stream);

/* ---- One whole step for callers that cannot allocate ------------------------------------------------------
 * For code that runs where no device memory can be allocated or handed over as a workspace (under HIP graph
 * capture, in a tight serving loop, in a harness that forbids it): compams_init + compams_step +
 * compams_state(COMPAMS_STATE_E) + compams_destroy in one call that allocates nothing, on the device or through
 * any library.  The tables of the selection live in a device array inside the library, COMPAMS_STATIC_SCRATCH_BYTES
 * large, that every device the library has run this call on holds until the process ends.
 *   cfg: as for compams_init (same checks, same status codes), with compressor = COMPAMS_TOPK (else
 *        COMPAMS_BAD_STATE: the other compressors need tables copied from the host) and with workspace and
 *        workspace_bytes ignored.  A configuration whose compams_workspace_size() exceeds
 *        COMPAMS_STATIC_SCRATCH_BYTES is rejected with COMPAMS_WORKSPACE_TOO_SMALL before anything is enqueued.
 *        Without COMPAMS_KEEP_STATE the call first zeroes e, m, v, vhat (a first step); with it, e must hold the
 *        error accumulators in their settled form (as compams_state(COMPAMS_STATE_E) or this call left them).
 *   g, lr: as for compams_step.
 *   idx_out, val_out: DEVICE, n * k entries each, or NULL: receive what the workers sent (COMPAMS_STATE_LAST_IDX,
 *        COMPAMS_STATE_LAST_VAL).
 * Only enqueues kernels on hip_stream (no copy or memset node, no synchronisation).  When the stream has passed
 * the call, theta, m, v, vhat and e hold the result of one iteration of Algorithm 2 with nothing left pending:
 * bit for bit what the four calls above give.  Nothing is carried from one call to the next (no threshold guess:
 * every call reads the rows of corrected gradients a second time), so it is the slower way to step.
 * All calls on one device share that device's array: calls that overlap in time on one device (two streams, two
 * threads) race; calls on one stream, or otherwise ordered, do not. */
#define COMPAMS_STATIC_SCRATCH_BYTES (32u << 20)
int compams_step_static(const compams_config* cfg, const float* g, float lr, int32_t* idx_out, float* val_out,
                        void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* COMPAMS_H */
