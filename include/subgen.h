/*
 * subgen.h — C ABI of the SubGen decode-step library for AMD MI355X (gfx950).
 *
 * SubGen (Zandieh, Han, Mirrokni, Karbasi: "SubGen: Token Generation in
 * Sublinear Time and Memory") keeps, per attention stream, a compressed KV
 * cache made of
 *   D  — an online threshold clustering of the keys: representatives x_i and
 *        counts n_i (Algorithm 1, procedure UpdateSoftmaxNormalizer; Lemma 2),
 *   M  — s slots of (k, v) pairs sampled with probability proportional to
 *        ||v||^2, and mu = sum ||v||^2 (procedure UpdateMatrixProduct; Lemma 1),
 *   W  — the w most recent tokens, kept exactly (Section 3.2, sliding window),
 * and answers a query q with z / tau (procedure QueryStreamAttn).
 *
 * A "stream" is one (sequence, layer, KV head).  All streams of a context
 * advance in lock-step, one token per call.  Every entry point below runs on
 * the GPU in hand-written HIP kernels; there is no host fallback.
 *
 * Conventions
 *   - Pointers named K*, V*, Q*, out are DEVICE pointers owned by the caller,
 *     16-byte aligned, valid until the work enqueued by the call has run
 *     (calls are asynchronous on the context's HIP stream).  Host pointers
 *     are marked "host".
 *   - Element type (fp32 or bf16) is fixed per context; rows are stored as
 *     verbatim copies of the inputs.
 *   - No 1/sqrt(d) is applied: the paper's attention is softmax(K q) (Eq. 1);
 *     callers pre-scale q.
 *   - Every function returns SUBGEN_OK (0) or a negative error code; nothing
 *     aborts, throws or prints.  A context is not thread-safe; distinct
 *     contexts are independent.
 *   - Semantics of the window: a token is held exactly while it is among the
 *     last w; when it leaves the window it is clustered and offered to the
 *     sampler.  So counts, samples and mu cover the tokens that left the
 *     window ("evicted"), window tokens contribute exact terms, nothing is
 *     counted twice:  sum_i n_i + |W| = tokens seen.
 */
#ifndef SUBGEN_H
#define SUBGEN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct subgen_ctx subgen_ctx; /* opaque; owned by the library from create to destroy */

enum {
    SUBGEN_OK = 0,
    SUBGEN_EINVAL = -1,    /* bad argument (null, misaligned, unsupported shape, non-finite delta) */
    SUBGEN_ENOMEM = -2,    /* device or host allocation failed                                     */
    SUBGEN_EHIP = -3,      /* a HIP call failed; see subgen_last_hip_error                         */
    SUBGEN_EEMPTY = -4,    /* attend before any token                                              */
    SUBGEN_ECAPACITY = -5  /* a size given to this call exceeds what it can take (a workspace that is too
                              small, more workgroups than a launch holds).  Device-side capacities do not
                              use it: a full center table raises SUBGEN_FLAG_CENTER_OVERFLOW, and the
                              assignment log simply stops after assign_log_tokens entries                 */
};

enum { SUBGEN_F32 = 0, SUBGEN_BF16 = 1 };

/* bits of the sticky per-stream flag word (subgen_stats, subgen_export_state) */
enum {
    SUBGEN_FLAG_CENTER_OVERFLOW = 1u, /* the center table was full: a token joined its nearest center regardless of delta */
    SUBGEN_FLAG_NONFINITE = 2u        /* a token that left the window held NaN or Inf (or a squared norm beyond fp32):
                                         it was dropped, i.e. neither clustered nor sampled                           */
};

/* Options of subgen_create.  Zero-initialise, set struct_size = sizeof(subgen_opts), then override. */
typedef struct subgen_opts {
    uint32_t struct_size;
    int32_t dtype;          /* SUBGEN_F32 (default) or SUBGEN_BF16: element type of K, V, Q and stored rows */
    int32_t q_per_stream;   /* g: queries answered per stream per attend (GQA group size); 0 -> 1; 1, 2 or 4 */
    int32_t max_centers;    /* per-stream capacity of the center table; 0 -> 4096                          */
    int64_t assign_log_tokens; /* if > 0: record the center index of the first this-many evicted tokens of every stream */
    uint64_t seed;          /* key of the counter-based generator behind the sampling coin flips           */
    void *hip_stream;       /* hipStream_t every call enqueues on; NULL = the default stream               */
    int32_t device;         /* HIP device ordinal; -1 (or struct zeroed with device_set = 0) = current     */
    int32_t device_set;     /* non-zero: use `device`                                                      */
    int32_t kernel_path;    /* 0 = automatic (bf16 rows are scored on the matrix cores where the shape allows);
                               1 = always the generic vector-ALU kernels (any dtype; same results up to fp32
                               rounding of the outputs, identical decisions);
                               2 = as 0, but never the wide-workgroup kernels that 0 picks for contexts of at
                               most 256 streams (the kernels of large contexts on a small one: for tests)     */
    int32_t t_per_cluster;  /* t: reservoir slots per cluster.  0 (default) = representative mode: the normaliser is
                               sum_i n_i e^{<q,x_i>}.  t >= 1 = Algorithm 1 as printed: every cluster keeps t uniform
                               samples S_i of its keys and the normaliser is sum_i (n_i/t) sum_{k in S_i} e^{<q,k>}
                               (Lemma 2 (5), QueryStreamAttn); at most 64                                      */
    int32_t device_counter; /* 1 = the number of tokens seen is kept in device memory and advanced by a one-lane
                               kernel behind every update, so that update / attend / step / ingest launches can
                               be captured into a HIP graph and replayed (each replay consumes the buffers it was
                               captured with, at the position the stream has reached by then).  The host's own
                               count, which the argument checks (SUBGEN_EEMPTY, the log capacity) and
                               subgen_export_state use, is brought up to date by every synchronising call; call
                               subgen_sync after replaying graphs.  0 (default) = the count is a kernel argument */
    int32_t out_dtype;      /* element type of the attention outputs: SUBGEN_F32 (default; what the 2e-3 parity bar is
                               stated on) or SUBGEN_BF16 (the fp32 result rounded to nearest even at the store)  */
    int32_t split_workgroups; /* workgroups that share one stream in update / attend / step.  0 = automatic: one per
                               stream, except in contexts of at most 32 streams (kernel_path 0, representative mode),
                               where 8 to 32 of them bring the launch to about 256 workgroups: a context of a few
                               streams would otherwise leave most of the chip idle.  1 = always one per
                               stream.  2 .. 64 = that many.  State and decisions do not depend on this; outputs
                               agree to fp32 rounding                                                          */
    int32_t reserved_;      /* padding: zero */
} subgen_opts;

/*
 * subgen_create — allocate the state of `streams` independent streams (Section 2.1: the data
 * structure of the streaming attention problem; Algorithm 1, initialisation: mu = 0, D empty,
 * M all null).
 *   d              head dimension; row bytes (d * element size) must be 128, 256 or 512
 *                  (fp32: d = 32, 64, 128; bf16: d = 64, 128, 256)
 *   delta          cluster threshold (Definition 1; Algorithm 1 joins iff ||k - x|| <= delta), >= 0
 *   sample_budget  s >= 1, number of slots of M
 *   window         w >= 0, recent tokens kept exactly (Section 3.2)
 *   opts           may be NULL (all defaults)
 * All device memory of the context is allocated here and released by subgen_destroy.
 */
int subgen_create(subgen_ctx **out, int64_t streams, int32_t d, float delta, int32_t sample_budget,
                  int32_t window, const subgen_opts *opts);

void subgen_destroy(subgen_ctx *ctx);

/*
 * subgen_update — one new token per stream (Algorithm 1, main loop: UpdateSoftmaxNormalizer,
 * UpdateMatrixProduct, mu += ||v||^2, applied to the token the window pushes out).
 *   K_t, V_t   device, [streams, d] contiguous, context dtype.
 */
int subgen_update(subgen_ctx *ctx, const void *K_t, const void *V_t);

/*
 * subgen_attend — QueryStreamAttn (Algorithm 1) plus the exact window terms:
 *   den = sum_{j in W} e^{<q,k_j>} + sum_i n_i e^{<q,x_i>}      (or the t-sample form, see t_per_cluster)
 *   num = sum_{j in W} e^{<q,k_j>} v_j + sum_{j in M} mu / (s ||v_j||^2) e^{<q,k_j>} v_j
 *   out = num / den      (a common maximum is subtracted from every exponent; fp32 accumulation)
 *   Q_t   device, [streams, g, d] contiguous, context dtype
 *   out   device, [streams, g, d] contiguous, fp32 (or bf16 with opts.out_dtype), fully overwritten
 * Returns SUBGEN_EEMPTY if no token has been given yet.
 */
int subgen_attend(subgen_ctx *ctx, const void *Q_t, void *out);

/*
 * subgen_attend_many — QueryStreamAttn (Algorithm 1, with the window of Section 3.2) for a block of
 * n_queries queries per stream against the current state: the queries of a chunk of prompt tokens, of a
 * speculative draft, or of a wide grouped-query head group.  Every query gets exactly what subgen_attend
 * would give it; n_queries is independent of the context's q_per_stream.  The state is not changed.
 *   Q     device, [streams, n_queries, d] contiguous, context dtype
 *   out   device, [streams, n_queries, d] contiguous, fp32 (or bf16 with opts.out_dtype), fully overwritten
 * bf16 contexts with d = 64 or 128 in representative mode run both contractions (scores, weights x values)
 * on the matrix cores and read the state once per 64 queries; other contexts answer the queries in groups of
 * at most four with the decode kernels.
 * Returns SUBGEN_EINVAL for n_queries outside 1..2^20, SUBGEN_EEMPTY if no token has been given yet.
 */
int subgen_attend_many(subgen_ctx *ctx, const void *Q, int32_t n_queries, void *out);

/*
 * subgen_step — one decode step of Algorithm 1 (update with (K_t, V_t), then query with Q_t) in a
 * single pass over the center table.  State and output equal subgen_update followed by subgen_attend.
 */
int subgen_step(subgen_ctx *ctx, const void *K_t, const void *V_t, const void *Q_t, void *out);

/*
 * subgen_ingest_prefix — stream n prompt tokens per stream through the update (the paper counts
 * prompt and generated tokens alike, Section 1.2); equals n calls of subgen_update in order, and
 * may be called repeatedly with consecutive chunks.
 *   K, V            device; token t of stream j starts at element j*stream_stride + t*token_stride
 *   stream_stride, token_stride   in elements; rows must stay 16-byte aligned; token_stride >= d
 */
int subgen_ingest_prefix(subgen_ctx *ctx, const void *K, const void *V, int64_t n, int64_t stream_stride,
                         int64_t token_stride);

/*
 * subgen_exact_attend — exact full-KV decode attention softmax(K q)^T V (Eq. 1), for context
 * numbers beside the compressed path.  Independent of any context.
 *   K, V       device, [streams, n, d] contiguous, `dtype`
 *   Q          device, [streams, g, d]; out device [streams, g, d] fp32
 *   workspace  device scratch of at least subgen_exact_workspace_bytes(streams, n, d, g) bytes
 *   hip_stream hipStream_t or NULL
 */
size_t subgen_exact_workspace_bytes(int64_t streams, int64_t n, int32_t d, int32_t g);
int subgen_exact_attend(const void *K, const void *V, const void *Q, void *out, int64_t streams, int64_t n,
                        int32_t d, int32_t g, int32_t dtype, void *workspace, size_t workspace_bytes,
                        void *hip_stream);

/*
 * subgen_exact_attend_noalloc — subgen_exact_attend for callers that cannot allocate device memory and have no
 * workspace to pass: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * kernels, same arguments and same results as subgen_exact_attend; the split partials go to a buffer that is part
 * of the library itself (a 32 MiB array in device memory, one copy per GPU that loads the library, held until
 * the process ends).  The call path contains no hipMalloc, hipFree or other allocating routine.
 *   Returns SUBGEN_ECAPACITY when subgen_exact_workspace_bytes(streams, n, d, g) exceeds
 *   subgen_exact_noalloc_max_bytes() (32 MiB: e.g. up to 16384 streams x 4 queries at d = 128).
 *   The device that is current at the call is the one whose buffer is used; K, V, Q, out must live there.
 *   All calls on one GPU share that GPU's buffer: two such calls that overlap in time on one GPU (different
 *   HIP streams, or host threads) race.  Calls on one HIP stream are ordered and need no clearing in between:
 *   every partial a call reads it has written itself.
 */
size_t subgen_exact_noalloc_max_bytes(void);
int subgen_exact_attend_noalloc(const void *K, const void *V, const void *Q, void *out, int64_t streams, int64_t n,
                                int32_t d, int32_t g, int32_t dtype, void *hip_stream);

/*
 * subgen_kcenter_compress — one-shot greedy k-center compression of a prompt's KV cache (Section 3.2: the
 * variant of the paper's line-retrieval experiment: the greedy k-center algorithm is applied once to the whole
 * cache, the r most recent tokens are retained in addition to k centers selected from the remaining tokens).
 * Farthest-point traversal: the first center is token 0, each next center is the token (older than the window)
 * farthest from the centers chosen so far, lowest index on ties; squared distances in double precision.
 * Independent of any context; the result is a cache of k + r rows to run subgen_exact_attend on.
 *   K, V        device, [streams, n, d] contiguous, `dtype`
 *   out_K, out_V device, [streams, k + r, d]: the centers in selection order, then the r most recent tokens
 *                (oldest first); rows that do not exist (n - r < k, or n < r) are zero
 *   out_idx     device, [streams, k + r] int32: token index of every output row, -1 for rows that do not exist
 *   out_counts  device, [streams, k] int32 or NULL: number of tokens older than the window whose nearest center
 *                (lowest index on ties) is that center
 *   workspace   device scratch of at least subgen_kcenter_workspace_bytes(streams, n, r) bytes
 */
size_t subgen_kcenter_workspace_bytes(int64_t streams, int64_t n, int32_t r);
int subgen_kcenter_compress(const void *K, const void *V, int64_t streams, int64_t n, int32_t d, int32_t dtype, int32_t k,
                            int32_t r, void *out_K, void *out_V, int32_t *out_idx, int32_t *out_counts,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * subgen_hbm_read_probe — measurement aid, not part of the method: one plain streaming read of
 * `bytes` bytes of device memory (16-byte loads, grid-stride over `workgroups` workgroups of 256
 * lanes).  Timed by the caller, it gives the HBM read bandwidth a kernel reaches on this device,
 * the practical ceiling quoted beside the step kernel's roofline fraction.
 *   buf   device, 16-byte aligned, at least `bytes` bytes; sink  device, 4 bytes (never read back)
 *   region_bytes 0: grid-stride over the buffer; else workgroup b reads its own contiguous region
 *                [b*region_bytes, (b+1)*region_bytes), the pattern of one-stream-per-workgroup kernels
 *   nontemporal  non-zero: use the non-temporal (streaming) loads the decode kernels use for state rows
 */
int subgen_hbm_read_probe(const void *buf, size_t bytes, int32_t workgroups, int32_t nontemporal,
                          size_t region_bytes, void *sink, void *hip_stream);

/* Aggregate counters; synchronises the context's stream. */
typedef struct subgen_stats_t {
    uint32_t struct_size;
    uint32_t flags_or;        /* OR of all streams' sticky flag words           */
    int64_t streams;
    int64_t n_seen;           /* tokens given so far (same for every stream)    */
    int64_t n_evicted;        /* tokens that left the window, per stream        */
    int64_t total_centers;    /* sum over streams of m                          */
    int32_t min_centers, max_centers;
    int64_t flagged_streams;  /* streams with a non-zero flag word              */
} subgen_stats_t;

int subgen_stats(subgen_ctx *ctx, subgen_stats_t *host_out);

/* Per-stream number of centers; host_m is a host array of `streams` int32.  Synchronises. */
int subgen_center_counts(subgen_ctx *ctx, int32_t *host_m);

/*
 * subgen_export_state — copy one stream's state to host buffers (parity checks, checkpointing).
 * Scalars are always filled.  Each buffer pointer may be NULL (skipped); otherwise it must hold
 * the stated number of entries.  Rows are in the context dtype.  Synchronises.
 */
typedef struct subgen_state_view {
    uint32_t struct_size;
    uint32_t flags;           /* out: sticky flag word of the stream                      */
    int32_t m;                /* out: number of centers                                   */
    int32_t window_fill;      /* out: min(n_seen, w)                                      */
    int64_t n_seen;           /* out                                                      */
    int64_t n_evicted;        /* out                                                      */
    double mu;                /* out: sum of ||v||^2 over evicted tokens                  */
    int64_t centers_cap;      /* in: rows the two arrays below can hold (>= m else EINVAL) */
    void *centers;            /* host [centers_cap, d]                                    */
    int32_t *counts;          /* host [centers_cap]                                       */
    void *sample_K, *sample_V;/* host [s, d]                                              */
    int32_t *sample_idx;      /* host [s]: token index held by each slot, -1 = null; the index is kept in 32
                                 bits for reporting only (exact below 2^31 tokens per stream) — the sampler's
                                 counter-based coins use the full 64-bit token index                       */
    float *sample_vn;         /* host [s]: ||v||^2 of that token                          */
    void *window_K, *window_V;/* host [w, d], ring order: slot = token index mod w        */
    int64_t assign_cap;       /* in: entries assign can hold                              */
    int32_t *assign;          /* host: center index of evicted token 0.. (needs assign_log_tokens > 0) */
    int64_t assign_len;       /* out: entries written                                     */
    void *reservoirs;         /* host [centers_cap, t, d]: S_i of every cluster (t_per_cluster >= 1) */
} subgen_state_view;

int subgen_export_state(subgen_ctx *ctx, int64_t stream, subgen_state_view *host_view);

/*
 * subgen_import_state — the inverse of subgen_export_state: load one stream's state from host buffers
 * (checkpoint / resume).  The view must carry m, n_seen, mu, flags and every buffer (centers and counts
 * with at least m rows; sample_K, sample_V, sample_idx, sample_vn; window_K, window_V when w > 0), in the
 * layout export writes.  All streams of a context share one token counter: the first import into a fresh
 * context sets it, every further import must carry the same n_seen (else SUBGEN_EINVAL).  Because the coin
 * flips are counter-based (seed, stream, token, slot), a context restored this way and created with the same
 * seed continues bit-identically.  Synchronises.
 */
int subgen_import_state(subgen_ctx *ctx, int64_t stream, const subgen_state_view *host_view);

/* Block until everything enqueued on the context's stream has run. */
int subgen_sync(subgen_ctx *ctx);

const char *subgen_strerror(int code);

/* hipError_t of the last failing HIP call on this context (0 if none). */
int subgen_last_hip_error(const subgen_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* SUBGEN_H */
