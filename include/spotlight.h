/*
 * spotlight.h - C ABI of the Spotlight Attention decode hot path for AMD MI355X (gfx950).
 *
 * Per layer and per decode step the path is (paper: Sec. 3.1 Eq. 1-2, Sec. 3.2 Eq. 3-6, appendix
 * "Bit-Packing CUDA Kernel"):
 *
 *   1. hash      c = pack(sign(W2 SiLU(W1 x + b1)))   for the query and for each new key
 *   2. retrieve  Hamming distance (XOR + popcount) of the query code to every cached key code of
 *                the head, then the k nearest tokens per query head
 *   3. attend    softmax attention over exactly the gathered K/V rows
 *
 * Conventions for every entry point
 *   - All tensor arguments are DEVICE pointers owned by the caller, dense and contiguous in the
 *     layout written next to them.  The library never frees, resizes or keeps them after the call.
 *   - Work is enqueued on the HIP stream given at creation (or by spotlight_set_stream) and the
 *     call returns without waiting for it.  spotlight_create, spotlight_destroy and
 *     spotlight_profile_read are the only calls that synchronise.
 *   - Return value: SPOTLIGHT_OK (0) or a negative SPOTLIGHT_ERR_* code.  Arguments are checked
 *     on the host before the first HIP call, so argument errors never touch the GPU.
 *   - One context must not be used from two threads at once; calls that overlap on one context
 *     share its workspace and race.
 *
 * Symbols: d = head_dim (128), B = batch, Hq / Hkv = query / key-value heads, G = Hq / Hkv,
 * L = code_bits, W = L / 32, h = hidden, Nmax = max_tokens.  Query head hq reads key-value head
 * (and hash weights) hq / G.
 */
#ifndef SPOTLIGHT_H
#define SPOTLIGHT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct spotlight_ctx spotlight_ctx; /* opaque; owns only its workspace and timing events */

enum { SPOTLIGHT_F32 = 0, SPOTLIGHT_BF16 = 1 };

enum {
    SPOTLIGHT_OK = 0,
    SPOTLIGHT_ERR_INVALID_ARG = -1, /* null pointer, size out of range, inconsistent shapes  */
    SPOTLIGHT_ERR_UNSUPPORTED = -2, /* a well-formed request outside what the kernels cover  */
    SPOTLIGHT_ERR_WORKSPACE = -3,   /* workspace allocation failed                           */
    SPOTLIGHT_ERR_HIP = -4,         /* a HIP runtime call or kernel launch reported an error */
    SPOTLIGHT_ERR_TOO_LARGE = -5    /* spotlight_decode_step_noalloc: the shape needs more scratch than the fixed buffer holds */
};

/* Kernel stages, for spotlight_profile_read. */
enum {
    SPOTLIGHT_STAGE_HASH_KEYS = 0,  /* hash + pack of key rows                                   */
    SPOTLIGHT_STAGE_HASH_QUERY = 1, /* hash + pack of the query vectors                          */
    SPOTLIGHT_STAGE_SCORE = 2,      /* Hamming distances, histograms, candidate lists            */
    SPOTLIGHT_STAGE_SELECT = 3,     /* threshold, offsets, ordered output of the selected tokens */
    SPOTLIGHT_STAGE_ATTEND = 4,     /* gather + softmax attention over a split of the rows       */
    SPOTLIGHT_STAGE_MERGE = 5,      /* merge of the splits' partial results                      */
    SPOTLIGHT_STAGE_STEP_SMALL = 6, /* the whole decode step of a short context, as one kernel   */
    SPOTLIGHT_STAGE_COUNT = 7
};

/* Switches of a context, for spotlight_set_option. */
enum {
    /* 1 (default): a bulk spotlight_hash_keys call with bfloat16 weights evaluates the second hash
     * layer on the matrix cores (same codes, see spotlight_hash_keys); 0: everything on the binary32
     * fused-multiply-add chain. */
    SPOTLIGHT_OPT_BULK_HASH_MATRIX_CORES = 0,
    /* 1: the matrix-core bulk hash also evaluates EVERY output with the chain and records how far
     * the two results are apart (spotlight_bulk_hash_audit_read).  Slow; for tests.  Default 0. */
    SPOTLIGHT_OPT_BULK_HASH_AUDIT = 1,
    /* 1: spotlight_decode_step runs a short context (at most 65536 tokens, codes of at most 256
     * bits, at most 32 MB of codes in all) as ONE kernel launch, a workgroup per (batch, key-value
     * head); 0 (default): always the five launches of the general path.  Same codes and indices.
     * Off by default because it measured slower above about 4096 tokens per head (one compute
     * unit per head against eight or more). */
    SPOTLIGHT_OPT_STEP_SINGLE_LAUNCH = 2,
    SPOTLIGHT_OPT_COUNT = 3
};

typedef struct {
    int32_t batch;        /* B  >= 1                                                     */
    int32_t n_q_heads;    /* Hq >= 1, multiple of n_kv_heads, Hq / Hkv in 1 .. 8         */
    int32_t n_kv_heads;   /* Hkv >= 1                                                    */
    int32_t head_dim;     /* d; only 128 is supported                                    */
    int32_t code_bits;    /* L; multiple of 32 in [32, 512], or 1024 (then Hq / Hkv <= 2)   */
    int32_t hidden;       /* h in [0, 4096]; 0 selects the linear hash sign(xR), Eq. 4   */
    int64_t max_tokens;   /* Nmax: token capacity = row stride of K, V and codes         */
    int32_t max_topk;     /* largest k any call will pass, 1 <= max_topk <= max_tokens   */
    int32_t kv_dtype;     /* SPOTLIGHT_F32 or SPOTLIGHT_BF16: element type of q, K, V    */
    int32_t weight_dtype; /* SPOTLIGHT_F32 or SPOTLIGHT_BF16: element type of W1, b1, W2 */
    void *stream;         /* hipStream_t of the caller (NULL = the default stream)       */
} spotlight_config;

/* Hash MLP parameters (Eq. 5), device pointers, one MLP per key-value head, shared by the keys of
 * that head and by the G query heads that read it.
 *   hidden > 0 : w1 [Hkv, h, d], b1 [Hkv, h], w2 [Hkv, L, h]   (row = output unit)
 *   hidden == 0: w1 = R stored as [Hkv, L, d] (row = hash output), b1 = w2 = NULL      (Eq. 4) */
typedef struct {
    const void *w1;
    const void *b1;
    const void *w2;
} spotlight_hash_weights;

/* Checks a configuration on the host only (no HIP call).  SPOTLIGHT_OK if spotlight_create would
 * accept it. */
int spotlight_validate_config(const spotlight_config *cfg);

/* Bytes of device workspace spotlight_create allocates for cfg; 0 if cfg is invalid.  Host only. */
size_t spotlight_workspace_bytes(const spotlight_config *cfg);

/* Allocates the context and its device workspace on the current device.  *out is set only on
 * success.  The workspace holds the query codes, per-block distance histograms and candidate
 * lists (about one byte per (query head, token)), the partial attention results, and room for
 * one copy of the hash weights (spotlight_prepack_weights). */
int spotlight_create(spotlight_ctx **out, const spotlight_config *cfg);

/* Waits for the stream, frees the workspace and the context.  NULL is accepted. */
int spotlight_destroy(spotlight_ctx *ctx);

/* Changes the stream later calls enqueue on. */
int spotlight_set_stream(spotlight_ctx *ctx, void *stream);

/* Static text for a return code. */
const char *spotlight_strerror(int rc);

/* "SPOTLIGHT_BUILD_ID=" followed by the hash of the sources this library was compiled from. */
const char *spotlight_build_id(void);

/* Sets a SPOTLIGHT_OPT_* switch of the context.  Host only.  Errors: INVALID_ARG for a NULL context,
 * an unknown option or a value other than 0 / 1. */
int spotlight_set_option(spotlight_ctx *ctx, int option, int value);

/*
 * Optional, for callers whose hash weights stay put (inference): copies the weights into the
 * context's workspace in the order the kernel that hashes ONE vector per head reads them, so that
 * its loads are contiguous (the decode-step hashing of Eq. 5-6 for the queries and the appended
 * key: 28 -> 15 us for 640 vectors of a 128 -> 512 -> 256 network).  Later calls that pass the same
 * three pointers use the copy; the codes are the same bit for bit.  The copy is made on the
 * context's stream, in stream order with the calls around it.  It is a snapshot: after changing the
 * CONTENTS of the arrays (an update in place, or memory freed and handed out again at the same
 * address) call this again, or pass NULL to drop the copy; calls that pass other pointers read
 * their own arrays.  Hidden widths that are not a multiple of 128 have no such
 * kernel: the call succeeds and changes nothing.
 * Errors: INVALID_ARG for a NULL context or missing / misaligned arrays.
 */
int spotlight_prepack_weights(spotlight_ctx *ctx, const spotlight_hash_weights *w);

/*
 * Hash the key rows [t0, t0 + n_new) of every (batch, key-value head) and write their packed
 * codes into the code cache: the append of a decode step (n_new = 1) or the bulk build after
 * prefill.  Eq. 5-6 (Eq. 4 if hidden == 0), then bit-packing: hash output c*W + j of a key lands
 * in word j, bit 31 - c (appendix "Bit-Packing CUDA Kernel").  sign(y) is the bit (y > 0).
 * The codes are those of IEEE binary32 arithmetic with one fused multiply-add chain per output
 * in increasing index order, so they do not depend on launch shape.  (With bfloat16 weights a
 * bulk call evaluates the second layer on the matrix cores and recomputes, with that chain, every
 * output whose sign the matrix-core result does not settle: same bits.
 * SPOTLIGHT_OPT_BULK_HASH_MATRIX_CORES = 0 keeps everything on the chain.)
 *
 *   K      [B, Hkv, Nmax, d]  kv_dtype   read rows t0 .. t0+n_new-1 of every head
 *   codes  [B, Hkv, Nmax, W]  uint32     those rows written, all others untouched
 * Errors: INVALID_ARG for NULL pointers, t0 < 0, n_new < 0 or t0 + n_new > Nmax (n_new = 0 is a
 * no-op); missing b1 / w2 with hidden > 0.
 */
int spotlight_hash_keys(spotlight_ctx *ctx, const void *K, const spotlight_hash_weights *w,
                        int64_t t0, int64_t n_new, uint32_t *codes);

/*
 * Evidence for the bound behind the matrix-core bulk hash.  With SPOTLIGHT_OPT_BULK_HASH_AUDIT on,
 * every bulk spotlight_hash_keys call that takes the matrix-core path adds to four totals kept in
 * the workspace; this call waits for the stream, returns them and clears them (NULL outputs are
 * skipped):
 *   outputs    hash outputs (key x code bit) evaluated on the matrix cores
 *   listed     of those, outputs whose sign the error bound did not settle (recomputed on the chain)
 *   wrong      outputs the bound did settle whose sign differs from the chain's; the method relies
 *              on this being 0
 *   max_ratio  largest |y_matrix - y_chain| / (||W2[j]|| ||h||) seen; the bound assumes it stays
 *              below eps = 1.01 (h (2^-24 + 1.01 2^-22) + 2^-17), returned in *eps
 */
int spotlight_bulk_hash_audit_read(spotlight_ctx *ctx, int64_t *outputs, int64_t *listed, int64_t *wrong,
                                   double *max_ratio, double *eps);

/*
 * Hash the queries (Eq. 5-6), score every cached key code of the head by Hamming distance
 * (Eq. 3: the paper's NXOR/popcount score is L minus this distance) and select, per query head,
 * the k tokens of smallest distance; equal distances are resolved towards the lower token index.
 *
 *   q          [B, Hq, d]         kv_dtype
 *   codes      [B, Hkv, Nmax, W]  uint32   rows 0 .. n_tokens-1 are read
 *   out_idx    [B, Hq, k]         int32    selected token indices in increasing order
 *   out_qcode  [B, Hq, W]         uint32   the query codes, or NULL
 *   out_dist   [B, Hq, n_tokens]  uint16   every distance (debugging / tests), or NULL
 * Errors: INVALID_ARG unless 1 <= n_tokens <= Nmax and 1 <= k <= min(n_tokens, max_topk).
 */
int spotlight_retrieve_topk(spotlight_ctx *ctx, const void *q, const spotlight_hash_weights *w,
                            const uint32_t *codes, int64_t n_tokens, int32_t k,
                            int32_t *out_idx, uint32_t *out_qcode, uint16_t *out_dist);

/*
 * Attention over exactly the rows listed in idx (Eq. 2 gather, then Eq. 1 restricted to the
 * gathered rows; the current token takes part only if its index is listed):
 *   out[b,hq] = sum_i softmax_i(scale * <q[b,hq], K[b,hq/G,idx_i]>) V[b,hq/G,idx_i]
 * with binary32 accumulation.  Entries of idx outside [0, Nmax) are skipped.
 *
 *   q    [B, Hq, d]         kv_dtype
 *   K,V  [B, Hkv, Nmax, d]  kv_dtype
 *   idx  [B, Hq, k]         int32      any order; duplicates count twice
 *   out  [B, Hq, d]         float32
 * Errors: INVALID_ARG unless 1 <= k <= max_topk.
 */
int spotlight_sparse_decode(spotlight_ctx *ctx, const void *q, const void *K, const void *V,
                            const int32_t *idx, int32_t k, float scale, float *out);

/*
 * One decode step of a layer in one call, in the order the method runs it: the key of the token
 * just appended (row n_tokens-1 of K) is hashed into the code cache, the queries are hashed
 * (both in one kernel launch), scored against the n_tokens cached codes and the top-k taken per
 * query head, and attention runs over the selected rows (Eq. 5-6, Eq. 3, Eq. 2, Eq. 1).
 *
 * Forced tokens: the first n_sink and the last n_local tokens of the cache are always selected
 * (the "Sink (4)" and "Local (64)" columns of the paper's perplexity comparison with MagicPIG);
 * the remaining k - |forced| places go to the nearest of the OTHER tokens, ties to the lower
 * index.  n_local >= 1 attends the current token as Eq. 1's concatenation does.  n_sink = n_local
 * = 0 gives exactly spotlight_hash_keys(t0 = n_tokens-1, n_new = 1) + spotlight_retrieve_topk +
 * spotlight_sparse_decode.
 *
 *   q        [B, Hq, d]         kv_dtype
 *   K, V     [B, Hkv, Nmax, d]  kv_dtype   rows 0 .. n_tokens-1 valid, row n_tokens-1 the new token
 *   codes    [B, Hkv, Nmax, W]  uint32     row n_tokens-1 is written, rows 0 .. n_tokens-1 are read
 *   out_idx  [B, Hq, k]         int32      selected token indices in increasing order
 *   out      [B, Hq, d]         float32
 * The call enqueues five kernels on the context's stream (one kernel for a short context under
 * SPOTLIGHT_OPT_STEP_SINGLE_LAUNCH) and nothing else (no allocation, no memset, no copy), so it can
 * be captured into a HIP graph.
 * Errors: INVALID_ARG unless 1 <= n_tokens <= Nmax, 1 <= k <= min(n_tokens, max_topk),
 * n_sink >= 0, n_local >= 0 and the number of forced tokens is at most k.
 */
int spotlight_decode_step(spotlight_ctx *ctx, const void *q, const void *K, const void *V,
                          const spotlight_hash_weights *w, uint32_t *codes, int64_t n_tokens,
                          int32_t k, int32_t n_sink, int32_t n_local, float scale,
                          int32_t *out_idx, float *out);

/*
 * spotlight_decode_step for callers that cannot allocate device memory or create a context: code
 * under HIP graph capture set-up rules, tight serving loops, harnesses that forbid hipMalloc.  It
 * takes the configuration instead of a context and uses, in place of a context's workspace, a
 * fixed buffer of SPOTLIGHT_NOALLOC_SCRATCH_BYTES (32 MiB) of device memory that is part of the
 * library's code object: every GPU the library runs on holds it until the process ends.  The call
 * allocates and frees nothing, on the device or through any library, and does not synchronise;
 * the five kernels are those of spotlight_decode_step and run on cfg->stream of the current device.
 * Arguments, layouts, results and argument errors are those of spotlight_decode_step (cfg->max_topk
 * bounds k as it does for a context); the hash weights are read as stored (no packed copy).
 *
 * Limit: the workspace of the shape (spotlight_workspace_bytes without the room for the packed
 * weights: about 1 KiB per (query head, block of 4096 tokens of max_tokens) x 4 + 516 B per
 * (query head, 32 of max_topk)) must fit the buffer, else SPOTLIGHT_ERR_TOO_LARGE and nothing is
 * launched.  Batch 1, 32 heads, 524288 tokens, top-k 10486 needs 24.4 MB and fits.
 * All calls on one GPU share the one buffer: calls that overlap in time on the same GPU (two
 * streams, two threads) race; calls in stream order are safe, each clears what it needs cleared.
 */
#define SPOTLIGHT_NOALLOC_SCRATCH_BYTES (32u << 20)
int spotlight_decode_step_noalloc(const spotlight_config *cfg, const void *q, const void *K, const void *V,
                                  const spotlight_hash_weights *w, uint32_t *codes, int64_t n_tokens,
                                  int32_t k, int32_t n_sink, int32_t n_local, float scale,
                                  int32_t *out_idx, float *out);

/*
 * Stage timing for benchmarks.  While enabled, every kernel launch carries two HIP events that are
 * stamped when the kernel starts and when it ends.  spotlight_profile_read waits for the stream,
 * adds the elapsed times of the launches recorded since the last read to the per-stage totals and
 * returns the totals for `stage` (milliseconds, number of launches).  Do not capture into a HIP
 * graph while it is enabled.  spotlight_profile_enable(ctx, 0) stops recording
 * and clears the totals.  At most 8192 launches are recorded between two reads; later ones are
 * not timed.
 */
int spotlight_profile_enable(spotlight_ctx *ctx, int on);
int spotlight_profile_read(spotlight_ctx *ctx, int stage, double *total_ms, int64_t *launches);

#ifdef __cplusplus
}
#endif
#endif /* SPOTLIGHT_H */
