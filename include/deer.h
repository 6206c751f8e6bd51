/* deer.h - C ABI of libdeer: DEER's draft-verify step on one AMD MI355X (gfx950).
 *
 * One iteration of the paper's inference loop (Algorithm 1, body of the while):
 *     deer_draft_block        y^_{j+1:j+k} ~ q_theta(. | x_{1:j})        (Sec. 3.2, first display)
 *     deer_verify_block       p_AR(. | x_{1:j+i-1}), i = 1..k, one pass  (Sec. 3.2, Eq. "accept")
 *     deer_accept_and_commit  accept / residual-resample, append, j <- length(x)
 *                                                     (Sec. 3.2 Eq. "accept", "resample"; Alg. 1)
 * preceded once per batch of sequences by deer_init_models, deer_load_tensor (weights) and
 * deer_prefill (build both KV caches for the prefix x_{1:j}; Alg. 1 "Input").
 *
 * Conventions
 *  - Plain C.  No exceptions cross the boundary.  Every call returns a deer_status; on failure
 *    nothing observable has changed except for DEER_EHIP (a HIP call failed mid-way; destroy the
 *    context).  deer_last_error() gives a human-readable string for the last failure.
 *  - "dev" pointers are device (HBM) addresses on the context's device, "host" pointers are
 *    ordinary host memory.  The library NEVER allocates or frees device memory: the caller
 *    allocates the buffers whose sizes deer_query_sizes reports (e.g. as torch tensors), passes
 *    them to deer_init_models, and keeps them alive until deer_destroy.  (Host side, a context
 *    owns a few KB of page-locked memory through which deer_accept_and_commit's results arrive.)
 *  - All device work is enqueued on the hipStream_t given at init.  deer_draft_block and
 *    deer_verify_block return without waiting; deer_accept_and_commit and deer_prefill wait for
 *    the stream before they return (they hand results to the host).
 *  - Call order per batch:  init -> load_tensor* -> prefill -> { draft -> verify -> accept }*.
 *    A call out of order returns DEER_ESTATE.
 *  - Token positions are 0-indexed: committed token x_t (1-indexed in the paper) sits at position
 *    and cache slot t-1.  The target cache holds x_{1:j-1}; x_j is "pending" and is the first row
 *    of the next verify pass, so verify sees exactly k rows [x_j, y^_1 .. y^_{k-1}] and yields
 *    p_1 .. p_k (no bonus token: the largest accepted length is k, as in the paper's Table 4).
 *  - Acceptance stops at the first rejected draft; that position receives the residual sample
 *    (T > 0) or the target's argmax (T = 0) and the rest of the block is discarded.
 */
#ifndef DEER_H
#define DEER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DEER_ABI_VERSION 1u

typedef enum {
    DEER_OK = 0,
    DEER_EINVAL = -1,    /* null pointer, k < 1, k > max_k, T < 0, batch > max_batch, bad shape      */
    DEER_ESTATE = -2,    /* call out of order                                                       */
    DEER_ECAPACITY = -3, /* a sequence would exceed max_seq, or a caller buffer is too small        */
    DEER_EHIP = -4,      /* a HIP runtime call failed; see deer_last_error                          */
    DEER_EVERSION = -5   /* struct_size / abi_version mismatch                                      */
} deer_status;

enum { DEER_TARGET = 0, DEER_DRAFTER = 1 };
enum { DEER_F32 = 0, DEER_BF16 = 1 };

/* Tensor ids for deer_load_tensor.  Every projection is given in [in][out] row-major order
 * (y = x W); the embedding table is [vocab][d_model]. */
enum {
    DEER_T_EMBED = 1, DEER_T_LM_HEAD = 2, DEER_T_WQ = 3, DEER_T_WK = 4, DEER_T_WV = 5, DEER_T_WO = 6,
    DEER_T_WG = 7, DEER_T_WU = 8, DEER_T_WD = 9, DEER_T_ROUTER = 10
};

/* Decoder shape (pre-norm, RMSNorm with unit gains, GQA attention with rotate-half RoPE, SwiGLU
 * FFN, untied LM head, no biases).  n_experts = 0 selects a dense FFN of width d_ff; otherwise
 * a top_k-of-n_experts mixture (softmax over all experts, top_k kept, renormalised) with expert
 * width d_ff_expert. */
typedef struct {
    int32_t n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
    int32_t n_experts, top_k, d_ff_expert;
    float rope_base, rms_eps;
} deer_model_cfg;

typedef struct {
    uint32_t struct_size;   /* sizeof(deer_init_params) */
    uint32_t abi_version;   /* DEER_ABI_VERSION */
    deer_model_cfg target, drafter;
    int32_t max_batch;      /* sequences decoded together                                         */
    int32_t max_seq;        /* cache slots per sequence (prefix + generated + one block)          */
    int32_t max_k;          /* largest block size, 1..32                                          */
    int32_t mask_token_id;  /* the drafter's [MASK] id                                            */
    int32_t eos_token_id;   /* -1: none.  A commit is cut after the first EOS (Alg. 1, break)     */
    int32_t keep_logits;    /* 1: materialise [B][k][vocab] fp32 logits at T = 0 too (parity)     */
    int32_t device;         /* HIP device ordinal                                                 */
    void *hip_stream;       /* hipStream_t, default priority; NULL = the default stream          */
} deer_init_params;

/* Bytes the caller must provide.  All buffers 256-byte aligned. */
typedef struct {
    size_t weights[2];   /* per model: projections in the library's tiled layout + embedding     */
    size_t kv[2];        /* per model: K and V caches, bf16, max_batch * max_seq slots           */
    size_t workspace;    /* activations, split-K partials, logits, per-sequence state            */
    size_t staging;      /* scratch that deer_load_tensor needs beyond the source tensor: 0      */
} deer_sizes;

typedef struct {
    void *weights[2];    /* dev */
    void *kv[2];         /* dev */
    void *workspace;     /* dev */
} deer_buffers;

typedef struct deer_ctx deer_ctx;

/* Host-only: fills *out from *p.  DEER_EINVAL on unsupported shapes (head_dim not in
 * {32,64,128}, widths not multiples of the 128-column tile, max_k > 32, ...). */
int deer_query_sizes(const deer_init_params *p, deer_sizes *out);

/* Creates a context over caller-owned device buffers (each at least as large as
 * deer_query_sizes reported; sizes are passed for checking).  *out is NULL on failure. */
int deer_init_models(const deer_init_params *p, const deer_buffers *bufs, const deer_sizes *buf_sizes,
                     deer_ctx **out);

/* Copies one canonical tensor (device pointer `src_dev`, dtype DEER_F32 or DEER_BF16, `rows` x
 * `cols` row-major) into the library's layout, converting to bf16 (round to nearest even).
 * layer = -1 for embedding / LM head; expert = -1 unless the model is a mixture and the tensor is
 * WG/WU/WD.  Enqueued on the stream; `src_dev` may be reused after the stream has passed it. */
int deer_load_tensor(deer_ctx *c, int model, int tensor_id, int layer, int expert,
                     const void *src_dev, int src_dtype, int64_t rows, int64_t cols);

/* Prefix x_{1:j} for `batch` sequences (Alg. 1, Input).  prompt_ids_host: concatenated ids;
 * prompt_lens_host[b] >= 1.  Builds the target cache for x_{1:j-1} and the drafter cache for
 * x_{1:j} with causal attention, in passes of up to 4096 rows (512 for mixture models) that hold the rows
 * of as many sequences as fit (each pass streams the weights once).  Waits for completion. */
int deer_prefill(deer_ctx *c, int32_t batch, const int32_t *prompt_ids_host, const int32_t *prompt_lens_host);

/* Sets the state as if `lens_host[b]` tokens had been prefilled, WITHOUT running the models:
 * the caller has written cache contents itself (deer_debug_load_kv) - used where a real prefill
 * is too costly (32k-token prefixes).  last_token_host[b] = x_j, the pending token.  The drafter
 * cache is taken to hold all lens_host[b] tokens. */
int deer_set_prefilled(deer_ctx *c, int32_t batch, const int32_t *lens_host, const int32_t *last_token_host);

/* Drafter pass (Sec. 3.2: one pass proposes the whole block; position i's law does not depend
 * on the other drafted tokens).  Rows per sequence: the committed tokens the drafter has not
 * cached yet (causal, appended to its cache) followed by k MASK rows at positions j..j+k-1 that
 * see the whole cache and each other.  T = 0: y^_i = argmax (lowest index on ties); T > 0:
 * y^_i ~ softmax(z_i / T) by Gumbel-max with the counter generator keyed by (seed, sequence,
 * position).  Writes draft tokens to draft_tokens_dev[batch][k] (int32). */
int deer_draft_block(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t *draft_tokens_dev);

/* Multi-pass draft (block regeneration, Sec. "Generative Capabilities": the drafter fills in a partially
 * masked block), an extension beside Alg. 1: n_passes drafter passes, 1 <= n_passes <= k.  Pass s sees the
 * tokens fixed so far at the first ceil(k (s-1) / n_passes) block positions and MASK at the others, and
 * fixes the positions up to ceil(k s / n_passes) (left to right, so the law a token is drawn from depends
 * on the prefix and on EARLIER drafts only, which keeps the acceptance rule exact).  The logits and
 * log-normalisers kept for deer_accept_and_commit are, per position, those of the pass that fixed it.
 * n_passes = 1 is deer_draft_block.  Same state rules, errors and output as deer_draft_block. */
int deer_draft_block_multipass(deer_ctx *c, int32_t k, float T, uint64_t seed, int32_t n_passes,
                               int32_t *draft_tokens_dev);

/* Target pass over rows [x_j, y^_1 .. y^_{k-1}] (block-causal over the cache), reading the
 * drafts from draft_tokens_dev[batch][k] - normally the buffer deer_draft_block filled; tests
 * may inject blocks.  Leaves per-row argmax / log-normaliser (and logits at T > 0) on device. */
int deer_verify_block(deer_ctx *c, int32_t k, float T, const int32_t *draft_tokens_dev);

/* Acceptance (Sec. 3.2 Eq. "accept"/"resample"; Alg. 1 inner loop, stopped at the first
 * rejection) and commit: appends the accepted drafts and the correction, cuts at EOS, rolls the
 * target cache back to (new length - 1).  Host outputs, per sequence b:
 *   accept_len[b] in [0,k];  n_committed[b] = min(accept_len+1, k) (less after EOS);
 *   committed[b*k .. b*k+n_committed[b]).   Waits for the stream. */
int deer_accept_and_commit(deer_ctx *c, int32_t k, float T, uint64_t seed,
                           int32_t *accept_len_host, int32_t *committed_host, int32_t *n_committed_host);

/* deer_accept_and_commit for callers that must not allocate device memory or have the library use scratch
 * of the caller's sizing (code under HIP graph capture around it, tight serving loops, harnesses that forbid
 * hipMalloc).  Same arguments, results, state rules and errors as deer_accept_and_commit; the sampling
 * kernel's scratch (per-share candidates and arrival counters) lives in a static device array inside the
 * library (65.8 KB per GPU, held until the process ends) instead of the workspace, and the call makes no
 * hipMalloc / hipFree and no host allocation.  Limit: at most 64 sequences in the batch (DEER_ECAPACITY
 * beyond).  All contexts on one GPU share that array: calls that overlap on one GPU (two contexts on
 * different streams) race; calls one after the other are fine (the counters are cleared at the start of
 * every call).  Waits for the stream. */
int deer_accept_and_commit_static(deer_ctx *c, int32_t k, float T, uint64_t seed,
                                  int32_t *accept_len_host, int32_t *committed_host, int32_t *n_committed_host);

/* Bonus token (an extension beside Alg. 1, off by default; Appendix, Theorem: its induction step is a
 * draw from p_AR given an exactly distributed prefix, which holds for one more position).  When enabled,
 * deer_verify_block feeds k + 1 rows [x_j, y^_1 .. y^_k] (draft_tokens_dev is read in full) and
 * deer_accept_and_commit, after k accepted drafts, commits a (k+1)-th token: the argmax of p_{k+1} at
 * T = 0, else a draw from p_{k+1} made with the residual stream of the counter generator at position
 * j + k (a residual with no draft to subtract).  Then n_committed[b] <= k + 1 and committed_host holds
 * batch * (k + 1) entries with stride k + 1.  The rows of a sequence stay within one 32-row tile, so
 * calls need k <= 31 while the bonus token is on (DEER_EINVAL otherwise).  Not allowed between
 * deer_draft_block and deer_accept_and_commit (DEER_ESTATE). */
int deer_set_bonus_token(deer_ctx *c, int enable);

int deer_destroy(deer_ctx *c);
const char *deer_last_error(const deer_ctx *c); /* c may be NULL: last init-time error */

/* ---- inspection surface used by tests and the benchmark (not part of the timed path) -------- */

/* Copies the last pass's logits [batch][k][vocab] (fp32) of `model` to host; needs keep_logits
 * or T > 0 in that pass.  Waits for the stream. */
int deer_debug_get_logits(deer_ctx *c, int model, float *logits_host, size_t n_floats);

/* Launch timing for the benchmark.  While enabled, the launches of the weight-streaming GEMM
 * (kernel_class 0) and of the block-attention kernel (kernel_class 1) are bracketed by HIP events
 * on the context's stream; launches of one class that follow each other directly share one pair of
 * events (an event between two of them costs more than the gap it would measure), so the summed time
 * includes the gaps inside such a run.  deer_debug_profile(c, on) waits for the stream, switches recording and forgets earlier
 * records; deer_debug_profile_read waits for the stream and returns, for one class, the summed event
 * time (ms), the number of launches, and their algorithmic bytes (weight bytes of each GEMM; K and V
 * rows visible to each attention launch). */
int deer_debug_profile(deer_ctx *c, int enable);
int deer_debug_profile_read(deer_ctx *c, int kernel_class, double *total_ms, int64_t *launches, double *bytes);

/* Lock-step aid for parity tests: stands in for deer_accept_and_commit after deer_verify_block and
 * commits, per sequence b, the n_host[b] tokens tokens_host[b * stride ..] (0 <= n_host[b] <= k, or
 * k + 1 with the bonus token; stride <= 32) instead of the acceptance rule's choice.  The caller keeps
 * the cache consistent: all but the last of a sequence's tokens must be the drafts that the verify
 * pass was given at those positions (their K,V rows are already cached), as is the case for the commit
 * of an oracle that judged the same block.  Waits for the stream. */
int deer_debug_force_commit(deer_ctx *c, const int32_t *tokens_host, const int32_t *n_host, int32_t stride);

/* Injected cache contents (where running a real prefill is too costly): writes canonical rows
 * k_rows_dev, v_rows_dev ([n_slots][n_kv_heads][head_dim] bf16, device memory) into cache slots
 * first_slot .. first_slot + n_slots - 1 of sequence `seq`, layer `layer` of `model`, in the
 * library's cache layout.  Enqueued on the stream; follow with deer_set_prefilled. */
int deer_debug_load_kv(deer_ctx *c, int model, int32_t layer, int32_t seq, int32_t first_slot, int32_t n_slots,
                       const void *k_rows_dev, const void *v_rows_dev);

/* Benchmarking aid for random-init mixture models, whose router sends every row of a block to the same few
 * experts: when enabled, each row is routed to top_k distinct pseudo-random experts (a function of layer and
 * row) with equal weights instead of the router's own choice, so that a block touches as many experts as a
 * trained router's would (n_experts must be a power of two, else ignored).  Changes the computed function:
 * never on in parity tests. */
int deer_debug_route_spread(deer_ctx *c, int enable);

/* Mixture models: the number of (layer, expert) pairs whose expert weights the passes since the last call
 * had to stream (an expert counts once per layer and pass if any row was routed to it), then resets the
 * count - the data-dependent part of a pass's algorithmic bytes.  0 for dense models.  Waits for the stream. */
int deer_debug_experts_streamed(deer_ctx *c, int64_t *pairs);

/* Measurement aid: the rate at which a plain kernel reads a buffer, i.e. what "streaming at memory speed" means for
 * that size on this chip (buffers up to the 32 MB of L2 or the 256 MB memory-side cache are served from there when
 * read again).  Reads `bytes` (a multiple of 16) of caller-owned device memory at buf_dev (16-byte aligned) with
 * `workgroups` workgroups of 512 threads, plain or non-temporal loads, 3 untimed launches and then `reps` timed ones
 * back to back on the context's stream (launch gaps included); *ms_per_read = mean time of one launch.  Must not
 * run while launch timing (deer_debug_profile) is on.  Waits for the stream. */
int deer_debug_stream_read(deer_ctx *c, const void *buf_dev, size_t bytes, int32_t workgroups, int32_t nontemporal,
                           int32_t reps, float *ms_per_read);

/* Debugging aid: where a weight-streaming GEMM launch spends its time.  Copies the stamps recorded so far
 * (2 x 2048 workgroup rows x 8 ticks of the 100 MHz device clock: the first 2048 rows belong to the chosen launch,
 * the second 2048 to the streaming GEMM launched after it, so that the hand-over between two kernels can be seen;
 * per row: 0 workgroup started, 1 its first wave has multiplied its K slice, 2 its tile is stored (after the
 * epilogue if the matrix is not split), 3 it has arrived at the column group's counter, 4 it was the last to arrive
 * and has finished the group; 0 = not reached or no such workgroup) into stamps_host (at most max_blocks rows; *blocks = rows available, 0 if nothing was recorded), then
 * selects the launch that records from now on: the `launch`-th streaming GEMM (counted from 0) of every following
 * pass of `model`; launch < 0 switches recording off.  Waits for the stream. */
int deer_debug_gemm_stamps(deer_ctx *c, int model, int launch, uint64_t *stamps_host, int32_t max_blocks, int32_t *blocks);

/* GEMMs of passes with at least 256 rows run blocked for the matrix cores (256 x 256 tiles through LDS)
 * where a launch has at least `min_tiles` such tiles (default 128: enough to fill the chip), else as the
 * weight-streaming kernel.  0 switches the blocked kernel off; tests lower the threshold to cover it at
 * small sizes.  Results agree within rounding (different summation order over K). */
int deer_debug_gemm_tiled(deer_ctx *c, int min_tiles);

/* Current committed length j per sequence (host mirror). */
int deer_get_lengths(const deer_ctx *c, int32_t *len_host);

/* Where the caches live inside the model's kv buffer (bf16; offsets in elements from its start):
 *   K at k_base + layer * layer_stride + seq * seq_stride + kv_head * head_stride, V at v_base + the same.
 * Inside a (layer, sequence, kv head) region the slots (slot < max_seq, a multiple of 64) are stored in blocks of
 * 32, and a block in the order the attention kernels' matrix instructions read it: head_dim / 16 fragments of
 * 64 lanes x 8 elements (1 KB each).
 *   K block, fragment s: lane (r, half) = half * 32 + r holds elements 16 s + 8 half .. + 7 of slot
 *   32 * block + key(r), key(r) = 16 * ((r >> 2) & 1) + 4 * (r >> 3) + (r & 3).
 *   V block, fragment 2 tt + s2: lane half * 32 + c holds slots 32 * block + 16 half + 8 s2 .. + 7 of channel
 *   32 tt + c (V is stored transposed).
 * A caller that wants to fill cache rows should not write this layout itself: deer_debug_load_kv takes canonical
 * [slot][kv_head][head_dim] rows. */
typedef struct {
    size_t k_base, v_base;            /* element offsets of K and Vt blocks                        */
    size_t layer_stride, seq_stride, head_stride; /* same for both                                 */
    int32_t max_seq, head_dim;
} deer_kv_layout;
int deer_get_kv_layout(const deer_ctx *c, int model, deer_kv_layout *out);

#ifdef __cplusplus
}
#endif
#endif /* DEER_H */
