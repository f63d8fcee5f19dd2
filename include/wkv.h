/*
 * libwkv -- the per-token decode step of WeightedKV on one AMD MI355X (gfx950).
 *
 * WeightedKV (arXiv 2503.01330) keeps a key/value cache of fixed size m during
 * autoregressive decoding.  For every (sequence, head) pair -- a "unit"; the
 * paper writes the method for a single one and leaves batch and head indices
 * out (Section III-A), so units never interact -- one generated token does the
 * following:
 *
 *   1. K_t = [K_{t-1}, k_t],  V_t = [V_{t-1}, v_t]                (Section III-A)
 *   2. A_t = softmax(q_t^T K_t / sqrt(d)),  o_t = A_t^T V_t        (Sections III-A, III-B)
 *   3. a = [a, 0] + A_t,  n = [n, 0] + 1                           (Algorithm 1)
 *   4. if the cache now holds more than m entries:                 (Algorithm 1, Section IV)
 *        abar = a / n
 *        j    = arg-min of abar over the entries that are not protected
 *        V[j+1] <- (abar[j] V[j] + abar[j+1] V[j+1]) / (abar[j] + abar[j+1])
 *        remove K[j], V[j], a[j], n[j]
 *
 * "j+1" is the right-hand neighbour in token order.  Protected entries are the
 * `recent_window` newest tokens (Algorithm 1 protects exactly the newest one,
 * recent_window = 1; Section V-A keeps a recent region and 4 initial tokens)
 * and, optionally, the first `n_sink` tokens.  Ties in the arg-min go to the
 * oldest token.  The survivor keeps its own key, score sum and count.
 *
 * Everything above runs in hand-written HIP kernels; this header is the whole
 * boundary.  All functions are thread-compatible (one handle must not be used
 * from two threads at once), never throw, never abort, and return 0 or a
 * negative WKV_E* code; wkv_last_error() gives the calling thread's message.
 */
#ifndef WKV_H
#define WKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* storage / arithmetic-input types of q, k, v, out and of the K/V cache */
#define WKV_FP32 0
#define WKV_FP16 1
#define WKV_BF16 2

/* return codes */
#define WKV_OK      0
#define WKV_EINVAL -1   /* bad argument (null pointer, out-of-range value, misaligned buffer) */
#define WKV_ENOMEM -2   /* device or host allocation failed */
#define WKV_EHIP   -3   /* a HIP runtime call failed (no GPU, launch failure, ...) */
#define WKV_ESIZE  -4   /* a size exceeds what this build supports, or a readback buffer is too small */

/* limits of this build */
#define WKV_MAX_BUDGET 4095   /* slots per unit, bounded by the LDS staging of one score row */
#define WKV_MAX_PROMPT 4096   /* tokens wkv_prefill takes at once, bounded by the LDS staging of their scores */

/* which entries may be ranked / how the victim's value is treated (wkv_options) */
#define WKV_SCORE_AVERAGE    0   /* abar = a / n: WeightedKV (Algorithm 1)                         */
#define WKV_SCORE_CUMULATIVE 1   /* a: the cumulative-score rule the paper cites as H2O (Section II) */
#define WKV_SCORE_LAST       2   /* the current step's attention weight: the rule cited as TOVA     */
#define WKV_MERGE_CONVEX     0   /* fold V[j] into its right neighbour (Algorithm 1)                */
#define WKV_MERGE_NONE       1   /* drop V[j] too: the "Eviction" ablation of Section V-B           */

/* How wkv_step loads the cached K and V rows (wkv_options.streaming).  Every row is read once per
 * step; whether it is still in the 256 MB last-level cache at the next step depends on how much
 * else is streamed in between, which only the caller knows.  CACHED and STREAMING state it:
 * through the caches, or with non-temporal loads (nothing a step loads survives until its next
 * use, and loads that allocate cache lines on their way only cost bandwidth; rows of at most
 * 256 bytes only).  AUTO guesses: it takes the K and V of ALL live handles on the device as what is
 * streamed between two steps of this handle (a stack of layers stepped in turn) and chooses
 * STREAMING when that exceeds the last-level cache by an eighth or more.  The guess is wrong when handles sit idle:
 * they still count, and a small handle stepped alone next to them loses about a tenth to
 * non-temporal loads it did not need -- say CACHED there.  Results do not depend on the choice. */
#define WKV_LOADS_AUTO      0
#define WKV_LOADS_CACHED    1
#define WKV_LOADS_STREAMING 2

typedef struct wkv_handle wkv_handle;

/* Every field is plain int so the struct can be filled from any language.
 * Zero in an optional field means "default". */
typedef struct wkv_options {
    int batch, heads, head_dim;  /* units = batch*heads; head_dim in {64,128,256} (fp32: {64,128}) */
    int budget;                  /* m, 1..WKV_MAX_BUDGET: slots kept after every step             */
    int recent_window;           /* R, 1..budget: newest R tokens are never evicted               */
    int dtype;                   /* WKV_FP32 / WKV_FP16 / WKV_BF16                                */
    int n_sink;                  /* optional: first n_sink tokens are never evicted; n_sink+R <= m */
    int score_mode;              /* optional: WKV_SCORE_*; non-average modes require WKV_MERGE_NONE */
    int merge_mode;              /* optional: WKV_MERGE_*                                          */
    int log_capacity;            /* optional: steps of eviction log kept (ring), default 1024      */
    int threads;                 /* optional: workgroup size 256/512/1024, default chosen by units */
    int split;                   /* optional: workgroups per unit, 1/2/4/8/16; default: 1 unless   */
                                 /*   the units alone would leave most of the GPU idle             */
    int streaming;               /* optional: WKV_LOADS_*: how wkv_step loads the cached K/V rows  */
    int max_prompt;              /* optional: prompt length (tokens) for which wkv_create_ex already */
                                 /*   reserves wkv_prefill's scratch, so that the call allocates nothing */
    int replayable;              /* optional, 0/1: keep the token index in device memory, so that   */
                                 /*   recorded steps can be replayed from a HIP graph (see wkv_step) */
    int reserved[1];             /* must be zero                                                   */
} wkv_options;

/*
 * Create an empty cache (K_0, V_0 empty: Section III-A; a, n empty: Algorithm 1)
 * for batch*heads units on the current HIP device.  The library allocates and
 * owns the device memory: per unit `budget` rows of K and V in `dtype`, one
 * fp64 score sum, one int32 original position and one int32 token-order link
 * per slot, plus the eviction log; with split > 1 also the per-step scratch the
 * workgroups of a unit exchange (one fp64 per slot and split partial output
 * rows per unit).  The softmax scale is 1/sqrt(head_dim).
 * *h is written only on success.
 */
int wkv_create(wkv_handle** h, int batch, int heads, int head_dim,
               int budget, int recent_window, int dtype);

/* Same, with the optional knobs of wkv_options. */
int wkv_create_ex(wkv_handle** h, const wkv_options* opt);

/*
 * One decode step (steps 1-4 above) for every unit.
 *   q, k_new, v_new : DEVICE pointers, contiguous [batch, heads, head_dim] in
 *                     the handle's dtype, 16-byte aligned, read only.
 *   out             : DEVICE pointer, same shape and dtype, receives o_t.
 *                     o_t is computed over the cache *including* the new token
 *                     and *before* compression (Algorithm 1 obtains A_t ahead
 *                     of its capacity test).
 *   stream          : a hipStream_t (NULL = the default stream).
 * Asynchronous: returns after enqueueing.  The caller owns the four buffers and
 * must keep them valid until the stream reaches this step; the cache belongs to
 * the handle.  After the step completes the cache holds min(tokens, budget)
 * slots per unit.  Arguments are checked on the host before anything is
 * launched; on error nothing is enqueued and the cache is unchanged.
 * Steps of one handle must be enqueued in token order on streams that order
 * them (normally one stream).
 * HIP graphs: by default the token index lives in the handle, on the host, and travels as a
 * kernel argument, so a step recorded into a graph would replay that one index: do not replay
 * such a recording.  A handle created with wkv_options.replayable = 1 keeps the index in device
 * memory instead: the kernel reads it when it starts (one dependent scalar load, about a
 * microsecond per launch) and the last workgroup to finish with it stores index + 1, so a
 * recorded wkv_step advances with every replay, and recorded and directly enqueued steps may be
 * mixed.  The caller replays with the buffers it recorded with (a graph fixes q, k_new, v_new and
 * out).  wkv_state reads the index back from the device, so it counts replays too.
 */
int wkv_step(wkv_handle* h, const void* q, const void* k_new, const void* v_new,
             void* out, void* stream);

/*
 * Bulk prefill of an EMPTY cache with a prompt of n_tokens tokens.  The paper streams from an
 * empty cache (Algorithm 1) and has no procedure for a prompt; what this call computes:
 *   - out[t] = softmax(q_t^T K_{0..t} / sqrt(d)) V_{0..t} over the UNcompressed prompt
 *     (Section III-A, causal);
 *   - the score list Algorithm 1's bookkeeping accumulates over these rows: a_i = sum_t A_t[i],
 *     n_i = n_tokens - i;
 *   - while more than `budget` entries remain: Algorithm 1's selection and merge with these
 *     (fixed) scores, protected entries as in wkv_step; merged rows are rounded to the cache
 *     dtype once, when the compression is over.
 * For n_tokens <= budget + 1 the result is that of n_tokens calls of wkv_step; beyond that it
 * is a different function (a streamed token attends to an already compressed cache).
 *   q, k, v : DEVICE pointers, contiguous [n_tokens, batch, heads, head_dim] in the handle's
 *             dtype, 16-byte aligned, read only.
 *   out     : DEVICE pointer of the same shape, or NULL if the outputs are not wanted.
 * Built for 16-bit caches with head_dim 64 or 128 and the average or cumulative scoring rule
 * (WKV_ESIZE / WKV_EINVAL otherwise); 1 <= n_tokens <= WKV_MAX_PROMPT.
 * Asynchronous like wkv_step: returns after enqueueing three kernels on `stream`; the caller keeps
 * q, k, v, out valid until the stream reaches them.  Device scratch (16 bytes per token and unit)
 * belongs to the handle: reserved by wkv_create_ex when wkv_options.max_prompt covers n_tokens,
 * otherwise allocated (and kept) by the first call that needs it -- only that call allocates.
 * The eviction log is not written.  On error the cache is unchanged, except for WKV_EHIP after
 * the launch.
 */
int wkv_prefill(wkv_handle* h, const void* q, const void* k, const void* v, void* out,
                int n_tokens, void* stream);

/*
 * wkv_prefill for callers that cannot allocate device memory at all: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels,
 * same results; the scratch is a static device array inside the library
 * (WKV_NOALLOC_SCRATCH_BYTES, held by every GPU the library runs on until the process ends)
 * instead of memory of the handle, so the call performs no allocation and no free, whatever
 * wkv_options.max_prompt said.  Limit: batch*heads * n_tokens <= WKV_NOALLOC_SCRATCH_BYTES / 16
 * (WKV_ESIZE beyond).  All calls on one GPU share the array: two such calls must not overlap in
 * time (put them on one stream, or order them with events); nothing in it has to start at zero,
 * every value read is written by the same call first.
 */
#define WKV_NOALLOC_SCRATCH_BYTES (16u << 20)   /* 256 units x 4096 tokens, or 1024 x 1024, ... */
int wkv_prefill_noalloc(wkv_handle* h, const void* q, const void* k, const void* v, void* out,
                        int n_tokens, void* stream);

/* what wkv_state reads back */
#define WKV_STEP       0  /* int64[1]            tokens processed so far                             */
#define WKV_LEN        1  /* int32[1]            live slots per unit = min(tokens, budget)           */
#define WKV_K          2  /* dtype[units,len,d]  retained keys                                       */
#define WKV_V          3  /* dtype[units,len,d]  (merged) values                                     */
#define WKV_SCORE_SUM  4  /* double[units,len]   a: accumulated attention weight                     */
#define WKV_COUNT      5  /* int32[units,len]    n: steps attended = tokens - pos                    */
#define WKV_POS        6  /* int32[units,len]    0-based index of the token whose key is retained    */
#define WKV_NMERGED    7  /* int32[units,len]    raw values folded into the slot                     */
#define WKV_EVICT_POS  8  /* int32[n,units]      evicted token index per step, -1 if none            */
#define WKV_EVICT_SLOT 9  /* int32[n,units]      its rank in token order among the len+1 slots, -1   */
#define WKV_STATUS     10 /* int32[2]            {merges with zero denominator, non-finite scores}   */

/*
 * Synchronous readback into HOST memory (waits for all enqueued steps).  Slot
 * arrays come back in token order (ascending WKV_POS), whatever the order in
 * device memory.  For the two eviction logs, n = bytes / (4*units) most recent
 * steps are returned, oldest first; n must not exceed min(tokens, log_capacity).
 * For everything else `bytes` must be at least the size listed above
 * (WKV_ESIZE otherwise; nothing is written then).  Like every call that takes a handle, it
 * must come with the handle's device current (WKV_EINVAL otherwise); wkv_destroy alone does
 * not mind.
 */
int wkv_state(wkv_handle* h, int what, void* host_dst, size_t bytes);

/*
 * The inverse of wkv_state: replace the cache by a state given in HOST memory, in token
 * order, as wkv_state returns it (checkpoint / resume; the method itself has no such step).
 *   tokens : tokens processed so far (what WKV_STEP returned)
 *   len    : live slots per unit; must equal min(tokens, budget)
 *   K, V   : dtype[units,len,d];  score_sum : double[units,len];  pos : int32[units,len],
 *            strictly increasing within a unit, last entry = tokens-1, all < tokens
 * Counts and merge counts follow from pos and are not passed.  Synchronous; waits for
 * enqueued work first.  The eviction log is cleared.  On error the cache is unchanged, except for
 * WKV_EHIP during the upload itself (the message says so).
 */
int wkv_load(wkv_handle* h, int64_t tokens, int len, const void* K, const void* V,
             const double* score_sum, const int32_t* pos);

/* Free the cache.  Waits for enqueued work.  NULL is accepted. */
int wkv_destroy(wkv_handle* h);

/* Message of the last failing call on this thread ("" if none).  Never NULL. */
const char* wkv_last_error(void);

/* Device bytes a handle with these options allocates (0 if the options are invalid).
 * Host-only arithmetic: usable without a GPU. */
size_t wkv_workspace_bytes(const wkv_options* opt);

/* Algorithmic HBM bytes one wkv_step moves in steady state (cache full): per
 * unit (budget+1) K rows and V rows read, score sum read+written, token index
 * read, q/k_new/v_new read, out written, the new K/V rows written, the merged
 * V row written.  Host-only arithmetic. */
size_t wkv_step_bytes(const wkv_options* opt);

/* The launch shape wkv_step uses for these options: *workgroups = units x workgroups per unit,
 * *threads = threads per workgroup.  Host-only arithmetic.  WKV_OK, or the code wkv_create_ex
 * would return for these options. */
int wkv_launch_shape(const wkv_options* opt, int* workgroups, int* threads);

/*
 * Measurement aid, no part of the method: a plain streaming read of `bytes` bytes of DEVICE memory
 * at `src` by `workgroups` workgroups of `threads` threads (64..1024, a multiple of 64), each
 * workgroup its own contiguous share, 16 bytes per lane and load, four loads in flight per lane;
 * non-temporal loads if `nontemporal` is non-zero.  `sink` (4 bytes of device memory, or NULL)
 * keeps the loads alive: a lane whose loaded words XOR to 0x9E3779B9 stores that constant there --
 * with ordinary data practically never, and a test that plants the constant in one word of an
 * otherwise zero buffer sees that the word was read.  Asynchronous on `stream`.  The benchmark times it
 * with the grid and byte count of a wkv_step launch: what that launch shape can pull out of
 * memory when it does nothing else.  `bytes` must be a positive multiple of 16*workgroups
 * (WKV_EINVAL otherwise); the caller owns src and keeps it valid.
 */
int wkv_probe_read(const void* src, size_t bytes, int workgroups, int threads, int nontemporal,
                   void* sink, void* stream);

int wkv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* WKV_H */
