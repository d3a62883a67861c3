/*
 * mpa — mixed-batch paged attention for AMD MI355X (gfx950).  C ABI of libmpa.so.
 *
 * The library implements the attention step of one serving iteration over a block-based KV
 * cache for a batch that mixes prompt-chunk tasks and single-token generation tasks, plus the
 * append of the iteration's new K/V into the cache:
 *
 *   - attention is scaled dot-product self-attention per head, softmax(Q K^T / sqrt(d_k)) V
 *     (paper Sec. 2.1, the self-attention equation), each query token attending to the keys of
 *     all earlier tokens of its sequence and to itself;
 *   - K/V are stored in fixed-size token blocks that need not be contiguous (Sec. 2.2,
 *     block-based KVC allocation);
 *   - a prompt may be processed in chunks over successive iterations, each chunk batched with
 *     other prompts' chunks and with generation tasks (Sec. 2.3; Sec. 4.2 dynamic chunking), and
 *     a chunk may start and end anywhere, also in the middle of a block (Sec. 4.4, KVC demand of
 *     a non-first chunk).
 *
 * Conventions
 *   - Every function returns an int status (MPA_OK == 0, errors < 0) unless stated; nothing
 *     throws or aborts (a host allocation that fails inside a call is reported as
 *     MPA_ERR_NO_MEMORY, by any function that plans a batch).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *     host memory read during the call only.  The library allocates no device memory.
 *   - Work is enqueued on the HIP stream passed as `stream` (a hipStream_t cast to void*,
 *     NULL = the default stream) and the call returns without waiting for the GPU.
 *   - The attention calls plan on the host from the two host arrays and hand the plan to the GPU
 *     through a ring of pinned host buffers owned by the context: they are asynchronous, but not
 *     meant for capture into a HIP graph (a replay would re-read a buffer that later calls reuse);
 *     mpa_mixed_paged_attention_static is the form that can be captured.
 *   - Elements are 16-bit (bf16 or fp16, fixed per context; passed as bit patterns); scores,
 *     softmax sums and outputs accumulate in fp32.
 *
 * Tensor layouts (row-major, innermost last)
 *   q, out               : [T, H, D]        T = number of query rows in the batch
 *   k_new, v_new         : [T, HK, D]       HK = num_kv_heads
 *   k_cache, v_cache     : [NB, HK, bs, D]  NB blocks of bs tokens; one (block, kv head) tile is
 *                                           bs*D contiguous elements
 *   block_table          : [S, stride] int32, entry j of row i = physical block of tokens
 *                          j*bs .. j*bs+bs-1 of sequence i; entries past ceil(ctx_i/bs) are
 *                          never read (pad with -1)
 */
#ifndef MPA_H
#define MPA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mpa_ctx mpa_ctx; /* opaque, host-side */

/* Version of this interface: raised whenever a declaration, an option or a status of this header or
 * of mpa_sched.h changes meaning.  mpa_abi_version() returns the value the library was built with:
 * a caller compiled against another header (or a binding written for one) can tell. */
#define MPA_ABI_VERSION 3
int mpa_abi_version(void);

enum {
    MPA_OK = 0,
    MPA_ERR_INVALID_ARG = -1, /* null pointer, negative size, misaligned pointer           */
    MPA_ERR_UNSUPPORTED = -2, /* head_dim / block_size / dtype / head layout not built      */
    MPA_ERR_WORKSPACE = -3,   /* workspace missing or smaller than the batch needs          */
    MPA_ERR_BAD_BATCH = -4,   /* chunk_starts / context_lens describe no valid batch        */
    MPA_ERR_HIP = -5,         /* a HIP runtime call failed; see mpa_last_hip_error          */
    MPA_ERR_NO_MEMORY = -6    /* the host ran out of memory inside the call (work lists and
                                 scheduler state live in ordinary host memory); the object stays
                                 usable, a cached plan is dropped                            */
};

enum {
    MPA_BF16 = 1, /* bfloat16: the upper 16 bits of an IEEE single                              */
    MPA_FP16 = 2  /* IEEE half, the precision of the paper's experiments (Sec. 6.1)             */
};

typedef struct {
    int32_t num_heads;    /* H, query heads                                                   */
    int32_t num_kv_heads; /* HK, K/V heads; divides H.  Query head h reads K/V head h / (H/HK)
                             (grouped-query attention); HK == H is multi-head attention       */
    int32_t head_dim;     /* D: 64 or 128                                                     */
    int32_t block_size;   /* bs, tokens per KV block: 16, 32, 64 or 128                       */
    int32_t dtype;        /* MPA_BF16 or MPA_FP16: element type of q, k/v, the caches and out   */
} mpa_config;

/* Tuning / testing knobs for mpa_set_option. */
enum {
    MPA_OPT_TG_SPLIT_BLOCKS = 1, /* KV blocks per generation-row work item; 0 = automatic     */
    MPA_OPT_PP_SPLIT_TOKENS = 2, /* keys per prompt-tile work item (multiple of 64); 0 = auto */
    MPA_OPT_PP_ROWSTREAM = 3,    /* 1 = run prompt rows through the row-streaming body
                                    (slow; cross-check of the matrix-core body)               */
    MPA_OPT_PP_RESIDENT_WGS = 4, /* work-groups that share the prompt-tile work (each takes
                                    every n-th unit); 0 = automatic                           */
    MPA_OPT_PP_TEAM_MIN_STEPS = 5, /* > 0: the query tiles over one key range of at least this
                                    many 64-key steps keep pace with each other (bounded
                                    pauses of those ahead); 0 (default) = no pacing: such
                                    tiles are launched next to each other and stay together */
    MPA_OPT_PROFILE_EVERY = 7,   /* with mpa_profile_enable: time every k-th attention call only
                                    (default 1); a pair of timing events costs the queue about
                                    ten microseconds per call                                 */
    MPA_OPT_PROFILE_REPEAT = 11, /* with mpa_profile_enable: a timed call launches the attention
                                    kernel this many times back to back between its two events
                                    (default 1) and mpa_profile_read reports the time per launch:
                                    for timing launches of a few tens of microseconds, against
                                    which a pair of events weighs 10-20 %.  The launches are
                                    identical (same inputs, same outputs); set it before
                                    profiling and leave it unchanged until the series is read  */
    MPA_OPT_TILE_MODE = 10,      /* work-group shape of the attention launch: 0 or 1 (default) = four
                                    wavefronts, 128-row prompt tiles, two work-groups per compute
                                    unit; 2 = eight wavefronts, 256-row prompt tiles over a ring of
                                    five K/V tiles, one work-group per compute unit (prompt tiles and
                                    generation rows then run on separate compute units).  Same
                                    results; measured within 2 % of the default on prompts alone and
                                    slower on mixed batches, so it is never chosen automatically   */
    MPA_OPT_STAGING_TIMEOUT_MS = 8, /* how long a call waits for the upload kernel that last used a
                                    staging buffer to report that it has read it (default 5000;
                                    normally it has, long before the ring of buffers comes round).
                                    After that the call fails with MPA_ERR_HIP (hipErrorNotReady)
                                    before it writes to the buffer or launches anything          */
    MPA_OPT_TEST_STUCK_UPLOAD = 9, /* value 1, for tests of that error path: the staging buffer the
                                    next call would use is marked as still being read by an upload
                                    that never reports back (no GPU involved)                    */
    MPA_OPT_FUSE_APPEND = 12,    /* 1 = mpa_append_and_attend stores the iteration's K/V from inside the
                                    attention launch (extra work-groups of its grid) instead
                                    of in a launch before it, and every row takes the keys of its own
                                    sequence's new positions -- the chunk's own tokens, a generation
                                    row's own token -- from k_new / v_new, since the cache slots are
                                    being written meanwhile (Sec. 2.2: the K/V of a step's tokens are
                                    computed, stored in the KVC and used by that step).  One launch
                                    fewer per layer; same results bit for bit provided no token of the
                                    batch has a negative slot (such a token is still attended to here,
                                    whereas the two-call form reads whatever its cache slot holds).
                                    0 (default) = the append precedes the attention launch            */
    MPA_OPT_PLAN_CACHE = 6       /* 1 (default) = a call whose chunk_starts / context_lens equal
                                    the previous call's reuses its work list (the layers of one
                                    model iteration all present the same batch); 0 = plan anew
                                    on every call; 2 = as 1, and if workspace and stream are the
                                    previous call's too, the work list already in that workspace
                                    is used as it is and nothing is copied: the caller promises
                                    not to write to the workspace between such calls          */
};

/* Create a context for one cache geometry: the head layout of the attention layer (Sec. 2.1: the
 * attention operations run per head; Sec. 6.1 for layers whose query heads share K/V heads), the
 * block size of the block-based KVC (Sec. 2.2) and the 16-bit element type (Sec. 6.1).  Validates
 * cfg; makes no HIP call.
 * Errors: INVALID_ARG (null), UNSUPPORTED (shape or dtype not built). */
int mpa_create(mpa_ctx **out, const mpa_config *cfg);

/* Free the context (and the pinned host staging it may hold).  NULL is accepted. */
int mpa_destroy(mpa_ctx *ctx);

int mpa_set_option(mpa_ctx *ctx, int32_t option, int64_t value);

/* Raw hipError_t of the last failing HIP call made through ctx (0 if none). */
int mpa_last_hip_error(const mpa_ctx *ctx);

const char *mpa_status_string(int status);

/* The attention call cuts long contexts into key ranges that run in parallel and merges their
 * partial results (an exact re-association of the softmax sums of Sec. 2.1); the partial results and
 * the work list live in a caller-provided device workspace.
 * Bytes of device workspace mpa_mixed_paged_attention needs for this very batch
 * (chunk_starts [num_seqs+1] and context_lens [num_seqs] are host pointers, as below).
 * Returns 0 on a malformed batch. */
size_t mpa_workspace_bytes_for_batch(const mpa_ctx *ctx, const int32_t *chunk_starts,
                                     const int32_t *context_lens, int32_t num_seqs);

/* Upper bound of the above over all batches with at most max_seqs sequences, max_tokens query
 * rows in total and context lengths up to max_ctx. */
size_t mpa_workspace_bytes(const mpa_ctx *ctx, int32_t max_seqs, int32_t max_tokens,
                           int32_t max_ctx);

/*
 * KV-cache append (Sec. 2.2 "KVC allocation": the K/V of all tokens of a step are stored in the
 * cache).  For every token t in [0, num_tokens) with slot_map[t] >= 0 and every K/V head h, copies
 * k_new[t,h,:] to k_cache[slot/bs, h, slot%bs, :] and the same for V; bit-exact.
 *
 *   k_new, v_new : device, [num_tokens, HK, D], 16-byte aligned, read only
 *   slot_map     : device, [num_tokens] int64; negative = skip the token.  Non-negative
 *                  entries must be pairwise distinct and below NB*bs (not checked).
 *   k_cache, v_cache : device, [NB, HK, bs, D], 16-byte aligned, written in place
 *   num_tokens == 0 is a no-op.
 * Errors: INVALID_ARG, HIP.
 */
int mpa_kv_append(mpa_ctx *ctx, const void *k_new, const void *v_new, const int64_t *slot_map,
                  int32_t num_tokens, void *k_cache, void *v_cache, void *stream);

/*
 * Whole-block copies between cache pools: for i in [0, num_pairs), block pairs[2i+1] of the
 * destination pool becomes block pairs[2i] of the source pool, K and V, all K/V heads; bit-exact.
 * For moving the blocks of a preempted request to another pool and back (the paper leaves KVC
 * overflow to the engine's swapping, Sec. 5) and for migrating blocks inside one pool.
 *
 *   src_k, src_v : device (or host memory mapped to the device), [NBs, HK, bs, D], read only
 *   dst_k, dst_v : same geometry, [NBd, HK, bs, D], written in place; may be the source pool itself
 *                  as long as no destination block is also a source block of the call
 *   pairs        : device, [num_pairs, 2] int64 {source block, destination block}; a pair with a
 *                  negative id is skipped; ids must be inside their pools and destination ids
 *                  pairwise distinct (not checked)
 *   num_pairs == 0 is a no-op.
 * Errors: INVALID_ARG, HIP.
 */
int mpa_copy_blocks(mpa_ctx *ctx, const void *src_k, const void *src_v, void *dst_k, void *dst_v,
                    const int64_t *pairs, int32_t num_pairs, void *stream);

/*
 * Attention of every query row of a mixed batch over its sequence's cached K/V: the self-attention
 * equation of Sec. 2.1, softmax(Q K^T / sqrt(d_k)) V per head, for a batch that holds prompt chunks
 * (Sec. 2.3 chunking; Sec. 4.2: a chunk is whatever run of a prompt's tokens the token budget and
 * the KVC admitted, so it starts and ends anywhere) next to generation tasks, which contribute one
 * token per iteration once their prompt is done (Sec. 2.3), over the block-based KVC of Sec. 2.2.
 *
 * Sequence i owns rows chunk_starts[i] .. chunk_starts[i+1]-1 of q/out (q_len_i of them; the
 * row boundaries of the ragged batch).  context_lens[i] is the sequence's KV length including
 * this iteration's tokens, which the caller has appended before (same stream => ordered).  Row
 * j of sequence i sits at absolute position p = context_lens[i] - q_len_i + j and gets
 *     out = sum_{t<=p} softmax_t(scale * q . k_t) v_t
 * with k_t, v_t of the head's K/V head read through block_table[i] (the paper also serves
 * Llama-3-70B, Sec. 6.1, whose query heads share K/V heads).  q_len_i == 1 is a generation task, q_len_i > 1 a
 * prompt chunk; both kinds run in one kernel launch.
 *
 *   q            : device, [num_tokens, H, D] of the context's dtype, 16-byte aligned
 *   k_cache, v_cache : device, read only here
 *   block_table  : device, [num_seqs, block_table_stride] int32; entries
 *                  [0, ceil(context_lens[i]/bs)) of row i must be valid block ids (not checked)
 *   chunk_starts : HOST, [num_seqs+1], chunk_starts[0] == 0, strictly increasing,
 *                  chunk_starts[num_seqs] == num_tokens
 *   context_lens : HOST, [num_seqs], context_lens[i] >= q_len_i
 *   scale        : multiplies the scores; <= 0 selects 1/sqrt(D)
 *   out          : device, [num_tokens, H, D], same dtype (round to nearest even of the fp32
 *                  result)
 *   workspace    : device, 256-byte aligned, at least mpa_workspace_bytes_for_batch bytes; holds
 *                  the work list and split partial results for the duration of the call's GPU
 *                  work; contents need no initialisation.  Two calls that may overlap on the GPU
 *                  need different workspaces.
 *   num_seqs == 0 (and num_tokens == 0) is a no-op.
 * Slots past a sequence's context length, unreferenced blocks and table padding never influence
 * the result (they may hold NaN patterns).
 * Errors: INVALID_ARG, BAD_BATCH, WORKSPACE, HIP.
 */
int mpa_mixed_paged_attention(mpa_ctx *ctx, const void *q, const void *k_cache,
                              const void *v_cache, const int32_t *block_table,
                              int32_t block_table_stride, const int32_t *chunk_starts,
                              const int32_t *context_lens, int32_t num_seqs, int32_t num_tokens,
                              float scale, void *out, void *workspace, size_t workspace_bytes,
                              void *stream);

/*
 * mpa_kv_append of all num_tokens rows followed by mpa_mixed_paged_attention, as one call: the
 * append shares a launch with the upload of the call's work list (neither depends on the other,
 * both precede the attention kernel), which takes one kernel out of the chain of an iteration.
 * Arguments and errors as in the two calls; k_cache / v_cache are written (the new tokens' slots)
 * and then read.  Same results, bit for bit, as the two separate calls.
 */
int mpa_append_and_attend(mpa_ctx *ctx, const void *k_new, const void *v_new, const int64_t *slot_map,
                          const void *q, void *k_cache, void *v_cache, const int32_t *block_table,
                          int32_t block_table_stride, const int32_t *chunk_starts, const int32_t *context_lens,
                          int32_t num_seqs, int32_t num_tokens, float scale, void *out, void *workspace,
                          size_t workspace_bytes, void *stream);

/*
 * mpa_mixed_paged_attention for callers that cannot allocate device memory or hand over a
 * workspace: code running under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same kernels, same results bit for bit.  The
 * work list and the partial results of split key ranges live in a device array of
 * MPA_STATIC_SCRATCH_BYTES that is part of the library (every GPU the library runs on holds its
 * copy until the process ends); the work list reaches it as kernel arguments.  The call makes no
 * hipMalloc / hipHostMalloc / hipFree and uses no pinned staging buffer.
 *
 *   - A batch whose work list and partial results need more than MPA_STATIC_SCRATCH_BYTES (what
 *     mpa_workspace_bytes_for_batch returns) is refused with MPA_ERR_WORKSPACE before any HIP call;
 *     use the workspace form for such batches.
 *   - Every context and every call on a GPU shares that GPU's array: calls that may overlap on one
 *     GPU (different streams, different threads) race.  Calls on one stream are ordered and safe;
 *     nothing is assumed to be in the array from an earlier call.
 *   - The device that is current at the call must be the one `stream` belongs to.
 *   - Under stream capture the call records kernel launches only (no memset, no copy, nothing that
 *     reads host memory later: the plan is made at capture time and travels inside the launches'
 *     arguments), so a graph holding it replays the attention step of that very batch layout
 *     (chunk_starts, context_lens, pointers) on whatever the buffers then hold.  Call it once
 *     outside a capture first: the first call on a device looks up the array's address.
 * Errors: INVALID_ARG, BAD_BATCH, WORKSPACE (batch too large for the array), HIP.
 */
#define MPA_STATIC_SCRATCH_BYTES ((size_t)64 << 20)
int mpa_mixed_paged_attention_static(mpa_ctx *ctx, const void *q, const void *k_cache,
                                     const void *v_cache, const int32_t *block_table,
                                     int32_t block_table_stride, const int32_t *chunk_starts,
                                     const int32_t *context_lens, int32_t num_seqs,
                                     int32_t num_tokens, float scale, void *out, void *stream);

/*
 * Kernel timing for benchmarks.  mpa_profile_enable(ctx, n) with n > 0 makes every following
 * mpa_mixed_paged_attention call record a pair of HIP events on its stream directly around the
 * launch of the main attention kernel (after the work-list copy, before the merge), for up to n
 * calls; n == 0 switches it off and frees the events.  mpa_profile_read waits for the recorded
 * events, writes the elapsed milliseconds of up to `cap` calls (oldest first) to `ms` (host),
 * stores the count in *n_out and starts a new series.
 * Errors: INVALID_ARG (also n above 2^24), HIP, NO_MEMORY.
 */
int mpa_profile_enable(mpa_ctx *ctx, int32_t max_calls);
int mpa_profile_read(mpa_ctx *ctx, float *ms, int32_t cap, int32_t *n_out);

/*
 * Measurement aid for benchmarks: launches one micro-kernel on `stream` and returns the amount of
 * work it does (bytes read, or floating-point operations), or a negative status.  The caller
 * times it (events on the stream) to learn what this machine reaches for the patterns the
 * attention kernels are made of; the rates serve as "achievable" denominators next to the
 * published peaks.
 *   MPA_CEIL_STREAM_READ : every byte of buf[0, bytes) once, 16 bytes per lane, non-temporal
 *                          (rounded down to whole passes of the grid; bytes >= 1 MiB)
 *   MPA_CEIL_RANDOM_4K   : 16,384 wavefronts each read iters + 1 contiguous 4 KiB chunks at
 *   MPA_CEIL_RANDOM_16K    pseudo-random chunk positions of buf (16 KiB chunks for the second
 *                          kind), two chunks in flight; iters even, >= 2
 *   MPA_CEIL_MFMA_BF16   : 4,096 wavefronts each issue 4 * iters 32x32x16 bf16 matrix
 *                          instructions from registers (buf and bytes unused); operands with few
 *                          mantissa bits set
 *   MPA_CEIL_MFMA_BF16_NOISY : the same with pseudo-random operands of unit scale (the chip
 *                          sustains a lower clock under them)
 *   buf  : device, 16-byte aligned, read only;   sink : device, 4 bytes, practically never written
 * Errors: INVALID_ARG, HIP.
 */
enum { MPA_CEIL_STREAM_READ = 1, MPA_CEIL_RANDOM_4K = 2, MPA_CEIL_RANDOM_16K = 3, MPA_CEIL_MFMA_BF16 = 4,
       MPA_CEIL_MFMA_BF16_NOISY = 5 };
int64_t mpa_ceiling_launch(int32_t kind, const void *buf, size_t bytes, int32_t iters, void *sink,
                           void *stream);

/*
 * Host-only view of the work decomposition of a batch (no HIP call; usable without a GPU).
 * Writes up to `cap` work items as 8 int32 each
 *   {seq, q_row0, q_rows, q_pos0, kv_begin, kv_end, part_row, kind}
 * and returns the total number of items (which may exceed cap), or a negative status.
 * kind & 0xFF: 0 = a row for all heads on the streaming body, 1 = a tile of prompt rows for all
 * heads on the matrix-core body, 2 = one generation row for the query heads of K/V head
 * kind >> 8 on the matrix-core body (grouped K/V heads, group size >= 4).  Bit 8 of a tile's kind
 * is set when no other tile of the batch reads its keys (and no K/V head is shared): its K/V is
 * then fetched as data that is read once; kind >> 9 of a tile is its first row counted from the
 * first row of its chunk.
 * counts (optional, 4 int32): {matrix-core items, row items, merge rows, partial rows}.
 */
int64_t mpa_plan_describe(const mpa_ctx *ctx, const int32_t *chunk_starts,
                          const int32_t *context_lens, int32_t num_seqs, int32_t *items,
                          int64_t cap, int32_t *counts);

#ifdef __cplusplus
}
#endif
#endif /* MPA_H */
