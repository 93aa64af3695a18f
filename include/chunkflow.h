/*
 * chunkflow.h -- C ABI of the ChunkFlow hot path on one MI355X (gfx950).
 *
 * The library does two things:
 *   1. host side: turn a batch of sequence lengths into uniformly sized chunks (paper section 4.1,
 *      Algorithm 1) and order the chunks' forward/backward passes (section 4.2, Algorithm 2);
 *   2. device side: causal attention forward and backward over one chunk, where a chunk is either
 *      several short sequences packed under a per-sequence causal mask (section 2.2) or one slice
 *      of a long sequence that also attends to the retained key/value state of that sequence's
 *      earlier chunks, the key/value gradients of those earlier rows being accumulated by the
 *      later chunks' backward passes (section 4.2).
 *
 * Conventions
 *   - Every function returns CF_OK (0) or a negative error code; nothing throws, aborts or prints.
 *     cf_last_error() gives a message for the last failing call on the calling thread.
 *   - "host" / "device" on a pointer says where the memory must live.  The library never takes
 *     ownership of a caller's buffer and never allocates device memory.
 *   - Device entry points only enqueue work on the given HIP stream: no synchronisation.
 *   - Tensors are token-major: X[token][head][d] with d contiguous; strides are in ELEMENTS.
 */
#ifndef CHUNKFLOW_H
#define CHUNKFLOW_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    CF_OK = 0,
    CF_EINVAL = -1,       /* NULL pointer, size out of range, inconsistent arguments          */
    CF_EUNSUPPORTED = -2, /* well-formed but not built (head_dim, dtype)                        */
    CF_ENOMEM = -3,       /* host allocation failed                                             */
    CF_EHIP = -4          /* a HIP call failed; cf_last_error() carries hipGetErrorString text  */
};

/* Message of the last error on this thread; static storage, valid until the next failing call. */
const char *cf_last_error(void);
/* major*10000 + minor*100 + patch */
int cf_version(void);

/* ============================================================================================
 * Host planner (no HIP calls).
 * ========================================================================================== */

typedef struct cf_plan cf_plan; /* opaque; owned by the caller after a successful build */

/*
 * Chunk construction, Algorithm 1 (section 4.1).
 *   seq_lens   host, [n_seqs], every entry >= 1
 *   chunk_size 1 .. INT32_MAX
 * Sequences LONGER than chunk_size are cut into ceil(len/chunk_size) consecutive slices, one chunk
 * each, forming one dependency group in ascending order.  The others (length <= chunk_size) are
 * bin-packed: for BinCnt = 1, 2, ... the sequences, longest first (ties: input order), each go
 * to the currently least-loaded bin (ties: lowest bin); the first BinCnt for which no bin exceeds
 * chunk_size wins.  Each non-empty bin becomes one packed chunk (a group of size 1) whose
 * segments are in input order.  Chunk ids: slices of long sequences first (input order), then
 * packed chunks (bin order).
 * Errors: NULL seq_lens with n_seqs > 0, NULL out, n_seqs < 0, chunk_size out of range, a length
 * < 1 -> CF_EINVAL and *out is untouched.  n_seqs == 0 gives a valid empty plan.
 */
int cf_build_chunks(const int64_t *seq_lens, int64_t n_seqs, int64_t chunk_size, cf_plan **out);

/*
 * Algorithm 1 with options (flags = 0: exactly cf_build_chunks).
 *   CF_PLAN_MERGE_TAILS  A variant section 4.1 leaves open: the last slice of a split sequence, when shorter
 *     than chunk_size, is not a chunk of its own but one more item of the bin-packing (its weight is its
 *     length), so that it shares a chunk with short sequences instead of leaving that chunk mostly empty.
 *     Items (short sequences and tails) are placed longest first (ties: sequence order) into the
 *     least-loaded bin (ties: lowest bin); a tail only goes to a bin that holds no tail yet, so a chunk
 *     depends on at most one split sequence.  An attempt fails when an item does not fit or a tail finds no
 *     tail-free bin; the first BinCnt (1, 2, ...) that succeeds wins.
 *     The chunk that holds a tail is the LAST chunk of that sequence's group (chunk_group, chunk_idx_in_group
 *     say so; group_chunks lists it after the slices); its chunk_prefix_len is the tail's seg_seq_start and
 *     its segments are in sequence order like any packed chunk.  Only the tail segment has seg_seq_start > 0:
 *     for the kernels that is a chunk with one segment whose keys are longer than its queries.
 * Errors as cf_build_chunks; unknown flag bits -> CF_EINVAL.
 */
enum { CF_PLAN_MERGE_TAILS = 1 };
int cf_build_chunks_ex(const int64_t *seq_lens, int64_t n_seqs, int64_t chunk_size, uint32_t flags, cf_plan **out);
void cf_plan_free(cf_plan *plan); /* NULL is fine */

/* Read-only view of a plan.  All pointers are host memory borrowed from the plan and stay valid
 * until cf_plan_free.  Segments of chunk c are [chunk_seg_ptr[c], chunk_seg_ptr[c+1]). */
typedef struct {
    int64_t n_chunks, n_segments, n_groups, total_tokens, chunk_size;
    const int64_t *chunk_seg_ptr;      /* [n_chunks+1]                                          */
    const int32_t *chunk_tokens;       /* [n_chunks]  tokens in the chunk (<= chunk_size)        */
    const int64_t *chunk_prefix_len;   /* [n_chunks]  tokens of the same sequence in earlier chunks (of the tail's
                                          sequence for a chunk that holds a merged tail)          */
    const int32_t *chunk_group;        /* [n_chunks]                                            */
    const int32_t *chunk_idx_in_group; /* [n_chunks]  0-based                                   */
    const int64_t *seg_seq_id;         /* [n_segments] index into seq_lens                      */
    const int64_t *seg_seq_start;      /* [n_segments] first token of that sequence covered     */
    const int32_t *seg_len;            /* [n_segments]                                          */
    const int32_t *cu_seqlens;         /* [n_segments+n_chunks]; chunk c's local exclusive prefix
                                          sums (n_seg_c+1 entries, first is 0) start at index
                                          chunk_seg_ptr[c] + c                                   */
    const int64_t *group_chunk_ptr;    /* [n_groups+1]                                          */
    const int64_t *group_chunks;       /* [n_chunks]  chunk ids per group, ascending dependency (forward) order */
    const int64_t *group_seq_id;       /* [n_groups]  the split sequence, or -1 for a packed chunk that depends on none */
} cf_plan_view;
int cf_plan_get(const cf_plan *plan, cf_plan_view *out);

/*
 * State-aware chunk scheduling, Algorithm 2 (section 4.2), applied to every group in group order.
 * K >= 1 is the number of chunks whose activations may be kept.  For a group of N chunks:
 *   N <= K : FWD_KEEP 0..N-1, then BWD N-1..0.
 *   N >  K : FWD_DISCARD 0..N-K-1, FWD_KEEP N-K..N-1, BWD N-1..N-K, then for m = N-K-1 .. 0:
 *            FWD_KEEP m, BWD m   (the first N-K chunks run forward twice).
 * *ops is host memory owned by the plan, valid until the next cf_build_schedule on this plan or
 * cf_plan_free.
 */
enum { CF_OP_FWD_KEEP = 0, CF_OP_FWD_DISCARD = 1, CF_OP_BWD = 2 };
typedef struct {
    int32_t op;
    int32_t reserved;
    int64_t chunk;
} cf_sched_op;
int cf_build_schedule(cf_plan *plan, int32_t K, const cf_sched_op **ops, int64_t *n_ops);

/*
 * What a schedule costs and holds (section 4.2: the first N-K chunks of a group run forward twice; the
 * memory kept for the backward passes is bounded by K * ChunkSize).  Replays the ops of
 * cf_build_schedule(plan, K): a FWD_KEEP op adds its chunk to the kept set, the chunk's BWD op removes it,
 * a FWD_DISCARD op keeps nothing.
 *   n_forward, n_backward   ops of each kind (FWD_KEEP + FWD_DISCARD, BWD)
 *   n_reforward             forward ops beyond one per chunk (= sum over groups of max(0, N - K))
 *   peak_kept_chunks        largest size of the kept set           (<= K when every group has >= K chunks ...
 *   peak_kept_tokens        largest token count of the kept set     ... and always <= K * chunk_size)
 *   state_tokens            largest key/value state alive at once: tokens of the longest split sequence
 *                           (the state of a group is released when the group is done), 0 if none is split
 * Errors as cf_build_schedule; NULL out -> CF_EINVAL.  The plan's stored schedule is replaced by this K's.
 */
typedef struct {
    int64_t n_forward, n_backward, n_reforward;
    int64_t peak_kept_chunks, peak_kept_tokens;
    int64_t state_tokens;
} cf_sched_stats;
int cf_schedule_stats(cf_plan *plan, int32_t K, cf_sched_stats *out);

/*
 * Pipeline bubble ratio of a 1F1B schedule under the paper's cost model for its pipeline examples (section 3.3:
 * the time of a micro-batch is proportional to its length, backward = 2 x forward; equation 1: bubble ratio =
 * total bubble time / total execution time over all stages).  Integer ticks: forward of n tokens = n, backward 2n.
 *
 * cf_sim_1f1b_sequences  standard 1F1B (section 3.3) with every sequence a micro-batch of its own, in the given
 *     order: stage s of p runs p-1-s warm-up forwards, then one forward / one backward alternately, then drains.
 * cf_sim_1f1b            state-aware 1F1B (section 4.3) over the chunks of a plan: the same shape, but the
 *     forward-type passes (first forwards and the re-forwards of discarded chunks) and the backward passes are
 *     those of Algorithm 2 with K kept chunks, each kind in Algorithm 2's order; on every stage a pass waits for the
 *     previous op of its own dependency group; a stage starts a forward that keeps activations while it holds fewer
 *     than p-s kept chunks or while the next backward may not run yet, otherwise it runs the next backward.
 *     Groups are taken standalone chunks first, then the dependent groups (the numbering of the paper's chunk
 *     figure); CF_SIM_PLAN_ORDER takes them in plan order instead.
 * Every op starts as early as its stage and its pipeline neighbour allow (forward: the same op one stage earlier;
 * backward: one stage later).
 *   out->makespan        ticks until the last stage is done
 *   out->busy_per_stage  ticks of work on each stage (equal on all stages; re-forwards count as work)
 *   out->bubble_ticks / out->total_ticks = the bubble ratio, total_ticks = n_stages * makespan
 * Reproduces the paper's 57.14 %, 42.8 % (3/7), 47.8 % (22/46) and 60 %; its 54.1 % (ChunkSize 2 Units, K = 1) is
 * not reachable in this cost model (every pass there lasts an even number of Units).
 * Errors: NULL arguments, K < 1, n_stages < 1, a length < 1, unknown flags -> CF_EINVAL.  The plan's stored schedule
 * (cf_build_schedule) is not touched.
 */
typedef struct {
    int64_t makespan, busy_per_stage, bubble_ticks, total_ticks;
    int64_t n_ops;
    int32_t n_stages, reserved;
} cf_pipeline_stats;
enum { CF_SIM_PLAN_ORDER = 1 };
int cf_sim_1f1b_sequences(const int64_t *seq_lens, int64_t n_seqs, int32_t n_stages, cf_pipeline_stats *out);
int cf_sim_1f1b(cf_plan *plan, int32_t K, int32_t n_stages, uint32_t flags, cf_pipeline_stats *out);

/* ============================================================================================
 * Device kernels.
 * ========================================================================================== */

enum { CF_BF16 = 0, CF_FP32 = 1 };
/* flags: CF_FLAG_SCALAR_KERNELS runs the plain scalar kernels even where an MFMA kernel exists
 * (same results up to rounding; for cross-checks).
 * CF_FLAG_DKV_SINGLE_WRITER (backward, bf16 head_dim 128): every dK/dV row is updated by ONE workgroup that loops
 * over the query heads of its key/value head, with a plain read-modify-write -- dK/dV are then bitwise reproducible
 * from run to run.  Without the flag the library takes that mode only when a launch has enough key tiles to fill
 * the GPU that way (>= 4096 key-tile x kv-head pairs: long prefixes) and otherwise splits the query heads of a
 * group over workgroups that meet in dK/dV through fp32 atomic adds (faster on short chunks; last bits vary). */
enum { CF_FLAG_SCALAR_KERNELS = 1, CF_FLAG_DKV_SINGLE_WRITER = 2 };

/*
 * One chunk of attention (sections 2.1, 2.2, 4.2).  The chunk has n_segments segments; segment g
 * owns query rows [cu_seqlens_q[g], cu_seqlens_q[g+1]) of q/o and key rows
 * [cu_seqlens_k[g], cu_seqlens_k[g+1]) of k/v, with Lk_g >= Lq_g >= 1.  The causal mask is aligned
 * to the END of the keys: query i (local) sees key j (local) iff j <= i + (Lk_g - Lq_g).
 *   packed chunk    : cu_seqlens_k == cu_seqlens_q, k/v are the chunk's own keys/values.
 *   dependent chunk : one segment, cu_seqlens_k = {0, P+T}; k/v point at the base of the
 *                     sequence's state buffer whose rows [0,P) were written by earlier chunks and
 *                     whose rows [P,P+T) the caller filled with this chunk's keys/values.
 * Query head h reads key/value head h / (n_q_heads / n_kv_heads).
 * dtype CF_BF16: q,k,v,o are bf16, arithmetic accumulates in fp32.  CF_FP32: all fp32.
 * cu_seqlens are NOT validated (they live on the device): the caller guarantees they are
 * non-decreasing, start at 0, end at n_tokens (q) / n_kv_tokens (k) and satisfy Lk_g >= Lq_g.
 */
typedef struct {
    int32_t dtype;                      /* CF_BF16 or CF_FP32                                    */
    int32_t flags;                      /* 0, or CF_FLAG_* bits                                  */
    int32_t n_q_heads, n_kv_heads;      /* n_q_heads % n_kv_heads == 0                           */
    int32_t head_dim;                   /* 64 or 128                                             */
    float softmax_scale;
    int32_t n_tokens;                   /* query rows T >= 1                                     */
    int32_t n_kv_tokens;                /* key rows  (sum of Lk_g) >= n_tokens                   */
    int32_t n_segments;                 /* >= 1                                                  */
    const int32_t *cu_seqlens_q;        /* device, [n_segments+1]                                */
    const int32_t *cu_seqlens_k;        /* device, [n_segments+1]                                */
    const void *q;                      /* device, [T][Hq][D]                                    */
    int64_t q_stride_tok, q_stride_head;
    const void *k, *v;                  /* device, [n_kv_tokens][Hkv][D], same strides for both  */
    int64_t kv_stride_tok, kv_stride_head;
    void *o;                            /* device, [T][Hq][D], written                           */
    int64_t o_stride_tok, o_stride_head;
    float *lse;                         /* device, [Hq][T] natural-log sum of exponentials, written */
    const struct cf_q_tile *q_tiles;    /* device, [n_q_tiles], or NULL (see cf_attn_q_tiles)    */
    int32_t n_q_tiles;                  /* 0 when q_tiles is NULL                                */
} cf_attn_fwd_params;

/*
 * Optional launch order of a chunk (not part of the paper's method; a descriptor like cu_seqlens).  The bf16
 * head_dim-128 kernels give every 128 query rows of a segment to one workgroup per head, and the work of such
 * a tile grows with its position in the sequence.  Workgroups start in grid order, so the order decides how
 * well the last ones fill the machine.  Without a table each workgroup finds its tile by searching
 * cu_seqlens (tiles of the last segment first); with one, workgroup rank r takes q_tiles[r]: the tiles of the
 * whole chunk sorted by the number of keys they read, longest first, each with its segment's bounds so that
 * the kernel reads one 32-byte record instead of searching.
 * cf_attn_q_tiles builds the table on the HOST from host copies of cu_seqlens (it depends only on the chunk's
 * geometry: build it once per plan, upload it, pass the device pointer).  Like cu_seqlens the device copy is
 * not validated.  The scalar kernels ignore it.
 *   out       host, [capacity] records, or NULL to only count
 *   returns   the number of tiles = sum over segments of ceil(Lq_g / 128), or CF_EINVAL (NULL cu arrays,
 *             n_segments < 1, a segment with Lq < 1 or Lk < Lq, capacity too small for a non-NULL out)
 */
typedef struct cf_q_tile {
    int32_t q_begin, q_len;             /* the segment's query rows: cu_seqlens_q[g], Lq_g       */
    int32_t k_begin, k_len;             /* the segment's key rows:   cu_seqlens_k[g], Lk_g       */
    int32_t tile;                       /* this tile covers rows [128*tile, 128*tile+128) of the segment */
    int32_t segment;                    /* g                                                     */
    int32_t reserved[2];
} cf_q_tile;
int64_t cf_attn_q_tiles(const int32_t *cu_seqlens_q_host, const int32_t *cu_seqlens_k_host, int32_t n_segments,
                        cf_q_tile *out, int64_t capacity);

/* Enqueue the forward pass.  Errors: NULL pointers, sizes < 1, n_kv_tokens < n_tokens,
 * Hq % Hkv != 0, misaligned base pointers or strides (bf16: multiples of 8 elements, fp32: of 4),
 * q_tiles without a plausible n_q_tiles (or the reverse) -> CF_EINVAL; head_dim / dtype not built -> CF_EUNSUPPORTED; launch failure -> CF_EHIP. */
int cf_attn_fwd(const cf_attn_fwd_params *p, void *hip_stream);

/*
 * Backward pass of the same chunk.  f repeats the forward call's arguments (o and lse are inputs
 * here).  d_q is overwritten.  d_k / d_v are fp32 [n_kv_tokens][Hkv][D] and are ADDED TO: for a
 * dependent chunk they point at the base of the sequence's gradient state, so that rows [0,P)
 * collect the contributions of later chunks when the group's chunks run in descending order; the
 * caller zeroes them once per long sequence / per packed chunk.  Launches on one stream are
 * ordered, and inside one launch every d_k/d_v element has a single writer.
 * workspace: device scratch of at least cf_attn_bwd_workspace_bytes(&f) bytes, 256-byte aligned;
 * contents need not be initialised and are not preserved.
 */
typedef struct {
    cf_attn_fwd_params f;
    const void *d_o;                    /* device, [T][Hq][D], dtype as f.dtype                  */
    int64_t do_stride_tok, do_stride_head;
    void *d_q;                          /* device, [T][Hq][D], dtype as f.dtype, overwritten     */
    int64_t dq_stride_tok, dq_stride_head;
    float *d_k, *d_v;                   /* device, fp32, accumulated                             */
    int64_t dkv_stride_tok, dkv_stride_head;
    void *workspace;
    int64_t workspace_bytes;
} cf_attn_bwd_params;

/* Bytes of workspace cf_attn_bwd needs for these shapes (only sizes/dtype are read), or a
 * negative error code. */
int64_t cf_attn_bwd_workspace_bytes(const cf_attn_fwd_params *p);
int cf_attn_bwd(const cf_attn_bwd_params *p, void *hip_stream);

/*
 * cf_attn_bwd for callers that cannot allocate device memory or carry a workspace around: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as cf_attn_bwd,
 * except that p->workspace / p->workspace_bytes are IGNORED: delta and the dK/dV work list live in a buffer of
 * CF_STATIC_SCRATCH_BYTES that is part of the library's device code (one copy per GPU, held until the process
 * ends).  The call allocates and frees nothing (no hipMalloc / hipFree, no allocating library routine) and, like
 * cf_attn_bwd, only enqueues kernels on the stream.
 *   - A chunk whose cf_attn_bwd_workspace_bytes exceeds CF_STATIC_SCRATCH_BYTES -> CF_EINVAL (decided on the
 *     host before any HIP call; n_q_heads * n_tokens * 4 bytes dominate: 64 heads x 32768 tokens need 8.3 MiB).
 *   - Every call on a GPU uses that GPU's one buffer, which keeps the previous call's contents; nothing in it
 *     has to start at zero (each call overwrites what it reads).  Calls that OVERLAP on one GPU (two streams,
 *     two threads) race on it: keep them on one stream or order them with events.
 *   - The first call on a device looks the buffer's address up (hipGetSymbolAddress); a failure -> CF_EHIP.
 * Other errors as cf_attn_bwd.
 */
#define CF_STATIC_SCRATCH_BYTES (16 << 20)
int cf_attn_bwd_static(const cf_attn_bwd_params *p, void *hip_stream);

/*
 * Whole-plan launches: several chunks in one call.  The results are those of calling cf_attn_fwd /
 * cf_attn_bwd for params[0], params[1], ... in that order on the stream (dK/dV that several chunks share --
 * the chunks of one long sequence, section 4.2 -- accumulate in exactly that order).  What changes is the
 * launch shape: for a run of consecutive chunks that take the bf16 head_dim-128 path with equal head counts
 * (up to 16 forward, 8 backward), the forward kernels -- and in the backward the dQ kernels, which touch
 * nothing another chunk's backward writes -- become ONE launch whose workgroups are dealt heaviest chunk
 * first, so that the last, partly filled wave of workgroups of a big chunk is filled by the next chunk's
 * instead of leaving compute units idle.  The dK/dV kernels still run chunk by chunk.
 *   params  host array [n]; for the backward every chunk needs a workspace of its OWN (they are in use at
 *           the same time; overlapping workspaces -> CF_EINVAL)
 * Errors: as the single-chunk calls, checked for every chunk before anything is enqueued; n == 0 is a no-op.
 */
int cf_attn_fwd_batch(const cf_attn_fwd_params *params, int32_t n, void *hip_stream);
int cf_attn_bwd_batch(const cf_attn_bwd_params *params, int32_t n, void *hip_stream);

/*
 * Measurement aid (not part of the paper's method): when both events (hipEvent_t, created by the
 * caller with timing enabled) are non-NULL, the NEXT cf_attn_fwd / cf_attn_bwd call on this thread
 * records `start` right before and `stop` right after its main kernel (forward: the attention
 * kernel; backward: the dK/dV kernel -- both of its launches where it takes two -- without the dQ kernel that
 * runs before it) on that call's
 * stream, then the hook clears itself.  The batch entry points clear an armed hook without recording (they time
 * nothing); a call that fails its argument checks leaves it armed.  Passing NULLs clears it.
 * The hook is per-thread state of the library (its only state besides cf_last_error's message).  Never fails.
 */
int cf_profile_next_call(void *start_event, void *stop_event);

/* Number of unmasked (query, key) pairs of a chunk described by HOST copies of its cu_seqlens:
 * sum over segments of Lq*(Lk-Lq) + Lq*(Lq+1)/2.  Used to turn run time into FLOP/s. */
int64_t cf_count_pairs(const int32_t *cu_seqlens_q_host, const int32_t *cu_seqlens_k_host,
                       int32_t n_segments);

#ifdef __cplusplus
}
#endif
#endif /* CHUNKFLOW_H */
