/*
 * dit_attn.h - C ABI of the MI355X (gfx950) DiT denoising-step self-attention.
 *
 * One call computes, for a packed batch of independent token sequences, the
 * self-attention of a DiT block during one denoising step:
 *
 *     for every sequence i with rows R_i = [cu_seqlens[i], cu_seqlens[i+1]),
 *     every head h and every query row r in R_i:
 *         O[r,h,:] = sum_{j in R_i} softmax_j( scale * <Q[r,h,:], K[j,h,:]> ) * V[j,h,:]
 *
 * The batch is what the paper's serving loop hands to a GPU for one step:
 * same-resolution image requests coalesced into one call (paper Section 4.3,
 * "SLO-aware Dynamic Batching"), a whole video request (Section 4.4, one
 * request per GPU set), or one GPU's head subset of a sequence-parallel video
 * (Section 5, Unified Sequence Parallel attention; Section 4.3, "Elastic
 * Sequence Parallelism").  Attention is bidirectional inside a sequence and
 * never crosses sequences.  Text and latent tokens are ordinary rows.
 *
 * Precision: bf16 inputs, fp32 scores / softmax state / accumulators, the
 * probabilities are rounded to bf16 (nearest-even) before the second
 * contraction and the row sum l is taken over the rounded values (O / l is
 * then a convex combination of V rows whatever the rounding did; lse carries
 * at most their 2^-8 relative error, i.e. 4e-3 absolute), bf16 output
 * (nearest-even).  The softmax reference value of a row follows its running
 * maximum lazily (it moves when exceeded by more than 8 in the base-2
 * exponent); the quotient O / l does not depend on it.
 *
 * All functions are thread-compatible, not thread-safe: one context must not
 * be used from two host threads, or for two streams, at the same time.
 * No C++ exception crosses this boundary.
 */
#ifndef DIT_ATTN_H_
#define DIT_ATTN_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Return codes. */
#define DIT_ATTN_OK                 0
#define DIT_ATTN_ERR_NULL          (-1)  /* a required pointer is NULL */
#define DIT_ATTN_ERR_HEAD_DIM      (-2)  /* head_dim is not 64 or 128 */
#define DIT_ATTN_ERR_CU_SEQLENS    (-3)  /* cu_seqlens[0] != 0, decreasing, or n_seqs < 0 */
#define DIT_ATTN_ERR_HIP           (-4)  /* a HIP runtime call failed; see dit_attn_last_error */
#define DIT_ATTN_ERR_SCALE         (-5)  /* scale is NaN or infinite */
#define DIT_ATTN_ERR_N_HEADS       (-6)  /* n_heads < 1 or > 65535 */
#define DIT_ATTN_ERR_ALIGN         (-7)  /* q, k, v or out is not 16-byte aligned */
#define DIT_ATTN_ERR_CAPACITY      (-8)  /* output buffer of dit_attn_plan too small */
#define DIT_ATTN_ERR_KERNEL        (-9)  /* dit_attn_set_kernel: no such kernel */
#define DIT_ATTN_ERR_PARTS         (-10) /* dit_attn_merge: n_parts outside 1..8 */
#define DIT_ATTN_ERR_LIMIT         (-11) /* dit_attn_varlen_fwd_noalloc: the pack exceeds the fixed scratch limits */
#define DIT_ATTN_ERR_CAPTURE       (-12) /* the stream is capturing and the call would have to allocate or copy */

typedef struct dit_attn_ctx dit_attn_ctx; /* opaque */

/*
 * Create a context bound to HIP device `device_id` (host call).
 * The context owns a small amount of device memory: cached work-lists (one per
 * distinct (cu_seqlens, n_heads, head_dim) seen, 16 bytes per work item) and a
 * work counter.  *out_ctx is written only on success.
 * Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL, or DIT_ATTN_ERR_HIP (no such device,
 * not a gfx950 device, allocation failure).
 */
int dit_attn_create(dit_attn_ctx** out_ctx, int device_id);

/*
 * One denoising-step attention call over a packed variable-length batch
 * (paper Sections 4.3 and 5; the math is the definition at the top of this file).
 *
 *   q, k, v     DEVICE pointers, bf16, shape [T, n_heads, head_dim], contiguous
 *               (row stride n_heads*head_dim elements), T = cu_seqlens[n_seqs].
 *               16-byte aligned.  Read only.
 *   cu_seqlens  HOST pointer, n_seqs + 1 int32 entries, cu_seqlens[0] == 0,
 *               non-decreasing.  Read during the call only (the batch is formed
 *               by host code, which knows the lengths).  Zero-length sequences
 *               are legal and contribute no rows.
 *   n_seqs      number of sequences, >= 0.  n_seqs == 0 or T == 0: returns
 *               DIT_ATTN_OK and launches nothing.
 *   n_heads     heads in q, k and v alike (no grouped-query sharing), 1..65535.
 *   head_dim    64 or 128.
 *   scale       multiplies the fp32 scores before the softmax; any finite value
 *               (zero and negative included).
 *   out         DEVICE pointer, bf16, same shape and layout as q; must not
 *               overlap q, k or v.  Exactly the rows [0, T) are written.
 *   stream      a hipStream_t (as void*); NULL is the default stream.
 *
 * The work is enqueued on `stream`; the call does not synchronise.  The first
 * call with a new (cu_seqlens, n_heads, head_dim) builds a work-list on the host
 * and uploads it (one device allocation and one synchronous copy); later
 * calls with the same pack reuse it and do no host work beyond a compare.
 * Under HIP graph capture only such a later call is possible (else DIT_ATTN_ERR_CAPTURE); the captured pack stays
 * cached until the context is destroyed (see dit_attn_plan_cache_victim).
 * The caller keeps ownership of every buffer.  Validation precedes any launch:
 * on a non-zero return `out` is untouched.
 */
int dit_attn_varlen_fwd(dit_attn_ctx* ctx,
                        const void* q, const void* k, const void* v,
                        const int32_t* cu_seqlens, int32_t n_seqs,
                        int32_t n_heads, int32_t head_dim, float scale,
                        void* out, void* stream);

/*
 * For callers that cannot allocate device memory: code being recorded into a HIP graph that meets a pack for the first
 * time, tight serving loops, harnesses that forbid hipMalloc.  The same operation as dit_attn_varlen_fwd, same
 * arguments, same result bit for bit, but the call allocates nothing and copies nothing: the work-list is written by a
 * small kernel on `stream` (the sequence boundaries travel as its argument) into a fixed device array of the library
 * (256 KB + 256 B per GPU, held until the process ends), which also holds the kernels' work counters.
 * Limits: n_seqs <= 64 and at most 16384 work items per pack (an item is 256 query rows of one head, 128 for packs that
 * the 128-row kernel runs; the five benchmark configurations need 32 to 4632); beyond them DIT_ATTN_ERR_LIMIT, `out`
 * untouched.  No split-KV, no plan cache, dit_attn_last_launch_clock is not updated.
 * Every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, contexts or threads) race;
 * calls on one stream are ordered and safe.  Other return codes as dit_attn_varlen_fwd.
 */
int dit_attn_varlen_fwd_noalloc(dit_attn_ctx* ctx,
                                const void* q, const void* k, const void* v,
                                const int32_t* cu_seqlens, int32_t n_seqs,
                                int32_t n_heads, int32_t head_dim, float scale,
                                void* out, void* stream);

/*
 * Destroy a context and free its device memory (host call).  The caller must
 * have synchronised every stream the context was used on.  NULL is a no-op.
 */
void dit_attn_destroy(dit_attn_ctx* ctx);

/*
 * The same operation, also returning the row-wise log-sum-exp
 *     lse[r, h] = ln sum_j exp(scale * <Q[r,h,:], K[j,h,:]>)     (natural log, fp32, [T, H] contiguous, DEVICE)
 * which is what makes results over disjoint key sets combinable (dit_attn_merge).  Sequence parallelism along the
 * sequence - the ring half of the unified sequence parallelism that the paper's elastic SP builds on (Section 5,
 * Section 4.3) - hands a GPU one block of keys per step and needs exactly this pair per block.
 * lse must be 4-byte aligned and hold total_tokens * n_heads floats; everything else as dit_attn_varlen_fwd.
 * Accuracy contract: |lse - exact| <= 4e-3.  The sum inside the logarithm is taken over the probabilities as rounded to
 * bf16 for the second contraction (each within 2^-8 relative, all positive), so lse is within ln(1 + 2^-8) = 3.9e-3
 * of the exact value plus ~1e-5 of fp32 arithmetic; the bound is approached only by rows that one key dominates
 * (typically < 1e-3).  In exchange a merge that uses these lse values reproduces exactly the quotient that a single
 * pass over all keys forms from the same rounded probabilities.
 */
int dit_attn_varlen_fwd_lse(dit_attn_ctx* ctx,
                            const void* q, const void* k, const void* v,
                            const int32_t* cu_seqlens, int32_t n_seqs,
                            int32_t n_heads, int32_t head_dim, float scale,
                            void* out, float* lse, void* stream);

/*
 * Cross-attention over a packed batch (paper Section 2.1: the DiT blocks also attend to the text tokens for text
 * alignment): queries and keys have separate boundaries.  Sequence i's query rows
 * cu_seqlens_q[i] .. cu_seqlens_q[i+1] of q ([Tq, H, D]) see key rows cu_seqlens_k[i] .. cu_seqlens_k[i+1] of k and v
 * ([Tk, H, D]); both arrays are HOST pointers with n_seqs + 1 entries starting at 0, non-decreasing.  out is
 * [Tq, H, D]; lse ([Tq, H], DEVICE) may be NULL.  Query rows of a sequence that has no keys get O = 0 and
 * lse = -inf (an empty sum).  Errors and all other arguments as dit_attn_varlen_fwd.
 */
int dit_attn_cross_varlen_fwd(dit_attn_ctx* ctx,
                              const void* q, const void* k, const void* v,
                              const int32_t* cu_seqlens_q, const int32_t* cu_seqlens_k, int32_t n_seqs,
                              int32_t n_heads, int32_t head_dim, float scale,
                              void* out, float* lse, void* stream);

/*
 * Merge n_parts (1..8) partial results of the SAME queries over DISJOINT key sets (paper Section 5: sequence
 * parallelism splits a long video's sequence over GPUs; each block of keys yields one partial result):
 *     lse = ln sum_p exp(lse_p),     O = sum_p exp(lse_p - lse) O_p.
 * o_parts / lse_parts: HOST arrays of n_parts DEVICE pointers, each to bf16 [total_rows, H, D] / fp32
 * [total_rows, H] as written by dit_attn_varlen_fwd_lse or dit_attn_cross_varlen_fwd.  A part whose lse is -inf in a
 * row has weight 0 there; a row whose parts are all -inf becomes 0 with lse -inf.  out may alias one of the parts;
 * lse_out may be NULL.  fp32 arithmetic, bf16 output rounded to nearest even.  Enqueues one kernel on `stream`.
 * Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL, _HEAD_DIM, _N_HEADS, _PARTS, _CU_SEQLENS (total_rows < 0), _ALIGN, _HIP.
 */
int dit_attn_merge(dit_attn_ctx* ctx,
                   const void* const* o_parts, const float* const* lse_parts, int32_t n_parts,
                   int64_t total_rows, int32_t n_heads, int32_t head_dim,
                   void* out, float* lse_out, void* stream);

/*
 * Single-GPU halves of the head-split sequence-parallel exchange (paper Section 4.3: elastic sequence parallelism
 * gives a video p in {1,2,4,8} GPUs; Section 5: the head-split half of the unified sequence parallelism).  A rank
 * holds n_rows rows of the sequence with all n_heads heads; attention needs the whole sequence for n_heads / p heads.
 *     pack:    src [n_rows, H, D]        -> dst [p, n_rows, H/p, D]   dst[g, r, h, :] = src[r, g*H/p + h, :]
 *     unpack:  src [p, n_rows, H/p, D]   -> dst [n_rows, H, D]        dst[r, g*H/p + h, :] = src[g, r, h, :]
 * Block g of pack's output is what goes to rank g before attention (the blocks a rank receives, in source-rank order,
 * are its [L, H/p, D] input without further copying); unpack's input is the blocks a rank receives after attention,
 * in source-rank order.  bf16, DEVICE buffers, 16-byte aligned, src and dst must not overlap.  sp_degree (p) >= 1 must
 * divide n_heads.  Enqueues one kernel on `stream`; moves every byte once (HBM bound).
 * Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL, _HEAD_DIM, _N_HEADS (also: p does not divide n_heads), _CU_SEQLENS
 * (n_rows < 0), _ALIGN, _HIP.
 */
int dit_attn_sp_pack_heads(dit_attn_ctx* ctx, const void* src, void* dst, int64_t n_rows,
                           int32_t n_heads, int32_t head_dim, int32_t sp_degree, void* stream);
int dit_attn_sp_unpack_heads(dit_attn_ctx* ctx, const void* src, void* dst, int64_t n_rows,
                             int32_t n_heads, int32_t head_dim, int32_t sp_degree, void* stream);

/*
 * Kernel choice of a context.  The library has two kernels for the same
 * operation (which one is fastest depends on the pack, Section 4.3 / Table 3:
 * image steps are short, video steps long):
 *     DIT_ATTN_KERNEL_AUTO   (-1) chosen per pack: the ping-pong kernel when
 *                                 its 256-row items fill the compute units,
 *                                 the 128-row kernel for packs with under half
 *                                 such an item per compute unit, whose second
 *                                 round would be under 40 % full, or
 *                                 (cross-attention) with at most 320 keys per
 *                                 item on average
 *     DIT_ATTN_KERNEL_128     (0) 128 query rows per tile
 *     DIT_ATTN_KERNEL_PINGPONG(1) 256 rows per tile, two alternating groups
 * The kernels do the same arithmetic in the same order: their results agree
 * bit for bit.  A forced kernel applies to later calls on `ctx`; meant for
 * tests and measurements.
 * Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL or DIT_ATTN_ERR_KERNEL.
 */
#define DIT_ATTN_KERNEL_AUTO     (-1)
#define DIT_ATTN_KERNEL_128        0
#define DIT_ATTN_KERNEL_PINGPONG   1
int dit_attn_set_kernel(dit_attn_ctx* ctx, int kernel);

/*
 * Split-KV for small packs (paper Section 3 / Table 3: a low-resolution image step is far too small to fill a GPU).
 * With max_splits > 1, a pack that runs the 128-row kernel and has fewer work items than compute units has the keys of
 * every sequence cut into up to max_splits chunks (as many as it takes to reach two items per compute unit, and only
 * where a cost model measured on MI355X says the split pays: roughly from 3100 keys on for four chunks, 2200 for eight,
 * 4400 for three, 13800 for two); the chunks run as separate items that leave normalised fp32 partial results and their
 * log-sum-exp in a workspace owned by the context (grown with hipMalloc when a call needs more), and one merge kernel
 * on the same stream writes `out`.  Off (max_splits = 1) by default, because it changes the summation order: with it
 * a sequence's bits depend on what it is packed with (they stay within the same tolerance of the exact result).
 * Applies to every forward entry point.  Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL or DIT_ATTN_ERR_PARTS (outside 1..8).
 */
int dit_attn_set_split_kv(dit_attn_ctx* ctx, int max_splits);

/*
 * Clock sample of the last kernel launched through `ctx`: the first workgroup
 * of every launch reads the GPU's shader-cycle counter and its constant 100 MHz
 * counter when it starts and when it ends.  shader_mhz is the ratio (the clock
 * the chip sustained under that kernel; MI355X lowers it under matrix load, so
 * throughput at a fixed number of cycles per tile moves with it); kernel_ms is
 * how long that workgroup ran.  Either pointer may be NULL; both values are 0
 * before the first launch.  Synchronises the whole device.
 * Returns DIT_ATTN_OK, DIT_ATTN_ERR_NULL or DIT_ATTN_ERR_HIP.
 */
int dit_attn_last_launch_clock(dit_attn_ctx* ctx, double* shader_mhz, double* kernel_ms);

/*
 * Which attention kernel the last forward call on `ctx` launched:
 * DIT_ATTN_KERNEL_128 or DIT_ATTN_KERNEL_PINGPONG, or DIT_ATTN_KERNEL_AUTO (-1)
 * if no attention kernel has been launched yet.  For measurements that name
 * the kernel they timed.  Host state only; NULL returns DIT_ATTN_KERNEL_AUTO.
 */
int dit_attn_last_launch_kernel(const dit_attn_ctx* ctx);

/*
 * Text of the last error recorded in `ctx` (or of the last failed
 * dit_attn_create when ctx is NULL).  The string is owned by the library and
 * valid until the next call on the same context.
 */
const char* dit_attn_last_error(const dit_attn_ctx* ctx);

/*
 * Host-only: the work-list that dit_attn_varlen_fwd would run for this pack,
 * in execution order (paper Section 4.3: a batch mixes requests of different
 * lengths; the list balances their tiles over compute units by handing out the
 * costliest items first).  Needs no GPU and no context.
 *
 * Each item is one (sequence, head, query tile): 4 int32 values
 *     [0] q_start   first global query row of the tile
 *     [1] kv_start  first global key row (= start of the tile's sequence)
 *     [2] kv_len    number of keys (= length of the sequence)
 *     [3] (q_rows << 16) | head     q_rows in 1..block_m
 * Query tiles start at the sequence start (not at multiples of block_m of the
 * global row index), so a sequence's result does not depend on what it is
 * packed with.
 *
 *   items      HOST output buffer of capacity_items * 4 int32, may be NULL when
 *              capacity_items == 0 (to query the count).
 *   block_m    out: query rows per tile used for this head_dim.
 *   returns    the number of items (>= 0), or a negative error code;
 *              DIT_ATTN_ERR_CAPACITY if capacity_items > 0 is too small.
 */
int64_t dit_attn_plan(const int32_t* cu_seqlens, int32_t n_seqs,
                      int32_t n_heads, int32_t head_dim,
                      int32_t* items, int64_t capacity_items, int32_t* block_m);

/*
 * Host-only: the eviction policy of a context's cache of uploaded work-lists (at most 32 packs; paper Section 4.3:
 * dynamic batching produces many distinct packs over a serving run).  A forward call that is recorded into a HIP graph
 * pins its pack: the recorded launch reads the pack's device work-list (and, with split-KV, the context's workspace)
 * on every replay, so neither is freed before dit_attn_destroy; when every cached pack is pinned the cache grows
 * instead.  A call under capture for a pack that has no cached work-list yet (or whose split-KV workspace would have
 * to grow) returns DIT_ATTN_ERR_CAPTURE: call once outside the capture first.
 * Given last_use[i] (a use counter) and pinned[i] (non-zero: pinned) of n cached packs, returns the index the cache
 * evicts next: the least recently used unpinned one, or -1 if there is none (also for n < 0 or NULL arrays).
 */
int32_t dit_attn_plan_cache_victim(const uint64_t* last_use, const uint8_t* pinned, int32_t n);

/* Library version string, e.g. "dit_attn 0.1 gfx950". */
const char* dit_attn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DIT_ATTN_H_ */
