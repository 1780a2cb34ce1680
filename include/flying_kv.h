/*
 * flying_kv.h -- C ABI of the MI355X (gfx950) paged decode attention / KV repack library.
 *
 * The library implements the device side of the paper's KV Cache Adaptor (Sec. 4.2): one
 * physical pool of constant-size KV blocks that is read either as a DP replica's blocks
 * (all KV heads, B_base tokens per block) or as one TP rank's blocks (H/p heads,
 * p * B_base tokens per block); the kernels receive each request's token stride and block
 * capacity (Sec. 4.2.3).  On top of that contract it provides the decode
 * attention kernel, a block repack kernel for the transitions where bytes must move (the
 * paper recomputes the cache there, Sec. 5.2.2), and the KV append kernel.
 *
 * Conventions
 *   - Every function returns 0 (KV_OK) or a negative kv_status.  Nothing throws, nothing
 *     synchronises the stream, nothing allocates device memory (kv_validate_tables, a
 *     debugging aid, is the one exception to the first two).
 *   - "device" pointers are HIP device memory owned by the caller; "host" pointers are
 *     ordinary host memory.  The library owns only kv_view objects (host).
 *   - bf16 everywhere in memory; all accumulation is fp32 on the device.
 *   - Physical layout of the pool: n_pool_blocks blocks of block_bytes each.  A block read
 *     under a view with capacity Bv (tokens) and Hrow KV heads per token row is the array
 *         bf16 [2 (0 = K, 1 = V)] [Bv] [Hrow] [head_dim]
 *     and Bv * Hrow = base_block_size * n_kv_heads for every view, so block_bytes
 *     = 2 * base_block_size * n_kv_heads * head_dim * 2 never changes (Eq. 2 held constant).
 *   - Token t of sequence s lives in block block_table[s][t / Bv], slot t % Bv.
 *   - Calls may be issued from several host threads and on several streams at once as long as
 *     calls that share a workspace (or write the same blocks or rows) are ordered by the caller,
 *     on one stream or by events: the library keeps nothing between calls except the
 *     process-wide options, the calling thread's last HIP error text and the measurement
 *     records below.
 */
#ifndef FLYING_KV_H
#define FLYING_KV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    KV_OK = 0,
    KV_ERR_INVALID_ARG = -1, /* null pointer, negative size, impossible view parameters      */
    KV_ERR_UNSUPPORTED = -2, /* valid in principle, not built (dtype, head_dim, group size)   */
    KV_ERR_WORKSPACE = -3,   /* workspace smaller than paged_decode_attn_workspace_bytes()   */
    KV_ERR_HIP = -4,         /* a HIP call or kernel launch failed; see kv_last_hip_error()   */
    KV_ERR_RANGE = -5,       /* kv_validate_tables: block id outside [0, n_pool_blocks)       */
    KV_ERR_ALIAS = -6        /* kv_validate_tables: a block appears twice / src meets dst     */
} kv_status;

/* Model-side constants (Alg. 1 "Require": B_base, H_base) plus the attention shape. */
typedef struct {
    int32_t n_q_heads;       /* total query heads of the layer (before any TP split)          */
    int32_t n_kv_heads;      /* total KV heads H_base                                          */
    int32_t head_dim;        /* elements per head; supported: 64, 128                          */
    int32_t base_block_size; /* B_base: tokens per block in DP mode                            */
    int32_t dtype;           /* 0 = bf16 (the only one)                                        */
} kv_geometry;

/* How the rows of a block are physically arranged. */
typedef enum {
    KV_LAYOUT_DP = 0, /* [B_base tokens][all H_base heads][d]                                  */
    KV_LAYOUT_TP = 1  /* [p * B_base tokens][H_base / p heads][d]  (Eq. 3, Eq. 4)              */
} kv_layout;

typedef struct kv_view kv_view; /* opaque, immutable, host memory */

/*
 * kv_view_create -- resolve (layout, tp_degree p, rank r) over a geometry (Eq. 3:
 * B(p) = p * B_base; Alg. 1 step 4 / Eq. 4: H_req = H_base / N_eng; Sec. 4.1.1: rank r owns
 * the r-th contiguous slice of heads, KV heads [r*H/p, (r+1)*H/p) and the query heads of
 * those groups).
 *   KV_LAYOUT_DP, p = 1, r = 0 : the DP replica view, all heads.
 *   KV_LAYOUT_TP, p, r         : rank r's blocks in the TP arrangement.
 *   KV_LAYOUT_DP, p > 1, r     : rank r's head slice read in place from DP-arranged blocks
 *                                (strided rows, no bytes moved).
 * Errors: KV_ERR_INVALID_ARG for null pointers, p < 1, r outside [0, p), p not dividing
 * n_kv_heads or n_q_heads, n_kv_heads not dividing n_q_heads, non-positive sizes, head_dim
 * not a multiple of 8, unknown layout; KV_ERR_UNSUPPORTED for dtype != 0.
 * *out is written only on success; release it with kv_view_destroy.
 */
int kv_view_create(const kv_geometry* geometry, int layout, int tp_degree, int rank,
                   kv_view** out);
void kv_view_destroy(kv_view* view);

/*
 * kv_view_query -- read back what the view resolved to.  Any output pointer may be null.
 * block_tokens = B(p) (capacity), n_kv_local = KV heads exposed, n_q_local = query heads
 * exposed, kv_head0 = first global KV head exposed, block_bytes = constant block size.
 */
int kv_view_query(const kv_view* view, int32_t* block_tokens, int32_t* n_kv_local,
                  int32_t* n_q_local, int32_t* kv_head0, int64_t* block_bytes);

/*
 * kv_view_strides -- the "stride" half of the per-request kernel parameters (Sec. 4.2.3):
 * elements between consecutive tokens of a block (row_heads * head_dim), KV heads stored
 * per token row, and the position of the first exposed head inside a row.
 */
int kv_view_strides(const kv_view* view, int32_t* token_stride_elems, int32_t* row_heads,
                    int32_t* row_head0);

/*
 * paged_decode_attn -- one decode step of attention for a batch (Sec. 2.1: attention over
 * the cached keys and values; Sec. 4.2.2: KV blocks found through the logical table):
 *     out[s][i][:] = sum_t softmax_t(scale * q[s][i] . K[s][t][i / G]) * V[s][t][i / G]
 * for t in [0, ctx_lens[s]), local query head i in [0, n_q_local), G = n_q_heads /
 * n_kv_heads.  No mask other than t < ctx_lens[s].
 *
 *   q            device, bf16 [batch][n_q_local][head_dim]     (read)
 *   out          device, bf16 [batch][n_q_local][head_dim]     (written; rows with
 *                ctx_lens[s] == 0 are written as zeros)
 *   kv_pool      device, the block pool described above         (read only)
 *   n_pool_blocks  number of blocks in the pool (host check of sizes only)
 *   block_table  device, int32 [batch][block_table_stride]; entries at index >=
 *                ceil(ctx_lens[s] / block_tokens) are never read for effect (may be -1)
 *   ctx_lens     device, int32 [batch], each in [0, max_ctx_len]
 *   max_ctx_len  host upper bound of ctx_lens (sizes the launch; a larger bound is legal,
 *                a smaller one makes the result undefined)
 *   scale        softmax scale; <= 0 selects 1 / sqrt(head_dim)
 *   workspace    device scratch of at least paged_decode_attn_workspace_bytes(view, batch,
 *                max_ctx_len) bytes, 256-byte aligned.  Its first KV_DECODE_SYNC_BYTES hold the
 *                arrival words through which the wavefronts that share a long sequence find
 *                out which of them finishes it: they must be ZERO when the workspace is first
 *                used (one hipMemsetAsync after allocating it) and every call leaves them zero
 *                again, so one workspace serves any sequence of calls, of any shapes and views.
 *                The rest need not be initialised; all of it is undefined while a call runs.
 *                A workspace whose first bytes are not zero gives undefined output rows.
 *   hip_stream   hipStream_t to launch on (null = default stream)
 *
 * Block ids inside [0, n_pool_blocks) for every valid token are a precondition (not
 * checked on the hot path; see kv_validate_tables).
 * Errors: KV_ERR_INVALID_ARG (null pointers, negative sizes, block_table_stride too small
 * for max_ctx_len), KV_ERR_UNSUPPORTED (head_dim or group size without a kernel),
 * KV_ERR_WORKSPACE, KV_ERR_HIP.
 */
#define KV_DECODE_SYNC_BYTES (16384 * 8)
size_t paged_decode_attn_workspace_bytes(const kv_view* view, int batch, int max_ctx_len);
int paged_decode_attn(const void* q, void* out, const void* kv_pool, int64_t n_pool_blocks,
                      const int32_t* block_table, int64_t block_table_stride,
                      const int32_t* ctx_lens, int batch, int max_ctx_len,
                      const kv_view* view, float scale, void* workspace,
                      size_t workspace_bytes, void* hip_stream);

/*
 * paged_decode_attn_mixed -- paged_decode_attn for a batch whose sequences do not all keep
 * their KV in the same block layout (Sec. 5.2.3: blocks written under different parallelism
 * modes coexist in one pool; Sec. 4.2.3: the kernels are told each request's stride and block
 * capacity).  Sequence s is read under views[view_ids[s]].  The result is the one
 * paged_decode_attn defines, sequence by sequence, under that sequence's view.
 *
 * Every view must have the geometry, TP degree p and rank r of views[0]: the batch runs on one
 * rank, so all sequences expose the same heads (q, out: [batch][n_q_local][head_dim] as above)
 * and the views differ only in layout -- e.g. views[0] = (TP, p, r) for requests admitted in TP
 * mode and views[1] = (DP, p, r), the same head slice read in place from blocks a DP engine
 * wrote, for requests taken over without a repack.
 *
 *   view_ids     device, int32 [batch], each in [0, n_views) (values outside are clamped)
 *   views        host array of n_views views, 1 <= n_views <= 4
 *   block_table  row s is indexed with the block capacity of sequence s's view;
 *                block_table_stride must cover max_ctx_len under the smallest capacity
 *   workspace    at least paged_decode_attn_workspace_bytes(views[0], batch, max_ctx_len)
 * Other arguments and errors as paged_decode_attn; in addition KV_ERR_INVALID_ARG for views
 * that disagree in geometry, p or r, and KV_ERR_UNSUPPORTED when n_views > 1 and the shape is
 * not served by the matrix-core kernel (head_dim 128, group <= 16, batch <= 2048).
 */
int paged_decode_attn_mixed(const void* q, void* out, const void* kv_pool, int64_t n_pool_blocks,
                            const int32_t* block_table, int64_t block_table_stride,
                            const int32_t* ctx_lens, const int32_t* view_ids, int batch,
                            int max_ctx_len, const kv_view* const* views, int n_views, float scale,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * paged_decode_attn_static -- paged_decode_attn for callers that cannot allocate device memory or
 * carry a workspace: code running under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, result and errors as paged_decode_attn, without the
 * workspace: the scratch memory of the kernels is a fixed device array of
 * KV_STATIC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds until
 * the process ends.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine); the first call on a device looks the array's address up once (hipGetSymbolAddress),
 * so make that first call outside any stream capture.
 *   KV_ERR_WORKSPACE   paged_decode_attn_workspace_bytes(view, batch, max_ctx_len) exceeds
 *                      KV_STATIC_SCRATCH_BYTES (with the default options the array serves e.g. 1024
 *                      sequences under the 8B-shaped DP view, 32 local query heads, and 2048 under
 *                      its TP4 or TP8 rank views); nothing is launched
 *   KV_ERR_UNSUPPORTED also for a device ordinal of 64 or more
 * All calls on one GPU share that GPU's array: calls that may overlap there (different streams
 * without an ordering between them, several host threads) race on it and give undefined results;
 * order them on one stream or by events.  The array keeps the previous call's contents: its
 * arrival words start out zero (the array is zero when the library is loaded) and every call puts
 * them back to zero; every other word a call reads is written earlier in that call, so nothing
 * needs clearing between calls.  (The measurement aid kv_profile_enable creates events while it
 * is on; leave it off.)
 */
#define KV_STATIC_SCRATCH_BYTES (32u << 20)
int paged_decode_attn_static(const void* q, void* out, const void* kv_pool, int64_t n_pool_blocks,
                             const int32_t* block_table, int64_t block_table_stride,
                             const int32_t* ctx_lens, int batch, int max_ctx_len,
                             const kv_view* view, float scale, void* hip_stream);

/*
 * paged_prefill_attn -- causal attention from several new tokens per sequence to everything
 * cached up to each of them, through a view: one chunk of a prefill (Sec. 2.1; chunked prefill
 * is kept, Sec. 3) or the recompute step of Soft Preempt (Sec. 5.2.2).  The new tokens' K and V
 * are already in the pool (kv_append).  Sequence s has ctx_lens[s] cached tokens, the last
 * q_len[s] = q_offsets[s + 1] - q_offsets[s] of which are the new ones; for its j-th new token,
 * at position pos = ctx_lens[s] - q_len[s] + j, and local query head i:
 *     out[q_offsets[s] + j][i][:] = sum_{t <= pos} softmax_t(scale * q[..][i] . K[s][t][i / G]) V[s][t][i / G]
 *
 *   q, out       device, bf16 [total_q][n_q_local][head_dim], total_q = q_offsets[batch]
 *   q_offsets    device, int32 [batch + 1], non-decreasing, q_offsets[0] = 0
 *   ctx_lens     device, int32 [batch]; q_len[s] <= ctx_lens[s] <= max_ctx_len is a precondition
 *   total_q      q_offsets[batch], known to the host (the number of rows of q and out)
 *   max_q_len    host upper bound of q_len (sizes the launch)
 *   workspace    device scratch of at least paged_prefill_attn_workspace_bytes(...) bytes (0 when
 *                the launch fills the chip without splitting the key range: null is then
 *                accepted), 256-byte aligned; contents need not be initialised
 * Other arguments as paged_decode_attn.  q_len[s] = 1 for every s is paged_decode_attn.  Errors: KV_ERR_INVALID_ARG (null pointers, negative sizes, max_q_len >
 * max_ctx_len, block_table_stride too small), KV_ERR_UNSUPPORTED (head_dim != 128, group size
 * above 16, block capacity not a multiple of 16), KV_ERR_WORKSPACE, KV_ERR_HIP.
 */
size_t paged_prefill_attn_workspace_bytes(const kv_view* view, int batch, int64_t total_q,
                                          int max_ctx_len, int max_q_len);
int paged_prefill_attn(const void* q, void* out, const void* kv_pool, int64_t n_pool_blocks,
                       const int32_t* block_table, int64_t block_table_stride,
                       const int32_t* ctx_lens, const int32_t* q_offsets, int batch, int64_t total_q,
                       int max_ctx_len, int max_q_len, const kv_view* view, float scale,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Weight shard views (Model Weights Manager, Sec. 4.1; Eq. 1: W_active^(r) = View(W_full, dim, r,
 * m)).  A weight is stored once, whole, as bf16 [out_features][in_features] row-major; a view
 * names the stored rows (up to three contiguous segments, concatenated) and the contiguous range
 * of stored columns that are active for rank r of an m-way TP group.  Plain host data: the
 * caller owns it, nothing on the device is touched or copied.
 */
typedef struct kv_weight_view {
    int32_t n_segments;      /* 1..3 */
    int64_t row_start[3];    /* first stored row of each segment */
    int64_t row_count[3];
    int64_t col_start;
    int64_t col_count;
} kv_weight_view;

/* The r-th of m equal parts along dim (0: stored rows = output features, the column-parallel
 * layer of Sec. 4.1.1; 1: stored columns = input features, the row-parallel layer).
 * KV_ERR_INVALID_ARG if r is not in [0, m) or the dimension is not divisible by m. */
int kv_weight_view_make(int dim, int r, int m, int64_t n_rows, int64_t n_cols, kv_weight_view* out);

/* Rank r's slice of a fused QKV weight [(n_q_heads + 2 n_kv_heads) * head_dim][hidden] (query
 * heads, then key heads, then value heads): three row segments holding the rank's contiguous
 * head range of each part (Sec. 4.1.1).  KV_ERR_INVALID_ARG if m does not divide the head counts. */
int kv_weight_view_fused_qkv(const kv_geometry* g, int64_t hidden, int r, int m, kv_weight_view* out);

/*
 * kv_linear_view -- y = x W_active^T on the view, reading the full weight in place.
 *   x       device, bf16 [M][view->col_count], row stride ldx elements          (read)
 *   w_full  device, bf16 [w_rows][ldw]: the whole stored weight, ldw its row length (read)
 *   y       device, bf16 [M][sum of row_count], row stride ldy elements          (written)
 *   workspace device scratch of at least kv_linear_view_workspace_bytes(view, M) bytes (may be
 *           0: then null is accepted), 16-byte aligned; contents need not be initialised
 * fp32 accumulation, one rounding to bf16 at the end.  For the row-parallel layer y is the
 * rank's partial sum (the all-reduce over ranks is the caller's).  Tuned for decode batches (M up
 * to a few hundred); any M is accepted.
 * Errors: KV_ERR_INVALID_ARG (null pointers, view outside the weight, strides too small),
 * KV_ERR_WORKSPACE,
 * KV_ERR_UNSUPPORTED (col_count not a multiple of 128, a row segment not a multiple of 64,
 * col_start / ldx / ldw not multiples of 8 elements, ldy not a multiple of 4, pointers not
 * 16-byte aligned), KV_ERR_HIP.
 */
size_t kv_linear_view_workspace_bytes(const kv_weight_view* view, int M);
int kv_linear_view(const void* x, int64_t ldx, const void* w_full, int64_t w_rows, int64_t ldw,
                   const kv_weight_view* view, void* y, int64_t ldy, int M, void* workspace,
                   size_t workspace_bytes, void* hip_stream);

/*
 * kv_repack -- move KV rows between two arrangements inside one pool, bit-exactly.  This
 * is what a DP->TP or TP->DP transition needs when the existing blocks cannot simply be
 * re-interpreted (the paper's Soft Preempt recomputes the cache instead, Sec. 5.2.2; a
 * group dissolved under load, Sec. 2.3 use case 1, needs the reverse direction).
 * For every sequence s, token t < n_tokens[s], plane (K, V) and every global KV head
 * exposed by BOTH views, the head_dim-element row is copied from its address under
 * src_view (through src_block_table) to its address under dst_view (through
 * dst_block_table).  Every other byte of the pool keeps its value.
 *
 *   kv_pool          device, read and written
 *   src_block_table  device, int32 [n_seqs][src_stride]
 *   dst_block_table  device, int32 [n_seqs][dst_stride]
 *   n_tokens         device, int32 [n_seqs], each in [0, max_tokens]
 *   max_tokens       host upper bound of n_tokens (sizes the launch)
 *
 * Preconditions (not checked on the hot path): block ids in range; the source and the
 * destination block sets are disjoint (an in-place repack is not defined).
 * Errors: KV_ERR_INVALID_ARG (null pointers, negative sizes, views over different
 * geometries, strides too small for max_tokens), KV_ERR_HIP.
 */
int kv_repack(void* kv_pool, int64_t n_pool_blocks, const kv_view* src_view,
              const kv_view* dst_view, const int32_t* src_block_table, int64_t src_stride,
              const int32_t* dst_block_table, int64_t dst_stride, const int32_t* n_tokens,
              int n_seqs, int max_tokens, void* hip_stream);

/*
 * kv_append -- the "KV cache kernel" of Sec. 4.2.3: write the new token's K and V rows of
 * every sequence into the pool at position positions[s] (normally the current context
 * length), using the view's stride and capacity.
 *
 *   k_new, v_new  device, bf16 [n_seqs][n_kv_local][head_dim]
 *   positions     device, int32 [n_seqs]; a negative position skips the sequence
 * Errors: KV_ERR_INVALID_ARG, KV_ERR_HIP.
 */
int kv_append(void* kv_pool, int64_t n_pool_blocks, const kv_view* view, const void* k_new,
              const void* v_new, const int32_t* block_table, int64_t block_table_stride,
              const int32_t* positions, int n_seqs, void* hip_stream);

/*
 * kv_validate_tables -- debugging aid, NOT for the hot path: copies the tables to the host
 * (synchronises the stream) and checks that every block id a valid token needs lies in
 * [0, n_pool_blocks) (KV_ERR_RANGE) and that no block is used twice within the table
 * (KV_ERR_ALIAS).  With other_table != null also checks that the two tables share no
 * block (repack precondition).  other_* describe the second table under other_view.
 */
int kv_validate_tables(const kv_view* view, int64_t n_pool_blocks, const int32_t* block_table,
                       int64_t block_table_stride, const int32_t* n_tokens, int n_seqs,
                       const kv_view* other_view, const int32_t* other_table,
                       int64_t other_stride, void* hip_stream);

/* Test and tuning hooks.  Process-wide and NOT synchronised with calls in flight: set them from one
 * thread while no other thread is inside the library, e.g. before serving starts or inside a test.
 * A call reads each option once, when it is issued (a captured HIP graph keeps what it was
 * captured with).  0 = automatic unless stated otherwise.
 *   "chunk_tokens"   split-KV granularity of the chunked decode kernels, a multiple of 64
 *   "force_kernel"   decode kernel: 1 even split over resident wavefronts, 2 vector ALU, 3 chunked
 *                    matrix-core (KV_ERR_UNSUPPORTED from the call if the shape is not served)
 *   "waves_per_cu"   wavefronts per compute unit launched by the even-split kernel, a multiple of 4.
 *                    paged_decode_attn_workspace_bytes follows "force_kernel", "waves_per_cu" and
 *                    "chunk_tokens": size the workspace after setting them
 *   "heads_per_wave" 1: one KV head per wavefront even where several adjacent heads are possible
 *   "merge_mode"     how the pieces of a sequence cut over several wavefronts are combined:
 *                    1 inside the main kernel by the last piece to arrive, 2 by a second launch
 *   "xcd_skew"       even-split decode kernels: share moved from each odd-numbered to each even-numbered
 *                    XCD, in 1/1024 of an even share (0..256; -1 = the library's default)
 *   "piece_cost"     even-split decode kernels: what the start of a (sequence, head group) pair counts
 *                    for when the work is cut over the wavefronts, in eighths of a 16 KiB tile
 *                    (0..64; -1 = the library's default, 16)
 *   "linear_splits"  kv_linear_view cuts the input dimension into at least this many slices (1..16;
 *                    a slice is never longer than 1024 input features nor shorter than 128);
 *                    kv_linear_view_workspace_bytes follows the option, so size the workspace after
 *                    setting it
 * Returns KV_ERR_INVALID_ARG for an unknown key or an illegal value. */
int kv_set_option(const char* key, int64_t value);
int64_t kv_get_option(const char* key);

/*
 * Measurement aid (not part of the method).  While enabled, the entry points time their kernels
 * with HIP events on the caller's stream, so that a benchmark can read per-kernel durations
 * without an external profiler: the even-split decode kernels are launched with events that
 * take the kernel's own start and end times (hipExtLaunchKernelGGL; what a profiler reports),
 * the other kernels are bracketed by events recorded before and after the launch (which also
 * counts the dispatch, 2-3 us; the two kernels of paged_prefill_attn and of kv_linear_view
 * share one bracket).
 *   kv_profile_enable(on)  : 1 = start recording (drops earlier records), 0 = stop.
 *   kv_profile_read(which, &total_ms, &n) : synchronises on the recorded events, returns the
 *       summed duration and the number of launches of kernel `which` since enabling, and
 *       clears them.  which: 0 = decode main kernel, 1 = decode merge kernel, 2 = repack kernel.
 * Not thread-safe; at most 4096 launches per kernel are kept between reads.  Leave it off while a
 * HIP graph is being captured on the stream (event records are not part of the method's work).
 */
enum { KV_PROF_DECODE_MAIN = 0, KV_PROF_DECODE_MERGE = 1, KV_PROF_REPACK = 2, KV_PROF_PREFILL = 3,
       KV_PROF_LINEAR = 4, KV_PROF_KINDS = 5 };
int kv_profile_enable(int on);
int kv_profile_read(int which, double* total_ms, int64_t* n_launches);

/*
 * Streaming kernels of known traffic (measurement aids, not part of the method): read `bytes`
 * once (kv_probe_read) or copy them once (kv_probe_copy) with n_workgroups workgroups of 256
 * lanes, 16 bytes per lane per access.  They give the achievable HBM rate on the box and the
 * reference against which profiler byte counters are scaled.  src/dst/sink are device
 * pointers, bytes a multiple of 16; sink may be null.
 */
int kv_probe_read(const void* src, size_t bytes, void* sink, int n_workgroups, void* hip_stream);
int kv_probe_copy(void* dst, const void* src, size_t bytes, int n_workgroups, void* hip_stream);
/* Same read, but of whole pool blocks in the order of block_ids (device, int32[n_ids]): the
 * ceiling of a paged pool's access pattern, with no arithmetic on the data. */
int kv_probe_read_blocks(const void* pool, const int32_t* block_ids, int n_ids, int64_t block_bytes,
                         void* sink, int n_workgroups, void* hip_stream);

/* Placement probe: workgroup g reads the g-th of n_workgroups equal contiguous shares of `bytes`
 * (the shares are rounded down to whole 16-byte pieces per wavefront) and writes three int64 values
 * to records[3 g ..] (device): the XCD it ran on (hardware register XCC_ID), and its start and end
 * times in ticks of the 100 MHz constant-rate counter.  Shows how workgroup indices map to XCDs and
 * whether the XCDs stream at the same rate. */
int kv_probe_read_placed(const void* src, size_t bytes, int64_t* records, void* sink, int n_workgroups,
                         void* hip_stream);

const char* kv_strerror(int status);   /* static string, never null */
const char* kv_last_hip_error(void);   /* text of the last HIP failure seen by this thread */
const char* kv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLYING_KV_H */
