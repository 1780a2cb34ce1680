// Internal definitions shared by the translation units of libflyingkv (never installed).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flying_kv.h"

#define KV_VIEW_MAGIC 0x4b565657u

// 16-byte register vector (four dwords), the unit of every KV load and store.
typedef uint32_t kv_u32x4 __attribute__((ext_vector_type(4)));

// Host-side resolved view (Eq. 3 / Eq. 4 of the paper and the head partition of Sec. 4.1.1).
struct kv_view {
    uint32_t magic;
    kv_geometry geom;
    int32_t layout, p, r;
    int32_t block_tokens;  // Bv: capacity of a block under this view
    int32_t row_heads;     // KV heads stored in one token row of a block
    int32_t n_kv_local;    // KV heads exposed
    int32_t n_q_local;     // query heads exposed
    int32_t kv_head0;      // first global KV head exposed
    int32_t row_head0;     // where that head sits in a token row
    int32_t group;         // G = n_q_heads / n_kv_heads
    int64_t plane_elems;   // base_block_size * n_kv_heads * head_dim
    int64_t block_bytes;   // 2 planes * plane_elems * sizeof(bf16)
};

// What a kernel needs to know about a view; passed by value as a kernel argument.
struct kv_view_dev {
    int32_t block_tokens;      // Bv
    int32_t block_shift;       // log2(Bv) if Bv is a power of two, else -1
    int32_t token_stride;      // elements between consecutive tokens of a block
    int32_t head_off;          // elements from the start of a token row to the first exposed head
    int32_t n_kv_local;
    int32_t n_q_local;
    int32_t head_dim;
    int32_t kv_head0;
    int64_t plane_elems;
    int64_t block_elems;       // 2 * plane_elems
};

static inline kv_view_dev kv_view_to_dev(const kv_view* v)
{
    kv_view_dev d;
    d.block_tokens = v->block_tokens;
    d.block_shift = -1;
    if ((v->block_tokens & (v->block_tokens - 1)) == 0) {
        int s = 0;
        while ((1 << s) < v->block_tokens) ++s;
        d.block_shift = s;
    }
    d.token_stride = v->row_heads * v->geom.head_dim;
    d.head_off = v->row_head0 * v->geom.head_dim;
    d.n_kv_local = v->n_kv_local;
    d.n_q_local = v->n_q_local;
    d.head_dim = v->geom.head_dim;
    d.kv_head0 = v->kv_head0;
    d.plane_elems = v->plane_elems;
    d.block_elems = 2 * v->plane_elems;
    return d;
}

static inline bool kv_view_ok(const kv_view* v) { return v && v->magic == KV_VIEW_MAGIC; }

// t -> (index into the block table row, slot inside the block)
__device__ __forceinline__ void kv_split_token(const kv_view_dev& v, int t, int& j, int& slot)
{
    if (v.block_shift >= 0) {
        j = t >> v.block_shift;
        slot = t & (v.block_tokens - 1);
    } else {
        j = t / v.block_tokens;
        slot = t - j * v.block_tokens;
    }
}

int kv_record_hip_error(hipError_t e, const char* what);

// Library-wide tunables (kv_set_option).
int64_t kv_option_chunk_tokens();
int64_t kv_option_force_kernel();
int64_t kv_option_waves_per_cu();
int64_t kv_option_heads_per_wave();  // 0: as many adjacent KV heads per wavefront as the shape allows; 1: always one
int64_t kv_option_merge_mode();      // 0: automatic; 1: pieces combined inside the main kernel; 2: by a second launch
int64_t kv_option_piece_cost();  // -1: library default; else 0..64 eighths of a tile
int64_t kv_option_xcd_skew();  // -1: library default; else 0..256 in 1/1024 of an even share
int64_t kv_option_linear_splits();

// Per-kernel event brackets for kv_profile_*: begin returns a slot (or -1 when disabled).
int kv_prof_begin(int which, hipStream_t st);
void kv_prof_end(int which, int slot, hipStream_t st);
// The same record filled by the launch itself: while profiling is on, hands out the two events of the
// next record, to be passed to hipExtLaunchKernelGGL, which stamps them with the kernel's own start
// and end (what a profiler reports as the kernel's duration; an event recorded on the stream before
// and after the launch also counts the dispatch).  False when profiling is off: launch normally.
bool kv_prof_kernel_events(int which, hipEvent_t* start, hipEvent_t* stop);

// ---- matrix-core decode kernel with an even split over resident wavefronts --------------------
#define KV_STREAMK_MAX_BATCH 2048
#define KV_MAX_MIXED_VIEWS 4
// The part of a view that may differ between the sequences of one batch: how the tokens of a
// sequence are laid out in its blocks.  Head counts and the head range are common to the batch.
struct kv_layout_dev {
    int32_t block_tokens, block_shift, token_stride, head_off;
};
struct kv_streamk_args {
    const uint16_t* q;
    uint16_t* out;
    const uint16_t* pool;
    const int32_t* table;
    int64_t table_stride;
    const int32_t* ctx_lens;
    kv_view_dev v;
    float scale_log2e;
    int32_t group;     // query heads per KV head
    int32_t batch;
    int32_t n_waves;   // wavefronts launched (multiple of 4)
    float* part_acc;   // [n_waves + batch * pairs][cols][128]
    float* part_ml;    // [n_waves + batch * pairs][cols][2]
    int32_t* pair_desc;   // [batch * pairs][2] numbers of the wavefronts holding a pair's first and last piece
                          // (read by the merge kernel; unused when the main kernel combines the pieces)
    unsigned long long* pair_sync;  // [batch * pairs] arrival words of the pairs, zero between calls
    int32_t fused;        // 1: the last piece of a pair to arrive combines them all (no merge kernel)
    const int32_t* view_ids;  // [batch] index into lay[] per sequence, or null: every sequence under v
    int32_t n_views;
    kv_layout_dev lay[KV_MAX_MIXED_VIEWS];
    // unit of the split, filled in by kv_streamk_launch: a pair is (sequence, `heads_per_wave`
    // adjacent local KV heads), a tile 2^tile_shift tokens of a pair
    int32_t heads_per_wave;  // 1, 2 or 4
    int32_t pairs;           // pairs per sequence = n_kv_local / heads_per_wave
    int32_t cols;            // output rows per pair = heads_per_wave * group (<= 16)
    int32_t tile_shift;      // 5 (one head), 4 (two heads) or 3 (four heads)
    uint32_t wt_prefix[9];   // wt_prefix[x] = summed weight of XCDs < x; a wavefront's share of the tiles
                             // is proportional to the weight of the XCD its workgroup runs on
    double inv_weight;       // 1 / (summed weight of all wavefronts)
    int32_t piece_units;     // weight of the start of a pair on the axis that is cut, a tile weighing 8
};
// Bytes at the start of every decode workspace that hold the arrival words: zero before the first
// call on a workspace, and zero again when a call has finished.
#define KV_DECODE_SYNC_WORDS (KV_DECODE_SYNC_BYTES / 8)
size_t kv_streamk_workspace_bytes(const kv_view* view, int batch, int n_waves);
int kv_streamk_launch(kv_streamk_args a, const kv_view* view, void* workspace, hipStream_t st);
