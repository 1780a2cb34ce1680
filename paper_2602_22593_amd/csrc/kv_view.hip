// Host side of the library: view resolution (paper Eq. 3, Eq. 4, Sec. 4.1.1), status strings,
// options, and the debugging table validator.  No kernels here.
#include <string.h>

#include <atomic>
#include <new>
#include <string>
#include <unordered_set>
#include <vector>

#include "kv_internal.h"

static thread_local std::string g_last_hip_error;

int kv_record_hip_error(hipError_t e, const char* what)
{
    if (e == hipSuccess) return KV_OK;
    g_last_hip_error = std::string(what) + ": " + hipGetErrorString(e);
    return KV_ERR_HIP;
}

static std::atomic<int64_t> g_chunk_tokens{0};
static std::atomic<int64_t> g_force_kernel{0};
static std::atomic<int64_t> g_waves_per_cu{0};
static std::atomic<int64_t> g_heads_per_wave{0};
static std::atomic<int64_t> g_merge_mode{0};
static std::atomic<int64_t> g_xcd_skew{-1};
static std::atomic<int64_t> g_piece_cost{-1};
static std::atomic<int64_t> g_linear_splits{0};

int64_t kv_option_chunk_tokens() { return g_chunk_tokens.load(); }
int64_t kv_option_force_kernel() { return g_force_kernel.load(); }
int64_t kv_option_waves_per_cu() { return g_waves_per_cu.load(); }
int64_t kv_option_heads_per_wave() { return g_heads_per_wave.load(); }
int64_t kv_option_merge_mode() { return g_merge_mode.load(); }
int64_t kv_option_xcd_skew() { return g_xcd_skew.load(); }
int64_t kv_option_piece_cost() { return g_piece_cost.load(); }
int64_t kv_option_linear_splits() { return g_linear_splits.load(); }

// ---- per-kernel event brackets -----------------------------------------------------------
namespace {
struct prof_kind {
    std::vector<hipEvent_t> begin, end;  // created lazily, reused
    size_t used = 0;
};
bool g_prof_on = false;
prof_kind g_prof[KV_PROF_KINDS];
constexpr size_t kProfMax = 4096;
}  // namespace

int kv_prof_begin(int which, hipStream_t st)
{
    if (!g_prof_on) return -1;
    prof_kind& k = g_prof[which];
    if (k.used >= kProfMax) return -1;
    if (k.used == k.begin.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return -1;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return -1; }
        k.begin.push_back(a);
        k.end.push_back(b);
    }
    const int slot = (int)k.used++;
    (void)hipEventRecord(k.begin[slot], st);
    return slot;
}

void kv_prof_end(int which, int slot, hipStream_t st)
{
    if (slot < 0) return;
    (void)hipEventRecord(g_prof[which].end[slot], st);
}

bool kv_prof_kernel_events(int which, hipEvent_t* start, hipEvent_t* stop)
{
    if (!g_prof_on) return false;
    prof_kind& k = g_prof[which];
    if (k.used >= kProfMax) return false;
    if (k.used == k.begin.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return false;
        if (hipEventCreate(&b) != hipSuccess) { (void)hipEventDestroy(a); return false; }
        k.begin.push_back(a);
        k.end.push_back(b);
    }
    const size_t slot = k.used++;
    *start = k.begin[slot];
    *stop = k.end[slot];
    return true;
}

extern "C" {

int kv_profile_enable(int on)
{
    g_prof_on = on != 0;
    if (g_prof_on)
        for (auto& k : g_prof) k.used = 0;
    return KV_OK;
}

int kv_profile_read(int which, double* total_ms, int64_t* n_launches)
{
    if (which < 0 || which >= KV_PROF_KINDS || !total_ms || !n_launches) return KV_ERR_INVALID_ARG;
    prof_kind& k = g_prof[which];
    double sum = 0.0;
    for (size_t i = 0; i < k.used; ++i) {
        hipError_t e = hipEventSynchronize(k.end[i]);
        if (e != hipSuccess) return kv_record_hip_error(e, "kv_profile_read sync");
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, k.begin[i], k.end[i]);
        if (e != hipSuccess) return kv_record_hip_error(e, "kv_profile_read elapsed");
        sum += ms;
    }
    *total_ms = sum;
    *n_launches = (int64_t)k.used;
    k.used = 0;
    return KV_OK;
}

int kv_view_create(const kv_geometry* g, int layout, int tp_degree, int rank, kv_view** out)
{
    if (!g || !out) return KV_ERR_INVALID_ARG;
    if (g->n_q_heads <= 0 || g->n_kv_heads <= 0 || g->head_dim <= 0 || g->base_block_size <= 0)
        return KV_ERR_INVALID_ARG;
    if (g->dtype != 0) return KV_ERR_UNSUPPORTED;
    if (g->head_dim % 8 != 0) return KV_ERR_INVALID_ARG;  // rows must be 16-byte multiples
    if (g->n_q_heads % g->n_kv_heads != 0) return KV_ERR_INVALID_ARG;
    if (layout != KV_LAYOUT_DP && layout != KV_LAYOUT_TP) return KV_ERR_INVALID_ARG;
    if (tp_degree < 1 || rank < 0 || rank >= tp_degree) return KV_ERR_INVALID_ARG;
    if (g->n_kv_heads % tp_degree != 0 || g->n_q_heads % tp_degree != 0) return KV_ERR_INVALID_ARG;
    // block capacity and byte size must stay inside 32-bit / 63-bit arithmetic
    const int64_t cap = (int64_t)g->base_block_size * tp_degree;
    const int64_t plane = (int64_t)g->base_block_size * g->n_kv_heads * g->head_dim;
    if (cap > (1 << 24) || plane > ((int64_t)1 << 40)) return KV_ERR_INVALID_ARG;

    kv_view* v = new (std::nothrow) kv_view;
    if (!v) return KV_ERR_INVALID_ARG;
    v->magic = KV_VIEW_MAGIC;
    v->geom = *g;
    v->layout = layout;
    v->p = tp_degree;
    v->r = rank;
    v->n_kv_local = g->n_kv_heads / tp_degree;          // H_req = H_base / N_eng
    v->n_q_local = g->n_q_heads / tp_degree;
    v->kv_head0 = rank * v->n_kv_local;
    v->group = g->n_q_heads / g->n_kv_heads;
    v->plane_elems = plane;
    v->block_bytes = 2 * plane * 2;
    if (layout == KV_LAYOUT_TP) {
        v->block_tokens = (int32_t)cap;                 // B_req = B_base * N_eng
        v->row_heads = v->n_kv_local;
        v->row_head0 = 0;
    } else {
        v->block_tokens = g->base_block_size;
        v->row_heads = g->n_kv_heads;
        v->row_head0 = v->kv_head0;
    }
    *out = v;
    return KV_OK;
}

void kv_view_destroy(kv_view* v)
{
    if (!kv_view_ok(v)) return;
    v->magic = 0;
    delete v;
}

int kv_view_query(const kv_view* v, int32_t* block_tokens, int32_t* n_kv_local, int32_t* n_q_local,
                  int32_t* kv_head0, int64_t* block_bytes)
{
    if (!kv_view_ok(v)) return KV_ERR_INVALID_ARG;
    if (block_tokens) *block_tokens = v->block_tokens;
    if (n_kv_local) *n_kv_local = v->n_kv_local;
    if (n_q_local) *n_q_local = v->n_q_local;
    if (kv_head0) *kv_head0 = v->kv_head0;
    if (block_bytes) *block_bytes = v->block_bytes;
    return KV_OK;
}

int kv_view_strides(const kv_view* v, int32_t* token_stride_elems, int32_t* row_heads,
                    int32_t* row_head0)
{
    if (!kv_view_ok(v)) return KV_ERR_INVALID_ARG;
    if (token_stride_elems) *token_stride_elems = v->row_heads * v->geom.head_dim;
    if (row_heads) *row_heads = v->row_heads;
    if (row_head0) *row_head0 = v->row_head0;
    return KV_OK;
}

int kv_set_option(const char* key, int64_t value)
{
    if (!key) return KV_ERR_INVALID_ARG;
    if (!strcmp(key, "chunk_tokens")) {
        if (value < 0 || (value % 64) != 0 || value > (1 << 20)) return KV_ERR_INVALID_ARG;
        g_chunk_tokens.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "force_kernel")) {
        if (value < 0 || value > 8) return KV_ERR_INVALID_ARG;
        g_force_kernel.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "heads_per_wave")) {
        if (value < 0 || value > 1) return KV_ERR_INVALID_ARG;
        g_heads_per_wave.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "merge_mode")) {
        if (value < 0 || value > 2) return KV_ERR_INVALID_ARG;
        g_merge_mode.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "linear_splits")) {
        if (value < 0 || value > 16) return KV_ERR_INVALID_ARG;
        g_linear_splits.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "piece_cost")) {
        if (value < -1 || value > 64) return KV_ERR_INVALID_ARG;
        g_piece_cost.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "xcd_skew")) {
        if (value < -1 || value > 256) return KV_ERR_INVALID_ARG;
        g_xcd_skew.store(value);
        return KV_OK;
    }
    if (!strcmp(key, "waves_per_cu")) {
        if (value < 0 || value > 32 || (value % 4) != 0) return KV_ERR_INVALID_ARG;
        g_waves_per_cu.store(value);
        return KV_OK;
    }
    return KV_ERR_INVALID_ARG;
}

int64_t kv_get_option(const char* key)
{
    if (!key) return -1;
    if (!strcmp(key, "chunk_tokens")) return g_chunk_tokens.load();
    if (!strcmp(key, "force_kernel")) return g_force_kernel.load();
    if (!strcmp(key, "waves_per_cu")) return g_waves_per_cu.load();
    if (!strcmp(key, "heads_per_wave")) return g_heads_per_wave.load();
    if (!strcmp(key, "merge_mode")) return g_merge_mode.load();
    if (!strcmp(key, "xcd_skew")) return g_xcd_skew.load();
    if (!strcmp(key, "piece_cost")) return g_piece_cost.load();
    if (!strcmp(key, "linear_splits")) return g_linear_splits.load();
    return -1;
}

const char* kv_strerror(int status)
{
    switch (status) {
        case KV_OK: return "ok";
        case KV_ERR_INVALID_ARG: return "invalid argument";
        case KV_ERR_UNSUPPORTED: return "unsupported configuration";
        case KV_ERR_WORKSPACE: return "workspace too small";
        case KV_ERR_HIP: return "HIP runtime error";
        case KV_ERR_RANGE: return "block id out of range";
        case KV_ERR_ALIAS: return "block used more than once";
        default: return "unknown status";
    }
}

const char* kv_last_hip_error(void) { return g_last_hip_error.c_str(); }

const char* kv_version(void) { return "flying-kv 0.1 (gfx950)"; }

// Copy a table and its lengths to the host and collect the block ids valid tokens need.
static int fetch_ids(const kv_view* v, const int32_t* table, int64_t stride, const int32_t* n_tokens,
                     int n_seqs, hipStream_t st, int64_t n_pool_blocks, std::vector<int32_t>& ids)
{
    std::vector<int32_t> lens((size_t)n_seqs);
    std::vector<int32_t> tab((size_t)n_seqs * (size_t)stride);
    hipError_t e = hipMemcpyAsync(lens.data(), n_tokens, lens.size() * 4, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return kv_record_hip_error(e, "kv_validate_tables copy lengths");
    e = hipMemcpyAsync(tab.data(), table, tab.size() * 4, hipMemcpyDeviceToHost, st);
    if (e != hipSuccess) return kv_record_hip_error(e, "kv_validate_tables copy table");
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return kv_record_hip_error(e, "kv_validate_tables sync");
    for (int s = 0; s < n_seqs; ++s) {
        if (lens[s] < 0) return KV_ERR_RANGE;
        const int64_t nb = ((int64_t)lens[s] + v->block_tokens - 1) / v->block_tokens;
        if (nb > stride) return KV_ERR_RANGE;
        for (int64_t j = 0; j < nb; ++j) {
            const int32_t id = tab[(size_t)s * stride + j];
            if (id < 0 || id >= n_pool_blocks) return KV_ERR_RANGE;
            ids.push_back(id);
        }
    }
    return KV_OK;
}

int kv_validate_tables(const kv_view* view, int64_t n_pool_blocks, const int32_t* block_table,
                       int64_t block_table_stride, const int32_t* n_tokens, int n_seqs,
                       const kv_view* other_view, const int32_t* other_table, int64_t other_stride,
                       void* hip_stream)
{
    if (!kv_view_ok(view) || !block_table || !n_tokens || n_seqs < 0 || block_table_stride < 0 ||
        n_pool_blocks < 0)
        return KV_ERR_INVALID_ARG;
    if (other_table && (!kv_view_ok(other_view) || other_stride < 0)) return KV_ERR_INVALID_ARG;
    if (n_seqs == 0) return KV_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    std::vector<int32_t> a, b;
    int rc = fetch_ids(view, block_table, block_table_stride, n_tokens, n_seqs, st, n_pool_blocks, a);
    if (rc) return rc;
    std::unordered_set<int32_t> seen;
    for (int32_t id : a)
        if (!seen.insert(id).second) return KV_ERR_ALIAS;
    if (other_table) {
        rc = fetch_ids(other_view, other_table, other_stride, n_tokens, n_seqs, st, n_pool_blocks, b);
        if (rc) return rc;
        std::unordered_set<int32_t> seen_b;
        for (int32_t id : b) {
            if (!seen_b.insert(id).second) return KV_ERR_ALIAS;
            if (seen.count(id)) return KV_ERR_ALIAS;
        }
    }
    return KV_OK;
}

}  // extern "C"
