// kv_repack and kv_append: byte-exact movement of KV rows between / into pool blocks under
// layout views.  Pure integer and 16-byte copy work, bound by HBM read + write bandwidth.
//
// A token's rows for a run of consecutive KV heads are contiguous in every arrangement
// (a block is [plane][token][head][d]), so the unit of work is one 16-byte piece of such a
// run: consecutive lanes take consecutive pieces, a wavefront covers whole 256-byte rows.
#include "kv_internal.h"

namespace {

constexpr int kRepackThreads = 256;
constexpr int kRepackUnroll = 4;

struct repack_args {
    kv_view_dev src, dst;
    int32_t src_run_off;   // elements from the start of a src token row to the first common head
    int32_t dst_run_off;   // same for dst
    int32_t run_chunks;    // 16-byte pieces in one token's run of common heads (one plane)
    int32_t run_shift;     // log2(run_chunks) or -1
    int32_t tokens_per_wg;
};

__device__ __forceinline__ int64_t token_base(const kv_view_dev& v, const int32_t* __restrict__ row,
                                              int t)
{
    int j, slot;
    kv_split_token(v, t, j, slot);
    return (int64_t)row[j] * v.block_elems + (int64_t)slot * v.token_stride;
}

__global__ __launch_bounds__(kRepackThreads) void kv_repack_kernel(
    uint16_t* __restrict__ pool, const int32_t* __restrict__ src_tab, int64_t src_stride,
    const int32_t* __restrict__ dst_tab, int64_t dst_stride, const int32_t* __restrict__ n_tokens,
    repack_args a)
{
    const int s = blockIdx.y;
    const int n = n_tokens[s];
    const int t0 = blockIdx.x * a.tokens_per_wg;
    if (t0 >= n) return;
    const int t1 = min(n, t0 + a.tokens_per_wg);
    const int32_t* srow = src_tab + (int64_t)s * src_stride;
    const int32_t* drow = dst_tab + (int64_t)s * dst_stride;
    const int per_tok = 2 * a.run_chunks;  // both planes
    const int total = (t1 - t0) * per_tok;

    for (int base = threadIdx.x; base < total; base += kRepackThreads * kRepackUnroll) {
        kv_u32x4 val[kRepackUnroll];
        int64_t dst_elem[kRepackUnroll];
#pragma unroll
        for (int u = 0; u < kRepackUnroll; ++u) {
            const int idx = base + u * kRepackThreads;
            dst_elem[u] = -1;
            if (idx < total) {
                int tt, rem, plane, c;
                if (a.run_shift >= 0) {
                    tt = idx >> (a.run_shift + 1);
                    rem = idx & (per_tok - 1);
                    plane = rem >> a.run_shift;
                    c = rem & (a.run_chunks - 1);
                } else {
                    tt = idx / per_tok;
                    rem = idx - tt * per_tok;
                    plane = rem / a.run_chunks;
                    c = rem - plane * a.run_chunks;
                }
                const int t = t0 + tt;
                const int64_t se = token_base(a.src, srow, t) + (int64_t)plane * a.src.plane_elems +
                                   a.src_run_off + c * 8;
                dst_elem[u] = token_base(a.dst, drow, t) + (int64_t)plane * a.dst.plane_elems +
                              a.dst_run_off + c * 8;
                val[u] = __builtin_nontemporal_load(reinterpret_cast<const kv_u32x4*>(pool + se));
            }
        }
#pragma unroll
        for (int u = 0; u < kRepackUnroll; ++u) {
            if (dst_elem[u] >= 0)
                __builtin_nontemporal_store(val[u], reinterpret_cast<kv_u32x4*>(pool + dst_elem[u]));
        }
    }
}

// One workgroup per sequence: lanes cover (plane, local head, 16-byte piece) of the new row.
__global__ __launch_bounds__(256) void kv_append_kernel(
    uint16_t* __restrict__ pool, const uint16_t* __restrict__ k_new,
    const uint16_t* __restrict__ v_new, const int32_t* __restrict__ table, int64_t stride,
    const int32_t* __restrict__ positions, kv_view_dev v)
{
    const int s = blockIdx.x;
    const int pos = positions[s];
    if (pos < 0) return;
    const int row_chunks = v.n_kv_local * v.head_dim / 8;
    const int64_t base = token_base(v, table + (int64_t)s * stride, pos) + v.head_off;
    for (int idx = threadIdx.x; idx < 2 * row_chunks; idx += blockDim.x) {
        const int plane = idx / row_chunks;
        const int c = idx - plane * row_chunks;
        const uint16_t* src = (plane ? v_new : k_new) + (int64_t)s * row_chunks * 8 + c * 8;
        *reinterpret_cast<uint4*>(pool + base + (int64_t)plane * v.plane_elems + c * 8) =
            *reinterpret_cast<const uint4*>(src);
    }
}

bool same_geometry(const kv_view* a, const kv_view* b)
{
    return a->geom.n_q_heads == b->geom.n_q_heads && a->geom.n_kv_heads == b->geom.n_kv_heads &&
           a->geom.head_dim == b->geom.head_dim &&
           a->geom.base_block_size == b->geom.base_block_size && a->geom.dtype == b->geom.dtype;
}

}  // namespace

extern "C" int kv_repack(void* kv_pool, int64_t n_pool_blocks, const kv_view* src_view,
                         const kv_view* dst_view, const int32_t* src_block_table,
                         int64_t src_stride, const int32_t* dst_block_table, int64_t dst_stride,
                         const int32_t* n_tokens, int n_seqs, int max_tokens, void* hip_stream)
{
    if (!kv_view_ok(src_view) || !kv_view_ok(dst_view)) return KV_ERR_INVALID_ARG;
    if (!same_geometry(src_view, dst_view)) return KV_ERR_INVALID_ARG;
    if (n_seqs < 0 || max_tokens < 0 || n_pool_blocks < 0 || src_stride < 0 || dst_stride < 0)
        return KV_ERR_INVALID_ARG;
    if (n_seqs == 0 || max_tokens == 0) return KV_OK;
    if (!kv_pool || !src_block_table || !dst_block_table || !n_tokens) return KV_ERR_INVALID_ARG;
    const int64_t need_src = ((int64_t)max_tokens + src_view->block_tokens - 1) / src_view->block_tokens;
    const int64_t need_dst = ((int64_t)max_tokens + dst_view->block_tokens - 1) / dst_view->block_tokens;
    if (src_stride < need_src || dst_stride < need_dst) return KV_ERR_INVALID_ARG;

    // heads exposed by both views: [g_lo, g_hi)
    const int g_lo = src_view->kv_head0 > dst_view->kv_head0 ? src_view->kv_head0 : dst_view->kv_head0;
    const int s_hi = src_view->kv_head0 + src_view->n_kv_local;
    const int d_hi = dst_view->kv_head0 + dst_view->n_kv_local;
    const int g_hi = s_hi < d_hi ? s_hi : d_hi;
    if (g_hi <= g_lo) return KV_OK;  // nothing in common: nothing moves

    const int d = src_view->geom.head_dim;
    repack_args a;
    a.src = kv_view_to_dev(src_view);
    a.dst = kv_view_to_dev(dst_view);
    a.src_run_off = (src_view->row_head0 + (g_lo - src_view->kv_head0)) * d;
    a.dst_run_off = (dst_view->row_head0 + (g_lo - dst_view->kv_head0)) * d;
    a.run_chunks = (g_hi - g_lo) * d / 8;
    a.run_shift = -1;
    if ((a.run_chunks & (a.run_chunks - 1)) == 0) {
        int sh = 0;
        while ((1 << sh) < a.run_chunks) ++sh;
        a.run_shift = sh;
    }
    // about 64 KiB of payload per workgroup
    int tpw = (64 * 1024) / (2 * a.run_chunks * 16);
    if (tpw < 1) tpw = 1;
    a.tokens_per_wg = tpw;
    const int64_t gx = ((int64_t)max_tokens + tpw - 1) / tpw;
    if (gx > 0x7fffffff || n_seqs > 65535) return KV_ERR_INVALID_ARG;

    dim3 grid((unsigned)gx, (unsigned)n_seqs);
    const int slot = kv_prof_begin(KV_PROF_REPACK, (hipStream_t)hip_stream);
    hipLaunchKernelGGL(kv_repack_kernel, grid, dim3(kRepackThreads), 0, (hipStream_t)hip_stream,
                       (uint16_t*)kv_pool, src_block_table, src_stride, dst_block_table, dst_stride,
                       n_tokens, a);
    kv_prof_end(KV_PROF_REPACK, slot, (hipStream_t)hip_stream);
    return kv_record_hip_error(hipGetLastError(), "kv_repack launch");
}

extern "C" int kv_append(void* kv_pool, int64_t n_pool_blocks, const kv_view* view,
                         const void* k_new, const void* v_new, const int32_t* block_table,
                         int64_t block_table_stride, const int32_t* positions, int n_seqs,
                         void* hip_stream)
{
    if (!kv_view_ok(view) || n_seqs < 0 || n_pool_blocks < 0 || block_table_stride < 0)
        return KV_ERR_INVALID_ARG;
    if (n_seqs == 0) return KV_OK;
    if (!kv_pool || !k_new || !v_new || !block_table || !positions) return KV_ERR_INVALID_ARG;
    hipLaunchKernelGGL(kv_append_kernel, dim3((unsigned)n_seqs), dim3(256), 0,
                       (hipStream_t)hip_stream, (uint16_t*)kv_pool, (const uint16_t*)k_new,
                       (const uint16_t*)v_new, block_table, block_table_stride, positions,
                       kv_view_to_dev(view));
    return kv_record_hip_error(hipGetLastError(), "kv_append launch");
}
