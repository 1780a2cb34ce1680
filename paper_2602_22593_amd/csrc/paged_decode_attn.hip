// paged_decode_attn: batched single-query attention over a paged bf16 KV pool read through a
// layout view (paper Sec. 2.1 attention over cached K/V; Sec. 4.2.2-4.2.3: blocks found through
// the logical table, kernel told the view's stride and capacity).
//
// Work decomposition (split-KV): a workgroup owns (sequence, local KV head, chunk of
// chunk_tokens tokens) and serves the G query heads of that KV head together, so every K/V
// byte is fetched from HBM once.  A sequence with one chunk is finished in place; otherwise
// each chunk leaves an un-normalised partial (m, l, acc[d]) in the workspace and a second small
// kernel merges them:  m = max m_k, l = sum l_k 2^(m_k - m), acc = sum acc_k 2^(m_k - m).
// Scores are kept in base-2 units (q is pre-multiplied by scale * log2(e)).
#include <math.h>

#include "kv_internal.h"

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr float kNegInf = -INFINITY;

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

// fp32 -> bf16, round to nearest even (inputs here are finite or zero).
__device__ __forceinline__ uint16_t f32_to_bf16(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40);  // keep NaN a NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void unpack8(const uint4& r, float (&f)[8])
{
    f[0] = bf16_lo(r.x); f[1] = bf16_hi(r.x);
    f[2] = bf16_lo(r.y); f[3] = bf16_hi(r.y);
    f[4] = bf16_lo(r.z); f[5] = bf16_hi(r.z);
    f[6] = bf16_lo(r.w); f[7] = bf16_hi(r.w);
}

struct decode_args {
    const uint16_t* q;
    uint16_t* out;
    const uint16_t* pool;
    const int32_t* table;
    int64_t table_stride;
    const int32_t* ctx_lens;
    kv_view_dev v;
    float scale_log2e;
    int32_t chunk_tokens;
    int32_t max_chunks;
    float* part_acc;  // [batch][n_q_local][max_chunks][D]
    float* part_ml;   // [batch][n_q_local][max_chunks][2]
};

// Combine (m2, l2, a2[]) into (m, l, a[]); all maxima may be -inf (empty partials).
template <int N>
__device__ __forceinline__ void combine(float& m, float& l, float (&a)[N], float m2, float l2,
                                        const float (&a2)[N])
{
    const float mn = fmaxf(m, m2);
    const float ms = (mn == kNegInf) ? 0.f : mn;
    const float c1 = exp2f(m - ms), c2 = exp2f(m2 - ms);
    l = l * c1 + l2 * c2;
#pragma unroll
    for (int e = 0; e < N; ++e) a[e] = a[e] * c1 + a2[e] * c2;
    m = mn;
}

// ---------------------------------------------------------------------------------------------
// Vector-ALU kernel, any G in {1,2,4,8} and D in {64,128}.  A "row group" of D/8 lanes reads one
// 2*D-byte K (then V) row per load, 16 bytes per lane; a wavefront covers 64/(D/8) consecutive
// token rows per load.  Every row group keeps its own online-softmax state over the tokens it
// visits; row groups and wavefronts are merged once at the end.
// ---------------------------------------------------------------------------------------------
template <int D, int G>
__global__ __launch_bounds__(kThreads) void decode_valu_kernel(decode_args a)
{
    constexpr int LPR = D / 8;          // lanes per row
    constexpr int RPW = 64 / LPR;       // rows per wavefront load
    constexpr int ROWS = RPW * kWaves;  // row groups in the workgroup
    constexpr int TPI = 4;              // tokens per row group per iteration

    const int chunk = blockIdx.x, hl = blockIdx.y, s = blockIdx.z;
    const int n = a.ctx_lens[s];
    const int cs = chunk * a.chunk_tokens;
    if (cs >= n && chunk != 0) return;
    const int ce = min(n, cs + a.chunk_tokens);
    const int n_chunks = (n + a.chunk_tokens - 1) / a.chunk_tokens;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = lane % LPR;
    const int rg = wave * RPW + lane / LPR;
    const kv_view_dev& v = a.v;
    const int32_t* trow = a.table + (int64_t)s * a.table_stride;

    float qf[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        const uint4 r = *reinterpret_cast<const uint4*>(
            a.q + ((int64_t)s * v.n_q_local + hl * G + g) * D + c * 8);
        unpack8(r, qf[g]);
#pragma unroll
        for (int e = 0; e < 8; ++e) qf[g][e] *= a.scale_log2e;
    }

    float m[G], l[G], acc[G][8];
#pragma unroll
    for (int g = 0; g < G; ++g) {
        m[g] = kNegInf;
        l[g] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[g][e] = 0.f;
    }

    const int64_t head_elem = v.head_off + hl * D + c * 8;
    for (int tb = cs; tb < ce; tb += ROWS * TPI) {
        uint4 kr[TPI], vr[TPI];
        bool valid[TPI];
#pragma unroll
        for (int j = 0; j < TPI; ++j) {
            const int t = tb + j * ROWS + rg;
            valid[j] = t < ce;
            const int tc = valid[j] ? t : ce - 1;  // stay on a valid row; its score is masked
            int bj, slot;
            kv_split_token(v, tc, bj, slot);
            const int64_t base = (int64_t)trow[bj] * v.block_elems + (int64_t)slot * v.token_stride +
                                 head_elem;
            kr[j] = *reinterpret_cast<const uint4*>(a.pool + base);
            vr[j] = *reinterpret_cast<const uint4*>(a.pool + base + v.plane_elems);
        }
        float sc[TPI][G];
#pragma unroll
        for (int j = 0; j < TPI; ++j) {
            float kf[8];
            unpack8(kr[j], kf);
#pragma unroll
            for (int g = 0; g < G; ++g) {
                float d0 = 0.f;
#pragma unroll
                for (int e = 0; e < 8; ++e) d0 = fmaf(qf[g][e], kf[e], d0);
#pragma unroll
                for (int off = 1; off < LPR; off <<= 1) d0 += __shfl_xor(d0, off);
                sc[j][g] = valid[j] ? d0 : kNegInf;
            }
        }
        float vf[TPI][8];
#pragma unroll
        for (int j = 0; j < TPI; ++j) unpack8(vr[j], vf[j]);
#pragma unroll
        for (int g = 0; g < G; ++g) {
            float mn = m[g];
#pragma unroll
            for (int j = 0; j < TPI; ++j) mn = fmaxf(mn, sc[j][g]);
            const float ms = (mn == kNegInf) ? 0.f : mn;
            const float alpha = exp2f(m[g] - ms);
            float p[TPI], ps = 0.f;
#pragma unroll
            for (int j = 0; j < TPI; ++j) {
                p[j] = exp2f(sc[j][g] - ms);
                ps += p[j];
            }
            l[g] = l[g] * alpha + ps;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float x = acc[g][e] * alpha;
#pragma unroll
                for (int j = 0; j < TPI; ++j) x = fmaf(p[j], vf[j][e], x);
                acc[g][e] = x;
            }
            m[g] = mn;
        }
    }

    // merge the row groups of a wavefront (butterfly: every lane ends with the wave's result)
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
            const float m2 = __shfl_xor(m[g], off), l2 = __shfl_xor(l[g], off);
            float a2[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) a2[e] = __shfl_xor(acc[g][e], off);
            combine<8>(m[g], l[g], acc[g], m2, l2, a2);
        }
    }

    // merge the wavefronts through LDS
    __shared__ float s_acc[kWaves][G][D];
    __shared__ float s_ml[kWaves][G][2];
    if (lane < LPR) {
#pragma unroll
        for (int g = 0; g < G; ++g) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_acc[wave][g][c * 8 + e] = acc[g][e];
            if (c == 0) {
                s_ml[wave][g][0] = m[g];
                s_ml[wave][g][1] = l[g];
            }
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < G * D; idx += kThreads) {
        const int g = idx / D, e = idx - g * D;
        float mm = kNegInf;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) mm = fmaxf(mm, s_ml[w][g][0]);
        const float ms = (mm == kNegInf) ? 0.f : mm;
        float ll = 0.f, aa = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float cw = exp2f(s_ml[w][g][0] - ms);
            ll += s_ml[w][g][1] * cw;
            aa += s_acc[w][g][e] * cw;
        }
        const int qi = hl * G + g;
        if (n_chunks <= 1) {
            const float o = ll > 0.f ? aa / ll : 0.f;
            a.out[((int64_t)s * v.n_q_local + qi) * D + e] = f32_to_bf16(o);
        } else {
            const int64_t rec = ((int64_t)s * v.n_q_local + qi) * a.max_chunks + chunk;
            a.part_acc[rec * D + e] = aa;
            if (e == 0) {
                a.part_ml[rec * 2 + 0] = mm;
                a.part_ml[rec * 2 + 1] = ll;
            }
        }
    }
}

// Merge the partials of one (sequence, local query head); one thread per output element.
template <int D>
__global__ __launch_bounds__(D) void decode_merge_kernel(decode_args a)
{
    const int qi = blockIdx.x, s = blockIdx.y, e = threadIdx.x;
    const int n = a.ctx_lens[s];
    const int n_chunks = (n + a.chunk_tokens - 1) / a.chunk_tokens;
    if (n_chunks <= 1) return;  // finished in place by the main kernel
    const int64_t rec0 = ((int64_t)s * a.v.n_q_local + qi) * a.max_chunks;
    float mm = kNegInf;
    for (int k = 0; k < n_chunks; ++k) mm = fmaxf(mm, a.part_ml[(rec0 + k) * 2]);
    float ll = 0.f, aa = 0.f;
#pragma unroll 4
    for (int k = 0; k < n_chunks; ++k) {
        const float cw = exp2f(a.part_ml[(rec0 + k) * 2] - mm);
        ll += a.part_ml[(rec0 + k) * 2 + 1] * cw;
        aa += a.part_acc[(rec0 + k) * D + e] * cw;
    }
    a.out[((int64_t)s * a.v.n_q_local + qi) * D + e] = f32_to_bf16(aa / ll);
}

int pick_chunk_tokens(const kv_view* v, int batch, int max_ctx_len)
{
    const int64_t forced = kv_option_chunk_tokens();
    if (forced > 0) return (int)forced;
    (void)v; (void)batch; (void)max_ctx_len;
    return 512;
}

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

template <int D, int G>
void launch_valu(const decode_args& a, int max_chunks, int n_kv_local, int batch, hipStream_t st)
{
    dim3 grid((unsigned)max_chunks, (unsigned)n_kv_local, (unsigned)batch);
    hipLaunchKernelGGL((decode_valu_kernel<D, G>), grid, dim3(kThreads), 0, st, a);
}

template <int D>
int launch_for_group(const decode_args& a, int G, int max_chunks, int n_kv_local, int batch,
                     hipStream_t st)
{
    switch (G) {
        case 1: launch_valu<D, 1>(a, max_chunks, n_kv_local, batch, st); return KV_OK;
        case 2: launch_valu<D, 2>(a, max_chunks, n_kv_local, batch, st); return KV_OK;
        case 4: launch_valu<D, 4>(a, max_chunks, n_kv_local, batch, st); return KV_OK;
        case 8: launch_valu<D, 8>(a, max_chunks, n_kv_local, batch, st); return KV_OK;
        default: return KV_ERR_UNSUPPORTED;
    }
}

}  // namespace

extern "C" size_t paged_decode_attn_workspace_bytes(const kv_view* view, int batch, int max_ctx_len)
{
    if (!kv_view_ok(view) || batch <= 0 || max_ctx_len <= 0) return 256;
    const int chunk = pick_chunk_tokens(view, batch, max_ctx_len);
    const int64_t max_chunks = ((int64_t)max_ctx_len + chunk - 1) / chunk;
    if (max_chunks <= 1) return 256;
    const int64_t recs = (int64_t)batch * view->n_q_local * max_chunks;
    return align_up((size_t)recs * view->geom.head_dim * 4, 256) + align_up((size_t)recs * 2 * 4, 256);
}

extern "C" int paged_decode_attn(const void* q, void* out, const void* kv_pool,
                                 int64_t n_pool_blocks, const int32_t* block_table,
                                 int64_t block_table_stride, const int32_t* ctx_lens, int batch,
                                 int max_ctx_len, const kv_view* view, float scale, void* workspace,
                                 size_t workspace_bytes, void* hip_stream)
{
    if (!kv_view_ok(view) || batch < 0 || max_ctx_len < 0 || n_pool_blocks < 0 ||
        block_table_stride < 0)
        return KV_ERR_INVALID_ARG;
    if (batch == 0) return KV_OK;
    if (!q || !out || !ctx_lens) return KV_ERR_INVALID_ARG;
    if (max_ctx_len > 0 && (!kv_pool || !block_table)) return KV_ERR_INVALID_ARG;
    const int64_t need_cols = ((int64_t)max_ctx_len + view->block_tokens - 1) / view->block_tokens;
    if (block_table_stride < need_cols) return KV_ERR_INVALID_ARG;
    const int D = view->geom.head_dim, G = view->group;
    if (D != 64 && D != 128) return KV_ERR_UNSUPPORTED;
    if (G != 1 && G != 2 && G != 4 && G != 8) return KV_ERR_UNSUPPORTED;
    if (batch > 65535 || view->n_kv_local > 65535) return KV_ERR_UNSUPPORTED;

    const int chunk = pick_chunk_tokens(view, batch, max_ctx_len);
    int64_t max_chunks = ((int64_t)max_ctx_len + chunk - 1) / chunk;
    if (max_chunks < 1) max_chunks = 1;
    const size_t need = paged_decode_attn_workspace_bytes(view, batch, max_ctx_len);
    if (max_chunks > 1) {
        if (!workspace) return KV_ERR_INVALID_ARG;
        if (workspace_bytes < need) return KV_ERR_WORKSPACE;
        if (((uintptr_t)workspace & 255u) != 0) return KV_ERR_INVALID_ARG;
    }

    decode_args a;
    a.q = (const uint16_t*)q;
    a.out = (uint16_t*)out;
    a.pool = (const uint16_t*)kv_pool;
    a.table = block_table;
    a.table_stride = block_table_stride;
    a.ctx_lens = ctx_lens;
    a.v = kv_view_to_dev(view);
    const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    a.scale_log2e = sc * 1.4426950408889634f;
    a.chunk_tokens = chunk;
    a.max_chunks = (int32_t)max_chunks;
    const int64_t recs = (int64_t)batch * view->n_q_local * max_chunks;
    a.part_acc = (float*)workspace;
    a.part_ml = max_chunks > 1
                    ? (float*)((char*)workspace + align_up((size_t)recs * D * 4, 256))
                    : nullptr;

    hipStream_t st = (hipStream_t)hip_stream;
    int slot = kv_prof_begin(KV_PROF_DECODE_MAIN, st);
    int rc = (D == 128) ? launch_for_group<128>(a, G, (int)max_chunks, view->n_kv_local, batch, st)
                        : launch_for_group<64>(a, G, (int)max_chunks, view->n_kv_local, batch, st);
    if (rc) return rc;
    kv_prof_end(KV_PROF_DECODE_MAIN, slot, st);
    rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn launch");
    if (rc) return rc;
    if (max_chunks > 1) {
        slot = kv_prof_begin(KV_PROF_DECODE_MERGE, st);
        dim3 grid((unsigned)view->n_q_local, (unsigned)batch);
        if (D == 128)
            hipLaunchKernelGGL(decode_merge_kernel<128>, grid, dim3(128), 0, st, a);
        else
            hipLaunchKernelGGL(decode_merge_kernel<64>, grid, dim3(64), 0, st, a);
        kv_prof_end(KV_PROF_DECODE_MERGE, slot, st);
        rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn merge launch");
    }
    return rc;
}
