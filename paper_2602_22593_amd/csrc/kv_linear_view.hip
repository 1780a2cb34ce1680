// Linear layer on a zero-copy shard view of a full weight (Model Weights Manager, Sec. 4.1 of
// the paper; Eq. 1: W_active^(r) = View(W_full, dim, r, m)): y = x W_active^T, where W_active is
// a set of stored rows (output features; up to three contiguous segments, as rank r's Q, K and V
// heads of a fused QKV weight) and a contiguous range of stored columns (input features, for the
// row-parallel output projection) of a weight kept once, whole, as [out][in] bf16.  Nothing is
// copied: the kernel addresses the full matrix with its own leading dimension.
//
// Shaped for decode batches (M up to a few hundred rows): the weight slice is streamed from HBM
// once per 64 batch rows and is the dominant traffic; x is small, but every weight row needs all
// of it, so it must be shared: a workgroup of four wavefronts owns 64 logical weight rows (16 per
// wavefront) x 64 batch rows and walks its part of the input dimension in slabs of 128.  The x
// slab (64 rows x 128) is staged in LDS once per workgroup, laid out in MFMA operand order so
// that each B operand is one contiguous kilobyte, and every wavefront accumulates
//   y^T[weight row][batch row] += W[row][k .. k + 32) . x[batch row][k .. k + 32)
// with 16x16x32 bf16 MFMA.  Its 16 weight rows are fetched as they lie in memory (a load
// instruction covers four rows x 256 contiguous bytes) and pass through a wavefront-private,
// XOR-swizzled LDS buffer into the A-operand arrangement.
// The walk is paced by memory latency, not bandwidth (per-workgroup timestamps: one round trip
// under this load is 4-5 us), so the loads of four slabs (a chunk: 64 KiB of W and 64 KiB of x
// per workgroup) are all issued before anything waits, and the input dimension is cut over
// `splits` workgroups (grid.z) so that a workgroup has about two chunks: each then leaves an fp32
// partial tile in the workspace and a second, small kernel adds the splits in a fixed order and
// rounds to bf16 (deterministic; no atomics).
#include <string.h>

#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = 64;   // logical weight rows per workgroup: 16 per wavefront
constexpr int kColBlocks = 4;   // 16-row blocks of x per workgroup
constexpr int kSlab = 128;      // input features per slab
constexpr int kChunk = 4;       // slabs whose loads a workgroup issues together

struct linear_args {
    const uint16_t* x;
    int64_t ldx;
    const uint16_t* w;
    int64_t ldw;
    uint16_t* y;
    int64_t ldy;
    int32_t M, Nl, Kl;
    int64_t col_start;
    int32_t n_seg;
    int64_t seg_start[3];   // first stored row of each segment
    int32_t seg_first[4];   // first logical row of each segment; seg_first[n_seg] = Nl
    int32_t splits;         // workgroups sharing the input dimension of one output tile
    float* part;            // [splits][M][Nl] fp32 when splits > 1
};

__global__ __launch_bounds__(kThreads, 2) void linear_view_kernel(linear_args p)
{
    // x slabs of one chunk in operand order: piece (kk, cb, quad, c) = x[16 cb + c][32 kk + 8 quad .. + 8)
    // of a slab sits at ((kk * 4 + cb) * 4 + quad) * 16 + (c ^ (4 kk + quad)): a B operand is one
    // contiguous kilobyte, and the XOR spreads the row-wise staging writes over all banks
    __shared__ kv_u32x4 s_x[kChunk][4 * kColBlocks * 64];
    // weight rows of one slab, per wavefront: piece c (16 bytes) of row t at t * 16 + (c ^ t)
    __shared__ kv_u32x4 s_w[kThreads / 64][256];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, quad = lane >> 4;
    const int m0 = blockIdx.x * (16 * kColBlocks);
    const int n0 = blockIdx.y * kTileRows;

    // the 64 logical rows of this workgroup lie in one segment (segment sizes are multiples of 64)
    int seg = 0;
    while (seg + 1 < p.n_seg && n0 >= p.seg_first[seg + 1]) ++seg;
    const int64_t phys0 = p.seg_start[seg] + (n0 - p.seg_first[seg]);
    // load instruction u of a slab: row 4 u + quad of the wavefront's 16, piece r of its 16
    const char* wbase = reinterpret_cast<const char*>(p.w + (phys0 + 16 * wave + quad) * p.ldw + p.col_start) + r * 16;
    const int64_t w_step4 = 4 * p.ldw * 2;   // bytes between rows 4 apart
    kv_u32x4* const sw = s_w[wave];

    // staging: thread t moves pieces t, t + 256, t + 512, t + 768 of a slab; piece id = 16 row + q,
    // q = 4 kk + quad the 16-byte piece within the row's 128 elements (rows past M repeat the last)
    const char* xsrc[4];
    int xdst[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int id = tid + 256 * i, row = id >> 4, q = id & 15;
        xsrc[i] = reinterpret_cast<const char*>(p.x + (int64_t)min(m0 + row, p.M - 1) * p.ldx) + q * 16;
        xdst[i] = (((q >> 2) * kColBlocks + (row >> 4)) * 4 + (q & 3)) * 16 + ((row & 15) ^ q);
    }

    // this workgroup's slabs: [step, last)
    const int total = p.Kl / kSlab;
    const int per_split = (total + p.splits - 1) / p.splits;
    int step = (int)blockIdx.z * per_split;
    const int last = min(total, step + per_split);

    f32x4 acc[kColBlocks];
#pragma unroll
    for (int cb = 0; cb < kColBlocks; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // A chunk is up to kChunk slabs.  All of a chunk's loads (weights first, then x) are issued
    // before anything waits: the walk along the input dimension is paced by memory latency, so a
    // workgroup should need as few round trips as it can, and the splits are chosen to give it one
    // or two chunks.
    kv_u32x4 a_st[kChunk][4], x_st[kChunk][4];
    auto compute = [&](int j) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = 4 * u + quad;
            sw[row * 16 + (r ^ row)] = a_st[j][u];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const kv_u32x4 a = sw[r * 16 + ((4 * kk + quad) ^ r)];
#pragma unroll
            for (int cb = 0; cb < kColBlocks; ++cb) {
                const kv_u32x4 b = s_x[j][(kk * kColBlocks + cb) * 64 + quad * 16 + (r ^ (4 * kk + quad))];
                acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), acc[cb], 0, 0, 0);
            }
        }
        __builtin_amdgcn_wave_barrier();
    };
    for (bool first = true; step < last; step += kChunk, first = false) {
        const int n_slabs = min(kChunk, last - step);
        const int64_t off = (int64_t)step * (kSlab * 2);
#pragma unroll
        for (int j = 0; j < kChunk; ++j)
            if (j < n_slabs) {
#pragma unroll
                for (int u = 0; u < 4; ++u)
                    a_st[j][u] = __builtin_nontemporal_load(
                        reinterpret_cast<const kv_u32x4*>(wbase + off + j * (kSlab * 2) + u * w_step4));
            }
#pragma unroll
        for (int j = 0; j < kChunk; ++j)
            if (j < n_slabs) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
                    x_st[j][i] = *reinterpret_cast<const kv_u32x4*>(xsrc[i] + off + j * (kSlab * 2));
            }
        if (!first) __syncthreads();   // the previous chunk's operands have been read
#pragma unroll
        for (int j = 0; j < kChunk; ++j)
            if (j < n_slabs) {
#pragma unroll
                for (int i = 0; i < 4; ++i) s_x[j][xdst[i]] = x_st[j][i];
            }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < kChunk; ++j)
            if (j < n_slabs) compute(j);
    }

    // acc[cb][i] = y[m0 + 16 cb + r][n0 + 16 wave + 4 quad + i]
#pragma unroll
    for (int cb = 0; cb < kColBlocks; ++cb) {
        const int m = m0 + 16 * cb + r;
        if (m >= p.M) continue;
        const int n = n0 + 16 * wave + 4 * quad;
        if (p.splits > 1) {
            *reinterpret_cast<f32x4*>(p.part + ((int64_t)blockIdx.z * p.M + m) * p.Nl + n) = acc[cb];
        } else {
            uint2 pk;
            pk.x = pack_bf16x2(acc[cb][0], acc[cb][1]);
            pk.y = pack_bf16x2(acc[cb][2], acc[cb][3]);
            *reinterpret_cast<uint2*>(p.y + (int64_t)m * p.ldy + n) = pk;
        }
    }
}

// y[m][n .. n + 4) = bf16(sum over splits of part[z][m][n .. n + 4)), splits added in order
__global__ __launch_bounds__(256) void linear_reduce_kernel(linear_args p)
{
    const int64_t quads = (int64_t)p.M * (p.Nl / 4);
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= quads) return;
    const int64_t m = i / (p.Nl / 4), n = (i - m * (p.Nl / 4)) * 4;
    f32x4 s = {0.f, 0.f, 0.f, 0.f};
    // four partial tiles requested at a time, then added in order (one memory round trip per four
    // splits instead of one per split)
    const float* src = p.part + m * p.Nl + n;
    const int64_t step = (int64_t)p.M * p.Nl;
    for (int z0 = 0; z0 < p.splits; z0 += 4) {
        f32x4 v[4];
#pragma unroll
        for (int j = 0; j < 4; ++j)
            v[j] = *reinterpret_cast<const f32x4*>(src + (int64_t)min(z0 + j, p.splits - 1) * step);
#pragma unroll
        for (int j = 0; j < 4; ++j)
            if (z0 + j < p.splits) s += v[j];
    }
    uint2 pk;
    pk.x = pack_bf16x2(s[0], s[1]);
    pk.y = pack_bf16x2(s[2], s[3]);
    *reinterpret_cast<uint2*>(p.y + m * p.ldy + n) = pk;
}

// Workgroups sharing the input dimension of one output tile.  Measured on the Llama-8B
// projections (batch 16..256, TP 1..8): the optimum is flat around two chunks per workgroup; more
// splits shorten the chain of memory round trips but their partial tiles cost as much again, fewer
// leave compute units idle.  So: two chunks each, more splits only while the launch would have
// fewer than 192 workgroups, fewer when it would have more than 1024; at most 16.
int pick_splits(int64_t tiles, int total_slabs)
{
    int s = (total_slabs + 2 * kChunk - 1) / (2 * kChunk);
    while (s < 16 && s < total_slabs && tiles * s < 192) ++s;
    while (s > 1 && tiles * s > 1024) --s;
    const int64_t forced = kv_option_linear_splits();
    if (forced > 0) s = (int)forced;
    s = s > 16 ? 16 : s;
    s = s > total_slabs ? total_slabs : s;
    return s < 1 ? 1 : s;
}

int64_t view_rows(const kv_weight_view* view)
{
    int64_t n = 0;
    for (int i = 0; i < view->n_segments && i < 3; ++i) n += view->row_count[i];
    return n;
}

}  // namespace

extern "C" size_t kv_linear_view_workspace_bytes(const kv_weight_view* view, int M)
{
    if (!view || M <= 0 || view->n_segments < 1 || view->n_segments > 3 || view->col_count <= 0) return 0;
    const int64_t n_l = view_rows(view);
    if (n_l <= 0) return 0;
    const int64_t tiles = ((int64_t)M + 16 * kColBlocks - 1) / (16 * kColBlocks) * (n_l / kTileRows);
    const int splits = pick_splits(tiles > 0 ? tiles : 1, (int)(view->col_count / kSlab));
    return splits > 1 ? (size_t)splits * M * n_l * 4 : 0;
}

extern "C" int kv_weight_view_make(int dim, int r, int m, int64_t n_rows, int64_t n_cols, kv_weight_view* out)
{
    if (!out || m < 1 || r < 0 || r >= m || n_rows <= 0 || n_cols <= 0 || (dim != 0 && dim != 1))
        return KV_ERR_INVALID_ARG;
    if ((dim == 0 ? n_rows : n_cols) % m != 0) return KV_ERR_INVALID_ARG;
    memset(out, 0, sizeof(*out));
    out->n_segments = 1;
    if (dim == 0) {
        out->row_start[0] = r * (n_rows / m);
        out->row_count[0] = n_rows / m;
        out->col_start = 0;
        out->col_count = n_cols;
    } else {
        out->row_start[0] = 0;
        out->row_count[0] = n_rows;
        out->col_start = r * (n_cols / m);
        out->col_count = n_cols / m;
    }
    return KV_OK;
}

extern "C" int kv_weight_view_fused_qkv(const kv_geometry* g, int64_t hidden, int r, int m, kv_weight_view* out)
{
    if (!g || !out || m < 1 || r < 0 || r >= m || hidden <= 0 || g->n_q_heads <= 0 || g->n_kv_heads <= 0 ||
        g->head_dim <= 0 || g->n_q_heads % m != 0 || g->n_kv_heads % m != 0)
        return KV_ERR_INVALID_ARG;
    const int64_t d = g->head_dim, hq = g->n_q_heads / m, hkv = g->n_kv_heads / m;
    memset(out, 0, sizeof(*out));
    out->n_segments = 3;
    out->row_start[0] = r * hq * d;
    out->row_count[0] = hq * d;
    out->row_start[1] = (int64_t)g->n_q_heads * d + r * hkv * d;
    out->row_count[1] = hkv * d;
    out->row_start[2] = (int64_t)(g->n_q_heads + g->n_kv_heads) * d + r * hkv * d;
    out->row_count[2] = hkv * d;
    out->col_start = 0;
    out->col_count = hidden;
    return KV_OK;
}

extern "C" int kv_linear_view(const void* x, int64_t ldx, const void* w_full, int64_t w_rows, int64_t ldw,
                              const kv_weight_view* view, void* y, int64_t ldy, int M, void* workspace,
                              size_t workspace_bytes, void* hip_stream)
{
    if (!view || M < 0 || view->n_segments < 1 || view->n_segments > 3 || w_rows <= 0 || ldw <= 0)
        return KV_ERR_INVALID_ARG;
    int64_t n_l = 0;
    for (int i = 0; i < view->n_segments; ++i) {
        if (view->row_start[i] < 0 || view->row_count[i] <= 0 || view->row_start[i] + view->row_count[i] > w_rows)
            return KV_ERR_INVALID_ARG;
        n_l += view->row_count[i];
    }
    if (view->col_start < 0 || view->col_count <= 0 || view->col_start + view->col_count > ldw ||
        ldx < view->col_count || ldy < n_l)
        return KV_ERR_INVALID_ARG;
    if (M == 0) return KV_OK;
    if (!x || !w_full || !y) return KV_ERR_INVALID_ARG;
    // 16-byte operand loads, whole 128-wide steps, 64-row workgroup tiles inside one segment
    if (view->col_count % kSlab != 0 || view->col_start % 8 != 0 || ldx % 8 != 0 || ldw % 8 != 0 || ldy % 4 != 0 ||
        ((uintptr_t)x & 15) || ((uintptr_t)w_full & 15) || ((uintptr_t)y & 7) || n_l > 0x7fffffff ||
        view->col_count > 0x7fffffff)
        return KV_ERR_UNSUPPORTED;
    for (int i = 0; i < view->n_segments; ++i)
        if (view->row_count[i] % kTileRows != 0) return KV_ERR_UNSUPPORTED;
    linear_args p;
    p.x = (const uint16_t*)x;
    p.ldx = ldx;
    p.w = (const uint16_t*)w_full;
    p.ldw = ldw;
    p.y = (uint16_t*)y;
    p.ldy = ldy;
    p.M = M;
    p.Nl = (int32_t)n_l;
    p.Kl = (int32_t)view->col_count;
    p.col_start = view->col_start;
    p.n_seg = view->n_segments;
    int32_t first = 0;
    for (int i = 0; i < 3; ++i) {
        p.seg_start[i] = i < view->n_segments ? view->row_start[i] : 0;
        p.seg_first[i] = first;
        if (i < view->n_segments) first += (int32_t)view->row_count[i];
    }
    p.seg_first[3] = first;
    for (int i = view->n_segments; i < 4; ++i) p.seg_first[i] = first;
    const int64_t m_tiles = ((int64_t)M + 16 * kColBlocks - 1) / (16 * kColBlocks);
    const int64_t n_tiles = n_l / kTileRows;
    if (m_tiles > 0x7fffffff || n_tiles > 65535) return KV_ERR_UNSUPPORTED;
    p.splits = pick_splits(m_tiles * n_tiles, p.Kl / kSlab);
    p.part = (float*)workspace;
    if (p.splits > 1) {
        if (!workspace || ((uintptr_t)workspace & 15)) return KV_ERR_INVALID_ARG;
        if (workspace_bytes < (size_t)p.splits * M * n_l * 4) return KV_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const int slot = kv_prof_begin(KV_PROF_LINEAR, st);
    hipLaunchKernelGGL(linear_view_kernel, dim3((unsigned)m_tiles, (unsigned)n_tiles, (unsigned)p.splits),
                       dim3(kThreads), 0, st, p);
    if (p.splits > 1) {
        const int64_t quads = (int64_t)M * (n_l / 4);
        hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p);
    }
    kv_prof_end(KV_PROF_LINEAR, slot, st);
    return kv_record_hip_error(hipGetLastError(), "kv_linear_view launch");
}

