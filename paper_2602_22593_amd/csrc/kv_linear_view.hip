// Linear layer on a zero-copy shard view of a full weight (Model Weights Manager, Sec. 4.1 of
// the paper; Eq. 1: W_active^(r) = View(W_full, dim, r, m)): y = x W_active^T, where W_active is
// a set of stored rows (output features; up to three contiguous segments, as rank r's Q, K and V
// heads of a fused QKV weight) and a contiguous range of stored columns (input features, for the
// row-parallel output projection) of a weight kept once, whole, as [out][in] bf16.  Nothing is
// copied: the kernel addresses the full matrix with its own leading dimension.
//
// Shaped for decode batches (M up to a few hundred rows): the weight slice is streamed from HBM
// once per 64 batch rows and is the only traffic that matters; x is small, but every weight row
// needs all of it, so the workgroup shares it through LDS.  A workgroup of four wavefronts owns
// 16 RB logical weight rows (RB = 1 or 2 blocks of 16) x 64 batch rows over the whole input
// dimension (or its share of it), walked in slabs of 128 input features.  With RB row blocks the
// 4 / RB wavefronts of a row block each take a part of every slab and add up through LDS once, at
// the end, so no output tile is cut over workgroups unless the launch would otherwise be too small
// to fill the chip: partial tiles cost as much traffic as the weights they stand for at these
// batch sizes.  RB is the largest that still gives about two hundred workgroups.
//
// The walk is one continuous stream.  A load instruction fetches four rows, 256 contiguous bytes of
// each (64-byte pieces of a row per instruction, as the operand arrangement would ask for, halve the
// rate at which HBM delivers the weights), into a ring of registers four slabs deep; a slab's
// requests are issued three slabs before it is used, and every round issues exactly one slab's
// worth, rounds past the end included (those ask for 16 bytes and multiply by zero): with nothing
// conditional about the loads the compiler's count of outstanding requests is exact, and a round
// waits for its own slab only.  Arrived rows go into one of two LDS buffers, XOR-swizzled so that
// the row-wise writes and the operand-wise reads are both free of bank conflicts; one barrier per
// slab (a bare one: the fences of __syncthreads() would drain the request queue); the matrix
// instructions of a slab run in the round after, while the next slab's operand reads are under way.
// Every workgroup starts its walk at another slab, so that the workgroups do not ask for the same
// column range of all rows at the same time.
//   y^T[weight row][batch row] += W[row][k .. k + 32) . x[batch row][k .. k + 32)
// with 16x16x32 bf16 MFMA, fp32 accumulation, one rounding to bf16 at the end.  When the input
// dimension is cut over `splits` workgroups (small slices only), each leaves an fp32 partial tile in
// the workspace and a second, small kernel adds the splits in a fixed order (deterministic).
//
// Where the time goes (measured by replacing the requests by idle ones): on the 8B projections at
// M = 64 the kernel takes 16-19 us with no memory traffic at all.  A round costs a workgroup about
// 0.45 us: 24 KiB written to and 40 KiB read from LDS, eight matrix instructions per wavefront, and
// the barrier keeps the four wavefronts of a compute unit in the same phase, so LDS and matrix
// pipe take turns instead of overlapping.  The weight stream itself is not the limit yet.
#include <string.h>

#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kThreads = 256;
constexpr int kColBlocks = 4;   // 16-row blocks of x per workgroup
constexpr int kSlab = 128;      // input features per slab

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

// s_waitcnt vmcnt(N), N <= 63, leaving the other counters alone
template <int N>
__device__ __forceinline__ void wait_vm()
{
    static_assert(N >= 0 && N <= 63, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | 0x0f70);
}
// wait until at most `slabs` slabs of OPS loads each are outstanding
template <int OPS>
__device__ __forceinline__ void wait_slabs(int slabs)
{
    switch (slabs) {
        case 0: wait_vm<0>(); break;
        case 1: wait_vm<OPS>(); break;
        case 2: wait_vm<2 * OPS>(); break;
        case 3: wait_vm<3 * OPS>(); break;
        case 4: wait_vm<4 * OPS>(); break;
        case 5: wait_vm<5 * OPS>(); break;
        case 6: wait_vm<6 * OPS>(); break;
        default: wait_vm<(7 * OPS > 63 ? 63 : 7 * OPS)>(); break;
    }
}

// Workgroup barrier without the memory fences of __syncthreads(): those would make every wavefront
// wait for ALL its outstanding loads, the seven slabs in flight included.  What has to be complete
// at this barrier is stated by the caller's own vmcnt wait (the slab about to be consumed) and by the
// LDS reads of the previous slab having returned to the matrix instructions that used them.
__device__ __forceinline__ void stream_barrier()
{
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int RB>
__global__ __launch_bounds__(kThreads, 2) void linear_stream_kernel(linear_args p)
{
    constexpr int KP = 4 / RB;        // wavefronts sharing a row block, each a part of every slab
    constexpr int KK = 4 / KP;        // 32-wide steps of a slab per wavefront
    constexpr int NR = 4;             // slabs in the register ring: NR - 1 requested ahead (even)
    // A slab in LDS: rows of 16 16-byte pieces (x: 64 batch rows; w: the workgroup's 16 RB weight
    // rows), piece q of row t kept at position q ^ (t % 16): the row-wise staging writes and the MFMA
    // operand reads (lane (r, quad): row r, piece 4 kk + quad) both touch every bank once per 16 lanes.
    __shared__ kv_u32x4 s_x[2][1024];
    __shared__ kv_u32x4 s_w[2][256 * RB];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, quad = lane >> 4;
    const int rb = wave % RB, kp = wave / RB;
    const int m0 = blockIdx.x * (16 * kColBlocks);
    const int n0 = blockIdx.y * (16 * RB);

    // the rows of this workgroup lie in one segment (segment sizes are multiples of 64)
    int seg = 0;
    while (seg + 1 < p.n_seg && n0 >= p.seg_first[seg + 1]) ++seg;
    const int64_t phys0 = p.seg_start[seg] + (n0 - p.seg_first[seg]);

    // staging: a load instruction covers four rows, 256 contiguous bytes of each: lane = 16 g + pos
    // fetches piece pos of row 4 u + g.  x: wavefront w stages batch rows 16 w .. 16 w + 15 (rows past M
    // repeat the last one); weights: wavefront w stages rows 4 (RB w + i) .. + 3, i < RB
    const int g = lane >> 4, pos = lane & 15;
    const char* xsrc[4];
    int xdst[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 16 * wave + 4 * u + g;
        xsrc[u] = reinterpret_cast<const char*>(p.x + (int64_t)min(m0 + row, p.M - 1) * p.ldx) + (pos << 4);
        xdst[u] = row * 16 + (pos ^ (row & 15));
    }
    const char* wsrc[RB];
    int wdst[RB];
#pragma unroll
    for (int i = 0; i < RB; ++i) {
        const int row = 4 * (RB * wave + i) + g;
        wsrc[i] = reinterpret_cast<const char*>(p.w + (phys0 + row) * p.ldw + p.col_start) + (pos << 4);
        wdst[i] = row * 16 + (pos ^ (row & 15));
    }

    // this workgroup's slabs: [first, first + n)
    const int total = p.Kl / kSlab;
    const int per_split = (total + p.splits - 1) / p.splits;
    const int first = (int)blockIdx.z * per_split;
    const int n = min(total, first + per_split) - first;

    // Every workgroup starts its walk at another slab and wraps around, so that at any moment the
    // workgroups ask for different column ranges: rows are a power of two apart, and the same columns
    // of all rows share a few memory channels.
    const int rot = (int)((blockIdx.y * 5u + blockIdx.x * 3u) % (unsigned)n);
    // The walk is written without a single conditional load: every round requests exactly one slab
    // (rounds past the end request 16 bytes of x, the same for all lanes, and multiply by zero).  The
    // compiler then knows in every round that the registers it is about to use were requested NR - 1
    // requests ago and waits for exactly those; with requests that may or may not have been issued it
    // has to assume the worst and drains the whole queue.
    kv_u32x4 x_reg[NR][4], w_reg[NR][RB];
    auto issue = [&](int j, int slot) {   // loads of the j-th slab of this workgroup's walk into ring slot `slot`
        // (address arithmetic instead of a choice between two pointers: a choice on a condition that
        // is the same for the whole wavefront is compiled into two paths with a load and a wait each)
        const int64_t keep = j < n ? (int64_t)-1 : 0;
        int jr = j + rot;
        if (jr >= n) jr -= n;
        const int64_t off = (int64_t)(first + jr) * (kSlab * 2);
        const char* idle = reinterpret_cast<const char*>(p.x);
#pragma unroll
        for (int i = 0; i < RB; ++i)
            w_reg[slot][i] = __builtin_nontemporal_load(
                reinterpret_cast<const kv_u32x4*>(idle + (((wsrc[i] + off) - idle) & keep)));
#pragma unroll
        for (int u = 0; u < 4; ++u)
            x_reg[slot][u] = *reinterpret_cast<const kv_u32x4*>(idle + (((xsrc[u] + off) - idle) & keep));
    };

    f32x4 acc[kColBlocks];
#pragma unroll
    for (int cb = 0; cb < kColBlocks; ++cb) acc[cb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // Round j: slab j goes from this wavefront's registers into LDS buffer j % 2 and its ring slot
    // takes the next request; after the barrier the operands of slab j are read from LDS and, while
    // those reads are under way, the matrix instructions of slab j - 1 run on the operands read in the
    // round before: with one wavefront per SIMD nothing else would hide the LDS latency.
    kv_u32x4 a_op[2][KK], b_op[2][KK][kColBlocks];
    auto read_operands = [&](int buf, int which, bool real) {
        const kv_u32x4* xb = s_x[buf];
        const kv_u32x4* wrow = s_w[buf] + (16 * rb + r) * 16;
#pragma unroll
        for (int t = 0; t < KK; ++t) {
            const int q = 4 * (kp * KK + t) + quad;
            a_op[which][t] = wrow[q ^ r];
            if (!real) a_op[which][t] = kv_u32x4{0u, 0u, 0u, 0u};   // a round past the end adds nothing
#pragma unroll
            for (int cb = 0; cb < kColBlocks; ++cb) b_op[which][t][cb] = xb[(16 * cb + r) * 16 + (q ^ r)];
        }
    };
    auto multiply = [&](int which) {
#pragma unroll
        for (int t = 0; t < KK; ++t)
#pragma unroll
            for (int cb = 0; cb < kColBlocks; ++cb)
                acc[cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a_op[which][t]),
                                                                  as_bf16x8(b_op[which][t][cb]), acc[cb], 0, 0, 0);
    };
#pragma unroll
    for (int t = 0; t < KK; ++t) {
        a_op[1][t] = kv_u32x4{0u, 0u, 0u, 0u};
#pragma unroll
        for (int cb = 0; cb < kColBlocks; ++cb) b_op[1][t][cb] = kv_u32x4{0u, 0u, 0u, 0u};
    }

#pragma unroll
    for (int j = 0; j < NR - 1; ++j) issue(j, j);
    for (int j0 = 0; j0 < n; j0 += NR) {
#pragma unroll
        for (int jj = 0; jj < NR; ++jj) {
            const int j = j0 + jj;
            kv_u32x4* xb = s_x[jj & 1];
            kv_u32x4* wb = s_w[jj & 1];
#pragma unroll
            for (int i = 0; i < RB; ++i) wb[wdst[i]] = w_reg[jj][i];
#pragma unroll
            for (int u = 0; u < 4; ++u) xb[xdst[u]] = x_reg[jj][u];
            issue(j + NR - 1, (jj + NR - 1) % NR);
            // this wavefront's pieces are written, and its operand reads of the round before (from the
            // other buffer, which the next round overwrites) have returned
            __builtin_amdgcn_s_waitcnt(0xc07f);   // lgkmcnt(0)
            stream_barrier();
            read_operands(jj & 1, jj & 1, j < n);
            __builtin_amdgcn_sched_barrier(0);
            multiply((jj + 1) & 1);
        }
    }
    multiply((NR - 1) & 1);   // the last round's slab (NR is even: its operands are in set 1)

    // the wavefronts of a row block add up (buffers are free once everybody has left the loop)
    if (KP > 1) {
        __syncthreads();
        f32x4* red = reinterpret_cast<f32x4*>(&s_x[0][0]);   // [wave][cb][lane]
        if (kp > 0) {
#pragma unroll
            for (int cb = 0; cb < kColBlocks; ++cb) red[(wave * kColBlocks + cb) * 64 + lane] = acc[cb];
        }
        __syncthreads();
        if (kp > 0) return;
#pragma unroll
        for (int k = 1; k < KP; ++k)
#pragma unroll
            for (int cb = 0; cb < kColBlocks; ++cb) acc[cb] += red[((k * RB + rb) * kColBlocks + cb) * 64 + lane];
    }

    // acc[cb][i] = y[m0 + 16 cb + r][n0 + 16 rb + 4 quad + i]
#pragma unroll
    for (int cb = 0; cb < kColBlocks; ++cb) {
        const int m = m0 + 16 * cb + r;
        if (m >= p.M) continue;
        const int nn = n0 + 16 * rb + 4 * quad;
        if (p.splits > 1) {
            *reinterpret_cast<f32x4*>(p.part + ((int64_t)blockIdx.z * p.M + m) * p.Nl + nn) = acc[cb];
        } else {
            uint2 pk;
            pk.x = pack_bf16x2(acc[cb][0], acc[cb][1]);
            pk.y = pack_bf16x2(acc[cb][2], acc[cb][3]);
            *reinterpret_cast<uint2*>(p.y + (int64_t)m * p.ldy + nn) = pk;
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

// Row blocks per workgroup and workgroups sharing the input dimension of one output tile.
// Whole tiles per workgroup wherever that gives about two hundred workgroups (the launch has to
// keep enough bytes in flight, not to occupy every compute unit); the input dimension is cut only
// for slices too small for that, and then into as few parts as fill half the chip.
struct linear_cfg {
    int rb, splits;
};
linear_cfg pick_cfg(int64_t m_tiles, int64_t n_l, int total_slabs)
{
    linear_cfg c = {1, 1};
    for (int rb = 2; rb >= 1; rb >>= 1) {
        c.rb = rb;
        if (m_tiles * (n_l / (16 * rb)) >= 192) break;
    }
    const int64_t tiles = m_tiles * (n_l / (16 * c.rb));
    int s = 1;
    while (s < 16 && s < total_slabs && tiles * s < 128) ++s;
    const int64_t forced = kv_option_linear_splits();
    if (forced > 0) s = (int)forced;
    s = s > 16 ? 16 : s;
    s = s > total_slabs ? total_slabs : s;
    c.splits = s < 1 ? 1 : s;
    return c;
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
    const int64_t m_tiles = ((int64_t)M + 16 * kColBlocks - 1) / (16 * kColBlocks);
    const int splits = pick_cfg(m_tiles, n_l, (int)(view->col_count / kSlab)).splits;
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
        if (view->row_count[i] % 64 != 0) return KV_ERR_UNSUPPORTED;
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
    const linear_cfg cfg = pick_cfg(m_tiles, n_l, p.Kl / kSlab);
    const int64_t n_tiles = n_l / (16 * cfg.rb);
    if (m_tiles > 0x7fffffff || n_tiles > 65535) return KV_ERR_UNSUPPORTED;
    p.splits = cfg.splits;
    p.part = (float*)workspace;
    if (p.splits > 1) {
        if (!workspace || ((uintptr_t)workspace & 15)) return KV_ERR_INVALID_ARG;
        if (workspace_bytes < (size_t)p.splits * M * n_l * 4) return KV_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const int slot = kv_prof_begin(KV_PROF_LINEAR, st);
    const dim3 grid((unsigned)m_tiles, (unsigned)n_tiles, (unsigned)p.splits);
    if (cfg.rb == 2) hipLaunchKernelGGL(linear_stream_kernel<2>, grid, dim3(kThreads), 0, st, p);
    else hipLaunchKernelGGL(linear_stream_kernel<1>, grid, dim3(kThreads), 0, st, p);
    if (p.splits > 1) {
        const int64_t quads = (int64_t)M * (n_l / 4);
        hipLaunchKernelGGL(linear_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, p);
    }
    kv_prof_end(KV_PROF_LINEAR, slot, st);
    return kv_record_hip_error(hipGetLastError(), "kv_linear_view launch");
}

