// Linear layer on a zero-copy shard view of a full weight (Model Weights Manager, Sec. 4.1 of
// the paper; Eq. 1: W_active^(r) = View(W_full, dim, r, m)): y = x W_active^T, where W_active is
// a set of stored rows (output features; up to three contiguous segments, as rank r's Q, K and V
// heads of a fused QKV weight) and a contiguous range of stored columns (input features, for the
// row-parallel output projection) of a weight kept once, whole, as [out][in] bf16.  Nothing is
// copied: the kernel addresses the full matrix with its own leading dimension.
//
// Shaped for decode batches (M up to a few hundred rows): the weight slice is streamed from HBM
// once per 64 batch rows and is the only HBM traffic that matters.  What limits such a product on
// this chip is not HBM but the path from L2 into a compute unit (measured here: about 18 bytes per
// clock per compute unit for 16-byte loads that hit L2): every weight row needs all of x, so a
// workgroup that walks the whole input dimension pulls x (M x K, far more than fits in registers or
// LDS) through that path again and again, two to four times the bytes of the weights it streams.
//
// So x stays put.  The input dimension is cut into slices of at most 8 slabs of 128 input features,
// and a workgroup owns one slice x 64 batch rows x NB blocks of 16 logical weight rows.  Each of its
// four wavefronts takes two slabs of the slice (w and w + 4) and loads its 64 x 256 piece of x ONCE
// (row-order loads, passed through its private LDS area into the arrangement of the matrix
// instruction's B operand), where it stays for the whole kernel (128 registers).  Then the wavefront
// walks the NB row blocks: a block's 16 rows x 2 slabs are requested four rows of 256 contiguous
// bytes per load instruction (64-byte pieces of a row per instruction, as the operand arrangement
// would ask for, halve the rate at which HBM delivers the weights), two row blocks ahead of the
// arithmetic, pass through the private LDS area (XOR-swizzled so that the row-wise writes and the
// operand-wise reads are free of bank conflicts) and come back as A operands:
//   y^T[weight row][batch row] += W[row][k .. k + 32) . x[batch row][k .. k + 32)
// with 16x16x32 bf16 MFMA, fp32 accumulation.  The walk is straight-line code (NB is a template
// parameter): the compiler's count of outstanding requests is then exact and a row block waits for
// its own rows only.  All of x and the first two row blocks are requested before anything is waited
// for (48 requests): x, mostly from L2, is back first and is arranged while the weight rows are
// still on their way from HBM.  Registers decide how far ahead the requests can run: the matrix
// instructions take A and B operands from the 256 architectural registers only, and once x (128),
// the row blocks in flight and the raw x rows add up to more than that the compiler parks arrived
// data in accumulator registers, which makes it wait for that data in the middle of the request
// sequence (three row blocks ahead measured 1.2-2 us slower than two for this reason).  No workgroup
// barrier until the end, where the four wavefronts add their accumulators through LDS.  With one
// slice the sums are rounded to bf16 and stored; with several, each workgroup leaves an fp32 partial
// tile in the workspace and a second, small kernel adds the slices in a fixed order (deterministic)
// and rounds once.  NB is chosen so that the launch has at least one workgroup per compute unit.
//
// Measured, fused QKV weight of 6144 x 4096 at M = 64: 14.0 us for the first kernel, 4.1 us for the
// second; in a replayed graph 16.7 us per call (W^O 4096 x 4096: 12.7 us).  Time stamps inside the
// first kernel: x in the registers 3.2 us after the first wavefront starts, the six row blocks done
// at 8.9 us (about 1 us per block: the 50 MB stream runs at 6 TB/s from the first request on), the
// accumulators added and stored at 10.5 us; the rest is the launch and the write-back at the
// kernel's end.
#include <string.h>
#include <hip/hip_ext.h>

#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
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
    int32_t splits;         // slices of the input dimension
    int32_t slice_slabs;    // 128-wide slabs per slice (at most 8)
    float* part;            // [splits][workgroup tile][NB * 4 tiles][64 lanes] f32x4 when splits > 1
};

// sum[i] = y[m0 + 16 cb + r][16 (blk0 + b) + 4 quad + i] for tile (b, cb) = (tile / 4, tile % 4) of a
// workgroup: rounded to bf16 and stored
template <int NB>
__device__ __forceinline__ void store_tile(const linear_args& p, f32x4 sum, int tile, int m0, int blk0, int n_blocks,
                                           int r, int quad)
{
    const int b = tile / kColBlocks, cb = tile % kColBlocks;
    const int m = m0 + 16 * cb + r;
    if (m >= p.M || blk0 + b >= n_blocks) return;
    uint2 pk;
    pk.x = pack_bf16x2(sum[0], sum[1]);
    pk.y = pack_bf16x2(sum[2], sum[3]);
    *reinterpret_cast<uint2*>(p.y + (int64_t)m * p.ldy + (16 * (blk0 + b) + 4 * quad)) = pk;
}

// The partial tiles of all slices of one workgroup tile, added in slice order and stored.  Wavefront
// w takes tiles w NB .. w NB + NB - 1.
template <int NB>
__device__ __forceinline__ void add_slices(const linear_args& p, int64_t wg_tiles, int64_t wg_tile, int m0, int blk0,
                                           int n_blocks, int wave, int lane)
{
    const int r = lane & 15, quad = lane >> 4;
    const int64_t slice_step = wg_tiles * (NB * kColBlocks) * 256;   // floats between two slices
    const float* src = p.part + ((wg_tile * (NB * kColBlocks) + wave * NB) * 64 + lane) * 4;
    f32x4 sum[NB];
#pragma unroll
    for (int t = 0; t < NB; ++t) sum[t] = f32x4{0.f, 0.f, 0.f, 0.f};
    // four slices of all this wavefront's tiles are requested before any is added: one memory round
    // trip per four slices
    for (int z0 = 0; z0 < p.splits; z0 += 4) {
        f32x4 v[NB][4];
#pragma unroll
        for (int t = 0; t < NB; ++t)
#pragma unroll
            for (int j = 0; j < 4; ++j)
                v[t][j] = *reinterpret_cast<const f32x4*>(src + t * 256 + (int64_t)min(z0 + j, p.splits - 1) * slice_step);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (z0 + j >= p.splits) break;
#pragma unroll
            for (int t = 0; t < NB; ++t) sum[t] += v[t][j];
        }
    }
#pragma unroll
    for (int t = 0; t < NB; ++t) store_tile<NB>(p, sum[t], wave * NB + t, m0, blk0, n_blocks, r, quad);
}

template <int NB>
__global__ __launch_bounds__(kThreads, 1) void linear_slice_kernel(linear_args p)
{
    constexpr int NR = 2;             // row blocks requested ahead
    constexpr int kStagePieces = 2 * 256;                       // per wavefront: 2 slabs x 16 rows x 16 pieces
    constexpr int kRedPieces = kWaves * NB * kColBlocks * 64;   // all accumulators, one f32x4 per lane each
    constexpr int kLdsPieces = kWaves * kStagePieces > kRedPieces ? kWaves * kStagePieces : kRedPieces;
    __shared__ kv_u32x4 s_mem[kLdsPieces];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int r = lane & 15, quad = lane >> 4;
    const int g = lane >> 4, pos = lane & 15;
    const int blk0 = blockIdx.x * NB;                 // first 16-row block of this workgroup
    const int m0 = blockIdx.y * (16 * kColBlocks);
    kv_u32x4* stage = s_mem + wave * kStagePieces;

    // this workgroup's slabs: [first, first + n); this wavefront's: first + w and first + w + 4
    const int total = p.Kl / kSlab;
    const int first = (int)blockIdx.z * p.slice_slabs;
    const int n = min(total, first + p.slice_slabs) - first;
    bool have[2];
    int64_t koff[2];   // byte offset of the slab inside a row; a missing slab reads the slice's first one
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        have[t] = wave + kWaves * t < n;
        koff[t] = (int64_t)(first + (have[t] ? wave + kWaves * t : 0)) * (kSlab * 2);
    }

    // Addresses are a base that is the same for the whole wavefront (scalar registers) plus one
    // 32-bit offset per lane.  One load instruction covers four rows, 256 contiguous bytes of each:
    // lane 16 g + pos fetches piece pos of row 4 i + g (whole cache lines: the arrangement the matrix
    // instruction wants, 64 bytes of each of 16 rows, costs the load path twice as long per byte).
    // A block past the last row, or a missing slab, asks for bytes of x instead (there and cached)
    // and multiplies by zero; the choice is made by arithmetic on the base and the lane offset, never
    // between two loads (a choice between loads is compiled into two paths with a wait each).
    const char* idle = reinterpret_cast<const char*>(p.x);
    const uint32_t idle_lane = (uint32_t)(pos << 4);
    const uint32_t wlane = (uint32_t)(g * p.ldw * 2 + (pos << 4));
    const int64_t wstep = 4 * p.ldw * 2;
    const int n_blocks = p.Nl >> 4;
    kv_u32x4 w_reg[NR][2][4];
    auto issue = [&](int b, int slot) {
        const int blk = blk0 + b;
        const int row = min(blk, n_blocks - 1) << 4;     // (a block never straddles two segments)
        int seg = 0;
        seg += (p.n_seg > 1 && row >= p.seg_first[1]);
        seg += (p.n_seg > 2 && row >= p.seg_first[2]);
        const int64_t phys = p.seg_start[seg] + (row - p.seg_first[seg]);
        const char* rows = reinterpret_cast<const char*>(p.w + phys * p.ldw + p.col_start);
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int64_t keep = -(int64_t)(blk < n_blocks && have[t]);
            const uint32_t lane_off = idle_lane + ((wlane - idle_lane) & (uint32_t)keep);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const char* base = idle + (((rows + koff[t] + i * wstep) - idle) & keep);
                w_reg[slot][t][i] = __builtin_nontemporal_load(reinterpret_cast<const kv_u32x4*>(base + lane_off));
            }
        }
    };
    // x, once: fetched like weight rows (16 batch rows x 1 slab at a time), passed through the private
    // LDS area and kept as B operands: x_reg[t][kk][cb] = the 16 bytes of batch row 16 cb + r, 32-wide
    // step kk of slab t, that lane (r, quad) contributes (rows past M repeat the last one)
    kv_u32x4 x_reg[2][4][kColBlocks];
    {
        const char* xbase = reinterpret_cast<const char*>(p.x);
        kv_u32x4 raw[2][kColBlocks][4];
#pragma unroll
        for (int cb = 0; cb < kColBlocks; ++cb)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t xlane = (uint32_t)(min(m0 + 16 * cb + 4 * i + g, p.M - 1) * p.ldx * 2 + (pos << 4));
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    raw[t][cb][i] = *reinterpret_cast<const kv_u32x4*>(xbase + koff[t] + xlane);
            }
        // the first weight rows are requested right behind x: x (mostly from L2) is back first and is
        // arranged while the weight rows are still on their way from HBM
#pragma unroll
        for (int b = 0; b < NR && b < NB; ++b) issue(b, b);
#pragma unroll
        for (int cb = 0; cb < kColBlocks; ++cb) {
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int row = 4 * i + g;
                    stage[t * 256 + row * 16 + (pos ^ row)] = raw[t][cb][i];
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) x_reg[t][kk][cb] = stage[t * 256 + r * 16 + ((4 * kk + quad) ^ r)];
            __builtin_amdgcn_wave_barrier();
        }
    }

    f32x4 acc[NB][kColBlocks];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int cb = 0; cb < kColBlocks; ++cb) acc[b][cb] = f32x4{0.f, 0.f, 0.f, 0.f};

#pragma unroll
    for (int b = 0; b < NB; ++b) {
        const int slot = b % NR;
        // registers -> private LDS area (piece q of row t at position q ^ t) -> A operands
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 4 * i + g;
                stage[t * 256 + row * 16 + (pos ^ row)] = w_reg[slot][t][i];
            }
        if (b + NR < NB) issue(b + NR, slot);
        // (LDS serves a wavefront's requests in order: the reads below see these writes, and the next
        // block's writes come after these reads)
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const bool real = have[t] && blk0 + b < n_blocks;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                kv_u32x4 a_op = stage[t * 256 + r * 16 + ((4 * kk + quad) ^ r)];
                if (!real) a_op = kv_u32x4{0u, 0u, 0u, 0u};
#pragma unroll
                for (int cb = 0; cb < kColBlocks; ++cb)
                    acc[b][cb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a_op), as_bf16x8(x_reg[t][kk][cb]),
                                                                        acc[b][cb], 0, 0, 0);
            }
        }
    }

    // the four wavefronts add up: each writes its accumulators, then sums NB of the 4 NB tiles
    __syncthreads();
    f32x4* red = reinterpret_cast<f32x4*>(s_mem);   // [wave][b][cb][lane]
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int cb = 0; cb < kColBlocks; ++cb) red[((wave * NB + b) * kColBlocks + cb) * 64 + lane] = acc[b][cb];
    __syncthreads();
    const int64_t wg_tiles = (int64_t)gridDim.x * gridDim.y;
    const int64_t wg_tile = (int64_t)blockIdx.y * gridDim.x + blockIdx.x;
#pragma unroll
    for (int t = 0; t < NB; ++t) {
        const int tile = wave * NB + t;           // of the 4 NB (b, cb) tiles
        const int b = tile / kColBlocks, cb = tile % kColBlocks;
        f32x4 sum = red[((0 * NB + b) * kColBlocks + cb) * 64 + lane];
#pragma unroll
        for (int k = 1; k < kWaves; ++k) sum += red[((k * NB + b) * kColBlocks + cb) * 64 + lane];
        if (p.splits > 1) {
            // partial tile, kept lane for lane as it lies in the registers: 1 KiB contiguous per store
            *reinterpret_cast<f32x4*>(
                p.part + ((((int64_t)blockIdx.z * wg_tiles + wg_tile) * (NB * kColBlocks) + tile) * 64 + lane) * 4) = sum;
        } else {
            store_tile<NB>(p, sum, tile, m0, blk0, n_blocks, r, quad);
        }
    }
}

// The second kernel of a launch with several slices: one workgroup per workgroup tile adds them.
// (Letting the last slice to arrive do this inside the first kernel was measured and gains nothing:
// partials that cross XCDs inside a kernel need write-through stores, their acknowledgement, an
// arrival counter and cache-bypassing loads, a chain as long as the second launch.)
template <int NB>
__global__ __launch_bounds__(kThreads) void linear_add_kernel(linear_args p)
{
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    add_slices<NB>(p, (int64_t)gridDim.x * gridDim.y, (int64_t)blockIdx.y * gridDim.x + blockIdx.x,
                   blockIdx.y * (16 * kColBlocks), blockIdx.x * NB, p.Nl >> 4, wave, lane);
}

// Slices of the input dimension and row blocks per workgroup.  A slice is what a workgroup can keep
// of x in registers: 8 slabs; NB is the largest of 8, 6, 4, 3, 2, 1 that still gives one workgroup
// per compute unit (more rows per workgroup use the resident piece of x for longer).
constexpr int kSliceSlabs = 2 * kWaves;
struct linear_cfg {
    int nb, splits, slice_slabs;
};
linear_cfg pick_cfg(int64_t m_tiles, int64_t n_l, int total_slabs)
{
    linear_cfg c;
    c.slice_slabs = total_slabs < kSliceSlabs ? total_slabs : kSliceSlabs;
    const int64_t forced = kv_option_linear_splits();   // test hook: at least this many slices
    if (forced > 0) {
        const int per = (int)((total_slabs + forced - 1) / forced);
        c.slice_slabs = per < 1 ? 1 : per > kSliceSlabs ? kSliceSlabs : per;
    }
    c.splits = (total_slabs + c.slice_slabs - 1) / c.slice_slabs;
    const int64_t blocks = n_l / 16;
    static const int kNb[] = {8, 6, 4, 3, 2, 1};
    c.nb = 1;
    for (int nb : kNb) {
        if (m_tiles * ((blocks + nb - 1) / nb) * c.splits >= 256) {
            c.nb = nb;
            break;
        }
    }
    return c;
}

// Workspace of a launch with several slices: one padded fp32 tile per slice and workgroup tile.
size_t part_bytes(const linear_cfg& c, int64_t m_tiles, int64_t n_l)
{
    if (c.splits <= 1) return 0;
    const int64_t n_tiles = (n_l / 16 + c.nb - 1) / c.nb;
    return (size_t)c.splits * m_tiles * n_tiles * c.nb * kColBlocks * 1024;
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
    const linear_cfg cfg = pick_cfg(m_tiles, n_l, (int)(view->col_count / kSlab));
    return part_bytes(cfg, m_tiles, n_l);
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
    const int64_t n_tiles = (n_l / 16 + cfg.nb - 1) / cfg.nb;
    // (per-lane offsets are 32 bits wide)
    if (n_tiles > 0x7fffffff || m_tiles > 65535 || (int64_t)M * ldx >= (1ll << 31) || ldw >= (1ll << 28))
        return KV_ERR_UNSUPPORTED;
    p.splits = cfg.splits;
    p.slice_slabs = cfg.slice_slabs;
    p.part = (float*)workspace;
    if (p.splits > 1) {
        if (!workspace || ((uintptr_t)workspace & 15)) return KV_ERR_INVALID_ARG;
        if (workspace_bytes < part_bytes(cfg, m_tiles, n_l)) return KV_ERR_WORKSPACE;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    const dim3 grid((unsigned)n_tiles, (unsigned)m_tiles, (unsigned)p.splits);
    // (while kv_profile is on, a single-kernel call is launched with events that take the kernel's own
    // start and end times; with a second kernel the two share a bracket of recorded events)
    hipEvent_t e0, e1;
    const bool own_events = p.splits == 1 && kv_prof_kernel_events(KV_PROF_LINEAR, &e0, &e1);
    const int slot = own_events ? -1 : kv_prof_begin(KV_PROF_LINEAR, st);
    auto go = [&](auto kernel) {
        if (own_events) hipExtLaunchKernelGGL(kernel, grid, dim3(kThreads), 0, st, e0, e1, 0, p);
        else hipLaunchKernelGGL(kernel, grid, dim3(kThreads), 0, st, p);
    };
    switch (cfg.nb) {
        case 8: go(linear_slice_kernel<8>); break;
        case 6: go(linear_slice_kernel<6>); break;
        case 4: go(linear_slice_kernel<4>); break;
        case 3: go(linear_slice_kernel<3>); break;
        case 2: go(linear_slice_kernel<2>); break;
        default: go(linear_slice_kernel<1>); break;
    }
    if (p.splits > 1) {
        const dim3 tiles((unsigned)n_tiles, (unsigned)m_tiles);
        switch (cfg.nb) {
            case 8: hipLaunchKernelGGL(linear_add_kernel<8>, tiles, dim3(kThreads), 0, st, p); break;
            case 6: hipLaunchKernelGGL(linear_add_kernel<6>, tiles, dim3(kThreads), 0, st, p); break;
            case 4: hipLaunchKernelGGL(linear_add_kernel<4>, tiles, dim3(kThreads), 0, st, p); break;
            case 3: hipLaunchKernelGGL(linear_add_kernel<3>, tiles, dim3(kThreads), 0, st, p); break;
            case 2: hipLaunchKernelGGL(linear_add_kernel<2>, tiles, dim3(kThreads), 0, st, p); break;
            default: hipLaunchKernelGGL(linear_add_kernel<1>, tiles, dim3(kThreads), 0, st, p); break;
        }
    }
    if (!own_events) kv_prof_end(KV_PROF_LINEAR, slot, st);
    return kv_record_hip_error(hipGetLastError(), "kv_linear_view launch");
}

