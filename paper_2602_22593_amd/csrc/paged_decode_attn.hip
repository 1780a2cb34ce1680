// paged_decode_attn: batched single-query attention over a paged bf16 KV pool read through a
// layout view (paper Sec. 2.1 attention over cached K/V; Sec. 4.2.2-4.2.3: blocks found through
// the logical table, kernel told the view's stride and capacity).
//
// Work decomposition (split-KV): a workgroup owns (sequence, local KV head, chunk of
// chunk_tokens tokens) and serves the G query heads of that KV head together, so every K/V
// byte is fetched from HBM once.  A sequence with one chunk is finished in place; otherwise
// each chunk leaves an un-normalised partial (m, l, acc[d]) in the workspace and a second small
// kernel merges them:  m = max m_k, l = sum l_k 2^(m_k - m), acc = sum acc_k 2^(m_k - m).
// Scores are kept in base-2 units (multiplied by scale * log2(e)).
//
// Two main kernels:
//   decode_mfma_kernel  head_dim 128, G <= 16, block capacity a multiple of 16: QK^T and PV on
//                       the matrix cores (16x16x32 bf16 MFMA), the query group padded to 16.
//   decode_valu_kernel  any G in {1,2,4,8}, head_dim 64 or 128, any block capacity: vector ALU.
#include <math.h>
#include <string.h>

#include <atomic>
#include <mutex>

#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;

struct decode_args {
    const uint16_t* q;
    uint16_t* out;
    const uint16_t* pool;
    const int32_t* table;
    int64_t table_stride;
    const int32_t* ctx_lens;
    kv_view_dev v;
    float scale_log2e;
    int32_t group;         // G = query heads per KV head
    int32_t chunk_tokens;
    int32_t max_chunks;
    float* part_acc;  // [batch][n_q_local][max_chunks][D]
    float* part_ml;   // [batch][n_q_local][max_chunks][2]
};

// Workgroup epilogue shared by both main kernels: the kWaves per-wave results for G heads sit in
// LDS (s_acc[w][g][e], s_ml[w][g][0..1]); combine them and write either the final bf16 row (the
// sequence has a single chunk) or this chunk's partial.
template <int D, int GMAX>
__device__ __forceinline__ void finish_chunk(const decode_args& a, float (&s_acc)[kWaves][GMAX][D],
                                             float (&s_ml)[kWaves][GMAX][2], int G, int s, int hl,
                                             int chunk, int n_chunks)
{
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
            a.out[((int64_t)s * a.v.n_q_local + qi) * D + e] = f32_to_bf16(o);
        } else {
            const int64_t rec = ((int64_t)s * a.v.n_q_local + qi) * a.max_chunks + chunk;
            a.part_acc[rec * D + e] = aa;
            if (e == 0) {
                a.part_ml[rec * 2 + 0] = mm;
                a.part_ml[rec * 2 + 1] = ll;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Matrix-core kernel (head_dim 128).  One wavefront walks tiles of 32 tokens of its chunk.
//
// Lane l = (r = l % 16, quad = l / 16).  Both products put the KV data in the MFMA A operand
// (row index = r) and the query group in the B operand (column index = r = query head g):
//   S^T[token][g] = K[token][:] . Q[g][:]     A = K rows: lane (r, quad) holds the 8 elements
//                                              [32 kk + 8 quad, +8) of row r, kk = 0..3
//   O^T[e][g]     = sum_t V[t][e] P[g][t]     A = V^T, B = P^T; contraction over the 32 tokens
// The C layout of S^T (lane (g, quad) holds tokens 4 quad + i of a 16-row half) is, element for
// element, the B layout the PV product needs if the contraction index k = 8 quad + 4 h + i stands
// for token 16 h + 4 i + quad; so row r of half h of the K operand is token 16 h + 4 (r % 4) + r / 4,
// and V is loaded row-wise (lane (c = r, quad) reads the 16 bytes [8c, 8c+8) of tokens
// 4 i' + quad, i' = 0..7) and transposed inside the lane with byte permutes.  No data crosses
// lanes except the running maximum.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kThreads, 2) void decode_mfma_kernel(decode_args a)
{
    constexpr int D = 128;
    const int chunk = blockIdx.x, hl = blockIdx.y, s = blockIdx.z;
    const int n = a.ctx_lens[s];
    const int cs = chunk * a.chunk_tokens;
    if (cs >= n && chunk != 0) return;
    const int ce = min(n, cs + a.chunk_tokens);
    const int n_chunks = (n + a.chunk_tokens - 1) / a.chunk_tokens;

    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int r = lane & 15, quad = lane >> 4;
    const int G = a.group;
    const kv_view_dev& v = a.v;
    const int32_t* trow = a.table + (int64_t)s * a.table_stride;

    // B operand of the score product: lane (g = r, quad) holds q[g][32 kk + 8 quad, +8)
    bf16x8 qb[4];
    {
        const uint16_t* qrow = a.q + ((int64_t)s * v.n_q_local + hl * G + min(r, G - 1)) * D;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kv_u32x4 raw = *reinterpret_cast<const kv_u32x4*>(qrow + kk * 32 + quad * 8);
            if (r >= G) raw = kv_u32x4{0u, 0u, 0u, 0u};
            qb[kk] = as_bf16x8(raw);
        }
    }

    float m_run = kNegInf, l_run = 0.f;
    f32x4 oacc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) oacc[j] = f32x4{0.f, 0.f, 0.f, 0.f};

    const uint16_t* kplane = a.pool + v.head_off + hl * D;
    const int k_row = 4 * (r & 3) + (r >> 2);  // token (within a 16-token half) held in A row r

    for (int t0 = cs + 32 * wave; t0 < ce; t0 += 32 * kWaves) {
        // the two 16-token halves of the tile each lie inside one block (capacity % 16 == 0)
        const uint16_t* hbase[2];
        int hstart[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int ts = min(t0 + 16 * h, ce - 1);
            int bj, slot;
            kv_split_token(v, ts, bj, slot);
            hstart[h] = ts - slot;  // first token of that block
            hbase[h] = kplane + (int64_t)trow[bj] * v.block_elems;
        }
        kv_u32x4 kA[2][4], vN[8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int tok = min(t0 + 16 * h + k_row, ce - 1);
            const uint16_t* p = hbase[h] + (tok - hstart[h]) * v.token_stride + quad * 8;
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) kA[h][kk] = *reinterpret_cast<const kv_u32x4*>(p + kk * 32);
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int h = i >> 2;
            const int tok = min(t0 + 4 * i + quad, ce - 1);
            const uint16_t* p = hbase[h] + v.plane_elems + (tok - hstart[h]) * v.token_stride + r * 8;
            vN[i] = *reinterpret_cast<const kv_u32x4*>(p);
        }

        // scores
        f32x4 sacc[2];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            sacc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                sacc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(kA[h][kk]), qb[kk], sacc[h], 0, 0, 0);
        }
        float sv[8];
        float mx = kNegInf;
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tok = t0 + 16 * h + 4 * i + quad;
                const float x = tok < ce ? sacc[h][i] * a.scale_log2e : kNegInf;
                sv[4 * h + i] = x;
                mx = fmaxf(mx, x);
            }
        mx = fmaxf(mx, __shfl_xor(mx, 16));
        mx = fmaxf(mx, __shfl_xor(mx, 32));
        const float m_new = fmaxf(m_run, mx);  // finite: every tile holds at least one valid token
        const float alpha = exp2f(m_run - m_new);
        m_run = m_new;
        uint32_t pw[4];
        float psum = 0.f;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const uint32_t b0 = f32_to_bf16_bits(exp2f(sv[2 * u] - m_new));
            const uint32_t b1 = f32_to_bf16_bits(exp2f(sv[2 * u + 1] - m_new));
            psum += __uint_as_float(b0 << 16) + __uint_as_float(b1 << 16);
            pw[u] = b0 | (b1 << 16);
        }
        l_run = l_run * alpha + psum;
        const bf16x8 pb = as_bf16x8(kv_u32x4{pw[0], pw[1], pw[2], pw[3]});
#pragma unroll
        for (int j = 0; j < 8; ++j) oacc[j] *= alpha;

        // V^T operands: element j of the 8 loaded rows, packed token-pair-wise
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            kv_u32x4 lo, hi;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                lo[u] = __builtin_amdgcn_perm(vN[2 * u + 1][w], vN[2 * u][w], 0x05040100u);
                hi[u] = __builtin_amdgcn_perm(vN[2 * u + 1][w], vN[2 * u][w], 0x07060302u);
            }
            oacc[2 * w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(lo), pb, oacc[2 * w], 0, 0, 0);
            oacc[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(hi), pb, oacc[2 * w + 1], 0, 0, 0);
        }
    }

    // per-lane partial sums of l over the 4 quads
    l_run += __shfl_xor(l_run, 16);
    l_run += __shfl_xor(l_run, 32);

    // lane (g = r, quad) holds O[g][32 quad + 8 i + j] in oacc[j][i]
    __shared__ float s_acc[kWaves][16][D];
    __shared__ float s_ml[kWaves][16][2];
    if (r < G) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float4 lo4 = make_float4(oacc[0][i], oacc[1][i], oacc[2][i], oacc[3][i]);
            float4 hi4 = make_float4(oacc[4][i], oacc[5][i], oacc[6][i], oacc[7][i]);
            float* dst = &s_acc[wave][r][32 * quad + 8 * i];
            *reinterpret_cast<float4*>(dst) = lo4;
            *reinterpret_cast<float4*>(dst + 4) = hi4;
        }
        if (quad == 0) {
            s_ml[wave][r][0] = m_run;
            s_ml[wave][r][1] = l_run;
        }
    }
    __syncthreads();
    finish_chunk<D, 16>(a, s_acc, s_ml, G, s, hl, chunk, n_chunks);
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
    finish_chunk<D, G>(a, s_acc, s_ml, G, s, hl, chunk, n_chunks);
}

// ---------------------------------------------------------------------------------------------
// Merge the partials of one (sequence, local query head).  256 lanes = 32 column groups of
// D/32 elements x 8 slices of the chunk list; maxima first, then one weighted pass.
// ---------------------------------------------------------------------------------------------
template <int D>
__global__ __launch_bounds__(256) void decode_merge_kernel(decode_args a)
{
    constexpr int EPT = D / 32;  // elements per lane
    const int qi = blockIdx.x, s = blockIdx.y;
    const int n = a.ctx_lens[s];
    const int n_chunks = (n + a.chunk_tokens - 1) / a.chunk_tokens;
    if (n_chunks <= 1) return;  // finished in place by the main kernel
    const int tid = threadIdx.x, cg = tid & 31, slice = tid >> 5;
    const int64_t rec0 = ((int64_t)s * a.v.n_q_local + qi) * a.max_chunks;

    __shared__ float s_red[8][D];
    __shared__ float s_l[8];
    __shared__ float s_max[4];
    float mm = kNegInf;
    for (int k = tid; k < n_chunks; k += 256) mm = fmaxf(mm, a.part_ml[(rec0 + k) * 2]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mm = fmaxf(mm, __shfl_xor(mm, off));
    if ((tid & 63) == 0) s_max[tid >> 6] = mm;
    __syncthreads();
    mm = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));

    float ll = 0.f, acc[EPT];
#pragma unroll
    for (int e = 0; e < EPT; ++e) acc[e] = 0.f;
    for (int k = slice; k < n_chunks; k += 8) {
        const float cw = exp2f(a.part_ml[(rec0 + k) * 2] - mm);
        ll += a.part_ml[(rec0 + k) * 2 + 1] * cw;
        const float* src = a.part_acc + (rec0 + k) * D + cg * EPT;
#pragma unroll
        for (int e = 0; e < EPT; ++e) acc[e] += src[e] * cw;
    }
#pragma unroll
    for (int e = 0; e < EPT; ++e) s_red[slice][cg * EPT + e] = acc[e];
    if (cg == 0) s_l[slice] = ll;
    __syncthreads();
    if (tid < D) {
        float tot = 0.f, lt = 0.f;
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            tot += s_red[w][tid];
            lt += s_l[w];
        }
        a.out[((int64_t)s * a.v.n_q_local + qi) * D + tid] = f32_to_bf16(tot / lt);
    }
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
void launch_valu(const decode_args& a, dim3 grid, hipStream_t st)
{
    hipLaunchKernelGGL((decode_valu_kernel<D, G>), grid, dim3(kThreads), 0, st, a);
}

template <int D>
int launch_valu_for_group(const decode_args& a, dim3 grid, hipStream_t st)
{
    switch (a.group) {
        case 1: launch_valu<D, 1>(a, grid, st); return KV_OK;
        case 2: launch_valu<D, 2>(a, grid, st); return KV_OK;
        case 4: launch_valu<D, 4>(a, grid, st); return KV_OK;
        case 8: launch_valu<D, 8>(a, grid, st); return KV_OK;
        default: return KV_ERR_UNSUPPORTED;
    }
}

// Which main kernel serves a call: 1 = matrix-core kernel with the even split over resident
// wavefronts, 2 = vector-ALU kernel (chunked), 3 = matrix-core kernel (chunked), 0 = none.
int pick_kernel(const kv_view* view, int batch)
{
    const int D = view->geom.head_dim, G = view->group;
    const bool mfma_ok = D == 128 && G <= 16 && view->block_tokens % 16 == 0;
    const bool streamk_ok = mfma_ok && batch <= KV_STREAMK_MAX_BATCH;
    const bool valu_ok = (D == 64 || D == 128) && (G == 1 || G == 2 || G == 4 || G == 8);
    const int64_t forced = kv_option_force_kernel();
    if (forced == 1) return streamk_ok ? 1 : 0;
    if (forced == 2) return valu_ok ? 2 : 0;
    if (forced == 3) return mfma_ok ? 3 : 0;
    if (streamk_ok) return 1;
    if (mfma_ok) return 3;
    return valu_ok ? 2 : 0;
}

// Wavefronts the even-split kernel launches: all resident at once, one per SIMD by default
// (fewer, fatter streams measured faster than more, thinner ones).  The compute-unit count is that
// of the device current on the calling thread, asked once per device.
int streamk_waves()
{
    constexpr int kDevices = 64;
    static std::atomic<int> cus[kDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kDevices) dev = 0;
    int n = cus[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        cus[dev].store(n, std::memory_order_relaxed);
    }
    int64_t per_cu = kv_option_waves_per_cu();
    if (per_cu <= 0) per_cu = 4;
    return (int)(n * per_cu);
}

size_t chunked_workspace_bytes(const kv_view* view, int batch, int max_ctx_len)
{
    const int chunk = pick_chunk_tokens(view, batch, max_ctx_len);
    const int64_t max_chunks = ((int64_t)max_ctx_len + chunk - 1) / chunk;
    if (max_chunks <= 1) return KV_DECODE_SYNC_BYTES + 256;
    const int64_t recs = (int64_t)batch * view->n_q_local * max_chunks;
    return KV_DECODE_SYNC_BYTES + align_up((size_t)recs * view->geom.head_dim * 4, 256) +
           align_up((size_t)recs * 2 * 4, 256);
}

// The even-split matrix-core kernel.  views/view_ids non-null: sequence s is laid out as
// views[view_ids[s]] says (all of them expose the same heads as `view`).
static int launch_streamk(const void* q, void* out, const void* kv_pool, const int32_t* block_table,
                          int64_t block_table_stride, const int32_t* ctx_lens, int batch,
                          int max_ctx_len, const kv_view* view, float sc, void* workspace,
                          size_t workspace_bytes, hipStream_t st, const int32_t* view_ids,
                          const kv_view* const* views, int n_views)
{
    // tiles (of 8 tokens at the least) over all (sequence, head) pairs must fit 31 bits
    if (((int64_t)max_ctx_len / 8 + 1) * batch * view->n_kv_local >= ((int64_t)1 << 31))
        return KV_ERR_UNSUPPORTED;
    // and the weighted length of one sequence's pairs (8 units per tile plus a cost per pair) 32 bits
    if (((int64_t)max_ctx_len + 8 + 64) * 8 * view->n_kv_local >= ((int64_t)1 << 31))
        return KV_ERR_UNSUPPORTED;
    const int n_waves = streamk_waves();
    const size_t need_sk = kv_streamk_workspace_bytes(view, batch, n_waves);
    if (!workspace) return KV_ERR_INVALID_ARG;
    if (workspace_bytes < need_sk) return KV_ERR_WORKSPACE;
    if (((uintptr_t)workspace & 255u) != 0) return KV_ERR_INVALID_ARG;
    kv_streamk_args k;
    k.q = (const uint16_t*)q;
    k.out = (uint16_t*)out;
    k.pool = (const uint16_t*)kv_pool;
    k.table = block_table;
    k.table_stride = block_table_stride;
    k.ctx_lens = ctx_lens;
    k.v = kv_view_to_dev(view);
    k.scale_log2e = sc * 1.4426950408889634f;
    k.group = view->group;
    k.batch = batch;
    k.n_waves = n_waves;
    k.part_acc = nullptr;
    k.part_ml = nullptr;
    k.pair_desc = nullptr;
    k.view_ids = view_ids;
    k.n_views = view_ids ? n_views : 1;
    for (int i = 0; i < KV_MAX_MIXED_VIEWS; ++i) {
        const kv_view_dev d = kv_view_to_dev(view_ids && i < n_views ? views[i] : view);
        k.lay[i] = kv_layout_dev{d.block_tokens, d.block_shift, d.token_stride, d.head_off};
    }
    return kv_streamk_launch(k, view, workspace, st);
}

}  // namespace

extern "C" size_t paged_decode_attn_workspace_bytes(const kv_view* view, int batch, int max_ctx_len)
{
    if (!kv_view_ok(view) || batch <= 0 || max_ctx_len <= 0) return KV_DECODE_SYNC_BYTES + 256;
    const int kernel = pick_kernel(view, batch);
    if (kernel == 1) return kv_streamk_workspace_bytes(view, batch, streamk_waves());
    return chunked_workspace_bytes(view, batch, max_ctx_len);
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
    const int D = view->geom.head_dim;
    const int kernel = pick_kernel(view, batch);
    if (kernel == 0) return KV_ERR_UNSUPPORTED;
    if (batch > 65535 || view->n_kv_local > 65535) return KV_ERR_UNSUPPORTED;
    const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)D);
    hipStream_t st = (hipStream_t)hip_stream;

    if (kernel == 1 && max_ctx_len > 0)
        return launch_streamk(q, out, kv_pool, block_table, block_table_stride, ctx_lens, batch,
                              max_ctx_len, view, sc, workspace, workspace_bytes, st, nullptr, nullptr, 1);

    const int chunk = pick_chunk_tokens(view, batch, max_ctx_len);
    int64_t max_chunks = ((int64_t)max_ctx_len + chunk - 1) / chunk;
    if (max_chunks < 1) max_chunks = 1;
    const size_t need = chunked_workspace_bytes(view, batch, max_ctx_len);
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
    a.scale_log2e = sc * 1.4426950408889634f;
    a.group = view->group;
    a.chunk_tokens = chunk;
    a.max_chunks = (int32_t)max_chunks;
    const int64_t recs = (int64_t)batch * view->n_q_local * max_chunks;
    // (the chunked kernels keep off the arrival words at the start of the workspace)
    char* ws_base = workspace ? (char*)workspace + KV_DECODE_SYNC_BYTES : nullptr;
    a.part_acc = (float*)ws_base;
    a.part_ml = max_chunks > 1 ? (float*)(ws_base + align_up((size_t)recs * D * 4, 256)) : nullptr;

    const dim3 grid((unsigned)max_chunks, (unsigned)view->n_kv_local, (unsigned)batch);
    int slot = kv_prof_begin(KV_PROF_DECODE_MAIN, st);
    int rc = KV_OK;
    if (kernel == 3 || kernel == 1)
        hipLaunchKernelGGL(decode_mfma_kernel, grid, dim3(kThreads), 0, st, a);
    else
        rc = (D == 128) ? launch_valu_for_group<128>(a, grid, st) : launch_valu_for_group<64>(a, grid, st);
    if (rc) return rc;
    kv_prof_end(KV_PROF_DECODE_MAIN, slot, st);
    rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn launch");
    if (rc) return rc;
    if (max_chunks > 1) {
        slot = kv_prof_begin(KV_PROF_DECODE_MERGE, st);
        dim3 mgrid((unsigned)view->n_q_local, (unsigned)batch);
        if (D == 128)
            hipLaunchKernelGGL(decode_merge_kernel<128>, mgrid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(decode_merge_kernel<64>, mgrid, dim3(256), 0, st, a);
        kv_prof_end(KV_PROF_DECODE_MERGE, slot, st);
        rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn merge launch");
    }
    return rc;
}

// ---- paged_decode_attn for callers that cannot allocate ------------------------------------------
// The scratch memory of the decode kernels (partial results of the pieces, pair descriptors) lives in
// a file-scope device array instead of a caller's workspace.  Every GPU holds its own copy of the
// array at its own address: in host code the array's name is only a handle for
// hipGetSymbolAddress, which is asked once per device, with that device current; the pointer it
// returns is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[KV_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void* g_scratch_ptr[kMaxDevices];   // device address of `scratch` on device i, null until asked

int static_scratch(void** out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return kv_record_hip_error(e, "paged_decode_attn_static: hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return KV_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return kv_record_hip_error(e != hipSuccess ? e : hipErrorInvalidSymbol,
                                       "paged_decode_attn_static: hipGetSymbolAddress");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return KV_OK;
}
}  // namespace

extern "C" int paged_decode_attn_static(const void* q, void* out, const void* kv_pool,
                                        int64_t n_pool_blocks, const int32_t* block_table,
                                        int64_t block_table_stride, const int32_t* ctx_lens, int batch,
                                        int max_ctx_len, const kv_view* view, float scale,
                                        void* hip_stream)
{
    if (!kv_view_ok(view) || batch < 0 || max_ctx_len < 0) return KV_ERR_INVALID_ARG;
    if (batch == 0) return KV_OK;
    if (paged_decode_attn_workspace_bytes(view, batch, max_ctx_len) > (size_t)KV_STATIC_SCRATCH_BYTES)
        return KV_ERR_WORKSPACE;
    void* ws = nullptr;
    const int rc = static_scratch(&ws);
    if (rc) return rc;
    return paged_decode_attn(q, out, kv_pool, n_pool_blocks, block_table, block_table_stride, ctx_lens,
                             batch, max_ctx_len, view, scale, ws, (size_t)KV_STATIC_SCRATCH_BYTES,
                             hip_stream);
}


extern "C" int paged_decode_attn_mixed(const void* q, void* out, const void* kv_pool,
                                       int64_t n_pool_blocks, const int32_t* block_table,
                                       int64_t block_table_stride, const int32_t* ctx_lens,
                                       const int32_t* view_ids, int batch, int max_ctx_len,
                                       const kv_view* const* views, int n_views, float scale,
                                       void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!views || n_views < 1 || n_views > KV_MAX_MIXED_VIEWS) return KV_ERR_INVALID_ARG;
    for (int i = 0; i < n_views; ++i)
        if (!kv_view_ok(views[i])) return KV_ERR_INVALID_ARG;
    const kv_view* v0 = views[0];
    int min_block = v0->block_tokens;
    for (int i = 1; i < n_views; ++i) {
        const kv_view* v = views[i];
        // one pool, one head range: the views may differ only in how a block lays its tokens out
        if (memcmp(&v->geom, &v0->geom, sizeof(kv_geometry)) != 0 || v->p != v0->p || v->r != v0->r)
            return KV_ERR_INVALID_ARG;
        if (v->block_tokens < min_block) min_block = v->block_tokens;
    }
    if (n_views == 1 || batch <= 0 || max_ctx_len <= 0)
        return paged_decode_attn(q, out, kv_pool, n_pool_blocks, block_table, block_table_stride,
                                 ctx_lens, batch, max_ctx_len, v0, scale, workspace, workspace_bytes,
                                 hip_stream);
    if (n_pool_blocks < 0 || block_table_stride < 0) return KV_ERR_INVALID_ARG;
    if (!q || !out || !ctx_lens || !view_ids || !kv_pool || !block_table) return KV_ERR_INVALID_ARG;
    if (block_table_stride < ((int64_t)max_ctx_len + min_block - 1) / min_block) return KV_ERR_INVALID_ARG;
    for (int i = 0; i < n_views; ++i)
        if (pick_kernel(views[i], batch) != 1) return KV_ERR_UNSUPPORTED;
    if (batch > 65535 || v0->n_kv_local > 65535) return KV_ERR_UNSUPPORTED;
    const float sc = scale > 0.f ? scale : 1.0f / sqrtf((float)v0->geom.head_dim);
    return launch_streamk(q, out, kv_pool, block_table, block_table_stride, ctx_lens, batch, max_ctx_len,
                          v0, sc, workspace, workspace_bytes, (hipStream_t)hip_stream, view_ids, views,
                          n_views);
}
