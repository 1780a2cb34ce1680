// Matrix-core decode attention with an even split of the whole batch over resident wavefronts.
//
// The batch is flattened into tiles of 32 tokens of one (sequence, local KV head) pair, pairs
// ordered (sequence, head) with the head fastest.  With T tiles in total and W wavefronts
// launched, wavefront w owns tiles [w * ceil(T / W), (w + 1) * ceil(T / W)): every wavefront
// streams the same number of KV bytes whatever the mix of context lengths, and lives long
// enough to amortise its start-up (the grid is sized so that all W wavefronts are resident at
// once).  A wavefront's range may cover the end of one pair and the start of the next; each
// (wavefront, pair) piece yields either the final output row (the piece is the whole pair) or an
// un-normalised partial (m, l, acc[G][d]) in workspace slot w + pair_index, which is unique
// and keeps the pieces of a pair in consecutive slots for the merge kernel.
//
// Per tile, lane l = (r = l % 16, quad = l / 16).  Both products put the KV data in the MFMA
// A operand (row index r) and the query group, padded to 16, in the B operand (column r = g):
//   S^T[token][g] = K[token][:] . q[g][:]    lane (r, quad) holds elements [32 kk + 8 quad, +8)
//                                             of A row r, kk = 0..3
//   O^T[e][g]     = sum_t V[t][e] P[g][t]    contraction over the 32 tokens of the tile
// The C layout of S^T (lane (g, quad), half h, i = 0..3 <-> A row 4 quad + i) is already the B
// layout of the second product if contraction index k = 8 quad + 4 h + i stands for token
// 16 h + 4 i + quad: so A row r of half h is token 16 h + 4 (r % 4) + r / 4, V rows are loaded
// as they lie in memory (lane (c = r, quad) reads bytes [16 c, 16 c + 16) of tokens 4 i' + quad)
// and transposed inside the lane with byte permutes.  Only the running maximum crosses lanes.
#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kSkThreads = 256;
constexpr int kSkWaves = kSkThreads / 64;
constexpr int kMaxBatch = KV_STREAMK_MAX_BATCH;
constexpr int D = 128;

struct tile_regs {
    kv_u32x4 k[2][4];  // [half][kk]
    kv_u32x4 v[8];     // token 4 i + quad
};

// K/V bytes are used once per call: fetch them with the streaming (non-temporal) policy so that
// they do not displace each other in the cache hierarchy on their way through.
// `base` is the same for the whole wavefront, `byte_off` a 32-bit per-lane offset: the form the
// hardware addresses with a scalar base register pair plus one vector offset register.
__device__ __forceinline__ kv_u32x4 ld16(const char* base, uint32_t byte_off)
{
    return __builtin_nontemporal_load(reinterpret_cast<const kv_u32x4*>(base + byte_off));
}
__device__ __forceinline__ kv_u32x4 ld16_cached(const char* base, uint32_t byte_off)
{
    return *reinterpret_cast<const kv_u32x4*>(base + byte_off);
}

struct lane_consts {
    int r, quad;
    uint32_t koff;   // byte offset of this lane's K piece from the start of a 16-token half
    uint32_t voff;   // byte offset of this lane's V piece (token `quad` of a half)
    uint32_t vstep;  // bytes between V tokens 4 apart
};

// Full tile: both halves lie in one block each; kb[h] points at (block, first slot of the half,
// this head) in the K plane.  KMODE 0: K pieces are fetched directly in the MFMA operand
// arrangement (k[h][kk]); KMODE 1: K rows are fetched as they lie in memory, like V (k[h][i] =
// bytes [16 r, +16) of token 16 h + 4 i + quad), and re-arranged through LDS before use.
template <int KMODE>
__device__ __forceinline__ void load_full(tile_regs& t, const char* const (&kb)[2],
                                          int64_t plane_bytes, const lane_consts& lc)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            t.k[h][kk] = KMODE == 0 ? ld16(kb[h], lc.koff + kk * 64) : ld16(kb[h], lc.voff + kk * lc.vstep);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        const char* vb = kb[h] + plane_bytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) t.v[4 * h + i] = ld16(vb, lc.voff + i * lc.vstep);
    }
}

// Last, partial tile of a pair: rows past the last valid token are replaced by that token's row
// (finite data; their scores are masked).  `last` = index of the last valid token in the tile.
template <int KMODE>
__device__ __forceinline__ void load_tail(tile_regs& t, const char* const (&kb)[2],
                                          int64_t plane_bytes, const lane_consts& lc, int last,
                                          int token_stride_bytes)
{
    const int k_row = 4 * (lc.r & 3) + (lc.r >> 2);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // half h starts at token 16 h of the tile; if it holds no valid token its base was set
        // to the block of the last valid token by the caller and everything clamps to `last`
        const int first = (16 * h <= last) ? 16 * h : last;
        const int row = min(16 * h + k_row, last) - first;
        const uint32_t off = (uint32_t)(row * token_stride_bytes + lc.quad * 16);
        if (KMODE == 0) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) t.k[h][kk] = ld16(kb[h], off + kk * 64);
        }
        const char* vb = kb[h] + plane_bytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int vrow = min(16 * h + 4 * i + lc.quad, last) - first;
            const uint32_t voff = (uint32_t)(vrow * token_stride_bytes + lc.r * 16);
            t.v[4 * h + i] = ld16(vb, voff);
            if (KMODE == 1) t.k[h][i] = ld16(kb[h], voff);
        }
    }
}

struct softmax_state {
    float m, l;
    f32x4 o[8];  // o[j][i] = O[g = r][32 quad + 8 i + j]
};

// LDS staging of a K tile (KMODE 1), private to the wavefront: 32 rows of 16 16-byte pieces; piece c
// of row t is kept at position c ^ (t % 16), which makes both the row-wise writes and the
// operand-wise reads free of bank conflicts.
template <bool TAIL, int KMODE>
__device__ __forceinline__ void compute_tile(const tile_regs& t, const bf16x8 (&qb)[4],
                                             softmax_state& st, float scale_log2e, int last,
                                             int r, int quad, kv_u32x4* kstage)
{
    f32x4 sacc[2];
    if (KMODE == 1) {
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 16 * h + 4 * i + quad;
                kstage[row * 16 + (r ^ (row & 15))] = t.k[h][i];
            }
        __builtin_amdgcn_wave_barrier();
    }
    const int k_row = 4 * (r & 3) + (r >> 2);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        sacc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kv_u32x4 ka;
            if (KMODE == 1)
                ka = kstage[(16 * h + k_row) * 16 + ((4 * kk + quad) ^ k_row)];
            else
                ka = t.k[h][kk];
            sacc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka), qb[kk], sacc[h], 0, 0, 0);
        }
    }
    if (KMODE == 1) __builtin_amdgcn_wave_barrier();
    float sv[8];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float x = sacc[h][i] * scale_log2e;
            if (TAIL) x = (16 * h + 4 * i + quad <= last) ? x : kNegInf;
            sv[4 * h + i] = x;
        }
    float mx = fmaxf(fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3])),
                     fmaxf(fmaxf(sv[4], sv[5]), fmaxf(sv[6], sv[7])));
    mx = fmaxf(mx, __shfl_xor(mx, 16));
    mx = fmaxf(mx, __shfl_xor(mx, 32));
    const float m_new = fmaxf(st.m, mx);  // finite: the tile holds at least one valid token
    if (__builtin_amdgcn_ballot_w64(m_new != st.m) != 0) {
        const float alpha = fast_exp2(st.m - m_new);
        st.l *= alpha;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[j] *= alpha;
        st.m = m_new;
    }
    float p[8], psum = 0.f;
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        p[u] = fast_exp2(sv[u] - m_new);
        psum += p[u];
    }
    st.l += psum;
    const bf16x8 pb = as_bf16x8(kv_u32x4{pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]),
                                         pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])});
    // V^T operands: element j of the 8 loaded rows, token pairs packed per dword
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        kv_u32x4 lo, hi;
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            lo[u] = __builtin_amdgcn_perm(t.v[2 * u + 1][w], t.v[2 * u][w], 0x05040100u);
            hi[u] = __builtin_amdgcn_perm(t.v[2 * u + 1][w], t.v[2 * u][w], 0x07060302u);
        }
        st.o[2 * w] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(lo), pb, st.o[2 * w], 0, 0, 0);
        st.o[2 * w + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(hi), pb, st.o[2 * w + 1], 0, 0, 0);
    }
}

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

template <int KMODE, int PIPE, bool MIXED>
__global__ __launch_bounds__(kSkThreads, PIPE ? 2 : 3) void decode_streamk_kernel(kv_streamk_args a)
{
    __shared__ kv_u32x4 s_kstage[KMODE == 1 ? kSkWaves * 512 : 1];
    __shared__ int32_t s_prefix[kMaxBatch + 1];  // tiles of the sequences before s
    __shared__ int32_t s_ctx[kMaxBatch];
    __shared__ int32_t s_wsum[kSkWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const kv_view_dev& v = a.v;
    const int Hl = v.n_kv_local, G = a.group;

    // ---- exclusive prefix sum of tiles per sequence (whole workgroup) --------------------------
    {
        const int per = (a.batch + kSkThreads - 1) / kSkThreads;
        const int s0 = tid * per;
        int local = 0;
        for (int k = 0; k < per; ++k) {
            const int s = s0 + k;
            if (s < a.batch) {
                const int c = a.ctx_lens[s];
                s_ctx[s] = c;
                local += (c + 31) >> 5;
            }
        }
        int incl = local;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        if (lane == 63) s_wsum[wave] = incl;
        __syncthreads();
        int before = 0;
        for (int w = 0; w < wave; ++w) before += s_wsum[w];
        int run = before + incl - local;
        for (int k = 0; k < per; ++k) {
            const int s = s0 + k;
            if (s < a.batch) {
                s_prefix[s] = run;
                run += (s_ctx[s] + 31) >> 5;
            }
        }
        if (tid == kSkThreads - 1) s_prefix[a.batch] = before + incl;
        __syncthreads();
        // the merge kernel needs the same numbers: the first workgroup leaves them in the workspace
        if (blockIdx.x == 0)
            for (int k = tid; k <= a.batch; k += kSkThreads) a.prefix_out[k] = s_prefix[k];
    }

    // ---- this wavefront's share ---------------------------------------------------------------
    const int total = uniform(s_prefix[a.batch]) * Hl;
    const int tpw = (total + a.n_waves - 1) / a.n_waves;
    const int w = blockIdx.x * kSkWaves + wave;
    int x0 = w * tpw;
    const int x1 = min(x0 + tpw, total);
    if (x0 >= x1) return;

    // sequence holding tile x0: largest s with prefix[s] * Hl <= x0
    int s;
    {
        int lo = 0, hi = a.batch;
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (uniform(s_prefix[mid]) * Hl <= x0) lo = mid; else hi = mid;
        }
        s = lo;
    }
    int tiles_s = uniform(s_prefix[s + 1]) - uniform(s_prefix[s]);
    int hl, tile;
    {
        const int rem = x0 - uniform(s_prefix[s]) * Hl;
        hl = rem / tiles_s;
        tile = rem - hl * tiles_s;
    }

    lane_consts lc;
    lc.r = lane & 15;
    lc.quad = lane >> 4;
    const int64_t plane_bytes = v.plane_elems * 2;
    // layout of the current sequence's blocks (MIXED: looked up per sequence; else the view's own)
    kv_layout_dev lay = {v.block_tokens, v.block_shift, v.token_stride, v.head_off};
    int token_stride_bytes, halves_per_block, half_shift;
    auto use_layout = [&]() {
        token_stride_bytes = lay.token_stride * 2;
        lc.koff = (uint32_t)((4 * (lc.r & 3) + (lc.r >> 2)) * token_stride_bytes + lc.quad * 16);
        lc.voff = (uint32_t)(lc.quad * token_stride_bytes + lc.r * 16);
        lc.vstep = (uint32_t)(4 * token_stride_bytes);
        halves_per_block = lay.block_tokens >> 4;  // capacity is a multiple of 16
        half_shift = lay.block_shift >= 4 ? lay.block_shift - 4 : -1;
    };
    use_layout();

    while (x0 < x1) {
        if (MIXED) {
            const int vid = min(max(uniform(a.view_ids[s]), 0), a.n_views - 1);
            lay = a.lay[vid];
            use_layout();
        }
        const int n = uniform(s_ctx[s]);
        const int seg_end = min(tiles_s, tile + (x1 - x0));
        const int n_full = n >> 5;                 // tiles of this pair with all 32 tokens valid
        const int full_end = min(seg_end, n_full);
        const int32_t* trow = a.table + (int64_t)s * a.table_stride;
        const char* head_base = reinterpret_cast<const char*>(a.pool + lay.head_off + hl * D);
        const int last_block = (n - 1) / lay.block_tokens;

        bf16x8 qb[4];
        {
            const char* qrows = reinterpret_cast<const char*>(a.q + ((int64_t)s * v.n_q_local + hl * G) * D);
            const uint32_t qoff = (uint32_t)(min(lc.r, G - 1) * (D * 2) + lc.quad * 16);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                kv_u32x4 raw = ld16_cached(qrows, qoff + kk * 64);
                if (lc.r >= G) raw = kv_u32x4{0u, 0u, 0u, 0u};
                qb[kk] = as_bf16x8(raw);
            }
        }
        softmax_state st;
        st.m = kNegInf;
        st.l = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[j] = f32x4{0.f, 0.f, 0.f, 0.f};

        // block ids of 64 consecutive 16-token halves, one per lane, refilled every 32 tiles
        int id_base = 2 * tile;
        auto half_block = [&](int hh) -> int {  // index of the block holding 16-token half hh
            return half_shift >= 0 ? (hh >> half_shift) : hh / halves_per_block;
        };
        int idv = trow[min(half_block(id_base + lane), last_block)];
        auto half_base = [&](int hh) -> const char* {
            if (hh - id_base >= 64) {
                id_base = hh;
                idv = trow[min(half_block(id_base + lane), last_block)];
            }
            const int blk = __builtin_amdgcn_readlane(idv, hh - id_base);
            const int slot0 = (hh - half_block(hh) * halves_per_block) << 4;
            return head_base + (int64_t)blk * (v.block_elems * 2) + (int64_t)slot0 * token_stride_bytes;
        };

        kv_u32x4* kstage = s_kstage + (KMODE == 1 ? wave * 512 : 0);
        tile_regs ta;
        int i = tile;
        if (PIPE) {
            tile_regs tb;
            if (i < full_end) {
                const char* kb[2] = {half_base(2 * i), half_base(2 * i + 1)};
                load_full<KMODE>(ta, kb, plane_bytes, lc);
            }
            while (i + 2 <= full_end) {
                {
                    const char* kb[2] = {half_base(2 * i + 2), half_base(2 * i + 3)};
                    load_full<KMODE>(tb, kb, plane_bytes, lc);
                }
                compute_tile<false, KMODE>(ta, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
                if (i + 2 < full_end) {
                    const char* kb[2] = {half_base(2 * i + 4), half_base(2 * i + 5)};
                    load_full<KMODE>(ta, kb, plane_bytes, lc);
                }
                compute_tile<false, KMODE>(tb, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
                i += 2;
            }
            if (i < full_end) {
                compute_tile<false, KMODE>(ta, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
                ++i;
            }
        } else {
            for (; i < full_end; ++i) {
                const char* kb[2] = {half_base(2 * i), half_base(2 * i + 1)};
                load_full<KMODE>(ta, kb, plane_bytes, lc);
                compute_tile<false, KMODE>(ta, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
            }
        }
        if (seg_end > full_end) {
            // the pair's last tile, partly filled: tokens 32 * n_full .. n - 1
            const int last = n - 1 - 32 * n_full;  // 0..30
            const char* kb[2];
            kb[0] = half_base(2 * n_full);
            if (16 <= last) {
                kb[1] = half_base(2 * n_full + 1);
            } else {
                // second half empty: point it at the row of the last valid token
                kb[1] = kb[0] + (int64_t)last * token_stride_bytes;
            }
            load_tail<KMODE>(ta, kb, plane_bytes, lc, last, token_stride_bytes);
            compute_tile<true, KMODE>(ta, qb, st, a.scale_log2e, last, lc.r, lc.quad, kstage);
        }

        // ---- piece done: final row or partial ---------------------------------------------------
        st.l += __shfl_xor(st.l, 16);
        st.l += __shfl_xor(st.l, 32);
        const bool whole = (tile == 0 && seg_end == tiles_s);
        if (lc.r < G) {
            if (whole) {
                const float inv = 1.0f / st.l;
                uint16_t* dst = a.out + ((int64_t)s * v.n_q_local + hl * G + lc.r) * D + 32 * lc.quad;
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    kv_u32x4 pk;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
                        pk[u] = pack_bf16x2(st.o[2 * u][ii] * inv, st.o[2 * u + 1][ii] * inv);
                    *reinterpret_cast<kv_u32x4*>(dst + 8 * ii) = pk;
                }
            } else {
                const int64_t slot = (int64_t)w + (int64_t)s * Hl + hl;
                float* dst = a.part_acc + (slot * G + lc.r) * D + 32 * lc.quad;
#pragma unroll
                for (int ii = 0; ii < 4; ++ii) {
                    *reinterpret_cast<f32x4*>(dst + 8 * ii) =
                        f32x4{st.o[0][ii], st.o[1][ii], st.o[2][ii], st.o[3][ii]};
                    *reinterpret_cast<f32x4*>(dst + 8 * ii + 4) =
                        f32x4{st.o[4][ii], st.o[5][ii], st.o[6][ii], st.o[7][ii]};
                }
                if (lc.quad == 0) {
                    a.part_ml[(slot * G + lc.r) * 2 + 0] = st.m;
                    a.part_ml[(slot * G + lc.r) * 2 + 1] = st.l;
                }
            }
        }

        // ---- next pair ------------------------------------------------------------------------------
        x0 += seg_end - tile;
        tile = 0;
        if (++hl == Hl) {
            hl = 0;
            do {
                ++s;
                tiles_s = (s < a.batch) ? uniform(s_prefix[s + 1]) - uniform(s_prefix[s]) : 1;
            } while (tiles_s == 0);
        }
    }
}

// Merge the pieces of one (sequence, local query head), or write zeros for an empty context.
// The 256 lanes of a workgroup are column groups of 4 elements x slices of the piece list.  A
// short list (the common case: a pair cut over a few wavefronts) is merged by one workgroup as
// 32 column groups x 8 slices; a long one (one sequence cut over hundreds of wavefronts) by
// kMergeSplit workgroups, each owning 128 / kMergeSplit columns as 8 column groups x 32 slices.
// The host launches kMergeSplit workgroups per row only when the batch has few pairs for the
// wavefronts launched (long lists are then the rule); in such a grid all but the first leave at
// once for a short list.  Recomputes the split exactly as the main kernel did, from the per-sequence tile
// prefix that kernel left behind.
constexpr int kMergeSplit = 4;
constexpr int kMergeLong = 24;  // pieces from which a list counts as long
__global__ __launch_bounds__(256) void decode_streamk_merge_kernel(kv_streamk_args a)
{
    const int qi = blockIdx.x, s = blockIdx.y, z = blockIdx.z, tid = threadIdx.x;
    const kv_view_dev& v = a.v;
    const int Hl = v.n_kv_local, G = a.group;
    __shared__ float s_max[4];
    __shared__ float s_acc[8 * D];
    __shared__ float s_l[32];
    // tiles before sequence s and in total, as computed by the main kernel
    const int before = a.prefix_out[s];
    const int all = a.prefix_out[a.batch];

    const int n = a.ctx_lens[s];
    uint16_t* dst = a.out + ((int64_t)s * v.n_q_local + qi) * D;
    if (n == 0) {
        if (z == 0 && tid < D) dst[tid] = 0;
        return;
    }
    const int tiles_s = (n + 31) >> 5;
    const int hl = qi / G, g = qi - hl * G;
    const int total = all * Hl;
    const int tpw = (total + a.n_waves - 1) / a.n_waves;
    const int p0 = before * Hl + hl * tiles_s;          // first tile of the pair, flattened
    const int w_first = p0 / tpw, w_last = (p0 + tiles_s - 1) / tpw;
    if (w_first == w_last) return;                      // written in place by the main kernel
    const bool wide = (gridDim.z > 1 && w_last - w_first + 1 >= kMergeLong);
    if (!wide && z != 0) return;
    const int64_t pair = (int64_t)s * Hl + hl;
    const int ncg = wide ? D / 4 / kMergeSplit : D / 4;  // column groups of this workgroup
    const int cols = ncg * 4, nsl = 256 / ncg;
    const int col0 = wide ? z * cols : 0;
    const int cg = tid % ncg, slice = tid / ncg;

    float mm = kNegInf;
    for (int w = w_first + tid; w <= w_last; w += 256) mm = fmaxf(mm, a.part_ml[((w + pair) * G + g) * 2]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mm = fmaxf(mm, __shfl_xor(mm, off));
    if ((tid & 63) == 0) s_max[tid >> 6] = mm;
    __syncthreads();
    mm = fmaxf(fmaxf(s_max[0], s_max[1]), fmaxf(s_max[2], s_max[3]));

    float ll = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int w = w_first + slice; w <= w_last; w += nsl) {
        const int64_t rec = (w + pair) * G + g;
        const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + rec * 2);
        const float cw = fast_exp2(ml.x - mm);
        ll += ml.y * cw;
        acc += *reinterpret_cast<const f32x4*>(a.part_acc + rec * D + col0 + cg * 4) * cw;
    }
    *reinterpret_cast<f32x4*>(&s_acc[slice * cols + cg * 4]) = acc;
    if (cg == 0) s_l[slice] = ll;
    __syncthreads();
    if (tid < cols) {
        float tot = 0.f, lt = 0.f;
        for (int k = 0; k < nsl; ++k) {
            tot += s_acc[k * cols + tid];
            lt += s_l[k];
        }
        dst[col0 + tid] = f32_to_bf16(tot / lt);
    }
}

}  // namespace

size_t kv_streamk_workspace_bytes(const kv_view* view, int batch, int n_waves)
{
    const size_t slots = (size_t)n_waves + (size_t)batch * view->n_kv_local;
    const size_t acc = (slots * view->group * D * 4 + 255) / 256 * 256;
    const size_t ml = (slots * view->group * 2 * 4 + 255) / 256 * 256;
    const size_t prefix = ((size_t)(batch + 1) * 4 + 255) / 256 * 256;
    return acc + ml + prefix;
}

int kv_streamk_launch(kv_streamk_args a, const kv_view* view, void* workspace, hipStream_t st)
{
    const size_t slots = (size_t)a.n_waves + (size_t)a.batch * view->n_kv_local;
    const size_t acc = (slots * view->group * D * 4 + 255) / 256 * 256;
    a.part_acc = (float*)workspace;
    const size_t ml = (slots * view->group * 2 * 4 + 255) / 256 * 256;
    a.part_ml = (float*)((char*)workspace + acc);
    a.prefix_out = (int32_t*)((char*)workspace + acc + ml);
    int slot = kv_prof_begin(KV_PROF_DECODE_MAIN, st);
    const dim3 grid((unsigned)(a.n_waves / kSkWaves)), block(kSkThreads);
    if (a.view_ids) {
        hipLaunchKernelGGL((decode_streamk_kernel<1, 1, true>), grid, block, 0, st, a);
    } else
    switch (kv_option_variant() & 3) {
        case 0: hipLaunchKernelGGL((decode_streamk_kernel<1, 1, false>), grid, block, 0, st, a); break;
        case 1: hipLaunchKernelGGL((decode_streamk_kernel<0, 1, false>), grid, block, 0, st, a); break;
        case 2: hipLaunchKernelGGL((decode_streamk_kernel<1, 0, false>), grid, block, 0, st, a); break;
        default: hipLaunchKernelGGL((decode_streamk_kernel<0, 0, false>), grid, block, 0, st, a); break;
    }
    kv_prof_end(KV_PROF_DECODE_MAIN, slot, st);
    int rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn launch");
    if (rc) return rc;
    slot = kv_prof_begin(KV_PROF_DECODE_MERGE, st);
    // eight or more pieces per pair on average: expect long lists, split their columns
    const bool few_pairs = (int64_t)a.batch * view->n_kv_local * 8 <= a.n_waves;
    hipLaunchKernelGGL(decode_streamk_merge_kernel,
                       dim3((unsigned)view->n_q_local, (unsigned)a.batch, few_pairs ? (unsigned)kMergeSplit : 1u),
                       dim3(256), 0, st, a);
    kv_prof_end(KV_PROF_DECODE_MERGE, slot, st);
    return kv_record_hip_error(hipGetLastError(), "paged_decode_attn merge launch");
}
