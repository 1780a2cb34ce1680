// Multi-token causal attention over the paged KV pool, through a layout view: a chunk of a
// prefill, or the recompute step of Soft Preempt (Sec. 5.2.2 of the paper), both of which
// attend from several new tokens of a sequence to everything cached up to each of them.
//
// A workgroup of four wavefronts owns, for one (sequence, local KV head), a tile of query rows:
// 64 R rows = (64 R / G) consecutive new tokens x the G query heads that share the KV head; each
// wavefront holds R blocks of 16 rows.  The workgroup walks the cached tokens in staged tiles of
// 32, each K and V tile going once from global memory straight into LDS
// (16 bytes per lane with the load-to-LDS instruction, no registers in between; double buffered:
// the next tile lands while the current one is consumed); each wavefront then takes its MFMA
// operands from LDS and re-uses every K / V operand for its R row blocks.
//
// Per tile and row block, lane l = (c = l % 16, quad = l / 16), exactly as in the decode kernel:
//   S^T[token][c] = K[token][:] . q[c][:]     A operand = K rows from LDS (token 16 h + 4 (r % 4)
//                                             + r / 4 in A row r of half h), B operand = q
//   O^T[e][c]     = sum_t V[t][e] P[c][t]     A operand = V^T, read from the row-major V tile in
//                                             LDS with the transposing 64-bit read: a lane hands
//                                             in the address of four consecutive elements of one
//                                             row and receives one element of each of four rows
// so the accumulator layout of S^T is already the B layout of the second product and the running
// maximum crosses lanes only when it moves.  The sum of the weights of a column comes out of the
// matrix cores as well (one more product, with an all-ones A operand), from the same bf16 weights
// as the numerator.  Column c of row block b of wavefront w is row
// rho = (w R + b) 16 + c of the tile: token rho / Gp, head rho % Gp, Gp = G rounded up to a power
// of two (rows with head >= G are padding).  The causal mask keeps
// token t for a query at position pos iff t <= pos; since pos < ctx_len it also masks the slots
// past the end of the sequence.
#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int D = 128;
constexpr int kThreads = 256;
constexpr int kSub = 1;               // 32-key sub-tiles per staged tile
constexpr int kKeys = 32 * kSub;      // keys per staged tile (one barrier each)
constexpr float kUnset = 1e30f;       // exponent addend of a column that has no reference maximum yet

struct prefill_args {
    const uint16_t* q;      // [total_q][n_q_local][128]
    uint16_t* out;
    const uint16_t* pool;
    const int32_t* table;
    int64_t table_stride;
    const int32_t* ctx_lens;
    const int32_t* q_off;   // [batch + 1]
    kv_view_dev v;
    float scale_log2e;
    int32_t group;          // G <= 16 query heads per KV head
    int32_t group_shift;    // log2 of G rounded up to a power of two: rows per token in the tile
    int32_t splits;         // workgroups sharing the key range of one query tile
    int32_t wgs_per_pair;   // query tiles of the longest chunk x splits: workgroups per (sequence, KV head)
    int64_t rows;           // total_q * n_q_local: rows of the partial arrays
    float* part_o;          // [splits][rows][128] un-normalised sums, when splits > 1
    float* part_ml;         // [splits][rows][2]   (reference maximum in score units, sum of weights)
};

__device__ __forceinline__ int uniform(int x) { return __builtin_amdgcn_readfirstlane(x); }

typedef short bits16x4 __attribute__((ext_vector_type(4)));
typedef short bits16x8 __attribute__((ext_vector_type(8)));
typedef __attribute__((address_space(3))) bits16x4* lds_bits16x4_ptr;

// Transposing LDS read.  Within each group of 16 lanes, lane i passes the address of four
// consecutive 16-bit elements (a row); lane i receives, as element j, element i % 4 of the row
// passed by lane 4 j + i / 4 of its group.
__device__ __forceinline__ bits16x4 lds_read_transposed(const void* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_bits16x4_ptr)p);
}

// Three workgroups per compute unit (32 KiB of LDS and at most 168 registers each): with nothing staged
// in registers the kernel fits, and a third wavefront per SIMD hides more of the chain K read -> scores ->
// softmax -> V read -> output of the other two than the longer 64-key tiles of two workgroups did.
template <int R>
__global__ __launch_bounds__(kThreads, R <= 2 ? 3 : 1) void prefill_kernel(prefill_args a)
{
    // [buffer][row][piece]: K pieces swizzled (piece c of row t at c ^ (t % 16)); V pieces at
    // c ^ (2 * ((t / 4) % 4)), which puts the four rows a transposing read touches in different banks
    // one array per buffer: the compiler then knows that the loads landing in one buffer do not touch
    // the operands being read from the other
    __shared__ kv_u32x4 s_k0[512 * kSub], s_k1[512 * kSub];
    __shared__ kv_u32x4 s_v0[512 * kSub], s_v1[512 * kSub];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const int r = lane & 15, quad = lane >> 4;
    const kv_view_dev& v = a.v;
    const int G = a.group;
    // Which (sequence, KV head, query tile, key split) this workgroup takes.  The hardware deals
    // consecutive workgroups out to the eight XCDs in turn, each with its own L2; every query tile of
    // a (sequence, head) pair reads that pair's keys and values again, so all tiles of a pair go to
    // one XCD: workgroup L runs on XCD L % 8 and takes the (L / 8)-th item of that XCD's eighth of the
    // (pair-major) work list.  A pair's K/V (2 MiB per 4096 tokens) then stays in one 4 MiB L2 while
    // its tiles are worked on, instead of streaming through all eight.
    int item;
    {
        const int L = (int)blockIdx.x, N = (int)gridDim.x;
        const int xcd = L & 7, k = L >> 3, base = N >> 3, rem = N & 7;
        item = xcd * base + min(xcd, rem) + k;
    }
    const int pair = item / a.wgs_per_pair, in_pair = item - pair * a.wgs_per_pair;
    const int s = pair / a.v.n_kv_local, hl = pair - s * a.v.n_kv_local;
    const int tokens_per_wg = (64 * R) >> a.group_shift;

    const int n = a.ctx_lens[s];
    const int q0 = a.q_off[s];
    const int q_len = a.q_off[s + 1] - q0;
    // longest tiles first: the last query tile of a sequence sees the most keys
    const int split = in_pair % a.splits;
    const int j0 = (a.wgs_per_pair / a.splits - 1 - in_pair / a.splits) * tokens_per_wg;
    if (j0 >= q_len || n <= 0) return;
    const int first_pos = n - q_len;                         // position of the sequence's query 0
    const int j_last = min(j0 + tokens_per_wg, q_len) - 1;   // last query token of this tile
    const int all_tiles = (first_pos + j_last) / kKeys + 1;   // key tiles 0 .. all_tiles - 1 of the query tile
    // this workgroup's share of them: [t_begin, n_tiles)
    const int per_split = (all_tiles + a.splits - 1) / a.splits;
    const int t_begin = split * per_split;
    const int n_tiles = min(all_tiles, t_begin + per_split);

    // ---- staging: K and V tiles go from global memory straight into LDS, 16 bytes per lane; one
    // instruction of a wavefront fills 64 consecutive 16-byte slots = 4 rows of 16 pieces, and
    // which piece of its row a lane fetches is the LDS swizzle applied on the global side.
    // Instruction i of wavefront w fills rows 16 i + 4 w .. + 3 of the tile (group i of 16 rows lies
    // in one block).
    const int dma_r = lane >> 4, dma_c = lane & 15;
    const int row16 = 4 * wave + dma_r;                       // row within its group of 16
    const int token_stride_bytes = v.token_stride * 2;
    const int64_t plane_bytes = v.plane_elems * 2;
    const int halves_per_block = v.block_tokens >> 4;
    const int half_shift = v.block_shift >= 4 ? v.block_shift - 4 : -1;
    const int last_half = (n - 1) >> 4;
    typedef const __attribute__((address_space(4))) int32_t* const_ids;
    const const_ids ids = (const_ids)(a.table + (int64_t)s * a.table_stride);
    const char* pool_head = reinterpret_cast<const char*>(a.pool + v.head_off + hl * D);
    const int64_t block_bytes = (int64_t)v.block_elems * 2;
    const uint32_t k_piece = (uint32_t)((dma_c ^ row16) << 4);
    const uint32_t v_piece = (uint32_t)((dma_c ^ (2 * wave)) << 4);   // 2 ((row / 4) % 4), row / 4 = 4 i + w
    const uint32_t lane_off_k = (uint32_t)(row16 * token_stride_bytes) + k_piece;
    const uint32_t lane_off_v = (uint32_t)(row16 * token_stride_bytes) + v_piece;
    typedef const __attribute__((address_space(1))) void* global_ptr;
    typedef __attribute__((address_space(3))) void* lds_ptr;
    const int last_tile = n_tiles - 1;
    // rows past the end of the sequence are replaced by its last token (finite data, masked later)
    auto stage_tile = [&](int tile, kv_u32x4* dk, kv_u32x4* dv) {
        int hh[2 * kSub], hb[2 * kSub], blk[2 * kSub];
#pragma unroll
        for (int h = 0; h < 2 * kSub; ++h) hh[h] = min(2 * kSub * tile + h, last_half);
        if (half_shift >= 0) {
#pragma unroll
            for (int h = 0; h < 2 * kSub; ++h) hb[h] = hh[h] >> half_shift;
        } else {
#pragma unroll
            for (int h = 0; h < 2 * kSub; ++h) hb[h] = hh[h] / halves_per_block;
        }
#pragma unroll
        for (int h = 0; h < 2 * kSub; ++h) blk[h] = ids[hb[h]];
        // ordinary (cached) loads: every query tile of the sequence reads these keys again
        if (2 * kSub * tile + 2 * kSub - 1 < last_half) {
#pragma unroll
            for (int h = 0; h < 2 * kSub; ++h) {
                const char* base = pool_head + blk[h] * block_bytes +
                                   (int64_t)(16 * hh[h] - hb[h] * v.block_tokens) * token_stride_bytes;
                __builtin_amdgcn_global_load_lds((global_ptr)(base + lane_off_k), (lds_ptr)(dk + (4 * h + wave) * 64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_ptr)(base + plane_bytes + lane_off_v), (lds_ptr)(dv + (4 * h + wave) * 64), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int h = 0; h < 2 * kSub; ++h) {
                const int tok = min(16 * hh[h] + row16, n - 1);
                const int slot = tok - hb[h] * v.block_tokens;
                const char* p = pool_head + blk[h] * block_bytes + (int64_t)slot * token_stride_bytes;
                __builtin_amdgcn_global_load_lds((global_ptr)(p + k_piece), (lds_ptr)(dk + (4 * h + wave) * 64), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((global_ptr)(p + plane_bytes + v_piece), (lds_ptr)(dv + (4 * h + wave) * 64), 16, 0, 0);
            }
        }
    };
    // all of this wavefront's loads have landed in LDS; then every wavefront's
    auto staged = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0f70);   // vmcnt(0)
        __syncthreads();
    };

    float m[R];
    float neg_mc[R];  // -m scale log2(e), the addend of the exponent; kUnset while m = -inf
    f32x4 l[R];     // sum of the weights of the column, the same in all four entries and lanes of it
    f32x4 o[R][8];  // o[b][j][i] = O[column][16 j + 4 quad + i]
#pragma unroll
    for (int b = 0; b < R; ++b) {
        m[b] = kNegInf;
        neg_mc[b] = kUnset;
        l[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 8; ++j) o[b][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    // this lane's part of the V^T operand of output block j: elements [16 j + 4 (r % 4), + 4) of
    // tokens 4 (r / 4) + quad (first read) and 16 + 4 (r / 4) + quad (second) of the tile; A row r
    // then is element 16 j + r, contraction index 8 quad + 4 h + i is token 16 h + 4 i + quad, as
    // the scores have it
    const int vt_tok = 4 * (r >> 2) + quad;
    const int vt_swz = 2 * ((vt_tok >> 2) & 3);   // the same for token 16 + vt_tok
    const bf16x8 ones = as_bf16x8(kv_u32x4{0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u});

    if (t_begin < n_tiles) stage_tile(t_begin, s_k0, s_v0);
    // ---- this lane's query rows (B operands), one per row block --------------------------------
    bf16x8 qb[R][4];
    int pos[R];       // position of the column's query token
    // element offset of the row of column r of row block b in q and out, or -1 if the column is
    // padding (recomputed at the end rather than kept in registers through the loop)
    auto row_of = [&](int b, bool or_padding) -> int64_t {
        const int rho = (wave * R + b) * 16 + r;
        // a token takes 2^group_shift rows of the tile, the first G of which are its query heads
        const int jt = j0 + (rho >> a.group_shift), g = rho & ((1 << a.group_shift) - 1);
        const int jc = min(jt, q_len - 1);
        const int64_t row = ((int64_t)(q0 + jc) * v.n_q_local + hl * G + min(g, G - 1)) * D;
        return (or_padding || (jt < q_len && g < G)) ? row : -1;
    };
#pragma unroll
    for (int b = 0; b < R; ++b) {
        const int rho = (wave * R + b) * 16 + r;
        pos[b] = first_pos + min(j0 + (rho >> a.group_shift), q_len - 1);
        const int64_t row = row_of(b, true);
        const char* qrow = reinterpret_cast<const char*>(a.q + row) + quad * 16;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk)
            qb[b][kk] = as_bf16x8(*reinterpret_cast<const kv_u32x4*>(qrow + kk * 64));
    }
    // keys below this position need no mask for any column of the wavefront
    int min_pos = pos[0];
#pragma unroll
    for (int b = 1; b < R; ++b) min_pos = min(min_pos, pos[b]);
#pragma unroll
    for (int off = 1; off < 16; off <<= 1) min_pos = min(min_pos, __shfl_xor(min_pos, off));
    min_pos = uniform(min_pos);
    int max_pos = pos[R - 1];
    max_pos = uniform(__shfl(max_pos, 15));  // rows ascend with the column: the last is the largest

    staged();

    const int k_row = 4 * (r & 3) + (r >> 2);
    constexpr float kLag = 8.0f;
    auto compute = [&](int buf, int tile) {
#pragma unroll
      for (int sub = 0; sub < kSub; ++sub) {
        const int base = kKeys * tile + 32 * sub;
        const kv_u32x4* const sk = (buf ? s_k1 : s_k0) + 512 * sub;
        const kv_u32x4* const sv = (buf ? s_v1 : s_v0) + 512 * sub;
        if (base <= max_pos) {  // else every key of the sub-tile lies after all of this wavefront's queries
            // ---- S^T = K q^T ------------------------------------------------------------------------
            f32x4 sacc[R][2];
#pragma unroll
            for (int b = 0; b < R; ++b) sacc[b][0] = sacc[b][1] = f32x4{0.f, 0.f, 0.f, 0.f};
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const kv_u32x4 ka = sk[(16 * h + k_row) * 16 + ((4 * kk + quad) ^ k_row)];
#pragma unroll
                    for (int b = 0; b < R; ++b)
                        sacc[b][h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka), qb[b][kk],
                                                                            sacc[b][h], 0, 0, 0);
                }
            // ---- online softmax per column ------------------------------------------------------------
            __builtin_amdgcn_s_setprio(0);
            // the causal mask, only on the tiles that reach past some query of this wavefront (one
            // uniform branch around all of it: most tiles lie wholly before every query)
            if (base + 31 > min_pos) {
#pragma unroll
                for (int b = 0; b < R; ++b)
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            sacc[b][h][i] = (base + 16 * h + 4 * i + quad <= pos[b]) ? sacc[b][h][i] : kNegInf;
            }
            bf16x8 pb[R];
#pragma unroll
            for (int b = 0; b < R; ++b) {
                // Scores stay in the products' own units; the scale is folded into the exponent:
                // t = (score - m) scale log2(e), weight = 2^t.  m[b] is a reference maximum that is
                // allowed to lag behind the true running maximum by up to kLag in the exponent:
                // weights then reach 2^kLag at most (exact in fp32 and in the bf16 operand alike), and
                // the accumulators are rescaled only when some column's maximum has moved further than
                // that -- rarely, after the first tiles.  m[b] is the same in the four lanes of a
                // column, so each lane tests its own eight exponents and the maximum crosses lanes only
                // on the rare tile that moves it.  While a column has seen no valid key (m = -inf; with
                // the key range split it may never see one) its addend is kUnset: any finite score then
                // gives a huge exponent and forces the first move, a masked one stays at -inf.
                float t[8];
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        t[4 * h + i] = __builtin_fmaf(sacc[b][h][i], a.scale_log2e, neg_mc[b]);
                const float tmax = fmaxf(fmaxf(fmaxf(t[0], t[1]), fmaxf(t[2], t[3])),
                                         fmaxf(fmaxf(t[4], t[5]), fmaxf(t[6], t[7])));
                if (__builtin_amdgcn_ballot_w64(tmax > kLag) != 0) {
                    float mx = fmaxf(fmaxf(fmaxf(sacc[b][0][0], sacc[b][0][1]), fmaxf(sacc[b][0][2], sacc[b][0][3])),
                                     fmaxf(fmaxf(sacc[b][1][0], sacc[b][1][1]), fmaxf(sacc[b][1][2], sacc[b][1][3])));
                    mx = fmaxf(mx, __shfl_xor(mx, 16));
                    mx = fmaxf(mx, __shfl_xor(mx, 32));
                    const float m_new = fmaxf(m[b], mx);
                    if (m_new != kNegInf) {
                        const float alpha = fast_exp2((m[b] - m_new) * a.scale_log2e);   // 0 on the first move
                        l[b] *= alpha;
#pragma unroll
                        for (int j = 0; j < 8; ++j) o[b][j] *= alpha;
                        m[b] = m_new;
                        neg_mc[b] = -m_new * a.scale_log2e;
                    }
#pragma unroll
                    for (int h = 0; h < 2; ++h)
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            t[4 * h + i] = __builtin_fmaf(sacc[b][h][i], a.scale_log2e, neg_mc[b]);
                }
                float p[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) p[u] = fast_exp2(t[u]);
                pb[b] = as_bf16x8(kv_u32x4{pack_bf16x2(p[0], p[1]), pack_bf16x2(p[2], p[3]),
                                           pack_bf16x2(p[4], p[5]), pack_bf16x2(p[6], p[7])});
            }
            // ---- O^T += V^T P^T --------------------------------------------------------------------------
            __builtin_amdgcn_s_setprio(2);
#pragma unroll
            for (int b = 0; b < R; ++b) l[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pb[b], l[b], 0, 0, 0);
            const char* vt = reinterpret_cast<const char*>(sv) + vt_tok * 256 + (r & 1) * 8;
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                // elements [16 j + 4 (r % 4), + 4) of the row: piece 2 j + (r % 4) / 2 (swizzled), half r % 2
                const int piece_off = ((2 * j + ((r & 3) >> 1)) ^ vt_swz) * 16;
                const bits16x4 lo = lds_read_transposed(vt + piece_off);
                const bits16x4 hi = lds_read_transposed(vt + piece_off + 16 * 256);
                const bf16x8 va = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
#pragma unroll
                for (int b = 0; b < R; ++b)
                    o[b][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pb[b], o[b][j], 0, 0, 0);
            }
            __builtin_amdgcn_s_setprio(0);
        }
      }
    };
    for (int tile = t_begin; tile < n_tiles; tile += 2) {
        stage_tile(min(tile + 1, last_tile), s_k1, s_v1);
        compute(0, tile);
        staged();
        stage_tile(min(tile + 2, last_tile), s_k0, s_v0);
        if (tile + 1 < n_tiles) compute(1, tile + 1);
        staged();
    }

    // ---- normalise and store ------------------------------------------------------------------------
#pragma unroll
    for (int b = 0; b < R; ++b) {
        const float lt = l[b][0];
        const int64_t orow = row_of(b, false);
        if (orow >= 0 && a.splits > 1) {
            // partial of this key range: row = index of the output row
            const int64_t rec = (int64_t)split * a.rows + orow / D;
            float* dst = a.part_o + rec * D + 4 * quad;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) *reinterpret_cast<f32x4*>(dst + 16 * jj) = o[b][jj];
            if (quad == 0) {
                a.part_ml[rec * 2 + 0] = m[b];
                a.part_ml[rec * 2 + 1] = lt;
            }
        } else if (orow >= 0) {
            const float inv = 1.0f / lt;
            uint16_t* dst = a.out + orow + 4 * quad;
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) {
                uint2 pk;
                pk.x = pack_bf16x2(o[b][jj][0] * inv, o[b][jj][1] * inv);
                pk.y = pack_bf16x2(o[b][jj][2] * inv, o[b][jj][3] * inv);
                *reinterpret_cast<uint2*>(dst + 16 * jj) = pk;
            }
        }
    }
}

// out[row] = sum_z o_z 2^((m_z - M) c) / sum_z l_z 2^((m_z - M) c), M = max_z m_z; a split that saw
// no valid key for the row has l = 0 and is skipped.  32 lanes per row, 4 columns each.
__global__ __launch_bounds__(256) void prefill_merge_kernel(prefill_args a)
{
    const int64_t row = (int64_t)blockIdx.x * 8 + (threadIdx.x >> 5);
    const int cg = threadIdx.x & 31;
    if (row >= a.rows) return;
    float mm = kNegInf;
    for (int z = 0; z < a.splits; ++z) {
        const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + ((int64_t)z * a.rows + row) * 2);
        if (ml.y > 0.f) mm = fmaxf(mm, ml.x);
    }
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    float lt = 0.f;
    for (int z = 0; z < a.splits; ++z) {
        const int64_t rec = (int64_t)z * a.rows + row;
        const float2 ml = *reinterpret_cast<const float2*>(a.part_ml + rec * 2);
        if (!(ml.y > 0.f)) continue;
        const float w = fast_exp2((ml.x - mm) * a.scale_log2e);
        lt += ml.y * w;
        acc += *reinterpret_cast<const f32x4*>(a.part_o + rec * D + cg * 4) * w;
    }
    const float inv = 1.0f / lt;   // every query sees at least key 0
    uint2 pk;
    pk.x = pack_bf16x2(acc[0] * inv, acc[1] * inv);
    pk.y = pack_bf16x2(acc[2] * inv, acc[3] * inv);
    *reinterpret_cast<uint2*>(a.out + row * D + cg * 4) = pk;
}

constexpr int kRowBlocks = 2;  // 16-row blocks per wavefront (4 measured 2x slower: one wavefront per SIMD)

// Workgroups sharing the key range of a query tile: only when the launch would otherwise leave
// compute units idle (few sequences, few query tokens, long contexts): enough to fill the 768
// workgroup slots of the chip (three per compute unit) once, measured better than one and a half
// times; at least 512 keys each.
int prefill_splits(const kv_view* view, int batch, int max_ctx_len, int max_q_len)
{
    int shift = 0;
    while ((1 << shift) < view->group) ++shift;
    const int tokens_per_wg = (64 * kRowBlocks) >> shift;
    const int64_t wgs = (int64_t)((max_q_len + tokens_per_wg - 1) / tokens_per_wg) * view->n_kv_local * batch;
    if (wgs >= 512) return 1;
    int s = (int)((768 + wgs - 1) / wgs);
    const int most = max_ctx_len / 512;
    if (s > most) s = most;
    if (s > 16) s = 16;
    return s < 1 ? 1 : s;
}

}  // namespace

extern "C" size_t paged_prefill_attn_workspace_bytes(const kv_view* view, int batch, int64_t total_q,
                                                     int max_ctx_len, int max_q_len)
{
    if (!kv_view_ok(view) || batch <= 0 || total_q <= 0 || max_ctx_len <= 0 || max_q_len <= 0) return 0;
    const int s = prefill_splits(view, batch, max_ctx_len, max_q_len);
    return s > 1 ? (size_t)s * total_q * view->n_q_local * (D + 2) * 4 : 0;
}

extern "C" int paged_prefill_attn(const void* q, void* out, const void* kv_pool, int64_t n_pool_blocks,
                                  const int32_t* block_table, int64_t block_table_stride,
                                  const int32_t* ctx_lens, const int32_t* q_offsets, int batch,
                                  int64_t total_q, int max_ctx_len, int max_q_len, const kv_view* view,
                                  float scale, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!kv_view_ok(view) || batch < 0 || total_q < 0 || max_ctx_len < 0 || max_q_len < 0 ||
        n_pool_blocks < 0 || block_table_stride < 0 || max_q_len > max_ctx_len)
        return KV_ERR_INVALID_ARG;
    if (batch == 0 || max_q_len == 0 || total_q == 0) return KV_OK;
    if (!q || !out || !ctx_lens || !q_offsets || !kv_pool || !block_table) return KV_ERR_INVALID_ARG;
    const int64_t need_cols = ((int64_t)max_ctx_len + view->block_tokens - 1) / view->block_tokens;
    if (block_table_stride < need_cols) return KV_ERR_INVALID_ARG;
    const int G = view->group;
    if (view->geom.head_dim != D || view->block_tokens % 16 != 0 || G > 16)
        return KV_ERR_UNSUPPORTED;
    if (batch > 65535 || view->n_kv_local > 65535) return KV_ERR_UNSUPPORTED;
    prefill_args a;
    a.q = (const uint16_t*)q;
    a.out = (uint16_t*)out;
    a.pool = (const uint16_t*)kv_pool;
    a.table = block_table;
    a.table_stride = block_table_stride;
    a.ctx_lens = ctx_lens;
    a.q_off = q_offsets;
    a.v = kv_view_to_dev(view);
    a.scale_log2e = (scale > 0.f ? scale : 1.0f / sqrtf((float)D)) * 1.4426950408889634f;
    a.group = G;
    a.group_shift = 0;
    while ((1 << a.group_shift) < G) ++a.group_shift;
    hipStream_t st = (hipStream_t)hip_stream;
    constexpr int R = kRowBlocks;
    a.splits = prefill_splits(view, batch, max_ctx_len, max_q_len);
    a.rows = total_q * view->n_q_local;
    a.part_o = nullptr;
    a.part_ml = nullptr;
    if (a.splits > 1) {
        const size_t need = (size_t)a.splits * a.rows * (D + 2) * 4;
        if (!workspace || ((uintptr_t)workspace & 255u)) return KV_ERR_INVALID_ARG;
        if (workspace_bytes < need) return KV_ERR_WORKSPACE;
        a.part_o = (float*)workspace;
        a.part_ml = a.part_o + (size_t)a.splits * a.rows * D;
    }
    const int tokens_per_wg = (64 * R) >> a.group_shift;
    const int64_t q_tiles = (max_q_len + tokens_per_wg - 1) / tokens_per_wg;
    if (q_tiles * a.splits > 0x7fffffff) return KV_ERR_UNSUPPORTED;
    a.wgs_per_pair = (int32_t)(q_tiles * a.splits);
    const int64_t n_wgs = q_tiles * a.splits * view->n_kv_local * batch;
    if (n_wgs > 0x7fffffff) return KV_ERR_UNSUPPORTED;
    const dim3 grid((unsigned)n_wgs);
    int slot = kv_prof_begin(KV_PROF_PREFILL, st);
    hipLaunchKernelGGL(prefill_kernel<R>, grid, dim3(kThreads), 0, st, a);
    if (a.splits > 1)
        hipLaunchKernelGGL(prefill_merge_kernel, dim3((unsigned)((a.rows + 7) / 8)), dim3(256), 0, st, a);
    kv_prof_end(KV_PROF_PREFILL, slot, st);
    return kv_record_hip_error(hipGetLastError(), "paged_prefill_attn launch");
}
