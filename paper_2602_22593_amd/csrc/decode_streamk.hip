// Matrix-core decode attention with an even split of the whole batch over resident wavefronts.
// Two main kernels share the split, the workspace and the way pieces are combined:
// decode_streamk_kernel (one KV head per wavefront, described first) and decode_wide_kernel (2 or 4
// adjacent heads per wavefront, described where it is defined); kv_streamk_launch picks one per view.
//
// The batch is flattened into tiles of 32 tokens of one (sequence, local KV head) pair, pairs
// ordered (sequence, head) with the head fastest.  The T tiles are cut into W consecutive ranges,
// one per launched wavefront (the grid is sized so that all W are resident at once), of nearly
// equal length (a small, fixed correction per XCD, see split_prologue): every wavefront streams
// about the same number of KV bytes whatever the mix of context lengths, and lives long enough
// to amortise its start-up.  A wavefront's range may cover the end of one pair and the start of
// the next; each (wavefront, pair) piece yields either the final output row (the piece is the
// whole pair) or an un-normalised partial (m, l, acc[G][d]) in workspace slot w + pair_index,
// which is unique and keeps the pieces of a pair in consecutive slots.
//
// Combining the pieces of a cut pair (m = max m_k, l = sum l_k 2^(m_k - m), acc likewise) happens
// in one of two ways.  Normally inside this kernel, with no waiting anywhere: a wavefront writes
// its partials with device-coherent stores, and at the end of its range, once those stores are
// acknowledged, adds one 64-bit word to the pair's arrival word: 1 in the piece count, plus its
// own number in a "first" field if it held the pair's first piece or in a "last" field if it held
// the last.  The sum tells every arriver how many pieces there are and how many have arrived; the
// one that completes the count reads all partials back (device-coherent loads), writes the output
// rows and puts the word back to zero.  Batches in which a pair is cut over very many wavefronts
// (few, very long sequences) use a second launch instead, decode_streamk_merge_kernel, which
// spreads each long list over a workgroup; there the wavefronts holding a pair's first and last
// piece leave their numbers in the pair's descriptor.
//
// Per tile, lane l = (r = l % 16, quad = l / 16).  Both products put the KV data in the MFMA
// A operand (row index r) and the query group, padded to 16, in the B operand (column r = g):
//   S^T[token][g] = K[token][:] . q[g][:]    lane (r, quad) holds elements [32 kk + 8 quad, +8)
//                                             of A row r, kk = 0..3
//   O^T[e][g]     = sum_t V[t][e] P[g][t]    contraction over the 32 tokens of the tile
// The C layout of S^T (lane (g, quad), half h, i = 0..3 <-> A row 4 quad + i) is already the B
// layout of the second product if contraction index k = 8 quad + 4 h + i stands for token
// 16 h + 4 i + quad: so A row r of half h is token 16 h + 4 (r % 4) + r / 4.  K and V rows are
// loaded as they lie in memory (lane (c = r, quad) reads bytes [16 c, 16 c + 16) of tokens
// 4 i' + quad); K reaches the operand arrangement through a wavefront-private LDS buffer, V is
// transposed inside the lane with byte permutes.  Only the running maximum crosses lanes.
#include <hip/hip_ext.h>

#include "decode_common.h"

using namespace kvdec;

namespace {

constexpr int kSkThreads = 256;
constexpr int kSkWaves = kSkThreads / 64;
constexpr int kMaxBatch = KV_STREAMK_MAX_BATCH;
constexpr int D = 128;
constexpr int kMaxClasses = 8;
constexpr int kDefaultXcdSkew = 80;
// What a piece boundary counts for in the cut, in eighths of a tile (measured optimum: two tiles;
// flat between two and three on every named workload)
constexpr int kDefaultPieceUnits = 16;

struct tile_regs {
    kv_u32x4 k[2][4];  // [half][i]: bytes [16 r, +16) of token 16 h + 4 i + quad
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
    uint32_t voff;   // byte offset of this lane's piece of a row (token `quad` of a half)
    uint32_t vstep;  // bytes between tokens 4 apart
};

// Full tile: both halves lie in one block each; kb[h] points at (block, first slot of the half,
// this head) in the K plane.  K and V rows are fetched as they lie in memory.
__device__ __forceinline__ void load_full(tile_regs& t, const char* const (&kb)[2],
                                          int64_t plane_bytes, const lane_consts& lc)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
#pragma unroll
        for (int i = 0; i < 4; ++i) t.k[h][i] = ld16(kb[h], lc.voff + i * lc.vstep);
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
__device__ __forceinline__ void load_tail(tile_regs& t, const char* const (&kb)[2],
                                          int64_t plane_bytes, const lane_consts& lc, int last,
                                          int token_stride_bytes)
{
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // half h starts at token 16 h of the tile; if it holds no valid token its base was set
        // to the block of the last valid token by the caller and everything clamps to `last`
        const int first = (16 * h <= last) ? 16 * h : last;
        const char* vb = kb[h] + plane_bytes;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int vrow = min(16 * h + 4 * i + lc.quad, last) - first;
            const uint32_t voff = (uint32_t)(vrow * token_stride_bytes + lc.r * 16);
            t.v[4 * h + i] = ld16(vb, voff);
            t.k[h][i] = ld16(kb[h], voff);
        }
    }
}

struct softmax_state {
    float m, l;
    f32x4 o[8];  // o[j][i] = O[g = r][32 quad + 8 i + j]
};

// The two bf16 values of a packed pair, as fp32.
__device__ __forceinline__ float pair_sum(uint32_t packed) { return bf16_lo(packed) + bf16_hi(packed); }

// LDS staging of a K tile, private to the wavefront: 32 rows of 16 16-byte pieces; piece c
// of row t is kept at position c ^ (t % 16), which makes both the row-wise writes and the
// operand-wise reads free of bank conflicts.
template <bool TAIL>
__device__ __forceinline__ void compute_tile(const tile_regs& t, const bf16x8 (&qb)[4],
                                             softmax_state& st, float scale_log2e, int last,
                                             int r, int quad, kv_u32x4* kstage)
{
    f32x4 sacc[2];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int row = 16 * h + 4 * i + quad;
            kstage[row * 16 + (r ^ (row & 15))] = t.k[h][i];
        }
    __builtin_amdgcn_wave_barrier();
    const int k_row = 4 * (r & 3) + (r >> 2);
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        sacc[h] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const kv_u32x4 ka = kstage[(16 * h + k_row) * 16 + ((4 * kk + quad) ^ k_row)];
            sacc[h] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka), qb[kk], sacc[h], 0, 0, 0);
        }
    }
    __builtin_amdgcn_wave_barrier();
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
    // weights rounded to bf16 for the second product; the denominator sums the same rounded values
    kv_u32x4 pw;
#pragma unroll
    for (int u = 0; u < 4; ++u)
        pw[u] = pack_bf16x2(fast_exp2(sv[2 * u] - m_new), fast_exp2(sv[2 * u + 1] - m_new));
    st.l += (pair_sum(pw[0]) + pair_sum(pw[1])) + (pair_sum(pw[2]) + pair_sum(pw[3]));
    const bf16x8 pb = as_bf16x8(pw);
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


// Where a wavefront's share starts: tiles [x0, x1) of the flattened batch, the first one being
// tile `tile` of pair `pair` of sequence `s` (which has tiles_s tiles per pair); w numbers the
// wavefront.
struct split_pos {
    int x0, x1, s, tiles_s, pair, tile, w;
};

constexpr int kTileUnits = 8;   // weight of a tile on the axis that is cut; a pair's start weighs a.piece_units

// Inclusive prefix sum over the 64 lanes: shifts inside rows of 16 lanes, then the totals of the rows
// before a lane's own.
template <int CTRL>
__device__ __forceinline__ int dpp_shr(int x) { return __builtin_amdgcn_update_dpp(0, x, CTRL, 0xf, 0xf, true); }
__device__ __forceinline__ int wave_inclusive_sum(int x, int lane)
{
    x += dpp_shr<0x111>(x);   // row_shr:1 (lanes shifted in from outside the row read as 0)
    x += dpp_shr<0x112>(x);
    x += dpp_shr<0x114>(x);
    x += dpp_shr<0x118>(x);
    const int t0 = __builtin_amdgcn_readlane(x, 15), t1 = __builtin_amdgcn_readlane(x, 31),
              t2 = __builtin_amdgcn_readlane(x, 47);
    const int row = lane >> 4;
    return x + (row >= 1 ? t0 : 0) + (row >= 2 ? t1 : 0) + (row >= 3 ? t2 : 0);
}

// tile holding a weighted position: its number on the flattened tile axis and where it lies
struct tile_pos {
    int x, s, tiles_s, pair, tile;
};

// The cut of the batch over the wavefronts, as every wavefront evaluates it.
//
// What is cut evenly is not the tile axis itself but a weighted one, on which a tile is kTileUnits
// long and the start of every pair adds a.piece_units: a wavefront that has to close one piece
// and open another (write a partial, fetch new query rows and block ids, refill its load
// pipeline) gets that much less to stream.  Position u of the weighted axis maps to a tile by
// tile_at(), a monotone function that every wavefront evaluates alike, so the ranges
// [tile_at(u(w)), tile_at(u(w + 1))) are disjoint and cover all tiles.
struct splitter {
    const kv_streamk_args& a;
    int pairs, lane;
    const int32_t* s_prefix;              // [batch + 1] tiles of the sequences before s
    const unsigned long long* s_wpos;     // [batch + 1] weighted position of the first tile of s
    int total;                            // tiles in all
    uint32_t cu;                          // a.piece_units
    unsigned long long u_all;             // weighted length of the batch

    // Wavefront w = 4 * workgroup + wave owns the w-th range.  The ranges are not all of one
    // weighted length either: the hardware deals consecutive workgroups out to the XCDs in turn,
    // workgroup b runs on XCD b % 8, and a wavefront's share is proportional to the weight of its
    // XCD.  Range w starts at weighted position floor(u_all * W(w) / W(n_waves)), W(w) the summed
    // weight of the wavefronts before w (in double precision, with the reciprocal from the host).
    __device__ __forceinline__ unsigned long long range_u(int w) const
    {
        if (w >= a.n_waves) return u_all;
        const int grp = w / (kMaxClasses * kSkWaves), in_grp = w % (kMaxClasses * kSkWaves);
        const int x = in_grp / kSkWaves, i = in_grp % kSkWaves;   // XCD of the workgroup, wave in it
        const uint32_t before = (uint32_t)grp * (kSkWaves * a.wt_prefix[kMaxClasses]) + kSkWaves * a.wt_prefix[x] +
                                (uint32_t)i * (a.wt_prefix[x + 1] - a.wt_prefix[x]);
        const unsigned long long u = (unsigned long long)((double)u_all * ((double)before * a.inv_weight));
        return u < u_all ? u : u_all;
    }

    __device__ __forceinline__ tile_pos tile_at(unsigned long long u) const
    {
        tile_pos t;
        if (u >= u_all) {
            t.x = total;
            t.s = a.batch;
            t.tiles_s = 1;
            t.pair = t.tile = 0;
            return t;
        }
        // largest s with wpos(s) <= u (a non-empty sequence, since u < u_all), by a 64-way search:
        // every lane probes one sequence, a ballot counts the probes not above u (wpos is monotone)
        const int chunk = (a.batch + 63) >> 6;
        int lo = 0;
        {
            const int probe = lane * chunk;
            const bool ok = probe < a.batch && s_wpos[min(probe, a.batch)] <= u;
            lo = (__builtin_popcountll(__builtin_amdgcn_ballot_w64(ok)) - 1) * chunk;   // lane 0 always counts
        }
        if (chunk > 1) {
            const int probe = lo + lane;
            const bool ok = lane < chunk && probe < a.batch && s_wpos[min(probe, a.batch)] <= u;
            lo += __builtin_popcountll(__builtin_amdgcn_ballot_w64(ok)) - 1;
        }
        t.s = lo;
        const int before = uniform(s_prefix[lo]);
        t.tiles_s = uniform(s_prefix[lo + 1]) - before;
        const unsigned long long w_lo = s_wpos[lo];
        const uint32_t rel = (uint32_t)(u - (((unsigned long long)uniform((int)(w_lo >> 32)) << 32) |
                                             (uint32_t)uniform((int)w_lo)));   // < pairs * len: fits (host check)
        const uint32_t len = (uint32_t)kTileUnits * (uint32_t)t.tiles_s + cu;  // weighted length of a pair
        t.pair = (int)(rel / len);
        const uint32_t r = rel - (uint32_t)t.pair * len;
        t.tile = r < cu ? 0 : (int)((r - cu) / kTileUnits);
        t.x = before * pairs + t.pair * t.tiles_s + t.tile;
        return t;
    }

    // first tile of the range after wavefront w's: where w's range ends
    __device__ __forceinline__ int range_end(int w) const { return tile_at(range_u(w + 1)).x; }
};

// Common start of the even-split kernels (whole workgroup): exclusive prefix sums over the sequences
// of the tiles (2^TSHIFT tokens) into s_prefix, weighted positions into s_wpos, context lengths into
// s_ctx, then the position of this wavefront's first tile (sp.x0 and the fields after it; sp.x1 is
// left to range_end(), which the kernels call once their first loads are in flight).
template <int TSHIFT>
__device__ __forceinline__ splitter split_prologue(const kv_streamk_args& a, int pairs, int32_t* s_prefix,
                                                   unsigned long long* s_wpos, int32_t* s_ctx, int32_t* s_wsum,
                                                   split_pos& sp)
{
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const uint32_t cu = (uint32_t)a.piece_units;
    {
        const int per = (a.batch + kSkThreads - 1) / kSkThreads;
        const int s0 = tid * per;
        int local = 0, local_ne = 0;
        for (int k = 0; k < per; ++k) {
            const int s = s0 + k;
            if (s < a.batch) {
                const int c = a.ctx_lens[s];
                s_ctx[s] = c;
                local += (c + (1 << TSHIFT) - 1) >> TSHIFT;
                local_ne += c > 0 ? 1 : 0;
            }
        }
        const int incl = wave_inclusive_sum(local, lane), incl_ne = wave_inclusive_sum(local_ne, lane);
        if (lane == 63) {
            s_wsum[wave] = incl;
            s_wsum[kSkWaves + wave] = incl_ne;
        }
        __syncthreads();
        int before = 0, before_ne = 0;
        for (int w = 0; w < wave; ++w) {
            before += s_wsum[w];
            before_ne += s_wsum[kSkWaves + w];
        }
        // weighted position of the first tile of sequence s: its tiles and non-empty sequences before
        auto wpos = [&](int tiles_before, int ne_before) -> unsigned long long {
            return (unsigned long long)pairs * ((unsigned long long)kTileUnits * (uint32_t)tiles_before +
                                                (unsigned long long)cu * (uint32_t)ne_before);
        };
        int run = before + incl - local, run_ne = before_ne + incl_ne - local_ne;
        for (int k = 0; k < per; ++k) {
            const int s = s0 + k;
            if (s < a.batch) {
                s_prefix[s] = run;
                s_wpos[s] = wpos(run, run_ne);
                run += (s_ctx[s] + (1 << TSHIFT) - 1) >> TSHIFT;
                run_ne += s_ctx[s] > 0 ? 1 : 0;
            }
        }
        if (tid == kSkThreads - 1) {
            s_prefix[a.batch] = before + incl;
            s_wpos[a.batch] = wpos(before + incl, before_ne + incl_ne);
        }
        __syncthreads();
    }

    // Nobody else writes the output rows of a sequence without tokens: the workgroups share them
    // out (the merge kernel does it when there is one).
    if (a.fused) {
        const int words = a.v.n_q_local * (D / 2);
        for (int sq = blockIdx.x; sq < a.batch; sq += gridDim.x) {
            if (s_ctx[sq] != 0) continue;
            uint32_t* row = reinterpret_cast<uint32_t*>(a.out + (int64_t)sq * a.v.n_q_local * D);
            for (int e = tid; e < words; e += kSkThreads) row[e] = 0u;
        }
    }

    const unsigned long long w_all = s_wpos[a.batch];
    splitter sx = {a, pairs, lane, s_prefix, s_wpos, uniform(s_prefix[a.batch]) * pairs, cu,
                   ((unsigned long long)uniform((int)(w_all >> 32)) << 32) | (uint32_t)uniform((int)w_all)};
    sp.w = blockIdx.x * kSkWaves + wave;
    const tile_pos first = sx.tile_at(sx.range_u(sp.w));
    sp.x0 = first.x;
    sp.x1 = first.x;
    sp.s = first.s;
    sp.tiles_s = first.tiles_s;
    sp.pair = first.pair;
    sp.tile = first.tile;
    return sx;
}

// ---- partial results and their combination -----------------------------------------------------
// Partials travel between wavefronts that may run on different XCDs, each with its own L2.  They are
// written and read with relaxed device-scope atomic accesses of 64 bits, which the hardware serves
// at the device's point of coherence (write-through stores, loads that bypass the local caches);
// ordering comes from waiting for the stores' acknowledgement before the arrival word is touched,
// not from cache-wide fences.
// Lane (r, quad), r < cols, holds o[j][i] = O[row r][32 quad + 8 i + j] of the piece; m and l are the
// row's maximum and denominator (the same in the four lanes of a row).  The rows go through the
// wavefront's LDS buffer (8 KiB, free between tiles) so that one store instruction writes one whole
// row of 512 contiguous bytes: write-through stores of 8 bytes scattered over 64 cache lines, as
// the register arrangement would give, cost tens of microseconds per call.
__device__ __forceinline__ void store_partial(const kv_streamk_args& a, int64_t slot, int cols, int r,
                                              int quad, const f32x4 (&o)[8], float m, float l,
                                              kv_u32x4* stage16, int lane)
{
    float* stage = reinterpret_cast<float*>(stage16);
    __builtin_amdgcn_wave_barrier();
    if (r < cols) {
        float* row = stage + r * D + 32 * quad;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            *reinterpret_cast<f32x4*>(row + 8 * i) = f32x4{o[0][i], o[1][i], o[2][i], o[3][i]};
            *reinterpret_cast<f32x4*>(row + 8 * i + 4) = f32x4{o[4][i], o[5][i], o[6][i], o[7][i]};
        }
    }
    __builtin_amdgcn_wave_barrier();
    float* dst = a.part_acc + slot * cols * D + 2 * lane;
    for (int j = 0; j < cols; ++j) {
        const f32x2 x = *reinterpret_cast<const f32x2*>(stage + j * D + 2 * lane);
        st_coherent2(dst + j * D, x[0], x[1]);
    }
    if (quad == 0 && r < cols) st_coherent2(a.part_ml + (slot * cols + r) * 2, m, l);
    __builtin_amdgcn_wave_barrier();
}

// The partial of a wavefront that has no tiles but whose slot lies among a cut pair's pieces.
__device__ __forceinline__ void store_empty_partial(const kv_streamk_args& a, int64_t slot, int lane)
{
    for (int e = lane; e < a.cols * (D / 2); e += 64) st_coherent2(a.part_acc + slot * a.cols * D + 2 * e, 0.f, 0.f);
    if (lane < a.cols) st_coherent2(a.part_ml + (slot * a.cols + lane) * 2, kNegInf, 0.f);
}

__device__ __forceinline__ void store_final(uint16_t* out_rows, int cols, int r, int quad,
                                            const f32x4 (&o)[8], float l)
{
    if (r >= cols) return;
    const float inv = 1.0f / l;
    uint16_t* dst = out_rows + r * D + 32 * quad;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        kv_u32x4 pk;
#pragma unroll
        for (int u = 0; u < 4; ++u) pk[u] = pack_bf16x2(o[2 * u][i] * inv, o[2 * u + 1][i] * inv);
        *reinterpret_cast<kv_u32x4*>(dst + 8 * i) = pk;
    }
}

// Arrival word of a pair: bits 0..15 pieces arrived, bits 16..39 (number of the wavefront with the
// first piece) + 1, bits 40..63 (number of the wavefront with the last piece) + 1.
constexpr int kSyncFirstShift = 16, kSyncLastShift = 40;

// What a wavefront owes the cut pairs it held pieces of; settled at the end of its range, when the
// stores of its first piece have long been acknowledged.  At most two: the pair its range starts
// inside and the pair it ends inside.
struct cut_pieces {
    int n;
    int s[2], sub[2];            // sequence, index of the pair in the sequence
    unsigned long long add[2];
};

__device__ __forceinline__ void note_piece(cut_pieces& cp, int s, int sub, int w, bool first, bool last)
{
    // (n is 0 or 1 here; written without indexing by a variable so that the notes stay in registers)
    const unsigned long long add = 1ull | (first ? (unsigned long long)(w + 1) << kSyncFirstShift : 0ull) |
                                   (last ? (unsigned long long)(w + 1) << kSyncLastShift : 0ull);
    if (cp.n >= 2) return;   // (cannot happen: only the first and the last piece of a range can be cut)
    if (cp.n == 0) {
        cp.s[0] = s;
        cp.sub[0] = sub;
        cp.add[0] = add;
    } else {
        cp.s[1] = s;
        cp.sub[1] = sub;
        cp.add[1] = add;
    }
    ++cp.n;
}

// x of the lane that `CTRL` (a DPP control word) pairs this lane with.
template <int CTRL>
__device__ __forceinline__ float dpp_from(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
// Maximum / sum over aligned groups of N = 4, 8 or 16 adjacent lanes, left in every lane of the
// group: exchanges inside quads, then the mirror images of half rows and rows.
template <int N>
__device__ __forceinline__ float group_max(float x)
{
    x = fmaxf(x, dpp_from<0xB1>(x));   // lanes 1 0 3 2
    x = fmaxf(x, dpp_from<0x4E>(x));   // lanes 2 3 0 1
    if (N >= 8) x = fmaxf(x, dpp_from<0x141>(x));    // mirror of the half row
    if (N >= 16) x = fmaxf(x, dpp_from<0x140>(x));   // mirror of the row
    return x;
}
template <int N>
__device__ __forceinline__ float group_sum(float x)
{
    x += dpp_from<0xB1>(x);
    x += dpp_from<0x4E>(x);
    if (N >= 8) x += dpp_from<0x141>(x);
    if (N >= 16) x += dpp_from<0x140>(x);
    return x;
}

// Combine the pieces of a pair (sequence s, pair `sub` of it) held in the slots of wavefronts
// w_first..w_last and write the pair's output rows.  One wavefront does it, at the very end of the
// kernel, so the work per piece is kept to a load and two multiply-adds per row and lane.
// CP = rows compiled for (a power of two, cols <= CP; EXACT: cols == CP, so that the row offsets
// are constants of the load instructions).  The pieces are taken RB = 64 / CP at a time.  For the
// (m, l) of a batch, lane u stands for (row u / RB, piece u % RB): one load fetches all of them,
// the row-wise maximum and denominator are reductions over RB adjacent lanes, and the weight
// 2^(m - max) of a piece's row is computed once, in its lane, and handed to all lanes through LDS.
// For the accumulators, lane e owns elements 2 e, 2 e + 1 of every row: a piece's row is one load
// of 512 contiguous bytes from a base that is the same for the whole wavefront.
template <int CP, bool EXACT>
__device__ __forceinline__ void merge_pieces(const kv_streamk_args& a, int s, int sub, int w_first, int w_last,
                                             int lane, kv_u32x4* stage16)
{
    constexpr int RB = 64 / CP;
    constexpr int LOG_RB = RB == 16 ? 4 : RB == 8 ? 3 : 2;
    const int cols = EXACT ? CP : a.cols, n_pieces = w_last - w_first + 1;
    const int my_row = lane >> LOG_RB, my_sub = lane & (RB - 1);
    const int64_t slot0 = (int64_t)w_first + (int64_t)s * a.pairs + sub;
    float* stage = reinterpret_cast<float*>(stage16);   // [row * RB + piece]: weights; [64 + row]: keep
    const uint32_t lane_off = (uint32_t)lane * 8u;       // this lane's two elements of a row, in bytes
    const char* acc_bytes = reinterpret_cast<const char*>(a.part_acc);
    const int64_t rec_bytes = (int64_t)cols * (D * 4);
    float m_run = kNegInf, l_run = 0.f;     // of row my_row (the same in the RB lanes of that row)
    float acc0[CP], acc1[CP];
#pragma unroll
    for (int j = 0; j < CP; ++j) acc0[j] = acc1[j] = 0.f;

    for (int r0 = 0; r0 < n_pieces; r0 += RB) {
        // pieces and rows past the end are read again from the last valid one and weighted zero
        const bool mine = (r0 + my_sub < n_pieces) && (my_row < cols);
        const f32x2 ml = ld_coherent2(a.part_ml + ((slot0 + min(r0 + my_sub, n_pieces - 1)) * cols +
                                                    min(my_row, cols - 1)) * 2);
        f32x2 av[RB][CP];
#pragma unroll
        for (int rr = 0; rr < RB; ++rr) {
            const char* rec = acc_bytes + (slot0 + min(r0 + rr, n_pieces - 1)) * rec_bytes;
#pragma unroll
            for (int j = 0; j < CP; ++j) {
                const uint32_t off = lane_off + (uint32_t)((EXACT ? j : min(j, cols - 1)) * (D * 4));
                av[rr][j] = ld_coherent2(reinterpret_cast<const float*>(rec + off));
            }
        }
        const float m = mine ? ml[0] : kNegInf;   // (-inf also from a wavefront that had no tiles)
        const float m_new = fmaxf(m_run, group_max<RB>(m));
        const float ref = (m_new == kNegInf) ? 0.f : m_new;
        const float keep = fast_exp2(m_run - ref);       // what the running sums are scaled by
        const float wgt = fast_exp2(m - ref);            // weight of this lane's (row, piece)
        l_run = l_run * keep + group_sum<RB>(mine ? ml[1] * wgt : 0.f);
        m_run = m_new;
        __builtin_amdgcn_wave_barrier();
        stage[lane] = wgt;
        if (my_sub == 0) stage[64 + my_row] = keep;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int j = 0; j < CP; ++j) {
            const float kj = stage[64 + j];
            f32x4 w4[RB / 4];
#pragma unroll
            for (int q = 0; q < RB / 4; ++q) w4[q] = *reinterpret_cast<const f32x4*>(stage + j * RB + 4 * q);
            float x0 = acc0[j] * kj, x1 = acc1[j] * kj;
#pragma unroll
            for (int rr = 0; rr < RB; ++rr) {
                x0 = fmaf(w4[rr / 4][rr % 4], av[rr][j][0], x0);
                x1 = fmaf(w4[rr / 4][rr % 4], av[rr][j][1], x1);
            }
            acc0[j] = x0;
            acc1[j] = x1;
        }
    }
    __builtin_amdgcn_wave_barrier();
    if (my_sub == 0) stage[my_row] = 1.0f / l_run;
    __builtin_amdgcn_wave_barrier();
    uint32_t* dst = reinterpret_cast<uint32_t*>(a.out + ((int64_t)s * a.v.n_q_local + (int64_t)sub * cols) * D) + lane;
#pragma unroll
    for (int j = 0; j < CP; ++j) {
        const float inv = stage[j];
        if (EXACT || j < cols) dst[j * (D / 2)] = pack_bf16x2(acc0[j] * inv, acc1[j] * inv);
    }
    __builtin_amdgcn_wave_barrier();
}

// End of a wavefront's range: announce its cut pieces; where this completes a pair, combine it.
__device__ __forceinline__ void settle_pieces(const kv_streamk_args& a, const cut_pieces& cp, int lane, int w,
                                              kv_u32x4* stage)
{
    if (!a.fused || cp.n == 0) return;
    // every partial this wavefront stored has reached the point of coherence
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    unsigned long long seen0 = 0ull, seen1 = 0ull;
    if (lane == 0) {
        seen0 = __hip_atomic_fetch_add(a.pair_sync + ((int64_t)cp.s[0] * a.pairs + cp.sub[0]), cp.add[0],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cp.n > 1)
            seen1 = __hip_atomic_fetch_add(a.pair_sync + ((int64_t)cp.s[1] * a.pairs + cp.sub[1]), cp.add[1],
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
#pragma unroll 1
    for (int k = 0; k < cp.n; ++k) {
        const unsigned long long seen = k ? seen1 : seen0, add = k ? cp.add[1] : cp.add[0];
        const int s = k ? cp.s[1] : cp.s[0], sub = k ? cp.sub[1] : cp.sub[0];
        const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)seen);
        const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(seen >> 32));
        const unsigned long long now = (((unsigned long long)hi << 32) | lo) + add;
        const int count = (int)(now & 0xffffu);
        const int first = (int)((now >> kSyncFirstShift) & 0xffffffu), last = (int)(now >> kSyncLastShift);
        if (first == 0 || last == 0 || count != last - first + 1) continue;   // others are still to come
        // (a workspace handed over with arrival words that were not zero can yield anything here:
        // whatever it is, the slots read below lie inside the workspace)
        if (first > last || last > a.n_waves) continue;
        if (lane == 0)   // the word is this wavefront's now: back to zero for the next call
            __hip_atomic_store(a.pair_sync + ((int64_t)s * a.pairs + sub), 0ull, __ATOMIC_RELAXED,
                               __HIP_MEMORY_SCOPE_AGENT);
        switch (a.cols) {
            case 4: merge_pieces<4, true>(a, s, sub, first - 1, last - 1, lane, stage); break;
            case 8: merge_pieces<8, true>(a, s, sub, first - 1, last - 1, lane, stage); break;
            case 16: merge_pieces<16, true>(a, s, sub, first - 1, last - 1, lane, stage); break;
            default:
                if (a.cols < 4) merge_pieces<4, false>(a, s, sub, first - 1, last - 1, lane, stage);
                else if (a.cols < 8) merge_pieces<8, false>(a, s, sub, first - 1, last - 1, lane, stage);
                else merge_pieces<16, false>(a, s, sub, first - 1, last - 1, lane, stage);
        }
    }
}

// A wavefront without tiles (fewer tiles than wavefronts).  Its range is the empty one at tile x:
// if tiles x - 1 and x belong to the same pair, that pair is cut between the neighbouring
// wavefronts and this one counts among its pieces, with an empty partial (m = -inf, l = 0, zeros).
__device__ __forceinline__ void empty_wavefront(const kv_streamk_args& a, const int32_t* s_prefix, int pairs,
                                                int x, int w, int lane, kv_u32x4* stage)
{
    if (x <= 0) return;
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (uniform(s_prefix[mid]) * pairs <= x - 1) lo = mid; else hi = mid;
    }
    const int ts = uniform(s_prefix[lo + 1]) - uniform(s_prefix[lo]);
    const int rel = x - 1 - uniform(s_prefix[lo]) * pairs;
    const int pr = rel / ts;
    const bool inside = (rel - pr * ts) + 1 < ts;
    const int64_t pair = (int64_t)lo * pairs + pr;
    if (a.fused && !inside) return;
    store_empty_partial(a, (int64_t)w + pair, lane);
    if (a.fused) {
        cut_pieces cp;
        cp.n = 0;
        note_piece(cp, lo, pr, w, false, false);
        settle_pieces(a, cp, lane, w, stage);
    }
}

template <bool MIXED>
__global__ __launch_bounds__(kSkThreads, 1) void decode_streamk_kernel(kv_streamk_args a)
{
    __shared__ kv_u32x4 s_kstage[kSkWaves * 512];
    __shared__ int32_t s_prefix[kMaxBatch + 1];             // tiles of the sequences before s
    __shared__ int32_t s_ctx[kMaxBatch];
    __shared__ unsigned long long s_wpos[kMaxBatch + 1];    // weighted position of the first tile of s
    __shared__ int32_t s_wsum[2 * kSkWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const kv_view_dev& v = a.v;
    const int Hl = v.n_kv_local, G = a.group;
    kv_u32x4* kstage = s_kstage + wave * 512;

    split_pos sp;
    const splitter sx = split_prologue<5>(a, Hl, s_prefix, s_wpos, s_ctx, s_wsum, sp);
    int x0 = sp.x0, s = sp.s, tiles_s = sp.tiles_s, hl = sp.pair, tile = sp.tile;
    const int w = sp.w;
    if (x0 >= sx.total) {   // the range starts where the batch ends: no tiles
        empty_wavefront(a, s_prefix, Hl, x0, w, lane, kstage);
        return;
    }
    cut_pieces cp;
    cp.n = 0;

    lane_consts lc;
    lc.r = lane & 15;
    lc.quad = lane >> 4;
    const int64_t plane_bytes = v.plane_elems * 2;
    // layout of the current sequence's blocks (MIXED: looked up per sequence; else the view's own)
    kv_layout_dev lay = {v.block_tokens, v.block_shift, v.token_stride, v.head_off};
    int token_stride_bytes, halves_per_block, half_shift;
    auto use_layout = [&]() {
        token_stride_bytes = lay.token_stride * 2;
        lc.voff = (uint32_t)(lc.quad * token_stride_bytes + lc.r * 16);
        lc.vstep = (uint32_t)(4 * token_stride_bytes);
        halves_per_block = lay.block_tokens >> 4;  // capacity is a multiple of 16
        half_shift = lay.block_shift >= 4 ? lay.block_shift - 4 : -1;
    };
    use_layout();

    // state of the pair being walked
    int n, n_full, last_block, id_base, idv;
    const int32_t* trow;
    const char* head_base;
    bf16x8 qb[4];
    softmax_state st;
    auto half_block = [&](int hh) -> int {  // index of the block holding 16-token half hh
        return half_shift >= 0 ? (hh >> half_shift) : hh / halves_per_block;
    };
    // block ids of 64 consecutive 16-token halves, one per lane, refilled every 32 tiles
    auto half_base = [&](int hh) -> const char* {
        if (hh - id_base >= 64) {
            id_base = hh;
            idv = trow[min(half_block(id_base + lane), last_block)];
        }
        const int blk = __builtin_amdgcn_readlane(idv, hh - id_base);
        const int slot0 = (hh - half_block(hh) * halves_per_block) << 4;
        return head_base + (int64_t)blk * (v.block_elems * 2) + (int64_t)slot0 * token_stride_bytes;
    };
    // pair (s, hl), entered at tile `tile`: query rows, block ids, empty running state
    auto open_pair = [&]() {
        if (MIXED) {
            const int vid = min(max(uniform(a.view_ids[s]), 0), a.n_views - 1);
            lay = a.lay[vid];
            use_layout();
        }
        n = uniform(s_ctx[s]);
        n_full = n >> 5;                 // tiles of this pair with all 32 tokens valid
        trow = a.table + (int64_t)s * a.table_stride;
        head_base = reinterpret_cast<const char*>(a.pool + lay.head_off + hl * D);
        last_block = (n - 1) / lay.block_tokens;
        const char* qrows = reinterpret_cast<const char*>(a.q + ((int64_t)s * v.n_q_local + hl * G) * D);
        const uint32_t qoff = (uint32_t)(min(lc.r, G - 1) * (D * 2) + lc.quad * 16);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kv_u32x4 raw = ld16_cached(qrows, qoff + kk * 64);
            if (lc.r >= G) raw = kv_u32x4{0u, 0u, 0u, 0u};
            qb[kk] = as_bf16x8(raw);
        }
        st.m = kNegInf;
        st.l = 0.f;
#pragma unroll
        for (int j = 0; j < 8; ++j) st.o[j] = f32x4{0.f, 0.f, 0.f, 0.f};
        id_base = 2 * tile;
        idv = trow[min(half_block(id_base + lane), last_block)];
    };

    // The first pair is opened and its first tile requested before the end of the range is worked
    // out: that arithmetic then runs while the loads are under way.
    tile_regs ta, tb;
    open_pair();
    bool primed = tile < n_full;
    if (primed) {
        const char* kb[2] = {half_base(2 * tile), half_base(2 * tile + 1)};
        load_full(ta, kb, plane_bytes, lc);
    }
    const int x1 = sx.range_end(w);
    if (x0 >= x1) {
        empty_wavefront(a, s_prefix, Hl, x1, w, lane, kstage);
        return;
    }

    for (;;) {
        const int seg_end = min(tiles_s, tile + (x1 - x0));
        const int full_end = min(seg_end, n_full);

        // full tiles, one tile ahead of the arithmetic in a second register set
        int i = tile;
        if (i < full_end && !primed) {
            const char* kb[2] = {half_base(2 * i), half_base(2 * i + 1)};
            load_full(ta, kb, plane_bytes, lc);
        }
        primed = false;
        while (i + 2 <= full_end) {
            {
                const char* kb[2] = {half_base(2 * i + 2), half_base(2 * i + 3)};
                load_full(tb, kb, plane_bytes, lc);
            }
            compute_tile<false>(ta, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
            if (i + 2 < full_end) {
                const char* kb[2] = {half_base(2 * i + 4), half_base(2 * i + 5)};
                load_full(ta, kb, plane_bytes, lc);
            }
            compute_tile<false>(tb, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
            i += 2;
        }
        if (i < full_end) {
            compute_tile<false>(ta, qb, st, a.scale_log2e, 31, lc.r, lc.quad, kstage);
            ++i;
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
            load_tail(ta, kb, plane_bytes, lc, last, token_stride_bytes);
            compute_tile<true>(ta, qb, st, a.scale_log2e, last, lc.r, lc.quad, kstage);
        }

        // ---- piece done: final rows or partial --------------------------------------------------
        st.l += __shfl_xor(st.l, 16);
        st.l += __shfl_xor(st.l, 32);
        const bool is_first = tile == 0, is_last = seg_end == tiles_s;
        const int64_t pair = (int64_t)s * Hl + hl;
        if (is_first && is_last) {
            store_final(a.out + ((int64_t)s * v.n_q_local + hl * G) * D, G, lc.r, lc.quad, st.o, st.l);
            if (!a.fused && lane == 0)   // one piece: the merge kernel must find first == last here
                *reinterpret_cast<int2*>(a.pair_desc + pair * 2) = int2{w, w};
        } else {
            store_partial(a, (int64_t)w + pair, G, lc.r, lc.quad, st.o, st.m, st.l, kstage, lane);
            if (a.fused) {
                note_piece(cp, s, hl, w, is_first, is_last);
            } else if (lane == 0) {
                // first and last piece of the pair tell the merge kernel where its pieces lie
                if (is_first) a.pair_desc[pair * 2] = w;
                if (is_last) a.pair_desc[pair * 2 + 1] = w;
            }
        }

        // ---- next pair --------------------------------------------------------------------------
        x0 += seg_end - tile;
        if (x0 >= x1) break;
        tile = 0;
        if (++hl == Hl) {
            hl = 0;
            do {
                ++s;
                tiles_s = uniform(s_prefix[s + 1]) - uniform(s_prefix[s]);   // (s < batch: tiles are left)
            } while (tiles_s == 0);
        }
        open_pair();
    }
    settle_pieces(a, cp, lane, w, kstage);
}

// ---- several adjacent KV heads per wavefront ----------------------------------------------------
// In a block whose token rows hold several local KV heads, a wavefront that reads one head
// touches 256 bytes per token; measured on pure-read probes that pattern streams 10-12 % slower
// than rows of 512 or 1024 bytes.  This variant gives a wavefront HPW = 2 or 4 adjacent heads: a
// pair is (sequence, head group), its HPW * G <= 16 query rows fill the 16 columns of the B
// operand that the one-head kernel pads, and a tile is 2 * TG tokens, TG = 16 / HPW.
//
// The 16 A rows of the score product are (head a, token t) combinations of one group of TG tokens,
// row = a * TG + t; the B operand holds all 16 query rows, so S^T[(a, t)][(b, g)] is a score only
// where a == b.  In the C layout lane (col, quad) holds rows 4 quad + i: head a = row / TG is
// fixed per lane, so a lane either owns four tokens of its own column (a == b) or only cross
// products, which it masks to -inf.  The masked S^T is again the B operand of the second product,
// whose contraction index 4 quad + j = a * TG + t runs over heads as well as tokens: the A operand
// takes V rows of head a for index (a, t), and the zeros of P remove the other heads' terms.  One
// accumulator O^T[e][col] therefore serves all heads of the group, and a column's running maximum
// lives in the lanes that own it (HPW = 4: one lane; HPW = 2: two lanes 16 apart).
typedef short bf16x4_bits __attribute__((ext_vector_type(4)));

struct wide_tile {
    kv_u32x4 k[8];     // K rows as they lie in memory, 1 KiB per load instruction
    kv_u32x4 v[2][4];  // [group][j]: piece r of the V row for contraction index 4 quad + j
};

struct wide_lane {
    int r, quad;
    int ktok, kcol;   // K loads: token within an instruction's tokens, byte offset inside the token row
    int vtok, vcol;   // V loads: first token of this lane within a group, byte offset inside the row
    int krow;         // row of the K staging buffer holding A row r of group 0
    bool mine;        // this lane's rows of S^T belong to its own column
    int src;          // a lane owning this lane's column (source of the rescale factor)
};

struct wide_state {
    float m, l;   // m: reference maximum of the column (owners; 0 in other lanes), may lag the true one
    f32x4 o[8];   // o[e][i] = O[col = r][32 quad + 8 i + e]
};

constexpr float kWideLag = 8.0f;  // the reference maximum moves only when exceeded by 2^8

template <int HPW>
__device__ __forceinline__ void load_wide(wide_tile& t, const char* base, int64_t plane_bytes,
                                          const wide_lane& wl, int stride_bytes)
{
    constexpr int TG = 16 / HPW, TPI = 4 / HPW;
    const uint32_t koff = (uint32_t)(wl.ktok * stride_bytes + wl.kcol);
#pragma unroll
    for (int u = 0; u < 8; ++u) t.k[u] = ld16(base, koff + (uint32_t)(u * TPI * stride_bytes));
    const char* vb = base + plane_bytes;
    const uint32_t voff = (uint32_t)(wl.vtok * stride_bytes + wl.vcol);
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
        for (int j = 0; j < 4; ++j) t.v[gi][j] = ld16(vb, voff + (uint32_t)((gi * TG + j) * stride_bytes));
}

// Last, partial tile of a pair: rows past the last valid token (index `last` in the tile) are
// replaced by that token's row (finite data; their scores are masked).
template <int HPW>
__device__ __forceinline__ void load_wide_tail(wide_tile& t, const char* base, int64_t plane_bytes,
                                               const wide_lane& wl, int stride_bytes, int last)
{
    constexpr int TG = 16 / HPW, TPI = 4 / HPW;
#pragma unroll
    for (int u = 0; u < 8; ++u)
        t.k[u] = ld16(base, (uint32_t)(min(u * TPI + wl.ktok, last) * stride_bytes + wl.kcol));
    const char* vb = base + plane_bytes;
#pragma unroll
    for (int gi = 0; gi < 2; ++gi)
#pragma unroll
        for (int j = 0; j < 4; ++j)
            t.v[gi][j] = ld16(vb, (uint32_t)(min(gi * TG + wl.vtok + j, last) * stride_bytes + wl.vcol));
}

template <int HPW, bool TAIL>
__device__ __forceinline__ void compute_wide(const wide_tile& t, const bf16x8 (&qb)[4], wide_state& st,
                                             float scale_log2e, int last, const wide_lane& wl,
                                             kv_u32x4* kstage)
{
    constexpr int TG = 16 / HPW;
    const int r = wl.r, quad = wl.quad;
    // K rows -> staging buffer (row = token * HPW + head = 4 u + quad, pieces XOR-swizzled as in
    // the one-head kernel) -> A operands
#pragma unroll
    for (int u = 0; u < 8; ++u) {
        const int row = 4 * u + quad;
        kstage[row * 16 + (r ^ (row & 15))] = t.k[u];
    }
    __builtin_amdgcn_wave_barrier();
    f32x4 sacc[2];
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
        sacc[gi] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const kv_u32x4 ka = kstage[(16 * gi + wl.krow) * 16 + ((4 * kk + quad) ^ wl.krow)];
            sacc[gi] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(ka), qb[kk], sacc[gi], 0, 0, 0);
        }
    }
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int gi = 0; gi < 2; ++gi) {
        float sv[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            bool ok = wl.mine;
            if (TAIL) ok = ok && (gi * TG + wl.vtok + i <= last);
            sv[i] = ok ? sacc[gi][i] * scale_log2e : kNegInf;
        }
        float mx = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
        if (HPW == 2) mx = fmaxf(mx, __shfl_xor(mx, 16));
        if (__builtin_amdgcn_ballot_w64(mx > st.m + kWideLag) != 0) {
            const float m_new = (mx > st.m + kWideLag) ? mx : st.m;
            const float alpha = fast_exp2(st.m - m_new);  // 1 where unchanged, 0 on first use
            st.m = m_new;
            st.l *= alpha;
            const float col_alpha = __shfl(alpha, wl.src);
#pragma unroll
            for (int e = 0; e < 8; ++e) st.o[e] *= col_alpha;
        }
        // weights rounded to bf16 for the second product; the denominator sums the same rounded values
        const uint32_t p01 = pack_bf16x2(fast_exp2(sv[0] - st.m), fast_exp2(sv[1] - st.m));
        const uint32_t p23 = pack_bf16x2(fast_exp2(sv[2] - st.m), fast_exp2(sv[3] - st.m));
        st.l += pair_sum(p01) + pair_sum(p23);
        const bf16x4_bits pb = __builtin_bit_cast(bf16x4_bits, uint2{p01, p23});
        // V^T operands: element e of the four loaded pieces, token pairs packed per dword
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const int w = e >> 1;
            const uint32_t sel = (e & 1) ? 0x07060302u : 0x05040100u;
            const uint32_t lo = __builtin_amdgcn_perm(t.v[gi][1][w], t.v[gi][0][w], sel);
            const uint32_t hi = __builtin_amdgcn_perm(t.v[gi][3][w], t.v[gi][2][w], sel);
            const bf16x4_bits av = __builtin_bit_cast(bf16x4_bits, uint2{lo, hi});
            st.o[e] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(av, pb, st.o[e], 0, 0, 0);
        }
    }
}

template <int HPW, bool MIXED>
__global__ __launch_bounds__(kSkThreads, 1) void decode_wide_kernel(kv_streamk_args a)
{
    constexpr int TG = 16 / HPW, TSHIFT = HPW == 4 ? 3 : 4, TILE = 1 << TSHIFT;
    __shared__ kv_u32x4 s_kstage[kSkWaves * 512];
    __shared__ int32_t s_prefix[kMaxBatch + 1];             // tiles of the sequences before s
    __shared__ int32_t s_ctx[kMaxBatch];
    __shared__ unsigned long long s_wpos[kMaxBatch + 1];    // weighted position of the first tile of s
    __shared__ int32_t s_wsum[2 * kSkWaves];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = uniform(tid >> 6);
    const kv_view_dev& v = a.v;
    const int P = a.pairs, C = a.cols, G = a.group;
    kv_u32x4* kstage = s_kstage + wave * 512;

    split_pos sp;
    const splitter sx = split_prologue<TSHIFT>(a, P, s_prefix, s_wpos, s_ctx, s_wsum, sp);
    int x0 = sp.x0, s = sp.s, tiles_s = sp.tiles_s, hg = sp.pair, tile = sp.tile;
    const int w = sp.w;
    if (x0 >= sx.total) {   // the range starts where the batch ends: no tiles
        empty_wavefront(a, s_prefix, P, x0, w, lane, kstage);
        return;
    }
    cut_pieces cp;
    cp.n = 0;

    wide_lane wl;
    wl.r = lane & 15;
    wl.quad = lane >> 4;
    wl.ktok = lane / (16 * HPW);
    wl.kcol = (lane % (16 * HPW)) * 16;
    wl.vtok = HPW == 4 ? 0 : 4 * (wl.quad & 1);
    wl.vcol = HPW == 4 ? lane * 16 : (wl.quad >> 1) * 256 + wl.r * 16;
    wl.krow = (wl.r % TG) * HPW + wl.r / TG;
    {
        const int b = wl.r / G;                            // head of this lane's column
        const int head = HPW == 4 ? wl.quad : wl.quad >> 1;  // head of this lane's rows of S^T
        wl.mine = (wl.r < C) && (head == b);
        wl.src = (wl.r < C) ? (HPW == 4 ? b : 2 * b) * 16 + wl.r : lane;
    }
    const int64_t plane_bytes = v.plane_elems * 2;
    // layout of the current sequence's blocks (MIXED: looked up per sequence; else the view's own)
    kv_layout_dev lay = {v.block_tokens, v.block_shift, v.token_stride, v.head_off};
    int stride_bytes, tiles_per_block, tile_blk_shift;
    auto use_layout = [&]() {
        stride_bytes = lay.token_stride * 2;
        tiles_per_block = lay.block_tokens >> TSHIFT;  // capacity is a multiple of 16
        tile_blk_shift = lay.block_shift >= TSHIFT ? lay.block_shift - TSHIFT : -1;
    };
    use_layout();

    // state of the pair being walked
    int n, n_full, last_block, id_base, idv;
    const int32_t* trow;
    const char* head_base;
    bf16x8 qb[4];
    wide_state st;
    auto tile_block = [&](int i) -> int {
        return tile_blk_shift >= 0 ? (i >> tile_blk_shift) : i / tiles_per_block;
    };
    // block ids of 64 consecutive blocks, one per lane, refilled when the walk leaves them
    auto tile_base = [&](int i) -> const char* {
        const int jb = tile_block(i);
        if (jb - id_base >= 64) {
            id_base = jb;
            idv = trow[min(id_base + lane, last_block)];
        }
        const int blk = __builtin_amdgcn_readlane(idv, jb - id_base);
        const int slot0 = (i - jb * tiles_per_block) << TSHIFT;
        return head_base + (int64_t)blk * (v.block_elems * 2) + (int64_t)slot0 * stride_bytes;
    };
    // pair (s, hg), entered at tile `tile`: query rows, block ids, empty running state
    auto open_pair = [&]() {
        if (MIXED) {
            const int vid = min(max(uniform(a.view_ids[s]), 0), a.n_views - 1);
            lay = a.lay[vid];
            use_layout();
        }
        n = uniform(s_ctx[s]);
        n_full = n >> TSHIFT;            // tiles of this pair with every token valid
        trow = a.table + (int64_t)s * a.table_stride;
        head_base = reinterpret_cast<const char*>(a.pool + lay.head_off + hg * (HPW * D));
        last_block = (n - 1) / lay.block_tokens;
        const char* qrows = reinterpret_cast<const char*>(a.q + ((int64_t)s * v.n_q_local + hg * C) * D);
        const uint32_t qoff = (uint32_t)(min(wl.r, C - 1) * (D * 2) + wl.quad * 16);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kv_u32x4 raw = ld16_cached(qrows, qoff + kk * 64);
            if (wl.r >= C) raw = kv_u32x4{0u, 0u, 0u, 0u};
            qb[kk] = as_bf16x8(raw);
        }
        st.m = wl.mine ? kNegInf : 0.f;
        st.l = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[e] = f32x4{0.f, 0.f, 0.f, 0.f};
        id_base = tile_block(tile);
        idv = trow[min(id_base + lane, last_block)];
    };

    // The first pair is opened and its first tile requested before the end of the range is worked
    // out: that arithmetic then runs while the loads are under way.
    wide_tile ta, tb;
    open_pair();
    bool primed = tile < n_full;
    if (primed) load_wide<HPW>(ta, tile_base(tile), plane_bytes, wl, stride_bytes);
    const int x1 = sx.range_end(w);
    if (x0 >= x1) {
        empty_wavefront(a, s_prefix, P, x1, w, lane, kstage);
        return;
    }

    for (;;) {
        const int seg_end = min(tiles_s, tile + (x1 - x0));
        const int full_end = min(seg_end, n_full);

        int i = tile;
        if (i < full_end && !primed) load_wide<HPW>(ta, tile_base(i), plane_bytes, wl, stride_bytes);
        primed = false;
        while (i + 2 <= full_end) {
            load_wide<HPW>(tb, tile_base(i + 1), plane_bytes, wl, stride_bytes);
            compute_wide<HPW, false>(ta, qb, st, a.scale_log2e, TILE - 1, wl, kstage);
            if (i + 2 < full_end) load_wide<HPW>(ta, tile_base(i + 2), plane_bytes, wl, stride_bytes);
            compute_wide<HPW, false>(tb, qb, st, a.scale_log2e, TILE - 1, wl, kstage);
            i += 2;
        }
        if (i < full_end) {
            compute_wide<HPW, false>(ta, qb, st, a.scale_log2e, TILE - 1, wl, kstage);
            ++i;
        }
        if (seg_end > full_end) {
            // the pair's last tile, partly filled: tokens TILE * n_full .. n - 1
            const int last = n - 1 - TILE * n_full;  // 0 .. TILE - 2
            load_wide_tail<HPW>(ta, tile_base(n_full), plane_bytes, wl, stride_bytes, last);
            compute_wide<HPW, true>(ta, qb, st, a.scale_log2e, last, wl, kstage);
        }

        // ---- piece done: final rows or partial ------------------------------------------------------
        st.l += __shfl_xor(st.l, 16);
        st.l += __shfl_xor(st.l, 32);
        const float m_col = __shfl(st.m, wl.src);
        const bool is_first = tile == 0, is_last = seg_end == tiles_s;
        const int64_t pair = (int64_t)s * P + hg;
        if (is_first && is_last) {
            store_final(a.out + ((int64_t)s * v.n_q_local + hg * C) * D, C, wl.r, wl.quad, st.o, st.l);
            if (!a.fused && lane == 0)   // one piece: the merge kernel must find first == last here
                *reinterpret_cast<int2*>(a.pair_desc + pair * 2) = int2{w, w};
        } else {
            store_partial(a, (int64_t)w + pair, C, wl.r, wl.quad, st.o, m_col, st.l, kstage, lane);
            if (a.fused) {
                note_piece(cp, s, hg, w, is_first, is_last);
            } else if (lane == 0) {
                if (is_first) a.pair_desc[pair * 2] = w;
                if (is_last) a.pair_desc[pair * 2 + 1] = w;
            }
        }

        // ---- next pair ------------------------------------------------------------------------------
        x0 += seg_end - tile;
        if (x0 >= x1) break;
        tile = 0;
        if (++hg == P) {
            hg = 0;
            do {
                ++s;
                tiles_s = uniform(s_prefix[s + 1]) - uniform(s_prefix[s]);   // (s < batch: tiles are left)
            } while (tiles_s == 0);
        }
        open_pair();
    }
    settle_pieces(a, cp, lane, w, kstage);
}

// Merge the pieces of one (sequence, local query head), or write zeros for an empty context.
// The 256 lanes of a workgroup are column groups of 4 elements x slices of the piece list.  A
// short list (the common case: a pair cut over a few wavefronts) is merged by one workgroup as
// 32 column groups x 8 slices; a long one (one sequence cut over hundreds of wavefronts) by
// kMergeSplit workgroups, each owning 128 / kMergeSplit columns as 8 column groups x 32 slices.
// The host launches kMergeSplit workgroups per row only when the batch has few pairs for the
// wavefronts launched (long lists are then the rule); in such a grid all but the first leave at
// once for a short list.  Which slots hold the pieces of a pair is read from the pair's descriptor:
// the numbers of the wavefronts that held its first and its last piece, left by the main kernel,
// so this kernel does not depend on how the tiles were cut.
constexpr int kMergeSplit = 4;
constexpr int kMergeLong = 24;  // pieces from which a list counts as long
__global__ __launch_bounds__(256) void decode_streamk_merge_kernel(kv_streamk_args a)
{
    const int qi = blockIdx.x, s = blockIdx.y, z = blockIdx.z, tid = threadIdx.x;
    const kv_view_dev& v = a.v;
    const int Hl = a.pairs, G = a.cols;  // pairs per sequence, output rows per pair
    __shared__ float s_max[32];
    __shared__ float s_acc[8 * D];
    __shared__ float s_l[32];
    uint16_t* dst = a.out + ((int64_t)s * v.n_q_local + qi) * D;
    const int hl = qi / G, g = qi - hl * G;
    // the context length, and the numbers of the wavefronts that held the pair's first and last piece,
    // left by the main kernel (both requested before either is looked at: one round trip, not two)
    const int2 ends = *reinterpret_cast<const int2*>(a.pair_desc + ((int64_t)s * Hl + hl) * 2);
    const int n = a.ctx_lens[s];
    if (n == 0) {
        if (z == 0 && tid < D) dst[tid] = 0;
        return;
    }
    // (clamped: whatever the words hold, the slots read below lie inside the workspace)
    const int w_first = min(max(ends.x, 0), a.n_waves - 1), w_last = min(ends.y, a.n_waves - 1);
    if (w_first >= w_last) return;                      // one piece: written in place by the main kernel
    const bool wide = (gridDim.z > 1 && w_last - w_first + 1 >= kMergeLong);
    if (!wide && z != 0) return;
    const int64_t pair = (int64_t)s * Hl + hl;
    const int ncg = wide ? D / 4 / kMergeSplit : D / 4;  // column groups of this workgroup
    const int cols = ncg * 4, nsl = 256 / ncg;
    const int col0 = wide ? z * cols : 0;
    const int cg = tid % ncg, slice = tid / ncg;

    // one pass over the pieces of this slice, rescaling on the fly; the slices are then brought
    // to the common maximum and summed through LDS
    float mr = kNegInf, ll = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    constexpr int kBatch = 8;
    // (eight pieces requested at a time: one memory round trip per eight pieces, not one per piece)
    for (int w0 = w_first + slice; w0 <= w_last; w0 += kBatch * nsl) {
        float2 ml[kBatch];
        f32x4 part[kBatch];
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            const int64_t rec = (min(w0 + j * nsl, w_last) + pair) * G + g;
            ml[j] = *reinterpret_cast<const float2*>(a.part_ml + rec * 2);
            part[j] = *reinterpret_cast<const f32x4*>(a.part_acc + rec * D + col0 + cg * 4);
        }
#pragma unroll
        for (int j = 0; j < kBatch; ++j) {
            if (w0 + j * nsl > w_last) break;
            // (a wavefront that had no tiles left m = -inf, l = 0 and zeros: its weight comes out as 0)
            const float mn = fmaxf(mr, ml[j].x);
            const float ref = (mn == kNegInf) ? 0.f : mn;
            const float c_old = fast_exp2(mr - ref), c_new = fast_exp2(ml[j].x - ref);
            ll = ll * c_old + ml[j].y * c_new;
            acc = acc * c_old + part[j] * c_new;
            mr = mn;
        }
    }
    if (cg == 0) s_max[slice] = mr;
    __syncthreads();
    float mm = kNegInf;
    for (int k = 0; k < nsl; ++k) mm = fmaxf(mm, s_max[k]);
    const float cs = fast_exp2(mr - mm);           // 0 for a slice without pieces
    *reinterpret_cast<f32x4*>(&s_acc[slice * cols + cg * 4]) = acc * cs;
    if (cg == 0) s_l[slice] = ll * cs;
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


// Adjacent KV heads one wavefront takes (1: the one-head kernel).  With HPW heads the HPW * G
// query rows of a pair must fit the 16 columns of the matrix-core tile.
static int wide_heads(const kv_view* view, int batch, int n_waves)
{
    if (kv_option_heads_per_wave() == 1) return 1;
    // measured: a gain of 2-5 % where a wavefront then reads whole token rows or the query rows fill
    // the 16 columns
    const int G = view->group, Hl = view->n_kv_local;
    if (G <= 4 && Hl % 4 == 0) return 4;
    if (G > 4 && G <= 8 && Hl % 2 == 0 && Hl >= 4) return 2;
    // two-head rows with small groups (TP4 of the 8B shape): both heads of the row, 2.5 % faster than
    // one on a batch of many sequences (95.5 -> 93.1 us at batch 128); not where a few very long
    // sequences are cut into long piece lists, whose records it doubles (60.3 against 59.9 us)
    if (G <= 4 && Hl % 2 == 0 && (int64_t)batch * Hl * kMergeLong > n_waves) return 2;
    return 1;
}

// Partial results: one slot per (wavefront, pair) piece, n_waves + batch * pairs at most, each
// with `cols` rows of (acc[128], m, l).
static void workspace_layout(const kv_view* view, int batch, int n_waves, int hpw, size_t& acc, size_t& ml)
{
    const size_t pairs = (size_t)view->n_kv_local / hpw, cols = (size_t)view->group * hpw;
    const size_t slots = (size_t)n_waves + (size_t)batch * pairs;
    acc = (slots * cols * D * 4 + 255) / 256 * 256;
    ml = (slots * cols * 2 * 4 + 255) / 256 * 256;
}

// Sized for the larger of the kernels' needs so that the figure does not depend on the options.
// Layout: arrival words (fixed size, at the very start whatever the shape, so that they stay zero
// between calls of any shape), partial accumulators, partial (m, l), pair descriptors.
size_t kv_streamk_workspace_bytes(const kv_view* view, int batch, int n_waves)
{
    size_t need = 0;
    for (int hpw = 1; hpw <= 4; hpw *= 2) {
        if (view->n_kv_local % hpw != 0 || view->group * hpw > 16) continue;
        size_t acc, ml;
        workspace_layout(view, batch, n_waves, hpw, acc, ml);
        if (acc + ml > need) need = acc + ml;
    }
    // pair descriptors: two wavefront numbers per (sequence, pair)
    const size_t desc = ((size_t)batch * view->n_kv_local * 2 * 4 + 255) / 256 * 256;
    return KV_DECODE_SYNC_BYTES + need + desc;
}

int kv_streamk_launch(kv_streamk_args a, const kv_view* view, void* workspace, hipStream_t st)
{
    const int hpw = wide_heads(view, a.batch, a.n_waves);
    a.heads_per_wave = hpw;
    a.pairs = view->n_kv_local / hpw;
    a.cols = view->group * hpw;
    a.tile_shift = hpw == 4 ? 3 : hpw == 2 ? 4 : 5;
    size_t acc, ml;
    workspace_layout(view, a.batch, a.n_waves, hpw, acc, ml);
    char* ws = (char*)workspace;
    a.pair_sync = (unsigned long long*)ws;
    a.part_acc = (float*)(ws + KV_DECODE_SYNC_BYTES);
    a.part_ml = (float*)(ws + KV_DECODE_SYNC_BYTES + acc);
    a.pair_desc = (int32_t*)(ws + KV_DECODE_SYNC_BYTES + acc + ml);
    // How the pieces of a cut pair are combined.  Inside the main kernel, by the last piece to
    // arrive, unless the batch has so few pairs for the wavefronts launched that a pair is cut
    // into kMergeLong pieces or more on average: one wavefront walking such a list would take
    // longer than the second launch, whose merge kernel spreads a long list over a workgroup.
    const int64_t n_pairs = (int64_t)a.batch * a.pairs;
    const bool long_lists = n_pairs * kMergeLong <= a.n_waves;
    const int64_t mode = kv_option_merge_mode();
    // (measured: with up to 8 output rows per pair the one launch is 0.5-1.5 us faster; with the 16 rows
    // of several heads per wavefront the last wavefront's walk over the larger records costs 4 us more
    // than the merge kernel)
    a.fused = (mode == 1 || (mode == 0 && !long_lists && a.cols <= 8)) && n_pairs <= KV_DECODE_SYNC_WORDS &&
              a.n_waves < (1 << 16);
    // Weights of the XCDs.  Workgroup L runs on XCD L mod 8 (read back from the hardware's XCC_ID by
    // kv_probe_read_placed), and the XCDs do not stream equally fast: with equal shares the
    // wavefronts of the odd-numbered ones end later on average (a plain read of equal contiguous
    // shares takes them 2-3 % longer; in this kernel's time stamps the gap was larger).  `skew` / 1024
    // of an even share is therefore moved from each odd to each even one, which shortens the calls
    // measured by 1.5-2 %.  The workgroup -> XCD rule only holds for whole rounds of eight workgroups;
    // otherwise all weigh the same.
    {
        int64_t skew = kv_option_xcd_skew();
        if (skew < 0) skew = kDefaultXcdSkew;
        if ((a.n_waves / kSkWaves) % kMaxClasses != 0) skew = 0;
        a.wt_prefix[0] = 0;
        for (int x = 0; x < kMaxClasses; ++x)
            a.wt_prefix[x + 1] = a.wt_prefix[x] + (uint32_t)(1024 + ((x & 1) ? -skew : skew));
        // total weight = n_waves * 1024 in both cases (the skews of a round of eight cancel)
        a.inv_weight = 1.0 / ((double)a.n_waves * 1024.0);
        const int64_t pc = kv_option_piece_cost();
        a.piece_units = (int32_t)(pc < 0 ? kDefaultPieceUnits : pc);
    }
    const dim3 grid((unsigned)(a.n_waves / kSkWaves)), block(kSkThreads);
    // (while kv_profile is on, each kernel is launched with a pair of events that take its own start
    // and end times)
    auto launch = [&](auto kernel, const dim3& g, const dim3& b, int which) {
        hipEvent_t e0, e1;
        if (kv_prof_kernel_events(which, &e0, &e1)) hipExtLaunchKernelGGL(kernel, g, b, 0, st, e0, e1, 0, a);
        else hipLaunchKernelGGL(kernel, g, b, 0, st, a);
    };
    if (hpw == 4) {
        if (a.view_ids) launch(decode_wide_kernel<4, true>, grid, block, KV_PROF_DECODE_MAIN);
        else launch(decode_wide_kernel<4, false>, grid, block, KV_PROF_DECODE_MAIN);
    } else if (hpw == 2) {
        if (a.view_ids) launch(decode_wide_kernel<2, true>, grid, block, KV_PROF_DECODE_MAIN);
        else launch(decode_wide_kernel<2, false>, grid, block, KV_PROF_DECODE_MAIN);
    } else if (a.view_ids) {
        launch(decode_streamk_kernel<true>, grid, block, KV_PROF_DECODE_MAIN);
    } else {
        launch(decode_streamk_kernel<false>, grid, block, KV_PROF_DECODE_MAIN);
    }
    int rc = kv_record_hip_error(hipGetLastError(), "paged_decode_attn launch");
    if (rc || a.fused) return rc;
    launch(decode_streamk_merge_kernel,
           dim3((unsigned)view->n_q_local, (unsigned)a.batch, long_lists ? (unsigned)kMergeSplit : 1u), dim3(256),
           KV_PROF_DECODE_MERGE);
    return kv_record_hip_error(hipGetLastError(), "paged_decode_attn merge launch");
}
