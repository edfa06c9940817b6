// Split-K decode attention over resident KV (Sec. II-A: the query's similarity with the keys weights
// the values):  out[b,hq,:] = softmax_j(q[b,hq,:].K[b,h,j,:] / sqrt(D)) V[b,h,j,:],  h = hq / G.
//
// Partial kernel: one workgroup of 8 wavefronts per (sequence, query-head group, token split), about one
// workgroup per compute unit.  A step is a tile of 16 tokens (two tiles when D = 64); the steps of a split
// are handed out to the wavefronts on demand through a counter in LDS, so a wavefront whose loads come back
// late takes fewer steps and all eight reach the merge together (with a fixed round-robin the slowest
// wavefront, and the second workgroup of a compute unit, finished 2-4 us after the median).
//  * q K^T on the matrix cores: one v_mfma_f32_16x16x32 per 32-wide slice of D with the K tile as the
//    16 x 32 A operand (lane = token row, 16 contiguous bytes of it) and the query heads of the group,
//    repeated across the 16 columns, as the B operand.  A 16-byte global load is exactly one operand
//    register set, so K never passes through LDS, and no cross-lane reduction over D is needed.
//  * The 16 x 16 fp32 result leaves lane (column n, row group tg) with the scores of tokens 4tg..4tg+3
//    for query head n mod GT.  Each lane runs the running softmax (m, l) of its own (head, row group)
//    in fp32; probabilities and rescale factors reach the other heads' lanes by quad broadcasts (DPP).
//  * P V stays on the vector ALU: the 16 lanes of a row group hold the V rows of their own 4 tokens
//    (16 bytes per lane), so acc[g][d] += p[g][token] * V[token][d] needs no transpose of V.
//  * K and V are read once and never again: the loads are nontemporal.
// The 32 (wavefront, row group) softmax states of a head are merged through LDS and one fp32 partial per
// (b, hq, split) is written; the combine kernel merges the splits.  HBM-bound (G flop per byte).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <mutex>

#include "plan.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 8;
constexpr int kThreads = 64 * kWaves;
constexpr int kTile = 16;             // tokens per MFMA tile
constexpr int tiles_per_step(int D) { return D >= 128 ? 1 : 2; }  // 8 KiB of K and V in flight per wavefront
constexpr float kEmptyMax = -1.0e30f; // running maximum of a row group that has seen no token
constexpr int kMaxTableSeqs = 64;     // ragged batches up to this size get per-sequence split counts

// Ragged batch: sequence b owns work items [first[b], first[b+1]) of the grid's x dimension, each of
// tokens[b] token rows (the last one shorter).
struct SplitTable {
    int first[kMaxTableSeqs + 1];
    int tokens[kMaxTableSeqs];
};

struct AttnParams {
    const u32x4 *K, *V;    // attention-side buffers of the layer
    const u32x4 *q;        // [B, Hq, D]
    const int *seq_lens;   // device [B]
    int len_uniform;       // >= 0: every sequence has this length (saves the first dependent load); -1: read seq_lens
    float *part_acc;       // [B, Hq, n_splits, D]
    float *part_ml;        // [B, Hq, n_splits, 2]
    long long sb, sh, ss;  // strided layout, in 16-byte vectors
    const long long *seq_off;  // strided layout, optional: element offset of each sequence (replaces b*sb)
    const int *table;      // paged layout
    int max_blocks, bt, bt_shift, n_pool;
    int H, Hq, G, B;
    int use_table;         // 1: blockIdx.x is a work item of the split table; 0: grid (split, head group, sequence)
    int n_splits, split_tokens;
    int max_len;           // host-checked bound on every sequence length
    int one_id;            // paged: every 16-token tile lies inside one block (one table lookup per tile)
    float scale_log2e;     // log2(e) / sqrt(D)
};

template <bool BF16>
__device__ __forceinline__ void unpack8(u32x4 v, float f[8])
{
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned w = v[i];
        if (BF16) {
            f[2 * i] = __uint_as_float(w << 16);
            f[2 * i + 1] = __uint_as_float(w & 0xffff0000u);
        } else {
            const f16x2 h = __builtin_bit_cast(f16x2, w);
            f[2 * i] = (float)h[0];
            f[2 * i + 1] = (float)h[1];
        }
    }
}

template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float rdlane(float x, int l)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, x), l));
}
// Wavefront-wide maximum / sum over all 64 lanes, result uniform: four DPP steps inside each row of 16 lanes
// (vector-ALU speed, no trip through the LDS crossbar), then the four row results through scalar registers.
__device__ __forceinline__ float wave_max(float x)
{
    x = fmaxf(x, dpp_mov<0xB1>(x));   // quad_perm [1,0,3,2]
    x = fmaxf(x, dpp_mov<0x4E>(x));   // quad_perm [2,3,0,1]
    x = fmaxf(x, dpp_mov<0x141>(x));  // row_half_mirror
    x = fmaxf(x, dpp_mov<0x140>(x));  // row_mirror
    return fmaxf(fmaxf(rdlane(x, 0), rdlane(x, 16)), fmaxf(rdlane(x, 32), rdlane(x, 48)));
}
__device__ __forceinline__ float wave_sum(float x)
{
    x += dpp_mov<0xB1>(x);
    x += dpp_mov<0x4E>(x);
    x += dpp_mov<0x141>(x);
    x += dpp_mov<0x140>(x);
    return (rdlane(x, 0) + rdlane(x, 16)) + (rdlane(x, 32) + rdlane(x, 48));
}

// Value of quad lane Q (0..3) in every lane of the quad.
template <int Q>
__device__ __forceinline__ float quad_bcast(float x)
{
    return dpp_mov<Q * 0x55>(x);
}
template <int GT>
__device__ __forceinline__ float head_bcast(float x, int g)
{
    if (GT == 1) return x;
    switch (g) {
    case 0: return quad_bcast<0>(x);
    case 1: return quad_bcast<1>(x);
    case 2: return quad_bcast<2>(x);
    default: return quad_bcast<3>(x);
    }
}

// Merge the running softmax state of another lane into this one.
template <int N>
__device__ __forceinline__ void merge(float &m, float &l, float acc[N], float m2, float l2, const float acc2[N])
{
    const float M = fmaxf(m, m2);
    const float a = exp2f(m - M), b = exp2f(m2 - M);
    l = l * a + l2 * b;
#pragma unroll
    for (int i = 0; i < N; ++i) acc[i] = acc[i] * a + acc2[i] * b;
    m = M;
}

template <bool BF16>
__device__ __forceinline__ f32x4 mfma_16x16x32(u32x4 a, u32x4 b, f32x4 c)
{
    if (BF16)
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Sequence that owns work item `item` of the split table: the last b with first[b] <= item (uniform, scalar).
__device__ __forceinline__ int table_owner(const SplitTable &t, int B, int item)
{
    int lo = 0, hi = B;  // first[lo] <= item < first[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (t.first[mid] <= item) lo = mid; else hi = mid;
    }
    return lo;
}

template <int D, int GT, bool BF16, bool PAGED>
__global__ void __launch_bounds__(kThreads) kv_attn_partial_kernel(AttnParams p, SplitTable tab)
{
    constexpr int NJ = D / 32;               // MFMA slices along D
    constexpr int DV = D / 8;                // 16-byte vectors per row
    constexpr int LPRV = DV < 16 ? DV : 16;  // lanes holding one V row inside a 16-lane row group
    constexpr int TPL = 16 / LPRV;           // V rows one row group covers per load (1, or 2 when D = 64)
    constexpr int NV = DV / LPRV;            // vectors per lane per V row (1, or 2 when D = 256)
    constexpr int NU = 4 / TPL;              // V loads (per vector) for the 4 tokens of a row group
    constexpr int AE = 8 * NV;               // accumulator elements per head per lane
    constexpr int TI = tiles_per_step(D);    // tiles of one step
    constexpr int kStepTok = kTile * TI;

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int split = blockIdx.x, b = blockIdx.z, split_tokens = p.split_tokens;
    if (p.use_table) {
        // Ragged batch: the grid's x dimension counts only splits that hold tokens, sequence after sequence,
        // each sequence cut into its own number of equal splits (sized on the host so that every workgroup
        // gets about the same number of tokens).
        b = table_owner(tab, p.B, (int)blockIdx.x);
        split = (int)blockIdx.x - tab.first[b];
        split_tokens = tab.tokens[b];
    }
    const int hq0 = blockIdx.y * GT;
    const int h = hq0 / p.G;
    const int n = lane & 15;    // MFMA column; also the K row this lane loads
    const int tg = lane >> 4;   // row group: owns tokens 4tg..4tg+3 of a tile; also the D sub-slice of the operands
    const int g_own = n % GT;
    const int lr = n % LPRV, half = n / LPRV;

    const int len = p.len_uniform >= 0 ? p.len_uniform : min(p.seq_lens[b], p.max_len);
    const int t_begin = min(len, split * split_tokens);
    const int t_end = min(len, t_begin + split_tokens);

    // B operand: column n carries query head n mod GT; this lane holds elements 32j + 8tg .. +7 of it.
    u32x4 qv[NJ];
#pragma unroll
    for (int j = 0; j < NJ; ++j) qv[j] = p.q[((long long)b * p.Hq + hq0 + g_own) * DV + 4 * j + tg];

    float m_own = kEmptyMax, l_own = 0.f;
    float acc[GT][AE];
#pragma unroll
    for (int g = 0; g < GT; ++g)
#pragma unroll
        for (int e = 0; e < AE; ++e) acc[g][e] = 0.f;

    const long long head_off = PAGED ? 0 : (p.seq_off ? p.seq_off[b] / 8 : (long long)b * p.sb) + (long long)h * p.sh;
    const int *tbl = PAGED ? p.table + (long long)b * p.max_blocks : nullptr;
    auto block_of = [&](int row) -> int { return p.bt_shift >= 0 ? (row >> p.bt_shift) : (row / p.bt); };
    // vector index of the first element of token row `row` (paged: in pool block blk; ok = false for a block
    // id outside the pool, which then reads block 0 and is masked)
    auto row_base = [&](int row, int blk, bool &ok) -> long long {
        if (PAGED) {
            const int slot = row - block_of(row) * p.bt;
            if ((unsigned)blk >= (unsigned)p.n_pool) { blk = 0; ok = false; }
            return (((long long)blk * p.H + h) * p.bt + slot) * DV;
        }
        return head_off + (long long)row * p.ss;
    };
    // Paged layout: the block ids of one step's rows -- this lane's K row and the 4 tokens of its row group,
    // per tile -- are fetched one step ahead, so that the table lookup is off the load chain.  When the block
    // size is a multiple of the tile a tile lies inside one block, and one lookup per tile serves all five
    // (30.4 instead of 31.2 us at a ragged batch of 8 sequences of 2-8K tokens, 16-token blocks).
    struct Ids { int k[TI]; int t[TI][4]; };
    auto fetch_ids = [&](int Tw, Ids &ids) {
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            const int T0 = Tw + kTile * ti;
            const int fb = T0 < t_end ? T0 : Tw;   // a valid row of this tile's block (of the step's first tile when the tile is empty)
            if (p.one_id) {
                const int id = tbl[block_of(fb)];
                ids.k[ti] = id;
#pragma unroll
                for (int i = 0; i < 4; ++i) ids.t[ti][i] = id;
            } else {
                ids.k[ti] = tbl[block_of((T0 + n < t_end) ? T0 + n : fb)];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int tok = T0 + 4 * tg + i;
                    ids.t[ti][i] = tbl[block_of(tok < t_end ? tok : fb)];
                }
            }
        }
    };

    // Steps are handed out in order, on demand.  A wavefront always knows its current and its next step; the
    // one after that is claimed (one LDS atomic by lane 0) right after the current step's loads are issued,
    // so neither the atomic nor, for the paged layout, the block-table lookup sits on the load chain.
    __shared__ int sh_next;
    const int n_steps = (t_end - t_begin + kStepTok - 1) / kStepTok;
    if (threadIdx.x == 0) sh_next = 2 * kWaves;   // steps 0 .. 2*kWaves-1 are preassigned: w and w + kWaves to wavefront w
    __syncthreads();
    int s_cur = wave, s_nxt = wave + kWaves;
    Ids ids{};
    if (PAGED && s_cur < n_steps) fetch_ids(t_begin + s_cur * kStepTok, ids);

    while (s_cur < n_steps) {
        const int Tw = t_begin + s_cur * kStepTok;
        // ---- loads of the step's tiles: K tile in A-operand order, V rows of this row group's tokens
        u32x4 kvec[TI][NJ];
        u32x4 vvec[TI][NU][NV];
        bool tok_ok[TI][4];
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            const int T0 = Tw + kTile * ti;
            bool k_ok = true;
            const int fb = T0 < t_end ? T0 : Tw;
            const int krow = (T0 + n < t_end) ? T0 + n : fb;  // rows past the end re-read a valid row; masked below
            const long long kb = row_base(krow, PAGED ? ids.k[ti] : 0, k_ok);
#pragma unroll
            for (int j = 0; j < NJ; ++j) kvec[ti][j] = __builtin_nontemporal_load(p.K + kb + 4 * j + tg);
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // a token whose block id is outside the pool is not attended; every lane of the row group
                // sees the same four ids, so they agree on the flag
                tok_ok[ti][i] = (T0 + 4 * tg + i) < t_end;
                if (PAGED) tok_ok[ti][i] = tok_ok[ti][i] && (unsigned)ids.t[ti][i] < (unsigned)p.n_pool;
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const int i = u * TPL + half;
                const int tok = T0 + 4 * tg + i;
                bool ok = true;
                const int blk = !PAGED ? 0 : (TPL == 1 ? ids.t[ti][u] : (half ? ids.t[ti][(2 * u + 1) & 3] : ids.t[ti][(2 * u) & 3]));
                const long long vb = row_base(tok < t_end ? tok : fb, blk, ok);
#pragma unroll
                for (int w = 0; w < NV; ++w) vvec[ti][u][w] = __builtin_nontemporal_load(p.V + vb + lr + w * LPRV);
            }
        }
        int s_new = 0;
        if (lane == 0) s_new = atomicAdd(&sh_next, 1);
        s_new = __builtin_amdgcn_readfirstlane(s_new);
        if (PAGED && s_nxt < n_steps) fetch_ids(t_begin + s_nxt * kStepTok, ids);

#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            // ---- scores of 16 tokens x 16 columns on the matrix core
            f32x4 c = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int j = 0; j < NJ; ++j) c = mfma_16x16x32<BF16>(kvec[ti][j], qv[j], c);

            // ---- running softmax of (head n mod GT, row group tg)
            float s[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) s[i] = tok_ok[ti][i] ? c[i] * p.scale_log2e : -INFINITY;
            const float mn = fmaxf(fmaxf(m_own, fmaxf(s[0], s[1])), fmaxf(s[2], s[3]));
            const float alpha = exp2f(m_own - mn);
            float pr[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) pr[i] = exp2f(s[i] - mn);
            l_own = l_own * alpha + ((pr[0] + pr[1]) + (pr[2] + pr[3]));
            m_own = mn;

            // ---- acc[g] = acc[g] * alpha_g + sum_i p[g][i] * V[i]
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                const float ag = head_bcast<GT>(alpha, g);
#pragma unroll
                for (int e = 0; e < AE; ++e) acc[g][e] *= ag;
            }
#pragma unroll
            for (int u = 0; u < NU; ++u) {
                const float pi = TPL == 1 ? pr[u] : (half ? pr[(2 * u + 1) & 3] : pr[(2 * u) & 3]);
                float vf[NV][8];
#pragma unroll
                for (int w = 0; w < NV; ++w) unpack8<BF16>(vvec[ti][u][w], vf[w]);
#pragma unroll
                for (int g = 0; g < GT; ++g) {
                    const float pg = head_bcast<GT>(pi, g);
#pragma unroll
                    for (int w = 0; w < NV; ++w)
#pragma unroll
                        for (int e = 0; e < 8; ++e) acc[g][w * 8 + e] = fmaf(pg, vf[w][e], acc[g][w * 8 + e]);
                }
            }
        }
        s_cur = s_nxt;
        s_nxt = s_new;
    }

    // ---- merge: every (wavefront, row group) is one softmax state (m, l, acc[D]) per head.  The states go to
    // LDS as they are (when four heads of 256 columns would not fit, row-group pairs are first merged by one
    // shuffle round).  After one barrier a wavefront that forms 64 outputs of head g computes the weights
    // exp2(m - M) of that head's states itself (lane = state, two DPP reductions) and takes them from the lanes
    // by readlane while it sums the weighted states.
    constexpr int SR = GT * D > 512 ? 1 : 0;   // shuffle rounds before LDS
    constexpr int NS = kWaves * (4 >> SR);     // states per head in LDS
    static_assert(NS <= 64, "one lane per state");
    float mg = m_own, lg = l_own;
    if (TPL == 2) {  // the two halves of a row group share (m, l) and hold different tokens of the same d
#pragma unroll
        for (int g = 0; g < GT; ++g)
#pragma unroll
            for (int e = 0; e < AE; ++e) acc[g][e] += __shfl_xor(acc[g][e], 8);
    }
    if (SR == 1) {   // lane (n, tg) and lane (n, tg ^ 1) hold states of the same head n mod GT
        float mh[GT], lh[GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            mh[g] = head_bcast<GT>(m_own, g);
            lh[g] = head_bcast<GT>(l_own, g);
            const float m2 = __shfl_xor(mh[g], 16), l2 = __shfl_xor(lh[g], 16);
            float a2[AE];
#pragma unroll
            for (int e = 0; e < AE; ++e) a2[e] = __shfl_xor(acc[g][e], 16);
            merge<AE>(mh[g], lh[g], acc[g], m2, l2, a2);
        }
        // back to "lane n holds the state of head n mod GT"
        mg = mh[0]; lg = lh[0];
#pragma unroll
        for (int g = 1; g < GT; ++g)
            if (g_own == g) { mg = mh[g]; lg = lh[g]; }
    }

    __shared__ __attribute__((aligned(16))) float sh_acc[NS][GT][D];
    __shared__ f32x2 sh_ml[GT][NS];
    const int state = wave * (4 >> SR) + (tg >> SR);
    if ((tg & ((1 << SR) - 1)) == 0 && half == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int w = 0; w < NV; ++w) {
                // a wavefront's 16-byte stores are contiguous: position ((2w + e4) * LPRV + lr) * 4 + k of a state
                // row holds column d = (lr + w * LPRV) * 8 + 4 * e4 + k
                *(f32x4 *)&sh_acc[state][g][((2 * w) * LPRV + lr) * 4] = f32x4{acc[g][w * 8 + 0], acc[g][w * 8 + 1], acc[g][w * 8 + 2], acc[g][w * 8 + 3]};
                *(f32x4 *)&sh_acc[state][g][((2 * w + 1) * LPRV + lr) * 4] = f32x4{acc[g][w * 8 + 4], acc[g][w * 8 + 5], acc[g][w * 8 + 6], acc[g][w * 8 + 7]};
            }
        }
        if (n < GT) sh_ml[n][state] = f32x2{mg, lg};   // lane n < GT holds the state of head n
    }
    __syncthreads();
    for (int base = wave * 64; base < GT * D; base += kThreads) {   // 64 consecutive positions of one head per wavefront
        const int g = base / D, pos = base - g * D + lane;
        const int d = (((pos >> 2) % LPRV) + ((pos >> 2) / LPRV / 2) * LPRV) * 8 + (((pos >> 2) / LPRV) & 1) * 4 + (pos & 3);
        const f32x2 ml = lane < NS ? sh_ml[g][lane] : f32x2{kEmptyMax, 0.f};
        const float M = wave_max(ml[0]);
        const float wgt = exp2f(ml[0] - M);
        const float L = wave_sum(ml[1] * wgt);
        float A = 0.f;
#pragma unroll
        for (int st = 0; st < NS; ++st) A = fmaf(sh_acc[st][g][pos], rdlane(wgt, st), A);
        const long long o = ((long long)b * p.Hq + hq0 + g) * p.n_splits + split;
        p.part_acc[o * D + d] = A;
        if (pos == 0) *(f32x2 *)&p.part_ml[o * 2] = f32x2{M, L};
    }
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// out_mode: 0 fp32, 1 fp16, 2 bf16.  One workgroup of 256 threads per (hq, b): threads are (column, split group);
// a wavefront covers 64 columns of one split group, so the split index is uniform over the wavefront.  Every
// wavefront forms the split weights exp2(m_s - M) itself (lane = split, two DPP reductions; splits beyond 64 in
// further rounds) and takes them from the lanes by readlane.  The loads of the (m, l) pairs and of a thread's
// first 16 partial rows do not depend on each other and are issued together, so the kernel is one memory
// latency long; the split groups are added through LDS.
constexpr int kCombineThreads = 256;
constexpr int kMaxSplits = 1024;

template <int D>
__global__ void __launch_bounds__(kCombineThreads)
kv_attn_combine_kernel(const float *__restrict__ part_acc, const float *__restrict__ part_ml,
                       void *__restrict__ out, int Hq, int n_splits_alloc, int out_mode,
                       const int *__restrict__ seq_lens, int len_uniform, int max_len, int split_tokens,
                       int use_table, SplitTable tab)
{
    constexpr int CW = D / 64;                       // wavefronts that cover the columns once
    constexpr int NG = (kCombineThreads / 64) / CW;  // split groups (D = 256: 1, 128: 2, 64: 4)
    constexpr int kRows = 16;                        // partial rows a thread loads per round
    const int hq = blockIdx.x, b = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int grp = __builtin_amdgcn_readfirstlane(wave / CW), d = (wave % CW) * 64 + lane;
    const long long o = ((long long)b * Hq + hq) * n_splits_alloc;
    // only the splits that hold tokens of this sequence were written (and matter)
    int n_splits;
    if (use_table) {
        n_splits = tab.first[b + 1] - tab.first[b];
    } else {
        const int len = len_uniform >= 0 ? len_uniform : min(seq_lens[b], max_len);
        n_splits = min(n_splits_alloc, (len + split_tokens - 1) / split_tokens);
    }

    f32x2 ml0 = f32x2{kEmptyMax, 0.f};
    if (lane < n_splits) ml0 = *(const f32x2 *)&part_ml[(o + lane) * 2];
    float pre[kRows];
#pragma unroll
    for (int i = 0; i < kRows; ++i) {                // first round's rows: independent of the weights
        const int s = grp + i * NG;
        pre[i] = s < n_splits ? part_acc[(o + s) * D + d] : 0.f;
    }
    // global maximum over all splits (the pairs just loaded; a tail loop when there are more than 64)
    float M = ml0[0];
    for (int s = 64 + lane; s < n_splits; s += 64) M = fmaxf(M, part_ml[(o + s) * 2]);
    M = wave_max(M);

    float A = 0.f, L = 0.f;
    for (int s0 = 0; s0 < n_splits; s0 += 64) {      // rounds of 64 splits: lane = split
        f32x2 ml = ml0;
        if (s0 > 0) {
            ml = f32x2{kEmptyMax, 0.f};
            if (s0 + lane < n_splits) ml = *(const f32x2 *)&part_ml[(o + s0 + lane) * 2];
        }
        const float wgt = exp2f(ml[0] - M);
        L = fmaf(ml[1], wgt, L);
        for (int r0 = 0; r0 < 64 && s0 + r0 < n_splits; r0 += kRows * NG) {
#pragma unroll
            for (int i = 0; i < kRows; ++i) {
                const int sl = r0 + grp + i * NG;     // uniform over the wavefront
                const int s = s0 + sl;
                if (sl < 64 && s < n_splits) {
                    const float v = (s0 == 0 && r0 == 0) ? pre[i] : part_acc[(o + s) * D + d];
                    A = fmaf(v, rdlane(wgt, sl), A);
                }
            }
        }
    }
    L = wave_sum(L);

    __shared__ float colsum[NG][D];
    if (NG > 1) {
        colsum[grp][d] = A;
        __syncthreads();
        if (grp == 0) {
#pragma unroll
            for (int k = 1; k < NG; ++k) A += colsum[k][d];
        }
    }
    if (grp == 0) {
        const float r = L > 0.f ? A / L : 0.f;
        const long long oi = ((long long)b * Hq + hq) * D + d;
        if (out_mode == 0) ((float *)out)[oi] = r;
        else if (out_mode == 1) ((_Float16 *)out)[oi] = (_Float16)r;  // round to nearest even
        else ((unsigned short *)out)[oi] = f32_to_bf16_rne(r);
    }
}

int pick_gt(int G) { return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1); }

// Tokens per split are a multiple of this: half a round of the workgroup's wavefronts.
int split_quantum(int D) { return kWaves / 2 * kTile * tiles_per_step(D); }

// Most splits the automatic choice can make for sequences of up to max_len tokens (sizes the workspace).
int max_auto_splits(const kv_plan *p, int max_len)
{
    const int q = split_quantum(p->D);
    return (int)std::min<long long>(kMaxSplits, std::max<long long>(1, ((long long)max_len + q - 1) / q));
}

// Workgroups the automatic split choice aims at: one per compute unit (a workgroup is eight wavefronts; with
// one per compute unit every one of them starts at once and none waits for a second round).
int target_workgroups()
{
    static int cus = 0;
    if (cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) == hipSuccess && hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && n > 0)
            cus = n;
        else
            cus = 256;
    }
    return cus;
}

// Uniform batch: split length from the total token count, so that about one workgroup per compute unit has
// tokens to read; never shorter than the quantum.
int choose_splits(const kv_plan *p, long long total_tokens, int max_len)
{
    if (max_len <= 0) return 1;
    const int q = split_quantum(p->D);
    const long long groups_per_seq = p->Hq / pick_gt(p->Hq / p->H);
    const long long wgs = target_workgroups();
    long long st = (total_tokens * groups_per_seq + wgs - 1) / wgs;
    st = std::max<long long>(q, (st + q - 1) / q * q);
    const long long ns = ((long long)max_len + st - 1) / st;
    return (int)std::min<long long>(std::max<long long>(1, ns), max_auto_splits(p, max_len));
}

int split_tokens_for(const kv_plan *p, int n_splits, int max_len)
{
    const int q = split_quantum(p->D);
    long long st = ((long long)max_len + n_splits - 1) / n_splits;
    st = (st + q - 1) / q * q;
    return (int)std::max<long long>(st, q);
}

// Ragged batch of up to kMaxTableSeqs sequences: every sequence with tokens gets one split; the remaining
// workgroups of the budget (one per compute unit, shared by the query-head groups) go, one at a time, to the
// sequence whose splits are longest; no sequence gets more than cap splits or splits shorter than the quantum.
// A sequence's split length is then rounded up to whole steps only, not to the quantum: steps are handed out
// on demand, so nothing is gained by a whole number of rounds, and the longest split gets shorter.
// Returns the largest split count.
int apportion_splits(const kv_plan *p, const int32_t *lens, int cap, SplitTable *t)
{
    const int q = split_quantum(p->D);
    const long long groups_per_seq = p->Hq / pick_gt(p->Hq / p->H);
    int nb[kMaxTableSeqs];
    long long used = 0;
    for (int b = 0; b < p->B; ++b) { nb[b] = lens[b] > 0 ? 1 : 0; used += nb[b]; }
    const long long budget = std::max<long long>(used, target_workgroups() / groups_per_seq);
    while (used < budget) {
        int best = -1;
        double longest = 0.0;
        for (int b = 0; b < p->B; ++b) {
            if (nb[b] == 0 || nb[b] >= cap || (long long)(nb[b] + 1) * q > (long long)lens[b] + q - 1) continue;
            const double cur = (double)lens[b] / nb[b];
            if (cur > longest) { longest = cur; best = b; }
        }
        if (best < 0) break;
        ++nb[best];
        ++used;
    }
    const int step = kTile * tiles_per_step(p->D);
    int most = 1, first = 0;
    for (int b = 0; b < p->B; ++b) {
        t->first[b] = first;
        int st = q;
        if (nb[b] > 0) {
            st = std::max(q, (int)((((long long)lens[b] + nb[b] - 1) / nb[b] + step - 1) / step * step));
            nb[b] = (lens[b] + st - 1) / st;   // rounding the split length up may leave fewer splits
        }
        t->tokens[b] = st;
        first += nb[b];
        most = std::max(most, nb[b]);
    }
    for (int b = p->B; b <= kMaxTableSeqs; ++b) t->first[b] = first;
    return most;
}

template <int D, int GT>
void launch_partial(bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a, const SplitTable &t)
{
    if (bf16) {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, true, true>), grid, dim3(kThreads), 0, st, a, t);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, true, false>), grid, dim3(kThreads), 0, st, a, t);
    } else {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, false, true>), grid, dim3(kThreads), 0, st, a, t);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, false, false>), grid, dim3(kThreads), 0, st, a, t);
    }
}

template <int D>
void launch_partial_gt(int gt, bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a, const SplitTable &t)
{
    if (gt == 4) launch_partial<D, 4>(bf16, paged, grid, st, a, t);
    else if (gt == 2) launch_partial<D, 2>(bf16, paged, grid, st, a, t);
    else launch_partial<D, 1>(bf16, paged, grid, st, a, t);
}

}  // namespace

extern "C" size_t kv_decode_attn_workspace(const kv_plan_t *p, int n_splits, int max_len)
{
    if (!p || n_splits < 0 || max_len < 0) return 0;
    const int ns = n_splits > 0 ? n_splits : max_auto_splits(p, max_len);
    return (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
}

namespace {

// Split choice for the given lengths: fills the table (ragged batches of up to kMaxTableSeqs sequences) or the
// common split length; returns the split count the partials are laid out for.
int plan_splits(const kv_plan *p, const int32_t *lens, int n_splits, bool *use_table, SplitTable *tab, int *split_tokens)
{
    int max_len = 0;
    long long total_len = 0;
    bool uniform = true;
    for (int b = 0; b < p->B; ++b) {
        max_len = std::max(max_len, lens[b]);
        total_len += lens[b];
        if (lens[b] != lens[0]) uniform = false;
    }
    *use_table = !uniform && p->B <= kMaxTableSeqs;
    if (*use_table && n_splits == 0) {
        *split_tokens = split_quantum(p->D);  // not used by the kernels in table mode
        return apportion_splits(p, lens, max_auto_splits(p, max_len), tab);
    }
    const int ns = n_splits > 0 ? n_splits : choose_splits(p, total_len, max_len);
    *split_tokens = split_tokens_for(p, ns, max_len);
    if (*use_table) {
        int first = 0;
        for (int b = 0; b < p->B; ++b) {
            tab->first[b] = first;
            tab->tokens[b] = *split_tokens;
            first += (lens[b] + *split_tokens - 1) / *split_tokens;
        }
        for (int b = p->B; b <= kMaxTableSeqs; ++b) tab->first[b] = first;
    }
    return ns;
}

// Checks, split choice and the two launches; shared by both entry points.  Allocates nothing.
int decode_attn(const kv_plan_t *p, const kv_view_t *kv, int layer, const void *q, void *out, int out_dtype,
                int n_splits, void *workspace, size_t ws_bytes, void *hip_stream)
{
    if (!p || !kv || !q || !out || !workspace) return KV_EINVAL;
    if (out_dtype != KV_OUT_F32 && out_dtype != KV_OUT_SAME) return KV_EINVAL;
    if (n_splits < 0 || n_splits > kMaxSplits) return KV_EINVAL;
    if (p->D != 64 && p->D != 128 && p->D != 256) return KV_EINVAL;
    if (!kv->k_layers || !kv->v_layers || !kv->seq_lens_host || !kv->seq_lens_dev) return KV_EINVAL;
    if (layer < 0 || layer >= p->L || layer >= kv->n_layers) return KV_ERANGE;
    const void *K = kv->k_layers[layer], *V = kv->v_layers[layer];
    if (!K || !V) return KV_EINVAL;
    if (((uintptr_t)K | (uintptr_t)V | (uintptr_t)q | (uintptr_t)workspace) & 15) return KV_EINVAL;
    if (p->B > 65535 || p->Hq > 65535) return KV_EINVAL;

    int max_len = 0;
    for (int b = 0; b < p->B; ++b) {
        const int len = kv->seq_lens_host[b];
        if (len < 0) return KV_EINVAL;
        max_len = std::max(max_len, len);
    }
    AttnParams a{};
    const bool paged = kv->layout == KV_LAYOUT_PAGED;
    if (kv->layout == KV_LAYOUT_BHSD) {
        if (kv->stride_b < 0 || kv->stride_h < 0 || kv->stride_s < p->D) return KV_EINVAL;
        if ((kv->stride_b | kv->stride_h | kv->stride_s) & 7) return KV_EINVAL;
        if (max_len > kv->s_alloc) return KV_ERANGE;
        if ((kv->seq_off_host == nullptr) != (kv->seq_off_dev == nullptr)) return KV_EINVAL;
        for (int b = 0; b < p->B; ++b) {  // the last element any sequence reads must lie inside the buffer
            const int len = kv->seq_lens_host[b];
            if (len == 0) continue;
            if (kv->seq_off_host && (kv->seq_off_host[b] < 0 || (kv->seq_off_host[b] & 7))) return KV_EINVAL;
            const uint64_t base = kv->seq_off_host ? (uint64_t)kv->seq_off_host[b] : (uint64_t)b * kv->stride_b;
            const uint64_t max_elem = base + (uint64_t)(p->H - 1) * kv->stride_h + (uint64_t)(len - 1) * kv->stride_s + p->D;
            if (max_elem * 2 > kv->layer_bytes) return KV_ERANGE;
        }
        a.sb = kv->stride_b / 8; a.sh = kv->stride_h / 8; a.ss = kv->stride_s / 8;
        a.seq_off = (const long long *)kv->seq_off_dev;
    } else if (paged) {
        if (!kv->block_table || kv->block_tokens < 1 || kv->n_pool_blocks < 0) return KV_EINVAL;
        if ((uint64_t)kv->n_pool_blocks * p->H * kv->block_tokens * p->D * 2 > kv->layer_bytes) return KV_ERANGE;
        if (kvb::ceil_div((uint64_t)max_len, (uint64_t)kv->block_tokens) > (uint64_t)kv->max_blocks_per_seq)
            return KV_ERANGE;
        if (max_len > 0 && kv->n_pool_blocks < 1) return KV_ERANGE;
        a.table = kv->block_table;
        a.max_blocks = kv->max_blocks_per_seq;
        a.bt = kv->block_tokens;
        a.bt_shift = (a.bt & (a.bt - 1)) == 0 ? __builtin_ctz((unsigned)a.bt) : -1;
        a.n_pool = kv->n_pool_blocks;
        a.one_id = a.bt % kTile == 0;   // split starts are multiples of the quantum, itself a multiple of the tile
    } else {
        return KV_EINVAL;
    }

    a.len_uniform = max_len;
    for (int b = 0; b < p->B; ++b)
        if (kv->seq_lens_host[b] != max_len) a.len_uniform = -1;

    // Splits.  A uniform batch (or a split count given by the caller) takes one split length for all sequences
    // and the grid (split, query-head group, sequence).  A ragged batch of up to 64 sequences launches
    // workgroups only for splits that hold tokens: the x dimension of its grid walks a table of per-sequence
    // split counts, and with the automatic choice each sequence's split length is sized so that every
    // workgroup reads about the same number of tokens.
    SplitTable tab{};
    bool use_table = false;
    const int ns = plan_splits(p, kv->seq_lens_host, n_splits, &use_table, &tab, &a.split_tokens);
    a.use_table = use_table;
    const size_t need = (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
    if (ws_bytes < need) return KV_ENOSPC;

    const int G = p->Hq / p->H, gt = pick_gt(G);
    a.K = (const u32x4 *)K; a.V = (const u32x4 *)V; a.q = (const u32x4 *)q;
    a.seq_lens = kv->seq_lens_dev;
    a.part_acc = (float *)workspace;
    a.part_ml = a.part_acc + (size_t)p->B * p->Hq * ns * p->D;
    a.H = p->H; a.Hq = p->Hq; a.G = G; a.B = p->B;
    a.n_splits = ns;
    a.max_len = max_len;
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)p->D));

    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf16 = p->dtype == KV_BF16;
    const long long n_items = a.use_table ? tab.first[p->B] : (max_len > 0 ? (long long)ns * p->B : 0);
    dim3 grid((unsigned)ns, (unsigned)(p->Hq / gt), (unsigned)p->B);
    if (a.use_table) grid = dim3((unsigned)n_items, (unsigned)(p->Hq / gt), 1u);
    if (n_items > 0) {
        if (p->D == 64) launch_partial_gt<64>(gt, bf16, paged, grid, st, a, tab);
        else if (p->D == 128) launch_partial_gt<128>(gt, bf16, paged, grid, st, a, tab);
        else launch_partial_gt<256>(gt, bf16, paged, grid, st, a, tab);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    }

    const int out_mode = out_dtype == KV_OUT_F32 ? 0 : (bf16 ? 2 : 1);
    const dim3 cgrid((unsigned)p->Hq, (unsigned)p->B, 1u);
#define KV_COMBINE(DD)                                                                                                   \
    hipLaunchKernelGGL((kv_attn_combine_kernel<DD>), cgrid, dim3(kCombineThreads), 0, st, a.part_acc, a.part_ml, out,   \
                       p->Hq, ns, out_mode, a.seq_lens, a.len_uniform, max_len, a.split_tokens, a.use_table, tab)
    if (p->D == 64) KV_COMBINE(64);
    else if (p->D == 128) KV_COMBINE(128);
    else KV_COMBINE(256);
#undef KV_COMBINE
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    return KV_OK;
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];  // device address of `scratch` on each GPU, resolved on the first call there

}  // namespace

// Split partials of kv_decode_attn_static: every GPU the library runs on holds its own copy of this array
// until the process ends.  In host code the name is only a handle for hipGetSymbolAddress.
static __device__ __align__(256) unsigned char scratch[KV_ATTN_SCRATCH_BYTES];

extern "C" int kv_decode_attn_splits(const kv_plan_t *p, const int32_t *seq_lens_host, int n_splits, int *n_splits_out,
                                     int *first, int *tokens)
{
    if (!p || !seq_lens_host || !n_splits_out) return KV_EINVAL;
    if (n_splits < 0 || n_splits > kMaxSplits) return KV_EINVAL;
    if (p->D != 64 && p->D != 128 && p->D != 256) return KV_EINVAL;
    for (int b = 0; b < p->B; ++b)
        if (seq_lens_host[b] < 0) return KV_EINVAL;
    SplitTable tab{};
    bool use_table = false;
    int st = 0;
    *n_splits_out = plan_splits(p, seq_lens_host, n_splits, &use_table, &tab, &st);
    int acc = 0;
    for (int b = 0; b < p->B; ++b) {
        if (first) first[b] = acc;
        if (tokens) tokens[b] = use_table ? tab.tokens[b] : st;
        acc += use_table ? tab.first[b + 1] - tab.first[b] : std::min(*n_splits_out, (seq_lens_host[b] + st - 1) / st);
    }
    if (first) first[p->B] = acc;
    return KV_OK;
}

extern "C" int kv_decode_attn(const kv_plan_t *p, const kv_view_t *kv, int layer, const void *q, void *out,
                              int out_dtype, int n_splits, void *workspace, size_t ws_bytes, void *hip_stream)
{
    return decode_attn(p, kv, layer, q, out, out_dtype, n_splits, workspace, ws_bytes, hip_stream);
}

extern "C" int kv_decode_attn_static(const kv_plan_t *p, const kv_view_t *kv, int layer, const void *q, void *out,
                                     int out_dtype, int n_splits, void *hip_stream)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    if (dev < 0 || dev >= kMaxDevices) return KV_EINVAL;
    void *ws = nullptr;
    {
        std::lock_guard<std::mutex> g(g_scratch_mu);
        if (!g_scratch_ptr[dev]) {
            // the array's name is a host-side stand-in; its device address on the current GPU is looked up once
            void *ptr = nullptr;
            e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
            if (e != hipSuccess || !ptr) { kvb::set_hip_error((int)e); return KV_EHIP; }
            g_scratch_ptr[dev] = ptr;
        }
        ws = g_scratch_ptr[dev];
    }
    // decode_attn answers KV_ENOSPC when the partials of this call do not fit the array
    return decode_attn(p, kv, layer, q, out, out_dtype, n_splits, ws, (size_t)KV_ATTN_SCRATCH_BYTES, hip_stream);
}
