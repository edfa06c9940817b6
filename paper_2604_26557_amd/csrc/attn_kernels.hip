// Split-K decode attention over resident KV (Sec. II-A: the query's similarity with the keys weights
// the values):  out[b,hq,:] = softmax_j(q[b,hq,:].K[b,h,j,:] / sqrt(D)) V[b,h,j,:],  h = hq / G.
//
// Partial kernel, grid (split, query-head group, b), 4 wavefronts per workgroup, each walking 16-token
// tiles of its split.
//  * q K^T on the matrix cores: one v_mfma_f32_16x16x32 per 32-wide slice of D with the K tile as the
//    16 x 32 A operand (lane = token row, 16 contiguous bytes of it) and the query heads of the group,
//    repeated across the 16 columns, as the B operand.  A 16-byte global load is exactly one operand
//    register set, so K never passes through LDS, and no cross-lane reduction over D is needed.
//  * The 16 x 16 fp32 result leaves lane (column n, row group tg) with the scores of tokens 4tg..4tg+3
//    for query head n mod GT.  Each lane runs the running softmax (m, l) of its own (head, row group)
//    in fp32; probabilities and rescale factors reach the other heads' lanes by quad broadcasts (DPP).
//  * P V stays on the vector ALU: the 16 lanes of a row group hold the V rows of their own 4 tokens
//    (16 bytes per lane), so acc[g][d] += p[g][token] * V[token][d] needs no transpose of V.
// Row groups, then wavefronts, are merged at the end and one fp32 partial per (b, hq, split) is
// written; the combine kernel merges the splits.  HBM-bound (G flop per byte).
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

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kTile = 16;             // tokens per MFMA tile
constexpr int tiles_per_iter(int D) { return D >= 256 ? 1 : (D == 128 ? 2 : 4); }
constexpr float kEmptyMax = -1.0e30f; // running maximum of a row group that has seen no token

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
    int compact;           // 1: blockIdx.x counts only the splits that hold tokens, sequence after sequence
    int n_splits, split_tokens;
    int max_len;           // host-checked bound on every sequence length
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

// Value of quad lane Q (0..3) in every lane of the quad.
template <int Q>
__device__ __forceinline__ float quad_bcast(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), Q * 0x55, 0xf, 0xf, false));
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

// Merge the running softmax state of another lane / wavefront into this one.
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

template <int D, int GT, bool BF16, bool PAGED>
__global__ void __launch_bounds__(kThreads) kv_attn_partial_kernel(AttnParams p)
{
    constexpr int NJ = D / 32;               // MFMA slices along D
    constexpr int DV = D / 8;                // 16-byte vectors per row
    constexpr int LPRV = DV < 16 ? DV : 16;  // lanes holding one V row inside a 16-lane row group
    constexpr int TPL = 16 / LPRV;           // V rows one row group covers per load (1, or 2 when D = 64)
    constexpr int NV = DV / LPRV;            // vectors per lane per V row (1, or 2 when D = 256)
    constexpr int NU = 4 / TPL;              // V loads (per vector) for the 4 tokens of a row group
    constexpr int AE = 8 * NV;               // accumulator elements per head per lane
    constexpr int TI = tiles_per_iter(D);    // tiles whose loads are issued together (16 KiB in flight per wavefront)

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int split = blockIdx.x, b = blockIdx.z;
    if (p.compact) {
        // Ragged batch (B <= 64): no workgroup is launched for a split without tokens.  Lane s holds the split
        // count of sequence s; an inclusive scan over the wavefront and a ballot find the sequence that owns
        // work item blockIdx.x (every wavefront does the same).
        int nb = 0;
        if (lane < p.B) nb = (min(p.seq_lens[lane], p.max_len) + p.split_tokens - 1) / p.split_tokens;
        int incl = nb;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const int up = __shfl_up(incl, off);
            if (lane >= off) incl += up;
        }
        const unsigned long long owners = __ballot((int)blockIdx.x < incl);
        if (owners == 0) return;  // not reached: the grid has exactly the sum of the split counts
        b = __ffsll((long long)owners) - 1;
        split = (int)blockIdx.x - __shfl(incl - nb, b);
    }
    const int hq0 = blockIdx.y * GT;
    const int h = hq0 / p.G;
    const int n = lane & 15;    // MFMA column; also the K row this lane loads
    const int tg = lane >> 4;   // row group: owns tokens 4tg..4tg+3 of a tile; also the D sub-slice of the operands
    const int g_own = n % GT;
    const int lr = n % LPRV, half = n / LPRV;

    const int len = p.len_uniform >= 0 ? p.len_uniform : min(p.seq_lens[b], p.max_len);
    const int t_begin = min(len, split * p.split_tokens);
    const int t_end = min(len, t_begin + p.split_tokens);

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
    // Paged layout: the block ids of one iteration's rows -- this lane's K row and the 4 tokens of its row
    // group, per tile -- are fetched one iteration ahead, so that the table lookup is off the load chain.
    struct Ids { int k[TI]; int t[TI][4]; };
    auto fetch_ids = [&](int Tw, Ids &ids) {
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            const int T0 = Tw + kTile * ti;
            ids.k[ti] = tbl[block_of((T0 + n < t_end) ? T0 + n : t_begin)];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int tok = T0 + 4 * tg + i;
                ids.t[ti][i] = tbl[block_of(tok < t_end ? tok : t_begin)];
            }
        }
    };
    Ids ids{};
    const int Tw0 = t_begin + kTile * TI * wave;
    if (PAGED && Tw0 < t_end) fetch_ids(Tw0, ids);

    for (int Tw = Tw0; Tw < t_end; Tw += kTile * TI * kWaves) {
        // ---- loads of TI adjacent tiles: K tile in A-operand order, V rows of this row group's tokens
        u32x4 kvec[TI][NJ];
        u32x4 vvec[TI][NU][NV];
        bool tok_ok[TI][4];
#pragma unroll
        for (int ti = 0; ti < TI; ++ti) {
            const int T0 = Tw + kTile * ti;
            bool k_ok = true;
            const int krow = (T0 + n < t_end) ? T0 + n : t_begin;  // rows past the end re-read a valid row; masked below
            const long long kb = row_base(krow, PAGED ? ids.k[ti] : 0, k_ok);
#pragma unroll
            for (int j = 0; j < NJ; ++j) kvec[ti][j] = p.K[kb + 4 * j + tg];
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
                const long long vb = row_base(tok < t_end ? tok : t_begin, blk, ok);
#pragma unroll
                for (int w = 0; w < NV; ++w) vvec[ti][u][w] = p.V[vb + lr + w * LPRV];
            }
        }
        if (PAGED) {
            const int next = Tw + kTile * TI * kWaves;
            if (next < t_end) fetch_ids(next, ids);
        }

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
    }

    // ---- merge: every (wavefront, row group) is one softmax state (m, l, acc[D]) per head.  The states go
    // to LDS as they are (for D = 256 row-group pairs are first merged by one shuffle round, to halve the
    // LDS footprint), their weights exp2(m - M) are computed once per (state, head), and the workgroup then
    // forms the weighted sums: far fewer instructions than merging in registers through shuffles.
    constexpr int SR = D == 256 ? 1 : 0;       // shuffle rounds before LDS
    constexpr int NS = kWaves * (4 >> SR);     // states per head in LDS
    float mg[GT], lg[GT];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        mg[g] = head_bcast<GT>(m_own, g);
        lg[g] = head_bcast<GT>(l_own, g);
    }
    if (TPL == 2) {  // the two halves of a row group share (m, l) and hold different tokens of the same d
#pragma unroll
        for (int g = 0; g < GT; ++g)
#pragma unroll
            for (int e = 0; e < AE; ++e) acc[g][e] += __shfl_xor(acc[g][e], 8);
    }
#pragma unroll
    for (int r = 0; r < SR; ++r) {
        const int off = 16 << r;
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const float m2 = __shfl_xor(mg[g], off), l2 = __shfl_xor(lg[g], off);
            float a2[AE];
#pragma unroll
            for (int e = 0; e < AE; ++e) a2[e] = __shfl_xor(acc[g][e], off);
            merge<AE>(mg[g], lg[g], acc[g], m2, l2, a2);
        }
    }

    __shared__ __attribute__((aligned(16))) float sh_acc[NS][GT][D];
    __shared__ float sh_ml[NS][GT][2];
    __shared__ float sh_w[NS][GT];
    __shared__ float sh_ML[GT][2];
    const int state = wave * (4 >> SR) + (tg >> SR);
    if ((tg & ((1 << SR) - 1)) == 0 && half == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int w = 0; w < NV; ++w) {
                float *dst = &sh_acc[state][g][(lr + w * LPRV) * 8];
                *(f32x4 *)dst = f32x4{acc[g][w * 8 + 0], acc[g][w * 8 + 1], acc[g][w * 8 + 2], acc[g][w * 8 + 3]};
                *(f32x4 *)(dst + 4) = f32x4{acc[g][w * 8 + 4], acc[g][w * 8 + 5], acc[g][w * 8 + 6], acc[g][w * 8 + 7]};
            }
            if (n == 0) { sh_ml[state][g][0] = mg[g]; sh_ml[state][g][1] = lg[g]; }
        }
    }
    __syncthreads();
    if (threadIdx.x < GT) {  // one thread per head: maximum, weights, denominator
        const int g = threadIdx.x;
        float M = sh_ml[0][g][0];
#pragma unroll
        for (int st = 1; st < NS; ++st) M = fmaxf(M, sh_ml[st][g][0]);
        float L = 0.f;
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            const float a = exp2f(sh_ml[st][g][0] - M);
            sh_w[st][g] = a;
            L += sh_ml[st][g][1] * a;
        }
        sh_ML[g][0] = M;
        sh_ML[g][1] = L;
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < GT * D; idx += kThreads) {
        const int g = idx / D, d = idx - g * D;
        float A = 0.f;
#pragma unroll
        for (int st = 0; st < NS; ++st) A = fmaf(sh_acc[st][g][d], sh_w[st][g], A);
        const long long o = ((long long)b * p.Hq + hq0 + g) * p.n_splits + split;
        p.part_acc[o * D + d] = A;
        if (d == 0) { p.part_ml[o * 2] = sh_ML[g][0]; p.part_ml[o * 2 + 1] = sh_ML[g][1]; }
    }
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// out_mode: 0 fp32, 1 fp16, 2 bf16.  One workgroup of 256 threads per (hq, b, 32 output columns): threads are
// (column, split group), eight groups, group k summing splits k, k+8, ...  The loads of a thread's first
// kCombinePrefetch partial rows do not depend on the split weights, so they are issued first and the two
// memory latencies (weights' inputs, partial rows) overlap.  The weights exp2(m_s - M) go to LDS.
constexpr int kCombineThreads = 256;
constexpr int kCombineCols = 32;
constexpr int kCombineGroups = kCombineThreads / kCombineCols;
constexpr int kCombinePrefetch = 8;
constexpr int kMaxSplits = 1024;

__global__ void __launch_bounds__(kCombineThreads)
kv_attn_combine_kernel(const float *__restrict__ part_acc, const float *__restrict__ part_ml,
                       void *__restrict__ out, int Hq, int D, int n_splits_alloc, int out_mode,
                       const int *__restrict__ seq_lens, int len_uniform, int max_len, int split_tokens)
{
    __shared__ float w[kMaxSplits];
    __shared__ float colsum[kCombineThreads / 64][kCombineCols];
    const int hq = blockIdx.x, b = blockIdx.y, d = blockIdx.z * kCombineCols + (threadIdx.x & (kCombineCols - 1));
    const int tid = threadIdx.x, lane = tid & 63, grp = tid / kCombineCols;
    const long long o = ((long long)b * Hq + hq) * n_splits_alloc;
    // only the splits that hold tokens of this sequence were written (and matter)
    const int len = len_uniform >= 0 ? len_uniform : min(seq_lens[b], max_len);
    const int n_splits = min(n_splits_alloc, (len + split_tokens - 1) / split_tokens);

    float pre[kCombinePrefetch];
#pragma unroll
    for (int i = 0; i < kCombinePrefetch; ++i) {
        const int s = grp + i * kCombineGroups;
        pre[i] = s < n_splits ? part_acc[(o + s) * D + d] : 0.f;
    }

    // Wavefront 0 alone forms the maximum, the weights and the denominator: one load of its lanes' (m, l)
    // pairs (two per lane cover 128 splits; a rare tail loop takes the rest), two shuffle reductions.
    float L = 0.f;
    if (tid < 64) {
        float m2[2], l2[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int s = lane + 64 * i;
            m2[i] = kEmptyMax;
            l2[i] = 0.f;
            if (s < n_splits) {
                const f32x2 v = *(const f32x2 *)&part_ml[(o + s) * 2];
                m2[i] = v[0];
                l2[i] = v[1];
            }
        }
        float mx = fmaxf(m2[0], m2[1]);
        for (int s = lane + 128; s < n_splits; s += 64) mx = fmaxf(mx, part_ml[(o + s) * 2]);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
        const float M = mx;
        float lsum = 0.f;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int s = lane + 64 * i;
            const float a = exp2f(m2[i] - M);
            if (s < n_splits) w[s] = a;
            lsum += l2[i] * a;
        }
        for (int s = lane + 128; s < n_splits; s += 64) {
            const float a = exp2f(part_ml[(o + s) * 2] - M);
            w[s] = a;
            lsum += part_ml[(o + s) * 2 + 1] * a;
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off);
        L = lsum;
    }
    __syncthreads();

    float A = 0.f;
#pragma unroll
    for (int i = 0; i < kCombinePrefetch; ++i) {
        const int s = grp + i * kCombineGroups;
        if (s < n_splits) A = fmaf(pre[i], w[s], A);
    }
#pragma unroll 4
    for (int s = grp + kCombinePrefetch * kCombineGroups; s < n_splits; s += kCombineGroups)
        A = fmaf(part_acc[(o + s) * D + d], w[s], A);
    A += __shfl_xor(A, 32);  // the two split groups of a wavefront
    if (lane < kCombineCols) colsum[tid >> 6][lane] = A;
    __syncthreads();
    if (tid < kCombineCols) {
#pragma unroll
        for (int k = 1; k < kCombineThreads / 64; ++k) A += colsum[k][tid];
        const float r = L > 0.f ? A / L : 0.f;
        const long long oi = ((long long)b * Hq + hq) * D + d;
        if (out_mode == 0) ((float *)out)[oi] = r;
        else if (out_mode == 1) ((_Float16 *)out)[oi] = (_Float16)r;  // round to nearest even
        else ((unsigned short *)out)[oi] = f32_to_bf16_rne(r);
    }
}

int pick_gt(int G) { return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1); }

// Tokens per split: a multiple of the rows one workgroup iteration covers.
int split_quantum(int D) { return kWaves * kTile * tiles_per_iter(D); }

// Most splits the automatic choice can make for sequences of up to max_len tokens (sizes the workspace).
int max_auto_splits(const kv_plan *p, int max_len)
{
    const int q = split_quantum(p->D);
    return (int)std::min<long long>(kMaxSplits, std::max<long long>(1, ((long long)max_len + q - 1) / q));
}

// Split length from the total token count, so that about 512 workgroups (two per compute unit; the
// measured best at the 4K, 8K and 32K shapes) have tokens to read even when the batch is ragged;
// never shorter than one workgroup iteration.
int choose_splits(const kv_plan *p, long long total_tokens, int max_len)
{
    if (max_len <= 0) return 1;
    const int q = split_quantum(p->D);
    const long long groups_per_seq = p->Hq / pick_gt(p->Hq / p->H);
    long long st = (total_tokens * groups_per_seq + 511) / 512;
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

template <int D, int GT>
void launch_partial(bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a)
{
    if (bf16) {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, true, true>), grid, dim3(kThreads), 0, st, a);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, true, false>), grid, dim3(kThreads), 0, st, a);
    } else {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, false, true>), grid, dim3(kThreads), 0, st, a);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<D, GT, false, false>), grid, dim3(kThreads), 0, st, a);
    }
}

template <int D>
void launch_partial_gt(int gt, bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a)
{
    if (gt == 4) launch_partial<D, 4>(bf16, paged, grid, st, a);
    else if (gt == 2) launch_partial<D, 2>(bf16, paged, grid, st, a);
    else launch_partial<D, 1>(bf16, paged, grid, st, a);
}

}  // namespace

extern "C" size_t kv_decode_attn_workspace(const kv_plan_t *p, int n_splits, int max_len)
{
    if (!p || n_splits < 0 || max_len < 0) return 0;
    const int ns = n_splits > 0 ? n_splits : max_auto_splits(p, max_len);
    return (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
}

namespace {

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
    long long total_len = 0;
    for (int b = 0; b < p->B; ++b) {
        const int len = kv->seq_lens_host[b];
        if (len < 0) return KV_EINVAL;
        max_len = std::max(max_len, len);
        total_len += len;
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
    } else {
        return KV_EINVAL;
    }

    const int ns = n_splits > 0 ? n_splits : choose_splits(p, total_len, max_len);
    const size_t need = (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
    if (ws_bytes < need) return KV_ENOSPC;

    const int G = p->Hq / p->H, gt = pick_gt(G);
    a.K = (const u32x4 *)K; a.V = (const u32x4 *)V; a.q = (const u32x4 *)q;
    a.seq_lens = kv->seq_lens_dev;
    a.len_uniform = max_len;
    for (int b = 0; b < p->B; ++b)
        if (kv->seq_lens_host[b] != max_len) a.len_uniform = -1;
    a.part_acc = (float *)workspace;
    a.part_ml = a.part_acc + (size_t)p->B * p->Hq * ns * p->D;
    a.H = p->H; a.Hq = p->Hq; a.G = G; a.B = p->B;
    a.n_splits = ns;
    a.max_len = max_len;
    a.split_tokens = split_tokens_for(p, ns, max_len);
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)p->D));

    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf16 = p->dtype == KV_BF16;
    // A ragged batch of up to 64 sequences launches workgroups only for the splits that hold tokens (placed
    // over the compute units evenly); otherwise the grid is (split, query-head group, sequence).
    long long n_items = 0;
    for (int b = 0; b < p->B; ++b) n_items += (std::min(kv->seq_lens_host[b], max_len) + a.split_tokens - 1) / a.split_tokens;
    a.compact = a.len_uniform < 0 && p->B <= 64;
    dim3 grid((unsigned)ns, (unsigned)(p->Hq / gt), (unsigned)p->B);
    if (a.compact) grid = dim3((unsigned)n_items, (unsigned)(p->Hq / gt), 1u);
    if (n_items > 0) {
        if (p->D == 64) launch_partial_gt<64>(gt, bf16, paged, grid, st, a);
        else if (p->D == 128) launch_partial_gt<128>(gt, bf16, paged, grid, st, a);
        else launch_partial_gt<256>(gt, bf16, paged, grid, st, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    }

    const int out_mode = out_dtype == KV_OUT_F32 ? 0 : (bf16 ? 2 : 1);
    hipLaunchKernelGGL(kv_attn_combine_kernel, dim3((unsigned)p->Hq, (unsigned)p->B, (unsigned)(p->D / kCombineCols)), dim3(kCombineThreads), 0,
                       st, a.part_acc, a.part_ml, out, p->Hq, p->D, ns, out_mode, a.seq_lens, a.len_uniform, max_len,
                       a.split_tokens);
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
