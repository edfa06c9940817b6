// Split-K decode attention over resident KV (Sec. II-A: the query's similarity with the keys weights
// the values):  out[b,hq,:] = softmax_j(q[b,hq,:].K[b,h,j,:] / sqrt(D)) V[b,h,j,:],  h = hq / G.
//
// Partial kernel, grid (split, query-head group, b), 4 wavefronts per workgroup.  A K or V row of D
// 16-bit elements is held by D/8 lanes (16 bytes each), so one wavefront load covers 64/(D/8)
// consecutive rows = 1 KiB of contiguous memory.  Each lane group keeps its own running (m, l, acc)
// in fp32 for the GT query heads that share the kv head (K and V are read once for all of them);
// groups, then wavefronts, are merged at the end and one fp32 partial per (b, hq, split) is written.
// The combine kernel merges the splits.  The path is HBM-bound (G flop per byte).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>

#include "plan.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int kR = 4;                 // rows in flight per lane group
constexpr float kEmptyMax = -1.0e30f; // running maximum of a group that has seen no token

struct AttnParams {
    const u32x4 *K, *V;    // attention-side buffers of the layer
    const u32x4 *q;        // [B, Hq, D]
    const int *seq_lens;   // device [B]
    float *part_acc;       // [B, Hq, n_splits, D]
    float *part_ml;        // [B, Hq, n_splits, 2]
    long long sb, sh, ss;  // strided layout, in 16-byte vectors
    const int *table;      // paged layout
    int max_blocks, bt, bt_shift, n_pool;
    int H, Hq, G;
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

template <int LPR, int GT, bool BF16, bool PAGED>
__global__ void __launch_bounds__(kThreads) kv_attn_partial_kernel(AttnParams p)
{
    constexpr int RPW = 64 / LPR;  // rows per wavefront load
    constexpr int D = LPR * 8;
    const int split = blockIdx.x, hq0 = blockIdx.y * GT, b = blockIdx.z;
    const int h = hq0 / p.G;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lr = lane % LPR;  // position inside the row (16-byte vector index)
    const int rg = lane / LPR;  // lane group = which of the RPW rows of a load

    const int len = min(p.seq_lens[b], p.max_len);
    const int t_begin = min(len, split * p.split_tokens);
    const int t_end = min(len, t_begin + p.split_tokens);

    // q for the GT heads, pre-scaled so that scores are in log2 units.
    float qf[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        const u32x4 qv = p.q[((long long)b * p.Hq + hq0 + g) * LPR + lr];
        unpack8<BF16>(qv, qf[g]);
#pragma unroll
        for (int i = 0; i < 8; ++i) qf[g][i] *= p.scale_log2e;
    }

    float m[GT], l[GT], acc[GT][8];
#pragma unroll
    for (int g = 0; g < GT; ++g) {
        m[g] = kEmptyMax;
        l[g] = 0.f;
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;
    }

    const long long head_off = PAGED ? 0 : (long long)b * p.sb + (long long)h * p.sh + lr;
    const int *tbl = PAGED ? p.table + (long long)b * p.max_blocks : nullptr;
    constexpr int kRowsPerIter = kWaves * RPW * kR;

    for (int t0 = t_begin; t0 < t_end; t0 += kRowsPerIter) {
        u32x4 kv[kR], vv[kR];
        bool ok[kR];
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            const int row = t0 + (u * kWaves + wave) * RPW + rg;
            ok[u] = row < t_end;
            const int rr = ok[u] ? row : t_begin;  // a valid row; its score is masked below
            long long a;
            if (PAGED) {
                const int j = p.bt_shift >= 0 ? (rr >> p.bt_shift) : (rr / p.bt);
                const int slot = rr - j * p.bt;
                int blk = tbl[j];
                if ((unsigned)blk >= (unsigned)p.n_pool) { blk = 0; ok[u] = false; }
                a = (((long long)blk * p.H + h) * p.bt + slot) * LPR + lr;
            } else {
                a = head_off + (long long)rr * p.ss;
            }
            kv[u] = p.K[a];
            vv[u] = p.V[a];
        }

        float s[kR][GT];
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            float kf[8];
            unpack8<BF16>(kv[u], kf);
#pragma unroll
            for (int g = 0; g < GT; ++g) {
                float d = 0.f;
#pragma unroll
                for (int i = 0; i < 8; ++i) d = fmaf(qf[g][i], kf[i], d);
#pragma unroll
                for (int off = 1; off < LPR; off <<= 1) d += __shfl_xor(d, off);
                s[u][g] = ok[u] ? d : -INFINITY;
            }
        }

        float pr[kR][GT];
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            float mn = m[g];
#pragma unroll
            for (int u = 0; u < kR; ++u) mn = fmaxf(mn, s[u][g]);
            const float alpha = exp2f(m[g] - mn);
            float ps = 0.f;
#pragma unroll
            for (int u = 0; u < kR; ++u) {
                pr[u][g] = exp2f(s[u][g] - mn);
                ps += pr[u][g];
            }
            l[g] = l[g] * alpha + ps;
            m[g] = mn;
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g][i] *= alpha;
        }
#pragma unroll
        for (int u = 0; u < kR; ++u) {
            float vf[8];
            unpack8<BF16>(vv[u], vf);
#pragma unroll
            for (int g = 0; g < GT; ++g)
#pragma unroll
                for (int i = 0; i < 8; ++i) acc[g][i] = fmaf(pr[u][g], vf[i], acc[g][i]);
        }
    }

    // Merge the lane groups of this wavefront (lanes LPR, 2*LPR, ... apart hold the same d positions).
#pragma unroll
    for (int off = LPR; off < 64; off <<= 1) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
            const float m2 = __shfl_xor(m[g], off), l2 = __shfl_xor(l[g], off);
            float a2[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) a2[i] = __shfl_xor(acc[g][i], off);
            merge<8>(m[g], l[g], acc[g], m2, l2, a2);
        }
    }

    // Merge the wavefronts through LDS.
    __shared__ float sh_acc[kWaves][GT][D];
    __shared__ float sh_ml[kWaves][GT][2];
    if (rg == 0) {
#pragma unroll
        for (int g = 0; g < GT; ++g) {
#pragma unroll
            for (int i = 0; i < 8; ++i) sh_acc[wave][g][lr * 8 + i] = acc[g][i];
            if (lr == 0) { sh_ml[wave][g][0] = m[g]; sh_ml[wave][g][1] = l[g]; }
        }
    }
    __syncthreads();
    for (int idx = threadIdx.x; idx < GT * D; idx += kThreads) {
        const int g = idx / D, d = idx - g * D;
        float M = sh_ml[0][g][0];
#pragma unroll
        for (int w = 1; w < kWaves; ++w) M = fmaxf(M, sh_ml[w][g][0]);
        float L = 0.f, A = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) {
            const float a = exp2f(sh_ml[w][g][0] - M);
            L += sh_ml[w][g][1] * a;
            A += sh_acc[w][g][d] * a;
        }
        const long long o = ((long long)b * p.Hq + hq0 + g) * p.n_splits + split;
        p.part_acc[o * D + d] = A;
        if (d == 0) { p.part_ml[o * 2] = M; p.part_ml[o * 2 + 1] = L; }
    }
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float f)
{
    unsigned u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (unsigned short)((u >> 16) | 0x40);  // quiet NaN
    u += 0x7fffu + ((u >> 16) & 1u);
    return (unsigned short)(u >> 16);
}

// out_mode: 0 fp32, 1 fp16, 2 bf16.  One workgroup of 256 threads per (hq, b).  The split weights
// exp2(m_s - M) are computed once, in parallel over the splits, and kept in LDS; then thread d sums
// its column over the splits with independent (pipelined) loads.
constexpr int kCombineThreads = 256;
constexpr int kMaxSplits = 1024;

__global__ void __launch_bounds__(kCombineThreads)
kv_attn_combine_kernel(const float *__restrict__ part_acc, const float *__restrict__ part_ml,
                       void *__restrict__ out, int Hq, int D, int n_splits, int out_mode)
{
    __shared__ float w[kMaxSplits];
    __shared__ float red[kCombineThreads / 64];
    __shared__ float sh_M, sh_L;
    const int hq = blockIdx.x, b = blockIdx.y, tid = threadIdx.x;
    const long long o = ((long long)b * Hq + hq) * n_splits;

    float mx = kEmptyMax;
    for (int s = tid; s < n_splits; s += kCombineThreads) mx = fmaxf(mx, part_ml[(o + s) * 2]);
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    if ((tid & 63) == 0) red[tid >> 6] = mx;
    __syncthreads();
    if (tid == 0) {
        float M = red[0];
        for (int i = 1; i < kCombineThreads / 64; ++i) M = fmaxf(M, red[i]);
        sh_M = M;
    }
    __syncthreads();
    const float M = sh_M;
    float lsum = 0.f;
    for (int s = tid; s < n_splits; s += kCombineThreads) {
        const float a = exp2f(part_ml[(o + s) * 2] - M);
        w[s] = a;
        lsum += part_ml[(o + s) * 2 + 1] * a;
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) lsum += __shfl_xor(lsum, off);
    __syncthreads();  // red is reused
    if ((tid & 63) == 0) red[tid >> 6] = lsum;
    __syncthreads();
    if (tid == 0) {
        float L = 0.f;
        for (int i = 0; i < kCombineThreads / 64; ++i) L += red[i];
        sh_L = L;
    }
    __syncthreads();
    const float L = sh_L;
    for (int d = tid; d < D; d += kCombineThreads) {
        float A = 0.f;
#pragma unroll 8
        for (int s = 0; s < n_splits; ++s) A = fmaf(part_acc[(o + s) * D + d], w[s], A);
        const float r = L > 0.f ? A / L : 0.f;
        const long long oi = ((long long)b * Hq + hq) * D + d;
        if (out_mode == 0) ((float *)out)[oi] = r;
        else if (out_mode == 1) ((_Float16 *)out)[oi] = (_Float16)r;  // round to nearest even
        else ((unsigned short *)out)[oi] = f32_to_bf16_rne(r);
    }
}

int pick_gt(int G) { return G % 4 == 0 ? 4 : (G % 2 == 0 ? 2 : 1); }

// Tokens per split: a multiple of the rows one workgroup iteration covers.
int split_quantum(int D) { return kWaves * (64 / (D / 8)) * kR; }

int choose_splits(const kv_plan *p, int max_len)
{
    if (max_len <= 0) return 1;
    const int q = split_quantum(p->D);
    const long long groups = (long long)p->B * (p->Hq / pick_gt(p->Hq / p->H));
    // aim at ~4 workgroups per compute unit, at least 2 iterations each
    long long want = std::max<long long>(1, (1024 + groups - 1) / groups);
    const long long max_by_len = std::max<long long>(1, (long long)max_len / (2 * q));
    want = std::min(want, max_by_len);
    return (int)std::min<long long>(want, 1024);
}

int split_tokens_for(const kv_plan *p, int n_splits, int max_len)
{
    const int q = split_quantum(p->D);
    long long st = ((long long)max_len + n_splits - 1) / n_splits;
    st = (st + q - 1) / q * q;
    return (int)std::max<long long>(st, q);
}

template <int LPR, int GT>
void launch_partial(bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a)
{
    if (bf16) {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<LPR, GT, true, true>), grid, dim3(kThreads), 0, st, a);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<LPR, GT, true, false>), grid, dim3(kThreads), 0, st, a);
    } else {
        if (paged) hipLaunchKernelGGL((kv_attn_partial_kernel<LPR, GT, false, true>), grid, dim3(kThreads), 0, st, a);
        else hipLaunchKernelGGL((kv_attn_partial_kernel<LPR, GT, false, false>), grid, dim3(kThreads), 0, st, a);
    }
}

template <int LPR>
void launch_partial_gt(int gt, bool bf16, bool paged, dim3 grid, hipStream_t st, const AttnParams &a)
{
    if (gt == 4) launch_partial<LPR, 4>(bf16, paged, grid, st, a);
    else if (gt == 2) launch_partial<LPR, 2>(bf16, paged, grid, st, a);
    else launch_partial<LPR, 1>(bf16, paged, grid, st, a);
}

}  // namespace

extern "C" size_t kv_decode_attn_workspace(const kv_plan_t *p, int n_splits, int max_len)
{
    if (!p || n_splits < 0 || max_len < 0) return 0;
    const int ns = n_splits > 0 ? n_splits : choose_splits(p, max_len);
    return (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
}

extern "C" int kv_decode_attn(const kv_plan_t *p, const kv_view_t *kv, int layer, const void *q, void *out,
                              int out_dtype, int n_splits, void *workspace, size_t ws_bytes, void *hip_stream)
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
        if (max_len > 0) {
            const uint64_t max_elem = (uint64_t)(p->B - 1) * kv->stride_b + (uint64_t)(p->H - 1) * kv->stride_h +
                                      (uint64_t)(max_len - 1) * kv->stride_s + p->D;
            if (max_elem * 2 > kv->layer_bytes) return KV_ERANGE;
        }
        a.sb = kv->stride_b / 8; a.sh = kv->stride_h / 8; a.ss = kv->stride_s / 8;
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

    const int ns = n_splits > 0 ? n_splits : choose_splits(p, max_len);
    const size_t need = (size_t)p->B * p->Hq * ns * (p->D + 2) * sizeof(float);
    if (ws_bytes < need) return KV_ENOSPC;

    const int G = p->Hq / p->H, gt = pick_gt(G);
    a.K = (const u32x4 *)K; a.V = (const u32x4 *)V; a.q = (const u32x4 *)q;
    a.seq_lens = kv->seq_lens_dev;
    a.part_acc = (float *)workspace;
    a.part_ml = a.part_acc + (size_t)p->B * p->Hq * ns * p->D;
    a.H = p->H; a.Hq = p->Hq; a.G = G;
    a.n_splits = ns;
    a.max_len = max_len;
    a.split_tokens = split_tokens_for(p, ns, max_len);
    a.scale_log2e = (float)(1.4426950408889634 / std::sqrt((double)p->D));

    hipStream_t st = (hipStream_t)hip_stream;
    const bool bf16 = p->dtype == KV_BF16;
    dim3 grid((unsigned)ns, (unsigned)(p->Hq / gt), (unsigned)p->B);
    if (p->D == 64) launch_partial_gt<8>(gt, bf16, paged, grid, st, a);
    else if (p->D == 128) launch_partial_gt<16>(gt, bf16, paged, grid, st, a);
    else launch_partial_gt<32>(gt, bf16, paged, grid, st, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }

    const int out_mode = out_dtype == KV_OUT_F32 ? 0 : (bf16 ? 2 : 1);
    hipLaunchKernelGGL(kv_attn_combine_kernel, dim3((unsigned)p->Hq, (unsigned)p->B), dim3(kCombineThreads), 0,
                       st, a.part_acc, a.part_ml, out, p->Hq, p->D, ns, out_mode);
    e = hipGetLastError();
    if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    return KV_OK;
}
