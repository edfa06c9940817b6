/*
 * kv_oracle.c -- TEST INFRASTRUCTURE, not product code.
 *
 * A plain, slow, single-threaded CPU statement of what the KV offloading hot path
 * computes: the residency split, the LBA bind, the tensor-index-to-LBA translation,
 * the per-chunk command parameters, the extent byte order (pack / unpack) and one
 * decode-attention step.  Every function is the definition written out as scalar
 * loops in the paper's notation; there is no blocking, fusion or reordering.
 * It shares no code with the GPU library and is only used by the tests, the smoke
 * check and the CPU-baseline leg of the benchmark.
 *
 * The defining build is plain C, one thread (what every test uses).  The same file compiled
 * with -fopenmp is the all-core timing variant of the benchmark's CPU baseline: the loops over
 * tokens (pack / unpack) and over (b, h_q) (attention) are then shared among the threads; the
 * arithmetic of every output element is the same statement sequence in both builds.
 *
 * Pins (tests/test_oracle_*.py): sizes the paper prints (Table 2, Sec. III request
 * sizes and KV totals, Sec. V-A device parameters), the three bind invariants, brute
 * force sector sets on tiny shapes, NumPy transposes for the byte order, closed forms
 * for attention.  No function here is "parity unpinned".
 *
 * Readings taken where the paper leaves a choice:
 *  - n_blocks uses ceiling division and the pad bytes are zero; under the paper's
 *    alignment precondition (Sec. IV-B) this equals Eq. 5.
 *  - only direct-path tensors consume LBAs; page-cache-path tensors get byte offsets
 *    in one arena by the same padded recurrence, starting at 0.
 *  - tensor order is layer ascending, K before V (the id chain ..._k, ..._v, ..._k of
 *    Sec. IV-B).
 *  - offset_bytes / lba_size in Alg. 2 must divide exactly; otherwise ORC_EALIGN.
 *  - n_remains of Eq. 10 = ceil(req_bytes / lba_size) - (N-1) * n_maxBlocks.
 *  - attention = softmax(q K^T / sqrt(D)) V over tokens [0, len_b), kv head = h_q div G.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#define ORC_PARALLEL_FOR _Pragma("omp parallel for schedule(static)")
#else
#define ORC_PARALLEL_FOR
#endif

/* Threads the loops of this build are shared among (1 in the defining build). */
int orc_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

#define ORC_OK 0
#define ORC_EINVAL (-1)
#define ORC_EALIGN (-2)
#define ORC_ERANGE (-3)

/* ------------------------------------------------------------------ */
/* Alg. 1: KPU residency planner.  n1 = min(floor(X / (2 S_kpu)), L);  */
/* layers 1..n1 (0-based: 0..n1-1) take the page-cache path (x_i = 1). */
/* ------------------------------------------------------------------ */
int64_t orc_residency(uint64_t X, uint64_t S_kpu, int64_t L, int32_t *x /* [L] */)
{
    uint64_t fit = X / (2u * S_kpu);
    int64_t n1 = fit < (uint64_t)L ? (int64_t)fit : L;
    for (int64_t i = 1; i <= L; ++i)
        x[i - 1] = (i <= n1) ? 1 : 0;
    return n1;
}

/*
 * Eq. 1-2: page-cache budget.  M* = min(M_avail, M_max - M_anon+shmem);
 * B_pc = max(0, M* - N_threads * M_pin).  Signed 64-bit so that an over-committed cgroup
 * (M_anon+shmem > M_max) gives a negative M* and a zero budget.
 */
void orc_budget(int64_t M_avail, int64_t M_max, int64_t M_anon_shmem, int64_t N_threads, int64_t M_pin,
                int64_t *M_star, int64_t *B_pc)
{
    int64_t limit = M_max - M_anon_shmem;
    *M_star = M_avail < limit ? M_avail : limit;
    int64_t b = *M_star - N_threads * M_pin;
    *B_pc = b > 0 ? b : 0;
}

/*
 * Dataset-management deallocate (Sec. IV-B "TRIM"): for tensor n, the range <lba_start, n_blocks> of M
 * no longer holds valid data.  In the host-memory model a deallocated block reads back as zeros.
 * buf is the tensor's host buffer (region or arena), off the byte offset of its extent.
 */
void orc_trim(uint8_t *buf, uint64_t off, uint64_t n_blocks, uint64_t lba_size)
{
    memset(buf + off, 0, n_blocks * lba_size);
}

/*
 * Adaptive strategy selection (Sec. IV-C), per path group.  Decode iterations are counted from 1:
 * iteration 1 is the warm-up (not measured), iteration 2 runs overlap-intra (code 1), iteration 3
 * overlap-cross (code 0); from iteration 4 on the strategy with the higher measured throughput is used.
 * Readings: the warm-up runs overlap-intra; a tie keeps overlap-intra.
 */
int orc_adapt_order(int64_t iteration /* 1-based, the one about to run */, double thr_intra, double thr_cross)
{
    if (iteration <= 2) return 1;
    if (iteration == 3) return 0;
    return thr_cross > thr_intra ? 0 : 1;
}

/* Blocks of one sequence's rows: ceil(cap * row_bytes / lba_size). */
static uint64_t blocks_of(uint64_t bytes, uint64_t lba_size)
{
    return (bytes + lba_size - 1) / lba_size;
}

/*
 * Extent size of one K or V tensor, in blocks.
 * token-major (per_seq = 0): one extent of shape (S_cap, B*H, D); all cap[b] equal.
 * per-sequence (per_seq = 1): concatenation over b of sub-extents (cap_b, H, D), each
 * padded to a whole number of blocks; seq_base[b] = blocks before sequence b.
 * payload_bytes receives the unpadded byte count.
 */
int orc_tensor_blocks(int per_seq, int64_t B, const int32_t *cap, int64_t H, int64_t D,
                      int64_t e, uint64_t lba_size, uint64_t *n_blocks,
                      uint64_t *seq_base /* [B] or NULL */, uint64_t *payload_bytes)
{
    if (!per_seq) {
        for (int64_t b = 1; b < B; ++b)
            if (cap[b] != cap[0]) return ORC_EINVAL;
        uint64_t bytes = (uint64_t)cap[0] * (uint64_t)(B * H * D * e);
        *n_blocks = blocks_of(bytes, lba_size);
        *payload_bytes = bytes;
        if (seq_base)
            for (int64_t b = 0; b < B; ++b) seq_base[b] = 0;
        return ORC_OK;
    }
    uint64_t acc = 0, pay = 0;
    for (int64_t b = 0; b < B; ++b) {
        if (seq_base) seq_base[b] = acc;
        uint64_t bytes = (uint64_t)cap[b] * (uint64_t)(H * D * e);
        acc += blocks_of(bytes, lba_size);
        pay += bytes;
    }
    *n_blocks = acc;
    *payload_bytes = pay;
    return ORC_OK;
}

/*
 * Eq. 3-6: the map M : n -> <lba_start, n_blocks> for direct-path tensors, n = 2*layer + kind
 * (K = 0, V = 1), ascending.  lba_start(first direct tensor) is user-given, then
 * lba_start(n+1) = lba_start(n) + n_blocks(n).  Page-cache-path tensors get file_off in
 * bytes by the same recurrence from 0 and carry no LBA (lba_start written as 0).
 */
void orc_bind(int64_t L, const int32_t *x, uint64_t n_blocks_per_tensor, uint64_t lba_size,
              uint64_t lba_start_first, int32_t *path /* [2L] */, uint64_t *lba_start /* [2L] */,
              uint64_t *n_blocks /* [2L] */, uint64_t *file_off /* [2L] */)
{
    uint64_t next_lba = lba_start_first;
    uint64_t next_off = 0;
    for (int64_t layer = 0; layer < L; ++layer) {
        for (int kind = 0; kind < 2; ++kind) {
            int64_t n = 2 * layer + kind;
            n_blocks[n] = n_blocks_per_tensor;
            path[n] = x[layer];
            if (x[layer] == 0) {
                lba_start[n] = next_lba;
                file_off[n] = 0;
                next_lba += n_blocks_per_tensor;
            } else {
                lba_start[n] = 0;
                file_off[n] = next_off;
                next_off += n_blocks_per_tensor * lba_size;
            }
        }
    }
}

/*
 * Alg. 2: tensor-index-to-LBA translation.
 * shape_src = (f0,f1,f2), shape_tgt = (d0,d1,d2), offset indices (i0,j0,k0) in the target,
 * e bytes per element.  offset_elem = (i0*d1 + j0)*d2 + k0; offset_bytes = offset_elem*e;
 * slba* = lba_start + offset_bytes / lba_size; req_bytes = f0*f1*f2*e.
 */
int orc_translate(uint64_t lba_start, const int64_t f[3], const int64_t d[3], const int64_t idx[3],
                  int64_t e, uint64_t lba_size, uint64_t *slba_star, uint64_t *req_bytes)
{
    if (idx[0] < 0 || idx[1] < 0 || idx[2] < 0) return ORC_EINVAL;
    if (idx[0] >= d[0] || idx[1] >= d[1] || idx[2] >= d[2]) return ORC_ERANGE;
    uint64_t offset_elem = ((uint64_t)idx[0] * (uint64_t)d[1] + (uint64_t)idx[1]) * (uint64_t)d[2]
                           + (uint64_t)idx[2];
    uint64_t offset_bytes = offset_elem * (uint64_t)e;
    uint64_t req = (uint64_t)f[0] * (uint64_t)f[1] * (uint64_t)f[2] * (uint64_t)e;
    uint64_t total = (uint64_t)d[0] * (uint64_t)d[1] * (uint64_t)d[2] * (uint64_t)e;
    if (offset_bytes + req > total) return ORC_ERANGE;
    if (offset_bytes % lba_size != 0) return ORC_EALIGN;
    *slba_star = lba_start + offset_bytes / lba_size;
    *req_bytes = req;
    return ORC_OK;
}

/* Eq. 7: the largest LBA-aligned size within the device's maximum data transfer size. */
uint64_t orc_chunk_size(uint64_t mdts_bytes, uint64_t lba_size)
{
    return mdts_bytes / lba_size * lba_size;
}

/*
 * Eq. 7-11: chunking of one request.  chunk_bytes is a multiple of lba_size (Eq. 7 makes it
 * so from MDTS); n_chunks = ceil(req_bytes / chunk_bytes); n_maxBlocks = chunk_bytes / lba_size;
 * for N = 1..n_chunks: slba = slba* + (N-1) n_maxBlocks, nlb = min(n_maxBlocks, n_remains) - 1
 * (0-based count), dbuf = buf + (N-1) chunk_bytes.
 * Returns n_chunks (or a negative code); writes at most cap entries.
 */
int64_t orc_chunk_cmds(uint64_t slba_star, uint64_t req_bytes, uint64_t chunk_bytes, uint64_t lba_size,
                       int64_t cap, uint64_t *slba, uint32_t *nlb, uint64_t *dbuf_off)
{
    if (chunk_bytes == 0 || chunk_bytes % lba_size != 0) return ORC_EALIGN;
    uint64_t n_chunks = (req_bytes + chunk_bytes - 1) / chunk_bytes;
    uint64_t n_maxBlocks = chunk_bytes / lba_size;
    uint64_t n_total = (req_bytes + lba_size - 1) / lba_size;
    for (uint64_t N = 1; N <= n_chunks && (int64_t)N <= cap; ++N) {
        uint64_t n_remains = n_total - (N - 1) * n_maxBlocks;
        uint64_t blocks = n_maxBlocks < n_remains ? n_maxBlocks : n_remains;
        slba[N - 1] = slba_star + (N - 1) * n_maxBlocks;
        nlb[N - 1] = (uint32_t)(blocks - 1);
        dbuf_off[N - 1] = (N - 1) * chunk_bytes;
    }
    return (int64_t)n_chunks;
}

/* ------------------------------------------------------------------ */
/* Attention-side layouts.                                             */
/* ------------------------------------------------------------------ */
typedef struct {
    int32_t paged;          /* 0: strided [B,H,S,D]; 1: block pool [n_pool,H,block_tokens,D] */
    int64_t stride_b, stride_h, stride_s; /* elements, strided layout; d stride is 1 */
    const int32_t *block_table;           /* [B, max_blocks] */
    int64_t max_blocks;
    int64_t block_tokens;
    int64_t H, D;
} orc_src_t;

/* Element index of (b,h,s,d) in the attention-side buffer. */
static int64_t src_index(const orc_src_t *v, int64_t b, int64_t h, int64_t s, int64_t d)
{
    if (!v->paged)
        return b * v->stride_b + h * v->stride_h + s * v->stride_s + d;
    int64_t blk = v->block_table[b * v->max_blocks + s / v->block_tokens];
    int64_t slot = s % v->block_tokens;
    return ((blk * v->H + h) * v->block_tokens + slot) * v->D + d;
}

/*
 * Extent byte order (Sec. IV-B precondition; Alg. 2 row-major offset): the extent of a tensor is
 * the row-major array (S, B*H, D).  Pack writes extent element ((s*B + b)*H + h)*D + d from the
 * attention-side element (b,h,s,d); bytes between the payload and n_blocks*lba_size are zero.
 * Per-sequence mode: sequence b has its own row-major (len_b, H, D) array starting seq_base[b]
 * blocks into the extent, padded with zeros to a whole block.
 * ext points at the first byte of the tensor's extent (region + lba_start*lba_size).
 */
void orc_pack(const orc_src_t *v, const uint16_t *src, int per_seq, int64_t B, const int32_t *len,
              const uint64_t *seq_base, uint64_t n_blocks, uint64_t lba_size, uint8_t *ext)
{
    int64_t H = v->H, D = v->D;
    uint16_t *out = (uint16_t *)ext;
    if (!per_seq) {
        int64_t S = len[0];
        ORC_PARALLEL_FOR
        for (int64_t s = 0; s < S; ++s)
            for (int64_t b = 0; b < B; ++b)
                for (int64_t h = 0; h < H; ++h)
                    for (int64_t d = 0; d < D; ++d)
                        out[((s * B + b) * H + h) * D + d] = src[src_index(v, b, h, s, d)];
        uint64_t bytes = (uint64_t)(S * B * H * D) * 2u;
        memset(ext + bytes, 0, n_blocks * lba_size - bytes);
        return;
    }
    for (int64_t b = 0; b < B; ++b) {
        uint16_t *sub = (uint16_t *)(ext + seq_base[b] * lba_size);
        ORC_PARALLEL_FOR
        for (int64_t s = 0; s < len[b]; ++s)
            for (int64_t h = 0; h < H; ++h)
                for (int64_t d = 0; d < D; ++d)
                    sub[(s * H + h) * D + d] = src[src_index(v, b, h, s, d)];
        uint64_t bytes = (uint64_t)(len[b] * H * D) * 2u;
        uint64_t end = (b + 1 < B ? seq_base[b + 1] : n_blocks) * lba_size;
        memset((uint8_t *)sub + bytes, 0, end - seq_base[b] * lba_size - bytes);
    }
}

/* Inverse assignment, valid tokens only; other destination elements are left as they are. */
void orc_unpack(const orc_src_t *v, uint16_t *dst, int per_seq, int64_t B, const int32_t *len,
                const uint64_t *seq_base, uint64_t lba_size, const uint8_t *ext)
{
    int64_t H = v->H, D = v->D;
    const uint16_t *in = (const uint16_t *)ext;
    if (!per_seq) {
        int64_t S = len[0];
        ORC_PARALLEL_FOR
        for (int64_t s = 0; s < S; ++s)
            for (int64_t b = 0; b < B; ++b)
                for (int64_t h = 0; h < H; ++h)
                    for (int64_t d = 0; d < D; ++d)
                        dst[src_index(v, b, h, s, d)] = in[((s * B + b) * H + h) * D + d];
        return;
    }
    for (int64_t b = 0; b < B; ++b) {
        const uint16_t *sub = (const uint16_t *)(ext + seq_base[b] * lba_size);
        ORC_PARALLEL_FOR
        for (int64_t s = 0; s < len[b]; ++s)
            for (int64_t h = 0; h < H; ++h)
                for (int64_t d = 0; d < D; ++d)
                    dst[src_index(v, b, h, s, d)] = sub[(s * H + h) * D + d];
    }
}

/* ------------------------------------------------------------------ */
/* 16-bit float decoding, exact in double.                             */
/* ------------------------------------------------------------------ */
double orc_f16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, ex = (h >> 10) & 0x1f, man = h & 0x3ff;
    double v;
    if (ex == 0) v = ldexp((double)man, -24);
    else if (ex == 31) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 0x400), ex - 25);
    return sign ? -v : v;
}

double orc_bf16_to_double(uint16_t h)
{
    int sign = (h >> 15) & 1, ex = (h >> 7) & 0xff, man = h & 0x7f;
    double v;
    if (ex == 0) v = ldexp((double)man, -133);
    else if (ex == 255) v = man ? NAN : INFINITY;
    else v = ldexp((double)(man | 0x80), ex - 134);
    return sign ? -v : v;
}

/*
 * One decode-attention step (Sec. II-A: similarity of Q with K weights V), unblocked:
 * for each b and query head hq, kv head h = hq / G (G = Hq / H):
 *   s_j = (sum_d q[d] K[j][d]) / sqrt(D), j in [0, len_b)
 *   p   = softmax(s)   (subtract the maximum, exponentiate, normalise)
 *   out[d] = sum_j p_j V[j][d]
 * all in double.  is_bf16 selects the input decoding.  out is [B, Hq, D] doubles.
 * A sequence with len_b = 0 yields zeros.
 */
int orc_attention(const orc_src_t *v, const uint16_t *K, const uint16_t *V, const uint16_t *q,
                  int is_bf16, int64_t B, int64_t Hq, const int32_t *len, double *out)
{
    int64_t H = v->H, D = v->D;
    if (Hq % H != 0) return ORC_EINVAL;
    int64_t G = Hq / H;
    double (*dec)(uint16_t) = is_bf16 ? orc_bf16_to_double : orc_f16_to_double;
    int failed = 0;
    /* every (b, hq) is independent: its own score buffer, its own output row */
    ORC_PARALLEL_FOR
    for (int64_t bh = 0; bh < B * Hq; ++bh) {
        int64_t b = bh / Hq, hq = bh % Hq;
        int64_t h = hq / G;
        double *o = out + (b * Hq + hq) * D;
        for (int64_t d = 0; d < D; ++d) o[d] = 0.0;
        int64_t n = len[b];
        if (n == 0) continue;
        double *s = (double *)malloc(sizeof(double) * (size_t)n);
        if (!s) { failed = 1; continue; }
        double m = -INFINITY;
        for (int64_t j = 0; j < n; ++j) {
            double dot = 0.0;
            for (int64_t d = 0; d < D; ++d)
                dot += dec(q[(b * Hq + hq) * D + d]) * dec(K[src_index(v, b, h, j, d)]);
            s[j] = dot / sqrt((double)D);
            if (s[j] > m) m = s[j];
        }
        double denom = 0.0;
        for (int64_t j = 0; j < n; ++j) {
            s[j] = exp(s[j] - m);
            denom += s[j];
        }
        for (int64_t j = 0; j < n; ++j) {
            double p = s[j] / denom;
            for (int64_t d = 0; d < D; ++d)
                o[d] += p * dec(V[src_index(v, b, h, j, d)]);
        }
        free(s);
    }
    return failed ? ORC_EINVAL : ORC_OK;
}
