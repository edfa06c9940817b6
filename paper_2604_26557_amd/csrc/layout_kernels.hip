// Pack / unpack: the byte permutation between the attention-side KV layout (strided [B,H,S,D] or a
// paged block pool) and extent order, the row-major (S, B*H, D) array of Sec. IV-B.
//
// The innermost D row (D*2 bytes, a multiple of 16) is preserved by the permutation, so the kernels
// move whole 16-byte vectors: one lane = one global_load_dwordx4 + one global_store_dwordx4.
// Threads are laid out as (rx, ty): rx walks the vectors of one extent row (consecutive lanes ->
// consecutive extent bytes, so a wavefront touches >= 1 KiB of contiguous extent and whole head rows
// of the source), ty walks token rows.  The (b, h, d) decomposition of a row position is done once
// per thread per row position and reused for every token, so the inner loop is adds, U independent
// 16-byte loads, then U stores.  HBM-bound: 2 bytes of traffic per payload byte, no reuse, no LDS.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <climits>

#include "plan.hpp"

namespace {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

constexpr int kThreads = 256;
constexpr int kMaxSegs = 32;
constexpr int kTblStage = 64;  // block-table entries one workgroup can stage in LDS

// Attention-side addressing, in 16-byte vectors.
struct SrcDesc {
    long long sb, sh, ss;  // strided layout: vectors per batch / head / token step
    const int *table;      // paged layout
    int max_blocks, bt, bt_shift, n_pool;
    int H, dvec;           // heads, vectors per head row
};

// One contiguous run of token rows of one (sub-)extent inside the image buffer.
struct Seg {
    unsigned long long img_off;  // vector index in the image of row 0 of this run
    unsigned long long pad_off;  // vector index of the first pad vector (pack only)
    unsigned int pad_vecs;       // zero vectors to write (pack only)
    int b;                       // sequence, or -1: the batch index is part of the row position
    int tok0, ntok;
    u32x4 *base;                 // the attention-side buffer this run belongs to (K or V of some layer)
};

struct SegTable {
    Seg seg[kMaxSegs];
};

// Every byte is touched once: nontemporal loads and stores keep the streams out of each other's way in L2.
__device__ __forceinline__ u32x4 ld(const u32x4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }

// PACK: source -> image.  !PACK: image -> source.  U = token rows in flight per thread.
template <bool PACK, bool PAGED, int U>
__global__ void __launch_bounds__(kThreads)
kv_layout_kernel(SrcDesc s, u32x4 *__restrict__ img, SegTable segs, int rowv, int rx_log2, int tpb, int rchunk)
{
    const Seg sg = segs.seg[blockIdx.y];
    const int tid = threadIdx.x;
    u32x4 *const base = sg.base;

    if (PACK && sg.pad_vecs && blockIdx.z == 0) {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (unsigned int i = blockIdx.x * kThreads + tid; i < sg.pad_vecs; i += gridDim.x * kThreads)
            img[sg.pad_off + i] = z;
    }

    const int t_begin = blockIdx.x * tpb;
    if (t_begin >= sg.ntok) return;
    const int t_end = min(sg.ntok, t_begin + tpb);

    const int RX = 1 << rx_log2;
    const int TY = kThreads >> rx_log2;
    const int rx = tid & (RX - 1);
    const int ty = tid >> rx_log2;
    const int hd = s.H * s.dvec;

    // Paged source, one sequence per segment: the few block-table entries this tile touches are staged in
    // LDS once, so the per-token lookup is not a second dependent trip to memory.
    __shared__ int sh_tbl[kTblStage];
    int j_first = 0;
    bool tbl_in_lds = false;
    if (PAGED && sg.b >= 0) {
        j_first = (sg.tok0 + t_begin) / s.bt;
        const int nj = (sg.tok0 + t_end - 1) / s.bt - j_first + 1;
        if (nj <= kTblStage) {  // uniform over the workgroup
            const int *row = s.table + (long long)sg.b * s.max_blocks;
            for (int i = tid; i < nj; i += kThreads) sh_tbl[i] = row[j_first + i];
            __syncthreads();
            tbl_in_lds = true;
        }
    }

    // this workgroup's share of the row positions (a wide row is cut into chunks, so that a tile spans fewer
    // source head rows and more tokens of each)
    const int r_begin = blockIdx.z * rchunk, r_end = min(rowv, r_begin + rchunk);
    for (int r = r_begin + rx; r < r_end; r += RX) {
        int b, rem;
        if (sg.b >= 0) { b = sg.b; rem = r; } else { b = r / hd; rem = r - b * hd; }
        const int h = rem / s.dvec;
        const int dv = rem - h * s.dvec;
        const long long row_off = PAGED ? 0 : (long long)b * s.sb + (long long)h * s.sh + dv;
        const int *tbl = PAGED ? s.table + (long long)b * s.max_blocks : nullptr;

        for (int t0 = t_begin + ty; t0 < t_end; t0 += TY * U) {
            u32x4 v[U];
            long long a[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int t = t0 + u * TY;
                ok[u] = t < t_end;
                a[u] = 0;
                if (ok[u]) {
                    const int tok = sg.tok0 + t;
                    if (PAGED) {
                        const int j = s.bt_shift >= 0 ? (tok >> s.bt_shift) : (tok / s.bt);
                        const int slot = tok - j * s.bt;
                        const int blk = tbl_in_lds ? sh_tbl[j - j_first] : tbl[j];
                        ok[u] = (unsigned)blk < (unsigned)s.n_pool;  // ids outside the pool are skipped
                        a[u] = (((long long)blk * s.H + h) * s.bt + slot) * s.dvec + dv;
                    } else {
                        a[u] = row_off + (long long)tok * s.ss;
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned long long i = sg.img_off + (unsigned long long)(t0 + u * TY) * rowv + r;
                if (ok[u]) v[u] = PACK ? ld(base + a[u]) : ld(img + i);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const unsigned long long i = sg.img_off + (unsigned long long)(t0 + u * TY) * rowv + r;
                if (PACK) {
                    // a skipped block id still owns its bytes of the image: they read as zero
                    const bool in = (t0 + u * TY) < t_end;
                    const u32x4 z = {0u, 0u, 0u, 0u};
                    if (in) st(img + i, ok[u] ? v[u] : z);
                } else if (ok[u]) {
                    st(base + a[u], v[u]);
                }
            }
        }
    }
}

int check_view(const kv_plan *p, const kv_view_t *v, int layer)
{
    if (!v || !v->k_layers || !v->v_layers || !v->seq_lens_host) return KV_EINVAL;
    if (layer < 0 || layer >= p->L || layer >= v->n_layers) return KV_ERANGE;
    if (!v->k_layers[layer] || !v->v_layers[layer]) return KV_EINVAL;
    if (((uintptr_t)v->k_layers[layer] | (uintptr_t)v->v_layers[layer]) & 15) return KV_EINVAL;
    if (v->seq_off_host || v->seq_off_dev) return KV_EINVAL;  // per-sequence offsets are for attention only
    if (v->layout == KV_LAYOUT_BHSD) {
        if (v->stride_b < 0 || v->stride_h < 0 || v->stride_s < 0 || v->s_alloc < 0) return KV_EINVAL;
        if ((v->stride_b | v->stride_h | v->stride_s) & 7) return KV_EINVAL;
        if (v->stride_s < p->D) return KV_EINVAL;
    } else if (v->layout == KV_LAYOUT_PAGED) {
        if (!v->block_table || v->block_tokens < 1 || v->n_pool_blocks < 0 || v->max_blocks_per_seq < 0)
            return KV_EINVAL;
        const uint64_t pool = (uint64_t)v->n_pool_blocks * p->H * v->block_tokens * p->D * 2;
        if (pool > v->layer_bytes) return KV_ERANGE;
    } else {
        return KV_EINVAL;
    }
    return KV_OK;
}

// Rows [tok0, tok0+ntok) of sequence b (or of every sequence when b < 0) must exist in the view.
int check_rows(const kv_plan *p, const kv_view_t *v, int b, int tok0, int ntok)
{
    const int b0 = b < 0 ? 0 : b, b1 = b < 0 ? p->B : b + 1;
    const long long last = (long long)tok0 + ntok;  // one past the last row
    if (ntok == 0) return KV_OK;
    if (v->layout == KV_LAYOUT_BHSD) {
        if (last > v->s_alloc) return KV_ERANGE;
        const uint64_t max_elem = (uint64_t)(b1 - 1) * v->stride_b + (uint64_t)(p->H - 1) * v->stride_h +
                                  (uint64_t)(last - 1) * v->stride_s + p->D;
        if (max_elem * 2 > v->layer_bytes) return KV_ERANGE;
    } else {
        for (int i = b0; i < b1; ++i) {
            if (last > v->seq_lens_host[i]) return KV_ERANGE;
            if (kvb::ceil_div((uint64_t)last, (uint64_t)v->block_tokens) > (uint64_t)v->max_blocks_per_seq)
                return KV_ERANGE;
        }
    }
    return KV_OK;
}

u32x4 *tensor_base(const kv_view_t *v, int layer, int which)
{
    return (u32x4 *)(which == 0 ? v->k_layers[layer] : v->v_layers[layer]);
}

SrcDesc make_src(const kv_plan *p, const kv_view_t *v)
{
    SrcDesc s{};
    s.H = p->H;
    s.dvec = p->D / 8;
    if (v->layout == KV_LAYOUT_BHSD) {
        s.sb = v->stride_b / 8; s.sh = v->stride_h / 8; s.ss = v->stride_s / 8;
    } else {
        s.table = v->block_table;
        s.max_blocks = v->max_blocks_per_seq;
        s.bt = v->block_tokens;
        s.bt_shift = (s.bt & (s.bt - 1)) == 0 ? __builtin_ctz((unsigned)s.bt) : -1;
        s.n_pool = v->n_pool_blocks;
    }
    return s;
}

// Launch shape.  rx_cap: most lanes (log2) along an extent row; unroll: token rows in flight per thread (2, 4
// or 8); tile_bytes: extent bytes one workgroup moves; run_bytes: consecutive source bytes per head row a tile
// should reach when the row is cut into chunks.
struct Shape {
    int rx_cap, unroll, tile_bytes, run_bytes;
};

// Measured best on MI355X (sweeps over rx_cap 4-8, unroll 2/4/8, tiles 16-512 KiB, runs 0.5-64 KiB at the 2 KiB-row
// and 32 KiB-row shapes, strided and paged, 8 MiB to 256 MiB tensors).  What the table encodes: a tile should touch
// few attention-side head streams, each for a long run of consecutive tokens; on the extent side 256-512 byte
// pieces are fine, since they fall inside one compact window of the image.  So a narrow row gets 16-32 lanes along
// the row and 64-128 tokens per tile, a very wide row is cut into chunks so that a tile does not touch every head's
// stream for a few hundred bytes, and launches too small to give every compute unit several tiles take the finer
// shape.  The pack / unpack difference in lane count and unroll is empirical.
Shape pick_shape(bool pack, bool paged, int rowv, unsigned long long launch_bytes)
{
    if (rowv > 256) return Shape{8, 4, 64 * 1024, 16 * 1024};
    if (paged) return pack ? Shape{8, 8, 32 * 1024, 16 * 1024} : Shape{4, 4, 32 * 1024, 16 * 1024};
    if (!pack || launch_bytes < (64ull << 20)) return Shape{4, 4, 32 * 1024, 16 * 1024};
    return Shape{5, 8, 64 * 1024, 32 * 1024};
}

template <bool PACK, bool PAGED, int U>
void launch_k(dim3 grid, hipStream_t stream, const SrcDesc &s, void *img, const SegTable &tab, int rowv, int rx_log2,
               int tpb, int rchunk)
{
    hipLaunchKernelGGL((kv_layout_kernel<PACK, PAGED, U>), grid, dim3(kThreads), 0, stream, s, (u32x4 *)img, tab, rowv,
                       rx_log2, tpb, rchunk);
}

template <bool PACK, bool PAGED>
void launch_u(int U, dim3 grid, hipStream_t stream, const SrcDesc &s, void *img, const SegTable &tab, int rowv,
              int rx_log2, int tpb, int rchunk)
{
    if (U == 8) launch_k<PACK, PAGED, 8>(grid, stream, s, img, tab, rowv, rx_log2, tpb, rchunk);
    else if (U == 2) launch_k<PACK, PAGED, 2>(grid, stream, s, img, tab, rowv, rx_log2, tpb, rchunk);
    else launch_k<PACK, PAGED, 4>(grid, stream, s, img, tab, rowv, rx_log2, tpb, rchunk);
}

template <bool PACK>
int launch(const kv_plan *p, const kv_view_t *v, const Seg *segs, int nseg, void *img, hipStream_t stream)
{
    const int rowv = (int)(p->row_bytes / 16);
    const bool paged = v->layout == KV_LAYOUT_PAGED;
    unsigned long long launch_bytes = 0;
    for (int i = 0; i < nseg; ++i) launch_bytes += (unsigned long long)segs[i].ntok * p->row_bytes;
    const Shape sh = pick_shape(PACK, paged, rowv, launch_bytes);
    int rx_log2 = 0;
    while ((1 << rx_log2) < rowv && rx_log2 < sh.rx_cap) ++rx_log2;
    const int TY = kThreads >> rx_log2;
    const int U = sh.unroll;
    const long long tile_bytes = sh.tile_bytes;
    // Tile = tpb token rows x rchunk row positions, about tile_bytes of extent.  A row wider than one sweep of
    // the workgroup is cut into chunks of row positions, and the tile gets more tokens instead, so that every
    // source head row it touches contributes at least run_bytes of consecutive tokens.
    const long long head_row_bytes = (long long)p->D * 2;
    long long want_tok = tile_bytes / (long long)p->row_bytes;
    if (rowv > (1 << rx_log2)) want_tok = std::max<long long>(want_tok, sh.run_bytes / head_row_bytes);
    int tpb = (int)std::max<long long>(1, want_tok);
    tpb = (tpb + TY * U - 1) / (TY * U) * (TY * U);
    const int RXv = 1 << rx_log2;
    long long chunk = std::max<long long>(RXv, tile_bytes / 16 / tpb);
    chunk = (chunk + RXv - 1) / RXv * RXv;
    const int rchunk = (int)std::min<long long>(chunk, (rowv + RXv - 1) / RXv * RXv);
    const unsigned n_rchunks = (unsigned)((rowv + rchunk - 1) / rchunk);
    const SrcDesc s = make_src(p, v);

    for (int g0 = 0; g0 < nseg; g0 += kMaxSegs) {
        const int n = std::min(kMaxSegs, nseg - g0);
        SegTable tab{};
        int max_tok = 0;
        for (int i = 0; i < n; ++i) {
            tab.seg[i] = segs[g0 + i];
            max_tok = std::max(max_tok, segs[g0 + i].ntok);
        }
        dim3 grid((unsigned)std::max(1, (max_tok + tpb - 1) / tpb), (unsigned)n, n_rchunks);
        if (paged) launch_u<PACK, true>(U, grid, stream, s, img, tab, rowv, rx_log2, tpb, rchunk);
        else launch_u<PACK, false>(U, grid, stream, s, img, tab, rowv, rx_log2, tpb, rchunk);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    }
    return KV_OK;
}

// Runs of the whole extent image of tensor (layer, which) placed at byte img_off of the image buffer: rows
// [0, len_b) of every sequence and the zero pad up to each (sub-)extent's end.
int whole_extent_segs(const kv_plan *p, const kv_view_t *v, int layer, int which, uint64_t img_off, std::vector<Seg> *segs)
{
    const uint64_t sec = (uint64_t)p->sector;
    const uint64_t image = p->tensor_blocks * sec;
    if (p->mode == KV_TOKEN_MAJOR) {
        const int len = v->seq_lens_host[0];
        for (int b = 0; b < p->B; ++b)
            if (v->seq_lens_host[b] != len) return KV_EINVAL;
        if (len < 0 || len > p->cap[0]) return KV_ERANGE;
        int rc = check_rows(p, v, -1, 0, len);
        if (rc != KV_OK) return rc;
        Seg s{};
        s.img_off = img_off / 16;
        s.b = -1; s.tok0 = 0; s.ntok = len; s.base = tensor_base(v, layer, which);
        s.pad_off = s.img_off + (uint64_t)len * p->row_bytes / 16;
        s.pad_vecs = (unsigned)((image - (uint64_t)len * p->row_bytes) / 16);
        segs->push_back(s);
        return KV_OK;
    }
    for (int b = 0; b < p->B; ++b) {
        const int len = v->seq_lens_host[b];
        if (len < 0 || len > p->cap[b]) return KV_ERANGE;
        int rc = check_rows(p, v, b, 0, len);
        if (rc != KV_OK) return rc;
        const uint64_t sub_bytes = kvb::round_up((uint64_t)p->cap[b] * p->row_bytes, sec);
        Seg s{};
        s.img_off = (img_off + p->seq_base[b] * sec) / 16;
        s.b = b; s.tok0 = 0; s.ntok = len; s.base = tensor_base(v, layer, which);
        s.pad_off = s.img_off + (uint64_t)len * p->row_bytes / 16;
        s.pad_vecs = (unsigned)((sub_bytes - (uint64_t)len * p->row_bytes) / 16);
        if (len > 0 || s.pad_vecs > 0) segs->push_back(s);
    }
    return KV_OK;
}

// Whole extent images of K and V of layers [layer_begin, layer_end), back to back in tensor-id order (layer
// ascending, K before V), in as few launches as the segment table allows: a small layer alone is too short a
// launch to reach HBM speed.
template <bool PACK>
int run_layers(const kv_plan *p, int layer_begin, int layer_end, const kv_view_t *v, void *img, size_t img_bytes,
               void *hip_stream)
{
    if (!p || !img || ((uintptr_t)img & 15)) return KV_EINVAL;
    if (layer_begin < 0 || layer_end > p->L || layer_begin > layer_end) return KV_ERANGE;
    if (p->row_bytes / 16 > (uint64_t)INT_MAX) return KV_EINVAL;
    const uint64_t image = p->tensor_blocks * (uint64_t)p->sector;
    if (img_bytes < (uint64_t)(layer_end - layer_begin) * 2 * image) return KV_ENOSPC;
    std::vector<Seg> segs;
    for (int l = layer_begin; l < layer_end; ++l) {
        int rc = check_view(p, v, l);
        if (rc != KV_OK) return rc;
        for (int w = 0; w < 2; ++w) {
            rc = whole_extent_segs(p, v, l, w, ((uint64_t)(l - layer_begin) * 2 + (uint64_t)w) * image, &segs);
            if (rc != KV_OK) return rc;
        }
    }
    if (!PACK)
        for (Seg &s : segs) s.pad_vecs = 0;
    if (segs.empty()) return KV_OK;
    return launch<PACK>(p, v, segs.data(), (int)segs.size(), img, (hipStream_t)hip_stream);
}

template <bool PACK>
int run(const kv_plan *p, int layer, int kind, const kv_view_t *v, int seq, int tok0, int ntok, void *img,
        size_t img_bytes, void *hip_stream)
{
    if (!p || !img) return KV_EINVAL;
    if (kind != KV_K && kind != KV_V && kind != KV_KV) return KV_EINVAL;
    if ((uintptr_t)img & 15) return KV_EINVAL;
    int rc = check_view(p, v, layer);
    if (rc != KV_OK) return rc;
    if (p->row_bytes / 16 > (uint64_t)INT_MAX) return KV_EINVAL;
    hipStream_t stream = (hipStream_t)hip_stream;
    const uint64_t sec = (uint64_t)p->sector;
    const int first = kind == KV_V ? 1 : 0, last = kind == KV_K ? 0 : 1;  // KV_KV: K image, then V image
    const uint64_t n_img = (uint64_t)(last - first + 1);

    std::vector<Seg> segs;
    if (seq == KV_SEQ_ALL && tok0 == 0 && ntok == 0) {
        // Whole extent image(s).
        const uint64_t image = p->tensor_blocks * sec;
        if (img_bytes < n_img * image) return KV_ENOSPC;
        for (int w = first; w <= last; ++w) {
            rc = whole_extent_segs(p, v, layer, w, (uint64_t)(w - first) * image, &segs);
            if (rc != KV_OK) return rc;
        }
    } else {
        kvb::RowRange r;
        rc = kvb::resolve_rows(p, seq, tok0, ntok, &r);
        if (rc != KV_OK) return rc;
        // with KV_KV the V range follows the K range at req_bytes
        if (img_bytes < (n_img - 1) * r.req_bytes + (PACK ? r.req_bytes : r.payload)) return KV_ENOSPC;
        const int b = p->mode == KV_TOKEN_MAJOR ? -1 : r.b;
        rc = check_rows(p, v, b, tok0, ntok);
        if (rc != KV_OK) return rc;
        for (int w = first; w <= last; ++w) {
            Seg s{};
            s.img_off = (uint64_t)(w - first) * r.req_bytes / 16;
            s.b = b; s.tok0 = tok0; s.ntok = ntok; s.base = tensor_base(v, layer, w);
            s.pad_off = s.img_off + r.payload / 16;
            s.pad_vecs = (unsigned)((r.req_bytes - r.payload) / 16);
            segs.push_back(s);
        }
    }
    if (!PACK)
        for (Seg &s : segs) s.pad_vecs = 0;
    if (segs.empty()) return KV_OK;
    return launch<PACK>(p, v, segs.data(), (int)segs.size(), img, stream);
}

}  // namespace

namespace kvb {
// The newest token row (row len_b - 1, len_b = v->seq_lens_host[b]) of every tensor of layers
// [layer_begin, layer_end) and every sequence, in extent order, packed back to back at dst in the order
// (layer, K then V, sequence) -- one row of all sequences per tensor in token-major mode.  No sector
// alignment rule and no padding: the decode append merges the rows into their sectors on the host.
// All tensors share launches (one run per row, up to 32 runs per launch).
int pack_last_rows(const kv_plan *p, const kv_view_t *v, int layer_begin, int layer_end, void *dst, size_t dst_bytes,
                   hipStream_t stream)
{
    if (!p || !dst || ((uintptr_t)dst & 15)) return KV_EINVAL;
    if (layer_begin < 0 || layer_end > p->L || layer_begin >= layer_end) return KV_ERANGE;
    const int nseq = p->mode == KV_TOKEN_MAJOR ? 1 : p->B;
    const uint64_t n_rows = (uint64_t)(layer_end - layer_begin) * 2 * (uint64_t)nseq;
    if (dst_bytes < n_rows * p->row_bytes) return KV_ENOSPC;
    std::vector<Seg> segs;
    segs.reserve((size_t)n_rows);
    for (int l = layer_begin; l < layer_end; ++l) {
        int rc = check_view(p, v, l);
        if (rc != KV_OK) return rc;
        for (int kind = 0; kind < 2; ++kind)
            for (int i = 0; i < nseq; ++i) {
                const int b = p->mode == KV_TOKEN_MAJOR ? -1 : i;
                const int len = v->seq_lens_host[i];
                if (len < 1 || len > p->cap[i]) return KV_ERANGE;
                rc = check_rows(p, v, b, len - 1, 1);
                if (rc != KV_OK) return rc;
                Seg s{};
                s.img_off = (uint64_t)segs.size() * (p->row_bytes / 16);
                s.b = b; s.tok0 = len - 1; s.ntok = 1; s.base = tensor_base(v, l, kind);
                segs.push_back(s);
            }
    }
    return launch<true>(p, v, segs.data(), (int)segs.size(), dst, stream);
}
}

extern "C" int kv_offload_pack(const kv_plan_t *plan, int layer, int kind, const kv_view_t *src, int seq, int tok0,
                               int ntok, void *dst_dev, size_t dst_bytes, void *hip_stream)
{
    return run<true>(plan, layer, kind, src, seq, tok0, ntok, dst_dev, dst_bytes, hip_stream);
}

extern "C" int kv_reload_unpack(const kv_plan_t *plan, int layer, int kind, const void *src_dev, size_t src_bytes,
                                const kv_view_t *dst, int seq, int tok0, int ntok, void *hip_stream)
{
    return run<false>(plan, layer, kind, dst, seq, tok0, ntok, const_cast<void *>(src_dev), src_bytes, hip_stream);
}

extern "C" int kv_offload_pack_layers(const kv_plan_t *plan, int layer_begin, int layer_end, const kv_view_t *src,
                                      void *dst_dev, size_t dst_bytes, void *hip_stream)
{
    return run_layers<true>(plan, layer_begin, layer_end, src, dst_dev, dst_bytes, hip_stream);
}

extern "C" int kv_reload_unpack_layers(const kv_plan_t *plan, int layer_begin, int layer_end, const void *src_dev,
                                       size_t src_bytes, const kv_view_t *dst, void *hip_stream)
{
    return run_layers<false>(plan, layer_begin, layer_end, dst, const_cast<void *>(src_dev), src_bytes, hip_stream);
}
