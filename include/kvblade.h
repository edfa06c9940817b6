/*
 * kvblade.h -- C ABI of the MI355X-native KV-cache offloading hot path.
 *
 * The library maps every per-layer K or V tensor to a contiguous, sector-aligned LBA extent,
 * marshals KV between the GPU's attention-side layout and extent byte order (pack on offload,
 * unpack on reload), moves extents between HBM and an LBA-addressed host region in chunks, and
 * runs split-K decode attention over the reloaded tensors.
 *
 * Conventions
 *  - Every function returns an int: KV_OK (0) or a negative KV_E* code.  Nothing throws or aborts.
 *  - "host" / "device" is stated for every pointer.  The library never takes ownership of a caller
 *    buffer.  Streams are hipStream_t passed as void* (NULL = the default stream).
 *  - Elements are 16-bit (fp16 or bf16); e = 2 bytes.  A tensor id is n = 2*layer + kind with
 *    KV_K = 0 before KV_V = 1, layers ascending (the id chain of Sec. IV-B "LBA Bind").
 *  - The storage tier is modelled: the direct path's namespace is a pinned host region whose byte
 *    offset is LBA * sector_bytes (region base = LBA 0); the page-cache path's files are byte
 *    offsets in one pageable host arena.
 */
#ifndef KVBLADE_H
#define KVBLADE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* ---- return codes ---- */
#define KV_OK 0
#define KV_EINVAL (-1) /* bad argument, dtype, shape, pointer kind */
#define KV_EALIGN (-2) /* an offset or size that must be a sector multiple is not */
#define KV_ERANGE (-3) /* token range, layer, sequence or buffer offset outside its bounds */
#define KV_ENOSPC (-4) /* LBA region, pageable arena, staging or workspace too small */
#define KV_EHIP (-5)   /* a HIP call failed; see kv_last_hip_error() */

#define KV_F16 0
#define KV_BF16 1

#define KV_TOKEN_MAJOR 0 /* one extent (S_cap, B*H, D) per tensor; uniform batch */
#define KV_PER_SEQ 1     /* per tensor: sub-extents (cap_b, H, D), each padded to a sector */

#define KV_PATH_DIRECT 0    /* Group 2: LBA extent in the pinned region */
#define KV_PATH_PAGECACHE 1 /* Group 1: byte range in the pageable arena */

#define KV_K 0
#define KV_V 1
#define KV_KV 2 /* pack / unpack only: K and V of the layer in one launch, V's image after K's */

#define KV_LAYOUT_BHSD 0  /* strided [B, H, S_alloc, D], d contiguous */
#define KV_LAYOUT_PAGED 1 /* block pool [n_pool, H, block_tokens, D] + block table */

#define KV_SEQ_ALL (-1)
#define KV_UNBOUNDED UINT64_MAX

#define KV_OUT_F32 0
#define KV_OUT_SAME 1 /* fp16 / bf16 as the plan's dtype, round to nearest even */

#define KV_DIR_OFFLOAD 0     /* pack -> D2H (-> memcpy into the arena) */
#define KV_DIR_RELOAD 1      /* (arena -> memcpy ->) H2D -> unpack */
#define KV_DIR_RELOAD_ATTN 2 /* RELOAD plus decode attention of each layer */

typedef struct kv_plan kv_plan_t; /* opaque; immutable after creation */

/*
 * Input of kv_layout_plan.  Alg. 1 (residency) needs L, the size of one K or V tensor and the
 * knob X; Eq. 3-6 (LBA bind) need the tensor byte size, the LBA size and the user-given first
 * start LBA.
 */
typedef struct kv_plan_desc {
    int32_t n_layers;     /* L >= 1 */
    int32_t n_kv_heads;   /* H >= 1 */
    int32_t n_q_heads;    /* H_q, a multiple of H */
    int32_t head_dim;     /* D; D*2 must be a multiple of 16 bytes */
    int32_t batch;        /* B >= 1 */
    int32_t dtype;        /* KV_F16 | KV_BF16 */
    int32_t sector_bytes; /* LBA size: 512 or 4096 */
    int32_t chunk_tokens; /* C: default token rows per chunk; C*row_bytes must be a sector multiple */
    int32_t extent_mode;  /* KV_TOKEN_MAJOR | KV_PER_SEQ */
    int32_t reserved;
    const int32_t *seq_cap;   /* host [B]: token capacity of each sequence's extent (copied);
                                 all equal in KV_TOKEN_MAJOR */
    uint64_t lba_start;       /* start LBA of the first direct-path tensor */
    uint64_t region_blocks;   /* sectors the LBA region holds, counted from LBA 0, or KV_UNBOUNDED */
    uint64_t pc_budget_bytes; /* X: bytes admitted to the page-cache path */
    uint64_t pageable_bytes;  /* bytes the pageable arena holds, or KV_UNBOUNDED */
} kv_plan_desc_t;

typedef struct kv_plan_info {
    int32_t n_layers, n_kv_heads, n_q_heads, head_dim, batch, dtype, sector_bytes, chunk_tokens, extent_mode;
    int32_t n_pagecache_layers;   /* n_1 of Alg. 1: layers [0, n_1) take the page-cache path */
    uint64_t row_bytes;           /* one token row of an extent: B*H*D*2 (token-major) or H*D*2 */
    uint64_t tensor_blocks;       /* n_blocks of every tensor (padded) */
    uint64_t tensor_payload_bytes;
    uint64_t region_bytes_needed;   /* (lba_start + sum of direct n_blocks) * sector_bytes */
    uint64_t pageable_bytes_needed; /* sum of page-cache-path n_blocks * sector_bytes */
} kv_plan_info_t;

/* One entry of the map M (Eq. 3-4) plus the page-cache-path twin. */
typedef struct kv_extent {
    int32_t path;       /* KV_PATH_* */
    int32_t reserved;
    uint64_t lba_start; /* direct path; 0 on the page-cache path */
    uint64_t n_blocks;
    uint64_t file_off;  /* byte offset in the pageable arena; 0 on the direct path */
    uint64_t bytes;     /* unpadded payload */
} kv_extent_t;

/* One per-chunk command (Eq. 9-11). */
typedef struct kv_cmd {
    uint64_t slba;    /* start LBA (direct) or sector index in the arena (page-cache path) */
    uint64_t buf_off; /* dbuf - buf_ptr: byte offset in the request's host/staging image */
    uint32_t nlb;     /* 0-based block count: nlb + 1 sectors move */
    uint32_t tok0;    /* first token row of the chunk */
    uint32_t ntok;    /* token rows in the chunk */
    uint32_t reserved;
} kv_cmd_t;

/* Attention-side KV buffers.  All arrays named "host" are read during the call only. */
typedef struct kv_view {
    int32_t layout;   /* KV_LAYOUT_* */
    int32_t n_layers; /* entries in k_layers / v_layers */
    void *const *k_layers; /* host array of device pointers, 16-byte aligned */
    void *const *v_layers; /* host array of device pointers, 16-byte aligned */
    uint64_t layer_bytes;  /* bytes addressable behind every k/v pointer (bounds check) */
    /* KV_LAYOUT_BHSD: strides in elements (multiples of 8); S_alloc rows exist per (b,h) */
    int64_t stride_b, stride_h, stride_s;
    int32_t s_alloc;
    /* KV_LAYOUT_PAGED */
    int32_t block_tokens;       /* tokens per block (16) */
    int32_t n_pool_blocks;      /* blocks in every pool */
    int32_t max_blocks_per_seq; /* row length of block_table */
    const int32_t *block_table; /* device [B, max_blocks_per_seq]; ids outside [0,n_pool) are skipped */
    /* valid tokens per sequence */
    const int32_t *seq_lens_host; /* host [B] */
    const int32_t *seq_lens_dev;  /* device [B] (decode attention reads it) */
    /* KV_LAYOUT_BHSD, decode attention only, optional: element offset (a multiple of 8) of sequence b's
     * first row, used instead of b*stride_b (sequences that are not equally spaced).  Both or neither. */
    const int64_t *seq_off_host; /* host [B] or NULL */
    const int64_t *seq_off_dev;  /* device [B] or NULL */
} kv_view_t;

typedef struct kv_attn_args {
    const void *const *q_layers; /* host array [n_layers] of device pointers, each [B, H_q, D] 16-bit */
    void *const *out_layers;     /* host array [n_layers] of device pointers, each [B, H_q, D] */
    int32_t out_dtype;           /* KV_OUT_* */
    int32_t n_splits;            /* 0 = choose */
} kv_attn_args_t;

#define KV_KERNEL_PACK 0
#define KV_KERNEL_UNPACK 1
#define KV_KERNEL_ATTN_PARTIAL 2
#define KV_KERNEL_ATTN_COMBINE 3

#define KV_PIPE_TIME_KERNELS 1u /* bracket every kernel with hipEvents and fill kernel_ms */
#define KV_PIPE_SERIALIZE 2u    /* run every stage (kernel, chunk transfer, host copy) to completion before
                                   the next starts: the no-overlap reference for the overlap fraction */

#define KV_COPY_AUTO 0   /* by measurement: the copy kernel for small commands (H2D up to 1 MiB, D2H below 1 MiB),
                            hipMemcpyAsync for larger ones (H2D on the SDMA engines: a copy kernel slows the other
                            wavefronts of the compute units it runs on) */
#define KV_COPY_MEMCPY 1 /* hipMemcpyAsync per chunk command */
#define KV_COPY_KERNEL 2 /* the library's copy kernel per chunk command */

#define KV_PIPE_ATTN_FROM_EXTENT 4u /* KV_DIR_RELOAD_ATTN, whole-extent spans only: decode
                                       attention reads the staged extent images directly (extent order is a
                                       strided [B,H,S,D] view) and nothing is unpacked: the view's K/V buffers
                                       are neither read nor written */
#define KV_PIPE_NO_PACING 8u /* queue every command as soon as the depth rule allows.  By default consecutive
                                commands are spaced by one command's own link time (at the link rate the library
                                measured on first use, or the best rate a run has sustained since), which keeps commands that share
                                the link from finishing together and leaving it idle while all are issued again */

#define KV_ORDER_CROSS 0 /* per layer all of K's commands, then V's: V's storage-side hop overlaps K's transfers */
#define KV_ORDER_INTRA 1 /* K's and V's commands alternate: both tensors' storage-side hops run side by side */

/* One chunk command as the pipeline ran it (kv_pipe_opts_t.trace), in issue order.  Times are the issuing
 * thread's clock in seconds since the call was entered: t_issue when the transfer was queued on its copy stream,
 * t_done when its completion was harvested (completions are harvested in issue order, each when the depth rule
 * or the final drain needs it, so t_done is an upper bound of the transfer's end). */
typedef struct kv_chunk_trace {
    uint64_t host_off;  /* byte offset in the LBA region (slba * sector) or in the arena */
    uint64_t bytes;     /* (nlb + 1) * sector */
    uint16_t layer;
    uint8_t kind;       /* KV_K | KV_V */
    uint8_t path;       /* KV_PATH_* */
    uint32_t reserved;
    double t_issue_s;
    double t_done_s;
} kv_chunk_trace_t;

typedef struct kv_pipe_opts {
    int32_t span_chunks;  /* chunks of one tensor per kernel launch and staging slot; 0 = whole extents: K and V
                             of a layer in one launch, and consecutive layers of one path together while their
                             images stay within 128 MiB (a launch must be tens of MiB to run at HBM speed) */
    int32_t host_workers; /* threads for the page-cache path's memcpy hop; 0 = default (8) */
    uint32_t flags;       /* KV_PIPE_* */
    int32_t copy_streams; /* streams the chunk commands rotate over, 1..4; 0 = default (3 for the copy kernel,
                             4 for hipMemcpyAsync); never more than depth */
    int32_t d2h_mode;     /* KV_COPY_* for offload transfers */
    int32_t h2d_mode;     /* KV_COPY_* for reload transfers */
    int32_t order_pagecache; /* KV_ORDER_* for page-cache-path layers (the two overlap strategies of Sec. IV-C) */
    int32_t order_direct;    /* KV_ORDER_* for direct-path layers */
    uint64_t max_cmd_bytes;  /* transfer-size limit of one command (MDTS of Eq. 7), 0 = none: a chunk larger than
                                align_down(max_cmd_bytes, sector) moves as several commands of at most that
                                size (Eq. 8-11 on the chunk), each counted against depth */
    void *caller_stream;     /* hipStream_t on which the caller produced (or still reads) the view's buffers, the
                                queries and the block table; NULL = the default stream.  The call's kernels are
                                launched on it, behind everything queued there; the copies on the library's own
                                streams follow them through events */
    kv_chunk_trace_t *trace; /* host, nullable: filled with the first trace_cap chunk commands of the call (the
                                queue-depth rule of Sec. IV-B "Data Flow" can be read off it: command c is issued
                                only after command c - depth was harvested); kv_pipe_stats_t.n_traced says how many */
    uint32_t trace_cap;
    uint32_t reserved;
} kv_pipe_opts_t;

typedef struct kv_pipe_stats {
    double wall_s;            /* call entry to drain */
    uint64_t bytes_direct;    /* bytes moved over the host link for direct-path tensors (with pad) */
    uint64_t bytes_pagecache; /* same for page-cache-path tensors */
    uint32_t n_chunks;        /* chunk commands issued */
    uint32_t n_spans;         /* staging slots filled */
    uint32_t max_in_flight;   /* largest number of chunk commands outstanding at once */
    double group_seconds[2];  /* per path group (0 page-cache, 1 direct): first command issued to last harvested */
    uint32_t kernel_launches[4];
    float kernel_ms[4];       /* summed event-bracketed time per kernel kind (KV_PIPE_TIME_KERNELS); the
                                 attention pair is bracketed together and reported under ATTN_PARTIAL */
    uint32_t lba_seq_breaks;  /* direct-path commands, in issue order, that do not start at the LBA where the
                                 previous one ended (Sec. IV-B "Sequential-LBA Placement": 0 for KV_ORDER_CROSS,
                                 the bind recurrence makes the whole stream one ascending run) */
    uint32_t n_traced;        /* entries written to kv_pipe_opts_t.trace */
    double host_copy_wait_s;  /* time the issuing thread waited for the page-cache path's memcpy hop (a bounce slot
                                 still being copied out of, or not yet filled): 0 when that hop keeps ahead of the link */
    double harvest_wait_s;    /* time the issuing thread waited for the oldest command's completion */
    double pace_GBps;         /* the link rate the issue pacing of this direction works from after this call
                                 (0 = none measured: commands are not paced) */
} kv_pipe_stats_t;

/* ------------------------------------------------------------------------------------------ */
/* Planner (host only, integer arithmetic; usable without a GPU)                              */
/* ------------------------------------------------------------------------------------------ */

/*
 * kv_layout_plan -- Alg. 1 (KPU residency planner) followed by the LBA bind of Eq. 3-6.
 *   n_1 = min(floor(X / (2*S_kpu)), L) with S_kpu = tensor_blocks*sector_bytes; layers [0,n_1) go to
 *   the page-cache path, the rest to the direct path.  Direct tensors get lba_start by the recurrence
 *   lba_start(n+1) = lba_start(n) + n_blocks(n) from desc->lba_start; n_blocks = ceil(bytes / sector)
 *   (zero padding; equal to Eq. 5 under the paper's alignment precondition).  Page-cache-path tensors
 *   get file_off by the same padded recurrence from 0.
 * desc: host.  *out: new plan, owned by the library, freed by kv_plan_destroy.
 * Errors: KV_EINVAL (shape/dtype/sector/mode, non-uniform caps in token-major), KV_EALIGN
 * (chunk_tokens*row_bytes not a sector multiple), KV_ENOSPC (region_blocks or pageable_bytes too small).
 */
int kv_layout_plan(const kv_plan_desc_t *desc, kv_plan_t **out);
void kv_plan_destroy(kv_plan_t *plan);

int kv_plan_info(const kv_plan_t *plan, kv_plan_info_t *out);
/* Map entry of tensor (layer, kind) -- Eq. 3-4.  KV_ERANGE for a bad layer, KV_EINVAL for a bad kind. */
int kv_plan_tensor(const kv_plan_t *plan, int layer, int kind, kv_extent_t *out);
/* Blocks before sequence seq's sub-extent inside a tensor's extent (0 in token-major mode). */
int kv_plan_seq_base(const kv_plan_t *plan, int seq, uint64_t *base_blocks);

/*
 * kv_plan_translate -- Alg. 2 for whole token rows: offset indices (tok0, 0, 0) in the target shape
 * (S_cap, B*H, D) [token-major; seq must be 0 or KV_SEQ_ALL] or (cap_seq, H, D) [per-sequence],
 * source shape (ntok, ., D).  *slba = first sector (LBA on the direct path, sector index in the
 * arena on the page-cache path); *req_bytes = ntok*row_bytes, rounded up to a sector multiple when
 * the range ends at the extent tail.
 * Errors: KV_EALIGN if tok0*row_bytes is not a sector multiple, or the range ends inside a sector
 * short of the tail; KV_ERANGE if tok0+ntok exceeds the capacity; KV_EINVAL for ntok <= 0, tok0 < 0.
 */
int kv_plan_translate(const kv_plan_t *plan, int layer, int kind, int seq, int tok0, int ntok,
                      uint64_t *slba, uint64_t *req_bytes);

/*
 * kv_plan_chunk_cmds -- Eq. 7-11 over the whole extent of (layer, kind) [token-major] or the whole
 * sub-extent of sequence seq [per-sequence], with chunk_bytes = chunk_tokens*row_bytes
 * (chunk_tokens = 0 takes the plan's).  Writes min(*n, cap) commands to out (host, caller-owned;
 * may be NULL with cap = 0 to query the count) and the total count to *n.  buf_off counts from the
 * first byte of that (sub-)extent.
 */
int kv_plan_chunk_cmds(const kv_plan_t *plan, int layer, int kind, int seq, int chunk_tokens,
                       kv_cmd_t *out, int cap, int *n);

/*
 * kv_plan_range_cmds -- Alg. 2 for token rows [tok0, tok0+ntok) of (layer, kind, seq) (same rules and
 * errors as kv_plan_translate), then Eq. 7-11 on that request with the chunk size taken from a device
 * transfer-size limit: chunk_size = align_down(mdts_bytes, sector) (Eq. 7; mdts_bytes = 0 takes the
 * plan's chunk_tokens*row_bytes; KV_EINVAL if the limit is below one sector).  buf_off counts from the
 * request's first byte; a command need not hold whole token rows: tok0/ntok name the rows its payload
 * bytes touch.  Output convention as kv_plan_chunk_cmds.
 */
int kv_plan_range_cmds(const kv_plan_t *plan, int layer, int kind, int seq, int tok0, int ntok,
                       uint64_t mdts_bytes, kv_cmd_t *out, int cap, int *n);

/* ------------------------------------------------------------------------------------------ */
/* Kernels (asynchronous on the given stream)                                                 */
/* ------------------------------------------------------------------------------------------ */

/*
 * kv_offload_pack -- attention-side layout -> extent byte order (row-major (S, B*H, D), Sec. IV-B
 * precondition and Alg. 2's row-major offset), for tensor (layer, kind).
 *   seq >= 0 (or 0 in token-major): token rows [tok0, tok0+ntok) of that (sub-)extent are written to
 *     dst_dev[0 ..); the byte count is kv_plan_translate's req_bytes (zero pad up to the sector
 *     boundary when the range reaches the tail), same error rules.
 *   seq = KV_SEQ_ALL (tok0 = ntok = 0): the whole extent image, n_blocks*sector bytes: rows
 *     [0, len_b) of every sequence (src->seq_lens_host, <= capacity; uniform in token-major) and
 *     zeros up to each (sub-)extent's end.
 *   kind = KV_KV moves both tensors of the layer in one launch: dst_dev holds K's bytes as above and
 *     V's bytes right after them (at n_blocks*sector, or at req_bytes for a row range).
 * src: host struct, device buffers; dst_dev: device, 16-byte aligned, dst_bytes >= bytes written
 * (else KV_ENOSPC).  Rows must exist in the source (BHSD: < s_alloc; paged: < seq_lens_host[b]) else
 * KV_ERANGE.  Nothing is launched on error.
 */
int kv_offload_pack(const kv_plan_t *plan, int layer, int kind, const kv_view_t *src, int seq,
                    int tok0, int ntok, void *dst_dev, size_t dst_bytes, void *hip_stream);

/*
 * kv_reload_unpack -- the inverse: bytes at src_dev[0 ..) in extent order -> the view's rows.  Only
 * the addressed valid token rows are written; pad bytes are ignored; every other element of the
 * view is left untouched.  Same arguments and errors as kv_offload_pack (src_bytes >= bytes read).
 */
int kv_reload_unpack(const kv_plan_t *plan, int layer, int kind, const void *src_dev, size_t src_bytes,
                     const kv_view_t *dst, int seq, int tok0, int ntok, void *hip_stream);

/*
 * kv_offload_pack_layers / kv_reload_unpack_layers -- the whole extent images (as kv_offload_pack with
 * seq = KV_SEQ_ALL) of K and V of layers [layer_begin, layer_end), back to back in tensor-id order (layer
 * ascending, K before V; the id chain of Sec. IV-B "LBA Bind"): tensor (l, kind) at byte
 * ((l - layer_begin)*2 + kind) * n_blocks*sector of dst_dev / src_dev.  All tensors share launches (a layer of a
 * few MiB alone is too short a launch to reach HBM speed).  Same rules and errors as the single-tensor calls;
 * dst_bytes / src_bytes >= (layer_end - layer_begin) * 2 * n_blocks*sector, else KV_ENOSPC.
 */
int kv_offload_pack_layers(const kv_plan_t *plan, int layer_begin, int layer_end, const kv_view_t *src,
                           void *dst_dev, size_t dst_bytes, void *hip_stream);
int kv_reload_unpack_layers(const kv_plan_t *plan, int layer_begin, int layer_end, const void *src_dev,
                            size_t src_bytes, const kv_view_t *dst, void *hip_stream);

/*
 * kv_decode_attn -- one decode-attention step of one layer over resident KV (Sec. II-A: similarity of
 * the query with the keys weights the values): out[b,hq,:] = softmax_j(q[b,hq,:].K[b,h,j,:] / sqrt(D))
 * V[b,h,j,:], j in [0, len_b), h = hq / (H_q/H); fp32 accumulation; split-K over tokens with a
 * combine pass.  len_b = kv->seq_lens_dev (device) with kv->seq_lens_host as its host mirror (both must
 * hold the same values: a batch whose sequences all have one length takes it from the host mirror at launch); a
 * sequence of length 0 yields zeros.  The wavefronts of a workgroup take their tiles on demand, so the order of the
 * fp32 sums, and with it the last bits of the result, can differ between two runs on the same inputs.
 * q: device [B,H_q,D] 16-bit, 16-byte aligned; out: device [B,H_q,D] fp32 or 16-bit (out_dtype);
 * workspace: device, >= kv_decode_attn_workspace() bytes (else KV_ENOSPC); n_splits 0 = choose.
 */
int kv_decode_attn(const kv_plan_t *plan, const kv_view_t *kv, int layer, const void *q, void *out,
                   int out_dtype, int n_splits, void *workspace, size_t ws_bytes, void *hip_stream);
/* Bytes of workspace kv_decode_attn needs for up to max_len tokens per sequence (n_splits 0 = enough
 * for whatever split count the library chooses at that length). */
size_t kv_decode_attn_workspace(const kv_plan_t *plan, int n_splits, int max_len);

/*
 * kv_decode_attn_splits -- the token splits kv_decode_attn makes for sequences of the given lengths (host [B]) and
 * the given n_splits argument (0 = choose): *n_splits_out = the split count the partials are laid out for (the
 * workspace holds batch * n_q_heads * that * (head_dim + 2) floats); first (host [B+1], nullable) = index of each
 * sequence's first split among the splits that hold tokens, first[B] = their number (workgroups launched per
 * query-head group); tokens (host [B], nullable) = token rows per split of each sequence.  Host arithmetic only.
 * A uniform batch, or a given n_splits, takes one split length for all sequences; a ragged batch of up to 64
 * sequences with n_splits = 0 gets per-sequence split lengths (whole 16-token tiles, 32 tokens for head_dim 64) such
 * that every workgroup reads about the same number of tokens (about one workgroup per compute unit in all).
 */
int kv_decode_attn_splits(const kv_plan_t *plan, const int32_t *seq_lens_host, int n_splits, int *n_splits_out,
                          int *first, int *tokens);

/*
 * kv_decode_attn_static -- kv_decode_attn for callers that cannot allocate device memory (code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, result and errors,
 * but no workspace argument.  The split partials live in an array of KV_ATTN_SCRATCH_BYTES that is part of
 * the library's device image (each GPU the library runs on holds it until the process ends); the call
 * allocates and frees nothing.  KV_ENOSPC if the partials of this call,
 * batch * n_q_heads * splits * (head_dim + 2) * 4 bytes, exceed the array (pass a smaller n_splits, or use
 * kv_decode_attn with a workspace).  Nothing in the array has to start at zero.  All calls on one GPU share
 * the array: calls that overlap on one GPU (different streams, or threads) race; calls on one stream do not.
 */
#define KV_ATTN_SCRATCH_BYTES (8u << 20)
int kv_decode_attn_static(const kv_plan_t *plan, const kv_view_t *kv, int layer, const void *q, void *out,
                          int out_dtype, int n_splits, void *hip_stream);

/* ------------------------------------------------------------------------------------------ */
/* Chunk pipeline (blocking; returns after the drain)                                         */
/* ------------------------------------------------------------------------------------------ */

/*
 * kv_pipeline_run -- move layers [layer_begin, layer_end) between the view and the storage model,
 * tensor by tensor (K then V), each as the per-chunk commands of Eq. 7-11, with at most `depth`
 * commands outstanding: a new command is issued only after the oldest has completed when `depth`
 * are in flight, and the call drains all of them before returning (Sec. IV-B "Data Flow").
 * Direct-path tensors move HBM <-> lba_region + slba*sector in two hops' worth of DMA only (Co-DMA:
 * the region is the buffer both sides address); page-cache-path tensors take the third hop, a host
 * memcpy between a pinned bounce ring and pageable + file_off (Sec. IV-B, 3-hop vs 2-hop).
 * KV_DIR_OFFLOAD: pack -> D2H.  KV_DIR_RELOAD: H2D -> unpack.  KV_DIR_RELOAD_ATTN: also decode
 * attention per layer into attn->out_layers[layer].
 * lba_region: pinned host memory (hipHostMalloc), region_bytes >= region_bytes_needed if any
 * direct-path layer is in range; pageable: ordinary host memory, pageable_bytes >=
 * pageable_bytes_needed if any page-cache-path layer is in range.  chunk_tokens 0 = the plan's.
 * The library owns its copy streams, events, staging slots, bounce ring and worker threads (created on
 * first use per plan, freed by kv_plan_destroy).  Calls on one plan must not overlap.
 * Stream order: the copies run on the library's streams, the kernels on opts->caller_stream (the default stream
 * when opts or the field is NULL), behind all work already queued there: KV rows, queries and block tables
 * written by kernels on that stream are complete before the first pack or attention launch reads them, and
 * kernels still reading the view finish before an unpack overwrites it.  Work on any other stream must be
 * complete (or ordered before caller_stream) when the call is made.  The call returns after its last kernel and
 * copy have finished (caller_stream is synchronised), so results are visible to every stream afterwards.
 * stats: host, may be NULL.
 */
int kv_pipeline_run(kv_plan_t *plan, int dir, int layer_begin, int layer_end, const kv_view_t *view,
                    void *lba_region, size_t region_bytes, void *pageable, size_t pageable_bytes,
                    int chunk_tokens, int depth, const kv_attn_args_t *attn, const kv_pipe_opts_t *opts,
                    kv_pipe_stats_t *stats);

/*
 * kv_append_tokens -- decode append (Sec. II-A: after each decode step the newly generated KV pair is
 * stored back; Sec. III: the 256 KB-class decode write).  For every tensor of layers
 * [layer_begin, layer_end) and every sequence b, token row len_b - 1 of the view (len_b =
 * view->seq_lens_host[b], which already counts the new token; 1 <= len_b <= capacity; uniform in
 * token-major mode) is packed on the GPU and written to its place in the extent: Alg. 2 with
 * i0 = len_b - 1 gives the byte range, the write carries the whole sectors that contain it.  A row that
 * starts inside a sector is merged with the sector's earlier bytes: the first append after an offload
 * reads that sector back (counted in n_rmw_reads), later appends use the image the library keeps;
 * bytes after the row up to the sector end are written as zeros (no later row exists yet).
 * Blocking.  lba_region / pageable as in kv_pipeline_run (pinned-ness is not required here).
 * The kept sector images are forgotten by kv_pipeline_run(KV_DIR_OFFLOAD), by kv_plan_trim, and whenever a call
 * names another lba_region or pageable base address than the one the images were taken from; they assume that
 * only this library writes the extents in between.
 * caller_stream: hipStream_t on which the new rows of the view were produced (NULL = the default stream); the
 * pack of the rows and their transfer are queued on it, behind everything already there.
 */
typedef struct kv_append_stats {
    uint32_t n_cmds;         /* write commands (one per tensor and sequence) */
    uint32_t n_rmw_reads;    /* sectors read back for read-modify-write */
    uint64_t blocks_written; /* sectors written */
} kv_append_stats_t;
int kv_append_tokens(kv_plan_t *plan, int layer_begin, int layer_end, const kv_view_t *view, void *lba_region,
                     size_t region_bytes, void *pageable, size_t pageable_bytes, void *caller_stream,
                     kv_append_stats_t *stats);

/*
 * kv_budget -- Eq. 1-2, the page-cache budget the knob X of kv_layout_plan is drawn from:
 * M* = min(M_avail, M_max - M_anon+shmem), B_pc = max(0, M* - N_threads * M_pin).  All in bytes, signed
 * (an over-committed limit gives a negative M* and B_pc = 0).  The caller samples the memory figures.
 */
int kv_budget(int64_t m_avail, int64_t m_max, int64_t m_anon_shmem, int32_t n_threads, int64_t m_pin,
              int64_t *m_star, int64_t *b_pc);

/*
 * kv_budget_sample -- the three memory figures of Eq. 1 (Sec. IV-A "Plan": system-wide and cgroup limits),
 * sampled now on this Linux host, in bytes: M_avail = MemAvailable of /proc/meminfo; M_max = the memory limit of
 * this process's cgroup (cgroup v2 memory.max, else v1 memory.limit_in_bytes), or MemTotal when there is no
 * limit; M_anon+shmem = anon + shmem of the cgroup's memory.stat (v1: rss + shmem) when it has a limit, else
 * AnonPages + Shmem of /proc/meminfo.  root = "" or NULL reads the real files; another root directory is
 * prepended to every path (for tests).  KV_EINVAL if /proc/meminfo cannot be read or lacks a field.
 */
int kv_budget_sample(const char *root, int64_t *m_avail, int64_t *m_max, int64_t *m_anon_shmem);

/*
 * kv_plan_trim -- context teardown (Sec. IV-B "Dataset Management--Deallocate"): for every tensor of
 * layers [layer_begin, layer_end) the range <lba_start, n_blocks> of the map M is given back.  In the
 * host-memory model a deallocated block reads back as zeros: the extent bytes in lba_region (direct
 * path) or pageable (page-cache path) are cleared.  *n_ranges, *n_blocks (nullable) count the ranges
 * and sectors released.  KV_ENOSPC if a buffer does not cover an extent; nothing is written then.
 * The sector images kv_append_tokens keeps for this plan are forgotten (the sectors now read zeros).
 */
int kv_plan_trim(const kv_plan_t *plan, int layer_begin, int layer_end, void *lba_region, size_t region_bytes,
                 void *pageable, size_t pageable_bytes, uint64_t *n_ranges, uint64_t *n_blocks);

/*
 * Adaptive strategy selection (Sec. IV-C): the first decode iteration is a warm-up and is not measured,
 * iteration 2 runs KV_ORDER_INTRA, iteration 3 KV_ORDER_CROSS; their throughputs are compared per path
 * group and the higher one is kept for every later iteration (a tie keeps KV_ORDER_INTRA).  The state is
 * a plain caller-owned struct.  kv_adapt_order gives the order a group must use in the coming iteration;
 * kv_adapt_update takes the stats of the iteration that has just run (bytes and group_seconds per group)
 * and advances the iteration count.  Groups: 0 = page-cache path, 1 = direct path.
 */
typedef struct kv_adapt {
    int32_t iteration;  /* decode iterations completed */
    int32_t chosen[2];  /* KV_ORDER_* once decided, else -1 */
    double gbps[2][2];  /* [group][order] throughput measured in iterations 2 and 3 */
} kv_adapt_t;
int kv_adapt_init(kv_adapt_t *a);
int kv_adapt_order(const kv_adapt_t *a, int group);
int kv_adapt_update(kv_adapt_t *a, const kv_pipe_stats_t *stats);

/* ------------------------------------------------------------------------------------------ */
int kv_last_hip_error(void);       /* hipError_t of the last KV_EHIP on this thread, else 0 */
const char *kv_strerror(int code); /* static string */
int kv_abi_version(void);
/* sizeof of the ABI struct number `which` as this library was compiled (0 kv_plan_desc_t, 1 kv_plan_info_t,
 * 2 kv_extent_t, 3 kv_cmd_t, 4 kv_view_t, 5 kv_attn_args_t, 6 kv_pipe_opts_t, 7 kv_pipe_stats_t,
 * 8 kv_append_stats_t, 9 kv_adapt_t, 10 kv_chunk_trace_t; 0 for any other number): lets a binding verify its own
 * layouts. */
size_t kv_abi_sizeof(int which);

#ifdef __cplusplus
}
#endif
#endif /* KVBLADE_H */
