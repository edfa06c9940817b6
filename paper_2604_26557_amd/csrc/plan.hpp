// Internal definition of the opaque plan object and the host-side range arithmetic shared by the
// planner accessors, the kernel launchers and the pipeline.
#pragma once

#include <hip/hip_runtime_api.h>

#include <cstdint>
#include <vector>

#include "kvblade.h"

struct kv_pipeline;  // pipeline.hip

struct kv_plan {
    int32_t L, H, Hq, D, B, dtype, sector, chunk_tokens, mode;
    std::vector<int32_t> cap;        // [B] token capacity of each sequence's (sub-)extent
    std::vector<uint64_t> seq_base;  // [B] blocks before sequence b inside a tensor's extent
    uint64_t row_bytes;              // one token row of an extent
    uint64_t tensor_blocks;          // n_blocks of every tensor
    uint64_t payload_bytes;          // unpadded bytes of every tensor
    int32_t n1;                      // page-cache-path layers (prefix)
    std::vector<kv_extent_t> ext;    // [2L] map M and its page-cache-path twin
    uint64_t lba_start_first;
    uint64_t region_bytes_needed, pageable_bytes_needed;
    kv_pipeline *pipe = nullptr;     // created on first kv_pipeline_run
};

namespace kvb {

// A run of whole token rows inside one (sub-)extent, resolved to bytes.
struct RowRange {
    int b;                  // sequence (0 in token-major mode)
    int tok0, ntok;
    uint64_t sub_off;       // byte offset of the (sub-)extent inside the tensor's extent
    uint64_t byte_off;      // byte offset of row tok0 inside the (sub-)extent
    uint64_t payload;       // ntok * row_bytes
    uint64_t req_bytes;     // payload, rounded up to a sector when the range reaches the tail
    uint64_t sub_bytes;     // padded size of the (sub-)extent
};

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline uint64_t round_up(uint64_t a, uint64_t b) { return ceil_div(a, b) * b; }

// Validates (seq, tok0, ntok) against the plan (alignment reading: a range starts on a sector
// boundary and ends on one unless it ends at the extent tail) and fills r.
int resolve_rows(const kv_plan *p, int seq, int tok0, int ntok, RowRange *r);

// Byte offset of tensor n's extent inside its host buffer (region base or arena base).
inline uint64_t extent_host_off(const kv_plan *p, int n)
{
    const kv_extent_t &e = p->ext[n];
    return e.path == KV_PATH_DIRECT ? e.lba_start * (uint64_t)p->sector : e.file_off;
}

int chunk_cmds(const kv_plan *p, int layer, int kind, int seq, int chunk_tokens, std::vector<kv_cmd_t> *out);
int range_cmds(const kv_plan *p, int layer, int kind, int seq, int tok0, int ntok, uint64_t mdts_bytes,
               std::vector<kv_cmd_t> *out);

void set_hip_error(int e);

// pipeline.hip: the decode append's kept tail-sector images are no longer valid (extents rewritten or trimmed)
void forget_tail_images(kv_pipeline *pipe);

// layout_kernels.hip
int pack_last_rows(const kv_plan *p, const kv_view_t *v, int layer_begin, int layer_end, void *dst, size_t dst_bytes,
                   hipStream_t stream);

}  // namespace kvb
