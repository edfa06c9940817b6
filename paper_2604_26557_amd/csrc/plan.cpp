// Extent planner: residency split (Alg. 1), LBA bind (Eq. 3-6), token-range translation (Alg. 2)
// and per-chunk command parameters (Eq. 7-11).  Host only, unsigned 64-bit integer arithmetic.
#include "plan.hpp"

#include <algorithm>
#include <cstdio>
#include <cstring>
#include <fstream>
#include <new>
#include <sstream>
#include <string>

namespace kvb {

static thread_local int g_last_hip_error = 0;
void set_hip_error(int e) { g_last_hip_error = e; }

int resolve_rows(const kv_plan *p, int seq, int tok0, int ntok, RowRange *r)
{
    int b = 0;
    if (p->mode == KV_TOKEN_MAJOR) {
        if (seq != 0 && seq != KV_SEQ_ALL) return KV_ERANGE;
    } else {
        if (seq < 0 || seq >= p->B) return KV_ERANGE;
        b = seq;
    }
    if (tok0 < 0 || ntok <= 0) return KV_EINVAL;
    const uint64_t cap = (uint64_t)p->cap[b];
    if ((uint64_t)tok0 + (uint64_t)ntok > cap) return KV_ERANGE;
    const uint64_t sec = (uint64_t)p->sector;
    r->b = b;
    r->tok0 = tok0;
    r->ntok = ntok;
    r->sub_off = p->seq_base[b] * sec;
    r->sub_bytes = round_up(cap * p->row_bytes, sec);
    r->byte_off = (uint64_t)tok0 * p->row_bytes;
    r->payload = (uint64_t)ntok * p->row_bytes;
    if (r->byte_off % sec != 0) return KV_EALIGN;
    const bool at_tail = (uint64_t)tok0 + (uint64_t)ntok == cap;
    if (at_tail) {
        r->req_bytes = round_up(r->payload, sec);
    } else {
        if (r->payload % sec != 0) return KV_EALIGN;
        r->req_bytes = r->payload;
    }
    return KV_OK;
}

int chunk_cmds(const kv_plan *p, int layer, int kind, int seq, int chunk_tokens, std::vector<kv_cmd_t> *out)
{
    out->clear();
    if (layer < 0 || layer >= p->L) return KV_ERANGE;
    if (kind != KV_K && kind != KV_V) return KV_EINVAL;
    int b = 0;
    if (p->mode == KV_TOKEN_MAJOR) {
        if (seq != 0 && seq != KV_SEQ_ALL) return KV_ERANGE;
    } else {
        if (seq < 0 || seq >= p->B) return KV_ERANGE;
        b = seq;
    }
    const uint64_t C = chunk_tokens > 0 ? (uint64_t)chunk_tokens : (uint64_t)p->chunk_tokens;
    if (chunk_tokens < 0) return KV_EINVAL;
    const uint64_t sec = (uint64_t)p->sector;
    const uint64_t chunk_bytes = C * p->row_bytes;
    if (chunk_bytes % sec != 0) return KV_EALIGN;
    const uint64_t cap = (uint64_t)p->cap[b];
    if (cap == 0) return KV_OK;
    const kv_extent_t &e = p->ext[2 * layer + kind];
    // Alg. 2 at (0,0,0): the request is the whole (sub-)extent.
    const uint64_t first = (e.path == KV_PATH_DIRECT ? e.lba_start : e.file_off / sec) + p->seq_base[b];
    const uint64_t req_bytes = cap * p->row_bytes;
    // Eq. 8
    const uint64_t n_chunks = ceil_div(req_bytes, chunk_bytes);
    const uint64_t n_max_blocks = chunk_bytes / sec;
    const uint64_t n_total = ceil_div(req_bytes, sec);
    out->reserve(n_chunks);
    for (uint64_t N = 1; N <= n_chunks; ++N) {
        const uint64_t remains = n_total - (N - 1) * n_max_blocks;
        kv_cmd_t c;
        c.slba = first + (N - 1) * n_max_blocks;              // Eq. 9
        c.nlb = (uint32_t)(std::min(n_max_blocks, remains) - 1);  // Eq. 10, 0-based
        c.buf_off = (N - 1) * chunk_bytes;                    // Eq. 11
        c.tok0 = (uint32_t)((N - 1) * C);
        c.ntok = (uint32_t)std::min(C, cap - (N - 1) * C);
        c.reserved = 0;
        out->push_back(c);
    }
    return KV_OK;
}

int range_cmds(const kv_plan *p, int layer, int kind, int seq, int tok0, int ntok, uint64_t mdts_bytes,
               std::vector<kv_cmd_t> *out)
{
    out->clear();
    if (layer < 0 || layer >= p->L) return KV_ERANGE;
    if (kind != KV_K && kind != KV_V) return KV_EINVAL;
    RowRange r;
    int rc = resolve_rows(p, seq, tok0, ntok, &r);  // Alg. 2: the request <slba*, req_bytes>
    if (rc != KV_OK) return rc;
    const uint64_t sec = (uint64_t)p->sector;
    // Eq. 7: the largest sector multiple within the transfer-size limit
    const uint64_t chunk_bytes = mdts_bytes == 0 ? (uint64_t)p->chunk_tokens * p->row_bytes : mdts_bytes / sec * sec;
    if (chunk_bytes == 0) return KV_EINVAL;
    const kv_extent_t &e = p->ext[2 * layer + kind];
    const uint64_t first = (e.path == KV_PATH_DIRECT ? e.lba_start : e.file_off / sec) + (r.sub_off + r.byte_off) / sec;
    const uint64_t n_chunks = ceil_div(r.req_bytes, chunk_bytes);  // Eq. 8
    const uint64_t n_max_blocks = chunk_bytes / sec;
    const uint64_t n_total = r.req_bytes / sec;
    out->reserve(n_chunks);
    for (uint64_t N = 1; N <= n_chunks; ++N) {
        const uint64_t remains = n_total - (N - 1) * n_max_blocks;
        const uint64_t blocks = std::min(n_max_blocks, remains);
        kv_cmd_t c;
        c.slba = first + (N - 1) * n_max_blocks;  // Eq. 9
        c.nlb = (uint32_t)(blocks - 1);           // Eq. 10, 0-based
        c.buf_off = (N - 1) * chunk_bytes;        // Eq. 11
        // token rows the command's payload bytes touch
        const uint64_t b0 = c.buf_off, b1 = std::min(c.buf_off + blocks * sec, r.payload);
        c.tok0 = (uint32_t)((uint64_t)tok0 + b0 / p->row_bytes);
        c.ntok = b1 > b0 ? (uint32_t)((b1 - 1) / p->row_bytes - b0 / p->row_bytes + 1) : 0;
        c.reserved = 0;
        out->push_back(c);
    }
    return KV_OK;
}

}  // namespace kvb

using namespace kvb;

extern "C" int kv_layout_plan(const kv_plan_desc_t *d, kv_plan_t **out)
{
    if (!d || !out) return KV_EINVAL;
    *out = nullptr;
    if (d->n_layers < 1 || d->n_kv_heads < 1 || d->n_q_heads < 1 || d->head_dim < 1 || d->batch < 1)
        return KV_EINVAL;
    if (d->n_q_heads % d->n_kv_heads != 0) return KV_EINVAL;
    if (d->dtype != KV_F16 && d->dtype != KV_BF16) return KV_EINVAL;
    if (d->sector_bytes != 512 && d->sector_bytes != 4096) return KV_EINVAL;
    if (d->extent_mode != KV_TOKEN_MAJOR && d->extent_mode != KV_PER_SEQ) return KV_EINVAL;
    if ((d->head_dim * 2) % 16 != 0) return KV_EINVAL;
    if (d->chunk_tokens < 1 || !d->seq_cap) return KV_EINVAL;
    for (int b = 0; b < d->batch; ++b) {
        if (d->seq_cap[b] < 0) return KV_EINVAL;
        if (d->extent_mode == KV_TOKEN_MAJOR && d->seq_cap[b] != d->seq_cap[0]) return KV_EINVAL;
    }

    kv_plan *p = new (std::nothrow) kv_plan();
    if (!p) return KV_EINVAL;
    p->L = d->n_layers; p->H = d->n_kv_heads; p->Hq = d->n_q_heads; p->D = d->head_dim; p->B = d->batch;
    p->dtype = d->dtype; p->sector = d->sector_bytes; p->chunk_tokens = d->chunk_tokens; p->mode = d->extent_mode;
    p->cap.assign(d->seq_cap, d->seq_cap + d->batch);
    p->lba_start_first = d->lba_start;
    const uint64_t sec = (uint64_t)p->sector, e = 2;

    // Extent size of one tensor.
    p->seq_base.assign(p->B, 0);
    if (p->mode == KV_TOKEN_MAJOR) {
        p->row_bytes = (uint64_t)p->B * p->H * p->D * e;
        p->payload_bytes = (uint64_t)p->cap[0] * p->row_bytes;
        p->tensor_blocks = ceil_div(p->payload_bytes, sec);
    } else {
        p->row_bytes = (uint64_t)p->H * p->D * e;
        uint64_t acc = 0, pay = 0;
        for (int b = 0; b < p->B; ++b) {
            p->seq_base[b] = acc;
            acc += ceil_div((uint64_t)p->cap[b] * p->row_bytes, sec);
            pay += (uint64_t)p->cap[b] * p->row_bytes;
        }
        p->tensor_blocks = acc;
        p->payload_bytes = pay;
    }
    if (p->tensor_blocks == 0) { delete p; return KV_EINVAL; }
    if (((uint64_t)p->chunk_tokens * p->row_bytes) % sec != 0) { delete p; return KV_EALIGN; }

    // Alg. 1: how many (K,V) pairs fit in X; the first n1 layers take the page-cache path.
    const uint64_t s_kpu = p->tensor_blocks * sec;
    const uint64_t fit = d->pc_budget_bytes / (2 * s_kpu);
    p->n1 = (int32_t)std::min<uint64_t>(fit, (uint64_t)p->L);

    // Eq. 3-6: walk tensors in id order, one running LBA for the direct path, one running byte
    // offset for the page-cache path.
    p->ext.resize(2 * (size_t)p->L);
    uint64_t lba = d->lba_start, off = 0;
    for (int layer = 0; layer < p->L; ++layer) {
        for (int kind = 0; kind < 2; ++kind) {
            kv_extent_t &x = p->ext[2 * layer + kind];
            x.reserved = 0;
            x.n_blocks = p->tensor_blocks;
            x.bytes = p->payload_bytes;
            if (layer < p->n1) {
                x.path = KV_PATH_PAGECACHE; x.lba_start = 0; x.file_off = off;
                off += p->tensor_blocks * sec;
            } else {
                x.path = KV_PATH_DIRECT; x.lba_start = lba; x.file_off = 0;
                lba += p->tensor_blocks;
            }
        }
    }
    const bool any_direct = p->n1 < p->L;
    p->region_bytes_needed = any_direct ? lba * sec : 0;
    p->pageable_bytes_needed = off;
    if (any_direct && d->region_blocks != KV_UNBOUNDED && lba > d->region_blocks) { delete p; return KV_ENOSPC; }
    if (d->pageable_bytes != KV_UNBOUNDED && off > d->pageable_bytes) { delete p; return KV_ENOSPC; }
    *out = p;
    return KV_OK;
}

extern "C" int kv_plan_info(const kv_plan_t *p, kv_plan_info_t *o)
{
    if (!p || !o) return KV_EINVAL;
    o->n_layers = p->L; o->n_kv_heads = p->H; o->n_q_heads = p->Hq; o->head_dim = p->D; o->batch = p->B;
    o->dtype = p->dtype; o->sector_bytes = p->sector; o->chunk_tokens = p->chunk_tokens; o->extent_mode = p->mode;
    o->n_pagecache_layers = p->n1;
    o->row_bytes = p->row_bytes;
    o->tensor_blocks = p->tensor_blocks;
    o->tensor_payload_bytes = p->payload_bytes;
    o->region_bytes_needed = p->region_bytes_needed;
    o->pageable_bytes_needed = p->pageable_bytes_needed;
    return KV_OK;
}

extern "C" int kv_plan_tensor(const kv_plan_t *p, int layer, int kind, kv_extent_t *o)
{
    if (!p || !o) return KV_EINVAL;
    if (layer < 0 || layer >= p->L) return KV_ERANGE;
    if (kind != KV_K && kind != KV_V) return KV_EINVAL;
    *o = p->ext[2 * layer + kind];
    return KV_OK;
}

extern "C" int kv_plan_seq_base(const kv_plan_t *p, int seq, uint64_t *base)
{
    if (!p || !base) return KV_EINVAL;
    if (seq < 0 || seq >= p->B) return KV_ERANGE;
    *base = p->seq_base[seq];
    return KV_OK;
}

extern "C" int kv_plan_translate(const kv_plan_t *p, int layer, int kind, int seq, int tok0, int ntok,
                                 uint64_t *slba, uint64_t *req_bytes)
{
    if (!p || !slba || !req_bytes) return KV_EINVAL;
    if (layer < 0 || layer >= p->L) return KV_ERANGE;
    if (kind != KV_K && kind != KV_V) return KV_EINVAL;
    RowRange r;
    int rc = resolve_rows(p, seq, tok0, ntok, &r);
    if (rc != KV_OK) return rc;
    const kv_extent_t &e = p->ext[2 * layer + kind];
    const uint64_t sec = (uint64_t)p->sector;
    const uint64_t first = e.path == KV_PATH_DIRECT ? e.lba_start : e.file_off / sec;
    *slba = first + (r.sub_off + r.byte_off) / sec;
    *req_bytes = r.req_bytes;
    return KV_OK;
}

extern "C" int kv_plan_chunk_cmds(const kv_plan_t *p, int layer, int kind, int seq, int chunk_tokens,
                                  kv_cmd_t *out, int cap, int *n)
{
    if (!p || !n || cap < 0 || (cap > 0 && !out)) return KV_EINVAL;
    std::vector<kv_cmd_t> v;
    int rc = chunk_cmds(p, layer, kind, seq, chunk_tokens, &v);
    if (rc != KV_OK) return rc;
    *n = (int)v.size();
    for (int i = 0; i < (int)v.size() && i < cap; ++i) out[i] = v[i];
    return KV_OK;
}

extern "C" int kv_plan_range_cmds(const kv_plan_t *p, int layer, int kind, int seq, int tok0, int ntok,
                                  uint64_t mdts_bytes, kv_cmd_t *out, int cap, int *n)
{
    if (!p || !n || cap < 0 || (cap > 0 && !out)) return KV_EINVAL;
    std::vector<kv_cmd_t> v;
    int rc = range_cmds(p, layer, kind, seq, tok0, ntok, mdts_bytes, &v);
    if (rc != KV_OK) return rc;
    *n = (int)v.size();
    for (int i = 0; i < (int)v.size() && i < cap; ++i) out[i] = v[i];
    return KV_OK;
}

extern "C" int kv_budget(int64_t m_avail, int64_t m_max, int64_t m_anon_shmem, int32_t n_threads, int64_t m_pin,
                         int64_t *m_star, int64_t *b_pc)
{
    if (!m_star || !b_pc || n_threads < 0 || m_pin < 0) return KV_EINVAL;
    const int64_t limit = m_max - m_anon_shmem;           // Eq. 1
    *m_star = std::min(m_avail, limit);
    const int64_t left = *m_star - (int64_t)n_threads * m_pin;  // Eq. 2
    *b_pc = std::max<int64_t>(0, left);
    return KV_OK;
}

namespace {

// value of "key" in a file of "key value [unit]" lines (a trailing ':' on the key is ignored); -1 if absent
int64_t file_field(const std::string &path, const std::string &key)
{
    std::ifstream f(path);
    std::string line;
    while (std::getline(f, line)) {
        std::istringstream ss(line);
        std::string k;
        long long v;
        if (!(ss >> k >> v)) continue;
        if (!k.empty() && k.back() == ':') k.pop_back();
        if (k == key) return (int64_t)v;
    }
    return -1;
}

// first token of a one-line file: a number, or "max" (-> -2); -1 if the file cannot be read
int64_t file_number(const std::string &path)
{
    std::ifstream f(path);
    std::string tok;
    if (!(f >> tok)) return -1;
    if (tok == "max") return -2;
    char *end = nullptr;
    const long long v = std::strtoll(tok.c_str(), &end, 10);
    return end && *end == 0 ? (int64_t)v : -1;
}

// this process's cgroup directory: v2 line "0::/path" -> /sys/fs/cgroup/path; v1 line "N:memory:/path" ->
// /sys/fs/cgroup/memory/path
void cgroup_dirs(const std::string &root, std::string *v2, std::string *v1)
{
    std::ifstream f(root + "/proc/self/cgroup");
    std::string line;
    *v2 = root + "/sys/fs/cgroup";
    *v1 = root + "/sys/fs/cgroup/memory";
    while (std::getline(f, line)) {
        const size_t a = line.find(':'), b = a == std::string::npos ? a : line.find(':', a + 1);
        if (b == std::string::npos) continue;
        const std::string ctrl = line.substr(a + 1, b - a - 1), path = line.substr(b + 1);
        if (ctrl.empty()) *v2 = root + "/sys/fs/cgroup" + (path == "/" ? "" : path);
        else if (("," + ctrl + ",").find(",memory,") != std::string::npos) *v1 = root + "/sys/fs/cgroup/memory" + (path == "/" ? "" : path);
    }
}

}  // namespace

extern "C" int kv_budget_sample(const char *root_c, int64_t *m_avail, int64_t *m_max, int64_t *m_anon_shmem)
{
    if (!m_avail || !m_max || !m_anon_shmem) return KV_EINVAL;
    const std::string root = root_c ? root_c : "";
    const std::string meminfo = root + "/proc/meminfo";
    const int64_t avail = file_field(meminfo, "MemAvailable"), total = file_field(meminfo, "MemTotal");
    const int64_t anon = file_field(meminfo, "AnonPages"), shmem = file_field(meminfo, "Shmem");
    if (avail < 0 || total < 0 || anon < 0 || shmem < 0) return KV_EINVAL;
    *m_avail = avail * 1024;   // /proc/meminfo counts KiB
    *m_max = total * 1024;
    *m_anon_shmem = (anon + shmem) * 1024;

    std::string v2, v1;
    cgroup_dirs(root, &v2, &v1);
    int64_t limit = file_number(v2 + "/memory.max");
    bool is_v2 = true;
    if (limit == -1) { limit = file_number(v1 + "/memory.limit_in_bytes"); is_v2 = false; }
    if (limit >= 0 && limit < *m_max) {  // a real limit below the machine's memory
        *m_max = limit;
        const std::string stat = (is_v2 ? v2 : v1) + "/memory.stat";
        const int64_t a = file_field(stat, is_v2 ? "anon" : "rss"), s = file_field(stat, "shmem");
        if (a >= 0 && s >= 0) *m_anon_shmem = a + s;   // memory.stat counts bytes
    }
    return KV_OK;
}

extern "C" int kv_plan_trim(const kv_plan_t *p, int layer_begin, int layer_end, void *lba_region, size_t region_bytes,
                            void *pageable, size_t pageable_bytes, uint64_t *n_ranges, uint64_t *n_blocks)
{
    if (!p) return KV_EINVAL;
    if (layer_begin < 0 || layer_end > p->L || layer_begin > layer_end) return KV_ERANGE;
    const uint64_t sec = (uint64_t)p->sector;
    uint64_t ranges = 0, blocks = 0;
    for (int pass = 0; pass < 2; ++pass) {  // validate everything first, then write
        for (int l = layer_begin; l < layer_end; ++l) {
            for (int kind = 0; kind < 2; ++kind) {
                const kv_extent_t &e = p->ext[2 * l + kind];      // the entry of M (Eq. 3-4)
                const bool direct = e.path == KV_PATH_DIRECT;
                char *base = (char *)(direct ? lba_region : pageable);
                const uint64_t cap = direct ? region_bytes : pageable_bytes;
                const uint64_t off = extent_host_off(p, 2 * l + kind);
                if (pass == 0) {
                    if (!base) return KV_EINVAL;
                    if (off + e.n_blocks * sec > cap) return KV_ENOSPC;
                } else {
                    std::memset(base + off, 0, e.n_blocks * sec);  // a deallocated block reads back as zeros
                    ++ranges;
                    blocks += e.n_blocks;
                }
            }
        }
    }
    if (p->pipe && ranges > 0) kvb::forget_tail_images(p->pipe);  // those sectors now read zeros
    if (n_ranges) *n_ranges = ranges;
    if (n_blocks) *n_blocks = blocks;
    return KV_OK;
}

extern "C" int kv_adapt_init(kv_adapt_t *a)
{
    if (!a) return KV_EINVAL;
    a->iteration = 0;
    for (int g = 0; g < 2; ++g) {
        a->chosen[g] = -1;
        a->gbps[g][0] = a->gbps[g][1] = 0.0;
    }
    return KV_OK;
}

extern "C" int kv_adapt_order(const kv_adapt_t *a, int group)
{
    if (!a || group < 0 || group > 1) return KV_EINVAL;
    if (a->iteration <= 1) return KV_ORDER_INTRA;  // warm-up, then the measured overlap-intra iteration
    if (a->iteration == 2) return KV_ORDER_CROSS;  // the measured overlap-cross iteration
    return a->chosen[group] >= 0 ? a->chosen[group] : KV_ORDER_INTRA;
}

extern "C" int kv_adapt_update(kv_adapt_t *a, const kv_pipe_stats_t *st)
{
    if (!a || !st) return KV_EINVAL;
    const uint64_t bytes[2] = {st->bytes_pagecache, st->bytes_direct};
    const int it = a->iteration;  // 0-based index of the iteration that has just run
    if (it == 1 || it == 2) {
        const int order = it == 1 ? KV_ORDER_INTRA : KV_ORDER_CROSS;
        for (int g = 0; g < 2; ++g)
            a->gbps[g][order] = st->group_seconds[g] > 0 ? (double)bytes[g] / st->group_seconds[g] / 1e9 : 0.0;
    }
    if (it == 2)
        for (int g = 0; g < 2; ++g)
            a->chosen[g] = a->gbps[g][KV_ORDER_CROSS] > a->gbps[g][KV_ORDER_INTRA] ? KV_ORDER_CROSS : KV_ORDER_INTRA;
    a->iteration = it + 1;
    return KV_OK;
}

extern "C" size_t kv_abi_sizeof(int which)
{
    switch (which) {
    case 0: return sizeof(kv_plan_desc_t);
    case 1: return sizeof(kv_plan_info_t);
    case 2: return sizeof(kv_extent_t);
    case 3: return sizeof(kv_cmd_t);
    case 4: return sizeof(kv_view_t);
    case 5: return sizeof(kv_attn_args_t);
    case 6: return sizeof(kv_pipe_opts_t);
    case 7: return sizeof(kv_pipe_stats_t);
    case 8: return sizeof(kv_append_stats_t);
    case 9: return sizeof(kv_adapt_t);
    case 10: return sizeof(kv_chunk_trace_t);
    default: return 0;
    }
}

extern "C" int kv_last_hip_error(void) { return g_last_hip_error; }

extern "C" const char *kv_strerror(int code)
{
    switch (code) {
    case KV_OK: return "ok";
    case KV_EINVAL: return "invalid argument";
    case KV_EALIGN: return "offset or size is not a sector multiple";
    case KV_ERANGE: return "index or range out of bounds";
    case KV_ENOSPC: return "buffer too small";
    case KV_EHIP: return "HIP call failed";
    default: return "unknown error";
    }
}

extern "C" int kv_abi_version(void) { return 4; }
