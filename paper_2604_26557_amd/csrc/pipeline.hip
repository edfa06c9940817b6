// Chunk pipeline: moves KV tensors between HBM and the storage model as the per-chunk commands of
// Eq. 7-11, overlapping the GPU marshalling kernels with host-link DMA and, on the page-cache path,
// with the host memcpy hop (Sec. IV-B "Co-DMA" / "Data Flow"; 3-hop vs 2-hop paths).
//
// Two granularities are kept apart on purpose:
//  * DMA runs per chunk command; at most `depth` commands are outstanding (the queue-depth rule:
//    when `depth` are in flight the oldest is harvested before the next is issued; a final drain
//    collects the rest).  hipEvents play the role of completion-queue entries.
//  * Kernels run per span = a whole tensor, K and V of a layer together while the pair is at most
//    256 MiB, or several small layers of one path together, by default (HBM is large, so staging whole
//    extents costs nothing and the pack / unpack launches are big enough to run at HBM speed), or every
//    `span_chunks` chunks of one tensor on request.
// Streams: the caller's own for kernels and up to four for copies (chunk c goes to copy stream c mod n, so the
// start-up and tail of one transfer hide behind the next); events order pack -> D2H and
// H2D -> unpack -> attention and guard staging-slot reuse.  All streams keep the default priority.
// Measured on MI355X (PCIe Gen5 x16, ~56.7 GB/s with 64 MiB copies): small commands (H2D up to 1 MiB, D2H
// below 1 MiB) move fastest as this file's own copy kernel over three streams (its completion event rides on
// the dispatch: the runtime's per-command cost dominates copies of a few hundred KiB); larger ones go through
// hipMemcpyAsync over up to four streams.  Both engines are options.  Commands are issued no closer together
// than one command's own link time, which keeps them from finishing in lockstep.
#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <algorithm>
#include <atomic>
#include <chrono>
#include <cstring>
#include <functional>
#include <mutex>
#include <thread>
#include <vector>

#include "pacer.hpp"
#include "workers.hpp"
#include "plan.hpp"

namespace {

#define KV_HIP(call)                                       \
    do {                                                   \
        hipError_t e_ = (call);                            \
        if (e_ != hipSuccess) {                            \
            kvb::set_hip_error((int)e_);                   \
            return KV_EHIP;                                \
        }                                                  \
    } while (0)

// Inside the issue loops: record the error and leave the loop so that the drain still runs.
#define KV_HIP_BRK(call)                                   \
    {                                                      \
        hipError_t e_ = (call);                            \
        if (e_ != hipSuccess) {                            \
            kvb::set_hip_error((int)e_);                   \
            err = KV_EHIP;                                 \
            break;                                         \
        }                                                  \
    }

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// One chunk command executed by the shader engines: 16-byte vectors, four loads in flight per lane.
// Either side may be pinned host memory (mapped into the device address space at its host address).
__global__ void __launch_bounds__(256)
kv_chunk_copy_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst, size_t nvec)
{
    constexpr int U = 4;
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (; i + (U - 1) * stride < nvec; i += U * stride) {
        u32x4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) v[u] = __builtin_nontemporal_load(src + i + u * stride);
#pragma unroll
        for (int u = 0; u < U; ++u) __builtin_nontemporal_store(v[u], dst + i + u * stride);
    }
    for (; i < nvec; i += stride) dst[i] = src[i];
}

constexpr int kMaxCopyStreams = 4;

// Same without leaving the loop (for use inside nested loops; the caller tests err).
#define KV_HIP_SET(call)                                   \
    {                                                      \
        hipError_t e_ = (call);                            \
        if (e_ != hipSuccess) {                            \
            kvb::set_hip_error((int)e_);                   \
            err = KV_EHIP;                                 \
        }                                                  \
    }

struct Chunk {
    uint64_t host_off;   // byte offset in the LBA region (slba * sector) or in the arena
    uint64_t stage_off;  // byte offset inside the span's staging slot
    uint64_t bytes;      // (nlb + 1) * sector
    int span;
    bool first, last;    // first / last chunk of its span
    int layer, kind;     // the tensor the command belongs to
};

struct Span {
    int layer, kind, seq, tok0, ntok;  // seq = KV_SEQ_ALL: whole tensor
    uint64_t bytes;                    // image bytes
    int path;
    bool last_of_layer;
    int n_layers;                      // > 1: whole K and V images of layers [layer, layer + n_layers), one launch
};

struct Schedule {
    std::vector<Span> spans;    // kernel launches / staging-slot fills, in issue order
    std::vector<Chunk> chunks;  // chunk commands, in issue order
    uint64_t slot_bytes = 0;    // largest span image, rounded up to 4 KiB
    long long group_last[2] = {-1, -1};
    uint32_t lba_seq_breaks = 0;  // direct-path commands that do not continue the previous one's LBA run
};

// What a schedule is built from (the plan itself does not change after creation).
struct ScheduleKey {
    int layer_begin = -1, layer_end = -1, span_chunks = 0, order_pc = 0, order_direct = 0;
    uint64_t C = 0, cmd_limit = 0, region_bytes = 0, pageable_bytes = 0;
    bool operator==(const ScheduleKey &o) const
    {
        return layer_begin == o.layer_begin && layer_end == o.layer_end && span_chunks == o.span_chunks &&
               order_pc == o.order_pc && order_direct == o.order_direct && C == o.C && cmd_limit == o.cmd_limit &&
               region_bytes == o.region_bytes && pageable_bytes == o.pageable_bytes;
    }
};

// Layers one whole-extent span may cover: as many as keep the images within 128 MiB (a launch of a few MiB is
// mostly ramp: 16 MiB per launch ran at half the HBM rate of 128 MiB), at most 16.
constexpr uint64_t kGroupBytes = 128ull << 20;
constexpr int kGroupLayersMax = 16;

struct Entry {
    hipEvent_t ev = nullptr;
    std::atomic<int> pending{0};
};

}  // namespace

struct kv_pipeline {
    int device = 0;
    hipStream_t s_compute = nullptr;  // the caller's stream of the running call (not owned): kernels are launched on it
    hipStream_t s_copy[kMaxCopyStreams] = {nullptr, nullptr, nullptr, nullptr};
    void *staging = nullptr;
    size_t staging_bytes = 0;
    void *bounce = nullptr;
    size_t bounce_bytes = 0;
    void *attn_ws = nullptr;
    size_t attn_ws_bytes = 0;
    std::vector<hipEvent_t> ev_ready, ev_free;  // per staging slot, recorded on the kernel stream
    std::vector<hipEvent_t> ev_done;            // per staging slot and copy stream
    std::vector<Entry> ring;                    // per in-flight command
    std::vector<hipEvent_t> timing;             // pairs
    kvb::Workers workers;
    // decode append: pinned landing buffer for the packed rows, and per (tensor, sequence) the image of
    // the last partly filled sector (so that only the first append after an offload has to read it back)
    void *seq_off_dev = nullptr;  // per-sequence element offsets inside an extent image (attention from extents)
    std::vector<int64_t> seq_off_host;
    void *append_host = nullptr;
    size_t append_host_bytes = 0;
    std::vector<char> tail_img;
    std::vector<int64_t> tail_sector;
    const void *tail_region = nullptr, *tail_pageable = nullptr;  // host buffers the images were taken from
    kvb::LinkRate link[2];       // issue pacing: the host link's rate per direction (0 offload, 1 reload)
    Schedule sched;              // the last call's spans and chunk commands: a decode loop repeats the same call
    ScheduleKey sched_key;       // (building them costs ~0.1 ms per 1000 commands)
    bool sched_valid = false;
    bool link_measured = false;

    ~kv_pipeline()
    {
        workers.stop();
        (void)hipSetDevice(device);
        for (auto st : s_copy) if (st) (void)hipStreamSynchronize(st);
        for (auto e : ev_ready) (void)hipEventDestroy(e);
        for (auto e : ev_free) (void)hipEventDestroy(e);
        for (auto e : ev_done) (void)hipEventDestroy(e);
        for (auto &e : ring) if (e.ev) (void)hipEventDestroy(e.ev);
        for (auto e : timing) (void)hipEventDestroy(e);
        if (staging) (void)hipFree(staging);
        if (bounce) (void)hipHostFree(bounce);
        if (append_host) (void)hipHostFree(append_host);
        if (seq_off_dev) (void)hipFree(seq_off_dev);
        if (attn_ws) (void)hipFree(attn_ws);
        for (auto st : s_copy) if (st) (void)hipStreamDestroy(st);
    }
};

namespace {

int ensure_events(std::vector<hipEvent_t> &v, size_t n, unsigned flags)
{
    while (v.size() < n) {
        hipEvent_t e;
        KV_HIP(hipEventCreateWithFlags(&e, flags));
        v.push_back(e);
    }
    return KV_OK;
}

// The host link's transfer rate in both directions, for the issue pacing: best of five timed copies of up to
// 64 MiB between a pinned buffer of its own and the staging memory (nothing of the caller's is touched).  Done once
// per process and device (about 12 ms), by the first pipeline whose staging memory is large enough; a rate that
// cannot be measured stays 0, and that direction is then not paced.
std::mutex g_link_mu;
double g_link_rate[64][2];   // per device, measured once per process
bool g_link_known[64];

int measure_link_rates(kv_pipeline *q)
{
    std::lock_guard<std::mutex> g(g_link_mu);
    const int dev = q->device >= 0 && q->device < 64 ? q->device : 0;
    if (g_link_known[dev]) {
        q->link[0].rate = std::max(q->link[0].rate, g_link_rate[dev][0]);
        q->link[1].rate = std::max(q->link[1].rate, g_link_rate[dev][1]);
        q->link_measured = true;
        return KV_OK;
    }
    const size_t bytes = std::min<size_t>(q->staging_bytes, 64u << 20);
    if (bytes < (1u << 20)) return KV_OK;
    void *pinned = nullptr;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    q->link_measured = true;   // one attempt only
    if (hipHostMalloc(&pinned, bytes, hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return KV_OK; }
    std::memset(pinned, 0, bytes);
    hipError_t e = hipEventCreate(&e0);
    if (e == hipSuccess) e = hipEventCreate(&e1);
    for (int dir = 0; dir < 2 && e == hipSuccess; ++dir) {
        for (int pass = 0; pass < 6 && e == hipSuccess; ++pass) {   // the first pass warms the path up
            e = hipEventRecord(e0, q->s_copy[0]);
            if (e == hipSuccess)
                e = dir == 0 ? hipMemcpyAsync(pinned, q->staging, bytes, hipMemcpyDeviceToHost, q->s_copy[0])
                             : hipMemcpyAsync(q->staging, pinned, bytes, hipMemcpyHostToDevice, q->s_copy[0]);
            if (e == hipSuccess) e = hipEventRecord(e1, q->s_copy[0]);
            if (e == hipSuccess) e = hipEventSynchronize(e1);
            float ms = 0.f;
            if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
            if (e == hipSuccess && pass > 0 && ms > 0.f) q->link[dir].rate = std::max(q->link[dir].rate, (double)bytes / (ms * 1e-3));
        }
    }
    if (e0) (void)hipEventDestroy(e0);
    if (e1) (void)hipEventDestroy(e1);
    (void)hipHostFree(pinned);
    if (e != hipSuccess) { kvb::set_hip_error((int)e); return KV_EHIP; }
    if (q->link[0].rate > 0.0 && q->link[1].rate > 0.0) {
        g_link_rate[dev][0] = q->link[0].rate;
        g_link_rate[dev][1] = q->link[1].rate;
        g_link_known[dev] = true;
    }
    return KV_OK;
}

// The plan's pipeline object with its copy streams (created on first use).
int create_pipe(kv_plan *p)
{
    if (!p->pipe) {
        p->pipe = new kv_pipeline();
        KV_HIP(hipGetDevice(&p->pipe->device));
        // The runtime maps streams onto a few hardware queues (four per process by default; a stream created when all
        // exist shares the least used one), and two streams on one queue run their commands one after the other: a
        // copy stream that shared its queue with the kernel stream made every third 512 KiB command 8 us late.  So
        // the library has no kernel stream of its own: kernels go to the caller's stream, which has its queue
        // already, and the three copy streams that small commands rotate over are created first.
        for (auto &st : p->pipe->s_copy) KV_HIP(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    }
    return KV_OK;
}

int ensure_pipeline(kv_plan *p, size_t n_slots, size_t slot_bytes, int depth, size_t chunk_bytes_max, bool need_bounce,
                    int n_workers, size_t attn_ws_bytes, size_t n_timing)
{
    int rc0 = create_pipe(p);
    if (rc0 != KV_OK) return rc0;
    kv_pipeline *q = p->pipe;
    const size_t need = n_slots * slot_bytes;
    if (q->staging_bytes < need) {
        if (q->staging) KV_HIP(hipFree(q->staging));
        q->staging = nullptr; q->staging_bytes = 0;
        KV_HIP(hipMalloc(&q->staging, need));
        q->staging_bytes = need;
    }
    if (need_bounce && q->bounce_bytes < (size_t)depth * chunk_bytes_max) {
        if (q->bounce) KV_HIP(hipHostFree(q->bounce));
        q->bounce = nullptr; q->bounce_bytes = 0;
        KV_HIP(hipHostMalloc(&q->bounce, (size_t)depth * chunk_bytes_max, hipHostMallocDefault));
        q->bounce_bytes = (size_t)depth * chunk_bytes_max;
    }
    if (attn_ws_bytes && q->attn_ws_bytes < attn_ws_bytes) {
        if (q->attn_ws) KV_HIP(hipFree(q->attn_ws));
        q->attn_ws = nullptr; q->attn_ws_bytes = 0;
        KV_HIP(hipMalloc(&q->attn_ws, attn_ws_bytes));
        q->attn_ws_bytes = attn_ws_bytes;
    }
    int rc = ensure_events(q->ev_ready, n_slots, hipEventDisableTiming);
    if (rc) return rc;
    rc = ensure_events(q->ev_free, n_slots, hipEventDisableTiming);
    if (rc) return rc;
    rc = ensure_events(q->ev_done, n_slots * kMaxCopyStreams, hipEventDisableTiming);
    if (rc) return rc;
    if (q->ring.size() < (size_t)depth) {
        std::vector<Entry> bigger((size_t)depth);
        for (size_t i = 0; i < q->ring.size(); ++i) bigger[i].ev = q->ring[i].ev;
        q->ring.swap(bigger);
    }
    for (auto &e : q->ring)
        if (!e.ev) KV_HIP(hipEventCreateWithFlags(&e.ev, hipEventDisableTiming));
    rc = ensure_events(q->timing, n_timing, hipEventDefault);
    if (rc) return rc;
    if (need_bounce) q->workers.start(n_workers);
    if (!q->link_measured && depth >= 2) {
        rc = measure_link_rates(q);
        if (rc) return rc;
    }
    return KV_OK;
}

// Spans and chunk commands of layers [layer_begin, layer_end): Eq. 7-11 per tensor (and sequence) with C token
// rows per chunk, each chunk cut once more under the transfer-size limit, emitted in the overlap order of the
// layer's path group.
int build_schedule(const kv_plan *p, int layer_begin, int layer_end, uint64_t C, int span_chunks, int order_pc,
                   int order_direct, uint64_t cmd_limit, uint64_t region_bytes, uint64_t pageable_bytes, Schedule *out)
{
    std::vector<Span> &spans = out->spans;
    std::vector<Chunk> &chunks = out->chunks;
    std::vector<kv_cmd_t> cmds;
    const uint64_t sec = (uint64_t)p->sector;
    const uint64_t image = p->tensor_blocks * sec;
    // Units: a span with its chunk commands.  Per layer the K units and the V units are emitted either one
    // tensor after the other (KV_ORDER_CROSS: V's storage-side hop runs while K's transfers are in flight)
    // or alternating (KV_ORDER_INTRA: both tensors' hops proceed side by side) -- the two overlap
    // strategies of Sec. IV-C.
    struct Unit { Span span; std::vector<Chunk> chunks; };
    for (int l = layer_begin; l < layer_end;) {
        const int order = l < p->n1 ? order_pc : order_direct;
        // Whole-extent spans: K and V of a layer share one launch while the pair stays within 256 MiB
        // (measured: pairing gains ~5 % at 64 MiB tensors and loses ~10 % at 256 MiB tensors), or when
        // their chunks alternate.  Small layers go together: consecutive layers of one path share a span
        // (K then V per layer, so the command stream stays one ascending run).
        const bool pair = span_chunks == 0 && (2 * image <= (256ull << 20) || order == KV_ORDER_INTRA);
        int group = 1;
        if (pair && order == KV_ORDER_CROSS) {
            const int path_end = l < p->n1 ? std::min(p->n1, layer_end) : layer_end;
            group = (int)std::min<uint64_t>(kGroupLayersMax, std::max<uint64_t>(1, kGroupBytes / (2 * image)));
            group = std::min(group, path_end - l);
        }
        std::vector<Unit> units[2];
        for (int lg = l; lg < l + group; ++lg)
        for (int kind = 0; kind < 2; ++kind) {
            const kv_extent_t &ext = p->ext[2 * lg + kind];
            const int nseq = p->mode == KV_TOKEN_MAJOR ? 1 : p->B;
            if (span_chunks == 0 && lg == l) {
                Unit u;
                u.span = pair ? Span{l, KV_KV, KV_SEQ_ALL, 0, 0, (uint64_t)group * 2 * image, ext.path, false, group}
                              : Span{l, kind, KV_SEQ_ALL, 0, 0, image, ext.path, false, 1};
                units[kind].push_back(u);
            }
            for (int b = 0; b < nseq; ++b) {
                int rc = kvb::chunk_cmds(p, lg, kind, b, (int)C, &cmds);
                if (rc != KV_OK) return rc;
                for (size_t i = 0; i < cmds.size(); ++i) {
                    const kv_cmd_t &c = cmds[i];
                    if (span_chunks > 0 && i % (size_t)span_chunks == 0) {
                        const size_t j = std::min(cmds.size(), i + (size_t)span_chunks) - 1;
                        Unit u;
                        u.span = Span{lg, kind, b, (int)c.tok0, (int)(cmds[j].tok0 + cmds[j].ntok - c.tok0), 0, ext.path, false, 1};
                        for (size_t k = i; k <= j; ++k) u.span.bytes += ((uint64_t)cmds[k].nlb + 1) * sec;
                        units[kind].push_back(u);
                    }
                    Unit &u = units[kind].back();
                    Chunk ch;
                    ch.host_off = c.slba * sec;
                    ch.bytes = ((uint64_t)c.nlb + 1) * sec;
                    ch.span = -1;
                    ch.stage_off = span_chunks == 0 ? (pair ? ((uint64_t)(lg - l) * 2 + (uint64_t)kind) * image : 0) + p->seq_base[b] * sec + c.buf_off
                                                    : c.buf_off - (uint64_t)u.span.tok0 * p->row_bytes;
                    ch.first = ch.last = false;
                    ch.layer = lg;
                    ch.kind = kind;
                    const uint64_t host_cap = ext.path == KV_PATH_DIRECT ? region_bytes : pageable_bytes;
                    if (ch.host_off + ch.bytes > host_cap) return KV_ENOSPC;
                    // transfer-size limit: Eq. 8-11 once more on the chunk's own request
                    for (uint64_t done = 0; done < ch.bytes; done += cmd_limit) {
                        Chunk part = ch;
                        part.host_off += done;
                        part.stage_off += done;
                        part.bytes = std::min(cmd_limit, ch.bytes - done);
                        u.chunks.push_back(part);
                    }
                }
            }
        }
        auto emit_span = [&](const Span &sp) { spans.push_back(sp); return (int)spans.size() - 1; };
        auto emit_chunk = [&](Chunk ch, int span) { ch.span = span; chunks.push_back(ch); };
        if (pair) {
            // one span; its commands layer by layer, K's and V's in the chosen order
            const int si = emit_span(units[0][0].span);
            std::vector<Chunk> &ck = units[0][0].chunks, &cv = units[1][0].chunks;
            if (order == KV_ORDER_INTRA) {
                for (size_t i = 0; i < std::max(ck.size(), cv.size()); ++i) {
                    if (i < ck.size()) emit_chunk(ck[i], si);
                    if (i < cv.size()) emit_chunk(cv[i], si);
                }
            } else {
                // tensor-id order: K of a layer, then its V, then the next layer
                std::vector<Chunk> all(ck);
                all.insert(all.end(), cv.begin(), cv.end());
                std::stable_sort(all.begin(), all.end(), [](const Chunk &a, const Chunk &b) {
                    return a.layer != b.layer ? a.layer < b.layer : a.kind < b.kind;
                });
                for (const Chunk &c : all) emit_chunk(c, si);
            }
        } else if (order == KV_ORDER_INTRA) {
            for (size_t i = 0; i < std::max(units[0].size(), units[1].size()); ++i)
                for (int kind = 0; kind < 2; ++kind)
                    if (i < units[kind].size()) {
                        const int si = emit_span(units[kind][i].span);
                        for (const Chunk &c : units[kind][i].chunks) emit_chunk(c, si);
                    }
        } else {
            for (int kind = 0; kind < 2; ++kind)
                for (const Unit &u : units[kind]) {
                    const int si = emit_span(u.span);
                    for (const Chunk &c : u.chunks) emit_chunk(c, si);
                }
        }
        if (!spans.empty()) spans.back().last_of_layer = true;
        l += group;
    }
    // last chunk command of each path group (for the per-group throughput figures)
    long long *group_last = out->group_last;
    for (size_t i = 0; i < chunks.size(); ++i) group_last[spans[chunks[i].span].path == KV_PATH_PAGECACHE ? 0 : 1] = (long long)i;
    for (size_t i = 0; i < chunks.size(); ++i) {
        chunks[i].first = i == 0 || chunks[i - 1].span != chunks[i].span;
        chunks[i].last = i + 1 == chunks.size() || chunks[i + 1].span != chunks[i].span;
    }
    uint64_t prev_end = UINT64_MAX;
    for (const Chunk &c : chunks) {
        if (spans[c.span].path != KV_PATH_DIRECT) continue;
        if (prev_end != UINT64_MAX && c.host_off != prev_end) out->lba_seq_breaks++;
        prev_end = c.host_off + c.bytes;
    }
    uint64_t slot_bytes = 0;
    for (const Span &s : spans) slot_bytes = std::max(slot_bytes, s.bytes);
    out->slot_bytes = kvb::round_up(slot_bytes, 4096);
    return KV_OK;
}

// The kernels of a call read (or overwrite) buffers the caller produced on its own stream, so they are launched on
// that stream: they follow everything queued there so far.  The copy streams only follow the kernels (offload) or
// touch library-owned staging (reload), through events.
int order_after_caller(kv_pipeline *q, void *caller_stream)
{
    q->s_compute = (hipStream_t)caller_stream;
    return KV_OK;
}

// Returns the seconds spent waiting (0 when the counter was already zero).
inline double spin_until_zero(std::atomic<int> &a)
{
    if (a.load(std::memory_order_acquire) == 0) return 0.0;
    const auto t0 = std::chrono::steady_clock::now();
    int spins = 0;
    while (a.load(std::memory_order_acquire) != 0) {
        if (++spins > 2000) std::this_thread::yield();
    }
    return std::chrono::duration<double>(std::chrono::steady_clock::now() - t0).count();
}

}  // namespace

void kvb::forget_tail_images(kv_pipeline *pipe)
{
    std::fill(pipe->tail_sector.begin(), pipe->tail_sector.end(), (int64_t)-1);
}

extern "C" void kv_plan_destroy(kv_plan_t *plan)
{
    if (!plan) return;
    delete plan->pipe;
    delete plan;
}

extern "C" int kv_pipeline_run(kv_plan_t *p, int dir, int layer_begin, int layer_end, const kv_view_t *view,
                               void *lba_region, size_t region_bytes, void *pageable, size_t pageable_bytes,
                               int chunk_tokens, int depth, const kv_attn_args_t *attn, const kv_pipe_opts_t *opts,
                               kv_pipe_stats_t *stats)
{
    const auto t_start = std::chrono::steady_clock::now();
    if (!p || !view) return KV_EINVAL;
    if (dir != KV_DIR_OFFLOAD && dir != KV_DIR_RELOAD && dir != KV_DIR_RELOAD_ATTN) return KV_EINVAL;
    if (layer_begin < 0 || layer_end > p->L || layer_begin > layer_end) return KV_ERANGE;
    if (layer_end > view->n_layers) return KV_ERANGE;
    if (depth < 1 || depth > 1024 || chunk_tokens < 0) return KV_EINVAL;
    if (dir == KV_DIR_RELOAD_ATTN && (!attn || !attn->q_layers || !attn->out_layers)) return KV_EINVAL;
    if (!view->seq_lens_host) return KV_EINVAL;
    const int span_chunks = opts ? opts->span_chunks : 0;
    const int n_workers = opts && opts->host_workers > 0 ? opts->host_workers : 8;
    const bool time_kernels = opts && (opts->flags & KV_PIPE_TIME_KERNELS);
    const bool serialize = opts && (opts->flags & KV_PIPE_SERIALIZE);
    const bool attn_from_extent = opts && (opts->flags & KV_PIPE_ATTN_FROM_EXTENT);
    if (attn_from_extent && (dir != KV_DIR_RELOAD_ATTN || span_chunks != 0)) return KV_EINVAL;
    if (span_chunks < 0 || n_workers > 64) return KV_EINVAL;
    const bool offload_dir = dir == KV_DIR_OFFLOAD;
    int ns = opts ? opts->copy_streams : 0;
    if (ns < 0 || ns > kMaxCopyStreams) return KV_EINVAL;
    const int d2h_mode = opts ? opts->d2h_mode : KV_COPY_AUTO, h2d_mode = opts ? opts->h2d_mode : KV_COPY_AUTO;
    if (d2h_mode < KV_COPY_AUTO || d2h_mode > KV_COPY_KERNEL || h2d_mode < KV_COPY_AUTO || h2d_mode > KV_COPY_KERNEL)
        return KV_EINVAL;
    // Engine defaults by measurement inside the paced pipeline (8B shape at 4K / 32K, ragged paged batch, Gemma
    // shape; three alternations per variant in one process).
    //  * H2D: the copy kernel over three streams for commands up to 1 MiB (512 KiB: 50 GB/s against 40 with
    //    hipMemcpyAsync), hipMemcpyAsync (SDMA engines) over up to four streams above.  The copy kernel would move
    //    2 and 8 MiB commands faster too (reload + attention 55.6-56.2 against 53.5-54.4 GB/s at the 32K shape, 57.2
    //    against 56.0-56.9 at the Gemma shape), but a compute unit that hosts a copy workgroup serves the loads of its
    //    other wavefronts behind the copy's PCIe reads: with it the unpack of a layer takes 135 instead of 68 us
    //    and the decode attention 127 instead of 42 us inside the pipeline (46 and 26 us with nothing else running).
    //    Where SDMA keeps up, the kernels that run next to the transfers -- here unpack and attention, in a
    //    serving system the model's own layers -- keep the compute units to themselves.
    //  * D2H: the copy kernel over three streams below 1 MiB (512 KiB: 48 against 42 GB/s), hipMemcpyAsync over up
    //    to four streams from 1 MiB on (1 MiB: 50.7-53.4 against a steady 52.9; 2 MiB: 54.4-55.9 against 54.0-54.7;
    //    8 MiB: 55.9-56.8 against 55.2-55.4).  The runtime runs those copies as a kernel of its own, which disturbs
    //    the pack next to it less than this file's copy kernel does (57-69 against 132-153 us per pack).
    //  * Eight workgroups per copy command in both directions: 16, 32 and 64 lose 2, 4 and 7-14 GB/s on the
    //    reload side.
    uint64_t cmd_bytes = (chunk_tokens > 0 ? (uint64_t)chunk_tokens : (uint64_t)p->chunk_tokens) * p->row_bytes;
    uint64_t cmd_limit = UINT64_MAX;  // Eq. 7 on the caller's transfer-size limit
    if (opts && opts->max_cmd_bytes) {
        cmd_limit = opts->max_cmd_bytes / (uint64_t)p->sector * (uint64_t)p->sector;
        if (cmd_limit == 0) return KV_EINVAL;
        cmd_bytes = std::min(cmd_bytes, cmd_limit);
    }
    const bool d2h_kernel = d2h_mode == KV_COPY_KERNEL || (d2h_mode == KV_COPY_AUTO && cmd_bytes < (1ull << 20));
    const bool h2d_kernel = h2d_mode == KV_COPY_KERNEL || (h2d_mode == KV_COPY_AUTO && cmd_bytes <= (1ull << 20));
    const int order_pc = opts ? opts->order_pagecache : KV_ORDER_CROSS;
    const int order_direct = opts ? opts->order_direct : KV_ORDER_CROSS;
    if ((order_pc != KV_ORDER_CROSS && order_pc != KV_ORDER_INTRA) ||
        (order_direct != KV_ORDER_CROSS && order_direct != KV_ORDER_INTRA))
        return KV_EINVAL;
    if (ns == 0) ns = (offload_dir ? d2h_kernel : h2d_kernel) ? 3 : 4;
    ns = std::min(ns, depth);
    if (stats) std::memset(stats, 0, sizeof(*stats));
    if (layer_begin == layer_end) return KV_OK;

    const uint64_t sec = (uint64_t)p->sector;
    const uint64_t C = chunk_tokens > 0 ? (uint64_t)chunk_tokens : (uint64_t)p->chunk_tokens;
    const uint64_t chunk_bytes = C * p->row_bytes;
    if (chunk_bytes % sec != 0) return KV_EALIGN;

    // Which host buffers does this layer range need?
    bool any_direct = false, any_pc = false;
    for (int l = layer_begin; l < layer_end; ++l) (l < p->n1 ? any_pc : any_direct) = true;
    if (any_direct) {
        if (!lba_region || ((uintptr_t)lba_region & 15)) return KV_EINVAL;
        if (region_bytes < p->region_bytes_needed) return KV_ENOSPC;
        hipPointerAttribute_t at;
        hipError_t e = hipPointerGetAttributes(&at, lba_region);
        if (e != hipSuccess) { (void)hipGetLastError(); return KV_EINVAL; }  // not pinned
        if (at.type != hipMemoryTypeHost) return KV_EINVAL;
    }
    if (any_pc) {
        if (!pageable) return KV_EINVAL;
        if (pageable_bytes < p->pageable_bytes_needed) return KV_ENOSPC;
    }

    // Valid lengths: a tensor moves rows [0, len_b) (padded to its extent); in span mode whole
    // capacity rows are addressed, so lengths must equal capacities there.
    for (int b = 0; b < p->B; ++b) {
        const int len = view->seq_lens_host[b];
        if (len < 0 || len > p->cap[b]) return KV_ERANGE;
        if (span_chunks > 0 && len != p->cap[b]) return KV_EINVAL;
    }

    {
        int rc = create_pipe(p);
        if (rc != KV_OK) return rc;
        ScheduleKey key;
        key.layer_begin = layer_begin; key.layer_end = layer_end; key.span_chunks = span_chunks;
        key.order_pc = order_pc; key.order_direct = order_direct;
        key.C = C; key.cmd_limit = cmd_limit; key.region_bytes = region_bytes; key.pageable_bytes = pageable_bytes;
        if (!(p->pipe->sched_valid && p->pipe->sched_key == key)) {
            p->pipe->sched_valid = false;
            p->pipe->sched = Schedule();
            rc = build_schedule(p, layer_begin, layer_end, C, span_chunks, order_pc, order_direct, cmd_limit, region_bytes,
                                pageable_bytes, &p->pipe->sched);
            if (rc != KV_OK) return rc;
            p->pipe->sched_key = key;
            p->pipe->sched_valid = true;
        }
    }
    const Schedule &sched = p->pipe->sched;
    const std::vector<Span> &spans = sched.spans;
    const std::vector<Chunk> &chunks = sched.chunks;
    const uint64_t slot_bytes = sched.slot_bytes;
    const long long *group_last = sched.group_last;
    const uint64_t image = p->tensor_blocks * sec;
    const size_t n_slots = span_chunks == 0 ? 4 : std::max<size_t>(4, (size_t)depth);

    size_t ws_bytes = 0;
    if (dir == KV_DIR_RELOAD_ATTN) {
        int max_len = 0;
        for (int b = 0; b < p->B; ++b) max_len = std::max(max_len, view->seq_lens_host[b]);
        ws_bytes = kv_decode_attn_workspace(p, attn->n_splits, max_len);
    }
    const size_t n_timing = time_kernels ? 2 * (spans.size() + 2 * (size_t)(layer_end - layer_begin)) : 0;
    // Ring entries (completion event, host-copy counter, bounce slot).  `depth` bounds the transfers in
    // flight; with page-cache-path layers the ring is twice as long, so that a bounce slot can wait for its
    // host copy (the memcpy hop is not a device command) without holding back the next transfer.
    const size_t NB = any_pc ? 2 * (size_t)depth : (size_t)depth;
    // a bounce slot holds the largest page-cache-path command of this schedule (not the nominal chunk size: a
    // chunk may be larger than every extent, or cut down by the transfer-size limit)
    uint64_t bounce_slot = 0;
    for (const Chunk &c : chunks)
        if (spans[c.span].path == KV_PATH_PAGECACHE) bounce_slot = std::max(bounce_slot, c.bytes);
    bounce_slot = kvb::round_up(bounce_slot, 4096);
    int rc = ensure_pipeline(p, n_slots, slot_bytes, (int)NB, bounce_slot, any_pc, n_workers, ws_bytes, n_timing);
    if (rc != KV_OK) return rc;
    kv_pipeline *q = p->pipe;
    rc = order_after_caller(q, opts ? opts->caller_stream : nullptr);
    if (rc != KV_OK) return rc;
    if (attn_from_extent && p->mode == KV_PER_SEQ && !q->seq_off_dev) {
        q->seq_off_host.resize((size_t)p->B);
        for (int b = 0; b < p->B; ++b) q->seq_off_host[b] = (int64_t)(p->seq_base[b] * sec / 2);
        KV_HIP(hipMalloc(&q->seq_off_dev, sizeof(int64_t) * (size_t)p->B));
        KV_HIP(hipMemcpy(q->seq_off_dev, q->seq_off_host.data(), sizeof(int64_t) * (size_t)p->B, hipMemcpyHostToDevice));
    }
    char *staging = (char *)q->staging;
    const int pieces_max = std::max(1, q->workers.size());

    // kernel timing bookkeeping
    std::vector<int> timing_kind;
    auto time_begin = [&](int kind) {
        if (!time_kernels) return;
        (void)hipEventRecord(q->timing[2 * timing_kind.size()], q->s_compute);
        timing_kind.push_back(kind);
    };
    auto time_end = [&]() {
        if (!time_kernels) return;
        (void)hipEventRecord(q->timing[2 * (timing_kind.size() - 1) + 1], q->s_compute);
    };

    const bool offload = offload_dir;
    if (offload) kvb::forget_tail_images(q);  // extents are rewritten
    const size_t N = chunks.size();
    std::vector<unsigned> slot_used(n_slots, 0u);  // copy streams that carried the slot's last span
    size_t n_waited = 0;  // chunks [0, n_waited) are known complete
    size_t n_issued = 0;  // chunks [0, n_issued) have been issued
    uint32_t max_in_flight = 0;
    int err = KV_OK;

    // Per path group: host time from the issue of its first command to the harvest of its last.
    double group_t0[2] = {-1.0, -1.0}, group_t1[2] = {-1.0, -1.0};
    auto now_s = [&]() { return std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count(); };
    auto note_issue = [&](size_t c) {
        const int g = spans[chunks[c].span].path == KV_PATH_PAGECACHE ? 0 : 1;
        if (group_t0[g] < 0) group_t0[g] = now_s();
    };
    // optional per-command record: what was moved, when it was queued, when its completion was harvested
    kv_chunk_trace_t *const trace = opts ? opts->trace : nullptr;
    const size_t trace_cap = trace ? (size_t)opts->trace_cap : 0;
    size_t n_traced = 0;
    auto trace_issue = [&](size_t c) {
        if (c >= trace_cap) return;
        const Chunk &ch = chunks[c];
        kv_chunk_trace_t &t = trace[c];
        t.host_off = ch.host_off;
        t.bytes = ch.bytes;
        t.layer = (uint16_t)ch.layer;
        t.kind = (uint8_t)ch.kind;
        t.path = (uint8_t)spans[ch.span].path;
        t.reserved = 0;
        t.t_issue_s = now_s();
        t.t_done_s = -1.0;
        n_traced = c + 1;
    };
    auto host_ptr = [&](const Chunk &ch) -> char * {
        return (spans[ch.span].path == KV_PATH_DIRECT ? (char *)lba_region : (char *)pageable) + ch.host_off;
    };
    auto bounce_ptr = [&](size_t c) -> char * { return (char *)q->bounce + (c % NB) * bounce_slot; };
    // The memcpy hop of chunk c, cut into pieces for the worker threads; ring entry c counts the pieces down.
    auto fan_out = [&](size_t c, void *dst, const void *src, size_t bytes) {
        Entry &e = q->ring[c % NB];
        int pieces = (int)std::min<size_t>((size_t)pieces_max, std::max<size_t>(1, bytes / (256 * 1024)));
        e.pending.store(pieces, std::memory_order_release);
        const size_t step = kvb::round_up(kvb::ceil_div(bytes, (uint64_t)pieces), 4096);
        kvb::CopyTask tasks[64];
        size_t off = 0;
        int n_tasks = 0;
        for (int i = 0; i < pieces; ++i) {
            const size_t n = off < bytes ? std::min(step, bytes - off) : 0;
            if (n == 0) { e.pending.fetch_sub(1, std::memory_order_release); continue; }
            tasks[n_tasks++] = kvb::CopyTask{(char *)dst + off, (const char *)src + off, n, &e.pending};
            off += n;
        }
        q->workers.push(tasks, n_tasks);
    };

    const size_t in_flight_max = offload_dir && !d2h_kernel ? std::min<size_t>((size_t)depth, 4) : (size_t)depth;
    // Issue pacing (pacer.hpp): consecutive commands are queued no closer together than one command's own link time.
    // Both copy engines are paced: with hipMemcpyAsync commands of 2 and 8 MiB it gains 2-4 % as well.
    const int pace_dir = offload_dir ? 0 : 1;
    kvb::IssuePacer pacer(&q->link[pace_dir], !serialize && !(opts && (opts->flags & KV_PIPE_NO_PACING)), (int)in_flight_max,
                          (offload_dir ? d2h_kernel : h2d_kernel) ? 1.0 : 0.5);
    // forward declaration of the harvest (defined below): the pacer polls it while it waits
    std::function<int(size_t, bool)> harvest_ready;
    // Call right before command c is queued: waits until the pacer lets it go.  While it waits it harvests, without
    // blocking, whatever has completed, so that the pacer counts what is really outstanding (this costs nothing
    // when the host is the bottleneck: then there is no wait).
    auto pace_issue = [&](uint64_t bytes, size_t c) -> int {
        if (pacer.enabled()) {
            while (now_s() < pacer.due(c - n_waited)) {
                const int r = harvest_ready(c, false);
                if (r != KV_OK) return r;
                __builtin_ia32_pause();
            }
        }
        pacer.issued(now_s(), bytes);
        return KV_OK;
    };
    auto pace_harvest = [&](uint64_t bytes, bool waited) { pacer.harvested(now_s(), bytes, waited); };

    // Chunk c owns ring entry c % NB.  Transfers are harvested in issue order; n_waited counts them.
    double host_wait_s = 0.0, harvest_wait_s = 0.0;
    // Harvest the transfers of chunks [0, upto); block = false: only those that have already completed.
    auto harvest_until = [&](size_t upto, bool block = true) -> int {
        while (n_waited < upto) {
            bool waited = false;
            if (hipEventQuery(q->ring[n_waited % NB].ev) != hipSuccess) {
                if (!block) { (void)hipGetLastError(); break; }
                const double t0 = now_s();
                KV_HIP(hipEventSynchronize(q->ring[n_waited % NB].ev));
                harvest_wait_s += now_s() - t0;
                waited = true;
            }
            pace_harvest(chunks[n_waited].bytes, waited);
            // offload, page-cache path: the chunk's bytes are in its bounce slot now; start the memcpy hop
            if (offload_dir && spans[chunks[n_waited].span].path == KV_PATH_PAGECACHE)
                fan_out(n_waited, host_ptr(chunks[n_waited]), bounce_ptr(n_waited), chunks[n_waited].bytes);
            for (int g = 0; g < 2; ++g)
                if ((long long)n_waited == group_last[g]) group_t1[g] = now_s();
            if (n_waited < trace_cap) trace[n_waited].t_done_s = now_s();
            ++n_waited;
        }
        return KV_OK;
    };
    // At most `depth` transfers outstanding: the oldest is harvested before chunk c is issued.  The rule is an upper
    // bound, and D2H hipMemcpyAsync commands use less of it: each runs as a wide-grid kernel of the runtime's, and more
    // than four of those at once get in each other's way (2 MiB commands at depth 8: 40 GB/s, at depth 4: 56).
    harvest_ready = harvest_until;
    auto transfer_slot = [&](size_t c) -> int { return c >= in_flight_max ? harvest_until(c + 1 - in_flight_max) : KV_OK; };
    // Ring entry (and bounce slot) of chunk c is free once chunk c - NB has left it, host copy included.
    auto entry_free = [&](size_t c) -> int {
        if (c < NB) return KV_OK;
        int r = harvest_until(c - NB + 1);
        if (r != KV_OK) return r;
        host_wait_s += spin_until_zero(q->ring[c % NB].pending);
        return KV_OK;
    };
    // Transfer of one chunk command on copy stream `st`; `ev` is its completion entry.  The copy kernel carries
    // the event on its own dispatch (no separate record packet: measured +5-14 % on commands of 1 MiB and less).
    auto issue_copy = [&](void *dst, const void *src, size_t bytes, bool to_host, hipStream_t st, hipEvent_t ev) -> hipError_t {
        const bool by_kernel = to_host ? d2h_kernel : h2d_kernel;
        if (!by_kernel) {
            hipError_t e = hipMemcpyAsync(dst, src, bytes, to_host ? hipMemcpyDeviceToHost : hipMemcpyHostToDevice, st);
            return e != hipSuccess ? e : hipEventRecord(ev, st);
        }
        const size_t nvec = bytes / 16;
        // 8 workgroups saturate the link and give the lowest per-command cost (measured over 2-32: a command of
        // 512 KiB moves at 46 GB/s D2H / 52 GB/s H2D with 8, 45 / 42 with 32); a small grid also keeps the compute
        // units whose store path backs up behind PCIe writes few, so the concurrent pack kernel is disturbed less
        const unsigned blocks = (unsigned)std::min<size_t>(8, std::max<size_t>(1, nvec / (256 * 4)));
        hipExtLaunchKernelGGL(kv_chunk_copy_kernel, dim3(blocks), dim3(256), 0, st, nullptr, ev, 0, (const u32x4 *)src,
                              (u32x4 *)dst, nvec);
        return hipGetLastError();
    };
    unsigned used = 0;  // copy streams that carried a chunk of the current span
    std::vector<void *> ext_k((size_t)view->n_layers, nullptr), ext_v((size_t)view->n_layers, nullptr);
    char *ext_k_img = nullptr;
    int ext_k_slot = -1;

    if (offload) {
        // Pack of span i into its staging slot, on the kernel stream.  The kernel stream runs one span ahead of
        // the transfers (four slots exist), so the link does not wait for a pack at a span boundary.
        size_t n_packed = 0;
        auto pack_span = [&](size_t si) -> int {
            const Span &sp = spans[si];
            const size_t slot = si % n_slots;
            char *img = staging + slot * slot_bytes;
            // the slot's previous copies must have left it before the kernel overwrites it
            if (si >= n_slots)
                for (int s = 0; s < ns; ++s)
                    if (slot_used[slot] >> s & 1) KV_HIP(hipStreamWaitEvent(q->s_compute, q->ev_done[slot * kMaxCopyStreams + s], 0));
            time_begin(KV_KERNEL_PACK);
            const int rc = sp.n_layers > 1
                               ? kv_offload_pack_layers(p, sp.layer, sp.layer + sp.n_layers, view, img, slot_bytes, q->s_compute)
                               : kv_offload_pack(p, sp.layer, sp.kind, view, sp.seq, sp.tok0, sp.ntok, img, slot_bytes, q->s_compute);
            time_end();
            if (rc != KV_OK) return rc;
            if (stats) { stats->kernel_launches[KV_KERNEL_PACK]++; stats->n_spans++; }
            KV_HIP(hipEventRecord(q->ev_ready[slot], q->s_compute));
            if (serialize) KV_HIP(hipStreamSynchronize(q->s_compute));
            return KV_OK;
        };
        for (size_t c = 0; c < N && err == KV_OK; ++c) {
            const Chunk &ch = chunks[c];
            const Span &sp = spans[ch.span];
            const size_t slot = (size_t)ch.span % n_slots;
            char *img = staging + slot * slot_bytes;
            if (ch.first) {
                const size_t ahead = serialize ? 0 : 1;
                while (err == KV_OK && n_packed < spans.size() && n_packed <= (size_t)ch.span + ahead) err = pack_span(n_packed++);
                if (err != KV_OK) break;
                used = 0;
            }
            if ((err = entry_free(c)) != KV_OK || (err = transfer_slot(c)) != KV_OK) break;
            note_issue(c);
            Entry &e = q->ring[c % NB];
            const int s = (int)(c % (size_t)ns);
            hipStream_t st = q->s_copy[s];
            if (!(used >> s & 1)) {  // first chunk of this span on this stream: order it after the pack
                KV_HIP_BRK(hipStreamWaitEvent(st, q->ev_ready[slot], 0));
                used |= 1u << s;
            }
            if ((err = pace_issue(ch.bytes, c)) != KV_OK) break;
            if (sp.path == KV_PATH_DIRECT) {
                KV_HIP_BRK(issue_copy(host_ptr(ch), img + ch.stage_off, ch.bytes, true, st, e.ev));
            } else {
                // the memcpy hop starts when this transfer is harvested (its bytes are in the bounce slot then);
                // until then the entry counts one outstanding host copy
                KV_HIP_BRK(issue_copy(bounce_ptr(c), img + ch.stage_off, ch.bytes, true, st, e.ev));
                e.pending.store(1, std::memory_order_release);
            }
            trace_issue(c);
            n_issued = c + 1;
            max_in_flight = std::max<uint32_t>(max_in_flight, (uint32_t)(c + 1 - n_waited));
            if (serialize) {  // every stage to completion before the next starts
                if ((err = harvest_until(c + 1)) != KV_OK) break;
                host_wait_s += spin_until_zero(e.pending);
            }
            if (ch.last) {
                for (int k = 0; k < ns && err == KV_OK; ++k)
                    if (used >> k & 1) KV_HIP_SET(hipEventRecord(q->ev_done[slot * kMaxCopyStreams + k], q->s_copy[k]));
                slot_used[slot] = used;
            }
            if (stats) {
                stats->n_chunks++;
                (sp.path == KV_PATH_DIRECT ? stats->bytes_direct : stats->bytes_pagecache) += ch.bytes;
            }
        }
    } else {
        // Reload.  Page-cache-path chunks are started (arena -> bounce memcpy) up to `depth` commands ahead
        // of their H2D issue; a direct chunk starts when it is issued.
        const size_t look = serialize ? 1 : (size_t)depth;
        size_t cs = 0;  // next chunk to start
        for (size_t ci = 0; ci < N && err == KV_OK; ++ci) {
            while (cs < N && err == KV_OK) {
                const bool pc = spans[chunks[cs].span].path == KV_PATH_PAGECACHE;
                if (cs >= ci + (pc ? look : 1)) break;
                if ((err = entry_free(cs)) != KV_OK) break;
                note_issue(cs);
                Entry &e = q->ring[cs % NB];
                if (pc) fan_out(cs, bounce_ptr(cs), host_ptr(chunks[cs]), chunks[cs].bytes);
                else e.pending.store(0, std::memory_order_release);
                ++cs;
            }
            if (err != KV_OK) break;
            if ((err = transfer_slot(ci)) != KV_OK) break;
            const Chunk &ch = chunks[ci];
            const Span &sp = spans[ch.span];
            const size_t slot = (size_t)ch.span % n_slots;
            char *img = staging + slot * slot_bytes;
            Entry &e = q->ring[ci % NB];
            const int s = (int)(ci % (size_t)ns);
            hipStream_t st = q->s_copy[s];
            if (ch.first) used = 0;
            if (!(used >> s & 1)) {  // first chunk of this span on this stream: the slot must be free
                if ((size_t)ch.span >= n_slots) KV_HIP_BRK(hipStreamWaitEvent(st, q->ev_free[slot], 0));
                used |= 1u << s;
            }
            if (sp.path == KV_PATH_DIRECT) {
                if ((err = pace_issue(ch.bytes, ci)) != KV_OK) break;
                KV_HIP_BRK(issue_copy(img + ch.stage_off, host_ptr(ch), ch.bytes, false, st, e.ev));
            } else {
                host_wait_s += spin_until_zero(e.pending);  // the arena bytes are in the bounce slot
                if ((err = pace_issue(ch.bytes, ci)) != KV_OK) break;
                KV_HIP_BRK(issue_copy(img + ch.stage_off, bounce_ptr(ci), ch.bytes, false, st, e.ev));
            }
            trace_issue(ci);
            n_issued = ci + 1;
            max_in_flight = std::max<uint32_t>(max_in_flight, (uint32_t)(ci + 1 - n_waited));
            if (serialize && (err = harvest_until(ci + 1)) != KV_OK) break;
            if (stats) {
                stats->n_chunks++;
                (sp.path == KV_PATH_DIRECT ? stats->bytes_direct : stats->bytes_pagecache) += ch.bytes;
            }
            if (ch.last) {
                for (int k = 0; k < ns && err == KV_OK; ++k) {
                    if (!(used >> k & 1)) continue;
                    KV_HIP_SET(hipEventRecord(q->ev_done[slot * kMaxCopyStreams + k], q->s_copy[k]));
                    if (err == KV_OK) KV_HIP_SET(hipStreamWaitEvent(q->s_compute, q->ev_done[slot * kMaxCopyStreams + k], 0));
                }
                if (err != KV_OK) break;
                if (!attn_from_extent) {
                    time_begin(KV_KERNEL_UNPACK);
                    err = sp.n_layers > 1
                              ? kv_reload_unpack_layers(p, sp.layer, sp.layer + sp.n_layers, img, slot_bytes, view, q->s_compute)
                              : kv_reload_unpack(p, sp.layer, sp.kind, img, slot_bytes, view, sp.seq, sp.tok0, sp.ntok, q->s_compute);
                    time_end();
                    if (err != KV_OK) break;
                    if (stats) { stats->kernel_launches[KV_KERNEL_UNPACK]++; stats->n_spans++; }
                    KV_HIP_BRK(hipEventRecord(q->ev_free[slot], q->s_compute));
                    if (dir == KV_DIR_RELOAD_ATTN && sp.last_of_layer) {
                        for (int l = sp.layer; l < sp.layer + sp.n_layers && err == KV_OK; ++l) {
                            time_begin(KV_KERNEL_ATTN_PARTIAL);  // partial + combine bracketed together
                            err = kv_decode_attn(p, view, l, attn->q_layers[l], attn->out_layers[l], attn->out_dtype,
                                                 attn->n_splits, q->attn_ws, q->attn_ws_bytes, q->s_compute);
                            time_end();
                            if (err == KV_OK && stats) { stats->kernel_launches[KV_KERNEL_ATTN_PARTIAL]++; stats->kernel_launches[KV_KERNEL_ATTN_COMBINE]++; }
                        }
                        if (err != KV_OK) break;
                    }
                } else {
                    // Attention straight from the staged extent images: extent order (S, B*H, D) is the
                    // strided [B,H,S,D] view with strides (H*D, D, B*H*D), so nothing is unpacked.
                    if (stats) stats->n_spans++;
                    if (sp.kind != KV_V) ext_k_img = img;  // KV_K or KV_KV span
                    if (sp.kind == KV_K) { ext_k_slot = (int)slot; }
                    if (sp.last_of_layer) {
                        kv_view_t ev = *view;
                        ev.layout = KV_LAYOUT_BHSD;
                        ev.k_layers = ext_k.data();
                        ev.v_layers = ext_v.data();
                        ev.layer_bytes = image;
                        ev.stride_h = p->D;
                        if (p->mode == KV_TOKEN_MAJOR) {
                            ev.stride_b = (int64_t)p->H * p->D;
                            ev.stride_s = (int64_t)p->B * p->H * p->D;
                            ev.s_alloc = p->cap[0];
                        } else {  // per-sequence sub-extents (cap_b, H, D), each at its own sector offset
                            ev.stride_b = 0;
                            ev.stride_s = (int64_t)p->H * p->D;
                            ev.s_alloc = *std::max_element(p->cap.begin(), p->cap.end());
                            ev.seq_off_host = q->seq_off_host.data();
                            ev.seq_off_dev = (const int64_t *)q->seq_off_dev;
                        }
                        for (int l = sp.layer; l < sp.layer + sp.n_layers && err == KV_OK; ++l) {
                            // a span of several layers holds K and V of layer l at images 2(l - first), 2(l - first) + 1
                            const uint64_t j = (uint64_t)(l - sp.layer);
                            ext_k[l] = sp.kind == KV_KV ? img + 2 * j * image : ext_k_img;
                            ext_v[l] = sp.kind == KV_KV ? img + (2 * j + 1) * image : img;
                            time_begin(KV_KERNEL_ATTN_PARTIAL);
                            err = kv_decode_attn(p, &ev, l, attn->q_layers[l], attn->out_layers[l], attn->out_dtype,
                                                 attn->n_splits, q->attn_ws, q->attn_ws_bytes, q->s_compute);
                            time_end();
                            if (err == KV_OK && stats) { stats->kernel_launches[KV_KERNEL_ATTN_PARTIAL]++; stats->kernel_launches[KV_KERNEL_ATTN_COMBINE]++; }
                        }
                        if (err != KV_OK) break;
                        KV_HIP_BRK(hipEventRecord(q->ev_free[slot], q->s_compute));
                        if (sp.kind == KV_V && ext_k_slot >= 0) KV_HIP_BRK(hipEventRecord(q->ev_free[ext_k_slot], q->s_compute));
                    }
                }
                if (serialize) KV_HIP_BRK(hipStreamSynchronize(q->s_compute));
            }
        }
    }

    // Drain: every outstanding command, every kernel, every host copy.
    hipError_t e1 = hipSuccess;
    for (int k = 0; k < kMaxCopyStreams; ++k) {
        hipError_t ek = hipStreamSynchronize(q->s_copy[k]);
        if (ek != hipSuccess) e1 = ek;
    }
    hipError_t e2 = hipStreamSynchronize(q->s_compute);
    // every issued transfer has landed: harvest the rest (offload: this starts their memcpy hops; after an error
    // the events may not all be usable, and the hops of what was issued are started directly)
    if (err != KV_OK || harvest_until(n_issued) != KV_OK) {
        for (; offload_dir && n_waited < n_issued; ++n_waited)
            if (spans[chunks[n_waited].span].path == KV_PATH_PAGECACHE)
                fan_out(n_waited, host_ptr(chunks[n_waited]), bounce_ptr(n_waited), chunks[n_waited].bytes);
    }
    for (auto &e : q->ring) spin_until_zero(e.pending);
    if (err == KV_OK && (e1 != hipSuccess || e2 != hipSuccess)) {
        kvb::set_hip_error((int)(e1 != hipSuccess ? e1 : e2));
        err = KV_EHIP;
    }
    for (int g = 0; g < 2; ++g)
        if (group_t0[g] >= 0 && group_t1[g] < 0) group_t1[g] = now_s();  // harvested by the drain
    if (stats) {
        stats->group_seconds[0] = group_t0[0] >= 0 ? group_t1[0] - group_t0[0] : 0.0;
        stats->group_seconds[1] = group_t0[1] >= 0 ? group_t1[1] - group_t0[1] : 0.0;
        stats->max_in_flight = max_in_flight;
        stats->lba_seq_breaks = sched.lba_seq_breaks;
        stats->host_copy_wait_s = host_wait_s;
        stats->harvest_wait_s = harvest_wait_s;
        stats->n_traced = (uint32_t)n_traced;
        stats->pace_GBps = q->link[pace_dir].rate / 1e9;
        if (time_kernels && err == KV_OK) {
            for (size_t i = 0; i < timing_kind.size(); ++i) {
                float ms = 0.f;
                if (hipEventElapsedTime(&ms, q->timing[2 * i], q->timing[2 * i + 1]) == hipSuccess)
                    stats->kernel_ms[timing_kind[i]] += ms;
            }
        }
        stats->wall_s = std::chrono::duration<double>(std::chrono::steady_clock::now() - t_start).count();
    }
    return err;
}

// ------------------------------------------------------------------------------------------------
// Decode append.
extern "C" int kv_append_tokens(kv_plan_t *p, int layer_begin, int layer_end, const kv_view_t *view, void *lba_region,
                                size_t region_bytes, void *pageable, size_t pageable_bytes, void *caller_stream,
                                kv_append_stats_t *stats)
{
    if (!p || !view || !view->seq_lens_host) return KV_EINVAL;
    if (layer_begin < 0 || layer_end > p->L || layer_begin > layer_end || layer_end > view->n_layers) return KV_ERANGE;
    if (stats) std::memset(stats, 0, sizeof(*stats));
    if (layer_begin == layer_end) return KV_OK;
    const uint64_t sec = (uint64_t)p->sector, rb = p->row_bytes;
    const int nseq = p->mode == KV_TOKEN_MAJOR ? 1 : p->B;
    for (int b = 0; b < p->B; ++b) {
        const int len = view->seq_lens_host[b];
        if (len < 1 || len > p->cap[b]) return KV_ERANGE;
        if (p->mode == KV_TOKEN_MAJOR && len != view->seq_lens_host[0]) return KV_EINVAL;
    }
    bool any_direct = false, any_pc = false;
    for (int l = layer_begin; l < layer_end; ++l) (l < p->n1 ? any_pc : any_direct) = true;
    if (any_direct && (!lba_region || region_bytes < p->region_bytes_needed)) return lba_region ? KV_ENOSPC : KV_EINVAL;
    if (any_pc && (!pageable || pageable_bytes < p->pageable_bytes_needed)) return pageable ? KV_ENOSPC : KV_EINVAL;

    const size_t n_rows = (size_t)(layer_end - layer_begin) * 2 * (size_t)nseq;
    const size_t total = n_rows * rb;
    int rc = ensure_pipeline(p, 1, kvb::round_up(total, 4096), 1, 0, false, 0, 0, 0);
    if (rc != KV_OK) return rc;
    kv_pipeline *q = p->pipe;
    if (q->append_host_bytes < total) {
        if (q->append_host) KV_HIP(hipHostFree(q->append_host));
        q->append_host = nullptr; q->append_host_bytes = 0;
        KV_HIP(hipHostMalloc(&q->append_host, total, hipHostMallocDefault));
        q->append_host_bytes = total;
    }
    const size_t n_entries = (size_t)p->L * 2 * (size_t)nseq;
    if (q->tail_sector.size() != n_entries) {
        q->tail_sector.assign(n_entries, -1);
        q->tail_img.assign(n_entries * sec, 0);
    }
    // images taken from other host buffers say nothing about these
    if ((any_direct && q->tail_region != lba_region) || (any_pc && q->tail_pageable != pageable)) kvb::forget_tail_images(q);
    if (any_direct) q->tail_region = lba_region;
    if (any_pc) q->tail_pageable = pageable;
    rc = order_after_caller(q, caller_stream);
    if (rc != KV_OK) return rc;

    // GPU side: the new row of every tensor (and sequence) in extent order, then one transfer
    rc = kvb::pack_last_rows(p, view, layer_begin, layer_end, q->staging, q->staging_bytes, q->s_compute);
    if (rc != KV_OK) { (void)hipStreamSynchronize(q->s_compute); return rc; }
    KV_HIP(hipMemcpyAsync(q->append_host, q->staging, total, hipMemcpyDeviceToHost, q->s_compute));
    KV_HIP(hipStreamSynchronize(q->s_compute));

    // Host side: Alg. 2 with i0 = len-1 gives the row's byte range; the write command carries whole
    // sectors, so a row that starts inside a sector is merged with that sector's earlier bytes
    // (read-modify-write; the sector image is kept for the next append) and the rest is zeros.
    std::vector<char> tmp;
    size_t idx = 0;
    for (int l = layer_begin; l < layer_end; ++l)
        for (int kind = 0; kind < 2; ++kind)
            for (int b = 0; b < nseq; ++b, ++idx) {
                const int n = 2 * l + kind;
                const bool direct = p->ext[n].path == KV_PATH_DIRECT;
                const uint64_t a = (uint64_t)(view->seq_lens_host[b] - 1) * rb, e = a + rb;
                const uint64_t sec0 = a / sec, sec1 = kvb::ceil_div(e, sec), nsec = sec1 - sec0;
                const uint64_t off = kvb::extent_host_off(p, n) + p->seq_base[b] * sec + sec0 * sec;
                if (off + nsec * sec > (direct ? region_bytes : pageable_bytes)) return KV_ENOSPC;
                char *host = (char *)(direct ? lba_region : pageable) + off;
                const size_t entry = ((size_t)n * nseq) + (size_t)b;
                tmp.assign(nsec * sec, 0);
                const uint64_t head = a - sec0 * sec;
                if (head > 0) {
                    if (q->tail_sector[entry] == (int64_t)sec0) {
                        std::memcpy(tmp.data(), q->tail_img.data() + entry * sec, head);
                    } else {
                        std::memcpy(tmp.data(), host, head);  // the read of the read-modify-write
                        if (stats) stats->n_rmw_reads++;
                    }
                }
                std::memcpy(tmp.data() + head, (char *)q->append_host + idx * rb, rb);
                std::memcpy(host, tmp.data(), nsec * sec);    // write command: nlb = nsec - 1
                if (e % sec != 0) {
                    std::memcpy(q->tail_img.data() + entry * sec, tmp.data() + (nsec - 1) * sec, sec);
                    q->tail_sector[entry] = (int64_t)(sec1 - 1);
                } else {
                    q->tail_sector[entry] = -1;
                }
                if (stats) { stats->n_cmds++; stats->blocks_written += nsec; }
            }
    return KV_OK;
}
