// Host-side context of the library (not part of the ABI).
#pragma once

#include <cstdlib>
#include <cstring>
#include <string>
#include <vector>

#include "ob_internal.h"

// Growable host array of the graph store.  In a context that owns a device arena the memory is
// page-locked (hipHostMalloc), so that the upload copies straight from where the nodes were
// written; a host-only context (no arena, no GPU) uses ordinary memory.  Capacity is kept
// across graphs, so a training loop stops allocating after its first few minibatches.
template <typename T> struct HostVec {
    T *p = nullptr;
    size_t n = 0, cap = 0;
    bool pinned = false;
    HostVec() = default;
    HostVec(const HostVec &) = delete;
    HostVec &operator=(const HostVec &) = delete;
    ~HostVec() { release(); }
    void release()
    {
        if (p) { if (pinned) (void)hipHostFree(p); else free(p); }
        p = nullptr; n = cap = 0;
    }
    // false when memory cannot be had; the old contents stay valid then
    bool reserve(size_t want, bool pin)
    {
        if (want <= cap) return true;
        size_t c = cap ? cap : 1024;
        while (c < want) c *= 2;
        T *q = nullptr;
        if (pin) { if (hipHostMalloc((void **)&q, c * sizeof(T), hipHostMallocDefault) != hipSuccess) { (void)hipGetLastError(); return false; } }
        else q = (T *)malloc(c * sizeof(T));
        if (!q) return false;
        if (n) memcpy(q, p, n * sizeof(T));
        if (p) { if (pinned) (void)hipHostFree(p); else free(p); }
        p = q; cap = c; pinned = pin;
        return true;
    }
    size_t size() const { return n; }
    bool empty() const { return n == 0; }
    T *data() { return p; }
    const T *data() const { return p; }
    T &operator[](size_t i) { return p[i]; }
    const T &operator[](size_t i) const { return p[i]; }
    void clear() { n = 0; }
};

struct HostParam {
    int rows, cols;
    float *data;   // device, inside the arena
    float *grad;   // device, inside the arena
    u32 *marks;    // device: [0] dense gradient written, [1] number of touched rows (see ParamDesc)
    u32 *touched;  // device: rows that LOOKUP gradients were added to
    u32 *row_flag; // device: one word per row, 1 = listed in `touched`
};

struct ob_ctx;

// One later evaluation of a graph that grew after it was evaluated (Section 3.1): the nodes
// [n0, n1) as a graph of their own in a context of their own, whose first proxy.size() nodes are
// leaves that hold copies of the earlier values the new nodes read.
struct Stage {
    ob_ctx *c = nullptr;
    u32 n0 = 0, n1 = 0;
    std::vector<u32> proxy;     // ascending ids of the earlier nodes; the local id of proxy[i] is i
    std::vector<u32> lists;     // host copy of the fill lists (kept while the copy to the device may be in flight)
    u32 *lists_dev = nullptr;   // the same lists on the device: source ids | payload offsets | dimensions, proxy.size() each
};

struct ob_ctx {
    // caller-owned resources
    char *arena = nullptr;
    size_t arena_bytes = 0;
    hipStream_t stream = nullptr;        // execution: forward, backward, reads
    hipStream_t sched_stream = nullptr;  // upload + scheduling (same as `stream` unless set apart)
    ob_ctx *parent = nullptr;            // forked contexts share the parent's parameters
    int mode = 1;      // OB_BYDEPTH
    int launch = 0;    // OB_LAUNCH_STREAM
    int fuse = 2;      // launch fusion level: 0 off, 1 fused with early placement, 2 fused with late placement
    std::string err;

    // arena bump allocator: [0, persist_top) parameters; [persist_top, top) current graph
    size_t persist_top = 0;
    size_t top = 0;

    // parameters
    std::vector<HostParam> params;
    ParamDesc *params_dev = nullptr;   // in arena, uploaded lazily
    bool params_dirty = true;
    bool params_frozen = false;        // set by the first graph upload
    std::vector<PTile> wtiles, btiles; // static tiles of the deferred dW / db kernels
    PTile *wtiles_dev = nullptr, *btiles_dev = nullptr;
    float *wpart_dev = nullptr;        // partial dW blocks of the workgroups that share a tile
    float *bpart_dev = nullptr;        // partial db sums, 256 floats per (bias tile, run)
    int max_param_rows = 1;
    std::vector<std::vector<float>> pending;      // host copies of parameter data not yet on the device
    std::vector<u8> params_used_w, params_used_b; // parameter appeared as a MATVEC matrix / bias

    // host graph store: in_off always holds size(op) + 1 entries
    HostVec<u8> op;
    HostVec<u32> out_dim, in_off, in_idx;
    HostVec<i32> param, bias, aux0, aux1;
    HostVec<float> payload;
    std::vector<u32> manual;           // OB_MANUAL: the caller's batch label per node (empty = none given)
    u32 manual_max = 0;                // largest label
    u32 n_items_total = 0;             // parameter-use items (MATVEC matrix / bias uses, LOOKUPs) of the whole graph
    u64 sum_out_dim = 0;               // bounds the tile lists
    u32 max_arity = 0;
    u32 n_concat = 0;                  // CONCAT nodes in the graph store
    bool concat_views = true;          // CONCAT batches that only matrix products read are not copied
    bool uncopied_filled = false;      // their rows have been written after all (somebody read values)
    u64 sum_mv_d32 = 0, sum_mv_k32 = 0; // sums over MATVEC nodes of rows/32+1 and cols/32+1 (bound the GEMM tiles)
    size_t graph_top = 0;              // arena top right after the uploaded graph image

    // device state of the current graph
    void *pinned = nullptr;            // staging for the batch labels of manual batching
    size_t pinned_bytes = 0;
    bool uploaded = false;
    bool image_stale = false;          // nodes were added behind a live evaluation: the device image lacks them
    std::vector<Stage> stages;         // evaluations after the first, in order (empty: one schedule covers all)
    bool is_stage = false;             // this context is a Stage's own
    std::vector<ob_ctx *> stage_pool;  // retired stage contexts (events and pinned buffers are kept for the next stage)
    u32 n_sched = 0;                   // nodes covered by the last schedule (0 = none)
    bool sched_pending = false;        // scheduling is queued on the GPU, its results are not read yet
    u32 hdr_window = 0, n_items_sched = 0;
    u32 depth_spin_limit = 1u << 21;   // idle polls a range of the partitioned depth pass allows itself before it gives up
    bool depth_partitioned = false;    // the last schedule used the partitioned depth pass
    bool force_frontier = false;       // schedule with the single-workgroup depth pass (retry after a range gave up)
    int n_depth_retries = 0;           // schedules of this context that had to be repeated that way
    bool forward_done = false, backward_done = false;
    Tables T{};
    SchedHeader hdr{};
    std::vector<SlotRec> slots;   // host mirror of the per-slot launch table (n_slots + 1 entries)
    void *scratch = nullptr;           // scan / sort scratch in the arena
    u64 *key_a = nullptr, *key_b = nullptr;
    u32 *val_a = nullptr, *val_b = nullptr;
    u32 *tmp_u32_a = nullptr, *tmp_u32_b = nullptr;   // n+1 words each
    Lay *lay_in = nullptr, *lay_total = nullptr;
    u32 *scalars = nullptr;            // small device scalars
    void *hdr_pinned = nullptr;        // pinned host mirror for the header + step tables
    size_t hdr_pinned_bytes = 0;

    // events / stats
    hipEvent_t ev[10] = {};
    bool ev_ok = false;
    float ms_upload = 0, ms_schedule = 0, ms_forward = 0, ms_backward = 0, ms_param_grads = 0, ms_graph = 0;
    int n_launch_fwd = 0, n_launch_bwd = 0, n_launch_sched = 0;
    int n_launch_bwd_steps = 0;        // launches of the backward step kernel alone (n_launch_bwd also counts the root and parameter kernels)
    size_t upload_bytes = 0;

    // hipGraph of the per-step launches (rebuilt per schedule)
    hipGraph_t graph_fwd = nullptr, graph_bwd = nullptr;
    hipGraphExec_t gexec_fwd = nullptr, gexec_bwd = nullptr;
};

int ctx_fail(ob_ctx *ctx, int code, const char *fmt, ...);
#define HIP_TRY(ctx, expr)                                                                   \
    do {                                                                                     \
        hipError_t _e = (expr);                                                              \
        if (_e != hipSuccess)                                                                \
            return ctx_fail((ctx), -7, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(_e), \
                            __FILE__, __LINE__);                                             \
    } while (0)

// Bump allocation inside the caller's arena (256-byte aligned); nullptr when it does not fit.
void *arena_alloc(ob_ctx *ctx, size_t bytes);
template <typename T> inline T *arena_array(ob_ctx *ctx, size_t count)
{
    return (T *)arena_alloc(ctx, count * sizeof(T));
}
