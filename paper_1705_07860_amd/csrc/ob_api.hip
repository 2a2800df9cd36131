// C ABI of the library (see include/ob.h): host-side graph store with validation at add time,
// upload, and the forward / backward / read entry points.
#include "../../include/ob.h"
#include "ob_ctx.h"

#include <algorithm>
#include <chrono>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <condition_variable>
#include <functional>
#include <mutex>
#include <new>
#include <thread>

static std::string g_create_error;

// Three helper threads for the bulk hand-over of large graphs, started on first use and kept for
// the life of the process (starting threads per call costs more than the work they take over).
// One job at a time; the caller runs part 0 itself and waits for parts 1..3.
namespace {
struct BulkPool {
    static constexpr int HELPERS = 3;
    std::mutex call_m;                 // one bulk call at a time uses the pool
    std::mutex m;
    std::condition_variable cv, done_cv;
    const std::function<void(int)> *job = nullptr;
    unsigned long gen = 0;
    int pending = 0;
    BulkPool()
    {
        for (int t = 1; t <= HELPERS; ++t)
            std::thread([this, t] {
                unsigned long seen = 0;
                for (;;) {
                    const std::function<void(int)> *j;
                    {
                        std::unique_lock<std::mutex> lk(m);
                        cv.wait(lk, [&] { return gen != seen; });
                        seen = gen;
                        j = job;
                    }
                    (*j)(t);
                    {
                        std::lock_guard<std::mutex> lk(m);
                        if (--pending == 0) done_cv.notify_one();
                    }
                }
            }).detach();
    }
    void run(const std::function<void(int)> &f)
    {
        std::lock_guard<std::mutex> call(call_m);
        {
            std::lock_guard<std::mutex> lk(m);
            job = &f;
            pending = HELPERS;
            ++gen;
        }
        cv.notify_all();
        f(0);
        std::unique_lock<std::mutex> lk(m);
        done_cv.wait(lk, [&] { return pending == 0; });
    }
};
BulkPool &bulk_pool()
{
    static BulkPool *p = new BulkPool();   // never destroyed: its threads live until the process ends
    return *p;
}
}  // namespace

int ctx_fail(ob_ctx *ctx, int code, const char *fmt, ...)
{
    char buf[512];
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(buf, sizeof buf, fmt, ap);
    va_end(ap);
    if (ctx) ctx->err = buf; else g_create_error = buf;
    return code;
}

static inline size_t up256(size_t x) { return (x + 255) & ~(size_t)255; }

void *arena_alloc(ob_ctx *ctx, size_t bytes)
{
    const size_t need = up256(bytes ? bytes : 1);
    if (ctx->top + need > ctx->arena_bytes) return nullptr;
    void *p = ctx->arena + ctx->top;
    ctx->top += need;
    return p;
}

#define CHECK_CTX(ctx) do { if (!(ctx)) return OB_E_ARG; } while (0)

extern "C" {

const char *ob_last_error(ob_ctx *ctx) { return ctx ? ctx->err.c_str() : g_create_error.c_str(); }

int ob_ctx_create(void *arena_dev, size_t arena_bytes, void *hip_stream, ob_ctx **out)
{
    if (!out) return ctx_fail(nullptr, OB_E_ARG, "ob_ctx_create: out is null");
    if (((uintptr_t)arena_dev & 255u) != 0) return ctx_fail(nullptr, OB_E_ARG, "arena must be 256-byte aligned");
    ob_ctx *c = new (std::nothrow) ob_ctx();
    if (!c) return ctx_fail(nullptr, OB_E_OOM, "out of host memory");
    c->arena = (char *)arena_dev;
    c->arena_bytes = arena_dev ? arena_bytes : 0;
    c->stream = (hipStream_t)hip_stream;
    c->sched_stream = c->stream;
    *out = c;
    return OB_OK;
}

static int params_to_device(ob_ctx *ctx);

int ob_ctx_fork(ob_ctx *parent, void *arena_dev, size_t arena_bytes, void *hip_stream, ob_ctx **out)
{
    if (!parent) return OB_E_ARG;
    if (!out || !arena_dev) return ctx_fail(parent, OB_E_ARG, "ob_ctx_fork: null argument");
    if (int rc = params_to_device(parent)) return rc;
    ob_ctx *c = nullptr;
    if (int rc = ob_ctx_create(arena_dev, arena_bytes, hip_stream, &c)) return rc;
    c->parent = parent;
    c->params = parent->params;            // same device storage: values and gradients are shared
    c->max_param_rows = parent->max_param_rows;
    c->mode = parent->mode; c->launch = parent->launch; c->fuse = parent->fuse;
    c->params_dirty = true;
    *out = c;
    return OB_OK;
}

static void drop_stages(ob_ctx *ctx);
static int fill_uncopied(ob_ctx *u, hipStream_t s);

int ob_ctx_destroy(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    drop_stages(ctx);
    for (ob_ctx *c : ctx->stage_pool) (void)ob_ctx_destroy(c);
    ctx->stage_pool.clear();
    if (ctx->uploaded) { (void)hipStreamSynchronize(ctx->sched_stream); (void)hipStreamSynchronize(ctx->stream); }
    if (ctx->gexec_fwd) (void)hipGraphExecDestroy(ctx->gexec_fwd);
    if (ctx->gexec_bwd) (void)hipGraphExecDestroy(ctx->gexec_bwd);
    if (ctx->graph_fwd) (void)hipGraphDestroy(ctx->graph_fwd);
    if (ctx->graph_bwd) (void)hipGraphDestroy(ctx->graph_bwd);
    if (ctx->ev_ok) for (auto &e : ctx->ev) (void)hipEventDestroy(e);
    if (ctx->pinned) (void)hipHostFree(ctx->pinned);
    if (ctx->hdr_pinned) (void)hipHostFree(ctx->hdr_pinned);
    delete ctx;
    return OB_OK;
}

static int forget_evaluation(ob_ctx *ctx);
static int wait_own_work(ob_ctx *ctx);
static u32 evaluated_upto(const ob_ctx *ctx);
static int stage_forward(ob_ctx *ctx, u32 n0, u32 n1);
static int staged_backward(ob_ctx *ctx, u32 node);
constexpr int STAGED_FALLBACK = 1;   // staged_backward cannot serve: evaluate everything again as one graph
static int stage_schedule_read(ob_ctx *ctx, int *n_batches, int *batch_depth, uint64_t *batch_sig, int *batch_off,
                               int *node_ids, size_t cap_batches, size_t cap_nodes);

int ob_ctx_set_mode(ob_ctx *ctx, int mode)
{
    CHECK_CTX(ctx);
    if (mode != OB_NOBATCH && mode != OB_BYDEPTH && mode != OB_BYAGENDA && mode != OB_MANUAL)
        return ctx_fail(ctx, OB_E_ARG, "unknown mode %d", mode);
    if (mode != ctx->mode && ctx->n_sched)
        if (int rc = forget_evaluation(ctx)) return rc;
    ctx->mode = mode;
    return OB_OK;
}

int ob_ctx_set_schedule_stream(ob_ctx *ctx, void *hip_stream)
{
    CHECK_CTX(ctx);
    if (ctx->uploaded) return ctx_fail(ctx, OB_E_STATE, "set the schedule stream before the first upload of a graph");
    ctx->sched_stream = (hipStream_t)hip_stream;
    return OB_OK;
}

int ob_stream_create_on_cus(int first_cu, int n_cus, void **hip_stream_out)
{
    if (!hip_stream_out) return ctx_fail(nullptr, OB_E_ARG, "ob_stream_create_on_cus: no place for the stream");
    *hip_stream_out = nullptr;
    int dev = 0, count = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&count, hipDeviceAttributeMultiprocessorCount, dev);
    if (e != hipSuccess) return ctx_fail(nullptr, OB_E_HIP, "ob_stream_create_on_cus: %s", hipGetErrorString(e));
    if (first_cu < 0 || n_cus <= 0 || first_cu + n_cus > count)
        return ctx_fail(nullptr, OB_E_ARG, "ob_stream_create_on_cus: units [%d, %d) of a device with %d", first_cu, first_cu + n_cus, count);
    std::vector<uint32_t> mask((size_t)(count + 31) / 32, 0u);
    for (int b = first_cu; b < first_cu + n_cus; ++b) mask[(size_t)b / 32] |= 1u << (b % 32);
    hipStream_t s = nullptr;
    e = hipExtStreamCreateWithCUMask(&s, (uint32_t)mask.size(), mask.data());
    if (e != hipSuccess) return ctx_fail(nullptr, OB_E_HIP, "hipExtStreamCreateWithCUMask: %s", hipGetErrorString(e));
    *hip_stream_out = (void *)s;
    return OB_OK;
}

int ob_stream_destroy(void *hip_stream)
{
    if (!hip_stream) return OB_OK;
    const hipError_t e = hipStreamDestroy((hipStream_t)hip_stream);
    if (e != hipSuccess) return ctx_fail(nullptr, OB_E_HIP, "hipStreamDestroy: %s", hipGetErrorString(e));
    return OB_OK;
}

int ob_ctx_set_fusion(ob_ctx *ctx, int on)
{
    CHECK_CTX(ctx);
    if (on < 0 || on > 2) return ctx_fail(ctx, OB_E_ARG, "fusion level %d (0 .. 2)", on);
    ctx->fuse = on;
    return OB_OK;
}

int ob_ctx_set_launch(ob_ctx *ctx, int launch)
{
    CHECK_CTX(ctx);
    if (launch == OB_LAUNCH_PERSISTENT) return ctx_fail(ctx, OB_E_STATE, "persistent launch is not built");
    if (launch != OB_LAUNCH_STREAM && launch != OB_LAUNCH_GRAPH) return ctx_fail(ctx, OB_E_ARG, "unknown launch %d", launch);
    ctx->launch = launch;
    return OB_OK;
}

// ---- parameters ---------------------------------------------------------------------------------

}  // extern "C"

// Parameter data written before the GPU is first touched waits in host copies.
static int params_to_device(ob_ctx *ctx)
{
    if (ctx->pending.empty()) return 0;
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "the context has no device arena");
    for (size_t i = 0; i < ctx->pending.size(); ++i) {
        auto &v = ctx->pending[i];
        if (v.empty()) continue;
        HIP_TRY(ctx, hipMemcpyAsync(ctx->params[i].data, v.data(), v.size() * 4, hipMemcpyHostToDevice, ctx->stream));
        HIP_TRY(ctx, hipMemsetAsync(ctx->params[i].grad, 0, v.size() * 4, ctx->stream));
        HIP_TRY(ctx, hipMemsetAsync(ctx->params[i].marks, 0, 256, ctx->stream));
        HIP_TRY(ctx, hipMemsetAsync(ctx->params[i].row_flag, 0, (size_t)ctx->params[i].rows * 4, ctx->stream));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    ctx->pending.clear();
    return 0;
}

extern "C" {

int ob_param_create(ob_ctx *ctx, int rows, int cols, const float *host_init, int *id)
{
    CHECK_CTX(ctx);
    if (!host_init || !id) return ctx_fail(ctx, OB_E_ARG, "ob_param_create: null argument");
    if (rows <= 0 || cols <= 0) return ctx_fail(ctx, OB_E_DIM, "parameter shape %d x %d", rows, cols);
    if (ctx->parent) return ctx_fail(ctx, OB_E_STATE, "a forked context shares its parent's parameters and cannot create its own");
    if (ctx->top != ctx->persist_top)
        return ctx_fail(ctx, OB_E_STATE, "parameters must be created while no graph is on the device");
    const size_t count = (size_t)rows * cols;
    HostParam p;
    p.rows = rows; p.cols = cols;
    p.data = arena_array<float>(ctx, count);
    p.grad = arena_array<float>(ctx, count);
    p.marks = arena_array<u32>(ctx, 64);
    p.touched = arena_array<u32>(ctx, (size_t)rows);
    p.row_flag = arena_array<u32>(ctx, (size_t)rows);
    if (ctx->arena && (!p.data || !p.grad || !p.marks || !p.touched || !p.row_flag))
        return ctx_fail(ctx, OB_E_OOM, "arena too small for a %d x %d parameter", rows, cols);
    ctx->persist_top = ctx->top;
    ctx->params.push_back(p);
    ctx->pending.resize(ctx->params.size());
    ctx->pending.back().assign(host_init, host_init + count);
    ctx->params_dirty = true;
    if (rows > ctx->max_param_rows) ctx->max_param_rows = rows;
    *id = (int)ctx->params.size() - 1;
    return OB_OK;
}

static int check_param(ob_ctx *ctx, int id)
{
    if (id < 0 || id >= (int)ctx->params.size()) return ctx_fail(ctx, OB_E_BADID, "unknown parameter id %d", id);
    return 0;
}

int ob_param_write(ob_ctx *ctx, int id, const float *host_data)
{
    CHECK_CTX(ctx);
    if (!host_data) return ctx_fail(ctx, OB_E_ARG, "null data");
    if (int rc = check_param(ctx, id)) return rc;
    const size_t count = (size_t)ctx->params[id].rows * ctx->params[id].cols;
    if ((size_t)id < ctx->pending.size() && !ctx->pending[id].empty()) {
        ctx->pending[id].assign(host_data, host_data + count);
        return OB_OK;
    }
    HIP_TRY(ctx, hipMemcpyAsync(ctx->params[id].data, host_data, count * 4, hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return OB_OK;
}

static int param_read_impl(ob_ctx *ctx, int id, float *out, size_t cap, bool grad)
{
    if (!out) return ctx_fail(ctx, OB_E_ARG, "null output");
    if (int rc = check_param(ctx, id)) return rc;
    const size_t count = (size_t)ctx->params[id].rows * ctx->params[id].cols;
    if (cap < count) return ctx_fail(ctx, OB_E_RANGE, "buffer holds %zu of %zu elements", cap, count);
    if (int rc = params_to_device(ctx)) return rc;
    HIP_TRY(ctx, hipMemcpyAsync(out, grad ? ctx->params[id].grad : ctx->params[id].data, count * 4,
                                hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return OB_OK;
}

int ob_param_read(ob_ctx *ctx, int id, float *host_out, size_t cap)
{
    CHECK_CTX(ctx);
    return param_read_impl(ctx, id, host_out, cap, false);
}

int ob_param_grad_read(ob_ctx *ctx, int id, float *host_out, size_t cap)
{
    CHECK_CTX(ctx);
    return param_read_impl(ctx, id, host_out, cap, true);
}

int ob_param_grad_zero(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    if (int rc = params_to_device(ctx)) return rc;
    if (ctx->params_dev && !ctx->params_dirty && !ctx->params.empty()) {
        // the device copy of the parameter table is current: one launch clears every gradient
        size_t max_count = 0;
        for (auto &p : ctx->params) { const size_t c = (size_t)p.rows * p.cols; if (c > max_count) max_count = c; }
        hipError_t e = exec_sgd(ctx->params_dev, (u32)ctx->params.size(), max_count, 0.f, 2, ctx->stream);
        if (e != hipSuccess) return ctx_fail(ctx, OB_E_HIP, "clearing the gradients failed: %s", hipGetErrorString(e));
        return OB_OK;
    }
    // parameters and their gradients are adjacent allocations; zero each gradient block
    for (auto &p : ctx->params) {
        HIP_TRY(ctx, hipMemsetAsync(p.grad, 0, (size_t)p.rows * p.cols * 4, ctx->stream));
        HIP_TRY(ctx, hipMemsetAsync(p.marks, 0, 256, ctx->stream));
        HIP_TRY(ctx, hipMemsetAsync(p.row_flag, 0, (size_t)p.rows * 4, ctx->stream));
    }
    return OB_OK;
}

int ob_param_sgd_step(ob_ctx *ctx, float lr, int zero_grad)
{
    CHECK_CTX(ctx);
    if (int rc = params_to_device(ctx)) return rc;
    if (!ctx->params_dev || ctx->params_dirty)
        return ctx_fail(ctx, OB_E_STATE, "ob_param_sgd_step: no gradients yet (upload a graph and run backward first)");
    if (!(lr == lr)) return ctx_fail(ctx, OB_E_ARG, "learning rate is not a number");
    size_t max_count = 0;
    for (auto &p : ctx->params) { const size_t c = (size_t)p.rows * p.cols; if (c > max_count) max_count = c; }
    hipError_t e = exec_sgd(ctx->params_dev, (u32)ctx->params.size(), max_count, lr, zero_grad ? 1 : 0, ctx->stream);
    if (e != hipSuccess) return ctx_fail(ctx, OB_E_HIP, "sgd step failed: %s", hipGetErrorString(e));
    return OB_OK;
}

// ---- graph definition ----------------------------------------------------------------------------

int ob_graph_new(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    // The graph store and the arena behind the parameters are about to be reused: wait for what
    // this context itself still has in flight (its own events; other contexts on the same streams
    // are not waited for).
    if (int rc = wait_own_work(ctx)) return rc;
    ctx->op.clear(); ctx->out_dim.clear(); ctx->in_off.clear(); ctx->in_idx.clear();
    ctx->param.clear(); ctx->bias.clear(); ctx->aux0.clear(); ctx->aux1.clear(); ctx->payload.clear();
    ctx->n_items_total = 0;
    ctx->manual.clear();
    drop_stages(ctx);
    ctx->image_stale = false;
    ctx->sum_out_dim = 0;
    ctx->max_arity = 0;
    ctx->n_concat = 0;
    ctx->sum_mv_d32 = ctx->sum_mv_k32 = 0;
    ctx->top = ctx->persist_top;
    ctx->uploaded = false;
    ctx->n_sched = 0;
    ctx->sched_pending = false;
    ctx->forward_done = ctx->backward_done = false;
    return OB_OK;
}

int ob_graph_size(ob_ctx *ctx, int *n_nodes, int *n_edges)
{
    CHECK_CTX(ctx);
    if (n_nodes) *n_nodes = (int)ctx->op.size();
    if (n_edges) *n_edges = (int)ctx->in_idx.size();
    return OB_OK;
}

}  // extern "C"

// Validates one node against the graph so far and computes the dimension it implies.
// `n_before` = number of nodes that exist (operands must be smaller).
// Errors go to a sink of the caller's (several threads may validate parts of one bulk call).
struct ErrSink { int code = 0; char msg[256] = {0}; };
static int sink_fail(ErrSink *e, int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(e->msg, sizeof e->msg, fmt, ap);
    va_end(ap);
    e->code = code;
    return code;
}
template <typename Dims>
static inline int validate_node(const std::vector<HostParam> &params, ErrSink *es, u32 n_before, const Dims &dims, int op,
                                const u32 *ins, u32 arity, int param, int bias, int a0, int a1, u32 *dim_out, u32 in_dim_hint)
{
    for (u32 j = 0; j < arity; ++j)
        if (ins[j] >= n_before) return sink_fail(es, OB_E_BADID, "operand id %u of node %u does not exist yet", ins[j], n_before);
    auto pshape_ok = [&](int id) { return id >= 0 && id < (int)params.size(); };
    switch (op) {
    case OB_OP_INPUT:
        if (arity != 0) return sink_fail(es, OB_E_DIM, "INPUT takes no operands");
        if (in_dim_hint == 0) return sink_fail(es, OB_E_DIM, "INPUT of dimension 0");
        *dim_out = in_dim_hint;
        return 0;
    case OB_OP_LOOKUP:
        if (arity != 0) return sink_fail(es, OB_E_DIM, "LOOKUP takes no operands");
        if (!pshape_ok(param)) return sink_fail(es, OB_E_BADID, "unknown table id %d", param);
        if (a0 < 0 || a0 >= params[param].rows) return sink_fail(es, OB_E_RANGE, "row %d outside table of %d rows", a0, params[param].rows);
        *dim_out = (u32)params[param].cols;
        return 0;
    case OB_OP_MATVEC:
        if (arity != 1) return sink_fail(es, OB_E_DIM, "MATVEC takes one operand");
        if (!pshape_ok(param)) return sink_fail(es, OB_E_BADID, "unknown matrix id %d", param);
        if ((u32)params[param].cols != dims[ins[0]])
            return sink_fail(es, OB_E_DIM, "MATVEC: matrix has %d columns, operand has %u elements", params[param].cols, dims[ins[0]]);
        if (bias != -1) {
            if (!pshape_ok(bias)) return sink_fail(es, OB_E_BADID, "unknown bias id %d", bias);
            if (params[bias].cols != 1 || params[bias].rows != params[param].rows)
                return sink_fail(es, OB_E_DIM, "bias must be %d x 1", params[param].rows);
        }
        *dim_out = (u32)params[param].rows;
        return 0;
    case OB_OP_ADD:
    case OB_OP_CMULT:
        if (arity < 1 || (op == OB_OP_CMULT && arity != 2)) return sink_fail(es, OB_E_DIM, "wrong operand count %u", arity);
        for (u32 j = 1; j < arity; ++j)
            if (dims[ins[j]] != dims[ins[0]]) return sink_fail(es, OB_E_DIM, "operand dimensions differ (%u vs %u)", dims[ins[j]], dims[ins[0]]);
        *dim_out = dims[ins[0]];
        return 0;
    case OB_OP_TANH:
    case OB_OP_SIGMOID:
        if (arity != 1) return sink_fail(es, OB_E_DIM, "unary op takes one operand");
        *dim_out = dims[ins[0]];
        return 0;
    case OB_OP_CONCAT: {
        if (arity < 1) return sink_fail(es, OB_E_DIM, "CONCAT needs operands");
        u64 d = 0;
        for (u32 j = 0; j < arity; ++j) d += dims[ins[j]];
        if (d > 0x7fffffffu) return sink_fail(es, OB_E_DIM, "CONCAT too long");
        *dim_out = (u32)d;
        return 0;
    }
    case OB_OP_SLICE:
        if (arity != 1) return sink_fail(es, OB_E_DIM, "SLICE takes one operand");
        if (a0 < 0 || a1 <= a0 || (u32)a1 > dims[ins[0]]) return sink_fail(es, OB_E_RANGE, "slice [%d,%d) outside %u elements", a0, a1, dims[ins[0]]);
        *dim_out = (u32)(a1 - a0);
        return 0;
    case OB_OP_PICK_NLS:
        if (arity != 1) return sink_fail(es, OB_E_DIM, "PICK_NLS takes one operand");
        if (a0 < 0 || (u32)a0 >= dims[ins[0]]) return sink_fail(es, OB_E_RANGE, "label %d outside %u classes", a0, dims[ins[0]]);
        *dim_out = 1;
        return 0;
    case OB_OP_SQNORM:
        if (arity != 1) return sink_fail(es, OB_E_DIM, "SQNORM takes one operand");
        *dim_out = 1;
        return 0;
    default:
        return sink_fail(es, OB_E_ARG, "unknown op %d", op);
    }
}

// Room for `nodes` more nodes, `edges` more operand references and `floats` more payload elements.
// Growing a page-locked array frees the old one, so an upload that may still read it is waited for.
static int store_reserve(ob_ctx *ctx, size_t nodes, size_t edges, size_t floats)
{
    const bool pin = ctx->arena != nullptr;
    const size_t n = ctx->op.size() + nodes, E = ctx->in_idx.size() + edges, P = ctx->payload.size() + floats;
    const bool grows = n + 1 > ctx->in_off.cap || n > ctx->op.cap || E > ctx->in_idx.cap || P > ctx->payload.cap;
    if (grows && ctx->uploaded && ctx->ev_ok) HIP_TRY(ctx, hipEventSynchronize(ctx->ev[1]));
    const bool ok = ctx->op.reserve(n, pin) && ctx->out_dim.reserve(n, pin) && ctx->in_off.reserve(n + 1, pin) &&
                    ctx->in_idx.reserve(E, pin) && ctx->param.reserve(n, pin) && ctx->bias.reserve(n, pin) &&
                    ctx->aux0.reserve(n, pin) && ctx->aux1.reserve(n, pin) && ctx->payload.reserve(P, pin);
    if (!ok) return ctx_fail(ctx, OB_E_OOM, "out of %s host memory for the graph store", pin ? "page-locked" : "");
    if (ctx->in_off.n == 0) { ctx->in_off[0] = 0; ctx->in_off.n = 1; }
    return 0;
}

// extending a graph that was already evaluated keeps the evaluation: the next ob_forward
// evaluates only the new nodes (Section 3.1's lazy evaluation).  A schedule that was never
// executed holds nothing worth keeping.
static int before_append(ob_ctx *ctx, bool *keep)
{
    *keep = ctx->n_sched && ctx->forward_done && !ctx->sched_pending;
    if (ctx->n_sched && !*keep)
        if (int rc = forget_evaluation(ctx)) return rc;
    ctx->manual.clear();   // labels cover the graph they were given for
    return 0;
}

static inline void note_matvec(ob_ctx *ctx, int param, int bias)
{
    ctx->sum_mv_d32 += (u64)ctx->params[param].rows / GT + 1;
    ctx->sum_mv_k32 += (u64)ctx->params[param].cols / DXT + 1;
    if (!ctx->params_used_w[param]) { ctx->params_used_w[param] = 1; ctx->params_dirty = true; }
    if (bias >= 0 && !ctx->params_used_b[bias]) { ctx->params_used_b[bias] = 1; ctx->params_dirty = true; }
}

static int append_node(ob_ctx *ctx, int op, const u32 *ins, u32 arity, int param, int bias, int a0, int a1, u32 dim)
{
    bool keep;
    if (int rc = before_append(ctx, &keep)) return rc;
    if (ctx->op.size() >= 0x7ffffff0u) return ctx_fail(ctx, OB_E_RANGE, "too many nodes");
    if (int rc = store_reserve(ctx, 1, arity, 0)) return rc;
    const size_t v = ctx->op.n, e0 = ctx->in_idx.n;
    ctx->op[v] = (u8)op; ctx->out_dim[v] = dim;
    for (u32 j = 0; j < arity; ++j) ctx->in_idx[e0 + j] = ins[j];
    ctx->in_idx.n = e0 + arity;
    ctx->in_off[v + 1] = (u32)ctx->in_idx.n;
    ctx->param[v] = param; ctx->bias[v] = bias; ctx->aux0[v] = a0; ctx->aux1[v] = a1;
    ctx->op.n = ctx->out_dim.n = ctx->param.n = ctx->bias.n = ctx->aux0.n = ctx->aux1.n = v + 1;
    ctx->in_off.n = v + 2;
    const u32 items = (op == OB_OP_MATVEC) ? (1u + (bias >= 0 ? 1u : 0u)) : (op == OB_OP_LOOKUP ? 1u : 0u);
    ctx->n_items_total += items;
    ctx->sum_out_dim += dim;
    if (arity > ctx->max_arity) ctx->max_arity = arity;
    if (op == OB_OP_CONCAT) ++ctx->n_concat;
    if (op == OB_OP_MATVEC) note_matvec(ctx, param, bias);
    if (keep) ctx->image_stale = true; else ctx->uploaded = false;
    return (int)v;
}

static void sync_used_flags(ob_ctx *ctx)
{
    ctx->params_used_w.resize(ctx->params.size(), 0);
    ctx->params_used_b.resize(ctx->params.size(), 0);
}

static int add_one(ob_ctx *ctx, int op, const u32 *ins, u32 arity, int param, int bias, int a0, int a1, u32 in_dim_hint,
                   const float *payload)
{
    sync_used_flags(ctx);
    u32 dim = 0;
    ErrSink es;
    if (int rc = validate_node(ctx->params, &es, (u32)ctx->op.size(), ctx->out_dim, op, ins, arity, param, bias, a0, a1, &dim,
                               in_dim_hint))
        return ctx_fail(ctx, rc, "%s", es.msg);
    if (op == OB_OP_INPUT) {
        if (!payload) return ctx_fail(ctx, OB_E_ARG, "INPUT without data");
        if (int rc = store_reserve(ctx, 0, 0, dim)) return rc;
        a0 = (int)ctx->payload.size();
        memcpy(ctx->payload.data() + ctx->payload.n, payload, (size_t)dim * 4);
        ctx->payload.n += dim;
    }
    return append_node(ctx, op, ins, arity, param, bias, a0, a1, dim);
}

extern "C" {

int ob_add_input(ob_ctx *ctx, int dim, const float *host_data)
{
    CHECK_CTX(ctx);
    if (dim <= 0) return ctx_fail(ctx, OB_E_DIM, "INPUT of dimension %d", dim);
    return add_one(ctx, OB_OP_INPUT, nullptr, 0, -1, -1, 0, 0, (u32)dim, host_data);
}

int ob_add_lookup(ob_ctx *ctx, int table, int row)
{
    CHECK_CTX(ctx);
    return add_one(ctx, OB_OP_LOOKUP, nullptr, 0, table, -1, row, 0, 0, nullptr);
}

int ob_add_matvec(ob_ctx *ctx, int w, int bias_or_neg1, int x)
{
    CHECK_CTX(ctx);
    if (x < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
    if (bias_or_neg1 < -1) return ctx_fail(ctx, OB_E_BADID, "bias id %d", bias_or_neg1);
    const u32 in = (u32)x;
    return add_one(ctx, OB_OP_MATVEC, &in, 1, w, bias_or_neg1, 0, 0, 0, nullptr);
}

int ob_add_unary(ob_ctx *ctx, int op, int x)
{
    CHECK_CTX(ctx);
    if (op != OB_OP_TANH && op != OB_OP_SIGMOID) return ctx_fail(ctx, OB_E_ARG, "op %d is not unary", op);
    if (x < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
    const u32 in = (u32)x;
    return add_one(ctx, op, &in, 1, -1, -1, 0, 0, 0, nullptr);
}

int ob_add_nary(ob_ctx *ctx, int op, int k, const int *xs)
{
    CHECK_CTX(ctx);
    if (op != OB_OP_ADD && op != OB_OP_CMULT && op != OB_OP_CONCAT) return ctx_fail(ctx, OB_E_ARG, "op %d is not n-ary", op);
    if (k <= 0 || !xs) return ctx_fail(ctx, OB_E_ARG, "no operands");
    std::vector<u32> ins((size_t)k);
    for (int j = 0; j < k; ++j) {
        if (xs[j] < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
        ins[j] = (u32)xs[j];
    }
    return add_one(ctx, op, ins.data(), (u32)k, -1, -1, 0, 0, 0, nullptr);
}

int ob_add_slice(ob_ctx *ctx, int x, int lo, int hi)
{
    CHECK_CTX(ctx);
    if (x < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
    const u32 in = (u32)x;
    return add_one(ctx, OB_OP_SLICE, &in, 1, -1, -1, lo, hi, 0, nullptr);
}

int ob_add_pick_nls(ob_ctx *ctx, int x, int label)
{
    CHECK_CTX(ctx);
    if (x < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
    const u32 in = (u32)x;
    return add_one(ctx, OB_OP_PICK_NLS, &in, 1, -1, -1, label, 0, 0, nullptr);
}

int ob_add_sqnorm(ob_ctx *ctx, int x)
{
    CHECK_CTX(ctx);
    if (x < 0) return ctx_fail(ctx, OB_E_BADID, "negative operand id");
    const u32 in = (u32)x;
    return add_one(ctx, OB_OP_SQNORM, &in, 1, -1, -1, 0, 0, 0, nullptr);
}

int ob_add_bulk(ob_ctx *ctx, int n, const uint8_t *op, const uint32_t *out_dim, const uint32_t *in_off,
                const uint32_t *in_idx, const int32_t *param, const int32_t *bias, const int32_t *aux0,
                const int32_t *aux1, const float *payload, size_t payload_len)
{
    CHECK_CTX(ctx);
    if (n <= 0) return ctx_fail(ctx, OB_E_ARG, "n = %d", n);
    if (!op || !out_dim || !in_off || !param || !bias || !aux0 || !aux1) return ctx_fail(ctx, OB_E_ARG, "null array");
    sync_used_flags(ctx);
    const u32 n0 = (u32)ctx->op.size();
    if ((u64)n0 + (u64)n >= 0x7ffffff0ull) return ctx_fail(ctx, OB_E_RANGE, "too many nodes");
    if (in_off[0] != 0) return ctx_fail(ctx, OB_E_ARG, "in_off[0] must be 0");
    // The new nodes are validated and written behind the end of the graph store, in up to four
    // threads over ranges of node ids, and only a call that found no error moves the end (nothing
    // is appended on error).  An operand's dimension is the stored one for a node that already
    // exists and the caller's out_dim for an earlier node of this call: every node's out_dim is
    // checked against the dimension its operation implies, so if all checks pass all were right.
    const size_t E_new = in_off[n];
    if (E_new && !in_idx) return ctx_fail(ctx, OB_E_ARG, "null in_idx");
    if (int rc = store_reserve(ctx, (size_t)n, E_new, payload_len)) return rc;
    const u32 pay0 = (u32)ctx->payload.size(), e0 = (u32)ctx->in_idx.size();
    struct DimView {
        const u32 *old; u32 n0; const u32 *fresh;
        u32 operator[](u32 u) const { return u < n0 ? old[u] : fresh[u - n0]; }
    } dims{ctx->out_dim.data(), n0, out_dim};
    struct Part {
        ErrSink es; u64 sum_dim = 0, mv_d32 = 0, mv_k32 = 0; u32 max_ar = 0, items = 0, concats = 0;
        std::vector<u8> used_w, used_b;
    };
    const int n_parts = n >= 32768 ? 1 + BulkPool::HELPERS : 1;
    std::vector<Part> parts((size_t)n_parts);
    const std::vector<HostParam> &params = ctx->params;
    auto work = [&](int t) {
        Part &P = parts[(size_t)t];
        P.used_w.assign(params.size(), 0); P.used_b.assign(params.size(), 0);
        const int a = (int)((long long)n * t / n_parts), b = (int)((long long)n * (t + 1) / n_parts);
        i32 *a0_out = ctx->aux0.data() + n0;
        for (int i = a; i < b; ++i) {
            if (in_off[i + 1] < in_off[i] || in_off[i + 1] > E_new) { sink_fail(&P.es, OB_E_ARG, "in_off not monotone at %d", i); return; }
            const u32 ar = in_off[i + 1] - in_off[i];
            u32 dim = 0, hint = 0;
            const u8 o = op[i];
            if (o == OB_OP_INPUT) {
                hint = out_dim[i];
                if (aux0[i] < 0 || (size_t)aux0[i] + out_dim[i] > payload_len || (!payload && out_dim[i])) {
                    sink_fail(&P.es, OB_E_RANGE, "INPUT payload of node %d outside the payload array", i);
                    return;
                }
            }
            if (validate_node(params, &P.es, n0 + (u32)i, dims, o, in_idx + in_off[i], ar, param[i], bias[i], aux0[i], aux1[i],
                              &dim, hint))
                return;
            if (dim != out_dim[i]) { sink_fail(&P.es, OB_E_DIM, "node %d: out_dim %u but the operation implies %u", i, out_dim[i], dim); return; }
            P.sum_dim += dim;
            if (ar > P.max_ar) P.max_ar = ar;
            a0_out[i] = (o == OB_OP_INPUT) ? (i32)(pay0 + (u32)aux0[i]) : aux0[i];
            if (o == OB_OP_MATVEC) {
                P.items += 1u + (bias[i] >= 0 ? 1u : 0u);
                P.mv_d32 += (u64)params[param[i]].rows / GT + 1;
                P.mv_k32 += (u64)params[param[i]].cols / DXT + 1;
                P.used_w[param[i]] = 1;
                if (bias[i] >= 0) P.used_b[bias[i]] = 1;
            } else if (o == OB_OP_LOOKUP) {
                P.items += 1u;
            } else if (o == OB_OP_CONCAT) {
                ++P.concats;
            }
        }
        // this range's share of the plain copies
        const size_t cnt = (size_t)(b - a);
        memcpy(ctx->op.data() + n0 + a, op + a, cnt);
        memcpy(ctx->out_dim.data() + n0 + a, out_dim + a, cnt * 4);
        memcpy(ctx->param.data() + n0 + a, param + a, cnt * 4);
        memcpy(ctx->bias.data() + n0 + a, bias + a, cnt * 4);
        memcpy(ctx->aux1.data() + n0 + a, aux1 + a, cnt * 4);
        if (e0 == 0) memcpy(ctx->in_off.data() + n0 + 1 + a, in_off + 1 + a, cnt * 4);
        else for (int i = a; i < b; ++i) ctx->in_off[n0 + 1 + (size_t)i] = e0 + in_off[i + 1];
        if (in_off[b] > in_off[a]) memcpy(ctx->in_idx.data() + e0 + in_off[a], in_idx + in_off[a], (size_t)(in_off[b] - in_off[a]) * 4);
        const size_t pa = payload_len * (size_t)t / (size_t)n_parts, pb = payload_len * (size_t)(t + 1) / (size_t)n_parts;
        if (pb > pa) memcpy(ctx->payload.data() + pay0 + pa, payload + pa, (pb - pa) * 4);
    };
    if (n_parts == 1) {
        work(0);
    } else {
        const std::function<void(int)> job = work;
        bulk_pool().run(job);
    }
    for (const Part &P : parts)   // the first failing range holds the first failing node
        if (P.es.code) return ctx_fail(ctx, P.es.code, "%s", P.es.msg);
    bool keep;
    if (int rc = before_append(ctx, &keep)) return rc;
    for (const Part &P : parts) {
        ctx->sum_out_dim += P.sum_dim;
        if (P.max_ar > ctx->max_arity) ctx->max_arity = P.max_ar;
        ctx->n_items_total += P.items;
        ctx->n_concat += P.concats;
        ctx->sum_mv_d32 += P.mv_d32; ctx->sum_mv_k32 += P.mv_k32;
        for (size_t q = 0; q < params.size(); ++q) {
            if (P.used_w[q] && !ctx->params_used_w[q]) { ctx->params_used_w[q] = 1; ctx->params_dirty = true; }
            if (P.used_b[q] && !ctx->params_used_b[q]) { ctx->params_used_b[q] = 1; ctx->params_dirty = true; }
        }
    }
    const size_t n1 = (size_t)n0 + n;
    ctx->op.n = ctx->out_dim.n = ctx->param.n = ctx->bias.n = ctx->aux0.n = ctx->aux1.n = n1;
    ctx->in_off.n = n1 + 1;
    ctx->in_idx.n = e0 + E_new;
    ctx->payload.n = pay0 + payload_len;
    if (keep) ctx->image_stale = true; else ctx->uploaded = false;
    return (int)n0;
}

// ---- upload ---------------------------------------------------------------------------------------

static int ensure_events(ob_ctx *ctx)
{
    if (ctx->ev_ok) return 0;
    for (auto &e : ctx->ev) HIP_TRY(ctx, hipEventCreate(&e));
    ctx->ev_ok = true;
    return 0;
}

static int upload_param_tables(ob_ctx *ctx)
{
    // descriptor array + static tiles of the deferred parameter-gradient kernels (persistent region)
    sync_used_flags(ctx);
    ctx->wtiles.clear(); ctx->btiles.clear();
    std::vector<ParamDesc> desc(ctx->params.size());
    for (size_t p = 0; p < ctx->params.size(); ++p) {
        const HostParam &hp = ctx->params[p];
        desc[p].data = hp.data; desc[p].grad = hp.grad; desc[p].rows = hp.rows; desc[p].cols = hp.cols;
        desc[p].marks = hp.marks; desc[p].touched = hp.touched; desc[p].row_flag = hp.row_flag;
        if (ctx->params_used_w[p]) {
            // Workgroup g of a launch runs on XCD g % 8, and every XCD has its own L2.  A dW tile
            // (i0, j0) reads columns i0.. of every gradient row and columns j0.. of every operand
            // row, so tiles are ordered such that an XCD keeps to one eighth of the gradient
            // columns: the (larger) gradient block is then fetched once instead of once per XCD.
            const int R = (hp.rows + PWTILE - 1) / PWTILE, C = (hp.cols + PWTILE - 1) / PWTILE;
            std::vector<std::vector<PTile>> group(8);
            for (int rt = 0; rt < R; ++rt)
                for (int ct = 0; ct < C; ++ct)
                    group[(size_t)((long long)rt * 8 / R)].push_back(PTile{(i32)p, rt * PWTILE, ct * PWTILE, R * C >= 32 ? 4 : (R * C >= 8 ? 8 : PW_SPLIT_MAX)});
            size_t left = (size_t)R * C;
            std::vector<size_t> next(8, 0);
            while (left) {
                size_t x = ctx->wtiles.size() % 8;
                if (next[x] >= group[x].size()) {     // this XCD's share is used up: take from the fullest other share
                    size_t best = 0, most = 0;
                    for (size_t y = 0; y < 8; ++y)
                        if (group[y].size() - next[y] > most) { most = group[y].size() - next[y]; best = y; }
                    x = best;
                }
                ctx->wtiles.push_back(group[x][next[x]++]);
                --left;
            }
        }
        if (ctx->params_used_b[p])
            for (int i0 = 0; i0 < hp.rows; i0 += 256) {   // pad = runs | first partial block << 8
                ctx->btiles.push_back(PTile{(i32)p, i0, 0, (i32)((u32)PB_SPLIT | ((u32)ctx->btiles.size() * PB_SPLIT) << 8)});
            }
    }
    ctx->params_dev = arena_array<ParamDesc>(ctx, desc.size() + 1);
    ctx->wtiles_dev = arena_array<PTile>(ctx, ctx->wtiles.size() + 1);
    ctx->btiles_dev = arena_array<PTile>(ctx, ctx->btiles.size() + 1);
    // a matrix of few tiles gets more workgroups per tile; pad = runs | first partial block << 8
    size_t n_part = 0;
    for (PTile &t : ctx->wtiles) { const size_t runs = (size_t)t.pad; t.pad = (i32)(runs | (n_part << 8)); n_part += runs; }
    if (n_part >= (1u << 23)) return ctx_fail(ctx, OB_E_RANGE, "too many weight-gradient tiles");
    ctx->wpart_dev = arena_array<float>(ctx, n_part * (size_t)PWTILE * PWTILE + 1);
    ctx->bpart_dev = arena_array<float>(ctx, ctx->btiles.size() * (size_t)PB_SPLIT * 256 + 1);
    if (!ctx->params_dev || !ctx->wtiles_dev || !ctx->btiles_dev || !ctx->wpart_dev || !ctx->bpart_dev)
        return ctx_fail(ctx, OB_E_OOM, "arena too small for parameter tables");
    ctx->persist_top = ctx->top;
    if (!desc.empty())
        HIP_TRY(ctx, hipMemcpyAsync(ctx->params_dev, desc.data(), desc.size() * sizeof(ParamDesc), hipMemcpyHostToDevice, ctx->stream));
    if (!ctx->wtiles.empty())
        HIP_TRY(ctx, hipMemcpyAsync(ctx->wtiles_dev, ctx->wtiles.data(), ctx->wtiles.size() * sizeof(PTile), hipMemcpyHostToDevice, ctx->stream));
    if (!ctx->btiles.empty())
        HIP_TRY(ctx, hipMemcpyAsync(ctx->btiles_dev, ctx->btiles.data(), ctx->btiles.size() * sizeof(PTile), hipMemcpyHostToDevice, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));   // the host vectors may change after return
    ctx->params_dirty = false;
    return 0;
}

int ob_upload(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    if (ctx->uploaded) return OB_OK;
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "the context has no device arena");
    if (ctx->op.empty()) return ctx_fail(ctx, OB_E_STATE, "empty graph");
    if (ctx->n_sched)
        if (int rc = forget_evaluation(ctx)) return rc;
    if (int rc = ensure_events(ctx)) return rc;
    if (int rc = params_to_device(ctx)) return rc;
    ctx->top = ctx->persist_top;
    if (ctx->params_dirty)
        if (int rc = upload_param_tables(ctx)) return rc;
    if (!ctx->hdr_pinned) {
        ctx->hdr_pinned_bytes = 1 << 16;
        HIP_TRY(ctx, hipHostMalloc(&ctx->hdr_pinned, ctx->hdr_pinned_bytes, hipHostMallocDefault));
    }

    const size_t n = ctx->op.size(), E = ctx->in_idx.size(), P = ctx->payload.size();
    // one block of the arena: op | out_dim | in_off | in_idx | param | bias | aux0 | aux1 | payload | labels,
    // each array copied straight from the page-locked graph store
    size_t off[11];
    size_t cur = 0;
    const bool labels = ctx->manual.size() == n;
    const size_t sizes[10] = {n, n * 4, (n + 1) * 4, (E + 1) * 4, n * 4, n * 4, n * 4, n * 4, (P + 1) * 4,
                              labels ? n * 4 : 0};
    for (int i = 0; i < 10; ++i) { off[i] = cur; cur += up256(sizes[i]); }
    off[10] = cur;
    if (labels && n * 4 > ctx->pinned_bytes) {
        if (ctx->pinned) HIP_TRY(ctx, hipHostFree(ctx->pinned));
        ctx->pinned = nullptr;
        ctx->pinned_bytes = n * 4 + n * 2;
        HIP_TRY(ctx, hipHostMalloc(&ctx->pinned, ctx->pinned_bytes, hipHostMallocDefault));
    }
    if (labels) memcpy(ctx->pinned, ctx->manual.data(), n * 4);
    char *dev = (char *)arena_alloc(ctx, cur);
    if (!dev) return ctx_fail(ctx, OB_E_OOM, "arena too small for the graph (%zu bytes)", cur);
    hipStream_t us = ctx->sched_stream;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[0], us));
    const void *src[10] = {ctx->op.data(), ctx->out_dim.data(), ctx->in_off.data(), ctx->in_idx.data(), ctx->param.data(),
                           ctx->bias.data(), ctx->aux0.data(), ctx->aux1.data(), ctx->payload.data(), ctx->pinned};
    const size_t bytes[10] = {n, n * 4, (n + 1) * 4, E * 4, n * 4, n * 4, n * 4, n * 4, P * 4, labels ? n * 4 : 0};
    size_t total = 0;
    for (int i = 0; i < 10; ++i) {
        if (!bytes[i]) continue;
        HIP_TRY(ctx, hipMemcpyAsync(dev + off[i], src[i], bytes[i], hipMemcpyHostToDevice, us));
        total += bytes[i];
    }
    HIP_TRY(ctx, hipEventRecord(ctx->ev[1], us));
    cur = total;
    Tables &T = ctx->T;
    T = Tables{};
    T.op = (const u8 *)(dev + off[0]); T.out_dim = (const u32 *)(dev + off[1]); T.in_off = (const u32 *)(dev + off[2]);
    T.in_idx = (const u32 *)(dev + off[3]); T.param = (const i32 *)(dev + off[4]); T.bias = (const i32 *)(dev + off[5]);
    T.aux0 = (const i32 *)(dev + off[6]); T.aux1 = (const i32 *)(dev + off[7]); T.payload = (const float *)(dev + off[8]);
    T.manual = labels ? (const u32 *)(dev + off[9]) : nullptr;
    T.params = ctx->params_dev;
    T.n_params = (u32)ctx->params.size();
    T.root = 0xffffffffu;
    ctx->upload_bytes = cur;
    ctx->graph_top = ctx->top;
    ctx->uploaded = true;
    return OB_OK;
}

// Manual batching (Section 2): the caller's grouping is checked against the two things any
// batch needs -- operands come from earlier batches, members are the same operation on the same
// shapes and shared parameters (the signature tuple of Section 3.2, compared field by field).
int ob_set_manual_batches(ob_ctx *ctx, const int32_t *batch_of_node, size_t n)
{
    CHECK_CTX(ctx);
    if (!batch_of_node) return ctx_fail(ctx, OB_E_ARG, "null label array");
    if (n != ctx->op.size()) return ctx_fail(ctx, OB_E_ARG, "%zu labels for a graph of %zu nodes", n, ctx->op.size());
    if (n == 0) return ctx_fail(ctx, OB_E_STATE, "empty graph");
    u32 mx = 0;
    for (size_t v = 0; v < n; ++v) {
        if (batch_of_node[v] < 0) return ctx_fail(ctx, OB_E_ARG, "node %zu: negative batch label %d", v, batch_of_node[v]);
        if ((u32)batch_of_node[v] > mx) mx = (u32)batch_of_node[v];
        for (u32 e = ctx->in_off[v]; e < ctx->in_off[v + 1]; ++e)
            if (batch_of_node[ctx->in_idx[e]] >= batch_of_node[v])
                return ctx_fail(ctx, OB_E_ARG, "node %zu (batch %d) reads node %u of batch %d: operands must come from earlier batches",
                                v, batch_of_node[v], ctx->in_idx[e], batch_of_node[ctx->in_idx[e]]);
    }
    // first node of every label, then every node against the first of its label
    std::vector<u32> head((size_t)mx + 1, 0xffffffffu);
    for (size_t v = 0; v < n; ++v) {
        u32 &h = head[(u32)batch_of_node[v]];
        if (h == 0xffffffffu) { h = (u32)v; continue; }
        const u32 ar = ctx->in_off[v + 1] - ctx->in_off[v];
        bool same = ctx->op[v] == ctx->op[h] && ctx->out_dim[v] == ctx->out_dim[h] &&
                    ar == ctx->in_off[h + 1] - ctx->in_off[h] && ctx->param[v] == ctx->param[h] &&
                    ctx->bias[v] == ctx->bias[h];
        if (same && ctx->op[v] == OB_OP_SLICE) same = ctx->aux0[v] == ctx->aux0[h] && ctx->aux1[v] == ctx->aux1[h];
        for (u32 j = 0; same && j < ar; ++j)
            same = ctx->out_dim[ctx->in_idx[ctx->in_off[v] + j]] == ctx->out_dim[ctx->in_idx[ctx->in_off[h] + j]];
        if (!same)
            return ctx_fail(ctx, OB_E_ARG, "nodes %u and %zu of batch %d differ in operation, shapes or shared parameters",
                            h, v, batch_of_node[v]);
    }
    if (ctx->n_sched)
        if (int rc = forget_evaluation(ctx)) return rc;
    ctx->manual.assign((const u32 *)batch_of_node, (const u32 *)batch_of_node + n);
    ctx->manual_max = mx;
    ctx->uploaded = false;
    return OB_OK;
}

// ---- execution ------------------------------------------------------------------------------------

static int schedule_begin(ob_ctx *ctx, int node)
{
    if (node < 0 || node >= (int)ctx->op.size()) return ctx_fail(ctx, OB_E_BADID, "unknown node id %d", node);
    if (ctx->n_sched) {
        if ((u32)node < ctx->n_sched || (u32)node < evaluated_upto(ctx)) return OB_OK;   // already scheduled (or being scheduled)
        // a node beyond the scheduled prefix: schedule the longer prefix from the start
        if (int rc = forget_evaluation(ctx)) return rc;
    }
    if (ctx->mode == OB_MANUAL && ctx->manual.size() != ctx->op.size())
        return ctx_fail(ctx, OB_E_STATE, "manual batching: no batch labels for the current graph (ob_set_manual_batches)");
    if (int rc = ob_upload(ctx)) return rc;
    Tables &T = ctx->T;
    T.n = (u32)node + 1;
    T.E = ctx->in_off[T.n];
    ctx->top = ctx->graph_top;
    ctx->ms_graph = 0;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[7], ctx->sched_stream));
    if (int rc = sched_enqueue(ctx)) return rc;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[9], ctx->sched_stream));
    ctx->n_sched = T.n;
    ctx->sched_pending = true;
    ctx->forward_done = ctx->backward_done = false;
    return OB_OK;
}

static int schedule_end(ob_ctx *ctx)
{
    if (!ctx->sched_pending) return OB_OK;
    ctx->sched_pending = false;
    if (int rc = sched_finish(ctx)) { ctx->n_sched = 0; return rc; }
    return OB_OK;
}

int ob_schedule_async(ob_ctx *ctx, int node)
{
    CHECK_CTX(ctx);
    return schedule_begin(ctx, node);
}

int ob_schedule(ob_ctx *ctx, int node)
{
    CHECK_CTX(ctx);
    if (int rc = schedule_begin(ctx, node)) return rc;
    return schedule_end(ctx);
}

int ob_forward(ob_ctx *ctx, int node)
{
    CHECK_CTX(ctx);
    if (node < 0 || node >= (int)ctx->op.size()) return ctx_fail(ctx, OB_E_BADID, "unknown node id %d", node);
    if (ctx->forward_done && !ctx->sched_pending) {
        const u32 done = evaluated_upto(ctx);
        if ((u32)node < done) return OB_OK;           // already evaluated
        if (!ctx->is_stage && ctx->mode != OB_MANUAL) {
            // Section 3.1: only the nodes that have no value yet are evaluated
            const int rc = stage_forward(ctx, done, (u32)node + 1);
            if (rc != OB_E_OOM) return rc;
            // no room to stack another evaluation behind the earlier ones: evaluate everything again instead
        }
    }
    if (int rc = ob_schedule(ctx, node)) return rc;
    if (ctx->forward_done) return OB_OK;              // already evaluated
    if (ctx->sched_stream != ctx->stream) HIP_TRY(ctx, hipStreamWaitEvent(ctx->stream, ctx->ev[9], 0));
    HIP_TRY(ctx, hipEventRecord(ctx->ev[8], ctx->stream));
    if (int rc = exec_forward(ctx)) return rc;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[3], ctx->stream));
    ctx->forward_done = true;
    ctx->uncopied_filled = false;
    ctx->backward_done = false;
    return OB_OK;
}

int ob_backward(ob_ctx *ctx, int node)
{
    CHECK_CTX(ctx);
    if (!ctx->forward_done) return ctx_fail(ctx, OB_E_STATE, "ob_backward before ob_forward");
    if (!ctx->stages.empty()) {
        // The graph was evaluated in stages.  The backward pass runs stage by stage, last first:
        // what a stage computes for its stand-ins of earlier nodes is handed down to those nodes'
        // owners.  Where that is not possible (see staged_backward) everything evaluated so far is
        // scheduled and evaluated once more as one graph instead.
        const u32 done = evaluated_upto(ctx);
        if (node < 0 || (u32)node >= done) return ctx_fail(ctx, OB_E_BADID, "node %d was not evaluated", node);
        if (ctx->out_dim[node] != 1) return ctx_fail(ctx, OB_E_NOTSCALAR, "node %d has %u elements", node, ctx->out_dim[node]);
        const int rc = staged_backward(ctx, (u32)node);
        if (rc != STAGED_FALLBACK) return rc;
        if (int rc2 = forget_evaluation(ctx)) return rc2;
        if (int rc2 = ob_forward(ctx, (int)done - 1)) return rc2;
    }
    if (node < 0 || (u32)node >= ctx->n_sched) return ctx_fail(ctx, OB_E_BADID, "node %d was not evaluated", node);
    if (ctx->out_dim[node] != 1) return ctx_fail(ctx, OB_E_NOTSCALAR, "node %d has %u elements", node, ctx->out_dim[node]);
    ctx->T.root = (u32)node;
    ctx->T.Gx = nullptr;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[4], ctx->stream));
    if (int rc = exec_backward(ctx)) return rc;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[5], ctx->stream));
    ctx->backward_done = true;
    return OB_OK;
}

// waits until the work this context last enqueued has finished (its own events, not the whole
// stream: other contexts may share the streams)
static int wait_own_work(ob_ctx *ctx)
{
    if (!ctx->uploaded || !ctx->ev_ok) return 0;
    if (ctx->backward_done) HIP_TRY(ctx, hipEventSynchronize(ctx->ev[5]));
    else if (ctx->forward_done) HIP_TRY(ctx, hipEventSynchronize(ctx->ev[3]));
    else if (ctx->n_sched) HIP_TRY(ctx, hipEventSynchronize(ctx->ev[9]));
    else HIP_TRY(ctx, hipEventSynchronize(ctx->ev[1]));
    return 0;
}

// Stage contexts are kept for later stages: creating events and pinned buffers costs more than
// evaluating a small stage.
static void drop_stages(ob_ctx *ctx)
{
    if (ctx->stages.empty()) return;
    // everything the stages queued runs in order on the two streams of this context: when the
    // last stage has finished, all have
    bool waited = wait_own_work(ctx->stages.back().c) == 0;
    for (Stage &st : ctx->stages) {
        if (!st.c) continue;
        if (waited) { st.c->uploaded = false; ctx->stage_pool.push_back(st.c); }
        else (void)ob_ctx_destroy(st.c);   // waits for the streams itself
    }
    ctx->stages.clear();
}

// A retired stage context, set up again over another part of the owner's arena.
static void stage_rebase(ob_ctx *c, ob_ctx *owner, char *arena, size_t bytes)
{
    (void)ob_graph_new(c);   // nothing of it is in flight (see drop_stages), so this only empties the host graph store
    c->arena = arena; c->arena_bytes = bytes;
    c->persist_top = c->top = 0;
    c->stream = owner->stream; c->sched_stream = owner->sched_stream;
    c->mode = owner->mode; c->launch = owner->launch; c->fuse = owner->fuse;
    c->params = owner->params; c->max_param_rows = owner->max_param_rows;
    c->params_used_w.assign(c->params.size(), 0);
    c->params_used_b.assign(c->params.size(), 0);
    c->params_dev = nullptr; c->wtiles_dev = c->btiles_dev = nullptr; c->wpart_dev = nullptr; c->bpart_dev = nullptr;
    c->params_dirty = true;
    c->err.clear();
}

static int forget_evaluation(ob_ctx *ctx)
{
    if (int rc = wait_own_work(ctx)) return rc;
    drop_stages(ctx);
    ctx->sched_pending = false;
    ctx->n_sched = 0;
    ctx->forward_done = ctx->backward_done = false;
    if (ctx->uploaded) ctx->top = ctx->graph_top;
    if (ctx->image_stale) { ctx->uploaded = false; ctx->image_stale = false; }
    return 0;
}

// nodes [0, result) have values
static u32 evaluated_upto(const ob_ctx *ctx)
{
    if (!ctx->forward_done) return 0;
    return ctx->stages.empty() ? ctx->n_sched : ctx->stages.back().n1;
}

// Evaluates the nodes [n0, n1) of a graph whose nodes [0, n0) already have values (Section 3.1:
// a value is computed when it is asked for, and what is computed stays).  The new nodes become a
// graph of their own: every earlier node they read is a leaf of that graph, holding a copy of the
// earlier value, and the new nodes follow in id order.  The graph gets a context of its own over
// the free end of the arena, is scheduled like any other graph (so "depth" counts from the
// leaves of this stage) and executed; earlier values stay where they are.
static int stage_forward(ob_ctx *ctx, u32 n0, u32 n1)
{
    ctx->stages.emplace_back();
    Stage &st = ctx->stages.back();
    st.n0 = n0; st.n1 = n1;
    auto fail = [&](int rc) {   // the caller has put the message into ctx->err
        if (st.c) (void)ob_ctx_destroy(st.c);
        ctx->stages.pop_back();
        return rc;
    };
    auto hip_fail = [&](hipError_t e, const char *what) {
        return fail(ctx_fail(ctx, OB_E_HIP, "%s failed: %s", what, hipGetErrorString(e)));
    };
    // earlier nodes the new ones read
    for (u32 e = ctx->in_off[n0]; e < ctx->in_off[n1]; ++e)
        if (ctx->in_idx[e] < n0) st.proxy.push_back(ctx->in_idx[e]);
    std::sort(st.proxy.begin(), st.proxy.end());
    st.proxy.erase(std::unique(st.proxy.begin(), st.proxy.end()), st.proxy.end());
    const u32 P = (u32)st.proxy.size(), nl = P + (n1 - n0);
    if ((u64)P + (n1 - n0) >= 0x7ffffff0ull) return fail(ctx_fail(ctx, OB_E_RANGE, "too many nodes"));

    // the stage's graph
    std::vector<u8> op(nl, (u8)OB_OP_INPUT);
    std::vector<u32> od(nl), ioff((size_t)nl + 1, 0), iidx;
    std::vector<i32> par(nl, -1), bia(nl, -1), a0(nl, 0), a1(nl, 0);
    std::vector<float> pay;
    u64 pfl = 0;
    for (u32 i = 0; i < P; ++i) {
        od[i] = ctx->out_dim[st.proxy[i]];
        a0[i] = (i32)pfl;
        pfl += od[i];
    }
    if (pfl >= 0x7fffffffull) return fail(ctx_fail(ctx, OB_E_RANGE, "the new nodes read too many earlier elements"));
    pay.assign((size_t)pfl, 0.f);
    iidx.reserve(ctx->in_off[n1] - ctx->in_off[n0]);
    for (u32 v = n0; v < n1; ++v) {
        const u32 l = P + (v - n0);
        op[l] = ctx->op[v]; od[l] = ctx->out_dim[v];
        par[l] = ctx->param[v]; bia[l] = ctx->bias[v]; a0[l] = ctx->aux0[v]; a1[l] = ctx->aux1[v];
        if (ctx->op[v] == OB_OP_INPUT) {
            a0[l] = (i32)pay.size();
            pay.insert(pay.end(), ctx->payload.data() + ctx->aux0[v], ctx->payload.data() + ctx->aux0[v] + ctx->out_dim[v]);
        }
        for (u32 e = ctx->in_off[v]; e < ctx->in_off[v + 1]; ++e) {
            const u32 u = ctx->in_idx[e];
            iidx.push_back(u < n0 ? (u32)(std::lower_bound(st.proxy.begin(), st.proxy.end(), u) - st.proxy.begin())
                                  : P + (u - n0));
        }
        ioff[l + 1] = (u32)iidx.size();
    }

    // its context: the arena behind everything the earlier evaluations hold
    size_t used = ctx->top;
    if (ctx->stages.size() > 1) {
        const Stage &prev = ctx->stages[ctx->stages.size() - 2];
        used = (size_t)(prev.c->arena - ctx->arena) + prev.c->top;
    }
    used = (used + 255) & ~(size_t)255;
    if (used + (1u << 16) > ctx->arena_bytes) return fail(ctx_fail(ctx, OB_E_OOM, "arena too small for another evaluation stage"));
    if (!ctx->stage_pool.empty()) {
        st.c = ctx->stage_pool.back();
        ctx->stage_pool.pop_back();
        stage_rebase(st.c, ctx, ctx->arena + used, ctx->arena_bytes - used);
    } else if (int rc = ob_ctx_fork(ctx, ctx->arena + used, ctx->arena_bytes - used, ctx->stream, &st.c)) {
        return fail(rc);
    }
    ob_ctx *c = st.c;
    c->sched_stream = ctx->sched_stream;
    c->is_stage = true;
    c->concat_views = ctx->concat_views;
    u32 *lists_dev = arena_array<u32>(c, (size_t)3 * P + 1);
    if (!lists_dev) return fail(ctx_fail(ctx, OB_E_OOM, "arena too small for another evaluation stage"));
    st.lists_dev = lists_dev;
    c->persist_top = c->top;
    int rc = ob_add_bulk(c, (int)nl, op.data(), od.data(), ioff.data(), iidx.data(), par.data(), bia.data(), a0.data(),
                         a1.data(), pay.data(), pay.size());
    if (rc < 0) { ctx->err = c->err; return fail(rc); }
    if (ctx->params_dev) {
        // a stage only runs forward: the owner's parameter table serves (its entries do not depend on
        // which parameters a graph uses), and the tile lists of the parameter-gradient kernels are not needed
        c->params_dev = ctx->params_dev; c->wtiles_dev = ctx->wtiles_dev; c->btiles_dev = ctx->btiles_dev;
        c->wpart_dev = ctx->wpart_dev; c->bpart_dev = ctx->bpart_dev;
        c->wtiles = ctx->wtiles; c->btiles = ctx->btiles;   // (a backward pass over the stages runs the owner's tile lists)
        c->params_dirty = false;
    }
    if ((rc = ob_upload(c)) != 0) { ctx->err = c->err; return fail(rc); }

    // copies of the earlier values, owner by owner (proxies ascend, and so do the owners' id ranges)
    st.lists.resize((size_t)3 * P + 1);
    u32 *src = st.lists.data(), *dst = src + P, *dim = dst + P;
    for (u32 i = 0; i < P; ++i) { dst[i] = (u32)a0[i]; dim[i] = od[i]; }
    const size_t n_own = ctx->stages.size() - 1;   // earlier stages (the last entry is the new one)
    {   // source ids first: the whole list goes to the device in one copy
        u32 i = 0;
        for (size_t k = 0; k <= n_own && i < P; ++k) {   // k = 0: the first evaluation, k >= 1: stage k - 1
            const Stage *own = k ? &ctx->stages[k - 1] : nullptr;
            const u32 hi = own ? own->n1 : ctx->n_sched;
            for (; i < P && st.proxy[i] < hi; ++i)
                src[i] = own ? (u32)own->proxy.size() + (st.proxy[i] - own->n0) : st.proxy[i];
        }
    }
    if (P) {
        hipError_t e = hipMemcpyAsync(lists_dev, st.lists.data(), (size_t)3 * P * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e != hipSuccess) return hip_fail(e, "copying the stage lists");
    }
    if (ctx->sched_stream != ctx->stream) {   // the stage's image (queued on the schedule stream) must be in place
        hipError_t e = hipStreamWaitEvent(ctx->stream, c->ev[1], 0);
        if (e != hipSuccess) return hip_fail(e, "hipStreamWaitEvent");
    }
    float *payload_dev = const_cast<float *>(c->T.payload);
    u32 i = 0;
    for (size_t k = 0; k <= n_own && i < P; ++k) {
        const Stage *own = k ? &ctx->stages[k - 1] : nullptr;
        const u32 hi = own ? own->n1 : ctx->n_sched;
        const u32 i0 = i;
        while (i < P && st.proxy[i] < hi) ++i;
        if (i == i0) continue;
        const Tables &OT = own ? own->c->T : ctx->T;
        if (int frc = fill_uncopied(own ? own->c : ctx, ctx->stream)) { if (own) ctx->err = own->c->err; return fail(frc); }
        hipError_t e = exec_stage_fill(OT.V, OT.val_off, lists_dev + i0, lists_dev + P + i0, lists_dev + 2 * (size_t)P + i0,
                                       i - i0, payload_dev, ctx->stream);
        if (e != hipSuccess) return hip_fail(e, "copying earlier values");
    }
    if ((rc = ob_forward(c, (int)nl - 1)) != 0) { ctx->err = c->err; return fail(rc); }
    ctx->backward_done = false;   // gradients of the shorter graph are not gradients of this one
    return OB_OK;
}

// Backward pass over a graph that was evaluated in stages (Section 3.1 / 3.3), without evaluating
// anything again.  Units: the first evaluation (nodes [0, n_sched)) and every stage.  They run in
// reverse order, each a backward pass of its own graph; a unit's pull adds, per node, the gradient
// that later units have handed down (an extra block with the offsets of the gradient arena, zero at
// first), and after a stage has run, the gradients of its leaves that stand for earlier nodes are
// added to those nodes' entries of their owners' blocks.  Needs room for the extra blocks behind
// the last stage, and every parameter the stages use among the owner's gradient tiles; otherwise
// STAGED_FALLBACK.
static int staged_backward(ob_ctx *ctx, u32 node)
{
    const size_t S = ctx->stages.size();
    for (const Stage &st : ctx->stages)
        for (size_t p = 0; p < ctx->params.size(); ++p) {
            const bool w = p < st.c->params_used_w.size() && st.c->params_used_w[p];
            const bool b = p < st.c->params_used_b.size() && st.c->params_used_b[p];
            if ((w && !(p < ctx->params_used_w.size() && ctx->params_used_w[p])) ||
                (b && !(p < ctx->params_used_b.size() && ctx->params_used_b[p])))
                return STAGED_FALLBACK;
        }
    if (ctx->params_dirty || !ctx->params_dev) return STAGED_FALLBACK;
    auto unit = [&](size_t k) { return k ? ctx->stages[k - 1].c : ctx; };
    ob_ctx *last = unit(S);
    std::vector<float *> gx(S + 1, nullptr);
    const size_t save = last->top;
    for (size_t k = 0; k < S; ++k) {   // (nothing comes after the last unit)
        const size_t floats = (size_t)unit(k)->hdr.grad_floats + VAL_ALIGN;
        gx[k] = arena_array<float>(last, floats);
        if (!gx[k]) { last->top = save; return STAGED_FALLBACK; }
        HIP_TRY(ctx, hipMemsetAsync(gx[k], 0, floats * sizeof(float), ctx->stream));
    }
    for (size_t k = S + 1; k-- > 0;) {
        ob_ctx *u = unit(k);
        u32 root = 0xffffffffu;
        if (k == 0) { if (node < ctx->n_sched) root = node; }
        else {
            const Stage &st = ctx->stages[k - 1];
            if (node >= st.n0 && node < st.n1) root = (u32)st.proxy.size() + (node - st.n0);
        }
        u->T.root = root;
        u->T.Gx = gx[k];
        HIP_TRY(ctx, hipEventRecord(u->ev[4], ctx->stream));
        if (int rc = exec_backward(u)) { if (u != ctx) ctx->err = u->err; return rc; }
        HIP_TRY(ctx, hipEventRecord(u->ev[5], ctx->stream));
        u->backward_done = true;
        if (k == 0) break;
        // hand the leaves' gradients down, owner by owner (leaves ascend, and so do the owners' id ranges)
        const Stage &st = ctx->stages[k - 1];
        const u32 P = (u32)st.proxy.size();
        u32 i = 0;
        for (size_t o = 0; o < k && i < P; ++o) {
            const Stage *own = o ? &ctx->stages[o - 1] : nullptr;
            const u32 hi = own ? own->n1 : ctx->n_sched;
            const u32 i0 = i;
            while (i < P && st.proxy[i] < hi) ++i;
            if (i == i0) continue;
            hipError_t e = exec_stage_scatter(u->T.G, u->T.nat_off, i0, st.lists_dev + i0, st.lists_dev + 2 * (size_t)P + i0, i - i0,
                                              unit(o)->T.nat_off, gx[o], ctx->stream);
            if (e != hipSuccess) return ctx_fail(ctx, OB_E_HIP, "handing gradients to an earlier stage failed: %s", hipGetErrorString(e));
        }
    }
    ctx->backward_done = true;
    return OB_OK;
}

// The last stage's schedule in the caller's node ids: the leaves that stand for earlier nodes are
// left out, and so are batches that held nothing else.
static int stage_schedule_read(ob_ctx *ctx, int *n_batches, int *batch_depth, uint64_t *batch_sig, int *batch_off,
                               int *node_ids, size_t cap_batches, size_t cap_nodes)
{
    const Stage &st = ctx->stages.back();
    const u32 P = (u32)st.proxy.size();
    int nb = 0;
    if (int rc = ob_schedule_read(st.c, &nb, nullptr, nullptr, nullptr, nullptr, 0, 0)) { ctx->err = st.c->err; return rc; }
    const size_t nl = st.c->op.size();
    std::vector<int> depth((size_t)nb + 1), off((size_t)nb + 1), ids(nl + 1);
    std::vector<uint64_t> sig((size_t)nb + 1);
    if (int rc = ob_schedule_read(st.c, &nb, depth.data(), sig.data(), off.data(), ids.data(), (size_t)nb, nl)) {
        ctx->err = st.c->err;
        return rc;
    }
    std::vector<int> k_depth, k_off(1, 0), k_ids;
    std::vector<uint64_t> k_sig;
    for (int b = 0; b < nb; ++b) {
        const size_t before = k_ids.size();
        for (int q = off[b]; q < off[b + 1]; ++q)
            if ((u32)ids[q] >= P) k_ids.push_back((int)(st.n0 + ((u32)ids[q] - P)));
        if (k_ids.size() == before) continue;
        k_depth.push_back(depth[b]);
        k_sig.push_back(sig[b]);
        k_off.push_back((int)k_ids.size());
    }
    if (n_batches) *n_batches = (int)k_depth.size();
    if (!batch_depth && !batch_sig && !batch_off && !node_ids) return OB_OK;
    if (cap_batches < k_depth.size() || cap_nodes < k_ids.size())
        return ctx_fail(ctx, OB_E_RANGE, "schedule has %zu batches, %zu nodes", k_depth.size(), k_ids.size());
    for (size_t b = 0; b < k_depth.size(); ++b) {
        if (batch_depth) batch_depth[b] = k_depth[b];
        if (batch_sig) batch_sig[b] = k_sig[b];
        if (batch_off) batch_off[b] = k_off[b];
    }
    if (batch_off) batch_off[k_depth.size()] = k_off.back();
    if (node_ids) std::copy(k_ids.begin(), k_ids.end(), node_ids);
    return OB_OK;
}

int ob_reset(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    return forget_evaluation(ctx);
}

int ob_sync(ob_ctx *ctx)
{
    CHECK_CTX(ctx);
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return OB_OK;
}

// ---- reads ----------------------------------------------------------------------------------------

// The forward pass leaves the rows of CONCAT batches that only matrix products read unwritten (the products
// read the pieces in place).  Whoever reads values of evaluation unit u from outside the forward pass (a value
// read, the leaves of a later evaluation stage) calls this first: the rows are written once, on stream s.
static int fill_uncopied(ob_ctx *u, hipStream_t s)
{
    if (!u->forward_done || u->uncopied_filled || u->hdr.virt_batches == 0) return OB_OK;
    hipError_t e = exec_fill_uncopied(u->T, s);
    if (e != hipSuccess) return ctx_fail(u, OB_E_HIP, "filling in uncopied rows failed: %s", hipGetErrorString(e));
    u->uncopied_filled = true;
    return OB_OK;
}

static int node_read(ob_ctx *ctx, int node, float *out, size_t cap, bool grad)
{
    if (!out) return ctx_fail(ctx, OB_E_ARG, "null output");
    if (!ctx->forward_done || (grad && !ctx->backward_done)) return ctx_fail(ctx, OB_E_STATE, "nothing to read yet");
    if (node < 0 || (u32)node >= evaluated_upto(ctx)) return ctx_fail(ctx, OB_E_BADID, "node %d was not evaluated", node);
    if ((u32)node >= ctx->n_sched) {   // the value lives in a later evaluation stage
        for (Stage &st : ctx->stages) {
            if ((u32)node >= st.n1) continue;
            const int rc = node_read(st.c, (int)(st.proxy.size() + ((u32)node - st.n0)), out, cap, grad);
            if (rc) ctx->err = st.c->err;
            return rc;
        }
    }
    const u32 d = ctx->out_dim[node];
    if (cap < d) return ctx_fail(ctx, OB_E_RANGE, "buffer holds %zu of %u elements", cap, d);
    if (!grad) if (int rc = fill_uncopied(ctx, ctx->stream)) return rc;
    u32 off = 0;
    HIP_TRY(ctx, hipMemcpyAsync(&off, (grad ? ctx->T.nat_off : ctx->T.val_off) + node, 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    HIP_TRY(ctx, hipMemcpyAsync(out, (grad ? ctx->T.G : ctx->T.V) + off, (size_t)d * 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return OB_OK;
}

int ob_value_read(ob_ctx *ctx, int node, float *host_out, size_t cap)
{
    CHECK_CTX(ctx);
    return node_read(ctx, node, host_out, cap, false);
}

int ob_grad_read(ob_ctx *ctx, int node, float *host_out, size_t cap)
{
    CHECK_CTX(ctx);
    return node_read(ctx, node, host_out, cap, true);
}

int ob_all_read(ob_ctx *ctx, int which, float *host_out, size_t cap)
{
    CHECK_CTX(ctx);
    if (!host_out) return ctx_fail(ctx, OB_E_ARG, "null output");
    if (!ctx->forward_done || (which && !ctx->backward_done)) return ctx_fail(ctx, OB_E_STATE, "nothing to read yet");
    // Units: the first evaluation and every later stage; each gathers its own nodes (a stage's leaves
    // that stand for earlier nodes are left out) into one staging block behind the last unit.
    const size_t S = ctx->stages.size();
    const u32 n = evaluated_upto(ctx);
    std::vector<u32> off((size_t)n + 1);
    u64 tot = 0;
    for (u32 v = 0; v < n; ++v) { off[v] = (u32)tot; tot += ctx->out_dim[v]; }
    if (tot > 0xffffffffull) return ctx_fail(ctx, OB_E_RANGE, "too many elements");
    if (cap < tot) return ctx_fail(ctx, OB_E_RANGE, "buffer holds %zu of %llu elements", cap, (unsigned long long)tot);
    ob_ctx *last = S ? ctx->stages.back().c : ctx;
    const size_t save = last->top;
    float *dst = arena_array<float>(last, tot + 1);
    int rc = OB_OK;
    std::vector<std::vector<u32>> keep(S + 1);    // host lists stay alive until the copies have run
    for (size_t k = 0; k <= S && rc == OB_OK && dst; ++k) {
        ob_ctx *u = k ? ctx->stages[k - 1].c : ctx;
        if (which && !u->backward_done) { rc = ctx_fail(ctx, OB_E_STATE, "no gradients in evaluation stage %zu", k); break; }
        const u32 P = k ? (u32)ctx->stages[k - 1].proxy.size() : 0u;
        const u32 n0 = k ? ctx->stages[k - 1].n0 : 0u;
        const u32 nl = u->T.n;
        std::vector<u32> &loc = keep[k];
        loc.assign((size_t)nl + 1, 0xffffffffu);
        for (u32 l = P; l < nl; ++l) loc[l] = off[n0 + (l - P)];
        u32 *off_dev = arena_array<u32>(last, (size_t)nl + 1);
        if (!off_dev) { dst = nullptr; break; }
        if (!which && fill_uncopied(u, ctx->stream)) { rc = ctx_fail(ctx, OB_E_HIP, "%s", u->err.c_str()); break; }
        hipError_t e = hipMemcpyAsync(off_dev, loc.data(), (size_t)nl * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = exec_gather_some(u->T, which, dst, off_dev, ctx->stream);
        if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "read-back failed: %s", hipGetErrorString(e));
    }
    if (!dst) { last->top = save; return ctx_fail(ctx, OB_E_OOM, "arena too small for the read-back staging"); }
    if (rc == OB_OK) {
        hipError_t e = hipMemcpyAsync(host_out, dst, tot * 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "read-back failed: %s", hipGetErrorString(e));
    } else {
        (void)hipStreamSynchronize(ctx->stream);
    }
    last->top = save;
    return rc;
}

int ob_schedule_read(ob_ctx *ctx, int *n_batches, int *batch_depth, uint64_t *batch_sig, int *batch_off, int *node_ids,
                     size_t cap_batches, size_t cap_nodes)
{
    CHECK_CTX(ctx);
    if (!ctx->forward_done) return ctx_fail(ctx, OB_E_STATE, "no schedule yet");
    if (!ctx->stages.empty())
        return stage_schedule_read(ctx, n_batches, batch_depth, batch_sig, batch_off, node_ids, cap_batches, cap_nodes);
    const u32 nb = ctx->hdr.n_batches, n = ctx->n_sched;
    if (n_batches) *n_batches = (int)nb;
    if (!batch_depth && !batch_sig && !batch_off && !node_ids) return OB_OK;
    if (cap_batches < nb || cap_nodes < n) return ctx_fail(ctx, OB_E_RANGE, "schedule has %u batches, %u nodes", nb, n);
    std::vector<BatchRec> recs(nb);
    HIP_TRY(ctx, hipMemcpyAsync(recs.data(), ctx->T.batches, (size_t)nb * sizeof(BatchRec), hipMemcpyDeviceToHost, ctx->stream));
    std::vector<u64> sig;
    std::vector<u32> order(n);
    HIP_TRY(ctx, hipMemcpyAsync(order.data(), ctx->T.order, (size_t)n * 4, hipMemcpyDeviceToHost, ctx->stream));
    if (batch_sig) {
        sig.resize(n);
        HIP_TRY(ctx, hipMemcpyAsync(sig.data(), ctx->T.sig, (size_t)n * 8, hipMemcpyDeviceToHost, ctx->stream));
    }
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    for (u32 b = 0; b < nb; ++b) {
        if (batch_depth) batch_depth[b] = (int)recs[b].step;
        if (batch_off) batch_off[b] = (int)recs[b].pos0;
        if (batch_sig) batch_sig[b] = sig[order[recs[b].pos0]];
    }
    if (batch_off) batch_off[nb] = (int)n;
    if (node_ids) for (u32 p = 0; p < n; ++p) node_ids[p] = (int)order[p];
    return OB_OK;
}

int ob_stats_read(ob_ctx *ctx, ob_stats *out)
{
    CHECK_CTX(ctx);
    if (!out) return ctx_fail(ctx, OB_E_ARG, "null output");
    memset(out, 0, sizeof *out);
    out->n_nodes = (int32_t)ctx->op.size();
    out->n_edges = (int32_t)ctx->in_idx.size();
    if (!ctx->forward_done) return OB_OK;
    if (!ctx->stages.empty()) {   // counters and times of the last stage's evaluation
        const Stage &st = ctx->stages.back();
        const int rc = ob_stats_read(st.c, out);
        if (rc) { ctx->err = st.c->err; return rc; }
        out->n_nodes = (int32_t)(st.n1 - st.n0);
        out->n_stages = (int32_t)ctx->stages.size() + 1;
        out->n_proxies = (int32_t)st.proxy.size();
        return OB_OK;
    }
    out->n_stages = 1;
    HIP_TRY(ctx, hipStreamSynchronize(ctx->sched_stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    out->n_nodes = (int32_t)ctx->n_sched;
    out->n_edges = (int32_t)ctx->T.E;
    out->n_steps = (int32_t)ctx->hdr.n_steps;
    out->n_batches = (int32_t)ctx->hdr.n_batches;
    out->n_tiles_fwd = (int32_t)ctx->hdr.tiles_fwd;
    out->n_tiles_bwd_pull = (int32_t)ctx->hdr.tiles_pull;
    out->n_tiles_bwd_dx = (int32_t)ctx->hdr.tiles_dx;
    out->n_param_uses = (int32_t)ctx->hdr.n_items;
    out->n_launch_fwd = ctx->n_launch_fwd;
    out->n_launch_bwd = ctx->n_launch_bwd;
    out->n_launch_sched = ctx->n_launch_sched;
    out->n_slots = (int32_t)ctx->hdr.n_slots;
    out->value_floats = ctx->hdr.val_floats;
    out->grad_floats = ctx->hdr.grad_floats;
    out->arena_used_bytes = ctx->top;
    out->upload_bytes = ctx->upload_bytes;
    (void)hipEventElapsedTime(&out->ms_upload, ctx->ev[0], ctx->ev[1]);
    (void)hipEventElapsedTime(&out->ms_schedule, ctx->ev[7], ctx->ev[9]);
    (void)hipEventElapsedTime(&out->ms_forward, ctx->ev[8], ctx->ev[3]);
    if (ctx->backward_done) {
        (void)hipEventElapsedTime(&out->ms_backward, ctx->ev[4], ctx->ev[5]);
        (void)hipEventElapsedTime(&out->ms_param_grads, ctx->ev[6], ctx->ev[5]);
    }
    out->ms_graph_build = ctx->ms_graph;
    out->n_depth_retries = ctx->n_depth_retries;
    out->n_launch_bwd_steps = ctx->n_launch_bwd_steps;
    out->n_view_batches = (int32_t)ctx->hdr.view_batches;
    out->n_uncopied_batches = (int32_t)ctx->hdr.virt_batches;
    out->view_floats = ctx->hdr.view_floats;
    out->uncopied_floats = ctx->hdr.virt_floats;
    (void)hipGetLastError();
    return OB_OK;
}

int ob_debug_set(ob_ctx *ctx, int which, uint64_t value)
{
    CHECK_CTX(ctx);
    switch (which) {
    case OB_DBG_SET_DEPTH_SPIN:
        ctx->depth_spin_limit = value > 0xffffffffull ? 0xffffffffu : (u32)value;
        return OB_OK;
    case OB_DBG_SET_CONCAT_COPY:
        ctx->concat_views = value == 0;
        return OB_OK;
    default:
        return ctx_fail(ctx, OB_E_ARG, "unknown knob %d", which);
    }
}

int ob_debug_read(ob_ctx *ctx, int which, uint32_t *host_out, size_t cap_words, size_t *n_words)
{
    CHECK_CTX(ctx);
    if (!ctx->forward_done) return ctx_fail(ctx, OB_E_STATE, "no schedule yet");
    if (!ctx->stages.empty()) return ctx_fail(ctx, OB_E_STATE, "the graph was evaluated in stages: no single set of tables");
    const Tables &T = ctx->T;
    const void *src = nullptr;
    size_t words = 0;
    switch (which) {
    case OB_DBG_DEPTH: src = T.step; words = T.n; break;
    case OB_DBG_SIG: src = T.sig; words = (size_t)T.n * 2; break;
    case OB_DBG_SUCC_OFF: src = T.succ_off; words = (size_t)T.n + 1; break;
    case OB_DBG_SUCC_EDGE: src = T.succ_edge; words = T.E; break;
    case OB_DBG_ORDER: src = T.order; words = T.n; break;
    case OB_DBG_VAL_OFF: src = T.val_off; words = T.n; break;
    case OB_DBG_TILES_FWD: src = T.tiles_f; words = (size_t)ctx->hdr.tiles_fwd * (sizeof(TileDesc) / 4); break;
    case OB_DBG_TILES_PULL: src = T.tiles_a; words = (size_t)ctx->hdr.tiles_pull * (sizeof(PullDesc) / 4); break;
    case OB_DBG_CHAINS: src = T.chains; words = (size_t)ctx->hdr.n_chains * (sizeof(ChainRec) / 4); break;
    case OB_DBG_LORDER: src = T.lorder; words = ctx->hdr.n_batches; break;
    default: return ctx_fail(ctx, OB_E_ARG, "unknown table %d", which);
    }
    if (n_words) *n_words = words;
    if (!host_out) return OB_OK;
    if (cap_words < words) return ctx_fail(ctx, OB_E_RANGE, "table has %zu words", words);
    if (words) HIP_TRY(ctx, hipMemcpyAsync(host_out, src, words * 4, hipMemcpyDeviceToHost, ctx->stream));
    HIP_TRY(ctx, hipStreamSynchronize(ctx->stream));
    return OB_OK;
}

// ---- stand-alone primitives for tests ----------------------------------------------------------

int ob_test_sort(ob_ctx *ctx, size_t n, const uint64_t *keys, const uint32_t *vals, int lo_bit, int n_bits,
                 uint64_t *keys_out, uint32_t *vals_out)
{
    CHECK_CTX(ctx);
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "no arena");
    if (n == 0) return OB_OK;
    const size_t save = ctx->top;
    u64 *ka = arena_array<u64>(ctx, n), *kb = arena_array<u64>(ctx, n);
    u32 *va = arena_array<u32>(ctx, n), *vb = arena_array<u32>(ctx, n);
    void *scratch = arena_alloc(ctx, prim_sort_scratch_bytes(n));
    int rc = OB_OK;
    if (!ka || !kb || !va || !vb || !scratch) rc = ctx_fail(ctx, OB_E_OOM, "arena too small");
    if (rc == OB_OK) {
        hipError_t e = hipMemcpyAsync(ka, keys, n * 8, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(va, vals, n * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = prim_sort_pairs(ka, va, kb, vb, n, lo_bit, n_bits, scratch, ctx->stream, nullptr);
        if (e == hipSuccess) e = hipMemcpyAsync(keys_out, ka, n * 8, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(vals_out, va, n * 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "sort failed: %s", hipGetErrorString(e));
    }
    ctx->top = save;
    return rc;
}

int ob_test_scan(ob_ctx *ctx, size_t n, const uint32_t *in, uint32_t *out_exclusive, uint32_t *total)
{
    CHECK_CTX(ctx);
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "no arena");
    const size_t save = ctx->top;
    u32 *a = arena_array<u32>(ctx, n + 1), *b = arena_array<u32>(ctx, n + 1), *t = arena_array<u32>(ctx, 1);
    void *scratch = arena_alloc(ctx, prim_scan_scratch_bytes(n + 1, 4));
    int rc = OB_OK;
    if (!a || !b || !t || !scratch) rc = ctx_fail(ctx, OB_E_OOM, "arena too small");
    if (rc == OB_OK) {
        hipError_t e = n ? hipMemcpyAsync(a, in, n * 4, hipMemcpyHostToDevice, ctx->stream) : hipSuccess;
        if (e == hipSuccess) e = prim_scan_u32(a, b, n, t, scratch, ctx->stream);
        if (e == hipSuccess && n) e = hipMemcpyAsync(out_exclusive, b, n * 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(total, t, 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "scan failed: %s", hipGetErrorString(e));
    }
    ctx->top = save;
    return rc;
}

int ob_test_launch_cost(ob_ctx *ctx, int n, int touch, float *us_per_launch)
{
    CHECK_CTX(ctx);
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "no arena");
    if (n <= 0 || !us_per_launch) return ctx_fail(ctx, OB_E_ARG, "bad argument");
    const size_t save = ctx->top;
    float *scratch = arena_array<float>(ctx, 64);
    if (!scratch) return ctx_fail(ctx, OB_E_OOM, "arena too small");
    int rc = OB_OK;
    hipError_t e = hipMemsetAsync(scratch, 0, 256, ctx->stream);
    if (e == hipSuccess) e = exec_launch_probe(scratch, n, touch, us_per_launch, ctx->stream);
    if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "launch probe failed: %s", hipGetErrorString(e));
    ctx->top = save;
    return rc;
}

int ob_test_gemm(ob_ctx *ctx, int M, int N, int K, const float *A, const float *B, float *C)
{
    CHECK_CTX(ctx);
    if (!ctx->arena) return ctx_fail(ctx, OB_E_STATE, "no arena");
    if (M <= 0 || N <= 0 || K <= 0) return ctx_fail(ctx, OB_E_ARG, "bad shape");
    if ((u64)M * (u64)K >= 0xffffffffull) return ctx_fail(ctx, OB_E_RANGE, "operand of more than 2^32 elements");
    const size_t save = ctx->top;
    float *a = arena_array<float>(ctx, (size_t)M * K), *b = arena_array<float>(ctx, (size_t)N * K);
    float *c = arena_array<float>(ctx, (size_t)M * N);
    int rc = OB_OK;
    if (!a || !b || !c) rc = ctx_fail(ctx, OB_E_OOM, "arena too small");
    if (rc == OB_OK) {
        hipError_t e = hipMemcpyAsync(a, A, (size_t)M * K * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(b, B, (size_t)N * K * 4, hipMemcpyHostToDevice, ctx->stream);
        if (e == hipSuccess) e = exec_test_gemm(M, N, K, a, b, c, ctx->stream);
        if (e == hipSuccess) e = hipMemcpyAsync(C, c, (size_t)M * N * 4, hipMemcpyDeviceToHost, ctx->stream);
        if (e == hipSuccess) e = hipStreamSynchronize(ctx->stream);
        if (e != hipSuccess) rc = ctx_fail(ctx, OB_E_HIP, "gemm failed: %s", hipGetErrorString(e));
    }
    ctx->top = save;
    return rc;
}

}  // extern "C"
