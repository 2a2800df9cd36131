// GPU scheduler: node signatures as integer hashes (Appendix B), depth by level-synchronous
// frontier passes over a successor CSR with per-node unresolved-dependency counters
// (Section 3.2), batches = equal (depth, signature) found by a stable radix sort, then the
// memory layout of the batched execution (Section 3.3: operands of a batch must be
// addressable as one matrix; results are laid out contiguously in batch order).
#include "ob_ctx.h"

namespace {

constexpr int TPB = 256;
inline unsigned blocks_for(size_t n, int per = TPB) { return (unsigned)((n + per - 1) / per); }

__device__ inline u64 mix64(u64 x)
{
    x ^= x >> 33; x *= 0xff51afd7ed558ccdULL;
    x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ULL;
    x ^= x >> 33;
    return x;
}
__device__ inline u64 comb(u64 h, u64 x) { return mix64(h ^ (x + 0x9e3779b97f4a7c15ULL + (h << 6) + (h >> 2))); }

// ---- stage 1: signatures, dependency counters, out-degrees, initial frontier ---------------
// Signature tuple (Section 3.2 / Appendix A): operation, output dimension, arity, shared
// parameter ids (the A and y of A x + y), slice range, operand dimensions.  LOOKUP's row,
// PICK_NLS's label and INPUT's payload are data and stay out.  The node's own fields are hashed
// here; every operand edge then adds a position-salted hash of the operand's dimension
// (k_edge_init), so nodes with thousands of operands cost no more than a thread per edge.
__global__ void k_node_init(Tables T, int by_depth)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n) return;
    const u32 lo = T.in_off[v], hi = T.in_off[v + 1];
    const u32 o = T.op[v];
    u64 h = mix64(o + 1);
    h = comb(h, T.out_dim[v]);
    h = comb(h, hi - lo);
    h = comb(h, (u64)(u32)(T.param[v] + 1));
    h = comb(h, (u64)(u32)(T.bias[v] + 1));
    h = comb(h, o == OP_SLICE ? (u64)(u32)T.aux0[v] : 0);
    h = comb(h, o == OP_SLICE ? (u64)(u32)T.aux1[v] : 0);
    T.sig[v] = h;
    T.indeg[v] = hi - lo;
    if (by_depth) {
        if (hi == lo) {
            const u32 pos = atomicAdd(&T.qcount[0], 1u);
            T.queue[pos] = v;
            T.step[v] = 0;
        }
    } else {
        T.step[v] = v;   // unbatched: every node is its own step, in id order
    }
}

// consumer node of edge e: the v with in_off[v] <= e < in_off[v+1]
__device__ inline u32 consumer_of(const Tables &T, u32 e)
{
    u32 lo = 0, hi = T.n;   // invariant: in_off[lo] <= e < in_off[hi]
    while (hi - lo > 1) {
        const u32 mid = (lo + hi) >> 1;
        if (T.in_off[mid] <= e) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void k_edge_init(Tables T, u64 *keys, u32 *vals)
{
    const u32 e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= T.E) return;
    const u32 v = consumer_of(T, e);
    const u32 u = T.in_idx[e];
    const u32 j = e - T.in_off[v];
    T.edge_cons[e] = v;
    atomicAdd(&T.outdeg[u], 1u);
    atomicAdd((unsigned long long *)&T.sig[v], (unsigned long long)mix64(comb(0x5bd1e995ULL + j, T.out_dim[u])));
    keys[e] = u;
    vals[e] = e;
}

// after the sort: succ_edge[q] = edge id, succ_node[q] = its consumer (stored in T.queue's
// sibling array to save one hop in the frontier loop)
__global__ void k_succ_finish(Tables T, const u32 *sorted_edge, u32 *succ_node)
{
    const u32 q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= T.E) return;
    const u32 e = sorted_edge[q];
    T.succ_edge[q] = e;
    succ_node[q] = T.edge_cons[e];
}

// ---- stage 2: depth by frontier passes ---------------------------------------------------------
// One workgroup walks the graph level by level.  queue[head, tail) is the current frontier
// (all nodes of depth `level`); a node joins the next frontier when its last unresolved
// dependency is resolved, which is exactly when the deepest of its operands has been
// processed, so its depth is level + 1 (depth = longest path from a leaf, Section 3.2).
constexpr int FRONTIER_THREADS = 1024;
__global__ __launch_bounds__(FRONTIER_THREADS) void k_depth_frontier(Tables T, const u32 *succ_node)
{
    __shared__ u32 s_head, s_tail, s_next;
    if (threadIdx.x == 0) { s_head = 0; s_tail = T.qcount[0]; s_next = T.qcount[0]; }
    __syncthreads();
    u32 level = 0;
    while (true) {
        const u32 head = s_head, tail = s_tail;
        if (head == tail) break;
        for (u32 i = head + threadIdx.x; i < tail; i += FRONTIER_THREADS) {
            const u32 u = T.queue[i];
            const u32 q1 = T.succ_off[u + 1];
            for (u32 q = T.succ_off[u]; q < q1; ++q) {
                const u32 s = succ_node[q];
                if (atomicSub(&T.indeg[s], 1u) == 1u) {
                    T.step[s] = level + 1;
                    const u32 pos = atomicAdd(&s_next, 1u);
                    T.queue[pos] = s;
                }
            }
        }
        __syncthreads();
        if (threadIdx.x == 0) { s_head = tail; s_tail = s_next; }
        __syncthreads();
        ++level;
    }
    if (threadIdx.x == 0) {
        T.hdr->frontier_done = s_tail;
        if (s_tail != T.n) atomicOr(&T.hdr->err, (u32)ERR_CYCLE);
    }
}

// ---- stage 3: batch representative = smallest node id with the same (depth, signature) ------
__device__ inline u64 batch_key(u64 sig, u32 step)
{
    u64 k = comb(sig, step);
    return k ? k : 1;
}

__global__ void k_rep_insert(Tables T)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n) return;
    const u64 k = batch_key(T.sig[v], T.step[v]);
    u32 slot = (u32)k & T.ht_mask;
    for (u32 probe = 0; probe <= T.ht_mask; ++probe) {
        const u64 old = atomicCAS((unsigned long long *)&T.ht_keys[slot], 0ULL, (unsigned long long)k);
        if (old == 0 || old == k) {
            atomicMin(&T.ht_vals[slot], v);
            T.ht_slot[v] = slot;
            return;
        }
        slot = (slot + 1) & T.ht_mask;
    }
    atomicOr(&T.hdr->err, (u32)ERR_TABLE_FULL);
    T.ht_slot[v] = 0;
}

__global__ void k_sort_keys(Tables T, u64 *keys, u32 *vals, int by_depth)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n) return;
    const u32 rep = by_depth ? T.ht_vals[T.ht_slot[v]] : v;
    keys[v] = ((u64)T.step[v] << 32) | rep;
    vals[v] = v;
}

// ---- stage 4: batches from the sorted order -----------------------------------------------------
__global__ void k_heads(Tables T, const u64 *skey, const u32 *sval, u32 *head_flag, u32 *s_arity, u32 *s_items)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const u32 v = sval[p];
    T.order[p] = v;
    T.pos_of[v] = p;
    T.s_aux0[p] = (u32)T.aux0[v];
    head_flag[p] = (p == 0 || skey[p] != skey[p - 1]) ? 1u : 0u;
    s_arity[p] = T.in_off[v + 1] - T.in_off[v];
    const u32 o = T.op[v];
    s_items[p] = (o == OP_MATVEC) ? (1u + (T.bias[v] >= 0 ? 1u : 0u)) : (o == OP_LOOKUP ? 1u : 0u);
}

__global__ void k_batch_off(Tables T, const u32 *head_flag, const u32 *head_excl)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const u32 b = head_excl[p] + head_flag[p] - 1;
    T.batch_of_pos[p] = b;
    if (head_flag[p]) T.batch_off[b] = p;
    if (p == T.n - 1) {
        T.batch_off[b + 1] = T.n;
        T.hdr->n_batches = b + 1;
    }
}

__host__ __device__ inline u32 cdiv(u64 a, u32 b) { return (u32)((a + b - 1) / b); }

__device__ inline u32 fwd_tiles_of(u32 op, u32 B, u32 d, u32 arity)
{
    switch (op) {
    case OP_MATVEC: return cdiv(B, GT) * cdiv(d, GT);
    case OP_PICK_NLS:
    case OP_SQNORM: return cdiv(B, ROWS_PER_RED_TILE);
    case OP_ADD: if (arity >= (u32)WIDE_ADD_ARITY) return B;  // fallthrough for narrow sums
    default: return cdiv((u64)B * d, EW_TILE);
    }
}

// one thread per batch: record + sizes for the layout scan (entries b >= n_batches are zero)
__global__ void k_batch_layout(Tables T, Lay *lay_in)
{
    const u32 b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= T.n) return;
    Lay L; L.val = 0; L.dx = 0; L.tf = L.ta = L.tb = L.ind = 0;
    if (b < T.hdr->n_batches) {
        const u32 p0 = T.batch_off[b], B = T.batch_off[b + 1] - p0;
        const u32 h = T.order[p0];
        BatchRec r;
        r.pos0 = p0; r.B = B; r.op = T.op[h]; r.d = T.out_dim[h];
        r.arity = T.in_off[h + 1] - T.in_off[h];
        r.param = T.param[h]; r.bias = T.bias[h];
        r.aux0 = T.aux0[h]; r.aux1 = T.aux1[h];
        r.step = T.step[h];
        r.k = r.arity ? T.out_dim[T.in_idx[T.in_off[h]]] : 0;
        r.val_off = r.dx_off = r.indim = 0;
        r.opnd = T.s_in_off[p0];
        r.vec4 = 3;   // bit 0: float4 component-wise path; bit 1: operand rows are 16-byte aligned
        T.batches[b] = r;
        const u64 vs = (u64)B * r.d;
        L.val = (vs + VAL_ALIGN - 1) / VAL_ALIGN * VAL_ALIGN;
        L.tf = fwd_tiles_of(r.op, B, r.d, r.arity);
        L.ta = cdiv(vs, EW_TILE);
        if (r.op == OP_MATVEC) {
            const u64 xs = (u64)B * r.k;
            L.dx = (xs + VAL_ALIGN - 1) / VAL_ALIGN * VAL_ALIGN;
            L.tb = cdiv(B, GT) * cdiv(r.k, GT);
        }
        L.ind = r.arity;
    }
    lay_in[b] = L;
}

__global__ void k_batch_finish(Tables T, const Lay *lay_ex, const Lay *total)
{
    const u32 b = blockIdx.x * blockDim.x + threadIdx.x;
    const u32 nb = T.hdr->n_batches;
    if (b >= nb) return;
    const Lay L = lay_ex[b];
    const Lay tot = *total;
    BatchRec &r = T.batches[b];
    r.val_off = (u32)L.val;
    r.dx_off = (u32)(tot.val + L.dx);
    r.indim = L.ind;
    const u32 s = r.step;
    if (b == 0 || T.batches[b - 1].step != s) {
        T.step_first[s] = b; T.step_tf[s] = L.tf; T.step_ta[s] = L.ta; T.step_tb[s] = L.tb;
    }
    if (b == nb - 1) {
        T.step_first[s + 1] = nb; T.step_tf[s + 1] = tot.tf; T.step_ta[s + 1] = tot.ta; T.step_tb[s + 1] = tot.tb;
        T.hdr->n_steps = s + 1;
        T.hdr->val_floats = tot.val;
        T.hdr->grad_floats = tot.val + tot.dx;
        T.hdr->tiles_fwd = tot.tf; T.hdr->tiles_pull = tot.ta; T.hdr->tiles_dx = tot.tb;
        if (tot.val + tot.dx >= 0xffffffffULL) atomicOr(&T.hdr->err, (u32)ERR_OVERFLOW);
    }
}

__global__ void k_node_offsets(Tables T)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const BatchRec &r = T.batches[T.batch_of_pos[p]];
    const u32 row = p - r.pos0;
    const u32 v = T.order[p];
    T.val_off[v] = r.val_off + row * r.d;
    T.dx_off[v] = (r.op == OP_MATVEC) ? r.dx_off + row * r.k : 0u;
}

// Per node: the check that every member of a batch really has the signature tuple of the batch
// head (a 64-bit hash collision would otherwise merge incompatible nodes), and whether the
// float4 component-wise path is allowed.
__global__ void k_member_check(Tables T)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    BatchRec &r = T.batches[T.batch_of_pos[p]];
    const u32 v = T.order[p];
    const u32 ar = T.in_off[v + 1] - T.in_off[v];
    bool same = T.op[v] == r.op && T.out_dim[v] == r.d && ar == r.arity && T.param[v] == r.param &&
                T.bias[v] == r.bias && T.step[v] == r.step;
    if (r.op == OP_SLICE) same = same && T.aux0[v] == r.aux0 && T.aux1[v] == r.aux1;
    bool vec = (r.d & 3u) == 0;
    if (r.op == OP_SLICE) vec = vec && ((u32)r.aux0 & 3u) == 0;
    if (r.op == OP_INPUT) vec = vec && ((u32)T.aux0[v] & 3u) == 0;
    if (!same) atomicOr(&T.hdr->err, (u32)ERR_COLLISION);
    if (!vec) atomicAnd(&r.vec4, 2u);
}

// Per edge: operand row offsets per batch (slot-major), operand dimensions of the batch, the
// operand part of the membership check, and the alignment flags.
__global__ void k_opnd(Tables T)
{
    const u32 e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= T.E) return;
    const u32 v = T.edge_cons[e];
    const u32 j = e - T.in_off[v];
    const u32 p = T.pos_of[v];
    BatchRec &r = T.batches[T.batch_of_pos[p]];
    const u32 row = p - r.pos0;
    const u32 h = T.order[r.pos0];
    const u32 u = T.in_idx[e];
    const u32 du = T.out_dim[u];
    if (j >= r.arity || du != T.out_dim[T.in_idx[T.in_off[h] + j]]) {
        atomicOr(&T.hdr->err, (u32)ERR_COLLISION);
        return;
    }
    const u32 off = T.val_off[u];
    T.opnd_off[r.opnd + j * r.B + row] = off;
    if (row == 0) T.b_indim[r.indim + j] = du;
    if (off & 3u) atomicAnd(&r.vec4, 0u);
    else if (r.op == OP_CONCAT && (du & 3u)) atomicAnd(&r.vec4, 2u);
}

// ---- tile descriptors ------------------------------------------------------------------------------
__device__ inline u32 tiles_field(const Lay &L, int which) { return which == 0 ? L.tf : (which == 1 ? L.ta : L.tb); }

// batch that owns global tile index t of list `which`: the largest b with offset(b) <= t
__device__ inline u32 batch_of_tile(const Lay *lay_ex, u32 nb, int which, u32 t)
{
    u32 lo = 0, hi = nb;
    while (hi - lo > 1) {
        const u32 mid = (lo + hi) >> 1;
        if (tiles_field(lay_ex[mid], which) <= t) lo = mid; else hi = mid;
    }
    return lo;
}

constexpr u32 CONTIG_MAX_ROWS = 32;   // tiles with more rows skip the contiguity test

__device__ inline void fill_tile_desc(const Tables &T, const BatchRec &r, u32 t, bool dx, TileDesc &d)
{
    d.op = r.op; d.B = r.B; d.d = r.d; d.arity = r.arity;
    d.pos0 = r.pos0; d.val_off = r.val_off; d.dx_off = r.dx_off; d.k = r.k;
    d.param = r.param; d.bias = r.bias; d.aux0 = r.aux0; d.aux1 = r.aux1;
    d.opnd = r.opnd; d.indim = r.indim; d.flags = r.vec4; d.t = t;
    d.contig = 0; d.row0 = 0;
    for (int j = 0; j < 4; ++j) { d.base[j] = 0; d.sdim[j] = 0; }
    for (int j = 0; j < 6; ++j) d.pad[j] = 0;
    if (dx || r.arity == 0) return;
    // rows this tile touches
    u32 r_lo, r_hi;
    if (r.op == OP_MATVEC) {
        const u32 ntn = (r.d + GT - 1) / GT;
        r_lo = (t / ntn) * GT; r_hi = r_lo + GT - 1;
    } else if (r.op == OP_PICK_NLS || r.op == OP_SQNORM) {
        r_lo = t * ROWS_PER_RED_TILE; r_hi = r_lo + ROWS_PER_RED_TILE - 1;
    } else if (r.op == OP_ADD && r.arity >= (u32)WIDE_ADD_ARITY) {
        r_lo = r_hi = t;
    } else {
        r_lo = (u32)(((u64)t * EW_TILE) / r.d);
        r_hi = (u32)(((u64)t * EW_TILE + EW_TILE - 1) / r.d);
    }
    if (r_hi >= r.B) r_hi = r.B - 1;
    d.row0 = r_lo;
    const u32 ns = r.arity < 4 ? r.arity : 4;
    for (u32 j = 0; j < ns; ++j) {
        const u32 *op = T.opnd_off + r.opnd + j * r.B;
        const u32 sd = T.b_indim[r.indim + j];
        const u32 base = op[r_lo];
        d.base[j] = base; d.sdim[j] = sd;
        bool ok = (r_hi - r_lo) < CONTIG_MAX_ROWS;
        for (u32 rr = r_lo + 1; ok && rr <= r_hi; ++rr) ok = op[rr] == base + (rr - r_lo) * sd;
        if (ok) d.contig |= 1u << j;
    }
}

constexpr u32 PULL_MAX_ROWS = 16;

__device__ inline void fill_pull_desc(const Tables &T, const BatchRec &r, u32 t, PullDesc &d)
{
    d.pos0 = r.pos0; d.B = r.B; d.d = r.d; d.val_off = r.val_off;
    d.t = t; d.flags = 0; d.n_uni = PULL_GENERIC;
    for (int j = 0; j < 4; ++j) { UEdge z; z.kind = 0; z.goff = z.voff = z.gs = z.vs = 0; z.a0 = z.a1 = 0; d.e[j] = z; }
    for (int j = 0; j < 4; ++j) d.pad[j] = 0;
    u32 r_lo = (u32)(((u64)t * EW_TILE) / r.d);
    u32 r_hi = (u32)(((u64)t * EW_TILE + EW_TILE - 1) / r.d);
    if (r_hi >= r.B) r_hi = r.B - 1;
    d.row0 = r_lo;
    if (r_hi - r_lo >= PULL_MAX_ROWS) return;
    const u32 u0 = T.order[r.pos0 + r_lo];
    const u32 q0 = T.succ_off[u0];
    const u32 cnt = T.succ_off[u0 + 1] - q0;
    if (cnt > 4) return;
    EdgeRec first[4];
    for (u32 j = 0; j < cnt; ++j) {
        first[j] = T.edges[q0 + j];
        if (first[j].kind == EK_NLS) return;     // the label is per-row data
        UEdge ue; ue.kind = first[j].kind; ue.goff = first[j].goff; ue.voff = first[j].voff;
        ue.gs = ue.vs = 0; ue.a0 = first[j].a0; ue.a1 = first[j].a1;
        d.e[j] = ue;
    }
    for (u32 rr = r_lo + 1; rr <= r_hi; ++rr) {
        const u32 u = T.order[r.pos0 + rr];
        const u32 q = T.succ_off[u];
        if (T.succ_off[u + 1] - q != cnt) return;
        for (u32 j = 0; j < cnt; ++j) {
            const EdgeRec er = T.edges[q + j];
            if (er.kind != first[j].kind || er.a0 != first[j].a0 || er.a1 != first[j].a1) return;
            const u32 dg = er.goff - first[j].goff, dv = er.voff - first[j].voff;
            if (rr == r_lo + 1) { d.e[j].gs = dg; d.e[j].vs = dv; }
            else if (dg != d.e[j].gs * (rr - r_lo) || dv != d.e[j].vs * (rr - r_lo)) return;
        }
    }
    d.n_uni = cnt;
}

__global__ void k_tiles(Tables T, const Lay *lay_ex, const Lay *total, u32 cap_f, u32 cap_a, u32 cap_b)
{
    const u32 nb = T.hdr->n_batches;
    for (int which = 0; which < 3; ++which) {
        u32 nt = tiles_field(*total, which);
        const u32 cap = which == 0 ? cap_f : (which == 1 ? cap_a : cap_b);
        if (nt > cap) {   // cannot happen with the host's bound; never write past the lists
            if (blockIdx.x == 0 && threadIdx.x == 0) atomicOr(&T.hdr->err, (u32)ERR_OVERFLOW);
            nt = cap;
        }
        for (u32 t = blockIdx.x * blockDim.x + threadIdx.x; t < nt; t += gridDim.x * blockDim.x) {
            const u32 b = batch_of_tile(lay_ex, nb, which, t);
            const BatchRec r = T.batches[b];
            const u32 tt = t - tiles_field(lay_ex[b], which);
            if (which == 1) {
                PullDesc d;
                fill_pull_desc(T, r, tt, d);
                T.tiles_a[t] = d;
            } else {
                TileDesc d;
                fill_tile_desc(T, r, tt, which == 2, d);
                (which == 0 ? T.tiles_f : T.tiles_b)[t] = d;
            }
        }
    }
}

// consumer-edge records in (producer, consumer, slot) order: what the producer adds to its
// gradient for this use, as one of a few plain formulas over the value / gradient arenas
__global__ void k_edges(Tables T)
{
    const u32 q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= T.E) return;
    const u32 e = T.succ_edge[q];
    const u32 v = T.edge_cons[e];
    const u32 lo = T.in_off[v];
    const u32 j = e - lo;
    EdgeRec r; r.kind = EK_PLAIN; r.goff = T.val_off[v]; r.voff = 0; r.a0 = 0; r.a1 = 0;
    switch (T.op[v]) {
    case OP_MATVEC: r.goff = T.dx_off[v]; break;
    case OP_ADD: break;
    case OP_CMULT: r.kind = EK_MUL; r.voff = T.val_off[T.in_idx[lo + (1 - j)]]; break;
    case OP_TANH: r.kind = EK_DTANH; r.voff = T.val_off[v]; break;
    case OP_SIGMOID: r.kind = EK_DSIGM; r.voff = T.val_off[v]; break;
    case OP_CONCAT: {
        u32 o = 0;
        for (u32 jj = 0; jj < j; ++jj) o += T.out_dim[T.in_idx[lo + jj]];
        r.goff += o;
        break;
    }
    case OP_SLICE: r.kind = EK_RANGE; r.a0 = T.aux0[v]; r.a1 = T.aux1[v]; break;
    case OP_PICK_NLS: r.kind = EK_NLS; r.voff = T.val_off[v]; r.a0 = T.aux0[v]; break;
    case OP_SQNORM: r.kind = EK_SQN; break;
    default: break;
    }
    T.edges[q] = r;
}

// ---- parameter-use items: every MATVEC is a use of W (kind 0) and of its bias (kind 1), every
// LOOKUP a use of (table, row) (kind 2).  Sorted by (parameter, kind, row), stably from
// schedule order, they give each deferred parameter-gradient reduction a fixed summation order.
__global__ void k_item_emit(Tables T, const u32 *item_base, u64 *keys, u32 *vals)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const u32 v = T.order[p];
    const u32 o = T.op[v];
    u32 i = item_base[p];
    if (o == OP_MATVEC) {
        keys[i] = ((u64)((u32)T.param[v] * 4u + 0u)) << 32; vals[i] = p; ++i;
        if (T.bias[v] >= 0) { keys[i] = ((u64)((u32)T.bias[v] * 4u + 1u)) << 32; vals[i] = p; }
    } else if (o == OP_LOOKUP) {
        keys[i] = (((u64)((u32)T.param[v] * 4u + 2u)) << 32) | (u32)T.aux0[v]; vals[i] = p;
    }
}

__global__ void k_item_finish(Tables T, const u64 *keys, const u32 *vals, u32 n_items)
{
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_items) return;
    const u64 k = keys[i];
    const u32 slot = (u32)(k >> 32);
    const u32 p = vals[i];
    const u32 v = T.order[p];
    T.it_key[i] = k;
    T.it_pos[i] = p;
    T.it_goff[i] = T.val_off[v];
    T.it_xoff[i] = (T.op[v] == OP_MATVEC) ? T.val_off[T.in_idx[T.in_off[v]]] : 0u;
    if (i == 0 || (u32)(keys[i - 1] >> 32) != slot) T.pu_start[slot] = i;
    if (i == n_items - 1 || (u32)(keys[i + 1] >> 32) != slot) T.pu_end[slot] = i + 1;
}

inline int bit_width_u32(u32 x) { int b = 0; while (x) { ++b; x >>= 1; } return b; }

}  // namespace

#define K(kern, n_threads, ...)                                                                         \
    do {                                                                                                \
        if ((n_threads) > 0) {                                                                          \
            hipLaunchKernelGGL(kern, dim3(blocks_for(n_threads)), dim3(TPB), 0, s, __VA_ARGS__);        \
            ++ctx->n_launch_sched;                                                                      \
        }                                                                                               \
    } while (0)

// Allocates the scheduler tables for n nodes / E edges in the arena and runs every stage on the
// context's stream.  Ends with one small device-to-host copy of the header and the per-step
// tile offsets (the only synchronisation of a forward call).
int sched_run(ob_ctx *ctx)
{
    Tables &T = ctx->T;
    hipStream_t s = ctx->stream;
    const u32 n = T.n, E = T.E;
    const int by_depth = ctx->mode == 1;
    ctx->n_launch_sched = 0;

    const size_t maxne = (size_t)(n > E ? n : E) + 1;
    u32 n_items = ctx->items_upto[n - 1];
    const size_t n_slots = (size_t)ctx->params.size() * 4 + 4;

    // ---- allocation (all from the caller's arena) ----
    u32 ht_size = 1;
    while (ht_size < 2 * n) ht_size <<= 1;
    if (!by_depth) ht_size = 1;
    // upper bounds of the three tile lists from sums the host keeps while nodes are added
    const size_t cap_f = (size_t)(ctx->sum_out_dim / EW_TILE) + 2 * (size_t)n + (size_t)ctx->sum_mv_d32 + 16;
    const size_t cap_a = (size_t)(ctx->sum_out_dim / EW_TILE) + (size_t)n + 16;
    const size_t cap_b = (size_t)ctx->sum_mv_k32 + 16;
#define A(field, type, count)                                               \
    do {                                                                    \
        field = arena_array<type>(ctx, (count));                            \
        if (!field) return ctx_fail(ctx, -5, "arena too small for scheduler tables (%s)", #field); \
    } while (0)
    A(T.sig, u64, n); A(T.step, u32, n); A(T.indeg, u32, n); A(T.outdeg, u32, n + 1);
    A(T.succ_off, u32, n + 1); A(T.succ_edge, u32, E + 1); A(T.edge_cons, u32, E + 1);
    A(T.queue, u32, n); A(T.qcount, u32, 64);
    A(T.ht_keys, u64, ht_size); A(T.ht_vals, u32, ht_size); A(T.ht_slot, u32, n);
    T.ht_mask = ht_size - 1;
    A(T.order, u32, n); A(T.pos_of, u32, n); A(T.batch_of_pos, u32, n); A(T.s_aux0, u32, n);
    A(T.s_in_off, u32, n + 1);
    A(T.batch_off, u32, n + 1); A(T.batches, BatchRec, n); A(T.lay, Lay, n); A(T.b_indim, u32, E + 1);
    A(T.val_off, u32, n); A(T.dx_off, u32, n); A(T.opnd_off, u32, E + 1);
    A(T.step_first, u32, n + 2); A(T.step_tf, u32, n + 2); A(T.step_ta, u32, n + 2); A(T.step_tb, u32, n + 2);
    A(T.tiles_f, TileDesc, cap_f); A(T.tiles_a, PullDesc, cap_a); A(T.tiles_b, TileDesc, cap_b);
    A(T.root_pos, u32, 64);
    A(T.edges, EdgeRec, E + 1);
    A(T.it_key, u64, n_items + 1); A(T.it_pos, u32, n_items + 1); A(T.it_goff, u32, n_items + 1);
    A(T.it_xoff, u32, n_items + 1); A(T.pu_start, u32, n_slots); A(T.pu_end, u32, n_slots);
    A(T.hdr, SchedHeader, 1);
    u32 *succ_node;
    A(succ_node, u32, E + 1);
    A(ctx->key_a, u64, maxne); A(ctx->key_b, u64, maxne); A(ctx->val_a, u32, maxne); A(ctx->val_b, u32, maxne);
    A(ctx->tmp_u32_a, u32, n + 1); A(ctx->tmp_u32_b, u32, n + 1);
    u32 *tmp_c, *tmp_d;
    A(tmp_c, u32, n + 1); A(tmp_d, u32, n + 1);
    A(ctx->lay_in, Lay, n); A(ctx->lay_total, Lay, 1);
    {
        size_t sb = prim_sort_scratch_bytes(maxne);
        size_t sc = prim_scan_scratch_bytes(maxne, sizeof(Lay));
        ctx->scratch = arena_alloc(ctx, sb > sc ? sb : sc);
        if (!ctx->scratch) return ctx_fail(ctx, -5, "arena too small for scheduler scratch");
    }
#undef A

    // ---- stage 1 ----
    HIP_TRY(ctx, hipMemsetAsync(T.hdr, 0, sizeof(SchedHeader), s));
    HIP_TRY(ctx, hipMemsetAsync(T.outdeg, 0, (size_t)(n + 1) * 4, s));
    HIP_TRY(ctx, hipMemsetAsync(T.qcount, 0, 64 * 4, s));
    HIP_TRY(ctx, hipMemsetAsync(T.pu_start, 0, n_slots * 4, s));
    HIP_TRY(ctx, hipMemsetAsync(T.pu_end, 0, n_slots * 4, s));
    K(k_node_init, n, T, by_depth);
    if (E > 0) K(k_edge_init, E, T, ctx->key_a, ctx->val_a);
    HIP_TRY(ctx, prim_scan_u32(T.outdeg, T.succ_off, (size_t)n + 1, nullptr, ctx->scratch, s));
    ctx->n_launch_sched += 3;
    if (E > 0) {
        HIP_TRY(ctx, prim_sort_pairs(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, E, 0,
                                     bit_width_u32(n - 1), ctx->scratch, s, &ctx->n_launch_sched));
        K(k_succ_finish, E, T, ctx->val_a, succ_node);
    }

    // ---- stage 2 / 3 ----
    if (by_depth) {
        hipLaunchKernelGGL(k_depth_frontier, dim3(1), dim3(FRONTIER_THREADS), 0, s, T, succ_node);
        ++ctx->n_launch_sched;
        HIP_TRY(ctx, hipMemsetAsync(T.ht_keys, 0, (size_t)ht_size * 8, s));
        HIP_TRY(ctx, hipMemsetAsync(T.ht_vals, 0xff, (size_t)ht_size * 4, s));
        K(k_rep_insert, n, T);
    }
    K(k_sort_keys, n, T, ctx->key_a, ctx->val_a, by_depth);
    if (by_depth) {
        const int lb = bit_width_u32(n - 1);
        HIP_TRY(ctx, prim_sort_pairs(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n, 0, lb, ctx->scratch, s,
                                     &ctx->n_launch_sched));
        HIP_TRY(ctx, prim_sort_pairs(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n, 32, lb, ctx->scratch, s,
                                     &ctx->n_launch_sched));
    }

    // ---- stage 4 ----
    u32 *head_flag = ctx->tmp_u32_a, *head_excl = ctx->tmp_u32_b, *s_arity = tmp_c, *s_items = tmp_d;
    K(k_heads, n, T, ctx->key_a, ctx->val_a, head_flag, s_arity, s_items);
    HIP_TRY(ctx, prim_scan_u32(head_flag, head_excl, n, nullptr, ctx->scratch, s));
    HIP_TRY(ctx, prim_scan_u32(s_arity, T.s_in_off, n, nullptr, ctx->scratch, s));
    HIP_TRY(ctx, prim_scan_u32(s_items, s_items, n, nullptr, ctx->scratch, s));
    ctx->n_launch_sched += 9;
    K(k_batch_off, n, T, head_flag, head_excl);
    K(k_batch_layout, n, T, ctx->lay_in);
    HIP_TRY(ctx, prim_scan_lay(ctx->lay_in, T.lay, n, ctx->lay_total, ctx->scratch, s));
    ctx->n_launch_sched += 3;
    K(k_batch_finish, n, T, T.lay, ctx->lay_total);
    K(k_node_offsets, n, T);
    K(k_member_check, n, T);
    if (E > 0) K(k_opnd, E, T);
    if (E > 0) K(k_edges, E, T);
    hipLaunchKernelGGL(k_tiles, dim3(1024), dim3(TPB), 0, s, T, T.lay, ctx->lay_total, (u32)cap_f, (u32)cap_a,
                       (u32)cap_b);
    ++ctx->n_launch_sched;

    // ---- parameter-use items ----
    if (n_items > 0) {
        K(k_item_emit, n, T, s_items, ctx->key_a, ctx->val_a);
        HIP_TRY(ctx, prim_sort_pairs(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n_items, 0,
                                     bit_width_u32((u32)ctx->max_param_rows), ctx->scratch, s,
                                     &ctx->n_launch_sched));
        HIP_TRY(ctx, prim_sort_pairs(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n_items, 32,
                                     bit_width_u32((u32)n_slots), ctx->scratch, s, &ctx->n_launch_sched));
        K(k_item_finish, n_items, T, ctx->key_a, ctx->val_a, n_items);
    }
    HIP_TRY(ctx, hipGetLastError());

    // ---- read back the header and the per-step tile offsets ----
    HIP_TRY(ctx, hipMemcpyAsync(ctx->hdr_pinned, T.hdr, sizeof(SchedHeader), hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    ctx->hdr = *(SchedHeader *)ctx->hdr_pinned;
    ctx->hdr.n_items = n_items;
    if (ctx->hdr.err & ERR_CYCLE)
        return ctx_fail(ctx, -6, "frontier pass resolved %u of %u nodes (cyclic or malformed graph)",
                        ctx->hdr.frontier_done, n);
    if (ctx->hdr.err & ERR_COLLISION) return ctx_fail(ctx, -6, "signature hash collision detected");
    if (ctx->hdr.err & ERR_TABLE_FULL) return ctx_fail(ctx, -6, "signature table full");
    if (ctx->hdr.err & ERR_OVERFLOW) return ctx_fail(ctx, -5, "value arena exceeds 2^32 elements");
    const u32 ns = ctx->hdr.n_steps;
    const size_t words = (size_t)ns + 1;
    if (words * 16 > ctx->hdr_pinned_bytes) {
        if (ctx->hdr_pinned) HIP_TRY(ctx, hipHostFree(ctx->hdr_pinned));
        ctx->hdr_pinned = nullptr;
        ctx->hdr_pinned_bytes = words * 16 + 4096;
        HIP_TRY(ctx, hipHostMalloc(&ctx->hdr_pinned, ctx->hdr_pinned_bytes, hipHostMallocDefault));
    }
    u32 *hp = (u32 *)ctx->hdr_pinned;
    HIP_TRY(ctx, hipMemcpyAsync(hp, T.step_tf, words * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipMemcpyAsync(hp + words, T.step_ta, words * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipMemcpyAsync(hp + 2 * words, T.step_tb, words * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipMemcpyAsync(hp + 3 * words, T.step_first, words * 4, hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipStreamSynchronize(s));
    ctx->step_tf.assign(hp, hp + words);
    ctx->step_ta.assign(hp + words, hp + 2 * words);
    ctx->step_tb.assign(hp + 2 * words, hp + 3 * words);
    ctx->step_first.assign(hp + 3 * words, hp + 4 * words);

    // ---- value and gradient arenas ----
    T.V = arena_array<float>(ctx, ctx->hdr.val_floats + VAL_ALIGN);
    T.G = arena_array<float>(ctx, ctx->hdr.grad_floats + VAL_ALIGN);
    if (!T.V || !T.G)
        return ctx_fail(ctx, -5, "arena too small: values need %llu floats, gradients %llu",
                        (unsigned long long)ctx->hdr.val_floats, (unsigned long long)ctx->hdr.grad_floats);
    return 0;
}
