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
// steps: 0 = every node is its own step, 1 = steps come from the depth pass (leaves are queued
// here), 2 = steps are the caller's batch labels.
__global__ void k_node_init(Tables T, int steps)
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
    if (steps == 1) {
        if (hi == lo) {
            const u32 pos = atomicAdd(&T.qcount[0], 1u);
            T.queue[pos] = v;
            T.step[v] = 0;
        }
    } else if (steps == 2) {
        T.step[v] = T.manual[v];   // manual batching: replaced by the label's rank once batches are cut
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

constexpr u32 DEPTH_PART = 4096;      // nodes per workgroup of the partitioned depth pass

__global__ void k_edge_init(Tables T, u64 *keys, u32 *vals)
{
    const u32 e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= T.E) return;
    const u32 v = consumer_of(T, e);
    const u32 u = T.in_idx[e];
    const u32 j = e - T.in_off[v];
    T.edge_cons[e] = v;
    atomicAdd(&T.outdeg[u], 1u);
    if (u / DEPTH_PART != v / DEPTH_PART) { atomicAdd(&T.ext_indeg[v], 1u); atomicAdd(&T.ext_left[v], 1u); }   // operand owned by another partition
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

// Partitioned frontier pass: the same dependency-counter algorithm, with the node ids cut into
// ranges of DEPTH_PART nodes, one workgroup per range.  A workgroup keeps the counters, the
// partial depths, its frontier queue and the successor lists of its range in LDS, so advancing
// its frontier costs LDS latency only.  An edge into another range resolves through global
// atomics: the producer raises the consumer's depth bound and lowers its count of unresolved
// external operands; whoever resolves the last one posts the node to the owner's inbox, where it
// counts as one more resolved dependency.  Ids are a topological order, so a range only ever
// waits for lower ranges and the lowest never waits, whenever each workgroup happens to start (a
// range reads its nodes' external counts from the fixed copy, never from the counters that lower
// ranges are already taking down); every wait is bounded.
constexpr u32 DEPTH_SCAP = 12288;     // successor entries of a range held in LDS
constexpr u32 DEPTH_THREADS = 256;    // set-up and write-out; in between the waves have roles of their own
constexpr u32 DEPTH_MAX_PARTS = 240;
constexpr u32 DEPTH_NONE = 0xffffffffu;
constexpr u32 DEPTH_UNROLL = 2;       // successors of a frontier node handled per pass of the inner loop
constexpr u32 DEPTH_OUT_CAP = 1024;   // ring of resolutions that leave the range, waiting for the wave that posts them

__device__ inline u32 lds_load(const u32 *p) { return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP); }

// A resolution that leaves the range: raise the consumer's depth bound, take one of its external
// dependencies off; whoever takes the last one posts the node to its owner's inbox.
__device__ inline void depth_post_external(const Tables &T, u32 sn, u32 d1, u32 *g_dep, u32 *inbox, u32 *inbox_tail)
{
    atomicMax(&g_dep[sn], d1);
    __threadfence();
    if (atomicSub(&T.ext_left[sn], 1u) == 1u) {
        const u32 k2 = sn / DEPTH_PART;
        const u32 slot = atomicAdd(&inbox_tail[k2], 1u);
        __hip_atomic_store(&inbox[k2 * DEPTH_PART + slot], sn, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
}

__global__ __launch_bounds__(DEPTH_THREADS) void k_depth_partitioned(Tables T, const u32 *succ_node, u32 *g_dep,
                                                                         u32 *inbox, u32 *inbox_tail, u32 spin_limit)
{
    __shared__ u32 s_pending[DEPTH_PART];
    __shared__ u32 s_dep[DEPTH_PART];
    __shared__ unsigned short s_queue[DEPTH_PART];
    __shared__ u32 s_soff[DEPTH_PART + 1];
    __shared__ u32 s_snode[DEPTH_SCAP];
    __shared__ u32 s_out_sn[DEPTH_OUT_CAP], s_out_d1[DEPTH_OUT_CAP];
    __shared__ unsigned short s_in[DEPTH_PART];
    __shared__ u32 s_next, s_done, s_out_tail, s_out_head, s_in_tail, s_fin;
    const u32 tid = threadIdx.x;
    const u32 k = blockIdx.x;
    const u32 lo = k * DEPTH_PART;
    const u32 hi = lo + DEPTH_PART < T.n ? lo + DEPTH_PART : T.n;
    const u32 cnt = hi - lo;
    const u32 ebase = T.succ_off[lo];
    const u32 ecnt = T.succ_off[hi] - ebase;
    if (tid == 0) { s_next = 0; s_done = 0; s_out_tail = 0; s_out_head = 0; s_in_tail = 0; s_fin = 0; }
    __syncthreads();
    for (u32 i = tid; i < cnt; i += DEPTH_THREADS) {
        const u32 v = lo + i;
        const u32 ext = T.ext_indeg[v];
        const u32 pend = T.indeg[v] - ext + (ext ? 1u : 0u);
        s_pending[i] = pend;
        s_dep[i] = 0;
        s_soff[i] = T.succ_off[v] - ebase;
        if (pend == 0) s_queue[atomicAdd(&s_next, 1u)] = (unsigned short)i;
    }
    if (tid == 0) s_soff[cnt] = ecnt;
    for (u32 e = tid; e < ecnt && e < DEPTH_SCAP; e += DEPTH_THREADS) s_snode[e] = succ_node[ebase + e];
    __syncthreads();
    // The frontier of a range is small (tens of nodes per level), so after the cooperative set-up
    // wave 0 runs the level loop alone: its LDS operations complete in program order, the loop state
    // (head, tail, counters) sits in scalar registers, new frontier entries get their queue
    // positions from a ballot, and nothing in the loop waits for global memory.  Traffic with other
    // ranges goes through the two helper waves: wave 1 watches this range's inbox (coherent memory)
    // and hands what arrives to wave 0 through LDS, depth bound already applied; wave 2 takes the
    // resolutions that leave the range from a ring in LDS and posts them with global atomics.
    const u32 wave = tid >> 6, lane = tid & 63u;
    const u64 lt_mask = (1ull << lane) - 1ull;
    if (wave == 0) {
        u32 head = 0, tail = __builtin_amdgcn_readfirstlane(s_next), done = 0, seen = 0, spin = 0, out_tail = 0;
        while (!(head == tail && done == cnt)) {
            const u32 avail = __builtin_amdgcn_readfirstlane(__hip_atomic_load(&s_in_tail, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
            u32 new_tail = tail;
            for (u32 base = head; base < tail; base += 64) {
                const u32 i = base + lane;
                const bool act = i < tail;
                const u32 ul = act ? s_queue[i] : 0u;
                const u32 d1 = s_dep[ul] + 1u;
                u32 e = s_soff[ul];
                const u32 e1 = act ? s_soff[ul + 1] : e;
                while (__ballot(e < e1) != 0ull) {
                    // two successors per pass (most nodes have one or two): the loop is bound by the number of
                    // instructions the one wave issues, so the common case is kept short
                    u32 sn[DEPTH_UNROLL], was[DEPTH_UNROLL];
                    bool any_ext = false;
#pragma unroll
                    for (u32 j = 0; j < DEPTH_UNROLL; ++j)
                        sn[j] = e + j < e1 ? (e + j < DEPTH_SCAP ? s_snode[e + j] : succ_node[ebase + e + j]) : DEPTH_NONE;
#pragma unroll
                    for (u32 j = 0; j < DEPTH_UNROLL; ++j) {   // successors have larger ids than their producer, so sn >= lo
                        was[j] = 0;
                        if (sn[j] < hi) { atomicMax(&s_dep[sn[j] - lo], d1); was[j] = atomicSub(&s_pending[sn[j] - lo], 1u); }
                        else any_ext = any_ext || sn[j] != DEPTH_NONE;
                    }
#pragma unroll
                    for (u32 j = 0; j < DEPTH_UNROLL; ++j) {
                        const bool ready = was[j] == 1u;
                        const u64 m = __ballot(ready);
                        if (ready) s_queue[new_tail + (u32)__popcll(m & lt_mask)] = (unsigned short)(sn[j] - lo);
                        new_tail += (u32)__popcll(m);
                    }
                    if (__ballot(any_ext) != 0ull) {
#pragma unroll
                        for (u32 j = 0; j < DEPTH_UNROLL; ++j) {
                            const bool ext = sn[j] != DEPTH_NONE && sn[j] >= hi;
                            const u64 m = __ballot(ext);
                            if (m == 0ull) continue;
                            const u32 c = (u32)__popcll(m);
                            if (out_tail + c - lds_load(&s_out_head) <= DEPTH_OUT_CAP) {
                                if (ext) {
                                    const u32 pos = (out_tail + (u32)__popcll(m & lt_mask)) % DEPTH_OUT_CAP;
                                    s_out_sn[pos] = sn[j]; s_out_d1[pos] = d1;
                                }
                                out_tail += c;
                                __hip_atomic_store(&s_out_tail, out_tail, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
                            } else if (ext) {
                                depth_post_external(T, sn[j], d1, g_dep, inbox, inbox_tail);   // ring full: post it here
                            }
                        }
                    }
                    e += DEPTH_UNROLL;
                }
            }
            // what wave 1 took from the inbox: the node's depth bound is applied, one dependency comes off
            for (u32 base = seen; base < avail; base += 64) {
                const u32 j = base + lane;
                bool ready = false;
                u32 sl = 0;
                if (j < avail) { sl = s_in[j]; ready = atomicSub(&s_pending[sl], 1u) == 1u; }
                const u64 m = __ballot(ready);
                if (ready) s_queue[new_tail + (u32)__popcll(m & lt_mask)] = (unsigned short)sl;
                new_tail += (u32)__popcll(m);
            }
            __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
            done += tail - head;
            const bool idle = head == tail && new_tail == tail && seen == avail;   // nothing to do: waiting for another range
            seen = avail;
            head = tail;
            tail = new_tail;
            if (idle) {
                if (++spin > spin_limit) break;     // bounded: the host then runs the single-workgroup pass instead
                __builtin_amdgcn_s_sleep(4);
            } else {
                spin = 0;
            }
        }
        if (lane == 0) s_done = done;
        __hip_atomic_store(&s_fin, 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
    } else if (wave == 1) {
        // inbox entries are posted after their slot is reserved: take them in order, stop at a hole
        u32 seen = 0;
        while (lds_load(&s_fin) == 0u) {
            const u32 avail = __builtin_amdgcn_readfirstlane(__hip_atomic_load(&inbox_tail[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
            if (seen >= avail) { __builtin_amdgcn_s_sleep(2); continue; }
            const u32 j = seen + lane;
            u32 sn = DEPTH_NONE;
            if (j < avail) sn = __hip_atomic_load(&inbox[k * DEPTH_PART + j], __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT);
            const u32 in_chunk = avail - seen < 64u ? avail - seen : 64u;
            const u64 holes = __ballot(j < avail && sn == DEPTH_NONE);
            const u32 good = holes ? (u32)__builtin_ctzll(holes) : in_chunk;
            if (lane < good) {
                const u32 sl = sn - lo;
                atomicMax(&s_dep[sl], __hip_atomic_load(&g_dep[sn], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                s_in[j] = (unsigned short)sl;
            }
            seen += good;
            if (good) __hip_atomic_store(&s_in_tail, seen, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    } else if (wave == 2) {
        u32 head = 0;
        while (true) {
            const u32 fin = lds_load(&s_fin);
            const u32 tail = __builtin_amdgcn_readfirstlane(__hip_atomic_load(&s_out_tail, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_WORKGROUP));
            if (head == tail) {
                if (fin) break;
                __builtin_amdgcn_s_sleep(1);
                continue;
            }
            const u32 j = head + lane;
            if (j < tail) depth_post_external(T, s_out_sn[j % DEPTH_OUT_CAP], s_out_d1[j % DEPTH_OUT_CAP], g_dep, inbox, inbox_tail);
            head += tail - head < 64u ? tail - head : 64u;
            __hip_atomic_store(&s_out_head, head, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_WORKGROUP);
        }
    }
    __syncthreads();
    for (u32 i = tid; i < cnt; i += DEPTH_THREADS) T.step[lo + i] = s_dep[i];
    if (tid == 0) {
        atomicAdd(&T.hdr->frontier_done, s_done);
        if (s_done != cnt) atomicOr(&T.hdr->err, (u32)ERR_CYCLE);
    }
}

// ---- agenda-based batching (Section 3.2, second strategy) -------------------------------------------
// The agenda holds the nodes whose operands are all resolved.  Each iteration takes every
// available node of one signature as a batch; the signature is the one with the smallest average
// depth over ALL nodes of the graph that carry it (a fixed number per signature), equal averages
// go to the cheaper operation class (leaf < component-wise / copy < per-row reduction < matrix
// product), then to the signature whose first node has the smaller id.  Because the priority of a
// signature never changes, signatures are ranked once; the agenda is then one ready list per rank
// and "select" is the lowest rank with a non-empty list.  The iteration index becomes the node's
// step, and everything downstream (grouping by (step, signature), layout, launch plan) is shared
// with depth-based batching.
constexpr u32 AG_TABLE = 4096;        // open-addressing table of signatures
constexpr u32 AG_MAX_CLASSES = 1024;  // distinct signatures an agenda plan can rank
constexpr u32 AG_NONE = 0xffffffffu;

struct AgendaTables {
    u64 *keys;        // [AG_TABLE] signature hash, 0 = empty
    u64 *sum;         // [AG_TABLE] sum of depths
    u32 *cnt;         // [AG_TABLE] nodes
    u32 *first;       // [AG_TABLE] smallest node id
    u32 *op;          // [AG_TABLE] operation of the signature
    u32 *rank_of;     // [AG_TABLE] rank of the signature in a table slot
    u32 *seg_off;     // [AG_MAX_CLASSES + 1] ready-list segment of each rank inside `seg`
    u32 *n_classes;   // [1]
    u32 *cls;         // [n] rank of each node's signature
    u32 *pending;     // [n] unresolved operands
    u32 *seg;         // [n] ready lists, one segment per rank (each node is appended once)
};

__device__ inline u32 ag_cost_class(u32 op)
{
    if (op == OP_INPUT || op == OP_LOOKUP) return 0;
    if (op == OP_MATVEC) return 3;
    if (op == OP_PICK_NLS || op == OP_SQNORM) return 2;
    return 1;
}

// per node: find / create the table entry of its signature and add (depth, 1, id) to it.  Lanes
// of a wave that carry the same signature are combined first, so the table sees one update per
// distinct signature per wave.
__global__ void k_class_insert(Tables T, AgendaTables A)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    const u32 lane = threadIdx.x & 63;
    const bool active = v < T.n;
    const u64 sig = active ? (T.sig[v] ? T.sig[v] : 1ull) : 0ull;
    const u32 depth = active ? T.step[v] : 0u;
    u64 todo = __ballot(active);
    u32 my_slot = 0;
    while (todo) {
        const u32 leader = (u32)__builtin_ctzll(todo);
        const u64 lsig = ((u64)(u32)__builtin_amdgcn_readlane((int)(u32)(sig >> 32), leader) << 32) |
                         (u32)__builtin_amdgcn_readlane((int)(u32)sig, leader);
        const bool mine = active && sig == lsig;
        const u64 match = __ballot(mine);
        u32 dsum = mine ? depth : 0u;
        for (int o = 32; o > 0; o >>= 1) dsum += __shfl_xor(dsum, o);
        u32 slot = 0;
        if (lane == leader) {
            slot = (u32)(lsig * 0x9e3779b97f4a7c15ull >> 52) & (AG_TABLE - 1);
            bool placed = false;
            for (u32 probe = 0; probe < AG_TABLE; ++probe) {
                const u64 old = atomicCAS((unsigned long long *)&A.keys[slot], 0ULL, (unsigned long long)lsig);
                if (old == 0 || old == lsig) { placed = true; break; }
                slot = (slot + 1) & (AG_TABLE - 1);
            }
            if (!placed) { atomicOr(&T.hdr->err, (u32)ERR_CLASSES); slot = 0; }
            else {
                atomicAdd(&A.cnt[slot], (u32)__popcll(match));
                atomicAdd((unsigned long long *)&A.sum[slot], (unsigned long long)dsum);
                atomicMin(&A.first[slot], v);     // the leader is the lowest matching lane: the smallest id of the wave
                A.op[slot] = T.op[v];
            }
        }
        slot = (u32)__builtin_amdgcn_readlane((int)slot, leader);
        if (mine) my_slot = slot;
        todo &= ~match;
    }
    if (active) T.ht_slot[v] = my_slot;
}

// One workgroup: collect the used table entries, rank them, lay out the ready-list segments.
__global__ __launch_bounds__(1024) void k_class_rank(Tables T, AgendaTables A)
{
    __shared__ u32 s_n;
    __shared__ u32 s_slot[AG_MAX_CLASSES];
    __shared__ u64 s_sum[AG_MAX_CLASSES];
    __shared__ u32 s_cnt[AG_MAX_CLASSES];
    __shared__ u32 s_key2[AG_MAX_CLASSES];   // cost class
    __shared__ u32 s_first[AG_MAX_CLASSES];
    __shared__ u32 s_cnt_by_rank[AG_MAX_CLASSES];
    const u32 tid = threadIdx.x;
    if (tid == 0) s_n = 0;
    __syncthreads();
    for (u32 slot = tid; slot < AG_TABLE; slot += 1024) {
        if (A.keys[slot] != 0) {
            const u32 i = atomicAdd(&s_n, 1u);
            if (i < AG_MAX_CLASSES) s_slot[i] = slot;
        }
    }
    __syncthreads();
    u32 C = s_n;
    if (C > AG_MAX_CLASSES) { if (tid == 0) atomicOr(&T.hdr->err, (u32)ERR_CLASSES); C = AG_MAX_CLASSES; }
    if (tid < C) {
        const u32 slot = s_slot[tid];
        s_sum[tid] = A.sum[slot]; s_cnt[tid] = A.cnt[slot];
        s_key2[tid] = ag_cost_class(A.op[slot]); s_first[tid] = A.first[slot];
    }
    __syncthreads();
    if (tid < C) {
        // rank = number of signatures taken before this one (first ids differ, so the order is strict)
        const u64 si = s_sum[tid]; const u32 ci = s_cnt[tid], ki = s_key2[tid], fi = s_first[tid];
        u32 rank = 0;
        for (u32 j = 0; j < C; ++j) {
            const u64 lhs = s_sum[j] * ci, rhs = si * s_cnt[j];    // avg_j < avg_i  <=>  sum_j * cnt_i < sum_i * cnt_j
            bool before = lhs < rhs;
            if (lhs == rhs) before = s_key2[j] < ki || (s_key2[j] == ki && s_first[j] < fi);
            rank += before ? 1u : 0u;
        }
        A.rank_of[s_slot[tid]] = rank;
        s_cnt_by_rank[rank] = ci;
    }
    __syncthreads();
    if (tid == 0) {
        u32 acc = 0;
        for (u32 r = 0; r < C; ++r) { A.seg_off[r] = acc; acc += s_cnt_by_rank[r]; }
        A.seg_off[C] = acc;
        A.n_classes[0] = C;
    }
}

// per node: rank of its signature, and one word holding that rank above the count of unresolved
// operands ((rank << 22) | count), so that the decrement that resolves the last operand also
// tells which ready list the node joins
constexpr u32 AG_COUNT_BITS = 22;
__global__ void k_class_of(Tables T, AgendaTables A)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n) return;
    const u32 rank = A.rank_of[T.ht_slot[v]];
    A.cls[v] = rank;
    // the operand count comes from the graph itself: the single-workgroup depth pass counts T.indeg down to zero
    const u32 arity = T.in_off[v + 1] - T.in_off[v];
    if (arity >> AG_COUNT_BITS) atomicOr(&T.hdr->err, (u32)ERR_CLASSES);
    A.pending[v] = (rank << AG_COUNT_BITS) | arity;
}

// One workgroup runs the agenda.  head / tail of every rank's ready list live in LDS; the lists
// themselves, the dependency counters and the successor lists are in global memory (this
// workgroup's L2).  Nodes that become available while a batch is being taken are appended behind
// the batch's end, so a node never joins the batch of one of its own operands.
constexpr int AGENDA_THREADS = 1024;
__global__ __launch_bounds__(AGENDA_THREADS) void k_agenda(Tables T, AgendaTables A, const u32 *succ_node)
{
    __shared__ u32 s_head[AG_MAX_CLASSES], s_tail[AG_MAX_CLASSES], s_off[AG_MAX_CLASSES + 1];
    __shared__ u32 s_min, s_done, s_t;
    const u32 tid = threadIdx.x;
    const u32 C = A.n_classes[0] < AG_MAX_CLASSES ? A.n_classes[0] : AG_MAX_CLASSES;
    for (u32 c = tid; c < C; c += AGENDA_THREADS) { s_head[c] = 0; s_tail[c] = 0; }
    for (u32 c = tid; c <= C; c += AGENDA_THREADS) s_off[c] = A.seg_off[c];
    if (tid == 0) { s_min = AG_NONE; s_done = 0; s_t = 0; }
    __syncthreads();
    for (u32 v = tid; v < T.n; v += AGENDA_THREADS) {
        const u32 w = A.pending[v];
        if ((w & ((1u << AG_COUNT_BITS) - 1u)) == 0) {
            const u32 c = w >> AG_COUNT_BITS;
            A.seg[s_off[c] + atomicAdd(&s_tail[c], 1u)] = v;
        }
    }
    __syncthreads();
    while (true) {
        for (u32 c = tid; c < C; c += AGENDA_THREADS)
            if (s_tail[c] > s_head[c]) atomicMin(&s_min, c);
        __syncthreads();
        const u32 c = s_min;
        if (c == AG_NONE) break;          // nothing available: all done, or a cycle
        const u32 lo = s_head[c], hi = s_tail[c], base = s_off[c], t = s_t;
        __syncthreads();
        for (u32 i = lo + tid; i < hi; i += AGENDA_THREADS) {
            const u32 v = A.seg[base + i];
            T.step[v] = t;
            const u32 e1 = T.succ_off[v + 1];
            for (u32 e = T.succ_off[v]; e < e1; ++e) {
                const u32 sn = succ_node[e];
                const u32 was = atomicSub(&A.pending[sn], 1u);
                if ((was & ((1u << AG_COUNT_BITS) - 1u)) == 1u) {
                    const u32 cs = was >> AG_COUNT_BITS;
                    A.seg[s_off[cs] + atomicAdd(&s_tail[cs], 1u)] = sn;
                }
            }
        }
        __syncthreads();
        if (tid == 0) { s_head[c] = hi; s_done += hi - lo; s_t = t + 1; s_min = AG_NONE; }
        __syncthreads();
    }
    if (tid == 0 && s_done != T.n) atomicOr(&T.hdr->err, (u32)ERR_CYCLE);
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
    // Thousands of nodes share a key: a node first looks (keys never change once set, values only fall, so
    // whatever a look returns is safe to act on) and takes the atomic path only for an empty slot or a value
    // above its own id; low ids mostly run first, so most nodes end up with two reads.
    for (u32 probe = 0; probe <= T.ht_mask; ++probe) {
        u64 cur = __hip_atomic_load(&T.ht_keys[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (cur == 0) {
            cur = atomicCAS((unsigned long long *)&T.ht_keys[slot], 0ULL, (unsigned long long)k);
            if (cur == 0) cur = k;
        }
        if (cur == k) {
            if (__hip_atomic_load(&T.ht_vals[slot], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) > v) atomicMin(&T.ht_vals[slot], v);
            T.ht_slot[v] = slot;
            return;
        }
        slot = (slot + 1) & T.ht_mask;
    }
    atomicOr(&T.hdr->err, (u32)ERR_TABLE_FULL);
    T.ht_slot[v] = 0;
}

// rep_src: 0 = the node itself (unbatched), 1 = the representative found by k_rep_insert,
// 2 = none (manual batching: one batch per step, the stable sort keeps ids ascending)
__global__ void k_sort_keys(Tables T, u64 *keys, u32 *vals, int rep_src)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n) return;
    const u32 rep = rep_src == 1 ? T.ht_vals[T.ht_slot[v]] : (rep_src == 2 ? 0u : v);
    keys[v] = ((u64)T.step[v] << 32) | rep;
    vals[v] = v;
}

// ---- stage 4: batches from the sorted order -----------------------------------------------------
__global__ void k_heads(Tables T, const u64 *skey, const u32 *sval, u32 *head_flag, Tri *counts)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const u32 v = sval[p];
    T.order[p] = v;
    T.pos_of[v] = p;
    T.s_aux0[p] = (u32)T.aux0[v];
    Tri c;
    c.a = (p == 0 || skey[p] != skey[p - 1]) ? 1u : 0u;
    const u32 o = T.op[v];
    c.b = (o == OP_MATVEC) ? XP_MAX : T.in_off[v + 1] - T.in_off[v];   // a product's operand may be listed in up to XP_MAX pieces
    c.c = (o == OP_MATVEC) ? (1u + (T.bias[v] >= 0 ? 1u : 0u)) : (o == OP_LOOKUP ? 1u : 0u);
    c.d = 0;
    head_flag[p] = c.a;
    counts[p] = c;
}

__global__ void k_batch_off(Tables T, const u32 *head_flag, const Tri *before, u32 *item_base, int manual)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    const Tri ex = before[p];          // batch heads, operand references and parameter uses before position p
    const u32 b = ex.a + head_flag[p] - 1;
    T.s_in_off[p] = ex.b;
    item_base[p] = ex.c;
    T.batch_of_pos[p] = b;
    if (manual) T.step[T.order[p]] = b;   // labels need not be dense: a batch's step is its rank
    if (head_flag[p]) T.batch_off[b] = p;
    if (p == T.n - 1) {
        T.batch_off[b + 1] = T.n;
        T.hdr->n_batches = b + 1;
    }
}

__host__ __device__ inline u32 cdiv(u64 a, u32 b) { return (u32)((a + b - 1) / b); }

// one thread per batch: record + sizes for the layout scan (entries b >= n_batches are zero)
__global__ void k_batch_layout(Tables T, Lay *lay_in, int virt)
{
    const u32 b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= T.n) return;
    Lay L; L.val = 0; L.dx = 0; L.ind = L.p0 = L.p1 = L.p2 = 0;
    if (b < T.hdr->n_batches) {
        const u32 p0 = T.batch_off[b], B = T.batch_off[b + 1] - p0;
        const u32 h = T.order[p0];
        BatchRec r;
        r.pos0 = p0; r.B = B; r.op = T.op[h]; r.d = T.out_dim[h];
        r.arity = T.in_off[h + 1] - T.in_off[h];
        r.param = T.param[h]; r.bias = T.bias[h];
        r.aux0 = T.aux0[h]; r.aux1 = T.aux1[h];
        if (r.op == OP_MATVEC) { r.aux0 = -1; r.aux1 = 0; }
        r.step = T.step[h];
        r.k = r.arity ? T.out_dim[T.in_idx[T.in_off[h]]] : 0;
        r.val_off = r.dx_off = r.indim = 0;
        r.opnd = T.s_in_off[p0];
        r.vec4 = TF_VEC4 | TF_ALIGNED | TF_G_ALIAS;   // cleared below by whatever a member violates
        if (r.op == OP_MATVEC && B >= WIDE_MIN_ROWS && r.d >= (u32)GTW) r.vec4 |= TF_WIDE;
        if (r.op == OP_SLICE) r.vec4 |= TF_VIEW;
        if (r.op == OP_CONCAT && virt) r.vec4 |= TF_VIRT;   // taken back by k_node_offsets / k_opnd
        if (r.op == OP_MATVEC && virt) r.vec4 |= TF_XP;     // taken back by k_xp_check
        T.batches[b] = r;
        const u64 vs = (u64)B * r.d;
        L.val = (vs + VAL_ALIGN - 1) / VAL_ALIGN * VAL_ALIGN;
        if (r.op == OP_MATVEC) {
            const u64 xs = (u64)B * r.k;
            L.dx = (xs + VAL_ALIGN - 1) / VAL_ALIGN * VAL_ALIGN;
        }
        L.ind = r.op == OP_MATVEC ? XP_MAX : r.arity;
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
    if (b == nb - 1) {
        T.hdr->n_steps = r.step + 1;
        T.hdr->val_floats = tot.val;
        T.hdr->grad_floats = tot.val + tot.dx;
        if (tot.val + tot.dx >= 0xffffffffULL) atomicOr(&T.hdr->err, (u32)ERR_OVERFLOW);
    }
}

__global__ void k_node_offsets(Tables T)
{
    const u32 p = blockIdx.x * blockDim.x + threadIdx.x;
    if (p >= T.n) return;
    BatchRec &r = T.batches[T.batch_of_pos[p]];
    const u32 row = p - r.pos0;
    const u32 v = T.order[p];
    T.val_off[v] = T.nat_off[v] = r.val_off + row * r.d;
    T.dx_off[v] = (r.op == OP_MATVEC) ? r.dx_off + row * r.k : 0u;
    // a CONCAT batch can stay uncopied only with at most XP_MAX pieces whose dimensions are multiples of 4
    if (r.op == OP_CONCAT && (r.vec4 & TF_VIRT)) {
        const u32 ar = T.in_off[v + 1] - T.in_off[v];
        bool ok = ar <= XP_MAX;
        for (u32 j = 0; ok && j < ar; ++j) ok = (T.out_dim[T.in_idx[T.in_off[v] + j]] & 3u) == 0;
        if (!ok) atomicAnd(&r.vec4, ~(u32)TF_VIRT);
    }
    // a product whose operand is a CONCAT node: the lowest such CONCAT batch gives the piece structure of the batch
    if (r.op == OP_MATVEC && (r.vec4 & TF_XP)) {
        const u32 x = T.in_idx[T.in_off[v]];
        if (T.op[x] == OP_CONCAT) atomicMin((u32 *)&r.aux0, T.batch_of_pos[T.pos_of[x]]);
    }
}

// SLICE nodes are views: their value is the range [lo, hi) of the operand's row where it lies
// (through any number of slices of slices), so nothing is copied forward and every reader of the
// node is pointed there.  Their gradient rows stay in their own batch's block (nat_off).
__global__ void k_view_offsets(Tables T)
{
    const u32 v = blockIdx.x * blockDim.x + threadIdx.x;
    if (v >= T.n || T.op[v] != OP_SLICE) return;
    u32 x = v, acc = 0;
    while (T.op[x] == OP_SLICE) { acc += (u32)T.aux0[x]; x = T.in_idx[T.in_off[x]]; }   // ids fall: ends at a node that owns its row
    T.val_off[v] = T.nat_off[x] + acc;
}

// CONCAT batches that only matrix products read are not copied (Section 3.3: operands that already lie in
// memory are used where they are): the product reads each row's pieces from their producers' rows.  This needs
// one piece structure per product batch.  Per product row whose operand is a CONCAT node: its pieces must
// have the dimensions of the batch's reference CONCAT batch (aux0), which must itself qualify; rows with any
// other operand are read whole, which every piece structure allows.  (The reference batch and the CONCAT batches
// that qualify at all were settled by k_node_offsets.)
__device__ inline void xp_check(const Tables &T, u32 p, BatchRec &r)
{
    if (r.op != OP_MATVEC || !(r.vec4 & TF_XP) || r.aux0 < 0) return;
    const u32 x = T.in_idx[T.in_off[T.order[p]]];
    if (T.op[x] != OP_CONCAT) return;
    const BatchRec &rr = T.batches[r.aux0];
    const u32 hr = T.order[rr.pos0];
    const u32 P = rr.arity;
    bool ok = (rr.vec4 & TF_VIRT) && T.in_off[x + 1] - T.in_off[x] == P;
    for (u32 j = 0; ok && j < P; ++j) ok = T.out_dim[T.in_idx[T.in_off[x] + j]] == T.out_dim[T.in_idx[T.in_off[hr] + j]];
    if (!ok) { atomicAnd(&r.vec4, ~(u32)TF_XP); return; }
    if (T.batch_of_pos[T.pos_of[x]] == (u32)r.aux0) {   // (every such row writes the same values)
        r.aux1 = (i32)P;
        for (u32 j = 0; j < P; ++j) T.b_indim[r.indim + j] = T.out_dim[T.in_idx[T.in_off[x] + j]];
    }
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
    if (!vec) atomicAnd(&r.vec4, ~(u32)TF_VEC4);
    // A one-element MATVEC node may become the backward root (chosen after scheduling): its gradient is
    // the seed, not its consumer's row, so such batches never alias.
    if (r.op == OP_MATVEC && (T.outdeg[v] != 1 || r.d == 1)) atomicAnd(&r.vec4, ~(u32)TF_G_ALIAS);
    xp_check(T, p, r);
}

__device__ inline bool batch_xp(const BatchRec &r) { return r.op == OP_MATVEC && (r.vec4 & TF_XP) && r.aux1 > 0; }

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
    const bool xp = batch_xp(r);
    // an edge into a CONCAT node: any reader that is not a product reading in pieces needs the row in place
    if (T.op[u] == OP_CONCAT && !xp) {
        BatchRec &ru = T.batches[T.batch_of_pos[T.pos_of[u]]];
        if (ru.vec4 & TF_VIRT) atomicAnd(&ru.vec4, ~(u32)TF_VIRT);
    }
    if (xp) {
        // the operand in pieces: the rows of a CONCAT node's operands (where the producers left them, whether or
        // not the CONCAT batch ends up copied for another reader's sake), or the whole row once per piece
        const u32 P = (u32)r.aux1;
        const bool pieces = T.op[u] == OP_CONCAT;
        u32 start = 0;
        for (u32 q = 0; q < P; ++q) {
            u32 off = T.val_off[u];
            if (pieces) { const u32 w = T.in_idx[T.in_off[u] + q]; off = T.val_off[w] - start; start += T.out_dim[w]; }
            T.opnd_off[r.opnd + q * r.B + row] = off;
            if (off & 3u) atomicAnd(&r.vec4, ~(u32)(TF_VEC4 | TF_ALIGNED));
        }
        return;
    }
    const u32 off = T.val_off[u];
    T.opnd_off[r.opnd + j * r.B + row] = off;
    if (row == 0) T.b_indim[r.indim + j] = du;
    if (off & 3u) atomicAnd(&r.vec4, ~(u32)(TF_VEC4 | TF_ALIGNED));
    else if (r.op == OP_CONCAT && (du & 3u)) atomicAnd(&r.vec4, ~(u32)TF_VEC4);
}

// ---- launch planning ---------------------------------------------------------------------------------
// The schedule (which nodes form a batch, and the order of batches) is fixed above.  What follows
// only decides which batches share a kernel launch.  Component-wise batches whose operands are
// row-aligned with their producer (row r reads row r) can run in the producer's launch: a
// workgroup that owns a block of rows walks such a chain with workgroup barriers, no grid-wide
// synchronisation is needed.  Every other dependency costs one launch boundary.

__device__ inline bool op_chainable(u32 op, u32 arity)
{
    switch (op) {
    case OP_ADD: return arity < (u32)WIDE_ADD_ARITY;
    case OP_CMULT: case OP_TANH: case OP_SIGMOID: case OP_CONCAT: case OP_SLICE: return true;
    default: return false;
    }
}
__device__ inline bool op_chain_source(u32 op, u32 arity)
{
    return op == OP_INPUT || op == OP_LOOKUP || op_chainable(op, arity);
}

// producer batch of operand slot j of the node at schedule position p, and the producer's row
__device__ inline u32 producer_batch(const Tables &T, u32 p, u32 j, u32 *prow)
{
    const u32 v = T.order[p];
    const u32 pu = T.pos_of[T.in_idx[T.in_off[v] + j]];
    const u32 by = T.batch_of_pos[pu];
    *prow = pu - T.batches[by].pos0;
    return by;
}

constexpr u32 FUSE_MAX_MULT = 4;
__device__ inline u32 gcd_u32(u32 a, u32 b) { while (b) { const u32 t = a % b; a = b; b = t; } return a; }

// Batch-level dependencies.  Per graph edge: consumer batch, producer batch, and whether a launch
// boundary is needed.  The edge can be fused (weight 0) when both batches are component-wise (the
// producer may also be a leaf) and, with G = gcd of the two row counts, the consumer row and the
// producer row lie in the same group (consumer group = row / (B_cons / G), producer group =
// row / (B_prod / G)).  A group may hold at most FUSE_MAX_MULT rows of a batch: fusing must keep
// that many independent groups, or a fused launch would serialise what a launch per level runs
// wide.  Two batches end up in one slot only if every edge between them is fusable (any other
// edge pushes the consumer to a later slot), so the test is per edge.  Distinct (consumer,
// producer, weight) triples are collected once each through a hash set.
constexpr u32 SLOT_MAX_NB = 4096;     // batches a fused plan can hold (12-bit ids)
constexpr u32 BSET_SIZE = 1u << 16;   // open-addressing set of packed triples
constexpr u32 BLIST_MAX = 20480;      // distinct triples the slot kernel keeps in LDS (80 KB)
constexpr int SLOT_BITS = 13;         // bits of a slot or a label when the plan is fused

__global__ void k_bedges(Tables T, u32 *bset, u32 *blist)
{
    const u32 e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= T.E) return;
    if (T.hdr->n_batches > SLOT_MAX_NB) return;
    const u32 v = T.edge_cons[e];
    const u32 j = e - T.in_off[v];
    const u32 p = T.pos_of[v];
    const u32 b = T.batch_of_pos[p];
    const BatchRec &r = T.batches[b];
    u32 prow;
    const u32 by = producer_batch(T, p, j, &prow);
    const BatchRec &y = T.batches[by];
    bool ok = op_chainable(r.op, r.arity) && op_chain_source(y.op, y.arity);
    if (ok) {
        const u32 G = gcd_u32(r.B, y.B);
        const u32 mc = r.B / G, mp = y.B / G;
        ok = mc <= FUSE_MAX_MULT && mp <= FUSE_MAX_MULT && (p - r.pos0) / mc == prow / mp;
    }
    const u32 key = ((b << 13) | (by << 1) | (ok ? 0u : 1u)) + 1u;
    u32 h = (key * 2654435761u) & (BSET_SIZE - 1);
    for (u32 probe = 0; probe < BSET_SIZE; ++probe) {
        // (all edges between two batches carry the same triple: look before the compare-and-swap)
        u32 old = __hip_atomic_load(&bset[h], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (old == key) return;
        if (old == 0u) old = atomicCAS(&bset[h], 0u, key);
        if (old == key) return;
        if (old == 0u) {
            const u32 i = atomicAdd(&T.hdr->n_bedges, 1u);
            if (i < BLIST_MAX) blist[i] = key;
            return;
        }
        h = (h + 1) & (BSET_SIZE - 1);
    }
    atomicAdd(&T.hdr->n_bedges, BLIST_MAX);   // table full: forces the unfused plan
}

// One workgroup.  Over the batch dependencies, where a fusable edge costs 0 and any other edge one
// launch boundary: head(b) = longest path from any source to b, tail(b) = longest path from b to any
// sink.  Batch ids are a topological order (a batch's operands lie in earlier batches in every batching
// mode), so the distinct dependencies are first put in the order of their consumer (a counting sort in
// LDS) and then walked once by one wave, 64 at a time: forward for the heads (every producer of a chunk's
// consumers was settled by an earlier chunk or is settled inside the chunk, which is passed over until
// nothing changes), backward for the tails.  That is as many dependent steps as the list has chunks
// instead of as many as the longest path has edges.  The
// plan has L + 1 slots, L = max head.  fuse == 1 places a batch as early as possible (slot =
// head), fuse == 2 as late as possible (slot = L - tail): batches off the critical path then
// gather in the slots next to their consumers instead of trailing the recurrence one small
// launch at a time.  Batches joined by fusable edges inside one slot then get a common chain
// label (the smallest batch id of the chain).
constexpr int SLOT_THREADS = 1024;
__global__ __launch_bounds__(SLOT_THREADS) void k_slots(Tables T, int fuse, const u32 *blist)
{
    __shared__ u32 s_slot[SLOT_MAX_NB];
    __shared__ u32 s_label[SLOT_MAX_NB];   // tail lengths first, chain labels afterwards
    __shared__ u32 s_edge[BLIST_MAX];
    __shared__ u32 s_changed;
    __shared__ u32 s_flag[3];
    __shared__ u32 s_wsum[SLOT_THREADS / 64];
    const u32 nb = T.hdr->n_batches;
    const u32 ne = T.hdr->n_bedges;
    const u32 tid = threadIdx.x;
    if (!fuse || nb > SLOT_MAX_NB || ne > BLIST_MAX) {   // one slot per step, no fusion
        for (u32 b = tid; b < nb; b += SLOT_THREADS) { T.slot_of[b] = T.batches[b].step; T.label_of[b] = b; }
        if (tid == 0) { T.hdr->n_slots = T.hdr->n_steps; T.hdr->slot_sweeps = 0; T.hdr->p0 = 1; }
        return;
    }
    // ---- the dependencies in the order of their consumer: count per consumer (in s_label), exclusive scan,
    // scatter (the order among one consumer's entries does not matter: only maxima and minima are taken)
    for (u32 b = tid; b < SLOT_MAX_NB; b += SLOT_THREADS) { s_slot[b] = 0; s_label[b] = 0; }
    __syncthreads();
    for (u32 e = tid; e < ne; e += SLOT_THREADS) atomicAdd(&s_label[(blist[e] - 1u) >> 13], 1u);
    __syncthreads();
    {
        constexpr u32 PER = SLOT_MAX_NB / SLOT_THREADS;   // consecutive counters per thread
        u32 c[PER], sum = 0;
        for (u32 i = 0; i < PER; ++i) { c[i] = s_label[tid * PER + i]; sum += c[i]; }
        u32 inc = sum;                                     // inclusive scan over the wave
        for (u32 o = 1; o < 64; o <<= 1) { const u32 v = (u32)__shfl_up((int)inc, o); if ((tid & 63u) >= o) inc += v; }
        if ((tid & 63u) == 63u) s_wsum[tid >> 6] = inc;
        __syncthreads();
        u32 before = inc - sum;
        for (u32 w = 0; w < (tid >> 6); ++w) before += s_wsum[w];
        for (u32 i = 0; i < PER; ++i) { s_label[tid * PER + i] = before; before += c[i]; }
    }
    __syncthreads();
    for (u32 e = tid; e < ne; e += SLOT_THREADS) {
        const u32 k = blist[e] - 1u;
        s_edge[atomicAdd(&s_label[k >> 13], 1u)] = k;
    }
    __syncthreads();
    for (u32 b = tid; b < SLOT_MAX_NB; b += SLOT_THREADS) s_label[b] = 0;
    __syncthreads();
    // ---- heads forward, tails backward: one wave, chunk by chunk (its LDS operations complete in order)
    u32 walked = 0;      // passes over chunks, for the statistics
    if (tid < 64) {
        const u32 n_chunks = (ne + 63u) / 64u;
        for (u32 ch = 0; ch < n_chunks; ++ch) {
            const u32 e = ch * 64u + tid;
            const bool valid = e < ne;
            const u32 k = valid ? s_edge[e] : 0u;
            const u32 c = k >> 13, y = (k >> 1) & 0xfffu, cost = k & 1u;
            for (u32 rep = 0; rep < 66u; ++rep) {          // (a chain inside a chunk has at most 64 links)
                bool changed = false;
                if (valid) {
                    const u32 want = lds_load(&s_slot[y]) + cost;
                    if (want > lds_load(&s_slot[c])) { atomicMax(&s_slot[c], want); changed = true; }
                }
                ++walked;
                if (__ballot(changed) == 0ull) break;
            }
        }
        for (u32 ch = n_chunks; ch-- > 0;) {
            const u32 e = ch * 64u + tid;
            const bool valid = e < ne;
            const u32 k = valid ? s_edge[e] : 0u;
            const u32 c = k >> 13, y = (k >> 1) & 0xfffu, cost = k & 1u;
            for (u32 rep = 0; rep < 66u; ++rep) {
                bool changed = false;
                if (valid) {
                    const u32 tw = lds_load(&s_label[c]) + cost;
                    if (tw > lds_load(&s_label[y])) { atomicMax(&s_label[y], tw); changed = true; }
                }
                ++walked;
                if (__ballot(changed) == 0ull) break;
            }
        }
    }
    __syncthreads();
    {   // number of slots; late placement; labels start as the batch's own id
        u32 mx = 0;
        for (u32 b = tid; b < nb; b += SLOT_THREADS) mx = s_slot[b] > mx ? s_slot[b] : mx;
        if (tid == 0) s_changed = 0;
        __syncthreads();
        atomicMax(&s_changed, mx);
        __syncthreads();
        const u32 L = s_changed;
        __syncthreads();
        for (u32 b = tid; b < nb; b += SLOT_THREADS) {
            if (fuse == 2) s_slot[b] = L - s_label[b];
            s_label[b] = b;
        }
        if (tid == 0) T.hdr->n_slots = L + 1;
        __syncthreads();
    }
    // One barrier per sweep: sweep k raises s_flag[k % 3] when it changes anything, everybody reads
    // it behind the sweep's barrier, and the flag of sweep k + 1 is cleared during sweep k (its last
    // readers were those of sweep k - 2, who have all passed the barrier of sweep k - 1).
    if (tid < 3) s_flag[tid] = 0;
    __syncthreads();
    u32 sweeps = 0;
    while (true) {
        const u32 f = sweeps % 3u;
        if (tid == 0) s_flag[(sweeps + 1u) % 3u] = 0;
        for (u32 e = tid; e < ne; e += SLOT_THREADS) {
            const u32 k = s_edge[e];
            if (k & 1u) continue;
            const u32 c = k >> 13, y = (k >> 1) & 0xfffu;
            if (s_slot[c] != s_slot[y]) continue;
            const u32 a = s_label[c], bb = s_label[y];
            if (a != bb) {
                const u32 m = a < bb ? a : bb;
                atomicMin(&s_label[c], m);
                atomicMin(&s_label[y], m);
                s_flag[f] = 1;
            }
        }
        __syncthreads();
        ++sweeps;
        if (!s_flag[f] || sweeps > 2 * nb + 2) break;
    }
    for (u32 b = tid; b < nb; b += SLOT_THREADS) { T.slot_of[b] = s_slot[b]; T.label_of[b] = s_label[b]; }
    if (tid == 0) T.hdr->slot_sweeps = walked + sweeps;
}

__global__ void k_launch_keys(Tables T, u64 *keys, u32 *vals, u32 n_pad)
{
    const u32 b = blockIdx.x * blockDim.x + threadIdx.x;
    const bool in = b < n_pad;
    if (in) vals[b] = b;
    // batches without forward work, counted for the statistics: summed over the wave first (every lane takes
    // part), one atomic per wave
    const bool live = in && b < T.hdr->n_batches;
    u32 cnt[4] = {0u, 0u, 0u, 0u};
    if (live) {
        const BatchRec &r = T.batches[b];
        if (r.vec4 & TF_VIEW) { cnt[0] = 1u; cnt[1] = r.B * r.d; }
        if (r.vec4 & TF_VIRT) { cnt[2] = 1u; cnt[3] = r.B * r.d; }
    }
    if (__ballot(cnt[0] | cnt[2]) != 0ull) {
        for (int q = 0; q < 4; ++q)
            for (int o = 32; o > 0; o >>= 1) cnt[q] += __shfl_xor(cnt[q], o);
        if ((threadIdx.x & 63u) == 0u) {
            if (cnt[0]) { atomicAdd(&T.hdr->view_batches, cnt[0]); atomicAdd(&T.hdr->view_floats, cnt[1]); }
            if (cnt[2]) { atomicAdd(&T.hdr->virt_batches, cnt[2]); atomicAdd(&T.hdr->virt_floats, cnt[3]); }
        }
    }
    if (!in) return;
    if (!live) { keys[b] = ~0ull; return; }
    // unfused plans are already in launch order (slot = step): equal keys keep that order
    keys[b] = T.hdr->p0 ? 0ull : (((u64)T.slot_of[b] << SLOT_BITS) | T.label_of[b]);
}

__device__ inline u32 rows_per_block(u32 d) { return d >= (u32)EW_TILE ? 1u : (u32)EW_TILE / d; }

// chains from the launch order: head flags, then one thread per chain head fills the record
__device__ inline u64 chain_key(const Tables &T, u32 b) { return ((u64)T.slot_of[b] << 32) | T.label_of[b]; }

__global__ void k_chain_flags(Tables T, const u32 *sval, u32 *flag, u32 n_pad)
{
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pad) return;
    const u32 nb = T.hdr->n_batches;
    if (i < nb) T.lorder[i] = sval[i];
    flag[i] = (i < nb && (i == 0 || chain_key(T, sval[i]) != chain_key(T, sval[i - 1]))) ? 1u : 0u;
}

// whether batch c reads a result of batch y through a fusable dependency (the set k_bedges filled)
__device__ inline bool bset_has(const u32 *bset, u32 c, u32 y)
{
    const u32 key = ((c << 13) | (y << 1)) + 1u;
    u32 h = (key * 2654435761u) & (BSET_SIZE - 1);
    for (u32 probe = 0; probe < BSET_SIZE; ++probe) {
        const u32 k = bset[h];
        if (k == key) return true;
        if (k == 0u) return false;
        h = (h + 1) & (BSET_SIZE - 1);
    }
    return false;
}

constexpr u32 LEVEL_MAX_MEMBERS = 32;   // chains with more members keep their step order and one tile group per member

__global__ void k_chain_recs(Tables T, int agenda, const u32 *bset, const u32 *flag, const u32 *flag_excl, CLay *clay_in,
                             u32 n_pad)
{
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pad) return;
    const u32 nb = T.hdr->n_batches;
    CLay L; L.tf = L.wf = L.ta = L.wa = L.tb = L.p0 = L.p1 = L.p2 = 0;
    if (i < nb) {
        const u32 c = flag_excl[i] + flag[i] - 1;
        T.chain_of_lpos[i] = c;
        T.chain_of_batch[T.lorder[i]] = c;   // (a chain's members may still be reordered below: same chain)
        if (i == nb - 1) T.hdr->n_chains = c + 1;
    }
    if (i < nb && flag[i]) {
        const u32 c = flag_excl[i];
        u32 k = 1;
        while (i + k < nb && !flag[i + k]) ++k;
        // Members of a chain run level by level, the tiles of one level without a barrier between
        // them.  In depth mode a member's level is its depth.  Agenda batches are steps of their
        // own, so there the levels come from the dependencies inside the chain (level = 1 + the
        // largest level of the members it reads), and the members are put in (level, batch) order.
        if (!agenda || T.hdr->p0) {
            for (u32 m = 0; m < k; ++m) T.blevel[T.lorder[i + m]] = T.batches[T.lorder[i + m]].step;
        } else if (k > LEVEL_MAX_MEMBERS) {
            for (u32 m = 0; m < k; ++m) T.blevel[T.lorder[i + m]] = m;
        } else {
            u32 ids[LEVEL_MAX_MEMBERS], lv[LEVEL_MAX_MEMBERS];
            for (u32 m = 0; m < k; ++m) {
                ids[m] = T.lorder[i + m];
                u32 l = 0;
                for (u32 mm = 0; mm < m; ++mm)
                    if (lv[mm] + 1 > l && bset_has(bset, ids[m], ids[mm])) l = lv[mm] + 1;
                lv[m] = l;
            }
            for (u32 m = 1; m < k; ++m) {   // stable insertion sort by level
                const u32 id = ids[m], l = lv[m];
                u32 j = m;
                while (j > 0 && lv[j - 1] > l) { ids[j] = ids[j - 1]; lv[j] = lv[j - 1]; --j; }
                ids[j] = id; lv[j] = l;
            }
            for (u32 m = 0; m < k; ++m) { T.lorder[i + m] = ids[m]; T.blevel[ids[m]] = lv[m]; }
        }
        const BatchRec r0 = T.batches[T.lorder[i]];
        ChainRec cr;
        cr.first = i; cr.k = k; cr.slot = T.slot_of[T.lorder[i]];
        cr.fused = (op_chainable(r0.op, r0.arity) || r0.op == OP_INPUT || r0.op == OP_LOOKUP) ? 1u : 0u;
        u32 dmax = r0.d, G = r0.B;
        for (u32 m = 1; m < k; ++m) {
            const BatchRec &rm = T.batches[T.lorder[i + m]];
            dmax = rm.d > dmax ? rm.d : dmax;
            G = gcd_u32(G, rm.B);
        }
        u32 kt = 0, ktf = 0, per_group = 0;   // tiles per block (all members / members with forward work); floats one group of every member takes
        for (u32 m = 0; m < k; ++m) {
            const BatchRec &rm = T.batches[T.lorder[i + m]];
            kt += rm.B / G;
            if (!(rm.vec4 & TF_NOFWD)) ktf += rm.B / G;
            per_group += (rm.B / G) * rm.d;
        }
        cr.G = G; cr.Rg = rows_per_block(dmax);
        if (cr.fused && k > 1) {
            // hand results from member to member through LDS when a block of groups fits (each
            // member's region is rounded up to 4 floats); fewer groups per block if that is what it takes
            const u32 fit = (CHAIN_LDS_FLOATS - 3u * k) / per_group;
            if (fit >= 1) { cr.fused = 2u; if (fit < cr.Rg) cr.Rg = fit; }
        }
        cr.nrb = cdiv(G, cr.Rg); cr.kt = cr.fused ? kt : 1u;
        cr.ktf = cr.fused ? ktf : 1u; cr.pad0 = cr.pad1 = cr.pad2 = 0;
        if (cr.fused) {
            L.ta = cr.nrb * kt; L.wa = cr.nrb;
            L.tf = cr.nrb * ktf; L.wf = ktf ? cr.nrb : 0u;     // a chain of views only has no forward work
        } else {
            switch (r0.op) {
            case OP_MATVEC: {
                const u32 gt = (r0.vec4 & TF_WIDE) ? (u32)GTW : (u32)GT;
                const u32 dt = dx_tile_edge(r0.vec4, r0.k);
                L.tf = cdiv(r0.B, gt) * cdiv(r0.d, gt); L.tb = cdiv(r0.B, dt) * cdiv(r0.k, dt);
                break;
            }
            case OP_PICK_NLS:
            case OP_SQNORM: L.tf = cdiv(r0.B, ROWS_PER_RED_TILE); break;
            default: L.tf = r0.B; break;   // wide sum: one workgroup per row
            }
            L.wf = L.tf;
            L.ta = L.wa = cr.nrb;          // pull tiles are row blocks of the batch
        }
        T.chains[c] = cr;
        clay_in[c] = L;
    }
}

__global__ void k_clay_zero(CLay *clay_in, u32 n_pad)
{
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_pad) return;
    CLay L; L.tf = L.wf = L.ta = L.wa = L.tb = L.p0 = L.p1 = L.p2 = 0;
    clay_in[i] = L;
}

// floats of a fused chain's LDS copy taken by one member: its rows of a block of groups, rounded up to 4
__device__ inline u32 chain_region(const ChainRec &cr, const BatchRec &r) { return (cr.Rg * (r.B / cr.G) * r.d + 3u) & ~3u; }

// every entry a plan can use (n_slots + 1 <= n + 2) starts out as "no batch here"
__global__ void k_slot_init(Tables T)
{
    const u32 s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s > T.hdr->n_slots) return;
    SlotRec r; r.wf = r.wa = r.tb = r.tf = r.ta = r.lmin = r.nlmax = r.dx_free = 0xffffffffu;
    r.lds_need = 0;
    r.lminf = r.nlmaxf = 0xffffffffu;
    r.plain = 0xffffffffu;
    T.slots[s] = r;
}

// per chain: first work item / tile of every launch slot and its run lengths, totals in the header
__global__ void k_slot_tables(Tables T, const CLay *clay_ex, const CLay *total)
{
    const u32 c = blockIdx.x * blockDim.x + threadIdx.x;
    const u32 nc = T.hdr->n_chains;
    if (c >= nc) return;
    const ChainRec cr = T.chains[c];
    const u32 s = cr.slot;
    const CLay L = clay_ex[c];
    SlotRec &S = T.slots[s];
    if (c == 0 || T.chains[c - 1].slot != s) { S.wf = L.wf; S.wa = L.wa; S.tb = L.tb; S.tf = L.tf; S.ta = L.ta; }
    const BatchRec &hb = T.batches[T.lorder[cr.first]];
    if (hb.op == OP_MATVEC && !(hb.vec4 & TF_G_ALIAS)) S.dx_free = 0;   // this slot's dX tiles need the slot's own pull first
    if (!cr.fused) atomicAnd(&S.plain, ~1u);     // a GEMM, reduction or wide-sum batch runs in this slot
    if (batch_xp(hb) && hb.aux1 > 1) atomicAnd(&S.plain, ~2u);   // a product that reads its operand rows in pieces
    if (cr.fused == 2u) {
        u32 need = 0;
        for (u32 m = 0; m < cr.k; ++m) need += chain_region(cr, T.batches[T.lorder[cr.first + m]]);
        atomicMax(&S.lds_need, need);
    }
    const u32 len = cr.fused ? cr.kt : 1u;
    atomicMin(&S.lmin, len);
    atomicMin(&S.nlmax, ~len);
    const u32 lenf = cr.fused ? cr.ktf : 1u;
    if (lenf) {   // (a chain of views has no forward work item)
        atomicMin(&S.lminf, lenf);
        atomicMin(&S.nlmaxf, ~lenf);
    }
    if (c == nc - 1) {
        const CLay t = *total;
        SlotRec &E = T.slots[s + 1];
        E.wf = t.wf; E.wa = t.wa; E.tb = t.tb; E.tf = t.tf; E.ta = t.ta;
        T.hdr->tiles_fwd = t.tf; T.hdr->tiles_pull = t.ta; T.hdr->tiles_dx = t.tb;
        T.hdr->works_fwd = t.wf; T.hdr->works_pull = t.wa;
    }
}

// launch slots that hold no batch (neither placement produces one today; the launch tables
// simply do not rely on it) inherit the offsets of the next slot that does, so that their launch
// range is empty
__global__ void k_slot_fill(Tables T)
{
    const u32 s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= T.hdr->n_slots) return;
    u32 t = s;
    while (T.slots[t].wf == 0xffffffffu) ++t;   // entry n_slots is always set
    if (t != s) {
        const SlotRec N = T.slots[t];
        SlotRec &S = T.slots[s];
        S.wf = N.wf; S.wa = N.wa; S.tb = N.tb; S.tf = N.tf; S.ta = N.ta;
    }
}

// ---- tile descriptors ------------------------------------------------------------------------------
constexpr u32 CONTIG_MAX_ROWS = 64;   // tiles with more rows skip the even-spacing test

// Where a tile of a fused chain sits: chain, member, block of groups [g0, g0 + ng).
struct ChainCtx { ChainRec cr; u32 m, g0, ng; };


// For up to four row-offset ranges [lo[j], hi[j]] (first element of the lowest / highest row read
// through slot j; offsets in the value arena, which the gradient arena mirrors): state 0 = no
// member of the chain produces these rows, 1 = all of them lie in this block's rows of one member
// (LDS index = offset + delta[j]), 2 = produced in the chain but not covered by one region.
__device__ inline void chain_lookup(const Tables &T, const ChainCtx &cc, u32 ns, const u32 *lo, const u32 *hi,
                                    u32 *state, u32 *delta)
{
    for (u32 j = 0; j < ns; ++j) { state[j] = 0; delta[j] = 0; }
    u32 lds = 0;
    for (u32 mm = 0; mm < cc.cr.k; ++mm) {
        const BatchRec &y = T.batches[T.lorder[cc.cr.first + mm]];
        const u32 mult = y.B / cc.cr.G;
        const u32 full_lo = y.val_off, full_hi = y.val_off + y.B * y.d;
        const u32 ch_lo = y.val_off + cc.g0 * mult * y.d, ch_hi = ch_lo + cc.ng * mult * y.d;
        if (mm != cc.m) {
            for (u32 j = 0; j < ns; ++j) {
                if (hi[j] < full_lo || lo[j] >= full_hi) continue;
                if (state[j] == 0 && cc.cr.fused == 2u && lo[j] >= ch_lo && hi[j] < ch_hi) { state[j] = 1; delta[j] = lds - ch_lo; }
                else state[j] = 2;
            }
        }
        lds += chain_region(cc.cr, y);
    }
}

// LDS index offset of the block's own rows of member cc.m (index = arena offset + result)
__device__ inline u32 chain_own_delta(const Tables &T, const ChainCtx &cc, const BatchRec &r)
{
    u32 lds = 0;
    for (u32 mm = 0; mm < cc.m; ++mm) lds += chain_region(cc.cr, T.batches[T.lorder[cc.cr.first + mm]]);
    return lds - (r.val_off + cc.g0 * (r.B / cc.cr.G) * r.d);
}

// descriptor of a forward or dX tile of batch r.  Component-wise tiles (row_block) cover the rows
// row0 + i * rstride, i < nrows; the other kinds derive their rows from the tile index t.
__device__ inline void fill_tile_desc(const Tables &T, const BatchRec &r, u32 t, bool dx, bool row_block, u32 row0,
                                      u32 nrows, u32 rstride, TileDesc &d, const ChainCtx *cc = nullptr)
{
    d.op = r.op; d.B = r.B; d.d = r.d; d.arity = r.arity;
    d.pos0 = r.pos0; d.val_off = r.val_off; d.dx_off = r.dx_off; d.k = r.k;
    d.aux0 = r.aux0; d.rstride = rstride;
    d.w = r.param >= 0 ? T.params[r.param].data : nullptr;
    d.b = r.bias >= 0 ? T.params[r.bias].data : nullptr;
    d.lds_out = 0;
    for (int j = 0; j < 4; ++j) d.lds_src[j] = 0;
    d.pad = 0;
    d.opnd = r.opnd; d.indim = r.indim; d.flags = r.vec4; d.t = t;
    d.contig = 0; d.row0 = row0; d.nrows = nrows; d.depth = r.step;
    for (int j = 0; j < 4; ++j) { d.base[j] = 0; d.sdim[j] = 0; d.sstride[j] = 0; }
    if (dx) {
        // dX tile: rows (t / ntn) * DXT ...; with TF_G_ALIAS the gradient rows are read where the
        // consumer left them, evenly spaced or through the per-row list
        if (r.vec4 & TF_G_ALIAS) {
            const u32 dt = dx_tile_edge(r.vec4, r.k);
            const u32 ntn = (r.k + dt - 1) / dt;
            const u32 r_lo = (t / ntn) * dt;
            u32 r_hi = r_lo + dt - 1;
            if (r_hi >= r.B) r_hi = r.B - 1;
            const u32 *gs = T.dx_gsrc + r.pos0;
            const u32 base = gs[r_lo];
            bool ok = true;
            u32 ss = 0;
            if (r_hi > r_lo) {
                ss = gs[r_lo + 1] - base;
                for (u32 i0 = 2; r_lo + i0 <= r_hi; i0 += 8) {      // eight reads in flight
                    u32 o[8];
#pragma unroll
                    for (u32 q = 0; q < 8; ++q) o[q] = gs[r_lo + (r_lo + i0 + q <= r_hi ? i0 + q : 0u)];
#pragma unroll
                    for (u32 q = 0; q < 8; ++q) ok = ok && (r_lo + i0 + q > r_hi || o[q] == base + (i0 + q) * ss);
                }
            }
            d.base[0] = base; d.sstride[0] = ss;
            if (ok) d.contig |= 1u;
        }
        return;
    }
    if (!row_block && r.arity == 0) return;
    if (!row_block) {
        u32 r_lo, r_hi;
        if (r.op == OP_MATVEC) {
            const u32 gt = (r.vec4 & TF_WIDE) ? (u32)GTW : (u32)GT;
            const u32 ntn = (r.d + gt - 1) / gt;
            r_lo = (t / ntn) * gt; r_hi = r_lo + gt - 1;
        } else if (r.op == OP_PICK_NLS || r.op == OP_SQNORM) {
            r_lo = t * ROWS_PER_RED_TILE; r_hi = r_lo + ROWS_PER_RED_TILE - 1;
        } else {
            r_lo = r_hi = t;   // wide sum
        }
        if (r_hi >= r.B) r_hi = r.B - 1;
        d.row0 = row0 = r_lo; d.nrows = nrows = r_hi - r_lo + 1; d.rstride = rstride = 1;
    }
    const bool xp = batch_xp(r);
    const u32 ns = xp ? (u32)r.aux1 : (r.arity < 4 ? r.arity : 4);   // a product reading in pieces: one operand slot per piece
    if (xp) d.arity = ns;
    u32 lo[4], hi[4];
    for (u32 j = 0; j < ns; ++j) {
        const u32 *op = T.opnd_off + r.opnd + j * r.B;
        const u32 base = op[row0];
        d.base[j] = base; d.sdim[j] = T.b_indim[r.indim + j];
        bool ok = nrows <= CONTIG_MAX_ROWS;
        u32 ss = 0;
        lo[j] = hi[j] = base;
        if (ok && nrows > 1) {
            ss = op[row0 + rstride] - base;
            for (u32 i0 = 1; i0 < nrows; i0 += 8) {      // eight reads in flight
                u32 o[8];
#pragma unroll
                for (u32 q = 0; q < 8; ++q) o[q] = op[row0 + (i0 + q < nrows ? i0 + q : 0u) * rstride];
#pragma unroll
                for (u32 q = 0; q < 8; ++q) {
                    if (i0 + q >= nrows) continue;
                    ok = ok && o[q] == base + (i0 + q) * ss;
                    lo[j] = o[q] < lo[j] ? o[q] : lo[j]; hi[j] = o[q] > hi[j] ? o[q] : hi[j];
                }
            }
        }
        d.sstride[j] = ss;
        if (ok) d.contig |= 1u << j;
    }
    if (row_block && (d.flags & TF_VEC4) && r.arity >= 1 && r.arity <= 4 && (d.contig & 0xfu) == (1u << r.arity) - 1u &&
        (r.op == OP_ADD || r.op == OP_CMULT || r.op == OP_TANH || r.op == OP_SIGMOID || r.op == OP_SLICE))
        d.flags |= TF_SIMPLE;
    if (!cc) return;
    // tile of a fused chain: which operands come from the chain's LDS copy, and whether any
    // operand produced earlier in the same launch still has to come from global memory
    if (cc->cr.fused != 2u || nrows > CONTIG_MAX_ROWS || r.arity > 4) { d.flags |= TF_GLOBAL_DEP; }
    if (cc->cr.fused != 2u) return;
    d.lds_out = chain_own_delta(T, *cc, r);
    d.flags |= TF_OUT_LDS;
    if (d.lds_out & 3u) d.flags &= ~(u32)(TF_VEC4 | TF_SIMPLE);   // (never with d % 4 == 0: regions and block rows start at multiples of 4)
    if (nrows > CONTIG_MAX_ROWS) return;
    u32 state[4], delta[4];
    chain_lookup(T, *cc, ns, lo, hi, state, delta);
    for (u32 j = 0; j < ns; ++j) {
        if (state[j] == 1 && (!(d.flags & TF_VEC4) || (delta[j] & 3u) == 0)) { d.flags |= TF_SRC_LDS << j; d.lds_src[j] = delta[j]; }
        else if (state[j] != 0) d.flags |= TF_GLOBAL_DEP;
    }
}

constexpr u32 PULL_MAX_ROWS = 16;

__device__ inline void fill_pull_base(const Tables &T, const BatchRec &r, u32 row0, u32 nrows, u32 rstride, PullDesc &d)
{
    d.lflags = 0; d.lds_out = 0;
    d.own0 = r.val_off + row0 * r.d; d.rowstep = rstride * r.d;
    d.dshift = (r.d & (r.d - 1u)) == 0u && r.d ? (u32)__ffs(r.d) - 1u : PULL_NO_SHIFT;
    d.pos0 = r.pos0; d.B = r.B; d.d = r.d; d.val_off = r.val_off;
    d.depth = r.step; d.row0 = row0; d.nrows = nrows; d.n_uni = PULL_GENERIC; d.rstride = rstride;
    for (int j = 0; j < 4; ++j) { UEdge z; z.kind = 0; z.goff = z.voff = z.gs = z.vs = 0; z.a0 = z.a1 = 0; z.dl = 0; d.e[j] = z; }
    d.grp_len = 1; d.vec4 = (r.vec4 & TF_VIEW) ? 2u : 0u;   // bit 1: the batch is a view (its values lie in its operands' rows)
    if (nrows > PULL_MAX_ROWS) return;
    const u32 u0 = T.order[r.pos0 + row0];
    const u32 q0 = T.succ_off[u0];
    const u32 cnt = T.succ_off[u0 + 1] - q0;
    if (cnt > 4) return;
    EdgeRec first[4];
    for (u32 j = 0; j < cnt; ++j) {
        first[j] = T.edges[q0 + j];
        if (first[j].kind == EK_NLS) return;     // the label is per-row data
        if (first[j].kind == EK_SQN && (r.vec4 & TF_VIEW)) return;   // needs the rows' own values, which a view keeps elsewhere
        UEdge ue; ue.kind = first[j].kind; ue.goff = first[j].goff; ue.voff = first[j].voff;
        ue.gs = ue.vs = 0; ue.a0 = first[j].a0; ue.a1 = first[j].a1; ue.dl = 0;
        d.e[j] = ue;
    }
    // The other rows must have the same edges, shifted by constant strides.  Every step is a read that
    // depends on the one before (row -> node -> its consumer list -> the edge records), so each step is
    // taken for all rows at once (rows past the tile's last repeat row 0: no read leaves the lists).
    if (nrows > 1) {
        u32 qs[PULL_MAX_ROWS];
        bool same = true;
#pragma unroll
        for (u32 i = 1; i < PULL_MAX_ROWS; ++i) {
            const u32 u = T.order[r.pos0 + row0 + (i < nrows ? i : 0u) * rstride];
            qs[i] = T.succ_off[u];
            same = same && T.succ_off[u + 1] - qs[i] == cnt;
        }
        if (!same) return;
        for (u32 j = 0; j < cnt; ++j) {
            EdgeRec er[PULL_MAX_ROWS];
#pragma unroll
            for (u32 i = 1; i < PULL_MAX_ROWS; ++i) er[i] = T.edges[qs[i] + j];
            const u32 gs = er[1].goff - first[j].goff, vs = er[1].voff - first[j].voff;
            bool ok = true;
#pragma unroll
            for (u32 i = 1; i < PULL_MAX_ROWS; ++i) {
                if (i >= nrows) continue;
                ok = ok && er[i].kind == first[j].kind && er[i].a0 == first[j].a0 && er[i].a1 == first[j].a1 &&
                     er[i].goff - first[j].goff == gs * i && er[i].voff - first[j].voff == vs * i;
            }
            if (!ok) return;
            d.e[j].gs = gs; d.e[j].vs = vs;
        }
    }
    d.n_uni = cnt;
    bool vec = (r.d & 3u) == 0;
    for (u32 j = 0; j < cnt; ++j) {
        const UEdge &ue = d.e[j];
        const bool scalar_g = ue.kind == EK_SQN;                 // these read one gradient scalar per row
        if (!scalar_g && ((ue.goff | ue.gs) & 3u)) vec = false;
        if ((ue.kind == EK_MUL || ue.kind == EK_DTANH || ue.kind == EK_DSIGM) && ((ue.voff | ue.vs) & 3u)) vec = false;
        if (ue.kind == EK_RANGE && (((u32)ue.a0 | (u32)ue.a1) & 3u)) vec = false;
    }
    u32 worst = 0;
    for (u32 j = 0; j < cnt; ++j) worst = d.e[j].kind > worst ? d.e[j].kind : worst;
    // (the short routine finds rows and columns by shifting: one row, or a power of two of columns)
    const bool shifts = nrows == 1u || d.dshift != PULL_NO_SHIFT;
    d.vec4 = (d.vec4 & 2u) | (vec ? 1u : 0u) | (vec && shifts && worst <= (u32)EK_DSIGM ? 4u : 0u);
}

__device__ inline void fill_pull_desc(const Tables &T, const BatchRec &r, u32 row0, u32 nrows, u32 rstride, PullDesc &d,
                                      const ChainCtx *cc = nullptr)
{
    fill_pull_base(T, r, row0, nrows, rstride, d);
    if (!cc) return;
    // tile of a fused chain: consumer gradients computed earlier in the same launch come from the
    // chain's LDS copy where the whole tile finds them in one member's region
    if (cc->cr.fused != 2u) { d.lflags = TF_GLOBAL_DEP; return; }
    d.lds_out = chain_own_delta(T, *cc, r);
    d.lflags = TF_OUT_LDS;
    if (d.lds_out & 3u) d.vec4 &= ~5u;
    if (d.n_uni == PULL_GENERIC) { d.lflags |= TF_GLOBAL_DEP; return; }
    u32 lo[4], hi[4], state[4], delta[4];
    for (u32 j = 0; j < d.n_uni; ++j) {
        const u32 a = d.e[j].goff, b = d.e[j].goff + (nrows - 1) * d.e[j].gs;
        lo[j] = a < b ? a : b; hi[j] = a < b ? b : a;
    }
    chain_lookup(T, *cc, d.n_uni, lo, hi, state, delta);
    for (u32 j = 0; j < d.n_uni; ++j) {
        if (state[j] == 1 && (!(d.vec4 & 1u) || (delta[j] & 3u) == 0)) { d.lflags |= TF_SRC_LDS << j; d.e[j].dl = delta[j]; }
        else if (state[j] != 0) d.lflags |= TF_GLOBAL_DEP;
    }
}

// Tiles with uniform edges carry them resolved (see PullDesc).
__device__ inline void resolve_pull_desc(PullDesc &d)
{
    if (d.n_uni == PULL_GENERIC) return;
    for (u32 j = 0; j < d.n_uni; ++j) {
        if (d.e[j].kind == EK_RANGE) d.e[j].goff -= (u32)d.e[j].a0;
        if (d.lflags & (TF_SRC_LDS << j)) d.e[j].goff += d.e[j].dl;
    }
}

// chain that owns global tile / work index x of list `which` (0 fwd tiles, 1 pull tiles, 2 dX tiles,
// 3 fwd works, 4 pull works): the largest c with offset(c) <= x
__device__ inline u32 clay_field(const CLay &L, int which)
{
    switch (which) { case 0: return L.tf; case 1: return L.ta; case 2: return L.tb; case 3: return L.wf; default: return L.wa; }
}
__device__ inline u32 chain_of_index(const CLay *clay_ex, u32 nc, int which, u32 x)
{
    u32 lo = 0, hi = nc;
    while (hi - lo > 1) {
        const u32 mid = (lo + hi) >> 1;
        if (clay_field(clay_ex[mid], which) <= x) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void k_tiles(Tables T, const CLay *clay_ex, const CLay *total, u32 cap_f, u32 cap_a, u32 cap_b)
{
    const u32 nc = T.hdr->n_chains;
    const u32 gtid = blockIdx.x * blockDim.x + threadIdx.x, gsz = gridDim.x * blockDim.x;
    // the five lists laid end to end, one entry per thread and pass: an entry is a chain of dependent reads
    // (chain, batch, operand rows), so a thread that took one entry of each list in turn would take five
    // times as long as the slowest entry
    u32 nts[5];
#pragma unroll
    for (int which = 0; which < 5; ++which) {
        u32 nt = clay_field(*total, which);
        const u32 cap = (which == 0 || which == 3) ? cap_f : ((which == 1 || which == 4) ? cap_a : cap_b);
        if (nt > cap) {   // cannot happen with the host's bound; never write past the lists
            if (gtid == 0) atomicOr(&T.hdr->err, (u32)ERR_OVERFLOW);
            nt = cap;
        }
        nts[which] = nt;
    }
    const u32 f1 = nts[0], f2 = f1 + nts[1], f3 = f2 + nts[2], f4 = f3 + nts[3], f5 = f4 + nts[4];
    for (u32 idx = gtid; idx < f5; idx += gsz) {
        const int which = (idx >= f1) + (idx >= f2) + (idx >= f3) + (idx >= f4);
        {
            const u32 x = idx - (which == 0 ? 0u : (which == 1 ? f1 : (which == 2 ? f2 : (which == 3 ? f3 : f4))));
            const u32 c = chain_of_index(clay_ex, nc, which, x);
            const ChainRec cr = T.chains[c];
            const u32 xx = x - clay_field(clay_ex[c], which);
            if (which >= 3) {   // work item = one block of a fused chain, or one tile
                WorkRec w;
                const bool fwd = which == 3;
                const u32 len = cr.fused ? (fwd ? cr.ktf : cr.kt) : 1u;
                w.first = (fwd ? clay_ex[c].tf : clay_ex[c].ta) + xx * len;
                w.len = len;
                (fwd ? T.works_f : T.works_a)[x] = w;
            } else if (which == 2 || (which == 0 && !cr.fused)) {
                const BatchRec r = T.batches[T.lorder[cr.first]];
                TileDesc d;
                fill_tile_desc(T, r, xx, which == 2, false, 0, 0, 1, d);
                (which == 0 ? T.tiles_f : T.tiles_b)[x] = d;
            } else {
                // tile `it` of block rb: member m, its q-th row of every group in the block
                // (pull tiles walk the members deepest first)
                // (forward: members that are views have no tiles and are stepped over)
                const u32 ktx = which == 0 ? cr.ktf : cr.kt;
                const u32 rb = xx / ktx;
                u32 it = xx % ktx;
                if (which == 1) it = ktx - 1 - it;
                u32 m = 0, mult = 1;
                if (cr.fused) {
                    for (;; ++m) {
                        const BatchRec &rq = T.batches[T.lorder[cr.first + m]];
                        if (which == 0 && (rq.vec4 & TF_NOFWD)) continue;
                        mult = rq.B / cr.G;
                        if (it < mult) break;
                        it -= mult;
                    }
                } else {
                    it = 0;
                }
                const BatchRec r = T.batches[T.lorder[cr.first + m]];
                const u32 g0 = rb * cr.Rg;
                const u32 ng = (g0 + cr.Rg <= cr.G) ? cr.Rg : cr.G - g0;
                const u32 row0 = g0 * mult + it;
                // tiles of the same level that follow this one in run order (this one included)
                u32 glen = 1;
                const u32 my_level = T.blevel[T.lorder[cr.first + m]];
                if (cr.fused) {
                    if (which == 0) {
                        glen = mult - it;
                        for (u32 mm = m + 1; mm < cr.k; ++mm) {
                            const BatchRec &rn = T.batches[T.lorder[cr.first + mm]];
                            if (T.blevel[T.lorder[cr.first + mm]] != my_level) break;
                            if (!(rn.vec4 & TF_NOFWD)) glen += rn.B / cr.G;
                        }
                    } else {
                        glen = it + 1;
                        for (u32 mm = m; mm-- > 0;) {
                            const BatchRec &rn = T.batches[T.lorder[cr.first + mm]];
                            if (T.blevel[T.lorder[cr.first + mm]] != my_level) break;
                            glen += rn.B / cr.G;
                        }
                    }
                }
                ChainCtx cc; cc.cr = cr; cc.m = m; cc.g0 = g0; cc.ng = ng;
                const ChainCtx *pcc = (cr.fused && ktx > 1) ? &cc : nullptr;
                if (which == 1) {
                    PullDesc d;
                    fill_pull_desc(T, r, row0, ng, mult, d, pcc);
                    resolve_pull_desc(d);
                    d.grp_len = glen;
                    T.tiles_a[x] = d;
                } else {
                    TileDesc d;
                    fill_tile_desc(T, r, xx, false, true, row0, ng, mult, d, pcc);
                    d.contig |= (glen > 0xffffu ? 0xffffu : glen) << 16;
                    T.tiles_f[x] = d;
                }
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
    EdgeRec r; r.kind = EK_PLAIN; r.goff = T.nat_off[v]; r.voff = 0; r.a0 = 0; r.a1 = 0;
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
    case OP_PICK_NLS: r.kind = EK_NLS; r.voff = T.val_off[v]; r.a0 = T.aux0[v]; r.a1 = (i32)T.out_dim[T.in_idx[e]]; break;
    case OP_SQNORM: r.kind = EK_SQN; break;
    default: break;
    }
    T.edges[q] = r;
    // a MATVEC node's own gradient row: with one plain consumer it is that consumer's row as it is
    const u32 u = T.in_idx[e];
    if (T.op[u] == OP_MATVEC) {
        const u32 pu = T.pos_of[u];
        T.dx_gsrc[pu] = r.goff;
        if (r.kind != EK_PLAIN || (r.goff & 3u)) atomicAnd(&T.batches[T.batch_of_pos[pu]].vec4, ~(u32)TF_G_ALIAS);
    }
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
    T.it_goff[i] = T.nat_off[v];
    u32 xoff = 0;
    if (T.op[v] == OP_MATVEC) {
        const BatchRec &r = T.batches[T.batch_of_pos[p]];
        xoff = T.val_off[T.in_idx[T.in_off[v]]];
        if (batch_xp(r)) {
            // the operand row in pieces: the row's offsets from the batch's operand list and the cuts between pieces
            xoff = XP_LIST;
            const u32 P = (u32)r.aux1, row = p - r.pos0;
            u32 o[XP_MAX], c[XP_MAX];
            u32 end = 0;
            for (u32 q = 0; q < XP_MAX; ++q) {
                o[q] = T.opnd_off[r.opnd + (q < P ? q : P - 1) * r.B + row];
                end += q < P ? T.b_indim[r.indim + q] : 0u;
                c[q] = q + 1 < P ? end : 0xffffffffu;
            }
            T.it_xrec[2 * (size_t)i] = make_uint4(o[0], o[1], o[2], o[3]);
            T.it_xrec[2 * (size_t)i + 1] = make_uint4(c[0], c[1], c[2], 0u);
        }
    }
    T.it_xoff[i] = xoff;
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

constexpr size_t SLOT_WINDOW = 2048;   // per-slot table entries read back together with the header

// First half of scheduling: allocates the scheduler tables for n nodes / E edges in the arena and
// queues every stage on the schedule stream, ending with the device-to-host copies of the header
// and the per-slot launch tables.  Does not wait.
int sched_enqueue(ob_ctx *ctx)
{
    Tables &T = ctx->T;
    hipStream_t s = ctx->sched_stream;
    const u32 n = T.n, E = T.E;
    const int manual = ctx->mode == 3;     // the caller's batches: no depth pass, no signatures to group by
    const int by_depth = ctx->mode == 1 || ctx->mode == 2;   // steps are depths (mode 1) or agenda iterations (mode 2)
    const int batched = ctx->mode != 0;
    const int agenda = ctx->mode == 2;
    ctx->n_launch_sched = 0;

    const size_t maxne = (size_t)(n > E ? n : E) + 1;
    u32 n_items = ctx->n_items_total;
    if ((size_t)n != ctx->op.size()) {   // a prefix of the graph: count its parameter uses
        n_items = 0;
        for (u32 v = 0; v < n; ++v)
            n_items += ctx->op[v] == OP_MATVEC ? 1u + (ctx->bias[v] >= 0 ? 1u : 0u) : (ctx->op[v] == OP_LOOKUP ? 1u : 0u);
    }
    const size_t n_slots = (size_t)ctx->params.size() * 4 + 4;

    // ---- allocation (all from the caller's arena) ----
    u32 ht_size = 1;
    while (ht_size < 2 * n) ht_size <<= 1;
    if (!by_depth) ht_size = 1;
    // upper bounds of the three tile lists from sums the host keeps while nodes are added
    // (a node contributes at most one component-wise / reduction tile; MATVEC nodes their GEMM tiles)
    const size_t cap_f = (size_t)n + (size_t)ctx->sum_mv_d32 + 16;
    const size_t cap_a = (size_t)n + 16;
    const size_t cap_b = (size_t)ctx->sum_mv_k32 + 16;
#define A(field, type, count)                                               \
    do {                                                                    \
        field = arena_array<type>(ctx, (count));                            \
        if (!field) return ctx_fail(ctx, -5, "arena too small for scheduler tables (%s)", #field); \
    } while (0)
    // Tables that must start at zero lie next to each other, and so do those that start as all ones:
    // two fills clear them all.
    u32 *g_dep, *inbox, *inbox_tail;
    const u32 n_parts = (n + DEPTH_PART - 1) / DEPTH_PART;
    u32 *bset, *blist;
    AgendaTables AG{};
    char *zero_lo = (char *)ctx->arena + ctx->top;
    A(T.hdr, SchedHeader, 1);
    A(T.outdeg, u32, n + 1); A(T.qcount, u32, 64); A(T.ext_indeg, u32, n + 1); A(T.ext_left, u32, n + 1);
    A(g_dep, u32, n + 1); A(inbox_tail, u32, n_parts + 1);
    A(T.pu_start, u32, n_slots); A(T.pu_end, u32, n_slots);
    A(T.ht_keys, u64, ht_size); A(bset, u32, BSET_SIZE);
    if (agenda) { A(AG.keys, u64, AG_TABLE); A(AG.sum, u64, AG_TABLE); A(AG.cnt, u32, AG_TABLE); }
    char *zero_hi = (char *)ctx->arena + ctx->top;
    A(inbox, u32, (size_t)n_parts * DEPTH_PART); A(T.ht_vals, u32, ht_size);
    if (agenda) A(AG.first, u32, AG_TABLE);
    char *ones_hi = (char *)ctx->arena + ctx->top;
    A(T.sig, u64, n); A(T.step, u32, n); A(T.indeg, u32, n);
    A(T.succ_off, u32, n + 1); A(T.succ_edge, u32, E + 1); A(T.edge_cons, u32, E + 1);
    A(T.queue, u32, n);
    A(T.ht_slot, u32, n);
    T.ht_mask = ht_size - 1;
    A(T.order, u32, n); A(T.pos_of, u32, n); A(T.batch_of_pos, u32, n); A(T.s_aux0, u32, n);
    A(T.s_in_off, u32, n + 1);
    A(T.batch_off, u32, n + 1); A(T.batches, BatchRec, n); A(T.lay, Lay, n); A(T.b_indim, u32, E + (size_t)XP_MAX * n + 1);
    A(T.val_off, u32, n); A(T.nat_off, u32, n); A(T.dx_off, u32, n); A(T.opnd_off, u32, E + (size_t)XP_MAX * n + 1); A(T.dx_gsrc, u32, n);
    A(T.slot_of, u32, n); A(T.label_of, u32, n); A(T.blevel, u32, n);
    A(T.chain_of_batch, u32, n);
    A(T.lorder, u32, n); A(T.chains, ChainRec, n); A(T.clay, CLay, n); A(T.chain_of_lpos, u32, n);
    // a plan has at most one slot per node; twice that leaves room for plans that insert slots
    const size_t slot_cap = 2 * (size_t)n + 4;
    A(T.slots, SlotRec, slot_cap);
    A(T.works_f, WorkRec, cap_f); A(T.works_a, WorkRec, cap_a);
    A(T.tiles_f, TileDesc, cap_f); A(T.tiles_a, PullDesc, cap_a); A(T.tiles_b, TileDesc, cap_b);
    A(T.root_pos, u32, 64);
    A(T.edges, EdgeRec, E + 1);
    A(T.it_key, u64, n_items + 1); A(T.it_pos, u32, n_items + 1); A(T.it_goff, u32, n_items + 1);
    A(T.it_xoff, u32, n_items + 1);
    T.it_xrec = nullptr;
    if (ctx->concat_views && ctx->n_concat > 0) A(T.it_xrec, uint4, 2 * ((size_t)n_items + 1));
    u32 *succ_node;
    A(succ_node, u32, E + 1);
    A(ctx->key_a, u64, maxne); A(ctx->key_b, u64, maxne); A(ctx->val_a, u32, maxne); A(ctx->val_b, u32, maxne);
    A(ctx->tmp_u32_a, u32, n + 1); A(ctx->tmp_u32_b, u32, n + 1);
    u32 *tmp_d;
    A(tmp_d, u32, n + 1);
    Tri *tri_in, *tri_ex;
    A(tri_in, Tri, n); A(tri_ex, Tri, n);
    A(ctx->lay_in, Lay, n); A(ctx->lay_total, Lay, 1);
    CLay *clay_in, *clay_total;
    A(clay_in, CLay, n); A(clay_total, CLay, 1);
    A(blist, u32, BLIST_MAX);
    if (agenda) {
        A(AG.op, u32, AG_TABLE); A(AG.rank_of, u32, AG_TABLE); A(AG.seg_off, u32, AG_MAX_CLASSES + 1);
        A(AG.n_classes, u32, 64);
        AG.cls = ctx->tmp_u32_a; AG.pending = ctx->tmp_u32_b; AG.seg = T.queue;
    }
    {
        size_t sb = prim_sort_scratch_bytes(maxne);
        size_t sc = prim_scan_scratch_bytes(maxne, sizeof(Lay));
        ctx->scratch = arena_alloc(ctx, sb > sc ? sb : sc);
        if (!ctx->scratch) return ctx_fail(ctx, -5, "arena too small for scheduler scratch");
    }
#undef A

    // ---- stage 1 ----
    HIP_TRY(ctx, hipMemsetAsync(zero_lo, 0, (size_t)(zero_hi - zero_lo), s));
    HIP_TRY(ctx, hipMemsetAsync(zero_hi, 0xff, (size_t)(ones_hi - zero_hi), s));
    const bool part_depth = by_depth && n_parts <= DEPTH_MAX_PARTS && ctx->max_arity < 60000 && !ctx->force_frontier;
    ctx->depth_partitioned = part_depth;
    K(k_node_init, n, T, manual ? 2 : by_depth);
    if (E > 0) K(k_edge_init, E, T, ctx->key_a, ctx->val_a);
    HIP_TRY(ctx, prim_scan_u32(T.outdeg, T.succ_off, (size_t)n + 1, nullptr, ctx->scratch, s));
    // a scan of a short array is one launch, up to 256 blocks of 1024 elements two, beyond that three
    const int scan_launches = (size_t)n + 1 <= 4096 ? 1 : ((size_t)n + 1 <= 256 * 1024 ? 2 : 3);
    ctx->n_launch_sched += scan_launches;
    if (E > 0) {
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, E, 0,
                                     bit_width_u32(n - 1), ctx->scratch, s, &ctx->n_launch_sched));
        K(k_succ_finish, E, T, ctx->val_a, succ_node);
    }

    // ---- stage 2 / 3 ----
    if (by_depth) {
        if (part_depth)
            hipLaunchKernelGGL(k_depth_partitioned, dim3(n_parts), dim3(DEPTH_THREADS), 0, s, T, succ_node, g_dep, inbox,
                               inbox_tail, ctx->depth_spin_limit);
        else
            hipLaunchKernelGGL(k_depth_frontier, dim3(1), dim3(FRONTIER_THREADS), 0, s, T, succ_node);
        ++ctx->n_launch_sched;
        if (agenda) {   // steps become agenda iterations; T.step holds the depths until k_agenda rewrites it
            K(k_class_insert, n, T, AG);
            hipLaunchKernelGGL(k_class_rank, dim3(1), dim3(1024), 0, s, T, AG);
            K(k_class_of, n, T, AG);
            hipLaunchKernelGGL(k_agenda, dim3(1), dim3(AGENDA_THREADS), 0, s, T, AG, succ_node);
            ctx->n_launch_sched += 2;
        }
        K(k_rep_insert, n, T);
    }
    K(k_sort_keys, n, T, ctx->key_a, ctx->val_a, manual ? 2 : by_depth);
    if (manual) {
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n, 32, bit_width_u32(ctx->manual_max | 1u),
                                     ctx->scratch, s, &ctx->n_launch_sched));
    } else if (by_depth) {
        const int lb = bit_width_u32(n - 1);
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n, 0, lb, ctx->scratch, s,
                                     &ctx->n_launch_sched));
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n, 32, lb, ctx->scratch, s,
                                     &ctx->n_launch_sched));
    }

    // ---- stage 4 ----
    u32 *head_flag = ctx->tmp_u32_a, *s_items = tmp_d;
    K(k_heads, n, T, ctx->key_a, ctx->val_a, head_flag, tri_in);
    HIP_TRY(ctx, prim_scan_tri(tri_in, tri_ex, n, nullptr, ctx->scratch, s));
    ctx->n_launch_sched += scan_launches;
    K(k_batch_off, n, T, head_flag, tri_ex, s_items, manual);
    const int virt = ctx->concat_views && ctx->n_concat > 0;   // CONCAT batches that only products read stay uncopied
    K(k_batch_layout, n, T, ctx->lay_in, virt);
    HIP_TRY(ctx, prim_scan_lay(ctx->lay_in, T.lay, n, ctx->lay_total, ctx->scratch, s));
    ctx->n_launch_sched += scan_launches;
    K(k_batch_finish, n, T, T.lay, ctx->lay_total);
    K(k_node_offsets, n, T);
    K(k_view_offsets, n, T);
    K(k_member_check, n, T);
    if (E > 0) K(k_opnd, E, T);
    if (E > 0) K(k_edges, E, T);

    // ---- launch planning: slots, chains, tile descriptors ----
    const int fuse = batched && ctx->fuse;
    if (fuse && E > 0) K(k_bedges, E, T, bset, blist);
    hipLaunchKernelGGL(k_slots, dim3(1), dim3(SLOT_THREADS), 0, s, T, (fuse && E > 0) ? ctx->fuse : 0, blist);
    ++ctx->n_launch_sched;
    K(k_launch_keys, n, T, ctx->key_a, ctx->val_a, n);
    if (fuse && E > 0) {
        const size_t n_sort = n < SLOT_MAX_NB + 1 ? n : SLOT_MAX_NB + 1;
        // entries from n_batches on carry the largest key and stay where they are
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n_sort, 0, 2 * SLOT_BITS,
                                     ctx->scratch, s, &ctx->n_launch_sched, &T.hdr->n_batches));
    }
    u32 *cflag = ctx->tmp_u32_a, *cflag_excl = ctx->tmp_u32_b;
    K(k_chain_flags, n, T, ctx->val_a, cflag, n);
    HIP_TRY(ctx, prim_scan_u32(cflag, cflag_excl, n, nullptr, ctx->scratch, s));
    K(k_clay_zero, n, clay_in, n);
    K(k_chain_recs, n, T, agenda || manual, bset, cflag, cflag_excl, clay_in, n);
    HIP_TRY(ctx, prim_scan_clay(clay_in, T.clay, n, clay_total, ctx->scratch, s));
    ctx->n_launch_sched += 2 * scan_launches;
    K(k_slot_init, (size_t)n + 2, T);
    K(k_slot_tables, n, T, T.clay, clay_total);
    if (fuse) K(k_slot_fill, (size_t)n + 2, T);
    hipLaunchKernelGGL(k_tiles, dim3(1024), dim3(TPB), 0, s, T, T.clay, clay_total, (u32)cap_f, (u32)cap_a,
                       (u32)cap_b);
    ++ctx->n_launch_sched;

    // ---- parameter-use items ----
    if (n_items > 0) {
        K(k_item_emit, n, T, s_items, ctx->key_a, ctx->val_a);
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n_items, 0,
                                     bit_width_u32((u32)ctx->max_param_rows), ctx->scratch, s,
                                     &ctx->n_launch_sched));
        HIP_TRY(ctx, prim_sort_pairs_swap(ctx->key_a, ctx->val_a, ctx->key_b, ctx->val_b, n_items, 32,
                                     bit_width_u32((u32)n_slots), ctx->scratch, s, &ctx->n_launch_sched));
        K(k_item_finish, n_items, T, ctx->key_a, ctx->val_a, n_items);
    }
    HIP_TRY(ctx, hipGetLastError());

    // ---- queue the read-back of the header and of a first window of the per-slot tables ----
    // pinned layout: [header 256 B][first hdr_window entries of the slot table]
    ctx->hdr_window = (u32)(slot_cap < SLOT_WINDOW ? slot_cap : SLOT_WINDOW);
    const size_t need = 256 + (size_t)ctx->hdr_window * sizeof(SlotRec);
    if (need > ctx->hdr_pinned_bytes) {
        if (ctx->hdr_pinned) HIP_TRY(ctx, hipHostFree(ctx->hdr_pinned));
        ctx->hdr_pinned = nullptr;
        ctx->hdr_pinned_bytes = need + 4096;
        HIP_TRY(ctx, hipHostMalloc(&ctx->hdr_pinned, ctx->hdr_pinned_bytes, hipHostMallocDefault));
    }
    char *hp = (char *)ctx->hdr_pinned;
    HIP_TRY(ctx, hipMemcpyAsync(hp, T.hdr, sizeof(SchedHeader), hipMemcpyDeviceToHost, s));
    HIP_TRY(ctx, hipMemcpyAsync(hp + 256, T.slots, (size_t)ctx->hdr_window * sizeof(SlotRec), hipMemcpyDeviceToHost, s));
    ctx->n_items_sched = n_items;
    return 0;
}

// Second half of scheduling: waits for the queued work, checks the error flags, takes the
// per-slot launch tables and carves the value and gradient arenas.
int sched_finish(ob_ctx *ctx)
{
    Tables &T = ctx->T;
    hipStream_t s = ctx->sched_stream;
    // wait for this context's own scheduling work only (its event was recorded behind the header
    // copy): other contexts may already have queued theirs on the same stream
    HIP_TRY(ctx, hipEventSynchronize(ctx->ev[9]));
    const char *hp = (const char *)ctx->hdr_pinned;
    ctx->hdr = *(const SchedHeader *)hp;
    if ((ctx->hdr.err & ERR_CYCLE) && ctx->depth_partitioned) {
        // A range of the partitioned depth pass ran into the bound on its wait for another range.
        // Node ids are a topological order (checked when nodes are added), so the graph has no
        // cycle: schedule once more with the single-workgroup pass, which waits for nothing.
        ++ctx->n_depth_retries;
        ctx->force_frontier = true;
        ctx->top = ctx->graph_top;
        int rc = sched_enqueue(ctx);
        ctx->force_frontier = false;
        if (rc) return rc;
        HIP_TRY(ctx, hipEventRecord(ctx->ev[9], s));
        HIP_TRY(ctx, hipEventSynchronize(ctx->ev[9]));
        hp = (const char *)ctx->hdr_pinned;
        ctx->hdr = *(const SchedHeader *)hp;
    }
    ctx->hdr.n_items = ctx->n_items_sched;
    if (ctx->hdr.err & ERR_CYCLE)
        return ctx_fail(ctx, -6, "%s resolved %u of %u nodes: the graph on the device is cyclic or damaged",
                        ctx->mode == 2 ? "the single-workgroup depth pass / the agenda" : "the single-workgroup depth pass",
                        ctx->hdr.frontier_done, T.n);
    if (ctx->hdr.err & ERR_COLLISION) return ctx_fail(ctx, -6, "signature hash collision detected");
    if (ctx->hdr.err & ERR_TABLE_FULL) return ctx_fail(ctx, -6, "signature table full");
    if (ctx->hdr.err & ERR_OVERFLOW) return ctx_fail(ctx, -5, "value arena exceeds 2^32 elements");
    if (ctx->hdr.err & ERR_CLASSES) return ctx_fail(ctx, -6, "more than 1024 distinct signatures (or a node with more than 4 million operands): agenda-based batching cannot handle the graph");
    const size_t words = (size_t)ctx->hdr.n_slots + 1;
    if (words <= ctx->hdr_window) {
        const SlotRec *sr = (const SlotRec *)(hp + 256);
        ctx->slots.assign(sr, sr + words);
    } else {   // more launch slots than the window (unbatched mode): a plain copy
        ctx->slots.resize(words);
        HIP_TRY(ctx, hipMemcpyAsync(ctx->slots.data(), T.slots, words * sizeof(SlotRec), hipMemcpyDeviceToHost, s));
        HIP_TRY(ctx, hipStreamSynchronize(s));
    }

    // ---- value and gradient arenas ----
    T.V = arena_array<float>(ctx, ctx->hdr.val_floats + VAL_ALIGN);
    T.G = arena_array<float>(ctx, ctx->hdr.grad_floats + VAL_ALIGN);
    if (!T.V || !T.G)
        return ctx_fail(ctx, -5, "arena too small: values need %llu floats, gradients %llu",
                        (unsigned long long)ctx->hdr.val_floats, (unsigned long long)ctx->hdr.grad_floats);
    return 0;
}
