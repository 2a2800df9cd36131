// Internal declarations shared by the library's translation units (not part of the ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

typedef uint32_t u32;
typedef uint64_t u64;
typedef int32_t i32;
typedef uint8_t u8;

// ---- graph data format -------------------------------------------------------------------
enum : u32 {
    OP_INPUT = 0, OP_LOOKUP, OP_MATVEC, OP_ADD, OP_CMULT, OP_TANH, OP_SIGMOID,
    OP_CONCAT, OP_SLICE, OP_PICK_NLS, OP_SQNORM, OP_COUNT
};

// ---- execution geometry --------------------------------------------------------------------
constexpr int WG = 256;               // threads per workgroup of every tile kernel (4 wave64)
constexpr int EW_TILE = 1024;         // elements of one elementwise / pull tile
constexpr int GT = 32;                // forward / dW GEMM tile edge (one 32x32 MFMA accumulator block)
constexpr int PWTILE = 64;            // dW tile edge of the deferred weight-gradient kernel
constexpr int PB_SPLIT = 16;           // workgroups that share the use list of one 256-row bias-gradient tile
constexpr int PW_SPLIT_MAX = 16;       // most workgroups that share the use list of one dW tile (matrices of many tiles take 4 or 8)
constexpr int GTW = 64;               // forward GEMM tile edge of batches with at least WIDE_MIN_ROWS rows
constexpr u32 WIDE_MIN_ROWS = 256;
constexpr int DXT = 16;               // dX GEMM tile edge (16x16 blocks: its output is small, more tiles fill more CUs)
constexpr int DXTW = 32;              // dX tile edge of batches with at least WIDE_MIN_ROWS rows (when the matrix has 32+ columns)
// 8u = TF_WIDE of the batch flags
__host__ __device__ inline u32 dx_tile_edge(u32 batch_flags, u32 k) { return ((batch_flags & 8u) && k >= (u32)DXTW) ? (u32)DXTW : (u32)DXT; }
constexpr int ROWS_PER_RED_TILE = 4;  // rows of one row-reduction tile (one wave per row)
constexpr int WIDE_ADD_ARITY = 9;     // ADD with at least this many operands reduces per row
constexpr u32 VAL_ALIGN = 64;         // batch blocks start at multiples of 64 floats (256 B)
constexpr u32 RUN_STAGE_DESCS = 32;       // descriptors a step kernel stages at a time
constexpr u32 CHAIN_LDS_FLOATS = 16384;   // LDS a fused chain may use to hand results from one member to the next (64 KB)

// Descriptor flag bits of a tile inside a fused chain (TileDesc::flags, PullDesc::lflags).
enum : u32 {
    TF_VEC4 = 1u,            // float4 path allowed
    TF_ALIGNED = 2u,         // operand rows 16-byte aligned
    TF_G_ALIAS = 4u,         // MATVEC batch: the gradient of every row is a plain copy of one consumer row
    TF_WIDE = 8u,            // MATVEC batch with many rows: 64x64 forward tiles, one 32x32 block per wave, no split contraction
    TF_SRC_LDS = 16u,        // << j: operand slot / consumer edge j is read from the chain's LDS copy
    TF_OUT_LDS = 256u,       // the tile also writes its result to the chain's LDS copy
    TF_GLOBAL_DEP = 512u,    // reads a result of an earlier member of the same chain from global memory
    TF_SIMPLE = 1024u,       // float4 tile of ADD (<= 4 operands) / CMULT / TANH / SIGMOID / SLICE whose operand rows are all evenly spaced
    TF_VIEW = 2048u,         // batch flag: a SLICE batch; its rows are not copied, every reader is pointed at the range of the
                             // operand row instead (Section 3.3: inputs that already lie in place are used as they are)
    TF_VIRT = 4096u,         // batch flag: a CONCAT batch that only matrix products read; its rows are not written by the forward
                             // pass, the products read the pieces where their producers left them (TF_XP).  The rows are filled
                             // in when a value is read from outside the forward pass.
    TF_XP = 8192u            // batch flag: a MATVEC batch whose operand is read piece by piece (BatchRec::aux1 pieces of
                             // the dimensions b_indim[indim ..]); piece q of row r lies at opnd_off[opnd + q * B + r] + k for the
                             // contraction indices k of the piece (the piece's first index is already subtracted)
};
constexpr u32 TF_NOFWD = TF_VIEW | TF_VIRT;   // batches without forward work
constexpr u32 XP_MAX = 4;                     // most pieces of an operand that is read through a CONCAT
constexpr u32 XP_LIST = 0xffffffffu;          // it_xoff entry of a use whose operand row is in pieces (see Tables::it_xrec)

// Kinds of consumer-edge records read by the backward pull (one per graph edge).
enum : u32 {
    EK_PLAIN = 0,   // += G[goff + c]                       (ADD, CONCAT, MATVEC dX block)
    EK_RANGE,       // += G[goff + c - lo] if lo <= c < hi  (SLICE)
    EK_MUL,         // += G[goff + c] * V[voff + c]         (CMULT, voff = the other operand)
    EK_DTANH,       // += G[goff + c] * (1 - V[voff + c]^2)
    EK_DSIGM,       // += G[goff + c] * V[voff + c] * (1 - V[voff + c])
    EK_NLS,         // += G[goff] * (exp(x_c - lse) - [c == label]), lse = V[voff] + x_label; a0 = label, a1 = dimension of x
    EK_SQN          // += 2 G[goff] x_c
};

struct EdgeRec {   // 20 bytes, one per graph edge, ordered by (producer, consumer, slot)
    u32 kind, goff, voff;
    i32 a0, a1;
};

struct BatchRec {  // one per batch, 64 bytes
    u32 pos0;      // first position in schedule order
    u32 B;         // number of nodes (rows)
    u32 op;
    u32 d;         // out_dim
    u32 arity;
    i32 param, bias;
    i32 aux0, aux1;      // SLICE lo / hi (the only aux fields that are part of a signature); MATVEC: aux0 = the CONCAT batch
                         // whose pieces the batch's operand rows follow (-1: none), aux1 = number of pieces (0: read whole)
    u32 step;
    u32 val_off;         // element offset of row 0 in the value arena (same in the grad arena)
    u32 dx_off;          // MATVEC: element offset of the dX block in the grad arena
    u32 opnd;            // base into opnd_off[], slot-major: opnd_off[opnd + j*B + r]
    u32 k;               // dimension of operand 0 (MATVEC: columns of W)
    u32 indim;           // base into b_indim[] (operand dimensions, `arity` entries)
    u32 vec4;            // TF_VEC4 | TF_ALIGNED | TF_G_ALIAS
};

// marks[0]: a dense gradient kernel (dW / db) has added to this parameter since its gradient was last
// cleared; marks[1]: number of rows in `touched`.  touched / row_flag: the rows of the parameter that
// LOOKUP gradients have been added to since then (each once; row_flag[r] = 1 for listed rows).  With
// these the update and the clearing of an embedding table walk the touched rows only.
struct ParamDesc {
    float *data;
    float *grad;
    u32 *marks;
    u32 *touched;
    u32 *row_flag;
    i32 rows, cols;
};

// One forward (or dX) tile: everything the tile routine needs in one 160-byte record, so that a
// workgroup starts its data loads after a single descriptor load.  For up to four operand slots
// the record says whether the operand rows of THIS tile are consecutive in the value arena
// (then the i-th row of the tile reads slot j at base[j] + i * sstride[j] and the row-offset list
// is not read at all: the inputs are used as they are, without an index hop).
struct TileDesc {
    u32 op, B, d, arity;
    u32 pos0, val_off, dx_off, k;
    i32 aux0;
    u32 rstride;                     // component-wise tiles cover rows row0 + i * rstride, i < nrows
    const float *w;                  // MATVEC: matrix data; LOOKUP: table data (device pointers, so that
    const float *b;                  // no parameter record has to be fetched first); b: bias data or null
    u32 opnd, indim, flags, t;       // flags: bit 0 float4 path allowed, bit 1 operand rows 16-byte aligned
    u32 contig, row0;                // contig bits 0..3: operand rows of slot j are evenly spaced over this tile;
                                     // bits 16..31: tiles of the same depth that follow in the run, this one included
    u32 base[4];                     // operand row offset of slot j for the tile's first row
    u32 sdim[4];                     // dimension of operand slot j
    u32 nrows, depth;
    u32 sstride[4];                  // operand row spacing of slot j (elements per tile row step)
    u32 lds_out, lds_src[4];         // LDS index = arena offset + lds_out (own result) / + lds_src[j] (operand slot j),
    u32 pad;                         // in u32 wrap-around arithmetic; valid with TF_OUT_LDS / TF_SRC_LDS << j
};
static_assert(sizeof(TileDesc) == 160, "TileDesc must be 160 bytes");

// A consumer edge that is the same for every row of a pull tile up to constant row strides (32 bytes, two
// aligned 16-byte reads).  dl: with TF_SRC_LDS << j in the tile's lflags, the consumer's gradient is read
// from the fused run's LDS copy at index (gradient-arena offset + dl) in u32 wrap-around arithmetic.
struct UEdge { u32 kind, goff, voff, gs, vs; i32 a0, a1; u32 dl; };

// One backward pull tile.  n_uni <= 4: every row of the tile has exactly n_uni consumer edges and
// edge j of row r is e[j] shifted by (r - row0) * (gs, vs); n_uni == PULL_GENERIC: rows differ,
// walk the consumer CSR per element.  The record is twelve aligned 16-byte words.
constexpr u32 PULL_GENERIC = 0xffffffffu;
constexpr u32 PULL_NO_SHIFT = 0xffffffffu;
struct PullDesc {
    u32 pos0, B, d, val_off;
    u32 depth, row0, n_uni, nrows;   // rows row0 + i * rstride, i < nrows, of the batch, all columns
    UEdge e[4];                      // edge j of the i-th row: e[j] shifted by i * (gs, vs)
    u32 rstride, grp_len;            // grp_len: tiles of the same depth that follow in the run, this one included
    u32 vec4, lflags;                // vec4 bit 0: d % 4 == 0 and every offset / stride / range of e[] is a multiple of 4;
                                     // bit 1: the batch is a view; bit 2: bit 0 and no edge kind beyond EK_DSIGM (the short routine applies)
    u32 lds_out, dshift;             // LDS index of the own rows = gradient-arena offset + lds_out; dshift: log2(d), or PULL_NO_SHIFT
    u32 own0, rowstep;               // val_off + row0 * d and rstride * d: the tile's i-th row starts at own0 + i * rowstep
};
// Uniform edges (n_uni != PULL_GENERIC) are stored resolved: goff already has the slice's lower bound
// subtracted (EK_RANGE) and, for a consumer read from the run's LDS copy, dl added, so the index of column c
// of the tile's i-th row is goff + i * gs + c in either memory.
static_assert(sizeof(PullDesc) == 192, "PullDesc must be 192 bytes");

// A launch chain: batches that run in the same launch slot.  A fused chain holds component-wise
// batches whose rows fall into G groups (member b has B_b / G consecutive rows per group) such
// that every in-chain operand of a row lies in the row's own group.  One workgroup then owns a
// block of groups and runs the members one after the other with workgroup barriers only.
// Every other batch is a chain of its own.
struct ChainRec {
    u32 first, k;          // members are lorder[first .. first + k)
    u32 slot, fused;       // fused: component-wise members tiled by group blocks (2: with results handed on through LDS)
    u32 G, Rg, nrb, kt;    // groups, groups per block, number of blocks, tiles per block (sum of rows per group)
    u32 ktf, pad0, pad1, pad2;   // forward tiles per block: kt without the members that are views (they have no forward work)
};
struct CLay {              // scan element of the per-chain launch layout
    u32 tf, wf, ta, wa, tb, p0, p1, p2;   // forward tiles/work items, pull tiles/work items, dX tiles
    __host__ __device__ CLay operator+(const CLay &o) const {
        CLay r; r.tf = tf + o.tf; r.wf = wf + o.wf; r.ta = ta + o.ta; r.wa = wa + o.wa; r.tb = tb + o.tb;
        r.p0 = r.p1 = r.p2 = 0; return r;
    }
};
struct WorkRec { u32 first, len; };   // a workgroup runs tiles [first, first + len) in order

// Per launch slot (entry n_slots closes the ranges): first forward work item, pull work item,
// dX tile, forward tile and pull tile of the slot, and the smallest / complement of the largest
// run length (tiles per work item) over the slot's chains.  When the two lengths agree, work
// item w of the slot runs tiles tf + (w - wf) * len onwards and its WorkRec need not be read.
// dx_free != 0: no dX tile of the slot reads a gradient that the slot's own pull computes (every
// MATVEC batch in it has TF_G_ALIAS), so the slot's pull and dX work can share one launch.
// lds_need: floats of LDS the slot's fused chains use to hand results on (0: none); the step
// kernels are launched with that much dynamic LDS (and at least their GEMM reduction space), so
// slots without such chains keep more workgroups resident per CU.
// plain bit 0: every forward work item of the slot is component-wise (no GEMM, reduction or wide-sum
// tile), so the slot can run the lean instantiation of the forward kernel.  Bit 1: no product of the slot
// reads its operand rows in pieces (otherwise the slot runs the instantiation that can).
// lminf / nlmaxf: the same pair of run lengths over the slot's forward work items (views have none).
struct SlotRec { u32 wf, wa, tb, tf, ta, lmin, nlmax, dx_free, lds_need, plain, lminf, nlmaxf; };

// Static tile of the deferred parameter-gradient kernels (built on the host per parameter set).
struct PTile { i32 param; i32 i0, j0; i32 pad; };   // dW tiles: pad = runs of the use list | index of the tile's first partial block << 8

// Scan element of the per-batch layout pass.
struct Lay {
    u64 val, dx;           // floats
    u32 ind, p0, p1, p2;   // operand-dimension slots
    __host__ __device__ Lay operator+(const Lay &o) const {
        Lay r; r.val = val + o.val; r.dx = dx + o.dx; r.ind = ind + o.ind; r.p0 = r.p1 = r.p2 = 0; return r;
    }
};

// Scan element of the three per-position counts taken after the grouping sort (batch heads, operand
// counts, parameter uses): one scan instead of three.
struct Tri {
    u32 a, b, c, d;
    __host__ __device__ Tri operator+(const Tri &o) const { Tri r; r.a = a + o.a; r.b = b + o.b; r.c = c + o.c; r.d = 0; return r; }
};

// Header the host reads back after scheduling (one small D2H copy).
struct SchedHeader {
    u32 n_steps, n_batches, n_items, err;
    u64 val_floats, grad_floats;
    u32 tiles_fwd, tiles_pull, tiles_dx, frontier_done;
    u32 n_slots, n_chains, works_fwd, works_pull;
    u32 n_bedges, slot_sweeps, p0, p1;
    u32 view_batches, view_floats, virt_batches, virt_floats;   // SLICE batches that are views / CONCAT batches never copied, and their sizes
};
enum : u32 { ERR_CYCLE = 1, ERR_COLLISION = 2, ERR_TABLE_FULL = 4, ERR_OVERFLOW = 8, ERR_CLASSES = 16 };

// All device pointers of one scheduled graph.  Passed by value to kernels.
struct Tables {
    u32 n, E;              // nodes / edges covered by the schedule
    u32 root;              // backward root (node id), 0xffffffff when none
    u32 n_params;
    // graph as uploaded
    const u8 *op; const u32 *out_dim; const u32 *in_off; const u32 *in_idx;
    const i32 *param; const i32 *bias; const i32 *aux0; const i32 *aux1;
    const float *payload;
    const u32 *manual;     // the caller's batch label per node (manual batching only, else null)
    const ParamDesc *params;
    // scheduler tables
    u64 *sig; u32 *step; u32 *indeg; u32 *outdeg; u32 *succ_off; u32 *succ_edge; u32 *edge_cons;
    u32 *queue; u32 *qcount;            // frontier queue, [0]=tail
    u32 *ext_indeg;                     // operands owned by another range of the partitioned depth pass (fixed once counted)
    u32 *ext_left;                      // the same count, taken down as those operands resolve
    u64 *ht_keys; u32 *ht_vals; u32 ht_mask; u32 *ht_slot;
    u32 *order; u32 *pos_of; u32 *batch_of_pos; u32 *s_aux0; u32 *s_in_off;
    u32 *batch_off; BatchRec *batches; Lay *lay; u32 *b_indim;
    u32 *val_off;          // per node: where its value row lies in V (for a SLICE node: inside its operand's row)
    u32 *nat_off;          // per node: its row in its batch's own block; the gradient arena uses this one
    u32 *dx_off; u32 *opnd_off;
    u32 *dx_gsrc;          // per schedule position of a MATVEC node with one consumer: where that consumer's gradient row lies
    u32 *slot_of; u32 *label_of; u32 *lorder;
    u32 *blevel;           // per batch: its step (depth mode) or its level inside its fused chain (agenda mode)
    u32 *chain_of_batch;   // per batch: index of its launch chain
    ChainRec *chains; CLay *clay; u32 *chain_of_lpos;
    SlotRec *slots;
    WorkRec *works_f; WorkRec *works_a;
    TileDesc *tiles_f; PullDesc *tiles_a; TileDesc *tiles_b;
    u32 *root_pos;         // [0] = schedule position of the backward root
    EdgeRec *edges;
    // parameter-use items (deferred dW / db / dE)
    u64 *it_key; u32 *it_pos; u32 *it_goff; u32 *it_xoff; u32 *pu_start; u32 *pu_end;
    uint4 *it_xrec;        // per MATVEC use with it_xoff == XP_LIST, two entries: the operand row's offset per piece (contraction
                           // index k of piece q lies at offset q + k) and the first index behind pieces 0, 1, 2 (0xffffffff: none)
    SchedHeader *hdr;
    // arenas
    float *V; float *G;
    const float *Gx;       // gradients that reach this graph's nodes from later evaluation stages (same offsets as G), or null
};

// ---- primitives (ob_prims.hip) ------------------------------------------------------------
size_t prim_scan_scratch_bytes(size_t n, size_t elem);
hipError_t prim_fill_u32(u32 *p, u32 v, size_t n, hipStream_t s);
hipError_t prim_scan_u32(const u32 *in, u32 *out, size_t n, u32 *total_dev, void *scratch, hipStream_t s);
hipError_t prim_scan_lay(const Lay *in, Lay *out, size_t n, Lay *total_dev, void *scratch, hipStream_t s);
hipError_t prim_scan_clay(const CLay *in, CLay *out, size_t n, CLay *total_dev, void *scratch, hipStream_t s);
hipError_t prim_scan_tri(const Tri *in, Tri *out, size_t n, Tri *total_dev, void *scratch, hipStream_t s);
size_t prim_sort_scratch_bytes(size_t n);
// Stable LSD radix sort of (key, val) pairs on bits [lo_bit, lo_bit + n_bits) of the key.
// keys/vals are overwritten with the sorted result; tmp arrays have the same sizes.
// n_dev (device, optional): the caller promises that pairs from index *n_dev on already sit where
// a stable sort would leave them (padding with the largest key); short inputs then sort only the
// first *n_dev pairs.
hipError_t prim_sort_pairs(u64 *keys, u32 *vals, u64 *keys_tmp, u32 *vals_tmp, size_t n, int lo_bit,
                           int n_bits, void *scratch, hipStream_t s, int *n_launches, const u32 *n_dev = nullptr);

hipError_t prim_sort_pairs_swap(u64 *&keys, u32 *&vals, u64 *&keys_tmp, u32 *&vals_tmp, size_t n, int lo_bit,
                                int n_bits, void *scratch, hipStream_t s, int *n_launches, const u32 *n_dev = nullptr);

// ---- scheduler / executor entry points ---------------------------------------------------
struct ob_ctx;
int sched_enqueue(ob_ctx *ctx);
int sched_finish(ob_ctx *ctx);
int exec_forward(ob_ctx *ctx);
int exec_backward(ob_ctx *ctx);
hipError_t exec_gather_all(const Tables &T, int which, float *dst, const u32 *dst_off, hipStream_t s);
hipError_t exec_stage_scatter(const float *G, const u32 *nat_off, u32 first_proxy, const u32 *src, const u32 *dim, u32 count,
                              const u32 *owner_nat_off, float *owner_gx, hipStream_t s);
hipError_t exec_fill_uncopied(const Tables &T, hipStream_t s);
hipError_t exec_gather_some(const Tables &T, int which, float *dst, const u32 *dst_off, hipStream_t s);
hipError_t exec_stage_fill(const float *V, const u32 *val_off, const u32 *src, const u32 *dst, const u32 *dim, u32 count,
                           float *payload, hipStream_t s);
hipError_t exec_launch_probe(float *scratch, int n, int touch, float *us_per_launch, hipStream_t s);
hipError_t exec_sgd(const ParamDesc *params_dev, u32 n_params, size_t max_count, float lr, int zero_grad, hipStream_t s);
hipError_t exec_test_gemm(int M, int N, int K, const float *A, const float *B, float *C, hipStream_t s);
