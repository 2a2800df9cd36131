// Batched execution (Section 3.3): every batch of the schedule runs as one batched operation.
// One launch covers one launch slot (one or several depth levels whose batches need no grid-wide
// ordering between them, or one node when batching is off) and runs a tile interpreter: each
// workgroup takes work items of the slot's batches and runs the matching routine.
//  - shared-weight matrix-vector groups W h_i become one W H product on fp32 MFMA, operand rows
//    gathered through the batch's row-offset list (the sparse-to-dense copy of Appendix B is
//    fused into the operand load), results written to the batch's contiguous block (so the
//    dense-to-sparse copy is the identity);
//  - component-wise groups, slices, concatenations and lookups are gathers fused with the op;
//  - log-softmax picks, squared norms and wide sums are per-row wavefront reductions.
// Backward mirrors it in reverse slot order without atomics: a node's gradient is the sum, in
// fixed (consumer, slot) order, of what each consumer edge contributes ("pull"), and the
// weight, bias and embedding gradients are reduced once per parameter over all their uses.
#include "ob_ctx.h"

#include <chrono>

typedef float floatx16 __attribute__((ext_vector_type(16)));
constexpr int LDS_FLOATS = 4 * 16 * 64;   // 16 KB: the four waves' accumulator blocks

namespace {

__device__ inline float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ inline float sigmoidf_(float x) { return 1.0f / (1.0f + expf(-x)); }

__device__ inline float wave_sum(float v)
{
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    return v;
}
__device__ inline float wave_max(float v)
{
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o));
    return v;
}

// ------------------------------------------------------------------------------------------------
// forward: component-wise / copy family
// ------------------------------------------------------------------------------------------------
// Element offset of operand slot j for the i-th row of the tile (batch row `row`).  When the
// descriptor says the tile's operand rows are evenly spaced, the address is computed and the
// row-offset list is not read.
__device__ inline u32 opnd_row(const Tables &T, const TileDesc &d, u32 j, u32 i, u32 row)
{
    // written slot by slot so that the descriptor stays in scalar registers (no dynamic indexing)
    if (j == 0 && (d.contig & 1u)) return d.base[0] + i * d.sstride[0];
    if (j == 1 && (d.contig & 2u)) return d.base[1] + i * d.sstride[1];
    if (j == 2 && (d.contig & 4u)) return d.base[2] + i * d.sstride[2];
    if (j == 3 && (d.contig & 8u)) return d.base[3] + i * d.sstride[3];
    return T.opnd_off[d.opnd + j * d.B + row];
}
__device__ inline u32 slot_dim(const Tables &T, const TileDesc &d, u32 j)
{
    if (j == 0) return d.sdim[0];
    if (j == 1) return d.sdim[1];
    if (j == 2) return d.sdim[2];
    if (j == 3) return d.sdim[3];
    return T.b_indim[d.indim + j];
}

// The fused chains' LDS copy is always reached through an LDS-typed pointer, so that these
// accesses are LDS instructions (a generic pointer would make them flat accesses, which also
// wait on outstanding global stores).
// Parameter pointers come out of descriptors as generic pointers; they always point to global
// memory, and saying so keeps their loads global instructions.
typedef __attribute__((address_space(1))) const float gl_float;
typedef float vec4f __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(1))) const vec4f gl_vec4f;
__device__ inline gl_float *as_global(const float *p) { return (gl_float *)p; }
__device__ inline float4 gl_ld4(gl_float *p)
{
    const vec4f t = *reinterpret_cast<gl_vec4f *>(p);
    return make_float4(t.x, t.y, t.z, t.w);
}

typedef __attribute__((address_space(3))) float lds_float;
typedef __attribute__((address_space(3))) vec4f lds_vec4f;
__device__ inline float4 lds_ld4(const lds_float *p)
{
    const vec4f t = *reinterpret_cast<const lds_vec4f *>(p);
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ inline void lds_st4(lds_float *p, float4 v)
{
    vec4f t; t.x = v.x; t.y = v.y; t.z = v.z; t.w = v.w;
    *reinterpret_cast<lds_vec4f *>(p) = t;
}

__device__ inline u32 slot_lds(const TileDesc &d, u32 j)
{
    if (j == 0) return d.lds_src[0];
    if (j == 1) return d.lds_src[1];
    if (j == 2) return d.lds_src[2];
    return d.lds_src[3];
}
// Operand element at arena offset `off` of slot j: from the chain's LDS copy `cl` when the
// descriptor says an earlier member of the same fused chain left it there, else from the arena.
__device__ inline float ldv(const Tables &T, const TileDesc &d, const lds_float *cl, u32 j, u32 off)
{
    float v;
    if (j < 4 && (d.flags & (TF_SRC_LDS << j))) v = cl[(u32)(off + slot_lds(d, j))];
    else v = T.V[off];
    return v;
}
__device__ inline float4 ldv4(const Tables &T, const TileDesc &d, const lds_float *cl, u32 j, u32 off)
{
    float4 v;
    if (j < 4 && (d.flags & (TF_SRC_LDS << j))) v = lds_ld4(cl + (u32)(off + slot_lds(d, j)));
    else v = ld4(T.V + off);
    return v;
}

__device__ inline float ew_value(const Tables &T, const TileDesc &d, const lds_float *cl, u32 i, u32 row, u32 col)
{
    switch (d.op) {
    case OP_INPUT: return T.payload[T.s_aux0[d.pos0 + row] + col];
    case OP_LOOKUP: return as_global(d.w)[(size_t)T.s_aux0[d.pos0 + row] * d.d + col];
    case OP_ADD: {
        float acc = 0.f;
        for (u32 j = 0; j < d.arity; ++j) acc += ldv(T, d, cl, j, opnd_row(T, d, j, i, row) + col);
        return acc;
    }
    case OP_CMULT: return ldv(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col) * ldv(T, d, cl, 1, opnd_row(T, d, 1, i, row) + col);
    case OP_TANH: return tanhf(ldv(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col));
    case OP_SIGMOID: return sigmoidf_(ldv(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col));
    case OP_SLICE: return ldv(T, d, cl, 0, opnd_row(T, d, 0, i, row) + (u32)d.aux0 + col);
    case OP_CONCAT: {
        u32 c = col;
        for (u32 j = 0; j < d.arity; ++j) {
            const u32 dj = slot_dim(T, d, j);
            if (c < dj) return ldv(T, d, cl, j, opnd_row(T, d, j, i, row) + c);
            c -= dj;
        }
        return 0.f;
    }
    default: return 0.f;
    }
}

__device__ inline float4 ew_value4(const Tables &T, const TileDesc &d, const lds_float *cl, u32 i, u32 row, u32 col)
{
    switch (d.op) {
    case OP_INPUT: return ld4(T.payload + T.s_aux0[d.pos0 + row] + col);
    case OP_LOOKUP: return gl_ld4(as_global(d.w) + (size_t)T.s_aux0[d.pos0 + row] * d.d + col);
    case OP_ADD: {
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (u32 j = 0; j < d.arity; ++j) {
            const float4 x = ldv4(T, d, cl, j, opnd_row(T, d, j, i, row) + col);
            acc.x += x.x; acc.y += x.y; acc.z += x.z; acc.w += x.w;
        }
        return acc;
    }
    case OP_CMULT: {
        const float4 a = ldv4(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col), b = ldv4(T, d, cl, 1, opnd_row(T, d, 1, i, row) + col);
        return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w);
    }
    case OP_TANH: {
        const float4 a = ldv4(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col);
        return make_float4(tanhf(a.x), tanhf(a.y), tanhf(a.z), tanhf(a.w));
    }
    case OP_SIGMOID: {
        const float4 a = ldv4(T, d, cl, 0, opnd_row(T, d, 0, i, row) + col);
        return make_float4(sigmoidf_(a.x), sigmoidf_(a.y), sigmoidf_(a.z), sigmoidf_(a.w));
    }
    case OP_SLICE: return ldv4(T, d, cl, 0, opnd_row(T, d, 0, i, row) + (u32)d.aux0 + col);
    case OP_CONCAT: {
        u32 c = col;
        for (u32 j = 0; j < d.arity; ++j) {
            const u32 dj = slot_dim(T, d, j);
            if (c < dj) return ldv4(T, d, cl, j, opnd_row(T, d, j, i, row) + c);
            c -= dj;
        }
        return make_float4(0.f, 0.f, 0.f, 0.f);
    }
    default: return make_float4(0.f, 0.f, 0.f, 0.f);
    }
}

// Tiles flagged TF_SIMPLE: every operand address is base + i * stride + column, so the whole
// descriptor is read once up front and the element loop has no table look-ups and one switch.
__device__ inline float4 ld_slot4(const Tables &T, const lds_float *cl, bool from_lds, u32 idx, u32 delta)
{
    float4 v;
    if (from_lds) v = lds_ld4(cl + (u32)(idx + delta));
    else v = ld4(T.V + idx);
    return v;
}
__device__ inline void ew_fwd_tile_simple(const Tables &T, const TileDesc &d, lds_float *cl, u32 tid, u32 nthr)
{
    const u32 op = d.op, dd = d.d, total = d.nrows * dd, flags = d.flags, ar = d.arity;
    const u32 shift = op == OP_SLICE ? (u32)d.aux0 : 0u;
    const u32 b0 = d.base[0] + shift, b1 = d.base[1], b2 = d.base[2], b3 = d.base[3];
    const u32 s0 = d.sstride[0], s1 = d.sstride[1], s2 = d.sstride[2], s3 = d.sstride[3];
    const u32 l0 = d.lds_src[0], l1 = d.lds_src[1], l2 = d.lds_src[2], l3 = d.lds_src[3];
    const u32 outb = d.val_off + d.row0 * dd, outs = d.rstride * dd, lo = d.lds_out;
    const bool f0 = (flags & (TF_SRC_LDS << 0)) != 0, f1 = (flags & (TF_SRC_LDS << 1)) != 0;
    const bool f2 = (flags & (TF_SRC_LDS << 2)) != 0, f3 = (flags & (TF_SRC_LDS << 3)) != 0;
    const bool keep = (flags & TF_OUT_LDS) != 0;
    for (u32 x = tid * 4; x < total; x += nthr * 4) {
        const u32 i = x / dd, col = x - i * dd;
        float4 v = ld_slot4(T, cl, f0, b0 + i * s0 + col, l0);
        switch (op) {
        case OP_ADD:
            if (ar > 1) { const float4 y = ld_slot4(T, cl, f1, b1 + i * s1 + col, l1); v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w; }
            if (ar > 2) { const float4 y = ld_slot4(T, cl, f2, b2 + i * s2 + col, l2); v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w; }
            if (ar > 3) { const float4 y = ld_slot4(T, cl, f3, b3 + i * s3 + col, l3); v.x += y.x; v.y += y.y; v.z += y.z; v.w += y.w; }
            break;
        case OP_CMULT: {
            const float4 y = ld_slot4(T, cl, f1, b1 + i * s1 + col, l1);
            v.x *= y.x; v.y *= y.y; v.z *= y.z; v.w *= y.w;
            break;
        }
        case OP_TANH: v = make_float4(tanhf(v.x), tanhf(v.y), tanhf(v.z), tanhf(v.w)); break;
        case OP_SIGMOID: v = make_float4(sigmoidf_(v.x), sigmoidf_(v.y), sigmoidf_(v.z), sigmoidf_(v.w)); break;
        default: break;   // OP_SLICE: a copy
        }
        const u32 o = outb + i * outs + col;
        st4(T.V + o, v);
        if (keep) lds_st4(cl + (u32)(o + lo), v);
    }
}

// rows row0 + i * rstride (i < nrows) of the batch, all columns; worked by threads tid < nthr.
// cl: the fused chain's LDS copy (results are written there too when the descriptor asks for it).
__device__ inline void ew_fwd_tile(const Tables &T, const TileDesc &d, lds_float *cl, u32 tid, u32 nthr)
{
    if (d.flags & TF_SIMPLE) { ew_fwd_tile_simple(T, d, cl, tid, nthr); return; }
    const u32 total = d.nrows * d.d;
    float *out = T.V + d.val_off;
    const bool keep = (d.flags & TF_OUT_LDS) != 0;
    if (d.flags & TF_VEC4) {
        for (u32 x = tid * 4; x < total; x += nthr * 4) {
            const u32 i = x / d.d, col = x % d.d, row = d.row0 + i * d.rstride;
            const float4 v = ew_value4(T, d, cl, i, row, col);
            st4(out + row * d.d + col, v);
            if (keep) lds_st4(cl + (u32)(d.val_off + row * d.d + col + d.lds_out), v);
        }
    } else {
        for (u32 x = tid; x < total; x += nthr) {
            const u32 i = x / d.d, col = x % d.d, row = d.row0 + i * d.rstride;
            const float v = ew_value(T, d, cl, i, row, col);
            out[row * d.d + col] = v;
            if (keep) cl[(u32)(d.val_off + row * d.d + col + d.lds_out)] = v;
        }
    }
}

// ------------------------------------------------------------------------------------------------
// forward: per-row reductions (one wave per row)
// ------------------------------------------------------------------------------------------------
__device__ inline void red_fwd_tile(const Tables &T, const TileDesc &d)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const u32 row = d.t * ROWS_PER_RED_TILE + w;
    if (row >= d.B) return;
    const float *x = T.V + opnd_row(T, d, 0, row - d.row0, row);
    const u32 K = d.k;
    if (d.op == OP_SQNORM) {
        float acc = 0.f;
        for (u32 c = lane; c < K; c += 64) { const float a = x[c]; acc += a * a; }
        acc = wave_sum(acc);
        if (lane == 0) T.V[d.val_off + row] = acc;
    } else {  // OP_PICK_NLS: logsumexp(x) - x[label], shifted by the row maximum
        float mx = -INFINITY;
        for (u32 c = lane; c < K; c += 64) mx = fmaxf(mx, x[c]);
        mx = wave_max(mx);
        // The first element that holds the maximum contributes exp(0) = 1: it stays out of the sum
        // and log1p takes its place, so that a confident row (sum barely above 1) keeps the small
        // part of its loss instead of rounding it away.
        u32 am = 0xffffffffu;
        for (u32 c = lane; c < K; c += 64)
            if (x[c] == mx && c < am) am = c;
        for (int o = 32; o > 0; o >>= 1) { const u32 t = (u32)__shfl_xor((int)am, o); am = t < am ? t : am; }
        float s = 0.f;
        for (u32 c = lane; c < K; c += 64)
            if (c != am) s += expf(x[c] - mx);
        s = wave_sum(s);
        if (lane == 0) T.V[d.val_off + row] = log1pf(s) + (mx - x[T.s_aux0[d.pos0 + row]]);
    }
}

// wide sum: one workgroup per row, operands strided over threads, fixed-shape tree in LDS
__device__ inline void wide_add_tile(const Tables &T, const TileDesc &d, float *lds)
{
    const u32 row = d.t;
    const u32 *opnd = T.opnd_off + d.opnd;
    for (u32 c = 0; c < d.d; ++c) {
        float acc = 0.f;
        for (u32 j = threadIdx.x; j < d.arity; j += WG) acc += T.V[opnd[j * d.B + row] + c];
        lds[threadIdx.x] = acc;
        __syncthreads();
        for (int o = WG / 2; o > 0; o >>= 1) {
            if ((int)threadIdx.x < o) lds[threadIdx.x] += lds[threadIdx.x + o];
            __syncthreads();
        }
        if (threadIdx.x == 0) T.V[d.val_off + row * d.d + c] = lds[0];
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// MFMA tile: one 32x32 fp32 accumulator block per workgroup; the 4 waves split the contraction
// and their partial blocks are summed through LDS in wave order.
// v_mfma_f32_32x32x2f32: lane l supplies A[l%32][l/32] and B[l/32][l%32]; accumulator register v
// of lane l is C[8*(v/4) + 4*(l/32) + v%4][l%32].  The contraction index may be permuted freely as
// long as A and B use the same permutation: within a block of 8, lane half h takes the four
// consecutive indices 4h..4h+3, so that K-contiguous operands are read as one float4.
// ------------------------------------------------------------------------------------------------
__device__ inline floatx16 mfma4(float4 a, float4 b, floatx16 acc)
{
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.x, b.x, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.y, b.y, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.z, b.z, acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a.w, b.w, acc, 0, 0, 0);
    return acc;
}

// Sums the NW waves' accumulators in wave order; on return wave w holds in out[0 .. 16/NW) the
// accumulator registers v = (16/NW) * w + i, i.e. rows 8*(v/4) + 4*(lane/32) + v%4 of column lane%32.
template <int NW>
__device__ inline void reduce_waves(const floatx16 &acc, float *lds, float *out)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    for (int v = 0; v < 16; ++v) lds[(w * 16 + v) * 64 + lane] = acc[v];
    __syncthreads();
    for (int i = 0; i < 16 / NW; ++i) {
        const int v = (16 / NW) * w + i;
        float s = lds[v * 64 + lane];
        for (int ww = 1; ww < NW; ++ww) s += lds[(ww * 16 + v) * 64 + lane];
        out[i] = s;
    }
    __syncthreads();
}

// split [0, total) in units of 8 over the NW waves
template <int NW>
__device__ inline void wave_range(u32 total, u32 &lo, u32 &hi)
{
    const u32 w = threadIdx.x >> 6;
    const u32 n8 = (total + 7) / 8;
    const u32 per = (n8 + NW - 1) / NW;
    lo = w * per * 8;
    hi = (w + 1) * per * 8;
    const u32 pad = n8 * 8;
    if (lo > pad) lo = pad;
    if (hi > pad) hi = pad;
}

constexpr int KU = 8;   // blocks of 8 contraction indices whose loads are issued together

// The operand row of one product row.  Read whole, it starts at o0.  Read in pieces (the operand is a
// CONCAT node that was never copied, Section 3.3), contraction index k lies at o<q> + k for the piece q that
// holds k (c<q> = first index behind piece q, 0xffffffff from the last piece on; the piece's first index
// is already subtracted from o<q>, in wrap-around arithmetic).  Pieces are multiples of four indices long.
struct XRow { u32 o0, o1, o2, o3; };
struct XCuts { u32 c0, c1, c2; };
static_assert(XP_MAX == 4, "XRow holds four piece offsets");
template <bool XP>
__device__ inline u32 x_at(const XRow &x, const XCuts &c, u32 k)
{
    u32 o = x.o0;
    if (XP) {
        // (the empty statements keep the three selects as they are: taken together the compiler would turn them
        // into an indexed read of a four-entry table in scratch memory)
        if (k >= c.c0) o = x.o1;
        asm volatile("" : "+v"(o));
        if (k >= c.c1) o = x.o2;
        asm volatile("" : "+v"(o));
        if (k >= c.c2) o = x.o3;
    }
    return o + k;
}
__device__ inline XCuts x_cuts(const TileDesc &d)
{
    XCuts c;
    u32 s = d.sdim[0];
    c.c0 = d.arity > 1 ? s : 0xffffffffu; s += d.sdim[1];
    c.c1 = d.arity > 2 ? s : 0xffffffffu; s += d.sdim[2];
    c.c2 = d.arity > 3 ? s : 0xffffffffu;
    return c;
}
template <bool XP>
__device__ inline XRow x_row(const Tables &T, const TileDesc &d, bool row_ok, u32 i, u32 row)
{
    XRow x;
    x.o0 = row_ok ? opnd_row(T, d, 0, i, row) : 0u;
    x.o1 = x.o2 = x.o3 = x.o0;
    if (XP && row_ok) {
        if (d.arity > 1) x.o1 = opnd_row(T, d, 1, i, row);
        if (d.arity > 2) x.o2 = opnd_row(T, d, 2, i, row);
        if (d.arity > 3) x.o3 = opnd_row(T, d, 3, i, row);
    }
    return x;
}

constexpr int DX_WAVES = 8;   // the dX kernel splits its long contraction (rows of W) over 8 waves

// Y[B x m] = X[B x K] W^T + b.   xrow: this lane's X row (valid when row_ok), W row-major [m x K].
template <bool XP>
__device__ inline void gemm_nt_tile(const float *V, const XRow &xr, const XCuts &xc, bool row_ok, u32 B, const float *W,
                                    const float *bias, u32 m, u32 K, bool fast, float *Y, u32 r0, u32 i0, float *lds)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const u32 l32 = lane & 31, h = lane >> 5;
    const u32 col = i0 + l32;
    const bool col_ok = col < m;
    gl_float *wrow = as_global(W) + (size_t)(col_ok ? col : 0u) * K;
    u32 lo, hi;
    wave_range<4>(K, lo, hi);
    floatx16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (fast) {
        for (u32 kb = lo; kb < hi; kb += 8 * KU) {
            float4 a[KU], b[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const u32 k0 = kb + 8 * u + 4 * h;
                const bool in = kb + 8 * u < hi && k0 < K;
                a[u] = (in && row_ok) ? ld4(V + x_at<XP>(xr, xc, k0)) : z4;
                b[u] = (in && col_ok) ? gl_ld4(wrow + k0) : z4;
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) acc = mfma4(a[u], b[u], acc);
        }
    } else {
        for (u32 kb = lo; kb < hi; kb += 8) {
            const u32 k0 = kb + 4 * h;
            float av[4] = {0.f, 0.f, 0.f, 0.f}, bv[4] = {0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < 4; ++s)
                if (k0 + s < K) {
                    if (row_ok) av[s] = V[x_at<XP>(xr, xc, k0 + s)];
                    if (col_ok) bv[s] = wrow[k0 + s];
                }
            acc = mfma4(make_float4(av[0], av[1], av[2], av[3]), make_float4(bv[0], bv[1], bv[2], bv[3]), acc);
        }
    }
    float out[4];
    reduce_waves<4>(acc, lds, out);
    if (col_ok) {
        const float bb = bias ? as_global(bias)[col] : 0.f;
        for (int i = 0; i < 4; ++i) {
            const u32 rr = r0 + 8 * w + 4 * h + i;
            if (rr < B) Y[(size_t)rr * m + col] = out[i] + bb;
        }
    }
}

// Batches with many rows: a workgroup covers 64 x 64 outputs, wave w the 32x32 block (w / 2, w % 2)
// over the whole contraction, so no partial sums cross waves and nothing goes through LDS.
template <bool XP>
__device__ inline void matvec_fwd_tile_wide(const Tables &T, const TileDesc &d)
{
    const u32 lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const u32 l32 = lane & 31, h = lane >> 5;
    const u32 ntn = (d.d + GTW - 1) / GTW;
    const u32 r0 = (d.t / ntn) * GTW + 32 * (w >> 1), i0 = (d.t % ntn) * GTW + 32 * (w & 1);
    const u32 row = r0 + l32, col = i0 + l32;
    const bool row_ok = row < d.B, col_ok = col < d.d;
    const u32 K = d.k;
    const XRow xr = x_row<XP>(T, d, row_ok, row - d.row0, row);
    const XCuts xc = x_cuts(d);
    gl_float *wrow = as_global(d.w) + (size_t)(col_ok ? col : 0u) * K;
    const bool fast = (d.flags & TF_ALIGNED) && (K & 3u) == 0;
    floatx16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    const u32 Kp = (K + 7u) & ~7u;
    if (fast) {
        for (u32 kb = 0; kb < Kp; kb += 8 * KU) {
            float4 a[KU], b[KU];
#pragma unroll
            for (int u = 0; u < KU; ++u) {
                const u32 k0 = kb + 8 * u + 4 * h;
                const bool in = k0 < K;
                a[u] = (in && row_ok) ? ld4(T.V + x_at<XP>(xr, xc, k0)) : z4;
                b[u] = (in && col_ok) ? gl_ld4(wrow + k0) : z4;
            }
#pragma unroll
            for (int u = 0; u < KU; ++u) acc = mfma4(a[u], b[u], acc);
        }
    } else {
        for (u32 kb = 0; kb < Kp; kb += 8) {
            const u32 k0 = kb + 4 * h;
            float av[4] = {0.f, 0.f, 0.f, 0.f}, bv[4] = {0.f, 0.f, 0.f, 0.f};
            for (int s = 0; s < 4; ++s)
                if (k0 + s < K) {
                    if (row_ok) av[s] = T.V[x_at<XP>(xr, xc, k0 + s)];
                    if (col_ok) bv[s] = wrow[k0 + s];
                }
            acc = mfma4(make_float4(av[0], av[1], av[2], av[3]), make_float4(bv[0], bv[1], bv[2], bv[3]), acc);
        }
    }
    if (col_ok) {
        const float bb = d.b ? as_global(d.b)[col] : 0.f;
        float *Y = T.V + d.val_off;
        for (int v = 0; v < 16; ++v) {
            const u32 rr = r0 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (rr < d.B) Y[(size_t)rr * d.d + col] = acc[v] + bb;
        }
    }
}

// The same 64 x 64 tile with the operands staged through LDS.  Reading one operand row per lane
// straight from memory touches 64 different cache lines per load instruction, which the address
// path serialises; here the workgroup loads each 64-float piece of a row with 16 adjacent lanes
// (two full lines), writes it to LDS, and the MFMA operands (lane = row, four consecutive k) are
// LDS reads.  The next 64-wide chunk of the contraction is loaded into registers while the
// current one is multiplied.  Rows are padded to 68 floats so that the 32 rows read together by
// a half-wave spread over the banks.  Needs K % 4 == 0 and 16-byte aligned operand rows.
constexpr u32 WKC = 64;             // contraction chunk
constexpr u32 WLD = WKC + 4;        // padded LDS row
constexpr u32 WIDE_LDS_FLOATS = 2 * GTW * WLD;   // X tile + W tile
template <bool XP>
__device__ inline void matvec_fwd_tile_wide_lds(const Tables &T, const TileDesc &d, float *lds)
{
    const u32 tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const u32 l32 = lane & 31, h = lane >> 5;
    const u32 ntn = (d.d + GTW - 1) / GTW;
    const u32 r0 = (d.t / ntn) * GTW, i0 = (d.t % ntn) * GTW;
    const u32 K = d.k, m = d.d;
    lds_float *xs = (lds_float *)lds, *ws = xs + GTW * WLD;
    // loader role: piece c4 (four floats) of rows lr + 16 p, p < 4
    const u32 lr = tid >> 4, c4 = (tid & 15u) * 4u;
    XRow xr[4];
    const XCuts xc = x_cuts(d);
    bool xok[4], wok[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const u32 row = r0 + lr + 16u * p, col = i0 + lr + 16u * p;
        xok[p] = row < d.B;
        wok[p] = col < m;
        xr[p] = x_row<XP>(T, d, xok[p], row - d.row0, row);
    }
    gl_float *W = as_global(d.w);
    float4 px[4], pw[4];
    auto prefetch = [&](u32 kc) {
        const u32 k = kc + c4;
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            // (zeros written out: a zero vector captured by reference becomes a stack object here and the
            // choice between it and the load a choice between two addresses)
            px[p] = make_float4(0.f, 0.f, 0.f, 0.f);
            pw[p] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (xok[p] && k < K) px[p] = ld4(T.V + x_at<XP>(xr[p], xc, k));
            if (wok[p] && k < K) pw[p] = gl_ld4(W + (size_t)(i0 + lr + 16u * p) * K + k);
        }
    };
    floatx16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const u32 arow = (32u * (w >> 1) + l32) * WLD + 4u * h, brow = (32u * (w & 1u) + l32) * WLD + 4u * h;
    prefetch(0);
    for (u32 kc = 0; kc < K; kc += WKC) {
        __syncthreads();            // the previous chunk has been read
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            lds_st4(xs + (lr + 16u * p) * WLD + c4, px[p]);
            lds_st4(ws + (lr + 16u * p) * WLD + c4, pw[p]);
        }
        __syncthreads();
        if (kc + WKC < K) prefetch(kc + WKC);
#pragma unroll
        for (u32 k8 = 0; k8 < WKC / 8; ++k8)
            acc = mfma4(lds_ld4(xs + arow + 8u * k8), lds_ld4(ws + brow + 8u * k8), acc);
    }
    const u32 col = i0 + 32u * (w & 1u) + l32;
    if (col < m) {
        const float bb = d.b ? as_global(d.b)[col] : 0.f;
        float *Y = T.V + d.val_off;
        for (int v = 0; v < 16; ++v) {
            const u32 rr = r0 + 32u * (w >> 1) + 8u * (v >> 2) + 4u * h + (v & 3);
            if (rr < d.B) Y[(size_t)rr * m + col] = acc[v] + bb;
        }
    }
    __syncthreads();                // the LDS space is free for the workgroup's next tile
}

// XP: the launch holds products whose operand rows are read in pieces (a slot with such a batch runs the
// step kernel built with XP; products read whole take the same code there, with no cut inside the row).
template <bool XP>
__device__ inline void matvec_fwd_tile(const Tables &T, const TileDesc &d, float *lds)
{
    if (d.flags & TF_WIDE) {
        if ((d.flags & TF_ALIGNED) && (d.k & 3u) == 0) matvec_fwd_tile_wide_lds<XP>(T, d, lds);
        else matvec_fwd_tile_wide<XP>(T, d);
        return;
    }
    const u32 ntn = (d.d + GT - 1) / GT;
    const u32 r0 = (d.t / ntn) * GT, i0 = (d.t % ntn) * GT;
    const bool fast = (d.flags & 2u) && (d.k & 3u) == 0;
    const u32 row = r0 + (threadIdx.x & 31);
    const bool row_ok = row < d.B;
    gemm_nt_tile<XP>(T.V, x_row<XP>(T, d, row_ok, row - d.row0, row), x_cuts(d), row_ok, d.B, d.w, d.b, d.d, d.k, fast,
                     T.V + d.val_off, r0, i0, lds);
}

// dX[B x K] = G[B x m] W, contraction over m.  G rows are the batch's own contiguous block.
// 16x16 output tiles (v_mfma_f32_16x16x4f32: lane l supplies A[l%16][l/16] and B[l/16][l%16];
// accumulator register v of lane l is C[4*(l/16) + v][l%16]); the DX_WAVES waves split the
// contraction, lane quarter q takes the four consecutive indices 4q..4q+3 of every block of 16.
// Batches with many rows: 32x32 dX tiles (v_mfma_f32_32x32x2f32), the DX_WAVES waves split the
// contraction over the rows of W and their blocks are summed through LDS in wave order.
__device__ inline void matvec_dx_tile_wide(const Tables &T, const TileDesc &d, float *lds)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const u32 l32 = lane & 31, h = lane >> 5;
    const u32 K = d.k, m = d.d;
    const u32 ntn = (K + DXTW - 1) / DXTW;
    const u32 r0 = (d.t / ntn) * DXTW, c0 = (d.t % ntn) * DXTW;
    const u32 row = r0 + l32, col = c0 + l32;
    const bool row_ok = row < d.B, col_ok = col < K;
    const u32 grow_row = row_ok ? row : r0;
    const float *grow = T.G + (((d.flags & TF_G_ALIAS) && !T.Gx) ? ((d.contig & 1u) ? d.base[0] + (grow_row - r0) * d.sstride[0]
                                                                             : T.dx_gsrc[d.pos0 + grow_row])
                                                        : d.val_off + grow_row * m);
    gl_float *wcol = as_global(d.w) + (col_ok ? col : 0u);
    const bool fast = (m & 3u) == 0;
    u32 lo, hi;
    wave_range<DX_WAVES>(m, lo, hi);
    floatx16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (u32 ib = lo; ib < hi; ib += 8 * KU) {
        float4 a[KU], b[KU];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const u32 i0 = ib + 8 * u + 4 * h;
            const bool in = ib + 8 * u < hi && i0 < m;
            if (fast) {
                a[u] = (in && row_ok) ? ld4(grow + i0) : z4;
                if (in && col_ok) {
                    gl_float *wp = wcol + (size_t)i0 * K;
                    b[u] = make_float4(wp[0], wp[K], wp[2 * (size_t)K], wp[3 * (size_t)K]);
                } else {
                    b[u] = z4;
                }
            } else {
                float av[4] = {0.f, 0.f, 0.f, 0.f}, bv[4] = {0.f, 0.f, 0.f, 0.f};
                for (int s = 0; s < 4; ++s)
                    if (in && i0 + s < m) {
                        if (row_ok) av[s] = grow[i0 + s];
                        if (col_ok) bv[s] = wcol[(size_t)(i0 + s) * K];
                    }
                a[u] = make_float4(av[0], av[1], av[2], av[3]);
                b[u] = make_float4(bv[0], bv[1], bv[2], bv[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) acc = mfma4(a[u], b[u], acc);
    }
    float out[16 / DX_WAVES];
    reduce_waves<DX_WAVES>(acc, lds, out);
    if (col_ok) {
        float *dX = T.G + d.dx_off;
        for (int i = 0; i < 16 / DX_WAVES; ++i) {
            const int v = (16 / DX_WAVES) * w + i;
            const u32 rr = r0 + 8 * (v >> 2) + 4 * h + (v & 3);
            if (rr < d.B) dX[(size_t)rr * K + col] = out[i];
        }
    }
}

typedef float floatx4 __attribute__((ext_vector_type(4)));
__device__ inline void matvec_dx_tile(const Tables &T, const TileDesc &d, float *lds)
{
    if (dx_tile_edge(d.flags, d.k) == (u32)DXTW) { matvec_dx_tile_wide(T, d, lds); return; }
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    const u32 l16 = lane & 15, q = lane >> 4;
    const u32 K = d.k, m = d.d;
    const u32 ntn = (K + DXT - 1) / DXT;
    const u32 r0 = (d.t / ntn) * DXT, c0 = (d.t % ntn) * DXT;
    const u32 row = r0 + l16, col = c0 + l16;
    const bool row_ok = row < d.B, col_ok = col < K;
    // this lane's gradient row: the batch's own block, or (TF_G_ALIAS) the one consumer's row as it is
    const u32 grow_row = row_ok ? row : r0;
    const float *grow = T.G + (((d.flags & TF_G_ALIAS) && !T.Gx) ? ((d.contig & 1u) ? d.base[0] + (grow_row - r0) * d.sstride[0]
                                                                             : T.dx_gsrc[d.pos0 + grow_row])
                                                        : d.val_off + grow_row * m);
    gl_float *wcol = as_global(d.w) + (col_ok ? col : 0u);
    const bool fast = (m & 3u) == 0;
    // split [0, m) in units of 16 over the waves
    const u32 n16 = (m + 15) / 16, per = (n16 + DX_WAVES - 1) / DX_WAVES;
    u32 lo = (u32)w * per * 16, hi = ((u32)w + 1) * per * 16;
    if (lo > n16 * 16) lo = n16 * 16;
    if (hi > n16 * 16) hi = n16 * 16;
    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    for (u32 ib = lo; ib < hi; ib += 16 * KU) {
        float4 a[KU], b[KU];
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            const u32 i0 = ib + 16 * u + 4 * q;
            const bool in = ib + 16 * u < hi && i0 < m;
            if (fast) {
                a[u] = (in && row_ok) ? ld4(grow + i0) : z4;
                if (in && col_ok) {
                    gl_float *wp = wcol + (size_t)i0 * K;
                    b[u] = make_float4(wp[0], wp[K], wp[2 * (size_t)K], wp[3 * (size_t)K]);
                } else {
                    b[u] = z4;
                }
            } else {
                float av[4] = {0.f, 0.f, 0.f, 0.f}, bv[4] = {0.f, 0.f, 0.f, 0.f};
                for (int s = 0; s < 4; ++s)
                    if (in && i0 + s < m) {
                        if (row_ok) av[s] = grow[i0 + s];
                        if (col_ok) bv[s] = wcol[(size_t)(i0 + s) * K];
                    }
                a[u] = make_float4(av[0], av[1], av[2], av[3]);
                b[u] = make_float4(bv[0], bv[1], bv[2], bv[3]);
            }
        }
#pragma unroll
        for (int u = 0; u < KU; ++u) {
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].x, b[u].x, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].y, b[u].y, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].z, b[u].z, acc, 0, 0, 0);
            acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a[u].w, b[u].w, acc, 0, 0, 0);
        }
    }
    // sum the waves' 16x16 blocks in wave order; wave 0 writes the tile
    for (int v = 0; v < 4; ++v) lds[(w * 4 + v) * 64 + lane] = acc[v];
    __syncthreads();
    if (w == 0 && col_ok) {
        float *dX = T.G + d.dx_off;
        for (int v = 0; v < 4; ++v) {
            float s = lds[v * 64 + lane];
            for (int ww = 1; ww < DX_WAVES; ++ww) s += lds[(ww * 4 + v) * 64 + lane];
            const u32 rr = r0 + 4 * q + v;
            if (rr < d.B) dX[(size_t)rr * K + col] = s;
        }
    }
    __syncthreads();
}

// dW[m x K] += sum over uses of g x^T (deferred: once per parameter over every use in the graph).
// A workgroup owns a 64 x 64 block of dW; wave w the 32 x 32 quarter (w / 2, w % 2) over all uses,
// so no partial sums cross waves and the order of the sum is the order of the sorted use list.
// The uses are walked in chunks of 32: the 64-float pieces of the 32 gradient rows and of the 32
// operand rows are loaded by 16 adjacent lanes each (two full lines per row) into LDS, the MFMA
// operands are LDS reads, and the next chunk (and the row offsets of the one after) are on their
// way while the current one is multiplied.
constexpr u32 PWT = 64;              // dW tile edge
constexpr u32 PWC = 32;              // uses per chunk
constexpr u32 PWLD = PWT + 4;        // padded LDS row
constexpr u32 PW_LDS_FLOATS = 2 * PWC * PWLD;
static_assert(PWT == (u32)PWTILE, "host tile list and kernel agree on the tile edge");

// four consecutive floats of a row that may end early (n valid) or start unaligned
__device__ inline float4 ld4_guard(const float *base, u32 off, u32 n)
{
    if (n >= 4u && ((off & 3u) == 0u)) return ld4(base + off);
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (n > 0u) v.x = base[off];
    if (n > 1u) v.y = base[off + 1];
    if (n > 2u) v.z = base[off + 2];
    if (n > 3u) v.w = base[off + 3];
    return v;
}

// The use list of a tile is cut into up to `nsp` runs of whole chunks, one workgroup each (a tile
// alone would walk 1000+ uses one chunk after the other, with one chunk's loads in flight).  Each
// workgroup leaves its partial block in `part`; a second small kernel adds the partial blocks, in
// run order, to the gradient (a kernel boundary costs less here than device-wide fences between
// workgroups, which write back every dirty line of an XCD's L2).
__device__ inline void param_w_tile(const Tables &T, const PTile &pt, float *lds, u32 sp, float *part)
{
    const u32 nsp = (u32)pt.pad & 0xffu, pbase = (u32)pt.pad >> 8;
    if (sp >= nsp) return;
    const u32 tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const u32 l32 = lane & 31, h = lane >> 5;
    const u32 slot = (u32)pt.param * 4u;
    const u32 start = T.pu_start[slot], end = T.pu_end[slot];
    if (start == end) return;
    const ParamDesc P = T.params[pt.param];
    const u32 m = (u32)P.rows, K = (u32)P.cols;
    const u32 i0 = (u32)pt.i0, j0 = (u32)pt.j0;
    lds_float *gs = (lds_float *)lds, *xs = gs + PWC * PWLD;
    // loader role: piece c4 of the rows of uses lu and lu + 16 of the chunk
    const u32 lu = tid >> 4, c4 = (tid & 15u) * 4u;
    const u32 gi = i0 + c4, xj = j0 + c4;
    const u32 gn = gi < m ? m - gi : 0u, xn = xj < K ? K - xj : 0u;    // valid elements from this piece on
    const u32 all_chunks = (end - start + PWC - 1) / PWC;
    const u32 nsp_eff = all_chunks < nsp ? all_chunks : nsp;      // runs that hold at least one chunk
    if (sp >= nsp_eff) return;
    const u32 per = (all_chunks + nsp_eff - 1) / nsp_eff;
    const u32 c_lo = sp * per, c_hi = (sp + 1) * per < all_chunks ? (sp + 1) * per : all_chunks;
    const u32 n_uses = end - start;
    // Row offsets run ahead of the rows in two steps, each a round trip to memory of its own: heads() asks for
    // the offsets of the chunk after next, resolve() makes the next chunk's offsets current and, for a use whose
    // operand row is in pieces (its batch reads through an uncopied CONCAT: it_xoff is XP_LIST), asks for the
    // use's piece record; fetch() picks the piece this thread's four columns lie in and asks for the rows.
    u32 go[2] = {0u, 0u}, xo[2] = {0u, 0u}, ngo[2] = {0u, 0u}, nxo[2] = {0u, 0u}, rec[2] = {0u, 0u};
    uint4 ro[2] = {make_uint4(0u, 0u, 0u, 0u), make_uint4(0u, 0u, 0u, 0u)}, rc[2] = {ro[0], ro[0]};
    bool ok[2] = {false, false}, nok[2] = {false, false};
    auto heads = [&](u32 c) {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const u32 it = c * PWC + lu + 16u * p;
            nok[p] = it < n_uses;
            rec[p] = start + it;
            ngo[p] = nok[p] ? T.it_goff[start + it] : 0u;
            nxo[p] = nok[p] ? T.it_xoff[start + it] : 0u;
        }
    };
    u32 crec[2] = {0u, 0u};
    auto resolve = [&]() {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            ok[p] = nok[p]; go[p] = ngo[p]; xo[p] = nxo[p]; crec[p] = rec[p];
            if (ok[p] && xo[p] == XP_LIST) { ro[p] = T.it_xrec[2 * (size_t)crec[p]]; rc[p] = T.it_xrec[2 * (size_t)crec[p] + 1]; }
        }
    };
    const float4 z4 = make_float4(0.f, 0.f, 0.f, 0.f);
    float4 pg[2], px[2];
    auto fetch = [&]() {
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            u32 x = xo[p];
            if (ok[p] && x == XP_LIST) x = xj >= rc[p].z ? ro[p].w : (xj >= rc[p].y ? ro[p].z : (xj >= rc[p].x ? ro[p].y : ro[p].x));
            pg[p] = ok[p] ? ld4_guard(T.G, go[p] + gi, gn) : z4;
            px[p] = ok[p] ? ld4_guard(T.V, x + xj, xn) : z4;
        }
    };
    floatx16 acc;
    for (int v = 0; v < 16; ++v) acc[v] = 0.f;
    const u32 n_chunks = c_hi;
    if (c_lo < c_hi) {
        heads(c_lo);
        resolve();
        if (c_lo + 1 < c_hi) heads(c_lo + 1);
        fetch();
        if (c_lo + 1 < c_hi) {
            resolve();
            if (c_lo + 2 < c_hi) heads(c_lo + 2);
        }
    }
    const u32 acol = 32u * (w >> 1) + l32, bcol = 32u * (w & 1u) + l32;
    for (u32 c = c_lo; c < n_chunks; ++c) {
        __syncthreads();            // the previous chunk has been read
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            lds_st4(gs + (lu + 16u * p) * PWLD + c4, pg[p]);
            lds_st4(xs + (lu + 16u * p) * PWLD + c4, px[p]);
        }
        __syncthreads();
        if (c + 1 < n_chunks) {
            fetch();                                   // chunk c + 1: its offsets (and piece records) are here
            if (c + 2 < n_chunks) {
                resolve();                             // chunk c + 2
                if (c + 3 < n_chunks) heads(c + 3);
            }
        }
#pragma unroll
        for (u32 b8 = 0; b8 < PWC / 8; ++b8) {
            const u32 r = (8u * b8 + 4u * h) * PWLD;
            const float4 a = make_float4(gs[r + acol], gs[r + PWLD + acol], gs[r + 2 * PWLD + acol], gs[r + 3 * PWLD + acol]);
            const float4 bq = make_float4(xs[r + bcol], xs[r + PWLD + bcol], xs[r + 2 * PWLD + bcol], xs[r + 3 * PWLD + bcol]);
            acc = mfma4(a, bq, acc);
        }
    }
    // partial block, accumulator register v of lane l of wave w at (w * 16 + v) * 64 + l
    float *mine = part + ((size_t)pbase + sp) * (PWT * PWT);
    for (int v = 0; v < 16; ++v) mine[(w * 16 + v) * 64 + lane] = acc[v];
}

// second half: the partial blocks of a tile, added in run order, join the gradient
__device__ inline void param_w_reduce(const Tables &T, const PTile &pt, const float *part)
{
    const u32 nsp = (u32)pt.pad & 0xffu, pbase = (u32)pt.pad >> 8;
    const u32 slot = (u32)pt.param * 4u;
    const u32 start = T.pu_start[slot], end = T.pu_end[slot];
    if (start == end) return;
    const ParamDesc P = T.params[pt.param];
    const u32 m = (u32)P.rows, K = (u32)P.cols;
    const u32 i0 = (u32)pt.i0, j0 = (u32)pt.j0;
    const u32 all_chunks = (end - start + PWC - 1) / PWC;
    const u32 nsp_eff = all_chunks < nsp ? all_chunks : nsp;
    const float *all = part + (size_t)pbase * (PWT * PWT);
    // four consecutive entries of a partial block are four consecutive columns of one row; all loads of
    // a thread are issued before the first sum
    constexpr u32 PER = PWT * PWT / 4 / WG;   // float4 groups per thread
    float4 sum[PER];
#pragma unroll
    for (u32 g = 0; g < PER; ++g) sum[g] = ld4(all + 4u * (threadIdx.x + g * WG));
    for (u32 q = 1; q < nsp_eff; ++q) {
        float4 t[PER];
#pragma unroll
        for (u32 g = 0; g < PER; ++g) t[g] = ld4(all + (size_t)q * (PWT * PWT) + 4u * (threadIdx.x + g * WG));
#pragma unroll
        for (u32 g = 0; g < PER; ++g) { sum[g].x += t[g].x; sum[g].y += t[g].y; sum[g].z += t[g].z; sum[g].w += t[g].w; }
    }
#pragma unroll
    for (u32 g = 0; g < PER; ++g) {
        const u32 idx = 4u * (threadIdx.x + g * WG);
        const u32 l = idx & 63u, v = (idx >> 6) & 15u, ww = idx >> 10;
        const u32 rr = i0 + 32u * (ww >> 1) + 8u * (v >> 2) + 4u * (l >> 5) + (v & 3u);
        const u32 jj = j0 + 32u * (ww & 1u) + (l & 31u);
        if (rr >= m || jj >= K) continue;
        float *gp = P.grad + (size_t)rr * K + jj;
        if (jj + 3u < K && (((size_t)rr * K + jj) & 3u) == 0u) {
            float4 o = ld4(gp);
            o.x += sum[g].x; o.y += sum[g].y; o.z += sum[g].z; o.w += sum[g].w;
            st4(gp, o);
        } else {
            gp[0] += sum[g].x;
            if (jj + 1u < K) gp[1] += sum[g].y;
            if (jj + 2u < K) gp[2] += sum[g].z;
            if (jj + 3u < K) gp[3] += sum[g].w;
        }
    }
    if (threadIdx.x == 0) P.marks[0] = 1u;   // this parameter's gradient is dense now
}

// db[i] += sum over uses of g[i].  A tile is 256 rows (one per thread: a use's rows are one
// contiguous kilobyte) and one of PB_SPLIT equal runs of the parameter's use list; it leaves a
// partial sum, and the summing kernel adds the runs' partial sums in run order.
constexpr u32 PB_ROWS = 256;
constexpr u32 PB_UNROLL = 8;
__device__ inline void param_b_tile(const Tables &T, const PTile &pt, u32 sp, float *part)
{
    const u32 slot = (u32)pt.param * 4u + 1u;
    const u32 start = T.pu_start[slot], end = T.pu_end[slot];
    if (start == end) return;
    const ParamDesc P = T.params[pt.param];
    const u32 nsp = (u32)pt.pad & 0xffu, pbase = (u32)pt.pad >> 8;
    const u32 i = (u32)pt.i0 + threadIdx.x;
    const bool i_ok = i < (u32)P.rows;
    const u32 n_uses = end - start, per = (n_uses + nsp - 1) / nsp;
    const u32 lo = start + (sp * per < n_uses ? sp * per : n_uses), hi = start + ((sp + 1) * per < n_uses ? (sp + 1) * per : n_uses);
    float acc = 0.f;
    for (u32 it0 = lo; it0 < hi; it0 += PB_UNROLL) {
        float g[PB_UNROLL];
#pragma unroll
        for (u32 q = 0; q < PB_UNROLL; ++q) g[q] = (it0 + q < hi && i_ok) ? T.G[T.it_goff[it0 + q] + i] : 0.f;
#pragma unroll
        for (u32 q = 0; q < PB_UNROLL; q += 4) acc += (g[q] + g[q + 1]) + (g[q + 2] + g[q + 3]);
    }
    part[((size_t)pbase + sp) * PB_ROWS + threadIdx.x] = acc;
}

__device__ inline void param_b_reduce(const Tables &T, const PTile &pt, const float *part)
{
    const u32 slot = (u32)pt.param * 4u + 1u;
    if (T.pu_start[slot] == T.pu_end[slot]) return;
    const ParamDesc P = T.params[pt.param];
    const u32 nsp = (u32)pt.pad & 0xffu, pbase = (u32)pt.pad >> 8;
    const u32 i = (u32)pt.i0 + threadIdx.x;
    if (i < (u32)P.rows) {
        float s = 0.f;
        for (u32 q = 0; q < nsp; ++q) s += part[((size_t)pbase + q) * PB_ROWS + threadIdx.x];
        P.grad[i] += s;
    }
    if (threadIdx.x == 0) P.marks[0] = 1u;
}

// ------------------------------------------------------------------------------------------------
// backward pull: gradient of every node of a batch from its consumer edges
// ------------------------------------------------------------------------------------------------
// Consumer gradient at gradient-arena offset idx: from the fused chain's LDS copy (index idx + delta)
// when the descriptor says the consumer ran earlier in the same launch, else from the arena.
__device__ inline float ldg(const Tables &T, const lds_float *cl, bool from_lds, u32 delta, u32 idx)
{
    float v;
    if (from_lds) v = cl[(u32)(idx + delta)];
    else v = T.G[idx];
    return v;
}
__device__ inline float4 ldg4(const Tables &T, const lds_float *cl, bool from_lds, u32 delta, u32 idx)
{
    float4 v;
    if (from_lds) v = lds_ld4(cl + (u32)(idx + delta));
    else v = ld4(T.G + idx);
    return v;
}

// What the consumer's gradient is multiplied by, from the forward value y the edge names: 1 (plain and range
// edges), y (product), 1 - y^2 (tanh), y (1 - y) (logistic).  Every routine that evaluates such an edge forms
// gradient x factor with these and with separately rounded products and sums, so that a node's gradient does
// not depend on which routine its tile went through.
__device__ inline float mul_r(float a, float b)
{
#pragma clang fp contract(off)
    return a * b;
}
__device__ inline float add_r(float a, float b)
{
#pragma clang fp contract(off)
    return a + b;
}
__device__ inline float edge_factor(u32 kind, float y)
{
    const float ft = __builtin_fmaf(-y, y, 1.0f), fs = mul_r(y, 1.0f - y);
    float f = 1.0f;
    f = kind == (u32)EK_MUL ? y : f;
    f = kind == (u32)EK_DTANH ? ft : f;
    f = kind == (u32)EK_DSIGM ? fs : f;
    return f;
}
__device__ inline float4 edge_factor4(u32 kind, float4 y)
{
    return make_float4(edge_factor(kind, y.x), edge_factor(kind, y.y), edge_factor(kind, y.z), edge_factor(kind, y.w));
}

__device__ inline float edge_term(const Tables &T, const lds_float *cl, bool fl, u32 dl, u32 kind, u32 goff, u32 voff, i32 a0,
                                  i32 a1, u32 own, u32 col, bool resolved = false)
{
    switch (kind) {
    case EK_PLAIN: return ldg(T, cl, fl, dl, goff + col);
    case EK_RANGE: return ((i32)col >= a0 && (i32)col < a1) ? ldg(T, cl, fl, dl, goff + col - (resolved ? 0u : (u32)a0)) : 0.f;
    case EK_MUL:
    case EK_DTANH:
    case EK_DSIGM: return mul_r(ldg(T, cl, fl, dl, goff + col), edge_factor(kind, T.V[voff + col]));
    case EK_NLS: {   // a1: the row's dimension
        const float lse = T.V[voff] + T.V[own + (u32)a0];
        float p;
        if ((i32)col == a0) {
            // p_label - 1 as minus the sum of the other probabilities: no cancellation when p_label is close to 1
            // (eight logits are asked for at a time: one after the other, each would wait for memory in turn)
            float others = 0.f;
            for (i32 c0 = 0; c0 < a1; c0 += 8) {
                float xv[8];
#pragma unroll
                for (i32 k = 0; k < 8; ++k) xv[k] = T.V[own + (u32)(c0 + k < a1 ? c0 + k : a1 - 1)];
#pragma unroll
                for (i32 k = 0; k < 8; ++k)
                    if (c0 + k < a1 && c0 + k != a0) others += expf(xv[k] - lse);
            }
            p = -others;
        } else {
            p = expf(T.V[own + col] - lse);
        }
        return T.G[goff] * p;
    }
    case EK_SQN: return 2.0f * T.G[goff] * T.V[own + col];
    default: return 0.f;
    }
}

// four consecutive columns of one uniform edge (all offsets are multiples of 4; EK_NLS never is uniform)
__device__ inline float4 edge_term4(const Tables &T, const lds_float *cl, bool fl, u32 dl, u32 kind, u32 goff, u32 voff, i32 a0,
                                    i32 a1, u32 own, u32 col, bool resolved = false)
{
    const float4 z = make_float4(0.f, 0.f, 0.f, 0.f);
    switch (kind) {
    case EK_PLAIN: return ldg4(T, cl, fl, dl, goff + col);
    case EK_RANGE: return ((i32)col >= a0 && (i32)col < a1) ? ldg4(T, cl, fl, dl, goff + col - (resolved ? 0u : (u32)a0)) : z;
    case EK_MUL:
    case EK_DTANH:
    case EK_DSIGM: {
        const float4 g = ldg4(T, cl, fl, dl, goff + col), f = edge_factor4(kind, ld4(T.V + voff + col));
        return make_float4(mul_r(g.x, f.x), mul_r(g.y, f.y), mul_r(g.z, f.z), mul_r(g.w, f.w));
    }
    case EK_SQN: {
        const float g2 = 2.0f * T.G[goff];
        const float4 x = ld4(T.V + own + col);
        return make_float4(g2 * x.x, g2 * x.y, g2 * x.z, g2 * x.w);
    }
    default: return z;
    }
}

// four consecutive floats at an index that need not be a multiple of four
__device__ inline float4 ldu4(const float *base, u32 idx)
{
    if ((idx & 3u) == 0u) return ld4(base + idx);
    return make_float4(base[idx], base[idx + 1], base[idx + 2], base[idx + 3]);
}

// Columns col .. col + 3 of one consumer edge as it stands in the edge list (nothing resolved, any alignment):
// the arithmetic of edge_term, four columns at a time.
__device__ inline float4 edge_term4_any(const Tables &T, const EdgeRec &er, u32 own, u32 col)
{
    switch (er.kind) {
    case EK_PLAIN: return ldu4(T.G, er.goff + col);
    case EK_MUL:
    case EK_DTANH:
    case EK_DSIGM: {
        const float4 g = ldu4(T.G, er.goff + col), f = edge_factor4(er.kind, ldu4(T.V, er.voff + col));
        return make_float4(mul_r(g.x, f.x), mul_r(g.y, f.y), mul_r(g.z, f.z), mul_r(g.w, f.w));
    }
    default:   // a slice's range may cut the four columns, a label is one of them: column by column
        return make_float4(edge_term(T, nullptr, false, 0u, er.kind, er.goff, er.voff, er.a0, er.a1, own, col),
                           edge_term(T, nullptr, false, 0u, er.kind, er.goff, er.voff, er.a0, er.a1, own, col + 1u),
                           edge_term(T, nullptr, false, 0u, er.kind, er.goff, er.voff, er.a0, er.a1, own, col + 2u),
                           edge_term(T, nullptr, false, 0u, er.kind, er.goff, er.voff, er.a0, er.a1, own, col + 3u));
    }
}

__device__ inline void pull_tile(const Tables &T, const PullDesc &d, lds_float *cl, u32 tid, u32 nthr)
{
    const u32 total = d.nrows * d.d;
    const u32 root_pos = T.root_pos[0];
    const bool keep = (d.lflags & TF_OUT_LDS) != 0;
    if (d.n_uni != PULL_GENERIC && (d.vec4 & 1u)) {
        for (u32 x = tid * 4; x < total; x += nthr * 4) {
            const u32 dr = x / d.d, col = x % d.d, row = d.row0 + dr * d.rstride;
            const u32 own = d.val_off + row * d.d;
            const float seed = (d.pos0 + row == root_pos) ? 1.0f : 0.0f;   // a root has d == 1, never here
            float4 acc = make_float4(seed, seed, seed, seed);
            if (T.Gx) { const float4 e = ld4(T.Gx + own + col); acc.x += e.x; acc.y += e.y; acc.z += e.z; acc.w += e.w; }
#pragma unroll
            for (u32 j = 0; j < 4; ++j) {
                if (j < d.n_uni) {
                    const UEdge ue = d.e[j];
                    const float4 t = edge_term4(T, cl, (d.lflags & (TF_SRC_LDS << j)) != 0, 0u, ue.kind,
                                                ue.goff + dr * ue.gs, ue.voff + dr * ue.vs, ue.a0, ue.a1, own, col, true);
                    acc.x = add_r(acc.x, t.x); acc.y = add_r(acc.y, t.y); acc.z = add_r(acc.z, t.z); acc.w = add_r(acc.w, t.w);
                }
            }
            st4(T.G + own + col, acc);
            if (keep) lds_st4(cl + (u32)(own + col + d.lds_out), acc);
        }
        return;
    }
    if (d.n_uni == PULL_GENERIC && (d.d & 3u) == 0u) {
        // rows whose consumer edges differ, four columns per thread: what is looked up per row (the node, its
        // edge range, the edge records) is looked up once for four columns, and the columns come as float4
        for (u32 x = tid * 4; x < total; x += nthr * 4) {
            const u32 dr = x / d.d, col = x % d.d, row = d.row0 + dr * d.rstride;
            const u32 own = d.val_off + row * d.d;
            float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);        // (a root has one column, never here)
            if (T.Gx) acc = ld4(T.Gx + own + col);
            const u32 u = T.order[d.pos0 + row];
            const u32 ownv = (d.vec4 & 2u) ? T.val_off[u] : own;
            const u32 q1 = T.succ_off[u + 1];
            for (u32 q = T.succ_off[u]; q < q1; ++q) {
                const EdgeRec er = T.edges[q];
                const float4 t = edge_term4_any(T, er, ownv, col);
                acc.x = add_r(acc.x, t.x); acc.y = add_r(acc.y, t.y); acc.z = add_r(acc.z, t.z); acc.w = add_r(acc.w, t.w);
            }
            st4(T.G + own + col, acc);
            if (keep) {
                lds_float *o = cl + (u32)(own + col + d.lds_out);
                o[0] = acc.x; o[1] = acc.y; o[2] = acc.z; o[3] = acc.w;
            }
        }
        return;
    }
    for (u32 x = tid; x < total; x += nthr) {
        const u32 dr = x / d.d, col = x % d.d, row = d.row0 + dr * d.rstride;
        const u32 own = d.val_off + row * d.d;
        float acc = (d.pos0 + row == root_pos) ? 1.0f : 0.0f;
        if (T.Gx) acc += T.Gx[own + col];     // what consumers in later evaluation stages passed down
        if (d.n_uni != PULL_GENERIC) {
#pragma unroll
            for (u32 j = 0; j < 4; ++j) {
                if (j < d.n_uni) {
                    const UEdge ue = d.e[j];
                    acc = add_r(acc, edge_term(T, cl, (d.lflags & (TF_SRC_LDS << j)) != 0, 0u, ue.kind, ue.goff + dr * ue.gs,
                                     ue.voff + dr * ue.vs, ue.a0, ue.a1, own, col, true));
                }
            }
        } else {
            const u32 u = T.order[d.pos0 + row];
            const u32 ownv = (d.vec4 & 2u) ? T.val_off[u] : own;   // a view's own values lie in its operand's row
            const u32 q1 = T.succ_off[u + 1];
            for (u32 q = T.succ_off[u]; q < q1; ++q) {
                const EdgeRec er = T.edges[q];
                acc = add_r(acc, edge_term(T, cl, false, 0u, er.kind, er.goff, er.voff, er.a0, er.a1, ownv, col));
            }
        }
        T.G[own + col] = acc;
        if (keep) cl[(u32)(own + col + d.lds_out)] = acc;
    }
}

// The tile of a fused backward run as it nearly always is: every row has the same (at most four) consumer
// edges up to constant row strides, of the kinds that need one gradient and at most one forward value per
// column, and the columns go by fours (bit 2 of the descriptor's vec4 field; its edges are stored resolved).
// A level of a run is one such tile per wave, so what a level costs is the number of instructions this
// routine issues: the descriptor comes in twelve 16-byte LDS reads asked for together, control values go to
// scalar registers, a tile of one row per thread block (the usual case) needs no row arithmetic, absent
// edges are skipped, and everything the thread's columns need is asked for before any of it is used.
// d must lie in LDS.
typedef u32 vec4u __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) const vec4u lds_vec4u;
__device__ inline uint4 lds_q(const PullDesc &d, u32 k)
{
    const vec4u t = ((lds_vec4u *)(&d))[k];
    return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ inline u32 sreg(u32 v) { return __builtin_amdgcn_readfirstlane(v); }

// One or two edges of such a tile: loads first, sums after.
template <u32 J0, u32 NJ>
__device__ inline void pull_uni4_edges(const Tables &T, const uint4 *q, lds_float *cl, u32 n_uni, u32 lflags, bool one_row, u32 dr,
                                       u32 col, float4 &acc)
{
    float4 g[NJ], v[NJ];
    u32 kind[NJ];
#pragma unroll
    for (u32 jj = 0; jj < NJ; ++jj) {
        const u32 j = J0 + jj;
        if (j < n_uni) {
            const uint4 ea = q[2 + 2 * j], eb = q[3 + 2 * j];   // kind, goff, voff, gs | vs, a0, a1, dl
            kind[jj] = sreg(ea.x);
            u32 gi = ea.y + col, vi = ea.z + col;
            if (!one_row) { gi += dr * ea.w; vi += dr * eb.x; }
            if (kind[jj] >= (u32)EK_MUL) v[jj] = ld4(T.V + vi);
            const bool in = kind[jj] != (u32)EK_RANGE || (col >= eb.y && col < eb.z);
            g[jj] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (lflags & (TF_SRC_LDS << j)) { if (in) g[jj] = lds_ld4(cl + gi); }
            else if (in) g[jj] = ld4(T.G + gi);
        }
    }
#pragma unroll
    for (u32 jj = 0; jj < NJ; ++jj) {
        if (J0 + jj < n_uni) {
            float4 t = g[jj];
            if (kind[jj] >= (u32)EK_MUL) {
                const float4 f = edge_factor4(kind[jj], v[jj]);
                t = make_float4(mul_r(t.x, f.x), mul_r(t.y, f.y), mul_r(t.z, f.z), mul_r(t.w, f.w));
            }
            acc.x = add_r(acc.x, t.x); acc.y = add_r(acc.y, t.y); acc.z = add_r(acc.z, t.z); acc.w = add_r(acc.w, t.w);
        }
    }
}

// q: the tile's descriptor as its twelve 16-byte words, already asked for by the caller
__device__ inline void pull_tile_uni4(const Tables &T, const uint4 *q, lds_float *cl, u32 tid, u32 nthr)
{
    const u32 dd = q[0].z, n_uni = sreg(q[1].z), nrows = sreg(q[1].w), lflags = sreg(q[10].w);
    const u32 lds_out = q[11].x, dshift = sreg(q[11].y), own0 = q[11].z, rowstep = q[11].w;
    const bool one_row = nrows == 1u;
    const u32 total = one_row ? dd : nrows << dshift;
    const float *Gx = T.Gx;
    for (u32 x = tid * 4u; x < total; x += nthr * 4u) {
        u32 dr = 0, col = x;
        if (!one_row) { dr = x >> dshift; col = x & (dd - 1u); }
        const u32 own = own0 + col + (one_row ? 0u : dr * rowstep);
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        if (Gx) acc = ld4(Gx + own);
        pull_uni4_edges<0, 2>(T, q, cl, n_uni, lflags, one_row, dr, col, acc);
        if (n_uni > 2u) pull_uni4_edges<2, 2>(T, q, cl, n_uni, lflags, one_row, dr, col, acc);
        st4(T.G + own, acc);
        if (lflags & TF_OUT_LDS) lds_st4(cl + (u32)(own + lds_out), acc);
    }
}

// ------------------------------------------------------------------------------------------------
// kernels
// ------------------------------------------------------------------------------------------------
template <bool XP>
__device__ inline void run_fwd_tile(const Tables &T, const TileDesc &d, float *lds)
{
    switch (d.op) {
    case OP_MATVEC: matvec_fwd_tile<XP>(T, d, lds); break;
    case OP_PICK_NLS:
    case OP_SQNORM: red_fwd_tile(T, d); break;
    case OP_ADD:
        if (d.arity >= (u32)WIDE_ADD_ARITY) { wide_add_tile(T, d, lds); break; }
        ew_fwd_tile(T, d, (lds_float *)lds, threadIdx.x, WG);
        break;
    default: ew_fwd_tile(T, d, (lds_float *)lds, threadIdx.x, WG); break;
    }
}

constexpr u32 RUN_STAGE = RUN_STAGE_DESCS;   // descriptors of a fused run staged in LDS at a time

// Barrier between two depths of a fused run.  When every result the next depth needs from this
// launch is handed on through LDS, only the LDS writes have to be complete (the global copies
// of the results are not waited for); otherwise the full workgroup barrier orders the global
// stores and loads as well.
__device__ inline void run_barrier(bool heavy)
{
    if (heavy) __syncthreads();
    else asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
}

// Copies n descriptors of W words (a multiple of 4) from global memory to LDS.  All loads of a
// thread are issued before the first is waited for.
template <u32 W, u32 NT>
__device__ inline void stage_descriptors(const void *src, void *dst, u32 n)
{
    static_assert(W % 4 == 0 && RUN_STAGE * W / 4 <= 2 * NT, "two float4 per thread cover a stage");
    const uint4 *s4 = reinterpret_cast<const uint4 *>(src);
    uint4 *d4 = reinterpret_cast<uint4 *>(dst);
    const u32 n4 = n * (W / 4), x0 = threadIdx.x, x1 = threadIdx.x + NT;
    uint4 v0 = make_uint4(0, 0, 0, 0), v1 = v0;
    if (x0 < n4) v0 = s4[x0];
    if (x1 < n4) v1 = s4[x1];
    if (x0 < n4) d4[x0] = v0;
    if (x1 < n4) d4[x1] = v1;
}

// One launch = one slot.  A work item is a run of tiles that one workgroup executes in order.
// Runs of one tile (GEMM, reduction and single-batch tiles) keep their descriptor in scalar
// registers.  Longer runs are fused chains of group-aligned component-wise batches over one block
// of groups: the descriptors are staged in LDS with one coalesced load, tiles of the same depth
// are spread over the four waves, and a workgroup barrier separates depths.  The LDS array is the
// GEMM tiles' reduction space or the fused run's copy of its own results, whichever is running.
// run_len != 0: every work item of the launch has run_len tiles, item w starts at tile
// tile_lo + (w - work_lo) * run_len and the work records are not read.
extern __shared__ __align__(16) float dyn_lds[];   // sized per launch: GEMM reduction space or a fused chain's copy

// KIND: FWD_ANY every kind of tile; FWD_LEAN the launch holds component-wise work only (this instantiation
// carries no GEMM or reduction code, needs half the registers and keeps twice the waves per CU); FWD_XP every
// kind, and the products may read their operand rows in pieces.
enum : int { FWD_ANY = 0, FWD_LEAN = 1, FWD_XP = 2 };
template <int KIND>
__global__ __launch_bounds__(WG, KIND == FWD_LEAN ? 6 : 3) void k_fwd_step(u32 work_lo, u32 work_hi, u32 tile_lo, u32 run_len,
                                                                const TileDesc *tiles_f, const WorkRec *works_f, Tables T)
{
    // the leading arguments arrive in scalar registers with the wave (so the descriptor loads start
    // at once); the table of pointers behind them is read from the argument block
    float *lds = dyn_lds;
    __shared__ __align__(16) TileDesc sdesc[RUN_STAGE];
    const u32 lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    for (u32 w = work_lo + blockIdx.x; w < work_hi; w += gridDim.x) {
        WorkRec wr;
        if (run_len) { wr.first = tile_lo + (w - work_lo) * run_len; wr.len = run_len; }
        else wr = works_f[w];
        if (wr.len == 1) {
            const TileDesc d = tiles_f[wr.first];
            if (KIND == FWD_LEAN) ew_fwd_tile(T, d, (lds_float *)lds, threadIdx.x, WG);
            else run_fwd_tile<KIND == FWD_XP>(T, d, lds);
            continue;
        }
        for (u32 c0 = 0; c0 < wr.len; c0 += RUN_STAGE) {
            const u32 cn = wr.len - c0 < RUN_STAGE ? wr.len - c0 : RUN_STAGE;
            __syncthreads();
            stage_descriptors<sizeof(TileDesc) / 4, WG>(tiles_f + wr.first + c0, sdesc, cn);
            __syncthreads();
            const bool heavy = __ballot(lane < cn && (sdesc[lane < cn ? lane : 0].flags & TF_GLOBAL_DEP)) != 0ull;
            u32 i = 0;
            while (i < cn) {
                u32 glen = __builtin_amdgcn_readfirstlane(sdesc[i].contig) >> 16;
                if (glen == 0) glen = 1;
                if (glen > cn - i) glen = cn - i;   // a depth group cut by the staging window: still same depth
                if (glen == 1) ew_fwd_tile(T, sdesc[i], (lds_float *)lds, threadIdx.x, WG);
                else for (u32 t = i + wave; t < i + glen; t += WG / 64) ew_fwd_tile(T, sdesc[t], (lds_float *)lds, lane, 64);
                i += glen;
                if (i < cn) run_barrier(heavy);
            }
        }
        __syncthreads();   // the LDS copy is free for the next work item
    }
}

// One backward launch: the slot's dX tiles (blocks first: they run longest) and its pull work
// items.  Both kinds may share a launch only when no dX tile reads a gradient that this slot's
// pull computes; otherwise the host launches the pull range and the dX range one after the other.
constexpr int BWD_THREADS = DX_WAVES * 64;
template <bool LEAN>
__global__ __launch_bounds__(BWD_THREADS, 4) void k_bwd_step(u32 work_lo, u32 work_hi, u32 tile_lo, u32 run_len,
                                                                        u32 dx_lo, u32 dx_hi, const PullDesc *tiles_a,
                                                                        const WorkRec *works_a, const TileDesc *tiles_b, Tables T)
{
    float *lds = dyn_lds;
    __shared__ __align__(16) PullDesc sdesc[RUN_STAGE];
    const u32 lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const u32 n_dx = dx_hi - dx_lo, n_items = n_dx + (work_hi - work_lo);
    float sink = 0.f;   // keeps the early requests of a run alive; never stored
    for (u32 item = blockIdx.x; item < n_items; item += gridDim.x) {
        if (!LEAN && item < n_dx) {
            const TileDesc d = tiles_b[dx_lo + item];
            matvec_dx_tile(T, d, lds);
            continue;
        }
        const u32 w = work_lo + (item - n_dx);
        WorkRec wr;
        if (run_len) { wr.first = tile_lo + (w - work_lo) * run_len; wr.len = run_len; }
        else { wr = works_a[w]; wr.first = sreg(wr.first); wr.len = sreg(wr.len); }
        if (wr.len == 1) {
            const PullDesc d = tiles_a[wr.first];
            pull_tile(T, d, (lds_float *)lds, threadIdx.x, BWD_THREADS);
            continue;
        }
        for (u32 c0 = 0; c0 < wr.len; c0 += RUN_STAGE) {
            const u32 cn = wr.len - c0 < RUN_STAGE ? wr.len - c0 : RUN_STAGE;
            __syncthreads();
            stage_descriptors<sizeof(PullDesc) / 4, BWD_THREADS>(tiles_a + wr.first + c0, sdesc, cn);
            __syncthreads();
            const bool heavy = __ballot(lane < cn && (sdesc[lane < cn ? lane : 0].lflags & TF_GLOBAL_DEP)) != 0ull;
            // Every level of a run reads forward values (and gradients from outside the run) that no
            // level before it touches: ask for all of them now, one lane per 128-byte line, so the
            // levels find them in the cache instead of each waiting for memory in turn.  Nothing waits
            // for these loads themselves: their sum is taken when the run is over.
            float early[4] = {0.f, 0.f, 0.f, 0.f};
            if (LEAN) {   // (runs are rare in launches that also hold GEMM tiles, and that instantiation has no registers to spare)
#pragma unroll
                for (u32 h = 0; h < 2; ++h) {
                    const u32 x = threadIdx.x + h * BWD_THREADS;
                    if (x < cn * 32u) {
                        const PullDesc &pd = sdesc[x >> 5];
                        const u32 j = (x >> 3) & 3u, el = (x & 7u) * 32u;
                        if (pd.n_uni != PULL_GENERIC && j < pd.n_uni && el < pd.nrows * pd.d) {
                            const UEdge ue = pd.e[j];
                            const u32 dr = el / pd.d, col = el % pd.d;
                            const bool uses_v = ue.kind == EK_MUL || ue.kind == EK_DTANH || ue.kind == EK_DSIGM;
                            const bool far_g = !(pd.lflags & (TF_SRC_LDS << j)) && (ue.kind == EK_PLAIN || uses_v);
                            if (uses_v) early[2 * h] = T.V[ue.voff + dr * ue.vs + col];
                            if (far_g) early[2 * h + 1] = T.G[ue.goff + dr * ue.gs + col];
                        }
                    }
                }
            }
            // Tiles of one level are spread over the waves: with fewer than eight of them a tile is cut
            // into parts (8 / tiles, rounded down), one wave each.  Where the levels start is found once,
            // as a bit mask over the staged tiles (a tile starts a level when the one before it ends one).
            unsigned long long starts =
                __ballot(lane < cn && (lane == 0u || sdesc[lane == 0u || lane >= cn ? 0u : lane - 1u].grp_len <= 1u));
            u32 i = 0;
            while (i < cn) {
                starts &= starts - 1ull;
                const u32 next = starts ? (u32)__builtin_ctzll(starts) : cn;
                const u32 glen = next - i;
                const u32 g8 = glen < 8u ? glen : 8u;
                const u32 parts = g8 == 1u ? 8u : g8 == 2u ? 4u : g8 <= 4u ? 2u : 1u;
                u32 part = 0, tw = wave;
                if (g8 == 1u) { part = wave; tw = 0; }
                else while (tw >= g8) { tw -= g8; ++part; }
                if (part < parts) {
                    for (u32 t = i + tw; t < next; t += BWD_THREADS / 64) {
                        const PullDesc &d = sdesc[t];
                        if (LEAN) {   // (the instantiation with the GEMM tiles has no registers to spare for the short routine)
                            uint4 q[12];
#pragma unroll
                            for (u32 k = 0; k < 12; ++k) q[k] = lds_q(d, k);
                            if (sreg(q[10].z) & 4u) { pull_tile_uni4(T, q, (lds_float *)lds, part * 64u + lane, parts * 64u); continue; }
                        }
                        pull_tile(T, d, (lds_float *)lds, part * 64u + lane, parts * 64u);
                    }
                }
                i = next;
                if (i < cn) run_barrier(heavy);
            }
            sink += (early[0] + early[1]) + (early[2] + early[3]);
        }
        __syncthreads();
    }
    if (sink != sink && work_lo == 0xffffffffu) T.G[0] = sink;   // (no launch has this range)
}

__global__ void k_set_root(Tables T) { T.root_pos[0] = T.root == 0xffffffffu ? 0xffffffffu : T.pos_of[T.root]; }   // (no root in this graph: nothing is seeded)

// Workgroup g runs on XCD g % 8 and the tile list is ordered so that tile t belongs on XCD t % 8 (an
// XCD then keeps to one eighth of the gradient columns, which fit its L2): the runs of a tile are
// therefore a multiple of eight workgroups apart.
// (the workgroups behind the dW ones take the bias tiles: PB_SPLIT consecutive workgroups per tile)
__global__ __launch_bounds__(WG) void k_param_w(Tables T, const PTile *tiles, u32 n_tiles, u32 n_tiles_pad, float *part,
                                                const PTile *btiles, float *bpart)
{
    __shared__ __align__(16) float lds[PW_LDS_FLOATS];
    const u32 w_blocks = n_tiles_pad * PW_SPLIT_MAX;
    if (blockIdx.x >= w_blocks) {
        const u32 x = blockIdx.x - w_blocks;
        param_b_tile(T, btiles[x / PB_SPLIT], x % PB_SPLIT, bpart);
        return;
    }
    const u32 tile = blockIdx.x % n_tiles_pad, sp = blockIdx.x / n_tiles_pad;
    if (tile >= n_tiles) return;
    param_w_tile(T, tiles[tile], lds, sp, part);
}

__global__ __launch_bounds__(WG) void k_param_w_sum(Tables T, const PTile *tiles, u32 n_tiles, const float *part, const PTile *btiles,
                                                    const float *bpart)
{
    if (blockIdx.x >= n_tiles) { param_b_reduce(T, btiles[blockIdx.x - n_tiles], bpart); return; }
    param_w_reduce(T, tiles[blockIdx.x], part);
}

// dE[row, :] += sum of the gradients of every LOOKUP of (table, row): one wave per run of equal
// keys in the sorted item list, rows summed in sorted (= schedule) order
__global__ __launch_bounds__(WG) void k_param_e(Tables T, u32 n_items)
{
    const int lane = threadIdx.x & 63;
    const u32 wave = (blockIdx.x * WG + threadIdx.x) >> 6;
    const u32 n_waves = (gridDim.x * WG) >> 6;
    for (u32 i = wave; i < n_items; i += n_waves) {
        const u64 k = T.it_key[i];
        const u32 slot = (u32)(k >> 32);
        if ((slot & 3u) != 2u) continue;
        if (i > 0 && T.it_key[i - 1] == k) continue;
        const ParamDesc P = T.params[slot >> 2];
        const u32 rowi = (u32)k;
        u32 end = i + 1;
        while (end < n_items && T.it_key[end] == k) ++end;
        for (u32 c = lane; c < (u32)P.cols; c += 64) {
            float acc = 0.f;
            for (u32 it = i; it < end; ++it) acc += T.G[T.it_goff[it] + c];
            P.grad[(size_t)rowi * P.cols + c] += acc;
        }
        // list the row for the update (once, however many minibatches add to it before the next clearing)
        if (lane == 0 && atomicExch(&P.row_flag[rowi], 1u) == 0u) P.touched[atomicAdd(&P.marks[1], 1u)] = rowi;
    }
}

// theta <- theta - lr * gradient for every parameter (blockIdx.y = parameter); with zero_grad the
// gradient is cleared in the same pass, ready for the next minibatch (zero_grad == 2: only clear).
// A parameter that only LOOKUPs have added to since its gradient was last cleared (an embedding
// table) is walked by its touched rows, one workgroup per row: every other row has gradient zero,
// so leaving it alone gives the same bits as the dense update (Section 2's update line touches the
// parameters an instance used).  k_sgd_reset then empties the lists.
__global__ __launch_bounds__(WG) void k_sgd(const ParamDesc *params, float lr, int zero_grad)
{
    const ParamDesc P = params[blockIdx.y];
    const size_t count = (size_t)P.rows * P.cols;
    if (P.marks[0]) {
        if (zero_grad == 2) {
            for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < count; i += (size_t)gridDim.x * WG) P.grad[i] = 0.f;
            return;
        }
        for (size_t i = (size_t)blockIdx.x * WG + threadIdx.x; i < count; i += (size_t)gridDim.x * WG) {
            P.data[i] -= lr * P.grad[i];
            if (zero_grad) P.grad[i] = 0.f;
        }
        return;
    }
    const u32 nt = P.marks[1];
    for (u32 t = blockIdx.x; t < nt; t += gridDim.x) {
        const size_t base = (size_t)P.touched[t] * P.cols;
        for (u32 c = threadIdx.x; c < (u32)P.cols; c += WG) {
            if (zero_grad != 2) P.data[base + c] -= lr * P.grad[base + c];
            if (zero_grad) P.grad[base + c] = 0.f;
        }
    }
}

// after k_sgd with zero_grad: the gradients are zero again, so no row is touched and nothing is dense
__global__ __launch_bounds__(WG) void k_sgd_reset(const ParamDesc *params)
{
    const ParamDesc P = params[blockIdx.x];
    const u32 nt = P.marks[1];
    if (P.marks[0]) {   // (a dense gradient may hide touched rows beyond the list's reach: clear every flag)
        for (u32 r = threadIdx.x; r < (u32)P.rows; r += WG) P.row_flag[r] = 0u;
    } else {
        for (u32 t = threadIdx.x; t < nt; t += WG) P.row_flag[P.touched[t]] = 0u;
    }
    __syncthreads();
    if (threadIdx.x == 0) { P.marks[0] = 0u; P.marks[1] = 0u; }
}

__global__ void k_gather_all(Tables T, const float *src, const u32 *src_off, float *dst, const u32 *dst_off)
{
    const u32 v = blockIdx.x;
    const u32 d = T.out_dim[v];
    const float *s = src + src_off[v];
    float *o = dst + dst_off[v];
    for (u32 c = threadIdx.x; c < d; c += blockDim.x) o[c] = s[c];
}

// Rows of the CONCAT batches that the forward pass left uncopied (TF_VIRT), written when somebody outside the
// forward pass asks for values: one workgroup per node, the operands' rows copied side by side.
__global__ void k_fill_uncopied(Tables T)
{
    const u32 v = blockIdx.x;
    if (T.op[v] != OP_CONCAT) return;
    if (!(T.batches[T.batch_of_pos[T.pos_of[v]]].vec4 & TF_VIRT)) return;
    float *o = T.V + T.val_off[v];
    for (u32 e = T.in_off[v]; e < T.in_off[v + 1]; ++e) {
        const u32 u = T.in_idx[e];
        const u32 d = T.out_dim[u];
        const float *s = T.V + T.val_off[u];
        for (u32 c = threadIdx.x; c < d; c += blockDim.x) o[c] = s[c];
        o += d;
    }
}

// Values of already evaluated nodes, copied into the payload block of a later evaluation stage
// whose graph holds them as leaves: entry i copies dim[i] elements from the row of node src[i] in
// the earlier evaluation's value arena to payload + dst[i].
__global__ void k_stage_fill(const float *V, const u32 *val_off, const u32 *src, const u32 *dst, const u32 *dim,
                             float *payload)
{
    const u32 i = blockIdx.x;
    const float *s = V + val_off[src[i]];
    float *o = payload + dst[i];
    const u32 d = dim[i];
    for (u32 c = threadIdx.x; c < d; c += blockDim.x) o[c] = s[c];
}

__global__ __launch_bounds__(WG) void k_test_gemm(const float *A, const float *Bm, float *C, int M, int N, int K)
{
    __shared__ float lds[LDS_FLOATS];
    const u32 ntn = (N + GT - 1) / GT;
    const u32 r0 = (blockIdx.x / ntn) * GT, i0 = (blockIdx.x % ntn) * GT;
    const u32 Ku = (u32)K;
    const u32 row = r0 + (threadIdx.x & 31);
    const bool row_ok = row < (u32)M;
    XRow xr;
    xr.o0 = xr.o1 = xr.o2 = xr.o3 = (row_ok ? row : 0u) * Ku;
    XCuts xc;
    xc.c0 = xc.c1 = xc.c2 = 0xffffffffu;
    gemm_nt_tile<false>(A, xr, xc, row_ok, (u32)M, Bm, nullptr, (u32)N, Ku, (Ku & 3u) == 0, C, r0, i0, lds);
}

inline u32 grid_for(u32 tiles, u32 cap) { return tiles < cap ? tiles : cap; }
constexpr u32 GRID_CAP = 4096;

}  // namespace

// ---- host side -----------------------------------------------------------------------------------

// run length to pass to a step kernel: the slot's common tiles-per-work-item count, or 0 when its
// chains differ (the kernel then reads each work item's record)
static inline u32 slot_run_len(const SlotRec &r) { return r.lmin == ~r.nlmax ? r.lmin : 0u; }
static inline u32 slot_run_len_fwd(const SlotRec &r) { return r.lminf == ~r.nlmaxf ? r.lminf : 0u; }

// dynamic LDS of a step launch: the slot's fused chains' need, at least the GEMM reduction space
constexpr size_t FWD_LDS_MIN = (size_t)(WIDE_LDS_FLOATS > (u32)LDS_FLOATS ? WIDE_LDS_FLOATS : (u32)LDS_FLOATS) * 4;   // staged wide tile / accumulator blocks
constexpr size_t BWD_LDS_MIN = (size_t)DX_WAVES * 16 * 64 * 4;         // eight waves' blocks of a wide dX tile
static inline size_t slot_lds_bytes(const SlotRec &r, size_t floor_bytes)
{
    const size_t need = (size_t)r.lds_need * 4;
    return need > floor_bytes ? need : floor_bytes;
}

// the step kernels may ask for a full fused-chain copy (64 KB) on top of their static descriptor
// stage: raise their dynamic-LDS limit once per process
static hipError_t allow_large_dynamic_lds()
{
    static hipError_t result = [] {
        const int bytes = (int)(CHAIN_LDS_FLOATS * 4);
        const void *kernels[5] = {(const void *)k_fwd_step<FWD_ANY>, (const void *)k_fwd_step<FWD_LEAN>,
                                  (const void *)k_fwd_step<FWD_XP>,
                                  (const void *)k_bwd_step<false>, (const void *)k_bwd_step<true>};
        hipError_t e = hipSuccess;
        for (const void *k : kernels)
            if (e == hipSuccess) e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
        return e;
    }();
    return result;
}

static int launch_forward_steps(ob_ctx *ctx)
{
    HIP_TRY(ctx, allow_large_dynamic_lds());
    const Tables &T = ctx->T;
    hipStream_t s = ctx->stream;
    const u32 ns = ctx->hdr.n_slots;
    for (u32 st = 0; st < ns; ++st) {
        const SlotRec &r = ctx->slots[st];
        const u32 lo = r.wf, hi = ctx->slots[st + 1].wf;
        if (hi > lo) {
            if (r.plain & 1u)
                hipLaunchKernelGGL(k_fwd_step<FWD_LEAN>, dim3(grid_for(hi - lo, GRID_CAP)), dim3(WG), slot_lds_bytes(r, 16), s,
                                   lo, hi, r.tf, slot_run_len_fwd(r), T.tiles_f, T.works_f, T);
            else if (r.plain & 2u)
                hipLaunchKernelGGL(k_fwd_step<FWD_ANY>, dim3(grid_for(hi - lo, GRID_CAP)), dim3(WG),
                                   slot_lds_bytes(r, FWD_LDS_MIN), s, lo, hi, r.tf, slot_run_len_fwd(r), T.tiles_f, T.works_f, T);
            else   // a product of the slot reads its operand rows in pieces
                hipLaunchKernelGGL(k_fwd_step<FWD_XP>, dim3(grid_for(hi - lo, GRID_CAP)), dim3(WG),
                                   slot_lds_bytes(r, FWD_LDS_MIN), s, lo, hi, r.tf, slot_run_len_fwd(r), T.tiles_f, T.works_f, T);
            ++ctx->n_launch_fwd;
        }
    }
    return 0;
}

static int launch_backward_steps(ob_ctx *ctx)
{
    HIP_TRY(ctx, allow_large_dynamic_lds());
    const Tables &T = ctx->T;
    hipStream_t s = ctx->stream;
    const u32 ns = ctx->hdr.n_slots;
    hipLaunchKernelGGL(k_set_root, dim3(1), dim3(1), 0, s, T);
    ++ctx->n_launch_bwd;
    const int before_steps = ctx->n_launch_bwd;
    for (u32 st = ns; st-- > 0;) {
        const SlotRec &r = ctx->slots[st], &e = ctx->slots[st + 1];
        const u32 n_pull = e.wa - r.wa, n_dx = e.tb - r.tb;
        const size_t lds_bytes = slot_lds_bytes(r, BWD_LDS_MIN);
        // (with gradients arriving from later stages a product's gradient is no longer its one consumer's row:
        // the dX tiles then read the rows the slot's own pull has just written)
        if (n_pull && n_dx && r.dx_free && !T.Gx) {
            hipLaunchKernelGGL(k_bwd_step<false>, dim3(grid_for(n_pull + n_dx, GRID_CAP)), dim3(BWD_THREADS), lds_bytes, s,
                               r.wa, e.wa, r.ta, slot_run_len(r), r.tb, e.tb, T.tiles_a, T.works_a, T.tiles_b, T);
            ++ctx->n_launch_bwd;
            continue;
        }
        if (n_pull) {
            hipLaunchKernelGGL(k_bwd_step<true>, dim3(grid_for(n_pull, GRID_CAP)), dim3(BWD_THREADS), slot_lds_bytes(r, 16), s,
                               r.wa, e.wa, r.ta, slot_run_len(r), 0u, 0u, T.tiles_a, T.works_a, T.tiles_b, T);
            ++ctx->n_launch_bwd;
        }
        if (n_dx) {
            hipLaunchKernelGGL(k_bwd_step<false>, dim3(grid_for(n_dx, GRID_CAP)), dim3(BWD_THREADS), BWD_LDS_MIN, s, 0u, 0u,
                               0u, 0u, r.tb, e.tb, T.tiles_a, T.works_a, T.tiles_b, T);
            ++ctx->n_launch_bwd;
        }
    }
    ctx->n_launch_bwd_steps = ctx->n_launch_bwd - before_steps;
    return 0;
}

static int launch_param_grads(ob_ctx *ctx)
{
    const Tables &T = ctx->T;
    hipStream_t s = ctx->stream;
    if (ctx->hdr.n_items == 0) return 0;
    if (!ctx->wtiles.empty() || !ctx->btiles.empty()) {
        const u32 n_tiles = (u32)ctx->wtiles.size(), n_pad = (n_tiles + 7u) & ~7u, n_b = (u32)ctx->btiles.size();
        hipLaunchKernelGGL(k_param_w, dim3(n_pad * PW_SPLIT_MAX + n_b * PB_SPLIT), dim3(WG), 0, s, T, ctx->wtiles_dev, n_tiles, n_pad,
                           ctx->wpart_dev, ctx->btiles_dev, ctx->bpart_dev);
        hipLaunchKernelGGL(k_param_w_sum, dim3(n_tiles + n_b), dim3(WG), 0, s, T, ctx->wtiles_dev, n_tiles,
                           (const float *)ctx->wpart_dev, ctx->btiles_dev, (const float *)ctx->bpart_dev);
        ctx->n_launch_bwd += 2;
    }
    u32 blocks = (ctx->hdr.n_items + 3) / 4;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_param_e, dim3(blocks), dim3(WG), 0, s, T, ctx->hdr.n_items);
    ++ctx->n_launch_bwd;
    return 0;
}

// Runs `body` either directly on the stream or captured into a hipGraph that is instantiated
// and launched once (the graph differs per minibatch, so building it is part of the cost).
template <typename F>
static int run_maybe_graph(ob_ctx *ctx, hipGraph_t *graph, hipGraphExec_t *gexec, F body)
{
    if (ctx->launch != 1) return body();
    if (!ctx->stream) return ctx_fail(ctx, -6, "hipGraph launch needs a stream other than the default stream");
    auto t0 = std::chrono::steady_clock::now();
    if (*gexec) { HIP_TRY(ctx, hipGraphExecDestroy(*gexec)); *gexec = nullptr; }
    if (*graph) { HIP_TRY(ctx, hipGraphDestroy(*graph)); *graph = nullptr; }
    HIP_TRY(ctx, hipStreamBeginCapture(ctx->stream, hipStreamCaptureModeThreadLocal));
    int rc = body();
    hipError_t e = hipStreamEndCapture(ctx->stream, graph);
    if (rc) return rc;
    HIP_TRY(ctx, e);
    HIP_TRY(ctx, hipGraphInstantiate(gexec, *graph, nullptr, nullptr, 0));
    auto t1 = std::chrono::steady_clock::now();
    ctx->ms_graph += std::chrono::duration<float, std::milli>(t1 - t0).count();
    HIP_TRY(ctx, hipGraphLaunch(*gexec, ctx->stream));
    return 0;
}

int exec_forward(ob_ctx *ctx)
{
    ctx->n_launch_fwd = 0;
    int rc = run_maybe_graph(ctx, &ctx->graph_fwd, &ctx->gexec_fwd, [ctx]() { return launch_forward_steps(ctx); });
    if (rc) return rc;
    HIP_TRY(ctx, hipGetLastError());
    return 0;
}

int exec_backward(ob_ctx *ctx)
{
    ctx->n_launch_bwd = 0;
    int rc = run_maybe_graph(ctx, &ctx->graph_bwd, &ctx->gexec_bwd, [ctx]() {
        int r = launch_backward_steps(ctx);
        if (r) return r;
        return 0;
    });
    if (rc) return rc;
    HIP_TRY(ctx, hipEventRecord(ctx->ev[6], ctx->stream));
    rc = launch_param_grads(ctx);
    if (rc) return rc;
    HIP_TRY(ctx, hipGetLastError());
    return 0;
}

__global__ void k_launch_probe(float *p, int touch)
{
    // touch = 0: empty kernel; touch = 1: one dependent load -> store per launch (thread 0)
    if (touch && threadIdx.x == 0 && blockIdx.x == 0) p[0] = p[0] + 1.0f;
}

// average duration, in microseconds, of n dependent launches of a (nearly) empty kernel
hipError_t exec_launch_probe(float *scratch, int n, int touch, float *us_per_launch, hipStream_t s)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) return e;
    for (int i = 0; i < 16; ++i) hipLaunchKernelGGL(k_launch_probe, dim3(64), dim3(WG), 0, s, scratch, touch);
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < n; ++i) hipLaunchKernelGGL(k_launch_probe, dim3(64), dim3(WG), 0, s, scratch, touch);
    (void)hipEventRecord(e1, s);
    e = hipStreamSynchronize(s);
    float ms = 0.f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    *us_per_launch = n > 0 ? ms * 1000.0f / (float)n : 0.f;
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    return e;
}

hipError_t exec_sgd(const ParamDesc *params_dev, u32 n_params, size_t max_count, float lr, int zero_grad, hipStream_t s)
{
    if (n_params == 0) return hipSuccess;
    size_t bx = (max_count + WG * 4 - 1) / (WG * 4);
    if (bx < 1) bx = 1;
    if (bx > 1024) bx = 1024;
    hipLaunchKernelGGL(k_sgd, dim3((unsigned)bx, n_params), dim3(WG), 0, s, params_dev, lr, zero_grad);
    if (zero_grad) hipLaunchKernelGGL(k_sgd_reset, dim3(n_params), dim3(WG), 0, s, params_dev);
    return hipGetLastError();
}

hipError_t exec_gather_all(const Tables &T, int which, float *dst, const u32 *dst_off, hipStream_t s)
{
    if (T.n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_all, dim3(T.n), dim3(64), 0, s, T, which ? T.G : T.V, which ? T.nat_off : T.val_off, dst, dst_off);
    return hipGetLastError();
}

hipError_t exec_fill_uncopied(const Tables &T, hipStream_t s)
{
    if (T.n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_fill_uncopied, dim3(T.n), dim3(64), 0, s, T);
    return hipGetLastError();
}

// The backward counterpart of k_stage_fill: the gradient a stage computed for leaf i (its stand-in
// for an earlier node) is added to that node's row of its owner's incoming-gradient block.
__global__ void k_stage_scatter(const float *G, const u32 *nat_off, u32 first_proxy, const u32 *src, const u32 *dim,
                                const u32 *owner_nat_off, float *owner_gx)
{
    const u32 i = blockIdx.x;
    const float *g = G + nat_off[first_proxy + i];
    float *o = owner_gx + owner_nat_off[src[i]];
    const u32 d = dim[i];
    for (u32 c = threadIdx.x; c < d; c += blockDim.x) o[c] += g[c];
}

hipError_t exec_stage_scatter(const float *G, const u32 *nat_off, u32 first_proxy, const u32 *src, const u32 *dim, u32 count,
                              const u32 *owner_nat_off, float *owner_gx, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_stage_scatter, dim3(count), dim3(64), 0, s, G, nat_off, first_proxy, src, dim, owner_nat_off, owner_gx);
    return hipGetLastError();
}

// k_gather_all for one evaluation stage of several: nodes whose destination is 0xffffffff (the
// stage's stand-ins for earlier nodes) are left out.
__global__ void k_gather_some(Tables T, const float *src, const u32 *src_off, float *dst, const u32 *dst_off)
{
    const u32 v = blockIdx.x;
    if (dst_off[v] == 0xffffffffu) return;
    const u32 d = T.out_dim[v];
    const float *s = src + src_off[v];
    float *o = dst + dst_off[v];
    for (u32 c = threadIdx.x; c < d; c += blockDim.x) o[c] = s[c];
}

hipError_t exec_gather_some(const Tables &T, int which, float *dst, const u32 *dst_off, hipStream_t s)
{
    if (T.n == 0) return hipSuccess;
    hipLaunchKernelGGL(k_gather_some, dim3(T.n), dim3(64), 0, s, T, which ? T.G : T.V, which ? T.nat_off : T.val_off, dst, dst_off);
    return hipGetLastError();
}

hipError_t exec_stage_fill(const float *V, const u32 *val_off, const u32 *src, const u32 *dst, const u32 *dim, u32 count,
                           float *payload, hipStream_t s)
{
    if (count == 0) return hipSuccess;
    hipLaunchKernelGGL(k_stage_fill, dim3(count), dim3(64), 0, s, V, val_off, src, dst, dim, payload);
    return hipGetLastError();
}

hipError_t exec_test_gemm(int M, int N, int K, const float *A, const float *B, float *C, hipStream_t s)
{
    const unsigned tiles = (unsigned)(((M + GT - 1) / GT) * ((N + GT - 1) / GT));
    hipLaunchKernelGGL(k_test_gemm, dim3(tiles), dim3(WG), 0, s, A, B, C, M, N, K);
    return hipGetLastError();
}
