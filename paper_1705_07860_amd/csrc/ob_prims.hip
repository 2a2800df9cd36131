// Device-wide primitives of the GPU scheduler: fill, exclusive scan, stable LSD radix sort.
// Written for wave64 (gfx950): ranking inside a wave uses 64-bit ballots.
#include "../../include/ob.h"
#include "ob_ctx.h"

#include <mutex>

namespace {

constexpr int SCAN_THREADS = 256;
constexpr int SCAN_ITEMS = 4;
constexpr int SCAN_BLOCK = SCAN_THREADS * SCAN_ITEMS;  // 1024 elements per block

__global__ void k_fill_u32(u32 *p, u32 v, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) p[i] = v;
}

template <typename T> __device__ inline T zero_of();
template <> __device__ inline u32 zero_of<u32>() { return 0u; }
template <> __device__ inline Lay zero_of<Lay>() { Lay z; z.val = 0; z.dx = 0; z.ind = z.p0 = z.p1 = z.p2 = 0; return z; }
template <> __device__ inline Tri zero_of<Tri>() { Tri z; z.a = z.b = z.c = z.d = 0; return z; }
template <> __device__ inline CLay zero_of<CLay>() { CLay z; z.tf = z.wf = z.ta = z.wa = z.tb = z.p0 = z.p1 = z.p2 = 0; return z; }

// Exclusive scan of the 256 per-thread values of a block through LDS (Kogge-Stone).
// Returns the exclusive prefix of this thread; *block_total gets the sum of all 256.
template <typename T>
__device__ inline T block_exclusive(T mine, T *lds, T *block_total)
{
    const int t = threadIdx.x;
    lds[t] = mine;
    __syncthreads();
    for (int off = 1; off < SCAN_THREADS; off <<= 1) {
        T add = zero_of<T>();
        if (t >= off) add = lds[t - off];
        __syncthreads();
        if (t >= off) lds[t] = lds[t] + add;
        __syncthreads();
    }
    T incl = lds[t];
    T total = lds[SCAN_THREADS - 1];
    __syncthreads();
    *block_total = total;
    // exclusive = inclusive of the previous thread
    T excl = zero_of<T>();
    lds[t] = incl;
    __syncthreads();
    if (t > 0) excl = lds[t - 1];
    __syncthreads();
    return excl;
}

template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_local(const T *in, T *out, T *block_sums, size_t n)
{
    __shared__ T lds[SCAN_THREADS];
    const size_t base = (size_t)blockIdx.x * SCAN_BLOCK + (size_t)threadIdx.x * SCAN_ITEMS;
    T item[SCAN_ITEMS];
    T sum = zero_of<T>();
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        item[i] = (base + i < n) ? in[base + i] : zero_of<T>();
        sum = sum + item[i];
    }
    T total;
    T run = block_exclusive<T>(sum, lds, &total);
    for (int i = 0; i < SCAN_ITEMS; ++i) {
        if (base + i < n) out[base + i] = run;
        run = run + item[i];
    }
    if (threadIdx.x == 0) block_sums[blockIdx.x] = total;
}

// One block turns the per-block sums into exclusive offsets, chunk by chunk with a carry.
template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_sums(T *block_sums, size_t nblk, T *total_out)
{
    __shared__ T lds[SCAN_THREADS];
    T carry = zero_of<T>();
    for (size_t c0 = 0; c0 < nblk; c0 += SCAN_THREADS) {
        const size_t i = c0 + threadIdx.x;
        T mine = (i < nblk) ? block_sums[i] : zero_of<T>();
        T total;
        T ex = block_exclusive<T>(mine, lds, &total);
        if (i < nblk) block_sums[i] = carry + ex;
        carry = carry + total;
    }
    if (threadIdx.x == 0 && total_out) *total_out = carry;
}

template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_add(T *out, const T *block_sums, size_t n)
{
    const T add = block_sums[blockIdx.x];
    const size_t base = (size_t)blockIdx.x * SCAN_BLOCK + (size_t)threadIdx.x * SCAN_ITEMS;
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n) out[base + i] = out[base + i] + add;
}

// Up to SCAN_THREADS blocks: every block adds up the sums of the blocks before it itself (a few hundred
// integers), so the launch that scans the block sums is not needed.  Block 0 also leaves the total.
template <typename T>
__device__ inline T block_sum(T mine, T *lds)
{
    const int t = threadIdx.x;
    lds[t] = mine;
    __syncthreads();
    for (int off = SCAN_THREADS / 2; off > 0; off >>= 1) {
        if (t < off) lds[t] = lds[t] + lds[t + off];
        __syncthreads();
    }
    const T r = lds[0];
    __syncthreads();
    return r;
}
template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_add_own(T *out, const T *block_sums, size_t nblk, size_t n, T *total_out)
{
    __shared__ T lds[SCAN_THREADS];
    const size_t t = threadIdx.x;
    const T add = block_sum<T>(t < blockIdx.x ? block_sums[t] : zero_of<T>(), lds);
    const size_t base = (size_t)blockIdx.x * SCAN_BLOCK + t * SCAN_ITEMS;
    for (int i = 0; i < SCAN_ITEMS; ++i)
        if (base + i < n) out[base + i] = out[base + i] + add;
    if (blockIdx.x == 0 && total_out) {
        const T total = block_sum<T>(t < nblk ? block_sums[t] : zero_of<T>(), lds);
        if (t == 0) *total_out = total;
    }
}

// Short inputs: one workgroup walks the chunks with a carry, one launch instead of two or three
// (the scheduler of a small graph is bound by the number of its launches).  in == out is fine.
constexpr size_t SCAN_SMALL_MAX = 4 * SCAN_BLOCK;
template <typename T>
__global__ __launch_bounds__(SCAN_THREADS) void k_scan_small(const T *in, T *out, size_t n, T *total_out)
{
    __shared__ T lds[SCAN_THREADS];
    T carry = zero_of<T>();
    for (size_t c0 = 0; c0 < n; c0 += SCAN_BLOCK) {
        const size_t base = c0 + (size_t)threadIdx.x * SCAN_ITEMS;
        T item[SCAN_ITEMS];
        T sum = zero_of<T>();
        for (int i = 0; i < SCAN_ITEMS; ++i) {
            item[i] = (base + i < n) ? in[base + i] : zero_of<T>();
            sum = sum + item[i];
        }
        T total;
        T run = carry + block_exclusive<T>(sum, lds, &total);
        for (int i = 0; i < SCAN_ITEMS; ++i) {
            if (base + i < n) out[base + i] = run;
            run = run + item[i];
        }
        carry = carry + total;
    }
    if (threadIdx.x == 0 && total_out) *total_out = carry;
}

template <typename T>
hipError_t scan_impl(const T *in, T *out, size_t n, T *total_dev, void *scratch, hipStream_t s)
{
    if (n == 0) {
        // total = 0
        if (total_dev) return hipMemsetAsync(total_dev, 0, sizeof(T), s);
        return hipSuccess;
    }
    if (n <= SCAN_SMALL_MAX) {
        hipLaunchKernelGGL(k_scan_small<T>, dim3(1), dim3(SCAN_THREADS), 0, s, in, out, n, total_dev);
        return hipGetLastError();
    }
    const size_t nblk = (n + SCAN_BLOCK - 1) / SCAN_BLOCK;
    T *sums = (T *)scratch;
    hipLaunchKernelGGL(k_scan_local<T>, dim3((unsigned)nblk), dim3(SCAN_THREADS), 0, s, in, out, sums, n);
    if (nblk <= (size_t)SCAN_THREADS) {
        hipLaunchKernelGGL(k_scan_add_own<T>, dim3((unsigned)nblk), dim3(SCAN_THREADS), 0, s, out, sums, nblk, n, total_dev);
        return hipGetLastError();
    }
    hipLaunchKernelGGL(k_scan_sums<T>, dim3(1), dim3(SCAN_THREADS), 0, s, sums, nblk, total_dev);
    if (nblk > 1)
        hipLaunchKernelGGL(k_scan_add<T>, dim3((unsigned)nblk), dim3(SCAN_THREADS), 0, s, out, sums, n);
    return hipGetLastError();
}

// ---- radix sort ------------------------------------------------------------------------------
constexpr int RS_BITS = 8;
constexpr int RS_RADIX = 1 << RS_BITS;
constexpr int RS_THREADS = 256;                  // 4 waves
constexpr int RS_WAVES = RS_THREADS / 64;
constexpr int RS_ROUNDS = 4;                     // keys per lane
constexpr int RS_WAVE_KEYS = 64 * RS_ROUNDS;     // 256 consecutive keys per wave
constexpr int RS_BLOCK = RS_WAVE_KEYS * RS_WAVES;  // 1024 keys per block

__device__ inline u32 digit_of(u64 key, int shift, u32 mask) { return (u32)(key >> shift) & mask; }

// number of keys of block blk whose digit is d: table[blk * 256 + d], or (dmajor, many blocks: the
// table is then scanned as it lies) table[d * nblk + blk]
__global__ __launch_bounds__(RS_THREADS) void k_rs_hist(const u64 *keys, size_t n, int shift, u32 mask,
                                                       u32 *table, u32 nblk, u32 dmajor)
{
    __shared__ u32 hist[RS_RADIX];
    hist[threadIdx.x] = 0;
    __syncthreads();
    const size_t base = (size_t)blockIdx.x * RS_BLOCK;
    for (int i = 0; i < RS_BLOCK / RS_THREADS; ++i) {
        const size_t idx = base + (size_t)i * RS_THREADS + threadIdx.x;
        if (idx < n) atomicAdd(&hist[digit_of(keys[idx], shift, mask)], 1u);
    }
    __syncthreads();
    table[dmajor ? (size_t)threadIdx.x * nblk + blockIdx.x : (size_t)blockIdx.x * RS_RADIX + threadIdx.x] = hist[threadIdx.x];
}

// One workgroup turns the per-block digit counts into the blocks' first output positions (an
// exclusive scan in digit-major, block-minor order) in place: thread (segment, digit) first sums
// its quarter of the blocks for its digit, the 256 digit totals are scanned in LDS, then every
// thread walks its blocks again with a running position.  One launch where a general scan of the
// table takes three.
constexpr int RSO_THREADS = 1024;
constexpr int RSO_SEGS = RSO_THREADS / RS_RADIX;
constexpr u32 RSO_MAX_BLOCKS = 256;
__global__ __launch_bounds__(RSO_THREADS) void k_rs_offsets(u32 *table, u32 nblk)
{
    __shared__ u32 seg_sum[RSO_SEGS][RS_RADIX];
    __shared__ u32 dig[RS_RADIX];
    const u32 d = threadIdx.x & (RS_RADIX - 1), seg = threadIdx.x / RS_RADIX;
    const u32 per = (nblk + RSO_SEGS - 1) / RSO_SEGS;
    const u32 b0 = seg * per < nblk ? seg * per : nblk, b1 = (seg + 1) * per < nblk ? (seg + 1) * per : nblk;
    u32 sum = 0;
    for (u32 b = b0; b < b1; b += 8) {       // eight loads in flight per thread
        u32 c[8];
#pragma unroll
        for (u32 q = 0; q < 8; ++q) c[q] = b + q < b1 ? table[(size_t)(b + q) * RS_RADIX + d] : 0u;
#pragma unroll
        for (u32 q = 0; q < 8; ++q) sum += c[q];
    }
    seg_sum[seg][d] = sum;
    __syncthreads();
    if (seg == 0) {
        u32 tot = 0;
        for (int q = 0; q < RSO_SEGS; ++q) tot += seg_sum[q][d];
        dig[d] = tot;
    }
    __syncthreads();
    // inclusive scan of the digit totals (Kogge-Stone over 256 entries; the other threads only keep step at the barriers)
    for (u32 off = 1; off < (u32)RS_RADIX; off <<= 1) {
        u32 add = 0;
        if (seg == 0 && d >= off) add = dig[d - off];
        __syncthreads();
        if (seg == 0) dig[d] += add;
        __syncthreads();
    }
    u32 run = d ? dig[d - 1] : 0u;     // keys with a smaller digit
    for (u32 q = 0; q < seg; ++q) run += seg_sum[q][d];
    for (u32 b = b0; b < b1; b += 8) {
        u32 c[8];
#pragma unroll
        for (u32 q = 0; q < 8; ++q) c[q] = b + q < b1 ? table[(size_t)(b + q) * RS_RADIX + d] : 0u;
#pragma unroll
        for (u32 q = 0; q < 8; ++q) {
            if (b + q < b1) table[(size_t)(b + q) * RS_RADIX + d] = run;
            run += c[q];
        }
    }
}

// Stable scatter.  Wave w of a block owns keys [w*256, w*256+256) of the block's chunk and
// walks them in 4 rounds of 64; inside a round lanes with equal digits are ranked by lane id.
__global__ __launch_bounds__(RS_THREADS) void k_rs_scatter(const u64 *keys, const u32 *vals, u64 *keys_out,
                                                          u32 *vals_out, size_t n, int shift, u32 mask,
                                                          const u32 *table, u32 nblk, u32 dmajor)
{
    __shared__ u32 cnt[RS_WAVES][RS_RADIX];
    const int lane = threadIdx.x & 63;
    const int w = threadIdx.x >> 6;
    for (int i = 0; i < RS_WAVES; ++i) cnt[i][threadIdx.x] = 0;
    __syncthreads();

    const size_t wbase = (size_t)blockIdx.x * RS_BLOCK + (size_t)w * RS_WAVE_KEYS;
    u64 key[RS_ROUNDS];
    u32 val[RS_ROUNDS];
    bool ok[RS_ROUNDS];
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const size_t idx = wbase + (size_t)r * 64 + lane;
        ok[r] = idx < n;
        key[r] = ok[r] ? keys[idx] : 0;
        val[r] = ok[r] ? vals[idx] : 0;
        if (ok[r]) atomicAdd(&cnt[w][digit_of(key[r], shift, mask)], 1u);
    }
    __syncthreads();
    {   // thread d turns the per-wave counts of digit d into per-wave start positions
        const int d = threadIdx.x;
        u32 run = table[dmajor ? (size_t)d * nblk + blockIdx.x : (size_t)blockIdx.x * RS_RADIX + d];
        for (int i = 0; i < RS_WAVES; ++i) {
            const u32 c = cnt[i][d];
            cnt[i][d] = run;
            run += c;
        }
    }
    __syncthreads();
    for (int r = 0; r < RS_ROUNDS; ++r) {
        const u32 d = digit_of(key[r], shift, mask);
        u64 peers = __ballot(ok[r]);
        for (int b = 0; b < RS_BITS; ++b) {
            const bool bit = (d >> b) & 1u;
            const u64 m = __ballot(bit);
            peers &= bit ? m : ~m;
        }
        if (!ok[r]) peers = 0;
        const u32 rank = (u32)__popcll(peers & ((1ull << lane) - 1ull));
        const u32 count = (u32)__popcll(peers);
        const int leader = peers ? (__ffsll((unsigned long long)peers) - 1) : lane;
        u32 start = 0;
        if (ok[r] && leader == lane) start = atomicAdd(&cnt[w][d], count);
        start = __shfl(start, leader);
        if (ok[r]) {
            keys_out[start + rank] = key[r];
            vals_out[start + rank] = val[r];
        }
    }
}

// Short inputs: the whole sort in one workgroup, all passes in one launch.  Every pass counts the
// digits of all keys, scans the 256 counts, then scatters tile by tile (1024 keys, one per thread):
// lanes of a wave with equal digits are ranked by lane id, waves by their order in the tile, tiles
// by the running start of every digit, which keeps the sort stable.  Passes alternate between the
// two buffer pairs in global memory; a workgroup sees its own global writes after a barrier.
constexpr int RSS_THREADS = 1024;
constexpr int RSS_WAVES = RSS_THREADS / 64;
constexpr size_t RS_SMALL_MAX = 8192;
__global__ __launch_bounds__(RSS_THREADS) void k_rs_small(u64 *keys, u32 *vals, u64 *keys_tmp, u32 *vals_tmp, u32 n,
                                                         int lo_bit, int n_bits, const u32 *n_dev)
{
    if (n_dev) n = *n_dev < n ? *n_dev : n;   // the same value for every thread: barriers below stay uniform
    __shared__ u32 start[RS_RADIX];             // running first output position of every digit
    __shared__ u32 cnt[RSS_WAVES][RS_RADIX];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, t = threadIdx.x;
    u64 *kin = keys, *kout = keys_tmp;
    u32 *vin = vals, *vout = vals_tmp;
    for (int b = 0; b < n_bits; b += RS_BITS) {
        const int bits = (n_bits - b < RS_BITS) ? (n_bits - b) : RS_BITS;
        const u32 mask = (1u << bits) - 1u;
        const int shift = lo_bit + b;
        if (t < RS_RADIX) start[t] = 0;
        __syncthreads();
        for (u32 i = t; i < n; i += RSS_THREADS) atomicAdd(&start[digit_of(kin[i], shift, mask)], 1u);
        __syncthreads();
        if (t < RS_RADIX) cnt[0][t] = start[t];
        __syncthreads();
        for (int off = 1; off < RS_RADIX; off <<= 1) {
            u32 add = 0;
            if (t < RS_RADIX && t >= off) add = cnt[0][t - off];
            __syncthreads();
            if (t < RS_RADIX) cnt[0][t] += add;
            __syncthreads();
        }
        if (t < RS_RADIX) start[t] = cnt[0][t] - start[t];   // inclusive -> exclusive
        __syncthreads();
        for (u32 t0 = 0; t0 < n; t0 += RSS_THREADS) {
            for (int i = 0; i < RSS_WAVES * RS_RADIX / RSS_THREADS; ++i) (&cnt[0][0])[i * RSS_THREADS + t] = 0;
            __syncthreads();
            const u32 idx = t0 + t;
            const bool ok = idx < n;
            const u64 key = ok ? kin[idx] : 0;
            const u32 val = ok ? vin[idx] : 0;
            const u32 d = digit_of(key, shift, mask);
            u64 peers = __ballot(ok);
            for (int q = 0; q < RS_BITS; ++q) {
                const bool bit = (d >> q) & 1u;
                const u64 m = __ballot(bit);
                peers &= bit ? m : ~m;
            }
            if (!ok) peers = 0;
            const u32 rank = (u32)__popcll(peers & ((1ull << lane) - 1ull));
            const int leader = peers ? (__ffsll((unsigned long long)peers) - 1) : lane;
            if (ok && leader == lane) cnt[w][d] = (u32)__popcll(peers);
            __syncthreads();
            if (t < RS_RADIX) {
                u32 run = start[t];
                for (int i = 0; i < RSS_WAVES; ++i) {
                    const u32 c = cnt[i][t];
                    cnt[i][t] = run;
                    run += c;
                }
                start[t] = run;
            }
            __syncthreads();
            if (ok) {
                const u32 pos = cnt[w][d] + rank;
                kout[pos] = key;
                vout[pos] = val;
            }
            __syncthreads();
        }
        u64 *tk = kin; kin = kout; kout = tk;
        u32 *tv = vin; vin = vout; vout = tv;
    }
    if (kin != keys)   // an odd number of passes: the result sits in the second pair
        for (u32 i = t; i < n; i += RSS_THREADS) { keys[i] = kin[i]; vals[i] = vin[i]; }
}

}  // namespace

// ---- host wrappers -------------------------------------------------------------------------------

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t prim_scan_scratch_bytes(size_t n, size_t elem)
{
    return align256(((n + SCAN_BLOCK - 1) / SCAN_BLOCK + 1) * elem);
}

hipError_t prim_fill_u32(u32 *p, u32 v, size_t n, hipStream_t s)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 1023) / 1024;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(k_fill_u32, dim3((unsigned)blocks), dim3(256), 0, s, p, v, n);
    return hipGetLastError();
}

hipError_t prim_scan_u32(const u32 *in, u32 *out, size_t n, u32 *total_dev, void *scratch, hipStream_t s)
{
    return scan_impl<u32>(in, out, n, total_dev, scratch, s);
}

hipError_t prim_scan_lay(const Lay *in, Lay *out, size_t n, Lay *total_dev, void *scratch, hipStream_t s)
{
    return scan_impl<Lay>(in, out, n, total_dev, scratch, s);
}

hipError_t prim_scan_clay(const CLay *in, CLay *out, size_t n, CLay *total_dev, void *scratch, hipStream_t s)
{
    return scan_impl<CLay>(in, out, n, total_dev, scratch, s);
}

hipError_t prim_scan_tri(const Tri *in, Tri *out, size_t n, Tri *total_dev, void *scratch, hipStream_t s)
{
    return scan_impl<Tri>(in, out, n, total_dev, scratch, s);
}

size_t prim_sort_scratch_bytes(size_t n)
{
    const size_t nblk = (n + RS_BLOCK - 1) / RS_BLOCK;
    const size_t table = align256((size_t)RS_RADIX * (nblk ? nblk : 1) * sizeof(u32));
    return table + prim_scan_scratch_bytes((size_t)RS_RADIX * (nblk ? nblk : 1), sizeof(u32));
}

static hipError_t sort_pairs_impl(u64 *keys, u32 *vals, u64 *keys_tmp, u32 *vals_tmp, size_t n, int lo_bit,
                                  int n_bits, void *scratch, hipStream_t s, int *n_launches, const u32 *n_dev, bool *in_tmp)
{
    if (in_tmp) *in_tmp = false;
    if (n <= 1 || n_bits <= 0) return hipSuccess;
    if (n <= RS_SMALL_MAX) {
        hipLaunchKernelGGL(k_rs_small, dim3(1), dim3(RSS_THREADS), 0, s, keys, vals, keys_tmp, vals_tmp, (u32)n, lo_bit,
                           n_bits, n_dev);
        if (n_launches) *n_launches += 1;
        return hipGetLastError();
    }
    const u32 nblk = (u32)((n + RS_BLOCK - 1) / RS_BLOCK);
    u32 *table = (u32 *)scratch;
    void *scan_scratch = (char *)scratch + align256((size_t)RS_RADIX * nblk * sizeof(u32));
    u64 *kin = keys, *kout = keys_tmp;
    u32 *vin = vals, *vout = vals_tmp;
    int passes = 0;
    for (int b = 0; b < n_bits; b += RS_BITS) {
        const int bits = (n_bits - b < RS_BITS) ? (n_bits - b) : RS_BITS;
        const u32 mask = (1u << bits) - 1u;
        const int shift = lo_bit + b;
        // up to RSO_MAX_BLOCKS blocks one workgroup turns the counts into positions in one launch; beyond, the
        // table is laid out digit-major and scanned by the general three-launch scan
        const u32 dmajor = nblk > RSO_MAX_BLOCKS ? 1u : 0u;
        hipLaunchKernelGGL(k_rs_hist, dim3(nblk), dim3(RS_THREADS), 0, s, kin, n, shift, mask, table, nblk, dmajor);
        if (dmajor) {
            hipError_t e = scan_impl<u32>(table, table, (size_t)RS_RADIX * nblk, (u32 *)nullptr, scan_scratch, s);
            if (e != hipSuccess) return e;
        } else {
            hipLaunchKernelGGL(k_rs_offsets, dim3(1), dim3(RSO_THREADS), 0, s, table, nblk);
        }
        hipLaunchKernelGGL(k_rs_scatter, dim3(nblk), dim3(RS_THREADS), 0, s, kin, vin, kout, vout, n, shift,
                           mask, table, nblk, dmajor);
        u64 *tk = kin; kin = kout; kout = tk;
        u32 *tv = vin; vin = vout; vout = tv;
        ++passes;
        if (n_launches) *n_launches += dmajor ? 5 : 3;
    }
    if ((passes & 1) && in_tmp) {   // the caller takes the result where it is
        *in_tmp = true;
    } else if (passes & 1) {  // result sits in the tmp arrays: copy back
        hipError_t e = hipMemcpyAsync(keys, kin, n * sizeof(u64), hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
        e = hipMemcpyAsync(vals, vin, n * sizeof(u32), hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

hipError_t prim_sort_pairs(u64 *keys, u32 *vals, u64 *keys_tmp, u32 *vals_tmp, size_t n, int lo_bit,
                           int n_bits, void *scratch, hipStream_t s, int *n_launches, const u32 *n_dev)
{
    return sort_pairs_impl(keys, vals, keys_tmp, vals_tmp, n, lo_bit, n_bits, scratch, s, n_launches, n_dev, nullptr);
}

// The same sort without the copy back after an odd number of passes: the two buffer pairs change
// roles instead (on return keys / vals point at the sorted data, keys_tmp / vals_tmp at the other pair).
hipError_t prim_sort_pairs_swap(u64 *&keys, u32 *&vals, u64 *&keys_tmp, u32 *&vals_tmp, size_t n, int lo_bit,
                                int n_bits, void *scratch, hipStream_t s, int *n_launches, const u32 *n_dev)
{
    bool in_tmp = false;
    hipError_t e = sort_pairs_impl(keys, vals, keys_tmp, vals_tmp, n, lo_bit, n_bits, scratch, s, n_launches, n_dev, &in_tmp);
    if (in_tmp) {
        u64 *tk = keys; keys = keys_tmp; keys_tmp = tk;
        u32 *tv = vals; vals = vals_tmp; vals_tmp = tv;
    }
    return e;
}

// ---- the sort for callers that cannot allocate ------------------------------------------------------
// Everything the sort needs beyond the caller's two arrays (the second key / value buffer of the
// ping-pong passes, the per-block digit table and the scan's block sums) lies in one array in the
// library's own device image, so the call reaches no allocator.  Each GPU holds its own copy of
// the array at its own address; the address is looked up once per device and kept.
constexpr size_t NOALLOC_TABLE_BYTES = ((size_t)OB_NOALLOC_MAX_PAIRS / RS_BLOCK + 1) * RS_RADIX * sizeof(u32) + 4096;
constexpr size_t NOALLOC_KEYS_OFF = 0;
constexpr size_t NOALLOC_VALS_OFF = (size_t)OB_NOALLOC_MAX_PAIRS * sizeof(u64);
constexpr size_t NOALLOC_TABLE_OFF = NOALLOC_VALS_OFF + (size_t)OB_NOALLOC_MAX_PAIRS * sizeof(u32);
constexpr size_t NOALLOC_BYTES = NOALLOC_TABLE_OFF + 2 * NOALLOC_TABLE_BYTES;
static_assert(NOALLOC_VALS_OFF % 256 == 0 && NOALLOC_TABLE_OFF % 256 == 0, "sections of the scratch array stay 256-byte aligned");
static __device__ __align__(256) unsigned char scratch[NOALLOC_BYTES];

constexpr int NOALLOC_MAX_DEVICES = 64;
static std::mutex g_noalloc_mutex;
static void *g_noalloc_ptr[NOALLOC_MAX_DEVICES] = {};

// device address of the current device's copy of `scratch` (host code never uses the array's name
// for anything else: on the host it is only a handle for this look-up)
static int noalloc_scratch(char **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return ctx_fail(nullptr, OB_E_HIP, "hipGetDevice failed: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return ctx_fail(nullptr, OB_E_RANGE, "device index %d outside 0 .. %d", dev, NOALLOC_MAX_DEVICES - 1);
    std::lock_guard<std::mutex> lock(g_noalloc_mutex);
    if (!g_noalloc_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return ctx_fail(nullptr, OB_E_HIP, "hipGetSymbolAddress(scratch) failed on device %d: %s", dev, hipGetErrorString(e));
        g_noalloc_ptr[dev] = ptr;
    }
    *out = (char *)g_noalloc_ptr[dev];
    return OB_OK;
}

extern "C" int ob_sort_pairs_noalloc(void *hip_stream, size_t n, uint64_t *keys_dev, uint32_t *vals_dev, int lo_bit, int n_bits)
{
    if (n > (size_t)OB_NOALLOC_MAX_PAIRS)
        return ctx_fail(nullptr, OB_E_RANGE, "ob_sort_pairs_noalloc: %zu pairs, the built-in scratch holds at most %d", n,
                        (int)OB_NOALLOC_MAX_PAIRS);
    if (lo_bit < 0 || n_bits < 0 || lo_bit + n_bits > 64)
        return ctx_fail(nullptr, OB_E_ARG, "ob_sort_pairs_noalloc: bits [%d, %d) outside a 64-bit key", lo_bit, lo_bit + n_bits);
    if (n == 0) return OB_OK;
    if (!keys_dev || !vals_dev) return ctx_fail(nullptr, OB_E_ARG, "ob_sort_pairs_noalloc: null array");
    char *base = nullptr;
    if (int rc = noalloc_scratch(&base)) return rc;
    // Nothing in the scratch has to start at zero: every pass writes each entry of the digit table
    // and of the block sums it reads, and the second buffers are written before they are read, so
    // what an earlier (larger) call left behind is never looked at.
    hipError_t e = prim_sort_pairs(keys_dev, vals_dev, (u64 *)(base + NOALLOC_KEYS_OFF), (u32 *)(base + NOALLOC_VALS_OFF), n, lo_bit,
                                   n_bits, base + NOALLOC_TABLE_OFF, (hipStream_t)hip_stream, nullptr);
    if (e != hipSuccess) return ctx_fail(nullptr, OB_E_HIP, "ob_sort_pairs_noalloc: %s", hipGetErrorString(e));
    return OB_OK;
}
