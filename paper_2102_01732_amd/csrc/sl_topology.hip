// Topology of a truly sparse layer on the GPU (gfx950): Erdos-Renyi initialisation, the SET
// prune / regrow cycle of Algorithm 2 (radix-select threshold, prefix-sum compaction, Philox
// counter-based regrowth, merge into a sorted CSR) and the derived structures (CSC view for the
// backward pass, virtual-row tables).  Device-wide scans and radix sorts come from rocPRIM; every
// other step is a kernel of this file.  All steps are deterministic: the resulting CSR depends
// only on (pattern, weights, seed, layer_id, generation).
#include <climits>
#include <cstring>

#include <rocprim/rocprim.hpp>

#include "sl_internal.h"

namespace sl {

static constexpr int TB = 256;
static inline unsigned nblk(long n) { return n <= 0 ? 1u : (unsigned)((n + TB - 1) / TB); }

// ------------------------------------------------------------------------------------------------
// Philox4x32-10 (Salmon et al., SC'11) and the stream layout of this library:
// key = (lo32(seed) ^ layer_id*0x9E3779B9, hi32(seed)), counter = (index_lo, index_hi, purpose,
// generation); purpose 1 = candidate position, 2 = dense-mode ordering key, 3 = weight value.
// ------------------------------------------------------------------------------------------------
struct Rng {
    uint32_t k0, k1, generation;
};

__device__ inline float fresh_weight(const Rng &r, uint64_t p, float limit)
{
    uint32_t o[4];
    philox((uint32_t)p, (uint32_t)(p >> 32), 3u, r.generation, r.k0, r.k1, o);
    const int odd = (int)(2u * (o[0] >> 9) + 1u) - (1 << 23);
    return ((float)odd * (1.0f / 8388608.0f)) * limit;
}

// ------------------------------------------------------------------------------------------------
// small search helpers
// ------------------------------------------------------------------------------------------------
__device__ inline int lower_bound_i32(const int *a, int lo, int hi, int x)
{
    while (lo < hi) {
        const int mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}
__device__ inline long lower_bound_u64(const uint64_t *a, long n, uint64_t x)
{
    long lo = 0, hi = n;
    while (lo < hi) {
        const long mid = lo + ((hi - lo) >> 1);
        if (a[mid] < x) lo = mid + 1; else hi = mid;
    }
    return lo;
}
// row that owns CSR position p: largest r with ptr[r] <= p
__device__ inline int row_of(const int *ptr, int n_rows, int p)
{
    int lo = 0, hi = n_rows;   // invariant: ptr[lo] <= p < ptr[hi]
    while (hi - lo > 1) {
        const int mid = lo + ((hi - lo) >> 1);
        if (ptr[mid] <= p) lo = mid; else hi = mid;
    }
    return lo;
}

// ------------------------------------------------------------------------------------------------
// rocPRIM wrappers
// ------------------------------------------------------------------------------------------------
template <typename T>
static hipError_t scan_excl(void *temp, size_t temp_bytes, const T *in, T *out, size_t n, hipStream_t s)
{
    size_t need = temp_bytes;
    return rocprim::exclusive_scan(temp, need, in, out, (T)0, n, rocprim::plus<T>(), s);
}
template <typename K>
static hipError_t sort_pairs(void *temp, size_t temp_bytes, K *kA, K *kB, uint32_t *vA, uint32_t *vB, size_t n,
                             unsigned bits, K **k_out, uint32_t **v_out, hipStream_t s)
{
    rocprim::double_buffer<K> kb(kA, kB);
    rocprim::double_buffer<uint32_t> vb(vA, vB);
    size_t need = temp_bytes;
    hipError_t e = rocprim::radix_sort_pairs(temp, need, kb, vb, n, 0u, bits, s);
    *k_out = kb.current();
    *v_out = vb.current();
    return e;
}
static unsigned bit_length(uint64_t x)
{
    unsigned b = 0;
    while (x) { ++b; x >>= 1; }
    return b ? b : 1;
}

int topo_check_temp(sl_layer *L, hipStream_t s)
{
    size_t need = 0, worst = 0;
    const size_t n = (size_t)L->nnz + 1, w = (size_t)L->cp.w_cap + 1;
    SL_HIP(L, rocprim::exclusive_scan(nullptr, need, (uint32_t *)nullptr, (uint32_t *)nullptr, 0u, w > n ? w : n,
                                      rocprim::plus<uint32_t>(), s));
    worst = need;
    SL_HIP(L, rocprim::exclusive_scan(nullptr, need, (uint64_t *)nullptr, (uint64_t *)nullptr, (uint64_t)0, n,
                                      rocprim::plus<uint64_t>(), s));
    worst = need > worst ? need : worst;
    {
        rocprim::double_buffer<uint64_t> kb((uint64_t *)nullptr, (uint64_t *)nullptr);
        rocprim::double_buffer<uint32_t> vb((uint32_t *)nullptr, (uint32_t *)nullptr);
        SL_HIP(L, rocprim::radix_sort_pairs(nullptr, need, kb, vb, w, 0u, 64u, s));
        worst = need > worst ? need : worst;
    }
    {
        rocprim::double_buffer<uint32_t> kb((uint32_t *)nullptr, (uint32_t *)nullptr);
        rocprim::double_buffer<uint32_t> vb((uint32_t *)nullptr, (uint32_t *)nullptr);
        SL_HIP(L, rocprim::radix_sort_pairs(nullptr, need, kb, vb, n, 0u, 32u, s));
        worst = need > worst ? need : worst;
    }
    if (worst > L->cp.temp_bytes)
        return set_err(L, SL_ENOMEM, "rocPRIM temporaries need %zu bytes, %zu reserved", worst, L->cp.temp_bytes);
    return SL_OK;
}

// ------------------------------------------------------------------------------------------------
// Pruning threshold by radix select (four 8-bit passes, most significant digit first) on the
// magnitude bits of the weights.  class 0 = all weights (mode 0) or weights >= 0 (mode 1),
// class 1 = weights < 0 (mode 1 only).
// ------------------------------------------------------------------------------------------------
__device__ inline int weight_class(float w, int mode) { return (mode == 1 && w < 0.f) ? 1 : 0; }

__global__ void class_count_kernel(const float *val, long n, uint32_t *counts)
{
    __shared__ uint32_t c;
    if (threadIdx.x == 0) c = 0;
    __syncthreads();
    uint32_t mine = 0;
    for (long p = (long)blockIdx.x * TB + threadIdx.x; p < n; p += (long)gridDim.x * TB) mine += val[p] < 0.f;
    // wavefront-level reduction, one atomic per wavefront
    for (int m = 32; m >= 1; m >>= 1) mine += __shfl_xor(mine, m);
    if ((threadIdx.x & 63) == 0) atomicAdd(&c, mine);
    __syncthreads();
    if (threadIdx.x == 0) atomicAdd(&counts[0], c);
}

__global__ void select_setup_kernel(SelState *st, uint32_t k0, uint32_t k1)
{
    const int c = blockIdx.x;
    SelState &s = st[c];
    if (threadIdx.x == 0) {
        const uint32_t k = c == 0 ? k0 : k1;
        s.prefix = 0; s.krem = k; s.active = k > 0; s.thresh = 0; s.need = 0;
    }
    s.hist[threadIdx.x] = 0;
}

// Few, large workgroups: every workgroup ends with up to 512 atomic additions to the same 512 global counters, and
// those serialise per counter (with 2048 workgroups they took three quarters of the pass).
constexpr int HIST_TB = 1024, HIST_BLOCKS = 512;
__global__ __launch_bounds__(HIST_TB) void select_hist_kernel(const float *val, long n, int mode, int shift, SelState *st)
{
    __shared__ uint32_t h[2][256];
    if (threadIdx.x < 256) {
        h[0][threadIdx.x] = 0;
        h[1][threadIdx.x] = 0;
    }
    __syncthreads();
    const uint32_t act0 = st[0].active, act1 = st[1].active;
    const uint32_t pre0 = st[0].prefix, pre1 = st[1].prefix;
    // Neighbouring weights mostly share their leading digit (the first pass sees two or three exponent values in
    // all), and additions of a whole wavefront to one LDS counter serialise: a lane adds a run of equal digits at once.
    int run_bin = -1;
    uint32_t run_len = 0;
    auto flush = [&]() {
        if (run_len) atomicAdd(&h[run_bin >> 8][run_bin & 255], run_len);
        run_len = 0;
    };
    auto count = [&](float w) {
        const int c = weight_class(w, mode);
        const uint32_t mag = __float_as_uint(w) & 0x7FFFFFFFu;
        const uint32_t act = c ? act1 : act0, pre = c ? pre1 : pre0;
        const bool in = act && (shift == 24 || (mag >> (shift + 8)) == pre);
        if (!in) return;
        const int bin = (c << 8) | (int)((mag >> shift) & 255u);
        if (bin != run_bin) { flush(); run_bin = bin; }
        ++run_len;
    };
    // eight weights per lane and trip (two 16-byte loads issued before the first is used)
    const long n8 = n / 8;
    const float4 *v4 = (const float4 *)val;
    for (long q = (long)blockIdx.x * HIST_TB + threadIdx.x; q < n8; q += (long)gridDim.x * HIST_TB) {
        const float4 a = v4[2 * q], b = v4[2 * q + 1];
        count(a.x); count(a.y); count(a.z); count(a.w);
        count(b.x); count(b.y); count(b.z); count(b.w);
    }
    for (long p = n8 * 8 + (long)blockIdx.x * HIST_TB + threadIdx.x; p < n; p += (long)gridDim.x * HIST_TB) count(val[p]);
    flush();
    __syncthreads();
    if (threadIdx.x < 256) {
        if (h[0][threadIdx.x]) atomicAdd(&st[0].hist[threadIdx.x], h[0][threadIdx.x]);
        if (h[1][threadIdx.x]) atomicAdd(&st[1].hist[threadIdx.x], h[1][threadIdx.x]);
    }
}

static void launch_select_hist(const float *val, long n, int mode, int shift, SelState *st, hipStream_t s)
{
    const long blocks = std::max<long>(1, std::min<long>(HIST_BLOCKS, (n + 8 * HIST_TB - 1) / (8 * HIST_TB)));
    hipLaunchKernelGGL(select_hist_kernel, dim3((unsigned)blocks), dim3(HIST_TB), 0, s, val, n, mode, shift, st);
}

// picks the digit that contains the krem-th smallest remaining key; on the last pass the prefix is
// the threshold and krem the number of entries equal to it that still have to go.
__global__ void select_pick_kernel(SelState *st, int last)
{
    SelState &s = st[blockIdx.x];
    __shared__ uint32_t inc[2][256];          // running sums of the histogram (256 threads, eight doubling steps)
    __shared__ int first;
    const int t = threadIdx.x;
    const uint32_t mine = s.hist[t];
    inc[0][t] = mine;
    if (t == 0) first = 255;
    __syncthreads();
    int cur = 0;
    for (int o = 1; o < 256; o <<= 1) {
        inc[cur ^ 1][t] = inc[cur][t] + (t >= o ? inc[cur][t - o] : 0u);
        cur ^= 1;
        __syncthreads();
    }
    // the first digit (below 255) whose running sum reaches krem, else digit 255
    const uint32_t krem = s.krem;
    if (t < 255 && inc[cur][t] >= krem) atomicMin(&first, t);
    __syncthreads();
    const int d = first;
    __syncthreads();                           // every thread has read krem and first before they change
    if (t == d && s.active) {
        s.krem = krem - (inc[cur][t] - mine);  // minus the entries in the digits below d
        s.prefix = (s.prefix << 8) | (uint32_t)d;
        if (last) { s.thresh = s.prefix; s.need = s.krem; }
    }
    s.hist[t] = 0;
}

// tie[p] = 1 in the low (class 0) or high (class 1) half iff |val[p]| equals its class threshold
__global__ void tie_flag_kernel(const float *val, long n, int mode, const SelState *st, uint64_t *tie)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p > n) return;
    uint64_t t = 0;
    if (p < n) {
        const float w = val[p];
        const int c = weight_class(w, mode);
        const uint32_t mag = __float_as_uint(w) & 0x7FFFFFFFu;
        if (st[c].active && mag == st[c].thresh) t = c ? (1ull << 32) : 1ull;
    }
    tie[p] = t;
}

// keep[p] = 0 iff the entry is among the removed ones: magnitude below the threshold, or equal to
// it and among the first `need` such entries in CSR order (= smallest flat positions).
__global__ void keep_flag_kernel(const float *val, long n, int mode, const SelState *st, const uint64_t *trank,
                                 uint32_t *keep)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p > n) return;
    uint32_t k = 0;
    if (p < n) {
        const float w = val[p];
        const int c = weight_class(w, mode);
        const uint32_t mag = __float_as_uint(w) & 0x7FFFFFFFu;
        bool gone = false;
        if (st[c].active) {
            const uint32_t rank = c ? (uint32_t)(trank[p] >> 32) : (uint32_t)trank[p];
            gone = mag < st[c].thresh || (mag == st[c].thresh && rank < st[c].need);
        }
        k = gone ? 0u : 1u;
    }
    keep[p] = k;
}

// The same decisions for the prune / regrow cycle without device-wide scans over the connections: every workgroup of
// PRUNE_TILE consecutive entries (four per thread) counts its ties (tie_count_kernel), a scan over the per-workgroup
// counts gives each workgroup the number of ties before it, a second pass counts the survivors per workgroup
// (keep_count_kernel), and after the scan of those counts the compaction (compact_block_kernel) recomputes the
// decision and places the survivors.  Ranks and slots inside a workgroup come from a wavefront prefix sum of the
// threads' counts.  Entry n is a sentinel that is never kept.
constexpr int PRUNE_PER = 4, PRUNE_TILE = PRUNE_PER * TB;

__device__ __forceinline__ uint32_t block_excl_sum(uint32_t v, uint32_t *wave_tot, uint32_t &block_total)
{
    const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
    uint32_t inc = v;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t t = __shfl_up(inc, o);
        if (lane >= o) inc += t;
    }
    __syncthreads();                       // wave_tot may still be read from an earlier call
    if (lane == 63) wave_tot[wv] = inc;
    __syncthreads();
    uint32_t off = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < TB / 64; ++w) {
        const uint32_t c = wave_tot[w];
        if (w < wv) off += c;
        tot += c;
    }
    block_total = tot;
    return off + inc - v;
}

// the thread's four entries p0 .. p0+3 (those below n): magnitude, class, whether the class prunes at all, tie with its threshold
struct Quad {
    float w[PRUNE_PER];
    uint32_t mag[PRUNE_PER];
    int c[PRUNE_PER];
    bool active[PRUNE_PER], tie[PRUNE_PER];
};
__device__ __forceinline__ Quad quad_of(const float *val, long p0, long n, int mode, const SelState *st)
{
    Quad q;
    if (p0 + PRUNE_PER <= n) {
        const float4 v = *(const float4 *)(val + p0);
        q.w[0] = v.x; q.w[1] = v.y; q.w[2] = v.z; q.w[3] = v.w;
    } else {
#pragma unroll
        for (int e = 0; e < PRUNE_PER; ++e) q.w[e] = p0 + e < n ? val[p0 + e] : 0.f;
    }
#pragma unroll
    for (int e = 0; e < PRUNE_PER; ++e) {
        const bool in = p0 + e < n;
        q.c[e] = weight_class(q.w[e], mode);
        q.mag[e] = __float_as_uint(q.w[e]) & 0x7FFFFFFFu;
        q.active[e] = in && st[q.c[e]].active != 0;
        q.tie[e] = q.active[e] && q.mag[e] == st[q.c[e]].thresh;
    }
    return q;
}
__device__ __forceinline__ void tie_counts(const Quad &q, uint32_t &n0, uint32_t &n1)
{
    n0 = 0; n1 = 0;
#pragma unroll
    for (int e = 0; e < PRUNE_PER; ++e) {
        n0 += (q.tie[e] && q.c[e] == 0) ? 1u : 0u;
        n1 += (q.tie[e] && q.c[e] == 1) ? 1u : 0u;
    }
}

__global__ __launch_bounds__(TB) void tie_count_kernel(const float *val, long n, int mode, const SelState *st, uint64_t *blk_tie)
{
    __shared__ uint32_t wt[TB / 64];
    const long p0 = ((long)blockIdx.x * TB + threadIdx.x) * PRUNE_PER;
    const Quad q = quad_of(val, p0, n, mode, st);
    uint32_t n0, n1, t0, t1;
    tie_counts(q, n0, n1);
    block_excl_sum(n0, wt, t0);
    block_excl_sum(n1, wt, t1);
    if (threadIdx.x == 0) blk_tie[blockIdx.x] = ((uint64_t)t1 << 32) | t0;
}

// keep = not among the removed ones: magnitude below the threshold, or equal to it and among the first `need` such
// entries in CSR order (= smallest flat positions).  Returns the four decisions as bits.
__device__ __forceinline__ uint32_t keep_of(const Quad &q, long p0, long n, const SelState *st, uint64_t ties_before_block,
                                            uint32_t *wt)
{
    uint32_t n0, n1, tot;
    tie_counts(q, n0, n1);
    uint32_t r0 = (uint32_t)ties_before_block + block_excl_sum(n0, wt, tot);
    uint32_t r1 = (uint32_t)(ties_before_block >> 32) + block_excl_sum(n1, wt, tot);
    uint32_t bits = 0;
#pragma unroll
    for (int e = 0; e < PRUNE_PER; ++e) {
        bool keep = p0 + e < n;
        if (q.active[e]) {
            const uint32_t rank = q.c[e] ? r1 : r0;
            if (q.mag[e] < st[q.c[e]].thresh || (q.tie[e] && rank < st[q.c[e]].need)) keep = false;
            if (q.tie[e]) { if (q.c[e]) ++r1; else ++r0; }
        }
        bits |= keep ? (1u << e) : 0u;
    }
    return bits;
}

__global__ __launch_bounds__(TB) void keep_count_kernel(const float *val, long n, int mode, const SelState *st,
                                                        const uint64_t *blk_tie_off, uint32_t *blk_keep)
{
    __shared__ uint32_t wt[TB / 64];
    const long p0 = ((long)blockIdx.x * TB + threadIdx.x) * PRUNE_PER;
    const Quad q = quad_of(val, p0, n, mode, st);
    const uint32_t bits = keep_of(q, p0, n, st, blk_tie_off[blockIdx.x], wt);
    uint32_t kept;
    block_excl_sum((uint32_t)__popc(bits), wt, kept);
    if (threadIdx.x == 0) blk_keep[blockIdx.x] = kept;
}

// kscan[p] = survivors before entry p (for p = 0 .. n; the row pointers of the survivors are read from it)
__global__ __launch_bounds__(TB) void compact_block_kernel(const float *val, long n, int mode, const SelState *st,
                                                           const uint64_t *blk_tie_off, const uint32_t *blk_keep_off,
                                                           const int *col, const float *vel, uint32_t *kscan, int *s_col,
                                                           float *s_val, float *s_vel)
{
    __shared__ uint32_t wt[TB / 64];
    const long p0 = ((long)blockIdx.x * TB + threadIdx.x) * PRUNE_PER;
    const Quad q = quad_of(val, p0, n, mode, st);
    const uint32_t bits = keep_of(q, p0, n, st, blk_tie_off[blockIdx.x], wt);
    uint32_t kept;
    uint32_t d = blk_keep_off[blockIdx.x] + block_excl_sum((uint32_t)__popc(bits), wt, kept);
    if (p0 > n) return;
    int ci[PRUNE_PER];
    float ve[PRUNE_PER];
    if (p0 + PRUNE_PER <= n) {
        const int4 c4 = *(const int4 *)(col + p0);
        const float4 v4 = *(const float4 *)(vel + p0);
        ci[0] = c4.x; ci[1] = c4.y; ci[2] = c4.z; ci[3] = c4.w;
        ve[0] = v4.x; ve[1] = v4.y; ve[2] = v4.z; ve[3] = v4.w;
    } else {
#pragma unroll
        for (int e = 0; e < PRUNE_PER; ++e) {
            ci[e] = p0 + e < n ? col[p0 + e] : 0;
            ve[e] = p0 + e < n ? vel[p0 + e] : 0.f;
        }
    }
    uint32_t ks[PRUNE_PER];
#pragma unroll
    for (int e = 0; e < PRUNE_PER; ++e) {
        ks[e] = d;
        if (bits & (1u << e)) {
            s_col[d] = ci[e];
            s_val[d] = q.w[e];
            s_vel[d] = ve[e];
            ++d;
        }
    }
    if (p0 + PRUNE_PER <= n + 1) {
        *(uint4 *)(kscan + p0) = make_uint4(ks[0], ks[1], ks[2], ks[3]);
    } else {
#pragma unroll
        for (int e = 0; e < PRUNE_PER; ++e)
            if (p0 + e <= n) kscan[p0 + e] = ks[e];
    }
}

__global__ void compact_kernel(long n, const uint32_t *keep, const uint32_t *kscan, const int *col, const float *val,
                               const float *vel, int *s_col, float *s_val, float *s_vel)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= n || !keep[p]) return;
    const uint32_t d = kscan[p];
    s_col[d] = col[p];
    s_val[d] = val[p];
    s_vel[d] = vel[p];
}

__global__ void survivor_rowptr_kernel(int n_rows, const int *rowptr, const uint32_t *kscan, int *rowptr_s)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r > n_rows) return;
    rowptr_s[r] = (int)kscan[rowptr[r]];   // kscan has n+1 entries; kscan[n] = number of survivors
}

// ------------------------------------------------------------------------------------------------
// Sampler: k distinct empty positions.
// sparse mode: candidate t -> position (row, col) from Philox(purpose 1, index t); a candidate is
//   accepted iff it is not occupied and no earlier candidate had the same position; the first k
//   accepted candidates (in t order) are the result.  Evaluated for a whole window of t at once:
//   stable sort by position, first-of-run + not-occupied test, prefix count in t order.
// dense mode: every empty position gets a 64-bit Philox ordering key (purpose 2); the k smallest
//   (key, position) are the result.
// ------------------------------------------------------------------------------------------------
__global__ void cand_kernel(long W, Rng r, uint32_t n_in, uint32_t n_out, uint64_t *key, uint32_t *pay)
{
    const long t = (long)blockIdx.x * TB + threadIdx.x;
    if (t >= W) return;
    uint32_t o[4];
    philox((uint32_t)t, (uint32_t)((uint64_t)t >> 32), 1u, r.generation, r.k0, r.k1, o);
    const uint64_t j = ((uint64_t)o[0] * n_out) >> 32;
    const uint64_t i = ((uint64_t)o[1] * n_in) >> 32;
    key[t] = j * n_in + i;
    pay[t] = (uint32_t)t;
}

__device__ inline bool occupied(const int *rowptr_s, const int *s_col, uint32_t n_in, uint64_t p)
{
    const int j = (int)(p / n_in), i = (int)(p % n_in);
    const int lo = rowptr_s[j], hi = rowptr_s[j + 1];
    const int q = lower_bound_i32(s_col, lo, hi, i);
    return q < hi && s_col[q] == i;
}

// in sorted order: ok = first of its run and not occupied; scattered to t order as well
__global__ void cand_ok_kernel(long W, const uint64_t *key, const uint32_t *pay, const int *rowptr_s,
                               const int *s_col, uint32_t n_in, uint32_t *ok_sorted, uint32_t *ok_by_t)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x > W) return;
    if (x == W) { ok_sorted[W] = 0; ok_by_t[W] = 0; return; }
    const uint64_t p = key[x];
    const bool ok = (x == 0 || key[x - 1] != p) && !occupied(rowptr_s, s_col, n_in, p);
    ok_sorted[x] = ok;
    ok_by_t[pay[x]] = ok;
}

// The number of accepted candidates before candidate t never decreases with t, so "fewer than k accepted candidates
// precede it" holds exactly for t < T, T = the first t whose count reaches k: one search, then a comparison per
// candidate instead of a gather per candidate.
__global__ void cand_limit_kernel(long W, const uint32_t *rank_by_t, uint32_t k, uint32_t *limit)
{
    if (threadIdx.x != 0 || blockIdx.x != 0) return;
    long lo = 0, hi = W;                       // rank_by_t has W + 1 entries and rank_by_t[W] >= k
    while (lo < hi) {
        const long mid = lo + ((hi - lo) >> 1);
        if (rank_by_t[mid] < k) lo = mid + 1; else hi = mid;
    }
    *limit = (uint32_t)lo;
}
// in sorted order: selected = ok and candidate index below the limit
__global__ void cand_select_kernel(long W, const uint32_t *pay, const uint32_t *limit, uint32_t *ok_sorted)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x >= W) return;
    ok_sorted[x] = (ok_sorted[x] && pay[x] < *limit) ? 1u : 0u;
}

__global__ void gather_selected_kernel(long W, const uint32_t *sel, const uint32_t *sscan, const uint64_t *key,
                                       uint64_t *new_p)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x >= W || !sel[x]) return;
    new_p[sscan[x]] = key[x];
}

// dense mode
__global__ void empty_flag_kernel(long M, const int *rowptr_s, const int *s_col, uint32_t n_in, uint32_t *flag)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p > M) return;
    flag[p] = (p < M && !occupied(rowptr_s, s_col, n_in, (uint64_t)p)) ? 1u : 0u;
}
__global__ void empty_key_kernel(long M, const uint32_t *flag, const uint32_t *fscan, Rng r, uint64_t *key,
                                 uint32_t *pay)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= M || !flag[p]) return;
    uint32_t o[4];
    philox((uint32_t)p, (uint32_t)((uint64_t)p >> 32), 2u, r.generation, r.k0, r.k1, o);
    const uint32_t d = fscan[p];
    key[d] = ((uint64_t)o[0] << 32) | o[1];
    pay[d] = (uint32_t)p;
}
__global__ void zero_u32_kernel(long n, uint32_t *a)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p < n) a[p] = 0;
}
__global__ void mark_chosen_kernel(long k, const uint32_t *pay_sorted, uint32_t *flag)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x < k) flag[pay_sorted[x]] = 1u;
}
__global__ void gather_marked_kernel(long M, const uint32_t *flag, const uint32_t *fscan, uint64_t *new_p)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= M || !flag[p]) return;
    new_p[fscan[p]] = (uint64_t)p;
}

// ------------------------------------------------------------------------------------------------
// Merge survivors (CSR order) and the sorted new positions into the final CSR.
// ------------------------------------------------------------------------------------------------
__global__ void merge_rowptr_kernel(int n_rows, uint32_t n_in, const int *rowptr_s, const uint64_t *new_p, long k,
                                    int *rowptr)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r > n_rows) return;
    rowptr[r] = rowptr_s[r] + (int)lower_bound_u64(new_p, k, (uint64_t)r * n_in);
}
// The new CSR is written front to back, eight consecutive slots per thread, so that every array is stored once in
// whole cache lines.  Inside a row the survivors and the new connections are both ascending by column, and a slot's
// rank in their union says how many of each precede it (a bisection).  merge_tile_kernel does that for the first slot
// of every tile of MERGE_TILE slots, which fixes the runs of survivors and of new connections that the tile consumes;
// the tile's workgroup copies exactly those runs into LDS (coalesced), each thread bisects for its own first slot and
// then walks: the next slot takes the smaller of the next survivor and the next new connection, and both cursors run
// on through the following rows, whose entries follow in the same two arrays.
// The merge also leaves (row, weight, velocity) of every slot packed in 16 bytes for the rebuild of the transposed
// view, which then needs one 16-byte gather per connection, and (KEYS) the (column, slot) pairs that view is sorted from.
struct __align__(16) RowValVel { int row; float val; float vel; int pad; };
constexpr int MERGE_RUN = 8;                    // consecutive slots per thread
constexpr int MERGE_TILE = MERGE_RUN * TB;      // slots per block

// survivors of row j left of the slot of rank m in the row, searched in [a_lo, a_hi]; A(i) / B(i) = column of the
// row's i-th survivor / i-th new connection
template <typename FA, typename FB>
__device__ __forceinline__ int merge_split(int m, int a_lo, int a_hi, FA &&A, FB &&B)
{
    while (a_lo < a_hi) {
        const int mid = (a_lo + a_hi) >> 1;
        if (A(mid) < B(m - mid - 1)) a_lo = mid + 1; else a_hi = mid;
    }
    return a_lo;
}

// per tile: x, y = first and last row with a slot in the tile; z, w = survivors and new connections consumed by the
// tiles before it.  Entry n_tiles closes the list with (.., .., ns, k).
__global__ void merge_tile_kernel(long n_tiles, int n_rows, uint32_t n_in, const int *rowptr_s, const int *rowptr,
                                  const int *s_col, const uint64_t *new_p, long nnz, long ns, long k, int4 *tile)
{
    const long b = (long)blockIdx.x * TB + threadIdx.x;
    if (b > n_tiles) return;
    if (b == n_tiles) { tile[b] = make_int4(n_rows - 1, n_rows - 1, (int)ns, (int)k); return; }
    const long first = b * MERGE_TILE, last = min(first + MERGE_TILE, nnz) - 1;
    const int j = row_of(rowptr, n_rows, (int)first);
    const int d0 = rowptr[j], s0 = rowptr_s[j];
    const int na = rowptr_s[j + 1] - s0, nb = (rowptr[j + 1] - d0) - na;
    const long t0 = (long)d0 - s0;
    const int m = (int)(first - d0);
    const uint64_t base = (uint64_t)j * n_in;
    const int a = merge_split(m, max(0, m - nb), min(m, na), [&](int i) { return (uint64_t)s_col[s0 + i]; },
                              [&](int i) { return new_p[t0 + i] - base; });
    tile[b] = make_int4(j, row_of(rowptr, n_rows, (int)last), s0 + a, (int)(t0 + (m - a)));
}

template <bool KEYS>
__global__ __launch_bounds__(TB) void merge_rows_kernel(long nnz, uint32_t n_in, const int4 *tile, const int *rowptr_s,
                                                        const int *rowptr, const int *s_col, const float *s_val,
                                                        const float *s_vel, const uint64_t *new_p, Rng rng, float limit,
                                                        int *col, float *val, float *vel, RowValVel *packed, uint32_t *key,
                                                        uint32_t *pay)
{
    __shared__ int l_col[MERGE_TILE];
    __shared__ float l_val[MERGE_TILE], l_vel[MERGE_TILE];
    __shared__ uint64_t l_new[MERGE_TILE];
    const int4 here = tile[blockIdx.x], next = tile[blockIdx.x + 1];
    const int SA0 = here.z, TB0 = here.w;
    const int n_sa = min(next.z - SA0, MERGE_TILE), n_tb = min(next.w - TB0, MERGE_TILE);   // they add up to the tile's slots
    for (int i = threadIdx.x; i < n_sa; i += TB) {
        l_col[i] = s_col[SA0 + i];
        l_val[i] = s_val[SA0 + i];
        l_vel[i] = s_vel[SA0 + i];
    }
    for (int i = threadIdx.x; i < n_tb; i += TB) l_new[i] = new_p[TB0 + i];
    __syncthreads();
    const long d_first = (long)blockIdx.x * MERGE_TILE + (long)threadIdx.x * MERGE_RUN;
    const int run = (int)max(0L, min((long)MERGE_RUN, nnz - d_first));
    int ci[MERGE_RUN], rj[MERGE_RUN];
    float cw[MERGE_RUN], cv[MERGE_RUN];
#pragma unroll
    for (int u = 0; u < MERGE_RUN; ++u) { ci[u] = 0; rj[u] = 0; cw[u] = 0.f; cv[u] = 0.f; }
    if (run > 0) {
        int lo = here.x, hi = here.y;                  // the last row that starts at or before the first slot
        while (lo < hi) {
            const int mid = (lo + hi + 1) >> 1;
            if (rowptr[mid] <= d_first) lo = mid; else hi = mid - 1;
        }
        int j = lo;
        int sa, tb;                                    // cursors into the tile's runs: next survivor, next new connection
        int s_end, row_end;                            // end of row j in the survivor array and in the new CSR
        {
            const int d0 = rowptr[j], s0 = rowptr_s[j];
            s_end = rowptr_s[j + 1];
            row_end = rowptr[j + 1];
            const int na = s_end - s0, nb = (row_end - d0) - na;
            const int t0 = d0 - s0;
            const int m = (int)(d_first - d0);         // rank of the first slot in its row
            const uint64_t base = (uint64_t)j * n_in;
            // the cursors at this slot lie inside the tile's runs, which bounds the search to what LDS holds
            const int a_lo = max(max(0, m - nb), max(SA0 - s0, m - (TB0 + n_tb - t0)));
            const int a_hi = min(min(m, na), min(SA0 + n_sa - s0, m - (TB0 - t0)));
            const int a = merge_split(m, a_lo, a_hi, [&](int i) { return (uint64_t)l_col[s0 + i - SA0]; },
                                      [&](int i) { return l_new[t0 + i - TB0] - base; });
            sa = s0 + a - SA0;
            tb = t0 + (m - a) - TB0;
        }
#pragma unroll
        for (int u = 0; u < MERGE_RUN; ++u) {
            if (u < run) {
                while (d_first + u >= row_end) {       // on to the next row that has a slot (empty rows are skipped)
                    ++j;
                    s_end = rowptr_s[j + 1];
                    row_end = rowptr[j + 1];
                }
                const int sa_end = min(s_end - SA0, n_sa);             // end of row j in the tile's run of survivors
                const int tb_end = min(row_end - s_end - TB0, n_tb);   // and in its run of new connections
                const uint64_t base = (uint64_t)j * n_in;
                const int ca = sa < sa_end ? l_col[sa] : 0;
                const uint64_t pb = tb < tb_end ? l_new[tb] : 0;
                const bool survivor = sa < sa_end && (tb >= tb_end || (uint64_t)ca < pb - base);
                rj[u] = j;
                if (survivor) { ci[u] = ca; cw[u] = l_val[sa]; cv[u] = l_vel[sa]; ++sa; }
                else { ci[u] = (int)(pb - base); cw[u] = fresh_weight(rng, pb, limit); ++tb; }
            }
        }
    }
    // The results change hands through LDS (the input runs are no longer needed) so that every store instruction of a
    // wavefront covers one contiguous kilobyte.
    __syncthreads();
    int *l_row = (int *)l_new;
    {
        const int o = threadIdx.x * MERGE_RUN;
#pragma unroll
        for (int h = 0; h < MERGE_RUN; h += 4) {
            *(int4 *)(l_col + o + h) = make_int4(ci[h], ci[h + 1], ci[h + 2], ci[h + 3]);
            *(float4 *)(l_val + o + h) = make_float4(cw[h], cw[h + 1], cw[h + 2], cw[h + 3]);
            *(float4 *)(l_vel + o + h) = make_float4(cv[h], cv[h + 1], cv[h + 2], cv[h + 3]);
            *(int4 *)(l_row + o + h) = make_int4(rj[h], rj[h + 1], rj[h + 2], rj[h + 3]);
        }
    }
    __syncthreads();
    const long D0 = (long)blockIdx.x * MERGE_TILE;
    const int cnt = (int)min((long)MERGE_TILE, nnz - D0);
    for (int i4 = threadIdx.x; 4 * i4 + 3 < cnt; i4 += TB) {
        const int4 c = *(const int4 *)(l_col + 4 * i4);
        *(int4 *)(col + D0 + 4 * i4) = c;
        *(float4 *)(val + D0 + 4 * i4) = *(const float4 *)(l_val + 4 * i4);
        *(float4 *)(vel + D0 + 4 * i4) = *(const float4 *)(l_vel + 4 * i4);
        if (KEYS) {
            *(uint4 *)(key + D0 + 4 * i4) = make_uint4(c.x, c.y, c.z, c.w);
            const uint32_t q = (uint32_t)(D0 + 4 * i4);
            *(uint4 *)(pay + D0 + 4 * i4) = make_uint4(q, q + 1, q + 2, q + 3);
        }
    }
    for (int i = (cnt & ~3) + threadIdx.x; i < cnt; i += TB) {
        col[D0 + i] = l_col[i]; val[D0 + i] = l_val[i]; vel[D0 + i] = l_vel[i];
        if (KEYS) { key[D0 + i] = (uint32_t)l_col[i]; pay[D0 + i] = (uint32_t)(D0 + i); }
    }
    if (packed)
        for (int i = threadIdx.x; i < cnt; i += TB) packed[D0 + i] = RowValVel{l_row[i], l_val[i], l_vel[i], 0};
}
__global__ void pack_rows_kernel(int n_rows, const int *ptr, const float *val, const float *vel, RowValVel *packed)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r >= n_rows) return;
    for (int p = ptr[r]; p < ptr[r + 1]; ++p) packed[p] = RowValVel{r, val[p], vel[p], 0};
}
__global__ void csc_fill_packed_kernel(long n, const uint32_t *pos_sorted, const RowValVel *packed, int *rowidx, int *csr_pos,
                                       float *valT, float *velT)
{
    const long q = (long)blockIdx.x * TB + threadIdx.x;
    if (q >= n) return;
    const int p = (int)pos_sorted[q];
    const RowValVel e = packed[p];
    csr_pos[q] = p;
    rowidx[q] = e.row;
    valT[q] = e.val;
    velT[q] = e.vel;
}
__global__ void copy_u32_kernel(const uint32_t *src, uint32_t *dst)
{
    if (threadIdx.x == 0 && blockIdx.x == 0) *dst = *src;
}

// ------------------------------------------------------------------------------------------------
// Derived structures
// ------------------------------------------------------------------------------------------------
__global__ void max_len_kernel(int n_rows, const int *ptr, int *out)
{
    __shared__ int part[TB / 64];
    int m = 0;
    for (long r = (long)blockIdx.x * TB + threadIdx.x; r < n_rows; r += (long)gridDim.x * TB)
        m = max(m, ptr[r + 1] - ptr[r]);
    for (int s = 32; s >= 1; s >>= 1) m = max(m, __shfl_xor(m, s));
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = m;
    __syncthreads();
    if (threadIdx.x == 0) {                    // one atomic per block, on a few hundred blocks
        for (int w = 1; w < TB / 64; ++w) m = max(m, part[w]);
        atomicMax(out, m);
    }
}
__global__ void vcount_kernel(int n_rows, const int *ptr, int seg, uint32_t *cnt)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r > n_rows) return;
    uint32_t c = 0;
    if (r < n_rows) {
        const int len = ptr[r + 1] - ptr[r];
        c = len <= seg ? 1u : (uint32_t)((len + seg - 1) / seg);
    }
    cnt[r] = c;
}
// one thread per virtual row: its row is the last r with rvptr[r] <= v
__global__ void vfill_kernel(int n_rows, const int *ptr, int seg, const int *rvptr, int *vptr, int *v2row, int nnz, int nv)
{
    const int v = blockIdx.x * TB + threadIdx.x;
    if (v > nv) return;
    if (v == nv) { vptr[nv] = nnz; return; }
    const int r = row_of(rvptr, n_rows, v);
    vptr[v] = ptr[r] + (v - rvptr[r]) * seg;
    v2row[v] = r;
}
__global__ void iota_copy_kernel(long n, const int *col, uint32_t *key, uint32_t *pay)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= n) return;
    key[p] = (uint32_t)col[p];
    pay[p] = (uint32_t)p;
}
__global__ void colptr_kernel(int n_cols, const uint32_t *key_sorted, long n, int *colptr)
{
    const int c = blockIdx.x * TB + threadIdx.x;
    if (c > n_cols) return;
    long lo = 0, hi = n;
    while (lo < hi) {
        const long mid = lo + ((hi - lo) >> 1);
        if (key_sorted[mid] < (uint32_t)c) lo = mid + 1; else hi = mid;
    }
    colptr[c] = (int)lo;
}
// transposed view of a matrix with few, long rows: the row of a CSR slot is found by search in the row pointers
__global__ void csc_fill_kernel(long n, int n_rows, const int *rowptr, const uint32_t *pos_sorted, const float *val,
                                const float *vel, int *rowidx, int *csr_pos, float *valT, float *velT)
{
    const long q = (long)blockIdx.x * TB + threadIdx.x;
    if (q >= n) return;
    const int p = (int)pos_sorted[q];
    csr_pos[q] = p;
    rowidx[q] = row_of(rowptr, n_rows, p);
    valT[q] = val[p];
    velT[q] = vel[p];
}
__global__ void scatter_f32_kernel(long n, const int *pos, const float *src, float *dst)
{
    const long q = (long)blockIdx.x * TB + threadIdx.x;
    if (q < n) dst[pos[q]] = src[q];
}
__global__ void fill_f32_kernel(long n, float *a, float v)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p < n) a[p] = v;
}
__global__ void fill_i32_kernel(long n, int *a, int v)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p < n) a[p] = v;
}

// ------------------------------------------------------------------------------------------------
// Importance Pruning (eq. 4 and Algorithm 2): I_j = sum of |w| over the incoming connections of
// neuron j, added in fp32 in stored order (one thread per neuron, so that the value -- and with it
// the decision I_j < t -- is the same whoever evaluates it); every connection of a neuron with
// I_j < t is removed.
// ------------------------------------------------------------------------------------------------
__global__ void importance_kernel(int n_rows, const int *rowptr, const float *val, float *imp)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r >= n_rows) return;
    float s = 0.f;
    for (int p = rowptr[r]; p < rowptr[r + 1]; ++p) s = s + fabsf(val[p]);
    imp[r] = s;
}
__global__ void importance_keep_kernel(long n, int n_rows, const int *rowptr, const float *imp, float threshold,
                                       uint32_t *keep)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p > n) return;
    keep[p] = (p < n && !(imp[row_of(rowptr, n_rows, (int)p)] < threshold)) ? 1u : 0u;
}
__global__ void copy_back_kernel(long n, const int *s_col, const float *s_val, const float *s_vel, int *col, float *val,
                                 float *vel)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= n) return;
    col[p] = s_col[p];
    val[p] = s_val[p];
    vel[p] = s_vel[p];
}

// ------------------------------------------------------------------------------------------------
// Sparse model averaging (eq. 2, last step of Algorithm 1): the stored entries of K replicas are
// keyed by flat position, sorted stably (equal positions stay in replica order), every run of equal
// positions is added in fp32 in that order and divided by K (a connection missing from a replica
// counts as zero), and the union is pruned back by magnitude with the radix select of the evolution.
// ------------------------------------------------------------------------------------------------
__global__ void avg_keys_kernel(long n, int n_rows, uint32_t n_in, const int *rowptr, const int *col, const float *val,
                                long offset, uint64_t *key, uint32_t *pay, float *vals)
{
    const long p = (long)blockIdx.x * TB + threadIdx.x;
    if (p >= n) return;
    key[offset + p] = (uint64_t)row_of(rowptr, n_rows, (int)p) * n_in + (uint64_t)col[p];
    pay[offset + p] = (uint32_t)(offset + p);
    vals[offset + p] = val[p];
}
__global__ void avg_head_kernel(long T, const uint64_t *key, uint32_t *head)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x > T) return;
    head[x] = (x < T && (x == 0 || key[x] != key[x - 1])) ? 1u : 0u;
}
__global__ void avg_sum_kernel(long T, const uint64_t *key, const uint32_t *pay, const float *vals, const uint32_t *head,
                               const uint32_t *uidx, float K, uint64_t *ukey, float *uval)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x >= T || !head[x]) return;
    const uint64_t k = key[x];
    float sum = vals[pay[x]];
    for (long y = x + 1; y < T && key[y] == k; ++y) sum = sum + vals[pay[y]];
    ukey[uidx[x]] = k;
    uval[uidx[x]] = sum / K;
}
__global__ void avg_compact_kernel(long U, const uint32_t *keep, const uint32_t *kscan, const uint64_t *ukey,
                                   const float *uval, uint32_t n_in, int *col, float *val, float *vel)
{
    const long x = (long)blockIdx.x * TB + threadIdx.x;
    if (x >= U || !keep[x]) return;
    const uint32_t d = kscan[x];
    col[d] = (int)(ukey[x] % n_in);
    val[d] = uval[x];
    vel[d] = 0.f;
}
__global__ void avg_rowptr_kernel(int n_rows, uint32_t n_in, const uint64_t *ukey, long U, const uint32_t *kscan, int *rowptr)
{
    const int r = blockIdx.x * TB + threadIdx.x;
    if (r > n_rows) return;
    rowptr[r] = (int)kscan[lower_bound_u64(ukey, U, (uint64_t)r * n_in)];   // kscan[U] = number kept
}
struct BiasPtrs { const float *b[16]; };
__global__ void avg_bias_kernel(int n, BiasPtrs src, int K, float *bias, float *bias_vel)
{
    const int j = blockIdx.x * TB + threadIdx.x;
    if (j >= n) return;
    float s = src.b[0][j];
    for (int k = 1; k < K; ++k) s = s + src.b[k][j];
    bias[j] = s / (float)K;
    bias_vel[j] = 0.f;
}

// ------------------------------------------------------------------------------------------------
// host orchestration
// ------------------------------------------------------------------------------------------------
template <typename T>
static T *at(sl_layer *L, size_t off) { return reinterpret_cast<T *>(L->scratch + off); }

static int read_back(sl_layer *L, void *host, const void *dev, size_t bytes, hipStream_t s)
{
    SL_HIP(L, hipMemcpyAsync(host, dev, bytes, hipMemcpyDeviceToHost, s));
    SL_HIP(L, hipStreamSynchronize(s));
    return SL_OK;
}

static Rng make_rng(const sl_layer *L, uint32_t generation)
{
    Rng r;
    r.k0 = (uint32_t)L->cfg.seed ^ (uint32_t)(L->cfg.layer_id * 0x9E3779B9u);
    r.k1 = (uint32_t)(L->cfg.seed >> 32);
    r.generation = generation;
    return r;
}

// slots of the `small` scratch region (one read-back fetches what several steps left there)
enum { SMALL_MAXLEN_F = 0, SMALL_MAXLEN_B = 1, SMALL_KEPT = 2, SMALL_ACCEPTED = 3, SMALL_CLASS = 4, SMALL_LIMIT = 5 };

static bool short_rows(const sl_layer *L)   // many rows, none of them expected to be long: the per-row kernels apply
{
    return L->cfg.n_out >= 8192 && L->nnz <= 512 * L->cfg.n_out;
}

static void launch_max_len(sl_layer *L, const SegMat &m, int slot, hipStream_t s)
{
    int *small = at<int>(L, L->cp.small);
    hipLaunchKernelGGL(fill_i32_kernel, dim3(1), dim3(TB), 0, s, 1L, small + slot, 0);
    hipLaunchKernelGGL(max_len_kernel, dim3(std::min(256u, nblk(m.n_rows))), dim3(TB), 0, s, m.n_rows, m.ptr, small + slot);
}

static int finish_vrows(sl_layer *L, SegMat &m, int nnz, int maxlen, hipStream_t s)
{
    m.seg = choose_seg(m.n_rows, nnz);
    if (maxlen <= m.seg) {
        m.split = 0; m.vptr = m.ptr; m.v2row = nullptr; m.rvptr = nullptr; m.nv = m.n_rows;
        return SL_OK;
    }
    uint32_t *cnt = at<uint32_t>(L, L->cp.f0);
    hipLaunchKernelGGL(vcount_kernel, dim3(nblk(m.n_rows + 1)), dim3(TB), 0, s, m.n_rows, m.ptr, m.seg, cnt);
    SL_HIP(L, scan_excl<uint32_t>(at<char>(L, L->cp.temp), L->cp.temp_bytes, cnt, (uint32_t *)m.rvptr_store,
                                  (size_t)m.n_rows + 1, s));
    int nv = 0;
    int rc = read_back(L, &nv, m.rvptr_store + m.n_rows, sizeof(int), s);
    if (rc) return rc;
    if (nv > m.nv_cap) return set_err(L, SL_ENOMEM, "virtual rows %d exceed capacity %d", nv, m.nv_cap);
    hipLaunchKernelGGL(vfill_kernel, dim3(nblk(nv + 1)), dim3(TB), 0, s, m.n_rows, m.ptr, m.seg, m.rvptr_store,
                       m.vptr_store, m.v2row_store, nnz, nv);
    m.split = 1; m.vptr = m.vptr_store; m.v2row = m.v2row_store; m.rvptr = m.rvptr_store; m.nv = nv;
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

// from_merge: the merge has already left (row, weight, velocity) of every CSR slot in the `packed` scratch region and
// the (column, slot) pairs in the sort's input buffers
int topo_finalize(sl_layer *L, hipStream_t s, bool from_merge)
{
    const int n = (int)L->nnz, n_in = (int)L->cfg.n_in, n_out = (int)L->cfg.n_out;
    L->fwd.n_rows = n_out; L->fwd.ptr = L->rowptr; L->fwd.idx = L->colidx;
    launch_max_len(L, L->fwd, SMALL_MAXLEN_F, s);
    if (L->has_csc) {
        // CSC view: stable sort of (column, CSR position) keeps rows ascending inside a column
        uint32_t *kA = at<uint32_t>(L, L->cp.keyA), *kB = at<uint32_t>(L, L->cp.keyB);
        uint32_t *vA = at<uint32_t>(L, L->cp.payA), *vB = at<uint32_t>(L, L->cp.payB);
        uint32_t *ks = kA, *vs = vA;
        if (n > 0) {
            if (!from_merge)
                hipLaunchKernelGGL(iota_copy_kernel, dim3(nblk(n)), dim3(TB), 0, s, (long)n, L->colidx, kA, vA);
            SL_HIP(L, sort_pairs<uint32_t>(at<char>(L, L->cp.temp), L->cp.temp_bytes, kA, kB, vA, vB, (size_t)n,
                                           bit_length((uint64_t)n_in - 1), &ks, &vs, s));
            if (from_merge || short_rows(L)) {
                RowValVel *packed = at<RowValVel>(L, L->cp.packed);
                if (!from_merge)
                    hipLaunchKernelGGL(pack_rows_kernel, dim3(nblk(n_out)), dim3(TB), 0, s, n_out, L->rowptr, L->val, L->vel,
                                       packed);
                hipLaunchKernelGGL(csc_fill_packed_kernel, dim3(nblk(n)), dim3(TB), 0, s, (long)n, vs, packed, L->rowidx,
                                   L->csr_pos, L->valT, L->velT);
            } else {
                // few, long rows: the row of a CSR slot is found by search in the row pointers
                hipLaunchKernelGGL(csc_fill_kernel, dim3(nblk(n)), dim3(TB), 0, s, (long)n, n_out, L->rowptr, vs, L->val, L->vel,
                                   L->rowidx, L->csr_pos, L->valT, L->velT);
            }
        }
        hipLaunchKernelGGL(colptr_kernel, dim3(nblk(n_in + 1)), dim3(TB), 0, s, n_in, ks, (long)n, L->colptr);
        L->bwd.n_rows = n_in; L->bwd.ptr = L->colptr; L->bwd.idx = L->rowidx;
        launch_max_len(L, L->bwd, SMALL_MAXLEN_B, s);
    }
    SL_HIP(L, hipGetLastError());
    int maxlen[2] = {0, 0};
    int rc = read_back(L, maxlen, at<int>(L, L->cp.small) + SMALL_MAXLEN_F, sizeof(int) * (L->has_csc ? 2 : 1), s);
    if (rc) return rc;
    rc = finish_vrows(L, L->fwd, n, maxlen[0], s);
    if (rc || !L->has_csc) return rc;
    return finish_vrows(L, L->bwd, n, maxlen[1], s);
}

int topo_sync_csr_vel(sl_layer *L, hipStream_t s)
{
    if (!L->has_csc || L->nnz == 0) return SL_OK;
    hipLaunchKernelGGL(scatter_f32_kernel, dim3(nblk(L->nnz)), dim3(TB), 0, s, (long)L->nnz, L->csr_pos, L->velT, L->vel);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int topo_sync_csr_grad(sl_layer *L, float *grad_csr_dev, hipStream_t s)
{
    if (L->nnz == 0) return SL_OK;
    hipLaunchKernelGGL(scatter_f32_kernel, dim3(nblk(L->nnz)), dim3(TB), 0, s, (long)L->nnz, L->csr_pos, L->grad,
                       grad_csr_dev);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

// Draws k distinct positions that are empty w.r.t. the survivors (rowptr_s, s_col) into new_p,
// ascending.  n_occ = number of survivors.
// expect_kept >= 0: the survivor count that the caller left in the SMALL_KEPT slot must equal it (checked at the first
// read-back; -1: nothing to check)
static int sample_positions(sl_layer *L, long k, long n_occ, uint32_t generation, hipStream_t s, long expect_kept)
{
    if (k == 0) return SL_OK;
    const uint32_t n_in = (uint32_t)L->cfg.n_in, n_out = (uint32_t)L->cfg.n_out;
    const uint64_t M = (uint64_t)n_in * n_out;
    const Rng r = make_rng(L, generation);
    const int *rowptr_s = at<int>(L, L->cp.rowptr_s), *s_col = at<int>(L, L->cp.s_col);
    uint64_t *kA = at<uint64_t>(L, L->cp.keyA), *kB = at<uint64_t>(L, L->cp.keyB);
    uint32_t *vA = at<uint32_t>(L, L->cp.payA), *vB = at<uint32_t>(L, L->cp.payB);
    uint32_t *f0 = at<uint32_t>(L, L->cp.f0), *f1 = at<uint32_t>(L, L->cp.f1);
    uint32_t *f2 = at<uint32_t>(L, L->cp.f2), *f3 = at<uint32_t>(L, L->cp.f3);
    uint64_t *new_p = at<uint64_t>(L, L->cp.new_p);
    char *temp = at<char>(L, L->cp.temp);
    uint64_t *ks; uint32_t *vs;
    const bool dense_mode = (double)M <= 4.0 * (double)(n_occ + k);   // the definition's rule on the current nnz
    if (dense_mode && (int64_t)M > L->cp.w_cap) return set_err(L, SL_ENOMEM, "dense sampler needs %llu slots", (unsigned long long)M);
    if (dense_mode) {
        if (expect_kept >= 0) {
            uint32_t kept = 0;
            int rc = read_back(L, &kept, at<uint32_t>(L, L->cp.small) + SMALL_KEPT, sizeof(uint32_t), s);
            if (rc) return rc;
            if ((long)kept != expect_kept) return set_err(L, SL_ESTATE, "prune kept %u entries, expected %ld", kept, expect_kept);
        }
        const long Ml = (long)M;
        hipLaunchKernelGGL(empty_flag_kernel, dim3(nblk(Ml + 1)), dim3(TB), 0, s, Ml, rowptr_s, s_col, n_in, f0);
        SL_HIP(L, scan_excl<uint32_t>(temp, L->cp.temp_bytes, f0, f1, (size_t)Ml + 1, s));
        hipLaunchKernelGGL(empty_key_kernel, dim3(nblk(Ml)), dim3(TB), 0, s, Ml, f0, f1, r, kA, vA);
        const long n_empty = Ml - n_occ;
        SL_HIP(L, sort_pairs<uint64_t>(temp, L->cp.temp_bytes, kA, kB, vA, vB, (size_t)n_empty, 64u, &ks, &vs, s));
        hipLaunchKernelGGL(zero_u32_kernel, dim3(nblk(Ml + 1)), dim3(TB), 0, s, Ml + 1, f2);
        hipLaunchKernelGGL(mark_chosen_kernel, dim3(nblk(k)), dim3(TB), 0, s, k, vs, f2);
        SL_HIP(L, scan_excl<uint32_t>(temp, L->cp.temp_bytes, f2, f3, (size_t)Ml + 1, s));
        hipLaunchKernelGGL(gather_marked_kernel, dim3(nblk(Ml)), dim3(TB), 0, s, Ml, f2, f3, new_p);
        SL_HIP(L, hipGetLastError());
        return SL_OK;
    }
    // Acceptance of candidate t depends only on the candidates before it, so a window [0, W) that yields fewer than
    // k accepted positions is simply evaluated again twice as long, until k are accepted or the capacity is reached.
    const long cap = (L->sampler_max > 0 && L->sampler_max < L->cp.w_cap) ? (long)L->sampler_max : (long)L->cp.w_cap;
    long W = L->sampler_first > 0 ? (long)L->sampler_first : sampler_window((double)M, (double)n_occ, (double)k);
    for (;;) {
        if (W > cap) W = cap;
        hipLaunchKernelGGL(cand_kernel, dim3(nblk(W)), dim3(TB), 0, s, W, r, n_in, n_out, kA, vA);
        SL_HIP(L, sort_pairs<uint64_t>(temp, L->cp.temp_bytes, kA, kB, vA, vB, (size_t)W, bit_length(M - 1), &ks, &vs, s));
        hipLaunchKernelGGL(cand_ok_kernel, dim3(nblk(W + 1)), dim3(TB), 0, s, W, ks, vs, rowptr_s, s_col, n_in, f0, f1);
        SL_HIP(L, scan_excl<uint32_t>(temp, L->cp.temp_bytes, f1, f2, (size_t)W + 1, s));
        // one read-back fetches the number of accepted candidates and the survivor count that the pruning left
        uint32_t *small = at<uint32_t>(L, L->cp.small);
        hipLaunchKernelGGL(copy_u32_kernel, dim3(1), dim3(64), 0, s, f2 + W, small + SMALL_ACCEPTED);
        uint32_t both[2] = {0, 0};
        int rc = read_back(L, both, small + SMALL_KEPT, sizeof(both), s);
        if (rc) return rc;
        if (expect_kept >= 0 && (long)both[0] != expect_kept)
            return set_err(L, SL_ESTATE, "prune kept %u entries, expected %ld", both[0], expect_kept);
        expect_kept = -1;
        const uint32_t accepted = both[1];
        if ((long)accepted >= k) {
            hipLaunchKernelGGL(cand_limit_kernel, dim3(1), dim3(64), 0, s, W, f2, (uint32_t)k, small + SMALL_LIMIT);
            hipLaunchKernelGGL(cand_select_kernel, dim3(nblk(W)), dim3(TB), 0, s, W, vs, small + SMALL_LIMIT, f0);
            SL_HIP(L, scan_excl<uint32_t>(temp, L->cp.temp_bytes, f0, f3, (size_t)W + 1, s));
            hipLaunchKernelGGL(gather_selected_kernel, dim3(nblk(W)), dim3(TB), 0, s, W, f0, f3, ks, new_p);
            SL_HIP(L, hipGetLastError());
            return SL_OK;
        }
        if (W >= cap) break;
        W *= 2;
    }
    return set_err(L, SL_ESTATE, "position sampler: window exhausted before %ld positions were accepted", k);
}

// survivors (ns of them, in scratch) + k new connections at `generation` -> CSR arrays of L
static int rebuild(sl_layer *L, long ns, long k, uint32_t generation, hipStream_t s, long expect_kept)
{
    const int n_out = (int)L->cfg.n_out;
    const uint32_t n_in = (uint32_t)L->cfg.n_in;
    int rc = sample_positions(L, k, ns, generation, s, expect_kept);
    if (rc) return rc;
    const int *rowptr_s = at<int>(L, L->cp.rowptr_s), *s_col = at<int>(L, L->cp.s_col);
    const float *s_val = at<float>(L, L->cp.s_val), *s_vel = at<float>(L, L->cp.s_vel);
    const uint64_t *new_p = at<uint64_t>(L, L->cp.new_p);
    hipLaunchKernelGGL(merge_rowptr_kernel, dim3(nblk(n_out + 1)), dim3(TB), 0, s, n_out, n_in, rowptr_s, new_p, k,
                       L->rowptr);
    const long n = ns + k;
    if (n > 0) {
        const long n_tiles = (n + MERGE_TILE - 1) / MERGE_TILE;
        int4 *tile = at<int4>(L, L->cp.f0);           // the sampler is done with its flag arrays
        hipLaunchKernelGGL(merge_tile_kernel, dim3(nblk(n_tiles + 1)), dim3(TB), 0, s, n_tiles, n_out, n_in, rowptr_s, L->rowptr,
                           s_col, new_p, n, ns, k, tile);
        const Rng rng = make_rng(L, generation);
        if (L->has_csc)
            hipLaunchKernelGGL(merge_rows_kernel<true>, dim3((unsigned)n_tiles), dim3(TB), 0, s, n, n_in, tile, rowptr_s,
                               L->rowptr, s_col, s_val, s_vel, new_p, rng, L->cfg.init_limit, L->colidx, L->val, L->vel,
                               at<RowValVel>(L, L->cp.packed), at<uint32_t>(L, L->cp.keyA), at<uint32_t>(L, L->cp.payA));
        else
            hipLaunchKernelGGL(merge_rows_kernel<false>, dim3((unsigned)n_tiles), dim3(TB), 0, s, n, n_in, tile, rowptr_s,
                               L->rowptr, s_col, s_val, s_vel, new_p, rng, L->cfg.init_limit, L->colidx, L->val, L->vel,
                               (RowValVel *)nullptr, (uint32_t *)nullptr, (uint32_t *)nullptr);
    }
    SL_HIP(L, hipGetLastError());
    return topo_finalize(L, s, true);
}

// RetainValidUpdates (Algorithm 1): the gradient of master entry t is the old gradient of the same
// (row, column) if the old pattern has it, else zero.  Row bounds read from the caller's rowptr are
// clamped to [0, old_nnz], so a malformed old pattern cannot send the search out of bounds.
__global__ void retain_valid_kernel(long n, int n_rows, const int *rowptr, const int *colidx, const int *rowidx,
                                    const int *csr_pos, const int *old_rowptr, const int *old_col, const float *old_grad,
                                    int old_nnz, float *grad)
{
    const long t = blockIdx.x * (long)TB + threadIdx.x;
    if (t >= n) return;
    const int p = csr_pos ? csr_pos[t] : (int)t;
    const int j = rowidx ? rowidx[t] : row_of(rowptr, n_rows, p);
    const int i = colidx[p];
    const int lo = min(max(old_rowptr[j], 0), old_nnz);
    const int hi = min(max(old_rowptr[j + 1], lo), old_nnz);
    const int q = lower_bound_i32(old_col, lo, hi, i);
    grad[t] = (q < hi && old_col[q] == i) ? old_grad[q] : 0.f;
}

int topo_retain_valid(sl_layer *L, const int *old_rowptr, const int *old_col, const float *old_grad, int64_t old_nnz,
                      hipStream_t s)
{
    if (L->nnz == 0) return SL_OK;
    hipLaunchKernelGGL(retain_valid_kernel, dim3(nblk(L->nnz)), dim3(TB), 0, s, (long)L->nnz, (int)L->cfg.n_out, L->rowptr,
                       L->colidx, L->has_csc ? L->rowidx : nullptr, L->has_csc ? L->csr_pos : nullptr, old_rowptr, old_col,
                       old_grad, (int)old_nnz, L->grad);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int topo_importance(sl_layer *L, float *imp_dev, hipStream_t s)
{
    hipLaunchKernelGGL(importance_kernel, dim3(nblk(L->cfg.n_out)), dim3(TB), 0, s, (int)L->cfg.n_out, L->rowptr, L->val,
                       imp_dev);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int topo_importance_prune(sl_layer *L, float threshold, int64_t *removed, hipStream_t s)
{
    const long n = L->nnz;
    const int n_out = (int)L->cfg.n_out;
    if (removed) *removed = 0;
    if (n == 0) return SL_OK;
    int rc = topo_sync_csr_vel(L, s);
    if (rc) return rc;
    float *imp = at<float>(L, L->cp.f0);
    uint32_t *keep = at<uint32_t>(L, L->cp.keep), *kscan = at<uint32_t>(L, L->cp.kscan);
    int *s_col = at<int>(L, L->cp.s_col), *rowptr_s = at<int>(L, L->cp.rowptr_s);
    float *s_val = at<float>(L, L->cp.s_val), *s_vel = at<float>(L, L->cp.s_vel);
    rc = topo_importance(L, imp, s);
    if (rc) return rc;
    hipLaunchKernelGGL(importance_keep_kernel, dim3(nblk(n + 1)), dim3(TB), 0, s, n, n_out, L->rowptr, imp, threshold, keep);
    SL_HIP(L, scan_excl<uint32_t>(at<char>(L, L->cp.temp), L->cp.temp_bytes, keep, kscan, (size_t)n + 1, s));
    uint32_t kept = 0;
    rc = read_back(L, &kept, kscan + n, sizeof(uint32_t), s);
    if (rc) return rc;
    if ((long)kept == n) return SL_OK;
    hipLaunchKernelGGL(compact_kernel, dim3(nblk(n)), dim3(TB), 0, s, n, keep, kscan, L->colidx, L->val, L->vel, s_col,
                       s_val, s_vel);
    hipLaunchKernelGGL(survivor_rowptr_kernel, dim3(nblk(n_out + 1)), dim3(TB), 0, s, n_out, L->rowptr, kscan, rowptr_s);
    hipLaunchKernelGGL(copy_back_kernel, dim3(nblk(kept)), dim3(TB), 0, s, (long)kept, s_col, s_val, s_vel, L->colidx,
                       L->val, L->vel);
    SL_HIP(L, hipMemcpyAsync(L->rowptr, rowptr_s, sizeof(int) * ((size_t)n_out + 1), hipMemcpyDeviceToDevice, s));
    SL_HIP(L, hipGetLastError());
    L->nnz = kept;
    if (removed) *removed = n - (long)kept;
    return topo_finalize(L, s);
}

size_t average_scratch_bytes(int64_t T)
{
    const size_t t = (size_t)T + 1;
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    // keys A/B, payload A/B, values, head, uidx, ukey, uval, tie, trank, keep, kscan, rocPRIM temporaries
    return 2 * up(8 * t) + 2 * up(4 * t) + up(4 * t) + 2 * up(4 * t) + up(8 * t) + up(4 * t) + 2 * up(8 * t) + 2 * up(4 * t) +
           up(((size_t)32 << 20) + 2 * t) + 4096;
}

int topo_average(sl_layer *D, sl_layer *const *reps, int K, char *scr, size_t scr_bytes, hipStream_t s)
{
    const uint32_t n_in = (uint32_t)D->cfg.n_in;
    const int n_out = (int)D->cfg.n_out;
    long T = 0;
    for (int k = 0; k < K; ++k) T += reps[k]->nnz;
    if (scr_bytes < average_scratch_bytes(T)) return set_err(D, SL_ENOMEM, "average: scratch of %zu bytes needed", average_scratch_bytes(T));
    const long n_keep = D->nnz;
    size_t cur = 0;
    auto take = [&](size_t bytes) { char *p = scr + cur; cur = (cur + bytes + 255) & ~(size_t)255; return p; };
    const size_t t1 = (size_t)T + 1;
    uint64_t *kA = (uint64_t *)take(8 * t1), *kB = (uint64_t *)take(8 * t1);
    uint32_t *vA = (uint32_t *)take(4 * t1), *vB = (uint32_t *)take(4 * t1);
    float *vals = (float *)take(4 * t1);
    uint32_t *head = (uint32_t *)take(4 * t1), *uidx = (uint32_t *)take(4 * t1);
    uint64_t *ukey = (uint64_t *)take(8 * t1);
    float *uval = (float *)take(4 * t1);
    uint64_t *tie = (uint64_t *)take(8 * t1), *trank = (uint64_t *)take(8 * t1);
    uint32_t *keep = (uint32_t *)take(4 * t1), *kscan = (uint32_t *)take(4 * t1);
    const size_t temp_bytes = ((size_t)32 << 20) + 2 * t1;
    char *temp = take(temp_bytes);
    // biases first: they only need the replicas' current values
    BiasPtrs bp;
    for (int k = 0; k < K; ++k) bp.b[k] = reps[k]->bias;
    hipLaunchKernelGGL(avg_bias_kernel, dim3(nblk(n_out)), dim3(TB), 0, s, n_out, bp, K, D->bias, D->bias_vel);
    if (T == 0) { SL_HIP(D, hipGetLastError()); return SL_OK; }
    long off = 0;
    for (int k = 0; k < K; ++k) {
        const sl_layer *R = reps[k];
        if (R->nnz > 0)
            hipLaunchKernelGGL(avg_keys_kernel, dim3(nblk(R->nnz)), dim3(TB), 0, s, (long)R->nnz, n_out, n_in, R->rowptr,
                               R->colidx, R->val, off, kA, vA, vals);
        off += R->nnz;
    }
    uint64_t *ks; uint32_t *vs;
    SL_HIP(D, sort_pairs<uint64_t>(temp, temp_bytes, kA, kB, vA, vB, (size_t)T, bit_length((uint64_t)n_in * n_out - 1), &ks, &vs, s));
    hipLaunchKernelGGL(avg_head_kernel, dim3(nblk(T + 1)), dim3(TB), 0, s, T, ks, head);
    SL_HIP(D, scan_excl<uint32_t>(temp, temp_bytes, head, uidx, (size_t)T + 1, s));
    uint32_t U32 = 0;
    int rc = read_back(D, &U32, uidx + T, sizeof(uint32_t), s);
    if (rc) return rc;
    const long U = U32;
    hipLaunchKernelGGL(avg_sum_kernel, dim3(nblk(T)), dim3(TB), 0, s, T, ks, vs, vals, head, uidx, (float)K, ukey, uval);
    // prune the union back to n_keep connections: remove the U - n_keep smallest magnitudes
    const long k_remove = U > n_keep ? U - n_keep : 0;
    hipLaunchKernelGGL(select_setup_kernel, dim3(2), dim3(256), 0, s, D->sel, (uint32_t)k_remove, 0u);
    if (k_remove > 0)
        for (int shift = 24; shift >= 0; shift -= 8) {
            launch_select_hist(uval, U, 0, shift, D->sel, s);
            hipLaunchKernelGGL(select_pick_kernel, dim3(2), dim3(256), 0, s, D->sel, shift == 0 ? 1 : 0);
        }
    hipLaunchKernelGGL(tie_flag_kernel, dim3(nblk(U + 1)), dim3(TB), 0, s, uval, U, 0, D->sel, tie);
    SL_HIP(D, scan_excl<uint64_t>(temp, temp_bytes, tie, trank, (size_t)U + 1, s));
    hipLaunchKernelGGL(keep_flag_kernel, dim3(nblk(U + 1)), dim3(TB), 0, s, uval, U, 0, D->sel, trank, keep);
    SL_HIP(D, scan_excl<uint32_t>(temp, temp_bytes, keep, kscan, (size_t)U + 1, s));
    hipLaunchKernelGGL(avg_compact_kernel, dim3(nblk(U)), dim3(TB), 0, s, U, keep, kscan, ukey, uval, n_in, D->colidx,
                       D->val, D->vel);
    hipLaunchKernelGGL(avg_rowptr_kernel, dim3(nblk(n_out + 1)), dim3(TB), 0, s, n_out, n_in, ukey, U, kscan, D->rowptr);
    SL_HIP(D, hipGetLastError());
    D->nnz = U - k_remove;
    return topo_finalize(D, s);
}

int topo_init(sl_layer *L, hipStream_t s)
{
    const int n_out = (int)L->cfg.n_out;
    int rc = topo_check_temp(L, s);
    if (rc) return rc;
    hipLaunchKernelGGL(fill_i32_kernel, dim3(nblk(n_out + 1)), dim3(TB), 0, s, (long)n_out + 1,
                       at<int>(L, L->cp.rowptr_s), 0);
    hipLaunchKernelGGL(fill_f32_kernel, dim3(nblk(n_out)), dim3(TB), 0, s, (long)n_out, L->bias, 0.f);
    hipLaunchKernelGGL(fill_f32_kernel, dim3(nblk(n_out)), dim3(TB), 0, s, (long)n_out, L->bias_vel, 0.f);
    hipLaunchKernelGGL(fill_f32_kernel, dim3(nblk(n_out)), dim3(TB), 0, s, (long)n_out, L->grad_bias, 0.f);
    if (L->nnz > 0) hipLaunchKernelGGL(fill_f32_kernel, dim3(nblk(L->nnz)), dim3(TB), 0, s, (long)L->nnz, L->grad, 0.f);
    SL_HIP(L, hipGetLastError());
    return rebuild(L, 0, L->nnz, 0u, s, -1);
}

int topo_evolve(sl_layer *L, double zeta, uint32_t generation, hipStream_t s)
{
    const long n = L->nnz;
    const int n_out = (int)L->cfg.n_out;
    const int mode = L->cfg.prune_mode;
    int rc = topo_sync_csr_vel(L, s);
    if (rc) return rc;
    // number of removals per class, floor(zeta*count + 0.5) in double
    long cnt[2] = {n, 0};
    if (mode == 1) {
        uint32_t *small = at<uint32_t>(L, L->cp.small) + SMALL_CLASS;
        hipLaunchKernelGGL(zero_u32_kernel, dim3(1), dim3(TB), 0, s, 1L, small);
        if (n > 0) hipLaunchKernelGGL(class_count_kernel, dim3(std::min(256u, nblk(n))), dim3(TB), 0, s, L->val, n, small);
        uint32_t neg = 0;
        rc = read_back(L, &neg, small, sizeof(uint32_t), s);
        if (rc) return rc;
        cnt[1] = neg; cnt[0] = n - neg;
    }
    long kc[2];
    for (int c = 0; c < 2; ++c) {
        kc[c] = (long)floor(zeta * (double)cnt[c] + 0.5);
        if (kc[c] < 0) kc[c] = 0;
        if (kc[c] > cnt[c]) kc[c] = cnt[c];
    }
    const long k = kc[0] + kc[1];
    if (k == 0) return SL_OK;
    hipLaunchKernelGGL(select_setup_kernel, dim3(2), dim3(256), 0, s, L->sel, (uint32_t)kc[0], (uint32_t)kc[1]);
    for (int shift = 24; shift >= 0; shift -= 8) {
        launch_select_hist(L->val, n, mode, shift, L->sel, s);
        hipLaunchKernelGGL(select_pick_kernel, dim3(2), dim3(256), 0, s, L->sel, shift == 0 ? 1 : 0);
    }
    const unsigned nb = (unsigned)((n + 1 + PRUNE_TILE - 1) / PRUNE_TILE);   // workgroups of PRUNE_TILE entries, the sentinel entry n included
    uint64_t *blk_tie = at<uint64_t>(L, L->cp.tie64), *blk_tie_off = at<uint64_t>(L, L->cp.trank);
    uint32_t *blk_keep = at<uint32_t>(L, L->cp.keep), *blk_keep_off = at<uint32_t>(L, L->cp.f0);   // the sampler's flags: not yet in use
    uint32_t *kscan = at<uint32_t>(L, L->cp.kscan);
    char *temp = at<char>(L, L->cp.temp);
    hipLaunchKernelGGL(tie_count_kernel, dim3(nb), dim3(TB), 0, s, L->val, n, mode, L->sel, blk_tie);
    SL_HIP(L, scan_excl<uint64_t>(temp, L->cp.temp_bytes, blk_tie, blk_tie_off, (size_t)nb, s));
    hipLaunchKernelGGL(keep_count_kernel, dim3(nb), dim3(TB), 0, s, L->val, n, mode, L->sel, blk_tie_off, blk_keep);
    SL_HIP(L, scan_excl<uint32_t>(temp, L->cp.temp_bytes, blk_keep, blk_keep_off, (size_t)nb, s));
    hipLaunchKernelGGL(compact_block_kernel, dim3(nb), dim3(TB), 0, s, L->val, n, mode, L->sel, blk_tie_off, blk_keep_off,
                       L->colidx, L->vel, kscan, at<int>(L, L->cp.s_col), at<float>(L, L->cp.s_val), at<float>(L, L->cp.s_vel));
    hipLaunchKernelGGL(survivor_rowptr_kernel, dim3(nblk(n_out + 1)), dim3(TB), 0, s, n_out, L->rowptr, kscan,
                       at<int>(L, L->cp.rowptr_s));
    // the survivor count is checked at the sampler's read-back
    hipLaunchKernelGGL(copy_u32_kernel, dim3(1), dim3(64), 0, s, kscan + n, at<uint32_t>(L, L->cp.small) + SMALL_KEPT);
    return rebuild(L, n - k, k, generation, s, n - k);
}

}  // namespace sl
