// Per-minibatch kernels of a truly sparse layer (gfx950): forward SpMM fused with All-ReLU,
// activation derivative, backward (transposed SpMM fused with the pattern-restricted SDDMM),
// momentum-SGD update and the softmax cross-entropy loss.
//
// Common shape of the sparse kernels.  Dense operands are feature-major [n][ld], so one stored
// connection touches ONE contiguous run of 4*B bytes of the dense operand.  A group of G lanes
// (G = 8/16/32/64 for B <= 32/64/128/256) owns one virtual row: each lane holds four batch
// columns as a float4, so a gather of one operand row is a single fully coalesced
// global_load_dwordx4 across the group, and 64/G rows are in flight per wavefront.  Entries are
// processed U at a time (U = 2/4/8 by mean row length) so that U independent row gathers are
// outstanding per group; the work is HBM-bound (0.5 flop/byte), so there is no MFMA here.
#include <stdarg.h>
#include <stdio.h>

#include <mutex>
#include <type_traits>
#include <utility>

#include "sl_internal.h"

namespace sl {

static constexpr int BLOCK = 256;
static constexpr int FIX_BLOCK = 1024;
static constexpr int MAX_MULTI = SL_MAX_MULTI;

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }
__device__ __forceinline__ float4 zero4() { return make_float4(0.f, 0.f, 0.f, 0.f); }

// zero the components of v whose column c+k is >= B (ragged batch sizes only)
__device__ __forceinline__ float4 clip4(float4 v, int c, int B)
{
    v.y = (c + 1 < B) ? v.y : 0.f;
    v.z = (c + 2 < B) ? v.z : 0.f;
    v.w = (c + 3 < B) ? v.w : 0.f;
    return v;
}

// Cross-lane moves whose lane pattern sits in the instruction, so that none needs an address register.
// DPP forms (dpp_ctrl: quad_perm 0x00-0xFF, row_shl:n 0x100+n, row_shr:n 0x110+n, row_ror:n 0x120+n,
// row_newbcast:n 0x150+n; a row is 16 lanes) run in the vector ALU; ds_swizzle (bit mode: source lane =
// ((lane & AND) | OR) ^ XOR within each half of 32 lanes) takes a trip through the LDS crossbar.
template <int CTRL, int BANKS>
__device__ __forceinline__ int dpp_mov(int old, int v)
{
    return __builtin_amdgcn_update_dpp(old, v, CTRL, 0xF, BANKS, false);
}
// value of lane (lane ^ XOR); the partner is inside the caller's group for every use below
template <int G, int XOR>
__device__ __forceinline__ float xor_partner(float v)
{
    static_assert(XOR >= 1 && XOR < G && (XOR & (XOR - 1)) == 0, "partner outside the group");
    const int i = __float_as_int(v);
    if constexpr (XOR == 1) return __int_as_float(dpp_mov<0xB1, 0xF>(i, i));        // quad_perm [1,0,3,2]
    else if constexpr (XOR == 2) return __int_as_float(dpp_mov<0x4E, 0xF>(i, i));   // quad_perm [2,3,0,1]
    else if constexpr (XOR == 4) {
        const int t = dpp_mov<0x104, 0x5>(i, i);             // lanes 0-3, 8-11 of a row read lane + 4
        return __int_as_float(dpp_mov<0x114, 0xA>(t, i));    // lanes 4-7, 12-15 read lane - 4
    } else if constexpr (XOR == 8) return __int_as_float(dpp_mov<0x128, 0xF>(i, i));   // row_ror:8
    else if constexpr (XOR == 16) return __int_as_float(__builtin_amdgcn_ds_swizzle(i, (16 << 10) | 0x1F));
    else return __shfl_xor(v, XOR, G);
}
// Value of entry K of a chunk, which every lane with (lane & (U - 1)) == K holds (U <= 8 <= K's row of 16
// lanes): lane K of the caller's row for groups of 16 lanes or more, lane K of the group of 8 otherwise.
template <int G, int K>
__device__ __forceinline__ int chunk_entry(int v)
{
    static_assert(K >= 0 && K < 8, "chunks have at most eight entries");
    if constexpr (G >= 16) return dpp_mov<0x150 + K, 0xF>(v, v);
    else return __builtin_amdgcn_ds_swizzle(v, (K << 5) | 0x18);
}
// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <typename F, int... I>
__device__ __forceinline__ void static_for_seq(F &&f, std::integer_sequence<int, I...>)
{
    (f(std::integral_constant<int, I>()), ...);
}
template <int N, typename F>
__device__ __forceinline__ void static_for(F &&f)
{
    static_for_seq(f, std::make_integer_sequence<int, N>());
}

__device__ __forceinline__ void store_row4(float *row, int c, int B, float4 v)
{
    if (c + 3 < B) {
        st4(row + c, v);
    } else {
        row[c] = v.x;
        if (c + 1 < B) row[c + 1] = v.y;
        if (c + 2 < B) row[c + 2] = v.z;
    }
}

// Momentum SGD, eq. (1) in velocity form, for one connection.  The products are rounded separately (no
// fused multiply-add) so that the result is the plain fp32 evaluation of
// vel = mu*vel - eta*(g + lambda*w);  w = w + vel.
__device__ __forceinline__ void update_one(float &w, float &vel, float g, float lr, float mu, float wd)
{
#pragma clang fp contract(off)   // separate roundings: this must equal the plain fp32 evaluation
    const float gg = g + wd * w;
    const float vn = mu * vel - lr * gg;
    vel = vn;
    w = w + vn;
}

// ------------------------------------------------------------------------------------------------
// What happens to a finished row of accumulators.
//   EPI_FWD   : + bias, All-ReLU (eq. 3), sign mask of z saved for backward      -> a
//   EPI_PLAIN : stored as is                                                     -> grad_x
//   EPI_DZ    : the row is dLoss/da of a neuron of the layer that owns `mask_r`; it is multiplied
//               by that layer's f' (from its saved sign mask) and stored as its dz, and the row sum
//               is its bias gradient.  Used by the activation-derivative kernel, and by a consumer
//               layer's backward to hand the input gradient to its producer without a separate
//               elementwise pass.
// ------------------------------------------------------------------------------------------------
enum { EPI_FWD = 0, EPI_PLAIN = 1, EPI_DZ = 2 };
struct Epi {
    int mode;
    float *out;
    long ldo;
    const float *bias;
    uint8_t *mask_w;
    const uint8_t *mask_r;
    long ldm;
    float *gb;
    int act_kind;
    float slope;   // -alpha (even layer) or +alpha (odd layer)
    int B;
    // dropout of the layer that owns the mask: element (row, column b) is kept iff word b&3 of
    // Philox(row, b>>2, 4, step) >= drop_thr; kept values are multiplied by drop_scale.  0 = off.
    uint32_t drop_thr, drop_step, k0, k1;
    float drop_scale;
};

// Every lane of the group must call this (EPI_DZ reduces across the group).
template <int G>
__device__ __forceinline__ void finish(const Epi &e, long row, int c, bool active, float4 acc, int lane, int tile)
{
    if (e.mode == EPI_FWD) {
        if (!active) return;
        const float b = e.bias ? e.bias[row] : 0.f;
        float4 z = make_float4(acc.x + b, acc.y + b, acc.z + b, acc.w + b);
        float4 r = z;
        if (e.act_kind != 0) {
            unsigned nib = (z.x > 0.f ? 1u : 0u) | (z.y > 0.f ? 2u : 0u) | (z.z > 0.f ? 4u : 0u) | (z.w > 0.f ? 8u : 0u);
            r.x = z.x > 0.f ? z.x : e.slope * z.x;
            r.y = z.y > 0.f ? z.y : e.slope * z.y;
            r.z = z.z > 0.f ? z.z : e.slope * z.z;
            r.w = z.w > 0.f ? z.w : e.slope * z.w;
            if (e.drop_thr != 0u && e.mask_w) {   // training forward only; the keep bits go to the high nibble
                uint32_t o[4];
                philox((uint32_t)row, (uint32_t)(c >> 2), 4u, e.drop_step, e.k0, e.k1, o);
                nib |= (o[0] >= e.drop_thr ? 16u : 0u) | (o[1] >= e.drop_thr ? 32u : 0u) |
                       (o[2] >= e.drop_thr ? 64u : 0u) | (o[3] >= e.drop_thr ? 128u : 0u);
                r.x = (nib & 16u) ? r.x * e.drop_scale : 0.f;
                r.y = (nib & 32u) ? r.y * e.drop_scale : 0.f;
                r.z = (nib & 64u) ? r.z * e.drop_scale : 0.f;
                r.w = (nib & 128u) ? r.w * e.drop_scale : 0.f;
            }
            if (e.mask_w) e.mask_w[row * e.ldm + (c >> 2)] = (uint8_t)nib;
        }
        store_row4(e.out + row * e.ldo, c, e.B, r);
    } else if (e.mode == EPI_PLAIN) {
        if (active) store_row4(e.out + row * e.ldo, c, e.B, acc);
    } else {
        float4 d = zero4();
        if (active) {
            d = acc;
            if (e.act_kind != 0) {
                const unsigned nib = e.mask_r[row * e.ldm + (c >> 2)];
                if (e.drop_thr != 0u) {
                    d.x = (nib & 16u) ? d.x * e.drop_scale : 0.f;
                    d.y = (nib & 32u) ? d.y * e.drop_scale : 0.f;
                    d.z = (nib & 64u) ? d.z * e.drop_scale : 0.f;
                    d.w = (nib & 128u) ? d.w * e.drop_scale : 0.f;
                }
                d.x = d.x * ((nib & 1u) ? 1.f : e.slope);
                d.y = d.y * ((nib & 2u) ? 1.f : e.slope);
                d.z = d.z * ((nib & 4u) ? 1.f : e.slope);
                d.w = d.w * ((nib & 8u) ? 1.f : e.slope);
            }
            if (c + 3 >= e.B) d = clip4(d, c, e.B);
            st4(e.out + row * e.ldo + c, d);   // dz is library-owned: ld >= roundup4(B), zeros past B
        }
        float s = (d.x + d.y) + (d.z + d.w);
#pragma unroll
        for (int m = G / 2; m >= 1; m >>= 1) s += __shfl_xor(s, m, G);
        if (lane == 0) e.gb[row] = tile == 0 ? s : e.gb[row] + s;
    }
}

// ------------------------------------------------------------------------------------------------
// Forward: z = Wt x + b, a = f_l(z) (eq. 3).  One group per virtual row, batch tiles in grid.y.
// ------------------------------------------------------------------------------------------------
struct FwdArgs {
    const int *vptr;
    const int *v2row;
    int nv;
    const int *idx;
    const float *w;
    const float *x;
    int ldx;         // fits 31 bits (checked by the entry points)
    int twin_rows;   // > 0: fully dense matrix of this many rows, each cut into nv / twin_rows equal runs (see fwd_kernel)
    float *part;     // partial sums [nv][ldp] when the matrix is split, else null
    long ldp;
    Epi epi;
};

template <int G, int U>
__global__ __launch_bounds__(BLOCK) void fwd_kernel(FwdArgs a)
{
    const int lane = threadIdx.x % G;
    long v = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    const int c = (blockIdx.y * G + lane) * 4;
    if (v >= a.nv || c >= a.epi.B) return;
    // Fully dense narrow matrices (the output layers): neighbouring groups take the SAME run of columns of
    // neighbouring rows, so the groups of a wavefront and of a block gather the same operand rows at the same
    // time and all but the first are served by the CU's cache instead of by memory.
    if (a.twin_rows > 0) v = (v % a.twin_rows) * (a.nv / a.twin_rows) + v / a.twin_rows;
    const int p0 = a.vptr[v], p1 = a.vptr[v + 1];
    const float *xb = a.x + c;
    float4 acc = zero4();
    for (int p = p0; p < p1; p += U) {
        int cc[U];
        float ww[U];
        float4 xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = min(p + u, p1 - 1);
            cc[u] = a.idx[q];
            ww[u] = (p + u < p1) ? a.w[q] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) xv[u] = ld4(xb + (long)cc[u] * a.ldx);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            acc.x = fmaf(ww[u], xv[u].x, acc.x);
            acc.y = fmaf(ww[u], xv[u].y, acc.y);
            acc.z = fmaf(ww[u], xv[u].z, acc.z);
            acc.w = fmaf(ww[u], xv[u].w, acc.w);
        }
    }
    if (a.part) {
        st4(a.part + v * a.ldp + c, acc);
        return;
    }
    finish<G>(a.epi, a.v2row ? a.v2row[v] : v, c, true, acc, lane, 0);   // EPI_FWD: no cross-lane step
}

// ------------------------------------------------------------------------------------------------
// Split matrices: add the partial sums of a row's virtual rows in a fixed order, then finish the row.
// fix_kernel: one group per row (matrices with many rows, few of them split).
// fix_block_kernel: one 1024-thread block per row (narrow matrices: 2 or 10 rows of thousands of
// partial sums); groups stride over the row's virtual rows, then group 0 adds the group sums in order.
// ------------------------------------------------------------------------------------------------
struct FixArgs {
    const int *rvptr;
    int n_rows;
    const float *part;
    long ldp;
    Epi epi;
};

__device__ __forceinline__ float4 sum_partials(const float *part, long ldp, int c, int v0, int v1, int stride)
{
    float4 acc = zero4();
    int v = v0;
    for (; v + 3 * stride < v1; v += 4 * stride) {
        const float4 t0 = ld4(part + (long)v * ldp + c), t1 = ld4(part + (long)(v + stride) * ldp + c);
        const float4 t2 = ld4(part + (long)(v + 2 * stride) * ldp + c), t3 = ld4(part + (long)(v + 3 * stride) * ldp + c);
        acc.x = (((acc.x + t0.x) + t1.x) + t2.x) + t3.x;
        acc.y = (((acc.y + t0.y) + t1.y) + t2.y) + t3.y;
        acc.z = (((acc.z + t0.z) + t1.z) + t2.z) + t3.z;
        acc.w = (((acc.w + t0.w) + t1.w) + t2.w) + t3.w;
    }
    for (; v < v1; v += stride) {
        const float4 t = ld4(part + (long)v * ldp + c);
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    return acc;
}

template <int G>
__global__ __launch_bounds__(BLOCK) void fix_kernel(FixArgs a)
{
    const int lane = threadIdx.x % G;
    const long row = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (row >= a.n_rows) return;   // whole groups leave together
    const int v0 = a.rvptr[row], v1 = a.rvptr[row + 1];
    for (int tile = 0; tile * 4 * G < a.epi.B; ++tile) {
        const int c = (tile * G + lane) * 4;
        const bool active = c < a.epi.B;
        float4 acc = zero4();
        if (active) acc = sum_partials(a.part, a.ldp, c, v0, v1, 1);
        finish<G>(a.epi, row, c, active, acc, lane, tile);
    }
}

template <int G>
__global__ __launch_bounds__(FIX_BLOCK) void fix_block_kernel(FixArgs a)
{
    constexpr int NG = FIX_BLOCK / G;
    __shared__ float4 sh[FIX_BLOCK];
    const int lane = threadIdx.x % G, grp = threadIdx.x / G;
    const long row = blockIdx.x;
    const int v0 = a.rvptr[row], v1 = a.rvptr[row + 1];
    for (int tile = 0; tile * 4 * G < a.epi.B; ++tile) {
        const int c = (tile * G + lane) * 4;
        const bool active = c < a.epi.B;
        float4 acc = zero4();
        if (active) acc = sum_partials(a.part, a.ldp, c, v0 + grp, v1, NG);
        sh[threadIdx.x] = acc;
        __syncthreads();
        if (grp == 0) {
            float4 tot = sh[lane];
            for (int g = 1; g < NG; ++g) {
                const float4 t = sh[g * G + lane];
                tot.x += t.x; tot.y += t.y; tot.z += t.z; tot.w += t.w;
            }
            finish<G>(a.epi, row, c, active, tot, lane, tile);
        }
        __syncthreads();
    }
}

// ------------------------------------------------------------------------------------------------
// dz = grad_a * f_l'(z), grad_bias = row sums of dz (layers whose consumer did not hand dz over).
// One group per row, tiles of 4*G columns.
// ------------------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(BLOCK) void actgrad_kernel(const float *ga, long ldg, int n_out, Epi e)
{
    const int lane = threadIdx.x % G;
    const long row = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (row >= n_out) return;   // whole groups leave together
    for (int tile = 0; tile * 4 * G < e.B; ++tile) {
        const int c = (tile * G + lane) * 4;
        const bool active = c < e.B;
        float4 g = zero4();
        if (active) {
            if (c + 3 < e.B) {
                g = ld4(ga + row * ldg + c);
            } else {
                g.x = ga[row * ldg + c];
                g.y = (c + 1 < e.B) ? ga[row * ldg + c + 1] : 0.f;
                g.z = (c + 2 < e.B) ? ga[row * ldg + c + 2] : 0.f;
            }
        }
        finish<G>(e, row, c, active, g, lane, tile);
    }
}

// ------------------------------------------------------------------------------------------------
// Backward.  One kernel covers both uses:
//   SPMM = true  (layers that need grad_x; runs over the CSC view, one group per input neuron i):
//       holds x[i], gathers dz[j] for every stored (j,i) ONCE and uses it twice:
//       grad_x[i] += Wt[j,i] * dz[j]          (transposed SpMM)
//       grad[q]    = <dz[j], x[i]>            (SDDMM restricted to the pattern)
//   SPMM = false (first layer; runs over CSR, one group per output neuron j):
//       holds dz[j], gathers x[i], grad[p] = <dz[j], x[i]>.
// The U dot products of a chunk are reduced together: log2(U) exchange steps fold U values per lane
// into one (lane l keeps the sum for entry l % U), the remaining log2(G/U) steps are plain
// butterflies, so a chunk of 8 costs 7 + log2(G/8) cross-lane moves instead of 8 * log2(G).
// ------------------------------------------------------------------------------------------------
struct BwdArgs {
    const int *vptr;
    const int *v2row;
    int nv;
    const int *idx;
    const float *w;
    const float *held;
    int ldh;         // leading dimensions fit 31 bits (checked by the entry points): one 32x32->64 multiply per row address
    const float *gath;
    int ldga;
    float *g;        // per stored entry, in the order of this orientation
    float *part;     // SPMM partial sums [nv][ldp] when the matrix is split, else null
    long ldp;
    int B;
    int ragged;      // B % 4 != 0
    int tile0, tile1; // the batch tiles this launch covers
    int slice_tiles;  // host only: > 0 = one launch per this many tiles (operands sliced for L2 residency)
    Epi epi;         // SPMM, not split: what to do with the finished grad_x row
    // Update fused behind the SDDMM (eq. 1 applied where the gradient entry is produced): on the last batch
    // tile the lane that holds a finished gradient entry also holds (or fetches) that connection's weight
    // and velocity, so it writes the new velocity and weight instead of the gradient.  upd_mode 0: off (the
    // gradient is stored), 1: update, gradient not stored, 2: update and store the gradient.
    int upd_mode;
    int n_tiles;     // batch tiles of the whole call (the update happens on the last one)
    float *upd_w, *upd_vel;      // master weights / velocities in the order of this orientation
    const int *upd_pos;          // CSC slot -> CSR slot of the weight copy read by forward (null: none)
    float *upd_w_csr;
    float lr, mu, wd;
};

// What the lane that finished gradient entry q does with it.  w: the connection's weight before the update where the
// caller holds it (the SPMM form: a writer lane's own entry is entry `lane` of its chunk).  The update's other
// operands are fetched here, after the chunk's row gathers have been consumed, so that they occupy no register
// while those gathers are in flight (one register more there costs the fused backward a wave of occupancy).
template <bool UPD, bool HAVE_W>
__device__ __forceinline__ void store_entry(const BwdArgs &a, unsigned q, float gval, bool last_tile, float w, float v, unsigned pos)
{
    if (!UPD || !last_tile) { a.g[q] = gval; return; }
    if (!HAVE_W) w = a.upd_w[q];
    update_one(w, v, gval, a.lr, a.mu, a.wd);
    a.upd_vel[q] = v;
    a.upd_w[q] = w;
    if (a.upd_pos) a.upd_w_csr[pos] = w;
    if (a.upd_mode == 2) a.g[q] = gval;
}

template <int G, int U>
__device__ __forceinline__ float reduce_chunk(float (&s)[U], int lane)
{
    constexpr int LOGU = U == 8 ? 3 : U == 4 ? 2 : 1;
    static_for<LOGU>([&](auto mc) {
        constexpr int m = decltype(mc)::value;
        const bool up = (lane >> m) & 1;
#pragma unroll
        for (int t = 0; t < (U >> (m + 1)); ++t) {
            const float lo = s[2 * t], hi = s[2 * t + 1];
            const float send = up ? lo : hi;
            const float keep = up ? hi : lo;
            s[t] = keep + xor_partner<G, (1 << m)>(send);
        }
    });
    float r = s[0];
    if constexpr (U < G) r += xor_partner<G, U>(r);
    if constexpr (2 * U < G) r += xor_partner<G, 2 * U>(r);
    if constexpr (4 * U < G) r += xor_partner<G, 4 * U>(r);
    if constexpr (8 * U < G) r += xor_partner<G, 8 * U>(r);
    if constexpr (16 * U < G) r += xor_partner<G, 16 * U>(r);
    return r;
}

// Index handling: lane u of a group fetches entry u of a chunk (column index and weight, one register
// each) and the group reads them with cross-lane moves, so the NEXT chunk's indices can be fetched
// while the current chunk's row gathers are in flight at a cost of two registers.  The gathered
// operand of the SPMM form is the library's own dz, whose columns past B are zero; the caller's x
// (gathered by the SDDMM form, held by the SPMM form) may hold anything there and is clipped.
template <int G, int U, bool SPMM, bool UPD>
__global__ __launch_bounds__(BLOCK) void bwd_kernel(BwdArgs a)
{
    const int lane = threadIdx.x % G;
    const long v = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (v >= a.nv) return;   // whole groups leave together
    const int p0 = a.vptr[v], p1 = a.vptr[v + 1];
    const long row = a.v2row ? a.v2row[v] : v;
    const int sub = lane & (U - 1);
    for (int tile = a.tile0; tile < a.tile1; ++tile) {   // the batch tiles of this launch (all of them, or one slice)
        const int c = (tile * G + lane) * 4;
        const bool active = c < a.B;
        const bool upd = UPD && tile + 1 == a.n_tiles;   // last batch tile: the gradient entries are final
        const int cg = active ? c : 0;   // idle lanes gather columns 0..3 and multiply them by a zero h
        float4 h = zero4();
        if (active) {
            h = ld4(a.held + row * a.ldh + c);
            if (a.ragged) h = clip4(h, c, a.B);
        }
        float4 acc = zero4();
        int my_c = 0;
        float my_w = 0.f;
        if (p0 < p1) {
            const int q = min(p0 + sub, p1 - 1);
            my_c = a.idx[q];
            if (SPMM) my_w = a.w[q];
        }
        for (int p = p0; p < p1; p += U) {
            float4 xv[U];
            float s[U];
            // the chunk after this one (clamped to the row's last entry: always a valid position)
            const int qn = min(p + U + sub, p1 - 1);
            const int nx_c = a.idx[qn];
            float nx_w = 0.f;
            if (SPMM) nx_w = a.w[qn];
            // later batch tiles add to what the earlier ones stored; fetch it with the indices, not after
            // the reduction, so that its latency hides behind the row gathers
            const bool writer = lane < U && p + lane < p1;
            float g_prev = 0.f, vel_prev = 0.f;
            unsigned pos = 0;
            if (tile > 0 && writer) g_prev = a.g[p + lane];
            if (UPD && upd && writer) {   // the update's own operands travel with the indices
                vel_prev = a.upd_vel[(unsigned)(p + lane)];
                if (a.upd_pos) pos = (unsigned)a.upd_pos[(unsigned)(p + lane)];
            }
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                const int cc = chunk_entry<G, u>(my_c);
                xv[u] = ld4(a.gath + (long)cc * a.ldga + cg);
                if (!SPMM && a.ragged) xv[u] = clip4(xv[u], c, a.B);
            });
            if (SPMM && p + sub >= p1) my_w = 0.f;   // entries past the end of the row repeat its last one
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                if (SPMM) {
                    const float w = __int_as_float(chunk_entry<G, u>(__float_as_int(my_w)));
                    acc.x = fmaf(w, xv[u].x, acc.x);
                    acc.y = fmaf(w, xv[u].y, acc.y);
                    acc.z = fmaf(w, xv[u].z, acc.z);
                    acc.w = fmaf(w, xv[u].w, acc.w);
                }
                s[u] = fmaf(h.x, xv[u].x, fmaf(h.y, xv[u].y, fmaf(h.z, xv[u].z, h.w * xv[u].w)));
            });
            const float r = reduce_chunk<G, U>(s, lane);
            if (writer) store_entry<UPD, SPMM>(a, (unsigned)(p + lane), g_prev + r, upd, my_w, vel_prev, pos);
            my_c = nx_c;
            my_w = nx_w;
        }
        if (SPMM) {
            if (a.part) {
                if (active) st4(a.part + v * a.ldp + c, acc);
            } else {
                finish<G>(a.epi, row, c, active, acc, lane, tile);
            }
        }
    }
}

// The same walk for batches above 256 columns: a group of 64 lanes carries T = 2 batch tiles (of 256
// columns) at once and covers the tiles [tile0, tile1) of its launch.  A lane holds two float4 per gathered
// row, the two tiles' products are added before the cross-lane reduction, and the per-entry gradient is
// written once per pair of tiles instead of once per tile.  (Kept apart from bwd_kernel: folding the two
// into one template cost the single-tile instances twelve registers and one wave of occupancy.)
template <int U, bool SPMM, bool UPD>
__global__ __launch_bounds__(BLOCK) void bwd_pair_kernel(BwdArgs a)
{
    constexpr int G = 64, T = 2;
    const int lane = threadIdx.x % G;
    const long v = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (v >= a.nv) return;   // whole groups leave together
    const int p0 = a.vptr[v], p1 = a.vptr[v + 1];
    const long row = a.v2row ? a.v2row[v] : v;
    const int sub = lane & (U - 1);
    for (int tile = a.tile0; tile < a.tile1; tile += T) {
        int c[T], cg[T];
        bool active[T];
        float4 h[T], acc[T];
        const bool upd = UPD && tile + T >= a.n_tiles;   // the pair that holds the last batch tile
#pragma unroll
        for (int t = 0; t < T; ++t) {
            c[t] = ((tile + t) * G + lane) * 4;
            active[t] = c[t] < a.B;
            cg[t] = active[t] ? c[t] : 0;   // idle lanes gather columns 0..3 and multiply them by a zero h
            h[t] = zero4();
            if (active[t]) {
                h[t] = ld4(a.held + row * a.ldh + c[t]);
                if (a.ragged) h[t] = clip4(h[t], c[t], a.B);
            }
            acc[t] = zero4();
        }
        int my_c = 0;
        float my_w = 0.f;
        if (p0 < p1) {
            const int q = min(p0 + sub, p1 - 1);
            my_c = a.idx[q];
            if (SPMM) my_w = a.w[q];
        }
        for (int p = p0; p < p1; p += U) {
            float4 xv[U][T];
            float s[U];
            const int qn = min(p + U + sub, p1 - 1);   // the chunk after this one, clamped to a valid position
            const int nx_c = a.idx[qn];
            float nx_w = 0.f;
            if (SPMM) nx_w = a.w[qn];
            // later tile pairs add to what the earlier ones stored; fetch it with the indices, not after the
            // reduction, so that its latency hides behind the row gathers
            const bool writer = lane < U && p + lane < p1;
            float g_prev = 0.f, vel_prev = 0.f;
            unsigned pos = 0;
            if (tile > 0 && writer) g_prev = a.g[p + lane];
            if (UPD && upd && writer) {
                vel_prev = a.upd_vel[(unsigned)(p + lane)];
                if (a.upd_pos) pos = (unsigned)a.upd_pos[(unsigned)(p + lane)];
            }
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                const float *src = a.gath + (long)chunk_entry<G, u>(my_c) * a.ldga;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    xv[u][t] = ld4(src + cg[t]);
                    if (!SPMM && a.ragged) xv[u][t] = clip4(xv[u][t], c[t], a.B);
                }
            });
            if (SPMM && p + sub >= p1) my_w = 0.f;   // entries past the end of the row repeat its last one
            static_for<U>([&](auto uc) {
                constexpr int u = decltype(uc)::value;
                float w = 0.f;
                if (SPMM) w = __int_as_float(chunk_entry<G, u>(__float_as_int(my_w)));
                float d = 0.f;
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    const float4 x4 = xv[u][t];
                    if (SPMM) {
                        acc[t].x = fmaf(w, x4.x, acc[t].x);
                        acc[t].y = fmaf(w, x4.y, acc[t].y);
                        acc[t].z = fmaf(w, x4.z, acc[t].z);
                        acc[t].w = fmaf(w, x4.w, acc[t].w);
                    }
                    const float dt = fmaf(h[t].x, x4.x, fmaf(h[t].y, x4.y, fmaf(h[t].z, x4.z, h[t].w * x4.w)));
                    d = t == 0 ? dt : d + dt;
                }
                s[u] = d;
            });
            const float r = reduce_chunk<G, U>(s, lane);
            if (writer) store_entry<UPD, SPMM>(a, (unsigned)(p + lane), g_prev + r, upd, my_w, vel_prev, pos);
            my_c = nx_c;
            my_w = nx_w;
        }
        if (SPMM) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                if (tile + t < a.tile1) {   // uniform over the group
                    if (a.part) {
                        if (active[t]) st4(a.part + v * a.ldp + c[t], acc[t]);
                    } else {
                        finish<G>(a.epi, row, c[t], active[t], acc[t], lane, tile + t);
                    }
                }
            }
        }
    }
}


// ------------------------------------------------------------------------------------------------
// Span kernel for the forward pass of matrices whose rows are very short (mean <= 3 entries: the
// epsilon = 1 layers).  The backward kernels keep one row per group: their span variants were measured
// slower, twice over (four held rows, four accumulators and the per-entry row selection cost 120 registers
// and half the occupancy: 0.50 instead of 0.28 ms on the 10^6 -> 2 layer).  A group owns R = 2 CONSECUTIVE rows
// (measured against 3, 4 and 8: 4-5 % faster at every batch size) and walks their entries as one stream in chunks
// of 8, so that the gathers of both rows are in flight together.  Which of the rows an entry belongs to follows
// from the R + 1 row pointers held in registers; each row's accumulator takes the entry with a weight
// that is zero for the other rows.  Same arithmetic per row, in the same order, as the row kernels.
// ------------------------------------------------------------------------------------------------
static constexpr int SPAN_R = 2;
static constexpr int SPAN_U = 8;

template <int G>
__global__ __launch_bounds__(BLOCK) void fwd_span_kernel(FwdArgs a)
{
    constexpr int R = SPAN_R, U = SPAN_U;
    const int lane = threadIdx.x % G;
    const long r0 = ((long)blockIdx.x * (BLOCK / G) + threadIdx.x / G) * R;
    const int c = (blockIdx.y * G + lane) * 4;
    if (r0 >= a.nv || c >= a.epi.B) return;
    int pp[R + 1];
#pragma unroll
    for (int r = 0; r <= R; ++r) pp[r] = a.vptr[min(r0 + r, (long)a.nv)];
    const float *xb = a.x + c;
    float4 acc[R];
#pragma unroll
    for (int r = 0; r < R; ++r) acc[r] = zero4();
    const int p1 = pp[R];
    for (int p = pp[0]; p < p1; p += U) {
        int cc[U];
        float ww[U];
        float4 xv[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = min(p + u, p1 - 1);
            cc[u] = a.idx[q];
            ww[u] = (p + u < p1) ? a.w[q] : 0.f;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) xv[u] = ld4(xb + (long)cc[u] * a.ldx);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int q = p + u;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const bool mine = q >= pp[r] && q < pp[r + 1];   // selected, not multiplied by zero: other rows
                acc[r].x = mine ? fmaf(ww[u], xv[u].x, acc[r].x) : acc[r].x;   // must not see this entry at all
                acc[r].y = mine ? fmaf(ww[u], xv[u].y, acc[r].y) : acc[r].y;
                acc[r].z = mine ? fmaf(ww[u], xv[u].z, acc[r].z) : acc[r].z;
                acc[r].w = mine ? fmaf(ww[u], xv[u].w, acc[r].w) : acc[r].w;
            }
        }
    }
#pragma unroll
    for (int r = 0; r < R; ++r)
        if (r0 + r < a.nv) finish<G>(a.epi, r0 + r, c, true, acc[r], lane, 0);
}

// ------------------------------------------------------------------------------------------------
// Momentum SGD, eq. (1) in velocity form, over the stored connections and the biases.  The
// products are rounded separately (no fused multiply-add) so that the result is the plain fp32
// evaluation of  vel = mu*vel - eta*(g + lambda*w);  w = w + vel.
// With a CSC view the master copy is in CSC order and the CSR copy read by forward is refreshed
// through csr_pos.
// ------------------------------------------------------------------------------------------------
struct UpdateOne {
    long n;          // stored connections
    long first;      // first global thread index of this layer (update_many_kernel)
    float *w, *vel;
    const float *g;
    const int *scatter_pos;
    float *w_csr;
    int nb;
    float *bias, *bias_vel;
    const float *gbias;
    float lr, mu, wd;
};
// Thread t of a layer takes the four connections 4t .. 4t+3 (16-byte loads and stores of the three streams;
// the state arrays are 256-byte aligned), the threads after ceil(n/4) take one bias each.
__device__ __forceinline__ void update_thread(const UpdateOne &u, long t)
{
#pragma clang fp contract(off)
    const long quads = (u.n + 3) / 4;
    if (t < quads) {
        const long e = 4 * t;
        if (e + 3 < u.n) {
            float4 w = ld4(u.w + e), v = ld4(u.vel + e);
            const float4 g = ld4(u.g + e);
            update_one(w.x, v.x, g.x, u.lr, u.mu, u.wd);
            update_one(w.y, v.y, g.y, u.lr, u.mu, u.wd);
            update_one(w.z, v.z, g.z, u.lr, u.mu, u.wd);
            update_one(w.w, v.w, g.w, u.lr, u.mu, u.wd);
            st4(u.vel + e, v);
            st4(u.w + e, w);
            if (u.scatter_pos) {
                const int4 pos = *reinterpret_cast<const int4 *>(u.scatter_pos + e);
                u.w_csr[pos.x] = w.x;
                u.w_csr[pos.y] = w.y;
                u.w_csr[pos.z] = w.z;
                u.w_csr[pos.w] = w.w;
            }
        } else {
            for (long i = e; i < u.n; ++i) {
                float w = u.w[i], v = u.vel[i];
                update_one(w, v, u.g[i], u.lr, u.mu, u.wd);
                u.vel[i] = v;
                u.w[i] = w;
                if (u.scatter_pos) u.w_csr[u.scatter_pos[i]] = w;
            }
        }
    } else if (t - quads < u.nb) {
        const long j = t - quads;
        const float vn = u.mu * u.bias_vel[j] - u.lr * u.gbias[j];
        u.bias_vel[j] = vn;
        u.bias[j] = u.bias[j] + vn;
    }
}
static long update_threads(long n, int nb) { return (n + 3) / 4 + nb; }

__global__ __launch_bounds__(BLOCK) void update_kernel(UpdateOne u)
{
    update_thread(u, (long)blockIdx.x * BLOCK + threadIdx.x);
}

// The same update for up to MAX_MULTI layers in ONE launch (small networks are bound by the number
// of dependent launches per step, not by bandwidth).
struct UpdateMany {
    int count;
    UpdateOne l[MAX_MULTI];
};
__global__ __launch_bounds__(BLOCK) void update_many_kernel(UpdateMany a)
{
    const long gt = (long)blockIdx.x * BLOCK + threadIdx.x;
    int k = 0;
    while (k + 1 < a.count && gt >= a.l[k + 1].first) ++k;
    update_thread(a.l[k], gt - a.l[k].first);
}

// ------------------------------------------------------------------------------------------------
// Softmax + cross-entropy.  One block; thread t handles samples t, t+blockDim, ...
// When gb is given (the output layer's bias gradient), the row sums of dz are produced as well, so
// that the output layer needs no separate activation-derivative pass.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void softmax_ce_kernel(const float *z, long ldz, const int *y, int B, int C,
                                                          float *dz, long lddz, float *loss_sum, float *gb)
{
    __shared__ float red[BLOCK];
    float loss = 0.f;
    const float invB = 1.f / (float)B;
    for (int b = threadIdx.x; b < B; b += BLOCK) {
        float m = z[b];
        for (int c = 1; c < C; ++c) m = fmaxf(m, z[c * ldz + b]);
        float s = 0.f;
        for (int c = 0; c < C; ++c) s += expf(z[c * ldz + b] - m);
        const int yb = y[b];
        const bool labelled = yb >= 0 && yb < C;   // a label outside [0, C) is "no target": never used as an index
        const float inv = 1.f / s;
        for (int c = 0; c < C; ++c) {
            const float p = expf(z[c * ldz + b] - m) * inv;
            dz[c * lddz + b] = (p - (c == yb ? 1.f : 0.f)) * invB;
        }
        if (labelled) loss += logf(s) - (z[(long)yb * ldz + b] - m);
    }
    red[threadIdx.x] = loss;
    __syncthreads();
    for (int m = BLOCK / 2; m >= 1; m >>= 1) {
        if ((int)threadIdx.x < m) red[threadIdx.x] += red[threadIdx.x + m];
        __syncthreads();
    }
    if (threadIdx.x == 0 && loss_sum) *loss_sum += red[0];
    if (!gb) return;
    // bias gradient of the output layer: gb[c] = sum_b dz[c][b], one block reduction per class; the
    // columns B .. roundup4(B)-1 of dz are zeroed for the float4 gathers of the backward kernel
    for (int c = 0; c < C; ++c) {
        __syncthreads();
        float s = 0.f;
        for (int b = threadIdx.x; b < B; b += BLOCK) s += dz[c * lddz + b];
        red[threadIdx.x] = s;
        __syncthreads();
        for (int m = BLOCK / 2; m >= 1; m >>= 1) {
            if ((int)threadIdx.x < m) red[threadIdx.x] += red[threadIdx.x + m];
            __syncthreads();
        }
        if (threadIdx.x == 0) gb[c] = red[0];
        if ((int)threadIdx.x < ((B + 3) & ~3) - B) dz[c * lddz + B + threadIdx.x] = 0.f;
    }
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
static int group_width(int B) { return B <= 32 ? 8 : B <= 64 ? 16 : B <= 128 ? 32 : 64; }
// rows so short that four of them are walked as one stream (span kernels)
static bool use_span(const SegMat &m, long nnz) { return !m.split && m.nv >= 64 && (double)nnz <= 3.0 * (double)m.nv; }

static int chunk_width(const SegMat &m, long nnz)
{
    const double mean = m.nv > 0 ? (double)nnz / (double)m.nv : 0.0;
    return mean <= 2.5 ? 2 : mean <= 6.0 ? 4 : 8;
}

template <typename F>
static void dispatch_gu(int G, int U, F &&f)
{
#define SL_CASE_U(GG)                                                                              \
    switch (U) {                                                                                   \
        case 2: f(std::integral_constant<int, GG>(), std::integral_constant<int, 2>()); break;     \
        case 4: f(std::integral_constant<int, GG>(), std::integral_constant<int, 4>()); break;     \
        default: f(std::integral_constant<int, GG>(), std::integral_constant<int, 8>()); break;    \
    }
    switch (G) {
        case 8: SL_CASE_U(8) break;
        case 16: SL_CASE_U(16) break;
        case 32: SL_CASE_U(32) break;
        default: SL_CASE_U(64) break;
    }
#undef SL_CASE_U
}
template <typename F>
static void dispatch_g(int G, F &&f)
{
    switch (G) {
        case 8: f(std::integral_constant<int, 8>()); break;
        case 16: f(std::integral_constant<int, 16>()); break;
        case 32: f(std::integral_constant<int, 32>()); break;
        default: f(std::integral_constant<int, 64>()); break;
    }
}

// the gathered operand of a CSR-ordered pass over L (its input x): rows used very many times each, and a 32-column slice
// of a few MB
static bool sliceable_operand(const sl_layer *L, const SegMat &m)
{
    return !m.split && (long)L->cfg.n_in * 128 <= (8L << 20) && L->nnz >= 64 * L->cfg.n_in;
}

static unsigned groups_to_blocks(long n_groups, int G) { return (unsigned)((n_groups + BLOCK / G - 1) / (BLOCK / G)); }

static void set_dropout(Epi &e, const sl_layer *owner)
{
    e.drop_thr = owner->drop_thr; e.drop_step = owner->drop_step; e.drop_scale = owner->drop_scale;
    e.k0 = (uint32_t)owner->cfg.seed ^ (uint32_t)(owner->cfg.layer_id * 0x9E3779B9u);
    e.k1 = (uint32_t)(owner->cfg.seed >> 32);
}

static Epi dz_epilogue(sl_layer *owner, int B)
{
    Epi e;
    e.mode = EPI_DZ; e.out = owner->dz; e.ldo = owner->ldz; e.bias = nullptr; e.mask_w = nullptr;
    e.mask_r = owner->mask; e.ldm = owner->ldm; e.gb = owner->grad_bias; e.act_kind = owner->cfg.act_kind;
    e.slope = owner->cfg.act_parity == 0 ? -owner->cfg.alpha : owner->cfg.alpha; e.B = B;
    set_dropout(e, owner);
    return e;
}

static void launch_fix(sl_layer *L, const SegMat &m, const Epi &epi, int G, int kernel_id, hipStream_t s,
                       const float *part = nullptr)
{
    FixArgs fx;
    fx.rvptr = m.rvptr; fx.n_rows = m.n_rows; fx.part = part ? part : (const float *)(L->scratch + L->cp.partial); fx.ldp = L->ldz;
    fx.epi = epi;
    ProfScope ps(L, kernel_id, s);
    dispatch_g(G, [&](auto g) {
        constexpr int GG = decltype(g)::value;
        if (m.n_rows < 8192) hipLaunchKernelGGL(fix_block_kernel<GG>, dim3((unsigned)m.n_rows), dim3(FIX_BLOCK), 0, s, fx);
        else hipLaunchKernelGGL(fix_kernel<GG>, dim3(groups_to_blocks(m.n_rows, GG)), dim3(BLOCK), 0, s, fx);
    });
}

int launch_forward(sl_layer *L, const float *x, int64_t ldx, int B, float *a, int64_t lda, bool save_sign, hipStream_t s,
                   float *part)
{
    const SegMat &m = L->fwd;
    int G = group_width(B);
    // An operand whose rows are each gathered very many times and whose 32-column slice (128 bytes per row) is a
    // few MB -- the 65 536-feature input block of the 10^6-neuron network: 8 MB per slice, every row used 160
    // times -- is walked one 32-column slice after the other (batch tiles in grid.y are dispatched in order), so
    // that an L2 serves a good part of the gathers.  Same arithmetic per element in the same order: same bits.
    if (G > 8 && sliceable_operand(L, m)) G = 8;
    const int U = chunk_width(m, L->nnz);
    const int tiles = (B + 4 * G - 1) / (4 * G);
    FwdArgs f;
    f.vptr = m.vptr; f.v2row = m.v2row; f.nv = m.nv; f.idx = m.idx; f.w = L->val; f.x = x; f.ldx = (int)ldx;
    // every row of a fully dense matrix has the same length, hence the same number of equal runs
    const bool dense = m.split && L->nnz == L->cfg.n_in * L->cfg.n_out && m.nv % m.n_rows == 0;
    f.twin_rows = dense && m.n_rows > 1 ? m.n_rows : 0;
    if (!part) part = (float *)(L->scratch + L->cp.partial);
    f.part = m.split ? part : nullptr; f.ldp = L->ldz;
    Epi &e = f.epi;
    e.mode = EPI_FWD; e.out = a; e.ldo = lda; e.bias = L->bias; e.mask_w = save_sign ? L->mask : nullptr; e.mask_r = nullptr; e.ldm = L->ldm;
    e.gb = nullptr; e.act_kind = L->cfg.act_kind; e.slope = L->cfg.act_parity == 0 ? -L->cfg.alpha : L->cfg.alpha; e.B = B;
    set_dropout(e, L);
    {
        ProfScope ps(L, K_FWD, s);
        if (use_span(m, L->nnz)) {
            dispatch_g(G, [&](auto g) {
                constexpr int GG = decltype(g)::value;
                dim3 grid(groups_to_blocks((m.nv + SPAN_R - 1) / SPAN_R, GG), (unsigned)tiles);
                hipLaunchKernelGGL(fwd_span_kernel<GG>, grid, dim3(BLOCK), 0, s, f);
            });
        } else {
            dispatch_gu(G, U, [&](auto g, auto u) {
                constexpr int GG = decltype(g)::value, UU = decltype(u)::value;
                dim3 grid(groups_to_blocks(m.nv, GG), (unsigned)tiles);
                hipLaunchKernelGGL((fwd_kernel<GG, UU>), grid, dim3(BLOCK), 0, s, f);
            });
        }
    }
    if (m.split) launch_fix(L, m, e, G, K_FWD_FIX, s, part);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

// ------------------------------------------------------------------------------------------------
// Forward pass whose partial sums live in a buffer that is part of the library's code object instead of
// the caller's scratch buffer (sparse_layer_infer_static): for callers that cannot allocate.  Every GPU
// holds its own copy of the array at its own address; `scratch` below is only the host-side name of the
// symbol, and the address that kernels and copies may use is the one hipGetSymbolAddress returns on that
// device.
// ------------------------------------------------------------------------------------------------
static constexpr size_t STATIC_SCRATCH_BYTES = (size_t)SL_STATIC_SCRATCH_MIB << 20;
static constexpr int STATIC_MAX_DEVICES = 64;
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
static std::mutex static_mu;
static void *static_ptr[STATIC_MAX_DEVICES] = {};

// Looks the array up on the current device (once per device).  Called from sparse_layer_init, so that the
// forward call itself finds the address ready, and again from the forward call in case the layer was
// created while another device was current.
int static_scratch_setup(sl_layer *L, void **ptr)
{
    int dev = -1;
    SL_HIP(L, hipGetDevice(&dev));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return set_err(L, SL_EINVAL, "device ordinal %d not supported", dev);
    std::lock_guard<std::mutex> lock(static_mu);
    if (!static_ptr[dev]) {
        void *p = nullptr;
        SL_HIP(L, hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return set_err(L, SL_EHIP, "hipGetSymbolAddress returned a null address");
        static_ptr[dev] = p;
    }
    if (ptr) *ptr = static_ptr[dev];
    return SL_OK;
}

int launch_forward_static(sl_layer *L, const float *x, int64_t ldx, int B, float *a, int64_t lda, hipStream_t s)
{
    if (L->prof_on) return set_err(L, SL_ESTATE, "infer_static: per-kernel profiling creates events; end it first");
    const SegMat &m = L->fwd;
    const size_t need = m.split ? sizeof(float) * (size_t)m.nv * (size_t)L->ldz : 0;
    if (need > STATIC_SCRATCH_BYTES)
        return set_err(L, SL_ENOMEM, "infer_static: %zu bytes of partial sums exceed the built-in buffer of %zu bytes", need,
                       STATIC_SCRATCH_BYTES);
    void *p = nullptr;
    int rc = static_scratch_setup(L, &p);
    if (rc) return rc;
    // nothing has to start at zero: the SpMM kernel writes every partial sum that the fix-up kernel reads
    return launch_forward(L, x, ldx, B, a, lda, false, s, (float *)p);
}

template <bool SPMM, bool UPD>
static void launch_bwd_kernel_u(int G, int U, int B, int nv, BwdArgs b, hipStream_t s)
{
    b.tile0 = 0;
    b.tile1 = (B + 4 * G - 1) / (4 * G);
    if (B > 256 && G == 64) {
        // One launch per pair of tiles: all groups then gather from the same 512 columns at a time (measured
        // 15 % faster at 1024 columns), and the stream order makes a later pair add to the gradient entries
        // that the earlier pair stored.  Very short rows (chunks of 2) walk all pairs in one launch instead:
        // there the second pass over the row pointers costs more than the locality gains.
        const dim3 grid(groups_to_blocks(nv, 64));
        const int tiles = b.tile1;
        if (U < 4) {
            hipLaunchKernelGGL((bwd_pair_kernel<2, SPMM, UPD>), grid, dim3(BLOCK), 0, s, b);
            return;
        }
        for (int t0 = 0; t0 < tiles; t0 += 2) {
            b.tile0 = t0;
            b.tile1 = min(t0 + 2, tiles);
            // only the launch that holds the last tile sees finished gradient entries
            if (UPD && b.tile1 == tiles) {
                if (U >= 8) hipLaunchKernelGGL((bwd_pair_kernel<4, SPMM, UPD>), grid, dim3(BLOCK), 0, s, b);
                else hipLaunchKernelGGL((bwd_pair_kernel<2, SPMM, UPD>), grid, dim3(BLOCK), 0, s, b);
            } else {
                if (U >= 8) hipLaunchKernelGGL((bwd_pair_kernel<4, SPMM, false>), grid, dim3(BLOCK), 0, s, b);
                else hipLaunchKernelGGL((bwd_pair_kernel<2, SPMM, false>), grid, dim3(BLOCK), 0, s, b);
            }
        }
        return;
    }
    const int tiles = b.tile1;
    const int per_launch = b.slice_tiles > 0 ? b.slice_tiles : tiles;   // slice_tiles: one launch per that many tiles
    for (int t0 = 0; t0 < tiles; t0 += per_launch) {
        b.tile0 = t0;
        b.tile1 = min(t0 + per_launch, tiles);
        dispatch_gu(G, U, [&](auto g, auto u) {
            constexpr int GG = decltype(g)::value, UU = decltype(u)::value;
            hipLaunchKernelGGL((bwd_kernel<GG, UU, SPMM, UPD>), dim3(groups_to_blocks(nv, GG)), dim3(BLOCK), 0, s, b);
        });
    }
}
// Batches above 256 columns take two tiles per pass with half the chunk width (the same number of row
// gathers in flight per lane).
template <bool SPMM>
static void launch_bwd_kernel(int G, int U, int B, int nv, const BwdArgs &b, hipStream_t s)
{
    if (b.upd_mode != 0) launch_bwd_kernel_u<SPMM, true>(G, U, B, nv, b, s);
    else launch_bwd_kernel_u<SPMM, false>(G, U, B, nv, b, s);
}

int launch_backward(sl_layer *L, const float *x, int64_t ldx, const float *ga, int64_t ldg, int B, float *gx,
                    int64_t ldgx, hipStream_t s)
{
    const int G = group_width(B);
    const int n_out = (int)L->cfg.n_out;
    if (L->dz_ready != B) {
        const Epi e = dz_epilogue(L, B);
        ProfScope ps(L, K_ACTGRAD, s);
        dispatch_g(G, [&](auto g) {
            constexpr int GG = decltype(g)::value;
            hipLaunchKernelGGL(actgrad_kernel<GG>, dim3(groups_to_blocks(n_out, GG)), dim3(BLOCK), 0, s, ga, (long)ldg,
                               n_out, e);
        });
    }
    L->dz_ready = 0;
    BwdArgs b;
    b.B = B; b.g = L->grad; b.ragged = (B % 4) != 0; b.part = nullptr; b.ldp = L->ldz;
    b.upd_mode = L->fuse_mode; b.n_tiles = (B + 4 * G - 1) / (4 * G); b.slice_tiles = 0;
    b.upd_w = L->has_csc ? L->valT : L->val; b.upd_vel = L->has_csc ? L->velT : L->vel;
    b.upd_pos = L->has_csc ? L->csr_pos : nullptr; b.upd_w_csr = L->val;
    b.lr = L->cfg.lr; b.mu = L->cfg.momentum; b.wd = L->cfg.weight_decay;
    if (L->has_csc) {
        const SegMat &m = L->bwd;
        const int U = chunk_width(m, L->nnz);
        b.vptr = m.vptr; b.v2row = m.v2row; b.nv = m.nv; b.idx = m.idx; b.w = L->valT;
        b.held = x; b.ldh = (int)ldx; b.gath = L->dz; b.ldga = L->ldz;
        if (m.split) b.part = (float *)(L->scratch + L->cp.partial);
        // Wide batches over columns of 7 to 16 connections: per-row work (row pointers, held row, epilogue) weighs
        // more against so few gathers of 1 KB, and one launch of 32-lane groups per 128-column slice is faster than
        // the 64-lane pair walk (262 144 x 262 144 layer with 8 connections per column, B = 512: 0.90 -> 0.77 ms);
        // from about 32 connections per column on the pair walk wins.
        int Gb = G;
        if (B > 256 && U == 8 && L->nnz <= 16 * (int64_t)m.nv) {
            Gb = 32;
            b.slice_tiles = 1;
            b.n_tiles = (B + 127) / 128;
        }
        sl_layer *P = gx ? nullptr : L->producer;
        if (P) {   // hand dz straight to the layer that produced x
            b.epi = dz_epilogue(P, B);
        } else {
            Epi &e = b.epi;
            e.mode = EPI_PLAIN; e.out = gx; e.ldo = ldgx; e.bias = nullptr; e.mask_w = nullptr; e.mask_r = nullptr;
            e.ldm = 0; e.gb = nullptr; e.act_kind = 0; e.slope = 0.f; e.B = B; e.drop_thr = 0u;
        }
        {
            ProfScope ps(L, K_BWD_FUSED, s);
            launch_bwd_kernel<true>(Gb, U, B, m.nv, b, s);
        }
        if (m.split) launch_fix(L, m, b.epi, Gb, K_BWD_FIX, s);
        if (P) P->dz_ready = B;
    } else {
        const SegMat &m = L->fwd;
        const int U = chunk_width(m, L->nnz);
        b.vptr = m.vptr; b.v2row = m.v2row; b.nv = m.nv; b.idx = m.idx; b.w = nullptr;
        b.held = L->dz; b.ldh = L->ldz; b.gath = x; b.ldga = (int)ldx;
        b.epi = Epi();
        int Gs = G;
        if (G > 8 && B <= 256 && sliceable_operand(L, m)) {   // as in the forward pass: one 32-column slice per launch
            Gs = 8;
            b.slice_tiles = 1;
            b.n_tiles = (B + 31) / 32;
        }
        ProfScope ps(L, K_SDDMM, s);
        launch_bwd_kernel<false>(Gs, U, B, m.nv, b, s);
    }
    SL_HIP(L, hipGetLastError());
    L->weights_updated = L->fuse_mode != 0;
    L->grad_stored = L->fuse_mode != 1;
    return SL_OK;
}

static UpdateOne update_args(const sl_layer *L)
{
    UpdateOne u;
    // after a backward pass that already applied eq. (1) to the connections only the biases are left
    u.n = L->weights_updated ? 0 : L->nnz; u.first = 0; u.nb = (int)L->cfg.n_out;
    u.w = L->has_csc ? L->valT : L->val; u.vel = L->has_csc ? L->velT : L->vel; u.g = L->grad;
    u.scatter_pos = L->has_csc ? L->csr_pos : nullptr; u.w_csr = L->has_csc ? L->val : nullptr;
    u.bias = L->bias; u.bias_vel = L->bias_vel; u.gbias = L->grad_bias;
    u.lr = L->cfg.lr; u.mu = L->cfg.momentum; u.wd = L->cfg.weight_decay;
    return u;
}

int launch_update(sl_layer *L, hipStream_t s)
{
    const UpdateOne u = update_args(L);
    const long total = update_threads(u.n, u.nb);
    ProfScope ps(L, K_UPDATE, s);
    hipLaunchKernelGGL(update_kernel, dim3((unsigned)((total + BLOCK - 1) / BLOCK)), dim3(BLOCK), 0, s, u);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int launch_softmax_ce(const float *z, int64_t ldz, const int32_t *y, int B, int C, float *dz, int64_t lddz,
                      float *loss_sum, float *gb, hipStream_t s)
{
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(1), dim3(BLOCK), 0, s, z, (long)ldz, y, B, C, dz, (long)lddz, loss_sum, gb);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_EHIP;
}

int launch_update_many(sl_layer *const *layers, int count, hipStream_t s)
{
    UpdateMany a;
    a.count = count;
    long first = 0;
    for (int k = 0; k < count; ++k) {
        a.l[k] = update_args(layers[k]);
        a.l[k].first = first;
        // every layer starts on a block boundary so that a block never straddles two layers
        first += ((update_threads(a.l[k].n, a.l[k].nb) + BLOCK - 1) / BLOCK) * BLOCK;
    }
    ProfScope ps(layers[0], K_UPDATE, s);
    hipLaunchKernelGGL(update_many_kernel, dim3((unsigned)(first / BLOCK)), dim3(BLOCK), 0, s, a);
    SL_HIP(layers[0], hipGetLastError());
    return SL_OK;
}

}  // namespace sl
