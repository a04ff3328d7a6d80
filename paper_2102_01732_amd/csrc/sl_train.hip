// Per-minibatch kernels of a truly sparse layer (gfx950): forward SpMM fused with All-ReLU,
// activation derivative, backward (transposed SpMM fused with the pattern-restricted SDDMM),
// momentum-SGD update and the softmax cross-entropy loss.
//
// Common shape of the sparse kernels.  Dense operands are feature-major [n][ld], so one stored
// connection touches ONE contiguous run of 4*B bytes of the dense operand.  A group of G lanes
// (G = 8/16/32/64 for B <= 32/64/128/256) owns one virtual row: each lane holds four batch
// columns as a float4, so a gather of one operand row is a single fully coalesced
// global_load_dwordx4 across the group, and 64/G rows are in flight per wavefront.  Entries are
// processed U at a time so that U independent row gathers are outstanding per group; the work is
// HBM-bound (0.5 flop/byte), so there is no MFMA here.
#include <stdarg.h>
#include <stdio.h>

#include "sl_internal.h"

namespace sl {

static constexpr int BLOCK = 256;
static constexpr int UNROLL = 8;

__device__ __forceinline__ float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ __forceinline__ void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }

// zero the components of v whose column c+k is >= B (ragged batch sizes only)
__device__ __forceinline__ float4 clip4(float4 v, int c, int B)
{
    v.y = (c + 1 < B) ? v.y : 0.f;
    v.z = (c + 2 < B) ? v.z : 0.f;
    v.w = (c + 3 < B) ? v.w : 0.f;
    return v;
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

// ------------------------------------------------------------------------------------------------
// Forward: z = Wt x + b, a = f_l(z) (eq. 3).  One group per virtual row.
// ------------------------------------------------------------------------------------------------
struct FwdArgs {
    const int *vptr;
    const int *v2row;
    int nv;
    const int *idx;
    const float *w;
    const float *x;
    long ldx;
    const float *bias;
    float *out;      // a [n_out][ldo], or partial sums [nv][ldo] when partial != 0
    long ldo;
    uint8_t *mask;   // [n_out][ldm] one byte per float4: bit k set <=> z[4q+k] > 0
    long ldm;
    int B;
    int act_kind;
    float slope;     // -alpha (even layer) or +alpha (odd layer)
    int partial;
};

__device__ __forceinline__ void finish_row(const FwdArgs &a, long row, int c, float4 z)
{
    float4 r = z;
    if (a.act_kind != 0) {
        unsigned nib = (z.x > 0.f ? 1u : 0u) | (z.y > 0.f ? 2u : 0u) | (z.z > 0.f ? 4u : 0u) | (z.w > 0.f ? 8u : 0u);
        a.mask[row * a.ldm + (c >> 2)] = (uint8_t)nib;
        r.x = z.x > 0.f ? z.x : a.slope * z.x;
        r.y = z.y > 0.f ? z.y : a.slope * z.y;
        r.z = z.z > 0.f ? z.z : a.slope * z.z;
        r.w = z.w > 0.f ? z.w : a.slope * z.w;
    }
    store_row4(a.out + row * a.ldo, c, a.B, r);
}

template <int G>
__global__ __launch_bounds__(BLOCK) void fwd_kernel(FwdArgs a)
{
    constexpr int U = UNROLL;
    const int lane = threadIdx.x % G;
    const long v = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    const int c = (blockIdx.y * G + lane) * 4;
    if (v >= a.nv || c >= a.B) return;
    const int p0 = a.vptr[v], p1 = a.vptr[v + 1];
    const float *xb = a.x + c;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
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
    if (a.partial) {
        st4(a.out + v * a.ldo + c, acc);
        return;
    }
    const long row = a.v2row ? a.v2row[v] : v;
    const float b = a.bias ? a.bias[row] : 0.f;
    finish_row(a, row, c, make_float4(acc.x + b, acc.y + b, acc.z + b, acc.w + b));
}

// Split matrices only: adds the partial sums of a row's virtual rows in order, then finishes the
// row (bias, activation, sign mask).  One group per row.
struct FixArgs {
    const int *rvptr;
    int n_rows;
    const float *part;
    long ldp;
    FwdArgs f;
};

template <int G>
__global__ __launch_bounds__(BLOCK) void fix_kernel(FixArgs a)
{
    const int lane = threadIdx.x % G;
    const long row = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    const int c = (blockIdx.y * G + lane) * 4;
    if (row >= a.n_rows || c >= a.f.B) return;
    const int v0 = a.rvptr[row], v1 = a.rvptr[row + 1];
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    int v = v0;
    for (; v + 4 <= v1; v += 4) {
        float4 t0 = ld4(a.part + (long)(v + 0) * a.ldp + c), t1 = ld4(a.part + (long)(v + 1) * a.ldp + c);
        float4 t2 = ld4(a.part + (long)(v + 2) * a.ldp + c), t3 = ld4(a.part + (long)(v + 3) * a.ldp + c);
        acc.x = ((acc.x + t0.x) + t1.x) + t2.x + t3.x;
        acc.y = ((acc.y + t0.y) + t1.y) + t2.y + t3.y;
        acc.z = ((acc.z + t0.z) + t1.z) + t2.z + t3.z;
        acc.w = ((acc.w + t0.w) + t1.w) + t2.w + t3.w;
    }
    for (; v < v1; ++v) {
        float4 t = ld4(a.part + (long)v * a.ldp + c);
        acc.x += t.x; acc.y += t.y; acc.z += t.z; acc.w += t.w;
    }
    const float b = a.f.bias ? a.f.bias[row] : 0.f;
    finish_row(a.f, row, c, make_float4(acc.x + b, acc.y + b, acc.z + b, acc.w + b));
}

// ------------------------------------------------------------------------------------------------
// dz = grad_a * f_l'(z), grad_bias = row sums of dz.  One group per row, tiles of 4*G columns.
// Columns B .. roundup4(B)-1 of dz are written as zeros so that later float4 gathers are clean.
// ------------------------------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(BLOCK) void actgrad_kernel(const float *ga, long ldg, const uint8_t *mask, long ldm,
                                                       float *dz, long ldz, float *gb, int n_out, int B,
                                                       int act_kind, float slope)
{
    const int lane = threadIdx.x % G;
    const long row = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (row >= n_out) return;   // whole groups leave together
    float sum = 0.f;
    for (int c = lane * 4; c < B; c += 4 * G) {
        float4 g;
        if (c + 3 < B) {
            g = ld4(ga + row * ldg + c);
        } else {
            g.x = ga[row * ldg + c];
            g.y = (c + 1 < B) ? ga[row * ldg + c + 1] : 0.f;
            g.z = (c + 2 < B) ? ga[row * ldg + c + 2] : 0.f;
            g.w = 0.f;
        }
        if (act_kind != 0) {
            const unsigned nib = mask[row * ldm + (c >> 2)];
            g.x = g.x * ((nib & 1u) ? 1.f : slope);
            g.y = g.y * ((nib & 2u) ? 1.f : slope);
            g.z = g.z * ((nib & 4u) ? 1.f : slope);
            g.w = g.w * ((nib & 8u) ? 1.f : slope);
            g = clip4(g, c, B);
        }
        st4(dz + row * ldz + c, g);
        sum += (g.x + g.y) + (g.z + g.w);
    }
#pragma unroll
    for (int m = G / 2; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, G);
    if (lane == 0) gb[row] = sum;
}

// ------------------------------------------------------------------------------------------------
// Backward.  One kernel covers both uses:
//   SPMM = true  (layers that need grad_x; runs over the CSC view, one group per input neuron i):
//       holds x[i], gathers dz[j] for every stored (j,i) ONCE and uses it twice:
//       grad_x[i] += Wt[j,i] * dz[j]          (transposed SpMM)
//       grad[q]    = <dz[j], x[i]>            (SDDMM restricted to the pattern)
//   SPMM = false (first layer; runs over CSR, one group per output neuron j):
//       holds dz[j], gathers x[i], grad[p] = <dz[j], x[i]>.
// The U dot products of a chunk are reduced together: three exchange steps fold 8 values per lane
// into one (lane l keeps the sum for entry l & 7), the remaining log2(G/8) steps are plain
// butterflies, so a chunk costs 7 + log2(G/8) cross-lane moves instead of 8 * log2(G).
// ------------------------------------------------------------------------------------------------
struct BwdArgs {
    const int *vptr;
    const int *v2row;
    int nv;
    const int *idx;
    const float *w;
    const float *held;
    long ldh;
    const float *gath;
    long ldga;
    float *g;        // per stored entry, in the order of this orientation
    float *out;      // SPMM result rows [n][ldo], or partial sums [nv][ldo]
    long ldo;
    int B;
    int partial;
};

template <int G>
__device__ __forceinline__ float reduce8(float (&s)[8], int lane)
{
#pragma unroll
    for (int m = 0; m < 3; ++m) {
        const bool up = (lane >> m) & 1;
#pragma unroll
        for (int t = 0; t < (4 >> m); ++t) {
            const float lo = s[2 * t], hi = s[2 * t + 1];
            const float send = up ? lo : hi;
            const float keep = up ? hi : lo;
            s[t] = keep + __shfl_xor(send, 1 << m, G);
        }
    }
    float r = s[0];
#pragma unroll
    for (int m = 8; m < G; m <<= 1) r += __shfl_xor(r, m, G);
    return r;
}

template <int G, bool SPMM, bool RAGGED>
__global__ __launch_bounds__(BLOCK) void bwd_kernel(BwdArgs a)
{
    constexpr int U = 8;
    const int lane = threadIdx.x % G;
    const long v = (long)blockIdx.x * (BLOCK / G) + threadIdx.x / G;
    if (v >= a.nv) return;   // whole groups leave together
    const int p0 = a.vptr[v], p1 = a.vptr[v + 1];
    const long row = a.v2row ? a.v2row[v] : v;
    for (int tile = 0; tile * 4 * G < a.B; ++tile) {
        const int c = (tile * G + lane) * 4;
        const bool active = c < a.B;
        float4 h = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active) {
            h = ld4(a.held + row * a.ldh + c);
            if (RAGGED) h = clip4(h, c, a.B);
        }
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int p = p0; p < p1; p += U) {
            int cc[U];
            float ww[U];
            float4 xv[U];
            float s[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int q = min(p + u, p1 - 1);
                cc[u] = a.idx[q];
                if (SPMM) ww[u] = (p + u < p1) ? a.w[q] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                xv[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (active) {
                    xv[u] = ld4(a.gath + (long)cc[u] * a.ldga + c);
                    if (RAGGED) xv[u] = clip4(xv[u], c, a.B);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (SPMM) {
                    acc.x = fmaf(ww[u], xv[u].x, acc.x);
                    acc.y = fmaf(ww[u], xv[u].y, acc.y);
                    acc.z = fmaf(ww[u], xv[u].z, acc.z);
                    acc.w = fmaf(ww[u], xv[u].w, acc.w);
                }
                s[u] = fmaf(h.x, xv[u].x, fmaf(h.y, xv[u].y, fmaf(h.z, xv[u].z, h.w * xv[u].w)));
            }
            const float r = reduce8<G>(s, lane);
            if (lane < U && p + lane < p1) {
                if (tile == 0) a.g[p + lane] = r;
                else a.g[p + lane] += r;
            }
        }
        if (SPMM && active) {
            if (a.partial) st4(a.out + v * a.ldo + c, acc);
            else store_row4(a.out + row * a.ldo, c, a.B, acc);
        }
    }
}

// ------------------------------------------------------------------------------------------------
// Momentum SGD, eq. (1) in velocity form, over the stored connections and the biases.  The
// products are rounded separately (no fused multiply-add) so that the result is the plain fp32
// evaluation of  vel = mu*vel - eta*(g + lambda*w);  w = w + vel.
// With a CSC view the master copy is in CSC order and the CSR copy read by forward is refreshed
// through csr_pos.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void update_kernel(long n, float *w, float *vel, const float *g, float lr,
                                                      float mu, float wd, const int *scatter_pos, float *w_csr,
                                                      int nb, float *bias, float *bias_vel, const float *gbias)
{
#pragma clang fp contract(off)   // separate roundings: this must equal the plain fp32 evaluation
    const long t = (long)blockIdx.x * BLOCK + threadIdx.x;
    if (t < n) {
        const float wt = w[t];
        const float gg = g[t] + wd * wt;
        const float vn = mu * vel[t] - lr * gg;
        const float wn = wt + vn;
        vel[t] = vn;
        w[t] = wn;
        if (scatter_pos) w_csr[scatter_pos[t]] = wn;
    } else if (t - n < nb) {
        const long j = t - n;
        const float vn = mu * bias_vel[j] - lr * gbias[j];
        bias_vel[j] = vn;
        bias[j] = bias[j] + vn;
    }
}

// ------------------------------------------------------------------------------------------------
// Softmax + cross-entropy.  One block; thread t handles samples t, t+blockDim, ...
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(BLOCK) void softmax_ce_kernel(const float *z, long ldz, const int *y, int B, int C,
                                                          float *dz, long lddz, float *loss_sum)
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
        const float inv = 1.f / s;
        for (int c = 0; c < C; ++c) {
            const float p = expf(z[c * ldz + b] - m) * inv;
            dz[c * lddz + b] = (p - (c == yb ? 1.f : 0.f)) * invB;
        }
        loss += logf(s) - (z[(long)yb * ldz + b] - m);
    }
    red[threadIdx.x] = loss;
    __syncthreads();
    for (int m = BLOCK / 2; m >= 1; m >>= 1) {
        if ((int)threadIdx.x < m) red[threadIdx.x] += red[threadIdx.x + m];
        __syncthreads();
    }
    if (threadIdx.x == 0 && loss_sum) *loss_sum += red[0];
}

// ------------------------------------------------------------------------------------------------
// host launchers
// ------------------------------------------------------------------------------------------------
static int group_width(int B) { return B <= 32 ? 8 : B <= 64 ? 16 : B <= 128 ? 32 : 64; }

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

int launch_forward(sl_layer *L, const float *x, int64_t ldx, int B, float *a, int64_t lda, hipStream_t s)
{
    const SegMat &m = L->fwd;
    const int G = group_width(B);
    const int tiles = (B + 4 * G - 1) / (4 * G);
    FwdArgs f;
    f.vptr = m.vptr; f.v2row = m.v2row; f.nv = m.nv; f.idx = m.idx; f.w = L->val; f.x = x; f.ldx = ldx;
    f.bias = L->bias; f.out = a; f.ldo = lda; f.mask = L->mask; f.ldm = L->ldm; f.B = B;
    f.act_kind = L->cfg.act_kind; f.slope = L->cfg.act_parity == 0 ? -L->cfg.alpha : L->cfg.alpha;
    f.partial = 0;
    if (!m.split) {
        dispatch_g(G, [&](auto g) {
            constexpr int GG = decltype(g)::value;
            dim3 grid((unsigned)((m.nv + BLOCK / GG - 1) / (BLOCK / GG)), (unsigned)tiles);
            ProfScope ps(L, K_FWD, s);
            hipLaunchKernelGGL(fwd_kernel<GG>, grid, dim3(BLOCK), 0, s, f);
        });
    } else {
        FwdArgs pa = f;
        pa.partial = 1; pa.out = (float *)(L->scratch + L->cp.partial); pa.ldo = L->ldz;
        FixArgs fx;
        fx.rvptr = m.rvptr; fx.n_rows = m.n_rows; fx.part = pa.out; fx.ldp = L->ldz; fx.f = f;
        dispatch_g(G, [&](auto g) {
            constexpr int GG = decltype(g)::value;
            dim3 grid((unsigned)((m.nv + BLOCK / GG - 1) / (BLOCK / GG)), (unsigned)tiles);
            {
                ProfScope ps(L, K_FWD, s);
                hipLaunchKernelGGL(fwd_kernel<GG>, grid, dim3(BLOCK), 0, s, pa);
            }
            dim3 grid2((unsigned)((m.n_rows + BLOCK / GG - 1) / (BLOCK / GG)), (unsigned)tiles);
            ProfScope ps(L, K_FWD_FIX, s);
            hipLaunchKernelGGL(fix_kernel<GG>, grid2, dim3(BLOCK), 0, s, fx);
        });
    }
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int launch_backward(sl_layer *L, const float *x, int64_t ldx, const float *ga, int64_t ldg, int B, float *gx,
                    int64_t ldgx, hipStream_t s)
{
    const int G = group_width(B);
    const float slope = L->cfg.act_parity == 0 ? -L->cfg.alpha : L->cfg.alpha;
    const int n_out = (int)L->cfg.n_out;
    dispatch_g(G, [&](auto g) {
        constexpr int GG = decltype(g)::value;
        dim3 grid((unsigned)((n_out + BLOCK / GG - 1) / (BLOCK / GG)));
        ProfScope ps(L, K_ACTGRAD, s);
        hipLaunchKernelGGL(actgrad_kernel<GG>, grid, dim3(BLOCK), 0, s, ga, (long)ldg, L->mask, (long)L->ldm, L->dz,
                           (long)L->ldz, L->grad_bias, n_out, B, L->cfg.act_kind, slope);
    });
    const bool ragged = (B % 4) != 0;
    BwdArgs b;
    b.B = B; b.g = L->grad; b.partial = 0;
    if (L->has_csc) {
        const SegMat &m = L->bwd;
        b.vptr = m.vptr; b.v2row = m.v2row; b.nv = m.nv; b.idx = m.idx; b.w = L->valT;
        b.held = x; b.ldh = ldx; b.gath = L->dz; b.ldga = L->ldz; b.out = gx; b.ldo = ldgx;
        if (m.split) { b.partial = 1; b.out = (float *)(L->scratch + L->cp.partial); b.ldo = L->ldz; }
        dispatch_g(G, [&](auto g) {
            constexpr int GG = decltype(g)::value;
            dim3 grid((unsigned)((m.nv + BLOCK / GG - 1) / (BLOCK / GG)));
            {
                ProfScope ps(L, K_BWD_FUSED, s);
                if (ragged) hipLaunchKernelGGL((bwd_kernel<GG, true, true>), grid, dim3(BLOCK), 0, s, b);
                else hipLaunchKernelGGL((bwd_kernel<GG, true, false>), grid, dim3(BLOCK), 0, s, b);
            }
            if (m.split) {
                FixArgs fx;
                fx.rvptr = m.rvptr; fx.n_rows = m.n_rows; fx.part = b.out; fx.ldp = L->ldz;
                fx.f.vptr = nullptr; fx.f.v2row = nullptr; fx.f.nv = 0; fx.f.idx = nullptr; fx.f.w = nullptr;
                fx.f.x = nullptr; fx.f.ldx = 0; fx.f.bias = nullptr; fx.f.out = gx; fx.f.ldo = ldgx;
                fx.f.mask = nullptr; fx.f.ldm = 0; fx.f.B = B; fx.f.act_kind = 0; fx.f.slope = 0.f; fx.f.partial = 0;
                const int tiles = (B + 4 * GG - 1) / (4 * GG);
                dim3 grid2((unsigned)((m.n_rows + BLOCK / GG - 1) / (BLOCK / GG)), (unsigned)tiles);
                ProfScope ps(L, K_BWD_FIX, s);
                hipLaunchKernelGGL(fix_kernel<GG>, grid2, dim3(BLOCK), 0, s, fx);
            }
        });
    } else {
        const SegMat &m = L->fwd;
        b.vptr = m.vptr; b.v2row = m.v2row; b.nv = m.nv; b.idx = m.idx; b.w = nullptr;
        b.held = L->dz; b.ldh = L->ldz; b.gath = x; b.ldga = ldx; b.out = nullptr; b.ldo = 0;
        dispatch_g(G, [&](auto g) {
            constexpr int GG = decltype(g)::value;
            dim3 grid((unsigned)((m.nv + BLOCK / GG - 1) / (BLOCK / GG)));
            ProfScope ps(L, K_SDDMM, s);
            if (ragged) hipLaunchKernelGGL((bwd_kernel<GG, false, true>), grid, dim3(BLOCK), 0, s, b);
            else hipLaunchKernelGGL((bwd_kernel<GG, false, false>), grid, dim3(BLOCK), 0, s, b);
        });
    }
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int launch_update(sl_layer *L, hipStream_t s)
{
    const long n = L->nnz;
    const int nb = (int)L->cfg.n_out;
    const long total = n + nb;
    dim3 grid((unsigned)((total + BLOCK - 1) / BLOCK));
    ProfScope ps(L, K_UPDATE, s);
    if (L->has_csc)
        hipLaunchKernelGGL(update_kernel, grid, dim3(BLOCK), 0, s, n, L->valT, L->velT, L->grad, L->cfg.lr,
                           L->cfg.momentum, L->cfg.weight_decay, L->csr_pos, L->val, nb, L->bias, L->bias_vel,
                           L->grad_bias);
    else
        hipLaunchKernelGGL(update_kernel, grid, dim3(BLOCK), 0, s, n, L->val, L->vel, L->grad, L->cfg.lr,
                           L->cfg.momentum, L->cfg.weight_decay, (const int *)nullptr, (float *)nullptr, nb, L->bias,
                           L->bias_vel, L->grad_bias);
    SL_HIP(L, hipGetLastError());
    return SL_OK;
}

int launch_softmax_ce(const float *z, int64_t ldz, const int32_t *y, int B, int C, float *dz, int64_t lddz,
                      float *loss_sum, hipStream_t s)
{
    hipLaunchKernelGGL(softmax_ce_kernel, dim3(1), dim3(BLOCK), 0, s, z, (long)ldz, y, B, C, dz, (long)lddz, loss_sum);
    return hipGetLastError() == hipSuccess ? SL_OK : SL_EHIP;
}

}  // namespace sl
