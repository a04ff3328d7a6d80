// Stand-alone microbenchmark (not part of libsparse_set.so): the rate at which one MI355X can gather
// random rows of 16*G bytes (one stored connection at a batch of 4*G columns: G = 8, 32, 64 lanes for
// B = 32, 128, 256) as a function of the number of rows of the operand they come from.  It gives the
// ceiling the sparse kernels are measured against.  At 512-byte rows: ~26 TB/s while the operand fits the
// 4 MB L2 of an XCD, ~8.5 TB/s at 32 MB, ~7.5 TB/s at 512 MB (L2 miss path), ~6.8 TB/s at 2 GB.
//   python -m paper_2102_01732_amd.build --gather-ceiling && paper_2102_01732_amd/gather_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#include <random>

#define CHECK(e) do { hipError_t r_ = (e); if (r_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #e, hipGetErrorString(r_)); exit(1); } } while (0)

// each group of G lanes gathers `per` rows of 16*G bytes (float4 per lane), 8 in flight
template <int G>
__global__ __launch_bounds__(256) void gather(const float *x, const int *idx, long ngroups, int per, float *out)
{
    const long g = (long)blockIdx.x * (256 / G) + threadIdx.x / G;
    const int lane = threadIdx.x % G;
    if (g >= ngroups) return;
    const int *my = idx + g * per;
    float4 acc = make_float4(0, 0, 0, 0);
    for (int p = 0; p < per; p += 8) {
        int c[8];
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = my[p + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *(const float4 *)(x + (long)c[u] * (4 * G) + lane * 4);
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    if (acc.x == 12345.f) out[g] = acc.y + acc.z + acc.w;   // never true: keeps the loads alive
}

template <int G>
static void run(const std::vector<long> &row_counts, long total_bytes)
{
    const int per = 16;
    const long row_bytes = 16L * G;
    const long ngroups = total_bytes / (row_bytes * per);   // the same gathered volume for every width
    std::vector<int> h((size_t)ngroups * per);
    float *out;
    int *didx;
    CHECK(hipMalloc(&out, ngroups * 4));
    CHECK(hipMalloc(&didx, h.size() * 4));
    printf("# rows of %ld bytes (B = %d), %.1f M gathers per launch, 8 outstanding per %d-lane group\n", row_bytes, 4 * G,
           ngroups * per / 1e6, G);
    for (long rows : row_counts) {
        std::mt19937 rng(1);
        for (auto &v : h) v = (int)(rng() % rows);
        CHECK(hipMemcpy(didx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
        float *x;
        CHECK(hipMalloc(&x, rows * row_bytes));
        CHECK(hipMemset(x, 0, rows * row_bytes));
        hipEvent_t a, b;
        CHECK(hipEventCreate(&a));
        CHECK(hipEventCreate(&b));
        const unsigned blocks = (unsigned)((ngroups + 256 / G - 1) / (256 / G));
        for (int rep = 0; rep < 2; ++rep) {   // the second pass is the measurement
            CHECK(hipEventRecord(a));
            for (int i = 0; i < 5; ++i) hipLaunchKernelGGL(gather<G>, dim3(blocks), dim3(256), 0, 0, x, didx, ngroups, per, out);
            CHECK(hipEventRecord(b));
            CHECK(hipEventSynchronize(b));
        }
        float ms;
        CHECK(hipEventElapsedTime(&ms, a, b));
        ms /= 5;
        printf("operand %8ld rows %7.1f MB: %.3f ms, %.2f TB/s gathered (+%.2f GB index stream)\n", rows, rows * row_bytes / 1e6, ms,
               ngroups * per * (double)row_bytes / ms / 1e9, h.size() * 4 / 1e9);
        fflush(stdout);
        CHECK(hipEventDestroy(a));
        CHECK(hipEventDestroy(b));
        CHECK(hipFree(x));
    }
    CHECK(hipFree(out));
    CHECK(hipFree(didx));
}

// Second question: would a traversal blocked by operand rows let the per-XCD L2 serve the gathers WITHOUT barriers?
// Resident groups (the whole grid fits the chip at once) each walk the column blocks of a 128 MB operand in the same
// order, four passes, eight random rows of the current block per step -- the access stream of a blocked forward pass of
// the densest sweep layer (262 144 x 262 144, 3.4e7 connections, B = 128) with accumulators kept on chip.  Nothing
// synchronises the groups; if they stayed within a block or two of each other an L2 (4 MB) would hold what they read.
__global__ __launch_bounds__(256) void walk(const float *x, const int *idx, int ngroups, int steps, float *out)
{
    const int g = blockIdx.x * 8 + threadIdx.x / 32;
    const int lane = threadIdx.x % 32;
    if (g >= ngroups) return;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const int *my = idx + (long)g * steps * 8;
    for (int s = 0; s < steps; ++s) {
        int c[8];
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) c[u] = my[s * 8 + u];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = *(const float4 *)(x + (long)c[u] * 128 + lane * 4);
#pragma unroll
        for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
    }
    if (acc.x == 12345.f) out[g] = acc.y + acc.z + acc.w;   // never true: keeps the loads alive
}

static void run_walk()
{
    const int n = 262144;
    const long total = 33554432;   // gathers per launch
    float *x, *out;
    int *didx;
    CHECK(hipMalloc(&x, (size_t)n * 512));
    CHECK(hipMemset(x, 0, (size_t)n * 512));
    CHECK(hipMalloc(&didx, total * 4));
    CHECK(hipMalloc(&out, 16384 * 4));
    printf("# blocked walk without barriers: 3.4e7 gathers of 512-byte rows from a 134 MB operand by resident groups that visit its\n"
           "# column blocks in the same order (4 passes); 1 block = no blocking\n");
    std::vector<int> h((size_t)total);
    for (int ngroups : {16384, 8192})
        for (int nb : {1, 32, 64, 128, 256}) {
            const int steps = (int)(total / 8 / ngroups);
            const int passes = nb == 1 ? 1 : 4;
            const int per_block = steps / (passes * nb) > 0 ? steps / (passes * nb) : 1;
            const int bsize = n / nb;
            std::mt19937 rng(7);
            for (int g = 0; g < ngroups; ++g)
                for (int s = 0; s < steps; ++s) {
                    const int blk = nb == 1 ? 0 : (s / per_block) % nb;
                    for (int u = 0; u < 8; ++u) h[((size_t)g * steps + s) * 8 + u] = blk * bsize + (int)(rng() % bsize);
                }
            CHECK(hipMemcpy(didx, h.data(), total * 4, hipMemcpyHostToDevice));
            hipEvent_t a, b;
            CHECK(hipEventCreate(&a));
            CHECK(hipEventCreate(&b));
            float best = 1e9f;
            for (int rep = 0; rep < 4; ++rep) {
                CHECK(hipEventRecord(a));
                hipLaunchKernelGGL(walk, dim3(ngroups / 8), dim3(256), 0, 0, x, didx, ngroups, steps, out);
                CHECK(hipEventRecord(b));
                CHECK(hipEventSynchronize(b));
                float ms;
                CHECK(hipEventElapsedTime(&ms, a, b));
                if (rep > 0 && ms < best) best = ms;
            }
            printf("%5d groups, %3d column blocks of %6.2f MB: %.3f ms, %.2f TB/s gathered\n", ngroups, nb, bsize * 512.0 / 1e6,
                   best, total * 512.0 / best / 1e9);
            fflush(stdout);
            CHECK(hipEventDestroy(a));
            CHECK(hipEventDestroy(b));
        }
    CHECK(hipFree(x));
    CHECK(hipFree(out));
    CHECK(hipFree(didx));
}

// The same walk in lock-step: the workgroups of one XCD (read from the XCC_ID hardware register) wait, before they start
// column block k, until all of them have finished block k - slack, so that the XCD's L2 holds the blocks being read.
// Every wait is bounded (spin_limit polls, then the workgroup goes on and the launch counts a time-out), every workgroup
// of the grid is resident (1024 or 2048 workgroups of 256 threads on 256 CUs), so every wave reaches the end.
__device__ __forceinline__ unsigned ld_acquire(const unsigned *p) { return __hip_atomic_load(p, __ATOMIC_ACQUIRE, __HIP_MEMORY_SCOPE_AGENT); }

__global__ __launch_bounds__(256) void walk_sync(const float *x, const int *idx, int ngroups, int steps, int per_block, int n_visits,
                                                 int slack, int spin_limit, unsigned *done /* [8][n_visits] */,
                                                 unsigned *xcd_groups /* [8] workgroups per XCD, [8] = all arrived, [9] = time-outs */,
                                                 float *out)
{
    __shared__ unsigned my_total;
    const int xcc = (int)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 7u);   // HW_REG_XCC_ID, bits 3:0
    if (threadIdx.x == 0) {
        // sign in, then wait (bounded) until the whole grid has: after that the per-XCD head counts are final
        __hip_atomic_fetch_add(&xcd_groups[xcc], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_fetch_add(&xcd_groups[8], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
        int spins = 0;
        while (ld_acquire(&xcd_groups[8]) < gridDim.x && ++spins < 100 * spin_limit) __builtin_amdgcn_s_sleep(2);
        my_total = ld_acquire(&xcd_groups[xcc]);
    }
    __syncthreads();
    const unsigned mates = my_total;
    const int g = blockIdx.x * 8 + threadIdx.x / 32;
    const int lane = threadIdx.x % 32;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    const int *my = idx + (long)min(g, ngroups - 1) * steps * 8;
    for (int kb = 0; kb < n_visits; ++kb) {
        if (kb >= slack) {
            if (threadIdx.x == 0) {
                int spins = 0;
                while (ld_acquire(&done[xcc * n_visits + kb - slack]) < mates && ++spins < spin_limit) __builtin_amdgcn_s_sleep(1);
                if (spins >= spin_limit) __hip_atomic_fetch_add(&xcd_groups[9], 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            __syncthreads();
        }
        for (int s = kb * per_block; s < (kb + 1) * per_block; ++s) {
            int c[8];
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) c[u] = my[s * 8 + u];
#pragma unroll
            for (int u = 0; u < 8; ++u) v[u] = *(const float4 *)(x + (long)c[u] * 128 + lane * 4);
#pragma unroll
            for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
        }
        __syncthreads();   // the loads above have returned (their values were added) in every wave of the workgroup
        if (threadIdx.x == 0) __hip_atomic_fetch_add(&done[xcc * n_visits + kb], 1u, __ATOMIC_RELEASE, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (acc.x == 12345.f) out[g] = acc.y + acc.z + acc.w;   // never true: keeps the loads alive
}

static void run_walk_sync()
{
    const int n = 262144;
    const long total = 33554432;   // gathers per launch
    float *x, *out;
    int *didx;
    unsigned *done, *xg;
    CHECK(hipMalloc(&x, (size_t)n * 512));
    CHECK(hipMemset(x, 0, (size_t)n * 512));
    CHECK(hipMalloc(&didx, total * 4));
    CHECK(hipMalloc(&out, 16384 * 4));
    CHECK(hipMalloc(&done, 8 * 4096 * 4));
    CHECK(hipMalloc(&xg, 16 * 4));
    printf("# blocked walk in lock-step per XCD (bounded waits; slack = column blocks a workgroup may run ahead of the slowest of its XCD)\n");
    std::vector<int> h((size_t)total);
    for (int ngroups : {16384, 8192})
        for (int nb : {32, 64, 128})
            for (int slack : {1, 2}) {
                const int steps = (int)(total / 8 / ngroups);
                const int passes = 4;
                const int per_block = steps / (passes * nb);
                if (per_block < 1) continue;
                const int n_visits = passes * nb;
                const int bsize = n / nb;
                std::mt19937 rng(7);
                for (int g = 0; g < ngroups; ++g)
                    for (int s = 0; s < steps; ++s) {
                        const int blk = (s / per_block) % nb;
                        for (int u = 0; u < 8; ++u) h[((size_t)g * steps + s) * 8 + u] = blk * bsize + (int)(rng() % bsize);
                    }
                CHECK(hipMemcpy(didx, h.data(), total * 4, hipMemcpyHostToDevice));
                hipEvent_t a, b;
                CHECK(hipEventCreate(&a));
                CHECK(hipEventCreate(&b));
                float best = 1e9f;
                unsigned info[16] = {0};
                for (int rep = 0; rep < 4; ++rep) {
                    CHECK(hipMemset(done, 0, 8 * 4096 * 4));
                    CHECK(hipMemset(xg, 0, 16 * 4));
                    CHECK(hipEventRecord(a));
                    hipLaunchKernelGGL(walk_sync, dim3(ngroups / 8), dim3(256), 0, 0, x, didx, ngroups, steps, per_block, n_visits, slack,
                                       2000, done, xg, out);
                    CHECK(hipEventRecord(b));
                    CHECK(hipEventSynchronize(b));
                    float ms;
                    CHECK(hipEventElapsedTime(&ms, a, b));
                    if (rep > 0 && ms < best) best = ms;
                    CHECK(hipMemcpy(info, xg, sizeof(info), hipMemcpyDeviceToHost));
                }
                printf("%5d groups, %3d column blocks of %5.2f MB, slack %d: %.3f ms, %.2f TB/s gathered; workgroups per XCD %u %u %u %u %u %u %u %u, waits timed out %u\n",
                       ngroups, nb, bsize * 512.0 / 1e6, slack, best, total * 512.0 / best / 1e9, info[0], info[1], info[2], info[3], info[4],
                       info[5], info[6], info[7], info[9]);
                fflush(stdout);
                CHECK(hipEventDestroy(a));
                CHECK(hipEventDestroy(b));
            }
    CHECK(hipFree(x));
    CHECK(hipFree(out));
    CHECK(hipFree(didx));
    CHECK(hipFree(done));
    CHECK(hipFree(xg));
}

// Third question: what does the mix of the sparsest sweep layer (epsilon = 1: two random 512-byte row gathers per
// 512-byte output row written, i.e. a third of the traffic in writes) reach when nothing else is done?  Each group
// produces four consecutive output rows (as the span forward kernel does), each the sum of `fan` gathered rows.
__global__ __launch_bounds__(256) void gather_write(const float *x, const int *idx, long nrows_out, int fan, float *y)
{
    const long g = (long)blockIdx.x * 8 + threadIdx.x / 32;
    const int lane = threadIdx.x % 32;
    const long r0 = g * 4;
    if (r0 >= nrows_out) return;
    float4 v[8];
    const int *my = idx + r0 * fan;
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = u < 4 * fan ? *(const float4 *)(x + (long)my[u] * 128 + lane * 4) : make_float4(0, 0, 0, 0);
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        float4 a = v[r * fan];
        if (fan == 2) { a.x += v[r * 2 + 1].x; a.y += v[r * 2 + 1].y; a.z += v[r * 2 + 1].z; a.w += v[r * 2 + 1].w; }
        *(float4 *)(y + (r0 + r) * 128 + lane * 4) = a;
    }
}

static void run_gather_write()
{
    const long n = 262144;
    float *x, *y;
    int *didx;
    CHECK(hipMalloc(&x, n * 512));
    CHECK(hipMemset(x, 0, n * 512));
    CHECK(hipMalloc(&y, n * 512));
    CHECK(hipMalloc(&didx, n * 2 * 4));
    printf("# gather + write: %ld output rows of 512 bytes, each the sum of `fan` random rows of a 134 MB operand (fan = 2: the\n"
           "# traffic mix of the epsilon = 1, B = 128 forward pass)\n", n);
    for (int fan : {1, 2}) {
        std::vector<int> h((size_t)n * fan);
        std::mt19937 rng(3);
        for (auto &v : h) v = (int)(rng() % n);
        CHECK(hipMemcpy(didx, h.data(), h.size() * 4, hipMemcpyHostToDevice));
        hipEvent_t a, b;
        CHECK(hipEventCreate(&a));
        CHECK(hipEventCreate(&b));
        float best = 1e9f;
        for (int rep = 0; rep < 6; ++rep) {
            CHECK(hipEventRecord(a));
            hipLaunchKernelGGL(gather_write, dim3((unsigned)(n / 4 / 8)), dim3(256), 0, 0, x, didx, n, fan, y);
            CHECK(hipEventRecord(b));
            CHECK(hipEventSynchronize(b));
            float ms;
            CHECK(hipEventElapsedTime(&ms, a, b));
            if (rep > 0 && ms < best) best = ms;
        }
        const double bytes = (double)n * 512 * (fan + 1) + h.size() * 4.0;
        printf("fan %d: %.4f ms, %.0f MB moved, %.2f TB/s\n", fan, best, bytes / 1e6, bytes / best / 1e9);
        fflush(stdout);
        CHECK(hipEventDestroy(a));
        CHECK(hipEventDestroy(b));
    }
    CHECK(hipFree(x));
    CHECK(hipFree(y));
    CHECK(hipFree(didx));
}

int main()
{
    const long total = 8L << 30;   // 8 GiB gathered per launch
    run<32>({4096L, 8192L, 16384L, 65536L, 262144L, 1048576L, 4194304L}, total);
    run<8>({65536L, 262144L, 1048576L}, total / 4);
    run<4>({32768L, 65536L, 131072L}, total / 8);   // 64-byte rows: half a cache line
    run<64>({65536L, 262144L, 1048576L}, total);
    run_walk();
    run_walk_sync();
    run_gather_write();
    return 0;
}
