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
    run<64>({65536L, 262144L, 1048576L}, total);
    run_walk();
    run_gather_write();
    return 0;
}
