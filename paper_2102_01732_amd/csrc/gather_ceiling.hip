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

int main()
{
    const long total = 8L << 30;   // 8 GiB gathered per launch
    run<32>({4096L, 8192L, 16384L, 65536L, 262144L, 1048576L, 4194304L}, total);
    run<8>({65536L, 262144L, 1048576L}, total / 4);
    run<64>({65536L, 262144L, 1048576L}, total);
    return 0;
}
