// Stand-alone microbenchmark (not part of libsparse_set.so): the rate at which one MI355X can gather
// random 512-byte rows (one stored connection at B = 128) as a function of the size of the operand
// they come from.  It gives the ceiling the sparse kernels are measured against: ~26 TB/s while the
// operand fits the 4 MB L2 of an XCD, ~8.5 TB/s at 32 MB, ~7.5 TB/s at 512 MB (L2 miss path).
//   hipcc --offload-arch=gfx950 -O3 paper_2102_01732_amd/csrc/gather_ceiling.hip -o gather_ceiling && ./gather_ceiling
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
#include <random>
// each group of 32 lanes gathers `per` rows of 512 B (float4 per lane), 8 in flight
__global__ __launch_bounds__(256) void gather(const float* x, const int* idx, long ngroups, int per, float* out) {
  long g = (long)blockIdx.x * 8 + threadIdx.x / 32; int lane = threadIdx.x % 32;
  if (g >= ngroups) return;
  const int* my = idx + g * per;
  float4 acc = make_float4(0,0,0,0);
  for (int p = 0; p < per; p += 8) {
    int c[8]; float4 v[8];
    #pragma unroll
    for (int u = 0; u < 8; ++u) c[u] = my[p + u];
    #pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = *(const float4*)(x + (long)c[u] * 128 + lane * 4);
    #pragma unroll
    for (int u = 0; u < 8; ++u) { acc.x += v[u].x; acc.y += v[u].y; acc.z += v[u].z; acc.w += v[u].w; }
  }
  if (acc.x == 12345.f) out[g] = acc.y + acc.z + acc.w;
}
int main() {
  const long ngroups = 1 << 20; const int per = 16;   // 16.7M gathers = 8.6 GB
  std::vector<int> h(ngroups * per);
  float* out; (void)hipMalloc(&out, ngroups * 4);
  int* didx; (void)hipMalloc(&didx, h.size() * 4);
  for (long rows : {4096L, 8192L, 16384L, 65536L, 262144L, 1048576L, 4194304L}) {
    std::mt19937 rng(1); for (auto& v : h) v = rng() % rows;
    (void)hipMemcpy(didx, h.data(), h.size() * 4, hipMemcpyHostToDevice);
    float* x; (void)hipMalloc(&x, rows * 512); (void)hipMemset(x, 0, rows * 512);
    hipEvent_t a, b; (void)hipEventCreate(&a); (void)hipEventCreate(&b);
    for (int rep = 0; rep < 2; ++rep) {
      (void)hipEventRecord(a);
      for (int i = 0; i < 5; ++i) hipLaunchKernelGGL(gather, dim3(ngroups / 8), dim3(256), 0, 0, x, didx, ngroups, per, out);
      (void)hipEventRecord(b); (void)hipEventSynchronize(b);
    }
    float ms; (void)hipEventElapsedTime(&ms, a, b); ms /= 5;
    printf("operand %7.1f MB: %.3f ms, %.2f TB/s gathered (+%.2f GB index stream)\n", rows * 512 / 1e6, ms, ngroups * per * 512.0 / ms / 1e9, h.size() * 4 / 1e9);
    (void)hipFree(x);
  }
}
