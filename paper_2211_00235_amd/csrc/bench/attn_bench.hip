// Stand-alone timing of the attention kernels (pe_attn.h) on random data: every kernel alone on the chip, 20 launches
// after 3 warm-up launches, HIP events on the null stream.  Built by paper_2211_00235_amd/build.py (build_attn_bench);
//   attn_bench [B L H d [masked_tail]]      default 256 256 4 32 0: the triangle attention of s=128, r=256
// (128 256 8 32 is that workload's row attention).  Prints microseconds per launch and the rates of the algorithmic
// bytes and flops.  Used under rocprofv3 --pmc for the counters of the kernels alone.
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#include <vector>
#include "../pe_attn.h"
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)
template <typename F> static float timeit(const char* name, int reps, double bytes, double flops, F f) {
  hipEvent_t a, b; CK(hipEventCreate(&a)); CK(hipEventCreate(&b));
  for (int i = 0; i < 3; i++) f();
  CK(hipDeviceSynchronize());
  CK(hipEventRecord(a));
  for (int i = 0; i < reps; i++) f();
  CK(hipEventRecord(b)); CK(hipEventSynchronize(b));
  float ms; CK(hipEventElapsedTime(&ms, a, b));
  CK(hipGetLastError());
  printf("%-28s %8.2f us  %7.1f GB/s  %7.1f TFLOP/s\n", name, 1e3 * ms / reps, bytes / (ms / reps * 1e6), flops / (ms / reps * 1e9));
  fflush(stdout);
  return ms / reps;
}
int main(int argc, char** argv) {
  const int B = argc > 1 ? atoi(argv[1]) : 256, L = argc > 2 ? atoi(argv[2]) : 256, H = argc > 3 ? atoi(argv[3]) : 4, d = argc > 4 ? atoi(argv[4]) : 32;
  const int nmask = argc > 5 ? atoi(argv[5]) : 0;   // trailing masked keys
  const int reps = 20;
  typedef bf16 T;
  const long long M = (long long)B * L, plane = M * d;
  const long long nt = (L + 31) / 32, bplane = nt * L * 32;
  std::vector<T> hq(4 * H * plane), hb(H * bplane), hdog(H * plane);
  srand(1);
  auto rnd = []() { return (float)rand() / RAND_MAX * 2.0f - 1.0f; };
  for (auto& v : hq) v = (T)rnd();
  for (auto& v : hb) v = (T)rnd();
  for (auto& v : hdog) v = (T)rnd();
  std::vector<float> hm((size_t)B * L, 1.0f);
  for (int b = 0; b < B; b++) for (int j = L - nmask; j < L; j++) hm[(size_t)b * L + j] = 0.0f;
  T *qkvg, *biasQ, *biasK, *o, *og, *dog, *dO, *dqkvg, *dS; float *mask, *lse, *D;
  CK(hipMalloc(&qkvg, hq.size() * 2)); CK(hipMalloc(&biasQ, hb.size() * 2)); CK(hipMalloc(&biasK, hb.size() * 2));
  CK(hipMalloc(&o, H * plane * 2)); CK(hipMalloc(&og, H * plane * 2)); CK(hipMalloc(&dog, H * plane * 2)); CK(hipMalloc(&dO, H * plane * 2));
  CK(hipMalloc(&dqkvg, 4 * H * plane * 2)); CK(hipMalloc(&dS, (size_t)((B + 1) / 2) * H * bplane * 2));
  CK(hipMalloc(&mask, hm.size() * 4)); CK(hipMalloc(&lse, (size_t)B * H * L * 4)); CK(hipMalloc(&D, (size_t)B * H * L * 4));
  CK(hipMemcpy(qkvg, hq.data(), hq.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(biasQ, hb.data(), hb.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(biasK, hb.data(), hb.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(dog, hdog.data(), hdog.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(dO, hdog.data(), hdog.size() * 2, hipMemcpyHostToDevice));
  CK(hipMemcpy(mask, hm.data(), hm.size() * 4, hipMemcpyHostToDevice));
  CK(hipMemset(D, 0, (size_t)B * H * L * 4));
  AttnArgs a; memset(&a, 0, sizeof(a));
  a.qkvg = qkvg; a.plane = plane; a.B = B; a.L = L; a.H = H; a.d = d; a.biasQ = biasQ; a.biasK = biasK;
  a.mask = mask; a.mask_bs = L; a.mask_ks = 1; a.o = o; a.og = og; a.lse = lse; a.scale = 1.0f / sqrtf((float)d);
  a.dog = dog; a.dO = dO; a.D = D; a.dqkvg = dqkvg; a.dS = dS;
  const dim3 grid(attn_grid_size(B, H, L));
  const double e = 2.0;
  const double ll = (double)B * H * L * L;
  printf("B %d L %d H %d d %d masked tail %d\n", B, L, H, d, nmask);
  timeit("attn_fwd<bias>", reps, 6.0 * H * plane * e, 4.0 * ll * d, [&] { hipLaunchKernelGGL((attn_fwd_kernel<T, true>), grid, dim3(256), 0, 0, a); });
  timeit("attn_fwd<nobias>", reps, 6.0 * H * plane * e, 4.0 * ll * d, [&] { hipLaunchKernelGGL((attn_fwd_kernel<T, false>), grid, dim3(256), 0, 0, a); });
  timeit("attn_bwd_dq2", reps, 5.0 * H * plane * e + ll, 6.0 * ll * d, [&] { hipLaunchKernelGGL((attn_bwd_dq2_kernel<T>), dim3(attn_grid_size((B + 1) / 2, H, L)), dim3(512), 0, 0, a); });
  AttnArgs a0 = a; a0.dS = nullptr;   // the unbiased kernel would write one dS plane per batch row: the buffer holds half of them
  timeit("attn_bwd_dq<nobias>", reps, 5.0 * H * plane * e, 6.0 * ll * d, [&] { hipLaunchKernelGGL((attn_bwd_dq_kernel<T, false>), grid, dim3(256), 0, 0, a0); });
  timeit("attn_bwd_dkv<bias>", reps, 6.0 * H * plane * e, 8.0 * ll * d, [&] { hipLaunchKernelGGL((attn_bwd_dkv_kernel<T, true>), grid, dim3(256), 0, 0, a); });
  timeit("attn_bwd_dkv<nobias>", reps, 6.0 * H * plane * e, 8.0 * ll * d, [&] { hipLaunchKernelGGL((attn_bwd_dkv_kernel<T, false>), grid, dim3(256), 0, 0, a); });
  return 0;
}
