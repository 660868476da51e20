// Read-bandwidth probe: what a kernel that only reads can take in on this chip, by where the bytes come from (HBM,
// Infinity Cache, L2) and by how many waves and bytes in flight a CU has.  It is the yardstick the streaming and
// GEMM kernels of the library are held against (their rates are quoted against 8 TB/s nominal; this gives the rate a
// plain read loop reaches).  Built by paper_2211_00235_amd/build.py (build_mem_probe);  mem_probe  (no arguments).
// Every workgroup walks `reps` times over a window of `win` bytes that starts `stride` bytes after the previous
// workgroup's (stride 0: all workgroups read the same window), with U 16-byte loads in flight per lane, plain or
// non-temporal.  2 GiB are allocated; every case stays inside (checked on the host before the launch).
#include <hip/hip_runtime.h>
#include <stdio.h>
#include <stdlib.h>
typedef float f4 __attribute__((ext_vector_type(4)));
#define CK(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); exit(1); } } while (0)

template <int U, bool NT>
__global__ __launch_bounds__(1024) void read_kernel(const f4* p, size_t win_elems, int reps, size_t stride_elems, float* out) {
  const f4* base = p + (size_t)blockIdx.x * stride_elems;
  const size_t nthr = blockDim.x;
  f4 acc[U];
#pragma unroll
  for (int u = 0; u < U; u++) acc[u] = f4{0.0f, 0.0f, 0.0f, 0.0f};
  for (int r = 0; r < reps; r++)
    for (size_t i = threadIdx.x; i + (U - 1) * nthr < win_elems; i += U * nthr) {
#pragma unroll
      for (int u = 0; u < U; u++) {
        const f4 v = NT ? __builtin_nontemporal_load(base + i + u * nthr) : base[i + u * nthr];
        acc[u] += v;
      }
    }
  float s = 0.0f;
#pragma unroll
  for (int u = 0; u < U; u++) s += acc[u][0] + acc[u][1] + acc[u][2] + acc[u][3];
  if (s == 12345.678f) out[0] = s;   // never true for the zero-filled buffer: keeps the loads alive
}

struct Case { const char* name; int wgs, threads; size_t win, stride; int reps; };

int main() {
  const size_t total = (size_t)2 << 30;
  f4* buf; float* out;
  CK(hipMalloc(&buf, total)); CK(hipMalloc(&out, 4)); CK(hipMemset(buf, 0, total));
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  const size_t KiB = 1024, MiB = 1024 * 1024;
  const Case cases[] = {
    {"HBM, 2 GiB read once: 8192 wg x 256 thr", 8192, 256, 256 * KiB, 256 * KiB, 1},
    {"HBM, 2 GiB read once: 2048 wg x 256 thr", 2048, 256, 1 * MiB, 1 * MiB, 1},
    {"HBM, 1.75 GiB read once: 1024 wg x 256 thr", 1024, 256, 1792 * KiB, 2 * MiB, 1},
    {"HBM, 1.75 GiB read once: 512 wg x 256 thr (2 wg per CU)", 512, 256, 3584 * KiB, 4 * MiB, 1},
    {"HBM, 1.75 GiB read once: 256 wg x 256 thr (4 waves per CU)", 256, 256, 7 * MiB, 8 * MiB, 1},
    {"HBM, 1.75 GiB read once: 256 wg x 256 thr, odd stride", 256, 256, 7 * MiB, 7 * MiB + 37 * KiB, 1},
    {"HBM, 1.75 GiB read once: 256 wg x 512 thr (8 waves per CU)", 256, 512, 7 * MiB, 8 * MiB, 1},
    {"HBM, 1.75 GiB read once: 256 wg x 1024 thr (16 waves per CU)", 256, 1024, 7 * MiB, 8 * MiB, 1},
    {"Infinity Cache: 2048 private 64 KiB windows x 256", 2048, 256, 64 * KiB, 64 * KiB, 256},
    {"L2: one 1 MiB window shared by 2048 wg x 64", 2048, 256, 1 * MiB, 0, 64},
    {"L2: one 1 MiB window shared by 256 wg x 64 (4 waves per CU)", 256, 256, 1 * MiB, 0, 64},
    {"L2: one 16 MiB window shared by 2048 wg x 4", 2048, 256, 16 * MiB, 0, 4},
  };
  printf("%-62s %-8s %10s %9s %12s\n", "case", "loads", "us", "TB/s", "GB/s per CU");
  for (const Case& c : cases) {
    if ((size_t)(c.wgs - 1) * c.stride + c.win > total) { printf("case out of bounds: %s\n", c.name); return 1; }
    for (int variant = 0; variant < 4; variant++) {
      const int U = variant < 2 ? 4 : 8;
      const bool nt = variant & 1;
      const size_t we = c.win / 16, se = c.stride / 16;
      auto launch = [&]() {
        if (U == 4 && !nt) hipLaunchKernelGGL((read_kernel<4, false>), dim3(c.wgs), dim3(c.threads), 0, 0, buf, we, c.reps, se, out);
        if (U == 4 && nt) hipLaunchKernelGGL((read_kernel<4, true>), dim3(c.wgs), dim3(c.threads), 0, 0, buf, we, c.reps, se, out);
        if (U == 8 && !nt) hipLaunchKernelGGL((read_kernel<8, false>), dim3(c.wgs), dim3(c.threads), 0, 0, buf, we, c.reps, se, out);
        if (U == 8 && nt) hipLaunchKernelGGL((read_kernel<8, true>), dim3(c.wgs), dim3(c.threads), 0, 0, buf, we, c.reps, se, out);
      };
      launch();
      CK(hipDeviceSynchronize());
      CK(hipEventRecord(e0));
      for (int i = 0; i < 5; i++) launch();
      CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
      CK(hipGetLastError());
      float ms; CK(hipEventElapsedTime(&ms, e0, e1)); ms /= 5;
      const double bytes = (double)c.wgs * c.win * c.reps;
      printf("%-62s U=%d %-3s %10.1f %9.2f %12.1f\n", c.name, U, nt ? "nt" : "", ms * 1e3, bytes / ms / 1e9, bytes / ms / 1e6 / 256);
      fflush(stdout);
    }
  }
  return 0;
}
