// hbm_probe: a small stand-alone program (no library dependency) that
//   (a) measures the HBM read rate a streaming kernel reaches on this GPU, with the default and
//       the non-temporal cache policy, in the access shape of the attention kernels, and
//   (b) runs a plain copy of known size (1 GiB read + 1 GiB written per launch), the reference
//       against which the profiler's FETCH_SIZE / WRITE_SIZE counters are scaled.
// Usage: hbm_probe        all measurements
//        hbm_probe 1      the copy kernel only (for counter calibration runs)
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
#define CK(x) do { hipError_t e = (x); if (e != hipSuccess) { printf("HIP error %s at %d\n", hipGetErrorString(e), __LINE__); exit(1);} } while (0)
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

// each workgroup streams a contiguous segment of `seg` bytes; wave w takes 16 KB blocks w, w+NW, ...
template <int UNROLL, int AUX>
__global__ __launch_bounds__(256) void read_kernel(const char* base, size_t seg, unsigned* out) {
  const char* p = base + (size_t)blockIdx.x * seg;
  __amdgpu_buffer_rsrc_t r = __builtin_amdgcn_make_buffer_rsrc((void*)p, 0, (int)seg, 0x00020000);
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  u32x4 acc = {0,0,0,0};
  const unsigned blk = 1024u * UNROLL;     // bytes per wave per iteration
  for (unsigned off = wave * blk; off < seg; off += 4 * blk) {
    u32x4 v[UNROLL];
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(r, off + i * 1024 + lane * 16, 0, AUX);
#pragma unroll
    for (int i = 0; i < UNROLL; ++i) acc ^= v[i];
  }
  if ((acc[0] ^ acc[1] ^ acc[2] ^ acc[3]) == 0x12345678u) out[0] = 1;
}

__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ a, uint4* __restrict__ b, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) b[i] = a[i];
}

template <typename F> float timeit(F f, int reps) {
  hipEvent_t e0, e1; CK(hipEventCreate(&e0)); CK(hipEventCreate(&e1));
  f(); CK(hipDeviceSynchronize());
  CK(hipEventRecord(e0)); for (int i = 0; i < reps; ++i) f(); CK(hipEventRecord(e1)); CK(hipEventSynchronize(e1));
  float ms; CK(hipEventElapsedTime(&ms, e0, e1)); return ms / reps;
}

int main(int argc, char** argv) {
  const size_t bytes = (size_t)4 << 30;
  char* a; unsigned* out; char* b;
  CK(hipMalloc(&a, bytes)); CK(hipMalloc(&b, bytes)); CK(hipMalloc(&out, 4));
  CK(hipMemset(a, 1, bytes)); CK(hipMemset(b, 0, bytes));
  hipDeviceProp_t prop; CK(hipGetDeviceProperties(&prop, 0));
  printf("device %s CUs %d clock %d kHz memclock %d kHz bus %d bits L2 %d\n", prop.name, prop.multiProcessorCount, prop.clockRate, prop.memoryClockRate, prop.memoryBusWidth, prop.l2CacheSize);
  const bool copy_only = argc > 1 && atoi(argv[1]) == 1;
  if (!copy_only) {
    for (size_t seg : {(size_t)1 << 20, (size_t)2 << 20, (size_t)4 << 20}) {
      unsigned grid = bytes / seg;
      float ms;
      ms = timeit([&] { hipLaunchKernelGGL((read_kernel<8, 0>), dim3(grid), dim3(256), 0, 0, a, seg, out); }, 10);
      printf("read seg %zu KB unroll 8 aux0: %.3f ms %.1f GB/s\n", seg >> 10, ms, bytes / ms / 1e6);
      ms = timeit([&] { hipLaunchKernelGGL((read_kernel<16, 0>), dim3(grid), dim3(256), 0, 0, a, seg, out); }, 10);
      printf("read seg %zu KB unroll 16 aux0: %.3f ms %.1f GB/s\n", seg >> 10, ms, bytes / ms / 1e6);
      ms = timeit([&] { hipLaunchKernelGGL((read_kernel<16, 2>), dim3(grid), dim3(256), 0, 0, a, seg, out); }, 10);
      printf("read seg %zu KB unroll 16 aux2(nt): %.3f ms %.1f GB/s\n", seg >> 10, ms, bytes / ms / 1e6);
      ms = timeit([&] { hipLaunchKernelGGL((read_kernel<4, 0>), dim3(grid), dim3(256), 0, 0, a, seg, out); }, 10);
      printf("read seg %zu KB unroll 4 aux0: %.3f ms %.1f GB/s\n", seg >> 10, ms, bytes / ms / 1e6);
    }
  }
  // plain copy of known size: 1 GiB read + 1 GiB written per launch (for counter calibration)
  size_t n = ((size_t)1 << 30) / 16;
  float ms = timeit([&] { hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, 0, (const uint4*)a, (uint4*)b, n); }, copy_only ? 3 : 10);
  printf("copy 1GiB: %.3f ms  read+write %.1f GB/s\n", ms, 2.0 * (1 << 30) / ms / 1e6);
  return 0;
}
