// hbm_probe: a small stand-alone program (no library dependency) that
//   (a) measures the HBM read rate a streaming kernel reaches on this GPU, with the default and
//       the non-temporal cache policy, in the access shape of the attention kernels, and
//   (b) streams the shared store tile by tile the way the LDS-staged attention kernels do, without
//       their arithmetic, with and without the partial rows they write, and
//   (c) runs a plain copy of known size (1 GiB read + 1 GiB written per launch), the reference
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

// The access shape of the LDS-staged shared-attention tiles without their arithmetic: one workgroup
// per tile streams 1 MiB of K and 1 MiB of V in stages of 16 KiB + 16 KiB through LDS (one stage of
// loads in flight, 64 KiB of LDS -> two workgroups per CU), then writes the tile's 32 partial rows of
// 512 B (row stride 9 x 512 B, 64-byte pieces as the kernels write them).  ST: 0 no stores,
// 1 write-back stores, 2 non-temporal stores.  Shows what the partial rows cost inside a saturated
// read stream.
template <int ST>
__global__ __launch_bounds__(256, 2) void tile_stream_kernel(const char* K, const char* V, int ntiles, size_t seg,
                                                             float* part, unsigned* out) {
  __shared__ u32x4 lds[4096];
  const unsigned tid = threadIdx.x;
  const int t = blockIdx.x;
  if (t >= ntiles) return;
  const size_t base = (size_t)((t * 1031) % ntiles) * seg;    // scattered tile order (1031 is coprime to the tile count)
  __amdgpu_buffer_rsrc_t rk = __builtin_amdgcn_make_buffer_rsrc((void*)(K + base), 0, (int)seg, 0x00020000);
  __amdgpu_buffer_rsrc_t rv = __builtin_amdgcn_make_buffer_rsrc((void*)(V + base), 0, (int)seg, 0x00020000);
  u32x4 acc = {0,0,0,0}, k[4], v[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) { k[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, tid * 16 + i * 4096, 0, 2); v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, tid * 16 + i * 4096, 0, 2); }
  for (unsigned off = 16384; off <= seg; off += 16384) {      // the last round's loads are past the end: dropped by the range check
#pragma unroll
    for (int i = 0; i < 4; ++i) { lds[tid + 256 * i] = k[i]; lds[1024 + tid + 256 * i] = v[i]; }
#pragma unroll
    for (int i = 0; i < 4; ++i) { k[i] = __builtin_amdgcn_raw_buffer_load_b128(rk, off + tid * 16 + i * 4096, 0, 2); v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv, off + tid * 16 + i * 4096, 0, 2); }
    __syncthreads();
    for (int s = 0; s < 16; ++s) acc ^= lds[(tid * 7 + s * 13) & 2047];
    __syncthreads();
  }
  if (ST) {
    const int lane = tid & 63, wave = tid >> 6, q = lane >> 4, x = lane & 15;
    if (wave < 2) {
      typedef __attribute__((ext_vector_type(4))) float f32x4;
      float* o = part + ((size_t)(t * 32 + wave * 16 + x) * 9) * 128 + 4 * q;
      const f32x4 val = {(float)acc[0], 1.f, 2.f, 3.f};
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (ST == 1) *(f32x4*)(o + 16 * e) = val; else __builtin_nontemporal_store(val, (f32x4*)(o + 16 * e));
      }
    }
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
  if (!copy_only) {
    // 2040 tiles of 1 MiB K + 1 MiB V (the shared store of 256 chunks x 8 KV heads) out of a and b
    const int ntiles = 2040; const size_t seg = (size_t)1 << 20;
    float* part; CK(hipMalloc(&part, (size_t)ntiles * 32 * 9 * 512));
    float ms;
    ms = timeit([&] { hipLaunchKernelGGL((tile_stream_kernel<0>), dim3(ntiles), dim3(256), 0, 0, a, b, ntiles, seg, part, out); }, 10);
    printf("tile streams, no partial rows written: %.3f ms %.1f GB/s\n", ms, 2.0 * ntiles * seg / ms / 1e6);
    ms = timeit([&] { hipLaunchKernelGGL((tile_stream_kernel<1>), dim3(ntiles), dim3(256), 0, 0, a, b, ntiles, seg, part, out); }, 10);
    printf("tile streams, 33 MB of partial rows, write-back stores: %.3f ms %.1f GB/s\n", ms, 2.0 * ntiles * seg / ms / 1e6);
    ms = timeit([&] { hipLaunchKernelGGL((tile_stream_kernel<2>), dim3(ntiles), dim3(256), 0, 0, a, b, ntiles, seg, part, out); }, 10);
    printf("tile streams, 33 MB of partial rows, non-temporal stores: %.3f ms %.1f GB/s\n", ms, 2.0 * ntiles * seg / ms / 1e6);
    CK(hipFree(part));
  }
  // plain copy of known size: 1 GiB read + 1 GiB written per launch (for counter calibration)
  size_t n = ((size_t)1 << 30) / 16;
  float ms = timeit([&] { hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, 0, (const uint4*)a, (uint4*)b, n); }, copy_only ? 3 : 10);
  printf("copy 1GiB: %.3f ms  read+write %.1f GB/s\n", ms, 2.0 * (1 << 30) / ms / 1e6);
  return 0;
}
