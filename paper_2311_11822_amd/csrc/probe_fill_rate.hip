// Stand-alone probe (not part of the library): how fast can the compute units pull data from L2, the
// memory-side cache and HBM with buffer_load ... lds (16 B per lane, the load the large-tile kernels
// use) and with plain buffer loads to registers?  One or two 256-thread workgroups per compute unit,
// every access inside the buffer (descriptors sized to each workgroup's window).
// Build and run:  python -m paper_2311_11822_amd.profiling fill-rate
#include <hip/hip_runtime.h>
#include <cstdio>
#include <cstdlib>
#include <vector>
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

__device__ __forceinline__ i32x4 make_rsrc(const void* base, unsigned bytes) {
  const uint64_t p = reinterpret_cast<uint64_t>(base);
  i32x4 r; r[0] = (int)(uint32_t)p; r[1] = (int)(uint32_t)(p >> 32) & 0xFFFF; r[2] = (int)bytes; r[3] = 0x00020000; return r;
}
__device__ __forceinline__ void load_to_lds(i32x4 rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds" : : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// Each workgroup streams over its own window of `window` bytes (starting at blockIdx * stride), iters times.
// ROWS: bytes contiguous per row segment per lane-group: lanes read 16 B each; 8 lanes cover 128 B of a row;
// consecutive 8-lane groups read rows `pitch` bytes apart (like the ghost kernel, pitch = row width), or contiguous.
__global__ void __launch_bounds__(256) k_dma(const char* src, size_t stride, unsigned window, unsigned pitch, int iters, int* out) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[];
  const unsigned lds0 = (unsigned)(uintptr_t)lds_raw;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  i32x4 rs = make_rsrc(src + blockIdx.x * stride, window);
  // lane's offset inside a 1 KB wave-load: pitch == 0 -> 1 KB contiguous; else 8 rows x 128 B
  const unsigned lane_off = pitch ? (unsigned)(lane >> 3) * pitch + (lane & 7) * 16 : lane * 16;
  const unsigned per_wave = pitch ? 8 * pitch : 1024;
  unsigned off = wave * per_wave;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      load_to_lds(rs, lane_off, off, lds0 + (wave * 8 + j) * 1024);
      off += 4 * per_wave;
      if (off + per_wave > window) off = wave * per_wave;
    }
    asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  if (threadIdx.x == 0) out[blockIdx.x] = lds_raw[5];
}
__global__ void __launch_bounds__(256) k_reg(const char* src, size_t stride, unsigned window, unsigned pitch, int iters, int* out) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc((void*)(src + blockIdx.x * stride), 0, (int)window, 0x00020000);
  const unsigned lane_off = pitch ? (unsigned)(lane >> 3) * pitch + (lane & 7) * 16 : lane * 16;
  const unsigned per_wave = pitch ? 8 * pitch : 1024;
  unsigned off = wave * per_wave;
  u32x4 acc = {0, 0, 0, 0};
  for (int it = 0; it < iters; ++it) {
    u32x4 v[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      v[j] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rs, lane_off, off, 0));
      off += 4 * per_wave;
      if (off + per_wave > window) off = wave * per_wave;
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc ^= v[j];
  }
  out[blockIdx.x * 256 + threadIdx.x] = acc[0] ^ acc[1] ^ acc[2] ^ acc[3];
}

int main() {
  const size_t total = (size_t)4 << 30;
  char* src; int* out;
  hipMalloc(&src, total); hipMalloc(&out, 1 << 20);
  hipMemset(src, 1, total);
  hipFuncSetAttribute((const void*)k_dma, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
  hipEvent_t e0, e1; hipEventCreate(&e0); hipEventCreate(&e1);
  struct Case { const char* name; size_t stride; unsigned window; unsigned pitch; int grid; int lds; };
  std::vector<Case> cases = {
    {"L2-hot, all CUs same 256 KB, contiguous", 0, 256 << 10, 0, 256, 160 << 10},
    {"L2-hot, own 64 KB per CU, contiguous", 64 << 10, 64 << 10, 0, 256, 160 << 10},
    {"own 1 MB per CU (256 MB total: memory-side cache), contiguous", 1 << 20, 1 << 20, 0, 256, 160 << 10},
    {"own 16 MB per CU (4 GB total: HBM), contiguous", (size_t)16 << 20, 16u << 20, 0, 256, 160 << 10},
    {"own 16 MB per CU (HBM), rows of 128 B, pitch 24576 B", (size_t)16 << 20, 16u << 20, 24576, 256, 160 << 10},
    {"L2-hot same 1 MB, rows of 128 B pitch 4096", 0, 1 << 20, 4096, 256, 160 << 10},
    {"L2-hot same 256 KB, contiguous, 2 WG per CU (64 KB LDS)", 0, 256 << 10, 0, 512, 64 << 10},
    {"HBM own 8 MB, contiguous, 2 WG per CU", (size_t)8 << 20, 8u << 20, 0, 512, 64 << 10},
  };
  for (auto& c : cases) {
    for (int mode = 0; mode < 2; ++mode) {
      const int iters = 2000;
      auto launch = [&]() {
        if (mode == 0) hipLaunchKernelGGL(k_dma, dim3(c.grid), dim3(256), c.lds, 0, src, c.stride, c.window, c.pitch, iters, out);
        else hipLaunchKernelGGL(k_reg, dim3(c.grid), dim3(256), 0, 0, src, c.stride, c.window, c.pitch, iters, out);
      };
      launch(); hipDeviceSynchronize();
      hipEventRecord(e0); launch(); hipEventRecord(e1); hipEventSynchronize(e1);
      float ms; hipEventElapsedTime(&ms, e0, e1);
      const double bytes = (double)c.grid * iters * 8 * 4 * 1024;
      printf("%-70s %s: %.3f ms  %.1f TB/s aggregate, %.1f GB/s per CU\n", c.name, mode == 0 ? "to LDS " : "to regs", ms, bytes / ms / 1e9, bytes / ms / 1e6 / 256);
      fflush(stdout);
    }
  }
  printf("status %d\n", (int)hipGetLastError());
  return 0;
}
