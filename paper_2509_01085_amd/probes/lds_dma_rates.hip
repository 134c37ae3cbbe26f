// Probe, not part of the library: data-movement rates of one CU on gfx950.
//   1. L2 / Infinity Cache -> LDS streaming of 32 KB tiles: global_load_lds_dwordx4 (DMA, no registers)
//      against global_load_dwordx4 + ds_write_b128, from a window that fits every XCD's L2 (2 MB) and
//      from one that only the Infinity Cache holds (64 MB).  One tile at a time per workgroup.
//   2. LDS read rate with every wavefront of the CU reading: ds_read_b128 against ds_read_b64_tr_b16
//      with the attention kernels' swizzled, conflict-free transposed-fragment addressing.
//   hipcc --offload-arch=gfx950 -O3 -o /tmp/lds_dma_rates lds_dma_rates.hip && /tmp/lds_dma_rates
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((address_space(3))) void* lds_ptr_t;

__device__ inline void dma16_raw(uint64_t sbase, uint32_t lane_offset, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" : : "v"(lane_offset), "s"(sbase), "s"(lds_addr) : "memory", "m0");
}

// each workgroup (NW wavefronts) copies `tiles` tiles of 32 KB from a window of `window` bytes into a ring of two LDS slots
template <int MODE, int NW>
__global__ __launch_bounds__(NW * 64) void stream_kernel(const uint8_t* src, size_t window, int tiles, uint32_t* out) {
  extern __shared__ __align__(16) uint8_t smem[];
  const int tid = threadIdx.x, wave = tid >> 6;
  constexpr int PER = 32768 / (NW * 64 * 16);  // 16-byte chunks per thread per tile
  const uint32_t lds_base = (uint32_t)(uintptr_t)(lds_ptr_t)smem;
  uint32_t acc = 0;
  size_t off = ((size_t)blockIdx.x * 32768 * 7) % window;
  for (int t = 0; t < tiles; ++t) {
    const uint8_t* p = src + off;
    off += 32768;
    if (off >= window) off = 0;
    const uint32_t slot = (t & 1) * 32768;
    if (MODE == 0) {
      const uint64_t sb = (uint64_t)(uintptr_t)p;
      const uint64_t sbu = ((uint64_t)(uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)(sb >> 32)) << 32) |
                           (uint32_t)__builtin_amdgcn_readfirstlane((uint32_t)sb);
#pragma unroll
      for (int n = 0; n < PER; ++n)
        dma16_raw(sbu, (uint32_t)(tid * 16 + n * NW * 1024), __builtin_amdgcn_readfirstlane(lds_base + slot + wave * 1024 + n * NW * 1024));
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    } else {
      u32x4 v[PER];
#pragma unroll
      for (int n = 0; n < PER; ++n) v[n] = *reinterpret_cast<const u32x4*>(p + tid * 16 + n * NW * 1024);
#pragma unroll
      for (int n = 0; n < PER; ++n) *reinterpret_cast<u32x4*>(smem + slot + tid * 16 + n * NW * 1024) = v[n];
    }
    __syncthreads();
    acc += reinterpret_cast<uint32_t*>(smem + slot)[(tid * 37 + t) & 8191];
  }
  out[blockIdx.x * blockDim.x + tid] = acc;
}

template <int MODE, int NW>
static void stream(const char* name, const uint8_t* src, size_t window, uint32_t* out, int wgs) {
  const int tiles = 2000;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(stream_kernel<MODE, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
  hipLaunchKernelGGL((stream_kernel<MODE, NW>), dim3(wgs), dim3(NW * 64), 65536, 0, src, window, 10, out);
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL((stream_kernel<MODE, NW>), dim3(wgs), dim3(NW * 64), 65536, 0, src, window, tiles, out);
  (void)hipEventRecord(e1);
  (void)hipEventSynchronize(e1);
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  const double bytes = (double)wgs * tiles * 32768;
  printf("%-52s %8.3f ms  %6.2f TB/s  %5.1f B/clk/CU\n", name, ms, bytes / ms * 1e-9, bytes / (ms * 1e-3 * 2.4e9) / 256);
}

template <int MODE, int NW>
__global__ __launch_bounds__(NW * 64) void lds_kernel(float* out, int iters) {
  extern __shared__ __align__(16) uint8_t smem[];  // 64 KB
  for (int i = threadIdx.x; i < 16384; i += NW * 64) reinterpret_cast<float*>(smem)[i] = i;
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned base = (unsigned)(uintptr_t)(lds_ptr_t)smem;
  const unsigned ab = base + wave * 2048 + lane * 16;  // b128: 64 lanes x 16 contiguous bytes
  // transposed fragments of a 64-row tile of 256-byte rows whose 16-byte chunks are swizzled (chunk c of row r at c ^ swz(r))
  const int grp = lane >> 5, L16 = lane & 15, q16 = lane >> 4, rsub = L16 >> 2, jj = L16 & 3, cl = 2 * (q16 & 1) + (jj >> 1);
  auto voff = [&](int h, int dt) { return (8 * h + 4 * grp + rsub) * 256 + ((((dt ^ rsub) << 2) | (cl ^ (2 * h + grp))) << 4) + 8 * (jj & 1); };
  const unsigned at = base + (wave & 3) * 16384;
  const unsigned t0 = at + voff(0, 0), t1 = at + voff(1, 0), t2 = at + voff(0, 1), t3 = at + voff(1, 1), t4 = at + voff(0, 2),
                 t5 = at + voff(1, 2), t6 = at + voff(0, 3), t7 = at + voff(1, 3);
  f32x4 q0 = {0, 0, 0, 0}, q1 = q0, q2 = q0, q3 = q0;
  float s = 0;
  for (int it = 0; it < iters; ++it) {
    if (MODE == 0)
      asm volatile("ds_read_b128 %0, %4\n ds_read_b128 %1, %4 offset:4096\n ds_read_b128 %2, %4 offset:8192\n ds_read_b128 %3, %4 offset:12288\n"
                   "ds_read_b128 %0, %4 offset:16384\n ds_read_b128 %1, %4 offset:20480\n ds_read_b128 %2, %4 offset:24576\n ds_read_b128 %3, %4 offset:28672\n s_waitcnt lgkmcnt(0)"
                   : "+v"(q0), "+v"(q1), "+v"(q2), "+v"(q3) : "v"(ab) : "memory");
    else
      asm volatile("ds_read_b64_tr_b16 %0, %4\n ds_read_b64_tr_b16 %1, %5\n ds_read_b64_tr_b16 %2, %6\n ds_read_b64_tr_b16 %3, %7\n"
                   "ds_read_b64_tr_b16 %0, %8 offset:4096\n ds_read_b64_tr_b16 %1, %9 offset:4096\n ds_read_b64_tr_b16 %2, %10 offset:4096\n ds_read_b64_tr_b16 %3, %11 offset:4096\n s_waitcnt lgkmcnt(0)"
                   : "+v"(*(double*)&q0), "+v"(*(double*)&q1), "+v"(*(double*)&q2), "+v"(*(double*)&q3)
                   : "v"(t0), "v"(t1), "v"(t2), "v"(t3), "v"(t4), "v"(t5), "v"(t6), "v"(t7) : "memory");
    s += q0[0];
  }
  out[blockIdx.x * blockDim.x + threadIdx.x] = s + q1[0] + q2[1] + q3[0];
}

template <int MODE, int NW>
static void lds(const char* name, float* d) {
  const int iters = 20000;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  (void)hipFuncSetAttribute(reinterpret_cast<const void*>(lds_kernel<MODE, NW>), hipFuncAttributeMaxDynamicSharedMemorySize, 65536);
  hipLaunchKernelGGL((lds_kernel<MODE, NW>), dim3(256), dim3(NW * 64), 65536, 0, d, 100);
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL((lds_kernel<MODE, NW>), dim3(256), dim3(NW * 64), 65536, 0, d, iters);
  (void)hipEventRecord(e1);
  (void)hipEventSynchronize(e1);
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  const double cyc = ms * 1e-3 * 2.4e9 / iters / 8;  // per instruction per wavefront
  printf("%-52s %8.3f ms  %6.1f cycles per instruction per wavefront  %6.1f B/clk/CU\n", name, ms, cyc, (MODE == 0 ? 1024.0 : 512.0) * NW / cyc);
}

int main() {
  const size_t big = 64u << 20, small = 2u << 20;
  uint8_t* src;
  uint32_t* out;
  if (hipMalloc(&src, big) != hipSuccess || hipMalloc(&out, 1024 * 512 * 4) != hipSuccess) return 1;
  (void)hipMemset(src, 1, big);
  stream<0, 4>("DMA  4 wavefronts, 1 workgroup/CU, 2 MB window", src, small, out, 256);
  stream<1, 4>("regs 4 wavefronts, 1 workgroup/CU, 2 MB window", src, small, out, 256);
  stream<0, 4>("DMA  4 wavefronts, 2 workgroups/CU, 2 MB window", src, small, out, 512);
  stream<1, 4>("regs 4 wavefronts, 2 workgroups/CU, 2 MB window", src, small, out, 512);
  stream<0, 8>("DMA  8 wavefronts, 2 workgroups/CU, 2 MB window", src, small, out, 512);
  stream<0, 4>("DMA  4 wavefronts, 2 workgroups/CU, 64 MB window", src, big, out, 512);
  stream<1, 4>("regs 4 wavefronts, 2 workgroups/CU, 64 MB window", src, big, out, 512);
  float* d = reinterpret_cast<float*>(out);
  lds<0, 4>("ds_read_b128        4 wavefronts/CU", d);
  lds<1, 4>("ds_read_b64_tr_b16  4 wavefronts/CU", d);
  lds<0, 8>("ds_read_b128        8 wavefronts/CU", d);
  lds<1, 8>("ds_read_b64_tr_b16  8 wavefronts/CU", d);
  lds<0, 16>("ds_read_b128       16 wavefronts/CU", d);
  lds<1, 16>("ds_read_b64_tr_b16 16 wavefronts/CU", d);
  printf("status %s\n", hipGetErrorString(hipDeviceSynchronize()));
  return 0;
}
