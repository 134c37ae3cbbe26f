// Probe, not part of the library: do matrix-core (MFMA) and vector-ALU instructions co-execute on
// gfx950, within one wavefront and across two wavefronts of a SIMD, and at what issue rates?
// Every loop body is one inline-asm block, so the instruction order is exactly what is written.
// One workgroup per CU; 256 threads = one wavefront per SIMD, 512 = two (wavefronts 0-3 run the
// first body, 4-7 the second), 768 and 1024 = three and four.  Times are converted to cycles at 2.4 GHz.
//   hipcc --offload-arch=gfx950 -O3 -o /tmp/mfma_valu_coexec mfma_valu_coexec.hip && /tmp/mfma_valu_coexec
#include <hip/hip_runtime.h>

#include <cstdint>
#include <cstdio>
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
#define MF(c) "v_mfma_f32_32x32x16_bf16 %" #c ", %12, %13, %" #c "\n"
#define FMA(i) "v_fma_f32 %" #i ", %" #i ", %14, %15\n"
#define FMAC(i) "v_fmac_f32 %" #i ", %14, %15\n"
#define ADD(i) "v_add_f32 %" #i ", %" #i ", %14\n"
#define MAX3(i, j) "v_max3_f32 %" #i ", %" #i ", %" #j ", %14\n"
#define EXP(i) "v_exp_f32 %" #i ", %" #i "\n"
#define CVT(i, j) "v_cvt_pk_bf16_f32 %" #i ", %" #i ", %" #j "\n"
#define DSR(q) "ds_read_b128 %" #q ", %16\n"
#define DSR2(q) "ds_read_b128 %" #q ", %16 offset:4096\n"
#define WAITL "s_waitcnt lgkmcnt(0)\n"
// operands: 0-3 accumulators c0..c3; 4-9 v0..v5; 10,11 q0,q1 (LDS destinations); 12,13 a,b; 14,15 k1,k2; 16 LDS address
#define OPS                                                                                                  \
  : "+v"(c0), "+v"(c1), "+v"(c2), "+v"(c3), "+v"(v0), "+v"(v1), "+v"(v2), "+v"(v3), "+v"(v4), "+v"(v5), "+v"(q0), "+v"(q1) \
  : "v"(a), "v"(b), "v"(k1), "v"(k2), "v"(laddr)
#define BODY(txt) asm volatile(txt OPS : "memory")
#define X8(M) M(4) M(5) M(6) M(7) M(8) M(9) M(4) M(5)
#define X4a(M) M(4) M(5) M(6) M(7)
#define X4b(M) M(8) M(9) M(4) M(5)
// softmax-like mix for two score registers: 1 max3, 2 fmac, 2 exp, 2 add, 1 convert = 8 instructions
#define SM2a MAX3(4, 5) FMAC(6) FMAC(7) EXP(8) EXP(9) ADD(6) ADD(7) CVT(4, 5)
#define SM2b MAX3(6, 7) FMAC(8) FMAC(9) EXP(4) EXP(5) ADD(8) ADD(9) CVT(6, 7)
// the attention tile's own ratio: one score register per MFMA (1 max3, 1 fmac, 1 exp, 2 add, 1 convert = 6 instructions)
#define SM1a MAX3(4, 5) FMAC(6) EXP(8) ADD(6) ADD(7) CVT(4, 5)
#define SM1b MAX3(6, 7) FMAC(8) EXP(4) ADD(8) ADD(9) CVT(6, 7)

enum { M4, M1CHAIN, FMA32, FMAC32, EXP16, DS8, M_DS2, M_FMAC8, M_FMAC4, M4_THEN_FMAC32, MIX32, M_MIX, M_DS_MIX, M_DS_FMAC4, M_DS_TILE, TILE_PHASES };

template <int MODE>
__device__ __forceinline__ void body(f32x16& c0, f32x16& c1, f32x16& c2, f32x16& c3, f32x4 a, f32x4 b, float& v0, float& v1,
                                     float& v2, float& v3, float& v4, float& v5, float k1, float k2, f32x4& q0, f32x4& q1, unsigned laddr) {
  if (MODE == M4) BODY(MF(0) MF(1) MF(2) MF(3));
  if (MODE == M1CHAIN) BODY(MF(0) MF(0) MF(0) MF(0));  // every MFMA accumulates into the result of the one before
  if (MODE == FMA32) BODY(X8(FMA) X8(FMA) X8(FMA) X8(FMA));
  if (MODE == FMAC32) BODY(X8(FMAC) X8(FMAC) X8(FMAC) X8(FMAC));
  if (MODE == EXP16) BODY(X8(EXP) X8(EXP));
  if (MODE == DS8) BODY(DSR(10) DSR2(11) DSR(10) DSR2(11) DSR(10) DSR2(11) DSR(10) DSR2(11) WAITL);
  if (MODE == M_DS2) BODY(MF(0) DSR(10) DSR2(11) MF(1) DSR(10) DSR2(11) MF(2) DSR(10) DSR2(11) MF(3) DSR(10) DSR2(11) WAITL);
  if (MODE == M_FMAC8) BODY(MF(0) X8(FMAC) MF(1) X8(FMAC) MF(2) X8(FMAC) MF(3) X8(FMAC));
  if (MODE == M_FMAC4) BODY(MF(0) X4a(FMAC) MF(1) X4b(FMAC) MF(2) X4a(FMAC) MF(3) X4b(FMAC));
  if (MODE == M4_THEN_FMAC32) BODY(MF(0) MF(1) MF(2) MF(3) X8(FMAC) X8(FMAC) X8(FMAC) X8(FMAC));
  if (MODE == MIX32) BODY(SM2a SM2b SM2a SM2b);
  if (MODE == M_MIX) BODY(MF(0) SM2a MF(1) SM2b MF(2) SM2a MF(3) SM2b);
  if (MODE == M_DS_MIX) BODY(MF(0) DSR(10) SM2a MF(1) DSR2(11) SM2b MF(2) DSR(10) SM2a MF(3) DSR2(11) SM2b WAITL);
  if (MODE == M_DS_TILE) BODY(MF(0) DSR(10) SM1a MF(1) DSR2(11) SM1b MF(2) DSR(10) SM1a MF(3) DSR2(11) SM1b WAITL);
  // the same work in the kernels' order: the MFMAs with their LDS reads first, then the vector block
  if (MODE == TILE_PHASES) BODY(MF(0) DSR(10) MF(1) DSR2(11) MF(2) DSR(10) MF(3) DSR2(11) SM1a SM1b SM1a SM1b WAITL);
  if (MODE == M_DS_FMAC4) BODY(MF(0) DSR(10) X4a(FMAC) MF(1) DSR2(11) X4b(FMAC) MF(2) DSR(10) X4a(FMAC) MF(3) DSR2(11) X4b(FMAC) WAITL);
}

template <int MA, int MB, int NW>
__global__ __launch_bounds__(NW * 64) void k(float* out, int iters, float seed) {
  __shared__ float lds[4096];
  const int wave = threadIdx.x >> 6;
  for (int i = threadIdx.x; i < 4096; i += NW * 64) lds[i] = seed * i;
  __syncthreads();
  f32x4 a = {seed, seed * 2, seed * 3, seed * 4}, b = {seed, -seed, seed, -seed};
  f32x4 q0 = a, q1 = b;
  f32x16 c0, c1, c2, c3;
  for (int i = 0; i < 16; ++i) c0[i] = c1[i] = c2[i] = c3[i] = 0.f;
  float v0 = seed, v1 = seed + 1, v2 = seed + 2, v3 = seed + 3, v4 = seed + 4, v5 = seed + 5;
  const float k1 = 0.999f, k2 = 0.001f * seed;
  const unsigned laddr = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void*)lds + (threadIdx.x & 63) * 16;
  if ((wave & 4) == 0) {
    for (int it = 0; it < iters; ++it) body<MA>(c0, c1, c2, c3, a, b, v0, v1, v2, v3, v4, v5, k1, k2, q0, q1, laddr);
  } else {
    for (int it = 0; it < iters; ++it) body<MB>(c0, c1, c2, c3, a, b, v0, v1, v2, v3, v4, v5, k1, k2, q0, q1, laddr);
  }
  asm volatile("s_nop 15\n s_nop 15\n s_waitcnt lgkmcnt(0)" ::: "memory");
  float s = v0 + v1 + v2 + v3 + v4 + v5 + q0[0] + q1[1];
  for (int i = 0; i < 16; ++i) s += c0[i] + c1[i] + c2[i] + c3[i];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

template <int MA, int MB, int NW>
static void run(const char* name, float* d) {
  const int iters = 40000;
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0);
  (void)hipEventCreate(&e1);
  hipLaunchKernelGGL((k<MA, MB, NW>), dim3(256), dim3(NW * 64), 0, 0, d, 100, 1.0f);
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL((k<MA, MB, NW>), dim3(256), dim3(NW * 64), 0, 0, d, iters, 1.0f);
  (void)hipEventRecord(e1);
  (void)hipEventSynchronize(e1);
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  printf("%-58s %7.3f ms  %7.1f cycles per iteration\n", name, ms, ms * 1e-3 * 2.4e9 / iters);
}

int main() {
  float* d;
  if (hipMalloc(&d, 256 * 1024 * 4) != hipSuccess) return 1;
  printf("one wavefront per SIMD (an MFMA 32x32x16 bf16 occupies the matrix core for 32 cycles)\n");
  run<M4, M4, 4>("4 mfma, 4 accumulators", d);
  run<M1CHAIN, M1CHAIN, 4>("4 mfma, one dependent chain", d);
  run<FMA32, FMA32, 4>("32 v_fma_f32 (64-bit encoding)", d);
  run<FMAC32, FMAC32, 4>("32 v_fmac_f32 (32-bit encoding)", d);
  run<EXP16, EXP16, 4>("16 v_exp_f32", d);
  run<DS8, DS8, 4>("8 ds_read_b128, then wait", d);
  run<MIX32, MIX32, 4>("softmax-like mix, 32 valu (8 of them v_exp)", d);
  run<M_FMAC4, M_FMAC4, 4>("4 x (mfma, 4 v_fmac)", d);
  run<M_FMAC8, M_FMAC8, 4>("4 x (mfma, 8 v_fmac)", d);
  run<M4_THEN_FMAC32, M4_THEN_FMAC32, 4>("4 mfma, then 32 v_fmac", d);
  run<M_MIX, M_MIX, 4>("4 x (mfma, 8-valu softmax mix)", d);
  run<M_DS2, M_DS2, 4>("4 x (mfma, 2 ds_read_b128)", d);
  run<M_DS_FMAC4, M_DS_FMAC4, 4>("4 x (mfma, ds_read_b128, 4 v_fmac)", d);
  run<M_DS_MIX, M_DS_MIX, 4>("4 x (mfma, ds_read_b128, 8-valu mix)", d);
  printf("two wavefronts per SIMD (first body | second body)\n");
  run<M4, M4, 8>("4 mfma | 4 mfma", d);
  run<FMAC32, FMAC32, 8>("32 v_fmac | 32 v_fmac", d);
  run<EXP16, EXP16, 8>("16 v_exp | 16 v_exp", d);
  run<MIX32, MIX32, 8>("softmax mix | softmax mix", d);
  run<M4, FMAC32, 8>("4 mfma | 32 v_fmac", d);
  run<M4, EXP16, 8>("4 mfma | 16 v_exp", d);
  run<M4, MIX32, 8>("4 mfma | softmax mix", d);
  run<M_MIX, M_MIX, 8>("4 x (mfma, mix) | 4 x (mfma, mix)", d);
  run<M_DS_MIX, M_DS_MIX, 8>("4 x (mfma, ds_read, mix) | the same", d);
  run<M_DS_FMAC4, M_DS_FMAC4, 8>("4 x (mfma, ds_read, 4 v_fmac) | the same", d);
  run<M_DS_TILE, M_DS_TILE, 4>("one wavefront: 4 x (mfma, ds_read, 6-valu tile mix)", d);
  run<TILE_PHASES, TILE_PHASES, 4>("one wavefront: 4 x (mfma, ds_read), then 24 valu", d);
  run<M_DS_TILE, M_DS_TILE, 8>("4 x (mfma, ds_read, 6-valu tile mix) | the same", d);
  run<TILE_PHASES, TILE_PHASES, 8>("4 x (mfma, ds_read), then 24 valu | the same", d);
  printf("three and four wavefronts per SIMD, all running the same body\n");
  run<M_DS_TILE, M_DS_TILE, 12>("3 x 4 x (mfma, ds_read, 6-valu tile mix)", d);
  run<TILE_PHASES, TILE_PHASES, 12>("3 x (4 x (mfma, ds_read), then 24 valu)", d);

  run<M4, M4, 12>("3 x 4 mfma", d);
  run<M_MIX, M_MIX, 12>("3 x 4 x (mfma, mix)", d);
  run<M_DS_MIX, M_DS_MIX, 12>("3 x 4 x (mfma, ds_read, mix)", d);
  run<M_DS_FMAC4, M_DS_FMAC4, 12>("3 x 4 x (mfma, ds_read, 4 v_fmac)", d);
  run<M_MIX, M_MIX, 16>("4 x 4 x (mfma, mix)", d);
  run<M_DS_MIX, M_DS_MIX, 16>("4 x 4 x (mfma, ds_read, mix)", d);
  run<M_DS_FMAC4, M_DS_FMAC4, 16>("4 x 4 x (mfma, ds_read, 4 v_fmac)", d);
  printf("status %s\n", hipGetErrorString(hipDeviceSynchronize()));
  return 0;
}
