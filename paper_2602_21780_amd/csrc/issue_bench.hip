// Issue-rate microbenchmarks for gfx950: what one SIMD of a compute unit can issue per cycle for the instruction
// kinds of the attention kernel's inner loop (fp32 multiply-add, exponential, bf16 pack, bf16 dot product, the
// 32x32x16 bf16 MFMA, and mixtures), with one to four waves per SIMD.  A standalone program:
//   python -m paper_2602_21780_amd.build      (builds paper_2602_21780_amd/issue_bench beside the library)
//   ./paper_2602_21780_amd/issue_bench
// Every workgroup runs the same straight-line loop; wave 0 of workgroup 0 reports its cycle counter (s_memtime),
// the host the wall time of the launch.  The figures are what the design notes of the attention kernel quote.
#include <hip/hip_runtime.h>
#include <cstdio>
#include <vector>
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;

#define REP4(x) x x x x
#define REP16(x) REP4(x) REP4(x) REP4(x) REP4(x)
#define REP64(x) REP16(x) REP16(x) REP16(x) REP16(x)

__device__ __forceinline__ unsigned long long now() { return __builtin_amdgcn_s_memtime(); }

template <int MODE>
__global__ __launch_bounds__(1024) void k(unsigned long long* out, float* sink, int iters) {
  float a0 = threadIdx.x, a1 = a0 + 1, a2 = a0 + 2, a3 = a0 + 3, a4 = a0 * .5f, a5 = a0 * .25f, a6 = a0 * .125f, a7 = 7.f;
  const float c = 1.0001f, d = 0.0001f;
  f32x16 acc0 = {0}, acc1 = {0}, acc2 = {0}, acc3 = {0};
  f32x4 q0 = {0}, q1 = {0}, q2 = {0}, q3 = {0};
  bf16x8 fa = {1, 1, 1, 1, 1, 1, 1, 1}, fb = fa;
  asm volatile("" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7));
  asm volatile("" : "+v"(fa), "+v"(fb));
  __syncthreads();
  const unsigned long long t0 = now();
  for (int it = 0; it < iters; ++it) {
    if constexpr (MODE == 0) {  // 64 independent fma (8 chains)
      REP4(asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n"
                        "v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n"
                        "v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n"
                        "v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n"
                        : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 1) {  // 64 exp (8 chains)
      REP4(asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n"
                        "v_exp_f32 %4, %4\n v_exp_f32 %5, %5\n v_exp_f32 %6, %6\n v_exp_f32 %7, %7\n"
                        "v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n"
                        "v_exp_f32 %4, %4\n v_exp_f32 %5, %5\n v_exp_f32 %6, %6\n v_exp_f32 %7, %7\n"
                        : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7));)
    } else if constexpr (MODE == 2) {  // 64 dependent dot2c (one chain)
      REP64(asm volatile("v_dot2c_f32_bf16 %0, %1, %2" : "+v"(a0) : "v"(a1), "v"(a2));)
    } else if constexpr (MODE == 3) {  // 64 dot2c, 8 chains
      REP4(asm volatile("v_dot2c_f32_bf16 %0, %8, %9\n v_dot2c_f32_bf16 %1, %8, %9\n v_dot2c_f32_bf16 %2, %8, %9\n v_dot2c_f32_bf16 %3, %8, %9\n"
                        "v_dot2c_f32_bf16 %4, %8, %9\n v_dot2c_f32_bf16 %5, %8, %9\n v_dot2c_f32_bf16 %6, %8, %9\n v_dot2c_f32_bf16 %7, %8, %9\n"
                        "v_dot2c_f32_bf16 %0, %8, %9\n v_dot2c_f32_bf16 %1, %8, %9\n v_dot2c_f32_bf16 %2, %8, %9\n v_dot2c_f32_bf16 %3, %8, %9\n"
                        "v_dot2c_f32_bf16 %4, %8, %9\n v_dot2c_f32_bf16 %5, %8, %9\n v_dot2c_f32_bf16 %6, %8, %9\n v_dot2c_f32_bf16 %7, %8, %9\n"
                        : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 4) {  // 64 cvt_pk_bf16
      REP4(asm volatile("v_cvt_pk_bf16_f32 %0, %0, %8\n v_cvt_pk_bf16_f32 %1, %1, %8\n v_cvt_pk_bf16_f32 %2, %2, %8\n v_cvt_pk_bf16_f32 %3, %3, %8\n"
                        "v_cvt_pk_bf16_f32 %4, %4, %8\n v_cvt_pk_bf16_f32 %5, %5, %8\n v_cvt_pk_bf16_f32 %6, %6, %8\n v_cvt_pk_bf16_f32 %7, %7, %8\n"
                        "v_cvt_pk_bf16_f32 %0, %0, %8\n v_cvt_pk_bf16_f32 %1, %1, %8\n v_cvt_pk_bf16_f32 %2, %2, %8\n v_cvt_pk_bf16_f32 %3, %3, %8\n"
                        "v_cvt_pk_bf16_f32 %4, %4, %8\n v_cvt_pk_bf16_f32 %5, %5, %8\n v_cvt_pk_bf16_f32 %6, %6, %8\n v_cvt_pk_bf16_f32 %7, %7, %8\n"
                        : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c));)
    } else if constexpr (MODE == 5) {  // 16 mfma, 4 independent accumulators
      REP4(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);
           acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc1, 0, 0, 0);
           acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc2, 0, 0, 0);
           acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc3, 0, 0, 0);)
    } else if constexpr (MODE == 6) {  // 16 mfma each followed by 4 independent fma (= 64 fma)
      REP4(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc1, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc2, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc3, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 7) {  // 16 mfma each followed by 8 fma (= 128 fma)
      REP4(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc1, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc2, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc3, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %8, %9\n v_fma_f32 %1, %1, %8, %9\n v_fma_f32 %2, %2, %8, %9\n v_fma_f32 %3, %3, %8, %9\n v_fma_f32 %4, %4, %8, %9\n v_fma_f32 %5, %5, %8, %9\n v_fma_f32 %6, %6, %8, %9\n v_fma_f32 %7, %7, %8, %9\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3), "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 8) {  // 16 mfma each followed by 4 exp (= 64 exp)
      REP4(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);
           asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));
           acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc1, 0, 0, 0);
           asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7));
           acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc2, 0, 0, 0);
           asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3));
           acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc3, 0, 0, 0);
           asm volatile("v_exp_f32 %0, %0\n v_exp_f32 %1, %1\n v_exp_f32 %2, %2\n v_exp_f32 %3, %3\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7));)
    } else if constexpr (MODE == 10) {  // the attention loop's mix per 16 MFMAs: 96 fma + 32 exp, spread evenly
      REP4(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           acc1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc1, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc2, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           acc3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc3, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_exp_f32 %3, %3\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 11) {  // 32 mfma 16x16x32 (the flops of 16 of the 32x32x16), 4 accumulators
      REP4(q0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q0, 0, 0, 0); q1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q1, 0, 0, 0);
           q2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q2, 0, 0, 0); q3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q3, 0, 0, 0);
           q0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q0, 0, 0, 0); q1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q1, 0, 0, 0);
           q2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q2, 0, 0, 0); q3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q3, 0, 0, 0);)
    } else if constexpr (MODE == 12) {  // the same 32 mfma 16x16x32, each followed by 4 fma (= 128 fma)
      REP4(q0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q0, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           q1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q1, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           q2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q2, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           q3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q3, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           q0 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q0, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           q1 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q1, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));
           q2 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q2, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a0), "+v"(a1), "+v"(a2), "+v"(a3) : "v"(c), "v"(d));
           q3 = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, q3, 0, 0, 0);
           asm volatile("v_fma_f32 %0, %0, %4, %5\n v_fma_f32 %1, %1, %4, %5\n v_fma_f32 %2, %2, %4, %5\n v_fma_f32 %3, %3, %4, %5\n" : "+v"(a4), "+v"(a5), "+v"(a6), "+v"(a7) : "v"(c), "v"(d));)
    } else if constexpr (MODE == 9) {  // 16 dependent mfma (one accumulator)
      REP16(acc0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, acc0, 0, 0, 0);)
    }
  }
  const unsigned long long t1 = now();
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * 16 + (threadIdx.x >> 6)] = t1 - t0;
  sink[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3 + a4 + a5 + a6 + a7 + acc0[0] + acc1[1] + acc2[2] + acc3[3] + q0[0] + q1[1] + q2[2] + q3[3];
}

// The attention kernel's tile loop without its memory traffic: two query blocks per wave, four softmax blocks per
// "tile" with the MFMAs of the other block issued inside them in the kernel's order, operands from registers that stay
// as they are.  PART: 0 = everything, 2 = no softmax arithmetic (conversions only).
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
__device__ __forceinline__ unsigned int pk_bf16(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f2;
  typedef __attribute__((ext_vector_type(2))) __bf16 b2;
  const f2 v = {a, b};
  return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, b2));
}
template <int PART>
__global__ __launch_bounds__(512) void tile_loop(unsigned long long* out, float* sink, int iters) {
  f32x16 o0[2], o1[2], sA, sB;
  bf16x8 qf[2][4], kf[4], vf[2][2];
  u32x4 pA[2], pB[2];
  float mc[2] = {-3.f, -2.f}, l[2] = {0.f, 0.f};
  const float c2 = 0.18f;
  for (int i = 0; i < 16; ++i) { o0[0][i] = o0[1][i] = o1[0][i] = o1[1][i] = 0.f; sA[i] = 0.01f * (threadIdx.x + i); sB[i] = 0.02f * (threadIdx.x + i); }
  for (int i = 0; i < 4; ++i) { qf[0][i] = qf[1][i] = kf[i] = bf16x8{1, 1, 1, 1, 1, 1, 1, 1}; vf[i >> 1][i & 1] = kf[i]; }
  pA[0] = pA[1] = pB[0] = pB[1] = u32x4{0x3c003c00u, 0x3c003c00u, 0x3c003c00u, 0x3c003c00u};
  asm volatile("" : "+v"(sA), "+v"(sB));
  auto qk = [&](f32x16& sv, int cb, int i) {
    if constexpr (PART != 1) sv = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[i], qf[cb][i], sv, 0, 0, 0);
  };
  auto pv = [&](int cb, const u32x4 (&pb)[2], int i) {
    if constexpr (PART != 1) {
      const bf16x8 p = __builtin_bit_cast(bf16x8, pb[i >> 1]);
      if (i & 1) o1[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i >> 1][1], p, o1[cb], 0, 0, 0);
      else o0[cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[i >> 1][0], p, o0[cb], 0, 0, 0);
    }
  };
  auto softmax = [&](f32x16& sv, u32x4 (&pb)[2], float mcr, float& lsum, auto&& hook, int n_mfma) {
    float psum = lsum;
#pragma unroll
    for (int q4 = 0; q4 < 4; ++q4) {
      hook(q4);
#pragma unroll
      for (int r = 4 * q4; r < 4 * q4 + 4; r += 2) {
        unsigned int w;
        if constexpr (PART == 2) {
          w = pk_bf16(sv[r], sv[r + 1]);
        } else {
          const float p0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], c2, mcr));
          const float p1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r + 1], c2, mcr));
          w = pk_bf16(p0, p1);
          psum = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(__attribute__((ext_vector_type(2))) __bf16, w),
                                                 __builtin_bit_cast(__attribute__((ext_vector_type(2))) __bf16, 0x3f803f80u), psum, false);
        }
        pb[r >> 3][(r >> 1) & 3] = w;
      }
    }
    if (PART == 0) {
#pragma unroll
      for (int q4 = 0; q4 < 4; ++q4) {
        if (n_mfma == 2) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 2, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        } else {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x400, 4, 0);
          __builtin_amdgcn_sched_group_barrier(0x002, 4, 0);
        }
      }
    }
    asm volatile("" : "+v"(pb[0]), "+v"(pb[1]));
    lsum = psum;
    __builtin_amdgcn_sched_barrier(0);
  };
  __syncthreads();
  const unsigned long long r0 = __builtin_amdgcn_s_memrealtime();
  const unsigned long long t0 = now();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 4; ++i) qk(sA, 0, i);
    softmax(sA, pA, mc[0], l[0], [&](int i) { qk(sB, 1, i); }, 1);
    softmax(sB, pB, mc[1], l[1], [&](int i) { pv(0, pA, i); qk(sA, 0, i); }, 2);
    softmax(sA, pA, mc[0], l[0], [&](int i) { pv(1, pB, i); qk(sB, 1, i); }, 2);
    softmax(sB, pB, mc[1], l[1], [&](int i) { pv(0, pA, i); }, 1);
#pragma unroll
    for (int i = 0; i < 4; ++i) pv(1, pB, i);
    // keep the logits where they were (the products above would otherwise grow them without bound)
#pragma unroll
    for (int i = 0; i < 16; ++i) { sA[i] = 0.01f * i; sB[i] = 0.02f * i; }
    asm volatile("" : "+v"(sA), "+v"(sB));
  }
  const unsigned long long t1 = now();
  if ((threadIdx.x & 63) == 0) out[blockIdx.x * 16 + (threadIdx.x >> 6)] = t1 - t0;
  if (threadIdx.x == 0) out[256 * 16 + blockIdx.x] = __builtin_amdgcn_s_memrealtime() - r0;  // 100 MHz wall clock
  float acc = l[0] + l[1];
  for (int i = 0; i < 16; ++i) acc += o0[0][i] + o0[1][i] + o1[0][i] + o1[1][i] + sA[i] + sB[i];
  sink[blockIdx.x * blockDim.x + threadIdx.x] = acc;
}

template <int PART>
void run_tile(const char* name, int threads, unsigned long long* dout, float* sink) {
  const int iters = 500, blocks = 256;
  hipLaunchKernelGGL(tile_loop<PART>, dim3(blocks), dim3(threads), 0, 0, dout, sink, 10);
  (void)hipDeviceSynchronize();
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL(tile_loop<PART>, dim3(blocks), dim3(threads), 0, 0, dout, sink, iters);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  std::vector<unsigned long long> h(blocks * 17);
  if (hipMemcpy(h.data(), dout, h.size() * 8, hipMemcpyDeviceToHost) != hipSuccess) { printf("copy failed\n"); return; }
  // shader clock of workgroup 0 while the loop ran: its cycle count over its 100 MHz wall-clock count
  const double mhz = (double)h[0] / ((double)h[blocks * 16] / 100.0);
  printf("%-44s waves/SIMD %d: wave 0 %7.1f cycles per tile; launch %7.1f ns per tile; shader clock %4.0f MHz\n", name, threads / 256,
         (double)h[0] / iters, ms * 1e6 / iters, mhz);
}

template <int MODE>
void run(const char* name, int per_iter, int threads, unsigned long long* dout, float* sink) {
  const int iters = 2000, blocks = 256;
  hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(threads), 0, 0, dout, sink, 10);
  (void)hipDeviceSynchronize();
  hipEvent_t e0, e1;
  (void)hipEventCreate(&e0); (void)hipEventCreate(&e1);
  (void)hipEventRecord(e0);
  hipLaunchKernelGGL(k<MODE>, dim3(blocks), dim3(threads), 0, 0, dout, sink, iters);
  (void)hipEventRecord(e1);
  (void)hipDeviceSynchronize();
  float ms = 0.f;
  (void)hipEventElapsedTime(&ms, e0, e1);
  std::vector<unsigned long long> h(blocks * 16);
  if (hipMemcpy(h.data(), dout, h.size() * 8, hipMemcpyDeviceToHost) != hipSuccess) { printf("copy failed\n"); return; }
  double cyc = (double)h[0] / iters;
  // wall: all waves of a SIMD together; cycles: the reporting wave alone (with two waves per SIMD the older wave is
  // served first, so its own count can stay at the one-wave figure while the launch takes up to twice as long)
  printf("%-32s waves/SIMD %d: wave 0 %7.1f cycles/iteration = %5.2f per instruction (%3d); launch %7.1f ns/iteration = %6.1f ns per wave\n",
         name, threads / 256, cyc, cyc / per_iter, per_iter, ms * 1e6 / iters, ms * 1e6 / iters / (threads / 256));
}

int main() {
  unsigned long long* dout; float* sink;
  if (hipMalloc(&dout, 256 * 17 * 8) != hipSuccess || hipMalloc(&sink, 256 * 1024 * 4) != hipSuccess) { printf("no device memory\n"); return 1; }
  for (int threads : {256, 512, 768, 1024}) {
    run<0>("64 fma (8 chains)", 64, threads, dout, sink);
    run<1>("64 exp (8 chains)", 64, threads, dout, sink);
    run<2>("64 dot2c (1 chain)", 64, threads, dout, sink);
    run<3>("64 dot2c (8 chains)", 64, threads, dout, sink);
    run<4>("64 cvt_pk_bf16 (8 chains)", 64, threads, dout, sink);
    run<5>("16 mfma (4 accumulators)", 16, threads, dout, sink);
    run<9>("16 mfma (1 accumulator)", 16, threads, dout, sink);
    run<6>("16 mfma + 64 fma interleaved", 80, threads, dout, sink);
    run<7>("16 mfma + 128 fma interleaved", 144, threads, dout, sink);
    run<8>("16 mfma + 64 exp interleaved", 80, threads, dout, sink);
    run<10>("16 mfma + 96 fma + 32 exp", 144, threads, dout, sink);
    run<11>("32 mfma 16x16x32", 32, threads, dout, sink);
    run<12>("32 mfma 16x16x32 + 128 fma", 160, threads, dout, sink);
  }
  for (int threads : {256, 512}) {
    run_tile<0>("tile loop of the attention kernel, registers only", threads, dout, sink);
    run_tile<2>("  without its softmax arithmetic", threads, dout, sink);
  }
  return 0;
}
