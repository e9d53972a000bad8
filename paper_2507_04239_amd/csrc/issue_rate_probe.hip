// Standalone measurement program (not part of the library): issue rates of the instruction mixes the
// state kernels are made of, on one and on two waves per SIMD of every compute unit.  It backs the
// choice between "one fat wave per SIMD that keeps a large slab of the state in registers" and
// "two thinner waves per SIMD": the operand expansion of the tiled symmetric-power embedding
// (arXiv 2507.04239, Sec. 4.1.1) costs two multiplies and one bf16 conversion per MFMA operand dword,
// i.e. three vector-ALU instructions per 16 x 16 x 32 MFMA at 64 value columns.
// Build: hipcc --offload-arch=gfx950 -O3 issue_rate_probe.hip -o issue_rate_probe;  run without arguments.
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;

#define MF16(A) A = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fb, A, 0, 0, 0);
#define MF32(A) A = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa, fb, A, 0, 0, 0);
// two multiplies and the conversion of their results: one operand dword of an expanded fragment
#define V3 asm volatile("v_mul_f32 %0, %3, %4\n v_mul_f32 %1, %3, %4\n s_nop 0\n v_cvt_pk_bf16_f32 %2, %0, %1\n" : "=&v"(r0), "=&v"(r1), "=v"(u0) : "v"(a), "v"(b));
#define D3 asm volatile("v_mul_f32_dpp %0, %3, %4 row_newbcast:1 row_mask:0xf bank_mask:0xf\n v_mul_f32_dpp %1, %3, %4 row_newbcast:2 row_mask:0xf bank_mask:0xf\n s_nop 0\n v_cvt_pk_bf16_f32 %2, %0, %1\n" : "=&v"(r0), "=&v"(r1), "=v"(u0) : "v"(a), "v"(b));

template <int MODE, int NT>
__global__ __launch_bounds__(NT, 1) void k_probe(float* out, int iters, float seed) {
    float a = seed + threadIdx.x, b = seed * 2 + threadIdx.x;
    float r0 = 0, r1 = 0;
    uint32_t u0 = 0;
    f32x4 c0 = {0, 0, 0, 0}, c1 = c0, c2 = c0, c3 = c0, c4 = c0, c5 = c0, c6 = c0, c7 = c0, c8 = c0, c9 = c0, c10 = c0,
          c11 = c0, c12 = c0, c13 = c0, c14 = c0, c15 = c0;
    f32x16 d0, d1, d2, d3;
    for (int i = 0; i < 16; ++i) d0[i] = d1[i] = d2[i] = d3[i] = 0;
    bf16x8 fa, fb;
    for (int i = 0; i < 8; ++i) {
        fa[i] = (__bf16)(a + i);
        fb[i] = (__bf16)(b - i);
    }
    for (int it = 0; it < iters; ++it) {   // every mode: the FLOPs of 16 MFMAs of 16 x 16 x 32 per iteration
        if (MODE == 0) { MF16(c0) MF16(c1) MF16(c2) MF16(c3) MF16(c4) MF16(c5) MF16(c6) MF16(c7) MF16(c8) MF16(c9) MF16(c10) MF16(c11) MF16(c12) MF16(c13) MF16(c14) MF16(c15) }
        if (MODE == 1) { MF16(c0) V3 MF16(c1) V3 MF16(c2) V3 MF16(c3) V3 MF16(c4) V3 MF16(c5) V3 MF16(c6) V3 MF16(c7) V3 MF16(c8) V3 MF16(c9) V3 MF16(c10) V3 MF16(c11) V3 MF16(c12) V3 MF16(c13) V3 MF16(c14) V3 MF16(c15) V3 }
        if (MODE == 2) { MF32(d0) MF32(d1) MF32(d2) MF32(d3) MF32(d0) MF32(d1) MF32(d2) MF32(d3) }
        if (MODE == 3) { MF32(d0) V3 V3 MF32(d1) V3 V3 MF32(d2) V3 V3 MF32(d3) V3 V3 MF32(d0) V3 V3 MF32(d1) V3 V3 MF32(d2) V3 V3 MF32(d3) V3 V3 }
        if (MODE == 4) { MF16(c0) D3 MF16(c1) D3 MF16(c2) D3 MF16(c3) D3 MF16(c4) D3 MF16(c5) D3 MF16(c6) D3 MF16(c7) D3 MF16(c8) D3 MF16(c9) D3 MF16(c10) D3 MF16(c11) D3 MF16(c12) D3 MF16(c13) D3 MF16(c14) D3 MF16(c15) D3 }
        if (MODE == 5) { V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 V3 }
    }
    float s = r0 + r1 + (float)u0 + c0[0] + c1[0] + c2[0] + c3[0] + c4[0] + c5[0] + c6[0] + c7[0] + c8[0] + c9[0] + c10[0] +
              c11[0] + c12[0] + c13[0] + c14[0] + c15[0] + d0[0] + d1[0] + d2[0] + d3[0];
    if (s == 123.456f) out[0] = s;
}

template <int MODE, int NT>
void run(const char* name, float* d) {
    const int iters = 20000;
    hipEvent_t e0, e1;
    (void)hipEventCreate(&e0);
    (void)hipEventCreate(&e1);
    hipLaunchKernelGGL((k_probe<MODE, NT>), dim3(256), dim3(NT), 0, 0, d, 100, 1.0f);
    (void)hipEventRecord(e0);
    hipLaunchKernelGGL((k_probe<MODE, NT>), dim3(256), dim3(NT), 0, 0, d, iters, 1.0f);
    (void)hipEventRecord(e1);
    (void)hipEventSynchronize(e1);
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    const double waves = 256.0 * NT / 64;
    if (MODE == 5)
        printf("%-44s waves/SIMD=%d  %7.3f ms  %6.2f ns per group of three instructions and wave\n", name, NT / 256, ms,
               ms * 1e6 / iters / 16);
    else
        printf("%-44s waves/SIMD=%d  %7.3f ms  %7.1f TFLOP/s on the chip\n", name, NT / 256, ms,
               waves * 16 * 16384.0 * iters / (ms * 1e-3) / 1e12);
}

int main() {
    float* d = nullptr;
    if (hipMalloc(&d, 64) != hipSuccess) return 1;
    run<0, 256>("mfma 16x16x32 bf16, 16 accumulators", d);
    run<0, 512>("mfma 16x16x32 bf16, 16 accumulators", d);
    run<2, 256>("mfma 32x32x16 bf16, 4 accumulators", d);
    run<2, 512>("mfma 32x32x16 bf16, 4 accumulators", d);
    run<1, 256>("mfma 16x16x32 + 2 mul + cvt_pk", d);
    run<1, 512>("mfma 16x16x32 + 2 mul + cvt_pk", d);
    run<4, 256>("mfma 16x16x32 + 2 dpp mul + cvt_pk", d);
    run<4, 512>("mfma 16x16x32 + 2 dpp mul + cvt_pk", d);
    run<3, 256>("mfma 32x32x16 + 2 x (2 mul + cvt_pk)", d);
    run<3, 512>("mfma 32x32x16 + 2 x (2 mul + cvt_pk)", d);
    run<5, 256>("2 mul + cvt_pk alone", d);
    (void)hipFree(d);
    return 0;
}
