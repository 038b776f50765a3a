// Measurement aid of bench.py, not part of the attention library: loops of matrix
// instructions on operands taken from memory, to measure what the matrix pipes of the GPU
// sustain on given operand values (on random data the part is power-bound well below its
// nominal peak).  Built into libbench_mfma_probe.so next to bench.py.
//
//   int bench_mfma_probe(const void* operands, long long* clocks, int form, int iters, void* stream)
//
//   operands : 64 KB of device memory, 16-byte aligned, read as operand values (bfloat16 for
//              forms 0 and 1, E4M3 bytes for forms 2 to 4).
//   clocks   : 3 int64 on the device, 8-byte aligned; receives {shader clocks, 100 MHz reference
//              ticks} spent in the loop by workgroup 0 (the third is scratch).
//   form     : 0 = v_mfma_f32_32x32x16_bf16 (16 per iteration), 1 = v_mfma_f32_16x16x32_bf16 (32
//              per iteration), 2 = v_mfma_f32_16x16x128_f8f6f4 on E4M3 (8 per iteration); in every
//              form 256 * 4 waves * iters * 16 * 32768 flop per launch.  Forms 3 and 4 are form 2
//              with, pinned behind every matrix instruction, the other instructions that one wave
//              of an all-E4M3 attention kernel issues per matrix instruction: a 16-byte LDS read
//              and, 3: one scaled convert and two register moves (L2 normaliser); 4: scale-and-
//              shift, exponential, running max and sum for two scores and one convert (SoftMax,
//              without its cross-lane maximum and rescaling).  Their ratio is what the
//              exponential costs at the fp8 matrix rate (paper, Section 1).
//   iters    : 1 .. 2^24.
// One launch of 256 workgroups of 256 threads on `stream`; returns 0, or -1 (null pointer),
// -2 (form, iters), -5 (alignment), -6 (launch refused).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;

// ---------------------------------------------------------------------------
// Measurement aid: a loop of nothing but matrix instructions on operands taken from memory
// (the benchmark fills them with Gaussian values), to measure what the matrix pipes sustain at
// the power limit next to the attention kernel.  FORM 0: v_mfma_f32_32x32x16_bf16, 1:
// v_mfma_f32_16x16x32_bf16 (twice as many, same flops) or v_mfma_f32_16x16x128_f8f6f4 on E4M3
// operands (half as many, same flops).  Each lane keeps 16 operand pairs in
// rotation; clocks[0] / clocks[1] of workgroup 0 = shader clocks / 100 MHz reference ticks.
// ---------------------------------------------------------------------------
template <int FORM>
__global__ __launch_bounds__(256)
void mfma_probe_kernel(const i32x4* __restrict__ operands, long long* __restrict__ clocks, int iters)
{
    constexpr int NP = 16;
    i32x4 a[NP], b[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        a[i] = operands[(threadIdx.x * 8 + 2 * i) % 4096];
        b[i] = operands[(threadIdx.x * 8 + 2 * i + 1) % 4096];
    }
    f32x16 c32[4];
    f32x4 c16[16];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) c32[i][e] = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) c16[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    // forms 3, 4: state of the instructions pinned behind the matrix instructions
    __shared__ __attribute__((aligned(16))) unsigned char mix_lds[FORM >= 3 ? 16384 : 16];
    i32x4 mix_ld = {0, 0, 0, 0};
    float mix_x0 = 0.25f, mix_x1 = 0.5f, mix_e0 = 0.f, mix_e1 = 0.f, mix_m = 0.f, mix_s = 0.f;
    const float mix_c = 1.0f;
    int mix_w = 0;
    uint32_t mix_addr = 0;
    if constexpr (FORM >= 3) {
        for (int i = threadIdx.x; i < 1024; i += 256)
            reinterpret_cast<i32x4*>(mix_lds)[i] = i32x4{0, 0, 0, 0};
        __syncthreads();
        const int l = threadIdx.x & 63;            // rows of 64 bytes, as the kernels' fragment reads
        mix_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) unsigned char*)mix_lds + (l & 15) * 64 + (l >> 4) * 16;
    }
    const long long t0 = clock64(), w0 = wall_clock64();
    for (int it = 0; it < iters; ++it) {
        if constexpr (FORM == 0) {
#pragma unroll
            for (int i = 0; i < NP; ++i)
                c32[i % 4] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b[i]), c32[i % 4], 0, 0, 0);
        } else if constexpr (FORM == 1) {
#pragma unroll
            for (int i = 0; i < 2 * NP; ++i)
                c16[i % 16] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                    __builtin_bit_cast(bf16x8, a[i % NP]), __builtin_bit_cast(bf16x8, b[(i + i / NP) % NP]), c16[i % 16], 0, 0, 0);
        } else {
            // E4M3 operands, k = 128: 8 instructions carry the flops of 16 of the bf16 forms.
            // Forms 3 and 4 put, behind every matrix instruction and pinned there, what one
            // wave has to issue per matrix instruction in an attention kernel whose scores go
            // back to the matrix cores as E4M3: one 16-byte LDS read and
            //   form 3 (L2 normaliser): one scaled convert and two register moves;
            //   form 4 (SoftMax): scale-and-shift, exponential, running max and running sum
            //                     for two scores, and one convert
            // -- without the cross-lane maximum and the rescaling that a real SoftMax adds.
            typedef __attribute__((ext_vector_type(8))) int i32x8;
#pragma unroll
            for (int i = 0; i < NP / 2; ++i) {
                const i32x8 a8 = __builtin_shufflevector(a[2 * i], a[2 * i + 1], 0, 1, 2, 3, 4, 5, 6, 7);
                const i32x8 b8 = __builtin_shufflevector(b[2 * i], b[2 * i + 1], 0, 1, 2, 3, 4, 5, 6, 7);
                c16[i] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a8, b8, c16[i], 0, 0, 0, 0, 0, 0);
                if constexpr (FORM >= 3) {
                    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(mix_ld) : "v"(mix_addr), "n"(i * 2048));
                    if constexpr (FORM == 4) {
                        asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(mix_e0) : "v"(mix_x0), "v"(mix_c), "v"(mix_x1));
                        asm volatile("v_fma_f32 %0, %1, %2, %3" : "=v"(mix_e1) : "v"(mix_x1), "v"(mix_c), "v"(mix_x0));
                        asm volatile("v_exp_f32 %0, %1" : "=v"(mix_x0) : "v"(mix_e0));
                        asm volatile("v_exp_f32 %0, %1" : "=v"(mix_x1) : "v"(mix_e1));
                        asm volatile("v_max_f32 %0, %1, %2" : "=v"(mix_m) : "v"(mix_e0), "v"(mix_m));
                        asm volatile("v_add_f32 %0, %1, %2" : "=v"(mix_s) : "v"(mix_x0), "v"(mix_s));
                    } else {
                        asm volatile("v_mov_b32 %0, %1" : "=v"(mix_e0) : "v"(mix_w));
                        asm volatile("v_mov_b32 %0, %1" : "=v"(mix_e1) : "v"(mix_e0));
                    }
                    asm volatile("v_cvt_scalef32_pk_fp8_f32 %0, %1, %2, %3" : "+v"(mix_w) : "v"(mix_x0), "v"(mix_x1), "v"(mix_c));
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
            if constexpr (FORM >= 3) {
                if ((it & 3) == 3) asm volatile("s_waitcnt lgkmcnt(0)");
            }
        }
        if ((it & 63) == 63) {                     // keep the sums finite
#pragma unroll
            for (int i = 0; i < 4; ++i) c32[i] *= 0.001f;
#pragma unroll
            for (int i = 0; i < 16; ++i) c16[i] *= 0.001f;
        }
    }
    if constexpr (FORM >= 3) asm volatile("s_waitcnt lgkmcnt(0)");
    const long long t1 = clock64(), w1 = wall_clock64();
    float sum = (float)mix_ld[0] + mix_x0 + mix_x1 + mix_e0 + mix_e1 + mix_m + mix_s + (float)mix_w;
#pragma unroll
    for (int i = 0; i < 4; ++i) sum += c32[i][0] + c32[i][7];
#pragma unroll
    for (int i = 0; i < 16; ++i) sum += c16[i][0] + c16[i][3];
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        clocks[0] = t1 - t0;
        clocks[1] = w1 - w0;
    }
    if (sum == 12345.678f) clocks[2] = 1;          // keeps the loop alive; never true in practice
}


template <int FORM>
int launch(const void* operands, long long* clocks, int iters, hipStream_t stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel<FORM>, dim3(256), dim3(256), 0, stream,
                       (const i32x4*)operands, clocks, iters);
    return hipGetLastError() == hipSuccess ? 0 : -6;
}

}  // namespace

extern "C" int bench_mfma_probe(const void* operands, long long* clocks, int form, int iters, void* stream)
{
    if (!operands || !clocks) return -1;
    if (iters <= 0 || iters > (1 << 24) || form < 0 || form > 4) return -2;
    if (((uintptr_t)operands & 15) || ((uintptr_t)clocks & 7)) return -5;
    hipStream_t st = (hipStream_t)stream;
    switch (form) {
    case 0: return launch<0>(operands, clocks, iters, st);
    case 1: return launch<1>(operands, clocks, iters, st);
    case 2: return launch<2>(operands, clocks, iters, st);
    case 3: return launch<3>(operands, clocks, iters, st);
    default: return launch<4>(operands, clocks, iters, st);
    }
}
