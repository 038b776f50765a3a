// Measurement aid of bench.py, not part of the attention library: one workgroup of four waves
// (one per SIMD of a CU) issues LDS fragment reads with a given lane -> address pattern, 16 in
// flight per wave, so that the LDS pipe of the CU is what bounds it.  Under
// `rocprofv3 --pmc SQ_LDS_IDX_ACTIVE SQ_LDS_BANK_CONFLICT SQ_INSTS_LDS` every launch is one
// dispatch, and the two counters per instruction give the cycles a read occupies the LDS and
// how many of them are bank conflicts.  Built into libbench_lds_probe.so next to bench.py.
//
//   int bench_lds_probe(long long* clocks, int pattern, int iters, void* stream)
//
//   clocks  : 4 int64 on the device, 8-byte aligned; receives the shader clocks that each wave
//             spent on its iters * 16 reads.
//   pattern : the byte offset of lane (n16 = lane % 16, g = lane / 16) inside a 1 KB block:
//             ds_read_b128
//               0  16 lane                                   linear
//               1  64 n16 + 16 g                             piece g of row n16, rows of 64 bytes
//               2  64 n16 + 16 ((g ^ (n16 >> 1)) & 3)        the same with the pieces of a row permuted
//               3  512 (g / 2) + 32 n16 + 16 (g % 2)         two blocks of 16 rows x 32 bytes
//               100 + j  (j = 0..63)  linear, but lane 1 reads lane j's 16 bytes: no conflict if the
//                        two are served in the same pass (one address, broadcast) or j = 1, 17,
//                        33, 49 (lane 1's own banks); otherwise lane 1 collides with the lane of
//                        its pass that owns those banks
//             ds_read_b64_tr_b16
//               10 8 lane                                    linear (16 rows x 32 bytes)
//               11 64 (4g + n16/4) + 8 (n16 % 4)             the transposed operand on rows of 64 bytes
//               12 the same on rows with permuted pieces
//               200 + j  (j = 0..63)  linear, but lane 1 reads lane j's 8 bytes (own banks: j = 1, 33)
//   iters   : 1 .. 2^20.
// Returns 0, or -1 (null pointer), -2 (pattern, iters), -5 (alignment), -6 (launch refused).
// Every address stays inside the kernel's 64 KB of LDS (4 waves x 8 KB regions, offsets below
// 1024 + 7168).
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

#define PROBE_LDS __attribute__((address_space(3)))
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(2))) int i32x2;

__device__ int lane_offset(int pat, int lane)
{
    const int n16 = lane & 15, g = lane >> 4;
    if (pat >= 100 && pat < 164) return (lane == 1 ? pat - 100 : lane) * 16;
    if (pat >= 200 && pat < 264) return (lane == 1 ? pat - 200 : lane) * 8;
    switch (pat) {
    case 0: return lane * 16;
    case 1: return n16 * 64 + g * 16;
    case 2: return n16 * 64 + ((g ^ (n16 >> 1)) & 3) * 16;
    case 3: return (g >> 1) * 512 + n16 * 32 + (g & 1) * 16;
    case 10: return lane * 8;
    case 11: return (4 * g + (n16 >> 2)) * 64 + (n16 & 3) * 8;
    case 12: {
        const int row = 4 * g + (n16 >> 2), piece = (n16 & 3) >> 1;
        return row * 64 + ((piece ^ (row >> 1)) & 3) * 16 + (n16 & 1) * 8;
    }
    default: return 0;
    }
}

#define PROBE_READ8(dst, OP)                                                          \
    asm volatile(OP " %0, %1 offset:0" : "=v"(dst[0]) : "v"(addr));                   \
    asm volatile(OP " %0, %1 offset:1024" : "=v"(dst[1]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:2048" : "=v"(dst[2]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:3072" : "=v"(dst[3]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:4096" : "=v"(dst[4]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:5120" : "=v"(dst[5]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:6144" : "=v"(dst[6]) : "v"(addr));                \
    asm volatile(OP " %0, %1 offset:7168" : "=v"(dst[7]) : "v"(addr));

template <bool TR>
__global__ __launch_bounds__(256)
void lds_probe_kernel(long long* __restrict__ clocks, int pat, int iters)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    PROBE_LDS unsigned char* smem = (PROBE_LDS unsigned char*)smem_raw;
    for (int i = threadIdx.x; i < 65536 / 16; i += 256) ((PROBE_LDS i32x4*)smem)[i] = i32x4{i, i, i, i};
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const uint32_t addr = (uint32_t)(uintptr_t)smem + wave * 8192 + lane_offset(pat, lane);
    i32x4 acc = {0, 0, 0, 0};
    i32x4 ra[8], rb[8];
    i32x2 qa[8], qb[8];
    const long long t0 = clock64();
    if constexpr (!TR) { PROBE_READ8(ra, "ds_read_b128") } else { PROBE_READ8(qa, "ds_read_b64_tr_b16") }
    for (int it = 0; it < iters; ++it) {
        // eight more in flight, then wait for the eight before them
        if constexpr (!TR) { PROBE_READ8(rb, "ds_read_b128") } else { PROBE_READ8(qb, "ds_read_b64_tr_b16") }
        asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (!TR) acc ^= ra[i];
            else { acc[0] ^= qa[i][0]; acc[1] ^= qa[i][1]; }
        }
        if constexpr (!TR) { PROBE_READ8(ra, "ds_read_b128") } else { PROBE_READ8(qa, "ds_read_b64_tr_b16") }
        asm volatile("s_waitcnt lgkmcnt(8)" ::: "memory");
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if constexpr (!TR) acc ^= rb[i];
            else { acc[0] ^= qb[i][0]; acc[1] ^= qb[i][1]; }
        }
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if constexpr (!TR) acc ^= ra[i];
        else { acc[0] ^= qa[i][0]; acc[1] ^= qa[i][1]; }
    }
    const long long t1 = clock64();
    if (lane == 0) clocks[wave] = t1 - t0;
    if (acc[0] == 0x7fffffff && acc[1] == 12345) clocks[0] = 0;   // keeps the reads alive; never true in practice
}

}  // namespace

extern "C" int bench_lds_probe(long long* clocks, int pattern, int iters, void* stream)
{
    if (!clocks) return -1;
    const bool b128 = (pattern >= 0 && pattern <= 3) || (pattern >= 100 && pattern < 164);
    const bool tr64 = (pattern >= 10 && pattern <= 12) || (pattern >= 200 && pattern < 264);
    if ((!b128 && !tr64) || iters <= 0 || iters > (1 << 20)) return -2;
    if ((uintptr_t)clocks & 7) return -5;
    hipStream_t st = (hipStream_t)stream;
    if (b128) {
        if (hipFuncSetAttribute((const void*)lds_probe_kernel<false>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess)
            return -6;
        hipLaunchKernelGGL(lds_probe_kernel<false>, dim3(1), dim3(256), 65536, st, clocks, pattern, iters);
    } else {
        if (hipFuncSetAttribute((const void*)lds_probe_kernel<true>, hipFuncAttributeMaxDynamicSharedMemorySize, 65536) != hipSuccess)
            return -6;
        hipLaunchKernelGGL(lds_probe_kernel<true>, dim3(1), dim3(256), 65536, st, clocks, pattern, iters);
    }
    return hipGetLastError() == hipSuccess ? 0 : -6;
}
