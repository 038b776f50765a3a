// Device code for spherical attention forward on gfx950 (CDNA4, 64-wide wavefronts).
//
// One workgroup = 4 wavefronts (one per SIMD) = one tile of BR = 4*32*QB query rows
// of one (b,h).  The key axis is streamed in tiles of 64 rows (Theorem 1: the query
// axis is partitioned, the key axis is streamed); the only state carried between key
// tiles is the pair (o, z) of Lemma 1, held in fp32 registers:
//
//     o_i += sum_j s_ij * v_j        z_i += sum_j s_ij^2        tail: O_i = o_i / sqrt(z_i)
//
// Matrix-core mapping.  Scores are produced TRANSPOSED, S^T = K Q^T, with a 32x32
// MFMA (A = 32 keys x k, B = k x 32 queries).  In the accumulator layout of the
// 32x32 instructions lane l owns query column (l & 31) and, in register 4g+t, key
// row 8g + 4(l>>5) + t.  Eight consecutive accumulator registers are therefore
// exactly one B operand (8 k-slots of one query column) of the second contraction
// O^T += V^T P^T (v_mfma_f32_32x32x16_bf16), so the scores never leave their
// registers: they are squared and summed into z in place (plain fp32 FMAs), rounded
// to bf16 in place, and fed straight back to the matrix cores.  The A operand V^T
// comes from the row-major V tile in LDS through the transposing read
// ds_read_b64_tr_b16.  z is a per-lane partial sum; the two lanes that share a
// query (l and l^32) are combined once, in the tail.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sphattn {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;

#define SPH_LDS __attribute__((address_space(3)))

constexpr int kWaves = 4;          // wavefronts per workgroup, one per SIMD
constexpr int kThreads = 64 * kWaves;
constexpr int kXcds = 8;           // accelerator complex dies, each with its own L2
constexpr int kBC = 64;            // key rows per LDS tile
constexpr int kNBuf = 4;           // LDS tile buffers in rotation

// Normalizers N(x)_i = a1(x_i) / b(sum_j a2(x_j)) of Appendix A.1, Definition 2:
//   Spherical (x, x^2, sqrt)   Softmax (exp, exp, id; with running maximum)
//   L1 (x, |x|, id)            SqRelu (relu(x)^2, relu(x)^2, id)
enum class Norm { Spherical, Softmax, L1, SqRelu };
// Storage: Bf16 = Q,K,V,O bfloat16; Fp8 = Q,K OCP E4M3 with V,O bfloat16; F16 = Q,K,V,O IEEE half
// (the paper's own precision).  The 16-bit type of V and O is also the type P is rounded to.
enum class QKType { Bf16, Fp8, F16 };

// Workgroup ids are dealt round-robin to the 8 XCDs.  Remap so that each XCD
// works through a contiguous range of (head, query-tile) pairs: the query tiles
// that run together on one XCD then stream the same K/V through one L2.
__device__ __forceinline__ int xcd_contiguous_id(int wg, int n_wg)
{
    int xcd = wg % kXcds, idx = wg / kXcds;
    int base = n_wg / kXcds, rem = n_wg % kXcds;
    int start = xcd * base + (xcd < rem ? xcd : rem);
    return start + idx;
}

// LDS rows are padded instead of swizzled, so that every fragment address is one per-lane
// register plus an instruction immediate:
//   K rows: +16 bytes.  16 lanes reading the same column of 16 consecutive rows (the
//           matrix-core A-operand pattern, ds_read_b128) then hit 16 different 16-byte groups
//           of the 256-byte LDS line.
//   V rows: +64 bytes.  The 16 lanes of a transposing-read block touch 4 consecutive rows x
//           32 bytes; consecutive rows land in different 64-byte groups.
constexpr int kKPad = 16;
constexpr int kVPad = 64;

__device__ __forceinline__ i32x4 lds_read_b128(const SPH_LDS unsigned char* p)
{
    return *reinterpret_cast<const SPH_LDS i32x4*>(p);
}

typedef __attribute__((ext_vector_type(2))) int i32x2;

// ds_read_b64_tr_b16: each lane supplies the address of 4 consecutive 16-bit elements; within
// every block of 16 lanes the 16 x 4 elements are transposed, so lane i receives element (i & 3)
// of the pieces supplied by lanes (i >> 2), 4 + (i >> 2), 8 + (i >> 2), 12 + (i >> 2).
__device__ __forceinline__ i32x2 lds_read_tr64(const SPH_LDS unsigned char* p)
{
    s16x4 v = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (SPH_LDS s16x4*)const_cast<SPH_LDS unsigned char*>(p));
    return __builtin_bit_cast(i32x2, v);
}

// Two fp32 values rounded (to nearest even) and packed into one register of the 16-bit type.
template <bool HALF>
__device__ __forceinline__ int pack2(float a, float b)
{
    f32x2 v = {a, b};
    if constexpr (HALF) return __builtin_bit_cast(int, __builtin_convertvector(v, f16x2));   // v_cvt_pk_f16_f32
    else return __builtin_bit_cast(int, __builtin_convertvector(v, bf16x2));                 // v_cvt_pk_bf16_f32
}

// D = A(32 x 16) B(16 x 32) + C on 16-bit operands held as 4 raw registers each.
template <bool HALF>
__device__ __forceinline__ f32x16 mfma16(i32x4 a, i32x4 b, f32x16 c)
{
    if constexpr (HALF)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32 lanes
// of its second.  Fed two copies of x it leaves x[lane & 31] in the first and
// x[32 + (lane & 31)] in the second register of every lane: one instruction, no LDS traffic.
// Written as inline assembly (with the wait states the instruction needs around it) because
// the compiler builtin hands back the same register for both results.
struct HalfPair { float lo, hi; };
__device__ __forceinline__ HalfPair both_halves(float x)
{
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    return HalfPair{a, b};
}

__device__ __forceinline__ float max_across_halves(float x)
{
    const HalfPair r = both_halves(x);
    return fmaxf(r.lo, r.hi);
}

__device__ __forceinline__ float sum_across_halves(float x)
{
    const HalfPair r = both_halves(x);
    return r.lo + r.hi;
}

__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_rsrc(const void* base, uint32_t bytes)
{
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, bytes, 0x00020000);
}

// ---------------------------------------------------------------------------
// Software-pipelined forward kernel: 16-bit V/O (bf16 or fp16); Q/K in the same type or OCP E4M3.
//
// The key axis advances in sub-steps of 32 keys.  Three stages of three
// consecutive sub-steps are in flight at once in every wavefront, so that the
// matrix pipe, the vector ALU and the LDS all stay busy with one wave per SIMD:
//     A(t+1)  S^T = K Q^T            matrix cores -> score registers (next)
//     B(t)    normaliser on scores   plain VALU on score registers (current)
//                spherical: z += s^2, P = bf16(s)   (no exp, no max, no rescale)
//                SoftMax twin: running max, exp2, running sum, rescale factor
//     C(t-1)  O^T += V^T P^T         matrix cores <- P registers (previous)
// A sub-step is cut into SLOTS slots (one V^T fragment each); LDS fragment reads
// run PD slots ahead of their use, across sub-step and tile boundaries.  K/V
// tiles of 64 keys rotate through four LDS buffers: in iteration j tiles j and
// j+1 feed stage A, tiles j-1 and j feed stage C, tile j+2 is written and tile
// j+3 is on its way from HBM/L2 into registers, with one workgroup barrier per
// tile.  Global loads go through buffer descriptors whose range check returns
// zeros past the end of the head: a zero key contributes nothing to o or z, so
// ragged N needs no masking in the spherical case.
// ---------------------------------------------------------------------------
// Gene-regulatory-network options (paper, Section 3.1; Appendix A.2): MULT multiplies the
// score of key j by that gene's multiplicity mult[b, j] (the key row scaled by a scalar, applied
// to the fp32 score before it is squared and rounded); kv_group query heads share one K/V head.
//
// Shapes: Q and O have Nq rows per head, K and V have Nk.  Zv, when not null, receives z_i.
// PARTIAL (Lemma 1 without the tail): the key axis is cut into n_splits slices of
// keys_per_split rows (a multiple of the tile) and a workgroup accumulates one slice only; it
// writes the unnormalised fp32 pair, o to Ov[split][b,h,i,:] and z to Zv[split][b,h,i].
// Because the accumulator is a plain sum, the slices are added afterwards (combine_kernel)
// and the tail is applied once.
template <int D, int QB, QKType QKT, Norm NORM, bool MULT, bool PARTIAL = false>
__global__ __launch_bounds__(kThreads, 1)
void fwd_pipelined_kernel(const void* __restrict__ Qv, const void* __restrict__ Kv,
                          const void* __restrict__ Vv, void* __restrict__ Ov,
                          const float* __restrict__ mult, float* __restrict__ Zv,
                          int Nq, int Nk, int H, int kv_group, int n_qtiles, int n_wg,
                          int n_splits, int keys_per_split, float scale_log2)
{
    constexpr bool FP8 = QKT == QKType::Fp8;
    constexpr bool HALF = QKT == QKType::F16;      // 16-bit type of V, O and P
    constexpr int BC = kBC;
    constexpr int BR = kWaves * 32 * QB;
    constexpr int EQ = FP8 ? 1 : 2;                // bytes per Q/K element
    constexpr int KROWB = D * EQ, KCH = KROWB / 16, KTILE = BC * KROWB;   // as stored in HBM
    constexpr int VROWB = D * 2, VCH = VROWB / 16, VTILE = BC * VROWB;
    constexpr int KSTR = KROWB + kKPad, VSTR = VROWB + kVPad;             // LDS row strides
    constexpr int KLDS = BC * KSTR;                                        // K tile in LDS
    constexpr int BUF_BYTES = KLDS + BC * VSTR;    // K tile then V tile
    constexpr int LDK = BC * KCH / kThreads;       // 16-byte chunks per thread per K tile
    constexpr int LDV = BC * VCH / kThreads;
    constexpr int NST = LDK + LDV;                 // staged chunks per thread per tile
    constexpr int DB = D / 32;
    constexpr int SLOTS = 2 * DB;                  // slots per sub-step: one V^T fragment each
    constexpr int KSTEPS = FP8 ? D / 64 : D / 16;  // MFMA k-steps of K Q^T
    constexpr int PD = 3;                          // LDS prefetch distance in slots
    constexpr int RING = 4;                        // fragment registers in rotation
    constexpr int VALU_PER_MFMA = 6;               // VALU instructions issued behind each MFMA (measured best of 2..6)
    static_assert(D == 64 || D == 128, "head dimension 128 or 64");
    static_assert(FP8 || KSTEPS == SLOTS, "bf16: one K fragment per slot");
    static_assert(!FP8 || QB == 2, "fp8 slot plan is written for two query blocks");
    static_assert(NST <= SLOTS, "one staged chunk per slot of the second half");
    static_assert((2 * SLOTS) % RING == 0 && PD < RING && PD <= SLOTS, "ring indices must repeat");
    static_assert(QKT == QKType::Bf16 || NORM == Norm::Spherical, "fp8 and fp16 storage: spherical only");
    static_assert(!MULT || NORM == Norm::Spherical, "multiplicities belong to the spherical variant");
    static_assert(!PARTIAL || NORM == Norm::Spherical, "partial accumulators: spherical only");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, blk = (lane >> 4) & 1;

    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    // consecutive ids: the query tiles of one (head, key slice), which stream the same K/V
    const int qt = lid % n_qtiles;
    const int split = PARTIAL ? (lid / n_qtiles) % n_splits : 0;
    const int bh = PARTIAL ? lid / (n_qtiles * n_splits) : lid / n_qtiles;
    const size_t head_off = (size_t)bh * Nq * D;   // in elements
    const int bidx = bh / H;
    const int k0 = PARTIAL ? split * keys_per_split : 0;                     // this workgroup's keys:
    const int N = PARTIAL ? min(Nk - k0, keys_per_split) : Nk;               // k0 .. k0 + N - 1
    const size_t kv_off = ((size_t)(bidx * (H / kv_group) + (bh % H) / kv_group) * Nk + k0) * D;
    const unsigned char* Qh = (const unsigned char*)Qv + head_off * EQ;
    const unsigned short* V = (const unsigned short*)Vv;
    const __amdgpu_buffer_rsrc_t krs =
        make_rsrc((const unsigned char*)Kv + kv_off * EQ, (uint32_t)N * KROWB);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc(V + kv_off, (uint32_t)N * VROWB);
    // multiplicities of this cell; reads past the last key return 0 (those keys are zero anyway)
    const __amdgpu_buffer_rsrc_t mrs =
        make_rsrc(MULT ? mult + (size_t)bidx * Nk + k0 : nullptr, MULT ? (uint32_t)N * 4 : 0);
    const int q0 = qt * BR + wave * 32 * QB;

    // ---- per-lane LDS byte offsets inside a tile; everything else is an immediate
    // K fragment, bf16 (sub, kk): row sub*32 + l32, bytes 32kk + 16h .. +15
    // K fragment, fp8  (sub, kk): row sub*32 + l32, bytes 64kk + 32h .. +31 (two 16-byte reads)
    const int klane = l32 * KSTR + (FP8 ? 32 : 16) * h;
    // V^T fragment (sub, ks, db): rows sub*32 + 16ks + 4h + (i16>>2) [+8], 8 bytes at column
    // db*32 + 16*blk + 4*(i16&3).  Within a 16-lane block, lane i supplies the 8-byte piece
    // row (i>>2), columns 4(i&3)..+3 and receives column i of all 4 rows.
    const int vlane = KLDS + (4 * h + (i16 >> 2)) * VSTR + (16 * blk + 4 * (i16 & 3)) * 2;
    // staging: chunks 0..LDK-1 are K, LDK..NST-1 are V; chunk id = tid + i*256 of its tile,
    // i.e. row tid/CH + i*(256/CH), 16-byte column tid%CH
    const int kst_lane = (tid / KCH) * KSTR + (tid % KCH) * 16;
    const int vst_lane = KLDS + (tid / VCH) * VSTR + (tid % VCH) * 16;
    const int kld_lane = tid * 16, vld_lane = tid * 16;      // tiles are contiguous in HBM

    // ---- Q fragments (B operands of S^T = K Q^T), held for the whole kernel.  The k index
    // that a (lane half, element) slot stands for is the same for A and B operands, so any
    // split of the head dimension over slots is valid as long as Q and K use the same one.
    constexpr int QREGS = FP8 ? 8 : 4;
    typedef __attribute__((ext_vector_type(QREGS))) int qfrag_t;
    qfrag_t qf[QB][KSTEPS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + l32;
        row = row < Nq ? row : Nq - 1;             // rows past the end are computed and dropped
        const unsigned char* src = Qh + (size_t)row * KROWB + (FP8 ? 32 : 16) * h;
#pragma unroll
        for (int kk = 0; kk < KSTEPS; ++kk) {
            if constexpr (FP8) {
                const i32x4 lo = *reinterpret_cast<const i32x4*>(src + kk * 64);
                const i32x4 hi = *reinterpret_cast<const i32x4*>(src + kk * 64 + 16);
                qf[qb][kk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                qf[qb][kk] = *reinterpret_cast<const i32x4*>(src + kk * 32);
            }
        }
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
    // spherical: zacc = per-lane partial sums of s^2 (two chains per query block)
    // SoftMax:   zacc[qb][0] = per-lane partial denominator, zacc[qb][1] = exponent offset of
    //            the current sub-step, mrun = running max of raw scores, apend = factor that
    //            o still has to be multiplied with before the next stage C
    float zacc[QB][2], mrun[QB], apend[QB], anext[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        zacc[qb][0] = zacc[qb][1] = 0.f;
        mrun[qb] = -INFINITY;
        apend[qb] = anext[qb] = 1.f;
    }

    // multipliers of the lane's 16 keys (8g + 4h + t) of a sub-step, double-buffered by parity
    f32x4 mreg[MULT ? 2 : 1][4];
    auto mload = [&](int par, int g, int substep) {
        if constexpr (MULT)
            mreg[par][g] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
                mrs, (8 * g + 4 * h) * 4, substep * 128, 0));
    };

    i32x4 stage[NST];
    auto gload_chunk = [&](int c, int tile) {
        if (c < LDK)
            stage[c] = __builtin_amdgcn_raw_buffer_load_b128(krs, kld_lane, tile * KTILE + c * kThreads * 16, 0);
        else
            stage[c] = __builtin_amdgcn_raw_buffer_load_b128(vrs, vld_lane, tile * VTILE + (c - LDK) * kThreads * 16, 0);
    };
    auto lstore_chunk = [&](int c, SPH_LDS unsigned char* buf) {
        const int off = c < LDK ? kst_lane + c * (kThreads / KCH) * KSTR
                                : vst_lane + (c - LDK) * (kThreads / VCH) * VSTR;
        *reinterpret_cast<SPH_LDS i32x4*>(buf + off) = stage[c];
    };

    const int n_tiles = (N + BC - 1) / BC;

    // ---- prologue: buffer 3 plays "tile -1" (zeros) for the first stage C; tiles 0 and 1 go
    // to buffers 0 and 1; tile 2 waits in registers
    {
        const i32x4 zero4 = {0, 0, 0, 0};
        for (int i = tid; i < BUF_BYTES / 16; i += kThreads)
            *reinterpret_cast<SPH_LDS i32x4*>(smem + 3 * BUF_BYTES + i * 16) = zero4;
    }
    {   // all three tiles are requested before the first is waited for: one memory latency
        i32x4 first[2][NST];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < NST; ++c) { gload_chunk(c, t); first[t][c] = stage[c]; }
#pragma unroll
        for (int c = 0; c < NST; ++c) gload_chunk(c, 2);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < NST; ++c) {
                const i32x4 keep = stage[c];
                stage[c] = first[t][c];
                lstore_chunk(c, smem + t * BUF_BYTES);
                stage[c] = keep;
            }
    }
#pragma unroll
    for (int g = 0; g < 4; ++g) mload(0, g, 0);
    __syncthreads();

    f32x16 S0[QB], S1[QB];
    i32x4 P0[QB][2], P1[QB][2];                    // P of a sub-step: two B operands per query block
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
#pragma unroll
        for (int r = 0; r < 16; ++r) { S0[qb][r] = 0.f; S1[qb][r] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) { P0[qb][ks] = i32x4{0, 0, 0, 0}; P1[qb][ks] = i32x4{0, 0, 0, 0}; }
    }

    auto mfma_qk = [&](qfrag_t a, qfrag_t b, f32x16 c) -> f32x16 {
        if constexpr (FP8)
            return __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
        else
            return mfma16<HALF>(a, b, c);
    };

    // S0 = scores of sub-step 0
#pragma unroll
    for (int kk = 0; kk < KSTEPS; ++kk) {
        qfrag_t kfr;
        if constexpr (FP8) {
            const i32x4 lo = lds_read_b128(smem + klane + 64 * kk);
            const i32x4 hi = lds_read_b128(smem + klane + 64 * kk + 16);
            kfr = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            kfr = lds_read_b128(smem + klane + 32 * kk);
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) S0[qb] = mfma_qk(kfr, qf[qb][kk], S0[qb]);
    }

    // Fragment registers.  bf16: one K fragment per slot, in a ring.  fp8: the K fragment of
    // k-step kk arrives as two 16-byte halves aimed at slots 2*QB*kk and 2*QB*kk+1 and is used
    // in the odd slots that follow; two sets alternate between consecutive sub-steps.
    i32x4 kf[FP8 ? 1 : RING];
    i32x4 kf8[FP8 ? 2 : 1][FP8 ? KSTEPS : 1][2];
    i32x4 vf[RING];
    // Reads for slot u of an iteration whose tiles j-1, j, j+1 sit at bprv, bcur, bnxt:
    //   u in [0,SLOTS)        first half : K_j sub 1,     V_{j-1} sub 1
    //   u in [SLOTS,2SLOTS)   second half: K_{j+1} sub 0, V_j sub 0
    //   u >= 2SLOTS           next iteration's first half: K_{j+1} sub 1, V_j sub 1
    auto issue_reads = [&](int u, const SPH_LDS unsigned char* bprv, const SPH_LDS unsigned char* bcur,
                           const SPH_LDS unsigned char* bnxt) {
        const int hh = u / SLOTS, i = u % SLOTS;
        const SPH_LDS unsigned char* kp = hh == 0 ? bcur + 32 * KSTR : hh == 1 ? bnxt : bnxt + 32 * KSTR;
        const SPH_LDS unsigned char* vp = hh == 0 ? bprv + 32 * VSTR : hh == 1 ? bcur : bcur + 32 * VSTR;
        // V first, K last: LDS returns in order, so the one wait in front of the slot's first
        // matrix instruction (which needs K) covers all three reads
        const int ks = i / DB, db = i % DB;
        const SPH_LDS unsigned char* a = vp + vlane + (16 * ks) * VSTR + db * 64;
        const i32x2 lo = lds_read_tr64(a);
        const i32x2 hi = lds_read_tr64(a + 8 * VSTR);
        vf[u % RING] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
        if constexpr (FP8) {
            const int kk = i / (2 * QB), part = i % (2 * QB);
            if (kk < KSTEPS && part < 2) kf8[hh & 1][kk][part] = lds_read_b128(kp + klane + 64 * kk + 16 * part);
        } else {
            kf[u % RING] = lds_read_b128(kp + klane + 32 * i);
        }
    };

    // buffers of tiles j-1, j, j+1, j+2
    SPH_LDS unsigned char* bprv = smem + 3 * BUF_BYTES;
    SPH_LDS unsigned char* bcur = smem;
    SPH_LDS unsigned char* bnxt = smem + BUF_BYTES;
    SPH_LDS unsigned char* bnn = smem + 2 * BUF_BYTES;
#pragma unroll
    for (int u = 0; u < PD; ++u) issue_reads(u, bprv, bcur, bnxt);

    for (int j = 0; j < n_tiles; ++j) {
#pragma unroll
        for (int s = 0; s < 2 * SLOTS; ++s) {
            const int hf = s / SLOTS, i = s % SLOTS;
            f32x16 (&Sn)[QB] = hf == 0 ? S1 : S0;
            f32x16 (&Sc)[QB] = hf == 0 ? S0 : S1;
            i32x4 (&Pc)[QB][2] = hf == 0 ? P0 : P1;
            i32x4 (&Pp)[QB][2] = hf == 0 ? P1 : P0;
            __builtin_amdgcn_sched_barrier(0);
            // The one barrier per tile.  Tile j+1, written to LDS during the previous
            // iteration, becomes visible before its first read (the prefetch below); and
            // every wave has finished the previous iteration, whose first half was the last
            // reader of the buffer that this iteration's second half overwrites.
            if (s == SLOTS - PD) {
                // LDS operations complete in issue order.  At least OUT of them have been
                // issued since this wave's last staging write of the previous iteration, so
                // once no more than OUT are outstanding that write has landed.  No full
                // drain: the fragment reads already in flight keep flying across the barrier.
                constexpr int NRD = FP8 ? 2 : 3;   // LDS reads per slot, at least
                constexpr int OUT = NRD * (SLOTS - PD) < 15 ? NRD * (SLOTS - PD) : 15;
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F | (OUT << 8));
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            issue_reads(s + PD, bprv, bcur, bnxt);

            // SoftMax twin: o must carry the factor from the previous sub-step's new maximum
            // before stage C adds to it; skipped when no lane's maximum moved.
            if constexpr (NORM == Norm::Softmax) {
                if (i < DB) {
                    bool moved = false;
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) moved |= apend[qb] != 1.f;
                    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                            for (int r = 0; r < 16; ++r) oacc[i][qb][r] *= apend[qb];
                    }
                }
            }

            // A: next sub-step's scores
            if constexpr (FP8) {
                if (i & 1) {
                    const int idx = i / 2, kk = idx / QB, qb = idx % QB;
                    if (kk < KSTEPS) {
                        const qfrag_t kfr = __builtin_shufflevector(kf8[hf][kk][0], kf8[hf][kk][1],
                                                                    0, 1, 2, 3, 4, 5, 6, 7);
                        f32x16 zero = {0};
                        Sn[qb] = mfma_qk(kfr, qf[qb][kk], kk == 0 ? zero : Sn[qb]);
                    }
                }
            } else {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    f32x16 zero = {0};
                    Sn[qb] = mfma_qk(kf[s % RING], qf[qb][i], i == 0 ? zero : Sn[qb]);
                }
            }
            // C: V^T fragment i against the previous sub-step's P
            {
                const int ks = i / DB, db = i % DB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[db][qb] = mfma16<HALF>(vf[s % RING], Pp[qb][ks], oacc[db][qb]);
            }
            // B: a slice of the current sub-step's scores, 16*QB/SLOTS registers per slot
            constexpr int PER = 16 * QB / SLOTS;
            if constexpr (NORM != Norm::Softmax) {
#pragma unroll
                for (int u = 0; u < PER; u += 2) {
                    const int idx = i * PER + u;
                    const int qb = idx / 16, r = idx % 16;
                    float a = Sc[qb][r], b = Sc[qb][r + 1];
                    if constexpr (MULT) {
                        a *= mreg[hf][r / 4][r % 4];
                        b *= mreg[hf][r / 4][r % 4 + 1];
                    }
                    if constexpr (NORM == Norm::Spherical) {        // a2 = x^2, a1 = x
                        zacc[qb][0] = __builtin_fmaf(a, a, zacc[qb][0]);
                        zacc[qb][1] = __builtin_fmaf(b, b, zacc[qb][1]);
                    } else if constexpr (NORM == Norm::L1) {        // a2 = |x|, a1 = x
                        zacc[qb][0] += __builtin_fabsf(a);
                        zacc[qb][1] += __builtin_fabsf(b);
                    } else {                                         // a1 = a2 = relu(x)^2
                        a = fmaxf(a, 0.f);
                        b = fmaxf(b, 0.f);
                        a *= a;
                        b *= b;
                        zacc[qb][0] += a;
                        zacc[qb][1] += b;
                    }
                    Pc[qb][r / 8][(r % 8) / 2] = pack2<HALF>(a, b);
                }
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)     // keep the running sums where they were computed
                    asm volatile("" : "+v"(zacc[qb][0]), "+v"(zacc[qb][1]));
            } else {
                if (i == 0) {
                    // keys past N (ragged last tile only) must not take part in the SoftMax
                    const int key0 = (2 * j + hf) * 32;      // first key of the current sub-step
                    if (key0 + 32 > N) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                            for (int r = 0; r < 16; ++r)
                                if (key0 + 8 * (r >> 2) + 4 * h + (r & 3) >= N) Sc[qb][r] = -INFINITY;
                    }
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) {
                        float mx = Sc[qb][0];
#pragma unroll
                        for (int r = 1; r < 16; ++r) mx = fmaxf(mx, Sc[qb][r]);
                        mx = max_across_halves(mx);
                        const float mnew = fmaxf(mrun[qb], mx);
                        anext[qb] = __builtin_amdgcn_exp2f((mrun[qb] - mnew) * scale_log2);
                        mrun[qb] = mnew;
                        zacc[qb][0] *= anext[qb];
                        zacc[qb][1] = -mnew * scale_log2;    // offset of this sub-step's exponents
                    }
                }
#pragma unroll
                for (int u = 0; u < PER; u += 2) {
                    const int idx = i * PER + u;
                    const int qb = idx / 16, r = idx % 16;
                    const float a = __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[qb][r], scale_log2, zacc[qb][1]));
                    const float b = __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[qb][r + 1], scale_log2, zacc[qb][1]));
                    zacc[qb][0] += a + b;
                    Pc[qb][r / 8][(r % 8) / 2] = pack2<HALF>(a, b);
                }
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    asm volatile("" : "+v"(zacc[qb][0]));
                if (i == SLOTS - 1) {
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) apend[qb] = anext[qb];
                }
            }
            if (MULT && i < 4) mload(hf ^ 1, i, 2 * j + hf + 1);
            // staging, second half only: tile j+2 into LDS, tile j+3 out of HBM/L2
            if (hf == 1 && i < NST) {
                lstore_chunk(i, bnn);
                gload_chunk(i, j + 3);
            }
            // issue order inside the slot: after each matrix instruction, one LDS read and a
            // few VALU instructions, so that the matrix pipe never waits on the issue port
            if constexpr (NORM != Norm::Softmax) {
                constexpr int NM = FP8 ? QB + 1 : 2 * QB;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
                    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);   // VALU
                    if (hf == 1 && m == NM - 2) __builtin_amdgcn_sched_group_barrier(0x200, 1, 0);   // DS write
                    if (hf == 1 && m == NM - 1) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read
                }
            }
        }
        SPH_LDS unsigned char* t = bprv; bprv = bcur; bcur = bnxt; bnxt = bnn; bnn = t;
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- drain: stage C of the last sub-step (V of the last tile, sub 1, now at bprv)
    {
        if constexpr (NORM == Norm::Softmax) {
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= apend[qb];
        }
        const SPH_LDS unsigned char* vp = bprv + 32 * VSTR;
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const int ks = i / DB, db = i % DB;
            const SPH_LDS unsigned char* a = vp + vlane + (16 * ks) * VSTR + db * 64;
            const i32x2 lo = lds_read_tr64(a);
            const i32x2 hi = lds_read_tr64(a + 8 * VSTR);
            const i32x4 vfr = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                oacc[db][qb] = mfma16<HALF>(vfr, P1[qb][ks], oacc[db][qb]);
        }
    }

    // ---- partial result: the pair (o, z) as it stands, in fp32
    if constexpr (PARTIAL) {
        const size_t rows0 = ((size_t)split * (n_wg / (n_qtiles * n_splits)) + bh) * Nq;
        float* Op = (float*)Ov + rows0 * D;
        float* Zp = Zv + rows0;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float z = sum_across_halves(zacc[qb][0] + zacc[qb][1]);
            const int row = q0 + qb * 32 + l32;
            if (row < Nq) {
                if (h == 0) Zp[row] = z;
                float* dst = Op + (size_t)row * D + 4 * h;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        const f32x4 o4 = {oacc[db][qb][4 * g], oacc[db][qb][4 * g + 1],
                                          oacc[db][qb][4 * g + 2], oacc[db][qb][4 * g + 3]};
                        *reinterpret_cast<f32x4*>(dst + db * 32 + 8 * g) = o4;
                    }
            }
        }
        return;
    }

    // ---- tail t(o, z) = o / b(z): spherical b = sqrt, the others b = id
    unsigned short* Oh = (unsigned short*)Ov + head_off;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float inv, z;
        if constexpr (NORM == Norm::Spherical) {
            z = sum_across_halves(zacc[qb][0] + zacc[qb][1]);
            inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        } else if constexpr (NORM == Norm::Softmax) {
            z = sum_across_halves(zacc[qb][0]);
            inv = 1.0f / z;
        } else {
            z = sum_across_halves(zacc[qb][0] + zacc[qb][1]);
            inv = z > 0.f ? 1.0f / z : 0.f;
        }
        const int row = q0 + qb * 32 + l32;
        if (row < Nq) {
            if (Zv != nullptr && h == 0) Zv[(size_t)bh * Nq + row] = z;
            unsigned short* dst = Oh + (size_t)row * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const i32x2 o4 = {pack2<HALF>(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv),
                                      pack2<HALF>(oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv)};
                    *reinterpret_cast<i32x2*>(dst + db * 32 + 8 * g) = o4;
                }
        }
    }
}

// ---------------------------------------------------------------------------
// fp32 Q/K/V/O kernel on the fp32 matrix instruction v_mfma_f32_32x32x2_f32.
// Same mapping as above with k = 2 per instruction: lane l holds row/column
// (l & 31) and k index (l >> 5), so accumulator register 4g+t of S^T (key
// 8g + 4h + t) is directly the B operand of the k-step that pairs it with the
// V row of that key; V needs no transpose (one scalar per lane).
//
// fp32 problems are small and latency-bound, so the work is cut for parallelism
// rather than for reuse: a workgroup owns 32 query rows, and its four wavefronts
// split the KEY axis (wave w takes key tiles w, w+4, ...), each carrying its own
// partial (o, z).  Lemma 1's accumulator is a plain sum, so the four partials are
// simply added (through LDS) before the tail o / sqrt(z) is applied once.  Each
// wave stages its tiles in a private LDS region; there is no workgroup barrier in
// the loop.
// ---------------------------------------------------------------------------
// Nq, Nk, Zv, PARTIAL, n_splits and keys_per_split as in fwd_pipelined_kernel.
template <int D, bool MULT, bool PARTIAL = false>
__global__ __launch_bounds__(kThreads, 1)
void fwd_f32_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                    const float* __restrict__ V, float* __restrict__ O,
                    const float* __restrict__ mult, float* __restrict__ Zv,
                    int Nq, int Nk, int H, int kv_group, int n_qtiles, int n_wg,
                    int n_splits, int keys_per_split)
{
    constexpr int BC = 32;                         // keys per tile
    constexpr int ROWF = D + 4;                    // padded row, in floats: conflict-free columns
    constexpr int TILE_F = BC * ROWF;
    constexpr int WAVE_F = 2 * TILE_F;             // K tile then V tile, private to a wave
    constexpr int DB = D / 32;
    constexpr int LD = BC * D / 4 / 64;            // float4 loads per lane per tensor per tile
    static_assert(kWaves * (DB * 16 + 1) * 64 <= kWaves * WAVE_F, "partials fit the staging space");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS float* smem = (SPH_LDS float*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int qt = lid % n_qtiles;
    const int split = PARTIAL ? (lid / n_qtiles) % n_splits : 0;
    const int bh = PARTIAL ? lid / (n_qtiles * n_splits) : lid / n_qtiles;
    const size_t head_off = (size_t)bh * Nq * D;
    const int bidx = bh / H;
    const int k0 = PARTIAL ? split * keys_per_split : 0;
    const int N = PARTIAL ? min(Nk - k0, keys_per_split) : Nk;      // keys k0 .. k0 + N - 1
    const size_t kv_off = ((size_t)(bidx * (H / kv_group) + (bh % H) / kv_group) * Nk + k0) * D;
    const float* Qh = Q + head_off;
    const float* Kh = K + kv_off;
    const float* Vh = V + kv_off;
    const float* mrow = MULT ? mult + (size_t)bidx * Nk + k0 : nullptr;
    const int q0 = qt * 32;

    // Q as B operand of S^T = K Q^T: lane holds Q[q0 + l32][2kk + h]
    float qf[D / 2];
    {
        int row = q0 + l32;
        row = row < Nq ? row : Nq - 1;
#pragma unroll
        for (int kk = 0; kk < D / 2; ++kk) qf[kk] = Qh[(size_t)row * D + 2 * kk + h];
    }
    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float z = 0.f;

    SPH_LDS float* kb = smem + wave * WAVE_F;
    SPH_LDS float* vb = kb + TILE_F;
    f32x4 kreg[LD], vreg[LD];
    auto load_tile = [&](int j0) {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int id = lane + i * 64;
            const int r = id / (D / 4), c = id % (D / 4);
            if (j0 + r < N) {
                kreg[i] = *reinterpret_cast<const f32x4*>(Kh + (size_t)(j0 + r) * D + 4 * c);
                vreg[i] = *reinterpret_cast<const f32x4*>(Vh + (size_t)(j0 + r) * D + 4 * c);
            } else {                               // zero keys add nothing to o or z
                kreg[i] = f32x4{0, 0, 0, 0};
                vreg[i] = f32x4{0, 0, 0, 0};
            }
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int i = 0; i < LD; ++i) {
            const int id = lane + i * 64;
            const int r = id / (D / 4), c = id % (D / 4);
            *reinterpret_cast<SPH_LDS f32x4*>(kb + r * ROWF + 4 * c) = kreg[i];
            *reinterpret_cast<SPH_LDS f32x4*>(vb + r * ROWF + 4 * c) = vreg[i];
        }
    };

    const int n_tiles = (N + BC - 1) / BC;
    if (wave < n_tiles) load_tile(wave * BC);
    for (int jt = wave; jt < n_tiles; jt += kWaves) {
        // LDS executes one wave's operations in order: the reads of the previous tile are done
        // before these writes land, and the reads below see them
        store_tile();
        if (jt + kWaves < n_tiles) load_tile((jt + kWaves) * BC);
        // S^T (32 keys x 32 queries)
        f32x16 s;
#pragma unroll
        for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 2; ++kk)
            s = __builtin_amdgcn_mfma_f32_32x32x2f32(kb[l32 * ROWF + 2 * kk + h], qf[kk], s, 0, 0, 0);
        if constexpr (MULT) {                    // s_ij = m_j (q_i . k_j); keys past N are zero
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = jt * BC + 8 * (r >> 2) + 4 * h + (r & 3);
                s[r] *= key < N ? mrow[key] : 0.f;
            }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) z = __builtin_fmaf(s[r], s[r], z);
        // O^T (D x 32 queries) += V^T S^T: k-step r pairs key 8(r>>2) + 4h + (r&3) on both sides
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int key = 8 * (r >> 2) + 4 * h + (r & 3);
#pragma unroll
            for (int db = 0; db < DB; ++db)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x2f32(vb[key * ROWF + db * 32 + l32], s[r], oacc[db], 0, 0, 0);
        }
    }

    // ---- add the four waves' partial (o, z): register r of block db of wave w at
    // part[w][db*16 + r][lane], z at part[w][DB*16][lane]
    __syncthreads();                               // every wave is done with its staging space
    constexpr int PART = (DB * 16 + 1) * 64;
    SPH_LDS float* part = smem;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) part[wave * PART + (db * 16 + r) * 64 + lane] = oacc[db][r];
    part[wave * PART + DB * 16 * 64 + lane] = z;
    __syncthreads();

    // wave w finishes output block db = w (32 columns of the head dimension)
    if (wave < DB) {
        float zt = 0.f;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) zt += part[w * PART + DB * 16 * 64 + lane];
        zt = sum_across_halves(zt);
        const float inv = PARTIAL ? 1.f : zt > 0.f ? 1.0f / __builtin_sqrtf(zt) : 0.f;
        const int row = q0 + l32;
        // partial: the fp32 pair (o, z) of this key slice, slice-major
        const size_t rows0 = PARTIAL ? ((size_t)split * (n_wg / (n_qtiles * n_splits)) + bh) * Nq
                                     : (size_t)bh * Nq;
        if (wave == 0 && h == 0 && row < Nq && (PARTIAL || Zv != nullptr)) Zv[rows0 + row] = zt;
        float* dst = O + (rows0 + row) * D + wave * 32 + 4 * h;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            f32x4 o4;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float acc = 0.f;
#pragma unroll
                for (int w = 0; w < kWaves; ++w) acc += part[w * PART + (wave * 16 + 4 * g + t) * 64 + lane];
                o4[t] = acc * inv;
            }
            if (row < Nq) *reinterpret_cast<f32x4*>(dst + 8 * g) = o4;
        }
    }
}

// ---------------------------------------------------------------------------
// Adds the partial pairs (o, z) of n_parts key slices and applies the tail once
// (Lemma 1: the accumulator of a concatenation is the sum of the accumulators):
//     O[r,:] = (sum_p o_p[r,:]) / sqrt(sum_p z_p[r])        (0 if the sum of z is 0)
// rows = B*H*N query rows; part p starts rows*D floats (o) / rows floats (z) after part
// p-1.  One thread per 4 output columns; the parts are added in ascending order, so the
// result does not depend on the launch.  OUT: 0 fp32, 1 bfloat16, 2 IEEE half.
// ---------------------------------------------------------------------------
template <int D, int OUT>
__global__ __launch_bounds__(256)
void combine_kernel(const float* __restrict__ o_parts, const float* __restrict__ z_parts,
                    int n_parts, void* __restrict__ Ov, float* __restrict__ Zv, size_t rows)
{
    constexpr int C4 = D / 4;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    const size_t row = idx / C4;
    const int c4 = (int)(idx % C4);
    if (row >= rows) return;
    float z = 0.f;
    f32x4 acc = {0.f, 0.f, 0.f, 0.f};
    for (int p = 0; p < n_parts; ++p) {
        z += z_parts[(size_t)p * rows + row];
        acc += *reinterpret_cast<const f32x4*>(o_parts + ((size_t)p * rows + row) * D + 4 * c4);
    }
    const float inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
    if (Zv != nullptr && c4 == 0) Zv[row] = z;
    if constexpr (OUT == 0) {
        *reinterpret_cast<f32x4*>((float*)Ov + row * D + 4 * c4) = acc * inv;
    } else {
        const i32x2 o4 = {pack2<OUT == 2>(acc[0] * inv, acc[1] * inv), pack2<OUT == 2>(acc[2] * inv, acc[3] * inv)};
        *reinterpret_cast<i32x2*>((unsigned short*)Ov + row * D + 4 * c4) = o4;
    }
}

}  // namespace sphattn
