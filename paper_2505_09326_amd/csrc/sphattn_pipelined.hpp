// Software-pipelined forward kernel on the 16x16 matrix instructions of gfx950:
// 16-bit V/O (bf16 or fp16); Q/K in the same type or OCP E4M3.
//
// One workgroup = 4 wavefronts (one per SIMD) = one tile of BR = 4*16*NQ query rows of one
// (b,h); a wavefront owns NQ blocks of 16 query rows.  The key axis is streamed in tiles of 64
// rows (Theorem 1: the query axis is partitioned, the key axis is streamed); the only state
// carried between key tiles is the pair (o, z) of Lemma 1, held in fp32 registers:
//
//     o_i += sum_j s_ij * v_j        z_i += sum_j s_ij^2        tail: O_i = o_i / sqrt(z_i)
//
// Matrix-core mapping.  Scores are produced TRANSPOSED,
//     S^T[kb][qb] (16 keys x 16 queries) += K frag (A: 16 keys x k) * Q frag (B: k x 16 queries)
// with v_mfma_f32_16x16x32_{bf16,f16} (k = 32) or v_mfma_f32_16x16x128_f8f6f4 (k = 128, E4M3).
// In the accumulator layout of the 16x16 instructions lane l owns query column (l & 15) and, in
// register t, key row 4(l>>4) + t.  The two key blocks kb = 0, 1 of a 32-key sub-step therefore
// put 8 scores of one query into every lane, and 8 values of one column are exactly one B
// operand of the second contraction
//     O^T[db][qb] (16 columns of d x 16 queries) += V^T frag (A: 16 x 32 keys) * P^T (B: 32 keys x 16)
// where k-slot e of lane group g = l>>4 stands for key 4g + e (e < 4) or 16 + 4g + (e - 4):
// any assignment of keys to k-slots is valid as long as A and B use the same one.  So the
// scores never leave their registers: they are squared and summed into z in place (plain fp32
// FMAs), rounded to the 16-bit type in place, and fed straight back to the matrix cores.  The
// A operand V^T comes from the row-major V tile in LDS through two transposing reads
// (ds_read_b64_tr_b16: keys 4g..4g+3 and 16+4g..16+4g+3).  z is a per-lane partial sum; the
// four lanes that share a query (l, l^16, l^32, l^48) are combined once, in the tail.
//
// Why 16x16 and not 32x32 instructions: on Gaussian operands the part is power-bound, and the
// 16x16x32 form sustains about 10 % more flop/s at the power limit than 32x32x16 (measured with
// loops of nothing but matrix instructions: 1930 against 1755 TFLOP/s), which outweighs its
// lower issue efficiency with one wave per SIMD.
//
// Pipeline.  The key axis advances in sub-steps of 32 keys.  Three stages of three consecutive
// sub-steps are in flight at once in every wavefront, so that the matrix pipe, the vector ALU
// and the LDS all stay busy with one wave per SIMD:
//     A(t+1)  S^T = K Q^T            matrix cores -> score registers (next)
//     B(t)    normaliser on scores   plain VALU on score registers (current)
//                spherical: z += s^2, P = bf16(s)   (no exp, no max, no rescale)
//                SoftMax twin: running max, exp2, running sum, rescale factor
//     C(t-1)  O^T += V^T P^T         matrix cores <- P registers (previous)
// A sub-step is cut into SLOTS slots (one V^T fragment each); LDS fragment reads run PD slots
// ahead of their use, across sub-step and tile boundaries.  K/V tiles of 64 keys rotate through
// four LDS buffers: in iteration j tiles j and j+1 feed stage A, tiles j-1 and j feed stage C
// and tile j+2 is on its way from HBM/L2 straight into LDS (buffer_load ... lds, no registers
// and no LDS store instructions in between), with one workgroup barrier per tile.  Global
// loads go through buffer descriptors whose range check returns
// zeros past the end of the head: a zero key contributes nothing to o or z, so ragged N needs
// no masking in the spherical case.
//
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
#pragma once
#include "sphattn_device.hpp"

namespace sphattn {

typedef __attribute__((ext_vector_type(8))) int i32x8;

template <bool HALF>
__device__ __forceinline__ f32x4 mfma16x16(i32x4 a, i32x4 b, f32x4 c)
{
    if constexpr (HALF)
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// v_permlane16_swap exchanges the odd rows (of 16 lanes) of its first operand with the even rows
// of its second.  Fed two copies of x, every lane ends up with x of the even and of the odd row
// of its pair of rows; with both_halves() on top, a value is combined over the four lanes
// l, l^16, l^32, l^48 without LDS traffic.
__device__ __forceinline__ HalfPair both_rows(float x)
{
    float a = x, b = x;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
    return HalfPair{a, b};
}

__device__ __forceinline__ float max_across_groups(float x)
{
    const HalfPair r = both_rows(x);
    return max_across_halves(fmaxf(r.lo, r.hi));
}

__device__ __forceinline__ float sum_across_groups(float x)
{
    const HalfPair r = both_rows(x);
    return sum_across_halves(r.lo + r.hi);
}

// The four words of a raw buffer descriptor (base, no stride, size in bytes, 32-bit raw format)
// for use as an inline-assembly operand.
__device__ __forceinline__ i32x4 rsrc_words(const void* base, uint32_t bytes)
{
    const uint64_t a = (uint64_t)base;
    return i32x4{(int)(uint32_t)a, (int)(uint32_t)(a >> 32) & 0xffff, (int)bytes, 0x00020000};
}

// One 1 KB global -> LDS copy: lane l fetches 16 bytes at rsrc[voff + soff] and they land at LDS
// byte lds + 16 l (buffer_load_dwordx4 ... lds takes its LDS base from M0).  Written as inline
// assembly so that the compiler does not make every later LDS read wait for the copy: the
// kernel orders copies and reads itself, with one vmcnt wait and a barrier per tile.  Bytes
// outside the descriptor's range arrive as zeros.
__device__ __forceinline__ void copy_to_lds(i32x4 rsrc, uint32_t lds, int voff, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :: "s"(lds), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// The same with 4 bytes per lane: 256 bytes per wave instruction, lane l landing at LDS byte
// lds + 4 l.  For the per-key and per-query fp32 rows that travel with a tile (64 values): every
// wave of the workgroup issues the same copy, instead of one wave or a part of its lanes under a
// branch.  The bytes are the same whoever's copy lands last, and the tile loops stay one basic
// block (with the branch the register allocator loses track of the accumulators across the
// blocks and moves them around: 78 register moves per tile in the forward with multiplicities).
__device__ __forceinline__ void copy_to_lds_b32(i32x4 rsrc, uint32_t lds, int voff, int soff)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dword %1, %2, %3 offen lds"
                 :: "s"(lds), "v"(voff), "s"(rsrc), "s"(soff) : "memory", "m0");
}

// One work item: the query tile (and key slice) number `item` of the launch's n_items, streamed
// forwards or backwards over its keys.  Called by every thread of the workgroup.
template <int D, int NQ, QKType QKT, Norm NORM, bool MULT, bool PARTIAL>
__device__ __forceinline__
void fwd_pipelined_item(const void* __restrict__ Qv, const void* __restrict__ Kv,
                        const void* __restrict__ Vv, void* __restrict__ Ov,
                        const float* __restrict__ mult, float* __restrict__ Zv,
                        int Nq, int Nk, int H, int kv_group, int n_qtiles, int n_items,
                        int n_splits, int keys_per_split, float scale_log2,
                        int item, bool backwards, bool stream_out, int tile_rows, int row_off)
{
    constexpr bool FP8 = QKT == QKType::Fp8;
    constexpr bool HALF = QKT == QKType::F16;      // 16-bit type of V, O and P
    constexpr int BC = kBC;
    constexpr int BR = kWaves * 16 * NQ;
    constexpr int EQ = FP8 ? 1 : 2;                // bytes per Q/K element
    constexpr int KROWB = D * EQ, KCH = KROWB / 16, KTILE = BC * KROWB;   // as stored in HBM
    constexpr int VROWB = D * 2, VCH = VROWB / 16, VTILE = BC * VROWB;
    constexpr int DB = D / 16;                     // 16-column blocks of the head dimension
    // LDS image of a tile: fragment-sized blocks, each contiguous, so that a wave's 1 KB
    // global->LDS copy fills whole blocks (no padding; no bank conflicts: the K blocks with the
    // pieces of a row permuted, see block_piece_offset, the V blocks read linearly in the lane id):
    //   K block (rb, c): key rows 16rb..16rb+15 x bytes 64c..64c+63, row-major, 1 KB
    //   V block (rb, db): key rows 16rb..16rb+15 x bytes 32db..32db+31, row-major, 512 B
    constexpr int KBLK = KROWB / 64;               // K blocks per 16 rows
    constexpr int KLDS = KTILE;                    // K tile in LDS
    constexpr int MLDS = KTILE + VTILE;            // the tile's 64 multiplicities (MULT only)
    constexpr int BUF_BYTES = KTILE + VTILE + (MULT ? BC * 4 : 0);   // K tile, V tile, multiplicities
    constexpr int LDK = KBLK;                      // 1 KB copies per wave per K tile (wave w: rows 16w..16w+15)
    constexpr int LDV = DB / 2;                    // ... per V tile (two V blocks each)
    constexpr int NST = LDK + LDV + (MULT ? 1 : 0);   // and one 256-byte copy (wave 0) of multiplicities
    constexpr int SLOTS = DB;                      // slots per sub-step: one V^T fragment each
    constexpr int KK = D / 32;                     // 16-bit: k-steps of K Q^T
    constexpr int QKM = FP8 ? 2 * NQ / SLOTS : NQ; // score matrix instructions per slot
    constexpr int PAIRS = 4 * NQ / SLOTS;          // score register pairs of stage B per slot
    constexpr int NBUF = kNBuf;                    // LDS tile buffers in rotation (a fifth, with copies
                                                   // issued a tile earlier, measured no faster)
    constexpr int PD = 3;                          // LDS prefetch distance in slots (2: no faster)
    constexpr int RING = 4;                        // fragment registers in rotation
    // VALU instructions issued behind each MFMA (measured best of 1..4; SoftMax: of 0..6).  At
    // d = 64 a slot has 12 VALU instructions for its 8 matrix instructions, so 1 leaves a third
    // of them to the end of the slot.
    constexpr int VALU_PER_MFMA = NORM == Norm::Softmax ? 3 : (MULT || D == 64) ? 2 : 1;
    static_assert(NBUF == 4, "tiles j-1 .. j+2 are resident");
    static_assert(D == 64 || D == 128, "head dimension 128 or 64");
    static_assert(NQ == 4 || NQ == 2, "64 or 32 query rows per wave");
    static_assert(FP8 || 2 * KK == SLOTS, "16-bit: one K fragment (key block, k-step) per slot");
    static_assert(!FP8 || (2 * NQ) % SLOTS == 0, "fp8: whole score instructions per slot");
    static_assert(PAIRS >= 1 && NST <= SLOTS + PD - 1, "slot plan");
    static_assert(KCH >= 1 && VCH >= 1, "rows are whole 16-byte chunks");
    static_assert((2 * SLOTS) % RING == 0 && PD < RING && PD <= SLOTS, "ring indices must repeat");
    static_assert(QKT == QKType::Bf16 || NORM == Norm::Spherical || (QKT == QKType::Fp8 && NORM == Norm::Softmax),
                  "fp16 storage: spherical only; fp8 Q/K: spherical and the SoftMax twin");
    static_assert(!MULT || NORM == Norm::Spherical, "multiplicities belong to the spherical variant");
    static_assert(!PARTIAL || NORM == Norm::Spherical, "partial accumulators: spherical only");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;

    const int lid = xcd_contiguous_id(item, n_items);
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
    // query tiles are tile_rows apart (BR, or twice BR when the item is one half, row_off, of a wider tile)
    const int q0 = qt * tile_rows + row_off + wave * 16 * NQ;

    // ---- per-lane LDS byte offsets inside a tile; everything else is an immediate
    // K fragment, 16-bit (kb, kk): row 16kb + n16, bytes 64kk + 16g .. +15: piece g of row n16 of
    //                              block (kb, kk)
    // K fragment, fp8    (kb)    : row 16kb + n16, bytes 16g .. 16g+15 and 64 + 16g .. (any
    //                              assignment of the 128 k-slots to lanes works if Q agrees): piece
    //                              g of row n16 of blocks (kb, 0) and (kb, 1); at d = 64 there is
    //                              no second block and the upper 16 k-slots of every lane are zero
    const int klane = block_piece_offset(n16, g);
    // V^T fragment db: rows 4g + (n16>>2) [+16], 8 bytes at column 16db + 4(n16&3): block
    // (0 [1], db), offset 32 (4g + (n16>>2)) + 8 (n16&3) = 8 lane.  Within a 16-lane block, lane i
    // supplies the 8-byte piece row (i>>2), columns 4(i&3)..+3 and receives column i of all 4 rows.
    const int vlane = KLDS + lane * 8;
    // global -> LDS copies: lane l of a copy lands at LDS byte 16 l of the copy's 1 KB
    //   K copy c of wave w: block (w, c): row 16w + l/4, bytes 64c + 16 p, p = the piece of slot l%4
    //   V copy c of wave w: blocks (w, 2c), (w, 2c+1): row 16w + (l%32)/2, bytes 64c + 32 (l/32) + 16 (l%2)
    const int kld_lane = (16 * wave + (lane >> 2)) * KROWB + block_piece_in_slot(lane) * 16;
    const int vld_lane = (16 * wave + ((lane & 31) >> 1)) * VROWB + (lane >> 5) * 32 + (lane & 1) * 16;

    // Q is read once and O written once by this workgroup and by no other: both go past the L2's
    // retention (non-temporal), so that what stays in the XCD's L2 between batches of workgroups
    // is the K/V stream (measured: with ordinary loads and stores the 2 MB of O and 2 MB of Q that
    // 32 workgroups move at a batch boundary flush a 4 MB L2 completely).
    // ---- Q fragments (B operands of S^T = K Q^T), held for the whole kernel: lane holds
    // Q[q0 + 16qb + n16][k-slots of group g].  fp8 with d = 64 fills half of the k = 128 of
    // the instruction: the upper 16 k-slots of every lane hold zeros on both sides.
    constexpr int QREGS = FP8 ? 8 : 4;
    constexpr int QSTEPS = FP8 ? 1 : KK;
    typedef __attribute__((ext_vector_type(QREGS))) int qfrag_t;
    qfrag_t qf[NQ][QSTEPS];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        int row = q0 + qb * 16 + n16;
        row = row < Nq ? row : Nq - 1;             // rows past the end are computed and dropped
        const unsigned char* src = Qh + (size_t)row * KROWB + 16 * g;
#pragma unroll
        for (int kk = 0; kk < QSTEPS; ++kk) {
            if constexpr (FP8) {
                const i32x4 lo = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src));
                i32x4 hi = {0, 0, 0, 0};
                if constexpr (D == 128) hi = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src + 64));
                qf[qb][kk] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            } else {
                qf[qb][kk] = __builtin_nontemporal_load(reinterpret_cast<const i32x4*>(src + kk * 64));
            }
        }
    }

    f32x4 oacc[DB][NQ];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) oacc[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};
    // spherical: zacc = per-lane partial sums of s^2 (two chains per query block)
    // SoftMax:   zacc[qb][0] = per-lane partial denominator, zacc[qb][1] = exponent offset of
    //            the current sub-step, mrun = running max of raw scores, apend = factor that
    //            o still has to be multiplied with before the next stage C
    float zacc[NQ][2], mrun[NQ], apend[NQ], anext[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        zacc[qb][0] = zacc[qb][1] = 0.f;
        mrun[qb] = -INFINITY;
        apend[qb] = anext[qb] = 1.f;
    }

    // multipliers of the lane's 4 keys (16kb + 4g + t) of key block kb of the sub-step whose scores
    // stage B works on.  A sub-step's slots take block 0 first, then block 1, so each register
    // quad is reloaded half a sub-step (SLOTS / 2 slots) before its next use.  The multipliers
    // travel with their tile: copied into LDS behind K and V.
    f32x4 mreg[2];
    auto mload = [&](int kb, const SPH_LDS unsigned char* buf, int sub) {
        if constexpr (MULT)
            mreg[kb] = __builtin_bit_cast(f32x4, lds_read_b128(buf + MLDS + (32 * sub + 16 * kb + 4 * g) * 4));
    };

    const int n_tiles = (N + BC - 1) / BC;
    // Direction of the key stream: see fwd_pipelined_kernel.  Tiles past the end (the pipeline
    // runs two ahead) map past the end in either direction.
    auto src_tile = [&](int t) { return t >= n_tiles ? n_tiles : backwards ? n_tiles - 1 - t : t; };

    // copy c (K: c < LDK, V: the rest) of this wave's share of tile `tile` into buffer `buf`.
    // Rows past the end of the head are out of the descriptor's range and arrive as zeros.
    const i32x4 krw = rsrc_words((const unsigned char*)Kv + kv_off * EQ, (uint32_t)N * KROWB);
    const i32x4 vrw = rsrc_words(V + kv_off, (uint32_t)N * VROWB);
    // multiplicities of this cell's keys; those past the last key arrive as 0 (their keys are zero anyway)
    const i32x4 mrw = rsrc_words(MULT ? mult + (size_t)bidx * Nk + k0 : nullptr, MULT ? (uint32_t)N * 4 : 0);
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    auto copy_chunk = [&](int c, int t, SPH_LDS unsigned char* buf) {
        const uint32_t base = (uint32_t)(uintptr_t)buf;
        const int tile = src_tile(t);
        if (c < LDK)
            copy_to_lds(krw, base + (wave_u * KBLK + c) * 1024, kld_lane, tile * KTILE + c * 64);
        else if (c < LDK + LDV)
            copy_to_lds(vrw, base + KLDS + (wave_u * DB + 2 * (c - LDK)) * 512, vld_lane, tile * VTILE + (c - LDK) * 64);
        else                                       // the tile's 64 multiplicities, by every wave
            copy_to_lds_b32(mrw, base + MLDS, lane * 4, tile * BC * 4);
    };

    // ---- prologue: buffer 3 plays "tile -1" (zeros) for the first stage C; tiles 0 and 1 go
    // to buffers 0 and 1
    {
        const i32x4 zero4 = {0, 0, 0, 0};
        for (int i = tid; i < BUF_BYTES / 16; i += kThreads)
            *reinterpret_cast<SPH_LDS i32x4*>(smem + (NBUF - 1) * BUF_BYTES + i * 16) = zero4;
    }
#pragma unroll
    for (int t = 0; t < NBUF - 2; ++t)
#pragma unroll
        for (int c = 0; c < NST; ++c) copy_chunk(c, t, smem + t * BUF_BYTES);
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0): this wave's copies have landed
    __syncthreads();
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) mload(kb, smem, 0);

    // scores of a sub-step: [key block][query block]; P of a sub-step: one B operand per query block
    f32x4 S0[2][NQ], S1[2][NQ];
    i32x4 P0[NQ], P1[NQ];
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) { S0[kb][qb] = f32x4{0, 0, 0, 0}; S1[kb][qb] = f32x4{0, 0, 0, 0}; }
        P0[qb] = i32x4{0, 0, 0, 0};
        P1[qb] = i32x4{0, 0, 0, 0};
    }

    auto mfma_qk = [&](qfrag_t a, qfrag_t b, f32x4 c) -> f32x4 {
        if constexpr (FP8)
            return __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(a, b, c, 0, 0, 0, 0, 0, 0);
        else
            return mfma16x16<HALF>(a, b, c);
    };
    // the two 16-byte halves of an fp8 K fragment; the second comes from the row's second block
    // (d = 128 only)
    auto k8frag = [&](i32x4 lo, i32x4 hi) -> i32x8 {
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    };
    auto k8hi = [&](const SPH_LDS unsigned char* a) -> i32x4 {
        if constexpr (D == 128) return lds_read_b128(a + 1024);
        else return i32x4{0, 0, 0, 0};
    };

    // S0 = scores of sub-step 0
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
        if constexpr (FP8) {
            const SPH_LDS unsigned char* a = smem + klane + kb * KBLK * 1024;
            const qfrag_t kfr = k8frag(lds_read_b128(a), k8hi(a));
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) S0[kb][qb] = mfma_qk(kfr, qf[qb][0], S0[kb][qb]);
        } else {
#pragma unroll
            for (int kk = 0; kk < KK; ++kk) {
                const qfrag_t kfr = lds_read_b128(smem + klane + (kb * KBLK + kk) * 1024);
#pragma unroll
                for (int qb = 0; qb < NQ; ++qb) S0[kb][qb] = mfma_qk(kfr, qf[qb][kk], S0[kb][qb]);
            }
        }
    }

    // Fragment registers.  16-bit: one K fragment per slot, in a ring.  fp8: the K fragment of
    // key block kb arrives as two 16-byte halves with the V^T fragment of the first slot that
    // uses it; two sets alternate between consecutive sub-steps.
    i32x4 kf[FP8 ? 1 : RING];
    i32x4 kf8[FP8 ? 2 : 1][2][2];
    i32x4 vf[RING];
    // Reads for slot u of an iteration whose tiles j-1, j, j+1 sit at bprv, bcur, bnxt:
    //   u in [0,SLOTS)        first half : K_j sub 1,     V_{j-1} sub 1
    //   u in [SLOTS,2SLOTS)   second half: K_{j+1} sub 0, V_j sub 0
    //   u >= 2SLOTS           next iteration's first half: K_{j+1} sub 1, V_j sub 1
    auto issue_reads = [&](int u, const SPH_LDS unsigned char* bprv, const SPH_LDS unsigned char* bcur,
                           const SPH_LDS unsigned char* bnxt) {
        const int hh = u / SLOTS, i = u % SLOTS;
        // second sub-step of a tile: key rows 32..63 = row blocks 2 and 3
        const SPH_LDS unsigned char* kp = hh == 0 ? bcur + 2 * KBLK * 1024 : hh == 1 ? bnxt : bnxt + 2 * KBLK * 1024;
        const SPH_LDS unsigned char* vp = hh == 0 ? bprv + 2 * DB * 512 : hh == 1 ? bcur : bcur + 2 * DB * 512;
        // V first, K last: LDS returns in order, so the one wait in front of the slot's first
        // matrix instruction (which needs K) covers all reads of the slot
        const SPH_LDS unsigned char* a = vp + vlane + i * 512;
        const i32x2 lo = lds_read_tr64(a);
        const i32x2 hi = lds_read_tr64(a + DB * 512);
        vf[u % RING] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
        if constexpr (FP8) {
            if (i % (SLOTS / 2) == 0) {
                const int kb = i / (SLOTS / 2);
                kf8[hh & 1][kb][0] = lds_read_b128(kp + klane + kb * KBLK * 1024);
                kf8[hh & 1][kb][1] = k8hi(kp + klane + kb * KBLK * 1024);
            }
        } else {
            const int kb = i / KK, kk = i % KK;
            kf[u % RING] = lds_read_b128(kp + klane + (kb * KBLK + kk) * 1024);
        }
    };

    // buffers of tiles j-1, j, j+1, j+2
    SPH_LDS unsigned char* bprv = smem + (NBUF - 1) * BUF_BYTES;
    SPH_LDS unsigned char* bcur = smem;
    SPH_LDS unsigned char* bnxt = smem + BUF_BYTES;
    SPH_LDS unsigned char* bnn = smem + 2 * BUF_BYTES;
#pragma unroll
    for (int u = 0; u < PD; ++u) issue_reads(u, bprv, bcur, bnxt);

    auto run_tiles = [&](const int j_begin, const int j_end) __attribute__((always_inline)) {
      for (int j = j_begin; j < j_end; ++j) {
#pragma unroll
        for (int s = 0; s < 2 * SLOTS; ++s) {
            const int hf = s / SLOTS, i = s % SLOTS;
            f32x4 (&Sn)[2][NQ] = hf == 0 ? S1 : S0;
            f32x4 (&Sc)[2][NQ] = hf == 0 ? S0 : S1;
            i32x4 (&Pc)[NQ] = hf == 0 ? P0 : P1;
            i32x4 (&Pp)[NQ] = hf == 0 ? P1 : P0;
            __builtin_amdgcn_sched_barrier(0);
            // The one barrier per tile.  Tile j+1, copied into LDS during the previous
            // iteration, becomes visible before its first read (the prefetch below): every wave
            // waits for its own copies (they are its only vector-memory operations in flight) and
            // then for the others.  Past the barrier
            // every wave has also finished the previous iteration, whose first half was the
            // last reader of the buffer that this iteration's copies overwrite.
            if (s == SLOTS - PD) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0x0F70);                   // vmcnt(0)
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            issue_reads(s + PD, bprv, bcur, bnxt);

            // SoftMax twin: o must carry the factor from the previous sub-step's new maximum
            // before stage C adds to it.  One test per sub-step; the whole accumulator is
            // rescaled in the (rare, once the maxima have settled) case that a maximum moved.
            if constexpr (NORM == Norm::Softmax) {
                if (i == 0) {
                    bool moved = false;
#pragma unroll
                    for (int qb = 0; qb < NQ; ++qb) moved |= apend[qb] != 1.f;
                    if (__builtin_amdgcn_ballot_w64(moved) != 0) {
#pragma unroll
                        for (int db = 0; db < DB; ++db)
#pragma unroll
                            for (int qb = 0; qb < NQ; ++qb) oacc[db][qb] *= apend[qb];
                    }
                }
            }

            // A: next sub-step's scores
            if constexpr (FP8) {
#pragma unroll
                for (int u = 0; u < QKM; ++u) {
                    const int idx = i * QKM + u, kb = idx / NQ, qb = idx % NQ;
                    const qfrag_t kfr = k8frag(kf8[hf][kb][0], kf8[hf][kb][1]);
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    Sn[kb][qb] = mfma_qk(kfr, qf[qb][0], zero);
                }
            } else {
                const int kb = i / KK, kk = i % KK;
#pragma unroll
                for (int qb = 0; qb < NQ; ++qb) {
                    const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
                    Sn[kb][qb] = mfma_qk(kf[s % RING], qf[qb][kk], kk == 0 ? zero : Sn[kb][qb]);
                }
            }
            // C: V^T fragment i (columns 16i .. 16i+15 of d) against the previous sub-step's P
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb)
                oacc[i][qb] = mfma16x16<HALF>(vf[s % RING], Pp[qb], oacc[i][qb]);

            // B: PAIRS register pairs of the current sub-step's scores.  Pair p = (block p/2,
            // registers 2(p%2), 2(p%2)+1); block = (kb, qb); the pair becomes register
            // 2kb + p%2 of the B operand P[qb].
            if constexpr (NORM == Norm::Softmax) {
                if (i == 0) {
                    // keys past N (ragged last tile only) must not take part in the SoftMax
                    const int key0 = (2 * src_tile(j) + hf) * 32;      // first key of the current sub-step
                    if (key0 + 32 > N) {
#pragma unroll
                        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                            for (int qb = 0; qb < NQ; ++qb)
#pragma unroll
                                for (int t = 0; t < 4; ++t)
                                    if (key0 + 16 * kb + 4 * g + t >= N) Sc[kb][qb][t] = -INFINITY;
                    }
#pragma unroll
                    for (int qb = 0; qb < NQ; ++qb) {
                        float mx = fmaxf(Sc[0][qb][0], Sc[1][qb][0]);
#pragma unroll
                        for (int t = 1; t < 4; ++t) mx = fmaxf(mx, fmaxf(Sc[0][qb][t], Sc[1][qb][t]));
                        mx = max_across_groups(mx);
                        const float mnew = fmaxf(mrun[qb], mx);
                        anext[qb] = __builtin_amdgcn_exp2f((mrun[qb] - mnew) * scale_log2);
                        mrun[qb] = mnew;
                        zacc[qb][0] *= anext[qb];
                        zacc[qb][1] = -mnew * scale_log2;    // offset of this sub-step's exponents
                    }
                }
            }
#pragma unroll
            for (int u = 0; u < PAIRS; ++u) {
                const int p = i * PAIRS + u;
                const int blkid = p / 2, c = p % 2, kb = blkid / NQ, qb = blkid % NQ;
                float a = Sc[kb][qb][2 * c], b = Sc[kb][qb][2 * c + 1];
                if constexpr (MULT) {
                    a *= mreg[kb][2 * c];
                    b *= mreg[kb][2 * c + 1];
                }
                if constexpr (NORM == Norm::Spherical) {           // a2 = x^2, a1 = x
                    zacc[qb][0] = __builtin_fmaf(a, a, zacc[qb][0]);
                    zacc[qb][1] = __builtin_fmaf(b, b, zacc[qb][1]);
                } else if constexpr (NORM == Norm::L1) {           // a2 = |x|, a1 = x
                    zacc[qb][0] += __builtin_fabsf(a);
                    zacc[qb][1] += __builtin_fabsf(b);
                } else if constexpr (NORM == Norm::SqRelu) {       // a1 = a2 = relu(x)^2
                    a = fmaxf(a, 0.f);
                    b = fmaxf(b, 0.f);
                    a *= a;
                    b *= b;
                    zacc[qb][0] += a;
                    zacc[qb][1] += b;
                } else {                                            // a1 = a2 = exp(x/sqrt(d) - max)
                    a = __builtin_amdgcn_exp2f(__builtin_fmaf(a, scale_log2, zacc[qb][1]));
                    b = __builtin_amdgcn_exp2f(__builtin_fmaf(b, scale_log2, zacc[qb][1]));
                    zacc[qb][0] += a + b;
                }
                Pc[qb][2 * kb + c] = pack2<HALF>(a, b);
            }
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) {      // keep the running sums where they were computed
                if constexpr (NORM == Norm::Softmax) asm volatile("" : "+v"(zacc[qb][0]));
                else asm volatile("" : "+v"(zacc[qb][0]), "+v"(zacc[qb][1]));
            }
            if constexpr (NORM == Norm::Softmax) {
                if (i == SLOTS - 1) {
#pragma unroll
                    for (int qb = 0; qb < NQ; ++qb) apend[qb] = anext[qb];
                }
            }
            // multipliers: block 1 of this sub-step while block 0 is in use, block 0 of the next
            // sub-step (second half of tile j, or first half of tile j+1) once block 1 is
            if (MULT && i == 0) mload(1, bcur, hf);
            if (MULT && i == SLOTS / 2) mload(0, hf == 0 ? bcur : bnxt, hf ^ 1);
            // copies of tile j+2 out of HBM/L2 into the free buffer, one per slot, right after
            // the barrier: they have a whole tile's time to land
            constexpr int FIRST_COPY = SLOTS - PD + 1;
            if (s >= FIRST_COPY && s < FIRST_COPY + NST) copy_chunk(s - FIRST_COPY, j + 2, bnn);
            // issue order inside the slot: after each matrix instruction, at most one LDS read
            // and one VALU instruction, so that the matrix pipe never waits on the issue port
            {
                constexpr int NM = QKM + NQ;
#pragma unroll
                for (int m = 0; m < NM; ++m) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // MFMA
                    if (m < 4) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // DS read
                    __builtin_amdgcn_sched_group_barrier(0x002, VALU_PER_MFMA, 0);   // VALU
                    if (s >= FIRST_COPY && s < FIRST_COPY + NST && m == NM - 1)
                        __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);   // VMEM read (the copy)
                }
            }
        }
        SPH_LDS unsigned char* t = bprv; bprv = bcur; bcur = bnxt; bnxt = bnn; bnn = t;
      }
    };
    if constexpr (D == 64) {
        // Two workgroups share a CU: tiles in groups of 8, the wave priority set per group
        // (priority_by_tile) outside the loop over tiles, which stays free of branches.  Up to
        // 128 tiles a head's K and V (2 MB) stay in the 4 MB L2 however far the workgroups
        // drift apart, and the tiles run as one group (a group boundary costs about 40 ns).
        const int group = n_tiles > 128 ? 8 : n_tiles;
        for (int j0 = 0; j0 < n_tiles; j0 += group) {
            priority_by_tile(j0);
            run_tiles(j0, j0 + group < n_tiles ? j0 + group : n_tiles);
        }
    } else {
        run_tiles(0, n_tiles);
    }
    __builtin_amdgcn_sched_barrier(0);
    // the copies of the two tiles past the end (all zeros) must not outlive the workgroup's LDS
    __builtin_amdgcn_s_waitcnt(0x0F70);            // vmcnt(0)

    // ---- drain: stage C of the last sub-step (V of the last tile, sub 1, now at bprv)
    {
        const SPH_LDS unsigned char* vp = bprv + 2 * DB * 512;
#pragma unroll
        for (int i = 0; i < SLOTS; ++i) {
            const SPH_LDS unsigned char* a = vp + vlane + i * 512;
            const i32x2 lo = lds_read_tr64(a);
            const i32x2 hi = lds_read_tr64(a + DB * 512);
            const i32x4 vfr = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) {
                if constexpr (NORM == Norm::Softmax) oacc[i][qb] *= apend[qb];
                oacc[i][qb] = mfma16x16<HALF>(vfr, P1[qb], oacc[i][qb]);
            }
        }
    }

    // ---- partial result: the pair (o, z) as it stands, in fp32
    if constexpr (PARTIAL) {
        const size_t rows0 = ((size_t)split * (n_items / (n_qtiles * n_splits)) + bh) * Nq;
        float* Op = (float*)Ov + rows0 * D;
        float* Zp = Zv + rows0;
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) {
            const float z = sum_across_groups(zacc[qb][0] + zacc[qb][1]);
            const int row = q0 + qb * 16 + n16;
            if (row < Nq) {
                if (g == 0) Zp[row] = z;
                float* dst = Op + (size_t)row * D + 4 * g;
#pragma unroll
                for (int db = 0; db < DB; ++db) *reinterpret_cast<f32x4*>(dst + db * 16) = oacc[db][qb];   // read back soon: let the L2 keep it
            }
        }
        return;
    }

    // ---- tail t(o, z) = o / b(z): spherical b = sqrt, the others b = id.  The rows go out
    // through a per-wave LDS stage (the tile buffers are free once every wave has read its last
    // tile), 16 bytes per lane and whole rows per instruction.
    const __amdgpu_buffer_rsrc_t orw = make_rsrc((unsigned short*)Ov + head_off, (uint32_t)Nq * D * 2);
    constexpr int ROWS = 16 * NQ;
    static_assert(kWaves * ROWS * (D * 2 + 16) <= NBUF * BUF_BYTES, "the output stage fits the tile buffers");
    SPH_LDS unsigned char* stage = smem + wave * ROWS * (D * 2 + 16);
    __syncthreads();
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        float inv, z;
        if constexpr (NORM == Norm::Spherical) {
            z = sum_across_groups(zacc[qb][0] + zacc[qb][1]);
            inv = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        } else if constexpr (NORM == Norm::Softmax) {
            z = sum_across_groups(zacc[qb][0]);
            inv = 1.0f / z;
        } else {
            z = sum_across_groups(zacc[qb][0] + zacc[qb][1]);
            inv = z > 0.f ? 1.0f / z : 0.f;
        }
        const int row = q0 + qb * 16 + n16;
        if (Zv != nullptr && g == 0 && row < Nq) Zv[(size_t)bh * Nq + row] = z;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            const i32x2 o4 = {pack2<HALF>(oacc[db][qb][0] * inv, oacc[db][qb][1] * inv),
                              pack2<HALF>(oacc[db][qb][2] * inv, oacc[db][qb][3] * inv)};
            put_piece<D * 2>(stage, qb * 16 + n16, db * 32 + 8 * g, o4);
        }
    }
    store_tile<ROWS, D * 2>(stage, orw, q0, Nq, lane, stream_out);
}

// The kernel: PERSISTENT workgroups.  The launch has n_items work items (query tile x key slice
// x head) and at most as many workgroups as the chip runs at once; workgroup w takes the items
// w, w + gridDim, w + 2 gridDim, ..., so that "the workgroups an XCD runs at the same time" is
// a fact of the launch (batch k = items k gridDim ..) rather than a guess about the dispatcher.
// (It also removes the 11 us between the last wave of a workgroup leaving a CU and the first of
// its successor arriving, measured with 4 items of 173 us per CU; on Gaussian data that buys
// nothing, because the part is power-limited and gives idle time back as clock.)
//
// Workgroup ids are dealt round-robin to the XCDs and gridDim is a multiple of the number of
// XCDs (or the launch is a single batch), so every item of a workgroup falls into that XCD's
// contiguous range of (head, query tile) pairs, and the workgroups of an XCD work on
// consecutive tiles of one head at the same time: they stream the same K/V through one L2.
//
// Direction of the key stream.  When a head has more query tiles than an XCD runs at once, the
// next batch streams the same K/V again; if the head's K/V is larger than the L2, what the first
// batch left there is the END of the stream, so every other batch walks the keys backwards and
// starts on what is still resident (a sum over keys: any order gives the same accumulator up to
// fp32 rounding).  O goes past the L2's retention (non-temporal stores) only when later batches
// follow; a one-batch launch gains nothing from that, and its last stores would complete later
// (measured on 256 workgroups of 32 tiles: 30.9 against 28.9 us).
// At d = 64 two workgroups share a CU (64 KB of LDS each, 48 KB with fp8 Q/K; two waves per SIMD,
// which fill each other's waits): the kernels are held to the 256 registers that this takes.  The
// spherical one needs 258 otherwise, and one workgroup per CU costs it 5 % on 8 x 32768 x 64; the
// SoftMax normalizer, whose stage B is the longer, gains 21 % (with 32 bytes of scratch per lane),
// the fp8 Q/K kernel 4.5 % (20 to 68 bytes).
template <int D, int NQ, QKType QKT, Norm NORM, bool MULT, bool PARTIAL = false>
__global__ __launch_bounds__(kThreads, D == 64 ? 2 : 1)
void fwd_pipelined_kernel(const void* __restrict__ Qv, const void* __restrict__ Kv,
                          const void* __restrict__ Vv, void* __restrict__ Ov,
                          const float* __restrict__ mult, float* __restrict__ Zv,
                          int Nq, int Nk, int H, int kv_group, int n_qtiles, int n_items,
                          int n_splits, int keys_per_split, float scale_log2,
                          int item_begin, int item_end, int halves)
{
    constexpr int BR = kWaves * 16 * NQ;
    if (halves) {
        // Remainder launch: the items item_begin .. item_end - 1 of a launch whose tiles are
        // 2 BR rows (n_qtiles and n_items count those), one half of an item per workgroup.
        // Workgroups 16u .. 16u+7 take the first halves of items item_begin + 8u .. +7,
        // workgroups 16u+8 .. 16u+15 the second halves: a workgroup stays on the XCD that owns
        // its item's range (item_begin is a multiple of the XCD count).
        const int t = blockIdx.x, half = (t / kXcds) & 1;
        const int item = item_begin + (t / (2 * kXcds)) * kXcds + t % kXcds;
        if (item >= item_end) return;
        const int qt = xcd_contiguous_id(item, n_items) % n_qtiles;
        if (qt * 2 * BR + half * BR >= Nq) return;     // the tile's second half lies past the last row
        fwd_pipelined_item<D, NQ, QKT, NORM, MULT, PARTIAL>(Qv, Kv, Vv, Ov, mult, Zv, Nq, Nk, H, kv_group, n_qtiles, n_items,
                                                            n_splits, keys_per_split, scale_log2,
                                                            item, halves == 2, true, 2 * BR, half * BR);
        return;
    }
    const bool several_batches = item_end - item_begin > (int)gridDim.x || item_end < n_items;
    int batch = 0;
    for (int item = item_begin + blockIdx.x; item < item_end; item += gridDim.x, ++batch) {
        // the LDS buffers change hands: every wave must be done with the previous item's tiles
        if (batch > 0) __syncthreads();
        fwd_pipelined_item<D, NQ, QKT, NORM, MULT, PARTIAL>(Qv, Kv, Vv, Ov, mult, Zv, Nq, Nk, H, kv_group, n_qtiles, n_items,
                                                            n_splits, keys_per_split, scale_log2,
                                                            item, batch % 2 == 1, several_batches, BR, 0);
    }
}

}  // namespace sphattn
