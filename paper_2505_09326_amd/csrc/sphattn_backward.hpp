// Backward of spherical attention for gfx950, 16-bit storage (bf16 or fp16).
//
// The paper gives no backward pass; this is the chain rule on its definition (Appendix A.1,
// Definition 2 with a1 = id, a2 = square, b = sqrt).  With r_i = z_i^(-1/2) (z from the
// forward), O_i = r_i sum_j s_ij v_j, upstream gradient dO and delta_i = dO_i . O_i:
//
//     dV_j  = sum_i (r_i s_ij) dO_i
//     ds_ij = r_i (dO_i . v_j) - delta_i r_i^2 s_ij
//     dQ_i  = sum_j ds_ij k_j            dK_j = sum_i ds_ij q_i
//
// Nothing N x N is stored: the scores are recomputed tile by tile, as in the forward.  Two
// kernels, no atomics, so the result does not depend on the launch:
//   bwd_dq_kernel   a workgroup owns 256 query rows and streams the keys: S^T = K Q^T,
//                   G^T = V dO^T, dS^T / r_i = G^T - delta_i r_i S^T in registers,
//                   dQ^T += K^T dS^T / r_i, times r_i at the end.  Also writes, per row,
//                   delta_i r_i^2 and r_i for the other kernel (which would otherwise take the
//                   reciprocal square root of every z_i once per wave and key tile).
//   bwd_dkv_kernel  a workgroup owns 128 keys and streams the queries: S = Q K^T, G = dO V^T,
//                   W and dS in registers, dV^T += dO^T W, dK^T += Q^T dS.
// Both use the forward's building blocks: 16x16x32 matrix instructions with the product
// arranged so that the accumulator registers of the first contraction are, after the
// elementwise step, directly a B operand of the second (k-slot e of lane group g = key or
// query 4g + e, or 16 + 4g + e - 4); the streamed operand's tiles copied from HBM/L2 straight
// into LDS as 512-byte blocks of 16 rows x 32 bytes (the forward's V blocks), which serve both
// as row-major A operands (lane (n16, g) reads piece g % 2 of row n16 of block g / 2 of a pair)
// and, through ds_read_b64_tr_b16 at 8 bytes per lane in lane order, as transposed A operands;
// the LDS banks serve both reads at full rate (blocks of 16 rows x 64 bytes read the same way
// cost every 16-byte read twice its cycles: see block_piece_offset).  Two LDS buffers, one
// barrier per streamed tile.
//
// Gene-regulatory-network options (MULT, kv_group), as in the forward: s_ij = m_j (q_i . k_j),
// so dQ_i = sum_j ds_ij m_j k_j and dK_j = m_j sum_i ds_ij q_i (the multiplicities are data and
// get no gradient); kv_group query heads share a K/V head, whose dK and dV sum over the
// group's query heads (the dK/dV workgroup streams them one after the other).
#pragma once
#include "sphattn_pipelined.hpp"

namespace sphattn {

// fp32 value of one 16-bit storage element held in the low half of `bits`
template <bool HALF>
__device__ __forceinline__ float widen16(unsigned bits)
{
    if constexpr (HALF) return (float)__builtin_bit_cast(_Float16, (unsigned short)bits);
    else return __builtin_bit_cast(float, bits << 16);
}

// sum over the 8 elements of two 16-byte fragments of the products a_e * b_e, in fp32
template <bool HALF>
__device__ __forceinline__ float dot8(i32x4 a, i32x4 b, float acc)
{
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const unsigned x = (unsigned)a[w], y = (unsigned)b[w];
        acc = __builtin_fmaf(widen16<HALF>(x & 0xffff), widen16<HALF>(y & 0xffff), acc);
        acc = __builtin_fmaf(widen16<HALF>(x >> 16), widen16<HALF>(y >> 16), acc);
    }
    return acc;
}

// ---------------------------------------------------------------------------
// dQ.  Workgroup = 4 waves x 64 query rows (four blocks of 16).  Streams K/V tiles of 64 keys.
// ---------------------------------------------------------------------------
template <int D, bool HALF, bool MULT>
__global__ __launch_bounds__(kThreads, 1)
void bwd_dq_kernel(const void* __restrict__ Qv, const void* __restrict__ Kv, const void* __restrict__ Vv,
                   const float* __restrict__ mult,
                   const void* __restrict__ Ov, const void* __restrict__ dOv, const float* __restrict__ Z,
                   void* __restrict__ dQv, float* __restrict__ delta, float* __restrict__ rnorm,
                   int N, int H, int kv_group, int n_qtiles, int n_wg)
{
    constexpr int BC = kBC, NQ = 4, BR = kWaves * 16 * NQ;
    constexpr int ROWB = D * 2, TILE = BC * ROWB;
    constexpr int KK = D / 32, DB = D / 16, KBLK = ROWB / 64;
    constexpr int VLDS = TILE;                     // V tile behind the K tile
    constexpr int MLDS = 2 * TILE;                 // then the tile's 64 multiplicities (MULT only)
    constexpr int BUF_BYTES = 2 * TILE + (MULT ? BC * 4 : 0);

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int bh = lid / n_qtiles, qt = lid % n_qtiles;
    const size_t head_off = (size_t)bh * N * D;
    const int bidx = bh / H;
    const size_t kv_off = (size_t)(bidx * (H / kv_group) + (bh % H) / kv_group) * N * D;
    const int q0 = qt * BR + wave * 16 * NQ;

    // own rows: Q and dO as B operands (lane: row q0 + 16qb + n16, elements 32kk + 8g .. +7);
    // r and delta of the lane's query of every block
    i32x4 qf[NQ][KK], gf[NQ][KK];
    float c1[NQ], c3[NQ];                          // r_i and delta_i r_i
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        int row = q0 + qb * 16 + n16;
        const bool live = row < N;
        row = live ? row : N - 1;
        const size_t off = (head_off + (size_t)row * D) * 2 + 16 * g;
        float dsum = 0.f;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            qf[qb][kk] = *reinterpret_cast<const i32x4*>((const unsigned char*)Qv + off + kk * 64);
            gf[qb][kk] = *reinterpret_cast<const i32x4*>((const unsigned char*)dOv + off + kk * 64);
            const i32x4 of = *reinterpret_cast<const i32x4*>((const unsigned char*)Ov + off + kk * 64);
            dsum = dot8<HALF>(gf[qb][kk], of, dsum);
        }
        dsum = sum_across_groups(dsum);            // delta_i = dO_i . O_i
        const float z = Z[(size_t)bh * N + row];
        const float r = z > 0.f ? 1.0f / __builtin_sqrtf(z) : 0.f;
        c1[qb] = r;
        c3[qb] = dsum * r;
        // for the dK/dV kernel: r_i and delta_i r_i^2, the factors of G_ij and s_ij in ds_ij
        if (live && g == 0) {
            delta[(size_t)bh * N + row] = c3[qb] * r;
            rnorm[(size_t)bh * N + row] = r;
        }
    }

    f32x4 dq[DB][NQ];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < NQ; ++qb) dq[db][qb] = f32x4{0.f, 0.f, 0.f, 0.f};

    // tile copies: wave w brings rows 16w .. 16w+15 of the K and of the V tile (KBLK blocks each)
    const i32x4 krw = rsrc_words((const unsigned char*)Kv + kv_off * 2, (uint32_t)N * ROWB);
    const i32x4 vrw = rsrc_words((const unsigned char*)Vv + kv_off * 2, (uint32_t)N * ROWB);
    const i32x4 mrw = rsrc_words(MULT ? mult + (size_t)bidx * N : nullptr, MULT ? (uint32_t)N * 4 : 0);
    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    // a 1 KB copy fills two blocks: lane l lands in block l / 32, row (l % 32) / 2, piece l % 2
    const int ld_lane = (16 * wave + ((lane & 31) >> 1)) * ROWB + (lane >> 5) * 32 + (lane & 1) * 16;
    // piece 0 .. 2 KBLK - 1 of this wave's share of a tile: its 16 rows of K (even) or V (odd),
    // 64-byte column block piece / 2
    auto copy_piece = [&](int piece, int tile, uint32_t buf) {
        const int c = piece >> 1;
        copy_to_lds((piece & 1) ? vrw : krw, buf + ((piece & 1) ? VLDS : 0) + (wave_u * KBLK + c) * 1024, ld_lane,
                    tile * TILE + c * 64);
    };
    auto copy_mult = [&](int tile, uint32_t buf) {
        if constexpr (MULT) copy_to_lds_b32(mrw, buf + MLDS, lane * 4, tile * BC * 4);   // by every wave
    };
    const int alane = (g >> 1) * 512 + n16 * 32 + (g & 1) * 16;    // row-major A operand
    const int tlane = lane * 8;                                    // transposed A operand

    const int n_tiles = (N + BC - 1) / BC;
    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    copy_mult(0, lds0);
#pragma unroll
    for (int piece = 0; piece < 2 * KBLK; ++piece) copy_piece(piece, 0, lds0);
    for (int j = 0; j < n_tiles; ++j) {
        if constexpr (D == 64) priority_by_tile(j);   // two workgroups per CU: keep them at the same tile
        const uint32_t cur = (j & 1) * BUF_BYTES;
        // tile j has landed (own copies), every wave is done with the other buffer
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        // tile j + 1 goes to the other buffer: its big copies one per step below, where their
        // scalar instructions issue while the matrix pipe works
        const uint32_t nxt = lds0 + BUF_BYTES - cur;
        copy_mult(j + 1, nxt);
        const SPH_LDS unsigned char* kb_ = smem + cur;
        const SPH_LDS unsigned char* vb_ = smem + cur + VLDS;
        // The tile is worked off in a fixed sequence of steps, each with its own fragments:
        //   per 32-key sub-step: 2 KK score steps (key block kb, k-step kk: a K and a V fragment,
        //   8 matrix instructions) and then DB output steps (a K^T fragment, 4 matrix instructions).
        // The fragments of step st+1 are read from LDS before the matrix instructions of step st
        // are issued, and the VALU work on a key block's scores is issued behind the first
        // matrix instructions of the following step, so that neither the LDS latency nor the
        // matrix pipeline's is waited for in the open.
        constexpr int QG = 2 * KK, PER_SUB = QG + DB, STEPS = 2 * PER_SUB;
        i32x4 fa[2], fb[2];
        auto load_step = [&](int st) {
            const int sub = st / PER_SUB, u = st % PER_SUB;
            if (u < QG) {
                const int rb = 2 * sub + u / KK, kk = u % KK;
                fa[st & 1] = lds_read_b128(kb_ + (rb * KBLK + kk) * 1024 + alane);
                fb[st & 1] = lds_read_b128(vb_ + (rb * KBLK + kk) * 1024 + alane);
            } else {
                const int db = u - QG;
                const SPH_LDS unsigned char* a = kb_ + 2 * sub * KBLK * 1024 + db * 512 + tlane;
                const i32x2 lo = lds_read_tr64(a);
                const i32x2 hi = lds_read_tr64(a + KBLK * 1024);
                fa[st & 1] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
            }
        };
        f32x4 sc[2][NQ], gg[2][NQ];                // scores and dO V^T of key block kb
        i32x4 dsp[NQ];                             // dS^T / r_i of 32 keys as B operands
        // ds_ij / r_i = G_ij - delta_i r_i s_ij of key block kb of sub-step sub (registers 2kb,
        // 2kb+1 of dsp): r_i is the same for a whole row of dQ and is applied once, at the end
        auto finish_block = [&](int sub, int kb) {
            const int rb = 2 * sub + kb;
            f32x4 mk = {1.f, 1.f, 1.f, 1.f};       // multipliers of the lane's keys 16rb + 4g + t
            if constexpr (MULT)
                mk = __builtin_bit_cast(f32x4, lds_read_b128(smem + cur + MLDS + (16 * rb + 4 * g) * 4));
#pragma unroll
            for (int qb = 0; qb < NQ; ++qb) {
                f32x4 ds;
                if constexpr (MULT) ds = (gg[kb][qb] - (sc[kb][qb] * mk) * c3[qb]) * mk;
                else ds = gg[kb][qb] - sc[kb][qb] * c3[qb];
                dsp[qb][2 * kb] = pack2<HALF>(ds[0], ds[1]);
                dsp[qb][2 * kb + 1] = pack2<HALF>(ds[2], ds[3]);
            }
        };
        load_step(0);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int sub = st / PER_SUB, u = st % PER_SUB;
            if (st + 1 < STEPS) load_step(st + 1);
            if (st < 2 * KBLK) copy_piece(st, j + 1, nxt);
            if (u < QG) {
                const int kb = u / KK, kk = u % KK;
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int qb = 0; qb < NQ; ++qb) {
                    sc[kb][qb] = mfma16x16<HALF>(fa[st & 1], qf[qb][kk], kk == 0 ? zero : sc[kb][qb]);
                    gg[kb][qb] = mfma16x16<HALF>(fb[st & 1], gf[qb][kk], kk == 0 ? zero : gg[kb][qb]);
                }
                if (kb == 1 && kk == 0) finish_block(sub, 0);      // behind the next block's first step
                if (u == QG - 1) finish_block(sub, 1);             // the output steps need it now
            } else {
                const int db = u - QG;
#pragma unroll
                for (int qb = 0; qb < NQ; ++qb) dq[db][qb] = mfma16x16<HALF>(fa[st & 1], dsp[qb], dq[db][qb]);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);            // the copy of the tile past the end (zeros)

    unsigned short* dQh = (unsigned short*)dQv + head_off;
#pragma unroll
    for (int qb = 0; qb < NQ; ++qb) {
        const int row = q0 + qb * 16 + n16;
        if (row < N) {
            unsigned short* dst = dQh + (size_t)row * D + 4 * g;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                dq[db][qb] *= c1[qb];
                const i32x2 o4 = {pack2<HALF>(dq[db][qb][0], dq[db][qb][1]), pack2<HALF>(dq[db][qb][2], dq[db][qb][3])};
                *reinterpret_cast<i32x2*>(dst + db * 16) = o4;
            }
        }
    }
}

// ---------------------------------------------------------------------------
// dK and dV.  Workgroup = 4 waves x 32 keys (two blocks of 16).  Streams Q/dO tiles of 64
// queries together with their r and delta r^2.
// ---------------------------------------------------------------------------
// NK = key blocks of 16 per wave.  Every LDS fragment feeds NK matrix instructions of each
// product, so NK sets the LDS instructions per matrix instruction (0.75 at NK = 2; 0.5 at 3;
// 0.375 at 4, the forward's ratio).  The accumulators (2 NK D / 4 registers) bound it: NK = 2
// leaves room for two workgroups per CU (two waves per SIMD), NK = 3 (d = 128) and NK = 4
// (d = 64) fill the register file with one.  Measured with this step sequence (C3 / C4
// shapes): NK = 2 1.85 / 1.98 ms, NK = 3 2.29 / 2.05 ms, NK = 4 (d = 64) 2.14 ms: with one
// wave per SIMD the second wave's latency hiding is worth more than the saved LDS reads, so
// the library launches NK = 2.
template <int D, bool HALF, bool MULT, int NK>
__global__ __launch_bounds__(kThreads, NK == 2 ? 2 : 1)
void bwd_dkv_kernel(const void* __restrict__ Qv, const void* __restrict__ Kv, const void* __restrict__ Vv,
                    const float* __restrict__ mult,
                    const void* __restrict__ dOv, const float* __restrict__ rnorm, const float* __restrict__ delta,
                    void* __restrict__ dKv, void* __restrict__ dVv,
                    int N, int H, int kv_group, int n_ktiles, int n_wg)
{
    constexpr int BC = kBC, BKEYS = kWaves * 16 * NK;
    constexpr int ROWB = D * 2, TILE = BC * ROWB;
    constexpr int KK = D / 32, DB = D / 16, KBLK = ROWB / 64;
    constexpr int GLDS = TILE, ZLDS = 2 * TILE, DLDS = 2 * TILE + BC * 4;   // Q tile, dO tile, r, delta r^2
    constexpr int BUF_BYTES = 2 * TILE + 2 * BC * 4;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n16 = lane & 15, g = lane >> 4;
    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    // lid counts (K/V head, key tile); the query heads h0 .. h0 + kv_group - 1 of batch bidx use it
    const int kvh = lid / n_ktiles, kt = lid % n_ktiles;
    const int H_kv = H / kv_group;
    const int bidx = kvh / H_kv, h0 = (kvh % H_kv) * kv_group;
    const size_t head_off = (size_t)kvh * N * D;   // of K, V, dK, dV
    const int k0 = kt * BKEYS + wave * 16 * NK;

    // own keys: K and V as B operands (lane: key k0 + 16kb + n16, elements 32kk + 8g .. +7)
    i32x4 kf[NK][KK], vf[NK][KK];
    // The lane's keys' multiplicities wait in LDS behind the tile buffers (one float per key of
    // the workgroup, written and read by the same lanes): held in registers for the whole kernel
    // they are what pushes the d = 128 kernel out of the 256 registers of two workgroups per CU.
    constexpr int MKLDS = 2 * BUF_BYTES;
    const SPH_LDS unsigned char* mk_own = smem + MKLDS + (wave * NK * 16 + n16) * 4;
    auto mk = [&](int kb) { return MULT ? lds_read_f32(mk_own + kb * 64) : 1.f; };
#pragma unroll
    for (int kb = 0; kb < NK; ++kb) {
        int row = k0 + kb * 16 + n16;
        row = row < N ? row : N - 1;               // keys past the end are computed and dropped
        if constexpr (MULT)
            *reinterpret_cast<SPH_LDS float*>(smem + MKLDS + (wave * NK * 16 + kb * 16 + n16) * 4) = mult[(size_t)bidx * N + row];
        const size_t off = (head_off + (size_t)row * D) * 2 + 16 * g;
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            kf[kb][kk] = *reinterpret_cast<const i32x4*>((const unsigned char*)Kv + off + kk * 64);
            vf[kb][kk] = *reinterpret_cast<const i32x4*>((const unsigned char*)Vv + off + kk * 64);
        }
    }
    f32x4 dk[DB][NK], dv[DB][NK];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int kb = 0; kb < NK; ++kb) { dk[db][kb] = f32x4{0, 0, 0, 0}; dv[db][kb] = f32x4{0, 0, 0, 0}; }

    const uint32_t wave_u = __builtin_amdgcn_readfirstlane(wave);
    // a 1 KB copy fills two blocks: lane l lands in block l / 32, row (l % 32) / 2, piece l % 2
    const int ld_lane = (16 * wave + ((lane & 31) >> 1)) * ROWB + (lane >> 5) * 32 + (lane & 1) * 16;
    const int n_tiles = (N + BC - 1) / BC;
    // streamed tile `it` = tile it % n_tiles of query head h0 + it / n_tiles; each head has its
    // own descriptors, so that rows past the end of a head arrive as zeros
    struct HeadSource { i32x4 q, g, r, c; };       // buffer descriptors of Q, dO, r and delta r^2 of one query head
    auto head_source = [&](int hq) {
        const size_t qh = (size_t)(bidx * H + h0 + hq);
        return HeadSource{rsrc_words((const unsigned char*)Qv + qh * N * D * 2, (uint32_t)N * ROWB),
                          rsrc_words((const unsigned char*)dOv + qh * N * D * 2, (uint32_t)N * ROWB),
                          rsrc_words(rnorm + qh * N, (uint32_t)N * 4), rsrc_words(delta + qh * N, (uint32_t)N * 4)};
    };
    // piece 0 .. 2 KBLK - 1 of this wave's share of a tile: its 16 rows of Q (even) or dO (odd), 64-byte column block piece / 2
    auto copy_piece = [&](const HeadSource& hs, int piece, int tile, uint32_t buf) {
        const int c = piece >> 1;
        copy_to_lds((piece & 1) ? hs.g : hs.q, buf + ((piece & 1) ? GLDS : 0) + (wave_u * KBLK + c) * 1024, ld_lane,
                    tile * TILE + c * 64);
    };
    // 64 r and 64 delta r^2 values: 16 lanes x 16 bytes each; queries past N arrive as 0.
    // (Under a branch, unlike the multiplicities of the other kernels: this kernel gains
    // nothing from the all-wave form, and its 48-key variant, at 512 registers, came out
    // of the compiler with 196 bytes of scratch and wrong dK with it.)
    auto copy_planes = [&](const HeadSource& hs, int tile, uint32_t buf) {
        if (wave == 0 && lane < BC / 4) copy_to_lds(hs.r, buf + ZLDS, lane * 16, tile * BC * 4);
        if (wave == 1 && lane < BC / 4) copy_to_lds(hs.c, buf + DLDS, lane * 16, tile * BC * 4);
    };
    const int alane = (g >> 1) * 512 + n16 * 32 + (g & 1) * 16;
    const int tlane = lane * 8;

    const uint32_t lds0 = (uint32_t)(uintptr_t)smem;
    {
        const HeadSource hs = head_source(0);
        copy_planes(hs, 0, lds0);
#pragma unroll
        for (int piece = 0; piece < 2 * KBLK; ++piece) copy_piece(hs, piece, 0, lds0);
    }
    int next_hq = 0, next_tile = 0;                // head and tile of the copies issued in iteration j
    for (int j = 0; j < kv_group * n_tiles; ++j) {
        const uint32_t cur = (j & 1) * BUF_BYTES;
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0F70);        // vmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        if (++next_tile == n_tiles) { next_tile = 0; ++next_hq; }
        // The next tile goes to the other buffer, which every wave has left: the two small copies
        // here, the 2 KBLK big ones one per step below, where their scalar instructions (LDS
        // base into M0, source offset) issue while the matrix pipe works.  Past the last head:
        // the first head's first tile again, unused.
        const HeadSource hs = head_source(next_hq < kv_group ? next_hq : 0);
        const uint32_t nxt = lds0 + BUF_BYTES - cur;
        copy_planes(hs, next_tile, nxt);
        const SPH_LDS unsigned char* qb_ = smem + cur;
        const SPH_LDS unsigned char* gb_ = smem + cur + GLDS;
        // Fixed sequence of steps, each with a Q-side and a dO-side fragment and 2 NK matrix
        // instructions; the fragments of step st+1 are read from LDS before the matrix
        // instructions of step st are issued.  Per 32-query sub-step:
        //   2 KK score steps (query block qb, k-step kk): S = Q K^T, G = dO V^T
        //   DB output steps (column block db): dV^T += dO^T W, dK^T += Q^T dS
        constexpr int QG = 2 * KK, PER_SUB = QG + DB, STEPS = 2 * PER_SUB;
        i32x4 fa[2], fb[2];
        auto load_step = [&](int st) {
            const int sub = st / PER_SUB, u = st % PER_SUB;
            if (u < QG) {
                const int rb = 2 * sub + u / KK, kk = u % KK;
                fa[st & 1] = lds_read_b128(qb_ + (rb * KBLK + kk) * 1024 + alane);
                fb[st & 1] = lds_read_b128(gb_ + (rb * KBLK + kk) * 1024 + alane);
            } else {
                const int db = u - QG;
                const int boff = 2 * sub * KBLK * 1024 + db * 512 + tlane;
                const i32x2 qlo = lds_read_tr64(qb_ + boff), qhi = lds_read_tr64(qb_ + boff + KBLK * 1024);
                const i32x2 glo = lds_read_tr64(gb_ + boff), ghi = lds_read_tr64(gb_ + boff + KBLK * 1024);
                fa[st & 1] = __builtin_shufflevector(qlo, qhi, 0, 1, 2, 3);
                fb[st & 1] = __builtin_shufflevector(glo, ghi, 0, 1, 2, 3);
            }
        };
        // S[qb][kb], G[qb][kb]: lane owns key column n16 of block kb and queries 16qb + 4g + t
        f32x4 s[2][NK], gg[2][NK];
        i32x4 wp[NK], dsp[NK];
        // W and dS of query block qb of sub-step sub: registers 2qb, 2qb+1 of wp and dsp
        auto finish_block = [&](int sub, int qb) {
            const int qoff = (32 * sub + 16 * qb + 4 * g) * 4;
            // r_i and delta_i r_i^2 of the lane's four queries, as the dQ kernel left them
            const f32x4 r = __builtin_bit_cast(f32x4, lds_read_b128(smem + cur + ZLDS + qoff));
            const f32x4 c = __builtin_bit_cast(f32x4, lds_read_b128(smem + cur + DLDS + qoff));
            // s holds q_i . k_j without the multiplicity m_j of the lane's key j = n16: m_j is a
            // factor of the whole row j of dV and dK and is applied once, at the end; inside the
            // sums only the second term of dS carries one more
#pragma unroll
            for (int kb = 0; kb < NK; ++kb) {
                const f32x4 cm = MULT ? c * mk(kb) : c;
                const f32x4 w = s[qb][kb] * r;
                const f32x4 ds = gg[qb][kb] * r - s[qb][kb] * cm;
                wp[kb][2 * qb] = pack2<HALF>(w[0], w[1]);
                wp[kb][2 * qb + 1] = pack2<HALF>(w[2], w[3]);
                dsp[kb][2 * qb] = pack2<HALF>(ds[0], ds[1]);
                dsp[kb][2 * qb + 1] = pack2<HALF>(ds[2], ds[3]);
            }
        };
        load_step(0);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int sub = st / PER_SUB, u = st % PER_SUB;
            if (st + 1 < STEPS) load_step(st + 1);
            if (st < 2 * KBLK) copy_piece(hs, st, next_tile, nxt);
            if (u < QG) {
                const int qb = u / KK, kk = u % KK;
                const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int kb = 0; kb < NK; ++kb) {
                    s[qb][kb] = mfma16x16<HALF>(fa[st & 1], kf[kb][kk], kk == 0 ? zero : s[qb][kb]);
                    gg[qb][kb] = mfma16x16<HALF>(fb[st & 1], vf[kb][kk], kk == 0 ? zero : gg[qb][kb]);
                }
                // W and dS of a query block are formed right behind its last score step, so that its
                // S and G are dead before the next block's are written (16 registers that this
                // kernel, which sits at the 256 of two workgroups per CU, does not have: with them
                // alive across the next block's first step the d = 128 kernel spills, 28 bytes
                // per lane without and 324 with multiplicities); the other wave of the SIMD
                // covers the wait for the matrix pipeline
                if (qb == 0 && kk == KK - 1) finish_block(sub, 0);
                if (u == QG - 1) finish_block(sub, 1);             // the output steps need it now
            } else {
                const int db = u - QG;
#pragma unroll
                for (int kb = 0; kb < NK; ++kb) {
                    dv[db][kb] = mfma16x16<HALF>(fb[st & 1], wp[kb], dv[db][kb]);
                    dk[db][kb] = mfma16x16<HALF>(fa[st & 1], dsp[kb], dk[db][kb]);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);

    unsigned short* dKh = (unsigned short*)dKv + head_off;
    unsigned short* dVh = (unsigned short*)dVv + head_off;
#pragma unroll
    for (int kb = 0; kb < NK; ++kb) {
        const int row = k0 + kb * 16 + n16;
        const float mk_row = mk(kb);
        if (row < N) {
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                if constexpr (MULT) { dk[db][kb] *= mk_row; dv[db][kb] *= mk_row; }
                const i32x2 k4 = {pack2<HALF>(dk[db][kb][0], dk[db][kb][1]), pack2<HALF>(dk[db][kb][2], dk[db][kb][3])};
                const i32x2 v4 = {pack2<HALF>(dv[db][kb][0], dv[db][kb][1]), pack2<HALF>(dv[db][kb][2], dv[db][kb][3])};
                *reinterpret_cast<i32x2*>(dKh + (size_t)row * D + 4 * g + db * 16) = k4;
                *reinterpret_cast<i32x2*>(dVh + (size_t)row * D + 4 * g + db * 16) = v4;
            }
        }
    }
}

}  // namespace sphattn
