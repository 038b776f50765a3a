// SoftMax attention on the 32x32x16 matrix instructions: the comparison twin in the form that
// is fastest for SoftMax on gfx950 (bf16 storage only).
//
// Same tile sizes, three-stage pipeline, four rotating LDS buffers and one barrier per 64-key
// tile as fwd_pipelined_kernel (sphattn_pipelined.hpp), but its own data path: tiles are
// staged through registers (global load, ds_write) into row-major LDS rows padded against bank
// conflicts, where the spherical kernel copies global -> LDS directly into unpadded fragment
// blocks.  A timing ratio against the spherical kernel therefore contains that data-path
// difference as well as the exponential; the like-for-like twin is the Norm::Softmax
// instantiation of fwd_pipelined_kernel.  The matrix instruction differs too: a wavefront owns 64 query rows as two blocks of 32, scores are produced
// transposed with v_mfma_f32_32x32x16_bf16 (lane l owns query column l & 31 and, in register
// 4g+t, key row 8g + 4(l>>5) + t), and eight consecutive accumulator registers are one B
// operand of O^T += V^T P^T.  The exponential is a quarter-rate instruction (16 cycles per
// wave); behind a 32-cycle matrix instruction two of them fit, behind a 16-cycle one (the
// 16x16x32 form that serves the spherical kernel best) they do not, so SoftMax is measured in
// both forms and this one is the faster (C3: 1.18 ms against 1.41 ms).
//
// Per score: 1 FMA (scale and subtract the running maximum), 1 v_exp_f32, 1 add, half a
// packed convert; per 32 keys and query: a maximum over the lane's 16 scores and across the
// two lanes that share the query, one exponential for the rescale factor; the accumulator o is
// multiplied by that factor only when some lane's maximum moved.
#pragma once
#include "sphattn_device.hpp"

namespace sphattn {

template <int D>
__global__ __launch_bounds__(kThreads, 1)
void softmax32_kernel(const void* __restrict__ Qv, const void* __restrict__ Kv,
                      const void* __restrict__ Vv, void* __restrict__ Ov,
                      int N, int n_qtiles, int n_wg, float scale_log2)
{
    constexpr int BC = kBC;
    constexpr int QB = 2;                          // query blocks of 32 rows per wave
    constexpr int BR = kWaves * 32 * QB;
    constexpr int ROWB = D * 2, CH = ROWB / 16, TILE = BC * ROWB;          // as stored in HBM
    constexpr int KSTR = ROWB + kKPad, VSTR = ROWB + kVPad;                // LDS row strides
    constexpr int KLDS = BC * KSTR;
    constexpr int BUF_BYTES = KLDS + BC * VSTR;    // K tile then V tile
    constexpr int LDT = BC * CH / kThreads;        // 16-byte chunks per thread per tile and tensor
    constexpr int NST = 2 * LDT;
    constexpr int DB = D / 32;
    constexpr int SLOTS = 2 * DB;                  // slots per sub-step: one V^T and one K fragment each
    constexpr int PD = 3;                          // LDS prefetch distance in slots
    constexpr int RING = 4;
    static_assert(D == 64 || D == 128, "head dimension 128 or 64");
    static_assert(NST <= SLOTS && (2 * SLOTS) % RING == 0 && PD < RING && PD <= SLOTS, "slot plan");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    SPH_LDS unsigned char* smem = (SPH_LDS unsigned char*)smem_raw;

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, h = lane >> 5;
    const int i16 = lane & 15, blk = (lane >> 4) & 1;

    const int lid = xcd_contiguous_id(blockIdx.x, n_wg);
    const int bh = lid / n_qtiles, qt = lid % n_qtiles;
    const size_t head_off = (size_t)bh * N * D;    // in elements
    const unsigned char* Qh = (const unsigned char*)Qv + head_off * 2;
    const __amdgpu_buffer_rsrc_t krs = make_rsrc((const unsigned char*)Kv + head_off * 2, (uint32_t)N * ROWB);
    const __amdgpu_buffer_rsrc_t vrs = make_rsrc((const unsigned char*)Vv + head_off * 2, (uint32_t)N * ROWB);
    const int q0 = qt * BR + wave * 32 * QB;

    // K fragment (sub, kk): row sub*32 + l32, bytes 32kk + 16h .. +15
    const int klane = l32 * KSTR + 16 * h;
    // V^T fragment (sub, ks, db): rows sub*32 + 16ks + 4h + (i16>>2) [+8], 8 bytes at column
    // db*32 + 16*blk + 4*(i16&3)
    const int vlane = KLDS + (4 * h + (i16 >> 2)) * VSTR + (16 * blk + 4 * (i16 & 3)) * 2;
    const int kst_lane = (tid / CH) * KSTR + (tid % CH) * 16;
    const int vst_lane = KLDS + (tid / CH) * VSTR + (tid % CH) * 16;
    const int ld_lane = tid * 16;                  // tiles are contiguous in HBM

    // Q fragments (B operands of S^T = K Q^T), held for the whole kernel
    i32x4 qf[QB][SLOTS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        int row = q0 + qb * 32 + l32;
        row = row < N ? row : N - 1;               // rows past the end are computed and dropped
        const unsigned char* src = Qh + (size_t)row * ROWB + 16 * h;
#pragma unroll
        for (int kk = 0; kk < SLOTS; ++kk) qf[qb][kk] = *reinterpret_cast<const i32x4*>(src + kk * 32);
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[db][qb][r] = 0.f;
    // zsum = per-lane partial denominator, zoff = exponent offset of the current sub-step,
    // mrun = running max of raw scores, apend = factor that o still has to be multiplied with
    // before the next stage C
    float zsum[QB], zoff[QB], mrun[QB], apend[QB], anext[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        zsum[qb] = zoff[qb] = 0.f;
        mrun[qb] = -INFINITY;
        apend[qb] = anext[qb] = 1.f;
    }

    i32x4 stage[NST];
    auto gload_chunk = [&](int c, int tile) {
        if (c < LDT)
            stage[c] = __builtin_amdgcn_raw_buffer_load_b128(krs, ld_lane, tile * TILE + c * kThreads * 16, 0);
        else
            stage[c] = __builtin_amdgcn_raw_buffer_load_b128(vrs, ld_lane, tile * TILE + (c - LDT) * kThreads * 16, 0);
    };
    auto lstore_chunk = [&](int c, SPH_LDS unsigned char* buf) {
        const int off = c < LDT ? kst_lane + c * (kThreads / CH) * KSTR
                                : vst_lane + (c - LDT) * (kThreads / CH) * VSTR;
        *reinterpret_cast<SPH_LDS i32x4*>(buf + off) = stage[c];
    };

    const int n_tiles = (N + BC - 1) / BC;

    // prologue: buffer 3 plays "tile -1" (zeros) for the first stage C; tiles 0 and 1 go to
    // buffers 0 and 1; tile 2 waits in registers
    {
        const i32x4 zero4 = {0, 0, 0, 0};
        for (int i = tid; i < BUF_BYTES / 16; i += kThreads)
            *reinterpret_cast<SPH_LDS i32x4*>(smem + 3 * BUF_BYTES + i * 16) = zero4;
    }
    {
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

    // S0 = scores of sub-step 0
#pragma unroll
    for (int kk = 0; kk < SLOTS; ++kk) {
        const i32x4 kfr = lds_read_b128(smem + klane + 32 * kk);
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) S0[qb] = mfma16<false>(kfr, qf[qb][kk], S0[qb]);
    }

    i32x4 kf[RING], vf[RING];
    // Reads for slot u of an iteration whose tiles j-1, j, j+1 sit at bprv, bcur, bnxt:
    //   u in [0,SLOTS)        first half : K_j sub 1,     V_{j-1} sub 1
    //   u in [SLOTS,2SLOTS)   second half: K_{j+1} sub 0, V_j sub 0
    //   u >= 2SLOTS           next iteration's first half: K_{j+1} sub 1, V_j sub 1
    auto issue_reads = [&](int u, const SPH_LDS unsigned char* bprv, const SPH_LDS unsigned char* bcur,
                           const SPH_LDS unsigned char* bnxt) {
        const int hh = u / SLOTS, i = u % SLOTS;
        const SPH_LDS unsigned char* kp = hh == 0 ? bcur + 32 * KSTR : hh == 1 ? bnxt : bnxt + 32 * KSTR;
        const SPH_LDS unsigned char* vp = hh == 0 ? bprv + 32 * VSTR : hh == 1 ? bcur : bcur + 32 * VSTR;
        const int ks = i / DB, db = i % DB;
        const SPH_LDS unsigned char* a = vp + vlane + (16 * ks) * VSTR + db * 64;
        const i32x2 lo = lds_read_tr64(a);
        const i32x2 hi = lds_read_tr64(a + 8 * VSTR);
        vf[u % RING] = __builtin_shufflevector(lo, hi, 0, 1, 2, 3);
        kf[u % RING] = lds_read_b128(kp + klane + 32 * i);
    };

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
            // the one barrier per tile; see fwd_pipelined_kernel for why a bounded wait on the
            // LDS queue is enough in front of it
            if (s == SLOTS - PD) {
                constexpr int OUT = 3 * (SLOTS - PD) < 15 ? 3 * (SLOTS - PD) : 15;
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(0xC07F | (OUT << 8));
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
            issue_reads(s + PD, bprv, bcur, bnxt);

            // o must carry the factor from the previous sub-step's new maximum before stage C
            // adds to it; skipped when no lane's maximum moved
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

            // A: next sub-step's scores
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                f32x16 zero = {0};
                Sn[qb] = mfma16<false>(kf[s % RING], qf[qb][i], i == 0 ? zero : Sn[qb]);
            }
            // C: V^T fragment i against the previous sub-step's P
            {
                const int ks = i / DB, db = i % DB;
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[db][qb] = mfma16<false>(vf[s % RING], Pp[qb][ks], oacc[db][qb]);
            }
            // B: a slice of the current sub-step's scores, 16*QB/SLOTS registers per slot
            constexpr int PER = 16 * QB / SLOTS;
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
                    zsum[qb] *= anext[qb];
                    zoff[qb] = -mnew * scale_log2;       // offset of this sub-step's exponents
                }
            }
#pragma unroll
            for (int u = 0; u < PER; u += 2) {
                const int idx = i * PER + u;
                const int qb = idx / 16, r = idx % 16;
                const float a = __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[qb][r], scale_log2, zoff[qb]));
                const float b = __builtin_amdgcn_exp2f(__builtin_fmaf(Sc[qb][r + 1], scale_log2, zoff[qb]));
                zsum[qb] += a + b;
                Pc[qb][r / 8][(r % 8) / 2] = pack2<false>(a, b);
            }
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) asm volatile("" : "+v"(zsum[qb]));
            if (i == SLOTS - 1) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) apend[qb] = anext[qb];
            }
            // staging, second half only: tile j+2 into LDS, tile j+3 out of HBM/L2
            if (hf == 1 && i < NST) {
                lstore_chunk(i, bnn);
                gload_chunk(i, j + 3);
            }
        }
        SPH_LDS unsigned char* t = bprv; bprv = bcur; bcur = bnxt; bnxt = bnn; bnn = t;
    }
    __builtin_amdgcn_sched_barrier(0);

    // drain: stage C of the last sub-step (V of the last tile, sub 1, now at bprv)
    {
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][qb][r] *= apend[qb];
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
                oacc[db][qb] = mfma16<false>(vfr, P1[qb][ks], oacc[db][qb]);
        }
    }

    // tail: O = o / sum
    unsigned short* Oh = (unsigned short*)Ov + head_off;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float inv = 1.0f / sum_across_halves(zsum[qb]);
        const int row = q0 + qb * 32 + l32;
        if (row < N) {
            unsigned short* dst = Oh + (size_t)row * D + 4 * h;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const i32x2 o4 = {pack2<false>(oacc[db][qb][4 * g] * inv, oacc[db][qb][4 * g + 1] * inv),
                                      pack2<false>(oacc[db][qb][4 * g + 2] * inv, oacc[db][qb][4 * g + 3] * inv)};
                    *reinterpret_cast<i32x2*>(dst + db * 32 + 8 * g) = o4;
                }
        }
    }
}

}  // namespace sphattn
