// The chunk-parallel backward kernel for head sizes whose chunk operands do not fit the LDS at once
// (d_k = d_v = 256 in bf16: S and dS' alone are 2 x 128 KB per chunk).  Same mathematics as k_bwd_chunk
// (adjoint of Eq. 8-11, plain delta rule only); the operands with a d_v axis are streamed in column
// blocks, in two sweeps, because the C x C adjoints of the UT transform couple all of d_k and d_v:
//
//   sweep 1 (blocks of 64 state columns, S with all of d_k):
//       dP  += dO_b Ut_b^T                      (tril taken at the end)
//       R_b  = V_b - K S_b                      (C x 64, rounded to the element type)
//       dX' += dUt_b R_b^T                      (= dU V^T + dW K^T with dW = -dUt S^T: the contraction
//                                                over d_k is taken first, so dW is not needed here)
//       dV_b = diag(beta) X^T dUt_b             (leaves the chip)
//   C x C part, as in k_bwd_chunk: G = K K^T, dX = dX' diag(beta), dA = -tril(X^T dX X^T, -1),
//       Ah = diag(beta) dA, dbeta.
//   sweep 2, per block of 128 columns of d_k (blocks of 32 state columns of S and dS'):
//       dQ_kb = dO S_kb^T + dP K_kb
//       dW_kb = -dUt S_kb^T
//       dK_kb = dP^T Q_kb + Ut dS'_kb^T + diag(beta) X^T dW_kb + Ah K_kb + Ah^T K_kb
//
// K, X, dP and Ah stay in LDS for the whole chunk; S is read twice, dO, Ut and dUt three times, dS' once.
// Every block is requested into registers one block ahead of its use.
#pragma once
#include "dn_kernels.hpp"

namespace dn {

template <typename T, int DK, int DV> struct WideSmem {
    static constexpr int BV1 = 64, BV2 = 32, KB = 128;
    static constexpr int LK = ldn<T>(DK), LT = ldn<T>(C), LF = C + 4, LU = ldc<T>(C);
    static constexpr int LV1 = ldn<T>(BV1), LV2 = ldn<T>(BV2), LB = ldn<T>(KB); // LB: rows of every C x 128 or 32 x 128 tile of sweep 2
    static constexpr size_t szCC = align16(sizeof(T) * C * LT);
    static constexpr size_t oK = 0;
    static constexpr size_t oX = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oDP = oX + szCC;
    static constexpr size_t oAh = oDP + szCC;
    // region A: sweep 1: the S^T block; C x C part: dX and M1^T; sweep 2: the Q block
    static constexpr size_t oA = oAh + szCC;
    static constexpr size_t oS1 = oA, oDX = oA, oM1T = oA + szCC, oQ2 = oA;
    static constexpr size_t szA = cmax(cmax(sizeof(T) * BV1 * LK, 2 * szCC), sizeof(T) * C * LB);
    // region B: the streamed blocks and the output staging tiles
    static constexpr size_t oB = oA + align16(szA);
    static constexpr size_t oDO1 = oB;
    static constexpr size_t oUt1 = oDO1 + align16(sizeof(T) * C * LV1);
    static constexpr size_t oDU1 = oUt1 + align16(sizeof(T) * BV1 * LU);
    static constexpr size_t oV1 = oDU1 + align16(sizeof(T) * BV1 * LU);
    static constexpr size_t oR1 = oV1 + align16(sizeof(T) * C * LV1);
    static constexpr size_t oStage1 = oR1 + align16(sizeof(T) * C * LV1); // four waves store dV tiles
    static constexpr size_t endB1 = oStage1 + 4 * sizeof(T) * Stage<T>::ELEMS;
    static constexpr size_t oProd = oB; // C x C part: dA o G in fp32
    static constexpr size_t endProd = oProd + sizeof(float) * C * LF;
    static constexpr size_t oS2 = oB;
    static constexpr size_t oDS2 = oS2 + align16(sizeof(T) * BV2 * LB);
    static constexpr size_t oDO2 = oDS2 + align16(sizeof(T) * BV2 * LB);
    static constexpr size_t oUt2 = oDO2 + align16(sizeof(T) * C * LV2);
    static constexpr size_t oDU2 = oUt2 + align16(sizeof(T) * BV2 * LU);
    static constexpr size_t oStage2 = oDU2 + align16(sizeof(T) * BV2 * LU);
    static constexpr size_t endB2 = oStage2 + NWC * sizeof(T) * Stage<T>::ELEMS;
    static constexpr size_t oDW = oS2; // dW_kb takes the place of the last S and dS' blocks
    static_assert(sizeof(T) * C * LB <= oDO2 - oS2, "dW block over the S / dS' blocks");
    static constexpr size_t oBeta = align16(cmax(cmax(endB1, endProd), endB2));
    static constexpr size_t oDb = oBeta + sizeof(float) * C;
    static constexpr size_t bytes = oDb + sizeof(float) * 4 * C;
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTC) void k_bwd_chunk_wide(SeqMap sm, int H, Ptrs p, int chunks_total) {
    using SM = WideSmem<T, DK, DV>;
    constexpr int BV1 = SM::BV1, BV2 = SM::BV2, KB = SM::KB, NB1 = DV / BV1, NB2 = DV / BV2, NKB = DK / KB;
    static_assert(DK % KB == 0 && DV % BV1 == 0 && BV1 == C && C * KB == 32 * 32 * NWC, "tiling");
    constexpr int MB = 4; // operand fragments per request batch of the long contractions
    extern __shared__ __align__(16) unsigned char smem[];
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sX = reinterpret_cast<T *>(smem + SM::oX);
    T *sDP = reinterpret_cast<T *>(smem + SM::oDP);
    T *sAh = reinterpret_cast<T *>(smem + SM::oAh);
    T *sS1 = reinterpret_cast<T *>(smem + SM::oS1);
    T *sDX = reinterpret_cast<T *>(smem + SM::oDX), *sM1T = reinterpret_cast<T *>(smem + SM::oM1T);
    T *sQ2 = reinterpret_cast<T *>(smem + SM::oQ2);
    T *sDO1 = reinterpret_cast<T *>(smem + SM::oDO1), *sUt1 = reinterpret_cast<T *>(smem + SM::oUt1);
    T *sDU1 = reinterpret_cast<T *>(smem + SM::oDU1), *sV1 = reinterpret_cast<T *>(smem + SM::oV1);
    T *sR1 = reinterpret_cast<T *>(smem + SM::oR1);
    float *sProd = reinterpret_cast<float *>(smem + SM::oProd);
    T *sS2 = reinterpret_cast<T *>(smem + SM::oS2), *sDS2 = reinterpret_cast<T *>(smem + SM::oDS2);
    T *sDO2 = reinterpret_cast<T *>(smem + SM::oDO2), *sUt2 = reinterpret_cast<T *>(smem + SM::oUt2);
    T *sDU2 = reinterpret_cast<T *>(smem + SM::oDU2), *sDW = reinterpret_cast<T *>(smem + SM::oDW);
    float *sBeta = reinterpret_cast<float *>(smem + SM::oBeta), *sDb = reinterpret_cast<float *>(smem + SM::oDb);

    const int lane = threadIdx.x & 63;
    int tid = threadIdx.x, wave = tid >> 6;

    for (TileIter it(chunks_total, H); it.valid(); it.next()) {
        // the wave number is made opaque once per chunk, so that the tile offsets derived from it are computed where they
        // are used instead of being carried in registers through the whole loop
        asm volatile("" : "+v"(wave));
        asm volatile("" : "+v"(tid)); // ... and the thread number, for the offsets of the tile loads
        const bool grp_a = tid < 256; // the small blocks are fetched by half of the workgroup each
        const int th = tid & 255;
        const int mi = (wave >> 1) & 1, ni = wave & 1; // tile of every C x C matrix (waves 0..3), of a C x 64 block (waves 4..7)
        const bool cc = wave < 4, upper = (mi == 0 && ni == 1);
        T *stg1 = reinterpret_cast<T *>(smem + SM::oStage1) + (wave & 3) * Stage<T>::ELEMS;
        const TilePos tp = tile_pos(sm, H, it.gid(), it.head());
        if (!tp.ok) continue; // packed layout: past the last real chunk
        const int nvalid = tp.nvalid, h = tp.h;
        const long row0 = tp.row0, tile = tp.tile;
        const T *gS = (const T *)p.Sc + tile * DV * DK, *gDS = (const T *)p.dSc + tile * DV * DK;
        const T *gUt = (const T *)p.Ut + tile * DV * C, *gDU = (const T *)p.dUt + tile * DV * C;
        const T *gDO = (const T *)p.d_o + (row0 * H + h) * DV, *gV = (const T *)p.v + (row0 * H + h) * DV;
        const long sv = (long)H * DV, sk = (long)H * DK;

        // ---- sweep 1
        struct {
            TileRegs<T, BV1, DK, NTC> s;
            TileRegs<T, C, BV1, 256> a, b; // first half of the workgroup: dO_b, Ut_b^T; second half: dUt_b^T, V_b
        } r1;
        auto fetch1 = [&](int vb) __attribute__((always_inline)) {
            r1.s.load(gS + (long)vb * BV1 * DK, DK, BV1, tid);
            if (grp_a) {
                r1.a.load(gDO + vb * BV1, sv, nvalid, th);
                r1.b.load(gUt + (long)vb * BV1 * C, C, BV1, th);
            } else {
                r1.a.load(gDU + (long)vb * BV1 * C, C, BV1, th);
                r1.b.load(gV + vb * BV1, sv, nvalid, th);
            }
        };
        {
            TileRegs<T, C, DK, NTC> rk;
            TileRegs<T, C, C, NTC> rx;
            rk.load((const T *)p.k + (row0 * H + h) * DK, sk, nvalid, tid);
            rx.load((const T *)p.Xm + tile * C * C, C, C, tid);
            float b = 0.f;
            if (tid < C) b = tid < nvalid ? to_f32(((const T *)p.beta)[(row0 + tid) * H + h]) : 0.f;
            fetch1(0);
            rk.store(sK, SM::LK, tid);
            rx.store(sX, SM::LT, tid);
            if (tid < C) sBeta[tid] = b;
        }
        f32x16 dp = zero16(), dxp = zero16();
#pragma unroll 1
        for (int vb = 0; vb < NB1; ++vb) {
            r1.s.store(sS1, SM::LK, tid);
            if (grp_a) { r1.a.store(sDO1, SM::LV1, th); r1.b.store(sUt1, SM::LU, th); }
            else { r1.a.store(sDU1, SM::LU, th); r1.b.store(sV1, SM::LV1, th); }
            lds_barrier();
            if (vb + 1 < NB1) fetch1(vb + 1);
            if (cc) {
                if (!upper) mma<BV1, false, true, T, true, MB>(dp, sDO1 + 32 * mi * SM::LV1, SM::LV1, sUt1 + 32 * ni, SM::LU);
            } else { // R_b = V_b - K S_b, tile (mi, ni) of the C x 64 block
                f32x16 ks = zero16();
                mma<DK, false, false, T, true, MB>(ks, sK + 32 * mi * SM::LK, SM::LK, sS1 + 32 * ni * SM::LK, SM::LK);
                acc_each(ks, [&](int rr, int c, float &val) { val = to_f32(sV1[(32 * mi + rr) * SM::LV1 + 32 * ni + c]) - val; });
                acc_to_lds<T>(sR1, SM::LV1, 32 * mi, 32 * ni, ks);
            }
            lds_barrier();
            if (cc) {
                if (!upper) mma<BV1, true, false, T, true, MB>(dxp, sDU1 + 32 * mi, SM::LU, sR1 + 32 * ni * SM::LV1, SM::LV1);
            } else { // dV_b = diag(beta) X^T dUt_b (X^T is upper triangular)
                f32x16 acc = zero16();
                if (mi == 1) mma<32, true, false, T, true, MB>(acc, sX + 32 * SM::LT + 32, SM::LT, sDU1 + 32 * ni * SM::LU + 32, SM::LU);
                else mma<C, true, false, T, true, MB>(acc, sX, SM::LT, sDU1 + 32 * ni * SM::LU, SM::LU);
                acc_each(acc, [&](int rr, int, float &val) { val *= sBeta[32 * mi + rr]; });
                acc_store<T>(stg1, (T *)p.dv + (row0 * H + h) * DV, sv, 32 * mi, vb * BV1 + 32 * ni, nvalid, acc);
            }
            lds_barrier();
        }

        // ---- sweep 2's first blocks are requested before the C x C part.  Its blocks are small (28 KB), so two of them
        // are kept in flight: two register sets, used alternately.
        struct Blk {
            TileRegs<T, BV2, KB, NTC> s, ds;
            TileRegs<T, C, BV2, 256> a;  // first half of the workgroup: dO_b
            TileRegs<T, BV2, C, 256> b;  // first half: Ut_b^T; second half: dUt_b^T
        } r2a, r2b;
        TileRegs<T, C, KB, NTC> rq;
        auto fetch2 = [&](Blk &r, int kb, int vb) __attribute__((always_inline)) {
            if (vb >= NB2) { vb -= NB2; ++kb; } // blocks are numbered across the d_k blocks
            if (kb >= NKB) return;
            r.s.load(gS + (long)vb * BV2 * DK + kb * KB, DK, BV2, tid);
            r.ds.load(gDS + (long)vb * BV2 * DK + kb * KB, DK, BV2, tid);
            if (grp_a) {
                r.a.load(gDO + vb * BV2, sv, nvalid, th);
                r.b.load(gUt + (long)vb * BV2 * C, C, BV2, th);
            } else {
                r.b.load(gDU + (long)vb * BV2 * C, C, BV2, th);
            }
        };
        rq.load((const T *)p.q + (row0 * H + h) * DK, sk, nvalid, tid);
        fetch2(r2a, 0, 0);
        fetch2(r2b, 0, 1);

        // ---- the C x C part (adjoint of Eq. 10-11)
        f32x16 g = zero16();
        if (cc) {
            acc_each(dp, [&](int rr, int c, float &val) { if (32 * ni + c > 32 * mi + rr) val = 0.f; }); // dP = tril(dO Ut^T)
            acc_to_lds<T>(sDP, SM::LT, 32 * mi, 32 * ni, dp);
            if (!upper) mma<DK, false, false, T, true, MB>(g, sK + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK);
            acc_each(g, [&](int rr, int c, float &val) { if (32 * ni + c >= 32 * mi + rr) val = 0.f; }); // strictly lower G
            float part = 0.f; // dbeta part 1 (column sums of X o dX'), dX = dX' diag(beta)
            acc_each(dxp, [&](int rr, int c, float &val) {
                const int i = 32 * mi + rr, j = 32 * ni + c;
                part += to_f32(sX[i * SM::LT + j]) * val;
                val *= sBeta[j];
            });
            sDb[(2 * mi + (lane >> 5)) * C + 32 * ni + (lane & 31)] = part; // summed in a fixed order below
            acc_to_lds<T>(sDX, SM::LT, 32 * mi, 32 * ni, dxp);
        }
        lds_barrier();
        if (cc) { // M1 = dX X^T
            f32x16 m1 = zero16();
            mma<C, false, false, T, true, MB>(m1, sDX + 32 * mi * SM::LT, SM::LT, sX + 32 * ni * SM::LT, SM::LT);
            acc_to_lds_t<T>(sM1T, SM::LT, 32 * mi, 32 * ni, m1);
        }
        lds_barrier();
        if (cc) { // dA = -tril(X^T M1, -1); dA o G to sProd; Ah = diag(beta) dA
            f32x16 acc = zero16();
            if (!upper) {
                if (mi == 1) mma<32, true, false, T, true, MB>(acc, sX + 32 * SM::LT + 32, SM::LT, sM1T + 32 * ni * SM::LT + 32, SM::LT);
                else mma<C, true, false, T, true, MB>(acc, sX, SM::LT, sM1T + 32 * ni * SM::LT, SM::LT);
            }
            const int l31 = lane & 31, hh = lane >> 5;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = 32 * mi + 8 * (e >> 2) + 4 * hh + (e & 3), j = 32 * ni + l31;
                const float da = j < i ? -acc[e] : 0.f;
                sProd[i * SM::LF + j] = da * g[e];
                sAh[i * SM::LT + j] = from_f32<T>(sBeta[i] * da);
            }
        }
        lds_barrier();
        if (tid < 256) { // dbeta = column sums from part 1 + row sums of dA o G
            const int i = tid >> 2, seg = tid & 3;
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += sProd[i * SM::LF + seg * 16 + j];
            sum += __shfl_xor(sum, 1);
            sum += __shfl_xor(sum, 2);
            if (seg == 0 && i < nvalid) p.dbeta[(row0 + i) * H + h] = sum + ((sDb[i] + sDb[C + i]) + (sDb[2 * C + i] + sDb[3 * C + i]));
        }
        lds_barrier(); // dX, M1^T and dA o G are dead: their bytes take the blocks of sweep 2

        // ---- sweep 2
#pragma unroll 1
        for (int kb = 0; kb < NKB; ++kb) {
            asm volatile("" : "+v"(wave));
            const int ka = wave >> 2, kc = wave & 3; // this wave's tile of a C x 128 block
            T *stg2 = reinterpret_cast<T *>(smem + SM::oStage2) + wave * Stage<T>::ELEMS;
            f32x16 dq = zero16(), dw = zero16(), dk1 = zero16();
            auto block = [&](Blk &r, int vb) __attribute__((always_inline)) {
                r.s.store(sS2, SM::LB, tid); r.ds.store(sDS2, SM::LB, tid);
                if (grp_a) { r.a.store(sDO2, SM::LV2, th); r.b.store(sUt2, SM::LU, th); }
                else r.b.store(sDU2, SM::LU, th);
                if (vb == 0) {
                    rq.store(sQ2, SM::LB, tid);
                    if (kb + 1 < NKB) rq.load((const T *)p.q + (row0 * H + h) * DK + (kb + 1) * KB, sk, nvalid, tid);
                }
                lds_barrier();
                fetch2(r, kb, vb + 2); // this set's registers are free again
                mma<BV2, false, true, T, true, MB>(dq, sDO2 + 32 * ka * SM::LV2, SM::LV2, sS2 + 32 * kc, SM::LB);  // dO S^T
                mma<BV2, true, true, T, true, MB>(dw, sDU2 + 32 * ka, SM::LU, sS2 + 32 * kc, SM::LB);              // dUt S^T
                mma<BV2, true, true, T, true, MB>(dk1, sUt2 + 32 * ka, SM::LU, sDS2 + 32 * kc, SM::LB);            // Ut dS'^T
                lds_barrier();
            };
            static_assert(NB2 % 2 == 0, "blocks are taken in pairs");
#pragma unroll 1
            for (int vb = 0; vb < NB2; vb += 2) {
                block(r2a, vb);
                block(r2b, vb + 1);
            }
            const T *sKb = sK + kb * KB + 32 * kc; // this wave's 32 columns of K
            // dQ = dO S^T + dP K
            if (ka == 0) mma<32, false, true, T, true, MB>(dq, sDP, SM::LT, sKb, SM::LK);
            else mma<C, false, true, T, true, MB>(dq, sDP + 32 * SM::LT, SM::LT, sKb, SM::LK);
            acc_store<T>(stg2, (T *)p.dq + (row0 * H + h) * DK, sk, 32 * ka, kb * KB + 32 * kc, nvalid, dq);
            // dK1 = dP^T Q + Ut dS'^T
            if (ka == 1) mma<32, true, true, T, true, MB>(dk1, sDP + 32 * SM::LT + 32, SM::LT, sQ2 + 32 * SM::LB + 32 * kc, SM::LB);
            else mma<C, true, true, T, true, MB>(dk1, sDP, SM::LT, sQ2 + 32 * kc, SM::LB);
            acc_each(dw, [&](int, int, float &val) { val = -val; }); // dW = -dUt S^T, as an operand
            acc_to_lds<T>(sDW, SM::LB, 32 * ka, 32 * kc, dw);
            lds_barrier();
            { // + diag(beta) X^T dW (X^T is upper triangular)
                f32x16 dKb = zero16();
                if (ka == 1) mma<32, true, true, T, true, MB>(dKb, sX + 32 * SM::LT + 32, SM::LT, sDW + 32 * SM::LB + 32 * kc, SM::LB);
                else mma<C, true, true, T, true, MB>(dKb, sX, SM::LT, sDW + 32 * kc, SM::LB);
                acc_each(dKb, [&](int rr, int, float &val) { val *= sBeta[32 * ka + rr]; });
                dk1 += dKb;
            }
            // + Ah K + Ah^T K; Ah is strictly lower triangular
            if (ka == 0) mma<32, false, true, T, true, MB>(dk1, sAh, SM::LT, sKb, SM::LK);
            else mma<C, false, true, T, true, MB>(dk1, sAh + 32 * SM::LT, SM::LT, sKb, SM::LK);
            if (ka == 1) mma<32, true, true, T, true, MB>(dk1, sAh + 32 * SM::LT + 32, SM::LT, sKb + 32 * SM::LK, SM::LK);
            else mma<C, true, true, T, true, MB>(dk1, sAh, SM::LT, sKb, SM::LK);
            acc_store<T>(stg2, (T *)p.dk + (row0 * H + h) * DK, sk, 32 * ka, kb * KB + 32 * kc, nvalid, dk1);
            lds_barrier(); // dW and Q_kb are dead
        }
    }
}

} // namespace dn
