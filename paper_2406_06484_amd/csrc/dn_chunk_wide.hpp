// The chunk-parallel backward kernel for head sizes whose chunk operands do not fit the LDS at once
// (d_k = d_v = 256 in bf16: S and dS' alone are 2 x 128 KB per chunk).  Same mathematics as k_bwd_chunk
// (adjoint of Eq. 8-11; all three variants, see VAR_* below); the operands with a d_v axis are streamed in blocks of
// state columns, each read from global memory exactly once except Ut (twice):
//
//   sweep 1 (blocks of 32 state columns: S_b with all of d_k, dO_b, Ut_b, dUt_b, V_b):
//       dP  += dO_b Ut_b^T                      (tril taken at the end)
//       dX' += dUt_b V_b^T                      (the dU V^T part)
//       dQ  += dO_b S_b^T,   dW -= dUt_b S_b^T  (C x d_k accumulators in registers: every wave owns 32 columns of d_k)
//       dV_b = diag(beta) X^T dUt_b             (leaves the chip)
//   then dQ += dP K leaves the chip, dW goes to LDS as an operand, dX' += dW K^T, and the C x C part runs as in
//   k_bwd_chunk: G = K K^T, dX = dX' diag(beta), dA = -tril(X^T dX X^T, -1), Ah = diag(beta) dA, dbeta;
//   sweep 2 (blocks of 32 state columns: dS'_b with all of d_k, Ut_b):
//       dK1 += Ut_b dS'_b^T
//   and dK = dK1 + dP^T Q + diag(beta) X^T dW + Ah K + Ah^T K.
//
// K, X, dP, Ah (and dW from the end of sweep 1) stay in LDS for the whole chunk.  Every block is requested into
// registers ahead of its use: two blocks ahead in both sweeps (32 KB and 20 KB per block; two register sets used alternately).
#pragma once
#include <type_traits>

#include "dn_kernels.hpp"

namespace dn {

struct NoTile {};

template <typename T, int DK, int DV> struct WideSmem {
    static constexpr int BV1 = 32, BV2 = 32;
    static constexpr int LK = ldn<T>(DK), LT = ldn<T>(C), LF = C + 4, LU = ldc<T>(C), LV1 = ldn<T>(BV1);
    static constexpr size_t szCC = align16(sizeof(T) * C * LT);
    static constexpr size_t oK = 0;
    static constexpr size_t oX = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oDP = oX + szCC;
    static constexpr size_t oAh = oDP + szCC;
    // region A: the S^T block of sweep 1, then dW
    static constexpr size_t oA = oAh + szCC;
    static constexpr size_t oS1 = oA, oDW = oA;
    static constexpr size_t szA = align16(sizeof(T) * cmax(BV1, C) * LK);
    // region B: the small blocks of sweep 1; dA o G, dX, M1^T of the C x C part; the blocks of sweep 2, then Q
    static constexpr size_t oB = oA + szA;
    static constexpr size_t oDO1 = oB;
    static constexpr size_t oV1 = oDO1 + align16(sizeof(T) * C * LV1);
    static constexpr size_t oUt1 = oV1 + align16(sizeof(T) * C * LV1);
    static constexpr size_t oDU1 = oUt1 + align16(sizeof(T) * BV1 * LU);
    static constexpr size_t endB1 = oDU1 + align16(sizeof(T) * BV1 * LU);
    static constexpr size_t oProd = oB;
    static constexpr size_t oDX = oProd + align16(sizeof(float) * C * LF);
    static constexpr size_t oM1T = oDX + szCC;
    static constexpr size_t endBc = oM1T + szCC;
    static constexpr size_t oDS2 = oB;
    static constexpr size_t oUt2 = oDS2 + align16(sizeof(T) * BV2 * LK);
    static constexpr size_t endB2 = oUt2 + align16(sizeof(T) * BV2 * LU);
    static constexpr size_t oQ = oB;
    static constexpr size_t endBq = oQ + align16(sizeof(T) * C * LK);
    static constexpr size_t oStage = align16(cmax(cmax(endB1, endBc), cmax(endB2, endBq))); // per-wave output staging tiles
    static constexpr size_t oBeta = oStage + NWC * sizeof(T) * Stage<T>::ELEMS;
    static constexpr size_t oDb = oBeta + sizeof(float) * C;
    static constexpr size_t oGi = oDb + sizeof(float) * 4 * C;  // gated: 1 / gamma_i
    static constexpr size_t oZ = oGi + sizeof(float) * C;       // gated: per-wave shares of z
    static constexpr size_t bytes = oZ + sizeof(float) * NWC;
};

// VAR_PROLOGUE: beta arrives as a logit (beta = sigmoid(logit), section 2.2) and dbeta leaves as the gradient with respect
// to it; q and k are the mapped ones that k_wy_prep left in the workspace, and k_feature_map_bwd below takes dq and dk back
// through the feature map afterwards.
// VAR_GATED: as in k_bwd_chunk the chunk is the plain rule on v_i / gamma_i with outputs gamma_i o~_i: dO rows come in scaled
// by gamma_i, V rows by 1 / gamma_i, dV goes out scaled by 1 / gamma_i.  Of the gate gradient this kernel leaves, per chunk,
// z = <dS_C, S_C> = <dS~', S_0> + <K, Ut dS~'^T> in p.zg (S is read a second time in sweep 2 for the first term, registers
// only); k_gate_grad below adds the per-token terms.
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTC) void k_bwd_chunk_wide(SeqMap sm, int H, Ptrs p, int chunks_total) {
    constexpr bool PRO = VAR == VAR_PROLOGUE, GATED = VAR == VAR_GATED;
    using SM = WideSmem<T, DK, DV>;
    constexpr int BV1 = SM::BV1, BV2 = SM::BV2, NB1 = DV / BV1, NB2 = DV / BV2;
    static_assert(DK == 32 * NWC && DV % BV1 == 0 && NB1 % 2 == 0 && NB2 % 2 == 0, "one block of 32 columns of d_k per wave");
    constexpr int MB = 4; // operand fragments per request batch
    extern __shared__ __align__(16) unsigned char smem[];
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sX = reinterpret_cast<T *>(smem + SM::oX);
    T *sDP = reinterpret_cast<T *>(smem + SM::oDP);
    T *sAh = reinterpret_cast<T *>(smem + SM::oAh);
    T *sS1 = reinterpret_cast<T *>(smem + SM::oS1), *sDW = reinterpret_cast<T *>(smem + SM::oDW);
    T *sDO1 = reinterpret_cast<T *>(smem + SM::oDO1), *sV1 = reinterpret_cast<T *>(smem + SM::oV1);
    T *sUt1 = reinterpret_cast<T *>(smem + SM::oUt1), *sDU1 = reinterpret_cast<T *>(smem + SM::oDU1);
    float *sProd = reinterpret_cast<float *>(smem + SM::oProd);
    T *sDX = reinterpret_cast<T *>(smem + SM::oDX), *sM1T = reinterpret_cast<T *>(smem + SM::oM1T);
    T *sDS2 = reinterpret_cast<T *>(smem + SM::oDS2), *sUt2 = reinterpret_cast<T *>(smem + SM::oUt2);
    T *sQ = reinterpret_cast<T *>(smem + SM::oQ);
    float *sBeta = reinterpret_cast<float *>(smem + SM::oBeta), *sDb = reinterpret_cast<float *>(smem + SM::oDb);
    float *sGi = reinterpret_cast<float *>(smem + SM::oGi), *sZ = reinterpret_cast<float *>(smem + SM::oZ);

    const int lane = threadIdx.x & 63;
    int tid = threadIdx.x, wave = tid >> 6;

    // What a chunk needs first (K, X, beta and the first two blocks of sweep 1) is requested while the previous chunk's last
    // products run: with one workgroup per CU nothing else would keep the memory system busy then.
    struct Blk1 {
        TileRegs<T, BV1, DK, NTC> s;
        TileRegs<T, C, BV1, 256> a;  // first half of the workgroup: dO_b; second half: V_b
        TileRegs<T, BV1, C, 256> b;  // first half: Ut_b^T; second half: dUt_b^T
    } r1a, r1b;
    struct Head {
        TileRegs<T, C, DK, NTC> k;
        TileRegs<T, C, C, NTC> x;
        float beta;
        float rowf[1], gi; // gated: gamma (first half of the workgroup) or 1 / gamma (second half) of this lane's dO / V row; 1 / gamma_tid
    } rh;
    auto pos_of = [&](const TileIter &i) __attribute__((always_inline)) { return i.valid() ? tile_pos(sm, H, i.gid(), i.head()) : TilePos{0, 0, 0, 0, false}; };
    // (no branches in the request code: the compiler then knows how many requests are in flight at every point and waits
    // for exactly the block it needs; past the last block the last one is requested again, which costs an L2 hit)
    const bool first_half = __builtin_amdgcn_readfirstlane((int)(threadIdx.x < 256)) != 0; // wave-uniform, in a scalar register
    auto fetch1 = [&](Blk1 &r, const TilePos &t, int vb) __attribute__((always_inline)) {
        vb = min(vb, NB1 - 1);
        r.s.load((const T *)p.Sc + (t.tile * DV + vb * BV1) * DK, DK, BV1, tid);
        const T *pa = first_half ? (const T *)p.d_o : (const T *)p.v, *pb = first_half ? (const T *)p.Ut : (const T *)p.dUt;
        r.a.load(pa + (t.row0 * H + t.h) * DV + vb * BV1, (long)H * DV, t.nvalid, tid & 255);
        r.b.load(pb + (t.tile * DV + vb * BV1) * C, C, BV1, tid & 255);
    };
    auto fetch_head = [&](const TilePos &t) __attribute__((always_inline)) {
        rh.k.load((const T *)p.k + (t.row0 * H + t.h) * DK, (long)H * DK, t.nvalid, tid);
        rh.x.load((const T *)p.Xm + t.tile * C * C, C, C, tid);
        rh.beta = to_f32(((const T *)p.beta)[(t.row0 + min(tid, t.nvalid - 1)) * H + t.h]); // (masked where it is used)
        if (GATED) {
            const float *gt = p.gam + t.tile * 2 * C;
            rh.rowf[0] = gt[(first_half ? 0 : C) + (tid & 255) / TileRegs<T, C, BV1, 256>::TPR];
            rh.gi = gt[C + (tid & (C - 1))];
        }
        fetch1(r1a, t, 0);
        fetch1(r1b, t, 1);
    };
    TileIter it(chunks_total, H);
    TilePos tp = pos_of(it);
    if (tp.ok) fetch_head(tp);
    while (tp.ok) { // packed layout: the first chunk past the last real one ends the walk (so would every later one)
        // the wave and thread numbers are made opaque once per chunk, so that the tile offsets derived from them are
        // computed where they are used instead of being carried in registers through the whole loop
        // (... and again at every phase of the chunk: `derive`)
        bool grp_a, cc, upper; // grp_a: the small blocks are fetched by half of the workgroup each
        int th, mi, ni, kc;    // (mi, ni): tile of every C x C matrix (waves 0..3); mi: tile of the C x 32 block of dV (waves 4 and 6); kc: this wave's columns of d_k
        T *stg;
        auto derive = [&]() __attribute__((always_inline)) {
            asm volatile("" : "+v"(wave));
            asm volatile("" : "+v"(tid));
            grp_a = tid < 256; th = tid & 255;
            mi = (wave >> 1) & 1; ni = wave & 1;
            cc = wave < 4; upper = (mi == 0 && ni == 1);
            kc = 32 * wave;
            stg = reinterpret_cast<T *>(smem + SM::oStage) + wave * Stage<T>::ELEMS;
        };
        derive();
        const int nvalid = tp.nvalid, h = tp.h;
        const long row0 = tp.row0, tile = tp.tile;
        const T *gDS = (const T *)p.dSc + tile * DV * DK, *gUt = (const T *)p.Ut + tile * DV * C;
        const long sv = (long)H * DV, sk = (long)H * DK;

        // ---- sweep 1
        rh.k.store(sK, SM::LK, tid);
        rh.x.store(sX, SM::LT, tid);
        if (tid < C) sBeta[tid] = tid < nvalid ? (PRO ? sigmoid_f32(rh.beta) : rh.beta) : 0.f;
        if (GATED && tid < C) sGi[tid] = rh.gi;
        const float rowf[1] = {rh.rowf[0]}; // (rh is refilled for the next chunk before this chunk's last blocks are stored)
        f32x16 dp = zero16(), dxp = zero16();
        f32x16 dq0 = zero16(), dq1 = zero16(), dw0 = zero16(), dw1 = zero16(); // rows 0..31 and 32..63 of this wave's columns
        auto block1 = [&](Blk1 &r, int vb) __attribute__((always_inline)) {
            r.s.store(sS1, SM::LK, tid);
            if (GATED) r.a.scale_rows(rowf);
            if (grp_a) { r.a.store(sDO1, SM::LV1, th); r.b.store(sUt1, SM::LU, th); }
            else { r.a.store(sV1, SM::LV1, th); r.b.store(sDU1, SM::LU, th); }
            lds_barrier();
            fetch1(r, tp, vb + 2); // this set's registers are free again
            mma<BV1, false, true, T, true, MB>(dq0, sDO1, SM::LV1, sS1 + kc, SM::LK);               // dO S^T
            mma<BV1, false, true, T, true, MB>(dq1, sDO1 + 32 * SM::LV1, SM::LV1, sS1 + kc, SM::LK);
            mma<BV1, true, true, T, true, MB>(dw0, sDU1, SM::LU, sS1 + kc, SM::LK);                 // dUt S^T
            mma<BV1, true, true, T, true, MB>(dw1, sDU1 + 32, SM::LU, sS1 + kc, SM::LK);
            if (cc) {
                if (!upper) {
                    mma<BV1, false, true, T, true, MB>(dp, sDO1 + 32 * mi * SM::LV1, SM::LV1, sUt1 + 32 * ni, SM::LU);   // dO Ut^T
                    mma<BV1, true, false, T, true, MB>(dxp, sDU1 + 32 * mi, SM::LU, sV1 + 32 * ni * SM::LV1, SM::LV1);   // dU V^T
                }
            } else if (ni == 0) { // dV_b = diag(beta) X^T dUt_b (X^T is upper triangular): two tiles, waves 4 and 6
                f32x16 acc = zero16();
                if (mi == 1) mma<32, true, false, T, true, MB>(acc, sX + 32 * SM::LT + 32, SM::LT, sDU1 + 32, SM::LU);
                else mma<C, true, false, T, true, MB>(acc, sX, SM::LT, sDU1, SM::LU);
                acc_each(acc, [&](int rr, int, float &val) { val *= GATED ? sBeta[32 * mi + rr] * sGi[32 * mi + rr] : sBeta[32 * mi + rr]; });
                acc_store<T>(stg, (T *)p.dv + (row0 * H + h) * DV, sv, 32 * mi, vb * BV1, nvalid, acc);
            }
            lds_barrier();
        };
#pragma unroll 1
        for (int vb = 0; vb < NB1; vb += 2) {
            block1(r1a, vb);
            block1(r1b, vb + 1);
        }

        // ---- sweep 2's first blocks and Q are requested here.  The blocks of sweep 2 are small (20 KB), so two of them
        // are kept in flight: two register sets, used alternately.
        struct Blk {
            TileRegs<T, BV2, DK, NTC> ds;
            TileRegs<T, BV2, C, 256> ut; // first half of the workgroup
            std::conditional_t<GATED, TileRegs<T, BV2, DK, NTC>, NoTile> s; // gated: the S block once more, for <dS~', S_0>
        } r2a, r2b;
        TileRegs<T, C, DK, NTC> rq;
        auto fetch2 = [&](Blk &r, int vb) __attribute__((always_inline)) {
            vb = min(vb, NB2 - 1);
            r.ds.load(gDS + (long)vb * BV2 * DK, DK, BV2, tid);
            r.ut.load(gUt + (long)vb * BV2 * C, C, BV2, th); // (both halves of the workgroup hold a copy)
            if constexpr (GATED) r.s.load((const T *)p.Sc + (tile * DV + (long)vb * BV2) * DK, DK, BV2, tid);
        };
        fetch2(r2a, 0);
        fetch2(r2b, 1);
        rq.load((const T *)p.q + (row0 * H + h) * DK, sk, nvalid, tid);

        // ---- dQ leaves; dW becomes an operand
        derive();
        if (cc) {
            acc_each(dp, [&](int rr, int c, float &val) { if (32 * ni + c > 32 * mi + rr) val = 0.f; }); // dP = tril(dO Ut^T)
            acc_to_lds<T>(sDP, SM::LT, 32 * mi, 32 * ni, dp);
        }
        acc_each(dw0, [&](int, int, float &val) { val = -val; }); // dW = -dUt S^T
        acc_each(dw1, [&](int, int, float &val) { val = -val; });
        acc_to_lds<T>(sDW, SM::LK, 0, kc, dw0);
        acc_to_lds<T>(sDW, SM::LK, 32, kc, dw1);
        lds_barrier();
        mma<32, false, true, T, true, MB>(dq0, sDP, SM::LT, sK + kc, SM::LK); // dQ = dO S^T + dP K
        mma<C, false, true, T, true, MB>(dq1, sDP + 32 * SM::LT, SM::LT, sK + kc, SM::LK);
        acc_store<T>(stg, (T *)p.dq + (row0 * H + h) * DK, sk, 0, kc, nvalid, dq0);
        acc_store<T>(stg, (T *)p.dq + (row0 * H + h) * DK, sk, 32, kc, nvalid, dq1);

        // ---- the C x C part (adjoint of Eq. 10-11)
        derive();
        f32x16 g = zero16();
        if (cc) {
            if (!upper) {
                mma<DK, false, false, T, true, MB>(g, sK + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK);
                mma<DK, false, false, T, true, MB>(dxp, sDW + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK); // + dW K^T
            }
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
            if (seg == 0 && i < nvalid) {
                float db = sum + ((sDb[i] + sDb[C + i]) + (sDb[2 * C + i] + sDb[3 * C + i]));
                if (PRO) db *= sBeta[i] * (1.f - sBeta[i]); // through the sigmoid
                p.dbeta[(row0 + i) * H + h] = db;
            }
        }
        lds_barrier(); // dX, M1^T and dA o G are dead: their bytes take the blocks of sweep 2

        // ---- sweep 2: dK1 = Ut dS'^T
        derive();
        f32x16 dk0 = zero16(), dk1 = zero16();
        float zp = 0.f; // gated: this thread's share of z
        auto block = [&](Blk &r, int vb) __attribute__((always_inline)) {
            if constexpr (GATED) zp += r.ds.dot(r.s);
            r.ds.store(sDS2, SM::LK, tid);
            if (grp_a) r.ut.store(sUt2, SM::LU, th);
            lds_barrier();
            fetch2(r, vb + 2); // this set's registers are free again
            mma<BV2, true, true, T, true, MB>(dk0, sUt2, SM::LU, sDS2 + kc, SM::LK);
            mma<BV2, true, true, T, true, MB>(dk1, sUt2 + 32, SM::LU, sDS2 + kc, SM::LK);
            lds_barrier();
        };
#pragma unroll 1
        for (int vb = 0; vb < NB2; vb += 2) {
            block(r2a, vb);
            block(r2b, vb + 1);
        }
        derive();
        if (GATED) { // <K, Ut dS~'^T>, while dK1 holds just that product; then this wave's share of z
            acc_each(dk0, [&](int rr, int c, float &val) { zp += val * to_f32(sK[rr * SM::LK + kc + c]); });
            acc_each(dk1, [&](int rr, int c, float &val) { zp += val * to_f32(sK[(32 + rr) * SM::LK + kc + c]); });
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) zp += __shfl_xor(zp, d);
            if (lane == 0) sZ[wave] = zp;
        }
        // the next chunk's head (this chunk's once more if there is none: no branch around the requests)
        TileIter nx = it;
        nx.next();
        const TilePos np = pos_of(nx);
        fetch_head(np.ok ? np : tp);
        rq.store(sQ, SM::LK, tid); // over the blocks of sweep 2
        lds_barrier();
        if (GATED && tid == 0) p.zg[tile] = ((sZ[0] + sZ[1]) + (sZ[2] + sZ[3])) + ((sZ[4] + sZ[5]) + (sZ[6] + sZ[7]));
        // dK = dK1 + dP^T Q + diag(beta) X^T dW + Ah K + Ah^T K (dP and Ah are lower triangular, X^T upper)
        mma<C, true, true, T, true, MB>(dk0, sDP, SM::LT, sQ + kc, SM::LK);
        mma<32, true, true, T, true, MB>(dk1, sDP + 32 * SM::LT + 32, SM::LT, sQ + 32 * SM::LK + kc, SM::LK);
        {
            f32x16 b0 = zero16(), b1 = zero16();
            mma<C, true, true, T, true, MB>(b0, sX, SM::LT, sDW + kc, SM::LK);
            mma<32, true, true, T, true, MB>(b1, sX + 32 * SM::LT + 32, SM::LT, sDW + 32 * SM::LK + kc, SM::LK);
            acc_each(b0, [&](int rr, int, float &val) { val *= sBeta[rr]; });
            acc_each(b1, [&](int rr, int, float &val) { val *= sBeta[32 + rr]; });
            dk0 += b0; dk1 += b1;
        }
        mma<32, false, true, T, true, MB>(dk0, sAh, SM::LT, sK + kc, SM::LK);
        mma<C, false, true, T, true, MB>(dk1, sAh + 32 * SM::LT, SM::LT, sK + kc, SM::LK);
        mma<C, true, true, T, true, MB>(dk0, sAh, SM::LT, sK + kc, SM::LK);
        mma<32, true, true, T, true, MB>(dk1, sAh + 32 * SM::LT + 32, SM::LT, sK + 32 * SM::LK + kc, SM::LK);
        acc_store<T>(stg, (T *)p.dk + (row0 * H + h) * DK, sk, 0, kc, nvalid, dk0);
        acc_store<T>(stg, (T *)p.dk + (row0 * H + h) * DK, sk, 32, kc, nvalid, dk1);
        lds_barrier(); // every buffer is free for the next chunk
        it = nx;
        tp = np;
    }
}

// Gradient through the query/key feature map of section 3.3, row by row, in place: x = the pre-activations ([rows, DK],
// contiguous), dy = on entry the gradient with respect to the mapped rows, on exit the gradient with respect to x.
// One workgroup per 64 rows; a thread reads back from LDS only what it put there itself.
template <typename T, int DK>
__global__ __launch_bounds__(NTHR) void k_feature_map_bwd(const T *x, T *dy, long rows) {
    constexpr int LD = ldn<T>(DK);
    extern __shared__ __align__(16) unsigned char smem[];
    T *sD = reinterpret_cast<T *>(smem);
    const long r0 = (long)blockIdx.x * C;
    const int nvalid = (int)(rows - r0 < C ? rows - r0 : C);
    TileRegs<T, C, DK, NTHR> rx, rd;
    rx.load(x + r0 * DK, DK, nvalid);
    rd.load(dy + r0 * DK, DK, nvalid);
    rd.store(sD, LD);
    wave_lds_fence();
    rx.feature_map_bwd_store(sD, LD, dy + r0 * DK, DK, nvalid);
}

// The gate gradient of the gated variant for head sizes that take k_bwd_chunk_wide: o_t is linear in q_t and in the state, so
// the sensitivity to a rescaling of the state at token j can be read off the other gradients,
//     dg_j = z + sum_{i = j .. end of the chunk} (q_i . dq_i - v_i . dv_i),
// with z = <dS_C, S_C> per chunk from k_bwd_chunk_wide.  One workgroup per (chunk, head), 256 threads.
template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_gate_grad(SeqMap sm, int H, Ptrs p) {
    __shared__ float sC[C];
    const TilePos tp = tile_pos(sm, H, blockIdx.x, blockIdx.y);
    if (!tp.ok) return;
    const int tid = threadIdx.x;
    auto row_dots = [&](auto &a, auto &b, float sign) __attribute__((always_inline)) { // sC[row] += sign * a[row] . b[row]
        typedef typename std::remove_reference<decltype(a)>::type TR;
#pragma unroll
        for (int it = 0; it < TR::NIT; ++it) {
            alignas(16) T x[TR::VEC], y[TR::VEC];
            *reinterpret_cast<uint4 *>(x) = a.v[it];
            *reinterpret_cast<uint4 *>(y) = b.v[it];
            float s = 0.f;
#pragma unroll
            for (int u = 0; u < TR::VEC; ++u) s += to_f32(x[u]) * to_f32(y[u]);
#pragma unroll
            for (int d = 1; d < TR::TPR; d <<= 1) s += __shfl_xor(s, d); // the TPR lanes of a row are adjacent
            if (tid % TR::TPR == 0) sC[it * TR::RPI + tid / TR::TPR] += sign * s; // one lane per row, rows differ between lanes
        }
    };
    if (tid < C) sC[tid] = 0.f;
    __syncthreads();
    {
        TileRegs<T, C, DK, NTHR> a, b;
        a.load((const T *)p.q + (tp.row0 * H + tp.h) * DK, (long)H * DK, tp.nvalid);
        b.load((const T *)p.dq + (tp.row0 * H + tp.h) * DK, (long)H * DK, tp.nvalid);
        row_dots(a, b, 1.f);
    }
    __syncthreads();
    {
        TileRegs<T, C, DV, NTHR> a, b;
        a.load((const T *)p.v + (tp.row0 * H + tp.h) * DV, (long)H * DV, tp.nvalid);
        b.load((const T *)p.dv + (tp.row0 * H + tp.h) * DV, (long)H * DV, tp.nvalid);
        row_dots(a, b, -1.f);
    }
    __syncthreads();
    if (tid < C) { // thread t takes token C - 1 - t; an inclusive scan over t is the suffix sum over tokens
        const int tok = C - 1 - tid;
        float c = sC[tok];
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float up = __shfl_up(c, d);
            if (tid >= d) c += up;
        }
        if (tok < tp.nvalid) p.dg[(tp.row0 + tok) * H + tp.h] = c + p.zg[tp.tile];
    }
}

} // namespace dn
