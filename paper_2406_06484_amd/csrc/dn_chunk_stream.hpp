// The chunk-parallel backward kernel of the plain delta rule in bf16 for head sizes up to 128, in a form that needs
// neither Ut = U - W S nor dUt from the scans: both are rebuilt on chip from the chunk-initial state S and the gradient
// dS' with respect to the state after the chunk, which arrive in blocks of 32 state columns (all of d_k) and are read
// exactly once.  With R = V - K S (the part of the values the state does not predict yet, section 2.2), T = X diag(beta),
// X = (I + A)^-1 of Eq. 10 and P = tril(Q K^T) of Eq. 9, per block b of state columns:
//
//   R_b  = V_b - K S_b            Ut_b  = T R_b                    (Eq. 8-9, Eq. 11)
//   dUt_b = P^T dO_b + K dS'_b    dV_b  = diag(beta) X^T dUt_b     (adjoint of Eq. 8-9; dV leaves the chip)
//   dP  += dO_b Ut_b^T            dX'  += dUt_b R_b^T
//   dQ  += dO_b S_b^T             dK   += Ut_b dS'_b^T - dV_b S_b^T
//
// and after the last block dQ += tril(dP) K, dK += tril(dP)^T Q, and the C x C part of the adjoint of Eq. 10-11:
// dX = dX' diag(beta), dA = -tril(X^T dX X^T, -1), Ah = diag(beta) dA, dK += Ah K + Ah^T K,
// dbeta_i = sum_m X[m][i] dX'[m][i] + sum_j dA[i][j] (K K^T)[i][j].
// (dX' = dW K^T + dUt V^T with dW = -dUt S^T is dUt R^T, and diag(beta) X^T dW is -dV S^T: the gradient with respect to W
// never has to exist.)
//
// Waves 0..3 own the tiles with a state-column axis (R, Ut: waves 0, 1; K dS', dUt: waves 2, 3; dV: waves 0, 1) and the
// C x C accumulators (dP, dX': waves 1, 2, 3); waves 4..7 own the C x d_k accumulators dQ and dK.  Three barriers per
// block.  K, dO, V, X, P^T stay in LDS for the chunk; the blocks of S^T and dS'^T alternate between two buffers.  Every
// thread holds its share of the chunk's tiles in registers from the moment they are requested; as soon as a tile has
// moved to LDS the same registers request that tile of the workgroup's next chunk, so about one chunk's worth of
// loads is in flight at any time.
#pragma once
#include <type_traits>

#include "dn_kernels.hpp"

namespace dn {

template <typename T, int DK, int DV> struct StreamSmem {
    static constexpr int BV = 32, NB = DV / BV;
    static constexpr int LK = ldn<T>(DK), LV = ldn<T>(DV), LT = ldn<T>(C), LU = ldc<T>(C), LF = C + 4;
    static constexpr size_t szCC = align16(sizeof(T) * C * LT);
    static constexpr size_t szBlk = align16(sizeof(T) * BV * LK); // one block of S^T or dS'^T
    static constexpr size_t szDer = align16(sizeof(T) * BV * LU);  // one C x BV tile, transposed
    static constexpr size_t szProd = sizeof(float) * C * LF;
    static constexpr size_t szK = align16(sizeof(T) * C * LK), szV = align16(sizeof(T) * C * LV);
    static constexpr size_t oK = 0;
    static constexpr size_t oDO = oK + szK;
    static constexpr size_t oV = oDO + szV;                        // V; Q once the last block has used V
    static constexpr size_t oX = oV + (szV > szK ? szV : szK);
    static constexpr size_t oPT = oX + szCC;                       // P^T; dP after the last block
    // the two stream buffers, each a block of S^T followed by a block of dS'^T.  Q sits in the second one while P^T
    // is formed (C = 2 BV, so it has exactly Q's size); after the last block the first one takes dX, then Ah
    static constexpr size_t oStr = oPT + szCC;
    static_assert(2 * szBlk == szK && 2 * szBlk >= szCC, "Q and dX fit a stream buffer");
    // R^T, (diag(beta) R)^T, Ut^T, dUt^T, -dV^T of the current block; M1^T after the last block
    static constexpr size_t oDer = oStr + 4 * szBlk;
    static_assert(4 * szDer >= szCC, "M1^T fits the derived tiles");
    // dA o G (fp32) after the last block: in the second stream buffer, else in dO's bytes, else in bytes of its own
    static constexpr int prodAt = 2 * szBlk >= szProd ? 0 : (szV >= szProd ? 1 : 2);
    static constexpr size_t oStage = oDer + 5 * szDer;
    static constexpr size_t oBeta = oStage + 8 * sizeof(T) * Stage<T>::ELEMS;
    static constexpr size_t oDb = oBeta + sizeof(float) * C;
    static constexpr size_t oOwnProd = align16(oDb + sizeof(float) * 4 * C);
    static constexpr size_t oProd = prodAt == 0 ? oStr + 2 * szBlk : (prodAt == 1 ? oDO : oOwnProd);
    static constexpr size_t bytes = prodAt == 2 ? oOwnProd + szProd : oOwnProd;
};

// acc -= V for a 32 x 32 tile: one more contraction step pair with A = -I, B = the tile of V ([row][col] storage,
// `B` points at its first element), which spares reading V in the accumulator layout
__device__ inline void mma_minus_tile(f32x16 &acc, const bf16 *B, int ldb, int tx) {
    const int lane = tx & 63, r = lane & 31, kh = 8 * (lane >> 5);
#pragma unroll
    for (int step = 0; step < 2; ++step) {
        bf16x8 a;
#pragma unroll
        for (int e = 0; e < 8; ++e) a[e] = (r == 16 * step + kh + e) ? (bf16)-1.f : (bf16)0.f;
        mfma32(acc, a, frag_ks(B, ldb, 16 * step, tx));
    }
}

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTC) void k_bwd_stream(SeqMap sm, int H, Ptrs p, int chunks_total) {
    using SM = StreamSmem<T, DK, DV>;
    static_assert(sizeof(T) == 2, "bf16 only");
    constexpr int BV = SM::BV, NB = SM::NB, NKT = DK / 32, KT = 2 * NKT, KW = KT / 4; // C x d_k tiles per wave of the second half
    static_assert(KT % 4 == 0 && NB >= 2, "tile ownership");
    constexpr int MB = 2; // operand fragments per request batch
    extern __shared__ __align__(16) unsigned char smem_[];
    // Every LDS address below is (a scalar base) + (one of a few per-lane patterns).  Left alone, the compiler forms all
    // those sums once, ahead of the chunk loop, and carries more than a hundred of them through it (they do not fit the
    // registers).  `smem` and the thread index are therefore re-derived through an empty asm at the top of every barrier
    // interval: sums cannot be merged or hoisted across that point, so each is formed where it is used.
    unsigned char *smem = smem_;
    int tq = threadIdx.x; // the thread index as the helpers of this kernel see it
    auto fresh = [&]() __attribute__((always_inline)) {
        int z = 0;
        asm volatile("" : "+s"(z));
        smem = smem_ + z;
        tq = threadIdx.x;
        asm volatile("" : "+v"(tq));
    };
#define DN_S(name, off) auto name = [&]() __attribute__((always_inline)) { return reinterpret_cast<T *>(smem + (off)); }
    DN_S(sK, SM::oK); DN_S(sDO, SM::oDO); DN_S(sV, SM::oV); DN_S(sQ1, SM::oV); DN_S(sX, SM::oX); DN_S(sPT, SM::oPT); DN_S(sDP, SM::oPT);
    DN_S(sQ0, SM::oStr + 2 * SM::szBlk); DN_S(sDX, SM::oStr); DN_S(sAh, SM::oStr);
    DN_S(sRT, SM::oDer); DN_S(sRbT, SM::oDer + SM::szDer); DN_S(sUT, SM::oDer + 2 * SM::szDer); DN_S(sDUT, SM::oDer + 3 * SM::szDer);
    DN_S(sDVT, SM::oDer + 4 * SM::szDer); DN_S(sM1T, SM::oDer);
#undef DN_S
    auto sProd = [&]() __attribute__((always_inline)) { return reinterpret_cast<float *>(smem + SM::oProd); };
    auto sBeta = [&]() __attribute__((always_inline)) { return reinterpret_cast<float *>(smem + SM::oBeta); };
    auto sDb = [&]() __attribute__((always_inline)) { return reinterpret_cast<float *>(smem + SM::oDb); };
    auto sS = [&](int b) __attribute__((always_inline)) { return reinterpret_cast<T *>(smem + SM::oStr + (size_t)(b & 1) * 2 * SM::szBlk); };
    auto sDS = [&](int b) __attribute__((always_inline)) { return reinterpret_cast<T *>(smem + SM::oStr + (size_t)(b & 1) * 2 * SM::szBlk + SM::szBlk); };

    const int tid = threadIdx.x;
    // wave-uniform, in a scalar register: every tile offset derived from it is scalar arithmetic, and the role branches
    // below are scalar branches
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // a block of S^T (and of dS'^T) is 16 bytes per thread for NTB threads: at d_k = 128 every thread holds a piece of
    // both, at d_k = 64 the first half of the workgroup holds S^T and the second half dS'^T
    constexpr int NTB = BV * DK / El<T>::VEC;
    constexpr bool SPLIT = NTB < NTC;
    static_assert(NTB == NTC || 2 * NTB == NTC, "block shape");
    struct Empty {};
    struct Regs {
        TileRegs<T, C, DK, NTC> k, q;
        TileRegs<T, C, DV, NTC> d_o, v;
        TileRegs<T, C, C, NTC> x;
        TileRegs<T, BV, DK, NTB> s[2];   // blocks b and b + 1, alternating
        std::conditional_t<SPLIT, Empty, TileRegs<T, BV, DK, NTB>> ds[2];
        T beta;
    } r;
    const bool first_half = __builtin_amdgcn_readfirstlane((int)(threadIdx.x < 256)) != 0; // wave-uniform, in a scalar register
    const long sk = (long)H * DK, sv = (long)H * DV;
    // (no branches around the requests: the compiler then knows how many are in flight at every point and waits for
    // exactly the tile it needs; where the workgroup has no next chunk the request is issued with every row masked)
    // (the row count and the tile number pass through an empty asm where they are used, for the same reason as `smem`
    // below: the per-lane offsets and row masks of a request or a store are then formed at that point, not carried)
    auto here = [](int x) __attribute__((always_inline)) { asm volatile("" : "+s"(x)); return x; };
    auto herel = [](long x) __attribute__((always_inline)) { asm volatile("" : "+s"(x)); return x; };
    auto fetch_k = [&](const TilePos &t, int live = 1) __attribute__((always_inline)) { r.k.load((const T *)p.k + (herel(t.row0) * H + t.h) * DK, sk, here(t.nvalid) * live, tq); };
    auto fetch_q = [&](const TilePos &t, int live = 1) __attribute__((always_inline)) { r.q.load((const T *)p.q + (herel(t.row0) * H + t.h) * DK, sk, here(t.nvalid) * live, tq); };
    auto fetch_do = [&](const TilePos &t, int live = 1) __attribute__((always_inline)) { r.d_o.load((const T *)p.d_o + (herel(t.row0) * H + t.h) * DV, sv, here(t.nvalid) * live, tq); };
    auto fetch_v = [&](const TilePos &t, int live = 1) __attribute__((always_inline)) { r.v.load((const T *)p.v + (herel(t.row0) * H + t.h) * DV, sv, here(t.nvalid) * live, tq); };
    auto fetch_x = [&](const TilePos &t, int live = 1) __attribute__((always_inline)) {
        r.x.load((const T *)p.Xm + herel(t.tile) * C * C, C, here(C) * live, tq);
        if (tq < C) r.beta = ((const T *)p.beta)[(herel(t.row0) + min(tq, here(t.nvalid) - 1)) * H + t.h];
    };
    auto fetch_blk = [&](const TilePos &t, int b, int live = 1) __attribute__((always_inline)) { // into register set b & 1
        const long off = (herel(t.tile) * DV + (long)b * BV) * DK;
        if constexpr (SPLIT) {
            r.s[b & 1].load((first_half ? (const T *)p.Sc : (const T *)p.dSc) + off, DK, BV * live, tq & (NTB - 1));
        } else {
            r.s[b & 1].load((const T *)p.Sc + off, DK, BV * live, tq);
            r.ds[b & 1].load((const T *)p.dSc + off, DK, BV * live, tq);
        }
    };
    auto stash_blk = [&](int b) __attribute__((always_inline)) { // block b: registers -> its stream buffer
        if constexpr (SPLIT) {
            r.s[b & 1].store(first_half ? sS(b) : sDS(b), SM::LK, tq & (NTB - 1));
        } else {
            r.s[b & 1].store(sS(b), SM::LK, tq);
            r.ds[b & 1].store(sDS(b), SM::LK, tq);
        }
    };
    // the block two ahead of b: of this chunk, or the first ones of the workgroup's next chunk
    auto fetch_ahead = [&](const TilePos &cur, const TilePos &next, int next_live, int b) __attribute__((always_inline)) {
        if (b + 2 < NB) fetch_blk(cur, b + 2);
        else fetch_blk(next, b + 2 - NB, next_live);
    };
    // where a tile lives: the same for every lane, so it is moved to scalar registers
    auto uni = [](int x) __attribute__((always_inline)) { return __builtin_amdgcn_readfirstlane(x); };
    auto unil = [&](long x) __attribute__((always_inline)) {
        return (long)(((unsigned long)(unsigned)uni((int)((unsigned long)x >> 32)) << 32) | (unsigned)uni((int)x));
    };
    auto pos_of = [&](const TileIter &i) __attribute__((always_inline)) {
        TilePos t = i.valid() ? tile_pos(sm, H, i.gid(), i.head()) : TilePos{0, 0, 0, 0, false};
        t.nvalid = uni(t.nvalid); t.h = uni(t.h); t.row0 = unil(t.row0); t.tile = unil(t.tile); t.ok = uni((int)t.ok) != 0;
        return t;
    };

    TileIter it(chunks_total, H);
    TilePos tp = pos_of(it);
    if (tp.ok) {
        fetch_k(tp); fetch_q(tp); fetch_do(tp); fetch_v(tp); fetch_x(tp);
        fetch_blk(tp, 0); fetch_blk(tp, 1);
    }
    // workgroups that start together would issue their load bursts together: stagger them (as k_bwd_chunk does)
    if ((long)chunks_total * H >= 4l * gridDim.x)
        for (int i = 0; i < (int)(blockIdx.x & 3); ++i) __builtin_amdgcn_s_sleep(64);

    while (tp.ok) { // packed layout: the first chunk past the last real one ends the walk (so would every later one)
        TileIter nx = it;
        nx.next();
        const TilePos np = pos_of(nx);
        const TilePos nf = np.ok ? np : tp; // what the freed registers request (every row masked where there is no next chunk)
        const int nl = np.ok ? 1 : 0;
        const bool first = wave < 4;
        const int mi = wave & 1;                                   // row block of this wave's C x 32 tile (waves 0..3)
        // C x C tile of this wave (waves 1, 2, 3): (1,1), (0,0), (1,0); wave 0 has none and clears the masked tile
        const int ci = wave == 2 ? 0 : 1, cj = wave == 1 ? 1 : 0;
        const bool cc = wave >= 1 && wave < 4;
        auto stg_of = [&]() __attribute__((always_inline)) { return reinterpret_cast<T *>(smem + SM::oStage) + wave * Stage<T>::ELEMS; };
        const int nvalid = tp.nvalid, h = tp.h;
        const long row0 = tp.row0;
        // tile s of this wave (waves 4..7) in a C x d_k matrix: row block ra, column block kb
        auto ra = [&](int s) __attribute__((always_inline)) { return ((wave - 4) + 4 * s) / NKT; };
        auto kb = [&](int s) __attribute__((always_inline)) { return ((wave - 4) + 4 * s) % NKT; };

        // ---- the chunk's resident tiles and its first block
        r.k.store(sK(), SM::LK, tq); r.d_o.store(sDO(), SM::LV, tq); r.v.store(sV(), SM::LV, tq); r.x.store(sX(), SM::LT, tq);
        r.q.store(sQ0(), SM::LK, tq); // (stays in registers: it is needed in LDS once more at the end of the chunk)
        stash_blk(0);
        if (tq < C) sBeta()[tq] = tq < nvalid ? to_f32(r.beta) : 0.f;
        fetch_k(nf, nl); fetch_do(nf, nl); fetch_v(nf, nl); fetch_x(nf, nl); fetch_ahead(tp, nf, nl, 0);
        lds_barrier();
            fresh();

        // accumulators: waves 0..3: a[0] = K dS'_b / dUt_b, a[1] = dP, a[2] = dX', a[3] = K K^T;
        //               waves 4..7: a[s] = dQ tile s, a[2 + s] = dK tile s
        f32x16 a[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[i] = zero16();

#pragma unroll
        for (int b = 0; b < NB; ++b) {
    #define sSb sS(b)
#define sDSb sDS(b)
            // -- first interval: R_b, K dS'_b; dQ += dO_b S_b^T; (first block) P^T
            if (first) {
                if (wave < 2) { // -R_b = K S_b - V_b, rows 32 mi .. (a[0] is free in these two waves)
                    f32x16 &acc = a[0];
                    acc = zero16();
                    mma<DK, false, false, T, true, MB>(acc, sK() + 32 * mi * SM::LK, SM::LK, sSb, SM::LK, tq);
                    mma_minus_tile(acc, sV() + 32 * mi * SM::LV + b * BV, SM::LV, tq);
                    acc_each4(acc, [&](int rr, int c, float x0, float x1, float x2, float x3) {
                        const int i = 32 * mi + rr;
                        st4(sRT() + c * SM::LU + i, -x0, -x1, -x2, -x3);
                        st4(sRbT() + c * SM::LU + i, -x0 * sBeta()[i], -x1 * sBeta()[i + 1], -x2 * sBeta()[i + 2], -x3 * sBeta()[i + 3]);
                    }, tq);
                } else { // K dS'_b
                    a[0] = zero16();
                    mma<DK, false, false, T, true, MB>(a[0], sK() + 32 * mi * SM::LK, SM::LK, sDSb, SM::LK, tq);
                }
            } else {
#pragma unroll
                for (int s = 0; s < KW; ++s)
                    mma<BV, false, true, T, true, MB>(a[s], sDO() + 32 * ra(s) * SM::LV + b * BV, SM::LV, sSb + 32 * kb(s), SM::LK, tq);
                if (b == 0 && wave >= 5) { // P = tril(Q K^T) of Eq. 9, tile (jb, ib) = (0,0), (1,0), (1,1), stored transposed
                    const int jb = wave == 5 ? 0 : 1, ib = wave == 7 ? 1 : 0;
                    f32x16 pa = zero16();
                    mma<DK, false, false, T, true, MB>(pa, sQ0() + 32 * jb * SM::LK, SM::LK, sK() + 32 * ib * SM::LK, SM::LK, tq);
                    acc_each(pa, [&](int rr, int c, float &val) { if (32 * jb + rr < 32 * ib + c) val = 0.f; }, tq);
                    acc_to_lds_t<T>(sPT(), SM::LT, 32 * jb, 32 * ib, pa, tq);
                }
            }
            lds_barrier();
            fresh();
            // -- second interval: Ut_b = T R_b (X is lower triangular), dUt_b = K dS'_b + P^T dO_b (P^T is upper
            //    triangular); the second half subtracts dV S^T of the previous block
            if (first) {
                if (wave < 2) {
                    f32x16 &acc = a[0];
                    acc = zero16();
                    if (mi == 0) mma<32, false, false, T, true, MB>(acc, sX(), SM::LT, sRbT(), SM::LU, tq);
                    else mma<C, false, false, T, true, MB>(acc, sX() + 32 * SM::LT, SM::LT, sRbT(), SM::LU, tq);
                    acc_to_lds_t<T>(sUT(), SM::LU, 32 * mi, 0, acc, tq);
                } else {
                    if (mi == 0) mma<C, false, true, T, true, MB>(a[0], sPT(), SM::LT, sDO() + b * BV, SM::LV, tq);
                    else mma<32, false, true, T, true, MB>(a[0], sPT() + 32 * SM::LT + 32, SM::LT, sDO() + 32 * SM::LV + b * BV, SM::LV, tq);
                    acc_to_lds_t<T>(sDUT(), SM::LU, 32 * mi, 0, a[0], tq);
                }
            } else if (b > 0) {
#pragma unroll
                for (int s = 0; s < KW; ++s)
                    mma<BV, true, true, T, true, MB>(a[2 + s], sDVT() + 32 * ra(s), SM::LU, sS(b - 1) + 32 * kb(s), SM::LK, tq);
            }
            lds_barrier();
            fresh();
            // -- third interval: the next block moves to LDS (its buffer's last reader was the interval above);
            //    dV_b; dP += dO_b Ut_b^T, dX' += dUt_b R_b^T; dK += Ut_b dS'_b^T
            if (b + 1 < NB) {
                stash_blk(b + 1);
                fetch_ahead(tp, nf, nl, b + 1);
            }
            if (first) {
                if (wave < 2) { // dV_b = diag(beta) X^T dUt_b (X^T is upper triangular), rows 32 mi ..
                    f32x16 &acc = a[0];
                    acc = zero16();
                    if (mi == 0) mma<C, true, false, T, true, MB>(acc, sX(), SM::LT, sDUT(), SM::LU, tq);
                    else mma<32, true, false, T, true, MB>(acc, sX() + 32 * SM::LT + 32, SM::LT, sDUT() + 32, SM::LU, tq);
                    acc_each(acc, [&](int rr, int, float &val) { val *= sBeta()[32 * mi + rr]; }, tq);
                    acc_each4(acc, [&](int rr, int c, float x0, float x1, float x2, float x3) {
                        st4(sDVT() + c * SM::LU + 32 * mi + rr, -x0, -x1, -x2, -x3);
                    }, tq);
                    acc_store<T>(stg_of(), (T *)p.dv + (herel(row0) * H + h) * DV, sv, 32 * mi, b * BV, here(nvalid), acc, tq);
                }
                if (cc) {
                    mma<BV, false, true, T, true, MB>(a[1], sDO() + 32 * ci * SM::LV + b * BV, SM::LV, sUT() + 32 * cj, SM::LU, tq);
                    mma<BV, true, true, T, true, MB>(a[2], sDUT() + 32 * ci, SM::LU, sRT() + 32 * cj, SM::LU, tq);
                }
            } else {
#pragma unroll
                for (int s = 0; s < KW; ++s)
                    mma<BV, true, true, T, true, MB>(a[2 + s], sUT() + 32 * ra(s), SM::LU, sDSb + 32 * kb(s), SM::LK, tq);
            }
            lds_barrier();
            fresh();
#undef sSb
#undef sDSb
        }

        // ---- after the last block
        // dV S^T of the last block; Q back to LDS; dP, dX = dX' diag(beta), K K^T; dbeta part 1
        r.q.store(sQ1(), SM::LK, tq);
        fetch_q(nf, nl);
        if (!first) {
#pragma unroll
            for (int s = 0; s < KW; ++s)
                mma<BV, true, true, T, true, MB>(a[2 + s], sDVT() + 32 * ra(s), SM::LU, sS(NB - 1) + 32 * kb(s), SM::LK, tq);
        } else if (cc) {
            acc_each(a[1], [&](int rr, int c, float &val) { if (32 * cj + c > 32 * ci + rr) val = 0.f; }, tq); // dP = tril(dO Ut^T)
            acc_to_lds<T>(sDP(), SM::LT, 32 * ci, 32 * cj, a[1], tq);
            mma<DK, false, false, T, true, MB>(a[3], sK() + 32 * ci * SM::LK, SM::LK, sK() + 32 * cj * SM::LK, SM::LK, tq);
            acc_each(a[3], [&](int rr, int c, float &val) { if (32 * cj + c >= 32 * ci + rr) val = 0.f; }, tq); // strictly lower K K^T
            float part = 0.f; // column sums of X o dX'
            acc_each(a[2], [&](int rr, int c, float &val) {
                const int i = 32 * ci + rr, j = 32 * cj + c;
                part += to_f32(sX()[i * SM::LT + j]) * val;
                val *= sBeta()[j];
            }, tq);
            sDb()[(2 * ci + ((tq & 63) >> 5)) * C + 32 * cj + (tq & 31)] = part; // summed in a fixed order at the end
            acc_to_lds<T>(sDX(), SM::LT, 32 * ci, 32 * cj, a[2], tq);
        } else { // wave 0: the tile above the diagonal
            f32x16 z = zero16();
            acc_to_lds<T>(sDX(), SM::LT, 0, 32, z, tq);
            sDb()[((tq & 63) >> 5) * C + 32 + (tq & 31)] = 0.f;
        }
        lds_barrier();
            fresh();
        // dQ += dP K leaves; dK += dP^T Q; M1 = dX X^T
        if (!first) {
#pragma unroll
            for (int s = 0; s < KW; ++s) {
                if (ra(s) == 0) mma<32, false, true, T, true, MB>(a[s], sDP(), SM::LT, sK() + 32 * kb(s), SM::LK, tq);
                else mma<C, false, true, T, true, MB>(a[s], sDP() + 32 * SM::LT, SM::LT, sK() + 32 * kb(s), SM::LK, tq);
                acc_store<T>(stg_of(), (T *)p.dq + (herel(row0) * H + h) * DK, sk, 32 * ra(s), 32 * kb(s), here(nvalid), a[s], tq);
                if (ra(s) == 1) mma<32, true, true, T, true, MB>(a[2 + s], sDP() + 32 * SM::LT + 32, SM::LT, sQ1() + 32 * SM::LK + 32 * kb(s), SM::LK, tq);
                else mma<C, true, true, T, true, MB>(a[2 + s], sDP(), SM::LT, sQ1() + 32 * kb(s), SM::LK, tq);
            }
        } else {
            const int m1i = wave >> 1, m1j = wave & 1;
            f32x16 m1 = zero16();
            mma<C, false, false, T, true, MB>(m1, sDX() + 32 * m1i * SM::LT, SM::LT, sX() + 32 * m1j * SM::LT, SM::LT, tq);
            acc_to_lds_t<T>(sM1T(), SM::LT, 32 * m1i, 32 * m1j, m1, tq);
        }
        lds_barrier();
            fresh();
        // dA = -tril(X^T M1, -1); dA o G for dbeta; Ah = diag(beta) dA
        if (first) {
            f32x16 acc = zero16();
            if (cc) {
                if (ci == 1) mma<32, true, false, T, true, MB>(acc, sX() + 32 * SM::LT + 32, SM::LT, sM1T() + 32 * cj * SM::LT + 32, SM::LT, tq);
                else mma<C, true, false, T, true, MB>(acc, sX(), SM::LT, sM1T() + 32 * cj * SM::LT, SM::LT, tq);
            }
            const int ti = cc ? ci : 0, tj = cc ? cj : 1; // wave 0 writes the zero tile above the diagonal
            const int l31 = tq & 31, hh = (tq & 63) >> 5;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = 32 * ti + 8 * (e >> 2) + 4 * hh + (e & 3), j = 32 * tj + l31;
                const float da = (cc && j < i) ? -acc[e] : 0.f;
                sProd()[i * SM::LF + j] = cc ? da * a[3][e] : 0.f;
                sAh()[i * SM::LT + j] = from_f32<T>(sBeta()[i] * da);
            }
        }
        lds_barrier();
            fresh();
        // dK += Ah K + Ah^T K leaves; dbeta
        if (!first) {
#pragma unroll
            for (int s = 0; s < KW; ++s) {
                if (ra(s) == 0) mma<32, false, true, T, true, MB>(a[2 + s], sAh(), SM::LT, sK() + 32 * kb(s), SM::LK, tq);
                else mma<C, false, true, T, true, MB>(a[2 + s], sAh() + 32 * SM::LT, SM::LT, sK() + 32 * kb(s), SM::LK, tq);
                if (ra(s) == 1) mma<32, true, true, T, true, MB>(a[2 + s], sAh() + 32 * SM::LT + 32, SM::LT, sK() + 32 * SM::LK + 32 * kb(s), SM::LK, tq);
                else mma<C, true, true, T, true, MB>(a[2 + s], sAh(), SM::LT, sK() + 32 * kb(s), SM::LK, tq);
                acc_store<T>(stg_of(), (T *)p.dk + (herel(row0) * H + h) * DK, sk, 32 * ra(s), 32 * kb(s), here(nvalid), a[2 + s], tq);
            }
        } else { // dbeta = column sums from part 1 + row sums of dA o G
            const int i = tq >> 2, seg = tq & 3;
            float sum = 0.f;
#pragma unroll
            for (int j = 0; j < 16; ++j) sum += sProd()[i * SM::LF + seg * 16 + j];
            sum += __shfl_xor(sum, 1);
            sum += __shfl_xor(sum, 2);
            if (seg == 0 && i < nvalid)
                p.dbeta[(herel(row0) + i) * H + h] = sum + ((sDb()[i] + sDb()[C + i]) + (sDb()[2 * C + i] + sDb()[3 * C + i]));
        }
        lds_barrier();
            fresh(); // every buffer is free for the next chunk
        it = nx;
        tp = np;
    }
}

} // namespace dn
