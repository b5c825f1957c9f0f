// The five kernels of the chunkwise DeltaNet forward/backward (gfx950), templated on the element
// type T (float: fp32 MFMA; bf16: bf16 MFMA with fp32 accumulation) and the head dims.
//
//   k_wy_prep    per chunk            A = tril(diag(beta) K K^T,-1); X = (I+A)^-1; W = X diag(beta) K; U = X diag(beta) V   (Eq. 10-11)
//   k_scan_fwd   per chain x v-block  serial over chunks: Ut = U - W S; O = Q S + tril(Q K^T) Ut; S += K^T Ut          (Eq. 8-9)
//   k_scan_bwd   per chain x v-block  reverse over chunks: dUt = P^T dO + K dS'; dS = dS' + Q^T dO - W^T dUt
//   k_bwd_dqkw   per chunk            dQ, the part of dK that comes through Eq. 8-9, and dW = -dUt S^T
//   k_bwd_wy     per chunk            adjoint of Eq. 10-11: dK, dV, dbeta
//
// State S is [d_k][d_v] (orientation of the paper's pseudocode listing), fp32 in registers.
#pragma once
#include "dn_device.hpp"
#include "dn_host.hpp"

namespace dn {

constexpr int cmax(int a, int b) { return a > b ? a : b; }
constexpr size_t align16(size_t x) { return (x + 15) & ~size_t(15); }

// ---------------------------------------------------------------------------------------------
// per-sequence chunk-count prefix for the packed layout: coff[n] = sum_{m<n} ceil(len_m / C)
static __global__ void k_chunk_offsets(const int32_t *cu, int N, int32_t *coff) {
    __shared__ int part[NTHR];
    const int tid = threadIdx.x;
    const int per = (N + NTHR - 1) / NTHR;
    const int lo = tid * per, hi = min(N, lo + per);
    int s = 0;
    for (int n = lo; n < hi; ++n) s += (cu[n + 1] - cu[n] + C - 1) / C;
    part[tid] = s;
    __syncthreads();
    if (tid == 0) {
        int run = 0;
        for (int i = 0; i < NTHR; ++i) { int t = part[i]; part[i] = run; run += t; }
        coff[N] = run;
    }
    __syncthreads();
    int run = part[tid];
    for (int n = lo; n < hi; ++n) { coff[n] = run; run += (cu[n + 1] - cu[n] + C - 1) / C; }
}

// =============================================================================================
// k_wy_prep
template <typename T, int DK, int DV> struct PrepSmem {
    static constexpr int LK = ldn<T>(DK), LV = ldn<T>(DV), LT = ldn<T>(C), LF = C + 4, LM = 52;
    static constexpr size_t oK = 0;
    static constexpr size_t oKT = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oVT = oKT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oR1 = oVT + align16(sizeof(T) * DV * LT); // V staging, then A and X, then U staging
    static constexpr size_t szR1 = cmax(sizeof(T) * C * LV, 2 * sizeof(float) * C * LF);
    static constexpr size_t oT = oR1 + align16(szR1);
    static constexpr size_t oM = oT + align16(sizeof(T) * C * LT);
    static constexpr size_t oBeta = oM + sizeof(float) * 16 * LM;
    static constexpr size_t bytes = oBeta + sizeof(float) * C;
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_wy_prep(SeqMap sm, int H, Ptrs p) {
    using SM = PrepSmem<T, DK, DV>;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sKT = reinterpret_cast<T *>(smem + SM::oKT);
    T *sVT = reinterpret_cast<T *>(smem + SM::oVT);
    T *sV = reinterpret_cast<T *>(smem + SM::oR1);
    float *sA = reinterpret_cast<float *>(smem + SM::oR1);
    float *sX = sA + C * SM::LF;
    T *sT = reinterpret_cast<T *>(smem + SM::oT);
    float *sM = reinterpret_cast<float *>(smem + SM::oM);
    float *sBeta = reinterpret_cast<float *>(smem + SM::oBeta);

    int n, ic;
    if (!sm.chunk(blockIdx.x, n, ic)) return;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int h = blockIdx.y, tid = threadIdx.x, wave = tid >> 6;
    const int nvalid = min(C, len - ic * C);
    const long row0 = (long)t0 + (long)ic * C;
    const long tile = ((long)(cb + ic) * H + h);

    load_tile<T, C, DK>(sK, SM::LK, (const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid);
    load_tile<T, C, DV>(sV, SM::LV, (const T *)p.v + (row0 * H + h) * DV, (long)H * DV, nvalid);
    if (tid < C) sBeta[tid] = tid < nvalid ? to_f32(((const T *)p.beta)[(row0 + tid) * H + h]) : 0.f;
    __syncthreads();
    transpose_tile<T, DK>(sKT, SM::LT, sK, SM::LK);
    transpose_tile<T, DV>(sVT, SM::LT, sV, SM::LV);
    // Gram tile of this wave: rows 32*mi.., cols 32*ni..
    const int mi = wave >> 1, ni = wave & 1;
    f32x16 g = zero16();
    if (!(mi == 0 && ni == 1)) mma_nt<DK>(g, sK + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK);
    __syncthreads(); // sV (aliasing sA/sX) is dead now
    acc_each(g, [&](int r, int c, float &val) {
        const int i = 32 * mi + r, j = 32 * ni + c;
        sA[i * SM::LF + j] = j < i ? sBeta[i] * val : 0.f;
    });
    __syncthreads();
    tri_inverse_64(sA, sX, sM, SM::LF, SM::LM);
    // T = X diag(beta), Eq. 10
    for (int e = tid; e < C * C; e += NTHR) {
        const int i = e >> 6, j = e & 63;
        sT[i * SM::LT + j] = from_f32<T>(sX[i * SM::LF + j] * sBeta[j]);
    }
    __syncthreads();
    // W = T K -> staged in sK; U = T V -> staged in R1 (Eq. 11)
    T *sWout = sK, *sUout = sV;
    for (int t = wave; t < 2 * (DK / 32); t += NWAVE) {
        const int a = t / (DK / 32), b = t % (DK / 32);
        f32x16 acc = zero16();
        if (a == 0) mma_nt<32>(acc, sT, SM::LT, sKT + 32 * b * SM::LT, SM::LT);
        else mma_nt<C>(acc, sT + 32 * SM::LT, SM::LT, sKT + 32 * b * SM::LT, SM::LT);
        acc_to_lds<T>(sWout, SM::LK, 32 * a, 32 * b, acc);
    }
    for (int t = wave; t < 2 * (DV / 32); t += NWAVE) {
        const int a = t / (DV / 32), b = t % (DV / 32);
        f32x16 acc = zero16();
        if (a == 0) mma_nt<32>(acc, sT, SM::LT, sVT + 32 * b * SM::LT, SM::LT);
        else mma_nt<C>(acc, sT + 32 * SM::LT, SM::LT, sVT + 32 * b * SM::LT, SM::LT);
        acc_to_lds<T>(sUout, SM::LV, 32 * a, 32 * b, acc);
    }
    __syncthreads();
    store_tile<T, C, DK>((T *)p.W + tile * C * DK, DK, sWout, SM::LK, C);
    store_tile<T, C, DV>((T *)p.U + tile * C * DV, DV, sUout, SM::LV, C);
}

// =============================================================================================
// k_scan_fwd: STORE = false writes O and the final state; STORE = true (backward's recompute pass)
// writes every chunk-initial state and Ut to the workspace instead of O.
template <int DV> struct VBlock { static constexpr int BV = DV < 64 ? DV : 64; static constexpr int NV = DV / BV; };

template <typename T, int DK, int DV> struct ScanFwdSmem {
    static constexpr int BV = VBlock<DV>::BV;
    static constexpr int LK = ldn<T>(DK), LB = ldn<T>(BV), LT = ldn<T>(C);
    static constexpr size_t oQ = 0;
    static constexpr size_t oK = oQ + align16(sizeof(T) * C * LK);
    static constexpr size_t oW = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oKT = oW + align16(sizeof(T) * C * LK);
    static constexpr size_t oU = oKT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oST = oU + align16(sizeof(T) * C * LB);
    static constexpr size_t oUT = oST + align16(sizeof(T) * BV * LK);
    static constexpr size_t oP = oUT + align16(sizeof(T) * BV * LT);
    static constexpr size_t bytes = oP + align16(sizeof(T) * C * LT);
};

template <typename T, int DK, int DV, bool STORE>
__global__ __launch_bounds__(NTHR) void k_scan_fwd(SeqMap sm, int H, Ptrs p) {
    using SM = ScanFwdSmem<T, DK, DV>;
    constexpr int BV = SM::BV, NVT = BV / 32, NKT = DK / 32;
    constexpr int S_TILES = NKT * NVT, S_TPW = (S_TILES + NWAVE - 1) / NWAVE;
    constexpr int U_TILES = 2 * NVT;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sQ = reinterpret_cast<T *>(smem + SM::oQ);
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sW = reinterpret_cast<T *>(smem + SM::oW);
    T *sKT = reinterpret_cast<T *>(smem + SM::oKT);
    T *sU = reinterpret_cast<T *>(smem + SM::oU);
    T *sST = reinterpret_cast<T *>(smem + SM::oST);
    T *sUT = reinterpret_cast<T *>(smem + SM::oUT);
    T *sP = reinterpret_cast<T *>(smem + SM::oP);

    const int vb = blockIdx.x * BV, h = blockIdx.y, n = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int nchunks = (len + C - 1) / C;
    const long chain = (long)n * H + h;

    f32x16 S[S_TPW];
#pragma unroll
    for (int s = 0; s < S_TPW; ++s) {
        S[s] = zero16();
        const int t = wave + s * NWAVE;
        if (t < S_TILES && p.S0) {
            const int a = t / NVT, b = t % NVT;
            const float *src = p.S0 + chain * DK * DV + vb;
            acc_each(S[s], [&](int r, int c, float &val) { val = src[(long)(32 * a + r) * DV + 32 * b + c]; });
        }
    }
    auto publish_state = [&]() { // S -> sST (transposed, operand precision)
#pragma unroll
        for (int s = 0; s < S_TPW; ++s) {
            const int t = wave + s * NWAVE;
            if (t < S_TILES) acc_to_lds_t<T>(sST, SM::LK, 32 * (t / NVT), 32 * (t % NVT), S[s]);
        }
    };
    publish_state();

    for (int ic = 0; ic < nchunks; ++ic) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        const long tile = ((long)(cb + ic) * H + h);
        load_tile<T, C, DK>(sQ, SM::LK, (const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid);
        load_tile<T, C, DK>(sK, SM::LK, (const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid);
        load_tile<T, C, DK>(sW, SM::LK, (const T *)p.W + tile * C * DK, DK, C);
        load_tile<T, C, BV>(sU, SM::LB, (const T *)p.U + tile * C * DV + vb, DV, C);
        if (STORE) { // chunk-initial state for the chunk-parallel backward kernel
            T *dst = (T *)p.Sc + tile * DK * DV + vb;
#pragma unroll
            for (int s = 0; s < S_TPW; ++s) {
                const int t = wave + s * NWAVE;
                if (t < S_TILES) acc_to_global<T>(dst, DV, 32 * (t / NVT), 32 * (t % NVT), DK, S[s]);
            }
        }
        __syncthreads();
        transpose_tile<T, DK>(sKT, SM::LT, sK, SM::LK);
        if (!STORE) { // P = tril(Q K^T), diagonal included (Eq. 9)
            const int a = wave >> 1, b = wave & 1;
            f32x16 acc = zero16();
            if (!(a == 0 && b == 1)) mma_nt<DK>(acc, sQ + 32 * a * SM::LK, SM::LK, sK + 32 * b * SM::LK, SM::LK);
            acc_each(acc, [&](int r, int c, float &val) {
                sP[(32 * a + r) * SM::LT + 32 * b + c] = from_f32<T>((32 * b + c <= 32 * a + r) ? val : 0.f);
            });
        }
        // Ut = U - W S  (inner term of Eq. 8-9)
        for (int t = wave; t < U_TILES; t += NWAVE) {
            const int a = t / NVT, b = t % NVT;
            f32x16 acc = zero16();
            mma_nt<DK>(acc, sW + 32 * a * SM::LK, SM::LK, sST + 32 * b * SM::LK, SM::LK);
            acc_each(acc, [&](int r, int c, float &val) { val = to_f32(sU[(32 * a + r) * SM::LB + 32 * b + c]) - val; });
            acc_to_lds_t<T>(sUT, SM::LT, 32 * a, 32 * b, acc);
            if (STORE) acc_to_global<T>((T *)p.Ut + tile * C * DV + vb, DV, 32 * a, 32 * b, C, acc);
        }
        __syncthreads();
        if (!STORE) { // O = Q S + P Ut (Eq. 9)
            for (int t = wave; t < U_TILES; t += NWAVE) {
                const int a = t / NVT, b = t % NVT;
                f32x16 acc = zero16();
                mma_nt<DK>(acc, sQ + 32 * a * SM::LK, SM::LK, sST + 32 * b * SM::LK, SM::LK);
                if (a == 0) mma_nt<32>(acc, sP, SM::LT, sUT + 32 * b * SM::LT, SM::LT);
                else mma_nt<C>(acc, sP + 32 * SM::LT, SM::LT, sUT + 32 * b * SM::LT, SM::LT);
                acc_to_global<T>((T *)p.o + (row0 * H + h) * DV + vb, (long)H * DV, 32 * a, 32 * b, nvalid, acc);
            }
        }
        // S += K^T Ut (Eq. 8)
#pragma unroll
        for (int s = 0; s < S_TPW; ++s) {
            const int t = wave + s * NWAVE;
            if (t < S_TILES) mma_nt<C>(S[s], sKT + 32 * (t / NVT) * SM::LT, SM::LT, sUT + 32 * (t % NVT) * SM::LT, SM::LT);
        }
        __syncthreads();
        publish_state();
    }
    if (!STORE && p.ST) {
        float *dst = p.ST + chain * DK * DV + vb;
#pragma unroll
        for (int s = 0; s < S_TPW; ++s) {
            const int t = wave + s * NWAVE;
            if (t < S_TILES) acc_to_global<float>(dst, DV, 32 * (t / NVT), 32 * (t % NVT), DK, S[s]);
        }
    }
}

// =============================================================================================
// k_scan_bwd: reverse over chunks, carrying dS (gradient w.r.t. the chunk-initial state).
template <typename T, int DK, int DV> struct ScanBwdSmem {
    static constexpr int BV = VBlock<DV>::BV;
    static constexpr int LK = ldn<T>(DK), LB = ldn<T>(BV), LT = ldn<T>(C);
    static constexpr size_t oQ = 0;
    static constexpr size_t oK = oQ + align16(sizeof(T) * C * LK);
    static constexpr size_t oQT = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oWT = oQT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oDO = oWT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oDOT = oDO + align16(sizeof(T) * C * LB);
    static constexpr size_t oPT = oDOT + align16(sizeof(T) * BV * LT);
    static constexpr size_t oDST = oPT + align16(sizeof(T) * C * LT);
    // W is staged row-major here only until it has been transposed; afterwards the same bytes
    // hold -dUt^T (written two barriers later, read before the barrier that ends the iteration)
    static constexpr size_t oW = oDST + align16(sizeof(T) * BV * LK);
    static constexpr size_t oDUT = oW;
    static constexpr size_t bytes = oW + align16(cmax(sizeof(T) * C * LK, sizeof(T) * BV * LT));
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_scan_bwd(SeqMap sm, int H, Ptrs p) {
    using SM = ScanBwdSmem<T, DK, DV>;
    constexpr int BV = SM::BV, NVT = BV / 32, NKT = DK / 32;
    constexpr int S_TILES = NKT * NVT, S_TPW = (S_TILES + NWAVE - 1) / NWAVE;
    constexpr int U_TILES = 2 * NVT;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sQ = reinterpret_cast<T *>(smem + SM::oQ);
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sW = reinterpret_cast<T *>(smem + SM::oW);
    T *sQT = reinterpret_cast<T *>(smem + SM::oQT);
    T *sWT = reinterpret_cast<T *>(smem + SM::oWT);
    T *sDO = reinterpret_cast<T *>(smem + SM::oDO);
    T *sDOT = reinterpret_cast<T *>(smem + SM::oDOT);
    T *sPT = reinterpret_cast<T *>(smem + SM::oPT);
    T *sDST = reinterpret_cast<T *>(smem + SM::oDST);
    T *sDUT = reinterpret_cast<T *>(smem + SM::oDUT);

    const int vb = blockIdx.x * BV, h = blockIdx.y, n = blockIdx.z;
    const int tid = threadIdx.x, wave = tid >> 6;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int nchunks = (len + C - 1) / C;
    const long chain = (long)n * H + h;

    f32x16 dS[S_TPW];
#pragma unroll
    for (int s = 0; s < S_TPW; ++s) {
        dS[s] = zero16();
        const int t = wave + s * NWAVE;
        if (t < S_TILES && p.dST) {
            const int a = t / NVT, b = t % NVT;
            const float *src = p.dST + chain * DK * DV + vb;
            acc_each(dS[s], [&](int r, int c, float &val) { val = src[(long)(32 * a + r) * DV + 32 * b + c]; });
        }
    }

    for (int ic = nchunks - 1; ic >= 0; --ic) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        const long tile = ((long)(cb + ic) * H + h);
        load_tile<T, C, DK>(sQ, SM::LK, (const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid);
        load_tile<T, C, DK>(sK, SM::LK, (const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid);
        load_tile<T, C, DK>(sW, SM::LK, (const T *)p.W + tile * C * DK, DK, C);
        load_tile<T, C, BV>(sDO, SM::LB, (const T *)p.d_o + (row0 * H + h) * DV + vb, (long)H * DV, nvalid);
        { // dS' (gradient w.r.t. the state after this chunk): to the workspace and, transposed, to LDS
            T *dst = (T *)p.dSc + tile * DK * DV + vb;
#pragma unroll
            for (int s = 0; s < S_TPW; ++s) {
                const int t = wave + s * NWAVE;
                if (t < S_TILES) {
                    acc_to_global<T>(dst, DV, 32 * (t / NVT), 32 * (t % NVT), DK, dS[s]);
                    acc_to_lds_t<T>(sDST, SM::LK, 32 * (t / NVT), 32 * (t % NVT), dS[s]);
                }
            }
        }
        __syncthreads();
        transpose_tile<T, DK>(sQT, SM::LT, sQ, SM::LK);
        transpose_tile<T, DK>(sWT, SM::LT, sW, SM::LK);
        transpose_tile<T, BV>(sDOT, SM::LT, sDO, SM::LB);
        { // P^T, P = tril(Q K^T)
            const int a = wave >> 1, b = wave & 1;
            f32x16 acc = zero16();
            if (!(a == 0 && b == 1)) mma_nt<DK>(acc, sQ + 32 * a * SM::LK, SM::LK, sK + 32 * b * SM::LK, SM::LK);
            acc_each(acc, [&](int r, int c, float &val) { if (32 * b + c > 32 * a + r) val = 0.f; });
            acc_to_lds_t<T>(sPT, SM::LT, 32 * a, 32 * b, acc);
        }
        __syncthreads();
        // dUt = P^T dO + K dS'; kept negated in LDS for the state update below
        for (int t = wave; t < U_TILES; t += NWAVE) {
            const int a = t / NVT, b = t % NVT;
            f32x16 acc = zero16();
            if (a == 1) mma_nt<32>(acc, sPT + 32 * SM::LT + 32, SM::LT, sDOT + 32 * b * SM::LT + 32, SM::LT);
            else mma_nt<C>(acc, sPT, SM::LT, sDOT + 32 * b * SM::LT, SM::LT);
            mma_nt<DK>(acc, sK + 32 * a * SM::LK, SM::LK, sDST + 32 * b * SM::LK, SM::LK);
            acc_to_global<T>((T *)p.dUt + tile * C * DV + vb, DV, 32 * a, 32 * b, C, acc);
            acc_each(acc, [&](int, int, float &val) { val = -val; });
            acc_to_lds_t<T>(sDUT, SM::LT, 32 * a, 32 * b, acc);
        }
        __syncthreads();
        // dS = dS' + Q^T dO - W^T dUt
#pragma unroll
        for (int s = 0; s < S_TPW; ++s) {
            const int t = wave + s * NWAVE;
            if (t < S_TILES) {
                const int a = t / NVT, b = t % NVT;
                mma_nt<C>(dS[s], sQT + 32 * a * SM::LT, SM::LT, sDOT + 32 * b * SM::LT, SM::LT);
                mma_nt<C>(dS[s], sWT + 32 * a * SM::LT, SM::LT, sDUT + 32 * b * SM::LT, SM::LT);
            }
        }
        __syncthreads();
    }
    if (p.dS0) {
        float *dst = p.dS0 + chain * DK * DV + vb;
#pragma unroll
        for (int s = 0; s < S_TPW; ++s) {
            const int t = wave + s * NWAVE;
            if (t < S_TILES) acc_to_global<float>(dst, DV, 32 * (t / NVT), 32 * (t % NVT), DK, dS[s]);
        }
    }
}

// =============================================================================================
// k_bwd_dqkw: per chunk, with S (chunk-initial state), dS' (gradient w.r.t. the state after the
// chunk), Ut, dUt:  dP = tril(dO Ut^T); dQ = dO S^T + dP K; dK1 = dP^T Q + Ut dS'^T; dW = -dUt S^T.
template <typename T, int DK, int DV> struct DqkwSmem {
    static constexpr int LK = ldn<T>(DK), LV = ldn<T>(DV), LT = ldn<T>(C);
    static constexpr size_t oDO = 0;
    static constexpr size_t oUt = oDO + align16(sizeof(T) * C * LV);
    static constexpr size_t oDUt = oUt + align16(sizeof(T) * C * LV);
    static constexpr size_t oKT = oDUt + align16(sizeof(T) * C * LV);
    static constexpr size_t oQT = oKT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oDP = oQT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oDPT = oDP + align16(sizeof(T) * C * LT);
    static constexpr size_t oS = oDPT + align16(sizeof(T) * C * LT); // K,Q staging, then S, then dS'
    static constexpr size_t szS = cmax(sizeof(T) * DK * LV, 2 * align16(sizeof(T) * C * LK));
    static constexpr size_t bytes = oS + align16(szS);
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_bwd_dqkw(SeqMap sm, int H, Ptrs p) {
    using SM = DqkwSmem<T, DK, DV>;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sDO = reinterpret_cast<T *>(smem + SM::oDO);
    T *sUt = reinterpret_cast<T *>(smem + SM::oUt);
    T *sDUt = reinterpret_cast<T *>(smem + SM::oDUt);
    T *sKT = reinterpret_cast<T *>(smem + SM::oKT);
    T *sQT = reinterpret_cast<T *>(smem + SM::oQT);
    T *sDP = reinterpret_cast<T *>(smem + SM::oDP);
    T *sDPT = reinterpret_cast<T *>(smem + SM::oDPT);
    T *sS = reinterpret_cast<T *>(smem + SM::oS);
    T *sKn = sS;
    T *sQn = reinterpret_cast<T *>(smem + SM::oS + align16(sizeof(T) * C * SM::LK));

    int n, ic;
    if (!sm.chunk(blockIdx.x, n, ic)) return;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int h = blockIdx.y, tid = threadIdx.x, wave = tid >> 6;
    const int nvalid = min(C, len - ic * C);
    const long row0 = (long)t0 + (long)ic * C;
    const long tile = ((long)(cb + ic) * H + h);

    load_tile<T, C, DV>(sDO, SM::LV, (const T *)p.d_o + (row0 * H + h) * DV, (long)H * DV, nvalid);
    load_tile<T, C, DV>(sUt, SM::LV, (const T *)p.Ut + tile * C * DV, DV, C);
    load_tile<T, C, DV>(sDUt, SM::LV, (const T *)p.dUt + tile * C * DV, DV, C);
    load_tile<T, C, DK>(sKn, SM::LK, (const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid);
    load_tile<T, C, DK>(sQn, SM::LK, (const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid);
    __syncthreads();
    transpose_tile<T, DK>(sKT, SM::LT, sKn, SM::LK);
    transpose_tile<T, DK>(sQT, SM::LT, sQn, SM::LK);
    { // dP = tril(dO Ut^T), both orientations
        const int a = wave >> 1, b = wave & 1;
        f32x16 acc = zero16();
        if (!(a == 0 && b == 1)) mma_nt<DV>(acc, sDO + 32 * a * SM::LV, SM::LV, sUt + 32 * b * SM::LV, SM::LV);
        acc_each(acc, [&](int r, int c, float &val) { if (32 * b + c > 32 * a + r) val = 0.f; });
        acc_to_lds<T>(sDP, SM::LT, 32 * a, 32 * b, acc);
        acc_to_lds_t<T>(sDPT, SM::LT, 32 * a, 32 * b, acc);
    }
    __syncthreads();
    load_tile<T, DK, DV>(sS, SM::LV, (const T *)p.Sc + tile * DK * DV, DV, DK);
    __syncthreads();
    for (int t = wave; t < 2 * (DK / 32); t += NWAVE) {
        const int a = t / (DK / 32), b = t % (DK / 32);
        f32x16 acc = zero16(); // dQ = dO S^T + dP K
        mma_nt<DV>(acc, sDO + 32 * a * SM::LV, SM::LV, sS + 32 * b * SM::LV, SM::LV);
        if (a == 0) mma_nt<32>(acc, sDP, SM::LT, sKT + 32 * b * SM::LT, SM::LT);
        else mma_nt<C>(acc, sDP + 32 * SM::LT, SM::LT, sKT + 32 * b * SM::LT, SM::LT);
        acc_to_global<T>((T *)p.dq + (row0 * H + h) * DK, (long)H * DK, 32 * a, 32 * b, nvalid, acc);
        f32x16 w = zero16(); // dW = -dUt S^T
        mma_nt<DV>(w, sDUt + 32 * a * SM::LV, SM::LV, sS + 32 * b * SM::LV, SM::LV);
        acc_each(w, [&](int, int, float &val) { val = -val; });
        acc_to_global<T>((T *)p.dW + tile * C * DK, DK, 32 * a, 32 * b, C, w);
    }
    __syncthreads();
    load_tile<T, DK, DV>(sS, SM::LV, (const T *)p.dSc + tile * DK * DV, DV, DK);
    __syncthreads();
    for (int t = wave; t < 2 * (DK / 32); t += NWAVE) {
        const int a = t / (DK / 32), b = t % (DK / 32);
        f32x16 acc = zero16(); // dK1 = dP^T Q + Ut dS'^T
        if (a == 1) mma_nt<32>(acc, sDPT + 32 * SM::LT + 32, SM::LT, sQT + 32 * b * SM::LT + 32, SM::LT);
        else mma_nt<C>(acc, sDPT, SM::LT, sQT + 32 * b * SM::LT, SM::LT);
        mma_nt<DV>(acc, sUt + 32 * a * SM::LV, SM::LV, sS + 32 * b * SM::LV, SM::LV);
        acc_to_global<T>((T *)p.dK1 + tile * C * DK, DK, 32 * a, 32 * b, C, acc);
    }
}

// =============================================================================================
// k_bwd_wy: adjoint of the UT transform (Eq. 10-11).  With X = (I+A)^-1, A = tril(diag(beta) G,-1),
// G = K K^T, W = X diag(beta) K, U = X diag(beta) V and incoming dW, dU (= dUt):
//   dX' = dW K^T + dU V^T;  dX = dX' diag(beta);  dKb = X^T dW;  dVb = X^T dU;
//   dA = -tril(X^T dX X^T, -1);  Ah = diag(beta) dA;
//   dK = dK1 + diag(beta) dKb + (Ah + Ah^T) K;  dV = diag(beta) dVb;
//   dbeta_i = sum_m X[m][i] dX'[m][i] + sum_j dA[i][j] G[i][j].
template <typename T, int DK, int DV> struct WySmem {
    static constexpr int LK = ldn<T>(DK), LV = ldn<T>(DV), LT = ldn<T>(C), LF = C + 4, LM = 52;
    // region N: phase 1 = K, V, dW, dU row-major; phase 2 = A, X, G (fp32), inverse scratch, M1^T
    static constexpr size_t p1K = 0;
    static constexpr size_t p1V = p1K + align16(sizeof(T) * C * LK);
    static constexpr size_t p1dW = p1V + align16(sizeof(T) * C * LV);
    static constexpr size_t p1dU = p1dW + align16(sizeof(T) * C * LK);
    static constexpr size_t p1end = p1dU + align16(sizeof(T) * C * LV);
    static constexpr size_t p2A = 0;
    static constexpr size_t p2X = p2A + sizeof(float) * C * LF;
    static constexpr size_t p2G = p2X + sizeof(float) * C * LF;
    static constexpr size_t p2M = p2G + sizeof(float) * C * LF;
    static constexpr size_t p2M1T = p2A; // M1^T overwrites A once the inverse is done
    static constexpr size_t p2end = p2M + align16(sizeof(float) * 16 * LM);
    static constexpr size_t oKT = align16(cmax(p1end, p2end));
    static constexpr size_t oDWT = oKT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oDUT = oDWT + align16(sizeof(T) * DK * LT);
    static constexpr size_t oXn = oDUT + align16(sizeof(T) * DV * LT);
    // in fp32 the inverse itself (same leading dimension) serves as the row-major operand copy
    static constexpr bool kXnIsX = sizeof(T) == sizeof(float);
    static constexpr size_t oXT = oXn + (kXnIsX ? 0 : align16(sizeof(T) * C * LT));
    static constexpr size_t oDX = oXT + align16(sizeof(T) * C * LT); // dX, later Ah + Ah^T
    static constexpr size_t oBeta = oDX + align16(sizeof(T) * C * LT);
    static constexpr size_t oDb = oBeta + sizeof(float) * C;
    static constexpr size_t bytes = oDb + sizeof(float) * 4 * C; // one slot per (row tile, lane half)
};

template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_bwd_wy(SeqMap sm, int H, Ptrs p) {
    using SM = WySmem<T, DK, DV>;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sK = reinterpret_cast<T *>(smem + SM::p1K);
    T *sV = reinterpret_cast<T *>(smem + SM::p1V);
    T *sDW = reinterpret_cast<T *>(smem + SM::p1dW);
    T *sDU = reinterpret_cast<T *>(smem + SM::p1dU);
    float *sA = reinterpret_cast<float *>(smem + SM::p2A);
    float *sX = reinterpret_cast<float *>(smem + SM::p2X);
    float *sG = reinterpret_cast<float *>(smem + SM::p2G);
    float *sM = reinterpret_cast<float *>(smem + SM::p2M);
    T *sM1T = reinterpret_cast<T *>(smem + SM::p2M1T);
    T *sKT = reinterpret_cast<T *>(smem + SM::oKT);
    T *sDWT = reinterpret_cast<T *>(smem + SM::oDWT);
    T *sDUT = reinterpret_cast<T *>(smem + SM::oDUT);
    T *sXn = SM::kXnIsX ? reinterpret_cast<T *>(smem + SM::p2X) : reinterpret_cast<T *>(smem + SM::oXn);
    static_assert(!SM::kXnIsX || SM::LT == SM::LF, "fp32 operand copy aliases the inverse");
    T *sXT = reinterpret_cast<T *>(smem + SM::oXT);
    T *sDX = reinterpret_cast<T *>(smem + SM::oDX);
    float *sBeta = reinterpret_cast<float *>(smem + SM::oBeta);
    float *sDb = reinterpret_cast<float *>(smem + SM::oDb);

    int n, ic;
    if (!sm.chunk(blockIdx.x, n, ic)) return;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int h = blockIdx.y, tid = threadIdx.x, wave = tid >> 6;
    const int nvalid = min(C, len - ic * C);
    const long row0 = (long)t0 + (long)ic * C;
    const long tile = ((long)(cb + ic) * H + h);
    const int mi = wave >> 1, ni = wave & 1; // this wave's 32x32 tile of every C x C matrix
    const bool upper = (mi == 0 && ni == 1);

    load_tile<T, C, DK>(sK, SM::LK, (const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid);
    load_tile<T, C, DV>(sV, SM::LV, (const T *)p.v + (row0 * H + h) * DV, (long)H * DV, nvalid);
    load_tile<T, C, DK>(sDW, SM::LK, (const T *)p.dW + tile * C * DK, DK, C);
    load_tile<T, C, DV>(sDU, SM::LV, (const T *)p.dUt + tile * C * DV, DV, C);
    if (tid < C) {
        sBeta[tid] = tid < nvalid ? to_f32(((const T *)p.beta)[(row0 + tid) * H + h]) : 0.f;
    }
    __syncthreads();
    f32x16 g = zero16(), dxp = zero16();
    if (!upper) {
        mma_nt<DK>(g, sK + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK);
        mma_nt<DK>(dxp, sDW + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK);
        mma_nt<DV>(dxp, sDU + 32 * mi * SM::LV, SM::LV, sV + 32 * ni * SM::LV, SM::LV);
    }
    transpose_tile<T, DK>(sKT, SM::LT, sK, SM::LK);
    transpose_tile<T, DK>(sDWT, SM::LT, sDW, SM::LK);
    transpose_tile<T, DV>(sDUT, SM::LT, sDU, SM::LV);
    __syncthreads(); // phase 1 buffers are dead
    acc_each(g, [&](int r, int c, float &val) {
        const int i = 32 * mi + r, j = 32 * ni + c;
        const float gij = j < i ? val : 0.f;
        sG[i * SM::LF + j] = gij;
        sA[i * SM::LF + j] = sBeta[i] * gij;
    });
    __syncthreads();
    tri_inverse_64(sA, sX, sM, SM::LF, SM::LM);
    for (int e = tid; e < C * C; e += NTHR) {
        const int i = e >> 6, j = e & 63;
        const T x = from_f32<T>(sX[i * SM::LF + j]);
        if (!SM::kXnIsX) sXn[i * SM::LT + j] = x;
        sXT[j * SM::LT + i] = x;
    }
    { // dbeta part 1 (column sums of X o dX') and dX = dX' diag(beta)
        const int lane = tid & 63, c = lane & 31;
        float part = 0.f;
        acc_each(dxp, [&](int r, int cc, float &val) {
            const int i = 32 * mi + r, j = 32 * ni + cc;
            part += sX[i * SM::LF + j] * val;
            val *= sBeta[j];
        });
        sDb[(2 * mi + (lane >> 5)) * C + 32 * ni + c] = part; // summed in a fixed order at the end
        acc_to_lds<T>(sDX, SM::LT, 32 * mi, 32 * ni, dxp);
    }
    __syncthreads();
    { // M1 = dX X^T, stored transposed
        f32x16 acc = zero16();
        mma_nt<C>(acc, sDX + 32 * mi * SM::LT, SM::LT, sXn + 32 * ni * SM::LT, SM::LT);
        acc_to_lds_t<T>(sM1T, SM::LT, 32 * mi, 32 * ni, acc);
    }
    constexpr int KB_TILES = 2 * (DK / 32), KB_TPW = (KB_TILES + NWAVE - 1) / NWAVE;
    f32x16 dKb[KB_TPW];
#pragma unroll
    for (int s = 0; s < KB_TPW; ++s) { // dKb = X^T dW (X^T is upper triangular)
        dKb[s] = zero16();
        const int t = wave + s * NWAVE;
        if (t < KB_TILES) {
            const int a = t / (DK / 32), b = t % (DK / 32);
            if (a == 1) mma_nt<32>(dKb[s], sXT + 32 * SM::LT + 32, SM::LT, sDWT + 32 * b * SM::LT + 32, SM::LT);
            else mma_nt<C>(dKb[s], sXT, SM::LT, sDWT + 32 * b * SM::LT, SM::LT);
        }
    }
    for (int t = wave; t < 2 * (DV / 32); t += NWAVE) { // dV = diag(beta) X^T dU
        const int a = t / (DV / 32), b = t % (DV / 32);
        f32x16 acc = zero16();
        if (a == 1) mma_nt<32>(acc, sXT + 32 * SM::LT + 32, SM::LT, sDUT + 32 * b * SM::LT + 32, SM::LT);
        else mma_nt<C>(acc, sXT, SM::LT, sDUT + 32 * b * SM::LT, SM::LT);
        acc_each(acc, [&](int r, int, float &val) { val *= sBeta[32 * a + r]; });
        acc_to_global<T>((T *)p.dv + (row0 * H + h) * DV, (long)H * DV, 32 * a, 32 * b, nvalid, acc);
    }
    __syncthreads();
    { // dA = -tril(X^T M1, -1); dbeta part 2 products into sG; Ah + Ah^T into sDX
        f32x16 acc = zero16();
        if (!upper) {
            if (mi == 1) mma_nt<32>(acc, sXT + 32 * SM::LT + 32, SM::LT, sM1T + 32 * ni * SM::LT + 32, SM::LT);
            else mma_nt<C>(acc, sXT, SM::LT, sM1T + 32 * ni * SM::LT, SM::LT);
        }
        acc_each(acc, [&](int r, int c, float &val) {
            const int i = 32 * mi + r, j = 32 * ni + c;
            const float da = j < i ? -val : 0.f;
            sG[i * SM::LF + j] *= da; // dA o G, summed by rows below
            if (!upper) {
                if (j < i) {
                    const T ah = from_f32<T>(sBeta[i] * da);
                    sDX[i * SM::LT + j] = ah;
                    sDX[j * SM::LT + i] = ah;
                } else if (j == i) {
                    sDX[i * SM::LT + i] = from_f32<T>(0.f);
                }
            }
        });
    }
    __syncthreads();
#pragma unroll
    for (int s = 0; s < KB_TPW; ++s) { // dK = dK1 + diag(beta) dKb + (Ah + Ah^T) K
        const int t = wave + s * NWAVE;
        if (t < KB_TILES) {
            const int a = t / (DK / 32), b = t % (DK / 32);
            const T *k1 = (const T *)p.dK1 + tile * C * DK;
            acc_each(dKb[s], [&](int r, int c, float &val) {
                val = val * sBeta[32 * a + r] + to_f32(k1[(32 * a + r) * DK + 32 * b + c]);
            });
            mma_nt<C>(dKb[s], sDX + 32 * a * SM::LT, SM::LT, sKT + 32 * b * SM::LT, SM::LT);
            acc_to_global<T>((T *)p.dk + (row0 * H + h) * DK, (long)H * DK, 32 * a, 32 * b, nvalid, dKb[s]);
        }
    }
    { // dbeta = column sums from part 1 + row sums of dA o G
        const int i = tid >> 2, seg = tid & 3;
        float s = 0.f;
#pragma unroll
        for (int j = 0; j < 16; ++j) s += sG[i * SM::LF + seg * 16 + j];
        s += __shfl_xor(s, 1);
        s += __shfl_xor(s, 2);
        if (seg == 0 && i < nvalid)
            p.dbeta[(row0 + i) * H + h] = s + ((sDb[i] + sDb[C + i]) + (sDb[2 * C + i] + sDb[3 * C + i]));
    }
}

} // namespace dn
