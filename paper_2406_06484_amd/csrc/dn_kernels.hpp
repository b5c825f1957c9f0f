// The kernels of the chunkwise DeltaNet forward/backward (gfx950), templated on the element
// type T (float: fp32 MFMA; bf16: bf16 MFMA with fp32 accumulation) and the head dims.
//
//   k_wy_prep    per chunk            A = tril(diag(beta) K K^T,-1); X = (I+A)^-1; T = X diag(beta); P = tril(Q K^T)   (Eq. 10)
//   k_scan_fwd   per chain x v-block  serial over chunks: W = T K, U = T V (Eq. 11); Ut = U - W S; O = Q S + P Ut; S += K^T Ut  (Eq. 8-9)
//   k_scan_pair  per chain x v-block  backward: the state-recompute scan (stores chunk-initial S and Ut) and the reverse
//                                     scan (dUt = P^T dO + K dS'; dS = dS' + Q^T dO - W^T dUt) as one grid
//   k_scan_fwd_save / k_scan_bwd      the forward scan that also stores what the recompute scan would, and the reverse
//                                     scan alone, for a backward pass that keeps the forward pass's tiles
//   k_bwd_chunk  per chunk            adjoint of Eq. 8-9 given S, dS', Ut, dUt, then adjoint of Eq. 10-11: dQ, dK, dV, dbeta
//
// State S is [d_k][d_v] (orientation of the paper's pseudocode listing), fp32 in registers.
#pragma once
#include "dn_device.hpp"
#include "dn_host.hpp"

namespace dn {

constexpr int cmax(int a, int b) { return a > b ? a : b; }
// Kernel variants (a compile-time template argument, so that each carries only its own registers):
// the plain delta rule; the gated rule; the plain rule with the layer's prologue (q, k = SiLU(x) /
// ||SiLU(x)||_2 of section 3.3, beta = sigmoid(b) of section 2.2).  For the prologue k_wy_prep maps q
// and k once and leaves them in the workspace for the scans, which run the plain variant on them;
// k_bwd_chunk maps its tiles itself on the way to LDS and sends the gradients back through the map on
// the way out, so dq, dk never reach HBM in the mapped coordinates.
enum { VAR_PLAIN = 0, VAR_GATED = 1, VAR_PROLOGUE = 2 };
constexpr size_t align16(size_t x) { return (x + 15) & ~size_t(15); }

// ---------------------------------------------------------------------------------------------
// Packed layout, one workgroup.  The caller's offsets are first bounded: cus[n] = the running maximum of cu[0..n], held
// inside [0, L].  For a valid array (0 = cu[0] <= cu[1] <= ... <= cu[N] = L) that is the array itself; a malformed one that
// no host copy was there to reject becomes some non-decreasing sequence inside the tensors, so that every row index and
// every workspace tile the other kernels derive from it stays in bounds (the results are then meaningless).  Every other
// kernel reads cus, never cu.  Then the per-sequence chunk-count prefix coff[n] = sum_{m<n} ceil(len_m / C) and, behind
// it, order[i] = the i-th longest sequence (ties by index): the chain-serial kernels start the long chains first, so
// that the short ones fill the tail (up to kMaxOrdered sequences; more than that balance by themselves and keep their order).
// Workspace: coff [N + 1], order [N], cus [N + 1].
constexpr int kMaxOrdered = 512;
static __global__ void k_chunk_offsets(const int32_t *cu_in, int N, int L, int32_t *coff) {
    int32_t *order = coff + N + 1, *cu = order + N;
    __shared__ int part[NTHR];
    const int tid = threadIdx.x;
    {
        const int per1 = (N + 1 + NTHR - 1) / NTHR, lo1 = tid * per1, hi1 = min(N + 1, lo1 + per1);
        int m = 0;
        for (int n = lo1; n < hi1; ++n) m = max(m, min(cu_in[n], L));
        part[tid] = m;
        __syncthreads();
        if (tid == 0) {
            int run = 0;
            for (int i = 0; i < NTHR; ++i) { const int t = part[i]; part[i] = run; run = max(run, t); }
        }
        __syncthreads();
        int run = part[tid];
        for (int n = lo1; n < hi1; ++n) { run = max(run, min(cu_in[n], L)); cu[n] = run; }
        __syncthreads();
    }
    if (N <= kMaxOrdered) {
        for (int n = threadIdx.x; n < N; n += NTHR) {
            const int len = cu[n + 1] - cu[n];
            int rank = 0;
            for (int m = 0; m < N; ++m) {
                const int lm = cu[m + 1] - cu[m];
                rank += (lm > len) || (lm == len && m < n);
            }
            order[rank] = n;
        }
    } else {
        for (int n = threadIdx.x; n < N; n += NTHR) order[n] = n;
    }
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

// final_state of a pass over no tokens at all: the initial state, or zero
static __global__ void k_state_copy(float *dst, const float *src, long count) {
    for (long i = (long)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (long)gridDim.x * blockDim.x) dst[i] = src ? src[i] : 0.f;
}

// =============================================================================================
// k_wy_prep: per chunk, T = (I + tril(diag(beta) K K^T, -1))^-1 diag(beta) (Eq. 10).
// W = T K and U = T V (Eq. 11) are rebuilt from T inside the scan kernels: T is 8 KB per chunk
// where W and U are 32 KB.  In the backward pass the inverse X itself is stored as well, so that the
// chunk kernel does not have to invert again.
template <typename T, int DK, int DV> struct PrepSmem {
    static constexpr int LD = ldc<T>(DK), LF = C + 4, LO = 40;
    // region 1: K while the two Gram products run, then the fp32 matrix that is inverted in place
    static constexpr size_t oK = 0, oX = 0;
    static constexpr size_t sz1 = cmax(sizeof(T) * C * LD, sizeof(float) * C * LF);
    // region 2: the operands of the inverse's MFMA stage
    static constexpr size_t oOp = oX + align16(sz1);
    static constexpr size_t sz2 = cmax(sizeof(T) * 3 * 32 * LO, sizeof(float) * 512); // ... and, before that, the merges' scratch
    static constexpr size_t oM = oOp;
    static constexpr size_t oBeta = oOp + align16(sz2);
    static constexpr size_t bytes = oBeta + sizeof(float) * C;
};

// (bf16 up to d_k = 128: held to the registers of six workgroups per CU, which is what its LDS allows; the other
// instantiations would spill under that cap)
template <typename T, int DK> struct PrepWaves { static constexpr int lo = (sizeof(T) == 2 && DK <= 128) ? 6 : 1, hi = (sizeof(T) == 2 && DK <= 128) ? 6 : 8; };
template <typename T, int DK, int DV>
__global__ __launch_bounds__(NTHR) __attribute__((amdgpu_waves_per_eu(PrepWaves<T, DK>::lo, PrepWaves<T, DK>::hi))) void k_wy_prep(SeqMap sm, int H, Ptrs p) {
    using SM = PrepSmem<T, DK, DV>;
    extern __shared__ __align__(16) unsigned char smem[];
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    float *sX = reinterpret_cast<float *>(smem + SM::oX);
    T *sOp = reinterpret_cast<T *>(smem + SM::oOp);
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
    const int mi = wave >> 1, ni = wave & 1; // this wave's 32 x 32 tile of the C x C matrices
    const bool upper = mi == 0 && ni == 1;

    {
        TileRegs<T, C, DK> kr;
        kr.template load_aux<kAuxKeep>((const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid, threadIdx.x);
        if (p.pro) { // prologue variant: q and k arrive before the feature map of section 3.3
            TileRegs<T, C, DK> qr;
            qr.load((const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid);
            float inv[TileRegs<T, C, DK>::NIT];
            kr.feature_map(inv);
            kr.store_global((T *)p.Km + (row0 * H + h) * DK, (long)H * DK, nvalid);
            qr.feature_map(inv);
            qr.store_global((T *)p.Qm + (row0 * H + h) * DK, (long)H * DK, nvalid);
        }
        kr.store(sK, SM::LD);
    }
    if (tid < C) {
        float b = tid < nvalid ? to_f32(((const T *)p.beta)[(row0 + tid) * H + h]) : 0.f;
        if (p.pro) b = tid < nvalid ? sigmoid_f32(b) : 0.f; // ... and beta before the sigmoid
        sBeta[tid] = b;
    }
    if (p.g && tid < C) {
        // Gated variant: with the running decay exp(g_1 + ... + g_i) within the chunk (rows past the end keep the last
        // value), the state divided by it follows the plain delta rule on equally divided values, so the other kernels
        // only rescale rows with gamma_i and 1 / gamma_i; T and X do not depend on the gate.  The table holds the decay
        // relative to the chunk's geometric middle, gamma_i = exp(g_1 + ... + g_i - (g_1 + ... + g_C) / 2): both
        // gamma_i and 1 / gamma_i then stay within exp(+-sum|g| / 2), which doubles the decay per chunk that fp32 holds.
        // The chain scans move the state into these coordinates when a chunk begins (factor gamma_C, which in them is
        // also the decay from the chunk's start to its middle) and out of them when it ends (gamma_C again).
        float cs = tid < nvalid ? p.g[(row0 + tid) * H + h] : 0.f;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const float up = __shfl_up(cs, d);
            if (tid >= d) cs += up;
        }
        const float half = 0.5f * __shfl(cs, C - 1);
        p.gam[tile * 2 * C + tid] = __expf(cs - half);
        p.gam[tile * 2 * C + C + tid] = __expf(half - cs);
    }
    lds_barrier();
    f32x16 g = zero16();
    if (!upper) mma<DK, false, false, T>(g, sK + 32 * mi * SM::LD, SM::LD, sK + 32 * ni * SM::LD, SM::LD); // K K^T
    lds_barrier(); // K is dead from here on; its bytes take the fp32 matrix
    acc_each(g, [&](int r, int c, float &val) { // A = tril(diag(beta) K K^T, -1)
        const int i = 32 * mi + r, j = 32 * ni + c;
        sX[i * SM::LF + j] = j < i ? sBeta[i] * val : 0.f;
    });
    lds_barrier();
    tri_inverse_64_inplace<T>(sX, SM::LF, sM, sOp, SM::LO);
    // T = X diag(beta), and X itself for the backward pass, converted and written 16 bytes at a time
    constexpr int VEC = El<T>::VEC, SEGS = C / VEC;
    for (int e = tid; e < C * SEGS; e += NTHR) {
        const int i = e / SEGS, j0 = (e % SEGS) * VEC;
        alignas(16) T tv[VEC], xv[VEC];
#pragma unroll
        for (int u = 0; u < VEC; ++u) {
            const float x = sX[i * SM::LF + j0 + u];
            tv[u] = from_f32<T>(x * sBeta[j0 + u]);
            xv[u] = from_f32<T>(x);
        }
        __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(tv), reinterpret_cast<u32x4 *>((T *)p.Tm + tile * C * C + i * C + j0));
        if (p.want_x) __builtin_nontemporal_store(*reinterpret_cast<const u32x4 *>(xv), reinterpret_cast<u32x4 *>((T *)p.Xm + tile * C * C + i * C + j0));
    }
}

// =============================================================================================
// The two chain-serial kernels.  One workgroup of 8 wavefronts owns one chain and BV = 64 columns
// of the state; the state lives in accumulator registers, one 32 x 32 tile per wave.
// Waves 0..3 own the Ut / dUt tiles of the dependent chain; waves 4..7 have the lighter work between
// barriers and double as loaders: they request the next chunk's tiles and send most of the results
// out of LDS, so that the chain waves do not queue behind the CU's 64 B/clk vector-memory path in the
// intervals whose length they set (the one exception: the kept Ut / dUt tile of the previous step
// leaves through the chain waves in the last interval, where the loader waves are the busier side).
// W = T K (Eq. 11) is rebuilt per chunk from the 64 x 64 T.
// Workgroup ids are laid out so that the v-blocks of one chain land on the same XCD (ids are dealt
// round-robin over the 8 XCDs) and share its L2 for the Q, K, T tiles they both read.
constexpr int NTS = 512, NWS = 8, NTL = 256; // threads / waves of a scan workgroup; loader threads
// bf16 workgroups own 64 state columns; fp32 ones, and bf16 ones with d_k = 256, own 32, so that the
// tiles (whose rows are d_k long) still fit the 160 KB of LDS
template <typename T, int DV, int DK> struct VBlock {
    static constexpr int WANT = (sizeof(T) == 2 && DK <= 128) ? DN_VBLOCK_COLS : 32;
    static constexpr int BV = DV < WANT ? DV : WANT;
    static constexpr int NV = DV / BV;
};

__device__ inline bool chain_of_block(int bid, int nchains, int nv, int &chain, int &vbi) {
    const int xcd = bid & 7, slot = bid >> 3;
    vbi = slot % nv;
    chain = (slot / nv) * 8 + xcd;
    return chain < nchains;
}
__host__ inline int chain_grid(int nchains, int nv) { return ((nchains + 7) / 8) * 8 * nv; }

// Which tiles a scan wave owns.  State tile (sa, sb): rows 32*sa of d_k, cols 32*sb of the v-block.
// W tile: d_k block wk, chunk-row block wi.  Waves < U_TILES own U / Ut tile (ua, ub); waves 4..
// own the tile of O (forward) of the same shape.
template <int DK, int BV> struct ScanMap {
    static constexpr int NVT = BV / 32, NKT = DK / 32, S_TILES = NKT * NVT, U_TILES = 2 * NVT, W_TILES = 2 * NKT;
    static_assert(S_TILES <= NWS && U_TILES <= 4, "state tiling");
    int sa, sb, ua, ub;
    bool has_s, does_u, does_o;
    __device__ ScanMap(int wave) {
        sa = wave / NVT; sb = wave % NVT; has_s = wave < S_TILES;
        const int u = wave & 3;
        ua = u / NVT; ub = u % NVT;
        does_u = wave < U_TILES; does_o = wave >= 4 && u < U_TILES;
    }
};

// scan_fwd_body: MODE = SCAN_OUT writes O and the final state; SCAN_STORE (the backward's recompute pass)
// writes every chunk-initial state and Ut to the workspace instead of O; SCAN_BOTH (a forward pass whose
// backward pass will not recompute) does both; SCAN_STATE writes only the final state (the first pass of a
// forward pass that is split over segments of the sequence, see k_scan_state).
enum { SCAN_OUT = 0, SCAN_STORE = 1, SCAN_BOTH = 2, SCAN_STATE = 3 };
template <typename T, int DK, int DV> struct ScanFwdSmem {
    static constexpr int BV = VBlock<T, DV, DK>::BV;
    static constexpr int LQ = ldc<T>(DK), LK = ldn<T>(DK), LV = ldn<T>(BV), LS = ldc<T>(DK), LT = ldc<T>(C);
    static constexpr size_t oQ = 0;
    static constexpr size_t oK = oQ + align16(sizeof(T) * C * LQ);
    static constexpr size_t oV = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oW = oV + align16(sizeof(T) * C * LV);
    static constexpr size_t oST = oW + align16(sizeof(T) * C * LQ);
    static constexpr size_t oUT = oST + align16(sizeof(T) * BV * LS);
    static constexpr size_t szUT = align16(sizeof(T) * BV * LT);     // two Ut^T buffers, alternating by chunk parity
    static constexpr size_t oT = oUT + 2 * szUT;
    static constexpr size_t oP = oT + align16(sizeof(T) * C * LT);
    static constexpr size_t oStage = oP + align16(sizeof(T) * C * LT); // per-wave output staging tiles
    static constexpr int NSTG = ScanMap<DK, BV>::U_TILES; // only the output waves stage tiles
    static constexpr size_t oGam = oStage + NSTG * sizeof(T) * Stage<T>::ELEMS; // gated: gamma_i, 1 / gamma_i of the chunk
    static constexpr size_t bytes1 = oGam + sizeof(float) * 2 * C;
    // Where a second K tile and a second gamma table fit, the tiles of the next chunk move to LDS in the interval that
    // updates the state (which still reads the current K), and a chunk step takes three barrier intervals instead of four.
    static constexpr size_t szK = align16(sizeof(T) * C * LK);
    static constexpr bool kMerge = bytes1 + szK + sizeof(float) * 2 * C <= 160 * 1024;
    static constexpr size_t oK2 = bytes1, oGam2 = oK2 + szK;
    static constexpr size_t bytes = kMerge ? oGam2 + sizeof(float) * 2 * C : bytes1;
};

template <typename T, int DK, int DV, int MODE, int VAR>
__device__ __forceinline__ void scan_fwd_body(const SeqMap &sm, int H, const Ptrs &p, int bid) {
    using SM = ScanFwdSmem<T, DK, DV>;
    static_assert(VAR != VAR_PROLOGUE, "the scans read q and k already mapped");
    constexpr bool GATED = VAR == VAR_GATED;
    constexpr bool OUT = MODE == SCAN_OUT || MODE == SCAN_BOTH, SAVE = MODE == SCAN_STORE || MODE == SCAN_BOTH;
    constexpr int BV = SM::BV, NV = VBlock<T, DV, DK>::NV;
    using Map = ScanMap<DK, BV>;
    constexpr int NWT = (Map::W_TILES + 3) / 4; // W tiles per chain wave
    extern __shared__ __align__(16) unsigned char smem[];
    T *stg = reinterpret_cast<T *>(smem + SM::oStage) + ((threadIdx.x >> 6) % SM::NSTG) * Stage<T>::ELEMS;
    T *sQ = reinterpret_cast<T *>(smem + SM::oQ);
    constexpr bool MERGE = SM::kMerge;
    T *sK0 = reinterpret_cast<T *>(smem + SM::oK), *sK1 = MERGE ? reinterpret_cast<T *>(smem + SM::oK2) : sK0;
    T *sV = reinterpret_cast<T *>(smem + SM::oV);
    T *sW = reinterpret_cast<T *>(smem + SM::oW);
    T *sST = reinterpret_cast<T *>(smem + SM::oST);
    T *sUT0 = reinterpret_cast<T *>(smem + SM::oUT), *sUT1 = reinterpret_cast<T *>(smem + SM::oUT + SM::szUT);
    T *sT = reinterpret_cast<T *>(smem + SM::oT);
    T *sP = reinterpret_cast<T *>(smem + SM::oP);
    float *sGam0 = reinterpret_cast<float *>(smem + SM::oGam), *sGam1 = MERGE ? reinterpret_cast<float *>(smem + SM::oGam2) : sGam0;
    constexpr bool gated = GATED; // compile-time, so the plain kernels carry none of the gate's registers
    // the gated kernels, and those with d_k = 256, request operand fragments in smaller batches: they have no registers to spare
    constexpr int MB = (GATED || MODE == SCAN_BOTH) ? 2 : (sizeof(T) == 4 ? 2 : (DK > 128 ? 4 : 0)); // SCAN_BOTH: the loader waves hold more
    // a workgroup's rows of V and O are whole 128-byte lines: non-temporal; with narrower column blocks a line is shared with
    // the neighbouring workgroup of the chain and keeps the default policy
    constexpr bool kWholeLines = BV * sizeof(T) >= 128;

    int chain, vbi;
    if (!chain_of_block(bid, sm.N * H, NV, chain, vbi)) return;
    int n = chain / H;
    const int h = chain - n * H, vb = vbi * BV;
    if (sm.order) { n = sm.order[n]; chain = n * H + h; } // packed: longest sequences first
    const int wave = threadIdx.x >> 6;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int nchunks = (len + C - 1) / C;
    const Map m(wave);
    const bool loader = wave >= 4, does_o = OUT && m.does_o;
    const int lt = threadIdx.x - NTL; // index among the loader threads
    // waves 0..3 build the tiles (pmi, pni) = (0,0), (1,0), (1,1), (0,1) of P; the last one is all zero
    const int pmi = (wave == 1) | (wave == 2), pni = wave >> 1;

    f32x16 S = zero16();
    if (m.has_s && p.S0) {
        const float *src = p.S0 + (long)chain * DK * DV + vb;
        acc_each(S, [&](int r, int c, float &val) { val = src[(long)(32 * m.sa + r) * DV + 32 * m.sb + c]; });
    }
    if (MODE == SCAN_STATE && p.unit_state && m.has_s) // start from the identity: the final state is then the segment's transition matrix
        acc_each(S, [&](int r, int c, float &val) { val = (32 * m.sa + r == vb + 32 * m.sb + c) ? 1.f : 0.f; });
    // settle these loads here: otherwise the compiler keeps "state registers may still be in flight"
    // alive around the loop and drains the memory counter (and with it the prefetch) in every step
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0)

    struct Regs {
        TileRegs<T, C, DK, NTL> q, k;
        TileRegs<T, C, BV, NTL> v;
        TileRegs<T, C, C, NTL> t;
        float vs[TileRegs<T, C, BV, NTL>::NIT], gm; // gated: 1 / gamma of this lane's V rows; one entry of the gamma table
    } r;
    auto fetch_a = [&](int ic) __attribute__((always_inline)) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        const long tile = ((long)(cb + ic) * H + h);
        r.k.template load_aux<kAuxKeep>((const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid, lt);
        // (the transition-matrix pass of k_scan_state runs on v = 0: no row is valid)
        r.v.template load_aux<kWholeLines ? kAuxOnce : kAuxKeep>((const T *)p.v + (row0 * H + h) * DV + vb, (long)H * DV, (MODE == SCAN_STATE && p.unit_state) ? 0 : nvalid, lt);
        r.t.template load_aux<kAuxKeep>((const T *)p.Tm + tile * C * C, C, C, lt);
        if (gated) {
            r.v.load_row_factors(r.vs, p.gam + tile * 2 * C + C, lt);
            if (lt < 2 * C) r.gm = p.gam[tile * 2 * C + lt];
        }
    };
    auto fetch_b = [&](int ic) __attribute__((always_inline)) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        if (OUT) r.q.template load_aux<kAuxKeep>((const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid, lt);
    };
    // Everything that touches global memory is issued by the loader waves in one burst right after
    // the first barrier of a step: the loads for the next chunk, then the stores of what the previous
    // step left in LDS (its Ut^T, or its staged output tile).  The compiler drains the memory counter
    // when the loaded registers are moved to LDS at the top of the next step; by then all of it is a
    // full step old.
    auto flush_ut = [&](int icp, int t) __attribute__((always_inline)) { // Ut^T of chunk icp, still in LDS; t = 0 .. NTL - 1
        const long tile = ((long)(cb + icp) * H + h);
        copy_out<T, BV, C, NTL, true>((T *)p.Ut + (tile * DV + vb) * C, (icp & 1) ? sUT1 : sUT0, SM::LT, t);
    };
    auto flush_out = [&](int icp) __attribute__((always_inline)) { // this wave's staged output tile of chunk icp
        if (m.does_o)
            stage_flush<T, kWholeLines>(stg, (T *)p.o + (((long)t0 + (long)icp * C) * H + h) * DV + vb, (long)H * DV, 32 * m.ua, 32 * m.ub,
                           min(C, len - icp * C));
    };
    auto stash = [&](int par) __attribute__((always_inline)) { // fetched tiles of a chunk of parity `par`: registers -> LDS
        if (OUT) r.q.store(sQ, SM::LQ, lt);
        r.k.store(par ? sK1 : sK0, SM::LK, lt);
        if (gated) { // the chunk runs the plain rule on v_i / gamma_i
            r.v.scale_rows(r.vs);
            if (lt < 2 * C) (par ? sGam1 : sGam0)[lt] = r.gm;
        }
        r.v.store(sV, SM::LV, lt);
        r.t.store(sT, SM::LT, lt);
    };
    if (loader && nchunks > 0) { fetch_a(0); fetch_b(0); stash(0); }
    // gated: gamma at the end of the chunk, which rescales the state when the chunk is done; every wave
    // requests the next chunk's value one step ahead
    float gC = 1.f, gCn = 1.f;
    if (gated && nchunks > 0) {
        gCn = p.gam[((long)cb * H + h) * 2 * C + C - 1];
        S *= gCn; // into the first chunk's coordinates
    }
    for (int ic = 0; ic < nchunks; ++ic) {
        const long tile = ((long)(cb + ic) * H + h);
        T *sUT = (ic & 1) ? sUT1 : sUT0;
        T *sK = (ic & 1) ? sK1 : sK0;
        float *sGam = (ic & 1) ? sGam1 : sGam0;
        gC = gCn; // out of this chunk's coordinates when it ends (gC), and into the next one's (gCn)
        if (gated) gCn = ic + 1 < nchunks ? p.gam[(tile + H) * 2 * C + C - 1] : 1.f;
        if (!MERGE || ic == 0) {
            if (m.has_s) acc_to_lds_t<T>(sST, SM::LS, 32 * m.sa, 32 * m.sb, S);
        }
        lds_barrier();
        if (loader && ic + 1 < nchunks) fetch_a(ic + 1);
        if (MODE == SCAN_BOTH && loader) {
            // the chunk-initial state, kept for the backward pass, leaves in this interval (transposed, as it sits in
            // LDS); the previous chunk's Ut^T follows in the third one: both in one interval make it the longest
            copy_out<T, BV, DK, NTL, true>((T *)p.Sc + (tile * DV + vb) * DK, sST, SM::LS, lt);
        }
        f32x16 acc = zero16();
        if (!loader) {
            // What does not depend on the state, while the loader waves are busy with global memory.
            // Straight-line on purpose (full contraction length even where T's zero block makes half
            // of it idle, a masked all-zero P tile on wave 3): independent products in one basic
            // block are what lets the scheduler overlap one product's LDS and MFMA latency with the next.
            // (with more than two W tiles per wave, d_k = 256, the tiles are finished one at a time instead:
            // there are not enough registers to keep them all in flight)
            constexpr bool SEQ = GATED || NWT > 2;
            f32x16 w[NWT];
#pragma unroll
            for (int i = 0; i < NWT; ++i) { // W = T K (Eq. 11) as W^T = K^T T^T
                const int t = wave + 4 * i, wk = t % Map::NKT, wi = t / Map::NKT;
                w[i] = zero16();
                if (Map::W_TILES % 4 == 0 || t < Map::W_TILES) {
                    mma<C, true, false, T, SEQ, MB>(w[i], sK + 32 * wk, SM::LK, sT + 32 * wi * SM::LT, SM::LT);
                    if (NWT > 2) acc_to_lds_t<T>(sW, SM::LQ, 32 * wk, 32 * wi, w[i]);
                }
            }
            if (m.does_u) mma<C, false, true, T, SEQ, MB>(acc, sT + 32 * m.ua * SM::LT, SM::LT, sV + 32 * m.ub, SM::LV); // U = T V
            f32x16 pa = zero16();
            if (OUT) // P = tril(Q K^T), the causal intra-chunk scores of Eq. 9, as the tile (pni, pmi) of P^T
                mma<DK, false, false, T, SEQ, MB>(pa, sK + 32 * pni * SM::LK, SM::LK, sQ + 32 * pmi * SM::LQ, SM::LQ);
            if (NWT <= 2) {
#pragma unroll
                for (int i = 0; i < NWT; ++i) {
                    const int t = wave + 4 * i, wk = t % Map::NKT, wi = t / Map::NKT;
                    if (Map::W_TILES % 4 == 0 || t < Map::W_TILES) acc_to_lds_t<T>(sW, SM::LQ, 32 * wk, 32 * wi, w[i]);
                }
            }
            if (OUT) {
                acc_each(pa, [&](int r, int c, float &val) { if (32 * pni + r > 32 * pmi + c) val = 0.f; });
                acc_to_lds_t<T>(sP, SM::LT, 32 * pni, 32 * pmi, pa);
            }
        } else if (does_o) {
            // Q S, the inter-chunk part of Eq. 9: it needs only the state, so the output waves form it here,
            // where they would otherwise wait for the chain waves' products
            mma<DK, false, false, T, true, MB>(acc, sQ + 32 * m.ua * SM::LQ, SM::LQ, sST + 32 * m.ub * SM::LS, SM::LS);
        }
        lds_barrier();
        if (loader) {
            if (ic + 1 < nchunks) fetch_b(ic + 1);
            // the chunk-initial state leaves transposed, as it sits in LDS
            if (MODE == SCAN_STORE) copy_out<T, BV, DK, NTL, true>((T *)p.Sc + (tile * DV + vb) * DK, sST, SM::LS, lt);
            if (OUT && ic > 0) flush_out(ic - 1);
        }
        if (m.does_u) { // Ut = U - W S (inner term of Eq. 8-9)
            f32x16 ws = zero16();
            mma<DK, false, false, T, true, MB>(ws, sW + 32 * m.ua * SM::LQ, SM::LQ, sST + 32 * m.ub * SM::LS, SM::LS);
            acc -= ws;
            acc_to_lds_t<T>(sUT, SM::LT, 32 * m.ua, 32 * m.ub, acc);
        }
        lds_barrier();
        // the previous chunk's Ut^T leaves here, sent by the chain waves, which have no output tile to form in this interval
        if (SAVE && !loader && ic > 0 && !p.skip_ut) flush_ut(ic - 1, (int)threadIdx.x);
        if (does_o) { // O = Q S + P Ut (Eq. 9); the tile waits in this wave's staging area until the next step
            if (m.ua == 0) mma<32, false, false, T, true, MB>(acc, sP, SM::LT, sUT + 32 * m.ub * SM::LT, SM::LT);
            else mma<C, false, false, T, true, MB>(acc, sP + 32 * SM::LT, SM::LT, sUT + 32 * m.ub * SM::LT, SM::LT);
            if (gated) acc_each(acc, [&](int rr, int, float &val) { val *= sGam[32 * m.ua + rr]; }); // o_i = gamma_i o~_i
            acc_to_lds<T>(stg, Stage<T>::LD, 0, 0, acc);
        }
        if (m.has_s) mma<C, true, false, T, true, MB>(S, sK + 32 * m.sa, SM::LK, sUT + 32 * m.sb * SM::LT, SM::LT); // S += K^T Ut (Eq. 8)
        if (gated) { // from this chunk's coordinates to the state itself, then to the next chunk's (one factor at a time: their product may leave the fp32 range)
            S *= gC;
            S *= gCn;
        }
        if (MERGE) {
            // nothing read in this interval is written here: the state's LDS copy serves only the first two intervals of a
            // step, Q, V, T only the first, and the next K and gamma table go to the buffers of the other parity
            if (m.has_s && ic + 1 < nchunks) acc_to_lds_t<T>(sST, SM::LS, 32 * m.sa, 32 * m.sb, S);
        } else {
            lds_barrier();
        }
        // The next chunk's tiles move to LDS here, in the iteration that requested them: the wait the
        // compiler puts in front counts the stores issued after the loads and lets those stay in flight.
        if (loader && ic + 1 < nchunks) stash((ic + 1) & 1);
    }
    if (loader && nchunks > 0) {
        if (SAVE && !p.skip_ut) flush_ut(nchunks - 1, lt);
        if (OUT) flush_out(nchunks - 1);
    }
    if ((OUT || MODE == SCAN_STATE) && p.ST && m.has_s) {
        float *dst = p.ST + (long)chain * DK * DV + vb;
        acc_each(S, [&](int r, int c, float &val) { dst[(long)(32 * m.sa + r) * DV + 32 * m.sb + c] = val; });
    }
}
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_fwd(SeqMap sm, int H, Ptrs p) {
    scan_fwd_body<T, DK, DV, SCAN_OUT, VAR>(sm, H, p, blockIdx.x);
}
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_fwd_save(SeqMap sm, int H, Ptrs p) {
    scan_fwd_body<T, DK, DV, SCAN_BOTH, VAR>(sm, H, p, blockIdx.x);
}

template <typename T, int DK, int DV, int VAR, bool STATE>
__device__ __forceinline__ void scan_bwd_body(const SeqMap &sm, int H, const Ptrs &p, int bid);

// A forward pass over few, long chains leaves most CUs idle.  Every stretch of a chain acts on the state as an
// affine map S_out = M S_in + N (M = the product of the chunks' (I - K^T W), d_k x d_k; N = what the stretch writes
// starting from zero; Eq. 8), so the sequence is cut into G segments that are scanned side by side:
//   k_scan_state   per segment, both in one grid: N (the scan from a zero state) and M (the same scan on v = 0
//                  starting from the identity; needs d_v = d_k), final states only
//   k_seg_combine  per chain: S_in of every segment by S <- M_g S + N_g, in fp32 on the matrix cores
//   k_scan_fwd     per segment, from its S_in: the outputs
// `sm` describes the segments as sequences (dense layout: [B, L] viewed as [B G, L / G]); `half` = workgroups per pass.
// The backward pass is cut the same way: the gradient with respect to a segment's start state is
// M^T (gradient with respect to its end state) + R, R = the reverse scan of the segment from a zero gradient; a grid of
// three parts adds that pass (k_scan_state), a grid of one part runs it alone (k_scan_bwd_state).
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_state(SeqMap sm, int H, Ptrs p, int half) {
    Ptrs ps = p;
    ps.S0 = nullptr;
    const int part = (int)blockIdx.x / half, bid = (int)blockIdx.x - part * half;
    if (part == 2) {
        ps.dST = nullptr; ps.dS0 = p.Rseg;
        scan_bwd_body<T, DK, DV, VAR, true>(sm, H, ps, bid);
        return;
    }
    if (part == 0) { ps.unit_state = 0; ps.ST = p.Nseg; }
    else { ps.unit_state = 1; ps.ST = p.Mseg; }
    scan_fwd_body<T, DK, DV, SCAN_STATE, VAR>(sm, H, ps, bid);
}
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_bwd_state(SeqMap sm, int H, Ptrs p) {
    Ptrs ps = p;
    ps.dST = nullptr; ps.dS0 = p.Rseg;
    scan_bwd_body<T, DK, DV, VAR, true>(sm, H, ps, blockIdx.x);
}

// S_in(0) = the caller's initial state (or zero); S_in(g + 1) = M_g S_in(g) + N_g; the state after the last segment is
// the final state.  Backward (blockIdx.z = 1): D(G) = the caller's gradient with respect to the final state (or zero);
// every segment's end gradient dSout(g) = D(g + 1), D(g) = M_g^T D(g + 1) + R_g; D(0) is the gradient with respect to the
// initial state.  One workgroup per (chain, block of 32 state columns, direction): the columns evolve independently.
// fp32 on the matrix cores; the next segment's M and N (R) tile travel from global memory while the current product runs.
template <int DK, int DV> struct CombineSmem {
    static constexpr int LM = DK + 4, LSB = 32 + 4;
    static constexpr size_t oM = 0, oS = sizeof(float) * DK * LM, bytes = oS + sizeof(float) * DK * LSB;
};
struct CombineArgs {
    const float *Mseg, *Nseg, *S0; // forward: per-segment N, the caller's initial state (may be null)
    float *Sin, *ST;               // forward outputs: start state per segment, final state (may be null)
    const float *Rseg, *dST;       // backward: per-segment R, the caller's final-state gradient (may be null)
    float *dSout, *dS0;            // backward outputs: end gradient per segment, initial-state gradient (may be null)
    int G, H, first_dir;           // grid.z directions run from first_dir: 0 = forward, 1 = backward
};
template <int DK, int DV>
__global__ __launch_bounds__(NTHR) void k_seg_combine(CombineArgs a) {
    using SM = CombineSmem<DK, DV>;
    static_assert(DK % 32 == 0 && DK / 32 <= NTHR / 64, "one 32-row tile per wave");
    extern __shared__ __align__(16) unsigned char smem[];
    float *sM = reinterpret_cast<float *>(smem + SM::oM), *sS = reinterpret_cast<float *>(smem + SM::oS);
    const int chain = blockIdx.x, b = chain / a.H, h = chain - b * a.H, c0 = 32 * blockIdx.y;
    const bool bwd = (int)blockIdx.z + a.first_dir == 1;
    const int tid = threadIdx.x, wave = tid >> 6;
    const bool act = wave < DK / 32;
    const float *init = bwd ? a.dST : a.S0, *add = bwd ? a.Rseg : a.Nseg;
    float *start = bwd ? a.dSout : a.Sin, *last = bwd ? a.dS0 : a.ST;
    auto seg_of = [&](int i) __attribute__((always_inline)) { return ((long)(b * a.G + (bwd ? a.G - 1 - i : i)) * a.H + h); };
    TileRegs<float, DK, DK, NTHR> mreg;
    f32x16 nreg = zero16();
    auto request = [&](int i) __attribute__((always_inline)) { // M and the additive tile of step i, into registers
        const long seg = seg_of(i);
        mreg.load(a.Mseg + seg * DK * DK, DK, DK);
        if (act) acc_each(nreg, [&](int r, int c, float &val) { val = add[(seg * DK + 32 * wave + r) * DV + c0 + c]; });
    };
    request(0);
    for (int e = tid; e < DK * 32; e += NTHR) {
        const int i = e >> 5, j = e & 31;
        sS[i * SM::LSB + j] = init ? init[((long)chain * DK + i) * DV + c0 + j] : 0.f;
    }
    lds_barrier(); // (LDS only: the requests and stores in flight are not waited for)
    for (int i = 0; i < a.G; ++i) {
        const long seg = seg_of(i);
        for (int e = tid; e < DK * 32; e += NTHR) { // this segment starts from (backward: ends with) the current value
            const int r = e >> 5, j = e & 31;
            start[(seg * DK + r) * DV + c0 + j] = sS[r * SM::LSB + j];
        }
        mreg.store(sM, SM::LM);
        f32x16 acc = nreg;
        lds_barrier();
        if (i + 1 < a.G) request(i + 1);
        if (act) {
            if (bwd) mma<DK, true, true, float>(acc, sM + 32 * wave, SM::LM, sS, SM::LSB); // M^T D: down the rows of M
            else mma<DK, false, true, float>(acc, sM + 32 * wave * SM::LM, SM::LM, sS, SM::LSB);
        }
        lds_barrier(); // every wave has read the old value
        if (act) acc_to_lds<float>(sS, SM::LSB, 32 * wave, 0, acc);
        lds_barrier();
    }
    if (last)
        for (int e = tid; e < DK * 32; e += NTHR) {
            const int r = e >> 5, j = e & 31;
            last[((long)chain * DK + r) * DV + c0 + j] = sS[r * SM::LSB + j];
        }
}

// scan_bwd_body: reverse over chunks, carrying dS (gradient w.r.t. the chunk-initial state):
//   dUt = P^T dO + K dS';  dS = dS' + Q^T dO - W^T dUt
// Per chunk it leaves dS'^T and dUt^T in the workspace (the transposed LDS copies, written out by the loader waves).
template <typename T, int DK, int DV> struct ScanBwdSmem {
    static constexpr int BV = VBlock<T, DV, DK>::BV;
    static constexpr int LQ = ldn<T>(DK), LK = ldn<T>(DK), LD = ldn<T>(BV), LS = ldc<T>(DK), LT = ldc<T>(C);
    static constexpr size_t oQ = 0;
    static constexpr size_t oK = oQ + align16(sizeof(T) * C * LQ);
    static constexpr size_t oW = oK + align16(sizeof(T) * C * LK);
    static constexpr size_t oDO = oW + align16(sizeof(T) * C * LQ);
    static constexpr size_t oDST = oDO + align16(sizeof(T) * C * LD);
    static constexpr size_t oDUT = oDST + align16(sizeof(T) * BV * LS);
    static constexpr size_t szDUT = align16(sizeof(T) * BV * LT);    // two dUt^T buffers, alternating by chunk parity
    static constexpr size_t oT = oDUT + 2 * szDUT;
    static constexpr size_t oPT = oT + align16(sizeof(T) * C * LT);
    static constexpr size_t bytes = oPT + align16(sizeof(T) * C * LT);
};

// STATE = true: only the gradient with respect to the initial state leaves the kernel (the first pass of a backward
// pass that is split over segments of the sequence).
template <typename T, int DK, int DV, int VAR, bool STATE>
__device__ __forceinline__ void scan_bwd_body(const SeqMap &sm, int H, const Ptrs &p, int bid) {
    using SM = ScanBwdSmem<T, DK, DV>;
    static_assert(VAR != VAR_PROLOGUE, "the scans read q and k already mapped");
    constexpr bool GATED = VAR == VAR_GATED;
    constexpr int BV = SM::BV, NV = VBlock<T, DV, DK>::NV;
    using Map = ScanMap<DK, BV>;
    constexpr int NWT = (Map::W_TILES + 3) / 4; // W tiles per chain wave
    extern __shared__ __align__(16) unsigned char smem[];
    T *sQ = reinterpret_cast<T *>(smem + SM::oQ);
    T *sK = reinterpret_cast<T *>(smem + SM::oK);
    T *sW = reinterpret_cast<T *>(smem + SM::oW);
    T *sDO = reinterpret_cast<T *>(smem + SM::oDO);
    T *sDST = reinterpret_cast<T *>(smem + SM::oDST);
    T *sDUT0 = reinterpret_cast<T *>(smem + SM::oDUT), *sDUT1 = reinterpret_cast<T *>(smem + SM::oDUT + SM::szDUT);
    T *sT = reinterpret_cast<T *>(smem + SM::oT);
    T *sPT = reinterpret_cast<T *>(smem + SM::oPT);
    constexpr bool gated = GATED; // compile-time, so the plain kernels carry none of the gate's registers
    // the gated kernels, and those with d_k = 256, request operand fragments in smaller batches: they have no registers to spare
    constexpr int MB = GATED ? 2 : (sizeof(T) == 4 ? 2 : (DK > 128 ? 4 : 0));

    int chain, vbi;
    if (!chain_of_block(bid, sm.N * H, NV, chain, vbi)) return;
    int n = chain / H;
    const int h = chain - n * H, vb = vbi * BV;
    if (sm.order) { n = sm.order[n]; chain = n * H + h; } // packed: longest sequences first
    const int wave = threadIdx.x >> 6;
    int t0, len, cb;
    sm.seq(n, t0, len, cb);
    const int nchunks = (len + C - 1) / C;
    const Map m(wave);
    const bool loader = wave >= 4;
    const int lt = threadIdx.x - NTL;
    // waves 0..3 build the tiles (pmi, pni) = (0,0), (0,1), (1,1), (1,0) of P^T; the last one is all zero
    const int pmi = wave >> 1, pni = (wave == 1) | (wave == 2);

    f32x16 dS = zero16();
    if (m.has_s && p.dST) {
        const float *src = p.dST + (long)chain * DK * DV + vb;
        acc_each(dS, [&](int r, int c, float &val) { val = src[(long)(32 * m.sa + r) * DV + 32 * m.sb + c]; });
    }
    __builtin_amdgcn_s_waitcnt(0x0F70); // vmcnt(0): see k_scan_fwd

    struct Regs {
        TileRegs<T, C, DK, NTL> q, k;
        TileRegs<T, C, BV, NTL> d_o;
        TileRegs<T, C, C, NTL> t;
        float dos[TileRegs<T, C, BV, NTL>::NIT]; // gated: gamma of this lane's dO rows
    } r;
    auto fetch_a = [&](int ic) __attribute__((always_inline)) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        r.q.template load_aux<kAuxKeep>((const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid, lt);
        r.k.template load_aux<kAuxKeep>((const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid, lt);
    };
    auto fetch_b = [&](int ic) __attribute__((always_inline)) {
        const int nvalid = min(C, len - ic * C);
        const long row0 = (long)t0 + (long)ic * C;
        const long tile = ((long)(cb + ic) * H + h);
        r.d_o.template load_aux<kAuxKeep>((const T *)p.d_o + (row0 * H + h) * DV + vb, (long)H * DV, nvalid, lt);
        r.t.template load_aux<kAuxKeep>((const T *)p.Tm + tile * C * C, C, C, lt);
        if (gated) r.d_o.load_row_factors(r.dos, p.gam + tile * 2 * C, lt);
    };
    auto flush_dut = [&](int icp, int t) __attribute__((always_inline)) { // dUt^T of chunk icp, still in LDS; t = 0 .. NTL - 1
        copy_out<T, BV, C, NTL, true>((T *)p.dUt + (((long)(cb + icp) * H + h) * DV + vb) * C, (icp & 1) ? sDUT1 : sDUT0, SM::LT, t);
    };
    // As in the forward scan, the loader waves issue all global traffic of a step in one burst after
    // its first barrier: next chunk's loads, this chunk's dS'^T, the previous step's dUt^T.
    auto stash = [&]() __attribute__((always_inline)) { // fetched tiles: registers -> LDS
        r.q.store(sQ, SM::LQ, lt); r.k.store(sK, SM::LK, lt);
        if (gated) r.d_o.scale_rows(r.dos); // o_i = gamma_i o~_i, so the plain rule's output gradient is gamma_i dO_i
        r.d_o.store(sDO, SM::LD, lt);
        r.t.store(sT, SM::LT, lt);
    };
    if (loader && nchunks > 0) { fetch_a(nchunks - 1); fetch_b(nchunks - 1); stash(); }
    // gated: the state after the chunk is gamma_C times the plain rule's, so its gradient is scaled by
    // gamma_C on entry; every wave requests the value for the next step one step ahead
    float gCn = 1.f, gHere = 1.f; // gHere: gamma_C of the chunk of the current step
    if (gated && nchunks > 0) gCn = gHere = p.gam[((long)(cb + nchunks - 1) * H + h) * 2 * C + C - 1];
    // dS' of the last chunk (the gradient with respect to the state after it) goes to LDS here; every later one at the end
    // of the step that produced it: that interval reads only W and dUt^T, so the state gradient's LDS copy and the next
    // chunk's tiles can be written in it, and a chunk step takes three barrier intervals.
    if (gated) dS *= gCn;
    if (m.has_s && nchunks > 0) acc_to_lds_t<T>(sDST, SM::LS, 32 * m.sa, 32 * m.sb, dS);
    for (int ic = nchunks - 1; ic >= 0; --ic) {
        const long tile = ((long)(cb + ic) * H + h);
        T *sDUT = (ic & 1) ? sDUT1 : sDUT0;
        if (gated && ic > 0) gCn = p.gam[(tile - H) * 2 * C + C - 1]; // for the end of this step
        lds_barrier();
        if (loader && ic > 0) fetch_a(ic - 1);
        // dS'^T to the workspace, in the interval whose length the chain waves' products set
        if (loader && !STATE) copy_out<T, BV, DK, NTL, true>((T *)p.dSc + (tile * DV + vb) * DK, sDST, SM::LS, lt);
        f32x16 acc = zero16();
        if (!loader) { // straight-line, as in the forward scan; the loader waves are busy with global memory meanwhile
            // (with more than two W tiles per wave, d_k = 256, the tiles are finished one at a time, as in the forward scan)
            constexpr bool SEQ = GATED || NWT > 2;
            f32x16 pa = zero16(); // P^T = triu(K Q^T), the transposed causal scores, computed as the tile (pni, pmi) of P
            mma<DK, false, false, T, SEQ, MB>(pa, sQ + 32 * pni * SM::LQ, SM::LQ, sK + 32 * pmi * SM::LK, SM::LK);
            if (m.does_u) // K dS' part of the dUt tile (ua, ub)
                mma<DK, false, false, T, SEQ, MB>(acc, sK + 32 * m.ua * SM::LK, SM::LK, sDST + 32 * m.ub * SM::LS, SM::LS);
            f32x16 w[NWT];
#pragma unroll
            for (int i = 0; i < NWT; ++i) { // W = T K (Eq. 11), computed as W^T = K^T T^T
                const int t = wave + 4 * i, wk = t % Map::NKT, wi = t / Map::NKT;
                w[i] = zero16();
                if (Map::W_TILES % 4 == 0 || t < Map::W_TILES) {
                    mma<C, true, false, T, SEQ, MB>(w[i], sK + 32 * wk, SM::LK, sT + 32 * wi * SM::LT, SM::LT);
                    if (NWT > 2) acc_to_lds_t<T>(sW, SM::LQ, 32 * wk, 32 * wi, w[i]);
                }
            }
            acc_each(pa, [&](int r, int c, float &val) { if (32 * pni + r < 32 * pmi + c) val = 0.f; });
            acc_to_lds_t<T>(sPT, SM::LT, 32 * pni, 32 * pmi, pa);
            if (NWT <= 2) {
#pragma unroll
                for (int i = 0; i < NWT; ++i) {
                    const int t = wave + 4 * i, wk = t % Map::NKT, wi = t / Map::NKT;
                    if (Map::W_TILES % 4 == 0 || t < Map::W_TILES) acc_to_lds_t<T>(sW, SM::LQ, 32 * wk, 32 * wi, w[i]);
                }
            }
        }
        lds_barrier();
        if (loader) {
            if (ic > 0) fetch_b(ic - 1);
        }
        if (m.does_u) { // + P^T dO; P^T is upper triangular
            if (m.ua == 0) mma<C, false, true, T, true, MB>(acc, sPT, SM::LT, sDO + 32 * m.ub, SM::LD);
            else mma<32, false, true, T, true, MB>(acc, sPT + 32 * SM::LT + 32, SM::LT, sDO + 32 * SM::LD + 32 * m.ub, SM::LD);
            acc_to_lds_t<T>(sDUT, SM::LT, 32 * m.ua, 32 * m.ub, acc);
        }
        if (m.has_s) mma<C, true, true, T, true, MB>(dS, sQ + 32 * m.sa, SM::LQ, sDO + 32 * m.sb, SM::LD); // + Q^T dO
        lds_barrier();
        // (sent by the chain waves, as in the forward scan: the loader waves have the next chunk's tiles to move in this interval)
        if (!STATE && !loader && ic + 1 < nchunks && !p.skip_ut) flush_dut(ic + 1, (int)threadIdx.x);
        if (m.has_s) { // - W^T dUt
            f32x16 wd = zero16();
            mma<C, true, false, T, true, MB>(wd, sW + 32 * m.sa, SM::LQ, sDUT + 32 * m.sb * SM::LT, SM::LT);
            dS -= wd;
        }
        if (ic > 0) {
            if (gated) { // across the boundary: out of this chunk's coordinates, into those of the chunk before
                dS *= gHere; // (one factor at a time: their product may leave the fp32 range)
                dS *= gCn;
                gHere = gCn;
            }
            if (m.has_s) acc_to_lds_t<T>(sDST, SM::LS, 32 * m.sa, 32 * m.sb, dS); // dS' of the next step
            if (loader) stash(); // see k_scan_fwd
        }
    }
    if (!STATE && loader && nchunks > 0 && !p.skip_ut) flush_dut(0, lt);
    if (p.dS0 && m.has_s) {
        float *dst = p.dS0 + (long)chain * DK * DV + vb;
        if (gated) dS *= gHere; // out of the first chunk's coordinates
        acc_each(dS, [&](int r, int c, float &val) { dst[(long)(32 * m.sa + r) * DV + 32 * m.sb + c] = val; });
    }
}

// The backward pass's two scans in one launch.  They do not depend on each other (the recompute
// scan needs T; the reverse scan needs T and P^T), so the first half of the grid runs the reverse
// scan and the second half the recompute scan: a CU picks up one of each with no kernel boundary
// in between.  `half` = workgroups per scan.
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_pair(SeqMap sm, int H, Ptrs p, int half) {
    if ((int)blockIdx.x < half) scan_bwd_body<T, DK, DV, VAR, false>(sm, H, p, blockIdx.x);
    else scan_fwd_body<T, DK, DV, SCAN_STORE, VAR>(sm, H, p, blockIdx.x - half);
}
// the reverse scan alone, for a backward pass that finds the forward scan's tiles already in the workspace
template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTS) void k_scan_bwd(SeqMap sm, int H, Ptrs p) {
    scan_bwd_body<T, DK, DV, VAR, false>(sm, H, p, blockIdx.x);
}

// =============================================================================================
// The chunk-parallel backward kernel.  Workgroups are persistent: each walks over (chunk, head)
// tiles with a grid stride; a tile's operands (168 KB in bf16 at d = 128) fill the whole LDS, so
// overlap of loads and MFMA work comes from the CUs running out of step with each other.
constexpr int NTC = 512, NWC = 8;

struct TileIter { // grid-stride walk over (global chunk id, head) tiles
    int id, total, H;
    __device__ TileIter(int chunks_total, int H_) : id(blockIdx.x), total(chunks_total * H_), H(H_) {}
    __device__ bool valid() const { return id < total; }
    __device__ void next() { id += gridDim.x; }
    __device__ int gid() const { return id / H; }
    __device__ int head() const { return id % H; }
};
struct TilePos { int nvalid, h; long row0, tile; bool ok; };
__device__ inline TilePos tile_pos(const SeqMap &sm, int H, int gid, int h) {
    TilePos tp;
    int n, ic, t0, len, cb;
    tp.ok = sm.chunk(gid, n, ic);
    tp.h = h; tp.nvalid = 0; tp.row0 = 0; tp.tile = 0;
    if (tp.ok) {
        sm.seq(n, t0, len, cb);
        tp.nvalid = min(C, len - ic * C);
        tp.row0 = (long)t0 + (long)ic * C;
        tp.tile = (long)(cb + ic) * H + h;
    }
    return tp;
}

// k_bwd_chunk: everything of the backward pass that is local to one chunk, given the chunk-initial
// state S, the gradient dS' w.r.t. the state after the chunk, Ut and dUt from the two scans (all four
// arrive transposed, [d_v][d_k] and [d_v][C], as the scans hold them in LDS):
//   adjoint of Eq. 8-9:  dP = tril(dO Ut^T); dQ = dO S^T + dP K; dK1 = dP^T Q + Ut dS'^T; dW = -dUt S^T
//   adjoint of Eq. 10-11, with X = (I+A)^-1 (read back from k_wy_prep), A = tril(diag(beta) G,-1), G = K K^T, dU = dUt:
//     dX' = dW K^T + dU V^T;  dX = dX' diag(beta);  dKb = X^T dW;  dV = diag(beta) X^T dU;
//     dA = -tril(X^T dX X^T, -1);  Ah = diag(beta) dA;
//     dK = dK1 + diag(beta) dKb + Ah K + Ah^T K;
//     dbeta_i = sum_m X[m][i] dX'[m][i] + sum_j dA[i][j] G[i][j].
// dW and dK1 never leave the chip.  LDS buffers are reused as operands die; V and dS' wait in
// registers until their buffer is free.
template <typename T, int DK, int DV> struct ChunkSmem {
    static constexpr int LK = ldn<T>(DK), LV = ldn<T>(DV), LT = ldn<T>(C), LF = C + 4;
    static constexpr int LQO = ldc<T>(DK); // rows of the dq / dk matrix of the prologue variant
    static constexpr int LU = ldc<T>(C), LSK = ldn<T>(DK); // rows of Ut^T / dUt^T ([d_v][C]) and of S^T / dS'^T ([d_v][d_k])
    static constexpr size_t szX = sizeof(float) * C * LF, szCC = sizeof(T) * C * LT;
    static constexpr size_t oB1 = 0;                                   // dO; V; dA o G (fp32)
    static constexpr size_t oB2 = oB1 + align16(cmax(sizeof(T) * C * LV, szX));     // Ut^T; dW
    static constexpr size_t oB3 = oB2 + align16(cmax(sizeof(T) * DV * LU, sizeof(T) * C * LK)); // dUt^T
    static constexpr size_t oB4 = oB3 + align16(sizeof(T) * DV * LU);  // K
    static constexpr size_t oB5 = oB4 + align16(sizeof(T) * C * LK);   // Q; M1^T
    static constexpr size_t oB6 = oB5 + align16(cmax(sizeof(T) * C * LK, szCC)); // dP; dX; Ah
    static constexpr size_t oB7 = oB6 + align16(szCC);                 // S^T; dS'^T; X
    static constexpr size_t szB7 = cmax(sizeof(T) * DV * LSK, szCC);
    static constexpr size_t oBeta = oB7 + align16(szB7);
    static constexpr size_t oGam = oBeta + sizeof(float) * C;          // gated: gamma_i, then 1 / gamma_i
    static constexpr size_t oDb = oGam + sizeof(float) * 2 * C;
    static constexpr size_t oZ = oDb + sizeof(float) * 4 * C;          // gated: per-wave shares of <dS_C, S_C>
    static constexpr size_t oCq = oZ + sizeof(float) * NWC;            // gated: q_i . dq_i per column block of d_k
    static constexpr size_t oCv = oCq + sizeof(float) * (DK / 32) * C; // gated: v_i . dv_i per column block of d_v
    static constexpr size_t oStage = align16(oCv + sizeof(float) * (DV / 32) * C);
    static constexpr size_t bytes = oStage + NWC * sizeof(T) * Stage<T>::ELEMS;
};

template <typename T, int DK, int DV, int VAR>
__global__ __launch_bounds__(NTC) void k_bwd_chunk(SeqMap sm, int H, Ptrs p, int chunks_total) {
    using SM = ChunkSmem<T, DK, DV>;
    constexpr bool GATED = VAR == VAR_GATED, PRO = VAR == VAR_PROLOGUE;
    constexpr int KT = 2 * (DK / 32), VT = 2 * (DV / 32);        // 32 x 32 tiles of a C x DK / C x DV matrix
    constexpr int KW = (KT + NWC - 1) / NWC, VW = (VT + NWC - 1) / NWC; // ... per wave
    extern __shared__ __align__(16) unsigned char smem[];
    T *sDO = reinterpret_cast<T *>(smem + SM::oB1), *sV = sDO;
    float *sProd = reinterpret_cast<float *>(smem + SM::oB1);
    T *sUt = reinterpret_cast<T *>(smem + SM::oB2), *sDW = sUt;
    T *sDU = reinterpret_cast<T *>(smem + SM::oB3);
    T *sK = reinterpret_cast<T *>(smem + SM::oB4);
    T *sQ = reinterpret_cast<T *>(smem + SM::oB5), *sM1T = sQ;
    T *sDP = reinterpret_cast<T *>(smem + SM::oB6), *sDX = sDP;
    T *sS = reinterpret_cast<T *>(smem + SM::oB7);
    T *sXn = reinterpret_cast<T *>(smem + SM::oB7); // X = (I + A)^-1 as computed by k_wy_prep
    float *sBeta = reinterpret_cast<float *>(smem + SM::oBeta);
    float *sGam = reinterpret_cast<float *>(smem + SM::oGam), *sGi = sGam + C;
    float *sDb = reinterpret_cast<float *>(smem + SM::oDb);
    float *sZ = reinterpret_cast<float *>(smem + SM::oZ);
    float *sCq = reinterpret_cast<float *>(smem + SM::oCq), *sCv = reinterpret_cast<float *>(smem + SM::oCv);
    // prologue variant: dq (dk) as a C x d_k matrix, in bytes that are free when it is complete, for the way back through the map
    T *sDQ = reinterpret_cast<T *>(smem + SM::oB1), *sDK = reinterpret_cast<T *>(smem + SM::oB2);
    static_assert(!PRO || (sizeof(T) * C * SM::LQO <= SM::oB2 - SM::oB1 && sizeof(T) * C * SM::LQO <= SM::oB3 - SM::oB2), "dq / dk staging");
    constexpr bool gated = GATED; // compile-time, so the plain kernels carry none of the gate's registers
    // operand fragments are requested two contraction steps at a time (measured best among 2, 4 and 8 in every variant: the
    // LDS is the busy unit here, and long batches only hold registers)
    constexpr int MB = 2;
    // The thread index as the helpers see it: re-read through an empty asm at the top of every barrier interval, so that the
    // per-lane offsets and masks derived from it are formed where they are used.  Left to itself the compiler forms all of
    // them ahead of the tile loop and carries them through it, which costs more registers than the kernel has to spare.
    int tq = threadIdx.x;
    auto fresh = [&]() __attribute__((always_inline)) { tq = threadIdx.x; asm volatile("" : "+v"(tq)); };
    const int tid = threadIdx.x;
    // The wave number, and with it every tile offset derived from it, is recomputed per tile in the variants
    // that are short of registers: hoisted out of the tile loop, those offsets alone would take some 90 VGPRs.
    int wave = tid >> 6;
    // tile number sI of this wave in a C x DK (C x DV) matrix: row block ka, column block kb
    // (head sizes with at most four such tiles give them to waves 4..7: the first four waves own the C x C tiles, and the
    // two kinds of products then run side by side instead of one after the other on the same waves)
    constexpr int TSHIFT = KT <= 4 ? 4 : 0;
    auto kt = [&](int sI) __attribute__((always_inline)) { return TSHIFT ? ((wave + TSHIFT) & (NWC - 1)) + sI * NWC : wave + sI * NWC; };
    auto ka = [&](int sI) __attribute__((always_inline)) { return kt(sI) / (DK / 32); };
    auto kb = [&](int sI) __attribute__((always_inline)) { return kt(sI) % (DK / 32); };
    auto va = [&](int sI) __attribute__((always_inline)) { return kt(sI) / (DV / 32); };
    auto vbk = [&](int sI) __attribute__((always_inline)) { return kt(sI) % (DV / 32); };

    struct Regs {
        TileRegs<T, C, DV, NTC> d_o, v;
        TileRegs<T, DV, C, NTC> ut, dut;
        TileRegs<T, DV, DK, NTC> s, ds;
        TileRegs<T, C, DK, NTC> k, q;
        TileRegs<T, C, DK, NTC> raw; // prologue variant: the pre-activations of q, then of k, for the way back through the map
        TileRegs<T, C, C, NTC> x;
        T beta; // kept in storage format: converting here would wait for the whole prefetch
        // gated: gamma of this lane's dO rows, 1 / gamma of its V rows; entry tid of the chunk's table of gamma_i, 1 / gamma_i
        float dos[TileRegs<T, C, DV, NTC>::NIT], vsc[TileRegs<T, C, DV, NTC>::NIT], gm;
    } r;
    // Every tile of a chunk waits in registers from the moment it is requested.  As soon as one has moved to LDS, the same
    // registers request that tile of the workgroup's next chunk (where there is none the request is issued with every
    // row masked: no branch around a request, so the compiler knows how many are in flight and waits for exactly the
    // one it needs), so about one chunk's worth of loads is in flight at any time.
    // (`live` = 0 masks every row of a request: the instruction is issued, no memory is touched)
    auto fetch_early = [&](const TilePos &tp, int live = 1) __attribute__((always_inline)) {
        r.d_o.load_once((const T *)p.d_o + (tp.row0 * H + tp.h) * DV, (long)H * DV, tp.nvalid * live, tq);
        r.ut.load_once((const T *)p.Ut + tp.tile * DV * C, C, DV * live, tq);
        r.s.load_once((const T *)p.Sc + tp.tile * DV * DK, DK, DV * live, tq);
        r.dut.load_once((const T *)p.dUt + tp.tile * DV * C, C, DV * live, tq);
        if (gated) r.d_o.load_row_factors(r.dos, p.gam + tp.tile * 2 * C);
    };
    auto fetch_kq = [&](const TilePos &tp, int live = 1) __attribute__((always_inline)) {
        // (prologue variant: the q and k that k_wy_prep mapped and left in the workspace, in the layout of q and k)
        r.k.load_once((const T *)(PRO ? p.Km : p.k) + (tp.row0 * H + tp.h) * DK, (long)H * DK, tp.nvalid * live, tq);
        r.q.load_once((const T *)(PRO ? p.Qm : p.q) + (tp.row0 * H + tp.h) * DK, (long)H * DK, tp.nvalid * live, tq);
        if (tq < C) r.beta = ((const T *)p.beta)[(tp.row0 + min(tq, tp.nvalid - 1)) * H + tp.h];
        if (gated && tid < 2 * C) r.gm = p.gam[tp.tile * 2 * C + tid];
    };
    auto fetch_ds = [&](const TilePos &tp, int live = 1) __attribute__((always_inline)) { r.ds.load_once((const T *)p.dSc + tp.tile * DV * DK, DK, DV * live, tq); };
    auto fetch_v = [&](const TilePos &tp, int live = 1) __attribute__((always_inline)) {
        r.v.load_once((const T *)p.v + (tp.row0 * H + tp.h) * DV, (long)H * DV, tp.nvalid * live, tq);
        if (gated) r.v.load_row_factors(r.vsc, p.gam + tp.tile * 2 * C + C);
    };
    auto fetch_x = [&](const TilePos &tp, int live = 1) __attribute__((always_inline)) { r.x.load_once((const T *)p.Xm + tp.tile * C * C, C, C * live, tq); };
    auto fetch_all = [&](const TilePos &tp) __attribute__((always_inline)) { fetch_early(tp); fetch_kq(tp); fetch_ds(tp); fetch_v(tp); fetch_x(tp); };
    auto pos_of = [&](const TileIter &it) __attribute__((always_inline)) { return it.valid() ? tile_pos(sm, H, it.gid(), it.head()) : TilePos{0, 0, 0, 0, false}; };

    // Workgroups that start together stay in lockstep: every CU issues its tile's load burst at the same
    // moment and then all of them compute while HBM idles.  When each workgroup has several tiles to
    // walk, delay it by (blockIdx mod 4) steps of s_sleep(32), about 2K cycles each (measured best among
    // none, 2K, 4K and 8K, and against eight steps), so the bursts of neighbouring CUs interleave with each
    // other's MFMA phases.
    if ((long)chunks_total * H >= 4l * gridDim.x)
        for (int i = 0; i < (int)(blockIdx.x & 3); ++i) __builtin_amdgcn_s_sleep(32);
    TileIter it(chunks_total, H);
    TilePos cur = pos_of(it);
    if (cur.ok) fetch_all(cur);
    while (cur.ok) { // packed layout: the first chunk past the last real one ends the walk (so would every later one)
        TileIter nx = it;
        nx.next();
        const TilePos np = pos_of(nx);
        const TilePos nf = np.ok ? np : cur; // what the freed registers request (masked where there is no next chunk)
        const int nl = np.ok ? 1 : 0;
        asm volatile("" : "+v"(wave)); // opaque: see above
        const int mi = (wave >> 1) & 1, ni = wave & 1; // tile of every C x C matrix, for the first four waves
        const bool cc = wave < 4, upper = (mi == 0 && ni == 1);
        T *stg = reinterpret_cast<T *>(smem + SM::oStage) + wave * Stage<T>::ELEMS;
        const int nvalid = cur.nvalid, h = cur.h;
        const long row0 = cur.row0;
        // ---- adjoint of Eq. 8-9
        // gated: the chunk is the plain rule on v_i / gamma_i with outputs gamma_i o~_i, so dO rows come in
        // scaled by gamma_i, V rows by 1 / gamma_i, and dV goes out scaled by 1 / gamma_i.
        // zp: this thread's share of <dS_C, S_C> = <dS~', S_0> + <K, Ut dS~'^T>, for the gate gradient
        float zp = 0.f;
        if (gated) r.d_o.scale_rows(r.dos);
        r.d_o.store(sDO, SM::LV, tq); r.ut.store(sUt, SM::LU, tq); r.s.store(sS, SM::LSK, tq);
        r.dut.store(sDU, SM::LU, tq);
        fetch_early(nf, nl);
        // prologue variant: q and k come mapped (section 3.3) from the workspace, as k_wy_prep left them; the pre-activations
        // are fetched on the side, q's now and k's once q's gradient has left, for the way back through the map
        r.k.store(sK, SM::LK, tq); r.q.store(sQ, SM::LK, tq);
        if (PRO) r.raw.load_once((const T *)p.q + (row0 * H + h) * DK, (long)H * DK, nvalid, tq); // the pre-activations of q
        if (tq < C) {
            float b = tq < nvalid ? to_f32(r.beta) : 0.f;
            if (PRO) b = tq < nvalid ? sigmoid_f32(b) : 0.f; // beta = sigmoid(logit), section 2.2
            sBeta[tq] = b;
        }
        if (gated && tid < 2 * C) sGam[tid] = r.gm;
        fetch_kq(nf, nl);
        lds_barrier(); fresh();
        if (cc) { // dP = tril(dO Ut^T)
            f32x16 acc = zero16();
            if (!upper) mma<DV, false, true, T, true, MB>(acc, sDO + 32 * mi * SM::LV, SM::LV, sUt + 32 * ni, SM::LU, tq);
            acc_each(acc, [&](int rr, int c, float &val) { if (32 * ni + c > 32 * mi + rr) val = 0.f; }, tq);
            acc_to_lds<T>(sDP, SM::LT, 32 * mi, 32 * ni, acc, tq);
        }
        f32x16 dq[KW], dw[KW], dk1[KW];
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) {
            dq[sI] = zero16(); dw[sI] = zero16(); dk1[sI] = zero16();
            if (kt(sI) < KT) {
                // dO S^T and dUt S^T: the fragments of S are read once for both
                mma_shared_b<DV, false, true, true, T, 2>(dq[sI], dw[sI], sDO + 32 * ka(sI) * SM::LV, SM::LV, sDU + 32 * ka(sI), SM::LU,
                                                          sS + 32 * kb(sI), SM::LSK, tq);
            }
        }
        lds_barrier(); fresh(); // dP visible; S is dead
        if (gated) zp = r.ds.dot_lds(sS, SM::LSK); // <dS~', S_0>: each thread meets the S values it parked there itself
        r.ds.store(sS, SM::LSK, tq);
        fetch_ds(nf, nl);
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) if (kt(sI) < KT) { // dQ += dP K
            if (ka(sI) == 0) mma<32, false, true, T, true, MB>(dq[sI], sDP, SM::LT, sK + 32 * kb(sI), SM::LK, tq);
            else mma<C, false, true, T, true, MB>(dq[sI], sDP + 32 * SM::LT, SM::LT, sK + 32 * kb(sI), SM::LK, tq);
            if (gated) { // also q_i . dq_i over this tile's columns, for the gate gradient
                acc_to_lds<T>(stg, Stage<T>::LD, 0, 0, dq[sI], tq);
                stage_flush_dot<T>(stg, (T *)p.dq + (row0 * H + h) * DK, (long)H * DK, 32 * ka(sI), 32 * kb(sI), nvalid, sQ, SM::LK,
                                   sCq + kb(sI) * C);
            } else if (PRO) { // dO's bytes are free: dq is assembled there for the way back through the map
                acc_to_lds<T>(sDQ, SM::LQO, 32 * ka(sI), 32 * kb(sI), dq[sI], tq);
            } else {
                acc_store<T, true>(stg, (T *)p.dq + (row0 * H + h) * DK, (long)H * DK, 32 * ka(sI), 32 * kb(sI), nvalid, dq[sI], tq);
            }
        }
        lds_barrier(); fresh();
        if (PRO) { // gradient through the feature map: dq~ = SiLU'(q~) (dq - q (q . dq)) / ||SiLU(q~)||
            r.raw.feature_map_bwd_store(sDQ, SM::LQO, (T *)p.dq + (row0 * H + h) * DK, (long)H * DK, nvalid, tq);
            r.raw.load_once((const T *)p.k + (row0 * H + h) * DK, (long)H * DK, nvalid, tq); // ... and those of k, for the end of the chunk
        }
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) if (kt(sI) < KT) { // dK1 = dP^T Q + Ut dS'^T
            if (gated) { // <K, Ut dS~'^T>, the second half of <dS_C, S_C>, taken while dK1 holds just that product
                mma<DV, true, true, T, true, MB>(dk1[sI], sUt + 32 * ka(sI), SM::LU, sS + 32 * kb(sI), SM::LSK, tq);
                acc_each(dk1[sI], [&](int rr, int c, float &val) { zp += val * to_f32(sK[(32 * ka(sI) + rr) * SM::LK + 32 * kb(sI) + c]); }, tq);
            }
            if (ka(sI) == 1) mma<32, true, true, T, true, MB>(dk1[sI], sDP + 32 * SM::LT + 32, SM::LT, sQ + 32 * SM::LK + 32 * kb(sI), SM::LK, tq);
            else mma<C, true, true, T, true, MB>(dk1[sI], sDP, SM::LT, sQ + 32 * kb(sI), SM::LK, tq);
            if (!gated) mma<DV, true, true, T, true, MB>(dk1[sI], sUt + 32 * ka(sI), SM::LU, sS + 32 * kb(sI), SM::LSK, tq);
        }
        lds_barrier(); fresh(); // dO, Ut, Q, dP, dS' are dead
        // ---- adjoint of Eq. 10-11
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) if (kt(sI) < KT) { // dW = -dUt S^T, as an operand
            acc_each(dw[sI], [&](int, int, float &val) { val = -val; }, tq);
            acc_to_lds<T>(sDW, SM::LK, 32 * ka(sI), 32 * kb(sI), dw[sI], tq);
        }
        if (gated) r.v.scale_rows(r.vsc);
        r.v.store(sV, SM::LV, tq);
        fetch_v(nf, nl);
        r.x.store(sXn, SM::LT, tq); // over dS', which dK1 was the last to read
        fetch_x(nf, nl);
        lds_barrier(); fresh();
        f32x16 g = zero16(), dxp = zero16();
        if (cc && !upper) {
            mma<DK, false, false, T, true, MB>(g, sK + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK, tq);
            mma<DK, false, false, T, true, MB>(dxp, sDW + 32 * mi * SM::LK, SM::LK, sK + 32 * ni * SM::LK, SM::LK, tq);
            mma<DV, true, false, T, true, MB>(dxp, sDU + 32 * mi, SM::LU, sV + 32 * ni * SM::LV, SM::LV, tq);
        }
        acc_each(g, [&](int rr, int c, float &val) { if (32 * ni + c >= 32 * mi + rr) val = 0.f; }, tq); // strictly lower G
        // (dX goes to dP's bytes, dead since dK1: no barrier between the product and its scaled copy)
        if (cc) { // dbeta part 1 (column sums of X o dX'), dX = dX' diag(beta)
            float part = 0.f;
            acc_each(dxp, [&](int rr, int c, float &val) {
                const int i = 32 * mi + rr, j = 32 * ni + c;
                part += to_f32(sXn[i * SM::LT + j]) * val;
                val *= sBeta[j];
            }, tq);
            sDb[(2 * mi + ((tq & 63) >> 5)) * C + 32 * ni + (tq & 31)] = part; // summed in a fixed order at the end
            acc_to_lds<T>(sDX, SM::LT, 32 * mi, 32 * ni, dxp, tq);
        }
        lds_barrier(); fresh();
        f32x16 m1 = zero16(); // M1 = dX X^T
        if (cc) mma<C, false, false, T, true, MB>(m1, sDX + 32 * mi * SM::LT, SM::LT, sXn + 32 * ni * SM::LT, SM::LT, tq);
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) if (kt(sI) < KT) { // dKb = X^T dW (X^T is upper triangular)
            f32x16 dKb = zero16();
            if (ka(sI) == 1) mma<32, true, true, T, true, MB>(dKb, sXn + 32 * SM::LT + 32, SM::LT, sDW + 32 * SM::LK + 32 * kb(sI), SM::LK, tq);
            else mma<C, true, true, T, true, MB>(dKb, sXn, SM::LT, sDW + 32 * kb(sI), SM::LK, tq);
            acc_each(dKb, [&](int rr, int, float &val) { val *= sBeta[32 * ka(sI) + rr]; }, tq);
            dk1[sI] += dKb; // dK1 + diag(beta) dKb
        }
#pragma unroll
        for (int sI = 0; sI < VW; ++sI) if (kt(sI) < VT) { // dV = diag(beta) X^T dU
            f32x16 acc = zero16();
            if (va(sI) == 1) mma<32, true, false, T, true, MB>(acc, sXn + 32 * SM::LT + 32, SM::LT, sDU + 32 * vbk(sI) * SM::LU + 32, SM::LU, tq);
            else mma<C, true, false, T, true, MB>(acc, sXn, SM::LT, sDU + 32 * vbk(sI) * SM::LU, SM::LU, tq);
            acc_each(acc, [&](int rr, int, float &val) {
                val *= gated ? sBeta[32 * va(sI) + rr] * sGi[32 * va(sI) + rr] : sBeta[32 * va(sI) + rr];
            }, tq);
            if (gated) { // also (v_i / gamma_i) . dv_i over this tile's columns
                acc_to_lds<T>(stg, Stage<T>::LD, 0, 0, acc, tq);
                stage_flush_dot<T>(stg, (T *)p.dv + (row0 * H + h) * DV, (long)H * DV, 32 * va(sI), 32 * vbk(sI), nvalid, sV, SM::LV,
                                   sCv + vbk(sI) * C);
            } else {
                acc_store<T, true>(stg, (T *)p.dv + (row0 * H + h) * DV, (long)H * DV, 32 * va(sI), 32 * vbk(sI), nvalid, acc, tq);
            }
        }
        if (cc) acc_to_lds_t<T>(sM1T, SM::LT, 32 * mi, 32 * ni, m1, tq); // Q's bytes: dead since dK1 (the inverse scratch, too)
        lds_barrier(); fresh(); // dX is dead
        if (cc) { // dA = -tril(X^T M1, -1); dA o G to sProd; Ah = diag(beta) dA into sDX
            f32x16 acc = zero16();
            if (!upper) {
                if (mi == 1) mma<32, true, false, T, true, MB>(acc, sXn + 32 * SM::LT + 32, SM::LT, sM1T + 32 * ni * SM::LT + 32, SM::LT, tq);
                else mma<C, true, false, T, true, MB>(acc, sXn, SM::LT, sM1T + 32 * ni * SM::LT, SM::LT, tq);
            }
            const int l31 = tq & 31, hh = (tq & 63) >> 5;
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = 32 * mi + 8 * (e >> 2) + 4 * hh + (e & 3), j = 32 * ni + l31;
                const float da = j < i ? -acc[e] : 0.f;
                sProd[i * SM::LF + j] = da * g[e];
                sDX[i * SM::LT + j] = from_f32<T>(sBeta[i] * da);
            }
        }
        if (gated) { // this wave's share of <dS_C, S_C>, summed in a fixed order after the barrier
            float zw = zp;
#pragma unroll
            for (int d = 32; d >= 1; d >>= 1) zw += __shfl_xor(zw, d);
            if ((tq & 63) == 0) sZ[wave] = zw;
        }
        lds_barrier(); fresh();
#pragma unroll
        for (int sI = 0; sI < KW; ++sI) if (kt(sI) < KT) { // dK = dK1 + diag(beta) dKb + Ah K + Ah^T K; Ah is strictly lower triangular
            if (ka(sI) == 0) mma<32, false, true, T, true, MB>(dk1[sI], sDX, SM::LT, sK + 32 * kb(sI), SM::LK, tq);
            else mma<C, false, true, T, true, MB>(dk1[sI], sDX + 32 * SM::LT, SM::LT, sK + 32 * kb(sI), SM::LK, tq);
            if (ka(sI) == 1) mma<32, true, true, T, true, MB>(dk1[sI], sDX + 32 * SM::LT + 32, SM::LT, sK + 32 * SM::LK + 32 * kb(sI), SM::LK, tq);
            else mma<C, true, true, T, true, MB>(dk1[sI], sDX, SM::LT, sK + 32 * kb(sI), SM::LK, tq);
            if (PRO) { // dW's bytes are free
                acc_to_lds<T>(sDK, SM::LQO, 32 * ka(sI), 32 * kb(sI), dk1[sI], tq);
            } else {
                acc_store<T, true>(stg, (T *)p.dk + (row0 * H + h) * DK, (long)H * DK, 32 * ka(sI), 32 * kb(sI), nvalid, dk1[sI], tq);
            }
        }
        if (gated && tid < C) {
            // Gate gradient.  o_t is linear in q_t and in the state, so the sensitivity to a rescaling of the
            // state at token j can be read off the other gradients:
            //     dg_j = <dS_C, S_C> + sum_{i = j .. end of the chunk} (q_i . dq_i - v_i . dv_i).
            // Thread t takes token C - 1 - t; an inclusive scan over t is the suffix sum over tokens.
            const int tok = C - 1 - tid;
            float c = 0.f;
#pragma unroll
            for (int b = 0; b < DK / 32; ++b) c += sCq[b * C + tok];
            float cv = 0.f;
#pragma unroll
            for (int b = 0; b < DV / 32; ++b) cv += sCv[b * C + tok];
            c -= cv * sGam[tok]; // v_i . dv_i = gamma_i (v_i / gamma_i) . dv_i
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const float up = __shfl_up(c, d);
                if (tid >= d) c += up;
            }
            const float z = ((sZ[0] + sZ[1]) + (sZ[2] + sZ[3])) + ((sZ[4] + sZ[5]) + (sZ[6] + sZ[7]));
            if (tok < nvalid) p.dg[(row0 + tok) * H + h] = c + z;
        }
        if (tq < 256) { // dbeta = column sums from part 1 + row sums of dA o G
            const int i = tq >> 2, seg = tq & 3;
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
        if (PRO) { // dk is assembled: back through the feature map, as for dq
            lds_barrier(); fresh();
            r.raw.feature_map_bwd_store(sDK, SM::LQO, (T *)p.dk + (row0 * H + h) * DK, (long)H * DK, nvalid, tq);
        }
        lds_barrier(); fresh(); // every buffer is free for the next tile
        it = nx;
        cur = np;
    }
}

} // namespace dn
