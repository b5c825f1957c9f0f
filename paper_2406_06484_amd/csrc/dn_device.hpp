// Device-side building blocks for the gfx950 DeltaNet kernels: MFMA tile products from LDS,
// accumulator <-> LDS/global movers, tile loaders, the 64x64 unit-lower-triangular inverse.
// The chunk is C = 64 tokens; the prep kernel runs 4 wavefronts, the scans and the chunk kernel 8.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace dn {

constexpr int C = 64;     // chunk size (section 3.2)
constexpr int NTHR = 256; // threads per workgroup
constexpr int NWAVE = 4;

typedef __bf16 bf16;
typedef bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also drains every outstanding
// global load and store of the wave (it is a full workgroup fence), which would serialise the
// register prefetch of the next chunk and the output stores with the barrier.  Every barrier in
// these kernels guards LDS contents only; nothing written to global memory is read back by the
// same launch.
__device__ inline void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

// Global loads go through raw buffer descriptors: one 32-bit per-lane offset serves a whole tile
// (the row step rides in the scalar offset), and rows past the end of a ragged chunk are masked by
// pointing their lanes beyond the descriptor's range, which makes the hardware return zeros.
// This keeps 64-bit per-load address pairs and exec-mask branches out of the prefetch code.
typedef int i32x4 __attribute__((ext_vector_type(4)));
// Cache-policy bits of the loads and stores, per stream of tiles (0 = default, 2 = non-temporal; measured variant by
// variant on the fwd+bwd step, kernels of one step timed side by side on the same device):
//   tiles the launch reads once and no later kernel of the same call needs: non-temporal loads (every operand of the
//     chunk kernel; V in the forward scan, whose two workgroups per chain read different column blocks)
//   tiles that the other workgroup of the chain reads too (Q, K, T in the scans) or that the next kernel of the call reads
//     (K in k_wy_prep, dO in the reverse scan): default policy, they are found in the L2 or the memory-side cache
//   every tile store of the scans, k_wy_prep and the chunk kernel: non-temporal (nothing is read back by the same launch)
constexpr int kAuxOnce = 2, kAuxKeep = 0;
constexpr int kBufRange = 0x40000000; // bytes covered by a descriptor; offsets >= this read as zero
__device__ inline __amdgpu_buffer_rsrc_t make_rsrc(const void *base) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, kBufRange, 0x00020000);
}
// AUX = the instruction's cache-policy bits: 0 = default, 2 = non-temporal (data that this launch reads once)
template <int AUX = 0> __device__ inline uint4 buf_load16(__amdgpu_buffer_rsrc_t rs, int voff, int soff) {
    return __builtin_bit_cast(uint4, __builtin_amdgcn_raw_buffer_load_b128(rs, voff, soff, AUX));
}

// Per-element-type constants: LDS row padding (elements) and elements per 16 bytes.
template <typename T> struct El;
template <> struct El<float> { static constexpr int PAD = 4; static constexpr int VEC = 4; };
template <> struct El<bf16>  { static constexpr int PAD = 16; static constexpr int VEC = 8; };

template <typename T> __host__ __device__ constexpr int ldn(int cols) { return cols + El<T>::PAD; }
// leading dimension for tiles that are only ever read with the contraction index contiguous
template <typename T> __host__ __device__ constexpr int ldc(int cols) { return cols + 16 / (int)sizeof(T); }

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ inline T from_f32(float x) { return (T)x; }
// logistic function in explicit single-rounding steps, so that every kernel that evaluates it gets the same bits
__device__ inline float sigmoid_f32(float x) { return __frcp_rn(__fadd_rn(1.f, __expf(-x))); }
// ... and with the hardware reciprocal (1 ulp), for values that no other kernel has to reproduce bit for bit
__device__ inline float sigmoid_fast_f32(float x) { return __builtin_amdgcn_rcpf(1.f + __expf(-x)); }

// Where the chains live.  Dense batches are N = B sequences of length L at rows n*L; packed
// batches read cu_seqlens and a device-computed prefix of per-sequence chunk counts.
struct SeqMap {
    const int32_t *cu;   // device [N+1] or nullptr
    const int32_t *coff; // device [N+1] chunk offsets (packed only)
    const int32_t *order; // device [N] sequences by decreasing length (packed only), for the chain-serial kernels
    int N, L, ncd;       // ncd = chunks per dense sequence
    __device__ void seq(int n, int &t0, int &len, int &cb) const {
        if (cu) { t0 = cu[n]; len = cu[n + 1] - t0; cb = coff[n]; }
        else { t0 = n * L; len = L; cb = n * ncd; }
    }
    // maps a global chunk id to (sequence, chunk within it); false if past the end
    __device__ bool chunk(int gid, int &n, int &ic) const {
        if (!cu) {
            if (gid >= N * ncd) return false;
            n = gid / ncd; ic = gid - n * ncd; return true;
        }
        if (gid >= coff[N]) return false;
        int lo = 0, hi = N; // coff[lo] <= gid < coff[hi]
        while (hi - lo > 1) { int mid = (lo + hi) >> 1; if (coff[mid] <= gid) lo = mid; else hi = mid; }
        n = lo; ic = gid - coff[lo]; return true;
    }
};

// ---------------------------------------------------------------------------------------------
// The 32x32 MFMAs.  v_mfma_f32_32x32x16_bf16: lane l feeds row/col (l & 31) and 8 consecutive k
// starting at 8*(l >> 5); v_mfma_f32_32x32x2_f32: one k = (l >> 5).  The accumulator holds, for
// lane l, column (l & 31) and rows 8*g + 4*(l >> 5) + i at index 4*g + i.
//
// Operand fragments for the 32x32 MFMAs, from LDS, in two storage orders:
//   KC  storage [n][k], contraction index contiguous  (one 16-byte read per lane in bf16)
//   KS  storage [k][n], contraction index strided     (bf16: two ds_read_b64_tr_b16, the CDNA4
//       transposing LDS read; fp32: a plain read, since an fp32 fragment is one element per lane)
// `base` points at (n0, k = 0) for KC and at (k = 0, n0) for KS.  Both orders give lane l the
// operand row/column n0 + (l & 31) and, in bf16, k = k0 + 8*(l >> 5) + 0..7.
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

// (`tx`: the thread index as the caller wants it seen.  The default is threadIdx.x itself; a kernel that wants the per-lane
// address arithmetic formed where it is used, rather than hoisted out of its outer loop and carried through it, passes a
// copy it has taken through an empty asm.)
__device__ inline bf16x8 frag_kc(const bf16 *base, int ld, int k0, int tx = threadIdx.x) {
    const int lane = tx & 63;
    return *reinterpret_cast<const bf16x8 *>(base + (lane & 31) * ld + k0 + 8 * (lane >> 5));
}
__device__ inline bf16x8 frag_ks(const bf16 *base, int ld, int k0, int tx = threadIdx.x) {
    // Within each group of 16 lanes the transposing read hands lane i the 16-bit element (i & 3) of
    // the four 8-byte rows addressed by lanes (i >> 2), (i >> 2) + 4, + 8, + 12.  With lane i
    // pointing at row k0' + (i >> 2), columns 4*(i & 3).., lane i ends up with column i, rows k0'..k0'+3.
    const int lane = tx & 63, i = lane & 15;
    const bf16 *p = base + (k0 + 8 * (lane >> 5) + (i >> 2)) * ld + (lane & 16) + 4 * (i & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * ld));
    const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, v);
}
__device__ inline float frag_kc(const float *base, int ld, int k0, int tx = threadIdx.x) {
    const int lane = tx & 63;
    return base[(lane & 31) * ld + k0 + (lane >> 5)];
}
__device__ inline float frag_ks(const float *base, int ld, int k0, int tx = threadIdx.x) {
    const int lane = tx & 63;
    return base[(k0 + (lane >> 5)) * ld + (lane & 31)];
}
__device__ inline void mfma32(f32x16 &acc, bf16x8 a, bf16x8 b) { acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0); }
__device__ inline void mfma32(f32x16 &acc, float a, float b) { acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, acc, 0, 0, 0); }
template <typename T> struct FragOf;
template <> struct FragOf<bf16> { typedef bf16x8 type; static constexpr int KPL = 8; };
template <> struct FragOf<float> { typedef float type; static constexpr int KPL = 1; };
template <typename T> struct KStep;
template <> struct KStep<bf16> { static constexpr int value = 16; };
template <> struct KStep<float> { static constexpr int value = 2; };

// acc(32x32) += A * B over KDIM contraction steps; AKS / BKS select the storage order of each operand.
// The operand fragments of up to BATCH steps are requested from LDS before the first MFMA of the
// batch issues (and the next batch's before this batch's MFMAs), so one LDS latency is exposed per
// product instead of one per pair of steps, which is what the compiler's own schedule gives.
template <typename T> struct MmaBatch;
template <> struct MmaBatch<bf16> { static constexpr int value = 8; };   // 8 steps x 2 operands x 4 VGPRs
template <> struct MmaBatch<float> { static constexpr int value = 16; }; // 16 steps x 2 operands x 1 VGPR
template <int KDIM, bool AKS, bool BKS, typename T, bool FENCE = true, int BATCH_ = 0>
__device__ inline void mma(f32x16 &acc, const T *A, int lda, const T *B, int ldb, int tx = threadIdx.x) {
    constexpr int KS = KStep<T>::value, N = KDIM / KS;
    constexpr int WANT = BATCH_ ? BATCH_ : MmaBatch<T>::value;
    constexpr int BATCH = N < WANT ? N : WANT, NB = (N + BATCH - 1) / BATCH;
    static_assert(N % BATCH == 0, "contraction length must be a multiple of the batch");
    typedef typename FragOf<T>::type frag_t;
    frag_t a[2][BATCH], b[2][BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
        a[0][j] = AKS ? frag_ks(A, lda, j * KS, tx) : frag_kc(A, lda, j * KS, tx);
        b[0][j] = BKS ? frag_ks(B, ldb, j * KS, tx) : frag_kc(B, ldb, j * KS, tx);
    }
#pragma unroll
    for (int ib = 0; ib < NB; ++ib) {
        if (ib + 1 < NB) {
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const int k0 = ((ib + 1) * BATCH + j) * KS;
                a[(ib + 1) & 1][j] = AKS ? frag_ks(A, lda, k0, tx) : frag_kc(A, lda, k0, tx);
                b[(ib + 1) & 1][j] = BKS ? frag_ks(B, ldb, k0, tx) : frag_kc(B, ldb, k0, tx);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < BATCH; ++j) mfma32(acc, a[ib & 1][j], b[ib & 1][j]);
    }
    // FENCE keeps the scheduler from hoisting the next product's operand loads over this one (register
    // pressure); without it the next product's loads may overlap this product's MFMAs.
    if (FENCE) __builtin_amdgcn_sched_barrier(0);
}

// Two products with the same B operand: acc1 += A1 * B, acc2 += A2 * B; B's fragments are read from LDS once.
template <int KDIM, bool A1KS, bool A2KS, bool BKS, typename T, int BATCH_>
__device__ inline void mma_shared_b(f32x16 &acc1, f32x16 &acc2, const T *A1, int lda1, const T *A2, int lda2, const T *B, int ldb,
                                    int tx = threadIdx.x) {
    constexpr int KS = KStep<T>::value, N = KDIM / KS;
    constexpr int BATCH = N < BATCH_ ? N : BATCH_, NB = N / BATCH;
    static_assert(N % BATCH == 0, "contraction length must be a multiple of the batch");
    typedef typename FragOf<T>::type frag_t;
    frag_t a1[2][BATCH], a2[2][BATCH], b[2][BATCH];
#pragma unroll
    for (int j = 0; j < BATCH; ++j) {
        b[0][j] = BKS ? frag_ks(B, ldb, j * KS, tx) : frag_kc(B, ldb, j * KS, tx);
        a1[0][j] = A1KS ? frag_ks(A1, lda1, j * KS, tx) : frag_kc(A1, lda1, j * KS, tx);
        a2[0][j] = A2KS ? frag_ks(A2, lda2, j * KS, tx) : frag_kc(A2, lda2, j * KS, tx);
    }
#pragma unroll
    for (int ib = 0; ib < NB; ++ib) {
        if (ib + 1 < NB) {
#pragma unroll
            for (int j = 0; j < BATCH; ++j) {
                const int k0 = ((ib + 1) * BATCH + j) * KS;
                b[(ib + 1) & 1][j] = BKS ? frag_ks(B, ldb, k0, tx) : frag_kc(B, ldb, k0, tx);
                a1[(ib + 1) & 1][j] = A1KS ? frag_ks(A1, lda1, k0, tx) : frag_kc(A1, lda1, k0, tx);
                a2[(ib + 1) & 1][j] = A2KS ? frag_ks(A2, lda2, k0, tx) : frag_kc(A2, lda2, k0, tx);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int j = 0; j < BATCH; ++j) {
            mfma32(acc1, a1[ib & 1][j], b[ib & 1][j]);
            mfma32(acc2, a2[ib & 1][j], b[ib & 1][j]);
        }
    }
    __builtin_amdgcn_sched_barrier(0);
}

__device__ inline f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// visit every accumulator element: f(row, col, value&) with row, col inside the 32x32 tile
template <typename F> __device__ inline void acc_each(f32x16 &acc, F f, int tx = threadIdx.x) {
    const int lane = tx & 63, col = lane & 31, h = lane >> 5;
#pragma unroll
    for (int g = 0; g < 4; ++g)
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float v = acc[4 * g + i]; // vector elements cannot bind to a reference
            f(8 * g + 4 * h + i, col, v);
            acc[4 * g + i] = v;
        }
}
// visit runs of 4 consecutive rows: f(row0, col, v0, v1, v2, v3)
template <typename F> __device__ inline void acc_each4(const f32x16 &acc, F f, int tx = threadIdx.x) {
    const int lane = tx & 63, col = lane & 31, h = lane >> 5;
#pragma unroll
    for (int g = 0; g < 4; ++g) f(8 * g + 4 * h, col, acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
}

__device__ inline void st4(float *p, float a, float b, float c, float d) {
    *reinterpret_cast<f32x4 *>(p) = f32x4{a, b, c, d};
}
__device__ inline void st4(bf16 *p, float a, float b, float c, float d) {
    *reinterpret_cast<bf16x4 *>(p) = bf16x4{(bf16)a, (bf16)b, (bf16)c, (bf16)d};
}

// tile (32x32) of the accumulator -> LDS, row-major destination dst[row][col]
template <typename T> __device__ inline void acc_to_lds(T *dst, int ld, int row0, int col0, f32x16 &acc, int tx = threadIdx.x) {
    acc_each(acc, [&](int r, int c, float &v) { dst[(row0 + r) * ld + col0 + c] = from_f32<T>(v); }, tx);
}
// ... and transposed: dstT[col][row], 4 consecutive rows per store
template <typename T> __device__ inline void acc_to_lds_t(T *dstT, int ldT, int row0, int col0, const f32x16 &acc, int tx = threadIdx.x) {
    acc_each4(acc, [&](int r, int c, float a, float b, float cc, float d) {
        st4(dstT + (col0 + c) * ldT + row0 + r, a, b, cc, d);
    }, tx);
}
// Wave-private LDS staging for coalesced tile stores.  A 32 x 32 accumulator tile is first laid
// out row-major in LDS (cheap narrow LDS writes), then each lane moves 16 bytes at a time to global
// memory, so a store instruction covers whole 64-byte (bf16) or 128-byte (fp32) row segments.
// Scattered 2-byte global stores straight from the accumulator layout cost ~100 cycles apiece.
template <typename T> struct Stage {
    static constexpr int LD = 32 + 16 / (int)sizeof(T);       // row stride in elements, 16-byte aligned
    static constexpr int ELEMS = 32 * LD;                      // per wave
    static constexpr int SEGS = 32 * (int)sizeof(T) / 16;      // 16-byte segments per row
};
__device__ inline void wave_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

// ONCE: non-temporal store, for output that nothing reads again before the launch ends
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
template <typename T, bool ONCE = false>
__device__ inline void stage_flush(const T *stage, T *dst, long row_stride, int row0, int col0, int nvalid, int tx = threadIdx.x) {
    const int lane = tx & 63;
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < 32 * Stage<T>::SEGS / 64; ++it) {
        const int idx = it * 64 + lane, r = idx / Stage<T>::SEGS, sg = idx % Stage<T>::SEGS;
        if (row0 + r < nvalid) {
            const u32x4 val = *reinterpret_cast<const u32x4 *>(stage + r * Stage<T>::LD + sg * El<T>::VEC);
            u32x4 *to = reinterpret_cast<u32x4 *>(dst + (long)(row0 + r) * row_stride + col0 + sg * El<T>::VEC);
            if (ONCE) __builtin_nontemporal_store(val, to);
            else *to = val;
        }
    }
    wave_lds_fence(); // the staging tile may be rewritten right away
}
// stage_flush that also returns row dot products of the staged tile with the matching 32 x 32 block of
// an LDS-resident matrix `other` (leading dimension ldo): slot[row0 + r] = sum_c stage(r, c) *
// other(row0 + r, col0 + c), written by one lane per row.  Used for the per-token terms of the gate gradient.
template <typename T>
__device__ inline void stage_flush_dot(const T *stage, T *dst, long row_stride, int row0, int col0, int nvalid,
                                       const T *other, int ldo, float *slot) {
    constexpr int SEGS = Stage<T>::SEGS, VEC = El<T>::VEC;
    const int lane = threadIdx.x & 63;
    wave_lds_fence();
#pragma unroll
    for (int it = 0; it < 32 * SEGS / 64; ++it) {
        const int idx = it * 64 + lane, r = idx / SEGS, sg = idx % SEGS;
        alignas(16) T a[VEC], b[VEC];
        *reinterpret_cast<uint4 *>(a) = *reinterpret_cast<const uint4 *>(stage + r * Stage<T>::LD + sg * VEC);
        *reinterpret_cast<uint4 *>(b) = *reinterpret_cast<const uint4 *>(other + (row0 + r) * ldo + col0 + sg * VEC);
        if (row0 + r < nvalid)
            *reinterpret_cast<uint4 *>(dst + (long)(row0 + r) * row_stride + col0 + sg * VEC) = *reinterpret_cast<const uint4 *>(a);
        float s = 0.f;
#pragma unroll
        for (int u = 0; u < VEC; ++u) s += to_f32(a[u]) * to_f32(b[u]);
#pragma unroll
        for (int d = 1; d < SEGS; d <<= 1) s += __shfl_xor(s, d); // the SEGS lanes of one row are adjacent
        if (sg == 0) slot[row0 + r] = s;
    }
    wave_lds_fence();
}
// dst[row0 + r][col0 + c] = acc(r, c), rows >= nvalid dropped; `stage` is this wave's staging tile
template <typename T, bool ONCE = false>
__device__ inline void acc_store(T *stage, T *dst, long row_stride, int row0, int col0, int nvalid, f32x16 &acc, int tx = threadIdx.x) {
    acc_to_lds<T>(stage, Stage<T>::LD, 0, 0, acc, tx);
    stage_flush<T, ONCE>(stage, dst, row_stride, row0, col0, nvalid, tx);
}
// ---------------------------------------------------------------------------------------------
// A ROWS x COLS tile fetched from global memory into registers (16 bytes per lane and step; rows >=
// nvalid read as zero), to be parked while LDS is busy and stored to LDS later.
template <typename T, int ROWS, int COLS, int NT = NTHR> struct TileRegs {
    static constexpr int VEC = El<T>::VEC, TPR = COLS / VEC, RPI = NT / TPR, NIT = ROWS / RPI;
    static_assert(COLS % VEC == 0 && NT % TPR == 0 && ROWS % RPI == 0, "tile shape");
    uint4 v[NIT];
    // `t` is the caller's index among the NT threads that share the tile (defaults to the whole workgroup)
    template <int AUX> __device__ inline void load_aux(const T *src, long row_stride, int nvalid, int t) {
        const int tr = t / TPR, tc = (t % TPR) * VEC;
        const __amdgpu_buffer_rsrc_t rs = make_rsrc(src);
        const int rs_bytes = (int)row_stride * (int)sizeof(T);
        const int voff = tr * rs_bytes + tc * (int)sizeof(T);
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            v[it] = buf_load16<AUX>(rs, it * RPI + tr < nvalid ? voff : kBufRange, it * RPI * rs_bytes);
    }
    __device__ inline void load(const T *src, long row_stride, int nvalid, int t = threadIdx.x) { load_aux<0>(src, row_stride, nvalid, t); }
    // for a tile that no other workgroup of the launch reads: non-temporal, it does not displace what the caches hold
    __device__ inline void load_once(const T *src, long row_stride, int nvalid, int t = threadIdx.x) { load_aux<kAuxOnce>(src, row_stride, nvalid, t); }
    __device__ inline void store(T *dst, int ld, int t = threadIdx.x) const {
        const int tr = t / TPR, tc = (t % TPR) * VEC;
#pragma unroll
        for (int it = 0; it < NIT; ++it) *reinterpret_cast<uint4 *>(dst + (it * RPI + tr) * ld + tc) = v[it];
    }
    // sum over the elements this lane holds of (this tile) * (a tile of the same shape parked in LDS by store())
    __device__ inline float dot_lds(const T *src, int ld, int t = threadIdx.x) const {
        const int tr = t / TPR, tc = (t % TPR) * VEC;
        float s = 0.f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T a[VEC], b[VEC];
            *reinterpret_cast<uint4 *>(a) = v[it];
            *reinterpret_cast<uint4 *>(b) = *reinterpret_cast<const uint4 *>(src + (it * RPI + tr) * ld + tc);
#pragma unroll
            for (int u = 0; u < VEC; ++u) s += to_f32(a[u]) * to_f32(b[u]);
        }
        return s;
    }
    // sum over the elements this lane holds of (this tile) * (another held tile of the same shape)
    __device__ inline float dot(const TileRegs &o) const {
        float s = 0.f;
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T a[VEC], b[VEC];
            *reinterpret_cast<uint4 *>(a) = v[it];
            *reinterpret_cast<uint4 *>(b) = o.v[it];
#pragma unroll
            for (int u = 0; u < VEC; ++u) s += to_f32(a[u]) * to_f32(b[u]);
        }
        return s;
    }
    // The query/key feature map of section 3.3 on the held tile, in place: every row x becomes
    // SiLU(x) / ||SiLU(x)||_2 (a row whose image is exactly zero, such as a row past the end, stays zero).
    // The TPR lanes that share a row are adjacent, so the row sum is a butterfly over them.
    // inv[it] = 1 / norm of the row held in step it (0 for a zero row).
    __device__ inline void feature_map(float (&inv)[NIT]) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T e[VEC];
            *reinterpret_cast<uint4 *>(e) = v[it];
            float sv[VEC], ss = 0.f;
#pragma unroll
            for (int u = 0; u < VEC; ++u) { // every step an explicit single-rounding operation: all kernels get the same bits
                const float x = to_f32(e[u]);
                sv[u] = __fmul_rn(x, sigmoid_f32(x));
                ss = __fmaf_rn(sv[u], sv[u], ss);
            }
#pragma unroll
            for (int d = 1; d < TPR; d <<= 1) ss = __fadd_rn(ss, __shfl_xor(ss, d));
            inv[it] = ss > 0.f ? __frsqrt_rn(ss) : 0.f;
#pragma unroll
            for (int u = 0; u < VEC; ++u) e[u] = from_f32<T>(__fmul_rn(sv[u], inv[it]));
            v[it] = *reinterpret_cast<const uint4 *>(e);
            __builtin_amdgcn_sched_barrier(0); // one step at a time: interleaved, the steps' temporaries do not fit
        }
    }
    // the same map, written to an LDS tile; the held tile keeps the pre-activations for feature_map_bwd_store
    __device__ inline void feature_map_to(T *dst, int ld, float (&inv)[NIT], int t = threadIdx.x) const {
        TileRegs y = *this;
        y.feature_map(inv);
        y.store(dst, ld, t);
    }
    // Gradient through the map, for a tile whose pre-activations x this object holds: src = dy in LDS
    // (same shape, leading dimension ld);
    //     dx = SiLU'(x) (dy - y (y . dy)) / ||SiLU(x)||,  SiLU'(x) = sig (1 + x (1 - sig)),  y = SiLU(x) / ||SiLU(x)||,
    // written to global memory (rows >= nvalid dropped).  A first pass forms the rows' norms and keeps every sigmoid (the
    // fast one: y need not have the bits of the mapped tile here); a row's sums are butterflies over its TPR lanes.
    __device__ inline void feature_map_bwd_store(const T *src, int ld, T *dst, long row_stride, int nvalid, int t = threadIdx.x) const {
        const int tr = t / TPR, tc = (t % TPR) * VEC;
        float sg[NIT][VEC], inv[NIT];
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T x[VEC];
            *reinterpret_cast<uint4 *>(x) = v[it];
            float ss = 0.f;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                const float xv = to_f32(x[u]);
                sg[it][u] = sigmoid_fast_f32(xv);
                const float sv = __fmul_rn(xv, sg[it][u]);
                ss = __fmaf_rn(sv, sv, ss);
            }
#pragma unroll
            for (int d = 1; d < TPR; d <<= 1) ss = __fadd_rn(ss, __shfl_xor(ss, d));
            inv[it] = ss > 0.f ? __frsqrt_rn(ss) : 0.f;
        }
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T x[VEC], a[VEC];
            *reinterpret_cast<uint4 *>(x) = v[it];
            *reinterpret_cast<uint4 *>(a) = *reinterpret_cast<const uint4 *>(src + (it * RPI + tr) * ld + tc);
            float y[VEC], dsl[VEC], dot = 0.f;
#pragma unroll
            for (int u = 0; u < VEC; ++u) {
                const float xv = to_f32(x[u]), s1 = sg[it][u];
                y[u] = __fmul_rn(__fmul_rn(xv, s1), inv[it]);
                dsl[u] = s1 * (1.f + xv * (1.f - s1)) * inv[it];
                dot += to_f32(a[u]) * y[u];
            }
#pragma unroll
            for (int d = 1; d < TPR; d <<= 1) dot += __shfl_xor(dot, d);
#pragma unroll
            for (int u = 0; u < VEC; ++u) a[u] = from_f32<T>((to_f32(a[u]) - y[u] * dot) * dsl[u]);
            if (it * RPI + tr < nvalid)
                *reinterpret_cast<uint4 *>(dst + (long)(it * RPI + tr) * row_stride + tc) = *reinterpret_cast<const uint4 *>(a);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // held tile -> global memory (rows >= nvalid dropped)
    __device__ inline void store_global(T *dst, long row_stride, int nvalid, int t = threadIdx.x) const {
        const int tr = t / TPR, tc = (t % TPR) * VEC;
#pragma unroll
        for (int it = 0; it < NIT; ++it)
            if (it * RPI + tr < nvalid)
                *reinterpret_cast<uint4 *>(dst + (long)(it * RPI + tr) * row_stride + tc) = v[it];
    }
    // Per-row factors for scale_rows: f[it] = src[row held in step it] (rows of the tile this lane touches).
    __device__ inline void load_row_factors(float (&f)[NIT], const float *src, int t = threadIdx.x) const {
        const int tr = t / TPR;
#pragma unroll
        for (int it = 0; it < NIT; ++it) f[it] = src[it * RPI + tr];
    }
    // held tile <- diag(f) * tile, in the storage type
    __device__ inline void scale_rows(const float (&f)[NIT]) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            alignas(16) T e[VEC];
            *reinterpret_cast<uint4 *>(e) = v[it];
#pragma unroll
            for (int u = 0; u < VEC; ++u) e[u] = from_f32<T>(to_f32(e[u]) * f[it]);
            v[it] = *reinterpret_cast<const uint4 *>(e);
        }
    }
};
// ---------------------------------------------------------------------------------------------
// Global -> LDS: ROWS x COLS tile, 16-byte loads, rows >= nvalid become zero.
template <typename T, int ROWS, int COLS>
__device__ inline void load_tile(T *dst, int ld, const T *src, long row_stride, int nvalid) {
    constexpr int VEC = El<T>::VEC, TPR = COLS / VEC, RPI = NTHR / TPR;
    static_assert(COLS % VEC == 0 && NTHR % TPR == 0 && ROWS % RPI == 0, "tile shape");
    TileRegs<T, ROWS, COLS> regs;
    regs.load(src, row_stride, nvalid);
    regs.store(dst, ld);
}
// LDS -> global copy of a ROWS x COLS tile by NT cooperating threads (t = index among them); the
// destination is a contiguous row-major block
template <typename T, int ROWS, int COLS, int NT, bool ONCE = false>
__device__ inline void copy_out(T *dst, const T *src, int ld, int t) {
    constexpr int VEC = El<T>::VEC, TPR = COLS / VEC, RPI = NT / TPR;
    static_assert(COLS % VEC == 0 && NT % TPR == 0 && ROWS % RPI == 0, "tile shape");
    const int tr = t / TPR, tc = (t % TPR) * VEC;
#pragma unroll
    for (int r0 = 0; r0 < ROWS; r0 += RPI) {
        const u32x4 val = *reinterpret_cast<const u32x4 *>(src + (r0 + tr) * ld + tc);
        u32x4 *to = reinterpret_cast<u32x4 *>(dst + (long)(r0 + tr) * COLS + tc);
        if (ONCE) __builtin_nontemporal_store(val, to);
        else *to = val;
    }
}
// ---------------------------------------------------------------------------------------------
// X = (I + A)^{-1} for a 64x64 strictly-lower-triangular A (section 3.2: the inverse of the unit
// lower-triangular matrix of Eq. 10 by forward substitution), done blockwise and in place.
// On entry sX (fp32, leading dimension ld) holds the
// strictly lower triangular A with zeros elsewhere; on exit it holds X = (I + A)^{-1}.
// Blocked forward substitution: the eight 8x8 diagonal blocks are solved column by column (16
// lanes of every wavefront), then 2x2 block merges X21 = -X22 (A21 X11) double the block size
// 8 -> 16 -> 32 on the vector ALU in fp32 and 32 -> 64 on the matrix cores with operands of type T.
// sM: 512 floats of scratch (may share its bytes with sOp: it is dead before sOp is written).  sOp: 3 x 32 x LO elements of
// type T, LO >= 32 + 8.  Ends with a barrier.
template <typename T, int NT = NTHR>
__device__ inline void tri_inverse_64_inplace(float *sX, int ld, float *sM, T *sOp, int LO) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    const bool act = tid < 256; // the fp32 stages are laid out for 256 threads; extra waves only join the barriers
    if (act && lane < 16) {
        const int b = (2 * wave + (lane >> 3)) * 8, j = lane & 7;
        float x[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            float s = (i == j) ? 1.f : 0.f;
#pragma unroll
            for (int m = 0; m < i; ++m) s -= sX[(b + i) * ld + b + m] * x[m];
            x[i] = (i < j) ? 0.f : s;
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) sX[(b + i) * ld + b + j] = x[i];
    }
    lds_barrier();
    { // 8 -> 16: four merges, one output element per thread
        const int m = (tid >> 6) & 3, i = (tid >> 3) & 7, j = tid & 7, r0 = 16 * m + 8, c0 = 16 * m;
        float s = 0.f;
        if (act) {
#pragma unroll
            for (int k = 0; k < 8; ++k) s += sX[(r0 + i) * ld + c0 + k] * sX[(c0 + k) * ld + c0 + j];
            sM[tid] = s;
        }
        lds_barrier();
        if (act) {
            s = 0.f;
#pragma unroll
            for (int k = 0; k < 8; ++k) s += sX[(r0 + i) * ld + r0 + k] * sM[(m << 6) + k * 8 + j];
            sX[(r0 + i) * ld + c0 + j] = -s;
        }
        lds_barrier();
    }
    { // 16 -> 32: two merges, two output elements per thread
        const int m = (tid >> 7) & 1, i = (tid >> 3) & 15, j = 2 * (tid & 7), r0 = 32 * m + 16, c0 = 32 * m;
        float s0 = 0.f, s1 = 0.f;
        if (act) {
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float a = sX[(r0 + i) * ld + c0 + k];
                s0 += a * sX[(c0 + k) * ld + c0 + j];
                s1 += a * sX[(c0 + k) * ld + c0 + j + 1];
            }
            sM[(m << 8) + i * 16 + j] = s0;
            sM[(m << 8) + i * 16 + j + 1] = s1;
        }
        lds_barrier();
        if (act) {
            s0 = s1 = 0.f;
#pragma unroll
            for (int k = 0; k < 16; ++k) {
                const float a = sX[(r0 + i) * ld + r0 + k];
                s0 += a * sM[(m << 8) + k * 16 + j];
                s1 += a * sM[(m << 8) + k * 16 + j + 1];
            }
            sX[(r0 + i) * ld + c0 + j] = -s0;
            sX[(r0 + i) * ld + c0 + j + 1] = -s1;
        }
        lds_barrier();
    }
    // 32 -> 64 on the matrix cores: operands A21, X11^T, X22 and (later) M^T, each 32 x LO
    T *oA = sOp, *oX11T = sOp + 32 * LO, *oX22 = sOp + 64 * LO, *oMT = oA; // M^T takes A21's place: one wave reads the one, then writes the other
    for (int e = tid; e < 32 * 32; e += NT) {
        const int i = e >> 5, k = e & 31;
        oA[i * LO + k] = from_f32<T>(sX[(32 + i) * ld + k]);
        oX11T[k * LO + i] = from_f32<T>(sX[i * ld + k]);
        oX22[i * LO + k] = from_f32<T>(sX[(32 + i) * ld + 32 + k]);
    }
    lds_barrier();
    f32x16 acc = zero16();
    if (wave == 0) {
        mma<32, false, false, T>(acc, oA, LO, oX11T, LO); // M = A21 X11
        acc_to_lds_t<T>(oMT, LO, 0, 0, acc);
    }
    lds_barrier();
    if (wave == 0) {
        acc = zero16();
        mma<32, false, false, T>(acc, oX22, LO, oMT, LO); // X22 M
        acc_each(acc, [&](int r, int c, float &v) { sX[(32 + r) * ld + c] = -v; });
    }
    lds_barrier();
}

} // namespace dn
