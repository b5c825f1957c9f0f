// Device-side building blocks for the gfx950 DeltaNet kernels: MFMA tile products from LDS,
// accumulator <-> LDS/global movers, tile loaders, the 64x64 unit-lower-triangular inverse.
// Every kernel here runs with 256 threads (4 wavefronts of 64) and a chunk of C = 64 tokens.
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

// Per-element-type constants: LDS row padding (elements) and elements per 16 bytes.
template <typename T> struct El;
template <> struct El<float> { static constexpr int PAD = 4; static constexpr int VEC = 4; };
template <> struct El<bf16>  { static constexpr int PAD = 8; static constexpr int VEC = 8; };

template <typename T> __host__ __device__ constexpr int ldn(int cols) { return cols + El<T>::PAD; }

__device__ inline float to_f32(float x) { return x; }
__device__ inline float to_f32(bf16 x) { return (float)x; }
template <typename T> __device__ inline T from_f32(float x) { return (T)x; }

// Where the chains live.  Dense batches are N = B sequences of length L at rows n*L; packed
// batches read cu_seqlens and a device-computed prefix of per-sequence chunk counts.
struct SeqMap {
    const int32_t *cu;   // device [N+1] or nullptr
    const int32_t *coff; // device [N+1] chunk offsets (packed only)
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
// acc(32x32) += A(32 x KDIM) * B(32 x KDIM)^T, both operands in LDS with the contraction index
// contiguous.  v_mfma_f32_32x32x16_bf16: lane l feeds row/col (l & 31) and 8 consecutive k starting
// at 8*(l >> 5); v_mfma_f32_32x32x2_f32: one k = (l >> 5).  The accumulator holds, for lane l,
// column (l & 31) and rows 8*g + 4*(l >> 5) + i at index 4*g + i.
template <int KDIM>
__device__ inline void mma_nt(f32x16 &acc, const bf16 *A, int lda, const bf16 *B, int ldb) {
    const int lane = threadIdx.x & 63, r = lane & 31, h = lane >> 5;
    const bf16 *pa = A + r * lda + h * 8;
    const bf16 *pb = B + r * ldb + h * 8;
#pragma unroll
    for (int k0 = 0; k0 < KDIM; k0 += 16) {
        bf16x8 a = *reinterpret_cast<const bf16x8 *>(pa + k0);
        bf16x8 b = *reinterpret_cast<const bf16x8 *>(pb + k0);
        acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
    }
}
template <int KDIM>
__device__ inline void mma_nt(f32x16 &acc, const float *A, int lda, const float *B, int ldb) {
    const int lane = threadIdx.x & 63, r = lane & 31, h = lane >> 5;
    const float *pa = A + r * lda + h;
    const float *pb = B + r * ldb + h;
#pragma unroll 8
    for (int k0 = 0; k0 < KDIM; k0 += 2)
        acc = __builtin_amdgcn_mfma_f32_32x32x2f32(pa[k0], pb[k0], acc, 0, 0, 0);
}

__device__ inline f32x16 zero16() {
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// visit every accumulator element: f(row, col, value&) with row, col inside the 32x32 tile
template <typename F> __device__ inline void acc_each(f32x16 &acc, F f) {
    const int lane = threadIdx.x & 63, col = lane & 31, h = lane >> 5;
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
template <typename F> __device__ inline void acc_each4(const f32x16 &acc, F f) {
    const int lane = threadIdx.x & 63, col = lane & 31, h = lane >> 5;
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
template <typename T> __device__ inline void acc_to_lds(T *dst, int ld, int row0, int col0, f32x16 &acc) {
    acc_each(acc, [&](int r, int c, float &v) { dst[(row0 + r) * ld + col0 + c] = from_f32<T>(v); });
}
// ... and transposed: dstT[col][row], 4 consecutive rows per store
template <typename T> __device__ inline void acc_to_lds_t(T *dstT, int ldT, int row0, int col0, const f32x16 &acc) {
    acc_each4(acc, [&](int r, int c, float a, float b, float cc, float d) {
        st4(dstT + (col0 + c) * ldT + row0 + r, a, b, cc, d);
    });
}
// tile -> global, rows >= nvalid dropped; dst points at (row 0, col 0) of the C-row block
template <typename T>
__device__ inline void acc_to_global(T *dst, long row_stride, int row0, int col0, int nvalid, f32x16 &acc) {
    acc_each(acc, [&](int r, int c, float &v) {
        if (row0 + r < nvalid) dst[(long)(row0 + r) * row_stride + col0 + c] = from_f32<T>(v);
    });
}

// ---------------------------------------------------------------------------------------------
// Global -> LDS: ROWS x COLS tile, 16-byte loads, rows >= nvalid become zero.
template <typename T, int ROWS, int COLS>
__device__ inline void load_tile(T *dst, int ld, const T *src, long row_stride, int nvalid) {
    constexpr int VEC = El<T>::VEC, TPR = COLS / VEC, RPI = NTHR / TPR;
    static_assert(COLS % VEC == 0 && NTHR % TPR == 0 && ROWS % RPI == 0, "tile shape");
    const int tr = threadIdx.x / TPR, tc = (threadIdx.x % TPR) * VEC;
#pragma unroll
    for (int r0 = 0; r0 < ROWS; r0 += RPI) {
        const int r = r0 + tr;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (r < nvalid) val = *reinterpret_cast<const uint4 *>(src + (long)r * row_stride + tc);
        *reinterpret_cast<uint4 *>(dst + r * ld + tc) = val;
    }
}
// LDS -> global, ROWS x COLS, rows >= nvalid dropped
template <typename T, int ROWS, int COLS>
__device__ inline void store_tile(T *dst, long row_stride, const T *src, int ld, int nvalid) {
    constexpr int VEC = El<T>::VEC, TPR = COLS / VEC, RPI = NTHR / TPR;
    const int tr = threadIdx.x / TPR, tc = (threadIdx.x % TPR) * VEC;
#pragma unroll
    for (int r0 = 0; r0 < ROWS; r0 += RPI) {
        const int r = r0 + tr;
        if (r < nvalid)
            *reinterpret_cast<uint4 *>(dst + (long)r * row_stride + tc) = *reinterpret_cast<const uint4 *>(src + r * ld + tc);
    }
}
// LDS -> LDS transpose of a C x COLS tile: dstT[c][r] = src[r][c].  Lanes run along r so that the
// narrow stores of one instruction fall into consecutive addresses.
template <typename T, int COLS>
__device__ inline void transpose_tile(T *dstT, int ldT, const T *src, int ld) {
    constexpr int VEC = El<T>::VEC, NG = COLS / VEC;
    const int r = threadIdx.x & 63, g0 = threadIdx.x >> 6;
#pragma unroll
    for (int g = g0; g < NG; g += NWAVE) {
        alignas(16) T tmp[VEC];
        *reinterpret_cast<uint4 *>(tmp) = *reinterpret_cast<const uint4 *>(src + r * ld + g * VEC);
#pragma unroll
        for (int i = 0; i < VEC; ++i) dstT[(g * VEC + i) * ldT + r] = tmp[i];
    }
}

// ---------------------------------------------------------------------------------------------
// X = (I + A)^{-1} for a 64x64 strictly-lower-triangular A (fp32, LDS, leading dimension ld).
// Forward substitution (section 3.2, "inverse of lower triangular matrices ... forward
// substitution") done blockwise: the four 16x16 diagonal blocks column by column inside one
// wavefront each, then block row a = 1..3 from X_ab = -X_aa * sum_{c=b}^{a-1} A_ac X_cb.
// sM is scratch of 16 x ldm floats, ldm >= 48.  Ends with a barrier; sX holds the full matrix.
__device__ inline void tri_inverse_64(const float *sA, float *sX, float *sM, int ld, int ldm) {
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
    for (int e = tid; e < C * C; e += NTHR) sX[(e >> 6) * ld + (e & 63)] = 0.f;
    __syncthreads();
    if (lane < 16) {
        const int b = wave * 16, j = lane;
        float x[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            float s = (i == j) ? 1.f : 0.f;
#pragma unroll
            for (int m = 0; m < i; ++m) s -= sA[(b + i) * ld + b + m] * x[m];
            x[i] = (i < j) ? 0.f : s;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) sX[(b + i) * ld + b + j] = x[i];
    }
    __syncthreads();
    const int i = tid >> 4, j = tid & 15;
    for (int a = 1; a < 4; ++a) {
        for (int b = 0; b < a; ++b) {
            float s = 0.f;
            for (int c = b; c < a; ++c)
#pragma unroll
                for (int m = 0; m < 16; ++m) s += sA[(16 * a + i) * ld + 16 * c + m] * sX[(16 * c + m) * ld + 16 * b + j];
            sM[i * ldm + 16 * b + j] = s;
        }
        __syncthreads();
        for (int b = 0; b < a; ++b) {
            float s = 0.f;
#pragma unroll
            for (int m = 0; m < 16; ++m) s += sX[(16 * a + i) * ld + 16 * a + m] * sM[m * ldm + 16 * b + j];
            sX[(16 * a + i) * ld + 16 * b + j] = -s;
        }
        __syncthreads();
    }
}

} // namespace dn
