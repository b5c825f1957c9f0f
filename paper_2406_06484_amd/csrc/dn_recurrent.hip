// Token-serial (recurrent-form) DeltaNet forward for gfx950: the delta-rule update of section 2.2
// applied one token at a time,
//
//     u_t = beta_t (v_t - S_{t-1}^T k_t),   S_t = S_{t-1} + k_t u_t^T,   o_t = S_t^T q_t,
//
// with the state in fp32 registers for the whole sequence.  This is the form the paper's speed
// comparison (section 3.3, the figure with sequence length on the x axis) measures the chunkwise
// form against, and the one a decoder runs for single-token steps.  There is no contraction wide
// enough for the matrix cores here: the work is 6 d_k fused multiply-adds per state column per token
// on the vector ALU.
//
// Mapping.  The d_v columns of the state are independent, so one wavefront owns 16 of them for one
// chain and never talks to another wavefront (no barrier).  Inside the wave, lane l = 16 * rb + j
// holds column j and the quarter rb of the d_k rows; the two reductions over d_k (S^T k and
// S^T q) finish with the two gfx950 lane swaps (v_permlane32_swap, v_permlane16_swap), which stay on
// the vector ALU.  A 16-column slice per wave gives chains * d_v / 16 waves: 1024 for 128 chains at
// d_v = 128, one per SIMD of the chip.
// Global latency (longer than a token takes) is hidden by staging: the wave fetches q, k, v, beta
// for a block of TB tokens with coalesced 16-byte loads, parks them in its private slice of LDS
// (two buffers), and works through the previous block meanwhile; all 16 lanes of a row quarter read
// the same k and q words from LDS (a broadcast, no bank conflict).  k and q are expanded to fp32 once,
// when the wave parks them, not by every one of the 16 column lanes that read them.
#include "dn_host.hpp"

namespace dn {

typedef __bf16 rbf16;

__device__ inline float rec_to_f32(float x) { return x; }
__device__ inline float rec_to_f32(rbf16 x) { return (float)x; }
__device__ inline void rec_store(float *p, float x) { *p = x; }
__device__ inline void rec_store(rbf16 *p, float x) { *p = (rbf16)x; }

// sum over the four lanes l, l ^ 16, l ^ 32, l ^ 48, delivered to all of them
__device__ inline float rec_sum4(float x) {
    const unsigned u = __float_as_uint(x);
    const auto a = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    const unsigned v = __float_as_uint(__uint_as_float(a[0]) + __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// R consecutive elements of type T held as raw 16-byte words, expanded to fp32 on demand
template <typename T, int R> struct RowRegs {
    static constexpr int NW = R * (int)sizeof(T) / 16;
    static_assert(NW >= 1 && NW * 16 == R * (int)sizeof(T), "row slice must be whole 16-byte words");
    uint4 w[NW];
    __device__ inline void load(const T *src) { // LDS or global, 16-byte aligned
#pragma unroll
        for (int i = 0; i < NW; ++i) w[i] = reinterpret_cast<const uint4 *>(src)[i];
    }
    __device__ inline void unpack(float (&f)[R]) const {
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const unsigned d[4] = {w[i].x, w[i].y, w[i].z, w[i].w};
#pragma unroll
            for (int c = 0; c < 4; ++c) {
                if (sizeof(T) == 4) f[4 * i + c] = __uint_as_float(d[c]);
                else { // two bf16 per dword: the fp32 value is the 16 bits moved to the top half
                    f[8 * i + 2 * c] = __uint_as_float(d[c] << 16);
                    f[8 * i + 2 * c + 1] = __uint_as_float(d[c] & 0xffff0000u);
                }
            }
        }
    }
};

constexpr int kRecCols = 16; // state columns per wavefront

// Tokens per staged block: 2 KB of k (and of q) per wave and buffer, at most 16 tokens.
template <typename T, int DK> struct RecStage {
    static constexpr int ROWB = DK * (int)sizeof(T);                  // bytes of one k or q row
    static constexpr int TB = 2048 / ROWB < 16 ? 2048 / ROWB : 16;
    static constexpr int ROWW = ROWB / 16;                            // 16-byte words per row
    static constexpr int NKW = TB * ROWW / 64;                        // k (or q) words per lane and block
    static constexpr int VROWW = kRecCols * (int)sizeof(T) / 16;      // 16-byte words of one token's v slice
    static_assert(TB >= 1 && TB * ROWW % 64 == 0 && TB * VROWW <= 64, "staging layout");
    static constexpr int ROWF = DK * 4;                               // k and q rows are parked as fp32
    static constexpr int oK = 0, oQ = TB * ROWF, oV = 2 * TB * ROWF, oB = oV + TB * kRecCols * (int)sizeof(T);
    static constexpr int oG = (oB + TB * (int)sizeof(T) + 3) & ~3;      // gated: alpha_t = exp(g_t), fp32
    static constexpr int bytes = (oG + TB * 4 + 15) & ~15;              // one buffer of one wave
};

template <typename T, int DK, bool GATED>
__global__ __launch_bounds__(256) void k_recurrent_fwd(RecArgs a) {
    using ST = RecStage<T, DK>;
    constexpr int R = DK / 4, TB = ST::TB; // rows per lane; tokens per block
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane & 15, rb = lane >> 4;
    const int chain = blockIdx.x, n = chain / a.H, h = chain - n * a.H;
    const int col0 = (blockIdx.y * 4 + wave) * kRecCols, col = col0 + j;
    if (col0 >= a.DV) return; // whole wave past the last column slice (no barriers below)
    int t0, len;
    if (a.cu) { // bounded to the tensors' rows, whatever the array holds: a malformed one no host copy was there to reject stays in bounds
        t0 = min(max(a.cu[n], 0), a.L);
        len = min(max(a.cu[n + 1], t0), a.L) - t0;
    }
    else { t0 = n * a.L; len = a.L; }
    const int H = a.H, DV = a.DV;
    unsigned char *buf0 = smem + wave * 2 * ST::bytes, *buf1 = buf0 + ST::bytes;

    float S[R];
    if (a.S0) {
        const float *src = a.S0 + ((long)chain * DK + rb * R) * DV + col;
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = src[(long)r * DV];
    } else {
#pragma unroll
        for (int r = 0; r < R; ++r) S[r] = 0.f;
    }

    // one block of tokens in flight: global -> registers (fetch), registers -> LDS (park)
    uint4 gk[ST::NKW], gq[ST::NKW], gv;
    T gb;
    float ga = 1.f; // gated variant (section 6, the overview table's last row): decay alpha_t = exp(g_t) on the old state
    auto fetch = [&](int tb) __attribute__((always_inline)) { // tokens tb .. tb + TB - 1 of this sequence
#pragma unroll
        for (int i = 0; i < ST::NKW; ++i) {
            const int w = i * 64 + lane, tok = w / ST::ROWW, pos = w % ST::ROWW;
            if (tb + tok < len) {
                const long row = ((long)(t0 + tb + tok) * H + h) * DK;
                gk[i] = reinterpret_cast<const uint4 *>((const T *)a.k + row)[pos];
                gq[i] = reinterpret_cast<const uint4 *>((const T *)a.q + row)[pos];
            } else { // past the end: zeros, so that the unrolled block below multiplies finite numbers
                gk[i] = make_uint4(0, 0, 0, 0);
                gq[i] = make_uint4(0, 0, 0, 0);
            }
        }
        {
            const int tok = lane / ST::VROWW, pos = lane % ST::VROWW;
            if (tok < TB && tb + tok < len)
                gv = reinterpret_cast<const uint4 *>((const T *)a.v + ((long)(t0 + tb + tok) * H + h) * DV + col0)[pos];
            if (lane < TB && tb + lane < len) {
                gb = ((const T *)a.beta)[(long)(t0 + tb + lane) * H + h];
                if (GATED) ga = __expf(a.g[(long)(t0 + tb + lane) * H + h]);
            }
        }
    };
    auto park = [&](unsigned char *buf) __attribute__((always_inline)) {
#pragma unroll
        for (int i = 0; i < ST::NKW; ++i) {
            constexpr int EPW = 16 / (int)sizeof(T); // elements per 16-byte word
            float fk[EPW], fq[EPW];
            RowRegs<T, EPW> wk, wq;
            wk.w[0] = gk[i]; wq.w[0] = gq[i];
            wk.unpack(fk); wq.unpack(fq);
            float *dk_ = reinterpret_cast<float *>(buf + ST::oK) + (i * 64 + lane) * EPW;
            float *dq_ = reinterpret_cast<float *>(buf + ST::oQ) + (i * 64 + lane) * EPW;
#pragma unroll
            for (int e = 0; e < EPW; e += 4) {
                *reinterpret_cast<float4 *>(dk_ + e) = make_float4(fk[e], fk[e + 1], fk[e + 2], fk[e + 3]);
                *reinterpret_cast<float4 *>(dq_ + e) = make_float4(fq[e], fq[e + 1], fq[e + 2], fq[e + 3]);
            }
        }
        if (lane < TB * ST::VROWW) reinterpret_cast<uint4 *>(buf + ST::oV)[lane] = gv;
        if (lane < TB) {
            reinterpret_cast<T *>(buf + ST::oB)[lane] = gb;
            if (GATED) reinterpret_cast<float *>(buf + ST::oG)[lane] = ga;
        }
    };

    T *op = (T *)a.o + ((long)t0 * H + h) * DV + col;
    const long sv = (long)H * DV;
    if (len > 0) { fetch(0); park(buf0); }
    if (len > TB) fetch(TB);
    for (int tb = 0; tb < len; tb += TB) {
        const unsigned char *cur = ((tb / TB) & 1) ? buf1 : buf0;
        const int nt = min(TB, len - tb);
        // Unrolled over the whole block so that the LDS reads and bf16 expansions of later tokens can
        // be scheduled under the dependent chain of earlier ones; tokens past the end of the sequence
        // leave the state alone (u = 0) and store nothing.
#pragma unroll
        for (int tt = 0; tt < TB; ++tt) {
            const bool live = tt < nt;
            RowRegs<float, R> kr, qr;
            kr.load(reinterpret_cast<const float *>(cur + ST::oK) + tt * DK + rb * R);
            qr.load(reinterpret_cast<const float *>(cur + ST::oQ) + tt * DK + rb * R);
            const float vt = rec_to_f32(reinterpret_cast<const T *>(cur + ST::oV)[tt * kRecCols + j]);
            const float bt = rec_to_f32(reinterpret_cast<const T *>(cur + ST::oB)[tt]);
            const float at = GATED ? reinterpret_cast<const float *>(cur + ST::oG)[tt] : 1.f;
            float kf[R], qf[R];
            kr.unpack(kf);
            qr.unpack(qf);
            float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f; // S_{t-1}^T k_t, this lane's quarter of the rows
#pragma unroll
            for (int r = 0; r < R; r += 4) {
                d0 = fmaf(S[r], kf[r], d0); d1 = fmaf(S[r + 1], kf[r + 1], d1);
                d2 = fmaf(S[r + 2], kf[r + 2], d2); d3 = fmaf(S[r + 3], kf[r + 3], d3);
            }
            const float u = live ? bt * (vt - at * rec_sum4((d0 + d1) + (d2 + d3))) : 0.f;
            const float keep = live ? at : 1.f; // S_t = alpha_t S_{t-1} + k_t u_t^T
            float o0 = 0.f, o1 = 0.f, o2 = 0.f, o3 = 0.f; // S_t^T q_t, read-out from the updated state
#pragma unroll
            for (int r = 0; r < R; r += 4) {
                if (GATED) { S[r] *= keep; S[r + 1] *= keep; S[r + 2] *= keep; S[r + 3] *= keep; }
                S[r] = fmaf(kf[r], u, S[r]); o0 = fmaf(S[r], qf[r], o0);
                S[r + 1] = fmaf(kf[r + 1], u, S[r + 1]); o1 = fmaf(S[r + 1], qf[r + 1], o1);
                S[r + 2] = fmaf(kf[r + 2], u, S[r + 2]); o2 = fmaf(S[r + 2], qf[r + 2], o2);
                S[r + 3] = fmaf(kf[r + 3], u, S[r + 3]); o3 = fmaf(S[r + 3], qf[r + 3], o3);
            }
            const float out = rec_sum4((o0 + o1) + (o2 + o3));
            if (rb == 0 && live) rec_store(op, out);
            op += sv;
        }
        if (tb + TB < len) { // the block fetched during this one goes to the other buffer; request the one after it
            park(((tb / TB) & 1) ? buf0 : buf1);
            if (tb + 2 * TB < len) fetch(tb + 2 * TB);
        }
    }
    if (a.ST) {
        float *dst = a.ST + ((long)chain * DK + rb * R) * DV + col;
#pragma unroll
        for (int r = 0; r < R; ++r) dst[(long)r * DV] = S[r];
    }
}

template <typename T, int DK> static int launch_rec(const RecArgs &a, hipStream_t stream) {
    const dim3 grid(a.N * a.H, (a.DV + 4 * kRecCols - 1) / (4 * kRecCols));
    constexpr int lds = 4 * 2 * RecStage<T, DK>::bytes; // four waves, two buffers each
    static_assert(lds <= 160 * 1024, "staging fits the LDS");
    // the launch's own status (an error some earlier, unrelated call left behind is neither reported nor cleared)
    void *args[] = {const_cast<RecArgs *>(&a)};
    const void *fn = a.g ? reinterpret_cast<const void *>(k_recurrent_fwd<T, DK, true>) : reinterpret_cast<const void *>(k_recurrent_fwd<T, DK, false>);
    if (const hipError_t e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds)) return (int)e;
    prof_begin("k_recurrent_fwd", stream);
    const hipError_t e = hipLaunchKernel(fn, grid, dim3(256), args, lds, stream);
    prof_end(stream);
    return (int)e;
}

// dtype: 0 = fp32, 1 = bf16.  Returns 0, a hipError_t (> 0), or -1 when (dtype, d_k) is not compiled.
int run_recurrent_fwd(int dtype, int d_k, const RecArgs &a, hipStream_t stream) {
    if (a.N == 0) return 0;
    if (dtype == 0) {
        if (d_k == 32) return launch_rec<float, 32>(a, stream);
        if (d_k == 64) return launch_rec<float, 64>(a, stream);
        if (d_k == 128) return launch_rec<float, 128>(a, stream);
        if (d_k == 256) return launch_rec<float, 256>(a, stream);
    } else {
        if (d_k == 32) return launch_rec<rbf16, 32>(a, stream);
        if (d_k == 64) return launch_rec<rbf16, 64>(a, stream);
        if (d_k == 128) return launch_rec<rbf16, 128>(a, stream);
        if (d_k == 256) return launch_rec<rbf16, 256>(a, stream);
    }
    return -1;
}

} // namespace dn
