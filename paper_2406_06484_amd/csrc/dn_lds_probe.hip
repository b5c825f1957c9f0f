// deltanet_lds_probe: a measurement aid.  Each probe kernel repeats ONE of the LDS access patterns the DeltaNet kernels
// are built from (the same helper, the same leading dimension, the same number of wavefronts), so that the LDS counters of
// a profiler run (bank-conflict cycles against active cycles) can be read per pattern instead of per kernel.
// Nothing of the method is computed here.
#include "../../include/deltanet.h"

#include "dn_device.hpp"

namespace dn {
namespace {

constexpr int kProbeThreads = 512, kProbeLdsBytes = 96 * 1024, kProbeGrid = 256;

// an offset of zero that the compiler cannot see through: it keeps the accesses inside the repeat loop
__device__ inline int opaque_zero(int it) {
    int z = it & 0;
    asm volatile("" : "+v"(z));
    return z;
}
template <typename V> __device__ inline void keep(const V &v) { asm volatile("" ::"v"(v)); }

// PATTERN (bf16 tiles; ld = leading dimension in elements):
//  0..3   contraction-contiguous operand fragments (frag_kc, one 16-byte read per lane), ld 136, 144, 72, 80
//  4, 5   contraction-strided operand fragments (frag_ks, two transposing 8-byte reads per lane), ld 144, 80
//  6, 7   accumulator tile to a row-major tile (acc_to_lds, 2-byte writes), ld 40 (the staging tile), 144
//  8, 9   accumulator tile to a transposed tile (acc_to_lds_t, 8-byte writes), ld 136, 72
//  10, 11 register tile to LDS (TileRegs::store, 16-byte writes): 64 x 128 by 512 threads at ld 144, by 256 threads at ld 136
//  12     16-byte row-segment reads of a 64 x 128 tile by 256 threads (copy_out), ld 136
//  13     16-byte reads of the staging tile (stage_flush), ld 40
//  14, 15 contraction-strided operand fragments at the leading dimensions the kernels do not use for them, ld 136, 72
//  16, 17 accumulator tile to a transposed tile at the leading dimensions the kernels do not use for it, ld 144, 80
template <int PATTERN> __global__ __launch_bounds__(kProbeThreads) void k_lds_probe(float *sink, int iters) {
    extern __shared__ __align__(16) unsigned char smem[];
    bf16 *s = reinterpret_cast<bf16 *>(smem);
    const int tid = threadIdx.x, wave = tid >> 6;
    for (int i = tid; i < kProbeLdsBytes / 2; i += kProbeThreads) s[i] = (bf16)(float)(i & 7);
    lds_barrier();
    f32x16 acc;
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = (float)(tid + i);
    TileRegs<bf16, 64, 128, kProbeThreads> wide;
    TileRegs<bf16, 64, 128, 256> half;
#pragma unroll
    for (int i = 0; i < TileRegs<bf16, 64, 128, kProbeThreads>::NIT; ++i) wide.v[i] = make_uint4(tid, i, 0, 1);
#pragma unroll
    for (int i = 0; i < TileRegs<bf16, 64, 128, 256>::NIT; ++i) half.v[i] = make_uint4(tid, i, 0, 1);
    constexpr int kLd[18] = {136, 144, 72, 80, 144, 80, 40, 144, 136, 72, 144, 136, 136, 40, 136, 72, 144, 80};
    constexpr int ld = kLd[PATTERN];
    for (int it = 0; it < iters; ++it) {
        bf16 *base = s + opaque_zero(it);
        if (PATTERN <= 3) { // the row block of this wave, the whole contraction length the tile has
            constexpr int klen = ld >= 128 ? 128 : 64;
#pragma unroll
            for (int k0 = 0; k0 < klen; k0 += 16) keep(__builtin_bit_cast(u32x4, frag_kc(base + 32 * (wave & 1) * ld, ld, k0)));
        } else if (PATTERN <= 5 || PATTERN == 14 || PATTERN == 15) {
            constexpr int ncol = ld >= 128 ? 128 : 64;
#pragma unroll
            for (int k0 = 0; k0 < 64; k0 += 16) keep(__builtin_bit_cast(u32x4, frag_ks(base + 32 * (wave % (ncol / 32)), ld, k0)));
        } else if (PATTERN == 6) {
            acc_to_lds<bf16>(base + wave * Stage<bf16>::ELEMS, ld, 0, 0, acc);
        } else if (PATTERN == 7) {
            acc_to_lds<bf16>(base, ld, 32 * (wave & 1), 32 * (wave >> 1), acc);
        } else if (PATTERN == 8 || PATTERN == 16) { // the transposed tile is [128][ld]: tile (row block of 64, column block of 128)
            acc_to_lds_t<bf16>(base, ld, 32 * (wave & 1), 32 * (wave >> 1), acc);
        } else if (PATTERN == 9 || PATTERN == 17) {
            acc_to_lds_t<bf16>(base, ld, 32 * (wave & 1), 32 * ((wave >> 1) & 1), acc);
        } else if (PATTERN == 10) {
            wide.store(base, ld);
        } else if (PATTERN == 11) {
            if (tid < 256) half.store(base, ld, tid);
        } else if (PATTERN == 12) {
            if (tid < 256) {
                constexpr int TPR = 128 / 8, RPI = 256 / TPR;
                const int tr = tid / TPR, tc = (tid % TPR) * 8;
#pragma unroll
                for (int r0 = 0; r0 < 64; r0 += RPI) keep(*reinterpret_cast<const u32x4 *>(base + (r0 + tr) * ld + tc));
            }
        } else {
            const bf16 *stage = base + wave * Stage<bf16>::ELEMS;
            const int lane = tid & 63;
#pragma unroll
            for (int j = 0; j < 32 * Stage<bf16>::SEGS / 64; ++j) {
                const int idx = j * 64 + lane, r = idx / Stage<bf16>::SEGS, sg = idx % Stage<bf16>::SEGS;
                keep(*reinterpret_cast<const u32x4 *>(stage + r * ld + sg * 8));
            }
        }
        wave_lds_fence();
    }
    if (sink && tid == 0 && iters < 0) sink[blockIdx.x] = acc[0]; // never taken: keeps `sink` an argument like any kernel's
}

template <int PATTERN> int launch_probe(float *sink, int iters, hipStream_t stream) {
    auto kernel = k_lds_probe<PATTERN>;
    if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, kProbeLdsBytes) != hipSuccess)
        return DN_ERR_LAUNCH;
    void *args[] = {&sink, &iters};
    return hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3(kProbeGrid), dim3(kProbeThreads), args, kProbeLdsBytes, stream) == hipSuccess
               ? DN_OK : DN_ERR_LAUNCH;
}

} // namespace
} // namespace dn

extern "C" int deltanet_lds_probe(int pattern, int iters, void *hip_stream) {
    if (iters < 0 || iters > (1 << 20)) return DN_ERR_SHAPE;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    switch (pattern) {
#define DN_PROBE_CASE(P) case P: return dn::launch_probe<P>(nullptr, iters, stream);
        DN_PROBE_CASE(0) DN_PROBE_CASE(1) DN_PROBE_CASE(2) DN_PROBE_CASE(3) DN_PROBE_CASE(4) DN_PROBE_CASE(5) DN_PROBE_CASE(6)
        DN_PROBE_CASE(7) DN_PROBE_CASE(8) DN_PROBE_CASE(9) DN_PROBE_CASE(10) DN_PROBE_CASE(11) DN_PROBE_CASE(12) DN_PROBE_CASE(13) DN_PROBE_CASE(14) DN_PROBE_CASE(15) DN_PROBE_CASE(16) DN_PROBE_CASE(17)
#undef DN_PROBE_CASE
    default: return DN_ERR_UNSUPPORTED;
    }
}
