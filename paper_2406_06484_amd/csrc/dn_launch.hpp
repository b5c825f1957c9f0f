// Launch sequences of the forward and backward pass for one (T, DK, DV); included only by the
// instantiation files.
#pragma once
#include <atomic>
#include <tuple>

#include "dn_host.hpp"
#include "dn_kernels.hpp"
#include "dn_chunk_wide.hpp"
#include "dn_chunk_stream.hpp"

namespace dn {

constexpr size_t kLdsPerWorkgroup = 160 * 1024; // gfx950

// Raises the dynamic-LDS limit of `kernel` once per device and call site (every call site names one kernel
// instantiation), then launches it; returns the launch's own status, so an error some earlier, unrelated call left
// behind is neither reported as this launch's nor cleared.
template <typename... Params, typename... Args>
static inline int launch_kernel(void (*kernel)(Params...), std::atomic<uint64_t> &lds_set, int device, dim3 grid, int nthreads,
                                size_t lds, hipStream_t stream, Args... args) {
    const uint64_t bit = 1ull << (device & 63);
    if (lds > 0 && !(lds_set.load(std::memory_order_relaxed) & bit)) { // (a call site always asks for the same amount)
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return (int)e;
        lds_set.fetch_or(bit, std::memory_order_relaxed);
    }
    std::tuple<Params...> held(static_cast<Params>(args)...); // the kernel's own parameter types, by value
    void *ptrs[sizeof...(Params)];
    int i = 0;
    std::apply([&](auto &...a) { ((ptrs[i++] = (void *)&a), ...); }, held);
    return (int)hipLaunchKernel(reinterpret_cast<const void *>(kernel), grid, dim3(nthreads), ptrs, lds, stream);
}

#define DN_LAUNCH(kernel, grid, lds, ...) DN_LAUNCH_NT(kernel, grid, NTHR, lds, __VA_ARGS__)
#define DN_LAUNCH_NT(kernel, grid, nthreads, lds, ...)                                                        \
    do {                                                                                                      \
        static std::atomic<uint64_t> lds_set_{0};                                                             \
        prof_begin(#kernel, pb.stream);                                                                       \
        const int e_ = launch_kernel(kernel, lds_set_, pb.device, grid, nthreads, lds, pb.stream, __VA_ARGS__); \
        prof_end(pb.stream);                                                                                  \
        if (e_) return e_;                                                                                    \
    } while (0)

static inline SeqMap make_map(const Problem &pb) {
    SeqMap sm;
    sm.cu = pb.cu; sm.coff = pb.coff; sm.N = pb.N; sm.L = pb.L; sm.ncd = (pb.L + C - 1) / C;
    sm.order = pb.cu ? pb.coff + pb.N + 1 : nullptr;
    // (pb.cu is the bounded copy of the caller's offsets that k_chunk_offsets leaves behind the order)
    return sm;
}

static inline int launch_offsets(const Problem &pb) {
    if (!pb.cu) return 0;
    DN_LAUNCH(k_chunk_offsets, dim3(1), 0, pb.cu_user, pb.N, pb.L, pb.coff);
    return 0;
}

// Head sizes whose chunk operands do not fit the LDS at once take the streaming chunk kernel.
template <typename T, int DK, int DV> constexpr bool kChunkFits = ChunkSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup;
template <typename T, int DK, int DV> constexpr bool kWideBwd = !kChunkFits<T, DK, DV> && sizeof(T) == 2 && DK % 128 == 0 && DV % 64 == 0;
// The plain delta rule in bf16 at head sizes whose resident tiles fit can take the chunk kernel that rebuilds Ut and dUt
// from the streamed blocks of S and dS' (k_bwd_stream; option DN_OPT_STREAMED_CHUNK_KERNEL); the scans then skip those two stores.
template <typename T, int DK, int DV> constexpr bool stream_fits() {
    if constexpr (sizeof(T) == 2 && DK % 64 == 0 && DV % 64 == 0 && DK <= 128 && DV <= 128) return StreamSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup;
    else return false;
}
template <typename T, int DK, int DV> constexpr bool kStreamBwd = stream_fits<T, DK, DV>();
static inline bool use_stream_kernel(bool compiled, const Ptrs &p) { return compiled && p.streamed && !p.g && !p.pro; }
// whether the backward pass is compiled for this head size
template <typename T, int DK, int DV> constexpr bool kHasBwd = kChunkFits<T, DK, DV> || kWideBwd<T, DK, DV>;

template <typename T, int DK, int DV> size_t max_lds_bytes() {
    static_assert(PrepSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_wy_prep LDS");
    static_assert(ScanFwdSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_scan_fwd LDS");
    static_assert(ScanBwdSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_scan_bwd LDS");
    size_t m = PrepSmem<T, DK, DV>::bytes;
    if (ScanFwdSmem<T, DK, DV>::bytes > m) m = ScanFwdSmem<T, DK, DV>::bytes;
    if (ScanBwdSmem<T, DK, DV>::bytes > m) m = ScanBwdSmem<T, DK, DV>::bytes;
    if constexpr (kStreamBwd<T, DK, DV>)
        if (StreamSmem<T, DK, DV>::bytes > m) m = StreamSmem<T, DK, DV>::bytes;
    if constexpr (kChunkFits<T, DK, DV>) {
        if (ChunkSmem<T, DK, DV>::bytes > m) m = ChunkSmem<T, DK, DV>::bytes;
    } else {
        static_assert(WideSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_bwd_chunk_wide LDS");
        if (WideSmem<T, DK, DV>::bytes > m) m = WideSmem<T, DK, DV>::bytes;
    }
    return m;
}

// forward-only instantiations (head sizes whose backward tiles do not fit)
template <typename T, int DK, int DV> size_t max_lds_fwd_bytes() {
    static_assert(PrepSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_wy_prep LDS");
    static_assert(ScanFwdSmem<T, DK, DV>::bytes <= kLdsPerWorkgroup, "k_scan_fwd LDS");
    return PrepSmem<T, DK, DV>::bytes > ScanFwdSmem<T, DK, DV>::bytes ? PrepSmem<T, DK, DV>::bytes : ScanFwdSmem<T, DK, DV>::bytes;
}

// launches kernel<T, DK, DV, variant> for the variant the pointers ask for.  The scans know two variants
// (for the prologue they run the plain one on the q, k that k_wy_prep mapped), the chunk kernel three.
#define DN_LAUNCH_SCAN(kernel, grid, nthreads, lds, ...)                                                    \
    do {                                                                                                    \
        if (p.g) DN_LAUNCH_NT((kernel<T, DK, DV, VAR_GATED>), grid, nthreads, lds, __VA_ARGS__);            \
        else DN_LAUNCH_NT((kernel<T, DK, DV, VAR_PLAIN>), grid, nthreads, lds, __VA_ARGS__);                \
    } while (0)
#define DN_LAUNCH_VAR(kernel, grid, nthreads, lds, ...)                                                     \
    do {                                                                                                    \
        if (p.g) DN_LAUNCH_NT((kernel<T, DK, DV, VAR_GATED>), grid, nthreads, lds, __VA_ARGS__);            \
        else if (p.pro) DN_LAUNCH_NT((kernel<T, DK, DV, VAR_PROLOGUE>), grid, nthreads, lds, __VA_ARGS__);  \
        else DN_LAUNCH_NT((kernel<T, DK, DV, VAR_PLAIN>), grid, nthreads, lds, __VA_ARGS__);                \
    } while (0)

// what the scans see: with the prologue, the mapped q and k in the workspace
static inline Ptrs scan_ptrs(const Ptrs &p, bool stream_compiled) {
    Ptrs ps = p;
    ps.skip_ut = use_stream_kernel(stream_compiled, p);
    if (p.pro) { ps.q = p.Qm; ps.k = p.Km; ps.pro = 0; }
    return ps;
}

template <typename T, int DK, int DV> int run_fwd(const Problem &pb, const Ptrs &p) {
    if (pb.N == 0) return 0;
    if (pb.chunks_ub == 0) { // no tokens at all: the state passes through (section 2.2: nothing is written)
        if (p.ST) {
            const long count = (long)pb.N * pb.H * DK * DV;
            DN_LAUNCH(k_state_copy, dim3((unsigned)((count + 4 * NTHR - 1) / (4 * NTHR))), 0, p.ST, p.S0, count);
        }
        return 0;
    }
    SeqMap sm = make_map(pb);
    if (int e = launch_offsets(pb)) return e;
    const dim3 gchunk(pb.chunks_ub, pb.H);
    dim3 gchain(chain_grid(pb.N * pb.H, VBlock<T, DV, DK>::NV));
    DN_LAUNCH((k_wy_prep<T, DK, DV>), gchunk, (PrepSmem<T, DK, DV>::bytes), sm, pb.H, p);
    Ptrs ps = scan_ptrs(p, kStreamBwd<T, DK, DV>);
    if constexpr (DK == DV && DK <= 128) {
        // few long chains: cut the sequences into G segments, get every segment's start state from a first pass
        // (k_scan_state, k_seg_combine), then run the scan below over the segments side by side
        const int G = segment_count(pb.N, pb.L, pb.H, DK, DV, VBlock<T, DV, DK>::NV, pb.cu != nullptr);
        if (G > 1 && p.Sin) {
            sm.N = pb.N * G; sm.L = pb.L / G; sm.ncd = sm.L / C;
            const dim3 gseg(chain_grid(sm.N * pb.H, VBlock<T, DV, DK>::NV));
            const dim3 gstate(2 * gseg.x);
            DN_LAUNCH_SCAN(k_scan_state, gstate, NTS, (ScanFwdSmem<T, DK, DV>::bytes), sm, pb.H, ps, (int)gseg.x);
            const CombineArgs ca{p.Mseg, p.Nseg, p.S0, p.Sin, p.ST, nullptr, nullptr, nullptr, nullptr, G, pb.H, 0};
            DN_LAUNCH_NT((k_seg_combine<DK, DV>), dim3(pb.N * pb.H, DV / 32, 1), NTHR, (CombineSmem<DK, DV>::bytes), ca);
            ps.S0 = p.Sin; ps.ST = nullptr;
            gchain = gseg;
        }
    }
    if constexpr (kHasBwd<T, DK, DV>) {
        if (pb.save) {
            DN_LAUNCH_SCAN(k_scan_fwd_save, gchain, NTS, (ScanFwdSmem<T, DK, DV>::bytes), sm, pb.H, ps);
            return 0;
        }
    }
    DN_LAUNCH_SCAN(k_scan_fwd, gchain, NTS, (ScanFwdSmem<T, DK, DV>::bytes), sm, pb.H, ps);
    return 0;
}

template <typename T, int DK, int DV> int run_bwd(const Problem &pb, const Ptrs &p) {
    if (pb.N == 0) return 0;
    const SeqMap sm = make_map(pb);
    if (int e = launch_offsets(pb)) return e;
    const dim3 gchunk(pb.chunks_ub, pb.H), gchain(chain_grid(pb.N * pb.H, VBlock<T, DV, DK>::NV));
    Ptrs ps = scan_ptrs(p, kStreamBwd<T, DK, DV>);
    constexpr size_t lds_pair = cmax(ScanFwdSmem<T, DK, DV>::bytes, ScanBwdSmem<T, DK, DV>::bytes);
    // few long chains: the scans run over G segments of the sequences side by side (see k_scan_state)
    int G = 1;
    if constexpr (DK == DV && DK <= 128) G = segment_count_bwd(pb.N, pb.L, pb.H, DK, DV, VBlock<T, DV, DK>::NV, pb.cu != nullptr);
    if (G > 1 && p.Sin && pb.chunks_ub) {
        if constexpr (DK == DV && DK <= 128) {
            SeqMap sg = sm;
            sg.N = pb.N * G; sg.L = pb.L / G; sg.ncd = sg.L / C;
            const dim3 gseg(chain_grid(sg.N * pb.H, VBlock<T, DV, DK>::NV));
            if (pb.save) { // the forward pass left its tiles and the segments' transition matrices
                DN_LAUNCH_SCAN(k_scan_bwd_state, gseg, NTS, (ScanBwdSmem<T, DK, DV>::bytes), sg, pb.H, ps);
                const CombineArgs ca{p.Mseg, nullptr, nullptr, nullptr, nullptr, p.Rseg, p.dST, p.dSout, p.dS0, G, pb.H, 1};
                DN_LAUNCH_NT((k_seg_combine<DK, DV>), dim3(pb.N * pb.H, DV / 32, 1), NTHR, (CombineSmem<DK, DV>::bytes), ca);
                ps.dST = p.dSout; ps.dS0 = nullptr;
                DN_LAUNCH_SCAN(k_scan_bwd, gseg, NTS, (ScanBwdSmem<T, DK, DV>::bytes), sg, pb.H, ps);
            } else {
                DN_LAUNCH((k_wy_prep<T, DK, DV>), gchunk, (PrepSmem<T, DK, DV>::bytes), sm, pb.H, p);
                DN_LAUNCH_SCAN(k_scan_state, dim3(3 * gseg.x), NTS, lds_pair, sg, pb.H, ps, (int)gseg.x);
                const CombineArgs ca{p.Mseg, p.Nseg, p.S0, p.Sin, nullptr, p.Rseg, p.dST, p.dSout, p.dS0, G, pb.H, 0};
                DN_LAUNCH_NT((k_seg_combine<DK, DV>), dim3(pb.N * pb.H, DV / 32, 2), NTHR, (CombineSmem<DK, DV>::bytes), ca);
                ps.S0 = p.Sin; ps.dST = p.dSout; ps.dS0 = nullptr;
                DN_LAUNCH_SCAN(k_scan_pair, dim3(2 * gseg.x), NTS, lds_pair, sg, pb.H, ps, (int)gseg.x);
            }
        }
    } else if (pb.save) { // T, X, Ut and the chunk-initial states are the forward pass's: only the reverse scan is left
        DN_LAUNCH_SCAN(k_scan_bwd, gchain, NTS, (ScanBwdSmem<T, DK, DV>::bytes), sm, pb.H, ps);
    } else {
        if (pb.chunks_ub) DN_LAUNCH((k_wy_prep<T, DK, DV>), gchunk, (PrepSmem<T, DK, DV>::bytes), sm, pb.H, p);
        // both scans of the backward pass as one grid: reverse scan first, recompute scan behind it
        const dim3 gpair(2 * gchain.x);
        DN_LAUNCH_SCAN(k_scan_pair, gpair, NTS, lds_pair, sm, pb.H, ps, (int)gchain.x);
    }
    if (pb.chunks_ub) {
        const long tiles = (long)pb.chunks_ub * pb.H;
        const dim3 gpers((unsigned)(tiles < pb.num_cus ? tiles : pb.num_cus)); // one persistent workgroup per CU
        if constexpr (kWideBwd<T, DK, DV>) {
            if (p.pro) { // on the mapped q, k; then dq and dk go back through the feature map, in place
                DN_LAUNCH_NT((k_bwd_chunk_wide<T, DK, DV, VAR_PROLOGUE>), gpers, NTC, (WideSmem<T, DK, DV>::bytes), sm, pb.H, ps, pb.chunks_ub);
                const long rows = (long)(pb.cu ? pb.L : (long)pb.N * pb.L) * pb.H;
                const dim3 grows((unsigned)((rows + C - 1) / C));
                constexpr size_t lds_map = sizeof(T) * C * ldn<T>(DK);
                DN_LAUNCH((k_feature_map_bwd<T, DK>), grows, lds_map, (const T *)p.q, (T *)p.dq, rows);
                DN_LAUNCH((k_feature_map_bwd<T, DK>), grows, lds_map, (const T *)p.k, (T *)p.dk, rows);
            } else if (p.g) { // the kernel leaves <dS_C, S_C> per chunk; the per-token terms of the gate gradient follow
                DN_LAUNCH_NT((k_bwd_chunk_wide<T, DK, DV, VAR_GATED>), gpers, NTC, (WideSmem<T, DK, DV>::bytes), sm, pb.H, p, pb.chunks_ub);
                DN_LAUNCH((k_gate_grad<T, DK, DV>), gchunk, 0, sm, pb.H, p);
            } else {
                DN_LAUNCH_NT((k_bwd_chunk_wide<T, DK, DV, VAR_PLAIN>), gpers, NTC, (WideSmem<T, DK, DV>::bytes), sm, pb.H, p, pb.chunks_ub);
            }
        } else {
            if constexpr (kStreamBwd<T, DK, DV>) {
                if (use_stream_kernel(true, p)) {
                    DN_LAUNCH_NT((k_bwd_stream<T, DK, DV>), gpers, NTC, (StreamSmem<T, DK, DV>::bytes), sm, pb.H, p, pb.chunks_ub);
                    return 0;
                }
            }
            DN_LAUNCH_VAR(k_bwd_chunk, gpers, NTC, (ChunkSmem<T, DK, DV>::bytes), sm, pb.H, p, pb.chunks_ub);
        }
    }
    return 0;
}

#define DN_INSTANTIATE_FWD(T, DK, DV)                                    \
    template int run_fwd<T, DK, DV>(const Problem &, const Ptrs &);      \
    template size_t max_lds_fwd_bytes<T, DK, DV>();
#define DN_INSTANTIATE(T, DK, DV)                                        \
    template int run_fwd<T, DK, DV>(const Problem &, const Ptrs &);      \
    template int run_bwd<T, DK, DV>(const Problem &, const Ptrs &);      \
    template size_t max_lds_bytes<T, DK, DV>();

} // namespace dn
