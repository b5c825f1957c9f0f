// Host-side launch plan shared by the C ABI (dn_api.hip) and the per-dtype instantiation files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace dn {

struct Problem {
    int N, L, H;            // N sequences (dense: B sequences of L rows; packed: L = total rows)
    int chunks_ub;          // upper bound on the total number of chunks (grid size of per-chunk kernels)
    const int32_t *cu;      // packed: the bounded copy of the caller's cu_seqlens that k_chunk_offsets writes (workspace); else nullptr
    const int32_t *cu_user; // packed: the caller's device cu_seqlens, read by k_chunk_offsets only
    int32_t *coff;          // device chunk-offset prefix [N+1] inside the workspace (packed only), then the length order [N]
    hipStream_t stream;
    int device;             // the current device
    int num_cus;            // its compute units
    int save;               // forward: also leave X, Ut and the chunk-initial states in the workspace;
                            // backward: find them there instead of recomputing them
};

struct Ptrs {
    // user tensors (device)
    const void *q, *k, *v, *beta, *d_o;
    const float *S0, *dST;
    void *o, *dq, *dk, *dv;
    float *ST, *dbeta, *dS0;
    // workspace tiles, indexed by (global chunk * H + head)
    void *Tm, *Xm, *Ut, *dUt, *Sc, *dSc;
    int want_x; // backward: k_wy_prep also stores the inverse X for the chunk kernel
    // gated variant (all null for the plain delta rule): g = log decay per token and head (fp32, user
    // tensor), dg its gradient; workspace: gam = per chunk the running decay gamma_i and 1/gamma_i
    // ([tile][2][C] fp32)
    const float *g;
    float *dg, *gam;
    float *zg; // gated, head sizes that take the streaming chunk kernel: <dS_C, S_C> per (chunk, head), for the gate gradient
    // prologue variant: q and k hold the pre-activations of the feature map, beta the logits; dq, dk and
    // dbeta receive the gradients with respect to those; workspace: Qm, Km = q, k after the map (layout of q, k)
    int pro;
    void *Qm, *Km;
    // forward pass split over segments of the sequence (workspace): per segment the state written from zero, the
    // transition matrix, and the state the segment starts from, all fp32 [segment][H][d_k][d_v or d_k]
    float *Nseg, *Mseg, *Sin;
    // ... and of the backward pass: per segment the gradient the reverse scan produces from zero, and the gradient
    // with respect to the segment's end state
    float *Rseg, *dSout;
    int streamed;   // option: the backward pass takes the chunk kernel that streams S and dS' and rebuilds Ut, dUt (k_bwd_stream)
    int skip_ut;    // that kernel will run: the scans do not write Ut and dUt
    int unit_state; // set inside k_scan_state for its transition-matrix pass
};

// How many segments a dense forward pass over N sequences of length L is cut into (1 = not at all).  Few chains
// cannot fill the 256 CUs of the chip; segments are whole chunks, at least four of them, d_v = d_k (the transition
// matrix is scanned with the state kernels).  nv = workgroups per chain (d_v / columns per workgroup).
inline int segment_count(int N, int L, int H, int d_k, int d_v, int nv, bool packed, int chunk = 64) {
    if (packed || d_k != d_v || d_k > 128 || L <= 0) return 1;
    const long wgs = (long)N * H * nv;
    if (wgs > 64) return 1; // three scan passes over the segments instead of one: pays from a quarter of the chip down
    int G = 1;
    while (G < 16 && wgs * (2 * G) <= 256 && L % (2 * G * chunk) == 0 && L / (2 * G * chunk) >= 4) G *= 2;
    return G;
}
// The backward pass runs five scan passes over the segments where the uncut one runs two, so it is cut (into the
// same segments as the forward pass, whose transition matrices it may find in the workspace) only when its two
// scans would occupy a quarter of the chip or less.
inline int segment_count_bwd(int N, int L, int H, int d_k, int d_v, int nv, bool packed, int chunk = 64) {
    return (long)N * H * nv <= 32 ? segment_count(N, L, H, d_k, d_v, nv, packed, chunk) : 1;
}
// State columns per scan workgroup: 64 in bf16 up to d_k = 128, else 32 (what fits the LDS).  DN_VBLOCK_COLS (a build
// option, for the tiling study: 32 or 64) overrides the 64.
#ifndef DN_VBLOCK_COLS
#define DN_VBLOCK_COLS 64
#endif
inline int scan_vblock_cols(int elem_bytes, int d_k, int d_v) {
    const int want = (elem_bytes == 2 && d_k <= 128) ? DN_VBLOCK_COLS : 32;
    return d_v < want ? d_v : want;
}

// Optional per-kernel timing (see deltanet_profile_* in the C header): when enabled, every launch is
// bracketed by a pair of HIP events on the launch stream.  No-ops when disabled.
void prof_begin(const char *kernel_name, hipStream_t stream);
void prof_end(hipStream_t stream);

// 0 on success, else the hipError_t of the failing launch.  Defined once per (T, DK, DV).
template <typename T, int DK, int DV> int run_fwd(const Problem &pb, const Ptrs &p);
template <typename T, int DK, int DV> int run_bwd(const Problem &pb, const Ptrs &p);
// largest dynamic LDS any kernel of this instantiation needs
template <typename T, int DK, int DV> size_t max_lds_bytes();
template <typename T, int DK, int DV> size_t max_lds_fwd_bytes(); // prep and forward scan only

// The compiled (element type, d_k, d_v) instantiations: X(enum value of the C header, element type, d_k, d_v).
// (bf16_t names __bf16 where the list is expanded; d = 256: the chunk tiles of its backward pass are streamed, they do
// not fit the LDS)
#define DN_FOR_EACH_IMPL(X)                                                                        \
    X(DN_F32, float, 64, 64) X(DN_F32, float, 32, 64) X(DN_F32, float, 64, 32)                     \
    X(DN_BF16, bf16_t, 128, 128) X(DN_BF16, bf16_t, 64, 64) X(DN_BF16, bf16_t, 64, 128)            \
    X(DN_BF16, bf16_t, 128, 64) X(DN_BF16, bf16_t, 256, 256)

// Token-serial forward (dn_recurrent.hip).  dtype: 0 = fp32, 1 = bf16.  Returns 0, a hipError_t
// (> 0), or -1 when (dtype, d_k) has no compiled kernel.  d_v must be a multiple of 16.
struct RecArgs {
    const void *q, *k, *v, *beta;
    const float *S0;
    void *o;
    float *ST;
    const int32_t *cu; // device cu_seqlens or nullptr
    const float *g;    // gated variant: log decay per token and head, or nullptr
    int N, L, H, DV;
};
int run_recurrent_fwd(int dtype, int d_k, const RecArgs &a, hipStream_t stream);

} // namespace dn
