// C ABI of the DeltaNet library (declared in include/deltanet.h): validation, workspace layout,
// dispatch to the compiled (dtype, d_k, d_v) instantiation.  Host code only.
#include "../../include/deltanet.h"
#include "dn_host.hpp"

#include <string.h>

#include <atomic>
#include <mutex>
#include <string>
#include <vector>

namespace dn {
namespace {
struct ProfRec { std::string name; hipEvent_t a, b; };
std::atomic<int> g_opt_streamed{0}; // DN_OPT_STREAMED_CHUNK_KERNEL
std::mutex g_prof_mu;
std::atomic<bool> g_prof_on{false};
std::vector<ProfRec> g_prof;
} // namespace

void prof_begin(const char *kernel_name, hipStream_t stream) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    ProfRec r;
    r.name = kernel_name;
    if (hipEventCreate(&r.a) != hipSuccess) return;
    if (hipEventCreate(&r.b) != hipSuccess) { (void)hipEventDestroy(r.a); return; }
    (void)hipEventRecord(r.a, stream);
    g_prof.push_back(r);
}
void prof_end(hipStream_t stream) {
    if (!g_prof_on) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_prof.empty()) (void)hipEventRecord(g_prof.back().b, stream);
}
} // namespace dn

namespace {

using namespace dn;
typedef __bf16 bf16_t;

constexpr int kChunk = 64;

struct Plan {
    Problem pb;
    size_t off_coff, off_T, off_X, off_Ut, off_dUt, off_Sc, off_dSc, off_gam, off_zg, off_Qm, off_Km, off_seg, seg_bytes, total;
    size_t esz;
};

size_t up256(size_t x) { return (x + 255) & ~size_t(255); }

typedef int (*run_fn)(const Problem &, const Ptrs &);
struct Impl { int dtype, dk, dv; run_fn fwd, bwd; size_t (*lds)(); };

#define DN_IMPL(ENUM, T, DK, DV) { ENUM, DK, DV, &run_fwd<T, DK, DV>, &run_bwd<T, DK, DV>, &max_lds_bytes<T, DK, DV> },
const Impl kImpls[] = { DN_FOR_EACH_IMPL(DN_IMPL) };

const Impl *find_impl(const dn_shape *s) {
    for (const Impl &im : kImpls)
        if (im.dtype == s->dtype && im.dk == s->d_k && im.dv == s->d_v) return &im;
    return nullptr;
}

int validate_shape(const dn_shape *s, const Impl **impl, bool need_impl = true) {
    if (!s) return DN_ERR_NULL;
    if (s->B <= 0 || s->L < 0 || s->H <= 0 || s->d_k <= 0 || s->d_v <= 0) return DN_ERR_SHAPE;
    if (s->dtype != DN_F32 && s->dtype != DN_BF16) return DN_ERR_UNSUPPORTED;
    if (s->chunk != kChunk) return DN_ERR_UNSUPPORTED;
    if (s->cu_seqlens) {
        if (s->B != 1 || s->num_seqs < 0) return DN_ERR_SHAPE;
        if (s->cu_seqlens_host) {
            const int32_t *c = s->cu_seqlens_host;
            if (c[0] != 0 || c[s->num_seqs] != s->L) return DN_ERR_CUSEQLENS;
            for (int n = 0; n < s->num_seqs; ++n)
                if (c[n + 1] < c[n]) return DN_ERR_CUSEQLENS;
        }
    }
    // 32-bit row indices and grid limits
    const long long rows = (long long)s->B * s->L;
    // H also bounds the byte extent of one strided tile (128 rows of H * d elements), which must
    // stay inside the 1 GiB window of a buffer descriptor
    if (rows * s->H >= (1ll << 31) || s->H > 8192) return DN_ERR_SHAPE;
    const long long nseq = s->cu_seqlens ? s->num_seqs : s->B;
    if (nseq > 65535) return DN_ERR_SHAPE;
    if (!need_impl) return DN_OK;
    *impl = find_impl(s);
    return *impl ? DN_OK : DN_ERR_UNSUPPORTED;
}

void make_plan(const dn_shape *s, int want_bwd, Plan *pl, bool gated = false, bool prologue = false) {
    memset(pl, 0, sizeof(*pl));
    Problem &pb = pl->pb;
    const bool packed = s->cu_seqlens != nullptr;
    pb.N = packed ? s->num_seqs : s->B;
    pb.L = s->L;
    pb.H = s->H;
    pb.cu_user = s->cu_seqlens;
    const long long per = (s->L + kChunk - 1) / kChunk;
    pb.chunks_ub = packed ? (int)(s->L / kChunk + s->num_seqs) : (int)(per * s->B);
    if (packed && s->L == 0) pb.chunks_ub = 0;
    pl->esz = s->dtype == DN_BF16 ? 2 : 4;
    const size_t tiles = (size_t)pb.chunks_ub * s->H;
    const size_t tV = up256(tiles * kChunk * s->d_v * pl->esz);
    const size_t tS = up256(tiles * (size_t)s->d_k * s->d_v * pl->esz);
    size_t o = 0;
    // chunk offsets [N + 1], the length order [N], the bounded copy of cu_seqlens [N + 1]
    pl->off_coff = o; o += packed ? up256(sizeof(int32_t) * (3 * (size_t)pb.N + 2)) : 0;
    const size_t tC = up256(tiles * kChunk * kChunk * pl->esz);
    pl->off_T = o; o += tC; // T of Eq. 10
    if (want_bwd) {
        pl->off_X = o; o += tC; // (I + A)^-1 of Eq. 10, reused by the chunk kernel
        pl->off_Ut = o; o += tV;
        pl->off_dUt = o; o += tV;
        pl->off_Sc = o; o += tS;
        pl->off_dSc = o; o += tS;
    }
    if (gated) {
        pl->off_gam = o; o += up256(tiles * 2 * kChunk * sizeof(float)); // gamma_i and 1 / gamma_i per chunk row
        pl->off_zg = o; o += up256(tiles * sizeof(float)); // <dS_C, S_C> per chunk, where the gate gradient takes a second kernel
    }
    { // forward pass split over segments of the sequence: N, M and the start state per segment
        const int nv = s->d_v / scan_vblock_cols((int)pl->esz, s->d_k, s->d_v);
        const int G = segment_count(pb.N, s->L, s->H, s->d_k, s->d_v, nv, packed, kChunk);
        pl->seg_bytes = G > 1 ? up256((size_t)pb.N * G * s->H * s->d_k * s->d_v * sizeof(float)) : 0;
        pl->off_seg = o; o += 5 * pl->seg_bytes;
    }
    if (prologue) { // q and k after the feature map, in the layout of q and k
        const size_t tQ = up256((size_t)s->B * s->L * s->H * s->d_k * pl->esz);
        pl->off_Qm = o; o += tQ;
        pl->off_Km = o; o += tQ;
    }
    pl->total = o;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

void bind_workspace(const Plan &pl, void *ws, Ptrs *p, Problem *pb, bool want_bwd, bool gated = false, bool prologue = false) {
    unsigned char *b = static_cast<unsigned char *>(ws);
    pb->coff = pb->cu_user ? reinterpret_cast<int32_t *>(b + pl.off_coff) : nullptr;
    pb->cu = pb->cu_user ? pb->coff + 2 * (size_t)pb->N + 1 : nullptr;
    p->Tm = b + pl.off_T;
    p->want_x = want_bwd;
    if (want_bwd) {
        p->Xm = b + pl.off_X;
        p->Ut = b + pl.off_Ut; p->dUt = b + pl.off_dUt; p->Sc = b + pl.off_Sc;
        p->dSc = b + pl.off_dSc;
    }
    if (gated) {
        p->gam = reinterpret_cast<float *>(b + pl.off_gam);
        p->zg = reinterpret_cast<float *>(b + pl.off_zg);
    }
    if (prologue) {
        p->Qm = b + pl.off_Qm; p->Km = b + pl.off_Km;
    }
    if (pl.seg_bytes) {
        p->Nseg = reinterpret_cast<float *>(b + pl.off_seg);
        p->Mseg = reinterpret_cast<float *>(b + pl.off_seg + pl.seg_bytes);
        p->Sin = reinterpret_cast<float *>(b + pl.off_seg + 2 * pl.seg_bytes);
        p->Rseg = reinterpret_cast<float *>(b + pl.off_seg + 3 * pl.seg_bytes);
        p->dSout = reinterpret_cast<float *>(b + pl.off_seg + 4 * pl.seg_bytes);
    }
}

// LDS capacity and CU count of a device, asked for once per device
struct DevInfo { std::atomic<int> known{0}; int lds = 0, cus = 0; };
DevInfo g_dev[64];

int check_device(const Impl *impl, Problem *pb) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return DN_ERR_LAUNCH;
    DevInfo &di = g_dev[dev];
    if (!di.known.load(std::memory_order_acquire)) {
        int lds = 0, cus = 0;
        if (hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerBlock, dev) != hipSuccess) return DN_ERR_LAUNCH;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return DN_ERR_LAUNCH;
        di.lds = lds; di.cus = cus; // (two threads may both write the same values)
        di.known.store(1, std::memory_order_release);
    }
    pb->device = dev;
    pb->num_cus = di.cus;
    return (size_t)di.lds >= impl->lds() ? DN_OK : DN_ERR_UNSUPPORTED;
}

int fwd_impl(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta, const float *g,
             bool gated, const float *initial_state, void *o, float *final_state, void *workspace,
             size_t workspace_bytes, void *hip_stream, bool save = false, bool prologue = false) {
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl)) return rc;
    if (save && !impl->bwd) return DN_ERR_UNSUPPORTED;
    const bool no_rows = (long long)shape->B * shape->L == 0; // a tensor without rows may come with a null pointer
    if (!no_rows && (!q || !k || !v || !beta || !o || (gated && !g))) return DN_ERR_NULL;
    const void *al[] = {q, k, v, beta, g, initial_state, o, final_state, workspace, shape->cu_seqlens};
    for (const void *ptr : al) if (misaligned(ptr)) return DN_ERR_ALIGN;
    Plan pl;
    make_plan(shape, save, &pl, gated, prologue);
    if (pl.total && (!workspace || workspace_bytes < pl.total)) return DN_ERR_WORKSPACE;
    if (int rc = check_device(impl, &pl.pb)) return rc;
    Ptrs p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.k = k; p.v = v; p.beta = beta; p.g = gated ? g : nullptr; p.S0 = initial_state; p.o = o; p.ST = final_state;
    pl.pb.stream = static_cast<hipStream_t>(hip_stream);
    pl.pb.save = save;
    p.pro = prologue;
    p.streamed = dn::g_opt_streamed.load(std::memory_order_relaxed);
    bind_workspace(pl, workspace, &p, &pl.pb, save, gated, prologue);
    return impl->fwd(pl.pb, p) == 0 ? DN_OK : DN_ERR_LAUNCH;
}

int bwd_impl(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta, const float *g,
             bool gated, const float *initial_state, const void *d_o, const float *dfinal_state, void *dq, void *dk,
             void *dv, float *dbeta, float *dg, float *dinitial_state, void *workspace, size_t workspace_bytes,
             void *hip_stream, bool saved = false, bool prologue = false) {
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl)) return rc;
    if (!impl->bwd) return DN_ERR_UNSUPPORTED;
    const bool no_rows = (long long)shape->B * shape->L == 0; // a tensor without rows may come with a null pointer
    if (!no_rows && (!q || !k || !v || !beta || !d_o || !dq || !dk || !dv || !dbeta || (gated && (!g || !dg)))) return DN_ERR_NULL;
    const void *al[] = {q, k, v, beta, g, initial_state, d_o, dfinal_state, dq, dk, dv, dbeta, dg, dinitial_state,
                        workspace, shape->cu_seqlens};
    for (const void *ptr : al) if (misaligned(ptr)) return DN_ERR_ALIGN;
    Plan pl;
    make_plan(shape, 1, &pl, gated, prologue);
    if (pl.total && (!workspace || workspace_bytes < pl.total)) return DN_ERR_WORKSPACE;
    if (int rc = check_device(impl, &pl.pb)) return rc;
    Ptrs p;
    memset(&p, 0, sizeof(p));
    p.q = q; p.k = k; p.v = v; p.beta = beta; p.g = gated ? g : nullptr; p.S0 = initial_state; p.d_o = d_o; p.dST = dfinal_state;
    p.dq = dq; p.dk = dk; p.dv = dv; p.dbeta = dbeta; p.dg = gated ? dg : nullptr; p.dS0 = dinitial_state;
    pl.pb.stream = static_cast<hipStream_t>(hip_stream);
    pl.pb.save = saved;
    p.pro = prologue;
    p.streamed = dn::g_opt_streamed.load(std::memory_order_relaxed);
    bind_workspace(pl, workspace, &p, &pl.pb, true, gated, prologue);
    return impl->bwd(pl.pb, p) == 0 ? DN_OK : DN_ERR_LAUNCH;
}

} // namespace

extern "C" {

int deltanet_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes) {
    if (!out_bytes) return DN_ERR_NULL;
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl)) return rc;
    if (want_bwd && !impl->bwd) return DN_ERR_UNSUPPORTED;
    Plan pl;
    make_plan(shape, want_bwd, &pl);
    *out_bytes = pl.total;
    return DN_OK;
}

int deltanet_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                 const float *initial_state, void *o, float *final_state, void *workspace,
                 size_t workspace_bytes, void *hip_stream) {
    return fwd_impl(shape, q, k, v, beta, nullptr, false, initial_state, o, final_state, workspace, workspace_bytes, hip_stream);
}

int deltanet_bwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                 const float *initial_state, const void *d_o, const float *dfinal_state, void *dq,
                 void *dk, void *dv, float *dbeta, float *dinitial_state, void *workspace,
                 size_t workspace_bytes, void *hip_stream) {
    return bwd_impl(shape, q, k, v, beta, nullptr, false, initial_state, d_o, dfinal_state, dq, dk, dv, dbeta, nullptr,
                    dinitial_state, workspace, workspace_bytes, hip_stream);
}

int deltanet_fwd_save(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                      const float *initial_state, void *o, float *final_state, void *saved, size_t saved_bytes,
                      void *hip_stream) {
    return fwd_impl(shape, q, k, v, beta, nullptr, false, initial_state, o, final_state, saved, saved_bytes, hip_stream, true);
}

int deltanet_bwd_saved(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const void *d_o, const float *dfinal_state, void *dq, void *dk, void *dv, float *dbeta,
                       float *dinitial_state, void *saved, size_t saved_bytes, void *hip_stream) {
    return bwd_impl(shape, q, k, v, beta, nullptr, false, nullptr, d_o, dfinal_state, dq, dk, dv, dbeta, nullptr,
                    dinitial_state, saved, saved_bytes, hip_stream, true);
}

int deltanet_fused_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes) {
    if (!out_bytes) return DN_ERR_NULL;
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl)) return rc;
    if (want_bwd && !impl->bwd) return DN_ERR_UNSUPPORTED;
    Plan pl;
    make_plan(shape, want_bwd, &pl, false, true);
    *out_bytes = pl.total;
    return DN_OK;
}

int deltanet_fused_fwd(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v, const void *beta_logit,
                       const float *initial_state, void *o, float *final_state, void *workspace, size_t workspace_bytes,
                       void *hip_stream) {
    return fwd_impl(shape, q_pre, k_pre, v, beta_logit, nullptr, false, initial_state, o, final_state, workspace,
                    workspace_bytes, hip_stream, false, true);
}

int deltanet_fused_bwd(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v, const void *beta_logit,
                       const float *initial_state, const void *d_o, const float *dfinal_state, void *dq_pre, void *dk_pre,
                       void *dv, float *dbeta_logit, float *dinitial_state, void *workspace, size_t workspace_bytes,
                       void *hip_stream) {
    return bwd_impl(shape, q_pre, k_pre, v, beta_logit, nullptr, false, initial_state, d_o, dfinal_state, dq_pre, dk_pre, dv,
                    dbeta_logit, nullptr, dinitial_state, workspace, workspace_bytes, hip_stream, false, true);
}

int deltanet_fused_fwd_save(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v,
                            const void *beta_logit, const float *initial_state, void *o, float *final_state, void *saved,
                            size_t saved_bytes, void *hip_stream) {
    return fwd_impl(shape, q_pre, k_pre, v, beta_logit, nullptr, false, initial_state, o, final_state, saved, saved_bytes,
                    hip_stream, true, true);
}

int deltanet_fused_bwd_saved(const dn_shape *shape, const void *q_pre, const void *k_pre, const void *v,
                             const void *beta_logit, const void *d_o, const float *dfinal_state, void *dq_pre, void *dk_pre,
                             void *dv, float *dbeta_logit, float *dinitial_state, void *saved, size_t saved_bytes,
                             void *hip_stream) {
    return bwd_impl(shape, q_pre, k_pre, v, beta_logit, nullptr, false, nullptr, d_o, dfinal_state, dq_pre, dk_pre, dv,
                    dbeta_logit, nullptr, dinitial_state, saved, saved_bytes, hip_stream, true, true);
}

int deltanet_gated_workspace_bytes(const dn_shape *shape, int want_bwd, size_t *out_bytes) {
    if (!out_bytes) return DN_ERR_NULL;
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl)) return rc;
    if (want_bwd && !impl->bwd) return DN_ERR_UNSUPPORTED;
    Plan pl;
    make_plan(shape, want_bwd, &pl, true);
    *out_bytes = pl.total;
    return DN_OK;
}

int deltanet_gated_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const float *g, const float *initial_state, void *o, float *final_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream) {
    return fwd_impl(shape, q, k, v, beta, g, true, initial_state, o, final_state, workspace, workspace_bytes, hip_stream);
}

int deltanet_gated_bwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                       const float *g, const float *initial_state, const void *d_o, const float *dfinal_state,
                       void *dq, void *dk, void *dv, float *dbeta, float *dg, float *dinitial_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream) {
    return bwd_impl(shape, q, k, v, beta, g, true, initial_state, d_o, dfinal_state, dq, dk, dv, dbeta, dg, dinitial_state,
                    workspace, workspace_bytes, hip_stream);
}

int deltanet_gated_fwd_save(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                            const float *g, const float *initial_state, void *o, float *final_state, void *saved,
                            size_t saved_bytes, void *hip_stream) {
    return fwd_impl(shape, q, k, v, beta, g, true, initial_state, o, final_state, saved, saved_bytes, hip_stream, true);
}

int deltanet_gated_bwd_saved(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                             const float *g, const void *d_o, const float *dfinal_state, void *dq, void *dk, void *dv,
                             float *dbeta, float *dg, float *dinitial_state, void *saved, size_t saved_bytes,
                             void *hip_stream) {
    return bwd_impl(shape, q, k, v, beta, g, true, nullptr, d_o, dfinal_state, dq, dk, dv, dbeta, dg, dinitial_state,
                    saved, saved_bytes, hip_stream, true);
}

static int recurrent_impl(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                          const float *g, bool gated, const float *initial_state, void *o, float *final_state,
                          void *hip_stream) {
    const Impl *impl = nullptr;
    if (int rc = validate_shape(shape, &impl, false)) return rc;
    const bool no_rows = (long long)shape->B * shape->L == 0; // a tensor without rows may come with a null pointer
    if (!no_rows && (!q || !k || !v || !beta || !o || (gated && !g))) return DN_ERR_NULL;
    const void *al[] = {q, k, v, beta, g, initial_state, o, final_state, shape->cu_seqlens};
    for (const void *ptr : al) if (misaligned(ptr)) return DN_ERR_ALIGN;
    if (shape->d_v % 16 != 0) return DN_ERR_UNSUPPORTED;
    if (shape->d_k != 32 && shape->d_k != 64 && shape->d_k != 128 && shape->d_k != 256) return DN_ERR_UNSUPPORTED;
    RecArgs a;
    a.q = q; a.k = k; a.v = v; a.beta = beta; a.S0 = initial_state; a.o = o; a.ST = final_state;
    a.cu = shape->cu_seqlens;
    a.g = gated ? g : nullptr;
    a.N = shape->cu_seqlens ? shape->num_seqs : shape->B;
    a.L = shape->L; a.H = shape->H; a.DV = shape->d_v;
    const int rc = run_recurrent_fwd(shape->dtype == DN_BF16 ? 1 : 0, shape->d_k, a, static_cast<hipStream_t>(hip_stream));
    return rc == 0 ? DN_OK : (rc < 0 ? DN_ERR_UNSUPPORTED : DN_ERR_LAUNCH);
}

int deltanet_recurrent_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                           const float *initial_state, void *o, float *final_state, void *hip_stream) {
    return recurrent_impl(shape, q, k, v, beta, nullptr, false, initial_state, o, final_state, hip_stream);
}

int deltanet_gated_recurrent_fwd(const dn_shape *shape, const void *q, const void *k, const void *v, const void *beta,
                                 const float *g, const float *initial_state, void *o, float *final_state,
                                 void *hip_stream) {
    return recurrent_impl(shape, q, k, v, beta, g, true, initial_state, o, final_state, hip_stream);
}

int deltanet_set_option(int option, int value) {
    if (option != DN_OPT_STREAMED_CHUNK_KERNEL) return DN_ERR_UNSUPPORTED;
    dn::g_opt_streamed.store(value != 0, std::memory_order_relaxed);
    return DN_OK;
}

int deltanet_profile_enable(int on) {
    std::lock_guard<std::mutex> lk(dn::g_prof_mu);
    dn::g_prof_on.store(on != 0);
    return DN_OK;
}

int deltanet_profile_collect(dn_kernel_time *out, int max_entries, int *num_entries) {
    if (!num_entries || (max_entries > 0 && !out)) return DN_ERR_NULL;
    std::lock_guard<std::mutex> lk(dn::g_prof_mu);
    int n = 0;
    int rc = DN_OK;
    for (dn::ProfRec &r : dn::g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) rc = DN_ERR_LAUNCH;
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
        int i = 0;
        for (; i < n; ++i) if (r.name == out[i].name) break;
        if (i == n) {
            if (n == max_entries) continue;
            memset(&out[n], 0, sizeof(out[n]));
            strncpy(out[n].name, r.name.c_str(), sizeof(out[n].name) - 1);
            ++n;
        }
        out[i].total_ms += ms;
        out[i].launches += 1;
    }
    dn::g_prof.clear();
    *num_entries = n;
    return rc;
}

const char *deltanet_status_string(int status) {
    switch (status) {
    case DN_OK: return "ok";
    case DN_ERR_NULL: return "a required pointer is NULL";
    case DN_ERR_SHAPE: return "a size is non-positive, inconsistent or too large";
    case DN_ERR_UNSUPPORTED: return "no compiled kernel for this (dtype, d_k, d_v, chunk), or the device lacks the LDS it needs";
    case DN_ERR_ALIGN: return "a data pointer is not 16-byte aligned";
    case DN_ERR_WORKSPACE: return "workspace is NULL or too small";
    case DN_ERR_CUSEQLENS: return "cu_seqlens_host is not a non-decreasing sequence from 0 to L";
    case DN_ERR_LAUNCH: return "the HIP runtime reported an error";
    default: return "unknown status";
    }
}

} // extern "C"
