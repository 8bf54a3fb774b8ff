// C-ABI boundary of libosdn: argument validation, workspace carving, kernel launches.
// See include/osdn.h for the contract of every entry point.
#include "../../include/osdn.h"
#include "osdn_kernels.h"

#include <cmath>
#include <vector>

namespace {

using namespace osdn;

// Optional per-kernel timing with HIP events on the caller's stream (off by default; the
// only process-wide state the library has).  Not thread-safe; meant for benchmarks.
enum { KID_PRECOND_FWD, KID_CHUNK_PREP, KID_STATE_FWD, KID_OUTPUT_FWD, KID_BWD_LOCAL, KID_BWD_CHAIN,
       KID_BWD_POST, KID_PRECOND_MASK, KID_PRECOND_CHAIN, KID_PRECOND_POST, KID_COUNT };
const char *const kKernelNames[KID_COUNT] = {"precond_fwd", "chunk_prep", "state_fwd", "output_fwd",
                                             "bwd_local", "bwd_chain", "bwd_post", "precond_mask",
                                             "precond_chain", "precond_post"};
struct Timed { int id; hipEvent_t e0, e1; };
bool g_prof_on = false;
std::vector<Timed> g_prof;

template <typename F> int timed(int id, hipStream_t st, F &&launch) {
    if (!g_prof_on) return launch();
    Timed t{id, nullptr, nullptr};
    if (hipEventCreate(&t.e0) != hipSuccess || hipEventCreate(&t.e1) != hipSuccess) return launch();
    (void)hipEventRecord(t.e0, st);
    const int rc = launch();
    (void)hipEventRecord(t.e1, st);
    g_prof.push_back(t);
    return rc;
}

struct Layout {
    size_t kt, d_ckpt, tok_scalars, Tm, W, Wt, Ktr, Ut, Et, S_ckpt;   // forward
    size_t dElt, Qt, dOt, dEt, dS_ckpt, dk_read, dkt, masks, a_ckpt;   // backward only
    size_t total_fwd, total_bwd;
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

int check_params(const osdn_params *p, bool need_chunks) {
    if (!p) return OSDN_ERR_NULL;
    if (p->io_dtype != OSDN_F32 && p->io_dtype != OSDN_BF16) return OSDN_ERR_DTYPE;
    if (p->B < 1 || p->T < 1 || p->H < 1 || p->chunk != C) return OSDN_ERR_SHAPE;
    if (p->K != 64 && p->K != 128) return OSDN_ERR_SHAPE;
    if (need_chunks) {
        if (p->T % C != 0) return OSDN_ERR_SHAPE;
        if (p->V < 64 || p->V > 512 || p->V % 64 != 0) return OSDN_ERR_SHAPE;
        if (p->B > 65535 || p->H > 65535) return OSDN_ERR_SHAPE;
    }
    if ((long long)p->B * p->H > 0x7fffffffLL / 64) return OSDN_ERR_SHAPE;
    if (!(p->eta >= 0.f) || !(p->eps > 0.f) || !std::isfinite(p->eta) || !std::isfinite(p->eps) ||
        !std::isfinite(p->scale) || std::isnan(p->d_min) || std::isnan(p->d_max))
        return OSDN_ERR_PARAM;
    return OSDN_OK;
}

Layout make_layout(const osdn_params *p) {
    const size_t es = p->io_dtype == OSDN_BF16 ? 2 : 4;
    const size_t B = p->B, T = p->T, H = p->H, K = p->K, V = p->V, N = T / C;
    Layout L;
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    L.kt = take(B * T * H * K * es);
    L.d_ckpt = take(B * H * N * K * 4);
    L.tok_scalars = take(B * T * H * 4 * 4);
    L.Tm = take(B * H * N * C * C * es);
    L.W = take(B * T * H * K * es);
    L.Wt = take(B * T * H * K * es);
    L.Ktr = take(B * T * H * K * es);
    L.Ut = take(B * T * H * V * es);
    L.Et = take(B * T * H * V * es);
    L.S_ckpt = take(B * H * N * V * K * es);
    L.total_fwd = off;
    L.dElt = take(B * T * H * V * es);
    L.Qt = take(B * T * H * K * es);
    L.dOt = take(B * T * H * V * es);
    L.dEt = take(B * T * H * V * es);
    L.dS_ckpt = take(B * H * N * V * K * es);
    L.dk_read = take(B * T * H * K * 4);
    L.dkt = take(B * T * H * K * 4);
    L.masks = take(B * H * N * K * 8);
    L.a_ckpt = take(B * H * N * K * 4);
    L.total_bwd = off;
    return L;
}

int check_ws(const void *ws, size_t bytes, size_t need) {
    if (!ws) return OSDN_ERR_NULL;
    if ((reinterpret_cast<uintptr_t>(ws) & 255) != 0 || bytes < need) return OSDN_ERR_WORKSPACE;
    return OSDN_OK;
}

int launch_status() { return hipGetLastError() == hipSuccess ? OSDN_OK : OSDN_ERR_LAUNCH; }

PrecondArgs precond_args(const osdn_params *p) {
    PrecondArgs a{};
    a.B = p->B; a.T = p->T; a.H = p->H; a.K = p->K;
    a.eta = p->eta; a.d_min = p->d_min; a.d_max = p->d_max; a.eps = p->eps;
    a.beta_aware = p->beta_aware;
    return a;
}

ChunkArgs chunk_args(const osdn_params *p, const Layout &L, char *ws) {
    ChunkArgs c{};
    c.B = p->B; c.T = p->T; c.H = p->H; c.K = p->K; c.V = p->V; c.N = p->T / C;
    c.scale = p->scale;
    c.kt = ws + L.kt; c.Tm = ws + L.Tm; c.W = ws + L.W; c.Wt = ws + L.Wt; c.Ktr = ws + L.Ktr;
    c.Ut = ws + L.Ut; c.Et = ws + L.Et;
    c.S_ckpt = ws + L.S_ckpt;
    return c;
}

}  // namespace

extern "C" {

size_t osdn_workspace_bytes(const osdn_params *p, int for_backward) {
    if (check_params(p, true) != OSDN_OK) return 0;
    Layout L = make_layout(p);
    return for_backward ? L.total_bwd : L.total_fwd;
}

const char *osdn_strerror(int status) {
    switch (status) {
        case OSDN_OK: return "ok";
        case OSDN_ERR_NULL: return "a required pointer is NULL";
        case OSDN_ERR_SHAPE: return "unsupported shape (chunk must be 64, T % 64 == 0, K in {64,128}, V % 64 == 0, V <= 512)";
        case OSDN_ERR_DTYPE: return "io_dtype must be OSDN_F32 or OSDN_BF16";
        case OSDN_ERR_WORKSPACE: return "workspace too small or not 256-byte aligned";
        case OSDN_ERR_PARAM: return "invalid scalar parameter (eta < 0, eps <= 0 or non-finite)";
        case OSDN_ERR_LAUNCH: return "HIP launch error";
        default: return "unknown status";
    }
}

int osdn_precond_update(const osdn_params *p, const void *k, const float *beta,
                        const float *retention, const float *d_in, void *k_tilde, float *d_out,
                        float *d_ckpt, void *stream) {
    int rc = check_params(p, false);
    if (rc != OSDN_OK) return rc;
    if (!k || !beta || !k_tilde || !d_out) return OSDN_ERR_NULL;
    if (d_ckpt && p->T % C != 0) return OSDN_ERR_SHAPE;
    PrecondArgs a = precond_args(p);
    a.k = k; a.beta = beta; a.retention = retention; a.d_in = d_in;
    a.k_tilde = k_tilde; a.d_out = d_out; a.d_ckpt = d_ckpt; a.tok_scalars = nullptr;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;
    if (timed(KID_PRECOND_FWD, st, [&] { return launch_precond_fwd(a, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    return launch_status();
}

int osdn_fwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             void *o, float *S_out, float *d_out, void *workspace, size_t workspace_bytes,
             void *stream) {
    int rc = check_params(p, true);
    if (rc != OSDN_OK) return rc;
    if (!q || !k || !v || !beta || !o || !S_out || !d_out) return OSDN_ERR_NULL;
    Layout L = make_layout(p);
    rc = check_ws(workspace, workspace_bytes, L.total_fwd);
    if (rc != OSDN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;

    PrecondArgs pa = precond_args(p);
    pa.k = k; pa.beta = beta; pa.retention = retention; pa.d_in = d_in;
    pa.k_tilde = ws + L.kt; pa.d_out = d_out; pa.d_ckpt = reinterpret_cast<float *>(ws + L.d_ckpt);
    pa.tok_scalars = reinterpret_cast<float *>(ws + L.tok_scalars);
    if (timed(KID_PRECOND_FWD, st, [&] { return launch_precond_fwd(pa, bf, st); }) != 0) return OSDN_ERR_SHAPE;

    ChunkArgs c = chunk_args(p, L, ws);
    c.q = q; c.k = k; c.v = v; c.beta = beta; c.log_alpha = log_alpha; c.S_in = S_in;
    c.o = o; c.S_out = S_out;
    if (timed(KID_CHUNK_PREP, st, [&] { return launch_chunk_prep(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_STATE_FWD, st, [&] { return launch_state_fwd(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_OUTPUT_FWD, st, [&] { return launch_output_fwd(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    return launch_status();
}

int osdn_bwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
             float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
             void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_params(p, true);
    if (rc != OSDN_OK) return rc;
    if (!q || !k || !v || !beta || !dO || !dq || !dk || !dv || !dbeta || !dd_in || !dS_in)
        return OSDN_ERR_NULL;
    if ((log_alpha && !dlog_alpha) || (retention && !dretention)) return OSDN_ERR_NULL;
    (void)d_in; (void)S_in;
    Layout L = make_layout(p);
    rc = check_ws(workspace, workspace_bytes, L.total_bwd);
    if (rc != OSDN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;

    ChunkArgs c = chunk_args(p, L, ws);
    c.q = q; c.k = k; c.v = v; c.beta = beta; c.log_alpha = log_alpha;
    c.dO = dO; c.dS_out = dS_out;
    c.dElt = ws + L.dElt; c.Qt = ws + L.Qt; c.dOt = ws + L.dOt; c.dEt = ws + L.dEt; c.dS_ckpt = ws + L.dS_ckpt;
    c.dS_in = dS_in; c.dq = dq; c.dv = dv;
    c.dk_read = reinterpret_cast<float *>(ws + L.dk_read);
    c.dkt = reinterpret_cast<float *>(ws + L.dkt);
    c.dbeta = dbeta; c.dlog_alpha = log_alpha ? dlog_alpha : nullptr;
    if (timed(KID_BWD_LOCAL, st, [&] { return launch_bwd_local(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_BWD_CHAIN, st, [&] { return launch_bwd_chain(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_BWD_POST, st, [&] { return launch_bwd_post(c, bf, st); }) != 0) return OSDN_ERR_SHAPE;

    PrecondBwdArgs pb{};
    pb.B = p->B; pb.T = p->T; pb.H = p->H; pb.K = p->K;
    pb.eta = p->eta; pb.d_min = p->d_min; pb.d_max = p->d_max; pb.eps = p->eps;
    pb.beta_aware = p->beta_aware;
    pb.k = k; pb.beta = beta; pb.retention = retention;
    pb.d_ckpt = reinterpret_cast<const float *>(ws + L.d_ckpt);
    pb.tok_scalars = reinterpret_cast<float *>(ws + L.tok_scalars);
    pb.masks = reinterpret_cast<uint2 *>(ws + L.masks);
    pb.a_ckpt = reinterpret_cast<float *>(ws + L.a_ckpt);
    pb.dkt = c.dkt; pb.dk_read = c.dk_read; pb.dd_out = dd_out;
    pb.dk = dk; pb.dbeta = dbeta; pb.dretention = retention ? dretention : nullptr; pb.dd_in = dd_in;
    if (pb.d_min <= pb.d_max &&
        timed(KID_PRECOND_MASK, st, [&] { return launch_precond_mask(pb, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_PRECOND_CHAIN, st, [&] { return launch_precond_chain(pb, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    if (timed(KID_PRECOND_POST, st, [&] { return launch_precond_post(pb, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    return launch_status();
}

void osdn_profile_enable(int on) { g_prof_on = on != 0; }

int osdn_profile_kernel_count(void) { return KID_COUNT; }

const char *osdn_profile_kernel_name(int id) { return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : ""; }

int osdn_profile_read(double *ms_sum, int *launches, int n) {
    for (int i = 0; i < n; ++i) { ms_sum[i] = 0.0; launches[i] = 0; }
    int rc = OSDN_OK;
    for (Timed &t : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(t.e1) != hipSuccess || hipEventElapsedTime(&ms, t.e0, t.e1) != hipSuccess)
            rc = OSDN_ERR_LAUNCH;
        else if (t.id < n) { ms_sum[t.id] += ms; launches[t.id] += 1; }
        (void)hipEventDestroy(t.e0);
        (void)hipEventDestroy(t.e1);
    }
    g_prof.clear();
    return rc;
}

}  // extern "C"
