// C-ABI boundary of libosdn: argument validation, workspace carving, kernel launches.
// See include/osdn.h for the contract of every entry point.
#include "../../include/osdn.h"
#include "osdn_kernels.h"

#include <cmath>
#include <map>
#include <mutex>
#include <vector>

namespace {

using namespace osdn;

// Optional per-kernel timing with HIP events on the caller's stream (off by default; the
// only process-wide state the library has).  Not thread-safe; meant for benchmarks.
enum { KID_PRECOND_FWD, KID_CHUNK_PREP, KID_STATE_FWD, KID_OUTPUT_FWD, KID_BWD_CHAIN,
       KID_BWD_POST, KID_PRECOND_MASK, KID_PRECOND_CHAIN, KID_PRECOND_POST, KID_STEP, KID_PAD, KID_UNFOLD, KID_PRECOND_LIN,
       KID_COUNT };
const char *const kKernelNames[KID_COUNT] = {"precond_fwd", "chunk_prep", "state_fwd", "output_fwd",
                                             "bwd_chain", "bwd_post", "precond_mask",
                                             "precond_chain", "precond_post", "step", "pad", "unfold", "precond_lin"};
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
    size_t Qg, Kg, Kd, gamC, dgamC;                                      // per-channel state gate
    size_t tables;                                                       // packed sequences: the index tables
    size_t kt, d_ckpt, tok_scalars, Wt, Ktr, Ut, Et, S_ckpt;       // forward
    size_t piece_start, piece_map, piece_flags;                          // phase 1 as sweeps over the whole sequence
    size_t Tm, Pm;                                                       // written by the forward pass for the backward pass only
    size_t dEt, dS_ckpt, dk_read, dkt, masks, a_ckpt;                    // backward only
    size_t lin_clean, lin_M, lin_r0, lin_t0, lin_aux;                           // backward: chunks of phase 1 in solved form
    // padded copies of the caller's tensors, only when T is not a multiple of the chunk length
    size_t p_q, p_k, p_v, p_beta, p_g, p_r, p_o;                        // forward
    size_t p_dO, p_dq, p_dk, p_dv, p_dbeta, p_dg, p_dr;                 // backward
    size_t total_fwd, total_bwd;
};

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// Phase 1 as sweeps over the whole sequence: at most this many pieces over all chains, and at
// most this many sweeps before the sequential kernel takes over.
constexpr int MAX_PIECES = 512, MAX_PIECE_SWEEPS = 13;

int check_params(const osdn_params *p, bool need_chunks) {
    if (!p) return OSDN_ERR_NULL;
    if (p->io_dtype != OSDN_F32 && p->io_dtype != OSDN_BF16) return OSDN_ERR_DTYPE;
    if (p->B < 1 || p->T < 1 || p->H < 1 || p->chunk != C) return OSDN_ERR_SHAPE;
    if (p->K != 64 && p->K != 128) return OSDN_ERR_SHAPE;
    if (need_chunks) {
        if (p->V < 64 || p->V > 512 || p->V % 64 != 0) return OSDN_ERR_SHAPE;
        if (p->B > 65535 || p->H > 65535) return OSDN_ERR_SHAPE;
    }
    if ((long long)p->B * p->H > 0x7fffffffLL / 64) return OSDN_ERR_SHAPE;
    // the kernels address the 64 token rows of a chunk with 32-bit byte offsets (V only matters to
    // the entry points that have a value tensor)
    const int widest = (need_chunks && p->V > p->K) ? p->V : p->K;
    if ((long long)p->H * widest * 4 * C >= (1LL << 32)) return OSDN_ERR_SHAPE;
    if (!(p->eta >= 0.f) || !(p->eps > 0.f) || !std::isfinite(p->eta) || !std::isfinite(p->eps) ||
        !std::isfinite(p->scale) || std::isnan(p->d_min) || std::isnan(p->d_max))
        return OSDN_ERR_PARAM;
    if (p->retention_per_channel != 0 && p->retention_per_channel != 1) return OSDN_ERR_PARAM;
    if (p->gate_per_channel != 0 && p->gate_per_channel != 1) return OSDN_ERR_PARAM;
    if (p->segments < 0 || p->p1_pieces < -1 || p->p1_piece_sweeps < 0 || p->p1_piece_sweeps > MAX_PIECE_SWEEPS ||
        p->p1_solved < -1 || p->p1_solved > 1)
        return OSDN_ERR_PARAM;
    return OSDN_OK;
}

// Host-side description of a batch of packed sequences (n_seqs == 0: a plain [B,T] batch).
struct Packing {
    int n_seqs = 0;
    int N = 0;                   // chunks of the padded token axis (per batch entry)
    int longest = 0;             // chunks of the longest sequence
    bool ragged = false;         // some sequence is not a whole number of chunks: work on padded copies
    std::vector<int> tables;     // seq_chunks [n_seqs + 1], chunk_row [N], chunk_len [N]
};

// cu_seqlens: n_seqs + 1 ascending token offsets, from 0 to T, on the host
int make_packing(const osdn_params *p, const int32_t *cu, int n_seqs, Packing &pk) {
    if (!cu) return OSDN_ERR_NULL;
    if (p->B != 1 || n_seqs < 1 || (long long)n_seqs * p->H > 0x7fffffffLL / 64) return OSDN_ERR_SHAPE;
    if (cu[0] != 0 || cu[n_seqs] != p->T) return OSDN_ERR_SHAPE;
    long long N = 0;
    for (int s = 0; s < n_seqs; ++s) {
        const long long len = (long long)cu[s + 1] - cu[s];
        if (len < 1) return OSDN_ERR_SHAPE;
        N += (len + C - 1) / C;
        if ((len + C - 1) / C > pk.longest) pk.longest = (int)((len + C - 1) / C);
        pk.ragged = pk.ragged || len % C != 0;
    }
    if (N * C > 0x7fffffffLL) return OSDN_ERR_SHAPE;
    pk.n_seqs = n_seqs;
    pk.N = (int)N;
    pk.tables.assign((size_t)n_seqs + 1 + 2 * (size_t)N, 0);
    int *seq_chunks = pk.tables.data(), *chunk_row = seq_chunks + n_seqs + 1, *chunk_len = chunk_row + N;
    int c = 0;
    for (int s = 0; s < n_seqs; ++s) {
        seq_chunks[s] = c;
        for (int t = cu[s]; t < cu[s + 1]; t += C, ++c) {
            chunk_row[c] = t;
            chunk_len[c] = cu[s + 1] - t < C ? cu[s + 1] - t : C;
        }
    }
    seq_chunks[n_seqs] = c;
    return OSDN_OK;
}

void plain_packing(const osdn_params *p, Packing &pk) {
    pk.N = (p->T + C - 1) / C;
    pk.longest = pk.N;
    pk.ragged = pk.N * C != p->T;
}

// every buffer is sized for the padded token axis of pk.N whole chunks
Layout make_layout(const osdn_params *p, const Packing &pk) {
    const size_t es = p->io_dtype == OSDN_BF16 ? 2 : 4;
    const size_t B = p->B, H = p->H, K = p->K, V = p->V, N = (size_t)pk.N, T = N * C;
    const size_t RK = p->retention_per_channel ? K : 1;    // retention values per (token, head)
    const size_t GK = p->gate_per_channel ? K : 1;         // state gates per (token, head)
    const bool ragged = pk.ragged;
    Layout L{};
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align256(off + bytes); return o; };
    L.tables = take(pk.tables.size() * sizeof(int));
    L.kt = take(B * T * H * K * es);
    L.d_ckpt = take(B * H * N * K * 4);
    L.tok_scalars = take(B * T * H * 4 * 4);
    L.Wt = take(B * T * H * K * es);
    L.Ktr = take(B * T * H * K * es);
    L.Ut = take(B * T * H * V * es);
    L.Et = take(B * T * H * V * es);
    L.S_ckpt = take(B * H * N * V * K * es);
    if (p->gate_per_channel) {
        L.Qg = take(B * T * H * K * es); L.Kg = take(B * T * H * K * es); L.Kd = take(B * T * H * K * es);
        L.gamC = take(B * H * N * K * 4);
    }
    if (ragged) {
        L.p_q = take(B * T * H * K * es); L.p_k = take(B * T * H * K * es);
        L.p_v = take(B * T * H * V * es); L.p_o = take(B * T * H * V * es);
        L.p_beta = take(B * T * H * 4); L.p_g = take(B * T * H * 4 * GK); L.p_r = take(B * T * H * 4 * RK);
    }
    L.piece_start = take((size_t)2 * MAX_PIECES * K * 4);
    L.piece_map = take((size_t)2 * MAX_PIECES * K * 16);
    L.piece_flags = take((MAX_PIECES / 2) * sizeof(int));       // one "settled" flag per chain
    L.total_fwd = off;
    L.Tm = take(B * H * N * C * C * es);
    L.Pm = take(B * H * N * C * C * es);
    L.dEt = take(B * T * H * V * es);
    L.dS_ckpt = take(B * H * N * V * K * es);
    L.dk_read = take(B * T * H * K * es);
    L.dkt = take(B * T * H * K * es);
    L.masks = take(B * H * N * K * 8);
    L.a_ckpt = take(B * H * N * K * 4);
    L.lin_clean = take(B * H * N * 4);
    L.lin_M = take(B * H * N * C * C * es);
    L.lin_r0 = take(B * H * N * C * 4);
    L.lin_t0 = take(B * H * N * K * 4);
    L.lin_aux = take(B * H * N * 2048);
    if (p->gate_per_channel) L.dgamC = take(B * H * N * K * 4);
    if (ragged) {
        L.p_dO = take(B * T * H * V * es); L.p_dv = take(B * T * H * V * es);
        L.p_dq = take(B * T * H * K * es); L.p_dk = take(B * T * H * K * es);
        L.p_dbeta = take(B * T * H * 4); L.p_dg = take(B * T * H * 4 * GK); L.p_dr = take(B * T * H * 4 * RK);
    }
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
    a.ret_vec = p->retention_per_channel;
    return a;
}

ChunkArgs chunk_args(const osdn_params *p, const Layout &L, char *ws) {      // p: the padded problem
    ChunkArgs c{};
    c.B = p->B; c.T = p->T; c.H = p->H; c.K = p->K; c.V = p->V; c.N = p->T / C;
    c.scale = p->scale;
    c.kt = ws + L.kt; c.Wt = ws + L.Wt; c.Ktr = ws + L.Ktr;
    c.Ut = ws + L.Ut; c.Et = ws + L.Et;
    c.S_ckpt = ws + L.S_ckpt;
    return c;
}


// ---- pipelining of the two phases --------------------------------------------------------
// Phase 1 (the preconditioner chains, one workgroup per (batch, head)) leaves most of the chip
// idle, and phase 2 only needs the k~ of the chunks it is working on.  With more than one
// segment the sequence is cut into ranges of chunks: phase 1 runs on a side stream, segment by
// segment, and phase 2 follows one segment behind on the caller's stream (in the backward
// pass the other way round, right to left).  The side stream is forked from and joined back
// into the caller's stream with events, so to the caller the call still behaves as work
// enqueued on its stream.  One side stream and one set of events per (device, caller stream),
// created on first use and kept (pipeline_for below); a mutex guards only the table of them.
constexpr int MAX_SEGMENTS = 16;
struct Pipeline {
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr, early[2] = {}, a[MAX_SEGMENTS] = {};
    bool ok = false;
};
std::mutex g_pipe_mu;
std::map<std::pair<int, hipStream_t>, Pipeline> g_pipes;

// The side stream and events that go with one caller stream on the current device (created on
// first use, kept until the process ends).  One set per caller stream: a call that is being
// captured into a graph on one stream pulls only its own side stream into the capture, and
// calls on other streams, from other threads, neither wait for it nor enqueue into it.  Calls
// that share a caller stream have to be ordered by the caller, as for any work on one stream.
Pipeline *pipeline_for(hipStream_t caller) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return nullptr;
    std::lock_guard<std::mutex> lock(g_pipe_mu);
    const auto key = std::make_pair(dev, caller);
    auto it = g_pipes.find(key);
    if (it == g_pipes.end()) {
        Pipeline pl;
        bool ok = hipStreamCreateWithFlags(&pl.side, hipStreamNonBlocking) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&pl.fork, hipEventDisableTiming) == hipSuccess;
        ok = ok && hipEventCreateWithFlags(&pl.join, hipEventDisableTiming) == hipSuccess;
        for (int i = 0; ok && i < 2; ++i) ok = hipEventCreateWithFlags(&pl.early[i], hipEventDisableTiming) == hipSuccess;
        for (int i = 0; ok && i < MAX_SEGMENTS; ++i)
            ok = hipEventCreateWithFlags(&pl.a[i], hipEventDisableTiming) == hipSuccess;
        pl.ok = ok;
        it = g_pipes.emplace(key, pl).first;
    }
    return it->second.ok ? &it->second : nullptr;
}

// Number of segments for a sequence of N chunks (params->segments > 0 overrides it; 1 = no
// pipelining).  At least two (any sequence of at least two chunks, so that short
// sequences take the same path).  A segment more shortens the stretch of phase 1 that runs with
// nothing beside it (the first segment of the forward pass, the last of the backward pass) and
// costs launches, cross-stream waits and partly filled rounds of workgroups.
//  - forward: about 16 chunks per segment, at most six segments (measured flat beyond).
//  - backward: a segment more costs more there, because every launch of the phase-2 chain kernel
//    meets a phase-1 chain kernel on the other stream and the two do not fit on one CU together:
//    when the workgroups of both (chain_wgs) outnumber the CUs, the count that balances the
//    exposed tail against that cost is about sqrt(N / 15) (2 at 64 chunks, 4 at 256); when they
//    all fit side by side, about 32 chunks per segment, at most twelve: of that count and the two
//    above it, the one whose segments fill whole rounds of bwd_post workgroups (one per chunk and
//    chain, one per CU at a time) best.
// Segments cut the chunk axis as a whole.  With packed sequences the sequential kernels of a
// segment only have the sequences that cross it to work on, one after the other segment by
// segment, so cutting pays only while one sequence makes up most of the axis; otherwise the
// many independent chains fill the chip by themselves and everything runs in one piece.
constexpr int NUM_CU = 256;
int segment_count(int forced, int N, int longest, long long chain_wgs, bool backward, long long chains = 0) {
    if (forced <= 0 && (long long)longest * 4 < (long long)N * 3) return 1;
    int S = forced;
    if (forced <= 0) {
        if (!backward) S = N / 16 > 6 ? 6 : N / 16;
        else if (chain_wgs > NUM_CU) S = (int)std::lround(std::sqrt(N / 15.0)) > 6 ? 6 : (int)std::lround(std::sqrt(N / 15.0));
        else {
            S = N / 32 > 12 ? 12 : N / 32;
            if (S < 2) S = 2;
            double best = 0.0;
            int pick = S;
            for (int c = S; c <= S + 2 && c <= 12 && c <= N && chains > 0; ++c) {
                const int first = N / (2 * c) > 0 ? N / (2 * c) : 1;
                const double wgs = (double)(N - first) / (c - 1) * (double)chains;   // bwd_post workgroups of a segment
                const double fill = wgs / (std::ceil(wgs / NUM_CU) * NUM_CU);
                if (fill > best + 1e-9) { best = fill; pick = c; }
            }
            S = pick;
        }
        if (S < 2 && N >= 2) S = 2;
    }
    if (S > MAX_SEGMENTS) S = MAX_SEGMENTS;
    if (S > N) S = N;
    return S < 1 ? 1 : S;
}
// first chunk of segment s.  Segment 0 is half as long as the others: it is the one that runs
// without a partner (phase 1 of it before anything of phase 2 can start in the forward pass,
// and after everything else in the backward pass).
// First chunk of segment s when every segment is r times as long as the one before.  Used by
// the forward pass when phase 2 is the slower of the two phases (many chains): phase 2 then
// starts early on a short segment and is never left waiting for phase 1, and the long last
// segment runs when phase 1 is already out of the way.
inline int seg_begin_grow(int N, int S, int s, double r) {
    if (s <= 0) return 0;
    if (s >= S) return N;
    const double f = (std::pow(r, s) - 1.0) / (std::pow(r, S) - 1.0);
    int b = (int)std::lround(N * f);
    if (b < s) b = s;                       // at least one chunk per segment
    if (b > N - (S - s)) b = N - (S - s);
    return b;
}
inline int seg_begin(int N, int S, int s) {
    if (s <= 0) return 0;
    if (s >= S) return N;
    const int first = N / (2 * S) > 0 ? N / (2 * S) : 1;
    return first + (int)((long long)(N - first) * (s - 1) / (S - 1));
}

// Phase 1 of the forward pass as sweeps over the whole sequence, for few long chains: with
// chains on at most an eighth of the CUs the sequential kernel leaves most of the chip idle and
// its walk over the chunks is the whole forward pass.  Every chain is cut into pieces (one
// workgroup per CU over all chains, at least 8 chunks each); a sweep runs all pieces side by
// side, each from its current start value, and leaves every piece as a composed map per
// coordinate; the next sweep walks those maps for its start values; a chain is settled when none
// of its start values moves any more.  Plain batches only.  params->p1_pieces forces a number of
// pieces per chain (-1: never), params->p1_piece_sweeps the sweep limit.
inline void pieces_plan(const osdn_params *p, int N, long long chains, bool packed, int &pieces, int &piece_chunks,
                        int &sweeps) {
    pieces = 0; piece_chunks = 0;
    // sweeps needed without retention, measured: 4 at 64 and 128 chunks, then one more per
    // doubling (7 at 1024); the limit leaves two in hand
    sweeps = 7;                                  // (the last one only finds that nothing moved)
    for (int n = 128; n < N && sweeps < MAX_PIECE_SWEEPS; n *= 2) ++sweeps;
    if (packed || chains > MAX_PIECES / 2) return;
    const int forced = p->p1_pieces;              // 0: decide here; -1: never; n > 0: n pieces per chain
    int target, min_chunks;
    if (forced != 0) { target = forced > 0 ? forced : 0; min_chunks = 1; }
    else if (chains * 8 <= NUM_CU && N >= 64) { target = (int)(NUM_CU / chains); min_chunks = 8; }
    else return;
    if ((long long)target * chains > MAX_PIECES) target = (int)(MAX_PIECES / chains);
    if (target < 2) return;
    int len = (N + target - 1) / target;
    if (len < min_chunks) len = min_chunks;
    const int P = (N + len - 1) / len;
    if (P < 2) return;
    pieces = P; piece_chunks = len;
    if (p->p1_piece_sweeps >= 1) sweeps = p->p1_piece_sweeps;
}

#define OSDN_HIP_OK(x) do { if ((x) != hipSuccess) return OSDN_ERR_LAUNCH; } while (0)

// ---- scratch of osdn_fwd_noalloc: device memory that belongs to the library ---------------
// A file-scope device array (every GPU the library runs on holds its own copy, at its own
// address, from the moment the code object is loaded until the process ends).  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address kernels can use is looked
// up once per device, with that device current, and only that pointer is ever passed on.
constexpr size_t STATIC_SCRATCH_BYTES = OSDN_NOALLOC_MAX_WORKSPACE;
static __device__ __align__(256) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of the current device's copy of the array (null on failure).
void *static_scratch_for_current_device() {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// Once the side stream has been forked off, every way out of the call joins it back into the
// caller's stream: also an error return must not leave work behind that the caller's stream does
// not wait for (or, under stream capture, a branch that never rejoins).
struct SideJoin {
    Pipeline *pl;
    hipStream_t st;
    bool armed;
    ~SideJoin() {
        if (armed && hipEventRecord(pl->join, pl->side) == hipSuccess) (void)hipStreamWaitEvent(st, pl->join, 0);
    }
};

}  // namespace

extern "C" {

size_t osdn_workspace_bytes(const osdn_params *p, int for_backward) {
    if (check_params(p, true) != OSDN_OK) return 0;
    Packing pk;
    plain_packing(p, pk);
    Layout L = make_layout(p, pk);
    return for_backward ? L.total_bwd : L.total_fwd;
}

size_t osdn_workspace_bytes_packed(const osdn_params *p, const int32_t *cu_seqlens, int32_t n_seqs,
                                   int for_backward) {
    Packing pk;
    if (check_params(p, true) != OSDN_OK || make_packing(p, cu_seqlens, n_seqs, pk) != OSDN_OK) return 0;
    Layout L = make_layout(p, pk);
    return for_backward ? L.total_bwd : L.total_fwd;
}

size_t osdn_debug_mask_offset(const osdn_params *p) {
    if (check_params(p, true) != OSDN_OK) return 0;
    Packing pk;
    plain_packing(p, pk);
    return make_layout(p, pk).masks;
}

const char *osdn_strerror(int status) {
    switch (status) {
        case OSDN_OK: return "ok";
        case OSDN_ERR_NULL: return "a required pointer is NULL";
        case OSDN_ERR_SHAPE: return "unsupported shape (chunk must be 64, K in {64,128}, V % 64 == 0, V <= 512, at most 64 tokens per osdn_step)";
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
    a.n0 = 0; a.n1 = (p->T + C - 1) / C;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;
    if (timed(KID_PRECOND_FWD, st, [&] { return launch_precond_fwd(a, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    return launch_status();
}

int osdn_step(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
              const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
              void *o, float *S_out, float *d_out, void *stream) {
    int rc = check_params(p, false);
    if (rc != OSDN_OK) return rc;
    if (p->T > C || p->V < 64 || p->V > 512 || p->V % 64 != 0) return OSDN_ERR_SHAPE;
    if (!q || !k || !v || !beta || !o || !S_out || !d_out) return OSDN_ERR_NULL;
    if (d_out == d_in) return OSDN_ERR_NULL;         // every workgroup of a chain reads d_in
    StepArgs a{};
    a.B = p->B; a.T = p->T; a.H = p->H; a.K = p->K; a.V = p->V;
    a.scale = p->scale; a.eta = p->eta; a.d_min = p->d_min; a.d_max = p->d_max; a.eps = p->eps;
    a.beta_aware = p->beta_aware;
    a.ret_vec = p->retention_per_channel;
    a.gate_vec = p->gate_per_channel;
    a.q = q; a.k = k; a.v = v; a.beta = beta; a.log_alpha = log_alpha; a.retention = retention;
    a.d_in = d_in; a.S_in = S_in; a.o = o; a.S_out = S_out; a.d_out = d_out;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;
    if (timed(KID_STEP, st, [&] { return launch_step(a, bf, st); }) != 0) return OSDN_ERR_SHAPE;
    return launch_status();
}

// cu_seqlens == null: a plain [B,T] batch; otherwise n_seqs sequences packed on the token axis (B == 1)
static int fwd_impl(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             void *o, float *S_out, float *d_out, const int32_t *cu_seqlens, int n_seqs, void *workspace,
             size_t workspace_bytes, void *stream) {
    int rc = check_params(p, true);
    if (rc != OSDN_OK) return rc;
    if (!q || !k || !v || !beta || !o || !S_out || !d_out) return OSDN_ERR_NULL;
    if (p->gate_per_channel && !log_alpha) return OSDN_ERR_NULL;
    Packing pk;
    if (cu_seqlens || n_seqs != 0) {
        rc = make_packing(p, cu_seqlens, n_seqs, pk);
        if (rc != OSDN_OK) return rc;
    } else {
        plain_packing(p, pk);
    }
    Layout L = make_layout(p, pk);
    rc = check_ws(workspace, workspace_bytes, L.total_fwd);
    if (rc != OSDN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;
    int *tables = reinterpret_cast<int *>(ws + L.tables);
    const int *seq_chunks = pk.n_seqs ? tables : nullptr;
    const int *chunk_row = tables + pk.n_seqs + 1, *chunk_len = chunk_row + pk.N;
    if (pk.n_seqs && timed(KID_PAD, st, [&] { return launch_upload_ints(pk.tables.data(), pk.tables.size(), tables, st); }) != 0)
        return OSDN_ERR_SHAPE;

    // ragged chunks (the tail of the sequence, or of any packed sequence): work on padded copies
    // (no-op pad tokens) and move the output back at the end
    osdn_params padded = *p;
    padded.T = pk.N * C;
    const int T_user = p->T;
    const bool ragged = pk.ragged;
    void *o_user = o;
    auto move = [&](const void *src, void *dst, size_t row, bool to_padded, uint32_t fill) {
        return timed(KID_PAD, st, [&] {
            if (pk.n_seqs) return launch_move_chunk_rows(src, dst, chunk_row, chunk_len, pk.N, row, to_padded, fill, st);
            return to_padded ? launch_copy_rows(src, T_user, dst, padded.T, p->B, row, fill, st)
                             : launch_copy_rows(src, padded.T, dst, T_user, p->B, row, fill, st);
        });
    };
    if (ragged) {
        const size_t es = bf ? 2 : 4, rk = (size_t)p->H * p->K * es, rv = (size_t)p->H * p->V * es, rg = (size_t)p->H * 4;
        auto pad = [&](const void *src, size_t off, size_t row, uint32_t fill) { return move(src, ws + off, row, true, fill); };
        if (pad(q, L.p_q, rk, 0u) != 0 || pad(k, L.p_k, rk, 0u) != 0 || pad(v, L.p_v, rv, 0u) != 0 ||
            pad(beta, L.p_beta, rg, 0u) != 0 || (log_alpha && pad(log_alpha, L.p_g, p->gate_per_channel ? rg * p->K : rg, 0u) != 0) ||
            (retention && pad(retention, L.p_r, p->retention_per_channel ? rg * p->K : rg, 0x3f800000u) != 0))
            return OSDN_ERR_SHAPE;
        q = ws + L.p_q; k = ws + L.p_k; v = ws + L.p_v; o = ws + L.p_o;
        beta = reinterpret_cast<const float *>(ws + L.p_beta);
        if (log_alpha) log_alpha = reinterpret_cast<const float *>(ws + L.p_g);
        if (retention) retention = reinterpret_cast<const float *>(ws + L.p_r);
        p = &padded;
    }
    auto finish = [&]() -> int {
        if (ragged && move(o, o_user, (size_t)p->H * p->V * (bf ? 2 : 4), false, 0u) != 0) return OSDN_ERR_SHAPE;
        return launch_status();
    };

    PrecondArgs pa = precond_args(p);
    pa.k = k; pa.beta = beta; pa.retention = retention;
    pa.k_tilde = ws + L.kt; pa.d_out = d_out; pa.d_ckpt = reinterpret_cast<float *>(ws + L.d_ckpt);
    pa.tok_scalars = reinterpret_cast<float *>(ws + L.tok_scalars);
    pa.n_seqs = pk.n_seqs; pa.seq_chunks = seq_chunks; pa.d_first = d_in;
    ChunkArgs c = chunk_args(p, L, ws);
    c.q = q; c.k = k; c.v = v; c.beta = beta; c.log_alpha = log_alpha;
    c.o = o; c.S_out = S_out;
    // (I + A)^-1 and P are only of use to a backward pass: they are written when the workspace is
    // the one osdn_workspace_bytes(p, 1) asks for, which osdn_bwd requires anyway
    if (workspace_bytes >= L.total_bwd) { c.Tm = ws + L.Tm; c.Pm = ws + L.Pm; }
    c.n_seqs = pk.n_seqs; c.seq_chunks = seq_chunks; c.S_first = S_in;
    // one state gate per key channel: chunk_prep folds the channel decays into the operands and
    // leaves Gamma . Q and K~ / Gamma, on which the state and output kernels run as if ungated
    const bool gv = p->gate_per_channel != 0;
    ChunkArgs cg = c;                                  // what state_fwd and output_fwd see
    if (gv) {
        c.gate_vec = 1;
        c.Qg = ws + L.Qg; c.Kg = ws + L.Kg; c.Kd = ws + L.Kd; c.gamC = reinterpret_cast<float *>(ws + L.gamC);
        cg = c;
        cg.log_alpha = nullptr; cg.q = c.Qg; cg.kt = c.Kd;
    }

    const int N = p->T / C;
    const long long chains = (long long)(pk.n_seqs ? pk.n_seqs : p->B) * p->H;
    int pieces, piece_chunks, piece_sweeps;
    pieces_plan(p, N, chains, pk.n_seqs != 0, pieces, piece_chunks, piece_sweeps);
    int S = pieces ? 1 : segment_count(p->segments, N, pk.longest, 0, false);
    Pipeline *pl = S > 1 ? pipeline_for(st) : nullptr;
    if (!pl) S = 1;
    // chain workgroups of both phases (32 rows of the state per workgroup in state_fwd) against the CUs
    const bool crowded = chains * (p->V / 32) + chains > NUM_CU;
    // Few chains: the state kernel takes slices of 16 values instead of 32 when its workgroups then
    // still find a CU each (beside those of phase 1, unless phase 1 runs ahead as sweeps over pieces):
    // its time per chunk is latency, not work, and half the work per workgroup shortens it.
    c.narrow_slices = cg.narrow_slices = chains * (p->V / 16) + (pieces ? 0 : chains) <= NUM_CU;
    auto seg_range = [&](int sidx, int &n0, int &n1) {
        if (crowded) { n0 = seg_begin_grow(N, S, sidx, 1.7); n1 = seg_begin_grow(N, S, sidx + 1, 1.7); return; }
        n0 = seg_begin(N, S, sidx); n1 = seg_begin(N, S, sidx + 1);
    };
    auto precond = [&](int sidx, hipStream_t s1) {
        seg_range(sidx, pa.n0, pa.n1);
        pa.d_in = sidx == 0 ? d_in : d_out;          // d is carried in d_out
        return timed(KID_PRECOND_FWD, s1, [&] { return launch_precond_fwd(pa, bf, s1); });
    };
    auto phase2 = [&](int kid, int sidx) {
        ChunkArgs &ck = (gv && kid != KID_CHUNK_PREP) ? cg : c;
        seg_range(sidx, ck.n0, ck.n1);
        ck.S_in = sidx == 0 ? S_in : S_out;          // S is carried in S_out
        return timed(kid, st, [&] {
            return kid == KID_CHUNK_PREP ? launch_chunk_prep(ck, bf, st)
                 : kid == KID_STATE_FWD ? launch_state_fwd(ck, bf, st) : launch_output_fwd(ck, bf, st);
        });
    };
    // phase 1 as sweeps over the pieces of every chain, launched ahead of time; behind them the
    // sequential kernel for the chains that have not settled by then
    auto precond_pieces = [&]() {
        int *settled = reinterpret_cast<int *>(ws + L.piece_flags);
        PrecondArgs pp = pa;
        pp.n0 = 0; pp.n1 = N; pp.d_in = d_in;
        pp.pieces = pieces; pp.piece_chunks = piece_chunks;
        pp.piece_start = reinterpret_cast<float *>(ws + L.piece_start);
        pp.piece_map = reinterpret_cast<float4 *>(ws + L.piece_map);
        pp.settled = settled;
        for (int i = 0; i < piece_sweeps; ++i) {
            pp.sweep = i;
            if (timed(KID_PRECOND_FWD, st, [&] { return launch_precond_fwd(pp, bf, st); }) != 0) return -1;
        }
        pa.n0 = 0; pa.n1 = N; pa.d_in = d_in; pa.settled = settled;
        const int rc1 = timed(KID_PRECOND_FWD, st, [&] { return launch_precond_fwd(pa, bf, st); });
        pa.settled = nullptr;
        return rc1;
    };
    if (!pl) {
        if ((pieces ? precond_pieces() : precond(0, st)) != 0 || phase2(KID_CHUNK_PREP, 0) != 0 ||
            phase2(KID_STATE_FWD, 0) != 0 || phase2(KID_OUTPUT_FWD, 0) != 0)
            return OSDN_ERR_SHAPE;
        return finish();
    }
    // side: phase 1, segment after segment          (a[s]: phase 1 of segment s done)
    // main: phase 2 of segment s once a[s] has fired
    hipStream_t s1 = pl->side;
    OSDN_HIP_OK(hipEventRecord(pl->fork, st));
    OSDN_HIP_OK(hipStreamWaitEvent(s1, pl->fork, 0));
    SideJoin rejoin{pl, st, true};
    for (int s = 0; s < S; ++s) {
        if (precond(s, s1) != 0) return OSDN_ERR_SHAPE;
        OSDN_HIP_OK(hipEventRecord(pl->a[s], s1));
    }
    for (int s = 0; s < S; ++s) {
        OSDN_HIP_OK(hipStreamWaitEvent(st, pl->a[s], 0));
        if (phase2(KID_CHUNK_PREP, s) != 0 || phase2(KID_STATE_FWD, s) != 0 || phase2(KID_OUTPUT_FWD, s) != 0)
            return OSDN_ERR_SHAPE;
    }
    rejoin.armed = false;               // the wait for the last segment's event was the join
    return finish();
}

static int bwd_impl(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
             float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
             const int32_t *cu_seqlens, int n_seqs, void *workspace, size_t workspace_bytes, void *stream) {
    int rc = check_params(p, true);
    if (rc != OSDN_OK) return rc;
    if (!q || !k || !v || !beta || !dO || !dq || !dk || !dv || !dbeta || !dd_in || !dS_in)
        return OSDN_ERR_NULL;
    if ((log_alpha && !dlog_alpha) || (retention && !dretention)) return OSDN_ERR_NULL;
    if (p->gate_per_channel && !log_alpha) return OSDN_ERR_NULL;
    (void)d_in; (void)S_in;
    Packing pk;
    if (cu_seqlens || n_seqs != 0) {
        rc = make_packing(p, cu_seqlens, n_seqs, pk);
        if (rc != OSDN_OK) return rc;
    } else {
        plain_packing(p, pk);
    }
    Layout L = make_layout(p, pk);
    rc = check_ws(workspace, workspace_bytes, L.total_bwd);
    if (rc != OSDN_OK) return rc;
    char *ws = static_cast<char *>(workspace);
    hipStream_t st = static_cast<hipStream_t>(stream);
    const bool bf = p->io_dtype == OSDN_BF16;
    int *tables = reinterpret_cast<int *>(ws + L.tables);
    const int *seq_chunks = pk.n_seqs ? tables : nullptr;
    const int *chunk_row = tables + pk.n_seqs + 1, *chunk_len = chunk_row + pk.N;
    if (pk.n_seqs && timed(KID_PAD, st, [&] { return launch_upload_ints(pk.tables.data(), pk.tables.size(), tables, st); }) != 0)
        return OSDN_ERR_SHAPE;

    // ragged chunks: the padded inputs are the ones the forward call left in the workspace; dO
    // is padded here, the gradients are produced padded and moved back at the end
    osdn_params padded = *p;
    padded.T = pk.N * C;
    const int T_user = p->T;
    const bool ragged = pk.ragged;
    auto move = [&](const void *src, void *dst, size_t row, bool to_padded) {
        return timed(KID_PAD, st, [&] {
            if (pk.n_seqs) return launch_move_chunk_rows(src, dst, chunk_row, chunk_len, pk.N, row, to_padded, 0u, st);
            return to_padded ? launch_copy_rows(src, T_user, dst, padded.T, p->B, row, 0u, st)
                             : launch_copy_rows(src, padded.T, dst, T_user, p->B, row, 0u, st);
        });
    };
    void *dq_user = dq, *dk_user = dk, *dv_user = dv;
    float *dbeta_user = dbeta, *dg_user = dlog_alpha, *dr_user = dretention;
    const size_t es_ = bf ? 2 : 4, rk_ = (size_t)p->H * p->K * es_, rv_ = (size_t)p->H * p->V * es_, rg_ = (size_t)p->H * 4;
    if (ragged) {
        if (move(dO, ws + L.p_dO, rv_, true) != 0) return OSDN_ERR_SHAPE;
        q = ws + L.p_q; k = ws + L.p_k; v = ws + L.p_v; dO = ws + L.p_dO;
        beta = reinterpret_cast<const float *>(ws + L.p_beta);
        if (log_alpha) log_alpha = reinterpret_cast<const float *>(ws + L.p_g);
        if (retention) retention = reinterpret_cast<const float *>(ws + L.p_r);
        dq = ws + L.p_dq; dk = ws + L.p_dk; dv = ws + L.p_dv;
        dbeta = reinterpret_cast<float *>(ws + L.p_dbeta);
        dlog_alpha = reinterpret_cast<float *>(ws + L.p_dg);
        dretention = reinterpret_cast<float *>(ws + L.p_dr);
        p = &padded;
    }
    auto finish = [&]() -> int {
        if (ragged) {
            auto cut = [&](const void *src, void *dst, size_t row) { return move(src, dst, row, false); };
            if (cut(dq, dq_user, rk_) != 0 || cut(dk, dk_user, rk_) != 0 || cut(dv, dv_user, rv_) != 0 ||
                cut(dbeta, dbeta_user, rg_) != 0 || (log_alpha && cut(dlog_alpha, dg_user, p->gate_per_channel ? rg_ * p->K : rg_) != 0) ||
                (retention && cut(dretention, dr_user, p->retention_per_channel ? rg_ * p->K : rg_) != 0))
                return OSDN_ERR_SHAPE;
        }
        return launch_status();
    };

    ChunkArgs c = chunk_args(p, L, ws);
    c.q = q; c.k = k; c.v = v; c.beta = beta; c.log_alpha = log_alpha;
    c.dO = dO; c.dS_out = dS_out;
    c.Tm = ws + L.Tm; c.Pm = ws + L.Pm; c.dEt = ws + L.dEt; c.dS_ckpt = ws + L.dS_ckpt;
    c.dS_in = dS_in; c.dq = dq; c.dv = dv;
    c.dk_read = ws + L.dk_read;
    c.dkt = ws + L.dkt;
    c.dbeta = dbeta; c.dlog_alpha = log_alpha ? dlog_alpha : nullptr;
    c.n_seqs = pk.n_seqs; c.seq_chunks = seq_chunks; c.dS_last = dS_out;
    // one state gate per key channel: phase 2 runs ungated on the folded operands the forward
    // pass left (Gamma . Q, Gamma . K, K~ / Gamma) and the unfold kernel maps its gradients back
    const bool gv = p->gate_per_channel != 0;
    UnfoldArgs un{};
    if (gv) {
        un.B = p->B; un.T = p->T; un.H = p->H; un.K = p->K; un.N = p->T / C;
        un.log_alpha = log_alpha; un.q = q; un.k = k; un.kt = c.kt;
        un.dq = dq; un.dk_read = c.dk_read; un.dkt = c.dkt;
        un.gamC = reinterpret_cast<const float *>(ws + L.gamC);
        un.dgamC = reinterpret_cast<const float *>(ws + L.dgamC);
        un.dlog_alpha = dlog_alpha;
        c.gate_vec = 1;
        c.q = ws + L.Qg; c.k = ws + L.Kg; c.kt = ws + L.Kd;
        c.log_alpha = nullptr; c.dlog_alpha = nullptr;
        c.gamC = reinterpret_cast<float *>(ws + L.gamC); c.dgamC = reinterpret_cast<float *>(ws + L.dgamC);
    }
    PrecondBwdArgs pb{};
    pb.B = p->B; pb.T = p->T; pb.H = p->H; pb.K = p->K;
    pb.eta = p->eta; pb.d_min = p->d_min; pb.d_max = p->d_max; pb.eps = p->eps;
    pb.beta_aware = p->beta_aware;
    pb.ret_vec = p->retention_per_channel;
    pb.k = k; pb.beta = beta; pb.retention = retention;
    pb.d_ckpt = reinterpret_cast<const float *>(ws + L.d_ckpt);
    pb.tok_scalars = reinterpret_cast<float *>(ws + L.tok_scalars);
    pb.masks = reinterpret_cast<uint2 *>(ws + L.masks);
    pb.a_ckpt = reinterpret_cast<float *>(ws + L.a_ckpt);
    pb.dkt = c.dkt; pb.dk_read = c.dk_read;
    pb.n_seqs = pk.n_seqs; pb.seq_chunks = seq_chunks; pb.dd_last = dd_out;
    pb.dk = dk; pb.dbeta = dbeta; pb.dretention = retention ? dretention : nullptr; pb.dd_in = dd_in;
    // Without retention, chunks that never met the box can take the solved form of the reverse
    // sweep: a dependent chain less than half as long for about 0.6 KB more memory traffic per
    // token-head.  It pays while the phase-1 chain is what the pass waits for: chains on at most a
    // quarter of the CUs (measured at 64 chains: 3 % of forward + backward; with more chains the
    // chains fill the chip by themselves and the pass is bound by its memory traffic).  With fp32
    // I/O the inverses are twice the size and the form stops paying earlier: an eighth of the CUs.
    const long long chains_all = (long long)(pk.n_seqs ? pk.n_seqs : p->B) * p->H;
    const bool general = retention && !p->retention_per_channel;      // the form with a retention gate and any masks
    const bool solved = general ? p->p1_solved > 0
                                : !retention && (p->p1_solved > 0 || (p->p1_solved == 0 && chains_all * (bf ? 4 : 8) <= NUM_CU));
    if (solved) {
        pb.lin_clean = reinterpret_cast<int *>(ws + L.lin_clean);
        pb.lin_M = ws + L.lin_M;
        pb.lin_r0 = reinterpret_cast<float *>(ws + L.lin_r0);
        pb.lin_t0 = reinterpret_cast<float *>(ws + L.lin_t0);
        pb.lin_aux = reinterpret_cast<unsigned char *>(ws + L.lin_aux);
    }

    const int N = p->T / C;
    const long long chains = (long long)(pk.n_seqs ? pk.n_seqs : p->B) * p->H;
    int S = segment_count(p->segments, N, pk.longest, chains * (p->V / 32) + chains, true, chains);   // chain kernel: 32 rows of the state per workgroup
    // (the backward chain keeps slices of 32 values: with 16 the kernel itself is a fifth faster on
    // few chains, but its workgroups then hold twice the CUs and what they take from the phase-1
    // chain beside them, which bounds the pass there, costs more.  The exception is fp32 I/O at
    // K = 128, where the wide slice does not fit the registers: 131 spilled against 19.)
    c.narrow_slices = !bf && p->K == 128;
    Pipeline *pl = S > 1 ? pipeline_for(st) : nullptr;
    if (!pl) S = 1;
    auto seg_range = [&](int sidx, int &n0, int &n1) { n0 = seg_begin(N, S, sidx); n1 = seg_begin(N, S, sidx + 1); };
    auto phase2 = [&](int kid, int sidx) {
        seg_range(sidx, c.n0, c.n1);
        c.dS_out = sidx == S - 1 ? dS_out : dS_in;   // dS is carried in dS_in
        const int rc2 = timed(kid, st, [&] {
            return kid == KID_BWD_CHAIN ? launch_bwd_chain(c, bf, st) : launch_bwd_post(c, bf, st);
        });
        if (rc2 != 0 || !gv || kid != KID_BWD_POST) return rc2;
        un.n0 = c.n0; un.n1 = c.n1;                    // the segment's gradients, back to q, k, k~ and log alpha
        return timed(KID_UNFOLD, st, [&] { return launch_unfold(un, bf, st); });
    };
    // the box masks depend on the forward pass only: one launch for the whole sequence, up front
    auto masks = [&](hipStream_t s1) {
        pb.n0 = 0; pb.n1 = N;
        if (pb.d_min > pb.d_max || pb.lin_clean) return 0;      // (the solved form's first kernel writes them itself)
        return timed(KID_PRECOND_MASK, s1, [&] { return launch_precond_mask(pb, bf, s1); });
    };
    // solved form: which of the chunks [n0, n1) take it, and their inverses (forward data and the masks only)
    auto lin_m = [&](int n0, int n1, hipStream_t s1) {
        if (!pb.lin_clean) return 0;
        pb.n0 = n0; pb.n1 = n1;
        return timed(KID_PRECOND_LIN, s1, [&] { return general ? launch_precond_gen(pb, bf, 0, s1) : launch_precond_lin_bwd(pb, bf, true, s1); });
    };
    // solved form: what its chunks need from dk~ (rho0, the sums of lambda)
    auto lin_r = [&](int sidx, hipStream_t s1) {
        if (!pb.lin_clean) return 0;
        seg_range(sidx, pb.n0, pb.n1);
        return timed(KID_PRECOND_LIN, s1, [&] { return general ? launch_precond_gen(pb, bf, 1, s1) : launch_precond_lin_bwd(pb, bf, false, s1); });
    };
    auto phase1 = [&](int sidx, hipStream_t s1) {
        seg_range(sidx, pb.n0, pb.n1);
        pb.dd_out = sidx == S - 1 ? dd_out : dd_in;  // the adjoint of d is carried in dd_in
        if (timed(KID_PRECOND_CHAIN, s1, [&] { return (general && pb.lin_clean) ? launch_precond_gen(pb, bf, 2, s1) : launch_precond_chain(pb, bf, s1); }) != 0) return -1;
        return timed(KID_PRECOND_POST, s1, [&] { return launch_precond_post(pb, bf, s1); });
    };
    if (!pl) {
        if (phase2(KID_BWD_CHAIN, 0) != 0 || phase2(KID_BWD_POST, 0) != 0 ||
            masks(st) != 0 || lin_m(0, N, st) != 0 || lin_r(0, st) != 0 || phase1(0, st) != 0)
            return OSDN_ERR_SHAPE;
        return finish();
    }
    // main: phase 2, segments right to left          (a[s]: phase 2 of segment s done)
    // side: the masks at once, then phase 1 of segment s once a[s] has fired; joined back at the end
    // The small kernels of the solved form go where they find CUs: when the workgroups of bwd_chain
    // fill the chip (they share a CU with nothing), a kernel on the side stream that becomes ready
    // while bwd_chain runs waits until that is through, and the phase-1 chain behind it waits too.
    // Then the inverses of the first segment are built on the side stream at once (beside
    // bwd_post), and everything else runs on the caller's stream behind the segment's bwd_post,
    // where the phase-1 chain of the segment before covers it.
    const bool lin_on_main = pb.lin_clean && chains * (p->V / 32) + chains > NUM_CU;
    hipStream_t s1 = pl->side;
    OSDN_HIP_OK(hipEventRecord(pl->fork, st));
    OSDN_HIP_OK(hipStreamWaitEvent(s1, pl->fork, 0));
    SideJoin rejoin{pl, st, true};
    if (masks(s1) != 0) return OSDN_ERR_SHAPE;
    if (lin_on_main) {
        OSDN_HIP_OK(hipEventRecord(pl->early[0], s1));               // the masks are there
        if (lin_m(seg_begin(N, S, S - 1), N, s1) != 0) return OSDN_ERR_SHAPE;
        OSDN_HIP_OK(hipEventRecord(pl->early[1], s1));               // ... and the first segment's inverses
    } else if (lin_m(0, N, s1) != 0) {
        return OSDN_ERR_SHAPE;
    }
    for (int s = S - 1; s >= 0; --s) {
        if (phase2(KID_BWD_CHAIN, s) != 0 || phase2(KID_BWD_POST, s) != 0)
            return OSDN_ERR_SHAPE;
        if (lin_on_main) {
            OSDN_HIP_OK(hipStreamWaitEvent(st, pl->early[s == S - 1 ? 1 : 0], 0));
            if (s < S - 1 && lin_m(seg_begin(N, S, s), seg_begin(N, S, s + 1), st) != 0) return OSDN_ERR_SHAPE;
            if (lin_r(s, st) != 0) return OSDN_ERR_SHAPE;
        }
        OSDN_HIP_OK(hipEventRecord(pl->a[s], st));
    }
    for (int s = S - 1; s >= 0; --s) {
        OSDN_HIP_OK(hipStreamWaitEvent(s1, pl->a[s], 0));
        if (!lin_on_main && lin_r(s, s1) != 0) return OSDN_ERR_SHAPE;
        if (phase1(s, s1) != 0) return OSDN_ERR_SHAPE;
    }
    OSDN_HIP_OK(hipEventRecord(pl->join, s1));
    OSDN_HIP_OK(hipStreamWaitEvent(st, pl->join, 0));
    rejoin.armed = false;
    return finish();
}

int osdn_fwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             void *o, float *S_out, float *d_out, void *workspace, size_t workspace_bytes,
             void *stream) {
    return fwd_impl(p, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, nullptr, 0, workspace,
                    workspace_bytes, stream);
}

int osdn_fwd_noalloc(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                     const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                     void *o, float *S_out, float *d_out, void *stream) {
    int rc = check_params(p, true);
    if (rc != OSDN_OK) return rc;
    // everything on the caller's stream: no side stream or event is ever created from here
    osdn_params one = *p;
    one.segments = 1;
    Packing pk;
    plain_packing(&one, pk);
    if (make_layout(&one, pk).total_fwd > STATIC_SCRATCH_BYTES) return OSDN_ERR_WORKSPACE;
    void *scratch = static_scratch_for_current_device();
    if (!scratch) return OSDN_ERR_LAUNCH;
    return fwd_impl(&one, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, nullptr, 0, scratch,
                    STATIC_SCRATCH_BYTES, stream);
}

int osdn_fwd_packed(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                    const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                    void *o, float *S_out, float *d_out, const int32_t *cu_seqlens, int32_t n_seqs,
                    void *workspace, size_t workspace_bytes, void *stream) {
    if (!cu_seqlens) return OSDN_ERR_NULL;
    return fwd_impl(p, q, k, v, beta, log_alpha, retention, d_in, S_in, o, S_out, d_out, cu_seqlens, n_seqs,
                    workspace, workspace_bytes, stream);
}

int osdn_bwd(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
             const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
             const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
             float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
             void *workspace, size_t workspace_bytes, void *stream) {
    return bwd_impl(p, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out, dq, dk, dv, dbeta,
                    dlog_alpha, dretention, dd_in, dS_in, nullptr, 0, workspace, workspace_bytes, stream);
}

int osdn_bwd_packed(const osdn_params *p, const void *q, const void *k, const void *v, const float *beta,
                    const float *log_alpha, const float *retention, const float *d_in, const float *S_in,
                    const void *dO, const float *dS_out, const float *dd_out, void *dq, void *dk, void *dv,
                    float *dbeta, float *dlog_alpha, float *dretention, float *dd_in, float *dS_in,
                    const int32_t *cu_seqlens, int32_t n_seqs, void *workspace, size_t workspace_bytes,
                    void *stream) {
    if (!cu_seqlens) return OSDN_ERR_NULL;
    return bwd_impl(p, q, k, v, beta, log_alpha, retention, d_in, S_in, dO, dS_out, dd_out, dq, dk, dv, dbeta,
                    dlog_alpha, dretention, dd_in, dS_in, cu_seqlens, n_seqs, workspace, workspace_bytes, stream);
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
