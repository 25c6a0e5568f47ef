// The C ABI of include/la.h: argument checks, the segment schedule, workspace
// carving and kernel launches.  No allocation, no synchronisation, no retained
// pointers.
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

#include <mutex>
#include <new>
#include <vector>

#include "../../include/la.h"
#include "la_launch.h"

namespace {

constexpr int kVersion = 401;   // 0.4.1

// ---- schedule ---------------------------------------------------------------------------------
// One wavefront (forward) or one two-wave workgroup (backward) walks one segment of one
// sequence.  MI355X holds 256 CUs x 4 SIMDs x 2 such waves; a sequence is cut into segments
// only as far as needed to reach that many waves, never into segments shorter than a couple of
// chunks, and not at all once the sequences alone fill half the machine.
struct Plan {
    int nchunks, nseg, cps;
    bool fold;      // few segments per sequence: no scan launch, every pass adds up the
                    // segment totals before (after) its own segment itself
};

int env_int(const char *name, int dflt) {
    const char *s = getenv(name);
    if (s == nullptr || *s == '\0') return dflt;
    const long v = strtol(s, nullptr, 10);
    return v > 0 && v < (1 << 24) ? (int)v : dflt;
}

// The schedule's knobs.  The environment is read once, at the first call that needs a value (and
// again only on la_tuning_reload): a workspace query and the calls that use the workspace then see
// the same values, and no entry point calls getenv while another thread changes the environment.
struct Tuning {
    int target_waves;   // LA_TARGET_WAVES
    int min_chunks;     // LA_MIN_SEG_CHUNKS
    int fold_max;       // LA_FOLD_MAX_SEGS
    int bwd_group;      // LA_BWD_SEG_GROUP, 0 = by head size
    int stream;         // LA_STREAM_LOADS: 0, 1, or -1 = by tensor size
};

std::mutex g_tuning_mu;
Tuning g_tuning;
bool g_tuning_read = false;

Tuning read_tuning() {
    Tuning t;
    t.target_waves = env_int("LA_TARGET_WAVES", 2048);
    t.min_chunks = env_int("LA_MIN_SEG_CHUNKS", 2);
    t.fold_max = env_int("LA_FOLD_MAX_SEGS", 8);
    t.bwd_group = env_int("LA_BWD_SEG_GROUP", 0);
    const char *s = getenv("LA_STREAM_LOADS");
    t.stream = (s != nullptr && (s[0] == '0' || s[0] == '1') && s[1] == '\0') ? s[0] - '0' : -1;
    return t;
}

Tuning tuning() {
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    if (!g_tuning_read) {
        g_tuning = read_tuning();
        g_tuning_read = true;
    }
    return g_tuning;
}

Plan make_plan(long BH, int N) {
    const Tuning tn = tuning();
    const int target_waves = tn.target_waves;
    const int min_chunks = tn.min_chunks;
    Plan p;
    p.nchunks = (N + la::kChunk - 1) / la::kChunk;
    long want = (target_waves + BH - 1) / BH;
    long maxseg = p.nchunks / min_chunks;
    if (maxseg < 1) maxseg = 1;
    long nseg = want < 1 ? 1 : (want > maxseg ? maxseg : want);
    // Cutting costs a second sweep over K, V (and Q, dO) plus the scan: measured on MI355X it
    // pays from four segments per sequence on; with half the target already there, don't cut.
    if (2 * BH >= target_waves) nseg = 1;
    p.cps = (int)((p.nchunks + nseg - 1) / nseg);
    p.nseg = (p.nchunks + p.cps - 1) / p.cps;
    p.fold = p.nseg > 1 && p.nseg <= tn.fold_max;
    return p;
}

// How many of the forward's segments one workgroup of the backward takes.  The backward's kernels
// run two waves per workgroup; with a 64-wide head dimension they need so many registers that
// two waves fill a SIMD, half as many workgroups fill the machine, and taking the segments in
// pairs is 10 % faster.  At D = M = 32 four waves fit a SIMD and the finer cut wins.
int backward_group(int C, int M) {
    const int g = tuning().bwd_group;
    if (g == 0) return (C == 32 && M == 32) ? 1 : 2;
    return g == 1 ? 1 : 2;
}

// Whether a call fetches its tiles with non-temporal loads.  A step sweeps Q, K, V (and dO) several
// times, one kernel after the other.  Where those tensors fit the last-level cache (256 MB) the
// later sweeps find them there if the loads are plain (measured: MNIST / CIFAR shapes 2 % and 9 %
// faster than with non-temporal loads); where they do not, the two kinds are equally fast for fp32
// tensors and plain loads 1.5 % faster for bf16 ones (N = 65536).  So plain loads are the default
// and LA_STREAM_LOADS=1 is there for measuring.  (The outputs are always stored non-temporally and
// the segment states always loaded plain.)
int stream_loads() {
    return tuning().stream == 1 ? 1 : 0;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t esize(la_dtype t) { return (t == LA_BF16 || t == LA_BF16_FEATURES) ? 2 : 4; }

size_t states_bytes(long BH, const Plan &p, int D, int M) {
    return align256((size_t)BH * p.nseg * la::state_stride(D, M) * sizeof(float));
}

// Feature width C of Q and K inside the kernels: D itself, or D^2 for the degree-2 polynomial
// map (section 3.2), whose Q and K hold D = 8 raw values per token.
int feat_width(int D, la_dtype t) { return t == LA_F32_POLY2 ? D * D : D; }

int check_dims(int B, int H, int N, int D, int M, float eps, la_dtype t) {
    if (t != LA_F32 && t != LA_BF16 && t != LA_F32_FEATURES && t != LA_BF16_FEATURES && t != LA_F32_POLY2)
        return LA_ERR_UNSUPPORTED;
    if (t == LA_F32_POLY2) {
        if (!(D == 8 && (M == 32 || M == 64))) return LA_ERR_UNSUPPORTED;
    } else if (!((D == 32 || D == 64) && (M == 32 || M == 64))) {
        return LA_ERR_UNSUPPORTED;
    }
    if (B < 1 || H < 1 || N < 1) return LA_ERR_SHAPE;
    if (!(eps >= 0.0f) || !isfinite(eps)) return LA_ERR_SHAPE;
    const double elems = (double)B * H * (double)N * (D > M ? D : M);
    if (elems >= 1099511627776.0) return LA_ERR_SHAPE;                 // 2^40
    if ((double)B * H >= 1048576.0) return LA_ERR_SHAPE;               // grid size stays in int
    return LA_OK;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

// Aliasing: no buffer that a call writes may overlap any other buffer of the call.
struct Span {
    const void *p;
    size_t bytes;
};
bool overlap(const Span &a, const Span &b) {
    if (a.p == nullptr || b.p == nullptr || a.bytes == 0 || b.bytes == 0) return false;
    const uintptr_t x = reinterpret_cast<uintptr_t>(a.p), y = reinterpret_cast<uintptr_t>(b.p);
    return x < y + b.bytes && y < x + a.bytes;
}
// outs: written (or read and written); ins: read only
template <size_t NO, size_t NI>
bool aliased(const Span (&outs)[NO], const Span (&ins)[NI]) {
    for (size_t i = 0; i < NO; ++i) {
        for (size_t j = i + 1; j < NO; ++j)
            if (overlap(outs[i], outs[j])) return true;
        for (size_t j = 0; j < NI; ++j)
            if (overlap(outs[i], ins[j])) return true;
    }
    return false;
}

struct Carver {
    char *base;
    size_t off;
    void *take(size_t bytes) {
        void *p = base + off;
        off += align256(bytes);
        return p;
    }
};

int hip_status(hipError_t e) { return e == hipSuccess ? LA_OK : LA_ERR_HIP; }

// ---- built-in scratch of la_causal_fwd_noalloc --------------------------------------------------
// Device memory that belongs to the library's code object: every GPU the library runs on holds
// its own copy at its own address from the moment the code object is loaded there until the
// process ends.  In host code the array's name is only a stand-in for those copies; the address
// on the current device comes from hipGetSymbolAddress, once per device, and is what the
// kernels are handed.
constexpr size_t kScratchBytes = (size_t)40 << 20;       // 40 MiB
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};                    // guarded by g_scratch_mu

int scratch_on_current_device(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LA_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_scratch_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr)
            return LA_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return LA_OK;
}

// ---- optional profiling hook: HIP events around selected launches ----------------------------
// The state lives in an object the caller owns (la_profile_create); la_profile_begin attaches it
// to the calling thread, and only launches made by that thread are bracketed.  No process-wide
// state, no lock.
struct ProfRec {
    int kid;
    hipEvent_t a, b;
};
}  // namespace

struct la_profile {
    unsigned mask = 0;
    std::vector<ProfRec> recs;
    std::vector<hipEvent_t> pool;
    hipEvent_t event() {
        if (!pool.empty()) {
            hipEvent_t e = pool.back();
            pool.pop_back();
            return e;
        }
        hipEvent_t e = nullptr;
        if (hipEventCreate(&e) != hipSuccess) return nullptr;
        return e;
    }
};

namespace {
thread_local la_profile *t_profile = nullptr;
constexpr size_t kProfMaxRecs = 8192;

// Brackets one launch when its kernel is selected; otherwise one thread-local load.
struct ProfScope {
    hipEvent_t stop = nullptr;
    hipStream_t s;
    ProfScope(int kid, hipStream_t stream) : s(stream) {
        la_profile *p = t_profile;
        if (p == nullptr || (p->mask & (1u << kid)) == 0 || p->recs.size() >= kProfMaxRecs) return;
        hipEvent_t a = p->event(), b = p->event();
        if (a == nullptr || b == nullptr) return;
        if (hipEventRecord(a, s) != hipSuccess) return;
        p->recs.push_back({kid, a, b});
        stop = b;
    }
    ~ProfScope() {
        if (stop != nullptr) (void)hipEventRecord(stop, s);
    }
};

#define LA_TRY(expr)                          \
    do {                                      \
        const int st_ = hip_status(expr);     \
        if (st_ != LA_OK) return st_;         \
    } while (0)

// forward on already-validated arguments; `states` holds states_bytes() when p.nseg > 1
// heads / tok_heads: the layout of the [., N, .] tensors (see la::PassArgs); 0, 0 = [B, H, N, .]
int run_causal_fwd(const void *Q, const void *K, const void *V, void *O, float *den, long BH, int N,
                   int D, int M, float eps, la_dtype t, const Plan &p, float *states,
                   hipStream_t s, const float *S0 = nullptr, const float *z0 = nullptr,
                   float *S1 = nullptr, float *z1 = nullptr, int heads = 0, int tok_heads = 0) {
    const int nblocks = (int)(BH * p.nseg);
    const int nt_loads = stream_loads();
    if (p.nseg > 1) {
        la::SegArgs sa{};
        sa.stream = nt_loads;
        sa.Y = K; sa.Z = V; sa.state = states;
        sa.N = N; sa.nseg = p.nseg; sa.chunks_per_seg = p.cps; sa.skip_seg = p.nseg - 1;
        sa.heads = heads; sa.tok_heads = tok_heads;
        { ProfScope ps(LA_K_SEG_KV, s); LA_TRY(la::launch_segment_state(D, M, (int)t, sa, nblocks, s)); }
        if (!p.fold)
            { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(states, (int)BH, p.nseg, la::state_stride(D, M), la::kScanForward, s, S0, z0, D * M)); }
    }
    const bool scanned = p.nseg > 1 && !p.fold;      // the scan has added the caller's state already
    la::PassArgs a{};
    a.stream = nt_loads;
    a.heads = heads; a.tok_heads = tok_heads;
    a.Q = Q; a.K = K; a.V = V; a.G = nullptr; a.rden = nullptr; a.delta = nullptr;
    a.out = O; a.den = den; a.state = p.nseg > 1 ? states : nullptr; a.fold = p.fold;
    a.init_S = scanned ? nullptr : S0; a.init_z = scanned ? nullptr : z0; a.final_S = S1; a.final_z = z1;
    a.N = N; a.nseg = p.nseg; a.chunks_per_seg = p.cps; a.eps = eps;
    { ProfScope ps(LA_K_FWD, s); LA_TRY(la::launch_pass_fwd(false, D, M, (int)t, a, nblocks, s)); }
    return LA_OK;
}

// eq. 5-6: the K, V grand total (left in slot 0 of `states`), then the read-out
int run_global_fwd(const void *Q, const void *K, const void *V, void *O, float *den, long BH,
                   int N, int D, int M, float eps, la_dtype t, const Plan &p, float *states,
                   hipStream_t s, int heads = 0, int tok_heads = 0) {
    const int nblocks = (int)(BH * p.nseg);
    const int nt_loads = stream_loads();
    la::SegArgs sa{};
    sa.stream = nt_loads;
    sa.heads = heads; sa.tok_heads = tok_heads;
    sa.Y = K; sa.Z = V; sa.state = states;
    sa.N = N; sa.nseg = p.nseg; sa.chunks_per_seg = p.cps; sa.skip_seg = -1;
    { ProfScope ps(LA_K_SEG_KV, s); LA_TRY(la::launch_segment_state(D, M, (int)t, sa, nblocks, s)); }
    if (p.nseg > 1 && !p.fold)
        { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(states, (int)BH, p.nseg, la::state_stride(D, M), la::kScanTotal, s)); }
    la::PassArgs a{};
    a.stream = nt_loads;
    a.heads = heads; a.tok_heads = tok_heads;
    a.Q = Q; a.K = K; a.V = V; a.out = O; a.den = den; a.state = states; a.fold = p.fold;
    a.N = N; a.nseg = p.nseg; a.chunks_per_seg = p.cps; a.eps = eps;
    { ProfScope ps(LA_K_GLOBAL, s); LA_TRY(la::launch_pass_fwd(true, D, M, (int)t, a, nblocks, s)); }
    return LA_OK;
}
}  // namespace

extern "C" {

const char *la_status_string(int status) {
    switch (status) {
        case LA_OK: return "ok";
        case LA_ERR_NULL: return "a required pointer is NULL";
        case LA_ERR_SHAPE: return "invalid size (B, H, N must be >= 1, eps finite and >= 0, total size < 2^40)";
        case LA_ERR_UNSUPPORTED: return "unsupported D, M (each must be 32 or 64) or dtype";
        case LA_ERR_WORKSPACE: return "workspace is NULL or smaller than the workspace query";
        case LA_ERR_HIP: return "a HIP call or kernel launch failed";
        case LA_ERR_ALIGN: return "a tensor pointer is not 16-byte aligned";
        case LA_ERR_ALIAS: return "an output or workspace buffer overlaps another buffer of the call";
        case LA_ERR_SCRATCH: return "the call needs more scratch memory than the library's built-in array holds";
        default: return "unknown status";
    }
}

int la_version(void) { return kVersion; }

void la_tuning_reload(void) {
    const Tuning t = read_tuning();
    std::lock_guard<std::mutex> lock(g_tuning_mu);
    g_tuning = t;
    g_tuning_read = true;
}

size_t la_causal_fwd_workspace(int B, int H, int N, int D, int M, la_dtype t) {
    if (check_dims(B, H, N, D, M, 0.0f, t) != LA_OK) return 0;
    const int C = feat_width(D, t);
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    return p.nseg > 1 ? states_bytes(BH, p, C, M) : 0;
}

size_t la_causal_bwd_workspace(int B, int H, int N, int D, int M, la_dtype t) {
    if (check_dims(B, H, N, D, M, 0.0f, t) != LA_OK) return 0;
    const int C = feat_width(D, t);
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t rows = (size_t)BH * N;
    size_t bytes = 3 * align256(rows * sizeof(float));      // 1/den, delta, and den if it is recomputed
    if (p.nseg > 1) bytes += 2 * states_bytes(BH, p, C, M); // S and R states
    (void)t;
    return bytes;
}

size_t la_global_fwd_workspace(int B, int H, int N, int D, int M, la_dtype t) {
    if (check_dims(B, H, N, D, M, 0.0f, t) != LA_OK) return 0;
    const int C = feat_width(D, t);
    const long BH = (long)B * H;
    return states_bytes(BH, make_plan(BH, N), C, M);
}

size_t la_global_bwd_workspace(int B, int H, int N, int D, int M, la_dtype t) {
    if (check_dims(B, H, N, D, M, 0.0f, t) != LA_OK) return 0;
    const int C = feat_width(D, t);
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t rows = (size_t)BH * N;
    size_t bytes = 2 * states_bytes(BH, p, C, M);           // the two grand totals
    bytes += align256(rows * sizeof(float));                // den if it is recomputed
    (void)t;
    return bytes;
}

static int causal_fwd_impl(const void *Q, const void *K, const void *V, void *O, float *den,
                           int B, int H, int N, int D, int M, float eps, la_dtype t,
                           void *ws, size_t ws_bytes, void *stream, int tok_heads) {
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(ws))
        return LA_ERR_ALIGN;
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t need = p.nseg > 1 ? states_bytes(BH, p, C, M) : 0;
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return LA_ERR_WORKSPACE;
    const size_t rows = (size_t)BH * N, e = esize(t);
    const Span outs[] = {{O, rows * M * e}, {den, rows * 4}, {ws, need}};
    const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e}};
    if (aliased(outs, ins)) return LA_ERR_ALIAS;
    return run_causal_fwd(Q, K, V, O, den, BH, N, C, M, eps, t, p, static_cast<float *>(ws),
                          static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, nullptr, H,
                          tok_heads);
}

int la_causal_fwd(const void *Q, const void *K, const void *V, void *O, float *den,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream) {
    return causal_fwd_impl(Q, K, V, O, den, B, H, N, D, M, eps, t, ws, ws_bytes, stream, 0);
}

int la_causal_fwd_bnhd(const void *Q, const void *K, const void *V, void *O, float *den,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream) {
    return causal_fwd_impl(Q, K, V, O, den, B, H, N, D, M, eps, t, ws, ws_bytes, stream,
                           H > 1 ? H : 0);
}

int la_causal_fwd_noalloc(const void *Q, const void *K, const void *V, void *O, float *den,
                          int B, int H, int N, int D, int M, float eps, la_dtype t, void *stream) {
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O)) return LA_ERR_ALIGN;
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t need = p.nseg > 1 ? states_bytes(BH, p, C, M) : 0;
    if (need > kScratchBytes) return LA_ERR_SCRATCH;
    const size_t rows = (size_t)BH * N, e = esize(t);
    const Span outs[] = {{O, rows * M * e}, {den, rows * 4}};
    const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e}};
    if (aliased(outs, ins)) return LA_ERR_ALIAS;
    void *states = nullptr;
    if (need > 0) {
        // the states are written (segment sums), scanned and read within this call: nothing in
        // the array has to start at zero, whatever the call before left there
        const int ss = scratch_on_current_device(&states);
        if (ss != LA_OK) return ss;
    }
    return run_causal_fwd(Q, K, V, O, den, BH, N, C, M, eps, t, p, static_cast<float *>(states),
                          static_cast<hipStream_t>(stream), nullptr, nullptr, nullptr, nullptr, H, 0);
}

static int causal_fwd_state_impl(const void *Q, const void *K, const void *V, const float *S0,
                                 const float *z0, void *O, float *den, float *S1, float *z1,
                                 int B, int H, int N, int D, int M, float eps, la_dtype t,
                                 void *ws, size_t ws_bytes, void *stream, int tok_heads) {
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return LA_ERR_NULL;
    if ((S0 == nullptr) != (z0 == nullptr) || (S1 == nullptr) != (z1 == nullptr)) return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(ws) ||
        misaligned(S0) || misaligned(z0) || misaligned(S1) || misaligned(z1))
        return LA_ERR_ALIGN;
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t need = p.nseg > 1 ? states_bytes(BH, p, C, M) : 0;
    if (need > 0 && (ws == nullptr || ws_bytes < need)) return LA_ERR_WORKSPACE;
    const size_t rows = (size_t)BH * N, e = esize(t);
    const Span outs[] = {{O, rows * M * e}, {den, rows * 4}, {ws, need},
                         {S1, (size_t)BH * C * M * 4}, {z1, (size_t)BH * C * 4}};
    const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e},
                        {S0, (size_t)BH * C * M * 4}, {z0, (size_t)BH * C * 4}};
    if (aliased(outs, ins)) return LA_ERR_ALIAS;
    return run_causal_fwd(Q, K, V, O, den, BH, N, C, M, eps, t, p, static_cast<float *>(ws),
                          static_cast<hipStream_t>(stream), S0, z0, S1, z1, H, tok_heads);
}

int la_causal_fwd_state(const void *Q, const void *K, const void *V, const float *S0,
                        const float *z0, void *O, float *den, float *S1, float *z1,
                        int B, int H, int N, int D, int M, float eps, la_dtype t,
                        void *ws, size_t ws_bytes, void *stream) {
    return causal_fwd_state_impl(Q, K, V, S0, z0, O, den, S1, z1, B, H, N, D, M, eps, t, ws,
                                 ws_bytes, stream, 0);
}

int la_causal_fwd_state_bnhd(const void *Q, const void *K, const void *V, const float *S0,
                             const float *z0, void *O, float *den, float *S1, float *z1,
                             int B, int H, int N, int D, int M, float eps, la_dtype t,
                             void *ws, size_t ws_bytes, void *stream) {
    return causal_fwd_state_impl(Q, K, V, S0, z0, O, den, S1, z1, B, H, N, D, M, eps, t, ws,
                                 ws_bytes, stream, H > 1 ? H : 0);
}

static int causal_bwd_impl(const void *Q, const void *K, const void *V, const float *S0,
                           const float *z0, const void *O, const float *den, const void *fwd_ws,
                           const void *dO, const float *dS1, const float *dz1, void *dQ, void *dK,
                           void *dV, float *dS0, float *dz0, int B, int H, int N, int D, int M,
                           float eps, la_dtype t, void *ws, size_t ws_bytes, void *stream,
                           int tok_heads = 0) {
    if (Q == nullptr || K == nullptr || V == nullptr || dO == nullptr || dQ == nullptr ||
        dK == nullptr || dV == nullptr)
        return LA_ERR_NULL;
    if ((S0 == nullptr) != (z0 == nullptr) || (dS1 == nullptr) != (dz1 == nullptr) ||
        (dS0 == nullptr) != (dz0 == nullptr))
        return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(dO) || misaligned(dQ) ||
        misaligned(dK) || misaligned(dV) || misaligned(O) || misaligned(den) || misaligned(ws) ||
        misaligned(fwd_ws) || misaligned(S0) || misaligned(z0) || misaligned(dS1) ||
        misaligned(dz1) || misaligned(dS0) || misaligned(dz0))
        return LA_ERR_ALIGN;
    const size_t need = la_causal_bwd_workspace(B, H, N, D, M, t);
    if (ws == nullptr || ws_bytes < need) return LA_ERR_WORKSPACE;

    hipStream_t s = static_cast<hipStream_t>(stream);
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t rows = (size_t)BH * N;
    {
        const size_t e = esize(t), sb = (size_t)BH * C * M * 4, zb = (size_t)BH * C * 4;
        const Span outs[] = {{dQ, rows * D * e}, {dK, rows * D * e}, {dV, rows * M * e},
                             {ws, need}, {dS0, sb}, {dz0, zb}};
        const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e},
                            {dO, rows * M * e}, {den, rows * 4}, {S0, sb}, {z0, zb}, {dS1, sb},
                            {dz1, zb}, {fwd_ws, p.nseg > 1 ? states_bytes(BH, p, C, M) : 0}};
        if (aliased(outs, ins)) return LA_ERR_ALIAS;
    }
    const int nt_loads = stream_loads();
    Carver cv{static_cast<char *>(ws), 0};
    float *rden = static_cast<float *>(cv.take(rows * sizeof(float)));
    float *delta = static_cast<float *>(cv.take(rows * sizeof(float)));
    float *stS = nullptr, *stR = nullptr;
    if (p.nseg > 1) {
        stS = static_cast<float *>(cv.take(states_bytes(BH, p, C, M)));
        stR = static_cast<float *>(cv.take(states_bytes(BH, p, C, M)));
    }
    (void)O;                                   // not read: delta is rebuilt from the state
    const bool recompute_fwd = (den == nullptr);
    // the forward's own workspace still holds the prefix states: no need to rebuild them
    const bool have_states = p.nseg > 1 && (fwd_ws != nullptr || recompute_fwd);
    if (p.nseg > 1 && fwd_ws != nullptr && !recompute_fwd)
        stS = const_cast<float *>(static_cast<const float *>(fwd_ws));
    if (recompute_fwd) {                       // recompute the forward's denominators (no output)
        float *dentmp = static_cast<float *>(cv.take(rows * sizeof(float)));
        const int fs = run_causal_fwd(Q, K, V, nullptr, dentmp, BH, N, C, M, eps, t, p, stS, s, S0, z0,
                                      nullptr, nullptr, H, tok_heads);
        if (fs != LA_OK) return fs;
        den = dentmp;
    }
    const int nblocks = (int)(BH * p.nseg);
    if (p.nseg > 1 && !have_states) {
        la::SegArgs sa{};
        sa.stream = nt_loads;
        sa.N = N; sa.nseg = p.nseg; sa.chunks_per_seg = p.cps;
        sa.Y = K; sa.Z = V; sa.state = stS;
        sa.skip_seg = p.nseg - 1;
        sa.heads = H; sa.tok_heads = tok_heads;
        { ProfScope ps(LA_K_SEG_KV, s); LA_TRY(la::launch_segment_state(C, M, (int)t, sa, nblocks, s)); }
        if (!p.fold)
            { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(stS, (int)BH, p.nseg, la::state_stride(C, M), la::kScanForward, s, S0, z0, C * M)); }
    }
    // The two kernels of the backward run two waves per workgroup, so (for 64-wide heads) half as
    // many workgroups fill the machine: they take the forward's segments in pairs, see
    // backward_group.  The prefix states (laid out for the forward's cut) are then read at every
    // second slot.
    const int group = backward_group(C, M);
    Plan pb = p;
    if (p.nseg > 1) {
        pb.cps = group * p.cps;
        pb.nseg = (p.nchunks + pb.cps - 1) / pb.cps;
    }
    const int nblocks_b = (int)(BH * pb.nseg);
    // forward direction: dQ; on the way 1/den and delta per token and, when the sequences
    // are cut, the per-segment sums that the reverse direction starts from
    la::PassArgs a{};
    a.stream = nt_loads;
    a.heads = H; a.tok_heads = tok_heads;
    a.Q = Q; a.K = K; a.V = V; a.G = dO; a.rden = rden; a.delta = delta; a.den = nullptr;
    a.den_in = den; a.rden_out = rden; a.delta_out = delta; a.totals = pb.nseg > 1 ? stR : nullptr;
    a.N = N; a.nseg = pb.nseg; a.chunks_per_seg = pb.cps; a.eps = eps;
    a.out = dQ; a.state = stS; a.state_nseg = p.nseg; a.state_step = group; a.fold = p.fold;
    // the caller's state: the scan has added it to the prefix states already, if there was one
    const bool scanned = p.nseg > 1 && !p.fold;
    a.init_S = scanned ? nullptr : S0; a.init_z = scanned ? nullptr : z0;
    { ProfScope ps(LA_K_DQ, s); LA_TRY(la::launch_pass_dq(true, C, M, (int)t, a, nblocks_b, s)); }
    const bool scanned_b = pb.nseg > 1 && !p.fold;
    if (scanned_b)
        { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(stR, (int)BH, pb.nseg, la::state_stride(C, M), la::kScanReverse, s, dS1, dz1, C * M)); }
    a.out = dV; a.out2 = dK; a.state = pb.nseg > 1 ? stR : nullptr;
    a.state_nseg = 0; a.state_step = 0;      // stR is laid out for this very cut
    a.init_S = scanned_b ? nullptr : dS1; a.init_z = scanned_b ? nullptr : dz1;
    a.final_S = dS0; a.final_z = dz0;
    { ProfScope ps(LA_K_REV, s); LA_TRY(la::launch_pass_reverse(C, M, (int)t, a, nblocks_b, s)); }
    return LA_OK;
}

int la_causal_bwd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                  const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream) {
    return causal_bwd_impl(Q, K, V, nullptr, nullptr, O, den, fwd_ws, dO, nullptr, nullptr, dQ, dK,
                           dV, nullptr, nullptr, B, H, N, D, M, eps, t, ws, ws_bytes, stream);
}

int la_causal_bwd_bnhd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                       const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream) {
    return causal_bwd_impl(Q, K, V, nullptr, nullptr, O, den, fwd_ws, dO, nullptr, nullptr, dQ, dK,
                           dV, nullptr, nullptr, B, H, N, D, M, eps, t, ws, ws_bytes, stream,
                           H > 1 ? H : 0);
}

int la_causal_bwd_state(const void *Q, const void *K, const void *V, const float *S0,
                        const float *z0, const void *O, const float *den, const void *fwd_ws,
                        const void *dO, const float *dS1, const float *dz1, void *dQ, void *dK,
                        void *dV, float *dS0, float *dz0, int B, int H, int N, int D, int M,
                        float eps, la_dtype t, void *ws, size_t ws_bytes, void *stream) {
    return causal_bwd_impl(Q, K, V, S0, z0, O, den, fwd_ws, dO, dS1, dz1, dQ, dK, dV, dS0, dz0, B, H,
                           N, D, M, eps, t, ws, ws_bytes, stream);
}

int la_causal_bwd_state_bnhd(const void *Q, const void *K, const void *V, const float *S0,
                             const float *z0, const void *O, const float *den, const void *fwd_ws,
                             const void *dO, const float *dS1, const float *dz1, void *dQ, void *dK,
                             void *dV, float *dS0, float *dz0, int B, int H, int N, int D, int M,
                             float eps, la_dtype t, void *ws, size_t ws_bytes, void *stream) {
    return causal_bwd_impl(Q, K, V, S0, z0, O, den, fwd_ws, dO, dS1, dz1, dQ, dK, dV, dS0, dz0, B, H,
                           N, D, M, eps, t, ws, ws_bytes, stream, H > 1 ? H : 0);
}

static int global_fwd_impl(const void *Q, const void *K, const void *V, void *O, float *den,
                           int B, int H, int N, int D, int M, float eps, la_dtype t,
                           void *ws, size_t ws_bytes, void *stream, int tok_heads) {
    if (Q == nullptr || K == nullptr || V == nullptr || O == nullptr) return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(O) || misaligned(ws) ||
        misaligned(den))
        return LA_ERR_ALIGN;
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    if (ws == nullptr || ws_bytes < states_bytes(BH, p, C, M)) return LA_ERR_WORKSPACE;
    const size_t rows = (size_t)BH * N, e = esize(t);
    const Span outs[] = {{O, rows * M * e}, {den, rows * 4}, {ws, states_bytes(BH, p, C, M)}};
    const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e}};
    if (aliased(outs, ins)) return LA_ERR_ALIAS;
    return run_global_fwd(Q, K, V, O, den, BH, N, C, M, eps, t, p, static_cast<float *>(ws),
                          static_cast<hipStream_t>(stream), H, tok_heads);
}

int la_global_fwd(const void *Q, const void *K, const void *V, void *O, float *den,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream) {
    return global_fwd_impl(Q, K, V, O, den, B, H, N, D, M, eps, t, ws, ws_bytes, stream, 0);
}

int la_global_fwd_bnhd(const void *Q, const void *K, const void *V, void *O, float *den,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream) {
    return global_fwd_impl(Q, K, V, O, den, B, H, N, D, M, eps, t, ws, ws_bytes, stream,
                           H > 1 ? H : 0);
}

static int global_bwd_impl(const void *Q, const void *K, const void *V, const void *O,
                           const float *den, const void *fwd_ws, const void *dO, void *dQ,
                           void *dK, void *dV, int B, int H, int N, int D, int M, float eps,
                           la_dtype t, void *ws, size_t ws_bytes, void *stream, int tok_heads) {
    if (Q == nullptr || K == nullptr || V == nullptr || dO == nullptr || dQ == nullptr ||
        dK == nullptr || dV == nullptr)
        return LA_ERR_NULL;
    const int st = check_dims(B, H, N, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(Q) || misaligned(K) || misaligned(V) || misaligned(dO) || misaligned(dQ) ||
        misaligned(dK) || misaligned(dV) || misaligned(O) || misaligned(den) || misaligned(ws) ||
        misaligned(fwd_ws))
        return LA_ERR_ALIGN;
    const size_t need = la_global_bwd_workspace(B, H, N, D, M, t);
    if (ws == nullptr || ws_bytes < need) return LA_ERR_WORKSPACE;
    (void)O;                                   // not read: delta is rebuilt from the read-out

    hipStream_t s = static_cast<hipStream_t>(stream);
    const long BH = (long)B * H;
    const Plan p = make_plan(BH, N);
    const size_t rows = (size_t)BH * N;
    {
        const size_t e = esize(t);
        const Span outs[] = {{dQ, rows * D * e}, {dK, rows * D * e}, {dV, rows * M * e}, {ws, need}};
        const Span ins[] = {{Q, rows * D * e}, {K, rows * D * e}, {V, rows * M * e},
                            {dO, rows * M * e}, {den, rows * 4}, {fwd_ws, states_bytes(BH, p, C, M)}};
        if (aliased(outs, ins)) return LA_ERR_ALIAS;
    }
    const int nt_loads = stream_loads();
    Carver cv{static_cast<char *>(ws), 0};
    float *stS = static_cast<float *>(cv.take(states_bytes(BH, p, C, M)));
    float *stR = static_cast<float *>(cv.take(states_bytes(BH, p, C, M)));
    const int nblocks = (int)(BH * p.nseg);
    if (den == nullptr) {                      // recompute the forward's denominators (no output);
        float *dentmp = static_cast<float *>(cv.take(rows * sizeof(float)));   // also leaves the K, V sums in stS
        const int fs = run_global_fwd(Q, K, V, nullptr, dentmp, BH, N, C, M, eps, t, p, stS, s, H,
                                      tok_heads);
        if (fs != LA_OK) return fs;
        den = dentmp;
    } else if (fwd_ws != nullptr) {            // the forward's workspace still holds that total
        stS = const_cast<float *>(static_cast<const float *>(fwd_ws));
    } else {
        la::SegArgs sa{};
        sa.stream = nt_loads;
        sa.heads = H; sa.tok_heads = tok_heads;
        sa.N = N; sa.nseg = p.nseg; sa.chunks_per_seg = p.cps; sa.skip_seg = -1;
        sa.Y = K; sa.Z = V; sa.state = stS;
        { ProfScope ps(LA_K_SEG_KV, s); LA_TRY(la::launch_segment_state(C, M, (int)t, sa, nblocks, s)); }
        if (p.nseg > 1 && !p.fold)
            { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(stS, (int)BH, p.nseg, la::state_stride(C, M), la::kScanTotal, s)); }
    }
    // dQ against the K, V total; on the way the per-segment Q, dO sums.  A kernel with two
    // waves per workgroup: it takes the segments in pairs (see the causal backward).
    Plan pb = p;
    if (p.nseg > 1) {
        pb.cps = backward_group(C, M) * p.cps;
        pb.nseg = (p.nchunks + pb.cps - 1) / pb.cps;
    }
    la::PassArgs a{};
    a.stream = nt_loads;
    a.heads = H; a.tok_heads = tok_heads;
    a.Q = Q; a.K = K; a.V = V; a.G = dO; a.den_in = den; a.totals = stR;
    a.N = N; a.nseg = pb.nseg; a.chunks_per_seg = pb.cps; a.eps = eps;
    a.out = dQ; a.state = stS; a.state_nseg = p.nseg; a.fold = p.fold;
    { ProfScope ps(LA_K_DQ, s); LA_TRY(la::launch_pass_dq(false, C, M, (int)t, a, (int)(BH * pb.nseg), s)); }
    if (pb.nseg > 1 && !p.fold)
        { ProfScope ps(LA_K_SCAN, s); LA_TRY(la::launch_scan(stR, (int)BH, pb.nseg, la::state_stride(C, M), la::kScanTotal, s)); }
    // dV and dK against the Q, dO total: one kernel, two waves per workgroup over the same
    // pairs of segments
    a.totals = nullptr;
    a.state = stR; a.state_nseg = pb.nseg;
    ProfScope ps(LA_K_GLOBAL_BWD, s);
    a.out = dV; a.out2 = dK;
    LA_TRY(la::launch_global_dkdv(C, M, (int)t, a, (int)(BH * pb.nseg), s));
    return LA_OK;
}

int la_global_bwd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                  const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                  int B, int H, int N, int D, int M, float eps, la_dtype t,
                  void *ws, size_t ws_bytes, void *stream) {
    return global_bwd_impl(Q, K, V, O, den, fwd_ws, dO, dQ, dK, dV, B, H, N, D, M, eps, t, ws,
                           ws_bytes, stream, 0);
}

int la_global_bwd_bnhd(const void *Q, const void *K, const void *V, const void *O, const float *den,
                       const void *fwd_ws, const void *dO, void *dQ, void *dK, void *dV,
                       int B, int H, int N, int D, int M, float eps, la_dtype t,
                       void *ws, size_t ws_bytes, void *stream) {
    return global_bwd_impl(Q, K, V, O, den, fwd_ws, dO, dQ, dK, dV, B, H, N, D, M, eps, t, ws,
                           ws_bytes, stream, H > 1 ? H : 0);
}

int la_recurrent_step(const void *q, const void *k, const void *v, float *S, float *z, void *out,
                      int B, int H, int D, int M, float eps, la_dtype t, void *stream) {
    if (q == nullptr || k == nullptr || v == nullptr || S == nullptr || z == nullptr ||
        out == nullptr)
        return LA_ERR_NULL;
    const int st = check_dims(B, H, 1, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(S) || misaligned(z) ||
        misaligned(out))
        return LA_ERR_ALIGN;
    {
        const size_t bh = (size_t)B * H, e = esize(t);
        const Span outs[] = {{out, bh * M * e}, {S, bh * C * M * 4}, {z, bh * C * 4}};
        const Span ins[] = {{q, bh * D * e}, {k, bh * D * e}, {v, bh * M * e}};
        if (aliased(outs, ins)) return LA_ERR_ALIAS;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfScope ps(LA_K_STEP, s);
    LA_TRY(la::launch_recurrent_step(q, k, v, S, z, out, (int)((long)B * H), C, M, eps, (int)t, s));
    return LA_OK;
}

int la_recurrent_steps(const void *q, const void *k, const void *v, float *S, float *z, void *out,
                       int T, int B, int H, int D, int M, float eps, la_dtype t, void *stream) {
    if (q == nullptr || k == nullptr || v == nullptr || S == nullptr || z == nullptr ||
        out == nullptr)
        return LA_ERR_NULL;
    const int st = check_dims(B, H, T, D, M, eps, t);
    if (st != LA_OK) return st;
    const int C = feat_width(D, t);
    if (misaligned(q) || misaligned(k) || misaligned(v) || misaligned(S) || misaligned(z) ||
        misaligned(out))
        return LA_ERR_ALIGN;
    {
        const size_t bh = (size_t)B * H, e = esize(t);
        const Span outs[] = {{out, (size_t)T * bh * M * e}, {S, bh * C * M * 4}, {z, bh * C * 4}};
        const Span ins[] = {{q, (size_t)T * bh * D * e}, {k, (size_t)T * bh * D * e},
                            {v, (size_t)T * bh * M * e}};
        if (aliased(outs, ins)) return LA_ERR_ALIAS;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    ProfScope ps(LA_K_STEP, s);
    LA_TRY(la::launch_recurrent_steps(q, k, v, S, z, out, T, (int)((long)B * H), C, M, eps, (int)t, s));
    return LA_OK;
}

const char *la_kernel_name(int kernel_id) {
    static const char *const names[LA_K_COUNT] = {"segment_state_kv", "scan_states", "causal_pass_fwd",
                                                  "global_readout", "pass_dq", "reverse_pass_dv_dk",
                                                  "recurrent_step", "global_bwd_readouts"};
    return kernel_id >= 0 && kernel_id < LA_K_COUNT ? names[kernel_id] : "unknown";
}

la_profile *la_profile_create(void) { return new (std::nothrow) la_profile(); }

void la_profile_destroy(la_profile *p) {
    if (p == nullptr) return;
    if (t_profile == p) t_profile = nullptr;
    for (const ProfRec &r : p->recs) {
        (void)hipEventDestroy(r.a);
        (void)hipEventDestroy(r.b);
    }
    for (hipEvent_t e : p->pool) (void)hipEventDestroy(e);
    delete p;
}

int la_profile_begin(la_profile *p, unsigned mask) {
    if (p == nullptr) return LA_ERR_NULL;
    for (const ProfRec &r : p->recs) {
        p->pool.push_back(r.a);
        p->pool.push_back(r.b);
    }
    p->recs.clear();
    p->mask = mask & ((1u << LA_K_COUNT) - 1u);
    t_profile = p;
    return LA_OK;
}

int la_profile_end(la_profile *p, float *ms_total, int *launches) {
    if (p == nullptr) return LA_ERR_NULL;
    if (t_profile == p) t_profile = nullptr;
    p->mask = 0;
    int status = LA_OK;
    if (ms_total != nullptr)
        for (int k = 0; k < LA_K_COUNT; ++k) ms_total[k] = 0.f;
    if (launches != nullptr)
        for (int k = 0; k < LA_K_COUNT; ++k) launches[k] = 0;
    for (const ProfRec &r : p->recs) {
        float ms = 0.f;
        if (hipEventSynchronize(r.b) != hipSuccess || hipEventElapsedTime(&ms, r.a, r.b) != hipSuccess) {
            status = LA_ERR_HIP;
        } else {
            if (ms_total != nullptr) ms_total[r.kid] += ms;
            if (launches != nullptr) launches[r.kid] += 1;
        }
        p->pool.push_back(r.a);
        p->pool.push_back(r.b);
    }
    p->recs.clear();
    return status;
}

}  // extern "C"
