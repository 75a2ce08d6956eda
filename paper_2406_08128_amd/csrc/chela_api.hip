// Host side of libchela.so: argument validation, work partitioning, scratch management, dispatch.
// Every check below runs before the first HIP call so that a rejected call has touched nothing.
#include "../../include/chela.h"
#include "../../include/chela_bench.h"
#include "chela_internal.h"
#include <cmath>

#include <cstdlib>
#include <mutex>
#include <vector>

namespace chela {

static int env_int(const char* name, int dflt)
{
    const char* s = std::getenv(name);
    if (!s || !*s) return dflt;
    return std::atoi(s);
}

constexpr long kMaxBwdWalkTokens = 8192;   // longest stretch the bf16 backward walks its state back over

// Workgroups of the sweep kernel that the plan counts on at once (256 compute units x resident workgroups per unit,
// the latter set by the kernel's LDS and register footprint).
static long sweep_slots(int dk, int dv, int chunk, int dtype, bool is_bwd)
{
    const bool narrow = (dk == 64 && dv == 64), wide = (dk == 128 && dv == 128);
    if (dtype != CHELA_DTYPE_BF16) return narrow ? 512 : 256;     // fp32 sweep: 66 KB of LDS at the 64-wide shape, > 80 KB else
    int per_cu;
    if (is_bwd) per_cu = (chunk == 64 && !wide) ? 2 : 1;      // (one width of 128: the two states share an LDS tile)
    // (the 64-wide forward sweep holds four per unit, but is planned for two: filling the other two with shorter
    // segments buys nothing a state more per segment does not cost -- 10 segments instead of 20 at the LM shape took
    // 2.5 % off the step, 5 % at half that length)
    else if (chunk == 64) per_cu = wide ? 1 : 2;
    else per_cu = narrow ? 2 : 1;
    return 256L * per_cu;
}

// Segments per (b,h).  Every extra segment costs HBM traffic (its d_k x d_v fp32 state is written by the pre-pass,
// read and written by the scan and read by the sweep), too few leave compute units idle, and a workgroup count just
// above a multiple of what the GPU holds at once wastes most of a round.  The plan minimises a small cost model, in
// units of one chunk step of one workgroup on a full GPU:
//     sweep  = (full rounds + g(fill of the last round)) * (chunks per segment + 0.5) * (1 + 0.09 (rounds - 1))
//     states = segments * heads * w   (+ 2 when there are too many segments for the sweeps to add the totals up
//                                        themselves: then the scan is a kernel of its own)
// g() says that a sparsely filled last round runs its workgroups faster, but not proportionally (and not at all when
// a compute unit only ever holds one workgroup: then nothing hides that workgroup's latencies); w is the measured
// cost of one more segment state relative to a chunk step.  The factor on several rounds is measured too: at 48
// (b,h) pairs of 32768 and 65536 tokens, one round of 480 long-lived workgroups beat two rounds of 480 by 7 .. 10 %
// and three rounds of 512 by 13 .. 19 %, forward and backward alike (fewer, longer streams; no tail in which the
// last round's stragglers have the GPU to themselves).  Segments longer than max_cps chunks are not considered
// (see make_plan), a single segment always is.  With single_from or more (b,h) pairs one workgroup per pair keeps
// every unit busy and the pre-pass (which re-reads K and V) disappears altogether, so no segmentation is used.
static long choose_segments(long BH, long n_chunks, long slots, double g_min, double w_state, long max_cps,
                            long max_folded_segments, long single_from)
{
    if (BH >= single_from || n_chunks <= 4) return 1;
    long best = 1;
    double best_cost = 1e300;
    // at least 4 chunks per segment -- unless the whole problem fits the GPU at once even with one workgroup per chunk:
    // then the time is the launches plus the serial chunk steps of a segment, and shorter segments only help
    const long min_cps = BH * n_chunks <= slots ? 1 : 4;
    const long max_seg = n_chunks / min_cps > 0 ? n_chunks / min_cps : 1;
    for (long n = 1; n <= max_seg && n <= 4096; ++n) {
        const long cps = (n_chunks + n - 1) / n;
        const long real_n = (n_chunks + cps - 1) / cps;
        if (real_n != n) continue;                                 // same split as a smaller n
        if (n > 1 && max_cps > 0 && cps > max_cps) continue;
        const long wgs = BH * n;
        const long full = wgs / slots;
        const double f = (double)(wgs - full * slots) / (double)slots;
        double g = 0.0;
        if (f > 0.0) { g = f / 0.75; if (g > 1.0) g = 1.0; if (g < g_min) g = g_min; }
        const long rounds = full + (f > 0.0 ? 1 : 0);
        double cost = ((double)full + g) * ((double)cps + 0.5) * (1.0 + 0.09 * (double)(rounds - 1))
                    + (double)(n * BH) * w_state;
        if (n > 1) cost += 0.5 * (double)(n_chunks * BH) / (double)slots + 3.0;   // pre-pass re-read + two more launches
        if (n > 1 && n > max_folded_segments) cost += 2.0;                        // the scan as a kernel of its own
        if (cost < best_cost) { best_cost = cost; best = n; }
    }
    return best;
}

Plan make_plan(long BH, int N, int dk, int dv, int chunk, int dtype, bool is_bwd, bool stateful, bool can_checkpoint)
{
    Plan p{};
    p.chunk = chunk;
    p.state_elems = (size_t)dk * dv;
    if (BH <= 0 || N <= 0) { p.seg_len = chunk; p.n_seg = 0; p.ws_bytes = 0; return p; }
    const long n_chunks = ((long)N + chunk - 1) / chunk;
    const long slots = sweep_slots(dk, dv, chunk, dtype, is_bwd);
    // one more state costs about 48 KB (fp32, 64 x 64) of traffic spread over the whole GPU; a chunk step moves
    // 32 KB (forward) or 56 KB (backward) per resident workgroup
    const double w_state = (is_bwd ? 0.0019 : 0.0033) * ((double)dk * dv / 4096.0) * (512.0 / (double)slots);
    const long max_walk = kMaxBwdWalkTokens / chunk;
    const bool walk_capped = is_bwd && dtype == CHELA_DTYPE_BF16;
    const long max_folded = stateful ? 0 : (long)(kMaxFoldedStateBytes / (p.state_elems * sizeof(float)));
    // A forward workgroup runs faster with fewer neighbours (the GPU's bandwidth is what it shares); a backward
    // workgroup does not: its chunk step took 5.0 .. 5.1 us with 192, 384 and 480 workgroups on the GPU alike
    // (192 sequences of 16384 tokens: one segment each 1307 us, two 839 us).
    // So 256 sequences, one workgroup per unit, still gain from two segments each in the backward (250 sequences of
    // 4096 tokens: 272 us against 337 us), while the forward is at its best there with one.
    const bool lone_is_slow = is_bwd && dtype == CHELA_DTYPE_BF16;
    const double g_min = (slots > 256 && !lone_is_slow) ? 0.55 : 1.0;
    long n_seg = choose_segments(BH, n_chunks, slots, g_min, w_state, walk_capped ? max_walk : 0, max_folded,
                                 lone_is_slow && slots > 256 ? 257 : 256);
    long cps = (n_chunks + n_seg - 1) / n_seg;
    const int forced = env_int("CHELA_SEG_TOKENS", 0);
    if (forced > 0) cps = (forced + chunk - 1) / chunk;
    if (cps > n_chunks) cps = n_chunks;
    if (cps < 1) cps = 1;
    // The bf16 backward sweep enters a segment with the state at the segment's END and walks it back one chunk per
    // step in fp32 (S_{c-1} = S_c - K_c^T V_c).  For states that grow with the position (keys and values with a
    // non-zero mean) the rounding of that walk, relative to the small early states, grows with the length walked to
    // the power 1.5: measured on such data, the worst row of dQ in the first chunk is off by 1e-2 of its norm after
    // 32768 tokens, 2.8e-2 after 65536, 0.23 after 262144, against 4e-3 .. 6e-3 from bf16 rounding alone.  The walk
    // is therefore never longer than kMaxBwdWalkTokens (1.2e-3 by the same law): a single segment whose sweep builds
    // the state itself drops copies of it on the way forward and picks them up on the way back; every other plan
    // gets shorter segments (more states to scan, nothing else).
    if (walk_capped && cps > max_walk) {
        if (cps >= n_chunks && !stateful && can_checkpoint) p.ckpt_every = (int)max_walk;
        else if (forced <= 0) cps = max_walk;
    }
    if ((n_chunks + cps - 1) / cps > 32768) cps = (n_chunks + 32767) / 32768;   // segments ride on grid.y
    p.seg_len = (int)(cps * chunk);
    p.n_seg = (int)((n_chunks + cps - 1) / cps);
    const int n_states = (dtype == CHELA_DTYPE_BF16 && is_bwd) ? 2 : 1;   // fp32 bwd reuses one array 3 times
    // a carried-in state goes through the scan even when there is a single segment
    if (p.n_seg > 1 || stateful) {
        p.ckpt_every = 0;
        p.ws_bytes = (size_t)BH * p.n_seg * p.state_elems * sizeof(float) * n_states;
    } else {
        p.ws_bytes = (size_t)BH * (size_t)plan_n_ckpt(p, N) * p.state_elems * sizeof(float);
    }
    return p;
}

// Training pair.  The backward's segments are fixed first (its sweep is the dominant kernel); the forward then cuts
// each of them into save_every equal pieces, as close as the chunk grid allows to the split it would have chosen
// for itself, so that every backward boundary is also a forward boundary.
TrainPlans make_train_plans(long BH, int N, int dk, int dv, int chunk)
{
    TrainPlans t{};
    const int cb = (chunk == 128 && dk == 64 && dv == 64) ? 128 : 64;      // the backward's chunk
    t.bwd = make_plan(BH, N, dk, dv, cb, CHELA_DTYPE_BF16, true, false);
    t.fwd = make_plan(BH, N, dk, dv, cb, CHELA_DTYPE_BF16, false, false);   // both calls tile with the same chunk
    t.save_every = 1;
    if (BH <= 0 || N <= 0) return t;
    // 256 sequences: the plain backward gains from cutting each in two; the pair gains less, since its backward has
    // no pre-pass to lose and its forward pays for the cut -- 3 % with 64 x 64 states, and with larger states it
    // loses 6 % (32 x 8 sequences of 4096 tokens, 64 x 128: 492 us uncut, 524 us cut)
    const long n_chunks = ((long)N + cb - 1) / cb;
    if (BH >= 256 && !(dk == 64 && dv == 64) && t.bwd.n_seg > 1 && n_chunks * cb <= kMaxBwdWalkTokens &&
        env_int("CHELA_SEG_TOKENS", 0) <= 0) {
        t.bwd.seg_len = (int)(n_chunks * cb);
        t.bwd.n_seg = 1;
        t.bwd.ckpt_every = 0;
    }
    const long cps_b = t.bwd.seg_len / cb;             // chunks per backward segment
    const double want = (double)t.fwd.n_seg / (double)t.bwd.n_seg;
    long best = 1;
    double best_d = 1e300;
    for (long m = 1; m <= cps_b; ++m) {
        if (cps_b % m) continue;
        if (((long)N + t.bwd.seg_len / m - 1) / (t.bwd.seg_len / m) > 32768) break;   // segments ride on grid.y
        const double d = want > (double)m ? want - (double)m : (double)m - want;
        if (d < best_d) { best_d = d; best = m; }
    }
    t.save_every = (int)best;
    t.fwd.seg_len = (int)(t.bwd.seg_len / best);
    t.fwd.n_seg = (int)(((long)N + t.fwd.seg_len - 1) / t.fwd.seg_len);
    t.fwd.ws_bytes = t.fwd.n_seg > 1 ? (size_t)BH * t.fwd.n_seg * t.fwd.state_elems * sizeof(float) : 0;
    // the backward only needs the suffix array now
    t.bwd.ws_bytes = t.bwd.n_seg > 1 ? (size_t)BH * t.bwd.n_seg * t.bwd.state_elems * sizeof(float) : 0;
    return t;
}

// Non-causal form: the pre-pass is the only part that is split, and only to fill the GPU (two workgroups per compute
// unit measured best: every further segment is a state to write, scan and read), in pieces of at least 256 tokens.
Plan make_noncausal_plan(long BH, int N, int dk, int dv, bool is_bwd)
{
    Plan p{};
    p.chunk = 64;
    p.state_elems = (size_t)dk * dv;
    if (BH <= 0 || N <= 0) { p.seg_len = 64; p.n_seg = 0; p.ws_bytes = 0; return p; }
    const int pairs = is_bwd ? 2 : 1;
    long n_seg = (512 + BH * pairs - 1) / (BH * pairs);
    const long max_seg = N / 256 > 0 ? N / 256 : 1;
    const int forced = env_int("CHELA_NC_SEGS", 0);     // tuning aid: segments per (b,h) of the non-causal pre-pass
    if (forced > 0) n_seg = forced;
    if (n_seg > max_seg) n_seg = max_seg;
    if (n_seg < 1) n_seg = 1;
    long seg_len = (((long)N + n_seg - 1) / n_seg + 63) / 64 * 64;
    p.seg_len = (int)seg_len;
    p.n_seg = (int)(((long)N + seg_len - 1) / seg_len);
    p.ws_bytes = (size_t)BH * p.n_seg * p.state_elems * sizeof(float) * pairs;
    return p;
}

// ------------------------------------------------------------------ per-kernel timing aid
struct ProfRec { int id; hipEvent_t a, b; };
static bool g_prof_on = false;
static std::vector<ProfRec> g_prof;          // records in use
static std::vector<ProfRec> g_prof_free;     // event pairs to re-use
static const char* const kKernelNames[KID_COUNT] = {
    "bf16_seg_state_kernel", "scan_states_kernel", "bf16_fwd_sweep_kernel", "bf16_bwd_sweep_kernel",
    "f32_seg_state_kernel", "f32_sweep_kernel", "copy_probe_kernel", "bf16_step_kernel", "affine_grad_kernel",
    "bf16_apply_state_kernel", "longconv_spectrum_kernel", "shortlong_conv_kernel",
    "shortconv_bwd_kernel", "longconv_bwd_kernel", "gate_norm_kernel", "stream_probe_kernel", "mfma_probe_kernel"};

ProfScope::ProfScope(int id, hipStream_t s) : slot(-1), st(s)
{
    if (!g_prof_on) return;
    ProfRec r{};
    if (!g_prof_free.empty()) { r = g_prof_free.back(); g_prof_free.pop_back(); }
    else if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
    r.id = id;
    (void)hipEventRecord(r.a, st);
    g_prof.push_back(r);
    slot = (int)g_prof.size() - 1;
}

ProfScope::~ProfScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof[slot].b, st);
}

// ------------------------------------------------------------------ scratch
// Two sources.  A caller-owned buffer, set per HOST THREAD (chela_set_workspace): a thread's calls use what that
// thread set last, so threads that each drive a stream of their own cannot disturb each other.  Otherwise an
// allocation of the library's own, one per (device, stream): calls enqueued on different streams may overlap in
// time and therefore never share scratch; calls on one stream are ordered by the stream.
static std::mutex g_mu;
static thread_local void* t_user_ws = nullptr;
static thread_local size_t t_user_bytes = 0;
static constexpr int kMaxDev = 64;
struct OwnWs { hipStream_t stream; void* ptr; size_t bytes; };
static constexpr size_t kMaxOwnStreams = 64;    // per device
static std::vector<OwnWs> g_own_ws[kMaxDev];

static int get_workspace(size_t bytes, void* stream, float** out)
{
    *out = nullptr;
    if (bytes == 0) return CHELA_OK;
    if (t_user_ws) {
        if (bytes > t_user_bytes) return CHELA_ERR_WORKSPACE;
        *out = (float*)t_user_ws;
        return CHELA_OK;
    }
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return CHELA_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDev) return CHELA_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_mu);
    OwnWs* w = nullptr;
    for (OwnWs& x : g_own_ws[dev]) if (x.stream == (hipStream_t)stream) { w = &x; break; }
    if (!w) {
        // Nothing is ever taken away from a stream that may still have work in flight (another thread may hold a
        // pointer it has not launched with yet): a caller that goes through more streams than this hands in
        // buffers of its own, or calls chela_shutdown() at a quiet moment.
        if (g_own_ws[dev].size() >= kMaxOwnStreams) return CHELA_ERR_WORKSPACE;
        g_own_ws[dev].push_back(OwnWs{(hipStream_t)stream, nullptr, 0});
        w = &g_own_ws[dev].back();
    }
    if (w->bytes < bytes) {
        if (w->ptr) { (void)hipDeviceSynchronize(); (void)hipFree(w->ptr); }
        w->ptr = nullptr; w->bytes = 0;
        const size_t want = bytes + bytes / 4;
        void* p = nullptr;
        if (hipMalloc(&p, want) != hipSuccess) { (void)hipGetLastError(); return CHELA_ERR_WORKSPACE; }
        w->ptr = p; w->bytes = want;
    }
    *out = (float*)w->ptr;
    return CHELA_OK;
}

// ------------------------------------------------------------------ scratch that is never allocated
// For callers that cannot allocate (HIP graph capture, serving loops, harnesses that forbid hipMalloc): a
// file-scope device array that the code object brings with it.  Every GPU the library runs on holds its own copy at
// its own address until the process ends.  The name below is a host-side stand-in, not a device address: host code
// asks the runtime for the address once per device and from then on uses only that pointer.
constexpr size_t kStaticScratchBytes = (size_t)32 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
static void* g_scratch_ptr[kMaxDev] = {nullptr};

// The current device's copy of `scratch` (looked up on first use on that device, with that device current).
static int static_scratch(float** out)
{
    *out = nullptr;
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) { (void)hipGetLastError(); return CHELA_ERR_HIP; }
    if (dev < 0 || dev >= kMaxDev) return CHELA_ERR_HIP;
    std::lock_guard<std::mutex> lk(g_mu);
    if (g_scratch_ptr[dev] == nullptr) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
            (void)hipGetLastError();
            return CHELA_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = (float*)g_scratch_ptr[dev];
    return CHELA_OK;
}

// ------------------------------------------------------------------ validation
struct Range { const char* p; size_t n; };
static bool overlap(const Range& a, const Range& b)
{
    if (!a.n || !b.n) return false;
    return a.p < b.p + b.n && b.p < a.p + a.n;
}

static int validate(const void* const* in, const size_t* in_bytes, int n_in,
                    void* const* out, const size_t* out_bytes, int n_out,
                    int B, int H, int N, int dk, int dv, int chunk, int dtype, bool* empty)
{
    *empty = false;
    if (B < 0 || H < 0 || N < 0) return CHELA_ERR_BAD_SHAPE;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return CHELA_ERR_UNSUPPORTED_DIM;
    if (dtype == CHELA_DTYPE_BF16) { if (!(chunk == 64 || chunk == 128)) return CHELA_ERR_BAD_CHUNK; }
    else { if (!(chunk == 16 || chunk == 32 || chunk == 64)) return CHELA_ERR_BAD_CHUNK; }
    const unsigned long long elems = (unsigned long long)B * (unsigned long long)H * (unsigned long long)N;
    if (elems > (1ull << 40)) return CHELA_ERR_BAD_SHAPE;
    if ((unsigned long long)B * (unsigned long long)H > 0x7fffffffull) return CHELA_ERR_BAD_SHAPE;
    if (elems == 0) { *empty = true; return CHELA_OK; }
    for (int i = 0; i < n_in; ++i) if (!in[i]) return CHELA_ERR_NULL_POINTER;
    for (int i = 0; i < n_out; ++i) if (!out[i]) return CHELA_ERR_NULL_POINTER;
    for (int i = 0; i < n_in; ++i) if ((uintptr_t)in[i] & 15u) return CHELA_ERR_MISALIGNED;
    for (int i = 0; i < n_out; ++i) if ((uintptr_t)out[i] & 15u) return CHELA_ERR_MISALIGNED;
    for (int o = 0; o < n_out; ++o) {
        Range ro{(const char*)out[o], out_bytes[o]};
        for (int i = 0; i < n_in; ++i)
            if (overlap(ro, Range{(const char*)in[i], in_bytes[i]})) return CHELA_ERR_ALIASING;
        for (int o2 = o + 1; o2 < n_out; ++o2)
            if (overlap(ro, Range{(const char*)out[o2], out_bytes[o2]})) return CHELA_ERR_ALIASING;
    }
    return CHELA_OK;
}

// The fp32 kernels tile with the chunk that fits LDS next to the fp32 state: 64 tokens, 32 when both head widths
// are 128.  The `chunk` argument (validated, {16, 32, 64}) is a hint and, like every chunking, cannot change the result
// beyond re-association.
static int f32_effective_chunk(int dk, int dv, int chunk)
{
    (void)chunk;
    return (dk == 128 && dv == 128) ? 32 : 64;
}

// The backward sweep keeps four input tiles and two states in LDS; 128-token chunks only fit with 64-wide heads.
static int bf16_bwd_effective_chunk(int dk, int dv, int chunk)
{
    return (chunk == 128 && dk == 64 && dv == 64) ? 128 : 64;
}

// static_ws: the segment states go into the file-scope device array instead of the workspace (nothing is allocated;
// a problem whose states do not fit is rejected).
static int fwd_common(const void* Q, const void* K, const void* V, void* O, const float* S_in, float* S_out, int B,
                      int H, int N, int dk, int dv, int chunk, void* stream, int dtype, bool static_ws = false)
{
    const size_t es = dtype == CHELA_DTYPE_BF16 ? 2 : 4;
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const size_t sb = (B > 0 && H > 0) ? (size_t)B * H * dk * dv * sizeof(float) : 0;
    const void* in[4] = {Q, K, V, S_in};
    // S_out may be S_in (state updated in place): the carried-in state is consumed by the scan before the sweep's
    // last workgroup writes the final one
    const size_t inb[4] = {th * dk * es, th * dk * es, th * dv * es, (S_in && (const void*)S_in != (const void*)S_out) ? sb : 0};
    void* out[2] = {O, S_out};
    const size_t outb[2] = {th * dv * es, S_out ? sb : 0};
    bool empty = false;
    // the optional states are validated like tensors where present (a placeholder stands in where absent)
    const void* in_v[4] = {Q, K, V, S_in ? (const void*)S_in : Q};
    void* out_v[2] = {O, S_out ? (void*)S_out : O};
    int rc = validate(in_v, inb, 4, out_v, outb, 2, B, H, N, dk, dv, chunk, dtype, &empty);
    (void)in; (void)out;
    if (rc != CHELA_OK) return rc;
    const long BH = (long)B * H;
    if (empty) {
        // no tokens: the state passes through unchanged
        if (S_out && BH > 0) {
            hipError_t e = S_in ? hipMemcpyAsync(S_out, S_in, sb, hipMemcpyDeviceToDevice, (hipStream_t)stream)
                                : launch_zero_fill(S_out, sb / sizeof(float), (hipStream_t)stream);
            return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
        }
        return CHELA_OK;
    }
    if (dtype == CHELA_DTYPE_F32) chunk = f32_effective_chunk(dk, dv, chunk);
    Plan plan = make_plan(BH, N, dk, dv, chunk, dtype, false, S_in != nullptr);
    float* ws = nullptr;
    if (static_ws) {
        if (plan.ws_bytes > kStaticScratchBytes) return CHELA_ERR_WORKSPACE;
        rc = plan.ws_bytes ? static_scratch(&ws) : CHELA_OK;
    } else {
        rc = get_workspace(plan.ws_bytes, stream, &ws);
    }
    if (rc != CHELA_OK) return rc;
    hipError_t e = dtype == CHELA_DTYPE_BF16
        ? launch_bf16_fwd(Q, K, V, O, S_in, S_out, nullptr, 1, BH, N, dk, dv, plan, ws, (hipStream_t)stream)
        : launch_f32((const float*)Q, (const float*)K, (const float*)V, (float*)O, BH, N, dk, dv, plan, false, ws,
                     (hipStream_t)stream);
    return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int bwd_common(const void* Q, const void* K, const void* V, const void* dO, const float* S_in,
                      const float* dS_out, void* dQ, void* dK, void* dV, float* dS_in, int B, int H, int N, int dk,
                      int dv, int chunk, void* stream, int dtype)
{
    const size_t es = dtype == CHELA_DTYPE_BF16 ? 2 : 4;
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const size_t sb = (B > 0 && H > 0) ? (size_t)B * H * dk * dv * sizeof(float) : 0;
    const void* in_v[6] = {Q, K, V, dO, S_in ? (const void*)S_in : Q, dS_out ? (const void*)dS_out : Q};
    // dS_in may be dS_out (in place), for the same reason as in the forward
    const size_t inb[6] = {th * dk * es, th * dk * es, th * dv * es, th * dv * es, S_in ? sb : 0,
                           (dS_out && (const void*)dS_out != (const void*)dS_in) ? sb : 0};
    void* out_v[4] = {dQ, dK, dV, dS_in ? (void*)dS_in : dQ};
    const size_t outb[4] = {th * dk * es, th * dk * es, th * dv * es, dS_in ? sb : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 6, out_v, outb, 4, B, H, N, dk, dv, chunk, dtype, &empty);
    if (rc != CHELA_OK) return rc;
    const long BH = (long)B * H;
    hipStream_t st = (hipStream_t)stream;
    if (empty) {
        if (dS_in && BH > 0) {
            hipError_t e = dS_out ? hipMemcpyAsync(dS_in, dS_out, sb, hipMemcpyDeviceToDevice, st)
                                  : launch_zero_fill(dS_in, sb / sizeof(float), st);
            return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
        }
        return CHELA_OK;
    }
    if (dtype == CHELA_DTYPE_BF16) {
        Plan plan = make_plan(BH, N, dk, dv, bf16_bwd_effective_chunk(dk, dv, chunk), dtype, true,
                              S_in != nullptr || dS_out != nullptr, true);
        float* ws = nullptr;
        rc = get_workspace(plan.ws_bytes, stream, &ws);
        if (rc != CHELA_OK) return rc;
        hipError_t e = launch_bf16_bwd(Q, K, V, dO, S_in, dS_out, dQ, dK, dV, dS_in, nullptr, BH, N, dk, dv, plan, ws, st);
        return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
    }
    // fp32: the gradient is three instances of the forward map (time-reversal duality):
    //   dQ = LinAttn(query dO, key V, value K)             causal
    //   dV = LinAttn(query K,  key Q, value dO)            anti-causal
    //   dK = LinAttn(query V,  key dO, value Q)            anti-causal
    const int c1 = f32_effective_chunk(dv, dk, chunk);   // query/key width dv, value width dk
    const int c2 = f32_effective_chunk(dk, dv, chunk);
    Plan p1 = make_plan(BH, N, dv, dk, c1, dtype, true, false);
    Plan p2 = make_plan(BH, N, dk, dv, c2, dtype, true, false);
    float* ws = nullptr;
    rc = get_workspace(p1.ws_bytes > p2.ws_bytes ? p1.ws_bytes : p2.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    hipError_t e = launch_f32((const float*)dO, (const float*)V, (const float*)K, (float*)dQ, BH, N, dv, dk, p1,
                              false, ws, st);
    if (e == hipSuccess)
        e = launch_f32((const float*)K, (const float*)Q, (const float*)dO, (float*)dV, BH, N, dk, dv, p2, true, ws, st);
    // the third call's segment states dO^T Q are the transposes of the second call's Q^T dO, which are still there
    const bool same_split = p1.n_seg == p2.n_seg && p1.seg_len == p2.seg_len;
    if (e == hipSuccess)
        e = launch_f32((const float*)V, (const float*)dO, (const float*)Q, (float*)dK, BH, N, dv, dk, p1, true, ws, st,
                       same_split);
    return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static size_t saved_bytes(long BH, const TrainPlans& t) { return (size_t)BH * t.bwd.n_seg * t.bwd.state_elems * sizeof(float); }

// Eq. 11-12 variants.  The kernels tile with 64-token chunks whatever the (validated) hint says.  `saved` (optional,
// with want_saved): the training-pair hand-over of boundary states, as for the plain pair.
static int zfwd_common(const void* Z, const float* aff, const void* V, void* O, void* saved, bool want_saved, int B,
                       int H, int N, int dk, int dv, int chunk, void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const size_t ab = th ? (size_t)4 * H * dk * sizeof(float) : 0;
    const long BH = (long)B * H;
    TrainPlans t{};
    const bool dims_ok = (dk == 64 || dk == 128) && (dv == 64 || dv == 128);
    if (want_saved && th && dims_ok) t = make_train_plans(BH, N, dk, dv, 64);
    const void* in_v[3] = {Z, aff, V};
    const size_t inb[3] = {th * dk * 2, ab, th * dv * 2};
    void* out_v[2] = {O, want_saved ? saved : O};
    const size_t outb[2] = {th * dv * 2, (want_saved && th && dims_ok) ? saved_bytes(BH, t) : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 3, out_v, outb, 2, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    Plan plan = want_saved ? t.fwd : make_plan(BH, N, dk, dv, 64, CHELA_DTYPE_BF16, false, false);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_zfwd(Z, aff, V, O, want_saved ? (float*)saved : nullptr, want_saved ? t.save_every : 1, B, H, N,
                            dk, dv, plan, ws, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int zbwd_common(const void* Z, const float* aff, const void* V, const void* dO, void* dZ, float* d_aff,
                       void* dV, const void* saved, bool want_saved, int B, int H, int N, int dk, int dv, int chunk,
                       void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const size_t ab = (H > 0) ? (size_t)4 * H * dk * sizeof(float) : 0;
    const long BH = (long)B * H;
    TrainPlans t{};
    const bool dims_ok = (dk == 64 || dk == 128) && (dv == 64 || dv == 128);
    if (want_saved && th && dims_ok) t = make_train_plans(BH, N, dk, dv, 64);
    const void* in_v[5] = {Z, aff, V, dO, want_saved ? saved : Z};
    const size_t inb[5] = {th * dk * 2, th ? ab : 0, th * dv * 2, th * dv * 2,
                           (want_saved && th && dims_ok) ? saved_bytes(BH, t) : 0};
    void* out_v[3] = {dZ, d_aff, dV};
    const size_t outb[3] = {th * dk * 2, th ? ab : 0, th * dv * 2};
    bool empty = false;
    int rc = validate(in_v, inb, 5, out_v, outb, 3, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK) return rc;
    if (empty) {
        // no tokens: the parameters received no gradient
        if (d_aff && ab) return launch_zero_fill(d_aff, ab / sizeof(float), (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
        return CHELA_OK;
    }
    Plan plan = want_saved ? t.bwd : make_plan(BH, N, dk, dv, 64, CHELA_DTYPE_BF16, true, false, true);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes + zbwd_extra_ws_bytes(BH, plan, dk), stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_zbwd(Z, aff, V, dO, dZ, d_aff, dV, want_saved ? (const float*)saved : nullptr, B, H, N, dk, dv,
                            plan, ws, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int fwd_save_common(const void* Q, const void* K, const void* V, void* O, void* saved, int B, int H, int N,
                           int dk, int dv, int chunk, void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const long BH = (long)B * H;
    TrainPlans t{};
    if (th && (dk == 64 || dk == 128) && (dv == 64 || dv == 128) && (chunk == 64 || chunk == 128))
        t = make_train_plans(BH, N, dk, dv, chunk);
    const void* in_v[3] = {Q, K, V};
    const size_t inb[3] = {th * dk * 2, th * dk * 2, th * dv * 2};
    void* out_v[2] = {O, saved};
    const size_t outb[2] = {th * dv * 2, th ? saved_bytes(BH, t) : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 3, out_v, outb, 2, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    float* ws = nullptr;
    rc = get_workspace(t.fwd.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_fwd(Q, K, V, O, nullptr, nullptr, (float*)saved, t.save_every, BH, N, dk, dv, t.fwd, ws,
                           (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int bwd_saved_common(const void* Q, const void* K, const void* V, const void* dO, const void* saved, void* dQ,
                            void* dK, void* dV, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const long BH = (long)B * H;
    TrainPlans t{};
    if (th && (dk == 64 || dk == 128) && (dv == 64 || dv == 128) && (chunk == 64 || chunk == 128))
        t = make_train_plans(BH, N, dk, dv, chunk);
    const void* in_v[5] = {Q, K, V, dO, saved};
    const size_t inb[5] = {th * dk * 2, th * dk * 2, th * dv * 2, th * dv * 2, th ? saved_bytes(BH, t) : 0};
    void* out_v[3] = {dQ, dK, dV};
    const size_t outb[3] = {th * dk * 2, th * dk * 2, th * dv * 2};
    bool empty = false;
    int rc = validate(in_v, inb, 5, out_v, outb, 3, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    float* ws = nullptr;
    rc = get_workspace(t.bwd.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_bwd(Q, K, V, dO, nullptr, nullptr, dQ, dK, dV, nullptr, (const float*)saved, BH, N, dk, dv,
                           t.bwd, ws, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

// Forward with the Eq. 9 epilogue; aff non-null: Z in place of Q and K.  O and saved are optional outputs.
static int fwd_gated_common(const void* Q, const void* K, const float* aff, bool zqk, const void* V, const void* G,
                            void* O, void* Y, void* saved, float eps, int B, int H, int N, int dk, int dv, int chunk,
                            void* stream)
{
    if (!(eps >= 0.f) || !std::isfinite(eps)) return CHELA_ERR_BAD_SHAPE;
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const size_t ab = (zqk && th) ? (size_t)4 * H * dk * sizeof(float) : 0;
    const long BH = (long)B * H;
    const bool dims_ok = (dk == 64 || dk == 128) && (dv == 64 || dv == 128);
    TrainPlans t{};
    if (saved && th && dims_ok) t = make_train_plans(BH, N, dk, dv, 64);
    // optional pointers stand in as copies of required ones so that the null / alignment / overlap checks skip them
    const void* in_v[4] = {Q, zqk ? (const void*)aff : K, V, G};
    const size_t inb[4] = {th * dk * 2, zqk ? ab : th * dk * 2, th * dv * 2, th * dv * 2};
    void* out_v[3] = {Y, O ? O : Y, saved ? saved : Y};
    const size_t outb[3] = {th * dv * 2, O ? th * dv * 2 : 0, (saved && th && dims_ok) ? saved_bytes(BH, t) : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 4, out_v, outb, 3, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    Plan plan = saved ? t.fwd : make_plan(BH, N, dk, dv, 64, CHELA_DTYPE_BF16, false, false);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_fwd_gated(Q, K, V, G, O, Y, eps, zqk ? aff : nullptr, (float*)saved, saved ? t.save_every : 1, B,
                                 H, N, dk, dv, plan, ws, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int gate_norm_common(const void* O, const void* G, const void* dY, void* out0, void* out1, bool bwd, float eps,
                            long long rows, int dv, void* stream)
{
    if (!(eps >= 0.f) || !std::isfinite(eps)) return CHELA_ERR_BAD_SHAPE;
    if (rows < 0 || rows > (1ll << 37)) return CHELA_ERR_BAD_SHAPE;   // keeps the grid below 2^31 workgroups
    if (!(dv == 64 || dv == 128)) return CHELA_ERR_UNSUPPORTED_DIM;
    if (rows == 0) return CHELA_OK;
    const size_t nb = (size_t)rows * dv * 2;
    const void* in_v[3] = {O, G, bwd ? dY : O};
    void* out_v[2] = {out0, bwd ? out1 : out0};
    for (int i = 0; i < 3; ++i) if (!in_v[i]) return CHELA_ERR_NULL_POINTER;
    for (int i = 0; i < 2; ++i) if (!out_v[i]) return CHELA_ERR_NULL_POINTER;
    for (int i = 0; i < 3; ++i) if ((uintptr_t)in_v[i] & 15u) return CHELA_ERR_MISALIGNED;
    for (int i = 0; i < 2; ++i) if ((uintptr_t)out_v[i] & 15u) return CHELA_ERR_MISALIGNED;
    const int n_out = bwd ? 2 : 1;
    for (int o = 0; o < n_out; ++o) {
        const Range ro{(const char*)out_v[o], nb};
        for (int i = 0; i < (bwd ? 3 : 2); ++i) {
            if (bwd && o == 0 && i == 2 && out_v[0] == dY) continue;   // dO written over dY, element for element
            if (overlap(ro, Range{(const char*)in_v[i], nb})) return CHELA_ERR_ALIASING;
        }
    }
    if (bwd && overlap(Range{(const char*)out0, nb}, Range{(const char*)out1, nb})) return CHELA_ERR_ALIASING;
    return launch_gate_norm(O, G, bwd ? dY : nullptr, out0, bwd ? out1 : nullptr, eps, (long)rows, dv,
                            (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

// [B,N,H,d] tensors: same extents and aliasing rules as the [B,H,N,d] calls, 64-token chunks.
static int bnhd_common(const void* Q, const void* K, const void* V, const void* dO, void* O_or_dQ, void* dK, void* dV,
                       bool is_bwd, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const void* in_v[4] = {Q, K, V, is_bwd ? dO : Q};
    const size_t inb[4] = {th * dk * 2, th * dk * 2, th * dv * 2, is_bwd ? th * dv * 2 : 0};
    void* out_v[3] = {O_or_dQ, is_bwd ? dK : O_or_dQ, is_bwd ? dV : O_or_dQ};
    const size_t outb[3] = {th * (is_bwd ? dk : dv) * 2, is_bwd ? th * dk * 2 : 0, is_bwd ? th * dv * 2 : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 4, out_v, outb, 3, B, H, N, dk, dv, chunk, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    Plan plan = make_plan((long)B * H, N, dk, dv, 64, CHELA_DTYPE_BF16, is_bwd, false, true);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    hipError_t e = is_bwd ? launch_bf16_bwd_nh(Q, K, V, dO, O_or_dQ, dK, dV, B, H, N, dk, dv, plan, ws, (hipStream_t)stream)
                          : launch_bf16_fwd_nh(Q, K, V, O_or_dQ, B, H, N, dk, dv, plan, ws, (hipStream_t)stream);
    return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

static int noncausal_common(const void* Q, const void* K, const void* V, const void* dO, void* O_or_dQ, void* dK,
                            void* dV, bool is_bwd, int B, int H, int N, int dk, int dv, void* stream)
{
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const void* in_v[4] = {Q, K, V, is_bwd ? dO : Q};
    const size_t inb[4] = {th * dk * 2, th * dk * 2, th * dv * 2, is_bwd ? th * dv * 2 : 0};
    void* out_v[3] = {O_or_dQ, is_bwd ? dK : O_or_dQ, is_bwd ? dV : O_or_dQ};
    const size_t outb[3] = {th * (is_bwd ? dk : dv) * 2, is_bwd ? th * dk * 2 : 0, is_bwd ? th * dv * 2 : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 4, out_v, outb, 3, B, H, N, dk, dv, 64, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    const long BH = (long)B * H;
    Plan plan = make_noncausal_plan(BH, N, dk, dv, is_bwd);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    hipError_t e = is_bwd ? launch_bf16_noncausal_bwd(Q, K, V, dO, O_or_dQ, dK, dV, BH, N, dk, dv, plan, ws,
                                                      (hipStream_t)stream)
                          : launch_bf16_noncausal_fwd(Q, K, V, O_or_dQ, BH, N, dk, dv, plan, ws, (hipStream_t)stream);
    return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

// Non-causal forward with the Eq. 9 epilogue: Y = Norm(Q (K^T V)) * G; O optional.
static int noncausal_gated_common(const void* Q, const void* K, const void* V, const void* G, void* O, void* Y,
                                  float eps, int B, int H, int N, int dk, int dv, void* stream)
{
    if (!(eps >= 0.f) || !std::isfinite(eps)) return CHELA_ERR_BAD_SHAPE;
    const size_t th = (B > 0 && H > 0 && N > 0) ? (size_t)B * H * N : 0;
    const void* in_v[4] = {Q, K, V, G};
    const size_t inb[4] = {th * dk * 2, th * dk * 2, th * dv * 2, th * dv * 2};
    void* out_v[2] = {Y, O ? O : Y};
    const size_t outb[2] = {th * dv * 2, O ? th * dv * 2 : 0};
    bool empty = false;
    int rc = validate(in_v, inb, 4, out_v, outb, 2, B, H, N, dk, dv, 64, CHELA_DTYPE_BF16, &empty);
    if (rc != CHELA_OK || empty) return rc;
    const long BH = (long)B * H;
    Plan plan = make_noncausal_plan(BH, N, dk, dv, false);
    float* ws = nullptr;
    rc = get_workspace(plan.ws_bytes, stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_bf16_noncausal_fwd(Q, K, V, O, BH, N, dk, dv, plan, ws, (hipStream_t)stream, G, Y, eps) == hipSuccess
               ? CHELA_OK : CHELA_ERR_HIP;
}

}  // namespace chela

using namespace chela;

extern "C" {

int chela_linattn_fwd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk, int dv,
                      int chunk, void* stream)
{
    return fwd_common(Q, K, V, O, nullptr, nullptr, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_BF16);
}

int chela_linattn_fwd_noalloc(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk,
                              int dv, int chunk, void* stream)
{
    return fwd_common(Q, K, V, O, nullptr, nullptr, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_BF16, true);
}

int chela_linattn_fwd_f32(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk,
                          int dv, int chunk, void* stream)
{
    return fwd_common(Q, K, V, O, nullptr, nullptr, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_F32);
}

int chela_linattn_bwd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK, void* dV,
                      int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return bwd_common(Q, K, V, dO, nullptr, nullptr, dQ, dK, dV, nullptr, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_BF16);
}

int chela_linattn_bwd_f32(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK,
                          void* dV, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return bwd_common(Q, K, V, dO, nullptr, nullptr, dQ, dK, dV, nullptr, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_F32);
}

int chela_linattn_fwd_state(const void* Q, const void* K, const void* V, const float* S_in, void* O, float* S_out,
                            int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return fwd_common(Q, K, V, O, S_in, S_out, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_BF16);
}

int chela_linattn_bwd_state(const void* Q, const void* K, const void* V, const float* S_in, const void* dO,
                            const float* dS_out, void* dQ, void* dK, void* dV, float* dS_in, int B, int H, int N,
                            int dk, int dv, int chunk, void* stream)
{
    return bwd_common(Q, K, V, dO, S_in, dS_out, dQ, dK, dV, dS_in, B, H, N, dk, dv, chunk, stream, CHELA_DTYPE_BF16);
}

int chela_linattn_zfwd(const void* Z, const float* affine, const void* V, void* O, int B, int H, int N, int dk,
                       int dv, int chunk, void* stream)
{
    return zfwd_common(Z, affine, V, O, nullptr, false, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_zbwd(const void* Z, const float* affine, const void* V, const void* dO, void* dZ, float* d_affine,
                       void* dV, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return zbwd_common(Z, affine, V, dO, dZ, d_affine, dV, nullptr, false, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_zfwd_save(const void* Z, const float* affine, const void* V, void* O, void* saved, int B, int H,
                            int N, int dk, int dv, int chunk, void* stream)
{
    return zfwd_common(Z, affine, V, O, saved, true, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_zbwd_saved(const void* Z, const float* affine, const void* V, const void* dO, const void* saved,
                             void* dZ, float* d_affine, void* dV, int B, int H, int N, int dk, int dv, int chunk,
                             void* stream)
{
    return zbwd_common(Z, affine, V, dO, dZ, d_affine, dV, saved, true, B, H, N, dk, dv, chunk, stream);
}

size_t chela_linattn_z_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk, int is_bwd)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return 0;
    if (!(chunk == 64 || chunk == 128)) return 0;
    const long BH = (long)B * H;
    Plan plan = make_plan(BH, N, dk, dv, 64, CHELA_DTYPE_BF16, is_bwd != 0, false, true);
    size_t need = plan.ws_bytes + (is_bwd ? zbwd_extra_ws_bytes(BH, plan, dk) : 0);
    // the training pair (chela_linattn_zfwd_save / _zbwd_saved, the gated forward with `saved`) splits on its own grid
    const TrainPlans t = make_train_plans(BH, N, dk, dv, 64);
    const size_t pair = is_bwd ? t.bwd.ws_bytes + zbwd_extra_ws_bytes(BH, t.bwd, dk) : t.fwd.ws_bytes;
    return need > pair ? need : pair;
}

int chela_linattn_fwd_save(const void* Q, const void* K, const void* V, void* O, void* saved, int B, int H, int N,
                           int dk, int dv, int chunk, void* stream)
{
    return fwd_save_common(Q, K, V, O, saved, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_bwd_saved(const void* Q, const void* K, const void* V, const void* dO, const void* saved, void* dQ,
                            void* dK, void* dV, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return bwd_saved_common(Q, K, V, dO, saved, dQ, dK, dV, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_fwd_gated(const void* Q, const void* K, const void* V, const void* G, void* O, void* Y, void* saved,
                            float eps, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return fwd_gated_common(Q, K, nullptr, false, V, G, O, Y, saved, eps, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_zfwd_gated(const void* Z, const float* affine, const void* V, const void* G, void* O, void* Y,
                             void* saved, float eps, int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return fwd_gated_common(Z, nullptr, affine, true, V, G, O, Y, saved, eps, B, H, N, dk, dv, chunk, stream);
}

int chela_gate_norm_fwd(const void* O, const void* G, void* Y, float eps, long long rows, int dv, void* stream)
{
    return gate_norm_common(O, G, nullptr, Y, nullptr, false, eps, rows, dv, stream);
}

int chela_gate_norm_bwd(const void* O, const void* G, const void* dY, void* dO, void* dG, float eps, long long rows,
                        int dv, void* stream)
{
    return gate_norm_common(O, G, dY, dO, dG, true, eps, rows, dv, stream);
}

size_t chela_linattn_saved_bytes(int B, int H, int N, int dk, int dv, int chunk)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return 0;
    if (!(chunk == 64 || chunk == 128)) return 0;
    return saved_bytes((long)B * H, make_train_plans((long)B * H, N, dk, dv, chunk));
}

int chela_linattn_fwd_bnhd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk, int dv,
                           int chunk, void* stream)
{
    return bnhd_common(Q, K, V, nullptr, O, nullptr, nullptr, false, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_bwd_bnhd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK, void* dV,
                           int B, int H, int N, int dk, int dv, int chunk, void* stream)
{
    return bnhd_common(Q, K, V, dO, dQ, dK, dV, true, B, H, N, dk, dv, chunk, stream);
}

int chela_linattn_noncausal_fwd(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk,
                                int dv, void* stream)
{
    return noncausal_common(Q, K, V, nullptr, O, nullptr, nullptr, false, B, H, N, dk, dv, stream);
}

int chela_linattn_noncausal_bwd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK,
                                void* dV, int B, int H, int N, int dk, int dv, void* stream)
{
    return noncausal_common(Q, K, V, dO, dQ, dK, dV, true, B, H, N, dk, dv, stream);
}

int chela_linattn_noncausal_fwd_gated(const void* Q, const void* K, const void* V, const void* G, void* O, void* Y,
                                      float eps, int B, int H, int N, int dk, int dv, void* stream)
{
    return noncausal_gated_common(Q, K, V, G, O, Y, eps, B, H, N, dk, dv, stream);
}

size_t chela_linattn_noncausal_workspace_bytes(int B, int H, int N, int dk, int dv, int is_bwd)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return 0;
    return make_noncausal_plan((long)B * H, N, dk, dv, is_bwd != 0).ws_bytes;
}

size_t chela_longconv_spectrum_bytes(int d, int L)
{
    const int M = (d > 0 && L > 0) ? conv_fft_size(L) : 0;
    if (d > 0 && L > 0 && conv_blocks(L)) return conv_blocked_spectrum_bytes(d, L);
    // one (K[k], K[M-k]) pair per 16 bytes; behind them, for the sizes the matrix-core kernel serves, its own copy
    if (!M) return 0;
    const size_t extra = convmx_spectrum_bytes(d, L);
    return extra ? conv_pairs_bytes(d, L) + extra : (size_t)d * (size_t)(M / 2 + 1) * 4 * sizeof(float);
}

int chela_longconv_spectrum(const float* k_long, void* spectrum, int d, int L, void* stream)
{
    if (d < 0 || L < 0) return CHELA_ERR_BAD_SHAPE;
    if (d == 0 || L == 0) return CHELA_OK;
    if (conv_fft_size(L) == 0 && conv_blocks(L) == 0) return CHELA_ERR_BAD_SHAPE;
    if (!k_long || !spectrum) return CHELA_ERR_NULL_POINTER;
    if (((uintptr_t)k_long | (uintptr_t)spectrum) & 15u) return CHELA_ERR_MISALIGNED;
    if (overlap(Range{(const char*)k_long, (size_t)d * L * 4}, Range{(const char*)spectrum, chela_longconv_spectrum_bytes(d, L)}))
        return CHELA_ERR_ALIASING;
    if (launch_longconv_spectrum(k_long, spectrum, d, L, (hipStream_t)stream) != hipSuccess) return CHELA_ERR_HIP;
    if (convmx_spectrum_bytes(d, L) &&
        launch_convmx_spectrum(k_long, spectrum, (char*)spectrum + conv_pairs_bytes(d, L), d, L, (hipStream_t)stream) != hipSuccess)
        return CHELA_ERR_HIP;
    return CHELA_OK;
}

static int shortlong_common(const void* X, const float* w_short, int m, const void* spectrum, void* Y, int B, int d,
                            int L, int dtype, void* stream)
{
    if (B < 0 || d < 0 || L < 0) return CHELA_ERR_BAD_SHAPE;
    if (w_short != nullptr && (m < 1 || m > 32)) return CHELA_ERR_BAD_SHAPE;
    if ((unsigned long long)B * (unsigned long long)d > 0x7fffffffull) return CHELA_ERR_BAD_SHAPE;
    if (B == 0 || d == 0 || L == 0) return CHELA_OK;
    if (conv_fft_size(L) == 0 && conv_blocks(L) == 0) return CHELA_ERR_BAD_SHAPE;
    if (!X || !spectrum || !Y) return CHELA_ERR_NULL_POINTER;
    if (((uintptr_t)X | (uintptr_t)spectrum | (uintptr_t)Y | (uintptr_t)w_short) & 15u) return CHELA_ERR_MISALIGNED;
    const size_t es = dtype == CHELA_DTYPE_BF16 ? 2 : 4, tb = (size_t)B * d * L * es;
    const Range ry{(const char*)Y, tb};
    if (overlap(ry, Range{(const char*)X, tb}) || overlap(ry, Range{(const char*)spectrum, chela_longconv_spectrum_bytes(d, L)}) ||
        (w_short && overlap(ry, Range{(const char*)w_short, (size_t)d * m * 4})))
        return CHELA_ERR_ALIASING;
    if (convmx_applies(L, dtype == CHELA_DTYPE_BF16 ? 0 : 1))
        return launch_convmx_fwd(X, w_short, m, (const char*)spectrum + conv_pairs_bytes(d, L), Y, B, d, L,
                                 (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
    return launch_shortlong_conv(X, w_short, m, spectrum, Y, (long)B * d, d, L, dtype == CHELA_DTYPE_BF16 ? 0 : 1,
                                 (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_shortlong_conv_fwd(const void* X, const float* w_short, int m, const void* spectrum, void* Y, int B, int d,
                             int L, void* stream)
{
    return shortlong_common(X, w_short, m, spectrum, Y, B, d, L, CHELA_DTYPE_BF16, stream);
}

int chela_shortlong_conv_fwd_f32(const void* X, const float* w_short, int m, const void* spectrum, void* Y, int B,
                                 int d, int L, void* stream)
{
    return shortlong_common(X, w_short, m, spectrum, Y, B, d, L, CHELA_DTYPE_F32, stream);
}

static size_t conv_bwd_ws_bytes(int B, int d, int L, int dtype, bool has_short)
{
    if (B <= 0 || d <= 0 || L <= 0) return 0;
    const size_t acc = conv_bwd_acc_floats(B, d, L, dtype == CHELA_DTYPE_BF16) * sizeof(float);      // running sums of the long-kernel gradient
    if (!has_short) return acc;
    const size_t n = (size_t)B * d * L, tiles = ((size_t)L + 2047) / 2048;
    (void)dtype;
    return acc + n * sizeof(float) + (size_t)B * d * tiles * 32 * sizeof(float);
}

size_t chela_shortlong_conv_bwd_workspace_bytes(int B, int d, int L, int has_short_kernel, int dtype)
{
    if (dtype != CHELA_DTYPE_BF16 && dtype != CHELA_DTYPE_F32) return 0;
    return conv_bwd_ws_bytes(B, d, L, dtype, has_short_kernel != 0);
}

static int shortlong_bwd_common(const void* X, const float* w_short, int m, const void* spectrum, const void* dZ,
                                void* dX, float* d_w_short, float* d_k_long, int B, int d, int L, int dtype,
                                void* stream)
{
    if (B < 0 || d < 0 || L < 0) return CHELA_ERR_BAD_SHAPE;
    if (w_short != nullptr && (m < 1 || m > 32)) return CHELA_ERR_BAD_SHAPE;
    if (B > 65535) return CHELA_ERR_BAD_SHAPE;                                    // batch entries ride on grid.y
    if ((unsigned long long)B * (unsigned long long)d > 0x7fffffffull) return CHELA_ERR_BAD_SHAPE;
    if (d == 0 || L == 0) return CHELA_OK;
    if (conv_fft_size(L) == 0 && conv_blocks(L) == 0) return CHELA_ERR_BAD_SHAPE;
    hipStream_t st = (hipStream_t)stream;
    if (B == 0) {
        // no data: the kernels received no gradient
        if (!d_k_long || (w_short && !d_w_short)) return CHELA_ERR_NULL_POINTER;
        hipError_t e = launch_zero_fill(d_k_long, (size_t)d * L, st);
        if (e == hipSuccess && w_short) e = launch_zero_fill(d_w_short, (size_t)d * m, st);
        return e == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
    }
    if (!X || !spectrum || !dZ || !dX || !d_k_long || (w_short && !d_w_short)) return CHELA_ERR_NULL_POINTER;
    if (((uintptr_t)X | (uintptr_t)spectrum | (uintptr_t)dZ | (uintptr_t)dX | (uintptr_t)d_k_long | (uintptr_t)w_short |
         (uintptr_t)d_w_short) & 15u)
        return CHELA_ERR_MISALIGNED;
    const size_t es = dtype == CHELA_DTYPE_BF16 ? 2 : 4, tb = (size_t)B * d * L * es;
    const Range in[4] = {{(const char*)X, tb}, {(const char*)dZ, tb},
                         {(const char*)spectrum, chela_longconv_spectrum_bytes(d, L)},
                         {(const char*)w_short, w_short ? (size_t)d * m * 4 : 0}};
    const Range out[3] = {{(const char*)dX, tb}, {(const char*)d_k_long, (size_t)d * L * 4},
                          {(const char*)d_w_short, w_short ? (size_t)d * m * 4 : 0}};
    for (int o = 0; o < 3; ++o) {
        for (const Range& r : in) if (overlap(out[o], r)) return CHELA_ERR_ALIASING;
        for (int o2 = o + 1; o2 < 3; ++o2) if (overlap(out[o], out[o2])) return CHELA_ERR_ALIASING;
    }
    float* ws = nullptr;
    int rc = get_workspace(conv_bwd_ws_bytes(B, d, L, dtype, w_short != nullptr), stream, &ws);
    if (rc != CHELA_OK) return rc;
    return launch_shortlong_conv_bwd(X, w_short, m, spectrum, dZ, dX, d_w_short, d_k_long, ws, B, d, L,
                                     dtype == CHELA_DTYPE_BF16 ? 0 : 1, st) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_shortlong_conv_bwd(const void* X, const float* w_short, int m, const void* spectrum, const void* dZ,
                             void* dX, float* d_w_short, float* d_k_long, int B, int d, int L, void* stream)
{
    return shortlong_bwd_common(X, w_short, m, spectrum, dZ, dX, d_w_short, d_k_long, B, d, L, CHELA_DTYPE_BF16, stream);
}

int chela_shortlong_conv_bwd_f32(const void* X, const float* w_short, int m, const void* spectrum, const void* dZ,
                                 void* dX, float* d_w_short, float* d_k_long, int B, int d, int L, void* stream)
{
    return shortlong_bwd_common(X, w_short, m, spectrum, dZ, dX, d_w_short, d_k_long, B, d, L, CHELA_DTYPE_F32, stream);
}

static int step_common(const void* q, const void* k, const void* v, const void* g, bool gated, float eps, float* S,
                       void* o, int B, int H, int dk, int dv, void* stream)
{
    if (gated && (!(eps >= 0.f) || !std::isfinite(eps))) return CHELA_ERR_BAD_SHAPE;
    if (B < 0 || H < 0) return CHELA_ERR_BAD_SHAPE;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return CHELA_ERR_UNSUPPORTED_DIM;
    if ((unsigned long long)B * (unsigned long long)H > 0x7fffffffull) return CHELA_ERR_BAD_SHAPE;
    if (B == 0 || H == 0) return CHELA_OK;
    if (!q || !k || !v || !S || !o || (gated && !g)) return CHELA_ERR_NULL_POINTER;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)S | (uintptr_t)o | (uintptr_t)(gated ? g : q)) & 15u)
        return CHELA_ERR_MISALIGNED;
    const size_t bh = (size_t)B * H;
    const Range ro{(const char*)o, bh * dv * 2}, rs{(const char*)S, bh * dk * dv * 4};
    const Range ri[4] = {{(const char*)q, bh * dk * 2}, {(const char*)k, bh * dk * 2}, {(const char*)v, bh * dv * 2},
                         {(const char*)g, gated ? bh * dv * 2 : 0}};
    if (overlap(ro, rs)) return CHELA_ERR_ALIASING;
    for (const Range& r : ri) if (overlap(ro, r) || overlap(rs, r)) return CHELA_ERR_ALIASING;
    return launch_bf16_step(q, k, v, S, o, gated ? g : nullptr, eps, (long)bh, dk, dv, (hipStream_t)stream) == hipSuccess
               ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_linattn_step(const void* q, const void* k, const void* v, float* S, void* o, int B, int H, int dk, int dv,
                       void* stream)
{
    return step_common(q, k, v, nullptr, false, 0.f, S, o, B, H, dk, dv, stream);
}

int chela_linattn_step_gated(const void* q, const void* k, const void* v, const void* g, float* S, void* y, float eps,
                             int B, int H, int dk, int dv, void* stream)
{
    return step_common(q, k, v, g, true, eps, S, y, B, H, dk, dv, stream);
}

size_t chela_linattn_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk, int is_bwd, int dtype)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return 0;
    if (dtype == CHELA_DTYPE_BF16) {
        if (!(chunk == 64 || chunk == 128)) return 0;
        // the larger need of the calls this query stands for: with and without carried states
        const int cb = is_bwd ? bf16_bwd_effective_chunk(dk, dv, chunk) : chunk;
        const size_t a = make_plan((long)B * H, N, dk, dv, cb, dtype, is_bwd != 0, true, true).ws_bytes;
        const size_t b = make_plan((long)B * H, N, dk, dv, cb, dtype, is_bwd != 0, false, true).ws_bytes;
        return a > b ? a : b;
    }
    if (dtype != CHELA_DTYPE_F32) return 0;
    if (!(chunk == 16 || chunk == 32 || chunk == 64)) return 0;
    size_t a = make_plan((long)B * H, N, dk, dv, f32_effective_chunk(dk, dv, chunk), dtype, is_bwd != 0, false).ws_bytes;
    if (is_bwd) {
        size_t b = make_plan((long)B * H, N, dv, dk, f32_effective_chunk(dv, dk, chunk), dtype, true, false).ws_bytes;
        if (b > a) a = b;
    }
    return a;
}

size_t chela_linattn_train_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk, int is_bwd)
{
    if (B <= 0 || H <= 0 || N <= 0) return 0;
    if (!((dk == 64 || dk == 128) && (dv == 64 || dv == 128))) return 0;
    if (!(chunk == 64 || chunk == 128)) return 0;
    size_t need = 0;
    for (int c : {chunk, 64}) {      // (the gated forwards that fill `saved` always tile with 64 tokens)
        const TrainPlans t = make_train_plans((long)B * H, N, dk, dv, c);
        const size_t x = is_bwd ? t.bwd.ws_bytes : t.fwd.ws_bytes;
        if (x > need) need = x;
    }
    return need;
}

int chela_set_workspace(void* dev_ptr, size_t bytes)
{
    if (dev_ptr == nullptr || bytes == 0) { t_user_ws = nullptr; t_user_bytes = 0; return CHELA_OK; }
    if ((uintptr_t)dev_ptr & 255u) return CHELA_ERR_MISALIGNED;
    t_user_ws = dev_ptr; t_user_bytes = bytes;
    return CHELA_OK;
}

int chela_get_workspace(void** dev_ptr, size_t* bytes)
{
    if (!dev_ptr || !bytes) return CHELA_ERR_NULL_POINTER;
    *dev_ptr = t_user_ws; *bytes = t_user_bytes;
    return CHELA_OK;
}

const char* chela_status_string(int status)
{
    switch (status) {
        case CHELA_OK: return "CHELA_OK";
        case CHELA_ERR_NULL_POINTER: return "CHELA_ERR_NULL_POINTER: a tensor pointer is NULL";
        case CHELA_ERR_BAD_SHAPE: return "CHELA_ERR_BAD_SHAPE: negative or overflowing B, H or N";
        case CHELA_ERR_UNSUPPORTED_DIM: return "CHELA_ERR_UNSUPPORTED_DIM: dk and dv must be 64 or 128";
        case CHELA_ERR_BAD_CHUNK: return "CHELA_ERR_BAD_CHUNK: chunk must be 64/128 (bf16) or 16/32/64 (fp32)";
        case CHELA_ERR_MISALIGNED: return "CHELA_ERR_MISALIGNED: pointer not sufficiently aligned";
        case CHELA_ERR_ALIASING: return "CHELA_ERR_ALIASING: an output overlaps an input or another output";
        case CHELA_ERR_WORKSPACE: return "CHELA_ERR_WORKSPACE: workspace too small or allocation failed";
        case CHELA_ERR_HIP: return "CHELA_ERR_HIP: a HIP runtime call failed";
        default: return "CHELA: unknown status";
    }
}

int chela_version(void) { return CHELA_VERSION; }

int chela_copy_probe(const void* src, void* dst, size_t bytes, void* stream)
{
    if (bytes == 0) return CHELA_OK;
    if (!src || !dst) return CHELA_ERR_NULL_POINTER;
    if (((uintptr_t)src | (uintptr_t)dst | (uintptr_t)bytes) & 15u) return CHELA_ERR_MISALIGNED;
    if (overlap(Range{(const char*)src, bytes}, Range{(const char*)dst, bytes})) return CHELA_ERR_ALIASING;
    return launch_copy(src, dst, bytes, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_stream_probe(const void* const* in, int n_in, void* const* out, int n_out, size_t bytes, void* stream)
{
    if (n_in < 1 || n_in > 4 || n_out < 0 || n_out > 4) return CHELA_ERR_BAD_SHAPE;
    if (bytes == 0) return CHELA_OK;
    if (!in || (n_out > 0 && !out)) return CHELA_ERR_NULL_POINTER;
    if (bytes & 15u) return CHELA_ERR_MISALIGNED;
    for (int k = 0; k < n_in; ++k) {
        if (!in[k]) return CHELA_ERR_NULL_POINTER;
        if ((uintptr_t)in[k] & 15u) return CHELA_ERR_MISALIGNED;
    }
    for (int k = 0; k < n_out; ++k) {
        if (!out[k]) return CHELA_ERR_NULL_POINTER;
        if ((uintptr_t)out[k] & 15u) return CHELA_ERR_MISALIGNED;
        const Range ro{(const char*)out[k], bytes};
        for (int i = 0; i < n_in; ++i)
            if (overlap(ro, Range{(const char*)in[i], bytes})) return CHELA_ERR_ALIASING;
        for (int j = k + 1; j < n_out; ++j)
            if (overlap(ro, Range{(const char*)out[j], bytes})) return CHELA_ERR_ALIASING;
    }
    return launch_stream_probe(in, n_in, out, n_out, bytes, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_mfma_probe(float* out, int blocks, int iters, void* stream)
{
    if (blocks < 0 || iters < 0 || blocks > (1 << 20) || iters > (1 << 24)) return CHELA_ERR_BAD_SHAPE;
    if (blocks == 0) return CHELA_OK;
    if (!out) return CHELA_ERR_NULL_POINTER;
    if ((uintptr_t)out & 15u) return CHELA_ERR_MISALIGNED;
    return launch_mfma_probe(out, blocks, iters, (hipStream_t)stream) == hipSuccess ? CHELA_OK : CHELA_ERR_HIP;
}

int chela_profile_enable(int on) { g_prof_on = (on != 0); return CHELA_OK; }

int chela_profile_num_kernels(void) { return KID_COUNT; }

const char* chela_profile_kernel_name(int id) { return (id >= 0 && id < KID_COUNT) ? kKernelNames[id] : ""; }

int chela_profile_read(int id, long long* launches, double* total_ms)
{
    if (id < 0 || id >= KID_COUNT || !launches || !total_ms) return CHELA_ERR_BAD_SHAPE;
    long long n = 0;
    double ms = 0.0;
    for (const ProfRec& r : g_prof) {
        if (r.id != id) continue;
        if (hipEventSynchronize(r.b) != hipSuccess) return CHELA_ERR_HIP;
        float t = 0.f;
        if (hipEventElapsedTime(&t, r.a, r.b) != hipSuccess) return CHELA_ERR_HIP;
        ms += t; ++n;
    }
    *launches = n; *total_ms = ms;
    return CHELA_OK;
}

void chela_profile_reset(void)
{
    for (const ProfRec& r : g_prof) g_prof_free.push_back(r);
    g_prof.clear();
}

void chela_shutdown(void)
{
    std::lock_guard<std::mutex> lk(g_mu);
    int cur = 0;
    bool have_cur = false;
    for (int d = 0; d < kMaxDev; ++d) {
        if (g_own_ws[d].empty()) continue;
        if (!have_cur) { have_cur = (hipGetDevice(&cur) == hipSuccess); }
        if (hipSetDevice(d) == hipSuccess) {
            (void)hipDeviceSynchronize();
            for (OwnWs& w : g_own_ws[d]) if (w.ptr) (void)hipFree(w.ptr);
        }
        g_own_ws[d].clear();
    }
    if (have_cur) (void)hipSetDevice(cur);
}

}  // extern "C"
