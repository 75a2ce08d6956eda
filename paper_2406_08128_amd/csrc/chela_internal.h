// Internal declarations shared by the translation units of libchela.so (not installed).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace chela {

// How one call is cut up.  A (b,h) sequence of N tokens is split into n_seg segments of seg_len tokens
// (a multiple of the chunk); one workgroup walks one segment chunk by chunk with the d_k x d_v state in
// registers, starting from a state that a cheap pre-pass (segment totals + scan) provides.
struct Plan {
    int chunk;     // tokens per chunk actually used by the kernels
    int seg_len;   // tokens per segment, multiple of chunk
    int n_seg;     // segments per (b,h); 1 means no pre-pass and no workspace
    size_t state_elems;  // dk*dv
    size_t ws_bytes;     // scratch bytes for the whole call
    int ckpt_every;      // bf16 backward with a single segment: the sweep's first pass leaves the running state every
                         // ckpt_every chunks and its walk back picks those copies up again (0: none needed)
};

// The sweeps add the segment totals up themselves (no scan kernel) while one (b,h) pair's totals stay below this:
// every workgroup re-reads, on average, half of them from the L2.
constexpr size_t kMaxFoldedStateBytes = (size_t)256 << 10;

// The memory-side cache holds 256 MB.  A backward call whose four input tensors come to more than this reads two of
// them (dO, Q) with the streaming hint in its pre-pass, so that the other two stay cached for the sweep.
constexpr size_t kStreamPairAboveBytes = (size_t)224 << 20;

// Checkpoints of a single-segment backward: how many, and where they live ([BH][n][dk*dv] fp32 at the workspace's start).
inline long plan_n_ckpt(const Plan& p, int N)
{
    if (p.ckpt_every <= 0) return 0;
    const long n_ch = ((long)N + p.chunk - 1) / p.chunk;
    return (n_ch - 1) / p.ckpt_every;
}

// can_checkpoint: the caller's backward builds the state itself in a first pass over the sequence when there is a
// single segment (the plain calls without carried or saved states), so long single segments are allowed.
Plan make_plan(long BH, int N, int dk, int dv, int chunk, int dtype, bool is_bwd, bool stateful,
               bool can_checkpoint = false);

// scan modes for scan_states()
enum { SCAN_EXCL_PREFIX = 0, SCAN_INCL_PREFIX = 1, SCAN_EXCL_SUFFIX = 2 };

// In-place scan over the segment axis of n_arrays (1 or 2) arrays states[z][BH][n_seg][elems] (fp32), the arrays
// `array_stride` floats apart, array z scanned in mode modes[z].  elems must be a multiple of 4.  init (may be null,
// entries may be null): per-head seeds [BH][elems] of the running sums; init_cols > 0 says the arrays hold the
// transpose of what init holds and gives the arrays' row length.
hipError_t scan_states(float* states, size_t array_stride, int n_arrays, const int* modes, const float* const* init,
                       int init_cols, long BH, int n_seg, int elems, hipStream_t st);

// Streaming copy used to calibrate byte counters.
hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st);
// n_in (1..4) arrays read, n_out (1..4) arrays written, `bytes` each, by a plain grid-stride kernel.
hipError_t launch_zero_fill(float* p, size_t n_floats, hipStream_t st);      // a fill kernel, not a memset node
hipError_t launch_stream_probe(const void* const* in, int n_in, void* const* out, int n_out, size_t bytes,
                               hipStream_t st);
// Matrix-core rate probe: blocks * 4 waves, each issuing iters * 16 bf16 32x32x16 matrix instructions; out: blocks * 256 floats.
hipError_t launch_mfma_probe(float* out, int blocks, int iters, hipStream_t st);

// fp32 path.  `rev` runs the same map on the time-reversed sequence (anti-causal mask), which is what the
// gradient with respect to K and V is (the backward is three calls of this launcher).
hipError_t launch_f32(const float* Q, const float* K, const float* V, float* O, long BH, int N, int dk, int dv,
                      const Plan& plan, bool rev, float* ws, hipStream_t st, bool reuse_states_T = false);

// bf16 path.  S_in / S_out / dS_out / dS_in: optional carried states and their gradients, [BH][dk][dv] fp32.
// saved (optional): the forward writes the running state at the end of every save_every-th of its segments and of
// the last one, [BH][ceil(n_seg / save_every)][dv][dk] fp32; given to the backward (whose plan must have exactly
// those segments) it replaces the pre-pass over K and V.
hipError_t launch_bf16_fwd(const void* Q, const void* K, const void* V, void* O, const float* S_in, float* S_out,
                           float* saved, int save_every, long BH, int N, int dk, int dv, const Plan& plan, float* ws,
                           hipStream_t st);
hipError_t launch_bf16_bwd(const void* Q, const void* K, const void* V, const void* dO, const float* S_in,
                           const float* dS_out, void* dQ, void* dK, void* dV, float* dS_in, const float* saved,
                           long BH, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st);
// The two plans of a forward call that saves states and the backward call that uses them: the backward's segment
// length is save_every times the forward's.
struct TrainPlans { Plan fwd, bwd; int save_every; };
TrainPlans make_train_plans(long BH, int N, int dk, int dv, int chunk);
// The same two maps for [B,N,H,d] tensors; plan.chunk must be 64.
hipError_t launch_bf16_fwd_nh(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk, int dv,
                              const Plan& plan, float* ws, hipStream_t st);
hipError_t launch_bf16_bwd_nh(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK, void* dV,
                              int B, int H, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st);
// Eq. 11-12 variants: Z [BH][N][dk] stands in for Q and K, aff = [4][H][dk] fp32 (alpha_q, beta_q, alpha_k, beta_k).
// plan.chunk must be 64.  The backward needs zbwd_extra_ws_bytes() of workspace behind plan.ws_bytes.
// `saved` as for launch_bf16_fwd / launch_bf16_bwd (optional).
hipError_t launch_bf16_zfwd(const void* Z, const float* aff, const void* V, void* O, float* saved, int save_every,
                            int B, int H, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st);
hipError_t launch_bf16_zbwd(const void* Z, const float* aff, const void* V, const void* dO, void* dZ, float* d_aff,
                            void* dV, const float* saved, int B, int H, int N, int dk, int dv, const Plan& plan,
                            float* ws, hipStream_t st);
// Eq. 9 epilogue Y = Norm(O) * G (Norm: x / sqrt(mean x^2 + eps) over a head's dv features).
// launch_bf16_fwd_gated: the causal forward with the epilogue fused; O optional, aff optional (Eq. 11-12 prologue),
// saved as for launch_bf16_fwd.  launch_gate_norm: the epilogue alone on [rows][dv]; dY null: out0 = Y; dY given:
// out0 = dO, out1 = dG.
hipError_t launch_bf16_fwd_gated(const void* Q, const void* K, const void* V, const void* G, void* O, void* Y, float eps,
                                 const float* aff, float* saved, int save_every, int B, int H, int N, int dk, int dv,
                                 const Plan& plan, float* ws, hipStream_t st);
hipError_t launch_gate_norm(const void* O, const void* G, const void* dY, void* out0, void* out1, float eps, long rows,
                            int dv, hipStream_t st);
inline size_t zbwd_extra_ws_bytes(long BH, const Plan& plan, int dk)
{
    return (size_t)BH * plan.n_seg * 4 * dk * sizeof(float);
}
// Non-causal form O = Q (K^T V) and its gradient.  `plan` comes from make_noncausal_plan(): n_seg / seg_len split
// the pre-pass, ws holds one (forward) or two (backward) arrays of BH * n_seg states.
Plan make_noncausal_plan(long BH, int N, int dk, int dv, bool is_bwd);
// G non-null: the Eq. 9 epilogue is applied on the way out, Y = Norm(O) * G; O may then be null.
hipError_t launch_bf16_noncausal_fwd(const void* Q, const void* K, const void* V, void* O, long BH, int N, int dk,
                                     int dv, const Plan& plan, float* ws, hipStream_t st, const void* G = nullptr,
                                     void* Y = nullptr, float eps = 0.f);
hipError_t launch_bf16_noncausal_bwd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK,
                                     void* dV, long BH, int N, int dk, int dv, const Plan& plan, float* ws,
                                     hipStream_t st);
// gate (optional, [BH][dv] bf16): o leaves as Norm(o) * gate with the given eps.
hipError_t launch_bf16_step(const void* q, const void* k, const void* v, float* S, void* o, const void* gate, float eps,
                            long BH, int dk, int dv, hipStream_t st);

// Short-long convolutions (Sec. 4.2).  conv_fft_size(L): length M of the complex transform used for sequences of
// L steps (0: L too long); the kernel spectrum is [d][M/2 + 1] pairs of complex fp32.  dtype 0: bf16 I/O, 1: fp32 I/O.
int conv_fft_size(int L);
// Longer sequences (16384 < L <= kConvMaxL) are convolved block by block, 16384 steps per block: the number of
// blocks (0: L is served by one transform, or too long).  The spectrum buffer then holds one spectrum per channel
// and block, [d][blocks][8193] pairs of complex fp32.
constexpr int kConvMaxL = 1 << 20;
inline int conv_blocks(int L) { return (L > 16384 && L <= kConvMaxL) ? (L + 16383) / 16384 : 0; }
inline size_t conv_blocked_spectrum_bytes(int d, int L)
{
    return (size_t)d * (size_t)conv_blocks(L) * 8193 * 4 * sizeof(float);
}
hipError_t launch_longconv_spectrum(const float* k, void* Kf, int d, int L, hipStream_t st);
// The forward convolution on the matrix cores (bf16 I/O, 4096 < L <= 16384): its own copy of the kernel spectrum
// (convmx_spectrum_bytes, derived from the pairs above) lives behind them in the caller's spectrum buffer.
bool convmx_applies(int L, int dtype);
size_t convmx_spectrum_bytes(int d, int L);
hipError_t launch_convmx_spectrum(const float* k_long, const void* pairs, void* extra, int d, int L, hipStream_t st);
hipError_t launch_convmx_fwd(const void* X, const float* w_short, int m, const void* extra, void* Y, int B, int d, int L,
                             hipStream_t st);
// The two long-stage gradients (dV: fp32 for the short-stage kernel, or dX itself in bf16 when there is no short stage;
// Hs: 32768 words of scratch for each of up to kConvMxMaxWgs workgroups).
hipError_t launch_convmx_longbwd(const void* X, const float* w_short, int m, const void* extra, const void* dZ, void* dV,
                                 bool dv_is_f32, float* dk, float* Hs, int B, int d, int L, hipStream_t st);
inline size_t conv_pairs_bytes(int d, int L)       // the (K[k], K[M-k]) pairs: where the matrix-core copy starts
{
    const int M = conv_fft_size(L);
    return M ? (((size_t)d * (size_t)(M / 2 + 1) * 4 * sizeof(float)) + 255) & ~(size_t)255 : 0;
}
hipError_t launch_shortlong_conv(const void* X, const float* w_short, int m, const void* Kf, void* Y, long BD, int d,
                                 int L, int dtype, hipStream_t st);
// Gradient: dX [B][d][L] (I/O dtype), dw [d][m] (only with a short kernel, m <= 32), dk [d][L] fp32.
// ws: conv_bwd_acc_floats(B, d, L) floats (running sums of the long-kernel gradient: at the largest transform size
// they no longer fit the registers of 1024 threads, and workgroups that share a channel leave their shares there), then, with a short kernel, B*d*L floats (dV) and the workgroups' tap
// sums.
// Workgroups that share a channel in the long-stage gradient kernel (each takes every G-th sequence): more than one
// when the channels alone would leave the GPU underfilled.
constexpr int kConvMxMaxWgs = 256;       // workgroups of the matrix-core gradient kernel at most
inline int conv_bwd_groups(int B, int d, int L)
{
    const int M = conv_fft_size(L);
    if (M == 0 || B <= 1 || d <= 0) return 1;
    // resident workgroups of that kernel: 256 compute units x what its registers allow per unit (workgroups of 1, 1, 4
    // and 16 waves at M = 256, 1024, 4096, 16384)
    const long slots = 256L * (M >= 16384 ? 1 : M >= 4096 ? 3 : M >= 1024 ? 12 : 20);
    long g = (2 * slots + d - 1) / d;
    if (g > B) g = B;
    if (g > 64) g = 64;
    return g < 1 ? 1 : (int)g;
}
inline size_t conv_bwd_acc_floats(int B, int d, int L, bool bf16_io)
{
    if (conv_blocks(L)) return conv_blocked_spectrum_bytes(d, L) / sizeof(float);    // one sum per channel and block distance
    const int M = conv_fft_size(L), G = conv_bwd_groups(B, d, L);
    const size_t pairs = (M >= 16384 || G > 1) ? (size_t)G * d * (M / 2 + 1) * 4 : 0;
    // (the matrix-core kernel -- bf16 I/O, 4096 < L <= 16384, L a multiple of 8 -- parks one spectrum of half-precision
    // pairs per workgroup; sized for either kernel, whichever runs)
    const size_t mx = (bf16_io && M >= 16384 && (L & 7) == 0) ? (size_t)kConvMxMaxWgs * 32768 : 0;
    return pairs > mx ? pairs : mx;
}
hipError_t launch_shortlong_conv_bwd(const void* X, const float* w_short, int m, const void* Kf, const void* dZ,
                                     void* dX, float* dw, float* dk, float* ws_dV, int B, int d, int L, int dtype,
                                     hipStream_t st);

// Kernel classes for the per-kernel timing aid.
enum { KID_SEG_STATE_BF16 = 0, KID_SCAN = 1, KID_FWD_SWEEP_BF16 = 2, KID_BWD_SWEEP_BF16 = 3, KID_SEG_STATE_F32 = 4,
       KID_SWEEP_F32 = 5, KID_COPY = 6, KID_STEP_BF16 = 7, KID_AFFINE_GRAD = 8, KID_APPLY_BF16 = 9, KID_CONV_SPECTRUM = 10, KID_CONV_FWD = 11, KID_CONV_SHORT_BWD = 12, KID_CONV_LONG_BWD = 13, KID_GATE_NORM = 14, KID_STREAM_PROBE = 15, KID_MFMA_PROBE = 16, KID_COUNT = 17 };

// Brackets one kernel launch with HIP events on its stream while profiling is enabled; otherwise does nothing.
struct ProfScope {
    ProfScope(int id, hipStream_t st);
    ~ProfScope();
    int slot;
    hipStream_t st;
};

}  // namespace chela
