/*
 * chela.h -- C ABI of libchela.so: causal linear attention for AMD gfx950 (MI355X).
 *
 * The operation is the hardware-efficient linear attention of CHELA Sec. 4.1:
 * given Q, K, V it returns
 *
 *        O[b,h,t,:] = sum_{s <= t} ( Q[b,h,t,:] . K[b,h,s,:] ) * V[b,h,s,:]
 *
 * i.e. the right-product linear attention of Sec. 2.1 Eq. 2 under a causal mask
 * that includes the diagonal, evaluated block-wise as Sec. 4.1 describes: the
 * masked left product (Q K^T) V inside a block of `chunk` tokens, the right
 * product Q (K^T V) between blocks through a d_k x d_v state that is carried
 * on chip, the two parts summed before the result goes to HBM.  Norm, the
 * 1/sqrt(d) scale and any feature map are NOT applied: callers pre-scale Q, K.
 * The backward entry points return the exact gradient of that map (the paper
 * times a backward pass, Fig. 4, but does not describe one).
 *
 * Conventions for every entry point
 *   Pointers : DEVICE pointers (hipMalloc'ed or owned by a framework such as
 *              PyTorch), 16-byte aligned, valid on the current HIP device.
 *   Layout   : [B, H, N, d] contiguous, d fastest.  Q, K, dQ, dK use d = dk;
 *              V, O, dO, dV use d = dv.  No strides.
 *   Dtype    : *_fwd / *_bwd take bfloat16 tensors and accumulate in fp32
 *              (scores and states are rounded to bf16 only as matrix-core
 *              operands); *_f32 take and return IEEE fp32.
 *   Shapes   : B, H, N >= 0 (any of them 0 -> nothing is done, success);
 *              dk, dv in {64, 128}; chunk in {64, 128} for bf16 and
 *              {16, 32, 64} for fp32.  N need not be a multiple of chunk.
 *              `chunk` is a tiling choice: it never changes the result beyond
 *              floating-point re-association.
 *   Ownership: the caller owns all tensors; the library keeps no reference
 *              once the enqueued work has finished.  Outputs are overwritten,
 *              never accumulated into, and must not overlap any input.
 *   Stream   : `stream` is a hipStream_t passed as void* (NULL = the default
 *              stream).  Work is enqueued and the call returns without
 *              synchronising.
 *   Scratch  : per-(b,h)-segment states, chela_linattn_workspace_bytes() bytes.
 *              Taken from the buffer the CALLING THREAD gave to
 *              chela_set_workspace(), else from an allocation of the library's
 *              own, one per (device, stream), that grows on demand (growing it
 *              synchronises the device) and lives until chela_shutdown(); at most
 *              64 streams per device are served this way, the next one gets
 *              CHELA_ERR_WORKSPACE (hand in buffers, or shut down in between).
 *   Threads  : calls may be made from several host threads at once.  Calls that
 *              may overlap in time must not share scratch: the library's own
 *              allocations never are shared between streams; a caller-owned
 *              buffer belongs to the thread that set it, and that thread must
 *              not use it on two streams whose work may overlap (it sets another
 *              buffer before the calls on the other stream: a call's kernels
 *              use the buffer that was in force when the call was made).
 *   Errors   : 0 on success, a negative CHELA_ERR_* otherwise.  Every argument
 *              check is done on the host before the first HIP call, so a
 *              rejected call has touched nothing.  No exceptions, no abort.
 */
#ifndef CHELA_H
#define CHELA_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CHELA_VERSION 100 /* 0.1.0 */

enum {
    CHELA_OK                  = 0,
    CHELA_ERR_NULL_POINTER    = -1, /* a tensor pointer is NULL while B*H*N > 0            */
    CHELA_ERR_BAD_SHAPE       = -2, /* B, H or N negative, or element count overflows      */
    CHELA_ERR_UNSUPPORTED_DIM = -3, /* dk or dv not in {64, 128}                           */
    CHELA_ERR_BAD_CHUNK       = -4, /* chunk not in the supported set for this dtype       */
    CHELA_ERR_MISALIGNED      = -5, /* a tensor pointer is not 16-byte aligned             */
    CHELA_ERR_ALIASING        = -6, /* an output range overlaps an input or another output */
    CHELA_ERR_WORKSPACE       = -7, /* caller workspace too small / allocation failed      */
    CHELA_ERR_HIP             = -8  /* a HIP call failed (launch, allocation, no device)   */
};

enum { CHELA_DTYPE_BF16 = 0, CHELA_DTYPE_F32 = 1 };

/* Forward, bf16 I/O, fp32 accumulation (Sec. 4.1; Eq. 2 with the causal mask).
 * Q, K: [B,H,N,dk] in; V: [B,H,N,dv] in; O: [B,H,N,dv] out. */
int chela_linattn_fwd(const void *Q, const void *K, const void *V, void *O,
                      int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* Backward of the map above, bf16 I/O, fp32 accumulation.  Nothing is saved by
 * the forward call: the states are recomputed from Q, K, V, dO.
 *   dQ_t = sum_{s<=t} (dO_t . v_s) k_s
 *   dK_s = sum_{t>=s} (dO_t . v_s) q_t
 *   dV_s = sum_{t>=s} (q_t . k_s) dO_t
 * dO: [B,H,N,dv] in; dQ, dK: [B,H,N,dk] out; dV: [B,H,N,dv] out.
 * The sweep walks a stretch of a sequence (at most 8192 tokens) from its end to its start and obtains the state in
 * front of each chunk by subtracting the chunk's K^T V from the state behind it, in fp32.  Two consequences: dQ_t
 * depends on the keys and values AFTER t within such a stretch through rounding of the order of 1e-7 of the state
 * (never through more: the exact terms cancel), and a non-finite key or value row makes dQ non-finite for the
 * earlier tokens of its stretch as well as for the later ones.  dK and dV depend on nothing before their token. */
int chela_linattn_bwd(const void *Q, const void *K, const void *V, const void *dO,
                      void *dQ, void *dK, void *dV,
                      int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* chela_linattn_fwd for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  Same arguments, same kernels and the same result as chela_linattn_fwd
 * (bf16 I/O), but the per-segment states live in a fixed array of device memory that is part of the library's code
 * object (32 MiB; every GPU the library runs on holds its own copy until the process ends), so the call never
 * calls hipMalloc, hipFree or any allocating routine, whatever chela_set_workspace() was given.
 *   Limit    : problems whose segment states need more than 32 MiB
 *              (chela_linattn_workspace_bytes(B, H, N, dk, dv, chunk, 0, CHELA_DTYPE_BF16) says how much) are rejected
 *              with CHELA_ERR_WORKSPACE before anything is enqueued.  All five benchmark shapes fit.
 *   Set-up   : the first call on a device asks the runtime for the array's address on that device (the device must
 *              be current, as for every call); make that first call outside a graph capture.
 *   Sharing  : all calls on one GPU use that GPU's one array, which keeps the previous call's contents (nothing in
 *              it has to start at zero: every slot that is read has been written by the same call first).  Calls
 *              that may overlap in time on one GPU -- two streams, two threads -- race on it: serialise them, or use
 *              chela_linattn_fwd with a workspace per stream. */
int chela_linattn_fwd_noalloc(const void *Q, const void *K, const void *V, void *O,
                              int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* The same two maps with fp32 tensors and fp32 arithmetic throughout. */
int chela_linattn_fwd_f32(const void *Q, const void *K, const void *V, void *O,
                          int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_bwd_f32(const void *Q, const void *K, const void *V, const void *dO,
                          void *dQ, void *dK, void *dV,
                          int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* ---- the same two maps for tensors laid out [B, N, H, d] (all heads of a token next to each other, which is how
 * a projection `X W` leaves them: no transposition pass is needed before or after).  bf16 I/O; Q, K, dQ, dK are
 * [B,N,H,dk], V, O, dO, dV are [B,N,H,dv], contiguous.  64-token chunks (`chunk` is validated, {64, 128}, and
 * otherwise ignored).  Scratch as for chela_linattn_fwd / _bwd with chunk 64.  Everything else as above. */
int chela_linattn_fwd_bnhd(const void *Q, const void *K, const void *V, void *O,
                           int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_bwd_bnhd(const void *Q, const void *K, const void *V, const void *dO,
                           void *dQ, void *dK, void *dV,
                           int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* ---- carried state (segment-wise processing, Sec. 5.3 / App. A: sequences are cut into segments that are
 * processed one after the other; the running d_k x d_v state is all one segment hands to the next) ------------
 * Same maps as above, bf16 I/O, with the state made explicit.  States are fp32, [B, H, dk, dv], 16-byte aligned.
 *   forward : S_0 = S_in (NULL: zero);  O_t = q_t . (S_in + sum_{s<=t} k_s v_s^T);  S_out = S_in + sum_s k_s v_s^T
 *             (NULL: not written).  S_out may equal S_in (update in place).
 *   backward: for upstream gradients dO and dS_out (NULL: zero) returns dQ, dK, dV and, unless NULL,
 *             dS_in = dS_out + sum_t q_t dO_t^T.  dS_in may equal dS_out.
 * With N = 0 the state passes through (S_out = S_in, dS_in = dS_out).  Everything else as for the calls above. */
int chela_linattn_fwd_state(const void *Q, const void *K, const void *V, const float *S_in,
                            void *O, float *S_out,
                            int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_bwd_state(const void *Q, const void *K, const void *V, const float *S_in,
                            const void *dO, const float *dS_out,
                            void *dQ, void *dK, void *dV, float *dS_in,
                            int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* ---- queries and keys from one tensor (Sec. 4.3, Eq. 11-12: Q = alpha_q * Z + beta_q, K = alpha_k * Z + beta_k,
 * learnable per-feature scales and offsets) --------------------------------------------------------------------
 * Same map as chela_linattn_fwd / _bwd, bf16 I/O, but the library reads Z once and forms Q and K on chip, so the
 * forward moves three tensors instead of four and the backward five instead of seven.
 *   Z        : [B,H,N,dk] bf16 in.
 *   affine   : [4,H,dk] fp32 in, rows alpha_q, beta_q, alpha_k, beta_k: head h owns its dk-slice of the four
 *              d-vectors; broadcast over batch and tokens.  Q and K are computed in fp32 and rounded to bf16 once,
 *              as matrix-core operands.
 *   forward  : O[b,h,t,:] = sum_{s<=t} (q_t . k_s) v_s.
 *   backward : dZ = alpha_q * dQ + alpha_k * dK ([B,H,N,dk] bf16 out), dV as before, and
 *              d_affine ([4,H,dk] fp32 out, overwritten) = (sum dQ*Z, sum dQ, sum dK*Z, sum dK), sums over batch and
 *              tokens, accumulated in fp32 from the fp32 dQ, dK (deterministic: fixed summation order).
 * The kernels use 64-token chunks; `chunk` is validated ({64, 128}) and otherwise ignored.  Scratch:
 * chela_linattn_z_workspace_bytes().  With B*H*N = 0 nothing is done, except that d_affine is zeroed if H > 0.
 * Everything else (pointers, alignment, aliasing, stream, errors) as for the calls above. */
int chela_linattn_zfwd(const void *Z, const float *affine, const void *V, void *O,
                       int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_zbwd(const void *Z, const float *affine, const void *V, const void *dO,
                       void *dZ, float *d_affine, void *dV,
                       int B, int H, int N, int dk, int dv, int chunk, void *stream);
size_t chela_linattn_z_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk, int is_bwd);
/* The same two calls as a training pair (see chela_linattn_fwd_save below): `saved` is a caller-owned buffer of
 * chela_linattn_saved_bytes(B, H, N, dk, dv, 64) bytes that carries the boundary states from the forward to the
 * backward call, which then needs no pass over K(Z), V to rebuild them. */
int chela_linattn_zfwd_save(const void *Z, const float *affine, const void *V, void *O, void *saved,
                            int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_zbwd_saved(const void *Z, const float *affine, const void *V, const void *dO, const void *saved,
                             void *dZ, float *d_affine, void *dV,
                             int B, int H, int N, int dk, int dv, int chunk, void *stream);

/* ---- training pair: forward that leaves the running state for the backward ------------------------------------
 * chela_linattn_bwd rebuilds the state at its segment boundaries from K and V (one extra pass over both).  In a
 * training step the forward call has just walked those states: chela_linattn_fwd_save writes them (fp32, at the
 * boundaries the backward will use) into `saved`, a caller-owned device buffer of chela_linattn_saved_bytes() bytes
 * (16-byte aligned, opaque), and chela_linattn_bwd_saved reads them back instead of re-reading K and V.  Same
 * results as chela_linattn_fwd / _bwd up to floating-point re-association (the segment split may differ).
 * `saved` must reach the backward call unchanged, with the same B, H, N, dk, dv and chunk, in the same process (its
 * layout follows the library's work split for the current GPU).  bf16 I/O; everything else as for the plain calls. */
int chela_linattn_fwd_save(const void *Q, const void *K, const void *V, void *O, void *saved,
                           int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_bwd_saved(const void *Q, const void *K, const void *V, const void *dO, const void *saved,
                            void *dQ, void *dK, void *dV,
                            int B, int H, int N, int dk, int dv, int chunk, void *stream);
size_t chela_linattn_saved_bytes(int B, int H, int N, int dk, int dv, int chunk);
/* Scratch of the training pair, which splits the sequences on a grid of its own (the forward cuts wherever the
 * backward will want a state): bytes chela_linattn_fwd_save and the gated forwards given `saved` (is_bwd = 0) or
 * chela_linattn_bwd_saved (is_bwd = 1) take from the workspace; 0 for invalid arguments. */
size_t chela_linattn_train_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk, int is_bwd);

/* ---- non-causal form (Sec. 2.1, Eq. 2 as written, without Norm): O = Q (K^T V), every token sees every token.
 * This is what the paper's sequence classifiers run (no mask); bf16 I/O, fp32 accumulation, the d_k x d_v matrix
 * K^T V rounded to bf16 once as a matrix-core operand.  Two passes: K^T V summed over the sequence, then O = Q S for
 * independent blocks of tokens.  The backward returns, with S = K^T V and R = Q^T dO,
 *     dQ = dO S^T,  dK = V R^T,  dV = K R.
 * Tensors, layout, alignment, aliasing rules, stream and errors as for chela_linattn_fwd / _bwd (there is no chunk
 * argument: nothing here is sequential).  Scratch: chela_linattn_noncausal_workspace_bytes(). */
int chela_linattn_noncausal_fwd(const void *Q, const void *K, const void *V, void *O,
                                int B, int H, int N, int dk, int dv, void *stream);
int chela_linattn_noncausal_bwd(const void *Q, const void *K, const void *V, const void *dO,
                                void *dQ, void *dK, void *dV,
                                int B, int H, int N, int dk, int dv, void *stream);
size_t chela_linattn_noncausal_workspace_bytes(int B, int H, int N, int dk, int dv, int is_bwd);

/* ---- gated, normalised output (Sec. 4.3, Eq. 9: M = Norm(Q (K^T V)) * G_a) ---------------------------------------
 * The paper attributes Norm to the TransNormer line of work (Sec. 2.1) and does not write it out; this library takes
 * the root-mean-square normalisation without learnable gain, per token and per head over that head's dv features:
 *        Norm(o) = o / sqrt(mean_j o_j^2 + eps),      Y = Norm(O) * G            (eps >= 0, a finite constant;
 * with eps = 0 an all-zero row of O gives NaN, as the formula does).  The gate G ([B,H,N,dv] bf16) is an input: the
 * projection and activation that produce it (Eq. 10) are dense layers outside this library.
 *   chela_linattn_fwd_gated : O as chela_linattn_fwd computes it, then Y, in one pass: the sum of squares is taken
 *       from the fp32 accumulators, so Y is rounded once.  Y [B,H,N,dv] bf16 out.  O: bf16 out or NULL (a backward
 *       pass needs O, inference does not: with NULL the call moves the same five tensors as the plain forward plus
 *       the gate).  saved: NULL, or the buffer of the training pair below (chela_linattn_saved_bytes(..., 64)
 *       bytes), filled for chela_linattn_bwd_saved / _zbwd_saved.
 *   chela_linattn_zfwd_gated: the same with the Eq. 11-12 prologue (Z, affine as for chela_linattn_zfwd).
 *   chela_gate_norm_fwd     : the epilogue alone on `rows` rows of dv features (any [..., dv] tensor, contiguous),
 *       e.g. behind the non-causal call.  rows >= 0; dv in {64, 128}.
 *   chela_gate_norm_bwd     : its gradient,  dG = dY * Norm(O),  dO = r (u - n mean_j(u_j n_j))  with
 *       r = 1 / sqrt(mean_j o_j^2 + eps), n = r o, u = dY * G.  dO is what the attention backward calls take as their
 *       dO.  dO may be the same buffer as dY (exactly the same pointer); no other overlap is allowed.
 * 64-token chunks (`chunk` validated and otherwise ignored); scratch as for chela_linattn_fwd / _zfwd; a negative or
 * non-finite eps gives CHELA_ERR_BAD_SHAPE.  Everything else as for the calls above. */
int chela_linattn_fwd_gated(const void *Q, const void *K, const void *V, const void *G, void *O, void *Y, void *saved,
                            float eps, int B, int H, int N, int dk, int dv, int chunk, void *stream);
int chela_linattn_zfwd_gated(const void *Z, const float *affine, const void *V, const void *G, void *O, void *Y,
                             void *saved, float eps, int B, int H, int N, int dk, int dv, int chunk, void *stream);
/* The non-causal form with the same epilogue, Y = Norm(Q (K^T V)) * G (what the paper's classifiers run): the second
 * kernel of chela_linattn_noncausal_fwd normalises and gates its output tiles on the way out.  O: bf16 out or NULL.
 * Scratch: chela_linattn_noncausal_workspace_bytes(..., 0). */
int chela_linattn_noncausal_fwd_gated(const void *Q, const void *K, const void *V, const void *G, void *O, void *Y,
                                      float eps, int B, int H, int N, int dk, int dv, void *stream);
int chela_gate_norm_fwd(const void *O, const void *G, void *Y, float eps, long long rows, int dv, void *stream);
int chela_gate_norm_bwd(const void *O, const void *G, const void *dY, void *dO, void *dG, float eps, long long rows,
                        int dv, void *stream);

/* ---- short-long convolutions (Sec. 4.2, Eq. 8): Z = K_l( silu( K_s(X) ) ), the other half of the token mixer -----
 * Depthwise (one kernel per channel) and causal with zero history:
 *     v[b,c,t] = silu( sum_{j<m, j<=t} w_short[c,j] * X[b,c,t-j] ),   Z[b,c,t] = sum_{s<=t} k_long[c,s] * v[b,c,t-s].
 *   X, Z     : [B, d, L] (time fastest), bf16 (plain name) or fp32 (_f32).  Arithmetic is fp32 throughout, with one
 *              exception: bf16 I/O with 4096 < L <= 16384, L a multiple of 8, runs the transforms on the matrix
 *              cores with half-precision operands and fp32 sums (input scaled by its largest magnitude, kernel by
 *              its 1-norm, so no range is lost): 5e-4 relative before the output is rounded to bf16 (2e-3).
 *   w_short  : [d, m] fp32, 1 <= m <= 32: the paper's two parallel short kernels (sizes 3 and 2 log10(L) + 1) summed
 *              tap by tap into one, i.e. after the structural re-parameterisation of Sec. 4.2.  NULL: no short kernel
 *              and no activation (v = X), a plain long convolution.
 *   k_long   : [d, L] fp32, as long as the sequence.  It enters through its spectrum (Eq. 7: y = F^-1 D_K F u):
 *              chela_longconv_spectrum() turns k_long into `spectrum`, an opaque device buffer of
 *              chela_longconv_spectrum_bytes(d, L) bytes that is valid for this d and L and is reused for every batch
 *              until the kernel's weights change.
 * Sequences are zero-padded on chip to twice a transform length M >= L (M in {256, 1024, 4096, 16384}), which makes
 * the circular product of Eq. 7 equal the causal sum.  16384 < L <= 1048576: the sequence and the kernel are cut into
 * blocks of 16384 steps; every block goes through the same on-chip transform, the products of a block of the input
 * with the blocks of the kernel that reach from it into an output block are added up on the spectra, and one inverse
 * transform per output block follows (fp32 arithmetic for either I/O type; exact up to rounding like the single
 * transform, but its work grows with the square of the number of blocks, and `spectrum` holds one spectrum per
 * channel and block: 128 KB each).  L > 1048576 is rejected (CHELA_ERR_BAD_SHAPE).  The forward needs no scratch.  Pointers 16-byte aligned; Z must not overlap an input.  Everything else as for the calls above.
 * Environment (read per call, tuning aid): CHELA_CONV_MATRIX=0 keeps the vector-ALU kernels for every size. */
size_t chela_longconv_spectrum_bytes(int d, int L);
int chela_longconv_spectrum(const float *k_long, void *spectrum, int d, int L, void *stream);
int chela_shortlong_conv_fwd(const void *X, const float *w_short, int m, const void *spectrum, void *Z,
                             int B, int d, int L, void *stream);
int chela_shortlong_conv_fwd_f32(const void *X, const float *w_short, int m, const void *spectrum, void *Z,
                                 int B, int d, int L, void *stream);
/* Gradient of the map above for an upstream gradient dZ [B,d,L] (the paper gives no backward: this is the exact
 * gradient of the two sums).  With u = K_s(X), v = silu(u):
 *     dv[t] = sum_{s>=t} k_long[s-t] dZ[s]              (correlation with the long kernel: its conjugate spectrum)
 *     d_k_long[c,s] = sum_b sum_{t>=s} dZ[b,c,t] v[b,c,t-s]         ([d,L] fp32 out, overwritten)
 *     du = dv * silu'(u),  dX[t] = sum_j w_short[j] du[t+j]         ([B,d,L] out, I/O dtype)
 *     d_w_short[c,j] = sum_b sum_t du[b,c,t] X[b,c,t-j]             ([d,m] fp32 out, overwritten)
 * bf16 I/O with 4096 < L <= 16384, L a multiple of 8, runs the long-stage transforms on the matrix cores like the
 * forward (half-precision operands, fp32 sums): d_k_long and d_w_short, although they leave as fp32, then carry
 * 3e-4 .. 8e-4 of relative error instead of 1e-6 (CHELA_CONV_MATRIX=0: the vector-ALU kernels, fp32 throughout).
 * Nothing is saved by the forward call: u and v are recomputed from X.  With w_short = NULL (no short stage) dX = dv,
 * v = X and d_w_short is ignored.  m <= 32 as in the forward.  Scratch (library workspace):
 * chela_shortlong_conv_bwd_workspace_bytes().  Sums over batch and time are taken in a fixed order (deterministic). */
int chela_shortlong_conv_bwd(const void *X, const float *w_short, int m, const void *spectrum, const void *dZ,
                             void *dX, float *d_w_short, float *d_k_long, int B, int d, int L, void *stream);
int chela_shortlong_conv_bwd_f32(const void *X, const float *w_short, int m, const void *spectrum, const void *dZ,
                                 void *dX, float *d_w_short, float *d_k_long, int B, int d, int L, void *stream);
size_t chela_shortlong_conv_bwd_workspace_bytes(int B, int d, int L, int has_short_kernel, int dtype);

/* One decode step of autoregressive inference (the recurrent form, one token per (b,h)):
 *     S += k v^T  (in place, fp32) ;  o = S^T q.
 * q, k: [B, H, dk] bf16; v, o: [B, H, dv] bf16; S: [B, H, dk, dv] fp32.  Needs no scratch. */
int chela_linattn_step(const void *q, const void *k, const void *v, float *S, void *o,
                       int B, int H, int dk, int dv, void *stream);
/* The same step with the Eq. 9 epilogue of chela_linattn_fwd_gated:  y = Norm(S^T q) * g,  g, y: [B, H, dv] bf16,
 * Norm and eps as defined there (the sum of squares is taken from the fp32 o, y is rounded once). */
int chela_linattn_step_gated(const void *q, const void *k, const void *v, const void *g, float *S, void *y, float eps,
                             int B, int H, int dk, int dv, void *stream);

/* Bytes of device scratch one call with these arguments needs, with or without
 * carried states (0 if the arguments are invalid; the training pair has its own query,
 * chela_linattn_train_workspace_bytes).  The size is B*H*dk*dv*4 bytes per segment.
 * Forward: the number of segments per (b,h) is set by the GPU, not by N, so the scratch
 * does not grow with N once the GPU is full -- the fixed-memory property claimed in
 * Sec. 1.  bf16 backward: in addition no segment is longer than 8192 tokens (see
 * chela_linattn_bwd), i.e. at least two states per 8192 tokens of a sequence: 0.4 % of
 * the bytes of the tensors themselves. */
size_t chela_linattn_workspace_bytes(int B, int H, int N, int dk, int dv, int chunk,
                                     int is_bwd, int dtype);

/* Hand the library a caller-owned device buffer to use as scratch (256-byte
 * aligned) for the calls THIS host thread makes from now on.  NULL/0 returns the
 * thread to the library's own allocations.  The buffer must stay valid until
 * every call that used it has finished.  chela_get_workspace reports the calling
 * thread's current setting (NULL, 0 if none). */
int chela_set_workspace(void *dev_ptr, size_t bytes);
int chela_get_workspace(void **dev_ptr, size_t *bytes);

/* Environment variables read by the library (tuning aids for measurements; results stay within the rounding of any
 * other split, defaults are what the planner picks):
 *   CHELA_SEG_TOKENS=n   force segments of n tokens (rounded up to whole chunks) in the causal calls
 *   CHELA_NC_SEGS=n      force n segments per (b,h) in the non-causal pre-pass
 *   CHELA_PREPASS_REV=0  walk the forward pre-pass front to back instead of back to front
 *   CHELA_FOLD_SCAN=0    always scan the segment totals in a kernel of its own (by default the sweep's workgroups add
 *                        them up themselves when the states of one sequence's segments come to at most 256 KB) */

/* Human-readable name of a status code (static storage, never NULL). */
const char *chela_status_string(int status);

/* CHELA_VERSION of the loaded library. */
int chela_version(void);

/* Free the internal workspace (synchronises the device).  Safe to call twice. */
void chela_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* CHELA_H */
