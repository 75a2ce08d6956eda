// Long convolution of Eq. 7-8 (Sec. 4.2) with the transforms on the matrix cores, for bf16 I/O and sequences of
// 4097 .. 16384 steps.
//
// Two sequences of one channel ride in one complex signal z = v_a + i v_b (the kernel is real, so the convolution of
// z has the two results as its real and imaginary part: nothing has to be untangled), zero-padded to N = 32768 = 32^3
// points so that the circular product equals the causal sum.  With n = 1024 n1 + 32 n2 + n3 and k = k1 + 32 k2 +
// 1024 k3 the transform is three passes of the SAME 32-point transform, one along each axis of a 32 x 32 x 32 cube,
// with an element-wise rotation after the first two:
//     X1[k1,n2,n3] = W_N^(k1 (32 n2 + n3)) sum_n1 w^(k1 n1) z[n1,n2,n3]          (w = exp(-2 pi i / 32))
//     X2[k1,k2,n3] = W_1024^(k2 n3)        sum_n2 w^(k2 n2) X1[k1,n2,n3]
//     X [k1,k2,k3] =                       sum_n3 w^(k3 n3) X2[k1,k2,n3]
// The way back is conj(T'(conj P)) where T' takes the axes in the opposite order (3, 2, 1) with the same matrix and
// the same rotations, so one pass routine serves all six passes and nothing is ever reordered.  A 32-point complex
// transform of 32 columns is a real 64 x 64 matrix times a 64 x 32 tile: v_mfma_f32_32x32x16_f16, the matrix in
// registers for the whole kernel (fp16, entries cos / sin of multiples of pi/16), the data as fp16 pairs (re, im)
// in LDS, sums in fp32.  The rows of the matrix are ordered so that the lane that receives a set of results is the
// lane that would have to supply them as operands of a pass along the same axis: the third pass forward, the product
// with the kernel's spectrum and the first pass back happen in registers, without a trip through LDS.
// Ranges: the pair is scaled by 1 / max|v| on the way in (|z| <= sqrt 2, so no sum on the way forward exceeds
// 23171), the kernel's spectrum is stored divided by 4 |k|_1 (so that no sum on the way back exceeds 32768 either:
// the half-precision range ends at 65504); both factors are put back on the way out.  Measured against the fp64
// definition on the workload's recipe: 4.8e-4 relative before the rounding of the output to bf16 (2.3e-3 on its own).
#include "chela_internal.h"
#include <cstdlib>

namespace chela {

typedef __bf16 bf16;
typedef _Float16 f16;
typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

constexpr int MX_N = 32768;                  // points of the complex transform
constexpr int MX_L_MAX = 16384;              // steps of a sequence at most
constexpr int MX_PLANE = 1032;               // words (one complex fp16 pair each) from one n1 plane to the next
constexpr int MX_CUBE = 32 * MX_PLANE;       // 132 096 bytes
constexpr int MX_T = 512;                    // threads: each owns one row of the lower half of the cube (32 steps)
constexpr int MX_W = MX_T / 64;              // waves

// Word of cube element (d1, d2, d3).  Rows (d1, d2) of 32 words; passes along an axis read, per instruction, the same
// columns of two rows that lie 4 apart along that axis (the two half-waves): the plane stride (4 x 1032 = 32 mod 64)
// and the order of the rows within a plane (bit 2 of d2 stored as bit 0) put those on the two halves of the banks.
// The pass along d3 reads and writes 16 bytes per lane with the lanes on consecutive rows: the 16-byte pieces of a
// row are exchanged by the row number so that 16 lanes meet 16 different pieces.
__device__ __forceinline__ int mx_addr(int d1, int d2, int d3)
{
    const int r = (d2 & 24) | ((d2 & 3) << 1) | ((d2 >> 2) & 1);
    return d1 * MX_PLANE + r * 32 + ((((d3 >> 2) ^ (r >> 1)) & 7) << 2) + (d3 & 3);
}

__device__ __forceinline__ f32x16 mx_mfma(f16x8 a, f16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 mx_zero()
{
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// (re, im) -> one word of two halves, round to nearest even
__device__ __forceinline__ unsigned mx_pack(float re, float im)
{
    f16x2 v;
    v[0] = (f16)re;
    v[1] = (f16)im;
    return __builtin_bit_cast(unsigned, v);
}
__device__ __forceinline__ void mx_unpack(unsigned w, float& re, float& im)
{
    const f16x2 v = __builtin_bit_cast(f16x2, w);
    re = (float)v[0];
    im = (float)v[1];
}

// The matrix operand.  Real form of the 32-point transform F[p][q] = exp(-2 pi i p q / 32) acting on (re, im) pairs:
// contraction index kk = 2 q + c_in, rows 2 p + c_out in an order of our choosing.  Accumulator register 4a + b of
// lane (r, h) is row 8a + 4h + b of a 32-row block: we let block rb, row 8a + 4h + b stand for
//     p = 16 rb + 8 (a >> 1) + 4 h + 2 (a & 1) + (b >> 1),   c_out = b & 1,
// so that a lane ends up with the complex results p = 8 s + 4 h + i (s = 2 rb + (a >> 1) = 0..3, i = 0..3): exactly the
// inputs q = 8 s + 4 h + i it has to supply, as four (re, im) words, for step s of a contraction over the same axis.
// Operand layout of the instruction: lane (r, h) holds row r, contraction indices 16 s + 8 h + 0..7.
__device__ __forceinline__ void mx_build_matrix(f16x8 (&A)[2][4], int lane)
{
    const int r = lane & 31, hh = lane >> 5;
    const int a = r >> 3, h = (r >> 2) & 1, b = r & 3;
#pragma unroll
    for (int rb = 0; rb < 2; ++rb) {
        const int p = 16 * rb + 8 * (a >> 1) + 4 * h + 2 * (a & 1) + (b >> 1), c_out = b & 1;
#pragma unroll
        for (int s = 0; s < 4; ++s)
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int kk = 16 * s + 8 * hh + j, q = kk >> 1, c_in = kk & 1;
                float sn, cs;
                sincospif((float)((p * q) & 31) * 0.0625f, &sn, &cs);      // F = cs - i sn
                // re_out = cs x_re + sn x_im ;  im_out = -sn x_re + cs x_im
                const float v = c_out == 0 ? (c_in == 0 ? cs : sn) : (c_in == 0 ? -sn : cs);
                A[rb][s][j] = (f16)v;
            }
    }
}

enum { MX_AX1 = 1, MX_AX2 = 2, MX_AX3 = 3 };
enum { MX_TW_NONE = 0, MX_TW_F1 = 1, MX_TW_T2 = 2, MX_TW_I2 = 3 };

// Element q of column `col` of tile t along the axis: tiles are (n2 | columns n3) along axis 1, (d1 | columns n3)
// along axis 2, (d1 | columns d2) along axis 3.
template <int AX>
__device__ __forceinline__ int mx_word(int t, int col, int q)
{
    return AX == MX_AX1 ? mx_addr(q, t, col) : AX == MX_AX2 ? mx_addr(t, q, col) : mx_addr(t, col, q);
}

template <int AX, int KS>
__device__ __forceinline__ void mx_load(const unsigned* cube, int t, int col, int h, f16x8 (&Bv)[4])
{
#pragma unroll
    for (int s = 0; s < KS; ++s) {
        u32x4 v;
        if (AX == MX_AX3) {
            v = *reinterpret_cast<const u32x4*>(cube + mx_addr(t, col, 8 * s + 4 * h));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = cube[mx_word<AX>(t, col, 8 * s + 4 * h + i)];
        }
        Bv[s] = __builtin_bit_cast(f16x8, v);
    }
}

template <int KS, int RB>
__device__ __forceinline__ void mx_mul(const f16x8 (&A)[2][4], const f16x8 (&Bv)[4], f32x16 (&acc)[2])
{
#pragma unroll
    for (int rb = 0; rb < RB; ++rb) {
        acc[rb] = mx_zero();
#pragma unroll
        for (int s = 0; s < KS; ++s) acc[rb] = mx_mfma(A[rb][s], Bv[s], acc[rb]);
    }
}

// complex result i (0..3) of step s (0..3) in a lane's accumulators: p = 8 s + 4 h + i
__device__ __forceinline__ float mx_re(const f32x16 (&acc)[2], int s, int i) { return acc[s >> 1][4 * (2 * (s & 1) + (i >> 1)) + 2 * (i & 1)]; }
__device__ __forceinline__ float mx_im(const f32x16 (&acc)[2], int s, int i) { return acc[s >> 1][4 * (2 * (s & 1) + (i >> 1)) + 2 * (i & 1) + 1]; }

// The rotations that follow a pass are kept in registers, one per result a lane owns (index 4 s + i for row
// p = 8 s + 4 h + i); reading them from LDS per tile cost more LDS time than the data itself.  With T2[a][b] =
// W_1024^(a b) and T1[a][b] = W_32768^(a b) (32 x 32 tables in LDS, read a few times per pair only):
//   fixed (forward after axis 2: rows k2, columns n3; back after axis 3: rows n3, columns k2):  T2[p][col], the same
//         sixteen numbers for every tile and every pair
//   F1 (forward after axis 1: rows k1 = p, tile n2 = t, columns n3):  W_N^(k1 (32 n2 + n3)) = T1[p][col] T2[p][t]
//   I2 (back after axis 2: rows n2 = p, tile k1 = t, columns n3):     W_N^(k1 (32 n2 + n3)) = T2[p][t] T1[t][col]
//   a wave's tiles are t = w, w + MX_W, ...: the running values are set for t = w and multiplied by the step to the
//   next tile (T2[p][MX_W], times T1[MX_W][col] for I2) after each tile.
struct MxRot { float2 v[16]; };

__device__ __forceinline__ float2 mx_cmul(float2 a, float2 b) { return make_float2(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }

__device__ __forceinline__ void mx_rot_fixed(MxRot& r, const float2* T2, int col, int h)
{
#pragma unroll
    for (int j = 0; j < 16; ++j) r.v[j] = T2[(8 * (j >> 2) + 4 * h + (j & 3)) * 32 + col];
}
template <int TW>
__device__ __forceinline__ void mx_rot_start(MxRot& cur, MxRot& step, const float2* T2, const float2* T1, int w, int col, int h)
{
    const float2 c0 = T1[w * 32 + col], c1 = T1[MX_W * 32 + col];       // (I2 only)
#pragma unroll
    for (int j = 0; j < 16; ++j) {
        const int p = 8 * (j >> 2) + 4 * h + (j & 3);
        if (TW == MX_TW_F1) {
            cur.v[j] = mx_cmul(T1[p * 32 + col], T2[p * 32 + w]);
            step.v[j] = T2[p * 32 + MX_W];
        } else {
            cur.v[j] = mx_cmul(T2[p * 32 + w], c0);
            step.v[j] = mx_cmul(T2[p * 32 + MX_W], c1);
        }
    }
}

template <int AX, bool ROT, int RB>
__device__ __forceinline__ void mx_store(unsigned* cube, const f32x16 (&acc)[2], const MxRot& rot, int t, int col, int h)
{
#pragma unroll
    for (int s = 0; s < 2 * RB; ++s) {
        u32x4 v;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            float re = mx_re(acc, s, i), im = mx_im(acc, s, i);
            if (ROT) {
                const float2 w = rot.v[4 * s + i];
                const float x = re * w.x - im * w.y, y = re * w.y + im * w.x;
                re = x;
                im = y;
            }
            v[i] = mx_pack(re, im);
        }
        if (AX == MX_AX3) {
            *reinterpret_cast<u32x4*>(cube + mx_addr(t, col, 8 * s + 4 * h)) = v;
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) cube[mx_word<AX>(t, col, 8 * s + 4 * h + i)] = v[i];
        }
    }
}

// One pass over the cube in place: wave w takes tiles w, w + MX_W, ... (32 columns each).  KS: steps of the contraction
// (2 when only the first 16 inputs along the axis can be non-zero), RB: row blocks wanted (1: results 0..15 only).
// TW: MX_TW_NONE, MX_TW_T2 (the same rotations for every tile) or MX_TW_F1 / MX_TW_I2 (stepped from tile to tile).
template <int AX, int TW, int KS, int RB>
__device__ __forceinline__ void mx_pass(unsigned* cube, const f16x8 (&A)[2][4], const float2* T2, const float2* T1, int w,
                                        int lane)
{
    const int col = lane & 31, h = lane >> 5;
    constexpr bool RUN = TW == MX_TW_F1 || TW == MX_TW_I2;
    MxRot cur, step;
    if (RUN) mx_rot_start<TW>(cur, step, T2, T1, w, col, h);
    if (TW == MX_TW_T2) mx_rot_fixed(cur, T2, col, h);
#pragma unroll 1
    for (int t = w; t < 32; t += MX_W) {
        f16x8 Bv[4];
        f32x16 acc[2];
        mx_load<AX, KS>(cube, t, col, h, Bv);
        mx_mul<KS, RB>(A, Bv, acc);
        mx_store<AX, TW != MX_TW_NONE, RB>(cube, acc, cur, t, col, h);
        if (RUN) {
#pragma unroll
            for (int j = 0; j < 16; ++j) cur.v[j] = mx_cmul(cur.v[j], step.v[j]);
        }
    }
}

// Spectrum of one channel's long kernel for these passes: bin k = k1 + 32 k2 + 1024 k3 of the 32768-point transform,
// divided by 4 |k|_1, as half-precision (re, im) pairs, stored where the lane that holds it after the forward passes
// will look:
// index ((k1 * 4 + s) * 64 + lane) * 4 + i with lane = k2 + 32 h and k3 = 8 s + 4 h + i.  Taken from the array of
// (K[k], K[16384 - k]) pairs, k = 0 .. 8192, that the spectrum kernel of the other convolution kernels leaves (the
// spectrum of a real sequence: the upper half is the conjugate of the lower).  scale[c] = 4 |k|_1.
__global__ __launch_bounds__(1024) void convmx_spectrum_kernel(const float* __restrict__ k_long,
                                                               const float4* __restrict__ pairs, unsigned* __restrict__ Ks,
                                                               float* __restrict__ scale, int L)
{
    __shared__ float red[16];
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const long c = blockIdx.x;
    float sum = 0.f;
    for (int t = tid; t < L; t += 1024) sum += fabsf(k_long[c * L + t]);
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
    if (lane == 0) red[w] = sum;
    __syncthreads();
    float n1 = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) n1 += red[i];
    const float inv = n1 > 0.f ? 0.25f / n1 : 0.f;
    if (tid == 0) scale[c] = n1 > 0.f ? 4.f * n1 : 0.f;
    const float4* pc = pairs + c * (long)(8192 + 1);
    unsigned* out = Ks + c * (long)MX_N;
    for (int o = tid; o < MX_N; o += 1024) {
        const int t = o >> 10, s = (o >> 8) & 3, ln = (o >> 2) & 63, i = o & 3;
        const int k = t + 32 * (ln & 31) + 1024 * (8 * s + 4 * (ln >> 5) + i);
        const bool upper = k > 16384;
        const int kk = upper ? MX_N - k : k;                 // 0 .. 16384
        const bool second = kk > 8192;
        const int kp = second ? 16384 - kk : kk;             // 0 .. 8192: the pair that holds bin kk
        const int l = kp == 8192 ? 8192 : (((kp & 127) << 6) | (kp >> 7));
        const float4 v = pc[l];
        float re = second ? v.z : v.x, im = second ? v.w : v.y;
        if (upper) im = -im;
        out[o] = mx_pack(re * inv, im * inv);
    }
}

// 32 consecutive steps [t0, t0 + 32) of one sequence (t0 = 32 tid: one row of the cube) through the short kernel and
// the activation, from registers only: the steps themselves and the HALO steps in front of them (the taps' history;
// zero in front of the sequence) come in as 16-byte pieces.  L is a multiple of 8 (so are the rows' starts), pieces
// beyond L read as zero, steps beyond L give zero.  HALO = 0: no short kernel, v = x.
template <int HALO>
__device__ __forceinline__ void mx_steps(const bf16* __restrict__ row, bool present, int t0, int L,
                                         const float* __restrict__ wc, int m, float (&v)[32])
{
    float x[HALO + 32];
#pragma unroll
    for (int k = 0; k < (HALO + 32) / 8; ++k) {
        const int pos = t0 - HALO + 8 * k;
        u32x4 r = {0u, 0u, 0u, 0u};
        if (present && pos >= 0 && pos < L) r = *reinterpret_cast<const u32x4*>(row + pos);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            x[8 * k + 2 * e] = __builtin_bit_cast(float, r[e] << 16);
            x[8 * k + 2 * e + 1] = __builtin_bit_cast(float, r[e] & 0xffff0000u);
        }
    }
    if (HALO == 0) {
#pragma unroll
        for (int o = 0; o < 32; ++o) v[o] = x[o];
        return;
    }
#pragma unroll
    for (int o = 0; o < 32; ++o) v[o] = 0.f;
#pragma unroll
    for (int j = 0; j <= HALO && j < 32; ++j) {
        const float wj = j < m ? wc[j] : 0.f;
#pragma unroll
        for (int o = 0; o < 32; ++o) v[o] = fmaf(wj, x[HALO + o - j], v[o]);
    }
#pragma unroll
    for (int o = 0; o < 32; ++o) v[o] = (t0 + o < L) ? v[o] * __builtin_amdgcn_rcpf(1.f + __expf(-v[o])) : 0.f;
}

// Pairs of sequences (2 pb, 2 pb + 1) of channel c, pair id = c * ceil(B / 2) + pb; a workgroup walks the ids
// blockIdx.x, blockIdx.x + gridDim.x, ...  HALO: steps of history the short kernel needs (m - 1 <= HALO; v =
// silu(K_s x)); 0: no short kernel, v = x.  L is a multiple of 8.
template <int HALO>
__global__ __launch_bounds__(MX_T) void convmx_fwd_kernel(const bf16* __restrict__ X, const float* __restrict__ w_short,
                                                          int m, const unsigned* __restrict__ Ks,
                                                          const float* __restrict__ kscale, bf16* __restrict__ Y, int B,
                                                          int d, int L, long n_pairs)
{
    __shared__ __attribute__((aligned(16))) unsigned cube[MX_CUBE];
    __shared__ float2 T2[1024];
    __shared__ float2 T1[1024];
    __shared__ float red[MX_W];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int e = tid; e < 1024; e += MX_T) {
        const int a = e >> 5, b = e & 31;
        float sn, cs;
        sincospif(-2.0f * (float)(a * b) / 1024.0f, &sn, &cs);
        T2[e] = make_float2(cs, sn);
        sincospif(-2.0f * (float)(a * b) / 32768.0f, &sn, &cs);
        T1[e] = make_float2(cs, sn);
    }
    f16x8 A[2][4];
    mx_build_matrix(A, lane);
    __syncthreads();
    const int PB = (B + 1) / 2;
    const int col = lane & 31, h = lane >> 5;
    const int my_d1 = tid >> 5, my_d2 = tid & 31;      // the cube row that holds this thread's 32 steps

    for (long pid = blockIdx.x; pid < n_pairs; pid += gridDim.x) {
        const int c = (int)(pid / PB), pb = (int)(pid - (long)c * PB);
        const bool two = 2 * pb + 1 < B;
        const long row_a = ((long)(2 * pb) * d + c) * (long)L, row_b = row_a + (long)d * L;
        // ---- the two sequences, short kernel and activation, in registers
        float va[32], vb[32];
        const float* wc = HALO ? w_short + (long)c * m : nullptr;
        mx_steps<HALO>(X + row_a, true, 32 * tid, L, wc, m, va);
        mx_steps<HALO>(X + row_b, two, 32 * tid, L, wc, m, vb);
        // ---- 1 / max |v| over the pair
        float mx = 0.f;
#pragma unroll
        for (int i = 0; i < 32; ++i) mx = fmaxf(mx, fmaxf(fabsf(va[i]), fabsf(vb[i])));
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o));
        if (lane == 0) red[w] = mx;
        __syncthreads();        // (also: the previous pair has been read out of the cube)
        float bm = 0.f;
#pragma unroll
        for (int i = 0; i < MX_W; ++i) bm = fmaxf(bm, red[i]);
        const float s1 = bm > 0.f ? 1.0f / bm : 1.0f;
        if (my_d1 < 16) {
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                u32x4 v;
#pragma unroll
                for (int e = 0; e < 4; ++e) v[e] = mx_pack(va[4 * g + e] * s1, vb[4 * g + e] * s1);
                *reinterpret_cast<u32x4*>(cube + mx_addr(my_d1, my_d2, 4 * g)) = v;
            }
        }
        // the spectrum pieces of this wave's first tile of the third pass, on their way while the first two passes run
        const u32x4* kc = reinterpret_cast<const u32x4*>(Ks + (long)c * MX_N);
        u32x4 kq[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) kq[q] = kc[(w * 4 + q) * 64 + lane];
        __syncthreads();
        // ---- forward: axis 1 (only planes 0..15 hold data), axis 2
        mx_pass<MX_AX1, MX_TW_F1, 2, 2>(cube, A, T2, T1, w, lane);
        __syncthreads();
        mx_pass<MX_AX2, MX_TW_T2, 4, 2>(cube, A, T2, T1, w, lane);
        __syncthreads();
        // ---- axis 3 forward, times the kernel's spectrum, conjugate, axis 3 on the way back: in registers
        MxRot fixed;
        mx_rot_fixed(fixed, T2, col, h);
#pragma unroll 1
        for (int t = w; t < 32; t += MX_W) {
            f16x8 Bv[4];
            f32x16 acc[2];
            mx_load<MX_AX3, 4>(cube, t, col, h, Bv);
            mx_mul<4, 2>(A, Bv, acc);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                u32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float zr = mx_re(acc, s, i), zi = mx_im(acc, s, i);
                    float kr, ki;
                    mx_unpack(kq[s][i], kr, ki);
                    v[i] = mx_pack(zr * kr - zi * ki, -(zr * ki + zi * kr));
                }
                Bv[s] = __builtin_bit_cast(f16x8, v);
            }
            if (t + MX_W < 32) {
#pragma unroll
                for (int q = 0; q < 4; ++q) kq[q] = kc[((t + MX_W) * 4 + q) * 64 + lane];
            }
            mx_mul<4, 2>(A, Bv, acc);
            mx_store<MX_AX3, true, 2>(cube, acc, fixed, t, col, h);
        }
        __syncthreads();
        mx_pass<MX_AX2, MX_TW_I2, 4, 2>(cube, A, T2, T1, w, lane);
        __syncthreads();
        mx_pass<MX_AX1, MX_TW_NONE, 4, 1>(cube, A, T2, T1, w, lane);     // only steps n < 16384 are wanted
        __syncthreads();
        // ---- out: y_a = Re, y_b = -Im (the conjugate that closes the way back), scales put back
        const float osc = kscale[c] / (s1 * (float)MX_N);
        if (32 * tid < L) {
            typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                if (32 * tid + 8 * g < L) {
                    const u32x4 v0 = *reinterpret_cast<const u32x4*>(cube + mx_addr(my_d1, my_d2, 8 * g));
                    const u32x4 v1 = *reinterpret_cast<const u32x4*>(cube + mx_addr(my_d1, my_d2, 8 * g + 4));
                    bf16x8 oa, ob;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        float re, im;
                        mx_unpack(e < 4 ? v0[e & 3] : v1[e & 3], re, im);
                        oa[e] = (bf16)(re * osc);
                        ob[e] = (bf16)(-im * osc);
                    }
                    *reinterpret_cast<bf16x8*>(Y + row_a + 32 * tid + 8 * g) = oa;
                    if (two) *reinterpret_cast<bf16x8*>(Y + row_b + 32 * tid + 8 * g) = ob;
                }
            }
        }
    }
}

// One row (32 steps) of each sequence of a pair out of the cube after the way back: a = Re, b = -Im, times `osc`.
template <typename OUT>
__device__ __forceinline__ void mx_rows_out(const unsigned* cube, OUT* __restrict__ ya, OUT* __restrict__ yb, bool two,
                                            int tid, int L, float osc)
{
    const int d1 = tid >> 5, d2 = tid & 31;
    if (32 * tid >= L) return;
#pragma unroll
    for (int g = 0; g < 4; ++g) {
        if (32 * tid + 8 * g < L) {
            const u32x4 v0 = *reinterpret_cast<const u32x4*>(cube + mx_addr(d1, d2, 8 * g));
            const u32x4 v1 = *reinterpret_cast<const u32x4*>(cube + mx_addr(d1, d2, 8 * g + 4));
            float fa[8], fb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                float re, im;
                mx_unpack(e < 4 ? v0[e & 3] : v1[e & 3], re, im);
                fa[e] = re * osc;
                fb[e] = -im * osc;
            }
            if (sizeof(OUT) == 2) {
                typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
                bf16x8 oa, ob;
#pragma unroll
                for (int e = 0; e < 8; ++e) { oa[e] = (bf16)fa[e]; ob[e] = (bf16)fb[e]; }
                *reinterpret_cast<bf16x8*>(ya + 32 * tid + 8 * g) = oa;
                if (two) *reinterpret_cast<bf16x8*>(yb + 32 * tid + 8 * g) = ob;
            } else {
                float4* pa = reinterpret_cast<float4*>(ya + 32 * tid + 8 * g);
                pa[0] = make_float4(fa[0], fa[1], fa[2], fa[3]);
                pa[1] = make_float4(fa[4], fa[5], fa[6], fa[7]);
                if (two) {
                    float4* pq = reinterpret_cast<float4*>(yb + 32 * tid + 8 * g);
                    pq[0] = make_float4(fb[0], fb[1], fb[2], fb[3]);
                    pq[1] = make_float4(fb[4], fb[5], fb[6], fb[7]);
                }
            }
        }
    }
}

// From each thread's own largest magnitude and sum of squares: 1 / (largest magnitude in the workgroup) (1 if that is
// zero) and the workgroup's sum of squares; two barriers.
__device__ __forceinline__ float mx_inv_max(float mx, float& ss, float* red, int lane, int w)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) {
        mx = fmaxf(mx, __shfl_xor(mx, o));
        ss += __shfl_xor(ss, o);
    }
    __syncthreads();            // (the previous use of red[] is over)
    if (lane == 0) { red[w] = mx; red[MX_W + w] = ss; }
    __syncthreads();
    float bm = 0.f;
    ss = 0.f;
#pragma unroll
    for (int i = 0; i < MX_W; ++i) { bm = fmaxf(bm, red[i]); ss += red[MX_W + i]; }
    return bm > 0.f ? 1.0f / bm : 1.0f;
}

__device__ __forceinline__ void mx_rows_in(unsigned* cube, const float (&va)[32], const float (&vb)[32], float s, int tid)
{
#pragma unroll
    for (int g = 0; g < 8; ++g) {
        u32x4 v;
#pragma unroll
        for (int e = 0; e < 4; ++e) v[e] = mx_pack(va[4 * g + e] * s, vb[4 * g + e] * s);
        *reinterpret_cast<u32x4*>(cube + mx_addr(tid >> 5, tid & 31, 4 * g)) = v;
    }
}

// The two long-stage gradients of the convolution (they share the spectrum of dZ), pairs of sequences as above; one
// workgroup walks the pairs of a channel, then the next channel blockIdx.x + gridDim.x, ...
//   dv = corr(dZ, k_long):   Wd = T(dZ_a + i dZ_b);  conj(T'(conj(Wd conj(K)))) / N:  Re -> dv_a, Im -> dv_b
//   dk[c][s] = sum_b sum_t dZ_b[t] v_b[t - s]:  Wv = T(v_a + i v_b), v = silu(K_s x) recomputed;  for the two real
//   sequences of a pair DZ_a conj(V_a) + DZ_b conj(V_b) = (H[k] + conj H[-k]) / 2 with H = Wd conj(Wv), whose transform
//   back is the real part of that of H: the pair's share of dk is Re T'(conj H) / N, added up over the pairs in the time
//   domain (64 KB per channel, each step by the thread that owns it), so no spectrum-sized sums ever go to memory.
//   Range of H: sum_k |Wd||Wv| <= |Wd|_2 |Wv|_2 = N |z_d|_2 |z_v|_2, so H times 32768 / (N |z_d|_2 |z_v|_2) keeps every
//   sum on the way back within 32768 and leaves a typical bin at order one.
//   Wd waits in memory while v is transformed (this workgroup's own 128 KB, in the order its lanes hold it).
// dV: fp32 [B][d][L] for the short-stage kernel, or dX itself (bf16) when there is no short stage (HALO = 0, v = x).
template <int HALO, typename DVT>
__global__ __launch_bounds__(MX_T) void convmx_longbwd_kernel(const bf16* __restrict__ X, const float* __restrict__ w_short,
                                                              int m, const unsigned* __restrict__ Ks,
                                                              const float* __restrict__ kscale,
                                                              const bf16* __restrict__ dZ, DVT* __restrict__ dV,
                                                              float* __restrict__ dk, u32x4* __restrict__ Wds,
                                                              int B, int d, int L)
{
    __shared__ __attribute__((aligned(16))) unsigned cube[MX_CUBE];
    __shared__ float2 T2[1024];
    __shared__ float2 T1[1024];
    __shared__ float red[2 * MX_W];
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    for (int e = tid; e < 1024; e += MX_T) {
        const int a = e >> 5, b = e & 31;
        float sn, cs;
        sincospif(-2.0f * (float)(a * b) / 1024.0f, &sn, &cs);
        T2[e] = make_float2(cs, sn);
        sincospif(-2.0f * (float)(a * b) / 32768.0f, &sn, &cs);
        T1[e] = make_float2(cs, sn);
    }
    f16x8 A[2][4];
    mx_build_matrix(A, lane);
    __syncthreads();
    const int PB = (B + 1) / 2;
    const int col = lane & 31, h = lane >> 5;
    constexpr int NT = 32 / MX_W;        // tiles of a pass per wave
    u32x4* wdm = Wds + (size_t)blockIdx.x * (MX_N / 4);

    for (int c = blockIdx.x; c < d; c += gridDim.x) {
        const u32x4* kc = reinterpret_cast<const u32x4*>(Ks + (long)c * MX_N);
        const float* wc = HALO ? w_short + (long)c * m : nullptr;
        const float ksc = kscale[c];
        for (int pb = 0; pb < PB; ++pb) {
            const bool two = 2 * pb + 1 < B;
            const long row_a = ((long)(2 * pb) * d + c) * (long)L, row_b = row_a + (long)d * L;
            float s_d, n_d = 0.f;
            {
                float va[32], vb[32];
                mx_steps<0>(dZ + row_a, true, 32 * tid, L, nullptr, 0, va);
                mx_steps<0>(dZ + row_b, two, 32 * tid, L, nullptr, 0, vb);
                float mx = 0.f;
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    mx = fmaxf(mx, fmaxf(fabsf(va[i]), fabsf(vb[i])));
                    n_d = fmaf(va[i], va[i], fmaf(vb[i], vb[i], n_d));
                }
                s_d = mx_inv_max(mx, n_d, red, lane, w);      // (its barriers: the cube is free again)
                mx_rows_in(cube, va, vb, s_d, tid);
            }
            __syncthreads();
            mx_pass<MX_AX1, MX_TW_F1, 2, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            mx_pass<MX_AX2, MX_TW_T2, 4, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            {
                MxRot fixed;
                mx_rot_fixed(fixed, T2, col, h);
                u32x4 kq[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) kq[q] = kc[(w * 4 + q) * 64 + lane];
#pragma unroll 1
                for (int n = 0; n < NT; ++n) {
                    const int t = w + MX_W * n;
                    f16x8 Bv[4];
                    f32x16 acc[2];
                    mx_load<MX_AX3, 4>(cube, t, col, h, Bv);
                    mx_mul<4, 2>(A, Bv, acc);
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        u32x4 v, keep;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float zr = mx_re(acc, s, i), zi = mx_im(acc, s, i);
                            keep[i] = mx_pack(zr, zi);
                            float kr, ki;
                            mx_unpack(kq[s][i], kr, ki);
                            // conj(Z conj(K)) = (zr kr + zi ki) + i (zr ki - zi kr)
                            v[i] = mx_pack(zr * kr + zi * ki, zr * ki - zi * kr);
                        }
                        Bv[s] = __builtin_bit_cast(f16x8, v);
                        wdm[(t * 4 + s) * 64 + lane] = keep;
                    }
                    if (n + 1 < NT) {       // the next tile's pieces of the spectrum, on their way during the products
#pragma unroll
                        for (int q = 0; q < 4; ++q) kq[q] = kc[((t + MX_W) * 4 + q) * 64 + lane];
                    }
                    mx_mul<4, 2>(A, Bv, acc);
                    mx_store<MX_AX3, true, 2>(cube, acc, fixed, t, col, h);
                }
            }
            __syncthreads();
            mx_pass<MX_AX2, MX_TW_I2, 4, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            mx_pass<MX_AX1, MX_TW_NONE, 4, 1>(cube, A, T2, T1, w, lane);
            __syncthreads();
            mx_rows_out<DVT>(cube, dV + row_a, dV + row_b, two, tid, L, ksc / (s_d * (float)MX_N));

            // ---- v = silu(K_s x) (or x), its spectrum, H (+)= Wd conj(Wv) with the two scales taken out
            float s_v, n_v = 0.f;
            {
                float va[32], vb[32];
                mx_steps<HALO>(X + row_a, true, 32 * tid, L, wc, m, va);
                mx_steps<HALO>(X + row_b, two, 32 * tid, L, wc, m, vb);
                float mx = 0.f;
#pragma unroll
                for (int i = 0; i < 32; ++i) {
                    mx = fmaxf(mx, fmaxf(fabsf(va[i]), fabsf(vb[i])));
                    n_v = fmaf(va[i], va[i], fmaf(vb[i], vb[i], n_v));
                }
                s_v = mx_inv_max(mx, n_v, red, lane, w);      // (its barriers: dv has been read out of the cube)
                mx_rows_in(cube, va, vb, s_v, tid);
            }
            __syncthreads();
            mx_pass<MX_AX1, MX_TW_F1, 2, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            mx_pass<MX_AX2, MX_TW_T2, 4, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            // |z|_2 of the scaled signals: sqrt(sum of squares) * scale
            const float nn = sqrtf(n_d) * s_d * sqrtf(n_v) * s_v;
            const float g = nn > 0.f ? 1.0f / nn : 0.f;          // = 32768 / (N |z_d|_2 |z_v|_2)
            {
                MxRot fixed;
                mx_rot_fixed(fixed, T2, col, h);
                u32x4 wn[4];                                     // Wd of the tile in hand, fetched one tile ahead
#pragma unroll
                for (int s = 0; s < 4; ++s) wn[s] = wdm[(w * 4 + s) * 64 + lane];
#pragma unroll 1
                for (int n = 0; n < NT; ++n) {
                    const int t = w + MX_W * n;
                    f16x8 Bv[4];
                    f32x16 acc[2];
                    mx_load<MX_AX3, 4>(cube, t, col, h, Bv);
                    mx_mul<4, 2>(A, Bv, acc);
#pragma unroll
                    for (int s = 0; s < 4; ++s) {
                        u32x4 v;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            float dr, di;
                            mx_unpack(wn[s][i], dr, di);
                            const float vr = mx_re(acc, s, i), vi = mx_im(acc, s, i);
                            // conj(Wd conj(Wv)) = (dr vr + di vi) + i (dr vi - di vr)
                            v[i] = mx_pack((dr * vr + di * vi) * g, (dr * vi - di * vr) * g);
                        }
                        Bv[s] = __builtin_bit_cast(f16x8, v);
                    }
                    if (n + 1 < NT) {
#pragma unroll
                        for (int s = 0; s < 4; ++s) wn[s] = wdm[((t + MX_W) * 4 + s) * 64 + lane];
                    }
                    mx_mul<4, 2>(A, Bv, acc);
                    mx_store<MX_AX3, true, 2>(cube, acc, fixed, t, col, h);
                }
            }
            __syncthreads();
            mx_pass<MX_AX2, MX_TW_I2, 4, 2>(cube, A, T2, T1, w, lane);
            __syncthreads();
            mx_pass<MX_AX1, MX_TW_NONE, 4, 1>(cube, A, T2, T1, w, lane);
            __syncthreads();
            // this pair's share of dk: Re / (N g s_d s_v), each step by the thread that owns it
            if (32 * tid < L) {
                const float osc = g > 0.f ? 1.0f / (g * s_d * s_v * (float)MX_N) : 0.f;
                float* out = dk + (long)c * L + 32 * tid;
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    if (32 * tid + 4 * q < L) {
                        const u32x4 v = *reinterpret_cast<const u32x4*>(cube + mx_addr(tid >> 5, tid & 31, 4 * q));
                        float r0, r1, r2, r3, im;
                        mx_unpack(v[0], r0, im);
                        mx_unpack(v[1], r1, im);
                        mx_unpack(v[2], r2, im);
                        mx_unpack(v[3], r3, im);
                        float4 o = make_float4(0.f, 0.f, 0.f, 0.f);
                        if (pb > 0) o = *reinterpret_cast<const float4*>(out + 4 * q);
                        o.x += r0 * osc; o.y += r1 * osc; o.z += r2 * osc; o.w += r3 * osc;
                        *reinterpret_cast<float4*>(out + 4 * q) = o;
                    }
                }
            }
            // (the next stage starts with barriers before it touches the cube)
        }
        __syncthreads();        // the cube is free for the next channel
    }
}

// ------------------------------------------------------------------------------------------------ host side
bool convmx_applies(int L, int dtype)
{
    // (rows of a multiple of 8 steps start on 16-byte boundaries: the kernel moves 16-byte pieces only)
    if (dtype != 0 || L <= 4096 || L > MX_L_MAX || (L & 7) != 0) return false;
    const char* e = getenv("CHELA_CONV_MATRIX");      // tuning aid: 0 keeps the vector-ALU kernels for every size
    return !(e && atoi(e) == 0);
}

size_t convmx_spectrum_bytes(int d, int L)
{
    if (d <= 0 || L <= 4096 || L > MX_L_MAX) return 0;
    return (size_t)d * MX_N * sizeof(unsigned) + (((size_t)d * sizeof(float) + 255) & ~(size_t)255);
}

hipError_t launch_convmx_spectrum(const float* k_long, const void* pairs, void* extra, int d, int L, hipStream_t st)
{
    unsigned* Ks = (unsigned*)extra;
    float* scale = (float*)((char*)extra + (size_t)d * MX_N * sizeof(unsigned));
    hipLaunchKernelGGL(convmx_spectrum_kernel, dim3(d), dim3(1024), 0, st, k_long, (const float4*)pairs, Ks, scale, L);
    return hipGetLastError();
}

hipError_t launch_convmx_fwd(const void* X, const float* w_short, int m, const void* extra, void* Y, int B, int d, int L,
                             hipStream_t st)
{
    const unsigned* Ks = (const unsigned*)extra;
    const float* scale = (const float*)((const char*)extra + (size_t)d * MX_N * sizeof(unsigned));
    const long n_pairs = (long)d * ((B + 1) / 2);
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    (void)hipGetLastError();
    const long slots = cus;                              // 132 KB of LDS + tables: one workgroup per compute unit
    const long rounds = (n_pairs + slots - 1) / slots;
    const dim3 grid((unsigned)((n_pairs + rounds - 1) / rounds));
    ProfScope prof(KID_CONV_FWD, st);
    if (!w_short)
        hipLaunchKernelGGL((convmx_fwd_kernel<0>), grid, dim3(MX_T), 0, st, (const bf16*)X, w_short, m, Ks, scale,
                           (bf16*)Y, B, d, L, n_pairs);
    else if (m <= 9)
        hipLaunchKernelGGL((convmx_fwd_kernel<8>), grid, dim3(MX_T), 0, st, (const bf16*)X, w_short, m, Ks, scale,
                           (bf16*)Y, B, d, L, n_pairs);
    else
        hipLaunchKernelGGL((convmx_fwd_kernel<32>), grid, dim3(MX_T), 0, st, (const bf16*)X, w_short, m, Ks, scale,
                           (bf16*)Y, B, d, L, n_pairs);
    return hipGetLastError();
}

hipError_t launch_convmx_longbwd(const void* X, const float* w_short, int m, const void* extra, const void* dZ, void* dV,
                                 bool dv_is_f32, float* dk, float* Hs, int B, int d, int L, hipStream_t st)
{
    const unsigned* Ks = (const unsigned*)extra;
    const float* scale = (const float*)((const char*)extra + (size_t)d * MX_N * sizeof(unsigned));
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    (void)hipGetLastError();
    if (cus > kConvMxMaxWgs) cus = kConvMxMaxWgs;       // (the scratch behind the sums holds that many workgroups' Wd)
    const int rounds = (d + cus - 1) / cus;
    const dim3 grid((unsigned)((d + rounds - 1) / rounds));
    ProfScope prof(KID_CONV_LONG_BWD, st);
#define CHELA_MX_BWD(H_, T_)                                                                                            \
    hipLaunchKernelGGL((convmx_longbwd_kernel<H_, T_>), grid, dim3(MX_T), 0, st, (const bf16*)X, w_short, m, Ks, scale,  \
                       (const bf16*)dZ, (T_*)dV, dk, (u32x4*)Hs, B, d, L)
    if (!w_short) {
        if (dv_is_f32) CHELA_MX_BWD(0, float); else CHELA_MX_BWD(0, bf16);
    } else if (m <= 9) {
        if (dv_is_f32) CHELA_MX_BWD(8, float); else CHELA_MX_BWD(8, bf16);
    } else {
        if (dv_is_f32) CHELA_MX_BWD(32, float); else CHELA_MX_BWD(32, bf16);
    }
#undef CHELA_MX_BWD
    return hipGetLastError();
}

}  // namespace chela
