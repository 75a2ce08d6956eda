// Short-long convolutions (Sec. 4.2, Eq. 8): Z = K_l( silu( K_s(X) ) ), depthwise and causal, tensors [B][d][L].
//
// The long kernel is as long as the sequence, so K_l goes through the Fourier domain (Eq. 7).  One workgroup
// owns one (batch, channel) sequence and never leaves the chip between load and store:
//   load x, short kernel + silu  ->  real sequence v, zero-padded to N = 2M >= 2L (so that the circular product of
//   Eq. 7 equals the causal sum), packed as M complex numbers z[n] = v[2n] + i v[2n+1]  ->  complex FFT of length M
//   in LDS  ->  untangle to the spectrum of v, multiply by the kernel's spectrum, tangle back  ->  inverse FFT
//   ->  y[2n], y[2n+1] = Re, Im.
// FFT: in place, decimation in frequency forward (natural order in, digit-reversed out) and the exact inverse of
// every pass in reverse order (digit-reversed in, natural out), so no reordering pass exists; the point-wise
// stage addresses the spectrum through the digit reversal.  M = 4^a 16^b: an optional leading radix-4 pass, then
// radix-16 passes with one 16-point transform per thread held in registers (two layers of radix 4).  The LDS
// array carries one complex of padding per 16, which makes the stride-1 and stride-16 passes conflict-free.
// Arithmetic is fp32 on the vector ALU: with one kernel per channel there is no operand shared across channels
// except the DFT matrix itself, and fp32 matrix instructions are no faster than the ALU on this chip.
#include "chela_internal.h"
#include <cstdlib>

namespace chela {

typedef __bf16 bf16;

struct cplx { float x, y; };
__device__ __forceinline__ cplx mk(float x, float y) { cplx c; c.x = x; c.y = y; return c; }
__device__ __forceinline__ cplx cadd(cplx a, cplx b) { return mk(a.x + b.x, a.y + b.y); }
__device__ __forceinline__ cplx csub(cplx a, cplx b) { return mk(a.x - b.x, a.y - b.y); }
__device__ __forceinline__ cplx cmul(cplx a, cplx b) { return mk(a.x * b.x - a.y * b.y, a.x * b.y + a.y * b.x); }
__device__ __forceinline__ cplx conj(cplx a) { return mk(a.x, -a.y); }
__device__ __forceinline__ cplx mul_neg_i(cplx a) { return mk(a.y, -a.x); }   // a * (-i)
__device__ __forceinline__ cplx mul_pos_i(cplx a) { return mk(-a.y, a.x); }   // a * (+i)

// 4-point DFT, kernel exp(-2 pi i p q / 4) (INV: the conjugate kernel), in place: (a,b,c,d) = x_0..x_3 -> X_0..X_3.
template <bool INV>
__device__ __forceinline__ void dft4(cplx& a, cplx& b, cplx& c, cplx& d)
{
    const cplx s0 = cadd(a, c), d0 = csub(a, c), s1 = cadd(b, d), d1 = csub(b, d);
    const cplx r = INV ? mul_pos_i(d1) : mul_neg_i(d1);
    a = cadd(s0, s1);
    c = csub(s0, s1);
    b = cadd(d0, r);
    d = csub(d0, r);
}

// 16-point DFT in registers.  In: v[q] = x_q.  Out: X_p sits in slot (p >> 2) + 4 * (p & 3).
// q = q0 + 4 q1, p = p1 + 4 p0:  X_p = sum_q0 w4^(p0 q0) w16^(p1 q0) [ sum_q1 x_(q0 + 4 q1) w4^(p1 q1) ].
template <bool INV>
__device__ __forceinline__ void dft16(cplx (&v)[16])
{
#pragma unroll
    for (int q0 = 0; q0 < 4; ++q0) dft4<INV>(v[q0], v[q0 + 4], v[q0 + 8], v[q0 + 12]);     // slot q0 + 4 p1
    constexpr float C1 = 0.92387953251128674f, S1 = 0.38268343236508977f, R2 = 0.70710678118654752f;
    // w16^k = exp(-2 pi i k / 16) for the products q0 * p1 in {1, 2, 3, 4, 6, 9}
    const cplx w1 = mk(C1, INV ? S1 : -S1), w2 = mk(R2, INV ? R2 : -R2), w3 = mk(S1, INV ? C1 : -C1);
    const cplx w6 = mk(-R2, INV ? R2 : -R2), w9 = mk(-C1, INV ? -S1 : S1);
    v[1 + 4 * 1] = cmul(v[1 + 4 * 1], w1);
    v[2 + 4 * 1] = cmul(v[2 + 4 * 1], w2);
    v[3 + 4 * 1] = cmul(v[3 + 4 * 1], w3);
    v[1 + 4 * 2] = cmul(v[1 + 4 * 2], w2);
    v[2 + 4 * 2] = INV ? mul_pos_i(v[2 + 4 * 2]) : mul_neg_i(v[2 + 4 * 2]);                 // w16^4 = -i
    v[3 + 4 * 2] = cmul(v[3 + 4 * 2], w6);
    v[1 + 4 * 3] = cmul(v[1 + 4 * 3], w3);
    v[2 + 4 * 3] = cmul(v[2 + 4 * 3], w6);
    v[3 + 4 * 3] = cmul(v[3 + 4 * 3], w9);
#pragma unroll
    for (int p1 = 0; p1 < 4; ++p1) dft4<INV>(v[4 * p1], v[4 * p1 + 1], v[4 * p1 + 2], v[4 * p1 + 3]);   // slot p0 + 4 p1
}

__host__ __device__ constexpr int conv_threads(int M) { return M / 16 < 64 ? 64 : M / 16; }
__host__ __device__ constexpr bool conv_lead4(int M) { return M == 1024 || M == 16384; }
__host__ __device__ constexpr int conv_pad(int i) { return i + (i >> 4); }

template <int M>
struct ConvLds {
    static constexpr int DATA = conv_pad(M);                 // complex slots
    static constexpr int BYTES = DATA * 8 + 2 * 128 * 8;     // + two twiddle tables of 128
};

// exp(-2 pi i e / M) for 0 <= e < M from two tables of 128: lo[x] = W^x, hi[y] = W^(128 y).
template <int M>
__device__ __forceinline__ cplx twiddle(const cplx* lo, const cplx* hi, int e)
{
    if (M <= 128) return lo[e];
    return cmul(lo[e & 127], hi[e >> 7]);
}

// Storage position of spectrum bin k (0 <= k < M) after the forward passes.
template <int M>
__device__ __forceinline__ int spectrum_pos(int k)
{
    int pos = 0, span = M;
    if (conv_lead4(M)) { span /= 4; pos += (k & 3) * span; k >>= 2; }
#pragma unroll
    for (int s = span; s > 1; s /= 16) { pos += (k & 15) * (s / 16); k >>= 4; }
    return pos;
}

// One radix-16 pass over sub-transforms of length N16 (stride N16 / 16), forward or inverse, 16-point transforms
// in registers, T threads.  With the length fixed at compile time the 16 LDS addresses are one base plus constants
// (the padding of a multiple of 16 is itself a constant), and the last pass (N16 = 16) has no twiddles at all.
template <int M, int T, int N16, bool INV>
__device__ __forceinline__ void pass16(cplx* a, const cplx* lo, const cplx* hi, int tid)
{
    constexpr int S = N16 / 16;
    constexpr int STEP = S >= 16 ? S + S / 16 : 1;                 // padded distance between the transform's points
    for (int g = tid; g < M / 16; g += T) {
        const int block = g / S, j = g - block * S;
        cplx* p0 = a + (S >= 16 ? conv_pad(block * N16 + j) : 17 * g);
        cplx v[16];
        cplx w1 = mk(1.f, 0.f);
        if (S > 1) {
            const cplx w1f = twiddle<M>(lo, hi, j * (M / N16));   // W_N16^j
            w1 = INV ? conj(w1f) : w1f;
        }
        if (INV) {
            // undo the forward pass: strip the twiddles, then the conjugate 16-point transform (the factor 1/16 is
            // left to the final scaling); inputs X_p in natural order p, outputs x_q in slot order
            cplx w = w1;
            v[0] = p0[0];
#pragma unroll
            for (int p = 1; p < 16; ++p) {
                v[p] = S > 1 ? cmul(p0[p * STEP], w) : p0[p * STEP];
                if (S > 1) w = cmul(w, w1);
            }
            dft16<true>(v);
#pragma unroll
            for (int q = 0; q < 16; ++q) p0[q * STEP] = v[(q >> 2) + 4 * (q & 3)];
        } else {
#pragma unroll
            for (int q = 0; q < 16; ++q) v[q] = p0[q * STEP];
            dft16<false>(v);
            cplx w = w1;
            p0[0] = v[0];
#pragma unroll
            for (int p = 1; p < 16; ++p) {
                p0[p * STEP] = S > 1 ? cmul(v[(p >> 2) + 4 * (p & 3)], w) : v[(p >> 2) + 4 * (p & 3)];
                if (S > 1) w = cmul(w, w1);
            }
        }
    }
}

// All forward passes (INV = false) or all inverse passes in reverse order (INV = true) over a[] in LDS.
// A __syncthreads() separates the passes; the caller synchronises before and after.
template <int M, int T, bool INV>
__device__ __forceinline__ void fft_passes(cplx* a, const cplx* lo, const cplx* hi, int tid)
{
    constexpr int M16 = conv_lead4(M) ? M / 4 : M;     // what the radix-16 passes transform (blocks of this length)
    static_assert(M16 == 256 || M16 == 4096, "radix-16 part must be 16^2 or 16^3");
    // The packed sequence has at most M/2 non-zero entries (L <= M real steps) and only its first M/2 entries are
    // ever read back: the leading radix-4 pass sees two zero inputs going forward and owes only two outputs coming back.
    auto lead4 = [&]() __attribute__((always_inline)) {
        constexpr int s = M / 4, sp = s + s / 16;
        for (int g = tid; g < s; g += T) {
            cplx* p0 = a + conv_pad(g);
            const cplx w1 = twiddle<M>(lo, hi, g);
            const cplx t1 = INV ? conj(w1) : w1, t2 = cmul(t1, t1), t3 = cmul(t2, t1);
            if (!INV) {
                const cplx v0 = p0[0], v1 = p0[sp], r = mul_neg_i(v1);
                p0[0] = cadd(v0, v1);
                p0[sp] = cmul(cadd(v0, r), t1);
                p0[2 * sp] = cmul(csub(v0, v1), t2);
                p0[3 * sp] = cmul(csub(v0, r), t3);
            } else {
                const cplx v0 = p0[0], v1 = cmul(p0[sp], t1), v2 = cmul(p0[2 * sp], t2), v3 = cmul(p0[3 * sp], t3);
                const cplx s02 = cadd(v0, v2), d02 = csub(v0, v2), s13 = cadd(v1, v3), d13 = csub(v1, v3);
                p0[0] = cadd(s02, s13);
                p0[sp] = cadd(d02, mul_pos_i(d13));
            }
        }
    };
    if (!INV) {
        if (conv_lead4(M)) { lead4(); __syncthreads(); }
        if (M16 == 4096) { pass16<M, T, 4096, false>(a, lo, hi, tid); __syncthreads(); }
        pass16<M, T, 256, false>(a, lo, hi, tid);
        __syncthreads();
        pass16<M, T, 16, false>(a, lo, hi, tid);
    } else {
        pass16<M, T, 16, true>(a, lo, hi, tid);
        __syncthreads();
        pass16<M, T, 256, true>(a, lo, hi, tid);
        if (M16 == 4096) { __syncthreads(); pass16<M, T, 4096, true>(a, lo, hi, tid); }
        if (conv_lead4(M)) { __syncthreads(); lead4(); }
    }
}

// raw_t: the pair (x[t], x[t+1]) as it sits in memory, so that a sequence fetched ahead costs as few registers as it
// costs bytes; raw_pair() reads an aligned pair, raw_scalars() builds one from single reads (odd row lengths, the
// second element optional), unpack() converts.
template <typename T> struct IoPair;
template <> struct IoPair<float> {
    typedef float2 raw_t;
    static __device__ __forceinline__ raw_t raw_zero() { return make_float2(0.f, 0.f); }
    static __device__ __forceinline__ raw_t raw_pair(const float* p) { return *reinterpret_cast<const float2*>(p); }
    static __device__ __forceinline__ raw_t raw_scalars(const float* p, bool second) { return make_float2(p[0], second ? p[1] : 0.f); }
    static __device__ __forceinline__ void unpack(raw_t r, float& a, float& b) { a = r.x; b = r.y; }
    static __device__ __forceinline__ void load2(const float* p, float& a, float& b) { const float2 v = *reinterpret_cast<const float2*>(p); a = v.x; b = v.y; }
    static __device__ __forceinline__ void store2(float* p, float a, float b) { *reinterpret_cast<float2*>(p) = make_float2(a, b); }
};
template <> struct IoPair<bf16> {
    typedef unsigned raw_t;
    static __device__ __forceinline__ raw_t raw_zero() { return 0u; }
    static __device__ __forceinline__ raw_t raw_pair(const bf16* p) { return *reinterpret_cast<const unsigned*>(p); }
    static __device__ __forceinline__ raw_t raw_scalars(const bf16* p, bool second)
    {
        const unsigned short* q = reinterpret_cast<const unsigned short*>(p);
        return (unsigned)q[0] | (second ? (unsigned)q[1] << 16 : 0u);
    }
    static __device__ __forceinline__ void unpack(raw_t u, float& a, float& b)
    {
        a = __builtin_bit_cast(float, u << 16);
        b = __builtin_bit_cast(float, u & 0xffff0000u);
    }
    static __device__ __forceinline__ void load2(const bf16* p, float& a, float& b)
    {
        const unsigned u = *reinterpret_cast<const unsigned*>(p);
        a = __builtin_bit_cast(float, u << 16);
        b = __builtin_bit_cast(float, u & 0xffff0000u);
    }
    static __device__ __forceinline__ void store2(bf16* p, float a, float b)
    {
        typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
        bf16x2 v;
        v[0] = (bf16)a;
        v[1] = (bf16)b;
        *reinterpret_cast<bf16x2*>(p) = v;
    }
};

// Eight consecutive elements at a 16-byte aligned position.
__device__ __forceinline__ void load8(const float* p, float (&v)[8])
{
    const float4 a = *reinterpret_cast<const float4*>(p), b = *reinterpret_cast<const float4*>(p + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
}
__device__ __forceinline__ void load8(const bf16* p, float (&v)[8])
{
    const uint4 u = *reinterpret_cast<const uint4*>(p);
    const unsigned w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        v[2 * e] = __builtin_bit_cast(float, w[e] << 16);
        v[2 * e + 1] = __builtin_bit_cast(float, w[e] & 0xffff0000u);
    }
}
__device__ __forceinline__ void store8(float* p, const float (&v)[8])
{
    *reinterpret_cast<float4*>(p) = make_float4(v[0], v[1], v[2], v[3]);
    *reinterpret_cast<float4*>(p + 4) = make_float4(v[4], v[5], v[6], v[7]);
}
__device__ __forceinline__ void store8(bf16* p, const float (&v)[8])
{
    typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
    bf16x8 o;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = (bf16)v[e];
    *reinterpret_cast<bf16x8*>(p) = o;
}

template <int M, int T>
__device__ __forceinline__ void build_tables(cplx* lo, cplx* hi, int tid)
{
    for (int t = tid; t < 128; t += T) {
        float s, c;
        sincospif(-2.0f * (float)t / (float)M, &s, &c);
        lo[t] = mk(c, s);
        sincospif(-2.0f * (float)(t * 128 % M) / (float)M, &s, &c);
        hi[t] = mk(c, s);
    }
}

// Order in which the point-wise stages walk the bin pairs (k, M - k), 0 <= k <= M/2.  The forward passes leave
// bin k at a digit-reversed position, so lanes that took consecutive k would all hit the same LDS banks (strides of
// M/4 and M/64 complex).  Pair l takes k = ((l & 63) << HB) | (l >> 6) instead: the 64 lanes of a wave then differ
// in the HIGH bits of k, i.e. in the low digits of the storage position.  l = M/2 stands for the self-paired bin
// M/2.  The kernel spectrum is stored in the same order, one float4 (K[k], K[M-k]) per pair, so its loads coalesce.
template <int M>
__device__ __forceinline__ int pair_bin(int l)
{
    constexpr int HALF = M / 2;
    int hb = 0;
#pragma unroll
    for (int x = HALF / 64; x > 1; x >>= 1) ++hb;
    return l >= HALF ? HALF : (((l & 63) << hb) | (l >> 6));
}

__device__ __forceinline__ cplx w2m(int k, int M)      // W_2M^k = exp(-i pi k / M)
{
    float s, c;
    sincospif(-(float)k / (float)M, &s, &c);
    return mk(c, s);
}

// W_2M^k for the bins a thread meets when it walks the pairs l = tid, tid + T, ... in pair order: k = (lane << HB) |
// (l >> 6), so W^k = W^(lane << HB) * W^(tid >> 6) * (W^(T/64))^i: two sincospi per thread and one rotation per pair
// instead of one sincospi per pair.  The self-paired bin M/2 (l = M/2) is -i.
template <int M, int T>
struct PairTwiddle {
    cplx cur, step;
    __device__ __forceinline__ PairTwiddle(int tid)
    {
        cur = w2m(pair_bin<M>(tid < M / 2 ? tid : 0), M);
        step = w2m(T / 64, M);
    }
    __device__ __forceinline__ cplx next(int l)
    {
        const cplx w = l >= M / 2 ? mk(0.f, -1.f) : cur;
        cur = cmul(cur, step);
        return w;
    }
};

// Bins k and M - k of the spectrum of a real sequence of length 2M from the length-M transform Z of its even/odd
// packing:  X[k] = (Z[k] + conj Z[M-k]) / 2 + W_2M^k (Z[k] - conj Z[M-k]) / (2i),  k = 0 .. M  (Z[M] = Z[0]).
// A = Z[k], Bc = conj Z[M-k], w = W_2M^k.  For k = 0 this gives X[0] and X[M] (both real).
__device__ __forceinline__ void untangle(cplx A, cplx Bc, cplx w, cplx& Xk, cplx& Xmk)
{
    const cplx xe = mk(0.5f * (A.x + Bc.x), 0.5f * (A.y + Bc.y));
    const cplx xo = mul_neg_i(mk(0.5f * (A.x - Bc.x), 0.5f * (A.y - Bc.y)));
    const cplx wx = cmul(w, xo);
    Xk = cadd(xe, wx);
    Xmk = conj(csub(xe, wx));
}

// The inverse: from bins Y[k], Y[M-k] of a real sequence's spectrum to Z[k], Z[M-k] of its packing.
//   Ye = (Y[k] + conj Y[M-k]) / 2, Yo = (Y[k] - conj Y[M-k]) / 2 * conj(W_2M^k); Z[k] = Ye + i Yo,
//   Z[M-k] = conj(Ye) + i conj(Yo).  For k = 0 (Y[0], Y[M] real) Z[0] = (Y0 + YM)/2 + i (Y0 - YM)/2.
__device__ __forceinline__ void tangle(cplx Yk, cplx Ymk, cplx w, cplx& Zk, cplx& Zmk)
{
    const cplx Yc = conj(Ymk);
    const cplx ye = mk(0.5f * (Yk.x + Yc.x), 0.5f * (Yk.y + Yc.y));
    const cplx yo = cmul(mk(0.5f * (Yk.x - Yc.x), 0.5f * (Yk.y - Yc.y)), conj(w));
    Zk = cadd(ye, mul_pos_i(yo));
    Zmk = cadd(conj(ye), mul_pos_i(conj(yo)));
}


// One sequence of L <= M steps in registers: the pairs (x[2n], x[2n+1]) for n = tid + T i.  Only n < M/2 can lie
// inside the sequence, so half of a thread's M/T slots are enough.  A kernel that walks several sequences fetches the
// next one into these registers while the transforms of the current one run.
template <int M, int T, typename IO>
struct SeqRegs {
    static constexpr int HELD = M / T / 2;
    typename IoPair<IO>::raw_t r[HELD];
    // vec_ok: x sits on a pair boundary (rows of an even number of steps; a block of a longer row may hold an even
    // number of steps and still start on an odd element, so the blocked kernels pass the parity of the whole row)
    __device__ __forceinline__ void load(const IO* __restrict__ x, int L, int tid) { load(x, L, tid, (L & 1) == 0); }
    __device__ __forceinline__ void load(const IO* __restrict__ x, int L, int tid, bool vec_ok)
    {
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            const int t = 2 * (tid + T * i);
            r[i] = IoPair<IO>::raw_zero();
            if (t < L) r[i] = vec_ok ? IoPair<IO>::raw_pair(x + t) : IoPair<IO>::raw_scalars(x + t, t + 1 < L);
        }
    }
};

// x (one sequence of L steps, in registers) -> optional short kernel and activation -> packed complex
// z[n] = v[2n] + i v[2n+1] in a[], zero beyond L.  Ends with the data in place but NOT synchronised.
// hist (only read with a short kernel): null for a sequence's first step (zero history), else a pointer at the first
// of these L steps inside a longer row, whose 32 predecessors are then the history.
template <int M, int T, typename IO>
__device__ __forceinline__ void stage_input(const SeqRegs<M, T, IO>& x, const float* __restrict__ wc, int m, int L,
                                            cplx* a, int tid, const IO* __restrict__ hist = nullptr)
{
    constexpr int PER = M / T, HELD = PER / 2;
    if (wc != nullptr) {
        // raw x as floats behind 32 steps of history (zeros at a sequence's start), so that no tap needs a bounds check
        float* sx = reinterpret_cast<float*>(a);
        constexpr int ZP = 32;
        if (tid < ZP) sx[tid] = hist != nullptr ? (float)hist[tid - ZP] : 0.f;
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            const int t = 2 * (tid + T * i);
            if (t < L) {
                float v0, v1;
                IoPair<IO>::unpack(x.r[i], v0, v1);
                *reinterpret_cast<float2*>(sx + ZP + t) = make_float2(v0, v1);
            }
        }
        __syncthreads();
        cplx z[HELD];
#pragma unroll
        for (int i = 0; i < HELD; ++i) z[i] = mk(0.f, 0.f);
        // outputs t and t+1 share all but one of their inputs; x is read in aligned pairs (x[t-2p], x[t-2p+1]):
        // x[t-2p+1] meets taps 2p (for t+1) and 2p-1 (for t), x[t-2p] meets taps 2p+1 (for t+1) and 2p (for t)
        for (int p = 0; 2 * p <= m; ++p) {
            const float w2p = 2 * p < m ? wc[2 * p] : 0.f, w2pm1 = p > 0 ? wc[2 * p - 1] : 0.f;
            const float w2pp1 = 2 * p + 1 < m ? wc[2 * p + 1] : 0.f;
#pragma unroll
            for (int i = 0; i < HELD; ++i) {
                const int t = 2 * (tid + T * i);
                if (t < L) {
                    const float2 xv = *reinterpret_cast<const float2*>(sx + ZP + t - 2 * p);
                    z[i].y = fmaf(w2p, xv.y, fmaf(w2pp1, xv.x, z[i].y));
                    z[i].x = fmaf(w2pm1, xv.y, fmaf(w2p, xv.x, z[i].x));
                }
            }
        }
#pragma unroll
        for (int i = 0; i < HELD; ++i) {
            const int t = 2 * (tid + T * i);
            z[i].x = z[i].x * __builtin_amdgcn_rcpf(1.f + __expf(-z[i].x));
            z[i].y = (t + 1 < L) ? z[i].y * __builtin_amdgcn_rcpf(1.f + __expf(-z[i].y)) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < PER; ++i) a[conv_pad(tid + T * i)] = i < HELD ? z[i < HELD ? i : 0] : mk(0.f, 0.f);
    } else {
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            float v0 = 0.f, v1 = 0.f;
            if (i < HELD) IoPair<IO>::unpack(x.r[i < HELD ? i : 0], v0, v1);
            a[conv_pad(tid + T * i)] = mk(v0, v1);
        }
    }
}

// Kernel spectrum of one channel: (K[k], K[M-k]) for the M/2 + 1 bin pairs in pair order, complex fp32.
template <int M>
__global__ __launch_bounds__(conv_threads(M)) void longconv_spectrum_kernel(const float* __restrict__ k,
                                                                           float4* __restrict__ Kf, int L)
{
    constexpr int T = conv_threads(M);
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const long c = blockIdx.x;
    build_tables<M, T>(lo, hi, tid);
    SeqRegs<M, T, float> kr;
    kr.load(k + c * (long)L, L, tid);
    stage_input<M, T, float>(kr, nullptr, 0, L, a, tid);
    __syncthreads();
    fft_passes<M, T, false>(a, lo, hi, tid);
    __syncthreads();
    float4* out = Kf + c * (long)(M / 2 + 1);
    for (int l = tid; l <= M / 2; l += T) {
        const int kk = pair_bin<M>(l);
        cplx Xk, Xmk;
        untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]), w2m(kk, M), Xk,
                 Xmk);
        out[l] = make_float4(Xk.x, Xk.y, Xmk.x, Xmk.y);
    }
}

// Workgroup g takes the sequences (b, c) = g, g + gridDim.x, ... of the B d in turn (w_short == nullptr: no short
// kernel and no activation, the plain long convolution).  The launch holds no more workgroups than are resident
// at once, so that the tables are built once per workgroup, a sequence's input is fetched while the inverse transform
// of the one before runs, and its kernel spectrum while the forward transform runs: with one workgroup per sequence
// each of those latencies was exposed once per sequence, since at the larger sizes a compute unit holds one
// workgroup only.
template <int M, typename IN, typename OUT>
__global__ __launch_bounds__(conv_threads(M)) void shortlong_conv_kernel(const IN* __restrict__ X,
                                                                        const float* __restrict__ w_short, int m,
                                                                        const float4* __restrict__ Kf,
                                                                        OUT* __restrict__ Y, int d, int L, long total)
{
    constexpr int T = conv_threads(M);
    constexpr int NP = (M / 2) / T + 1;          // bin pairs per thread (the last one only exists for l = M/2)
    constexpr bool FRESH = true;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    build_tables<M, T>(lo, hi, tid);
    // The storage positions of a thread's bin pairs (k, M - k), packed two to a register: the one thing that does not
    // depend on the sequence and is worth its registers (some 40 instructions per pair and sequence otherwise).
    unsigned pos[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int l = tid + T * i, kk = pair_bin<M>(l <= M / 2 ? l : 0);
        pos[i] = (unsigned)conv_pad(spectrum_pos<M>(kk)) | (unsigned)conv_pad(spectrum_pos<M>((M - kk) & (M - 1))) << 16;
    }
    SeqRegs<M, T, IN> xr;
    long bc = blockIdx.x;
    if (bc < total) xr.load(X + bc * (long)L, L, tid);
    for (; bc < total; bc += gridDim.x) {
        const int c = (int)(bc % d);
        OUT* y = Y + bc * (long)L;
        // what depends on the thread but not on the sequence (LDS addresses, bin positions, twiddles) is recomputed
        // per sequence behind an opaque copy of the thread index: hoisted out of this loop it would fill the
        // register file.  Every stage takes a fresh copy, so that values shared between stages do not stay live in
        // between (the registers go to the bin-pair positions above instead).
        int tp = tid;
        asm volatile("" : "+v"(tp));
        __syncthreads();        // the tables are built / the previous sequence has been read out of a[]
        stage_input<M, T, IN>(xr, w_short ? w_short + (long)c * m : nullptr, m, L, a, tp);
        const float4* Kc = Kf + (long)c * (M / 2 + 1);
        float4 kq[NP];
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int l = tp + T * i;
            if (l <= M / 2) kq[i] = Kc[l];
        }
        __syncthreads();

        if constexpr (FRESH) { tp = tid; asm volatile("" : "+v"(tp)); }
        fft_passes<M, T, false>(a, lo, hi, tp);
        __syncthreads();

        // ---- spectrum of v times spectrum of the kernel, re-packed for the inverse transform (pairs k, M - k)
        if constexpr (FRESH) { tp = tid; asm volatile("" : "+v"(tp)); }
        {
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) {
                    const int p1 = pos[i] & 0xffffu, p2 = pos[i] >> 16;
                    const cplx w = pw.next(l);
                    cplx Xk, Xmk, Zk, Zmk;
                    untangle(a[p1], conj(a[p2]), w, Xk, Xmk);
                    const cplx K1 = mk(kq[i].x, kq[i].y), K2 = mk(kq[i].z, kq[i].w);
                    if (l == 0) {       // (pair 0 is bin 0)
                        // bins 0 and M are real and share storage slot 0
                        const float y0 = Xk.x * K1.x, ym = Xmk.x * K2.x;
                        a[p1] = mk(0.5f * (y0 + ym), 0.5f * (y0 - ym));
                    } else {
                        tangle(cmul(Xk, K1), cmul(Xmk, K2), w, Zk, Zmk);
                        a[p1] = Zk;
                        if (p2 != p1) a[p2] = Zmk;
                    }
                }
            }
        }
        if (bc + gridDim.x < total) xr.load(X + (bc + gridDim.x) * (long)L, L, tp);     // the next sequence, in flight
        __syncthreads();

        if constexpr (FRESH) { tp = tid; asm volatile("" : "+v"(tp)); }
        fft_passes<M, T, true>(a, lo, hi, tp);
        __syncthreads();

        // ---- unpack, scale, store
        const bool vec_ok = (L & 1) == 0;
        const float scale = 1.0f / (float)M;
#pragma unroll
        for (int i = 0; i < M / T / 2; ++i) {
            const int n = tp + T * i, t = 2 * n;
            if (t < L) {
                const cplx v = a[conv_pad(n)];
                if (vec_ok) IoPair<OUT>::store2(y + t, v.x * scale, v.y * scale);
                else { y[t] = (OUT)(v.x * scale); if (t + 1 < L) y[t + 1] = (OUT)(v.y * scale); }
            }
        }
    }
}

// The two long-stage gradients in one kernel: they share the spectrum of dZ.  One workgroup per channel walks the
// batch; per sequence it transforms dZ once, keeps the untangled bins of its own bin pairs in registers, multiplies
// by the CONJUGATE kernel spectrum (correlation instead of convolution: dV[t] = sum_{s >= t} k[s - t] dZ[s]) and
// transforms back (out as DVT: fp32 scratch for the short-stage kernel, or dX itself when there is no short stage),
// then transforms v = silu(K_s x) (recomputed from x) and adds DZ conj(V) to the running sums of its bin pairs (in
// registers, at the largest size in memory); after the last sequence the sums are transformed back once (dk).  Three
// transforms per sequence, where a correlation kernel and a kernel-gradient kernel of their own would need four.
// SPLIT: grid.y workgroups share a channel, each takes every grid.y-th sequence and leaves its sums in its own slice
// of the scratch array ([grid.y][d][M/2 + 1] pairs); longconv_dk_finish_kernel adds the slices up and transforms back.
// Used when there are too few channels to fill the GPU.
template <int M, typename IO, typename DVT, bool SPLIT>
__global__ __launch_bounds__(conv_threads(M)) void longconv_bwd_kernel(const IO* __restrict__ X,
                                                                      const float* __restrict__ w_short, int m,
                                                                      const float4* __restrict__ Kf,
                                                                      const IO* __restrict__ dZ,
                                                                      DVT* __restrict__ dV, float* __restrict__ dk,
                                                                      float4* __restrict__ acc_ws, int B, int d, int L)
{
    constexpr int T = conv_threads(M);
    constexpr int NP = (M / 2) / T + 1;                  // bin pairs per thread
    // At the largest size 1024 threads share the register file: the running sums then live in a scratch array in
    // memory ([d][M/2 + 1] pairs; every thread only ever touches its own pairs, between uses they sit in the caches).
    constexpr bool ACC_MEM = M >= 16384;
    float4* accm = (ACC_MEM || SPLIT) ? acc_ws + ((long)blockIdx.y * d + blockIdx.x) * (M / 2 + 1) : nullptr;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const int c = blockIdx.x;
    build_tables<M, T>(lo, hi, tid);
    const float4* Kc = Kf + (long)c * (M / 2 + 1);
    const float* wc = w_short ? w_short + (long)c * m : nullptr;
    const bool vec_ok = (L & 1) == 0;
    const float scale = 1.0f / (float)M;
    cplx accK[ACC_MEM ? 1 : NP], accMK[ACC_MEM ? 1 : NP], Gk[NP], Gmk[NP];
    if constexpr (!ACC_MEM) {
#pragma unroll
        for (int i = 0; i < NP; ++i) { accK[i] = mk(0.f, 0.f); accMK[i] = mk(0.f, 0.f); }
    }

    // Inputs are fetched one stage ahead, into registers: dZ of the next sequence while v is transformed, x while the
    // correlation is transformed back.
    SeqRegs<M, T, IO> zr, xr;
    if ((int)blockIdx.y < B) zr.load(dZ + ((long)blockIdx.y * d + c) * L, L, tid);
    for (int b = blockIdx.y; b < B; b += gridDim.y) {
        const long row = ((long)b * d + c) * L;
        // what depends on the thread but not on the sequence (LDS addresses, bin positions, twiddles) is recomputed per
        // sequence behind an opaque copy of the thread index: left visible, the compiler keeps all of it in registers
        // across the transforms and spills
        // (a fresh copy per stage, or positions shared between stages stay live across the transforms between them)
        int tp = tid;
        asm volatile("" : "+v"(tp));
        // ---- spectrum of dZ; correlation with the kernel: DZ conj(K)
        stage_input<M, T, IO>(zr, nullptr, 0, L, a, tp);
        __syncthreads();
        fft_passes<M, T, false>(a, lo, hi, tp);
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        xr.load(X + row, L, tp);
        {
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    const int p1 = conv_pad(spectrum_pos<M>(kk)), p2 = conv_pad(spectrum_pos<M>((M - kk) & (M - 1)));
                    const cplx w = pw.next(l);
                    untangle(a[p1], conj(a[p2]), w, Gk[i], Gmk[i]);
                    const float4 kq = Kc[l];
                    const cplx K1 = mk(kq.x, -kq.y), K2 = mk(kq.z, -kq.w);
                    if (kk == 0) {
                        const float y0 = Gk[i].x * K1.x, ym = Gmk[i].x * K2.x;
                        a[p1] = mk(0.5f * (y0 + ym), 0.5f * (y0 - ym));
                    } else {
                        cplx Zk, Zmk;
                        tangle(cmul(Gk[i], K1), cmul(Gmk[i], K2), w, Zk, Zmk);
                        a[p1] = Zk;
                        if (p2 != p1) a[p2] = Zmk;
                    }
                }
                __builtin_amdgcn_sched_barrier(0);   // one pair at a time: the unrolled pairs must not pile up in registers
            }
        }
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        fft_passes<M, T, true>(a, lo, hi, tp);
        __syncthreads();
        {
            DVT* y = dV + row;
#pragma unroll
            for (int i = 0; i < M / T / 2; ++i) {
                const int n = tp + T * i, t = 2 * n;
                if (t < L) {
                    const cplx v = a[conv_pad(n)];
                    if (vec_ok) IoPair<DVT>::store2(y + t, v.x * scale, v.y * scale);
                    else { y[t] = (DVT)(v.x * scale); if (t + 1 < L) y[t + 1] = (DVT)(v.y * scale); }
                }
            }
        }
        __syncthreads();
        // ---- spectrum of v = silu(K_s x) (x itself without a short stage); running sums of DZ conj(V)
        tp = tid;
        asm volatile("" : "+v"(tp));
        stage_input<M, T, IO>(xr, wc, m, L, a, tp);
        if (b + (int)gridDim.y < B) zr.load(dZ + ((long)(b + gridDim.y) * d + c) * L, L, tp);
        __syncthreads();
        fft_passes<M, T, false>(a, lo, hi, tp);
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        {
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    const cplx w = pw.next(l);
                    cplx Vk, Vmk;
                    untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]), w,
                             Vk, Vmk);
                    const cplx pk = cmul(Gk[i], conj(Vk)), pmk = cmul(Gmk[i], conj(Vmk));
                    if constexpr (ACC_MEM) {
                        float4 t = make_float4(pk.x, pk.y, pmk.x, pmk.y);
                        if (b != (int)blockIdx.y) { const float4 o = accm[l]; t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w; }
                        accm[l] = t;
                    } else {
                        accK[i] = cadd(accK[i], pk);
                        accMK[i] = cadd(accMK[i], pmk);
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
    }
    if constexpr (SPLIT) {
        // this workgroup's share of the sums stays in its slice of the scratch array (it is there already when the
        // sums were kept in memory)
        if constexpr (!ACC_MEM) {
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tid + T * i;
                if (l <= M / 2) accm[l] = make_float4(accK[i].x, accK[i].y, accMK[i].x, accMK[i].y);
            }
        }
        return;
    }
    {
        PairTwiddle<M, T> pw(tid);
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int l = tid + T * i;
            if (l <= M / 2) {
                const int kk = pair_bin<M>(l);
                const int p1 = conv_pad(spectrum_pos<M>(kk)), p2 = conv_pad(spectrum_pos<M>((M - kk) & (M - 1)));
                const cplx w = pw.next(l);
                cplx sk, smk;
                if constexpr (ACC_MEM) {
                    const float4 t = B > 0 ? accm[l] : make_float4(0.f, 0.f, 0.f, 0.f);
                    sk = mk(t.x, t.y);
                    smk = mk(t.z, t.w);
                } else {
                    sk = accK[i];
                    smk = accMK[i];
                }
                if (kk == 0) {
                    a[p1] = mk(0.5f * (sk.x + smk.x), 0.5f * (sk.x - smk.x));
                } else {
                    cplx Zk, Zmk;
                    tangle(sk, smk, w, Zk, Zmk);
                    a[p1] = Zk;
                    if (p2 != p1) a[p2] = Zmk;
                }
            }
        }
    }
    __syncthreads();
    fft_passes<M, T, true>(a, lo, hi, tid);
    __syncthreads();
    float* out = dk + (long)c * L;
    for (int n = tid; n < M; n += T) {
        const int t = 2 * n;
        if (t < L) {
            const cplx v = a[conv_pad(n)];
            out[t] = v.x * scale;
            if (t + 1 < L) out[t + 1] = v.y * scale;
        }
    }
}

// Gradient through the activation and the short kernel.  dV is the gradient with respect to v = silu(u), u = K_s x:
//   dU = dV silu'(u),  dX[t] = sum_j w[j] dU[t+j],  dw[c][j] = sum_b sum_t dU[b,c,t] x[b,c,t-j].
// The (batch entry, tile of TL steps) pairs of a channel are dealt out to workgroups in runs of kShortTilesPerWg
// (a run may cross from one sequence into the next); x is staged with MT steps of history and dU with MT steps of
// look-ahead.  Each workgroup leaves its share of the tap sums in `part` ([d][n_share][MT]); shortconv_dw_kernel
// adds the shares of a channel in a fixed order.
constexpr int kShortTile = 2048, kShortMaxTaps = 32, kShortTilesPerWg = 4;

// TAPS: compile-time bound on the number of taps (m <= TAPS <= 32): the tap loops are as long as the kernel needs.
// Up to 16 taps every count has its own instantiation (the paper's sizes, 3 and 2 log10 L + 1, stay below 16 for any
// L up to 10^7) with 16 steps of history and look-ahead; longer kernels share one with 32.
template <typename IO, int TAPS>
__global__ __launch_bounds__(256) void shortconv_bwd_kernel(const IO* __restrict__ X, const float* __restrict__ w_short,
                                                           int m, const float* __restrict__ dV, IO* __restrict__ dX,
                                                           float* __restrict__ part, int B, int d, int L, int n_share)
{
    constexpr int TL = kShortTile, MT = TAPS <= 16 ? 16 : 32, H = MT;  // H: halo on either side
    constexpr int NX = MT + 8;                                        // inputs behind eight consecutive outputs
    __shared__ __attribute__((aligned(16))) float sx[TL + 2 * H];      // x[t0 - H .. t0 + TL + H)
    __shared__ __attribute__((aligned(16))) float su[TL + H + 8];      // dU[t0 .. t0 + TL + H) (+ slack for 16-byte reads)
    __shared__ float red[MT][4];
    const int tid = threadIdx.x, c = blockIdx.x % d, share = blockIdx.x / d;      // channels fastest
    const int tiles_per_row = (L + TL - 1) / TL, n_items = B * tiles_per_row;
    float wreg[TAPS], acc[TAPS];
#pragma unroll
    for (int j = 0; j < TAPS; ++j) { wreg[j] = j < m ? w_short[(long)c * m + j] : 0.f; acc[j] = 0.f; }
    const bool vec8 = (L & 7) == 0;       // every row starts 16-byte aligned
    for (int item = share * kShortTilesPerWg; item < (share + 1) * kShortTilesPerWg && item < n_items; ++item) {
    const int b = item / tiles_per_row, t0 = (item - b * tiles_per_row) * TL;
    const long row = ((long)b * d + c) * L;
    __syncthreads();
    for (int i8 = tid; i8 < (TL + 2 * H) / 8; i8 += 256) {      // eight steps per thread: one 16-byte load where whole
        const int t = t0 - H + 8 * i8;
        float xv[8];
        if (vec8 && t >= 0 && t + 8 <= L) load8(X + row + t, xv);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) xv[e] = (t + e >= 0 && t + e < L) ? (float)X[row + t + e] : 0.f;
        }
        *reinterpret_cast<float4*>(sx + 8 * i8) = make_float4(xv[0], xv[1], xv[2], xv[3]);
        *reinterpret_cast<float4*>(sx + 8 * i8 + 4) = make_float4(xv[4], xv[5], xv[6], xv[7]);
    }
    __syncthreads();
    // each thread takes 8 consecutive steps: the MT + 8 inputs they need are read once, as 16-byte LDS reads
    {
        const int i0 = 8 * tid;                         // TL = 8 * 256
        float xs[NX];                                   // x[t0 + i0 - MT .. t0 + i0 + 8)
#pragma unroll
        for (int r = 0; r < NX / 4; ++r) {
            const float4 v = *reinterpret_cast<const float4*>(sx + i0 + 4 * r);      // sx index of x[t0 + i] is H + i
            xs[4 * r] = v.x; xs[4 * r + 1] = v.y; xs[4 * r + 2] = v.z; xs[4 * r + 3] = v.w;
        }
        float du8[8], g8[8];
        const int tc = t0 + i0;
        const bool whole = vec8 && tc + 8 <= L;         // eight steps in range at a 16-byte aligned address
        if (whole) {
            const float4 a0 = *reinterpret_cast<const float4*>(dV + row + tc), a1 = *reinterpret_cast<const float4*>(dV + row + tc + 4);
            g8[0] = a0.x; g8[1] = a0.y; g8[2] = a0.z; g8[3] = a0.w; g8[4] = a1.x; g8[5] = a1.y; g8[6] = a1.z; g8[7] = a1.w;
        } else {
#pragma unroll
            for (int e = 0; e < 8; ++e) g8[e] = tc + e < L ? dV[row + tc + e] : 0.f;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float u = 0.f;
#pragma unroll
            for (int j = 0; j < TAPS; ++j) u = fmaf(wreg[j], xs[MT + e - j], u);
            const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-u));
            du8[e] = tc + e < L ? g8[e] * sg * (1.f + u * (1.f - sg)) : 0.f;
        }
        *reinterpret_cast<float4*>(su + i0) = make_float4(du8[0], du8[1], du8[2], du8[3]);
        *reinterpret_cast<float4*>(su + i0 + 4) = make_float4(du8[4], du8[5], du8[6], du8[7]);
    }
    if (tid < H) {
        // the H steps of look-ahead beyond the tile, one per thread (as two more 8-step pieces they would double the
        // first wave's share of this phase)
        const int i = TL + tid, t = t0 + i;
        float u = 0.f;
#pragma unroll
        for (int j = 0; j < TAPS; ++j) u = fmaf(wreg[j], sx[H + i - j], u);
        const float sg = __builtin_amdgcn_rcpf(1.f + __expf(-u));
        su[i] = t < L ? dV[row + t] * sg * (1.f + u * (1.f - sg)) : 0.f;
    }
    __syncthreads();
    {
        const int i0 = 8 * tid;                         // TL = 8 * 256
        float xs[NX], ds[NX];                           // x as above; dU[t0 + i0 .. t0 + i0 + MT + 8)
#pragma unroll
        for (int r = 0; r < NX / 4; ++r) {
            const float4 v = *reinterpret_cast<const float4*>(sx + i0 + 4 * r);
            xs[4 * r] = v.x; xs[4 * r + 1] = v.y; xs[4 * r + 2] = v.z; xs[4 * r + 3] = v.w;
            const float4 g = *reinterpret_cast<const float4*>(su + i0 + 4 * r);
            ds[4 * r] = g.x; ds[4 * r + 1] = g.y; ds[4 * r + 2] = g.z; ds[4 * r + 3] = g.w;
        }
        float dx8[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float dx = 0.f;
#pragma unroll
            for (int j = 0; j < TAPS; ++j) {
                dx = fmaf(wreg[j], ds[e + j], dx);
                acc[j] = fmaf(ds[e], xs[MT + e - j], acc[j]);
            }
            dx8[e] = dx;
        }
        const int tc = t0 + i0;
        if (vec8 && tc + 8 <= L) store8(dX + row + tc, dx8);
        else {
#pragma unroll
            for (int e = 0; e < 8; ++e) if (tc + e < L) dX[row + tc + e] = (IO)dx8[e];
        }
    }
    }
    // this workgroup's tap sums: wave reduction, then across the four waves
#pragma unroll
    for (int j = 0; j < TAPS; ++j) {
        float v = acc[j];
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
        if ((tid & 63) == 0) red[j][tid >> 6] = v;
    }
    __syncthreads();
    if (tid < TAPS)
        part[((long)c * n_share + share) * kShortMaxTaps + tid] = red[tid][0] + red[tid][1] + red[tid][2] + red[tid][3];
}

__global__ __launch_bounds__(64) void shortconv_dw_kernel(const float* __restrict__ part, float* __restrict__ dw, int m,
                                                         int n_share)
{
    const int c = blockIdx.x, j = threadIdx.x;
    if (j >= m) return;
    float t = 0.f;
    for (int s = 0; s < n_share; ++s) t += part[((long)c * n_share + s) * kShortMaxTaps + j];
    dw[(long)c * m + j] = t;
}


// =============================================================================================== sequences beyond one transform
// L > 16384: the sequence and the long kernel are cut into blocks of BK = 16384 steps, x_0 .. x_{nb-1} and
// k_0 .. k_{nb-1}.  Output block j of the causal sum is
//     y_j = sum_{i <= j}  low half of  circ_{2 BK}( [x_i ; 0] , [k_{j-i} ; k_{j-i-1}] )          (k_{-1} = 0)
// (the taps that reach from block i into block j are the 2 BK - 1 taps around lag (j - i) BK: the upper half of the
// second operand holds the ones below that lag, which a circular product of length 2 BK wraps onto the low outputs
// exactly where they belong).  So every block is transformed by the same length-M machinery as a short sequence
// (zero upper half in, low half out), the sum over i is taken on the spectra, in registers, and one inverse
// transform per output block follows.  The spectrum of [k_m ; k_{m-1}] is A_m + (-1)^bin A_{m-1} with A_m the
// spectrum of [k_m ; 0] (a shift by half the period), which is what longconv_spectrum_blocked_kernel stores:
// [d][nb][M/2 + 1] pairs in pair order.  The two long-stage gradients have the same shape:
//     dv_i = sum_{j >= i} low half of the circular CORRELATION of [dz_j ; 0] with [k_{j-i} ; k_{j-i-1}]   (conjugate spectra),
//     dk_m = low half of the inverse of  D_m + (-1)^bin D_{m+1},   D_m = sum_b sum_i DZ_{i+m} conj(V_i).
// The work per sequence grows with nb (nb + 1) / 2 block pairs, against nb log nb for one long transform held in
// memory: this path is here so that no length is refused, not to be the fastest way to convolve a million steps.
constexpr int kBlkM = 16384;                 // transform length and block length (steps)
// Threads per workgroup of the blocked kernels.  1024 leave each thread 128 registers, which the 36 accumulators of the
// forward kernel overflow (40-70 spilled registers); 512 threads with 256 registers each spill nothing and were
// measured slower all the same (2.39 against 1.94 ms at B1 d2048 L65536): sixteen waves hide the transforms' LDS
// latencies better than eight.
constexpr int kBlkT = conv_threads(kBlkM);

// Spectra G_m of the blocks of the long kernel; one workgroup per (channel, block).
__global__ __launch_bounds__(kBlkT) void longconv_spectrum_blocked_kernel(const float* __restrict__ k,
                                                                                       float4* __restrict__ Gf, int L,
                                                                                       int nb)
{
    constexpr int M = kBlkM, T = kBlkT, NP = (M / 2) / T + 1;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const long c = blockIdx.x;
    const int mb = blockIdx.y;
    const bool row_vec = (L & 1) == 0;
    build_tables<M, T>(lo, hi, tid);
    float4 sum[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) sum[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int which = (mb > 0 ? mb - 1 : mb); which <= mb; ++which) {
        const int len = min(M, L - which * M);
        SeqRegs<M, T, float> kr;
        kr.load(k + c * (long)L + (long)which * M, len, tid, row_vec);
        __syncthreads();                  // tables built / the block before has been read out of a[]
        stage_input<M, T, float>(kr, nullptr, 0, len, a, tid);
        __syncthreads();
        fft_passes<M, T, false>(a, lo, hi, tid);
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            const int l = tid + T * i;
            if (l <= M / 2) {
                const int kk = pair_bin<M>(l);
                cplx Xk, Xmk;
                untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]),
                         w2m(kk, M), Xk, Xmk);
                // the block before sits in the upper half of the period: (-1)^bin (bins kk and M - kk: same parity)
                const float sg = (which < mb && (kk & 1)) ? -1.f : 1.f;
                sum[i].x += sg * Xk.x; sum[i].y += sg * Xk.y; sum[i].z += sg * Xmk.x; sum[i].w += sg * Xmk.y;
            }
        }
    }
    float4* out = Gf + (c * nb + mb) * (long)(M / 2 + 1);
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        const int l = tid + T * i;
        if (l <= M / 2) out[l] = sum[i];
    }
}

// Forward (CORR = false: X -> optional short kernel and activation -> causal sum with the long kernel, block `blk` of
// the output from the blocks 0 .. blk of the input) and correlation (CORR = true: dZ -> dV, block blk from the blocks
// blk .. nb-1, conjugate spectra; no short stage).  Work items (sequence, output block), the costliest blocks first,
// dealt to a launch of no more workgroups than are resident at once.
template <typename IN, typename OUT, bool CORR>
__global__ __launch_bounds__(kBlkT) void longconv_blocked_kernel(const IN* __restrict__ X,
                                                                              const float* __restrict__ w_short, int m,
                                                                              const float4* __restrict__ Gf,
                                                                              OUT* __restrict__ Y, int d, int L, int nb,
                                                                              long BD)
{
    constexpr int M = kBlkM, T = kBlkT, NP = (M / 2) / T + 1;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const bool row_vec = (L & 1) == 0;
    const float scale = 1.0f / (float)M;
    build_tables<M, T>(lo, hi, tid);
    const long items = BD * nb;
    for (long id = blockIdx.x; id < items; id += gridDim.x) {
        const int r = (int)(id / BD);
        const long bc = id - (long)r * BD;
        const int blk = CORR ? r : nb - 1 - r;            // costliest first: nb - blk (CORR) or blk + 1 input blocks
        const int c = (int)(bc % d);
        const int o0 = CORR ? blk : 0, o1 = CORR ? nb - 1 : blk;
        const IN* xrow = X + bc * (long)L;
        const float* wc = (!CORR && w_short) ? w_short + (long)c * m : nullptr;
        cplx accK[NP], accMK[NP];                           // sums over the input blocks of X_o G_|o - blk|, bins k and M - k
#pragma unroll
        for (int i = 0; i < NP; ++i) { accK[i] = mk(0.f, 0.f); accMK[i] = mk(0.f, 0.f); }
        SeqRegs<M, T, IN> xr;
        xr.load(xrow + (long)o0 * M, min(M, L - o0 * M), tid, row_vec);
        for (int o = o0; o <= o1; ++o) {
            int tp = tid;
            asm volatile("" : "+v"(tp));
            __syncthreads();    // tables built / a[] has been read out
            stage_input<M, T, IN>(xr, wc, m, min(M, L - o * M), a, tp, (wc && o > 0) ? xrow + (long)o * M : nullptr);
            if (o < o1) xr.load(xrow + (long)(o + 1) * M, min(M, L - (o + 1) * M), tp, row_vec);   // the next block, in flight
            __syncthreads();
            tp = tid;
            asm volatile("" : "+v"(tp));
            fft_passes<M, T, false>(a, lo, hi, tp);
            __syncthreads();
            tp = tid;
            asm volatile("" : "+v"(tp));
            const float4* Gc = Gf + ((long)c * nb + (CORR ? o - blk : blk - o)) * (long)(M / 2 + 1);
            float4 kq[NP];
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) kq[i] = Gc[l];
            }
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    const cplx w = pw.next(l);
                    cplx Xk, Xmk;
                    untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]), w,
                             Xk, Xmk);
                    const cplx K1 = mk(kq[i].x, CORR ? -kq[i].y : kq[i].y), K2 = mk(kq[i].z, CORR ? -kq[i].w : kq[i].w);
                    accK[i] = cadd(accK[i], cmul(Xk, K1));
                    accMK[i] = cadd(accMK[i], cmul(Xmk, K2));
                }
                __builtin_amdgcn_sched_barrier(0);   // one pair at a time: the unrolled pairs must not pile up in registers
            }
        }
        __syncthreads();        // every thread has read its bins of the last input block
        {
            int tp = tid;
            asm volatile("" : "+v"(tp));
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int i = 0; i < NP; ++i) {
                const int l = tp + T * i;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    const int p1 = conv_pad(spectrum_pos<M>(kk)), p2 = conv_pad(spectrum_pos<M>((M - kk) & (M - 1)));
                    const cplx w = pw.next(l);
                    if (kk == 0) {      // bins 0 and M are real and share storage slot 0
                        a[p1] = mk(0.5f * (accK[i].x + accMK[i].x), 0.5f * (accK[i].x - accMK[i].x));
                    } else {
                        cplx Zk, Zmk;
                        tangle(accK[i], accMK[i], w, Zk, Zmk);
                        a[p1] = Zk;
                        if (p2 != p1) a[p2] = Zmk;
                    }
                }
            }
        }
        __syncthreads();
        {
            int tp = tid;
            asm volatile("" : "+v"(tp));
            fft_passes<M, T, true>(a, lo, hi, tp);
            __syncthreads();
            OUT* y = Y + bc * (long)L + (long)blk * M;
            const int len = min(M, L - blk * M);
#pragma unroll
            for (int i = 0; i < M / T / 2; ++i) {
                const int n = tp + T * i, t = 2 * n;
                if (t < len) {
                    const cplx v = a[conv_pad(n)];
                    if (row_vec) IoPair<OUT>::store2(y + t, v.x * scale, v.y * scale);
                    else { y[t] = (OUT)(v.x * scale); if (t + 1 < len) y[t + 1] = (OUT)(v.y * scale); }
                }
            }
        }
    }
}

// Sums D_mb = sum_b sum_i DZ_{i+mb} conj(V_i) of one channel and one block distance, kept in memory ([d][nb][M/2 + 1]
// pairs; every thread only ever touches its own pairs).  One workgroup per (channel, distance), the distances with
// the most block pairs first.
template <typename IO>
__global__ __launch_bounds__(kBlkT) void longconv_dk_blocked_kernel(const IO* __restrict__ X,
                                                                                 const float* __restrict__ w_short, int m,
                                                                                 const IO* __restrict__ dZ,
                                                                                 float4* __restrict__ acc_ws, int B, int d,
                                                                                 int L, int nb)
{
    constexpr int M = kBlkM, T = kBlkT, NP = (M / 2) / T + 1;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const int c = blockIdx.x, mb = blockIdx.y;
    const bool row_vec = (L & 1) == 0;
    build_tables<M, T>(lo, hi, tid);
    float4* accm = acc_ws + ((long)c * nb + mb) * (long)(M / 2 + 1);
    const float* wc = w_short ? w_short + (long)c * m : nullptr;
    const int n_i = nb - mb;                     // block pairs (i, i + mb) per sequence
    const long n_pairs = (long)B * n_i;
    cplx Gk[NP], Gmk[NP];
    SeqRegs<M, T, IO> zr, xr;
    zr.load(dZ + (long)c * L + (long)mb * M, min(M, L - mb * M), tid, row_vec);      // pair 0: b = 0, i = 0
    for (long pr = 0; pr < n_pairs; ++pr) {
        const int b = (int)(pr / n_i), i = (int)(pr - (long)b * n_i), j = i + mb;
        const long row = ((long)b * d + c) * (long)L;
        int tp = tid;
        asm volatile("" : "+v"(tp));
        __syncthreads();        // tables built / a[] has been read out
        stage_input<M, T, IO>(zr, nullptr, 0, min(M, L - j * M), a, tp);
        xr.load(X + row + (long)i * M, min(M, L - i * M), tp, row_vec);
        __syncthreads();
        fft_passes<M, T, false>(a, lo, hi, tp);
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        {
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int q = 0; q < NP; ++q) {
                const int l = tp + T * q;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]),
                             pw.next(l), Gk[q], Gmk[q]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        stage_input<M, T, IO>(xr, wc, m, min(M, L - i * M), a, tp, (wc && i > 0) ? X + row + (long)i * M : nullptr);
        if (pr + 1 < n_pairs) {
            const int b2 = (int)((pr + 1) / n_i), i2 = (int)(pr + 1 - (long)b2 * n_i);
            zr.load(dZ + ((long)b2 * d + c) * (long)L + (long)(i2 + mb) * M, min(M, L - (i2 + mb) * M), tp, row_vec);
        }
        __syncthreads();
        fft_passes<M, T, false>(a, lo, hi, tp);
        __syncthreads();
        tp = tid;
        asm volatile("" : "+v"(tp));
        {
            PairTwiddle<M, T> pw(tp);
#pragma unroll
            for (int q = 0; q < NP; ++q) {
                const int l = tp + T * q;
                if (l <= M / 2) {
                    const int kk = pair_bin<M>(l);
                    cplx Vk, Vmk;
                    untangle(a[conv_pad(spectrum_pos<M>(kk))], conj(a[conv_pad(spectrum_pos<M>((M - kk) & (M - 1)))]),
                             pw.next(l), Vk, Vmk);
                    const cplx pk = cmul(Gk[q], conj(Vk)), pmk = cmul(Gmk[q], conj(Vmk));
                    float4 t = make_float4(pk.x, pk.y, pmk.x, pmk.y);
                    if (pr > 0) { const float4 o = accm[l]; t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w; }
                    accm[l] = t;
                }
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    }
}

// dk block mb of a channel from the sums above: inverse of D_mb + (-1)^bin D_{mb+1}, low half.
__global__ __launch_bounds__(kBlkT) void longconv_dk_blocked_finish_kernel(const float4* __restrict__ acc_ws,
                                                                                        float* __restrict__ dk, int d,
                                                                                        int L, int nb)
{
    constexpr int M = kBlkM, T = kBlkT;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const int c = blockIdx.x, mb = blockIdx.y;
    build_tables<M, T>(lo, hi, tid);
    const float4* D0 = acc_ws + ((long)c * nb + mb) * (long)(M / 2 + 1);
    const float4* D1 = mb + 1 < nb ? D0 + (M / 2 + 1) : nullptr;
    PairTwiddle<M, T> pw(tid);
    for (int l = tid; l <= M / 2; l += T) {
        const int kk = pair_bin<M>(l);
        const int p1 = conv_pad(spectrum_pos<M>(kk)), p2 = conv_pad(spectrum_pos<M>((M - kk) & (M - 1)));
        const cplx w = pw.next(l);
        float4 t = D0[l];
        if (D1 != nullptr) {
            const float4 o = D1[l];
            const float sg = (kk & 1) ? -1.f : 1.f;
            t.x += sg * o.x; t.y += sg * o.y; t.z += sg * o.z; t.w += sg * o.w;
        }
        const cplx sk = mk(t.x, t.y), smk = mk(t.z, t.w);
        if (kk == 0) {
            a[p1] = mk(0.5f * (sk.x + smk.x), 0.5f * (sk.x - smk.x));
        } else {
            cplx Zk, Zmk;
            tangle(sk, smk, w, Zk, Zmk);
            a[p1] = Zk;
            if (p2 != p1) a[p2] = Zmk;
        }
    }
    __syncthreads();
    fft_passes<M, T, true>(a, lo, hi, tid);
    __syncthreads();
    float* out = dk + (long)c * L + (long)mb * M;
    const int len = min(M, L - mb * M);
    const float scale = 1.0f / (float)M;
    for (int n = tid; n < M / 2; n += T) {
        const int t = 2 * n;
        if (t < len) {
            const cplx v = a[conv_pad(n)];
            out[t] = v.x * scale;
            if (t + 1 < len) out[t + 1] = v.y * scale;
        }
    }
}

int conv_fft_size(int L)
{
    if (L <= 256) return 256;
    if (L <= 1024) return 1024;
    if (L <= 4096) return 4096;
    if (L <= 16384) return 16384;
    return 0;
}

hipError_t launch_longconv_spectrum(const float* k, void* Kf, int d, int L, hipStream_t st)
{
    const int M = conv_fft_size(L);
    ProfScope prof(KID_CONV_SPECTRUM, st);
    float4* out = (float4*)Kf;
    if (const int nb = conv_blocks(L)) {
        hipLaunchKernelGGL(longconv_spectrum_blocked_kernel, dim3(d, nb), dim3(kBlkT), 0, st, k, out, L, nb);
        return hipGetLastError();
    }
    switch (M) {
        case 256: hipLaunchKernelGGL((longconv_spectrum_kernel<256>), dim3(d), dim3(conv_threads(256)), 0, st, k, out, L); break;
        case 1024: hipLaunchKernelGGL((longconv_spectrum_kernel<1024>), dim3(d), dim3(conv_threads(1024)), 0, st, k, out, L); break;
        case 4096: hipLaunchKernelGGL((longconv_spectrum_kernel<4096>), dim3(d), dim3(conv_threads(4096)), 0, st, k, out, L); break;
        case 16384: hipLaunchKernelGGL((longconv_spectrum_kernel<16384>), dim3(d), dim3(conv_threads(16384)), 0, st, k, out, L); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Workgroups of `kernel` that the GPU holds at once (what its LDS and registers allow per compute unit x the units).
template <typename K>
static long resident_workgroups(K kernel, int threads)
{
    int per_cu = 0, dev = 0, cus = 0;
    if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, kernel, threads, 0) != hipSuccess || per_cu < 1) per_cu = 1;
    if (hipGetDevice(&dev) != hipSuccess ||
        hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus < 1)
        cus = 256;
    (void)hipGetLastError();
    return (long)cus * per_cu;
}

// The blocked kernel for L > 16384: work items (sequence, output block) over no more workgroups than are resident.
template <typename IN, typename OUT, bool CORR>
static hipError_t conv_blocked_launch(const IN* X, const float* w, int m, const float4* Gf, OUT* Y, long BD, int d, int L,
                                      hipStream_t st)
{
    const int nb = conv_blocks(L);
    static const long slots = resident_workgroups(longconv_blocked_kernel<IN, OUT, CORR>, kBlkT);
    const long items = BD * nb;
    const dim3 grid((unsigned)(items < slots ? items : slots));
    hipLaunchKernelGGL((longconv_blocked_kernel<IN, OUT, CORR>), grid, dim3(kBlkT), 0, st, X, w, m, Gf, Y, d,
                       L, nb, BD);
    return hipGetLastError();
}

template <typename IN, typename OUT>
static hipError_t conv_dispatch(const IN* X, const float* w, int m, const float4* Kf, OUT* Y, long BD, int d, int L,
                                hipStream_t st)
{
    const int M = conv_fft_size(L);
    ProfScope prof(KID_CONV_FWD, st);
    if (conv_blocks(L)) return conv_blocked_launch<IN, OUT, false>(X, w, m, Kf, Y, BD, d, L, st);
    // no more workgroups than are resident at once, each with an equal share of the sequences
#define CHELA_CONV_FWD(M_)                                                                                              \
    case M_: {                                                                                                          \
        static const long slots = resident_workgroups(shortlong_conv_kernel<M_, IN, OUT>, conv_threads(M_));            \
        const long rounds = (BD + slots - 1) / slots;                                                                   \
        const dim3 grid((unsigned)((BD + rounds - 1) / rounds));                                                        \
        hipLaunchKernelGGL((shortlong_conv_kernel<M_, IN, OUT>), grid, dim3(conv_threads(M_)), 0, st, X, w, m, Kf, Y, d, \
                           L, BD);                                                                                      \
    } break;
    switch (M) {
        CHELA_CONV_FWD(256) CHELA_CONV_FWD(1024) CHELA_CONV_FWD(4096) CHELA_CONV_FWD(16384)
        default: return hipErrorInvalidValue;
    }
#undef CHELA_CONV_FWD
    return hipGetLastError();
}

hipError_t launch_shortlong_conv(const void* X, const float* w_short, int m, const void* Kf, void* Y, long BD, int d,
                                 int L, int dtype, hipStream_t st)
{
    if (dtype == 0)
        return conv_dispatch<bf16, bf16>((const bf16*)X, w_short, m, (const float4*)Kf, (bf16*)Y, BD, d, L, st);
    return conv_dispatch<float, float>((const float*)X, w_short, m, (const float4*)Kf, (float*)Y, BD, d, L, st);
}

// Second step of the split long-stage gradient: add up the G slices of a channel's sums, transform back, store dk.
template <int M>
__global__ __launch_bounds__(conv_threads(M)) void longconv_dk_finish_kernel(const float4* __restrict__ part,
                                                                            float* __restrict__ dk, int G, int d, int L)
{
    constexpr int T = conv_threads(M);
    __shared__ __attribute__((aligned(16))) unsigned char lds[ConvLds<M>::BYTES];
    cplx* a = reinterpret_cast<cplx*>(lds);
    cplx* lo = a + ConvLds<M>::DATA;
    cplx* hi = lo + 128;
    const int tid = threadIdx.x;
    const int c = blockIdx.x;
    build_tables<M, T>(lo, hi, tid);
    PairTwiddle<M, T> pw(tid);
    for (int l = tid; l <= M / 2; l += T) {
        const int kk = pair_bin<M>(l);
        const int p1 = conv_pad(spectrum_pos<M>(kk)), p2 = conv_pad(spectrum_pos<M>((M - kk) & (M - 1)));
        const cplx w = pw.next(l);
        float4 t = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int g = 0; g < G; ++g) {      // fixed order: deterministic
            const float4 o = part[((long)g * d + c) * (M / 2 + 1) + l];
            t.x += o.x; t.y += o.y; t.z += o.z; t.w += o.w;
        }
        const cplx sk = mk(t.x, t.y), smk = mk(t.z, t.w);
        if (kk == 0) {
            a[p1] = mk(0.5f * (sk.x + smk.x), 0.5f * (sk.x - smk.x));
        } else {
            cplx Zk, Zmk;
            tangle(sk, smk, w, Zk, Zmk);
            a[p1] = Zk;
            if (p2 != p1) a[p2] = Zmk;
        }
    }
    __syncthreads();
    fft_passes<M, T, true>(a, lo, hi, tid);
    __syncthreads();
    float* out = dk + (long)c * L;
    const float scale = 1.0f / (float)M;
    for (int n = tid; n < M; n += T) {
        const int t = 2 * n;
        if (t < L) {
            const cplx v = a[conv_pad(n)];
            out[t] = v.x * scale;
            if (t + 1 < L) out[t + 1] = v.y * scale;
        }
    }
}

template <typename IO, typename DVT>
static hipError_t conv_longbwd_dispatch(const IO* X, const float* w, int m, const float4* Kf, const IO* dZ, DVT* dV,
                                        float* dk, float4* acc_ws, int B, int d, int L, hipStream_t st)
{
    const int M = conv_fft_size(L), G = conv_bwd_groups(B, d, L);
    ProfScope prof(KID_CONV_LONG_BWD, st);
    if (const int nb = conv_blocks(L)) {
        // dV block by block (correlation with the kernel's blocks), then the sums of the kernel gradient per block
        // distance and their way back
        hipError_t e = conv_blocked_launch<IO, DVT, true>(dZ, nullptr, 0, Kf, dV, (long)B * d, d, L, st);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((longconv_dk_blocked_kernel<IO>), dim3(d, nb), dim3(kBlkT), 0, st, X, w, m, dZ,
                           acc_ws, B, d, L, nb);
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(longconv_dk_blocked_finish_kernel, dim3(d, nb), dim3(kBlkT), 0, st, acc_ws, dk, d,
                           L, nb);
        return hipGetLastError();
    }
    const dim3 grid(d, G);
#define CHELA_LONGBWD(M_)                                                                                               \
    case M_:                                                                                                            \
        if (G > 1) {                                                                                                    \
            hipLaunchKernelGGL((longconv_bwd_kernel<M_, IO, DVT, true>), grid, dim3(conv_threads(M_)), 0, st, X, w, m, Kf, \
                               dZ, dV, dk, acc_ws, B, d, L);                                                            \
            hipLaunchKernelGGL((longconv_dk_finish_kernel<M_>), dim3(d), dim3(conv_threads(M_)), 0, st, acc_ws, dk, G, d, L); \
        } else                                                                                                          \
            hipLaunchKernelGGL((longconv_bwd_kernel<M_, IO, DVT, false>), grid, dim3(conv_threads(M_)), 0, st, X, w, m, Kf, \
                               dZ, dV, dk, acc_ws, B, d, L);                                                            \
        break;
    switch (M) {
        CHELA_LONGBWD(256) CHELA_LONGBWD(1024) CHELA_LONGBWD(4096) CHELA_LONGBWD(16384)
        default: return hipErrorInvalidValue;
    }
#undef CHELA_LONGBWD
    return hipGetLastError();
}

// ws: the running sums of the long-kernel gradient (largest transform size only), then, with a short kernel,
// B*d*L floats (dV) and the workgroups' tap sums.
template <typename IO>
static hipError_t conv_bwd_impl(const IO* X, const float* w_short, int m, const float4* Kf, const IO* dZ, IO* dX,
                                float* dw, float* dk, float* ws, int B, int d, int L, hipStream_t st)
{
    hipError_t e;
    const long BD = (long)B * d;
    float4* acc_ws = reinterpret_cast<float4*>(ws);
    ws += conv_bwd_acc_floats(B, d, L, sizeof(IO) == 2);
    // bf16 I/O at the lengths the matrix-core kernels serve: its own copy of the spectrum lies behind the pairs
    const bool mx = sizeof(IO) == 2 && convmx_applies(L, 0);
    const void* mx_spec = (const char*)Kf + conv_pairs_bytes(d, L);
    if (w_short == nullptr) { // no short stage: v = x and dX is the correlation of dZ with the long kernel itself
        if (mx) return launch_convmx_longbwd(X, nullptr, 0, mx_spec, dZ, dX, false, dk, (float*)acc_ws, B, d, L, st);
        return conv_longbwd_dispatch<IO, IO>(X, nullptr, 0, Kf, dZ, dX, dk, acc_ws, B, d, L, st);
    }
    float* ws_dV = ws;
    const long n_items = (long)B * ((L + kShortTile - 1) / kShortTile);                     // (batch entry, tile) pairs
    const int n_share = (int)((n_items + kShortTilesPerWg - 1) / kShortTilesPerWg);         // workgroups per channel
    if ((long)d * n_share > 0x7fffffffL) return hipErrorInvalidValue;
    float* ws_part = ws + (size_t)BD * L;                                   // [d][n_share][32] (room for [d][B * tiles][32])
    e = mx ? launch_convmx_longbwd(X, w_short, m, mx_spec, dZ, ws_dV, true, dk, (float*)acc_ws, B, d, L, st)
           : conv_longbwd_dispatch<IO, float>(X, w_short, m, Kf, dZ, ws_dV, dk, acc_ws, B, d, L, st);
    if (e != hipSuccess) return e;
    {
        ProfScope prof(KID_CONV_SHORT_BWD, st);
        const dim3 grid((unsigned)((long)d * n_share));
        // one instantiation per tap count: the tap loops are a third of this kernel's instructions
#define CHELA_SHORT_BWD(T_)                                                                                             \
    case T_:                                                                                                            \
        hipLaunchKernelGGL((shortconv_bwd_kernel<IO, T_>), grid, dim3(256), 0, st, X, w_short, m, ws_dV, dX, ws_part, B, d,  \
                           L, n_share);                                                                                 \
        break;
        switch (m) {
            CHELA_SHORT_BWD(1) CHELA_SHORT_BWD(2) CHELA_SHORT_BWD(3) CHELA_SHORT_BWD(4) CHELA_SHORT_BWD(5) CHELA_SHORT_BWD(6)
            CHELA_SHORT_BWD(7) CHELA_SHORT_BWD(8) CHELA_SHORT_BWD(9) CHELA_SHORT_BWD(10) CHELA_SHORT_BWD(11)
            CHELA_SHORT_BWD(12) CHELA_SHORT_BWD(13) CHELA_SHORT_BWD(14) CHELA_SHORT_BWD(15) CHELA_SHORT_BWD(16)
            default:
                if (m < 17 || m > kShortMaxTaps) return hipErrorInvalidValue;
                hipLaunchKernelGGL((shortconv_bwd_kernel<IO, 32>), grid, dim3(256), 0, st, X, w_short, m, ws_dV, dX, ws_part,
                                   B, d, L, n_share);
        }
#undef CHELA_SHORT_BWD
        if ((e = hipGetLastError()) != hipSuccess) return e;
        hipLaunchKernelGGL(shortconv_dw_kernel, dim3(d), dim3(64), 0, st, ws_part, dw, m, n_share);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    return hipSuccess;
}

// Backward of Z = K_l(silu(K_s X)): dX (I/O dtype), dw [d][m] (with a short kernel, m <= 32), dk [d][L] fp32.
hipError_t launch_shortlong_conv_bwd(const void* X, const float* w_short, int m, const void* Kf, const void* dZ,
                                     void* dX, float* dw, float* dk, float* ws, int B, int d, int L, int dtype,
                                     hipStream_t st)
{
    const float4* K = (const float4*)Kf;
    if (dtype == 0)
        return conv_bwd_impl<bf16>((const bf16*)X, w_short, m, K, (const bf16*)dZ, (bf16*)dX, dw, dk, ws, B, d, L, st);
    return conv_bwd_impl<float>((const float*)X, w_short, m, K, (const float*)dZ, (float*)dX, dw, dk, ws, B, d, L, st);
}

}  // namespace chela
