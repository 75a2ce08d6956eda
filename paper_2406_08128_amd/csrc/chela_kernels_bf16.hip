// bf16 kernels for gfx950: causal linear attention, forward and backward, on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation), tiles staged in LDS, 64-wide wavefronts.
//
// Structure (Sec. 4.1): a (b,h) sequence is cut into segments of a few hundred to a few thousand tokens.
//   pass 1  seg_state   : per segment, the total of X^T Y over its tokens (K^T V for the forward state)
//   pass 2  scan_states : prefix (or suffix) over the segments of one (b,h)                 [fp32 file]
//   pass 3  sweep       : one workgroup per segment walks its chunks with the state in accumulator registers:
//                         masked left product inside the chunk, right product with the carried state, both summed
//                         in registers before the result is written to HBM.
//
// Operand plumbing.  D = A B on a 32x32x16 MFMA wants, per lane, 8 consecutive k of one row of A and 8
// consecutive k of one column of B.  Products that contract over the feature axis read row-major tiles
// directly (ld_nat).  Products that contract over the token axis read the same row-major tiles through the
// LDS transposing read ds_read_b64_tr_b16 (ld_tr), so no transposed copy is ever written.  A score tile
// leaves the MFMA with 4 consecutive rows per lane; it is fed back as an A operand as it is, which permutes k
// inside each 16-wide step, and the partner operand is fetched with the same permutation (ld_tr_perm).
#include "chela_internal.h"

namespace chela {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

constexpr int PAD = 8;   // bf16 elements of padding per LDS row (16 bytes): keeps 16-byte row reads conflict-free

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16()
{
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// Row-major tile X[row][k]: lane (r = lane%32, h = lane/32) gets X[row0 + r][k0 + 8h .. +7].
__device__ __forceinline__ bf16x8 ld_nat(const bf16* X, int ld, int row0, int k0, int lane)
{
    return *reinterpret_cast<const bf16x8*>(X + (row0 + (lane & 31)) * ld + k0 + 8 * (lane >> 5));
}

__device__ __forceinline__ bf16x4 ds_tr(const bf16* p)
{
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_bf16x4*)p);
}

__device__ __forceinline__ bf16x8 cat(bf16x4 lo, bf16x4 hi)
{
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// Row-major tile T[k][m] read as the operand whose contraction index is the ROW: lane (r, h) gets
// T[k0 + 8h + e][m0 + r], e = 0..7.  Within a group of 16 lanes the transposing read hands lane p the
// column m0' + p of a 4 x 16 block whose rows the lanes address as (p / 4) and 8-byte pieces as (p % 4).
__device__ __forceinline__ bf16x8 ld_tr(const bf16* T, int ld, int k0, int m0, int lane)
{
    const int p = lane & 15, g = (lane >> 4) & 1, h = lane >> 5;
    const bf16* a = T + (k0 + 8 * h + (p >> 2)) * ld + m0 + 16 * g + 4 * (p & 3);
    return cat(ds_tr(a), ds_tr(a + 4 * ld));
}

// Same, with the k order of an accumulator tile re-used as A operand: slot e of lane (r, h) is
// row k0 + 8*(e/4) + 4h + (e%4).
__device__ __forceinline__ bf16x8 ld_tr_perm(const bf16* T, int ld, int k0, int m0, int lane)
{
    const int p = lane & 15, g = (lane >> 4) & 1, h = lane >> 5;
    const bf16* a = T + (k0 + 4 * h + (p >> 2)) * ld + m0 + 16 * g + 4 * (p & 3);
    return cat(ds_tr(a), ds_tr(a + 8 * ld));
}

// Accumulator registers [base, base+8) rounded to bf16 (round-to-nearest-even): one 16-wide k step of an A operand.
__device__ __forceinline__ bf16x8 cvt8(const f32x16& p, int base)
{
    bf16x8 r;
#pragma unroll
    for (int e = 0; e < 8; ++e) r[e] = (bf16)p[base + e];
    return r;
}

__device__ __forceinline__ bf16x8 negate(bf16x8 v)
{
    typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
    u32x4 u = __builtin_bit_cast(u32x4, v);
    u ^= 0x80008000u;
    return __builtin_bit_cast(bf16x8, u);
}

// Accumulator tile D[row][col]: register 4a+b of lane (r, h) is D[8a + 4h + b][r].
// Zero the strictly-upper part (row-index-in-tile > col-index-in-tile is kept or dropped by `keep_lower`):
//   rows_are_keys = true : tile is P^T[s][t], keep s <= t  -> zero where row > col
//   rows_are_keys = false: tile is P[t][s],   keep s <= t  -> zero where col > row
template <bool ROWS_ARE_KEYS>
__device__ __forceinline__ void mask_diag(f32x16& p, int lane)
{
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int row = 8 * a + 4 * h + b;
            const bool drop = ROWS_ARE_KEYS ? (row > r) : (r > row);
            if (drop) p[4 * a + b] = 0.f;
        }
}

__device__ __forceinline__ int phys_row(int p, int N, bool rev) { return rev ? (N - 1 - p) : p; }

// A C x D bf16 tile travels HBM -> registers (16-byte vectors, NV per thread) -> LDS (row stride D + PAD).
template <int C, int D>
struct TileRegs {
    static constexpr int VPR = D / 8;              // 16-byte vectors per row
    static constexpr int NV = C * D / 8 / 256;     // vectors per thread
    uint4 v[NV];
    __device__ __forceinline__ void load(const bf16* base, int c0, int p_end, int N, bool rev, int tid)
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / VPR, cv = x % VPR, p = c0 + row;
            if (p < p_end)
                v[n] = *reinterpret_cast<const uint4*>(base + (size_t)phys_row(p, N, rev) * D + cv * 8);
            else
                v[n] = make_uint4(0, 0, 0, 0);
        }
    }
    __device__ __forceinline__ void store(bf16* lds, int tid) const
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / VPR, cv = x % VPR;
            *reinterpret_cast<uint4*>(lds + row * (D + PAD) + cv * 8) = v[n];
        }
    }
};

// Store a 32x32 accumulator tile D[row][col] as bf16 into a row-major global matrix (leading dim ld);
// tile rows are logical positions p = prow0 + 8a+4h+b, stored only when p < p_end.
__device__ __forceinline__ void store_tile(bf16* G, int ld, int prow0, int col0, const f32x16& acc, int p_end, int N,
                                           bool rev, int lane)
{
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int p = prow0 + 8 * a + 4 * h + b;
            if (p < p_end) G[(size_t)phys_row(p, N, rev) * ld + col0 + r] = (bf16)acc[4 * a + b];
        }
}

// =============================================================================================== pass 1
// out[a][b] = sum over the segment's tokens s of X[s][a] * Y[s][b]   (fp32, [DA][DB] row-major).
// Two (X, Y) pairs can be served by one launch (blockIdx.z); `skip_seg[z]` names a segment whose total the
// following scan never uses (-1: none).
struct SegStateArgs {
    const bf16* X[2];
    const bf16* Y[2];
    float* out[2];
    int skip_seg[2];
};

template <int DA, int DB>
__global__ __launch_bounds__(256) void bf16_seg_state_kernel(SegStateArgs args, int N, int seg_len, int n_seg, int rev)
{
    constexpr int R = 64;
    __shared__ __attribute__((aligned(16))) bf16 sX[R * (DA + PAD)];
    __shared__ __attribute__((aligned(16))) bf16 sY[R * (DB + PAD)];
    const int z = blockIdx.z;
    const int seg = blockIdx.x;
    const long bh = blockIdx.y;
    if (seg == args.skip_seg[z]) return;
    const bf16* X = args.X[z] + (size_t)bh * N * DA;
    const bf16* Y = args.Y[z] + (size_t)bh * N * DB;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    constexpr int AB = DA / 32, BB = DB / 32, NT = AB * BB / 4;
    f32x16 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = zero16();
    TileRegs<R, DA> rx;
    TileRegs<R, DB> ry;
    rx.load(X, p0, p1, N, rev, tid);
    ry.load(Y, p0, p1, N, rev, tid);
    for (int c0 = p0; c0 < p1; c0 += R) {
        rx.store(sX, tid);
        ry.store(sY, tid);
        __syncthreads();
        if (c0 + R < p1) {
            rx.load(X, c0 + R, p1, N, rev, tid);
            ry.load(Y, c0 + R, p1, N, rev, tid);
        }
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
            for (int s0 = 0; s0 < R; s0 += 16)
                acc[n] = mfma(ld_tr(sX, DA + PAD, s0, ab * 32, lane), ld_tr(sY, DB + PAD, s0, bb * 32, lane), acc[n]);
        }
        __syncthreads();
    }
    float* o = args.out[z] + ((size_t)bh * n_seg + seg) * DA * DB;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                o[(ab * 32 + 8 * a + 4 * h + b) * DB + bb * 32 + r] = acc[n][4 * a + b];
    }
}

// Load / keep a [DA][DB] fp32 state as accumulator tiles: tile id = w + 4n -> (ab, bb) = (id / BB, id % BB).
template <int DA, int DB>
__device__ __forceinline__ void load_state(f32x16* acc, const float* src, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                acc[n][4 * a + b] = src ? src[(ab * 32 + 8 * a + 4 * h + b) * DB + bb * 32 + r] : 0.f;
    }
}

// Write a [DA][DB] state held as accumulator tiles into LDS as bf16, TRANSPOSED: dst[b][a] (row stride DA + PAD).
// A lane owns 4 consecutive a for one b, i.e. 8 contiguous bytes of dst.
template <int DA, int DB>
__device__ __forceinline__ void state_to_lds_T(bf16* dst, const f32x16* acc, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            bf16x4 v;
#pragma unroll
            for (int b = 0; b < 4; ++b) v[b] = (bf16)acc[n][4 * a + b];
            *reinterpret_cast<bf16x4*>(dst + (bb * 32 + r) * (DA + PAD) + ab * 32 + 8 * a + 4 * h) = v;
        }
    }
}

// =============================================================================================== forward sweep
// One workgroup (4 waves) per (segment, bh).  Per chunk of C tokens:
//   P^T = K Q^T (masked), O = P V + Q S_prev, store O, S += K^T V.
// Wave w owns output rows [32*tb, 32*tb+32) with tb = w % WT and NJ column tiles; it recomputes the score
// tiles of its row block itself (matrix-core time is cheap here, LDS round trips and barriers are not).
template <int C, int DK, int DV, bool REV>
__global__ __launch_bounds__(256) void bf16_fwd_sweep_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                            const bf16* __restrict__ V, bf16* __restrict__ O,
                                                            const float* __restrict__ S0, int N, int seg_len, int n_seg)
{
    constexpr int LDK = DK + PAD, LDV = DV + PAD;
    constexpr int TB = C / 32, JB = DV / 32, IB = DK / 32;
    constexpr int WT = TB < 4 ? TB : 4, WJ = 4 / WT, NJ = JB / WJ;
    constexpr int NS = IB * JB / 4;
    static_assert(TB <= 4 && JB % WJ == 0, "unsupported tile shape");
    __shared__ __attribute__((aligned(16))) bf16 sQ[C * LDK];
    __shared__ __attribute__((aligned(16))) bf16 sK[C * LDK];
    __shared__ __attribute__((aligned(16))) bf16 sV[C * LDV];
    __shared__ __attribute__((aligned(16))) bf16 sST[DV * LDK];   // S^T as bf16: [j][i]

    const int seg = blockIdx.x;
    const long bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int tb = w % WT, jg = w / WT;
    const bf16* Qb = Q + (size_t)bh * N * DK;
    const bf16* Kb = K + (size_t)bh * N * DK;
    const bf16* Vb = V + (size_t)bh * N * DV;
    bf16* Ob = O + (size_t)bh * N * DV;
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);

    f32x16 accS[NS];
    load_state<DK, DV>(accS, (S0 != nullptr && seg > 0) ? S0 + ((size_t)bh * n_seg + seg) * DK * DV : nullptr, w, lane);

    TileRegs<C, DK> rq, rk;
    TileRegs<C, DV> rv;
    rq.load(Qb, p0, p1, N, REV, tid);
    rk.load(Kb, p0, p1, N, REV, tid);
    rv.load(Vb, p0, p1, N, REV, tid);

    for (int c0 = p0; c0 < p1; c0 += C) {
        rq.store(sQ, tid);
        rk.store(sK, tid);
        rv.store(sV, tid);
        state_to_lds_T<DK, DV>(sST, accS, w, lane);
        __syncthreads();
        const bool more = c0 + C < p1;
        if (more) {
            rq.load(Qb, c0 + C, p1, N, REV, tid);
            rk.load(Kb, c0 + C, p1, N, REV, tid);
            rv.load(Vb, c0 + C, p1, N, REV, tid);
        }
        bf16x8 aQ[DK / 16];
#pragma unroll
        for (int kk = 0; kk < DK / 16; ++kk) aQ[kk] = ld_nat(sQ, LDK, tb * 32, kk * 16, lane);
        f32x16 accO[NJ];
#pragma unroll
        for (int n = 0; n < NJ; ++n) accO[n] = zero16();
        // inter-chunk part: Q S_prev
#pragma unroll
        for (int n = 0; n < NJ; ++n)
#pragma unroll
            for (int kk = 0; kk < DK / 16; ++kk)
                accO[n] = mfma(aQ[kk], ld_nat(sST, LDK, (jg * NJ + n) * 32, kk * 16, lane), accO[n]);
        // intra-chunk part: masked (Q K^T) V, key blocks sb <= tb
#pragma unroll
        for (int sb = 0; sb < TB; ++sb) {
            if (sb <= tb) {
                f32x16 pT = zero16();
#pragma unroll
                for (int kk = 0; kk < DK / 16; ++kk) pT = mfma(ld_nat(sK, LDK, sb * 32, kk * 16, lane), aQ[kk], pT);
                if (sb == tb) mask_diag<true>(pT, lane);
                const bf16x8 pa0 = cvt8(pT, 0), pa1 = cvt8(pT, 8);
#pragma unroll
                for (int n = 0; n < NJ; ++n) {
                    accO[n] = mfma(pa0, ld_tr_perm(sV, LDV, sb * 32, (jg * NJ + n) * 32, lane), accO[n]);
                    accO[n] = mfma(pa1, ld_tr_perm(sV, LDV, sb * 32 + 16, (jg * NJ + n) * 32, lane), accO[n]);
                }
            }
        }
#pragma unroll
        for (int n = 0; n < NJ; ++n) store_tile(Ob, DV, c0 + tb * 32, (jg * NJ + n) * 32, accO[n], p1, N, REV, lane);
        // state update S += K^T V (not needed after the segment's last chunk)
        if (more) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, ib = id / JB, jb = id % JB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accS[n] = mfma(ld_tr(sK, LDK, s0, ib * 32, lane), ld_tr(sV, LDV, s0, jb * 32, lane), accS[n]);
            }
        }
        __syncthreads();
    }
}

// =============================================================================================== backward sweep
// One workgroup per (segment, bh), walking the chunks from the LAST to the first, so that each input tile is
// read once for all three gradients.  Two states live in accumulator registers, both stored transposed
// ([dv][dk], lane = one feature i, 4 consecutive j):
//   S^T : sum of V^T K over tokens before the current chunk.  It enters as the inclusive prefix at the end of
//         the segment and is rolled BACK by one chunk per step (S_{c-1} = S_c - V_c^T K_c, fp32).
//   R^T : sum of dO^T Q over tokens after the current chunk; it grows by one chunk per step.
// Per chunk:  dQ = dP K + dO S^T',  dK = dP^T Q + V R^T',  dV = P^T dO + K R,
//             P = (Q K^T) o M,  dP = (dO V^T) o M.
template <int C, int DK, int DV>
__global__ __launch_bounds__(256) void bf16_bwd_sweep_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                            const bf16* __restrict__ V, const bf16* __restrict__ dO,
                                                            bf16* __restrict__ dQ, bf16* __restrict__ dK,
                                                            bf16* __restrict__ dV, const float* __restrict__ Send,
                                                            const float* __restrict__ Rnext, int N, int seg_len,
                                                            int n_seg)
{
    constexpr int LDK = DK + PAD, LDV = DV + PAD;
    constexpr int TB = C / 32, JB = DV / 32, IB = DK / 32;
    constexpr int WT = TB < 4 ? TB : 4, WJ = 4 / WT, NJ = JB / WJ, NI = IB / WJ;
    constexpr int NS = IB * JB / 4;
    static_assert(TB <= 4 && JB % WJ == 0 && IB % WJ == 0, "unsupported tile shape");
    __shared__ __attribute__((aligned(16))) bf16 sQ[C * LDK];
    __shared__ __attribute__((aligned(16))) bf16 sK[C * LDK];
    __shared__ __attribute__((aligned(16))) bf16 sV[C * LDV];
    __shared__ __attribute__((aligned(16))) bf16 sG[C * LDV];     // dO
    __shared__ __attribute__((aligned(16))) bf16 sS[DK * LDV];    // S  [i][j] bf16
    __shared__ __attribute__((aligned(16))) bf16 sR[DK * LDV];    // R  [i][j] bf16

    const int seg = blockIdx.x;
    const long bh = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int rb = w % WT, cg = w / WT;
    const bf16* Qb = Q + (size_t)bh * N * DK;
    const bf16* Kb = K + (size_t)bh * N * DK;
    const bf16* Vb = V + (size_t)bh * N * DV;
    const bf16* Gb = dO + (size_t)bh * N * DV;
    bf16* dQb = dQ + (size_t)bh * N * DK;
    bf16* dKb = dK + (size_t)bh * N * DK;
    bf16* dVb = dV + (size_t)bh * N * DV;
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    const int n_ch = (p1 - p0 + C - 1) / C;

    // states, transposed: [DV][DK]
    f32x16 accST[NS], accRT[NS];
    const size_t soff = ((size_t)bh * n_seg + seg) * DK * DV;
    load_state<DV, DK>(accST, Send ? Send + soff : nullptr, w, lane);
    load_state<DV, DK>(accRT, (Rnext != nullptr && seg < n_seg - 1) ? Rnext + soff : nullptr, w, lane);
    const bool single = (Send == nullptr);   // one segment: S is built below instead of being read

    TileRegs<C, DK> rq, rk;
    TileRegs<C, DV> rv, rg;

    if (single) {
        // whole sequence in this workgroup: accumulate S^T = sum V^T K over all chunks first
        for (int ci = 0; ci < n_ch; ++ci) {
            const int c0 = p0 + ci * C;
            rk.load(Kb, c0, p1, N, false, tid);
            rv.load(Vb, c0, p1, N, false, tid);
            __syncthreads();
            rk.store(sK, tid);
            rv.store(sV, tid);
            __syncthreads();
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accST[n] = mfma(ld_tr(sV, LDV, s0, jb * 32, lane), ld_tr(sK, LDK, s0, ib * 32, lane), accST[n]);
            }
        }
        __syncthreads();
    }

    {
        const int c0 = p0 + (n_ch - 1) * C;
        rq.load(Qb, c0, p1, N, false, tid);
        rk.load(Kb, c0, p1, N, false, tid);
        rv.load(Vb, c0, p1, N, false, tid);
        rg.load(Gb, c0, p1, N, false, tid);
    }

    for (int ci = n_ch - 1; ci >= 0; --ci) {
        const int c0 = p0 + ci * C;
        rq.store(sQ, tid);
        rk.store(sK, tid);
        rv.store(sV, tid);
        rg.store(sG, tid);
        // R (state after this chunk) is already final: publish it as bf16 [i][j]
        state_to_lds_T<DV, DK>(sR, accRT, w, lane);
        __syncthreads();
        if (ci > 0) {
            rq.load(Qb, c0 - C, p1, N, false, tid);
            rk.load(Kb, c0 - C, p1, N, false, tid);
            rv.load(Vb, c0 - C, p1, N, false, tid);
            rg.load(Gb, c0 - C, p1, N, false, tid);
        }
        // roll S back over this chunk: S^T -= V^T K, then publish S (state before this chunk)
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
            for (int s0 = 0; s0 < C; s0 += 16)
                accST[n] = mfma(negate(ld_tr(sV, LDV, s0, jb * 32, lane)), ld_tr(sK, LDK, s0, ib * 32, lane), accST[n]);
        }
        state_to_lds_T<DV, DK>(sS, accST, w, lane);
        __syncthreads();

        // ---------------- dQ rows of block tb = rb:  dQ = dP K + dO S^T'
        {
            bf16x8 aG[DV / 16];
#pragma unroll
            for (int kk = 0; kk < DV / 16; ++kk) aG[kk] = ld_nat(sG, LDV, rb * 32, kk * 16, lane);
            f32x16 acc[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) acc[n] = zero16();
#pragma unroll
            for (int n = 0; n < NI; ++n)
#pragma unroll
                for (int kk = 0; kk < DV / 16; ++kk)
                    acc[n] = mfma(aG[kk], ld_nat(sS, LDV, (cg * NI + n) * 32, kk * 16, lane), acc[n]);
#pragma unroll
            for (int sb = 0; sb < TB; ++sb) {
                if (sb <= rb) {
                    f32x16 t = zero16();   // dP^T[s][t] = v_s . dO_t
#pragma unroll
                    for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sV, LDV, sb * 32, kk * 16, lane), aG[kk], t);
                    if (sb == rb) mask_diag<true>(t, lane);
                    const bf16x8 a0 = cvt8(t, 0), a1 = cvt8(t, 8);
#pragma unroll
                    for (int n = 0; n < NI; ++n) {
                        acc[n] = mfma(a0, ld_tr_perm(sK, LDK, sb * 32, (cg * NI + n) * 32, lane), acc[n]);
                        acc[n] = mfma(a1, ld_tr_perm(sK, LDK, sb * 32 + 16, (cg * NI + n) * 32, lane), acc[n]);
                    }
                }
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) store_tile(dQb, DK, c0 + rb * 32, (cg * NI + n) * 32, acc[n], p1, N, false, lane);
        }
        // ---------------- dK rows of key block sb = rb:  dK = dP^T Q + V R^T'
        {
            bf16x8 bV[DV / 16];
#pragma unroll
            for (int kk = 0; kk < DV / 16; ++kk) bV[kk] = ld_nat(sV, LDV, rb * 32, kk * 16, lane);
            f32x16 acc[NI];
#pragma unroll
            for (int n = 0; n < NI; ++n) acc[n] = zero16();
#pragma unroll
            for (int n = 0; n < NI; ++n)
#pragma unroll
                for (int kk = 0; kk < DV / 16; ++kk)
                    acc[n] = mfma(bV[kk], ld_nat(sR, LDV, (cg * NI + n) * 32, kk * 16, lane), acc[n]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb >= rb) {
                    f32x16 t = zero16();   // dP[t][s] = dO_t . v_s
#pragma unroll
                    for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sG, LDV, tb * 32, kk * 16, lane), bV[kk], t);
                    if (tb == rb) mask_diag<false>(t, lane);
                    const bf16x8 a0 = cvt8(t, 0), a1 = cvt8(t, 8);
#pragma unroll
                    for (int n = 0; n < NI; ++n) {
                        acc[n] = mfma(a0, ld_tr_perm(sQ, LDK, tb * 32, (cg * NI + n) * 32, lane), acc[n]);
                        acc[n] = mfma(a1, ld_tr_perm(sQ, LDK, tb * 32 + 16, (cg * NI + n) * 32, lane), acc[n]);
                    }
                }
            }
#pragma unroll
            for (int n = 0; n < NI; ++n) store_tile(dKb, DK, c0 + rb * 32, (cg * NI + n) * 32, acc[n], p1, N, false, lane);
        }
        // ---------------- dV rows of key block sb = rb:  dV = P^T dO + K R
        {
            bf16x8 bK[DK / 16];
#pragma unroll
            for (int kk = 0; kk < DK / 16; ++kk) bK[kk] = ld_nat(sK, LDK, rb * 32, kk * 16, lane);
            f32x16 acc[NJ];
#pragma unroll
            for (int n = 0; n < NJ; ++n) acc[n] = zero16();
#pragma unroll
            for (int n = 0; n < NJ; ++n)
#pragma unroll
                for (int kk = 0; kk < DK / 16; ++kk)
                    acc[n] = mfma(bK[kk], ld_tr(sR, LDV, kk * 16, (cg * NJ + n) * 32, lane), acc[n]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb >= rb) {
                    f32x16 t = zero16();   // P[t][s] = q_t . k_s
#pragma unroll
                    for (int kk = 0; kk < DK / 16; ++kk) t = mfma(ld_nat(sQ, LDK, tb * 32, kk * 16, lane), bK[kk], t);
                    if (tb == rb) mask_diag<false>(t, lane);
                    const bf16x8 a0 = cvt8(t, 0), a1 = cvt8(t, 8);
#pragma unroll
                    for (int n = 0; n < NJ; ++n) {
                        acc[n] = mfma(a0, ld_tr_perm(sG, LDV, tb * 32, (cg * NJ + n) * 32, lane), acc[n]);
                        acc[n] = mfma(a1, ld_tr_perm(sG, LDV, tb * 32 + 16, (cg * NJ + n) * 32, lane), acc[n]);
                    }
                }
            }
#pragma unroll
            for (int n = 0; n < NJ; ++n) store_tile(dVb, DV, c0 + rb * 32, (cg * NJ + n) * 32, acc[n], p1, N, false, lane);
        }
        // ---------------- R^T += dO^T Q (not needed after the segment's first chunk)
        if (ci > 0) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accRT[n] = mfma(ld_tr(sG, LDV, s0, jb * 32, lane), ld_tr(sQ, LDK, s0, ib * 32, lane), accRT[n]);
            }
        }
        __syncthreads();
    }
}

// =============================================================================================== launchers
template <int DA, int DB>
static hipError_t run_seg_state(const SegStateArgs& a, int npairs, long BH, int N, const Plan& plan, bool rev,
                                hipStream_t st)
{
    dim3 grid(plan.n_seg, (unsigned)BH, npairs);
    ProfScope prof(KID_SEG_STATE_BF16, st);
    hipLaunchKernelGGL((bf16_seg_state_kernel<DA, DB>), grid, dim3(256), 0, st, a, N, plan.seg_len, plan.n_seg, (int)rev);
    return hipGetLastError();
}

template <int C, int DK, int DV>
static hipError_t fwd_impl(const bf16* Q, const bf16* K, const bf16* V, bf16* O, long BH, int N, const Plan& plan,
                           bool rev, float* ws, hipStream_t st)
{
    hipError_t e;
    if (plan.n_seg > 1) {
        SegStateArgs a{};
        a.X[0] = K; a.Y[0] = V; a.out[0] = ws; a.skip_seg[0] = plan.n_seg - 1;
        if ((e = run_seg_state<DK, DV>(a, 1, BH, N, plan, rev, st)) != hipSuccess) return e;
        if ((e = scan_states(ws, BH, plan.n_seg, DK * DV, SCAN_EXCL_PREFIX, st)) != hipSuccess) return e;
    }
    dim3 grid(plan.n_seg, (unsigned)BH);
    const float* s0 = plan.n_seg > 1 ? ws : nullptr;
    ProfScope prof(KID_FWD_SWEEP_BF16, st);
    if (rev)
        hipLaunchKernelGGL((bf16_fwd_sweep_kernel<C, DK, DV, true>), grid, dim3(256), 0, st, Q, K, V, O, s0, N,
                           plan.seg_len, plan.n_seg);
    else
        hipLaunchKernelGGL((bf16_fwd_sweep_kernel<C, DK, DV, false>), grid, dim3(256), 0, st, Q, K, V, O, s0, N,
                           plan.seg_len, plan.n_seg);
    return hipGetLastError();
}

template <int C, int DK, int DV>
static hipError_t bwd_impl(const bf16* Q, const bf16* K, const bf16* V, const bf16* dO, bf16* dQ, bf16* dK, bf16* dV,
                           long BH, int N, const Plan& plan, float* ws, hipStream_t st)
{
    hipError_t e;
    float* wsS = ws;
    float* wsR = ws ? ws + (size_t)BH * plan.n_seg * DK * DV : nullptr;
    if (plan.n_seg > 1) {
        SegStateArgs a{};
        a.X[0] = V;  a.Y[0] = K; a.out[0] = wsS; a.skip_seg[0] = -1;   // S^T totals: every segment is needed
        a.X[1] = dO; a.Y[1] = Q; a.out[1] = wsR; a.skip_seg[1] = 0;    // R^T totals: the first is never used
        if ((e = run_seg_state<DV, DK>(a, 2, BH, N, plan, false, st)) != hipSuccess) return e;
        if ((e = scan_states(wsS, BH, plan.n_seg, DK * DV, SCAN_INCL_PREFIX, st)) != hipSuccess) return e;
        if ((e = scan_states(wsR, BH, plan.n_seg, DK * DV, SCAN_EXCL_SUFFIX, st)) != hipSuccess) return e;
    }
    dim3 grid(plan.n_seg, (unsigned)BH);
    ProfScope prof(KID_BWD_SWEEP_BF16, st);
    hipLaunchKernelGGL((bf16_bwd_sweep_kernel<C, DK, DV>), grid, dim3(256), 0, st, Q, K, V, dO, dQ, dK, dV,
                       plan.n_seg > 1 ? wsS : nullptr, plan.n_seg > 1 ? wsR : nullptr, N, plan.seg_len, plan.n_seg);
    return hipGetLastError();
}

#define CHELA_DISPATCH(C_, DK_, DV_, CALL)                                  \
    if (plan.chunk == C_ && dk == DK_ && dv == DV_) return CALL;

hipError_t launch_bf16_fwd(const void* Q, const void* K, const void* V, void* O, long BH, int N, int dk, int dv,
                           const Plan& plan, bool rev, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V;
    bf16* o = (bf16*)O;
    CHELA_DISPATCH(64, 64, 64, (fwd_impl<64, 64, 64>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(128, 64, 64, (fwd_impl<128, 64, 64>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(64, 64, 128, (fwd_impl<64, 64, 128>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(128, 64, 128, (fwd_impl<128, 64, 128>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(64, 128, 64, (fwd_impl<64, 128, 64>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(128, 128, 64, (fwd_impl<128, 128, 64>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(64, 128, 128, (fwd_impl<64, 128, 128>(q, k, v, o, BH, N, plan, rev, ws, st)))
    CHELA_DISPATCH(128, 128, 128, (fwd_impl<128, 128, 128>(q, k, v, o, BH, N, plan, rev, ws, st)))
    return hipErrorInvalidValue;
}

hipError_t launch_bf16_bwd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK,
                           void* dV, long BH, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)dO;
    bf16 *dq = (bf16*)dQ, *dkk = (bf16*)dK, *dvv = (bf16*)dV;
    CHELA_DISPATCH(64, 64, 64, (bwd_impl<64, 64, 64>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st)))
    CHELA_DISPATCH(128, 64, 64, (bwd_impl<128, 64, 64>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st)))
    CHELA_DISPATCH(64, 64, 128, (bwd_impl<64, 64, 128>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st)))
    CHELA_DISPATCH(64, 128, 64, (bwd_impl<64, 128, 64>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st)))
    CHELA_DISPATCH(64, 128, 128, (bwd_impl<64, 128, 128>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st)))
    return hipErrorInvalidValue;
}

}  // namespace chela
