// bf16 kernels for gfx950: causal linear attention, forward and backward, on the matrix cores
// (v_mfma_f32_32x32x16_bf16, fp32 accumulation), tiles staged in LDS, 64-wide wavefronts.
//
// Structure (Sec. 4.1): a (b,h) sequence is cut into segments of a few hundred to a few thousand tokens.
//   pre-pass : per segment, the total of X^T Y over its tokens (K^T V for the forward state)
//   scan     : prefix (or suffix) over the segments of one (b,h)
//   sweep    : one workgroup per segment walks its chunks with the state in accumulator registers: masked left
//              product inside the chunk, right product with the carried state, both summed in registers before the
//              result is written to HBM.
//
// Operand plumbing.  D = A B on a 32x32x16 MFMA wants, per lane, 8 consecutive k of one row of A and 8
// consecutive k of one column of B.  Products that contract over the feature axis read row-major LDS tiles
// directly (ld_nat).  Products that contract over the token axis read the same row-major tiles through the
// LDS transposing read ds_read_b64_tr_b16 (ld_tr), so no transposed copy is ever written.  A score tile
// leaves the MFMA with 4 consecutive rows per lane; it is fed back as an operand as it is, which permutes k
// inside each 16-wide step, and the partner operand is fetched with the same permutation (ld_tr_perm).
// Every output tile is accumulated TRANSPOSED (features in rows, tokens in columns): a lane then owns 4
// consecutive features of one token, one v_permlane32_swap makes that 8, and the tile leaves as 16-byte stores.
#include "chela_internal.h"

#include <cstdlib>

namespace chela {

typedef __bf16 bf16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;
typedef __attribute__((address_space(3))) bf16x4 lds_bf16x4;

typedef __attribute__((ext_vector_type(4))) unsigned u32x4v;
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

// Same, with the k order of an accumulator tile re-used as an operand: slot e of lane (r, h) is
// row k0 + 8*(e/4) + 4h + (e%4).
__device__ __forceinline__ bf16x8 ld_tr_perm(const bf16* T, int ld, int k0, int m0, int lane)
{
    const int p = lane & 15, g = (lane >> 4) & 1, h = lane >> 5;
    const bf16* a = T + (k0 + 4 * h + (p >> 2)) * ld + m0 + 16 * g + 4 * (p & 3);
    return cat(ds_tr(a), ds_tr(a + 8 * ld));
}

// Two fp32 -> one register of two bf16 (round-to-nearest-even), first argument in the low half.
template <bool NEG = false>
__device__ __forceinline__ unsigned pack2(float lo, float hi)
{
    bf16x2 v;
    v[0] = (bf16)(NEG ? -lo : lo);
    v[1] = (bf16)(NEG ? -hi : hi);
    return __builtin_bit_cast(unsigned, v);
}

// Accumulator tile D[row][col]: register 4a+b of lane (r, h) is D[8a + 4h + b][r].
// Keep-masks for a DIAGONAL 32x32 score tile after packing to bf16 pairs (register 2a+p holds rows 8a+4h+2p, +1):
//   KEYS_IN_ROWS = true : tile is P^T[s][t], keep s <= t, i.e. row <= col
//   KEYS_IN_ROWS = false: tile is P[t][s],   keep s <= t, i.e. col <= row
template <bool KEYS_IN_ROWS>
__device__ __forceinline__ void make_masks(unsigned (&m)[8], int lane)
{
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int a = 0; a < 4; ++a)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
            const int row0 = 8 * a + 4 * h + 2 * p, row1 = row0 + 1;
            const bool k0 = KEYS_IN_ROWS ? (row0 <= r) : (r <= row0);
            const bool k1 = KEYS_IN_ROWS ? (row1 <= r) : (r <= row1);
            m[2 * a + p] = (k0 ? 0x0000ffffu : 0u) | (k1 ? 0xffff0000u : 0u);
        }
}

// A score tile rounded to bf16 as two 16-wide k steps of an MFMA operand (k permuted as ld_tr_perm expects).
__device__ __forceinline__ void cvt_tile(const f32x16& p, bf16x8& a0, bf16x8& a1)
{
    u32x4 lo, hi;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        lo[q] = pack2(p[2 * q], p[2 * q + 1]);
        hi[q] = pack2(p[8 + 2 * q], p[8 + 2 * q + 1]);
    }
    a0 = __builtin_bit_cast(bf16x8, lo);
    a1 = __builtin_bit_cast(bf16x8, hi);
}

__device__ __forceinline__ void cvt_tile_masked(const f32x16& p, const unsigned (&m)[8], bf16x8& a0, bf16x8& a1)
{
    u32x4 lo, hi;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        lo[q] = pack2(p[2 * q], p[2 * q + 1]) & m[q];
        hi[q] = pack2(p[8 + 2 * q], p[8 + 2 * q + 1]) & m[4 + q];
    }
    a0 = __builtin_bit_cast(bf16x8, lo);
    a1 = __builtin_bit_cast(bf16x8, hi);
}

// Eq. 11-12: queries and keys are per-feature affine maps of one tensor Z.  Eight consecutive features of one
// map, kept in registers: apply() turns 8 bf16 z into 8 bf16 (alpha * z + beta).
__device__ __forceinline__ float bf16_lo(unsigned u) { return __builtin_bit_cast(float, u << 16); }
__device__ __forceinline__ float bf16_hi(unsigned u) { return __builtin_bit_cast(float, u & 0xffff0000u); }

struct AffineCols {
    float a[8], b[8];
    __device__ __forceinline__ AffineCols(const float* alpha, const float* beta, int col0)
    {
        const float4 a0 = *reinterpret_cast<const float4*>(alpha + col0), a1 = *reinterpret_cast<const float4*>(alpha + col0 + 4);
        const float4 b0 = *reinterpret_cast<const float4*>(beta + col0), b1 = *reinterpret_cast<const float4*>(beta + col0 + 4);
        a[0] = a0.x; a[1] = a0.y; a[2] = a0.z; a[3] = a0.w; a[4] = a1.x; a[5] = a1.y; a[6] = a1.z; a[7] = a1.w;
        b[0] = b0.x; b[1] = b0.y; b[2] = b0.z; b[3] = b0.w; b[4] = b1.x; b[5] = b1.y; b[6] = b1.z; b[7] = b1.w;
    }
    __device__ __forceinline__ unsigned two(unsigned z, int c) const
    {
        return pack2(fmaf(a[c], bf16_lo(z), b[c]), fmaf(a[c + 1], bf16_hi(z), b[c + 1]));
    }
    __device__ __forceinline__ uint4 apply(uint4 z) const
    {
        return make_uint4(two(z.x, 0), two(z.y, 2), two(z.z, 4), two(z.w, 6));
    }
};

// A C x D bf16 tile (C consecutive rows of a row-major [N][D] matrix, i.e. one contiguous block of memory) travels
// HBM -> registers (16-byte vectors, NV per thread) -> LDS (row stride D + PAD).
// 16-byte global load, optionally with the streaming ("non-temporal") hint.  The hint is for streams that nobody
// reads again soon (the forward sweep's Q, the gate): they then do not push the K and V tiles that the pre-pass
// has just brought into the memory-side cache out before the sweep re-reads them.  Measured: forward sweep 74.0 ->
// 67.5 us on the headline shape.  On streams that ARE re-read (everything the backward touches) the hint only moves
// time from one kernel to the next, and on the 16-byte output stores it triples the time (no write combining).
template <bool NTL>
__device__ __forceinline__ uint4 ldg16(const uint4* p)
{
    if (NTL) {
        const u32x4v t = __builtin_nontemporal_load(reinterpret_cast<const u32x4v*>(p));
        return make_uint4(t[0], t[1], t[2], t[3]);
    }
    return *p;
}

template <int C, int D, bool NTL = false>
struct TileRegs {
    static constexpr int VPR = D / 8;              // 16-byte vectors per row
    static constexpr int NV = C * D / 8 / 256;     // vectors per thread
    uint4 v[NV];
    // `tile` points at the first row; rows >= valid_rows read as zero.
    // `ld` is the distance between rows in elements: D for [B,H,N,d] tensors (the tile is then one contiguous block
    // and the address below folds to 16 * x), H * D for [B,N,H,d] ones.
    // Vector n of thread tid is vector tid + 256 n of the tile.  In the strided case the address is split into a
    // part that is the same for the whole workgroup (tile start + n * (256 / VPR) rows: scalar registers) and one
    // 32-bit per-thread offset shared by all n, instead of one 64-bit address per vector.
    static __device__ __forceinline__ const uint4* at(const bf16* tile, int ld, int tid, int n)
    {
        if (ld == D) return reinterpret_cast<const uint4*>(tile) + (tid + 256 * n);   // (decided at compile time for [B,H,N,d])
        const bf16* rows = tile + (size_t)(n * (256 / VPR)) * (size_t)ld;
        const unsigned off = (unsigned)(tid / VPR) * (unsigned)ld + (unsigned)(tid % VPR) * 8u;
        return reinterpret_cast<const uint4*>(rows + off);
    }
    __device__ __forceinline__ void load(const bf16* tile, int ld, int valid_rows, int tid)
    {
        if (valid_rows >= C) {
#pragma unroll
            for (int n = 0; n < NV; ++n) v[n] = ldg16<NTL>(at(tile, ld, tid, n));
        } else {
            const int lim = valid_rows * VPR;
#pragma unroll
            for (int n = 0; n < NV; ++n) {
                const int x = tid + 256 * n;
                v[n] = x < lim ? ldg16<NTL>(at(tile, ld, tid, n)) : make_uint4(0, 0, 0, 0);
            }
        }
    }
    // All C rows exist: no predicate, so the loads are issued unconditionally and the compiler can count them
    // (s_waitcnt vmcnt(n) with the exact n instead of 0 wherever younger loads are meant to stay in flight).
    __device__ __forceinline__ void load_full(const bf16* tile, int ld, int tid)
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) v[n] = ldg16<NTL>(at(tile, ld, tid, n));
    }
    __device__ __forceinline__ void store(bf16* lds, int tid) const
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / VPR, cv = x % VPR;
            *reinterpret_cast<uint4*>(lds + row * (D + PAD) + cv * 8) = v[n];
        }
    }
    // The tile holds Z; write alpha * Z + beta (per feature, fp32 arithmetic, rounded once to bf16) instead.
    // A thread's vectors all sit in the same 8 columns because 256 is a multiple of VPR.
    __device__ __forceinline__ void store_affine(bf16* lds, const float* alpha, const float* beta, int tid) const
    {
        const AffineCols ac(alpha, beta, (tid % VPR) * 8);
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / VPR, cv = x % VPR;
            *reinterpret_cast<uint4*>(lds + row * (D + PAD) + cv * 8) = ac.apply(v[n]);
        }
    }
};

// Store a TRANSPOSED 32x32 accumulator tile (register 4a+b of lane (r,h) = feature 8a+4h+b of token r) as bf16 into
// rows [0,32) x columns [col0, col0+32) of the row-major matrix at `rows` (leading dimension ld).  The two half-waves
// trade registers so that every lane ends up with 8 consecutive features of its token: two 16-byte stores per lane.
__device__ __forceinline__ void store_tile_T(bf16* rows, int ld, int col0, const f32x16& acc, int valid_rows, int lane)
{
    const int r = lane & 31, h = lane >> 5;
    bf16* dst = rows + ((unsigned)r * (unsigned)ld + (unsigned)(col0 + 8 * h));   // uniform base + 32-bit lane offset
#pragma unroll
    for (int ap = 0; ap < 2; ++ap) {
        const unsigned x0 = pack2(acc[8 * ap + 0], acc[8 * ap + 1]), x1 = pack2(acc[8 * ap + 2], acc[8 * ap + 3]);
        const unsigned y0 = pack2(acc[8 * ap + 4], acc[8 * ap + 5]), y1 = pack2(acc[8 * ap + 6], acc[8 * ap + 7]);
        // lanes 32..63 of x <-> lanes 0..31 of y
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
        if (r < valid_rows) *reinterpret_cast<uint4*>(dst + 16 * ap) = make_uint4(s0[0], s1[0], s0[1], s1[1]);
    }
}

// The same tile into an LDS staging area instead (rows of D = 64 or 128 bf16, no padding: the 16-byte pieces of a
// row are permuted by an XOR with bits 1..3 of the row number so that neither these writes nor the row reads below
// pile up on banks), and the staging area out to memory as whole rows: eight neighbouring lanes write one 128-byte
// line.  store_tile_T sends 32 bytes per row and instruction; a plain streaming kernel with that store pattern loses
// a third of its bandwidth against whole-line stores on this GPU.
template <int D>
__device__ __forceinline__ int stage_at(int row, int piece)
{
    // rows of 128 bytes: neighbouring rows already differ by half the banks, so the row PAIR picks the permutation;
    // rows of 256 bytes all start on bank 0: the row itself does
    return row * D + ((piece ^ (D == 64 ? ((row >> 1) & 7) : (row & 15))) << 3);
}

template <int D>
__device__ __forceinline__ void stage_tile_T(bf16* stage, int row0, int col0, const f32x16& acc, int lane)
{
    const int r = lane & 31, h = lane >> 5, row = row0 + r;
#pragma unroll
    for (int ap = 0; ap < 2; ++ap) {
        const unsigned x0 = pack2(acc[8 * ap + 0], acc[8 * ap + 1]), x1 = pack2(acc[8 * ap + 2], acc[8 * ap + 3]);
        const unsigned y0 = pack2(acc[8 * ap + 4], acc[8 * ap + 5]), y1 = pack2(acc[8 * ap + 6], acc[8 * ap + 7]);
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(x0, y0, false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(x1, y1, false, false);
        *reinterpret_cast<uint4*>(stage + stage_at<D>(row, (col0 >> 3) + h + 2 * ap)) =
            make_uint4(s0[0], s1[0], s0[1], s1[1]);
    }
}

// ROWS x D staged tile -> rows of the row-major matrix at `out` (leading dimension ld), the first valid_rows of them.
template <int ROWS, int D, bool NTS = true>
__device__ __forceinline__ void flush_stage(const bf16* stage, bf16* out, int ld, int valid_rows, int tid)
{
    constexpr int PPR = D / 8;      // 16-byte pieces per row
#pragma unroll
    for (int n = 0; n < ROWS * PPR / 256; ++n) {
        const int x = tid + 256 * n, row = x / PPR, piece = x % PPR;
        if (row < valid_rows) {
            // streaming ("non-temporal") stores: nothing here reads an output again, whole 128-byte lines leave at
            // once, and lines that do not linger in the memory-side cache do not push the inputs out of it
            const uint4 t = *reinterpret_cast<const uint4*>(stage + stage_at<D>(row, piece));
            if (NTS) {
                u32x4v tv;
                tv[0] = t.x; tv[1] = t.y; tv[2] = t.z; tv[3] = t.w;
                __builtin_nontemporal_store(tv, reinterpret_cast<u32x4v*>(out + ((unsigned)row * (unsigned)ld + (unsigned)piece * 8u)));
            } else {
                *reinterpret_cast<uint4*>(out + ((unsigned)row * (unsigned)ld + (unsigned)piece * 8u)) = t;
            }
        }
    }
}

// Eq. 9 epilogue on a transposed accumulator tile: every value times `scale` (the token's 1/rms) times its gate.
// g[ap] holds the gate as store_tile_T would have stored it (8 consecutive features of this lane's token at
// col0 + 8h + 16ap); the same half-wave exchange that produces that order also undoes it.
__device__ __forceinline__ f32x16 gate_tile(const f32x16& acc, const uint4 (&g)[2], float scale)
{
    f32x16 out;
#pragma unroll
    for (int ap = 0; ap < 2; ++ap) {
        const u32x2 s0 = __builtin_amdgcn_permlane32_swap(g[ap].x, g[ap].z, false, false);
        const u32x2 s1 = __builtin_amdgcn_permlane32_swap(g[ap].y, g[ap].w, false, false);
        const unsigned x0 = s0[0], y0 = s0[1], x1 = s1[0], y1 = s1[1];
        out[8 * ap + 0] = acc[8 * ap + 0] * scale * bf16_lo(x0);
        out[8 * ap + 1] = acc[8 * ap + 1] * scale * bf16_hi(x0);
        out[8 * ap + 2] = acc[8 * ap + 2] * scale * bf16_lo(x1);
        out[8 * ap + 3] = acc[8 * ap + 3] * scale * bf16_hi(x1);
        out[8 * ap + 4] = acc[8 * ap + 4] * scale * bf16_lo(y0);
        out[8 * ap + 5] = acc[8 * ap + 5] * scale * bf16_hi(y0);
        out[8 * ap + 6] = acc[8 * ap + 6] * scale * bf16_lo(y1);
        out[8 * ap + 7] = acc[8 * ap + 7] * scale * bf16_hi(y1);
    }
    return out;
}

// =============================================================================================== shared pieces
// Load a [DA][DB] fp32 state as accumulator tiles: tile id = w + 4n -> (ab, bb) = (id / BB, id % BB).
template <int DA, int DB, bool NEG>
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
            for (int b = 0; b < 4; ++b) {
                const float v = src ? src[(ab * 32 + 8 * a + 4 * h + b) * DB + bb * 32 + r] : 0.f;
                acc[n][4 * a + b] = NEG ? -v : v;
            }
    }
}

// The same for the sum of `count` states that lie one behind the other at src (count == 0 or src == nullptr: zero):
// a workgroup that adds up the segment totals in front of (or behind) its own segment itself, in a fixed order,
// instead of reading what a scan kernel left.  The loads of two states are in flight at a time.
// The same sum for states stored in ACCUMULATOR ORDER, [wave][tile][lane][16] floats: what a lane adds up is then 64
// contiguous bytes per state and tile, four 16-byte loads instead of sixteen 4-byte ones.  The pre-pass writes its
// totals that way when the sweeps are going to add them up (same widths, so the same tile-to-wave mapping).
// U: states whose loads are in flight together (16 registers each; the caller knows how many it has to spare).
template <int DA, int DB, bool NEG, int U>
__device__ __forceinline__ void sum_states_acc(f32x16* acc, const float* src, int count, int w, int lane)
{
    constexpr int NT = (DA / 32) * (DB / 32) / 4;
    if (src == nullptr) count = 0;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const float4* p = reinterpret_cast<const float4*>(src) + ((size_t)(w * NT + n) * 64 + lane) * 4;
        f32x16 t = zero16();
        int k = 0;
        for (; k + U <= count; k += U) {
            float4 x[U][4];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int q = 0; q < 4; ++q) x[u][q] = p[(size_t)(k + u) * (DA * DB / 4) + q];
#pragma unroll
            for (int u = 0; u < U; ++u)          // (the order of the additions is the order of the states)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    t[4 * q] += x[u][q].x; t[4 * q + 1] += x[u][q].y; t[4 * q + 2] += x[u][q].z; t[4 * q + 3] += x[u][q].w;
                }
        }
        for (; k < count; ++k) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float4 v = p[(size_t)k * (DA * DB / 4) + q];
                t[4 * q] += v.x; t[4 * q + 1] += v.y; t[4 * q + 2] += v.z; t[4 * q + 3] += v.w;
            }
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = NEG ? -t[e] : t[e];
    }
}

template <int DA, int DB, bool NEG>
__device__ __forceinline__ void sum_states(f32x16* acc, const float* src, int count, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    constexpr int U = 4;                 // states whose loads are in flight together
    const int r = lane & 31, h = lane >> 5;
    if (src == nullptr) count = 0;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
        const float* p = src + (ab * 32 + 4 * h) * DB + bb * 32 + r;
        f32x16 t = zero16();
        int k = 0;
        for (; k + U <= count; k += U) {
            float x[U][16];
#pragma unroll
            for (int u = 0; u < U; ++u)
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) x[u][4 * a + b] = p[(size_t)(k + u) * (DA * DB) + (8 * a + b) * DB];
#pragma unroll
            for (int u = 0; u < U; ++u)          // (the order of the additions is the order of the states)
#pragma unroll
                for (int e = 0; e < 16; ++e) t[e] += x[u][e];
        }
        for (; k < count; ++k) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) t[4 * a + b] += p[(size_t)k * (DA * DB) + (8 * a + b) * DB];
        }
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[n][e] = NEG ? -t[e] : t[e];
    }
}

// Write a [DA][DB] state held as accumulator tiles into LDS as bf16, TRANSPOSED: dst[b][a] (row stride DA + PAD).
// A lane owns 4 consecutive a for one b, i.e. 8 contiguous bytes of dst.  NEG writes the negated value.
template <int DA, int DB, bool NEG>
__device__ __forceinline__ void state_to_lds_T(bf16* dst, const f32x16* acc, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a) {
            u32x2 v;
            v[0] = pack2<NEG>(acc[n][4 * a + 0], acc[n][4 * a + 1]);
            v[1] = pack2<NEG>(acc[n][4 * a + 2], acc[n][4 * a + 3]);
            *reinterpret_cast<u32x2*>(dst + (bb * 32 + r) * (DA + PAD) + ab * 32 + 8 * a + 4 * h) = v;
        }
    }
}

// Write a [DA][DB] state held as accumulator tiles to global memory, fp32, row-major [DA][DB].
template <int DA, int DB>
__device__ __forceinline__ void store_state(float* dst, const f32x16* acc, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) dst[(ab * 32 + 8 * a + 4 * h + b) * DB + bb * 32 + r] = acc[n][4 * a + b];
    }
}

// Same state written TRANSPOSED, as [DB][DA]: a lane owns 4 consecutive a for one b -> one 16-byte store.
template <int DA, int DB>
__device__ __forceinline__ void store_state_T(float* dst, const f32x16* acc, int w, int lane)
{
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
            *reinterpret_cast<float4*>(dst + (size_t)(bb * 32 + r) * DA + ab * 32 + 8 * a + 4 * h) =
                make_float4(acc[n][4 * a + 0], acc[n][4 * a + 1], acc[n][4 * a + 2], acc[n][4 * a + 3]);
    }
}

// =============================================================================================== pre-pass body
// out[a][b] = sum over `ntok` tokens s of X[s][a] * Y[s][b]   (fp32, [DA][DB] row-major).  One workgroup; wave w owns
// output tiles w, w+4, ...  LDS: 64 x (DA + PAD) + 64 x (DB + PAD) bf16.
// AFF = 1 (2): the X (Y) tensor is Z and the operand is alpha * Z + beta (Eq. 11-12), alpha and beta being this
// head's DA (DB) floats.
template <int DA, int DB, int AFF = 0>
struct PrepassLds {
    static constexpr int R = 64;
    static constexpr int TILES = (R * (DA + PAD) + R * (DB + PAD)) * 2;
    static constexpr int BYTES = TILES + (AFF == 1 ? 2 * DA * 4 : AFF == 2 ? 2 * DB * 4 : 0);
};

template <int DA, int DB, int AFF, bool NTL = false>
__device__ __forceinline__ void prepass_body(const bf16* __restrict__ X, const bf16* __restrict__ Y,
                                             float* __restrict__ out, const float* __restrict__ alpha,
                                             const float* __restrict__ beta, int lda, int ldb, int ntok,
                                             unsigned char* lds, int tid, int w, int lane, bool rev = false,
                                             bool acc_order = false)
{
    constexpr int R = 64;
    constexpr int PF = 2;          // 64-token blocks in flight per workgroup: this kernel only reads, so it lives
                                   // off memory-level parallelism
    bf16* sX = reinterpret_cast<bf16*>(lds);
    bf16* sY = sX + R * (DA + PAD);
    float* sAff = reinterpret_cast<float*>(lds + PrepassLds<DA, DB, 0>::TILES);
    constexpr int DAFF = AFF == 1 ? DA : DB;
    constexpr int BB = DB / 32, NT = (DA / 32) * BB / 4;
    f32x16 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = zero16();
    TileRegs<R, DA, NTL> rx[PF];     // NTL: nobody reads these tensors again soon (the non-causal forward)
    TileRegs<R, DB, NTL> ry[PF];
    if (AFF != 0) {
        if (tid < DAFF) { sAff[tid] = alpha[tid]; sAff[DAFF + tid] = beta[tid]; }
        __syncthreads();
    }
    auto consume = [&](int u) __attribute__((always_inline)) {   // registers of set u -> LDS -> accumulators
        if (AFF == 1) rx[u].store_affine(sX, sAff, sAff + DAFF, tid);
        else rx[u].store(sX, tid);
        if (AFF == 2) ry[u].store_affine(sY, sAff, sAff + DAFF, tid);
        else ry[u].store(sY, tid);
    };
    auto multiply = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
            for (int s0 = 0; s0 < R; s0 += 16)
                acc[n] = mfma(ld_tr(sX, DA + PAD, s0, ab * 32, lane), ld_tr(sY, DB + PAD, s0, bb * 32, lane), acc[n]);
        }
    };
    // The sum does not care about the order of its blocks.  `rev` (only taken when every block is complete) walks them
    // from the segment's end to its start, so that a forward sweep that follows finds the blocks it needs first
    // among the most recently read ones in the memory-side cache.
    rev = rev && ntok % R == 0;
    auto at = [&](int c) __attribute__((always_inline)) { return (size_t)(rev ? ntok - R - c : c); };
    int c0 = 0;
    if (ntok >= 2 * PF * R) {
        // Steady state: the PF blocks being consumed and the PF blocks being fetched are all complete, so every load
        // is unconditional and the wait before a set is consumed leaves the younger set's loads in flight.
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            rx[u].load_full(X + at(u * R) * lda, lda, tid);
            ry[u].load_full(Y + at(u * R) * ldb, ldb, tid);
            __builtin_amdgcn_sched_barrier(0);   // keep the sets in issue order: the wait for set 0 must not cover set 1
        }
        for (; c0 + 2 * PF * R <= ntok; c0 += PF * R) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                consume(u);
                __syncthreads();
                rx[u].load_full(X + at(c0 + (PF + u) * R) * lda, lda, tid);
                ry[u].load_full(Y + at(c0 + (PF + u) * R) * ldb, ldb, tid);
                multiply();
                __syncthreads();
            }
        }
    } else {
#pragma unroll
        for (int u = 0; u < PF; ++u)
            if (u * R < ntok) {
                rx[u].load(X + at(u * R) * lda, lda, rev ? R : ntok - u * R, tid);
                ry[u].load(Y + at(u * R) * ldb, ldb, rev ? R : ntok - u * R, tid);
            }
    }
    // The rest (at most 2 PF blocks, the last one possibly ragged): set u holds block c0 + u R if that block exists.
    for (; c0 < ntok; c0 += PF * R) {
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            const int c = c0 + u * R;
            if (c < ntok) {
                consume(u);
                __syncthreads();
                if (c + PF * R < ntok) {
                    rx[u].load(X + at(c + PF * R) * lda, lda, rev ? R : ntok - c - PF * R, tid);
                    ry[u].load(Y + at(c + PF * R) * ldb, ldb, rev ? R : ntok - c - PF * R, tid);
                }
                multiply();
                __syncthreads();
            }
        }
    }
    if (acc_order) {
        // for a sweep that adds the totals up itself (sum_states_acc): [wave][tile][lane][16]
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            float4* dst = reinterpret_cast<float4*>(out) + ((size_t)(w * NT + n) * 64 + lane) * 4;
#pragma unroll
            for (int q = 0; q < 4; ++q)
                dst[q] = make_float4(acc[n][4 * q], acc[n][4 * q + 1], acc[n][4 * q + 2], acc[n][4 * q + 3]);
        }
        return;
    }
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ab = id / BB, bb = id % BB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b)
                out[(ab * 32 + 8 * a + 4 * h + b) * DB + bb * 32 + r] = acc[n][4 * a + b];
    }
}

// =============================================================================================== forward sweep body
// One workgroup (4 waves) per segment.  Per chunk of C tokens:
//   P^T = K Q^T (masked), O^T = V^T P^T + S_prev^T Q^T, store O, S += K^T V.
// Wave w owns output rows [32*tb, 32*tb+32) with tb = w % WT and NJ column tiles; it recomputes the score
// tiles of its row block itself (matrix-core time is cheap here, LDS round trips and barriers are not).
// ZQK: Qb points at Z, Kb is unused, and `aff` at this head's alpha_q row of the [4][H][DK] parameter array
// (rows alpha_q, beta_q, alpha_k, beta_k, `aff_stride` floats apart): Q and K tiles are formed on the way into LDS.
template <int C, int DK, int DV, bool ZQK = false, bool GATE = false>
struct FwdLds {
    static constexpr int LDK = DK + PAD, LDV = DV + PAD;
    static constexpr int TILES = (2 * C * LDK + C * LDV + DV * LDK) * 2;
    static constexpr int SMALL = (ZQK ? 4 * DK * 4 : 0) + (GATE ? 4 * C * 4 : 0);      // affine parameters, sums of squares
    static constexpr int BYTES = TILES + SMALL + (GATE ? C * LDV * 2 : 0);            // + the gate tile
    static constexpr int STAGED = BYTES + (GATE ? 2 : 1) * C * DV * 2;                // + staging tile(s) for the output(s)
};

// GATE (Eq. 9, Y = Norm(O) * G with Norm(o) = o / sqrt(mean_j o_j^2 + eps) over the head's DV features): Gb and Yb
// point at the gate and at the output rows of this segment; Ob may then be null (O itself is only needed by a
// backward pass).  A token's features are spread over two half-waves and WJ waves: each wave leaves its share of
// the sum of squares in LDS, and the gated store happens after the barrier that ends the chunk anyway -- it needs
// nothing but registers by then -- so the epilogue costs no barrier of its own.  The gate tile comes in like V
// (whole 128- or 256-byte rows, one chunk ahead, via LDS) and is picked up from LDS in the order the output tile is
// stored in; fetching it from HBM in that order directly (32 bytes per row and instruction) cost 20 % more time.
// STAGE: the output tile leaves through an LDS staging tile as whole rows, after the barrier that ends the chunk.
// With GATE the gated output Y has a staging tile of its own: it is filled after that barrier (the normalisation needs
// every wave's share of the sums of squares) and leaves after the NEXT chunk's first barrier, or after the loop.
template <int C, int DK, int DV, bool ZQK, bool SAVE, bool GATE = false, bool STAGE = false>
__device__ __forceinline__ void fwd_sweep_body(const bf16* __restrict__ Qb, const bf16* __restrict__ Kb,
                                               const bf16* __restrict__ Vb, bf16* __restrict__ Ob,
                                               const float* __restrict__ S0, int n_s0, bool s0_acc,
                                               float* __restrict__ S_final,
                                               float* __restrict__ S_final_T, const float* __restrict__ aff,
                                               size_t aff_stride, int ldk, int ldv, int ntok, unsigned char* lds,
                                               int tid, int w, int lane, const bf16* __restrict__ Gb = nullptr,
                                               bf16* __restrict__ Yb = nullptr, float eps = 0.f)
{
    constexpr int LDK = DK + PAD, LDV = DV + PAD;
    constexpr int TB = C / 32, JB = DV / 32, IB = DK / 32;
    constexpr int WT = TB < 4 ? TB : 4, WJ = 4 / WT, NJ = JB / WJ;
    constexpr int NS = IB * JB / 4;
    static_assert(TB <= 4 && JB % WJ == 0, "unsupported tile shape");
    bf16* sQ = reinterpret_cast<bf16*>(lds);
    bf16* sK = sQ + C * LDK;
    bf16* sV = sK + C * LDK;
    bf16* sST = sV + C * LDV;          // S^T as bf16: [j][i]
    const int tb = w % WT, jg = w / WT;

    unsigned maskK[8];
    make_masks<true>(maskK, lane);

    TileRegs<C, DK, !ZQK> rq;   // Q is read once: streaming hint; with ZQK it holds Z, which the pre-pass shares
    TileRegs<C, DK> rk;         // (unused with ZQK)
    TileRegs<C, DV> rv;
    TileRegs<C, DV, true> rg;   // GATE: the gate tile travels like V (whole lines, one chunk ahead, through LDS)
    rq.load(Qb, ldk, ntok, tid);
    if (!ZQK) rk.load(Kb, ldk, ntok, tid);
    rv.load(Vb, ldv, ntok, tid);
    if (GATE) rg.load(Gb, ldv, ntok, tid);
    float* sAff = reinterpret_cast<float*>(lds + FwdLds<C, DK, DV, false>::TILES);
    float* sSq = sAff + (ZQK ? 4 * DK : 0);   // GATE: [WJ][C] partial sums of squares
    bf16* sG = reinterpret_cast<bf16*>(lds + FwdLds<C, DK, DV, false>::TILES + FwdLds<C, DK, DV, ZQK, true>::SMALL);
    if (ZQK) {
        for (int x = tid; x < 4 * DK; x += 256) sAff[x] = aff[(size_t)(x / DK) * aff_stride + x % DK];
        __syncthreads();
    }

    f32x16 accS[NS];
    // (n_s0 states, one behind the other, are added up; s0_acc: they are stored in accumulator order)
    if (s0_acc) sum_states_acc<DK, DV, false, 4>(accS, S0, n_s0, w, lane);
    else sum_states<DK, DV, false>(accS, S0, n_s0, w, lane);

    // staging tiles (STAGE): O, or with GATE: Y then O
    bf16* sOutY = reinterpret_cast<bf16*>(lds + FwdLds<C, DK, DV, ZQK, GATE>::BYTES);
    bf16* sOutO = GATE ? sOutY + C * DV : sOutY;
    for (int c0 = 0; c0 < ntok; c0 += C) {
        if (ZQK) {
            rq.store_affine(sQ, sAff, sAff + DK, tid);
            rq.store_affine(sK, sAff + 2 * DK, sAff + 3 * DK, tid);
        } else {
            rq.store(sQ, tid);
            rk.store(sK, tid);
        }
        rv.store(sV, tid);
        if (GATE) rg.store(sG, tid);
        state_to_lds_T<DK, DV, false>(sST, accS, w, lane);
        __syncthreads();
        if (GATE && STAGE && c0 > 0)    // the chunk before's gated output, complete in its staging tile since that barrier
            flush_stage<C, DV>(sOutY, Yb + (size_t)(c0 - C) * ldv, ldv, C, tid);
        const bool more = c0 + C < ntok;
        if (more) {
            rq.load(Qb + (size_t)(c0 + C) * ldk, ldk, ntok - c0 - C, tid);
            if (!ZQK) rk.load(Kb + (size_t)(c0 + C) * ldk, ldk, ntok - c0 - C, tid);
            rv.load(Vb + (size_t)(c0 + C) * ldv, ldv, ntok - c0 - C, tid);
            if (GATE) rg.load(Gb + (size_t)(c0 + C) * ldv, ldv, ntok - c0 - C, tid);
        }
        bf16x8 bQ[DK / 16];   // Q rows of this wave's token block: the B operand (n = token, k = feature i)
#pragma unroll
        for (int kk = 0; kk < DK / 16; ++kk) bQ[kk] = ld_nat(sQ, LDK, tb * 32, kk * 16, lane);
        f32x16 accO[NJ];      // O^T tiles: rows = features j, columns = tokens t
#pragma unroll
        for (int n = 0; n < NJ; ++n) accO[n] = zero16();
        // inter-chunk part: S_prev^T Q^T
#pragma unroll
        for (int n = 0; n < NJ; ++n)
#pragma unroll
            for (int kk = 0; kk < DK / 16; ++kk)
                accO[n] = mfma(ld_nat(sST, LDK, (jg * NJ + n) * 32, kk * 16, lane), bQ[kk], accO[n]);
        // intra-chunk part: V^T (masked K Q^T), key blocks sb <= tb
#pragma unroll
        for (int sb = 0; sb < TB; ++sb) {
            if (sb <= tb) {
                f32x16 pT = zero16();
#pragma unroll
                for (int kk = 0; kk < DK / 16; ++kk) pT = mfma(ld_nat(sK, LDK, sb * 32, kk * 16, lane), bQ[kk], pT);
                bf16x8 p0v, p1v;
                if (sb == tb) cvt_tile_masked(pT, maskK, p0v, p1v);
                else cvt_tile(pT, p0v, p1v);
#pragma unroll
                for (int n = 0; n < NJ; ++n) {
                    accO[n] = mfma(ld_tr_perm(sV, LDV, sb * 32, (jg * NJ + n) * 32, lane), p0v, accO[n]);
                    accO[n] = mfma(ld_tr_perm(sV, LDV, sb * 32 + 16, (jg * NJ + n) * 32, lane), p1v, accO[n]);
                }
            }
        }
        const int valid = ntok - (c0 + tb * 32);
        if (STAGE && (!GATE || Ob != nullptr)) {
#pragma unroll
            for (int n = 0; n < NJ; ++n) stage_tile_T<DV>(sOutO, tb * 32, (jg * NJ + n) * 32, accO[n], lane);
        } else if (!GATE || Ob != nullptr) {
            bf16* rows = Ob + (size_t)(c0 + tb * 32) * ldv;
#pragma unroll
            for (int n = 0; n < NJ; ++n) store_tile_T(rows, ldv, (jg * NJ + n) * 32, accO[n], valid, lane);
        }
        uint4 gate[GATE ? NJ : 1][2];   // this chunk's gate, in the order the output tile is stored in
        if (GATE) {
            // (read before the barrier that ends the chunk: the next chunk's gate tile overwrites this one after it)
            const bf16* g = sG + (tb * 32 + (lane & 31)) * LDV + 8 * (lane >> 5);
#pragma unroll
            for (int n = 0; n < NJ; ++n)
#pragma unroll
                for (int ap = 0; ap < 2; ++ap)
                    gate[n][ap] = *reinterpret_cast<const uint4*>(g + (jg * NJ + n) * 32 + 16 * ap);
            // this wave's share of sum_j O[t][j]^2: 16 features per tile and lane, the other 16 in lane ^ 32
            float ss = 0.f;
#pragma unroll
            for (int n = 0; n < NJ; ++n)
#pragma unroll
                for (int e = 0; e < 16; ++e) ss = fmaf(accO[n][e], accO[n][e], ss);
            const unsigned sb = __builtin_bit_cast(unsigned, ss);
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(sb, sb, false, false);
            const unsigned sw0 = sw[0], sw1 = sw[1];
            if (lane < 32) sSq[jg * C + tb * 32 + lane] = __builtin_bit_cast(float, sw0) + __builtin_bit_cast(float, sw1);
        }
        // state update S += K^T V (after the segment's last chunk only if the final state is asked for)
        if (more || S_final != nullptr || (SAVE && S_final_T != nullptr)) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, ib = id / JB, jb = id % JB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accS[n] = mfma(ld_tr(sK, LDK, s0, ib * 32, lane), ld_tr(sV, LDV, s0, jb * 32, lane), accS[n]);
            }
        }
        __syncthreads();
        if (STAGE && (!GATE || Ob != nullptr))   // (the staging tile is next written after the next chunk's first barrier)
            flush_stage<C, DV>(sOutO, Ob + (size_t)c0 * ldv, ldv, ntok - c0, tid);
        if (GATE) {
            // (the next chunk writes sSq only after its own first barrier, which every wave reaches after this read)
            float tot = 0.f;
#pragma unroll
            for (int g = 0; g < WJ; ++g) tot += sSq[g * C + tb * 32 + (lane & 31)];
            const float rinv = __builtin_amdgcn_rsqf(fmaf(tot, 1.f / DV, eps));
            if (STAGE) {
                // (the tile was last read, by the flush above, before the barrier that has just ended this chunk)
#pragma unroll
                for (int n = 0; n < NJ; ++n)
                    stage_tile_T<DV>(sOutY, tb * 32, (jg * NJ + n) * 32, gate_tile(accO[n], gate[n], rinv), lane);
            } else {
                bf16* rows = Yb + (size_t)(c0 + tb * 32) * ldv;
#pragma unroll
                for (int n = 0; n < NJ; ++n)
                    store_tile_T(rows, ldv, (jg * NJ + n) * 32, gate_tile(accO[n], gate[n], rinv), valid, lane);
            }
        }
    }
    if (GATE && STAGE && ntok > 0) {
        __syncthreads();        // the last chunk's gated tile is complete
        const int c_last = ((ntok - 1) / C) * C;
        flush_stage<C, DV>(sOutY, Yb + (size_t)c_last * ldv, ldv, ntok - c_last, tid);
    }
    if (S_final != nullptr) store_state<DK, DV>(S_final, accS, w, lane);
    if (SAVE && S_final_T != nullptr) store_state_T<DK, DV>(S_final_T, accS, w, lane);   // [dv][dk], as the backward reads it
}

// =============================================================================================== backward sweep body
// One workgroup per segment, walking the chunks from the LAST to the first, so that each input tile is read once
// for all three gradients.  Two states live in accumulator registers, both stored transposed ([dv][dk], lane = one
// feature i, 4 consecutive j):
//   -S^T: minus the sum of V^T K over tokens before the current chunk.  It enters as the inclusive prefix at the
//         end of the segment and is rolled BACK by one chunk per step (S_{c-1} = S_c - V_c^T K_c, fp32); keeping
//         the negative makes the roll-back a plain accumulate and the sign is restored for free when rounding.
//   R^T : sum of dO^T Q over tokens after the current chunk; it grows by one chunk per step.
// Per chunk:  dQ = dP K + dO S^T',  dK = dP^T Q + V R^T',  dV = P^T dO + K R,
//             P = (Q K^T) o M,  dP = (dO V^T) o M, every output accumulated transposed.
// Send == nullptr means the whole sequence is this one segment: S is then built here, R starts at zero.
// Otherwise the start states are sums of n_send and n_rnext states that lie one behind the other at Send and Rnext
// (one each if a scan has run; the segment totals themselves if not; Rnext may be null: zero).
// R_final, if given, receives the state R after the segment's first chunk has been added ([dk][dv], fp32).
// ckpt (only with Send == nullptr; may be null): the pass that builds S leaves a copy of the running state after
// every ckpt_every chunks there, and the walk back takes that copy up again when it reaches the same place, so that
// the fp32 rounding of the walk never accumulates over more than ckpt_every chunks (for states that grow with the
// position it would otherwise swamp the small states of the first chunks of a long sequence).  Every lane writes and
// later reads its own registers' worth: [copy][wave][tile][lane][16] floats.
//
// ZQK (Eq. 11-12, Q = alpha_q Z + beta_q, K = alpha_k Z + beta_k): Qb points at Z, Kb is unused, dQb receives
// dZ = alpha_q dQ + alpha_k dK and dKb is unused.  The parameter gradients are sums over tokens,
//   d_alpha_q = sum dQ * Z, d_beta_q = sum dQ, d_alpha_k = sum dK * Z, d_beta_k = sum dK;
// each workgroup writes its share of the four as [4][DK] floats to `part`, a later kernel adds the shares up.
template <int C, int DK, int DV, bool ZQK = false>
struct BwdLds {
    static constexpr int LDK = DK + PAD, LDV = DV + PAD;
    // With one head width of 128 the two published states share ONE tile (S while dQ is formed, then R for dK and dV,
    // two more barriers per chunk): that brings the workgroup under 80 KB, so that two of them fit a compute unit.
    static constexpr bool SHARE = (C == 64 && DK != DV);
    static constexpr int TILES = (2 * C * LDK + 2 * C * LDV + (SHARE ? 1 : 2) * DK * LDV) * 2;
    static constexpr int WORK = TILES + (ZQK ? C * LDK * 2 + 4 * DK * 4 : 0);
    // 64-wide heads: the output tiles leave through unpadded staging tiles (whole-line stores), 8 KB each
    static constexpr bool STAGE = (C == 64 && DK == 64 && DV == 64);
    // one width of 128 (without the Eq. 11-12 prologue): the 64-wide outputs take turns in ONE 8 KB staging tile, which
    // is what still fits beside two resident workgroups (78.8 / 79.9 KB); the 128-wide ones keep their direct stores
    static constexpr bool STAGE_NARROW = SHARE && !ZQK && DK == 64;
    static constexpr int BYTES = WORK + (STAGE ? (ZQK ? 2 : 3) * C * 64 * 2 : 0) + (STAGE_NARROW ? C * 64 * 2 : 0);
};

// Sum over the tokens of a wave half for the parameter gradients.  x holds, per lane, 16 values of one token (the
// token is lane % 32, the value index e = 4a + b stands for feature 8a + 4h + b, h = lane / 32).  Every exchange step
// pairs each lane with a partner, the two keep opposite halves of the live values and add the partner's copy of
// theirs, so the reduction costs 16 exchanges instead of 80; the lane ends with the total of value
// e = 8*b16 + 4*b8 + 2*b4 + b2 (b_m = bit m of the lane number).  All exchanges are register-to-register:
//   16: v_permlane16_swap (odd 16-lane rows of the first operand trade places with even rows of the second), which
//       also needs no per-lane choice between x[j] and x[j+8] (the compiler would turn that choice into a
//       dynamically indexed vector);
//    8: DPP row rotate by 8;   4: DPP half-row mirror (partner = lane ^ 7: differs in bit 4's place, and the two
//       steps after it still cover all eight lanes);   2, 1: DPP quad permutes.
template <int CTRL>
__device__ __forceinline__ float dpp_get(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

__device__ __forceinline__ float sum_tokens16(const f32x16& x, int lane)
{
    constexpr int ROW_ROR8 = 0x128, HALF_MIRROR = 0x141, QUAD_XOR2 = 0x4E, QUAD_XOR1 = 0xB1;
    float y8[8], y4[4], y2[2];
    const bool u8 = lane & 8, u4 = lane & 4, u2 = lane & 2;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        // (bit casts go through named scalars: applied to a vector element they read element 0)
        const float lo = x[j], hi = x[j + 8];
        const u32x2 s = __builtin_amdgcn_permlane16_swap(__builtin_bit_cast(unsigned, lo),
                                                         __builtin_bit_cast(unsigned, hi), false, false);
        const unsigned s0 = s[0], s1 = s[1];
        y8[j] = __builtin_bit_cast(float, s0) + __builtin_bit_cast(float, s1);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) y4[j] = (u8 ? y8[j + 4] : y8[j]) + dpp_get<ROW_ROR8>(u8 ? y8[j] : y8[j + 4]);
#pragma unroll
    for (int j = 0; j < 2; ++j) y2[j] = (u4 ? y4[j + 2] : y4[j]) + dpp_get<HALF_MIRROR>(u4 ? y4[j] : y4[j + 2]);
    const float y = (u2 ? y2[1] : y2[0]) + dpp_get<QUAD_XOR2>(u2 ? y2[0] : y2[1]);
    return y + dpp_get<QUAD_XOR1>(y);
}

template <int C, int DK, int DV, bool ZQK>
__device__ __forceinline__ void bwd_sweep_body(const bf16* __restrict__ Qb, const bf16* __restrict__ Kb,
                                               const bf16* __restrict__ Vb, const bf16* __restrict__ Gb,
                                               bf16* __restrict__ dQb, bf16* __restrict__ dKb, bf16* __restrict__ dVb,
                                               const float* __restrict__ Send, int n_send,
                                               const float* __restrict__ Rnext, int n_rnext, int acc_mask,
                                               float* __restrict__ R_final, const float* __restrict__ aff,
                                               size_t aff_stride, float* __restrict__ part, int ldk, int ldv,
                                               int ntok, unsigned char* lds, int tid, int w, int lane,
                                               float* ckpt = nullptr, int ckpt_every = 0)
{
    constexpr int LDK = DK + PAD, LDV = DV + PAD;
    constexpr int TB = C / 32, JB = DV / 32, IB = DK / 32;
    constexpr int WT = TB < 4 ? TB : 4, WJ = 4 / WT, NJ = JB / WJ, NI = IB / WJ;
    constexpr int NS = IB * JB / 4;
    static_assert(TB <= 4 && JB % WJ == 0 && IB % WJ == 0, "unsupported tile shape");
    bf16* sQ = reinterpret_cast<bf16*>(lds);
    bf16* sK = sQ + C * LDK;
    bf16* sV = sK + C * LDK;
    bf16* sG = sV + C * LDV;           // dO
    constexpr bool SHARE = BwdLds<C, DK, DV, false>::SHARE;
    constexpr bool STAGE = BwdLds<C, DK, DV, false>::STAGE;
    bf16* sOutQ = reinterpret_cast<bf16*>(lds + BwdLds<C, DK, DV, ZQK>::WORK);     // dQ (with ZQK: dZ)
    bf16* sOutV = sOutQ + C * 64;
    bf16* sOutK = sOutV + C * 64;                                                  // (not with ZQK)
    bf16* sS = sG + C * LDV;                        // S  [i][j] bf16
    bf16* sR = SHARE ? sS : sS + DK * LDV;          // R  [i][j] bf16 (the same tile, later in the chunk, with SHARE)
    const int rb = w % WT, cg = w / WT;
    const int n_ch = (ntok + C - 1) / C;

    unsigned maskK[8], maskQ[8];
    make_masks<true>(maskK, lane);
    make_masks<false>(maskQ, lane);

    // Q and dO with the streaming hint, K and V without: nothing reads Q and dO again after this sweep, and the
    // pre-pass has left K and V in the memory-side cache for it (launch_bf16_bwd).  With the hint on all four the
    // forward call that follows on the same tensors loses more on the K and V it no longer finds there than this sweep
    // gains (0.290 -> 0.294 ms per step at the LM shape).
    // (Not with ZQK: Z stands for Q and K alike, both pairs of the pre-pass read it, and the hint measured 0.7 % slower.)
    TileRegs<C, DK, !ZQK> rq;          // with ZQK only rq is used in the main loop: it holds Z
    TileRegs<C, DK> rk;
    TileRegs<C, DV> rv;
    TileRegs<C, DV, !ZQK> rg;
    f32x16 accNS[NS], accRT[NS];       // states, transposed: [DV][DK]; accNS holds MINUS S^T
    bf16* sZ = reinterpret_cast<bf16*>(lds + BwdLds<C, DK, DV, false>::TILES);
    float* sAff = reinterpret_cast<float*>(sZ + C * LDK);
    float pg[4][NI];                   // this lane's running share of the four parameter gradients
    if (ZQK) {
        for (int x = tid; x < 4 * DK; x += 256) sAff[x] = aff[(size_t)(x / DK) * aff_stride + x % DK];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int n = 0; n < NI; ++n) pg[q][n] = 0.f;
        __syncthreads();
    }

    if (Send == nullptr) {
        // single segment: no pre-pass ran, build -S^T = -sum V^T K over the whole sequence here
#pragma unroll
        for (int n = 0; n < NS; ++n) { accNS[n] = zero16(); accRT[n] = zero16(); }
        for (int ci = 0; ci < n_ch; ++ci) {
            const int c0 = ci * C;
            rk.load((ZQK ? Qb : Kb) + (size_t)c0 * ldk, ldk, ntok - c0, tid);
            rv.load(Vb + (size_t)c0 * ldv, ldv, ntok - c0, tid);
            __syncthreads();
            if (ZQK) rk.store_affine(sK, sAff + 2 * DK, sAff + 3 * DK, tid);
            else rk.store(sK, tid);
            rv.store(sV, tid);
            __syncthreads();
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16) {
                    u32x4 a = __builtin_bit_cast(u32x4, ld_tr(sV, LDV, s0, jb * 32, lane));
                    a ^= 0x80008000u;   // minus sign: flip the sign bits of one operand
                    accNS[n] = mfma(__builtin_bit_cast(bf16x8, a), ld_tr(sK, LDK, s0, ib * 32, lane), accNS[n]);
                }
            }
            if (ckpt != nullptr && (ci + 1) % ckpt_every == 0 && ci + 1 < n_ch) {
                float4* dst = reinterpret_cast<float4*>(ckpt + (size_t)((ci + 1) / ckpt_every - 1) * (DK * DV)) +
                              ((size_t)(w * NS) * 64 + lane) * 4;
#pragma unroll
                for (int n = 0; n < NS; ++n)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
                        dst[(size_t)n * 256 + q] = make_float4(accNS[n][4 * q], accNS[n][4 * q + 1], accNS[n][4 * q + 2],
                                                               accNS[n][4 * q + 3]);
            }
        }
        __syncthreads();
    }

    {
        const int c0 = (n_ch - 1) * C;
        rq.load(Qb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
        if (!ZQK) rk.load(Kb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
        rv.load(Vb + (size_t)c0 * ldv, ldv, ntok - c0, tid);
        rg.load(Gb + (size_t)c0 * ldv, ldv, ntok - c0, tid);
    }
    if (Send != nullptr) {
        // (n_send, n_rnext states are added up; acc_mask bit 0 / 1: those of S / R are stored in accumulator order)
        if (acc_mask & 1) sum_states_acc<DV, DK, true, 8>(accNS, Send, n_send, w, lane);
        else sum_states<DV, DK, true>(accNS, Send, n_send, w, lane);
        if (acc_mask & 2) sum_states_acc<DV, DK, false, 8>(accRT, Rnext, n_rnext, w, lane);
        else sum_states<DV, DK, false>(accRT, Rnext, n_rnext, w, lane);
    }

    for (int ci = n_ch - 1; ci >= 0; --ci) {
        const int c0 = ci * C;
        if constexpr (SHARE && !ZQK) {
            // One width of 128: the two published states share one LDS tile.  The gradients that need R (dK, dV) come
            // first, on the R published with the tiles; then S takes R's place for dQ: four barriers per chunk.  The
            // 64-wide outputs go through one staging tile in turn (dK or dV after the second barrier, dQ after the
            // last) and leave as whole-line streaming stores.  Every sum is formed as in the general flow below.
            bf16* sSt = sOutQ;
            rq.store(sQ, tid);
            rk.store(sK, tid);
            rv.store(sV, tid);
            rg.store(sG, tid);
            state_to_lds_T<DV, DK, false>(sR, accRT, w, lane);      // R: the state after this chunk
            __syncthreads();
            if (ci > 0) {
                rq.load(Qb + (size_t)(c0 - C) * ldk, ldk, C, tid);
                rk.load(Kb + (size_t)(c0 - C) * ldk, ldk, C, tid);
                rv.load(Vb + (size_t)(c0 - C) * ldv, ldv, C, tid);
                rg.load(Gb + (size_t)(c0 - C) * ldv, ldv, C, tid);
            }
            if (ckpt != nullptr && (ci + 1) % ckpt_every == 0 && ci + 1 < n_ch) {
                const float4* src = reinterpret_cast<const float4*>(ckpt + (size_t)((ci + 1) / ckpt_every - 1) * (DK * DV)) +
                                    ((size_t)(w * NS) * 64 + lane) * 4;
#pragma unroll
                for (int n = 0; n < NS; ++n)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const float4 v = src[(size_t)n * 256 + q];
                        accNS[n][4 * q] = v.x; accNS[n][4 * q + 1] = v.y; accNS[n][4 * q + 2] = v.z; accNS[n][4 * q + 3] = v.w;
                    }
            }
            const int valid = ntok - (c0 + rb * 32);
            {   // dK^T for key block sb = rb:  dK^T = Q^T dP + R V^T
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
                        acc[n] = mfma(ld_nat(sR, LDV, (cg * NI + n) * 32, kk * 16, lane), bV[kk], acc[n]);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    if (tb >= rb) {
                        f32x16 t = zero16();   // dP[t][s] = dO_t . v_s
#pragma unroll
                        for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sG, LDV, tb * 32, kk * 16, lane), bV[kk], t);
                        bf16x8 t0, t1;
                        if (tb == rb) cvt_tile_masked(t, maskQ, t0, t1);
                        else cvt_tile(t, t0, t1);
#pragma unroll
                        for (int n = 0; n < NI; ++n) {
                            acc[n] = mfma(ld_tr_perm(sQ, LDK, tb * 32, (cg * NI + n) * 32, lane), t0, acc[n]);
                            acc[n] = mfma(ld_tr_perm(sQ, LDK, tb * 32 + 16, (cg * NI + n) * 32, lane), t1, acc[n]);
                        }
                    }
                }
                bf16* rows = dKb + (size_t)(c0 + rb * 32) * ldk;
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    if (DK == 64) stage_tile_T<64>(sSt, rb * 32, (cg * NI + n) * 32, acc[n], lane);
                    else store_tile_T(rows, ldk, (cg * NI + n) * 32, acc[n], valid, lane);
                }
            }
            {   // dV^T for key block sb = rb:  dV^T = dO^T P + R^T K^T
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
                        acc[n] = mfma(ld_tr(sR, LDV, kk * 16, (cg * NJ + n) * 32, lane), bK[kk], acc[n]);
#pragma unroll
                for (int tb = 0; tb < TB; ++tb) {
                    if (tb >= rb) {
                        f32x16 t = zero16();   // P[t][s] = q_t . k_s
#pragma unroll
                        for (int kk = 0; kk < DK / 16; ++kk) t = mfma(ld_nat(sQ, LDK, tb * 32, kk * 16, lane), bK[kk], t);
                        bf16x8 t0, t1;
                        if (tb == rb) cvt_tile_masked(t, maskQ, t0, t1);
                        else cvt_tile(t, t0, t1);
#pragma unroll
                        for (int n = 0; n < NJ; ++n) {
                            acc[n] = mfma(ld_tr_perm(sG, LDV, tb * 32, (cg * NJ + n) * 32, lane), t0, acc[n]);
                            acc[n] = mfma(ld_tr_perm(sG, LDV, tb * 32 + 16, (cg * NJ + n) * 32, lane), t1, acc[n]);
                        }
                    }
                }
                bf16* rows = dVb + (size_t)(c0 + rb * 32) * ldv;
#pragma unroll
                for (int n = 0; n < NJ; ++n) {
                    store_tile_T(rows, ldv, (cg * NJ + n) * 32, acc[n], valid, lane);
                }
            }
            // R^T += dO^T Q (after the segment's first chunk only if the final state is asked for), and S rolled back
            // over this chunk: (-S^T) += V^T K
            if (ci > 0 || R_final != nullptr) {
#pragma unroll
                for (int n = 0; n < NS; ++n) {
                    const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                    for (int s0 = 0; s0 < C; s0 += 16)
                        accRT[n] = mfma(ld_tr(sG, LDV, s0, jb * 32, lane), ld_tr(sQ, LDK, s0, ib * 32, lane), accRT[n]);
                }
            }
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accNS[n] = mfma(ld_tr(sV, LDV, s0, jb * 32, lane), ld_tr(sK, LDK, s0, ib * 32, lane), accNS[n]);
            }
            __syncthreads();            // every wave is done with R (and has staged its 64-wide tile)
            if (DK == 64) flush_stage<C, 64>(sSt, dKb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
            state_to_lds_T<DV, DK, true>(sS, accNS, w, lane);       // S: the state before this chunk
            __syncthreads();
            {   // dQ^T for token block tb = rb:  dQ^T = K^T dP^T + S dO^T
                f32x16 acc[NI];
                bf16x8 bG[DV / 16];
#pragma unroll
                for (int kk = 0; kk < DV / 16; ++kk) bG[kk] = ld_nat(sG, LDV, rb * 32, kk * 16, lane);
#pragma unroll
                for (int n = 0; n < NI; ++n) acc[n] = zero16();
#pragma unroll
                for (int n = 0; n < NI; ++n)
#pragma unroll
                    for (int kk = 0; kk < DV / 16; ++kk)
                        acc[n] = mfma(ld_nat(sS, LDV, (cg * NI + n) * 32, kk * 16, lane), bG[kk], acc[n]);
#pragma unroll
                for (int sb = 0; sb < TB; ++sb) {
                    if (sb <= rb) {
                        f32x16 t = zero16();   // dP^T[s][t] = v_s . dO_t
#pragma unroll
                        for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sV, LDV, sb * 32, kk * 16, lane), bG[kk], t);
                        bf16x8 t0, t1;
                        if (sb == rb) cvt_tile_masked(t, maskK, t0, t1);
                        else cvt_tile(t, t0, t1);
#pragma unroll
                        for (int n = 0; n < NI; ++n) {
                            acc[n] = mfma(ld_tr_perm(sK, LDK, sb * 32, (cg * NI + n) * 32, lane), t0, acc[n]);
                            acc[n] = mfma(ld_tr_perm(sK, LDK, sb * 32 + 16, (cg * NI + n) * 32, lane), t1, acc[n]);
                        }
                    }
                }
                bf16* rows = dQb + (size_t)(c0 + rb * 32) * ldk;
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    // (the staging tile was last read by the flush above, before the barrier that let S in)
                    if (DK == 64) stage_tile_T<64>(sSt, rb * 32, (cg * NI + n) * 32, acc[n], lane);
                    else store_tile_T(rows, ldk, (cg * NI + n) * 32, acc[n], valid, lane);
                }
            }
            __syncthreads();            // tiles, S and the staged dQ are done with
            if (DK == 64) flush_stage<C, 64>(sSt, dQb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
            continue;
        }
        if (ZQK) {
            rq.store_affine(sQ, sAff, sAff + DK, tid);
            rq.store_affine(sK, sAff + 2 * DK, sAff + 3 * DK, tid);
            rq.store(sZ, tid);
        } else {
            rq.store(sQ, tid);
            rk.store(sK, tid);
        }
        rv.store(sV, tid);
        rg.store(sG, tid);
        // R (state after this chunk) is already final: publish it as bf16 [i][j]
        if (!SHARE) state_to_lds_T<DV, DK, false>(sR, accRT, w, lane);
        __syncthreads();
        if (ci > 0) {   // every chunk but a segment's last is complete
            rq.load(Qb + (size_t)(c0 - C) * ldk, ldk, C, tid);
            if (!ZQK) rk.load(Kb + (size_t)(c0 - C) * ldk, ldk, C, tid);
            rv.load(Vb + (size_t)(c0 - C) * ldv, ldv, C, tid);
            rg.load(Gb + (size_t)(c0 - C) * ldv, ldv, C, tid);
        }
        if (ckpt != nullptr && (ci + 1) % ckpt_every == 0 && ci + 1 < n_ch) {
            // the state after this chunk as the first pass left it, in place of the one walked back to here
            const float4* src = reinterpret_cast<const float4*>(ckpt + (size_t)((ci + 1) / ckpt_every - 1) * (DK * DV)) +
                                ((size_t)(w * NS) * 64 + lane) * 4;
#pragma unroll
            for (int n = 0; n < NS; ++n)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 v = src[(size_t)n * 256 + q];
                    accNS[n][4 * q] = v.x; accNS[n][4 * q + 1] = v.y; accNS[n][4 * q + 2] = v.z; accNS[n][4 * q + 3] = v.w;
                }
        }
        // roll S back over this chunk: (-S^T) += V^T K, then publish S (state before this chunk)
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
            for (int s0 = 0; s0 < C; s0 += 16)
                accNS[n] = mfma(ld_tr(sV, LDV, s0, jb * 32, lane), ld_tr(sK, LDK, s0, ib * 32, lane), accNS[n]);
        }
        state_to_lds_T<DV, DK, true>(sS, accNS, w, lane);
        __syncthreads();

        const int valid = ntok - (c0 + rb * 32);   // rows of this wave's 32-token block that exist
        // ---------------- dQ^T for token block tb = rb:  dQ^T = K^T dP^T + S dO^T
        f32x16 accQ[NI];
        {
            f32x16 (&acc)[NI] = accQ;
            bf16x8 bG[DV / 16];
#pragma unroll
            for (int kk = 0; kk < DV / 16; ++kk) bG[kk] = ld_nat(sG, LDV, rb * 32, kk * 16, lane);
#pragma unroll
            for (int n = 0; n < NI; ++n) acc[n] = zero16();
#pragma unroll
            for (int n = 0; n < NI; ++n)
#pragma unroll
                for (int kk = 0; kk < DV / 16; ++kk)
                    acc[n] = mfma(ld_nat(sS, LDV, (cg * NI + n) * 32, kk * 16, lane), bG[kk], acc[n]);
#pragma unroll
            for (int sb = 0; sb < TB; ++sb) {
                if (sb <= rb) {
                    f32x16 t = zero16();   // dP^T[s][t] = v_s . dO_t
#pragma unroll
                    for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sV, LDV, sb * 32, kk * 16, lane), bG[kk], t);
                    bf16x8 t0, t1;
                    if (sb == rb) cvt_tile_masked(t, maskK, t0, t1);
                    else cvt_tile(t, t0, t1);
#pragma unroll
                    for (int n = 0; n < NI; ++n) {
                        acc[n] = mfma(ld_tr_perm(sK, LDK, sb * 32, (cg * NI + n) * 32, lane), t0, acc[n]);
                        acc[n] = mfma(ld_tr_perm(sK, LDK, sb * 32 + 16, (cg * NI + n) * 32, lane), t1, acc[n]);
                    }
                }
            }
            if (!ZQK) {
                bf16* rows = dQb + (size_t)(c0 + rb * 32) * ldk;
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    if (STAGE) stage_tile_T<64>(sOutQ, rb * 32, (cg * NI + n) * 32, acc[n], lane);
                    else store_tile_T(rows, ldk, (cg * NI + n) * 32, acc[n], valid, lane);
                }
            }
        }
        if (SHARE) {
            __syncthreads();            // every wave is done with S ...
            state_to_lds_T<DV, DK, false>(sR, accRT, w, lane);
            __syncthreads();            // ... and R has taken its place
        }
        // ---------------- dK^T for key block sb = rb:  dK^T = Q^T dP + R V^T
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
                    acc[n] = mfma(ld_nat(sR, LDV, (cg * NI + n) * 32, kk * 16, lane), bV[kk], acc[n]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb >= rb) {
                    f32x16 t = zero16();   // dP[t][s] = dO_t . v_s
#pragma unroll
                    for (int kk = 0; kk < DV / 16; ++kk) t = mfma(ld_nat(sG, LDV, tb * 32, kk * 16, lane), bV[kk], t);
                    bf16x8 t0, t1;
                    if (tb == rb) cvt_tile_masked(t, maskQ, t0, t1);
                    else cvt_tile(t, t0, t1);
#pragma unroll
                    for (int n = 0; n < NI; ++n) {
                        acc[n] = mfma(ld_tr_perm(sQ, LDK, tb * 32, (cg * NI + n) * 32, lane), t0, acc[n]);
                        acc[n] = mfma(ld_tr_perm(sQ, LDK, tb * 32 + 16, (cg * NI + n) * 32, lane), t1, acc[n]);
                    }
                }
            }
            if (!ZQK) {
                bf16* rows = dKb + (size_t)(c0 + rb * 32) * ldk;
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    if (STAGE) stage_tile_T<64>(sOutK, rb * 32, (cg * NI + n) * 32, acc[n], lane);
                    else store_tile_T(rows, ldk, (cg * NI + n) * 32, acc[n], valid, lane);
                }
            } else {
                // dZ = alpha_q dQ + alpha_k dK; the lane owns features f0 + 8a + 4h + b of token rb*32 + r
                const int r = lane & 31, h = lane >> 5;
                bf16* rows = dQb + (size_t)(c0 + rb * 32) * ldk;
#pragma unroll
                for (int n = 0; n < NI; ++n) {
                    const int f0 = (cg * NI + n) * 32;
                    f32x16 dz, qz, kz;
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const int f = f0 + 8 * a + 4 * h;
                        const u32x2 zz = *reinterpret_cast<const u32x2*>(sZ + (rb * 32 + r) * LDK + f);
                        const float z[4] = {bf16_lo(zz[0]), bf16_hi(zz[0]), bf16_lo(zz[1]), bf16_hi(zz[1])};
                        const float4 aq = *reinterpret_cast<const float4*>(sAff + f);
                        const float4 ak = *reinterpret_cast<const float4*>(sAff + 2 * DK + f);
                        const float aqv[4] = {aq.x, aq.y, aq.z, aq.w}, akv[4] = {ak.x, ak.y, ak.z, ak.w};
#pragma unroll
                        for (int b = 0; b < 4; ++b) {
                            const int e = 4 * a + b;
                            dz[e] = fmaf(aqv[b], accQ[n][e], akv[b] * acc[n][e]);
                            qz[e] = accQ[n][e] * z[b];
                            kz[e] = acc[n][e] * z[b];
                        }
                    }
                    if (STAGE) stage_tile_T<64>(sOutQ, rb * 32, f0, dz, lane);
                    else store_tile_T(rows, ldk, f0, dz, valid, lane);
                    pg[0][n] += sum_tokens16(qz, lane);
                    pg[1][n] += sum_tokens16(accQ[n], lane);
                    pg[2][n] += sum_tokens16(kz, lane);
                    pg[3][n] += sum_tokens16(acc[n], lane);
                }
            }
        }
        // ---------------- dV^T for key block sb = rb:  dV^T = dO^T P + R^T K^T
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
                    acc[n] = mfma(ld_tr(sR, LDV, kk * 16, (cg * NJ + n) * 32, lane), bK[kk], acc[n]);
#pragma unroll
            for (int tb = 0; tb < TB; ++tb) {
                if (tb >= rb) {
                    f32x16 t = zero16();   // P[t][s] = q_t . k_s
#pragma unroll
                    for (int kk = 0; kk < DK / 16; ++kk) t = mfma(ld_nat(sQ, LDK, tb * 32, kk * 16, lane), bK[kk], t);
                    bf16x8 t0, t1;
                    if (tb == rb) cvt_tile_masked(t, maskQ, t0, t1);
                    else cvt_tile(t, t0, t1);
#pragma unroll
                    for (int n = 0; n < NJ; ++n) {
                        acc[n] = mfma(ld_tr_perm(sG, LDV, tb * 32, (cg * NJ + n) * 32, lane), t0, acc[n]);
                        acc[n] = mfma(ld_tr_perm(sG, LDV, tb * 32 + 16, (cg * NJ + n) * 32, lane), t1, acc[n]);
                    }
                }
            }
            bf16* rows = dVb + (size_t)(c0 + rb * 32) * ldv;
#pragma unroll
            for (int n = 0; n < NJ; ++n) {
                if (STAGE) stage_tile_T<64>(sOutV, rb * 32, (cg * NJ + n) * 32, acc[n], lane);
                else store_tile_T(rows, ldv, (cg * NJ + n) * 32, acc[n], valid, lane);
            }
        }
        // ---------------- R^T += dO^T Q (after the segment's first chunk only if the final state is asked for)
        if (ci > 0 || R_final != nullptr) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, jb = id / IB, ib = id % IB;
#pragma unroll
                for (int s0 = 0; s0 < C; s0 += 16)
                    accRT[n] = mfma(ld_tr(sG, LDV, s0, jb * 32, lane), ld_tr(sQ, LDK, s0, ib * 32, lane), accRT[n]);
            }
        }
        __syncthreads();
        if (STAGE) {
            // the chunk's output tiles are complete in their staging tiles (which are next written after two more
            // barriers): out they go, as whole rows
            flush_stage<C, 64>(sOutQ, dQb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
            if (!ZQK) flush_stage<C, 64>(sOutK, dKb + (size_t)c0 * ldk, ldk, ntok - c0, tid);
            flush_stage<C, 64>(sOutV, dVb + (size_t)c0 * ldv, ldv, ntok - c0, tid);
        }
    }
    if (R_final != nullptr) store_state_T<DV, DK>(R_final, accRT, w, lane);
    if (ZQK) {
        // The loop's last barrier has passed: the tile area is free.  Even lanes hold the sums (odd ones a copy) of
        // feature 32*(cg*NI+n) + 8*(e/4) + 4*h + e%4 with e = 8*b16 + 4*b8 + 2*b4 + b2; the WT waves that share
        // a column group each cover their own tokens, so their shares are added up here.
        float* sP = reinterpret_cast<float*>(lds);          // [WT][4][DK]
        const int r = lane & 31, h = lane >> 5;
        const int e = ((r >> 4) & 1) * 8 + ((r >> 3) & 1) * 4 + ((r >> 2) & 1) * 2 + ((r >> 1) & 1);
        if ((r & 1) == 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q)
#pragma unroll
                for (int n = 0; n < NI; ++n)
                    sP[(rb * 4 + q) * DK + (cg * NI + n) * 32 + 8 * (e >> 2) + 4 * h + (e & 3)] = pg[q][n];
        }
        __syncthreads();
        for (int x = tid; x < 4 * DK; x += 256) {
            float t = 0.f;
#pragma unroll
            for (int v = 0; v < WT; ++v) t += sP[v * 4 * DK + x];
            part[x] = t;
        }
    }
}

// =============================================================================================== kernels
struct SegStateArgs {
    const bf16* X[2];
    const bf16* Y[2];
    float* out[2];
    int skip_seg[2];   // a segment whose total the scan never uses (-1: none)
    // AFF != 0: per pair, the [H][D] rows of alpha and beta that map Z to the affine operand
    const float* alpha[2];
    const float* beta[2];
    int H;
    int reverse[2];    // walk the segment's blocks from its end to its start (same sum)
    int acc_order;     // write the totals in accumulator order, for sweeps that add them up themselves
};

// NH: the tensors are [B,N,H,d] (token rows H * d apart) instead of [B,H,N,d]; args.H is then the head count.
template <int D>
__device__ __forceinline__ size_t row_offset(bool nh, long bh, int H, int N, int p0)
{
    return nh ? ((size_t)(bh / H) * N + p0) * H * D + (size_t)(bh % H) * D : ((size_t)bh * N + p0) * D;
}

// NT: the two tensors are not read again after this kernel (streaming hint on their loads).
// NT1: the hint on the second pair's loads only (see bwd_impl).
template <int DA, int DB, int AFF, bool NH, bool NT, bool NT1 = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((DA == 64 && DB == 64) ? (AFF == 0 ? 6 : 5) : 1)))
void bf16_seg_state_kernel(SegStateArgs args, int N, int seg_len, int n_seg)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[PrepassLds<DA, DB, AFF>::BYTES];
    const int z = blockIdx.z, seg = blockIdx.y;   // heads on grid.x: its limit is 2^31-1, the others' 65535
    const long bh = blockIdx.x;
    if (seg == args.skip_seg[z]) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    const float *al = nullptr, *be = nullptr;
    if (AFF != 0) {
        const size_t hoff = (size_t)(bh % args.H) * (AFF == 1 ? DA : DB);
        al = args.alpha[z] + hoff;
        be = args.beta[z] + hoff;
    }
    if (NT1 && z == 1) {     // (uniform over the workgroup)
        prepass_body<DA, DB, AFF, true>(args.X[z] + row_offset<DA>(NH, bh, args.H, N, p0),
                                        args.Y[z] + row_offset<DB>(NH, bh, args.H, N, p0),
                                        args.out[z] + ((size_t)bh * n_seg + seg) * DA * DB, al, be, NH ? args.H * DA : DA,
                                        NH ? args.H * DB : DB, p1 - p0, lds, tid, w, lane, args.reverse[z] != 0,
                                        args.acc_order != 0);
        return;
    }
    prepass_body<DA, DB, AFF, NT>(args.X[z] + row_offset<DA>(NH, bh, args.H, N, p0),
                                  args.Y[z] + row_offset<DB>(NH, bh, args.H, N, p0),
                                  args.out[z] + ((size_t)bh * n_seg + seg) * DA * DB, al, be, NH ? args.H * DA : DA,
                                  NH ? args.H * DB : DB, p1 - p0, lds, tid, w, lane, args.reverse[z] != 0,
                                  args.acc_order != 0);
}

// (the narrowest shape is asked to stay within the registers that let three workgroups share a compute unit: with its
// staging tile it takes 45 KB of LDS)
template <int C, int DK, int DV, bool ZQK, bool SAVE, bool NH>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu((C == 64 && DK == 64 && DV == 64) ? 3 : 1)))
void bf16_fwd_sweep_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                            const bf16* __restrict__ V, bf16* __restrict__ O,
                                                            const float* __restrict__ S0, float* __restrict__ S_out,
                                                            const float* __restrict__ aff, int H,
                                                            float* __restrict__ saved, int save_every,
                                                            int first_loads_state, int N, int seg_len, int n_seg,
                                                            int fold)
{
    // whole-row streaming stores through a staging tile: every 64-token shape but 128 x 128 (there the tile costs
    // registers the sweep needs: sweep 196 -> 211 us on B1 H16 N65536, which the faster pre-pass behind it does not
    // repay).  The contiguous 64-wide shape gives up its fourth workgroup per unit for the tile and gains all the same
    // (256 .. 1024 sequences of 4096 tokens: 2 .. 10 % faster; the planner never asks for more than two per unit).
    // 128-token chunks at the 64-wide shape take a 16 KB tile (80.9 KB in all, still two per unit): 256 sequences of
    // 4096 tokens 104 -> 91 us.  (The backward sweep with 128-token chunks loses as much in the sweep as the kernels
    // around it gain: left with direct stores.)
    constexpr bool STAGE = (C == 64 && !(DK == 128 && DV == 128)) || (C == 128 && DK == 64 && DV == 64);
    __shared__ __attribute__((aligned(16))) unsigned char
        lds[STAGE ? FwdLds<C, DK, DV, ZQK>::STAGED : FwdLds<C, DK, DV, ZQK>::BYTES];
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    const size_t rk = row_offset<DK>(NH, bh, H, N, p0), rv = row_offset<DV>(NH, bh, H, N, p0);
    // S0: scanned start states (segment 0's slot holds the carried-in state, read only if there is one);
    // S_out: final state of the whole sequence, written by the last segment's workgroup
    const bool has_state = S0 != nullptr && (seg > 0 || first_loads_state);
    // saved: the running state at the end of every save_every-th segment (and of the last one), transposed, for a
    // backward call that walks segments save_every times as long: [bh][ceil(n_seg / save_every)][dv][dk]
    float* save_to = nullptr;
    if (SAVE && saved != nullptr && ((seg + 1) % save_every == 0 || seg == n_seg - 1)) {
        const int n_slots = (n_seg + save_every - 1) / save_every, slot = (seg + save_every) / save_every - 1;
        save_to = saved + ((size_t)bh * n_slots + slot) * DK * DV;
    }
    // fold: S0 holds the segments' own totals (no scan has run): this workgroup adds up those in front of its segment
    const float* s0 = fold ? ((S0 != nullptr && seg > 0) ? S0 + (size_t)bh * n_seg * DK * DV : nullptr)
                           : (has_state ? S0 + ((size_t)bh * n_seg + seg) * DK * DV : nullptr);
    fwd_sweep_body<C, DK, DV, ZQK, SAVE, false, STAGE>(Q + rk, ZQK ? nullptr : K + rk, V + rv, O + rv,
                                   s0, fold ? seg : 1, fold != 0,
                                   (S_out != nullptr && seg == n_seg - 1) ? S_out + (size_t)bh * DK * DV : nullptr,
                                   save_to, ZQK ? aff + (size_t)(bh % H) * DK : nullptr, (size_t)H * DK,
                                   NH ? H * DK : DK, NH ? H * DV : DV, p1 - p0, lds, tid, w, lane);
}

// The forward sweep with the Eq. 9 epilogue: Y = Norm(O) * G; O is written too when it is given.
template <int C, int DK, int DV, bool ZQK, bool SAVE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu((C == 64 && DK == 64 && DV == 64) ? 2 : 1)))
void bf16_fwd_gated_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
                           const bf16* __restrict__ G, bf16* __restrict__ O, bf16* __restrict__ Y, float eps,
                           const float* __restrict__ S0, const float* __restrict__ aff, int H,
                           float* __restrict__ saved, int save_every, int N, int seg_len, int n_seg, int fold)
{
    // Both outputs through staging tiles, as in the plain forward sweep, at the 64-wide shape: 63 KB, two per unit
    // (LM shape 107 -> 100 us, 256 sequences of 4096 tokens 133 -> 110 us).  With one width of 128 the two tiles would
    // leave a unit to a single workgroup (104 KB): measured 7 % slower, so those shapes keep the direct stores.
    constexpr bool STAGE = C == 64 && DK == 64 && DV == 64;
    __shared__ __attribute__((aligned(16))) unsigned char
        lds[STAGE ? FwdLds<C, DK, DV, ZQK, true>::STAGED : FwdLds<C, DK, DV, ZQK, true>::BYTES];
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    const size_t rk = ((size_t)bh * N + p0) * DK, rv = ((size_t)bh * N + p0) * DV;
    float* save_to = nullptr;
    if (SAVE && saved != nullptr && ((seg + 1) % save_every == 0 || seg == n_seg - 1)) {
        const int n_slots = (n_seg + save_every - 1) / save_every, slot = (seg + save_every) / save_every - 1;
        save_to = saved + ((size_t)bh * n_slots + slot) * DK * DV;
    }
    fwd_sweep_body<C, DK, DV, ZQK, SAVE, true, STAGE>(Q + rk, ZQK ? nullptr : K + rk, V + rv, O ? O + rv : nullptr,
                                               (S0 != nullptr && seg > 0)
                                                   ? S0 + ((size_t)bh * n_seg + (fold ? 0 : seg)) * DK * DV : nullptr,
                                               fold ? seg : 1, fold != 0, nullptr, save_to, ZQK ? aff + (size_t)(bh % H) * DK : nullptr,
                                               (size_t)H * DK, DK, DV, p1 - p0, lds, tid, w, lane, G + rv, Y + rv, eps);
}

// (shapes whose LDS footprint lets two workgroups share a compute unit are asked to keep to the 256 registers that
// allows)
template <int C, int DK, int DV, bool ZQK, bool NH>
__global__ __launch_bounds__(256)
__attribute__((amdgpu_waves_per_eu((BwdLds<C, DK, DV, ZQK>::SHARE && BwdLds<C, DK, DV, ZQK>::BYTES <= 81920 && !NH) ? 2 : 1)))
void bf16_bwd_sweep_kernel(const bf16* __restrict__ Q, const bf16* __restrict__ K,
                                                            const bf16* __restrict__ V, const bf16* __restrict__ dO,
                                                            bf16* __restrict__ dQ, bf16* __restrict__ dK,
                                                            bf16* __restrict__ dV, const float* __restrict__ Send,
                                                            const float* __restrict__ Rnext, float* __restrict__ dS_in,
                                                            const float* __restrict__ aff, int H,
                                                            float* __restrict__ part, int N, int seg_len, int n_seg,
                                                            float* ckpt, int ckpt_every, int fold)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[BwdLds<C, DK, DV, ZQK>::BYTES];
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    const size_t rk = row_offset<DK>(NH, bh, H, N, p0), rv = row_offset<DV>(NH, bh, H, N, p0);
    const size_t soff = ((size_t)bh * n_seg + seg) * DK * DV;
    // After a scan: one state each (the scan leaves zeros in the last segment's R slot, so Rnext can be read for every
    // segment).  fold bit 0 / bit 1: Send / Rnext hold the segments' own totals and this workgroup adds up those up
    // to and including its segment / those behind its segment.
    const size_t head = (size_t)bh * n_seg * DK * DV, st = (size_t)DK * DV;
    const float* send = Send ? ((fold & 1) ? Send + head : Send + soff) : nullptr;
    const float* rnext = Rnext ? ((fold & 2) ? (seg + 1 < n_seg ? Rnext + head + (size_t)(seg + 1) * st : nullptr)
                                             : Rnext + soff)
                               : nullptr;
    // dS_in: gradient with respect to the carried-in state = R after the very first chunk (segment 0's workgroup)
    bwd_sweep_body<C, DK, DV, ZQK>(Q + rk, ZQK ? nullptr : K + rk, V + rv, dO + rv, dQ + rk, ZQK ? nullptr : dK + rk,
                                   dV + rv, send, (fold & 1) ? seg + 1 : 1, rnext, (fold & 2) ? n_seg - 1 - seg : 1, fold,
                                   (dS_in != nullptr && seg == 0) ? dS_in + (size_t)bh * DK * DV : nullptr,
                                   ZQK ? aff + (size_t)(bh % H) * DK : nullptr, (size_t)H * DK,
                                   ZQK ? part + ((size_t)bh * n_seg + seg) * 4 * DK : nullptr, NH ? H * DK : DK,
                                   NH ? H * DV : DV, p1 - p0, lds, tid, w, lane,
                                   // (a single segment: N tokens, (n_ch - 1) / ckpt_every copies per (b,h) pair)
                                   (ckpt != nullptr && ckpt_every > 0)
                                       ? ckpt + (size_t)bh * (size_t)(((N + C - 1) / C - 1) / ckpt_every) * DK * DV
                                       : nullptr,
                                   ckpt_every);
}

// Adds up the workgroups' shares of the parameter gradients: part is [B][H][n_seg][4][DK], out is [4][H][DK].
// One workgroup per (head, quantity); thread = (slice of the B * n_seg shares, feature).
template <int DK>
__global__ __launch_bounds__(256) void affine_grad_kernel(const float* __restrict__ part, float* __restrict__ out,
                                                         int B, int H, int n_seg)
{
    constexpr int SL = 256 / DK;
    __shared__ float red[SL][DK];
    const int hq = blockIdx.x, hd = hq / 4, q = hq % 4;
    const int i = threadIdx.x % DK, sl = threadIdx.x / DK;
    const long n_sh = (long)B * n_seg;
    float t = 0.f;
    for (long x = sl; x < n_sh; x += SL) {
        const long b = x / n_seg, seg = x % n_seg;
        t += part[((((size_t)b * H + hd) * n_seg + seg) * 4 + q) * DK + i];
    }
    red[sl][i] = t;
    __syncthreads();
    if (sl == 0) {
#pragma unroll
        for (int v = 1; v < SL; ++v) t += red[v][i];
        out[((size_t)q * H + hd) * DK + i] = t;
    }
}

// =============================================================================================== Eq. 9 epilogue alone
// Y = Norm(O) * G and its gradient on [rows][DV] matrices, Norm(o) = o / sqrt(mean_j o_j^2 + eps): for outputs that
// did not come from the fused forward (the non-causal form) and for every backward pass.  A lane owns 8 consecutive
// features of a row (one 16-byte access per tensor), DV / 8 neighbouring lanes share a row and add up their shares
// with butterfly exchanges; RPT rows per thread are in flight at once.  Streaming work: 3 tensors forward,
// 5 backward, nothing is read twice.
__device__ __forceinline__ void unpack8(const uint4& u, float (&x)[8])
{
    x[0] = bf16_lo(u.x); x[1] = bf16_hi(u.x); x[2] = bf16_lo(u.y); x[3] = bf16_hi(u.y);
    x[4] = bf16_lo(u.z); x[5] = bf16_hi(u.z); x[6] = bf16_lo(u.w); x[7] = bf16_hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float (&x)[8])
{
    return make_uint4(pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7]));
}
template <int LANES>
__device__ __forceinline__ float row_sum(float v)
{
#pragma unroll
    for (int m = 1; m < LANES; m <<= 1) v += __shfl_xor(v, m);
    return v;
}

template <int DV, bool BWD>
__global__ __launch_bounds__(256) void gate_norm_kernel(const bf16* __restrict__ O, const bf16* __restrict__ G,
                                                       const bf16* __restrict__ dY, bf16* __restrict__ out0,
                                                       bf16* __restrict__ out1, float eps, long rows)
{
    constexpr int LPR = DV / 8, RPP = 256 / LPR, RPT = 4;   // lanes per row, rows per pass, rows per thread
    const int sub = threadIdx.x % LPR;
    const long row0 = (long)blockIdx.x * (RPP * RPT) + threadIdx.x / LPR;
    uint4 o[RPT], g[RPT], d[RPT];
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        // rows past the end read the last row (butterflies need every lane); nothing is stored for them
        const long r = min(row0 + (long)i * RPP, rows - 1);
        const size_t off = (size_t)r * DV + 8 * sub;
        o[i] = ldg16<true>(reinterpret_cast<const uint4*>(O + off));     // every input is read exactly once
        g[i] = ldg16<true>(reinterpret_cast<const uint4*>(G + off));
        if (BWD) d[i] = ldg16<true>(reinterpret_cast<const uint4*>(dY + off));
    }
#pragma unroll
    for (int i = 0; i < RPT; ++i) {
        const long r = row0 + (long)i * RPP;
        const size_t off = (size_t)r * DV + 8 * sub;
        float x[8], gg[8], y[8];
        unpack8(o[i], x);
        unpack8(g[i], gg);
        float ss = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) ss = fmaf(x[e], x[e], ss);
        const float rinv = __builtin_amdgcn_rsqf(fmaf(row_sum<LPR>(ss), 1.f / DV, eps));
        if (!BWD) {
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = x[e] * rinv * gg[e];
            // (plain stores: with the streaming hint on these whole-row stores the kernel after it gains where the
            // tensors are small and this kernel loses where they are large -- LM shape -3 %, 256 sequences of 4096
            // tokens +2 % on the two-pass epilogue)
            if (r < rows) *reinterpret_cast<uint4*>(out0 + off) = pack8(y);
        } else {
            // n = r o, u = dY g:  dG = dY n,  dO = r (u - n mean(u n))
            float dy[8], u[8], dg[8];
            unpack8(d[i], dy);
            float un = 0.f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[e] *= rinv;
                u[e] = dy[e] * gg[e];
                dg[e] = dy[e] * x[e];
                un = fmaf(u[e], x[e], un);
            }
            const float m = row_sum<LPR>(un) * (1.f / DV);
#pragma unroll
            for (int e = 0; e < 8; ++e) y[e] = rinv * fmaf(-x[e], m, u[e]);
            if (r < rows) {
                *reinterpret_cast<uint4*>(out0 + off) = pack8(y);
                *reinterpret_cast<uint4*>(out1 + off) = pack8(dg);
            }
        }
    }
}

hipError_t launch_gate_norm(const void* O, const void* G, const void* dY, void* out0, void* out1, float eps, long rows,
                            int dv, hipStream_t st)
{
    const bf16 *o = (const bf16*)O, *g = (const bf16*)G, *d = (const bf16*)dY;
    bf16 *a = (bf16*)out0, *b = (bf16*)out1;
    const bool bwd = dY != nullptr;
    const long rows_per_wg = (256 / (dv / 8)) * 4;
    const dim3 grid((unsigned)((rows + rows_per_wg - 1) / rows_per_wg));
    ProfScope prof(KID_GATE_NORM, st);
    if (dv == 64 && !bwd) hipLaunchKernelGGL((gate_norm_kernel<64, false>), grid, dim3(256), 0, st, o, g, d, a, b, eps, rows);
    else if (dv == 64) hipLaunchKernelGGL((gate_norm_kernel<64, true>), grid, dim3(256), 0, st, o, g, d, a, b, eps, rows);
    else if (dv == 128 && !bwd) hipLaunchKernelGGL((gate_norm_kernel<128, false>), grid, dim3(256), 0, st, o, g, d, a, b, eps, rows);
    else if (dv == 128) hipLaunchKernelGGL((gate_norm_kernel<128, true>), grid, dim3(256), 0, st, o, g, d, a, b, eps, rows);
    else return hipErrorInvalidValue;
    return hipGetLastError();
}

// =============================================================================================== decode step
// One token per (b,h): S += k v^T (fp32, in place), o = S^T q.  q, k: [BH][DK]; v, o: [BH][DV]; S: [BH][DK][DV].
// The state is read and written once: 2 * DK * DV * 4 bytes per token-head, nothing else of note.
// GATE: o leaves as Norm(o) * g (Eq. 9, Norm(o) = o / sqrt(mean_j o_j^2 + eps)), g: [BH][DV].
template <int DK, int DV, bool GATE>
__global__ __launch_bounds__(256) void bf16_step_kernel(const bf16* __restrict__ q, const bf16* __restrict__ k,
                                                       const bf16* __restrict__ v, float* __restrict__ S,
                                                       bf16* __restrict__ o, const bf16* __restrict__ gate, float eps)
{
    constexpr int G = 256 / DV;          // row groups
    constexpr int RPG = DK / G;          // rows of S per thread
    __shared__ float part[G][DV];
    __shared__ float sq[DV / 64];
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, j = tid % DV, g = tid / DV;
    float* s = S + (size_t)bh * DK * DV;
    const float vj = (float)v[bh * DV + j];
    float acc = 0.f;
#pragma unroll 8
    for (int r = 0; r < RPG; ++r) {
        const int i = g * RPG + r;
        const float sn = fmaf((float)k[bh * DK + i], vj, s[i * DV + j]);
        s[i * DV + j] = sn;
        acc = fmaf(sn, (float)q[bh * DK + i], acc);
    }
    part[g][j] = acc;
    __syncthreads();
    float t = 0.f;
    if (g == 0) {                        // the first DV threads (one or two whole waves) hold the output row
#pragma unroll
        for (int gg = 0; gg < G; ++gg) t += part[gg][j];
        if (GATE) {
            float ss = t * t;
#pragma unroll
            for (int m = 32; m > 0; m >>= 1) ss += __shfl_xor(ss, m);
            if ((tid & 63) == 0) sq[tid >> 6] = ss;
        }
    }
    if (GATE) {
        __syncthreads();
        if (g == 0) {
            float tot = 0.f;
#pragma unroll
            for (int x = 0; x < DV / 64; ++x) tot += sq[x];
            t *= __builtin_amdgcn_rsqf(fmaf(tot, 1.f / DV, eps)) * (float)gate[bh * DV + j];
        }
    }
    if (g == 0) o[bh * DV + j] = (bf16)t;
}

hipError_t launch_bf16_step(const void* q, const void* k, const void* v, float* S, void* o, const void* gate, float eps,
                            long BH, int dk, int dv, hipStream_t st)
{
    const bf16 *qq = (const bf16*)q, *kk = (const bf16*)k, *vv = (const bf16*)v, *gg = (const bf16*)gate;
    bf16* oo = (bf16*)o;
    ProfScope prof(KID_STEP_BF16, st);
#define CHELA_STEP(DK_, DV_)                                                                                          \
    if (dk == DK_ && dv == DV_) {                                                                                     \
        if (gate) hipLaunchKernelGGL((bf16_step_kernel<DK_, DV_, true>), dim3((unsigned)BH), dim3(256), 0, st, qq, kk, vv, S, oo, gg, eps); \
        else hipLaunchKernelGGL((bf16_step_kernel<DK_, DV_, false>), dim3((unsigned)BH), dim3(256), 0, st, qq, kk, vv, S, oo, gg, eps);     \
        return hipGetLastError();                                                                                     \
    }
    CHELA_STEP(64, 64) CHELA_STEP(64, 128) CHELA_STEP(128, 64) CHELA_STEP(128, 128)
#undef CHELA_STEP
    return hipErrorInvalidValue;
}

// =============================================================================================== launchers
// Pre-pass + scan over segments.  init[z] (optional, [dk][dv] fp32 per head) seeds the scan of array z.
static int prepass_reverse()
{
    static const int v = [] { const char* e = getenv("CHELA_PREPASS_REV"); return e ? atoi(e) : 1; }();
    return v;
}

// Short rows of segments: the sweep's workgroups add up the segment totals themselves (each reads the totals in front
// of or behind its own segment, which the memory-side cache still holds) and no scan kernel is launched.  That saves
// a launch of about 10 us whose work is latency, and costs every workgroup n/2 state reads at its start: it pays
// while those reads stay small next to the segment's own tiles (measured: 64 x 64 states, 10 segments: step 0.343 ->
// 0.337 ms; 64 x 128, step 0.280 -> 0.265 ms; 128 x 128 states, 16 segments: 0.327 -> 0.332 ms, so not there).
// CHELA_FOLD_SCAN=0 (read per call, a tuning aid) keeps the scan.
static bool fold_scan(const Plan& plan, bool stateful, bool is_bwd = false)
{
    if (stateful || plan.n_seg < 2) return false;
    if ((size_t)plan.n_seg * plan.state_elems * sizeof(float) > kMaxFoldedStateBytes) return false;
    const char* e = getenv("CHELA_FOLD_SCAN");
    const int mode = e ? atoi(e) : 2;          // 0: never, 1: forward calls only, 2: forward and backward calls
    return is_bwd ? mode >= 2 : mode >= 1;
}

template <int DA, int DB, int AFF = 0, bool NH = false, bool NT = false>
static hipError_t run_seg_state(const SegStateArgs& a, int npairs, const int* scan_modes, const float* const* init,
                                bool init_transposed, long BH, int N, const Plan& plan, hipStream_t st,
                                bool do_scan = true, bool stream_second_pair = false)
{
    hipError_t e;
    {
        dim3 grid((unsigned)BH, plan.n_seg, npairs);
        ProfScope prof(KID_SEG_STATE_BF16, st);
        if (AFF == 0 && !NT && stream_second_pair)
            hipLaunchKernelGGL((bf16_seg_state_kernel<DA, DB, AFF == 0 ? 0 : AFF, NH, false, AFF == 0 && !NT>), grid,
                               dim3(256), 0, st, a, N, plan.seg_len, plan.n_seg);
        else
            hipLaunchKernelGGL((bf16_seg_state_kernel<DA, DB, AFF, NH, NT>), grid, dim3(256), 0, st, a, N, plan.seg_len,
                               plan.n_seg);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (!do_scan) return hipSuccess;
    const size_t stride = npairs > 1 ? (size_t)(a.out[1] - a.out[0]) : 0;
    return scan_states(a.out[0], stride, npairs, scan_modes, init, init_transposed ? DB : 0, BH, plan.n_seg, DA * DB, st);
}

// `aff` (Eq. 11-12): non-null selects the kernels that take Z in place of Q and K; it points at the [4][H][DK] fp32
// parameters (alpha_q, beta_q, alpha_k, beta_k).  A carried-in state goes through the scan even when there is a
// single segment.
template <int C, int DK, int DV, bool ZQK, bool NH = false>
static hipError_t fwd_impl(const bf16* Q, const bf16* K, const bf16* V, bf16* O, const float* S_in, float* S_out,
                           const float* aff, int H, float* saved, int save_every, long BH, int N, const Plan& plan,
                           float* ws, hipStream_t st)
{
    hipError_t e;
    const bool use_ws = plan.n_seg > 1 || S_in != nullptr;
    const bool fold = fold_scan(plan, S_in != nullptr);
    if (use_ws) {
        SegStateArgs a{};
        a.X[0] = ZQK ? Q : K; a.Y[0] = V; a.out[0] = ws; a.skip_seg[0] = plan.n_seg - 1;
        a.H = H;
        a.reverse[0] = prepass_reverse();
        a.acc_order = fold ? 1 : 0;
        if (ZQK) { a.alpha[0] = aff + 2 * (size_t)H * DK; a.beta[0] = aff + 3 * (size_t)H * DK; }
        const int mode = SCAN_EXCL_PREFIX;
        const float* init[2] = {S_in, nullptr};
        if ((e = run_seg_state<DK, DV, ZQK ? 1 : 0, NH>(a, 1, &mode, init, false, BH, N, plan, st, !fold)) != hipSuccess)
            return e;
    }
    dim3 grid((unsigned)BH, plan.n_seg);
    ProfScope prof(KID_FWD_SWEEP_BF16, st);
    // the variant that can save boundary states needs a few more registers; the plain call keeps its own kernel
    if (saved != nullptr)
        hipLaunchKernelGGL((bf16_fwd_sweep_kernel<C, DK, DV, ZQK, true, NH>), grid, dim3(256), 0, st, Q, K, V, O,
                           use_ws ? ws : nullptr, S_out, aff, H, saved, save_every, S_in != nullptr ? 1 : 0, N,
                           plan.seg_len, plan.n_seg, fold ? 1 : 0);
    else
        hipLaunchKernelGGL((bf16_fwd_sweep_kernel<C, DK, DV, ZQK, false, NH>), grid, dim3(256), 0, st, Q, K, V, O,
                           use_ws ? ws : nullptr, S_out, aff, H, (float*)nullptr, 1, S_in != nullptr ? 1 : 0, N,
                           plan.seg_len, plan.n_seg, fold ? 1 : 0);
    return hipGetLastError();
}

// Forward with the Eq. 9 epilogue (Y = Norm(O) * G; O optional).  aff non-null: Z stands in for Q and K.
template <int DK, int DV, bool ZQK>
static hipError_t fwd_gated_impl(const bf16* Q, const bf16* K, const bf16* V, const bf16* G, bf16* O, bf16* Y, float eps,
                                 const float* aff, int H, float* saved, int save_every, long BH, int N,
                                 const Plan& plan, float* ws, hipStream_t st)
{
    hipError_t e;
    const bool fold = fold_scan(plan, false);
    if (plan.n_seg > 1) {
        SegStateArgs a{};
        a.X[0] = ZQK ? Q : K; a.Y[0] = V; a.out[0] = ws; a.skip_seg[0] = plan.n_seg - 1;
        a.H = H;
        a.reverse[0] = prepass_reverse();
        a.acc_order = fold ? 1 : 0;
        if (ZQK) { a.alpha[0] = aff + 2 * (size_t)H * DK; a.beta[0] = aff + 3 * (size_t)H * DK; }
        const int mode = SCAN_EXCL_PREFIX;
        const float* init[2] = {nullptr, nullptr};
        if ((e = run_seg_state<DK, DV, ZQK ? 1 : 0, false>(a, 1, &mode, init, false, BH, N, plan, st, !fold)) != hipSuccess)
            return e;
    }
    dim3 grid((unsigned)BH, plan.n_seg);
    ProfScope prof(KID_FWD_SWEEP_BF16, st);
    if (saved != nullptr)
        hipLaunchKernelGGL((bf16_fwd_gated_kernel<64, DK, DV, ZQK, true>), grid, dim3(256), 0, st, Q, K, V, G, O, Y, eps,
                           plan.n_seg > 1 ? ws : nullptr, aff, H, saved, save_every, N, plan.seg_len, plan.n_seg,
                           fold ? 1 : 0);
    else
        hipLaunchKernelGGL((bf16_fwd_gated_kernel<64, DK, DV, ZQK, false>), grid, dim3(256), 0, st, Q, K, V, G, O, Y,
                           eps, plan.n_seg > 1 ? ws : nullptr, aff, H, (float*)nullptr, 1, N, plan.seg_len, plan.n_seg,
                           fold ? 1 : 0);
    return hipGetLastError();
}

// With ZQK, dQ receives dZ, dK is unused and d_aff ([4][H][DK]) the parameter gradients; the workgroups' shares of
// those live behind the two state arrays in the workspace.
template <int C, int DK, int DV, bool ZQK, bool NH = false>
static hipError_t bwd_impl(const bf16* Q, const bf16* K, const bf16* V, const bf16* dO, const float* S_in,
                           const float* dS_out, bf16* dQ, bf16* dK, bf16* dV, float* dS_in, const float* aff,
                           float* d_aff, const float* saved, int B, int H, int N, const Plan& plan, float* ws,
                           hipStream_t st)
{
    hipError_t e;
    const long BH = (long)B * H;
    if (saved != nullptr) {
        // The forward call left the state at the end of every segment of THIS plan ([bh][seg][dv][dk]): only the
        // suffix sums of dO^T Q remain to be built, from dO and Q (or Z) alone.
        float* wsR = ws;
        float* wsP = ZQK ? ws + (plan.n_seg > 1 ? (size_t)BH * plan.n_seg * DK * DV : 0) : nullptr;
        const bool fold_saved = fold_scan(plan, false, true);      // (the saved states are complete; only R is summed)
        if (plan.n_seg > 1) {
            SegStateArgs a{};
            a.X[0] = dO; a.Y[0] = Q; a.out[0] = wsR; a.skip_seg[0] = 0;
            a.H = H;
            a.acc_order = fold_saved ? 1 : 0;
            if (ZQK) { a.alpha[0] = aff; a.beta[0] = aff + (size_t)H * DK; }
            const int mode = SCAN_EXCL_SUFFIX;
            if ((e = run_seg_state<DV, DK, ZQK ? 2 : 0, NH>(a, 1, &mode, nullptr, false, BH, N, plan, st, !fold_saved)) !=
                hipSuccess)
                return e;
        }
        {
            dim3 grid((unsigned)BH, plan.n_seg);
            ProfScope prof(KID_BWD_SWEEP_BF16, st);
            hipLaunchKernelGGL((bf16_bwd_sweep_kernel<C, DK, DV, ZQK, NH>), grid, dim3(256), 0, st, Q, K, V, dO, dQ, dK,
                               dV, saved, plan.n_seg > 1 ? wsR : nullptr, dS_in, aff, H, wsP, N, plan.seg_len,
                               plan.n_seg, (float*)nullptr, 0, fold_saved ? 2 : 0);
            if ((e = hipGetLastError()) != hipSuccess) return e;
        }
        if (ZQK) {
            ProfScope prof(KID_AFFINE_GRAD, st);
            hipLaunchKernelGGL((affine_grad_kernel<DK>), dim3(4 * H), dim3(256), 0, st, wsP, d_aff, B, H, plan.n_seg);
            e = hipGetLastError();
        }
        return e;
    }
    const bool use_ws = plan.n_seg > 1 || S_in != nullptr || dS_out != nullptr;
    const bool fold = fold_scan(plan, S_in != nullptr || dS_out != nullptr, true);
    const size_t state_floats = use_ws ? (size_t)BH * plan.n_seg * DK * DV : 0;
    // a single segment that is long: copies of the running state at the workspace's start (see bwd_sweep_body)
    const long n_ckpt = use_ws ? 0 : plan_n_ckpt(plan, N);
    float* wsS = ws;
    float* wsR = ws ? ws + state_floats : nullptr;
    float* wsP = ZQK ? ws + (use_ws ? 2 * state_floats : (size_t)BH * n_ckpt * DK * DV) : nullptr;
    if (use_ws) {
        SegStateArgs a{};
        // S^T totals: every segment is needed (inclusive prefix); R^T totals: the first is never used (exclusive suffix)
        a.X[0] = V;  a.Y[0] = ZQK ? Q : K; a.out[0] = wsS; a.skip_seg[0] = -1;
        a.X[1] = dO; a.Y[1] = Q;           a.out[1] = wsR; a.skip_seg[1] = 0;
        a.H = H;
        a.acc_order = fold ? 1 : 0;
        // The sweep re-reads all four tensors right after this pre-pass.  Once they no longer fit the memory-side
        // cache together, dO and Q are read with the streaming hint, here and in the sweep, so that K and V stay in it
        // whole instead of all four fighting for it: LM shape (403 MB) 0.292 -> 0.283 ms per step, backward sweep
        // 140 -> 130.5 us; 0.298 -> 0.293 ms on three sets of tensors used in turn.
        const bool stream_dO_Q = !ZQK && (size_t)BH * N * (2 * DK + 2 * DV) * sizeof(bf16) > kStreamPairAboveBytes;
        if (ZQK) {
            a.alpha[0] = aff + 2 * (size_t)H * DK; a.beta[0] = aff + 3 * (size_t)H * DK;   // K
            a.alpha[1] = aff;                      a.beta[1] = aff + (size_t)H * DK;       // Q
        }
        const int modes[2] = {SCAN_INCL_PREFIX, SCAN_EXCL_SUFFIX};
        const float* init[2] = {S_in, dS_out};   // given as [dk][dv]; the arrays are [dv][dk]
        if ((e = run_seg_state<DV, DK, ZQK ? 2 : 0, NH>(a, 2, modes, init, true, BH, N, plan, st, !fold, stream_dO_Q)) !=
            hipSuccess)
            return e;
    }
    {
        dim3 grid((unsigned)BH, plan.n_seg);
        ProfScope prof(KID_BWD_SWEEP_BF16, st);
        hipLaunchKernelGGL((bf16_bwd_sweep_kernel<C, DK, DV, ZQK, NH>), grid, dim3(256), 0, st, Q, K, V, dO, dQ, dK, dV,
                           use_ws ? wsS : nullptr, use_ws ? wsR : nullptr, dS_in, aff, H, wsP, N, plan.seg_len,
                           plan.n_seg, n_ckpt > 0 ? ws : nullptr, n_ckpt > 0 ? plan.ckpt_every : 0, fold ? 3 : 0);
        if ((e = hipGetLastError()) != hipSuccess) return e;
    }
    if (ZQK) {
        ProfScope prof(KID_AFFINE_GRAD, st);
        hipLaunchKernelGGL((affine_grad_kernel<DK>), dim3(4 * H), dim3(256), 0, st, wsP, d_aff, B, H, plan.n_seg);
        e = hipGetLastError();
    }
    return e;
}

// =============================================================================================== non-causal form
// Eq. 2 as written, O = Q (K^T V): no mask, so the state is one matrix per (b,h) -- the total of the pre-pass -- and
// every block of tokens is independent.  Y[t][:] = X[t][:] M for the tokens of one workgroup, M a [DA][DB] fp32
// matrix per head, given either as it is (M_IS_T = false) or transposed, [DB][DA] (true).  The matrix becomes the
// A operand (M^T, bf16, read from LDS once and kept in registers), a 64-token tile of X the B operand, the result
// tile is Y^T and leaves through 16-byte stores.  The X tile is double-buffered in LDS: one barrier per chunk.
template <int DA, int DB, bool GATE = false>
struct ApplyLds {
    static constexpr int LDA = DA + PAD;
    static constexpr int TILES = (2 * 64 * LDA + DB * LDA) * 2;
    static constexpr int SUMS = GATE ? 2 * 2 * 64 * 4 : 0;                  // [2][2][64] floats
    // not gated, 64 features out: the output leaves as whole rows through two staging tiles used in turn
    static constexpr bool STAGE = !GATE && DB == 64;
    static constexpr int BYTES = TILES + SUMS + (GATE ? 2 * 64 * (DB + PAD) * 2 : 0)    // + two gate tiles
                                 + (STAGE ? 2 * 64 * 64 * 2 : 0);
};

// GATE (Eq. 9): Yg = Norm(Y) * G with Norm(y) = y / sqrt(mean_j y_j^2 + eps) over the DB features of a token; Y itself
// is then optional.  The two waves that share a token block leave their shares of the sum of squares in LDS (two
// sets, used in turn) and the gated tile of chunk c leaves after the barrier of chunk c + 1, so the kernel still
// meets at one barrier per chunk.
template <int DA, int DB, bool M_IS_T, bool GATE>
__global__ __launch_bounds__(256) void bf16_apply_state_kernel(const bf16* __restrict__ X, bf16* __restrict__ Y,
                                                              const float* __restrict__ M, size_t m_stride, int N,
                                                              int rows_per_wg, const bf16* __restrict__ G,
                                                              bf16* __restrict__ Yg, float eps)
{
    constexpr int C = 64, LDA = DA + PAD;
    constexpr int JB = DB / 32, NJ = JB / 2;
    __shared__ __attribute__((aligned(16))) unsigned char lds[ApplyLds<DA, DB, GATE>::BYTES];
    bf16* sX = reinterpret_cast<bf16*>(lds);          // two buffers of C x LDA
    bf16* sMT = sX + 2 * C * LDA;                      // M^T: [DB][LDA]
    float* sSq = reinterpret_cast<float*>(lds + ApplyLds<DA, DB, false>::TILES);   // GATE: [2][2][C]
    constexpr int LDB = DB + PAD;
    bf16* sG = reinterpret_cast<bf16*>(lds + ApplyLds<DA, DB, false>::TILES + ApplyLds<DA, DB, true>::SUMS);   // [2][C][LDB]
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tb = w % 2, jg = w / 2;
    const int p0 = blockIdx.y * rows_per_wg, p1 = min(N, p0 + rows_per_wg), ntok = p1 - p0;
    const bf16* Xb = X + ((size_t)bh * N + p0) * DA;
    bf16* Yb = Y ? Y + ((size_t)bh * N + p0) * DB : nullptr;
    const bf16* Gb = GATE ? G + ((size_t)bh * N + p0) * DB : nullptr;
    bf16* Ygb = GATE ? Yg + ((size_t)bh * N + p0) * DB : nullptr;
    const float4* M4 = reinterpret_cast<const float4*>(M + (size_t)bh * m_stride);

    TileRegs<C, DA, true> rx;   // X is read here for the last time: streaming loads
    TileRegs<C, DB, true> rg;   // GATE: the gate tile travels like X (full lines in, LDS, then the order the tile is stored in)
    rx.load(Xb, DA, ntok, tid);
    if (GATE) rg.load(Gb, DB, ntok, tid);
    for (int x = tid; x < DA * DB / 4; x += 256) {
        const float4 v = M4[x];
        if (M_IS_T) {
            const int j = (4 * x) / DA, i = (4 * x) % DA;
            u32x2 pk;
            pk[0] = pack2(v.x, v.y);
            pk[1] = pack2(v.z, v.w);
            *reinterpret_cast<u32x2*>(sMT + j * LDA + i) = pk;
        } else {
            const int i = (4 * x) / DB, j = (4 * x) % DB;
            sMT[(j + 0) * LDA + i] = (bf16)v.x;
            sMT[(j + 1) * LDA + i] = (bf16)v.y;
            sMT[(j + 2) * LDA + i] = (bf16)v.z;
            sMT[(j + 3) * LDA + i] = (bf16)v.w;
        }
    }
    __syncthreads();
    bf16x8 aM[NJ][DA / 16];
#pragma unroll
    for (int n = 0; n < NJ; ++n)
#pragma unroll
        for (int kk = 0; kk < DA / 16; ++kk) aM[n][kk] = ld_nat(sMT, LDA, (jg * NJ + n) * 32, kk * 16, lane);

    // GATE: the tile of the previous chunk, its gate and where it goes, waiting for that chunk's sums of squares
    f32x16 held[GATE ? NJ : 1];
    uint4 gate[GATE ? NJ : 1][2];
    int held_c0 = -1;
    auto flush = [&](int par) __attribute__((always_inline)) {
        float tot = sSq[(par * 2 + 0) * C + tb * 32 + (lane & 31)] + sSq[(par * 2 + 1) * C + tb * 32 + (lane & 31)];
        const float rinv = __builtin_amdgcn_rsqf(fmaf(tot, 1.f / DB, eps));
        bf16* rows = Ygb + (size_t)(held_c0 + tb * 32) * DB;
        const int valid = ntok - (held_c0 + tb * 32);
#pragma unroll
        for (int n = 0; n < NJ; ++n)
            store_tile_T(rows, DB, (jg * NJ + n) * 32, gate_tile(held[n], gate[n], rinv), valid, lane);
    };

    constexpr bool STAGE = ApplyLds<DA, DB, GATE>::STAGE;
    bf16* sOut = reinterpret_cast<bf16*>(lds + ApplyLds<DA, DB, false>::TILES);      // STAGE: [2][C][64]
    int buf = 0;
    for (int c0 = 0; c0 < ntok; c0 += C, buf ^= 1) {
        bf16* sXb = sX + buf * C * LDA;
        rx.store(sXb, tid);
        if (GATE) rg.store(sG + buf * C * LDB, tid);
        __syncthreads();
        if (GATE && held_c0 >= 0) flush(buf ^ 1);      // the previous chunk's sums are complete now
        if (STAGE && c0 > 0)                            // the previous chunk's tile is complete in its staging tile
            flush_stage<C, 64>(sOut + (buf ^ 1) * C * 64, Yb + (size_t)(c0 - C) * DB, DB, C, tid);
        if (c0 + C < ntok) {
            rx.load(Xb + (size_t)(c0 + C) * DA, DA, ntok - c0 - C, tid);
            if (GATE) rg.load(Gb + (size_t)(c0 + C) * DB, DB, ntok - c0 - C, tid);
        }
        if (GATE) {
            const bf16* g = sG + buf * C * LDB + (tb * 32 + (lane & 31)) * LDB + 8 * (lane >> 5);
#pragma unroll
            for (int n = 0; n < NJ; ++n)
#pragma unroll
                for (int ap = 0; ap < 2; ++ap)
                    gate[n][ap] = *reinterpret_cast<const uint4*>(g + (jg * NJ + n) * 32 + 16 * ap);
        }
        f32x16 acc[NJ];
#pragma unroll
        for (int n = 0; n < NJ; ++n) acc[n] = zero16();
#pragma unroll
        for (int kk = 0; kk < DA / 16; ++kk) {
            const bf16x8 bX = ld_nat(sXb, LDA, tb * 32, kk * 16, lane);
#pragma unroll
            for (int n = 0; n < NJ; ++n) acc[n] = mfma(aM[n][kk], bX, acc[n]);
        }
        if (STAGE) {
#pragma unroll
            for (int n = 0; n < NJ; ++n) stage_tile_T<64>(sOut + buf * C * 64, tb * 32, (jg * NJ + n) * 32, acc[n], lane);
        } else if (!GATE || Yb != nullptr) {
            bf16* rows = Yb + (size_t)(c0 + tb * 32) * DB;
            const int valid = ntok - (c0 + tb * 32);
#pragma unroll
            for (int n = 0; n < NJ; ++n) store_tile_T(rows, DB, (jg * NJ + n) * 32, acc[n], valid, lane);
        }
        if (GATE) {
            float ss = 0.f;
#pragma unroll
            for (int n = 0; n < NJ; ++n) {
                held[n] = acc[n];
#pragma unroll
                for (int e = 0; e < 16; ++e) ss = fmaf(acc[n][e], acc[n][e], ss);
            }
            const unsigned sb = __builtin_bit_cast(unsigned, ss);
            const u32x2 sw = __builtin_amdgcn_permlane32_swap(sb, sb, false, false);
            const unsigned sw0 = sw[0], sw1 = sw[1];
            if (lane < 32)
                sSq[(buf * 2 + jg) * C + tb * 32 + lane] = __builtin_bit_cast(float, sw0) + __builtin_bit_cast(float, sw1);
            held_c0 = c0;
        }
    }
    if (GATE && held_c0 >= 0) {
        __syncthreads();
        flush(buf ^ 1);
    }
    if (STAGE && ntok > 0) {
        __syncthreads();
        const int last = (ntok - 1) / C * C;
        flush_stage<C, 64>(sOut + (buf ^ 1) * C * 64, Yb + (size_t)last * DB, DB, ntok - last, tid);
    }
}

constexpr int kApplyRows = 512;   // tokens per workgroup of the apply kernel

template <int DA, int DB, bool M_IS_T>
static hipError_t run_apply(const bf16* X, bf16* Y, const float* M, size_t m_stride, long BH, int N, hipStream_t st,
                            const bf16* G = nullptr, bf16* Yg = nullptr, float eps = 0.f)
{
    dim3 grid((unsigned)BH, (N + kApplyRows - 1) / kApplyRows);
    ProfScope prof(KID_APPLY_BF16, st);
    if (G != nullptr)
        hipLaunchKernelGGL((bf16_apply_state_kernel<DA, DB, M_IS_T, true>), grid, dim3(256), 0, st, X, Y, M, m_stride, N,
                           kApplyRows, G, Yg, eps);
    else
        hipLaunchKernelGGL((bf16_apply_state_kernel<DA, DB, M_IS_T, false>), grid, dim3(256), 0, st, X, Y, M, m_stride,
                           N, kApplyRows, G, Yg, eps);
    return hipGetLastError();
}

// plan.n_seg / seg_len describe the pre-pass split here; the totals end up in the last segment's slot.
template <int DK, int DV>
static hipError_t noncausal_fwd_impl(const bf16* Q, const bf16* K, const bf16* V, bf16* O, long BH, int N,
                                     const Plan& plan, float* ws, hipStream_t st, const bf16* G = nullptr,
                                     bf16* Y = nullptr, float eps = 0.f)
{
    hipError_t e;
    SegStateArgs a{};
    a.X[0] = V; a.Y[0] = K; a.out[0] = ws; a.skip_seg[0] = -1;       // S^T = V^T K, [dv][dk]
    const int mode = SCAN_INCL_PREFIX;
    // (K and V are not read again in this call: streaming loads)
    if ((e = run_seg_state<DV, DK, 0, false, true>(a, 1, &mode, nullptr, false, BH, N, plan, st, plan.n_seg > 1)) != hipSuccess)
        return e;
    const size_t el = (size_t)DK * DV;
    return run_apply<DK, DV, true>(Q, O, ws + (size_t)(plan.n_seg - 1) * el, plan.n_seg * el, BH, N, st, G, Y, eps);
}

template <int DK, int DV>
static hipError_t noncausal_bwd_impl(const bf16* Q, const bf16* K, const bf16* V, const bf16* dO, bf16* dQ, bf16* dK,
                                     bf16* dV, long BH, int N, const Plan& plan, float* ws, hipStream_t st)
{
    hipError_t e;
    const size_t el = (size_t)DK * DV, arr = (size_t)BH * plan.n_seg * el;
    float* wsS = ws;            // S^T = V^T K   [dv][dk]
    float* wsR = ws + arr;      // R^T = dO^T Q  [dv][dk]
    SegStateArgs a{};
    a.X[0] = V;  a.Y[0] = K; a.out[0] = wsS; a.skip_seg[0] = -1;
    a.X[1] = dO; a.Y[1] = Q; a.out[1] = wsR; a.skip_seg[1] = -1;
    const int modes[2] = {SCAN_INCL_PREFIX, SCAN_INCL_PREFIX};
    // (as in the causal backward: once the four tensors exceed the memory-side cache, dO and Q go through it with the
    // streaming hint, so that V and K are still there for the second and third of the kernels below)
    const bool stream_dO_Q = (size_t)BH * N * (2 * DK + 2 * DV) * sizeof(bf16) > kStreamPairAboveBytes;
    if ((e = run_seg_state<DV, DK>(a, 2, modes, nullptr, false, BH, N, plan, st, plan.n_seg > 1, stream_dO_Q)) != hipSuccess)
        return e;
    const size_t last = (size_t)(plan.n_seg - 1) * el, stride = plan.n_seg * el;
    // dQ = dO S^T, dK = V R^T, dV = K R
    if ((e = run_apply<DV, DK, false>(dO, dQ, wsS + last, stride, BH, N, st)) != hipSuccess) return e;
    if ((e = run_apply<DV, DK, false>(V, dK, wsR + last, stride, BH, N, st)) != hipSuccess) return e;
    return run_apply<DK, DV, true>(K, dV, wsR + last, stride, BH, N, st);
}

hipError_t launch_bf16_noncausal_fwd(const void* Q, const void* K, const void* V, void* O, long BH, int N, int dk,
                                     int dv, const Plan& plan, float* ws, hipStream_t st, const void* G, void* Y,
                                     float eps)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)G;
    bf16 *o = (bf16*)O, *y = (bf16*)Y;
    if (dk == 64 && dv == 64) return noncausal_fwd_impl<64, 64>(q, k, v, o, BH, N, plan, ws, st, g, y, eps);
    if (dk == 64 && dv == 128) return noncausal_fwd_impl<64, 128>(q, k, v, o, BH, N, plan, ws, st, g, y, eps);
    if (dk == 128 && dv == 64) return noncausal_fwd_impl<128, 64>(q, k, v, o, BH, N, plan, ws, st, g, y, eps);
    if (dk == 128 && dv == 128) return noncausal_fwd_impl<128, 128>(q, k, v, o, BH, N, plan, ws, st, g, y, eps);
    return hipErrorInvalidValue;
}

hipError_t launch_bf16_noncausal_bwd(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK,
                                     void* dV, long BH, int N, int dk, int dv, const Plan& plan, float* ws,
                                     hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)dO;
    bf16 *dq = (bf16*)dQ, *dkk = (bf16*)dK, *dvv = (bf16*)dV;
    if (dk == 64 && dv == 64) return noncausal_bwd_impl<64, 64>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st);
    if (dk == 64 && dv == 128) return noncausal_bwd_impl<64, 128>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st);
    if (dk == 128 && dv == 64) return noncausal_bwd_impl<128, 64>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st);
    if (dk == 128 && dv == 128) return noncausal_bwd_impl<128, 128>(q, k, v, g, dq, dkk, dvv, BH, N, plan, ws, st);
    return hipErrorInvalidValue;
}

#define CHELA_DISPATCH(C_, DK_, DV_, CALL)                                  \
    if (plan.chunk == C_ && dk == DK_ && dv == DV_) return CALL;

hipError_t launch_bf16_fwd(const void* Q, const void* K, const void* V, void* O, const float* S_in, float* S_out,
                           float* saved, int save_every, long BH, int N, int dk, int dv, const Plan& plan, float* ws,
                           hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V;
    bf16* o = (bf16*)O;
#define CHELA_FWD(C_, DK_, DV_)                                                                                       \
    CHELA_DISPATCH(C_, DK_, DV_, (fwd_impl<C_, DK_, DV_, false>(q, k, v, o, S_in, S_out, nullptr, 1, saved, save_every, \
                                                                BH, N, plan, ws, st)))
    CHELA_FWD(64, 64, 64) CHELA_FWD(128, 64, 64) CHELA_FWD(64, 64, 128) CHELA_FWD(128, 64, 128)
    CHELA_FWD(64, 128, 64) CHELA_FWD(128, 128, 64) CHELA_FWD(64, 128, 128) CHELA_FWD(128, 128, 128)
#undef CHELA_FWD
    return hipErrorInvalidValue;
}

hipError_t launch_bf16_bwd(const void* Q, const void* K, const void* V, const void* dO, const float* S_in,
                           const float* dS_out, void* dQ, void* dK, void* dV, float* dS_in, const float* saved,
                           long BH, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)dO;
    bf16 *dq = (bf16*)dQ, *dkk = (bf16*)dK, *dvv = (bf16*)dV;
#define CHELA_BWD(C_, DK_, DV_)                                                                                       \
    CHELA_DISPATCH(C_, DK_, DV_, (bwd_impl<C_, DK_, DV_, false>(q, k, v, g, S_in, dS_out, dq, dkk, dvv, dS_in, nullptr, \
                                                                nullptr, saved, (int)BH, 1, N, plan, ws, st)))
    CHELA_BWD(64, 64, 64) CHELA_BWD(128, 64, 64) CHELA_BWD(64, 64, 128) CHELA_BWD(64, 128, 64) CHELA_BWD(64, 128, 128)
#undef CHELA_BWD
    return hipErrorInvalidValue;
}

// [B,N,H,d] tensors (heads next to each other inside a token row), 64-token chunks, no carried or saved states.
hipError_t launch_bf16_fwd_nh(const void* Q, const void* K, const void* V, void* O, int B, int H, int N, int dk, int dv,
                              const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V;
    bf16* o = (bf16*)O;
    const long BH = (long)B * H;
#define CHELA_FWD_NH(DK_, DV_)                                                                                        \
    CHELA_DISPATCH(64, DK_, DV_, (fwd_impl<64, DK_, DV_, false, true>(q, k, v, o, nullptr, nullptr, nullptr, H, nullptr, \
                                                                      1, BH, N, plan, ws, st)))
    CHELA_FWD_NH(64, 64) CHELA_FWD_NH(64, 128) CHELA_FWD_NH(128, 64) CHELA_FWD_NH(128, 128)
#undef CHELA_FWD_NH
    return hipErrorInvalidValue;
}

hipError_t launch_bf16_bwd_nh(const void* Q, const void* K, const void* V, const void* dO, void* dQ, void* dK, void* dV,
                              int B, int H, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)dO;
    bf16 *dq = (bf16*)dQ, *dkk = (bf16*)dK, *dvv = (bf16*)dV;
#define CHELA_BWD_NH(DK_, DV_)                                                                                         \
    CHELA_DISPATCH(64, DK_, DV_, (bwd_impl<64, DK_, DV_, false, true>(q, k, v, g, nullptr, nullptr, dq, dkk, dvv, nullptr, \
                                                                      nullptr, nullptr, nullptr, B, H, N, plan, ws, st)))
    CHELA_BWD_NH(64, 64) CHELA_BWD_NH(64, 128) CHELA_BWD_NH(128, 64) CHELA_BWD_NH(128, 128)
#undef CHELA_BWD_NH
    return hipErrorInvalidValue;
}

// Eq. 9 epilogue fused into the forward; aff non-null selects the Eq. 11-12 prologue as well.  64-token chunks.
hipError_t launch_bf16_fwd_gated(const void* Q, const void* K, const void* V, const void* G, void* O, void* Y, float eps,
                                 const float* aff, float* saved, int save_every, int B, int H, int N, int dk, int dv,
                                 const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *q = (const bf16*)Q, *k = (const bf16*)K, *v = (const bf16*)V, *g = (const bf16*)G;
    bf16 *o = (bf16*)O, *y = (bf16*)Y;
    const long BH = (long)B * H;
#define CHELA_GFWD(DK_, DV_)                                                                                               if (dk == DK_ && dv == DV_)                                                                                                return aff ? fwd_gated_impl<DK_, DV_, true>(q, nullptr, v, g, o, y, eps, aff, H, saved, save_every, BH, N, plan,                                                     ws, st)                                                                               : fwd_gated_impl<DK_, DV_, false>(q, k, v, g, o, y, eps, nullptr, H, saved, save_every, BH, N, plan,                                                      ws, st);
    CHELA_GFWD(64, 64) CHELA_GFWD(64, 128) CHELA_GFWD(128, 64) CHELA_GFWD(128, 128)
#undef CHELA_GFWD
    return hipErrorInvalidValue;
}

// Eq. 11-12 variants: Z in place of Q and K, 64-token chunks.
hipError_t launch_bf16_zfwd(const void* Z, const float* aff, const void* V, void* O, float* saved, int save_every,
                            int B, int H, int N, int dk, int dv, const Plan& plan, float* ws, hipStream_t st)
{
    const bf16 *z = (const bf16*)Z, *v = (const bf16*)V;
    bf16* o = (bf16*)O;
    const long BH = (long)B * H;
#define CHELA_ZFWD(DK_, DV_) \
    CHELA_DISPATCH(64, DK_, DV_, (fwd_impl<64, DK_, DV_, true>(z, nullptr, v, o, nullptr, nullptr, aff, H, saved, save_every, BH, N, plan, ws, st)))
    CHELA_ZFWD(64, 64) CHELA_ZFWD(64, 128) CHELA_ZFWD(128, 64) CHELA_ZFWD(128, 128)
#undef CHELA_ZFWD
    return hipErrorInvalidValue;
}

hipError_t launch_bf16_zbwd(const void* Z, const float* aff, const void* V, const void* dO, void* dZ, float* d_aff,
                            void* dV, const float* saved, int B, int H, int N, int dk, int dv, const Plan& plan,
                            float* ws, hipStream_t st)
{
    const bf16 *z = (const bf16*)Z, *v = (const bf16*)V, *g = (const bf16*)dO;
    bf16 *dz = (bf16*)dZ, *dvv = (bf16*)dV;
#define CHELA_ZBWD(DK_, DV_)                                                                                       \
    CHELA_DISPATCH(64, DK_, DV_, (bwd_impl<64, DK_, DV_, true>(z, nullptr, v, g, nullptr, nullptr, dz, nullptr, dvv, \
                                                               nullptr, aff, d_aff, saved, B, H, N, plan, ws, st)))
    CHELA_ZBWD(64, 64) CHELA_ZBWD(64, 128) CHELA_ZBWD(128, 64) CHELA_ZBWD(128, 128)
#undef CHELA_ZBWD
    return hipErrorInvalidValue;
}

}  // namespace chela
