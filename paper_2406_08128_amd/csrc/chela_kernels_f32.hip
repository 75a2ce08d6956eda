// fp32 kernels: causal linear attention with fp32 I/O and fp32 arithmetic on the fp32 matrix instruction
// v_mfma_f32_32x32x2_f32 (products and sums in IEEE fp32; the path exists for accuracy, the bf16 path for speed).
// Also the state scan and the copy probe shared by both paths.
//
// Structure (Sec. 4.1): a (b,h) sequence is cut into segments; within a segment one workgroup walks the
// chunks in order with the d_k x d_v state S in accumulator registers.  Per chunk: masked left product
// P = (Q K^T) o M, O = P V + Q S (both parts summed in the same accumulators), then S += K^T V.  Segment start
// states come from a pre-pass (segment totals of K^T V) and a scan over segments.
//
// Operand plumbing is simpler than in the bf16 kernels: with k = 2 per instruction a lane supplies ONE float of A
// (row lane%32, k = lane/32) and ONE of B, so every operand is a 4-byte LDS read -- along a row of a row-major tile
// (stride = leading dimension, kept odd so the 32 rows fall into 32 different banks) or along its columns
// (contiguous).  Nothing is ever transposed.
#include "chela_internal.h"

namespace chela {

// ------------------------------------------------------------------------------------------------ scan
// states[z][bh][seg][e] (z = 0 .. n_arrays-1, arrays `array_stride` floats apart), one thread per (z, bh, 4 e's),
// serial over the (few) segments, coalesced over e.  The loads of U segments are issued before the first add so that
// one memory round trip serves U segments.
// An optional carried-in state seeds the running sum of array z: init[z] is [rows][cols] fp32 per head; if
// init_cols > 0 the array itself is stored transposed ([cols][rows], cols = init_cols... see below) and the seed is
// read transposed: element e = a * init_cols + b of the array takes init[b * (elems / init_cols) + a].
struct ScanModes { int mode[2]; const float* init[2]; };

__global__ __launch_bounds__(256) void scan_states_kernel(float* __restrict__ st, size_t array_stride, int n_seg,
                                                         int elems, ScanModes modes, int init_cols)
{
    const long bh = blockIdx.x;     // heads on grid.x: its limit is 2^31-1, the others' 65535
    const int z = blockIdx.z;
    const int mode = modes.mode[z];
    const int e = (blockIdx.y * 256 + threadIdx.x) * 4;
    if (e >= elems) return;
    float* p = st + (size_t)z * array_stride + (size_t)bh * n_seg * elems + e;
    float4 run = make_float4(0.f, 0.f, 0.f, 0.f);
    if (modes.init[z] != nullptr) {
        const float* in = modes.init[z] + (size_t)bh * elems;
        if (init_cols > 0) {
            const int a = e / init_cols, b = e % init_cols, rows = elems / init_cols;   // 4 consecutive b, one a
            run = make_float4(in[(size_t)b * rows + a], in[(size_t)(b + 1) * rows + a], in[(size_t)(b + 2) * rows + a],
                              in[(size_t)(b + 3) * rows + a]);
        } else {
            run = *reinterpret_cast<const float4*>(in + e);
        }
    }
    constexpr int U = 16;                      // segments in flight per thread
    const bool suffix = (mode == SCAN_EXCL_SUFFIX);
    for (int s0 = 0; s0 < n_seg; s0 += U) {
        float4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + u;
            const int idx = suffix ? (n_seg - 1 - s) : s;
            v[u] = s < n_seg ? *reinterpret_cast<const float4*>(p + (size_t)idx * elems) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int s = s0 + u;
            if (s < n_seg) {
                const int idx = suffix ? (n_seg - 1 - s) : s;
                float4* dst = reinterpret_cast<float4*>(p + (size_t)idx * elems);
                if (mode == SCAN_INCL_PREFIX) {
                    run.x += v[u].x; run.y += v[u].y; run.z += v[u].z; run.w += v[u].w;
                    *dst = run;
                } else {
                    *dst = run;
                    run.x += v[u].x; run.y += v[u].y; run.z += v[u].z; run.w += v[u].w;
                }
            }
        }
    }
}

hipError_t scan_states(float* states, size_t array_stride, int n_arrays, const int* modes, const float* const* init,
                       int init_cols, long BH, int n_seg, int elems, hipStream_t st)
{
    ScanModes m{};
    for (int z = 0; z < n_arrays && z < 2; ++z) { m.mode[z] = modes[z]; m.init[z] = init ? init[z] : nullptr; }
    dim3 grid((unsigned)BH, (elems / 4 + 255) / 256, n_arrays);
    ProfScope prof(KID_SCAN, st);
    hipLaunchKernelGGL(scan_states_kernel, grid, dim3(256), 0, st, states, array_stride, n_seg, elems, m, init_cols);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ copy probe
// Grid-stride 16-byte copy: the plain streaming kernel that byte counters are calibrated against.
__global__ __launch_bounds__(256) void copy_probe_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n)
{
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_copy(const void* src, void* dst, size_t bytes, hipStream_t st)
{
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    ProfScope prof(KID_COPY, st);
    hipLaunchKernelGGL(copy_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, st, (const uint4*)src, (uint4*)dst, n);
    return hipGetLastError();
}

// ------------------------------------------------------------------------------------------------ stream probe
// NI arrays read and NO arrays written, element i of every array by the same thread, grid-stride, 16 bytes per
// access: the friendliest kernel there is for a given mix of read and write streams.  What it reaches is the
// bandwidth this GPU actually delivers for that mix, the yardstick for kernels that move the same mix.
struct StreamArgs {
    const uint4* in[4];
    uint4* out[4];
};

template <int NI, int NO>
__global__ __launch_bounds__(256) void stream_probe_kernel(StreamArgs a, size_t n)
{
    // Array k is walked from a different starting point (wrapping round): arrays allocated at equal distances would
    // otherwise put all streams of a thread on the same memory channel at the same time.
    const size_t stride = (size_t)gridDim.x * 256;
    const size_t rot = n > 65536 ? 4099 : 0;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        uint4 v[NI];
#pragma unroll
        for (int k = 0; k < NI; ++k) {
            size_t j = i + k * rot;
            if (j >= n) j -= n;
            v[k] = a.in[k][j];
        }
        uint4 x = v[0];
#pragma unroll
        for (int k = 1; k < NI; ++k) { x.x ^= v[k].x; x.y ^= v[k].y; x.z ^= v[k].z; x.w ^= v[k].w; }
#pragma unroll
        for (int k = 0; k < NO; ++k) {
            size_t j = i + (NI + k) * rot;
            if (j >= n) j -= n;
            a.out[k][j] = x;
            x.x += 1u;
        }
        // nothing to write (a read-only mix): a store the compiler cannot rule out keeps the loads alive; the probe's
        // inputs never hold the pattern, so nothing is ever stored (the address is the thread's own element of input 0)
        if (NO == 0 && (x.x ^ x.y) == 0x9e3779b9u && x.z == 0x7f4a7c15u) const_cast<uint4*>(a.in[0])[i] = x;
    }
}

template <int NI>
static hipError_t stream_dispatch(const StreamArgs& a, int n_out, size_t n, dim3 grid, hipStream_t st)
{
    switch (n_out) {
    case 0: hipLaunchKernelGGL((stream_probe_kernel<NI, 0>), grid, dim3(256), 0, st, a, n); break;
    case 1: hipLaunchKernelGGL((stream_probe_kernel<NI, 1>), grid, dim3(256), 0, st, a, n); break;
    case 2: hipLaunchKernelGGL((stream_probe_kernel<NI, 2>), grid, dim3(256), 0, st, a, n); break;
    case 3: hipLaunchKernelGGL((stream_probe_kernel<NI, 3>), grid, dim3(256), 0, st, a, n); break;
    case 4: hipLaunchKernelGGL((stream_probe_kernel<NI, 4>), grid, dim3(256), 0, st, a, n); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

// Zero `n` floats.  Used instead of hipMemsetAsync so that every call of the library can be captured into a HIP graph
// (memset nodes have replayed wrongly on this platform).
__global__ __launch_bounds__(256) void zero_fill_kernel(float* __restrict__ p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = 0.f;
}

hipError_t launch_zero_fill(float* p, size_t n, hipStream_t st)
{
    if (n == 0) return hipSuccess;
    size_t blocks = (n + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(zero_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, st, p, n);
    return hipGetLastError();
}

hipError_t launch_stream_probe(const void* const* in, int n_in, void* const* out, int n_out, size_t bytes, hipStream_t st)
{
    StreamArgs a{};
    for (int k = 0; k < n_in; ++k) a.in[k] = (const uint4*)in[k];
    for (int k = 0; k < n_out; ++k) a.out[k] = (uint4*)out[k];
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    const dim3 grid((unsigned)blocks);
    ProfScope prof(KID_STREAM_PROBE, st);
    switch (n_in) {
    case 1: return stream_dispatch<1>(a, n_out, n, grid, st);
    case 2: return stream_dispatch<2>(a, n_out, n, grid, st);
    case 3: return stream_dispatch<3>(a, n_out, n, grid, st);
    case 4: return stream_dispatch<4>(a, n_out, n, grid, st);
    default: return hipErrorInvalidValue;
    }
}

typedef __attribute__((ext_vector_type(16))) float f32x16;

// ------------------------------------------------------------------------------------------------ matrix-core probe
// Nothing but v_mfma_f32_32x32x16_bf16 on registers: every wave keeps four independent accumulator tiles going, so
// that an instruction never waits for the one before it, `iters` rounds of four.  What this reaches is the matrix
// rate the GPU actually delivers (clock included), the yardstick next to the published 2.5 PFLOP/s.
typedef __attribute__((ext_vector_type(8))) __bf16 probe_bf16x8;

__global__ __launch_bounds__(256) void mfma_probe_kernel(float* __restrict__ out, int iters)
{
    const int lane = threadIdx.x & 63;
    probe_bf16x8 a, b;
#pragma unroll
    for (int e = 0; e < 8; ++e) { a[e] = (__bf16)(1.0f / (1 + ((lane + e) & 7))); b[e] = (__bf16)(0.25f * ((lane ^ e) & 3)); }
    f32x16 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[q], 0, 0, 0);
    }
    float t = 0.f;
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) t += acc[q][e];
    out[(size_t)blockIdx.x * 256 + threadIdx.x] = t;          // keeps the arithmetic alive
}

// `out` holds blocks * 256 floats; each of the blocks * 4 waves issues iters * 16 matrix instructions of 32768 FLOP.
hipError_t launch_mfma_probe(float* out, int blocks, int iters, hipStream_t st)
{
    ProfScope prof(KID_MFMA_PROBE, st);
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3(256), 0, st, out, iters);
    return hipGetLastError();
}

__device__ __forceinline__ f32x16 mfma_f32(float a, float b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ f32x16 zero16f()
{
    f32x16 z;
#pragma unroll
    for (int i = 0; i < 16; ++i) z[i] = 0.f;
    return z;
}

// Logical position p (0 = first token the causal sum sees) to physical row of the [N, d] matrix.
__device__ __forceinline__ int phys_row(int p, int N, bool rev) { return rev ? (N - 1 - p) : p; }

// acc[32x32] += A B over K2 values of k.
//   A element (m, k): a_base[(m) * a_rs + (k) * a_ks]   B element (k, n): b_base[(k) * b_ks + (n) * b_ns]
// with m = lane%32 (+ tile offset folded into the base), n = lane%32, k = k0 + lane/32, k0 stepping by 2.
__device__ __forceinline__ f32x16 gemm_tile(f32x16 acc, const float* a_base, int a_rs, int a_ks, const float* b_base,
                                            int b_ks, int b_ns, int K2, int lane)
{
    const int r = lane & 31, h = lane >> 5;
    const float* pa = a_base + r * a_rs + h * a_ks;
    const float* pb = b_base + h * b_ks + r * b_ns;
#pragma unroll 8
    for (int k0 = 0; k0 < K2; k0 += 2) acc = mfma_f32(pa[k0 * a_ks], pb[k0 * b_ks], acc);
    return acc;
}

// C rows of a row-major [N][D] fp32 matrix, starting at logical position c0 -> LDS tile with leading dimension D+1,
// in two steps so that the loads of the next chunk can be in flight while the current one is worked on: fetch() brings
// a thread's share of the tile into registers, stash() puts it into LDS.  Rows at or beyond p_end read as zero.
template <int C, int D>
struct TileRegsF32 {
    static constexpr int V4 = D / 4, NV = C * V4 / 256;
    float4 v[NV];
    __device__ __forceinline__ void fetch(const float* base, int c0, int p_end, int N, bool rev, int tid)
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / V4, c4 = x % V4, p = c0 + row;
            v[n] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (p < p_end) v[n] = *reinterpret_cast<const float4*>(base + (size_t)phys_row(p, N, rev) * D + c4 * 4);
        }
    }
    __device__ __forceinline__ void stash(float* lds, int tid) const
    {
#pragma unroll
        for (int n = 0; n < NV; ++n) {
            const int x = tid + 256 * n, row = x / V4, c4 = x % V4;
            float* d = lds + row * (D + 1) + c4 * 4;
            d[0] = v[n].x; d[1] = v[n].y; d[2] = v[n].z; d[3] = v[n].w;
        }
    }
};

// ------------------------------------------------------------------------------------------------ segment totals
// out[bh][seg][i*DV + j] = sum over the segment's tokens of K[t][i] * V[t][j].  The last segment's total is never
// used by an exclusive prefix, so its workgroups leave at once.  Wave w owns output tiles w, w+4, ...
template <int DK, int DV>
__global__ __launch_bounds__(256) void f32_seg_state_kernel(const float* __restrict__ K, const float* __restrict__ V,
                                                           float* __restrict__ out, int N, int seg_len, int n_seg,
                                                           int rev)
{
    constexpr int R = 32;                         // tokens staged per step
    constexpr int LDK = DK + 1, LDV = DV + 1;
    __shared__ float sK[R * LDK];
    __shared__ float sV[R * LDV];
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    if (seg == n_seg - 1) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float* Kb = K + (size_t)bh * N * DK;
    const float* Vb = V + (size_t)bh * N * DV;
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);
    constexpr int JB = DV / 32, NT = (DK / 32) * JB / 4;
    f32x16 acc[NT];
#pragma unroll
    for (int n = 0; n < NT; ++n) acc[n] = zero16f();
    TileRegsF32<R, DK> rk;
    TileRegsF32<R, DV> rv;
    rk.fetch(Kb, p0, p1, N, rev, tid);
    rv.fetch(Vb, p0, p1, N, rev, tid);
    for (int c0 = p0; c0 < p1; c0 += R) {
        __syncthreads();
        rk.stash(sK, tid);
        rv.stash(sV, tid);
        __syncthreads();
        if (c0 + R < p1) {     // the next step's rows, in flight during the products
            rk.fetch(Kb, c0 + R, p1, N, rev, tid);
            rv.fetch(Vb, c0 + R, p1, N, rev, tid);
        }
#pragma unroll
        for (int n = 0; n < NT; ++n) {
            const int id = w + 4 * n, ib = id / JB, jb = id % JB;
            // A[m=i][k=s] = K[s][i]: contiguous in i;  B[k=s][n=j] = V[s][j]: contiguous in j
            acc[n] = gemm_tile(acc[n], sK + ib * 32, 1, LDK, sV + jb * 32, LDV, 1, R, lane);
        }
    }
    float* o = out + ((size_t)bh * n_seg + seg) * DK * DV;
    const int r = lane & 31, h = lane >> 5;
#pragma unroll
    for (int n = 0; n < NT; ++n) {
        const int id = w + 4 * n, ib = id / JB, jb = id % JB;
#pragma unroll
        for (int a = 0; a < 4; ++a)
#pragma unroll
            for (int b = 0; b < 4; ++b) o[(ib * 32 + 8 * a + 4 * h + b) * DV + jb * 32 + r] = acc[n][4 * a + b];
    }
}

// ------------------------------------------------------------------------------------------------ main sweep
// One workgroup (4 waves) per (segment, bh).  Wave w owns output rows [32*tb, +32) with tb = w % WT and NJ column
// tiles, and the state tiles w, w+4, ...  LDS: Q, K [C][DK+1]; V [C][DV+1]; S [DK][DV+1]; P [C][C+1] in K's place.
template <int C, int DK, int DV>
__global__ __launch_bounds__(256) void f32_sweep_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                       const float* __restrict__ V, float* __restrict__ O,
                                                       const float* __restrict__ S0, int N, int seg_len, int n_seg,
                                                       int rev, int s0_transposed)
{
    constexpr int LDK = DK + 1, LDV = DV + 1, LDP = C + 1;
    constexpr int TB = C / 32, JB = DV / 32, IB = DK / 32;
    constexpr int WT = TB < 4 ? TB : 4, WJ = 4 / WT, NJ = JB / WJ;
    constexpr int NS = IB * JB / 4;
    static_assert(JB % WJ == 0, "unsupported tile shape");
    // The score tile P takes over K's place once K has done its two jobs (scores, state update): five tiles would be
    // 83 KB at the 64-wide shape and leave a compute unit to a single workgroup, four leave room for two.
    constexpr int KP = C * LDK > C * LDP ? C * LDK : C * LDP;
    __shared__ float sQ[C * LDK];
    __shared__ float sKP[KP];
    __shared__ float sV[C * LDV];
    __shared__ float sS[DK * LDV];
    float* sK = sKP;
    float* sP = sKP;
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tb = w % WT, jg = w / WT;
    const int r = lane & 31, h = lane >> 5;
    const float* Qb = Q + (size_t)bh * N * DK;
    const float* Kb = K + (size_t)bh * N * DK;
    const float* Vb = V + (size_t)bh * N * DV;
    float* Ob = O + (size_t)bh * N * DV;
    const int p0 = seg * seg_len, p1 = min(N, p0 + seg_len);

    // start state of this segment (exclusive prefix over earlier segments, zero for the first), as accumulator tiles;
    // s0_transposed: the array holds the states as [DV][DK] (left there by a call with keys and values exchanged)
    f32x16 accS[NS];
    const float* s0 = (S0 != nullptr && seg > 0) ? S0 + ((size_t)bh * n_seg + seg) * DK * DV : nullptr;
    // (the first chunk's tiles are asked for first: they are what the loop waits for)
    TileRegsF32<C, DK> rq, rk;
    TileRegsF32<C, DV> rv;
    rq.fetch(Qb, p0, p1, N, rev, tid);
    rk.fetch(Kb, p0, p1, N, rev, tid);
    rv.fetch(Vb, p0, p1, N, rev, tid);
#pragma unroll
    for (int n = 0; n < NS; ++n) {
        const int id = w + 4 * n, ib = id / JB, jb = id % JB;
        // (one uniform branch around each unrolled set of loads, so that the 16 loads of a tile are issued together)
        if (s0 == nullptr) {
            accS[n] = zero16f();
        } else if (s0_transposed) {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    accS[n][4 * a + b] = s0[(jb * 32 + r) * DK + ib * 32 + 8 * a + 4 * h + b];
        } else {
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    accS[n][4 * a + b] = s0[(ib * 32 + 8 * a + 4 * h + b) * DV + jb * 32 + r];
        }
    }
    for (int c0 = p0; c0 < p1; c0 += C) {
        __syncthreads();   // previous chunk fully consumed
        rq.stash(sQ, tid);
        rk.stash(sK, tid);
        rv.stash(sV, tid);
        // publish the state before this chunk, [i][j]
#pragma unroll
        for (int n = 0; n < NS; ++n) {
            const int id = w + 4 * n, ib = id / JB, jb = id % JB;
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) sS[(ib * 32 + 8 * a + 4 * h + b) * LDV + jb * 32 + r] = accS[n][4 * a + b];
        }
        __syncthreads();
        if (c0 + C < p1) {     // the next chunk, in flight during the arithmetic
            rq.fetch(Qb, c0 + C, p1, N, rev, tid);
            rk.fetch(Kb, c0 + C, p1, N, rev, tid);
            rv.fetch(Vb, c0 + C, p1, N, rev, tid);
        }
        // masked scores P[t][s] = q_t . k_s for s <= t, held in registers for now.  The WJ waves that share a row block
        // share its score tiles out among themselves (tile sb goes to wave sb % WJ); all of them read the whole row
        // block back from LDS below.
        constexpr int NPT = (TB + WJ - 1) / WJ;
        f32x16 pt[NPT];
#pragma unroll
        for (int sb = 0; sb < TB; ++sb) {
            // A[m=t][k=i] = Q[t][i] (row walk), B[k=i][n=s] = K[s][i] (row walk)
            if (sb <= tb && sb % WJ == jg)
                pt[sb / WJ] = gemm_tile(zero16f(), sQ + tb * 32 * LDK, LDK, 1, sK + sb * 32 * LDK, 1, LDK, DK, lane);
        }
        // state update S += K^T V (not needed after the segment's last chunk); the published copy in sS is the state
        // BEFORE this chunk, which is what the output below needs
        if (c0 + C < p1) {
#pragma unroll
            for (int n = 0; n < NS; ++n) {
                const int id = w + 4 * n, ib = id / JB, jb = id % JB;
                accS[n] = gemm_tile(accS[n], sK + ib * 32, 1, LDK, sV + jb * 32, LDV, 1, C, lane);
            }
        }
        __syncthreads();   // K has been read for the last time: its place now takes the scores
#pragma unroll
        for (int sb = 0; sb < TB; ++sb) {
            if (sb <= tb && sb % WJ == jg) {
#pragma unroll
                for (int a = 0; a < 4; ++a)
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        const int row = 8 * a + 4 * h + b;   // query within the block; r = key within the block
                        const float v = (sb == tb && r > row) ? 0.f : pt[sb / WJ][4 * a + b];
                        sP[(tb * 32 + row) * LDP + sb * 32 + r] = v;
                    }
            }
        }
        __syncthreads();   // the row blocks are complete; now every wave may read them
        f32x16 accO[NJ];
#pragma unroll
        for (int n = 0; n < NJ; ++n) {
            const int j0 = (jg * NJ + n) * 32;
            // inter-chunk part Q S_prev: A = Q rows (row walk), B[k=i][n=j] = S[i][j] (contiguous)
            accO[n] = gemm_tile(zero16f(), sQ + tb * 32 * LDK, LDK, 1, sS + j0, LDV, 1, DK, lane);
            // intra-chunk part P V over the key blocks sb <= tb: A = P rows (row walk), B[k=s][n=j] = V[s][j]
            accO[n] = gemm_tile(accO[n], sP + tb * 32 * LDP, LDP, 1, sV + j0, LDV, 1, (tb + 1) * 32, lane);
#pragma unroll
            for (int a = 0; a < 4; ++a)
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int pp = c0 + tb * 32 + 8 * a + 4 * h + b;
                    // (a streaming store: 32 lanes write one whole 128-byte line, and nothing here reads it again)
                    if (pp < p1)
                        __builtin_nontemporal_store(accO[n][4 * a + b], &Ob[(size_t)phys_row(pp, N, rev) * DV + j0 + r]);
                }
        }
    }
}

template <int DK, int DV>
static hipError_t launch_f32_impl(const float* Q, const float* K, const float* V, float* O, long BH, int N,
                                  const Plan& plan, bool rev, bool reuse_states_T, float* ws, hipStream_t st)
{
    hipError_t e;
    constexpr int C = (DK == 128 && DV == 128) ? 32 : 64;   // what fits 160 KB of LDS
    if (plan.n_seg > 1 && !reuse_states_T) {
        dim3 grid((unsigned)BH, plan.n_seg);
        {
            ProfScope prof(KID_SEG_STATE_F32, st);
            hipLaunchKernelGGL((f32_seg_state_kernel<DK, DV>), grid, dim3(256), 0, st, K, V, ws, N, plan.seg_len,
                               plan.n_seg, (int)rev);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        const int mode = SCAN_EXCL_PREFIX;
        if ((e = scan_states(ws, 0, 1, &mode, nullptr, 0, BH, plan.n_seg, DK * DV, st)) != hipSuccess) return e;
    }
    dim3 grid((unsigned)BH, plan.n_seg);
    ProfScope prof(KID_SWEEP_F32, st);
    hipLaunchKernelGGL((f32_sweep_kernel<C, DK, DV>), grid, dim3(256), 0, st, Q, K, V, O, plan.n_seg > 1 ? ws : nullptr,
                       N, plan.seg_len, plan.n_seg, (int)rev, (int)reuse_states_T);
    return hipGetLastError();
}

// reuse_states_T: the workspace already holds the scanned segment states of a call with the same split whose keys
// and values were this call's values and keys (so each state is the transpose of what this call needs): no pre-pass,
// no scan, the sweep reads them transposed.
hipError_t launch_f32(const float* Q, const float* K, const float* V, float* O, long BH, int N, int dk, int dv,
                      const Plan& plan, bool rev, float* ws, hipStream_t st, bool reuse_states_T)
{
    if (dk == 64 && dv == 64) return launch_f32_impl<64, 64>(Q, K, V, O, BH, N, plan, rev, reuse_states_T, ws, st);
    if (dk == 64 && dv == 128) return launch_f32_impl<64, 128>(Q, K, V, O, BH, N, plan, rev, reuse_states_T, ws, st);
    if (dk == 128 && dv == 64) return launch_f32_impl<128, 64>(Q, K, V, O, BH, N, plan, rev, reuse_states_T, ws, st);
    if (dk == 128 && dv == 128) return launch_f32_impl<128, 128>(Q, K, V, O, BH, N, plan, rev, reuse_states_T, ws, st);
    return hipErrorInvalidValue;
}

}  // namespace chela
