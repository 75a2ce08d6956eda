// fp32 kernels: causal linear attention with fp32 I/O and fp32 arithmetic (plain FMA, no matrix cores:
// the fp32 path exists for accuracy, the bf16 path for speed).  Also the state scan shared by both paths.
//
// Structure (Sec. 4.1): a (b,h) sequence is cut into segments; within a segment one workgroup walks the
// chunks in order, holding the d_k x d_v state S in LDS.  Per chunk: masked left product P = (Q K^T) o M,
// O = P V + Q S (both parts summed on chip), then S += K^T V.  Segment start states come from a pre-pass
// (segment totals of K^T V) and a scan over segments.
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

// Logical position p (0 = first token the causal sum sees) to physical row of the [N, d] matrix.
__device__ __forceinline__ int phys_row(int p, int N, bool rev) { return rev ? (N - 1 - p) : p; }

// ------------------------------------------------------------------------------------------------ segment totals
// out[bh][seg][i*dv + j] = sum over the segment's tokens of K[t][i] * V[t][j].  The last segment's total is never
// used by an exclusive prefix, so its workgroups leave at once.
__global__ __launch_bounds__(256) void f32_seg_state_kernel(const float* __restrict__ K, const float* __restrict__ V,
                                                           float* __restrict__ out, int N, int dk, int dv,
                                                           int seg_len, int n_seg, int rev)
{
    extern __shared__ float lds[];
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    if (seg == n_seg - 1) return;
    constexpr int R = 16;                         // rows staged per step
    float* sK = lds;                              // [R][dk]
    float* sV = lds + R * dk;                     // [R][dv]
    const int tid = threadIdx.x;
    const float* Kb = K + (size_t)bh * N * dk;
    const float* Vb = V + (size_t)bh * N * dv;
    const int p0 = seg * seg_len;
    const int p1 = min(N, p0 + seg_len);
    const int per_thread = dk * dv / 256;         // 16, 32 or 64
    float acc[64];
#pragma unroll
    for (int n = 0; n < 64; ++n) acc[n] = 0.f;
    for (int c0 = p0; c0 < p1; c0 += R) {
        for (int x = tid; x < R * dk; x += 256) {
            int r = x / dk, c = x - r * dk, p = c0 + r;
            sK[x] = p < p1 ? Kb[(size_t)phys_row(p, N, rev) * dk + c] : 0.f;
        }
        for (int x = tid; x < R * dv; x += 256) {
            int r = x / dv, c = x - r * dv, p = c0 + r;
            sV[x] = p < p1 ? Vb[(size_t)phys_row(p, N, rev) * dv + c] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int n = 0; n < 64; ++n) {
            if (n < per_thread) {
                const int e = tid + 256 * n, i = e / dv, j = e - i * dv;
                float a = acc[n];
                for (int r = 0; r < R; ++r) a = fmaf(sK[r * dk + i], sV[r * dv + j], a);
                acc[n] = a;
            }
        }
        __syncthreads();
    }
    float* o = out + ((size_t)bh * n_seg + seg) * dk * dv;
#pragma unroll
    for (int n = 0; n < 64; ++n)
        if (n < per_thread) o[tid + 256 * n] = acc[n];
}

// ------------------------------------------------------------------------------------------------ main sweep
// One workgroup per (segment, bh).  LDS: Q, K [C][dk+1]; V [C][dv+1]; P [C][C+1]; S [dk][dv+1] (the +1 keeps
// column walks off a single bank).
__global__ __launch_bounds__(256) void f32_sweep_kernel(const float* __restrict__ Q, const float* __restrict__ K,
                                                       const float* __restrict__ V, float* __restrict__ O,
                                                       const float* __restrict__ S0, int N, int dk, int dv, int C,
                                                       int seg_len, int n_seg, int rev)
{
    extern __shared__ float lds[];
    const int ldk = dk + 1, ldv = dv + 1, ldp = C + 1;
    float* sQ = lds;
    float* sK = sQ + C * ldk;
    float* sV = sK + C * ldk;
    float* sP = sV + C * ldv;
    float* sS = sP + C * ldp;
    const int seg = blockIdx.y;
    const long bh = blockIdx.x;
    const int tid = threadIdx.x;
    const float* Qb = Q + (size_t)bh * N * dk;
    const float* Kb = K + (size_t)bh * N * dk;
    const float* Vb = V + (size_t)bh * N * dv;
    float* Ob = O + (size_t)bh * N * dv;
    const int p0 = seg * seg_len;
    const int p1 = min(N, p0 + seg_len);

    // start state of this segment: exclusive prefix over earlier segments, zero for the first
    const float* s0 = (S0 != nullptr && seg > 0) ? S0 + ((size_t)bh * n_seg + seg) * dk * dv : nullptr;
    for (int e = tid; e < dk * dv; e += 256) {
        int i = e / dv, j = e - i * dv;
        sS[i * ldv + j] = s0 ? s0[e] : 0.f;
    }

    for (int c0 = p0; c0 < p1; c0 += C) {
        __syncthreads();     // previous chunk fully consumed, state visible
        for (int x = tid; x < C * dk; x += 256) {
            int r = x / dk, c = x - r * dk, p = c0 + r;
            bool ok = p < p1;
            size_t g = ok ? (size_t)phys_row(p, N, rev) * dk + c : 0;
            sQ[r * ldk + c] = ok ? Qb[g] : 0.f;
            sK[r * ldk + c] = ok ? Kb[g] : 0.f;
        }
        for (int x = tid; x < C * dv; x += 256) {
            int r = x / dv, c = x - r * dv, p = c0 + r;
            sV[r * ldv + c] = p < p1 ? Vb[(size_t)phys_row(p, N, rev) * dv + c] : 0.f;
        }
        __syncthreads();
        // P[t][s] = q_t . k_s for s <= t (the mask includes the diagonal), else 0
        for (int x = tid; x < C * C; x += 256) {
            int t = x / C, s = x - t * C;
            float a = 0.f;
            if (s <= t) {
                const float* q = sQ + t * ldk;
                const float* k = sK + s * ldk;
                for (int i = 0; i < dk; ++i) a = fmaf(q[i], k[i], a);
            }
            sP[t * ldp + s] = a;
        }
        __syncthreads();
        // O[t][j] = sum_{s<=t} P[t][s] V[s][j] + sum_i Q[t][i] S[i][j]   (inner and outer parts summed on chip)
        for (int x = tid; x < C * dv; x += 256) {
            int t = x / dv, j = x - t * dv;
            int p = c0 + t;
            if (p < p1) {
                float a = 0.f;
                const float* pr = sP + t * ldp;
                for (int s = 0; s <= t; ++s) a = fmaf(pr[s], sV[s * ldv + j], a);
                float b = 0.f;
                const float* q = sQ + t * ldk;
                for (int i = 0; i < dk; ++i) b = fmaf(q[i], sS[i * ldv + j], b);
                Ob[(size_t)phys_row(p, N, rev) * dv + j] = a + b;
            }
        }
        __syncthreads();
        // S[i][j] += sum_s K[s][i] V[s][j]
        if (c0 + C < p1) {
            for (int e = tid; e < dk * dv; e += 256) {
                int i = e / dv, j = e - i * dv;
                float a = sS[i * ldv + j];
                for (int s = 0; s < C; ++s) a = fmaf(sK[s * ldk + i], sV[s * ldv + j], a);
                sS[i * ldv + j] = a;
            }
        }
    }
}

static size_t f32_sweep_lds(int dk, int dv, int C)
{
    return sizeof(float) * ((size_t)2 * C * (dk + 1) + (size_t)C * (dv + 1) + (size_t)C * (C + 1) +
                            (size_t)dk * (dv + 1));
}

hipError_t launch_f32(const float* Q, const float* K, const float* V, float* O, long BH, int N, int dk, int dv,
                      const Plan& plan, bool rev, float* ws, hipStream_t st)
{
    hipError_t e;
    const int C = plan.chunk;
    if (plan.n_seg > 1) {
        dim3 grid((unsigned)BH, plan.n_seg);
        size_t lds1 = sizeof(float) * 16 * (size_t)(dk + dv);
        {
            ProfScope prof(KID_SEG_STATE_F32, st);
            hipLaunchKernelGGL(f32_seg_state_kernel, grid, dim3(256), lds1, st, K, V, ws, N, dk, dv, plan.seg_len,
                               plan.n_seg, (int)rev);
        }
        if ((e = hipGetLastError()) != hipSuccess) return e;
        const int mode = SCAN_EXCL_PREFIX;
        if ((e = scan_states(ws, 0, 1, &mode, nullptr, 0, BH, plan.n_seg, dk * dv, st)) != hipSuccess) return e;
    }
    const size_t lds = f32_sweep_lds(dk, dv, C);
    e = hipFuncSetAttribute((const void*)f32_sweep_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    dim3 grid((unsigned)BH, plan.n_seg);
    ProfScope prof(KID_SWEEP_F32, st);
    hipLaunchKernelGGL(f32_sweep_kernel, grid, dim3(256), lds, st, Q, K, V, O, plan.n_seg > 1 ? ws : nullptr, N, dk,
                       dv, C, plan.seg_len, plan.n_seg, (int)rev);
    return hipGetLastError();
}

}  // namespace chela
