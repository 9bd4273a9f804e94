// Plain fp32-FMA kernels of liblasp2: every supported (dtype, d, C) runs here
// unless the bf16 MFMA kernels take it.  They favour being easy to check over
// speed: one workgroup per state slot, fp32 arithmetic throughout, fixed
// summation order (run-to-run bit-identical, no atomics).
//
// Also holds the state prefix/suffix kernel, which is the same for every path.
#include "lasp2_common.h"

#include <hip/hip_bf16.h>

namespace lasp2 {
namespace {

constexpr int kThreads = 256;
constexpr int kRows = 16;  // query rows handled per pass of the attention kernel

__device__ __forceinline__ float ld(const float* p) { return *p; }
__device__ __forceinline__ float ld(const __hip_bfloat16* p) { return __bfloat162float(*p); }
__device__ __forceinline__ void st(float* p, float v) { *p = v; }
__device__ __forceinline__ void st(__hip_bfloat16* p, float v) { *p = __float2bfloat16(v); }

// M[slot] = sum over the slot's tokens of k^T v.  Thread (ty,tx) of a 16x16 grid owns
// the elements (ty + 16 i, tx + 16 j).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void states_generic_kernel(Geom g, const T* __restrict__ K,
                                                                  const T* __restrict__ V,
                                                                  float* __restrict__ M, int anchor_start)
{
    constexpr int TM = D / 16;
    const int s = blockIdx.x, grp = blockIdx.y;
    const int ty = threadIdx.x / 16, tx = threadIdx.x % 16;
    int tok0, len;
    slot_range(g, s, tok0, len);
    const size_t gbase = (size_t)grp * (size_t)g.N * D;

    float acc[TM][TM];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) acc[i][j] = 0.f;

    const float l2 = decay_log2(g, grp);
    for (int t = 0; t < len; ++t) {
        const T* kr = K + gbase + (size_t)(tok0 + t) * D;
        const T* vr = V + gbase + (size_t)(tok0 + t) * D;
        // decay: the token's weight as seen from the slot's last (or first) token
        const float wt = exp2f((float)(anchor_start ? t : len - 1 - t) * l2);
        float kk[TM], vv[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) kk[i] = wt * ld(kr + ty + 16 * i);
#pragma unroll
        for (int j = 0; j < TM; ++j) vv[j] = ld(vr + tx + 16 * j);
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TM; ++j) acc[i][j] = fmaf(kk[i], vv[j], acc[i][j]);
    }
    float* m = M + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TM; ++j) m[(ty + 16 * i) * D + tx + 16 * j] = acc[i][j];
}

// One workgroup walks the chunks of one slot.  Shared memory: the running state
// (D x D fp32), one block of kRows rows of A, and their masked scores.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void attn_generic_kernel(
    Geom g, const T* __restrict__ A, const T* __restrict__ Bk, const T* __restrict__ Cv,
    const float* __restrict__ state, T* __restrict__ out, int transpose_state, int reverse)
{
    constexpr int TM = D / 16;
    constexpr int AS = D + 1;  // padded row stride of the A block
    extern __shared__ float smem[];
    float* Mst = smem;                 // D*D
    float* Ablk = Mst + D * D;         // kRows*AS
    float* S = Ablk + kRows * AS;      // kRows*(C+1)
    const int SS = g.C + 1;

    const int tid = threadIdx.x;
    const int s = blockIdx.x, grp = blockIdx.y;
    int tok0, len;
    slot_range(g, s, tok0, len);
    const size_t gbase = (size_t)grp * (size_t)g.N * D;
    // state == NULL: every slot opens its document, so the prefix (suffix) it starts from is zero
    const float* st0 = state ? state + ((size_t)grp * g.T_s + s) * (size_t)(D * D) : nullptr;

    for (int e = tid; e < D * D; e += kThreads) {
        int a = e / D, b = e % D;
        Mst[e] = st0 ? (transpose_state ? st0[b * D + a] : st0[e]) : 0.f;
    }
    __syncthreads();

    // decay: lam^e = exp2f(e * l2); l2 = 0 without decay, and every weight is then exactly 1
    const float l2 = decay_log2(g, grp);
    const int nch = (len + g.C - 1) / g.C;
    for (int ci = 0; ci < nch; ++ci) {
        const int c = reverse ? nch - 1 - ci : ci;
        const int c0 = tok0 + c * g.C;
        const int clen = min(g.C, tok0 + len - c0);

        for (int r0 = 0; r0 < clen; r0 += kRows) {
            const int rl = min(kRows, clen - r0);
            for (int idx = tid; idx < kRows * D; idx += kThreads) {
                int r = idx / D, a = idx % D;
                Ablk[r * AS + a] = (r < rl) ? ld(A + gbase + (size_t)(c0 + r0 + r) * D + a) : 0.f;
            }
            __syncthreads();
            // masked scores S[r][j] = a_{r0+r} . b_j on allowed pairs, else 0
            for (int idx = tid; idx < kRows * clen; idx += kThreads) {
                int r = idx % kRows, j = idx / kRows;
                int i = r0 + r;
                bool keep = (r < rl) && (reverse ? (j >= i) : (j <= i));
                float acc = 0.f;
                if (keep) {
                    const T* br = Bk + gbase + (size_t)(c0 + j) * D;
                    for (int a = 0; a < D; ++a) acc = fmaf(Ablk[r * AS + a], ld(br + a), acc);
                    acc *= exp2f((float)(reverse ? j - i : i - j) * l2);
                }
                S[r * SS + j] = acc;
            }
            __syncthreads();
            // out[r][b] = sum_j S[r][j] c_j[b] + sum_a A[r][a] Mst[a][b]
            for (int idx = tid; idx < kRows * D; idx += kThreads) {
                int r = idx / D, b = idx % D;
                if (r >= rl) continue;
                int i = r0 + r;
                int jlo = reverse ? i : 0, jhi = reverse ? clen - 1 : i;
                float intra = 0.f, inter = 0.f;
                for (int j = jlo; j <= jhi; ++j)
                    intra = fmaf(S[r * SS + j], ld(Cv + gbase + (size_t)(c0 + j) * D + b), intra);
                for (int a = 0; a < D; ++a) inter = fmaf(Ablk[r * AS + a], Mst[a * D + b], inter);
                // the state sits one token before the chunk (causal) or one after it (anti-causal)
                const float wi = exp2f((float)(reverse ? clen - i : i + 1) * l2);
                st(out + gbase + (size_t)(c0 + i) * D + b, fmaf(wi, inter, intra));
            }
            __syncthreads();
        }

        if (ci + 1 < nch) {
            // running state = lam^clen * state + sum_t w_t Bk_t^T Cv_t, w_t = the token's weight as
            // seen from the chunk's last (causal) or first (anti-causal) token; each thread owns
            // its own elements
            const int ty = tid / 16, tx = tid % 16;
            const float wc = exp2f((float)clen * l2);
            float acc[TM][TM];
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) acc[i][j] = 0.f;
            for (int t = 0; t < clen; ++t) {
                const T* br = Bk + gbase + (size_t)(c0 + t) * D;
                const T* cr = Cv + gbase + (size_t)(c0 + t) * D;
                const float wt = exp2f((float)(reverse ? t : clen - 1 - t) * l2);
                float bb[TM], cc[TM];
#pragma unroll
                for (int i = 0; i < TM; ++i) bb[i] = wt * ld(br + ty + 16 * i);
#pragma unroll
                for (int j = 0; j < TM; ++j) cc[j] = ld(cr + tx + 16 * j);
#pragma unroll
                for (int i = 0; i < TM; ++i)
#pragma unroll
                    for (int j = 0; j < TM; ++j) acc[i][j] = fmaf(bb[i], cc[j], acc[i][j]);
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int j = 0; j < TM; ++j) {
                    float& m = Mst[(ty + 16 * i) * D + tx + 16 * j];
                    m = fmaf(wc, m, acc[i][j]);
                }
            __syncthreads();
        }
    }
}

// Exclusive prefix (or suffix) over the slots of each group, restarted per document.
// One thread owns four adjacent state elements and walks the slots in order; loads are
// batched ahead of the stores so that in-place use (P == M) stays correct and the
// memory system sees several requests in flight.
constexpr int kScanBatch = 8;

__global__ __launch_bounds__(kThreads) void state_prefix_kernel(Geom g, const float* M, float* P,
                                                                int reverse, int inclusive)
{
    const int dd = g.d * g.d;
    const int e = (blockIdx.x * kThreads + threadIdx.x) * 4;
    if (e >= dd) return;
    const size_t base = (size_t)blockIdx.y * (size_t)g.T_s * dd + e;
    const int ndocs = g.n_seqs ? g.n_seqs : 1;
    const float l2 = decay_log2(g, blockIdx.y);
    const int step = reverse ? -1 : 1;
    int s = reverse ? g.T_s - 1 : 0;
    for (int kk = 0; kk < ndocs; ++kk) {
        const int k = reverse ? ndocs - 1 - kk : kk;
        const int dlen = g.n_seqs ? (g.cu[k + 1] - g.cu[k]) : g.N;
        const int ns = (int)(((int64_t)dlen + g.L - 1) / g.L);
        float4 run = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int r = 0; r < ns; r += kScanBatch) {
            float4 m[kScanBatch];
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u)
                if (r + u < ns)
                    m[u] = *reinterpret_cast<const float4*>(M + base + (size_t)(s + step * u) * dd);
#pragma unroll
            for (int u = 0; u < kScanBatch; ++u)
                if (r + u < ns) {
                    float4* dst = reinterpret_cast<float4*>(P + base + (size_t)(s + step * u) * dd);
                    if (!inclusive) *dst = run;
                    // decay: the carried state ages by the length of the slot it crosses
                    // (slot index inside the document: r+u counted from the walk's start)
                    const int idx = reverse ? ns - 1 - (r + u) : r + u;
                    const int n = (int)min((int64_t)g.L, (int64_t)dlen - (int64_t)idx * g.L);
                    const float w = exp2f((float)n * l2);
                    run.x = fmaf(w, run.x, m[u].x); run.y = fmaf(w, run.y, m[u].y);
                    run.z = fmaf(w, run.z, m[u].z); run.w = fmaf(w, run.w, m[u].w);
                    if (inclusive) *dst = run;
                }
            s += step * min(kScanBatch, ns - r);
        }
    }
}

// S[s] = sum of M over all slots of the document that owns slot s (the state every rank holds
// after the gather and the sum when there is no mask).  Each thread owns four elements of the
// d x d state and sums the document's slots in ascending order before it writes any of them,
// so S may alias M.
__global__ __launch_bounds__(kThreads) void state_total_kernel(Geom g, const float* M, float* S)
{
    const int dd = g.d * g.d;
    const int e = (blockIdx.x * kThreads + threadIdx.x) * 4;
    if (e >= dd) return;
    const size_t base = (size_t)blockIdx.y * (size_t)g.T_s * dd + e;
    const int ndocs = g.n_seqs ? g.n_seqs : 1;
    int s0 = 0;
    for (int k = 0; k < ndocs; ++k) {
        const int dlen = g.n_seqs ? (g.cu[k + 1] - g.cu[k]) : g.N;
        const int ns = (int)(((int64_t)dlen + g.L - 1) / g.L);
        float4 run = make_float4(0.f, 0.f, 0.f, 0.f);
        for (int r = 0; r < ns; ++r) {
            const float4 m = *reinterpret_cast<const float4*>(M + base + (size_t)(s0 + r) * dd);
            run.x += m.x; run.y += m.y; run.z += m.z; run.w += m.w;
        }
        for (int r = 0; r < ns; ++r) *reinterpret_cast<float4*>(S + base + (size_t)(s0 + r) * dd) = run;
        s0 += ns;
    }
}

// out = A * state (or A * state^T) for the rows of one slot.  The state sits in LDS as
// sS[r][c] = the factor of A[.,r] in out[.,c]; thread (rg, c) produces column c of the rows
// rg, rg + NRG, ... of each tile of kProjRows * NRG rows.
constexpr int kProjRows = 8;

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void rows_state_generic_kernel(Geom g, const T* __restrict__ A,
                                                                      const float* __restrict__ state,
                                                                      T* __restrict__ out, int transpose)
{
    constexpr int NRG = kThreads / D, RT = kProjRows * NRG;
    extern __shared__ float smem_f[];
    float* sS = smem_f;            // [D][D]
    float* sA = smem_f + D * D;    // [RT][D]
    const int s = blockIdx.x, grp = blockIdx.y;
    int tok0, len;
    slot_range(g, s, tok0, len);
    if (len <= 0) return;
    const float* st_ = state + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
    for (int i = threadIdx.x; i < D * D; i += kThreads) {
        const int r = i / D, c = i % D;
        sS[i] = transpose ? st_[c * D + r] : st_[i];
    }
    const int c = threadIdx.x % D, rg = threadIdx.x / D;
    const size_t gbase = ((size_t)grp * (size_t)g.N + tok0) * D;
    for (int r0 = 0; r0 < len; r0 += RT) {
        __syncthreads();   // state staged / previous tile consumed
        for (int i = threadIdx.x; i < RT * D; i += kThreads) {
            const int row = r0 + i / D;
            sA[i] = row < len ? ld(A + gbase + (size_t)row * D + i % D) : 0.f;
        }
        __syncthreads();
        float acc[kProjRows];
#pragma unroll
        for (int j = 0; j < kProjRows; ++j) acc[j] = 0.f;
        for (int r = 0; r < D; ++r) {
            const float w = sS[r * D + c];
#pragma unroll
            for (int j = 0; j < kProjRows; ++j) acc[j] = fmaf(sA[(rg + j * NRG) * D + r], w, acc[j]);
        }
#pragma unroll
        for (int j = 0; j < kProjRows; ++j) {
            const int row = r0 + rg + j * NRG;
            if (row < len) st(out + gbase + (size_t)row * D + c, acc[j]);
        }
    }
}

template <typename T, int D>
hipError_t rows_state_generic_TD(const Geom& g, const T* A, const float* state, T* out, int tr,
                                 hipStream_t st)
{
    constexpr size_t smem = sizeof(float) * ((size_t)D * D + (size_t)kProjRows * (kThreads / D) * D);
    auto kern = rows_state_generic_kernel<T, D>;
    if (smem > 48 * 1024) {
        hipError_t e = allow_dynamic_lds<rows_state_generic_kernel<T, D>>((int)smem);
        if (e != hipSuccess) return e;
    }
    dim3 grid(g.T_s, g.G), block(kThreads);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, A, state, out, tr);
    return hipGetLastError();
}

template <typename T>
hipError_t rows_state_generic_T(const Geom& g, const T* A, const float* state, T* out, int tr,
                                hipStream_t st)
{
    switch (g.d) {
        case 16: return rows_state_generic_TD<T, 16>(g, A, state, out, tr, st);
        case 32: return rows_state_generic_TD<T, 32>(g, A, state, out, tr, st);
        case 64: return rows_state_generic_TD<T, 64>(g, A, state, out, tr, st);
        default: return rows_state_generic_TD<T, 128>(g, A, state, out, tr, st);
    }
}

// Softmax attention forward for kSmRows queries per workgroup, plain fp32: the keys of the
// workgroup's range are taken 64 at a time; scores go to LDS, one thread per query keeps the
// running maximum and sum and turns the scores into exp(s - m), and every thread owns the
// output elements (query r, columns c, c + 256/kSmRows ...) which it rescales and extends.
constexpr int kSmRows = 16, kSmKeys = 64;

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void softmax_fwd_generic_kernel(Geom g, const T* __restrict__ Q,
                                                                       const T* __restrict__ K,
                                                                       const T* __restrict__ V,
                                                                       T* __restrict__ O,
                                                                       float* __restrict__ LSE, int causal)
{
    constexpr int CPT = kSmRows * D / kThreads;     // output columns per thread (same query)
    constexpr int TPR = kThreads / kSmRows;         // threads per query
    __shared__ float sQ[kSmRows][D + 1];
    __shared__ float sS[kSmRows][kSmKeys + 1];
    __shared__ float sAlpha[kSmRows], sM[kSmRows], sL[kSmRows];
    __shared__ int sLo[kSmRows], sHi[kSmRows];
    const int tid = threadIdx.x, grp = blockIdx.y;
    const int r0 = blockIdx.x * kSmRows;                    // first of this workgroup's query rows
    const size_t gbase = (size_t)grp * (size_t)g.N * D;     // K, V
    const size_t qbase = (size_t)grp * (size_t)g.qn * D;    // Q, O (row r = token q0 + r)
    const float scale = rsqrtf((float)D);

    if (tid < kSmRows) {
        const int i = g.q0 + r0 + tid;
        int lo = 0, hi = 0;
        if (r0 + tid < g.qn) {
            lo = 0; hi = g.N;
            for (int k = 0; k < g.n_seqs; ++k)
                if (g.cu[k] <= i && i < g.cu[k + 1]) { lo = g.cu[k]; hi = g.cu[k + 1]; }
            if (causal) hi = i + 1;
        }
        sLo[tid] = lo; sHi[tid] = hi;
        sM[tid] = -INFINITY; sL[tid] = 0.f;
    }
    for (int idx = tid; idx < kSmRows * D; idx += kThreads) {
        const int r = idx / D, a = idx % D;
        sQ[r][a] = (r0 + r < g.qn) ? ld(Q + qbase + (size_t)(r0 + r) * D + a) : 0.f;
    }
    __syncthreads();
    int klo = g.N, khi = 0;
    for (int r = 0; r < kSmRows; ++r) { klo = min(klo, sHi[r] > sLo[r] ? sLo[r] : g.N); khi = max(khi, sHi[r]); }

    const int myr = tid / TPR, c0 = tid % TPR;
    float acc[CPT];
#pragma unroll
    for (int u = 0; u < CPT; ++u) acc[u] = 0.f;

    for (int k0 = klo; k0 < khi; k0 += kSmKeys) {
        for (int idx = tid; idx < kSmRows * kSmKeys; idx += kThreads) {
            const int r = idx % kSmRows, j = idx / kSmRows, key = k0 + j;
            float sres = -INFINITY;
            if (key >= sLo[r] && key < sHi[r]) {
                const T* kr = K + gbase + (size_t)key * D;
                float a = 0.f;
                for (int e = 0; e < D; ++e) a = fmaf(sQ[r][e], ld(kr + e), a);
                sres = a * scale;
            }
            sS[r][j] = sres;
        }
        __syncthreads();
        if (tid < kSmRows) {
            float mx = sM[tid];
            for (int j = 0; j < kSmKeys; ++j) mx = fmaxf(mx, sS[tid][j]);
            const float mu = (mx == -INFINITY) ? 0.f : mx;
            const float alpha = expf(sM[tid] - mu);
            float ps = 0.f;
            for (int j = 0; j < kSmKeys; ++j) { const float p = expf(sS[tid][j] - mu); sS[tid][j] = p; ps += p; }
            sL[tid] = sL[tid] * alpha + ps;
            sM[tid] = mx;
            sAlpha[tid] = alpha;
        }
        __syncthreads();
        {
            const float alpha = sAlpha[myr];
            const int nk = min(kSmKeys, g.N - k0);
#pragma unroll
            for (int u = 0; u < CPT; ++u) acc[u] *= alpha;
            for (int j = 0; j < nk; ++j) {
                const float p = sS[myr][j];
                const T* vr = V + gbase + (size_t)(k0 + j) * D;
#pragma unroll
                for (int u = 0; u < CPT; ++u) acc[u] = fmaf(p, ld(vr + c0 + u * TPR), acc[u]);
            }
        }
        __syncthreads();
    }
    if (r0 + myr < g.qn) {
        const float inv = 1.f / sL[myr];
#pragma unroll
        for (int u = 0; u < CPT; ++u) st(O + qbase + (size_t)(r0 + myr) * D + c0 + u * TPR, acc[u] * inv);
        if (c0 == 0) LSE[(size_t)grp * g.qn + r0 + myr] = sM[myr] + logf(sL[myr]);
    }
}

template <typename T>
hipError_t softmax_fwd_generic_T(const Geom& g, const T* Q, const T* K, const T* V, T* O, float* LSE,
                                 int causal, hipStream_t st)
{
    dim3 grid((g.qn + kSmRows - 1) / kSmRows, g.G), block(kThreads);
    switch (g.d) {
        case 16: hipLaunchKernelGGL((softmax_fwd_generic_kernel<T, 16>), grid, block, 0, st, g, Q, K, V, O, LSE, causal); break;
        case 32: hipLaunchKernelGGL((softmax_fwd_generic_kernel<T, 32>), grid, block, 0, st, g, Q, K, V, O, LSE, causal); break;
        case 64: hipLaunchKernelGGL((softmax_fwd_generic_kernel<T, 64>), grid, block, 0, st, g, Q, K, V, O, LSE, causal); break;
        default: hipLaunchKernelGGL((softmax_fwd_generic_kernel<T, 128>), grid, block, 0, st, g, Q, K, V, O, LSE, causal); break;
    }
    return hipGetLastError();
}

// delta_i = dO_i . O_i for every row (the row sums the softmax backward needs); one wave-sized
// group of 64 threads per row.  lse2, when given, receives the row's log-sum-exp times log2(e),
// the form in which the matrix-core dK/dV kernel subtracts it from base-2 scores.
template <typename T>
__global__ __launch_bounds__(kThreads) void softmax_delta_kernel(Geom g, const T* __restrict__ O,
                                                                 const T* __restrict__ dO,
                                                                 const float* __restrict__ LSE,
                                                                 float* __restrict__ delta,
                                                                 float* __restrict__ lse2)
{
    const size_t rows = (size_t)g.G * (size_t)g.qn;
    const size_t row = (size_t)blockIdx.x * (kThreads / 64) + threadIdx.x / 64;
    if (row >= rows) return;
    const int lane = threadIdx.x % 64;
    float acc = 0.f;
    for (int a = lane; a < g.d; a += 64) acc = fmaf(ld(O + row * g.d + a), ld(dO + row * g.d + a), acc);
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) acc += __shfl_xor(acc, o, 64);
    if (lane == 0) {
        delta[row] = acc;
        if (lse2) lse2[row] = LSE[row] * 1.4426950408889634f;
    }
}

// Softmax attention backward, plain fp32, in two kernels that mirror the forward one.
// WHICH == 0: dQ for kSmRows queries per workgroup, keys taken 64 at a time:
//     P = exp(s - lse_i), dP = dO_i . v_j, dS = P (dP - delta_i), dQ_i += scale * dS k_j.
// WHICH == 1: dK and dV for kSmRows keys per workgroup, queries taken 64 at a time:
//     dV_j += P dO_i,  dK_j += scale * dS q_i.
template <typename T, int D, int WHICH>
__global__ __launch_bounds__(kThreads) void softmax_bwd_generic_kernel(
    Geom g, const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    T* __restrict__ dQ, T* __restrict__ dK, T* __restrict__ dV, int causal)
{
    constexpr int CPT = kSmRows * D / kThreads, TPR = kThreads / kSmRows;
    __shared__ float sA[kSmRows][D + 1];      // the workgroup's own rows: q (dQ) or k (dK, dV)
    __shared__ float sB[kSmRows][D + 1];      //                            dO (dQ) or v (dK, dV)
    __shared__ float sP[kSmRows][kSmKeys + 1], sDS[kSmRows][kSmKeys + 1];
    __shared__ int sLo[kSmRows], sHi[kSmRows];
    const int tid = threadIdx.x, grp = blockIdx.y;
    const int r0 = blockIdx.x * kSmRows;      // own rows: local query rows (dQ) or keys (dK, dV)
    const size_t gbase = (size_t)grp * (size_t)g.N * D;     // K, V, dK, dV
    const size_t qbase = (size_t)grp * (size_t)g.qn * D;    // Q, dO, dQ (row r = token q0 + r)
    const size_t obase = WHICH == 0 ? qbase : gbase;
    const int own_n = WHICH == 0 ? g.qn : g.N;
    const float scale = rsqrtf((float)D);
    const T* ownA = WHICH == 0 ? Q : K;
    const T* ownB = WHICH == 0 ? dO : V;

    // range of partner tokens each own row interacts with: keys of a query, or the share's
    // queries of a key
    if (tid < kSmRows) {
        const int i = (WHICH == 0 ? g.q0 : 0) + r0 + tid;   // this row's token
        int lo = 0, hi = 0;
        if (r0 + tid < own_n) {
            lo = 0; hi = g.N;
            for (int k = 0; k < g.n_seqs; ++k)
                if (g.cu[k] <= i && i < g.cu[k + 1]) { lo = g.cu[k]; hi = g.cu[k + 1]; }
            if (causal) { if (WHICH == 0) hi = i + 1; else lo = i; }
            if (WHICH == 1) { lo = max(lo, g.q0); hi = min(hi, g.q0 + g.qn); }
        }
        sLo[tid] = lo; sHi[tid] = hi;
    }
    for (int idx = tid; idx < kSmRows * D; idx += kThreads) {
        const int r = idx / D, a = idx % D;
        const bool ok = r0 + r < own_n;
        sA[r][a] = ok ? ld(ownA + obase + (size_t)(r0 + r) * D + a) : 0.f;
        sB[r][a] = ok ? ld(ownB + obase + (size_t)(r0 + r) * D + a) : 0.f;
    }
    __syncthreads();
    int plo = g.N, phi = 0;
    for (int r = 0; r < kSmRows; ++r) { plo = min(plo, sHi[r] > sLo[r] ? sLo[r] : g.N); phi = max(phi, sHi[r]); }
    // partner arrays: keys (absolute rows of K, V) or queries (rows of Q, dO relative to q0)
    const size_t pbase = WHICH == 0 ? gbase : qbase;
    const int poff = WHICH == 0 ? 0 : g.q0;
    const int pend = WHICH == 0 ? g.N : g.q0 + g.qn;

    const int myr = tid / TPR, c0 = tid % TPR;
    float acc1[CPT], acc2[CPT];     // dQ (acc1) or dK (acc1), dV (acc2)
#pragma unroll
    for (int u = 0; u < CPT; ++u) { acc1[u] = 0.f; acc2[u] = 0.f; }

    for (int p0 = plo; p0 < phi; p0 += kSmKeys) {
        for (int idx = tid; idx < kSmRows * kSmKeys; idx += kThreads) {
            const int r = idx % kSmRows, j = idx / kSmRows, pr = p0 + j;     // own row r, partner row pr
            float pv = 0.f, ds = 0.f;
            if (pr >= sLo[r] && pr < sHi[r]) {
                // local query row of this pair
                const int qi = WHICH == 0 ? r0 + r : pr - g.q0;
                const T* prA = (WHICH == 0 ? K : Q) + pbase + (size_t)(pr - poff) * D;   // partner k (or q)
                const T* prB = (WHICH == 0 ? V : dO) + pbase + (size_t)(pr - poff) * D;  // partner v (or dO)
                float sdot = 0.f, dpdot = 0.f;
                for (int e = 0; e < D; ++e) {
                    sdot = fmaf(sA[r][e], ld(prA + e), sdot);     // q . k
                    dpdot = fmaf(sB[r][e], ld(prB + e), dpdot);   // dO . v
                }
                pv = expf(sdot * scale - LSE[(size_t)grp * g.qn + qi]);
                ds = pv * (dpdot - delta[(size_t)grp * g.qn + qi]);
            }
            sP[r][j] = pv;
            sDS[r][j] = ds;
        }
        __syncthreads();
        {
            const int np = min(kSmKeys, pend - p0);
            for (int j = 0; j < np; ++j) {
                const float ds = sDS[myr][j] * scale, pv = sP[myr][j];
                const T* xr = (WHICH == 0 ? K : Q) + pbase + (size_t)(p0 + j - poff) * D;
                const T* yr = dO + qbase + (size_t)(p0 + j - g.q0) * D;   // read only when WHICH == 1
#pragma unroll
                for (int u = 0; u < CPT; ++u) {
                    acc1[u] = fmaf(ds, ld(xr + c0 + u * TPR), acc1[u]);
                    if (WHICH == 1) acc2[u] = fmaf(pv, ld(yr + c0 + u * TPR), acc2[u]);
                }
            }
        }
        __syncthreads();
    }
    if (r0 + myr < own_n) {
#pragma unroll
        for (int u = 0; u < CPT; ++u) {
            const size_t o = obase + (size_t)(r0 + myr) * D + c0 + u * TPR;
            if (WHICH == 0) st(dQ + o, acc1[u]);
            else { st(dK + o, acc1[u]); st(dV + o, acc2[u]); }
        }
    }
}

template <typename T, int D>
hipError_t softmax_bwd_generic_TD(const Geom& g, const T* Q, const T* K, const T* V, const T* dO,
                                  const float* LSE, const float* delta, T* dQ, T* dK, T* dV, int causal,
                                  hipStream_t st)
{
    dim3 gridq((g.qn + kSmRows - 1) / kSmRows, g.G), gridk((g.N + kSmRows - 1) / kSmRows, g.G), block(kThreads);
    if (dQ && g.qn > 0)
        hipLaunchKernelGGL((softmax_bwd_generic_kernel<T, D, 0>), gridq, block, 0, st, g, Q, K, V, dO, LSE,
                           delta, dQ, dK, dV, causal);
    if (dK)
        hipLaunchKernelGGL((softmax_bwd_generic_kernel<T, D, 1>), gridk, block, 0, st, g, Q, K, V, dO, LSE,
                           delta, dQ, dK, dV, causal);
    return hipGetLastError();
}

template <typename T>
hipError_t softmax_bwd_generic_T(const Geom& g, const T* Q, const T* K, const T* V, const T* dO,
                                 const float* LSE, const float* delta, T* dQ, T* dK, T* dV, int causal,
                                 hipStream_t st)
{
    switch (g.d) {
        case 16: return softmax_bwd_generic_TD<T, 16>(g, Q, K, V, dO, LSE, delta, dQ, dK, dV, causal, st);
        case 32: return softmax_bwd_generic_TD<T, 32>(g, Q, K, V, dO, LSE, delta, dQ, dK, dV, causal, st);
        case 64: return softmax_bwd_generic_TD<T, 64>(g, Q, K, V, dO, LSE, delta, dQ, dK, dV, causal, st);
        default: return softmax_bwd_generic_TD<T, 128>(g, Q, K, V, dO, LSE, delta, dQ, dK, dV, causal, st);
    }
}

template <typename T>
hipError_t states_generic_T(const Geom& g, const T* K, const T* V, float* M, int anchor, hipStream_t st)
{
    dim3 grid(g.T_s, g.G), block(kThreads);
    switch (g.d) {
        case 16: hipLaunchKernelGGL((states_generic_kernel<T, 16>), grid, block, 0, st, g, K, V, M, anchor); break;
        case 32: hipLaunchKernelGGL((states_generic_kernel<T, 32>), grid, block, 0, st, g, K, V, M, anchor); break;
        case 64: hipLaunchKernelGGL((states_generic_kernel<T, 64>), grid, block, 0, st, g, K, V, M, anchor); break;
        default: hipLaunchKernelGGL((states_generic_kernel<T, 128>), grid, block, 0, st, g, K, V, M, anchor); break;
    }
    return hipGetLastError();
}

template <typename T, int D>
hipError_t attn_generic_TD(const Geom& g, const T* A, const T* Bk, const T* Cv, const float* state,
                           T* out, int tr, int rev, hipStream_t st)
{
    size_t smem = sizeof(float) * ((size_t)D * D + (size_t)kRows * (D + 1) + (size_t)kRows * (g.C + 1));
    auto kern = attn_generic_kernel<T, D>;
    if (smem > 48 * 1024) {
        hipError_t e = allow_dynamic_lds<attn_generic_kernel<T, D>>((int)smem);
        if (e != hipSuccess) return e;
    }
    dim3 grid(g.T_s, g.G), block(kThreads);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, A, Bk, Cv, state, out, tr, rev);
    return hipGetLastError();
}

template <typename T>
hipError_t attn_generic_T(const Geom& g, const T* A, const T* Bk, const T* Cv, const float* state,
                          T* out, int tr, int rev, hipStream_t st)
{
    switch (g.d) {
        case 16: return attn_generic_TD<T, 16>(g, A, Bk, Cv, state, out, tr, rev, st);
        case 32: return attn_generic_TD<T, 32>(g, A, Bk, Cv, state, out, tr, rev, st);
        case 64: return attn_generic_TD<T, 64>(g, A, Bk, Cv, state, out, tr, rev, st);
        default: return attn_generic_TD<T, 128>(g, A, Bk, Cv, state, out, tr, rev, st);
    }
}

}  // namespace

hipError_t launch_states_generic(const Geom& g, int dtype, const void* K, const void* V, float* M,
                                 int anchor_start, hipStream_t st)
{
    if (dtype == LASP2_F32)
        return states_generic_T(g, static_cast<const float*>(K), static_cast<const float*>(V), M,
                                anchor_start, st);
    return states_generic_T(g, static_cast<const __hip_bfloat16*>(K),
                            static_cast<const __hip_bfloat16*>(V), M, anchor_start, st);
}

hipError_t launch_attn_generic(const Geom& g, int dtype, const void* A, const void* Bk,
                               const void* Cv, const float* state, void* out, int transpose_state,
                               int reverse, hipStream_t st)
{
    if (dtype == LASP2_F32)
        return attn_generic_T(g, static_cast<const float*>(A), static_cast<const float*>(Bk),
                              static_cast<const float*>(Cv), state, static_cast<float*>(out),
                              transpose_state, reverse, st);
    return attn_generic_T(g, static_cast<const __hip_bfloat16*>(A),
                          static_cast<const __hip_bfloat16*>(Bk),
                          static_cast<const __hip_bfloat16*>(Cv), state,
                          static_cast<__hip_bfloat16*>(out), transpose_state, reverse, st);
}

hipError_t launch_softmax_fwd_generic(const Geom& g, int dtype, const void* Q, const void* K,
                                      const void* V, void* O, float* LSE, int causal, hipStream_t st)
{
    if (dtype == LASP2_F32)
        return softmax_fwd_generic_T(g, static_cast<const float*>(Q), static_cast<const float*>(K),
                                     static_cast<const float*>(V), static_cast<float*>(O), LSE, causal, st);
    return softmax_fwd_generic_T(g, static_cast<const __hip_bfloat16*>(Q),
                                 static_cast<const __hip_bfloat16*>(K),
                                 static_cast<const __hip_bfloat16*>(V), static_cast<__hip_bfloat16*>(O),
                                 LSE, causal, st);
}

hipError_t launch_softmax_delta(const Geom& g, int dtype, const void* O, const void* dO, const float* LSE,
                                float* delta, float* lse2, hipStream_t st)
{
    const size_t rows = (size_t)g.G * (size_t)g.qn;
    if (rows == 0) return hipSuccess;
    dim3 grid((unsigned)((rows + kThreads / 64 - 1) / (kThreads / 64))), block(kThreads);
    if (dtype == LASP2_F32)
        hipLaunchKernelGGL(softmax_delta_kernel<float>, grid, block, 0, st, g, static_cast<const float*>(O),
                           static_cast<const float*>(dO), LSE, delta, lse2);
    else
        hipLaunchKernelGGL(softmax_delta_kernel<__hip_bfloat16>, grid, block, 0, st, g,
                           static_cast<const __hip_bfloat16*>(O), static_cast<const __hip_bfloat16*>(dO), LSE,
                           delta, lse2);
    return hipGetLastError();
}

hipError_t launch_softmax_bwd_generic(const Geom& g, int dtype, const void* Q, const void* K,
                                      const void* V, const void* dO, const float* LSE, const float* delta,
                                      void* dQ, void* dK, void* dV, int causal, hipStream_t st)
{
    if (dtype == LASP2_F32)
        return softmax_bwd_generic_T(g, static_cast<const float*>(Q), static_cast<const float*>(K),
                                     static_cast<const float*>(V), static_cast<const float*>(dO), LSE, delta,
                                     static_cast<float*>(dQ), static_cast<float*>(dK), static_cast<float*>(dV),
                                     causal, st);
    typedef __hip_bfloat16 bf;
    return softmax_bwd_generic_T(g, static_cast<const bf*>(Q), static_cast<const bf*>(K),
                                 static_cast<const bf*>(V), static_cast<const bf*>(dO), LSE, delta,
                                 static_cast<bf*>(dQ), static_cast<bf*>(dK), static_cast<bf*>(dV), causal, st);
}

hipError_t launch_state_total(const Geom& g, const float* M, float* S, hipStream_t st)
{
    const int dd = g.d * g.d;
    dim3 grid((dd / 4 + kThreads - 1) / kThreads, g.G), block(kThreads);
    hipLaunchKernelGGL(state_total_kernel, grid, block, 0, st, g, M, S);
    return hipGetLastError();
}

hipError_t launch_rows_state_generic(const Geom& g, int dtype, const void* A, const float* state,
                                     void* out, int transpose_state, hipStream_t st)
{
    if (dtype == LASP2_F32)
        return rows_state_generic_T(g, static_cast<const float*>(A), state, static_cast<float*>(out),
                                    transpose_state, st);
    return rows_state_generic_T(g, static_cast<const __hip_bfloat16*>(A), state,
                                static_cast<__hip_bfloat16*>(out), transpose_state, st);
}

hipError_t launch_state_prefix(const Geom& g, const float* M, float* P, int reverse, int inclusive,
                               hipStream_t st)
{
    const int dd = g.d * g.d;
    dim3 grid((dd / 4 + kThreads - 1) / kThreads, g.G), block(kThreads);
    hipLaunchKernelGGL(state_prefix_kernel, grid, block, 0, st, g, M, P, reverse, inclusive);
    return hipGetLastError();
}

}  // namespace lasp2
