// Internal declarations shared by the host dispatch and the kernel files of
// liblasp2.  Nothing here is part of the public ABI (that is include/lasp2.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "lasp2.h"

namespace lasp2 {

constexpr int kDocMarks = 32;

// Problem geometry handed by value to every kernel.
struct Geom {
    int32_t G;            // B*H independent (batch, head) groups
    int32_t N;            // tokens per group
    int32_t d;            // head dimension
    int32_t C;            // chunk length
    int64_t L;            // tokens per state slot (multiple of C)
    int32_t T_s;          // slots per group
    int32_t n_seqs;       // packed: number of documents; 0 = not packed
    int32_t lone_slots;   // host decision: every document (sequence) is a single slot, so every
                          // exclusive prefix and suffix state is zero
    const int32_t* cu;    // packed: DEVICE pointer to n_seqs+1 offsets
    // packed: slots that lie before document j * doc_stride, j = 0 .. kDocMarks-1, filled on the
    // host (INT32_MAX past the last document): a kernel finds the document of a slot from the
    // nearest mark instead of counting from the first document
    int32_t doc_stride;
    int32_t doc_mark[kDocMarks];
    // The attention kernels may walk several of the caller's slots in one go (the carried state
    // at a slot boundary is that slot's prefix, so only the first one has to be read): then L and
    // T_s above describe the WALKS (L = wslots times the caller's slot length), and the caller's
    // state arrays [G][P_Ts][d][d] are indexed by the walk's first slot, see slot_range.
    // wslots = 1, P_Ts = T_s, doc_pmark = doc_mark: walks and the caller's slots are the same.
    int32_t wslots;
    int32_t P_Ts;
    int32_t doc_pmark[kDocMarks];   // the caller's slots before document j * doc_stride
    int32_t H;            // heads (group g uses decay[g % H])
    const float* decay;   // DEVICE pointer to H per-head decay factors; NULL = no decay
    int32_t decay_mfma;   // host decision: every factor is large enough for the MFMA decay kernels
    // Softmax attention only: the queries of one call are the tokens [q0, q0 + qn) of the
    // sequence (one rank's share; the whole sequence is q0 = 0, qn = N).  Arrays on the query
    // side (Q, O, LSE, dO, dQ, delta) then have qn rows per group, row r holding token q0 + r;
    // K, V, dK, dV always have N rows.
    int32_t q0, qn;
};

// log2 of the decay factor of group grp (0 when there is no decay): lam^e = exp2f(e * log2 lam).
__device__ __forceinline__ float decay_log2(const Geom& g, int grp)
{
    return g.decay ? log2f(g.decay[grp % g.H]) : 0.f;
}

// Token range [tok0, tok0+len) of slot (walk) s, and ps: the index, within the group, of the
// caller's slot that starts at tok0.  Unpacked: direct.  Packed: from the last host-made mark at
// or before s, then document by document (at most doc_stride of them; uniform scalar loads).
// Document lengths and L are below 2^31, so the slot counts are 32-bit divisions.
__device__ __forceinline__ void slot_range(const Geom& g, int s, int& tok0, int& len, int& ps)
{
    if (g.n_seqs == 0) {
        int64_t a = (int64_t)s * g.L;
        int64_t b = a + g.L;
        if (b > g.N) b = g.N;
        tok0 = (int)a;
        len = (int)(b - a);
        ps = s * g.wslots;
        return;
    }
    int j = 0;
#pragma unroll
    for (int step = kDocMarks / 2; step >= 1; step >>= 1)
        if (g.doc_mark[j + step] <= s) j += step;
    int base = g.doc_mark[j], pbase = g.doc_pmark[j];
    const uint32_t L = (uint32_t)min(g.L, (int64_t)INT32_MAX);   // a longer slot holds any document whole
    tok0 = 0;
    len = 0;
    ps = 0;
    for (int k = j * g.doc_stride; k < g.n_seqs; ++k) {
        const int a = g.cu[k], b = g.cu[k + 1];
        const int ns = (int)(((uint32_t)(b - a) + (L - 1u)) / L);
        if (s < base + ns) {
            const int64_t t0 = (int64_t)a + (int64_t)(s - base) * L;
            const int64_t t1 = min(t0 + (int64_t)L, (int64_t)b);
            tok0 = (int)t0;
            len = (int)(t1 - t0);
            ps = pbase + (s - base) * g.wslots;
            return;
        }
        base += ns;
        if (g.wslots > 1) {
            const uint32_t Lp = L / (uint32_t)g.wslots;   // exact: L is wslots times the caller's slot length
            pbase += (int)(((uint32_t)(b - a) + (Lp - 1u)) / Lp);
        } else {
            pbase += ns;
        }
    }
}

__device__ __forceinline__ void slot_range(const Geom& g, int s, int& tok0, int& len)
{
    int ps;
    slot_range(g, s, tok0, len, ps);
}

// Device ordinal of the calling thread's current device, or -1 when it cannot serve as an index
// into the small per-device caches below.
constexpr int kMaxDevices = 64;
inline int current_device_index()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return -1;
    return dev;
}

// Raises the dynamic-LDS limit of kernel Kern to `bytes` on the current device.  The runtime
// call is made once per kernel and device (and again only for a larger request), not at every
// launch: what was granted is remembered in a per-kernel array of atomics.  These caches, and
// cu_count() below, are the only things the library keeps between calls; they hold properties
// of the device, never of a problem.
template <auto Kern>
hipError_t allow_dynamic_lds(int bytes)
{
    static std::atomic<int> granted[kMaxDevices] = {};
    const int dev = current_device_index();
    if (dev >= 0 && granted[dev].load(std::memory_order_acquire) >= bytes) return hipSuccess;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(Kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    if (dev >= 0) {
        int seen = granted[dev].load(std::memory_order_relaxed);
        while (seen < bytes && !granted[dev].compare_exchange_weak(seen, bytes, std::memory_order_release)) {}
    }
    return hipSuccess;
}

// Compute units of the current device (asked once per device; 256 if the query fails).
inline int cu_count()
{
    static std::atomic<int> cached[kMaxDevices] = {};
    const int dev = current_device_index();
    int cus = dev >= 0 ? cached[dev].load(std::memory_order_relaxed) : 0;
    if (cus > 0) return cus;
    if (dev < 0 || hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0)
        cus = 256;
    if (dev >= 0) cached[dev].store(cus, std::memory_order_relaxed);
    return cus;
}

// ---- launchers implemented in the kernel files (return hipGetLastError()) ----

// Plain fp32-FMA kernels, any supported (dtype, d, C).
// anchor_start (decay only): weights lam^(token - slot start) instead of lam^(slot end - token).
hipError_t launch_states_generic(const Geom& g, int dtype, const void* K, const void* V,
                                 float* M, int anchor_start, hipStream_t st);
// out = [(A Bk^T) (.) mask] Cv + A * state, state += Bk^T Cv chunk by chunk.
//   reverse = 0: causal mask, chunks walked first to last, state = prefix;
//   reverse = 1: anti-causal mask (j >= i), chunks walked last to first, state = suffix.
//   transpose_state: the d x d slot state is read transposed.
hipError_t launch_attn_generic(const Geom& g, int dtype, const void* A, const void* Bk,
                               const void* Cv, const float* state, void* out,
                               int transpose_state, int reverse, hipStream_t st);
// inclusive = 0: P[s] excludes M[s] (the public entry point); 1: P[s] includes it.
hipError_t launch_state_prefix(const Geom& g, const float* M, float* P, int reverse, int inclusive,
                               hipStream_t st);

// S[s] = sum of M over the slots of s's document; S may alias M.
hipError_t launch_state_total(const Geom& g, const float* M, float* S, hipStream_t st);
// out = A * state[slot] (transpose_state: A * state[slot]^T), plain fp32-FMA kernel.
hipError_t launch_rows_state_generic(const Geom& g, int dtype, const void* A, const float* state,
                                     void* out, int transpose_state, hipStream_t st);

// bf16 MFMA kernels (d = 128; they tile slots in their own chunks, so any C).
bool mfma_path_supported(const Geom& g, int dtype);
hipError_t launch_states_mfma(const Geom& g, const void* K, const void* V, float* M,
                              int anchor_start, hipStream_t st);
// O = fused intra + inter pass with prefix states P.
hipError_t launch_attn_fwd_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                const float* P, void* O, hipStream_t st);
// dQ, dV, dK in one launch.  P: exclusive prefix states of K^T V (from the forward);
// dR: INCLUSIVE suffix states of Q^T dO (slot s holds the sum over slots >= s of its document);
// with decay: the EXCLUSIVE decayed suffix of the start-anchored states.
// pace: NULL, or G * T_s counters of scratch (see pace_bytes) through which the workgroups that
// share a slot's reads keep in step; the launch clears them itself.
hipError_t launch_attn_bwd_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                const void* dO, const float* P, const float* dR, unsigned* pace, void* dQ,
                                void* dK, void* dV, hipStream_t st);

// Row-times-state products of the unmasked path, up to three in one launch:
// out_i = A_i * state_i[slot] (or its transpose), i < n.
struct RowsStateProblem {
    const void* A;
    const float* state;
    void* out;
    int transpose_state;
};
hipError_t launch_rows_state_mfma(const Geom& g, const RowsStateProblem* probs, int n, hipStream_t st);

// Softmax attention forward over the whole sequence (document) of each group.
hipError_t launch_softmax_fwd_generic(const Geom& g, int dtype, const void* Q, const void* K,
                                      const void* V, void* O, float* LSE, int causal, hipStream_t st);
// delta[g][i] = dO_i . O_i (and, if lse2 != NULL, lse2[g][i] = LSE[g][i] * log2 e), then dQ, dK, dV of
// softmax attention from Q, K, V, dO, LSE, delta.  The matrix-core dK/dV kernel takes lse2.
hipError_t launch_softmax_delta(const Geom& g, int dtype, const void* O, const void* dO, const float* LSE,
                                float* delta, float* lse2, hipStream_t st);
// (dQ == NULL: only dK, dV are computed; dK == NULL: only dQ)
hipError_t launch_softmax_bwd_generic(const Geom& g, int dtype, const void* Q, const void* K,
                                      const void* V, const void* dO, const float* LSE, const float* delta,
                                      void* dQ, void* dK, void* dV, int causal, hipStream_t st);
bool softmax_mfma_supported(const Geom& g, int dtype);
hipError_t launch_softmax_bwd_dq_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                      const void* dO, const float* LSE, const float* delta, void* dQ,
                                      int causal, hipStream_t st);
hipError_t launch_softmax_bwd_dkv_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                       const void* dO, const float* LSE, const float* delta, void* dK,
                                       void* dV, int causal, hipStream_t st);
hipError_t launch_softmax_fwd_mfma(const Geom& g, const void* Q, const void* K, const void* V, void* O,
                                   float* LSE, int causal, hipStream_t st);

}  // namespace lasp2
