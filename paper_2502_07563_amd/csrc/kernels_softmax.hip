// Softmax attention (the standard-attention layers of the hybrid model) on the matrix cores,
// bf16, d = 128: forward, and the two backward kernels (dQ; dK and dV).  The tile layout, the LDS
// read shapes and the stage ring are those of the linear-attention kernels (mfma_tile.h).
#include "mfma_tile.h"

namespace lasp2 {
namespace {

// =====================================================================================
// Softmax attention forward, O = Softmax(Q K^T / sqrt(d)) V over the keys of the query's document
// (optionally causal): the local computation of AllGather-based context parallelism, K and V
// being whole in HBM.  One workgroup (8 waves x 32 rows) per block of 256 queries; the keys
// stream through the same ring of 64-token LDS stages as in the fused linear pass, scores^T
// tiles (keys x queries) come from the same MFMA sequence, and the softmax runs online per
// query, which in this orientation is per lane: lanes l and l+32 hold the two halves of the
// keys of one query, so a row maximum is 16 register maxima and one cross-lane exchange, the
// running sum stays a per-lane partial until the end, and rescaling the output accumulators
// is a per-lane scalar.  exp2 with the scale folded in; masked scores are -inf.
// Document and causal bounds are per query [lo, hi); a 32-key tile is skipped, taken whole or
// masked element-wise depending on how it lies against the bounds of the wave's 32 queries.
// =====================================================================================
constexpr int SM_NW = 8, SM_QB = SM_NW * 32;

__device__ __forceinline__ float xor32(float x)
{
    return __shfl_xor(x, 32, 64);
}

// 2^x by the hardware instruction alone: arguments here are <= 0 up to rounding (scores minus a
// maximum or a log-sum-exp), results below the smallest normal number may flush to zero, and
// -inf gives 0.  (exp2f adds range scaling for denormal results: four more instructions per call.)
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ int wave_min_i(int x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = min(x, __shfl_xor(x, o, 64));
    return x;
}

__device__ __forceinline__ int wave_max_i(int x)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) x = max(x, __shfl_xor(x, o, 64));
    return x;
}

// document [lo, hi) that holds token i (unpacked: the whole sequence)
__device__ __forceinline__ void doc_range(const Geom& g, int i, int& lo, int& hi)
{
    lo = 0;
    hi = g.N;
    if (g.n_seqs == 0) return;
    int a = 0, b = g.n_seqs;          // cu[a] <= i < cu[b]
    while (b - a > 1) {
        const int m = (a + b) >> 1;
        if (g.cu[m] <= i) a = m; else b = m;
    }
    lo = g.cu[a];
    hi = g.cu[a + 1];
}

__global__ __launch_bounds__(SM_NW * 64) void softmax_fwd_mfma_kernel(Geom g, const char* __restrict__ Q,
                                                                      const char* __restrict__ K,
                                                                      const char* __restrict__ V,
                                                                      char* __restrict__ O,
                                                                      float* __restrict__ LSE, int causal,
                                                                      float scale_log2e)
{
    constexpr int NW = SM_NW, DPS = 2 * (16 / NW);
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;
    char* sV = smem + NSTAGE * STAGE_BYTES;
    char* sO = smem + 2 * NSTAGE * STAGE_BYTES;   // output staging, 4 KiB per wave

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    // Units (group, query block) are numbered group-major with the later (for a causal mask:
    // heavier) query blocks first, and each XCD takes a contiguous range of them, so that the
    // workgroups resident on an XCD mostly share a group's keys in its L2.
    const int nqb = (g.qn + SM_QB - 1) / SM_QB;
    const unsigned units = (unsigned)g.G * (unsigned)nqb;
    const unsigned per_xcd = (units + 7u) / 8u;
    const unsigned unit = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || unit >= units) return;
    const int grp = (int)(unit / (unsigned)nqb);
    const int qb = nqb - 1 - (int)(unit % (unsigned)nqb);
    const int rl0 = qb * SM_QB;                      // first query row of the workgroup (row of Q, O)
    const int qend = g.q0 + g.qn;                    // one past the last query token of the call
    const int r0 = g.q0 + rl0;                       // ... as a token of the sequence
    const int rlast = min(r0 + SM_QB, qend) - 1;
    const size_t base = (size_t)grp * g.N * ROWB;    // K, V
    const size_t qbase = (size_t)grp * g.qn * ROWB;  // Q, O

    // key range of the workgroup (uniform) and bounds of this lane's query
    int blo, bhi, tmp;
    doc_range(g, r0, blo, tmp);
    doc_range(g, rlast, tmp, bhi);
    if (causal) bhi = rlast + 1;
    const int qi = r0 + 32 * w + l32;                // this lane's query
    int lo_i = 0, hi_i = 0;                          // empty range for rows past the end
    if (qi < qend) {
        doc_range(g, qi, lo_i, hi_i);
        if (causal) hi_i = qi + 1;
    }
    // bounds over the wave's valid queries, for the per-tile decision
    const bool valid = qi < qend;
    const int lo_min = __builtin_amdgcn_readfirstlane(wave_min_i(valid ? lo_i : g.N));
    const int lo_max = __builtin_amdgcn_readfirstlane(wave_max_i(valid ? lo_i : 0));
    const int hi_min = __builtin_amdgcn_readfirstlane(wave_min_i(valid ? hi_i : g.N));
    const int hi_max = __builtin_amdgcn_readfirstlane(wave_max_i(valid ? hi_i : 0));

    const int kb0 = blo / KB, kb1 = (bhi + KB - 1) / KB;   // key blocks [kb0, kb1)
    const int NBK = kb1 - kb0;
    uint32_t dvo[16 / NW];
#pragma unroll
    for (int u = 0; u < 16 / NW; ++u) dvo[u] = dma_lane_off(w * (16 / NW) + u, lane);
    auto issue = [&](int i) {
        dma_block<NW>(K, V, base, (kb0 + i) * KB, g.N, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, lane, dvo);
    };
    issue(0);
    if (NBK > 1) issue(1);

    // per-lane LDS addresses of the natural reads (K stages) and the transposed reads (V stages)
    // inside ring slot 0, first half; slot and half are added as immediates at the point of use
    uint32_t nat[8], pv[4][2];
    {
        const int i = lane & 15, g2 = (lane >> 4) & 1;
        const int cl = 16 * g2 + 4 * (i & 3), rl = i >> 2;
        const uint32_t aK = lds_addr_of(sK), aV = lds_addr_of(sV);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) nat[ks] = aK + tile_off(l32, 2 * ks + h);
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) {
            pv[tv][0] = aV + tr_off(4 * h + rl, 32 * tv + cl);
            pv[tv][1] = aV + tr_off(8 + 4 * h + rl, 32 * tv + cl);
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) pin_vgpr(nat[ks]);
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) { pin_vgpr(pv[tv][0]); pin_vgpr(pv[tv][1]); }
    }

    // this wave's 32 queries as B-operand fragments (column = query, k = d); zero past the end
    bf16x8 qf[8];
    {
        const char* p = Q + qbase + (size_t)(min(qi, qend - 1) - g.q0) * ROWB + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            const u32x4 x = *reinterpret_cast<const u32x4*>(p + 32 * ks);
            qf[ks] = __builtin_bit_cast(bf16x8, valid ? x : z);
        }
    }

    f32x16 Oacc[4];
#pragma unroll
    for (int tv = 0; tv < 4; ++tv)
#pragma unroll
        for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;
    float m = -INFINITY;   // running maximum of scale_log2e * score (shared by lanes l, l+32)
    float lsum = 0.f;      // this lane's part of the running sum of exp2(. - m)

    // One key block.  The ring slot is a compile-time constant (the block loop below is unrolled
    // by the ring length), which turns every LDS address into a per-lane register plus an
    // immediate offset: no address arithmetic in the loop.
    auto block = [&](auto stage_c, int bi) {
        constexpr int ST = decltype(stage_c)::value;
        char* tK = sK + ST * STAGE_BYTES;
        char* tV = sV + ST * STAGE_BYTES;
        const int k0b = (kb0 + bi) * KB;
        if (bi + 1 < NBK) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
        if (k0b + KB > g.N) zero_tail_rows<NW>(k0b, g.N, tK, tV, w, lane);
        __syncthreads();   // block complete in LDS; every wave is past the previous block
        if (bi + 2 < NBK) issue(bi + 2);

        bf16x8 bufA[4], bufB[4];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int k0 = k0b + 32 * half;          // first key of the tile
            if (k0 >= hi_max || k0 + 32 <= lo_min) continue;   // no query of this wave sees it
            const bool whole = (k0 >= lo_max) && (k0 + 32 <= hi_min);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_u(nat[ks] + (ST * STAGE_BYTES + half * (32 * ROWB)));
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_u(nat[ks + 4] + (ST * STAGE_BYTES + half * (32 * ROWB)));
            SCHED_FENCE();
            f32x16 sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufA[tv] = lds_read_tr8_u(pv[tv][0] + (ST * STAGE_BYTES + half * (32 * ROWB)),
                                          pv[tv][1] + (ST * STAGE_BYTES + half * (32 * ROWB)));
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufB[tv] = lds_read_tr8_u(pv[tv][0] + (ST * STAGE_BYTES + half * (32 * ROWB) + 16 * ROWB),
                                          pv[tv][1] + (ST * STAGE_BYTES + half * (32 * ROWB) + 16 * ROWB));
            SCHED_FENCE();
            if (!whole) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + 8 * (v >> 2) + 4 * h + (v & 3);
                    sc[v] = (key >= lo_i && key < hi_i) ? sc[v] : -INFINITY;
                }
            }
            // online softmax for this lane's query
            float mx = sc[0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sc[v]);
            mx = fmaxf(mx, xor32(mx));
            const float m_new = fmaxf(m, mx * scale_log2e);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;   // nothing seen yet: all terms are 0
            const float alpha = fast_exp2(m - m_use);
            float ps = 0.f;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                sc[v] = fast_exp2(fmaf(sc[v], scale_log2e, -m_use));
                ps += sc[v];
            }
            lsum = fmaf(lsum, alpha, ps);
            if (__any(m_new > m)) {
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
#pragma unroll
                    for (int v = 0; v < 16; ++v) Oacc[tv][v] *= alpha;
            }
            m = m_new;
            {
                u32x4 pk = {pack2(sc[0], sc[1]), pack2(sc[2], sc[3]), pack2(sc[4], sc[5]), pack2(sc[6], sc[7])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufA[tv], sb, Oacc[tv]);
            }
            {
                u32x4 pk = {pack2(sc[8], sc[9]), pack2(sc[10], sc[11]), pack2(sc[12], sc[13]), pack2(sc[14], sc[15])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufB[tv], sb, Oacc[tv]);
            }
            SCHED_FENCE();
        }
    };
    static_assert(NSTAGE == 3, "the block loop is unrolled by the ring length");
    for (int bi = 0; bi < NBK; bi += 3) {
        block(std::integral_constant<int, 0>{}, bi);
        if (bi + 1 < NBK) block(std::integral_constant<int, 1>{}, bi + 1);
        if (bi + 2 < NBK) block(std::integral_constant<int, 2>{}, bi + 2);
    }

    // normalise, write the log-sum-exp, store through the wave's LDS patch
    const float ltot = lsum + xor32(lsum);
    const float inv = ltot > 0.f ? 1.f / ltot : 0.f;
    if (valid && h == 0) LSE[(size_t)grp * g.qn + (qi - g.q0)] = (m + log2f(ltot)) * 0.6931471805599453f;
    {
        char* stg = sO + w * 4096;
        const int rbase = rl0 + 32 * w;
#pragma unroll
        for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
            for (int tvv = 0; tvv < 2; ++tvv)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& o = Oacc[2 * hv + tvv];
                    u32x2 pk = {pack2(o[4 * q] * inv, o[4 * q + 1] * inv), pack2(o[4 * q + 2] * inv, o[4 * q + 3] * inv)};
                    *reinterpret_cast<u32x2*>(stg + l32 * 128 + (((4 * tvv + q) ^ (l32 & 7)) << 4) + 8 * h) = pk;
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = lane + 64 * i, row = idx >> 3, ch = idx & 7;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stg + row * 128 + ((ch ^ (row & 7)) << 4));
                if (rbase + row < g.qn)
                    *reinterpret_cast<u32x4*>(O + qbase + (size_t)(rbase + row) * ROWB + 128 * hv + 16 * ch) = v;
            }
        }
    }
}

// =====================================================================================
// Softmax attention backward, dQ: the forward's walk again (one workgroup per 256 queries, keys
// and values streamed), with the probabilities rebuilt from the stored log-sum-exp instead of
// an online maximum:  P = exp(s - lse_i), dP = V_tile dO_w^T, dS = P (dP - delta_i) / sqrt(d),
// dQ^T += K_tile^T dS.  Everything per query is per lane, as in the forward.
// =====================================================================================
__global__ __launch_bounds__(SM_NW * 64) void softmax_bwd_dq_mfma_kernel(
    Geom g, const char* __restrict__ Q, const char* __restrict__ K, const char* __restrict__ V,
    const char* __restrict__ dO, const float* __restrict__ LSE, const float* __restrict__ delta,
    char* __restrict__ dQ, int causal, float scale_log2e, float scale)
{
    constexpr int NW = SM_NW, DPS = 2 * (16 / NW);
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;
    char* sV = smem + NSTAGE * STAGE_BYTES;
    char* sO = smem + 2 * NSTAGE * STAGE_BYTES;   // output staging, 4 KiB per wave

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const int nqb = (g.qn + SM_QB - 1) / SM_QB;
    const unsigned units = (unsigned)g.G * (unsigned)nqb;
    const unsigned per_xcd = (units + 7u) / 8u;
    const unsigned unit = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || unit >= units) return;
    const int grp = (int)(unit / (unsigned)nqb);
    const int qb = nqb - 1 - (int)(unit % (unsigned)nqb);
    const int rl0 = qb * SM_QB;                      // first query row (row of Q, dO, dQ)
    const int qend = g.q0 + g.qn;
    const int r0 = g.q0 + rl0;                       // ... as a token of the sequence
    const int rlast = min(r0 + SM_QB, qend) - 1;
    const size_t base = (size_t)grp * g.N * ROWB;    // K, V
    const size_t qbase = (size_t)grp * g.qn * ROWB;  // Q, dO, dQ

    int blo, bhi, tmp;
    doc_range(g, r0, blo, tmp);
    doc_range(g, rlast, tmp, bhi);
    if (causal) bhi = rlast + 1;
    const int qi = r0 + 32 * w + l32;
    const bool valid = qi < qend;
    int lo_i = 0, hi_i = 0;
    if (valid) {
        doc_range(g, qi, lo_i, hi_i);
        if (causal) hi_i = qi + 1;
    }
    const int lo_min = __builtin_amdgcn_readfirstlane(wave_min_i(valid ? lo_i : g.N));
    const int lo_max = __builtin_amdgcn_readfirstlane(wave_max_i(valid ? lo_i : 0));
    const int hi_min = __builtin_amdgcn_readfirstlane(wave_min_i(valid ? hi_i : g.N));
    const int hi_max = __builtin_amdgcn_readfirstlane(wave_max_i(valid ? hi_i : 0));

    const int kb0 = blo / KB, kb1 = (bhi + KB - 1) / KB;
    const int NBK = kb1 - kb0;
    uint32_t dvo[16 / NW];
#pragma unroll
    for (int u = 0; u < 16 / NW; ++u) dvo[u] = dma_lane_off(w * (16 / NW) + u, lane);
    auto issue = [&](int i) {
        dma_block<NW>(K, V, base, (kb0 + i) * KB, g.N, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, lane, dvo);
    };
    issue(0);
    if (NBK > 1) issue(1);

    // lane offsets of the natural and the transposed reads; the other k-steps and column blocks
    // differ from these only in address bits 5..7, which the row term leaves clear, so they are
    // derived with one XOR at the point of use instead of being held in registers
    // per-lane LDS addresses inside ring slot 0, first half: natural reads of the K and V tiles
    // (row = key) and transposed reads of the K tile (row = d); slot, half and k-step are added
    // as immediates at the point of use
    uint32_t natK[8], natV[8], trK[4][2];
    {
        const int i = lane & 15, g2 = (lane >> 4) & 1;
        const int cl = 16 * g2 + 4 * (i & 3), rl = i >> 2;
        const uint32_t aK = lds_addr_of(sK), aV = lds_addr_of(sV);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            natK[ks] = aK + tile_off(l32, 2 * ks + h);
            natV[ks] = aV + tile_off(l32, 2 * ks + h);
            pin_vgpr(natK[ks]);
            pin_vgpr(natV[ks]);
        }
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) {
            trK[tv][0] = aK + tr_off(4 * h + rl, 32 * tv + cl);
            trK[tv][1] = aK + tr_off(8 + 4 * h + rl, 32 * tv + cl);
            pin_vgpr(trK[tv][0]);
            pin_vgpr(trK[tv][1]);
        }
    }

    // this wave's 32 queries and their dO rows as B-operand fragments; zero past the end
    bf16x8 qf[8], gf[8];
    {
        const size_t ro = qbase + (size_t)(min(qi, qend - 1) - g.q0) * ROWB + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            const u32x4 x = *reinterpret_cast<const u32x4*>(Q + ro + 32 * ks);
            const u32x4 y = *reinterpret_cast<const u32x4*>(dO + ro + 32 * ks);
            qf[ks] = __builtin_bit_cast(bf16x8, valid ? x : z);
            gf[ks] = __builtin_bit_cast(bf16x8, valid ? y : z);
        }
    }
    const size_t li = (size_t)grp * g.qn + (min(qi, qend - 1) - g.q0);
    float lse2 = LSE[li] * 1.4426950408889634f;   // log2 of the row's sum of exponentials
    float dlt = delta[li];
    // Use both here, before the walk: the compiler waits for a loaded value at its first use with
    // vmcnt(0), and a first use inside the loop would put that wait, which also drains every
    // stage load in flight, into every tile.
    asm volatile("" : "+v"(lse2), "+v"(dlt));

    f32x16 Oacc[4];
#pragma unroll
    for (int tv = 0; tv < 4; ++tv)
#pragma unroll
        for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;

    // One key block; the ring slot is a compile-time constant (the loop below is unrolled by the
    // ring length), so every LDS read is a pinned register plus an immediate.
    auto block = [&](auto stage_c, int bi) {
        constexpr int ST = decltype(stage_c)::value;
        char* tK = sK + ST * STAGE_BYTES;
        char* tV = sV + ST * STAGE_BYTES;
        const int k0b = (kb0 + bi) * KB;
        if (bi + 1 < NBK) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
        if (k0b + KB > g.N) zero_tail_rows<NW>(k0b, g.N, tK, tV, w, lane);
        __syncthreads();
        if (bi + 2 < NBK) issue(bi + 2);

        bf16x8 bufA[4], bufB[4];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int k0 = k0b + 32 * half;
            if (k0 >= hi_max || k0 + 32 <= lo_min) continue;
            const bool whole = (k0 >= lo_max) && (k0 + 32 <= hi_min);
            const uint32_t HO = ST * STAGE_BYTES + half * (32 * ROWB);
            // scores^T = K_tile Q_w^T and dP^T = V_tile dO_w^T (keys x queries)
            f32x16 sc, dp;
#pragma unroll
            for (int v = 0; v < 16; ++v) { sc[v] = 0.f; dp[v] = 0.f; }
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_u(natK[ks] + HO);
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_u(natK[ks + 4] + HO);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_u(natV[ks] + HO);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_u(natV[ks + 4] + HO);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) dp = mfma(bufA[ks], gf[ks], dp);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) bufA[tv] = lds_read_tr8_u(trK[tv][0] + HO, trK[tv][1] + HO);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) dp = mfma(bufB[ks], gf[ks + 4], dp);
            SCHED_FENCE();
            // P (dP - delta), P = exp2(scale_log2e s - lse2), zero outside the mask (the factor
            // 1/sqrt(d) of dS is applied once, to the finished sum)
            if (whole) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    sc[v] = fast_exp2(fmaf(sc[v], scale_log2e, -lse2)) * (dp[v] - dlt);
            } else {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = k0 + 8 * (v >> 2) + 4 * h + (v & 3);
                    const float arg = (key >= lo_i && key < hi_i) ? fmaf(sc[v], scale_log2e, -lse2) : -INFINITY;
                    sc[v] = fast_exp2(arg) * (dp[v] - dlt);
                }
            }
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) bufB[tv] = lds_read_tr8_u(trK[tv][0] + (HO + 16 * ROWB), trK[tv][1] + (HO + 16 * ROWB));
            SCHED_FENCE();
            {
                u32x4 pk = {pack2(sc[0], sc[1]), pack2(sc[2], sc[3]), pack2(sc[4], sc[5]), pack2(sc[6], sc[7])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufA[tv], sb, Oacc[tv]);
            }
            {
                u32x4 pk = {pack2(sc[8], sc[9]), pack2(sc[10], sc[11]), pack2(sc[12], sc[13]), pack2(sc[14], sc[15])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufB[tv], sb, Oacc[tv]);
            }
            SCHED_FENCE();
        }
    };
    static_assert(NSTAGE == 3, "the block loop is unrolled by the ring length");
    for (int bi = 0; bi < NBK; bi += 3) {
        block(std::integral_constant<int, 0>{}, bi);
        if (bi + 1 < NBK) block(std::integral_constant<int, 1>{}, bi + 1);
        if (bi + 2 < NBK) block(std::integral_constant<int, 2>{}, bi + 2);
    }

    {
        char* stg = sO + w * 4096;
        const int rbase = rl0 + 32 * w;
#pragma unroll
        for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
            for (int tvv = 0; tvv < 2; ++tvv)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& o = Oacc[2 * hv + tvv];
                    u32x2 pk = {pack2(o[4 * q] * scale, o[4 * q + 1] * scale),
                                pack2(o[4 * q + 2] * scale, o[4 * q + 3] * scale)};
                    *reinterpret_cast<u32x2*>(stg + l32 * 128 + (((4 * tvv + q) ^ (l32 & 7)) << 4) + 8 * h) = pk;
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = lane + 64 * i, row = idx >> 3, ch = idx & 7;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stg + row * 128 + ((ch ^ (row & 7)) << 4));
                if (rbase + row < g.qn)
                    *reinterpret_cast<u32x4*>(dQ + qbase + (size_t)(rbase + row) * ROWB + 128 * hv + 16 * ch) = v;
            }
        }
    }
}

// =====================================================================================
// Softmax attention backward, dK and dV: one workgroup of four waves per 128 keys (32 per wave,
// one per lane), queries and their dO rows streamed in 64-token stages together with each
// query's log-sum-exp (times log2 e, as the delta kernel leaves it in LSE2) and delta.  With scores laid out queries x keys, every per-key quantity
// (mask bounds, the K and V rows as B operands, the two accumulators' columns) is per lane:
//   S = Q_tile K_w^T, dP = dO_tile V_w^T, P = exp(S/sqrt(d) - lse), dS = P (dP - delta)/sqrt(d),
//   dV^T += dO_tile^T P,  dK^T += Q_tile^T dS.
// Four waves, one per SIMD, so that a wave may hold both accumulators and both operand sets
// (about 330 registers, the upper part in the accumulation file).
// =====================================================================================
constexpr int SK_NW = 4, SK_KB = SK_NW * 32;

// four bytes per lane, otherwise as dma16 (M0 is written and named as clobbered)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma4(const char* sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dword %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory", "m0");
}
#pragma clang diagnostic pop

__global__ __launch_bounds__(SK_NW * 64) void softmax_bwd_dkv_mfma_kernel(
    Geom g, const char* __restrict__ Q, const char* __restrict__ K, const char* __restrict__ V,
    const char* __restrict__ dO, const float* __restrict__ LSE2, const float* __restrict__ delta,
    char* __restrict__ dK, char* __restrict__ dV, int causal, float scale_log2e, float scale)
{
    constexpr int NW = SK_NW, DPS = 2 * (16 / NW) + 2;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sQ = smem;
    char* sG = smem + NSTAGE * STAGE_BYTES;
    char* sL = smem + 2 * NSTAGE * STAGE_BYTES;   // per stage: 64 lse, then 64 delta (512 bytes)

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const int nkb = (g.N + SK_KB - 1) / SK_KB;
    const unsigned units = (unsigned)g.G * (unsigned)nkb;
    const unsigned per_xcd = (units + 7u) / 8u;
    const unsigned unit = (blockIdx.x & 7u) * per_xcd + (blockIdx.x >> 3);
    if ((blockIdx.x >> 3) >= per_xcd || unit >= units) return;
    const int grp = (int)(unit / (unsigned)nkb);
    const int kb = (int)(unit % (unsigned)nkb);     // causal: the first key blocks see the most queries
    const int c0 = kb * SK_KB;
    const int clast = min(c0 + SK_KB, g.N) - 1;
    const size_t base = (size_t)grp * g.N * ROWB;    // K, V, dK, dV
    const size_t qbase = (size_t)grp * g.qn * ROWB;  // Q, dO (row r = token q0 + r)
    const int qend = g.q0 + g.qn;

    // queries this workgroup must visit (those of the call's share only), and per key (lane) the
    // queries that attend to it
    int blo, bhi, tmp;
    doc_range(g, c0, blo, tmp);
    doc_range(g, clast, tmp, bhi);
    if (causal) blo = c0;
    blo = max(blo, g.q0);
    bhi = min(bhi, qend);
    const int kj = c0 + 32 * w + l32;
    const bool valid = kj < g.N;
    int lo_j = 0, hi_j = 0;
    if (valid) {
        doc_range(g, kj, lo_j, hi_j);
        if (causal) lo_j = kj;
        lo_j = max(lo_j, g.q0);
        hi_j = min(hi_j, qend);
    }
    const int lo_max = __builtin_amdgcn_readfirstlane(wave_max_i(valid ? lo_j : g.N));
    const int hi_min = __builtin_amdgcn_readfirstlane(wave_min_i(valid ? hi_j : 0));

    // 64-row blocks of the query-side arrays, counted from the share's first row
    const int qb0 = (blo - g.q0) / KB;
    const int NBK = bhi > blo ? (bhi - g.q0 + KB - 1) / KB - qb0 : 0;
    uint32_t dvo[16 / NW];
#pragma unroll
    for (int u = 0; u < 16 / NW; ++u) dvo[u] = dma_lane_off(w * (16 / NW) + u, lane);
    const char* lse_g = reinterpret_cast<const char*>(LSE2 + (size_t)grp * g.qn);
    const char* dlt_g = reinterpret_cast<const char*>(delta + (size_t)grp * g.qn);
    auto issue = [&](int i) {
        const int st = i % NSTAGE, q0 = (qb0 + i) * KB;     // first row of the block
        dma_block<NW>(Q, dO, qbase, q0, g.qn, sQ + st * STAGE_BYTES, sG + st * STAGE_BYTES, w, lane, dvo);
        // every wave fetches the stage's 64 log2-domain lse and 64 delta values (the same bytes to the same
        // place), which keeps the number of loads in flight equal across waves
        const uint32_t vo = 4u * (uint32_t)min(q0 + lane, g.qn - 1);
        dma4(lse_g, vo, lds_addr_of(sL + st * 512));
        dma4(dlt_g, vo, lds_addr_of(sL + st * 512 + 256));
    };
    if (NBK > 0) issue(0);
    if (NBK > 1) issue(1);

    // per-lane LDS addresses inside ring slot 0, first half: natural reads of Q and dO tiles
    // (row = query), transposed reads of both (row = d), and the lane's quarter of the staged
    // log-sum-exp / delta values; slot, half and k-step are added as immediates at the use
    uint32_t natQ[8], natG[8], trQ[4][2], trG[4][2], aL;
    {
        const int i = lane & 15, g2 = (lane >> 4) & 1;
        const int cl = 16 * g2 + 4 * (i & 3), rl = i >> 2;
        const uint32_t aQ = lds_addr_of(sQ), aG = lds_addr_of(sG);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            natQ[ks] = aQ + tile_off(l32, 2 * ks + h);
            natG[ks] = aG + tile_off(l32, 2 * ks + h);
            pin_vgpr(natQ[ks]);
            pin_vgpr(natG[ks]);
        }
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) {
            trQ[tv][0] = aQ + tr_off(4 * h + rl, 32 * tv + cl);
            trQ[tv][1] = aQ + tr_off(8 + 4 * h + rl, 32 * tv + cl);
            trG[tv][0] = aG + tr_off(4 * h + rl, 32 * tv + cl);
            trG[tv][1] = aG + tr_off(8 + 4 * h + rl, 32 * tv + cl);
            pin_vgpr(trQ[tv][0]); pin_vgpr(trQ[tv][1]); pin_vgpr(trG[tv][0]); pin_vgpr(trG[tv][1]);
        }
        aL = lds_addr_of(sL) + 16 * h;
        pin_vgpr(aL);
    }

    // this wave's 32 keys: K and V rows as B-operand fragments; zero past the end
    bf16x8 kf[8], vf[8];
    {
        const size_t ro = base + (size_t)min(kj, g.N - 1) * ROWB + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            const u32x4 x = *reinterpret_cast<const u32x4*>(K + ro + 32 * ks);
            const u32x4 y = *reinterpret_cast<const u32x4*>(V + ro + 32 * ks);
            kf[ks] = __builtin_bit_cast(bf16x8, valid ? x : z);
            vf[ks] = __builtin_bit_cast(bf16x8, valid ? y : z);
        }
    }

    f32x16 Kacc[4], Vacc[4];
#pragma unroll
    for (int tv = 0; tv < 4; ++tv)
#pragma unroll
        for (int v = 0; v < 16; ++v) { Kacc[tv][v] = 0.f; Vacc[tv][v] = 0.f; }

    typedef const __attribute__((address_space(3))) f32x4* lds_f32x4_ptr;

    // One stage of 64 queries.  The ring slot is a compile-time constant (the loop below is
    // unrolled by the ring length), so every LDS read is a pinned register plus an immediate.
    auto block = [&](auto stage_c, int bi) {
        constexpr int ST = decltype(stage_c)::value;
        constexpr uint32_t SO = ST * STAGE_BYTES;
        const int row0 = (qb0 + bi) * KB;      // first row of the block in Q, dO
        const int q0b = g.q0 + row0;           // ... as a token of the sequence
        if (bi + 1 < NBK) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
        if (row0 + KB > g.qn) zero_tail_rows<NW>(row0, g.qn, sQ + SO, sG + SO, w, lane);
        __syncthreads();
        if (bi + 2 < NBK) issue(bi + 2);

        // The mask enters through the accumulators the score products start from: 0 where the
        // (query, key) pair is kept, -inf where it is not, so that P = exp2(-inf) = 0 and
        // dS = 0 * (dP - delta) = 0 there with no compare in the per-element code.  Halves inside
        // every lane's range (all but the few at mask edges) start from zeros.  One code path for
        // every block also keeps the two accumulators in place from block to block.
        // The two halves are software-pipelined so that one half's exponentials run under the
        // other's MFMAs (a workgroup has one wave per SIMD; nothing else would fill those slots).
        const bool whole0 = (q0b >= lo_max) && (q0b + 32 <= hi_min);
        const bool whole1 = (q0b + 32 >= lo_max) && (q0b + 64 <= hi_min);
        bf16x8 A0[8], B0[8], A1[8], B1[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) A0[ks] = lds_read16_u(natQ[ks] + SO);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) B0[ks] = lds_read16_u(natG[ks] + SO);
        f32x4 ls[4], dl[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            ls[q] = *reinterpret_cast<lds_f32x4_ptr>(aL + (ST * 512 + 32 * q));
            dl[q] = *reinterpret_cast<lds_f32x4_ptr>(aL + (ST * 512 + 256 + 32 * q));
        }
        SCHED_FENCE();
        // phase A: S0 = Q0 K^T, dP0 = dO0 V^T
        f32x16 sc0, dp0;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sc0[v] = 0.f; dp0[v] = 0.f; }
        if (!whole0) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int qi = q0b + 8 * (v >> 2) + 4 * h + (v & 3);
                sc0[v] = (qi >= lo_j && qi < hi_j) ? 0.f : -INFINITY;
            }
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            // the first of half 1's natural operands arrive under these products, into the
            // registers that half 0's first ones have left
            if (ks >= 4) {
                A1[ks - 4] = lds_read16_u(natQ[ks - 4] + (SO + 32 * ROWB));
                B1[ks - 4] = lds_read16_u(natG[ks - 4] + (SO + 32 * ROWB));
            }
            sc0 = mfma(A0[ks], kf[ks], sc0);
            dp0 = mfma(B0[ks], vf[ks], dp0);
            SCHED_FENCE();
        }
        // transposed operands of half 0 (into the registers its natural operands used)
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) {
            A0[tv] = lds_read_tr8_u(trQ[tv][0] + SO, trQ[tv][1] + SO);
            A0[4 + tv] = lds_read_tr8_u(trQ[tv][0] + (SO + 16 * ROWB), trQ[tv][1] + (SO + 16 * ROWB));
            B0[tv] = lds_read_tr8_u(trG[tv][0] + SO, trG[tv][1] + SO);
            B0[4 + tv] = lds_read_tr8_u(trG[tv][0] + (SO + 16 * ROWB), trG[tv][1] + (SO + 16 * ROWB));
        }
        f32x16 sc1, dp1;
#pragma unroll
        for (int v = 0; v < 16; ++v) { sc1[v] = 0.f; dp1[v] = 0.f; }
        if (!whole1) {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int qi = q0b + 32 + 8 * (v >> 2) + 4 * h + (v & 3);
                sc1[v] = (qi >= lo_j && qi < hi_j) ? 0.f : -INFINITY;
            }
        }
        SCHED_FENCE();
        // phase B: S1, dP1 on the matrix unit; P0 and P0 (dP0 - delta) on the vector unit; half 1's
        // log-sum-exp and delta replace half 0's as those are used up
        uint32_t pp0[8], pd0[8];
        f32x4 ls1[4], dl1[4];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (j < 4) {
                A1[j + 4] = lds_read16_u(natQ[j + 4] + (SO + 32 * ROWB));
                B1[j + 4] = lds_read16_u(natG[j + 4] + (SO + 32 * ROWB));
            }
            sc1 = mfma(A1[j], kf[j], sc1);
            dp1 = mfma(B1[j], vf[j], dp1);
            const int v = 2 * j;
            const float pa = fast_exp2(fmaf(sc0[v], scale_log2e, -ls[v >> 2][v & 3]));
            const float pb = fast_exp2(fmaf(sc0[v + 1], scale_log2e, -ls[v >> 2][(v & 3) + 1]));
            pp0[j] = pack2(pa, pb);
            pd0[j] = pack2(pa * (dp0[v] - dl[v >> 2][v & 3]), pb * (dp0[v + 1] - dl[v >> 2][(v & 3) + 1]));
            if (j & 1) {
                ls1[j >> 1] = *reinterpret_cast<lds_f32x4_ptr>(aL + (ST * 512 + 128 + 32 * (j >> 1)));
                dl1[j >> 1] = *reinterpret_cast<lds_f32x4_ptr>(aL + (ST * 512 + 256 + 128 + 32 * (j >> 1)));
            }
            SCHED_FENCE();
        }
        // half 1's transposed operands
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) {
            A1[tv] = lds_read_tr8_u(trQ[tv][0] + (SO + 32 * ROWB), trQ[tv][1] + (SO + 32 * ROWB));
            A1[4 + tv] = lds_read_tr8_u(trQ[tv][0] + (SO + 48 * ROWB), trQ[tv][1] + (SO + 48 * ROWB));
            B1[tv] = lds_read_tr8_u(trG[tv][0] + (SO + 32 * ROWB), trG[tv][1] + (SO + 32 * ROWB));
            B1[4 + tv] = lds_read_tr8_u(trG[tv][0] + (SO + 48 * ROWB), trG[tv][1] + (SO + 48 * ROWB));
        }
        SCHED_FENCE();
        // phase C: half 0 into dV^T, dK^T on the matrix unit; P1 and dS1 on the vector unit
        uint32_t pp1[8], pd1[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kst = j >> 2, tv = j & 3;
            const u32x4 pk = {pp0[4 * kst], pp0[4 * kst + 1], pp0[4 * kst + 2], pp0[4 * kst + 3]};
            const u32x4 dk = {pd0[4 * kst], pd0[4 * kst + 1], pd0[4 * kst + 2], pd0[4 * kst + 3]};
            Vacc[tv] = mfma(B0[4 * kst + tv], __builtin_bit_cast(bf16x8, pk), Vacc[tv]);
            Kacc[tv] = mfma(A0[4 * kst + tv], __builtin_bit_cast(bf16x8, dk), Kacc[tv]);
            const int v = 2 * j;
            const float pa = fast_exp2(fmaf(sc1[v], scale_log2e, -ls1[v >> 2][v & 3]));
            const float pb = fast_exp2(fmaf(sc1[v + 1], scale_log2e, -ls1[v >> 2][(v & 3) + 1]));
            pp1[j] = pack2(pa, pb);
            pd1[j] = pack2(pa * (dp1[v] - dl1[v >> 2][v & 3]), pb * (dp1[v + 1] - dl1[v >> 2][(v & 3) + 1]));
            SCHED_FENCE();
        }
        // phase D: half 1 into dV^T, dK^T
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int kst = j >> 2, tv = j & 3;
            const u32x4 pk = {pp1[4 * kst], pp1[4 * kst + 1], pp1[4 * kst + 2], pp1[4 * kst + 3]};
            const u32x4 dk = {pd1[4 * kst], pd1[4 * kst + 1], pd1[4 * kst + 2], pd1[4 * kst + 3]};
            Vacc[tv] = mfma(B1[4 * kst + tv], __builtin_bit_cast(bf16x8, pk), Vacc[tv]);
            Kacc[tv] = mfma(A1[4 * kst + tv], __builtin_bit_cast(bf16x8, dk), Kacc[tv]);
        }
        SCHED_FENCE();
    };
    static_assert(NSTAGE == 3, "the block loop is unrolled by the ring length");
    for (int bi = 0; bi < NBK; bi += 3) {
        block(std::integral_constant<int, 0>{}, bi);
        if (bi + 1 < NBK) block(std::integral_constant<int, 1>{}, bi + 1);
        if (bi + 2 < NBK) block(std::integral_constant<int, 2>{}, bi + 2);
    }

    // dK^T and dV^T (d x keys) -> rows of dK, dV through a 4 KiB per-wave staging area that
    // reuses the first stage (all waves are past their last tile read after the barrier)
    __syncthreads();
    {
        char* stg = smem + w * 4096;
        const int rbase = c0 + 32 * w;
#pragma unroll
        for (int which = 0; which < 2; ++which) {
            char* out = which ? dV : dK;
#pragma unroll
            for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
                for (int tvv = 0; tvv < 2; ++tvv)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        const f32x16& o = which ? Vacc[2 * hv + tvv] : Kacc[2 * hv + tvv];
                        const float f = which ? 1.f : scale;
                        u32x2 pk = {pack2(o[4 * q] * f, o[4 * q + 1] * f), pack2(o[4 * q + 2] * f, o[4 * q + 3] * f)};
                        *reinterpret_cast<u32x2*>(stg + l32 * 128 + (((4 * tvv + q) ^ (l32 & 7)) << 4) + 8 * h) = pk;
                    }
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int idx = lane + 64 * i, row = idx >> 3, ch = idx & 7;
                    const u32x4 v = *reinterpret_cast<const u32x4*>(stg + row * 128 + ((ch ^ (row & 7)) << 4));
                    if (rbase + row < g.N)
                        *reinterpret_cast<u32x4*>(out + base + (size_t)(rbase + row) * ROWB + 128 * hv + 16 * ch) = v;
                }
            }
        }
    }
}

}  // namespace

bool softmax_mfma_supported(const Geom& g, int dtype) { return dtype == LASP2_BF16 && g.d == D; }

hipError_t launch_softmax_bwd_dkv_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                       const void* dO, const float* LSE2, const float* delta, void* dK,
                                       void* dV, int causal, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + NSTAGE * 512;   // 97.5 KiB
    hipError_t e = allow_dynamic_lds<softmax_bwd_dkv_mfma_kernel>(smem);
    if (e != hipSuccess) return e;
    const unsigned nkb = ((unsigned)g.N + SK_KB - 1) / SK_KB;
    const unsigned units = (unsigned)g.G * nkb;
    const unsigned gx = 8u * ((units + 7u) / 8u);
    const float scale = 1.f / sqrtf((float)g.d);
    hipLaunchKernelGGL(softmax_bwd_dkv_mfma_kernel, dim3(gx), dim3(SK_NW * 64), smem, st, g,
                       static_cast<const char*>(Q), static_cast<const char*>(K),
                       static_cast<const char*>(V), static_cast<const char*>(dO), LSE2, delta,
                       static_cast<char*>(dK), static_cast<char*>(dV), causal,
                       1.4426950408889634f * scale, scale);
    return hipGetLastError();
}

hipError_t launch_softmax_bwd_dq_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                      const void* dO, const float* LSE, const float* delta, void* dQ,
                                      int causal, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + SM_NW * 4096;   // 128 KiB
    hipError_t e = allow_dynamic_lds<softmax_bwd_dq_mfma_kernel>(smem);
    if (e != hipSuccess) return e;
    if (g.qn == 0) return hipSuccess;
    const unsigned nqb = ((unsigned)g.qn + SM_QB - 1) / SM_QB;
    const unsigned units = (unsigned)g.G * nqb;
    const unsigned gx = 8u * ((units + 7u) / 8u);
    const float scale = 1.f / sqrtf((float)g.d);
    hipLaunchKernelGGL(softmax_bwd_dq_mfma_kernel, dim3(gx), dim3(SM_NW * 64), smem, st, g,
                       static_cast<const char*>(Q), static_cast<const char*>(K),
                       static_cast<const char*>(V), static_cast<const char*>(dO), LSE, delta,
                       static_cast<char*>(dQ), causal, 1.4426950408889634f * scale, scale);
    return hipGetLastError();
}

hipError_t launch_softmax_fwd_mfma(const Geom& g, const void* Q, const void* K, const void* V, void* O,
                                   float* LSE, int causal, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + SM_NW * 4096;   // 128 KiB
    hipError_t e = allow_dynamic_lds<softmax_fwd_mfma_kernel>(smem);
    if (e != hipSuccess) return e;
    if (g.qn == 0) return hipSuccess;
    const unsigned nqb = ((unsigned)g.qn + SM_QB - 1) / SM_QB;
    const unsigned units = (unsigned)g.G * nqb;
    const unsigned gx = 8u * ((units + 7u) / 8u);
    const float scale_log2e = 1.4426950408889634f / sqrtf((float)g.d);
    hipLaunchKernelGGL(softmax_fwd_mfma_kernel, dim3(gx), dim3(SM_NW * 64), smem, st, g,
                       static_cast<const char*>(Q), static_cast<const char*>(K),
                       static_cast<const char*>(V), static_cast<char*>(O), LSE, causal, scale_log2e);
    return hipGetLastError();
}

}  // namespace lasp2
