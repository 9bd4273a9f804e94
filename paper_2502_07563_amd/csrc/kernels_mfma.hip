// bf16 MFMA kernels of liblasp2 for gfx950 (d = 128): chunk states and the fused
// intra + inter attention pass.  One workgroup walks the chunks of one state slot and
// carries the running d x d state in fp32 MFMA accumulators.
//
// Operand conventions (v_mfma_f32_32x32x16_bf16, wave of 64 lanes, h = lane/32):
//   A (32 x 16): lane holds row lane%32, k = 8h .. 8h+7
//   B (16 x 32): lane holds column lane%32, k = 8h .. 8h+7
//   C/D (32 x 32): lane holds column lane%32, rows 8*(v/4) + 4h + v%4 for v = 0..15
// Row-major [token][d] tiles serve directly when the contraction runs over d (16-byte
// LDS reads).  When it runs over tokens, ds_read_b64_tr_b16 fetches, for a 16-lane
// group, four consecutive rows of 16 columns and hands lane i the column i of those
// four rows, which is exactly four consecutive k of an operand.
//
// LDS tiles have 256-byte rows (128 bf16) with their 16-byte chunks XOR-swizzled by
// swz(row), which keeps both access shapes free of bank conflicts without padding.
#include "lasp2_common.h"

namespace lasp2 {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

constexpr int D = 128;
constexpr int ROWB = D * 2;          // bytes per tile row
constexpr int KB = 64;               // tokens per LDS stage
constexpr int STAGE_BYTES = KB * ROWB;  // one tensor, one stage: 16 KiB
constexpr int CHUNKS_PER_STAGE = KB * 16;  // 16-byte pieces per tensor per stage

__device__ __forceinline__ int swz(int row) { return ((row & 3) << 2) | ((row >> 2) & 3); }

// byte offset of 16-byte chunk `chunk` (0..15) of row `row` inside a swizzled tile
__device__ __forceinline__ int tile_off(int row, int chunk)
{
    return row * ROWB + (((chunk ^ swz(row)) & 15) << 4);
}

__device__ __forceinline__ bf16x8 lds_read16(const char* tile, int row, int chunk)
{
    return *reinterpret_cast<const bf16x8*>(tile + tile_off(row, chunk));
}

// Transposed fetch of 8 k-values for an MFMA operand whose k axis is the tile's row axis.
// The lane's non-contracted index is column `col0 + lane%32`; its k-slots 0..3 are rows
// rowA..rowA+3 and k-slots 4..7 rows rowB..rowB+3 (row bases already include the lane's h).
__device__ __forceinline__ bf16x8 lds_read_tr8(const char* tile, int rowA, int rowB, int col0, int lane)
{
    const int i = lane & 15, g2 = (lane >> 4) & 1;
    const int col = col0 + 16 * g2 + 4 * (i & 3);   // first of the 4 columns this lane's address covers
    const int chunk = col >> 3, within = (col & 7) * 2;
    const int r1 = rowA + (i >> 2), r2 = rowB + (i >> 2);
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + tile_off(r1, chunk) + within));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(tile + tile_off(r2, chunk) + within));
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

__device__ __forceinline__ f32x16 mfma(bf16x8 a, bf16x8 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

__device__ __forceinline__ uint32_t pack2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    bf16x2 p = {(__bf16)lo, (__bf16)hi};
    return __builtin_bit_cast(uint32_t, p);
}

// ---- global -> register -> LDS staging of one 64-token block of two [token][128] tensors ----
template <int NT>
struct BlockRegs {
    static constexpr int LPT = CHUNKS_PER_STAGE / NT;
    u32x4 x[LPT], y[LPT];
};

// Rows at or beyond `len` (slot-relative token index) read as zero and are never dereferenced.
template <int NT>
__device__ __forceinline__ void load_block(BlockRegs<NT>& r, const char* X, const char* Y,
                                           size_t row0_bytes, int tok, int len, int tid)
{
#pragma unroll
    for (int u = 0; u < BlockRegs<NT>::LPT; ++u) {
        const int idx = tid + u * NT;
        const int row = idx >> 4, chunk = idx & 15;
        const bool ok = (tok + row) < len;
        const size_t off = row0_bytes + (size_t)(tok + row) * ROWB + chunk * 16;
        u32x4 z = {0u, 0u, 0u, 0u};
        r.x[u] = ok ? *reinterpret_cast<const u32x4*>(X + off) : z;
        r.y[u] = ok ? *reinterpret_cast<const u32x4*>(Y + off) : z;
    }
}

template <int NT>
__device__ __forceinline__ void store_block(const BlockRegs<NT>& r, char* tx, char* ty, int tid)
{
#pragma unroll
    for (int u = 0; u < BlockRegs<NT>::LPT; ++u) {
        const int idx = tid + u * NT;
        const int row = idx >> 4, chunk = idx & 15;
        const int o = tile_off(row, chunk);
        *reinterpret_cast<u32x4*>(tx + o) = r.x[u];
        *reinterpret_cast<u32x4*>(ty + o) = r.y[u];
    }
}

// acc[u] += X_blk^T Y_blk restricted to the 32x32 tile (a, b) = ((t0+u)/4, (t0+u)%4) of the
// d x d state, for the 64 tokens of one LDS stage.
template <int TPW>
__device__ __forceinline__ void update_tiles(f32x16 (&acc)[TPW], const char* tx, const char* ty,
                                             int t0, int lane)
{
    const int h = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < KB / 16; ++ks) {
        const int rA = 16 * ks + 8 * h, rB = rA + 4;
        bf16x8 aop[TPW];
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int a = (t0 + u) >> 2;
            if (u == 0 || ((t0 + u) & 3) == 0) aop[u] = lds_read_tr8(tx, rA, rB, 32 * a, lane);
            else aop[u] = aop[u - 1];
        }
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int b = (t0 + u) & 3;
            bf16x8 bop = lds_read_tr8(ty, rA, rB, 32 * b, lane);
            acc[u] = mfma(aop[u], bop, acc[u]);
        }
    }
}

// =====================================================================================
// Chunk states: M[slot] = X^T Y over the slot's tokens (X = K, Y = V; or Q, dO).
// =====================================================================================
constexpr int ST_NW = 8, ST_NT = ST_NW * 64, ST_TPW = 16 / ST_NW;

__global__ __launch_bounds__(ST_NT) void states_mfma_kernel(Geom g, const char* __restrict__ X,
                                                            const char* __restrict__ Y,
                                                            float* __restrict__ M)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sX = smem;                     // 2 stages
    char* sY = smem + 2 * STAGE_BYTES;   // 2 stages
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int s = blockIdx.x, grp = blockIdx.y;
    int tok0, len;
    slot_range(g, s, tok0, len);
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;

    f32x16 acc[ST_TPW];
#pragma unroll
    for (int u = 0; u < ST_TPW; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;

    const int nblk = (len + KB - 1) / KB;
    BlockRegs<ST_NT> regs;
    load_block<ST_NT>(regs, X, Y, row0, 0, len, tid);
    for (int blk = 0; blk < nblk; ++blk) {
        char* tx = sX + (blk & 1) * STAGE_BYTES;
        char* ty = sY + (blk & 1) * STAGE_BYTES;
        store_block<ST_NT>(regs, tx, ty, tid);
        if (blk + 1 < nblk) load_block<ST_NT>(regs, X, Y, row0, (blk + 1) * KB, len, tid);
        __syncthreads();
        update_tiles<ST_TPW>(acc, tx, ty, w * ST_TPW, lane);
    }

    float* m = M + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
    const int h = lane >> 5, l32 = lane & 31;
#pragma unroll
    for (int u = 0; u < ST_TPW; ++u) {
        const int t = w * ST_TPW + u, a = t >> 2, b = t & 3;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int row = 32 * a + 8 * (v >> 2) + 4 * h + (v & 3);
            m[row * D + 32 * b + l32] = acc[u][v];
        }
    }
}

// =====================================================================================
// Fused attention pass over one slot:
//   out_c = [(A_c Bk_c^T) (.) mask] Cv_c + A_c S_c ,   S_{c+1} = S_c + Bk_c^T Cv_c
// with S starting from the slot's prefix (or suffix) state.  C/32 waves; wave w owns 32
// rows of the chunk for the whole chunk; the chunk's Bk/Cv rows stream through LDS in
// 64-token stages shared by all waves; every wave also owns 16/NW tiles of the state.
//
// Staging: global_load_lds_dwordx4 writes each lane's 16 bytes straight into LDS at
// (M0 base) + 16*lane, so a wave instruction fills four 256-byte tile rows; the swizzle
// is applied on the global side (lane -> which 16 bytes it fetches).  A ring of three
// stages keeps two blocks (64 KiB) in flight per workgroup while a third is consumed.
// The loads are issued from inline asm, invisible to the compiler's wait-count
// tracking, and are retired by explicit s_waitcnt vmcnt(n): each wave issues DPS loads
// per stage, memory operations retire in order, and at least the DPS loads of the next
// stage were issued after those of the stage about to be read, so vmcnt(DPS) is always
// sufficient (extra loads or stores issued in between only make the wait stricter).
// =====================================================================================
constexpr int NSTAGE = 3;

__device__ __forceinline__ uint32_t lds_addr_of(const char* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

__device__ __forceinline__ void dma16(const char* gptr, uint32_t lds_base)
{
    // lds_base is the same in every lane of the wave; readfirstlane moves it to a scalar register
    const uint32_t base = __builtin_amdgcn_readfirstlane(lds_base);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(base), "v"(gptr) : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Issue the loads of one 64-token block (rows tok .. tok+63 of the slot) of X and Y into the
// stage tiles tx, ty.  Rows past the slot's end are fetched from its last row (always in
// bounds) and zeroed afterwards by zero_tail_rows().
template <int NW>
__device__ __forceinline__ void dma_block(const char* X, const char* Y, size_t row0_bytes, int tok,
                                          int len, char* tx, char* ty, int w, int lane)
{
    constexpr int IPW = 16 / NW;   // wave instructions per tensor per stage
#pragma unroll
    for (int u = 0; u < IPW; ++u) {
        const int rowbase = 4 * (w * IPW + u);
        const int r = rowbase + (lane >> 4);
        const int lc = (lane & 15) ^ swz(r);
        const int gr = min(tok + r, len - 1);
        const size_t off = row0_bytes + (size_t)gr * ROWB + lc * 16;
        dma16(X + off, lds_addr_of(tx + rowbase * ROWB));
        dma16(Y + off, lds_addr_of(ty + rowbase * ROWB));
    }
}

template <int NW>
__device__ __forceinline__ void zero_tail_rows(int tok, int len, char* tx, char* ty, int w, int lane)
{
    constexpr int IPW = 16 / NW;
#pragma unroll
    for (int u = 0; u < IPW; ++u) {
        const int r = 4 * (w * IPW + u) + (lane >> 4);
        if (tok + r >= len) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(tx + r * ROWB + (lane & 15) * 16) = z;
            *reinterpret_cast<u32x4*>(ty + r * ROWB + (lane & 15) * 16) = z;
        }
    }
}

template <int C>
__global__ __launch_bounds__(C * 2) void attn_mfma_kernel(Geom g, const char* __restrict__ A,
                                                          const char* __restrict__ Bk,
                                                          const char* __restrict__ Cv,
                                                          const float* __restrict__ state,
                                                          char* __restrict__ out,
                                                          int transpose_state, int reverse)
{
    constexpr int NW = C / 32, TPW = 16 / NW, BPC = C / KB;
    constexpr int DPS = 2 * (16 / NW);     // loads per wave per stage
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;                              // Bk stages
    char* sV = smem + NSTAGE * STAGE_BYTES;       // Cv stages
    char* sM = smem + 2 * NSTAGE * STAGE_BYTES;   // state snapshot, bf16 [d_v][d_k]

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    const int s = blockIdx.x, grp = blockIdx.y;
    int tok0, len;
    slot_range(g, s, tok0, len);
    if (len <= 0) return;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;

    // Row block of this wave.  With 8 waves, waves w and w+4 (which share a SIMD under
    // round-robin placement) get blocks s and 7-s, so that their triangular work adds up evenly.
    const int rb = (NW == 8) ? (w < 4 ? w : 11 - w) : w;
    const int t0 = w * TPW;

    const int nch = (len + C - 1) / C;
    const int nblk_tail = ((len - (nch - 1) * C) + KB - 1) / KB;   // blocks of the (ragged) last chunk
    const int NB = (nch - 1) * BPC + nblk_tail;                     // blocks in the whole slot
    // slot-relative first token of the i-th block in walk order
    auto tok_of = [&](int i) -> int {
        if (!reverse) return i * KB;
        if (i < nblk_tail) return (nch - 1) * C + i * KB;
        const int j = i - nblk_tail;
        return (nch - 2 - j / BPC) * C + (j % BPC) * KB;
    };
    auto issue = [&](int i) {
        dma_block<NW>(Bk, Cv, row0, tok_of(i), len, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, lane);
    };
    issue(0);
    if (NB > 1) issue(1);

    // running state tiles, C/D layout: rows = d_k (first index), columns = d_v
    f32x16 Macc[TPW];
    {
        const float* st = state + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
            if (!transpose_state) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    Macc[u][v] = st[(32 * a + 8 * (v >> 2) + 4 * h + (v & 3)) * D + 32 * b + l32];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 x = *reinterpret_cast<const f32x4*>(st + (32 * b + l32) * D + 32 * a + 8 * q + 4 * h);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Macc[u][4 * q + e] = x[e];
                }
            }
        }
    }

    bf16x8 qf[8];   // this wave's 32 rows of A as B-operand fragments (column = row of A, k = d)
    auto load_q = [&](int c) {
        const int r = c * C + 32 * rb + l32;
        const bool ok = r < len;
        const char* p = A + row0 + (size_t)r * ROWB + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            u32x4 z = {0u, 0u, 0u, 0u};
            u32x4 x = ok ? *reinterpret_cast<const u32x4*>(p + 32 * ks) : z;
            qf[ks] = __builtin_bit_cast(bf16x8, x);
        }
    };
    load_q(reverse ? nch - 1 : 0);

    int bi = 0;          // index of the block being consumed, in walk order
    int prev_nblk = 0;
    for (int ci = 0; ci < nch; ++ci) {
        const int c = reverse ? nch - 1 - ci : ci;
        const int cn = reverse ? c - 1 : c + 1;          // next chunk in walk order
        const int nblk = (c == nch - 1) ? nblk_tail : BPC;
        const bool last_chunk = (ci + 1 == nch);

        // The previous chunk read the snapshot in its first block; a later block barrier has
        // separated that from this write unless the chunk had a single block.
        if (ci > 0 && prev_nblk < 2) __syncthreads();
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
            const int row = 32 * b + l32;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 pk = {pack2(Macc[u][4 * q], Macc[u][4 * q + 1]), pack2(Macc[u][4 * q + 2], Macc[u][4 * q + 3])};
                *reinterpret_cast<u32x2*>(sM + tile_off(row, 4 * a + q) + 8 * h) = pk;
            }
        }

        f32x16 Oacc[4];
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;

        for (int jb = 0; jb < nblk; ++jb, ++bi) {
            char* tK = sK + (bi % NSTAGE) * STAGE_BYTES;
            char* tV = sV + (bi % NSTAGE) * STAGE_BYTES;
            // this wave's loads of block bi have landed (those of bi+1 may still fly)
            if (bi + 1 < NB) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
            const int tok = tok_of(bi);
            if (tok + KB > len) zero_tail_rows<NW>(tok, len, tK, tV, w, lane);
            __syncthreads();   // block bi complete in LDS; every wave is past block bi-1
            if (bi + 2 < NB) issue(bi + 2);

            if (jb == 0) {
                // inter-chunk term: out^T += S^T A^T  with S^T = snapshot [d_v][d_k]
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
#pragma unroll
                    for (int tv = 0; tv < 4; ++tv)
                        Oacc[tv] = mfma(lds_read16(sM, 32 * tv + l32, 2 * ks + h), qf[ks], Oacc[tv]);
            }

#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int kt = 2 * jb + half;      // 32-key tile index inside the chunk
                const bool active = reverse ? (kt >= rb) : (kt <= rb);
                if (!active) continue;
                // scores^T (keys x queries) = Bk_tile A_w^T
                f32x16 sc;
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    sc = mfma(lds_read16(tK, 32 * half + l32, 2 * ks + h), qf[ks], sc);
                if (kt == rb) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = 8 * (v >> 2) + 4 * h + (v & 3);
                        const bool keep = reverse ? (key >= l32) : (key <= l32);
                        sc[v] = keep ? sc[v] : 0.f;
                    }
                }
                // out^T (d_v x queries) += Cv_tile^T scores^T ; k-slots follow the C/D row order
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    u32x4 pk = {pack2(sc[8 * k2 + 0], sc[8 * k2 + 1]), pack2(sc[8 * k2 + 2], sc[8 * k2 + 3]),
                                pack2(sc[8 * k2 + 4], sc[8 * k2 + 5]), pack2(sc[8 * k2 + 6], sc[8 * k2 + 7])};
                    bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
                    const int rA = 32 * half + 16 * k2 + 4 * h, rB = rA + 8;
#pragma unroll
                    for (int tv = 0; tv < 4; ++tv)
                        Oacc[tv] = mfma(lds_read_tr8(tV, rA, rB, 32 * tv, lane), sb, Oacc[tv]);
                }
            }

            // the rows of the next chunk replace qf while the state update and the store run
            if (jb + 1 == nblk && !last_chunk) load_q(cn);
            if (!last_chunk) update_tiles<TPW>(Macc, tK, tV, t0, lane);
        }
        prev_nblk = nblk;

        // out rows of this wave: lane owns query row l32, 4 consecutive d_v per (tv, q)
        {
            const int r = c * C + 32 * rb + l32;
            if (r < len) {
                char* p = out + row0 + (size_t)r * ROWB + 8 * h;
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
#pragma unroll
                    for (int q = 0; q < 4; ++q) {
                        u32x2 pk = {pack2(Oacc[tv][4 * q], Oacc[tv][4 * q + 1]),
                                    pack2(Oacc[tv][4 * q + 2], Oacc[tv][4 * q + 3])};
                        *reinterpret_cast<u32x2*>(p + 64 * tv + 16 * q) = pk;
                    }
            }
        }
    }
}

template <int C>
hipError_t launch_attn_C(const Geom& g, const void* A, const void* Bk, const void* Cv,
                         const float* state, void* out, int tr, int rev, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + D * ROWB;   // 128 KiB
    auto kern = attn_mfma_kernel<C>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    dim3 grid(g.T_s, g.G), block(C * 2);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, static_cast<const char*>(A),
                       static_cast<const char*>(Bk), static_cast<const char*>(Cv), state,
                       static_cast<char*>(out), tr, rev);
    return hipGetLastError();
}

}  // namespace

bool mfma_path_supported(const Geom& g, int dtype)
{
    return dtype == LASP2_BF16 && g.d == D && (g.C == 256 || g.C == 128);
}

hipError_t launch_states_mfma(const Geom& g, const void* K, const void* V, float* M, hipStream_t st)
{
    constexpr int smem = 4 * STAGE_BYTES;   // 64 KiB
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(states_mfma_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, smem);
    if (e != hipSuccess) return e;
    dim3 grid(g.T_s, g.G), block(ST_NT);
    hipLaunchKernelGGL(states_mfma_kernel, grid, block, smem, st, g, static_cast<const char*>(K),
                       static_cast<const char*>(V), M);
    return hipGetLastError();
}

hipError_t launch_attn_mfma(const Geom& g, const void* A, const void* Bk, const void* Cv,
                            const float* state, void* out, int transpose_state, int reverse,
                            hipStream_t st)
{
    if (g.C == 256) return launch_attn_C<256>(g, A, Bk, Cv, state, out, transpose_state, reverse, st);
    return launch_attn_C<128>(g, A, Bk, Cv, state, out, transpose_state, reverse, st);
}

}  // namespace lasp2
