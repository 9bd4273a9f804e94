// bf16 MFMA kernels of liblasp2 for gfx950 (d = 128, any chunk length C): chunk states and the
// fused intra + inter attention pass of chunked linear attention, with and without decay, and
// the rows-times-state products of the unmasked form.  One workgroup walks the chunks of one
// state slot and carries the running d x d state in fp32 MFMA accumulators.  Operand
// conventions, the LDS tile layout and the stage loads are described in mfma_tile.h.
#include "mfma_tile.h"
#include <algorithm>

namespace lasp2 {
namespace {

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
// d x d state, for the NTOK tokens at the head of an LDS tile.
template <int TPW, int NTOK = KB>
__device__ __forceinline__ void update_tiles(f32x16 (&acc)[TPW], const char* tx, const char* ty,
                                             int t0, int lane)
{
    const int h = lane >> 5;
#pragma unroll
    for (int ks = 0; ks < NTOK / 16; ++ks) {
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

// The eight bf16 of a 16-byte piece times w, rounded to nearest even.
__device__ __forceinline__ u32x4 scale_bf16x8(u32x4 x, float w)
{
    u32x4 r;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        const float lo = __builtin_bit_cast(float, x[e] << 16);
        const float hi = __builtin_bit_cast(float, x[e] & 0xffff0000u);
        r[e] = pack2(lo * w, hi * w);
    }
    return r;
}

// =====================================================================================
// Chunk states: M[slot] = X^T Y over the slot's tokens (X = K, Y = V; or Q, dO).
// With decay (DECAY) the rows of X carry the token's weight lam^(slot end - token), or
// lam^(token - slot start) when anchor_start is set; the weighted row is rounded to bf16
// before the product, like every other operand of the matrix cores.
//
// The kernel only reads (2 x 256 bytes per token against 64 KiB written per slot) and does
// little arithmetic per byte.  It streams the slot through a ring of five 32-token stages
// (80 KiB of LDS, so that two workgroups share a CU and one's start-up and final store hide
// under the other's stream), filled by direct global->LDS loads marked non-temporal (the data
// is read once): four stages are on their way while a fifth is consumed.  The grid is two
// workgroups per CU; each takes several slots in turn without letting the ring run empty.
// =====================================================================================
constexpr int ST_NW = 8, ST_NT = ST_NW * 64, ST_TPW = 16 / ST_NW, ST_NST = 5;
constexpr int ST_KB = 32, ST_STAGE = ST_KB * ROWB;   // tokens and bytes (per tensor) of a stage

template <bool DECAY>
__global__ __launch_bounds__(ST_NT) void states_mfma_kernel(Geom g, const char* __restrict__ X,
                                                            const char* __restrict__ Y,
                                                            float* __restrict__ M, int anchor_start)
{
    constexpr int DPS = 2;   // loads per wave per stage: one instruction (four rows) per tensor
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sX = smem;                       // ST_NST stages
    char* sY = smem + ST_NST * ST_STAGE;   // ST_NST stages
    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    // A workgroup takes a run of consecutive slots u (u = group * T_s + slot), which is one
    // contiguous stretch of each tensor, and keeps its ring full across their boundaries: the
    // loads of the next slot's first blocks are on their way while the last blocks of this one
    // are consumed.
    const int total = g.T_s * g.G;
    const int per_wg = (total + (int)gridDim.x - 1) / (int)gridDim.x;
    const int u_first = (int)blockIdx.x * per_wg, nunits = min(total, u_first + per_wg);
    struct Unit { int u, len, nblk; size_t row0; };
    auto open_unit = [&](int u) {
        Unit x;
        x.u = u; x.len = 0; x.nblk = 0; x.row0 = 0;
        if (u < nunits) {
            int tok0;
            slot_range(g, u % g.T_s, tok0, x.len);
            x.nblk = (x.len + ST_KB - 1) / ST_KB;
            x.row0 = ((size_t)(u / g.T_s) * g.N + tok0) * ROWB;
        }
        return x;
    };
    // wave w fetches rows 4w .. 4w+3 of a stage: lane l the 16 bytes that land swizzled at its place
    const int myrow = 4 * w + (lane >> 4);
    const uint32_t dvo = dma_lane_off(w, lane);

    Unit iu = open_unit(u_first);   // where the next load goes
    int ib = 0, fill = 0, inflight = 0;     // its next block; ring slot to fill; stages issued and not yet consumed
    auto issue_next = [&]() {
        while (iu.u < nunits && ib >= iu.nblk) { iu = open_unit(iu.u + 1); ib = 0; }   // next slot with tokens
        if (iu.u >= nunits) return;
        const int tok = ib * ST_KB;
        const size_t blk = iu.row0 + (size_t)tok * ROWB;
        // rows past the slot's end fetch its last row (always in bounds) and are zeroed after landing
        const uint32_t voff = (uint32_t)(min(myrow, iu.len - 1 - tok) * ROWB) + (dvo & (ROWB - 1));
        dma16_nt(X + blk, voff, lds_addr_of(sX + fill * ST_STAGE + 4 * w * ROWB));
        dma16_nt(Y + blk, voff, lds_addr_of(sY + fill * ST_STAGE + 4 * w * ROWB));
        fill = fill + 1 == ST_NST ? 0 : fill + 1;
        ++ib;
        ++inflight;
    };
    for (int i = 0; i < ST_NST - 1; ++i) issue_next();

    constexpr int NSTORE = 16 * ST_TPW;   // store instructions per wave that write a slot's state
    int slot = 0, older_than_stores = 0;
    for (Unit cu = open_unit(u_first); cu.u < nunits; cu = open_unit(cu.u + 1)) {
        f32x16 acc[ST_TPW];
#pragma unroll
        for (int u = 0; u < ST_TPW; ++u)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[u][v] = 0.f;
        float l2 = DECAY ? decay_log2(g, cu.u / g.T_s) : 0.f;
        asm volatile("" : "+v"(l2));   // waited for here, once per slot, not at its first use inside the block loop

        for (int blk = 0; blk < cu.nblk; ++blk) {
            char* tx = sX + slot * ST_STAGE;
            char* ty = sY + slot * ST_STAGE;
            // The oldest stage in flight has landed once at most the younger ones are outstanding.
            // Memory operations retire in order and stores count too: the stages that were already
            // on their way when the previous slot's state was stored are older than those NSTORE
            // stores, which may therefore stay outstanding as well (waiting for them here would
            // stop the stream at every slot boundary until the stores have been acknowledged).
            if (older_than_stores > 0) {
                --older_than_stores;
                if (inflight >= 4) wait_vmcnt<3 * DPS + NSTORE>();
                else if (inflight == 3) wait_vmcnt<2 * DPS + NSTORE>();
                else if (inflight == 2) wait_vmcnt<DPS + NSTORE>();
                else wait_vmcnt<NSTORE>();
            } else {
                if (inflight >= 4) wait_vmcnt<3 * DPS>();
                else if (inflight == 3) wait_vmcnt<2 * DPS>();
                else if (inflight == 2) wait_vmcnt<DPS>();
                else wait_vmcnt<0>();
            }
            --inflight;
            const int tok = blk * ST_KB + myrow;
            u32x4* px = reinterpret_cast<u32x4*>(tx + myrow * ROWB + (lane & 15) * 16);
            if (tok >= cu.len) {
                const u32x4 z = {0u, 0u, 0u, 0u};
                *px = z;
                *reinterpret_cast<u32x4*>(ty + myrow * ROWB + (lane & 15) * 16) = z;
            } else if (DECAY) {
                // weight this wave's own rows of the X tile (a row takes one weight: the swizzle does not matter)
                const float wt = exp2f((float)(anchor_start ? tok : cu.len - 1 - tok) * l2);
                *px = scale_bf16x8(*px, wt);
            }
            __syncthreads();   // block complete in LDS; every wave has left the block before it
            issue_next();      // into the ring slot that block occupied
            update_tiles<ST_TPW, ST_KB>(acc, tx, ty, w * ST_TPW, lane);
            slot = slot + 1 == ST_NST ? 0 : slot + 1;
        }

        float* m = M + (size_t)cu.u * (size_t)(D * D);
#pragma unroll
        for (int u = 0; u < ST_TPW; ++u) {
            const int t = w * ST_TPW + u, a = t >> 2, b = t & 3;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = 32 * a + 8 * (v >> 2) + 4 * h + (v & 3);
                __builtin_nontemporal_store(acc[u][v], m + row * D + 32 * b + l32);
            }
        }
        older_than_stores = inflight;
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
//
// The rows of A for the next chunk are fetched the same way (asm loads into registers,
// completed by a counted wait at the chunk's end), so that inside the walk the compiler
// places no vector-memory wait of its own: it cannot see the stage loads, and any wait it
// inserted for a load it does know would drain them all.  For the same reason the kernel
// must not spill (a reload from scratch is such a load); tests/test_isa_guards.py checks
// both properties on the compiled code.
// =====================================================================================

// Per-lane byte offsets into a swizzled tile, computed once per kernel.
template <int TPW>
struct LaneOffs {
    int nat[8];        // row l32, 16-byte piece holding d = 16 ks + 8h .. +7
    int pv[4][2];      // transposed fetch of columns 32 tv + l32: rows 4h.. (lo) and 8 + 4h.. (hi)
    int ua[2];         // state update, X^T operand: columns 32 a + l32, rows 8h.. (lo), 8h + 4.. (hi)
    int ub[TPW][2];    // state update, Y operand of tile u: columns 32 b_u + l32
};

template <int TPW>
__device__ __forceinline__ void make_lane_offs(LaneOffs<TPW>& o, int lane, int t0)
{
    const int h = lane >> 5, l32 = lane & 31, i = lane & 15, g2 = (lane >> 4) & 1;
    const int cl = 16 * g2 + 4 * (i & 3), rl = i >> 2;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) o.nat[ks] = tile_off(l32, 2 * ks + h);
#pragma unroll
    for (int tv = 0; tv < 4; ++tv) {
        o.pv[tv][0] = tr_off(4 * h + rl, 32 * tv + cl);
        o.pv[tv][1] = tr_off(8 + 4 * h + rl, 32 * tv + cl);
    }
    o.ua[0] = tr_off(8 * h + rl, 32 * (t0 >> 2) + cl);
    o.ua[1] = tr_off(8 * h + 4 + rl, 32 * (t0 >> 2) + cl);
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
        o.ub[u][0] = tr_off(8 * h + rl, 32 * ((t0 + u) & 3) + cl);
        o.ub[u][1] = tr_off(8 * h + 4 + rl, 32 * ((t0 + u) & 3) + cl);
    }
}

// inter-chunk operands: rows 32 tv + l32 of the snapshot for d_k step ks
template <int NOP>
__device__ __forceinline__ void rd_inter(bf16x8 (&buf)[NOP], const char* sM, int nat_ks)
{
#pragma unroll
    for (int tv = 0; tv < 4; ++tv) buf[tv] = lds_read16_at(sM + tv * (32 * ROWB), nat_ks);
}

template <int NOP>
__device__ __forceinline__ void mm_inter(f32x16 (&Oacc)[4], const bf16x8 (&buf)[NOP], bf16x8 q)
{
#pragma unroll
    for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(buf[tv], q, Oacc[tv]);
}

// state-update operands for 16-token step ks of a stage: buf[0] = X^T rows of the wave's tile
// row a, buf[1 + u] = Y columns of tile u (all of a wave's tiles share a).
template <int TPW, int NOP>
__device__ __forceinline__ void rd_update(bf16x8 (&buf)[NOP], const char* tx, const char* ty, int ks,
                                          const LaneOffs<TPW>& o)
{
    static_assert(TPW + 1 <= NOP, "operand buffer too small");
    buf[0] = lds_read_tr8_at(tx + ks * (16 * ROWB), o.ua[0], o.ua[1]);
#pragma unroll
    for (int u = 0; u < TPW; ++u) buf[1 + u] = lds_read_tr8_at(ty + ks * (16 * ROWB), o.ub[u][0], o.ub[u][1]);
}

template <int TPW, int NOP>
__device__ __forceinline__ void mm_update(f32x16 (&acc)[TPW], const bf16x8 (&buf)[NOP])
{
#pragma unroll
    for (int u = 0; u < TPW; ++u) acc[u] = mfma(buf[0], buf[1 + u], acc[u]);
}

// One problem instance for the fused attention pass.
struct AttnProblem {
    const char* A;        // rows that receive an output ("queries" of this problem)
    const char* Bk;       // rows scored against A
    const char* Cv;       // rows mixed by the scores
    const float* state;   // [G][T_s][d][d] slot states (see `anti`)
    int user_state;       // `state` is the caller's array, one entry per slot of the CALLER's length (Geom: P_Ts, wslots)
    char* out;
    int transpose_state;  // read the d x d slot state transposed
    int anti;             // 0: causal (j <= i); 1: anti-causal (j >= i)
    const unsigned* pace; // NULL, or per (group, slot): 64-token blocks another workgroup has begun
    int lead;             // with pace: this walk may be at most `lead` blocks ahead of that count
};

// The d x d state a walk starts from: entry `s` of an array with one state per walk, or, in the
// caller's own array, the entry of the caller's slot that starts where the walk starts.
__device__ __forceinline__ const float* walk_state(const Geom& g, const AttnProblem& pr, int grp, int s, int ps)
{
    const size_t i = pr.user_state ? (size_t)grp * g.P_Ts + ps : (size_t)grp * g.T_s + s;
    return pr.state + i * (size_t)(D * D);
}

// Holds wave 0 of a walk (and with it, at the next barrier, its workgroup) until the workgroup it
// shares its reads with has begun block `need`, so that the two stay within reach of each other
// in the L2.  Purely a matter of speed: the count is read through the scalar cache with glc (a
// scalar load does not disturb the vector-memory counter the walk's own waits rely on), no data
// depends on it, and the wait gives up after a bounded number of polls.
__device__ __forceinline__ void pace_wait(const unsigned* p, int need)
{
    if (need <= 0) return;
    for (int i = 0; i < 512; ++i) {
        unsigned v;
        asm volatile("s_load_dword %0, %1, 0x0 glc\n\ts_waitcnt lgkmcnt(0)" : "=s"(v) : "s"(p) : "memory");
        if ((int)v >= need) break;
        __builtin_amdgcn_s_sleep(4);
    }
}

// Snapshot of the running state for the inter-chunk product: bf16 [d_v][d_k] in LDS.
// negate: the accumulators hold minus the state (anti-causal walk, see the kernel).
template <int TPW>
__device__ __forceinline__ void write_snapshot(char* sM, const f32x16 (&Macc)[TPW], int t0, int l32, int h,
                                               bool negate)
{
    const float sg = negate ? -1.f : 1.f;
#pragma unroll
    for (int u = 0; u < TPW; ++u) {
        const int t = t0 + u, a = t >> 2, b = t & 3;
        const int row = 32 * b + l32;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            u32x2 pk = {pack2(sg * Macc[u][4 * q], sg * Macc[u][4 * q + 1]),
                        pack2(sg * Macc[u][4 * q + 2], sg * Macc[u][4 * q + 3])};
            *reinterpret_cast<u32x2*>(sM + tile_off(row, 4 * a + q) + 8 * h) = pk;
        }
    }
}

// inter-chunk term: out^T += S^T A^T with S^T = snapshot [d_v][d_k]; operands of d_k step
// ks+1 are fetched while the MFMAs of step ks run
template <int NOP>
__device__ __forceinline__ void inter_product(f32x16 (&Oacc)[4], const char* sM, const bf16x8 (&qf)[8],
                                              const int (&nat)[8])
{
    bf16x8 bufA[NOP], bufB[NOP];
    rd_inter<NOP>(bufA, sM, nat[0]);
    SCHED_FENCE();
#pragma unroll
    for (int ks = 0; ks < 8; ks += 2) {
        rd_inter<NOP>(bufB, sM, nat[ks + 1]);
        SCHED_FENCE();
        mm_inter<NOP>(Oacc, bufA, qf[ks]);
        SCHED_FENCE();
        if (ks + 2 < 8) rd_inter<NOP>(bufA, sM, nat[ks + 2]);
        SCHED_FENCE();
        mm_inter<NOP>(Oacc, bufB, qf[ks + 1]);
        SCHED_FENCE();
    }
}

// A value that is the same in every lane, moved to a scalar register (the builtin takes integers).
__device__ __forceinline__ float uniform_f32(float x)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, x)));
}

// Stores a wave's 32 output rows from the transposed accumulators (lane = row, four consecutive
// d_v per register group) through its private 4 KiB LDS patch, half of d_v at a time, so that
// every lane stores 16 contiguous bytes; rows at or beyond nrows are left out.  All lane-derived
// addresses are rebuilt here from an index the compiler cannot hoist out of the caller's loops:
// hoisted, they would be live across the whole walk and spilled.
__device__ __forceinline__ void store_out_rows(const f32x16 (&Oacc)[4], char* stg, char* out_rows, int nrows, int tid)
{
    int ln;
    asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
    const int l32 = ln & 31, h = ln >> 5, row = ln >> 3, ch = ln & 7;
    char* wr = stg + l32 * 128 + 8 * h;
    const int sw = l32 & 7;
    const char* rd = stg + row * 128 + ((ch ^ (row & 7)) << 4);
    char* gp = out_rows + (size_t)row * ROWB + 16 * ch;
#pragma unroll
    for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
        for (int tvv = 0; tvv < 2; ++tvv)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x16& o = Oacc[2 * hv + tvv];
                u32x2 pk = {pack2(o[4 * q], o[4 * q + 1]), pack2(o[4 * q + 2], o[4 * q + 3])};
                *reinterpret_cast<u32x2*>(wr + (((4 * tvv + q) ^ sw) << 4)) = pk;
            }
        // the four reads first (they need no predicate), so that they share one wait
        u32x4 v[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) v[i] = *reinterpret_cast<const u32x4*>(rd + 1024 * i);
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (row + 8 * i < nrows)   // written once, read by a later kernel: non-temporal
                __builtin_nontemporal_store(v[i], reinterpret_cast<u32x4*>(gp + (size_t)(8 * i) * ROWB + 128 * hv));
    }
}

// The grid is one-dimensional and carries nprob problems that walk the same slots.  The
// (group, slot) pairs are numbered unit = group * T_s + slot, and workgroup x handles unit
// 8*(x/(8 nprob)) + x%8 of problem (x/8)%nprob.  With workgroups dealt to the eight XCDs
// round-robin, consecutive units go to different XCDs whatever T_s is (one slot per head
// included), while the nprob workgroups of a unit land on the same XCD and run at about the
// same time, so a block of a tensor that several problems stream (the three backward problems
// all walk forward over Q, K, V, dO) comes from HBM once and from that XCD's L2 afterwards.
//
// Walk: chunks in ascending order in both modes.
//   causal: the accumulators hold S_c = prefix state before chunk c; snapshot and inter-chunk
//     product at the start of the chunk, then S += Bk_c^T Cv_c.
//   anti-causal: the slot state handed in is the INCLUSIVE suffix at the slot's start,
//     R = sum over this and all later slots of the document.  The accumulators hold -R and
//     add Bk_c^T Cv_c block by block, so after the chunk's own blocks they hold minus the
//     suffix beyond chunk c, which is the state its rows need; snapshot (negated) and
//     inter-chunk product therefore come at the end of the chunk.
template <int C>
__global__ __launch_bounds__(C * 2) void attn_mfma_kernel(Geom g, AttnProblem p0, AttnProblem p1,
                                                          AttnProblem p2, int nprob)
{
    constexpr int NW = C / 32, TPW = 16 / NW, BPC = C / KB;
    constexpr int DPS = 2 * (16 / NW);     // loads per wave per stage
    constexpr int NOP = (TPW + 1 > 4) ? 8 : 4;   // operands per register buffer
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;                              // Bk stages
    char* sV = smem + NSTAGE * STAGE_BYTES;       // Cv stages
    char* sM = smem + 2 * NSTAGE * STAGE_BYTES;   // state snapshot, bf16 [d_v][d_k]
    char* sO = sM + D * ROWB;                     // output staging, 4 KiB per wave

    const int tid = threadIdx.x, lane = tid & 63;
    // the wave index is the same in all 64 lanes: keep it, and all that derives from it, scalar
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const unsigned unit = (blockIdx.x / (8u * nprob)) * 8u + (blockIdx.x & 7u);
    const int prob = (int)(blockIdx.x >> 3) % nprob;
    if (unit >= (unsigned)g.T_s * (unsigned)g.G) return;
    const int s = (int)(unit % (unsigned)g.T_s), grp = (int)(unit / (unsigned)g.T_s);
    const AttnProblem& pr = prob == 0 ? p0 : (prob == 1 ? p1 : p2);
    const char* __restrict__ A = pr.A;
    const char* __restrict__ Bk = pr.Bk;
    const char* __restrict__ Cv = pr.Cv;
    const float* __restrict__ state = pr.state;
    char* __restrict__ out = pr.out;
    const int transpose_state = pr.transpose_state;
    const int anti = pr.anti;
    int tok0, len, ps;
    slot_range(g, s, tok0, len, ps);
    if (len <= 0) return;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;

    // Row block of this wave.  With 8 waves, waves w and w+4 (which share a SIMD under
    // round-robin placement) get blocks s and 7-s, so that their triangular work adds up evenly.
    const int rb = (NW == 8) ? (w < 4 ? w : 11 - w) : w;
    const int t0 = w * TPW;
    const int nch = (len + C - 1) / C;
    const int NB = (len + KB - 1) / KB;    // 64-token blocks in the whole slot
    uint32_t dvo[16 / NW];   // per-lane source offsets of this wave's stage loads
#pragma unroll
    for (int u = 0; u < 16 / NW; ++u) dvo[u] = dma_lane_off(w * (16 / NW) + u, lane);
    auto issue = [&](int i) {
        dma_block<NW>(Bk, Cv, row0, i * KB, len, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, lane, dvo);
    };
    issue(0);
    if (NB > 1) issue(1);

    // running state tiles, C/D layout: rows = d_k (first index), columns = d_v
    f32x16 Macc[TPW];
#pragma unroll
    for (int u = 0; u < TPW; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) Macc[u][v] = 0.f;
    if (state) {   // NULL: every slot opens its document and starts from a zero state
        const float* st = walk_state(g, pr, grp, s, ps);
        const float sg = anti ? -1.f : 1.f;
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
            if (!transpose_state) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    Macc[u][v] = sg * st[(32 * a + 8 * (v >> 2) + 4 * h + (v & 3)) * D + 32 * b + l32];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 x = *reinterpret_cast<const f32x4*>(st + (32 * b + l32) * D + 32 * a + 8 * q + 4 * h);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Macc[u][4 * q + e] = sg * x[e];
                }
            }
        }
    }

    LaneOffs<TPW> lo;
    make_lane_offs<TPW>(lo, lane, t0);

    // This wave's 32 rows of A as B-operand fragments (column = row of A, k = d).  The rows of
    // the next chunk are requested into tq once the current chunk has made its last use of qf;
    // rows past the slot's end fetch its last row (they only feed output rows that are not stored).
    u32x4 qv[8];
    auto issue_q = [&](int c) {
        // lane % 32 again, in a form the compiler cannot hoist out of the chunk loop: with every
        // register taken, a hoisted row index would be spilled, and its reload from scratch is a
        // vector-memory load whose wait drains the ring
        int lrow;
        asm volatile("v_and_b32 %0, 31, %1" : "=v"(lrow) : "v"(tid));
        const int r = min(c * C + 32 * rb + lrow, len - 1);
        const char* p = A + row0 + (size_t)r * ROWB + 16 * h;
        gload16_async<0>(qv[0], p);
        gload16_async<32>(qv[1], p);
        gload16_async<64>(qv[2], p);
        gload16_async<96>(qv[3], p);
        gload16_async<128>(qv[4], p);
        gload16_async<160>(qv[5], p);
        gload16_async<192>(qv[6], p);
        gload16_async<224>(qv[7], p);
    };
    auto take_q = [&](uint32_t zero) {
        const u32x4 z = {zero, zero, zero, zero};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qv[ks] = qv[ks] | z;
    };
    issue_q(0);
    take_q(wait_vmcnt_token<0>());
    const bf16x8 (&qf)[8] = reinterpret_cast<const bf16x8 (&)[8]>(qv);

    int bi = 0;          // index of the block being consumed
    int prev_nblk = BPC;
    for (int c = 0; c < nch; ++c) {
        const int nblk = min(BPC, NB - c * BPC);
        const bool last_chunk = (c + 1 == nch);

        if (!anti) {
            // The previous chunk read the snapshot in its first block; one of its later block
            // barriers separates that from this write unless it had a single block.
            if (prev_nblk < 2) __syncthreads();
            write_snapshot<TPW>(sM, Macc, t0, l32, h, false);
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
            // In the first two blocks after a chunk boundary the previous chunk's eight stores
            // were also issued after these loads, and need not have completed.
            if (c > 0 && jb < 2) {
                if (bi + 1 < NB) wait_vmcnt<DPS + 8>(); else wait_vmcnt<8>();
            } else {
                if (bi + 1 < NB) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
            }
            if (bi * KB + KB > len) zero_tail_rows<NW>(bi * KB, len, tK, tV, w, lane);
            __syncthreads();   // block bi complete in LDS; every wave is past block bi-1
            if (bi + 2 < NB) issue(bi + 2);

            if (!anti && jb == 0) inter_product<NOP>(Oacc, sM, qf, lo.nat);

            // Operand fetches are issued a batch ahead of the MFMAs that consume them (two
            // small register buffers); sched_barrier keeps the compiler from sinking the
            // reads back next to their uses.
            bf16x8 bufA[NOP], bufB[NOP];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int kt = 2 * jb + half;      // 32-key tile index inside the chunk
                const bool active = anti ? (kt >= rb) : (kt <= rb);
                if (!active) continue;
                // scores^T (keys x queries) = Bk_tile A_w^T ; the Cv operands of the second
                // product are fetched while the first one runs
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_at(tK + half * (32 * ROWB), lo.nat[ks]);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_at(tK + half * (32 * ROWB), lo.nat[ks + 4]);
                SCHED_FENCE();
                f32x16 sc;
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
                    bufA[tv] = lds_read_tr8_at(tV + half * (32 * ROWB), lo.pv[tv][0], lo.pv[tv][1]);
                SCHED_FENCE();
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
                    bufB[tv] = lds_read_tr8_at(tV + half * (32 * ROWB) + 16 * ROWB, lo.pv[tv][0], lo.pv[tv][1]);
                SCHED_FENCE();
                if (kt == rb) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = 8 * (v >> 2) + 4 * h + (v & 3);
                        const bool keep = anti ? (key >= l32) : (key <= l32);
                        sc[v] = keep ? sc[v] : 0.f;
                    }
                }
                // out^T (d_v x queries) += Cv_tile^T scores^T ; k-slots follow the C/D row order
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

            // causal: the rows of the next chunk replace qf while the state update and the
            // store run (anti-causal still needs qf for the inter product at the chunk's end)
            if (!anti && jb + 1 == nblk && !last_chunk) issue_q(c + 1);
            if (anti || !last_chunk) {
                // running state += Bk_blk^T Cv_blk on this wave's tiles, 16 tokens per step
                rd_update<TPW, NOP>(bufA, tK, tV, 0, lo);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufB, tK, tV, 1, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufA);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufA, tK, tV, 2, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufB);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufB, tK, tV, 3, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufA);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufB);
            }
        }
        prev_nblk = nblk;

        if (anti) {
            // every wave read the previous snapshot before its previous store, and at least one
            // block barrier has passed since
            write_snapshot<TPW>(sM, Macc, t0, l32, h, true);
            __syncthreads();
            inter_product<NOP>(Oacc, sM, qf, lo.nat);
            if (!last_chunk) issue_q(c + 1);
        }

        // store this wave's 32 output rows
        {
            const int rbase = c * C + 32 * rb;
            store_out_rows(Oacc, sO + w * 4096, out + row0 + (size_t)rbase * ROWB, len - rbase, tid);
        }
        // Only the eight stores above were issued after the rows of A for the next chunk (they
        // all execute: a chunk that is not the last is full).
        if (!last_chunk) take_q(wait_vmcnt_token<8>());
    }
}

// Counted waits with a run-time count.  A wave keeps the number of vector-memory instructions it
// has certainly issued (stage loads, row loads, full output stores; a store that may be skipped
// is left out, which only makes a wait stricter) and, for each batch of loads it will wait for,
// that number right after the batch.  The difference is how many younger instructions may still
// be outstanding when the batch is needed; memory instructions retire in order.  All batches here
// are multiples of four instructions.
__device__ __forceinline__ void wait_vmcnt_le(int n)
{
    if (n >= 24) wait_vmcnt<24>();
    else if (n >= 20) wait_vmcnt<20>();
    else if (n >= 16) wait_vmcnt<16>();
    else if (n >= 12) wait_vmcnt<12>();
    else if (n >= 8) wait_vmcnt<8>();
    else if (n >= 4) wait_vmcnt<4>();
    else wait_vmcnt<0>();
}

__device__ __forceinline__ uint32_t wait_vmcnt_token_le(int n)
{
    if (n >= 24) return wait_vmcnt_token<24>();
    if (n >= 20) return wait_vmcnt_token<20>();
    if (n >= 16) return wait_vmcnt_token<16>();
    if (n >= 12) return wait_vmcnt_token<12>();
    if (n >= 8) return wait_vmcnt_token<8>();
    if (n >= 4) return wait_vmcnt_token<4>();
    return wait_vmcnt_token<0>();
}

// The fused pass with 256-row chunks and eight waves (slots longer than 128 tokens).  Same
// problems, grid, tiles, stages, walk directions and asynchronous fetches as attn_mfma_kernel;
// waves w and w+4, which share a SIMD, own row blocks w and 7-w.  Two differences:
//
// Halves.  The masked products of a chunk are taken over its two 128-row halves separately:
// rows of a half against the keys of the same half only, and the half that lies further along
// the walk reads a second state snapshot taken between the halves (causal: rows 128.. start from
// the state that includes the first half's keys; anti-causal: rows ..127 have then seen all keys
// of their half and the accumulators hold minus the suffix beyond it).  The same sum, with 20
// score tiles per chunk instead of 36.
//
// Skew.  A 64-token block therefore concerns the rows of one half only, and at any time the
// four waves of the other half have nothing but their share of the state update to do.  They use
// that time for the work that would otherwise stop all eight waves at the end of a chunk:
//   - rows of the first half are complete once block 1 has been consumed (anti-causal: once the
//     state between the halves has been applied, at block 2): their waves request the next
//     chunk's rows in block 2 and store in block 3, while the second half's waves compute;
//   - rows of the second half are complete at the end of the chunk (anti-causal: once the state
//     at the chunk's end has been applied): their waves keep the accumulators, finish them and
//     request their next rows in block 0 of the next chunk and store in block 1, while the first
//     half's waves compute.  The snapshot taken at the top of a chunk is therefore the state the
//     previous chunk's second half still needs (anti-causal) as well as the one this chunk's
//     first half starts from (causal).
// Neither snapshot needs a barrier of its own: each is written at the end of a block's work (after
// block 3: the top of the next chunk; after block 1: between the halves), when every wave has
// passed that block's barrier and with it all reads of the previous snapshot, and the next
// block's barrier publishes it.
// With scalar decay (DECAY; weights as in attn_decay_mfma_kernel) the anti-causal problems walk
// backwards and every half takes its state on entry, like the causal ones; "first" and "second"
// half above then mean the order in which the walk reaches them.
// The two halves' waves and the two directions run separate copies of the walk (HC1, ANTI), each
// a straight line through the four blocks of a chunk, so that the accumulators and the rows in
// flight have one definition per place and are not copied at control-flow joins.  Every chunk is
// walked as four blocks: a block that lies wholly past the slot's end is not loaded but zeroed, and
// contributes nothing.  All copies pass the same barriers: one per block, and for the anti-causal
// walk one at the end.  Each half stores at a different time, so the waits are counted at run
// time (wait_vmcnt_le).
template <bool HC1, bool ANTI, bool DECAY>
__device__ __forceinline__ void skew_walk(const Geom& g, const AttnProblem& pr, char* smem, int tid, int w,
                                          int rb, int grp, int s, int tok0, int len, const float* wstate)
{
    constexpr int C = 256, NW = 8, TPW = 2, BPC = 4, DPS = 4, NOP = 4;
    // With decay the anti-causal problems walk the slot backwards from the exclusive suffix (see
    // attn_decay_mfma_kernel), so both directions take their states when the walk enters a half;
    // without it they walk forwards and subtract (see attn_mfma_kernel), and take them when it leaves.
    constexpr bool REV = DECAY && ANTI;        // blocks and chunks in descending order
    constexpr bool ENDSTATE = ANTI && !DECAY;  // rows take the state at the end of their half
    constexpr bool SECOND = REV ? !HC1 : HC1;  // this wave's rows lie in the half the walk reaches second
    char* sK = smem;                              // Bk stages
    char* sV = smem + NSTAGE * STAGE_BYTES;       // Cv stages
    char* sM = smem + 2 * NSTAGE * STAGE_BYTES;   // state snapshot, bf16 [d_v][d_k]
    char* sO = sM + D * ROWB;                     // output staging, 4 KiB per wave
    const int lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const char* __restrict__ A = pr.A;
    const char* __restrict__ Bk = pr.Bk;
    const char* __restrict__ Cv = pr.Cv;
    char* __restrict__ out = pr.out;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;
    const int t0 = w * TPW;
    const int nch = (len + C - 1) / C;
    const int NBP = nch * BPC;                 // blocks walked (the last chunk padded to four)
    const float l2 = DECAY ? uniform_f32(decay_log2(g, grp)) : 0.f;   // log2 of the head's factor
    const float wblk = DECAY ? uniform_f32(exp2f((float)KB * l2)) : 1.f;
    // walk position -> block of the slot, chunk of the slot
    auto blk = [&](int i) __attribute__((always_inline)) { return REV ? NBP - 1 - i : i; };
    auto chk = [&](int c) __attribute__((always_inline)) { return REV ? nch - 1 - c : c; };

    // Stage loads of the block at walk position i.  The per-lane source offsets are rebuilt at every call from a lane index
    // the compiler cannot hoist: kept across the walk they cost registers this kernel does not have.
    auto issue = [&](int i) __attribute__((always_inline)) {
        int ln;
        asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
        uint32_t dvo[16 / NW];
#pragma unroll
        for (int u = 0; u < 16 / NW; ++u) dvo[u] = dma_lane_off(w * (16 / NW) + u, ln);
        dma_block<NW>(Bk, Cv, row0, blk(i) * KB, len, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, ln, dvo);
    };
    if (blk(0) * KB < len) issue(0);
    if (blk(1) * KB < len) issue(1);

    // running state tiles, C/D layout: rows = d_k (first index), columns = d_v; the anti-causal
    // walk keeps minus the inclusive suffix and adds the blocks it passes (see attn_mfma_kernel)
    f32x16 Macc[TPW];
#pragma unroll
    for (int u = 0; u < TPW; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) Macc[u][v] = 0.f;
    if (wstate) {   // NULL: every slot opens its document and starts from a zero state
        const float* st = wstate;
        const float sg = ENDSTATE ? -1.f : 1.f;
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
            if (!pr.transpose_state) {
#pragma unroll
                for (int v = 0; v < 16; ++v)
                    Macc[u][v] = sg * st[(32 * a + 8 * (v >> 2) + 4 * h + (v & 3)) * D + 32 * b + l32];
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    f32x4 x = *reinterpret_cast<const f32x4*>(st + (32 * b + l32) * D + 32 * a + 8 * q + 4 * h);
#pragma unroll
                    for (int e = 0; e < 4; ++e) Macc[u][4 * q + e] = sg * x[e];
                }
            }
        }
    }

    // Per-lane byte offsets into a swizzled tile.  The swizzle is an XOR on the 16-byte chunk index
    // (with bits of the row index), so the offsets of a family differ by an XOR with a constant and
    // a multiple of the row size, and only one per family is kept in a register:
    //   natural row l32, d step ks:                        nat0 ^ (ks << 5)
    //   transposed fetch of columns 32 tv + l32, rows r:   pvA ^ (tv << 6);  rows r + 8: (.. ^ 32) + 8 rows
    //   state update, X^T operand, rows r:                 uaA;              rows r + 4: (uaA ^ 16) + 4 rows
    //   state update, Y operand of tile u:                 uaA ^ ydel ^ (u << 6), ydel the same in all lanes
    //   snapshot piece q of tile u:                        (s0 ^ (q << 4)) + u * 32 rows, s0 rebuilt at each snapshot
    // (a stage's base is a multiple of its 16 KiB, so base + offset can be formed first).
    const int li = lane & 15, g2 = (lane >> 4) & 1, cl = 16 * g2 + 4 * (li & 3), rl = li >> 2;
    const uint32_t nat0 = (uint32_t)tile_off(l32, h);
    const uint32_t pvA = (uint32_t)tr_off(4 * h + rl, cl);
    const uint32_t uaA = (uint32_t)tr_off(8 * h + rl, 32 * (t0 >> 2) + cl);
    const uint32_t ydel = (uint32_t)(((t0 >> 2) ^ (t0 & 3)) << 6);

    // this wave's 32 rows of A as B-operand fragments, fetched asynchronously (see attn_mfma_kernel);
    // rows past the slot's end fetch its last row
    u32x4 qv[8];
    auto issue_q = [&](int c) __attribute__((always_inline)) {   // c: chunk of the slot
        int ln;   // the lane index again, in a form the compiler cannot hoist out of the loop (and spill)
        asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
        const int r = max(min(c * C + 32 * rb + (ln & 31), len - 1), 0);
        const char* p = A + row0 + (size_t)r * ROWB + 16 * (ln >> 5);
        gload16_async<0>(qv[0], p);
        gload16_async<32>(qv[1], p);
        gload16_async<64>(qv[2], p);
        gload16_async<96>(qv[3], p);
        gload16_async<128>(qv[4], p);
        gload16_async<160>(qv[5], p);
        gload16_async<192>(qv[6], p);
        gload16_async<224>(qv[7], p);
    };
    auto take_q = [&](uint32_t zero) __attribute__((always_inline)) {
        const u32x4 z = {zero, zero, zero, zero};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qv[ks] = qv[ks] | z;
    };
    // The first half's waves need the rows of chunk 0 at once; the second half's request theirs in
    // block 0.  (A request whose registers are never read afterwards must not be made: the compiler
    // would reuse those registers while the load is still on its way.)
    if (!SECOND) {
        issue_q(chk(0));
        take_q(wait_vmcnt_token<0>());   // also completes blocks 0 and 1 and the state
    } else {
        wait_vmcnt<0>();
    }
    const bf16x8 (&qf)[8] = reinterpret_cast<const bf16x8 (&)[8]>(qv);

    // snapshot of the running state, bf16 [d_v][d_k] (the subtracting walk holds minus the state)
    auto snapshot = [&]() __attribute__((always_inline)) {
        const float sg = ENDSTATE ? -1.f : 1.f;
        int ln;   // built here from the lane index (twice per chunk) rather than held in a register
        asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
        const uint32_t s0 = lds_addr_of(sM) + (uint32_t)tile_off(32 * (t0 & 3) + (ln & 31), 4 * (t0 >> 2)) + 8 * (ln >> 5);
#pragma unroll
        for (int u = 0; u < TPW; ++u)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                u32x2 pk = {pack2(sg * Macc[u][4 * q], sg * Macc[u][4 * q + 1]),
                            pack2(sg * Macc[u][4 * q + 2], sg * Macc[u][4 * q + 3])};
                *reinterpret_cast<__attribute__((address_space(3))) u32x2*>((s0 ^ (q << 4)) + u * (32 * ROWB)) = pk;
            }
    };

    f32x16 Oacc[4];
    auto zero_out = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;
    };
    // inter-chunk term: out^T += S^T A^T with S^T = snapshot; operands of d_k step ks+1 are
    // fetched while the MFMAs of step ks run
    auto inter = [&]() __attribute__((always_inline)) {
        uint32_t n0 = nat0;
        pin_vgpr(n0);   // the sum below is formed here, not once before the walk (and then spilled)
        const uint32_t aM = lds_addr_of(sM) + n0;
        bf16x8 bA[4], bB[4];
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) bA[tv] = lds_read16_u(aM + tv * (32 * ROWB));
        SCHED_FENCE();
#pragma unroll
        for (int ks = 0; ks < 8; ks += 2) {
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) bB[tv] = lds_read16_u((aM ^ ((ks + 1) << 5)) + tv * (32 * ROWB));
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bA[tv], qf[ks], Oacc[tv]);
            SCHED_FENCE();
            if (ks + 2 < 8) {
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) bA[tv] = lds_read16_u((aM ^ ((ks + 2) << 5)) + tv * (32 * ROWB));
            }
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bB[tv], qf[ks + 1], Oacc[tv]);
            SCHED_FENCE();
        }
    };
    // With decay the state sits one token before the rows' half (causal) or one after it
    // (anti-causal): weight per query.  The accumulators hold nothing else yet.
    auto inter_decayed = [&](int cc) __attribute__((always_inline)) {
        inter();
        int ln;
        asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
        const int a = 32 * rb + (ln & 31), hb = HC1 ? 1 : 0;
        const int clen = min(C, len - cc * C);
        const int e = REV ? max(min(clen, 128 * (hb + 1)) - a, 0) : a - 128 * hb + 1;
        const float wq = __builtin_amdgcn_exp2f((float)e * l2);
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] *= wq;
    };

    // vector-memory instructions certainly issued since the full wait above, and the marks of the
    // batches to wait for
    int issued = 0, seq_cur = 0, seq_next = 0, seq_q = 0;

    // stores this wave's rows of chunk c of the slot (none when there is no such chunk) and clears
    // the accumulators
    auto store_rows = [&](int c) __attribute__((always_inline)) {
        const int rbase = c * C + 32 * rb;
        const int nrows = (c < 0 || c >= nch) ? 0 : len - rbase;
        store_out_rows(Oacc, sO + w * 4096, out + row0 + (ptrdiff_t)rbase * ROWB, nrows, tid);
        if (nrows >= 32) issued += 8;   // all eight stores certainly execute
        SCHED_FENCE();
        zero_out();
    };

    char* tK = sK;
    char* tV = sV;
    // start of block bi: its loads have landed, the block is complete in LDS, every wave is past
    // block bi - 1, and the loads of block bi + 2 are on their way
    auto begin = [&](int bi) __attribute__((always_inline)) {   // bi: walk position
        tK = sK + (bi % NSTAGE) * STAGE_BYTES;
        tV = sV + (bi % NSTAGE) * STAGE_BYTES;
        wait_vmcnt_le(issued - seq_cur);
        if (blk(bi) * KB + KB > len) {   // at the slot's end only: keep these addresses out of the walk's registers
            int ln;
            asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
            zero_tail_rows<NW>(blk(bi) * KB, len, tK, tV, w, ln);
        }
        if (DECAY) {
            // Weight this wave's own rows of the Bk tile by the token's factor as seen from the
            // block's last token (forward walk, lam^(63-b)) or first token (backward walk, lam^b); a
            // whole row takes one weight, so the swizzle does not matter here.
            int ln;
            asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
#pragma unroll
            for (int u = 0; u < 16 / NW; ++u) {
                const int b = 4 * (w * (16 / NW) + u) + (ln >> 4);
                const float wr = __builtin_amdgcn_exp2f((float)(REV ? b : KB - 1 - b) * l2);
                u32x4* pk = reinterpret_cast<u32x4*>(tK + b * ROWB + (ln & 15) * 16);
                *pk = scale_bf16x8(*pk, wr);
            }
        }
        // (blocks past the slot's end exist only in this walk's padding: nothing to wait for there)
        if (pr.pace && w == 0 && blk(bi) * KB < len) pace_wait(pr.pace + ((size_t)grp * g.T_s + s), bi - pr.lead);
        __syncthreads();
        seq_cur = seq_next;
        if (bi + 2 < NBP && blk(bi + 2) * KB < len) { issue(bi + 2); issued += DPS; }
        seq_next = issued;
    };

    // masked products of this wave's rows with the two 32-key tiles of block JB of the chunk
    auto tiles = [&](auto jw_c) __attribute__((always_inline)) {
        constexpr int JB = REV ? 3 - decltype(jw_c)::value : decltype(jw_c)::value;   // block of the chunk
        // per-lane addresses into this block's stage, opaque to the compiler: it would otherwise fold
        // the constants of every use into copies that it keeps (and spills) across the whole walk
        uint32_t oK = nat0, oV = pvA;
        pin_vgpr(oK); pin_vgpr(oV);   // (opaque before the sum too: no table of sums per stage)
        uint32_t aK = lds_addr_of(tK) + oK, aVA = lds_addr_of(tV) + oV;
        pin_vgpr(aK); pin_vgpr(aVA);
        bf16x8 bufA[NOP], bufB[NOP];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int kt = 2 * JB + half;      // 32-key tile index inside the chunk
            const bool active = ANTI ? (kt >= rb) : (kt <= rb);
            if (!active) continue;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_u((aK ^ (ks << 5)) + half * (32 * ROWB));
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_u((aK ^ ((ks + 4) << 5)) + half * (32 * ROWB));
            SCHED_FENCE();
            f32x16 sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufA[tv] = lds_read_tr8_u((aVA ^ (tv << 6)) + half * (32 * ROWB),
                                          (aVA ^ ((tv << 6) | 32)) + half * (32 * ROWB) + 8 * ROWB);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufB[tv] = lds_read_tr8_u((aVA ^ (tv << 6)) + half * (32 * ROWB) + 16 * ROWB,
                                          (aVA ^ ((tv << 6) | 32)) + half * (32 * ROWB) + 24 * ROWB);
            SCHED_FENCE();
            if (DECAY) {
                // from the row weights of the block to lam^|i-j|: one factor per query; query and keys
                // lie in the same 128-row half, so the exponent stays within -63..64
                int ln;
                asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
                const int qi = 32 * rb + (ln & 31) - KB * JB;   // query index relative to the block's start
                const float f = __builtin_amdgcn_exp2f((float)(REV ? -qi : qi - (KB - 1)) * l2);
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] *= f;
            }
            if (kt == rb) {
                // the diagonal tile's mask, from a lane index the compiler cannot hoist: hoisted, the 16
                // predicates would occupy 32 scalar registers across the whole walk
                int ln;
                asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
                const int lq = ln & 31, hq = ln >> 5;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 8 * (v >> 2) + 4 * hq + (v & 3);
                    const bool keep = ANTI ? (key >= lq) : (key <= lq);
                    sc[v] = keep ? sc[v] : 0.f;
                }
            }
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

    // running state += Bk_blk^T Cv_blk on this wave's tiles, 16 tokens per step
    auto update = [&](int bi) __attribute__((always_inline)) {   // bi: walk position
        if (DECAY) {
            // state = lam^n * state + (weighted Bk block)^T Cv block, n = the block's tokens
            const int n = min(max(len - blk(bi) * KB, 0), KB);
            const float wb = n == KB ? wblk : __builtin_amdgcn_exp2f((float)n * l2);
#pragma unroll
            for (int u = 0; u < TPW; ++u)
#pragma unroll
                for (int v = 0; v < 16; ++v) Macc[u][v] *= wb;
        }
        uint32_t oX = uaA;
        pin_vgpr(oX);   // (opaque before the sums too: no table of sums per stage)
        uint32_t aXA = lds_addr_of(tK) + oX, aYA = lds_addr_of(tV) + (oX ^ ydel);
        pin_vgpr(aXA); pin_vgpr(aYA);
        bf16x8 bufA[NOP], bufB[NOP];
        // operands of 16-token step ks: buf[0] = X^T rows of the wave's tile row, buf[1 + u] = Y
        // columns of tile u
        auto rd_upd = [&](bf16x8 (&buf)[NOP], int ks) __attribute__((always_inline)) {
            buf[0] = lds_read_tr8_u(aXA + ks * (16 * ROWB), (aXA ^ 16) + ks * (16 * ROWB) + 4 * ROWB);
#pragma unroll
            for (int u = 0; u < TPW; ++u)
                buf[1 + u] = lds_read_tr8_u((aYA ^ (u << 6)) + ks * (16 * ROWB),
                                            (aYA ^ ((u << 6) | 16)) + ks * (16 * ROWB) + 4 * ROWB);
        };
        rd_upd(bufA, 0);
        SCHED_FENCE();
        rd_upd(bufB, 1);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufA);
        SCHED_FENCE();
        rd_upd(bufA, 2);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufB);
        SCHED_FENCE();
        rd_upd(bufB, 3);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufA);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufB);
        SCHED_FENCE();
    };

    zero_out();
    using std::integral_constant;
    for (int c = 0; c < nch; ++c) {   // c: walk position of the chunk; cc: the chunk of the slot
        const int bi = c * BPC, cc = chk(c);
        // a walk that takes its states on entering a half needs the last chunk's update only for
        // the snapshot between its halves
        const bool carry = ENDSTATE || c + 1 < nch;

        // The state as the walk enters the chunk: what the rows of its first half start from, or
        // (subtracting walk) the suffix beyond the previous chunk that the rows of that chunk's
        // second half still need.  The previous chunk read its last snapshot in block 2; its block 3
        // barrier lies in between.
        snapshot();

        // ---- block 0
        begin(bi);
        if (!SECOND) {
            // the rows of this chunk (requested in block 2 of the previous one)
            take_q(wait_vmcnt_token_le(issued - seq_q));
            if (DECAY) inter_decayed(cc);
            else if (!ENDSTATE) inter();
            tiles(integral_constant<int, 0>{});
        } else {
            // finish the rows of the previous chunk's second half, request this chunk's
            if (ENDSTATE) inter();
            issue_q(cc); issued += 8; seq_q = issued;
        }
        update(bi);

        // ---- block 1 (the second half's waves have nothing else to do here: they store)
        begin(bi + 1);
        if (!SECOND) tiles(integral_constant<int, 1>{});
        else store_rows(REV ? cc + 1 : cc - 1);
        update(bi + 1);
        // The state between the halves.  Every wave has passed block 1's barrier, so the reads of the
        // chunk-top snapshot (in block 0) are over; block 2's barrier publishes this one.  Entering
        // walks: the second half starts from the state that includes the first half's keys.
        // Subtracting walk: rows ..127 have seen all keys of their half, and the accumulators hold
        // minus the suffix beyond it.
        snapshot();

        // ---- block 2
        begin(bi + 2);
        if (!SECOND) {
            if (ENDSTATE) inter();
            // the rows of the first half are complete: request the next chunk's
            issue_q(REV ? cc - 1 : cc + 1); issued += 8; seq_q = issued;
        } else {
            take_q(wait_vmcnt_token_le(issued - seq_q));
            if (DECAY) inter_decayed(cc);
            else if (!ENDSTATE) inter();
            tiles(integral_constant<int, 2>{});
        }
        if (carry) update(bi + 2);

        // ---- block 3 (the first half's waves store here)
        begin(bi + 3);
        if (SECOND) tiles(integral_constant<int, 3>{});
        else store_rows(cc);
        if (carry) update(bi + 3);
    }

    // The first half's waves requested rows beyond the last chunk in its block 2: let them land in
    // registers that are still theirs.
    if (!SECOND) {
        take_q(wait_vmcnt_token<0>());
        asm volatile("" ::"v"(qv[0]), "v"(qv[1]), "v"(qv[2]), "v"(qv[3]), "v"(qv[4]), "v"(qv[5]), "v"(qv[6]), "v"(qv[7]));
    }
    // the last chunk's second half
    if (ENDSTATE) {
        snapshot();
        __syncthreads();
        if (SECOND) inter();
    }
    if (SECOND) store_rows(chk(nch - 1));
}

template <bool DECAY>
__global__ __launch_bounds__(512) void attn_skew_mfma_kernel(Geom g, AttnProblem p0, AttnProblem p1,
                                                             AttnProblem p2, int nprob)
{
    extern __shared__ __attribute__((aligned(256))) char smem[];
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned unit = (blockIdx.x / (8u * nprob)) * 8u + (blockIdx.x & 7u);
    const int prob = (int)(blockIdx.x >> 3) % nprob;
    if (unit >= (unsigned)g.T_s * (unsigned)g.G) return;
    const int s = (int)(unit % (unsigned)g.T_s), grp = (int)(unit / (unsigned)g.T_s);
    const AttnProblem& pr = prob == 0 ? p0 : (prob == 1 ? p1 : p2);
    int tok0, len, ps;
    slot_range(g, s, tok0, len, ps);
    if (len <= 0) return;
    const float* wstate = pr.state ? walk_state(g, pr, grp, s, ps) : nullptr;
    const int rb = w < 4 ? w : 11 - w;   // waves w and w+4 share a SIMD: row blocks s and 7-s
    if (rb < 4) {
        if (pr.anti) skew_walk<false, true, DECAY>(g, pr, smem, tid, w, rb, grp, s, tok0, len, wstate);
        else skew_walk<false, false, DECAY>(g, pr, smem, tid, w, rb, grp, s, tok0, len, wstate);
    } else {
        if (pr.anti) skew_walk<true, true, DECAY>(g, pr, smem, tid, w, rb, grp, s, tok0, len, wstate);
        else skew_walk<true, false, DECAY>(g, pr, smem, tid, w, rb, grp, s, tok0, len, wstate);
    }
}

// =====================================================================================
// The anti-causal pair of the backward in one workgroup:
//   dV_j = sum_{i>=j} (q_i . k_j) dO_i ,   dK_j = sum_{i>=j} (dO_i . v_j) q_i
// (i, j over the tokens of j's document).  Both stream the same rows (Q and dO) and carry the
// same running state sum q^T dO, so one workgroup stages each 64-token block of Q and dO once
// and updates the state once for both: waves 0-3 own 32 rows each of a 128-row chunk for dV
// (their rows of K held as operand fragments, scores against the Q tile, dO tile mixed in) and
// waves 4-7 the same rows for dK (rows of V, scores against the dO tile, Q tile mixed in); all
// eight share the 16 state tiles, two each.  The state's bf16 snapshot is written once per
// chunk, [d_v][d_k]: the dV waves read it row-wise, the dK waves through the transposing LDS
// read, which hands them its transpose.  Waves s and s+4 share a SIMD and own row blocks s and
// 3-s, so that the triangular work of the two adds up evenly.
// Against two separate problems this saves half the stage loads, one of the two state updates
// (an eighth of the matrix-core work of the pair) and one snapshot per chunk.
//
// Walk: forwards, like the causal problem that shares the launch (and with it the L2 copies of K,
// V and dO).  The accumulators start from minus the inclusive suffix R at the slot's start and
// add q^T dO block by block, so on entering chunk c they hold minus R_c, the sum over chunk c and
// everything after it.  A row takes that state on ENTRY and subtracts what lies before it inside
// the chunk:  dV_j = k_j R_c - sum_{i<j, i in c} (q_i . k_j) dO_i  (dK alike).  The masked
// products therefore run over the strictly lower triangle (score tiles up to the row's own, the
// same number as for i >= j), a row is complete as soon as the walk has passed its own 32-row
// tile, and its fragments are then free for the next chunk's rows: row blocks 0 and 1 finish in
// the chunk's first 64-token block and request their next rows there, row blocks 2 and 3 in the
// second (template parameter LATE); all store in the second block, the early ones while the late
// ones still compute.  Every chunk is walked as two blocks; one that lies wholly past the slot's
// end is zeroed, not loaded.  Loads, counted waits (kept at run time as in skew_walk) and stores
// as in the other walks.
// =====================================================================================
struct PairProblem {
    const char* Q;
    const char* dO;
    const char* K;
    const char* V;
    const float* dR;   // [G][T_s][d][d]: inclusive suffix of Q^T dO at each slot's start
    char* dV;
    char* dK;
    unsigned* pace;    // NULL, or per (group, slot): receives the number of blocks this walk has begun
};

template <bool DKROLE, bool LATE>
__device__ __forceinline__ void pair_walk(const Geom& g, const PairProblem& pr, char* smem, int tid, int w,
                                          int rb, int grp, int s, int tok0, int len)
{
    constexpr int C = 128, NW = 8, TPW = 2, BPC = C / KB, IPW = 16 / NW, DPS = 2 * IPW, NOP = 4;
    char* sX = smem;                              // Q stages
    char* sY = smem + NSTAGE * STAGE_BYTES;       // dO stages
    char* sM = smem + 2 * NSTAGE * STAGE_BYTES;   // state snapshot, bf16 [d_v][d_k]
    char* sO = sM + D * ROWB;                     // output staging, 4 KiB per wave
    const int lane = tid & 63, h = lane >> 5, l32 = lane & 31;
    const char* __restrict__ A = DKROLE ? pr.V : pr.K;
    char* __restrict__ out = DKROLE ? pr.dK : pr.dV;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;
    const int t0 = w * TPW;
    const int nch = (len + C - 1) / C;
    const int NBP = nch * BPC;             // blocks walked (the last chunk padded to two)
    // Stage loads of block i.  The per-lane source offsets are rebuilt at every call from a lane index
    // the compiler cannot hoist: kept across the walk they cost registers this kernel does not have.
    auto issue = [&](int i) __attribute__((always_inline)) {
        int ln;
        asm volatile("v_and_b32 %0, 63, %1" : "=v"(ln) : "v"(tid));
        uint32_t dvo[IPW];
#pragma unroll
        for (int u = 0; u < IPW; ++u) dvo[u] = dma_lane_off(w * IPW + u, ln);
        dma_block<NW>(pr.Q, pr.dO, row0, i * KB, len, sX + (i % NSTAGE) * STAGE_BYTES,
                      sY + (i % NSTAGE) * STAGE_BYTES, w, ln, dvo);
    };
    issue(0);
    if (KB < len) issue(1);

    // running state tiles (rows d_k, columns d_v), holding minus the suffix
    f32x16 Macc[TPW];
    {
        const float* st = pr.dR + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
#pragma unroll
            for (int v = 0; v < 16; ++v)
                Macc[u][v] = -st[(32 * a + 8 * (v >> 2) + 4 * h + (v & 3)) * D + 32 * b + l32];
        }
    }

    // Per-lane byte offsets into a swizzled tile, one register per family as in skew_walk (the
    // swizzle is an XOR on the 16-byte chunk index, so the members of a family differ by an XOR
    // with a constant and a multiple of the row size):
    //   natural row l32, d step ks:                        nat0 ^ (ks << 5)
    //   transposed fetch of columns 32 tv + l32, rows r:   pvA ^ (tv << 6);  rows r + 8: (.. ^ 32) + 8 rows
    //   state update, X^T operand, rows r:                 uaA;              rows r + 4: (uaA ^ 16) + 4 rows
    //   state update, Y operand of tile u:                 uaA ^ ydel ^ (u << 6), ydel the same in all lanes
    //   snapshot read transposed (dK), columns 32 t + l32: uaA ^ xdel ^ (t << 6), rows r + 4 as above
    const int li = lane & 15, g2 = (lane >> 4) & 1, cl = 16 * g2 + 4 * (li & 3), rl = li >> 2;
    const uint32_t nat0 = (uint32_t)tile_off(l32, h);
    const uint32_t pvA = (uint32_t)tr_off(4 * h + rl, cl);
    const uint32_t uaA = (uint32_t)tr_off(8 * h + rl, 32 * (t0 >> 2) + cl);
    const uint32_t ydel = (uint32_t)(((t0 >> 2) ^ (t0 & 3)) << 6);
    const uint32_t xdel = (uint32_t)((t0 >> 2) << 6);

    // this wave's 32 rows of A as B-operand fragments, fetched asynchronously (see attn_mfma_kernel);
    // rows past the slot's end fetch its last row
    u32x4 qv[8];
    auto issue_q = [&](int c) __attribute__((always_inline)) {
        int lrow;   // lane % 32 in a form the compiler cannot hoist out of the chunk loop (and spill)
        asm volatile("v_and_b32 %0, 31, %1" : "=v"(lrow) : "v"(tid));
        const int r = min(c * C + 32 * rb + lrow, len - 1);
        const char* p = A + row0 + (size_t)r * ROWB + 16 * h;
        gload16_async<0>(qv[0], p);
        gload16_async<32>(qv[1], p);
        gload16_async<64>(qv[2], p);
        gload16_async<96>(qv[3], p);
        gload16_async<128>(qv[4], p);
        gload16_async<160>(qv[5], p);
        gload16_async<192>(qv[6], p);
        gload16_async<224>(qv[7], p);
    };
    auto take_q = [&](uint32_t zero) __attribute__((always_inline)) {
        const u32x4 z = {zero, zero, zero, zero};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qv[ks] = qv[ks] | z;
    };
    issue_q(0);
    take_q(wait_vmcnt_token<0>());   // also completes blocks 0 and 1 and the state
    const bf16x8 (&qf)[8] = reinterpret_cast<const bf16x8 (&)[8]>(qv);

    f32x16 Oacc[4];
    auto zero_out = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;
    };

    // vector-memory instructions certainly issued since the full wait above, and the marks of the
    // batches to wait for (see wait_vmcnt_le)
    int issued = 0, seq_cur = 0, seq_next = 0, seq_q = 0;

    char* tX = sX;
    char* tY = sY;
    // start of block bi: its loads have landed, the block is complete in LDS, every wave is past
    // block bi - 1, and the loads of block bi + 2 are on their way
    auto begin = [&](int bi) __attribute__((always_inline)) {
        tX = sX + (bi % NSTAGE) * STAGE_BYTES;
        tY = sY + (bi % NSTAGE) * STAGE_BYTES;
        wait_vmcnt_le(issued - seq_cur);
        if (bi * KB + KB > len) zero_tail_rows<NW>(bi * KB, len, tX, tY, w, lane);
        __syncthreads();
        if (pr.pace && w == 0) {
            if (lane == 0) __hip_atomic_store(pr.pace + ((size_t)grp * g.T_s + s), (unsigned)(bi + 1), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            issued += 1;
        }
        seq_cur = seq_next;
        if (bi + 2 < NBP && (bi + 2) * KB < len) { issue(bi + 2); issued += DPS; }
        seq_next = issued;
    };

    auto request_rows = [&](int c) __attribute__((always_inline)) {
        issue_q(c);
        issued += 8;
        seq_q = issued;
    };

    // The masked products of this wave's rows with the two 32-row tiles of block JB of the chunk, in
    // one of two forms.  EXIT: the rows take the state at the chunk's exit and GAIN what follows them
    // inside the chunk: their own tile from the diagonal on and the tiles after it.  Otherwise: the
    // rows take the state at the chunk's entry and LOSE what precedes them inside the chunk: the
    // tiles before their own, and their own strictly below the diagonal, all with a minus sign.
    auto tiles = [&](auto jb_c, auto exit_c) __attribute__((always_inline)) {
        constexpr int JB = decltype(jb_c)::value;
        constexpr bool EXIT = decltype(exit_c)::value;
        // rows scored against this wave's rows (S), rows mixed by the scores (C)
        const uint32_t aS = lds_addr_of(DKROLE ? tY : tX) + nat0, aC = lds_addr_of(DKROLE ? tX : tY) + pvA;
        bf16x8 bufA[NOP], bufB[NOP];
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const int kt = 2 * JB + half;      // 32-row tile of the streamed rows inside the chunk
            if (EXIT ? kt < rb : kt > rb) continue;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_u((aS ^ (ks << 5)) + half * (32 * ROWB));
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_u((aS ^ ((ks + 4) << 5)) + half * (32 * ROWB));
            SCHED_FENCE();
            f32x16 sc;
#pragma unroll
            for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufA[tv] = lds_read_tr8_u((aC ^ (tv << 6)) + half * (32 * ROWB),
                                          (aC ^ ((tv << 6) | 32)) + half * (32 * ROWB) + 8 * ROWB);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv)
                bufB[tv] = lds_read_tr8_u((aC ^ (tv << 6)) + half * (32 * ROWB) + 16 * ROWB,
                                          (aC ^ ((tv << 6) | 32)) + half * (32 * ROWB) + 24 * ROWB);
            SCHED_FENCE();
            if (kt == rb) {
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int key = 8 * (v >> 2) + 4 * h + (v & 3);
                    const bool keep = EXIT ? key >= l32 : key < l32;
                    sc[v] = keep ? sc[v] : 0.f;
                }
            }
            constexpr float sg = EXIT ? 1.f : -1.f;
            {
                u32x4 pk = {pack2(sg * sc[0], sg * sc[1]), pack2(sg * sc[2], sg * sc[3]), pack2(sg * sc[4], sg * sc[5]),
                            pack2(sg * sc[6], sg * sc[7])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufA[tv], sb, Oacc[tv]);
            }
            {
                u32x4 pk = {pack2(sg * sc[8], sg * sc[9]), pack2(sg * sc[10], sg * sc[11]), pack2(sg * sc[12], sg * sc[13]),
                            pack2(sg * sc[14], sg * sc[15])};
                bf16x8 sb = __builtin_bit_cast(bf16x8, pk);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufB[tv], sb, Oacc[tv]);
            }
            SCHED_FENCE();
        }
    };

    // running state += Q_blk^T dO_blk on this wave's two tiles, 16 tokens per step
    auto update = [&]() __attribute__((always_inline)) {
        const uint32_t aXA = lds_addr_of(tX) + uaA, aYA = lds_addr_of(tY) + (uaA ^ ydel);
        bf16x8 bufA[NOP], bufB[NOP];
        // operands of 16-token step ks: buf[0] = X^T rows of the wave's tile row, buf[1 + u] = Y
        // columns of tile u
        auto rd_upd = [&](bf16x8 (&buf)[NOP], int ks) __attribute__((always_inline)) {
            buf[0] = lds_read_tr8_u(aXA + ks * (16 * ROWB), (aXA ^ 16) + ks * (16 * ROWB) + 4 * ROWB);
#pragma unroll
            for (int u = 0; u < TPW; ++u)
                buf[1 + u] = lds_read_tr8_u((aYA ^ (u << 6)) + ks * (16 * ROWB),
                                            (aYA ^ ((u << 6) | 16)) + ks * (16 * ROWB) + 4 * ROWB);
        };
        rd_upd(bufA, 0);
        SCHED_FENCE();
        rd_upd(bufB, 1);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufA);
        SCHED_FENCE();
        rd_upd(bufA, 2);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufB);
        SCHED_FENCE();
        rd_upd(bufB, 3);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufA);
        SCHED_FENCE();
        mm_update<TPW, NOP>(Macc, bufB);
        SCHED_FENCE();
    };

    // inter-chunk term from the snapshot of the state at the chunk's entry
    auto inter = [&]() __attribute__((always_inline)) {
        bf16x8 bA[NOP], bB[NOP];
        if (!DKROLE) {
            // out^T (d_v x rows) += S^T (d_v x d_k) K_w^T: snapshot rows as they lie
            const uint32_t aM = lds_addr_of(sM) + nat0;
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) bA[tv] = lds_read16_u(aM + tv * (32 * ROWB));
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 8; ks += 2) {
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) bB[tv] = lds_read16_u((aM ^ ((ks + 1) << 5)) + tv * (32 * ROWB));
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bA[tv], qf[ks], Oacc[tv]);
                SCHED_FENCE();
                if (ks + 2 < 8) {
#pragma unroll
                    for (int tv = 0; tv < 4; ++tv) bA[tv] = lds_read16_u((aM ^ ((ks + 2) << 5)) + tv * (32 * ROWB));
                }
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bB[tv], qf[ks + 1], Oacc[tv]);
                SCHED_FENCE();
            }
        } else {
            // out^T (d_k x rows) += S (d_k x d_v) V_w^T: the snapshot read transposed
            const uint32_t aT = lds_addr_of(sM) + (uaA ^ xdel);
            auto rd = [&](bf16x8 (&buf)[NOP], int ks) __attribute__((always_inline)) {
#pragma unroll
                for (int t = 0; t < 4; ++t)
                    buf[t] = lds_read_tr8_u((aT ^ (t << 6)) + ks * (16 * ROWB),
                                            (aT ^ ((t << 6) | 16)) + ks * (16 * ROWB) + 4 * ROWB);
            };
            rd(bA, 0);
            SCHED_FENCE();
#pragma unroll
            for (int ks = 0; ks < 8; ks += 2) {
                rd(bB, ks + 1);
                SCHED_FENCE();
#pragma unroll
                for (int t = 0; t < 4; ++t) Oacc[t] = mfma(bA[t], qf[ks], Oacc[t]);
                SCHED_FENCE();
                if (ks + 2 < 8) rd(bA, ks + 2);
                SCHED_FENCE();
#pragma unroll
                for (int t = 0; t < 4; ++t) Oacc[t] = mfma(bB[t], qf[ks + 1], Oacc[t]);
                SCHED_FENCE();
            }
        }
    };

    // stores this wave's rows of chunk c (none when there is no such chunk) and clears the accumulators
    auto store_rows = [&](int c) __attribute__((always_inline)) {
        const int rbase = c * C + 32 * rb;
        const int nrows = c < 0 ? 0 : len - rbase;
        store_out_rows(Oacc, sO + w * 4096, out + row0 + (ptrdiff_t)rbase * ROWB, nrows, tid);
        if (nrows >= 32) issued += 8;   // all eight stores certainly execute
        SCHED_FENCE();
        zero_out();
    };

    using std::integral_constant;
    constexpr integral_constant<int, 0> B0{};
    constexpr integral_constant<int, 1> B1{};
    constexpr integral_constant<bool, false> ENTRY{};
    constexpr integral_constant<bool, true> EXIT{};

    // Rows 0..63 of a chunk (row blocks 0, 1; !LATE) use the entry form: they are complete after
    // the chunk's first block, are stored in its second, and their fragments are free for the next
    // chunk's rows a whole block before those are needed.  Rows 64..127 (LATE) use the exit form:
    // their tiles lie in the chunk's second block, the state at its exit is the snapshot at the
    // top of the NEXT chunk, so they are completed and stored in that chunk's first block, where
    // they also request their next rows.  Every snapshot thus serves both kinds of rows, and each
    // wave has a tile-free block per chunk for its stores and row fetches.
    // The slot's LAST chunk uses the exit form for all rows, against the state at the slot's end:
    // the entry form subtracts two sums of rounded terms, which is harmless while many later tokens
    // contribute to a row, but where a document ends inside or right after the chunk a row may
    // keep only a few terms, and those would then carry the rounding of all the cancelled ones.
    zero_out();
    const int n_loop = LATE ? nch : nch - 1;
    for (int c = 0; c < n_loop; ++c) {
        const int bi = c * BPC;
        // The state as the walk enters the chunk.  The previous chunk read its snapshot in its
        // first block; its second block's barrier lies in between.
        write_snapshot<TPW>(sM, Macc, t0, l32, h, true);

        // ---- block 0
        begin(bi);
        if (!LATE) {
            take_q(wait_vmcnt_token_le(issued - seq_q));
            inter();
            tiles(B0, ENTRY);
            request_rows(c + 1);   // the fragments are free for the next chunk's rows
        } else {
            // finish the rows of the previous chunk (at c = 0: the rows fetched before the walk, for
            // nothing; they are not stored), then ask for this chunk's
            inter();
            request_rows(c);
            store_rows(c - 1);
        }
        update();

        // ---- block 1
        begin(bi + 1);
        if (!LATE) {
            store_rows(c);
        } else {
            take_q(wait_vmcnt_token_le(issued - seq_q));
            tiles(B1, EXIT);
        }
        update();
    }
    if (!LATE) {
        // the last chunk, rows 0..63 in the exit form
        const int bi = (nch - 1) * BPC;
        write_snapshot<TPW>(sM, Macc, t0, l32, h, true);
        begin(bi);
        take_q(wait_vmcnt_token_le(issued - seq_q));
        tiles(B0, EXIT);
        update();
        begin(bi + 1);
        tiles(B1, EXIT);
        update();
    }
    // the state beyond the slot's last chunk, for the rows that await it
    write_snapshot<TPW>(sM, Macc, t0, l32, h, true);
    __syncthreads();
    inter();
    store_rows(nch - 1);
    // nothing left to keep in step with: release a partner that counts blocks this walk does not have
    // (the other walk pads its chunks to 256 rows)
    if (pr.pace && w == 0 && lane == 0)
        __hip_atomic_store(pr.pace + ((size_t)grp * g.T_s + s), 0x7fffffffu, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__global__ void zero_u32_kernel(unsigned* p, unsigned n)
{
    const unsigned i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// The backward's attention launch for slots longer than 128 tokens, without decay: per (group,
// slot) one workgroup for the anti-causal pair (pair_walk) and one for dQ (the causal skew_walk),
// dealt to the same XCD like the problems of attn_skew_mfma_kernel; the pair's workgroup, which
// has more to do, comes first in the grid.
__global__ __launch_bounds__(512) void attn_bwd_pair_mfma_kernel(Geom g, AttnProblem pq, PairProblem pp)
{
    extern __shared__ __attribute__((aligned(256))) char smem[];
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const unsigned unit = (blockIdx.x / 16u) * 8u + (blockIdx.x & 7u);
    const int prob = (int)(blockIdx.x >> 3) & 1;
    if (unit >= (unsigned)g.T_s * (unsigned)g.G) return;
    const int s = (int)(unit % (unsigned)g.T_s), grp = (int)(unit / (unsigned)g.T_s);
    int tok0, len, ps;
    slot_range(g, s, tok0, len, ps);
    if (len <= 0) return;
    if (prob == 0) {
        // waves s and s+4 share a SIMD: row block s for dV, 3-s for dK
        if (w < 2) pair_walk<false, false>(g, pp, smem, tid, w, w, grp, s, tok0, len);
        else if (w < 4) pair_walk<false, true>(g, pp, smem, tid, w, w, grp, s, tok0, len);
        else if (w < 6) pair_walk<true, true>(g, pp, smem, tid, w, 7 - w, grp, s, tok0, len);
        else pair_walk<true, false>(g, pp, smem, tid, w, 7 - w, grp, s, tok0, len);
    } else {
        const int rb = w < 4 ? w : 11 - w;
        const float* wstate = pq.state ? walk_state(g, pq, grp, s, ps) : nullptr;
        if (rb < 4) skew_walk<false, false, false>(g, pq, smem, tid, w, rb, grp, s, tok0, len, wstate);
        else skew_walk<true, false, false>(g, pq, smem, tid, w, rb, grp, s, tok0, len, wstate);
    }
}

template <int C>
hipError_t launch_attn_C(const Geom& g, const AttnProblem& p0, const AttnProblem& p1,
                         const AttnProblem& p2, int nprob, hipStream_t st)
{
    // stages + snapshot + 4 KiB of output staging per wave
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + D * ROWB + (C / 32) * 4096;
    auto kern = attn_mfma_kernel<C>;
    hipError_t e = allow_dynamic_lds<attn_mfma_kernel<C>>(smem);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)g.T_s * (unsigned)g.G;
    const unsigned gx = (unsigned)nprob * ((units + 7u) & ~7u);
    dim3 grid(gx), block(C * 2);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, p0, p1, p2, nprob);
    return hipGetLastError();
}

template <bool DECAY>
hipError_t launch_attn_skew(const Geom& g, const AttnProblem& p0, const AttnProblem& p1,
                            const AttnProblem& p2, int nprob, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + D * ROWB + 8 * 4096;
    auto kern = attn_skew_mfma_kernel<DECAY>;
    hipError_t e = allow_dynamic_lds<attn_skew_mfma_kernel<DECAY>>(smem);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)g.T_s * (unsigned)g.G;
    const unsigned gx = (unsigned)nprob * ((units + 7u) & ~7u);
    dim3 grid(gx), block(512);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, p0, p1, p2, nprob);
    return hipGetLastError();
}

// Internal chunk of the fused pass: 256 rows (eight waves) unless no slot is longer than 128.
bool wide_chunks(const Geom& g) { return g.L > 128; }

AttnProblem make_problem(const void* A, const void* Bk, const void* Cv, const float* state, int user_state,
                         void* out, int transpose_state, int anti)
{
    return AttnProblem{static_cast<const char*>(A), static_cast<const char*>(Bk),
                       static_cast<const char*>(Cv), state, user_state, static_cast<char*>(out),
                       transpose_state, anti, nullptr, 0};
}

// =====================================================================================
// Fused attention pass with scalar decay: out_i = sum_j lam^|i-j| (a_i . bk_j) cv_j over the
// allowed pairs plus the decayed inter-chunk term, for slots of at most 128 tokens (longer ones:
// skew_walk with DECAY).  Same tiles, stages, layouts and asynchronous fetches as
// attn_mfma_kernel<128>, with these differences:
//   - Anti-causal problems walk the slot BACKWARDS (blocks and chunks in descending order, the
//     slot state being the exclusive suffix): with decay the forward walk with a subtracted
//     suffix would have to divide by lam at every step.  Both directions therefore take the
//     state snapshot and the inter-chunk product when the walk enters a chunk.
//   - Each wave multiplies the rows of the Bk tile it staged by the token's weight as seen from
//     the block's last token (causal, lam^(63-b)) or first token (anti-causal, lam^b) before the
//     block barrier.  The state update then is lam^64 * state + Bk~^T Cv, and a score computed
//     from the weighted rows needs only a factor per query, lam^(i - block start - 63) resp.
//     lam^(block start - i), to become lam^|i-j| (a_i . bk_j); a query and the keys it meets lie
//     in the same 128 rows, so the exponents stay within -63..64.
//   - The inter-chunk product is scaled per query by lam^(a+1) (causal, a = index in the chunk)
//     or lam^(chunk length - a) (anti-causal).
// =====================================================================================
template <int C>
__global__ __launch_bounds__(C * 2) void attn_decay_mfma_kernel(Geom g, AttnProblem p0, AttnProblem p1,
                                                                AttnProblem p2, int nprob)
{
    constexpr int NW = C / 32, TPW = 16 / NW, BPC = C / KB, IPW = 16 / NW, DPS = 2 * IPW;
    constexpr int NOP = (TPW + 1 > 4) ? 8 : 4;
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sK = smem;                              // Bk stages
    char* sV = smem + NSTAGE * STAGE_BYTES;       // Cv stages
    char* sM = smem + 2 * NSTAGE * STAGE_BYTES;   // state snapshot, bf16 [d_v][d_k]
    char* sO = sM + D * ROWB;                     // output staging, 4 KiB per wave

    const int tid = threadIdx.x, lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int h = lane >> 5, l32 = lane & 31;
    const unsigned unit = (blockIdx.x / (8u * nprob)) * 8u + (blockIdx.x & 7u);
    const int prob = (int)(blockIdx.x >> 3) % nprob;
    if (unit >= (unsigned)g.T_s * (unsigned)g.G) return;
    const int s = (int)(unit % (unsigned)g.T_s), grp = (int)(unit / (unsigned)g.T_s);
    const AttnProblem& pr = prob == 0 ? p0 : (prob == 1 ? p1 : p2);
    const char* __restrict__ A = pr.A;
    const char* __restrict__ Bk = pr.Bk;
    const char* __restrict__ Cv = pr.Cv;
    char* __restrict__ out = pr.out;
    const bool rev = pr.anti != 0;
    int tok0, len, ps;
    slot_range(g, s, tok0, len, ps);
    if (len <= 0) return;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;
    const float l2 = uniform_f32(decay_log2(g, grp));   // one value per workgroup: scalar
    const int rb = (NW == 8) ? (w < 4 ? w : 11 - w) : w;   // as in attn_mfma_kernel
    const int t0 = w * TPW;

    const int nch = (len + C - 1) / C;
    const int NB = (len + KB - 1) / KB;    // 64-token blocks in the whole slot
    uint32_t dvo[IPW];
#pragma unroll
    for (int u = 0; u < IPW; ++u) dvo[u] = dma_lane_off(w * IPW + u, lane);
    // walk position i -> block of the slot
    auto issue = [&](int i) {
        const int bb = rev ? NB - 1 - i : i;
        dma_block<NW>(Bk, Cv, row0, bb * KB, len, sK + (i % NSTAGE) * STAGE_BYTES,
                      sV + (i % NSTAGE) * STAGE_BYTES, w, lane, dvo);
    };
    issue(0);
    if (NB > 1) issue(1);

    // running state tiles, C/D layout: rows = d_k (first index), columns = d_v
    f32x16 Macc[TPW];
#pragma unroll
    for (int u = 0; u < TPW; ++u)
#pragma unroll
        for (int v = 0; v < 16; ++v) Macc[u][v] = 0.f;
    if (pr.state) {   // NULL: every slot opens its document and starts from a zero state
        const float* st = walk_state(g, pr, grp, s, ps);
#pragma unroll
        for (int u = 0; u < TPW; ++u) {
            const int t = t0 + u, a = t >> 2, b = t & 3;
            if (!pr.transpose_state) {
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

    LaneOffs<TPW> lo;
    make_lane_offs<TPW>(lo, lane, t0);

    // lam^64 for the state (the same in every lane)
    const float wblk = uniform_f32(exp2f((float)KB * l2));

    // This wave's 32 rows of A as B-operand fragments, fetched asynchronously as in
    // attn_mfma_kernel; rows past the slot's end fetch its last row (they only feed output rows
    // that are not stored, and a column of the products depends on its own row alone).
    u32x4 qv[8];
    auto issue_q = [&](int cc) {
        int lrow;   // lane % 32 again, in a form the compiler cannot hoist (and then spill)
        asm volatile("v_and_b32 %0, 31, %1" : "=v"(lrow) : "v"(tid));
        const int r = min(cc * C + 32 * rb + lrow, len - 1);
        const char* p = A + row0 + (size_t)r * ROWB + 16 * h;
        gload16_async<0>(qv[0], p);
        gload16_async<32>(qv[1], p);
        gload16_async<64>(qv[2], p);
        gload16_async<96>(qv[3], p);
        gload16_async<128>(qv[4], p);
        gload16_async<160>(qv[5], p);
        gload16_async<192>(qv[6], p);
        gload16_async<224>(qv[7], p);
    };
    auto take_q = [&](uint32_t zero) {
        const u32x4 z = {zero, zero, zero, zero};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qv[ks] = qv[ks] | z;
    };
    issue_q(rev ? nch - 1 : 0);
    take_q(wait_vmcnt_token<0>());
    const bf16x8 (&qf)[8] = reinterpret_cast<const bf16x8 (&)[8]>(qv);

    int bi = 0;          // walk position of the block being consumed
    int prev_nblk = BPC;
    for (int c = 0; c < nch; ++c) {
        const int cc = rev ? nch - 1 - c : c;               // chunk of the slot
        const int b_lo = cc * BPC, b_hi = min(NB, b_lo + BPC);
        const int nblk = b_hi - b_lo;
        const int clen = min(C, len - cc * C);
        const bool last_chunk = (c + 1 == nch);

        // The previous chunk read its last snapshot in its first or third block; one of its later
        // block barriers separates that from this write unless it had a single block (a chunk of
        // three blocks is the slot's last one: nothing follows it in the forward walk, and the
        // backward walk enters its lower half at the second block).
        if (prev_nblk < 2) __syncthreads();
        write_snapshot<TPW>(sM, Macc, t0, l32, h, false);

        f32x16 Oacc[4];
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;

        for (int jb = 0; jb < nblk; ++jb, ++bi) {
            const int bb = rev ? b_hi - 1 - jb : b_lo + jb;   // block of the slot
            const int jbb = bb - b_lo;                         // its index inside the chunk
            char* tK = sK + (bi % NSTAGE) * STAGE_BYTES;
            char* tV = sV + (bi % NSTAGE) * STAGE_BYTES;
            // this wave's loads of block bi have landed (those of bi+1 may still fly); in the first
            // two blocks after a chunk boundary the previous chunk's eight stores are younger too
            if (c > 0 && jb < 2) {
                if (bi + 1 < NB) wait_vmcnt<DPS + 8>(); else wait_vmcnt<8>();
            } else {
                if (bi + 1 < NB) wait_vmcnt<DPS>(); else wait_vmcnt<0>();
            }
            if (bb * KB + KB > len) zero_tail_rows<NW>(bb * KB, len, tK, tV, w, lane);
            // weight this wave's own rows of the Bk tile (a whole row takes one weight, so the
            // swizzle does not matter here)
#pragma unroll
            for (int u = 0; u < IPW; ++u) {
                const int b = 4 * (w * IPW + u) + (lane >> 4);
                const float wr = __builtin_amdgcn_exp2f((float)(rev ? b : KB - 1 - b) * l2);
                u32x4* pk = reinterpret_cast<u32x4*>(tK + b * ROWB + (lane & 15) * 16);
                *pk = scale_bf16x8(*pk, wr);
            }
            __syncthreads();   // block complete and weighted in LDS; every wave is past the previous one
            if (bi + 2 < NB) issue(bi + 2);

            // The walk enters the chunk: its rows take the inter-chunk product from the state as it
            // stands, which sits one token before the chunk (causal) or one after it (anti-causal).
            if (jb == 0) {
                inter_product<NOP>(Oacc, sM, qf, lo.nat);
                int lrow;   // lane % 32, kept out of the loop-invariant (and then spilled) values
                asm volatile("v_and_b32 %0, 31, %1" : "=v"(lrow) : "v"(tid));
                const int a = 32 * rb + lrow;
                const int e = rev ? max(clen - a, 0) : a + 1;
                const float wq = __builtin_amdgcn_exp2f((float)e * l2);
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
#pragma unroll
                    for (int v = 0; v < 16; ++v) Oacc[tv][v] *= wq;
            }

            bf16x8 bufA[NOP], bufB[NOP];
#pragma unroll
            for (int half = 0; half < 2; ++half) {
                const int kt = 2 * jbb + half;      // 32-key tile index inside the chunk
                const bool active = rev ? (kt >= rb) : (kt <= rb);
                if (!active) continue;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) bufA[ks] = lds_read16_at(tK + half * (32 * ROWB), lo.nat[ks]);
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) bufB[ks] = lds_read16_at(tK + half * (32 * ROWB), lo.nat[ks + 4]);
                SCHED_FENCE();
                f32x16 sc;
#pragma unroll
                for (int v = 0; v < 16; ++v) sc[v] = 0.f;
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) sc = mfma(bufA[ks], qf[ks], sc);
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
                    bufA[tv] = lds_read_tr8_at(tV + half * (32 * ROWB), lo.pv[tv][0], lo.pv[tv][1]);
                SCHED_FENCE();
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) sc = mfma(bufB[ks], qf[ks + 4], sc);
                SCHED_FENCE();
#pragma unroll
                for (int tv = 0; tv < 4; ++tv)
                    bufB[tv] = lds_read_tr8_at(tV + half * (32 * ROWB) + 16 * ROWB, lo.pv[tv][0], lo.pv[tv][1]);
                SCHED_FENCE();
                {
                    // from the row weights of the block to lam^|i-j|: one factor per query
                    const int qi = 32 * rb + l32 - KB * jbb;   // query index relative to the block's start
                    const float f = __builtin_amdgcn_exp2f((float)(rev ? -qi : qi - (KB - 1)) * l2);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int key = 8 * (v >> 2) + 4 * h + (v & 3);
                        const bool keep = (kt != rb) || (rev ? (key >= l32) : (key <= l32));
                        sc[v] = keep ? sc[v] * f : 0.f;
                    }
                }
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

            // the rows of the next chunk replace qf while the state update and the store run
            if (jb + 1 == nblk && !last_chunk) issue_q(rev ? cc - 1 : cc + 1);
            if (!last_chunk) {
                // running state = lam^n * state + (weighted Bk block)^T Cv block, n = the block's
                // tokens (fewer than 64 only in the slot's last block, which the backward walk
                // meets first)
                const float wb = (bb * KB + KB <= len) ? wblk : __builtin_amdgcn_exp2f((float)(len - bb * KB) * l2);
#pragma unroll
                for (int u = 0; u < TPW; ++u)
#pragma unroll
                    for (int v = 0; v < 16; ++v) Macc[u][v] *= wb;
                rd_update<TPW, NOP>(bufA, tK, tV, 0, lo);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufB, tK, tV, 1, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufA);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufA, tK, tV, 2, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufB);
                SCHED_FENCE();
                rd_update<TPW, NOP>(bufB, tK, tV, 3, lo);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufA);
                SCHED_FENCE();
                mm_update<TPW, NOP>(Macc, bufB);
            }
        }
        prev_nblk = nblk;

        // store this wave's 32 output rows, as in attn_mfma_kernel
        {
            const int rbase = cc * C + 32 * rb;
            store_out_rows(Oacc, sO + w * 4096, out + row0 + (size_t)rbase * ROWB, len - rbase, tid);
        }
        // Only the eight stores above were issued after the rows of A for the next chunk.  All eight
        // execute when the chunk is full; the backward walk starts with the slot's last chunk, which
        // may not be.
        if (!last_chunk) {
            if (clen == C) take_q(wait_vmcnt_token<8>()); else take_q(wait_vmcnt_token<0>());
        }
    }
}

// =====================================================================================
// Rows times a slot state, for the path without masking: out = A W over the rows of one slot,
// W = state[slot] or its transpose (O_t = Q_t M_{1:T}; dQ_t = dO_t M_{1:T}^T, dK_t = V_t
// dM_{1:T}^T, dV_t = K_t dM_{1:T}).  The work is two passes over HBM per product (rows in,
// rows out), so the kernel only has to keep loads in flight: eight waves, each fetching its
// next 32 rows while the matrix cores handle the current ones.  W sits in LDS as bf16,
// [column of out][contracted index], the layout the inter-chunk product of the fused pass uses.
// =====================================================================================
constexpr int RS_NW = 8;

struct RowsStateArgs {
    const char* A;
    const float* state;
    char* out;
    int transpose_state;
};

__global__ __launch_bounds__(RS_NW * 64) void rows_state_mfma_kernel(Geom g, RowsStateArgs p0, RowsStateArgs p1,
                                                                     RowsStateArgs p2, int nprob)
{
    extern __shared__ __attribute__((aligned(16))) char smem[];
    char* sW = smem;               // bf16 [128 columns of out][128 contracted], swizzled tile
    char* sO = smem + D * ROWB;    // output staging, 4 KiB per wave

    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int h = lane >> 5, l32 = lane & 31;
    // same workgroup-to-slot mapping as the fused pass: the nprob products of a slot share an XCD
    const unsigned unit = (blockIdx.x / (8u * nprob)) * 8u + (blockIdx.x & 7u);
    const int prob = (int)(blockIdx.x >> 3) % nprob;
    if (unit >= (unsigned)g.T_s * (unsigned)g.G) return;
    const int s = (int)(unit % (unsigned)g.T_s), grp = (int)(unit / (unsigned)g.T_s);
    const RowsStateArgs& pr = prob == 0 ? p0 : (prob == 1 ? p1 : p2);
    int tok0, len;
    slot_range(g, s, tok0, len);
    if (len <= 0) return;
    const size_t row0 = ((size_t)grp * g.N + tok0) * ROWB;
    const char* __restrict__ A = pr.A + row0;
    char* __restrict__ out = pr.out + row0;

    {
        const float* st = pr.state + ((size_t)grp * g.T_s + s) * (size_t)(D * D);
        for (int i = tid; i < D * 16; i += RS_NW * 64) {
            float x[8];
            int c, q;   // column of out, 16-byte piece (contracted indices 8q .. 8q+7)
            if (pr.transpose_state) {
                c = i >> 4;
                q = i & 15;
                const f32x4 a = *reinterpret_cast<const f32x4*>(st + c * D + 8 * q);
                const f32x4 b = *reinterpret_cast<const f32x4*>(st + c * D + 8 * q + 4);
#pragma unroll
                for (int e = 0; e < 4; ++e) { x[e] = a[e]; x[4 + e] = b[e]; }
            } else {
                q = i >> 7;
                c = i & 127;
#pragma unroll
                for (int e = 0; e < 8; ++e) x[e] = st[(8 * q + e) * D + c];
            }
            const u32x4 pk = {pack2(x[0], x[1]), pack2(x[2], x[3]), pack2(x[4], x[5]), pack2(x[6], x[7])};
            *reinterpret_cast<u32x4*>(sW + tile_off(c, q)) = pk;
        }
    }
    __syncthreads();

    int nat[8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) nat[ks] = tile_off(l32, 2 * ks + h);

    // 32 rows of A as B-operand fragments (column = row of A, k = contracted index)
    auto load_rows = [&](u32x4 (&dst)[8], int r) {
        const bool ok = r < len;
        const char* p = A + (size_t)r * ROWB + 16 * h;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const u32x4 z = {0u, 0u, 0u, 0u};
            dst[ks] = ok ? *reinterpret_cast<const u32x4*>(p + 32 * ks) : z;
        }
    };

    const int nit = (len + RS_NW * 32 - 1) / (RS_NW * 32);
    u32x4 cur[8], nxt[8];
    load_rows(cur, 32 * w + l32);
    char* stg = sO + w * 4096;
    for (int it = 0; it < nit; ++it) {
        const int rbase = it * (RS_NW * 32) + 32 * w;
        if (it + 1 < nit) load_rows(nxt, rbase + RS_NW * 32 + l32);

        f32x16 Oacc[4];
#pragma unroll
        for (int tv = 0; tv < 4; ++tv)
#pragma unroll
            for (int v = 0; v < 16; ++v) Oacc[tv][v] = 0.f;
        bf16x8 bufA[4], bufB[4];
#pragma unroll
        for (int tv = 0; tv < 4; ++tv) bufA[tv] = lds_read16_at(sW + tv * (32 * ROWB), nat[0]);
#pragma unroll
        for (int ks = 0; ks < 8; ks += 2) {
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) bufB[tv] = lds_read16_at(sW + tv * (32 * ROWB), nat[ks + 1]);
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufA[tv], __builtin_bit_cast(bf16x8, cur[ks]), Oacc[tv]);
            SCHED_FENCE();
            if (ks + 2 < 8) {
#pragma unroll
                for (int tv = 0; tv < 4; ++tv) bufA[tv] = lds_read16_at(sW + tv * (32 * ROWB), nat[ks + 2]);
            }
            SCHED_FENCE();
#pragma unroll
            for (int tv = 0; tv < 4; ++tv) Oacc[tv] = mfma(bufB[tv], __builtin_bit_cast(bf16x8, cur[ks + 1]), Oacc[tv]);
            SCHED_FENCE();
        }

        // out^T tiles (lane = row) -> wave-private 4 KiB patch -> 16-byte row-contiguous stores,
        // half of the 128 columns at a time (as in the fused pass)
#pragma unroll
        for (int hv = 0; hv < 2; ++hv) {
#pragma unroll
            for (int tvv = 0; tvv < 2; ++tvv)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x16& o = Oacc[2 * hv + tvv];
                    u32x2 pk = {pack2(o[4 * q], o[4 * q + 1]), pack2(o[4 * q + 2], o[4 * q + 3])};
                    *reinterpret_cast<u32x2*>(stg + l32 * 128 + (((4 * tvv + q) ^ (l32 & 7)) << 4) + 8 * h) = pk;
                }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int idx = lane + 64 * i, row = idx >> 3, ch = idx & 7;
                const u32x4 v = *reinterpret_cast<const u32x4*>(stg + row * 128 + ((ch ^ (row & 7)) << 4));
                if (rbase + row < len)
                    __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(out + (size_t)(rbase + row) * ROWB + 128 * hv + 16 * ch));
            }
        }
        if (it + 1 < nit) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) cur[ks] = nxt[ks];
        }
    }
}

}  // namespace

bool mfma_path_supported(const Geom& g, int dtype)
{
    // The kernels tile a slot in their own chunks (the result does not depend on the chunk
    // length), so every C of the caller is served.  With decay the factors must keep lam^-63
    // and lam^63 well inside the fp32 / bf16 range (decided on the host, see make_geom).
    return dtype == LASP2_BF16 && g.d == D && (g.decay == nullptr || g.decay_mfma);
}

hipError_t launch_states_mfma(const Geom& g, const void* K, const void* V, float* M, int anchor_start,
                              hipStream_t st)
{
    constexpr int smem = 2 * ST_NST * ST_STAGE;   // 80 KiB: two workgroups per CU
    auto kern = g.decay ? states_mfma_kernel<true> : states_mfma_kernel<false>;
    hipError_t e = g.decay ? allow_dynamic_lds<states_mfma_kernel<true>>(smem)
                           : allow_dynamic_lds<states_mfma_kernel<false>>(smem);
    if (e != hipSuccess) return e;
    // two workgroups per CU, each walking through its share of the slots
    const int cus = cu_count();
    const long long nunits = (long long)g.T_s * g.G;
    if (nunits == 0) return hipSuccess;
    dim3 grid((unsigned)std::min<long long>(nunits, 2LL * cus)), block(ST_NT);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, static_cast<const char*>(K),
                       static_cast<const char*>(V), M, anchor_start);
    return hipGetLastError();
}

namespace {
template <int C>
hipError_t launch_attn_decay_C(const Geom& g, const AttnProblem& p0, const AttnProblem& p1,
                               const AttnProblem& p2, int nprob, hipStream_t st)
{
    constexpr int smem = 2 * NSTAGE * STAGE_BYTES + D * ROWB + (C / 32) * 4096;
    auto kern = attn_decay_mfma_kernel<C>;
    hipError_t e = allow_dynamic_lds<attn_decay_mfma_kernel<C>>(smem);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)g.T_s * (unsigned)g.G;
    const unsigned gx = (unsigned)nprob * ((units + 7u) & ~7u);
    dim3 grid(gx), block(C * 2);
    hipLaunchKernelGGL(kern, grid, block, smem, st, g, p0, p1, p2, nprob);
    return hipGetLastError();
}

hipError_t launch_attn_decay(const Geom& g, const AttnProblem& p0, const AttnProblem& p1,
                             const AttnProblem& p2, int nprob, hipStream_t st)
{
    if (wide_chunks(g)) return launch_attn_skew<true>(g, p0, p1, p2, nprob, st);
    return launch_attn_decay_C<128>(g, p0, p1, p2, nprob, st);
}
}  // namespace

hipError_t launch_attn_fwd_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                const float* P, void* O, hipStream_t st)
{
    const AttnProblem p = make_problem(Q, K, V, P, 1, O, 0, 0);
    if (g.decay) return launch_attn_decay(g, p, p, p, 1, st);
    if (wide_chunks(g)) return launch_attn_skew<false>(g, p, p, p, 1, st);
    return launch_attn_C<128>(g, p, p, p, 1, st);
}

hipError_t launch_attn_bwd_mfma(const Geom& g, const void* Q, const void* K, const void* V,
                                const void* dO, const float* P, const float* dR, unsigned* pace, void* dQ,
                                void* dK, void* dV, hipStream_t st)
{
    // dQ: the forward problem with (dO, V, K) in the roles of (Q, K, V); its state V^T K is the
    //     cached prefix read transposed.
    // dV: anti-causal problem with (K, Q, dO); state = suffix of Q^T dO.
    // dK: anti-causal problem with (V, dO, Q); state dO^T Q = that suffix transposed.
    const AttnProblem pq = make_problem(dO, V, K, P, 1, dQ, 1, 0);
    const AttnProblem pv = make_problem(K, Q, dO, dR, 0, dV, 0, 1);
    const AttnProblem pk = make_problem(V, dO, Q, dR, 0, dK, 1, 1);
    if (g.decay) return launch_attn_decay(g, pq, pv, pk, 3, st);
    if (wide_chunks(g)) {
        constexpr int smem = 2 * NSTAGE * STAGE_BYTES + D * ROWB + 8 * 4096;
        hipError_t e = allow_dynamic_lds<attn_bwd_pair_mfma_kernel>(smem);
        if (e != hipSuccess) return e;
        // The two workgroups of a slot share their reads of K, V and dO through the L2 only while
        // they stay close: the pair's workgroup counts the blocks it has begun in pace[unit], and the
        // faster dQ walk does not run ahead of that count.
        const unsigned units = (unsigned)g.T_s * (unsigned)g.G;
        AttnProblem pq2 = pq;
        if (pace) {
            hipLaunchKernelGGL(zero_u32_kernel, dim3((units + 255u) / 256u), dim3(256), 0, st, pace, units);
            pq2.pace = pace;
            pq2.lead = 0;   // (leads of -1 .. 2 blocks measured alike)
        }
        const PairProblem pp = {static_cast<const char*>(Q), static_cast<const char*>(dO),
                                static_cast<const char*>(K), static_cast<const char*>(V), dR,
                                static_cast<char*>(dV), static_cast<char*>(dK), pace};
        dim3 grid(2u * ((units + 7u) & ~7u)), block(512);
        hipLaunchKernelGGL(attn_bwd_pair_mfma_kernel, grid, block, smem, st, g, pq2, pp);
        return hipGetLastError();
    }
    return launch_attn_C<128>(g, pq, pv, pk, 3, st);
}

hipError_t launch_rows_state_mfma(const Geom& g, const RowsStateProblem* probs, int n, hipStream_t st)
{
    constexpr int smem = D * ROWB + RS_NW * 4096;   // 64 KiB
    RowsStateArgs a[3];
    for (int i = 0; i < 3; ++i) {
        const RowsStateProblem& p = probs[i < n ? i : 0];
        a[i] = RowsStateArgs{static_cast<const char*>(p.A), p.state, static_cast<char*>(p.out), p.transpose_state};
    }
    hipError_t e = allow_dynamic_lds<rows_state_mfma_kernel>(smem);
    if (e != hipSuccess) return e;
    const unsigned units = (unsigned)g.T_s * (unsigned)g.G;
    const unsigned gx = (unsigned)n * ((units + 7u) & ~7u);
    dim3 grid(gx), block(RS_NW * 64);
    hipLaunchKernelGGL(rows_state_mfma_kernel, grid, block, smem, st, g, a[0], a[1], a[2], n);
    return hipGetLastError();
}

}  // namespace lasp2
