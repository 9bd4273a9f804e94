// Building blocks shared by the bf16 MFMA kernels of liblasp2 (gfx950, d = 128): vector types,
// the swizzled 256-byte-row LDS tile and its two read shapes, the MFMA and conversion wrappers,
// the direct global->LDS stage loads with their hand-counted waits.
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
#ifndef LASP2_MFMA_TILE_H
#define LASP2_MFMA_TILE_H
#include "lasp2_common.h"
#include <type_traits>

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

// The swizzle depends on row % 16 only, so a lane's byte offset inside a tile can be computed
// once and reused for every tile, stage and 16-row step by adding a constant: the helpers below
// read at (tile + constant) + precomputed lane offset.
__device__ __forceinline__ int tr_off(int row, int col)
{
    return tile_off(row, col >> 3) + (col & 7) * 2;
}

__device__ __forceinline__ bf16x8 lds_read16_at(const char* base, int lane_off)
{
    return *reinterpret_cast<const bf16x8*>(base + lane_off);
}

// The same two reads from 32-bit LDS addresses (a per-lane register that already contains the
// array's base, plus a compile-time constant): the constant goes into the instruction's offset
// field, so the read costs no address arithmetic.
__device__ __forceinline__ bf16x8 lds_read16_u(uint32_t addr)
{
    return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(addr);
}

__device__ __forceinline__ bf16x8 lds_read_tr8_u(uint32_t addr_lo, uint32_t addr_hi)
{
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4_ptr>(addr_lo));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4_ptr>(addr_hi));
    s16x8 both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

// Makes a computed per-lane value opaque to the compiler, so that it is kept in its register
// instead of being re-derived from its parts (one more add) at every use inside a loop.
__device__ __forceinline__ void pin_vgpr(uint32_t& x) { asm volatile("" : "+v"(x)); }

__device__ __forceinline__ bf16x8 lds_read_tr8_at(const char* base, int off_lo, int off_hi)
{
    typedef s16x4 __attribute__((address_space(3))) * lds_s16x4_ptr;
    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + off_lo));
    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(base + off_hi));
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

// ---- ring of LDS stages filled by direct global->LDS loads ----
constexpr int NSTAGE = 3;

__device__ __forceinline__ uint32_t lds_addr_of(const char* p)
{
    return (uint32_t)(uintptr_t)(const __attribute__((address_space(3))) char*)p;
}

// One wave instruction of direct global->LDS load: lane l fetches the 16 bytes at sbase + voff
// (sbase and lds_base uniform, held in scalar registers; voff per lane) into LDS at
// lds_base + 16 l.  The statement writes M0 and says so in its clobber list, so that the
// compiler never carries a value of its own in M0 across it; the compiler reserves M0 and
// remarks on any clobber of a reserved register, which is silenced for these statements only.
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void dma16(const char* sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory", "m0");
}

// The same load marked non-temporal, for data that is read exactly once.
__device__ __forceinline__ void dma16_nt(const char* sbase, uint32_t voff, uint32_t lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2 nt" ::"s"(lds_base), "v"(voff), "s"(sbase) : "memory", "m0");
}
#pragma clang diagnostic pop

// Byte offset, inside a block of rows that starts at a multiple of 16, of the 16 bytes that lane
// `lane` of wave instruction `k` (rows 4k .. 4k+3) must fetch so that they land swizzled.
__device__ __forceinline__ uint32_t dma_lane_off(int k, int lane)
{
    const int r = 4 * k + (lane >> 4);
    return (uint32_t)(r * ROWB + (((lane & 15) ^ swz(r)) << 4));
}

// Issue the loads of one 64-token block (rows tok .. tok+63 of the slot) of X and Y into the
// stage tiles tx, ty; dvo[u] = dma_lane_off(w * IPW + u, lane), computed once per kernel.
// Rows past the slot's end are fetched from its last row (always in bounds) and zeroed
// afterwards by zero_tail_rows().
template <int NW, bool STREAM = false>
__device__ __forceinline__ void dma_block(const char* X, const char* Y, size_t row0_bytes, int tok,
                                          int len, char* tx, char* ty, int w, int lane,
                                          const uint32_t (&dvo)[16 / NW])
{
    constexpr int IPW = 16 / NW;   // wave instructions per tensor per stage
    const size_t blk = row0_bytes + (size_t)tok * ROWB;
    const bool full = tok + KB <= len;
#pragma unroll
    for (int u = 0; u < IPW; ++u) {
        const int k = w * IPW + u;
        uint32_t voff = dvo[u];
        if (!full) {
            const int r = 4 * k + (lane >> 4);
            voff = (uint32_t)(min(r, len - 1 - tok) * ROWB + (int)(voff & (ROWB - 1)));
        }
        if (STREAM) {
            dma16_nt(X + blk, voff, lds_addr_of(tx + 4 * k * ROWB));
            dma16_nt(Y + blk, voff, lds_addr_of(ty + 4 * k * ROWB));
        } else {
            dma16(X + blk, voff, lds_addr_of(tx + 4 * k * ROWB));
            dma16(Y + blk, voff, lds_addr_of(ty + 4 * k * ROWB));
        }
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

// Counted waits.  Built with -DLASP2_FULL_WAITS every one of them waits for ALL outstanding
// vector-memory operations instead (vmcnt(0)): slower, but free of any assumption about how many
// younger operations are in flight.  A result that differs between the two builds points at a
// miscounted wait; one that does not, at something else.
#ifdef LASP2_FULL_WAITS
#define LASP2_WAIT_COUNT(n) 0
#else
#define LASP2_WAIT_COUNT(n) (n)
#endif

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LASP2_WAIT_COUNT(N)) : "memory");
}

// Global loads whose completion the kernel tracks itself.  The compiler knows nothing of them, so
// it neither counts them nor waits for them: the destination registers hold the data only
// after the matching wait_vmcnt_token().  That wait returns a zero the compiler cannot see
// through; every expression that reads the loaded registers must also depend on this value,
// which keeps all such reads behind the wait.
template <int OFF>
__device__ __forceinline__ void gload16_async(u32x4& dst, const char* p)
{
    asm volatile("global_load_dwordx4 %0, %1, off offset:%2" : "=&v"(dst) : "v"(p), "n"(OFF) : "memory");
}

template <int N>
__device__ __forceinline__ uint32_t wait_vmcnt_token()
{
    uint32_t zero;
    asm volatile("s_waitcnt vmcnt(%1)\n\tv_mov_b32 %0, 0" : "=v"(zero) : "n"(LASP2_WAIT_COUNT(N)) : "memory");
    return zero;
}

#define SCHED_FENCE() __builtin_amdgcn_sched_barrier(0)

}  // namespace
}  // namespace lasp2
#endif  // LASP2_MFMA_TILE_H
