// Host side of liblasp2: argument validation, slot arithmetic and kernel dispatch
// for the entry points declared in include/lasp2.h.  Every argument error is
// reported before the first HIP call, so the error paths run on a machine
// without a GPU.
#include "lasp2_common.h"

#include <limits.h>
#include <stdlib.h>

#include <algorithm>

namespace lasp2 {
namespace {

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bool supported_d(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }

// Validates the descriptor and fills the kernel geometry.  *empty is set when
// there is nothing to compute.
int make_geom(const lasp2_desc_t* desc, Geom* g, bool* empty)
{
    if (!desc) return LASP2_ERR_NULL;
    if (desc->dtype != LASP2_F32 && desc->dtype != LASP2_BF16) return LASP2_ERR_DTYPE;
    if (desc->B < 0 || desc->H < 0 || desc->N < 0) return LASP2_ERR_SHAPE;
    if (!supported_d(desc->d)) return LASP2_ERR_SHAPE;
    if (desc->C < 1 || desc->C > 512) return LASP2_ERR_SHAPE;
    if (desc->L < 0) return LASP2_ERR_SHAPE;
    int64_t L = desc->L == 0 ? desc->C : desc->L;
    if (L % desc->C != 0) return LASP2_ERR_SHAPE;
    int64_t G = (int64_t)desc->B * desc->H;
    if (G > 65535) return LASP2_ERR_SHAPE;  // grid.y carries the group index
    // every element offset must fit int64 with a wide margin
    if (G > 0 && (int64_t)desc->N > (INT64_MAX / 8) / (G * desc->d)) return LASP2_ERR_SHAPE;
    if (desc->n_seqs < 0) return LASP2_ERR_SEQLENS;

    int64_t T_s = 0;
    if (desc->n_seqs > 0) {
        if (!desc->cu_seqlens_host || !desc->cu_seqlens_dev) return LASP2_ERR_SEQLENS;
        if (desc->B != 1) return LASP2_ERR_SEQLENS;
        const int32_t* cu = desc->cu_seqlens_host;
        if (cu[0] != 0 || cu[desc->n_seqs] != desc->N) return LASP2_ERR_SEQLENS;
        for (int k = 0; k < desc->n_seqs; ++k) {
            if (cu[k + 1] <= cu[k]) return LASP2_ERR_SEQLENS;
            T_s += ((int64_t)(cu[k + 1] - cu[k]) + L - 1) / L;
        }
        if (reinterpret_cast<uintptr_t>(desc->cu_seqlens_dev) & 3u) return LASP2_ERR_ALIGN;
    } else {
        if (desc->cu_seqlens_host || desc->cu_seqlens_dev) return LASP2_ERR_SEQLENS;
        T_s = ((int64_t)desc->N + L - 1) / L;
    }
    if (T_s > INT32_MAX) return LASP2_ERR_SHAPE;
    if (G > 0 && T_s > (INT64_MAX / 8) / (G * desc->d * desc->d)) return LASP2_ERR_SHAPE;
    // one-dimensional grids carry up to three workgroups per (group, slot) pair
    if (G * T_s > (int64_t)(INT32_MAX / 4)) return LASP2_ERR_SHAPE;

    // decay: both pointers or neither; every factor in (0, 1]
    if ((desc->decay_host == nullptr) != (desc->decay_dev == nullptr)) return LASP2_ERR_DECAY;
    if (desc->decay_host) {
        for (int h = 0; h < desc->H; ++h) {
            const float lam = desc->decay_host[h];
            if (!(lam > 0.f && lam <= 1.f)) return LASP2_ERR_DECAY;
        }
        if (reinterpret_cast<uintptr_t>(desc->decay_dev) & 3u) return LASP2_ERR_ALIGN;
    }

    g->G = (int32_t)G;
    g->H = desc->H > 0 ? desc->H : 1;
    g->decay = desc->decay_dev;
    // The MFMA decay kernels weight rows by lam^(0..63) in bf16 and undo it with lam^-(0..63)
    // in fp32; 0.35^63 = 2e-29 keeps both far from the ends of the exponent range.
    g->decay_mfma = 0;
    if (desc->decay_host) {
        g->decay_mfma = 1;
        for (int h = 0; h < desc->H; ++h)
            if (desc->decay_host[h] < 0.35f) g->decay_mfma = 0;
    }
    g->N = desc->N;
    g->q0 = 0;
    g->qn = desc->N;
    g->d = desc->d;
    g->C = desc->C;
    g->L = L;
    g->T_s = (int32_t)T_s;
    g->n_seqs = desc->n_seqs;
    g->lone_slots = (T_s == (desc->n_seqs > 0 ? (int64_t)desc->n_seqs : (int64_t)1)) ? 1 : 0;
    g->cu = desc->cu_seqlens_dev;
    // marks for slot_range: the number of slots before every doc_stride-th document
    g->wslots = 1;
    g->P_Ts = g->T_s;
    g->doc_stride = 1;
    for (int j = 0; j < kDocMarks; ++j) g->doc_mark[j] = j == 0 ? 0 : INT32_MAX;
    if (desc->n_seqs > 0) {
        const int32_t* cu = desc->cu_seqlens_host;
        g->doc_stride = (desc->n_seqs + kDocMarks - 1) / kDocMarks;
        int64_t before = 0;
        for (int k = 0; k < desc->n_seqs; ++k) {
            if (k % g->doc_stride == 0) g->doc_mark[k / g->doc_stride] = (int32_t)before;
            before += ((int64_t)(cu[k + 1] - cu[k]) + L - 1) / L;
        }
    }
    for (int j = 0; j < kDocMarks; ++j) g->doc_pmark[j] = g->doc_mark[j];
    *empty = (G == 0 || desc->N == 0);
    return LASP2_OK;
}

// ---- walks of several slots ---------------------------------------------------------------
// The state a fused pass carries across a slot boundary IS the next slot's prefix (up to the
// rounding order), so a workgroup may walk `ws` consecutive slots of a document and read the
// caller's state array only at the first.  The slot length the caller chose then no longer fixes
// how many workgroups a launch has nor how much of their time goes into starting up: one state
// per chunk (the paper's layout) still runs with walks as long as the device can keep busy.

constexpr int64_t kMaxWalkTokens = (int64_t)1 << 30;

// The geometry of the walks: g with L and T_s (and the document marks) for ws slots per walk;
// the caller's arrays stay described by P_Ts, wslots and doc_pmark.
Geom regroup(const Geom& g, const int32_t* cu_host, int ws)
{
    if (ws <= 1) return g;
    Geom w = g;
    w.wslots = ws;
    w.P_Ts = g.T_s;
    w.L = g.L * ws;
    if (g.n_seqs == 0) {
        w.T_s = (int32_t)(((int64_t)g.N + w.L - 1) / w.L);
        w.lone_slots = w.T_s == 1 ? 1 : 0;
        return w;
    }
    int64_t walks = 0, slots = 0;
    for (int j = 0; j < kDocMarks; ++j) w.doc_mark[j] = w.doc_pmark[j] = j == 0 ? 0 : INT32_MAX;
    for (int k = 0; k < g.n_seqs; ++k) {
        if (k % g.doc_stride == 0) {
            w.doc_mark[k / g.doc_stride] = (int32_t)walks;
            w.doc_pmark[k / g.doc_stride] = (int32_t)slots;
        }
        const int64_t len = cu_host[k + 1] - cu_host[k];
        walks += (len + w.L - 1) / w.L;
        slots += (len + g.L - 1) / g.L;
    }
    w.T_s = (int32_t)walks;
    w.lone_slots = walks == g.n_seqs ? 1 : 0;
    return w;
}

// Slots per walk for a launch that runs `par` walks at a time and gains little from walks longer
// than `target` tokens (measured: the forward launch is flat from about 2 048 tokens on, the
// backward from about 4 096; starting a walk costs what streaming about a hundred tokens does).
//   - Equal sequences, enough of them to fill the device by themselves: one walk per sequence,
//     which needs no prefix or suffix state at all (the serial-carry order of work).
//   - Otherwise the shortest walk of at least `target` tokens (a power of two of slots), made
//     shorter again while the launch would have fewer than two rounds of workgroups: a launch of
//     one round ends at the pace of its slowest CU, and less than one leaves CUs without work.
// The environment variable LASP2_WALK_SLOTS, when set to a positive number, overrides the choice
// (for tests and tuning).
int pick_walk_slots(const Geom& g, const int32_t* cu_host, int par, int64_t target)
{
    const int64_t longest_seq = [&] {
        if (g.n_seqs == 0) return (int64_t)g.N;
        int64_t m = 0;
        for (int k = 0; k < g.n_seqs; ++k) m = std::max<int64_t>(m, cu_host[k + 1] - cu_host[k]);
        return m;
    }();
    if (g.L >= longest_seq || g.G == 0) return 1;
    const int64_t ws_max = std::max<int64_t>(1, std::min<int64_t>(kMaxWalkTokens / g.L, INT32_MAX / 2));
    if (const char* e = getenv("LASP2_WALK_SLOTS")) {
        const long v = strtol(e, nullptr, 10);
        if (v >= 1) return (int)std::min<int64_t>(v, ws_max);
    }
    if (par < 1) par = 1;
    const int64_t ws_whole = (longest_seq + g.L - 1) / g.L;   // slots of the longest sequence
    if (g.n_seqs == 0 && ws_whole <= ws_max) {
        const int64_t rounds = ((int64_t)g.G + par - 1) / par;
        if ((int64_t)g.G * 100 >= rounds * par * 85) return (int)ws_whole;
    }
    auto units = [&](int64_t ws) {
        const int64_t W = g.L * ws;
        if (g.n_seqs == 0) return (int64_t)g.G * ((g.N + W - 1) / W);
        int64_t nw = 0;
        for (int k = 0; k < g.n_seqs; ++k) nw += ((int64_t)(cu_host[k + 1] - cu_host[k]) + W - 1) / W;
        return (int64_t)g.G * nw;
    };
    int64_t ws = 1;
    while (ws * g.L < target && ws * 2 <= ws_max && ws < ws_whole) ws *= 2;
    while (ws > 1 && units(ws) < 2 * (int64_t)par) ws /= 2;
    return (int)ws;
}

// (backward, equal sequences: two rounds of 16 384-token walks beat eight of 4 096 by 2 % at config 3 -
// the states kernel writes fewer states; ragged documents do best at 4 096)
constexpr int64_t kWalkTargetFwd = 2048, kWalkTargetBwd = 16384, kWalkTargetBwdPacked = 4096;

int check_ptrs(std::initializer_list<const void*> ptrs)
{
    for (const void* p : ptrs)
        if (!p) return LASP2_ERR_NULL;
    for (const void* p : ptrs)
        if (!aligned16(p)) return LASP2_ERR_ALIGN;
    return LASP2_OK;
}

int from_hip(hipError_t e) { return e == hipSuccess ? LASP2_OK : LASP2_ERR_LAUNCH; }

// Layout of the backward's workspace: the fp32 state array [G][T_s][d][d], then one 32-bit
// counter per (group, slot) through which the workgroups that share a slot's reads keep in
// step (used by the matrix-core kernels only; always part of the size).
size_t states_bytes(const Geom& g) { return (size_t)g.G * (size_t)g.T_s * (size_t)g.d * (size_t)g.d * sizeof(float); }
size_t pace_bytes(const Geom& g) { return (((size_t)g.G * (size_t)g.T_s * sizeof(unsigned)) + 15u) & ~(size_t)15u; }

// anchor_start matters with decay only: states as the slot's first token sees them (backward)
hipError_t run_states(const Geom& g, int dtype, const void* K, const void* V, float* M,
                      int anchor_start, hipStream_t st)
{
    if (mfma_path_supported(g, dtype)) return launch_states_mfma(g, K, V, M, anchor_start, st);
    return launch_states_generic(g, dtype, K, V, M, anchor_start, st);
}

// What lasp2_attn_bwd and lasp2_attn_bwd_noalloc have in common: the checks that need no
// workspace, and the launches.
struct BwdPlan {
    Geom g;             // the caller's slots (argument checks, workspace size)
    Geom gw;            // the walks of the kernels (= g unless the matrix-core kernels take several slots per walk)
    bool empty;
    bool fast;          // matrix-core kernels
    bool inclusive;     // suffix states in the inclusive form
    bool lone;          // every document a single slot
    bool need_states;   // dM_t go through a state array of `need` bytes
    size_t need;
    bool lone_w;        // every document a single walk
    bool need_states_w;
};

// `workspace`: address of the caller's workspace pointer, or NULL for an entry point that has none.
int plan_attn_bwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V, const void* dO,
                  const float* P, void* dQ, void* dK, void* dV, void* const* workspace, BwdPlan* pl)
{
    pl->empty = false;
    int rc = make_geom(desc, &pl->g, &pl->empty);
    if (rc != LASP2_OK || pl->empty) return rc;
    const Geom& g = pl->g;
    pl->fast = mfma_path_supported(g, desc->dtype);
    // Which suffix states the kernels want: the plain kernels and the MFMA kernels with decay walk
    // each slot backwards from the EXCLUSIVE suffix; the MFMA kernels without decay walk forwards
    // from the INCLUSIVE suffix and subtract (see attn_mfma_kernel), which lets the three
    // problems of a slot share their reads.
    pl->inclusive = pl->fast && !g.decay;
    // Every document a single slot (serial-carry schedule): all exclusive prefixes and suffixes are
    // zero.  P is then not read (and may be NULL), kernels that start from the exclusive suffix need
    // neither states nor workspace, and the inclusive suffix of a lone slot is its own state, so
    // the combine is skipped.
    pl->lone = g.lone_slots != 0;
    pl->need_states = !pl->lone || pl->inclusive;
    pl->need = states_bytes(g) + pace_bytes(g);
    const bool ws = workspace && pl->need_states;
    if ((!pl->lone && !P) || (ws && !*workspace)) return LASP2_ERR_NULL;   // NULL before alignment, as everywhere
    rc = check_ptrs({Q, K, V, dO, dQ, dK, dV});
    if (rc != LASP2_OK) return rc;
    if ((!pl->lone && !aligned16(P)) || (ws && !aligned16(*workspace))) return LASP2_ERR_ALIGN;
    // The kernels' own walks.  The backward's dM states live in the workspace only, so they are
    // built per walk, not per slot of the caller: fewer of them, never more bytes than `need`.
    pl->gw = g;
    if (pl->fast) {
        const int wgs = g.decay ? 3 : 2;   // workgroups per walk in the attention launch
        pl->gw = regroup(g, desc->cu_seqlens_host, pick_walk_slots(g, desc->cu_seqlens_host, std::max(1, cu_count() / wgs), g.n_seqs ? kWalkTargetBwdPacked : kWalkTargetBwd));
    }
    pl->lone_w = pl->gw.lone_slots != 0;
    pl->need_states_w = !pl->lone_w || pl->inclusive;
    return LASP2_OK;
}

int run_attn_bwd(const BwdPlan& pl, int dtype, const void* Q, const void* K, const void* V, const void* dO,
                 const float* P, void* dQ, void* dK, void* dV, float* dR, hipStream_t st)
{
    const Geom& g = pl.gw;
    if (pl.lone_w) P = nullptr;
    hipError_t e = hipSuccess;
    if (pl.need_states_w) {
        // dM_t = Q_t^T dO_t per walk, then its suffix combine in place
        e = run_states(g, dtype, Q, dO, dR, 1, st);
        if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    }
    if (!pl.lone_w) {
        e = launch_state_prefix(g, dR, dR, 1, pl.inclusive ? 1 : 0, st);
        if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    }
    if (pl.fast) {
        unsigned* pace = dR ? reinterpret_cast<unsigned*>(reinterpret_cast<char*>(dR) + states_bytes(g)) : nullptr;
        return from_hip(launch_attn_bwd_mfma(g, Q, K, V, dO, P, pl.need_states_w ? dR : nullptr, pace, dQ, dK, dV, st));
    }
    // dQ: the forward problem with (dO, V, K) in the roles of (Q, K, V); its state is
    // V^T K = (K^T V)^T, i.e. the cached prefix read transposed.
    e = launch_attn_generic(g, dtype, dO, V, K, P, dQ, 1, 0, st);
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    // dV: anti-causal problem with (K, Q, dO); state dM_{t+1:T} = sum Q^T dO.
    e = launch_attn_generic(g, dtype, K, Q, dO, dR, dV, 0, 1, st);
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    // dK: anti-causal problem with (V, dO, Q); state dO^T Q = dM^T.
    e = launch_attn_generic(g, dtype, V, dO, Q, dR, dK, 1, 1, st);
    return from_hip(e);
}

// Scratch of lasp2_attn_bwd_noalloc: device memory that belongs to the loaded library itself, one
// copy per GPU, held until the process ends.  In host code `scratch` is only a handle for the
// symbol, not a device address: the address is asked for once per device, with that device
// current, and kept; kernels and launchers only ever see that address.
static __device__ __align__(256) unsigned char scratch[LASP2_NOALLOC_SCRATCH_BYTES];

void* scratch_on_current_device()
{
    static std::atomic<void*> addr[kMaxDevices] = {};
    const int dev = current_device_index();
    if (dev < 0) return nullptr;
    void* p = addr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
    addr[dev].store(p, std::memory_order_release);   // the same value from whichever thread asks first
    return p;
}

}  // namespace
}  // namespace lasp2

using namespace lasp2;

extern "C" {

int lasp2_num_slots(const lasp2_desc_t* desc, int64_t* T_s)
{
    if (!T_s) return LASP2_ERR_NULL;
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    *T_s = g.T_s;
    return LASP2_OK;
}

int lasp2_walk_slots(const lasp2_desc_t* desc, int backward, int64_t* slots_per_walk)
{
    if (!slots_per_walk) return LASP2_ERR_NULL;
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    *slots_per_walk = 1;
    if (empty || !mfma_path_supported(g, desc->dtype)) return LASP2_OK;
    const int wgs = backward ? (g.decay ? 3 : 2) : 1;
    *slots_per_walk = pick_walk_slots(g, desc->cu_seqlens_host, std::max(1, cu_count() / wgs),
                                      backward ? (g.n_seqs ? kWalkTargetBwdPacked : kWalkTargetBwd) : kWalkTargetFwd);
    return LASP2_OK;
}

int lasp2_workspace_size(const lasp2_desc_t* desc, size_t* bytes)
{
    if (!bytes) return LASP2_ERR_NULL;
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    *bytes = states_bytes(g) + pace_bytes(g);
    return LASP2_OK;
}

int lasp2_chunk_states(const lasp2_desc_t* desc, const void* K, const void* V, float* M,
                       void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (empty) return LASP2_OK;
    rc = check_ptrs({K, V, M});
    if (rc != LASP2_OK) return rc;
    return from_hip(run_states(g, desc->dtype, K, V, M, 0, (hipStream_t)stream));
}

int lasp2_state_prefix(const lasp2_desc_t* desc, const float* M, float* P, int reverse,
                       void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (empty) return LASP2_OK;
    rc = check_ptrs({M, P});
    if (rc != LASP2_OK) return rc;
    return from_hip(launch_state_prefix(g, M, P, reverse ? 1 : 0, 0, (hipStream_t)stream));
}

int lasp2_attn_fwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                   const float* P, void* O, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (empty) return LASP2_OK;
    // Serial-carry schedule: when every document is one slot, each slot starts from a zero state
    // and P may be left out (NULL); the states and prefix calls are then not needed at all.
    rc = (P == nullptr && g.lone_slots) ? check_ptrs({Q, K, V, O}) : check_ptrs({Q, K, V, P, O});
    if (rc != LASP2_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (mfma_path_supported(g, desc->dtype)) {
        const Geom gw = regroup(g, desc->cu_seqlens_host, pick_walk_slots(g, desc->cu_seqlens_host, cu_count(), kWalkTargetFwd));
        return from_hip(launch_attn_fwd_mfma(gw, Q, K, V, gw.lone_slots ? nullptr : P, O, st));
    }
    return from_hip(launch_attn_generic(g, desc->dtype, Q, K, V, P, O, 0, 0, st));
}

int lasp2_attn_bwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                   const void* dO, const float* P, void* dQ, void* dK, void* dV,
                   void* workspace, size_t workspace_bytes, void* stream)
{
    BwdPlan pl;
    int rc = plan_attn_bwd(desc, Q, K, V, dO, P, dQ, dK, dV, &workspace, &pl);
    if (rc != LASP2_OK) return rc;
    if (pl.empty) return LASP2_OK;
    if (pl.need_states && workspace_bytes < pl.need) return LASP2_ERR_WORKSPACE;
    return run_attn_bwd(pl, desc->dtype, Q, K, V, dO, P, dQ, dK, dV,
                        pl.need_states ? static_cast<float*>(workspace) : nullptr, (hipStream_t)stream);
}

int lasp2_attn_bwd_noalloc(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                           const void* dO, const float* P, void* dQ, void* dK, void* dV, void* stream)
{
    BwdPlan pl;
    int rc = plan_attn_bwd(desc, Q, K, V, dO, P, dQ, dK, dV, nullptr, &pl);
    if (rc != LASP2_OK) return rc;
    if (pl.empty) return LASP2_OK;
    float* dR = nullptr;
    if (pl.need_states) {
        if (pl.need > (size_t)LASP2_NOALLOC_SCRATCH_BYTES) return LASP2_ERR_WORKSPACE;
        dR = static_cast<float*>(scratch_on_current_device());
        if (!dR) return LASP2_ERR_LAUNCH;
    }
    // Nothing in the array has to start at zero: the states kernel writes every slot's state
    // before the combine and the attention kernels read any of it.
    return run_attn_bwd(pl, desc->dtype, Q, K, V, dO, P, dQ, dK, dV, dR, (hipStream_t)stream);
}

int lasp2_state_total(const lasp2_desc_t* desc, const float* M, float* S, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (g.decay) return LASP2_ERR_DECAY;   // decay is defined for the masked path only
    if (empty) return LASP2_OK;
    rc = check_ptrs({M, S});
    if (rc != LASP2_OK) return rc;
    return from_hip(launch_state_total(g, M, S, (hipStream_t)stream));
}

int lasp2_nomask_fwd(const lasp2_desc_t* desc, const void* Q, const float* S, void* O, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (g.decay) return LASP2_ERR_DECAY;   // decay is defined for the masked path only
    if (empty) return LASP2_OK;
    rc = check_ptrs({Q, S, O});
    if (rc != LASP2_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (mfma_path_supported(g, desc->dtype)) {
        const RowsStateProblem p = {Q, S, O, 0};
        return from_hip(launch_rows_state_mfma(g, &p, 1, st));
    }
    return from_hip(launch_rows_state_generic(g, desc->dtype, Q, S, O, 0, st));
}

int lasp2_nomask_bwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                     const void* dO, const float* S, void* dQ, void* dK, void* dV,
                     void* workspace, size_t workspace_bytes, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = make_geom(desc, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (g.decay) return LASP2_ERR_DECAY;   // decay is defined for the masked path only
    if (empty) return LASP2_OK;
    rc = check_ptrs({Q, K, V, dO, S, dQ, dK, dV, workspace});
    if (rc != LASP2_OK) return rc;
    if (workspace_bytes < states_bytes(g) + pace_bytes(g)) return LASP2_ERR_WORKSPACE;   // one size for both backward calls

    hipStream_t st = (hipStream_t)stream;
    float* dS = static_cast<float*>(workspace);
    // dM_t = Q_t^T dO_t per slot, then the sum over the document's slots in place
    hipError_t e = run_states(g, desc->dtype, Q, dO, dS, 0, st);
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    e = launch_state_total(g, dS, dS, st);
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    if (mfma_path_supported(g, desc->dtype)) {
        const RowsStateProblem p[3] = {{dO, S, dQ, 1}, {V, dS, dK, 1}, {K, dS, dV, 0}};
        return from_hip(launch_rows_state_mfma(g, p, 3, st));
    }
    e = launch_rows_state_generic(g, desc->dtype, dO, S, dQ, 1, st);    // dQ = dO M^T
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    e = launch_rows_state_generic(g, desc->dtype, V, dS, dK, 1, st);    // dK = V dM^T
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    return from_hip(launch_rows_state_generic(g, desc->dtype, K, dS, dV, 0, st));   // dV = K dM
}

// Softmax attention for the queries [q_begin, q_begin + q_len) of the sequence; the entry points
// without a range are the whole sequence.
static int softmax_geom(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len, Geom* g, bool* empty)
{
    int rc = make_geom(desc, g, empty);
    if (rc != LASP2_OK) return rc;
    if (g->decay) return LASP2_ERR_DECAY;   // decay belongs to the linear layers
    if (q_begin < 0 || q_len < 0 || q_begin + q_len > (int64_t)g->N) return LASP2_ERR_SHAPE;
    g->q0 = (int32_t)q_begin;
    g->qn = (int32_t)q_len;
    return LASP2_OK;
}

static int softmax_fwd_impl(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len, const void* Q,
                            const void* K, const void* V, void* O, float* LSE, int causal, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = softmax_geom(desc, q_begin, q_len, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (empty || g.qn == 0) return LASP2_OK;
    rc = check_ptrs({Q, K, V, O, LSE});
    if (rc != LASP2_OK) return rc;
    hipStream_t st = (hipStream_t)stream;
    if (softmax_mfma_supported(g, desc->dtype))
        return from_hip(launch_softmax_fwd_mfma(g, Q, K, V, O, LSE, causal ? 1 : 0, st));
    return from_hip(launch_softmax_fwd_generic(g, desc->dtype, Q, K, V, O, LSE, causal ? 1 : 0, st));
}

static int softmax_bwd_impl(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len, const void* Q,
                            const void* K, const void* V, const void* O, const void* dO, const float* LSE,
                            void* dQ, void* dK, void* dV, void* workspace, size_t workspace_bytes,
                            int causal, void* stream)
{
    Geom g;
    bool empty = false;
    int rc = softmax_geom(desc, q_begin, q_len, &g, &empty);
    if (rc != LASP2_OK) return rc;
    if (empty) return LASP2_OK;
    // with no queries dK and dV are still written (zeros); the query-side arrays are not touched
    rc = g.qn == 0 ? check_ptrs({K, V, dK, dV}) : check_ptrs({Q, K, V, O, dO, LSE, dQ, dK, dV, workspace});
    if (rc != LASP2_OK) return rc;
    const size_t rows = (size_t)g.G * (size_t)g.qn;
    if (workspace_bytes < 2 * rows * sizeof(float)) return LASP2_ERR_WORKSPACE;
    hipStream_t st = (hipStream_t)stream;
    float* delta = static_cast<float*>(workspace);
    float* lse2 = delta + rows;
    const bool fast = softmax_mfma_supported(g, desc->dtype);
    hipError_t e = launch_softmax_delta(g, desc->dtype, O, dO, LSE, delta, fast ? lse2 : nullptr, st);
    if (e != hipSuccess) return LASP2_ERR_LAUNCH;
    if (fast) {
        e = launch_softmax_bwd_dq_mfma(g, Q, K, V, dO, LSE, delta, dQ, causal ? 1 : 0, st);
        if (e != hipSuccess) return LASP2_ERR_LAUNCH;
        return from_hip(launch_softmax_bwd_dkv_mfma(g, Q, K, V, dO, lse2, delta, dK, dV, causal ? 1 : 0, st));
    }
    return from_hip(launch_softmax_bwd_generic(g, desc->dtype, Q, K, V, dO, LSE, delta, dQ, dK, dV,
                                               causal ? 1 : 0, st));
}

int lasp2_softmax_fwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                      void* O, float* LSE, int causal, void* stream)
{
    return softmax_fwd_impl(desc, 0, desc ? desc->N : 0, Q, K, V, O, LSE, causal, stream);
}

int lasp2_softmax_workspace_size(const lasp2_desc_t* desc, size_t* bytes)
{
    return lasp2_softmax_share_workspace_size(desc, desc ? desc->N : 0, bytes);
}

int lasp2_softmax_bwd(const lasp2_desc_t* desc, const void* Q, const void* K, const void* V,
                      const void* O, const void* dO, const float* LSE, void* dQ, void* dK, void* dV,
                      void* workspace, size_t workspace_bytes, int causal, void* stream)
{
    return softmax_bwd_impl(desc, 0, desc ? desc->N : 0, Q, K, V, O, dO, LSE, dQ, dK, dV, workspace,
                            workspace_bytes, causal, stream);
}

int lasp2_softmax_fwd_share(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len, const void* Q_t,
                            const void* K, const void* V, void* O_t, float* LSE_t, int causal, void* stream)
{
    return softmax_fwd_impl(desc, q_begin, q_len, Q_t, K, V, O_t, LSE_t, causal, stream);
}

int lasp2_softmax_share_workspace_size(const lasp2_desc_t* desc, int64_t q_len, size_t* bytes)
{
    if (!bytes) return LASP2_ERR_NULL;
    Geom g;
    bool empty = false;
    int rc = softmax_geom(desc, 0, q_len, &g, &empty);
    if (rc != LASP2_OK) return rc;
    *bytes = 2 * (size_t)g.G * (size_t)g.qn * sizeof(float);   // delta, and the log-sum-exp in base 2
    return LASP2_OK;
}

int lasp2_softmax_bwd_share(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len, const void* Q_t,
                            const void* K, const void* V, const void* O_t, const void* dO_t,
                            const float* LSE_t, void* dQ_t, void* dK, void* dV, void* workspace,
                            size_t workspace_bytes, int causal, void* stream)
{
    return softmax_bwd_impl(desc, q_begin, q_len, Q_t, K, V, O_t, dO_t, LSE_t, dQ_t, dK, dV, workspace,
                            workspace_bytes, causal, stream);
}

const char* lasp2_status_string(int status)
{
    switch (status) {
        case LASP2_OK: return "ok";
        case LASP2_ERR_NULL: return "a required pointer is NULL";
        case LASP2_ERR_SHAPE: return "unsupported or inconsistent shape (B,H,N,d,C,L)";
        case LASP2_ERR_DTYPE: return "unsupported dtype";
        case LASP2_ERR_SEQLENS: return "invalid packed-sequence offsets";
        case LASP2_ERR_WORKSPACE: return "workspace too small";
        case LASP2_ERR_ALIGN: return "device pointer not 16-byte aligned";
        case LASP2_ERR_LAUNCH: return "HIP launch failed";
        case LASP2_ERR_DECAY: return "invalid decay factors, or decay given to an entry point without masking";
        default: return "unknown status";
    }
}

}  // extern "C"
