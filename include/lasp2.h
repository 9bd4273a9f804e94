/*
 * lasp2.h - C ABI of the single-GPU hot path of LASP-2 with masking:
 * chunked causal (unnormalised, identity-kernel) linear attention, forward and
 * backward, for AMD MI355X (gfx950); and, at the end, of LASP-2 without
 * masking.
 *
 * Problem statement (LASP-2 paper, Sec. "Preliminary", Eq. (3); Sec. "LASP-2
 * with Masking", Algorithm "LASP-2 w/ Masking"; appendix Algorithm "LASP-2 w/
 * Masking (Backward Pass)"): per (batch, head), Q, K, V in R^{N x d};
 *     o_s = sum_{i<=s} (q_s . k_i) v_i .
 * The sequence is cut into chunks; chunk t contributes a d x d memory state
 * M_t = K_t^T V_t.  The paper all-gathers the states of all devices; here all
 * of them sit in one HBM array [B,H,T_s,d,d] and an exclusive prefix combine
 * gives M_{1:t-1}.  The output of chunk t is
 *     O_t = [(Q_t K_t^T) (.) Psi] V_t + Q_t M_{1:t-1},   Psi_ij = [i >= j],
 * and the backward mirrors it with dM_t = Q_t^T dO_t and the reverse
 * (suffix) combine dM_{t+1:T}.
 *
 * Two granularities (the result depends on neither):
 *   C  chunk length: in the plain fp32 kernels the side of the masked quadratic
 *      block and the period at which the inter-chunk state operand is
 *      refreshed.  The matrix-core kernels (bf16, d = 128) tile a slot in
 *      blocks of their own (256 rows, masked products over 128-row halves;
 *      128 rows when no slot is longer) whatever C is: there C only fixes the
 *      slots through L;
 *   L  tokens per state slot, a multiple of C (0 means L = C, the paper-literal
 *      layout with one state per chunk).  One slot is what one sequence-
 *      parallel rank would own; its chunks are walked by one workgroup that
 *      carries the running state on chip.
 *   L >= the longest sequence (document) makes every sequence a single slot:
 *   the serial-carry schedule of LASP-1 on one device (Sec. "LASP-1 vs
 *   LASP-2"; appendix Algorithm "LASP-1 w/ Masking"), one pass that carries M
 *   from chunk to chunk with no state array at all.  Every prefix is then
 *   zero, lasp2_attn_fwd and lasp2_attn_bwd accept P = NULL, and
 *   lasp2_chunk_states / lasp2_state_prefix need not be called.
 *
 * Slots.  Unpacked input: every (b,h) row of N tokens has T_s = ceil(N/L)
 * slots, slot s = tokens [s*L, min(N,(s+1)*L)).  Packed input (B must be 1):
 * document k = tokens [cu[k], cu[k+1]) has ceil(len_k/L) slots of its own,
 * slots never span documents, and T_s is their total, in document order.
 * No state crosses a document boundary (paper appendix "Variable Length",
 * read as a block-diagonal causal mask).  Ragged last chunks/slots are fine.
 *
 * Scalar decay (optional; the Retention / Lightning Attention form of the
 * layers in the paper's Table 2, for which it prints no formulas).  With a
 * per-head factor lam in (0, 1] the mask entry Psi_ij = 1 becomes lam^(i-j):
 *     o_s = sum_{i<=s} lam^(s-i) (q_s . k_i) v_i ,
 * i.e. the recurrence M_s = lam M_{s-1} + k_s^T v_s, o_s = q_s M_s.  The steps
 * keep their shape with decayed weights: a slot's state is taken as its last
 * token sees it, M_t = sum_j lam^(end_t - j) k_j^T v_j; the combine carries
 * the slot lengths, P_t = lam^(n_{t-1}) P_{t-1} + M_{t-1}; the token at local
 * index a of a chunk reads the state before the chunk with weight lam^(a+1).
 * The backward mirrors this with states anchored at the slots' first tokens.
 * lam = 1 for every head computes the undecayed result (bit for bit on the
 * plain kernels; on the matrix cores within rounding, because the decayed
 * backward walks each slot in the opposite direction).  Decay is given by
 * the two `decay_*` pointers of the descriptor (both NULL: none).
 * Precision with decay on the matrix cores (bf16, d = 128, every factor
 * >= 0.35; a smaller factor sends the whole call to the plain fp32 kernels,
 * because lam^63 must stay inside the bf16 / fp32 exponent range): the rows
 * that enter a state product are weighted first and rounded to bf16 like every
 * matrix-core operand, so the states lasp2_chunk_states returns carry that
 * rounding (relative error 3e-4 .. 1e-3, against < 1e-6 without decay, where
 * the products of bf16 inputs are exact); O, dQ, dK, dV keep the bf16 bound.
 *
 * Conventions for every entry point
 *   - All tensor pointers are DEVICE pointers, 16-byte aligned, contiguous,
 *     d fastest: Q,K,V,O,dO,dQ,dK,dV are [B,H,N,d] in `dtype` (fp32 or bf16);
 *     states M,P and the workspace are fp32, [B,H,T_s,d,d] with M[a][b] =
 *     sum_tokens k[a]*v[b].
 *   - The caller owns every buffer.  The library allocates nothing and is
 *     re-entrant.  Between calls it keeps only per-device facts about the
 *     hardware (number of compute units; which kernels have had their LDS
 *     limit raised), never anything about a problem.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).
 *     Calls only enqueue work; outputs are valid once the stream has been
 *     synchronised.  The descriptor and `cu_seqlens_host` are read during the
 *     call and need not outlive it; `cu_seqlens_dev` is read by the kernels
 *     and must stay valid until they have run.
 *   - Return value: LASP2_OK or a negative lasp2_status_t.  Argument errors
 *     are detected on the host before anything is launched and never touch
 *     the device.  Nothing aborts or throws.
 *   - B, H or N equal to 0 is a valid empty problem: the call returns LASP2_OK
 *     and launches nothing (pointers are then not examined).
 *   - Supported: d in {16, 32, 64, 128}; 1 <= C <= 512; B*H <= 65535 (the
 *     plain kernels carry the group index in the grid's second dimension).
 *     The MFMA kernels cover bf16 with d = 128 for every C, with and without
 *     decay (with decay: every factor >= 0.35, see above); any other
 *     supported combination runs the plain fp32-FMA kernels.  There is no CPU
 *     fallback.
 */
#ifndef LASP2_H
#define LASP2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    LASP2_OK = 0,
    LASP2_ERR_NULL = -1,        /* a required pointer is NULL                           */
    LASP2_ERR_SHAPE = -2,       /* B,H,N < 0; d or C outside the supported set; L not a
                                   positive multiple of C; sizes overflow int64         */
    LASP2_ERR_DTYPE = -3,       /* dtype is neither LASP2_F32 nor LASP2_BF16            */
    LASP2_ERR_SEQLENS = -4,     /* packed: B != 1, cu[0] != 0, cu[n] != N, not strictly
                                   increasing, or only one of the two cu pointers given */
    LASP2_ERR_WORKSPACE = -5,   /* workspace smaller than lasp2_workspace_size()        */
    LASP2_ERR_ALIGN = -6,       /* a device pointer is not 16-byte aligned              */
    LASP2_ERR_LAUNCH = -7,      /* the HIP runtime reported an error at launch          */
    LASP2_ERR_DECAY = -8        /* only one of the two decay pointers given, a factor
                                   outside (0, 1], or decay passed to an entry point
                                   without masking                                      */
} lasp2_status_t;

typedef enum { LASP2_F32 = 0, LASP2_BF16 = 1 } lasp2_dtype_t;

typedef struct lasp2_desc {
    int32_t B, H, N, d;              /* tensor shape [B,H,N,d]                                   */
    int32_t C;                       /* chunk length                                             */
    int32_t L;                       /* tokens per state slot; 0 => C; else a multiple of C      */
    int32_t dtype;                   /* lasp2_dtype_t of the eight [B,H,N,d] tensors             */
    int32_t n_seqs;                  /* packed: number of documents (>= 1); 0 => not packed      */
    const int32_t* cu_seqlens_host;  /* HOST  ptr, n_seqs+1 offsets, cu[0]=0 < ... < cu[n]=N     */
    const int32_t* cu_seqlens_dev;   /* DEVICE ptr holding the same n_seqs+1 values              */
    const float* decay_host;         /* HOST  ptr, H per-head decay factors in (0, 1]; NULL => none */
    const float* decay_dev;          /* DEVICE ptr holding the same H values (NULL iff host is)  */
} lasp2_desc_t;

/* Number of state slots T_s per (b,h) for this descriptor (see "Slots" above). */
int lasp2_num_slots(const lasp2_desc_t* desc, int64_t* T_s);

/*
 * How many of the caller's slots one workgroup of the bf16, d = 128 attention
 * kernels walks in one go (`backward` = 0: lasp2_attn_fwd, else lasp2_attn_bwd),
 * 1 for every other path.  The state a fused pass carries across a slot
 * boundary is that slot's prefix M_{1:t-1} (the recurrence the prefix sum
 * itself follows), so a walk reads P only at its first slot and the slot length
 * fixes the granularity of the state arrays, not the number or length of the
 * workgroups' walks: the library picks the walk length that keeps the device's
 * CUs busy with the fewest starts (never across a document edge).  Results are
 * the same within the rounding order.  lasp2_attn_bwd builds its dM states per
 * walk.  The environment variable LASP2_WALK_SLOTS (a positive integer, read at
 * every call) overrides the choice; 1 gives one walk per slot.
 */
int lasp2_walk_slots(const lasp2_desc_t* desc, int backward, int64_t* slots_per_walk);

/* Bytes of device scratch lasp2_attn_bwd and lasp2_nomask_bwd need: room for one fp32 state
 * array [B,H,T_s,d,d] that holds dM_t and then, in place, its suffix combine (lasp2_attn_bwd
 * may build fewer states than that: one per walk, see lasp2_walk_slots), followed by one 32-bit
 * counter per (b,h,slot) with which the backward's workgroups that read the same tokens keep in
 * step (a matter of speed only: no result depends on a counter). */
int lasp2_workspace_size(const lasp2_desc_t* desc, size_t* bytes);

/*
 * Chunk states, Algorithm "LASP-2 w/ Masking" line "Compute M_t = K_t^T V_t",
 * one state per slot: M[b,h,s] = sum over the slot's tokens of k^T v (fp32).
 * With (Q, dO) in place of (K, V) it yields dM_t = Q_t^T dO_t of the backward.
 * In:  K, V [B,H,N,d] (device, `dtype`).   Out: M [B,H,T_s,d,d] fp32 (device).
 * With decay the sum carries the weights lam^(end of slot - token), the state
 * as the slot's last token sees it (the backward computes its own states,
 * anchored at the slots' first tokens, internally).
 */
int lasp2_chunk_states(const lasp2_desc_t* desc, const void* K, const void* V,
                       float* M, void* stream);

/*
 * Prefix combine that stands in for AllGather + PrefixSum (forward) and
 * AllGather + SuffixSum (backward): exclusive, restarted at document edges.
 *   reverse == 0:  P[s] = sum_{r<s, same doc} M[r]   (M_{1:t-1};  first = 0)
 *   reverse != 0:  P[s] = sum_{r>s, same doc} M[r]   (dM_{t+1:T}; last  = 0)
 * With decay: P[s] = lam^(n_r) P[r] + M[r] for the neighbouring slot r = s-1
 * (reverse: r = s+1) of n_r tokens; M is then expected anchored at slot ends
 * (reverse: at slot starts).
 * In: M [B,H,T_s,d,d] fp32.  Out: P same shape; P may alias M exactly
 * (in place); partial overlap is not allowed.
 */
int lasp2_state_prefix(const lasp2_desc_t* desc, const float* M, float* P,
                       int reverse, void* stream);

/*
 * Fused forward, Algorithm "LASP-2 w/ Masking" lines O_intra, O_inter, O_t:
 * for every chunk t of every slot, O_t = [(Q_t K_t^T)(.)Psi] V_t + Q_t M_{1:t-1},
 * where M_{1:t-1} = P[slot] + the states of the slot's earlier chunks (carried
 * on chip).  In: Q,K,V [B,H,N,d]; P [B,H,T_s,d,d] fp32 from lasp2_state_prefix
 * (reverse = 0).  Out: O [B,H,N,d] in `dtype`, written once.
 * Every entry of P must be valid, but not every entry is necessarily read
 * (see lasp2_walk_slots).
 * P may be NULL when every sequence (document) is a single slot: its prefix is
 * zero, the slot starts from a zero state (serial-carry schedule).  With more
 * than one slot in some sequence a NULL P is LASP2_ERR_NULL.
 */
int lasp2_attn_fwd(const lasp2_desc_t* desc, const void* Q, const void* K,
                   const void* V, const float* P, void* O, void* stream);

/*
 * Backward, Algorithm "LASP-2 w/ Masking (Backward Pass)":
 *   dM_t = Q_t^T dO_t, suffix combine dM_{t+1:T} (both into `workspace`), then
 *   dQ_t = [(dO_t V_t^T)(.)Psi] K_t   + dO_t M_{1:t-1}^T
 *   dK_t = [(dO_t V_t^T)(.)Psi]^T Q_t + V_t dM_{t+1:T}^T
 *   dV_t = [(Q_t K_t^T)(.)Psi]^T dO_t + K_t dM_{t+1:T}
 * In: Q,K,V,dO [B,H,N,d]; P = the forward's cached prefix array (the paper
 * keeps M_{1:t-1} in HBM for this purpose).  Out: dQ,dK,dV [B,H,N,d].
 * `workspace`: device scratch of at least lasp2_workspace_size() bytes,
 * 16-byte aligned; its contents on return are unspecified (suffix states in
 * the form the kernels that ran wanted them).
 * When every sequence (document) is a single slot, all prefixes and suffixes
 * are zero: P is not read and may be NULL, and the combine is skipped.  The
 * plain kernels and the decayed matrix-core kernels then need no workspace
 * either (NULL / 0 bytes accepted); the undecayed matrix-core kernels still
 * use it for the slots' own dM_t, from which their forward walk subtracts.
 */
int lasp2_attn_bwd(const lasp2_desc_t* desc, const void* Q, const void* K,
                   const void* V, const void* dO, const float* P,
                   void* dQ, void* dK, void* dV,
                   void* workspace, size_t workspace_bytes, void* stream);

/*
 * lasp2_attn_bwd for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and errors as lasp2_attn_bwd
 * without the workspace pair; dM_t and their suffix combine go through a fixed
 * array of LASP2_NOALLOC_SCRATCH_BYTES of device memory that is part of the
 * loaded library (one copy per GPU, held until the process ends).  The call
 * allocates and frees nothing; its first use on a device looks the array's
 * address up once.  LASP2_ERR_WORKSPACE if lasp2_workspace_size() exceeds
 * LASP2_NOALLOC_SCRATCH_BYTES (at d = 128 that is B*H*T_s > 1024 slot states,
 * 64 MiB of states and their counters; the limit does not apply where
 * lasp2_attn_bwd needs no workspace either).
 * All calls on one GPU share the array: two calls that overlap in time on the
 * same GPU (different streams or host threads) race and must be serialised by
 * the caller; calls on the same stream are ordered and safe.  Nothing in the
 * array needs clearing between calls (every state is written before it is
 * read), and its contents after a call are unspecified.
 */
#define LASP2_NOALLOC_SCRATCH_BYTES ((64u << 20) + (64u << 10))
int lasp2_attn_bwd_noalloc(const lasp2_desc_t* desc, const void* Q, const void* K,
                           const void* V, const void* dO, const float* P,
                           void* dQ, void* dK, void* dV, void* stream);

/*
 * ---- Without masking (LASP-2 paper, Sec. "LASP-2 without Masking", Algorithm
 * "LASP-2 w/o Masking" and appendix Algorithm "LASP-2 w/o Masking (Backward
 * Pass)") ----
 * Every token attends to every token of its sequence (document):
 *     O = (Q K^T) V = Q (K^T V),
 * so the states are summed instead of prefix-combined and each slot needs one
 * product with the total.  The slot states come from lasp2_chunk_states; C
 * plays no part here beyond fixing the slots through L.
 */

/*
 * Line "M_{1:T} = Sum([M_t])" of the algorithm, standing in for AllGather +
 * Sum: S[s] = sum of M[r] over all slots r of the document that owns slot s,
 * so that every slot holds its document's total (as every rank does after the
 * gather).  In: M [B,H,T_s,d,d] fp32.  Out: S, same shape; S may alias M
 * exactly (in place); partial overlap is not allowed.  The forward's S is the
 * array the paper caches in HBM for the backward.
 */
int lasp2_state_total(const lasp2_desc_t* desc, const float* M, float* S, void* stream);

/*
 * Line "O_t = Q_t M_{1:T}".  In: Q [B,H,N,d]; S [B,H,T_s,d,d] fp32 from
 * lasp2_state_total.  Out: O [B,H,N,d] in `dtype`, written once.
 */
int lasp2_nomask_fwd(const lasp2_desc_t* desc, const void* Q, const float* S, void* O,
                     void* stream);

/*
 * Backward without masking: dM_t = Q_t^T dO_t per slot and its total dM_{1:T}
 * (both into `workspace`; the range printed in the algorithm's Sum line is
 * read as the sum over all chunks), then
 *   dQ_t = dO_t M_{1:T}^T,   dK_t = V_t dM_{1:T}^T,   dV_t = K_t dM_{1:T}.
 * In: Q,K,V,dO [B,H,N,d]; S = the forward's cached totals.  Out: dQ,dK,dV
 * [B,H,N,d].  `workspace`: device scratch of at least lasp2_workspace_size()
 * bytes, 16-byte aligned; on return it holds dM_{1:T} in every slot.
 */
int lasp2_nomask_bwd(const lasp2_desc_t* desc, const void* Q, const void* K,
                     const void* V, const void* dO, const float* S,
                     void* dQ, void* dK, void* dV,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * ---- Standard (softmax) attention of the hybrid model (LASP-2H; Sec. "Hybrid
 * Model Sequence Parallelism", Algorithm "AllGather-based Context
 * Parallelism") ----
 * Line "O_t = Softmax(Q_t K^T / sqrt(d)) V" with K and V gathered, i.e. whole
 * in HBM here; every query block is what one rank computes.  Row-wise softmax
 * over the keys of the query's sequence (packed input: of its document, the
 * document-level mask the paper names as a reason for the gathered form);
 * causal != 0 additionally keeps keys j <= i only (the algorithm prints no
 * mask; Llama-style layers are causal).  C, L and the slots play no part.
 * In: Q,K,V [B,H,N,d].  Out: O [B,H,N,d] in `dtype`; LSE [B,H,N] fp32, the
 * natural-log sum of exp of each row's scaled scores (what a backward pass
 * needs to rebuild the probabilities).  Decay is rejected.  bf16 with d = 128
 * runs on the matrix cores, everything else on a plain fp32 kernel.
 */
int lasp2_softmax_fwd(const lasp2_desc_t* desc, const void* Q, const void* K,
                      const void* V, void* O, float* LSE, int causal, void* stream);

/* Bytes of device scratch lasp2_softmax_bwd needs (two fp32 per query row). */
int lasp2_softmax_workspace_size(const lasp2_desc_t* desc, size_t* bytes);

/*
 * Backward of lasp2_softmax_fwd (the paper prints the forward of the
 * standard-attention layers only; this is its gradient).  With P the row
 * softmax rebuilt from LSE, dP_ij = dO_i . v_j and delta_i = dO_i . O_i:
 *   dS = P (.) (dP - delta),  dQ = dS K / sqrt(d),  dK = dS^T Q / sqrt(d),
 *   dV = P^T dO.
 * In: Q,K,V,O,dO [B,H,N,d]; LSE [B,H,N] from the forward; same `causal`.
 * Out: dQ,dK,dV [B,H,N,d].  `workspace`: device scratch of at least
 * lasp2_softmax_workspace_size() bytes, 16-byte aligned (receives delta and
 * the log-sum-exp in base 2).
 * bf16 with d = 128 runs on the matrix cores (one kernel for dQ, one for dK
 * and dV), everything else on plain fp32 kernels.
 */
int lasp2_softmax_bwd(const lasp2_desc_t* desc, const void* Q, const void* K,
                      const void* V, const void* O, const void* dO, const float* LSE,
                      void* dQ, void* dK, void* dV,
                      void* workspace, size_t workspace_bytes, int causal, void* stream);

/*
 * One rank's share of the same layer (Algorithm "AllGather-based Context
 * Parallelism": rank t holds Q_t, gathers K and V, computes O_t): the queries
 * are the tokens [q_begin, q_begin + q_len) of the N-token sequence.
 * Q_t, O_t, dO_t, dQ_t are [B,H,q_len,d] and LSE_t is [B,H,q_len], row r being
 * token q_begin + r (masks use the token index); K, V, dK, dV are [B,H,N,d].
 * lasp2_softmax_bwd_share writes into dK, dV (all N rows, zeros where no query
 * of the share attends) this share's contribution only: the terms a
 * reduce-scatter over ranks would add up.  q_begin < 0, q_len < 0 or
 * q_begin + q_len > N gives LASP2_ERR_SHAPE; q_len = 0 is allowed.  The
 * workspace holds two fp32 per query row of the share.  Everything else is as
 * for lasp2_softmax_fwd / lasp2_softmax_bwd, which are the share
 * q_begin = 0, q_len = N.
 */
int lasp2_softmax_fwd_share(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len,
                            const void* Q_t, const void* K, const void* V, void* O_t,
                            float* LSE_t, int causal, void* stream);
int lasp2_softmax_share_workspace_size(const lasp2_desc_t* desc, int64_t q_len, size_t* bytes);
int lasp2_softmax_bwd_share(const lasp2_desc_t* desc, int64_t q_begin, int64_t q_len,
                            const void* Q_t, const void* K, const void* V, const void* O_t,
                            const void* dO_t, const float* LSE_t, void* dQ_t, void* dK, void* dV,
                            void* workspace, size_t workspace_bytes, int causal, void* stream);

/* Static, human-readable text for a status code (never NULL). */
const char* lasp2_status_string(int status);

#ifdef __cplusplus
}
#endif
#endif /* LASP2_H */
