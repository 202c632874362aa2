/*
 * bsfa.h — C ABI of the MI355X (gfx950) Block-Sparse FlashAttention forward library, libbsfa.so.
 *
 * The library implements the prefill attention of the paper "Block Sparse Flash Attention"
 * (Section 4 and Algorithm 1): tiled exact attention in which, for every query tile i
 * (B_M rows) and key block j (B_N rows), the score tile S_ij = Q_i K_j^T / sqrt(d) (Eq. 5) is
 * computed exactly, its maximum s_max (Eq. 6) is compared with a calibrated threshold, and a
 * block with s_max < threshold is skipped: its V block is not loaded, no exponentials are
 * taken, no P.V product is formed and the running softmax statistics are left untouched
 * (Section 4.1).  Key blocks that touch the causal boundary bypass the gate (Section 4.1,
 * last paragraph).  Equality keeps the block (Section 4.1 states the skip condition as a
 * strict inequality).
 *
 * Sequence lengths.  M_Q = ceil(seqlen / block_m) query tiles and M_KV = ceil(seqlen / block_n)
 * key blocks.  With causal != 0 seqlen need not fill its last tile or block: the sequence then
 * behaves as if padded by repeating its last token (Section 4.3).  Because of the causal mask that
 * amounts to ignoring the rows and columns that do not exist; the library never reads or writes
 * a token index >= seqlen.  With causal == 0 seqlen must be a multiple of block_m and block_n.
 *
 * Conventions
 *  - Every data pointer is a DEVICE pointer unless its comment says HOST.  The caller owns all
 *    buffers; the library keeps no device memory between calls.
 *  - Tensors are addressed through element strides; the head dimension is contiguous
 *    (stride 1).  Strides must be multiples of 8 elements and base pointers 16-byte aligned.
 *    [B, N, H, d] and [B, H, N, d] are both expressible.
 *  - Query head h reads KV head h / (n_q_heads / n_kv_heads).
 *  - bsfa_forward only enqueues work on `hip_stream` (a hipStream_t passed as void*; NULL is
 *    the default stream) and returns.  bsfa_calibrate synchronises that stream before it
 *    returns because it writes host memory.
 *  - On a validation error nothing is launched and no output is touched.  Functions return a
 *    bsfa_status; bsfa_last_error() gives a thread-local message for the last failure.
 *  - A NaN threshold gives undefined gate decisions (it is not detected).
 */
#ifndef BSFA_H
#define BSFA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    BSFA_OK = 0,
    BSFA_ERR_NULL = -1,        /* a required pointer is NULL                              */
    BSFA_ERR_SHAPE = -2,       /* sizes inconsistent, not tile aligned, bad stride/align  */
    BSFA_ERR_DTYPE = -3,       /* element type not supported                              */
    BSFA_ERR_UNSUPPORTED = -4, /* head_dim / tile shape the library was not built for     */
    BSFA_ERR_WORKSPACE = -5,   /* workspace missing or too small                          */
    BSFA_ERR_HIP = -6          /* a HIP runtime call failed (message in bsfa_last_error)  */
} bsfa_status;

/* Element type of q, k, v and out.  Scores, the gate comparison, the running statistics and both
 * accumulators are fp32 in either case; the probabilities are rounded to the element type for the
 * second product.  fp16 is the precision of the paper's own kernel (Section 5.1). */
typedef enum { BSFA_BF16 = 0, BSFA_FP16 = 1 } bsfa_dtype;

/* Problem descriptor (paper notation, Section 2.2: N tokens, head dim d, query tiles of B_M
 * rows, key/value blocks of B_N rows).  Zero-initialise it: a zero in an optional member selects
 * its default. */
typedef struct {
    int32_t batch, n_q_heads, n_kv_heads, seqlen, head_dim;
    int32_t block_m, block_n;     /* gate tile; see bsfa_query_build for the supported shapes */
    int64_t q_stride_b, q_stride_n, q_stride_h;   /* element strides: batch, token, head */
    int64_t k_stride_b, k_stride_n, k_stride_h;
    int64_t v_stride_b, v_stride_n, v_stride_h;
    int64_t o_stride_b, o_stride_n, o_stride_h;
    int32_t dtype;                /* bsfa_dtype */
    int32_t thresholds_per_tile;  /* 0: thresholds[n_q_heads] (one per head);
                                     1: thresholds[n_q_heads][threshold_tiles], the paper's
                                        T_{l,h,i} for one layer and one sparsity level
                                        (Section 4.2) */
    int32_t threshold_tiles;      /* optional, thresholds_per_tile = 1 only: number of query tiles
                                     the thresholds were calibrated for (row length of the array);
                                     0 = M_Q.  Query tiles at and beyond it use the last
                                     calibrated tile's threshold, the rule of Section 4.3 for
                                     sequences longer than the calibration length. */
    const int32_t *seqlens;       /* optional, DEVICE [batch], causal only: tokens of each batch
                                     element, clamped to [0, seqlen]; NULL = all have seqlen.
                                     Element b is handled as a sequence of seqlens[b] tokens stored
                                     at the start of its [seqlen] slot: rows of out and lse at and
                                     beyond seqlens[b] are left untouched, query tiles beyond it
                                     get NaN block maxima, an empty skip mask and add nothing to
                                     counts. */
    int32_t single_head_groups;   /* optional tuning knob, 0 by default: workgroups handle two query heads
                                     of a GQA group together when the group size is even (one K/V
                                     stream in LDS feeds both; fastest on the dense path, by ~2.5 %).
                                     1: one query head per workgroup — the heads' skip decisions no longer
                                     share a barrier, which measures ~1.5 % faster at 50 % skip and 4-7 %
                                     faster at 90 % skip (128K tokens).  Results are identical either way. */
    int32_t gate_mode;            /* optional, bsfa_forward only.  0: the paper's gate (block maximum against the
                                     threshold, Section 4.1).  1: the running-maximum predicate the paper
                                     describes for SpargeAttention's in-kernel filter (Section 3), provided for
                                     comparison inside the same kernel: with m_local the row maxima of the score
                                     tile and m_ij the running row maxima after the block (kept blocks only,
                                     ascending block order), a gateable block is skipped iff
                                     max over the tile's rows of (m_local - m_ij) < thresholds[h]; the
                                     thresholds then hold that lambda (natural score units, <= 0 to skip
                                     anything) instead of T, block_max holds the compared statistic, and the
                                     blocks that bypass the gate are the same.  Decisions now depend on the
                                     visiting order (ascending), unlike mode 0. */
    int32_t qk_fp8;               /* optional, 0 by default.  1: the score product Q K^T runs on fp8 (e4m3) copies of Q
                                     and K (rounded to nearest even, no scaling: |values| must stay below 448) with
                                     the 32x32x64 fp8 MFMA, fp32 accumulate; block maxima, the gate comparison, the
                                     softmax and the P V product are unchanged (fp32 / 16-bit).  The paper calls
                                     quantisation orthogonal to its gate (Section 5.1, Baselines); this is that
                                     combination.  Needs head_dim 128, block_m 128 and the workspace (bsfa_forward)
                                     resp. the larger calibration workspace; thresholds should be calibrated with
                                     the same setting, since block maxima of fp8-rounded operands differ from the
                                     16-bit ones by a few hundredths. */
    void   *workspace;            /* optional, DEVICE, 256-byte aligned, bsfa_forward only: scratch memory of at
                                     least bsfa_forward_workspace_bytes() bytes, overwritten by every call.
                                     With it (and block_m = 128) the forward pass first rewrites V, once, as
                                     transposed 64-key tiles (an O(N) pass: 2 x the size of V in traffic) so
                                     that the second matrix product reads its V operand from on-chip memory
                                     with full-width reads; the per-(tile, block) V loads stay conditional on
                                     the gate.  NULL: V is read in place.  Results are identical either way. */
    int64_t workspace_bytes;      /* size of workspace in bytes */
} bsfa_problem;

/* Optional outputs of bsfa_forward; any member may be NULL.  All DEVICE, caller allocated.
 * A key block is "reachable" for query tile i if causal masking leaves it any entry,
 * "gateable" if it leaves it every entry (these are the blocks the gate applies to). */
typedef struct {
    uint64_t *counts;     /* [batch][n_q_heads][3] = tiles skipped, gateable, reachable; the
                             measured density of Section 5.1 (Metrics) is 1 - skipped/reachable.
                             Overwritten (not accumulated). */
    uint32_t *skip_mask;  /* [batch][n_q_heads][M_Q][ceil(M_KV/32)], bit (j%32) of word j/32
                             set iff block j was skipped for query tile i */
    float    *block_max;  /* [batch][n_q_heads][M_Q][M_KV]: s_max (Eq. 6, natural score units,
                             1/sqrt(d) included) of gateable blocks, NaN elsewhere.  A diagnostic: asking
                             for it makes every key block take the kernel's general stages, which exchange
                             the maxima themselves instead of the waves' keep flags (a few per cent slower);
                             counts, skip_mask and lse cost nothing measurable. */
    float    *lse;        /* [batch][seqlen][n_q_heads]: L = m + log(l) over the kept blocks, natural
                             units (last line of Algorithm 1; what a backward pass or a merge of
                             partial results over key ranges needs) */
} bsfa_skip_stats;

/*
 * Forward pass (Algorithm 1 for every batch, head and query tile).
 *   q [batch, seqlen, n_q_heads, d], k and v [batch, seqlen, n_kv_heads, d], out like q, all
 *   through the strides in *p; thresholds: DEVICE fp32, natural score units.  -INFINITY
 *   disables the gate (dense attention, same code path); +INFINITY keeps only the blocks that
 *   bypass the gate.  causal != 0: causal mask; causal == 0: no mask, and the key blocks that
 *   overlap the query tile's own token range bypass the gate (the paper only says the method
 *   extends to the bidirectional case, Section 4.3; this keeps its "local blocks are always
 *   processed" rule).
 * Returns BSFA_OK after enqueueing; errors as listed above.
 */
bsfa_status bsfa_forward(const bsfa_problem *p, const void *q, const void *k, const void *v,
                         const float *thresholds, int causal, void *out,
                         const bsfa_skip_stats *skip_stats /* may be NULL */, void *hip_stream);

/* Bytes of workspace bsfa_forward can use for *p (size of V rounded up to whole 64-key blocks, plus
 * half as much for the fp8 copy of K if p->qk_fp8, plus alignment slack); 0 if *p is invalid or its
 * tile shape makes no use of a workspace. */
size_t bsfa_forward_workspace_bytes(const bsfa_problem *p);

/*
 * Calibration of per-head thresholds (Section 4.2 reduced over query positions): runs the
 * score / block-maximum half of the forward pass (Eq. 5-6) on a calibration batch and, for
 * each query head and each target skip fraction f, returns the order statistic x_r,
 * r = floor(f * n), of the n block maxima of that head's gateable tiles sorted ascending
 * (-INFINITY if r == 0, +INFINITY if r == n).  With the keep rule s_max >= threshold exactly r
 * tiles of the calibration batch are skipped, absent ties.
 *   target_skip_fractions HOST [n_levels], each in [0, 1]; n_levels <= 64
 *   thresholds_out        HOST [n_levels][n_q_heads]
 *   workspace             DEVICE, at least bsfa_calibrate_workspace_bytes(p) bytes
 * p->thresholds_per_tile must be 0.  The selection runs on the GPU (exact order statistics by radix
 * passes over the block maxima); only the n_levels x n_q_heads results are copied to the host.
 * Synchronises hip_stream.
 */
bsfa_status bsfa_calibrate(const bsfa_problem *p, const void *q, const void *k, int causal,
                           const float *target_skip_fractions, int n_levels,
                           float *thresholds_out, void *workspace, size_t workspace_bytes,
                           void *hip_stream);

/*
 * bsfa_calibrate for callers that cannot allocate device memory (code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc): same thresholds as bsfa_calibrate, bit for bit,
 * but the block maxima and the selection histograms live in a scratch array built into the library
 * (about 21 MiB of device memory per GPU, held until the process ends), the results are written to
 * DEVICE memory, and the call only enqueues kernels on hip_stream: no allocation, no memset, no copy,
 * no host synchronisation.
 *   thresholds_out_device DEVICE [n_levels][n_q_heads], usable as bsfa_forward thresholds once the
 *                         stream has reached this point
 * Limits (BSFA_ERR_WORKSPACE beyond them): batch * n_q_heads * M_Q * M_KV block maxima must not exceed
 * bsfa_calibrate_noalloc_max_values() (4 Mi: e.g. 32 heads at 32K tokens with 128 x 64 tiles), and
 * n_q_heads <= 64.  All calls on one GPU share the one scratch array: calls that overlap in time on
 * the same GPU (different streams or threads) race and give undefined thresholds.
 */
bsfa_status bsfa_calibrate_noalloc(const bsfa_problem *p, const void *q, const void *k, int causal,
                                   const float *target_skip_fractions, int n_levels,
                                   float *thresholds_out_device, void *hip_stream);
size_t bsfa_calibrate_noalloc_max_values(void);

/*
 * Calibration of per-query-tile thresholds, the rule of Section 4.2 itself: for every query head
 * and query tile, the threshold that retains exactly the top-k gateable key blocks of a
 * calibration sample (the k-th largest block maximum; -INFINITY where the tile has at most k
 * gateable blocks, which keeps the min(k, A) of Section 5.1; +INFINITY for k = 0), averaged over
 * calibration samples.  Each batch element of q, k is one sample.  Calls chain over further
 * samples: samples_done is the number of samples already averaged into thresholds_out (0 for the
 * first call, which overwrites it).
 *   ks             HOST [n_levels], the sparsity levels (number of retained gateable blocks)
 *   thresholds_out HOST [n_levels][n_q_heads][M_Q]: one slice [n_q_heads][M_Q] per level, usable
 *                  as bsfa_forward thresholds with thresholds_per_tile = 1 (and, on a longer
 *                  sequence, with threshold_tiles = this M_Q)
 *   workspace      DEVICE, at least bsfa_calibrate_workspace_bytes(p) bytes
 * p->thresholds_per_tile and p->threshold_tiles are ignored; p->seqlens must be NULL (samples of
 * one call have one length); p->gate_mode and p->qk_fp8 must be 0 (BSFA_ERR_UNSUPPORTED otherwise).
 * Synchronises hip_stream.
 */
bsfa_status bsfa_calibrate_topk(const bsfa_problem *p, const void *q, const void *k, int causal,
                                const int32_t *ks, int n_levels, int samples_done,
                                float *thresholds_out, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/* Bytes of device workspace bsfa_calibrate and bsfa_calibrate_topk need for *p (0 if *p is
 * invalid). */
size_t bsfa_calibrate_workspace_bytes(const bsfa_problem *p);

/* Tile shapes and head dims this build supports: fills up to `cap` entries of each array with
 * (block_m, block_n, head_dim) triples and returns the number of supported triples. */
int bsfa_query_build(int32_t *block_m, int32_t *block_n, int32_t *head_dim, int cap);

/*
 * Measurement utility, not an operation of the paper: enqueues one kernel in which every wave of
 * `workgroups` workgroups (512 threads each: two waves per SIMD, the occupancy of bsfa_forward) issues
 * 16 * iters back-to-back 32x32x16 bf16 matrix instructions whose operand registers are filled from
 * `operands`, and nothing else.  Timed with events on hip_stream, bsfa_mfma_rate_probe_flops(workgroups,
 * iters) / time is the matrix rate the card sustains for those operand VALUES: the chip lowers its shader
 * clock under dense matrix load, and how far depends on how much the operand bits toggle, so this rate --
 * not the published peak, which assumes the nominal clock -- is what a kernel built on the same
 * instruction can approach.  bench.py reports it beside the roofline figures.
 *   operands DEVICE [4096] floats (converted to bf16 in the kernel)
 *   sink     DEVICE, at least bsfa_mfma_rate_probe_sink_bytes(workgroups) bytes; receives the
 *            accumulators' sums (only there so that the work is not optimised away)
 * Errors: BSFA_ERR_NULL, BSFA_ERR_SHAPE (workgroups outside [1, 2^20] or iters < 1), BSFA_ERR_WORKSPACE
 * (sink too small), BSFA_ERR_HIP.  Nothing is launched on an error.
 */
bsfa_status bsfa_mfma_rate_probe(const float *operands, float *sink, size_t sink_bytes, int workgroups, int iters,
                                 void *hip_stream);
size_t bsfa_mfma_rate_probe_sink_bytes(int workgroups);
double bsfa_mfma_rate_probe_flops(int workgroups, int iters);

const char *bsfa_status_string(bsfa_status s);
const char *bsfa_last_error(void); /* thread-local, valid until the next failing call */

#ifdef __cplusplus
}
#endif
#endif /* BSFA_H */
