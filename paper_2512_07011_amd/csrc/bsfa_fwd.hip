// Block-Sparse FlashAttention forward kernel for gfx950 (MI355X), wave64, bf16 or fp16 MFMA.
//
// One workgroup = one query tile Q_i (B_M = 32 * NWH rows, NWH waves of 32 rows) of HP query heads
// that share a KV head (GQA); it walks the reachable key blocks j in ascending order (Algorithm 1):
//   S_ij^T = K_j Q_i^T        32x32x16 MFMA, fp32 accumulate                      (Eq. 5)
//   s_max  = max S_ij         lane max -> wave max -> cross-wave max through LDS   (Eq. 6)
//   gate   : s_max / sqrt(d) >= T keeps the block; blocks touching the causal boundary bypass
//            the gate (Section 4.1).  One decision per (head, query tile, key block).
//   kept   : V_j is requested only after the decision (and only if some head of the group keeps
//            the block), exp2-based online softmax, O^T += V_j^T P^T.
// The transposed products keep everything of one query row inside one lane pair (l, l^32):
// the S^T accumulator layout (column = query) is already the B-operand layout of the second
// MFMA up to a permutation of the keys, and the same permutation is applied to V when its
// A operand is gathered from LDS with the transposing read, so P never leaves registers.
//
// Software pipeline, one barrier per key block.  The scores of block j+1 are computed while block
// j is finished, so the gate decision is known one block ahead:
//   stage j:  softmax(S_j) -> P_j          (VALU) interleaved with
//             S_{j+1} = K_{j+1} Q^T        (MFMA); per-lane maximum of S_{j+1}; the wave's keep flag
//             (or, in the general stages, its block maximum) -> LDS
//             wait for the copies needed next; barrier
//             O^T += V_j^T P_j^T           (MFMA), and between those MFMAs, a few instructions at a
//             time: decide keep_{j+1}; request V_{j+1} (only if kept) and K_{j+KR+1}; running
//             maximum of block j+1; first score operands of block j+2
// K tiles sit in a ring of KR LDS slots and are requested KR+1 blocks ahead, V tiles in two slots;
// both go HBM -> LDS directly, and the waits are partial (vmcnt) so that only the tile needed
// next has to have landed.  With a workspace V arrives pre-transposed (transpose_v_kernel) and its
// operand is a plain 16-byte LDS read; without one it is gathered with the transposing read.
#include "bsfa_dev.h"

namespace bsfa {

struct ScoreTile {
    f32x16 s[2];          // S^T: [32-key half], raw q.k (no 1/sqrt(d)); column = this lane's query
    float mx;             // row max of the lane's query, equal in lanes l and l^32
    bool keep;            // gate decision of this wave's head (uniform over the head's waves)
    bool any_keep;        // some head of the workgroup keeps the block (workgroup-uniform): V is fetched
    float m_use;          // kept blocks: row max the exponentials are taken against (log2 units)
    float alpha;          // kept blocks: factor that rescales the running accumulator and normaliser
    bool resc;            // kept blocks: alpha differs from 1 in some lane of the wave
};

template <int D, int NWH, int HP, int KR, bool CALIB, bool F16, bool VT, bool QK8>
__global__ void __launch_bounds__(NWH * HP * 64, 2) bsfa_fwd_kernel(const FwdParams p)
{
    typedef typename Elem<F16>::T el;                    // element type of Q, K, V, P, O
    typedef typename Elem<F16>::x8 bf16x8;               // (the vector names keep the default type's name)
    typedef typename Elem<F16>::x4 bf16x4;
    typedef typename Elem<F16>::x2 bf16x2;
    constexpr int NW = NWH * HP;
    constexpr int NT = NW * 64;
    constexpr int BM = NWH * 32;
    constexpr int BN = kBlockN;
    constexpr int KS = D / 16;       // MFMA k-steps over the head dim
    constexpr int DB = D / 32;       // 32-row blocks of O^T
    constexpr int CPR = D / 8;       // 16-byte chunks per tile row
    constexpr int NST = 64 * CPR / NT;                   // copy repetitions per 16-bit tile (V; K unless QK8)
    constexpr int NSTK = QK8 ? NST / 2 : NST;            // ... per K tile (fp8 tiles are half the bytes)
    static_assert(!QK8 || (D == 128 && NST >= 2), "fp8 score operands: head_dim 128, at most 512 threads");
    constexpr int TILE_BYTES = BN * D * 2;
    constexpr int ROW_BYTES = D * 2;
    constexpr int R = KR + 1;        // K tiles are requested R blocks ahead
    constexpr int VR = CALIB ? 0 : 2;
    static_assert(NST >= 1 && (R < 4 || NSTK * (R - 3) < 64), "copy repetitions");

    __shared__ __attribute__((aligned(1024))) unsigned char lds_raw[(KR + VR) * TILE_BYTES];
    __shared__ float lds_red[2][NW];
    // V slots first: their gather offsets then fit the 16-bit immediate of the LDS reads
    const uint32_t lds_v0 = (uint32_t)(uintptr_t)((__attribute__((address_space(3))) unsigned char *)lds_raw);
    const uint32_t lds_k0 = lds_v0 + VR * TILE_BYTES;

    int b, h0, i;
    if (!decode_work<HP>(p, blockIdx.x, b, h0, i)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int hsel = wave / NWH, wrow = wave % NWH;      // which head of the group, which 32-row slice
    const int h = h0 + hsel;
    const int l32 = lane & 31, hh = lane >> 5;
    const int g = h0 / p.group;
    const bool stat_lane = (wrow == 0 && lane == 0);     // one lane per head writes statistics

    const int64_t row0 = (int64_t)i * BM;                 // first query row of the tile
    // tokens of this batch element; a sequence that does not fill its last query tile or key
    // block behaves as if padded by repeating its last token (Section 4.3): loads of rows
    // beyond the end read row n_tok - 1 instead, padded rows are not stored, and key blocks made
    // of padding only are not visited (the causal mask hides them from every real row).
    int n_tok = p.seqlen;
    if (p.seqlens) n_tok = min(max(__builtin_amdgcn_readfirstlane(p.seqlens[b]), 0), p.seqlen);
    const int64_t stat_row = ((int64_t)b * p.hq + h) * p.mq + i;
    if (row0 >= n_tok) {                                  // the tile lies beyond the sequence: empty statistics
        const int htid = tid - hsel * NWH * 64;
        if (p.block_max)
            for (int jj = htid; jj < p.mkv; jj += NWH * 64) p.block_max[stat_row * p.mkv + jj] = NAN;
        if (p.skip_mask)
            for (int w = htid; w < p.mask_words; w += NWH * 64) p.skip_mask[stat_row * p.mask_words + w] = 0u;
        return;
    }
    const int mkv_tok = (n_tok + BN - 1) / BN;
    const int partial_blk = (n_tok % BN) ? n_tok / BN : -1;   // the block that padding completes, if any
    const int partial_rows = n_tok % BN;
    const int n_blk = p.causal ? min((int)((row0 + BM + BN - 1) / BN), mkv_tok) : mkv_tok;   // reachable blocks
    // causal: blocks [0, n_gate) are gateable, [n_gate, n_blk) touch the boundary.
    // non-causal: blocks [own_lo, own_hi) overlap the tile's own tokens and bypass the gate.
    const int n_gate = p.causal ? (int)((row0 + 1) / BN) : 0;
    const int own_lo = (int)(row0 / BN), own_hi = (int)((row0 + BM + BN - 1) / BN);

    const uint16_t *kbase = p.k + (int64_t)b * p.ksb + (int64_t)g * p.ksh;
    // VT: V comes from the workspace, one pre-transposed, pre-swizzled 64-key tile after the other
    const uint16_t *vbase = VT ? p.vt + ((int64_t)b * p.hkv + g) * p.mkv * (int64_t)(BN * D)
                               : p.v + (int64_t)b * p.vsb + (int64_t)g * p.vsh;
    float tau_h[HP];                                      // thresholds of the group's heads for this tile
#pragma unroll
    for (int x = 0; x < HP; ++x)     // tiles past the calibrated length use its last tile's threshold (Section 4.3)
        tau_h[x] = CALIB ? -INFINITY      // the score half takes no decisions
                         : p.tau[p.tau_per_tile ? (int64_t)(h0 + x) * p.tau_tiles + min(i, p.tau_tiles - 1) : (h0 + x)];

    const float tau_own = hsel ? tau_h[HP - 1] : tau_h[0];
    uint32_t koff[NSTK], voff[NST];
#pragma unroll
    for (int r = 0; r < NST; ++r) {
        if (r < NSTK) koff[r] = QK8 ? (uint32_t)(r * NT + tid) * 16u : chunk_src_offset<D, NT, false>(r, tid, (int)p.ksn);
        voff[r] = VT ? (uint32_t)(r * NT + tid) * 16u : chunk_src_offset<D, NT, true>(r, tid, (int)p.vsn);
    }
    // QK8: K comes from the workspace as fp8 tiles (64 rows of D bytes, swizzled for the operand reads)
    const uint8_t *k8base = QK8 ? p.k8 + ((int64_t)b * p.hkv + g) * p.mkv * (int64_t)(BN * D) : nullptr;
    const int64_t kstep = (int64_t)BN * p.ksn, vstep = VT ? (int64_t)(BN * D) : (int64_t)BN * p.vsn;
    // K_t, whose first row is at `src`, into the ring slot at LDS byte address dst
    auto copy_k_from = [&](const unsigned char *src, int t, uint32_t dst) {
        if constexpr (QK8) {
            tile_copy_async<NSTK, NT>(src, koff, dst, wave);                                  // (padded already)
        } else {
            if (t == partial_blk) tile_copy_async_clamped<D, NT, false>(reinterpret_cast<const uint16_t *>(src), (int)p.ksn, partial_rows, dst, wave);
            else tile_copy_async<NSTK, NT>(src, koff, dst, wave);
        }
    };
    // V_t, whose first row is at `src`, into slot t & 1
    auto copy_v_from = [&](const unsigned char *src, int t) {
        const uint32_t dst = lds_v0 + (uint32_t)(t & 1) * TILE_BYTES;
        if (!VT && t == partial_blk) tile_copy_async_clamped<D, NT, true>(reinterpret_cast<const uint16_t *>(src), (int)p.vsn, partial_rows, dst, wave);
        else tile_copy_async<NST, NT>(src, voff, dst, wave);                                  // (workspace tiles are padded already)
    };
    const unsigned char *const k_bytes = QK8 ? reinterpret_cast<const unsigned char *>(k8base) : reinterpret_cast<const unsigned char *>(kbase);
    const unsigned char *const v_bytes = reinterpret_cast<const unsigned char *>(vbase);
    const int64_t kstep_b = QK8 ? (int64_t)(BN * D) : kstep * 2, vstep_b = vstep * 2;      // bytes from one tile to the next
    auto copy_k = [&](int t, uint32_t dst) { copy_k_from(k_bytes + t * kstep_b, t, dst); };
    auto copy_v = [&](int t) { copy_v_from(v_bytes + t * vstep_b, t); };

    // Operand gather addresses (bytes inside a tile slot).
    // K (A operand of S^T): lane reads key row 32*kb + l32, chunk (2s + hh) ^ swz_k(row).  The row
    // swizzle does not depend on kb (32 is a multiple of its period) and 2s only occupies chunk
    // bits 1.., so  addr(s, kb) = (ka_base ^ (s << 5)) + kb * 32 * ROW_BYTES.
    // QK8: the tile holds fp8, 64 rows of 128 bytes, chunk index XOR-ed with (row >> 1) & 7; a lane
    // reads row 32*kb + l32, head-dim bytes 64s + 32hh .. +31 as two b128 (chunks 4s + 2hh + {0, 1}):
    // addr(s, kb, e) = (ka_base ^ (s << 6) ^ (e << 4)) + kb * 32 * 128.
    const uint32_t ka_base = QK8 ? (uint32_t)(l32 * 128 + (((2 * hh) ^ ((l32 >> 1) & 7)) << 4))
                                 : (uint32_t)(l32 * ROW_BYTES + ((hh ^ swz_k<D>(l32)) << 4));
    // V (A operand of O^T, transposing read of 4 keys x 16 head-dim columns per 16 lanes): lane
    // reads row 16u + 4hh + (L >> 2) (+8 for the second half), 8 bytes.  Which head-dim column an
    // operand row stands for is free (it only permutes the rows of O^T, undone at the final
    // store): at D = 128 operand rows 0-15 of block x are columns 16x .. 16x+15 and rows 16-31 are
    // columns 64+16x .., which puts the two 16-lane groups of a read into different bank halves;
    // at D = 64 rows 0-31 are columns 32x .. 32x+31.  The row swizzle has period 8 rows, so it does
    // not depend on u or the +8, and x occupies chunk bits the swizzle only XORs, so
    // addr(u, x, half) = (va_base ^ (x << XSH)) + (16u + 8*half) * ROW_BYTES.
    constexpr int G16_COLS = (D == 128) ? 64 : 16;       // column distance of the two 16-lane groups
    constexpr int X_COLS = (D == 128) ? 16 : 32;         // column step of x
    constexpr int XSH = (D == 128) ? 5 : 6;              // log2(X_COLS * 2 bytes)
    const int L = lane & 15, g16 = (lane >> 4) & 1;
    const int vrow = 4 * hh + (L >> 2);
    const int vcol = G16_COLS * g16 + 4 * (L & 3);
    // VT: the tile holds V^T, D rows of 64 keys (128 bytes), the keys of every 16-key step ordered
    // so that the 8 keys a lane multiplies are contiguous, the 16-byte chunk index XOR-ed with
    // (row >> 1) & 7.  Lane reads row 32x + l32, chunk 2u + hh, as one b128:
    // addr(u, x) = (va_base ^ (u << 5)) + x * 32 * 128 -- conflict-free (16 lanes hit 16 distinct
    // (row parity, chunk) slots), and at twice the LDS rate of the transposing reads.
    const uint32_t va_base = VT ? (uint32_t)(l32 * 128 + ((hh ^ ((l32 >> 1) & 7)) << 4))
                                : (uint32_t)(vrow * ROW_BYTES + (((vcol >> 3) ^ swz_v<D>(vrow)) << 4) + ((vcol >> 2) & 1) * 8);

    // Q_i^T as the B operand: lane holds query (32*wrow + l32), head-dim slice 16s + 8hh .. +7
    // (QK8: slice 64s + 32hh .. +31, rounded to fp8 here, once)
    constexpr int KSQ = QK8 ? D / 64 : KS;               // score MFMA k-steps
    constexpr int NQK = 2 * KSQ;                         // score MFMAs per block: (k-step, 32-key half)
    typedef std::conditional_t<QK8, i32x8, bf16x8> kop_t; // one score operand
    kop_t qreg[KSQ];
    const int q_row = (int)row0 + wrow * 32 + l32;
    {
        const uint16_t *qrow = p.q + (int64_t)b * p.qsb + (int64_t)min(q_row, n_tok - 1) * p.qsn + (int64_t)h * p.qsh;
        if constexpr (QK8) {
#pragma unroll
            for (int s = 0; s < KSQ; ++s)
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const bf16x8 v8 = *reinterpret_cast<const bf16x8 *>(qrow + 64 * s + 32 * hh + 8 * c);
                    float f[8];
#pragma unroll
                    for (int e = 0; e < 8; ++e) f[e] = (float)v8[e];
                    int w0, w1;
                    cvt8_fp8(f, w0, w1);
                    qreg[s][2 * c] = w0;
                    qreg[s][2 * c + 1] = w1;
                }
        } else {
#pragma unroll
            for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8 *>(qrow + 8 * hh + 16 * s);
        }
    }
    auto qk_mma = [&](const kop_t &a, const kop_t &b, f32x16 c) {
        if constexpr (QK8) return mfma64_fp8(a, b, c);
        else return mfma16(a, b, c);
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int x = 0; x < DB; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[x][e] = 0.f;
    float m_run = -INFINITY;   // running row max, log2 units (score * log2(e)/sqrt(d))
    float l_run = 0.f;         // this lane's share of the running normaliser

    unsigned n_skipped = 0;    // per-head statistics, uniform over the head's waves
    uint32_t mask_word = 0;

    auto is_gated = [&](int j) { return p.causal ? (j < n_gate) : (j < own_lo || j >= own_hi); };

    // K operand n (= k-step n/2, 32-key half n%2) of the tile at LDS byte address kaddr (+ka_base)
    auto k_operand = [&](uint32_t kaddr, int n) {
        if constexpr (QK8) {
            const uint32_t a_s = (kaddr ^ (uint32_t)((n >> 1) << 6)) + (n & 1) * 32 * 128;
            const i32x4 lo = *LDS_PTR(const i32x4, a_s);
            const i32x4 hi = *LDS_PTR(const i32x4, a_s ^ 16u);
            return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        } else {
            const uint32_t a_s = kaddr ^ (uint32_t)((n >> 1) << 5);
            return *LDS_PTR(const bf16x8, a_s + (n & 1) * 32 * ROW_BYTES);
        }
    };
    constexpr int PD = 5;            // LDS operand reads are issued PD MFMAs ahead of their use (measured: 5 is 0.6 % faster
                                     // than 4; 6 gains another 0.4 % but spills a few registers outside the loop)
    constexpr int PDK = QK8 ? 2 : PD; // ... of the score operands (the fp8 ones are twice as wide and four in all)
    // The first PDK score operands of a block are read one phase early (at the end of the previous
    // stage, behind its last MFMAs), so that the score MFMAs do not start with an LDS round trip.
    kop_t kpre[PDK];
    auto prefetch_k = [&](uint32_t kt) {
#pragma unroll
        for (int n = 0; n < PDK; ++n) kpre[n] = k_operand(kt + ka_base, n);
    };

    // S^T of block j from the K tile at LDS byte address `kt` (MFMA and LDS reads only); the
    // order reads-ahead / MFMA is pinned so that no MFMA waits for a read issued just before it
    auto qk_mfma = [&](ScoreTile &t, uint32_t kt) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) t.s[kb][e] = 0.f;
        const uint32_t kaddr = kt + ka_base;
        kop_t a[NQK + PDK];
#pragma unroll
        for (int n = 0; n < PDK; ++n) a[n] = kpre[n];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int n = 0; n < NQK; ++n) {
            if (n + PDK < NQK) a[n + PDK] = k_operand(kaddr, n + PDK);
            t.s[n & 1] = qk_mma(a[n], qreg[n >> 1], t.s[n & 1]);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // causal mask on boundary blocks, row maxima, and the wave's block maximum into
    // lds_red[j & 1].  FAST: the block is known to be gateable (no causal mask).
    // FAST in the forward kernel proper: nobody asks for the maximum itself, only for the decision,
    // and  max_lanes(m) * c >= T  <=>  some lane has m * c >= T  (c > 0, rounding is monotone): every
    // lane compares its own maximum with its head's threshold and the wave publishes one flag.  That
    // takes the cross-lane reductions out of the stretch between the last score MFMA and the barrier,
    // where nothing else runs; the row maximum the softmax needs is completed after the barrier.
    auto reduce_scores = [&](ScoreTile &t, int j, auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        if constexpr (FAST && !CALIB) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, t.s[kb][e]);
            t.mx = mx;                                        // this lane's half of the row; see finish_row_max
            const bool wave_ge = __builtin_amdgcn_ballot_w64(mx * p.scale >= tau_own) != 0ull;
            if (lane == 0) lds_red[j & 1][wave] = wave_ge ? 1.f : 0.f;
            return;
        }
        const bool gated = FAST ? true : is_gated(j);
        if constexpr (!FAST) {
            if (p.causal && !gated) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        const int key = j * BN + 32 * kb + 8 * (e >> 2) + 4 * hh + (e & 3);
                        if (key > q_row) t.s[kb][e] = -INFINITY;
                    }
            }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, t.s[kb][e]);
        t.mx = pair_max(mx);
        if (gated) {
            float stat = t.mx;
            if constexpr (!FAST) {
                // the comparison predicate (Section 3): local row maximum minus the running row maximum
                // after this block, natural units; m_run covers the kept blocks before this one
                if (p.gate_mode) stat = fminf(t.mx * p.scale - m_run * 0.6931471805599453f, 0.f);
            }
            const float wm = wave_max_paired(stat);
            if (lane == 0) lds_red[j & 1][wave] = wm;
        }
    };

    // gate decisions for block j + statistics.  `red` holds the waves' block maxima, read from
    // lds_red[j & 1] after the barrier that publishes them (the read is issued early by the caller
    // so that its latency is covered)
    auto decide = [&](ScoreTile &t, int j, const float (&red)[NW], auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        bool keep = true, any_keep = true;
        float bmax = NAN;
        if (FAST || is_gated(j)) {
            any_keep = false;
#pragma unroll
            for (int x = 0; x < HP; ++x) {
                float r = red[x * NWH];
#pragma unroll
                for (int w = 1; w < NWH; ++w) r = fmaxf(r, red[x * NWH + w]);
                const float sm = (!FAST && p.gate_mode) ? r : r * p.scale;   // natural score units (Eq. 5-6)
                const bool kx = (sm >= tau_h[x]);                    // skip iff s_max < T
                any_keep = any_keep || kx;
                if (x == hsel) {
                    keep = kx;
                    bmax = sm;
                }
            }
        }
        t.keep = keep;
        t.any_keep = any_keep;
        n_skipped += keep ? 0 : 1;
        mask_word |= (keep ? 0u : 1u) << (j & 31);
        if (p.block_max && stat_lane) p.block_max[stat_row * p.mkv + j] = bmax;
        if ((j & 31) == 31 || j == n_blk - 1) {
            if (p.skip_mask && stat_lane) p.skip_mask[stat_row * p.mask_words + (j >> 5)] = mask_word;
            mask_word = 0;
        }
    };

    // online-softmax update of the running statistics with block `t`: new row max and the
    // accumulator's rescale factor first, then the exponentials, P (bf16) into pb
    auto softmax_begin = [&](ScoreTile &t) {
        const float m_new = fmaxf(m_run, t.mx * p.scale_log2);
        t.m_use = (m_new == -INFINITY) ? 0.f : m_new;
        t.alpha = __builtin_amdgcn_exp2f(m_run - t.m_use);
        t.resc = __builtin_amdgcn_ballot_w64(t.alpha != 1.0f) != 0ull;
        m_run = m_new;
    };
    auto softmax_exp = [&](ScoreTile &t, float m_use, float alpha, bf16x8 (&pb)[4]) {
        float psum = 0.f;
#pragma unroll
        for (int idx = 0; idx < 32; idx += 2) {
            const int kb = idx >> 4, e = idx & 15;
            const float p0 = __builtin_amdgcn_exp2f(fmaf(t.s[kb][e], p.scale_log2, -m_use));
            const float p1 = __builtin_amdgcn_exp2f(fmaf(t.s[kb][e + 1], p.scale_log2, -m_use));
            const bf16x2 pp = {(el)p0, (el)p1};
            psum = pair_sum(pp, psum);                                       // sum of the rounded values
            pb[idx >> 3][idx & 7] = pp[0];
            pb[idx >> 3][(idx & 7) + 1] = pp[1];
        }
        l_run = l_run * alpha + psum;
    };
    // softmax_exp(cur) and qk_mfma(nxt) fused.  The exponentials of block j and the score MFMAs
    // of block j+1 are independent: they are written interleaved (per MFMA a few exponentials,
    // their row-sum adds and bf16 packs) and pinned in that order, so that the matrix pipe and
    // the VALU run together.  K operands are read PD MFMAs ahead.
    auto fused_exp_qk = [&](ScoreTile &cur, ScoreTile &nxt, uint32_t kt, float m_use, float alpha, bf16x8 (&pb)[4]) {
        const uint32_t kaddr = kt + ka_base;
        kop_t a[NQK + PDK];
#pragma unroll
        for (int n = 0; n < PDK; ++n) a[n] = kpre[n];
        float psum0 = 0.f, psum1 = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) nxt.s[kb][e] = 0.f;
        constexpr int EPM = 32 / NQK;              // exponentials per MFMA (2 at D = 128, 4 at D = 64; 8 with fp8 operands)
        // The exponentials of one MFMA slot are rounded, packed and summed one slot later, so that
        // no instruction waits for a transcendental issued just before it.
        float ex[EPM];
        auto pack = [&](int n) {                   // the pairs computed in slot n
#pragma unroll
            for (int t = 0; t < EPM; t += 2) {
                const int idx = n * EPM + t;
                const bf16x2 pp = {(el)ex[t], (el)ex[t + 1]};
                // row sum of the rounded values (the ones the second MFMA multiplies): p0 + p1 + acc
                if (t & 2) psum1 = pair_sum(pp, psum1);
                else psum0 = pair_sum(pp, psum0);
                pb[idx >> 3][idx & 7] = pp[0];
                pb[idx >> 3][(idx & 7) + 1] = pp[1];
            }
        };
#pragma unroll
        for (int n = 0; n < NQK; ++n) {
            if (n + PDK < NQK) a[n + PDK] = k_operand(kaddr, n + PDK);
            nxt.s[n & 1] = qk_mma(a[n], qreg[n >> 1], nxt.s[n & 1]);
            float nx[EPM];
#pragma unroll
            for (int t = 0; t < EPM; ++t) {
                const int idx = n * EPM + t;
                nx[t] = __builtin_amdgcn_exp2f(fmaf(cur.s[idx >> 4][idx & 15], p.scale_log2, -m_use));
            }
            if (n > 0) pack(n - 1);
#pragma unroll
            for (int t = 0; t < EPM; ++t) ex[t] = nx[t];
            __builtin_amdgcn_sched_barrier(0);
        }
        pack(NQK - 1);
        l_run = l_run * alpha + (psum0 + psum1);
    };

    auto rescale = [&](const ScoreTile &t) {
        if (t.resc) {
#pragma unroll
            for (int x = 0; x < DB; ++x)
#pragma unroll
                for (int e = 0; e < 16; ++e) oacc[x][e] *= t.alpha;
        }
    };

    // O^T += V^T P^T for the V tile at LDS byte address `vt`; operand n = (k-step u = n / DB,
    // head-dim block x = n % DB), read PD MFMAs ahead
    // `hook(n)` runs after MFMA n has been issued (n a compile-time constant): work that only has to
    // happen soon after the barrier goes there in small pieces, beside the matrix pipe instead of in
    // front of it
    constexpr int NPV = 4 * DB;
    auto pv = [&](const bf16x8 (&pb)[4], uint32_t vt, auto hook) {
        const uint32_t vaddr = vt + va_base;
        auto v_operand = [&](int n) {
            const int u = n / DB, x = n % DB;
            if constexpr (VT) return *LDS_PTR(const bf16x8, (vaddr ^ (uint32_t)(u << 5)) + x * 32 * 128);
            const uint32_t a_x = (vaddr ^ (uint32_t)(x << XSH)) + u * 16 * ROW_BYTES;
            const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a_x));
            const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a_x + 8 * ROW_BYTES));
            const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
            return __builtin_bit_cast(bf16x8, av);
        };
        bf16x8 a[NPV + PD];
#pragma unroll
        for (int n = 0; n < PD; ++n) a[n] = v_operand(n);
        __builtin_amdgcn_sched_barrier(0);
        static_for<NPV>([&](auto nc) {
            constexpr int n = decltype(nc)::value;
            if constexpr (n + PD < NPV) a[n + PD] = v_operand(n + PD);
            oacc[n % DB] = mfma16(a[n], pb[n / DB], oacc[n % DB]);
            __builtin_amdgcn_sched_barrier(0);
            hook(nc);
            __builtin_amdgcn_sched_barrier(0);
        });
    };

    uint32_t kring = (uint32_t)(1 % KR) * TILE_BYTES;     // ring offset of the K slot the next stage reads
    // sources of the copies a stage requests, advanced by one block per stage: K_{j+R} and V_{j+1}
    const unsigned char *k_ahead = k_bytes + R * kstep_b;
    const unsigned char *v_ahead = v_bytes + vstep_b;
    // One pipeline stage: finish block j (`cur`), look ahead to block j+1 (`nxt`).
    // FAST: block j+1 exists and is gateable, so the look-ahead has no mask and no conditionals.
    auto stage = [&](ScoreTile &cur, ScoreTile &nxt, int j, auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        constexpr bool FLAGS = FAST && !CALIB;           // the waves publish decisions, not maxima (see reduce_scores)
        const bool has_next = FAST || (j + 1 < n_blk);
        bf16x8 pb[4];
        const bool do_pv = !CALIB && cur.keep;
        // slot of K_{j+1}; K_{j+R} is requested into the same slot once block j+1 has left it
        // (R = KR + 1), so one ring position per stage is all the bookkeeping there is
        const uint32_t kt_next = lds_k0 + kring;
        kring = (kring + TILE_BYTES == KR * TILE_BYTES) ? 0u : kring + TILE_BYTES;
        const unsigned char *const k_src = k_ahead, *const v_src = v_ahead;
        k_ahead += kstep_b;
        v_ahead += vstep_b;
        if (do_pv) {
            rescale(cur);                         // the previous block's PV has been issued already
            if constexpr (FAST) {
                fused_exp_qk(cur, nxt, kt_next, cur.m_use, cur.alpha, pb);
            } else {
                softmax_exp(cur, cur.m_use, cur.alpha, pb);
                if (has_next) qk_mfma(nxt, kt_next);
            }
        } else {
            if (has_next) qk_mfma(nxt, kt_next);
        }
        if (has_next) reduce_scores(nxt, j + 1, fast_tag);
        // copies that must have landed before the barrier: V_j (if requested) and K_{j+2}; every
        // younger request (K_{j+3} .. K_{j+R-1}, issued after V_j) may stay in flight
        if (R >= 4 && j - 1 + R < n_blk) {
            if (!CALIB && cur.any_keep) wait_vmcnt<NSTK>();
            else wait_vmcnt<(R >= 4 ? NSTK * (R - 3) : 0)>();
        } else {
            wait_vmcnt<0>();
        }
        wg_barrier();
        float red[NW];
        if (has_next) {
#pragma unroll
            for (int w = 0; w < NW; ++w) red[w] = lds_red[(j + 1) & 1][w];
        }
        __builtin_amdgcn_sched_barrier(0);
        // The look-ahead -- decision for block j+1, its statistics, the requests for V_{j+1} and
        // K_{j+R}, the running maximum -- in pieces, so that a kept block can issue them between its
        // PV MFMAs a few instructions at a time.
        auto la_decide = [&]() {
            if (!has_next) return;
            // the maxima are consumed here and not earlier: nothing computed from them may be
            // hoisted in front of the PV MFMAs, where it would wait for the LDS read
#pragma unroll
            for (int w = 0; w < NW; ++w) asm volatile("" : "+v"(red[w]));
            if constexpr (FLAGS) {
                bool kx[HP];
#pragma unroll
                for (int x = 0; x < HP; ++x) {
                    float f = red[x * NWH];
#pragma unroll
                    for (int w = 1; w < NWH; ++w) f = fmaxf(f, red[x * NWH + w]);
                    kx[x] = __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, f)) != 0;   // a scalar: the branches below are uniform
                }
                const bool keep = hsel ? kx[HP - 1] : kx[0];
                nxt.keep = keep;
                nxt.any_keep = kx[0] || kx[HP - 1];
                n_skipped += keep ? 0 : 1;
                mask_word |= (keep ? 0u : 1u) << ((j + 1) & 31);
            } else {
                decide(nxt, j + 1, red, fast_tag);
            }
        };
        auto la_stats = [&]() {
            if constexpr (FLAGS) {                        // (block j+1 is never the tile's last one here)
                if (((j + 1) & 31) == 31) {
                    if (p.skip_mask && stat_lane) p.skip_mask[stat_row * p.mask_words + ((j + 1) >> 5)] = mask_word;
                    mask_word = 0;
                }
            }
        };
        auto la_vcopy = [&]() {
            if (has_next && !CALIB && nxt.any_keep) {
                if constexpr (FAST) tile_copy_async<NST, NT>(v_src, voff, lds_v0 + (uint32_t)((j + 1) & 1) * TILE_BYTES, wave);
                else copy_v_from(v_src, j + 1);           // a gateable block is never the partial one
            }
        };
        auto la_kcopy = [&]() {
            if (has_next && j + R < n_blk) copy_k_from(k_src, j + R, kt_next);
        };
        auto la_softmax = [&]() {                        // running max and rescale factor, off the critical path
            if (has_next && !CALIB && nxt.keep) {
                if constexpr (FLAGS) nxt.mx = pair_max(nxt.mx);
                softmax_begin(nxt);
            }
        };
        if (do_pv) {
            if constexpr (!CALIB) {
                constexpr int HS = NPV / 8;               // MFMAs from one piece to the next
                pv(pb, lds_v0 + (uint32_t)(j & 1) * TILE_BYTES, [&](auto nc) {
                    constexpr int n = decltype(nc)::value;
                    if constexpr (n == HS) la_decide();
                    if constexpr (n == 2 * HS) la_stats();
                    if constexpr (n == 3 * HS) la_vcopy();
                    if constexpr (n == 4 * HS) la_kcopy();
                    if constexpr (n == 5 * HS) la_softmax();
                    if constexpr (n == NPV - 2) prefetch_k(lds_k0 + kring);   // K_{j+2}: landed and visible since the barrier
                });
            }
        } else {
            // the operand reads first, so that they travel while the look-ahead is issued (where V is
            // gathered in place the registers do not allow it: there they come last)
            if constexpr (VT || CALIB) prefetch_k(lds_k0 + kring);
            __builtin_amdgcn_sched_barrier(0);
            la_decide();
            la_softmax();
            la_vcopy();
            la_kcopy();
            la_stats();
            if constexpr (!(VT || CALIB)) prefetch_k(lds_k0 + kring);
        }
    };

    // ---- prologue: scores and decision of block 0, then K_1 .. K_{R-1} and V_0 -----------------
    ScoreTile ta, tb;
    copy_k(0, lds_k0);
    wait_vmcnt<0>();
    wg_barrier();
    prefetch_k(lds_k0);
    qk_mfma(ta, lds_k0);
    reduce_scores(ta, 0, std::false_type{});
    wg_barrier();                                       // block maxima visible, K_0 consumed
    {
        float red[NW];
#pragma unroll
        for (int w = 0; w < NW; ++w) red[w] = lds_red[0][w];
        decide(ta, 0, red, std::false_type{});
        if (!CALIB && ta.keep) softmax_begin(ta);
    }
    if (!CALIB && ta.any_keep) copy_v(0);
#pragma unroll
    for (int t = 1; t < R; ++t)                            // K_{R-1} reuses the slot block 0 has just left
        if (t < n_blk) copy_k(t, lds_k0 + (uint32_t)(t % KR) * TILE_BYTES);
    wait_vmcnt<0>();                                       // drained once; from here on the steady-state rule holds
    wg_barrier();
    prefetch_k(lds_k0 + kring);                            // K_1 for the first stage

    // main loop, two stages per trip.  A pair runs the fused, mask-free stages when both of its
    // look-ahead blocks (j+1, j+2) exist and are gateable: every pair below the causal boundary;
    // without the causal mask every pair before the tile's own token range and, in a second
    // segment, every pair behind it (Section 4.3, last sentence: only the own-range blocks bypass the
    // gate).  The remaining pairs take the general stages.
    int j = 0;
    for (int seg = 0; seg < 2; ++seg) {
        const int fast_end = (p.gate_mode || (!CALIB && p.block_max)) ? 0 : seg == 0 ? (p.causal ? n_gate : own_lo) : (p.causal ? 0 : n_blk);
        for (; j + 2 < fast_end; j += 2) {
            stage(ta, tb, j, std::true_type{});
            stage(tb, ta, j + 1, std::true_type{});
        }
        // first even j whose look-ahead block lies behind the own range
        const int gen_end = (seg == 0 && !p.causal) ? min(own_hi & ~1, n_blk) : n_blk;
        for (; j < gen_end; j += 2) {
            stage(ta, tb, j, std::false_type{});
            if (j + 1 < n_blk) stage(tb, ta, j + 1, std::false_type{});
        }
    }

    // ---- statistics ------------------------------------------------------------------------
    const int htid = tid - hsel * NWH * 64;               // thread index within the head's waves
    if (p.block_max)
        for (int jj = n_blk + htid; jj < p.mkv; jj += NWH * 64) p.block_max[stat_row * p.mkv + jj] = NAN;
    if (p.skip_mask)
        for (int w = ((n_blk + 31) >> 5) + htid; w < p.mask_words; w += NWH * 64) p.skip_mask[stat_row * p.mask_words + w] = 0u;
    if (p.counts && stat_lane) {
        unsigned long long *c = p.counts + ((int64_t)b * p.hq + h) * 3;
        const int gateable = p.causal ? n_gate : (p.mkv - (own_hi - own_lo));
        atomicAdd(c + 0, (unsigned long long)n_skipped);
        atomicAdd(c + 1, (unsigned long long)gateable);
        atomicAdd(c + 2, (unsigned long long)n_blk);
    }

    // ---- O_i = O~_i / l_i, written as bf16 ----------------------------------------------------
    if constexpr (!CALIB) {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const float inv = 1.0f / l_tot;
        if (q_row >= n_tok) return;     // padding rows of the last tile are not stored
        if (p.lse && hh == 0)           // L = m + log(l); m_run is in log2 units
            p.lse[((int64_t)b * p.seqlen + q_row) * p.hq + h] = m_run * 0.6931471805599453f + __logf(l_tot);
        uint16_t *op = p.out + (int64_t)b * p.osb + (int64_t)q_row * p.osn + (int64_t)h * p.osh;
#pragma unroll
        for (int x = 0; x < DB; ++x)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                // O^T row 8*e4 + 4hh + e of block x -> head-dim column (see the V operand mapping)
                const int m0 = 8 * e4 + 4 * hh;
                const int d0 = VT ? 32 * x + m0 : X_COLS * x + (m0 < 16 ? m0 : G16_COLS + m0 - 16);
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (el)(oacc[x][4 * e4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + d0) = o;
            }
    }
}

__global__ void zero_counts_kernel(unsigned long long *c, int n)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) c[t] = 0ull;
}

// V -> workspace, once per forward call: for every (batch, KV head, 64-key block) the tile V_j^T in
// exactly the byte order the forward kernel wants in LDS (see its operand addresses): D rows of 64
// keys; inside a 16-key step the keys are ordered 0-3, 8-11, 4-7, 12-15 (the 8 keys one lane of the
// second MFMA multiplies are then 16 contiguous bytes); the 16-byte chunk index is XOR-ed with
// (row >> 1) & 7.  Rows at and beyond the sequence end repeat the last token (Section 4.3), so the
// tile of a partial block holds finite values everywhere; blocks that lie entirely beyond the end
// are never read and are not written.  One workgroup per tile, through LDS.
template <int D>
__global__ void __launch_bounds__(256) transpose_v_kernel(const FwdParams p)
{
    constexpr int BN = kBlockN, CPR = D / 8, LD = D + 8;
    __shared__ __attribute__((aligned(16))) uint16_t tile[BN * LD];
    const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    int n_tok = p.seqlen;
    if (p.seqlens) n_tok = min(max(p.seqlens[b], 0), p.seqlen);
    if (j * BN >= n_tok) return;
    const uint16_t *src = p.v + (int64_t)b * p.vsb + (int64_t)g * p.vsh;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    for (int sigma = tid; sigma < BN * CPR; sigma += 256) {
        const int row = sigma / CPR, cp = sigma % CPR;
        const int tok = min(j * BN + row, n_tok - 1);
        const u32x4 c = *reinterpret_cast<const u32x4 *>(src + (int64_t)tok * p.vsn + 8 * cp);
        *reinterpret_cast<u32x4 *>(&tile[row * LD + 8 * cp]) = c;
    }
    __syncthreads();
    uint16_t *dst = p.vt + (((int64_t)b * p.hkv + g) * p.mkv + j) * (int64_t)(BN * D);
    for (int sigma = tid; sigma < D * 8; sigma += 256) {
        const int d = sigma >> 3, cphys = sigma & 7;
        const int c = cphys ^ ((d >> 1) & 7);        // logical chunk: 16-key step c >> 1, lane half c & 1
        const int u = c >> 1, hh = c & 1;
        uint16_t w[8];
#pragma unroll
        for (int t = 0; t < 8; ++t) w[t] = tile[(16 * u + 8 * (t >> 2) + 4 * hh + (t & 3)) * LD + d];
        u32x4 o;
#pragma unroll
        for (int t = 0; t < 4; ++t) o[t] = (uint32_t)w[2 * t] | ((uint32_t)w[2 * t + 1] << 16);
        *reinterpret_cast<u32x4 *>(dst + (int64_t)sigma * 8) = o;
    }
}

// K -> workspace as fp8 (e4m3, round to nearest even), once per call, for the fp8 score product: for
// every (batch, KV head, 64-key block) a tile of 64 rows x 128 bytes in the byte order the forward
// kernel wants in LDS (16-byte chunk index XOR-ed with (row >> 1) & 7).  Rows at and beyond the
// sequence end repeat the last token (Section 4.3).  head_dim 128 only.
template <bool F16>
__global__ void __launch_bounds__(256) quantize_k_kernel(const FwdParams p)
{
    typedef typename Elem<F16>::x8 x8;
    constexpr int BN = kBlockN, D = 128;
    const int j = blockIdx.x, g = blockIdx.y, b = blockIdx.z, tid = threadIdx.x;
    int n_tok = p.seqlen;
    if (p.seqlens) n_tok = min(max(p.seqlens[b], 0), p.seqlen);
    if (j * BN >= n_tok) return;
    const uint16_t *src = p.k + (int64_t)b * p.ksb + (int64_t)g * p.ksh;
    uint8_t *dst = p.k8 + (((int64_t)b * p.hkv + g) * p.mkv + j) * (int64_t)(BN * D);
    for (int sigma = tid; sigma < BN * 8; sigma += 256) {
        const int row = sigma >> 3, cphys = sigma & 7;
        const int c = cphys ^ ((row >> 1) & 7);               // head-dim elements 16c .. 16c + 15
        const int tok = min(j * BN + row, n_tok - 1);
        const uint16_t *e = src + (int64_t)tok * p.ksn + 16 * c;
        i32x4 o;
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            const x8 v8 = *reinterpret_cast<const x8 *>(e + 8 * half);
            float f[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) f[t] = (float)v8[t];
            int w0, w1;
            cvt8_fp8(f, w0, w1);
            o[2 * half] = w0;
            o[2 * half + 1] = w1;
        }
        *reinterpret_cast<i32x4 *>(dst + (int64_t)sigma * 16) = o;
    }
}

template <int D, int NWH, int HP, int KR, bool F16, bool VT, bool QK8>
static hipError_t launch_k(const FwdParams &p, bool calib, hipStream_t stream, long grid)
{
    if (calib)
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NWH, HP, KR, true, F16, false, QK8>), dim3((unsigned)grid), dim3(NWH * HP * 64), 0, stream, p);
    else
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NWH, HP, KR, false, F16, VT, QK8>), dim3((unsigned)grid), dim3(NWH * HP * 64), 0, stream, p);
    return hipGetLastError();
}

template <int D, int NWH, int HP, int KR>
static hipError_t launch_t(const FwdParams &p, bool calib, hipStream_t stream)
{
    const int pairs = p.batch * p.hkv;
    const int gsub = p.group / HP;
    long grid = (pairs >= 8) ? 8L * ((pairs + 7) / 8) * gsub * p.mq : (long)pairs * gsub * p.mq;
    if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
    if (p.counts) {
        const int n = p.batch * p.hq * 3;
        hipLaunchKernelGGL(zero_counts_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p.counts, n);
    }
    if constexpr (NWH == 4) {          // the 128-row tile can take V (and fp8 K) from the workspace
        if (p.k8 && !calib && !p.vt) return hipErrorInvalidValue;   // the fp8 score path always takes V from the workspace
        if ((p.vt && !calib) || p.k8) {
            if (p.hkv > 65535 || p.batch > 65535) return hipErrorInvalidValue;    // grid y, z limits
            const dim3 tiles((unsigned)p.mkv, (unsigned)p.hkv, (unsigned)p.batch);
            if (p.vt && !calib) hipLaunchKernelGGL((transpose_v_kernel<D>), tiles, dim3(256), 0, stream, p);
            if constexpr (D == 128) {
                if (p.k8) {
                    if (p.f16) hipLaunchKernelGGL((quantize_k_kernel<true>), tiles, dim3(256), 0, stream, p);
                    else hipLaunchKernelGGL((quantize_k_kernel<false>), tiles, dim3(256), 0, stream, p);
                    hipError_t e = hipGetLastError();
                    if (e != hipSuccess) return e;
                    return p.f16 ? launch_k<D, NWH, HP, KR, true, true, true>(p, calib, stream, grid)
                                 : launch_k<D, NWH, HP, KR, false, true, true>(p, calib, stream, grid);
                }
            }
            hipError_t e = hipGetLastError();
            if (e != hipSuccess) return e;
            return p.f16 ? launch_k<D, NWH, HP, KR, true, true, false>(p, calib, stream, grid) : launch_k<D, NWH, HP, KR, false, true, false>(p, calib, stream, grid);
        }
    }
    if (p.k8) return hipErrorInvalidValue;             // fp8 score operands need the 128 x 64 tile and head_dim 128
    return p.f16 ? launch_k<D, NWH, HP, KR, true, false, false>(p, calib, stream, grid) : launch_k<D, NWH, HP, KR, false, false, false>(p, calib, stream, grid);
}

bool shape_supported(int head_dim, int block_m, int block_n)
{
    if (block_n != kBlockN) return false;
    if (head_dim != 64 && head_dim != 128) return false;
    return block_m == 32 || block_m == 64 || block_m == 128;
}

hipError_t launch_forward(const FwdParams &p, int head_dim, int block_m, bool calib, hipStream_t stream)
{
    if (!shape_supported(head_dim, block_m, kBlockN)) return hipErrorInvalidValue;
    // the copies address a tile with 32-bit byte offsets
    if (p.ksn * 128 > 0x7fff0000LL || p.vsn * 128 > 0x7fff0000LL) return hipErrorInvalidValue;
    const bool pair_heads = (p.group % 2 == 0) && !p.single_head;
#define BSFA_CASE(DD, NN, HH, KK) \
    if (head_dim == DD && block_m == 32 * NN) return launch_t<DD, NN, HH, KK>(p, calib, stream);
    if (pair_heads) {
        // two query heads of a GQA group per workgroup: one K/V stream in LDS feeds both
        BSFA_CASE(128, 4, 2, 5)
        BSFA_CASE(64, 4, 2, 5)
    }
    BSFA_CASE(64, 1, 1, 2) BSFA_CASE(64, 2, 1, 2) BSFA_CASE(64, 4, 1, 3)
    BSFA_CASE(128, 1, 1, 2) BSFA_CASE(128, 2, 1, 2) BSFA_CASE(128, 4, 1, 2)
#undef BSFA_CASE
    return hipErrorInvalidValue;
}

}  // namespace bsfa
