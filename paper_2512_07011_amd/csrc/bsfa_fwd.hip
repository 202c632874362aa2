// Block-Sparse FlashAttention forward kernel for gfx950 (MI355X), wave64, bf16 MFMA.
//
// One workgroup = one query tile Q_i (B_M = 32 * QB * NW rows: NW waves, QB 32-row column blocks
// per wave) of one head; it walks the reachable key blocks j in ascending order (Algorithm 1):
//   S_ij^T = K_j Q_i^T        32x32x16 bf16 MFMA, fp32 accumulate                 (Eq. 5)
//   s_max  = max S_ij         lane max -> wave max -> cross-wave max through LDS   (Eq. 6)
//   gate   : s_max / sqrt(d) >= T keeps the block; blocks touching the causal boundary bypass
//            the gate (Section 4.1).  The decision is workgroup-uniform.
//   kept   : V_j is requested only after the decision, exp2-based online softmax,
//            O^T += V_j^T P^T.
// The transposed products keep everything of one query row inside one lane pair (l, l^32):
// the S^T accumulator layout (column = query) is already the B-operand layout of the second
// MFMA up to a permutation of the keys, and the same permutation is applied to V when its
// A operand is gathered from LDS with the transposing read, so P never leaves registers.
//
// Software pipeline (one barrier per key block).  While block j is being finished the scores
// of block j+1 are already computed, so its gate decision is known one block ahead:
//   iteration j:  S_{j+1} = K_{j+1} Q^T  (MFMA)   overlapped with   softmax(S_j)  (VALU)
//                 block max of S_{j+1} -> LDS;  wait for own global->LDS copies;  barrier
//                 decide keep_{j+1};  request V_{j+1} (only if kept) and K_{j+3}
//                 O^T += V_j^T P_j^T   (MFMA, V_j landed before the barrier)
// K and V tiles go HBM -> LDS directly (no register staging), two buffers each.
#include "bsfa_internal.h"

#include <math.h>
#include <stdlib.h>

#include <type_traits>

namespace bsfa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))
#define GLB_PTR(T, p) ((const __attribute__((address_space(1))) T *)(p))

// ---- LDS tile layout --------------------------------------------------------------------
// A K or V tile is 64 rows x D bf16, stored as 16-byte chunks, row-major, the chunk index
// XOR-ed with a function of the row so that the operand gathers spread over the banks.  The
// swizzle is applied on the global side of the copy (lane -> which chunk it fetches); the LDS
// side of a direct copy is always linear (wave base + lane * 16 bytes).
template <int D> __device__ __forceinline__ int swz_k(int row)
{
    return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int swz_v(int row)
{
    return (D == 128) ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
}

// Element offset (relative to the tile's first row) of the chunk thread `tid` copies in
// repetition r.
template <int D, int NT, bool ISV>
__device__ __forceinline__ int chunk_src_offset(int r, int tid, int stride_n)
{
    constexpr int CPR = D / 8;
    const int sigma = r * NT + tid;
    const int row = sigma / CPR, cp = sigma % CPR;
    const int c = cp ^ (ISV ? swz_v<D>(row) : swz_k<D>(row));
    return row * stride_n + 8 * c;
}

// Asynchronous HBM -> LDS copy of one 64 x D tile (completion is tracked by vmcnt).
template <int D, int NT>
__device__ __forceinline__ void tile_copy_async(const uint16_t *gtile, const int (&off)[64 * (D / 8) / NT],
                                                uint16_t *lds_tile, int wave)
{
#pragma unroll
    for (int r = 0; r < 64 * (D / 8) / NT; ++r)
        __builtin_amdgcn_global_load_lds(GLB_PTR(void, gtile + off[r]),
                                         LDS_PTR(void, lds_tile + (r * NT + wave * 64) * 8), 16, 0, 0);
}

template <int CTRL> __device__ __forceinline__ float dpp_max(float v)
{
    const int x = __builtin_bit_cast(int, v);
    return fmaxf(v, __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(x, x, CTRL, 0xf, 0xf, false)));
}

// max over lanes l and l^32, result in both lanes.  v_permlane32_swap exchanges the upper half
// of its first operand with the lower half of its second: with two copies of x the first
// register ends up holding x[l & 31] and the second x[32 + (l & 31)] in every lane.  Written as
// one asm block so that the two copies are guaranteed to live in different registers.
__device__ __forceinline__ float pair_max(float x)
{
    float a = x, b;
    asm volatile("v_mov_b32 %1, %0\n\ts_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "=&v"(b));
    return fmaxf(a, b);
}

// max over the wave of a value that is already equal in lanes l and l^32 (wave-uniform result)
__device__ __forceinline__ float wave_max_paired(float x)
{
    x = dpp_max<0xB1>(x);     // quad_perm [1,0,3,2]
    x = dpp_max<0x4E>(x);     // quad_perm [2,3,0,1]
    x = dpp_max<0x141>(x);    // row_half_mirror
    x = dpp_max<0x140>(x);    // row_mirror
    const int xi = __builtin_bit_cast(int, x);
    return fmaxf(__builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 0)),
                 __builtin_bit_cast(float, __builtin_amdgcn_readlane(xi, 16)));
}

// Work decomposition.  With at least 8 (batch, KV head) pairs the pair is chosen by the low
// three bits of the workgroup id, which is the XCD the hardware dispatches the group to, so
// that all groups streaming one K/V sequence share one L2.  Heavy (late) query tiles first.
__device__ __forceinline__ bool decode_work(const FwdParams &p, int w, int &b, int &h, int &i)
{
    const int pairs = p.batch * p.hkv;
    if (pairs >= 8) {
        const int x = w & 7, r = w >> 3;
        const int npx = (pairs + 7) >> 3;
        const int per_tile = npx * p.group;
        const int idesc = r / per_tile, rest = r - idesc * per_tile;
        const int pl = rest / p.group, hg = rest - pl * p.group;
        const int pair = x + 8 * pl;
        if (pair >= pairs) return false;
        b = pair / p.hkv;
        h = (pair - b * p.hkv) * p.group + hg;
        i = p.mq - 1 - idesc;
    } else {
        const int per_tile = p.batch * p.hq;
        const int idesc = w / per_tile, rest = w - idesc * per_tile;
        b = rest / p.hq;
        h = rest - b * p.hq;
        i = p.mq - 1 - idesc;
    }
    return true;
}

template <int QB> struct ScoreTile {
    f32x16 s[2][QB];      // S^T: [32-key half][32-query column block], raw q.k (no 1/sqrt(d))
    float mx[QB];         // row max of the lane's query, equal in lanes l and l^32
    bool keep;            // workgroup-uniform gate decision
};

template <int D, int NW, int QB, bool CALIB, int OCC>
__global__ void __launch_bounds__(NW * 64, OCC) bsfa_fwd_kernel(const FwdParams p)
{
    constexpr int NT = NW * 64;
    constexpr int BM = NW * QB * 32;
    constexpr int BN = kBlockN;
    constexpr int KS = D / 16;       // MFMA k-steps over the head dim
    constexpr int DB = D / 32;       // 32-row blocks of O^T
    constexpr int CPR = D / 8;       // 16-byte chunks per tile row
    constexpr int NST = 64 * CPR / NT;

    __shared__ __attribute__((aligned(1024))) uint16_t lds_k[2][BN * D];
    __shared__ __attribute__((aligned(1024))) uint16_t lds_v[CALIB ? 1 : 2][CALIB ? 8 : BN * D];
    __shared__ float lds_red[2][NW];

    int b, h, i;
    if (!decode_work(p, blockIdx.x, b, h, i)) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hh = lane >> 5;
    const int g = h / p.group;

    const int64_t row0 = (int64_t)i * BM;                 // first query row of the tile
    const int n_blk = p.causal ? (int)((row0 + BM + BN - 1) / BN) : p.mkv;   // reachable blocks
    // causal: blocks [0, n_gate) are gateable, [n_gate, n_blk) touch the boundary.
    // non-causal: blocks [own_lo, own_hi) overlap the tile's own tokens and bypass the gate.
    const int n_gate = p.causal ? (int)((row0 + 1) / BN) : 0;
    const int own_lo = (int)(row0 / BN), own_hi = (int)((row0 + BM + BN - 1) / BN);

    const uint16_t *kbase = p.k + (int64_t)b * p.ksb + (int64_t)g * p.ksh;
    const uint16_t *vbase = p.v + (int64_t)b * p.vsb + (int64_t)g * p.vsh;
    const float tau = p.tau[p.tau_per_tile ? (int64_t)h * p.mq + i : h];

    int koff[NST], voff[NST];
#pragma unroll
    for (int r = 0; r < NST; ++r) {
        koff[r] = chunk_src_offset<D, NT, false>(r, tid, (int)p.ksn);
        voff[r] = chunk_src_offset<D, NT, true>(r, tid, (int)p.vsn);
    }
    const int64_t kstep = (int64_t)BN * p.ksn, vstep = (int64_t)BN * p.vsn;

    // Q_i^T as the B operand: lane holds query (wave*32*QB + 32*qb + l32), head-dim slice 16s + 8hh .. +7
    bf16x8 qreg[QB][KS];
    int q_row[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        q_row[qb] = (int)row0 + (wave * QB + qb) * 32 + l32;
        const uint16_t *qp = p.q + (int64_t)b * p.qsb + (int64_t)q_row[qb] * p.qsn + (int64_t)h * p.qsh + 8 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[qb][s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
    }

    f32x16 oacc[DB][QB];
#pragma unroll
    for (int x = 0; x < DB; ++x)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int e = 0; e < 16; ++e) oacc[x][qb][e] = 0.f;
    float m_run[QB], l_run[QB];    // running row max (log2 units) and this lane's share of the normaliser
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
    }

    unsigned n_skipped = 0;      // workgroup-uniform statistics
    uint32_t mask_word = 0;
    const int64_t stat_row = ((int64_t)b * p.hq + h) * p.mq + i;

    auto is_gated = [&](int j) { return p.causal ? (j < n_gate) : (j < own_lo || j >= own_hi); };

    // S^T of block j from the K tile in `kt`, row maxima, and the wave's block maximum into
    // lds_red[j & 1].  FAST: the block is known to be gateable (no causal mask, always reduced),
    // which keeps the whole function free of branches.
    auto compute_scores = [&](ScoreTile<QB> &t, const uint16_t *kt, int j, auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int e = 0; e < 16; ++e) t.s[kb][qb][e] = 0.f;
        }
#pragma unroll
        for (int s = 0; s < KS; ++s) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb) {
                const int row = 32 * kb + l32;
                const int c = (2 * s + hh) ^ swz_k<D>(row);
                const bf16x8 a = *reinterpret_cast<const bf16x8 *>(kt + (row * CPR + c) * 8);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    t.s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[qb][s], t.s[kb][qb], 0, 0, 0);
            }
        }
        const bool gated = FAST ? true : is_gated(j);
        if constexpr (!FAST) {
            if (p.causal && !gated) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int key = j * BN + 32 * kb + 8 * (e >> 2) + 4 * hh + (e & 3);
                            if (key > q_row[qb]) t.s[kb][qb][e] = -INFINITY;
                        }
            }
        }
        float all = -INFINITY;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = -INFINITY;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) mx = fmaxf(mx, t.s[kb][qb][e]);
            t.mx[qb] = pair_max(mx);
            all = fmaxf(all, t.mx[qb]);
        }
        if (gated) {
            const float wm = wave_max_paired(all);
            if (lane == 0) lds_red[j & 1][wave] = wm;
        }
    };

    // gate decision for block j (after the barrier that publishes lds_red[j & 1]) + statistics
    auto decide = [&](ScoreTile<QB> &t, int j, auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        bool keep = true;
        float bmax = NAN;
        if (FAST || is_gated(j)) {
            float r = lds_red[j & 1][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) r = fmaxf(r, lds_red[j & 1][w]);
            bmax = r * p.scale;                          // natural score units (Eq. 5-6)
            keep = (bmax >= tau);                        // skip iff s_max < T
        }
        t.keep = keep;
        n_skipped += keep ? 0 : 1;
        mask_word |= (keep ? 0u : 1u) << (j & 31);
        if (p.block_max && tid == 0) p.block_max[stat_row * p.mkv + j] = bmax;
        if ((j & 31) == 31 || j == n_blk - 1) {
            if (p.skip_mask && tid == 0) p.skip_mask[stat_row * p.mask_words + (j >> 5)] = mask_word;
            mask_word = 0;
        }
    };

    // online-softmax update of the running statistics with block `t`; P (bf16) into pb; returns
    // in alpha[] the factor the accumulator still has to be multiplied with
    auto softmax = [&](ScoreTile<QB> &t, bf16x8 (&pb)[4][QB], float (&alpha)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float m_new = fmaxf(m_run[qb], t.mx[qb] * p.scale_log2);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            alpha[qb] = __builtin_amdgcn_exp2f(m_run[qb] - m_use);
            m_run[qb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(t.s[kb][qb][e], p.scale_log2, -m_use));
                    t.s[kb][qb][e] = pe;
                    psum += pe;
                }
            l_run[qb] = l_run[qb] * alpha[qb] + psum;
#pragma unroll
            for (int u = 0; u < 4; ++u)
#pragma unroll
                for (int e = 0; e < 8; ++e) pb[u][qb][e] = (__bf16)t.s[u >> 1][qb][8 * (u & 1) + e];
        }
    };

    auto rescale = [&](const float (&alpha)[QB]) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            if (__any(alpha[qb] != 1.0f)) {
#pragma unroll
                for (int x = 0; x < DB; ++x)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[x][qb][e] *= alpha[qb];
            }
        }
    };

    // O^T += V^T P^T for the V tile in `vt`
    auto pv = [&](const bf16x8 (&pb)[4][QB], const uint16_t *vt) {
        const int L = lane & 15, g16 = (lane >> 4) & 1;
#pragma unroll
        for (int u = 0; u < 4; ++u) {                     // 16 keys per MFMA k-step
            const int r0 = 16 * u + 4 * hh + (L >> 2);
            const int r1 = r0 + 8;
#pragma unroll
            for (int x = 0; x < DB; ++x) {
                const int dcol = 32 * x + 16 * g16 + 4 * (L & 3);         // element column
                const int c = dcol >> 3, half = (dcol >> 2) & 1;
                const uint16_t *a0 = vt + (r0 * CPR + (c ^ swz_v<D>(r0))) * 8 + 4 * half;
                const uint16_t *a1 = vt + (r1 * CPR + (c ^ swz_v<D>(r1))) * 8 + 4 * half;
                const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
                const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a1));
                const s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    oacc[x][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb[u][qb], oacc[x][qb], 0, 0, 0);
            }
        }
    };

    auto wait_copies_and_barrier = [&]() {
        __builtin_amdgcn_s_waitcnt(0x0f70);      // vmcnt(0): this wave's HBM -> LDS copies have landed
        __syncthreads();
    };

    // One pipeline stage: finish block j (`cur`), look ahead to block j+1 (`nxt`).
    // FAST: block j+1 exists and is gateable, so the look-ahead has no mask and no conditionals.
    auto stage = [&](ScoreTile<QB> &cur, ScoreTile<QB> &nxt, int j, auto fast_tag) {
        constexpr bool FAST = decltype(fast_tag)::value;
        const bool has_next = FAST || (j + 1 < n_blk);
        bf16x8 pb[4][QB];
        float alpha[QB];
        if (!CALIB && cur.keep) {
            if (has_next) compute_scores(nxt, lds_k[(j + 1) & 1], j + 1, fast_tag);
            softmax(cur, pb, alpha);
            rescale(alpha);
        } else {
            if (has_next) compute_scores(nxt, lds_k[(j + 1) & 1], j + 1, fast_tag);
        }
        wait_copies_and_barrier();
        if (has_next) {
            decide(nxt, j + 1, fast_tag);
            if (!CALIB && nxt.keep) tile_copy_async<D, NT>(vbase + (int64_t)(j + 1) * vstep, voff, lds_v[CALIB ? 0 : ((j + 1) & 1)], wave);
            if (j + 3 < n_blk) tile_copy_async<D, NT>(kbase + (int64_t)(j + 3) * kstep, koff, lds_k[(j + 1) & 1], wave);
        }
        if constexpr (!CALIB) {
            if (cur.keep) pv(pb, lds_v[j & 1]);
        }
    };

    // ---- prologue: K_0, K_1 in flight, scores and decision of block 0 -------------------------
    ScoreTile<QB> ta, tb;
    tile_copy_async<D, NT>(kbase, koff, lds_k[0], wave);
    if (1 < n_blk) tile_copy_async<D, NT>(kbase + kstep, koff, lds_k[1], wave);
    wait_copies_and_barrier();
    compute_scores(ta, lds_k[0], 0, std::false_type{});
    wait_copies_and_barrier();
    decide(ta, 0, std::false_type{});
    if (!CALIB && ta.keep) tile_copy_async<D, NT>(vbase, voff, lds_v[0], wave);
    if (2 < n_blk) tile_copy_async<D, NT>(kbase + 2 * kstep, koff, lds_k[0], wave);

    // main loop: pairs of stages whose look-ahead block is gateable (causal only), then the rest
    int j = 0;
    if (p.causal) {
        for (; j + 2 < n_gate; j += 2) {
            stage(ta, tb, j, std::true_type{});
            stage(tb, ta, j + 1, std::true_type{});
        }
    }
    for (; j < n_blk; j += 2) {
        stage(ta, tb, j, std::false_type{});
        if (j + 1 < n_blk) stage(tb, ta, j + 1, std::false_type{});
    }

    // ---- statistics ------------------------------------------------------------------------
    if (p.block_max)
        for (int j = n_blk + tid; j < p.mkv; j += NT) p.block_max[stat_row * p.mkv + j] = NAN;
    if (p.skip_mask)
        for (int w = ((n_blk + 31) >> 5) + tid; w < p.mask_words; w += NT) p.skip_mask[stat_row * p.mask_words + w] = 0u;
    if (p.counts && tid == 0) {
        unsigned long long *c = p.counts + ((int64_t)b * p.hq + h) * 3;
        const int gateable = p.causal ? n_gate : (p.mkv - (own_hi - own_lo));
        atomicAdd(c + 0, (unsigned long long)n_skipped);
        atomicAdd(c + 1, (unsigned long long)gateable);
        atomicAdd(c + 2, (unsigned long long)n_blk);
    }

    // ---- O_i = O~_i / l_i, written as bf16 ----------------------------------------------------
    if constexpr (!CALIB) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
            const float inv = 1.0f / l_tot;
            uint16_t *op = p.out + (int64_t)b * p.osb + (int64_t)q_row[qb] * p.osn + (int64_t)h * p.osh;
#pragma unroll
            for (int x = 0; x < DB; ++x)
#pragma unroll
                for (int e4 = 0; e4 < 4; ++e4) {
                    const int d0 = 32 * x + 8 * e4 + 4 * hh;
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (__bf16)(oacc[x][qb][4 * e4 + e] * inv);
                    *reinterpret_cast<bf16x4 *>(op + d0) = o;
                }
        }
    }
}

__global__ void zero_counts_kernel(unsigned long long *c, int n)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) c[t] = 0ull;
}

template <int D, int NW, int QB, int OCC>
static hipError_t launch_t(const FwdParams &p, bool calib, hipStream_t stream)
{
    const int pairs = p.batch * p.hkv;
    long grid = (pairs >= 8) ? 8L * ((pairs + 7) / 8) * p.group * p.mq : (long)p.batch * p.hq * p.mq;
    if (grid <= 0 || grid > 0x7fffffffL) return hipErrorInvalidValue;
    if (p.counts) {
        const int n = p.batch * p.hq * 3;
        hipLaunchKernelGGL(zero_counts_kernel, dim3((n + 255) / 256), dim3(256), 0, stream, p.counts, n);
    }
    if (calib)
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NW, QB, true, OCC>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, p);
    else
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NW, QB, false, OCC>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, p);
    return hipGetLastError();
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
    // the copies address a tile with 32-bit element offsets
    if (p.ksn * 64 > 0x7fffffffLL || p.vsn * 64 > 0x7fffffffLL) return hipErrorInvalidValue;
#define BSFA_CASE(DD, NN, QQ, OO) \
    if (head_dim == DD && block_m == 32 * NN * QQ) return launch_t<DD, NN, QQ, OO>(p, calib, stream);
    {
        const char *v = getenv("BSFA_VARIANT");
        const int variant = v ? atoi(v) : 0;
        if (variant == 1) { BSFA_CASE(128, 4, 1, 1) }
        if (variant == 2) { BSFA_CASE(128, 2, 2, 1) }
    }
    BSFA_CASE(64, 1, 1, 1) BSFA_CASE(64, 2, 1, 1) BSFA_CASE(64, 4, 1, 2)
    BSFA_CASE(128, 1, 1, 1) BSFA_CASE(128, 2, 1, 1) BSFA_CASE(128, 4, 1, 1)
#undef BSFA_CASE
    return hipErrorInvalidValue;
}

}  // namespace bsfa
