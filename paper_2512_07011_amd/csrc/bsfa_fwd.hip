// Block-Sparse FlashAttention forward kernel for gfx950 (MI355X), wave64, bf16 MFMA.
//
// One workgroup = one query tile Q_i (B_M = 32 * NW rows, NW waves, 32 query rows per wave) of
// one head; it walks the reachable key blocks j in ascending order (Algorithm 1 of the paper):
//   S_ij^T = K_j Q_i^T        32x32x16 bf16 MFMA, fp32 accumulate                 (Eq. 5)
//   s_max  = max S_ij         lane max -> wave max -> cross-wave max through LDS   (Eq. 6)
//   gate   : s_max / sqrt(d) >= T keeps the block; blocks touching the causal boundary bypass
//            the gate (Section 4.1).  The branch is workgroup-uniform.
//   kept   : V_j is fetched only now, exp2-based online softmax, O^T += V_j^T P^T.
// The transposed products keep everything of one query row inside one lane pair (l, l^32):
// the S^T accumulator layout (column = query) is already the B-operand layout of the second
// MFMA up to a permutation of the keys, and the same permutation is applied to V when its
// A operand is gathered from LDS with the transposing read, so P never leaves registers.
#include "bsfa_internal.h"

#include <math.h>

namespace bsfa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

// ---- LDS tile layout --------------------------------------------------------------------
// A K or V tile is 64 rows x D bf16.  It is stored as 16-byte chunks, row-major, with the
// chunk index XOR-ed by a function of the row so that the operand gathers below spread over
// the banks.  Any per-row bijection is correct; these two are chosen for the two read shapes.
template <int D> __device__ __forceinline__ int swz_k(int row)
{
    return (D == 128) ? (row & 15) : ((row >> 1) & 7);
}
template <int D> __device__ __forceinline__ int swz_v(int row)
{
    return (D == 128) ? ((row & 7) << 1) : (((row >> 1) & 3) << 1);
}

// Global -> registers: thread tid fetches chunks sigma = r * NT + tid of the linear LDS image,
// i.e. the logical chunk that the swizzle places there.
template <int D, int NT, bool ISV>
__device__ __forceinline__ void tile_fetch(uint4 (&st)[64 * (D / 8) / NT], const uint16_t *base,
                                           int64_t stride_n, int tid)
{
    constexpr int CPR = D / 8;
#pragma unroll
    for (int r = 0; r < 64 * CPR / NT; ++r) {
        int sigma = r * NT + tid;
        int row = sigma / CPR, cp = sigma % CPR;
        int c = cp ^ (ISV ? swz_v<D>(row) : swz_k<D>(row));
        st[r] = *reinterpret_cast<const uint4 *>(base + (int64_t)row * stride_n + 8 * c);
    }
}
template <int D, int NT>
__device__ __forceinline__ void tile_commit(const uint4 (&st)[64 * (D / 8) / NT], uint16_t *lds, int tid)
{
#pragma unroll
    for (int r = 0; r < 64 * (D / 8) / NT; ++r)
        *reinterpret_cast<uint4 *>(lds + (size_t)(r * NT + tid) * 8) = st[r];
}

__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
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

template <int D, int NW, bool CALIB>
__global__ void __launch_bounds__(NW * 64) bsfa_fwd_kernel(const FwdParams p)
{
    constexpr int NT = NW * 64;
    constexpr int BM = NW * 32;
    constexpr int BN = kBlockN;
    constexpr int KS = D / 16;       // MFMA k-steps over the head dim
    constexpr int DB = D / 32;       // 32-row blocks of O^T
    constexpr int CPR = D / 8;       // 16-byte chunks per tile row
    constexpr int NST = 64 * CPR / NT;

    __shared__ __attribute__((aligned(16))) uint16_t lds_k[2][BN * D];
    __shared__ __attribute__((aligned(16))) uint16_t lds_v[CALIB ? 8 : BN * D];
    __shared__ float lds_red[2][NW];

    int b, h, i;
    if (!decode_work(p, blockIdx.x, b, h, i)) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
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

    // Q_i^T as the B operand: lane holds query (wave*32 + l32), head-dim slice 16s + 8hh .. +7
    bf16x8 qreg[KS];
    {
        const uint16_t *qp = p.q + (int64_t)b * p.qsb + (row0 + wave * 32 + l32) * p.qsn + (int64_t)h * p.qsh + 8 * hh;
#pragma unroll
        for (int s = 0; s < KS; ++s) qreg[s] = *reinterpret_cast<const bf16x8 *>(qp + 16 * s);
    }

    f32x16 oacc[DB];
#pragma unroll
    for (int x = 0; x < DB; ++x)
#pragma unroll
        for (int e = 0; e < 16; ++e) oacc[x][e] = 0.f;
    float m_run = -INFINITY;   // running row max, log2 units (score * log2(e)/sqrt(d))
    float l_run = 0.f;         // this lane's share of the running normaliser
    const int q_row = (int)(row0) + wave * 32 + l32;      // token index of this lane's query

    unsigned long long n_skipped = 0;
    uint32_t mask_word = 0;
    const int64_t stat_row = ((int64_t)b * p.hq + h) * p.mq + i;

    uint4 stage[NST];
    tile_fetch<D, NT, false>(stage, kbase, p.ksn, tid);
    tile_commit<D, NT>(stage, lds_k[0], tid);
    __syncthreads();

    for (int j = 0; j < n_blk; ++j) {
        const uint16_t *kcur = lds_k[j & 1];
        const bool more = (j + 1 < n_blk);
        if (more) tile_fetch<D, NT, false>(stage, kbase + (int64_t)(j + 1) * BN * p.ksn, p.ksn, tid);

        // ---- S^T = K_j Q_i^T : two 32-key halves, raw (unscaled) scores --------------------
        f32x16 sacc[2];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int e = 0; e < 16; ++e) sacc[kb][e] = 0.f;
            const int row = 32 * kb + l32;
#pragma unroll
            for (int s = 0; s < KS; ++s) {
                const int c = (2 * s + hh) ^ swz_k<D>(row);
                bf16x8 a = *reinterpret_cast<const bf16x8 *>(kcur + (row * CPR + c) * 8);
                sacc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[s], sacc[kb], 0, 0, 0);
            }
        }

        const bool gated = p.causal ? (j < n_gate) : (j < own_lo || j >= own_hi);
        if (p.causal && !gated) {
            // boundary block: key token > query token is masked out
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = j * BN + 32 * kb + 8 * (e >> 2) + 4 * hh + (e & 3);
                    if (key > q_row) sacc[kb][e] = -INFINITY;
                }
        }
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int e = 0; e < 16; ++e) mx = fmaxf(mx, sacc[kb][e]);
        mx = fmaxf(mx, __shfl_xor(mx, 32));              // row max of this lane pair's query

        if (gated) {
            const float wm = wave_max(mx);
            if (lane == 0) lds_red[j & 1][wave] = wm;
        }
        if (more) tile_commit<D, NT>(stage, lds_k[(j + 1) & 1], tid);
        __syncthreads();

        bool keep = true;
        float bmax = NAN;
        if (gated) {
            float r = lds_red[j & 1][0];
#pragma unroll
            for (int w = 1; w < NW; ++w) r = fmaxf(r, lds_red[j & 1][w]);
            bmax = r * p.scale;                          // natural score units (Eq. 5-6)
            keep = (bmax >= tau);                        // skip iff s_max < T
        }
        if (tid == 0) {
            if (p.block_max) p.block_max[stat_row * p.mkv + j] = bmax;
            if (!keep) {
                ++n_skipped;
                mask_word |= 1u << (j & 31);
            }
            if (p.skip_mask && ((j & 31) == 31 || j == n_blk - 1)) {
                p.skip_mask[stat_row * p.mask_words + (j >> 5)] = mask_word;
                mask_word = 0;
            }
        }
        if (CALIB || !keep) continue;

        // ---- kept block: fetch V_j now, online softmax, O^T += V_j^T P^T --------------------
        if constexpr (!CALIB) {
            uint4 vst[NST];
            tile_fetch<D, NT, true>(vst, vbase + (int64_t)j * BN * p.vsn, p.vsn, tid);

            const float m_new = fmaxf(m_run, mx * p.scale_log2);
            const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run - m_use);
            m_run = m_new;
            float psum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const float pe = __builtin_amdgcn_exp2f(fmaf(sacc[kb][e], p.scale_log2, -m_use));
                    sacc[kb][e] = pe;
                    psum += pe;
                }
            l_run = l_run * alpha + psum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int x = 0; x < DB; ++x)
#pragma unroll
                    for (int e = 0; e < 16; ++e) oacc[x][e] *= alpha;
            }

            tile_commit<D, NT>(vst, lds_v, tid);
            __syncthreads();

            const int L = lane & 15, g16 = (lane >> 4) & 1;
#pragma unroll
            for (int u = 0; u < 4; ++u) {                 // 16 keys per MFMA k-step
                bf16x8 pb;
#pragma unroll
                for (int e = 0; e < 8; ++e) pb[e] = (__bf16)sacc[u >> 1][8 * (u & 1) + e];
                const int r0 = 16 * u + 4 * hh + (L >> 2);
                const int r1 = r0 + 8;
#pragma unroll
                for (int x = 0; x < DB; ++x) {
                    const int dcol = 32 * x + 16 * g16 + 4 * (L & 3);     // element column
                    const int c = dcol >> 3, half = (dcol >> 2) & 1;
                    const uint16_t *a0 = lds_v + (r0 * CPR + (c ^ swz_v<D>(r0))) * 8 + 4 * half;
                    const uint16_t *a1 = lds_v + (r1 * CPR + (c ^ swz_v<D>(r1))) * 8 + 4 * half;
                    s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a0));
                    s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, a1));
                    s16x8 av = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[x] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, av), pb, oacc[x], 0, 0, 0);
                }
            }
        }
    }

    // ---- statistics ------------------------------------------------------------------------
    if (p.block_max)
        for (int j = n_blk + tid; j < p.mkv; j += NT) p.block_max[stat_row * p.mkv + j] = NAN;
    if (p.skip_mask)
        for (int w = ((n_blk + 31) >> 5) + tid; w < p.mask_words; w += NT) p.skip_mask[stat_row * p.mask_words + w] = 0u;
    if (p.counts && tid == 0) {
        unsigned long long *c = p.counts + ((int64_t)b * p.hq + h) * 3;
        const int gateable = p.causal ? n_gate : (p.mkv - (own_hi - own_lo));
        atomicAdd(c + 0, n_skipped);
        atomicAdd(c + 1, (unsigned long long)gateable);
        atomicAdd(c + 2, (unsigned long long)n_blk);
    }
    if constexpr (CALIB) return;

    // ---- O_i = O~_i / l_i, written as bf16 ----------------------------------------------------
    if constexpr (!CALIB) {
        const float l_tot = l_run + __shfl_xor(l_run, 32);
        const float inv = 1.0f / l_tot;
        uint16_t *op = p.out + (int64_t)b * p.osb + (int64_t)q_row * p.osn + (int64_t)h * p.osh;
#pragma unroll
        for (int x = 0; x < DB; ++x)
#pragma unroll
            for (int e4 = 0; e4 < 4; ++e4) {
                const int d0 = 32 * x + 8 * e4 + 4 * hh;
                typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (__bf16)(oacc[x][4 * e4 + e] * inv);
                *reinterpret_cast<bf16x4 *>(op + d0) = o;
            }
    }
}

__global__ void zero_counts_kernel(unsigned long long *c, int n)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < n) c[t] = 0ull;
}

template <int D, int NW>
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
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NW, true>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, p);
    else
        hipLaunchKernelGGL((bsfa_fwd_kernel<D, NW, false>), dim3((unsigned)grid), dim3(NW * 64), 0, stream, p);
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
#define BSFA_CASE(DD, NN) \
    if (head_dim == DD && block_m == 32 * NN) return launch_t<DD, NN>(p, calib, stream);
    BSFA_CASE(64, 1) BSFA_CASE(64, 2) BSFA_CASE(64, 4)
    BSFA_CASE(128, 1) BSFA_CASE(128, 2) BSFA_CASE(128, 4)
#undef BSFA_CASE
    return hipErrorInvalidValue;
}

}  // namespace bsfa
