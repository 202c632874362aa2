// Per-head order statistics of block maxima on the GPU (the selection half of bsfa_calibrate).
//
// Input: the block-maximum dump of the score kernel, [batch][hq][per_head] floats with NaN where a
// block is not gateable.  For every query head h (all batch elements pooled) and every level l with
// target skip fraction f_l: n = number of non-NaN values, r = floor(f_l * n), result = the value of
// rank r in ascending order (x_r), -inf if r == 0, +inf if r >= n -- the rule of Section 4.2 reduced
// over query positions (the threshold that leaves exactly r blocks below it).
//
// Exact selection by three radix passes over the values' order-preserving 32-bit keys (11 + 11 + 10
// bits): a histogram pass counts, per head, the values whose leading bits equal the prefix found so
// far; a scan pass picks the bin that holds rank r and extends the prefix.  After the third pass the
// prefix is the key of x_r itself.  Up to kLevelsPerRound levels share one sweep over the dump.
#include "bsfa_internal.h"

#include <math.h>

#include <algorithm>

namespace bsfa {

namespace {

constexpr int kBins = 2048;

struct SelState {            // per (level slot, head)
    uint32_t prefix;         // leading key bits found so far
    uint32_t done;           // 0 searching, 1 result is -inf, 2 result is +inf
    unsigned long long rank; // rank of the wanted value among the values that share the prefix
};

// Layout of the selection area: hist0 [hq][kBins] (pass 0, shared by all levels),
// hist [kLevelsPerRound][hq][kBins] (passes 1 and 2), state [kLevelsPerRound][hq].
__host__ __device__ inline size_t hist0_words(int hq) { return (size_t)hq * kBins; }
__host__ __device__ inline size_t hist_words(int hq) { return (size_t)kLevelsPerRound * hq * kBins; }

__device__ __forceinline__ uint32_t ordered_key(float v)
{
    const uint32_t u = __float_as_uint(v);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float key_value(uint32_t k)
{
    return __uint_as_float((k & 0x80000000u) ? (k & 0x7fffffffu) : ~k);
}

__global__ void fill_zero_kernel(uint32_t *p, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Pass 0: per head, histogram of the leading 11 key bits of every value (private copy in LDS,
// flushed with one atomic per non-empty bin).  grid = (chunks, batch * hq).
__global__ void __launch_bounds__(256) hist0_kernel(const float *dump, long per_head, int hq, uint32_t *hist0)
{
    __shared__ uint32_t h[kBins];
    for (int i = threadIdx.x; i < kBins; i += 256) h[i] = 0u;
    __syncthreads();
    const int head = blockIdx.y % hq;
    const float *src = dump + (size_t)blockIdx.y * per_head;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < per_head; i += (long)gridDim.x * 256) {
        const float v = src[i];
        if (v == v) atomicAdd(&h[ordered_key(v) >> 21], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kBins; i += 256)
        if (h[i]) atomicAdd(&hist0[(size_t)head * kBins + i], h[i]);
}

// Passes 1 and 2: values whose leading bits equal a level's prefix are counted by their next bits.
// Few values match (one bin of the previous pass), so they go straight to global atomics.
// PASS 1: prefix = 11 bits, bin = bits 20..10.  PASS 2: prefix = 22 bits, bin = bits 9..0.
template <int PASS>
__global__ void __launch_bounds__(256) histn_kernel(const float *dump, long per_head, int hq, int n_lv,
                                                    const SelState *state, uint32_t *hist)
{
    const int head = blockIdx.y % hq;
    uint32_t pre[kLevelsPerRound];
    bool live[kLevelsPerRound];
    bool any = false;
    for (int l = 0; l < kLevelsPerRound; ++l) {
        live[l] = l < n_lv && state[(size_t)l * hq + head].done == 0u;
        pre[l] = live[l] ? state[(size_t)l * hq + head].prefix : 0u;
        any = any || live[l];
    }
    if (!any) return;
    const float *src = dump + (size_t)blockIdx.y * per_head;
    for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < per_head; i += (long)gridDim.x * 256) {
        const float v = src[i];
        if (!(v == v)) continue;
        const uint32_t key = ordered_key(v);
        const uint32_t lead = PASS == 1 ? key >> 21 : key >> 10;
        const uint32_t bin = PASS == 1 ? (key >> 10) & 2047u : key & 1023u;
#pragma unroll
        for (int l = 0; l < kLevelsPerRound; ++l)
            if (live[l] && lead == pre[l]) atomicAdd(&hist[((size_t)l * hq + head) * kBins + bin], 1u);
    }
}

// Scan: one workgroup per (level slot, head).  PASS 0 also turns the target fraction into a rank.
template <int PASS>
__global__ void __launch_bounds__(256) scan_kernel(const uint32_t *hist_base, int hq, SelectLevels lv, int l0,
                                                   SelState *state, float *out)
{
    __shared__ unsigned long long part[256];
    __shared__ unsigned long long total_s;
    const int l = blockIdx.x, head = blockIdx.y, t = threadIdx.x;
    SelState &st = state[(size_t)l * hq + head];
    const uint32_t *h = hist_base + (PASS == 0 ? (size_t)head * kBins : ((size_t)l * hq + head) * kBins);
    if (PASS != 0 && st.done != 0u) return;           // (uniform over the workgroup)
    uint32_t c[8];
    unsigned long long s = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { c[i] = h[t * 8 + i]; s += c[i]; }
    part[t] = s;
    __syncthreads();
    if (t == 0) {
        unsigned long long run = 0;
        for (int i = 0; i < 256; ++i) { const unsigned long long x = part[i]; part[i] = run; run += x; }
        total_s = run;
    }
    __syncthreads();
    unsigned long long rank;
    if (PASS == 0) {
        const unsigned long long n = total_s;
        const double f = (double)lv.f[l0 + l];
        const double rr = floor(f * (double)n);
        if (rr <= 0.0 || n == 0ull) {
            if (t == 0) { st.done = 1u; out[(size_t)(l0 + l) * hq + head] = -INFINITY; }
            return;
        }
        if (rr >= (double)n) {
            if (t == 0) { st.done = 2u; out[(size_t)(l0 + l) * hq + head] = INFINITY; }
            return;
        }
        rank = (unsigned long long)rr;
    } else {
        rank = st.rank;
    }
    __syncthreads();                                  // every thread has read st.rank before it is rewritten
    unsigned long long before = part[t];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        if (rank >= before && rank < before + c[i]) {         // exactly one bin of one thread
            const uint32_t bin = (uint32_t)(t * 8 + i);
            const uint32_t prefix = PASS == 0 ? bin : PASS == 1 ? (st.prefix << 11) | bin : (st.prefix << 10) | bin;
            st.prefix = prefix;
            st.rank = rank - before;
            if (PASS == 0) st.done = 0u;
            if (PASS == 2) out[(size_t)(l0 + l) * hq + head] = key_value(prefix);
        }
        before += c[i];
    }
}

}  // namespace

size_t select_area_bytes(int hq)
{
    return (hist0_words(hq) + hist_words(hq)) * sizeof(uint32_t) + (size_t)kLevelsPerRound * hq * sizeof(SelState);
}

hipError_t launch_select(const float *dump, long per_head, int batch, int hq, const SelectLevels &lv, int n_levels,
                         void *area, float *out_dev, hipStream_t stream)
{
    if (n_levels < 1 || n_levels > kMaxLevels || hq < 1 || hq > 65535 || batch < 1 || (long)batch * hq > 65535) return hipErrorInvalidValue;
    uint32_t *hist0 = static_cast<uint32_t *>(area);
    uint32_t *hist = hist0 + hist0_words(hq);
    SelState *state = reinterpret_cast<SelState *>(hist + hist_words(hq));
    const int chunks = (int)std::min<long>(64, (per_head + 16383) / 16384);
    const dim3 grid_v((unsigned)std::max(chunks, 1), (unsigned)(batch * hq));
    hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, stream, hist0, hist0_words(hq));
    hipLaunchKernelGGL(hist0_kernel, grid_v, dim3(256), 0, stream, dump, per_head, hq, hist0);
    for (int l0 = 0; l0 < n_levels; l0 += kLevelsPerRound) {
        const int n_lv = std::min(kLevelsPerRound, n_levels - l0);
        const dim3 grid_s((unsigned)n_lv, (unsigned)hq);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, stream, hist, hist_words(hq));
        hipLaunchKernelGGL((scan_kernel<0>), grid_s, dim3(256), 0, stream, hist0, hq, lv, l0, state, out_dev);
        hipLaunchKernelGGL((histn_kernel<1>), grid_v, dim3(256), 0, stream, dump, per_head, hq, n_lv, state, hist);
        hipLaunchKernelGGL((scan_kernel<1>), grid_s, dim3(256), 0, stream, hist, hq, lv, l0, state, out_dev);
        hipLaunchKernelGGL(fill_zero_kernel, dim3(256), dim3(256), 0, stream, hist, hist_words(hq));
        hipLaunchKernelGGL((histn_kernel<2>), grid_v, dim3(256), 0, stream, dump, per_head, hq, n_lv, state, hist);
        hipLaunchKernelGGL((scan_kernel<2>), grid_s, dim3(256), 0, stream, hist, hq, lv, l0, state, out_dev);
    }
    return hipGetLastError();
}

}  // namespace bsfa
