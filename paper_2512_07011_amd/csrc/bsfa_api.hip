// C ABI of libbsfa.so: argument validation, launch set-up, calibration driver, error strings.
#include "../../include/bsfa.h"
#include "bsfa_internal.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <functional>
#include <mutex>
#include <vector>

namespace {

thread_local char g_err[512] = "";

bsfa_status fail(bsfa_status s, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return s;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

bsfa_status check_problem(const bsfa_problem *p, int causal)
{
    if (!p) return fail(BSFA_ERR_NULL, "problem descriptor is NULL");
    if (p->dtype != BSFA_BF16 && p->dtype != BSFA_FP16) return fail(BSFA_ERR_DTYPE, "dtype %d not supported (bf16 and fp16 only)", p->dtype);
    if (p->batch < 1 || p->n_q_heads < 1 || p->n_kv_heads < 1 || p->seqlen < 1 || p->head_dim < 1)
        return fail(BSFA_ERR_SHAPE, "batch, head counts, seqlen and head_dim must be positive");
    if (p->n_q_heads % p->n_kv_heads)
        return fail(BSFA_ERR_SHAPE, "n_q_heads (%d) is not a multiple of n_kv_heads (%d)", p->n_q_heads, p->n_kv_heads);
    if (p->block_m < 1 || p->block_n < 1)
        return fail(BSFA_ERR_SHAPE, "block_m and block_n must be positive");
    if (!bsfa::shape_supported(p->head_dim, p->block_m, p->block_n))
        return fail(BSFA_ERR_UNSUPPORTED, "head_dim %d with tile %dx%d is not built (see bsfa_query_build)",
                    p->head_dim, p->block_m, p->block_n);
    if (!causal && (p->seqlen % p->block_m || p->seqlen % p->block_n))
        return fail(BSFA_ERR_SHAPE, "seqlen %d is not a multiple of block_m %d and block_n %d (required without the causal mask)",
                    p->seqlen, p->block_m, p->block_n);
    if (!causal && p->seqlens) return fail(BSFA_ERR_SHAPE, "per-element sequence lengths need the causal mask");
    if (p->seqlens && (reinterpret_cast<uintptr_t>(p->seqlens) & 3u)) return fail(BSFA_ERR_SHAPE, "seqlens must be 4-byte aligned");
    const int64_t st[12] = {p->q_stride_b, p->q_stride_n, p->q_stride_h, p->k_stride_b, p->k_stride_n, p->k_stride_h,
                            p->v_stride_b, p->v_stride_n, p->v_stride_h, p->o_stride_b, p->o_stride_n, p->o_stride_h};
    for (int x = 0; x < 12; ++x) {
        if (st[x] < 0 || st[x] % 8) return fail(BSFA_ERR_SHAPE, "stride #%d = %lld must be a non-negative multiple of 8 elements", x, (long long)st[x]);
        if (x % 3 != 0 && st[x] < p->head_dim) return fail(BSFA_ERR_SHAPE, "token/head stride #%d = %lld is smaller than head_dim", x, (long long)st[x]);
    }
    if (p->thresholds_per_tile != 0 && p->thresholds_per_tile != 1)
        return fail(BSFA_ERR_SHAPE, "thresholds_per_tile must be 0 or 1");
    if (p->threshold_tiles < 0) return fail(BSFA_ERR_SHAPE, "threshold_tiles must not be negative");
    if (p->single_head_groups != 0 && p->single_head_groups != 1) return fail(BSFA_ERR_SHAPE, "single_head_groups must be 0 or 1");
    if (p->workspace_bytes < 0) return fail(BSFA_ERR_WORKSPACE, "workspace_bytes must not be negative");
    if (p->gate_mode != 0 && p->gate_mode != 1) return fail(BSFA_ERR_SHAPE, "gate_mode must be 0 or 1");
    if (p->qk_fp8 != 0 && p->qk_fp8 != 1) return fail(BSFA_ERR_SHAPE, "qk_fp8 must be 0 or 1");
    if (p->qk_fp8 && (p->head_dim != 128 || p->block_m != 128))
        return fail(BSFA_ERR_UNSUPPORTED, "qk_fp8 needs head_dim 128 and block_m 128");
    return BSFA_OK;
}

// bytes of the fp8 copy of K: [batch][n_kv_heads][M_KV] tiles of block_n x head_dim bytes
size_t k8_bytes(const bsfa_problem *p)
{
    const size_t mkv = (size_t)((p->seqlen + p->block_n - 1) / p->block_n);
    return (size_t)p->batch * p->n_kv_heads * mkv * (size_t)p->block_n * p->head_dim;
}

void fill_params(bsfa::FwdParams &fp, const bsfa_problem *p, int causal)
{
    memset(&fp, 0, sizeof(fp));
    fp.qsb = p->q_stride_b; fp.qsn = p->q_stride_n; fp.qsh = p->q_stride_h;
    fp.ksb = p->k_stride_b; fp.ksn = p->k_stride_n; fp.ksh = p->k_stride_h;
    fp.vsb = p->v_stride_b; fp.vsn = p->v_stride_n; fp.vsh = p->v_stride_h;
    fp.osb = p->o_stride_b; fp.osn = p->o_stride_n; fp.osh = p->o_stride_h;
    fp.batch = p->batch; fp.hq = p->n_q_heads; fp.hkv = p->n_kv_heads;
    fp.group = p->n_q_heads / p->n_kv_heads;
    fp.seqlen = p->seqlen;
    fp.mq = (p->seqlen + p->block_m - 1) / p->block_m;
    fp.mkv = (p->seqlen + p->block_n - 1) / p->block_n;
    fp.seqlens = p->seqlens;
    fp.tau_tiles = p->threshold_tiles > 0 ? p->threshold_tiles : fp.mq;
    fp.mask_words = (fp.mkv + 31) / 32;
    fp.causal = causal ? 1 : 0;
    fp.f16 = (p->dtype == BSFA_FP16) ? 1 : 0;
    fp.single_head = p->single_head_groups ? 1 : 0;
    fp.gate_mode = p->gate_mode;
    fp.tau_per_tile = p->thresholds_per_tile;
    fp.scale = 1.0f / sqrtf((float)p->head_dim);
    fp.scale_log2 = (float)(1.4426950408889634 / sqrt((double)p->head_dim));
}

}  // namespace

extern "C" {

bsfa_status bsfa_forward(const bsfa_problem *p, const void *q, const void *k, const void *v,
                         const float *thresholds, int causal, void *out,
                         const bsfa_skip_stats *skip_stats, void *hip_stream)
{
    bsfa_status s = check_problem(p, causal);
    if (s != BSFA_OK) return s;
    if (!q || !k || !v || !thresholds || !out) return fail(BSFA_ERR_NULL, "q, k, v, thresholds and out must be non-NULL");
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out))
        return fail(BSFA_ERR_SHAPE, "q, k, v and out must be 16-byte aligned");
    bsfa::FwdParams fp;
    fill_params(fp, p, causal);
    fp.q = static_cast<const uint16_t *>(q);
    fp.k = static_cast<const uint16_t *>(k);
    fp.v = static_cast<const uint16_t *>(v);
    fp.out = static_cast<uint16_t *>(out);
    fp.tau = thresholds;
    if (p->workspace) {
        const size_t need = bsfa_forward_workspace_bytes(p);
        if (need) {                   // (tile shapes that take V in place ignore the workspace)
            if ((size_t)p->workspace_bytes < need)
                return fail(BSFA_ERR_WORKSPACE, "forward workspace of %zu bytes needed, %lld given", need, (long long)p->workspace_bytes);
            fp.vt = reinterpret_cast<uint16_t *>((reinterpret_cast<uintptr_t>(p->workspace) + 255) & ~(uintptr_t)255);
            if (p->qk_fp8) fp.k8 = reinterpret_cast<uint8_t *>((reinterpret_cast<uintptr_t>(fp.vt) + 2 * k8_bytes(p) + 255) & ~(uintptr_t)255);
        }
    }
    if (p->qk_fp8 && !fp.k8) return fail(BSFA_ERR_WORKSPACE, "qk_fp8 needs the forward workspace (bsfa_forward_workspace_bytes)");
    if (skip_stats) {
        fp.counts = reinterpret_cast<unsigned long long *>(skip_stats->counts);
        fp.skip_mask = skip_stats->skip_mask;
        fp.block_max = skip_stats->block_max;
        fp.lse = skip_stats->lse;
    }
    hipError_t e = bsfa::launch_forward(fp, p->head_dim, p->block_m, false, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "forward launch failed: %s", hipGetErrorString(e));
    return BSFA_OK;
}

size_t bsfa_forward_workspace_bytes(const bsfa_problem *p)
{
    if (check_problem(p, 1) != BSFA_OK || p->block_m != 128) return 0;
    // transposed V tiles | fp8 K tiles (if asked for), each 256-byte aligned
    return 2 * k8_bytes(p) + 256 + (p->qk_fp8 ? k8_bytes(p) + 256 : 0);
}

size_t bsfa_calibrate_workspace_bytes(const bsfa_problem *p)
{
    if (check_problem(p, 1) != BSFA_OK) return 0;
    const size_t mq = (size_t)((p->seqlen + p->block_m - 1) / p->block_m), mkv = (size_t)((p->seqlen + p->block_n - 1) / p->block_n);
    const size_t dump = (size_t)p->batch * p->n_q_heads * mq * mkv * sizeof(float);
    // block-maximum dump | selection area | per-level results, each 256-byte aligned
    return dump + bsfa::select_area_bytes(p->n_q_heads) + (size_t)bsfa::kMaxLevels * p->n_q_heads * sizeof(float) + 4 * 256
           + (p->qk_fp8 ? k8_bytes(p) + 256 : 0);           // ... | fp8 K tiles
}

// Shared front half of the calibration entry points: checks, score / block-maximum kernel,
// copy of the [batch][hq][mq][mkv] block maxima (NaN where not gateable) to the host.
static bsfa_status block_maxima_to_host(const bsfa_problem *p, const void *q, const void *k, int causal,
                                        void *workspace, size_t workspace_bytes, void *hip_stream,
                                        std::vector<float> &host, bsfa::FwdParams &fp)
{
    if (!aligned16(q) || !aligned16(k)) return fail(BSFA_ERR_SHAPE, "q and k must be 16-byte aligned");
    const size_t need = bsfa_calibrate_workspace_bytes(p);
    if (!workspace || workspace_bytes < need)
        return fail(BSFA_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    fill_params(fp, p, causal);
    fp.q = static_cast<const uint16_t *>(q);
    fp.k = static_cast<const uint16_t *>(k);
    fp.block_max = reinterpret_cast<float *>((reinterpret_cast<uintptr_t>(workspace) + 255) & ~(uintptr_t)255);
    fp.tau = nullptr;                 // the score half takes no decisions and reads no thresholds
    fp.tau_per_tile = 0;
    fp.tau_tiles = 1;
    hipError_t e = bsfa::launch_forward(fp, p->head_dim, p->block_m, true, stream);
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "calibration launch failed: %s", hipGetErrorString(e));
    host.resize((size_t)p->batch * p->n_q_heads * fp.mq * fp.mkv);
    e = hipMemcpyAsync(host.data(), fp.block_max, host.size() * sizeof(float), hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "calibration copy failed: %s", hipGetErrorString(e));
    return BSFA_OK;
}

// Shared body of the per-head calibration entry points: argument checks, the score / block-maximum
// kernel into `dump`, the order statistics on the GPU into out_dev.  Everything is enqueued on the
// stream; nothing is allocated and the host does not wait.
static bsfa_status calibrate_on_device(const bsfa_problem *p, const void *q, const void *k, int causal,
                                       const float *target_skip_fractions, int n_levels,
                                       float *dump, void *area, float *out_dev, uint8_t *k8, hipStream_t stream)
{
    if (p->thresholds_per_tile) return fail(BSFA_ERR_UNSUPPORTED, "per-head calibration produces per-head thresholds only");
    if (p->gate_mode) return fail(BSFA_ERR_UNSUPPORTED, "calibration is defined for the block-maximum gate (gate_mode 0) only");
    if (!q || !k || !target_skip_fractions) return fail(BSFA_ERR_NULL, "q, k and fractions must be non-NULL");
    if (!aligned16(q) || !aligned16(k)) return fail(BSFA_ERR_SHAPE, "q and k must be 16-byte aligned");
    if (n_levels < 1 || n_levels > bsfa::kMaxLevels) return fail(BSFA_ERR_SHAPE, "n_levels must be between 1 and %d", bsfa::kMaxLevels);
    bsfa::SelectLevels lv;
    memset(&lv, 0, sizeof(lv));
    for (int l = 0; l < n_levels; ++l) {
        if (!(target_skip_fractions[l] >= 0.f && target_skip_fractions[l] <= 1.f))
            return fail(BSFA_ERR_SHAPE, "target skip fraction #%d = %g is outside [0, 1]", l, (double)target_skip_fractions[l]);
        lv.f[l] = target_skip_fractions[l];
    }
    if ((long)p->batch * p->n_q_heads > 65535) return fail(BSFA_ERR_UNSUPPORTED, "batch * n_q_heads must not exceed 65535 for calibration");
    bsfa::FwdParams fp;
    fill_params(fp, p, causal);
    fp.q = static_cast<const uint16_t *>(q);
    fp.k = static_cast<const uint16_t *>(k);
    fp.block_max = dump;
    fp.k8 = k8;
    fp.tau = nullptr;                 // the score half takes no decisions and reads no thresholds
    fp.tau_per_tile = 0;
    fp.tau_tiles = 1;
    hipError_t e = bsfa::launch_forward(fp, p->head_dim, p->block_m, true, stream);
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "calibration launch failed: %s", hipGetErrorString(e));
    e = bsfa::launch_select(dump, (long)fp.mq * fp.mkv, p->batch, p->n_q_heads, lv, n_levels, area, out_dev, stream);
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "selection launch failed: %s", hipGetErrorString(e));
    return BSFA_OK;
}

static uintptr_t up256(uintptr_t x) { return (x + 255) & ~(uintptr_t)255; }

bsfa_status bsfa_calibrate(const bsfa_problem *p, const void *q, const void *k, int causal,
                           const float *target_skip_fractions, int n_levels, float *thresholds_out,
                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    bsfa_status s = check_problem(p, causal);
    if (s != BSFA_OK) return s;
    if (!thresholds_out) return fail(BSFA_ERR_NULL, "thresholds_out must be non-NULL");
    const size_t need = bsfa_calibrate_workspace_bytes(p);
    if (!workspace || workspace_bytes < need)
        return fail(BSFA_ERR_WORKSPACE, "workspace of %zu bytes needed, %zu given", need, workspace ? workspace_bytes : (size_t)0);
    const size_t mq = (size_t)((p->seqlen + p->block_m - 1) / p->block_m), mkv = (size_t)((p->seqlen + p->block_n - 1) / p->block_n);
    const uintptr_t dump = up256(reinterpret_cast<uintptr_t>(workspace));
    const uintptr_t area = up256(dump + (size_t)p->batch * p->n_q_heads * mq * mkv * sizeof(float));
    const uintptr_t outd = up256(area + bsfa::select_area_bytes(p->n_q_heads));
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const uintptr_t k8 = up256(outd + (size_t)bsfa::kMaxLevels * p->n_q_heads * sizeof(float));
    s = calibrate_on_device(p, q, k, causal, target_skip_fractions, n_levels, reinterpret_cast<float *>(dump),
                            reinterpret_cast<void *>(area), reinterpret_cast<float *>(outd),
                            p->qk_fp8 ? reinterpret_cast<uint8_t *>(k8) : nullptr, stream);
    if (s != BSFA_OK) return s;
    // only n_levels x n_q_heads floats travel to the host
    hipError_t e = hipMemcpyAsync(thresholds_out, reinterpret_cast<const void *>(outd), (size_t)n_levels * p->n_q_heads * sizeof(float),
                                  hipMemcpyDeviceToHost, stream);
    if (e == hipSuccess) e = hipStreamSynchronize(stream);
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "calibration copy failed: %s", hipGetErrorString(e));
    return BSFA_OK;
}

// ---- calibration without any allocation -----------------------------------------------------------
// Scratch memory of bsfa_calibrate_noalloc: the block-maximum dump, the selection area and nothing
// else, in a file-scope device array that every GPU the library runs on holds until the process
// ends.  In host code the array's name is only a handle: its device address is looked up once per
// device (with that device current) and the kernels get that address, never the name.
constexpr size_t kScratchDumpBytes = (size_t)16 << 20;          // block maxima: 4 Mi values
constexpr int kScratchMaxHeads = 64;                            // n_q_heads the selection area is sized for
constexpr size_t kScratchAreaBytes = ((size_t)(1 + bsfa::kLevelsPerRound) * kScratchMaxHeads * 2048 * 4
                                      + (size_t)bsfa::kLevelsPerRound * kScratchMaxHeads * 16 + 255) & ~(size_t)255;
constexpr size_t kScratchBytes = kScratchDumpBytes + kScratchAreaBytes;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];

constexpr int kMaxDevices = 64;
static void *g_scratch_ptr[kMaxDevices];                        // device address of `scratch`, per device
static std::mutex g_scratch_mutex;

// Device address of this device's copy of the scratch array (looked up on first use), or null with
// the error recorded.
static unsigned char *scratch_address()
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) {
        fail(BSFA_ERR_HIP, "cannot identify the current device (%s)", e == hipSuccess ? "index out of range" : hipGetErrorString(e));
        return nullptr;
    }
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr) {
            fail(BSFA_ERR_HIP, "scratch array address lookup failed: %s", hipGetErrorString(e));
            return nullptr;
        }
        g_scratch_ptr[dev] = ptr;
    }
    return static_cast<unsigned char *>(g_scratch_ptr[dev]);
}

size_t bsfa_calibrate_noalloc_max_values(void) { return kScratchDumpBytes / sizeof(float); }

bsfa_status bsfa_calibrate_noalloc(const bsfa_problem *p, const void *q, const void *k, int causal,
                                   const float *target_skip_fractions, int n_levels,
                                   float *thresholds_out_device, void *hip_stream)
{
    bsfa_status s = check_problem(p, causal);
    if (s != BSFA_OK) return s;
    if (!thresholds_out_device) return fail(BSFA_ERR_NULL, "thresholds_out_device must be non-NULL");
    const size_t mq = (size_t)((p->seqlen + p->block_m - 1) / p->block_m), mkv = (size_t)((p->seqlen + p->block_n - 1) / p->block_n);
    const size_t values = (size_t)p->batch * p->n_q_heads * mq * mkv;
    if (values * sizeof(float) > kScratchDumpBytes)
        return fail(BSFA_ERR_WORKSPACE, "batch * n_q_heads * M_Q * M_KV = %zu block maxima exceed the %zu the built-in scratch array holds "
                                        "(use bsfa_calibrate with a workspace)", values, kScratchDumpBytes / sizeof(float));
    if (p->n_q_heads > kScratchMaxHeads)
        return fail(BSFA_ERR_WORKSPACE, "n_q_heads = %d exceeds the %d the built-in scratch array is sized for", p->n_q_heads, kScratchMaxHeads);
    if (p->qk_fp8) return fail(BSFA_ERR_UNSUPPORTED, "qk_fp8 is not available without a workspace (use bsfa_calibrate)");
    unsigned char *base = scratch_address();
    if (!base) return BSFA_ERR_HIP;
    return calibrate_on_device(p, q, k, causal, target_skip_fractions, n_levels, reinterpret_cast<float *>(base),
                               base + kScratchDumpBytes, thresholds_out_device, nullptr, static_cast<hipStream_t>(hip_stream));
}

bsfa_status bsfa_calibrate_topk(const bsfa_problem *p, const void *q, const void *k, int causal,
                                const int32_t *ks, int n_levels, int samples_done, float *thresholds_out,
                                void *workspace, size_t workspace_bytes, void *hip_stream)
{
    bsfa_status s = check_problem(p, causal);
    if (s != BSFA_OK) return s;
    if (p->seqlens) return fail(BSFA_ERR_UNSUPPORTED, "bsfa_calibrate_topk takes samples of one length (seqlens must be NULL)");
    if (p->gate_mode) return fail(BSFA_ERR_UNSUPPORTED, "calibration is defined for the block-maximum gate (gate_mode 0) only");
    if (p->qk_fp8) return fail(BSFA_ERR_UNSUPPORTED, "bsfa_calibrate_topk runs the 16-bit score product only (qk_fp8 must be 0)");
    if (!q || !k || !ks || !thresholds_out) return fail(BSFA_ERR_NULL, "q, k, ks and thresholds_out must be non-NULL");
    if (n_levels < 1) return fail(BSFA_ERR_SHAPE, "n_levels must be positive");
    if (samples_done < 0) return fail(BSFA_ERR_SHAPE, "samples_done must be non-negative");
    for (int l = 0; l < n_levels; ++l)
        if (ks[l] < 0) return fail(BSFA_ERR_SHAPE, "k #%d = %d is negative", l, ks[l]);
    std::vector<float> host;
    bsfa::FwdParams fp;
    s = block_maxima_to_host(p, q, k, causal, workspace, workspace_bytes, hip_stream, host, fp);
    if (s != BSFA_OK) return s;

    // per (head, query tile): k-th largest gateable block maximum of each sample (= batch element),
    // folded into the running mean over samples
    const size_t mq = (size_t)fp.mq, mkv = (size_t)fp.mkv;
    std::vector<float> vals;
    for (int b = 0; b < p->batch; ++b) {
        const double done = (double)samples_done + b;
        for (int h = 0; h < p->n_q_heads; ++h)
            for (size_t i = 0; i < mq; ++i) {
                const float *src = host.data() + (((size_t)b * p->n_q_heads + h) * mq + i) * mkv;
                vals.clear();
                for (size_t x = 0; x < mkv; ++x)
                    if (!std::isnan(src[x])) vals.push_back(src[x]);
                const size_t avail = vals.size();
                for (int l = 0; l < n_levels; ++l) {
                    const size_t kk = (size_t)ks[l];
                    float t;
                    if (avail <= kk) t = -INFINITY;               // keeps min(k, A) = A blocks
                    else if (kk == 0) t = INFINITY;
                    else {
                        std::nth_element(vals.begin(), vals.begin() + (kk - 1), vals.end(), std::greater<float>());
                        t = vals[kk - 1];
                    }
                    float &dst = thresholds_out[((size_t)l * p->n_q_heads + h) * mq + i];
                    if (done == 0.0 || std::isinf(t)) dst = t;
                    else dst = (float)(((double)dst * done + (double)t) / (done + 1.0));
                }
            }
    }
    return BSFA_OK;
}

int bsfa_query_build(int32_t *block_m, int32_t *block_n, int32_t *head_dim, int cap)
{
    static const int bm[3] = {32, 64, 128};
    static const int hd[2] = {64, 128};
    int n = 0;
    for (int d = 0; d < 2; ++d)
        for (int m = 0; m < 3; ++m) {
            if (n < cap) {
                if (block_m) block_m[n] = bm[m];
                if (block_n) block_n[n] = bsfa::kBlockN;
                if (head_dim) head_dim[n] = hd[d];
            }
            ++n;
        }
    return n;
}

const char *bsfa_status_string(bsfa_status s)
{
    switch (s) {
    case BSFA_OK: return "BSFA_OK";
    case BSFA_ERR_NULL: return "BSFA_ERR_NULL";
    case BSFA_ERR_SHAPE: return "BSFA_ERR_SHAPE";
    case BSFA_ERR_DTYPE: return "BSFA_ERR_DTYPE";
    case BSFA_ERR_UNSUPPORTED: return "BSFA_ERR_UNSUPPORTED";
    case BSFA_ERR_WORKSPACE: return "BSFA_ERR_WORKSPACE";
    case BSFA_ERR_HIP: return "BSFA_ERR_HIP";
    }
    return "BSFA_ERR_UNKNOWN";
}

const char *bsfa_last_error(void) { return g_err; }

size_t bsfa_mfma_rate_probe_sink_bytes(int workgroups)
{
    return workgroups > 0 ? (size_t)workgroups * bsfa::kProbeThreads * sizeof(float) : 0;
}

double bsfa_mfma_rate_probe_flops(int workgroups, int iters)
{
    if (workgroups <= 0 || iters <= 0) return 0.0;
    return (double)workgroups * (bsfa::kProbeThreads / 64) * (double)iters * bsfa::kProbeMfmaPerIter * (2.0 * 32 * 32 * 16);
}

bsfa_status bsfa_mfma_rate_probe(const float *operands, float *sink, size_t sink_bytes, int workgroups, int iters,
                                 void *hip_stream)
{
    if (!operands || !sink) return fail(BSFA_ERR_NULL, "bsfa_mfma_rate_probe: operands and sink are required");
    if (workgroups <= 0 || iters <= 0 || workgroups > (1 << 20))
        return fail(BSFA_ERR_SHAPE, "bsfa_mfma_rate_probe: workgroups in [1, 2^20] and iters > 0 expected");
    if (sink_bytes < bsfa_mfma_rate_probe_sink_bytes(workgroups))
        return fail(BSFA_ERR_WORKSPACE, "bsfa_mfma_rate_probe: sink holds %zu bytes, %zu needed", sink_bytes,
                    bsfa_mfma_rate_probe_sink_bytes(workgroups));
    const hipError_t e = bsfa::launch_mfma_rate_probe(operands, sink, workgroups, iters, static_cast<hipStream_t>(hip_stream));
    if (e != hipSuccess) return fail(BSFA_ERR_HIP, "bsfa_mfma_rate_probe: %s", hipGetErrorString(e));
    return BSFA_OK;
}

}  // extern "C"
