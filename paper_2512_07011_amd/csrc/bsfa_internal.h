// Internal declarations shared by the translation units of libbsfa.so (not part of the ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace bsfa {

// Key/value block rows; the library is built for B_N = 64 only.
constexpr int kBlockN = 64;

struct FwdParams {
    const uint16_t *q, *k, *v;       // bf16 or fp16 bit patterns (f16 says which)
    uint16_t *out;
    uint16_t *vt;                    // workspace for the transposed V tiles ([batch][hkv][mkv] tiles of 64 x head_dim
                                     // elements), or null: V is then gathered with transposing LDS reads
    const float *tau;                // [hq] or [hq][tau_tiles]
    uint8_t *k8;                     // workspace for K as fp8 tiles ([batch][hkv][mkv] tiles of 64 x 128 bytes), or null:
                                     // the score product then runs on the 16-bit elements
    const int32_t *seqlens;          // [batch] tokens per batch element, or null (all have seqlen)
    int64_t qsb, qsn, qsh, ksb, ksn, ksh, vsb, vsn, vsh, osb, osn, osh;
    int batch, hq, hkv, group, seqlen, mq, mkv;
    int causal, tau_per_tile, tau_tiles;
    int f16;                         // element type of q, k, v, out: 0 bf16, 1 fp16
    int single_head;                 // 1: never pair the heads of a GQA group in one workgroup
    int gate_mode;                   // 0: block maximum vs threshold; 1: running-maximum predicate (general stages only)
    float scale;                     // 1/sqrt(d): natural score units, used by the gate
    float scale_log2;                // log2(e)/sqrt(d): softmax evaluated with exp2
    unsigned long long *counts;      // [batch][hq][3] or null
    uint32_t *skip_mask;             // [batch][hq][mq][mask_words] or null
    float *block_max;                // [batch][hq][mq][mkv] or null
    float *lse;                      // [batch][seqlen][hq] or null
    int mask_words;
};

// Launches the forward kernel (calib == false) or its score/block-maximum half only
// (calib == true: no V, no softmax, no output; block_max must be non-null).
// Returns hipSuccess or the launch error; hipErrorInvalidValue for an unsupported
// (head_dim, block_m) pair.
hipError_t launch_forward(const FwdParams &p, int head_dim, int block_m, bool calib, hipStream_t stream);

bool shape_supported(int head_dim, int block_m, int block_n);

// ---- order statistics of the block maxima on the GPU (bsfa_select.hip) ------------------------
constexpr int kMaxLevels = 64;        // target skip fractions per calibration call
constexpr int kLevelsPerRound = 8;    // levels that share one sweep over the block-maximum dump
struct SelectLevels {
    float f[kMaxLevels];              // target skip fractions, passed to the kernels by value
};
// Bytes of the histogram / state area launch_select needs for hq query heads (multiple of 16).
size_t select_area_bytes(int hq);
// dump: DEVICE [batch][hq][per_head] block maxima, NaN = not gateable.  out_dev: DEVICE
// [n_levels][hq]: per head (batch elements pooled) the order statistic x_r, r = floor(f * n), of its
// n non-NaN values, -inf if r == 0, +inf if r >= n.  area: DEVICE, select_area_bytes(hq) bytes,
// 16-byte aligned; it is cleared by the launch.  Enqueues on stream; no host synchronisation.
hipError_t launch_select(const float *dump, long per_head, int batch, int hq, const SelectLevels &lv, int n_levels,
                         void *area, float *out_dev, hipStream_t stream);

// ---- matrix-instruction rate probe (bsfa_probe.hip) --------------------------------------------
constexpr int kProbeThreads = 512;        // 8 waves per workgroup: two per SIMD, as the forward kernel runs
constexpr int kProbeMfmaPerIter = 16;     // 32x32x16 MFMAs per wave and iteration
// operands: DEVICE, 4096 floats; sink: DEVICE, workgroups * kProbeThreads floats.  Enqueues one kernel.
hipError_t launch_mfma_rate_probe(const float *operands, float *sink, int workgroups, int iters, hipStream_t stream);

}  // namespace bsfa
