// Internal: types shared by the host side of the library (flashoptim_api.hip) and its
// device code (flashoptim_kernels.hip).  Not part of the public ABI.
#ifndef FLASHOPTIM_DEVICE_H
#define FLASHOPTIM_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fo {

constexpr int kGroup = 32;                         // quantisation group (Algorithms 2, 3)
constexpr int kThreads = 256;                      // lanes per workgroup (codec and copy kernels)
// Launch shape of the step kernels, per optimizer kind (0 AdamW, 1 SGD, 2 Lion): consecutive
// elements per lane and lanes per workgroup.  One workgroup handles one tile of chunk_elems(kind)
// consecutive elements.
#ifndef FO_VEC_ADAMW
#define FO_VEC_ADAMW 8
#endif
#ifndef FO_VEC_SGD_LION
#define FO_VEC_SGD_LION 8
#endif
#ifndef FO_THREADS_ADAMW
#define FO_THREADS_ADAMW 256
#endif
#ifndef FO_THREADS_SGD_LION
#define FO_THREADS_SGD_LION 512
#endif
constexpr int step_vec(int kind) { return kind == 0 ? FO_VEC_ADAMW : FO_VEC_SGD_LION; }
constexpr int step_threads(int kind) { return kind == 0 ? FO_THREADS_ADAMW : FO_THREADS_SGD_LION; }
constexpr int chunk_elems(int kind) { return step_threads(kind) * step_vec(kind); }
#ifndef FO_COPY_CHUNK_KB
#define FO_COPY_CHUNK_KB 128
#endif
constexpr int kCopyChunkBytes = FO_COPY_CHUNK_KB * 1024;   // checkpoint copy: bytes per workgroup

// One tensor as the kernels see it (device pointers), 104 bytes.
struct TensorDev {
    void* param;
    int8_t* rho;
    const void* grad;
    int8_t* m_q;
    uint16_t* m_scale;
    uint8_t* v_q;
    uint16_t* v_scale;
    float* theta32;   // ablation variants: FP32 master weight (weights not split)
    float* m32;       // ablation variants: FP32 momentum (states not quantized)
    float* v32;       // ablation variants: FP32 variance
    int64_t numel;
    float lr, wd;
    uint32_t first_tile;   // multi-tensor launch: index of the workgroup that handles the tensor's first tile
    uint32_t n_tiles;      // multi-tensor launch: number of tiles (workgroups) of the tensor
};

// Per-call scalars, computed once on the host.
// Operand range of the short divisions of the AdamW kernels (numerator, denominator and eps inside it).
constexpr float kDivFastLo = 8.673617379884035e-19f;    // 2^-60
constexpr float kDivFastHi = 1.152921504606847e18f;     // 2^60

struct StepConsts {
    float beta1, beta2;   // AdamW/Lion betas; SGD: beta1 = momentum
    float omb1, omb2;     // 1.0f - beta (FP32 subtraction)
    float rbc1, rbc2;     // 1.0f / (float)(1 - beta^t), AdamW only
    float eps;
    float k255_hi, k255_lo;   // 255 * sqrt(1 / rbc2) in double, as two floats: used only to pre-estimate variance codes
    float v_max, m_max;   // largest v_t and |m_t| for which the short square root and division serve: 2^60 / rbc2 and
                          // 2^60 / rbc1 rounded down, or -1 when eps is outside [2^-60, 1] (the kernels then use
                          // sqrtf and the IEEE division throughout)
    float sqrt_min;       // smallest v_t for the same: 2^-96, or +inf while the short square root has not passed its
                          // check on this device; the step kernels fill it in from StepArgs::sqrt_min_word
};

// A multi-tensor launch maps workgroup b to (tensor, tile) in two steps: coarse[b >> coarse_shift] is
// the tensor that holds tile (b >> coarse_shift) << coarse_shift, and the tensors' first_tile /
// n_tiles fields carry the search on from there (usually zero further steps).  Both tables are
// small (at most 16 K coarse entries) and stay cache-resident, unlike a table with one entry per
// workgroup, whose entries every workgroup would fetch from HBM.
constexpr int kCoarseMaxEntries = 16384;
// One logical launch is issued as consecutive launches that cover at most this many elements each.
// Measured on the Llama list (8.03 G parameters): the memory-bound SGD and Lion steps run 3-9 % faster
// in ~30-60 launches than in one launch of 1.96 M workgroups (12.9-13.0 vs 13.4-14.0 ms); AdamW gains
// under 1 % and loses with segments below 64 M elements; below ~25 K workgroups per launch the gaps
// between launches take the gain back.
#ifndef FO_SEGMENT_ELEMS
#define FO_SEGMENT_ELEMS (1 << 28)
#endif
constexpr int64_t kSegmentElems = FO_SEGMENT_ELEMS;
struct StepArgs {
    const TensorDev* tensors;   // device table (multi-tensor launch)
    const uint32_t* coarse;     // device table: tensor index per 2^coarse_shift workgroups
    uint32_t coarse_shift;
    uint32_t n_tensors;
    uint32_t block_offset;      // tile index of this launch's workgroup 0 (a list or tensor is covered by several launches)
    TensorDev single;           // the one tensor of a direct launch
    StepConsts c;
    const float* sqrt_min_word; // AdamW steps: device word that holds StepConsts::sqrt_min for this device
};

struct CopySegment {
    const uint8_t* src;
    uint8_t* dst;
    int64_t bytes;       // bytes to copy
    int64_t pad_bytes;   // >= bytes; [bytes, pad_bytes) of dst is zero-filled
};

hipError_t launch_step(int kind, bool direct, bool split, bool quant, bool exact, const StepArgs& a, int64_t n_blocks,
                       hipStream_t s);
constexpr int kConvChunkElems = 256 * 8;   // elements per workgroup of the layout-conversion kernel
hipError_t launch_convert(bool has_v, bool compress, bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s);
hipError_t launch_probe(int kind, bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s);
void launch_split(int bits, const float* theta, void* param, void* rho, int64_t n, hipStream_t s);
void launch_reconstruct(int bits, const void* param, const void* rho, float* theta, int64_t n, hipStream_t s);
constexpr int kSweepStats = 8 + 3 * 256;
hipError_t launch_clock_monitor(unsigned long long* samples, int n_samples, unsigned long long ticks_per_sample,
                                hipStream_t s);
hipError_t launch_sweep(int bits, bool directional, uint64_t first, uint64_t stride, uint64_t count, double* stats,
                        hipStream_t s);
void launch_quantize(bool variance, bool linear, const float* x, void* q, uint16_t* scale, int64_t n, hipStream_t s);
void launch_dequantize(bool variance, bool linear, const void* q, const uint16_t* scale, float* x, int64_t n,
                       hipStream_t s);
void launch_nmse(bool variance, bool linear, const float* x, int64_t n, double* sums, hipStream_t s);
void launch_copy(const CopySegment* segs, const uint2* chunks, int64_t n_chunks, hipStream_t s);
constexpr int kSelftestSectionCount = 7;
constexpr unsigned long long kSelftestSqrtValues = 0x7f800000ull - 0x0f800000ull;   // section 2: every FP32 value in [2^-96, FLT_MAX]
constexpr int kSelftestCounters = 15;   // two per section, then the inexact count of section 6
// Section 4 (variance codes) runs once per (beta2, step, group scale): steps 1..20, then 50, 100, 200, 500, ... 10^6.
constexpr int kSelftestVarSteps = 34;
constexpr int64_t selftest_var_step(int i) {
    if (i < 20) return i + 1;
    const int j = i - 20;                        // 50, 100, 200, 500, 1000, ... (j = 0 .. 13)
    const int64_t lead[3] = {5, 10, 20};
    int64_t p = 10;
    for (int k = 0; k < j / 3; ++k) p *= 10;
    return lead[j % 3] * p;
}
static_assert(selftest_var_step(19) == 20 && selftest_var_step(20) == 50 && selftest_var_step(21) == 100 &&
              selftest_var_step(22) == 200 && selftest_var_step(33) == 1000000, "");
hipError_t launch_selftest(unsigned long long* counters, int section, const StepConsts& c, float scale_r,
                           hipStream_t s);

}  // namespace fo
#endif
