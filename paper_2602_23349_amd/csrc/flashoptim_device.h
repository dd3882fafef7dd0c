// Internal: types shared by the host side of the library (flashoptim_api.hip) and its
// device code (flashoptim_kernels.hip).  Not part of the public ABI.
#ifndef FLASHOPTIM_DEVICE_H
#define FLASHOPTIM_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace fo {

constexpr int kGroup = 32;                         // quantisation group (Algorithms 2, 3)
constexpr int kThreads = 256;                      // lanes per workgroup
#ifndef FO_VEC_ADAMW
#define FO_VEC_ADAMW 8
#endif
#ifndef FO_VEC_SGD_LION
#define FO_VEC_SGD_LION 8
#endif
constexpr int kVecAdamW = FO_VEC_ADAMW;            // consecutive elements per lane, AdamW kernel
constexpr int kVecSgdLion = FO_VEC_SGD_LION;       // consecutive elements per lane, SGD / Lion kernels
// elements per workgroup (= per chunk-table entry) for an optimizer kind
constexpr int chunk_elems(int kind) { return kThreads * (kind == 0 ? kVecAdamW : kVecSgdLion); }
constexpr int kCopyChunkBytes = 64 * 1024;         // checkpoint copy: bytes per workgroup

// One tensor as the kernels see it (device pointers), 72 bytes.
struct TensorDev {
    void* param;
    int8_t* rho;
    const void* grad;
    int8_t* m_q;
    uint16_t* m_scale;
    uint8_t* v_q;
    uint16_t* v_scale;
    int64_t numel;
    float lr, wd;
};

// Per-call scalars, computed once on the host.
struct StepConsts {
    float beta1, beta2;   // AdamW/Lion betas; SGD: beta1 = momentum
    float omb1, omb2;     // 1.0f - beta (FP32 subtraction)
    float rbc1, rbc2;     // 1.0f / (float)(1 - beta^t), AdamW only
    float eps;
    float root_bc2;       // (float)sqrt(1 / (double)rbc2): used only to pre-estimate variance codes
};

struct StepArgs {
    const TensorDev* tensors;   // device table (multi-tensor launch)
    const uint2* chunks;        // device chunk table: {tensor index, chunk index within the tensor}
    TensorDev single;           // the one tensor of a direct launch
    StepConsts c;
};

struct CopySegment {
    const uint8_t* src;
    uint8_t* dst;
    int64_t bytes;       // bytes to copy
    int64_t pad_bytes;   // >= bytes; [bytes, pad_bytes) of dst is zero-filled
};

hipError_t launch_step(int kind, bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s);
void launch_split(const float* theta, void* param, int8_t* rho, int64_t n, hipStream_t s);
void launch_reconstruct(const void* param, const int8_t* rho, float* theta, int64_t n, hipStream_t s);
void launch_quantize(bool variance, const float* x, void* q, uint16_t* scale, int64_t n, hipStream_t s);
void launch_dequantize(bool variance, const void* q, const uint16_t* scale, float* x, int64_t n, hipStream_t s);
void launch_copy(const CopySegment* segs, const uint2* chunks, int64_t n_chunks, hipStream_t s);

}  // namespace fo
#endif
