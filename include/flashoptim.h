/*
 * flashoptim.h - C ABI of the MI355X (gfx950) FlashOptim optimizer-step library.
 *
 * The library implements the fused per-parameter optimizer step of FlashAdamW,
 * FlashSGD and FlashLion (paper Section 3.3, Algorithms 4, 5, 6) on the
 * compressed per-parameter layout of Table 1:
 *
 *     theta'  BF16   2 B   low-precision weight the model trains on
 *     rho     INT8   1 B   weight correction            (Section 3.1, Eq. 1-2, Algorithm 1)
 *     g       BF16   2 B   gradient (0 B resident with gradient release, Section 3.4)
 *     m       INT8   1 B   companded momentum code      (Section 3.2, Eq. 3, Algorithm 2)
 *     v       UINT8  1 B   companded variance code      (Section 3.2, Eq. 4, Algorithm 3; AdamW only)
 *     scales  FP16   2 B per group of G = 32 consecutive elements, per state
 *
 * General conventions
 *  - Every data pointer is a DEVICE pointer on the current HIP device, owned by the
 *    caller, and must be 16-byte aligned.  Descriptor arrays and hyper-parameter
 *    structs are HOST memory and are read before the call returns.
 *  - A tensor is its flattened, contiguous element sequence; quantisation groups are
 *    elements [32k, 32k+32) of that sequence, the last group may be short, and groups
 *    never span tensors.  A scale array holds ceil(numel/32) FP16 bit patterns.
 *  - All-zero m_q/m_scale/v_q/v_scale buffers are the initial state Q_m(0), Q_v(0)
 *    (the initialisation of Algorithm 4): a zero scale decodes to exactly zero.
 *  - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = the default
 *    stream) and the call returns without waiting.  Buffers may be reused or freed
 *    by the caller in stream order.  Calls that touch the same tensors from different
 *    streams must be ordered by the caller, as for any other kernel; calls on disjoint
 *    lists may run concurrently (the library is thread-safe).
 *  - One call covers at most 2^31 - 1 workgroups (2048 elements each for AdamW, 4096 for
 *    SGD / Lion): more returns FLASHOPTIM_ERR_NUMEL_RANGE.
 *  - Return value: FLASHOPTIM_OK (0) or a negative flashoptim_status.  Arguments are
 *    validated before anything is enqueued: when an error is returned no buffer has
 *    been modified.  Nothing throws or aborts.
 *  - Inputs are expected to be finite.  NaN/Inf values propagate into the results of
 *    their own element or group but never cause out-of-bounds accesses.  An infinite
 *    weight keeps rho = 0; the rho byte stored next to a NaN weight is unspecified.
 *  - Arithmetic: IEEE binary32, round-to-nearest-even, subnormals kept, no fused
 *    multiply-add, in the order the algorithms print it (one documented exception: the
 *    default AdamW step rounds one division faithfully, see flashoptim_adamw_step); divisions by a group scale
 *    or by a bias correction 1 - beta^t multiply by the correctly rounded FP32
 *    reciprocal of that scalar.
 *  - There is no CPU fallback: without a HIP device every compute entry point
 *    returns FLASHOPTIM_ERR_HIP.
 */
#ifndef FLASHOPTIM_H
#define FLASHOPTIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum flashoptim_status {
    FLASHOPTIM_OK = 0,
    FLASHOPTIM_ERR_INVALID_ARG = -1, /* null pointer, negative count, bad kind, step < 1, ... */
    FLASHOPTIM_ERR_MISALIGNED = -2,  /* a device pointer is not 16-byte aligned               */
    FLASHOPTIM_ERR_NUMEL_RANGE = -3, /* numel < 0 or >= 2^40                                  */
    FLASHOPTIM_ERR_HIP = -4,         /* a HIP runtime call failed (see flashoptim_last_hip_error) */
    FLASHOPTIM_ERR_BAD_BLOB = -5,    /* checkpoint blob too small, or header/table mismatch   */
    FLASHOPTIM_ERR_SELFTEST = -6,    /* flashoptim_selftest found a failing check             */
    FLASHOPTIM_ERR_LIST_TOO_LONG = -7 /* flashoptim_adamw_step_noalloc: more than 1024 non-empty tensors */
} flashoptim_status;

/* Optimizer kinds (checkpoint entry points). */
enum { FLASHOPTIM_ADAMW = 0, FLASHOPTIM_SGD = 1, FLASHOPTIM_LION = 2 };

/* One parameter tensor in the compressed layout.  lr and weight_decay are per tensor
 * because the paper's recipes exempt biases and normalisation parameters from weight
 * decay (Appendix B) and follow a learning-rate schedule (Algorithm 4, Require). */
typedef struct flashoptim_tensor {
    void*       param;    /* [numel] BF16 theta', in/out                                    */
    int8_t*     rho;      /* [numel] INT8 weight correction, in/out                         */
    const void* grad;     /* [numel] BF16 gradient, in                                      */
    int8_t*     m_q;      /* [numel] INT8 momentum codes, in/out                            */
    uint16_t*   m_scale;  /* [ceil(numel/32)] FP16 bits, in/out                             */
    uint8_t*    v_q;      /* [numel] UINT8 variance codes, in/out; AdamW only, else NULL    */
    uint16_t*   v_scale;  /* [ceil(numel/32)] FP16 bits, in/out;   AdamW only, else NULL    */
    int64_t     numel;    /* >= 0; a tensor with numel == 0 is skipped                      */
    float       lr;       /* eta_t for this tensor                                          */
    float       weight_decay; /* lambda for this tensor (decoupled, multiplied by lr)       */
} flashoptim_tensor;

typedef struct flashoptim_adamw_hp {
    float   beta1, beta2, eps;
    int64_t step;         /* t >= 1: Algorithm 4 increments t before using it               */
} flashoptim_adamw_hp;

typedef struct flashoptim_sgd_hp { float momentum; } flashoptim_sgd_hp;

typedef struct flashoptim_lion_hp { float beta1, beta2; } flashoptim_lion_hp;

/* ---- fused steps over a list of tensors ------------------------------------------
 * One call covers the whole list: hundreds of small tensors fill the chip through a small
 * index table that the library builds once per distinct list and caches on the device; the
 * work is issued as a few back-to-back kernel launches on the given stream (one per 2^28
 * elements).  A list of length one is the gradient-release call (Section 3.4): it needs no
 * table and no device allocation.  Tables of the 256 most recently used lists are kept; a call
 * with a further distinct list frees the least recently used one after synchronising the device.  The grad pointers are not part of the
 * cached identity of a list, so gradients may live in different buffers each step.  A call whose descriptors
 * (pointers, grad pointers, numel, lr, weight_decay) equal those of the previous call on the same list enqueues
 * kernels only and may be captured into a HIP graph; changed descriptors are uploaded in stream order first.
 *
 * flashoptim_adamw_step: Algorithm 4, the body of the loop after the gradient (reconstruct m, v, theta; AdamW
 *   update with bias correction and decoupled weight decay; quantize m, v; split theta).
 * flashoptim_sgd_step:   Algorithm 5, loop body (m <- mu m + g; theta <- theta - eta (m + lambda theta)).
 * flashoptim_lion_step:  Algorithm 6, loop body (u = sign(b1 m + (1-b1) g); m <- b2 m + (1-b2) g;
 *   theta <- theta - eta (u + lambda theta)); sign(0) = 0.
 * tensors: host array of n_tensors descriptors (n_tensors >= 0).
 *
 * Rounding of the quotient m_hat / (sqrt(v_hat) + eps) of the AdamW update:
 *   flashoptim_adamw_step        faithful: the hardware reciprocal estimate, the quotient and one FMA residual
 *                                correction.  The result is within one ulp of the correctly rounded quotient
 *                                (flashoptim_selftest bounds this on the device) and differs from it only when
 *                                the exact quotient lies within 2^-23 ulp of the midpoint of two FP32 numbers:
 *                                about one operand pair in 10^9 (flashoptim_faithful_rounding_stats counts them).
 *                                Such a difference can move the new master weight by one FP32 ulp, hence rho by
 *                                one unit on a rare element.  Momentum codes, variance codes and all scales do
 *                                not depend on the quotient and are the exact ones in either case.  Used when
 *                                2^-60 <= eps <= 1 and the operands do not exceed 2^60; otherwise this entry point
 *                                takes the IEEE division (slower, same results as the exact entry point).
 *   flashoptim_adamw_step_exact  the quotient is correctly rounded for every input: the whole step is
 *                                bit-identical to the arithmetic stated above.  About 3 % slower on MI355X.
 * Everything else is identical between the two. */
int flashoptim_adamw_step(const flashoptim_tensor* tensors, int64_t n_tensors,
                          const flashoptim_adamw_hp* hp, void* stream);
int flashoptim_adamw_step_exact(const flashoptim_tensor* tensors, int64_t n_tensors,
                                const flashoptim_adamw_hp* hp, void* stream);
int flashoptim_sgd_step(const flashoptim_tensor* tensors, int64_t n_tensors,
                        const flashoptim_sgd_hp* hp, void* stream);
int flashoptim_lion_step(const flashoptim_tensor* tensors, int64_t n_tensors,
                         const flashoptim_lion_hp* hp, void* stream);

/* ---- the FlashAdamW step for callers that cannot allocate ---------------------------------
 * For code under HIP stream capture, tight serving loops and harnesses that forbid allocation: the same step
 * as flashoptim_adamw_step_exact, same arguments, same results bit for bit, but the call allocates nothing
 * (no hipMalloc / hipFree / hipHostMalloc, no host-to-device copy): the two device tables of a multi-tensor
 * launch are written by small kernels, from kernel arguments, into a fixed 172,032-byte device array that
 * each GPU holds from library load to process end.
 * Every table entry a call's launches read is written by that call first, so nothing left behind by an earlier
 * call (a longer list, larger tensors) is ever seen.
 * Limits: at most 1024 tensors with numel > 0 (FLASHOPTIM_ERR_LIST_TOO_LONG beyond that, nothing enqueued) and,
 * as for every step call, at most 2^31 - 1 workgroups.  Every call on a GPU shares that GPU's array: calls on
 * the same stream are ordered and safe; calls that may overlap on one GPU (different streams, several host
 * threads) race on it and must be ordered by the caller.  This entry point does not start the check of the
 * short square root (see flashoptim_short_sqrt_state): where no AdamW step call of another entry point has
 * put it on a stream of this device, or it has not finished yet, the kernels use sqrtf: same results, a few
 * percent slower. */
int flashoptim_adamw_step_noalloc(const flashoptim_tensor* tensors, int64_t n_tensors,
                                  const flashoptim_adamw_hp* hp, void* stream);

/* ---- sharding a flat tensor over ranks (Section 3.4, "Distributed training") ----------------
 * With ZeRO / FSDP-style sharding each rank owns a contiguous piece of every flattened tensor, keeps rho, the
 * state codes and their scales for that piece only, and steps it with the calls above; nothing but the BF16
 * weights is exchanged.  Quantisation groups must not straddle ranks, and every stream of a shard (the
 * 2-byte-per-group scales included) must start 16-byte aligned: this call cuts [0, numel) into `world`
 * consecutive shards on multiples of 256 elements, as evenly as that allows (sizes differ by at most 256; only
 * the last non-empty shard can be ragged; with fewer than `world` units the trailing ranks get len 0).
 * *begin, *len (HOST): the element range of `rank`.  A shard's descriptor is the tensor's descriptor with
 * param, rho, grad, m_q, v_q advanced by begin elements, m_scale and v_scale by begin / 32, numel = len;
 * stepping the shards (in one list or in `world` calls) gives the same bits as stepping the whole tensor.
 * Host arithmetic only. */
int flashoptim_shard_range(int64_t numel, int64_t world, int64_t rank, int64_t* begin, int64_t* len);

/* ---- ablation and reference variants of the steps (Section 4.3) -----------------------
 * The paper isolates its two techniques: "Weight Split" (split weights, FP32 states) and
 * "Opt. Quant." (FP32 master weights, 8-bit states); with both off the step is the plain FP32
 * optimizer (Algorithms 4-6 without their highlighted lines), here still fed BF16 gradients.
 * flags: FLASHOPTIM_SPLIT_WEIGHTS | FLASHOPTIM_QUANTIZE_STATES selects which technique is ON; both on
 * is identical to the plain entry points above.
 * With splitting off, `theta` ([numel] FP32, in/out) is the master weight and t.param / t.rho are
 * ignored; with state quantisation off, `m` (and `v` for AdamW; [numel] FP32, in/out) hold the
 * states and t.m_q / t.m_scale / t.v_q / t.v_scale are ignored.  Ignored pointers may be NULL.
 * Bytes moved per parameter (AdamW): 12.25 both on; 24 weight split only; 14.25 state quantisation
 * only; 26 both off. */
enum { FLASHOPTIM_SPLIT_WEIGHTS = 1, FLASHOPTIM_QUANTIZE_STATES = 2 };

typedef struct flashoptim_tensor_ex {
    flashoptim_tensor t;  /* compressed buffers, grad, numel, lr, weight_decay                   */
    float* theta;         /* [numel] FP32 master weight, used when weights are not split         */
    float* m;             /* [numel] FP32 momentum, used when states are not quantized           */
    float* v;             /* [numel] FP32 variance (AdamW), used when states are not quantized   */
} flashoptim_tensor_ex;

int flashoptim_adamw_step_ex(const flashoptim_tensor_ex* tensors, int64_t n_tensors,
                             const flashoptim_adamw_hp* hp, unsigned flags, void* stream);
int flashoptim_sgd_step_ex(const flashoptim_tensor_ex* tensors, int64_t n_tensors,
                           const flashoptim_sgd_hp* hp, unsigned flags, void* stream);
int flashoptim_lion_step_ex(const flashoptim_tensor_ex* tensors, int64_t n_tensors,
                            const flashoptim_lion_hp* hp, unsigned flags, void* stream);

/* ---- migration between a standard FP32 optimizer state and the compressed layout --------
 * compress_state:   theta', rho <- C(theta);  m_q, m_scale <- Q_m(m);  v_q, v_scale <- Q_v(v)
 *                   (Algorithms 1-3; the initialisation of Algorithm 4 when m = v = 0, and the way to
 *                   adopt the compressed layout from an existing 12 B/param FP32 state).
 * decompress_state: theta <- C^-1(theta', rho);  m <- Q_m^-1;  v <- Q_v^-1  (export).
 * One launch over the list.  Both layouts' buffers of every tensor are required (v, v_q, v_scale for
 * kind = FLASHOPTIM_ADAMW only); t.grad, t.lr, t.weight_decay are ignored. */
int flashoptim_compress_state(int kind, const flashoptim_tensor_ex* tensors, int64_t n_tensors, void* stream);
int flashoptim_decompress_state(int kind, const flashoptim_tensor_ex* tensors, int64_t n_tensors, void* stream);

/* ---- measurement aid (no passage of the paper: the memory ceiling of the step's access pattern) ----
 * stream_probe: reads every array a step of this kind reads (gradients included) and writes every
 * array it writes back UNCHANGED, through the same launch shape and access instructions as the step,
 * with no arithmetic.  Timing it gives the rate the memory system delivers for exactly the step's
 * traffic (12.25 B/param for AdamW, 10.125 for SGD and Lion), to set the step's own rate against.
 * Same arguments, validation, stream ordering and errors as the *_step calls; lr and weight_decay
 * are ignored; no state changes. */
int flashoptim_stream_probe(int kind, const flashoptim_tensor* tensors, int64_t n_tensors, void* stream);

/* ---- weight splitting (Section 3.1, Algorithm 1, N = 127) --------------------------
 * split:       theta (FP32) -> theta' = BF16 round-to-nearest-even, rho = Round(e / (ULP(theta')/2) * 127)
 *              Used once at the start of training (initialisation of Algorithm 4).
 * reconstruct: theta_hat = theta' + (rho/127) * ULP(theta')/2   (Eq. 2)
 * n >= 0 elements; all pointers device memory. */
int flashoptim_split_weights(const float* theta, void* param_bf16, int8_t* rho, int64_t n, void* stream);
int flashoptim_reconstruct_weights(const void* param_bf16, const int8_t* rho, float* theta, int64_t n,
                                   void* stream);

/* ---- 16-bit correction and the exhaustive reconstruction experiment (Section 4.4) ------
 * Algorithm 1 with N = 32767: rho is an INT16 (theta' + rho = 32 bits, near-lossless).  Same
 * conventions as the INT8 entry points above.  The fused steps use the INT8 form only.
 * reconstruction_sweep: pushes the FP32 bit patterns first, first + stride, ... (< 2^32; stride 1
 *   and first 0 = every FP32 value) through split then reconstruct with an 8- or 16-bit correction
 *   and returns error statistics in `stats`, a HOST array of 520 doubles:
 *   [0] values measured  [1] skipped (non-finite theta or theta')  [2] values with |theta - theta'| >
 *   ULP(theta')/2  [3] max |theta_hat - theta| / (ULP(theta')/(4N))  [4] max relative error over normal
 *   theta  [5] bit-exact reconstructions  [6] rho outside [-N, N]  [7] unused  [8 + E] sum and
 *   [264 + E] count of the relative errors of the normal values with FP32 exponent field E (their ratio
 *   is the mean relative error per exponent that Figure 3 plots).  Waits for completion. */
int flashoptim_split_weights_i16(const float* theta, void* param_bf16, int16_t* rho, int64_t n, void* stream);
int flashoptim_reconstruct_weights_i16(const void* param_bf16, const int16_t* rho, float* theta, int64_t n,
                                       void* stream);
int flashoptim_reconstruction_sweep(int correction_bits, uint64_t first, uint64_t stride, double* stats,
                                    void* stream);
/* The same experiment with a choice of how ULP(theta') is read, and per-exponent counts of bit-exact
 * reconstructions.  ulp_reading 0: Algorithm 1 as printed, one spacing per theta' (what every other entry
 * point of this library uses).  ulp_reading 1, "directional": the spacing of the BF16 grid on the side of
 * theta' on which theta lies, which is half as large when theta' is a power of two and theta lies towards
 * zero; Section 4.4 prints 99.92 % bit-exact reconstructions for the 16-bit correction, which this reading
 * reproduces over the mid-range exponents and the printed algorithm does not (99.73 %).  It exists for this
 * experiment only.  stats: HOST array of 776 doubles, the 520 above followed by [520 + E] bit-exact
 * reconstructions among the normal values with FP32 exponent field E.  [2] and [3] refer to the printed
 * ULP under both readings.  Waits for completion. */
int flashoptim_reconstruction_sweep_ex(int correction_bits, int ulp_reading, uint64_t first, uint64_t stride,
                                       double* stats, void* stream);

/* ---- companded 8-bit state codecs (Section 3.2, Algorithms 2 and 3) -----------------
 * quantize_momentum:   per group s = FP16(max|m|), code = Round(127 * 2m'/(1+|m'|)), m' = m/s
 * dequantize_momentum: m = (z / (2 - |z|)) * s, z = code/127
 * quantize_variance:   per group s = FP16(max sqrt(v)), code = Round(255 * sqrt(v)/s)
 * dequantize_variance: v = ((code/255) * s)^2
 * n >= 0 elements, scale arrays of ceil(n/32) FP16 bit patterns; all device memory. */
int flashoptim_quantize_momentum(const float* m, int8_t* q, uint16_t* scale, int64_t n, void* stream);
int flashoptim_dequantize_momentum(const int8_t* q, const uint16_t* scale, float* m, int64_t n, void* stream);
int flashoptim_quantize_variance(const float* v, uint8_t* q, uint16_t* scale, int64_t n, void* stream);
int flashoptim_dequantize_variance(const uint8_t* q, const uint16_t* scale, float* v, int64_t n, void* stream);

/* ---- linear baseline and quantisation error (Section 4.5) ------------------------------
 * The paper validates its companders against plain absmax-scaled integer quantisation: the same
 * group-wise FP16 absmax scale, no compander (momentum code = Round(127 m / s); variance code =
 * Round(255 v / s) with s the group maximum of v itself).
 * quantize_state / dequantize_state: state 0 = momentum (INT8 codes), 1 = variance (UINT8 codes);
 *   linear 0 = companded (identical to the four entry points above), 1 = the linear baseline.
 * quantization_nmse: quantizes and dequantizes x on the fly and returns in `sums` (HOST, 2 doubles)
 *   sum (x_hat - x)^2 and sum x^2, whose ratio is the normalised MSE the paper plots.  Waits for
 *   completion. */
int flashoptim_quantize_state(int state, int linear, const float* x, void* q, uint16_t* scale, int64_t n,
                              void* stream);
int flashoptim_dequantize_state(int state, int linear, const void* q, const uint16_t* scale, float* x, int64_t n,
                                void* stream);
int flashoptim_quantization_nmse(int state, int linear, const float* x, int64_t n, double* sums, void* stream);

/* ---- checkpoint (Section 3.4, "Checkpoint size": 2 + 1 + 1 + 1 bytes per parameter) --
 * The paper fixes the content, not a container.  Blob layout, little-endian:
 *   header (64 B): "FOPTCKPT" | u32 version = 1 | u32 kind | i64 step | i64 n_tensors |
 *                  i64 total_bytes | zero padding
 *   table: per tensor i64 numel | i64 offset of its first section from the blob start;
 *          padded to a multiple of 64 B
 *   per tensor, in list order, each section starting on a 64-byte boundary and zero
 *   padded: theta' (2n) | rho (n) | m codes (n) | m scales (2 ceil(n/32)) |
 *   AdamW only: v codes (n) | v scales (2 ceil(n/32))
 * checkpoint_size: total blob bytes for a list (numels: host array), or a negative status.
 * checkpoint_pack:   gathers the tensors' state into `blob` (DEVICE memory, 16-byte aligned,
 *                    blob_bytes >= checkpoint_size).  grad fields are ignored.
 * checkpoint_unpack: scatters `blob` (DEVICE memory) back into the tensors' buffers and
 *                    returns the stored step in *step_out (host).  The header and table
 *                    are validated against (kind, list) first; this reads the header back to
 *                    the host and therefore waits for prior work on `stream`. */
int64_t flashoptim_checkpoint_size(int kind, const int64_t* numels, int64_t n_tensors);
int flashoptim_checkpoint_pack(int kind, const flashoptim_tensor* tensors, int64_t n_tensors, int64_t step,
                               void* blob, int64_t blob_bytes, void* stream);
int flashoptim_checkpoint_unpack(int kind, const void* blob, int64_t blob_bytes,
                                 const flashoptim_tensor* tensors, int64_t n_tensors, int64_t* step_out,
                                 void* stream);

/* ---- housekeeping --------------------------------------------------------------------
 * strerror: static string for a status.  last_hip_error: hipError_t value of the most recent
 * failed HIP call on this thread (0 if none).  release_cache: frees the cached device chunk
 * tables (synchronises the device first).  version: (major << 16) | minor. */
const char* flashoptim_strerror(int status);

/* ---- device self-test ------------------------------------------------------------------
 * The step kernels obtain some correctly rounded results (1/s of an FP16 scale, sqrt, the
 * decision of an 8-bit code) from shorter instruction sequences that are exact provided the
 * hardware reciprocal and square root are within 1 ulp.  This call checks those provisions on
 * the current device against plain IEEE operations, exhaustively where the domain is small:
 *   [0] Newton reciprocal of every positive finite FP16 value      [1] v_rcp_f32 within 1 ulp on [1, 4)
 *   [2] short square root (reciprocal-square-root estimate + one correction) == sqrtf for EVERY FP32 value
 *       of its range [2^-96, FLT_MAX] (1,879,048,192 values)
 *   [3] momentum codes (Algorithm 2) and [4] variance codes (Algorithm 3): the estimate equals the
 *       exact code wherever the kernel's tie test does not ask for the exact evaluation.
 *   [5] short division == IEEE division on 2^30 + 2^24 operand pairs inside its range.
 *   [6] faithful division of flashoptim_adamw_step: within 1 ulp of the IEEE quotient on the pairs of [5].
 * n_checked, n_failed: HOST arrays of 7 counters (one per section above).  Waits for completion (a
 * fraction of a second).  Returns FLASHOPTIM_OK, FLASHOPTIM_ERR_SELFTEST if any check failed, or another status. */
int flashoptim_selftest(int64_t* n_checked, int64_t* n_failed, void* stream);
/* How often the faithful division differs from the exactly rounded quotient at all, measured on this device:
 * counts (HOST, 2 entries) = {operand pairs checked (2^30 + 2^24), of these not exact}.  Waits for
 * completion.  FLASHOPTIM_ERR_SELFTEST if any quotient is off by more than one ulp. */
int flashoptim_faithful_rounding_stats(int64_t* counts, void* stream);
/* The AdamW kernels take sqrt(v_hat) as the hardware reciprocal-square-root estimate plus one correction,
 * which is the correctly rounded root only if the estimate makes it so.  They read the lower limit of that
 * sequence's use from a word of device memory that holds +inf (never used: sqrtf throughout) until the device
 * has passed a check of every FP32 value of the sequence's range, [2^-96, FLT_MAX], against sqrtf.  The first
 * AdamW step call on a device (any entry point but flashoptim_adamw_step_noalloc) puts that check on its stream
 * ahead of its own kernels, once per process and device: about 4 ms on MI355X, no allocation, no wait on the
 * host.  Kernels that run before the verdict has landed (on another stream, say) use sqrtf, with the same
 * results.  A first call made under stream capture does not start the check (it belongs in front of a graph,
 * not inside it); a later call outside capture does.  With FLASHOPTIM_FORCE_GENERAL_SQRT set to a non-zero
 * value in the environment the check is not run and the word stays at +inf.
 * Returns the state for the current device: 0 check not started, 1 verified (short sequence in use), 2 not in
 * use; negative status on a HIP error.  If the check is on its way the call waits for its verdict; in states
 * 0 and 2 it reads the word back (a blocking 4-byte copy) and returns FLASHOPTIM_ERR_SELFTEST unless it holds
 * +inf. */
int flashoptim_short_sqrt_state(void);
/* A measurement aid: samples the clock the compute units run at while other kernels execute (a step kernel
 * under the package power limit runs well below the nominal clock).  Enqueues a one-wavefront kernel on
 * `stream` (use a stream of its own, next to the work to be observed) that takes n_samples samples of
 * seconds_per_sample each and then ends; it writes 2 * n_samples uint64 values to `samples` (DEVICE memory,
 * owned by the caller, valid until the kernel has finished): for each sample the ticks of the fixed-frequency
 * counter that went by and the shader-clock cycles in the same interval.  *tick_hz (HOST) receives the tick
 * rate, so that clock = cycles / ticks * tick_hz.  1 <= n_samples <= 100000, 0 < seconds_per_sample <= 1.
 * Does not wait for completion. */
int flashoptim_clock_monitor(uint64_t* samples, int64_t n_samples, double seconds_per_sample, double* tick_hz,
                             void* stream);
/* Number of kernel launches one step call of `kind` issues for a list with these element counts
 * (host arithmetic only; for reading profiles: per-kernel durations are per launch).  Negative
 * status on invalid arguments. */
int64_t flashoptim_step_launch_count(int kind, const int64_t* numels, int64_t n_tensors);
int flashoptim_last_hip_error(void);
int flashoptim_release_cache(void);
int flashoptim_version(void);

#ifdef __cplusplus
}
#endif
#endif /* FLASHOPTIM_H */
