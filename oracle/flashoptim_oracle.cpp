// FlashOptim CPU oracle: TEST INFRASTRUCTURE ONLY.
//
// A plain, slow, scalar implementation of what the fused FlashOptim optimizer
// step computes, written from the paper's definitions (Section 3, Eq. 1-4,
// Algorithms 1-6).  Nothing in the product library may call, link or import
// this file; only the tests, the smoke check and the benchmark's CPU-baseline
// leg do.  It shares no code, header, table or constant generator with the
// HIP path.
//
// Arithmetic model.  The paper fixes the working precision: master weights are
// FP32, Algorithm 1 converts through Float32(.), and the reference optimizer
// state is FP32.  Every floating-point operation below is therefore one IEEE
// binary32 operation, rounded to nearest-even, with subnormals kept and no
// fused multiply-add (build with -ffp-contract=off, never -ffast-math).
// Integer work is done in int32/int64.
//
// Readings taken where the paper is silent (each one is marked [R-xx] at the
// line that implements it):
//   [R-A1] Downcast to BF16 is round-to-nearest-even (Section 3.1 names
//          round-to-nearest; the 1e-5 -> 1.0014e-5 example pins it against
//          truncation).
//   [R-A2] ULP(theta') = 2^(max(E,1)-134) with E the biased exponent field of
//          theta'; zero and BF16 subnormals share the spacing of the lowest
//          binade.  The sign of the error is not consulted.
//          An alternative reading, "directional", exists ONLY for the Section 4.4 sweep (see
//          split_one_directional): the paper prints 99.92 % bit-exact 16-bit reconstructions, which
//          the literal reading does not reach and the directional one does.  The steps, the
//          codecs and the checkpoint never use it.
//   [R-A3] Round(.) in Algorithm 1 is round-half-to-even.
//   [R-A6] Non-finite theta': rho = 0 and reconstruction returns theta'.
//   [R-Q1] A group whose stored scale is zero encodes to all-zero codes and
//          decodes to exactly zero, so zero-filled buffers are Q_m(0), Q_v(0).
//   [R-Q2] The scale that normalises a group is the stored FP16 scale read
//          back as FP32 (what the decoder will see), not the FP32 absmax.
//          Codes are clamped to [-127,127] / [0,255].
//   [R-Q3] A group absmax above 65504 stores 65504 (saturates, never inf).
//          FP16-subnormal scales are legal.
//   [R-Q4] Round(., INT8/UINT8) is round-half-to-even, then clamp.
//   [R-Q5] Groups are consecutive runs of 32 elements of the flattened tensor
//          starting at element 0; the last group may be short.
//   [R-Q6] Division by a per-group scale is multiplication by the correctly
//          rounded FP32 reciprocal 1.0f/s of that scale; division by the
//          bias corrections is multiplication by 1.0f/(1-beta^t), with
//          1-beta^t evaluated in double and rounded to FP32 once.
//   [R-U2] epsilon is added outside the square root, after bias correction.
//   [R-U3] Weight decay is decoupled, scaled by the learning rate, and uses
//          the reconstructed theta_{t-1}.
//   [R-U4] sign(0) = 0 in Lion.
//   [R-U5] Update formulas are evaluated left to right as printed, each
//          operation rounded (see the step functions).
//
// Parity pins for every function here live in tests/test_oracle_*.py.
// "parity unpinned": the 100-step trajectory of Algorithm 4 has no value in
// the paper to compare against beyond the qualitative "nearly identical"
// statement of Section 4.2; only its per-step pieces are pinned.

#include <cmath>
#include <cstdint>
#include <cstring>
#include <cstdlib>

#ifdef _OPENMP
#include <omp.h>
#endif

namespace {

constexpr int kGroup = 32;  // Algorithms 2 and 3: G = 32

inline uint32_t f32_bits(float x) { uint32_t u; std::memcpy(&u, &x, 4); return u; }
inline float bits_f32(uint32_t u) { float x; std::memcpy(&x, &u, 4); return x; }

// ---------------------------------------------------------------- formats --

// FP32 -> BF16, round-to-nearest-even on the upper 16 bits.  [R-A1]
uint16_t bf16_rne(float x) {
    uint32_t u = f32_bits(x);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);  // quiet NaN
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7fffu + lsb;
    return (uint16_t)(u >> 16);
}

inline float bf16_to_f32(uint16_t b) { return bits_f32((uint32_t)b << 16); }

// FP32 -> FP16 (IEEE binary16), round-to-nearest-even, subnormals kept.
uint16_t fp16_rne(float x) {
    uint32_t u = f32_bits(x);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t a = u & 0x7fffffffu;
    if (a > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);  // NaN
    if (a >= 0x47800000u) return (uint16_t)(sign | 0x7c00u); // |x| >= 2^16 (incl. inf)
    if (a < 0x33000000u) return (uint16_t)sign;              // |x| < 2^-25 rounds to zero
    int e = (int)(a >> 23) - 127;                            // unbiased exponent, >= -25
    uint32_t sig = (a & 0x7fffffu) | 0x800000u;              // 24-bit significand
    int drop = (e >= -14) ? 13 : 13 + (-14 - e);             // low bits that do not fit
    uint32_t kept = sig >> drop;
    uint32_t rem = sig & ((1u << drop) - 1u);
    uint32_t half = 1u << (drop - 1);
    if (rem > half || (rem == half && (kept & 1u))) kept += 1u;
    if (e >= -14) {
        // kept in [0x400, 0x800]; a carry out of the significand moves into the
        // exponent field, and out of the top binade into the inf encoding.
        uint32_t h = ((uint32_t)(e + 15) << 10) + (kept - 0x400u);
        return (uint16_t)(sign | h);
    }
    return (uint16_t)(sign | kept);  // subnormal, or 0x0400 = smallest normal
}

float fp16_to_f32(uint16_t h) {
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    int e = (h >> 10) & 0x1f;
    uint32_t f = h & 0x3ffu;
    if (e == 0x1f) return bits_f32(sign | 0x7f800000u | (f << 13));
    if (e == 0) {
        float v = std::ldexp((float)f, -24);  // exact
        return sign ? -v : v;
    }
    return bits_f32(sign | ((uint32_t)(e - 15 + 127) << 23) | (f << 13));
}

inline int floor_div2(int a) { return (a >= 0) ? a / 2 : -((-a + 1) / 2); }

// ------------------------------------------------- weight splitting, Alg. 1 --

// l = floor(log2 ULP(theta')) - 1, i.e. 2^l = ULP(theta')/2.   [R-A2]
inline int half_ulp_log2(uint16_t thp) {
    int E = (thp >> 7) & 0xff;
    if (E < 1) E = 1;
    return (E - 127 - 7) - 1;
}

inline bool bf16_is_finite(uint16_t b) { return ((b >> 7) & 0xff) != 0xff; }

// C(theta) -> (theta', rho): the encoder of Algorithm 1 (Eq. 1).
void split_one(float theta, int N, uint16_t* thp_out, int* rho_out) {
    uint16_t thp = bf16_rne(theta);                       // the BF16 weight the model trains on
    *thp_out = thp;
    if (!bf16_is_finite(thp)) { *rho_out = 0; return; }   // [R-A6]
    float e = theta - bf16_to_f32(thp);                   // what the downcast lost (exact in FP32)
    int l = half_ulp_log2(thp);                           // 2^l is the largest magnitude e can have
    int h = floor_div2(-l);                               // the scaling by 2^-l is applied as two powers of
    float p1 = std::ldexp(1.0f, h);                       // two, 2^h and 2^(-l-h), neither of which can
    float p2 = std::ldexp(1.0f, -l - h);                  // overflow; both products are exact
    float e_norm = (e * p1) * p2;                         // e relative to its largest magnitude, in [-1, 1]
    float c = e_norm;                                     // (the clamp never acts on a finite theta')
    if (c < -1.0f) c = -1.0f;
    if (c > 1.0f) c = 1.0f;
    *rho_out = (int)std::rint(c * (float)N);              // N levels per side, ties to even   [R-A3]
}

// C^-1(theta', rho) -> theta_hat: the decoder of Algorithm 1 (Eq. 2).
float reconstruct_one(uint16_t thp, int rho, int N) {
    float base = bf16_to_f32(thp);
    if (!bf16_is_finite(thp)) return base;                // [R-A6]
    int l = half_ulp_log2(thp);
    int h = floor_div2(l);                                // again two power-of-two factors, 2^h and 2^(l-h)
    float q = (float)rho / (float)N;                      // the correction as a fraction of its range
    float e = (q * std::ldexp(1.0f, h)) * std::ldexp(1.0f, l - h);
    return base + e;
}

// "Directional" reading of ULP(theta') for the Section 4.4 experiment.  Algorithm 1 takes one spacing
// u per theta'.  The BF16 grid, however, is twice as fine just below a power of two as above it: when
// theta' = +-2^k (mantissa field 0, exponent field >= 2) and theta lies on the side of zero, the values
// that round to theta' fill only [theta' - u/4, theta'], so e / (u/2) uses half of [-1, 1].  Under this
// reading the spacing is taken on the side of theta' on which theta lies: u/2 in that one case, u
// otherwise.  The decoder recognises the case from the signs of rho and theta' (rho has the sign of e).
inline bool below_power_of_two(uint16_t thp, bool error_is_negative) {
    int E = (thp >> 7) & 0xff;
    bool negative = (thp & 0x8000) != 0;
    return (thp & 0x7f) == 0 && E >= 2 && (error_is_negative != negative);
}
void split_one_directional(float theta, int N, uint16_t* thp_out, int* rho_out) {
    uint16_t thp = bf16_rne(theta);
    *thp_out = thp;
    if (!bf16_is_finite(thp)) { *rho_out = 0; return; }
    float e = theta - bf16_to_f32(thp);
    int l = half_ulp_log2(thp);
    if (e != 0.0f && below_power_of_two(thp, e < 0.0f)) l -= 1;
    float e_norm = std::ldexp(e, -l);                     // exact: a power-of-two scaling within range
    if (e_norm < -1.0f) e_norm = -1.0f;
    if (e_norm > 1.0f) e_norm = 1.0f;
    *rho_out = (int)std::rint(e_norm * (float)N);
}
float reconstruct_one_directional(uint16_t thp, int rho, int N) {
    float base = bf16_to_f32(thp);
    if (!bf16_is_finite(thp)) return base;
    int l = half_ulp_log2(thp);
    if (rho != 0 && below_power_of_two(thp, rho < 0)) l -= 1;
    float q = (float)rho / (float)N;
    return base + std::ldexp(q, l);                       // one rounding at most (subnormal results)
}

// --------------------------------------------- companded quantizers, Alg. 2/3 --

// FP16 scale of a group from its FP32 absmax.  [R-Q2] [R-Q3]
inline uint16_t group_scale(float absmax) {
    float a = absmax;
    if (a > 65504.0f) a = 65504.0f;
    return fp16_rne(a);
}

// Q_m on one group of cnt <= 32 values: the encoder of Algorithm 2 (Eq. 3).
void quant_m_group(const float* m, int cnt, int8_t* q, uint16_t* scale_out) {
    float a = 0.0f;
    for (int i = 0; i < cnt; ++i) { float t = std::fabs(m[i]); if (t > a) a = t; }  // largest magnitude of the group
    uint16_t hs = group_scale(a);
    *scale_out = hs;
    float s = fp16_to_f32(hs);
    if (s == 0.0f) { for (int i = 0; i < cnt; ++i) q[i] = 0; return; }              // [R-Q1]
    float r = 1.0f / s;                                                             // [R-Q6]
    for (int i = 0; i < cnt; ++i) {
        float m1 = m[i] * r;                               // normalised to [-1, 1] by the group scale
        float num = 2.0f * m1;
        float den = 1.0f + std::fabs(m1);
        float m2 = num / den;                              // the compander phi_m: finer steps near zero
        float y = std::rint(m2 * 127.0f);                  // 127 levels per side, ties to even   [R-Q4]
        if (y > 127.0f) y = 127.0f;
        if (y < -127.0f) y = -127.0f;
        q[i] = (int8_t)(int)y;
    }
}

// Q_m^-1 on one element: the decoder of Algorithm 2.
inline float dequant_m_one(int8_t q, float s) {
    float m2 = (float)q / 127.0f;                          // the code as a fraction of its range
    float m1 = m2 / (2.0f - std::fabs(m2));                // phi_m inverted
    return m1 * s;                                         // back to the group's scale
}

// Q_v on one group: the encoder of Algorithm 3 (Eq. 4).
void quant_v_group(const float* v, int cnt, uint8_t* q, uint16_t* scale_out) {
    float vr[kGroup];
    float a = 0.0f;
    for (int i = 0; i < cnt; ++i) {
        vr[i] = std::sqrt(v[i]);                           // the compander phi_v: the root halves the dynamic range
        if (vr[i] > a) a = vr[i];                          // the scale is the largest root of the group
    }
    uint16_t hs = group_scale(a);
    *scale_out = hs;
    float s = fp16_to_f32(hs);
    if (s == 0.0f) { for (int i = 0; i < cnt; ++i) q[i] = 0; return; }  // [R-Q1]
    float r = 1.0f / s;                                                 // [R-Q6]
    for (int i = 0; i < cnt; ++i) {
        float y = std::rint((vr[i] * r) * 255.0f);         // 255 levels, ties to even   [R-Q4]
        if (y > 255.0f) y = 255.0f;
        if (y < 0.0f) y = 0.0f;
        q[i] = (uint8_t)(int)y;
    }
}

// Q_v^-1 on one element: the decoder of Algorithm 3.
inline float dequant_v_one(uint8_t q, float s) {
    float v1 = ((float)q / 255.0f) * s;                    // the root, back at the group's scale
    return v1 * v1;                                        // phi_v inverted
}

// Linear (no companding) group quantizers: plain absmax-scaled integer quantisation, the baseline that
// Section 4.5 compares the companders against.  Same scale rule [R-Q2] [R-Q3] and rounding [R-Q4]; the compander
// is dropped: momentum code = Round(127 m / s); variance code = Round(255 v / s) with s = max v.
void quant_m_linear_group(const float* m, int cnt, int8_t* q, uint16_t* scale_out) {
    float a = 0.0f;
    for (int i = 0; i < cnt; ++i) { float t = std::fabs(m[i]); if (t > a) a = t; }
    uint16_t hs = group_scale(a);
    *scale_out = hs;
    float s = fp16_to_f32(hs);
    if (s == 0.0f) { for (int i = 0; i < cnt; ++i) q[i] = 0; return; }
    float r = 1.0f / s;
    for (int i = 0; i < cnt; ++i) {
        float y = std::rint((m[i] * r) * 127.0f);
        if (y > 127.0f) y = 127.0f;
        if (y < -127.0f) y = -127.0f;
        q[i] = (int8_t)(int)y;
    }
}
inline float dequant_m_linear_one(int8_t q, float s) { return ((float)q / 127.0f) * s; }

void quant_v_linear_group(const float* v, int cnt, uint8_t* q, uint16_t* scale_out) {
    float a = 0.0f;
    for (int i = 0; i < cnt; ++i) if (v[i] > a) a = v[i];
    uint16_t hs = group_scale(a);
    *scale_out = hs;
    float s = fp16_to_f32(hs);
    if (s == 0.0f) { for (int i = 0; i < cnt; ++i) q[i] = 0; return; }
    float r = 1.0f / s;
    for (int i = 0; i < cnt; ++i) {
        float y = std::rint((v[i] * r) * 255.0f);
        if (y > 255.0f) y = 255.0f;
        if (y < 0.0f) y = 0.0f;
        q[i] = (uint8_t)(int)y;
    }
}
inline float dequant_v_linear_one(uint8_t q, float s) { return ((float)q / 255.0f) * s; }

// Reciprocal of a bias correction 1 - beta^t.  [R-Q6]
inline float recip_bias_correction(float beta, int64_t t) {
    float bc = (float)(1.0 - std::pow((double)beta, (double)t));
    return 1.0f / bc;
}

inline void set_threads(int nthreads) {
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
}

inline int64_t n_groups(int64_t n) { return (n + kGroup - 1) / kGroup; }
inline int64_t align64(int64_t x) { return (x + 63) & ~(int64_t)63; }

}  // namespace

extern "C" {

// ------------------------------------------------------------ scalar access --

uint16_t fo_oracle_bf16_rne(float x) { return bf16_rne(x); }
float fo_oracle_bf16_to_f32(uint16_t b) { return bf16_to_f32(b); }
uint16_t fo_oracle_fp16_rne(float x) { return fp16_rne(x); }
float fo_oracle_fp16_to_f32(uint16_t h) { return fp16_to_f32(h); }
int fo_oracle_half_ulp_log2(uint16_t thp) { return half_ulp_log2(thp); }

void fo_oracle_bf16_rne_array(const float* x, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = bf16_rne(x[i]);
}
void fo_oracle_fp16_rne_array(const float* x, uint16_t* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = fp16_rne(x[i]);
}
void fo_oracle_fp16_to_f32_array(const uint16_t* h, float* out, int64_t n) {
    for (int64_t i = 0; i < n; ++i) out[i] = fp16_to_f32(h[i]);
}

// ------------------------------------------------------------ array codecs --

// C over an array.  rho is written as int16 so that both N = 127 (values fit
// int8) and N = 32767 are served by one routine.
void fo_oracle_split(const float* theta, uint16_t* thp, int16_t* rho, int64_t n, int N) {
    for (int64_t i = 0; i < n; ++i) {
        int r; split_one(theta[i], N, &thp[i], &r); rho[i] = (int16_t)r;
    }
}

void fo_oracle_reconstruct(const uint16_t* thp, const int16_t* rho, float* theta, int64_t n, int N) {
    for (int64_t i = 0; i < n; ++i) theta[i] = reconstruct_one(thp[i], rho[i], N);
}

void fo_oracle_quantize_momentum(const float* m, int8_t* q, uint16_t* scale, int64_t n) {
    for (int64_t g = 0; g < n_groups(n); ++g) {
        int64_t o = g * kGroup; int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        quant_m_group(m + o, cnt, q + o, scale + g);
    }
}

void fo_oracle_dequantize_momentum(const int8_t* q, const uint16_t* scale, float* m, int64_t n) {
    for (int64_t i = 0; i < n; ++i) m[i] = dequant_m_one(q[i], fp16_to_f32(scale[i / kGroup]));
}

void fo_oracle_quantize_variance(const float* v, uint8_t* q, uint16_t* scale, int64_t n) {
    for (int64_t g = 0; g < n_groups(n); ++g) {
        int64_t o = g * kGroup; int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        quant_v_group(v + o, cnt, q + o, scale + g);
    }
}

void fo_oracle_dequantize_variance(const uint8_t* q, const uint16_t* scale, float* v, int64_t n) {
    for (int64_t i = 0; i < n; ++i) v[i] = dequant_v_one(q[i], fp16_to_f32(scale[i / kGroup]));
}

void fo_oracle_quantize_momentum_linear(const float* m, int8_t* q, uint16_t* scale, int64_t n) {
    for (int64_t g = 0; g < n_groups(n); ++g) {
        int64_t o = g * kGroup; int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        quant_m_linear_group(m + o, cnt, q + o, scale + g);
    }
}
void fo_oracle_dequantize_momentum_linear(const int8_t* q, const uint16_t* scale, float* m, int64_t n) {
    for (int64_t i = 0; i < n; ++i) m[i] = dequant_m_linear_one(q[i], fp16_to_f32(scale[i / kGroup]));
}
void fo_oracle_quantize_variance_linear(const float* v, uint8_t* q, uint16_t* scale, int64_t n) {
    for (int64_t g = 0; g < n_groups(n); ++g) {
        int64_t o = g * kGroup; int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        quant_v_linear_group(v + o, cnt, q + o, scale + g);
    }
}
void fo_oracle_dequantize_variance_linear(const uint8_t* q, const uint16_t* scale, float* v, int64_t n) {
    for (int64_t i = 0; i < n; ++i) v[i] = dequant_v_linear_one(q[i], fp16_to_f32(scale[i / kGroup]));
}

// ------------------------------------------------------------------- steps --
//
// Each step works on one flattened tensor of n elements.  Two flags select the
// paper's ablations (Section 4.3): split_weights = 0 keeps theta in the FP32
// array theta32 (thp/rho unused); quantize_states = 0 keeps m (and v) in the
// FP32 arrays m32 (v32) and leaves the code/scale arrays unused.  With both
// flags 0 the highlighted lines of Algorithms 4-6 disappear and what is left
// is plain AdamW / SGD with momentum / Lion.
// grad holds BF16 bit patterns.  t is 1-based (Algorithm 4 increments t before
// use).  Groups are independent, so the loop over groups may run in parallel
// without changing any result.

// FlashAdamW, Algorithm 4, the body of the loop after the gradient is known.
void fo_oracle_adamw_step(int64_t n, uint16_t* thp, int8_t* rho, float* theta32,
                          const uint16_t* grad,
                          int8_t* mq, uint16_t* ms, uint8_t* vq, uint16_t* vs,
                          float* m32, float* v32,
                          float lr, float wd, float beta1, float beta2, float eps, int64_t t,
                          int split_weights, int quantize_states, int nthreads) {
    set_threads(nthreads);
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    const float rbc1 = recip_bias_correction(beta1, t);
    const float rbc2 = recip_bias_correction(beta2, t);
    const int64_t ng = n_groups(n);
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < ng; ++g) {
        const int64_t o = g * kGroup;
        const int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        float m_new[kGroup], v_new[kGroup];
        float sm = 0.0f, sv = 0.0f;
        if (quantize_states) { sm = fp16_to_f32(ms[g]); sv = fp16_to_f32(vs[g]); }
        for (int i = 0; i < cnt; ++i) {
            const int64_t k = o + i;
            // reconstruct optimizer state and master weight
            float m = quantize_states ? dequant_m_one(mq[k], sm) : m32[k];
            float v = quantize_states ? dequant_v_one(vq[k], sv) : v32[k];
            float th = split_weights ? reconstruct_one(thp[k], rho[k], 127) : theta32[k];
            float gr = bf16_to_f32(grad[k]);
            // standard update  [R-U5]
            float mt = (beta1 * m) + (omb1 * gr);          // m_t = b1 m + (1-b1) g
            float gg = gr * gr;
            float vt = (beta2 * v) + (omb2 * gg);          // v_t = b2 v + (1-b2) g^2
            float mhat = mt * rbc1;                        // m_t / (1 - b1^t)   [R-Q6]
            float vhat = vt * rbc2;                        // v_t / (1 - b2^t)   [R-Q6]
            float den = std::sqrt(vhat) + eps;             // [R-U2]
            float upd = (mhat / den) + (wd * th);          // [R-U3]
            float tht = th - (lr * upd);
            m_new[i] = mt; v_new[i] = vt;
            // split the new master weight
            if (split_weights) { int r; split_one(tht, 127, &thp[k], &r); rho[k] = (int8_t)r; }
            else theta32[k] = tht;
        }
        // quantize the new optimizer state
        if (quantize_states) {
            quant_m_group(m_new, cnt, mq + o, ms + g);
            quant_v_group(v_new, cnt, vq + o, vs + g);
        } else {
            for (int i = 0; i < cnt; ++i) { m32[o + i] = m_new[i]; v32[o + i] = v_new[i]; }
        }
    }
}

// FlashSGD, Algorithm 5.
void fo_oracle_sgd_step(int64_t n, uint16_t* thp, int8_t* rho, float* theta32,
                        const uint16_t* grad, int8_t* mq, uint16_t* ms, float* m32,
                        float lr, float wd, float momentum,
                        int split_weights, int quantize_states, int nthreads) {
    set_threads(nthreads);
    const int64_t ng = n_groups(n);
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < ng; ++g) {
        const int64_t o = g * kGroup;
        const int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        float m_new[kGroup];
        float sm = quantize_states ? fp16_to_f32(ms[g]) : 0.0f;
        for (int i = 0; i < cnt; ++i) {
            const int64_t k = o + i;
            float m = quantize_states ? dequant_m_one(mq[k], sm) : m32[k];
            float gr = bf16_to_f32(grad[k]);
            float mt = (momentum * m) + gr;                // m_t = mu m + g
            float th = split_weights ? reconstruct_one(thp[k], rho[k], 127) : theta32[k];
            float tht = th - (lr * (mt + (wd * th)));      // theta - eta (m_t + lambda theta)
            m_new[i] = mt;
            if (split_weights) { int r; split_one(tht, 127, &thp[k], &r); rho[k] = (int8_t)r; }
            else theta32[k] = tht;
        }
        if (quantize_states) quant_m_group(m_new, cnt, mq + o, ms + g);
        else for (int i = 0; i < cnt; ++i) m32[o + i] = m_new[i];
    }
}

// FlashLion, Algorithm 6.
void fo_oracle_lion_step(int64_t n, uint16_t* thp, int8_t* rho, float* theta32,
                         const uint16_t* grad, int8_t* mq, uint16_t* ms, float* m32,
                         float lr, float wd, float beta1, float beta2,
                         int split_weights, int quantize_states, int nthreads) {
    set_threads(nthreads);
    const float omb1 = 1.0f - beta1;
    const float omb2 = 1.0f - beta2;
    const int64_t ng = n_groups(n);
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < ng; ++g) {
        const int64_t o = g * kGroup;
        const int cnt = (int)((n - o < kGroup) ? n - o : kGroup);
        float m_new[kGroup];
        float sm = quantize_states ? fp16_to_f32(ms[g]) : 0.0f;
        for (int i = 0; i < cnt; ++i) {
            const int64_t k = o + i;
            float m = quantize_states ? dequant_m_one(mq[k], sm) : m32[k];
            float gr = bf16_to_f32(grad[k]);
            float c = (beta1 * m) + (omb1 * gr);           // b1 m + (1-b1) g
            float u = (c > 0.0f) ? 1.0f : ((c < 0.0f) ? -1.0f : 0.0f);   // sign  [R-U4]
            float mt = (beta2 * m) + (omb2 * gr);          // m_t = b2 m + (1-b2) g
            float th = split_weights ? reconstruct_one(thp[k], rho[k], 127) : theta32[k];
            float tht = th - (lr * (u + (wd * th)));       // theta - eta (u + lambda theta)
            m_new[i] = mt;
            if (split_weights) { int r; split_one(tht, 127, &thp[k], &r); rho[k] = (int8_t)r; }
            else theta32[k] = tht;
        }
        if (quantize_states) quant_m_group(m_new, cnt, mq + o, ms + g);
        else for (int i = 0; i < cnt; ++i) m32[o + i] = m_new[i];
    }
}

// --------------------------------------------------------------- byte sizes --

// Resident bytes of the compressed optimizer-side state of an n-element
// tensor (what Tables 2, 5 and 7 call "Optim"): rho + m codes (+ v codes) +
// one FP16 scale per group per state (Section 3.2, last paragraphs).
// has_variance: 1 for AdamW, 0 for SGD / Lion.
int64_t fo_oracle_state_bytes(int64_t n, int has_variance) {
    int64_t per_state = n + 2 * n_groups(n);
    return n /*rho*/ + per_state * (has_variance ? 2 : 1);
}

// ---------------------------------------------------------------- checkpoint --
//
// The paper gives the checkpoint's content (2 + 1 + 1 + 1 bytes per parameter,
// Section 3.4) but no file format.  The container used here, little-endian:
//   header, 64 bytes: magic "FOPTCKPT" | u32 version = 1 | u32 kind |
//                     i64 step | i64 n_tensors | i64 total_bytes | zero pad
//   table, 16 bytes per tensor: i64 numel | i64 offset of the tensor's first
//                     section from the start of the blob; padded to 64 bytes
//   per tensor, in list order, each section starting on a 64-byte boundary and
//   zero-padded to the next: theta' (2n) | rho (n) | m codes (n) |
//   m scales (2 ceil(n/32)) | [v codes (n) | v scales (2 ceil(n/32))]
// kind: 0 = AdamW (with the v sections), 1 = SGD, 2 = Lion.

static const char kMagic[8] = {'F', 'O', 'P', 'T', 'C', 'K', 'P', 'T'};

static int64_t tensor_payload(int64_t n, int kind) {
    int64_t b = align64(2 * n) + align64(n) + align64(n) + align64(2 * n_groups(n));
    if (kind == 0) b += align64(n) + align64(2 * n_groups(n));
    return b;
}

int64_t fo_oracle_checkpoint_size(int kind, const int64_t* numels, int64_t n_tensors) {
    if (kind < 0 || kind > 2 || n_tensors < 0) return -1;
    int64_t total = 64 + align64(16 * n_tensors);
    for (int64_t i = 0; i < n_tensors; ++i) {
        if (numels[i] < 0) return -1;
        total += tensor_payload(numels[i], kind);
    }
    return total;
}

static void put_i64(uint8_t* p, int64_t v) { for (int i = 0; i < 8; ++i) p[i] = (uint8_t)((uint64_t)v >> (8 * i)); }
static void put_u32(uint8_t* p, uint32_t v) { for (int i = 0; i < 4; ++i) p[i] = (uint8_t)(v >> (8 * i)); }
static int64_t get_i64(const uint8_t* p) { uint64_t v = 0; for (int i = 0; i < 8; ++i) v |= (uint64_t)p[i] << (8 * i); return (int64_t)v; }
static uint32_t get_u32(const uint8_t* p) { uint32_t v = 0; for (int i = 0; i < 4; ++i) v |= (uint32_t)p[i] << (8 * i); return v; }

// Tensors are handed over as parallel arrays of host pointers.
int fo_oracle_checkpoint_pack(int kind, int64_t n_tensors, const int64_t* numels,
                              const uint16_t* const* thp, const int8_t* const* rho,
                              const int8_t* const* mq, const uint16_t* const* ms,
                              const uint8_t* const* vq, const uint16_t* const* vs,
                              int64_t step, uint8_t* blob, int64_t blob_bytes) {
    int64_t total = fo_oracle_checkpoint_size(kind, numels, n_tensors);
    if (total < 0 || blob_bytes < total) return -1;
    std::memset(blob, 0, (size_t)total);
    std::memcpy(blob, kMagic, 8);
    put_u32(blob + 8, 1u);
    put_u32(blob + 12, (uint32_t)kind);
    put_i64(blob + 16, step);
    put_i64(blob + 24, n_tensors);
    put_i64(blob + 32, total);
    int64_t off = 64 + align64(16 * n_tensors);
    for (int64_t i = 0; i < n_tensors; ++i) {
        const int64_t n = numels[i], ng = n_groups(n);
        put_i64(blob + 64 + 16 * i, n);
        put_i64(blob + 64 + 16 * i + 8, off);
        uint8_t* p = blob + off;
        std::memcpy(p, thp[i], (size_t)(2 * n)); p += align64(2 * n);
        std::memcpy(p, rho[i], (size_t)n);       p += align64(n);
        std::memcpy(p, mq[i], (size_t)n);        p += align64(n);
        std::memcpy(p, ms[i], (size_t)(2 * ng)); p += align64(2 * ng);
        if (kind == 0) {
            std::memcpy(p, vq[i], (size_t)n);        p += align64(n);
            std::memcpy(p, vs[i], (size_t)(2 * ng)); p += align64(2 * ng);
        }
        off += tensor_payload(n, kind);
    }
    return 0;
}

int fo_oracle_checkpoint_unpack(int kind, const uint8_t* blob, int64_t blob_bytes,
                                int64_t n_tensors, const int64_t* numels,
                                uint16_t* const* thp, int8_t* const* rho,
                                int8_t* const* mq, uint16_t* const* ms,
                                uint8_t* const* vq, uint16_t* const* vs, int64_t* step_out) {
    if (blob_bytes < 64 || std::memcmp(blob, kMagic, 8) != 0) return -1;
    if (get_u32(blob + 8) != 1u || get_u32(blob + 12) != (uint32_t)kind) return -1;
    if (get_i64(blob + 24) != n_tensors) return -1;
    int64_t total = fo_oracle_checkpoint_size(kind, numels, n_tensors);
    if (total < 0 || get_i64(blob + 32) != total || blob_bytes < total) return -1;
    int64_t off = 64 + align64(16 * n_tensors);
    for (int64_t i = 0; i < n_tensors; ++i) {
        const int64_t n = numels[i], ng = n_groups(n);
        if (get_i64(blob + 64 + 16 * i) != n || get_i64(blob + 64 + 16 * i + 8) != off) return -1;
        const uint8_t* p = blob + off;
        std::memcpy(thp[i], p, (size_t)(2 * n)); p += align64(2 * n);
        std::memcpy(rho[i], p, (size_t)n);       p += align64(n);
        std::memcpy(mq[i], p, (size_t)n);        p += align64(n);
        std::memcpy(ms[i], p, (size_t)(2 * ng)); p += align64(2 * ng);
        if (kind == 0) {
            std::memcpy(vq[i], p, (size_t)n);        p += align64(n);
            std::memcpy(vs[i], p, (size_t)(2 * ng)); p += align64(2 * ng);
        }
        off += tensor_payload(n, kind);
    }
    *step_out = get_i64(blob + 16);
    return 0;
}

// ------------------------------------------------ exhaustive split statistics --
//
// The experiment of Section 4.4: push FP32 bit patterns through C then C^-1
// and measure the error.  Covers the patterns first, first+stride, ... below
// 2^32 (stride 1 = every FP32 value); non-finite inputs and inputs that round
// to a non-finite BF16 are skipped and counted.  All error arithmetic is in
// double, which represents every quantity here exactly.
//
// out[0] = values measured
// out[1] = values skipped (non-finite theta or theta')
// out[2] = count with |theta - theta'| > ULP(theta')/2           (Section 3.1 interval)
// out[3] = max over values of |theta_hat - theta| / (ULP(theta')/(4N))
// out[4] = max relative error |theta_hat - theta| / |theta| over normal theta
// out[5] = count of bit-exact reconstructions
// out[6] = count of rho outside [-N, N]
// out[7] = count where rounding rho half-away-from-zero would differ from half-even
// out[8] = count where theta' is not the BF16 nearest to theta (checked against both neighbours)
// mean_rel[E] (256 entries, may be null) = mean relative error of the FP32
//          values with biased exponent E.
// directional != 0 runs the experiment under the directional reading of ULP(theta') instead of the
// literal one.  exact_by_exp / count_by_exp (256 entries each, may be null): bit-exact reconstructions
// and values measured among the normal FP32 values with biased exponent E.
void fo_oracle_split_sweep_ex(uint64_t first, uint64_t stride, int N, int directional, double* out,
                              double* mean_rel, double* exact_by_exp, double* count_by_exp, int nthreads) {
    set_threads(nthreads);
    double measured = 0, skipped = 0, viol = 0, exact = 0, range_bad = 0, tie_diff = 0, not_nearest = 0;
    double max_ratio = 0, max_rel = 0;
    double rel_sum[256]; double rel_cnt[256]; double ex_cnt[256];
    for (int i = 0; i < 256; ++i) { rel_sum[i] = 0; rel_cnt[i] = 0; ex_cnt[i] = 0; }
    const uint64_t count = (first < (1ull << 32)) ? (((1ull << 32) - first + stride - 1) / stride) : 0;
#pragma omp parallel
    {
        double l_meas = 0, l_skip = 0, l_viol = 0, l_exact = 0, l_range = 0, l_tie = 0, l_near = 0;
        double l_ratio = 0, l_rel = 0;
        double l_sum[256]; double l_cnt[256]; double l_ex[256];
        for (int i = 0; i < 256; ++i) { l_sum[i] = 0; l_cnt[i] = 0; l_ex[i] = 0; }
#pragma omp for schedule(static)
        for (int64_t j = 0; j < (int64_t)count; ++j) {
            uint32_t bits = (uint32_t)(first + (uint64_t)j * stride);
            float theta = bits_f32(bits);
            if (!std::isfinite(theta)) { l_skip += 1; continue; }
            uint16_t thp; int rho;
            if (directional) split_one_directional(theta, N, &thp, &rho); else split_one(theta, N, &thp, &rho);
            if (!bf16_is_finite(thp)) { l_skip += 1; continue; }
            float hat = directional ? reconstruct_one_directional(thp, rho, N) : reconstruct_one(thp, rho, N);
            l_meas += 1;
            double th = (double)theta, tp = (double)bf16_to_f32(thp);
            int E = (thp >> 7) & 0xff; if (E < 1) E = 1;
            double u = std::ldexp(1.0, E - 134);
            if (std::fabs(th - tp) > u / 2) l_viol += 1;
            // nearest check: neither BF16 neighbour of theta' is strictly closer
            {
                // BF16 values on a signed ordinal line: ..., -2, -1, 0, 1, 2, ...
                int ord = (thp & 0x8000) ? -(int)(thp & 0x7fff) : (int)(thp & 0x7fff);
                double d0 = std::fabs(th - tp);
                for (int step = -1; step <= 1; step += 2) {
                    int o2 = ord + step;
                    int mag = o2 < 0 ? -o2 : o2;
                    if (mag > 0x7f7f) continue;  // neighbour would be infinite
                    uint16_t nb = (uint16_t)((o2 < 0 ? 0x8000 : 0) | mag);
                    if (std::fabs(th - (double)bf16_to_f32(nb)) < d0) { l_near += 1; break; }
                }
            }
            double err = std::fabs((double)hat - th);
            double ratio = err / (u / (4.0 * N));
            if (ratio > l_ratio) l_ratio = ratio;
            const bool is_exact = f32_bits(hat) == bits || (hat == theta);
            if (is_exact) l_exact += 1;
            if (rho < -N || rho > N) l_range += 1;
            // would half-away-from-zero rounding have given a different rho? (literal reading only)
            if (!directional) {
                double en = (th - tp) / (u / 2);
                if (en < -1) en = -1; if (en > 1) en = 1;
                double y = en * N;
                double away = (y >= 0) ? std::floor(y + 0.5) : -std::floor(-y + 0.5);
                if ((int)away != rho) l_tie += 1;
            }
            uint32_t Ef = (bits >> 23) & 0xff;
            if (Ef >= 1) {
                double rel = err / std::fabs(th);
                if (rel > l_rel) l_rel = rel;
                l_sum[Ef] += rel; l_cnt[Ef] += 1;
                if (is_exact) l_ex[Ef] += 1;
            }
        }
#pragma omp critical
        {
            measured += l_meas; skipped += l_skip; viol += l_viol; exact += l_exact;
            range_bad += l_range; tie_diff += l_tie; not_nearest += l_near;
            if (l_ratio > max_ratio) max_ratio = l_ratio;
            if (l_rel > max_rel) max_rel = l_rel;
            for (int i = 0; i < 256; ++i) { rel_sum[i] += l_sum[i]; rel_cnt[i] += l_cnt[i]; ex_cnt[i] += l_ex[i]; }
        }
    }
    out[0] = measured; out[1] = skipped; out[2] = viol; out[3] = max_ratio; out[4] = max_rel;
    out[5] = exact; out[6] = range_bad; out[7] = tie_diff; out[8] = not_nearest;
    if (mean_rel) for (int i = 0; i < 256; ++i) mean_rel[i] = rel_cnt[i] > 0 ? rel_sum[i] / rel_cnt[i] : 0.0;
    if (exact_by_exp) for (int i = 0; i < 256; ++i) exact_by_exp[i] = ex_cnt[i];
    if (count_by_exp) for (int i = 0; i < 256; ++i) count_by_exp[i] = rel_cnt[i];
}
void fo_oracle_split_sweep(uint64_t first, uint64_t stride, int N, double* out, double* mean_rel,
                           int nthreads) {
    fo_oracle_split_sweep_ex(first, stride, N, 0, out, mean_rel, nullptr, nullptr, nthreads);
}
// Array forms of the directional reading (tests only).
void fo_oracle_split_directional(const float* theta, uint16_t* thp, int16_t* rho, int64_t n, int N) {
    for (int64_t i = 0; i < n; ++i) { int r; split_one_directional(theta[i], N, &thp[i], &r); rho[i] = (int16_t)r; }
}
void fo_oracle_reconstruct_directional(const uint16_t* thp, const int16_t* rho, float* theta, int64_t n, int N) {
    for (int64_t i = 0; i < n; ++i) theta[i] = reconstruct_one_directional(thp[i], (int)rho[i], N);
}

int fo_oracle_max_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

}  // extern "C"
