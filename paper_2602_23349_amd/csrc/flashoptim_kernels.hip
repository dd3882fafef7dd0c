// FlashOptim device code for gfx950 (MI355X): the fused optimizer-step kernels
// (paper Algorithms 4, 5, 6), the standalone codecs (Algorithms 1, 2, 3) and the
// checkpoint gather/scatter copy.
//
// Numerical contract.  Every floating-point operation is one IEEE binary32
// operation (round-to-nearest-even, subnormals kept).  This file must be built
// with -ffp-contract=off and correctly rounded division / square root (hipcc's
// default), because 8-bit codes and correction bytes are compared bit for bit
// against an independent CPU implementation of the same algorithms.
// One exception, selected by the EXACT template flag of the AdamW step: with EXACT = false
// (the default entry point) the quotient m_hat / (sqrt(v_hat) + eps) is faithfully rounded
// (within one ulp of the correctly rounded value, and equal to it for all but about one operand
// pair in 10^9); the state codes and scales are unaffected, the master weight can differ by one ulp.
//
// The step is bandwidth-bound by definition (12.25 algorithmic bytes per parameter
// for AdamW), but an exactly rounded body costs on the order of a hundred VALU
// issue slots per parameter, which at 8 TB/s is of the same order as the chip's
// non-packed FP32 rate.  The design choices below are about keeping VALU work per
// element low without changing a single rounding:
//   * decoding a state code is a function of one byte: rho/127, code/255 and
//     phi_m^-1(code/127) come from three 256-entry LDS tables that each workgroup
//     fills once with the same IEEE divisions the definition uses;
//   * the 2^l scalings of Algorithm 1 are LDS tables of exact powers of two indexed by the
//     exponent field of theta' (the decoder multiplies once: exact, or one rounding when
//     the result is subnormal - the same rounding the two-factor form of Algorithm 1
//     performs; the encoder multiplies by two exact factors);
//   * Round(x) to an 8-bit integer is one FP32 addition of 1.5 * 2^23, whose low
//     mantissa byte is the round-half-even integer in two's complement;
//   * BF16 rounding uses the hardware v_cvt_pk_bf16_f32 (two elements per issue);
//   * an 8-bit state code is Round(y) of a value y whose exact evaluation needs an IEEE
//     division (momentum) or square root (variance).  The kernel evaluates y with the 1-ulp hardware
//     reciprocal / with the square root it already has from the update; that estimate provably
//     differs from the exact y by less than a small w.  It rounds estimate - w and estimate + w
//     (v_cvt_pk_u8_f32: round-half-even, saturation and byte packing in one instruction); where both
//     give the same integer the code is decided.  Only when they differ for some lane of the
//     wavefront (a few percent of the wavefronts) are the four elements concerned recomputed with
//     the exact sequence.  Codes are bit-identical to the exact evaluation in every case;
//   * sqrt(v_hat) and m_hat / (sqrt(v_hat) + eps) use the 1-ulp hardware reciprocal square
//     root / reciprocal followed by FMA residual corrections that yield the correctly rounded
//     result for operands inside a stated range (the square root: verified for every value of
//     the range by the device self-test; the division: the classical refinement); a
//     wave-uniform range test selects the general sequence otherwise.  With EXACT = false the
//     division takes one residual correction instead of a refined reciprocal and two (div_faithful).
//
// Work decomposition.  A lane owns 8 consecutive elements per tile: BF16 streams move as
// 128-bit and byte streams as 64-bit accesses, and a quantisation group (32 elements) is a
// lane quad, so the group absmax needs two DPP quad permutes and no LDS.  A workgroup (256
// lanes for AdamW, 512 for SGD and Lion) handles one tile of consecutive elements of one
// tensor; a small two-level table maps the workgroup index to (tensor, tile) so that one call covers a
// whole parameter list, issued as a few consecutive launches.  Stream addresses are a scalar 64-bit
// tile base plus a 32-bit lane offset.

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "flashoptim_device.h"

namespace fo {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float floatx2_t __attribute__((ext_vector_type(2)));

// ------------------------------------------------------------------ helpers --

typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

#ifndef FO_NT_LOAD
#define FO_NT_LOAD 1
#endif
#ifndef FO_NT_STORE
#define FO_NT_STORE 1
#endif

// 128-bit global accesses of the streaming data (each byte is touched once per step).
__device__ __forceinline__ uint4 ld128(const void* p) {
#if FO_NT_LOAD
    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
#else
    const u32x4_t v = *reinterpret_cast<const u32x4_t*>(p);
#endif
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void st128(void* p, uint32_t a, uint32_t b, uint32_t c, uint32_t d) {
    const u32x4_t v = {a, b, c, d};
#if FO_NT_STORE
    __builtin_nontemporal_store(v, reinterpret_cast<u32x4_t*>(p));
#else
    *reinterpret_cast<u32x4_t*>(p) = v;
#endif
}

__device__ __forceinline__ float u2f(uint32_t u) { return __uint_as_float(u); }
__device__ __forceinline__ uint32_t f2u(float f) { return __float_as_uint(f); }

// Maximum over the lanes that share a 32-element group: a lane pair (16 elements per lane)
// or a lane quad (8 per lane).  Each step is ONE instruction, v_max_f32 with its first operand taken
// from the neighbouring lane through a DPP quad permute (written as inline assembly: from the
// builtin the compiler makes a DPP move, two canonicalising maxima and the maximum itself).  The
// s_nop covers the two wait states a DPP read needs after the instruction that wrote its source.
// v_max_f32 returns the other operand when one is NaN, like fmaxf.
__device__ __forceinline__ float max_across_lane_pair(float x) {
    float r;
    asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    return r;
}
__device__ __forceinline__ float max_across_pair_of_pairs(float x) {
    float r;
    asm("s_nop 1\n\tv_max_f32_dpp %0, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf" : "=v"(r) : "v"(x));
    return r;
}
template <int VEC>
__device__ __forceinline__ float group_max(float x) {
    x = max_across_lane_pair(x);
    if (VEC == 8) x = max_across_pair_of_pairs(x);
    return x;
}

// Round-half-even of y (|y| <= 2^21) to an integer, returned in two's complement in the
// low bits of the result.
__device__ __forceinline__ uint32_t round_to_int_bits(float y) { return f2u(y + 12582912.0f); }

// log2 of half the BF16 ULP of the value whose BF16 bit pattern is `b` (Algorithm 1:
// l = floor(log2 ULP(theta')) - 1).  Zero and subnormals use the lowest binade's spacing.
__device__ __forceinline__ int half_ulp_log2(uint32_t b) {
    int E = (int)((b >> 7) & 0xffu);
    E = E < 1 ? 1 : E;
    return E - 135;
}

// BF16 round-to-nearest-even of two floats: a in the low half, b in the high half.
__device__ __forceinline__ uint32_t bf16_pack(float a, float b) {
    floatx2_t f = {a, b};
    bf16x2_t r = __builtin_convertvector(f, bf16x2_t);
    return __builtin_bit_cast(uint32_t, r);
}

// FP16 scale of a group from its FP32 absmax: saturate at 65504, round to nearest even.
// Returns the FP16 bits; *r is the correctly rounded reciprocal of the scale as the decoder
// will read it (0 when the scale is 0, so that every code of the group becomes 0).
__device__ __forceinline__ uint32_t group_scale(float absmax, float* r) {
    const float a = fminf(absmax, 65504.0f);
    const _Float16 h = (_Float16)a;
    const float s = (float)h;
    *r = (s == 0.0f) ? 0.0f : 1.0f / s;
    return (uint32_t)__builtin_bit_cast(uint16_t, h);
}

// Same, with the reciprocal formed as hardware estimate + one Newton step.  The argument takes
// only the 31,743 positive finite FP16 values; for every one of them this sequence returns the
// correctly rounded 1/s (checked exhaustively on the device by flashoptim_selftest).
__device__ __forceinline__ float recip_of_fp16(float s) {
    const float r0 = __builtin_amdgcn_rcpf(s);
    const float e = fmaf(-s, r0, 1.0f);
    return fmaf(e, r0, r0);
}
__device__ __forceinline__ uint32_t group_scale_fast(float absmax, float* r) {
    const float a = fminf(absmax, 65504.0f);
    const _Float16 h = (_Float16)a;
    const float s = (float)h;
    *r = (s == 0.0f) ? 0.0f : recip_of_fp16(s);
    return (uint32_t)__builtin_bit_cast(uint16_t, h);
}

// Correctly rounded square root for 2^-96 <= x <= FLT_MAX: the hardware reciprocal-square-root
// estimate (1 ulp) and one Newton correction, each step one FMA.  That this sequence returns the
// correctly rounded root for EVERY FP32 value of that range is a property of the hardware estimate
// which is verified exhaustively on the device (all 1,879,048,192 values): ahead of the first AdamW
// step on a device (until that check has passed, the device word behind StepConsts::sqrt_min holds +inf
// and the kernels use sqrtf) and by flashoptim_selftest.  Below
// 2^-96 the residual x - s*s leaves the normal range and the result is only within one ulp; zero,
// infinity and NaN give NaN.  Callers check the range and use sqrtf() otherwise.
__device__ __forceinline__ float sqrt_rn_midrange(float x) {
    const float y = __builtin_amdgcn_rsqf(x);
    const float s = x * y, h = 0.5f * y;
    return fmaf(fmaf(-s, s, x), h, s);
}
// Correctly rounded n / d for operands well inside the normal range: 2^-60 <= |n|, d <= 2^60.
// This is the usual refinement of the 1-ulp hardware reciprocal (one Newton step on the
// reciprocal, two residual corrections of the quotient, every step one FMA); with the operands
// in that range no intermediate result leaves the normal range, so the range scaling and the
// special-case fix-up of the general division are not needed.  Callers check the range.
__device__ __forceinline__ float div_rn_midrange(float n, float d) {
    float r = __builtin_amdgcn_rcpf(d);
    const float e = fmaf(-d, r, 1.0f);
    r = fmaf(e, r, r);
    float q = n * r;
    q = fmaf(fmaf(-d, q, n), r, q);
    q = fmaf(fmaf(-d, q, n), r, q);
    return q;
}

// Faithful division: one residual correction of the quotient formed with the 1-ulp hardware reciprocal,
// each step one FMA.  The value before the final rounding is within 2^-23 ulp of the exact quotient, so the
// result is the correctly rounded one except when the exact quotient lies that close to the middle between
// two FP32 numbers; then it is the other neighbour (the device self-test bounds the difference to one ulp and
// counts such operand pairs: 52 among 2^36 random pairs on MI355X, 7.6e-10).  Denominator range as for
// div_rn_midrange.  A numerator below 2^-60 is admitted: down to 2^-103 nothing changes; below that the
// residual can leave the normal range and the error can reach a few ulp of a quotient smaller than 2^-43.
__device__ __forceinline__ float div_faithful(float n, float d) {
    const float r = __builtin_amdgcn_rcpf(d);
    const float q = n * r;
    return fmaf(fmaf(-d, q, n), r, q);
}

// Exact Q_m code (low byte of the result) of one element given the reciprocal group scale
// (Algorithm 2, encoder).
__device__ __forceinline__ uint32_t m_code_exact(float m, float r) {
    const float m1 = m * r;
    const float num = 2.0f * m1;
    const float den = 1.0f + fabsf(m1);
    const float m2 = num / den;
    const float y = __builtin_amdgcn_fmed3f(m2 * 127.0f, -127.0f, 127.0f);
    return round_to_int_bits(y);
}

// The same code decided from an estimate.  m1 and den are formed exactly as above; the quotient uses
// v_rcp_f32 (1 ulp), so y* = 254 * (m1 * rc) differs from the exact y by at most
// (2 + 1 + 1 + 1) * 2^-24 * 128 < 3.9e-5 wherever the clamp is not active.  The function returns
// y* + 128 -+ w, each formed by ONE fused multiply-add (its rounding, half an ulp of a value below 256,
// adds 7.7e-6, and 128 -+ w itself is off by at most 3.9e-6): if both round to the same integer no
// rounding tie lies within 4.7e-5 of y* on either side and that integer is the exact code plus 128.  The
// integers come from v_cvt_pk_u8_f32 (round-half-even, saturating at 0 and 255, one byte of a word per
// instruction): its saturation at 255 is the upper clamp of the code (+127); the lower clamp (-127) is
// the clamp of p at -1/2.
constexpr float kTieWindowM = 6.0e-5f;
__device__ __forceinline__ void m_code_bracket(float m, float r, float* lo, float* hi) {
    const float m1 = m * r;
    const float den = 1.0f + fabsf(m1);
    const float rc = __builtin_amdgcn_rcpf(den);
    const float p = fmaxf(m1 * rc, -0.5f);
    *lo = fmaf(p, 254.0f, 128.0f - kTieWindowM);
    *hi = fmaf(p, 254.0f, 128.0f + kTieWindowM);
}

// Exact Q_v code of one element from v and the reciprocal group scale (Algorithm 3, encoder).
__device__ __forceinline__ uint32_t v_code_exact(float v, float r) {
    const float y = __builtin_amdgcn_fmed3f((sqrtf(v) * r) * 255.0f, 0.0f, 255.0f);
    return round_to_int_bits(y);
}

// The same value when v is known to be inside the range of sqrt_rn_midrange.
__device__ __forceinline__ uint32_t v_code_exact_midrange(float v, float r) {
    const float y = __builtin_amdgcn_fmed3f((sqrt_rn_midrange(v) * r) * 255.0f, 0.0f, 255.0f);
    return round_to_int_bits(y);
}

// The same code decided from root_hat = sqrt(v * rbc2) (exactly rounded, already computed for the update)
// and kr255 = 255 * sqrt(1 / rbc2) * r, formed per group to within one rounding (the host passes the constant
// in two halves).  Relative errors of y* = root_hat * kr255 against the exact argument y of Round(), in units
// of 2^-24: the rounding of v * rbc2 (1/2 after the root), of the root (1), of kr255 (1), against the three
// roundings of the exact chain sqrt, * r, * 255 (3): 5.5 * 2^-24 * 255.5 < 8.4e-5 in y below the saturation
// point.  The function returns y* -+ w, each ONE fused multiply-add (rounding: half an ulp of a value below
// 256, 7.7e-6): if both round to the same integer no rounding tie lies within 9.2e-5 of y*, and that integer
// is the exact code.  The conversion's saturation at 255 is the clamp of Algorithm 3.
constexpr float kTieWindowV = 1.0e-4f;
__device__ __forceinline__ void v_code_bracket(float root_hat, float kr255, float* lo, float* hi) {
    *lo = fmaf(root_hat, kr255, -kTieWindowV);
    *hi = fmaf(root_hat, kr255, kTieWindowV);
}
// Round-half-even of x to 0..255 (saturating; NaN gives 0), placed in byte `k` of `word`.
__device__ __forceinline__ uint32_t put_u8(float x, uint32_t k, uint32_t word) {
    return __builtin_amdgcn_cvt_pk_u8_f32(x, k, word);
}

// Low bytes of four words -> one word (c0 in byte 0).
__device__ __forceinline__ uint32_t pack_low_bytes(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3) {
    const uint32_t t01 = __builtin_amdgcn_perm(c1, c0, 0x0c0c0400u);
    const uint32_t t23 = __builtin_amdgcn_perm(c3, c2, 0x0c0c0400u);
    return __builtin_amdgcn_perm(t23, t01, 0x05040100u);
}

__device__ __forceinline__ bool any_lane(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0; }

// ------------------------------------------------------------- decode tables --

struct DecodeTables {
    float rho[256];    // (float)(int8)i / 127
    float m[256];      // phi_m^-1((float)(int8)i / 127)
    float v[256];      // (float)i / 255
    float half_ulp[256];   // 2^l, l = max(E,1) - 135: half the BF16 ULP of a value with exponent field E
    float2 split[256];     // {2^h, 127 * 2^(-l-h)}, h = floor(-l/2): the two scalings of Algorithm 1's encoder
};

constexpr float pow2_const(int k) {     // 2^k, exact for -149 <= k <= 127
    float x = 1.0f;
    for (int i = 0; i < k; ++i) x *= 2.0f;
    for (int i = 0; i > k; --i) x *= 0.5f;
    return x;
}

// All tables are compile-time constants.  The compiler evaluates constant expressions in
// IEEE binary32 with round-to-nearest-even, so every entry is the result of the same single
// divisions the definitions prescribe (the decoders of Algorithms 1, 2 and 3); the powers of two
// are exact.
constexpr DecodeTables make_decode_tables() {
    DecodeTables t{};
    for (int i = 0; i < 256; ++i) {
        const int sb = i < 128 ? i : i - 256;
        const float z = (float)sb / 127.0f;
        const float az = z < 0.0f ? -z : z;
        t.rho[i] = z;
        t.m[i] = z / (2.0f - az);
        t.v[i] = (float)i / 255.0f;
        const int l = (i < 1 ? 1 : i) - 135;
        const int h = (-l >= 0) ? (-l) / 2 : -((l + 1) / 2);    // floor(-l / 2)
        t.half_ulp[i] = pow2_const(l);
        t.split[i].x = pow2_const(h);
        t.split[i].y = 127.0f * pow2_const(-l - h);
    }
    return t;
}
__device__ const DecodeTables g_decode_tables = make_decode_tables();

// Each workgroup stages the tables (6 KB, L2-resident) into LDS: one entry per lane per table.
// With 512 lanes the two halves of the workgroup share the work.  The staging is split into its
// load half and its store half so that a kernel can issue the loads first of all (they depend on
// nothing) and store to LDS only after it has issued its streaming loads.
struct TableEntries {
    float rho, m, v, half_ulp;
    float2 split;
};
template <int THREADS>
__device__ __forceinline__ void load_table_entries(TableEntries& e, int tid) {
    static_assert(THREADS == 256 || THREADS == 512, "");
    // scalar base + 32-bit lane offset, so that no 64-bit address arithmetic lands on the vector ALU
    typedef const __attribute__((address_space(1))) uint8_t* base_t;
    typedef const __attribute__((address_space(1))) float* fptr_t;
    typedef float f2_t __attribute__((ext_vector_type(2)));
    typedef const __attribute__((address_space(1))) f2_t* f2ptr_t;
    const base_t base = (base_t)&g_decode_tables;
    const uint32_t o4 = (uint32_t)(tid & 255) * 4u;
    if (THREADS == 256 || tid < 256) {
        e.rho = *(fptr_t)(base + offsetof(DecodeTables, rho) + o4);
        e.m = *(fptr_t)(base + offsetof(DecodeTables, m) + o4);
        e.v = *(fptr_t)(base + offsetof(DecodeTables, v) + o4);
    }
    if (THREADS == 256 || tid >= 256) {
        e.half_ulp = *(fptr_t)(base + offsetof(DecodeTables, half_ulp) + o4);
        const f2_t sp = *(f2ptr_t)(base + offsetof(DecodeTables, split) + (o4 + o4));
        e.split = make_float2(sp[0], sp[1]);
    }
}
template <int THREADS>
__device__ __forceinline__ void store_table_entries(DecodeTables& t, const TableEntries& e, int tid) {
    const int i = tid & 255;
    if (THREADS == 256 || tid < 256) {
        t.rho[i] = e.rho;
        t.m[i] = e.m;
        t.v[i] = e.v;
    }
    if (THREADS == 256 || tid >= 256) {
        t.half_ulp[i] = e.half_ulp;
        t.split[i] = e.split;
    }
}

// In-kernel forms of C^-1 and of the rho half of C through the LDS tables.  E is the exponent
// field of theta' (bits 7..14 of its BF16 pattern).
//   C^-1: theta_hat = theta' + q * 2^l.  The product is exact, or rounds once when it is
//         subnormal - exactly what the two-factor form in Algorithm 1's decoder does.
//   C:    rho = Round(((e * 2^h) * (127 * 2^(-l-h)))): both products are exact (e has at most
//         16 significant bits below theta'), so this is Round(e_norm * 127).  For a finite
//         theta' the clamp of Algorithm 1 is the identity (|e| <= 2^l under round-to-nearest);
//         for theta' = +-inf the products are +-inf or NaN and the low mantissa byte of
//         (+-inf or NaN) + 1.5 * 2^23 is 0.
__device__ __forceinline__ float reconstruct_lds(const DecodeTables& t, uint32_t E, float base, float q) {
    return base + (q * t.half_ulp[E]);
}
__device__ __forceinline__ uint32_t rho_bits_lds(const DecodeTables& t, float theta, uint32_t b16, uint32_t E) {
    const float e = theta - u2f(b16 << 16);
    const float2 sc = t.split[E];
    // (e * sc.x) * sc.y is exact, so adding the rounding constant inside one fused multiply-add rounds the same
    // value as Round() of the product would
    return f2u(fmaf(e * sc.x, sc.y, 12582912.0f));
}

// -------------------------------------------------------------- lane vectors --
//
// VEC consecutive elements per lane (8 or 16).  With 16, every stream moves as 128-bit
// accesses and a group of 32 is a lane pair; with 8, the byte streams move as 64-bit
// accesses and a group is a lane quad, but the kernel needs half the registers and more
// wavefronts fit on a SIMD.

template <int VEC>
struct LaneIO {
    uint32_t p[VEC / 2];    // VEC BF16 theta'
    uint32_t g[VEC / 2];    // VEC BF16 gradients
    uint32_t r[VEC / 4];    // VEC INT8 rho
    uint32_t mq[VEC / 4];   // VEC INT8 momentum codes
    uint32_t vq[VEC / 4];   // VEC UINT8 variance codes
    uint32_t ms, vs;        // FP16 scale bits of the lane's group
    // uncompressed halves (ablation variants only; dead otherwise)
    float th32[VEC];        // FP32 master weights when weights are not split
    float m32[VEC];         // FP32 momentum when states are not quantized
    float v32[VEC];         // FP32 variance when states are not quantized
};

// Streaming accesses of a full lane.  Every stream of a tile is addressed as a wave-uniform
// 64-bit base (tensor pointer + tile offset, kept in scalar registers) plus a 32-bit byte offset
// of the lane, and the pointers are marked as global memory: the loads and stores then take the
// "scalar base + vector offset" form and no 64-bit address arithmetic is left on the vector ALU.
typedef const __attribute__((address_space(1))) uint8_t* gcptr_t;
typedef __attribute__((address_space(1))) uint8_t* gptr_t;

// The base is passed through readfirstlane (a register copy for a value that is already uniform)
// so that the compiler keeps it apart from the lane offset instead of folding both into one
// 64-bit vector address.
__device__ __forceinline__ uint64_t uniform_u64(uint64_t v) {
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
    return ((uint64_t)hi << 32) | lo;
}
__device__ __forceinline__ gcptr_t gbase(const void* p, int64_t byte_off) {
    return (gcptr_t)uniform_u64((uint64_t)p + (uint64_t)byte_off);
}
__device__ __forceinline__ gptr_t gbase(void* p, int64_t byte_off) {
    return (gptr_t)uniform_u64((uint64_t)p + (uint64_t)byte_off);
}

// Redefines a 32-bit lane offset at the point of use (an empty asm statement, no instruction):
// its zero-extension then stays next to the access it feeds, which the "scalar base + 32-bit
// vector offset" addressing form requires.
__device__ __forceinline__ uint32_t block_local(uint32_t v) {
    asm volatile("" : "+v"(v));
    return v;
}

// 4 * N bytes from / to base + byte_off (4N-byte aligned, N <= 4)
template <int N>
__device__ __forceinline__ void gld(uint32_t (&w)[N], gcptr_t base, uint32_t byte_off) {
    static_assert(N == 2 || N == 4, "");
    typedef uint32_t vec_t __attribute__((ext_vector_type(N)));
    typedef const __attribute__((address_space(1))) vec_t* vptr_t;
#if FO_NT_LOAD
    const vec_t v = __builtin_nontemporal_load((vptr_t)(base + byte_off));
#else
    const vec_t v = *(vptr_t)(base + byte_off);
#endif
#pragma unroll
    for (int k = 0; k < N; ++k) w[k] = v[k];
}
template <int N>
__device__ __forceinline__ void gst(gptr_t base, uint32_t byte_off, const uint32_t (&w)[N]) {
    static_assert(N == 2 || N == 4, "");
    typedef uint32_t vec_t __attribute__((ext_vector_type(N)));
    typedef __attribute__((address_space(1))) vec_t* vptr_t;
    vec_t v;
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] = w[k];
#if FO_NT_STORE
    __builtin_nontemporal_store(v, (vptr_t)(base + byte_off));
#else
    *(vptr_t)(base + byte_off) = v;
#endif
}
// 4 * N bytes as consecutive 16-byte (or one 8-byte) accesses
template <int N>
__device__ __forceinline__ void gld_words(uint32_t (&w)[N], gcptr_t base, uint32_t byte_off) {
    if constexpr (N <= 4) {
        gld(w, base, byte_off);
    } else {
        static_assert(N % 4 == 0, "");
#pragma unroll
        for (int k = 0; k < N / 4; ++k) {
            uint32_t t[4];
            gld(t, base, byte_off + 16u * k);
            w[4 * k] = t[0]; w[4 * k + 1] = t[1]; w[4 * k + 2] = t[2]; w[4 * k + 3] = t[3];
        }
    }
}
template <int N>
__device__ __forceinline__ void gst_words(gptr_t base, uint32_t byte_off, const uint32_t (&w)[N]) {
    if constexpr (N <= 4) {
        gst(base, byte_off, w);
    } else {
        static_assert(N % 4 == 0, "");
#pragma unroll
        for (int k = 0; k < N / 4; ++k) {
            const uint32_t t[4] = {w[4 * k], w[4 * k + 1], w[4 * k + 2], w[4 * k + 3]};
            gst(base, byte_off + 16u * k, t);
        }
    }
}
// FP32 streams (ablation variants): VEC floats per lane are two or more 16-byte accesses, each of
// which covers only part of every cache line the wavefront touches.  These go without the
// non-temporal hint: with it the line is not kept between the two accesses and is fetched
// twice (measured 26.8 vs 19.9 ms for the variant with FP32 weights on the Llama list).
template <int VEC>
__device__ __forceinline__ void gld_floats(float (&f)[VEC], gcptr_t base, uint32_t byte_off) {
    static_assert(VEC % 4 == 0, "");
    typedef float vec_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int k = 0; k < VEC / 4; ++k) {
        const vec_t v = *(const __attribute__((address_space(1))) vec_t*)(base + byte_off + 16u * k);
        f[4 * k] = v[0]; f[4 * k + 1] = v[1]; f[4 * k + 2] = v[2]; f[4 * k + 3] = v[3];
    }
}
template <int VEC>
__device__ __forceinline__ void gst_floats(gptr_t base, uint32_t byte_off, const float (&f)[VEC]) {
    static_assert(VEC % 4 == 0, "");
    typedef float vec_t __attribute__((ext_vector_type(4)));
#pragma unroll
    for (int k = 0; k < VEC / 4; ++k) {
        const vec_t v = {f[4 * k], f[4 * k + 1], f[4 * k + 2], f[4 * k + 3]};
        *(__attribute__((address_space(1))) vec_t*)(base + byte_off + 16u * k) = v;
    }
}
__device__ __forceinline__ uint32_t gld_u16(gcptr_t base, uint32_t byte_off) {
    return *(const __attribute__((address_space(1))) uint16_t*)(base + byte_off);
}
__device__ __forceinline__ void gst_u16(gptr_t base, uint32_t byte_off, uint32_t v) {
    *(__attribute__((address_space(1))) uint16_t*)(base + byte_off) = (uint16_t)v;
}

// A full lane: tile0 = index of the tile's first element in the tensor (wave-uniform, a multiple
// of 32), lane_el = index of the lane's first element inside the tile (a multiple of VEC).
template <int VEC, bool HAS_V, bool SPLIT, bool QUANT>
__device__ __forceinline__ void load_full(LaneIO<VEC>& x, const TensorDev& T, int64_t tile0, uint32_t lane_el) {
    lane_el = block_local(lane_el);
    if (SPLIT) {
        gld_words(x.p, gbase(T.param, 2 * tile0), 2u * lane_el);
        gld_words(x.r, gbase(T.rho, tile0), lane_el);
    } else {
        gld_floats(x.th32, gbase(T.theta32, 4 * tile0), 4u * lane_el);
    }
    gld_words(x.g, gbase(T.grad, 2 * tile0), 2u * lane_el);
    if (QUANT) {
        const uint32_t scale_off = (lane_el >> 5) * 2u;
        gld_words(x.mq, gbase(T.m_q, tile0), lane_el);
        x.ms = gld_u16(gbase(T.m_scale, (tile0 >> 5) * 2), scale_off);
        if (HAS_V) {
            gld_words(x.vq, gbase(T.v_q, tile0), lane_el);
            x.vs = gld_u16(gbase(T.v_scale, (tile0 >> 5) * 2), scale_off);
        }
    } else {
        gld_floats(x.m32, gbase(T.m32, 4 * tile0), 4u * lane_el);
        if (HAS_V) gld_floats(x.v32, gbase(T.v32, 4 * tile0), 4u * lane_el);
    }
}

// Ragged end of a tensor: element-wise loads, missing elements read as zero (a zero
// element yields zero moments and therefore never raises its group's absmax).
template <int VEC, bool HAS_V, bool SPLIT, bool QUANT>
__device__ __forceinline__ void load_tail(LaneIO<VEC>& x, const TensorDev& T, int64_t off, int cnt) {
    const uint16_t* p = reinterpret_cast<const uint16_t*>(T.param) + off;
    const uint16_t* g = reinterpret_cast<const uint16_t*>(T.grad) + off;
    const uint8_t* r = reinterpret_cast<const uint8_t*>(T.rho) + off;
    const uint8_t* mq = reinterpret_cast<const uint8_t*>(T.m_q) + off;
    const uint8_t* vq = T.v_q + off;
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j) {
        uint32_t lo = (2 * j < cnt) ? g[2 * j] : 0u, hi = (2 * j + 1 < cnt) ? g[2 * j + 1] : 0u;
        x.g[j] = lo | (hi << 16);
        if (SPLIT) {
            lo = (2 * j < cnt) ? p[2 * j] : 0u; hi = (2 * j + 1 < cnt) ? p[2 * j + 1] : 0u;
            x.p[j] = lo | (hi << 16);
        }
    }
#pragma unroll
    for (int j = 0; j < VEC / 4; ++j) {
        uint32_t w = 0, wm = 0, wv = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            if (4 * j + k < cnt) {
                if (SPLIT) w |= (uint32_t)r[4 * j + k] << (8 * k);
                if (QUANT) wm |= (uint32_t)mq[4 * j + k] << (8 * k);
                if (QUANT && HAS_V) wv |= (uint32_t)vq[4 * j + k] << (8 * k);
            }
        }
        x.r[j] = w; x.mq[j] = wm; x.vq[j] = wv;
    }
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if (!SPLIT) x.th32[i] = (i < cnt) ? T.theta32[off + i] : 0.0f;
        if (!QUANT) x.m32[i] = (i < cnt) ? T.m32[off + i] : 0.0f;
        if (!QUANT && HAS_V) x.v32[i] = (i < cnt) ? T.v32[off + i] : 0.0f;
    }
    x.ms = 0; x.vs = 0;
    if (QUANT && cnt > 0) {
        x.ms = T.m_scale[off >> 5];
        if (HAS_V) x.vs = T.v_scale[off >> 5];
    }
}

template <int VEC, bool HAS_V, bool SPLIT, bool QUANT>
__device__ __forceinline__ void store_full(const LaneIO<VEC>& y, const TensorDev& T, int64_t tile0, uint32_t lane_el,
                                           bool group_leader) {
    lane_el = block_local(lane_el);
    if (SPLIT) {
        gst_words(gbase(T.param, 2 * tile0), 2u * lane_el, y.p);
        gst_words(gbase(T.rho, tile0), lane_el, y.r);
    } else {
        gst_floats(gbase(T.theta32, 4 * tile0), 4u * lane_el, y.th32);
    }
    if (QUANT) {
        gst_words(gbase(T.m_q, tile0), lane_el, y.mq);
        if (HAS_V) gst_words(gbase(T.v_q, tile0), lane_el, y.vq);
        if (group_leader) {
            const uint32_t scale_off = (lane_el >> 5) * 2u;
            gst_u16(gbase(T.m_scale, (tile0 >> 5) * 2), scale_off, y.ms);
            if (HAS_V) gst_u16(gbase(T.v_scale, (tile0 >> 5) * 2), scale_off, y.vs);
        }
    } else {
        gst_floats(gbase(T.m32, 4 * tile0), 4u * lane_el, y.m32);
        if (HAS_V) gst_floats(gbase(T.v32, 4 * tile0), 4u * lane_el, y.v32);
    }
}

template <int VEC, bool HAS_V, bool SPLIT, bool QUANT>
__device__ __forceinline__ void store_tail(const LaneIO<VEC>& y, const TensorDev& T, int64_t off, int cnt,
                                           bool group_leader) {
    uint16_t* p = reinterpret_cast<uint16_t*>(T.param) + off;
    uint8_t* r = reinterpret_cast<uint8_t*>(T.rho) + off;
    uint8_t* mq = reinterpret_cast<uint8_t*>(T.m_q) + off;
    uint8_t* vq = T.v_q + off;
#pragma unroll
    for (int i = 0; i < VEC; ++i) {
        if (i < cnt) {
            if (SPLIT) {
                p[i] = (uint16_t)(y.p[i >> 1] >> (16 * (i & 1)));
                r[i] = (uint8_t)(y.r[i >> 2] >> (8 * (i & 3)));
            } else {
                T.theta32[off + i] = y.th32[i];
            }
            if (QUANT) {
                mq[i] = (uint8_t)(y.mq[i >> 2] >> (8 * (i & 3)));
                if (HAS_V) vq[i] = (uint8_t)(y.vq[i >> 2] >> (8 * (i & 3)));
            } else {
                T.m32[off + i] = y.m32[i];
                if (HAS_V) T.v32[off + i] = y.v32[i];
            }
        }
    }
    if (QUANT && group_leader && cnt > 0) {
        T.m_scale[off >> 5] = (uint16_t)y.ms;
        if (HAS_V) T.v_scale[off >> 5] = (uint16_t)y.vs;
    }
}

// ------------------------------------------------------- the per-lane update --
//
// Splits (or stores as FP32) the four new master weights of block j of a lane.
template <int VEC, bool SPLIT>
__device__ __forceinline__ void split_block(LaneIO<VEC>& y, const DecodeTables& tab, const float (&tht)[4], int j) {
    if (SPLIT) {
        const uint32_t w0 = bf16_pack(tht[0], tht[1]), w1 = bf16_pack(tht[2], tht[3]);
        y.p[2 * j] = w0;
        y.p[2 * j + 1] = w1;
        const uint32_t e0 = w0 << 1, e1 = w1 << 1;     // exponent fields on byte boundaries
        y.r[j] = pack_low_bytes(rho_bits_lds(tab, tht[0], w0 & 0xffffu, (e0 >> 8) & 0xffu),
                                rho_bits_lds(tab, tht[1], w0 >> 16, e0 >> 24),
                                rho_bits_lds(tab, tht[2], w1 & 0xffffu, (e1 >> 8) & 0xffu),
                                rho_bits_lds(tab, tht[3], w1 >> 16, e1 >> 24));
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) y.th32[4 * j + k] = tht[k];
    }
}

// KIND: 0 AdamW (Algorithm 4), 1 SGD (Algorithm 5), 2 Lion (Algorithm 6).
// Operates on the VEC elements of one lane; the lanes holding the rest of the same 32-element
// group (lane ^ 1, and lane ^ 2, lane ^ 3 when VEC == 8) must execute this function with it.
// SPLIT / QUANT: the paper's ablations (Section 4.3).  SPLIT = false keeps the master weight in
// FP32 (x.th32 -> y.th32); QUANT = false keeps the states in FP32 (x.m32, x.v32 -> y.m32, y.v32).
// EXACT (AdamW only): the quotient m_hat / (sqrt(v_hat) + eps) is the correctly rounded one for every
// input; otherwise it is the faithful form above.  Everything else, the square root, the state codes and
// the scales included, is exact in both modes.
template <int KIND, int VEC, bool SPLIT, bool QUANT, bool EXACT>
__device__ __forceinline__ void update_lane(const LaneIO<VEC>& x, LaneIO<VEC>& y, const DecodeTables& tab,
                                            const StepConsts& c, float lr, float wd) {
    constexpr bool HAS_V = (KIND == 0);
    const float s_m = QUANT ? (float)__builtin_bit_cast(_Float16, (uint16_t)x.ms) : 0.0f;
    const float s_v = (QUANT && HAS_V) ? (float)__builtin_bit_cast(_Float16, (uint16_t)x.vs) : 0.0f;

    float mt[VEC];    // new momentum
    float vt[VEC];    // new variance (AdamW)
    float rh[VEC];    // sqrt of the bias-corrected new variance (AdamW)
    float tha[VEC];   // AdamW: master weights, held until the range tests below are known
    float amax_m = 0.0f, amax_v = 0.0f;
    float amin_m = 3.0e38f, amin_v = 3.0e38f;     // AdamW: smallest |m_t| and v_t of the lane
    bool fast = false;                            // AdamW: the wavefront takes the short square root and division

#pragma unroll
    for (int j = 0; j < VEC / 4; ++j) {
        // four elements at a time (one word of each byte stream)
        float tht[4];     // new master weights of this block (SGD, Lion)
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            const int i = 4 * j + k;
            const uint32_t gw = x.g[i >> 1];
            const float g = (i & 1) ? u2f(gw & 0xffff0000u) : u2f(gw << 16);
            // prologue: reconstruct optimizer state and master weight
            float m, th;
            if (QUANT) {
                const uint32_t mb = (x.mq[j] >> (8 * k)) & 0xffu;
                m = tab.m[mb] * s_m;                                 // Q_m^-1
            } else {
                m = x.m32[i];
            }
            if (SPLIT) {
                const uint32_t pw = x.p[i >> 1];
                // (pair << 1) puts the two exponent fields on byte boundaries (bytes 1 and 3)
                const uint32_t pE = (i & 1) ? ((pw << 1) >> 24) : (((pw << 1) >> 8) & 0xffu);
                const float base = (i & 1) ? u2f(pw & 0xffff0000u) : u2f(pw << 16);
                const uint32_t rb = (x.r[j] >> (8 * k)) & 0xffu;
                th = reconstruct_lds(tab, pE, base, tab.rho[rb]);    // C^-1
            } else {
                th = x.th32[i];
            }
            float m_new;
            if (KIND == 0) {
                float v;
                if (QUANT) {
                    const uint32_t vb = (x.vq[j] >> (8 * k)) & 0xffu;
                    const float v1 = tab.v[vb] * s_v;                // Q_v^-1
                    v = v1 * v1;
                } else {
                    v = x.v32[i];
                }
                m_new = (c.beta1 * m) + (c.omb1 * g);
                const float gg = g * g;
                const float v_new = (c.beta2 * v) + (c.omb2 * gg);
                tha[i] = th;
                vt[i] = v_new;
                amax_v = fmaxf(amax_v, v_new);
                amin_v = fminf(amin_v, v_new);
                amin_m = fminf(amin_m, fabsf(m_new));
            } else if (KIND == 1) {
                m_new = (c.beta1 * m) + g;                           // beta1 carries the momentum mu
                tht[k] = th - (lr * (m_new + (wd * th)));
            } else {
                const float cc = (c.beta1 * m) + (c.omb1 * g);
                const float u = (cc > 0.0f) ? 1.0f : ((cc < 0.0f) ? -1.0f : 0.0f);
                m_new = (c.beta2 * m) + (c.omb2 * g);
                tht[k] = th - (lr * (u + (wd * th)));
            }
            mt[i] = m_new;
            amax_m = fmaxf(amax_m, fabsf(m_new));
        }
        // epilogue, part 1 (SGD, Lion): split the new master weights of this block
        if (KIND != 0) split_block<VEC, SPLIT>(y, tab, tht, j);
    }
    if (KIND == 0) {
        // One wave-uniform range test, on the raw extremes of every lane, selects the short square root
        // and the short division for the whole wavefront (else sqrtf and the IEEE division throughout: same
        // results).  The bias corrections rbc1, rbc2 are at least 1 and multiplying by them is monotone, so
        //   v_t >= 2^-96 for every element   =>  v_hat, and v_t itself, are in the short square root's range;
        //   v_t <= c.v_max (2^60 / rbc2, rounded down)   =>  v_hat <= 2^60: finite, and sqrt(v_hat) + eps is a
        //                                                    denominator well inside the normal range;
        //   |m_t| <= c.m_max (2^60 / rbc1, rounded down) and, for the correctly rounded division only,
        //   |m_t| >= 2^-60   =>  the numerator m_hat is in the short division's range.
        // The host sets v_max = m_max = -1 when eps is outside [2^-60, 1], and sqrt_min = +inf when the short
        // square root is not to be used on this device: every test then fails.  Exact zeros fail it too.
        fast = !(any_lane(!(amax_v <= c.v_max)) | any_lane(!(amin_v >= c.sqrt_min)) |
                 any_lane(!(amax_m <= c.m_max)) | (EXACT ? any_lane(!(amin_m >= kDivFastLo)) : false));
#pragma unroll
        for (int j = 0; j < VEC / 4; ++j) {
            float mh4[4], vh4[4], quo[4], tht[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                mh4[k] = mt[4 * j + k] * c.rbc1;
                vh4[k] = vt[4 * j + k] * c.rbc2;
            }
            if (!fast) {
#pragma unroll
                for (int k = 0; k < 4; ++k) rh[4 * j + k] = sqrtf(vh4[k]);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) rh[4 * j + k] = sqrt_rn_midrange(vh4[k]);
            }
            if (!fast) {
#pragma unroll
                for (int k = 0; k < 4; ++k) quo[k] = mh4[k] / (rh[4 * j + k] + c.eps);
            } else if (EXACT) {
#pragma unroll
                for (int k = 0; k < 4; ++k) quo[k] = div_rn_midrange(mh4[k], rh[4 * j + k] + c.eps);
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) quo[k] = div_faithful(mh4[k], rh[4 * j + k] + c.eps);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const float upd = quo[k] + (wd * tha[4 * j + k]);
                tht[k] = tha[4 * j + k] - (lr * upd);
            }
            // epilogue, part 1 (AdamW): split the new master weights of this block
            split_block<VEC, SPLIT>(y, tab, tht, j);
        }
    }
    if (!QUANT) {
#pragma unroll
        for (int i = 0; i < VEC; ++i) {
            y.m32[i] = mt[i];
            if (HAS_V) y.v32[i] = vt[i];
        }
        return;
    }

    // epilogue, part 2: group scales (one DPP swap joins the two lanes of a group).  The square root
    // is monotone, so the group maximum of sqrt(v) is the square root of the maximum of v.
    amax_m = group_max<VEC>(amax_m);
    float r_m, r_v = 0.0f, kr255 = 0.0f;
    y.ms = group_scale_fast(amax_m, &r_m);
    if (HAS_V) {
        // the group's maximum lies between the extremes of the wavefront's lanes: in the short root's range if they are
        amax_v = group_max<VEC>(amax_v);
        const float root_max = fast ? sqrt_rn_midrange(amax_v) : sqrtf(amax_v);
        y.vs = group_scale_fast(root_max, &r_v);
        // 255 * sqrt(1 / rbc2) * r_v to within one rounding: the constant comes from the host as the two halves of
        // its double-precision value
        kr255 = fmaf(c.k255_hi, r_v, c.k255_lo * r_v);
    }
    const bool vt_root_general = !fast;
    // epilogue: state codes, four at a time (one word of each code stream).  Each code is converted
    // twice, from the two ends of an interval that contains the exact argument of Round(); where the
    // two words differ some element of the block may sit on the other side of a rounding tie, and the
    // block is recomputed with the exact sequence (for the whole wavefront: a few percent of the blocks).
#pragma unroll
    for (int j = 0; j < VEC / 4; ++j) {
        uint32_t lo_w = 0, hi_w = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float lo, hi;
            m_code_bracket(mt[4 * j + k], r_m, &lo, &hi);
            lo_w = put_u8(lo, k, lo_w);
            hi_w = put_u8(hi, k, hi_w);
        }
        if (any_lane(lo_w != hi_w)) {
            y.mq[j] = pack_low_bytes(m_code_exact(mt[4 * j], r_m), m_code_exact(mt[4 * j + 1], r_m),
                                     m_code_exact(mt[4 * j + 2], r_m), m_code_exact(mt[4 * j + 3], r_m));
        } else {
            y.mq[j] = lo_w ^ 0x80808080u;      // code + 128 -> two's complement
        }
        if (HAS_V) {
            lo_w = 0; hi_w = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                float lo, hi;
                v_code_bracket(rh[4 * j + k], kr255, &lo, &hi);
                lo_w = put_u8(lo, k, lo_w);
                hi_w = put_u8(hi, k, hi_w);
            }
            if (any_lane(lo_w != hi_w)) {
                // exact recomputation; the short exact root serves when every v_t of the wavefront
                // is in its range (v_t and v_hat differ by the factor rbc2 >= 1: a separate test)
                uint32_t cv[4];
                if (vt_root_general) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) cv[k] = v_code_exact(vt[4 * j + k], r_v);
                } else {
#pragma unroll
                    for (int k = 0; k < 4; ++k) cv[k] = v_code_exact_midrange(vt[4 * j + k], r_v);
                }
                y.vq[j] = pack_low_bytes(cv[0], cv[1], cv[2], cv[3]);
            } else {
                y.vq[j] = lo_w;
            }
        }
    }
}

// ------------------------------------------------------------ step kernels --
// The tensor and the tile within it that workgroup blockIdx.x handles.  Every load is wave-uniform
// (scalar).  The search loop ends at the last tensor at the latest.
template <bool DIRECT>
__device__ __forceinline__ int64_t locate_tile(const StepArgs& a, TensorDev& T) {
    const uint32_t b = blockIdx.x + a.block_offset;
    if (DIRECT) {
        T = a.single;
        return (int64_t)b;
    }
    uint32_t t = a.coarse[b >> a.coarse_shift];
    T = a.tensors[t];
    while (b - T.first_tile >= T.n_tiles && t + 1 < a.n_tensors) {
        ++t;
        T = a.tensors[t];
    }
    return (int64_t)(b - T.first_tile);
}


// One tile of one tensor.  FULL: every lane of the workgroup holds VEC elements (all tiles of a
// tensor but possibly its last); the code then has no per-lane case distinction at all.
// (Variants in which a workgroup loads two or four such tiles up front and then updates them in
// turn - fewer look-ups, more bytes in flight per workgroup - ran at the same rate.)
template <int KIND, int VEC, int THREADS, bool SPLIT, bool QUANT, bool EXACT, bool FULL>
__device__ __forceinline__ void step_tile(const TensorDev& T, const StepConsts& c, DecodeTables& tab,
                                          const TableEntries& entries, int64_t tile0, int tile_cnt, int tid) {
    constexpr bool HAS_V = (KIND == 0);
    const bool leader = (tid & (kGroup / VEC - 1)) == 0;
    const uint32_t lane_el = (uint32_t)tid * VEC;              // first element of the lane inside its tile
    // the number of the tile's elements that fall to this lane
    const int left = tile_cnt - (int)lane_el;
    const int cnt = FULL ? VEC : (left >= VEC ? VEC : (left > 0 ? left : 0));
    LaneIO<VEC> x, y;
    if (FULL || cnt == VEC) load_full<VEC, HAS_V, SPLIT, QUANT>(x, T, tile0, lane_el);
    else load_tail<VEC, HAS_V, SPLIT, QUANT>(x, T, tile0 + lane_el, cnt);
    store_table_entries<THREADS>(tab, entries, tid);
    __syncthreads();
    // All lanes of a group run the update together (a lane with cnt == 0 may share its group
    // with lanes that hold elements); lanes past the end compute on zeros and store nothing.
    update_lane<KIND, VEC, SPLIT, QUANT, EXACT>(x, y, tab, c, T.lr, T.wd);
    if (FULL || cnt == VEC) store_full<VEC, HAS_V, SPLIT, QUANT>(y, T, tile0, lane_el, leader);
    else store_tail<VEC, HAS_V, SPLIT, QUANT>(y, T, tile0 + lane_el, cnt, leader);
}

// A workgroup handles one tile of one tensor and then retires (persistent workgroups that loop
// over many tiles were measured 10 % slower: an iteration's loads then wait behind the previous
// iteration's stores).  Order of issue: decode-table loads, the (tensor, tile) look-up, the
// streaming loads; then the tables go to LDS.
template <int KIND, int VEC, int THREADS, bool DIRECT, bool SPLIT, bool QUANT, bool EXACT>
__global__ __launch_bounds__(THREADS) void step_kernel(StepArgs a) {
    constexpr int kTile = THREADS * VEC;       // elements per workgroup
    __shared__ DecodeTables tab;
    const int tid = (int)threadIdx.x;
    TableEntries entries;
    load_table_entries<THREADS>(entries, tid);
    TensorDev T;
    const int64_t chunk = locate_tile<DIRECT>(a, T);
    const int64_t tile0 = chunk * (int64_t)kTile;              // first element of the tile (wave-uniform)
    const int64_t rem = T.numel - tile0;                       // elements from there to the tensor's end
    StepConsts c = a.c;
    if (KIND == 0) c.sqrt_min = *a.sqrt_min_word;              // one scalar load, needed only after the streaming loads
    if (rem >= kTile) {
        step_tile<KIND, VEC, THREADS, SPLIT, QUANT, EXACT, true>(T, c, tab, entries, tile0, kTile, tid);
    } else {
        step_tile<KIND, VEC, THREADS, SPLIT, QUANT, EXACT, false>(T, c, tab, entries, tile0, rem > 0 ? (int)rem : 0,
                                                                 tid);
    }
}

template <int KIND, bool SPLIT, bool QUANT, bool EXACT>
static hipError_t launch_variant(bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s) {
    constexpr int VEC = step_vec(KIND), THREADS = step_threads(KIND);
    const dim3 grid((unsigned)n_blocks), block(THREADS);
    if (direct) hipLaunchKernelGGL((step_kernel<KIND, VEC, THREADS, true, SPLIT, QUANT, EXACT>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((step_kernel<KIND, VEC, THREADS, false, SPLIT, QUANT, EXACT>), grid, block, 0, s, a);
    return hipGetLastError();
}

template <int KIND>
static hipError_t launch_kind(bool direct, bool split, bool quant, const StepArgs& a, int64_t n_blocks,
                              hipStream_t s) {
    if (split && quant) return launch_variant<KIND, true, true, true>(direct, a, n_blocks, s);
    if (split) return launch_variant<KIND, true, false, true>(direct, a, n_blocks, s);
    if (quant) return launch_variant<KIND, false, true, true>(direct, a, n_blocks, s);
    return launch_variant<KIND, false, false, true>(direct, a, n_blocks, s);
}

// exact = false selects the faithful division; it exists for AdamW in the compressed
// layout only (SGD and Lion have neither operation; the ablation variants are always exact).
hipError_t launch_step(int kind, bool direct, bool split, bool quant, bool exact, const StepArgs& a, int64_t n_blocks,
                       hipStream_t s) {
    if (kind == 0 && !a.sqrt_min_word) return hipErrorInvalidValue;     // the AdamW kernels dereference it
    if (kind == 0 && split && quant && !exact) return launch_variant<0, true, true, false>(direct, a, n_blocks, s);
    if (kind == 0) return launch_kind<0>(direct, split, quant, a, n_blocks, s);
    if (kind == 1) return launch_kind<1>(direct, split, quant, a, n_blocks, s);
    return launch_kind<2>(direct, split, quant, a, n_blocks, s);
}

// ------------------------------------------------------------- stream probe --
//
// Moves exactly the bytes of one optimizer step with no arithmetic: every stream the step reads is
// read (gradients included) and every stream it writes is written back unchanged, through the same
// tile look-up, lane layout and access instructions.  Its rate is what the memory system delivers
// for this access pattern, the ceiling the step kernel's rate is compared with.
template <int KIND, int VEC, int THREADS, bool DIRECT>
__global__ __launch_bounds__(THREADS) void probe_kernel(StepArgs a) {
    constexpr bool HAS_V = (KIND == 0);
    constexpr int kTile = THREADS * VEC;
    const int tid = (int)threadIdx.x;
    TensorDev T;
    const int64_t chunk = locate_tile<DIRECT>(a, T);
    const bool leader = (tid & (kGroup / VEC - 1)) == 0;
    const uint32_t lane_el = (uint32_t)tid * VEC;
    const int64_t tile0 = chunk * (int64_t)kTile;
    const int64_t rem = T.numel - tile0;
    const int tile_cnt = rem >= kTile ? kTile : (int)rem;
    const int left = tile_cnt - (int)lane_el;
    const int cnt = left >= VEC ? VEC : (left > 0 ? left : 0);
    LaneIO<VEC> x;
    if (cnt == VEC) load_full<VEC, HAS_V, true, true>(x, T, tile0, lane_el);
    else load_tail<VEC, HAS_V, true, true>(x, T, tile0 + lane_el, cnt);
    // The gradient takes no part in what is stored; an empty asm statement that names its registers
    // keeps the load from being removed.
#pragma unroll
    for (int j = 0; j < VEC / 2; ++j) asm volatile("" : : "v"(x.g[j]));
    if (cnt == VEC) store_full<VEC, HAS_V, true, true>(x, T, tile0, lane_el, leader);
    else store_tail<VEC, HAS_V, true, true>(x, T, tile0 + lane_el, cnt, leader);
}

hipError_t launch_probe(int kind, bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s) {
    const dim3 grid((unsigned)n_blocks);
#define FO_PROBE(K, DR) hipLaunchKernelGGL((probe_kernel<K, step_vec(K), step_threads(K), DR>), grid, \
                                           dim3(step_threads(K)), 0, s, a)
    if (kind == 0) { if (direct) FO_PROBE(0, true); else FO_PROBE(0, false); }
    else if (kind == 1) { if (direct) FO_PROBE(1, true); else FO_PROBE(1, false); }
    else { if (direct) FO_PROBE(2, true); else FO_PROBE(2, false); }
#undef FO_PROBE
    return hipGetLastError();
}

// ------------------------------------------------------------ clock monitor --
//
// A measurement aid: ONE lane samples the shader clock while other kernels run.  Each sample spans
// ticks_per_sample ticks of the fixed-frequency counter (wall_clock64) and stores how many ticks and how many
// shader-clock cycles (clock64) went by; cycles / ticks x tick rate is the clock the compute units ran at
// in that interval.  The wait is bounded, so the kernel ends by itself after n_samples samples at the latest.
__global__ __launch_bounds__(64) void clock_monitor_kernel(unsigned long long* samples, int n_samples,
                                                           unsigned long long ticks_per_sample) {
    if (threadIdx.x != 0) return;
    for (int s = 0; s < n_samples; ++s) {
        const unsigned long long r0 = wall_clock64(), c0 = clock64();
        for (int it = 0; it < (1 << 22); ++it) {
            if (wall_clock64() - r0 >= ticks_per_sample) break;
            __builtin_amdgcn_s_sleep(8);
        }
        samples[2 * s] = wall_clock64() - r0;
        samples[2 * s + 1] = clock64() - c0;
    }
}
hipError_t launch_clock_monitor(unsigned long long* samples, int n_samples, unsigned long long ticks_per_sample,
                                hipStream_t s) {
    hipLaunchKernelGGL(clock_monitor_kernel, dim3(1), dim3(64), 0, s, samples, n_samples, ticks_per_sample);
    return hipGetLastError();
}

// -------------------------------------------------------- standalone codecs --
//
// Not on the per-step path (used at initialisation, for inspection and by tests).  They share
// the lane layout of the step kernels: a workgroup of 256 lanes covers a tile of 2048 consecutive
// elements, 8 per lane, so that BF16 data moves as 128-bit, byte data as 64-bit and FP32 data as
// two 128-bit accesses per lane, and a quantisation group is a lane quad.  The arithmetic is the
// plain exact form of each operation.

constexpr int kCodecVec = 8;
constexpr int kCodecTile = kThreads * kCodecVec;

struct LanePos {
    int64_t tile0;       // first element of the workgroup's tile (wave-uniform)
    uint32_t lane_el;    // first element of the lane inside the tile
    int cnt;             // elements of the lane that exist: kCodecVec, or fewer at the ragged end
};
__device__ __forceinline__ LanePos lane_pos_at(int64_t tile0, int64_t n) {
    LanePos L;
    L.tile0 = tile0;
    L.lane_el = (uint32_t)threadIdx.x * kCodecVec;
    const int64_t rem = n - tile0;
    const int tile_cnt = rem >= kCodecTile ? kCodecTile : (rem > 0 ? (int)rem : 0);
    const int left = tile_cnt - (int)L.lane_el;
    L.cnt = left >= kCodecVec ? kCodecVec : (left > 0 ? left : 0);
    return L;
}
__device__ __forceinline__ LanePos lane_pos(int64_t n) { return lane_pos_at((int64_t)blockIdx.x * kCodecTile, n); }

// Eight elements of a lane from / to an array of 4-, 2- or 1-byte elements.  Full lanes use
// vector accesses; ragged lanes go element by element and read missing elements as zero.
__device__ __forceinline__ void load_f32(float (&f)[kCodecVec], const float* p, const LanePos& L) {
    if (L.cnt == kCodecVec) {
        gld_floats(f, gbase(p, 4 * L.tile0), 4u * block_local(L.lane_el));
    } else {
        const float* q = p + L.tile0 + L.lane_el;
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) f[i] = (i < L.cnt) ? q[i] : 0.0f;
    }
}
__device__ __forceinline__ void store_f32(float* p, const LanePos& L, const float (&f)[kCodecVec]) {
    if (L.cnt == kCodecVec) {
        gst_floats(gbase(p, 4 * L.tile0), 4u * block_local(L.lane_el), f);
    } else {
        float* q = p + L.tile0 + L.lane_el;
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) if (i < L.cnt) q[i] = f[i];
    }
}
__device__ __forceinline__ void load_u16(uint32_t (&w)[kCodecVec / 2], const void* p, const LanePos& L) {
    if (L.cnt == kCodecVec) {
        gld_words(w, gbase(p, 2 * L.tile0), 2u * block_local(L.lane_el));
    } else {
        const uint16_t* q = reinterpret_cast<const uint16_t*>(p) + L.tile0 + L.lane_el;
#pragma unroll
        for (int j = 0; j < kCodecVec / 2; ++j) {
            const uint32_t lo = (2 * j < L.cnt) ? q[2 * j] : 0u, hi = (2 * j + 1 < L.cnt) ? q[2 * j + 1] : 0u;
            w[j] = lo | (hi << 16);
        }
    }
}
__device__ __forceinline__ void store_u16(void* p, const LanePos& L, const uint32_t (&w)[kCodecVec / 2]) {
    if (L.cnt == kCodecVec) {
        gst_words(gbase(p, 2 * L.tile0), 2u * block_local(L.lane_el), w);
    } else {
        uint16_t* q = reinterpret_cast<uint16_t*>(p) + L.tile0 + L.lane_el;
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) if (i < L.cnt) q[i] = (uint16_t)(w[i >> 1] >> (16 * (i & 1)));
    }
}
__device__ __forceinline__ void load_u8(uint32_t (&w)[kCodecVec / 4], const void* p, const LanePos& L) {
    if (L.cnt == kCodecVec) {
        gld_words(w, gbase(p, L.tile0), block_local(L.lane_el));
    } else {
        const uint8_t* q = reinterpret_cast<const uint8_t*>(p) + L.tile0 + L.lane_el;
#pragma unroll
        for (int j = 0; j < kCodecVec / 4; ++j) {
            uint32_t t = 0;
#pragma unroll
            for (int k = 0; k < 4; ++k) if (4 * j + k < L.cnt) t |= (uint32_t)q[4 * j + k] << (8 * k);
            w[j] = t;
        }
    }
}
__device__ __forceinline__ void store_u8(void* p, const LanePos& L, const uint32_t (&w)[kCodecVec / 4]) {
    if (L.cnt == kCodecVec) {
        gst_words(gbase(p, L.tile0), block_local(L.lane_el), w);
    } else {
        uint8_t* q = reinterpret_cast<uint8_t*>(p) + L.tile0 + L.lane_el;
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) if (i < L.cnt) q[i] = (uint8_t)(w[i >> 2] >> (8 * (i & 3)));
    }
}
__device__ __forceinline__ uint32_t byte_of(const uint32_t (&w)[kCodecVec / 4], int i) {
    return (w[i >> 2] >> (8 * (i & 3))) & 0xffu;
}
__device__ __forceinline__ uint32_t half_of(const uint32_t (&w)[kCodecVec / 2], int i) {
    return (w[i >> 1] >> (16 * (i & 1))) & 0xffffu;
}
// Eight small integers -> packed bytes / packed 16-bit fields (two's complement).
__device__ __forceinline__ void pack_u8(uint32_t (&w)[kCodecVec / 4], const uint32_t (&c)[kCodecVec]) {
#pragma unroll
    for (int j = 0; j < kCodecVec / 4; ++j) w[j] = pack_low_bytes(c[4 * j], c[4 * j + 1], c[4 * j + 2], c[4 * j + 3]);
}
__device__ __forceinline__ void pack_u16(uint32_t (&w)[kCodecVec / 2], const uint32_t (&c)[kCodecVec]) {
#pragma unroll
    for (int j = 0; j < kCodecVec / 2; ++j) w[j] = (c[2 * j] & 0xffffu) | (c[2 * j + 1] << 16);
}

// C and C^-1 for a correction of N = 127 (INT8) or N = 32767 (INT16) levels per side,
// written out plainly (Algorithm 1; the fused kernels use table-driven forms of the N = 127 case).
template <int N>
__device__ __forceinline__ int split_rho(float theta, uint32_t b) {
    const int E = (int)((b >> 7) & 0xffu);
    if (E == 255) return 0;                                   // non-finite theta': no correction
    const float e = theta - u2f(b << 16);
    const float en = ldexpf(e, 135 - (E < 1 ? 1 : E));        // e * 2^-l, exact
    const float c = __builtin_amdgcn_fmed3f(en, -1.0f, 1.0f);
    return (int)rintf(c * (float)N);
}
template <int N>
__device__ __forceinline__ float reconstruct_n(uint32_t b, int rho) {
    const float base = u2f(b << 16);
    if (((b >> 7) & 0xffu) == 255u) return base;
    const float q = (float)rho / (float)N;
    return base + ldexpf(q, half_ulp_log2(b));
}
// The 8-bit case with rho / 127 read from a staged copy of the table of these divisions.
__device__ __forceinline__ float reconstruct_tab(const float* rho_over_127, uint32_t b, uint32_t rho_byte) {
    const float base = u2f(b << 16);
    if (((b >> 7) & 0xffu) == 255u) return base;
    return base + ldexpf(rho_over_127[rho_byte], half_ulp_log2(b));
}

// The "directional" reading of ULP(theta'), for the experiment of Section 4.4 only.  The BF16 grid is twice
// as fine just below a power of two as above it, so for theta' = +-2^k (mantissa field 0, exponent field
// at least 2) with theta on the side of zero the values that round to theta' span a quarter of the upper
// spacing, not a half.  This reading takes the spacing of the side on which theta lies; the decoder knows
// the side from the signs of rho and theta'.  With a 16-bit correction it reproduces the fraction of
// bit-exact reconstructions that Section 4.4 prints.
__device__ __forceinline__ bool finer_side(uint32_t b, bool toward_negative) {
    const bool pow2 = (b & 0x7fu) == 0u && ((b >> 7) & 0xffu) >= 2u;
    return pow2 && (toward_negative != ((b & 0x8000u) != 0u));
}
template <int N>
__device__ __forceinline__ int split_rho_directional(float theta, uint32_t b) {
    const int E = (int)((b >> 7) & 0xffu);
    if (E == 255) return 0;
    const float e = theta - u2f(b << 16);
    const int shift = 135 - (E < 1 ? 1 : E) + ((e != 0.0f && finer_side(b, e < 0.0f)) ? 1 : 0);
    const float c = __builtin_amdgcn_fmed3f(ldexpf(e, shift), -1.0f, 1.0f);
    return (int)rintf(c * (float)N);
}
template <int N>
__device__ __forceinline__ float reconstruct_directional(uint32_t b, int rho) {
    const float base = u2f(b << 16);
    if (((b >> 7) & 0xffu) == 255u) return base;
    const float q = (float)rho / (float)N;
    return base + ldexpf(q, half_ulp_log2(b) - ((rho != 0 && finer_side(b, rho < 0)) ? 1 : 0));
}

// Copies one 256-entry decode table into LDS, one entry per lane of a 256-lane workgroup, and waits for
// it.  Every lane of the workgroup must call it.
__device__ __forceinline__ void stage_table(float* lds, const float* table) {
    static_assert(kThreads == 256, "one table entry per lane");
    lds[threadIdx.x] = table[threadIdx.x];
    __syncthreads();
}

template <int N, typename RHO>
__global__ __launch_bounds__(kThreads) void split_kernel(const float* theta, uint16_t* param, RHO* rho, int64_t n) {
    const LanePos L = lane_pos(n);
    if (L.cnt == 0) return;
    float th[kCodecVec];
    load_f32(th, theta, L);
    uint32_t pw[kCodecVec / 2], c[kCodecVec];
#pragma unroll
    for (int j = 0; j < kCodecVec / 2; ++j) pw[j] = bf16_pack(th[2 * j], th[2 * j + 1]);
#pragma unroll
    for (int i = 0; i < kCodecVec; ++i) c[i] = (uint32_t)split_rho<N>(th[i], half_of(pw, i));
    store_u16(param, L, pw);
    if constexpr (sizeof(RHO) == 1) {
        uint32_t rw[kCodecVec / 4];
        pack_u8(rw, c);
        store_u8(rho, L, rw);
    } else {
        uint32_t rw[kCodecVec / 2];
        pack_u16(rw, c);
        store_u16(rho, L, rw);
    }
}

template <int N, typename RHO>
__global__ __launch_bounds__(kThreads) void reconstruct_kernel(const uint16_t* param, const RHO* rho, float* theta,
                                                               int64_t n) {
    const LanePos L = lane_pos(n);
    __shared__ float rho_over_n[sizeof(RHO) == 1 ? 256 : 1];
    if constexpr (sizeof(RHO) == 1) stage_table(rho_over_n, g_decode_tables.rho);
    if (L.cnt == 0) return;
    uint32_t pw[kCodecVec / 2];
    load_u16(pw, param, L);
    float th[kCodecVec];
    if constexpr (sizeof(RHO) == 1) {
        static_assert(sizeof(RHO) != 1 || N == 127, "the table holds rho / 127");
        uint32_t rw[kCodecVec / 4];
        load_u8(rw, rho, L);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) th[i] = reconstruct_tab(rho_over_n, half_of(pw, i), byte_of(rw, i));
    } else {
        uint32_t rw[kCodecVec / 2];
        load_u16(rw, rho, L);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) th[i] = reconstruct_n<N>(half_of(pw, i), (int)(int16_t)half_of(rw, i));
    }
    store_f32(theta, L, th);
}

// The data-independent experiment of Section 4.4: FP32 bit patterns first, first + stride, ...
// (below 2^32) go through C then C^-1; errors are measured in double.  Statistics layout
// (doubles): [0] values measured, [1] skipped (non-finite theta or theta'), [2] values with
// |theta - theta'| > ULP(theta')/2, [3] max |theta_hat - theta| / (ULP(theta')/(4N)),
// [4] max relative error over normal theta, [5] bit-exact reconstructions, [6] rho outside
// [-N, N], [7] unused, [8 + E] sum of relative errors, [264 + E] count and [520 + E] bit-exact
// reconstructions of the normal values with FP32 exponent field E.  [3] and [4] are accumulated as the
// bit patterns of non-negative doubles with an integer maximum.  DIRECTIONAL selects the alternative
// reading of ULP(theta') above; [2] and [3] are measured against the printed (literal) ULP in both cases.
constexpr int kSweepPerLane = 256;

template <int N, bool DIRECTIONAL>
__global__ __launch_bounds__(kThreads) void sweep_kernel(uint64_t first, uint64_t stride, uint64_t count,
                                                         double* st) {
    __shared__ double bin_sum[256];
    __shared__ double bin_cnt[256];
    __shared__ double bin_exact[256];
    bin_sum[threadIdx.x] = 0.0;
    bin_cnt[threadIdx.x] = 0.0;
    bin_exact[threadIdx.x] = 0.0;
    __syncthreads();
    const uint64_t j0 = ((uint64_t)blockIdx.x * kThreads + threadIdx.x) * kSweepPerLane;
    double measured = 0, skipped = 0, viol = 0, exact = 0, range_bad = 0, max_ratio = 0, max_rel = 0;
    double run_sum = 0, run_cnt = 0, run_exact = 0;
    int run_exp = -1;
    for (int k = 0; k < kSweepPerLane; ++k) {
        const uint64_t j = j0 + (uint64_t)k;
        if (j >= count) break;
        const uint32_t bits = (uint32_t)(first + j * stride);
        const float theta = u2f(bits);
        const uint32_t Ef = (bits >> 23) & 0xffu;
        if (Ef == 255u) { skipped += 1; continue; }
        const uint32_t b = bf16_pack(theta, 0.0f) & 0xffffu;
        if (((b >> 7) & 0xffu) == 255u) { skipped += 1; continue; }
        const int rho = DIRECTIONAL ? split_rho_directional<N>(theta, b) : split_rho<N>(theta, b);
        const float hat = DIRECTIONAL ? reconstruct_directional<N>(b, rho) : reconstruct_n<N>(b, rho);
        measured += 1;
        const double th = (double)theta, tp = (double)u2f(b << 16);
        int E = (int)((b >> 7) & 0xffu);
        E = E < 1 ? 1 : E;
        const double u = ldexp(1.0, E - 134);
        if (fabs(th - tp) > 0.5 * u) viol += 1;
        const double err = fabs((double)hat - th);
        const double ratio = err / (u / (4.0 * N));
        max_ratio = ratio > max_ratio ? ratio : max_ratio;
        if (hat == theta) exact += 1;
        if (rho < -N || rho > N) range_bad += 1;
        if (Ef >= 1u) {
            const double rel = err / fabs(th);
            max_rel = rel > max_rel ? rel : max_rel;
            if ((int)Ef != run_exp) {
                if (run_cnt > 0) {
                    atomicAdd(&bin_sum[run_exp], run_sum); atomicAdd(&bin_cnt[run_exp], run_cnt);
                    atomicAdd(&bin_exact[run_exp], run_exact);
                }
                run_exp = (int)Ef; run_sum = 0; run_cnt = 0; run_exact = 0;
            }
            run_sum += rel; run_cnt += 1;
            if (hat == theta) run_exact += 1;
        }
    }
    if (run_cnt > 0) {
        atomicAdd(&bin_sum[run_exp], run_sum); atomicAdd(&bin_cnt[run_exp], run_cnt);
        atomicAdd(&bin_exact[run_exp], run_exact);
    }
    if (measured > 0) atomicAdd(&st[0], measured);
    if (skipped > 0) atomicAdd(&st[1], skipped);
    if (viol > 0) atomicAdd(&st[2], viol);
    if (exact > 0) atomicAdd(&st[5], exact);
    if (range_bad > 0) atomicAdd(&st[6], range_bad);
    atomicMax(reinterpret_cast<unsigned long long*>(&st[3]), (unsigned long long)__double_as_longlong(max_ratio));
    atomicMax(reinterpret_cast<unsigned long long*>(&st[4]), (unsigned long long)__double_as_longlong(max_rel));
    __syncthreads();
    if (bin_cnt[threadIdx.x] > 0) {
        atomicAdd(&st[8 + threadIdx.x], bin_sum[threadIdx.x]);
        atomicAdd(&st[264 + threadIdx.x], bin_cnt[threadIdx.x]);
        atomicAdd(&st[520 + threadIdx.x], bin_exact[threadIdx.x]);
    }
}

// Group quantizers written out plainly.  LINEAR drops the compander (the plain absmax-scaled integer
// quantisation that Section 4.5 takes as its baseline): momentum code = Round(127 m / s), variance
// code = Round(255 v / s) with s the group maximum of v itself.
// quantize_lane: the eight codes of a lane and the FP16 scale bits of its group.  All four lanes of
// a group must call it together; elements past the end are zero and do not raise the maximum.
// The group maximum of sqrt(v) is the square root of the maximum of v (the root is monotone).
template <bool VARIANCE, bool LINEAR>
__device__ __forceinline__ uint32_t quantize_lane(const float (&x)[kCodecVec], uint32_t (&codes)[kCodecVec]) {
    float a = 0.0f;
#pragma unroll
    for (int i = 0; i < kCodecVec; ++i) a = fmaxf(a, VARIANCE ? x[i] : fabsf(x[i]));
    a = group_max<kCodecVec>(a);
    if (VARIANCE && !LINEAR) a = sqrtf(a);
    float r;
    const uint32_t sbits = group_scale(a, &r);
#pragma unroll
    for (int i = 0; i < kCodecVec; ++i) {
        uint32_t c;
        if (!LINEAR) {
            c = VARIANCE ? v_code_exact(x[i], r) : m_code_exact(x[i], r);
        } else if (VARIANCE) {
            c = round_to_int_bits(__builtin_amdgcn_fmed3f((x[i] * r) * 255.0f, 0.0f, 255.0f));
        } else {
            c = round_to_int_bits(__builtin_amdgcn_fmed3f((x[i] * r) * 127.0f, -127.0f, 127.0f));
        }
        codes[i] = c & 0xffu;
    }
    return sbits;
}

// Decoders of Algorithms 2 and 3 (and of the linear baseline).  What is multiplied by the group scale
// is a function of the code byte alone - q / 255, q / 127, phi_m^-1(q / 127) - and comes from a staged
// copy of the table of those defining divisions instead of one or two IEEE divisions per element.
template <bool VARIANCE, bool LINEAR>
__device__ __forceinline__ const float* decode_table() {
    return VARIANCE ? g_decode_tables.v : (LINEAR ? g_decode_tables.rho : g_decode_tables.m);
}
template <bool VARIANCE, bool LINEAR>
__device__ __forceinline__ float dequantize_one(const float* tab, uint32_t q, float s) {
    const float f = tab[q] * s;
    return (VARIANCE && !LINEAR) ? f * f : f;
}

__device__ __forceinline__ bool group_leader(const LanePos& L) {
    return (threadIdx.x & (kGroup / kCodecVec - 1)) == 0 && L.cnt > 0;
}

template <bool VARIANCE, bool LINEAR>
__global__ __launch_bounds__(kThreads) void quantize_kernel(const float* x, uint8_t* q, uint16_t* scale,
                                                            int64_t n) {
    const LanePos L = lane_pos(n);
    float v[kCodecVec];
    load_f32(v, x, L);
    uint32_t codes[kCodecVec], w[kCodecVec / 4];
    const uint32_t sbits = quantize_lane<VARIANCE, LINEAR>(v, codes);
    pack_u8(w, codes);
    if (L.cnt > 0) store_u8(q, L, w);
    if (group_leader(L)) scale[(L.tile0 + L.lane_el) >> 5] = (uint16_t)sbits;
}

template <bool VARIANCE, bool LINEAR>
__global__ __launch_bounds__(kThreads) void dequantize_kernel(const uint8_t* q, const uint16_t* scale, float* x,
                                                              int64_t n) {
    const LanePos L = lane_pos(n);
    __shared__ float tab[256];
    stage_table(tab, decode_table<VARIANCE, LINEAR>());
    if (L.cnt == 0) return;
    uint32_t w[kCodecVec / 4];
    load_u8(w, q, L);
    const float s = (float)__builtin_bit_cast(_Float16, scale[(L.tile0 + L.lane_el) >> 5]);
    float v[kCodecVec];
#pragma unroll
    for (int i = 0; i < kCodecVec; ++i) v[i] = dequantize_one<VARIANCE, LINEAR>(tab, byte_of(w, i), s);
    store_f32(x, L, v);
}

// Quantisation error of a buffer (Section 4.5): sums[0] += sum (Q^-1(Q(x)) - x)^2 and
// sums[1] += sum x^2, in double.  A workgroup walks over tiles blockIdx.x, blockIdx.x + gridDim.x,
// ... and adds its partial sums once at the end (wavefront reduction, one atomic pair per
// wavefront), so the number of atomics on the two accumulators stays small.
template <bool VARIANCE, bool LINEAR>
__global__ __launch_bounds__(kThreads) void nmse_kernel(const float* x, int64_t n, double* sums) {
    const int64_t n_tiles = (n + kCodecTile - 1) / kCodecTile;
    __shared__ float tab[256];
    stage_table(tab, decode_table<VARIANCE, LINEAR>());
    double err = 0.0, ref = 0.0;
    for (int64_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
        const LanePos L = lane_pos_at(tile * kCodecTile, n);
        float v[kCodecVec];
        load_f32(v, x, L);
        uint32_t codes[kCodecVec];
        const uint32_t sbits = quantize_lane<VARIANCE, LINEAR>(v, codes);
        const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)sbits);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) {
            if (i < L.cnt) {
                const double xi = (double)v[i];
                const double d = (double)dequantize_one<VARIANCE, LINEAR>(tab, codes[i], s) - xi;
                err += d * d;
                ref += xi * xi;
            }
        }
    }
    for (int off = 32; off > 0; off >>= 1) {
        err += __shfl_down(err, off);
        ref += __shfl_down(ref, off);
    }
    if ((threadIdx.x & 63) == 0) {
        atomicAdd(&sums[0], err);
        atomicAdd(&sums[1], ref);
    }
}

constexpr unsigned kNmseMaxBlocks = 256 * 8;     // eight resident workgroups per compute unit

static inline unsigned tiles_for(int64_t n) { return (unsigned)((n + kCodecTile - 1) / kCodecTile); }

void launch_split(int bits, const float* theta, void* param, void* rho, int64_t n, hipStream_t s) {
    if (bits == 8) hipLaunchKernelGGL((split_kernel<127, int8_t>), dim3(tiles_for(n)), dim3(kThreads), 0, s, theta,
                                      (uint16_t*)param, (int8_t*)rho, n);
    else hipLaunchKernelGGL((split_kernel<32767, int16_t>), dim3(tiles_for(n)), dim3(kThreads), 0, s, theta,
                            (uint16_t*)param, (int16_t*)rho, n);
}
void launch_reconstruct(int bits, const void* param, const void* rho, float* theta, int64_t n, hipStream_t s) {
    if (bits == 8) hipLaunchKernelGGL((reconstruct_kernel<127, int8_t>), dim3(tiles_for(n)), dim3(kThreads), 0, s,
                                      (const uint16_t*)param, (const int8_t*)rho, theta, n);
    else hipLaunchKernelGGL((reconstruct_kernel<32767, int16_t>), dim3(tiles_for(n)), dim3(kThreads), 0, s,
                            (const uint16_t*)param, (const int16_t*)rho, theta, n);
}
hipError_t launch_sweep(int bits, bool directional, uint64_t first, uint64_t stride, uint64_t count, double* stats,
                        hipStream_t s) {
    const uint64_t lanes = (count + kSweepPerLane - 1) / kSweepPerLane;
    const dim3 grid((unsigned)((lanes + kThreads - 1) / kThreads)), block(kThreads);
#define FO_SWEEP(NN, DIR) hipLaunchKernelGGL((sweep_kernel<NN, DIR>), grid, block, 0, s, first, stride, count, stats)
    if (bits == 8) { if (directional) FO_SWEEP(127, true); else FO_SWEEP(127, false); }
    else { if (directional) FO_SWEEP(32767, true); else FO_SWEEP(32767, false); }
#undef FO_SWEEP
    return hipGetLastError();
}
template <bool VARIANCE, bool LINEAR>
static void launch_codec(int op, const void* in, const uint16_t* scale_in, void* out, uint16_t* scale_out, int64_t n,
                         double* sums, hipStream_t s) {
    if (op == 0) hipLaunchKernelGGL((quantize_kernel<VARIANCE, LINEAR>), dim3(tiles_for(n)), dim3(kThreads), 0, s,
                                    (const float*)in, (uint8_t*)out, scale_out, n);
    else if (op == 1) hipLaunchKernelGGL((dequantize_kernel<VARIANCE, LINEAR>), dim3(tiles_for(n)), dim3(kThreads), 0, s,
                                         (const uint8_t*)in, scale_in, (float*)out, n);
    else hipLaunchKernelGGL((nmse_kernel<VARIANCE, LINEAR>), dim3(tiles_for(n) < kNmseMaxBlocks ? tiles_for(n) : kNmseMaxBlocks),
                            dim3(kThreads), 0, s,
                            (const float*)in, n, sums);
}
static void dispatch_codec(bool variance, bool linear, int op, const void* in, const uint16_t* scale_in, void* out,
                           uint16_t* scale_out, int64_t n, double* sums, hipStream_t s) {
    if (variance) {
        if (linear) launch_codec<true, true>(op, in, scale_in, out, scale_out, n, sums, s);
        else launch_codec<true, false>(op, in, scale_in, out, scale_out, n, sums, s);
    } else {
        if (linear) launch_codec<false, true>(op, in, scale_in, out, scale_out, n, sums, s);
        else launch_codec<false, false>(op, in, scale_in, out, scale_out, n, sums, s);
    }
}
void launch_quantize(bool variance, bool linear, const float* x, void* q, uint16_t* scale, int64_t n, hipStream_t s) {
    dispatch_codec(variance, linear, 0, x, nullptr, q, scale, n, nullptr, s);
}
void launch_dequantize(bool variance, bool linear, const void* q, const uint16_t* scale, float* x, int64_t n,
                       hipStream_t s) {
    dispatch_codec(variance, linear, 1, q, scale, x, nullptr, n, nullptr, s);
}
void launch_nmse(bool variance, bool linear, const float* x, int64_t n, double* sums, hipStream_t s) {
    dispatch_codec(variance, linear, 2, x, nullptr, nullptr, nullptr, n, sums, s);
}

// ------------------------------------------------------ layout conversion --
//
// Migration between a standard FP32 optimizer state (theta, m, v: 12 B/param for AdamW) and
// the compressed layout: COMPRESS applies C, Q_m, Q_v (Algorithms 1-3) in one pass over a list;
// the other direction applies the inverses (its per-code factors from staged tables of the defining
// divisions).  Written with the plain exact forms; same tile
// look-up and lane layout (8 elements per lane, a lane quad per group) as the step kernels.
static_assert(kCodecTile == kConvChunkElems, "the host builds the conversion's tables for tiles of this size");

template <bool HAS_V, bool COMPRESS, bool DIRECT>
__global__ __launch_bounds__(kThreads) void convert_kernel(StepArgs a) {
    TensorDev T;
    const int64_t chunk = locate_tile<DIRECT>(a, T);
    const LanePos L = lane_pos_at(chunk * (int64_t)kCodecTile, T.numel);
    const int64_t group = (L.tile0 + L.lane_el) >> 5;
    if (COMPRESS) {
        // every lane of a group takes part in the group maxima, also those past the end
        float th[kCodecVec], m[kCodecVec], v[kCodecVec];
        load_f32(th, T.theta32, L);
        load_f32(m, T.m32, L);
        uint32_t pw[kCodecVec / 2], c[kCodecVec], w[kCodecVec / 4];
#pragma unroll
        for (int j = 0; j < kCodecVec / 2; ++j) pw[j] = bf16_pack(th[2 * j], th[2 * j + 1]);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) c[i] = (uint32_t)split_rho<127>(th[i], half_of(pw, i));
        if (L.cnt > 0) {
            store_u16(T.param, L, pw);
            pack_u8(w, c);
            store_u8(T.rho, L, w);
        }
        const uint32_t ms = quantize_lane<false, false>(m, c);
        if (L.cnt > 0) {
            pack_u8(w, c);
            store_u8(T.m_q, L, w);
        }
        if (group_leader(L)) T.m_scale[group] = (uint16_t)ms;
        if (HAS_V) {
            load_f32(v, T.v32, L);
            const uint32_t vs = quantize_lane<true, false>(v, c);
            if (L.cnt > 0) {
                pack_u8(w, c);
                store_u8(T.v_q, L, w);
            }
            if (group_leader(L)) T.v_scale[group] = (uint16_t)vs;
        }
    } else {
        __shared__ float tab[3][256];        // rho / 127, phi_m^-1(q / 127), q / 255
        tab[0][threadIdx.x] = g_decode_tables.rho[threadIdx.x];
        tab[1][threadIdx.x] = g_decode_tables.m[threadIdx.x];
        stage_table(tab[2], g_decode_tables.v);
        if (L.cnt == 0) return;
        uint32_t pw[kCodecVec / 2], w[kCodecVec / 4];
        float f[kCodecVec];
        load_u16(pw, T.param, L);
        load_u8(w, T.rho, L);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) f[i] = reconstruct_tab(tab[0], half_of(pw, i), byte_of(w, i));
        store_f32(T.theta32, L, f);
        const float s_m = (float)__builtin_bit_cast(_Float16, T.m_scale[group]);
        load_u8(w, T.m_q, L);
#pragma unroll
        for (int i = 0; i < kCodecVec; ++i) f[i] = dequantize_one<false, false>(tab[1], byte_of(w, i), s_m);
        store_f32(T.m32, L, f);
        if (HAS_V) {
            const float s_v = (float)__builtin_bit_cast(_Float16, T.v_scale[group]);
            load_u8(w, T.v_q, L);
#pragma unroll
            for (int i = 0; i < kCodecVec; ++i) f[i] = dequantize_one<true, false>(tab[2], byte_of(w, i), s_v);
            store_f32(T.v32, L, f);
        }
    }
}

hipError_t launch_convert(bool has_v, bool compress, bool direct, const StepArgs& a, int64_t n_blocks, hipStream_t s) {
    const dim3 grid((unsigned)n_blocks), block(kThreads);
#define FO_CONV(HV, CP, DR) hipLaunchKernelGGL((convert_kernel<HV, CP, DR>), grid, block, 0, s, a)
    if (has_v) {
        if (compress) { if (direct) FO_CONV(true, true, true); else FO_CONV(true, true, false); }
        else { if (direct) FO_CONV(true, false, true); else FO_CONV(true, false, false); }
    } else {
        if (compress) { if (direct) FO_CONV(false, true, true); else FO_CONV(false, true, false); }
        else { if (direct) FO_CONV(false, false, true); else FO_CONV(false, false, false); }
    }
#undef FO_CONV
    return hipGetLastError();
}

// ------------------------------------------------------------------ self-test --
//
// The step kernels replace some exactly rounded operations by shorter sequences that give
// the same bits provided the hardware estimates behave as documented (v_rcp_f32 within 1 ulp) or,
// for the square root built on v_rsq_f32, as verified here value by value.  This kernel checks
// those provisions on the device it runs on, against the plain IEEE operations:
//   section 0: recip_of_fp16(s) == 1.0f / s for every positive finite FP16 value s;
//   section 1: v_rcp_f32(d) within 1 ulp of 1.0f / d for every d in [1, 4);
//   section 2: sqrt_rn_midrange(x) == sqrtf(x) for EVERY FP32 value x of its range [2^-96, FLT_MAX];
//   section 3: momentum codes: wherever the two conversions of m_code_bracket agree, they agree with
//              m_code_exact, for every m' in [2^-13, 2) of either sign;
//   section 4: variance codes: same for v_code_bracket against v_code_exact, over every FP32 value of
//              four binades of v, for the bias-correction pair and group scale the host passes.
//   section 5: div_rn_midrange(n, d) == n / d on 2^30 pseudo-random operand pairs with magnitudes
//              in [2^-60, 2^60] (n of either sign), plus pairs that share d across all mantissas of n.
//   section 6: div_faithful(n, d) within 1 ulp of n / d on the operand pairs of section 5.  (It fails on
//              a difference of more than one ulp; how often the faithful quotient differs from the
//              exact one at all is reported by counters[14].)
// counters[2 * section] counts checks, counters[2 * section + 1] failures.

constexpr uint64_t kSelftestSqrtCount = kSelftestSqrtValues;
constexpr uint64_t kSelftestDivCount = (1ull << 30) + (1ull << 24);
constexpr uint64_t kSelftestVarCount = 4ull * (1ull << 23);
constexpr int kSelftestPerLane = 64;

__device__ __forceinline__ uint32_t selftest_hash(uint64_t x) {
    x ^= x >> 33; x *= 0xff51afd7ed558ccdull; x ^= x >> 33; x *= 0xc4ceb9fe1a85ec53ull; x ^= x >> 33;
    return (uint32_t)x;
}

// One check of `section` on value number gid of its domain.
__device__ __forceinline__ void selftest_one(int section, uint64_t gid, const StepConsts& c, float scale_r,
                                             bool& checked, bool& failed, bool& inexact) {
    checked = false; failed = false; inexact = false;
    if (section == 0) {
        if (gid >= 1 && gid <= 0x7bffu) {
            const float s = (float)__builtin_bit_cast(_Float16, (uint16_t)gid);
            checked = true;
            failed = f2u(recip_of_fp16(s)) != f2u(1.0f / s);
        }
    } else if (section == 1) {
        if (gid < (1ull << 24)) {
            const float d = u2f(0x3f800000u + (uint32_t)gid);            // [1, 4)
            const int32_t diff = (int32_t)f2u(__builtin_amdgcn_rcpf(d)) - (int32_t)f2u(1.0f / d);
            checked = true;
            failed = diff > 1 || diff < -1;
        }
    } else if (section == 2) {
        if (gid < kSelftestSqrtCount) {
            const float x = u2f(0x0f800000u + (uint32_t)gid);                     // 2^-96 ... FLT_MAX, every value
            checked = true;
            failed = f2u(sqrt_rn_midrange(x)) != f2u(sqrtf(x));
        }
    } else if (section == 3) {
        if (gid < 2ull * 14 * (1ull << 23)) {
            const uint32_t sign = (uint32_t)(gid & 1) << 31;
            const uint32_t mag = 0x39000000u + (uint32_t)(gid >> 1);     // 2^-13 ... 2
            const float m1 = u2f(sign | mag);
            float lo, hi;
            m_code_bracket(m1, 1.0f, &lo, &hi);
            const uint32_t a = put_u8(lo, 0, 0), b = put_u8(hi, 0, 0);
            const uint32_t exact = m_code_exact(m1, 1.0f) & 0xffu;
            checked = (a == b);
            failed = (a ^ 0x80u) != exact;
        }
    } else if (section == 5 || section == 6) {
        if (gid < kSelftestDivCount) {
            uint32_t nb, db;
            if (gid < (1ull << 30)) {
                const uint32_t h1 = selftest_hash(2 * gid + 1), h2 = selftest_hash(2 * gid + 2);
                // exponent fields 67..187 = 2^-60 .. 2^60
                nb = (h1 & 0x807fffffu) | ((67u + (h1 >> 23) % 121u) << 23);
                db = (h2 & 0x007fffffu) | ((67u + (h2 >> 23) % 121u) << 23);
            } else {
                const uint32_t k = (uint32_t)(gid - (1ull << 30));
                nb = 0x3a000000u + (k & 0x7fffffu) + ((k >> 23) << 31);      // all mantissas, both signs
                db = 0x38d1b717u + (k >> 23) * 0x00345678u;                   // a typical denominator ~1e-4
            }
            const float n = u2f(nb), d = u2f(db);
            checked = true;
            if (section == 5) {
                failed = f2u(div_rn_midrange(n, d)) != f2u(n / d);
            } else {
                const int32_t diff = (int32_t)f2u(div_faithful(n, d)) - (int32_t)f2u(n / d);
                failed = diff > 1 || diff < -1;
                inexact = diff != 0;
            }
        }
    } else {
        if (gid < kSelftestVarCount) {
            // binades of v starting at 2^-30, 2^-29, 2^-11, 2^-10 (odd and even exponents; with the
            // scales used by the host the codes land in 6..64 and in 180..255 and beyond)
            const uint32_t k = (uint32_t)(gid >> 23), mant = (uint32_t)gid & 0x7fffffu;
            const uint32_t ebits = (k == 0 ? 97u : k == 1 ? 98u : k == 2 ? 116u : 117u) << 23;
            const float v = u2f(ebits | mant);
            const float root_hat = sqrtf(v * c.rbc2);
            const float kr255 = fmaf(c.k255_hi, scale_r, c.k255_lo * scale_r);
            float lo, hi;
            v_code_bracket(root_hat, kr255, &lo, &hi);
            const uint32_t a = put_u8(lo, 0, 0), b = put_u8(hi, 0, 0);
            const uint32_t exact = v_code_exact(v, scale_r) & 0xffu;
            checked = (a == b);
            failed = a != exact;
        }
    }
}

// A lane checks kSelftestPerLane values (number gid = first + j * lanes in the grid) and keeps its counts in
// registers; a workgroup adds them up in LDS and issues at most three global atomics.  (One atomic per
// wavefront and value made the exhaustive square-root section take 350 ms, all of it spent on the
// 29 million updates of one counter.)
__global__ __launch_bounds__(kThreads) void selftest_kernel(unsigned long long* counters, int section,
                                                            StepConsts c, float scale_r) {
    __shared__ unsigned int tally[3];
    if (threadIdx.x < 3) tally[threadIdx.x] = 0;
    __syncthreads();
    const uint64_t lanes = (uint64_t)gridDim.x * kThreads;
    uint64_t gid = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
    unsigned int n_checked = 0, n_failed = 0, n_inexact = 0;
    for (int j = 0; j < kSelftestPerLane; ++j, gid += lanes) {
        bool checked, failed, inexact;
        selftest_one(section, gid, c, scale_r, checked, failed, inexact);
        n_checked += checked ? 1u : 0u;
        n_failed += (checked && failed) ? 1u : 0u;
        n_inexact += inexact ? 1u : 0u;
    }
    if (n_checked) atomicAdd(&tally[0], n_checked);
    if (n_failed) atomicAdd(&tally[1], n_failed);
    if (n_inexact) atomicAdd(&tally[2], n_inexact);
    __syncthreads();
    if (threadIdx.x == 0) {
        if (tally[0]) atomicAdd(&counters[2 * section], (unsigned long long)tally[0]);
        if (tally[1]) atomicAdd(&counters[2 * section + 1], (unsigned long long)tally[1]);
        if (tally[2]) atomicAdd(&counters[14], (unsigned long long)tally[2]);
    }
}

hipError_t launch_selftest(unsigned long long* counters, int section, const StepConsts& c, float scale_r,
                           hipStream_t s) {
    uint64_t n = 0;
    if (section == 0) n = 0x7c00;
    else if (section == 1) n = 1ull << 24;
    else if (section == 2) n = kSelftestSqrtCount;
    else if (section == 3) n = 2ull * 14 * (1ull << 23);
    else if (section == 5 || section == 6) n = kSelftestDivCount;
    else n = kSelftestVarCount;
    const uint64_t per_block = (uint64_t)kThreads * kSelftestPerLane;
    hipLaunchKernelGGL(selftest_kernel, dim3((unsigned)((n + per_block - 1) / per_block)), dim3(kThreads), 0, s,
                       counters, section, c, scale_r);
    return hipGetLastError();
}

// ----------------------------------------------------------- checkpoint copy --
//
// Gather / scatter of byte segments: each workgroup copies one kCopyChunkBytes piece of one
// segment with 128-bit accesses (segment starts are 16-byte aligned on both sides), the
// ragged end byte by byte, and - when packing - zero-fills the padding up to pad_bytes.

#ifndef FO_COPY_BATCH
#define FO_COPY_BATCH 16
#endif
#ifndef FO_COPY_THREADS
#define FO_COPY_THREADS 512
#endif
constexpr int kCopyThreads = FO_COPY_THREADS;
__global__ __launch_bounds__(kCopyThreads) void copy_kernel(const CopySegment* segs, const uint2* chunks) {
    const uint2 ck = chunks[blockIdx.x];
    const CopySegment sg = segs[ck.x];
    const int64_t begin = (int64_t)ck.y * kCopyChunkBytes;
    const int64_t total = sg.pad_bytes;                  // >= sg.bytes
    const int64_t end = (total - begin < kCopyChunkBytes) ? total : begin + kCopyChunkBytes;
    const uint8_t* src = sg.src;
    uint8_t* dst = sg.dst;
    constexpr int kBatch = FO_COPY_BATCH;                 // 128-bit loads in flight per lane
    constexpr int64_t kStride = (int64_t)kCopyThreads * 16;
    int64_t o = begin + (int64_t)threadIdx.x * 16;
    // whole batches inside the copied bytes: all loads of a batch are issued before its stores
    for (; o + (kBatch - 1) * kStride + 16 <= sg.bytes && o + (kBatch - 1) * kStride < end; o += kBatch * kStride) {
        uint4 v[kBatch];
#pragma unroll
        for (int k = 0; k < kBatch; ++k) v[k] = ld128(src + o + k * kStride);
#pragma unroll
        for (int k = 0; k < kBatch; ++k) st128(dst + o + k * kStride, v[k].x, v[k].y, v[k].z, v[k].w);
    }
    for (; o < end; o += kStride) {
        if (o + 16 <= sg.bytes) {
            const uint4 v = ld128(src + o);
            st128(dst + o, v.x, v.y, v.z, v.w);
        } else {
            for (int k = 0; k < 16 && o + k < end; ++k) dst[o + k] = (o + k < sg.bytes) ? src[o + k] : (uint8_t)0;
        }
    }
}

// (Issuing the copy as several shorter launches, which helps the step kernels, changed its rate by
// less than 2 %: it stays one launch.)
void launch_copy(const CopySegment* segs, const uint2* chunks, int64_t n_chunks, hipStream_t s) {
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)n_chunks), dim3(kCopyThreads), 0, s, segs, chunks);
}

}  // namespace fo
