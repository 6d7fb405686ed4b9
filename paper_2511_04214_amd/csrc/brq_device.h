// Device-side building blocks shared by the gfx950 kernels of the block-rotation MXFP4
// path: bf16 widening, wavefront lane exchange, the E8M0 scale rule and the packed E2M1
// encoder.  CDNA4 only (64-wide wavefronts, DPP, the scaled fp4 convert instruction).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace brq {

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef int v8i __attribute__((ext_vector_type(8)));
typedef int v4i __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float as_f32(uint32_t u) { return __builtin_bit_cast(float, u); }
__device__ __forceinline__ uint32_t as_u32(float f) { return __builtin_bit_cast(uint32_t, f); }

// A dword holds two bf16 values; bf16 is the upper half of an fp32, so widening is a
// shift (low element) or a mask (high element), both exact.
__device__ __forceinline__ float bf16_lo(uint32_t w) { return as_f32(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return as_f32(w & 0xffff0000u); }

// fp32 -> bf16 bits, round to nearest even (finite input), integer form.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
    uint32_t u = as_u32(f);
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// Two fp32 -> one dword of two bf16 (lo in the low half), round to nearest even:
// v_cvt_pk_bf16_f32.
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}

// Value of `v` held by lane (lane ^ MASK).  MASK 1 and 2 stay inside a quad and fold
// into the consuming VALU instruction as a DPP modifier; 4, 8, 16 use the swizzle
// crossbar; 32 crosses the two halves of the wavefront.
template <int MASK>
__device__ __forceinline__ float lane_xor(float v) {
    int iv = __builtin_bit_cast(int, v);
    if constexpr (MASK == 1) {
        iv = __builtin_amdgcn_update_dpp(iv, iv, 0xB1 /* quad_perm [1,0,3,2] */, 0xF, 0xF, true);
    } else if constexpr (MASK == 2) {
        iv = __builtin_amdgcn_update_dpp(iv, iv, 0x4E /* quad_perm [2,3,0,1] */, 0xF, 0xF, true);
    } else if constexpr (MASK == 4 || MASK == 8 || MASK == 16) {
        iv = __builtin_amdgcn_ds_swizzle(iv, 0x1F | (MASK << 10)); /* and 0x1f, or 0, xor MASK */
    } else {
        static_assert(MASK == 32, "lane_xor: mask must be a power of two below 64");
        int lane = (int)__builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
        iv = __builtin_amdgcn_ds_bpermute((lane ^ 32) << 2, iv);
    }
    return __builtin_bit_cast(float, iv);
}

// Radix-8 butterfly on 8 consecutive elements held by one lane: stages h = 1, 2, 4 of
// the ascending-order Walsh-Hadamard transform, pair (i, i+h) -> (a+b, a-b).
__device__ __forceinline__ void wht8(float (&v)[8]) {
#pragma unroll
    for (int h = 1; h < 8; h *= 2) {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            if ((i & h) == 0) {
                float a = v[i], b = v[i + h];
                v[i] = a + b;
                v[i + h] = a - b;
            }
        }
    }
}

// One cross-lane stage (partner lane = lane ^ MASK).  The lane whose MASK bit is clear
// owns a and needs a+b; the other owns b and needs a-b.  Both evaluate
// fma(partner, s, own) with s = +1 / -1: the lower lane gets a+b, the upper lane gets
// b-a, i.e. the NEGATED result (one rounding, so exactly -fl(a-b)).  The caller tracks
// the sign (it flips once per stage in which the lane is the upper one) and folds it into
// the final normalisation multiply; only the sign of exact zeros can differ, and the
// encoder stores every zero magnitude as code 0.
template <int MASK>
__device__ __forceinline__ void wht_cross(float (&v)[8], float s) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = __builtin_fmaf(lane_xor<MASK>(v[i]), s, v[i]);
}

// The two stages that stay inside a quad (partner lane ^ 1, then lane ^ 2), i.e. h = 8 and
// h = 16 at 8 elements per lane.  The compiler folds a DPP lane permute into v_add/v_sub
// but not into v_fmac, so the 16 fused multiply-adds are written out: v_fmac_f32_dpp
// computes D = dpp(S0) * S1 + D.  A VGPR written by a VALU instruction may be read through
// DPP only 2 wait states later: the leading s_nop covers the compiler's code in front, and
// inside the block 7 instructions separate every write from its DPP read.
#define BRQ_FMAC_DPP(r, s, perm) \
    "v_fmac_f32_dpp " r ", " r ", " s " quad_perm:" perm " row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
__device__ __forceinline__ void wht_cross_quad(float (&v)[8], float s1, float s2) {
    asm volatile(
        "s_nop 1\n\t"
        BRQ_FMAC_DPP("%0", "%8", "[1,0,3,2]") BRQ_FMAC_DPP("%1", "%8", "[1,0,3,2]")
        BRQ_FMAC_DPP("%2", "%8", "[1,0,3,2]") BRQ_FMAC_DPP("%3", "%8", "[1,0,3,2]")
        BRQ_FMAC_DPP("%4", "%8", "[1,0,3,2]") BRQ_FMAC_DPP("%5", "%8", "[1,0,3,2]")
        BRQ_FMAC_DPP("%6", "%8", "[1,0,3,2]") BRQ_FMAC_DPP("%7", "%8", "[1,0,3,2]")
        BRQ_FMAC_DPP("%0", "%9", "[2,3,0,1]") BRQ_FMAC_DPP("%1", "%9", "[2,3,0,1]")
        BRQ_FMAC_DPP("%2", "%9", "[2,3,0,1]") BRQ_FMAC_DPP("%3", "%9", "[2,3,0,1]")
        BRQ_FMAC_DPP("%4", "%9", "[2,3,0,1]") BRQ_FMAC_DPP("%5", "%9", "[2,3,0,1]")
        BRQ_FMAC_DPP("%6", "%9", "[2,3,0,1]") BRQ_FMAC_DPP("%7", "%9", "[2,3,0,1]")
        : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])
        : "v"(s1), "v"(s2));
}
#undef BRQ_FMAC_DPP

// A lane's chunk of 8 consecutive elements, read once with the streaming hint (16 bytes of bf16, 32 of fp32).
template <bool BF16>
__device__ __forceinline__ void load_chunk(const void* p, float (&v)[8]) {
    if constexpr (BF16) {
        v4i w = __builtin_nontemporal_load(reinterpret_cast<const v4i*>(p));
        v[0] = bf16_lo((uint32_t)w.x); v[1] = bf16_hi((uint32_t)w.x); v[2] = bf16_lo((uint32_t)w.y); v[3] = bf16_hi((uint32_t)w.y);
        v[4] = bf16_lo((uint32_t)w.z); v[5] = bf16_hi((uint32_t)w.z); v[6] = bf16_lo((uint32_t)w.w); v[7] = bf16_hi((uint32_t)w.w);
    } else {
        v4f a = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p));
        v4f b = __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p) + 1);
        v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
    }
}

// The random sign diagonal of a randomized Hadamard rotation, applied on load: `signs` points at the 8 sign
// bytes of this chunk (8-byte aligned); element i is negated where its byte is negative.
__device__ __forceinline__ void apply_signs(float (&v)[8], const int8_t* signs) {
    const uint2 sg = *reinterpret_cast<const uint2*>(signs);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t word = (i < 4) ? sg.x : sg.y;
        v[i] = as_f32(as_u32(v[i]) ^ ((word << (24 - 8 * (i & 3))) & 0x80000000u));
    }
}

// Stages of the order-2^LOG2B transform for the chunk in `v`; returns the value through
// sign-tracked cross-lane stages: afterwards v holds sigma * (x H), with sigma = -1 for
// lanes with an odd number of set bits among the lane bits that took part.
template <int LOG2B>
__device__ __forceinline__ void wht_inwave(float (&v)[8], uint32_t lane) {
    static_assert(LOG2B >= 3, "a lane holds 8 elements");
    wht8(v);
    if constexpr (LOG2B == 4) wht_cross<1>(v, (lane & 1) ? -1.0f : 1.0f);
    if constexpr (LOG2B >= 5) wht_cross_quad(v, (lane & 1) ? -1.0f : 1.0f, (lane & 2) ? -1.0f : 1.0f);
    if constexpr (LOG2B >= 6) wht_cross<4>(v, (lane & 4) ? -1.0f : 1.0f);
    if constexpr (LOG2B >= 7) wht_cross<8>(v, (lane & 8) ? -1.0f : 1.0f);
    if constexpr (LOG2B >= 8) wht_cross<16>(v, (lane & 16) ? -1.0f : 1.0f);
    if constexpr (LOG2B >= 9) wht_cross<32>(v, (lane & 32) ? -1.0f : 1.0f);
}

// silu(g) * u = g / (1 + exp(-g)) * u, the gated activation that produces the input of the rotated
// layer (Sec. 4.3: the online rotation sits in front of down_proj).  The paper fixes no arithmetic
// for it, so the kernel takes the cheapest one that stays within a stated bound of the definition:
// exp(-g) = 2^(g * -log2(e)) on v_exp_f32, the reciprocal of 1 + exp(-g) on v_rcp_f32 (1 ulp each),
// three multiplies and one add, each rounded once.  Error against the exact value:
//   z = g * -log2(e) carries half an ulp of its own size plus the rounding of log2(e), which the
//   exponential turns into 1.5 |g| 2^-24 relative; exp and rcp 2^-23 each; 1 + e, g * y and s * u
//   2^-24 each: together below (8 + 2 |g|) 2^-24 relative (brq.h states that bound, the tests
//   measure it).  Far below zero (g < -87) 1 + exp(-g) leaves the range whose reciprocal is a
//   normal number and the result may be flushed to zero: an absolute error below 2^-119 |u|.
// With this the SwiGLU-fused step costs 6 instructions per element for the activation instead of
// 22 for a correctly rounded sequence, and is bound by HBM like the plain step.
__device__ __forceinline__ float swiglu_f32(float g, float u) {
    const float z = g * -as_f32(0x3FB8AA3Bu);
    const float e = __builtin_amdgcn_exp2f(z);
    const float d = 1.0f + e;
    const float y = __builtin_amdgcn_rcpf(d);
    const float s = g * y;
    return s * u;
}

// The lane's 8 gate values in v become h = swiglu(v, w); with `to_bf16` (uniform) h passes
// through bf16 (round to nearest even) as if a separate activation kernel had stored it.
__device__ __forceinline__ void swiglu8(float (&v)[8], const float (&w)[8], bool to_bf16) {
#pragma unroll
    for (int i = 0; i < 8; ++i) v[i] = swiglu_f32(v[i], w[i]);
    if (to_bf16) {
#pragma unroll
        for (int i = 0; i < 8; i += 2) {
            const uint32_t pk = pack_bf16x2(v[i], v[i + 1]);
            v[i] = bf16_lo(pk);
            v[i + 1] = bf16_hi(pk);
        }
    }
}

// Maximum magnitude of the lane's 8 values.
__device__ __forceinline__ float absmax8(const float (&y)[8]) {
    float m = fmaxf(fmaxf(fabsf(y[0]), fabsf(y[1])), fabsf(y[2]));
    m = fmaxf(fmaxf(m, fabsf(y[3])), fabsf(y[4]));
    m = fmaxf(fmaxf(m, fabsf(y[5])), fabsf(y[6]));
    return fmaxf(m, fabsf(y[7]));
}

// Maximum over the 4 lanes of a quad (= one 32-element MXFP4 group at 8 per lane).  The
// argument is non-negative, so comparing the bit patterns as unsigned integers orders
// them like the floats.  Same DPP read-after-write spacing rule as above.
__device__ __forceinline__ float quad_max(float m) {
    uint32_t u = as_u32(m);
    asm volatile(
        "s_nop 1\n\t"
        "v_max_u32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\t"
        "v_max_u32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        : "+v"(u));
    return as_f32(u);
}

// Sum over the 4 lanes of a quad, every lane receiving it: two adds with the lane permute folded in
// (((v0 + v1) + (v2 + v3)) in lanes 0, 1 and the mirror image in lanes 2, 3: the same value, since fp32
// addition is commutative).  Same DPP read-after-write spacing rule as above.
__device__ __forceinline__ float quad_sum(float v) {
    asm volatile(
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        "s_nop 1\n\t"
        "v_add_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf bound_ctrl:1\n\t"
        : "+v"(v));
    return v;
}

// E8M0 byte of a group from its maximum magnitude: max(exponent field - 2, 0).
// (2 = exponent of the largest E2M1 value, 6 = 1.5 * 2^2.)
__device__ __forceinline__ uint32_t e8m0_from_amax(float amax) {
    uint32_t e = (as_u32(amax) >> 23) & 0xffu;
    return __builtin_elementwise_sub_sat(e, 2u);
}

// 8 fp32 values -> 8 packed E2M1 codes (element i in nibble i) under E8M0 byte `sb`.
// v_cvt_scalef32_pk_fp4_f32 divides by 2^(sb-127) (it reads only the exponent field of
// its scale operand, field 0 meaning 2^-127), rounds to nearest with ties to the even
// code and saturates at 6.  It keeps the sign of results that round to zero; those
// nibbles are cleared afterwards so that a zero magnitude is always code 0.
// encode8_e2m1_signed_zero is the instruction's own result (a zero magnitude may carry a sign bit): enough
// where the codes are only decoded again.
__device__ __forceinline__ uint32_t encode8_e2m1_signed_zero(const float (&y)[8], uint32_t sb) {
    float scale = as_f32(sb << 23);
    uint32_t w = 0;
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, y[0], y[1], scale, 0);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, y[2], y[3], scale, 1);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, y[4], y[5], scale, 2);
    w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, y[6], y[7], scale, 3);
    return w;
}
__device__ __forceinline__ uint32_t encode8_e2m1(const float (&y)[8], uint32_t sb) {
    const uint32_t w = encode8_e2m1_signed_zero(y, sb);
    uint32_t mag = w & 0x77777777u;
    uint32_t nz = mag + 0x77777777u;            // bit 3 of a nibble set <=> magnitude != 0
    return w & (nz | 0x77777777u);
}

// ---- LDS-DMA loads (global memory -> LDS without passing through VGPRs)

// One LDS-DMA load: 64 lanes x 16 bytes from base + voff(lane) to LDS lds_base + LDS_OFF +
// 16 * lane (M0 carries the LDS address).  lds_base and base must be wavefront-uniform.
template <int LDS_OFF>
__device__ __forceinline__ void dma16(uint32_t lds_base, const uint8_t* base, uint32_t voff) {
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2\n\t"
                 :: "s"(lds_base), "v"(voff), "s"(base), "n"(LDS_OFF)
                 : "memory", "scc", "m0");
}

// The same with the non-temporal hint, for data that is read once.
template <int LDS_OFF>
__device__ __forceinline__ void dma16_stream(uint32_t lds_base, const uint8_t* base, uint32_t voff) {
    asm volatile("s_add_u32 m0, %0, %3\n\tglobal_load_lds_dwordx4 %1, %2 nt\n\t"
                 :: "s"(lds_base), "v"(voff), "s"(base), "n"(LDS_OFF)
                 : "memory", "scc", "m0");
}

// A pointer that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ const uint8_t* uniform_ptr(const uint8_t* p) {
    uint64_t b = (uint64_t)p;
    uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b), hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return (const uint8_t*)(((uint64_t)hi << 32) | lo);
}

}  // namespace brq
