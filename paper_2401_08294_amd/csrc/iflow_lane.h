// Per-lane building blocks of the fused dequantize-and-multiply kernels: how one lane holds its activations
// and one row's weights, and the biased dot product of Eq.5 / Eq.2 in packed fp16 arithmetic.
#pragma once

#include "iflow_common.h"

namespace iflow {

// ---- per-format lane geometry -------------------------------------------------------------------
template <int KIND> struct Geo;
template <> struct Geo<KIND_Q3H> { static constexpr int WPL = 64, XD = 32, WD = 8; };   // weights, x dwords, weight dwords per lane
template <> struct Geo<KIND_Q4>  { static constexpr int WPL = 32, XD = 16, WD = 4; };
template <> struct Geo<KIND_Q8>  { static constexpr int WPL = 16, XD = 8,  WD = 4; };
// bit-plane formats: 32 weights per lane; d[0..] holds the low plane's words, then the high plane's
template <> struct Geo<KIND_Q6>  { static constexpr int WPL = 32, XD = 16, WD = 6; };   // 4 + 2 words
template <> struct Geo<KIND_Q5>  { static constexpr int WPL = 32, XD = 16, WD = 5; };   // 4 + 1
template <> struct Geo<KIND_Q3>  { static constexpr int WPL = 32, XD = 16, WD = 3; };   // 2 + 1
template <> struct Geo<KIND_Q2>  { static constexpr int WPL = 32, XD = 16, WD = 2; };   // 2


// Activations of one lane for one batch column, arranged for the format's decode, plus the two
// constants that undo the conversion bias: bias_sum = sum_k bias_k x_k and x_sum = sum_k x_k.
template <int KIND> struct XRegs {
    half2_t v[Geo<KIND>::XD];
    float bias_sum, x_sum;
};

__device__ __forceinline__ float dot2(half2_t a, half2_t b, float c) { return __builtin_amdgcn_fdot2(a, b, c, false); }

// All ones when a < b, else zero, as a value the optimizer cannot see through: used as an AND mask where a select
// would compile to v_cndmask_b32, which is several times slower than an AND on this part.
__device__ __forceinline__ uint32_t mask_lt(int a, int b)
{
    uint32_t m = (uint32_t)((a - b) >> 31);
    asm volatile("" : "+v"(m));
    return m;
}

// ---- bit planes ------------------------------------------------------------------------------------
// A plane word holds fields of W bits, the even weights' in its low half and the odd weights' in its high half, so
// field i of a word pairs with the activation pair (x[2i], x[2i+1]) of the word's weights.  A field at bit p < 8 of both
// halves becomes the fp16 pair (B + v_even, B + v_odd), B = 2^(10-p), with one AND-OR: the field lands in the mantissa
// of an fp16 number whose exponent makes bit p count 1.  Fields at bits 8..15 are reached through one shift by 8.
// plane_bias<W>(i): the B of field i of a word, as the decode below places it.
template <int W> __device__ __forceinline__ constexpr float plane_bias(int i) { return (float)(1024 >> (W * (i & (8 / W - 1)))); }

// sum over a word's fields of (bias + value) . x-pair, for NB columns; the word's first pair is xr[b].v[J0]
template <int W, int KIND, int NB, int J0>
__device__ __forceinline__ void plane_word_dot(uint32_t d, const XRegs<KIND> (&xr)[NB], float (&acc)[NB])
{
    constexpr int PER_BYTE = 8 / W;                           // fields in the low 8 bits of a half: 2, 4 or 8
    constexpr uint32_t ONES = (1u << W) - 1u;
    const uint32_t e = d >> 8;
#pragma unroll
    for (int i = 0; i < PER_BYTE; ++i) {
        const uint32_t mask = (ONES << (W * i)) * 0x00010001u;
        const uint32_t magic = (uint32_t)((25 - W * i) << 10) * 0x00010001u;
        const half2_t lo = as_h2((d & mask) | magic), hi = as_h2((e & mask) | magic);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            acc[b] = dot2(lo, xr[b].v[J0 + i], acc[b]);
            acc[b] = dot2(hi, xr[b].v[J0 + PER_BYTE + i], acc[b]);
        }
    }
}

// A lane's activations (n: its WPL values as fp16 pairs in natural order) into the order the format's decode wants, plus the
// two sums that undo the decode's bias.
template <int KIND>
__device__ __forceinline__ void arrange_x(XRegs<KIND> &xr, const uint32_t (&n)[Geo<KIND>::XD])
{
    constexpr int XD = Geo<KIND>::XD;
    const half2_t ones = {(half_t)1.0f, (half_t)1.0f};
    if constexpr (KIND == KIND_Q3H) {
        // decode slot m works on weights 4m..4m+3 and produces (q[4m], q[4m+2]) and (q[4m+1], q[4m+3]):
        // v[m] = (x[4m], x[4m+2]), v[16+m] = (x[4m+1], x[4m+3])
        float se = 0.f, so = 0.f;
#pragma unroll
        for (int m = 0; m < 16; ++m) {
            xr.v[m] = as_h2(__builtin_amdgcn_perm(n[2 * m + 1], n[2 * m], 0x05040100u));
            xr.v[16 + m] = as_h2(__builtin_amdgcn_perm(n[2 * m + 1], n[2 * m], 0x07060302u));
            se = dot2(xr.v[m], ones, se);
            so = dot2(xr.v[16 + m], ones, so);
        }
        xr.bias_sum = IFLOW_Q3H_BIAS1 * se + IFLOW_Q3H_BIAS2 * so;
        xr.x_sum = se + so;
    } else if constexpr (KIND == KIND_Q4) {
        // word g of the lane covers weights 8g..8g+7; slots 0 and 2 are biased by 1024, slots 1 and 3 by 64
        float sa = 0.f, sb = 0.f;
#pragma unroll
        for (int j = 0; j < XD; ++j) {
            xr.v[j] = as_h2(n[j]);
            if (j & 1) sb = dot2(xr.v[j], ones, sb); else sa = dot2(xr.v[j], ones, sa);
        }
        xr.bias_sum = 1024.0f * sa + 64.0f * sb;
        xr.x_sum = sa + sb;
    } else if constexpr (kind_has_planes(KIND)) {
        // natural pairs; pair j meets field j % (16 / WA) of a low-plane word and field j % (16 / WB) of a high-plane word
        constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
        float sb = 0.f, sx = 0.f;
#pragma unroll
        for (int j = 0; j < XD; ++j) {
            xr.v[j] = as_h2(n[j]);
            const float pair = dot2(xr.v[j], ones, 0.f);
            float bias = plane_bias<WA>(j % (16 / WA));
            if constexpr (WB > 0) bias += (float)(1 << WA) * plane_bias<WB>(j % (16 / WB));
            sb = __builtin_fmaf(bias, pair, sb);
            sx += pair;
        }
        xr.bias_sum = sb;
        xr.x_sum = sx;
    } else {
        float sx = 0.f;
#pragma unroll
        for (int j = 0; j < XD; ++j) { xr.v[j] = as_h2(n[j]); sx = dot2(xr.v[j], ones, sx); }
        xr.bias_sum = 1024.0f * sx;
        xr.x_sum = sx;
    }
}

template <int KIND>
__device__ __forceinline__ void load_x(XRegs<KIND> &xr, const uint16_t *__restrict__ x, int k0)
{
    constexpr int XD = Geo<KIND>::XD;
    uint32_t n[XD];
#pragma unroll
    for (int j = 0; j < XD / 4; ++j) {
        uint4 q = reinterpret_cast<const uint4 *>(x + k0)[j];
        n[4 * j] = q.x; n[4 * j + 1] = q.y; n[4 * j + 2] = q.z; n[4 * j + 3] = q.w;
    }
    arrange_x<KIND>(xr, n);
}

// Weights of one lane for one row: WD dwords of codes and the block header (scale | offset << 16).
template <int KIND> struct WRegs { uint32_t d[Geo<KIND>::WD]; uint32_t hdr; };

// The two constants of the 3.5-bit format's code extraction, held in registers so that (d & mask) | magic is one
// v_and_or_b32 (an instruction takes one literal at most).  A kernel that decodes in a loop makes them once, in front of it.
struct Q3HConsts { uint32_t cmask, magic; };
__device__ __forceinline__ Q3HConsts q3h_consts()
{
    Q3HConsts k = {0x007F007Fu, 0x64006400u};
    asm volatile("" : "+v"(k.cmask), "+v"(k.magic));
    return k;
}
// a . b, as the first term of a sum: the three-operand form of the instruction with a zero addend (the accumulating form
// the compiler picks for dot2(a, b, 0.f) needs its accumulator register cleared by a move first)
__device__ __forceinline__ float dot2_first(half2_t a, half2_t b)
{
    float r;
    asm("v_dot2_f32_f16 %0, %1, %2, 0" : "=v"(r) : "v"(a), "v"(b));
    return r;
}

// sum over the lane's weights of level * x (biased), for NB batch columns (3.5-bit format, constants from the caller)
template <int NB>
__device__ __forceinline__ void lane_dot_q3h(const WRegs<KIND_Q3H> &w, const XRegs<KIND_Q3H> (&xr)[NB], float (&acc)[NB], const Q3HConsts &k)
{
    float a1[NB], a2[NB];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const uint32_t hc0 = (w.d[i] & k.cmask) | k.magic;                        // codes 4i, 4i+1
        const uint32_t hc1 = ((w.d[i] >> 7) & k.cmask) | k.magic;                 // codes 4i+2, 4i+3
        const half2_t h1a = q3h_high_digit(hc0), h1b = q3h_high_digit(hc1);
        const half2_t h2a = q3h_low_digit(h1a, hc0), h2b = q3h_low_digit(h1b, hc1);
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            a1[b] = i == 0 ? dot2_first(h1a, xr[b].v[2 * i]) : dot2(h1a, xr[b].v[2 * i], a1[b]);
            a2[b] = i == 0 ? dot2_first(h2a, xr[b].v[16 + 2 * i]) : dot2(h2a, xr[b].v[16 + 2 * i], a2[b]);
            a1[b] = dot2(h1b, xr[b].v[2 * i + 1], a1[b]);
            a2[b] = dot2(h2b, xr[b].v[16 + 2 * i + 1], a2[b]);
        }
    }
#pragma unroll
    for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(a2[b], IFLOW_Q3H_SCALE2, a1[b]);
}

// sum over the lane's weights of level * x (biased), for NB batch columns
template <int KIND, int NB>
__device__ __forceinline__ void lane_dot(const WRegs<KIND> &w, const XRegs<KIND> (&xr)[NB], float (&acc)[NB])
{
    if constexpr (KIND == KIND_Q3H) {
        lane_dot_q3h<NB>(w, xr, acc, q3h_consts());
    } else if constexpr (KIND == KIND_Q4) {
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const uint32_t d = w.d[g], e = d >> 8;
            const half2_t t0 = as_h2((d & 0x000F000Fu) | 0x64006400u);            // 1024 + (v0, v1)
            const half2_t t1 = as_h2((d & 0x00F000F0u) | 0x54005400u);            //   64 + (v2, v3)
            const half2_t t2 = as_h2((e & 0x000F000Fu) | 0x64006400u);            // 1024 + (v4, v5)
            const half2_t t3 = as_h2((e & 0x00F000F0u) | 0x54005400u);            //   64 + (v6, v7)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                acc[b] = dot2(t0, xr[b].v[4 * g], acc[b]);
                acc[b] = dot2(t1, xr[b].v[4 * g + 1], acc[b]);
                acc[b] = dot2(t2, xr[b].v[4 * g + 2], acc[b]);
                acc[b] = dot2(t3, xr[b].v[4 * g + 3], acc[b]);
            }
        }
    } else if constexpr (kind_has_planes(KIND)) {
        // level = low plane + 2^WA * high plane: two biased sums, combined once
        constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
        // a lane's 32 weights take WA words of the low plane (d[0..WA-1]) and WB words of the high plane (d[WA..])
        float lo[NB], hi[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) { lo[b] = 0.f; hi[b] = 0.f; }
        plane_word_dot<WA, KIND, NB, 0>(w.d[0], xr, lo);
        plane_word_dot<WA, KIND, NB, 16 / WA>(w.d[1], xr, lo);
        if constexpr (WA == 4) {
            plane_word_dot<WA, KIND, NB, 8>(w.d[2], xr, lo);
            plane_word_dot<WA, KIND, NB, 12>(w.d[3], xr, lo);
        }
        if constexpr (WB > 0) plane_word_dot<WB, KIND, NB, 0>(w.d[WA], xr, hi);
        if constexpr (WB == 2) plane_word_dot<WB, KIND, NB, 8>(w.d[WA + 1], xr, hi);
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = WB ? __builtin_fmaf(hi[b], (float)(1 << WA), lo[b]) : lo[b];
    } else {
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = 0.f;
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const half2_t t0 = as_h2(__builtin_amdgcn_perm(0x64646464u, w.d[g], 0x04010400u));   // 1024 + (b0, b1)
            const half2_t t1 = as_h2(__builtin_amdgcn_perm(0x64646464u, w.d[g], 0x04030402u));   // 1024 + (b2, b3)
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                acc[b] = dot2(t0, xr[b].v[2 * g], acc[b]);
                acc[b] = dot2(t1, xr[b].v[2 * g + 1], acc[b]);
            }
        }
    }
}

// The block header of a Q3H lane is spread over the eight words: bits 14-15 of word i hold scale bits 2i, 2i+1, bits
// 30-31 the same two offset bits.  The bytes that carry them (1 and 3 of every word) are gathered from two words at a
// time, words i and i+4, so that four registers hold them in the byte order of the result; each register then
// contributes the top two bits of all its bytes at once: 11 instructions where one mask-and-merge per word takes 15.
__device__ __forceinline__ uint32_t q3h_header(const uint32_t (&d)[8])
{
    constexpr uint32_t sel = 0x07030501u;                  // (second.b1, first.b1, second.b3, first.b3)
    uint32_t h = __builtin_amdgcn_perm(d[4], d[0], sel) >> 6 & 0x03030303u;
    h = (__builtin_amdgcn_perm(d[5], d[1], sel) >> 4 & 0x0C0C0C0Cu) | h;
    h = (__builtin_amdgcn_perm(d[6], d[2], sel) >> 2 & 0x30303030u) | h;
    h = (__builtin_amdgcn_perm(d[7], d[3], sel) & 0xC0C0C0C0u) | h;
    return h;
}

// ---- transpose-reduce: U per-lane partials (one per row) -> row sums ---------------------------------
// On return, every lane with (lane & (U-1)) == u holds the sum over all 64 lanes of v[u].
__device__ __forceinline__ float xor_lanes_16(float v) { return __shfl_xor(v, 16); }
__device__ __forceinline__ float xor_lanes_32(float v) { return __shfl_xor(v, 32); }

template <int U>
__device__ __forceinline__ float reduce_rows(float (&v)[U], int lane)
{
    static_assert(U == 1 || U == 2 || U == 4, "group size");
    float r;
    if (U == 4) {
        const bool b0 = lane & 1, b1 = lane & 2;
        // keep one of each pair, hand the other to the neighbour that keeps it
        float k0 = b0 ? v[1] : v[0], g0 = b0 ? v[0] : v[1];
        float k1 = b0 ? v[3] : v[2], g1 = b0 ? v[2] : v[3];
        float r0 = k0 + dpp_f32<0xB1, 0xF>(g0);          // lanes ^1
        float r1 = k1 + dpp_f32<0xB1, 0xF>(g1);
        float k = b1 ? r1 : r0, g = b1 ? r0 : r1;
        r = k + dpp_f32<0x4E, 0xF>(g);                   // lanes ^2: lane & 3 == u holds the quad sum of v[u]
    } else if (U == 2) {
        const bool b0 = lane & 1;
        float k = b0 ? v[1] : v[0], g = b0 ? v[0] : v[1];
        r = k + dpp_f32<0xB1, 0xF>(g);
        r += dpp_f32<0x4E, 0xF>(r);
    } else {
        r = v[0];
        r += dpp_f32<0xB1, 0xF>(r);
        r += dpp_f32<0x4E, 0xF>(r);
    }
    r += dpp_f32<0x124, 0xF>(r);                         // row_ror:4  (rotations by 4 keep lane & 3)
    r += dpp_f32<0x128, 0xF>(r);                         // row_ror:8  -> sum over the 16-lane row
    r += xor_lanes_16(r);
    r += xor_lanes_32(r);
    return r;
}

}  // namespace iflow
