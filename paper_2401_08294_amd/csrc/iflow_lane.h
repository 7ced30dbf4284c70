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
    const half2_t ones = {(half_t)1.0f, (half_t)1.0f};
    if (KIND == KIND_Q3H) {
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
    } else if (KIND == KIND_Q4) {
        // word g of the lane covers weights 8g..8g+7; slots 0 and 2 are biased by 1024, slots 1 and 3 by 64
        float sa = 0.f, sb = 0.f;
#pragma unroll
        for (int j = 0; j < XD; ++j) {
            xr.v[j] = as_h2(n[j]);
            if (j & 1) sb = dot2(xr.v[j], ones, sb); else sa = dot2(xr.v[j], ones, sa);
        }
        xr.bias_sum = 1024.0f * sa + 64.0f * sb;
        xr.x_sum = sa + sb;
    } else {
        float sx = 0.f;
#pragma unroll
        for (int j = 0; j < XD; ++j) { xr.v[j] = as_h2(n[j]); sx = dot2(xr.v[j], ones, sx); }
        xr.bias_sum = 1024.0f * sx;
        xr.x_sum = sx;
    }
}

// Weights of one lane for one row: WD dwords of codes and the block header (scale | offset << 16).
template <int KIND> struct WRegs { uint32_t d[Geo<KIND>::WD]; uint32_t hdr; };

// sum over the lane's weights of level * x (biased), for NB batch columns
template <int KIND, int NB>
__device__ __forceinline__ void lane_dot(const WRegs<KIND> &w, const XRegs<KIND> (&xr)[NB], float (&acc)[NB])
{
    if (KIND == KIND_Q3H) {
        float a1[NB], a2[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) { a1[b] = 0.f; a2[b] = 0.f; }
        uint32_t cmask = 0x007F007Fu, magic = 0x64006400u;
        asm volatile("" : "+v"(cmask), "+v"(magic));                              // registers, so that (d & m) | k is one v_and_or_b32
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t hc0 = (w.d[i] & cmask) | magic;                        // codes 4i, 4i+1
            const uint32_t hc1 = ((w.d[i] >> 7) & cmask) | magic;                 // codes 4i+2, 4i+3
            const half2_t h1a = q3h_high_digit(hc0), h1b = q3h_high_digit(hc1);
            const half2_t h2a = q3h_low_digit(h1a, hc0), h2b = q3h_low_digit(h1b, hc1);
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                a1[b] = dot2(h1a, xr[b].v[2 * i], a1[b]);
                a2[b] = dot2(h2a, xr[b].v[16 + 2 * i], a2[b]);
                a1[b] = dot2(h1b, xr[b].v[2 * i + 1], a1[b]);
                a2[b] = dot2(h2b, xr[b].v[16 + 2 * i + 1], a2[b]);
            }
        }
#pragma unroll
        for (int b = 0; b < NB; ++b) acc[b] = __builtin_fmaf(a2[b], IFLOW_Q3H_SCALE2, a1[b]);
    } else if (KIND == KIND_Q4) {
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

// The block header of a Q3H lane is spread over the eight words: bits 14-15 hold two scale bits, bits
// 30-31 two offset bits; shifting the running value right by two before each merge lines them up.
__device__ __forceinline__ uint32_t q3h_header(const uint32_t (&d)[8])
{
    uint32_t h = d[0] & 0xC000C000u;
#pragma unroll
    for (int i = 1; i < 8; ++i) h = (d[i] & 0xC000C000u) | (h >> 2);
    return h;
}

}  // namespace iflow
