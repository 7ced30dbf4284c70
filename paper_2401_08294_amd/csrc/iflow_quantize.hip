// Quantizer (Eq.1 / Eq.3 / Eq.4 of the paper, Section 3) and the two plain readers of the packed layout:
// the dequantizer (Eq.5 + Eq.2) and the logical unpacker used by tests.  None of this is on the
// decode step's hot path; the kernels are written for bit-exactness first and coalescing second.
//
// Compile without fp contraction: the encoder's (w - o) / s must stay a subtract and a divide.
#include "iflow_common.h"

namespace iflow {

__device__ __forceinline__ int dpp_i32_quad_1032(int v) { return __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true); }
__device__ __forceinline__ int dpp_i32_quad_2301(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true); }
__device__ __forceinline__ int dpp_i32_half_mirror(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true); }
__device__ __forceinline__ int dpp_i32_mirror(int v) { return __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true); }
__device__ __forceinline__ float dpp_f32_quad_1032(float v) { return dpp_f32<0xB1, 0xF>(v); }
__device__ __forceinline__ float dpp_f32_quad_2301(float v) { return dpp_f32<0x4E, 0xF>(v); }
__device__ __forceinline__ float dpp_f32_half_mirror(float v) { return dpp_f32<0x141, 0xF>(v); }
__device__ __forceinline__ float dpp_f32_mirror(float v) { return dpp_f32<0x140, 0xF>(v); }

// Byte offset, inside the packed Q3H matrix, of 32-bit word `i` (0..7) of block `kb` of row `r`:
// rows are nbk*32 bytes; strips of 64 blocks; inside a strip two planes of 16 bytes per block.
__device__ __forceinline__ int64_t q3h_word_offset(int64_t r, int nbk, int kb, int i)
{
    int t = kb >> 6, jin = kb & 63;
    int n_t = min(64, nbk - (t << 6));
    return r * (int64_t)nbk * 32 + (int64_t)t * 2048 + (int64_t)(i >> 2) * n_t * 16 + jin * 16 + (i & 3) * 4;
}

// ---- quantize: one lane per four consecutive weights, block/4 lanes per block ----------------------
template <int F>
__global__ __launch_bounds__(256) void quantize_kernel(const float4 *__restrict__ w, int64_t n_quads, int nbk,
                                                       uint8_t *__restrict__ packed, int64_t header_offset)
{
    typedef Fmt<F> T;
    constexpr int LPB = T::block / 4;                       // lanes per block: 16 or 8
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = tid < n_quads;                        // whole blocks are live or dead together
    float4 v = live ? w[tid] : make_float4(0.f, 0.f, 0.f, 0.f);

    // block minimum and maximum: every lane of the block ends with both
    float mn = fminf(fminf(v.x, v.y), fminf(v.z, v.w));
    float mx = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
    mn = fminf(mn, dpp_f32_quad_1032(mn)); mx = fmaxf(mx, dpp_f32_quad_1032(mx));
    mn = fminf(mn, dpp_f32_quad_2301(mn)); mx = fmaxf(mx, dpp_f32_quad_2301(mx));
    mn = fminf(mn, dpp_f32_half_mirror(mn)); mx = fmaxf(mx, dpp_f32_half_mirror(mx));
    if (LPB == 16) { mn = fminf(mn, dpp_f32_mirror(mn)); mx = fmaxf(mx, dpp_f32_mirror(mx)); }
    mn = mn + 0.0f; mx = mx + 0.0f;                          // a zero of either sign becomes +0

    // the two stored fp16 numbers: scale = (max - min) / L, offset = min
    const float step = (mx - mn) / (float)T::L;
    const half_t sh = (half_t)step, oh = (half_t)mn;         // round to nearest even
    const float s = (float)sh, o = (float)oh;
    const uint32_t S = as_u16(sh), O = as_u16(oh);

    // Eq.1 / Eq.3 against the stored pair; Round() = half away from zero; clamp to [0, L]
    float in[4] = {v.x, v.y, v.z, v.w};
    uint32_t q[4];
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        float t = (in[e] - o) / s;
        float r = floorf(t);
        r = (t - r >= 0.5f) ? r + 1.0f : r;
        if (!(r >= 0.0f)) r = 0.0f;
        if (r > (float)T::L) r = (float)T::L;
        q[e] = (s == 0.0f) ? 0u : (uint32_t)r;
    }

    const int64_t blk = tid / LPB;                            // global block index, row-major
    const int j = (int)(tid % LPB);                           // lane inside the block
    if constexpr (T::kind == KIND_Q3H) {
        // Eq.4: two 7-bit pair codes per lane; lanes 2i and 2i+1 build word i of the block
        const uint32_t cA = q[0] * 11u + q[1], cB = q[2] * 11u + q[3];
        const uint32_t part = (j & 1) ? (cA << 7 | cB << 23) : (cA | cB << 16);
        const uint32_t other = (uint32_t)dpp_i32_quad_1032((int)part);
        const int i = j >> 1;
        const uint32_t word = part | other | ((S >> (2 * i)) & 3u) << 14 | ((O >> (2 * i)) & 3u) << 30;
        if (live && !(j & 1)) {
            const int64_t r = blk / nbk;
            const int kb = (int)(blk % nbk);
            *reinterpret_cast<uint32_t *>(packed + q3h_word_offset(r, nbk, kb, i)) = word;
        }
    } else if (T::kind == KIND_Q4) {
        // nibble order inside a word of eight weights v0..v7: v0 v2 v4 v6 v1 v3 v5 v7
        uint32_t part = q[0] | q[2] << 4 | q[1] << 16 | q[3] << 20;
        if (j & 1) part <<= 8;
        const uint32_t other = (uint32_t)dpp_i32_quad_1032((int)part);
        if (live && !(j & 1)) reinterpret_cast<uint32_t *>(packed)[tid >> 1] = part | other;
        if (live && j == 0) reinterpret_cast<uint32_t *>(packed + header_offset)[blk] = S | O << 16;
    } else if constexpr (kind_has_planes(T::kind)) {
        // Bit planes: a word of a W-bit plane holds 32/W consecutive weights, four per lane: the weights of 2 lanes
        // (W = 4), 4 lanes (W = 2) or 8 lanes (W = 1).  Lane jj of such a group holds weights 4jj..4jj+3 of the word:
        // the even ones go to fields 2jj, 2jj+1 of the low half, the odd ones to the same fields of the high half.  The
        // group's lanes OR their parts together (quad permutes, then the mirror inside eight lanes); its first lane stores.
        constexpr int WA = Planes<T::kind>::WA, WB = Planes<T::kind>::WB;
        auto plane_word = [&](int W, int shift, uint32_t *plane) {
            const uint32_t m = (1u << W) - 1u;
            const uint32_t v0 = (q[0] >> shift) & m, v1 = (q[1] >> shift) & m, v2 = (q[2] >> shift) & m, v3 = (q[3] >> shift) & m;
            const int lanes = 8 / W;                          // lanes per word: 2, 4 or 8
            const int jj = j & (lanes - 1);
            uint32_t part = (v0 | v2 << W | v1 << 16 | v3 << (16 + W)) << (2 * W * jj);
            part |= (uint32_t)dpp_i32_quad_1032((int)part);
            if (lanes >= 4) part |= (uint32_t)dpp_i32_quad_2301((int)part);
            if (lanes >= 8) part |= (uint32_t)dpp_i32_half_mirror((int)part);
            if (live && jj == 0) plane[tid / lanes] = part;
        };
        plane_word(WA, 0, reinterpret_cast<uint32_t *>(packed));
        if constexpr (WB > 0) plane_word(WB, WA, reinterpret_cast<uint32_t *>(packed + n_quads * 4 * WA / 8));
        if (live && j == 0) reinterpret_cast<uint32_t *>(packed + header_offset)[blk] = S | O << 16;
    } else {
        if (live) reinterpret_cast<uint32_t *>(packed)[tid] = q[0] | q[1] << 8 | q[2] << 16 | q[3] << 24;
        if (live && j == 0) reinterpret_cast<uint32_t *>(packed + header_offset)[blk] = S | O << 16;
    }
}

// ---- readers: one lane per eight consecutive weights ------------------------------------------------
// LEVELS = false: fp16 dequantized weights (Eq.5 then Eq.2, one rounding through the fp16 fma).
// LEVELS = true : the levels as bytes plus the block's two fp16 numbers.
template <int F, bool LEVELS>
__global__ __launch_bounds__(256) void read_kernel(const uint8_t *__restrict__ packed, int64_t n_octs, int nbk, int64_t header_offset,
                                                   uint16_t *__restrict__ w16, uint8_t *__restrict__ levels,
                                                   uint16_t *__restrict__ scale16, uint16_t *__restrict__ offset16)
{
    typedef Fmt<F> T;
    constexpr int OPB = T::block / 8;                        // lanes per block: 8 or 4
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const bool live = tid < n_octs;
    const int64_t blk = tid / OPB;
    const int i = (int)(tid % OPB);
    uint32_t q[8];
    uint32_t S = 0, O = 0;
    if (T::kind == KIND_Q3H) {
        uint32_t word = 0;
        if (live) word = *reinterpret_cast<const uint32_t *>(packed + q3h_word_offset(blk / nbk, nbk, (int)(blk % nbk), i));
        // gather the header: word i carries bits 2i, 2i+1 of scale (at 14-15) and of offset (at 30-31)
        int hb = (int)(((word >> 14) & 3u) << (2 * i) | ((word >> 30) & 3u) << (16 + 2 * i));
        hb += dpp_i32_quad_1032(hb);                         // disjoint bits: add == or
        hb += dpp_i32_quad_2301(hb);
        hb += dpp_i32_half_mirror(hb);
        S = (uint32_t)hb & 0xFFFFu; O = (uint32_t)hb >> 16;
        const uint32_t c[4] = {word & 127u, (word >> 16) & 127u, (word >> 7) & 127u, (word >> 23) & 127u};
#pragma unroll
        for (int m = 0; m < 4; ++m) { q[2 * m] = c[m] / 11u; q[2 * m + 1] = c[m] % 11u; }   // Eq.5
    } else {
        uint32_t h = live ? reinterpret_cast<const uint32_t *>(packed + header_offset)[blk] : 0u;
        S = h & 0xFFFFu; O = h >> 16;
        if (T::kind == KIND_Q4) {
            uint32_t word = live ? reinterpret_cast<const uint32_t *>(packed)[tid] : 0u;
            const int pos[8] = {0, 4, 1, 5, 2, 6, 3, 7};      // nibble position of weight v_e
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = (word >> (4 * pos[e])) & 15u;
        } else if constexpr (kind_has_planes(T::kind)) {
            // a plane word holds 32/W weights, eight per lane: this lane's are weights 8h..8h+7 of its word, h its index
            // among the word's 4/W lanes; weight n of a word sits at bit (n/2)*W + 16*(n%2)
            constexpr int WA = Planes<T::kind>::WA, WB = Planes<T::kind>::WB;
            auto plane_bits = [&](int W, const uint32_t *plane, uint32_t (&v)[8]) {
                const int per = 4 / W;                        // lanes per word: 1 (W = 4), 2 (W = 2), 4 (W = 1)
                const uint32_t word = live ? plane[tid / per] : 0u;
                const int h = (int)(tid % per);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int n = 8 * h + e;
                    v[e] = (word >> ((n >> 1) * W + 16 * (n & 1))) & ((1u << W) - 1u);
                }
            };
            uint32_t lo[8], hi[8] = {0, 0, 0, 0, 0, 0, 0, 0};
            plane_bits(WA, reinterpret_cast<const uint32_t *>(packed), lo);
            if constexpr (WB > 0) plane_bits(WB, reinterpret_cast<const uint32_t *>(packed + n_octs * 8 * WA / 8), hi);
#pragma unroll
            for (int e = 0; e < 8; ++e) q[e] = lo[e] | hi[e] << WA;
        } else {
            uint2 two = live ? reinterpret_cast<const uint2 *>(packed)[tid] : make_uint2(0u, 0u);
#pragma unroll
            for (int e = 0; e < 4; ++e) { q[e] = (two.x >> (8 * e)) & 255u; q[4 + e] = (two.y >> (8 * e)) & 255u; }
        }
    }
    if (!live) return;
    if (LEVELS) {
        uint2 out;
        out.x = q[0] | q[1] << 8 | q[2] << 16 | q[3] << 24;
        out.y = q[4] | q[5] << 8 | q[6] << 16 | q[7] << 24;
        reinterpret_cast<uint2 *>(levels)[tid] = out;
        if (i == 0) { scale16[blk] = (uint16_t)S; offset16[blk] = (uint16_t)O; }
    } else {
        const half_t s = as_h((uint16_t)S), o = as_h((uint16_t)O);
        uint32_t out[4];
#pragma unroll
        for (int m = 0; m < 4; ++m) {
            // level <= 255 is exact in fp16; the fused multiply-add rounds level*scale + offset once
            half_t a = __builtin_fmaf16((half_t)(float)q[2 * m], s, o);
            half_t b = __builtin_fmaf16((half_t)(float)q[2 * m + 1], s, o);
            out[m] = (uint32_t)as_u16(a) | (uint32_t)as_u16(b) << 16;
        }
        reinterpret_cast<uint4 *>(w16)[tid] = make_uint4(out[0], out[1], out[2], out[3]);
    }
}

template <int F>
static hipError_t quantize_one(const float *w, int64_t rows, int64_t cols, void *packed, hipStream_t s)
{
    typedef Fmt<F> T;
    const int64_t n_quads = rows * cols / 4;
    const int nbk = (int)(cols / T::block);
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    const int64_t grid = (n_quads + 255) / 256;
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(quantize_kernel<F>, dim3((unsigned)grid), dim3(256), 0, s,
                       reinterpret_cast<const float4 *>(w), n_quads, nbk, static_cast<uint8_t *>(packed), header_offset);
    return hipGetLastError();
}

template <int F, bool LEVELS>
static hipError_t read_one(const void *packed, int64_t rows, int64_t cols, uint16_t *w16, uint8_t *levels,
                           uint16_t *scale16, uint16_t *offset16, hipStream_t s)
{
    typedef Fmt<F> T;
    const int64_t n_octs = rows * cols / 8;
    const int nbk = (int)(cols / T::block);
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    const int64_t grid = (n_octs + 255) / 256;
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((read_kernel<F, LEVELS>), dim3((unsigned)grid), dim3(256), 0, s,
                       static_cast<const uint8_t *>(packed), n_octs, nbk, header_offset, w16, levels, scale16, offset16);
    return hipGetLastError();
}

// The 3.5-bit format's stored pair codes c = 11 q[2i] + q[2i+1] (Eq.4), one byte each, in weight order: code i of a block
// covers weights 2i, 2i+1.  One thread per word of a block: its four codes 4i .. 4i+3 sit at bits 0, 16, 7 and 23.
__global__ __launch_bounds__(256) void q3h_codes_kernel(const uint8_t *__restrict__ packed, int64_t n_words, int nbk, uint8_t *__restrict__ codes)
{
    const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (tid >= n_words) return;
    const int64_t blk = tid / 8;
    const int i = (int)(tid % 8);
    const uint32_t word = *reinterpret_cast<const uint32_t *>(packed + q3h_word_offset(blk / nbk, nbk, (int)(blk % nbk), i));
    reinterpret_cast<uint32_t *>(codes)[tid] = (word & 127u) | ((word >> 16) & 127u) << 8 | ((word >> 7) & 127u) << 16 | ((word >> 23) & 127u) << 24;
}

hipError_t launch_unpack_pair_codes(const void *packed, int64_t rows, int64_t cols, uint8_t *codes, hipStream_t s)
{
    const int nbk = (int)(cols / 64);
    const int64_t n_words = rows * nbk * 8;
    const int64_t grid = (n_words + 255) / 256;
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(q3h_codes_kernel, dim3((unsigned)grid), dim3(256), 0, s, static_cast<const uint8_t *>(packed), n_words, nbk, codes);
    return hipGetLastError();
}

hipError_t launch_quantize(int format, const float *w, int64_t rows, int64_t cols, void *packed, hipStream_t s)
{
    return for_format(format, [&](auto f) { return quantize_one<decltype(f)::value>(w, rows, cols, packed, s); });
}

hipError_t launch_dequant(int format, const void *packed, int64_t rows, int64_t cols, uint16_t *w16, hipStream_t s)
{
    return for_format(format, [&](auto f) { return read_one<decltype(f)::value, false>(packed, rows, cols, w16, nullptr, nullptr, nullptr, s); });
}

hipError_t launch_unpack(int format, const void *packed, int64_t rows, int64_t cols,
                         uint8_t *levels, uint16_t *scale16, uint16_t *offset16, hipStream_t s)
{
    return for_format(format, [&](auto f) { return read_one<decltype(f)::value, true>(packed, rows, cols, nullptr, levels, scale16, offset16, s); });
}

}  // namespace iflow
