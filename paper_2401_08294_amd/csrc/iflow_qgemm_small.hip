// Small batches (up to 16 activation vectors) on the matrix cores while the weights stream by once.
//
// Decoding a weight costs the same vector work whether one or sixteen activation vectors use it, so from a
// handful of vectors on the multiply moves to v_mfma_f32_16x16x16_f16 and only the decode stays on the vector
// units.  A wavefront owns four adjacent 64-weight block columns (256 columns of K) and walks down the rows in
// groups of sixteen: lane (i, g) = (lane & 15, lane >> 4) holds block (row r0 + i, column kb0 + g).  MFMA step
// s takes weights 4s..4s+3 of each lane's block as A[i][4g..4g+3] and the matching four activations of batch
// column j from lane (j, g) as B[4g..4g+3][j]; after sixteen steps D[i][j] is the product over the wavefront's
// 256 columns.  The activations of a lane never change (its block column is fixed), so they stay in 32
// registers, permuted once into the decoder's element order.  Weights are fully dequantized before the MFMA
// (the four blocks of a step have different scales): Eq.5 and Eq.2 of the paper with the single-rounded fp16
// fused multiply-add, i.e. exactly the values iflow_dequant produces.
// A workgroup is sixteen wavefronts = sixteen column groups = one 4096-column strip; longer rows take one pass per
// strip with the accumulators kept in registers.  The sixteen partial 16 x 16 tiles are added up through LDS.
#include "iflow_common.h"

namespace iflow {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Raw bytes of a lane's 64 weights and their block header(s), per format.
template <int KIND> struct SmallRaw;
template <> struct SmallRaw<KIND_Q3H> { uint32_t d[8]; uint32_t hdr[2]; };   // (header in the spare bits of d)
template <> struct SmallRaw<KIND_Q4>  { uint32_t d[8]; uint32_t hdr[2]; };   // 32 code bytes
template <> struct SmallRaw<KIND_Q8>  { uint32_t d[16]; uint32_t hdr[2]; };  // 64 code bytes

template <int F, int G>
__global__ __launch_bounds__(1024) void gemm_small_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                          uint16_t *__restrict__ Y, int rows, int cols, int batch, int nbk64, int nstrips,
                                                          int64_t header_offset)
{
    typedef Fmt<F> T;
    constexpr int KIND = T::kind;
    constexpr int HPL = 64 / T::block;                        // block headers per lane (1, or 2 for the 32-wide formats)
    __shared__ float red[16][4][64];                          // partial tiles: [wavefront][accumulator register][lane]
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, g = lane >> 4;
    const int r0 = blockIdx.x * (16 * G);                     // G groups of sixteen rows per workgroup: activations loaded once for all
    const int bj = min(i, batch - 1);                         // batch columns past the end repeat the last one and are not stored

    float4_t acc[G];
#pragma unroll
    for (int rg = 0; rg < G; ++rg) acc[rg] = (float4_t){0.f, 0.f, 0.f, 0.f};

    for (int t = 0; t < nstrips; ++t) {                       // one pass per 4096-column strip
        const int kb = t * 64 + wave * 4 + g;                 // this lane's 64-column group
        const bool live = kb < nbk64;                         // ragged last strip: dead lanes add nothing (their activations are zeroed)
        const int kbc = live ? kb : t * 64;                   // ... and redo the strip's first group so that loads stay in bounds
        const int n_t = min(64, nbk64 - t * 64);

        // activations of batch column bj for this column group
        const uint4 *xsrc = reinterpret_cast<const uint4 *>(X + (int64_t)bj * cols + (int64_t)kbc * 64);
        uint32_t n[32];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const uint4 v = xsrc[q];
            n[4 * q] = v.x; n[4 * q + 1] = v.y; n[4 * q + 2] = v.z; n[4 * q + 3] = v.w;
        }
        // weights of the lane's 64 columns for each row group; rows past the end repeat the last row
        SmallRaw<KIND> raw[G];
#pragma unroll
        for (int rg = 0; rg < G; ++rg) {
            const int64_t row = min(r0 + 16 * rg + i, rows - 1);
            if (KIND == KIND_Q3H) {                           // two planes of the strip, 16 bytes each
                const uint8_t *p0 = packed + row * ((int64_t)nbk64 * 32) + (int64_t)t * 2048 + (kbc & 63) * 16;
                const u32x4_t wa = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p0));
                const u32x4_t wc = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p0 + n_t * 16));
                raw[rg].d[0] = wa.x; raw[rg].d[1] = wa.y; raw[rg].d[2] = wa.z; raw[rg].d[3] = wa.w;
                raw[rg].d[4] = wc.x; raw[rg].d[5] = wc.y; raw[rg].d[6] = wc.z; raw[rg].d[7] = wc.w;
            } else {                                          // code bytes row-major, then the headers
                constexpr int BYTES = KIND == KIND_Q4 ? 32 : 64;
                const uint8_t *p0 = packed + row * ((int64_t)nbk64 * BYTES) + (int64_t)kbc * BYTES;
#pragma unroll
                for (int q = 0; q < BYTES / 16; ++q) {
                    const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p0 + q * 16));
                    raw[rg].d[4 * q] = v.x; raw[rg].d[4 * q + 1] = v.y; raw[rg].d[4 * q + 2] = v.z; raw[rg].d[4 * q + 3] = v.w;
                }
                const uint32_t *hp = reinterpret_cast<const uint32_t *>(packed + header_offset) + (row * nbk64 + kbc) * HPL;
#pragma unroll
                for (int h = 0; h < HPL; ++h) raw[rg].hdr[h] = hp[h];
            }
        }

        // MFMA B operands: the four activations of step s.  Q3H's decoder yields weights in the order (4s, 4s+2, 4s+1, 4s+3).
        const uint32_t keep = live ? 0xFFFFFFFFu : 0u;
        half4_t xq[16];
#pragma unroll
        for (int s = 0; s < 16; ++s) {
            uint32_t e, o;
            if (KIND == KIND_Q3H) {
                e = __builtin_amdgcn_perm(n[2 * s + 1], n[2 * s], 0x05040100u);   // (x[4s], x[4s+2])
                o = __builtin_amdgcn_perm(n[2 * s + 1], n[2 * s], 0x07060302u);   // (x[4s+1], x[4s+3])
            } else {
                e = n[2 * s]; o = n[2 * s + 1];                                   // natural order
            }
            xq[s] = __builtin_bit_cast(half4_t, make_uint2(e & keep, o & keep));
        }

        const half2_t m1025 = {(half_t)-1025.0f, (half_t)-1025.0f}, m1024 = {(half_t)-1024.0f, (half_t)-1024.0f};
        const half2_t m11 = {(half_t)-11.0f, (half_t)-11.0f}, m64 = {(half_t)-64.0f, (half_t)-64.0f};
#pragma unroll
        for (int rg = 0; rg < G; ++rg) {
            const uint32_t *d = raw[rg].d;
            if (KIND == KIND_Q3H) {
                // header from the spare bits of the eight words
                uint32_t h = d[0] & 0xC000C000u;
#pragma unroll
                for (int w = 1; w < 8; ++w) h = (d[w] & 0xC000C000u) | (h >> 2);
                const half2_t so = as_h2(h);
                const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
#pragma unroll
                for (int w = 0; w < 8; ++w) {
#pragma unroll
                    for (int hs = 0; hs < 2; ++hs) {          // decode slot s = 2w + hs: weights 4s .. 4s+3
                        const uint32_t hc = ((d[w] >> (7 * hs)) & 0x007F007Fu) | 0x64006400u;
                        const half2_t q1 = q3h_high_digit(hc) + m1025;                    // floor(c/11), exact
                        const half2_t c = as_h2(hc) + m1024;                              // c, exact
                        const half2_t q2 = __builtin_elementwise_fma(q1, m11, c);         // c mod 11, exact
                        const half2_t w1 = __builtin_elementwise_fma(q1, s2, o2);         // (w[4s], w[4s+2])   Eq.2, one rounding
                        const half2_t w2 = __builtin_elementwise_fma(q2, s2, o2);         // (w[4s+1], w[4s+3])
                        const half4_t a = __builtin_shufflevector(w1, w2, 0, 1, 2, 3);
                        acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a, xq[2 * w + hs], acc[rg], 0, 0, 0);
                    }
                }
            } else if (KIND == KIND_Q4) {
#pragma unroll
                for (int w = 0; w < 8; ++w) {                 // word w: weights 8w .. 8w+7, nibble order v0 v2 v4 v6 v1 v3 v5 v7
                    const half2_t so = as_h2(raw[rg].hdr[HPL == 2 ? w >> 2 : 0]);
                    const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
                    const uint32_t dw = d[w], e = dw >> 8;
                    const half2_t q0 = as_h2((dw & 0x000F000Fu) | 0x64006400u) + m1024;   // (v0, v1)
                    const half2_t q1 = as_h2((dw & 0x00F000F0u) | 0x54005400u) + m64;     // (v2, v3)
                    const half2_t q2 = as_h2((e & 0x000F000Fu) | 0x64006400u) + m1024;    // (v4, v5)
                    const half2_t q3 = as_h2((e & 0x00F000F0u) | 0x54005400u) + m64;      // (v6, v7)
                    const half4_t a0 = __builtin_shufflevector(__builtin_elementwise_fma(q0, s2, o2), __builtin_elementwise_fma(q1, s2, o2), 0, 1, 2, 3);
                    const half4_t a1 = __builtin_shufflevector(__builtin_elementwise_fma(q2, s2, o2), __builtin_elementwise_fma(q3, s2, o2), 0, 1, 2, 3);
                    acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a0, xq[2 * w], acc[rg], 0, 0, 0);
                    acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a1, xq[2 * w + 1], acc[rg], 0, 0, 0);
                }
            } else {
#pragma unroll
                for (int w = 0; w < 16; ++w) {                // word w: bytes = weights 4w .. 4w+3
                    const half2_t so = as_h2(raw[rg].hdr[HPL == 2 ? w >> 3 : 0]);
                    const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
                    const half2_t q0 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[w], 0x04010400u)) + m1024;   // (b0, b1)
                    const half2_t q1 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[w], 0x04030402u)) + m1024;   // (b2, b3)
                    const half4_t a0 = __builtin_shufflevector(__builtin_elementwise_fma(q0, s2, o2), __builtin_elementwise_fma(q1, s2, o2), 0, 1, 2, 3);
                    acc[rg] = __builtin_amdgcn_mfma_f32_16x16x16f16(a0, xq[w], acc[rg], 0, 0, 0);
                }
            }
        }
    }

    // add the sixteen column groups up: accumulator register e of lane (j, g') is D[4g' + e][j]
    const int tid = threadIdx.x;
#pragma unroll
    for (int rg = 0; rg < G; ++rg) {
        if (rg > 0) __syncthreads();                          // the previous group's sums have been read
#pragma unroll
        for (int e = 0; e < 4; ++e) red[wave][e][lane] = acc[rg][e];
        __syncthreads();
        if (tid < 256) {
            const int e = tid >> 6, l = tid & 63;
            float sum = 0.f;
#pragma unroll
            for (int w = 0; w < 16; ++w) sum += red[w][e][l];
            const int r = r0 + 16 * rg + 4 * (l >> 4) + e, b = l & 15;
            if (r < rows && b < batch) Y[(int64_t)b * rows + r] = as_u16((half_t)sum);
        }
    }
}

template <int F>
static hipError_t small_launch(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    typedef Fmt<F> T;
    const int nbk64 = (int)(cols / 64);
    const int nstrips = (nbk64 + 63) / 64;
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    // row groups per workgroup: measured on 7B/70B shapes, more than one group per workgroup is slower (11008 x 4096,
    // batch 16: 18.7 us with one group, 22.1 us with two), so only very tall matrices share the activation loads
    const int64_t G = rows / 16 / 8192;
#define IFLOW_SMALL_GO(GG) hipLaunchKernelGGL((gemm_small_kernel<F, GG>), dim3((unsigned)((rows + 16 * GG - 1) / (16 * GG))), dim3(1024), 0, s, \
        static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk64, nstrips, header_offset)
    if (T::kind == KIND_Q3H && G >= 4) IFLOW_SMALL_GO(4); else if (T::kind != KIND_Q8 && G >= 2) IFLOW_SMALL_GO(2); else IFLOW_SMALL_GO(1);
#undef IFLOW_SMALL_GO
    return hipGetLastError();
}

hipError_t launch_qgemm_small(int format, const void *packed, int64_t rows, int64_t cols,
                              const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    if (batch < 1 || batch > 16 || cols % 64 != 0) return hipErrorInvalidValue;
    switch (format) {
    case IFLOW_Q8_B32: return small_launch<IFLOW_Q8_B32>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q8_B64: return small_launch<IFLOW_Q8_B64>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q4_B32: return small_launch<IFLOW_Q4_B32>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q4_B64: return small_launch<IFLOW_Q4_B64>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q3H_B64: return small_launch<IFLOW_Q3H_B64>(packed, rows, cols, X, batch, Y, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace iflow
