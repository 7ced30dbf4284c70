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
// A workgroup is sixteen wavefronts = sixteen column groups = one 4096-column strip.  The grid is resident (at most one
// workgroup per compute unit) and a workgroup walks over groups of sixteen rows, strip by strip, with the strip's
// activations held in registers for all of them; the sixteen partial 16 x 16 tiles of a step are added up through LDS
// in a fixed order (so results do not vary from run to run), one workgroup barrier per step.
#include "iflow_common.h"

namespace iflow {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

// Raw bytes of a lane's 64 weights and their block header(s), per format.
template <int KIND> struct SmallRaw { uint32_t d[12]; uint32_t hdr[2]; };   // bit planes: up to 8 words of the low plane, then up to 4 of the high one
template <> struct SmallRaw<KIND_Q3H> { uint32_t d[8]; uint32_t hdr[2]; };   // (header in the spare bits of d)
template <> struct SmallRaw<KIND_Q4>  { uint32_t d[8]; uint32_t hdr[2]; };   // 32 code bytes
template <> struct SmallRaw<KIND_Q8>  { uint32_t d[16]; uint32_t hdr[2]; };  // 64 code bytes

// LDS of a workgroup: the activation staging area of each wavefront (eight batch rows of its 256 columns at a time,
// rows 528 bytes apart so that sixteen lanes reading 16 bytes each from eight different rows hit different banks), two
// buffers for the partial tiles of a round, and the running sums of the rounds when a row spans several strips.
constexpr int SMALL_XROW = 528;
constexpr int SMALL_XBYTES = 16 * 8 * SMALL_XROW;
constexpr int SMALL_RED_FLOATS = 16 * 4 * 64;
#ifndef IFLOW_SMALL_SETS
#define IFLOW_SMALL_SETS 2
#endif
constexpr int SMALL_SETS = IFLOW_SMALL_SETS;                                 // register sets of weights in flight per wavefront (even)
constexpr int SMALL_MAX_ROUNDS = 16;                          // rounds per workgroup when there is more than one strip
constexpr int SMALL_LDS_BYTES = SMALL_XBYTES + 2 * SMALL_RED_FLOATS * 4 + SMALL_MAX_ROUNDS * 256 * 4;
constexpr int SMALL_LDS_BYTES_OPS = SMALL_LDS_BYTES + 16 * 16 * 4;        // + the wavefronts' shares of sum x^2 per activation vector

// A grid of at most one workgroup per compute unit; workgroup b takes the groups of sixteen rows group0 + b,
// group0 + b + gridDim.x, ... below `ngroups` ("rounds").  Per strip the activations are loaded once, with loads
// in which neighbouring lanes read neighbouring addresses, turned through LDS into the operand layout and kept in
// registers for all rounds; the weights of the round after next are requested while a round is decoded.
// The modules of a decoder layer around the product, per activation vector (Section 2's module table: "rms" normalization,
// "silu" activation; Section 5: dynamic batching makes several vectors per step the served case): XOP = -1 none (the plain
// kernel), IFLOW_X_PLAIN (residual only), IFLOW_X_RMS_GAIN (v = fp16(x g) at the staging, sum x^2 per vector, the scalar
// 1/sqrt(mean + eps) at the store), IFLOW_X_SILU_MUL (v = fp16(silu(x) aux) at the staging, aux [batch][cols]); a residual
// [batch][rows] is added to the fp32 sum before its one rounding.
struct SmallOps {
    const uint16_t *aux;
    const uint16_t *residual;
    float eps;
};

template <int F, int S, int XOP>
__device__ __forceinline__ void gemm_small_body(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                uint16_t *__restrict__ Y, int rows, int cols, int batch, int nbk64, int nstrips,
                                                int64_t header_offset, int group0, int ngroups, const SmallOps ops)
{
    typedef Fmt<F> T;
    constexpr int KIND = T::kind;
    constexpr int HPL = 64 / T::block;                        // block headers per lane (1, or 2 for the 32-wide formats)
    constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;       // bit-plane formats: a lane's 64 weights take 2 WA + 2 WB words
    constexpr int NWORDS = kind_has_planes(KIND) ? 2 * WA + 2 * WB : KIND == KIND_Q8 ? 16 : 8;
    extern __shared__ __align__(16) uint8_t lds[];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int i = lane & 15, g = lane >> 4;
    uint8_t *xst = lds + wave * (8 * SMALL_XROW);
    float *red = reinterpret_cast<float *>(lds + SMALL_XBYTES);                       // [2][wavefront][register][lane]
    float *part = red + 2 * SMALL_RED_FLOATS;                                         // [round][256]
    const int first = group0 + (int)blockIdx.x;
    const int rounds = (ngroups - first + (int)gridDim.x - 1) / (int)gridDim.x;       // >= 1: the grid never exceeds the groups
    const int total = nstrips * rounds;                       // steps (strip, round) of this workgroup, strips outermost

    // weights of step k = (strip, round): the lane's 64 columns of row (group * 16 + i); steps past the end repeat the last one,
    // rows past the end the last row, dead column groups of a ragged strip the strip's first group: every load stays in bounds
    // The loads go out with four neighbouring lanes on one row (lane = 4 * row + column group: sixteen lanes touch four
    // 64-byte pieces instead of sixteen); round_body moves every word to the lane the MFMA layout wants it in.
    const int il = lane >> 2, gl = lane & 3;
    const int from = 4 * (4 * i + g);                         // ds_bpermute address of the lane that loaded block (i, g)
    auto load_step = [&](SmallRaw<KIND> &raw, int t, int r) {
        const bool beyond = t >= nstrips;                     // past the last step: every lane re-reads the matrix's first bytes
        if (beyond) { t = nstrips - 1; r = rounds - 1; }
        const int kb = t * 64 + wave * 4 + gl;
        const int kbc = kb < nbk64 ? kb : t * 64;
        const int n_t = min(64, nbk64 - t * 64);
        const int group = min(first + r * (int)gridDim.x, ngroups - 1);
        const int64_t row = min(group * 16 + il, rows - 1);
        if constexpr (KIND == KIND_Q3H) {                     // two planes of the strip, 16 bytes each
            const uint8_t *p0 = packed + row * ((int64_t)nbk64 * 32) + (int64_t)t * 2048 + (kbc & 63) * 16;
            const uint8_t *p1 = p0 + n_t * 16;
            if (beyond) { p0 = packed; p1 = packed; }
            const u32x4_t wa = *reinterpret_cast<const u32x4_t *>(p0);
            const u32x4_t wc = *reinterpret_cast<const u32x4_t *>(p1);
            raw.d[0] = wa.x; raw.d[1] = wa.y; raw.d[2] = wa.z; raw.d[3] = wa.w;
            raw.d[4] = wc.x; raw.d[5] = wc.y; raw.d[6] = wc.z; raw.d[7] = wc.w;
        } else if constexpr (kind_has_planes(KIND)) {         // low plane, high plane (each row-major over all rows), then the headers
            constexpr int ABYTES = 8 * WA, BBYTES = 8 * WB;   // bytes of a 64-weight block in each plane
            const uint8_t *pa = packed + row * ((int64_t)nbk64 * ABYTES) + (int64_t)kbc * ABYTES;
            const uint8_t *pb = packed + (int64_t)rows * nbk64 * ABYTES + row * ((int64_t)nbk64 * BBYTES) + (int64_t)kbc * BBYTES;
            if (beyond) { pa = packed; pb = packed; }
#pragma unroll
            for (int q = 0; q < ABYTES / 16; ++q) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t *>(pa + (beyond ? 0 : q * 16));
                raw.d[4 * q] = v.x; raw.d[4 * q + 1] = v.y; raw.d[4 * q + 2] = v.z; raw.d[4 * q + 3] = v.w;
            }
            if constexpr (BBYTES == 16) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t *>(pb);
                raw.d[2 * WA] = v.x; raw.d[2 * WA + 1] = v.y; raw.d[2 * WA + 2] = v.z; raw.d[2 * WA + 3] = v.w;
            } else if constexpr (BBYTES == 8) {
                const uint2 v = *reinterpret_cast<const uint2 *>(pb);
                raw.d[2 * WA] = v.x; raw.d[2 * WA + 1] = v.y;
            }
            const uint32_t *hp = reinterpret_cast<const uint32_t *>(packed + header_offset) + (beyond ? 0 : (row * nbk64 + kbc) * HPL);
#pragma unroll
            for (int h = 0; h < HPL; ++h) raw.hdr[h] = hp[h];
        } else {                                              // code bytes row-major, then the headers
            constexpr int BYTES = KIND == KIND_Q4 ? 32 : 64;
            const uint8_t *p0 = packed + row * ((int64_t)nbk64 * BYTES) + (int64_t)kbc * BYTES;
            if (beyond) p0 = packed;
#pragma unroll
            for (int q = 0; q < BYTES / 16; ++q) {
                const u32x4_t v = *reinterpret_cast<const u32x4_t *>(p0 + (beyond ? 0 : q * 16));
                raw.d[4 * q] = v.x; raw.d[4 * q + 1] = v.y; raw.d[4 * q + 2] = v.z; raw.d[4 * q + 3] = v.w;
            }
            const uint32_t *hp = reinterpret_cast<const uint32_t *>(packed + header_offset) + (beyond ? 0 : (row * nbk64 + kbc) * HPL);
#pragma unroll
            for (int h = 0; h < HPL; ++h) raw.hdr[h] = hp[h];
        }
    };

    const half2_t m1025 = {(half_t)-1025.0f, (half_t)-1025.0f}, m1024 = {(half_t)-1024.0f, (half_t)-1024.0f};
    const half2_t m11 = {(half_t)-11.0f, (half_t)-11.0f}, m64 = {(half_t)-64.0f, (half_t)-64.0f};
    half4_t xq[16];                                           // MFMA B operands of the current strip
    float ssq[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};  // (rms normalization) this lane's share of sum x^2 of the eight vectors it loads
    float *ssq_lds = reinterpret_cast<float *>(lds + SMALL_LDS_BYTES);                // [wavefront][vector]

    // one round: dequantize the lane's block, sixteen MFMA steps, add the sixteen wavefronts' tiles up through LDS
    auto round_body = [&](const SmallRaw<KIND> &raw, int t, int r, int which) {
        uint32_t d[NWORDS], hdr[2];
#pragma unroll
        for (int w = 0; w < NWORDS; ++w) d[w] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)raw.d[w]);
        if (KIND != KIND_Q3H) {
#pragma unroll
            for (int h = 0; h < HPL; ++h) hdr[h] = (uint32_t)__builtin_amdgcn_ds_bpermute(from, (int)raw.hdr[h]);
        }
        float4_t acc = {0.f, 0.f, 0.f, 0.f};
        if constexpr (KIND == KIND_Q3H) {
            uint32_t h = d[0] & 0xC000C000u;                  // header from the spare bits of the eight words
#pragma unroll
            for (int w = 1; w < 8; ++w) h = (d[w] & 0xC000C000u) | (h >> 2);
            const half2_t so = as_h2(h);
            const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
#pragma unroll
            for (int w = 0; w < 8; ++w) {
#pragma unroll
                for (int hs = 0; hs < 2; ++hs) {              // decode slot s = 2w + hs: weights 4s .. 4s+3
                    const uint32_t hc = ((d[w] >> (7 * hs)) & 0x007F007Fu) | 0x64006400u;
                    const half2_t q1 = q3h_high_digit(hc) + m1025;                    // floor(c/11), exact
                    const half2_t c = as_h2(hc) + m1024;                              // c, exact
                    const half2_t q2 = __builtin_elementwise_fma(q1, m11, c);         // c mod 11, exact
                    const half2_t w1 = __builtin_elementwise_fma(q1, s2, o2);         // (w[4s], w[4s+2])   Eq.2, one rounding
                    const half2_t w2 = __builtin_elementwise_fma(q2, s2, o2);         // (w[4s+1], w[4s+3])
                    const half4_t a = __builtin_shufflevector(w1, w2, 0, 1, 2, 3);
                    acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a, xq[2 * w + hs], acc, 0, 0, 0);
                }
            }
        } else if constexpr (kind_has_planes(KIND)) {
            // sixteen weights at a time: the fields of both planes as exact fp16 integers, level = high * 2^WA + low, Eq.2
            const half2_t up = {(half_t)(float)(1 << WA), (half_t)(float)(1 << WA)};
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                const half2_t so = as_h2(hdr[HPL == 2 ? gq >> 1 : 0]);
                const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
                half2_t lo[8], hi[8];
                plane_fields16<WA>(&d[WA == 4 ? 2 * gq : gq], 0, lo);
                if constexpr (WB == 2) plane_fields16<2>(&d[2 * WA + gq], 0, hi);
                if constexpr (WB == 1) plane_fields16<1>(&d[2 * WA + (gq >> 1)], gq & 1, hi);
                half2_t wv[8];
#pragma unroll
                for (int m = 0; m < 8; ++m) {
                    half2_t level = lo[m];
                    if constexpr (WB > 0) level = __builtin_elementwise_fma(hi[m], up, lo[m]);
                    wv[m] = __builtin_elementwise_fma(level, s2, o2);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const half4_t a = __builtin_shufflevector(wv[2 * j], wv[2 * j + 1], 0, 1, 2, 3);
                    acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a, xq[4 * gq + j], acc, 0, 0, 0);
                }
            }
        } else if constexpr (KIND == KIND_Q4) {
#pragma unroll
            for (int w = 0; w < 8; ++w) {                     // word w: weights 8w .. 8w+7, nibble order v0 v2 v4 v6 v1 v3 v5 v7
                const half2_t so = as_h2(hdr[HPL == 2 ? w >> 2 : 0]);
                const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
                const uint32_t dw = d[w], e = dw >> 8;
                const half2_t q0 = as_h2((dw & 0x000F000Fu) | 0x64006400u) + m1024;   // (v0, v1)
                const half2_t q1 = as_h2((dw & 0x00F000F0u) | 0x54005400u) + m64;     // (v2, v3)
                const half2_t q2 = as_h2((e & 0x000F000Fu) | 0x64006400u) + m1024;    // (v4, v5)
                const half2_t q3 = as_h2((e & 0x00F000F0u) | 0x54005400u) + m64;      // (v6, v7)
                const half4_t a0 = __builtin_shufflevector(__builtin_elementwise_fma(q0, s2, o2), __builtin_elementwise_fma(q1, s2, o2), 0, 1, 2, 3);
                const half4_t a1 = __builtin_shufflevector(__builtin_elementwise_fma(q2, s2, o2), __builtin_elementwise_fma(q3, s2, o2), 0, 1, 2, 3);
                acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a0, xq[2 * w], acc, 0, 0, 0);
                acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a1, xq[2 * w + 1], acc, 0, 0, 0);
            }
        } else {
#pragma unroll
            for (int w = 0; w < 16; ++w) {                    // word w: bytes = weights 4w .. 4w+3
                const half2_t so = as_h2(hdr[HPL == 2 ? w >> 3 : 0]);
                const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
                const half2_t q0 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[w], 0x04010400u)) + m1024;   // (b0, b1)
                const half2_t q1 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[w], 0x04030402u)) + m1024;   // (b2, b3)
                const half4_t a0 = __builtin_shufflevector(__builtin_elementwise_fma(q0, s2, o2), __builtin_elementwise_fma(q1, s2, o2), 0, 1, 2, 3);
                acc = __builtin_amdgcn_mfma_f32_16x16x16f16(a0, xq[w], acc, 0, 0, 0);
            }
        }
        // accumulator register e of lane (j, g') is D[4g' + e][j].  The buffer alternates from step to step: a wavefront that
        // is one step ahead writes the other buffer, and nobody is two steps ahead of a reader (one barrier per step).
        float *buf = red + which * SMALL_RED_FLOATS;
#pragma unroll
        for (int e = 0; e < 4; ++e) buf[(wave * 4 + e) * 64 + lane] = acc[e];
        __syncthreads();
        const int tid = threadIdx.x;
        if (tid < 256) {
            const int e = tid >> 6, l = tid & 63;
            float sum = (nstrips > 1 && t > 0) ? part[r * 256 + tid] : 0.f;
#pragma unroll
            for (int w = 0; w < 16; ++w) sum += buf[(w * 4 + e) * 64 + l];
            if (t + 1 < nstrips) {
                part[r * 256 + tid] = sum;
            } else {
                const int rr = (first + r * (int)gridDim.x) * 16 + 4 * (l >> 4) + e, b = l & 15;
                if constexpr (XOP == IFLOW_X_RMS_GAIN) {      // the vector's normalization scalar: the wavefronts' shares in a fixed order
                    float tot = 0.f;
#pragma unroll
                    for (int w = 0; w < 16; ++w) tot += ssq_lds[w * 16 + b];
                    sum *= 1.0f / __builtin_sqrtf(tot / (float)cols + ops.eps);
                }
                if constexpr (XOP >= 0) {
                    if (ops.residual != nullptr && rr < rows && b < batch) sum += (float)as_h(ops.residual[(int64_t)b * rows + rr]);
                }
                if (rr < rows && b < batch) Y[(int64_t)b * rows + rr] = as_u16((half_t)sum);
            }
        }
    };

    // activations of strip t: batch rows x the wavefront's 256 columns -> lane (j, g) holds row j, columns 64g .. 64g+63
    auto stage = [&](int t) {
        const int kb = t * 64 + wave * 4 + g;
        const bool live = kb < nbk64;                         // ragged last strip: dead lanes add nothing (their activations are zeroed)
        int c = (t * 64 + wave * 4) * 64 + (lane & 31) * 8;
        if (c >= cols) c = 0;                                 // columns past the end: any valid address, the values are masked below
        u32x4_t va[4], vb[4];                                  // load q: batch rows 2q and 2q+1 (vb: 8+2q, 9+2q), 512 bytes each, lane by lane
#pragma unroll
        for (int q = 0; q < 4; ++q)
            va[q] = *reinterpret_cast<const u32x4_t *>(X + (int64_t)min(2 * q + (lane >> 5), batch - 1) * cols + c);
#pragma unroll
        for (int q = 0; q < 4; ++q)
            vb[q] = *reinterpret_cast<const u32x4_t *>(X + (int64_t)min(8 + 2 * q + (lane >> 5), batch - 1) * cols + c);
        if constexpr (XOP == IFLOW_X_RMS_GAIN) {
            // the lane's eight columns of every vector it loaded: x^2 summed (columns past the end and dead column groups
            // were redirected to column 0: they do not count), then v = fp16(x g), an exact product rounded once
            const bool counts = (t * 64 + wave * 4) * 64 + (lane & 31) * 8 < cols;
            const u32x4_t gv = *reinterpret_cast<const u32x4_t *>(ops.aux + c);
            const uint32_t gw[4] = {gv.x, gv.y, gv.z, gv.w};
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                uint32_t xa[4] = {va[q].x, va[q].y, va[q].z, va[q].w}, xb[4] = {vb[q].x, vb[q].y, vb[q].z, vb[q].w};
                float sa = 0.f, sb = 0.f;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    sa = __builtin_amdgcn_fdot2(as_h2(xa[e]), as_h2(xa[e]), sa, false);
                    sb = __builtin_amdgcn_fdot2(as_h2(xb[e]), as_h2(xb[e]), sb, false);
                    xa[e] = as_u32(as_h2(xa[e]) * as_h2(gw[e]));
                    xb[e] = as_u32(as_h2(xb[e]) * as_h2(gw[e]));
                }
                ssq[q] += counts ? sa : 0.f;
                ssq[4 + q] += counts ? sb : 0.f;
                va[q] = (u32x4_t){xa[0], xa[1], xa[2], xa[3]};
                vb[q] = (u32x4_t){xb[0], xb[1], xb[2], xb[3]};
            }
            if (t == nstrips - 1) {
                // vector 2q + (lane >> 5) (and 8 + ...) over the wavefront's lanes: sum within each half of the wavefront
#pragma unroll
                for (int q = 0; q < 8; ++q) {
                    float v = row16_sum(ssq[q]);
                    v += __shfl_xor(v, 16);
                    if ((lane & 31) == 0) ssq_lds[wave * 16 + (q < 4 ? 2 * q : 8 + 2 * (q - 4)) + (lane >> 5)] = v;
                    ssq[q] = 0.f;
                }
            }
        } else if constexpr (XOP == IFLOW_X_SILU_MUL) {
            // v = fp16(silu(x) aux) in fp32 with the hardware exp and reciprocal, one rounding
            auto gate = [&](u32x4_t &v, int brow) {
                const u32x4_t av = *reinterpret_cast<const u32x4_t *>(ops.aux + (int64_t)min(brow, batch - 1) * cols + c);
                uint32_t xv[4] = {v.x, v.y, v.z, v.w};
                const uint32_t aw[4] = {av.x, av.y, av.z, av.w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const half2_t xa = as_h2(xv[e]), xb = as_h2(aw[e]);
                    const float g0 = (float)xa.x, g1 = (float)xa.y;
                    const float v0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * (float)xb.x;
                    const float v1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * (float)xb.y;
                    const half2_t rv = {(half_t)v0, (half_t)v1};
                    xv[e] = as_u32(rv);
                }
                v = (u32x4_t){xv[0], xv[1], xv[2], xv[3]};
            };
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                gate(va[q], 2 * q + (lane >> 5));
                gate(vb[q], 8 + 2 * q + (lane >> 5));
            }
        }
        uint32_t n[32];
#pragma unroll
        for (int q = 0; q < 32; ++q) n[q] = 0u;
        auto turn = [&](const u32x4_t (&v)[4], bool mine) {     // eight batch rows through the staging rows
#pragma unroll
            for (int q = 0; q < 4; ++q)
                *reinterpret_cast<u32x4_t *>(xst + (2 * q + (lane >> 5)) * SMALL_XROW + (lane & 31) * 16) = v[q];
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const u32x4_t u = *reinterpret_cast<const u32x4_t *>(xst + (i & 7) * SMALL_XROW + g * 128 + q * 16);
                n[4 * q] = mine ? u.x : n[4 * q]; n[4 * q + 1] = mine ? u.y : n[4 * q + 1];
                n[4 * q + 2] = mine ? u.z : n[4 * q + 2]; n[4 * q + 3] = mine ? u.w : n[4 * q + 3];
            }
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
            __builtin_amdgcn_wave_barrier();                  // the next turn overwrites the staging rows
        };
        turn(va, i < 8);
        turn(vb, i >= 8);
        // MFMA B operands: the four activations of step s.  Q3H's decoder yields weights in the order (4s, 4s+2, 4s+1, 4s+3).
        const uint32_t keep = live ? 0xFFFFFFFFu : 0u;
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
    };
    // (t, r) of the step `ahead` (<= S) steps after (t, r)
    auto step_after = [&](int t, int r, int ahead, int &t2, int &r2) {
        t2 = t; r2 = r + ahead;
#pragma unroll
        for (int q = 0; q < S; ++q)
            if (r2 >= rounds) { r2 -= rounds; ++t2; }
    };

    // Steps (strip, round) in order, S per trip through S register sets; a set is refilled for S steps ahead right
    // after its use.  The last trips, where some steps or refills no longer exist, run through a guarded copy of the
    // loop body so that the main loop has no load under a branch (the wait counters stay exact there) and nothing is
    // requested that is not used (a wavefront ends only when its last load has returned).
    SmallRaw<KIND> raw[S];
    int t = 0, r = 0, t2, r2;
#pragma unroll
    for (int j = 0; j < S; ++j) {
        step_after(0, 0, j, t2, r2);
        load_step(raw[j], t2, r2);
    }
    int k = 0;
    for (; k + 2 * S - 1 < total; k += S) {
#pragma unroll
        for (int j = 0; j < S; ++j) {
            if (r == 0) stage(t);
            round_body(raw[j], t, r, j & 1);
            step_after(t, r, S, t2, r2);
            load_step(raw[j], t2, r2);
            step_after(t, r, 1, t, r);
        }
    }
    for (; k < total; k += S) {
#pragma unroll
        for (int j = 0; j < S; ++j) {
            if (k + j < total) {                              // (uniform over the workgroup)
                if (r == 0) stage(t);
                round_body(raw[j], t, r, j & 1);
                if (k + j + S < total) {
                    step_after(t, r, S, t2, r2);
                    load_step(raw[j], t2, r2);
                }
                step_after(t, r, 1, t, r);
            }
        }
    }
}

template <int F, int S>
__global__ __launch_bounds__(1024) void gemm_small_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                          uint16_t *__restrict__ Y, int rows, int cols, int batch, int nbk64, int nstrips,
                                                          int64_t header_offset, int group0, int ngroups)
{
    gemm_small_body<F, S, -1>(packed, X, Y, rows, cols, batch, nbk64, nstrips, header_offset, group0, ngroups, SmallOps{});
}

template <int F, int S, int XOP>
__global__ __launch_bounds__(1024) void gemm_small_fused_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                                uint16_t *__restrict__ Y, int rows, int cols, int batch, int nbk64, int nstrips,
                                                                int64_t header_offset, int group0, int ngroups, const SmallOps ops)
{
    gemm_small_body<F, S, XOP>(packed, X, Y, rows, cols, batch, nbk64, nstrips, header_offset, group0, ngroups, ops);
}

template <int F, int XOP>
static hipError_t small_launch(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, uint16_t *Y, const SmallOps ops,
                               hipStream_t s)
{
    typedef Fmt<F> T;
    constexpr int S = SMALL_SETS;
    constexpr int LDS = XOP < 0 ? SMALL_LDS_BYTES : SMALL_LDS_BYTES_OPS;
    static PerDevice pd;
    int cus = 0;
    hipError_t e0 = once_per_device(pd, &cus, [] {
        if constexpr (XOP < 0)
            return hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_small_kernel<F, S>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
        else
            return hipFuncSetAttribute(reinterpret_cast<const void *>(&gemm_small_fused_kernel<F, S, XOP>), hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    });
    if (e0 != hipSuccess) return e0;
    const int nbk64 = (int)(cols / 64);
    const int nstrips = (nbk64 + 63) / 64;
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    const int64_t ngroups = (rows + 15) / 16;
    if (ngroups > 0x7FFFFFF || rows > 0x7FFFFFFF) return hipErrorInvalidValue;
    // rows spanning several strips keep a running sum per round in LDS: at most SMALL_MAX_ROUNDS rounds per launch then
    const int64_t per_launch = nstrips > 1 ? (int64_t)cus * SMALL_MAX_ROUNDS : ngroups;
    for (int64_t g0 = 0; g0 < ngroups; g0 += per_launch) {
        const int64_t g1 = g0 + per_launch < ngroups ? g0 + per_launch : ngroups;
        const int64_t grid = g1 - g0 < cus ? g1 - g0 : cus;
        if constexpr (XOP < 0)
            hipLaunchKernelGGL((gemm_small_kernel<F, S>), dim3((unsigned)grid), dim3(1024), LDS, s,
                               static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk64, nstrips, header_offset,
                               (int)g0, (int)g1);
        else
            hipLaunchKernelGGL((gemm_small_fused_kernel<F, S, XOP>), dim3((unsigned)grid), dim3(1024), LDS, s,
                               static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk64, nstrips, header_offset,
                               (int)g0, (int)g1, ops);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_qgemm_small(int format, const void *packed, int64_t rows, int64_t cols,
                              const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    if (batch < 1 || batch > 16 || cols % 64 != 0) return hipErrorInvalidValue;
    return for_format(format, [&](auto f) { return small_launch<decltype(f)::value, -1>(packed, rows, cols, X, batch, Y, SmallOps{}, s); });
}

hipError_t launch_qgemm_small_fused(int format, const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, int x_op,
                                    const uint16_t *aux, float eps, const uint16_t *residual, uint16_t *Y, hipStream_t s)
{
    if (batch < 1 || batch > 16 || cols % 64 != 0) return hipErrorInvalidValue;
    const SmallOps ops = {aux, residual, eps};
    return for_format(format, [&](auto f) {
        constexpr int F = decltype(f)::value;
        switch (x_op) {
        case IFLOW_X_PLAIN: return small_launch<F, IFLOW_X_PLAIN>(packed, rows, cols, X, batch, Y, ops, s);
        case IFLOW_X_RMS_GAIN: return small_launch<F, IFLOW_X_RMS_GAIN>(packed, rows, cols, X, batch, Y, ops, s);
        case IFLOW_X_SILU_MUL: return small_launch<F, IFLOW_X_SILU_MUL>(packed, rows, cols, X, batch, Y, ops, s);
        default: return hipErrorInvalidValue;
        }
    });
}

}  // namespace iflow
