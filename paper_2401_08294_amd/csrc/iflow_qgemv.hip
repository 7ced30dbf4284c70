// Fused dequantize-and-multiply on the vector units: y = W' x at batch 1 (the decode step's weight
// stream) and up to four activation vectors per pass.  Eq.5 and Eq.2 of the paper are applied in
// registers; the dequantized weights never exist in memory.
//
// Mapping ("activation-stationary"): a wavefront owns one strip of the reduction dimension, 64 lanes x
// WPL consecutive weights, and walks down the rows.  Each lane keeps the activations of its own
// WPL columns in registers for the whole walk, so the inner loop touches memory only for weights:
// one (Q4, Q8) or two (Q3H) 16-byte loads per lane and row, 1 KiB of consecutive bytes per wavefront
// load.  Because the levels of a lane all share one block header,
//     sum_k (q_k * s + o) x_k  =  s * sum_k q_k x_k  +  o * sum_k x_k ,
// the per-weight work is one packed conversion and one dot2 step; scale and offset are applied once per
// lane and row.  Levels are converted to fp16 by OR-ing them into the mantissa of a power of two
// (1024 + q, 64 + q), and the known bias times sum(x) is removed together with the header.
// Row sums are reduced across the wavefront with DPP, across the wavefronts of a workgroup (one per
// strip) through LDS.
#include "iflow_common.h"

namespace iflow {

template <int F> struct Lane;   // what one lane holds per row step

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

template <int KIND>
__device__ __forceinline__ void load_x(XRegs<KIND> &xr, const uint16_t *__restrict__ x, int k0, bool active)
{
    constexpr int XD = Geo<KIND>::XD;
    uint32_t n[XD];
#pragma unroll
    for (int j = 0; j < XD / 4; ++j) {
        uint4 q = active ? reinterpret_cast<const uint4 *>(x + k0)[j] : make_uint4(0u, 0u, 0u, 0u);
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
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const uint32_t hc0 = (w.d[i] & 0x007F007Fu) | 0x64006400u;            // codes 4i, 4i+1
            const uint32_t hc1 = ((w.d[i] >> 7) & 0x007F007Fu) | 0x64006400u;     // codes 4i+2, 4i+3
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
    for (int i = 1; i < 8; ++i) h = (h >> 2) | (d[i] & 0xC000C000u);
    return h;
}

template <int F, int NB, int U>
__global__ __launch_bounds__(1024) void qgemv_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                     uint16_t *__restrict__ Y, int rows, int cols, int nbk, int rows_per_wg,
                                                     int nstrips, int64_t header_offset)
{
    typedef Fmt<F> T;
    constexpr int KIND = T::kind;
    typedef Geo<KIND> G;
    __shared__ float part[16][NB][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int r0 = blockIdx.x * rows_per_wg;
    const int nr = min(rows_per_wg, rows - r0);               // 1..64 rows, row r0+i belongs to lane i
    float tot[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) tot[b] = 0.f;

    for (int t = wave; t < nstrips; t += nw) {
        const int k0 = (t * 64 + lane) * G::WPL;              // first column of this lane
        const bool active = k0 < cols;                        // the last strip may be ragged
        XRegs<KIND> xr[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) load_x<KIND>(xr[b], X + (int64_t)b * cols, k0, active);

        // where this lane's codes (and, for Q4/Q8, its header) sit inside a row
        int64_t code_off, row_stride, hdr_off = 0;
        int plane1 = 0;
        if (KIND == KIND_Q3H) {
            const int n_t = min(64, nbk - t * 64);
            row_stride = (int64_t)nbk * 32;
            code_off = (int64_t)t * 2048 + lane * 16;
            plane1 = n_t * 16;
        } else {
            row_stride = (KIND == KIND_Q4) ? cols / 2 : cols;
            code_off = (KIND == KIND_Q4) ? k0 / 2 : k0;
            hdr_off = header_offset + (int64_t)(k0 / T::block) * 4;
        }

        for (int i = 0; i < nr; i += U) {
            WRegs<KIND> w[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + min(i + u, nr - 1);        // rows past the end repeat the last one and are dropped below
                const uint8_t *p = packed + (int64_t)r * row_stride + code_off;
                uint4 a = active ? *reinterpret_cast<const uint4 *>(p) : make_uint4(0u, 0u, 0u, 0u);
                w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
                if (KIND == KIND_Q3H) {
                    uint4 c = active ? *reinterpret_cast<const uint4 *>(p + plane1) : make_uint4(0u, 0u, 0u, 0u);
                    w[u].d[4] = c.x; w[u].d[5] = c.y; w[u].d[6] = c.z; w[u].d[7] = c.w;
                } else {
                    w[u].hdr = active ? *reinterpret_cast<const uint32_t *>(packed + hdr_off + (int64_t)r * nbk * 4) : 0u;
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc[NB];
                lane_dot<KIND, NB>(w[u], xr, acc);
                uint32_t hdr;
                if (KIND == KIND_Q3H) hdr = q3h_header(reinterpret_cast<const uint32_t(&)[8]>(w[u].d)); else hdr = w[u].hdr;
                const half2_t so = as_h2(hdr);
                const float s = (float)so.x, o = (float)so.y;
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    float v = __builtin_fmaf(s, acc[b] - xr[b].bias_sum, o * xr[b].x_sum);
                    v = wave_sum(v);
                    if (lane == i + u) tot[b] += v;             // lanes >= nr are never written out
                }
            }
        }
    }

    if (nw > 1) {                                             // one wavefront per strip: add the strips up
#pragma unroll
        for (int b = 0; b < NB; ++b) part[wave][b][lane] = tot[b];
        __syncthreads();
        if (wave == 0) {
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float v = 0.f;
                for (int w2 = 0; w2 < nw; ++w2) v += part[w2][b][lane];
                tot[b] = v;
            }
        }
    }
    if (wave == 0 && lane < nr) {
#pragma unroll
        for (int b = 0; b < NB; ++b) Y[(int64_t)b * rows + r0 + lane] = as_u16((half_t)tot[b]);
    }
}

// ---- host side ------------------------------------------------------------------------------------
// Launch geometry: one wavefront per strip (at most 16 per workgroup, further strips are looped), and
// rows_per_wg chosen so that the grid has a few wavefronts per SIMD on a 256-CU part.
static int pick_rows_per_wg(int64_t rows, int waves_per_wg)
{
    const int64_t target_waves = 256 * 4 * 3;
    int64_t r = (rows * waves_per_wg + target_waves - 1) / target_waves;
    if (r < 2) r = 2;
    if (r > 64) r = 64;
    return (int)r;
}

template <int F, int NB>
static hipError_t gemv_launch(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, uint16_t *Y, hipStream_t s)
{
    typedef Fmt<F> T;
    typedef Geo<T::kind> G;
    const int nbk = (int)(cols / T::block);
    const int nstrips = (int)((cols + 64 * G::WPL - 1) / (64 * G::WPL));
    const int nw = nstrips < 16 ? nstrips : 16;
    const int rpw = pick_rows_per_wg(rows, nw);
    const int64_t grid = (rows + rpw - 1) / rpw;
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    constexpr int U = (T::kind == KIND_Q3H) ? 2 : 4;
    hipLaunchKernelGGL((qgemv_kernel<F, NB, U>), dim3((unsigned)grid), dim3(64 * nw), 0, s,
                       static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, nbk, rpw, nstrips, header_offset);
    return hipGetLastError();
}

template <int F>
static hipError_t gemv_batch(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    // up to four activation vectors share one pass over the weights; longer batches take several passes
    for (int64_t b0 = 0; b0 < batch; b0 += 4) {
        const int64_t nb = batch - b0 < 4 ? batch - b0 : 4;
        const uint16_t *Xb = X + b0 * cols;
        uint16_t *Yb = Y + b0 * rows;
        hipError_t e;
        switch (nb) {
        case 1: e = gemv_launch<F, 1>(packed, rows, cols, Xb, Yb, s); break;
        case 2: e = gemv_launch<F, 2>(packed, rows, cols, Xb, Yb, s); break;
        case 3: e = gemv_launch<F, 3>(packed, rows, cols, Xb, Yb, s); break;
        default: e = gemv_launch<F, 4>(packed, rows, cols, Xb, Yb, s); break;
        }
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

hipError_t launch_qgemv(int format, const void *packed, int64_t rows, int64_t cols,
                        const uint16_t *x, int64_t batch, uint16_t *y, hipStream_t s)
{
    switch (format) {
    case IFLOW_Q8_B32: return gemv_batch<IFLOW_Q8_B32>(packed, rows, cols, x, batch, y, s);
    case IFLOW_Q8_B64: return gemv_batch<IFLOW_Q8_B64>(packed, rows, cols, x, batch, y, s);
    case IFLOW_Q4_B32: return gemv_batch<IFLOW_Q4_B32>(packed, rows, cols, x, batch, y, s);
    case IFLOW_Q4_B64: return gemv_batch<IFLOW_Q4_B64>(packed, rows, cols, x, batch, y, s);
    case IFLOW_Q3H_B64: return gemv_batch<IFLOW_Q3H_B64>(packed, rows, cols, x, batch, y, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace iflow
