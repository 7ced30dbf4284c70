// Dequantize-and-multiply on the matrix cores for batches large enough to make the product a dense
// contraction: Y[b][n] = sum_k w'[n][k] X[b][k].
//
// A workgroup of four wavefronts owns a 128 (batch) x 64 (weight rows) tile of Y and walks along K in
// chunks of 64 columns, i.e. one quantization block per weight row (two for the 32-wide formats).  Per chunk
// it (1) copies the 128 x 64 fp16 activation tile into LDS, (2) decodes its 64 packed blocks into fp16
// weights in LDS - Eq.5 and Eq.2 of the paper, with the same single-rounded fp16 fused multiply-add as the
// stand-alone dequantizer, so the tile holds exactly the values iflow_dequant would produce - and (3) runs
// v_mfma_f32_32x32x8_f16 from LDS, fp32 accumulation.  Each wavefront owns a 64 x 32 part of the tile (two
// 32 x 32 accumulators).  Rows of the LDS tiles are padded to 68 halves so that the 32 lanes that read one
// operand column hit 32 different banks.
#include "iflow_common.h"

namespace iflow {

typedef _Float16 half4_t __attribute__((ext_vector_type(4)));
typedef float float16_t __attribute__((ext_vector_type(16)));

constexpr int GM_BM = 128, GM_BN = 64, GM_BK = 64, GM_LD = 68;   // tile sizes; LDS row pitch in halves

__device__ __forceinline__ uint32_t pack_h2(half2_t v) { return as_u32(v); }

// Sixteen consecutive dequantized weights (k = 16*qd .. 16*qd+15 of the chunk) of one row, as eight fp16 pairs
// in natural order.  `blk` is the row's first block of this chunk (global block index), `row`/`nbk` locate it.
template <int F>
__device__ __forceinline__ void dequant16(const uint8_t *__restrict__ packed, int64_t header_offset, int64_t row, int nbk,
                                          int kb /* 64-column chunk */, int qd, uint32_t (&out)[8])
{
    typedef Fmt<F> T;
    if (T::kind == KIND_Q3H) {
        // words 2qd, 2qd+1 of the block: plane qd/2, 8 bytes at offset (qd%2)*8 inside the block's 16 bytes
        const int t = kb >> 6, jin = kb & 63;
        const int n_t = min(64, nbk - (t << 6));
        const uint8_t *p = packed + row * (int64_t)nbk * 32 + (int64_t)t * 2048 + (qd >> 1) * n_t * 16 + jin * 16 + (qd & 1) * 8;
        const uint2 two = *reinterpret_cast<const uint2 *>(p);
        const uint32_t d[2] = {two.x, two.y};
        // header: word i carries scale bits 2i,2i+1 at 14-15 and offset bits at 30-31; the four threads of a
        // block sit in one quad of lanes and OR their parts together
        uint32_t h = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int wi = 2 * qd + i;
            h |= ((d[i] >> 14) & 3u) << (2 * wi) | ((d[i] >> 30) & 3u) << (16 + 2 * wi);
        }
        h |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h, 0xB1, 0xF, 0xF, true);
        h |= (uint32_t)__builtin_amdgcn_update_dpp(0, (int)h, 0x4E, 0xF, 0xF, true);
        const half2_t so = as_h2(h);
        const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
        const half2_t m1025 = {(half_t)-1025.0f, (half_t)-1025.0f}, m1024 = {(half_t)-1024.0f, (half_t)-1024.0f};
        const half2_t m11 = {(half_t)-11.0f, (half_t)-11.0f};
#pragma unroll
        for (int i = 0; i < 2; ++i) {
#pragma unroll
            for (int hsel = 0; hsel < 2; ++hsel) {
                // two pair codes in the two halves of a register: (4wi, 4wi+1) at bits 0/16, (4wi+2, 4wi+3) at bits 7/23
                const uint32_t hc = ((d[i] >> (7 * hsel)) & 0x007F007Fu) | 0x64006400u;
                const half2_t q1 = q3h_high_digit(hc) + m1025;                       // floor(c/11), exact
                const half2_t c = as_h2(hc) + m1024;                                 // c, exact
                const half2_t q2 = __builtin_elementwise_fma(q1, m11, c);            // c - 11 q1 = c mod 11, exact
                const half2_t w1 = __builtin_elementwise_fma(q1, s2, o2);            // (w[4m], w[4m+2])   Eq.2, one rounding
                const half2_t w2 = __builtin_elementwise_fma(q2, s2, o2);            // (w[4m+1], w[4m+3])
                out[4 * i + 2 * hsel] = __builtin_amdgcn_perm(pack_h2(w2), pack_h2(w1), 0x05040100u);      // (w[4m], w[4m+1])
                out[4 * i + 2 * hsel + 1] = __builtin_amdgcn_perm(pack_h2(w2), pack_h2(w1), 0x07060302u);  // (w[4m+2], w[4m+3])
            }
        }
    } else {
        const int k0 = kb * 64 + qd * 16;
        const uint32_t hdr = *reinterpret_cast<const uint32_t *>(packed + header_offset + (row * nbk + k0 / T::block) * 4);
        const half2_t so = as_h2(hdr);
        const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
        const half2_t m1024 = {(half_t)-1024.0f, (half_t)-1024.0f}, m64 = {(half_t)-64.0f, (half_t)-64.0f};
        if (T::kind == KIND_Q4) {
            const uint2 two = *reinterpret_cast<const uint2 *>(packed + row * (int64_t)(nbk * T::block / 2) + k0 / 2);
            const uint32_t d[2] = {two.x, two.y};
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t e = d[i] >> 8;
                const half2_t q0 = as_h2((d[i] & 0x000F000Fu) | 0x64006400u) + m1024;   // (v0, v1)
                const half2_t q1 = as_h2((d[i] & 0x00F000F0u) | 0x54005400u) + m64;     // (v2, v3)
                const half2_t q2 = as_h2((e & 0x000F000Fu) | 0x64006400u) + m1024;      // (v4, v5)
                const half2_t q3 = as_h2((e & 0x00F000F0u) | 0x54005400u) + m64;        // (v6, v7)
                out[4 * i] = pack_h2(__builtin_elementwise_fma(q0, s2, o2));
                out[4 * i + 1] = pack_h2(__builtin_elementwise_fma(q1, s2, o2));
                out[4 * i + 2] = pack_h2(__builtin_elementwise_fma(q2, s2, o2));
                out[4 * i + 3] = pack_h2(__builtin_elementwise_fma(q3, s2, o2));
            }
        } else {
            const uint4 four = *reinterpret_cast<const uint4 *>(packed + row * (int64_t)(nbk * T::block) + k0);
            const uint32_t d[4] = {four.x, four.y, four.z, four.w};
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const half2_t q0 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[i], 0x04010400u)) + m1024;   // (b0, b1)
                const half2_t q1 = as_h2(__builtin_amdgcn_perm(0x64646464u, d[i], 0x04030402u)) + m1024;   // (b2, b3)
                out[2 * i] = pack_h2(__builtin_elementwise_fma(q0, s2, o2));
                out[2 * i + 1] = pack_h2(__builtin_elementwise_fma(q1, s2, o2));
            }
        }
    }
}

template <int F>
__global__ __launch_bounds__(256) void qgemm_mfma_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                         uint16_t *__restrict__ Y, int rows, int cols, int batch, int nbk,
                                                         int64_t header_offset)
{
    __shared__ __align__(16) uint16_t xs[GM_BM * GM_LD];       // activations  [128][68]
    __shared__ __align__(16) uint16_t ws[GM_BN * GM_LD];       // weights      [64][68]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * GM_BN, m0 = blockIdx.y * GM_BM;
    const int wm = wave >> 1, wn = wave & 1;                   // this wavefront: batch rows wm*64.., weight rows wn*32..

    // loaders: activations - thread -> (row tid/2, 32 halves at (tid%2)*32); weights - thread -> (row tid/4, quarter tid%4)
    const int xr = tid >> 1, xh = tid & 1;
    const int64_t xrow = min(m0 + xr, batch - 1);              // rows past the batch repeat the last row, their outputs are not stored
    const uint4 *xsrc = reinterpret_cast<const uint4 *>(X + xrow * cols + xh * 32);
    const int wr = tid >> 2, wq = tid & 3;
    const int64_t wrow = min(n0 + wr, rows - 1);

    float16_t acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;

    const int nchunks = cols / GM_BK;
    for (int kb = 0; kb < nchunks; ++kb) {
        uint4 xv[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) xv[j] = xsrc[(int64_t)kb * 8 + j];   // 64 halves per row and chunk = 8 uint4; this thread's half = 4
        uint32_t wv[8];
        dequant16<F>(packed, header_offset, wrow, nbk, kb, wq, wv);
        __syncthreads();                                       // the previous chunk's MFMAs are done with LDS
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<uint4 *>(&xs[xr * GM_LD + xh * 32 + j * 8]) = xv[j];
        *reinterpret_cast<uint4 *>(&ws[wr * GM_LD + wq * 16]) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
        *reinterpret_cast<uint4 *>(&ws[wr * GM_LD + wq * 16 + 8]) = make_uint4(wv[4], wv[5], wv[6], wv[7]);
        __syncthreads();
        const int li = lane & 31, kg = lane >> 5;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const half4_t bfrag = *reinterpret_cast<const half4_t *>(&ws[(wn * 32 + li) * GM_LD + ks * 8 + kg * 4]);
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const half4_t afrag = *reinterpret_cast<const half4_t *>(&xs[(wm * 64 + i * 32 + li) * GM_LD + ks * 8 + kg * 4]);
                acc[i] = __builtin_amdgcn_mfma_f32_32x32x8f16(afrag, bfrag, acc[i], 0, 0, 0);
            }
        }
    }

    // 32x32 accumulator layout: register v of lane l is D[(v/4)*8 + (l/32)*4 + v%4][l%32]
    const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int brow = m0 + wm * 64 + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (brow < batch && col < rows) Y[(int64_t)brow * rows + col] = as_u16((half_t)acc[i][v]);
        }
}

template <int F>
static hipError_t gemm_one(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    typedef Fmt<F> T;
    const int nbk = (int)(cols / T::block);
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    const dim3 grid((unsigned)((rows + GM_BN - 1) / GM_BN), (unsigned)((batch + GM_BM - 1) / GM_BM));
    if (grid.y > 65535u) return hipErrorInvalidValue;
    hipLaunchKernelGGL((qgemm_mfma_kernel<F>), grid, dim3(256), 0, s,
                       static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk, header_offset);
    return hipGetLastError();
}

hipError_t launch_qgemm_mfma(int format, const void *packed, int64_t rows, int64_t cols,
                             const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    switch (format) {
    case IFLOW_Q8_B32: return gemm_one<IFLOW_Q8_B32>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q8_B64: return gemm_one<IFLOW_Q8_B64>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q4_B32: return gemm_one<IFLOW_Q4_B32>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q4_B64: return gemm_one<IFLOW_Q4_B64>(packed, rows, cols, X, batch, Y, s);
    case IFLOW_Q3H_B64: return gemm_one<IFLOW_Q3H_B64>(packed, rows, cols, X, batch, Y, s);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace iflow
