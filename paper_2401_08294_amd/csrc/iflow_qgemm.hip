// Dequantize-and-multiply on the matrix cores for batches large enough to make the product a dense
// contraction: Y[b][n] = sum_k w'[n][k] X[b][k].
//
// A workgroup of four wavefronts owns a 128 (batch; 64 for batches up to 64) x 64 (weight rows) tile of Y and walks along K in
// chunks of 64 columns, i.e. one quantization block per weight row (two for the 32-wide formats).  Per chunk
// it (1) copies the 128 x 64 fp16 activation tile into LDS, (2) decodes its 64 packed blocks into fp16
// weights in LDS - Eq.5 and Eq.2 of the paper, with the same single-rounded fp16 fused multiply-add as the
// stand-alone dequantizer, so the tile holds exactly the values iflow_dequant would produce - and (3) runs
// v_mfma_f32_32x32x16_f16 from LDS, fp32 accumulation.  Each wavefront owns a 64 x 32 part of the tile (two
// 32 x 32 output tiles).  Rows of the LDS tiles are padded to 72 halves (144 bytes) so that 16-byte operand reads
// of neighbouring rows fall into different banks.
#include "iflow_common.h"

namespace iflow {

typedef _Float16 half8_t __attribute__((ext_vector_type(8)));
typedef float float16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));

constexpr int GM_BN = 64, GM_BK = 64, GM_LD = 72;   // weight rows and columns per tile (batch rows: a template parameter); LDS row pitch in halves (144 bytes)

__device__ __forceinline__ uint32_t pack_h2(half2_t v) { return as_u32(v); }

// Raw material for sixteen consecutive weights (k = 16*qd .. 16*qd+15 of a 64-column chunk) of one row:
// the code words and the block header bits this thread can see.
struct Raw16 { uint32_t d[4]; uint32_t hdr; };

// (bit-plane formats: d[0..1] = the low plane's 8 or 4 bytes, d[2] = the high plane's word; `plane_b` = where the high
// plane starts in the packed matrix)
template <int F>
__device__ __forceinline__ void load16(const uint8_t *packed, int64_t header_offset, int64_t plane_b, int64_t row, int nbk,
                                       int kb /* 64-column chunk */, int qd, Raw16 &r)
{
    typedef Fmt<F> T;
    if constexpr (kind_has_planes(T::kind)) {
        constexpr int WA = Planes<T::kind>::WA, WB = Planes<T::kind>::WB;
        const int64_t cols = (int64_t)nbk * T::block;
        const int k0 = kb * 64 + qd * 16;
        r.hdr = *reinterpret_cast<const uint32_t *>(packed + header_offset + (row * nbk + k0 / T::block) * 4);
        r.d[1] = 0; r.d[2] = 0; r.d[3] = 0;
        if constexpr (WA == 4) {
            const uint2 two = *reinterpret_cast<const uint2 *>(packed + row * (cols / 2) + k0 / 2);
            r.d[0] = two.x; r.d[1] = two.y;
        } else {
            r.d[0] = *reinterpret_cast<const uint32_t *>(packed + row * (cols / 4) + k0 / 4);
        }
        if constexpr (WB == 2) r.d[2] = *reinterpret_cast<const uint32_t *>(packed + plane_b + row * (cols / 4) + k0 / 4);
        if constexpr (WB == 1) r.d[2] = *reinterpret_cast<const uint32_t *>(packed + plane_b + row * (cols / 8) + (k0 / 32) * 4);
    } else if (T::kind == KIND_Q3H) {
        // words 2qd, 2qd+1 of the block: plane qd/2, 8 bytes at offset (qd%2)*8 inside the block's 16 bytes
        const int t = kb >> 6, jin = kb & 63;
        const int n_t = min(64, nbk - (t << 6));
        const uint8_t *p = packed + row * (int64_t)nbk * 32 + (int64_t)t * 2048 + (qd >> 1) * n_t * 16 + jin * 16 + (qd & 1) * 8;
        const uint2 two = *reinterpret_cast<const uint2 *>(p);
        r.d[0] = two.x; r.d[1] = two.y; r.d[2] = 0; r.d[3] = 0; r.hdr = 0;
    } else {
        const int k0 = kb * 64 + qd * 16;
        r.hdr = *reinterpret_cast<const uint32_t *>(packed + header_offset + (row * nbk + k0 / T::block) * 4);
        if (T::kind == KIND_Q4) {
            const uint2 two = *reinterpret_cast<const uint2 *>(packed + row * (int64_t)(nbk * T::block / 2) + k0 / 2);
            r.d[0] = two.x; r.d[1] = two.y; r.d[2] = 0; r.d[3] = 0;
        } else {
            const uint4 four = *reinterpret_cast<const uint4 *>(packed + row * (int64_t)(nbk * T::block) + k0);
            r.d[0] = four.x; r.d[1] = four.y; r.d[2] = four.z; r.d[3] = four.w;
        }
    }
}

// Eq.5 and Eq.2: the sixteen weights as eight fp16 pairs in natural order, bit-identical to iflow_dequant.
template <int F>
__device__ __forceinline__ void decode16(const Raw16 &r, int qd, uint32_t (&out)[8])
{
    typedef Fmt<F> T;
    if constexpr (kind_has_planes(T::kind)) {
        constexpr int WA = Planes<T::kind>::WA, WB = Planes<T::kind>::WB;
        const half2_t so = as_h2(r.hdr);
        const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
        half2_t lo[8], hi[8];
        plane_fields16<WA>(&r.d[0], 0, lo);
        if constexpr (WB > 0) plane_fields16<WB>(&r.d[2], qd & 1, hi);                 // a 1-bit word serves two quarters
        const half2_t up = {(half_t)(float)(1 << WA), (half_t)(float)(1 << WA)};
#pragma unroll
        for (int m = 0; m < 8; ++m) {
            half2_t level = lo[m];
            if constexpr (WB > 0) level = __builtin_elementwise_fma(hi[m], up, lo[m]);   // exact: an integer below 64
            out[m] = pack_h2(__builtin_elementwise_fma(level, s2, o2));                  // Eq.2, one rounding
        }
    } else if (T::kind == KIND_Q3H) {
        // header: word i carries scale bits 2i,2i+1 at 14-15 and offset bits at 30-31; the four threads of a
        // block sit in one quad of lanes and OR their parts together
        uint32_t h = 0;
#pragma unroll
        for (int i = 0; i < 2; ++i) {
            const int wi = 2 * qd + i;
            h |= ((r.d[i] >> 14) & 3u) << (2 * wi) | ((r.d[i] >> 30) & 3u) << (16 + 2 * wi);
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
                const uint32_t hc = ((r.d[i] >> (7 * hsel)) & 0x007F007Fu) | 0x64006400u;
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
        const half2_t so = as_h2(r.hdr);
        const half2_t s2 = {so.x, so.x}, o2 = {so.y, so.y};
        const half2_t m1024 = {(half_t)-1024.0f, (half_t)-1024.0f}, m64 = {(half_t)-64.0f, (half_t)-64.0f};
        if (T::kind == KIND_Q4) {
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const uint32_t d = r.d[i], e = d >> 8;
                const half2_t q0 = as_h2((d & 0x000F000Fu) | 0x64006400u) + m1024;      // (v0, v1)
                const half2_t q1 = as_h2((d & 0x00F000F0u) | 0x54005400u) + m64;        // (v2, v3)
                const half2_t q2 = as_h2((e & 0x000F000Fu) | 0x64006400u) + m1024;      // (v4, v5)
                const half2_t q3 = as_h2((e & 0x00F000F0u) | 0x54005400u) + m64;        // (v6, v7)
                out[4 * i] = pack_h2(__builtin_elementwise_fma(q0, s2, o2));
                out[4 * i + 1] = pack_h2(__builtin_elementwise_fma(q1, s2, o2));
                out[4 * i + 2] = pack_h2(__builtin_elementwise_fma(q2, s2, o2));
                out[4 * i + 3] = pack_h2(__builtin_elementwise_fma(q3, s2, o2));
            }
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const half2_t q0 = as_h2(__builtin_amdgcn_perm(0x64646464u, r.d[i], 0x04010400u)) + m1024;   // (b0, b1)
                const half2_t q1 = as_h2(__builtin_amdgcn_perm(0x64646464u, r.d[i], 0x04030402u)) + m1024;   // (b2, b3)
                out[2 * i] = pack_h2(__builtin_elementwise_fma(q0, s2, o2));
                out[2 * i + 1] = pack_h2(__builtin_elementwise_fma(q1, s2, o2));
            }
        }
    }
}

// (The inputs are deliberately not declared __restrict__: loads from memory the compiler knows to be read-only and
// unaliased are free to move, and the scheduler then sinks the prefetch of a later chunk down to its use, four
// barriers later, to save registers - which turns every chunk into a full memory round trip.)
template <int F, int MT>
__global__ __launch_bounds__(256) void qgemm_mfma_kernel(const uint8_t *packed, const uint16_t *X, uint16_t *Y, int rows, int cols,
                                                         int batch, int nbk, int64_t header_offset)
{
    // two LDS stages: while the MFMAs read one, the next chunk is written into the other
    constexpr int BM = 64 * MT;                                // batch rows per workgroup: 128, or 64 where that gives the part more workgroups
    __shared__ __align__(16) uint16_t xs[2][BM * GM_LD];       // activations  [BM][72]
    __shared__ __align__(16) uint16_t ws[2][GM_BN * GM_LD];    // weights      [64][68]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n0 = blockIdx.x * GM_BN, m0 = blockIdx.y * BM;
    const int wm = wave >> 1, wn = wave & 1;                   // this wavefront: batch rows wm*64.., weight rows wn*32..

    // loaders: activations - thread -> (row tid/2, 32 halves at (tid%2)*32); weights - thread -> (row tid/4, quarter tid%4)
    const int xr = MT == 2 ? tid >> 1 : tid >> 2, xh = MT == 2 ? tid & 1 : tid & 3;   // (MT == 1: row tid/4, 16 halves at (tid%4)*16)
    const int64_t xrow = min(m0 + xr, batch - 1);              // rows past the batch repeat the last row, their outputs are not stored
    const u32x4_t *xsrc = reinterpret_cast<const u32x4_t *>(X + xrow * cols + xh * (16 * MT));
    const int wr = tid >> 2, wq = tid & 3;
    const int64_t wrow = min(n0 + wr, rows - 1);
    const int nchunks = cols / GM_BK;
    const int64_t plane_b = (int64_t)rows * cols * Planes<Fmt<F>::kind>::WA / 8;   // bit-plane formats: start of the high plane

    // (plain vector types and separately named stages: an array of structs that hold HIP's uint4 class is not split
    // into registers completely, and the part left over is parked in LDS, with a full wait right after its load)
    struct Stage { u32x4_t x0, x1, x2, x3; Raw16 w; };
    auto fetch = [&](Stage &st, int kb) {                      // global -> registers; chunks past the end repeat the last one
        const int kc = min(kb, nchunks - 1);
        const u32x4_t *xp = xsrc + (int64_t)kc * 8;            // 64 halves per row and chunk = 8 x 16 bytes; this thread's half = 4
        st.x0 = xp[0]; st.x1 = xp[1];
        if constexpr (MT == 2) { st.x2 = xp[2]; st.x3 = xp[3]; }
        load16<F>(packed, header_offset, plane_b, wrow, nbk, kc, wq, st.w);
    };
    auto stash = [&](const Stage &st, int buf) {               // registers -> LDS, weights decoded on the way
        uint32_t wv[8];
        decode16<F>(st.w, wq, wv);
        u32x4_t *xd = reinterpret_cast<u32x4_t *>(&xs[buf][xr * GM_LD + xh * (16 * MT)]);
        xd[0] = st.x0; xd[1] = st.x1;
        if constexpr (MT == 2) { xd[2] = st.x2; xd[3] = st.x3; }
        *reinterpret_cast<uint4 *>(&ws[buf][wr * GM_LD + wq * 16]) = make_uint4(wv[0], wv[1], wv[2], wv[3]);
        *reinterpret_cast<uint4 *>(&ws[buf][wr * GM_LD + wq * 16 + 8]) = make_uint4(wv[4], wv[5], wv[6], wv[7]);
    };

    // four independent accumulator chains per wavefront (two output tiles x even/odd k-steps), summed at the end:
    // a chain's next MFMA then never waits for its previous one
    float16_t acc[MT][2];
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int p = 0; p < 2; ++p)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][p][v] = 0.f;
    const int li = lane & 31, kg = lane >> 5;
    // The operand fragments of a whole chunk are read into registers of their own first (twelve 16-byte LDS reads), the
    // next chunk's decode and LDS writes are issued behind them, and only then come the eight MFMAs: left to itself the
    // compiler reads each fragment into the same few registers right before its MFMA and waits for it there - a full LDS
    // round trip in front of every MFMA, 1500 cycles per chunk for 256 cycles of matrix-core work.
    half8_t af[MT][4], bf[4];
    auto read_fragments = [&](int buf) {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {                       // 16 columns per step: lane (li, kg) holds k = 8 kg .. 8 kg + 7
            bf[ks] = *reinterpret_cast<const half8_t *>(&ws[buf][(wn * 32 + li) * GM_LD + ks * 16 + kg * 8]);
#pragma unroll
            for (int i = 0; i < MT; ++i)
                af[i][ks] = *reinterpret_cast<const half8_t *>(&xs[buf][(wm * 32 * MT + i * 32 + li) * GM_LD + ks * 16 + kg * 8]);
        }
    };
    auto multiply = [&]() {
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int i = 0; i < MT; ++i)
                acc[i][ks & 1] = __builtin_amdgcn_mfma_f32_32x32x16_f16(af[i][ks], bf[ks], acc[i][ks & 1], 0, 0, 0);
    };

    // Software pipeline: chunk c multiplies from one LDS stage while chunk c+1 is decoded into the other and chunks
    // c+2 .. c+4 are in flight from memory in four register stages (a request is issued about four chunk-times
    // before its data is needed, which covers the HBM latency with a single wavefront per SIMD).  Four chunks per
    // trip so that the register stages keep their roles without copies; chunks past the end repeat the last one
    // and are never multiplied.
    Stage sa, sb, sc, sd;
    fetch(sa, 0); fetch(sb, 1); fetch(sc, 2); fetch(sd, 3);
    stash(sa, 0);
    fetch(sa, 4);
    __syncthreads();
    // Whole trips first, without any branch around the loads: with a load under a branch the compiler can no longer
    // count which outstanding load a register belongs to and waits for all of them, the newest request included.
    int kb = 0;
#define IFLOW_GEMM_STEP(ST, U)        /* chunk kb+U multiplies; chunk kb+U+1 goes to the other LDS stage; ST is refilled */ \
    read_fragments((kb + U) & 1); __builtin_amdgcn_sched_barrier(0);                                                          \
    stash(ST, (kb + U + 1) & 1); fetch(ST, kb + U + 5); __builtin_amdgcn_sched_barrier(0);                                    \
    multiply(); __syncthreads();
    for (; kb + 4 <= nchunks; kb += 4) {
        IFLOW_GEMM_STEP(sb, 0) IFLOW_GEMM_STEP(sc, 1) IFLOW_GEMM_STEP(sd, 2) IFLOW_GEMM_STEP(sa, 3)
    }
#undef IFLOW_GEMM_STEP
#define IFLOW_GEMM_TAIL(ST, U) if (kb + U < nchunks) { read_fragments((kb + U) & 1); stash(ST, (kb + U + 1) & 1); multiply(); __syncthreads(); }
    IFLOW_GEMM_TAIL(sb, 0) IFLOW_GEMM_TAIL(sc, 1) IFLOW_GEMM_TAIL(sd, 2)      // the last one to three chunks
#undef IFLOW_GEMM_TAIL

    // 32x32 accumulator layout: register v of lane l is D[(v/4)*8 + (l/32)*4 + v%4][l%32]
    const int col = n0 + wn * 32 + (lane & 31);
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int brow = m0 + wm * 32 * MT + i * 32 + (v >> 2) * 8 + (lane >> 5) * 4 + (v & 3);
            if (brow < batch && col < rows) Y[(int64_t)brow * rows + col] = as_u16((half_t)(acc[i][0][v] + acc[i][1][v]));
        }
}

template <int F>
static hipError_t gemm_one(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    typedef Fmt<F> T;
    const int nbk = (int)(cols / T::block);
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    // 128 batch rows per workgroup; 64 for batches that would leave half of a 128-row tile empty (32-64 vectors: 25 us instead
    // of 33 on 4096 x 4096).  With more vectors the smaller tile only adds workgroups that re-read the weights (measured:
    // 36.7 against 34.7 us at 512 vectors).
    const int64_t nx = (rows + GM_BN - 1) / GM_BN;
    const bool small_tiles = batch <= 64;
    const int bm = small_tiles ? 64 : 128;
    const dim3 grid((unsigned)nx, (unsigned)((batch + bm - 1) / bm));
    if (grid.y > 65535u) return hipErrorInvalidValue;
    if (small_tiles)
        hipLaunchKernelGGL((qgemm_mfma_kernel<F, 1>), grid, dim3(256), 0, s,
                           static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk, header_offset);
    else
        hipLaunchKernelGGL((qgemm_mfma_kernel<F, 2>), grid, dim3(256), 0, s,
                           static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, (int)batch, nbk, header_offset);
    return hipGetLastError();
}

hipError_t launch_qgemm_mfma(int format, const void *packed, int64_t rows, int64_t cols,
                             const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s)
{
    return for_format(format, [&](auto f) { return gemm_one<decltype(f)::value>(packed, rows, cols, X, batch, Y, s); });
}

}  // namespace iflow
