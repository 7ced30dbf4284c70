// Fused dequantize-and-multiply on the vector units: y = W' x at batch 1 (the decode step's weight
// stream) and up to four activation vectors per pass.  Eq.5 and Eq.2 of the paper are applied in
// registers; the dequantized weights never exist in memory.
//
// Two kernels live here.  q3h_gemv_kernel (further down) is the 3.5-bit format's: activations staged once per
// workgroup, rows owned by wavefronts; the other formats' counterpart of it is in iflow_qgemv_rows.hip.  qgemv_kernel
// (first) is the older, format-generic one that the launchers fall back to - rows too long for the staging, three or
// four vectors when the column count rules out the MFMA kernels:
//
// Mapping ("activation-stationary"): a wavefront owns one strip of the reduction dimension, 64 lanes x
// WPL consecutive weights, and walks down the rows.  Each lane keeps the activations of its own
// WPL columns in registers for the whole walk, so the inner loop touches memory only for weights:
// one to three loads per lane and row (16 bytes of codes, or a lane's share of each bit plane, and the header).
// Because the levels of a lane all share one block header,
//     sum_k (q_k * s + o) x_k  =  s * sum_k q_k x_k  +  o * sum_k x_k ,
// the per-weight work is one packed conversion and one dot2 step; scale and offset are applied once per
// lane and row.  Levels are converted to fp16 by OR-ing them into the mantissa of a power of two
// (1024 + q, 64 + q, ...), and the known bias times sum(x) is removed together with the header.
// Row sums are reduced across the wavefront with DPP, across the wavefronts of a workgroup (one per
// strip) through LDS.

#include "iflow_lane.h"

namespace iflow {

template <int F, int NB, int U, bool MULTI>
__global__ __launch_bounds__(MULTI ? 1024 : 64) void qgemv_kernel(const uint8_t *__restrict__ packed, const uint16_t *__restrict__ X,
                                                                  uint16_t *__restrict__ Y, int rows, int cols, int nbk, int rows_per_wg,
                                                                  int nstrips, int64_t header_offset)
{
    typedef Fmt<F> T;
    constexpr int KIND = T::kind;
    typedef Geo<KIND> G;
    __shared__ float part[MULTI ? 16 : 1][NB][64];

    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nw = blockDim.x >> 6;
    const int r0 = blockIdx.x * rows_per_wg;
    const int nr = min(rows_per_wg, rows - r0);               // 1..64 rows, row r0+i belongs to lane i
    float tot[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) tot[b] = 0.f;
    for (int t = wave; t < nstrips; t += nw) {
        // The last strip may be ragged: lanes past the end redo the strip's first lane (every load stays in
        // bounds and unconditional, so the compiler can wait per load) and their sums are dropped.
        const bool active = (t * 64 + lane) * G::WPL < cols;
        const int k0 = (t * 64 + (active ? lane : 0)) * G::WPL;   // first column of this lane
        const int lane_a = active ? lane : 0;

        // where this lane's codes (and, for Q4/Q8, its header) sit inside a row
        int64_t code_off, row_stride, hdr_off = 0;
        int64_t code_off_b = 0, row_stride_b = 0;             // bit-plane formats: the high plane
        int plane1 = 0;
        if constexpr (KIND == KIND_Q3H) {
            const int n_t = min(64, nbk - t * 64);
            row_stride = (int64_t)nbk * 32;
            code_off = (int64_t)t * 2048 + lane_a * 16;
            plane1 = n_t * 16;
        } else if constexpr (kind_has_planes(KIND)) {
            constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
            row_stride = (int64_t)cols * WA / 8;
            code_off = (int64_t)k0 * WA / 8;
            row_stride_b = (int64_t)cols * WB / 8;
            code_off_b = (int64_t)rows * cols * WA / 8 + (int64_t)k0 * WB / 8;
            hdr_off = header_offset + (int64_t)(k0 / T::block) * 4;
        } else {
            row_stride = (KIND == KIND_Q4) ? cols / 2 : cols;
            code_off = (KIND == KIND_Q4) ? k0 / 2 : k0;
            hdr_off = header_offset + (int64_t)(k0 / T::block) * 4;
        }
        const uint8_t *lane_base = packed + code_off;

        auto load_group = [&](WRegs<KIND>(&w)[U], int i) {
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int r = r0 + min(i + u, nr - 1);        // rows past the end repeat the last one and are dropped below
                const uint8_t *p = lane_base + (int64_t)r * row_stride;
                if constexpr (kind_has_planes(KIND)) {
                    // 32 weights: 16 or 8 bytes of the low plane, 8, 4 or no bytes of the high plane, the block's header
                    constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
                    if constexpr (WA == 4) {
                        uint4 a = *reinterpret_cast<const uint4 *>(p);
                        w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
                    } else {
                        uint2 a = *reinterpret_cast<const uint2 *>(p);
                        w[u].d[0] = a.x; w[u].d[1] = a.y;
                    }
                    const uint8_t *pb = packed + code_off_b + (int64_t)r * row_stride_b;
                    if constexpr (WB == 2) {
                        uint2 c = *reinterpret_cast<const uint2 *>(pb);
                        w[u].d[WA] = c.x; w[u].d[WA + 1] = c.y;
                    } else if constexpr (WB == 1) {
                        w[u].d[WA] = *reinterpret_cast<const uint32_t *>(pb);
                    }
                    w[u].hdr = *reinterpret_cast<const uint32_t *>(packed + hdr_off + (int64_t)r * nbk * 4);
                } else {
                    uint4 a = *reinterpret_cast<const uint4 *>(p);
                    w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
                    if constexpr (KIND == KIND_Q3H) {
                        uint4 c = *reinterpret_cast<const uint4 *>(p + plane1);
                        w[u].d[4] = c.x; w[u].d[5] = c.y; w[u].d[6] = c.z; w[u].d[7] = c.w;
                    } else {
                        w[u].hdr = *reinterpret_cast<const uint32_t *>(packed + hdr_off + (int64_t)r * nbk * 4);
                    }
                }
            }
        };

        // the first rows' weights are requested before anything waits on the activations
        WRegs<KIND> wa[U], wb[U];
        load_group(wa, 0);
        XRegs<KIND> xr[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) load_x<KIND>(xr[b], X + (int64_t)b * cols, k0);
        const float keep = active ? 1.0f : 0.0f;

        auto compute_group = [&](const WRegs<KIND>(&w)[U], int i) {
            float v[NB][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc[NB];
                lane_dot<KIND, NB>(w[u], xr, acc);
                uint32_t hdr;
                if constexpr (KIND == KIND_Q3H) hdr = q3h_header(reinterpret_cast<const uint32_t(&)[8]>(w[u].d)); else hdr = w[u].hdr;
                const half2_t so = as_h2(hdr);
                const float s = (float)so.x, o = (float)so.y;
#pragma unroll
                for (int b = 0; b < NB; ++b) v[b][u] = keep * __builtin_fmaf(s, acc[b] - xr[b].bias_sum, o * xr[b].x_sum);
            }
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const float r = reduce_rows<U>(v[b], lane);
                if ((lane & ~(U - 1)) == i) tot[b] += r;      // lane i+u (u = lane & (U-1)) takes row i+u; lanes >= nr are never stored
            }
        };

        // Two groups per trip: one computes while the other loads.  The loads are unconditional (rows past the end
        // repeat the last row, which is in cache by then): with a load under a branch the compiler waits for all
        // outstanding loads at the next use instead of only for the group it needs.
        for (int i = 0; i < nr; i += 2 * U) {
            load_group(wb, i + U);
            compute_group(wa, i);
            load_group(wa, i + 2 * U);
            if (i + U < nr) compute_group(wb, i + U);
        }
    }

    if (MULTI) {                                              // one wavefront per strip: add the strips up
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

// Up to eight matrices per launch (see q3h_gemv_kernel).
constexpr int IFLOW_MAX_GROUP = 8;
struct GemvGroup {
    const uint8_t *packed[IFLOW_MAX_GROUP];
    uint16_t *y[IFLOW_MAX_GROUP];
    int rows[IFLOW_MAX_GROUP];
    int wg_end[IFLOW_MAX_GROUP];                              // one past the last workgroup of matrix i
    int count;
};

// What the fused variant (template parameter XOP >= 0) does to the activations on their way into LDS and to the row sums
// on their way out; x_op values are iflow_x_op_t's.  The plain instantiations never read it.
struct GemvOps {
    const uint16_t *residual[IFLOW_MAX_GROUP];                // per matrix: added to the outputs, or null
    float eps[IFLOW_MAX_GROUP];                               // the same value for every matrix (read next to its residual, see the kernel)
};

// ---- Q3H: workgroup-shared activations ----------------------------------------------------------------
// The activations are the same for every wavefront, and arranging a strip of them for the decode costs
// about as much as one row of weights.  So a workgroup does it once: its threads permute the activations
// of up to T strips into LDS in decode order (plus the two bias constants per lane), and after one barrier
// every wavefront fetches the 32 registers of a strip with eight 16-byte LDS reads.  A wavefront owns U
// consecutive rows and walks along them strip by strip: per strip it requests the 2U weight loads, reloads
// its activation registers from LDS and decodes each row as soon as that row's two loads have landed.  The
// per-lane partial sums of a row are carried across the strips in a register, so a row is reduced across
// the wavefront once, with DPP adds, and no wavefront ever waits for another one after the barrier.
// Measured on MI355X: v_cndmask and ds_bpermute cost several times a plain add, so selects are written as
// masks or multiplications by 0/1; row base addresses are wave-uniform (scalar registers), so a weight load
// costs no vector arithmetic; the activation loads are issued before the first weight loads because memory
// queues are served in order and the whole workgroup waits for the staged activations.
//
// LDS layout per (strip, batch column): float4 xs[8][64] (register quad jj of lane l at [jj][l]), then
// float2 sums[64] = (bias_sum, x_sum) of lane l.
//
// One launch can serve several weight matrices that share the activation vector and the number of columns
// (the q/k/v or the gate/up projections of a decoder layer): workgroup ranges are assigned to the matrices
// in order, each matrix keeps its own packed buffer and output vector.
//
// XOP >= 0 (batch 1 only) fuses the modules around the linear layer into the same launch (Section 2 lists them as the
// configurable pieces of a decoder layer, Section 5's Infer() runs them between the products):
//   IFLOW_X_RMS_GAIN   the staged activations are fp16(x_k g_k) and every row sum is multiplied by
//                      1 / sqrt(mean x^2 + eps) - rms normalization, with its scalar moved behind the product;
//   IFLOW_X_SILU_MUL   the staged activations are fp16(silu(x_k) aux_k) - the input of a gated feed-forward's last layer;
//   residual           out_n = fp16(row sum + residual_n).
// GATED (with XOP = plain or rms gain, one matrix pair): a wavefront's two rows in flight are row n of a "gate" matrix
// and row n of an "up" matrix (grp.packed[0] and [1], both rows0 x cols), and the one output is
// fp16(silu(gate sum x scale) (up sum x scale)) - the gated feed-forward's hidden vector without storing its two factors.
template <int NB, int U, bool MULTI, int XOP = -1, bool GATED = false>
__global__ __launch_bounds__(NB <= 1 ? 1024 : 512) void q3h_gemv_kernel(const uint8_t *__restrict__ packed0, uint16_t *__restrict__ y0,
                                                        const uint16_t *__restrict__ X, int rows0, int cols, int nbk, int nstrips,
                                                        int tgw, int x_op, const uint16_t *__restrict__ aux,
                                                        const GemvGroup grp, const GemvOps ops)
{
    // XOP < 0: the plain kernel.  XOP = an iflow_x_op_t: the fused variant for that operation (one instantiation each, so
    // that a launch runs through no code of the operations it does not perform: a launch is short, and every taken
    // branch over a block of cold code costs an instruction-cache miss)
    constexpr bool OPS = XOP >= 0;
    static_assert(!OPS || NB == 1, "the fused variant is built for one activation vector");
    static_assert(!GATED || (OPS && !MULTI && U == 2), "the gated variant: one pair of matrices, two rows in flight");
    constexpr int RPG = GATED ? 1 : U;                        // output rows per row group
    (void)x_op;
    // strips staged per pass, row groups per wavefront, wavefronts per workgroup: packed into one argument (8 bits each)
    // so that the fourteen argument registers reach as far as `aux`
    const int T = tgw & 255, G = (tgw >> 8) & 255, waves = tgw >> 16;
    // The single-matrix arguments come first so that they fit the kernel-argument registers the hardware can preload
    // at wavefront start (no scalar load, no wait, before the first address is formed); `grp` is read only when MULTI.
    // x_op and aux (used by the fused variant only) are the last two that fit: the staging needs them at once, and a
    // scalar load that misses its cache would hold up the first activation loads.
    extern __shared__ __align__(16) uint8_t lds[];
    constexpr int SLOT_BYTES = 8 * 64 * 16 + 64 * 8;          // xs + sums of one (strip, batch column)
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);   // wave-uniform by construction: keep it scalar
    int m = 0;                                                // which matrix this workgroup belongs to
    if (MULTI) {
#pragma unroll
        for (int i = 0; i + 1 < IFLOW_MAX_GROUP; ++i)
            if (i + 1 < grp.count && (int)blockIdx.x >= grp.wg_end[i]) m = i + 1;
    }
    const int wg = MULTI ? blockIdx.x - (m ? grp.wg_end[m - 1] : 0) : blockIdx.x;
    const uint8_t *__restrict__ packed = MULTI ? grp.packed[m] : packed0;
    uint16_t *__restrict__ Y = MULTI ? grp.y[m] : y0;
    const int rows = MULTI ? grp.rows[m] : rows0;
    const int rbase = (wg * waves + wave) * (G * RPG);        // first row of this wavefront: G groups of U rows
    const uint8_t *__restrict__ packed_up = GATED ? grp.packed[1] : nullptr;
    const int64_t row_stride = (int64_t)nbk * 32;

    // weights of U rows of one strip: wave-uniform row base + per-lane offset, streamed once (nontemporal);
    // rows past the end repeat the last row and are not stored
    // (`none`: the request after the last step; it is issued all the same, with every lane on the matrix's first bytes,
    // so that no load sits under a branch - see the wait counters - and nothing of any size is fetched in vain)
    auto load_step = [&](WRegs<KIND_Q3H>(&w)[U], int r0, int t, bool none) {
        const int n_t = none ? 0 : min(64, nbk - t * 64);     // blocks in this strip (ragged at the end of a row)
        // lanes past the end redo block 0 so that loads stay in bounds
        const uint32_t lane_off = (uint32_t)(lane * 16) & mask_lt(lane, n_t);
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const uint8_t *mat = (GATED && u == 1) ? packed_up : packed;
            const uint8_t *p0 = none ? packed : mat + (int64_t)min(GATED ? r0 : r0 + u, rows - 1) * row_stride + (int64_t)t * 2048;
            const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p0 + lane_off));
            const u32x4 c = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p0 + n_t * 16 + lane_off));
            w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
            w[u].d[4] = c.x; w[u].d[5] = c.y; w[u].d[6] = c.z; w[u].d[7] = c.w;
        }
    };

    float part[NB][U];                                        // per-lane partial sums of a row group, carried across strips
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int u = 0; u < U; ++u) part[b][u] = 0.f;

    // fused variant: lane l holds the residual of the wavefront's l-th row (read back with v_readlane at the store);
    // ssq collects this thread's share of sum x^2; out_scale is the normalization's scalar once all of x has been seen
    float ssq = 0.f, out_scale = 1.0f, fused_eps = 0.f;
    uint16_t res_raw = 0;                                     // fp16 bits of the lane's residual (a 16-bit variable: widened where it is used)
    uint32_t res_keep = 0;                                    // 0xFFFF when there is a residual

    for (int t0 = 0; t0 < nstrips; t0 += T) {                 // one pass unless the row is longer than T strips (then G is 1)
        const int nt = min(T, nstrips - t0);                  // strips staged in this pass

        // 1. request this thread's first chunk of activations BEFORE any weights.
        //    Chunk c of a pass = (strip, batch column, block blk, quarter qd) with qd fastest: 16 activations
        //    that feed decode slots 4qd..4qd+3 of lane blk.  (NB is a compile-time constant: no integer division on
        //    the way to the first load.)
        const int nchunks = NB * nt * 256;
        auto chunk_src_of = [&](const uint16_t *base, int c) {
            const int cc = c & 255, ts = (c >> 8) / NB, bcol = (c >> 8) % NB;
            const int n_t = min(64, nbk - (t0 + ts) * 64);
            const int ccl = cc & (int)mask_lt(cc >> 2, n_t);  // chunks past the end of the row read chunk 0 and are zeroed
            return reinterpret_cast<const uint4 *>(base + (int64_t)bcol * cols + (int64_t)(t0 + ts) * 4096 + ccl * 16);
        };
        auto chunk_src = [&](int c) { return chunk_src_of(X, c); };
        // the fused variant's second operand of a chunk (gains or the second factor); the activations themselves when there is none
        const uint16_t *aux_base = (XOP > IFLOW_X_PLAIN) ? aux : X;
        auto chunk_put = [&](int c, const uint4 q0, const uint4 q1, const uint4 a0, const uint4 a1) {
            const int cc = c & 255, ts = (c >> 8) / NB, bcol = (c >> 8) % NB, blk = cc >> 2, qd = cc & 3;
            const int n_t = min(64, nbk - (t0 + ts) * 64);
            const uint32_t live = mask_lt(blk, n_t);              // all ones inside the row: columns past its end count as zero
            uint32_t n[8] = {q0.x & live, q0.y & live, q0.z & live, q0.w & live, q1.x & live, q1.y & live, q1.z & live, q1.w & live};
            if (OPS) {
                const uint32_t av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                if (XOP == IFLOW_X_RMS_GAIN) {           // (uniform) x_k g_k: exact product, one rounding to fp16
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        ssq = dot2(as_h2(n[k]), as_h2(n[k]), ssq);
                        n[k] = as_u32(as_h2(n[k]) * as_h2(av[k]));
                    }
                } else if (XOP == IFLOW_X_SILU_MUL) {    // silu(x_k) aux_k in fp32, one rounding to fp16
#pragma unroll
                    for (int k = 0; k < 8; ++k) {
                        const half2_t xa = as_h2(n[k]), xb = as_h2(av[k] & live);
                        const float g0 = (float)xa.x, g1 = (float)xa.y;
                        // (hardware reciprocal: 1 ulp of fp32, far below the fp16 rounding that follows)
                        const float v0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * (float)xb.x, v1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * (float)xb.y;
                        const half2_t r = {(half_t)v0, (half_t)v1};
                        n[k] = as_u32(r);
                    }
                }
            }
            const half2_t ones = {(half_t)1.0f, (half_t)1.0f};
            uint32_t e[4], o[4];
            float se = 0.f, so = 0.f;
#pragma unroll
            for (int m = 0; m < 4; ++m) {
                e[m] = __builtin_amdgcn_perm(n[2 * m + 1], n[2 * m], 0x05040100u);    // (x[4m], x[4m+2])
                o[m] = __builtin_amdgcn_perm(n[2 * m + 1], n[2 * m], 0x07060302u);    // (x[4m+1], x[4m+3])
                se = dot2(as_h2(e[m]), ones, se);
                so = dot2(as_h2(o[m]), ones, so);
            }
            uint8_t *sl = lds + (size_t)(ts * NB + bcol) * SLOT_BYTES;
            *reinterpret_cast<uint4 *>(sl + (qd * 64 + blk) * 16) = make_uint4(e[0], e[1], e[2], e[3]);
            *reinterpret_cast<uint4 *>(sl + ((4 + qd) * 64 + blk) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
            float bs = IFLOW_Q3H_BIAS1 * se + IFLOW_Q3H_BIAS2 * so, xs = se + so;
            bs += dpp_f32<0xB1, 0xF>(bs); xs += dpp_f32<0xB1, 0xF>(xs);              // the four quarters of a block
            bs += dpp_f32<0x4E, 0xF>(bs); xs += dpp_f32<0x4E, 0xF>(xs);              // sit in one quad of lanes
            if (qd == 0) *reinterpret_cast<float2 *>(sl + 8 * 64 * 16 + blk * 8) = make_float2(bs, xs);
        };
        const int c0 = threadIdx.x;
        const bool has_chunk = c0 < nchunks;                  // whole wavefronts have a first chunk or not
        const uint4 *src0 = chunk_src(c0 & (int)mask_lt(c0, nchunks));
        const uint4 xq0 = src0[0], xq1 = src0[1];
        constexpr bool HAS_AUX = XOP > IFLOW_X_PLAIN;          // the operation has a second operand
        const uint4 *asrc0 = HAS_AUX ? chunk_src_of(aux_base, c0 & (int)mask_lt(c0, nchunks)) : src0;
        const uint4 aq0 = HAS_AUX ? asrc0[0] : xq0, aq1 = HAS_AUX ? asrc0[1] : xq1;

        // 2. request the weights of the first step (first row group, first strip of the pass)
        WRegs<KIND_Q3H> w[U];
        load_step(w, rbase, t0, false);
        // (fused variant) The residual pointers and eps arrive by scalar loads.  Read at the top of the kernel, the wait
        // for them (a scalar-cache miss each time a launch starts) would sit in front of the activation and weight
        // requests above; the index is made opaque so that the reads cannot be moved up there.
        const uint16_t *res = nullptr;
        if (OPS) {
            __builtin_amdgcn_sched_barrier(0);
            int mi = m;
            asm volatile("" : "+s"(mi));
            fused_eps = ops.eps[mi];
            res = ops.residual[mi];
            // the wavefront's residuals, lane l for its l-th row (without a residual: x[0], dropped).  Requested behind the
            // first weights and under no branch; kept as loaded and touched again only at the store, so that the only
            // wait it shares is the one in front of the step loop, which needs the first weights anyway.
            const uint16_t *rp = res != nullptr ? res + min(rbase + min(lane, G * U - 1), rows - 1) : X;
            res_raw = *rp;
            res_keep = res != nullptr ? 0xFFFFu : 0u;
        }

        // 3. stage: permute the activations into decode order in LDS
        if (t0 > 0) __syncthreads();                          // the previous pass is done with LDS
        if (has_chunk) chunk_put(c0, xq0, xq1, aq0, aq1);
#pragma unroll 1
        for (int c = c0 + waves * 64; c < nchunks; c += waves * 64) {
            const uint4 *src = chunk_src(c);
            const uint4 x0 = src[0], x1 = src[1];
            const uint4 *asrc = HAS_AUX ? chunk_src_of(aux_base, c) : src;
            chunk_put(c, x0, x1, HAS_AUX ? asrc[0] : x0, HAS_AUX ? asrc[1] : x1);
        }
        // fused normalization: the wavefronts' shares of sum x^2 go through sixteen floats behind the staged strips; the
        // sum is complete in the pass that stages the row's last strip, which is also the pass that stores the outputs
        float *ssq_part = reinterpret_cast<float *>(lds + (size_t)T * NB * SLOT_BYTES);
        if (OPS && XOP == IFLOW_X_RMS_GAIN && t0 + nt == nstrips) {
            const float wsum = wave_sum_to_lane63(ssq);
            if (lane == 63) ssq_part[wave] = wsum;
        }
        __syncthreads();
        if (OPS && t0 + nt == nstrips && XOP == IFLOW_X_RMS_GAIN) {
            const float mine = lane < waves ? ssq_part[lane] : 0.f;
            const float total = wave_sum(mine);
            out_scale = 1.0f / __builtin_sqrtf(total / (float)cols + fused_eps);
        }

        // 4. steps = (row group, strip): activation registers from LDS, then each row as its loads land, while
        //    the next step's weights are already requested
        XRegs<KIND_Q3H> xr[NB];
        const int nsteps = G * nt;
        int g = 0, ts = 0;
#pragma unroll 1
        for (int step = 0; step < nsteps; ++step) {
            const int r0 = rbase + g * RPG;
            if (nt > 1 || step == 0) {                        // a single strip stays in registers for all row groups
#pragma unroll
                for (int b = 0; b < NB; ++b) {
                    const uint8_t *sl = lds + (size_t)(ts * NB + b) * SLOT_BYTES;
#pragma unroll
                    for (int jj = 0; jj < 8; ++jj) {
                        const uint4 q = *reinterpret_cast<const uint4 *>(sl + (jj * 64 + lane) * 16);
                        xr[b].v[4 * jj] = as_h2(q.x); xr[b].v[4 * jj + 1] = as_h2(q.y);
                        xr[b].v[4 * jj + 2] = as_h2(q.z); xr[b].v[4 * jj + 3] = as_h2(q.w);
                    }
                    const float2 sm = *reinterpret_cast<const float2 *>(sl + 8 * 64 * 16 + lane * 8);
                    xr[b].bias_sum = sm.x; xr[b].x_sum = sm.y;
                }
            }
            float v[NB][U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                float acc[NB];
                lane_dot<KIND_Q3H, NB>(w[u], xr, acc);
                const half2_t so = as_h2(q3h_header(w[u].d));
                const float s = (float)so.x, o = (float)so.y;
#pragma unroll
                for (int b = 0; b < NB; ++b)                  // lanes past the end of a ragged strip see x = 0 and add nothing
                    v[b][u] = part[b][u] + __builtin_fmaf(s, acc[b] - xr[b].bias_sum, o * xr[b].x_sum);
            }
            // next step's weights (wave-uniform control flow only)
            int gn = g, tn = ts + 1;
            if (tn == nt) { tn = 0; gn = g + 1; }
            load_step(w, rbase + gn * RPG, t0 + tn, step + 1 >= nsteps);

            const bool group_done = ts == nt - 1 && t0 + nt == nstrips;
            if (GATED && group_done) {                        // both factors of output r0 end up in lane 63
                const float gate = wave_sum_to_lane63(v[0][0]) * out_scale, up = wave_sum_to_lane63(v[0][U - 1]) * out_scale;
                const float hv = gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
                if (lane == 63 && r0 < rows) Y[r0] = as_u16((half_t)hv);
#pragma unroll
                for (int u = 0; u < U; ++u) part[0][u] = 0.f;
            } else if (group_done) {                          // one reduction per row; lane 63 holds the sums
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        float sum = wave_sum_to_lane63(v[b][u]);
                        if (OPS) {
                            uint16_t rr = res_raw;
                            asm volatile("" : "+v"(rr));                      // first touched here: the load is not waited for before the loop
                            const uint32_t rb = (uint32_t)__builtin_amdgcn_readlane((int)rr, g * U + u) & res_keep;
                            sum = __builtin_fmaf(sum, out_scale, (float)as_h((uint16_t)rb));
                        }
                        if (lane == 63 && r0 + u < rows) Y[(int64_t)b * rows + r0 + u] = as_u16((half_t)sum);
                        part[b][u] = 0.f;
                    }
            } else {
#pragma unroll
                for (int b = 0; b < NB; ++b)
#pragma unroll
                    for (int u = 0; u < U; ++u) part[b][u] = v[b][u];
            }
            g = gn; ts = tn;
        }
    }
}

// ---- host side ------------------------------------------------------------------------------------
// Launch geometry: one wavefront per strip (at most 16 per workgroup, further strips are looped), and
// rows_per_wg chosen so that the grid has a few wavefronts per SIMD on a 256-CU part.
static int pick_rows_per_wg(int64_t rows, int waves_per_wg)
{
    const int64_t target_waves = 256 * 4 * 2;
    int64_t r = (rows * waves_per_wg + target_waves - 1) / target_waves;
    r = (r + 3) / 4 * 4;                                      // whole groups of four rows
    if (r < 4) r = 4;
    if (r > 64) r = 64;
    return (int)r;
}

template <int NB, int U, int XOP = -1, bool GATED = false>
static hipError_t q3h_launch_u(GemvGroup grp, int64_t cols, const uint16_t *X, int waves, int G, hipStream_t s, const GemvOps &ops = GemvOps(),
                              int x_op = IFLOW_X_PLAIN, const uint16_t *aux = nullptr)
{
    constexpr int SLOT = 8 * 64 * 16 + 64 * 8;
    const int nbk = (int)(cols / 64);
    const int nstrips = (nbk + 63) / 64;
    int T = (152 * 1024) / (SLOT * NB);
    if (T > nstrips) T = nstrips;
    const size_t lds = (size_t)T * NB * SLOT + (XOP >= 0 ? 64 : 0);  // (fused variant: sixteen floats for the sum of squares)
    static PerDevice pd;                                      // raise the dynamic-LDS cap once per instantiation and device
    int cus = 0;
    hipError_t e = once_per_device(pd, &cus, [] {
        hipError_t r = hipFuncSetAttribute(reinterpret_cast<const void *>(&q3h_gemv_kernel<NB, U, false, XOP, GATED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        if constexpr (!GATED) {
            if (r == hipSuccess)
                r = hipFuncSetAttribute(reinterpret_cast<const void *>(&q3h_gemv_kernel<NB, U, true, XOP>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 152 * 1024);
        }
        return r;
    });
    if (e != hipSuccess) return e;
    if (T < nstrips) G = 1;                                   // multi-pass rows: partial sums live in registers, one group only
    const int64_t rows_per_wg = (int64_t)waves * (GATED ? 1 : U) * G;
    int64_t grid = 0;
    for (int i = 0; i < (GATED ? 1 : grp.count); ++i) {       // (gated: the pair's two matrices are one set of output rows)
        grid += (grp.rows[i] + rows_per_wg - 1) / rows_per_wg;
        grp.wg_end[i] = (int)grid;
    }
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if constexpr (GATED)
        hipLaunchKernelGGL((q3h_gemv_kernel<NB, U, false, XOP, true>), dim3((unsigned)grid), dim3(64 * waves), lds, s,
                           grp.packed[0], grp.y[0], X, grp.rows[0], (int)cols, nbk, nstrips, T | (G << 8) | (waves << 16), x_op, aux, grp, ops);
    else if (grp.count == 1)
        hipLaunchKernelGGL((q3h_gemv_kernel<NB, U, false, XOP>), dim3((unsigned)grid), dim3(64 * waves), lds, s,
                           grp.packed[0], grp.y[0], X, grp.rows[0], (int)cols, nbk, nstrips, T | (G << 8) | (waves << 16), x_op, aux, grp, ops);
    else
        hipLaunchKernelGGL((q3h_gemv_kernel<NB, U, true, XOP>), dim3((unsigned)grid), dim3(64 * waves), lds, s,
                           grp.packed[0], grp.y[0], X, grp.rows[0], (int)cols, nbk, nstrips, T | (G << 8) | (waves << 16), x_op, aux, grp, ops);
    return hipGetLastError();
}

// Q3H launch geometry: a workgroup of `waves` wavefronts covers waves*U*G rows and stages the activations of
// up to T strips (8.5 KiB of LDS per strip and batch column, at most 152 KiB).  Long rows and small problems
// get larger workgroups (the staging is paid once per workgroup); tall problems let a wavefront walk several
// row groups.
template <int NB, int XOP = -1, bool GATED = false>
static hipError_t q3h_launch(const GemvGroup &grp, int64_t cols, const uint16_t *X, hipStream_t s, const GemvOps &ops = GemvOps(),
                            int x_op = IFLOW_X_PLAIN, const uint16_t *aux = nullptr)
{
    const int nstrips = (int)((cols / 64 + 63) / 64);
    int64_t rows = 0;
    for (int i = 0; i < grp.count; ++i) rows += grp.rows[i];
    int waves = (nstrips >= 3 || rows <= 8192) ? 8 : 4;
    if (NB > 2 && waves > 8) waves = 8;                       // those instantiations are built for at most 512 threads
    int G = (int)(rows / (NB <= 2 ? 2 : 1) / 2560);           // tall problems: several row groups per wavefront, staging paid once
    if (G < 1) G = 1;
    if (G > 3) G = 3;
    // rows in flight per wavefront: two, or one where 32 activation registers per batch column leave no room
    if constexpr (NB <= 2) return q3h_launch_u<NB, 2, XOP, GATED>(grp, cols, X, waves, G, s, ops, x_op, aux);
    else return q3h_launch_u<NB, 1>(grp, cols, X, waves, G, s);
}

template <int F, int NB>
static hipError_t gemv_launch(const void *packed, int64_t rows, int64_t cols, const uint16_t *X, uint16_t *Y, hipStream_t s)
{
    typedef Fmt<F> T;
    if (T::kind == KIND_Q3H) {
        GemvGroup grp = {};
        grp.packed[0] = static_cast<const uint8_t *>(packed); grp.y[0] = Y; grp.rows[0] = (int)rows; grp.count = 1;
        return q3h_launch<NB>(grp, cols, X, s);
    }
    if (NB <= 2) {                                            // one or two vectors: rows owned by wavefronts (iflow_qgemv_rows.hip)
        const hipError_t e = launch_qgemv_rows(F, packed, rows, cols, X, NB, Y, s);
        if (e != hipErrorNotSupported) return e;              // (rows too long for its staging: the kernel below)
    }
    typedef Geo<T::kind> G;
    const int nbk = (int)(cols / T::block);
    const int nstrips = (int)((cols + 64 * G::WPL - 1) / (64 * G::WPL));
    const int nw = nstrips < 16 ? nstrips : 16;
    const int rpw = pick_rows_per_wg(rows, nw);
    const int64_t grid = (rows + rpw - 1) / rpw;
    const int64_t header_offset = rows * (cols / T::block) * (int64_t)T::code_bytes;
    // rows in flight per wavefront; the two-plane formats hold up to six words per row, and with three or four activation
    // vectors four rows no longer fit the 128 registers of a 1024-thread workgroup
    constexpr int U = (kind_has_planes(T::kind) && NB >= 3) ? 2 : 4;
    if (nw == 1)
        hipLaunchKernelGGL((qgemv_kernel<F, NB, U, false>), dim3((unsigned)grid), dim3(64), 0, s,
                           static_cast<const uint8_t *>(packed), X, Y, (int)rows, (int)cols, nbk, rpw, nstrips, header_offset);
    else
        hipLaunchKernelGGL((qgemv_kernel<F, NB, U, true>), dim3((unsigned)grid), dim3(64 * nw), 0, s,
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

hipError_t launch_qgemv_multi(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols,
                              const uint16_t *x, uint16_t *const *y, hipStream_t s)
{
    if (format == IFLOW_Q3H_B64) {                            // one launch for all matrices
        GemvGroup grp = {};
        for (int i = 0; i < count; ++i) {
            grp.packed[i] = static_cast<const uint8_t *>(packed[i]); grp.y[i] = y[i]; grp.rows[i] = (int)rows[i];
        }
        grp.count = count;
        return q3h_launch<1>(grp, cols, x, s);
    }
    if (count > 1) {                                          // the other formats: one launch too, unless the rows are too long to stage
        const hipError_t e = launch_qgemv_rows_multi(format, count, packed, rows, cols, x, y, s);
        if (e != hipErrorNotSupported) return e;
    }
    for (int i = 0; i < count; ++i) {                         // (one launch per matrix)
        hipError_t e = launch_qgemv(format, packed[i], rows[i], cols, x, 1, y[i], s);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

// The fused variant: `count` 3.5-bit matrices that share x, the operation on x and its second operand; a residual per
// matrix (null: none).
hipError_t launch_qgemv_fused(int count, const void *const *packed, const int64_t *rows, int64_t cols, const uint16_t *x,
                              int x_op, const uint16_t *aux, float eps, const uint16_t *const *residual, uint16_t *const *y,
                              hipStream_t s)
{
    if (count < 1 || count > IFLOW_MAX_GROUP) return hipErrorInvalidValue;
    GemvGroup grp = {};
    GemvOps ops = {};
    for (int i = 0; i < count; ++i) {
        grp.packed[i] = static_cast<const uint8_t *>(packed[i]); grp.y[i] = y[i]; grp.rows[i] = (int)rows[i];
        ops.residual[i] = residual ? residual[i] : nullptr;
    }
    grp.count = count;
    for (int i = 0; i < IFLOW_MAX_GROUP; ++i) ops.eps[i] = eps;
    switch (x_op) {
    case IFLOW_X_PLAIN:    return q3h_launch<1, IFLOW_X_PLAIN>(grp, cols, x, s, ops, x_op, aux);
    case IFLOW_X_RMS_GAIN: return q3h_launch<1, IFLOW_X_RMS_GAIN>(grp, cols, x, s, ops, x_op, aux);
    case IFLOW_X_SILU_MUL: return q3h_launch<1, IFLOW_X_SILU_MUL>(grp, cols, x, s, ops, x_op, aux);
    default: return hipErrorInvalidValue;
    }
}

// The gated pair: y_n = silu(scale (W_gate' v)_n) (scale (W_up' v)_n), v and scale as x_op (plain or rms gain) says.
hipError_t launch_qgemv_gated(int format, const void *packed_gate, const void *packed_up, int64_t rows, int64_t cols, const uint16_t *x,
                              int x_op, const uint16_t *aux, float eps, uint16_t *y, hipStream_t s)
{
    if (format != IFLOW_Q3H_B64) return launch_qgemv_rows_gated(format, packed_gate, packed_up, rows, cols, x, x_op, aux, eps, y, s);
    GemvGroup grp = {};
    GemvOps ops = {};
    grp.packed[0] = static_cast<const uint8_t *>(packed_gate); grp.packed[1] = static_cast<const uint8_t *>(packed_up);
    grp.y[0] = y; grp.y[1] = y; grp.rows[0] = (int)rows; grp.rows[1] = (int)rows; grp.count = 2;
    for (int i = 0; i < IFLOW_MAX_GROUP; ++i) ops.eps[i] = eps;
    switch (x_op) {
    case IFLOW_X_PLAIN:    return q3h_launch<1, IFLOW_X_PLAIN, true>(grp, cols, x, s, ops, x_op, aux);
    case IFLOW_X_RMS_GAIN: return q3h_launch<1, IFLOW_X_RMS_GAIN, true>(grp, cols, x, s, ops, x_op, aux);
    default: return hipErrorInvalidValue;
    }
}

hipError_t launch_qgemv(int format, const void *packed, int64_t rows, int64_t cols,
                        const uint16_t *x, int64_t batch, uint16_t *y, hipStream_t s)
{
    return for_format(format, [&](auto f) { return gemv_batch<decltype(f)::value>(packed, rows, cols, x, batch, y, s); });
}

}  // namespace iflow
