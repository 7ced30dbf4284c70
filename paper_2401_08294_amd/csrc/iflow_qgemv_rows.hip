// One activation vector against a matrix in any block format but the 3.5-bit one (which has its own kernel): the
// skeleton of that kernel - activations staged once per workgroup, rows owned by wavefronts - for the 8-, 6-, 5-, 4-,
// 3- and 2-bit formats of Table 3 (Eq.1 levels, Eq.2 folded into the product).
//
// A "strip" is what one wavefront covers with one load per lane: 64 lanes x WPL weights (2048 columns, 1024 for 8-bit).
// The workgroup's threads convert the activations of every strip once (fp16 pairs in the order the decode wants, plus
// the two sums per lane that undo the decode's bias) and park them in LDS; after one barrier a wavefront owns U
// consecutive rows at a time and walks along them strip by strip: the next strip's loads are requested, the strip's
// activations come back from LDS with a few 16-byte reads, and each row's lane-partial sum is carried in a register until
// the row ends; then one DPP reduction per group of U rows.  No wavefront waits for another after the barrier, a row is
// reduced once, and nothing is combined through LDS.  (The older kernel gives every strip of a row to a different
// wavefront, each converting its own activations for a dozen rows and meeting the others in LDS at the end.)
//
// All loads are unconditional and in bounds: rows past the end repeat the last row (not stored), lanes past the end of
// a ragged last strip repeat the strip's first lane against activations staged as zeros (so they add nothing), and the
// request after the last step repeats the last step.  With a load under a branch the compiler would wait for every
// outstanding load at the next use instead of only for the set it needs.
#include "iflow_lane.h"

namespace iflow {

template <int KIND> struct RowsGeo {
    static constexpr int XQ = Geo<KIND>::XD / 4;                       // 16-byte quads of activation pairs per lane and strip
    static constexpr int SLOT = XQ * 64 * 16 + 64 * 8;                 // staged strip: quads [q][lane], then (bias_sum, x_sum)[lane]
};

constexpr int ROWS_LDS_LIMIT = 144 * 1024;

// Up to eight matrices that share the activation vector(s) and the column count in one launch (the q/k/v or the gate/up
// projections of a decoder layer): workgroup ranges are dealt to the matrices in order.
constexpr int ROWS_MAX_GROUP = 8;
struct RowsGroup {
    const uint8_t *packed[ROWS_MAX_GROUP];
    uint16_t *y[ROWS_MAX_GROUP];
    int rows[ROWS_MAX_GROUP];
    int wg_end[ROWS_MAX_GROUP];                                // one past the last workgroup of matrix i
    int count;
};

// What the fused variant (XOP >= 0, an iflow_x_op_t; one vector only) does besides the product - the modules Section 2
// lists around a decoder layer's linear layers, folded into the launch:
//   IFLOW_X_RMS_GAIN   the staged activations are fp16(x_k g_k) and every row sum is multiplied by
//                      1 / sqrt(mean x^2 + eps): rms normalization with its scalar moved behind the product;
//   IFLOW_X_SILU_MUL   the staged activations are fp16(silu(x_k) aux_k): the input of a gated feed-forward's last layer;
//   residual           out_n = fp16(row sum x scale + residual_n), per matrix, or none.
//   GATED              (one pair of matrices, XOP plain or rms gain) the wavefront's two rows in flight are row n of a
//                      "gate" and row n of an "up" matrix (grp.packed[0], [1]); out_n = fp16(silu(gate sum x scale)
//                      (up sum x scale)), the gated feed-forward's hidden vector without storing its two factors.
// (The same arithmetic, in the same order, as the 3.5-bit kernel's fused variant.)
struct RowsOps {
    const uint16_t *residual[ROWS_MAX_GROUP];
    const uint16_t *aux;
    float eps;
};

template <int F, int U, int NB, bool MULTI, int XOP, bool GATED = false>
__device__ __forceinline__ void gemv_rows_body(const uint8_t *__restrict__ packed0, const uint16_t *__restrict__ X,
                                               uint16_t *__restrict__ y0, int rows0, int cols, int nbk, int nstrips, int groups,
                                               const RowsGroup &grp, const RowsOps &ops)
{
    typedef Fmt<F> T;
    constexpr bool OPS = XOP >= 0;
    static_assert(!OPS || NB == 1, "the fused variant is built for one activation vector");
    static_assert(!GATED || (OPS && !MULTI && U == 2), "the gated variant: one pair of matrices, two rows in flight");
    constexpr int RPG = GATED ? 1 : U;                         // output rows per group
    int mi = 0;                                                // which matrix this workgroup belongs to
    if (MULTI) {
#pragma unroll
        for (int i = 0; i + 1 < ROWS_MAX_GROUP; ++i)
            if (i + 1 < grp.count && (int)blockIdx.x >= grp.wg_end[i]) mi = i + 1;
    }
    const int wg = MULTI ? blockIdx.x - (mi ? grp.wg_end[mi - 1] : 0) : blockIdx.x;
    const uint8_t *__restrict__ packed = MULTI ? grp.packed[mi] : packed0;
    const uint8_t *__restrict__ packed_up = GATED ? grp.packed[1] : nullptr;
    uint16_t *__restrict__ Y = MULTI ? grp.y[mi] : y0;
    const int rows = MULTI ? grp.rows[mi] : rows0;
    const int64_t header_offset = (int64_t)rows * nbk * T::code_bytes;
    constexpr int KIND = T::kind;
    typedef Geo<KIND> G;
    typedef RowsGeo<KIND> RG;
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    extern __shared__ __align__(16) uint8_t lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), waves = blockDim.x >> 6;

    // ---- stage the activations: item (strip, lane) -> converted registers -> LDS ----------------------------------
    float ssq = 0.f;                                          // (rms) this thread's share of sum x^2
    for (int item = tid; item < NB * nstrips * 64; item += blockDim.x) {      // slot (strip t, vector b) = t * NB + b
        const int tb = item >> 6, l = item & 63;
        const int t = tb / NB, b = tb - t * NB;
        const int k0 = (t * 64 + l) * G::WPL;
        XRegs<KIND> xr;
        if (k0 < cols) {
            if constexpr (XOP > IFLOW_X_PLAIN) {
                uint32_t n[G::XD], av[G::XD];
#pragma unroll
                for (int j = 0; j < G::XD / 4; ++j) {
                    const uint4 q = reinterpret_cast<const uint4 *>(X + k0)[j], a = reinterpret_cast<const uint4 *>(ops.aux + k0)[j];
                    n[4 * j] = q.x; n[4 * j + 1] = q.y; n[4 * j + 2] = q.z; n[4 * j + 3] = q.w;
                    av[4 * j] = a.x; av[4 * j + 1] = a.y; av[4 * j + 2] = a.z; av[4 * j + 3] = a.w;
                }
#pragma unroll
                for (int j = 0; j < G::XD; ++j) {
                    if constexpr (XOP == IFLOW_X_RMS_GAIN) {  // x_k g_k: exact product, one rounding to fp16
                        ssq = dot2(as_h2(n[j]), as_h2(n[j]), ssq);
                        n[j] = as_u32(as_h2(n[j]) * as_h2(av[j]));
                    } else {                                  // silu(x_k) aux_k in fp32, one rounding to fp16
                        const half2_t xa = as_h2(n[j]), xb = as_h2(av[j]);
                        const float g0 = (float)xa.x, g1 = (float)xa.y;
                        // (hardware reciprocal: 1 ulp of fp32, far below the fp16 rounding that follows)
                        const float v0 = g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * (float)xb.x;
                        const float v1 = g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * (float)xb.y;
                        const half2_t r = {(half_t)v0, (half_t)v1};
                        n[j] = as_u32(r);
                    }
                }
                arrange_x<KIND>(xr, n);
            } else {
                load_x<KIND>(xr, X + (int64_t)b * cols, k0);
            }
        } else {                                              // past the end of the last strip: contributes nothing
#pragma unroll
            for (int j = 0; j < G::XD; ++j) xr.v[j] = as_h2(0u);
            xr.bias_sum = 0.f; xr.x_sum = 0.f;
        }
        uint8_t *slot = lds + (size_t)tb * RG::SLOT;
#pragma unroll
        for (int q = 0; q < RG::XQ; ++q) {
            const u32x4 v = {as_u32(xr.v[4 * q]), as_u32(xr.v[4 * q + 1]), as_u32(xr.v[4 * q + 2]), as_u32(xr.v[4 * q + 3])};
            reinterpret_cast<u32x4 *>(slot)[q * 64 + l] = v;
        }
        reinterpret_cast<float2 *>(slot + RG::XQ * 64 * 16)[l] = make_float2(xr.bias_sum, xr.x_sum);
    }

    // ---- where a lane's codes and header sit inside a row, strip 0; a strip further on adds constants ------------
    // (lanes past the end of the last strip fall back to the strip's first lane, see above)
    int64_t row_stride, row_stride_b = 0, plane_b = 0;
    int lane_bytes, lane_bytes_b = 0;                         // bytes per lane and row in the (low) plane, in the high plane
    if constexpr (kind_has_planes(KIND)) {
        constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
        row_stride = (int64_t)cols * WA / 8; lane_bytes = G::WPL * WA / 8;
        row_stride_b = (int64_t)cols * WB / 8; lane_bytes_b = G::WPL * WB / 8;
        plane_b = (int64_t)rows * cols * WA / 8;
    } else if constexpr (KIND == KIND_Q4) {
        row_stride = cols / 2; lane_bytes = 16;
    } else {
        row_stride = cols; lane_bytes = 16;
    }
    const int hdr_per_strip = 64 * G::WPL / T::block;         // headers per strip: a lane's weights lie in one block

    auto load_step = [&](WRegs<KIND>(&w)[U], int r0, int t) {
        const bool in = (t * 64 + lane) * G::WPL < cols;
        const int la = in ? lane : 0;
        const int64_t code_off = ((int64_t)t * 64 + la) * lane_bytes;
        const int64_t code_off_b = plane_b + ((int64_t)t * 64 + la) * lane_bytes_b;
        const int64_t hdr_off = header_offset + ((int64_t)t * hdr_per_strip + la * G::WPL / T::block) * 4;
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const int64_t r = min(GATED ? r0 : r0 + u, rows - 1);
            const uint8_t *mat = (GATED && u == 1) ? packed_up : packed;
            const uint8_t *p = mat + r * row_stride + code_off;
            if constexpr (kind_has_planes(KIND)) {
                constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
                if constexpr (WA == 4) {
                    const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
                    w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
                } else {
                    const uint2 a = *reinterpret_cast<const uint2 *>(p);
                    w[u].d[0] = a.x; w[u].d[1] = a.y;
                }
                const uint8_t *pb = mat + r * row_stride_b + code_off_b;
                if constexpr (WB == 2) {
                    const uint2 c = *reinterpret_cast<const uint2 *>(pb);
                    w[u].d[WA] = c.x; w[u].d[WA + 1] = c.y;
                } else if constexpr (WB == 1) {
                    w[u].d[WA] = *reinterpret_cast<const uint32_t *>(pb);
                }
            } else {
                const u32x4 a = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
                w[u].d[0] = a.x; w[u].d[1] = a.y; w[u].d[2] = a.z; w[u].d[3] = a.w;
            }
            w[u].hdr = *reinterpret_cast<const uint32_t *>(mat + hdr_off + r * (int64_t)nbk * 4);
        }
    };

    // ---- the walk: steps (group, strip) of this wavefront, one set of weights ahead ---------------------------------
    const int rbase = (wg * waves + wave) * groups * RPG;
    const int nsteps = groups * nstrips;
    auto step_row = [&](int k, int &r0, int &t) {
        const int kk = min(k, nsteps - 1);
        const int g = kk / nstrips;
        t = kk - g * nstrips;
        r0 = rbase + g * RPG;
    };

    WRegs<KIND> wa[U], wb[U];
    float acc[NB][U];
#pragma unroll
    for (int b = 0; b < NB; ++b)
#pragma unroll
        for (int u = 0; u < U; ++u) acc[b][u] = 0.f;
    {
        int r0, t;
        step_row(0, r0, t);
        load_step(wa, r0, t);                                 // the first weights are on their way before the barrier
    }
    // fused variant: lane l holds the residual of the wavefront's l-th row (in bounds whatever the row; read before any
    // of these rows is stored, so the residual may be the output vector itself)
    float res = 0.f, out_scale = 1.0f;
    if constexpr (OPS) {
        const uint16_t *rp = ops.residual[mi];               // (no residual: x[0], dropped - the load is under no branch)
        const uint16_t raw = *(rp != nullptr ? rp + min(rbase + min(lane, groups * U - 1), rows - 1) : X);
        res = rp != nullptr ? (float)as_h(raw) : 0.f;
    }
    float *ssq_part = reinterpret_cast<float *>(lds + (size_t)NB * nstrips * RG::SLOT);     // sixteen floats behind the strips
    if constexpr (XOP == IFLOW_X_RMS_GAIN) {
        const float wsum = wave_sum_to_lane63(ssq);
        if (lane == 63) ssq_part[wave] = wsum;
    }
    __syncthreads();
    if constexpr (XOP == IFLOW_X_RMS_GAIN) {
        const float mine = lane < waves ? ssq_part[lane] : 0.f;
        const float total = wave_sum(mine);
        out_scale = 1.0f / __builtin_sqrtf(total / (float)cols + ops.eps);
    }

    auto compute_step = [&](const WRegs<KIND>(&w)[U], int k) {
        int r0, t;
        step_row(k, r0, t);
        XRegs<KIND> xr[NB];
#pragma unroll
        for (int b = 0; b < NB; ++b) {
            const uint8_t *slot = lds + (size_t)(t * NB + b) * RG::SLOT;
#pragma unroll
            for (int q = 0; q < RG::XQ; ++q) {
                const u32x4 v = reinterpret_cast<const u32x4 *>(slot)[q * 64 + lane];
                xr[b].v[4 * q] = as_h2(v.x); xr[b].v[4 * q + 1] = as_h2(v.y); xr[b].v[4 * q + 2] = as_h2(v.z); xr[b].v[4 * q + 3] = as_h2(v.w);
            }
            const float2 sums = reinterpret_cast<const float2 *>(slot + RG::XQ * 64 * 16)[lane];
            xr[b].bias_sum = sums.x; xr[b].x_sum = sums.y;
        }
#pragma unroll
        for (int u = 0; u < U; ++u) {
            float a[NB];
            lane_dot<KIND, NB>(w[u], xr, a);
            const half2_t so = as_h2(w[u].hdr);
#pragma unroll
            for (int b = 0; b < NB; ++b)
                acc[b][u] += __builtin_fmaf((float)so.x, a[b] - xr[b].bias_sum, (float)so.y * xr[b].x_sum);
        }
        if (GATED && t == nstrips - 1) {                      // even lanes hold the gate's sum, odd lanes the up projection's
            const float mine = reduce_rows<U>(acc[0], lane) * out_scale;
            const float other = dpp_f32<0xB1, 0xF>(mine);     // (lanes ^ 1)
            const float hv = mine * __builtin_amdgcn_rcpf(1.0f + __expf(-mine)) * other;
            if (lane == 0 && r0 < rows) Y[r0] = as_u16((half_t)hv);
#pragma unroll
            for (int u = 0; u < U; ++u) acc[0][u] = 0.f;
        } else if (t == nstrips - 1) {                        // the rows end here: reduce, store, start over
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                float r = reduce_rows<U>(acc[b], lane);
                if constexpr (OPS) {                          // lane u < U holds row r0 + u, the wavefront's row (r0 - rbase) + u
                    const float rr = __shfl(res, (r0 - rbase) + (lane & (U - 1)));
                    r = __builtin_fmaf(r, out_scale, rr);
                }
                if (lane < U && r0 + lane < rows) Y[(int64_t)b * rows + r0 + lane] = as_u16((half_t)r);
#pragma unroll
                for (int u = 0; u < U; ++u) acc[b][u] = 0.f;
            }
        }
    };

    if (rbase >= rows) return;                                // (after the barrier; a whole wavefront at a time)
    for (int k = 0; k < nsteps; k += 2) {
        int r0, t;
        step_row(k + 1, r0, t);
        load_step(wb, r0, t);
        compute_step(wa, k);
        step_row(k + 2, r0, t);
        load_step(wa, r0, t);
        if (k + 1 < nsteps) compute_step(wb, k + 1);
    }
}

template <int F, int U, int NB, bool MULTI>
__global__ __launch_bounds__(512) void gemv_rows_kernel(const uint8_t *__restrict__ packed0, const uint16_t *__restrict__ X,
                                                        uint16_t *__restrict__ y0, int rows0, int cols, int nbk, int nstrips,
                                                        int groups /* of U rows per wavefront */, const RowsGroup grp)
{
    gemv_rows_body<F, U, NB, MULTI, -1>(packed0, X, y0, rows0, cols, nbk, nstrips, groups, grp, RowsOps{});
}

template <int F, int U, bool MULTI, int XOP, bool GATED = false>
__global__ __launch_bounds__(512) void gemv_rows_fused_kernel(const uint8_t *__restrict__ packed0, const uint16_t *__restrict__ X,
                                                              uint16_t *__restrict__ y0, int rows0, int cols, int nbk, int nstrips,
                                                              int groups, const RowsGroup grp, const RowsOps ops)
{
    gemv_rows_body<F, U, 1, MULTI, XOP, GATED>(packed0, X, y0, rows0, cols, nbk, nstrips, groups, grp, ops);
}

template <int F, int U, int NB, bool MULTI, int XOP = -1, bool GATED = false>
static hipError_t rows_launch(RowsGroup grp, int64_t cols, const uint16_t *x, hipStream_t s, const RowsOps &ops = RowsOps{})
{
    typedef Fmt<F> T;
    typedef Geo<T::kind> G;
    typedef RowsGeo<T::kind> RG;
    const int nbk = (int)(cols / T::block);
    const int nstrips = (int)((cols + 64 * G::WPL - 1) / (64 * G::WPL));
    const size_t lds = (size_t)NB * nstrips * RG::SLOT + (XOP >= 0 ? 64 : 0);
    if (lds > (size_t)ROWS_LDS_LIMIT) return hipErrorNotSupported;
    static PerDevice pd;                                      // raise the dynamic-LDS cap once per instantiation and device
    int cus = 0;
    hipError_t e = once_per_device(pd, &cus, [] {
        const void *fn;
        if constexpr (XOP >= 0) fn = reinterpret_cast<const void *>(gemv_rows_fused_kernel<F, U, MULTI, XOP, GATED>);
        else fn = reinterpret_cast<const void *>(gemv_rows_kernel<F, U, NB, MULTI>);
        return hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, ROWS_LDS_LIMIT);
    });
    if (e != hipSuccess) return e;
    int64_t rows = 0;
    for (int i = 0; i < grp.count; ++i) rows += grp.rows[i];
    // wavefronts per workgroup and groups of U rows per wavefront: enough workgroups to fill the part a few times over,
    // but not so many that the staging (paid once per workgroup) outweighs the rows it serves
    // (measured over 4096 x 4096, 11008 x 4096 and 4096 x 11008 in four formats: every choice of 2-8 wavefronts, 1-2 groups
    // and 2 or 4 rows per group lands within 5 % of this one)
    const int waves = nstrips >= 3 ? 8 : 4;
    int groups = (int)(rows / ((int64_t)cus * 2 * waves * U));
    if (groups < 1) groups = 1;
    if (groups > 4) groups = 4;
    // ... unless that leaves the compute units unevenly loaded (28672 rows in groups of three: 598 workgroups for 256 units):
    // price each choice as (workgroups per unit, rounded up) x (groups + the staging's share) and move when it saves 10 %
    {
        const int rpg = GATED ? 1 : U;
        auto price = [&](int g) {
            int64_t n = 0;
            for (int i = 0; i < (GATED ? 1 : grp.count); ++i) n += (grp.rows[i] + (int64_t)waves * g * rpg - 1) / ((int64_t)waves * g * rpg);
            return (double)((n + cus - 1) / cus) * (g + 0.15);
        };
        int best = groups;
        for (int g = 1; g <= 4; ++g)
            if (price(g) < price(best)) best = g;
        if (price(best) < 0.9 * price(groups)) groups = best;
    }
    const int64_t rows_per_wg = (int64_t)waves * groups * (GATED ? 1 : U);
    int64_t grid = 0;
    for (int i = 0; i < (GATED ? 1 : grp.count); ++i) {       // (gated: the pair's two matrices are one set of output rows)
        grid += (grp.rows[i] + rows_per_wg - 1) / rows_per_wg;
        grp.wg_end[i] = (int)grid;
    }
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    if constexpr (XOP >= 0)
        hipLaunchKernelGGL((gemv_rows_fused_kernel<F, U, MULTI, XOP, GATED>), dim3((unsigned)grid), dim3(64 * waves), lds, s, grp.packed[0], x,
                           grp.y[0], grp.rows[0], (int)cols, nbk, nstrips, groups, grp, ops);
    else
        hipLaunchKernelGGL((gemv_rows_kernel<F, U, NB, MULTI>), dim3((unsigned)grid), dim3(64 * waves), lds, s, grp.packed[0], x, grp.y[0],
                           grp.rows[0], (int)cols, nbk, nstrips, groups, grp);
    return hipGetLastError();
}

template <int F>
static hipError_t rows_batch(const RowsGroup &grp, int64_t cols, const uint16_t *x, int batch, hipStream_t s)
{
    if (grp.count > 1) return rows_launch<F, 2, 1, true>(grp, cols, x, s);            // (several matrices: one vector only)
    return batch == 1 ? rows_launch<F, 2, 1, false>(grp, cols, x, s) : rows_launch<F, 2, 2, false>(grp, cols, x, s);
}

static hipError_t rows_dispatch(int format, const RowsGroup &grp, int64_t cols, const uint16_t *x, int batch, hipStream_t s)
{
    return for_format<false>(format, [&](auto f) { return rows_batch<decltype(f)::value>(grp, cols, x, batch, s); });
}

// One or two activation vectors (x: [batch][cols], y: [batch][rows]), any format but IFLOW_Q3H_B64.  hipErrorNotSupported:
// the rows are too long for the staged activations to fit in LDS (beyond about 60000 columns for one vector, half that
// for two) - the caller then takes the older kernel.
hipError_t launch_qgemv_rows(int format, const void *packed, int64_t rows, int64_t cols, const uint16_t *x, int batch, uint16_t *y,
                             hipStream_t s)
{
    if (batch < 1 || batch > 2) return hipErrorInvalidValue;
    RowsGroup grp = {};
    grp.packed[0] = static_cast<const uint8_t *>(packed); grp.y[0] = y; grp.rows[0] = (int)rows; grp.count = 1;
    return rows_dispatch(format, grp, cols, x, batch, s);
}

// `count` (1-8) matrices of one format that share x (one vector) and the column count, in one launch; same results as
// separate launches, bit for bit (a row's arithmetic does not depend on which workgroup runs it).
hipError_t launch_qgemv_rows_multi(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols, const uint16_t *x,
                                   uint16_t *const *y, hipStream_t s)
{
    if (count < 1 || count > ROWS_MAX_GROUP) return hipErrorInvalidValue;
    RowsGroup grp = {};
    for (int i = 0; i < count; ++i) {
        grp.packed[i] = static_cast<const uint8_t *>(packed[i]); grp.y[i] = y[i]; grp.rows[i] = (int)rows[i];
    }
    grp.count = count;
    return rows_dispatch(format, grp, cols, x, 1, s);
}

template <int F, int XOP>
static hipError_t rows_fused_count(const RowsGroup &grp, int64_t cols, const uint16_t *x, const RowsOps &ops, hipStream_t s)
{
    return grp.count > 1 ? rows_launch<F, 2, 1, true, XOP>(grp, cols, x, s, ops) : rows_launch<F, 2, 1, false, XOP>(grp, cols, x, s, ops);
}

// The fused variant for any format but IFLOW_Q3H_B64: `count` (1-8) matrices that share x (one vector), the operation on
// x and its second operand; a residual per matrix (null: none).  hipErrorNotSupported: rows too long for LDS (see above).
hipError_t launch_qgemv_rows_fused(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols,
                                   const uint16_t *x, int x_op, const uint16_t *aux, float eps, const uint16_t *const *residual,
                                   uint16_t *const *y, hipStream_t s)
{
    if (count < 1 || count > ROWS_MAX_GROUP) return hipErrorInvalidValue;
    if (x_op > IFLOW_X_PLAIN && aux == nullptr) return hipErrorInvalidValue;
    RowsGroup grp = {};
    RowsOps ops = {};
    for (int i = 0; i < count; ++i) {
        grp.packed[i] = static_cast<const uint8_t *>(packed[i]); grp.y[i] = y[i]; grp.rows[i] = (int)rows[i];
        ops.residual[i] = residual ? residual[i] : nullptr;
    }
    grp.count = count;
    ops.aux = aux;
    ops.eps = eps;
    return for_format<false>(format, [&](auto f) {
        constexpr int F = decltype(f)::value;
        switch (x_op) {
        case IFLOW_X_PLAIN:    return rows_fused_count<F, IFLOW_X_PLAIN>(grp, cols, x, ops, s);
        case IFLOW_X_RMS_GAIN: return rows_fused_count<F, IFLOW_X_RMS_GAIN>(grp, cols, x, ops, s);
        case IFLOW_X_SILU_MUL: return rows_fused_count<F, IFLOW_X_SILU_MUL>(grp, cols, x, ops, s);
        default: return hipErrorInvalidValue;
        }
    });
}

// The gated pair for any format but IFLOW_Q3H_B64: y_n = silu(scale (W_gate' v)_n) (scale (W_up' v)_n).
hipError_t launch_qgemv_rows_gated(int format, const void *packed_gate, const void *packed_up, int64_t rows, int64_t cols,
                                   const uint16_t *x, int x_op, const uint16_t *aux, float eps, uint16_t *y, hipStream_t s)
{
    if (x_op == IFLOW_X_RMS_GAIN && aux == nullptr) return hipErrorInvalidValue;
    RowsGroup grp = {};
    RowsOps ops = {};
    grp.packed[0] = static_cast<const uint8_t *>(packed_gate); grp.packed[1] = static_cast<const uint8_t *>(packed_up);
    grp.y[0] = y; grp.y[1] = y; grp.rows[0] = (int)rows; grp.rows[1] = (int)rows; grp.count = 2;
    ops.aux = aux;
    ops.eps = eps;
    return for_format<false>(format, [&](auto f) {
        constexpr int F = decltype(f)::value;
        switch (x_op) {
        case IFLOW_X_PLAIN:    return rows_launch<F, 2, 1, false, IFLOW_X_PLAIN, true>(grp, cols, x, s, ops);
        case IFLOW_X_RMS_GAIN: return rows_launch<F, 2, 1, false, IFLOW_X_RMS_GAIN, true>(grp, cols, x, s, ops);
        default: return hipErrorInvalidValue;
        }
    });
}

}  // namespace iflow
