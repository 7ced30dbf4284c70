// Shared declarations of libiflow's translation units: format traits, small device helpers and the
// host-side launcher prototypes.  gfx950 (CDNA4) only: 64-wide wavefronts, DPP, packed fp16 math.
#pragma once

#include <mutex>
#include <type_traits>
#include <vector>

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/iflow.h"

namespace iflow {

typedef _Float16 half_t;
typedef _Float16 half2_t __attribute__((ext_vector_type(2)));
typedef unsigned short ushort2_t __attribute__((ext_vector_type(2)));

// ---- formats (Table 3 of the paper: bits, block size; Eq.1 / Eq.3: number of steps L) -------------
// The 6-, 5-, 3- and 2-bit formats store a level as bit planes (Planes: widths of the low and the high plane; the high
// plane's value counts 2^WA); the 4-bit format is the one-plane case with its own, older code path.
enum Kind { KIND_Q8 = 0, KIND_Q4 = 1, KIND_Q3H = 2, KIND_Q6 = 3, KIND_Q5 = 4, KIND_Q3 = 5, KIND_Q2 = 6 };

template <int KIND> struct Planes { static constexpr int WA = 0, WB = 0; };
template <> struct Planes<KIND_Q6> { static constexpr int WA = 4, WB = 2; };
template <> struct Planes<KIND_Q5> { static constexpr int WA = 4, WB = 1; };
template <> struct Planes<KIND_Q3> { static constexpr int WA = 2, WB = 1; };
template <> struct Planes<KIND_Q2> { static constexpr int WA = 2, WB = 0; };
constexpr bool kind_has_planes(int kind) { return kind >= KIND_Q6; }

template <int F> struct Fmt;
template <> struct Fmt<IFLOW_Q8_B32>  { static constexpr int kind = KIND_Q8,  block = 32, L = 255, code_bytes = 32; };
template <> struct Fmt<IFLOW_Q8_B64>  { static constexpr int kind = KIND_Q8,  block = 64, L = 255, code_bytes = 64; };
template <> struct Fmt<IFLOW_Q4_B32>  { static constexpr int kind = KIND_Q4,  block = 32, L = 15,  code_bytes = 16; };
template <> struct Fmt<IFLOW_Q4_B64>  { static constexpr int kind = KIND_Q4,  block = 64, L = 15,  code_bytes = 32; };
template <> struct Fmt<IFLOW_Q3H_B64> { static constexpr int kind = KIND_Q3H, block = 64, L = 10,  code_bytes = 28; };
template <> struct Fmt<IFLOW_Q6_B64>  { static constexpr int kind = KIND_Q6,  block = 64, L = 63,  code_bytes = 48; };
template <> struct Fmt<IFLOW_Q5_B64>  { static constexpr int kind = KIND_Q5,  block = 64, L = 31,  code_bytes = 40; };
template <> struct Fmt<IFLOW_Q3_B32>  { static constexpr int kind = KIND_Q3,  block = 32, L = 7,   code_bytes = 12; };
template <> struct Fmt<IFLOW_Q2_B32>  { static constexpr int kind = KIND_Q2,  block = 32, L = 3,   code_bytes = 8; };

// Host side: run fn(std::integral_constant<int, F>) for the format's compile-time tag; hipErrorInvalidValue for an unknown
// format.  `with_q3h`: whether the 3.5-bit format is among the formats fn is instantiated for.
template <bool with_q3h = true, typename Fn>
inline hipError_t for_format(int format, Fn fn)
{
    switch (format) {
    case IFLOW_Q8_B32: return fn(std::integral_constant<int, IFLOW_Q8_B32>{});
    case IFLOW_Q8_B64: return fn(std::integral_constant<int, IFLOW_Q8_B64>{});
    case IFLOW_Q4_B32: return fn(std::integral_constant<int, IFLOW_Q4_B32>{});
    case IFLOW_Q4_B64: return fn(std::integral_constant<int, IFLOW_Q4_B64>{});
    case IFLOW_Q3H_B64:
        if constexpr (with_q3h) return fn(std::integral_constant<int, IFLOW_Q3H_B64>{});
        else return hipErrorInvalidValue;
    case IFLOW_Q6_B64: return fn(std::integral_constant<int, IFLOW_Q6_B64>{});
    case IFLOW_Q5_B64: return fn(std::integral_constant<int, IFLOW_Q5_B64>{});
    case IFLOW_Q3_B32: return fn(std::integral_constant<int, IFLOW_Q3_B32>{});
    case IFLOW_Q2_B32: return fn(std::integral_constant<int, IFLOW_Q2_B32>{});
    default: return hipErrorInvalidValue;
    }
}

// the same traits for a format known only at run time (host side)
struct FormatInfo { int kind, block, L, code_bytes; };
inline bool format_info(int f, FormatInfo *fi)
{
    return for_format(f, [&](auto tag) {
        typedef Fmt<decltype(tag)::value> T;
        *fi = {T::kind, T::block, T::L, T::code_bytes};
        return hipSuccess;
    }) == hipSuccess;
}

// ---- bit casts ----------------------------------------------------------------------------------
__device__ __forceinline__ half2_t as_h2(uint32_t u) { return __builtin_bit_cast(half2_t, u); }
__device__ __forceinline__ uint32_t as_u32(half2_t h) { return __builtin_bit_cast(uint32_t, h); }
__device__ __forceinline__ half_t as_h(uint16_t u) { return __builtin_bit_cast(half_t, u); }
__device__ __forceinline__ uint16_t as_u16(half_t h) { return __builtin_bit_cast(uint16_t, h); }

// ---- wavefront reductions over DPP (no LDS traffic) ---------------------------------------------
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xF, true));
}
// sum within each row of 16 lanes; every lane of the row ends with the row's sum
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f32<0xB1, 0xF>(v);    // quad_perm [1,0,3,2]
    v += dpp_f32<0x4E, 0xF>(v);    // quad_perm [2,3,0,1]
    v += dpp_f32<0x141, 0xF>(v);   // row_half_mirror
    v += dpp_f32<0x140, 0xF>(v);   // row_mirror
    return v;
}
// sum over all 64 lanes; the result is valid in lane 63
__device__ __forceinline__ float wave_sum_to_lane63(float v)
{
    v = row16_sum(v);
    v += dpp_f32<0x142, 0xA>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_f32<0x143, 0xC>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}
__device__ __forceinline__ float wave_sum(float v)
{
    v = wave_sum_to_lane63(v);
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 63));
}

// ---- Q3H word decode ------------------------------------------------------------------------------
// A stored 32-bit word holds four 7-bit pair codes (Eq.4) at bits 0, 7, 16 and 23 and header bits at
// 14-15 and 30-31.  `hc` is two codes placed in the two halves of a register and OR-ed with 0x6400,
// i.e. the fp16 pair (1024 + c_lo, 1024 + c_hi).  Eq.5 in packed fp16 / u16 arithmetic:
//   (1024 + c) * K1 + K2 with K1 = 1489 * 2^-14 (fp16 nearest 1/11) and K2 = 931.5 lies within
//   0.02 of 1025 + (c - 5)/11, so the fma's rounding to the unit grid of [1024, 2048) yields exactly
//   1025 + floor(c / 11) for every c in 0..120;
//   (0x6401 + q1) * (-11) + (0x6400 + c) mod 2^16 = 0x17F5 + (c mod 11), the fp16 number
//   2^-20 * (2037 + q2).
// Both results are affine in the level, which is all a dot product against x needs.
#define IFLOW_Q3H_K1 ((half_t)0.09088134765625f)
#define IFLOW_Q3H_K2 ((half_t)931.5f)
#define IFLOW_Q3H_BIAS1 1025.0f
#define IFLOW_Q3H_BIAS2 2037.0f
#define IFLOW_Q3H_SCALE2 1048576.0f /* 2^20 */

__device__ __forceinline__ half2_t q3h_high_digit(uint32_t hc)
{
    const half2_t k1 = {IFLOW_Q3H_K1, IFLOW_Q3H_K1}, k2 = {IFLOW_Q3H_K2, IFLOW_Q3H_K2};
    return __builtin_elementwise_fma(as_h2(hc), k1, k2);                  // (1025 + q1) in each half
}
__device__ __forceinline__ half2_t q3h_low_digit(half2_t h1, uint32_t hc)
{
    const ushort2_t m11 = {0xFFF5, 0xFFF5};
    ushort2_t r = __builtin_bit_cast(ushort2_t, h1) * m11 + __builtin_bit_cast(ushort2_t, hc);
    return __builtin_bit_cast(half2_t, r);                                // 2^-20 * (2037 + q2) in each half
}

// ---- bit planes: fields to exact fp16 integers (the dense kernels; the vector kernels multiply the biased values) ------
// The 8 / W fields in the low byte of both halves of a plane word, as exact fp16 pairs (even weight, odd weight).
template <int W>
__device__ __forceinline__ void plane_byte_fields(uint32_t word, half2_t *v)
{
#pragma unroll
    for (int i = 0; i < 8 / W; ++i) {
        const uint32_t mask = (((1u << W) - 1u) << (W * i)) * 0x00010001u;
        const uint32_t magic = (uint32_t)((25 - W * i) << 10) * 0x00010001u;            // bit W i counts 1
        const half_t bias = (half_t)(float)(1024 >> (W * i));
        const half2_t b2 = {bias, bias};
        v[i] = as_h2((word & mask) | magic) - b2;
    }
}
// Sixteen consecutive weights' fields of a W-bit plane: W bytes of each half, `first` = the byte they start at.
template <int W>
__device__ __forceinline__ void plane_fields16(const uint32_t *words, int first, half2_t (&v)[8])
{
    if constexpr (W == 4) {
        plane_byte_fields<4>(words[0], &v[0]); plane_byte_fields<4>(words[0] >> 8, &v[2]);
        plane_byte_fields<4>(words[1], &v[4]); plane_byte_fields<4>(words[1] >> 8, &v[6]);
    } else if constexpr (W == 2) {
        plane_byte_fields<2>(words[0], &v[0]); plane_byte_fields<2>(words[0] >> 8, &v[4]);
    } else {
        plane_byte_fields<1>(words[0] >> (8 * first), &v[0]);
    }
}

// ---- once-per-device set-up on the host -----------------------------------------------------------
// A launcher's per-device preparation (raising a kernel's dynamic-LDS limit) runs once for each device it is called
// on, under a lock, so that several host threads may call the library; the device's compute-unit count comes back.
constexpr int IFLOW_MAX_DEVICES = 64;
struct PerDevice {
    std::mutex lock;
    int cus[IFLOW_MAX_DEVICES] = {};
};
template <typename Prepare>
inline hipError_t once_per_device(PerDevice &pd, int *cus, Prepare prepare)
{
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= IFLOW_MAX_DEVICES) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(pd.lock);
    if (pd.cus[dev] == 0) {
        int n = 0;
        e = hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) e = prepare();
        if (e != hipSuccess) return e;
        if (n < 1) return hipErrorInvalidDevice;
        pd.cus[dev] = n;
    }
    *cus = pd.cus[dev];
    return hipSuccess;
}

// the current device's compute-unit count (looked up once per device)
inline hipError_t device_compute_units(int *cus)
{
    static PerDevice pd;
    return once_per_device(pd, cus, [] { return hipSuccess; });
}

// ---- host-side launchers, one per translation unit ------------------------------------------------
hipError_t launch_quantize(int format, const float *w, int64_t rows, int64_t cols, void *packed, hipStream_t s);
hipError_t launch_dequant(int format, const void *packed, int64_t rows, int64_t cols, uint16_t *w16, hipStream_t s);
hipError_t launch_unpack_pair_codes(const void *packed, int64_t rows, int64_t cols, uint8_t *codes, hipStream_t s);
hipError_t launch_unpack(int format, const void *packed, int64_t rows, int64_t cols,
                         uint8_t *levels, uint16_t *scale16, uint16_t *offset16, hipStream_t s);
hipError_t launch_calibration_copy(const void *src, void *dst, size_t bytes, hipStream_t s);
hipError_t launch_calibration_read(const void *src, size_t bytes, void *sink, hipStream_t s);
hipError_t launch_qgemv_multi(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols,
                              const uint16_t *x, uint16_t *const *y, hipStream_t s);
hipError_t launch_qgemv_fused(int count, const void *const *packed, const int64_t *rows, int64_t cols, const uint16_t *x,
                              int x_op, const uint16_t *aux, float eps, const uint16_t *const *residual, uint16_t *const *y,
                              hipStream_t s);
hipError_t launch_qgemv_rows_fused(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols,
                                   const uint16_t *x, int x_op, const uint16_t *aux, float eps, const uint16_t *const *residual,
                                   uint16_t *const *y, hipStream_t s);
hipError_t launch_qgemv_gated(int format, const void *packed_gate, const void *packed_up, int64_t rows, int64_t cols, const uint16_t *x,
                              int x_op, const uint16_t *aux, float eps, uint16_t *y, hipStream_t s);
hipError_t launch_qgemv_rows_gated(int format, const void *packed_gate, const void *packed_up, int64_t rows, int64_t cols,
                                   const uint16_t *x, int x_op, const uint16_t *aux, float eps, uint16_t *y, hipStream_t s);
hipError_t launch_rope_append(uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, int n_heads, int n_kv_heads, int head_dim, int64_t position,
                              int64_t max_seq, double base, int pair_mode, uint16_t *k_cache, uint16_t *v_cache, hipStream_t s);
size_t attn_workspace_bytes(int n_heads);
hipError_t launch_attn_decode(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads, int n_kv_heads,
                              int head_dim, int64_t seq_len, int64_t max_seq, float scale, uint16_t *out, void *workspace, hipStream_t s);
hipError_t launch_attn_decode_static(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads, int n_kv_heads,
                                     int head_dim, int64_t seq_len, int64_t max_seq, float scale, uint16_t *out, hipStream_t s);
// ---- the chained launch: description of a chain (host arrays of the caller), plan builder, model, launcher ----
struct ChainSpec {
    int format;                        // iflow_format_t
    int nphases;
    const int *counts;                 // matrices per phase
    const int *first;                  // index of each phase's first matrix
    const int64_t *cols;               // per phase
    const uint16_t *const *x;          // per phase
    const int *x_src;                  // per phase: matrix whose output is the phase's input, or -1 for an input of the launch
    const void *const *packed;         // per matrix
    const int64_t *rows;
    uint16_t *const *y;
    // the modules around the products (all four may be null: bare products)
    const int *x_op;                   // per phase: iflow_x_op_t
    const uint16_t *const *aux;        // per phase: gains of IFLOW_X_RMS_GAIN
    const float *eps;                  // per phase
    const int *gated;                  // per phase: 1 = the phase's two matrices are the gate and up projections of a gated feed-forward
    const uint16_t *const *residual;   // per matrix, entries may be null
    const int *residual_src;           // per matrix: the matrix whose output is the residual, or -1 for an input of the launch
    // decode attention inside the launch (may be absent: nattn = 0, kind = null)
    const int *kind;                   // per phase: 0 products; 1 / 2: first / second half of attention attn_of[p] (kind 1 owns one
    const int *attn_of;                //   matrix entry, the attention's output [n_heads * 128] with packed = null; kind 2 none)
    int nattn;
    const struct ChainAttnSpec *attn;
};
struct ChainAttnSpec {
    const uint16_t *q, *k_new, *v_new; // inputs of the launch, or null with the matrix that produces them:
    int q_src, k_src, v_src;
    uint16_t *k_cache, *v_cache;
    int n_heads, n_kv_heads, max_seq, pairing;
    float scale, base;
};
size_t chain_workspace_bytes(int nmatrices, const int64_t *rows);
size_t chain_attn_workspace_bytes(int n_heads, int n_kv_heads, int grid);
size_t chain_plan_bytes(int nphases, int nmatrices, int nattn = 0);
bool chain_build_plan(const ChainSpec &c, int grid, std::vector<uint8_t> &out);
hipError_t chain_grid_for_device(int *grid);
hipError_t launch_chain(const void *plan, void *workspace, int grid, int lds_bytes, bool fused, int format, int position, hipStream_t s);
int chain_lds_bytes(int format, int max_strips);
bool chain_supports_format(int format);
int64_t chain_max_cols(int format);
int chain_strips(int format, int64_t cols);
hipError_t launch_qgemm_small_fused(int format, const void *packed, int64_t rows, int64_t cols, const uint16_t *X, int64_t batch, int x_op,
                                    const uint16_t *aux, float eps, const uint16_t *residual, uint16_t *Y, hipStream_t s);
hipError_t launch_qgemm_small(int format, const void *packed, int64_t rows, int64_t cols,
                              const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s);
hipError_t launch_qgemm_mfma(int format, const void *packed, int64_t rows, int64_t cols,
                             const uint16_t *X, int64_t batch, uint16_t *Y, hipStream_t s);
hipError_t launch_qgemv_rows(int format, const void *packed, int64_t rows, int64_t cols, const uint16_t *x, int batch, uint16_t *y,
                             hipStream_t s);
hipError_t launch_qgemv_rows_multi(int format, int count, const void *const *packed, const int64_t *rows, int64_t cols, const uint16_t *x,
                                   uint16_t *const *y, hipStream_t s);
hipError_t launch_qgemv(int format, const void *packed, int64_t rows, int64_t cols,
                        const uint16_t *x, int64_t batch, uint16_t *y, hipStream_t s);

}  // namespace iflow
