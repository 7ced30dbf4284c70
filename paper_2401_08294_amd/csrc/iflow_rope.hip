// Rotary position embedding for one decode step and the step's append to the key/value cache (Section 2 of the paper lists
// "rope" as the position embedding module of the LLaMA-family models; the embedding itself is the published one: pair i of
// a head's components at position p turns by the angle p * base^(-2i/d)).
//
// One launch between the q/k/v projections and the attention: the queries are rotated in place, the step's keys are
// rotated and written to row `position` of the key cache, the step's values are copied to the same row of the value
// cache.  One workgroup per head (query heads first, then key/value heads), one pair of components per thread.  The work
// is a few kilobytes; what matters is that the angle is right at large positions: p * base^(-2i/d) reaches 10^6 radians
// for the first pairs, where fp32 holds it to 0.06 radians only - so the angle, its sine and cosine and the rotation are
// computed in fp64 (one per pair and head) and rounded to fp16 once.
#include "iflow_common.h"

namespace iflow {

constexpr int ROPE_MAX_D = 256;

__global__ __launch_bounds__(ROPE_MAX_D / 2) void rope_append_kernel(uint16_t *__restrict__ q, const uint16_t *__restrict__ k_new,
                                                                      const uint16_t *__restrict__ v_new, int n_heads, int head_dim, int64_t position,
                                                                  int64_t max_seq, double log2_base, int pair_mode,
                                                                  uint16_t *__restrict__ k_cache, uint16_t *__restrict__ v_cache)
{
    const int h = blockIdx.x, i = threadIdx.x;
    const double inv_freq = exp2(-(2.0 * i / head_dim) * log2_base);        // base^(-2i/d)
    const double angle = (double)position * inv_freq;
    double sn, cs;
    sincos(angle, &sn, &cs);
    const int ia = pair_mode == IFLOW_ROPE_HALVES ? i : 2 * i;            // the pair's two components
    const int ib = pair_mode == IFLOW_ROPE_HALVES ? i + head_dim / 2 : 2 * i + 1;
    const uint16_t *src;
    uint16_t *dst;
    if (h < n_heads) {                                                     // a query head: in place
        src = q + (int64_t)h * head_dim;
        dst = q + (int64_t)h * head_dim;
    } else {                                                               // a key/value head: into row `position` of the caches
        const int j = h - n_heads;
        src = k_new + (int64_t)j * head_dim;
        dst = k_cache + ((int64_t)j * max_seq + position) * head_dim;
        const uint16_t *vs = v_new + (int64_t)j * head_dim;
        uint16_t *vd = v_cache + ((int64_t)j * max_seq + position) * head_dim;
        vd[ia] = vs[ia];
        vd[ib] = vs[ib];
    }
    const double a = (double)(float)as_h(src[ia]), b = (double)(float)as_h(src[ib]);
    const double ra = a * cs - b * sn, rb = a * sn + b * cs;
    dst[ia] = as_u16((half_t)ra);                                          // fp64 -> fp16, one rounding
    dst[ib] = as_u16((half_t)rb);
}

hipError_t launch_rope_append(uint16_t *q, const uint16_t *k_new, const uint16_t *v_new, int n_heads, int n_kv_heads, int head_dim, int64_t position,
                              int64_t max_seq, double base, int pair_mode, uint16_t *k_cache, uint16_t *v_cache, hipStream_t s)
{
    if (head_dim < 2 || head_dim > ROPE_MAX_D || (head_dim & 1)) return hipErrorInvalidValue;
    hipLaunchKernelGGL(rope_append_kernel, dim3((unsigned)(n_heads + n_kv_heads)), dim3((unsigned)(head_dim / 2)), 0, s, q, k_new, v_new, n_heads,
                       head_dim, position, max_seq, log2(base), pair_mode, k_cache, v_cache);
    return hipGetLastError();
}

}  // namespace iflow
