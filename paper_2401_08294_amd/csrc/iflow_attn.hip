// One decode step of grouped-query attention over an fp16 key/value cache (arXiv 2401.08294, section "Grouped-query
// attention": head_i = Attention(Q_i, K^j, V^j) with j the group of query head i; Attention = scaled dot-product
// attention; with as many groups as heads it is multi-head attention).
//
// Next to the weight stream this is the other part of a decode step that is bound by memory: every cached key and
// value is read once per step and used for a handful of multiply-adds.  So the kernel is laid out like the GEMV: long
// contiguous 16-byte-per-lane reads, everything else in registers.
//   - The cache is [kv head][position][128] fp16, so the positions of a head are one contiguous stream.  A workgroup
//     (four wavefronts) takes one kv head and one contiguous range of positions (a "split"); the grid is
//     kv heads x splits, a few workgroups per compute unit.
//   - A wavefront walks its range in blocks of sixteen positions.  Sixteen lanes share a position (8 of the 128
//     components each), so one load instruction covers four consecutive positions = 1 KB; the four lane groups of a
//     wavefront keep separate running softmax states (maximum, sum, 128-component weighted value sum) for their
//     positions.  The block after the current one is already requested while a block is processed.
//   - All query heads of a group are served from the same loaded keys and values: one or two heads by the kernel
//     described here, on the vector units; four or eight by attn_decode_mfma_kernel further down, on the matrix cores.
//   - Softmax is computed the streaming way: per block one rescale of the running sums to the new maximum, then
//     exp2 of the (pre-scaled) score differences.  fp32 throughout; the output is rounded to fp16 once.
//   - A workgroup merges its sixteen states through LDS and writes one state per (head, split) to the caller's
//     workspace; a second, small kernel (one workgroup per query head) merges the splits and writes the output.  Two
//     launches rather than "the last workgroup to finish merges": device-wide release/acquire fences write back and
//     invalidate whole L2 caches on this part (several microseconds per workgroup, measured), and one workgroup per
//     kv head merging all its heads' splits one after the other is a long serial tail; the second launch costs about
//     two microseconds and merges all heads at once.  With a single split the first kernel writes the output itself.
#include "iflow_common.h"

namespace iflow {

constexpr int ATT_D = 128;                                    // head dimension
constexpr int ATT_WAVES = 4;
constexpr int ATT_TILES = 4;                                  // tiles of four positions per block: 16 positions per wavefront and block
constexpr int ATT_MAX_SPLITS = 64;
// workspace: value sums O[head][ATT_MAX_SPLITS][component], then maxima M[head][ATT_MAX_SPLITS], then sums L[head][ATT_MAX_SPLITS]
// (fp32; a state's 128 components are contiguous: written and read by 128 neighbouring threads)

typedef uint32_t att_u32x4 __attribute__((ext_vector_type(4)));

template <int R>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_decode_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc,
                                                                     const uint16_t *__restrict__ vc, uint16_t *__restrict__ out,
                                                                     float *__restrict__ ws, int n_heads, int seq_len, int64_t head_stride /* halves */,
                                                                     int chunk, int nsplit, float scale_log2e)
{
    __shared__ float s_acc[16][ATT_D];
    __shared__ float s_m[16], s_l[16];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int gq = lane >> 4, dseg = lane & 15;               // position inside a tile; which 8 of the 128 components
    const int j = blockIdx.x / nsplit, sp = blockIdx.x - j * nsplit;
    const int t_begin = sp * chunk, t_end = min(seq_len, t_begin + chunk);      // t_begin < seq_len by construction
    const uint16_t *kh = kc + (int64_t)j * head_stride + dseg * 8;
    const uint16_t *vh = vc + (int64_t)j * head_stride + dseg * 8;

    // the group's queries: lane holds components 8 dseg .. 8 dseg + 7 of each
    half2_t qr[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const att_u32x4 v = *reinterpret_cast<const att_u32x4 *>(q + (int64_t)(j * R + r) * ATT_D + dseg * 8);
        qr[r][0] = as_h2(v.x); qr[r][1] = as_h2(v.y); qr[r][2] = as_h2(v.z); qr[r][3] = as_h2(v.w);
    }
    float m[R], l[R], acc[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    }

    // positions past the range are loaded from the range's last position (in bounds) and their scores set to -inf
    auto load_block = [&](att_u32x4 (&kt)[ATT_TILES], att_u32x4 (&vt)[ATT_TILES], int p0) {
#pragma unroll
        for (int t = 0; t < ATT_TILES; ++t) {
            const int64_t pos = min(p0 + t * 4 + gq, t_end - 1);
            kt[t] = __builtin_nontemporal_load(reinterpret_cast<const att_u32x4 *>(kh + pos * ATT_D));
            vt[t] = __builtin_nontemporal_load(reinterpret_cast<const att_u32x4 *>(vh + pos * ATT_D));
        }
    };
    auto process_block = [&](const att_u32x4 (&kt)[ATT_TILES], const att_u32x4 (&vt)[ATT_TILES], int p0) {
        float vf[ATT_TILES][8];
#pragma unroll
        for (int t = 0; t < ATT_TILES; ++t) {
            const half2_t a = as_h2(vt[t].x), b = as_h2(vt[t].y), c = as_h2(vt[t].z), d = as_h2(vt[t].w);
            vf[t][0] = (float)a.x; vf[t][1] = (float)a.y; vf[t][2] = (float)b.x; vf[t][3] = (float)b.y;
            vf[t][4] = (float)c.x; vf[t][5] = (float)c.y; vf[t][6] = (float)d.x; vf[t][7] = (float)d.y;
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float s[ATT_TILES];
            float bm = -INFINITY;
#pragma unroll
            for (int t = 0; t < ATT_TILES; ++t) {
                float d = __builtin_amdgcn_fdot2(qr[r][0], as_h2(kt[t].x), 0.f, false);
                d = __builtin_amdgcn_fdot2(qr[r][1], as_h2(kt[t].y), d, false);
                d = __builtin_amdgcn_fdot2(qr[r][2], as_h2(kt[t].z), d, false);
                d = __builtin_amdgcn_fdot2(qr[r][3], as_h2(kt[t].w), d, false);
                d = row16_sum(d) * scale_log2e;               // the score of this lane group's position, in units of log2
                s[t] = (p0 + t * 4 + gq < t_end) ? d : -INFINITY;
                bm = fmaxf(bm, s[t]);
            }
            const float m_new = fmaxf(m[r], bm);
            // (a state that has not seen a valid position yet has maximum -inf: nothing to rescale, and no -inf - -inf)
            const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m[r] - m_new);
            const float base = (m_new == -INFINITY) ? 0.f : m_new;
            l[r] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] *= alpha;
#pragma unroll
            for (int t = 0; t < ATT_TILES; ++t) {
                const float p = __builtin_amdgcn_exp2f(s[t] - base);            // exp2(-inf) = 0 for masked positions
                l[r] += p;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[r][e] = __builtin_fmaf(p, vf[t][e], acc[r][e]);
            }
            m[r] = m_new;
        }
    };

    // blocks of this wavefront: wave, wave + 4, ... of the range, two per trip so that the two register sets alternate
    att_u32x4 ka[ATT_TILES], va[ATT_TILES], kb[ATT_TILES], vb[ATT_TILES];
    constexpr int STEP = 16 * ATT_WAVES;                      // positions between a wavefront's consecutive blocks
    int p0 = t_begin + wave * 16;
    // (the scheduling barriers pin the order in which the two sets are requested: the wait in front of a block counts
    // the requests issued after that block's own, and a reordered prologue would turn it into a wait for everything)
    load_block(ka, va, p0);
    __builtin_amdgcn_sched_barrier(0);
    load_block(kb, vb, p0 + STEP);
    __builtin_amdgcn_sched_barrier(0);
    for (; p0 < t_end; p0 += 2 * STEP) {
        process_block(ka, va, p0);
        __builtin_amdgcn_sched_barrier(0);
        load_block(ka, va, p0 + 2 * STEP);
        __builtin_amdgcn_sched_barrier(0);
        if (p0 + STEP < t_end) process_block(kb, vb, p0 + STEP);              // (uniform over the wavefront)
        __builtin_amdgcn_sched_barrier(0);
        load_block(kb, vb, p0 + 3 * STEP);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- merge the sixteen states (4 wavefronts x 4 lane groups) of each head, store or hand over -----------------------
    const int pid = wave * 4 + gq;
    float *ws_o = ws, *ws_m = ws + (int64_t)n_heads * ATT_D * ATT_MAX_SPLITS, *ws_l = ws_m + (int64_t)n_heads * ATT_MAX_SPLITS;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if (r > 0) __syncthreads();                           // the previous head's states have been read
#pragma unroll
        for (int e = 0; e < 8; ++e) s_acc[pid][dseg * 8 + e] = acc[r][e];
        if (dseg == 0) { s_m[pid] = m[r]; s_l[pid] = l[r]; }
        __syncthreads();
        if (tid < ATT_D) {
            float M = s_m[0];
#pragma unroll
            for (int i = 1; i < 16; ++i) M = fmaxf(M, s_m[i]);                  // finite: the range is not empty
            float L = 0.f, O = 0.f;
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                const float f = __builtin_amdgcn_exp2f(s_m[i] - M);
                L = __builtin_fmaf(s_l[i], f, L);
                O = __builtin_fmaf(s_acc[i][tid], f, O);
            }
            const int head = j * R + r;
            if (nsplit == 1) {
                out[(int64_t)head * ATT_D + tid] = as_u16((half_t)(O / L));
            } else {
                ws_o[((int64_t)head * ATT_MAX_SPLITS + sp) * ATT_D + tid] = O;
                if (tid == 0) { ws_m[(int64_t)head * ATT_MAX_SPLITS + sp] = M; ws_l[(int64_t)head * ATT_MAX_SPLITS + sp] = L; }
            }
        }
    }
}

// ---- groups of four or eight query heads per kv head: scores and weighted sums on the matrix cores --------------------
// With eight heads per loaded key the vector units bind (about 46 instructions per position in the kernel above).  But a
// block of sixteen positions against a group of heads is two small dense contractions:
//   S[position][head]  = sum_k K[position][k] Q[head][k]            16 x 128 x (16 heads, 4 or 8 of them real)
//   O[head][component] = sum_position P[position][head] V[position][component]
// and v_mfma_f32_16x16x16_f16 does each in eight instructions per block.  Operand layouts of that instruction, lane =
// i + 16 g: A: lane holds A[i][4g..4g+3]; B: lane holds B[4g..4g+3][i]; C/D: lane holds D[4g..4g+3][i].
//   - Scores: A = keys (row = position), B = queries (column = head).  A lane loads its position's keys in four 16-byte
//     pieces K[position][32u + 8g .. +8]; each piece feeds two instructions, so instruction (u, h) sums over the
//     components 32u + 8g + 4h + e - any order of k will do as long as the queries are loaded the same way.
//   - The result D[position 4g+e][head i] is, read the other way round, P^T[head i][positions 4g..4g+3]: exactly an A
//     operand of the second contraction (row = head, k = position).  So the probabilities never move between lanes.
//   - The second contraction wants B = values with k = position, i.e. four values of ONE component from four
//     consecutive positions per lane, while the cache holds a position's 128 components together.  The wavefront's
//     16 x 128 value tile therefore crosses LDS: written as loaded (16-byte pieces), read back by columns (rows 272 bytes
//     apart, which puts the four lane groups on different banks).
//   - Streaming softmax per head in the lanes that hold that head's column of S; the rescale factors of heads 4g..4g+3
//     are fetched across lanes for the accumulators, which are laid out by (head, component).
// RMAX (4, 8 or 16) is the number of query heads a workgroup serves from one pass over its keys and values: a group of up
// to RMAX heads takes one pass, a larger group (the paper's multi-query models: every head shares one key/value head) is
// cut into pieces of RMAX heads along the grid's second dimension.  D (64 or 128) is the head dimension: D / 32 pieces of
// 16 bytes per lane and position, D / 16 column groups of the weighted sum.
template <int RMAX, int D>
__global__ __launch_bounds__(64 * ATT_WAVES) void attn_decode_mfma_kernel(const uint16_t *__restrict__ q, const uint16_t *__restrict__ kc,
                                                                          const uint16_t *__restrict__ vc, uint16_t *__restrict__ out,
                                                                          float *__restrict__ ws, int n_heads, int group, int seq_len,
                                                                          int64_t head_stride /* halves */, int chunk, int nsplit,
                                                                          float scale_log2e)
{
    static_assert((RMAX == 4 || RMAX == 8 || RMAX == 16) && (D == 64 || D == 128), "group piece and head dimension");
    typedef _Float16 half4v __attribute__((ext_vector_type(4)));
    typedef float float4v __attribute__((ext_vector_type(4)));
    constexpr int NU = D / 32, NC = D / 16;
    constexpr int VROW = 2 * D + 16;                          // bytes between rows of the staged value tile (a multiple of 16)
    __shared__ __align__(16) uint8_t s_v[ATT_WAVES][16 * VROW];
    __shared__ float s_o[ATT_WAVES][RMAX][D];
    __shared__ float s_m[ATT_WAVES][16], s_l[ATT_WAVES][16];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int li = lane & 15, g = lane >> 4;
    const int j = blockIdx.x / nsplit, sp = blockIdx.x - j * nsplit;
    const int r0 = blockIdx.y * RMAX, rr = min(RMAX, group - r0);     // this workgroup's heads of the group: r0 .. r0 + rr - 1
    const int t_begin = sp * chunk, t_end = min(seq_len, t_begin + chunk);
    const uint16_t *kh = kc + (int64_t)j * head_stride + g * 8;
    const uint16_t *vh = vc + (int64_t)j * head_stride + g * 8;

    // queries as B operands: lane (head li, g) holds Q[head][32u + 8g + 4h + e]; heads past the piece are zero
    half4v qb[2 * NU];
#pragma unroll
    for (int u = 0; u < NU; ++u) {
        att_u32x4 v = {0u, 0u, 0u, 0u};
        if (li < rr) v = *reinterpret_cast<const att_u32x4 *>(q + (int64_t)(j * group + r0 + li) * D + 32 * u + 8 * g);
        qb[2 * u] = __builtin_bit_cast(half4v, make_uint2(v.x, v.y));
        qb[2 * u + 1] = __builtin_bit_cast(half4v, make_uint2(v.z, v.w));
    }
    float m = -INFINITY, l = 0.f;                             // of head li (the maximum is the same in the four lanes of a head)
    float4v oacc[NC];                                         // oacc[c][e] = O[head 4g+e][16c + li]
#pragma unroll
    for (int c = 0; c < NC; ++c) oacc[c] = (float4v){0.f, 0.f, 0.f, 0.f};

    auto load_block = [&](att_u32x4 (&kt)[NU], att_u32x4 (&vt)[NU], int p0) {
        const int64_t pos = min(p0 + li, t_end - 1);          // past the range: its last position, masked below
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            kt[u] = __builtin_nontemporal_load(reinterpret_cast<const att_u32x4 *>(kh + pos * D + 32 * u));
            vt[u] = __builtin_nontemporal_load(reinterpret_cast<const att_u32x4 *>(vh + pos * D + 32 * u));
        }
    };
    uint8_t *myv = s_v[wave];
    auto process_block = [&](const att_u32x4 (&kt)[NU], const att_u32x4 (&vt)[NU], int p0) {
        // values -> LDS as loaded: row = position li, bytes 64u + 16g
#pragma unroll
        for (int u = 0; u < NU; ++u) *reinterpret_cast<att_u32x4 *>(myv + li * VROW + 64 * u + 16 * g) = vt[u];
        // scores
        float4v sacc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int u = 0; u < NU; ++u) {
            const half4v a0 = __builtin_bit_cast(half4v, make_uint2(kt[u].x, kt[u].y));
            const half4v a1 = __builtin_bit_cast(half4v, make_uint2(kt[u].z, kt[u].w));
            sacc = __builtin_amdgcn_mfma_f32_16x16x16f16(a0, qb[2 * u], sacc, 0, 0, 0);
            sacc = __builtin_amdgcn_mfma_f32_16x16x16f16(a1, qb[2 * u + 1], sacc, 0, 0, 0);
        }
        float sc[4], bm = -INFINITY;
#pragma unroll
        for (int e = 0; e < 4; ++e) {                         // position p0 + 4g + e, head li
            sc[e] = (p0 + 4 * g + e < t_end) ? sacc[e] * scale_log2e : -INFINITY;
            bm = fmaxf(bm, sc[e]);
        }
        bm = fmaxf(bm, __shfl_xor(bm, 16));                   // the head's maximum over the block's sixteen positions
        bm = fmaxf(bm, __shfl_xor(bm, 32));
        const float m_new = fmaxf(m, bm);
        const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m - m_new);
        const float base = (m_new == -INFINITY) ? 0.f : m_new;
        float p[4];
        l *= alpha;
#pragma unroll
        for (int e = 0; e < 4; ++e) { p[e] = __builtin_amdgcn_exp2f(sc[e] - base); l += p[e]; }
        m = m_new;
        const half4v pa = {(_Float16)p[0], (_Float16)p[1], (_Float16)p[2], (_Float16)p[3]};
        // The accumulators hold heads 4g .. 4g+3: their rescale factors live in lanes 4g .. 4g+3.  Only when some head's
        // maximum has moved (after the first blocks of a range it rarely does): the accumulators sit in the matrix
        // cores' own registers, and rescaling them means moving all 32 out and back.
        if (__builtin_amdgcn_ballot_w64(alpha != 1.0f) != 0) {
            float al[4];
#pragma unroll
            for (int e = 0; e < 4; ++e) al[e] = __shfl(alpha, 4 * g + e);
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int e = 0; e < 4; ++e) oacc[c][e] *= al[e];
        }
        // weighted sums: B = values by columns from LDS (the wavefront's own tile: LDS operations of a wavefront are served in order)
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const uint16_t *col = reinterpret_cast<const uint16_t *>(myv + (4 * g) * VROW) + 16 * c + li;
            const half4v vb = {as_h(col[0]), as_h(col[VROW / 2]), as_h(col[2 * (VROW / 2)]), as_h(col[3 * (VROW / 2)])};
            oacc[c] = __builtin_amdgcn_mfma_f32_16x16x16f16(pa, vb, oacc[c], 0, 0, 0);
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();                      // the next block overwrites the tile
    };

    att_u32x4 ka[NU], va[NU], kb[NU], vb2[NU];
    constexpr int STEP = 16 * ATT_WAVES;
    int p0 = t_begin + wave * 16;
    load_block(ka, va, p0);                                   // (scheduling barriers: see attn_decode_kernel)
    __builtin_amdgcn_sched_barrier(0);
    load_block(kb, vb2, p0 + STEP);
    __builtin_amdgcn_sched_barrier(0);
    for (; p0 < t_end; p0 += 2 * STEP) {
        process_block(ka, va, p0);
        __builtin_amdgcn_sched_barrier(0);
        load_block(ka, va, p0 + 2 * STEP);
        __builtin_amdgcn_sched_barrier(0);
        if (p0 + STEP < t_end) process_block(kb, vb2, p0 + STEP);
        __builtin_amdgcn_sched_barrier(0);
        load_block(kb, vb2, p0 + 3 * STEP);
        __builtin_amdgcn_sched_barrier(0);
    }

    // ---- merge the four wavefronts' states ----------------------------------------------------------------------------------
    l += __shfl_xor(l, 16);                                   // a head's sum over its four lanes
    l += __shfl_xor(l, 32);
    if (g == 0) { s_m[wave][li] = m; s_l[wave][li] = l; }
    if (4 * g < RMAX) {
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int e = 0; e < 4; ++e) s_o[wave][4 * g + e][16 * c + li] = oacc[c][e];
    }
    __syncthreads();
    float *ws_o = ws, *ws_m = ws + (int64_t)n_heads * ATT_D * ATT_MAX_SPLITS, *ws_l = ws_m + (int64_t)n_heads * ATT_MAX_SPLITS;
    for (int idx = tid; idx < rr * D; idx += 64 * ATT_WAVES) {
        const int r = idx / D, d = idx & (D - 1);
        float M = s_m[0][r];
#pragma unroll
        for (int w = 1; w < ATT_WAVES; ++w) M = fmaxf(M, s_m[w][r]);            // finite: the range is not empty
        float L = 0.f, O = 0.f;
#pragma unroll
        for (int w = 0; w < ATT_WAVES; ++w) {
            const float f = __builtin_amdgcn_exp2f(s_m[w][r] - M);
            L = __builtin_fmaf(s_l[w][r], f, L);
            O = __builtin_fmaf(s_o[w][r][d], f, O);
        }
        const int head = j * group + r0 + r;
        if (nsplit == 1) {
            out[(int64_t)head * D + d] = as_u16((half_t)(O / L));
        } else {
            ws_o[((int64_t)head * ATT_MAX_SPLITS + sp) * ATT_D + d] = O;
            if (d == 0) { ws_m[(int64_t)head * ATT_MAX_SPLITS + sp] = M; ws_l[(int64_t)head * ATT_MAX_SPLITS + sp] = L; }
        }
    }
}

// Merge of the splits: one workgroup per query head, thread d for component d (a state keeps 128 slots whatever the head
// dimension).  Only entries below
// nsplit are read (the rest of the workspace is whatever earlier calls left there, possibly never touched).
__global__ __launch_bounds__(ATT_D) void attn_merge_kernel(const float *__restrict__ ws, uint16_t *__restrict__ out, int n_heads, int nsplit)
{
    const int head = blockIdx.x, d = threadIdx.x, head_dim = blockDim.x;
    const float *ws_o = ws + (int64_t)head * ATT_MAX_SPLITS * ATT_D + d;
    const float *ws_m = ws + (int64_t)n_heads * ATT_D * ATT_MAX_SPLITS + (int64_t)head * ATT_MAX_SPLITS;
    const float *ws_l = ws_m + (int64_t)n_heads * ATT_MAX_SPLITS;
    // eight ranges at a time, every load of a batch issued before anything waits (maxima, sums and value sums do not depend
    // on each other's addresses): one memory round trip per batch instead of one for the maxima and one for the rest
    float M = -INFINITY, L = 0.f, O = 0.f;
    for (int i0 = 0; i0 < nsplit; i0 += 8) {
        float m[8], l[8], o[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int i = min(i0 + u, nsplit - 1);            // past the end: the last range again (not added below)
            m[u] = ws_m[i]; l[u] = ws_l[i]; o[u] = ws_o[(int64_t)i * ATT_D];
        }
        float mb = m[0];
#pragma unroll
        for (int u = 1; u < 8; ++u) mb = fmaxf(mb, m[u]);     // (a repeated range does not change the maximum)
        const float m_new = fmaxf(M, mb);                     // finite: no range is empty
        const float keep = __builtin_amdgcn_exp2f(M - m_new); // 0 for the first batch
        L *= keep; O *= keep;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const float f = i0 + u < nsplit ? __builtin_amdgcn_exp2f(m[u] - m_new) : 0.f;
            L = __builtin_fmaf(l[u], f, L);
            O = __builtin_fmaf(o[u], f, O);
        }
        M = m_new;
    }
    out[(int64_t)head * head_dim + d] = as_u16((half_t)(O / L));
}

// positions per split (a multiple of 64, one block per wavefront) and number of splits for a sequence length
static void attn_geometry(int n_kv_heads, int64_t seq_len, int cus, int *chunk, int *nsplit)
{
    int64_t want = (1 * (int64_t)cus + n_kv_heads - 1) / n_kv_heads;          // about one workgroup per compute unit
    if (want < 1) want = 1;
    if (want > ATT_MAX_SPLITS) want = ATT_MAX_SPLITS;
    int64_t c = (seq_len + want - 1) / want;
    c = (c + 63) / 64 * 64;
    *chunk = (int)c;
    *nsplit = (int)((seq_len + c - 1) / c);
}

size_t attn_workspace_bytes(int n_heads)
{
    return (size_t)n_heads * (ATT_D + 2) * ATT_MAX_SPLITS * sizeof(float);
}

hipError_t launch_attn_decode(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads, int n_kv_heads,
                              int head_dim, int64_t seq_len, int64_t max_seq, float scale, uint16_t *out, void *workspace, hipStream_t s)
{
    static PerDevice pd;
    int cus = 0;
    hipError_t e = once_per_device(pd, &cus, [] { return hipSuccess; });
    if (e != hipSuccess) return e;
    if (n_kv_heads < 1 || n_kv_heads > 64 || n_heads % n_kv_heads != 0 || seq_len < 1 || seq_len > max_seq) return hipErrorInvalidValue;
    if (head_dim != 64 && head_dim != 128) return hipErrorInvalidValue;
    const int R = n_heads / n_kv_heads;
    int chunk = 0, nsplit = 0;
    attn_geometry(n_kv_heads, seq_len, cus, &chunk, &nsplit);
    if (nsplit < 1 || nsplit > ATT_MAX_SPLITS) return hipErrorInvalidValue;
    const dim3 block(64 * ATT_WAVES);
    const float scale_log2e = scale * 1.4426950408889634f;
    const int64_t head_stride = max_seq * head_dim;
#define IFLOW_ATT_GO(RR) hipLaunchKernelGGL((attn_decode_kernel<RR>), dim3((unsigned)(n_kv_heads * nsplit)), block, 0, s, q, k_cache, \
        v_cache, out, static_cast<float *>(workspace), n_heads, (int)seq_len, head_stride, chunk, nsplit, scale_log2e)
#define IFLOW_ATT_GO_MFMA(RMAX, DD) hipLaunchKernelGGL((attn_decode_mfma_kernel<RMAX, DD>), \
        dim3((unsigned)(n_kv_heads * nsplit), (unsigned)((R + RMAX - 1) / RMAX)), block, 0, s, q, k_cache, v_cache, out, \
        static_cast<float *>(workspace), n_heads, R, (int)seq_len, head_stride, chunk, nsplit, scale_log2e)
    // one or two heads per key/value head at 128 components: the vector kernel; everything else on the matrix cores, in
    // pieces of 4, 8 or 16 heads
    if (head_dim == 128 && R == 1) IFLOW_ATT_GO(1);
    else if (head_dim == 128 && R == 2) IFLOW_ATT_GO(2);
    else if (head_dim == 128 && R <= 4) IFLOW_ATT_GO_MFMA(4, 128);
    else if (head_dim == 128 && R <= 8) IFLOW_ATT_GO_MFMA(8, 128);
    else if (head_dim == 128) IFLOW_ATT_GO_MFMA(16, 128);
    else if (R <= 4) IFLOW_ATT_GO_MFMA(4, 64);
    else if (R <= 8) IFLOW_ATT_GO_MFMA(8, 64);
    else IFLOW_ATT_GO_MFMA(16, 64);
#undef IFLOW_ATT_GO
#undef IFLOW_ATT_GO_MFMA
    e = hipGetLastError();
    if (e != hipSuccess || nsplit == 1) return e;
    hipLaunchKernelGGL(attn_merge_kernel, dim3((unsigned)n_heads), dim3((unsigned)head_dim), 0, s, static_cast<const float *>(workspace), out, n_heads, nsplit);
    return hipGetLastError();
}

// ---- the same call for callers that cannot allocate ------------------------------------------------------------
// The partial results of the position ranges live in a file-scope device array instead of a caller's workspace.  In
// host code the array's name is only a handle: its device address is asked for once per device (each device holds its
// own copy at its own address) and only that address is ever handed to a kernel.
constexpr int ATT_STATIC_MAX_HEADS = IFLOW_ATTN_STATIC_MAX_HEADS;
static __device__ __align__(256) float scratch[(size_t)ATT_STATIC_MAX_HEADS * (ATT_D + 2) * ATT_MAX_SPLITS];

hipError_t launch_attn_decode_static(const uint16_t *q, const uint16_t *k_cache, const uint16_t *v_cache, int n_heads, int n_kv_heads,
                                     int head_dim, int64_t seq_len, int64_t max_seq, float scale, uint16_t *out, hipStream_t s)
{
    static std::mutex lock;
    static float *address[IFLOW_MAX_DEVICES] = {};
    if (n_heads < 1 || n_heads > ATT_STATIC_MAX_HEADS) return hipErrorInvalidValue;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= IFLOW_MAX_DEVICES) return hipErrorInvalidDevice;
    float *ptr = nullptr;
    {
        std::lock_guard<std::mutex> hold(lock);
        if (!address[dev]) {
            void *sym = nullptr;
            e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
            if (e != hipSuccess) return e;
            if (!sym) return hipErrorInvalidSymbol;
            address[dev] = static_cast<float *>(sym);
        }
        ptr = address[dev];
    }
    return launch_attn_decode(q, k_cache, v_cache, n_heads, n_kv_heads, head_dim, seq_len, max_seq, scale, out, ptr, s);
}

}  // namespace iflow
