// A chain of matrix-vector products in ONE launch (every format; written for the 3.5-bit one): phase after phase, each phase a group of matrices that
// share an activation vector, and a phase may take as its activations the output of a matrix of an earlier
// phase (q/k/v -> o -> gate/up -> down of a decoder layer).  At batch 1 a 7B-sized product lasts a few
// microseconds, of which a launch boundary costs 1.6 us of idle memory system plus the ramp of a fresh grid;
// here the grid stays resident, and the weights of the next phase are already on their way while the outputs
// of the current one are handed over.
//
// Resident grid: one workgroup of 12 wavefronts per compute unit (8 in the variant with the attention inside).  Each phase's
// rows are cut into equal contiguous ranges, one per workgroup; wavefront w of a workgroup takes the row pairs w, w + 12, ... of the range and walks
// each pair strip by strip (a strip = 64 blocks = 4096 columns, one block per lane, as in the single-product
// kernel; the two rows of a pair share the activation registers).  A wavefront keeps S steps (row pair, strip) of
// weights in flight in S register sets and requests step k + S as soon as step k is decoded, across phase
// boundaries: weights do not depend on the activations, so the memory system keeps streaming while a phase waits
// for its input.
//
// Hand-over without a grid barrier: outputs that a later phase consumes travel through the caller's workspace
// as 32-bit words (fp16 value, 16-bit tag), written with write-through stores once a wavefront has finished its
// rows of the phase, and read with cache-bypassing loads.  The tag comes from a launch counter kept in the workspace, so a
// word is its own "ready" flag: a consumer simply re-reads until every word of the vector carries this launch's
// tag.  There are no atomics on shared counters and no fences; one memory round trip separates the last producer
// from the first consumer.  The words are stored in the order in which the consumer's threads want them (below),
// so that their loads coalesce.  The count advances once per launch (every workgroup advances its own copy when it is
// done, and launches of a chain are ordered), so a
// word left by the previous launch never carries the current tag; a workspace that changes hands between chains
// of different shapes has to be zeroed in between (tags repeat every 65535 launches).  Every wait is bounded:
// when the budget runs out the workgroup raises the error word of the workspace and carries on, so the launch
// always ends (iflow_qgemv_chain_check reports it).
#include "iflow_lane.h"


#include <type_traits>

#define IFLOW_GLOBAL __attribute__((address_space(1)))

namespace iflow {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <typename T> __device__ __forceinline__ IFLOW_GLOBAL T *global_ptr(const void *p) { return (IFLOW_GLOBAL T *)(uint64_t)p; }

#ifndef IFLOW_CHAIN_WAVES
#define IFLOW_CHAIN_WAVES 12
#endif
#ifndef IFLOW_CHAIN_WAVES_ATTN
#define IFLOW_CHAIN_WAVES_ATTN 8
#endif
// Wavefronts per workgroup.  Launches of products only: 12 (measured on 7B-shaped layers with 8 / 10 / 12 / 16: 23.7 / 23.0 /
// 22.9 / 27.6 us per layer; 12 divides the row pairs of 7B-sized phases evenly, 16 leaves a wavefront 128 registers and
// spills).  Launches with the attention inside: 8 - two wavefronts per SIMD have 256 registers each, which the attention
// phases need (with 12 the kernel keeps 90 registers in scratch memory): a 7B decode step at 1024 cached positions 37.3 ->
// 33.9 us per layer.
constexpr int chain_waves(bool attn) { return attn ? IFLOW_CHAIN_WAVES_ATTN : IFLOW_CHAIN_WAVES; }
constexpr int CHAIN_WAVES_ATTN = IFLOW_CHAIN_WAVES_ATTN;       // (the attention's own code is built for that variant only)
// A strip is what the 64 lanes of a wavefront cover of a row in one step: 64 x (weights per lane) columns - 4096 for the
// 3.5-bit format (a block per lane), 2048 for the 4-bit and 1024 for the 8-bit formats (16 bytes of codes per lane).
// Staged activations of one strip: the lanes' registers in decode order, 16 bytes per lane and quarter, then the two sums
// per lane that undo the decode's bias (as in the single-product kernels).
template <int KIND> constexpr int chain_strip_cols() { return 64 * Geo<KIND>::WPL; }
template <int KIND> constexpr int chain_slot_bytes() { return Geo<KIND>::XD / 4 * 1024 + 512; }
constexpr int CHAIN_LDS_BYTES = 152 * 1024;
constexpr int CHAIN_MAX_COLS = 65536;
constexpr int CHAIN_MAX_GROUP = IFLOW_CHAIN_MAX_GROUP;         // matrices per phase
constexpr int CHAIN_MAX_GRID = 960;
constexpr int CHAIN_POLL_BUDGET = 1 << 17;                     // re-reads before a wait is given up (tens of milliseconds)
// Between two reads of a hand-over word that has not arrived, x 64 cycles.  Measured on 7B-shaped layers, us per layer of
// the plain stack with 0 / 2 / 8 / 24 / 64: 22.8 / 23.0 / 23.4 / 26.1 / 30.7 - the sooner the last producer's store is seen
// the better (0 and 2 are within the noise of each other once the modules are in; 2 is kept); two rounds of reads in
// flight at once (the words looked at twice per memory round trip) are slower again, 24.0: their traffic competes with
// the weights.
constexpr int CHAIN_POLL_SLEEP = 2;
// workspace header, in 32-bit words: [1] error, [8, 12) the launch's clock stamps (below), [64, 64 + grid) the launch count,
// one copy per workgroup;
// tagged outputs start at byte IFLOW_CHAIN_WS_HEADER
constexpr int CHAIN_WS_ERROR = 1, CHAIN_WS_CLOCKS = IFLOW_CHAIN_WS_CLOCKS, CHAIN_WS_SEEN = 64;

// The plan: what iflow_qgemv_chain_plan writes into the caller's device memory once, and every launch reads.  The weights
// of a model never change between tokens, so the chain is described once; a launch passes two pointers.  Everything a
// wavefront needs when it enters a phase sits in one 64-byte descriptor, and everything about a matrix in one 32-byte
// descriptor: a scalar load each, instead of a chain of dependent loads (a scalar load costs a few hundred nanoseconds
// of latency, and a phase of a 7B layer lasts a few microseconds).  Layout: ChainHeader, the phase descriptors, the matrix
// descriptors, the phases' operation records.
struct ChainPhase {
    const uint16_t *x;          // activations when they are an input of the launch
    int first, count;           // matrices [first, first + count)
    int nbk, nstrips;           // blocks (of the format's block size) and strips per row
    int x_src;                  // matrix whose output is this phase's activation vector, or -1
    int rows_per_wg;
    int total;                  // rows of the phase, all its matrices together
    int x_tag_word;             // tagged output of matrix x_src, in 32-bit words from the workspace start
    int mstart[CHAIN_MAX_GROUP];    // first row of each matrix within the phase; INT_MAX past `count`
    int kind;                   // 0: products; 1, 2: the two halves of a decode attention (below), with no rows of their own
    int attn;                   // which attention
};
struct ChainMatrix {
    const uint8_t *packed;
    uint16_t *y;
    int rows;                   // rows in the phase's row space; a gated pair: 2 x rows (row 2n = gate row n, row 2n+1 = up row n)
    int start;                  // first row of the matrix within its phase
    int tag_word;               // its tagged output, in 32-bit words from the workspace start
    int gated;                  // 1: `packed` is the gate and `packed2` the up matrix of a gated feed-forward, one output per row pair
    const uint8_t *packed2;
    const uint16_t *residual;   // added to the output: an input of the launch ([rows] fp16) ...
    int residual_tag_word;      // ... or the tagged output of an earlier matrix (0: none)
    uint32_t hdr_off4;          // formats that keep the block headers behind the codes: where they start, in 4-byte units from `packed`
    uint32_t hi_off4;           // bit-plane formats: where the high plane starts, in 4-byte units from `packed`
    int pad_;
};
// what only the fused variant of the kernel reads about a phase
struct ChainPhaseOps {
    const uint16_t *aux;        // IFLOW_X_RMS_GAIN: the gains [cols] fp16 (an input of the launch)
    float eps;
    int x_op;                   // iflow_x_op_t
    float inv_cols;
    int next_attn;              // the first phase of kind 1 behind this one (nphases: none)
    int pad_[2];
};
struct ChainHeader {
    uint32_t magic;
    int nphases, nmatrices, grid;
    int max_strips, fused, format, nattn, lds_bytes;
    int first_attn;             // the first phase of kind 1 (nphases: none)
    int pad_[6];
};
// One decode step of grouped-query attention inside the launch (section "Grouped-query attention"; Section 5's Infer() runs
// it between the q/k/v products and the output projection), head dimension 128, with the rotary position embedding of the
// step's query and key and the step's append to the key/value cache (what iflow_rope_append and iflow_attn_decode do as
// launches of their own).  It takes two phases.  Phase "part": workgroup (kv head j, range sp) rotates the group's queries,
// walks its range of cached positions with a streaming softmax and leaves one partial state (maximum, sum, 128 weighted value
// sums) per query head in the workspace, as 64-bit words (fp32 bits, launch tag); the workgroup whose range holds the step's
// own position rotates the new key, uses it and the new value from registers and writes both into the caches.  Phase "merge":
// every output component merges the partial states of its head's ranges and is published like any output of a product, for
// the output projection that follows.
struct ChainAttn {
    const uint16_t *q, *k_new, *v_new;  // where they are inputs of the launch (else null: tagged outputs of earlier products)
    uint16_t *k_cache, *v_cache;        // [n_kv_heads][max_seq][128] fp16
    uint16_t *out;                      // [n_heads][128] fp16
    int q_tag_word, k_tag_word, v_tag_word, out_tag_word;   // in 32-bit words from the workspace start
    int part_word;                      // partial states: 64-bit words [head][nsplit][130] (128 value sums, maximum, sum)
    int n_heads, n_kv_heads, nsplit;
    int max_seq, pairing;               // iflow_rope_pairing_t
    float scale_log2e;
    int pad0_;
    double log2_base;
    int pad_[6];
};
static_assert(sizeof(ChainPhase) == 64 && sizeof(ChainMatrix) == 64 && sizeof(ChainHeader) == 64 && sizeof(ChainPhaseOps) == 32 &&
              sizeof(ChainAttn) == 128, "descriptor sizes");
// the two descriptor arrays of a plan, as the kernel indexes them
struct ChainArgs {
    const ChainPhase *ph;
    const ChainMatrix *mat;
    const ChainPhaseOps *ops;
    const ChainAttn *attn;
};

// Position of output r inside a matrix's tagged vector, in 32-bit words.  A consumer thread stages one chunk of 16
// activations with eight 8-byte loads; the pair (2i, 2i+1) of chunk c of a strip sits at 8-byte word i * 256 + c,
// so the loads of neighbouring threads read neighbouring words.
__device__ __forceinline__ int chain_tag_word(int r)
{
    const int g = r >> 1;
    return 2 * ((g >> 11) * 2048 + (g & 7) * 256 + ((g >> 3) & 255)) + (r & 1);
}

// The step loop is bound by instruction issue (one scalar unit serves the sixteen wavefronts of a compute unit), so
// the bookkeeping of a step is kept to a handful of scalar instructions: a wavefront walks its rows segment by
// segment, a segment being consecutive rows of the wavefront (16 apart) inside one matrix and one 4096-row strip of
// its tagged output, so that within a segment every pointer advances by a constant.  Everything else (finding the
// matrix of a row, entering a phase) happens once per segment.  The walk exists twice: for the requests, S steps
// ahead, and for the consumption.
#define IFLOW_UNI(v) __builtin_amdgcn_readfirstlane(v)

// What a walk keeps in registers is only what a step needs; everything a segment change needs (which matrices the
// phase has, where they start) is read again from the kernel arguments then, to keep the scalar register file for the
// loop itself.
struct ChainWalk {
    int p;                      // phase; nphases when the walk is over
    int rows_left;              // rows of this wavefront in phase p that no segment covers yet
    int R;                      // the first of them, in the phase's row space
    int seg_left;               // rows left in the current segment, the current one included
};

// FUSED: the variant that also runs the modules between the products of a decoder layer (Section 2's module table: "rms"
// normalization, "silu" activation; Section 5's Infer() applies them between the products): rms gains folded into the
// staging of a phase's activations and the normalization's scalar into its outputs, the gate of a gated feed-forward
// applied where its two projections are summed, residuals added at the store.  The plain variant is the code without any
// of it (a launch of bare products pays nothing for the modules).
#ifndef IFLOW_CHAIN_SETS
#define IFLOW_CHAIN_SETS 2
#endif
#ifndef IFLOW_CHAIN_TRACE
#define IFLOW_CHAIN_TRACE 0
#endif
#ifndef IFLOW_CHAIN_EARLY
#define IFLOW_CHAIN_EARLY 0
#endif
// Measurement aid, off in the library (outputs are wrong with it on; every access stays where it is): 1 - the step loop
// requests and waits for its weights but does not decode them; 2 - it decodes whatever its registers hold and requests
// nothing.  Together with the clock stamps below these tell what a launch's time is made of.
#ifndef IFLOW_CHAIN_ABL
#define IFLOW_CHAIN_ABL 0
#endif
constexpr int CHAIN_SETS = IFLOW_CHAIN_SETS;
// Register sets (steps of weights in flight) per wavefront: a step of the 3.5-bit format is 4 KB (two rows of a 2 KB
// strip), a step of the 4- and 8-bit formats 2 KB, of the bit-plane formats 0.75 to 1.75 KB.  The counts are the fastest
// measured on 7B-shaped layers (eight layers in one launch, us per layer with 2 / 3 / 4 sets: Q4_B64 34.3 / 35.5 / 30.7,
// Q8_B64 46.9 / 44.2 / 44.3, Q6_B64 44.2 / 45.2 / 47.4, Q5_B64 43.5 / 35.4 / 46.5, Q3_B32 42.7 / 43.8 / 35.6, Q2_B32 23.5 / 34.9 /
// 36.0; the padding of a phase's steps to whole rounds is part of what they measure).  IFLOW_CHAIN_SETS_OTHER overrides
// them all (measurement builds).
constexpr int chain_sets(int format, bool attn = false)
{
#ifdef IFLOW_CHAIN_SETS_ATTN
    if (attn && format == IFLOW_Q3H_B64) return IFLOW_CHAIN_SETS_ATTN;
#endif
#ifdef IFLOW_CHAIN_SETS_OTHER
    return format == IFLOW_Q3H_B64 ? CHAIN_SETS : IFLOW_CHAIN_SETS_OTHER;
#else
    return format == IFLOW_Q3H_B64 ? CHAIN_SETS : (format == IFLOW_Q6_B64 || format == IFLOW_Q2_B32) ? 2 : format == IFLOW_Q5_B64 ? 3 : 4;
#endif
}

// The sums over all 64 lanes of two per-lane values, in the summation tree of wave_sum_to_lane63 (lanes ^1, ^2, the halves
// and the mirror of a 16-lane row, rows 0+1 and 2+3, then the two halves), so the results are bit-identical to two
// separate reductions: the four row totals of a and of b are brought side by side with one swap of the upper half of one
// register with the lower half of the other, after which both values finish in the same two instructions.  Lane 31 of the
// result holds the sum of a, lane 63 the sum of b.
__device__ __forceinline__ int pair_sums(float a, float b)
{
    a = row16_sum(a);
    b = row16_sum(b);
    // a <- rows (a0, a1, b0, b1), b <- rows (a2, a3, b2, b3); then rows 1 and 3 += lane 15 of the row before.  (Written
    // as instructions: this compiler's builtin for the swap loses its second result.  The idle cycles are what a
    // cross-lane read of a register written by the instruction before needs.)
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1\n\t"
                 "v_add_f32_dpp %0, %0, %0 row_bcast:15 row_mask:0xa bank_mask:0xf\n\t"
                 "v_add_f32_dpp %1, %1, %1 row_bcast:15 row_mask:0xa bank_mask:0xf\n\ts_nop 0" : "+v"(a), "+v"(b));
    const float lo = a, hi = b;
    return __builtin_bit_cast(int, hi + lo);
}

// lane `slot` of keep0 / keep1 <- value0 / value1 (all three uniform).  The lane select goes through m0: a lane write may
// name only one ordinary scalar register.
__device__ __forceinline__ void park(float &keep0, float &keep1, int value0, int value1, int slot)
{
    asm volatile("s_mov_b32 m0, %4\n\ts_nop 0\n\tv_writelane_b32 %0, %2, m0\n\tv_writelane_b32 %1, %3, m0"
                 : "+v"(keep0), "+v"(keep1) : "s"(value0), "s"(value1), "s"(slot) : "m0");
}

// ---- decode attention inside the launch ------------------------------------------------------------------------------------
typedef uint32_t attn_u32x4 __attribute__((ext_vector_type(4)));

// Two pairs of fp16 values (elements `element`, `element` + 1 and `partner`, `partner` + 1, both even) of a vector that is
// either an input of the launch (plain) or the tagged output of an earlier product; a tagged read repeats until all four
// carry the launch's tag (both pairs in the same pass: one memory latency).
__device__ __forceinline__ void chain_read_pairs(const uint16_t *plain, const uint32_t *ws, int tag_word, int element, int partner, uint32_t tag,
                                                 bool &failed, uint32_t &own, uint32_t &other)
{
    if (plain != nullptr) {
        own = *global_ptr<const uint32_t>(plain + element);
        other = *global_ptr<const uint32_t>(plain + partner);
        return;
    }
    // pair g of the vector sits at 8-byte word (g >> 11) * 2048 + (g & 7) * 256 + ((g >> 3) & 255)
    const uint64_t *base = reinterpret_cast<const uint64_t *>(ws + tag_word);
    const int g0 = element >> 1, g1 = partner >> 1;
    const uint64_t *src0 = base + (g0 >> 11) * 2048 + (g0 & 7) * 256 + ((g0 >> 3) & 255);
    const uint64_t *src1 = base + (g1 >> 11) * 2048 + (g1 & 7) * 256 + ((g1 >> 3) & 255);
    int budget = failed ? 1 : CHAIN_POLL_BUDGET;
    for (;;) {
        const uint64_t w0 = __hip_atomic_load(src0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint64_t w1 = __hip_atomic_load(src1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const uint32_t lo0 = (uint32_t)w0, hi0 = (uint32_t)(w0 >> 32), lo1 = (uint32_t)w1, hi1 = (uint32_t)(w1 >> 32);
        own = (lo0 & 0xFFFFu) | (hi0 << 16);
        other = (lo1 & 0xFFFFu) | (hi1 << 16);
        const bool ok = (((lo0 ^ tag) | (hi0 ^ tag) | (lo1 ^ tag) | (hi1 ^ tag)) >> 16) == 0;
        if (__builtin_amdgcn_ballot_w64(!ok) == 0) break;
        if (--budget <= 0) {
            failed = true;
            __hip_atomic_store(const_cast<uint32_t *>(ws) + CHAIN_WS_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
        }
        __builtin_amdgcn_s_sleep(CHAIN_POLL_SLEEP);
    }
}

// Rotary embedding of components c, c + 1 (c even) of a 128-component head (`own`), given the components the pairing joins
// them with (`other`: c +- 64, c +- 64 + 1 for the pairing by halves; unused for adjacent pairs).  table[i] = (cos, sin) of
// pair i's angle at this step's position.  fp64 arithmetic, one rounding to fp16: the values iflow_rope_append writes.
__device__ __forceinline__ uint32_t chain_rope_pair(uint32_t own, uint32_t other, int c, int pairing, const double2 *table)
{
    const half2_t a = as_h2(own), b = as_h2(other);
    const double ax = (double)(float)a.x, ay = (double)(float)a.y, bx = (double)(float)b.x, by = (double)(float)b.y;
    double lo, hi;
    if (pairing == IFLOW_ROPE_HALVES) {                     // component c pairs with c + 64; the pair's index is c mod 64
        const double2 t0 = table[c & 63], t1 = table[(c + 1) & 63];
        if (c < 64) { lo = ax * t0.x - bx * t0.y; hi = ay * t1.x - by * t1.y; }       // (a, b) = (own, partner): first of the pair
        else        { lo = bx * t0.y + ax * t0.x; hi = by * t1.y + ay * t1.x; }       // second of the pair: partner sin + own cos
    } else {                                                // components (c, c + 1) are a pair
        const double2 t = table[c >> 1];
        lo = ax * t.x - ay * t.y;
        hi = ax * t.y + ay * t.x;
    }
    const half2_t rv = {(half_t)lo, (half_t)hi};
    return as_u32(rv);
}

// Phase "part" for R of the query heads of a key/value head's group, heads r0 .. r0 + R - 1 of the group (a group larger than
// two heads takes several passes over its range).  lds: (4 * CHAIN_WAVES_ATTN) * 130 floats for the running states, and behind
// them CHAIN_ATTN_STAGE_BYTES for the step's rotated queries, rotated key and value.
constexpr int CHAIN_ATTN_STATE_BYTES = 4 * CHAIN_WAVES_ATTN * 130 * 4, CHAIN_ATTN_STAGE_BYTES = 64 * 16;
template <int R>
__device__ __forceinline__ void chain_attn_part(const ChainAttn &at, uint32_t *ws, float *lds, const double2 *table, uint32_t tag, int position,
                                                int wg, int wave, int lane, int r0, bool &failed, uint32_t *marks = nullptr)
{
    const int group = at.n_heads / at.n_kv_heads;
    constexpr int NST = 4 * CHAIN_WAVES_ATTN;                       // (the LDS area holds up to this many states of 128 sums; R per wavefront are used)
    const int nsplit = at.nsplit;
    if (wg >= at.n_kv_heads * nsplit) return;                  // (uniform over the workgroup)
    const int j = wg / nsplit, sp = wg - j * nsplit;
    const int seq_len = position + 1;
    const int chunk = ((seq_len + nsplit - 1) / nsplit + 15) & ~15;
    const int t_begin = sp * chunk, t_end = min(seq_len, t_begin + chunk);     // may be empty
    const bool has_new = t_begin <= position && position < t_end;             // this range holds the step's own position
    const int gq = lane >> 4, dseg = lane & 15, c0 = dseg * 8;
    float *s_acc = lds, *s_m = lds + NST * 128, *s_l = s_m + NST;
    attn_u32x4 *const stage = reinterpret_cast<attn_u32x4 *>(reinterpret_cast<uint8_t *>(lds) + CHAIN_ATTN_STATE_BYTES);

    // The wavefront's first block of cached keys and values is requested before anything of this step is waited for: rows
    // below the step's position do not depend on the step.  (Blocks of sixteen positions, wavefront w takes blocks w,
    // w + CHAIN_WAVES_ATTN, ...; four positions per load instruction, one per lane group; positions past the range read its last
    // position (in bounds) and are masked; the step's own position comes from registers: its cache row is being written.)
    const uint8_t *kh = reinterpret_cast<const uint8_t *>(at.k_cache) + (int64_t)j * at.max_seq * 256;     // (uniform; rows of 256 bytes)
    const uint8_t *vh = reinterpret_cast<const uint8_t *>(at.v_cache) + (int64_t)j * at.max_seq * 256;
    constexpr int STEP = 16 * CHAIN_WAVES_ATTN;
    attn_u32x4 kt[4], vt[4];
    auto load_block = [&](int p0) {
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const int pos = min(p0 + t * 4 + gq, t_end - 1);
            const int row = min(pos, has_new && pos == position ? max(position - 1, 0) : pos);   // never the row being written
            const uint32_t off = (uint32_t)row * 256u + (uint32_t)c0 * 2u;                      // (max_seq <= 2^20: below 2^28)
            kt[t] = __builtin_nontemporal_load(global_ptr<const attn_u32x4>(kh + off));
            vt[t] = __builtin_nontemporal_load(global_ptr<const attn_u32x4>(vh + off));
        }
    };
    const int p_first = t_begin + wave * 16;
    if (p_first < t_end) load_block(p_first);

    // The step's vectors, one pair of components per thread: thread u < 64 R has a pair of the group's queries (rotated), the
    // next 64 threads the key of this head (rotated), the last 64 its value; they go to LDS for everybody, and the key and
    // value also into the caches (by the workgroup whose range holds the step's position, on its first pass).
    {
        const int u = wave * 64 + lane, nq = 64 * R;
        if (u < nq + (has_new ? 128 : 0)) {
            const bool is_q = u < nq, is_v = u >= nq + 64;
            const int c = (u & 63) * 2;                        // the pair's first component
            const uint16_t *plain = is_q ? at.q : (is_v ? at.v_new : at.k_new);
            const int tag_word = is_q ? at.q_tag_word : (is_v ? at.v_tag_word : at.k_tag_word);
            const int e = is_q ? (j * group + r0 + (u >> 6)) * 128 : j * 128;     // the head's first element
            uint32_t val, oth;                                 // (the partner of the pairing by halves; else the pair itself again)
            chain_read_pairs(plain, ws, tag_word, e + c, e + (at.pairing == IFLOW_ROPE_HALVES && !is_v ? (c ^ 64) : c), tag, failed, val, oth);
#if IFLOW_CHAIN_TRACE
            if (marks && u == 0) marks[5] = (uint32_t)__builtin_amdgcn_s_memrealtime();     // wavefront 0 has read its pairs
#endif
            if (!is_v) val = chain_rope_pair(val, oth, c, at.pairing, table);
#if IFLOW_CHAIN_TRACE
            if (marks && u == 0) marks[6] = (uint32_t)__builtin_amdgcn_s_memrealtime();     // ... and rotated them
#endif
            reinterpret_cast<uint32_t *>(stage)[u] = val;
            if (!is_q && r0 == 0) {
                uint16_t *cache = is_v ? at.v_cache : at.k_cache;
                *global_ptr<uint32_t>(cache + ((int64_t)j * at.max_seq + position) * 128 + c) = val;
            }
        }
    }
    __syncthreads();
#if IFLOW_CHAIN_TRACE
    if (marks && wave == 0 && lane == 0) marks[1] = (uint32_t)__builtin_amdgcn_s_memrealtime();   // the step's vectors are staged
#endif
    half2_t qr[R][4];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const attn_u32x4 rot = stage[r * 16 + dseg];
        qr[r][0] = as_h2(rot.x); qr[r][1] = as_h2(rot.y); qr[r][2] = as_h2(rot.z); qr[r][3] = as_h2(rot.w);
    }
    attn_u32x4 k_now = {0u, 0u, 0u, 0u}, v_now = {0u, 0u, 0u, 0u};
    if (has_new) { k_now = stage[16 * R + dseg]; v_now = stage[16 * R + 16 + dseg]; }

    float m[R], l[R], acc[R][8];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        m[r] = -INFINITY; l[r] = 0.f;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[r][e] = 0.f;
    }
    for (int p0 = p_first; p0 < t_end; p0 += STEP) {
        if (p0 != p_first) load_block(p0);
#pragma unroll
        for (int t = 0; t < 4; ++t) {                          // (selects, not stores under a branch: those put the arrays into scratch memory)
            const bool now = min(p0 + t * 4 + gq, t_end - 1) == position;
            kt[t].x = now ? k_now.x : kt[t].x; kt[t].y = now ? k_now.y : kt[t].y; kt[t].z = now ? k_now.z : kt[t].z; kt[t].w = now ? k_now.w : kt[t].w;
            vt[t].x = now ? v_now.x : vt[t].x; vt[t].y = now ? v_now.y : vt[t].y; vt[t].z = now ? v_now.z : vt[t].z; vt[t].w = now ? v_now.w : vt[t].w;
        }
        // scores of the four positions for every head, the running maxima brought up to date; then the values, one position
        // at a time (converted once for all heads)
        float sc[R][4], base[R];
#pragma unroll
        for (int r = 0; r < R; ++r) {
            float bm = -INFINITY;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                float d = __builtin_amdgcn_fdot2(qr[r][0], as_h2(kt[t].x), 0.f, false);
                d = __builtin_amdgcn_fdot2(qr[r][1], as_h2(kt[t].y), d, false);
                d = __builtin_amdgcn_fdot2(qr[r][2], as_h2(kt[t].z), d, false);
                d = __builtin_amdgcn_fdot2(qr[r][3], as_h2(kt[t].w), d, false);
                d = row16_sum(d) * at.scale_log2e;
                sc[r][t] = (p0 + t * 4 + gq < t_end) ? d : -INFINITY;
                bm = fmaxf(bm, sc[r][t]);
            }
            const float m_new = fmaxf(m[r], bm);
            const float alpha = (m_new == -INFINITY) ? 1.0f : __builtin_amdgcn_exp2f(m[r] - m_new);
            base[r] = (m_new == -INFINITY) ? 0.f : m_new;
            l[r] *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] *= alpha;
            m[r] = m_new;
        }
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            const half2_t a = as_h2(vt[t].x), b = as_h2(vt[t].y), c = as_h2(vt[t].z), d = as_h2(vt[t].w);
            const float vf[8] = {(float)a.x, (float)a.y, (float)b.x, (float)b.y, (float)c.x, (float)c.y, (float)d.x, (float)d.y};
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const float pr = __builtin_amdgcn_exp2f(sc[r][t] - base[r]);
                l[r] += pr;
#pragma unroll
                for (int e = 0; e < 8; ++e) acc[r][e] = __builtin_fmaf(pr, vf[e], acc[r][e]);
            }
        }
    }
#if IFLOW_CHAIN_TRACE
    if (marks && wave == 0 && lane == 0) marks[2] = (uint32_t)__builtin_amdgcn_s_memrealtime();   // wavefront 0's positions are done
#endif
    // The four lane groups of a wavefront hold states of different positions for the same components: merged across lanes
    // first (lanes 16 and 32 apart; both lanes of a pair compute the same), so that a wavefront leaves one state per head.
#pragma unroll
    for (int r = 0; r < R; ++r) {
#pragma unroll
        for (int d = 16; d <= 32; d *= 2) {
            const float m2 = __shfl_xor(m[r], d), l2 = __shfl_xor(l[r], d);
            const float mx = fmaxf(m[r], m2);
            const bool none = mx == -INFINITY;                 // (neither has seen a position: sums are zero)
            const float f1 = none ? 1.0f : __builtin_amdgcn_exp2f(m[r] - mx), f2 = none ? 1.0f : __builtin_amdgcn_exp2f(m2 - mx);
            l[r] = l[r] * f1 + l2 * f2;
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[r][e] = acc[r][e] * f1 + __shfl_xor(acc[r][e], d) * f2;
            m[r] = mx;
        }
    }
    // the wavefronts' states of each head -> one partial state in the workspace (64-bit words: fp32 bits, launch tag);
    // threads 128 r .. 128 r + 127 merge head r
    const int tid = wave * 64 + lane;
    uint64_t *part = reinterpret_cast<uint64_t *>(ws + at.part_word);
    if (gq == 0) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
#pragma unroll
            for (int e = 0; e < 8; ++e) s_acc[(r * CHAIN_WAVES_ATTN + wave) * 128 + c0 + e] = acc[r][e];
            if (dseg == 0) { s_m[r * CHAIN_WAVES_ATTN + wave] = m[r]; s_l[r * CHAIN_WAVES_ATTN + wave] = l[r]; }
        }
    }
    __syncthreads();
    if (tid < 128 * R) {
        const int r = tid >> 7, c = tid & 127;
        const float *sm = s_m + r * CHAIN_WAVES_ATTN, *sl = s_l + r * CHAIN_WAVES_ATTN, *sa = s_acc + r * CHAIN_WAVES_ATTN * 128 + c;
        float M = sm[0];
#pragma unroll
        for (int i = 1; i < CHAIN_WAVES_ATTN; ++i) M = fmaxf(M, sm[i]);
        float L = 0.f, O = 0.f;
        if (M != -INFINITY) {                                  // (an empty range leaves maximum -inf, sums zero)
#pragma unroll
            for (int i = 0; i < CHAIN_WAVES_ATTN; ++i) {
                const float f = __builtin_amdgcn_exp2f(sm[i] - M);
                L = __builtin_fmaf(sl[i], f, L);
                O = __builtin_fmaf(sa[i * 128], f, O);
            }
        }
        uint64_t *dst = part + ((int64_t)(j * group + r0 + r) * nsplit + sp) * 130;
        const uint64_t hi = (uint64_t)tag << 32;
        __hip_atomic_store(dst + c, hi | __builtin_bit_cast(uint32_t, O), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (c == 0) {
            __hip_atomic_store(dst + 128, hi | __builtin_bit_cast(uint32_t, M), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(dst + 129, hi | __builtin_bit_cast(uint32_t, L), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
    }
    __syncthreads();                                           // the states in LDS are no longer needed
}

// Phase "merge": a workgroup takes a contiguous piece of the n_heads * 128 outputs (head, component).  One thread per (range,
// output) reads that range's partial state (re-reading until it carries the launch's tag) and leaves it in LDS - all ranges at
// once, one memory latency - then one thread per output merges the ranges in order and publishes the output: the plain fp16
// value and the tagged word a later phase stages from.  lds: nsplit * per_wg * 3 floats.
__device__ __forceinline__ int chain_attn_merge_per_wg(int n_heads, int nwg)
{
    return ((n_heads * 128 + nwg - 1) / nwg + 1) & ~1;       // (even, so that a workgroup writes whole pairs)
}
__device__ __forceinline__ void chain_attn_merge(const ChainAttn &at, uint32_t *ws, float *lds, uint32_t tag, int wg, int nwg, int tid, bool &failed)
{
    const int total = at.n_heads * 128;
    const int per_wg = chain_attn_merge_per_wg(at.n_heads, nwg);
    const int o_base = wg * per_wg, n_here = min(per_wg, total - o_base);
    if (n_here <= 0) return;                                   // (uniform over the workgroup)
    const uint64_t *parts = reinterpret_cast<const uint64_t *>(ws + at.part_word);
    const int nsplit = at.nsplit;
    for (int idx = tid; idx < nsplit * n_here; idx += 64 * CHAIN_WAVES_ATTN) {
        const int i = idx / n_here, ol = idx - i * n_here, o = o_base + ol;
        const uint64_t *src = parts + ((int64_t)(o >> 7) * nsplit + i) * 130;
        uint64_t wo, wm, wl;
        int budget = failed ? 1 : CHAIN_POLL_BUDGET;
        for (;;) {
            wo = __hip_atomic_load(src + (o & 127), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            wm = __hip_atomic_load(src + 128, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            wl = __hip_atomic_load(src + 129, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((uint32_t)(wo >> 32) == tag && (uint32_t)(wm >> 32) == tag && (uint32_t)(wl >> 32) == tag) break;
            if (--budget <= 0) {
                failed = true;
                __hip_atomic_store(ws + CHAIN_WS_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                break;
            }
            __builtin_amdgcn_s_sleep(CHAIN_POLL_SLEEP);
        }
        float *dst = lds + (i * per_wg + ol) * 3;
        dst[0] = __builtin_bit_cast(float, (uint32_t)wo);
        dst[1] = __builtin_bit_cast(float, (uint32_t)wm);
        dst[2] = __builtin_bit_cast(float, (uint32_t)wl);
    }
    __syncthreads();
    if (tid < n_here) {
        float M = -INFINITY, L = 0.f, O = 0.f;
        for (int i = 0; i < nsplit; ++i) {
            const float *st = lds + (i * per_wg + tid) * 3;
            const float oi = st[0], mi = st[1], li = st[2];
            const float m_new = fmaxf(M, mi);
            if (m_new != -INFINITY) {                          // (ranges in order: the first non-empty one sets the maximum)
                const float keep = __builtin_amdgcn_exp2f(M - m_new), f = __builtin_amdgcn_exp2f(mi - m_new);
                L = L * keep + li * f;
                O = O * keep + oi * f;
                M = m_new;
            }
        }
        const int o = o_base + tid;
        const uint32_t h = as_u16((half_t)(O / L));
        *global_ptr<uint16_t>(at.out + o) = (uint16_t)h;
        __hip_atomic_store(ws + at.out_tag_word + chain_tag_word(o), h | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();                                           // the states in LDS are no longer needed
}

// ATTN: the fused variant that also knows the two attention phases (a launch without them runs the code without them: the
// attention's registers would otherwise cost every fused launch spills around those phases).
template <int S, bool FUSED, int F, bool ATTN>
__global__ __launch_bounds__(64 * chain_waves(ATTN)) void chain_kernel(const uint8_t *__restrict__ plan, uint32_t *__restrict__ ws, int position)
{
    constexpr bool EARLY = IFLOW_CHAIN_EARLY != 0;
    constexpr int CHAIN_WAVES = chain_waves(ATTN);             // wavefronts of this workgroup
    constexpr int CHAIN_STRIDE = 2 * CHAIN_WAVES;              // a wavefront takes two rows per step: rows between its steps
    using T = Fmt<F>;
    constexpr int KIND = T::kind;
    using G = Geo<KIND>;
    constexpr bool Q3H = KIND == KIND_Q3H;
    constexpr bool PLANES = kind_has_planes(KIND);             // 6-, 5-, 3-, 2-bit: a low and (but for 2-bit) a high plane, then the headers
    constexpr int WA = Planes<KIND>::WA, WB = Planes<KIND>::WB;
    constexpr int LANE_BYTES = PLANES ? 4 * WA : 16;           // code bytes per lane, row and strip (bit planes: of the low plane)
    constexpr int LANE_BYTES_HI = 4 * WB;                      // ... of the high plane
    constexpr int XQ = G::XD / 4;                              // 16-byte quarters of a lane's staged activations
    constexpr int CHAIN_SLOT_BYTES = chain_slot_bytes<KIND>();
    constexpr int STRIP_COLS = chain_strip_cols<KIND>();
    constexpr int ROW_BITS = Q3H ? 4 : (PLANES ? WA : (KIND == KIND_Q4 ? 4 : 8));  // code bits per weight in a row's (first) code stream (Q3H: the whole block)
    constexpr int HDR_PER_STRIP = STRIP_COLS / T::block;       // block headers per strip (formats with headers behind the codes)
    const ChainHeader *const hd = reinterpret_cast<const ChainHeader *>(plan);
    const ChainArgs a = {reinterpret_cast<const ChainPhase *>(plan + sizeof(ChainHeader)),
                         reinterpret_cast<const ChainMatrix *>(plan + sizeof(ChainHeader) + (size_t)hd->nphases * sizeof(ChainPhase)),
                         reinterpret_cast<const ChainPhaseOps *>(plan + sizeof(ChainHeader) + (size_t)hd->nphases * sizeof(ChainPhase) +
                                                                 (size_t)hd->nmatrices * sizeof(ChainMatrix)),
                         reinterpret_cast<const ChainAttn *>(plan + sizeof(ChainHeader) + (size_t)hd->nphases * (sizeof(ChainPhase) + sizeof(ChainPhaseOps)) +
                                                             (size_t)hd->nmatrices * sizeof(ChainMatrix))};
    extern __shared__ __align__(16) uint8_t xs[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = IFLOW_UNI(tid >> 6);
    const int wg = blockIdx.x;
    const int nphases = hd->nphases;
    // Clock stamps of the launch, left in the workspace header by the first workgroup when it starts and when it ends: the
    // shader clock counter and the constant 100 MHz counter, low words.  Their ratio is the clock the launch really ran at,
    // which on a power-limited part is the first thing to know about a launch's duration.
    if (wg == 0 && tid == 0) {
        ws[CHAIN_WS_CLOCKS] = (uint32_t)__builtin_amdgcn_s_memtime();
        ws[CHAIN_WS_CLOCKS + 1] = (uint32_t)__builtin_amdgcn_s_memrealtime();
    }

    // A wavefront handles two adjacent rows (2i, 2i+1 of a matrix) per step, so "row" below means such a pair, named
    // by its even row; in a phase's row space every matrix starts at an even row (odd matrices are padded by one).
    // pairs of this wavefront in a phase: first row of the workgroup, number of pairs of the wavefront
    auto phase_rows = [&](int rows_per_wg, int total, int &rbeg, int &nrows) __attribute__((always_inline)) {
        rbeg = wg * rows_per_wg;
        const int rend = min(rbeg + rows_per_wg, total);
        nrows = max(0, (rend - rbeg - 2 * wave + CHAIN_STRIDE - 1) / CHAIN_STRIDE);
    };
    // the segment that starts at row k.R of phase k.p (k.rows_left > 0): its matrix, the row inside it, its length;
    // `single`: the segment is the lone last row of a matrix with an odd number of rows (always a segment of its own)
    auto walk_segment = [&](ChainWalk &k, int &m, int &r, bool &single) __attribute__((always_inline)) {
        const ChainPhase &ph = a.ph[k.p];
        m = ph.first + (k.R >= ph.mstart[1]) + (k.R >= ph.mstart[2]) + (k.R >= ph.mstart[3]);
        r = k.R - a.mat[m].start;
        const int rows_m = a.mat[m].rows;
        int n = min(k.rows_left, min((rows_m - r + CHAIN_STRIDE - 1) / CHAIN_STRIDE,
                                     (4096 - (r & 4095) + CHAIN_STRIDE - 1) / CHAIN_STRIDE));
        const bool tail = r + (n - 1) * CHAIN_STRIDE == rows_m - 1;     // the segment would end in the lone row
        single = tail && n == 1;
        if (tail && n > 1) n -= 1;
        k.seg_left = n; k.rows_left -= n; k.R += n * CHAIN_STRIDE;
    };

    // ---- requests ------------------------------------------------------------------------------------------------
    // A wavefront's steps of all phases form one sequence, and step k of it lives in register set k mod S: the requests
    // run S steps ahead of the decode across phase boundaries, and the sets are refilled in the order in which they are
    // decoded.  The two loads of a row are issued unconditionally (an empty step's lanes all read the first 16 bytes of the
    // workspace): with the same number of loads on every path the compiler can tell exactly how many younger loads may
    // still be in flight when a register set is decoded, instead of waiting for all.
    // PAD: a wavefront's steps per phase are padded to a multiple of S with empty steps, so that every phase starts at set 0
    // and the step loop is S steps unrolled once.  Without it every set always holds a step that will be used, a phase
    // starts at whatever set the sequence has reached, and the step exists in more copies (below).  Which is faster is
    // measured, per format: with two sets of 4 KB (3.5-bit) no padding is 3.5 % faster on 7B-shaped layers; with four sets
    // of 2 KB (4- and 8-bit) padding is 4-7 % faster - the empty sets at the head of a short phase are weights that are not
    // queued in front of the reads of the phase's activations.
    constexpr bool PAD = !Q3H;
    ChainWalk q = {-1, 0, 0, 0};
    const uint8_t *q_wptr = reinterpret_cast<const uint8_t *>(ws);     // weights of the step under the cursor
    int q_lt = 0, q_last = 0;                                  // its strip; the last strip of a row
    int q_nlast16 = 0;                                         // 16 x the blocks in that last strip (offset of its second plane)
    [[maybe_unused]] int q_pad = 0;                            // PAD: empty steps still owed by phase q.p
    int q_rowjump = 0;                                         // from the last strip of a row to the wavefront's next row, bytes
    std::conditional_t<FUSED, int64_t, int> q_row1 = 0;        // from the first to the second row of the pair, bytes (0: no second row)
    uint32_t q_voff_last = 0;                                  // per-lane offset inside the last (ragged) strip of a row
    const uint32_t voff_full = (uint32_t)lane * (Q3H ? 16 : LANE_BYTES);
    // formats whose block headers sit behind the codes: the same walk over the headers (4 bytes per block)
    const uint8_t *q_hptr = reinterpret_cast<const uint8_t *>(ws);
    int q_hrowjump = 0;
    std::conditional_t<FUSED, int64_t, int> q_hrow1 = 0;
    uint32_t q_hoff_last = 0;
    const uint32_t hoff_full = (uint32_t)(lane * G::WPL / T::block) * 4;
    // bit-plane formats: and over the high plane
    const uint8_t *q_pptr = reinterpret_cast<const uint8_t *>(ws);
    int q_prowjump = 0;
    std::conditional_t<FUSED, int64_t, int> q_prow1 = 0;
    uint32_t q_poff_last = 0;
    const uint32_t poff_full = (uint32_t)lane * LANE_BYTES_HI;
    auto request_empty = [&](int count) __attribute__((always_inline)) {                      // `count` empty steps: one "row" of one empty strip each
        q_wptr = reinterpret_cast<const uint8_t *>(ws);
        q_last = 0; q_nlast16 = 0; q_rowjump = 0; q_row1 = 0; q_voff_last = 0;
        q_hptr = q_wptr; q_hrowjump = 0; q_hrow1 = 0; q_hoff_last = 0;
        q_pptr = q_wptr; q_prowjump = 0; q_prow1 = 0; q_poff_last = 0;
        q.seg_left = count;
    };
    auto request_segment = [&]() __attribute__((always_inline)) {                             // q.seg_left == 0: find what the requests do next
        bool found = false;
        if constexpr (PAD) {
            if (q.rows_left == 0 && q_pad > 0) {
                request_empty(q_pad);
                q_pad = 0;
                found = true;
            }
        }
        while (!found && q.p < nphases) {
            if (q.rows_left == 0) {                            // the next phase in which this wavefront has rows
                q.p += 1;
                if (q.p < nphases) {
                    int rbeg, n;
                    phase_rows(a.ph[q.p].rows_per_wg, a.ph[q.p].total, rbeg, n);
                    q.rows_left = n; q.R = rbeg + 2 * wave;
                    if constexpr (PAD) {
                        const int real = n * a.ph[q.p].nstrips;
                        q_pad = (real + S - 1) / S * S - real;
                    }
                }
            }
            if (q.p < nphases && q.rows_left > 0) {
                const ChainPhase &ph = a.ph[q.p];
                int m, r;
                bool single;
                walk_segment(q, m, r, single);
                q_last = ph.nstrips - 1;
                if constexpr (Q3H) {
                    const int nlast = ph.nbk - (ph.nstrips - 1) * 64;
                    q_wptr = a.mat[m].packed + (int64_t)r * ((int64_t)ph.nbk * 32);
                    q_nlast16 = nlast * 16;
                    q_rowjump = (CHAIN_STRIDE * ph.nbk - (ph.nstrips - 1) * 64) * 32;
                    q_row1 = single ? 0 : ph.nbk * 32;
                    if constexpr (FUSED) {
                        if (a.mat[m].gated) {                  // rows 2n, 2n+1 of the row space are row n of the gate and of the up matrix
                            q_wptr = a.mat[m].packed + (int64_t)(r >> 1) * ((int64_t)ph.nbk * 32);
                            q_rowjump = ((CHAIN_STRIDE / 2) * ph.nbk - (ph.nstrips - 1) * 64) * 32;
                            q_row1 = a.mat[m].packed2 - a.mat[m].packed;
                        }
                    }
                    q_voff_last = voff_full & mask_lt(lane, nlast);            // lanes past a ragged end redo block 0
                } else {
                    // a row: cols * ROW_BITS / 8 bytes of codes, 64 * LANE_BYTES per strip; its headers: 4 bytes per block, behind
                    // all codes; bit planes: cols * WB / 8 bytes of the high plane between the two
                    const int cols = ph.nbk * T::block;
                    const int row_bytes = cols * ROW_BITS / 8, hrow_bytes = ph.nbk * 4, prow_bytes = cols * WB / 8;
                    const uint8_t *hi_plane = a.mat[m].packed + (int64_t)a.mat[m].hi_off4 * 4;
                    const int nlast = (cols - (ph.nstrips - 1) * STRIP_COLS) / G::WPL;     // lanes of the last strip
                    const uint8_t *headers = a.mat[m].packed + (int64_t)a.mat[m].hdr_off4 * 4;
                    q_wptr = a.mat[m].packed + (int64_t)r * row_bytes;
                    q_hptr = headers + (int64_t)r * hrow_bytes;
                    q_rowjump = CHAIN_STRIDE * row_bytes - (ph.nstrips - 1) * 64 * LANE_BYTES;
                    q_hrowjump = CHAIN_STRIDE * hrow_bytes - (ph.nstrips - 1) * HDR_PER_STRIP * 4;
                    q_row1 = single ? 0 : row_bytes;
                    q_hrow1 = single ? 0 : hrow_bytes;
                    if constexpr (WB > 0) {
                        q_pptr = hi_plane + (int64_t)r * prow_bytes;
                        q_prowjump = CHAIN_STRIDE * prow_bytes - (ph.nstrips - 1) * 64 * LANE_BYTES_HI;
                        q_prow1 = single ? 0 : prow_bytes;
                    }
                    if constexpr (FUSED) {
                        if (a.mat[m].gated) {                  // both matrices have the same shape: one distance for codes and headers
                            q_wptr = a.mat[m].packed + (int64_t)(r >> 1) * row_bytes;
                            q_hptr = headers + (int64_t)(r >> 1) * hrow_bytes;
                            q_rowjump = (CHAIN_STRIDE / 2) * row_bytes - (ph.nstrips - 1) * 64 * LANE_BYTES;
                            q_hrowjump = (CHAIN_STRIDE / 2) * hrow_bytes - (ph.nstrips - 1) * HDR_PER_STRIP * 4;
                            q_row1 = a.mat[m].packed2 - a.mat[m].packed;
                            q_hrow1 = q_row1;
                            if constexpr (WB > 0) {
                                q_pptr = hi_plane + (int64_t)(r >> 1) * prow_bytes;
                                q_prowjump = (CHAIN_STRIDE / 2) * prow_bytes - (ph.nstrips - 1) * 64 * LANE_BYTES_HI;
                                q_prow1 = q_row1;
                            }
                        }
                    }
                    q_voff_last = voff_full & mask_lt(lane, nlast);            // lanes past a ragged end redo lane 0 (their
                    q_hoff_last = hoff_full & mask_lt(lane, nlast);            // staged activations are zero)
                    q_poff_last = poff_full & mask_lt(lane, nlast);
                }
                found = true;
            }
        }
        if (!found) request_empty(0x7FFFFFFF);                 // the walk is over: empty steps from here on
        q_lt = 0;
    };
    auto request = [&](WRegs<KIND> (&w)[2]) __attribute__((always_inline)) {                  // request the step under the cursor, then advance it
        const bool last_strip = q_lt == q_last;
        const uint32_t voff = last_strip ? q_voff_last : voff_full;
        // (pointers that were read from the plan have to be told that they point to global memory: a generic pointer
        // makes flat loads, whose completion cannot be counted, and every wait in the step loop becomes "all")
        if constexpr (IFLOW_CHAIN_ABL == 2) {
#pragma unroll
            for (int i = 0; i < G::WD; ++i) asm volatile("" : "+v"(w[0].d[i]), "+v"(w[1].d[i]));
        } else if constexpr (Q3H) {
            const int plane2 = last_strip ? q_nlast16 : 1024;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const uint8_t *row = q_wptr + (int64_t)u * q_row1;
                const u32x4 c0 = __builtin_nontemporal_load(global_ptr<const u32x4>(row + voff));
                const u32x4 c1 = __builtin_nontemporal_load(global_ptr<const u32x4>(row + plane2 + voff));
                w[u].d[0] = c0.x; w[u].d[1] = c0.y; w[u].d[2] = c0.z; w[u].d[3] = c0.w;
                w[u].d[4] = c1.x; w[u].d[5] = c1.y; w[u].d[6] = c1.z; w[u].d[7] = c1.w;
            }
        } else {
            const uint32_t hoff = last_strip ? q_hoff_last : hoff_full;
            [[maybe_unused]] const uint32_t poff = last_strip ? q_poff_last : poff_full;
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                if constexpr (LANE_BYTES == 16) {
                    const u32x4 c0 = __builtin_nontemporal_load(global_ptr<const u32x4>(q_wptr + (int64_t)u * q_row1 + voff));
                    w[u].d[0] = c0.x; w[u].d[1] = c0.y; w[u].d[2] = c0.z; w[u].d[3] = c0.w;
                } else {                                       // (two-bit low plane: 8 bytes per lane)
                    const u32x2 c0 = __builtin_nontemporal_load(global_ptr<const u32x2>(q_wptr + (int64_t)u * q_row1 + voff));
                    w[u].d[0] = c0.x; w[u].d[1] = c0.y;
                }
                if constexpr (WB == 2) {
                    const u32x2 c1 = __builtin_nontemporal_load(global_ptr<const u32x2>(q_pptr + (int64_t)u * q_prow1 + poff));
                    w[u].d[WA] = c1.x; w[u].d[WA + 1] = c1.y;
                } else if constexpr (WB == 1) {
                    w[u].d[WA] = __builtin_nontemporal_load(global_ptr<const uint32_t>(q_pptr + (int64_t)u * q_prow1 + poff));
                }
                w[u].hdr = *global_ptr<const uint32_t>(q_hptr + (int64_t)u * q_hrow1 + hoff);
            }
            q_hptr += last_strip ? q_hrowjump : HDR_PER_STRIP * 4;
            if constexpr (WB > 0) q_pptr += last_strip ? q_prowjump : 64 * LANE_BYTES_HI;
        }
        q_wptr += last_strip ? q_rowjump : (Q3H ? 2048 : 64 * LANE_BYTES);
        q_lt = last_strip ? 0 : q_lt + 1;
        if (last_strip) {                                      // on to the wavefront's next row
            q.seg_left -= 1;
            if (q.seg_left == 0) request_segment();
        }
    };

    // ---- activations of a phase into LDS, in decode order ---------------------------------------------------
    // Chunk c = (strip ts, block blk, quarter qd), qd fastest: 16 activations that feed decode slots 4qd..4qd+3 of
    // lane blk.  n[k] holds the pair (x[2k], x[2k+1]) of the chunk.
    auto chunk_put = [&](int c, const uint32_t (&n)[8]) {
        const int cc = c & 255, ts = c >> 8, blk = cc >> 2, qd = cc & 3;
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
        uint8_t *sl = xs + (size_t)ts * CHAIN_SLOT_BYTES;
        *reinterpret_cast<uint4 *>(sl + (qd * 64 + blk) * 16) = make_uint4(e[0], e[1], e[2], e[3]);
        *reinterpret_cast<uint4 *>(sl + ((4 + qd) * 64 + blk) * 16) = make_uint4(o[0], o[1], o[2], o[3]);
        float bs = IFLOW_Q3H_BIAS1 * se + IFLOW_Q3H_BIAS2 * so, sx = se + so;
        bs += dpp_f32<0xB1, 0xF>(bs); sx += dpp_f32<0xB1, 0xF>(sx);              // the four quarters of a block
        bs += dpp_f32<0x4E, 0xF>(bs); sx += dpp_f32<0x4E, 0xF>(sx);              // sit in one quad of lanes
        if (qd == 0) *reinterpret_cast<float2 *>(sl + 8 * 64 * 16 + blk * 8) = make_float2(bs, sx);
    };
    // source of a chunk of launch-input activations; chunks past the end of the row read chunk 0 of their strip
    auto chunk_src = [&](const uint16_t *x, int c, int nbk) {
        const int cc = c & 255, ts = c >> 8;
        const int n_t = min(64, nbk - ts * 64);
        const int ccl = cc & (int)mask_lt(cc >> 2, n_t);
        return global_ptr<const u32x4>(x + (int64_t)ts * 4096 + ccl * 16);
    };
    auto chunk_live = [&](int c, int nbk) { return mask_lt((c & 255) >> 2, min(64, nbk - (c >> 8) * 64)); };
    // rms normalization, first half: v_k = fp16(x_k g_k) goes to LDS, x_k^2 is summed; the scalar 1 / sqrt(mean + eps)
    // commutes with the product and is applied to the row sums
    float sumsq = 0.f;
    auto apply_gain = [&](uint32_t (&n)[8], const u32x4 g0, const u32x4 g1) {
        const uint32_t g[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            sumsq = dot2(as_h2(n[i]), as_h2(n[i]), sumsq);
            n[i] = as_u32(as_h2(n[i]) * as_h2(g[i]));          // an exact product rounded once (packed fp16 multiply)
        }
    };
    auto put_plain = [&](int c, int nbk, const u32x4 q0, const u32x4 q1, const ChainPhaseOps *op) {
        const uint32_t live = chunk_live(c, nbk);              // columns past the end of the row count as zero
        uint32_t n[8] = {q0.x & live, q0.y & live, q0.z & live, q0.w & live, q1.x & live, q1.y & live, q1.z & live, q1.w & live};
        if constexpr (FUSED) {
            if (op->x_op == IFLOW_X_RMS_GAIN) {
                const IFLOW_GLOBAL u32x4 *gs = chunk_src(op->aux, c, nbk);
                apply_gain(n, gs[0], gs[1]);
            }
        }
        chunk_put(c, n);
    };
    // ---- the same for the formats with 16 bytes of codes per lane: thread c stages the activations of lane c % 64 of strip
    // c / 64, G::WPL consecutive values, arranged by the format's own arrange_x (the single-product kernels' layout)
    auto slot_put = [&](int c, uint32_t (&n)[G::XD], const ChainPhaseOps *op, const uint16_t *gains_at) {
        if constexpr (FUSED) {
            if (op->x_op == IFLOW_X_RMS_GAIN) {
#pragma unroll
                for (int j = 0; j < XQ; ++j) {
                    const u32x4 g = global_ptr<const u32x4>(gains_at)[j];
                    const uint32_t gv[4] = {g.x, g.y, g.z, g.w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        sumsq = dot2(as_h2(n[4 * j + e]), as_h2(n[4 * j + e]), sumsq);
                        n[4 * j + e] = as_u32(as_h2(n[4 * j + e]) * as_h2(gv[e]));   // an exact product rounded once
                    }
                }
            }
        }
        XRegs<KIND> t;
        arrange_x<KIND>(t, n);
        uint8_t *sl = xs + (size_t)(c >> 6) * CHAIN_SLOT_BYTES;
        const int l = c & 63;
#pragma unroll
        for (int j = 0; j < XQ; ++j)
            *reinterpret_cast<uint4 *>(sl + (j * 64 + l) * 16) = make_uint4(as_u32(t.v[4 * j]), as_u32(t.v[4 * j + 1]), as_u32(t.v[4 * j + 2]), as_u32(t.v[4 * j + 3]));
        *reinterpret_cast<float2 *>(sl + XQ * 64 * 16 + l * 8) = make_float2(t.bias_sum, t.x_sum);
    };

    // The first phase's activations are an input of the launch.  Their first chunk is requested BEFORE any weights,
    // because memory requests of a wavefront are served in order and the whole workgroup waits for the staged
    // activations; then S steps of weights; then the chunk is put in place.
    WRegs<KIND> w[S][2];
    // The launch count, the oldest load of the wavefront (so it never has to be waited for alone): every workgroup keeps its
    // own copy in the workspace header and advances it when it is done, so all copies read the same at the start of a launch
    // and nobody has to wait for anybody at the end of one.  A plain cached load: the word was last written by the previous
    // launch (the plan call zeroes them all).
    const uint32_t counter = __hip_atomic_load(ws + CHAIN_WS_SEEN + wg, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if constexpr (!Q3H) {                                      // (these formats stage the first phase like any other, below)
        request_segment();
#pragma unroll
        for (int j = 0; j < S - (EARLY ? 1 : 0); ++j) request(w[j]);
    } else {
        const ChainPhase ph0 = a.ph[0];
        const bool wg_has0 = wg * ph0.rows_per_wg < ph0.total;
        const int nchunks0 = wg_has0 ? ph0.nstrips * 256 : 0;
        const IFLOW_GLOBAL u32x4 *src0 = chunk_src(ph0.x, tid & (int)mask_lt(tid, nchunks0), ph0.nbk);   // threads without a chunk read chunk 0
        const u32x4 xq0 = src0[0], xq1 = src0[1];
        request_segment();
#pragma unroll
        for (int j = 0; j < S - (EARLY ? 1 : 0); ++j) request(w[j]);
        // (whole wavefronts have a chunk or not: loop bounds and conditions are written on the wavefront's first chunk)
        if (wave * 64 < nchunks0) put_plain(tid, ph0.nbk, xq0, xq1, a.ops);
#pragma unroll 1
        for (int cw = wave * 64 + 64 * CHAIN_WAVES; cw < nchunks0; cw += 64 * CHAIN_WAVES) {
            const IFLOW_GLOBAL u32x4 *src = chunk_src(ph0.x, cw + lane, ph0.nbk);
            put_plain(cw + lane, ph0.nbk, src[0], src[1], a.ops);
        }
    }
    // Every wavefront of the launch reads the same count and tags its outputs with it, 1..65535; 0 marks a word that was
    // never written.
    const uint32_t tag = (counter % 65535u + 1u) << 16;

#if IFLOW_CHAIN_TRACE
    // (development aid, off in the library: per-workgroup time stamps of a launch, 16 words per workgroup and phase, written to
    // the buffer whose address sits at byte 48 of the plan)
    uint32_t *const trace = *reinterpret_cast<uint32_t *const *>(plan + 48);
#define CHAIN_MARK(p, k) do { if (trace && lane == 0) trace[((size_t)wg * nphases + (p)) * 16 + (k)] = (uint32_t)__builtin_amdgcn_s_memrealtime(); } while (0)
#else
#define CHAIN_MARK(p, k) do { } while (0)
#endif
    bool failed = false;
    int cs = 0;                                                // this wavefront's steps so far, mod S: the register set of its next step
    XRegs<KIND> xr[1];
    [[maybe_unused]] const Q3HConsts q3h_k = q3h_consts();       // (made once: inside the step loop they would be made again per row)
    // Results are not stored row by row: lane 63's sums of the wavefront's i-th pair of rows are parked in lane i of two
    // registers, and when the phase's steps are done lanes 0..n-1 store them all at once - two store instructions
    // per wavefront and phase instead of two per row (in-order completion means every later load of the wavefront would
    // otherwise queue behind a write-through store), and no output pointers to advance inside the step loop.
    // (with attention in the plan: the rotary embedding's cosines and sines at this step's position, pair i of a 128-component
    // head turning by position * base^(-2i/128), computed once per workgroup in fp64 and kept in LDS behind everything else)
    double2 *const rope_table = reinterpret_cast<double2 *>(xs + hd->lds_bytes - 1024);
    if constexpr (ATTN) {
        static_assert(FUSED, "the attention phases belong to the fused variant");
        if (hd->nattn > 0 && wave == 0) {
            const double angle = (double)position * exp2(-(2.0 * lane / 128.0) * a.attn[0].log2_base);
            double sn, cs;
            sincos(angle, &sn, &cs);
            rope_table[lane] = make_double2(cs, sn);
        }
    }
    for (int p = 0; p < nphases; ++p) {
        const ChainPhase ph = a.ph[p];
        if constexpr (ATTN) {
            if (ph.kind != 0) {                                // a half of a decode attention: every workgroup takes part
                const ChainAttn &at = a.attn[ph.attn];          // (read where it is: a copy would live in scratch memory)
                __syncthreads();                               // (the table; LDS of the phase before is free)
                // (both halves in one pass of this loop: phase p + 1 is this attention's second half, by the plan's construction)
                float *const scratch = reinterpret_cast<float *>(xs);
                const int group = at.n_heads / at.n_kv_heads;
#if IFLOW_CHAIN_TRACE
                uint32_t *const marks = trace ? trace + ((size_t)wg * nphases + p) * 16 : nullptr;
                if (marks && tid == 0) marks[0] = (uint32_t)__builtin_amdgcn_s_memrealtime();
#else
                uint32_t *const marks = nullptr;
#endif
                if (group == 1) {
                    chain_attn_part<1>(at, ws, scratch, rope_table, tag, position, wg, wave, lane, 0, failed, marks);
                } else {                                       // (even by the plan's check)
#pragma unroll 1
                    for (int r0 = 0; r0 < group; r0 += 2)
                        chain_attn_part<2>(at, ws, scratch, rope_table, tag, position, wg, wave, lane, r0, failed);
                }
                CHAIN_MARK(p, 3 + (wave == 0 ? 0 : 8));           // (wavefront 0: slot 3) the partial states are written
                chain_attn_merge(at, ws, scratch, tag, wg, (int)gridDim.x, tid, failed);
                CHAIN_MARK(p, 4 + (wave == 0 ? 0 : 8));           // the workgroup's outputs are published
                p += 1;
                continue;
            }
        }
        const int nbk = ph.nbk, nstrips = ph.nstrips;
        int rbeg, n;                                           // first row of the workgroup, rows of this wavefront
        phase_rows(ph.rows_per_wg, ph.total, rbeg, n);
        if (rbeg < ph.total) {                                 // else: no rows for this workgroup (uniform over the workgroup)
            // 0. where this wavefront's outputs go, lane i for its i-th pair of rows: looked up before the wait for the
            //    activations, not after it
            uint16_t *out_y = nullptr;
            uint32_t *out_t = nullptr;
            bool out_single = false;                           // the pair is the lone last row of a matrix with an odd row count
            bool out_gated = false;                            // the pair is (gate row, up row): one output, silu(gate) * up
            const uint16_t *res_plain = nullptr;               // where the pair's residuals come from: a launch input ...
            const uint64_t *res_tagged = nullptr;              // ... or the tagged output of an earlier matrix
            if (lane < n) {
                const int R = rbeg + 2 * wave + lane * CHAIN_STRIDE;
                const int m = ph.first + (R >= ph.mstart[1]) + (R >= ph.mstart[2]) + (R >= ph.mstart[3]);
                const ChainMatrix mt = a.mat[m];
                const int r = R - mt.start;
                out_y = mt.y + r;
                out_t = ws + mt.tag_word + chain_tag_word(r);
                out_single = r == mt.rows - 1;
                if constexpr (FUSED) {
                    if (mt.gated) {
                        out_gated = true; out_single = true;
                        out_y = mt.y + (r >> 1);
                        out_t = ws + mt.tag_word + chain_tag_word(r >> 1);
                    } else if (mt.residual_tag_word) {
                        res_tagged = reinterpret_cast<const uint64_t *>(ws + mt.residual_tag_word + chain_tag_word(r));
                    } else if (mt.residual) {
                        res_plain = mt.residual + r;
                    }
                }
            }
            float res0 = 0.f, res1 = 0.f;
            int done = 0;                                      // pairs of rows summed so far
            // A tagged residual is read here for the first time, together with the phase's activations: its producer is an
            // earlier phase than theirs, so it is complete as a rule, and the read costs no round trip of its own (read behind
            // the barrier it costs one, in front of the phase's first step).  It is looked at behind the barrier.
            [[maybe_unused]] uint64_t res_first = 0;
            if constexpr (FUSED) {
                if (res_tagged) res_first = __hip_atomic_load(res_tagged, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                else if (res_plain) res_first = out_single ? (uint64_t)*global_ptr<const uint16_t>(res_plain) : (uint64_t)*global_ptr<const uint32_t>(res_plain);
            }
            // 1. stage the activations (those of the first phase are already on their way)
            const int nchunks = nstrips * 256;
            if constexpr (!Q3H) {
                const int cols = nbk * T::block, nslots = nstrips * 64;
                const uint64_t *base = reinterpret_cast<const uint64_t *>(ws + ph.x_tag_word);
#pragma unroll 1
                for (int cw = wave * 64; cw < nslots; cw += 64 * CHAIN_WAVES) {
                    const int c = cw + lane, k0 = c * G::WPL;
                    const bool live = k0 < cols;                   // lanes past the end of the row stage zeros (and read lane 0's words)
                    const int k = live ? k0 : 0;
                    uint32_t n[G::XD];
                    if (ph.x_src < 0) {                            // an input of the launch
#pragma unroll
                        for (int j = 0; j < XQ; ++j) {
                            const u32x4 v = global_ptr<const u32x4>(ph.x + k)[j];
                            n[4 * j] = v.x; n[4 * j + 1] = v.y; n[4 * j + 2] = v.z; n[4 * j + 3] = v.w;
                        }
                    } else {                                       // tagged words: pair g of the vector at 8-byte word
                        int budget = failed ? 1 : CHAIN_POLL_BUDGET;   // (g >> 11) * 2048 + (g & 7) * 256 + ((g >> 3) & 255)
                        bool again;
                        do {
                            bool ok = true;
#pragma unroll
                            for (int i = 0; i < G::XD; ++i) {
                                const int g = (k >> 1) + i;
                                const uint64_t wd = __hip_atomic_load(base + (g >> 11) * 2048 + (g & 7) * 256 + ((g >> 3) & 255),
                                                                      __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                const uint32_t lo = (uint32_t)wd, hi = (uint32_t)(wd >> 32);
                                ok = ok && ((lo ^ tag) >> 16) == 0 && ((hi ^ tag) >> 16) == 0;
                                n[i] = (lo & 0xFFFFu) | (hi << 16);
                            }
                            again = __builtin_amdgcn_ballot_w64(live && !ok) != 0;
                            if (again) {
                                budget -= 1;
                                if (budget <= 0) {
                                    failed = true;
                                    again = false;
                                    if (lane == 0) __hip_atomic_store(ws + CHAIN_WS_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                                } else {
                                    __builtin_amdgcn_s_sleep(CHAIN_POLL_SLEEP);
                                }
                            }
                        } while (again);
                    }
                    if (!live)
#pragma unroll
                        for (int i = 0; i < G::XD; ++i) n[i] = 0;
                    slot_put(c, n, a.ops + p, FUSED ? a.ops[p].aux + k : nullptr);
                }
            } else if (p > 0 && ph.x_src < 0) {
#pragma unroll 1
                for (int cw = wave * 64; cw < nchunks; cw += 64 * CHAIN_WAVES) {
                    const IFLOW_GLOBAL u32x4 *src = chunk_src(ph.x, cw + lane, nbk);
                    put_plain(cw + lane, nbk, src[0], src[1], a.ops + p);
                }
            } else if (p > 0) {
                const uint64_t *base = reinterpret_cast<const uint64_t *>(ws + ph.x_tag_word);
#pragma unroll 1
                for (int cw = wave * 64; cw < nchunks; cw += 64 * CHAIN_WAVES) {
                    const int ch = cw + lane;
                    // chunks past the end of the row were never written: their lanes read chunk 0 and ignore it
                    const bool live = chunk_live(ch, nbk) != 0;
                    const uint64_t *src = base + (ch >> 8) * 2048 + (live ? (ch & 255) : 0);
                    uint32_t n8[8];
                    u32x4 gain0 = {0, 0, 0, 0}, gain1 = {0, 0, 0, 0};  // the gains are requested before the wait for the activations
                    if constexpr (FUSED) {
                        if (a.ops[p].x_op == IFLOW_X_RMS_GAIN) {
                            const IFLOW_GLOBAL u32x4 *gs = chunk_src(a.ops[p].aux, ch, nbk);
                            gain0 = gs[0]; gain1 = gs[1];
                        }
                    }
                    int budget = failed ? 1 : CHAIN_POLL_BUDGET;
                    bool again;                                // the wavefront re-reads as long as any of its lanes has to
                    do {
                        uint64_t wd[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i)
                            wd[i] = __hip_atomic_load(src + i * 256, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        bool ok = true;
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const uint32_t lo = (uint32_t)wd[i], hi = (uint32_t)(wd[i] >> 32);
                            ok = ok && ((lo ^ tag) >> 16) == 0 && ((hi ^ tag) >> 16) == 0;
                            n8[i] = (lo & 0xFFFFu) | (hi << 16);
                        }
                        again = __builtin_amdgcn_ballot_w64(live && !ok) != 0;
                        if (again) {
                            budget -= 1;
                            if (budget <= 0) {
                                failed = true;
                                again = false;
                                if (lane == 0) __hip_atomic_store(ws + CHAIN_WS_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            } else {
                                __builtin_amdgcn_s_sleep(CHAIN_POLL_SLEEP);
                            }
                        }
                    } while (again);
                    if (!live)
#pragma unroll
                        for (int i = 0; i < 8; ++i) n8[i] = 0;
                    if constexpr (FUSED) {
                        if (a.ops[p].x_op == IFLOW_X_RMS_GAIN) apply_gain(n8, gain0, gain1);
                    }
                    chunk_put(ch, n8);
                }
            }
            // the normalization's scalar: every wavefront's share of sum x^2 through LDS (behind the staged strips), added
            // up in a fixed order by everybody
            float out_scale = 1.0f;
            float *const sq_slot = reinterpret_cast<float *>(xs + (size_t)hd->max_strips * CHAIN_SLOT_BYTES);
            if constexpr (FUSED) {
                const float wsum = wave_sum(sumsq);
                if (lane == 0) sq_slot[wave] = wsum;
                sumsq = 0.f;
            }
            CHAIN_MARK(p, wave < 8 ? wave : 15);               // this wavefront's share of the activations is staged
            __syncthreads();
            if (wave == 0) CHAIN_MARK(p, 8);                   // all of them are
            uint32_t resid = 0;                                // the pair's residuals (two fp16)
            if constexpr (FUSED) {
                if (a.ops[p].x_op == IFLOW_X_RMS_GAIN) {
                    float tot = 0.f;
#pragma unroll
                    for (int i = 0; i < CHAIN_WAVES; ++i) tot += sq_slot[i];
                    out_scale = 1.0f / __builtin_sqrtf(tot * a.ops[p].inv_cols + a.ops[p].eps);
                }
                // The residuals, requested in 0: behind the barrier the phase's own input is complete, and with it every output
                // of the phases before its producer.  A tagged residual is still checked (and re-read a bounded number of times).
                if (res_tagged) {
                    int budget = failed ? 1 : CHAIN_POLL_BUDGET;
                    uint64_t wd = res_first;
                    for (;;) {
                        const uint32_t lo = (uint32_t)wd, hi = (uint32_t)(wd >> 32);
                        resid = (lo & 0xFFFFu) | (hi << 16);
                        if (((lo ^ tag) >> 16) == 0 && (out_single || ((hi ^ tag) >> 16) == 0)) break;
                        if (--budget <= 0) {
                            failed = true;
                            __hip_atomic_store(ws + CHAIN_WS_ERROR, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                            break;
                        }
                        __builtin_amdgcn_s_sleep(CHAIN_POLL_SLEEP);
                        wd = __hip_atomic_load(res_tagged, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                } else if (res_plain) {
                    resid = (uint32_t)res_first;
                }
            }

            // 2. this wavefront's steps; step j of the phase uses register set j mod S
            auto load_xr = [&](int ts) __attribute__((always_inline)) {
                const uint8_t *sl = xs + (size_t)ts * CHAIN_SLOT_BYTES;
#pragma unroll
                for (int jj = 0; jj < XQ; ++jj) {
                    const uint4 qv = *reinterpret_cast<const uint4 *>(sl + (jj * 64 + lane) * 16);
                    xr[0].v[4 * jj] = as_h2(qv.x); xr[0].v[4 * jj + 1] = as_h2(qv.y);
                    xr[0].v[4 * jj + 2] = as_h2(qv.z); xr[0].v[4 * jj + 3] = as_h2(qv.w);
                }
                const float2 sm = *reinterpret_cast<const float2 *>(sl + XQ * 64 * 16 + lane * 8);
                xr[0].bias_sum = sm.x; xr[0].x_sum = sm.y;
            };
            if (nstrips == 1 && n > 0) load_xr(0);             // a single strip stays in registers for all rows
            float part[2] = {0.f, 0.f};                        // per-lane partial sums of the two rows, carried across strips
            const int nreal = n * nstrips;
            int t = 0;
            auto body = [&](auto stage, bool real = true) __attribute__((always_inline)) {     // the next step of the phase, from register set `stage`
                constexpr int st = decltype(stage)::value;     // (real == false: an empty step of the padding, which only passes its set on)
                float v[2] = {0.f, 0.f};
                if constexpr (EARLY) request(w[(st + S - 1) % S]);   // into the set decoded one step ago
                if (real && nstrips > 1) load_xr(t);
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    if (!real) continue;
                    if constexpr (IFLOW_CHAIN_ABL == 1) {      // (the weights are looked at, so that their loads stay)
                        uint32_t fold = 0;
#pragma unroll
                        for (int i = 0; i < G::WD; ++i) fold ^= w[st][u].d[i];
                        v[u] = part[u] + __builtin_bit_cast(float, fold & 0x3F800000u);
                        continue;
                    }
                    float acc[1];
                    if constexpr (Q3H) lane_dot_q3h<1>(w[st][u], xr, acc, q3h_k); else lane_dot<KIND, 1>(w[st][u], xr, acc);
                    half2_t so;
                    if constexpr (Q3H) so = as_h2(q3h_header(w[st][u].d)); else so = as_h2(w[st][u].hdr);
                    v[u] = part[u] + __builtin_fmaf((float)so.x, acc[0] - xr[0].bias_sum, (float)so.y * xr[0].x_sum);
                }
                if constexpr (!EARLY) request(w[st]);          // the register set takes the step S further on in the sequence
                const bool last = real && t == nstrips - 1;    // the rows are complete: two reductions, lane 63 publishes
                if (last) {
                    // lane `done` of res0 / res1 <- the two row sums (same summation tree as wave_sum_to_lane63)
                    const int both_lo = pair_sums(v[0], v[1]);
                    park(res0, res1, __builtin_amdgcn_readlane(both_lo, 31), __builtin_amdgcn_readlane(both_lo, 63), done);
                    done += 1;
                }
                // (plain selects: written as stores under branches, these end up in scratch memory)
                part[0] = last ? 0.f : (real ? v[0] : part[0]);
                part[1] = last ? 0.f : (real ? v[1] : part[1]);
                t = last ? 0 : t + (real ? 1 : 0);
            };
            using C0 = std::integral_constant<int, 0>;
            using C1 = std::integral_constant<int, (S > 1 ? 1 : 0)>;
            using C2 = std::integral_constant<int, (S > 2 ? 2 : 0)>;
            using C3 = std::integral_constant<int, (S > 3 ? 3 : 0)>;
            static_assert(S >= 1 && S <= 4, "register sets per wavefront");
            // The phase's first step sits in set `cs` (the wavefront's steps so far, mod S).  Up to S - 1 steps bring the
            // sequence round to set 0, then whole rounds of S steps, then the steps left over from sets 0, 1, ...: every
            // copy of a step names its register set at compile time, and no step is spent on padding.
            int left = nreal;
            if constexpr (PAD) {                               // whole rounds only, the last one filled up with empty steps
#pragma unroll 1
                for (int j = 0; j < nreal; j += S) {
                    body(C0{}, true);
                    if constexpr (S > 1) body(C1{}, j + 1 < nreal);
                    if constexpr (S > 2) body(C2{}, j + 2 < nreal);
                    if constexpr (S > 3) body(C3{}, j + 3 < nreal);
                }
                left = 0;
            }
            if (cs > 0) {
                if constexpr (S > 1) { if (cs <= 1 && left > 0) { body(C1{}); left -= 1; } }
                if constexpr (S > 2) { if (cs <= 2 && left > 0) { body(C2{}); left -= 1; } }
                if constexpr (S > 3) { if (cs <= 3 && left > 0) { body(C3{}); left -= 1; } }
            }
#pragma unroll 1
            for (; left >= S; left -= S) {
                body(C0{});
                if constexpr (S > 1) body(C1{});
                if constexpr (S > 2) body(C2{});
                if constexpr (S > 3) body(C3{});
            }
            if (left > 0) {                                    // (only reached with the sequence at set 0)
                body(C0{});
                if constexpr (S > 2) { if (left > 1) body(C1{}); }
                if constexpr (S > 3) { if (left > 2) body(C2{}); }
            }
            if constexpr (!PAD) cs = (cs + nreal) % S;
            if (wave == 0) CHAIN_MARK(p, 9);                   // steps done: wavefronts 0, 7 and 11
            if (wave == 7) CHAIN_MARK(p, 10);
            if (wave == 11) CHAIN_MARK(p, 11);
            // 3. publish: the caller's plain fp16 outputs, and the tagged words for later phases
            if (lane < n) {
                if constexpr (FUSED) {
                    res0 *= out_scale; res1 *= out_scale;
                    if (out_gated) {                           // silu(gate) * up in fp32, rounded once
                        res0 = res0 * __builtin_amdgcn_rcpf(1.0f + __expf(-res0)) * res1;
                    } else {
                        res0 += (float)as_h((uint16_t)(resid & 0xFFFFu));
                        res1 += (float)as_h((uint16_t)(resid >> 16));
                    }
                }
                const uint32_t h0 = as_u16((half_t)res0), h1 = as_u16((half_t)res1);
                if (!out_single) {
                    *global_ptr<uint32_t>(out_y) = h0 | (h1 << 16);
                    __hip_atomic_store(reinterpret_cast<uint64_t *>(out_t), (uint64_t)(h0 | tag) | ((uint64_t)(h1 | tag) << 32),
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                } else {
                    *global_ptr<uint16_t>(out_y) = (uint16_t)h0;
                    __hip_atomic_store(out_t, h0 | tag, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                }
            }
            __syncthreads();                                   // the staged activations are no longer needed
        }
    }

    // ---- the workgroup's copy of the launch count advances ----------------------------------------------------------------
    __syncthreads();
    if (tid == 0) __hip_atomic_store(ws + CHAIN_WS_SEEN + wg, counter + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (wg == 0 && tid == 0) {
        ws[CHAIN_WS_CLOCKS + 2] = (uint32_t)__builtin_amdgcn_s_memtime();
        ws[CHAIN_WS_CLOCKS + 3] = (uint32_t)__builtin_amdgcn_s_memrealtime();
    }
}

// ---- host side ------------------------------------------------------------------------------------------------
size_t chain_workspace_bytes(int nmatrices, const int64_t *rows)
{
    size_t bytes = IFLOW_CHAIN_WS_HEADER;
    for (int i = 0; i < nmatrices; ++i) bytes += (size_t)((rows[i] + 4095) / 4096) * 4096 * 4;
    return bytes;
}

static bool chain_format(int format, int *strip_cols, int *slot_bytes, int *block, int *row_bits);

size_t chain_plan_bytes(int nphases, int nmatrices, int nattn)
{
    return sizeof(ChainHeader) + (size_t)nphases * (sizeof(ChainPhase) + sizeof(ChainPhaseOps)) + (size_t)nmatrices * sizeof(ChainMatrix) +
           (size_t)nattn * sizeof(ChainAttn);
}

// position ranges per key/value head of an attention inside the launch: about one workgroup per (head, range)
static int chain_attn_splits(int n_kv_heads, int grid)
{
    const int n = grid / n_kv_heads;
    return n < 1 ? 1 : n > 64 ? 64 : n;
}

// the partial states of one attention: 64-bit words [head][range][130]
size_t chain_attn_workspace_bytes(int n_heads, int n_kv_heads, int grid)
{
    return (size_t)n_heads * chain_attn_splits(n_kv_heads, grid) * 130 * 8;
}

// Dynamic LDS of a launch: the staged activations of the widest phase (+ the shares of sum x^2) or the attention's running
// states, whichever is larger, and the rotary embedding's table behind them.
int chain_lds_bytes(int format, int max_strips)
{
    int strip_cols, slot_bytes, block, row_bits;
    if (!chain_format(format, &strip_cols, &slot_bytes, &block, &row_bits)) return 0;
    const int x_region = max_strips * slot_bytes + 64, attn_region = CHAIN_ATTN_STATE_BYTES + CHAIN_ATTN_STAGE_BYTES;
    return (x_region > attn_region ? x_region : attn_region) + 1024;
}

// The formats the chained launch is built for, and their strip geometry on the host side.
static bool chain_format(int format, int *strip_cols, int *slot_bytes, int *block, int *row_bits)
{
    switch (format) {
    case IFLOW_Q3H_B64: *strip_cols = chain_strip_cols<KIND_Q3H>(); *slot_bytes = chain_slot_bytes<KIND_Q3H>(); *block = 64; *row_bits = 4; return true;
    case IFLOW_Q4_B64: *strip_cols = chain_strip_cols<KIND_Q4>(); *slot_bytes = chain_slot_bytes<KIND_Q4>(); *block = 64; *row_bits = 4; return true;
    case IFLOW_Q4_B32: *strip_cols = chain_strip_cols<KIND_Q4>(); *slot_bytes = chain_slot_bytes<KIND_Q4>(); *block = 32; *row_bits = 4; return true;
    case IFLOW_Q8_B64: *strip_cols = chain_strip_cols<KIND_Q8>(); *slot_bytes = chain_slot_bytes<KIND_Q8>(); *block = 64; *row_bits = 8; return true;
    case IFLOW_Q8_B32: *strip_cols = chain_strip_cols<KIND_Q8>(); *slot_bytes = chain_slot_bytes<KIND_Q8>(); *block = 32; *row_bits = 8; return true;
    // bit planes: row_bits = the low plane's bits per weight (the first code stream of a row)
    case IFLOW_Q6_B64: *strip_cols = chain_strip_cols<KIND_Q6>(); *slot_bytes = chain_slot_bytes<KIND_Q6>(); *block = 64; *row_bits = 4; return true;
    case IFLOW_Q5_B64: *strip_cols = chain_strip_cols<KIND_Q5>(); *slot_bytes = chain_slot_bytes<KIND_Q5>(); *block = 64; *row_bits = 4; return true;
    case IFLOW_Q3_B32: *strip_cols = chain_strip_cols<KIND_Q3>(); *slot_bytes = chain_slot_bytes<KIND_Q3>(); *block = 32; *row_bits = 2; return true;
    case IFLOW_Q2_B32: *strip_cols = chain_strip_cols<KIND_Q2>(); *slot_bytes = chain_slot_bytes<KIND_Q2>(); *block = 32; *row_bits = 2; return true;
    default: return false;
    }
}

bool chain_supports_format(int format)
{
    int a, b, c, d;
    return chain_format(format, &a, &b, &c, &d);
}

// The longest row whose activations fit the kernel's LDS in this format (whole strips, and never more than CHAIN_MAX_COLS).
int64_t chain_max_cols(int format)
{
    int strip_cols, slot_bytes, block, row_bits;
    if (!chain_format(format, &strip_cols, &slot_bytes, &block, &row_bits)) return 0;
    const int64_t by_lds = (int64_t)((CHAIN_LDS_BYTES - 64 - 1024) / slot_bytes) * strip_cols;
    return by_lds < CHAIN_MAX_COLS ? by_lds : CHAIN_MAX_COLS;
}

#define IFLOW_CHAIN_FOR_FORMAT(DO, FF) DO(FF, false, false) DO(FF, true, false) DO(FF, true, true)
#define IFLOW_CHAIN_FOR_ALL(DO) \
    IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q3H_B64) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q4_B64) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q4_B32) \
    IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q8_B64) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q8_B32) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q6_B64) \
    IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q5_B64) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q3_B32) IFLOW_CHAIN_FOR_FORMAT(DO, IFLOW_Q2_B32)

// Launch geometry: as many workgroups as the device has compute units (one each: 768 threads
// and most of its LDS), so the whole grid is resident at once and producers and consumers of a hand-over run
// concurrently.
hipError_t chain_grid_for_device(int *grid)
{
    static PerDevice pd;
    int cus = 0;
    hipError_t e0 = once_per_device(pd, &cus, [] {
        hipError_t e = hipSuccess;
#define IFLOW_CHAIN_ATTR(FF, FUSED, ATTN) \
        if (e == hipSuccess) e = hipFuncSetAttribute(reinterpret_cast<const void *>(&chain_kernel<chain_sets(FF, ATTN), FUSED, FF, ATTN>), \
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, CHAIN_LDS_BYTES);
        IFLOW_CHAIN_FOR_ALL(IFLOW_CHAIN_ATTR)
#undef IFLOW_CHAIN_ATTR
        return e;
    });
    if (e0 != hipSuccess) return e0;
    *grid = cus < CHAIN_MAX_GRID ? cus : CHAIN_MAX_GRID;
    return hipSuccess;
}

// The plan for `grid` workgroups, in host memory (the caller copies it to the device).  Returns false for shapes outside
// the kernel's limits.
bool chain_build_plan(const ChainSpec &c, int grid, std::vector<uint8_t> &out)
{
    int strip_cols, slot_bytes, block, row_bits;
    if (!chain_format(c.format, &strip_cols, &slot_bytes, &block, &row_bits)) return false;
    const int nmat = c.first[c.nphases - 1] + c.counts[c.nphases - 1];
    out.assign(chain_plan_bytes(c.nphases, nmat, c.nattn), 0);
    ChainHeader *hd = reinterpret_cast<ChainHeader *>(out.data());
    ChainPhase *phs = reinterpret_cast<ChainPhase *>(out.data() + sizeof(ChainHeader));
    ChainMatrix *mats = reinterpret_cast<ChainMatrix *>(phs + c.nphases);
    ChainPhaseOps *ops = reinterpret_cast<ChainPhaseOps *>(mats + nmat);
    ChainAttn *attns = reinterpret_cast<ChainAttn *>(ops + c.nphases);
    bool fused = false;
    int m = 0, max_strips = 1;
    size_t word = IFLOW_CHAIN_WS_HEADER / 4;
    for (int p = 0; p < c.nphases; ++p) {
        ChainPhase &ph = phs[p];
        if (c.kind && c.kind[p] != 0) {                        // a half of an attention: no rows; the first half owns the output's entry
            if (p == 0) return false;                          // (the first phase's activations are staged ahead of everything)
            ph.kind = c.kind[p]; ph.attn = c.attn_of[p];
            ph.first = m; ph.count = 0; ph.x_src = -1;
            for (int j = 0; j < CHAIN_MAX_GROUP; ++j) ph.mstart[j] = 0x7FFFFFFF;
            ops[p].x_op = IFLOW_X_PLAIN;
            fused = true;
            if (c.kind[p] == 1) {
                if (c.counts[p] != 1 || ph.attn < 0 || ph.attn >= c.nattn) return false;
                // the second half follows at once (the kernel runs both in one go)
                if (p + 1 >= c.nphases || c.kind[p + 1] != 2 || c.attn_of[p + 1] != ph.attn) return false;
                const ChainAttnSpec &as = c.attn[ph.attn];
                ChainAttn &at = attns[ph.attn];
                mats[m].packed = nullptr; mats[m].y = c.y[m]; mats[m].rows = (int)c.rows[m]; mats[m].start = 0;
                mats[m].tag_word = (int)word;
                word += (size_t)((c.rows[m] + 4095) / 4096) * 4096;
                at.q = as.q; at.k_new = as.k_new; at.v_new = as.v_new;
                at.q_tag_word = as.q_src >= 0 ? mats[as.q_src].tag_word : 0;
                at.k_tag_word = as.k_src >= 0 ? mats[as.k_src].tag_word : 0;
                at.v_tag_word = as.v_src >= 0 ? mats[as.v_src].tag_word : 0;
                at.k_cache = as.k_cache; at.v_cache = as.v_cache; at.out = c.y[m];
                at.out_tag_word = mats[m].tag_word;
                at.n_heads = as.n_heads; at.n_kv_heads = as.n_kv_heads; at.nsplit = chain_attn_splits(as.n_kv_heads, grid);
                if (as.n_kv_heads * at.nsplit > grid) return false;
                // the second half's LDS: a state per (range, output of the workgroup); one thread per output
                const int per_wg = ((as.n_heads * 128 + grid - 1) / grid + 1) & ~1;
                if (per_wg > 64 * CHAIN_WAVES_ATTN || at.nsplit * per_wg * 3 > 4 * CHAIN_WAVES_ATTN * 130) return false;
                const int group = as.n_heads / as.n_kv_heads;
                if (as.n_heads % as.n_kv_heads != 0 || (group != 1 && (group & 1))) return false;
                at.max_seq = as.max_seq; at.pairing = as.pairing;
                at.scale_log2e = as.scale * 1.4426950408889634f; at.log2_base = log2((double)as.base);
                ++m;
            } else if (c.counts[p] != 0 || p == 0 || c.kind[p - 1] != 1) {
                return false;
            }
            continue;
        }
        const bool gated = c.gated && c.gated[p];
        ph.x = c.x[p]; ph.first = m; ph.count = gated ? 1 : c.counts[p];
        ops[p].x_op = c.x_op ? c.x_op[p] : IFLOW_X_PLAIN;
        ops[p].aux = c.aux ? c.aux[p] : nullptr;
        ops[p].eps = c.eps ? c.eps[p] : 0.0f;
        ops[p].inv_cols = 1.0f / (float)c.cols[p];
        fused = fused || gated || ops[p].x_op != IFLOW_X_PLAIN;
        for (int j = 0; j < CHAIN_MAX_GROUP; ++j) ph.mstart[j] = 0x7FFFFFFF;
        if (c.cols[p] < block || c.cols[p] % block != 0 || c.cols[p] > chain_max_cols(c.format) || c.counts[p] > CHAIN_MAX_GROUP) return false;
        ph.nbk = (int)(c.cols[p] / block); ph.nstrips = (int)((c.cols[p] + strip_cols - 1) / strip_cols);
        ph.x_src = c.x_src[p];
        ph.x_tag_word = c.x_src[p] >= 0 ? mats[c.x_src[p]].tag_word : 0;
        if (ph.nstrips > max_strips) max_strips = ph.nstrips;
        int64_t v = 0;
        for (int j = 0; j < c.counts[p]; ++j, ++m) {
            mats[m].packed = static_cast<const uint8_t *>(c.packed[m]); mats[m].y = c.y[m]; mats[m].rows = (int)c.rows[m];
            mats[m].start = (int)v;
            mats[m].tag_word = (int)word;
            // (formats with the headers behind the codes: rows x cols x row_bits / 8 bytes of codes come first)
            const int64_t code_bytes = c.rows[m] * c.cols[p] * row_bits / 8;
            const int code_bits = c.format == IFLOW_Q6_B64 ? 6 : c.format == IFLOW_Q5_B64 ? 5 : c.format == IFLOW_Q3_B32 ? 3 : row_bits;
            if (c.format != IFLOW_Q3H_B64 && code_bytes / 4 > 0xFFFFFFFFLL) return false;
            const int64_t all_code_bytes = c.rows[m] * c.cols[p] * code_bits / 8;      // (bit planes: both planes)
            if (c.format != IFLOW_Q3H_B64 && all_code_bytes / 4 > 0xFFFFFFFFLL) return false;
            mats[m].hdr_off4 = c.format != IFLOW_Q3H_B64 ? (uint32_t)(all_code_bytes / 4) : 0u;
            mats[m].hi_off4 = (uint32_t)(code_bytes / 4);
            word += (size_t)((c.rows[m] + 4095) / 4096) * 4096;
            if (gated) {                                       // the pair (gate, up) is one matrix of 2 x rows in the row space;
                if (j == 0) {                                  // the up matrix keeps an (unused) descriptor of its own
                    mats[m].rows = (int)(2 * c.rows[m]); mats[m].gated = 1;
                    mats[m].packed2 = static_cast<const uint8_t *>(c.packed[m + 1]);
                    ph.mstart[0] = 0;
                    v = 2 * c.rows[m];
                }
                continue;
            }
            ph.mstart[j] = (int)v;
            if (c.residual && c.residual[m]) {
                fused = true;
                if (c.residual_src[m] >= 0) mats[m].residual_tag_word = mats[c.residual_src[m]].tag_word;
                else mats[m].residual = c.residual[m];
            }
            v += (c.rows[m] + 1) & ~(int64_t)1;                // every matrix starts at an even row of the phase's row space
        }
        const int64_t rpw = ((v + grid - 1) / grid + 1) & ~(int64_t)1;
        if (v > 0x3FFFFFFF || word > 0x3FFFFFFF) return false;
        if (rpw > 64 * 2 * chain_waves(c.nattn > 0)) return false;      // a wavefront parks one pair of rows per lane
        ph.total = (int)v; ph.rows_per_wg = (int)rpw;
    }
    // the attentions' partial states, behind all tagged vectors
    for (int i = 0; i < c.nattn; ++i) {
        attns[i].part_word = (int)word;
        word += chain_attn_workspace_bytes(attns[i].n_heads, attns[i].n_kv_heads, grid) / 4;
        if (word > 0x3FFFFFFF) return false;
    }
    int next_attn = c.nphases;
    for (int p = c.nphases - 1; p >= 0; --p) {
        ops[p].next_attn = next_attn;
        if (phs[p].kind == 1) next_attn = p;
    }
    hd->first_attn = next_attn;
    hd->magic = IFLOW_CHAIN_MAGIC; hd->nphases = c.nphases; hd->nmatrices = nmat; hd->grid = grid; hd->max_strips = max_strips;
    hd->fused = fused ? 1 : 0; hd->format = c.format; hd->nattn = c.nattn; hd->lds_bytes = chain_lds_bytes(c.format, max_strips);
    return true;
}

// strips of the widest phase of a chain (what the launch sizes its LDS by)
int chain_strips(int format, int64_t cols)
{
    int strip_cols, slot_bytes, block, row_bits;
    if (!chain_format(format, &strip_cols, &slot_bytes, &block, &row_bits)) return 0;
    return (int)((cols + strip_cols - 1) / strip_cols);
}

// position: the decode step's position for a plan with attention phases, -1 for a plan without
hipError_t launch_chain(const void *plan, void *workspace, int grid, int lds_bytes, bool fused, int format, int position, hipStream_t s)
{
    const bool attn = position >= 0;
    if (attn && !fused) return hipErrorInvalidValue;
    int g = 0;
    hipError_t e = chain_grid_for_device(&g);                  // (raises the kernel's LDS limit on this device if it has not been)
    if (e != hipSuccess) return e;
    if (g != grid || lds_bytes < 1 || lds_bytes > CHAIN_LDS_BYTES) return hipErrorInvalidValue;   // planned for another device
    const size_t lds = (size_t)lds_bytes;
    bool launched = false;
#define IFLOW_CHAIN_GO(FF, FUSED, ATTN) \
    if (!launched && format == FF && fused == FUSED && attn == ATTN) { \
        hipLaunchKernelGGL((chain_kernel<chain_sets(FF, ATTN), FUSED, FF, ATTN>), dim3((unsigned)grid), dim3(64 * chain_waves(ATTN)), lds, s, \
                           static_cast<const uint8_t *>(plan), static_cast<uint32_t *>(workspace), position); \
        launched = true; \
    }
    IFLOW_CHAIN_FOR_ALL(IFLOW_CHAIN_GO)
#undef IFLOW_CHAIN_GO
    return launched ? hipGetLastError() : hipErrorInvalidValue;
}

}  // namespace iflow
