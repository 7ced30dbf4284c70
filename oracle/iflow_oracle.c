/*
 * CPU oracle for block-level linear quantization (Inferflow, arXiv 2401.08294, Section 3)
 * and for the matrix product on the dequantized weights.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, scalar reference that is used only by
 * the test-suite, by the smoke check and by the "cpu_baseline" leg of the benchmark.  The GPU
 * library never calls it and shares no code, table or header with it.
 *
 * Everything here follows the paper's equations in the paper's order:
 *   Eq.1  q  = Round((w - min) / (max - min) * (2^k - 1))           k-bit levels
 *   Eq.2  w' = q / (2^k - 1) * (max - min) + min                    dequantization
 *   Eq.3  q  = Round((w - min) / (max - min) * 10)                  3.5-bit: 11 levels
 *   Eq.4  c  = q[2i] * 11 + q[2i+1]                                 two levels in one 7-bit code
 *   Eq.5  q1 = floor(c / 11),  q2 = c mod 11                        decomposition before Eq.2
 * plus the remark after Table 3 that two FP16 numbers are stored with each block.
 *
 * Readings taken where the paper is silent (each is a choice, stated once here):
 *   - the two FP16 numbers of a block are  scale = (max - min) / L  and  offset = min,
 *     L = 2^k - 1 (Eq.1) or 10 (Eq.3);  Eq.2 then reads  w' = q * scale + offset;
 *   - the encoder divides by the STORED fp16 scale and subtracts the STORED fp16 offset, so it
 *     sees exactly what the decoder will use;
 *   - Round() is round-half-away-from-zero (C's roundf); levels are clamped to [0, L];
 *   - a block whose stored scale is zero (constant block, or a range that underflows fp16)
 *     gets all levels 0;
 *   - blocks are runs of Bs consecutive elements of a row of the row-major [rows][cols] matrix;
 *   - in Eq.4 the even element is the high base-11 digit; Eq.5's q1 is the even element;
 *   - Eq.2 is evaluated exactly and rounded ONCE to fp16 (round to nearest even);
 *   - the 6-, 5- and 3-bit formats take Table 3's block sizes (64, 64, 32); the 2-bit format, which the feature list of
 *     Section 1 names but Table 3 does not list, takes block size 32 like the 3-bit one (3 bits per weight stored).
 * All fp32 arithmetic below is plain IEEE single precision: compile with -ffp-contract=off and
 * without -ffast-math.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* ---- formats: names from the header rows of Table 3 (and Section 1's list for the 2-bit one) ----------- */
enum { ORC_Q8_B32 = 0, ORC_Q8_B64 = 1, ORC_Q4_B32 = 2, ORC_Q4_B64 = 3, ORC_Q3H_B64 = 4,
       ORC_Q6_B64 = 5, ORC_Q5_B64 = 6, ORC_Q3_B32 = 7, ORC_Q2_B32 = 8, ORC_NFMT = 9 };

/* k = bits of a level in Eq.1 (0 for the 3.5-bit format, whose levels come from Eq.3 and are stored as Eq.4 pairs) */
static int fmt_bits(int f)
{
    switch (f) {
    case ORC_Q8_B32: case ORC_Q8_B64: return 8;
    case ORC_Q6_B64: return 6;
    case ORC_Q5_B64: return 5;
    case ORC_Q4_B32: case ORC_Q4_B64: return 4;
    case ORC_Q3_B32: return 3;
    case ORC_Q2_B32: return 2;
    default: return 0;
    }
}
/* L = number of steps between min and max: 2^k - 1 (Eq.1) or 10 (Eq.3); Bs = block size */
static int fmt_L(int f)  { return f == ORC_Q3H_B64 ? 10 : (1 << fmt_bits(f)) - 1; }
static int fmt_Bs(int f) { return (f == ORC_Q8_B32 || f == ORC_Q4_B32 || f == ORC_Q3_B32 || f == ORC_Q2_B32) ? 32 : 64; }
static int fmt_ok(int f) { return f >= 0 && f < ORC_NFMT; }
/* bytes of codes in one block: k-bit levels -> Bs * k / 8; 3.5-bit -> 32 codes * 7 bits = 28 */
static int fmt_code_bytes(int f) { return f == ORC_Q3H_B64 ? 28 : fmt_Bs(f) * fmt_bits(f) / 8; }

int orc_format_levels(int f)     { return fmt_ok(f) ? fmt_L(f) + 1 : -1; }
int orc_format_block(int f)      { return fmt_ok(f) ? fmt_Bs(f) : -1; }
int orc_format_code_bytes(int f) { return fmt_ok(f) ? fmt_code_bytes(f) : -1; }

/* Storage of a whole matrix: codes plus two FP16 numbers (4 bytes) per block (remark after Table 3). */
int64_t orc_packed_bytes(int f, int64_t rows, int64_t cols)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    return rows * (cols / fmt_Bs(f)) * (int64_t)(fmt_code_bytes(f) + 4);
}

/* ---- IEEE binary16 <-> binary32/64, round to nearest even ---------------------------------- */
float orc_f16_to_f32(uint16_t h)
{
    int sign = h >> 15, e = (h >> 10) & 31, m = h & 1023;
    double v;
    if (e == 0)       v = ldexp((double)m, -24);                 /* zero and subnormals */
    else if (e == 31) v = m ? NAN : INFINITY;
    else              v = ldexp((double)(1024 + m), e - 25);     /* (1 + m/1024) * 2^(e-15) */
    return (float)(sign ? -v : v);                               /* every fp16 value is exact in fp32 */
}

uint16_t orc_f64_to_f16(double x)
{
    uint16_t sign = signbit(x) ? 0x8000 : 0;
    double a = fabs(x);
    if (isnan(a)) return (uint16_t)(sign | 0x7E00);
    if (a >= 65520.0) return (uint16_t)(sign | 0x7C00);          /* 65520 = midpoint above the largest finite value */
    if (a < ldexp(1.0, -14)) {                                   /* subnormal range: multiples of 2^-24 */
        double m = rint(ldexp(a, 24));                           /* rint: nearest, ties to even */
        return (uint16_t)(sign | (uint16_t)m);                   /* m == 1024 gives the smallest normal: correct bits */
    }
    int e2;
    (void)frexp(a, &e2);                                         /* a = f * 2^e2, f in [0.5, 1) */
    int e = e2 - 1;                                              /* a in [2^e, 2^(e+1)) */
    double m = rint(ldexp(a, 10 - e));                           /* in [1024, 2048] */
    if (m == 2048.0) { m = 1024.0; e += 1; }
    return (uint16_t)(sign | (uint16_t)((e + 15) << 10) | (uint16_t)((int)m - 1024));
}

uint16_t orc_f32_to_f16(float x) { return orc_f64_to_f16((double)x); }   /* fp32 -> fp64 is exact, so this rounds once */

/* ---- Eq.1 / Eq.3: one block -> levels + the two stored fp16 numbers ------------------------ */
void orc_quantize_block(const float *w, int n, int L, uint8_t *q, uint16_t *scale_h, uint16_t *offset_h)
{
    float mn = w[0], mx = w[0];
    for (int i = 1; i < n; ++i) { if (w[i] < mn) mn = w[i]; if (w[i] > mx) mx = w[i]; }
    mn = mn + 0.0f; mx = mx + 0.0f;                   /* -0 becomes +0 so that the stored pair is canonical */
    float step = (mx - mn) / (float)L;                /* (max - min) / L, fp32 */
    uint16_t sh = orc_f32_to_f16(step);
    uint16_t oh = orc_f32_to_f16(mn);
    *scale_h = sh; *offset_h = oh;
    float s = orc_f16_to_f32(sh), o = orc_f16_to_f32(oh);
    for (int i = 0; i < n; ++i) {
        if (s == 0.0f) { q[i] = 0; continue; }        /* max == min: Eq.1 is 0/0, all levels 0 */
        float t = (w[i] - o) / s;                     /* (w - min) / (max - min) * L with the stored pair */
        float r = roundf(t);                          /* Round(): half away from zero */
        if (!(r >= 0.0f)) r = 0.0f;                   /* below range (or NaN) -> 0 */
        if (r > (float)L) r = (float)L;
        q[i] = (uint8_t)r;
    }
}

/* whole matrix: q[rows*cols] levels, scale/offset[rows*cols/Bs] */
int orc_quantize(int f, const float *w, int64_t rows, int64_t cols, uint8_t *q, uint16_t *scale, uint16_t *offset)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    int L = fmt_L(f), Bs = fmt_Bs(f);
    int64_t nb = rows * (cols / Bs);
    for (int64_t b = 0; b < nb; ++b)
        orc_quantize_block(w + b * Bs, Bs, L, q + b * Bs, scale + b, offset + b);
    return 0;
}

/* ---- Eq.4 / Eq.5 ------------------------------------------------------------------------------ */
int orc_pair_encode(int q_even, int q_odd) { return q_even * 11 + q_odd; }
void orc_pair_decode(int c, int *q1, int *q2) { *q1 = c / 11; *q2 = c % 11; }

/* ---- Eq.2 with the stored pair, single rounding ------------------------------------------- */
uint16_t orc_dequant_value(int q, uint16_t scale_h, uint16_t offset_h)
{
    /* q <= 255 and both fp16 values are integer multiples of 2^-24 below 2^16, so q*s + o is exact in fp64 */
    double v = (double)q * (double)orc_f16_to_f32(scale_h) + (double)orc_f16_to_f32(offset_h);
    return orc_f64_to_f16(v);
}

/* ---- canonical packed record, block after block ---------------------------------------------
 * [scale fp16 LE][offset fp16 LE][codes]
 *   8-bit : byte j = q[j]
 *   4-bit : byte j = q[2j] | q[2j+1] << 4
 *   3.5-bit: 32 Eq.4 codes as a little-endian bit stream, code j in bits [7j, 7j+7)
 *   6-, 5-, 3-, 2-bit: the levels as a little-endian bit stream, level j in bits [kj, kj+k)
 *   (the 8- and 4-bit rules above are this same stream for k = 8 and 4)
 */
int orc_pack_canonical(int f, const uint8_t *q, const uint16_t *scale, const uint16_t *offset,
                       int64_t rows, int64_t cols, uint8_t *out)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    int L = fmt_L(f), Bs = fmt_Bs(f), cb = fmt_code_bytes(f);
    int64_t nb = rows * (cols / Bs);
    for (int64_t b = 0; b < nb; ++b) {
        uint8_t *rec = out + b * (cb + 4);
        const uint8_t *qb = q + b * Bs;
        rec[0] = scale[b] & 255; rec[1] = scale[b] >> 8; rec[2] = offset[b] & 255; rec[3] = offset[b] >> 8;
        uint8_t *cd = rec + 4;
        memset(cd, 0, cb);
        if (L == 255) for (int j = 0; j < Bs; ++j) cd[j] = qb[j];
        else if (L == 15) for (int j = 0; j < Bs / 2; ++j) cd[j] = (uint8_t)(qb[2 * j] | (qb[2 * j + 1] << 4));
        else if (L == 10) for (int j = 0; j < Bs / 2; ++j) {
            int c = orc_pair_encode(qb[2 * j], qb[2 * j + 1]);
            for (int t = 0; t < 7; ++t) if ((c >> t) & 1) { int bit = 7 * j + t; cd[bit >> 3] |= (uint8_t)(1u << (bit & 7)); }
        }
        else for (int j = 0, k = fmt_bits(f); j < Bs; ++j)
            for (int t = 0; t < k; ++t) if ((qb[j] >> t) & 1) { int bit = k * j + t; cd[bit >> 3] |= (uint8_t)(1u << (bit & 7)); }
    }
    return 0;
}

/* inverse of the above; for 3.5-bit it goes through Eq.5 */
int orc_unpack_canonical(int f, const uint8_t *in, int64_t rows, int64_t cols,
                         uint8_t *q, uint16_t *scale, uint16_t *offset)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    int L = fmt_L(f), Bs = fmt_Bs(f), cb = fmt_code_bytes(f);
    int64_t nb = rows * (cols / Bs);
    for (int64_t b = 0; b < nb; ++b) {
        const uint8_t *rec = in + b * (cb + 4), *cd = rec + 4;
        uint8_t *qb = q + b * Bs;
        scale[b] = (uint16_t)(rec[0] | (rec[1] << 8)); offset[b] = (uint16_t)(rec[2] | (rec[3] << 8));
        if (L == 255) for (int j = 0; j < Bs; ++j) qb[j] = cd[j];
        else if (L == 15) for (int j = 0; j < Bs / 2; ++j) { qb[2 * j] = cd[j] & 15; qb[2 * j + 1] = cd[j] >> 4; }
        else if (L == 10) for (int j = 0; j < Bs / 2; ++j) {
            int c = 0, q1, q2;
            for (int t = 0; t < 7; ++t) { int bit = 7 * j + t; c |= ((cd[bit >> 3] >> (bit & 7)) & 1) << t; }
            orc_pair_decode(c, &q1, &q2);
            qb[2 * j] = (uint8_t)q1; qb[2 * j + 1] = (uint8_t)q2;
        }
        else for (int j = 0, k = fmt_bits(f); j < Bs; ++j) {
            int v = 0;
            for (int t = 0; t < k; ++t) { int bit = k * j + t; v |= ((cd[bit >> 3] >> (bit & 7)) & 1) << t; }
            qb[j] = (uint8_t)v;
        }
    }
    return 0;
}

/* ---- the GPU library's device layout, written here from its specification -----------------
 * (the specification is the text of include/iflow.h; this function is an independent
 *  implementation of that text and is what the GPU quantizer's bytes are compared with)
 *
 * 3.5-bit, Bs = 64: a block is 32 bytes = 8 little-endian 32-bit words W0..W7.  With the 32 Eq.4
 *   codes c0..c31 of the block and the header bits S = scale fp16, O = offset fp16:
 *     Wi = c[4i] | c[4i+2] << 7 | ((S >> 2i) & 3) << 14 | c[4i+1] << 16 | c[4i+3] << 23 | ((O >> 2i) & 3) << 30
 *   A row of nbk = cols/64 blocks occupies nbk*32 consecutive bytes; rows follow each other.
 *   Inside a row the blocks are grouped into strips of 64 (the last strip holds the remainder,
 *   n_t blocks).  A strip is stored as two planes: first words W0..W3 of each of its n_t blocks
 *   (16 bytes per block, blocks in order), then words W4..W7 of each block.
 * 4-bit: first all code bytes, row after row (cols/2 bytes per row), then all headers
 *   (scale fp16, offset fp16; 4 bytes per block, blocks in row-major order).  The codes of eight
 *   consecutive weights v0..v7 form one 32-bit word whose nibbles, from the least significant,
 *   are v0 v2 v4 v6 v1 v3 v5 v7.
 * 8-bit: first all code bytes in natural order (cols bytes per row), then all headers as for 4-bit.
 * 6-, 5-, 3-, 2-bit: the level's bits are split over bit planes, stored one after the other (each plane: all rows, row
 *   after row), then all headers as for 4-bit.  Planes, from the level's least significant bits: 6-bit = 4 + 2 bits,
 *   5-bit = 4 + 1, 3-bit = 2 + 1, 2-bit = 2.  A plane of width w stores cols*w/8 bytes per row as little-endian 32-bit
 *   words; a word holds the plane's bits of n = 32/w consecutive weights u0..u(n-1): u(e) sits at bit
 *   (e/2)*w + 16*(e%2) - the even weights in the low half, the odd ones in the high half, each in order.
 *   (For w = 4 this is the 4-bit format's nibble order.)
 */
static void put32(uint8_t *p, uint32_t v) { p[0] = v & 255; p[1] = (v >> 8) & 255; p[2] = (v >> 16) & 255; p[3] = (uint8_t)(v >> 24); }

int orc_pack_device(int f, const uint8_t *q, const uint16_t *scale, const uint16_t *offset,
                    int64_t rows, int64_t cols, uint8_t *out)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    int L = fmt_L(f), Bs = fmt_Bs(f);
    int64_t nbk = cols / Bs;
    if (L == 10) {
        for (int64_t r = 0; r < rows; ++r)
            for (int64_t kb = 0; kb < nbk; ++kb) {
                const uint8_t *qb = q + (r * nbk + kb) * 64;
                uint32_t S = scale[r * nbk + kb], O = offset[r * nbk + kb];
                int c[32];
                for (int j = 0; j < 32; ++j) c[j] = orc_pair_encode(qb[2 * j], qb[2 * j + 1]);
                int64_t strip = kb / 64, j_in = kb % 64;
                int64_t n_t = (nbk - strip * 64 < 64) ? nbk - strip * 64 : 64;
                uint8_t *strip_base = out + r * nbk * 32 + strip * 64 * 32;
                for (int i = 0; i < 8; ++i) {
                    uint32_t W = (uint32_t)c[4 * i] | (uint32_t)c[4 * i + 2] << 7 | ((S >> (2 * i)) & 3u) << 14
                               | (uint32_t)c[4 * i + 1] << 16 | (uint32_t)c[4 * i + 3] << 23 | ((O >> (2 * i)) & 3u) << 30;
                    int plane = i / 4, word = i % 4;
                    put32(strip_base + plane * n_t * 16 + j_in * 16 + word * 4, W);
                }
            }
        return 0;
    }
    if (L != 255 && L != 15) {                         /* bit planes */
        int k = fmt_bits(f);
        int widths[2] = { k >= 5 ? 4 : 2, k == 6 ? 2 : (k == 5 || k == 3) ? 1 : 0 };
        uint8_t *plane = out;
        memset(out, 0, (size_t)(rows * cols * k / 8));
        for (int p = 0, shift = 0; p < 2 && widths[p]; shift += widths[p], ++p) {
            int w = widths[p], n = 32 / w;
            for (int64_t r = 0; r < rows; ++r)
                for (int64_t c = 0; c < cols; ++c) {
                    uint32_t v = ((uint32_t)q[r * cols + c] >> shift) & ((1u << w) - 1u);
                    int e = (int)(c % n);
                    int bit = (e / 2) * w + 16 * (e % 2);
                    uint8_t *word = plane + (r * (cols / n) + c / n) * 4;
                    uint32_t old = (uint32_t)word[0] | (uint32_t)word[1] << 8 | (uint32_t)word[2] << 16 | (uint32_t)word[3] << 24;
                    put32(word, old | v << bit);
                }
            plane += rows * cols * w / 8;
        }
        for (int64_t b = 0; b < rows * nbk; ++b) {
            plane[4 * b] = scale[b] & 255; plane[4 * b + 1] = scale[b] >> 8;
            plane[4 * b + 2] = offset[b] & 255; plane[4 * b + 3] = offset[b] >> 8;
        }
        return 0;
    }
    int64_t code_bytes_row = (L == 255) ? cols : cols / 2;
    uint8_t *hdr = out + rows * code_bytes_row;
    for (int64_t r = 0; r < rows; ++r) {
        const uint8_t *qr = q + r * cols;
        uint8_t *cr = out + r * code_bytes_row;
        if (L == 255) memcpy(cr, qr, (size_t)cols);
        else for (int64_t g = 0; g < cols / 8; ++g) {
            const uint8_t *v = qr + g * 8;
            uint32_t W = (uint32_t)v[0] | (uint32_t)v[2] << 4 | (uint32_t)v[4] << 8 | (uint32_t)v[6] << 12
                       | (uint32_t)v[1] << 16 | (uint32_t)v[3] << 20 | (uint32_t)v[5] << 24 | (uint32_t)v[7] << 28;
            put32(cr + g * 4, W);
        }
        for (int64_t kb = 0; kb < nbk; ++kb) {
            uint8_t *h = hdr + (r * nbk + kb) * 4;
            uint16_t S = scale[r * nbk + kb], O = offset[r * nbk + kb];
            h[0] = S & 255; h[1] = S >> 8; h[2] = O & 255; h[3] = O >> 8;
        }
    }
    return 0;
}

/* ---- Eq.2 over a whole matrix: fp16 [rows][cols] --------------------------------------------- */
int orc_dequant(int f, const uint8_t *q, const uint16_t *scale, const uint16_t *offset,
                int64_t rows, int64_t cols, uint16_t *w16)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0) return -1;
    int Bs = fmt_Bs(f);
    int64_t nb = rows * (cols / Bs);
    for (int64_t b = 0; b < nb; ++b)
        for (int j = 0; j < Bs; ++j)
            w16[b * Bs + j] = orc_dequant_value(q[b * Bs + j], scale[b], offset[b]);
    return 0;
}

/* ---- Y = X * W'^T by its definition: Y[b][n] = sum_k W'[n][k] * X[b][k], fp64, ascending k -------
 * w16: [rows][cols] fp16 (dequantized weights), x16: [batch][cols] fp16, y: [batch][rows] fp64.
 * threads > 1 splits the rows over that many OpenMP threads; returns the number of threads used.
 */
int orc_gemm(const uint16_t *w16, int64_t rows, int64_t cols, const uint16_t *x16, int64_t batch,
             double *y, int threads)
{
    int used = 1;
    double *xd = (double *)malloc(sizeof(double) * (size_t)(batch * cols));
    if (!xd) return -1;
    for (int64_t i = 0; i < batch * cols; ++i) xd[i] = (double)orc_f16_to_f32(x16[i]);
    if (threads < 1) threads = 1;
#ifdef _OPENMP
#pragma omp parallel num_threads(threads)
    {
#pragma omp single
        used = omp_get_num_threads();
#pragma omp for schedule(static)
#endif
        for (int64_t n = 0; n < rows; ++n)
            for (int64_t b = 0; b < batch; ++b) {
                double acc = 0.0;
                for (int64_t k = 0; k < cols; ++k)
                    acc += (double)orc_f16_to_f32(w16[n * cols + k]) * xd[b * cols + k];
                y[b * rows + n] = acc;
            }
#ifdef _OPENMP
    }
#endif
    free(xd);
    return used;
}

/* Same sum in sequential fp32 with an fp16 result: for information only (what a straightforward
 * fp32-accumulating implementation returns), never a parity target. */
void orc_gemm_f32(const uint16_t *w16, int64_t rows, int64_t cols, const uint16_t *x16, int64_t batch, uint16_t *y16)
{
    for (int64_t n = 0; n < rows; ++n)
        for (int64_t b = 0; b < batch; ++b) {
            float acc = 0.0f;
            for (int64_t k = 0; k < cols; ++k) {
                float p = orc_f16_to_f32(w16[n * cols + k]) * orc_f16_to_f32(x16[b * cols + k]);
                acc = acc + p;
            }
            y16[b * rows + n] = orc_f32_to_f16(acc);
        }
}

/* ---- the whole decode-side path on a packed canonical record, as timed for the CPU baseline:
 * unpack (Eq.5), dequantize (Eq.2), multiply (definition).  Scratch is allocated here. */
int orc_qgemm_canonical(int f, const uint8_t *packed, int64_t rows, int64_t cols,
                        const uint16_t *x16, int64_t batch, double *y, int threads)
{
    if (!fmt_ok(f) || rows <= 0 || cols <= 0 || cols % fmt_Bs(f) != 0 || batch <= 0) return -1;
    int Bs = fmt_Bs(f);
    int64_t nb = rows * (cols / Bs);
    uint8_t *q = (uint8_t *)malloc((size_t)(rows * cols));
    uint16_t *s = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)nb), *o = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)nb);
    uint16_t *w16 = (uint16_t *)malloc(sizeof(uint16_t) * (size_t)(rows * cols));
    int used = -1;
    if (q && s && o && w16) {
        orc_unpack_canonical(f, packed, rows, cols, q, s, o);
        orc_dequant(f, q, s, o, rows, cols, w16);
        used = orc_gemm(w16, rows, cols, x16, batch, y, threads);
    }
    free(q); free(s); free(o); free(w16);
    return used;
}
