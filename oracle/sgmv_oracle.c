/*
 * sgmv_oracle.c -- plain CPU definition of SGMV.  TEST INFRASTRUCTURE ONLY.
 *
 * This file is the slow, obviously-correct statement of what the operator
 * computes.  It exists so that the GPU library can be checked element by
 * element; it shares no code, header, table or helper with the GPU path and
 * must never be called from the product path (only tests, the smoke check and
 * the benchmark's CPU-baseline leg use it).
 *
 * What is computed (Punica, arxiv 2310.18547, section "Segmented Gather
 * Matrix-Vector Multiplication"):
 *   - A batch of s_n token rows is cut into n contiguous segments by the index
 *     sequence s_0 = 0 <= s_1 <= ... <= s_n (segment definition paragraph).
 *     Zero-based, segment i owns rows s_i .. s_{i+1}-1.
 *   - Rows of segment i receive the LoRA add-on x * A_i * B_i on top of the
 *     backbone output that is already in y (the section's displayed equation).
 *   - The add-on is evaluated as two steps, v := 0; v += x A_i ("shrink");
 *     y += v B_i ("expand") (the sentence after the displayed equation).
 *   - LoRA shapes: A in R^{h_in x r}, B in R^{r x h_out} (Background,
 *     "Low-Rank Adaptation").
 *
 * Readings where the paper is silent (all listed in the design notes):
 *   - x, y, A, B are 16-bit floats (the roofline analysis counts 2 bytes per
 *     element); every product and sum is taken in the accumulator type, and y
 *     is rounded once, to nearest-even, when stored.
 *   - v is kept in the accumulator type, never rounded to 16 bits.
 *   - `scale` multiplies the expand sum before it is added to y (scale = 1 is
 *     the paper's operator).
 *   - Weights are row-major, stacked per layer: A_i[layer][k][j],
 *     B_i[layer][j][c]; the segment's pointer plus layer_idx selects the layer.
 *   - An empty segment, or a segment whose A or B pointer is NULL, is a no-op.
 *   - Summation order is the index order of the definition (k ascending, then
 *     j ascending); there is no blocking or reordering.
 *
 * Two accumulator widths are offered: acc64 = 0 accumulates in fp32 (the
 * precision the GPU path is specified to accumulate in), acc64 = 1 in fp64
 * (the mathematical result up to one final rounding).
 *
 * The 16-bit <-> fp32 conversions below are written out from the IEEE-754
 * binary16 layout (1-5-10) and the bfloat16 layout (upper half of binary32).
 */
#include <pthread.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_F16 = 0, ORACLE_BF16 = 1 };

/* ---------------------------------------------------------------- formats */

static float bits_to_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t f32_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

float sgmv_oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = (uint32_t)(h >> 15) << 31;
    uint32_t e = (h >> 10) & 0x1Fu;
    uint32_t m = h & 0x3FFu;
    if (e == 0x1Fu)                       /* inf / nan */
        return bits_to_f32(sign | 0x7F800000u | (m << 13));
    if (e == 0) {                         /* zero / subnormal: m * 2^-24 */
        float mag = (float)m * (1.0f / 16777216.0f);
        return sign ? -mag : mag;
    }
    return bits_to_f32(sign | ((e + 112u) << 23) | (m << 13));
}

float sgmv_oracle_bf16_to_f32(uint16_t b)
{
    return bits_to_f32((uint32_t)b << 16);
}

/* fp32 -> binary16, round to nearest, ties to even */
uint16_t sgmv_oracle_f32_to_f16(float f)
{
    uint32_t u = f32_to_bits(f);
    uint16_t sign = (uint16_t)((u >> 16) & 0x8000u);
    uint32_t a = u & 0x7FFFFFFFu;
    if (a >= 0x7F800000u) {               /* inf or nan */
        if (a == 0x7F800000u) return (uint16_t)(sign | 0x7C00u);
        return (uint16_t)(sign | 0x7E00u | ((a >> 13) & 0x3FFu));
    }
    int32_t e = (int32_t)(a >> 23) - 127; /* unbiased */
    uint32_t m = a & 0x7FFFFFu;
    if (e > 15) return (uint16_t)(sign | 0x7C00u);      /* certainly overflows */
    if (e >= -14) {                       /* normal range of binary16 */
        uint32_t keep = m >> 13, rest = m & 0x1FFFu;
        uint32_t h = ((uint32_t)(e + 15) << 10) | keep;
        if (rest > 0x1000u || (rest == 0x1000u && (keep & 1u))) h += 1; /* may carry into exponent / inf */
        return (uint16_t)(sign | h);
    }
    if (e < -25) return sign;             /* below half of the smallest subnormal */
    /* subnormal result: value = (1.m) * 2^e, unit = 2^-24 */
    uint32_t full = m | 0x800000u;        /* 24-bit significand, value = full * 2^(e-23) */
    int shift = -e - 1;                   /* result = full >> shift, shift in 14..24 */
    uint32_t keep = full >> shift;
    uint32_t rest = full & ((1u << shift) - 1u);
    uint32_t half = 1u << (shift - 1);
    if (rest > half || (rest == half && (keep & 1u))) keep += 1;
    return (uint16_t)(sign | keep);
}

/* fp32 -> bfloat16, round to nearest, ties to even */
uint16_t sgmv_oracle_f32_to_bf16(float f)
{
    uint32_t u = f32_to_bits(f);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u)  /* nan: keep it a nan */
        return (uint16_t)((u >> 16) | 0x0040u);
    uint32_t keep = u >> 16, rest = u & 0xFFFFu;
    if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
    return (uint16_t)keep;
}

static float load16(int dtype, uint16_t b)
{
    return dtype == ORACLE_F16 ? sgmv_oracle_f16_to_f32(b) : sgmv_oracle_bf16_to_f32(b);
}
static uint16_t store16(int dtype, float f)
{
    return dtype == ORACLE_F16 ? sgmv_oracle_f32_to_f16(f) : sgmv_oracle_f32_to_bf16(f);
}

/* fp64 -> fp32 with round-to-odd: truncate toward zero and, if anything was
   lost, force the last significand bit to 1.  A later round-to-nearest-even
   to a format with fewer than 23 significand bits then gives the same result
   as rounding the fp64 value directly. */
static float narrow_round_to_odd(double t)
{
    float f = (float)t;                       /* nearest */
    if ((double)f == t || t != t) return f;   /* exact, or nan */
    uint32_t u = f32_to_bits(f);
    double af = (double)f < 0 ? -(double)f : (double)f;
    double at = t < 0 ? -t : t;
    if (af > at) u -= 1;                      /* step back toward zero (also from inf) */
    u |= 1u;
    return bits_to_f32(u);
}

/* ------------------------------------------------------------ one row */

/* shrink of one row, fp32: out[j] = sum_k x[k] * A[k][j], k ascending */
static void row_shrink_f32(int dtype, int h_in, int r, const uint16_t* xrow,
                           const uint16_t* A, float* out)
{
    for (int j = 0; j < r; ++j) {
        float s = 0.0f;
        for (int k = 0; k < h_in; ++k) {
            float p = load16(dtype, xrow[k]) * load16(dtype, A[(size_t)k * r + j]);
            s = s + p;
        }
        out[j] = s;
    }
}
static void row_shrink_f64(int dtype, int h_in, int r, const uint16_t* xrow,
                           const uint16_t* A, double* out)
{
    for (int j = 0; j < r; ++j) {
        double s = 0.0;
        for (int k = 0; k < h_in; ++k)
            s += (double)load16(dtype, xrow[k]) * (double)load16(dtype, A[(size_t)k * r + j]);
        out[j] = s;
    }
}

/* expand of one row: y[c] = round(y[c] + scale * sum_j v[j] * B[j][c]), j ascending */
static void row_expand_f32(int dtype, int r, int h_out, const float* v,
                           const uint16_t* B, float scale, uint16_t* yrow)
{
    for (int c = 0; c < h_out; ++c) {
        float s = 0.0f;
        for (int j = 0; j < r; ++j) {
            float p = v[j] * load16(dtype, B[(size_t)j * h_out + c]);
            s = s + p;
        }
        float t = scale * s;
        yrow[c] = store16(dtype, load16(dtype, yrow[c]) + t);
    }
}
static void row_expand_f64(int dtype, int r, int h_out, const double* v,
                           const uint16_t* B, double scale, uint16_t* yrow)
{
    for (int c = 0; c < h_out; ++c) {
        double s = 0.0;
        for (int j = 0; j < r; ++j)
            s += v[j] * (double)load16(dtype, B[(size_t)j * h_out + c]);
        double t = (double)load16(dtype, yrow[c]) + scale * s;
        /* exactly one rounding to the 16-bit type: narrow to fp32 with
           round-to-odd (which cannot create or destroy a 16-bit tie), then
           round that to nearest-even. */
        yrow[c] = store16(dtype, narrow_round_to_odd(t));
    }
}

/* ------------------------------------------------------------ the operator */

typedef struct {
    int op;                 /* 0 shrink, 1 expand, 2 add_lora */
    int dtype, h_in, h_out, r, acc64;
    const uint16_t* x;
    uint16_t* y;
    float* v;               /* shrink: in/out [T][r]; expand: in */
    const uint16_t* const* A_ptrs;
    const uint16_t* const* B_ptrs;
    const int32_t* seg_starts;
    int n_segs, layer_idx;
    float scale;
    int row_lo, row_hi;     /* this worker's rows */
} job_t;

static void* run_rows(void* arg)
{
    const job_t* J = (const job_t*)arg;
    int r = J->r;
    float* v32 = (float*)malloc(sizeof(float) * (size_t)r);
    double* v64 = (double*)malloc(sizeof(double) * (size_t)r);
    for (int i = 0; i < J->n_segs; ++i) {
        int lo = J->seg_starts[i], hi = J->seg_starts[i + 1];
        if (lo < J->row_lo) lo = J->row_lo;
        if (hi > J->row_hi) hi = J->row_hi;
        if (lo >= hi) continue;
        const uint16_t* A = J->A_ptrs ? J->A_ptrs[i] : NULL;
        const uint16_t* B = J->B_ptrs ? J->B_ptrs[i] : NULL;
        if (J->op != 1 && !A) continue;          /* no adapter: rows untouched */
        if (J->op != 0 && !B) continue;
        if (A) A += (size_t)J->layer_idx * (size_t)J->h_in * (size_t)r;
        if (B) B += (size_t)J->layer_idx * (size_t)r * (size_t)J->h_out;
        for (int row = lo; row < hi; ++row) {
            const uint16_t* xrow = J->x ? J->x + (size_t)row * J->h_in : NULL;
            uint16_t* yrow = J->y ? J->y + (size_t)row * J->h_out : NULL;
            float* vrow = J->v ? J->v + (size_t)row * r : NULL;
            if (J->op == 0) {                    /* v += x A */
                if (J->acc64) {
                    row_shrink_f64(J->dtype, J->h_in, r, xrow, A, v64);
                    for (int j = 0; j < r; ++j) vrow[j] = (float)((double)vrow[j] + v64[j]);
                } else {
                    row_shrink_f32(J->dtype, J->h_in, r, xrow, A, v32);
                    for (int j = 0; j < r; ++j) vrow[j] = vrow[j] + v32[j];
                }
            } else if (J->op == 1) {             /* y += scale * v B */
                if (J->acc64) {
                    for (int j = 0; j < r; ++j) v64[j] = (double)vrow[j];
                    row_expand_f64(J->dtype, r, J->h_out, v64, B, (double)J->scale, yrow);
                } else {
                    row_expand_f32(J->dtype, r, J->h_out, vrow, B, J->scale, yrow);
                }
            } else {                             /* v := 0; v += xA; y += scale * vB */
                if (J->acc64) {
                    row_shrink_f64(J->dtype, J->h_in, r, xrow, A, v64);
                    row_expand_f64(J->dtype, r, J->h_out, v64, B, (double)J->scale, yrow);
                } else {
                    row_shrink_f32(J->dtype, J->h_in, r, xrow, A, v32);
                    row_expand_f32(J->dtype, r, J->h_out, v32, B, J->scale, yrow);
                }
            }
        }
    }
    free(v32);
    free(v64);
    return NULL;
}

/* Rows are independent, so splitting them over threads changes no bit. */
static int run(job_t base, int n_threads)
{
    if (base.n_segs < 0) return -1;
    if (base.n_segs == 0) return 0;
    if (!base.seg_starts) return -1;
    int T = base.seg_starts[base.n_segs];
    if (T <= 0) return 0;
    if (n_threads < 1) n_threads = 1;
    if (n_threads > T) n_threads = T;
    if (n_threads == 1) {
        base.row_lo = 0; base.row_hi = T;
        run_rows(&base);
        return 0;
    }
    job_t* jobs = (job_t*)malloc(sizeof(job_t) * (size_t)n_threads);
    pthread_t* th = (pthread_t*)malloc(sizeof(pthread_t) * (size_t)n_threads);
    for (int t = 0; t < n_threads; ++t) {
        jobs[t] = base;
        jobs[t].row_lo = (int)((int64_t)T * t / n_threads);
        jobs[t].row_hi = (int)((int64_t)T * (t + 1) / n_threads);
        pthread_create(&th[t], NULL, run_rows, &jobs[t]);
    }
    for (int t = 0; t < n_threads; ++t) pthread_join(th[t], NULL);
    free(jobs);
    free(th);
    return 0;
}

/* v[s_i .. s_{i+1}) += x[s_i .. s_{i+1}) * A_i        (v fp32 [T][r], host memory) */
int sgmv_oracle_shrink(int dtype, int h_in, int r, float* v, const uint16_t* x,
                       const uint16_t* const* A_ptrs, const int32_t* seg_starts,
                       int n_segs, int layer_idx, int acc64, int n_threads)
{
    job_t j; memset(&j, 0, sizeof j);
    j.op = 0; j.dtype = dtype; j.h_in = h_in; j.r = r; j.acc64 = acc64;
    j.x = x; j.v = v; j.A_ptrs = A_ptrs; j.seg_starts = seg_starts;
    j.n_segs = n_segs; j.layer_idx = layer_idx;
    return run(j, n_threads);
}

/* y[s_i .. s_{i+1}) += scale * v[s_i .. s_{i+1}) * B_i   (y 16-bit [T][h_out]) */
int sgmv_oracle_expand(int dtype, int r, int h_out, uint16_t* y, const float* v,
                       const uint16_t* const* B_ptrs, const int32_t* seg_starts,
                       int n_segs, int layer_idx, float scale, int acc64, int n_threads)
{
    job_t j; memset(&j, 0, sizeof j);
    j.op = 1; j.dtype = dtype; j.h_out = h_out; j.r = r; j.acc64 = acc64;
    j.y = y; j.v = (float*)v; j.B_ptrs = B_ptrs; j.seg_starts = seg_starts;
    j.n_segs = n_segs; j.layer_idx = layer_idx; j.scale = scale;
    return run(j, n_threads);
}

/* y += scale * (x A_i) B_i per segment, v never leaves the accumulator type */
int sgmv_oracle_add_lora(int dtype, int h_in, int h_out, int r, uint16_t* y,
                         const uint16_t* x, const uint16_t* const* A_ptrs,
                         const uint16_t* const* B_ptrs, const int32_t* seg_starts,
                         int n_segs, int layer_idx, float scale, int acc64, int n_threads)
{
    job_t j; memset(&j, 0, sizeof j);
    j.op = 2; j.dtype = dtype; j.h_in = h_in; j.h_out = h_out; j.r = r; j.acc64 = acc64;
    j.x = x; j.y = y; j.A_ptrs = A_ptrs; j.B_ptrs = B_ptrs; j.seg_starts = seg_starts;
    j.n_segs = n_segs; j.layer_idx = layer_idx; j.scale = scale;
    return run(j, n_threads);
}

/* bulk conversions, exported so that tests can pin the format code itself */
void sgmv_oracle_decode(int dtype, const uint16_t* in, float* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = load16(dtype, in[i]);
}
void sgmv_oracle_encode(int dtype, const float* in, uint16_t* out, size_t n)
{
    for (size_t i = 0; i < n; ++i) out[i] = store16(dtype, in[i]);
}
