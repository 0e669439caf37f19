/*
 * CPU oracle for direct sparse convolution.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, single-threaded
 * statement of what the method computes.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product (the HIP library)
 * shares no code with it and never routes through it.
 *
 * What it follows (Pietron & Zurek, arXiv 2011.06295):
 *   - section 3, eq. 1: the convolution (cross-correlation, no kernel flip)
 *     and the output size E = (H + 2*padding - R)/stride + 1 (floor division);
 *   - section 5, eq. 4: pruned weights are w * mask;
 *   - section 6 (cluster quantisation) and section 9 (its 4-bit configuration):
 *     every weight is replaced by one of 16 centroids, each held in 16 bits,
 *     and stored as the 4-bit number of its centroid;
 *   - section 7: CSR of the pruned weights, one row per output channel, three
 *     arrays (values, column index, row pointer), and the option of padding
 *     every row to one unified non-zero count with explicit zeros placed at
 *     neighbouring indices;
 *   - section 8: direct sparse convolution multiplies those CSR rows straight
 *     against the NCHW input.  It is not an approximation: it evaluates eq. 1
 *     and skips exactly the masked-out terms.
 *
 * Readings where the paper is silent:
 *   - the column index of a stored weight is its flat position (c*R + r)*S + s,
 *     entries of a row in ascending column order, 32-bit indices;
 *   - the mask, not the value, decides what is stored (a kept 0.0 is stored, a
 *     dropped non-zero is not); values are copied bit for bit;
 *   - accumulation is in double in stored (ascending column) order, rounded
 *     once to float; a float-accumulate mode exists for the timed CPU baseline;
 *   - the half path stores IEEE binary16 with round-to-nearest-even and
 *     accumulates wide; the caller rounds weights and inputs with
 *     oracle_f32_to_f16 / oracle_f16_to_f32 and calls the same routines.
 *
 * Pins (tests/test_oracle_pins.py): brute-force 7-loop dense convolution
 * (oracle_dense_conv7, below, kept separate from the sparse routine),
 * hand-worked 3x3 examples, closed forms, delta inputs, linearity,
 * torch conv2d / scipy CSR special cases, an independent NumPy encoder.
 * The *choice* of which zeros pad a short row is under-determined by the
 * paper; that rule is pinned only by result invariance and a second
 * implementation of the same stated rule.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- shapes */

/* Section 3: output extent for one spatial dimension; -1 if the padded input
 * is smaller than the filter. */
int oracle_output_dim(int in, int pad, int filt, int stride)
{
    if (in <= 0 || filt <= 0 || stride < 1 || pad < 0) return -1;
    int span = in + 2 * pad - filt;
    if (span < 0) return -1;
    return span / stride + 1;
}

/* ---------------------------------------------------------------- binary16 */

/* float -> IEEE binary16 bits, round to nearest even, subnormals kept. */
uint16_t oracle_f32_to_f16(float f)
{
    uint32_t u;
    memcpy(&u, &f, 4);
    uint32_t sign = (u >> 16) & 0x8000u;
    uint32_t expo = (u >> 23) & 0xffu;
    uint32_t mant = u & 0x7fffffu;
    if (expo == 0xffu) { /* inf / nan */
        if (mant == 0) return (uint16_t)(sign | 0x7c00u);
        uint32_t m = mant >> 13;
        if (m == 0) m = 1; /* keep it a NaN */
        return (uint16_t)(sign | 0x7c00u | m | 0x200u);
    }
    int e = (int)expo - 127; /* unbiased */
    if (e > 15) return (uint16_t)(sign | 0x7c00u); /* overflow -> inf */
    if (e >= -14) {
        /* normal half: 10 mantissa bits, drop 13 */
        uint32_t half = ((uint32_t)(e + 15) << 10) | (mant >> 13);
        uint32_t rem = mant & 0x1fffu;
        if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) half++; /* may carry into exponent / inf */
        return (uint16_t)(sign | half);
    }
    if (e < -25) return (uint16_t)sign; /* below half of the smallest subnormal */
    /* subnormal half: value = m24 * 2^(e-23), unit 2^-24 */
    uint32_t m24 = mant | 0x800000u;
    int shift = -e - 1; /* 14..24 */
    uint32_t half = m24 >> shift;
    uint32_t rem = m24 & ((1u << shift) - 1u);
    uint32_t halfway = 1u << (shift - 1);
    if (rem > halfway || (rem == halfway && (half & 1u))) half++;
    return (uint16_t)(sign | half);
}

/* IEEE binary16 bits -> float, exact. */
float oracle_f16_to_f32(uint16_t h)
{
    uint32_t sign = ((uint32_t)h & 0x8000u) << 16;
    uint32_t expo = (h >> 10) & 0x1fu;
    uint32_t mant = h & 0x3ffu;
    float mag;
    if (expo == 0) {
        mag = ldexpf((float)mant, -24);
    } else if (expo == 31) {
        uint32_t u = sign | 0x7f800000u | (mant << 13);
        float f;
        memcpy(&f, &u, 4);
        return f;
    } else {
        mag = ldexpf((float)(mant | 0x400u), (int)expo - 25);
    }
    return sign ? -mag : mag;
}

void oracle_round_through_f16(const float* in, float* out, long long n)
{
    for (long long i = 0; i < n; ++i) out[i] = oracle_f16_to_f32(oracle_f32_to_f16(in[i]));
}

void oracle_to_f16_bits(const float* in, uint16_t* out, long long n)
{
    for (long long i = 0; i < n; ++i) out[i] = oracle_f32_to_f16(in[i]);
}

/* ---------------------------------------------------------------- CSR (section 7) */

/* Row pointer of the CSR of w*mask: rowptr[k+1]-rowptr[k] = kept entries of
 * output channel k.  mask is [K][L] with L = C*R*S; returns the total. */
long long oracle_csr_rowptr(const unsigned char* mask, int K, int L, int* rowptr)
{
    long long total = 0;
    rowptr[0] = 0;
    for (int k = 0; k < K; ++k) {
        for (int j = 0; j < L; ++j)
            if (mask[(size_t)k * L + j]) ++total;
        rowptr[k + 1] = (int)total;
    }
    return total;
}

/* Column indices and values in ascending column order per row.  mask codes:
 * 0 dropped, 1 kept (value copied bit for bit), 2 explicit zero added by the
 * unify step (stored as +0.0). */
void oracle_csr_fill(const float* w, const unsigned char* mask, int K, int L,
                     int* colidx, float* values)
{
    long long t = 0;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < L; ++j) {
            unsigned char m = mask[(size_t)k * L + j];
            if (!m) continue;
            colidx[t] = j;
            if (m == 2) values[t] = 0.0f;
            else memcpy(&values[t], &w[(size_t)k * L + j], 4);
            ++t;
        }
}

/* Cluster-quantised weights (section 6; section 9: 16 centroids of 16 bits each,
 * a 4-bit code per weight).  index is [K][L] with values 0..15, centroids[16]
 * are rounded to binary16 (centroid_bits), mask is 0/1/2 as for oracle_csr_fill.
 * In CSR order (as oracle_csr_fill) entry t gets code[t] = index of its weight
 * (mask 1) or the number of the first centroid that is zero (mask 2, an explicit
 * zero of the unify step); values[t] is that centroid widened to float.  Codes
 * are packed two to a byte, entry 2i in the low nibble of packed[i], entry 2i+1
 * in the high nibble, an unused last nibble zero.  Where the paper is silent
 * this is the reading: centroid numbers are taken as given (clustering itself
 * belongs to model preparation), the low nibble comes first.  Returns the number
 * of entries, -1 for an index above 15, -2 if an explicit zero is needed and no
 * centroid is zero. */
long long oracle_codebook_csr(const unsigned char* index, const float* centroids,
                              const unsigned char* mask, int K, int L,
                              uint16_t* centroid_bits, unsigned char* packed, float* values)
{
    int zero = -1;
    for (int i = 0; i < 16; ++i) {
        centroid_bits[i] = oracle_f32_to_f16(centroids[i]);
        if (zero < 0 && (centroid_bits[i] & 0x7fffu) == 0) zero = i;
    }
    long long t = 0;
    for (int k = 0; k < K; ++k)
        for (int j = 0; j < L; ++j) {
            unsigned char m = mask[(size_t)k * L + j];
            if (!m) continue;
            int code;
            if (m == 2) {
                if (zero < 0) return -2;
                code = zero;
            } else {
                code = index[(size_t)k * L + j];
                if (code > 15) return -1;
            }
            if (t % 2 == 0) packed[t / 2] = (unsigned char)code;
            else packed[t / 2] = (unsigned char)(packed[t / 2] | (code << 4));
            values[t] = oracle_f16_to_f32(centroid_bits[code]);
            ++t;
        }
    return t;
}

/* Unified non-zero count (section 7): every row is brought up to the count of
 * the fullest row by marking zeros as stored.  Which zeros: first, scanning
 * columns upwards, a dropped column whose left neighbour is stored (possibly
 * just added) is added, so existing runs grow to the right; if the row is
 * still short, the lowest dropped columns are added.  mask_out gets 0/1/2 as
 * described at oracle_csr_fill.  Returns the unified per-row count. */
int oracle_unify_mask(const unsigned char* mask, int K, int L, unsigned char* mask_out)
{
    int target = 0;
    for (int k = 0; k < K; ++k) {
        int c = 0;
        for (int j = 0; j < L; ++j) c += mask[(size_t)k * L + j] ? 1 : 0;
        if (c > target) target = c;
    }
    for (int k = 0; k < K; ++k) {
        const unsigned char* mi = mask + (size_t)k * L;
        unsigned char* mo = mask_out + (size_t)k * L;
        int c = 0;
        for (int j = 0; j < L; ++j) { mo[j] = mi[j] ? 1 : 0; c += mo[j]; }
        int deficit = target - c;
        for (int j = 1; j < L && deficit > 0; ++j)
            if (!mo[j] && mo[j - 1]) { mo[j] = 2; --deficit; }
        for (int j = 0; j < L && deficit > 0; ++j)
            if (!mo[j]) { mo[j] = 2; --deficit; }
    }
    return target;
}

/* ---------------------------------------------------------------- convolution */

/* Direct sparse convolution, eq. 1 restricted to the stored entries.
 *   x   [N][C][H][W] float (for the half path: values already rounded through binary16)
 *   out [N][K][E][F] float
 *   abs_out: optional (may be NULL) sum of |w*x| per output, for condition-aware error bounds
 *   acc_mode 0: accumulate in double, round once; 1: accumulate in float.
 * Returns 0, or -1 on a bad geometry. */
int oracle_sparse_conv(const int* rowptr, const int* colidx, const float* values,
                       const float* x, int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad, float* out, float* abs_out, int acc_mode)
{
    int E = oracle_output_dim(H, pad, R, stride);
    int F = oracle_output_dim(W, pad, S, stride);
    if (E < 0 || F < 0 || N < 0 || C <= 0 || K <= 0) return -1;
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < E; ++i)
                for (int j = 0; j < F; ++j) {
                    double acc = 0.0, aabs = 0.0;
                    float accf = 0.0f;
                    for (int t = rowptr[k]; t < rowptr[k + 1]; ++t) {
                        int col = colidx[t];
                        int c = col / (R * S);
                        int r = (col / S) % R;
                        int s = col % S;
                        int y = i * stride + r - pad;
                        int xx = j * stride + s - pad;
                        if (y < 0 || y >= H || xx < 0 || xx >= W) continue; /* zero padding */
                        float xv = x[(((size_t)n * C + c) * H + y) * W + xx];
                        if (acc_mode == 0) {
                            acc += (double)values[t] * (double)xv;
                            aabs += fabs((double)values[t] * (double)xv);
                        } else {
                            accf += values[t] * xv;
                        }
                    }
                    size_t o = (((size_t)n * K + k) * E + i) * F + j;
                    out[o] = acc_mode == 0 ? (float)acc : accf;
                    if (abs_out) abs_out[o] = (float)aabs;
                }
    return 0;
}

/* Same sum at selected output coordinates only: pts is [npts][4] = (n,k,i,j);
 * results in double, not rounded to float. */
int oracle_sparse_conv_points(const int* rowptr, const int* colidx, const float* values,
                              const float* x, int N, int C, int H, int W, int K, int R, int S,
                              int stride, int pad, const int* pts, int npts, double* out)
{
    int E = oracle_output_dim(H, pad, R, stride);
    int F = oracle_output_dim(W, pad, S, stride);
    if (E < 0 || F < 0) return -1;
    for (int p = 0; p < npts; ++p) {
        int n = pts[4 * p], k = pts[4 * p + 1], i = pts[4 * p + 2], j = pts[4 * p + 3];
        if (n < 0 || n >= N || k < 0 || k >= K || i < 0 || i >= E || j < 0 || j >= F) return -1;
        double acc = 0.0;
        for (int t = rowptr[k]; t < rowptr[k + 1]; ++t) {
            int col = colidx[t];
            int c = col / (R * S), r = (col / S) % R, s = col % S;
            int y = i * stride + r - pad, xx = j * stride + s - pad;
            if (y < 0 || y >= H || xx < 0 || xx >= W) continue;
            acc += (double)values[t] * (double)x[(((size_t)n * C + c) * H + y) * W + xx];
        }
        out[p] = acc;
    }
    return 0;
}

/* Brute-force dense convolution of w*mask: the seven loops of eq. 1 over an
 * explicitly zero-padded copy of the input.  Exists only to pin
 * oracle_sparse_conv on small layers; shares no index arithmetic with it. */
int oracle_dense_conv7(const float* w, const unsigned char* mask, const float* x,
                       int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad, float* out)
{
    int E = oracle_output_dim(H, pad, R, stride);
    int F = oracle_output_dim(W, pad, S, stride);
    if (E < 0 || F < 0) return -1;
    int Hp = H + 2 * pad, Wp = W + 2 * pad;
    double* xp = (double*)calloc((size_t)N * C * Hp * Wp, sizeof(double));
    if (!xp) return -2;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int y = 0; y < H; ++y)
                for (int xx = 0; xx < W; ++xx)
                    xp[(((size_t)n * C + c) * Hp + y + pad) * Wp + xx + pad] =
                        x[(((size_t)n * C + c) * H + y) * W + xx];
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int i = 0; i < E; ++i)
                for (int j = 0; j < F; ++j) {
                    double acc = 0.0;
                    for (int c = 0; c < C; ++c)
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                size_t wi = (((size_t)k * C + c) * R + r) * S + s;
                                double wv = mask[wi] ? (double)w[wi] : 0.0;
                                acc += wv * xp[(((size_t)n * C + c) * Hp + i * stride + r) * Wp + j * stride + s];
                            }
                    out[(((size_t)n * K + k) * E + i) * F + j] = (float)acc;
                }
    free(xp);
    return 0;
}

/* ---------------------------------------------------------------- glue between layers */

void oracle_relu(float* x, long long n)
{
    for (long long i = 0; i < n; ++i)
        if (!(x[i] > 0.0f)) x[i] = 0.0f;
}

/* 2x2 max-pool, stride 2, floor output size; x [planes][H][W] -> out [planes][H/2][W/2]. */
void oracle_maxpool2(const float* x, long long planes, int H, int W, float* out)
{
    int Ho = H / 2, Wo = W / 2;
    for (long long p = 0; p < planes; ++p)
        for (int i = 0; i < Ho; ++i)
            for (int j = 0; j < Wo; ++j) {
                const float* b = x + ((size_t)p * H + 2 * i) * W + 2 * j;
                float m = b[0];
                if (b[1] > m) m = b[1];
                if (b[W] > m) m = b[W];
                if (b[W + 1] > m) m = b[W + 1];
                out[((size_t)p * Ho + i) * Wo + j] = m;
            }
}
