/*
 * CPU oracle for low-bit matrix-vector multiplication by Redundant Segment
 * Reduction (RSR).  TEST INFRASTRUCTURE ONLY: the product (the HIP library)
 * never links, loads or calls anything in this file, and this file shares no
 * code with it.  Everything is plain, slow, single-threaded C in double
 * precision, written so it can be checked against the paper by eye.
 *
 * Conventions (paper, "System Overview": the product is M*v, the matrix is
 * split into horizontal blocks of k rows, and columns of a block that carry
 * the same k-entry pattern are grouped):
 *   M     row-major int8, rows x cols; binary entries {0,1}, ternary {-1,0,+1}
 *   v     length cols;  out length rows;  out = scale * M * v
 *   block b covers rows b*k .. b*k+k-1; rows past the end count as all-zero
 *   the pattern of column j in block b is the k entries M[b*k+r][j], r<k
 *
 * Readings where the paper is silent (kept identical in the product):
 *   - row r of a block is digit r of the pattern code, least significant first
 *   - binary code   = sum_r bit_r   * 2^r,            P = 2^k patterns
 *   - fused ternary = sum_r digit_r * 3^r, digit 0 for 0, 1 for +1, 2 for -1,
 *                     P = 3^k patterns (the paper's 4^k bucket space without
 *                     its unused symbol)
 *   - two-pass ternary = binary procedure on [M==+1], then on [M==-1]
 *   - columns keep ascending order inside a group ("Kernels Implementation":
 *     indices are sorted within each group), i.e. the counting sort is stable
 *
 * No function here is "parity unpinned": tests/test_oracle_*.py pin each one
 * to brute force, library routines, closed forms and a hand-worked example.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { MODE_BINARY = 0, MODE_POS = 1, MODE_NEG = 2, MODE_FUSED3 = 3 };

static int64_t ipow(int64_t base, int e) {
    int64_t p = 1;
    for (int i = 0; i < e; ++i) p *= base;
    return p;
}

/* Number of pattern codes for a mode and block height. */
int64_t rsr_oracle_num_patterns(int k, int mode) {
    return mode == MODE_FUSED3 ? ipow(3, k) : ipow(2, k);
}

/* The definition of the result: out[i] = scale * sum_j M[i][j] * v[j]
 * ("System Overview", problem definition). */
int rsr_oracle_dense(const int8_t *M, int64_t rows, int64_t cols,
                     const double *v, double scale, double *out) {
    for (int64_t i = 0; i < rows; ++i) {
        double acc = 0.0;
        for (int64_t j = 0; j < cols; ++j)
            acc += (double)M[i * cols + j] * v[j];
        out[i] = scale * acc;
    }
    return 0;
}

/* Digit that entry m contributes under a mode; -1 if m is not allowed. */
static int digit_of(int8_t m, int mode) {
    switch (mode) {
    case MODE_BINARY: return (m == 0) ? 0 : (m == 1) ? 1 : -1;
    case MODE_POS:    return (m == 1) ? 1 : (m == 0 || m == -1) ? 0 : -1;
    case MODE_NEG:    return (m == -1) ? 1 : (m == 0 || m == 1) ? 0 : -1;
    case MODE_FUSED3: return (m == 0) ? 0 : (m == 1) ? 1 : (m == -1) ? 2 : -1;
    }
    return -1;
}

/* Pattern encoding ("Kernels Implementation": each column's k entries in a
 * block form one discrete pattern).  code is [nb][cols]. Returns 2 on an
 * entry outside the alphabet. */
int rsr_oracle_encode(const int8_t *M, int64_t rows, int64_t cols, int k,
                      int mode, uint32_t *code) {
    int64_t nb = (rows + k - 1) / k;
    int64_t base = (mode == MODE_FUSED3) ? 3 : 2;
    for (int64_t b = 0; b < nb; ++b) {
        for (int64_t j = 0; j < cols; ++j) {
            int64_t c = 0, weight = 1;
            for (int r = 0; r < k; ++r) {
                int64_t i = b * k + r;
                int d = 0;                       /* padded rows are zero */
                if (i < rows) {
                    d = digit_of(M[i * cols + j], mode);
                    if (d < 0) return 2;
                }
                c += d * weight;
                weight *= base;
            }
            code[b * cols + j] = (uint32_t)c;
        }
    }
    return 0;
}

/* Counting sort of the columns of every block by pattern code ("Kernels
 * Implementation": counting sort over the discrete pattern space, O(n +
 * buckets) per block), producing the column permutation pi [nb][cols] and
 * the group boundaries off [nb][P+1].  Stable: equal codes keep ascending
 * column order. */
int rsr_oracle_sort(const uint32_t *code, int64_t nb, int64_t cols, int64_t P,
                    uint32_t *pi, uint32_t *off) {
    int64_t *cursor = (int64_t *)malloc((size_t)P * sizeof(int64_t));
    if (!cursor) return 4;
    for (int64_t b = 0; b < nb; ++b) {
        const uint32_t *cb = code + b * cols;
        uint32_t *ob = off + b * (P + 1);
        for (int64_t c = 0; c <= P; ++c) ob[c] = 0;
        for (int64_t j = 0; j < cols; ++j) ob[cb[j] + 1] += 1;   /* histogram */
        for (int64_t c = 0; c < P; ++c) ob[c + 1] += ob[c];      /* scan      */
        for (int64_t c = 0; c < P; ++c) cursor[c] = ob[c];
        for (int64_t j = 0; j < cols; ++j)                        /* placement */
            pi[b * cols + cursor[cb[j]]++] = (uint32_t)j;
    }
    free(cursor);
    return 0;
}

/* Aggregate phase for one block: u[c] = sum of v over the columns of group c
 * ("System Overview": vector entries of identical column segments are
 * aggregated before multiplication). */
void rsr_oracle_segment_sums(const uint32_t *pi_b, const uint32_t *off_b,
                             int64_t P, const double *v, double *u) {
    for (int64_t c = 0; c < P; ++c) {
        double s = 0.0;
        for (uint32_t t = off_b[c]; t < off_b[c + 1]; ++t) s += v[pi_b[t]];
        u[c] = s;
    }
}

/* Scatter phase for one block, i.e. the product u * B_k where row c of B_k
 * is pattern c written out: every group sum is distributed once to each
 * block row whose digit in the pattern is non-zero, with sign -1 for the
 * fused digit 2.  y has k entries. */
void rsr_oracle_expand(const double *u, int64_t P, int k, int mode, double *y) {
    int64_t base = (mode == MODE_FUSED3) ? 3 : 2;
    for (int r = 0; r < k; ++r) y[r] = 0.0;
    for (int64_t c = 0; c < P; ++c) {
        int64_t rest = c;
        for (int r = 0; r < k; ++r) {
            int d = (int)(rest % base);
            rest /= base;
            if (d == 1) y[r] += u[c];
            else if (d == 2) y[r] -= u[c];
        }
    }
}

/* Online phase for one pass: out[i] (+)= sign * scale * (RSR product).
 * sign lets the caller form M+ v - M- v for the two-pass ternary kind. */
int rsr_oracle_matvec_pass(const uint32_t *pi, const uint32_t *off,
                           int64_t rows, int64_t cols, int k, int mode,
                           const double *v, double sign_scale, int accumulate,
                           double *out) {
    int64_t P = rsr_oracle_num_patterns(k, mode);
    int64_t nb = (rows + k - 1) / k;
    double *u = (double *)malloc((size_t)P * sizeof(double));
    double y[64];
    if (!u || k > 64) { free(u); return 4; }
    for (int64_t b = 0; b < nb; ++b) {
        rsr_oracle_segment_sums(pi + b * cols, off + b * (P + 1), P, v, u);
        rsr_oracle_expand(u, P, k, mode, y);
        for (int r = 0; r < k; ++r) {
            int64_t i = b * k + r;
            if (i >= rows) break;                 /* padded rows are dropped */
            if (accumulate) out[i] += sign_scale * y[r];
            else            out[i]  = sign_scale * y[r];
        }
    }
    free(u);
    return 0;
}

/* Dense comparison format: 2 bits per entry, 4 entries per byte, entry j of
 * a row in bits 2*(j%4)..2*(j%4)+1 of byte j/4; 0 -> 00, +1 -> 01, -1 -> 11
 * (two's complement).  Rows are padded with zero entries to row_bytes. */
int rsr_oracle_pack2(const int8_t *M, int64_t rows, int64_t cols,
                     int64_t row_bytes, uint8_t *packed) {
    if (row_bytes * 4 < cols) return 1;
    memset(packed, 0, (size_t)(rows * row_bytes));
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            int8_t m = M[i * cols + j];
            if (m < -1 || m > 1) return 2;
            uint8_t two = (uint8_t)(m & 3);
            packed[i * row_bytes + j / 4] |= (uint8_t)(two << (2 * (j % 4)));
        }
    return 0;
}

int rsr_oracle_unpack2(const uint8_t *packed, int64_t rows, int64_t cols,
                       int64_t row_bytes, int8_t *M) {
    for (int64_t i = 0; i < rows; ++i)
        for (int64_t j = 0; j < cols; ++j) {
            uint8_t two = (packed[i * row_bytes + j / 4] >> (2 * (j % 4))) & 3;
            if (two == 2) return 2;               /* unused symbol */
            M[i * cols + j] = (two == 0) ? 0 : (two == 1) ? 1 : -1;
        }
    return 0;
}
