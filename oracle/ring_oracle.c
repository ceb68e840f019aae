/*
 * CPU oracle for replicated-share linear layers over the ring Z_{2^64}.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the yardstick the GPU library is
 * compared against; it is never part of the product path.  Only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may load it.  It shares
 * no code, header, table or helper with the HIP kernels.
 *
 * Everything here is the plain definition written out with C unsigned
 * 64-bit arithmetic, whose wraparound IS arithmetic mod 2^64 (paper Sec. III-B,
 * "Secret sharing": ring Z_n with n = 2^k, k = 64).  No blocking, no limb
 * splitting, no reordering of the three-term share product.  The only
 * concession to wall-clock time is an OpenMP "parallel for" over independent
 * output rows; integer sums mod 2^64 are exact in any order, so threading
 * cannot change a single bit.
 *
 * Pins (tests/test_oracle_*.py, run without a GPU): Python big-integer brute
 * force on tiny shapes, closed forms (identity, all-(-1), 2^32 squares to 0),
 * linearity, direct convolution == explicit patch matrix times weights,
 * 1x1 convolution == matmul, delta-kernel shift, output sizes printed in the
 * paper's AlexNet/VGG tables, share/reconstruct identity, sum of the three
 * parties' local products == product of the plaintext encodings, and the
 * decoded fixed-point product against an fp64 product; for the PRF part at
 * the end of this file (tests/test_oracle_prf.py): the FIPS-197 known-answer
 * vectors, the counter-mode word layout rebuilt block by block, stream
 * continuation, zero shares summing to zero, reshare keeping the opened value.
 * Every function here is covered by at least one of these pins.
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef uint64_t u64;

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Number of threads the loops below may use from now on (benchmark reporting only: no result
 * depends on it). */
void oracle_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n >= 1) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ---- fixed-point encoding (Sec. III-B "Fixed point representation") -------
 * A real x with t fractional bits is the integer nearest to x*2^t, embedded in
 * the ring as a two's-complement 64-bit word.  Ties go to even (the paper does
 * not fix the tie rule; this is the IEEE default of rint). */
void oracle_encode(const double *x, u64 *out, size_t n, int t)
{
    const double scale = ldexp(1.0, t);
    for (size_t i = 0; i < n; ++i)
        out[i] = (u64)(int64_t)rint(x[i] * scale);
}

/* Inverse map for a word at scale 2^bits: read it as signed, divide by 2^bits.
 * A product of two t-bit encodings is at scale 2^(2t) because the tensor
 * product is not truncated inside the linear layer (Sec. III-B,
 * "Convolutions and matrix multiplication", last paragraph). */
void oracle_decode(const u64 *z, double *out, size_t n, int bits)
{
    const double inv = ldexp(1.0, -bits);
    for (size_t i = 0; i < n; ++i)
        out[i] = (double)(int64_t)z[i] * inv;
}

/* ---- sharing (Sec. III-B "Secret sharing") --------------------------------
 * x = s0 + s1 + s2 in the ring.  Two words r0, r1 of caller-supplied
 * randomness fix s0 and s1; s2 is what is left.  Party i then holds the pair
 * (s_i, s_{(i+1) mod 3}). */
void oracle_share(const u64 *x, const u64 *r0, const u64 *r1,
                  u64 *s0, u64 *s1, u64 *s2, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        s0[i] = r0[i];
        s1[i] = r1[i];
        s2[i] = x[i] - r0[i] - r1[i];
    }
}

void oracle_reconstruct(const u64 *s0, const u64 *s1, const u64 *s2, u64 *out, size_t n)
{
    for (size_t i = 0; i < n; ++i)
        out[i] = s0[i] + s1[i] + s2[i];
}

/* ---- local linear operations (Sec. III-B "Linear operations") -------------
 * [[alpha*x + beta*y + gamma]] = (alpha*x1 + beta*y1 + gamma, alpha*x2 + beta*y2,
 * alpha*x3 + beta*y3): component-wise on every share, the public constant goes
 * into the first share only. */
void oracle_share_add(const u64 *xa, const u64 *xb, const u64 *ya, const u64 *yb,
                      u64 *za, u64 *zb, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        za[i] = xa[i] + ya[i];
        zb[i] = xb[i] + yb[i];
    }
}

void oracle_share_mul_public(const u64 *xa, const u64 *xb, u64 alpha,
                             u64 *za, u64 *zb, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        za[i] = alpha * xa[i];
        zb[i] = alpha * xb[i];
    }
}

/* Party `party` (0,1,2) holds (s_party, s_{party+1}).  The constant gamma is
 * added to share index 0 (the paper's x_1) only: that is the first component
 * of party 0 and the second component of party 2; party 1 holds neither. */
void oracle_share_add_public(const u64 *xa, const u64 *xb, u64 gamma, int party,
                             u64 *za, u64 *zb, size_t n)
{
    for (size_t i = 0; i < n; ++i) {
        za[i] = xa[i] + (party == 0 ? gamma : 0);
        zb[i] = xb[i] + (party == 2 ? gamma : 0);
    }
}

/* ---- ring matrix product ---------------------------------------------------
 * C[m][n] = sum_k A[m][k] * Y[n][k]  (mod 2^64).
 * A is [M,K] row-major; the right operand is stored as Y = [N,K] row-major
 * (K fastest, the usual weight layout of a fully connected layer), i.e. the
 * mathematical right factor is Y transposed. */
void oracle_matmul_u64(const u64 *A, const u64 *Y, u64 *C,
                       int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t m = 0; m < M; ++m)
        for (int64_t n = 0; n < N; ++n) {
            u64 acc = 0;
            for (int64_t k = 0; k < K; ++k)
                acc += A[m * K + k] * Y[n * K + k];
            C[m * N + n] = acc;
        }
}

/* ---- ring convolution ------------------------------------------------------
 * Cross-correlation with zero padding, as deep-learning layers define it:
 * Z[b][ho][wo][co] = sum_{r,s,c} X[b][ho*sh - ph + r][wo*sw - pw + s][c] * W[co][r][s][c]
 * with X read as 0 outside [0,H)x[0,W).  X is NHWC, W is [Cout,kh,kw,Cin],
 * Z is NHWC [B,Ho,Wo,Cout], Ho = floor((H + 2ph - kh)/sh) + 1 and likewise Wo.
 * Seven nested loops, no patch matrix. */
int64_t oracle_conv_out_dim(int64_t in, int64_t k, int64_t stride, int64_t pad)
{
    int64_t span = in + 2 * pad - k;
    if (span < 0) return 0;
    return span / stride + 1;
}

void oracle_conv2d_u64(const u64 *X, const u64 *W, u64 *Z,
                       int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                       int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t Ho = oracle_conv_out_dim(H, kh, sh, ph);
    const int64_t Wo = oracle_conv_out_dim(Wd, kw, sw, pw);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t b = 0; b < B; ++b)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t co = 0; co < Cout; ++co) {
                    u64 acc = 0;
                    for (int64_t r = 0; r < kh; ++r) {
                        const int64_t hi = ho * sh - ph + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int64_t s = 0; s < kw; ++s) {
                            const int64_t wi = wo * sw - pw + s;
                            if (wi < 0 || wi >= Wd) continue;
                            for (int64_t c = 0; c < Cin; ++c)
                                acc += X[((b * H + hi) * Wd + wi) * Cin + c] *
                                       W[((co * kh + r) * kw + s) * Cin + c];
                        }
                    }
                    Z[((b * Ho + ho) * Wo + wo) * Cout + co] = acc;
                }
}

/* ---- one party's local product (Sec. III-B "Multiplication" and
 * "Convolutions and matrix multiplication") ---------------------------------
 * z_i = x_i*y_i + x_{i+1}*y_i + x_i*y_{i+1}: three separate products, the
 * activation always on the left, then two ring additions.  The result is one
 * component of a 3-out-of-3 additive sharing of x*y: not re-shared, not
 * truncated.  Returns 0, or -1 if scratch memory could not be obtained. */
int oracle_party_matmul(const u64 *x_i, const u64 *x_ip1, const u64 *y_i, const u64 *y_ip1,
                        u64 *z_i, int64_t M, int64_t N, int64_t K)
{
    const size_t n = (size_t)M * (size_t)N;
    u64 *t1 = (u64 *)malloc(n * sizeof(u64)), *t2 = (u64 *)malloc(n * sizeof(u64));
    if (!t1 || !t2) { free(t1); free(t2); return -1; }
    oracle_matmul_u64(x_i,   y_i,   z_i, M, N, K);
    oracle_matmul_u64(x_ip1, y_i,   t1,  M, N, K);
    oracle_matmul_u64(x_i,   y_ip1, t2,  M, N, K);
    for (size_t j = 0; j < n; ++j) z_i[j] = z_i[j] + t1[j] + t2[j];
    free(t1); free(t2);
    return 0;
}

int oracle_party_conv2d(const u64 *x_i, const u64 *x_ip1, const u64 *w_i, const u64 *w_ip1,
                        u64 *z_i,
                        int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                        int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t Ho = oracle_conv_out_dim(H, kh, sh, ph);
    const int64_t Wo = oracle_conv_out_dim(Wd, kw, sw, pw);
    const size_t n = (size_t)B * (size_t)Ho * (size_t)Wo * (size_t)Cout;
    u64 *t1 = (u64 *)malloc(n * sizeof(u64)), *t2 = (u64 *)malloc(n * sizeof(u64));
    if (!t1 || !t2) { free(t1); free(t2); return -1; }
    oracle_conv2d_u64(x_i,   w_i,   z_i, B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_u64(x_ip1, w_i,   t1,  B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_u64(x_i,   w_ip1, t2,  B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    for (size_t j = 0; j < n; ++j) z_i[j] = z_i[j] + t1[j] + t2[j];
    free(t1); free(t2);
    return 0;
}

/* ---- backward products of a convolution layer (Sec. III-C: the gradients of a
 * linear / convolution layer are linear functions of the incoming gradient and are
 * evaluated with the same share protocols) --------------------------------------
 * For Z = conv(X, W) the two gradients are the adjoints of the map in each argument,
 * written here as the forward loop nest with the roles of "read" and "accumulate"
 * exchanged: every forward term X[b,hi,wi,c] * W[co,r,s,c] -> Z[b,ho,wo,co] becomes
 *   input gradient : G[b,ho,wo,co] * W[co,r,s,c] -> DX[b,hi,wi,c]
 *   weight gradient: G[b,ho,wo,co] * X[b,hi,wi,c] -> DW[co,r,s,c]
 * over Z_{2^64}.  G has the shape of Z; DX the shape of X; DW the shape of W. */
void oracle_conv2d_dgrad_u64(const u64 *G, const u64 *W, u64 *DX,
                             int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                             int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t Ho = oracle_conv_out_dim(H, kh, sh, ph);
    const int64_t Wo = oracle_conv_out_dim(Wd, kw, sw, pw);
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < B; ++b) {            /* images do not share entries of DX */
        for (int64_t j = 0; j < H * Wd * Cin; ++j) DX[b * H * Wd * Cin + j] = 0;
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t co = 0; co < Cout; ++co) {
                    const u64 g = G[((b * Ho + ho) * Wo + wo) * Cout + co];
                    for (int64_t r = 0; r < kh; ++r) {
                        const int64_t hi = ho * sh - ph + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int64_t s = 0; s < kw; ++s) {
                            const int64_t wi = wo * sw - pw + s;
                            if (wi < 0 || wi >= Wd) continue;
                            for (int64_t c = 0; c < Cin; ++c)
                                DX[((b * H + hi) * Wd + wi) * Cin + c] +=
                                    g * W[((co * kh + r) * kw + s) * Cin + c];
                        }
                    }
                }
    }
}

void oracle_conv2d_wgrad_u64(const u64 *G, const u64 *X, u64 *DW,
                             int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                             int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t Ho = oracle_conv_out_dim(H, kh, sh, ph);
    const int64_t Wo = oracle_conv_out_dim(Wd, kw, sw, pw);
#pragma omp parallel for schedule(static)
    for (int64_t co = 0; co < Cout; ++co) {      /* output channels do not share entries of DW */
        for (int64_t j = 0; j < kh * kw * Cin; ++j) DW[co * kh * kw * Cin + j] = 0;
        for (int64_t b = 0; b < B; ++b)
            for (int64_t ho = 0; ho < Ho; ++ho)
                for (int64_t wo = 0; wo < Wo; ++wo) {
                    const u64 g = G[((b * Ho + ho) * Wo + wo) * Cout + co];
                    for (int64_t r = 0; r < kh; ++r) {
                        const int64_t hi = ho * sh - ph + r;
                        if (hi < 0 || hi >= H) continue;
                        for (int64_t s = 0; s < kw; ++s) {
                            const int64_t wi = wo * sw - pw + s;
                            if (wi < 0 || wi >= Wd) continue;
                            for (int64_t c = 0; c < Cin; ++c)
                                DW[((co * kh + r) * kw + s) * Cin + c] +=
                                    g * X[((b * H + hi) * Wd + wi) * Cin + c];
                        }
                    }
                }
    }
}

/* One party's share of the two gradients: the three-term product with the incoming
 * gradient as the first factor, d_i = g_i*y_i + g_{i+1}*y_i + g_i*y_{i+1}, y the
 * filter (input gradient) or the layer input (weight gradient). */
int oracle_party_conv2d_dgrad(const u64 *g_i, const u64 *g_ip1, const u64 *w_i, const u64 *w_ip1,
                              u64 *dx_i,
                              int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                              int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const size_t n = (size_t)B * (size_t)H * (size_t)Wd * (size_t)Cin;
    u64 *t1 = (u64 *)malloc(n * sizeof(u64)), *t2 = (u64 *)malloc(n * sizeof(u64));
    if (!t1 || !t2) { free(t1); free(t2); return -1; }
    oracle_conv2d_dgrad_u64(g_i,   w_i,   dx_i, B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_dgrad_u64(g_ip1, w_i,   t1,   B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_dgrad_u64(g_i,   w_ip1, t2,   B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    for (size_t j = 0; j < n; ++j) dx_i[j] = dx_i[j] + t1[j] + t2[j];
    free(t1); free(t2);
    return 0;
}

int oracle_party_conv2d_wgrad(const u64 *g_i, const u64 *g_ip1, const u64 *x_i, const u64 *x_ip1,
                              u64 *dw_i,
                              int64_t B, int64_t H, int64_t Wd, int64_t Cin, int64_t Cout,
                              int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const size_t n = (size_t)Cout * (size_t)kh * (size_t)kw * (size_t)Cin;
    u64 *t1 = (u64 *)malloc(n * sizeof(u64)), *t2 = (u64 *)malloc(n * sizeof(u64));
    if (!t1 || !t2) { free(t1); free(t2); return -1; }
    oracle_conv2d_wgrad_u64(g_i,   x_i,   dw_i, B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_wgrad_u64(g_ip1, x_i,   t1,   B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    oracle_conv2d_wgrad_u64(g_i,   x_ip1, t2,   B, H, Wd, Cin, Cout, kh, kw, sh, sw, ph, pw);
    for (size_t j = 0; j < n; ++j) dw_i[j] = dw_i[j] + t1[j] + t2[j];
    free(t1); free(t2);
    return 0;
}

/* Single output element of one party's local matmul / conv, for spot checks on
 * shapes too large to compute in full.  Same three literal products. */
u64 oracle_party_matmul_at(const u64 *x_i, const u64 *x_ip1, const u64 *y_i, const u64 *y_ip1,
                           int64_t m, int64_t n, int64_t K)
{
    u64 p0 = 0, p1 = 0, p2 = 0;
    for (int64_t k = 0; k < K; ++k) p0 += x_i[m * K + k]   * y_i[n * K + k];
    for (int64_t k = 0; k < K; ++k) p1 += x_ip1[m * K + k] * y_i[n * K + k];
    for (int64_t k = 0; k < K; ++k) p2 += x_i[m * K + k]   * y_ip1[n * K + k];
    return p0 + p1 + p2;
}

static u64 conv_at(const u64 *X, const u64 *W, int64_t b, int64_t ho, int64_t wo, int64_t co,
                   int64_t H, int64_t Wd, int64_t Cin,
                   int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    u64 acc = 0;
    for (int64_t r = 0; r < kh; ++r) {
        const int64_t hi = ho * sh - ph + r;
        if (hi < 0 || hi >= H) continue;
        for (int64_t s = 0; s < kw; ++s) {
            const int64_t wi = wo * sw - pw + s;
            if (wi < 0 || wi >= Wd) continue;
            for (int64_t c = 0; c < Cin; ++c)
                acc += X[((b * H + hi) * Wd + wi) * Cin + c] * W[((co * kh + r) * kw + s) * Cin + c];
        }
    }
    return acc;
}

u64 oracle_party_conv2d_at(const u64 *x_i, const u64 *x_ip1, const u64 *w_i, const u64 *w_ip1,
                           int64_t b, int64_t ho, int64_t wo, int64_t co,
                           int64_t H, int64_t Wd, int64_t Cin,
                           int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    return conv_at(x_i,   w_i,   b, ho, wo, co, H, Wd, Cin, kh, kw, sh, sw, ph, pw)
         + conv_at(x_ip1, w_i,   b, ho, wo, co, H, Wd, Cin, kh, kw, sh, sw, ph, pw)
         + conv_at(x_i,   w_ip1, b, ho, wo, co, H, Wd, Cin, kh, kw, sh, sw, ph, pw);
}

/* =========================================================================
 * Zero shares from a PRF, and the reshare step (Sec. III-B "Protocol
 * initialization" and "Multiplication"; Sec. IV "Pseudorandom generators on
 * the GPU": AES is the PRF).
 *
 * Party P_i holds its own key k_i and its predecessor's key k_{i-1}.  The j-th
 * zero share is alpha_i[j] = F(k_i, j) - F(k_{i-1}, j) (mod 2^64); over the
 * three parties the terms telescope to 0.  After the local product, P_i
 * re-randomises its additive share as z_i + alpha_i before sending it on.
 *
 * Reading adopted where the paper is silent (it only says "AES as the PRF"):
 * F(k, j) is AES-128 in counter mode.  The 16-byte input block holds the block
 * index b = j >> 1 as a little-endian 64-bit integer in bytes 0..7 and a
 * caller-chosen 64-bit nonce (little-endian) in bytes 8..15; F(k, j) is the
 * little-endian 64-bit integer formed by bytes 0..7 of the ciphertext for even
 * j and bytes 8..15 for odd j.
 *
 * AES itself is FIPS-197 written out byte by byte: S-box from the field inverse
 * in GF(2^8) mod x^8+x^4+x^3+x+1 followed by the affine map, KeyExpansion,
 * SubBytes / ShiftRows / MixColumns / AddRoundKey.  Pinned by the FIPS-197
 * Appendix C.1 vector in the tests.
 * ========================================================================= */
static uint8_t gf_mul(uint8_t a, uint8_t b)
{
    uint8_t p = 0;
    for (int i = 0; i < 8; ++i) {
        if (b & 1) p ^= a;
        const uint8_t carry = a & 0x80;
        a = (uint8_t)(a << 1);
        if (carry) a ^= 0x1B;
        b >>= 1;
    }
    return p;
}

static uint8_t aes_sbox_entry(uint8_t x)
{
    uint8_t inv = 0;
    if (x)
        for (int c = 1; c < 256; ++c)
            if (gf_mul(x, (uint8_t)c) == 1) { inv = (uint8_t)c; break; }
    uint8_t r = 0x63, b = inv;
    for (int i = 0; i < 5; ++i) {   /* b ^ rotl(b,1) ^ rotl(b,2) ^ rotl(b,3) ^ rotl(b,4) ^ 0x63 */
        r ^= b;
        b = (uint8_t)((b << 1) | (b >> 7));
    }
    return r;
}

static void aes_sbox_table(uint8_t sbox[256])
{
    for (int i = 0; i < 256; ++i) sbox[i] = aes_sbox_entry((uint8_t)i);
}

/* 11 round keys of 16 bytes, byte order as in the key (w[i] occupies bytes 4i..4i+3). */
static void aes128_expand(const uint8_t key[16], const uint8_t sbox[256], uint8_t rk[176])
{
    memcpy(rk, key, 16);
    uint8_t rcon = 1;
    for (int i = 4; i < 44; ++i) {
        uint8_t t[4];
        memcpy(t, rk + 4 * (i - 1), 4);
        if (i % 4 == 0) {
            const uint8_t t0 = t[0];
            t[0] = sbox[t[1]] ^ rcon; t[1] = sbox[t[2]]; t[2] = sbox[t[3]]; t[3] = sbox[t0];
            rcon = gf_mul(rcon, 2);
        }
        for (int b = 0; b < 4; ++b) rk[4 * i + b] = rk[4 * (i - 4) + b] ^ t[b];
    }
}

static void aes128_encrypt(const uint8_t rk[176], const uint8_t sbox[256], const uint8_t in[16], uint8_t out[16])
{
    uint8_t s[16];   /* state byte (row r, column c) at s[r + 4c], the order of the input bytes */
    for (int i = 0; i < 16; ++i) s[i] = in[i] ^ rk[i];
    for (int round = 1; round <= 10; ++round) {
        uint8_t t[16];
        for (int c = 0; c < 4; ++c)             /* SubBytes + ShiftRows: row r moves left by r */
            for (int r = 0; r < 4; ++r)
                t[r + 4 * c] = sbox[s[r + 4 * ((c + r) % 4)]];
        if (round < 10) {
            for (int c = 0; c < 4; ++c) {       /* MixColumns */
                const uint8_t a0 = t[4 * c], a1 = t[4 * c + 1], a2 = t[4 * c + 2], a3 = t[4 * c + 3];
                s[4 * c]     = gf_mul(a0, 2) ^ gf_mul(a1, 3) ^ a2 ^ a3;
                s[4 * c + 1] = a0 ^ gf_mul(a1, 2) ^ gf_mul(a2, 3) ^ a3;
                s[4 * c + 2] = a0 ^ a1 ^ gf_mul(a2, 2) ^ gf_mul(a3, 3);
                s[4 * c + 3] = gf_mul(a0, 3) ^ a1 ^ a2 ^ gf_mul(a3, 2);
            }
        } else {
            memcpy(s, t, 16);
        }
        for (int i = 0; i < 16; ++i) s[i] ^= rk[16 * round + i];
    }
    memcpy(out, s, 16);
}

/* One AES-128 block, for the published test vectors. */
void oracle_aes128_encrypt_block(const uint8_t key[16], const uint8_t in[16], uint8_t out[16])
{
    uint8_t sbox[256], rk[176];
    aes_sbox_table(sbox);
    aes128_expand(key, sbox, rk);
    aes128_encrypt(rk, sbox, in, out);
}

/* out[j] = F(key, first + j) for j < n. */
void oracle_prf_words(const uint8_t key[16], u64 nonce, u64 first, u64 *out, size_t n)
{
    uint8_t sbox[256], rk[176];
    aes_sbox_table(sbox);
    aes128_expand(key, sbox, rk);
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < (int64_t)n; ++j) {
        const u64 idx = first + (u64)j, block = idx >> 1;
        uint8_t in[16], ct[16];
        for (int b = 0; b < 8; ++b) {
            in[b] = (uint8_t)(block >> (8 * b));
            in[8 + b] = (uint8_t)(nonce >> (8 * b));
        }
        aes128_encrypt(rk, sbox, in, ct);
        u64 w = 0;
        for (int b = 0; b < 8; ++b) w |= (u64)ct[8 * (idx & 1) + b] << (8 * b);
        out[j] = w;
    }
}

/* alpha[j] = F(key_self, first + j) - F(key_prev, first + j). */
int oracle_zero_share(const uint8_t key_self[16], const uint8_t key_prev[16], u64 nonce, u64 first,
                      u64 *alpha, size_t n)
{
    u64 *t = (u64 *)malloc((n ? n : 1) * sizeof(u64));
    if (!t) return -1;
    oracle_prf_words(key_self, nonce, first, alpha, n);
    oracle_prf_words(key_prev, nonce, first, t, n);
    for (size_t j = 0; j < n; ++j) alpha[j] -= t[j];
    free(t);
    return 0;
}

/* out[j] = z[j] + alpha[j]: the blinded additive share P_i sends to P_{i+1}. */
int oracle_reshare(const u64 *z, const uint8_t key_self[16], const uint8_t key_prev[16], u64 nonce, u64 first,
                   u64 *out, size_t n)
{
    u64 *a = (u64 *)malloc((n ? n : 1) * sizeof(u64));
    if (!a) return -1;
    if (oracle_zero_share(key_self, key_prev, nonce, first, a, n)) { free(a); return -1; }
    for (size_t j = 0; j < n; ++j) out[j] = z[j] + a[j];
    free(a);
    return 0;
}

/* ---- rescaling after a product (Sec. III-B "Multiplication": the two-round share
 * truncation cited from ABY3, which the paper names but does not list) -------------
 * Reading adopted here.  The parties hold the blinded additive shares
 * z'_i = z_i + alpha_i of the product.  P_2 sends z'_2 to P_1 (round 1), so that
 * (z'_0, z'_1 + z'_2) is a two-party additive sharing of z held by P_0 and P_1.  Each
 * of the two divides its summand by 2^d as a SIGNED integer, rounding down (an
 * arithmetic shift), which changes the shared value by at most one unit in the last
 * place unless the two summands wrap, an event of probability about |z| / 2^63.  P_1
 * and P_2 share the key k_1 and draw r_j = F(k_1, j) from it.  The new shares are
 *   s_0 = (z'_0) >> d,   s_1 = ((z'_1 + z'_2) >> d) - r,   s_2 = r,
 * and P_1 sends s_1 to P_0, P_0 sends s_0 to P_2 (round 2), which restores the
 * replicated form (s_i, s_{i+1}).
 *
 * One routine covers every party's local step:
 *   out[j] = asr64(z[j] + alpha[j] + (msg ? msg[j] : 0), d) - (key_mask ? F(key_mask, first + j) : 0)
 * with alpha[j] = F(key_self, first + j) - F(key_prev, first + j) under `nonce` and the
 * mask stream under `mask_nonce`.  d in [0, 63]. */
static u64 asr64(u64 v, int d)
{
    /* floor(v / 2^d) for v read as a two's-complement integer, without relying on the
     * implementation-defined right shift of negative values */
    if (d == 0) return v;
    const u64 shifted = v >> d;
    const u64 sign_fill = (v >> 63) ? (~(u64)0) << (64 - d) : 0;
    return shifted | sign_fill;
}

int oracle_trunc1_local(const u64 *z, const u64 *msg, const uint8_t key_self[16], const uint8_t key_prev[16],
                        u64 nonce, u64 first, int d, const uint8_t *key_mask, u64 mask_nonce,
                        u64 *out, size_t n)
{
    if (d < 0 || d > 63) return -2;
    u64 *a = (u64 *)malloc((n ? n : 1) * sizeof(u64)), *r = (u64 *)malloc((n ? n : 1) * sizeof(u64));
    if (!a || !r) { free(a); free(r); return -1; }
    if (oracle_zero_share(key_self, key_prev, nonce, first, a, n)) { free(a); free(r); return -1; }
    if (key_mask) oracle_prf_words(key_mask, mask_nonce, first, r, n);
    for (size_t j = 0; j < n; ++j) {
        const u64 sum = z[j] + a[j] + (msg ? msg[j] : 0);
        out[j] = asr64(sum, d) - (key_mask ? r[j] : 0);
    }
    free(a); free(r);
    return 0;
}

/* ---- binary replicated shares (Sec. III-B "Most significant bit") -------------------
 * A 64-bit word holds 64 independent bits, each shared as v = v_0 ^ v_1 ^ v_2 with
 * P_i holding (v_i, v_{i+1}).  XOR gates are local (share by share).  An AND gate is
 * the multiplication protocol over Z_2: P_i computes
 *   z_i = (x_i & y_i) ^ (x_{i+1} & y_i) ^ (x_i & y_{i+1}),
 * an XOR-sharing of x & y among the three parties, blinds it with a zero share
 *   beta_i[j] = F(k_i, j) ^ F(k_{i-1}, j)      (the three beta XOR to zero)
 * and passes it on.  The addition circuit that turns the arithmetic shares into
 * binary shares of their sum is a sequence of such gates on whole words. */
void oracle_bshare_and(const u64 *x_i, const u64 *x_ip1, const u64 *y_i, const u64 *y_ip1,
                       u64 *z_i, size_t n)
{
    for (size_t j = 0; j < n; ++j) {
        const u64 t0 = x_i[j] & y_i[j];
        const u64 t1 = x_ip1[j] & y_i[j];
        const u64 t2 = x_i[j] & y_ip1[j];
        z_i[j] = t0 ^ t1 ^ t2;
    }
}

int oracle_bzero_share(const uint8_t key_self[16], const uint8_t key_prev[16], u64 nonce, u64 first,
                       u64 *beta, size_t n)
{
    u64 *t = (u64 *)malloc((n ? n : 1) * sizeof(u64));
    if (!t) return -1;
    oracle_prf_words(key_self, nonce, first, beta, n);
    oracle_prf_words(key_prev, nonce, first, t, n);
    for (size_t j = 0; j < n; ++j) beta[j] ^= t[j];
    free(t);
    return 0;
}

/* =========================================================================
 * Other local linear-layer pieces on replicated shares.
 * ========================================================================= */

/* Element-wise local step of the multiplication protocol (Sec. III-B
 * "Multiplication"): z_i[j] = x_i[j] y_i[j'] + x_{i+1}[j] y_i[j'] + x_i[j] y_{i+1}[j'],
 * with j' = j mod period.  period == n is the plain element-wise product;
 * a smaller period broadcasts y along the leading dimensions, e.g. one secret
 * scale per channel of an NHWC tensor (batch normalisation at inference is such
 * an affine map with secret-shared parameters, Sec. V footnote on batch norm). */
void oracle_party_mul(const u64 *x_i, const u64 *x_ip1, const u64 *y_i, const u64 *y_ip1,
                      u64 *z_i, size_t n, size_t period)
{
    for (size_t j = 0; j < n; ++j) {
        const size_t jp = j % period;
        const u64 t0 = x_i[j] * y_i[jp];
        const u64 t1 = x_ip1[j] * y_i[jp];
        const u64 t2 = x_i[j] * y_ip1[jp];
        z_i[j] = t0 + t1 + t2;
    }
}

/* Bias of a linear layer on shares (Sec. III-B "Linear operations": adding shared
 * values is local).  Forward: every row of z [rows, cols] gets the bias share b [cols]
 * added, component by component.  Backward: the bias gradient is the column sum of the
 * incoming gradient, again component by component. */
void oracle_share_bias_add(const u64 *xa, const u64 *xb, const u64 *ba, const u64 *bb,
                           u64 *za, u64 *zb, size_t rows, size_t cols)
{
    for (size_t r = 0; r < rows; ++r)
        for (size_t c = 0; c < cols; ++c) {
            za[r * cols + c] = xa[r * cols + c] + ba[c];
            zb[r * cols + c] = xb[r * cols + c] + bb[c];
        }
}

void oracle_share_col_sum(const u64 *xa, const u64 *xb, u64 *za, u64 *zb, size_t rows, size_t cols)
{
    for (size_t c = 0; c < cols; ++c) {
        u64 sa = 0, sb = 0;
        for (size_t r = 0; r < rows; ++r) {
            sa += xa[r * cols + c];
            sb += xb[r * cols + c];
        }
        za[c] = sa;
        zb[c] = sb;
    }
}

/* Window sums of an NHWC tensor, zero padded: the linear part of average
 * pooling (Sec. V "Average pooling": pooling by averaging is linear, hence local
 * on shares).  Applied to each component of a replicated pair separately.  The
 * average is this sum times the public constant 1/(kh*kw) in fixed point. */
void oracle_sum_pool2d(const u64 *X, u64 *Z, int64_t B, int64_t H, int64_t Wd, int64_t C,
                       int64_t kh, int64_t kw, int64_t sh, int64_t sw, int64_t ph, int64_t pw)
{
    const int64_t Ho = oracle_conv_out_dim(H, kh, sh, ph);
    const int64_t Wo = oracle_conv_out_dim(Wd, kw, sw, pw);
    for (int64_t b = 0; b < B; ++b)
        for (int64_t ho = 0; ho < Ho; ++ho)
            for (int64_t wo = 0; wo < Wo; ++wo)
                for (int64_t c = 0; c < C; ++c) {
                    u64 acc = 0;
                    for (int64_t r = 0; r < kh; ++r)
                        for (int64_t s = 0; s < kw; ++s) {
                            const int64_t hi = ho * sh - ph + r, wi = wo * sw - pw + s;
                            if (hi >= 0 && hi < H && wi >= 0 && wi < Wd)
                                acc += X[((b * H + hi) * Wd + wi) * C + c];
                        }
                    Z[((b * Ho + ho) * Wo + wo) * C + c] = acc;
                }
}
