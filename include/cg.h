/*
 * cg.h -- replicated-share linear layers over the ring Z_{2^64} on one AMD MI355X.
 *
 * The library computes what ONE party of the three-party protocol computes
 * locally, between two communication steps, for a linear layer on 2-out-of-3
 * replicated secret shares (CryptGPU, Sec. III-B).  A secret x is split as
 * x = s_0 + s_1 + s_2 (mod 2^64); party i holds the pair (s_i, s_{i+1 mod 3}).
 * Ring elements are uint64_t; every operation is exact arithmetic mod 2^64.
 *
 * Conventions shared by all entry points
 *   - Every data pointer is DEVICE memory owned by the caller (8-byte aligned
 *     at least; 16-byte alignment lets the kernels use their widest loads).
 *     The library never allocates, frees or retains device memory and keeps
 *     no state between calls.
 *   - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *     Calls only enqueue work: on CG_OK the kernels have been launched, not
 *     finished.  Synchronise the stream before reading results on the host.
 *   - Arguments are validated on the host BEFORE any HIP call.  A failed
 *     validation returns a status other than CG_OK and launches nothing.
 *   - Outputs of cg_share_matmul / cg_share_conv2d must not overlap their
 *     inputs.  The element-wise calls may run in place (an output pointer equal
 *     to the input pointer of the same position); partial overlap is rejected.
 */
#ifndef CG_H
#define CG_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CG_API __attribute__((visibility("default")))

typedef enum {
    CG_OK = 0,
    CG_ERR_NULL = 1,        /* a required pointer is NULL */
    CG_ERR_SHAPE = 2,       /* a dimension is < 1, a product of dimensions overflows, or the
                               convolution has an empty output */
    CG_ERR_ALIGN = 3,       /* a pointer is not 8-byte aligned */
    CG_ERR_ALIAS = 4,       /* an output overlaps an input where that is not allowed */
    CG_ERR_UNSUPPORTED = 5, /* valid mathematics, but outside what the kernels address
                               (see each call) */
    CG_ERR_DEVICE = 6,      /* the HIP runtime reported an error at launch */
    CG_ERR_WORKSPACE = 7    /* the scratch memory passed to a *_ws call is too small */
} cg_status;

/* Human-readable name of a status; static storage, never freed. */
CG_API const char *cg_status_string(cg_status s);

/* Library version, major*10000 + minor*100 + patch. */
CG_API int cg_version(void);

/*
 * One party's local step of the share multiplication protocol, for a matrix
 * product (Sec. III-B, "Multiplication" and "Convolutions and matrix
 * multiplication"):
 *
 *     z_i = x_i * y_i  +  x_{i+1} * y_i  +  x_i * y_{i+1}      (mod 2^64)
 *
 * where "*" is the matrix product with the activation on the left.  Over the
 * three parties z_0 + z_1 + z_2 = x*y, so z_i is one component of a
 * 3-out-of-3 additive sharing.  It is NOT re-shared and NOT truncated: for
 * fixed-point operands with t fractional bits the result carries 2t.
 *
 *   x_i, x_ip1 : [M,K] row-major, the party's two shares of the left operand
 *   y_i, y_ip1 : [N,K] row-major (K fastest: the weight layout of a fully
 *                connected layer), the party's two shares of the right operand;
 *                the mathematical right factor is its transpose
 *   z_i        : [M,N] row-major, written in full
 *   M, N, K    : >= 1
 *
 * CG_ERR_UNSUPPORTED if K exceeds 2^30 or M or N exceeds 2^31-1.
 *
 * K and the two ways of addressing a row.  Up to K = 2^20 the kernel reads its
 * operands through buffer descriptors, whose 32-bit byte offsets and hardware
 * range check return zeros for ragged tiles without a branch (a block addresses
 * the up to 256 rows of its tile relative to the tile's first row, so
 * 256 * K * 8 bytes must stay below 2^31).  Longer rows take generators with
 * 64-bit addresses, 8-byte loads and explicit bounds: same result, bit for
 * bit, at a lower rate, and without the scratch-memory route (the *_ws and
 * *_static calls then compute as this call).  The longest contraction among
 * the networks the paper evaluates (Sec. IV-A: LeNet, AlexNet, VGG-16,
 * ResNet-50/101/152) is the 7*7*512 = 25088 inputs of ImageNet VGG-16's first
 * fully connected layer.  The convolution calls keep kh*kw*Cin <= 2^20; the
 * weight gradient, whose contraction runs over B*Ho*Wo output pixels, rebases
 * its descriptors slice by slice and accepts 2^30 (see cg_share_conv2d_wgrad).
 */
CG_API cg_status cg_share_matmul(const uint64_t *x_i, const uint64_t *x_ip1,
                          const uint64_t *y_i, const uint64_t *y_ip1,
                          uint64_t *z_i, int64_t M, int64_t N, int64_t K, void *stream);

/*
 * The same product with either operand stored transposed: the share products of
 * the backward pass of a fully connected layer are matrix products of the same
 * kind on gradients (Sec. III-C: linear-layer gradients are computed with the
 * same protocols).  With Z = X W^T the forward product (X [M,K], W [N,K]):
 *
 *   dX = dZ W    : cg_share_matmul_t(dZ.., W.., dX, M, K, N, 0, 1)   (W  is [N,K] = stored [K', N'])
 *   dW = dZ^T X  : cg_share_matmul_t(dZ.., X.., dW, N, K, M, 1, 1)   (dZ is [M,N] = stored [K', M'])
 *
 * In general z_i [M,N] is the three-term product of the left operand L [M,K] and
 * the right operand R [N,K] (contracted over K, as in cg_share_matmul), where
 *   trans_x = 0: x_i, x_ip1 hold L row-major [M,K];  trans_x = 1: they hold L^T, row-major [K,M];
 *   trans_y = 0: y_i, y_ip1 hold R row-major [N,K];  trans_y = 1: they hold R^T, row-major [K,N].
 * trans_x = trans_y = 0 is cg_share_matmul.  CG_ERR_SHAPE if a flag is not 0 or 1;
 * CG_ERR_UNSUPPORTED additionally if a transposed operand has more than 2^22 columns.
 */
CG_API cg_status cg_share_matmul_t(const uint64_t *x_i, const uint64_t *x_ip1,
                            const uint64_t *y_i, const uint64_t *y_ip1,
                            uint64_t *z_i, int64_t M, int64_t N, int64_t K,
                            int trans_x, int trans_y, void *stream);

/*
 * The same product with caller-supplied scratch memory (device memory, 16-byte
 * aligned, at least cg_share_matmul_workspace_bytes(M, N, K) bytes, not
 * overlapping any operand).  With scratch memory each share tensor is split
 * into its eight signed-byte digits ONCE, by a streaming pass that writes the
 * digits there, instead of once per output tile that needs it inside the product
 * kernel; the product kernel then only moves bytes.  Result and argument rules
 * are those of cg_share_matmul, bit for bit.  The scratch contents are
 * undefined afterwards and carry no state between calls.  When the digit route
 * does not apply (odd K, a pointer that is only 8-byte aligned, K above 2^20,
 * or a left operand of so few rows, at most 64, that the plain call's kernel for
 * such products is the faster one) the call
 * computes exactly as cg_share_matmul and does not touch the scratch memory;
 * cg_share_matmul_workspace_bytes then returns 0 (as it does for invalid sizes).
 * CG_ERR_WORKSPACE if workspace_bytes is too small, CG_ERR_NULL / CG_ERR_ALIGN /
 * CG_ERR_ALIAS for a missing, misaligned or overlapping workspace.
 */
CG_API size_t cg_share_matmul_workspace_bytes(int64_t M, int64_t N, int64_t K);

/*
 * 1 when, for these sizes (16-byte-aligned operands assumed), the route with scratch
 * memory is expected to be the faster one on MI355X, the conversion pass included; 0
 * when the plain call is, or when the sizes are invalid.  A measured rule of thumb
 * for callers that have scratch memory and want to pick per layer: large products
 * whose operands are small against M*N*K gain (square products about 15 %), skinny
 * or short ones lose.  Same for cg_share_conv2d_prefers_workspace below.
 */
CG_API int cg_share_matmul_prefers_workspace(int64_t M, int64_t N, int64_t K);

CG_API cg_status cg_share_matmul_ws(const uint64_t *x_i, const uint64_t *x_ip1,
                             const uint64_t *y_i, const uint64_t *y_ip1,
                             uint64_t *z_i, int64_t M, int64_t N, int64_t K,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * cg_share_matmul for callers that cannot allocate device memory or bring a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid allocation.  The digit planes of cg_share_matmul_ws go to a fixed
 * array of CG_STATIC_SCRATCH_BYTES bytes inside the library's device image
 * (one copy per GPU, held until the process ends); the call itself allocates and
 * frees nothing.  Result and argument rules are those of cg_share_matmul, bit
 * for bit.  CG_ERR_WORKSPACE when cg_share_matmul_workspace_bytes(M, N, K)
 * exceeds CG_STATIC_SCRATCH_BYTES (nothing is launched then); products the digit
 * route does not apply to (odd K, 8-byte-aligned pointers) run as
 * cg_share_matmul, whatever their size.  The array's address is looked up on the
 * first call on each device, which must be the current device, as for every
 * call here.  All calls on one GPU share the array and every call overwrites the part
 * it uses: calls that overlap in time on one GPU (different streams, or
 * threads) race and must be ordered by the caller.
 */
#define CG_STATIC_SCRATCH_BYTES (64u << 20)

CG_API cg_status cg_share_matmul_static(const uint64_t *x_i, const uint64_t *x_ip1,
                                 const uint64_t *y_i, const uint64_t *y_ip1,
                                 uint64_t *z_i, int64_t M, int64_t N, int64_t K,
                                 void *stream);

/*
 * Same local step for a 2-D convolution (Sec. III-B, "Convolutions and matrix
 * multiplication"), evaluated as an implicit matrix product: no patch matrix
 * is ever written to memory.  Convolution means cross-correlation with zero
 * padding, as neural-network layers define it:
 *
 *   Z[b][ho][wo][co] = sum_{r,s,c} X[b][ho*stride_h - pad_h + r][wo*stride_w - pad_w + s][c]
 *                                  * W[co][r][s][c]
 *
 * with X read as zero outside the image.  A zero in every share is a share of
 * zero, so padding each share with zeros pads the secret with zeros.
 *
 *   x_i, x_ip1 : NHWC [B,H,W,Cin]
 *   w_i, w_ip1 : [Cout,kh,kw,Cin]
 *   z_i        : NHWC [B,Ho,Wo,Cout], Ho = floor((H + 2*pad_h - kh)/stride_h) + 1, same for Wo
 *
 * No dilation, no groups.  CG_ERR_SHAPE if Ho or Wo would be < 1, a stride is
 * < 1 or a padding is negative.  CG_ERR_UNSUPPORTED if kh*kw*Cin exceeds 2^20,
 * if B*Ho*Wo or Cout exceeds 2^31-1, if a stride or padding exceeds 32767, or if
 * the images one 256-row block of outputs can touch ((255 / (Ho*Wo) + 2 of them,
 * at most B) exceed 2^31-1 bytes together.
 */
typedef struct {
    int64_t B, H, W, Cin, Cout, kh, kw, stride_h, stride_w, pad_h, pad_w;
} cg_conv2d_desc;

CG_API cg_status cg_share_conv2d(const uint64_t *x_i, const uint64_t *x_ip1,
                          const uint64_t *w_i, const uint64_t *w_ip1,
                          uint64_t *z_i, const cg_conv2d_desc *desc, void *stream);

/*
 * cg_share_conv2d with caller-supplied scratch memory; see cg_share_matmul_ws.
 * The digit route applies when Cin is a multiple of 32 (or the convolution is
 * 1x1, stride 1, unpadded with even Cin) and all pointers are 16-byte aligned.
 */
CG_API size_t cg_share_conv2d_workspace_bytes(const cg_conv2d_desc *desc);
CG_API int cg_share_conv2d_prefers_workspace(const cg_conv2d_desc *desc);

CG_API cg_status cg_share_conv2d_ws(const uint64_t *x_i, const uint64_t *x_ip1,
                             const uint64_t *w_i, const uint64_t *w_ip1,
                             uint64_t *z_i, const cg_conv2d_desc *desc,
                             void *workspace, size_t workspace_bytes, void *stream);

/*
 * The products above added to what z_i holds on entry: z_i <- z_i + (local product)
 * mod 2^64, everything else as cg_share_matmul / cg_share_conv2d (same argument
 * meaning, validation and errors; z_i is read as well as written, and still may not
 * overlap an input).  With z_i holding the party's zero share alpha_i (cg_zero_share:
 * it depends on no data, so it can be produced before the operands exist) the result
 * is z_i + alpha_i, the message of the multiplication protocol (Sec. III-B), formed
 * in the product's own fold with no further pass over z.  Also sums the products of
 * several operand pairs into one output.
 */
CG_API cg_status cg_share_matmul_acc(const uint64_t *x_i, const uint64_t *x_ip1,
                              const uint64_t *y_i, const uint64_t *y_ip1,
                              uint64_t *z_i, int64_t M, int64_t N, int64_t K, void *stream);

CG_API cg_status cg_share_conv2d_acc(const uint64_t *x_i, const uint64_t *x_ip1,
                              const uint64_t *w_i, const uint64_t *w_ip1,
                              uint64_t *z_i, const cg_conv2d_desc *desc, void *stream);

/*
 * cg_share_matmul computed the way the paper embeds ring products in floating point
 * (Sec. II-B): every word as four unsigned 16-bit blocks held in float64, the ten
 * block products whose weight stays below 2^64, on the float64 matrix instruction,
 * accumulators folded into the 64-bit result before they leave the exact range.
 * Same arguments, validation, errors and result (bit for bit) as cg_share_matmul,
 * except that K stops at 2^20 (CG_ERR_UNSUPPORTED beyond); several times slower.  A comparator: it exists so that the choice of 8-bit digits
 * on the integer matrix instruction is backed by a measurement, not to be called by
 * applications.
 */
CG_API cg_status cg_share_matmul_f64limb(const uint64_t *x_i, const uint64_t *x_ip1,
                                  const uint64_t *y_i, const uint64_t *y_ip1,
                                  uint64_t *z_i, int64_t M, int64_t N, int64_t K, void *stream);

/*
 * Backward products of a convolution layer on shares (Sec. III-C: the gradients of
 * a linear / convolution layer are linear functions of the incoming gradient and
 * are evaluated with the protocols of Sec. III-B, i.e. with the same three-term
 * local product).  `desc` is the descriptor of the FORWARD layer; G denotes the
 * gradient with respect to the layer output, NHWC [B,Ho,Wo,Cout].  Both gradients
 * are the adjoints of the forward map: every forward term
 * X[b][hi][wi][c] * W[co][r][s][c] -> Z[b][ho][wo][co] contributes
 *
 *   cg_share_conv2d_dgrad : G[b][ho][wo][co] * W[co][r][s][c] -> DX[b][hi][wi][c]
 *   cg_share_conv2d_wgrad : G[b][ho][wo][co] * X[b][hi][wi][c] -> DW[co][r][s][c]
 *
 * and the party's output is g_i*y_i + g_{i+1}*y_i + g_i*y_{i+1} with y the filter
 * (dgrad) or the layer input (wgrad): one additive share of the gradient, not
 * re-shared, not truncated.
 *
 *   g_i, g_ip1 : NHWC [B,Ho,Wo,Cout]
 *   w_i, w_ip1 : [Cout,kh,kw,Cin]        x_i, x_ip1 : NHWC [B,H,W,Cin]
 *   dx_i       : NHWC [B,H,W,Cin]        dw_i       : [Cout,kh,kw,Cin]
 *
 * All device pointers, 8-byte aligned, the output fully overwritten and disjoint
 * from the inputs (CG_ERR_ALIAS).  Nothing is written to memory besides the output:
 * the filter is read in place with its taps reversed, and the patch entries of the
 * weight gradient are gathered from the input.  The input gradient of a strided
 * layer runs one residue class (h mod stride_h, w mod stride_w) of the input
 * pixels at a time, each a unit-stride product with the filter taps that reach the
 * class (Cout a multiple of 32, 16-byte-aligned pointers, at most 64 classes; dx is
 * cleared first, pixels no tap reaches stay zero); other strided layers read the
 * gradient as if zeros stood between its pixels.  Shape errors as cg_share_conv2d.
 * CG_ERR_UNSUPPORTED: dgrad if kh*kw*Cout exceeds 2^20, B*H*W exceeds 2^31-1, the
 * gradient images one 256-row block can touch exceed 2^31-1 bytes, or (strided
 * layers, Cout not a multiple of 32, or 16-byte-unaligned pointers) the filter
 * exceeds 2^31-1 bytes; wgrad if B*Ho*Wo exceeds 2^30, Cout exceeds 2^22,
 * kh*kw*Cin exceeds 2^31-1 or the (31/(Ho*Wo) + 2) input images a run of 32
 * output pixels can touch exceed 2^31-1 bytes; either if a stride, padding or
 * window side exceeds 32767.  (A strided dgrad that runs class by class is held to
 * these limits per class, with the class's own tap and pixel counts, and falls back
 * to the other route when a class exceeds them.)
 */
CG_API cg_status cg_share_conv2d_dgrad(const uint64_t *g_i, const uint64_t *g_ip1,
                                const uint64_t *w_i, const uint64_t *w_ip1,
                                uint64_t *dx_i, const cg_conv2d_desc *desc, void *stream);

CG_API cg_status cg_share_conv2d_wgrad(const uint64_t *g_i, const uint64_t *g_ip1,
                                const uint64_t *x_i, const uint64_t *x_ip1,
                                uint64_t *dw_i, const cg_conv2d_desc *desc, void *stream);

/*
 * Local linear operations on a replicated pair (a = s_i, b = s_{i+1}), over n
 * elements (Sec. III-B, "Linear operations": shares of alpha*x + beta*y are
 * the same combination of the shares, component by component).
 *
 *   cg_share_add        : (za, zb) = (xa + ya, xb + yb)
 *   cg_share_mul_public : (za, zb) = (alpha*xa, alpha*xb), alpha a public ring element
 *   cg_share_add_public : adds the public ring element gamma to share index 0 only,
 *                         i.e. to the first component of party 0 and to the second
 *                         component of party 2; party 1's pair is copied unchanged.
 *                         party must be 0, 1 or 2 (CG_ERR_SHAPE otherwise).
 * n == 0 is allowed: the call returns CG_OK without looking at the pointers.
 */
CG_API cg_status cg_share_add(const uint64_t *xa, const uint64_t *xb,
                       const uint64_t *ya, const uint64_t *yb,
                       uint64_t *za, uint64_t *zb, size_t n, void *stream);

CG_API cg_status cg_share_mul_public(const uint64_t *xa, const uint64_t *xb, uint64_t alpha,
                              uint64_t *za, uint64_t *zb, size_t n, void *stream);

CG_API cg_status cg_share_add_public(const uint64_t *xa, const uint64_t *xb, uint64_t gamma, int party,
                              uint64_t *za, uint64_t *zb, size_t n, void *stream);

/*
 * Element-wise local step of the share multiplication (Sec. III-B "Multiplication"):
 *
 *     z_i[j] = x_i[j]*y_i[j'] + x_{i+1}[j]*y_i[j'] + x_i[j]*y_{i+1}[j'],   j' = j mod period
 *
 * over n elements; like cg_share_matmul the result is one component of a
 * 3-out-of-3 additive sharing of the element-wise product, not re-shared, not
 * truncated.  period == n is the plain element-wise product; a smaller period
 * (a divisor of n) broadcasts y, e.g. one secret scale per channel of an NHWC
 * tensor with period = C, which is how a batch normalisation with secret-shared
 * parameters is applied at inference (an affine map; add the shift with
 * cg_share_add).  y_i, y_ip1 have `period` elements.  z_i may equal x_i or x_ip1
 * (and y_i or y_ip1 when period == n).  CG_ERR_SHAPE if period is 0 or does not
 * divide n.  n == 0 returns CG_OK.
 */
CG_API cg_status cg_share_mul(const uint64_t *x_i, const uint64_t *x_ip1,
                       const uint64_t *y_i, const uint64_t *y_ip1,
                       uint64_t *z_i, size_t n, size_t period, void *stream);

/*
 * Bias of a linear layer on replicated pairs (Sec. III-B "Linear operations": sums
 * of shared values are computed share by share, locally).
 *
 *   cg_share_bias_add : (za, zb)[j] = (xa[j] + ba[j mod period], xb[j] + bb[j mod period]),
 *                       j < n: the bias pair [period] broadcast over the rows of a
 *                       [n / period, period] tensor (FC output, or NHWC with period = C).
 *                       period must divide n (CG_ERR_SHAPE).  za/zb may equal xa/xb.
 *   cg_share_col_sum  : (za, zb)[c] = sum over r < rows of (xa, xb)[r * cols + c]: the bias
 *                       gradient of the layer from the incoming gradient [rows, cols].
 *                       Outputs [cols] must not overlap the inputs or each other.
 *
 * When the first operand is the party's additive product share z_i rather than a pair,
 * pass it for both components and ignore zb.  n == 0 / cols == 0 return CG_OK.
 */
CG_API cg_status cg_share_bias_add(const uint64_t *xa, const uint64_t *xb, const uint64_t *ba,
                            const uint64_t *bb, uint64_t *za, uint64_t *zb, size_t n, size_t period,
                            void *stream);

CG_API cg_status cg_share_col_sum(const uint64_t *xa, const uint64_t *xb, uint64_t *za, uint64_t *zb,
                           size_t rows, size_t cols, void *stream);

/*
 * Window sums of both components of a replicated pair, NHWC, zero padded: the
 * linear, hence local, part of average pooling (Sec. V "Average pooling").
 *   z[b][ho][wo][c] = sum over the kh x kw window at (ho*stride_h - pad_h, wo*stride_w - pad_w) of x[b][.][.][c]
 * Output [B,Ho,Wo,C] with Ho = floor((H + 2*pad_h - kh)/stride_h) + 1, same for Wo.
 * The average is this sum times the public fixed-point constant 1/(kh*kw)
 * (cg_share_mul_public) followed by the protocol's truncation.  Outputs must not
 * overlap inputs or each other.
 */
typedef struct {
    int64_t B, H, W, C, kh, kw, stride_h, stride_w, pad_h, pad_w;
} cg_pool2d_desc;

CG_API cg_status cg_share_sum_pool2d(const uint64_t *xa, const uint64_t *xb, uint64_t *za, uint64_t *zb,
                              const cg_pool2d_desc *desc, void *stream);

/*
 * Zero shares and the reshare step (Sec. III-B "Protocol initialization" and
 * "Multiplication"; Sec. IV "Pseudorandom generators on the GPU").
 *
 * Party P_i holds its own PRF key k_i (key_self) and its predecessor's k_{i-1}
 * (key_prev); both are 16-byte AES-128 keys in HOST memory, read during the call.
 *
 *   cg_zero_share : alpha[j] = F(k_i, first + j) - F(k_{i-1}, first + j)   (mod 2^64), j < n
 *   cg_reshare    : out[j]   = z_i[j] + alpha[j]: the blinded additive share that
 *                   P_i sends to P_{i+1} after a share product; out may equal z_i.
 *
 * Over the three parties (keys k_0, k_1, k_2, predecessors taken cyclically) the
 * alpha_i sum to zero for every index, so the blinded shares still open to the
 * product.  The paper fixes AES as the PRF and nothing else; here F(k, j) is
 * AES-128 in counter mode: the input block is (j >> 1) as a 64-bit little-endian
 * integer followed by `nonce` as a 64-bit little-endian integer, and F(k, j) is
 * ciphertext bytes 0..7 (even j) or 8..15 (odd j) read as a little-endian integer.
 * `first` lets a caller continue a stream: never reuse (nonce, index) pairs under
 * the same keys.  n == 0 returns CG_OK.  alpha / z_i / out are device pointers.
 */
CG_API cg_status cg_zero_share(const uint8_t *key_self, const uint8_t *key_prev, uint64_t nonce,
                        uint64_t first, uint64_t *alpha, size_t n, void *stream);

CG_API cg_status cg_reshare(const uint64_t *z_i, const uint8_t *key_self, const uint8_t *key_prev,
                     uint64_t nonce, uint64_t first, uint64_t *out, size_t n, void *stream);

/*
 * Rescaling after a product (Sec. III-B "Multiplication": after a product of
 * fixed-point encodings the parties divide by the scaling factor with the two-round
 * share truncation of ABY3, which the paper names without listing its steps).  The
 * reading implemented here, for parties P_0, P_1, P_2 holding the additive product
 * shares z_0, z_1, z_2 and PRF keys as above (P_i: k_i and k_{i-1}):
 *
 *   round 1   P_2 sends m = z_2 + alpha_2 to P_1                     (cg_reshare)
 *   local     P_0: s_0 = asr(z_0 + alpha_0, d)
 *             P_1: s_1 = asr(z_1 + alpha_1 + m, d) - F(k_1, first + j)   (mask stream)
 *             P_1, P_2: s_2 = F(k_1, first + j)                      (cg_prf_words)
 *   round 2   P_1 sends s_1 to P_0, P_0 sends s_0 to P_2
 *
 * where asr is the signed (two's-complement, rounding down) shift of the 64-bit
 * word.  P_i ends with (s_i, s_{i+1}).  The opened result differs from
 * floor(z / 2^d) by at most one unit in the last place unless the two summands
 * z_0 + alpha_0 and z_1 + alpha_1 + m wrap as signed integers, which happens with
 * probability about |z| / 2^63 per element.
 *
 *   cg_trunc1_local : out[j] = asr(z_i[j] + alpha[j] + (msg ? msg[j] : 0), d)
 *                              - (key_mask ? F(key_mask, first + j) : 0),   j < n
 *       alpha as in cg_zero_share under `nonce`; the mask stream uses the same
 *       indices under `mask_nonce`, which must differ from `nonce` when key_mask is
 *       one of the two alpha keys (the mask would be a term of alpha itself and blind
 *       nothing: CG_ERR_SHAPE).  msg and key_mask may be NULL.  d in [0, 63]
 *       (CG_ERR_SHAPE otherwise).  out may equal z_i or msg; partial overlap is
 *       CG_ERR_ALIAS.
 *   cg_prf_words    : out[j] = F(key, first + j), j < n: the raw PRF stream.
 *
 * Keys are 16-byte AES-128 keys in HOST memory; z_i, msg, out are device pointers,
 * 8-byte aligned.  n == 0 returns CG_OK.
 */
CG_API cg_status cg_trunc1_local(const uint64_t *z_i, const uint64_t *msg,
                          const uint8_t *key_self, const uint8_t *key_prev, uint64_t nonce,
                          uint64_t first, int d, const uint8_t *key_mask, uint64_t mask_nonce,
                          uint64_t *out, size_t n, void *stream);

CG_API cg_status cg_prf_words(const uint8_t *key, uint64_t nonce, uint64_t first,
                       uint64_t *out, size_t n, void *stream);

/*
 * Gates on BINARY replicated shares (Sec. III-B "Most significant bit": the sign of
 * a shared value is found by adding its three arithmetic shares in a Boolean addition
 * circuit over binary shares built from bitwise AND and XOR gates).  A
 * 64-bit word carries 64 independent bits, each shared as v = v_0 ^ v_1 ^ v_2 with
 * P_i holding the pair (v_i, v_{i+1}); n counts words.
 *
 *   cg_bshare_xor  : (za, zb) = (xa ^ ya, xb ^ yb)                      XOR gate, local
 *   cg_bshare_and  : z_i = (x_i & y_i) ^ (x_ip1 & y_i) ^ (x_i & y_ip1)  local step of an AND
 *                    gate: the multiplication protocol over Z_2; the three z_i XOR to x & y
 *   cg_bshare_prefix_stage : one stage of a parallel-prefix adder on (propagate, generate)
 *                    words, two AND gates fused with the word shifts:
 *                      g_out = g_i ^ and3(p, g << shift),  p_out = and3(p, p << shift)
 *                    with and3 the three-term formula of cg_bshare_and applied to the
 *                    pairs; p_out may be NULL (last stage).  shift in [1, 63].
 *   cg_bzero_share : beta[j] = F(k_i, first + j) ^ F(k_{i-1}, first + j): the three
 *                    parties' beta XOR to zero (keys and F as for cg_zero_share)
 *   cg_breshare    : out[j] = z_i[j] ^ beta[j], the blinded share passed on after an AND
 *
 * The paper gives no gate list for the circuit; the tests assemble this one from the
 * calls above: the arithmetic shares x_0, x_1, x_2 are read as binary sharings
 * (x_0,0,0), (0,x_1,0), (0,0,x_2); a carry-save step S = A^B^C,
 * carry = ((A^C) & (B^C)) ^ C reduces them to two addends; a 64-bit parallel-prefix
 * adder (first generate word S & (carry << 1), then stages with shifts 1..32) adds
 * those: eight rounds of AND gates in all.  Bit 63 of the sum is the sign.
 *
 * Device pointers, 8-byte aligned; outputs may coincide with inputs element for
 * element but not partially overlap, and two outputs must be disjoint (CG_ERR_ALIAS).
 * n == 0 returns CG_OK.
 */
CG_API cg_status cg_bshare_xor(const uint64_t *xa, const uint64_t *xb, const uint64_t *ya,
                        const uint64_t *yb, uint64_t *za, uint64_t *zb, size_t n, void *stream);

CG_API cg_status cg_bshare_and(const uint64_t *x_i, const uint64_t *x_ip1, const uint64_t *y_i,
                        const uint64_t *y_ip1, uint64_t *z_i, size_t n, void *stream);

CG_API cg_status cg_bshare_prefix_stage(const uint64_t *p_i, const uint64_t *p_ip1,
                                 const uint64_t *g_i, const uint64_t *g_ip1, int shift,
                                 uint64_t *p_out, uint64_t *g_out, size_t n, void *stream);

/*
 * The same sign bit from a circuit pruned to that one output, on BIT PLANES: with 64 m
 * elements, plane b is m words holding bit b of every element (element 64 w + e in bit e of
 * word w).  Gates then cost in proportion to the bit positions they touch.
 *
 *   cg_bit_transpose64     : dst [64][m] = planes of src [64 m] (a 64 x 64 bit transpose per
 *                            block of 64 words; local, applied by a party to each of its shares).
 *                            n must be a multiple of 64 (CG_ERR_SHAPE); dst must not overlap src.
 *   cg_bshare_carry_level  : one level of the carry tree: inputs [2 planes_out][m], outputs
 *                            [planes_out][m]; output plane j merges the neighbouring segments
 *                            hi = plane 2j+1 and lo = plane 2j,
 *                              g_out = g_hi ^ and3(p_hi, g_lo),   p_out = and3(p_hi, p_lo)
 *                            (and3 = the three-term AND of cg_bshare_and); p_out may be NULL at
 *                            the root.  Outputs must not overlap the inputs or each other.
 *   cg_bits_unpack         : out[i] = bit (i mod 64) of plane[i / 64], i < n: one word per element
 *                            again, e.g. to read a share of the sign bit as an arithmetic share.
 *
 * Circuit assembled by the tests: transpose; carry-save step and first generate word on all 64
 * planes (cg_bshare_and); the leaves of the tree are the (propagate, generate) planes moved up
 * one bit position (the carry into bit 63 is the generate of bits 0..62); six levels on 32, 16,
 * 8, 4, 2, 1 planes; sign = propagate plane 63 ^ root generate.  254 plane-sized AND gates
 * instead of the 832 of the word-parallel adder, hence 3.3 times fewer PRF words.
 */
/*
 * Adder cells on binary sharings, one party's local step each (fused forms of the gates above
 * that read every operand once):
 *
 *   cg_bshare_csa        : carry-save (full) adder of three sharings A, B, C given as pairs:
 *                          sum pair (s_i, s_ip1) = A ^ B ^ C, and the party's XOR share of the carry
 *                          majority(A, B, C) = ((A ^ C) & (B ^ C)) ^ C before blinding, i.e.
 *                          and3(A ^ C, B ^ C) ^ c_i.  Bit by bit a + b + c = sum + 2 carry.  Any of the
 *                          six input pointers may be NULL: that component is zero everywhere and is
 *                          not read (the three summands of the sign-bit circuit are sharings with a
 *                          single non-zero share, so a party holds two non-zero components of six).
 *   cg_bshare_half_adder : propagate pair (p_i, p_ip1) = S ^ T and the party's XOR share of the
 *                          generate word and3(S, T) before blinding.
 *
 * Outputs may coincide element for element with inputs but not partially overlap them, and must be
 * disjoint from each other (CG_ERR_ALIAS).
 */
CG_API cg_status cg_bshare_csa(const uint64_t *a_i, const uint64_t *a_ip1, const uint64_t *b_i,
                        const uint64_t *b_ip1, const uint64_t *c_i, const uint64_t *c_ip1,
                        uint64_t *s_i, uint64_t *s_ip1, uint64_t *carry_i, size_t n, void *stream);

CG_API cg_status cg_bshare_half_adder(const uint64_t *s_i, const uint64_t *s_ip1, const uint64_t *t_i,
                               const uint64_t *t_ip1, uint64_t *p_i, uint64_t *p_ip1, uint64_t *g_i,
                               size_t n, void *stream);

CG_API cg_status cg_bit_transpose64(const uint64_t *src, uint64_t *dst, size_t n, void *stream);

CG_API cg_status cg_bshare_carry_level(const uint64_t *p_i, const uint64_t *p_ip1,
                                const uint64_t *g_i, const uint64_t *g_ip1,
                                uint64_t *p_out, uint64_t *g_out, size_t planes_out, size_t m,
                                void *stream);

CG_API cg_status cg_bits_unpack(const uint64_t *plane, uint64_t *out, size_t n, void *stream);

CG_API cg_status cg_bzero_share(const uint8_t *key_self, const uint8_t *key_prev, uint64_t nonce,
                         uint64_t first, uint64_t *beta, size_t n, void *stream);

CG_API cg_status cg_breshare(const uint64_t *z_i, const uint8_t *key_self, const uint8_t *key_prev,
                      uint64_t nonce, uint64_t first, uint64_t *out, size_t n, void *stream);

/*
 * out = s0 + s1 + s2 (mod 2^64), element-wise over n (Sec. III-B, "Secret
 * sharing").  Opens a replicated sharing (pass its three distinct shares) and
 * equally the three parties' additive outputs z_0, z_1, z_2 of
 * cg_share_matmul / cg_share_conv2d.  n == 0 is allowed (CG_OK, pointers not looked at).
 */
CG_API cg_status cg_reconstruct(const uint64_t *s0, const uint64_t *s1, const uint64_t *s2,
                         uint64_t *out, size_t n, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* CG_H */
