/*
 * circ.h — C ABI of the block-circulant layer library for MI355X (gfx950).
 *
 * The library evaluates the product of a block-circulant weight matrix with a
 * batch of activations (CirCNN, arXiv 1708.08917, Sec. 3): a p x q grid of
 * k x k circulant blocks, each stored as one length-k vector w_ij, applied as
 *
 *     a_i = sum_j IFFT( FFT(w_ij) o FFT(x_j) )                (Algorithm 1)
 *
 * for fully-connected layers (forward and backward, Algorithms 1 and 2) and for
 * CONV layers whose channel-mixing matrices are block-circulant (Sec. 3.2,
 * Eq. 6 and Eq. 7).
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - Orientation: W_ij[a][b] = w_ij[(a - b) mod k]; w_ij is the first column of
 *    its block and W_ij x_j is the circular convolution of w_ij with x_j.  This
 *    is the reading under which the FFT formula of Sec. 3.1 holds as printed.
 *  - All tensors are fp32, dense, row-major, in DEVICE memory of the current HIP
 *    device.  Every pointer must be 16-byte aligned.  The caller owns every
 *    buffer; the library allocates no device memory.  The only state it keeps is,
 *    per kernel and device, the note that it has opted that kernel in to more than
 *    64 KB of LDS, and per device the address of the fixed scratch array of
 *    circ_fc_forward_static (atomic values, set under a lock: entry points may be
 *    called from several host threads and on several devices).
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Calls only enqueue work on it and return; nothing synchronises.
 *  - Block size k: 1 <= k <= 512, and k must divide the layer widths exactly
 *    (p = m / k, q = n / k; the paper assumes the same).  Powers of two run on
 *    the radix-2 FFT kernels (Sec. 4.1) and, where the shape allows, on the fused
 *    kernels; any other k (Fig. 1 uses k = 3) takes the transforms by their
 *    definition, O(k^2) per block, around the same per-frequency contraction.
 *  - Errors are returned as circ_status; nothing aborts or throws across the
 *    ABI.  Argument errors are detected on the host before any launch, so a
 *    failing call has enqueued nothing.
 *  - Output buffers must not alias input buffers.
 */
#ifndef CIRC_H_
#define CIRC_H_

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  CIRC_OK = 0,
  CIRC_EINVAL = -1,     /* null/misaligned pointer, non-positive size, bad k, aliasing */
  CIRC_ENOTSUP = -2,    /* valid request this build does not implement (none at present; kept for the ABI) */
  CIRC_EWORKSPACE = -3, /* workspace NULL or smaller than the matching *_workspace_bytes */
  CIRC_EHIP = -4        /* a HIP launch failed; hipGetLastError holds the detail */
} circ_status;

/* epilogue bit flags for the forward entry points (Eq. 1: y = psi(Wx + theta)) */
enum { CIRC_EPI_NONE = 0, CIRC_EPI_BIAS = 1, CIRC_EPI_RELU = 2 };

/* Human-readable name of a status code (static storage, never NULL). */
const char* circ_status_string(circ_status s);

/*
 * Size in bytes of the cached weight spectra for `n_grids` grids of p x q
 * blocks of size k (n_grids = 1 for an FC layer, r*r for a CONV layer).
 * Returns 0 for invalid arguments.  (Sec. 3.1: only w_ij or FFT(w_ij) needs to
 * be stored; Sec. 4.2: the FFT results of the weights are what is kept in RAM.)
 */
size_t circ_spectra_bytes(int n_grids, int p, int q, int k);

/*
 * Weight-spectrum precompute: FFT(w_ij) for every block, half spectrum only
 * (real input, Sec. 4.1), in the library's private layout.
 *   w      device, [n_grids][p][q][k] fp32 (for CONV: grids in (dh, dw) order)
 *   w_hat  device, circ_spectra_bytes(n_grids,p,q,k) bytes, opaque; must be
 *          recomputed after every update of w.
 */
circ_status circ_precompute_spectra(const float* w, int n_grids, int p, int q, int k,
                                    void* w_hat, void* stream);

/* Workspace size of circ_fc_forward (backward = 0) or circ_fc_backward (backward = 1). */
size_t circ_fc_workspace_bytes(int p, int q, int k, int batch, int backward);

/*
 * FC forward (Algorithm 1 plus the bias/ReLU of Eq. 1):
 *   y[b][i*k + t] = psi( sum_j (W_ij x_j[b])[t] + bias[i*k + t] ).
 *   w_hat     device, from circ_precompute_spectra with n_grids = 1
 *   x         device, [batch][q*k]
 *   bias      device, [p*k]; required iff epilogue has CIRC_EPI_BIAS, else may be NULL
 *   y         device, [batch][p*k], overwritten
 *   workspace device scratch of at least circ_fc_workspace_bytes(p,q,k,batch,0) bytes
 */
circ_status circ_fc_forward(const void* w_hat, const float* x, const float* bias, float* y,
                            int p, int q, int k, int batch, int epilogue,
                            void* workspace, size_t workspace_bytes, void* stream);

/*
 * circ_fc_forward for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same
 * arguments, result and errors as circ_fc_forward, without the workspace: the scratch the kernels
 * need (activation spectra of the three-kernel route, partial spectra of the split batch <= 2
 * kernel) is a fixed array of CIRC_STATIC_SCRATCH_BYTES inside the library's code object, which
 * every device the library runs on holds until the process ends.  The call allocates and frees
 * nothing.  Shapes whose circ_fc_workspace_bytes(p,q,k,batch,0) exceeds CIRC_STATIC_SCRATCH_BYTES
 * return CIRC_EWORKSPACE (nothing is enqueued); use circ_fc_forward with a workspace for those.
 * All calls on one device share that device's array: calls that overlap in time on one device
 * (different streams, or different host threads without ordering) race on it and must be
 * ordered by the caller; consecutive calls on one stream are safe, and nothing has to be
 * cleared in between (each call overwrites what it reads).  The first call on a device looks
 * the array's address up (a host-side runtime query, no device work); make it outside a
 * graph capture.
 */
#define CIRC_STATIC_SCRATCH_BYTES (32u << 20)
circ_status circ_fc_forward_static(const void* w_hat, const float* x, const float* bias, float* y,
                                   int p, int q, int k, int batch, int epilogue, void* stream);

/*
 * FC backward (Algorithm 2; Eq. 4 and Eq. 5).  `dy` is the gradient with respect
 * to the pre-activation a = Wx + theta (the caller applies the ReLU mask).
 *   dx[b][j*k + :] = sum_i IFFT( conj(FFT w_ij) o FFT(dy_i[b]) )        (may be NULL)
 *   dw[i][j][:]    = sum_b IFFT( conj(FFT x_j[b]) o FFT(dy_i[b]) )      (may be NULL)
 * Both are overwritten, not accumulated; the batch sum carries no 1/batch.
 * The result is deterministic (no floating-point atomics).
 *   workspace  at least circ_fc_workspace_bytes(p,q,k,batch,1) bytes
 */
circ_status circ_fc_backward(const void* w_hat, const float* x, const float* dy,
                             float* dx, float* dw,
                             int p, int q, int k, int batch,
                             void* workspace, size_t workspace_bytes, void* stream);

/* Workspace size of circ_conv_forward for the same arguments. */
size_t circ_conv_workspace_bytes(int N, int C_in, int C_out, int H, int W,
                                 int r, int stride, int pad, int k);

/*
 * Block-circulant CONV forward (Sec. 3.2, Eq. 6 with the weight structure of Eq. 7),
 * cross-correlation with zero padding:
 *   y[n][co][h][w] = psi( sum_{dh,dw,ci} Wd[dh][dw][co][ci] * x[n][ci][h+dh-pad][w+dw-pad] + bias[co] )
 * where each Wd[dh][dw] is a (C_out/k) x (C_in/k) grid of k x k circulant blocks
 * and the FFT runs over the channel dimension of every pixel.
 *   w_hat  from circ_precompute_spectra with n_grids = r*r, p = C_out/k, q = C_in/k
 *   x      device, NCHW [N][C_in][H][W]
 *   bias   device, [C_out] (per output channel) or NULL
 *   y      device, NCHW [N][C_out][Ho][Wo], Ho = (H+2*pad-r)/stride + 1, Wo likewise
 * With stride > 1 (Eq. 6 is the stride-1 case) the filter moves `stride` pixels per output:
 * x is read at [h*stride+dh-pad][w*stride+dw-pad].  stride >= 1, r >= 1, 0 <= pad < r.
 */
circ_status circ_conv_forward(const void* w_hat, const float* x, const float* bias, float* y,
                              int N, int C_in, int C_out, int H, int W,
                              int r, int stride, int pad, int k, int epilogue,
                              void* workspace, size_t workspace_bytes, void* stream);

/* Workspace size of circ_conv_backward for the same arguments (0 for invalid ones). */
size_t circ_conv_backward_workspace_bytes(int N, int C_in, int C_out, int H, int W,
                                          int r, int stride, int pad, int k);

/*
 * Block-circulant CONV backward.  Sec. 3.2 gives the forward pass (Eq. 6, Eq. 7) and notes
 * that training is formulated like the FC case (Algorithm 2); these are the chain-rule
 * gradients of circ_conv_forward with respect to its input and its block vectors.  `dy` is
 * the gradient with respect to the pre-activation (the caller applies the ReLU mask).
 *   dx[n][ci][h][w]     = sum_{dh,dw,co} Wd[dh][dw][co][ci] * dy[n][co][h-dh+pad][w-dw+pad]   (may be NULL)
 *   dw[dh][dw][i][j][t] = sum over images, output pixels and a of
 *                         dy[n][i*k+a][ho][wo] * x[n][j*k+((a-t) mod k)][ho+dh-pad][wo+dw-pad]  (may be NULL)
 * (terms outside the image are zero; written for stride 1 - with stride s the output pixel
 * (ho, wo) pairs with input pixel (ho*s+dh-pad, wo*s+dw-pad) in both sums).  Both are overwritten, not accumulated, summed over the
 * batch without 1/N, and deterministic (no floating-point atomics).
 *   w_hat  from circ_precompute_spectra with n_grids = r*r, p = C_out/k, q = C_in/k
 *   x      device, NCHW [N][C_in][H][W]                    (needed for dw only)
 *   dy     device, NCHW [N][C_out][(H+2*pad-r)/stride+1][(W+2*pad-r)/stride+1]
 *   dx     device, NCHW like x;  dw device, [r][r][p][q][k]
 *   workspace  at least circ_conv_backward_workspace_bytes(...) bytes
 * stride >= 1, r >= 1, 0 <= pad < r.
 */
circ_status circ_conv_backward(const void* w_hat, const float* x, const float* dy,
                               float* dx, float* dw,
                               int N, int C_in, int C_out, int H, int W,
                               int r, int stride, int pad, int k,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * One gradient-descent step taken on the cached spectra (training, Sec. 3.1 / Algorithm 2).
 * Algorithm 2 yields dL/dw_ij as the inverse FFT of a spectrum G_ij summed over the batch; the
 * step w_ij <- w_ij - lr * dL/dw_ij and the FFT are both linear, so these calls subtract
 * (lr/k) * G_ij from the stored FFT(w_ij)/k directly: no inverse transform of the gradient, no
 * forward transform of the new weights.  Afterwards `w_hat` is what circ_precompute_spectra
 * would return for w - lr * dw (dw as defined at circ_fc_backward / circ_conv_backward), up to
 * fp32 rounding, in every operand order the blob holds.
 *   w_hat  device blob, updated in place; x, dy, dx and the workspace must not overlap it
 *   dx     optional (NULL to skip): backward-data, computed from the spectra before the step
 *   lr     step size (any finite float; 0 leaves the weights unchanged); NaN -> CIRC_EINVAL
 *   other arguments, workspace size and error behaviour as for the backward call of the layer
 * Deterministic.  Calls that share a blob must be ordered by the caller (same stream).
 */
circ_status circ_fc_sgd_step(void* w_hat, const float* x, const float* dy, float* dx, float lr,
                             int p, int q, int k, int batch,
                             void* workspace, size_t workspace_bytes, void* stream);
circ_status circ_conv_sgd_step(void* w_hat, const float* x, const float* dy, float* dx, float lr,
                               int N, int C_in, int C_out, int H, int W,
                               int r, int stride, int pad, int k,
                               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Block vectors back from a spectra blob (the inverse of circ_precompute_spectra; Sec. 3.1:
 * either w_ij or FFT(w_ij) represents a block).  Needed after circ_*_sgd_step, when the blob is
 * the only up-to-date copy of the weights.
 *   w_hat  device blob of (n_grids, p, q, k);  w  device, [n_grids][p][q][k] floats, overwritten
 */
circ_status circ_export_weights(const void* w_hat, int n_grids, int p, int q, int k,
                                float* w, void* stream);

/*
 * Half-width storage for FC inference.  The hardware of Sec. 4.2 keeps inputs and weights in a
 * 16-bit representation; here activations and spectra are IEEE fp16 in memory and every
 * butterfly and accumulation is fp32:
 *   y = psi( IFFT( (1/k) * sum_j fp16(FFT w_ij) o fp16(FFT x_j) ) + bias ),  y rounded to fp16.
 * Same orientation, layouts and epilogue flags as circ_fc_forward, with x and y holding fp16
 * values ([batch][q*k] and [batch][p*k]), bias fp32.  k must be a power of two, 8 <= k <= 512.
 * Against the exact result the error is a few fp16 roundings (2^-11 each: weights' spectra,
 * input spectra, output spectra, output), about 1e-3 of the largest output; spectra of inputs
 * are not normalised, so |x| * k must stay below the fp16 range (65504).  Small layers (the
 * ones circ_fc_forward runs as one fused launch) are computed in one launch here too: the
 * spectra of x and y then never leave the chip and only the weights' spectra and y are rounded.
 *   circ_spectra_bytes_f16        size of the fp16 spectra blob (0 for invalid arguments)
 *   circ_precompute_spectra_f16   w fp32 device [p][q][k] -> blob (opaque, caller-owned, 16-byte aligned)
 *   circ_fc_workspace_bytes_f16   workspace of circ_fc_forward_f16 for the same arguments
 * Errors as for circ_fc_forward.
 */
size_t circ_spectra_bytes_f16(int p, int q, int k);
circ_status circ_precompute_spectra_f16(const float* w, int p, int q, int k, void* w_hat, void* stream);
size_t circ_fc_workspace_bytes_f16(int p, int q, int k, int batch);
circ_status circ_fc_forward_f16(const void* w_hat, const void* x, const float* bias, void* y,
                                int p, int q, int k, int batch, int epilogue,
                                void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same with bfloat16 (the upper 16 bits of an fp32, rounded to nearest even) as the storage
 * format: the range of fp32, so no bound on |x| * k, at 2^-8 per rounding instead of 2^-11
 * (about 5e-3 of the largest output).  A blob made by circ_precompute_spectra_bf16 serves
 * circ_fc_forward_bf16 and circ_fc_backward_bf16 only.
 */
size_t circ_spectra_bytes_bf16(int p, int q, int k);
circ_status circ_precompute_spectra_bf16(const float* w, int p, int q, int k, void* w_hat, void* stream);
size_t circ_fc_workspace_bytes_bf16(int p, int q, int k, int batch);
circ_status circ_fc_forward_bf16(const void* w_hat, const void* x, const float* bias, void* y,
                                 int p, int q, int k, int batch, int epilogue,
                                 void* workspace, size_t workspace_bytes, void* stream);

/*
 * FC backward with 16-bit storage (Algorithm 2 on the same 16-bit spectra): dy and x hold fp16
 * (bf16) values, dx receives fp16 (bf16) values, dw receives the gradient of the block vectors
 * in fp32 (the copy of the weights an optimiser updates is fp32; its new spectra come from
 * circ_precompute_spectra_f16).  Layouts and orientation as for circ_fc_backward:
 *   dx_j  = IFFT( (1/k) * sum_i conj(h(FFT w_ij)) o h(FFT dy_i) ),   rounded to 16 bits
 *   dw_ij = IFFT( sum_b h(FFT dy_i) o conj(h(FFT x_j)) ),            h = rounding to 16 bits,
 * all sums in fp32; the spectrum of dw stays fp32 (a sum over a long batch leaves the fp16
 * range).  dx or dw may be NULL (not both); x may be NULL when dw is.  dx, dw are overwritten.
 *   circ_fc_backward_workspace_bytes_f16   workspace size for the same arguments (0 if invalid)
 * Errors as for circ_fc_backward: CIRC_EINVAL for bad dimensions, k not a power of two in
 * 8..512, a NULL required pointer, pointers not 16-byte aligned or overlapping outputs;
 * CIRC_EWORKSPACE for a short workspace; CIRC_EHIP for a failed launch.
 */
size_t circ_fc_backward_workspace_bytes_f16(int p, int q, int k, int batch);
circ_status circ_fc_backward_f16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw,
                                 int p, int q, int k, int batch,
                                 void* workspace, size_t workspace_bytes, void* stream);
size_t circ_fc_backward_workspace_bytes_bf16(int p, int q, int k, int batch);
circ_status circ_fc_backward_bf16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw,
                                  int p, int q, int k, int batch,
                                  void* workspace, size_t workspace_bytes, void* stream);

/*
 * CONV forward with 16-bit activations (inference in the 16-bit representation of Sec. 4.2):
 * x and y hold fp16 (bf16) values in NCHW, bias is fp32, and w_hat is the blob of
 * circ_precompute_spectra for the same (r*r, p, q, k): the cached weight spectra, about 0.1 %
 * of the bytes a layer moves, stay fp32, so that the only roundings are those of x (the caller's)
 * and of y.  Everything else as circ_conv_forward (layouts, stride, padding, epilogue flags,
 * workspace size from circ_conv_workspace_bytes); k must be a power of two, 8 <= k <= 512.
 * Errors as for circ_conv_forward.
 */
circ_status circ_conv_forward_f16(const void* w_hat, const void* x, const float* bias, void* y,
                                  int N, int C_in, int C_out, int H, int W, int r, int stride, int pad,
                                  int k, int epilogue, void* workspace, size_t workspace_bytes, void* stream);
circ_status circ_conv_forward_bf16(const void* w_hat, const void* x, const float* bias, void* y,
                                   int N, int C_in, int C_out, int H, int W, int r, int stride, int pad,
                                   int k, int epilogue, void* workspace, size_t workspace_bytes, void* stream);

/*
 * CONV backward with 16-bit activations: x, dy and dx hold fp16 (bf16) values, dw receives the
 * gradient of the block vectors in fp32; all spectra and the blob (circ_precompute_spectra) stay
 * fp32, so the roundings are those of the inputs (the caller's) and of dx.  Everything else as
 * circ_conv_backward, workspace size from circ_conv_backward_workspace_bytes; k a power of two,
 * 8 <= k <= 512.  dx or dw may be NULL (not both); x may be NULL when dw is.
 */
circ_status circ_conv_backward_f16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw,
                                   int N, int C_in, int C_out, int H, int W, int r, int stride, int pad,
                                   int k, void* workspace, size_t workspace_bytes, void* stream);
circ_status circ_conv_backward_bf16(const void* w_hat, const void* x, const void* dy, void* dx, float* dw,
                                    int N, int C_in, int C_out, int H, int W, int r, int stride, int pad,
                                    int k, void* workspace, size_t workspace_bytes, void* stream);

/*
 * Bias gradient (Eq. 1: a = Wx + theta, so dL/dtheta is dL/da summed over everything but the
 * channel).  dy is viewed as [outer][channels][inner]:
 *   db[c] = sum_{o, t} dy[(o*channels + c)*inner + t]
 * FC: outer = batch, channels = p*k, inner = 1.  CONV (NCHW): outer = N, channels = C_out,
 * inner = Ho*Wo.  db is overwritten; the sum order is fixed (deterministic).  No workspace.
 */
circ_status circ_bias_grad(const float* dy, float* db, long long outer, int channels,
                           long long inner, void* stream);

/*
 * Max-pooling, the subsampling (POOL) layer of Sec. 2.1, run by the peripheral block on
 * comparators in the paper's architecture (Sec. 4.2):
 *   y[n][c][ho][wo] = max_{a,b < window} x[n][c][ho*stride + a][wo*stride + b]
 *   x  device, NCHW [N][C][H][W];  y  device, NCHW [N][C][(H-window)/stride+1][(W-window)/stride+1]
 * Windows lie entirely inside the image (no padding); 1 <= window <= min(H, W), stride >= 1.
 * The result is exact (no arithmetic).  CIRC_EINVAL for bad sizes, NULL / misaligned / overlapping
 * pointers; CIRC_EHIP for a failed launch.
 */
circ_status circ_maxpool_forward(const float* x, float* y, int N, int C, int H, int W,
                                 int window, int stride, void* stream);

/*
 * A chain of layers evaluated back to back on one stream: the inference regime of Sec. 5.3 (one
 * image through a whole network; Sec. 2.1: DNNs cascade FC, CONV and POOL layers).  Each layer is
 * what the single-layer entry point computes (circ_fc_forward, circ_conv_forward,
 * circ_maxpool_forward); activations between layers stay in the workspace, and a batch of one
 * or two vectors takes the streaming kernels of the FC layers.  Activations are NCHW; an FC
 * layer reads the preceding image as the vector [C*H*W] it is in memory.
 *   layers   HOST array of n_layers descriptors (read during the call only):
 *     kind      CIRC_LAYER_FC: p, q, k, w_hat, bias, epilogue as for circ_fc_forward
 *               CIRC_LAYER_CONV: C_in, C_out, H, W (input image), r, stride, pad, k, w_hat, bias,
 *                                epilogue as for circ_conv_forward
 *               CIRC_LAYER_MAXPOOL: C_in (channels), H, W (input image), r (window), stride
 *     the output of every layer must have as many elements as the next layer's input
 *   x  device, input of the first layer, [batch][...];  y  device, output of the last layer
 *   workspace  device, at least circ_chain_workspace_bytes(layers, n_layers, batch) bytes
 *              (0 for an invalid chain); must not overlap x or y
 * CIRC_EINVAL: invalid or ill-fitting descriptors, NULL / misaligned pointers, overlaps;
 * CIRC_EWORKSPACE: short workspace; CIRC_EHIP: a failed launch (earlier layers are enqueued).
 */
typedef enum { CIRC_LAYER_FC = 0, CIRC_LAYER_CONV = 1, CIRC_LAYER_MAXPOOL = 2 } circ_layer_kind;
typedef struct {
  int kind;             /* circ_layer_kind */
  int epilogue;         /* CIRC_EPI_* flags (FC, CONV) */
  const void* w_hat;    /* device: spectra blob of the layer (FC, CONV) */
  const float* bias;    /* device: [p*k] (FC) / [C_out] (CONV), or NULL */
  int k;                /* block size (FC, CONV) */
  int p, q;             /* FC: grid of blocks (p*k outputs, q*k inputs) */
  int C_in, C_out;      /* CONV: channels; MAXPOOL: C_in = channels */
  int H, W;             /* CONV, MAXPOOL: input image */
  int r, stride, pad;   /* CONV: filter size, stride, padding; MAXPOOL: r = window, stride (pad unused) */
} circ_layer;
size_t circ_chain_workspace_bytes(const circ_layer* layers, int n_layers, int batch);
circ_status circ_chain_forward(const circ_layer* layers, int n_layers, const float* x, float* y,
                               int batch, void* workspace, size_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* CIRC_H_ */
