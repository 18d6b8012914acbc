/*
 * libinvact -- Inverted Activations (arXiv 2407.15545) for AMD MI355X (gfx950).
 *
 * C ABI of the hot path: a GELU / SiLU layer that saves its OUTPUT
 * and a 1-bit-per-element branch mask instead of its input, and rebuilds
 * f'(x) in the backward pass from the saved output with the paper's
 * closed-form approximation of f'(f^-1(y)).
 *
 * Conventions shared by every compute entry point
 *   - All data pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates, frees, copies to the host or synchronises.
 *   - Work is enqueued on `stream` (0 = the default stream); the call returns
 *     as soon as the kernel is launched.
 *   - Tensors are flat and contiguous, `n` elements each; shape is the caller's
 *     business.  dtype selects the storage format of every floating-point
 *     tensor of the call (arithmetic is binary32 in registers -- binary64
 *     in the forward of binary32 storage -- with one round-to-nearest-even
 *     at the store).
 *   - `mask` holds invact_mask_bytes(n) bytes: element i is bit (i mod 8) of
 *     byte (i div 8), i.e. bit (i mod 64) of little-endian 64-bit word
 *     (i div 64) (Method, "Space-efficient Boolean Indicator").  The forward
 *     entry points write every byte of it; bits past n are written as 0.
 *   - Floating-point pointers must be 16-byte aligned and `mask` 8-byte
 *     aligned, else INVACT_ERR_ALIGN.
 *   - Element-wise aliasing of an output with an input of the same call and
 *     the same dtype is allowed (y == x, grad_x == grad_y, grad_up == grad_h,
 *     grad_gate == grad_h, ...); any other overlap is undefined.
 *   - The return value is an invact_status (0 = success).  n == 0 succeeds
 *     without a launch.  Arguments are validated before anything is enqueued.
 *   - Calls are thread-safe; the library keeps no mutable state apart from the
 *     tuning parameters below and the per-GPU array of invact_sbit_linear_wgrad_static,
 *     whose calls must not overlap on one GPU (see there).
 */
#ifndef INVACT_H
#define INVACT_H

#include <stddef.h>
#include <hip/hip_runtime_api.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    INVACT_GELU_TANH = 0,   /* x (1 + tanh(sqrt(2/pi) (x + 0.044715 x^3))) / 2 */
    INVACT_GELU_ERF  = 1,   /* x Phi(x)                                        */
    INVACT_SILU      = 2    /* x sigmoid(x)                                    */
} invact_kind;

typedef enum { INVACT_FP32 = 0, INVACT_BF16 = 1 } invact_dtype;

typedef enum {
    INVACT_OK = 0,
    INVACT_ERR_KIND,        /* kind is not an invact_kind                      */
    INVACT_ERR_DTYPE,       /* dtype is not an invact_dtype                    */
    INVACT_ERR_NULL,        /* a required pointer is NULL (and n > 0)          */
    INVACT_ERR_ALIGN,       /* a pointer is not aligned as required            */
    INVACT_ERR_SIZE,        /* n is too large: for the mask size to fit size_t, or
                               for one launch (2^31 workgroups of 256 to 1024 elements) */
    INVACT_ERR_HIP          /* the HIP runtime refused the launch              */
} invact_status;

/* Bytes of the mask of an n-element tensor: 8 * ceil(n / 64). */
size_t invact_mask_bytes(size_t n);

/* Static, human-readable text for a status code. */
const char* invact_strerror(int status);

/*
 * Forward of the layer (Algorithm 1, forward; Eq. (1), Eq. (4)):
 *   y[i] = f(x[i]),  mask bit i = (x[i] < T),  T = the minimiser of f.
 * x: in, n elements.  y: out, n elements.  mask: out, invact_mask_bytes(n).
 * x == T and NaN give bit 0; f(-inf) = -0 with bit 1.
 */
int invact_fwd(int kind, int dtype, const void* x, void* y, void* mask,
               size_t n, hipStream_t stream);

/*
 * Backward of the layer (Algorithm 1, backward; Eqs. (5)-(8)):
 *   grad_x[i] = grad_y[i] * q(y[i], s_i),
 * q = q_left if the mask bit s_i is 1 else q_right, with the coefficients of
 * the appendix "Approximation Coefficients".  Square-root arguments are
 * clamped at 0; q(+inf, 0) = 1; NaN in y or grad_y gives NaN; an infinite grad_y gives the infinity of the sign of
 * grad_y * q (NaN where q is 0).
 * y, grad_y: in.  mask: in, as written by invact_fwd.  grad_x: out.
 */
int invact_bwd(int kind, int dtype, const void* y, const void* mask,
               const void* grad_y, void* grad_x, size_t n, hipStream_t stream);

/*
 * Gated block, forward (Experiments, "GeGLU" block; Limitations: the product
 * saves the activation's output anyway):
 *   act[i] = f(gate[i]),  mask bit i = (gate[i] < T),  h[i] = f(gate[i]) * up[i]
 * (h is formed from the unrounded activation: with binary32 storage in binary64, within 2 ulp for every gate and
 * up; with bfloat16 storage from the binary32 value, which below 2^-126 may be flushed or underflow gradually, so
 * that where |f(gate)| < 2^-126 h carries an absolute error of up to 2^-126 |up|).  The block saves act, up, mask.
 * gate, up: in.  act, h: out.  mask: out.
 * swiglu_invact_fwd is geglu_invact_fwd with kind = INVACT_SILU.
 */
int geglu_invact_fwd(int kind, int dtype, const void* gate, const void* up,
                     void* act, void* h, void* mask, size_t n, hipStream_t stream);
int swiglu_invact_fwd(int dtype, const void* gate, const void* up,
                      void* act, void* h, void* mask, size_t n, hipStream_t stream);

/*
 * Gated block, backward from the saved tensors (Algorithm 1, backward, applied
 * to the activation inside the product):
 *   grad_up[i]   = grad_h[i] * act[i]
 *   grad_gate[i] = grad_h[i] * up[i] * q(act[i], s_i)
 * (grad_h * up is formed first -- with binary32 storage without rounding -- so where that product is beyond
 * binary32's range grad_gate is the infinity, whatever q is: NaN where q is 0)
 * act, up, grad_h: in.  mask: in.  grad_gate, grad_up: out.
 * swiglu_invact_bwd is geglu_invact_bwd with kind = INVACT_SILU.
 */
int geglu_invact_bwd(int kind, int dtype, const void* act, const void* up,
                     const void* mask, const void* grad_h,
                     void* grad_gate, void* grad_up, size_t n, hipStream_t stream);
int swiglu_invact_bwd(int dtype, const void* act, const void* up,
                      const void* mask, const void* grad_h,
                      void* grad_gate, void* grad_up, size_t n, hipStream_t stream);

/*
 * Precision-bit variant (Method, "Precision Bit Inverted Activation"): no mask
 * tensor; the lowest significand bit of every stored y carries the indicator,
 * so the forward's output differs from f(x) by up to one more unit in the last
 * place.
 *   forward:  y[i] = f(x[i]) rounded to dtype, then bit 0 of its pattern := (x[i] < T)
 *   backward: s_i = bit 0 of y[i];  grad_x[i] = grad_y[i] * q(y[i], s_i),
 *             q evaluated at the stored (tagged) y
 * x, y, grad_y: in / out as named, n elements each; y == x and grad_x == grad_y
 * may alias.
 */
int invact_pbit_fwd(int kind, int dtype, const void* x, void* y, size_t n, hipStream_t stream);
int invact_pbit_bwd(int kind, int dtype, const void* y, const void* grad_y, void* grad_x,
                    size_t n, hipStream_t stream);

/*
 * Sign-bit variant (Section 3.3, "Sign-bit Inverted Activation", and its
 * listing): no mask tensor.  f is bounded below by C = f(T), so f(x) - C is
 * never negative and its sign bit is free to carry the indicator.  The saved
 * tensor is not the layer's output: its consumer (a GEMM prologue in the
 * paper's listing; invact_sbit_decode, or the two
 * invact_sbit_linear_* products below) first
 * rebuilds |y_tagged| + C.  In real arithmetic that is f(x) again; in the
 * storage dtype it is f(x) only to an absolute error of about one unit in
 * the last place of C, because both f(x) - C and the sum live on the grid of
 * max(|f(x)|, |C|): activations much smaller than |C| (x near 0) come back
 * with few of their own digits.
 *   forward:  y_tagged[i] = max(f(x[i]) - C, 0) rounded to dtype, sign bit := (x[i] < T)
 *   decode:   y[i] = |y_tagged[i]| + C rounded to dtype
 *   backward: s_i = sign bit of y_tagged[i];  y_i = |y_tagged[i]| + C formed in binary32;
 *             grad_x[i] = grad_y[i] * q(y_i, s_i)
 * C is the binary32-rounded minimum of the kind.  n elements each; y_tagged == x,
 * y == y_tagged and grad_x == grad_y may alias.
 */
int invact_sbit_fwd(int kind, int dtype, const void* x, void* y_tagged, size_t n, hipStream_t stream);
int invact_sbit_decode(int kind, int dtype, const void* y_tagged, void* y, size_t n, hipStream_t stream);
int invact_sbit_bwd(int kind, int dtype, const void* y_tagged, const void* grad_y, void* grad_x,
                    size_t n, hipStream_t stream);

/*
 * Sign-bit variant, the consumer (Section 3.3 and its listing, where the linear layer that
 * follows the activation multiplies Y + C by its weight in the forward and forms its weight
 * gradient from Y + C and dOut in the backward): matrix products that rebuild
 * |y_tagged| + C while they load the saved tensor, so that the activation itself is never
 * written to memory.  bfloat16 only (INVACT_ERR_DTYPE otherwise); products on the matrix
 * units with binary32 accumulation, |y_tagged| + C rounded to bfloat16 exactly as
 * invact_sbit_decode rounds it, one rounding of each output element to bfloat16.
 *   invact_sbit_linear_fwd:    out[m][n]         = sum_k (|y_tagged[m][k]| + C) * weight[n][k]  (+ bias[n])
 *   invact_sbit_linear_wgrad:  grad_weight[n][k] = sum_m grad_out[m][n] * (|y_tagged[m][k]| + C)
 * y_tagged: in, M x K.  weight: in, N x K (the layout of a linear layer's weight).  bias: in,
 * N elements, or NULL.  out, grad_out: M x N.  grad_weight: out, N x K.  All row-major and
 * dense.  K must be a multiple of 64 for the forward; M a multiple of 64 and N and K multiples
 * of 8 for the weight gradient; every matrix must hold fewer than 2^31 elements
 * (INVACT_ERR_SIZE otherwise; an output with no elements succeeds without a launch).  Matrix pointers must be 16-byte aligned.
 * No aliasing between an output and an input.
 */
int invact_sbit_linear_fwd(int kind, int dtype, const void* y_tagged, const void* weight, const void* bias,
                           void* out, size_t M, size_t N, size_t K, hipStream_t stream);
int invact_sbit_linear_wgrad(int kind, int dtype, const void* y_tagged, const void* grad_out,
                             void* grad_weight, size_t M, size_t N, size_t K, hipStream_t stream);

/*
 * Sign-bit variant, the layer's input gradient (Section 3.3, the last product of its listing, read as the
 * gradient at the activation's output, dOut W, times f'(f^-1(Y + C, S))):
 *   grad_x[m][k] = (sum_n grad_out[m][n] * weight[n][k]) * q(|y_tagged[m][k]| + C, sign bit of y_tagged[m][k])
 * One kernel: the product on the matrix units with binary32 accumulation, then every accumulator times q,
 * evaluated exactly as invact_sbit_bwd evaluates it, then one rounding to bfloat16.  Against a library GEMM
 * followed by invact_sbit_bwd the M x K product dOut W is never written to memory or rounded.
 * y_tagged: in, M x K.  grad_out: in, M x N.  weight: in, N x K.  grad_x: out, M x K.  All row-major and dense,
 * bfloat16 only (INVACT_ERR_DTYPE otherwise).  N must be a multiple of 64 and K a multiple of 8, every matrix must
 * hold fewer than 2^31 elements (INVACT_ERR_SIZE otherwise; an output with no elements succeeds without a launch).
 * Matrix pointers must be 16-byte aligned.  grad_x may not alias an input.
 */
int invact_sbit_linear_dgrad(int kind, int dtype, const void* y_tagged, const void* grad_out, const void* weight,
                             void* grad_x, size_t M, size_t N, size_t K, hipStream_t stream);

/*
 * The same weight gradient, allowed to split its contraction (same passage: the sum over the batch of
 * dOut^T (Y + C)).  A narrow layer has a small N x K output and a long sum over M: too few output tiles to
 * occupy the chip.  This entry point then cuts the sum over M into parts, has each part's workgroups leave binary32
 * partial sums in `workspace`, and adds them in a second kernel, always in the same order, so results are
 * reproducible; they differ from invact_sbit_linear_wgrad's by the order of the binary32 additions only, and
 * are the same bits where it does not split.
 *   invact_sbit_linear_wgrad_workspace(M, N, K): bytes of workspace the shape needs; 0 where the product is not
 *     split (then workspace may be NULL) or the shape is not one the product accepts.
 *   workspace: device memory, 16-byte aligned, owned by the caller, at least that many bytes (workspace_bytes says
 *     how many there are; INVACT_ERR_SIZE if too few).  Written and read by this call only: contents before and
 *     after mean nothing, and calls that may run at the same time need a workspace each.
 * Everything else as for invact_sbit_linear_wgrad.
 */
size_t invact_sbit_linear_wgrad_workspace(size_t M, size_t N, size_t K);
int invact_sbit_linear_wgrad_ws(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                void* grad_weight, size_t M, size_t N, size_t K,
                                void* workspace, size_t workspace_bytes, hipStream_t stream);

/*
 * invact_sbit_linear_wgrad_ws for callers that cannot allocate a workspace (code under HIP graph capture, serving
 * loops, harnesses that forbid hipMalloc): the partial sums go to a 64 MiB array that the library's code object
 * holds on every GPU it is loaded on, until the process ends.  Same arguments, results (bit for bit) and errors as
 * invact_sbit_linear_wgrad_ws with a workspace of that size; a shape that needs more (possible only with
 * invact_set_linear_splits) is refused with INVACT_ERR_SIZE.  It allocates and frees nothing.  All calls on one GPU
 * share the array: calls that may run at the same time on one GPU (different streams, different threads) race
 * and give wrong results; calls in one stream are ordered and safe.  Nothing in the array has to be cleared
 * between calls: every element a call reads it has written before.
 */
int invact_sbit_linear_wgrad_static(int kind, int dtype, const void* y_tagged, const void* grad_out,
                                    void* grad_weight, size_t M, size_t N, size_t K, hipStream_t stream);

/*
 * Launch tuning (process-wide, for benchmarking; results are bit-identical
 * whatever is set).  By default a workgroup is one wavefront that handles one
 * tile and retires, and every entry point caps the number of such workgroups
 * resident on a compute unit at the value measured best for it on MI355X.
 *
 * invact_set_resident_blocks: blocks in 1..32 forces that cap for all entry
 * points (32 = the hardware's own limit, i.e. no cap); 0 restores the
 * defaults.  invact_set_blocks_per_cu: blocks_per_cu in 1..64 switches to a
 * persistent grid of that many workgroups per compute unit striding over the
 * tensor (uncapped); 0 restores the default.  Both return their argument, or
 * a negative number if it is out of range.
 */
int invact_set_resident_blocks(int blocks);
int invact_set_blocks_per_cu(int blocks_per_cu);
/* The invact_sbit_linear_* products choose their workgroup shape by the size of the output (a 256 x 256 tile
 * where that still gives every compute unit a workgroup, 128 x 128 otherwise, with 8 wavefronts where a compute
 * unit gets one such tile at most and 4 where it gets more): t = 4, 3 or 2 forces the first, second or third,
 * 0 restores the choice.  Returns its argument, or a negative number if it is none of these. */
int invact_set_linear_tile(int t);
/* invact_sbit_linear_wgrad_ws chooses by the shape into how many parts it splits the sum over M (none where the
 * output has 256 tiles of 256 x 256 or more; else as many as give every compute unit a tile, each part at least 1024
 * rows long): splits = 1..64 forces that number, capped at M / 64; 0 restores the choice.
 * invact_sbit_linear_wgrad_workspace answers for the setting in force.  Returns its argument, or a negative number. */
int invact_set_linear_splits(int splits);

#ifdef __cplusplus
}
#endif
#endif /* INVACT_H */
