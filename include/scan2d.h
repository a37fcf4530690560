/*
 * scan2d.h -- C ABI of the MI355X (gfx950) 2D selective scan library.
 *
 * The operation is the 2D selective scan of 2DMamba (Sec. 3.3, Eq. 3, Eq. 5, Eq. 6 and the
 * output rule y = C h below Eq. 7; inputs and output as listed at the top of the
 * supplementary algorithm "2D selective scan": x, Delta, N, A, D, B, C -> y), batched over
 * Bt batch items and Dc channels.  For every batch item b, channel c and state n:
 *
 *     x_eff[i,j] = mask[b,i,j] ? +0 : x[b,c,i,j]
 *     a[i,j]     = exp(delta[b,c,i,j] * A[c,n])
 *     u[i,j]     = delta[b,c,i,j] * Bm[b,n,i,j] * x_eff[i,j]
 *     hhor[i,j]  = a[i,j] * hhor[i,j-1] + u[i,j]          (row scan,    hhor[i,-1] = 0)
 *     h[i,j]     = a[i,j] * h[i-1,j]   + hhor[i,j]        (column scan, h[-1,j]   = 0)
 *     y[b,c,i,j] = sum_n Cm[b,n,i,j] * h_n[i,j] + Dskip[c] * x_eff[i,j]
 *
 * delta is the already positive step (softplus applied by the caller); A is the negative
 * real parameter itself.  The N-wide states hhor and h only ever live in registers / LDS.
 *
 * ALL POINTERS ARE DEVICE POINTERS owned by the caller.  The library never allocates,
 * frees or synchronises; every call only enqueues kernels on `stream` (a hipStream_t,
 * passed as void*; NULL = the default stream) and returns.  Inputs and outputs must not
 * alias.  Outputs are overwritten, never accumulated into.
 *
 * Layouts (dense, row-major, last index fastest):
 *     x, delta, y, dy, dx, ddelta : [Bt][Dc][H][W]   element type given by desc.dtype
 *     Bm, Cm                      : [Bt][N][H][W]    element type given by desc.dtype
 *     dBm, dCm                    : [Bt][N][H][W]    fp32
 *     A, dA                       : [Dc][N]          fp32
 *     Dskip, dDskip               : [Dc]             fp32
 *     mask                        : [Bt][H][W]       uint8, nonzero = background cell
 * Base pointers must be aligned to 16 bytes.  State, exp and all accumulation are fp32;
 * bf16 outputs are rounded once, to nearest-even.
 *
 * Errors: every entry point returns SCAN2D_OK (0) or a negative code; on error nothing has
 * been enqueued and no output has been touched.  No exceptions, no abort.
 * Thread safety: entry points may be called concurrently from several host threads.
 *
 * Limits of this version: 1 <= N <= 64; N*H*W < 2^27 (the kernels address one map's states
 * with 32-bit lane offsets); any H, W >= 1 in the forward and in the backward (maps wider than
 * one lane-group panel are swept panel by panel and need workspace for the carries between the
 * panels, see scan2d_workspace_bytes).  Shapes outside these limits return SCAN2D_ERR_BAD_SHAPE.
 */
#ifndef SCAN2D_H_
#define SCAN2D_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SCAN2D_OK                   =  0,
    SCAN2D_ERR_NULL_POINTER     = -1,  /* a required pointer is NULL */
    SCAN2D_ERR_BAD_SHAPE        = -2,  /* a dimension < 1, N > 64, N*H*W >= 2^27, element count overflow */
    SCAN2D_ERR_BAD_DTYPE        = -3,
    SCAN2D_ERR_BAD_FLAGS        = -4,  /* flags holds an unknown bit */
    SCAN2D_ERR_WORKSPACE_SMALL  = -5,  /* workspace_bytes < scan2d_workspace_bytes() */
    SCAN2D_ERR_MISALIGNED       = -6,  /* a base pointer is not 16-byte aligned */
    SCAN2D_ERR_LAUNCH_FAILED    = -7,  /* the HIP runtime refused a launch */
    SCAN2D_ERR_UNSUPPORTED_DEVICE = -8, /* current device is not gfx950 */
    SCAN2D_ERR_SCRATCH_LIMIT    = -9   /* scan2d_bwd_static_scratch only: the call needs more than SCAN2D_STATIC_SCRATCH_BYTES */
};

enum { SCAN2D_F32 = 0, SCAN2D_BF16 = 1 };
/*
 * Mask mode (desc.flags).  By default a masked cell holds x = +0 (the zero-token form of the padded
 * non-tissue cells, Sec. 3.2) and still decays the state that passes through it.  With
 * SCAN2D_FLAG_IDENTITY_CELLS its step is 0 as well, i.e. A-bar = 1 and B-bar x = 0: the state passes through
 * unchanged, the padding the supplement describes for cells outside the map ("Tiling and edge cases").  A
 * fully masked row or column then behaves as if it were not there.  The backward returns ddelta = 0 at such
 * cells (with the softplus step: ddelta_raw = 0).  Honoured by every forward and backward entry point.
 */
enum { SCAN2D_FLAG_IDENTITY_CELLS = 1 };
/*
 * Scan order (desc.flags).  By default rows are scanned first, then columns (Eq. 5, then Eq. 6).  With
 * SCAN2D_FLAG_COLUMNS_FIRST the order is the other one, the supplement's ablation of the scan order:
 *     v[i,j] = a[i,j] * v[i-1,j] + u[i,j],    h[i,j] = a[i,j] * h[i,j-1] + v[i,j],    y = Cm . h + Dskip * x_eff
 * (different from the default whenever the decay depends on the position).  Tensor layouts do not change.
 * Where the kernels that share the per-position work of a map through LDS take the shape (forward: maps of at
 * most 256 columns whose state count they are built for; backward: at most 192 columns and 16 states) the order
 * is exchanged inside the kernels, at the cost of the default order and with its workspace.  For every other
 * shape the library transposes the maps into the workspace, runs the row-first kernels on H and W exchanged and
 * transposes the results back, which costs several passes over the tensors and a workspace of their size;
 * scan2d_workspace_bytes accounts for it and scan2d_describe_plan says which form runs.  Honoured by every
 * forward and backward entry point.
 */
enum { SCAN2D_FLAG_COLUMNS_FIRST = 2 };
enum { SCAN2D_PASS_FWD = 0, SCAN2D_PASS_BWD = 1, SCAN2D_PASS_BWD_GATED = 2, SCAN2D_PASS_BWD_SOFTPLUS = 3,
       SCAN2D_PASS_FWD_VARIANTS = 4, SCAN2D_PASS_BWD_VARIANTS = 5 };

typedef struct {
    int32_t  Bt, Dc, H, W, N;  /* batch, channels, grid height, grid width, states: all >= 1, N <= 64 */
    int32_t  dtype;            /* SCAN2D_F32 or SCAN2D_BF16: type of x, delta, Bm, Cm, y, dy, dx, ddelta */
    uint32_t flags;            /* 0 or a sum of SCAN2D_FLAG_IDENTITY_CELLS, SCAN2D_FLAG_COLUMNS_FIRST */
} scan2d_desc;

/*
 * Forward scan (Eq. 5, Eq. 6, y = C h + D x).
 *   Dskip : may be NULL (no skip term).
 *   mask  : may be NULL (no background).  A masked cell behaves exactly as x = +0 there,
 *           whatever is stored in x (a select, so NaN/Inf under the mask cannot leak); the
 *           decay a still acts on masked cells and y is still produced there.
 *   workspace : scratch of at least scan2d_workspace_bytes(desc, SCAN2D_PASS_FWD) bytes,
 *           16-byte aligned; may be NULL when that size is 0.  Contents are undefined after
 *           the call; two calls that overlap in time must not share a workspace.
 */
int scan2d_fwd(const scan2d_desc* desc,
               const void* x, const void* delta, const float* A,
               const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
               void* y,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * The same scan with the step computed inside the kernels (Eq. 3: the step is the softplus of its
 * projection; the supplementary algorithm adds a bias inside the softplus):
 *     delta[b,c,i,j] = softplus(delta_raw[b,c,i,j] + delta_bias[c]),   softplus(t) = log(1 + exp(t))
 * delta_raw has the layout and type of delta; delta_bias is [Dc] fp32 and may be NULL (no bias).
 * Everything else as in scan2d_fwd.
 */
int scan2d_fwd_softplus(const scan2d_desc* desc,
                        const void* x, const void* delta_raw, const float* delta_bias, const float* A,
                        const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                        void* y,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of the forward above for a given dy = dL/dy (Supp. B: two forward scans rebuild
 * the states, which are never stored by the forward; a reverse column scan and a reverse row
 * scan carry the gradients).  With g = dL/dh, q = dL/dhhor:
 *     g[i,j]  = dy[i,j] * Cm[n,i,j] + a[i+1,j] * g[i+1,j]
 *     q[i,j]  = g[i,j]              + a[i,j+1] * q[i,j+1]
 *     da[i,j] = g[i,j] * h[i-1,j] + q[i,j] * hhor[i,j-1]
 *     ddelta  = sum_n (da * a * A[c,n] + q * Bm * x_eff)      dA[c,n] = sum_{b,i,j} da * a * delta
 *     dBm     = sum_c q * delta * x_eff                       dCm     = sum_c dy * h
 *     dx      = mask ? +0 : sum_n q * delta * Bm + Dskip[c] * dy
 *     dDskip  = sum_{b,i,j} dy * x_eff
 * Gradients are with respect to the arrays as passed.  dDskip must be NULL iff Dskip is NULL.
 * Reductions use a fixed order: results are bit-reproducible from run to run.
 */
int scan2d_bwd(const scan2d_desc* desc,
               const void* x, const void* delta, const float* A,
               const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
               const void* dy,
               void* dx, void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip,
               void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of scan2d_fwd_softplus: as scan2d_bwd, but the step is softplus(delta_raw + delta_bias[c]) and
 * the gradients are those of the raw projection and of the bias (chain rule: d softplus(t)/dt =
 * 1/(1 + exp(-t))):
 *     ddelta_raw[b,c,i,j] = ddelta[b,c,i,j] / (1 + exp(-(delta_raw[b,c,i,j] + delta_bias[c])))
 *     ddelta_bias[c]      = sum_{b,i,j} ddelta_raw[b,c,i,j]      (summed from the stored ddelta_raw)
 * ddelta_raw has the layout and type of delta_raw; ddelta_bias is [Dc] fp32 and must be NULL iff
 * delta_bias is NULL.  Workspace: scan2d_workspace_bytes(desc, SCAN2D_PASS_BWD_SOFTPLUS) bytes (except for
 * small maps the step is written there once per position, as fp32, by a kernel of its own).
 */
int scan2d_bwd_softplus(const scan2d_desc* desc,
                        const void* x, const void* delta_raw, const float* delta_bias, const float* A,
                        const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                        const void* dy,
                        void* dx, void* ddelta_raw, float* ddelta_bias, float* dA, float* dBm, float* dCm,
                        float* dDskip,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * The scan as it sits in the block (Sec. 3.2 and Fig. 2: the Mamba block with its 1D scan replaced by the
 * 2D one): the step is softplus(delta_raw + delta_bias[c]) as in scan2d_fwd_softplus, and the output is
 * multiplied element by element by the SiLU of the block's gate branch z,
 *     y[b,c,i,j] = y_scan[b,c,i,j] * z[b,c,i,j] / (1 + exp(-z[b,c,i,j])),
 * by an element-wise kernel enqueued behind the scan on the same stream (y_scan is the stored scan output,
 * already rounded to the storage type; the product is rounded once more).
 *   z      : [Bt][Dc][H][W], dtype, device memory, read-only
 *   y_scan : [Bt][Dc][H][W], dtype, device memory, written: the ungated scan output, which the backward
 *            needs for dz; may be NULL (inference), then y holds it between the two kernels
 *   y      : [Bt][Dc][H][W], dtype, device memory, written; must not overlap y_scan
 * Everything else (layouts, mask, workspace, errors) as scan2d_fwd_softplus.
 */
int scan2d_fwd_softplus_gated(const scan2d_desc* desc,
                              const void* x, const void* delta_raw, const float* delta_bias, const float* A,
                              const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                              const void* z, void* y_scan, void* y,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Backward of scan2d_fwd_softplus_gated for a given dy = dL/dy (y the gated output).  With s = 1/(1+exp(-z)):
 *     dz[b,c,i,j] = dy * y_scan * s * (1 + z * (1 - s))
 * and every other gradient is that of scan2d_bwd_softplus fed dy * z * s in place of dy.  Where the scan's
 * backward sweep has an instantiation for it (flags 0, 16 states, at most 256 columns and the other shapes
 * whose plan reads "banded-shared" with one panel) dz and that product are formed inside the sweep and the
 * product is never rounded; elsewhere one element-wise kernel writes dz and the product (rounded to the
 * storage type) into the workspace and the backward of the scan runs on it.
 *   y_scan : as written by the forward (required)
 *   dz     : [Bt][Dc][H][W], dtype, device memory, written
 *   workspace : at least scan2d_workspace_bytes(desc, SCAN2D_PASS_BWD_GATED) bytes
 * Everything else as scan2d_bwd_softplus.
 */
int scan2d_bwd_softplus_gated(const scan2d_desc* desc,
                              const void* x, const void* delta_raw, const float* delta_bias, const float* A,
                              const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                              const void* z, const void* y_scan, const void* dy,
                              void* dx, void* ddelta_raw, float* ddelta_bias, float* dA, float* dBm, float* dCm,
                              float* dDskip, void* dz,
                              void* workspace, size_t workspace_bytes, void* stream);

/*
 * Two variants of the operator that the paper ablates, as optional extra parameters (all device pointers):
 *   A_v  [Dc][N] fp32: an independent decay parameter for the vertical scan (the supplement's ablation of
 *        re-using A-bar): the column recurrence becomes h[i,j] = exp(delta * A_v[c,n]) * h[i-1,j] + hhor[i,j],
 *        the row recurrence keeps exp(delta * A[c,n]).  NULL: A is used for both (the paper's default).
 *   pad  [Dc] fp32: a learnable padding token (Eq. 4 and the padding-token ablation): a masked cell holds
 *        x_eff = pad[c] instead of the fixed zero.  NULL, or mask == NULL: the zero token.  For bf16 storage the
 *        token is rounded to bf16 (it takes the place of stored x values).
 *   dA_v [Dc][N] fp32, dpad [Dc] fp32: their gradients, written by scan2d_bwd_variants; each must be non-NULL iff
 *        its parameter is.  With A_v the gradient through the decays splits: dA collects the row part
 *        q * hhor[i,j-1], dA_v the column part g * h[i-1,j].  dpad[c] = sum over batch items and masked cells of
 *        (sum_n q * delta * Bm + Dskip[c] * dy); dx is +0 under the mask as always.
 * Both run as ablation modes, not tuned paths: A_v through one guarded kernel tiling per storage type, pad through
 * an element-wise copy of x in front of the scan kernels (and one pass over dx behind them).
 */
typedef struct {
    const float* A_v;
    const float* pad;
    float* dA_v;     /* scan2d_bwd_variants only */
    float* dpad;     /* scan2d_bwd_variants only */
} scan2d_variants;

/*
 * scan2d_fwd / scan2d_bwd with the variants above (v == NULL or all fields NULL: exactly scan2d_fwd / scan2d_bwd).
 * desc.flags must be 0 (the variants do not combine with the identity cells or the columns-first order:
 * SCAN2D_ERR_BAD_FLAGS).  Workspace: scan2d_workspace_bytes(desc, SCAN2D_PASS_FWD_VARIANTS / _BWD_VARIANTS) is
 * enough for any combination.  Everything else as scan2d_fwd / scan2d_bwd.
 */
int scan2d_fwd_variants(const scan2d_desc* desc,
                        const void* x, const void* delta, const float* A,
                        const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                        const scan2d_variants* v,
                        void* y,
                        void* workspace, size_t workspace_bytes, void* stream);
int scan2d_bwd_variants(const scan2d_desc* desc,
                        const void* x, const void* delta, const float* A,
                        const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                        const scan2d_variants* v,
                        const void* dy,
                        void* dx, void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip,
                        void* workspace, size_t workspace_bytes, void* stream);

/*
 * Training pair (Supp. B: the backward first rebuilds the states with two forward scans).  The forward pass of a
 * training step can leave the column state at the top of every band of rows, which the backward pass otherwise
 * recomputes with a sweep of its own, in a buffer `saved` that the caller keeps until the backward pass:
 *   scan2d_saved_bytes(desc)  : size of that buffer; 0 when this shape has no saving forward (then pass saved = NULL:
 *                               the two calls below are exactly scan2d_fwd and scan2d_bwd).  It exists for
 *                               desc.flags == 0, N = 16 and maps of at most 192 columns with more rows than one band.
 *   scan2d_fwd_saving(...)    : scan2d_fwd that also writes `saved` ([Bt*Dc][bands][N][W] fp32, device memory,
 *                               16-byte aligned, at least scan2d_saved_bytes(desc) bytes: SCAN2D_ERR_WORKSPACE_SMALL)
 *   scan2d_bwd_saved(...)     : scan2d_bwd without its checkpoint sweep, reading `saved` (not modified)
 * y and the gradients are those of scan2d_fwd / scan2d_bwd up to the order of the fp32 sums over states (the saving
 * forward has one fixed tiling).  Workspaces as for scan2d_fwd / scan2d_bwd.  desc.flags must be 0 (SCAN2D_ERR_BAD_FLAGS).
 */
size_t scan2d_saved_bytes(const scan2d_desc* desc);
int scan2d_fwd_saving(const scan2d_desc* desc,
                      const void* x, const void* delta, const float* A,
                      const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                      void* y, void* saved, size_t saved_bytes,
                      void* workspace, size_t workspace_bytes, void* stream);
int scan2d_bwd_saved(const scan2d_desc* desc,
                     const void* x, const void* delta, const float* A,
                     const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                     const void* dy, const void* saved, size_t saved_bytes,
                     void* dx, void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip,
                     void* workspace, size_t workspace_bytes, void* stream);

/*
 * The two producers in front of the scan inside a 2DMamba block (Sec. 3.2, Fig. 2: "the design of the original Mamba
 * block" with the scan replaced; Sec. 3.3 names the layers in front of the scan as normalization, projection and
 * convolution; Eq. 3: Delta, B and C are linear functions of x).  Both write the storage type of desc.dtype, so
 * their outputs are the inputs of scan2d_fwd_softplus / scan2d_fwd_softplus_gated as they stand.  Forward only.
 * All pointers are device pointers, 16-byte aligned; asynchronous on `stream`; no workspace.
 *
 * scan2d_block_conv_silu: depth-wise cross-correlation over the map, zero outside it, then SiLU:
 *     t[b,c,i,j] = bias[c] + sum_{p<KH, q<KW} w[c,p,q] * u[b,c,i+p-PH,j+q-PW],     x = t / (1 + exp(-t))
 *   u, x : [Bt][Dc][H][W] storage type (x is written; u == x is not allowed);  w : [Dc][KH][KW] fp32;
 *   bias : [Dc] fp32 or NULL.  1 <= KH, KW <= 7, 0 <= PH < KH, 0 <= PW < KW (else SCAN2D_ERR_BAD_SHAPE):
 *   KH = KW = 3, PH = PW = 1 is the zero-padded 3x3 filter, KH = 1, KW = 4, PW = 3 the causal filter of the 1D
 *   block along the rows.  desc.N and desc.flags are not used.  fp32 arithmetic, one rounding.
 *
 * scan2d_block_xproj: at every position, low = Wx . x (R + 2N rows), then
 *     delta_raw[b,c,i,j] = sum_{r<R} Wdt[c,r] * low[r],    Bm[b,n,i,j] = low[R+n],    Cm[b,n,i,j] = low[R+N+n]
 *   x : [Bt][Dc][H][W], Wx : [R + 2N][Dc], both storage type;  Wdt : [Dc][R] fp32;
 *   delta_raw : [Bt][Dc][H][W], Bm, Cm : [Bt][N][H][W] storage type (written).  The bias of the step projection is
 *   the delta_bias argument of the softplus entry points.  The first product runs on the matrix cores (bf16 or
 *   fp32 inputs as stored, fp32 accumulation); low is not rounded before the second product.
 *   1 <= R <= 64 (else SCAN2D_ERR_BAD_SHAPE); any Dc.  desc.flags is not used.
 */
typedef struct { int32_t KH, KW, PH, PW; } scan2d_conv_shape;
int scan2d_block_conv_silu(const scan2d_desc* desc, const scan2d_conv_shape* shape,
                           const void* u, const float* w, const float* bias, void* x, void* stream);
int scan2d_block_xproj(const scan2d_desc* desc, int R,
                       const void* x, const void* Wx, const float* Wdt,
                       void* delta_raw, void* Bm, void* Cm, void* stream);

/*
 * The aggregator behind the last block (Supp. A "Aggregator": attention pooling with two linear layers, the weighted
 * sum and the attention weights): per batch item, over the positions k of the map that are in the bag,
 *     s_k = sum_{d<D} w[d] * tanh(sum_{m<M} V[d,m] * h[b,m,k]),   a_k = exp(s_k) / sum_j exp(s_j),   z[b,m] = sum_k a_k h[b,m,k]
 *   h : [Bt][M][H][W] with M = desc.Dc, V : [D][M], both storage type;  w : [D] fp32 (D = 128 in the paper);
 *   mask : [Bt][H][W] bytes or NULL, non-zero = the position is not in the bag (its h is never read into a or z);
 *   attn : [Bt][H][W] fp32 (written: a, 0 outside the bag);  z : [Bt][M] fp32 (written).  An empty bag gives a = 0, z = 0.
 *   V . h runs on the matrix cores (bf16 or fp32 inputs as stored, fp32 accumulation); all sums have a fixed order.
 *   1 <= D <= 128 and Bt <= 65535 (else SCAN2D_ERR_BAD_SHAPE); any M.  desc.N and desc.flags are not used.
 *   Device pointers, 16-byte aligned; asynchronous on `stream`; no workspace (attn holds the scores in between).
 */
int scan2d_block_attn_pool(const scan2d_desc* desc, int D, const void* h, const void* V, const float* w,
                           const uint8_t* mask, float* attn, float* z, void* stream);

/*
 * The linear layers of a block (Fig. 2: the projections into the block's inner width and back; Sec. 3.2 keeps the
 * design of the original block) at every position of a channel-major map:
 *     out[b,o,i,j] = bias[o] + sum_{c<Cin} Wt[o,c] * in[b,c,i,j] + residual[b,o,i,j]
 *   in : [Bt][Cin][H][W] with Cin = desc.Dc, Wt : [Cout][Cin], both storage type;  bias : [Cout] fp32 or NULL;
 *   residual : [Bt][Cout][H][W] storage type or NULL (the skip connection around the block; may be `out` itself);
 *   out : [Bt][Cout][H][W] storage type (written; out == in is refused with SCAN2D_ERR_BAD_SHAPE).
 *   The product runs on the matrix cores (inputs as stored, fp32 accumulation); bias and residual are added in fp32
 *   and the sum is rounded once.  The input projection of a block is two calls, one per half of its rows, so that
 *   both halves are tensors of their own.  Cout >= 1 (else SCAN2D_ERR_BAD_SHAPE); any Cin, any H*W (multiples of 4
 *   take the fast path).  desc.N and desc.flags are not used.  Device pointers, 16-byte aligned; asynchronous on
 *   `stream`; no workspace.
 */
int scan2d_block_linear(const scan2d_desc* desc, int Cout, const void* in, const void* Wt, const float* bias,
                        const void* residual, void* out, void* stream);

/*
 * The normalisation in front of a block (Sec. 3.3 lists normalization, projection and convolution in front of the scan
 * and does not say which normalisation; both kinds the Mamba blocks in use take are offered), over the channels c of
 * every position of a channel-major map:
 *     SCAN2D_LAYER_NORM : out = (in - mean_c in) / sqrt(var_c in + eps) * gamma[c] + beta[c]     (biased variance)
 *     SCAN2D_RMS_NORM   : out = in / sqrt(mean_c in^2 + eps) * gamma[c] + beta[c]
 *   in, out : [Bt][C][H][W] storage type with C = desc.Dc (out is written; out == in is allowed);
 *   gamma : [C] fp32;  beta : [C] fp32 or NULL (= 0).  fp32 arithmetic (mean first, then the mean of the squared
 *   deviations), one rounding.  eps >= 0 and kind one of the two (else SCAN2D_ERR_BAD_SHAPE).  desc.N and desc.flags
 *   are not used.  Device pointers, 16-byte aligned; asynchronous on `stream`; no workspace.
 */
enum { SCAN2D_LAYER_NORM = 0, SCAN2D_RMS_NORM = 1 };
int scan2d_block_norm(const scan2d_desc* desc, int kind, float eps, const void* in, const float* gamma,
                      const float* beta, void* out, void* stream);

/*
 * scan2d_bwd for callers that cannot allocate device memory (code under HIP graph capture, tight serving or
 * training loops, harnesses that forbid hipMalloc): the same computation and the same kernels as scan2d_bwd,
 * every argument as there, but no workspace argument.  The band checkpoints and partial sums go to a scratch
 * array of SCAN2D_STATIC_SCRATCH_BYTES bytes that is part of the library's device code: every GPU the library
 * runs on holds one copy from load time until the process ends.  The call allocates nothing and frees nothing.
 *   - A descriptor whose scan2d_workspace_bytes(desc, SCAN2D_PASS_BWD) exceeds SCAN2D_STATIC_SCRATCH_BYTES is
 *     refused with SCAN2D_ERR_SCRATCH_LIMIT before anything is enqueued (use scan2d_bwd with a workspace).
 *   - All calls on one GPU share that GPU's array: two calls that overlap in time on the same GPU (different
 *     streams, or different host threads) race on it.  Calls on one stream are ordered and safe.  Nothing in
 *     the array has to survive from one call to the next and nothing has to start at zero: every kernel
 *     writes what it later reads.
 *   - The first call on a device asks the runtime once for the array's address on that device.
 */
#define SCAN2D_STATIC_SCRATCH_BYTES (32u * 1024u * 1024u)
int scan2d_bwd_static_scratch(const scan2d_desc* desc,
                              const void* x, const void* delta, const float* A,
                              const void* Bm, const void* Cm, const float* Dskip, const uint8_t* mask,
                              const void* dy,
                              void* dx, void* ddelta, float* dA, float* dBm, float* dCm, float* dDskip,
                              void* stream);

/* Bytes of workspace a call with this descriptor needs (pass = SCAN2D_PASS_FWD for the three forward
 * calls, SCAN2D_PASS_BWD / _BWD_SOFTPLUS / _BWD_GATED for scan2d_bwd / _bwd_softplus / _bwd_softplus_gated).
 * Returns 0 for an invalid descriptor (the call itself then reports the error). */
size_t scan2d_workspace_bytes(const scan2d_desc* desc, int pass);

/*
 * Diagnostic, not part of the paper's operator: writes a one-line description of the launch plan
 * the library would use for this descriptor and pass (kernel form, lane-group width LG, columns K
 * and states NW per lane, wavefronts per workgroup, rows per barrier or per band, channels per
 * workgroup, workgroups, dynamic LDS bytes, workspace bytes) into `text` (host memory, at most
 * `text_bytes` bytes including the terminating 0).  The workspace figure is that of the scan kernels alone
 * (without the buffers of the gate, the identity cells and the columns-first order); with
 * SCAN2D_FLAG_COLUMNS_FIRST the text starts with "columns-first(in-kernel)" or with "columns-first(transposed)",
 * and the plan is then that of the transposed maps.  Touches no device memory and enqueues nothing.
 * Returns SCAN2D_OK, or the error code the corresponding call would return for this descriptor.
 */
int scan2d_describe_plan(const scan2d_desc* desc, int pass, char* text, size_t text_bytes);

/*
 * Test and tuning hook, not part of the paper's operator: forces a kernel variant for every later call of this
 * process (n = 0 clears the override).  kind 0: the plain forward kernels, values LG,K,NW,WAVES[,RPB];
 * kind 1: the forward kernels that share the per-position work of a map through LDS, values LG,K,NW,WAVES,RPB[,SKEW]
 * (SKEW = 1: the tilings with skewed rows, which nothing else selects; the single value 0 = never use that form); kind 2: the banded backward, values LG,K[,WAVES[,GS]].
 * A forced variant that does not fit a descriptor is ignored for that call.  The same overrides can be given
 * once at start-up through the environment (SCAN2D_FWD_VARIANT, SCAN2D_FWD_SHARED, SCAN2D_BWD_VARIANT, comma
 * separated); the environment is read once per process, never by the entry points.  `values` is host memory.
 * This is the library's only mutable process-wide state: do not call it while another thread is inside an
 * entry point.  Returns SCAN2D_OK, SCAN2D_ERR_BAD_FLAGS for an unknown kind, SCAN2D_ERR_NULL_POINTER.
 */
int scan2d_debug_force_variant(int kind, const int* values, int n);

/* Static, never-NULL description of an error code. */
const char* scan2d_strerror(int code);

/* Library version: major * 10000 + minor * 100 + patch. */
int scan2d_version(void);

#ifdef __cplusplus
}
#endif
#endif /* SCAN2D_H_ */
