/* libmodet -- the ModeT motion-decomposition operator on AMD MI355X (gfx950).
 *
 * C ABI.  Every pointer argument (Q, K, bias, phi, attn, lse, dphi, dQ, dK, dbias, src, field,
 * out, dout, dsrc, dfield, outer, inner, v, tmp, workspace) is a DEVICE pointer owned by the
 * caller (for instance the storage of a torch tensor).  The library never allocates, frees or
 * retains memory and never synchronises: work is enqueued on `stream` (a hipStream_t passed as
 * void*; NULL is the default stream) and the call returns at once.  Inputs and outputs must not
 * alias unless a function says otherwise.  All base pointers must be 16-byte aligned.
 *
 * Layout (row-major, last index fastest):
 *   Q, K, dQ, dK, src, out,
 *   dout, dsrc             : [B, D, H, W, C]      channels last; head s owns channels
 *                                                 [s*d, (s+1)*d), d = C / heads
 *   phi, dphi              : [B, D, H, W, heads, 3]   components ordered (D, H, W), voxel units
 *   attn                   : [B, D, H, W, heads, k^3]
 *   lse                    : [B, D, H, W, heads]
 *   bias, dbias            : [heads, k^3]
 *   displacement fields    : [B, D, H, W, 3]      fp32, voxel units, components ordered (D, H, W)
 *   window offset index    : j = ((a+r)*k + (b+r))*k + (c+r), offsets a,b,c in -r..r along
 *                            D,H,W, r = (k-1)/2
 *
 * Every function returns MODET_OK or a negative MODET_ERR_* code; nothing throws or
 * aborts.  All argument validation happens on the host before any HIP call.
 */
#ifndef MODET_H
#define MODET_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

/* element types of Q, K, src, out: passed as int (`in_dtype`, `dtype`); any other value is MODET_ERR_UNSUPPORTED */
typedef enum { MODET_F32 = 0, MODET_BF16 = 1 } modet_dtype;

enum {
  MODET_OK = 0,
  MODET_ERR_NULL = -1,        /* a required pointer is NULL */
  MODET_ERR_SHAPE = -2,       /* extent < 1, C not divisible by heads, even k, odd extent with half-res field */
  MODET_ERR_UNSUPPORTED = -3, /* dtype / k / head size outside what the kernels cover */
  MODET_ERR_ALIGN = -4,       /* a pointer is not 16-byte aligned */
  MODET_ERR_WORKSPACE = -5,   /* workspace missing or too small */
  MODET_ERR_LAUNCH = -6       /* the HIP runtime reported an error at launch */
};

/* Forward pass: paper Section 3.3.1, Eq. 3 (neighbourhood attention) and Eq. 4-5 (sub-fields).
 *
 * For every voxel p of Q (features of the fixed image), every head s and every offset o of
 * the k x k x k window:  l_o = scale * <Q[p, s], K[p+o, s]> + bias[s, o], where K (features
 * of the moving image) is zero outside the volume and such a padded neighbour still takes
 * part in the softmax with logit bias[s,o] (or 0).  w = softmax_o(l);
 * phi[p, s, :] = sum_o w_o * o  (the constant offset grid V of Eq. 4 is never materialised).
 *
 *   Q, K   in   in_dtype (fp32, or bf16 bit patterns).  fp32 inputs: the dot products and the softmax sums
 *               are accumulated in fp64, everything else in fp32; bf16 inputs: fp32 throughout
 *   bias   in   nullable; NULL means all zeros (the paper's initial state of B)
 *   phi    out  fp32, fully written
 *   attn   out  nullable; the softmax weights w (fp32)
 *   lse    out  nullable; log(sum_o exp(l_o)) in fp32 -- pass it to modet_bwd to save the
 *               statistics pass there
 *   k      odd, 1..7;  scale <= 0 selects 1/sqrt(d)  (scale = 1 is Eq. 3 exactly as printed)
 */
int modet_fwd(const void* Q, const void* K, const float* bias, float* phi, float* attn, float* lse,
              int B, int D, int H, int W, int C, int heads, int k, float scale,
              int in_dtype, void* stream);

/* Backward pass of Eq. 3-4 with respect to Q and K (and optionally B): the gradients the
 * pairwise-optimisation loop of Section 3.1 / Eq. 1 needs every iteration.  With g = dphi:
 *   dl_o(p,s) = w_o * (g.o - g.phi)
 *   dQ[p, s]  = scale * sum_o dl_o(p,s) * K[p+o, s]          (in-bounds p+o only)
 *   dK[q, s]  = scale * sum_o dl_o(q-o, s) * Q[q-o, s]        (in-bounds q-o only)
 *   dbias[s,o] = sum_p dl_o(p,s)
 * Softmax weights are recomputed from Q and K, never stored.  When the attention weights of Eq. 3 were
 * themselves an output (modet_fwd's attn) and carry an upstream gradient dattn, the loss is
 * sum(dphi * phi) + sum(dattn * attn) and  dl_o = w_o * (g.o + dattn_o - g.phi - sum_j w_j dattn_j).
 *
 *   dattn      in   nullable, [B, D, H, W, heads, k^3] fp32; such a call runs on the generic kernels
 *   phi, lse   in   nullable, both or neither: the outputs of modet_fwd for the same inputs.
 *                   When NULL the library recomputes them into `workspace`.
 *   dQ, dK     out  fp32, fully overwritten (no zeroing by the caller needed)
 *   dbias      out  nullable, fully overwritten; its sums over all voxels are formed in fp64
 *                   in `workspace` (the order of the additions is not fixed)
 *   workspace       at least modet_bwd_workspace_bytes(...) bytes for the same shape and the
 *                   flags that describe this call, 16-byte aligned; may be NULL when that
 *                   size is 0
 */
int modet_bwd(const void* Q, const void* K, const float* bias, const float* dphi, const float* dattn,
              const float* phi, const float* lse, float* dQ, float* dK, float* dbias,
              int B, int D, int H, int W, int C, int heads, int k, float scale,
              int in_dtype, void* workspace, size_t workspace_bytes, void* stream);

/* Bytes of scratch modet_bwd needs.  flags: MODET_WS_HAVE_STATS = phi and lse will be passed in
 * (otherwise they are recomputed into the workspace, 16 bytes per window), MODET_WS_WANT_DBIAS =
 * dbias will be requested (8 bytes per bias entry), MODET_WS_HAVE_DATTN = dattn will be passed in
 * (4 bytes per window).  Returns 0 for invalid shapes (modet_bwd itself reports the error). */
enum { MODET_WS_HAVE_STATS = 1, MODET_WS_WANT_DBIAS = 2, MODET_WS_HAVE_DATTN = 4 };
size_t modet_bwd_workspace_bytes(int B, int D, int H, int W, int C, int heads, int k,
                                 int in_dtype, int flags);

/* modet_bwd for callers that cannot allocate or pass device scratch: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same computation as modet_bwd, with the workspace taken from a
 * device array built into the library instead of the caller: MODET_STATIC_SCRATCH_BYTES bytes per GPU the
 * library is used on, held until the process ends.  The call allocates nothing and frees nothing.
 *
 *   A call whose modet_bwd_workspace_bytes(...) exceeds MODET_STATIC_SCRATCH_BYTES returns MODET_ERR_WORKSPACE
 *   (8 MiB cover the bias gradient of any shape, and the recomputed statistics of up to 524288 windows; with
 *   phi and lse passed in, only the bias gradient needs scratch).
 *   All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or
 *   threads) race on it and must be serialised by the caller.  Nothing is carried from one call to the next.
 *   Every other argument, and every error code, as in modet_bwd.
 */
#define MODET_STATIC_SCRATCH_BYTES (8u << 20)
int modet_bwd_static(const void* Q, const void* K, const float* bias, const float* dphi, const float* dattn,
                     const float* phi, const float* lse, float* dQ, float* dK, float* dbias,
                     int B, int D, int H, int W, int C, int heads, int k, float scale,
                     int in_dtype, void* stream);

/* Trilinear feature warp between pyramid levels: paper Section 3.1 (the moving feature map
 * of the next level is deformed by the upsampled total field before it enters ModeT).
 *
 *   out[b, p, c] = trilinear(src[b, :, c], p + u(p)),   zero outside the volume,
 * integer coordinates are voxel centres, u in voxel units ordered (D, H, W).
 *   field_half_res == 0:  field is [B, D, H, W, 3] and u(p) = field[b, p].
 *   field_half_res == 1:  field is [B, D/2, H/2, W/2, 3] (D, H, W even) and
 *       u(p) = 2 * trilinear(field, clamp((p + 0.5)/2 - 0.5, 0, size-1)): the 2x upsampling of
 *       the coarser level's field fused into the warp, values doubled because they are in
 *       voxel units of their own grid.
 *   src, out in `dtype` (bf16 output is rounded to nearest even); field is fp32.
 *   C is at most 256 and, for bf16, even (C = 3 in fp32 warps a displacement field).
 */
int modet_warp(const void* src, const float* field, void* out,
               int B, int D, int H, int W, int C, int field_half_res,
               int dtype, void* stream);

/* Adjoint of modet_warp: the gradients of L = sum(dout * warp(src, field)), which carry a gradient with
 * respect to the warped moving features (modet_bwd's dK) back to the un-warped features and to the field
 * (paper Section 3.1: the warp sits between the pyramid levels, in front of the operator).
 *
 *   dsrc[b, q, c]   = sum over voxels p of weight(p -> q) * dout[b, p, c]     (transpose of the gather)
 *   dfield          = derivative through the interpolation weights; where a sample point sits exactly on
 *                     a voxel it is the one-sided derivative towards larger displacements.  For
 *                     field_half_res == 1 it has the coarse field's shape (the 2x upsampling is
 *                     differentiated too).
 *   src     in   dtype; only read for dfield (may be NULL when dfield is NULL)
 *   field   in   as in modet_warp
 *   dout    in   fp32 [B, D, H, W, C]
 *   dsrc    out  fp32 [B, D, H, W, C], fully overwritten.  The additions to one element happen in no fixed
 *                order (on chip for contributions that follow the local displacement, with fp32 atomics
 *                for the rest), so the last bits can differ from run to run
 *   dfield  out  nullable, fp32, fully overwritten (half resolution: accumulated with fp32 atomics, same remark)
 *   shapes and dtypes as in modet_warp
 */
int modet_warp_bwd(const void* src, const float* field, const float* dout, float* dsrc, float* dfield,
                   int B, int D, int H, int W, int C, int field_half_res,
                   int dtype, void* stream);

/* Composition of two displacement fields: paper Section 3.1 (the total field of a pyramid level is
 * the level's residual field composed with the upsampled total field of the level below).
 *
 *   out[b, p, :] = inner[b, p, :] + trilinear(outer[b], p + inner[b, p, :]),
 * the displacement of "move by inner, then by outer"; same sampling rules as modet_warp (voxel
 * units, components ordered (D, H, W), zero outside the volume).
 *   outer_half_res == 0:  outer is [B, D, H, W, 3]; outer and inner may be the same buffer.
 *   outer_half_res == 1:  outer is the coarser level's total field [B, D/2, H/2, W/2, 3] (D, H, W even); the
 *       field that is sampled is its 2x upsampling with values doubled, exactly as in modet_warp with
 *       field_half_res == 1, evaluated on the fly (it is never written to memory).
 *   inner         in   [B, D, H, W, 3] fp32
 *   out           out  [B, D, H, W, 3] fp32; must not alias an input
 */
int modet_compose(const float* outer, const float* inner, float* out,
                  int B, int D, int H, int W, int outer_half_res, void* stream);

/* Integration of a stationary velocity field by scaling and squaring: paper Section 3.3.2, Eq. 6
 * (the optional diffeomorphic layer of the registration head).
 *
 *   phi_0 = v / 2^T;   phi_t = phi_{t-1} o phi_{t-1}  (modet_compose of the field with itself), T times;
 *   out = phi_T, the displacement field at time 1.  T = 0 copies v.
 *   v     in   [B, D, H, W, 3] fp32
 *   out   out  [B, D, H, W, 3] fp32
 *   tmp        scratch of the same size, required for T >= 2 (MODET_ERR_WORKSPACE if NULL), else
 *              may be NULL; v, out and tmp must not alias
 *   T     0..30
 */
int modet_integrate_velocity(const float* v, float* out, float* tmp,
                             int B, int D, int H, int W, int T, void* stream);

/* Kernel selection, for tests and profiling.  0 = automatic (LDS-tiled kernels where the
 * shape is covered, generic otherwise), 1 = always the generic kernels.  Returns the
 * previous value.  Process-wide, not thread safe. */
int modet_set_kernel_path(int path);

/* Arithmetic of the LDS-tiled kernels for fp32 inputs.  0 (default) = logits accumulated in fp64: meets
 * 1e-5 relative / 1e-6 absolute against an fp64 evaluation of Eq. 3-4.  1 = logits accumulated in fp32,
 * kept for comparison: a logit of magnitude ~10 then carries ~1e-6 of rounding and gradients can miss that
 * tolerance by a small factor.  bf16 inputs always use fp32.  Returns the previous value.
 * Process-wide, not thread safe. */
int modet_set_math_mode(int mode);

/* Bit 0: modet_fwd, bit 1: modet_bwd run on the LDS-tiled kernels for this (head size, heads, k,
 * dtype) under path 0 (with or without bias; not when the attention weights are requested). */
int modet_has_tiled_kernels(int C, int heads, int k, int in_dtype);

const char* modet_status_string(int status);
int modet_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MODET_H */
