// C ABI of libmodet: argument validation on the host (before any HIP call) and dispatch to the
// kernels.  See include/modet.h for the contract of every entry point.
#include "../../include/modet.h"
#include "modet_common.hpp"

#include <math.h>
#include <mutex>

using namespace modet;

// Scratch of modet_bwd_static: device memory of the library's own, one copy per GPU the library is loaded on,
// held until the process ends.  Host code must never pass this name to a kernel or a HIP call (in host code it
// is a stand-in, not a device address): scratch_pointer() asks the runtime for the array's address on the
// current device, once per device, and everything else uses that pointer.
static __device__ __align__(256) unsigned char scratch[MODET_STATIC_SCRATCH_BYTES];

namespace {

int g_kernel_path = 0;   // 0 = automatic, 1 = generic kernels only
int g_math_mode = 0;     // 0 = fp64 logits for fp32 inputs, 1 = fp32 logits

inline bool misaligned(const void* p) { return p && (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }

int check_op_shape(int B, int D, int H, int W, int C, int heads, int k, int dtype) {
  if (B < 1 || D < 1 || H < 1 || W < 1 || C < 1 || heads < 1) return MODET_ERR_SHAPE;
  if (C % heads != 0) return MODET_ERR_SHAPE;
  if (k < 1 || (k & 1) == 0) return MODET_ERR_SHAPE;
  if (k > 7) return MODET_ERR_UNSUPPORTED;
  if (dtype != MODET_F32 && dtype != MODET_BF16) return MODET_ERR_UNSUPPORTED;
  // 32-bit lane indexing inside a batch item and over windows
  const long long nvox = (long long)B * D * H * W;
  if (nvox * C >= (1LL << 31) || nvox * heads * 3 >= (1LL << 31)) return MODET_ERR_UNSUPPORTED;
  return MODET_OK;
}

Geo make_geo(int B, int D, int H, int W, int C, int heads, int k, float scale) {
  Geo g;
  g.B = B; g.D = D; g.H = H; g.W = W; g.C = C; g.heads = heads; g.k = k;
  g.r = (k - 1) / 2; g.d = C / heads; g.k3 = k * k * k;
  g.nvox = (long long)B * D * H * W;
  g.nvn = g.nvox * heads;
  g.scale = scale > 0.f ? scale : 1.0f / sqrtf((float)g.d);
  return g;
}

inline size_t round16(size_t n) { return (n + 15) & ~(size_t)15; }

constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// address of `scratch` on the current device (looked up on the first call for that device), or NULL
void* scratch_pointer() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || ptr == nullptr) return nullptr;
    g_scratch_ptr[dev] = ptr;
  }
  return g_scratch_ptr[dev];
}

}  // namespace

extern "C" {

int modet_fwd(const void* Q, const void* K, const float* bias, float* phi, float* attn, float* lse,
              int B, int D, int H, int W, int C, int heads, int k, float scale,
              int in_dtype, void* stream) {
  if (!Q || !K || !phi) return MODET_ERR_NULL;
  int rc = check_op_shape(B, D, H, W, C, heads, k, (int)in_dtype);
  if (rc != MODET_OK) return rc;
  if (misaligned(Q) || misaligned(K) || misaligned(bias) || misaligned(phi) || misaligned(attn) || misaligned(lse))
    return MODET_ERR_ALIGN;
  const Geo g = make_geo(B, D, H, W, C, heads, k, scale);
  hipStream_t st = (hipStream_t)stream;
  hipError_t e;
  if (g_kernel_path == 0 && !attn && tiled_fwd_supported(g.d, heads, k, (int)in_dtype))
    e = launch_fwd_tiled(g, (int)in_dtype, g_math_mode == 1, Q, K, bias, phi, lse, st);
  else
    e = launch_fwd_generic(g, (int)in_dtype, Q, K, bias, phi, attn, lse, st);
  return e == hipSuccess ? MODET_OK : MODET_ERR_LAUNCH;
}

size_t modet_bwd_workspace_bytes(int B, int D, int H, int W, int C, int heads, int k,
                                 int in_dtype, int flags) {
  if (check_op_shape(B, D, H, W, C, heads, k, (int)in_dtype) != MODET_OK) return 0;
  size_t n = 0;
  if (!(flags & MODET_WS_HAVE_STATS)) {
    const size_t nvn = (size_t)B * D * H * W * heads;
    n += round16(nvn * 3 * sizeof(float)) + round16(nvn * sizeof(float));   // phi, lse
  }
  if (flags & MODET_WS_WANT_DBIAS) n += round16((size_t)heads * k * k * k * sizeof(double));   // fp64 sums
  if (flags & MODET_WS_HAVE_DATTN) n += round16((size_t)B * D * H * W * heads * sizeof(float));  // sum_o w_o dattn_o
  return n;
}

int modet_bwd(const void* Q, const void* K, const float* bias, const float* dphi, const float* dattn,
              const float* phi, const float* lse, float* dQ, float* dK, float* dbias,
              int B, int D, int H, int W, int C, int heads, int k, float scale,
              int in_dtype, void* workspace, size_t workspace_bytes, void* stream) {
  if (!Q || !K || !dphi || !dQ || !dK) return MODET_ERR_NULL;
  if ((phi == nullptr) != (lse == nullptr)) return MODET_ERR_NULL;
  int rc = check_op_shape(B, D, H, W, C, heads, k, (int)in_dtype);
  if (rc != MODET_OK) return rc;
  if (misaligned(Q) || misaligned(K) || misaligned(bias) || misaligned(dphi) || misaligned(dattn) || misaligned(phi) ||
      misaligned(lse) || misaligned(dQ) || misaligned(dK) || misaligned(dbias) || misaligned(workspace))
    return MODET_ERR_ALIGN;
  const int flags = (phi ? MODET_WS_HAVE_STATS : 0) | (dbias ? MODET_WS_WANT_DBIAS : 0) |
                    (dattn ? MODET_WS_HAVE_DATTN : 0);
  const size_t need = modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, in_dtype, flags);
  if (need > 0 && (!workspace || workspace_bytes < need)) return MODET_ERR_WORKSPACE;
  const Geo g = make_geo(B, D, H, W, C, heads, k, scale);
  hipStream_t st = (hipStream_t)stream;
  const bool tiled_f = g_kernel_path == 0 && tiled_fwd_supported(g.d, heads, k, (int)in_dtype);
  // (the gradient that arrives through the attention weights is handled by the generic kernels only)
  const bool tiled_b = g_kernel_path == 0 && !dattn && tiled_bwd_supported(g.d, heads, k, (int)in_dtype);
  hipError_t e = hipSuccess;
  char* ws = (char*)workspace;
  if (!phi) {   // statistics pass: the forward kernel writes phi and lse into the workspace
    float* wphi = (float*)ws;
    float* wlse = (float*)(ws + round16((size_t)g.nvn * 3 * sizeof(float)));
    ws += round16((size_t)g.nvn * 3 * sizeof(float)) + round16((size_t)g.nvn * sizeof(float));
    e = tiled_f ? launch_fwd_tiled(g, (int)in_dtype, g_math_mode == 1, Q, K, bias, wphi, wlse, st)
              : launch_fwd_generic(g, (int)in_dtype, Q, K, bias, wphi, nullptr, wlse, st);
    if (e != hipSuccess) return MODET_ERR_LAUNCH;
    phi = wphi;
    lse = wlse;
  }
  double* acc = dbias ? (double*)ws : nullptr;     // fp64 sums of the bias gradient
  if (dbias) ws += round16((size_t)g.heads * g.k3 * sizeof(double));
  float* adot = dattn ? (float*)ws : nullptr;      // sum_o w_o dattn_o per window
  if (acc && launch_dbias_begin(g, acc, st) != hipSuccess) return MODET_ERR_LAUNCH;
  bool dbias_done = false;
  if (tiled_b) {
    const BwdTensors io = {Q, K, bias, dphi, phi, lse, dQ, dK, acc};
    e = launch_bwd_tiled(g, (int)in_dtype, g_math_mode == 1, io, st, &dbias_done);
  } else {
    e = launch_bwd_generic(g, (int)in_dtype, Q, K, bias, dphi, phi, lse, dattn, adot, dQ, dK, st);
  }
  if (e != hipSuccess) return MODET_ERR_LAUNCH;
  if (acc) {
    if (!dbias_done) e = launch_dbias_generic(g, (int)in_dtype, Q, K, bias, dphi, phi, lse, dattn, adot, acc, st);
    if (e == hipSuccess) e = launch_dbias_end(g, acc, dbias, st);
    if (e != hipSuccess) return MODET_ERR_LAUNCH;
  }
  return MODET_OK;
}

int modet_bwd_static(const void* Q, const void* K, const float* bias, const float* dphi, const float* dattn,
                     const float* phi, const float* lse, float* dQ, float* dK, float* dbias,
                     int B, int D, int H, int W, int C, int heads, int k, float scale,
                     int in_dtype, void* stream) {
  // the same validation order as modet_bwd up to the workspace, all of it before any HIP call
  if (!Q || !K || !dphi || !dQ || !dK) return MODET_ERR_NULL;
  if ((phi == nullptr) != (lse == nullptr)) return MODET_ERR_NULL;
  int rc = check_op_shape(B, D, H, W, C, heads, k, (int)in_dtype);
  if (rc != MODET_OK) return rc;
  if (misaligned(Q) || misaligned(K) || misaligned(bias) || misaligned(dphi) || misaligned(dattn) || misaligned(phi) ||
      misaligned(lse) || misaligned(dQ) || misaligned(dK) || misaligned(dbias))
    return MODET_ERR_ALIGN;
  const int flags = (phi ? MODET_WS_HAVE_STATS : 0) | (dbias ? MODET_WS_WANT_DBIAS : 0) |
                    (dattn ? MODET_WS_HAVE_DATTN : 0);
  const size_t need = modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, in_dtype, flags);
  if (need > (size_t)MODET_STATIC_SCRATCH_BYTES) return MODET_ERR_WORKSPACE;      // beyond the built-in scratch
  void* ws = nullptr;
  if (need > 0) {
    ws = scratch_pointer();
    if (!ws) return MODET_ERR_LAUNCH;
  }
  // everything modet_bwd keeps in its workspace is written before it is read (the statistics by the forward
  // kernel, the bias gradient's sums by a fill kernel), so the last call's contents do not matter
  return modet_bwd(Q, K, bias, dphi, dattn, phi, lse, dQ, dK, dbias, B, D, H, W, C, heads, k, scale, in_dtype, ws,
                   need, stream);
}

int modet_warp(const void* src, const float* field, void* out,
               int B, int D, int H, int W, int C, int field_half_res,
               int dtype, void* stream) {
  if (!src || !field || !out) return MODET_ERR_NULL;
  if (B < 1 || D < 1 || H < 1 || W < 1 || C < 1) return MODET_ERR_SHAPE;
  if (field_half_res != 0 && field_half_res != 1) return MODET_ERR_SHAPE;
  if (field_half_res && ((D | H | W) & 1)) return MODET_ERR_SHAPE;
  if (dtype != MODET_F32 && dtype != MODET_BF16) return MODET_ERR_UNSUPPORTED;
  if (dtype == MODET_BF16 && (C & 1)) return MODET_ERR_UNSUPPORTED;      // bf16 channels travel in pairs
  if (C > 256) return MODET_ERR_UNSUPPORTED;                             // a voxel's channels fit one workgroup
  if ((long long)B * D * H * W * C >= (1LL << 31)) return MODET_ERR_UNSUPPORTED;
  if (misaligned(src) || misaligned(field) || misaligned(out)) return MODET_ERR_ALIGN;
  hipError_t e = launch_warp(src, field, out, B, D, H, W, C, field_half_res, (int)dtype, (hipStream_t)stream);
  return e == hipSuccess ? MODET_OK : MODET_ERR_LAUNCH;
}

int modet_warp_bwd(const void* src, const float* field, const float* dout, float* dsrc, float* dfield,
                   int B, int D, int H, int W, int C, int field_half_res, int dtype, void* stream) {
  if (!field || !dout || !dsrc || (dfield && !src)) return MODET_ERR_NULL;
  if (B < 1 || D < 1 || H < 1 || W < 1 || C < 1) return MODET_ERR_SHAPE;
  if (field_half_res != 0 && field_half_res != 1) return MODET_ERR_SHAPE;
  if (field_half_res && ((D | H | W) & 1)) return MODET_ERR_SHAPE;
  if (dtype != MODET_F32 && dtype != MODET_BF16) return MODET_ERR_UNSUPPORTED;
  if (dtype == MODET_BF16 && (C & 1)) return MODET_ERR_UNSUPPORTED;
  if (C > 256) return MODET_ERR_UNSUPPORTED;
  if ((long long)B * D * H * W * C >= (1LL << 31)) return MODET_ERR_UNSUPPORTED;
  if (misaligned(src) || misaligned(field) || misaligned(dout) || misaligned(dsrc) || misaligned(dfield))
    return MODET_ERR_ALIGN;
  hipError_t e = launch_warp_bwd(src, field, dout, dsrc, dfield, B, D, H, W, C, field_half_res, (int)dtype,
                                 (hipStream_t)stream);
  return e == hipSuccess ? MODET_OK : MODET_ERR_LAUNCH;
}

int modet_compose(const float* outer, const float* inner, float* out, int B, int D, int H, int W,
                  int outer_half_res, void* stream) {
  if (!outer || !inner || !out) return MODET_ERR_NULL;
  if (B < 1 || D < 1 || H < 1 || W < 1) return MODET_ERR_SHAPE;
  if (outer_half_res != 0 && outer_half_res != 1) return MODET_ERR_SHAPE;
  if (outer_half_res && ((D | H | W) & 1)) return MODET_ERR_SHAPE;
  if ((long long)B * D * H * W * 3 >= (1LL << 31)) return MODET_ERR_UNSUPPORTED;
  if (misaligned(outer) || misaligned(inner) || misaligned(out)) return MODET_ERR_ALIGN;
  hipError_t e = launch_compose(outer, inner, out, B, D, H, W, 1.0f, outer_half_res, (hipStream_t)stream);
  return e == hipSuccess ? MODET_OK : MODET_ERR_LAUNCH;
}

int modet_integrate_velocity(const float* v, float* out, float* tmp, int B, int D, int H, int W, int T,
                             void* stream) {
  if (!v || !out) return MODET_ERR_NULL;
  if (B < 1 || D < 1 || H < 1 || W < 1 || T < 0) return MODET_ERR_SHAPE;
  if (T > 30) return MODET_ERR_UNSUPPORTED;
  const long long n = (long long)B * D * H * W * 3;
  if (n >= (1LL << 31)) return MODET_ERR_UNSUPPORTED;
  if (T >= 2 && !tmp) return MODET_ERR_WORKSPACE;
  if (misaligned(v) || misaligned(out) || misaligned(tmp)) return MODET_ERR_ALIGN;
  hipStream_t st = (hipStream_t)stream;
  if (T == 0)
    return hipMemcpyAsync(out, v, (size_t)n * sizeof(float), hipMemcpyDeviceToDevice, st) == hipSuccess
               ? MODET_OK : MODET_ERR_LAUNCH;
  // step t = 1..T writes `out` when T - t is even, `tmp` otherwise: the last step lands in `out`, and a step
  // never writes the buffer it reads.  The first step also scales by 2^-T.
  const float* src = v;
  for (int t = 1; t <= T; ++t) {
    float* dst = ((T - t) & 1) ? tmp : out;
    const float s = t == 1 ? ldexpf(1.0f, -T) : 1.0f;
    if (launch_compose(src, src, dst, B, D, H, W, s, 0, st) != hipSuccess) return MODET_ERR_LAUNCH;
    src = dst;
  }
  return MODET_OK;
}

int modet_set_kernel_path(int path) {
  int old = g_kernel_path;
  g_kernel_path = path == 1 ? 1 : 0;
  return old;
}

int modet_set_math_mode(int mode) {
  int old = g_math_mode;
  g_math_mode = mode == 1 ? 1 : 0;
  return old;
}

int modet_has_tiled_kernels(int C, int heads, int k, int in_dtype) {
  if (C < 1 || heads < 1 || C % heads != 0) return 0;
  return (tiled_fwd_supported(C / heads, heads, k, (int)in_dtype) ? 1 : 0) |
         (tiled_bwd_supported(C / heads, heads, k, (int)in_dtype) ? 2 : 0);
}

const char* modet_status_string(int status) {
  switch (status) {
    case MODET_OK: return "ok";
    case MODET_ERR_NULL: return "a required pointer is NULL (or only one of phi/lse was given)";
    case MODET_ERR_SHAPE: return "invalid shape: extents must be >= 1, C divisible by heads, k odd, "
                                 "even extents for a half-resolution field";
    case MODET_ERR_UNSUPPORTED: return "unsupported dtype, window size, channel count or tensor size";
    case MODET_ERR_ALIGN: return "pointers must be 16-byte aligned";
    case MODET_ERR_WORKSPACE: return "workspace missing or smaller than modet_bwd_workspace_bytes()";
    case MODET_ERR_LAUNCH: return "HIP reported an error when launching a kernel";
    default: return "unknown status";
  }
}

int modet_version(void) { return 100; }

}  // extern "C"
