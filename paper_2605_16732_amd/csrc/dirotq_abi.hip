// C-ABI entry points of libdirotq: argument validation, size queries, error
// reporting.  All checks run on the host before anything is enqueued.
#include <mutex>

#include "dirotq_internal.h"

namespace dirotq {

// Intermediates of dirotq_linear_static (x_h, packed x_l, s_x of one call): a fixed array in
// device memory, one copy per GPU the library runs on, held until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current GPU.  In host code the array's name is only a
// handle for the runtime: the address is asked for once per device and kept.
constexpr int kMaxDevices = 64;
static std::mutex g_scratch_mutex;
static void* g_scratch_ptr[kMaxDevices] = {};
static int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return hip_failed(e);
  if (dev < 0 || dev >= kMaxDevices) return DIROTQ_ERR_UNSUPPORTED;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return hip_failed(e);
    if (!p) return DIROTQ_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return DIROTQ_OK;
}

static thread_local int g_last_hip_error = 0;

int hip_failed(hipError_t e) {
  g_last_hip_error = (int)e;
  return DIROTQ_ERR_HIP;
}

int check_shape(long M, long N, long K, long r, long g) {
  if (M < 0 || N < 1) return DIROTQ_ERR_SHAPE;
  if (K < 32 || K % 32 != 0 || K > (1 << 20)) return DIROTQ_ERR_SHAPE;
  if (r < 0 || r > K || r % 32 != 0) return DIROTQ_ERR_SHAPE;
  if (!(g == 32 || g == 64 || g == 128)) return DIROTQ_ERR_SHAPE;
  if ((K - r) % g != 0) return DIROTQ_ERR_SHAPE;
  if (M > (1 << 24) || N > (1 << 24)) return DIROTQ_ERR_SHAPE;
  // the GEMM grids are one workgroup per 128 x 128 output tile, indexed with 32-bit integers
  if (((M + 127) / 128) * ((N + 127) / 128) > (1L << 30)) return DIROTQ_ERR_SHAPE;
  return DIROTQ_OK;
}

}  // namespace dirotq

using namespace dirotq;

extern "C" {

const char* dirotq_strerror(int status) {
  switch (status) {
    case DIROTQ_OK: return "ok";
    case DIROTQ_ERR_NULL: return "a required pointer is NULL";
    case DIROTQ_ERR_SHAPE:
      return "bad shape: need M>=0, N>=1, K%32==0, 0<=r<=K, r%32==0, g in {32,64,128}, (K-r)%g==0";
    case DIROTQ_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case DIROTQ_ERR_WORKSPACE: return "workspace or scratch buffer too small";
    case DIROTQ_ERR_UNSUPPORTED: return "request not supported by this build";
    case DIROTQ_ERR_HIP: return "a HIP call failed (see dirotq_last_hip_error)";
    case DIROTQ_ERR_STATIC_LIMIT:
      return "intermediates exceed the 64 MiB static scratch of dirotq_linear_static: use dirotq_linear";
    default: return "unknown status";
  }
}

int dirotq_last_hip_error(void) { return g_last_hip_error; }

int dirotq_weights_bytes(int N, int K, int r, int g, size_t* bytes) {
  if (!bytes) return DIROTQ_ERR_NULL;
  int st = check_shape(0, N, K, r, g);
  if (st) return st;
  *bytes = blob_layout(N, K, r, g).bytes;
  return DIROTQ_OK;
}

int dirotq_prepare_scratch_bytes(int N, int K, size_t* bytes) {
  if (!bytes) return DIROTQ_ERR_NULL;
  int st = check_shape(0, N, K, 0, 32);
  if (st) return st;
  *bytes = align_up((size_t)N * K * sizeof(float));
  return DIROTQ_OK;
}

int dirotq_workspace_bytes(int M, int K, int r, int g, size_t* bytes) {
  if (!bytes) return DIROTQ_ERR_NULL;
  int st = check_shape(M, 1, K, r, g);
  if (st) return st;
  *bytes = workspace_layout(M, K, r, g).bytes;
  return DIROTQ_OK;
}

int dirotq_prepare_rotation(const float* Q, int K, uint16_t* Qt_bf16, void* stream) {
  if (!Q || !Qt_bf16) return DIROTQ_ERR_NULL;
  int st = check_shape(0, 1, K, 0, 32);
  if (st) return st;
  if (misaligned(Q) || misaligned(Qt_bf16)) return DIROTQ_ERR_ALIGN;
  return launch_prepare_rotation(Q, K, Qt_bf16, (hipStream_t)stream);
}

int dirotq_prepare_weights(const float* W, const float* Q, int N, int K, int r, int g, void* blob,
                           void* scratch, size_t scratch_bytes, void* stream) {
  if (!W || !Q || !blob || !scratch) return DIROTQ_ERR_NULL;
  int st = check_shape(0, N, K, r, g);
  if (st) return st;
  if (misaligned(W) || misaligned(Q) || misaligned(blob) || misaligned(scratch)) return DIROTQ_ERR_ALIGN;
  if (scratch_bytes < (size_t)N * K * sizeof(float)) return DIROTQ_ERR_WORKSPACE;
  return launch_prepare_weights(W, Q, N, K, r, g, blob, (float*)scratch, (hipStream_t)stream);
}

int dirotq_import_weights(const uint16_t* Wh_bf16, const int8_t* codes, const uint16_t* sw_fp16, int N,
                          int K, int r, int g, void* blob, void* stream) {
  int st = check_shape(0, N, K, r, g);
  if (!blob) return DIROTQ_ERR_NULL;
  if (st) return st;
  if (r > 0 && !Wh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!codes || !sw_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(blob) || misaligned(Wh_bf16) || misaligned(codes) || misaligned(sw_fp16))
    return DIROTQ_ERR_ALIGN;
  return launch_import_weights(Wh_bf16, codes, sw_fp16, N, K, r, g, blob, (hipStream_t)stream);
}

int dirotq_export_weights(const void* blob, int N, int K, int r, int g, uint16_t* Wh_bf16, int8_t* codes,
                          uint16_t* sw_fp16, void* stream) {
  if (!blob) return DIROTQ_ERR_NULL;
  int st = check_shape(0, N, K, r, g);
  if (st) return st;
  if (misaligned(blob) || misaligned(Wh_bf16) || misaligned(codes) || misaligned(sw_fp16))
    return DIROTQ_ERR_ALIGN;
  return launch_export_weights(blob, N, K, r, g, Wh_bf16, codes, sw_fp16, (hipStream_t)stream);
}

int dirotq_rotate_quantize(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r, int g,
                           uint16_t* xh_bf16, uint8_t* xl_packed, uint16_t* sx_fp16, void* stream) {
  int st = check_shape(M, 1, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;   // nothing to do, no buffer is needed
  if (!x_bf16 || !Qt_bf16) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!xl_packed || !sx_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(xh_bf16) || misaligned(xl_packed) ||
      misaligned(sx_fp16))
    return DIROTQ_ERR_ALIGN;
  RqOut o;
  o.xh = xh_bf16, o.xl = xl_packed, o.sx = sx_fp16;
  return launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
}

int dirotq_w4a4_gemm(const uint16_t* xh_bf16, const uint8_t* xl_packed, const uint16_t* sx_fp16,
                     const void* blob, const uint16_t* bias_bf16, int M, int N, int K, int r, int g, void* y,
                     int y_dtype, void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (y_dtype != 0 && y_dtype != 1) return DIROTQ_ERR_UNSUPPORTED;
  if (M == 0) return DIROTQ_OK;
  if (!blob || !y) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!xl_packed || !sx_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(xh_bf16) || misaligned(xl_packed) || misaligned(sx_fp16) || misaligned(blob) ||
      misaligned(bias_bf16) || misaligned(y))
    return DIROTQ_ERR_ALIGN;
  return launch_w4a4_gemm(xh_bf16, xl_packed, sx_fp16, nullptr, blob, bias_bf16, M, N, K, r, g, y, y_dtype,
                          (hipStream_t)stream);
}

int dirotq_linear(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                  const uint16_t* bias_bf16, int M, int N, int K, int r, int g, uint16_t* y_bf16,
                  void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16 || !blob || !y_bf16 || !workspace) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(blob) || misaligned(bias_bf16) ||
      misaligned(y_bf16) || ((uintptr_t)workspace & (kAlign - 1)) != 0)
    return DIROTQ_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, K, r, g);
  if (workspace_bytes < L.bytes) return DIROTQ_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  uint16_t* xh = (uint16_t*)(ws + L.off_xh);
  uint8_t* xl = (uint8_t*)(ws + L.off_xl);
  uint16_t* sx = (uint16_t*)(ws + L.off_sx);
  RqOut o;
  o.xh = xh, o.xl = xl, o.sx = sx;
  st = launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
  if (st) return st;
  return launch_w4a4_gemm(xh, xl, sx, nullptr, blob, bias_bf16, M, N, K, r, g, y_bf16, 0, (hipStream_t)stream);
}

int dirotq_linear_static(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                         const uint16_t* bias_bf16, int M, int N, int K, int r, int g, uint16_t* y_bf16,
                         void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16 || !blob || !y_bf16) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(blob) || misaligned(bias_bf16) || misaligned(y_bf16))
    return DIROTQ_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, K, r, g);
  if (L.bytes > kStaticScratchBytes) return DIROTQ_ERR_STATIC_LIMIT;
  void* base = nullptr;
  st = static_scratch(&base);
  if (st) return st;
  char* ws = (char*)base;
  uint16_t* xh = (uint16_t*)(ws + L.off_xh);
  uint8_t* xl = (uint8_t*)(ws + L.off_xl);
  uint16_t* sx = (uint16_t*)(ws + L.off_sx);
  RqOut o;
  o.xh = xh, o.xl = xl, o.sx = sx;
  // every byte of the intermediates that the GEMM reads is written by the rotation kernel of
  // this call, so nothing of the previous call's contents has to be cleared
  st = launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
  if (st) return st;
  return launch_w4a4_gemm(xh, xl, sx, nullptr, blob, bias_bf16, M, N, K, r, g, y_bf16, 0, (hipStream_t)stream);
}

int dirotq_linear_shared(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int n_out, const void* const* blobs,
                         const uint16_t* const* biases, const int* Ns, uint16_t* const* ys, int M, int K, int r,
                         int g, void* workspace, size_t workspace_bytes, void* stream) {
  if (n_out < 1 || n_out > 16) return DIROTQ_ERR_SHAPE;
  if (!blobs || !Ns || !ys) return DIROTQ_ERR_NULL;
  for (int i = 0; i < n_out; i++) {
    int st = check_shape(M, Ns[i], K, r, g);
    if (st) return st;
  }
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16 || !workspace) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || ((uintptr_t)workspace & (kAlign - 1)) != 0) return DIROTQ_ERR_ALIGN;
  for (int i = 0; i < n_out; i++) {
    if (!blobs[i] || !ys[i]) return DIROTQ_ERR_NULL;
    if (misaligned(blobs[i]) || misaligned(ys[i]) || (biases && misaligned(biases[i]))) return DIROTQ_ERR_ALIGN;
  }
  const WorkspaceLayout L = workspace_layout(M, K, r, g);
  if (workspace_bytes < L.bytes) return DIROTQ_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  uint16_t* xh = (uint16_t*)(ws + L.off_xh);
  uint8_t* xl = (uint8_t*)(ws + L.off_xl);
  uint16_t* sx = (uint16_t*)(ws + L.off_sx);
  RqOut o;
  o.xh = xh, o.xl = xl, o.sx = sx;
  int st = launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
  for (int i = 0; i < n_out && !st; i++)
    st = launch_w4a4_gemm(xh, xl, sx, nullptr, blobs[i], biases ? biases[i] : nullptr, M, Ns[i], K, r, g, ys[i], 0,
                          (hipStream_t)stream);
  return st;
}

int dirotq_rotate_quantize_asym(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r, int g,
                                uint16_t* xh_bf16, uint8_t* xl_packed, uint16_t* sx_fp16, uint16_t* zx_fp16,
                                void* stream) {
  int st = check_shape(M, 1, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!xl_packed || !sx_fp16 || !zx_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(xh_bf16) || misaligned(xl_packed) ||
      misaligned(sx_fp16) || misaligned(zx_fp16))
    return DIROTQ_ERR_ALIGN;
  RqOut o;
  o.xh = xh_bf16;
  if (r < K) o.xl = xl_packed, o.sx = sx_fp16, o.zx = zx_fp16;   // (no 4-bit part: nothing to quantize)
  return launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
}

int dirotq_w4a4_gemm_asym(const uint16_t* xh_bf16, const uint8_t* xl_packed, const uint16_t* sx_fp16,
                          const uint16_t* zx_fp16, const void* blob, const uint16_t* bias_bf16, int M, int N,
                          int K, int r, int g, void* y, int y_dtype, void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (y_dtype != 0 && y_dtype != 1) return DIROTQ_ERR_UNSUPPORTED;
  if (M == 0) return DIROTQ_OK;
  if (!blob || !y) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!xl_packed || !sx_fp16 || !zx_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(xh_bf16) || misaligned(xl_packed) || misaligned(sx_fp16) || misaligned(zx_fp16) ||
      misaligned(blob) || misaligned(bias_bf16) || misaligned(y))
    return DIROTQ_ERR_ALIGN;
  return launch_w4a4_gemm(xh_bf16, xl_packed, sx_fp16, r < K ? zx_fp16 : nullptr, blob, bias_bf16, M, N, K, r, g, y,
                          y_dtype, (hipStream_t)stream);
}

int dirotq_linear_asym(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob,
                       const uint16_t* bias_bf16, int M, int N, int K, int r, int g, uint16_t* y_bf16,
                       void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16 || !blob || !y_bf16 || !workspace) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(blob) || misaligned(bias_bf16) ||
      misaligned(y_bf16) || ((uintptr_t)workspace & (kAlign - 1)) != 0)
    return DIROTQ_ERR_ALIGN;
  const WorkspaceLayout L = workspace_layout(M, K, r, g);
  if (workspace_bytes < L.bytes) return DIROTQ_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  uint16_t* xh = (uint16_t*)(ws + L.off_xh);
  uint8_t* xl = (uint8_t*)(ws + L.off_xl);
  uint16_t* sx = (uint16_t*)(ws + L.off_sx);
  uint16_t* zx = r < K ? (uint16_t*)(ws + L.off_zx) : nullptr;
  RqOut o;
  o.xh = xh, o.xl = xl, o.sx = sx, o.zx = zx;
  st = launch_rotate_quantize(x_bf16, Qt_bf16, M, K, r, g, o, (hipStream_t)stream);
  if (st) return st;
  return launch_w4a4_gemm(xh, xl, sx, zx, blob, bias_bf16, M, N, K, r, g, y_bf16, 0, (hipStream_t)stream);
}

int dirotq_a8_scratch_bytes(int M, int K, int r, size_t* bytes) {
  if (!bytes) return DIROTQ_ERR_NULL;
  int st = check_shape(M, 1, K, r, 32);
  if (st) return st;
  const WorkspaceA8Layout L = workspace_a8_layout(M, K, r);
  *bytes = L.bytes - L.off_xf;
  return DIROTQ_OK;
}

int dirotq_a8_workspace_bytes(int M, int K, int r, size_t* bytes) {
  if (!bytes) return DIROTQ_ERR_NULL;
  int st = check_shape(M, 1, K, r, 32);
  if (st) return st;
  *bytes = workspace_a8_layout(M, K, r).bytes;
  return DIROTQ_OK;
}

// rotation with fp32 output into the scratch, then the per-token quantizer
static int rotate_quantize_a8(const uint16_t* x, const uint16_t* Qt, int M, int K, int r, uint16_t* xh, uint8_t* x8,
                              uint16_t* sx, char* scratch, hipStream_t s) {
  const WorkspaceA8Layout L = workspace_a8_layout(M, K, r);
  RqOut o;
  o.xh = xh;
  if (r < K) o.xf = (float*)scratch, o.pmax = (float*)(scratch + (L.off_pmax - L.off_xf));
  int st = launch_rotate_quantize(x, Qt, M, K, r, 32, o, s);
  if (st || r == K) return st;
  return launch_quantize_tokens(o.xf, o.pmax, M, K - r, x8, sx, s);
}

int dirotq_rotate_quantize_a8(const uint16_t* x_bf16, const uint16_t* Qt_bf16, int M, int K, int r,
                              uint16_t* xh_bf16, uint8_t* x8, uint16_t* sx_fp16, void* scratch,
                              size_t scratch_bytes, void* stream) {
  int st = check_shape(M, 1, K, r, 32);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!x8 || !sx_fp16 || !scratch)) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(xh_bf16) || misaligned(x8) || misaligned(sx_fp16) ||
      ((uintptr_t)scratch & (kAlign - 1)) != 0)
    return DIROTQ_ERR_ALIGN;
  const WorkspaceA8Layout L = workspace_a8_layout(M, K, r);
  if (r < K && scratch_bytes < L.bytes - L.off_xf) return DIROTQ_ERR_WORKSPACE;
  return rotate_quantize_a8(x_bf16, Qt_bf16, M, K, r, xh_bf16, x8, sx_fp16, (char*)scratch, (hipStream_t)stream);
}

int dirotq_w4a8_gemm(const uint16_t* xh_bf16, const uint8_t* x8, const uint16_t* sx_fp16, const void* blob,
                     const uint16_t* bias_bf16, int M, int N, int K, int r, int g, void* y, int y_dtype,
                     void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (y_dtype != 0 && y_dtype != 1) return DIROTQ_ERR_UNSUPPORTED;
  if (M == 0) return DIROTQ_OK;
  if (!blob || !y) return DIROTQ_ERR_NULL;
  if (r > 0 && !xh_bf16) return DIROTQ_ERR_NULL;
  if (r < K && (!x8 || !sx_fp16)) return DIROTQ_ERR_NULL;
  if (misaligned(xh_bf16) || misaligned(x8) || misaligned(sx_fp16) || misaligned(blob) || misaligned(bias_bf16) ||
      misaligned(y))
    return DIROTQ_ERR_ALIGN;
  return launch_w4a8_gemm(xh_bf16, x8, sx_fp16, blob, bias_bf16, M, N, K, r, g, y, y_dtype, (hipStream_t)stream);
}

int dirotq_linear_a8(const uint16_t* x_bf16, const uint16_t* Qt_bf16, const void* blob, const uint16_t* bias_bf16,
                     int M, int N, int K, int r, int g, uint16_t* y_bf16, void* workspace, size_t workspace_bytes,
                     void* stream) {
  int st = check_shape(M, N, K, r, g);
  if (st) return st;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !Qt_bf16 || !blob || !y_bf16 || !workspace) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(Qt_bf16) || misaligned(blob) || misaligned(bias_bf16) ||
      misaligned(y_bf16) || ((uintptr_t)workspace & (kAlign - 1)) != 0)
    return DIROTQ_ERR_ALIGN;
  const WorkspaceA8Layout L = workspace_a8_layout(M, K, r);
  if (workspace_bytes < L.bytes) return DIROTQ_ERR_WORKSPACE;
  char* ws = (char*)workspace;
  uint16_t* xh = (uint16_t*)(ws + L.off_xh);
  uint8_t* x8 = (uint8_t*)(ws + L.off_x8);
  uint16_t* sx = (uint16_t*)(ws + L.off_sx);
  st = rotate_quantize_a8(x_bf16, Qt_bf16, M, K, r, xh, x8, sx, ws + L.off_xf, (hipStream_t)stream);
  if (st) return st;
  return launch_w4a8_gemm(xh, x8, sx, blob, bias_bf16, M, N, K, r, g, y_bf16, 0, (hipStream_t)stream);
}

int dirotq_w4a16_gemm(const uint16_t* x_bf16, const void* blob, const uint16_t* bias_bf16, int M, int N, int K,
                      int g, void* y, int y_dtype, void* stream) {
  int st = check_shape(M, N, K, 0, g);
  if (st) return st;
  if (y_dtype != 0 && y_dtype != 1) return DIROTQ_ERR_UNSUPPORTED;
  if (M == 0) return DIROTQ_OK;
  if (!x_bf16 || !blob || !y) return DIROTQ_ERR_NULL;
  if (misaligned(x_bf16) || misaligned(blob) || misaligned(bias_bf16) || misaligned(y)) return DIROTQ_ERR_ALIGN;
  return launch_w4a16_gemm(x_bf16, blob, bias_bf16, M, N, K, g, y, y_dtype, (hipStream_t)stream);
}

}  // extern "C"
