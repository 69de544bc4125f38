// C-ABI entry points: host-side validation, defaults, workspace, dispatch.
// See include/cotten_attn.h for the contract of every function.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <mutex>

#include "../../include/cotten_attn.h"
#include "cotten_launch.h"

namespace {

constexpr float kDefaultEps = 1e-6f;

bool head_dim_ok(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Shape checks shared by both directions.  Pure host arithmetic.
int check_shape(int B, int H, int N, int d_h, int dtype) {
  if (dtype != COTTEN_F32 && dtype != COTTEN_BF16 && dtype != COTTEN_F16)
    return COTTEN_ERR_BAD_DTYPE;
  if (B < 1 || H < 1 || N < 1) return COTTEN_ERR_BAD_SHAPE;
  if (!head_dim_ok(d_h)) return COTTEN_ERR_UNSUPPORTED_HEAD_DIM;
  const long long slices = static_cast<long long>(B) * H;
  if (slices > (1ll << 24)) return COTTEN_ERR_BAD_SHAPE;         // grid.x = slices * splits
  if (N > (1 << 24)) return COTTEN_ERR_BAD_SHAPE;
  return COTTEN_OK;
}

// Kernels whose dynamic-LDS attribute has been set, and on which devices (bit d = device d).
// Entries are appended under the mutex and never change place, so readers need no lock.
struct Granted {
  std::atomic<const void*> kernel{nullptr};
  std::atomic<uint64_t> devices{0};
};
constexpr int kMaxGranted = 256;
Granted g_granted[kMaxGranted];
std::atomic<int> g_granted_count{0};
std::mutex g_grant_mutex;

// Scratch of cotten_attn_bwd_static: the partial states of the split path, for callers that
// cannot bring a workspace.  One copy per GPU the library runs on, held until the process ends.
// In host code the array's name is only a handle: the device address comes from
// hipGetSymbolAddress, once per device, and that pointer is what kernels are given.
static __device__ __align__(256) unsigned char scratch[COTTEN_STATIC_SCRATCH_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (nullptr on failure).
void* static_scratch() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p != nullptr) return p;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
  if (p != nullptr) return p;
  void* addr = nullptr;
  if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || addr == nullptr) {
    (void)hipGetLastError();
    return nullptr;
  }
  g_scratch_ptr[dev].store(addr, std::memory_order_release);
  return addr;
}

int resolve(const cotten_params* prm, int N, float* scale, float* eps) {
  *scale = prm->scale > 0.0f ? prm->scale : 1.0f / static_cast<float>(N);
  *eps = prm->eps < 0.0f ? kDefaultEps : prm->eps;
  if (!std::isfinite(prm->scale) || !std::isfinite(prm->eps)) return COTTEN_ERR_BAD_PARAM;
  return COTTEN_OK;
}

int run(bool bwd, const void* Q, const void* K, const void* V, const uint8_t* mask,
        const void* dO, void* O, void* dQ, void* dK, void* dV, int B, int H, int N, int d_h,
        void* stream, const cotten_params* prm, bool use_static_scratch = false) {
  if (prm == nullptr) return COTTEN_ERR_NULL_POINTER;
  if (Q == nullptr || K == nullptr || V == nullptr) return COTTEN_ERR_NULL_POINTER;
  if (bwd ? (dO == nullptr || dQ == nullptr || dK == nullptr || dV == nullptr) : (O == nullptr))
    return COTTEN_ERR_NULL_POINTER;
  if (int rc = check_shape(B, H, N, d_h, prm->dtype)) return rc;
  const void* tensors[9] = {Q, K, V, bwd ? dO : O, dQ, dK, dV,
                            use_static_scratch ? nullptr : prm->workspace, prm->saved_state};
  for (const void* t : tensors)
    if (t != nullptr && !aligned16(t)) return COTTEN_ERR_MISALIGNED;

  cotten::Problem p{};
  if (int rc = resolve(prm, N, &p.scale, &p.eps)) return rc;
  if (prm->layout != COTTEN_BHND && prm->layout != COTTEN_BNHD) return COTTEN_ERR_BAD_SHAPE;
  if (prm->layout == COTTEN_BHND) {
    p.stride_batch = static_cast<long long>(H) * N * d_h;
    p.stride_head = static_cast<long long>(N) * d_h;
    p.stride_row = d_h;
  } else {
    p.stride_batch = static_cast<long long>(N) * H * d_h;
    p.stride_head = d_h;
    p.stride_row = static_cast<long long>(H) * d_h;
  }
  // the kernels address the rows of a slice with 31-bit byte offsets
  if ((static_cast<long long>(N - 1) * p.stride_row + d_h) * (prm->dtype == COTTEN_F32 ? 4 : 2) >=
      (1ll << 31))
    return COTTEN_ERR_BAD_SHAPE;
  if (prm->feature_map != COTTEN_MAP_COSINE && prm->feature_map != COTTEN_MAP_ELU1)
    return COTTEN_ERR_BAD_PARAM;
  if (prm->feature_map == COTTEN_MAP_ELU1) {
    if (prm->causal != 0) return COTTEN_ERR_BAD_PARAM;
    if (!cotten::mfma_supports(prm->dtype, d_h) && !cotten::wide_supports(prm->dtype, d_h))
      return COTTEN_ERR_UNSUPPORTED_HEAD_DIM;
  }
  p.feature_map = prm->feature_map;
  const bool causal = prm->causal != 0;
  if (causal) {
    if (prm->causal != 1 || (bwd && prm->dlog_scale != nullptr)) return COTTEN_ERR_BAD_PARAM;
    if (!cotten::causal_supports(d_h)) return COTTEN_ERR_UNSUPPORTED_HEAD_DIM;
  }
  cotten::Plan plan{};
  if (!causal)
    plan = cotten::make_plan(B, H, N, d_h, prm->dtype, bwd, prm->feature_map == COTTEN_MAP_COSINE);
  const size_t need = sizeof(float) * (causal ? cotten::causal_workspace_floats(B, H, N, d_h, prm->dtype, bwd)
                                              : plan.workspace_floats);
  if (use_static_scratch) {
    if (need > COTTEN_STATIC_SCRATCH_BYTES) return COTTEN_ERR_STATIC_SCRATCH;
    if (need > 0) {
      p.workspace = static_cast<float*>(static_scratch());
      if (p.workspace == nullptr) return COTTEN_ERR_STATIC_SCRATCH;
    }
  } else if (prm->workspace != nullptr) {
    if (prm->workspace_bytes < need) return COTTEN_ERR_WORKSPACE_TOO_SMALL;
    p.workspace = static_cast<float*>(prm->workspace);
  } else if (need > 0) {
    return COTTEN_ERR_WORKSPACE_TOO_SMALL;  // the library allocates nothing: the caller brings it
  }
  p.slice_scale = prm->slice_scale;
  p.dlog_scale = bwd ? prm->dlog_scale : nullptr;
  p.saved_state = prm->saved_state;
  p.Q = Q; p.K = K; p.V = V; p.mask = mask; p.dO = dO;
  p.O = O; p.dQ = dQ; p.dK = dK; p.dV = dV;
  p.B = B; p.H = H; p.N = N; p.D = d_h;
  p.dtype = prm->dtype;
  p.stream = static_cast<hipStream_t>(stream);
  hipError_t err;
  if (causal)  // no kept state, no dlog_scale (refused above)
    err = cotten::launch_causal(p, bwd);
  else if (plan.path == cotten::Plan::kGeneric)
    err = bwd ? cotten::launch_generic_bwd(p, plan) : cotten::launch_generic_fwd(p, plan);
  else if (plan.path == cotten::Plan::kResident)
    err = bwd ? cotten::launch_resident_bwd(p) : cotten::launch_resident_fwd(p);
  else
    err = bwd ? cotten::launch_mfma_bwd(p, plan) : cotten::launch_mfma_fwd(p, plan);
  return err == hipSuccess ? COTTEN_OK : COTTEN_ERR_LAUNCH;
}

// dtype, scale, eps, workspace, workspace_bytes, slice_scale, dlog_scale, layout, causal,
// saved_state, feature_map
const cotten_params kDefaults = {COTTEN_F32, 0.0f,    -1.0f,       nullptr, 0,      nullptr,
                                 nullptr,    COTTEN_BHND, 0,       nullptr, COTTEN_MAP_COSINE};

}  // namespace

namespace cotten {

hipError_t grant_dynamic_lds(const void* kernel, int bytes) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return hipErrorInvalidDevice;
  const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t{1} << dev : 0;
  const int known = g_granted_count.load(std::memory_order_acquire);
  int slot = -1;
  for (int i = 0; i < known; ++i)
    if (g_granted[i].kernel.load(std::memory_order_relaxed) == kernel) {
      if (g_granted[i].devices.load(std::memory_order_acquire) & bit) return hipSuccess;
      slot = i;
      break;
    }
  std::lock_guard<std::mutex> lock(g_grant_mutex);
  const hipError_t err =
      hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
  if (err != hipSuccess) return err;
  if (slot < 0) {
    const int n = g_granted_count.load(std::memory_order_relaxed);
    for (int i = 0; i < n && slot < 0; ++i)
      if (g_granted[i].kernel.load(std::memory_order_relaxed) == kernel) slot = i;
    if (slot < 0 && n < kMaxGranted) {
      slot = n;
      g_granted[n].kernel.store(kernel, std::memory_order_relaxed);
      g_granted_count.store(n + 1, std::memory_order_release);
    }
  }
  // a full table only means the attribute is set again on the next call
  if (slot >= 0) g_granted[slot].devices.fetch_or(bit, std::memory_order_release);
  return hipSuccess;
}

}  // namespace cotten

extern "C" {

int cotten_attn_fwd_ex(const void* Q, const void* K, const void* V, const uint8_t* mask, void* O,
                       int B, int H, int N, int d_h, void* stream, const cotten_params* params) {
  return run(false, Q, K, V, mask, nullptr, O, nullptr, nullptr, nullptr, B, H, N, d_h, stream,
             params);
}

int cotten_attn_bwd_ex(const void* Q, const void* K, const void* V, const uint8_t* mask,
                       const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N, int d_h,
                       void* stream, const cotten_params* params) {
  return run(true, Q, K, V, mask, dO, nullptr, dQ, dK, dV, B, H, N, d_h, stream, params);
}

int cotten_attn_bwd_static(const void* Q, const void* K, const void* V, const uint8_t* mask,
                           const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N,
                           int d_h, void* stream, const cotten_params* params) {
  return run(true, Q, K, V, mask, dO, nullptr, dQ, dK, dV, B, H, N, d_h, stream, params, true);
}

int cotten_attn_fwd(const void* Q, const void* K, const void* V, const uint8_t* mask, void* O,
                    int B, int H, int N, int d_h, void* stream) {
  return cotten_attn_fwd_ex(Q, K, V, mask, O, B, H, N, d_h, stream, &kDefaults);
}

int cotten_attn_bwd(const void* Q, const void* K, const void* V, const uint8_t* mask,
                    const void* dO, void* dQ, void* dK, void* dV, int B, int H, int N, int d_h,
                    void* stream) {
  return cotten_attn_bwd_ex(Q, K, V, mask, dO, dQ, dK, dV, B, H, N, d_h, stream, &kDefaults);
}

int cotten_normaliser_fwd(const float* m, const int32_t* n, float* slice_scale, int B, int H,
                          int N, void* stream) {
  if (m == nullptr || slice_scale == nullptr) return COTTEN_ERR_NULL_POINTER;
  if (B < 1 || H < 1 || N < 1) return COTTEN_ERR_BAD_SHAPE;
  return cotten::launch_normaliser_fwd(m, n, slice_scale, B, H, N,
                                       static_cast<hipStream_t>(stream)) == hipSuccess
             ? COTTEN_OK
             : COTTEN_ERR_LAUNCH;
}

int cotten_normaliser_bwd(const float* dlog_scale, const int32_t* n, float* dm, int B, int H,
                          int N, void* stream) {
  if (dlog_scale == nullptr || dm == nullptr) return COTTEN_ERR_NULL_POINTER;
  if (B < 1 || H < 1 || N < 1) return COTTEN_ERR_BAD_SHAPE;
  return cotten::launch_normaliser_bwd(dlog_scale, n, dm, B, H, N,
                                       static_cast<hipStream_t>(stream)) == hipSuccess
             ? COTTEN_OK
             : COTTEN_ERR_LAUNCH;
}

size_t cotten_attn_workspace_bytes(int B, int H, int N, int d_h, int dtype, int is_bwd) {
  if (check_shape(B, H, N, d_h, dtype) != COTTEN_OK) return 0;
  return cotten::make_plan(B, H, N, d_h, dtype, is_bwd != 0).workspace_floats * sizeof(float);
}

size_t cotten_attn_workspace_bytes_ex(int B, int H, int N, int d_h, int is_bwd,
                                      const cotten_params* params) {
  if (params == nullptr || check_shape(B, H, N, d_h, params->dtype) != COTTEN_OK) return 0;
  if (params->causal != 0)
    return cotten::causal_supports(d_h)
               ? cotten::causal_workspace_floats(B, H, N, d_h, params->dtype, is_bwd != 0) * sizeof(float)
               : 0;
  return cotten_attn_workspace_bytes(B, H, N, d_h, params->dtype, is_bwd);
}

const char* cotten_status_string(int status) {
  switch (status) {
    case COTTEN_OK: return "ok";
    case COTTEN_ERR_NULL_POINTER: return "a required pointer is NULL";
    case COTTEN_ERR_BAD_SHAPE: return "B, H and N must be >= 1 and within launch limits";
    case COTTEN_ERR_UNSUPPORTED_HEAD_DIM: return "d_h must be 16, 32, 64 or 128";
    case COTTEN_ERR_BAD_DTYPE: return "dtype must be COTTEN_F32, COTTEN_BF16 or COTTEN_F16";
    case COTTEN_ERR_MISALIGNED: return "tensor and workspace pointers must be 16-byte aligned";
    case COTTEN_ERR_WORKSPACE_TOO_SMALL: return "workspace smaller than cotten_attn_workspace_bytes()";
    case COTTEN_ERR_BAD_PARAM: return "scale and eps must be finite; option combination not available";
    case COTTEN_ERR_LAUNCH: return "HIP kernel launch failed";
    case COTTEN_ERR_STATIC_SCRATCH:
      return "the call needs more scratch than COTTEN_STATIC_SCRATCH_BYTES (use cotten_attn_bwd_ex "
             "with a workspace), or the scratch array's address could not be obtained";
    default: return "unknown status";
  }
}

}  // extern "C"
