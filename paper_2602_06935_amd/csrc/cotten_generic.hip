// What the kernel families share on the host and around the states: the launch plan, the
// three-launch structure of the kernels for wide rows (partial states -> fixed-order reduction ->
// apply), the reduction kernel itself, <S, dS> for d loss / d log(scale), and the kernels of
// the learnable normaliser.
#include "cotten_device.h"
#include "cotten_launch.h"

namespace cotten {
namespace {

constexpr int kThreads = 256;

// Sums the partial states of every slice in split order (fixed order => results do
// not depend on scheduling).  One thread per state element.
__global__ __launch_bounds__(kThreads) void reduce_states_kernel(
    const float* __restrict__ partial, float* __restrict__ reduced, int splits, int dd,
    size_t total) {
  const size_t e = static_cast<size_t>(blockIdx.x) * kThreads + threadIdx.x;
  if (e >= total) return;
  const size_t bh = e / dd, k = e % dd;
  const float* __restrict__ src = partial + bh * splits * dd + k;
  float s = 0.0f;
  for (int p = 0; p < splits; ++p) s += src[static_cast<size_t>(p) * dd];
  reduced[e] = s;
}

// dlog[bh] = scale_bh * <S_bh, dS'_bh> with dS' = sum_i qhat_i^T dO_i (the states in the
// workspace carry no scale), i.e. <S, dS> = sum_i dO_i . O_i.  One workgroup per slice; the
// sum runs in a fixed order (strided per thread, then a tree over the threads).
__global__ __launch_bounds__(kThreads) void state_inner_product_kernel(
    const float* __restrict__ states, const float* __restrict__ dstates, int dd, float scale,
    const float* __restrict__ slice_scale, float* __restrict__ dlog) {
  __shared__ float part[kThreads];
  const size_t off = static_cast<size_t>(blockIdx.x) * dd;
  float s = 0.0f;
  for (int e = threadIdx.x; e < dd; e += kThreads) s += states[off + e] * dstates[off + e];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0)
    dlog[blockIdx.x] = part[0] * (slice_scale != nullptr ? slice_scale[blockIdx.x] : scale);
}

// slice_scale[b*H+h] = n_b^(-m_h) = exp2(-m_h log2 n_b)
__global__ __launch_bounds__(kThreads) void normaliser_fwd_kernel(
    const float* __restrict__ m, const int32_t* __restrict__ n, float* __restrict__ slice_scale,
    int B, int H, int N) {
  const int e = blockIdx.x * kThreads + threadIdx.x;
  if (e >= B * H) return;
  const float nb = static_cast<float>(n != nullptr ? n[e / H] : N);
  slice_scale[e] = exp2f(-m[e % H] * log2f(nb));
}

// dm[h] = -sum_b ln(n_b) dlog[b*H+h]: one workgroup per head, fixed order (strided per
// thread, then a tree over the threads).
__global__ __launch_bounds__(kThreads) void normaliser_bwd_kernel(
    const float* __restrict__ dlog, const int32_t* __restrict__ n, float* __restrict__ dm, int B,
    int H, int N) {
  __shared__ float part[kThreads];
  const int h = blockIdx.x;
  float s = 0.0f;
  for (int b = threadIdx.x; b < B; b += kThreads)
    s += logf(static_cast<float>(n != nullptr ? n[b] : N)) * dlog[static_cast<size_t>(b) * H + h];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) part[threadIdx.x] += part[threadIdx.x + w];
    __syncthreads();
  }
  if (threadIdx.x == 0) dm[h] = -part[0];
}

// Where the reduced states live: behind the partials when a reduction
// is needed, otherwise the single partial of each slice already is the state.
const float* reduce_generic(const Problem& p, const Plan& plan, int nstates) {
  if (plan.splits == 1) return p.workspace;
  const size_t BH = static_cast<size_t>(p.B) * p.H;
  const int dd = p.D * p.D;
  float* reduced = p.workspace + BH * plan.splits * dd * nstates;
  // S and dS partials are contiguous [nstates][BH*splits][dd]: one launch covers both
  launch_reduce_states(p.workspace, reduced, plan.splits, dd, BH * nstates, p.stream);
  return reduced;
}

// The three-launch structure of the matrix-core kernels for wide rows (cotten_wide.hip): partial
// states, their reduction, the kept state, the apply kernels, <S, dS>; one launch per direction
// where the sequence is not cut.
hipError_t run_wide(const Problem& p, const Plan& plan, bool bwd) {
  if (wide_fused_applies(p.dtype, p.D, p.B, p.H, plan.splits, bwd)) return launch_wide_fused(p, plan, bwd);
  const int BH = p.B * p.H;
  const int dd = p.D * p.D;
  if (hipError_t err = launch_wide_states(p, plan, bwd)) return err;
  const float* states = reduce_generic(p, plan, bwd ? 2 : 1);
  const size_t second = static_cast<size_t>(BH) * plan.splits * dd;
  const float* dstates =
      bwd ? states + (plan.splits == 1 ? second : static_cast<size_t>(BH) * dd) : nullptr;
  if (!bwd && p.saved_state != nullptr)
    launch_reduce_states(states, p.saved_state, 1, dd, static_cast<size_t>(BH), p.stream);
  if (hipError_t err = launch_wide_apply(p, plan, states, dstates, bwd)) return err;
  if (bwd && p.dlog_scale != nullptr)
    hipLaunchKernelGGL(state_inner_product_kernel, dim3(static_cast<unsigned>(BH)),
                       dim3(kThreads), 0, p.stream, states, dstates, dd, p.scale, p.slice_scale,
                       p.dlog_scale);
  return hipGetLastError();
}

}  // namespace

void launch_reduce_states(const float* partial, float* reduced, int splits, int dd, size_t slices,
                          hipStream_t stream) {
  const size_t total = slices * dd;
  const dim3 grid(static_cast<unsigned>((total + kThreads - 1) / kThreads), 1, 1);
  hipLaunchKernelGGL(reduce_states_kernel, grid, dim3(kThreads), 0, stream, partial, reduced,
                     splits, dd, total);
}

Plan make_plan(int B, int H, int N, int D, int dtype, bool is_bwd, bool allow_resident) {
  const long BH = static_cast<long>(B) * H;
  const size_t nstates = is_bwd ? 2 : 1;
  Plan plan;
  long splits, rows;
  if (mfma_supports(dtype, D)) {
    // One workgroup per slice while that fills the chip or the slice is short; otherwise
    // cut the sequence so that about 512 workgroups exist, two per compute unit (measured at
    // N = 4096 with 64 slices: 256 workgroups 0.67 G tokens/s, 512: 0.71 G, 768 and 1024: 0.58 G
    // - a second workgroup covers the fixed work of the first, more only add fixed work), in
    // blocks of 64 rows.
    constexpr long kFusedMaxN = 2048, kBlock = 64;
    // 16-bit sequences that fit LDS go to the resident kernels - except the forward of the
    // longer ones when there are many slices, where the fused kernel that keeps its tiles in
    // registers is faster (N = 208, 512 slices: 9.6 against 10.2 us; the resident kernel wins
    // at N = 100, 7.1 against 7.6 us, and with 64 slices, 5.7 against 7.2 us).
    const bool fused_fwd_instead = !is_bwd && N > 160 && BH >= 256;
    if (allow_resident && resident_supports(dtype, D, N) && !fused_fwd_instead) {
      plan.path = Plan::kResident;
      plan.splits = 1;
      plan.rows_per_split = N;
      plan.workspace_floats = 0;
      return plan;
    }
    // Long sequences stay on one workgroup per slice as well when there are slices enough
    // (measured at N = 3000 ... 4096: the backward from 256 slices on, the forward from 512).
    constexpr long kFusedLongMaxN = 16384;  // key flags of the slice must fit LDS
    const bool fused_long = N <= kFusedLongMaxN && BH >= (is_bwd ? 256 : 512);
    if ((N <= kFusedMaxN && (BH >= 256 || N <= 256)) || fused_long) {
      plan.path = Plan::kFused;
      plan.splits = 1;
      plan.rows_per_split = N;
      plan.workspace_floats = 0;
      return plan;
    }
    plan.path = Plan::kSplit;
    splits = (512 + BH - 1) / BH;
    const long by_len = (N + kFusedMaxN - 1) / kFusedMaxN;
    if (splits < by_len) splits = by_len;
    const long max_splits = (N + kBlock - 1) / kBlock;
    if (splits > max_splits) splits = max_splits;
    rows = (N + splits - 1) / splits;
    rows = (rows + kBlock - 1) / kBlock * kBlock;
  } else {
    // Wide rows (256 or 512 bytes).  Their kernels build operand images per workgroup and stage
    // 64 rows per round: about two workgroups per compute unit, in blocks of 64 rows.
    // A d x d state is as large as 64 ... 256 rows of a tensor there, and every split writes one
    // and has the sum read back: no fewer than 256 rows per workgroup, and a sequence is not cut
    // at all once there is a workgroup per compute unit without it.
    plan.path = Plan::kGeneric;
    constexpr long kTarget = 512, kBlock = 64;
    splits = BH >= 256 ? 1 : (kTarget + BH - 1) / BH;
    const long max_splits = (N + 255) / 256;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    rows = (N + splits - 1) / splits;
    rows = (rows + kBlock - 1) / kBlock * kBlock;
  }
  splits = (N + rows - 1) / rows;
  plan.splits = static_cast<int>(splits);
  plan.rows_per_split = static_cast<int>(rows);
  if (plan.path == Plan::kSplit) {
    const size_t side = mfma_state_dim(dtype);
    plan.workspace_floats = static_cast<size_t>(BH) * side * side * splits * nstates;
  } else {
    // partial states, plus the reduced states when there is more than one partial
    // (one launch per direction: the state never leaves the compute unit)
    plan.workspace_floats =
        wide_fused_applies(dtype, D, B, H, static_cast<int>(splits), is_bwd)
            ? 0
            : static_cast<size_t>(BH) * D * D * nstates * (splits + (splits > 1 ? 1 : 0));
  }
  return plan;
}

hipError_t launch_generic_fwd(const Problem& p, const Plan& plan) {
  return wide_supports(p.dtype, p.D) ? run_wide(p, plan, false) : hipErrorInvalidValue;
}

hipError_t launch_generic_bwd(const Problem& p, const Plan& plan) {
  return wide_supports(p.dtype, p.D) ? run_wide(p, plan, true) : hipErrorInvalidValue;
}

hipError_t launch_normaliser_fwd(const float* m, const int32_t* n, float* slice_scale, int B,
                                 int H, int N, hipStream_t stream) {
  const unsigned blocks = static_cast<unsigned>((static_cast<long>(B) * H + kThreads - 1) / kThreads);
  hipLaunchKernelGGL(normaliser_fwd_kernel, dim3(blocks), dim3(kThreads), 0, stream, m, n,
                     slice_scale, B, H, N);
  return hipGetLastError();
}

hipError_t launch_normaliser_bwd(const float* dlog, const int32_t* n, float* dm, int B, int H,
                                 int N, hipStream_t stream) {
  hipLaunchKernelGGL(normaliser_bwd_kernel, dim3(static_cast<unsigned>(H)), dim3(kThreads), 0,
                     stream, dlog, n, dm, B, H, N);
  return hipGetLastError();
}

}  // namespace cotten
