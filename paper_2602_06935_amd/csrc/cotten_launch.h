// Host-side launch plan shared by the C-ABI layer and the kernel files.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace cotten {

// Everything a launcher needs; pointers are device pointers, already validated.
struct Problem {
  const void* Q;
  const void* K;
  const void* V;
  const uint8_t* mask;  // [B,N] or nullptr
  const void* dO;       // backward only
  void* O;              // forward only
  void* dQ;
  void* dK;
  void* dV;
  int B, H, N, D;
  int dtype;            // 0 = f32, 1 = bf16
  float scale, eps;
  float* workspace;     // partial states, see Plan
  hipStream_t stream;
};

// How a call is cut into workgroups.
//   splits      : workgroups per slice in the state-reduction kernel; each reduces
//                 `rows_per_split` consecutive rows to one partial d x d state
//   workspace   : floats = B*H*splits*D*D (forward) or twice that (backward: S and dS)
struct Plan {
  int splits;
  int rows_per_split;
  size_t workspace_floats;
};

Plan make_plan(int B, int H, int N, int D, bool is_bwd);

// Two-kernel path (state reduction, then apply) for any supported shape.
hipError_t launch_generic_fwd(const Problem& p, const Plan& plan);
hipError_t launch_generic_bwd(const Problem& p, const Plan& plan);

}  // namespace cotten
