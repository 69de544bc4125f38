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
  // element (b,h,n,c) of every tensor is at b*stride_batch + h*stride_head + n*stride_row + c
  // (in elements): [B,H,N,d] or [B,N,H,d]
  long long stride_batch, stride_head, stride_row;
  int dtype;            // 0 = f32, 1 = bf16, 2 = f16
  long long elem_bytes() const { return dtype == 0 ? 4 : 2; }
  float scale, eps;
  const float* slice_scale;  // [B*H] or nullptr: per-slice scale instead of `scale`
  float* dlog_scale;         // backward only, [B*H] or nullptr: receives <S, dS> per slice
  int feature_map;           // 0: row-wise L2 normalisation of Q and K, 1: ELU(x) + 1 element-wise
  float* saved_state;        // [B*H][D][D] or nullptr: S of every slice, written by the forward,
                             // read by the backward (which then does not rebuild it)
  float* workspace;     // partial and reduced states, see Plan
  hipStream_t stream;
};

// How a call is cut into workgroups.
//   path        : kResident one 16-wave workgroup keeps a short slice in LDS (no workspace)
//                 kFused   one workgroup per slice runs every phase in one launch (no workspace)
//                 kSplit   MFMA kernels, `splits` workgroups per slice, states via the workspace
//                 kGeneric kernels for wide rows (256 or 512 bytes): one launch per direction,
//                          or partial states, reduction and apply via the workspace
//   splits      : workgroups per slice in the state-reduction kernel; each reduces
//                 `rows_per_split` consecutive rows to one partial d x d state
//   workspace   : floats.  kGeneric: partial states [nstates][B*H*splits][D*D], followed, when
//                 splits > 1, by the reduced states [nstates][B*H][D*D].  kSplit: partial
//                 states [nstates][B*H][splits][D*D]; every consumer workgroup sums the
//                 partials of its slice itself, in split order
struct Plan {
  enum Path { kGeneric = 0, kFused = 1, kSplit = 2, kResident = 3 };
  Path path;
  int splits;
  int rows_per_split;
  size_t workspace_floats;
};

// allow_resident = false keeps short 16-bit sequences off the kernels that hold a slice in LDS
// (they implement the cosine map only); the workspace requirement is the same either way.
Plan make_plan(int B, int H, int N, int D, int dtype, bool is_bwd, bool allow_resident = true);

// Grants `kernel` `bytes` of dynamic LDS (kernels that use more than 64 KB must be granted it
// before their first launch).  The attribute is set once per kernel and device: later calls
// with the same kernel on the same device return at once, without a runtime call.  A kernel
// is always granted the same size.
hipError_t grant_dynamic_lds(const void* kernel, int bytes);

// reduced[s][e] = partial[s][0][e] + partial[s][1][e] + ... in split order, for `slices`
// slices of dd floats each.
void launch_reduce_states(const float* partial, float* reduced, int splits, int dd, size_t slices,
                          hipStream_t stream);

// Wide rows (Plan::kGeneric): everything the kernels for rows of up to 128 bytes do not serve.
hipError_t launch_generic_fwd(const Problem& p, const Plan& plan);
hipError_t launch_generic_bwd(const Problem& p, const Plan& plan);

// Matrix-core kernels for 256-byte rows (fp32 d_h = 64, 16-bit d_h = 128) and 512-byte rows (fp32
// d_h = 128): partial states into p.workspace, then, from the reduced states ([B*H][D*D] floats
// each), O or dQ, dK, dV.
bool wide_supports(int dtype, int D);
hipError_t launch_wide_states(const Problem& p, const Plan& plan, bool bwd);
hipError_t launch_wide_apply(const Problem& p, const Plan& plan, const float* states,
                             const float* dstates, bool bwd);
// Sequences that are not cut (wide_fused_applies): one launch per direction, the state stays in
// LDS, no workspace; the forward writes p.saved_state, the backward p.dlog_scale, when given.
bool wide_fused_applies(int dtype, int D, int B, int H, int splits, bool bwd);
hipError_t launch_wide_fused(const Problem& p, const Plan& plan, bool bwd);

// MFMA path: bf16 or fp16 I/O with d_h = 64 and fp32 I/O with d_h = 32 (128-byte rows), and
// the half-width shapes (16-bit d_h = 32, fp32 d_h = 16) zero-padded onto the same kernels.
bool mfma_supports(int dtype, int D);
int mfma_state_dim(int dtype);  // side of the (possibly zero-padded) state the MFMA kernels keep
hipError_t launch_mfma_fwd(const Problem& p, const Plan& plan);
hipError_t launch_mfma_bwd(const Problem& p, const Plan& plan);

// Resident kernels: short bf16 / fp16 sequences (a slice fits the LDS of one compute unit).  With
// fp32 rows the matrix cores, 16 times slower there, bound each of their phases and the
// tile-streaming kernels are faster, so those keep all fp32 shapes.
bool resident_supports(int dtype, int D, int N);
hipError_t launch_resident_fwd(const Problem& p);
hipError_t launch_resident_bwd(const Problem& p);
// The causal variant on the matrix cores, tile pair by tile pair with up to 208 rows in LDS: every
// element type, 128-byte rows or narrower.  Longer sequences are cut into chunks of 208 rows,
// one workgroup each; what a chunk gets from the chunks before it (and, in the backward, gives
// to the chunks after it) travels as d x d states through the workspace:
//   launch_chunk_states    state of every chunk on its own, [S_c of all slices][T_c of all slices]
//                          (T_c = sum of qhat^T dO over the chunk, backward only), each
//                          [slice][chunk][D*D] floats with D = mfma_state_dim(dtype)
//   launch_chunk_scan      in place: S_c <- sum of the S before chunk c, T_c <- sum of the T after it
//   launch_resident_causal the chunk kernels, reading those sums (chunks == 1: no workspace)
bool causal_resident_supports(int dtype, int D);
constexpr int kCausalChunkRows = 208;
inline int causal_chunks(int N) { return (N + kCausalChunkRows - 1) / kCausalChunkRows; }
hipError_t launch_chunk_states(const Problem& p, int chunk_tiles, int chunks, bool with_queries);
hipError_t launch_chunk_scan(float* states, int slices, int chunks, int dd, bool with_queries,
                             hipStream_t stream);
hipError_t launch_resident_causal(const Problem& p, bool bwd, int chunks);

// Learnable normaliser: slice_scale[b*H+h] = n_b^(-m_h), and dm[h] = -sum_b ln(n_b) dlog[b*H+h].
// n may be nullptr (n_b = N).
hipError_t launch_normaliser_fwd(const float* m, const int32_t* n, float* slice_scale, int B,
                                 int H, int N, hipStream_t stream);
hipError_t launch_normaliser_bwd(const float* dlog, const int32_t* n, float* dm, int B, int H,
                                 int N, hipStream_t stream);

// Causal variant (row i attends keys j <= i), d_h in {16, 32, 64}: the matrix-core kernels above
// where the rows are 128 bytes or narrower, vector-ALU scan kernels otherwise (fp32 d_h = 64).
// causal_workspace_floats: what p.workspace must hold for the call (0: none needed).
bool causal_supports(int D);
size_t causal_workspace_floats(int B, int H, int N, int D, int dtype, bool is_bwd);
hipError_t launch_causal(const Problem& p, bool bwd);

}  // namespace cotten
