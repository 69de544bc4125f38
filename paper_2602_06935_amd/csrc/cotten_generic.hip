// Generic two-kernel path of the cosine attention: vector-ALU arithmetic, tiles
// staged through LDS.  Written for every supported (dtype, d_h, N); the matrix-core
// kernels take over the shapes they cover, which leaves fp32 d_h = 128 to these
// (and their launch structure, reduction and workspace layout to the kernels for
// 256-byte rows).
//
//   state kernel : one workgroup reduces a block of rows of one slice to a
//                  partial d x d state  sum_j xhat_j^T y_j   (x,y) = (K,V) under
//                  the key mask, and for the backward also (Q,dO) unmasked.
//   apply kernels: sum the partial states of the slice in a fixed order, then
//                  stream row tiles:  O = s Qhat S   /   dQ, dK, dV.
//
// Thread mapping inside a 32-row tile: 8 consecutive lanes own one row, each
// lane owns D/8 consecutive columns of it (one 128-bit access for fp32/d_h=32
// and bf16/d_h=64), so a row norm is an in-lane sum plus three lane exchanges.
#include "cotten_device.h"
#include "cotten_launch.h"

namespace cotten {
namespace {

constexpr int kThreads = 256;
constexpr int kTileRows = kThreads / 8;  // 32

// Element (b,h,n,c) of a tensor is at b*batch + h*head + n*row + c.
struct ElemStrides {
  long long batch, head, row;
  __device__ __forceinline__ size_t slice_base(int bh, int H) const {
    return static_cast<size_t>(bh / H) * batch + static_cast<size_t>(bh % H) * head;
  }
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void state_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const uint8_t* __restrict__ mask, float* __restrict__ ws,
    int H, int N, int splits, int rows_per_split, size_t second_offset, float eps,
    ElemStrides lay) {
  constexpr int CH = D / 8;   // columns per lane when loading
  constexpr int R = D / 16;   // each thread accumulates an R x R block of the state
  __shared__ float xs[kTileRows][D];
  __shared__ float ys[kTileRows][D];

  const int tid = threadIdx.x;
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const bool second = blockIdx.y == 1;  // (Q,dO) -> dS instead of (K,V) -> S
  const size_t base = lay.slice_base(bh, H);
  const T* __restrict__ X = (second ? Q : K) + base;
  const T* __restrict__ Y = (second ? dO : V) + base;
  const uint8_t* __restrict__ m =
      (second || mask == nullptr) ? nullptr : mask + static_cast<size_t>(bh / H) * N;

  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int lrow = tid >> 3, chunk = tid & 7;
  const int ty = tid >> 4, tx = tid & 15;

  float acc[R][R];
#pragma unroll
  for (int i = 0; i < R; ++i)
#pragma unroll
    for (int j = 0; j < R; ++j) acc[i][j] = 0.0f;

  for (int r0 = r_begin; r0 < r_end; r0 += kTileRows) {
    const int row = r0 + lrow;
    bool live = row < r_end;
    if (live && m != nullptr) live = m[row] != 0;
    float x[CH], y[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) x[i] = y[i] = 0.0f;
    if (live) {
      load_chunk<T, CH>(X + static_cast<size_t>(row) * lay.row + chunk * CH, x);
      load_chunk<T, CH>(Y + static_cast<size_t>(row) * lay.row + chunk * CH, y);
    }
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < CH; ++i) ss += x[i] * x[i];
    ss = sum8(ss);
    const float inv = inv_norm(ss, eps);
#pragma unroll
    for (int i = 0; i < CH; ++i) {
      xs[lrow][chunk * CH + i] = live ? x[i] * inv : 0.0f;
      ys[lrow][chunk * CH + i] = y[i];
    }
    __syncthreads();
#pragma unroll 4
    for (int r = 0; r < kTileRows; ++r) {
      float a[R], c[R];
#pragma unroll
      for (int i = 0; i < R; ++i) a[i] = xs[r][ty * R + i];
#pragma unroll
      for (int j = 0; j < R; ++j) c[j] = ys[r][tx * R + j];
#pragma unroll
      for (int i = 0; i < R; ++i)
#pragma unroll
        for (int j = 0; j < R; ++j) acc[i][j] += a[i] * c[j];
    }
    __syncthreads();
  }

  float* __restrict__ out =
      ws + (second ? second_offset : 0) + static_cast<size_t>(blockIdx.x) * D * D;
#pragma unroll
  for (int i = 0; i < R; ++i)
#pragma unroll
    for (int j = 0; j < R; ++j) out[(ty * R + i) * D + tx * R + j] = acc[i][j];
}

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

// Copies the reduced state of one slice into LDS, times `scale`, either as is
// (dst[a][c]) or transposed (dst[c][a]).
template <int D, bool TRANSPOSE>
__device__ __forceinline__ void load_state(const float* __restrict__ state, float scale,
                                           float (*dst)[D]) {
  for (int e = threadIdx.x; e < D * D; e += kThreads) {
    const float s = state[e] * scale;
    const int a = e / D, c = e % D;
    if (TRANSPOSE) dst[c][a] = s; else dst[a][c] = s;
  }
}

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void apply_fwd_kernel(
    const T* __restrict__ Q, const float* __restrict__ states, T* __restrict__ O, int H, int N,
    int splits, int rows_per_split, float scale, const float* __restrict__ slice_scale,
    float eps, ElemStrides lay) {
  constexpr int CH = D / 8;
  extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
  float (*S)[D] = reinterpret_cast<float (*)[D]>(dyn_lds);
  float (*qs)[D + 4] = reinterpret_cast<float (*)[D + 4]>(dyn_lds + D * D);

  const int tid = threadIdx.x;
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const size_t base = lay.slice_base(bh, H);
  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int lrow = tid >> 3, chunk = tid & 7;

  if (slice_scale != nullptr) scale = slice_scale[bh];
  load_state<D, false>(states + static_cast<size_t>(bh) * D * D, scale, S);
  __syncthreads();

  for (int r0 = r_begin; r0 < r_end; r0 += kTileRows) {
    const int row = r0 + lrow;
    const bool live = row < r_end;
    float q[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) q[i] = 0.0f;
    if (live) load_chunk<T, CH>(Q + base + static_cast<size_t>(row) * lay.row + chunk * CH, q);
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < CH; ++i) ss += q[i] * q[i];
    const float inv = inv_norm(sum8(ss), eps);
#pragma unroll
    for (int i = 0; i < CH; ++i) qs[lrow][chunk * CH + i] = q[i] * inv;
    __syncthreads();
    float o[CH];
#pragma unroll
    for (int i = 0; i < CH; ++i) o[i] = 0.0f;
#pragma unroll 8
    for (int a = 0; a < D; ++a) {
      const float qa = qs[lrow][a];
#pragma unroll
      for (int i = 0; i < CH; ++i) o[i] += qa * S[a][chunk * CH + i];
    }
    if (live) store_chunk<T, CH>(O + base + static_cast<size_t>(row) * lay.row + chunk * CH, o);
    __syncthreads();
  }
}

// LDS of the backward apply kernel, in floats: the state matrices a block needs, then the
// tile buffers.  d_h = 128 does not have room for dS and dS^T together, so there dV and dK
// are computed by separate blocks (grid.y = 3 instead of 2).
template <int D>
constexpr int bwd_apply_lds_floats() {
  return (D <= 64 ? 2 : 1) * D * D + 2 * kTileRows * (D + 4);
}
template <int D>
constexpr int bwd_apply_grid_y() {
  return D <= 64 ? 2 : 3;
}

// blockIdx.y == 0: dQ from (Q, dO, S).   Other blocks: dK and/or dV from (K, V, dS).
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void apply_bwd_kernel(
    const T* __restrict__ Q, const T* __restrict__ K, const T* __restrict__ V,
    const T* __restrict__ dO, const uint8_t* __restrict__ mask,
    const float* __restrict__ states, const float* __restrict__ dstates, T* __restrict__ dQ,
    T* __restrict__ dK, T* __restrict__ dV, int H, int N, int splits, int rows_per_split,
    float scale, const float* __restrict__ slice_scale, float eps, ElemStrides lay) {
  constexpr int CH = D / 8;
  constexpr bool kTogether = D <= 64;  // dV and dK in one block
  extern __shared__ __attribute__((aligned(16))) float dyn_lds[];
  float (*M0)[D] = reinterpret_cast<float (*)[D]>(dyn_lds);  // S^T (dQ), dS (dV) or dS^T (dK alone)
  float (*M1)[D] = reinterpret_cast<float (*)[D]>(dyn_lds + D * D);  // dS^T when together
  float* tiles = dyn_lds + (kTogether ? 2 : 1) * D * D;
  float (*t0)[D + 4] = reinterpret_cast<float (*)[D + 4]>(tiles);  // dO rows or khat rows
  float (*t1)[D + 4] = reinterpret_cast<float (*)[D + 4]>(tiles + kTileRows * (D + 4));  // v rows

  const int tid = threadIdx.x;
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const size_t base = lay.slice_base(bh, H);
  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int lrow = tid >> 3, chunk = tid & 7;
  const int c0 = chunk * CH;
  if (slice_scale != nullptr) scale = slice_scale[bh];

  if (blockIdx.y == 0) {
    load_state<D, true>(states + static_cast<size_t>(bh) * D * D, scale, M0);  // M0[c][a] = s S[a][c]
    __syncthreads();
    for (int r0 = r_begin; r0 < r_end; r0 += kTileRows) {
      const int row = r0 + lrow;
      const bool live = row < r_end;
      float q[CH], g[CH];
#pragma unroll
      for (int i = 0; i < CH; ++i) q[i] = g[i] = 0.0f;
      if (live) {
        load_chunk<T, CH>(Q + base + static_cast<size_t>(row) * lay.row + c0, q);
        load_chunk<T, CH>(dO + base + static_cast<size_t>(row) * lay.row + c0, g);
      }
      float ss = 0.0f;
#pragma unroll
      for (int i = 0; i < CH; ++i) ss += q[i] * q[i];
      const float inv = inv_norm(sum8(ss), eps);
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        q[i] *= inv;
        t0[lrow][c0 + i] = g[i];
        g[i] = 0.0f;
      }
      __syncthreads();
#pragma unroll 8
      for (int c = 0; c < D; ++c) {
        const float dc = t0[lrow][c];
#pragma unroll
        for (int i = 0; i < CH; ++i) g[i] += dc * M0[c][c0 + i];  // g_a = s sum_c dO_c S[a][c]
      }
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < CH; ++i) proj += q[i] * g[i];
      proj = sum8(proj);
#pragma unroll
      for (int i = 0; i < CH; ++i) g[i] = (g[i] - q[i] * proj) * inv;
      if (live) store_chunk<T, CH>(dQ + base + static_cast<size_t>(row) * lay.row + c0, g);
      __syncthreads();
    }
  } else {
    const bool do_dv = kTogether || blockIdx.y == 1;
    const bool do_dk = kTogether || blockIdx.y == 2;
    const float* __restrict__ ds = dstates + static_cast<size_t>(bh) * D * D;
    float (*Mv)[D] = M0;                   // dS[a][c]
    float (*Mk)[D] = kTogether ? M1 : M0;  // dS^T[c][a]
    if (do_dv) load_state<D, false>(ds, scale, Mv);
    if (do_dk) load_state<D, true>(ds, scale, Mk);
    const uint8_t* __restrict__ m =
        mask == nullptr ? nullptr : mask + static_cast<size_t>(bh / H) * N;
    __syncthreads();
    for (int r0 = r_begin; r0 < r_end; r0 += kTileRows) {
      const int row = r0 + lrow;
      const bool inrange = row < r_end;
      bool live = inrange;
      if (live && m != nullptr) live = m[row] != 0;
      float k[CH], v[CH], gv[CH], h[CH];
#pragma unroll
      for (int i = 0; i < CH; ++i) k[i] = v[i] = 0.0f;
      if (live) {
        load_chunk<T, CH>(K + base + static_cast<size_t>(row) * lay.row + c0, k);
        if (do_dk) load_chunk<T, CH>(V + base + static_cast<size_t>(row) * lay.row + c0, v);
      }
      float ss = 0.0f;
#pragma unroll
      for (int i = 0; i < CH; ++i) ss += k[i] * k[i];
      const float inv = inv_norm(sum8(ss), eps);
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        k[i] *= inv;
        t0[lrow][c0 + i] = k[i];
        t1[lrow][c0 + i] = v[i];
        gv[i] = h[i] = 0.0f;
      }
      __syncthreads();
      if (kTogether) {
#pragma unroll 8
        for (int a = 0; a < D; ++a) {
          const float ka = t0[lrow][a];  // dV_c = sum_a khat_a dS[a][c]
          const float va = t1[lrow][a];  // h_a  = sum_c v_c dS[a][c] = sum_c v_c dS^T[c][a]
#pragma unroll
          for (int i = 0; i < CH; ++i) {
            gv[i] += ka * Mv[a][c0 + i];
            h[i] += va * Mk[a][c0 + i];
          }
        }
      } else if (do_dv) {
#pragma unroll 8
        for (int a = 0; a < D; ++a) {
          const float ka = t0[lrow][a];
#pragma unroll
          for (int i = 0; i < CH; ++i) gv[i] += ka * Mv[a][c0 + i];
        }
      } else {
#pragma unroll 8
        for (int a = 0; a < D; ++a) {
          const float va = t1[lrow][a];  // h_a  = sum_c v_c dS[a][c] = sum_c v_c dS^T[c][a]
#pragma unroll
          for (int i = 0; i < CH; ++i) h[i] += va * Mk[a][c0 + i];
        }
      }
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < CH; ++i) proj += k[i] * h[i];
      proj = sum8(proj);
#pragma unroll
      for (int i = 0; i < CH; ++i) {
        h[i] = live ? (h[i] - k[i] * proj) * inv : 0.0f;
        gv[i] = live ? gv[i] : 0.0f;
      }
      if (inrange) {
        if (do_dk) store_chunk<T, CH>(dK + base + static_cast<size_t>(row) * lay.row + c0, h);
        if (do_dv) store_chunk<T, CH>(dV + base + static_cast<size_t>(row) * lay.row + c0, gv);
      }
      __syncthreads();
    }
  }
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

// Where the reduced states of the generic path live: behind the partials when a reduction
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

// Dynamic LDS above 64 KB has to be granted per kernel first.
template <typename Kern>
hipError_t allow_lds(Kern kern, size_t bytes) {
  if (bytes <= 64 * 1024) return hipSuccess;
  return grant_dynamic_lds(reinterpret_cast<const void*>(kern), static_cast<int>(bytes));
}

ElemStrides elem_strides(const Problem& p) {
  return ElemStrides{p.stride_batch, p.stride_head, p.stride_row};
}

template <typename T, int D>
hipError_t run_fwd(const Problem& p, const Plan& plan) {
  const int BH = p.B * p.H;
  const dim3 grid(static_cast<unsigned>(BH) * plan.splits, 1, 1);
  hipLaunchKernelGGL((state_kernel<T, D>), grid, dim3(kThreads), 0, p.stream,
                     static_cast<const T*>(p.Q), static_cast<const T*>(p.K),
                     static_cast<const T*>(p.V), static_cast<const T*>(nullptr), p.mask,
                     p.workspace, p.H, p.N, plan.splits, plan.rows_per_split, size_t{0}, p.eps,
                     elem_strides(p));
  const float* states = reduce_generic(p, plan, 1);
  // the caller keeps the state for its backward call: same [B*H][D*D] layout, a plain copy
  if (p.saved_state != nullptr)
    launch_reduce_states(states, p.saved_state, 1, D * D, static_cast<size_t>(BH), p.stream);
  constexpr size_t lds = (D * D + kTileRows * (D + 4)) * sizeof(float);
  if (hipError_t err = allow_lds(apply_fwd_kernel<T, D>, lds)) return err;
  hipLaunchKernelGGL((apply_fwd_kernel<T, D>), grid, dim3(kThreads), lds, p.stream,
                     static_cast<const T*>(p.Q), states, static_cast<T*>(p.O), p.H, p.N,
                     plan.splits, plan.rows_per_split, p.scale, p.slice_scale, p.eps,
                     elem_strides(p));
  return hipGetLastError();
}

template <typename T, int D>
hipError_t run_bwd(const Problem& p, const Plan& plan) {
  const int BH = p.B * p.H;
  const dim3 grid(static_cast<unsigned>(BH) * plan.splits, 2, 1);
  const dim3 apply_grid(grid.x, bwd_apply_grid_y<D>(), 1);
  const size_t second = static_cast<size_t>(BH) * plan.splits * D * D;
  hipLaunchKernelGGL((state_kernel<T, D>), grid, dim3(kThreads), 0, p.stream,
                     static_cast<const T*>(p.Q), static_cast<const T*>(p.K),
                     static_cast<const T*>(p.V), static_cast<const T*>(p.dO), p.mask,
                     p.workspace, p.H, p.N, plan.splits, plan.rows_per_split, second, p.eps,
                     elem_strides(p));
  const float* states = reduce_generic(p, plan, 2);
  const float* dstates = states + (plan.splits == 1 ? second : static_cast<size_t>(BH) * D * D);
  constexpr size_t lds = bwd_apply_lds_floats<D>() * sizeof(float);
  if (hipError_t err = allow_lds(apply_bwd_kernel<T, D>, lds)) return err;
  hipLaunchKernelGGL((apply_bwd_kernel<T, D>), apply_grid, dim3(kThreads), lds, p.stream,
                     static_cast<const T*>(p.Q), static_cast<const T*>(p.K),
                     static_cast<const T*>(p.V), static_cast<const T*>(p.dO), p.mask, states,
                     dstates, static_cast<T*>(p.dQ), static_cast<T*>(p.dK),
                     static_cast<T*>(p.dV), p.H, p.N, plan.splits, plan.rows_per_split, p.scale,
                     p.slice_scale, p.eps, elem_strides(p));
  if (p.dlog_scale != nullptr)
    hipLaunchKernelGGL(state_inner_product_kernel, dim3(static_cast<unsigned>(BH)),
                       dim3(kThreads), 0, p.stream, states, dstates, D * D, p.scale,
                       p.slice_scale, p.dlog_scale);
  return hipGetLastError();
}

// The same launch structure with the matrix-core kernels for 256-byte rows (cotten_wide.hip) in
// place of the vector-ALU state and apply kernels; reduction, kept state and <S, dS> as above.
hipError_t run_wide(const Problem& p, const Plan& plan, bool bwd) {
  if (wide_fused_applies(p.B, p.H, plan.splits, bwd)) return launch_wide_fused(p, plan, bwd);
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
    // Enough workgroups to fill 256 compute units a few times over, at least one
    // 32-row tile each.
    plan.path = Plan::kGeneric;
    // The matrix-core kernels for 256-byte rows build operand images per workgroup and stage
    // 64 rows per round: about two workgroups per compute unit, in blocks of 64 rows.
    // A d x d state is as large as 64 (16-bit: 256) rows of a tensor there, and every split
    // writes one and has the sum read back: no fewer than 256 rows per workgroup, and a
    // sequence is not cut at all once there is a workgroup per compute unit without it.
    const bool wide = wide_supports(dtype, D);
    const long target = wide ? 512 : 2048, block = wide ? 64 : kTileRows;
    splits = wide && BH >= 256 ? 1 : (target + BH - 1) / BH;
    const long max_splits = wide ? (N + 255) / 256 : (N + block - 1) / block;
    if (splits > max_splits) splits = max_splits;
    if (splits < 1) splits = 1;
    rows = (N + splits - 1) / splits;
    rows = (rows + block - 1) / block * block;
  }
  splits = (N + rows - 1) / rows;
  plan.splits = static_cast<int>(splits);
  plan.rows_per_split = static_cast<int>(rows);
  if (plan.path == Plan::kSplit) {
    const size_t side = mfma_state_dim(dtype);
    plan.workspace_floats = static_cast<size_t>(BH) * side * side * splits * nstates;
  } else {
    // partial states, plus the reduced states when there is more than one partial
    // (256-byte rows, sequence not cut: the state never leaves the compute unit)
    plan.workspace_floats =
        wide_supports(dtype, D) && wide_fused_applies(B, H, static_cast<int>(splits), is_bwd)
            ? 0
            : static_cast<size_t>(BH) * D * D * nstates * (splits + (splits > 1 ? 1 : 0));
  }
  return plan;
}

// The vector-ALU kernels are written for any (element type, d_h); the one instance compiled in is
// the shape no matrix-core kernel serves, fp32 rows of 512 bytes.
hipError_t launch_generic_fwd(const Problem& p, const Plan& plan) {
  if (wide_supports(p.dtype, p.D)) return run_wide(p, plan, false);
  if (p.dtype == 0 && p.D == 128) return run_fwd<float, 128>(p, plan);
  return hipErrorInvalidValue;
}

hipError_t launch_generic_bwd(const Problem& p, const Plan& plan) {
  if (wide_supports(p.dtype, p.D)) return run_wide(p, plan, true);
  if (p.dtype == 0 && p.D == 128) return run_bwd<float, 128>(p, plan);
  return hipErrorInvalidValue;
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
