// Causal variant of the cosine attention (row i attends the valid keys j <= i), the form the
// paper's bidirectional model leaves out ("no causal mask"):
//
//     S_i = sum_{j <= i} m_j khat_j^T v_j          O_i = scale * qhat_i S_i
//
// computed as a scan over chunks of 16 rows with the d x d prefix state carried in LDS:
//
//     O_c = scale * ( Qhat_c S_before  +  tril(Qhat_c Khat_c^T) V_c ),     S_before += Khat_c^T V_c
//
// and, for the backward, one sweep forwards (dQ needs the prefix state) and one sweep backwards
// (dK, dV need the suffix state T = scale * sum_{i later} qhat_i^T dO_i), as two independent
// halves of one launch:
//
//     G = dO_c V_c^T, P = Qhat_c Khat_c^T          (16 x 16, lower triangle, valid keys)
//     g_c  = scale * (dO_c S_before^T + G Khat_c)              -> dQ
//     dV_c = Khat_c T_after + scale * P^T dO_c
//     h_c  = V_c T_after^T  + scale * G^T Qhat_c               -> dK
//
// Vector-ALU kernels, one workgroup of 256 threads per slice, any supported element type,
// d_h in {16, 32, 64}.  Not tuned: the bidirectional kernels are the benchmarked path.  They
// serve the shapes the matrix-core kernels do not take (fp32 d_h = 64); every other call is
// routed to those by launch_causal() below, which for sequences of more than one chunk also
// launches the scan over the chunk states defined at the end of this file.
#include "cotten_device.h"
#include "cotten_launch.h"

namespace cotten {
namespace {

constexpr int kThreads = 256;
constexpr int kChunk = 16;  // rows per step of the scan

struct ElemStrides {
  long long batch, head, row;
  __device__ __forceinline__ size_t slice_base(int bh, int H) const {
    return static_cast<size_t>(bh / H) * batch + static_cast<size_t>(bh % H) * head;
  }
};

// Sum over the 16 consecutive lanes that share a row.
__device__ __forceinline__ float sum16(float x) {
  x += __shfl_xor(x, 1);
  x += __shfl_xor(x, 2);
  x += __shfl_xor(x, 4);
  x += __shfl_xor(x, 8);
  return x;
}

// LDS of one workgroup: the carried d x d state and the rows of the current chunk.
template <int D>
struct Lds {
  float state[D][D + 1];
  float q[kChunk][D + 1];     // qhat rows
  float k[kChunk][D + 1];     // khat rows (zero for masked or absent keys)
  float v[kChunk][D + 1];     // v rows    (zero for masked or absent keys)
  float g[kChunk][D + 1];     // dO rows   (backward)
  float P[kChunk][kChunk + 1];
  float G[kChunk][kChunk + 1];
};

// Thread (r, c) of the workgroup: row r of the chunk, columns c, c + 16, c + 32, ...
struct Who {
  int r, c;
  __device__ __forceinline__ Who() : r(threadIdx.x >> 4), c(threadIdx.x & 15) {}
};

// Loads row (row0 + r) of X into x[] (zeros if the row does not take part).
template <typename T, int D>
__device__ __forceinline__ void load_row(const T* __restrict__ X, size_t base, long long row_stride,
                                         int row, bool live, const Who& w, float (&x)[D / 16]) {
#pragma unroll
  for (int i = 0; i < D / 16; ++i)
    x[i] = live ? to_float(X[base + static_cast<size_t>(row) * row_stride + w.c + 16 * i]) : 0.0f;
}

// x <- x / sqrt(|row|^2 + eps); returns 1/r (0 if the row does not take part).
template <int D>
__device__ __forceinline__ float normalise(float (&x)[D / 16], float eps, bool live) {
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < D / 16; ++i) ss += x[i] * x[i];
  const float inv = live ? 1.0f / sqrtf(sum16(ss) + eps) : 0.0f;
#pragma unroll
  for (int i = 0; i < D / 16; ++i) x[i] *= inv;
  return inv;
}

template <int D>
__device__ __forceinline__ void put_row(float (*dst)[D + 1], const Who& w, const float (&x)[D / 16]) {
#pragma unroll
  for (int i = 0; i < D / 16; ++i) dst[w.r][w.c + 16 * i] = x[i];
}

// state[a][c] += factor * sum_j X[j][a] * Y[j][c] over the chunk
template <int D>
__device__ __forceinline__ void add_outer(float (*state)[D + 1], const float (*X)[D + 1],
                                          const float (*Y)[D + 1], float factor) {
  for (int e = threadIdx.x; e < D * D; e += kThreads) {
    const int a = e / D, c = e % D;
    float acc = 0.0f;
#pragma unroll
    for (int j = 0; j < kChunk; ++j) acc += X[j][a] * Y[j][c];
    state[a][c] += factor * acc;
  }
}

struct Args {
  const void* Q;
  const void* K;
  const void* V;
  const void* dO;
  const uint8_t* mask;
  void* O;
  void* dQ;
  void* dK;
  void* dV;
  int H, N;
  float scale, eps;
  const float* scales;
  ElemStrides lay;
};

template <typename T, int D>
__global__ __launch_bounds__(kThreads) void causal_fwd_kernel(const Args a) {
  __shared__ Lds<D> s;
  const Who w;
  const int bh = blockIdx.x, N = a.N;
  const size_t base = a.lay.slice_base(bh, a.H);
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  T* O = static_cast<T*>(a.O);
  const uint8_t* mask = a.mask != nullptr ? a.mask + static_cast<size_t>(bh / a.H) * N : nullptr;
  const float scale = a.scales != nullptr ? a.scales[bh] : a.scale;
  for (int e = threadIdx.x; e < D * (D + 1); e += kThreads) (&s.state[0][0])[e] = 0.0f;

  for (int row0 = 0; row0 < N; row0 += kChunk) {
    const int row = row0 + w.r;
    const bool there = row < N;
    const bool key = there && (mask == nullptr || mask[row] != 0);
    float q[D / 16], k[D / 16], v[D / 16];
    load_row<T, D>(Q, base, a.lay.row, row, there, w, q);
    load_row<T, D>(K, base, a.lay.row, row, key, w, k);
    load_row<T, D>(V, base, a.lay.row, row, key, w, v);
    normalise<D>(q, a.eps, there);
    normalise<D>(k, a.eps, key);
    __syncthreads();  // the previous chunk is done with the row buffers and the state update
    put_row<D>(s.q, w, q);
    put_row<D>(s.k, w, k);
    put_row<D>(s.v, w, v);
    __syncthreads();
    {  // P[r][c] = qhat_r . khat_c for keys of the chunk not later than the row
      float p = 0.0f;
      if (w.c <= w.r) {
#pragma unroll 8
        for (int x = 0; x < D; ++x) p += s.q[w.r][x] * s.k[w.c][x];
      }
      s.P[w.r][w.c] = p;
    }
    __syncthreads();
    float o[D / 16];
#pragma unroll
    for (int i = 0; i < D / 16; ++i) o[i] = 0.0f;
#pragma unroll 4
    for (int x = 0; x < D; ++x) {
      const float qx = s.q[w.r][x];
#pragma unroll
      for (int i = 0; i < D / 16; ++i) o[i] += qx * s.state[x][w.c + 16 * i];
    }
#pragma unroll
    for (int j = 0; j < kChunk; ++j) {
      const float p = s.P[w.r][j];
#pragma unroll
      for (int i = 0; i < D / 16; ++i) o[i] += p * s.v[j][w.c + 16 * i];
    }
    if (there) {
#pragma unroll
      for (int i = 0; i < D / 16; ++i)
        O[base + static_cast<size_t>(row) * a.lay.row + w.c + 16 * i] = from_float<T>(scale * o[i]);
    }
    __syncthreads();  // everyone has read the state
    add_outer<D>(s.state, s.k, s.v, 1.0f);
  }
}

// blockIdx.y == 0: forward sweep, dQ.   blockIdx.y == 1: backward sweep, dK and dV.
template <typename T, int D>
__global__ __launch_bounds__(kThreads) void causal_bwd_kernel(const Args a) {
  __shared__ Lds<D> s;
  const Who w;
  const int bh = blockIdx.x, N = a.N;
  const bool backwards = blockIdx.y == 1;
  const size_t base = a.lay.slice_base(bh, a.H);
  const T* Q = static_cast<const T*>(a.Q);
  const T* K = static_cast<const T*>(a.K);
  const T* V = static_cast<const T*>(a.V);
  const T* dO = static_cast<const T*>(a.dO);
  const uint8_t* mask = a.mask != nullptr ? a.mask + static_cast<size_t>(bh / a.H) * N : nullptr;
  const float scale = a.scales != nullptr ? a.scales[bh] : a.scale;
  for (int e = threadIdx.x; e < D * (D + 1); e += kThreads) (&s.state[0][0])[e] = 0.0f;

  const int n_chunks = (N + kChunk - 1) / kChunk;
  for (int step = 0; step < n_chunks; ++step) {
    const int row0 = (backwards ? n_chunks - 1 - step : step) * kChunk;
    const int row = row0 + w.r;
    const bool there = row < N;
    const bool key = there && (mask == nullptr || mask[row] != 0);
    float q[D / 16], k[D / 16], v[D / 16], g[D / 16];
    load_row<T, D>(Q, base, a.lay.row, row, there, w, q);
    load_row<T, D>(K, base, a.lay.row, row, key, w, k);
    load_row<T, D>(V, base, a.lay.row, row, key, w, v);
    load_row<T, D>(dO, base, a.lay.row, row, there, w, g);
    const float inv_q = normalise<D>(q, a.eps, there);
    const float inv_k = normalise<D>(k, a.eps, key);
    __syncthreads();
    put_row<D>(s.q, w, q);
    put_row<D>(s.k, w, k);
    put_row<D>(s.v, w, v);
    put_row<D>(s.g, w, g);
    __syncthreads();
    {  // lower triangle of the chunk: P = qhat . khat,  G = dO . v
      float p = 0.0f, gg = 0.0f;
      if (w.c <= w.r) {
#pragma unroll 8
        for (int x = 0; x < D; ++x) {
          p += s.q[w.r][x] * s.k[w.c][x];
          gg += s.g[w.r][x] * s.v[w.c][x];
        }
      }
      s.P[w.r][w.c] = p;
      s.G[w.r][w.c] = gg;
    }
    __syncthreads();
    if (!backwards) {
      // state = S before the chunk:  g_r = scale * (dO_r S^T + sum_j G[r][j] khat_j)
      float t[D / 16];
#pragma unroll
      for (int i = 0; i < D / 16; ++i) t[i] = 0.0f;
#pragma unroll 4
      for (int x = 0; x < D; ++x) {
        const float gx = s.g[w.r][x];
#pragma unroll
        for (int i = 0; i < D / 16; ++i) t[i] += gx * s.state[w.c + 16 * i][x];
      }
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const float gj = s.G[w.r][j];
#pragma unroll
        for (int i = 0; i < D / 16; ++i) t[i] += gj * s.k[j][w.c + 16 * i];
      }
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < D / 16; ++i) {
        t[i] *= scale;
        proj += q[i] * t[i];
      }
      proj = sum16(proj);
      if (there) {
        T* out = static_cast<T*>(a.dQ);
#pragma unroll
        for (int i = 0; i < D / 16; ++i)
          out[base + static_cast<size_t>(row) * a.lay.row + w.c + 16 * i] =
              from_float<T>((t[i] - q[i] * proj) * inv_q);
      }
      __syncthreads();
      add_outer<D>(s.state, s.k, s.v, 1.0f);
    } else {
      // state = T after the chunk (scale included):
      //   dV_r = khat_r T + scale * sum_{i >= r} P[i][r] dO_i
      //   h_r  = v_r T^T  + scale * sum_{i >= r} G[i][r] qhat_i
      float dv[D / 16], h[D / 16];
#pragma unroll
      for (int i = 0; i < D / 16; ++i) dv[i] = h[i] = 0.0f;
#pragma unroll 4
      for (int x = 0; x < D; ++x) {
        const float kx = s.k[w.r][x], vx = s.v[w.r][x];
#pragma unroll
        for (int i = 0; i < D / 16; ++i) {
          dv[i] += kx * s.state[x][w.c + 16 * i];
          h[i] += vx * s.state[w.c + 16 * i][x];
        }
      }
#pragma unroll
      for (int j = 0; j < kChunk; ++j) {
        const float p = scale * s.P[j][w.r], gg = scale * s.G[j][w.r];  // zero for j < r
#pragma unroll
        for (int i = 0; i < D / 16; ++i) {
          dv[i] += p * s.g[j][w.c + 16 * i];
          h[i] += gg * s.q[j][w.c + 16 * i];
        }
      }
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < D / 16; ++i) proj += k[i] * h[i];
      proj = sum16(proj);
      if (there) {
        T* out_k = static_cast<T*>(a.dK);
        T* out_v = static_cast<T*>(a.dV);
#pragma unroll
        for (int i = 0; i < D / 16; ++i) {
          const size_t at = base + static_cast<size_t>(row) * a.lay.row + w.c + 16 * i;
          // masked keys: khat, v and 1/r are zero, so both come out as exact zeros
          out_k[at] = from_float<T>(key ? (h[i] - k[i] * proj) * inv_k : 0.0f);
          out_v[at] = from_float<T>(key ? dv[i] : 0.0f);
        }
      }
      __syncthreads();
      add_outer<D>(s.state, s.q, s.g, scale);
    }
  }
}

template <typename T, int D>
hipError_t run(const Problem& p, bool bwd) {
  Args a{};
  a.Q = p.Q; a.K = p.K; a.V = p.V; a.dO = p.dO; a.mask = p.mask;
  a.O = p.O; a.dQ = p.dQ; a.dK = p.dK; a.dV = p.dV;
  a.H = p.H; a.N = p.N;
  a.scale = p.scale; a.eps = p.eps; a.scales = p.slice_scale;
  a.lay = ElemStrides{p.stride_batch, p.stride_head, p.stride_row};
  const unsigned BH = static_cast<unsigned>(p.B) * p.H;
  if (bwd)
    hipLaunchKernelGGL((causal_bwd_kernel<T, D>), dim3(BH, 2), dim3(kThreads), 0, p.stream, a);
  else
    hipLaunchKernelGGL((causal_fwd_kernel<T, D>), dim3(BH), dim3(kThreads), 0, p.stream, a);
  return hipGetLastError();
}

// Chunked matrix-core path: the states of the chunks, [slice][chunk][dd] floats, become in
// place the sums a chunk needs.  Block row 0: every S_c is replaced by the sum of the S before
// chunk c, added in chunk order; block row 1 (backward): every T_c, stored behind all the S,
// by the sum of the T after chunk c, added from the last chunk down.  One thread per four
// consecutive floats of a state; the values of up to kAhead chunks are requested together.
// The last S and the first T were never written and are not read.
typedef float f32x4_t __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(kThreads) void chunk_scan_kernel(float* states, int slices, int chunks,
                                                              int quads) {
  constexpr int kAhead = 8;
  const int id = blockIdx.x * kThreads + threadIdx.x;
  if (id >= slices * quads) return;
  const bool downwards = blockIdx.y == 1;
  f32x4_t* base = reinterpret_cast<f32x4_t*>(states) +
                  (static_cast<size_t>(blockIdx.y) * slices + id / quads) * chunks * quads + id % quads;
  f32x4_t run = {0.f, 0.f, 0.f, 0.f};
  for (int s0 = 0; s0 < chunks; s0 += kAhead) {
    f32x4_t own[kAhead];
#pragma unroll
    for (int j = 0; j < kAhead; ++j) {
      const int step = s0 + j;  // chunk `step` counted from the end the sum starts at
      own[j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      if (step < chunks - 1)
        own[j] = base[static_cast<size_t>(downwards ? chunks - 1 - step : step) * quads];
    }
#pragma unroll
    for (int j = 0; j < kAhead; ++j) {
      const int step = s0 + j;
      if (step < chunks) {
        base[static_cast<size_t>(downwards ? chunks - 1 - step : step) * quads] = run;
        run += own[j];
      }
    }
  }
}

}  // namespace

hipError_t launch_chunk_scan(float* states, int slices, int chunks, int dd, bool with_queries,
                             hipStream_t stream) {
  const int quads = dd / 4;
  const dim3 grid((static_cast<unsigned>(slices) * quads + kThreads - 1) / kThreads,
                  with_queries ? 2 : 1);
  hipLaunchKernelGGL(chunk_scan_kernel, grid, dim3(kThreads), 0, stream, states, slices, chunks, quads);
  return hipGetLastError();
}

bool causal_supports(int D) { return D == 16 || D == 32 || D == 64; }

size_t causal_workspace_floats(int B, int H, int N, int D, int dtype, bool is_bwd) {
  const int chunks = causal_chunks(N);
  if (chunks < 2 || !causal_resident_supports(dtype, D)) return 0;
  const size_t side = static_cast<size_t>(mfma_state_dim(dtype));
  return static_cast<size_t>(B) * H * chunks * side * side * (is_bwd ? 2 : 1);
}

hipError_t launch_causal(const Problem& p, bool bwd) {
  if (!causal_resident_supports(p.dtype, p.D)) {
    // the one shape left to the scan; its other instances would be reached by no call
    if (p.dtype != 0 || p.D != 64) return hipErrorInvalidValue;
    return run<float, 64>(p, bwd);
  }
  // tile pairs on the matrix cores, up to 208 rows resident in LDS per workgroup
  const int chunks = causal_chunks(p.N);
  if (chunks > 1) {
    if (p.workspace == nullptr) return hipErrorInvalidValue;
    const int side = mfma_state_dim(p.dtype);
    hipError_t err = launch_chunk_states(p, kCausalChunkRows / 16, chunks, bwd);
    if (err != hipSuccess) return err;
    err = launch_chunk_scan(p.workspace, p.B * p.H, chunks, side * side, bwd, p.stream);
    if (err != hipSuccess) return err;
  }
  return launch_resident_causal(p, bwd, chunks);
}

}  // namespace cotten
