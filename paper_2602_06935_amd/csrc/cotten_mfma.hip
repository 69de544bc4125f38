// MFMA path of the cosine attention for 128-byte rows on gfx950:
//     bf16 or fp16 I/O with d_h = 64   and   fp32 I/O with d_h = 32.
//
// Work unit: one wavefront streams 16-row tiles of a slice.  A tile is loaded with
// 128-bit accesses (8 lanes per 128-byte row, 8 rows per instruction) and parked in a
// wave-private LDS tile, from which the matrix cores are fed:
//   state products  S += Xhat^T Y  (contraction over rows; Xhat normalised in fp32 registers
//                   before it is written to the tile)
//                   bf16: 32x32x16 MFMA, operands fetched with the transposing LDS read
//                   fp32: 32x32x2 MFMA, one LDS dword per lane and step
//   apply products  T = X W        (contraction over columns; X raw, the 1/r of each row is
//                   applied to the result; W held in registers)
//                   bf16: 16x16x32 MFMA      fp32: 16x16x4 MFMA
// Products are computed transposed, which leaves every lane with runs of neighbouring
// columns of one tile row; the epilogue (projection off the unit row, 1/r, masking) runs in
// fp32 in that layout, next to the tile rows fetched from LDS in the same arrangement, and
// results leave with 128-bit stores.
//
// Fused kernels (one workgroup = 4 waves per slice) run all phases in one launch;
// split kernels cut long sequences over several workgroups per slice and pass
// partial states through the workspace.
#include "cotten_launch.h"
#include "cotten_mfma_core.h"

// Optional phase timestamps for tuning builds (-DCOTTEN_TRACE): wave w of workgroup b < 8
// stores the shader clock at trace point i.  Compiles to nothing otherwise.
#ifdef COTTEN_TRACE
__device__ long long cotten_trace_buf[8 * 4 * 16];
#define COTTEN_TRACE_POINT(i)                                                        \
  do {                                                                               \
    if (blockIdx.x < 8 && blockIdx.y == 0 && (threadIdx.x & 63) == 0)                \
      cotten_trace_buf[(blockIdx.x * 4 + (threadIdx.x >> 6)) * 16 + (i)] = clock64(); \
  } while (0)
extern "C" int cotten_trace_read(long long* host, int n) {
  return static_cast<int>(hipMemcpyFromSymbol(host, HIP_SYMBOL(cotten_trace_buf), n * sizeof(long long)));
}
#else
#define COTTEN_TRACE_POINT(i) do {} while (0)
#endif

namespace cotten {
namespace {

using namespace mfma;

constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr bool kSplitStream = false;  // store policy of the split kernels (measured)

// ---- LDS map ----------------------------------------------------------------------------
// [working set of the 4 waves | (aliased) two reduction buffers][image 0][image 1][flags]

template <class F>
struct Layout {
  static constexpr int D = F::D;
  static constexpr int kWaveBytes = 2 * kTileBytes + TR * 4;           // two tiles, 1/r per row
  static constexpr int kRStride = D + 4;                              // floats, column-major
  static constexpr int kRFloats = D * kRStride;
  static constexpr int kWorkBytes =
      kWaves * kWaveBytes > 2 * kRFloats * 4 ? kWaves * kWaveBytes : 2 * kRFloats * 4;
  static constexpr int kImage0 = kWorkBytes;
  static constexpr int kImage1 = kImage0 + F::kImageBytes;
  static constexpr int kFlags = kImage1 + F::kImageBytes;
};

template <class F>
struct WaveLds {
  unsigned char* Xt;
  unsigned char* Yt;
  float* inv;
  __device__ __forceinline__ WaveLds(unsigned char* smem, int wave) {
    unsigned char* base = smem + wave * Layout<F>::kWaveBytes;
    Xt = base;
    Yt = base + kTileBytes;
    inv = reinterpret_cast<float*>(base + 2 * kTileBytes);
  }
};

// Copies the key mask of the workgroup's tiles into LDS as "takes part" flags.
__device__ __forceinline__ void fill_flags(uint8_t* flags, const uint8_t* __restrict__ mask,
                                           const Rows& rows) {
  for (int i = threadIdx.x; i < rows.n_tiles * TR; i += kThreads) {
    const int row = rows.row0(i / TR) + (i % TR);
    uint8_t f = 0;
    if (row < rows.limit) f = mask[row] != 0;
    flags[i] = f;
  }
}

// First tile of this wave (local tile index = wave), issued early by the caller.
template <bool USE_Y>
__device__ __forceinline__ void load_first(Raw& a, const Lane& L, const Src& src, const Rows& rows) {
  load_raw<USE_Y>(a, L, src, rows, L.wave);
}

// Walks the local tiles wave, wave+kWaves, ... owned by this wave with the global loads of
// the next DEPTH tiles in flight while the current one is processed.  `first` holds the
// wave's first tile, already loaded (or being loaded) by the caller.  body(raw, row0).
template <bool USE_Y, int DEPTH, typename Body>
__device__ __forceinline__ void for_each_tile(const Lane& L, const Src& src, const Rows& rows,
                                              Raw& first, Body&& body) {
  static_assert(DEPTH >= 1 && DEPTH <= 3, "prefetch depth");
  const int n_tiles = rows.n_tiles;
  if (L.wave >= n_tiles) return;
  Raw ring[DEPTH + 1];
  ring[0] = first;
#pragma unroll
  for (int i = 1; i < DEPTH; ++i) load_raw<USE_Y>(ring[i], L, src, rows, L.wave + i * kWaves);
  for (int t0 = L.wave;; t0 += (DEPTH + 1) * kWaves) {
#pragma unroll
    for (int j = 0; j <= DEPTH; ++j) {
      const int t = t0 + j * kWaves;
      if (t >= n_tiles) return;
      load_raw<USE_Y>(ring[(j + DEPTH) % (DEPTH + 1)], L, src, rows, t + DEPTH * kWaves);
      body(ring[j], rows.row0(t));
    }
  }
}

// For short sequences (at most 4 tiles per wave) a wave can simply keep all its tiles of a
// tensor pair in registers: every load is issued at the start of the kernel, and a second
// walk over the same tiles (K, V in the backward) costs no memory traffic.
struct Kept {
  static constexpr int kTiles = 4;
  Raw t[kTiles];
};

template <bool USE_Y>
__device__ __forceinline__ void load_kept(Kept& k, const Lane& L, const Src& src, const Rows& rows) {
#pragma unroll
  for (int i = 0; i < Kept::kTiles; ++i) load_raw<USE_Y>(k.t[i], L, src, rows, L.wave + i * kWaves);
}

template <bool USE_Y, int DEPTH, typename Body>
__device__ __forceinline__ void for_each_tile(const Lane& L, const Src&, const Rows& rows,
                                              Kept& kept, Body&& body) {
#pragma unroll
  for (int i = 0; i < Kept::kTiles; ++i) {
    const int t = L.wave + i * kWaves;
    if (t >= rows.n_tiles) return;
    body(kept.t[i], rows.row0(t));
  }
}

// Uniform spelling for the kernels that exist in both variants.
template <bool USE_Y>
__device__ __forceinline__ void load_tiles(Raw& r, const Lane& L, const Src& src, const Rows& rows) {
  load_first<USE_Y>(r, L, src, rows);
}
template <bool USE_Y>
__device__ __forceinline__ void load_tiles(Kept& k, const Lane& L, const Src& src, const Rows& rows) {
  load_kept<USE_Y>(k, L, src, rows);
}
// before a second walk over the same tiles
template <bool USE_Y>
__device__ __forceinline__ void reload_tiles(Raw& r, const Lane& L, const Src& src, const Rows& rows) {
  load_first<USE_Y>(r, L, src, rows);
}
template <bool USE_Y>
__device__ __forceinline__ void reload_tiles(Kept&, const Lane&, const Src&, const Rows&) {}
template <bool SHORT>
struct TilesOf {
  typedef Raw type;
};
template <>
struct TilesOf<true> {
  typedef Kept type;
};

// ---- passes -------------------------------------------------------------------------------
// Every pass takes the wave's first tile already loaded in `first` (or all its tiles, Kept).

// acc += sum over live rows of xhat^T y
template <class F, int DEPTH, class First>
__device__ __forceinline__ void state_pass(const Lane& L, const WaveLds<F>& W,
                                           const Src& src, const Rows rows, float eps, First& first,
                                           typename F::Acc& acc) {
  for_each_tile<true, DEPTH>(L, src, rows, first, [&](const Raw& r, int) {
    if (__ballot(r.live != 0) == 0) return;  // no live row in this tile (uniform)
    float inv[2];
    stage<F, kXNormalized, true>(r, L, eps, W.Xt, W.Yt, inv);
    wave_lds_fence();
    acc.mfma(W.Xt, W.Yt, L);
    wave_lds_fence();
  });
}

// The 1/r of the tile's 16 rows, handed from the load layout to the product layout.
template <class F>
__device__ __forceinline__ float inv_by_row(const WaveLds<F>& W, const Lane& L,
                                            const float (&inv)[2]) {
  if (L.ch == 0) {
    W.inv[L.r8] = inv[0];
    W.inv[L.r8 + 8] = inv[1];
  }
  wave_lds_fence();
  return W.inv[L.i16];
}

// O rows = (q rows x W) / r   (W = scale * S, image op[c][a])
template <class F, int DEPTH, bool STREAM, class First>
__device__ __forceinline__ void fwd_apply_pass(const Lane& L, const WaveLds<F>& W,
                                               const Src& src, unsigned char* __restrict__ O,
                                               const Rows rows, float eps, First& first,
                                               const typename F::Operand& Sop) {
  for_each_tile<false, DEPTH>(L, src, rows, first, [&](const Raw& r, int row0) {
    float inv[2];
    stage<F, kXRaw, false>(r, L, eps, W.Xt, W.Yt, inv);
    const float inv_r = inv_by_row(W, L, inv);
    typename F::TileRows x;
    x.load(W.Xt, L);
    f32x4_t out[F::NT];
    F::apply(x, Sop, out);
    float o[2 * F::EPL];
    product_rows<F>(out, o);
#pragma unroll
    for (int i = 0; i < 2 * F::EPL; ++i) o[i] *= inv_r;
    const int row = row0 + L.i16;
    if (row < rows.limit) store_product_row<F, STREAM>(O, row, src.row, L, o);
    wave_lds_fence();
  });
}

// dQ rows from (Q, dO) and W = scale * S (image op[a][c]); with ACCUM also dsacc += qhat^T dO.
template <class F, bool ACCUM, int DEPTH, bool STREAM, class First>
__device__ __forceinline__ void bwd_q_pass(const Lane& L, const WaveLds<F>& W,
                                           const Src& src, unsigned char* __restrict__ dQ,
                                           const Rows rows,
                                           float eps, First& first, const unsigned char* Simage,
                                           typename F::Acc& dsacc) {
  // With the state accumulators live, a large operand is re-read from LDS for every tile;
  // otherwise it stays in registers.
  constexpr bool kHold = !ACCUM || sizeof(typename F::Operand) <= 16 * 4;
  typename F::Operand held;
  if (kHold) held.load(Simage, L);
  for_each_tile<true, DEPTH>(L, src, rows, first, [&](const Raw& r, int row0) {
    float inv[2];
    stage<F, kXNormalized, true>(r, L, eps, W.Xt, W.Yt, inv);
    const float inv_r = inv_by_row(W, L, inv);
    if (ACCUM) dsacc.mfma(W.Xt, W.Yt, L);
    typename F::TileRows x, e;
    x.load(W.Yt, L);
    e.load(W.Xt, L);
    f32x4_t out[F::NT];
    if (kHold) {
      F::apply(x, held, out);  // g = scale * dO S^T
    } else {
      typename F::Operand fresh;
      fresh.load(Simage, L);
      F::apply(x, fresh, out);
    }
    float g[2 * F::EPL];
    product_rows<F>(out, g);
    project_rows<F, false>(g, e, inv_r, L);
    const int row = row0 + L.i16;
    if (row < rows.limit) store_product_row<F, STREAM>(dQ, row, src.row, L, g);
    wave_lds_fence();
  });
}

// dK, dV rows from (K, V) and scale * dS: dV = (k dS)/r (image op[c][a]),
// h = v dS^T (image op[a][c]).  Rows below the limit that are masked get zeros.
template <class F, int DEPTH, bool STREAM, class First>
__device__ __forceinline__ void bwd_kv_pass(const Lane& L, const WaveLds<F>& W,
                                            const Src& src, unsigned char* __restrict__ dK,
                                            unsigned char* __restrict__ dV, const Rows rows,
                                            float eps, First& first,
                                            const typename F::Operand& dSop_v,
                                            const typename F::Operand& dSop_h) {
  for_each_tile<true, DEPTH>(L, src, rows, first, [&](const Raw& r, int row0) {
    const int row = row0 + L.i16;
    if (__ballot(r.live != 0) == 0) {  // nothing live: only the zero rows are due
      float zeros[2 * F::EPL];
#pragma unroll
      for (int i = 0; i < 2 * F::EPL; ++i) zeros[i] = 0.0f;
      if (row < rows.limit) {
        store_product_row<F, STREAM>(dK, row, src.row, L, zeros);
        store_product_row<F, STREAM>(dV, row, src.row, L, zeros);
      }
      return;
    }
    float inv[2];
    stage<F, kXRaw, true>(r, L, eps, W.Xt, W.Yt, inv);
    // 1/r = 0 on masked rows, whose k and v registers are zero: dK and dV come out as exact zeros
    const float inv_r = inv_by_row(W, L, inv);
    typename F::TileRows xk, xv;
    xk.load(W.Xt, L);
    xv.load(W.Yt, L);
    f32x4_t out[F::NT];
    float gv[2 * F::EPL], hh[2 * F::EPL];
    F::apply(xk, dSop_v, out);
    product_rows<F>(out, gv);
    F::apply(xv, dSop_h, out);
    product_rows<F>(out, hh);
#pragma unroll
    for (int i = 0; i < 2 * F::EPL; ++i) gv[i] *= inv_r;
    project_rows_raw<F>(hh, xk, inv_r, L);
    if (row < rows.limit) {
      store_product_row<F, STREAM>(dK, row, src.row, L, hh);
      store_product_row<F, STREAM>(dV, row, src.row, L, gv);
    }
    wave_lds_fence();
  });
}

// ---- workgroup-level state handling ---------------------------------------------------------

// Sums the four per-wave accumulators in the fixed order (w0 + w1) + (w2 + w3): afterwards
// R0 + R1 (two fp32 images at the start of LDS, column-major with padded stride, so that the
// 4 consecutive state rows a register group holds move as one 128-bit access) is the total.
template <class F>
__device__ __forceinline__ void wg_reduce(const Lane& L, unsigned char* smem,
                                          const typename F::Acc& acc) {
  typedef typename F::Acc Acc;
  float* R = reinterpret_cast<float*>(smem) + (L.wave >> 1) * Layout<F>::kRFloats;
  f32x4_t* dst[Acc::kGroups];
#pragma unroll
  for (int g = 0; g < Acc::kGroups; ++g)
    dst[g] = reinterpret_cast<f32x4_t*>(R + Acc::group_col(g, L) * Layout<F>::kRStride +
                                        Acc::group_row(g, L));
  __syncthreads();  // working set no longer in use
  if ((L.wave & 1) == 0) {
#pragma unroll
    for (int g = 0; g < Acc::kGroups; ++g) *dst[g] = acc.group(g);
  }
  __syncthreads();
  if ((L.wave & 1) == 1) {
    f32x4_t other[Acc::kGroups];  // all reads first, so that they overlap
#pragma unroll
    for (int g = 0; g < Acc::kGroups; ++g) other[g] = *dst[g];
#pragma unroll
    for (int g = 0; g < Acc::kGroups; ++g) *dst[g] = other[g] + acc.group(g);
  }
  __syncthreads();
}

// Element (m, n) of a complete state held in LDS: either as the two reduction images
// R0 + R1 (column-major, padded), or as one row-major D x D array (after gather_partials).
template <class F>
struct StateSource {
  const float* lds;
  bool row_major;
  __device__ __forceinline__ float at(int m, int n) const {
    if (row_major) return lds[m * F::D + n];
    return lds[n * Layout<F>::kRStride + m] + lds[Layout<F>::kRFloats + n * Layout<F>::kRStride + m];
  }
};

// Split path: sums, in split order, the `splits` row-major partial states a slice has in
// global memory (written by an earlier kernel) into a row-major LDS array.  Every consumer
// workgroup repeats the same fixed-order sum, so there is no separate reduction launch and
// no cross-workgroup synchronisation.  Loads of four splits are kept in flight together.
template <class F>
__device__ __forceinline__ void gather_partials(const float* __restrict__ partials, int splits,
                                                float* dst) {
  constexpr int DD = F::D * F::D, kPer = DD / 4 / kThreads;  // 128-bit pieces per thread
  static_assert(kPer >= 1 && DD % (4 * kThreads) == 0, "state size");
  const f32x4_t* __restrict__ src = reinterpret_cast<const f32x4_t*>(partials);
  f32x4_t sum[kPer];
#pragma unroll
  for (int i = 0; i < kPer; ++i) sum[i] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  int p = 0;
  for (; p + 4 <= splits; p += 4) {
    f32x4_t v[4][kPer];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < kPer; ++i)
        v[q][i] = src[static_cast<size_t>(p + q) * (DD / 4) + threadIdx.x + i * kThreads];
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
      for (int i = 0; i < kPer; ++i) sum[i] += v[q][i];
  }
  for (; p < splits; ++p) {
    f32x4_t v[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i)
      v[i] = src[static_cast<size_t>(p) * (DD / 4) + threadIdx.x + i * kThreads];
#pragma unroll
    for (int i = 0; i < kPer; ++i) sum[i] += v[i];
  }
#pragma unroll
  for (int i = 0; i < kPer; ++i)
    reinterpret_cast<f32x4_t*>(dst)[threadIdx.x + i * kThreads] = sum[i];
}

// Builds operand images of scale * M for the apply products:
//   natural    op[m][n] = M[m][n]   (products contracting over n)
//   transposed op[n][m] = M[m][n]   (products contracting over m)
template <class F>
__device__ __forceinline__ void make_operands(const StateSource<F> src, float scale,
                                              unsigned char* natural, unsigned char* transposed) {
  constexpr int D = F::D;
  constexpr int kPer = D * D / 2 / kThreads;  // element pairs per thread
  // Thread -> element maps chosen so that consecutive lanes walk what is contiguous in the
  // source: state rows m in the column-major reduction images, state columns n in a gathered
  // row-major state (anything else lands all lanes of a wave in one LDS bank).
  if (natural != nullptr) {
    float lo[kPer], hi[kPer];
    int mm[kPer], nn[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads;
      mm[i] = src.row_major ? e / (D / 2) : e % D;
      nn[i] = src.row_major ? (e % (D / 2)) * 2 : (e / D) * 2;
      lo[i] = src.at(mm[i], nn[i]);
      hi[i] = src.at(mm[i], nn[i] + 1);
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i)
      F::write_image_pair(natural, mm[i], nn[i], lo[i] * scale, hi[i] * scale);
  }
  if (transposed != nullptr) {
    float lo[kPer], hi[kPer];
    int mm[kPer], nn[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads;
      mm[i] = src.row_major ? (e / D) * 2 : (e % (D / 2)) * 2;
      nn[i] = src.row_major ? e % D : e / (D / 2);
      lo[i] = src.at(mm[i], nn[i]);
      hi[i] = src.at(mm[i] + 1, nn[i]);
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i)
      F::write_image_pair(transposed, nn[i], mm[i], lo[i] * scale, hi[i] * scale);
  }
}

// ---- kernels ----------------------------------------------------------------------------------

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

// Arguments common to all kernels of this file (passed by value).
struct Args {
  const unsigned char* Q;
  const unsigned char* K;
  const unsigned char* V;
  const unsigned char* dO;
  const uint8_t* mask;
  unsigned char* O;
  unsigned char* dQ;
  unsigned char* dK;
  unsigned char* dV;
  // split path: partial states in the workspace, [B*H][splits][D*D] floats each
  float* s_partials;
  float* ds_partials;
  int H, N, splits;
  Strides st;
  float scale, eps;
  const float* scales;  // per-slice scale, or nullptr
  float* dlog;          // backward: sum_i dO_i . O_i per slice, or nullptr
};

__device__ __forceinline__ float slice_scale(const Args& a, int bh) {
  return a.scales != nullptr ? a.scales[bh] : a.scale;
}

// Sum of x over the workgroup in a fixed order (tree through `scratch`, kThreads floats of
// LDS not otherwise in use); every thread gets it.
__device__ __forceinline__ float block_sum(float x, float* scratch) {
  scratch[threadIdx.x] = x;
  __syncthreads();
  for (int w = kThreads / 2; w > 0; w >>= 1) {
    if (static_cast<int>(threadIdx.x) < w) scratch[threadIdx.x] += scratch[threadIdx.x + w];
    __syncthreads();
  }
  const float total = scratch[0];
  __syncthreads();
  return total;
}

// SHORT: at most 16 tiles (256 rows), every wave keeps all its tiles in registers (see Kept).
template <class F, bool SHORT>
__global__ __launch_bounds__(kThreads, 2) void fused_fwd_kernel(const Args a) {
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int bh = blockIdx.x, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  const int n_tiles = (N + TR - 1) / TR;
  uint8_t* kflags = a.mask != nullptr ? smem + Layout<F>::kFlags : nullptr;
  unsigned char* op0 = smem + Layout<F>::kImage0;
  const Rows keys{0, 1, n_tiles, N, kflags}, all{0, 1, n_tiles, N, nullptr};
  const Src q_src(a.Q + base, a.Q + base, N, a.st.row), kv_src(a.K + base, a.V + base, N, a.st.row);

  typename TilesOf<SHORT>::type qfirst, kfirst;
  // the query tiles do not depend on the mask: issue them right away
  load_tiles<false>(qfirst, L, q_src, all);
  if (kflags != nullptr) {
    fill_flags(kflags, a.mask + static_cast<size_t>(bh / a.H) * N, keys);
    __syncthreads();
  }
  load_tiles<true>(kfirst, L, kv_src, keys);

  typename F::Acc acc;
  acc.zero();
  state_pass<F, F::kDepthState>(L, W, kv_src, keys, a.eps, kfirst, acc);
  wg_reduce<F>(L, smem, acc);
  // O = qhat S: contraction over rows of S
  make_operands<F>(StateSource<F>{reinterpret_cast<const float*>(smem), false}, slice_scale(a, bh), nullptr,
                   op0);
  __syncthreads();
  typename F::Operand Sop;
  Sop.load(op0, L);
  fwd_apply_pass<F, F::kDepthFwd, true>(L, W, q_src, a.O + base, all, a.eps, qfirst, Sop);
}

template <class F, bool SHORT>
__global__ __launch_bounds__(kThreads, 2) void fused_bwd_kernel(const Args a) {
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int bh = blockIdx.x, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  const int n_tiles = (N + TR - 1) / TR;
  uint8_t* kflags = a.mask != nullptr ? smem + Layout<F>::kFlags : nullptr;
  unsigned char* op0 = smem + Layout<F>::kImage0;
  unsigned char* op1 = smem + Layout<F>::kImage1;
  const StateSource<F> reduced{reinterpret_cast<const float*>(smem), false};
  const Rows keys{0, 1, n_tiles, N, kflags}, all{0, 1, n_tiles, N, nullptr};
  const Src q_src(a.Q + base, a.dO + base, N, a.st.row), kv_src(a.K + base, a.V + base, N, a.st.row);

  COTTEN_TRACE_POINT(0);
  typename TilesOf<SHORT>::type qfirst, kfirst;
  load_tiles<true>(qfirst, L, q_src, all);
  if (kflags != nullptr) {
    fill_flags(kflags, a.mask + static_cast<size_t>(bh / a.H) * N, keys);
    __syncthreads();
  }
  COTTEN_TRACE_POINT(1);
  load_tiles<true>(kfirst, L, kv_src, keys);

  typename F::Acc acc;
  acc.zero();
  state_pass<F, F::kDepthState>(L, W, kv_src, keys, a.eps, kfirst, acc);
  COTTEN_TRACE_POINT(2);
  wg_reduce<F>(L, smem, acc);
  COTTEN_TRACE_POINT(3);
  const float scale = slice_scale(a, bh);
  make_operands<F>(reduced, scale, op0, nullptr);  // g = dO S^T: contraction over columns of S
  __syncthreads();
  acc.zero();
  COTTEN_TRACE_POINT(4);
  bwd_q_pass<F, true, F::kDepthQAccum, true>(L, W, q_src, a.dQ + base, all, a.eps,
                                       qfirst, op0, acc);
  COTTEN_TRACE_POINT(5);
  // the key/value tiles are walked again: get the first one moving before the reduction
  // (nothing to do when they were kept)
  reload_tiles<true>(kfirst, L, kv_src, keys);
  wg_reduce<F>(L, smem, acc);
  COTTEN_TRACE_POINT(6);
  if (a.dlog != nullptr) {
    // sum_i dO_i . O_i = <scale * S, sum_i qhat_i^T dO_i>: the S image against the sum just
    // reduced, before that image is replaced (image 1 is free and serves as scratch)
    float part = 0.0f;
    for (int e = threadIdx.x; e < F::D * F::D; e += kThreads)
      part += F::image_at(op0, e % F::D, e / F::D) * reduced.at(e % F::D, e / F::D);
    part = block_sum(part, reinterpret_cast<float*>(op1));
    if (threadIdx.x == 0) a.dlog[bh] = part;
  }
  make_operands<F>(reduced, scale, op0, op1);  // op0 = dS natural, op1 = dS transposed
  __syncthreads();
  typename F::Operand dS_v, dS_h;
  dS_v.load(op1, L);  // dV = khat dS: contraction over rows of dS
  dS_h.load(op0, L);  // h = v dS^T: contraction over columns of dS
  COTTEN_TRACE_POINT(7);
  bwd_kv_pass<F, F::kDepthKV, true>(L, W, kv_src, a.dK + base, a.dV + base, keys, a.eps,
                              kfirst, dS_v, dS_h);
  COTTEN_TRACE_POINT(8);
}

// The tiles of slice bh dealt to workgroup `split` of `splits`.
__device__ __forceinline__ Rows split_rows(int N, int split, int splits, const uint8_t* flags) {
  const int total = (N + TR - 1) / TR;
  const int mine = split < total ? (total - split + splits - 1) / splits : 0;
  return Rows{split, splits, mine, N, flags};
}

// Split path: the workgroup's partial state (R0 + R1 in LDS) goes to its slot in global memory.
template <class F>
__device__ __forceinline__ void publish_partial(float* partials, int bh, int split, int splits) {
  constexpr int DD = F::D * F::D;
  const StateSource<F> mine{reinterpret_cast<const float*>(smem), false};
  float* out = partials + (static_cast<size_t>(bh) * splits + split) * DD;
  for (int e = threadIdx.x; e < DD; e += kThreads) out[e] = mine.at(e / F::D, e % F::D);
}

// Split path, step 1 (both directions): partial S of this workgroup's (K,V) tiles.
template <class F>
__global__ __launch_bounds__(kThreads, 2) void split_state_kernel(const Args a) {
  constexpr int DD = F::D * F::D;
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int split = blockIdx.x % a.splits, bh = blockIdx.x / a.splits, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  COTTEN_TRACE_POINT(0);
  uint8_t* flags = a.mask != nullptr ? smem + Layout<F>::kFlags : nullptr;
  const Rows rows = split_rows(N, split, a.splits, flags);
  const Src src(a.K + base, a.V + base, N, a.st.row);
  if (flags != nullptr) {
    fill_flags(flags, a.mask + static_cast<size_t>(bh / a.H) * N, rows);
    __syncthreads();
  }
  COTTEN_TRACE_POINT(1);
  Raw first;
  load_first<true>(first, L, src, rows);
  typename F::Acc acc;
  acc.zero();
  state_pass<F, F::kDepthState>(L, W, src, rows, a.eps, first, acc);
  COTTEN_TRACE_POINT(2);
  wg_reduce<F>(L, smem, acc);
  COTTEN_TRACE_POINT(3);
  publish_partial<F>(a.s_partials, bh, split, a.splits);
  COTTEN_TRACE_POINT(4);
}

template <class F>
__global__ __launch_bounds__(kThreads, 2) void split_apply_fwd_kernel(const Args a) {
  constexpr int D = F::D;
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int split = blockIdx.x % a.splits, bh = blockIdx.x / a.splits, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* op0 = smem + Layout<F>::kImage0;
  const Rows all = split_rows(N, split, a.splits, nullptr);
  const Src q_src(a.Q + base, a.Q + base, N, a.st.row);
  Raw first;
  load_first<false>(first, L, q_src, all);
  float* gathered = reinterpret_cast<float*>(smem);
  gather_partials<F>(a.s_partials + static_cast<size_t>(bh) * a.splits * D * D, a.splits, gathered);
  __syncthreads();
  make_operands<F>(StateSource<F>{gathered, true}, slice_scale(a, bh), nullptr, op0);
  __syncthreads();
  typename F::Operand Sop;
  Sop.load(op0, L);
  fwd_apply_pass<F, F::kDepthFwd, kSplitStream>(L, W, q_src, a.O + base, all, a.eps, first, Sop);
}

// Backward, step 2: one pass over this workgroup's (Q,dO) tiles writes dQ (S is complete)
// and accumulates the partial dS.
template <class F>
__global__ __launch_bounds__(kThreads, 2) void split_q_kernel(const Args a) {
  constexpr int DD = F::D * F::D;
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int split = blockIdx.x % a.splits, bh = blockIdx.x / a.splits, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* op0 = smem + Layout<F>::kImage0;
  const Rows all = split_rows(N, split, a.splits, nullptr);
  const Src q_src(a.Q + base, a.dO + base, N, a.st.row);
  COTTEN_TRACE_POINT(0);
  Raw first;
  load_first<true>(first, L, q_src, all);
  float* gathered = reinterpret_cast<float*>(smem);
  gather_partials<F>(a.s_partials + static_cast<size_t>(bh) * a.splits * DD, a.splits, gathered);
  __syncthreads();
  COTTEN_TRACE_POINT(1);
  make_operands<F>(StateSource<F>{gathered, true}, slice_scale(a, bh), op0, nullptr);
  __syncthreads();
  COTTEN_TRACE_POINT(2);
  typename F::Acc acc;
  acc.zero();
  bwd_q_pass<F, true, F::kDepthQAccum, kSplitStream>(L, W, q_src, a.dQ + base, all, a.eps, first, op0, acc);
  COTTEN_TRACE_POINT(3);
  wg_reduce<F>(L, smem, acc);
  COTTEN_TRACE_POINT(4);
  publish_partial<F>(a.ds_partials, bh, split, a.splits);
  COTTEN_TRACE_POINT(5);
}

// Backward, step 3: dK, dV of this workgroup's (K,V) tiles from the complete dS.
template <class F>
__global__ __launch_bounds__(kThreads, 2) void split_kv_kernel(const Args a) {
  constexpr int DD = F::D * F::D;
  const Lane L;
  const WaveLds<F> W(smem, L.wave);
  const int split = blockIdx.x % a.splits, bh = blockIdx.x / a.splits, N = a.N;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* op0 = smem + Layout<F>::kImage0;
  unsigned char* op1 = smem + Layout<F>::kImage1;
  uint8_t* flags = a.mask != nullptr ? smem + Layout<F>::kFlags : nullptr;
  const Rows keys = split_rows(N, split, a.splits, flags);
  const Src kv_src(a.K + base, a.V + base, N, a.st.row);
  if (flags != nullptr) fill_flags(flags, a.mask + static_cast<size_t>(bh / a.H) * N, keys);
  float* gathered = reinterpret_cast<float*>(smem);
  gather_partials<F>(a.ds_partials + static_cast<size_t>(bh) * a.splits * DD, a.splits, gathered);
  __syncthreads();
  const float scale = slice_scale(a, bh);
  if (a.dlog != nullptr && split == 0) {
    // sum_i dO_i . O_i = scale * <S, sum_i qhat_i^T dO_i>: the first workgroup of the slice
    // sums the partial S once more (image 1 is free and serves as scratch)
    float* s_total = gathered + DD;
    gather_partials<F>(a.s_partials + static_cast<size_t>(bh) * a.splits * DD, a.splits, s_total);
    __syncthreads();
    float part = 0.0f;
    for (int e = threadIdx.x; e < DD; e += kThreads) part += s_total[e] * gathered[e];
    part = block_sum(part, reinterpret_cast<float*>(op1));
    if (threadIdx.x == 0) a.dlog[bh] = scale * part;
  }
  make_operands<F>(StateSource<F>{gathered, true}, scale, op0, op1);
  __syncthreads();
  Raw first;
  load_first<true>(first, L, kv_src, keys);
  typename F::Operand dS_v, dS_h;
  dS_v.load(op1, L);
  dS_h.load(op0, L);
  bwd_kv_pass<F, F::kDepthKV, kSplitStream>(L, W, kv_src, a.dK + base, a.dV + base, keys, a.eps, first, dS_v,
                              dS_h);
}

// ---- host side ----------------------------------------------------------------------------------

// Dynamic LDS above 64 KB has to be granted per kernel first; two workgroups share a
// compute unit's 160 KB.
constexpr int kMaxLdsBytes = 80 * 1024;
template <typename Kern>
hipError_t allow_lds(Kern kern, size_t bytes) {
  if (bytes > static_cast<size_t>(kMaxLdsBytes)) return hipErrorInvalidValue;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
}

template <class F>
size_t lds_bytes(int flag_rows) {
  return static_cast<size_t>(Layout<F>::kFlags) + static_cast<size_t>(flag_rows) + 16;
}

Args make_args(const Problem& p, const Plan& plan, int D) {
  Args a{};
  a.Q = static_cast<const unsigned char*>(p.Q);
  a.K = static_cast<const unsigned char*>(p.K);
  a.V = static_cast<const unsigned char*>(p.V);
  a.dO = static_cast<const unsigned char*>(p.dO);
  a.mask = p.mask;
  a.O = static_cast<unsigned char*>(p.O);
  a.dQ = static_cast<unsigned char*>(p.dQ);
  a.dK = static_cast<unsigned char*>(p.dK);
  a.dV = static_cast<unsigned char*>(p.dV);
  if (plan.path == Plan::kSplit) {
    a.s_partials = p.workspace;
    a.ds_partials = p.workspace + static_cast<size_t>(p.B) * p.H * plan.splits * D * D;
  }
  a.H = p.H;
  a.N = p.N;
  a.splits = plan.splits;
  a.st = Strides{p.stride_batch * p.elem_bytes(), p.stride_head * p.elem_bytes(),
                 RowAddr{static_cast<int>(p.stride_row * p.elem_bytes()),
                         static_cast<int>(p.D * p.elem_bytes())}};
  a.scale = p.scale;
  a.eps = p.eps;
  a.scales = p.slice_scale;
  a.dlog = p.dlog_scale;
  return a;
}

// Short fp32 sequences use the kernels that keep every tile in registers (the 16-bit formats
// of that length are served by the resident kernels, and would not have the registers).
template <class F>
bool keeps_tiles(int N) {
  return F::kShortKernels && (N + TR - 1) / TR <= Kept::kTiles * kWaves;
}

template <class F>
hipError_t run_fwd(const Problem& p, const Plan& plan) {
  const Args a = make_args(p, plan, F::D);
  const unsigned BH = static_cast<unsigned>(p.B) * p.H;
  hipError_t err;
  if (plan.path == Plan::kFused) {
    const size_t lds = lds_bytes<F>((p.N + TR - 1) / TR * TR);
    if (keeps_tiles<F>(p.N)) {
      if ((err = allow_lds(fused_fwd_kernel<F, F::kShortKernels>, lds)) != hipSuccess) return err;
      hipLaunchKernelGGL((fused_fwd_kernel<F, F::kShortKernels>), dim3(BH), dim3(kThreads), lds,
                         p.stream, a);
    } else {
      if ((err = allow_lds(fused_fwd_kernel<F, false>, lds)) != hipSuccess) return err;
      hipLaunchKernelGGL((fused_fwd_kernel<F, false>), dim3(BH), dim3(kThreads), lds, p.stream, a);
    }
    return hipGetLastError();
  }
  const size_t lds = lds_bytes<F>(plan.rows_per_split);
  if ((err = allow_lds(split_state_kernel<F>, lds)) != hipSuccess) return err;
  if ((err = allow_lds(split_apply_fwd_kernel<F>, lds)) != hipSuccess) return err;
  const dim3 grid(BH * plan.splits, 1, 1);
  hipLaunchKernelGGL(split_state_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  hipLaunchKernelGGL(split_apply_fwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  return hipGetLastError();
}

template <class F>
hipError_t run_bwd(const Problem& p, const Plan& plan) {
  const Args a = make_args(p, plan, F::D);
  const unsigned BH = static_cast<unsigned>(p.B) * p.H;
  hipError_t err;
  if (plan.path == Plan::kFused) {
    const size_t lds = lds_bytes<F>((p.N + TR - 1) / TR * TR);
    if (keeps_tiles<F>(p.N)) {
      if ((err = allow_lds(fused_bwd_kernel<F, F::kShortKernels>, lds)) != hipSuccess) return err;
      hipLaunchKernelGGL((fused_bwd_kernel<F, F::kShortKernels>), dim3(BH), dim3(kThreads), lds,
                         p.stream, a);
    } else {
      if ((err = allow_lds(fused_bwd_kernel<F, false>, lds)) != hipSuccess) return err;
      hipLaunchKernelGGL((fused_bwd_kernel<F, false>), dim3(BH), dim3(kThreads), lds, p.stream, a);
    }
    return hipGetLastError();
  }
  const size_t lds = lds_bytes<F>(plan.rows_per_split);
  if ((err = allow_lds(split_state_kernel<F>, lds)) != hipSuccess) return err;
  if ((err = allow_lds(split_q_kernel<F>, lds)) != hipSuccess) return err;
  if ((err = allow_lds(split_kv_kernel<F>, lds)) != hipSuccess) return err;
  const dim3 grid(BH * plan.splits, 1, 1);
  hipLaunchKernelGGL(split_state_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  hipLaunchKernelGGL(split_q_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  hipLaunchKernelGGL(split_kv_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  return hipGetLastError();
}

}  // namespace

// Full-width rows (128 bytes) and narrower rows (64 or 32 bytes, run zero-padded on the same
// formats).
bool mfma_supports(int dtype, int D) {
  return dtype == 0 ? (D == 32 || D == 16) : (D == 64 || D == 32 || D == 16);
}

int mfma_state_dim(int dtype) { return dtype == 0 ? F32x32::D : Bf16x64::D; }

hipError_t launch_mfma_fwd(const Problem& p, const Plan& plan) {
  return p.dtype == 1   ? run_fwd<Bf16x64>(p, plan)
         : p.dtype == 2 ? run_fwd<F16x64>(p, plan)
                        : run_fwd<F32x32>(p, plan);
}

hipError_t launch_mfma_bwd(const Problem& p, const Plan& plan) {
  return p.dtype == 1   ? run_bwd<Bf16x64>(p, plan)
         : p.dtype == 2 ? run_bwd<F16x64>(p, plan)
                        : run_bwd<F32x32>(p, plan);
}

}  // namespace cotten
