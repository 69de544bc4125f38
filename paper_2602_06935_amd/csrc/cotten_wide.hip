// Matrix-core kernels for 256-byte rows: fp32 I/O with d_h = 64, bf16 / fp16 I/O with d_h = 128
// (d_model = 128 or 256 with two heads, "Sequence Length and Embedding Size").
//
// A 256-byte row is handled as two 128-byte halves, a d_h x d_h state as four quadrants of
// the size the 128-byte-row formats work on (cotten_mfma_core.h), so that their tile layout,
// MFMA products, operand images and row epilogues serve unchanged:
//
//     S[p][q] = sum_j khat_j[half p]^T v_j[half q]           (state kernel)
//     O[half q] = sum_p Qhat[half p] S[p][q]                 (apply kernels; likewise dQ, dK, dV)
//
// with the row norm taken over both halves.  The launch structure is that of the vector-ALU
// path whose place these kernels take for the shapes above (same plan, same workspace):
//
//   wide_state_kernel   a workgroup of four (or eight) waves reduces a block of rows of one slice
//                       to a partial state: per round every wave stages one 16-row tile in LDS,
//                       then wave (p, q) adds four tiles of the round to its quadrant (with eight
//                       waves two waves share a quadrant and their sums meet at the end)
//   (the partial states of a slice are summed in split order by the reduction kernel of the
//    vector-ALU path)
//   wide_fwd_kernel / wide_bwd_kernel
//                       a workgroup builds the operand images of the state it needs from the
//                       reduced state, then every wave streams 16-row tiles through a private
//                       LDS tile set: products per quadrant, epilogue per half row, 128-bit
//                       stores.  The backward runs dQ, dV and dK as three roles of one launch
//                       (blockIdx.y), each with the one set of images it needs.
#include "cotten_launch.h"
#include "cotten_mfma_core.h"

namespace cotten {
namespace {
namespace wide {

using namespace mfma;

// Every kernel exists for workgroups of 4 and of 8 waves (template parameter WAVES): 4 when there
// are workgroups enough to put two on every compute unit, 8 when there are not.
constexpr int kHalfBytes = kRowBytes;    // one half of a 256-byte row

// A 16-row tile of a tensor pair in the load layout: piece [h][c] is bytes 128 c + 16 ch .. + 15 of
// row r8 + 8 h.  `live` bit h: the row takes part.
struct WideRaw {
  u32x4_t x[2][2], y[2][2];
  int live;
};

// The two tensors of a pass as buffer resources over one slice (see Src in cotten_mfma_core.h:
// lanes whose row does not take part get zeros and cause no traffic).
struct WideSrc {
  __amdgpu_buffer_rsrc_t x, y;
  int stride;
  __device__ __forceinline__ WideSrc(const unsigned char* X, const unsigned char* Y, int N, int stride_bytes)
      : stride(stride_bytes) {
    const int bytes = (N - 1) * stride + 2 * kHalfBytes;
    x = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(X), 0, bytes, 0x00020000);
    y = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(Y), 0, bytes, 0x00020000);
  }
};

// Bit h: row row0 + r8 + 8 h is below `limit` and, if a mask is given, a valid key.
__device__ __forceinline__ int row_bits(const uint8_t* __restrict__ mask, int row0, int limit,
                                        const Lane& L) {
  int bits = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = row0 + L.r8 + 8 * h;
    if (row < limit) bits |= static_cast<int>(mask == nullptr || mask[row] != 0) << h;
  }
  return bits;
}

template <bool USE_Y>
__device__ __forceinline__ void load_wide(WideRaw& r, const Lane& L, const WideSrc& src, int row0,
                                          int bits) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const bool live = ((bits >> h) & 1) != 0;
    const uint32_t off =
        live ? static_cast<uint32_t>(row0 + L.r8 + 8 * h) * src.stride + L.ch * 16 : kOutOfBuffer;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      r.x[h][c] = __builtin_amdgcn_raw_buffer_load_b128(src.x, off + c * kHalfBytes, 0, 0);
      if (USE_Y) r.y[h][c] = __builtin_amdgcn_raw_buffer_load_b128(src.y, off + c * kHalfBytes, 0, 0);
      else r.y[h][c] = u32x4_t{0, 0, 0, 0};
    }
  }
  r.live = bits;
}

// The tile into LDS as four 16 x 128-byte tiles [x half 0 | x half 1 | y half 0 | y half 1]
// (each in the layout of cotten_mfma_core.h); x normalised over the whole row, or raw.
// inv[h] = 1/r of row r8 + 8 h (0 for a row that does not take part).
template <class F, bool NORMALIZE, bool USE_Y>
__device__ __forceinline__ void stage_wide(const WideRaw& r, const Lane& L, float eps,
                                           unsigned char* tiles, float (&inv)[2]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float f[2][F::EPL];
    float ss = 0.0f;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      F::unpack(r.x[h][c], f[c]);
#pragma unroll
      for (int i = 0; i < F::EPL; ++i) ss += f[c][i] * f[c][i];
    }
    inv[h] = inv_norm_or_zero(row_sum8(ss), eps, (r.live >> h) & 1);
    const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      if (NORMALIZE) {
#pragma unroll
        for (int i = 0; i < F::EPL; ++i) f[c][i] *= inv[h];
        *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = F::pack(f[c]);
      } else {
        *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = r.x[h][c];
      }
      if (USE_Y) *reinterpret_cast<u32x4_t*>(tiles + (2 + c) * kTileBytes + off) = r.y[h][c];
    }
  }
}

// 1/r of the tile's rows from the load layout to the product layout, through 16 floats of LDS.
__device__ __forceinline__ float inv_by_row(float* slot, const Lane& L, const float (&inv)[2]) {
  if (L.ch == 0) {
    slot[L.r8] = inv[0];
    slot[L.r8 + 8] = inv[1];
  }
  wave_lds_fence();
  return slot[L.i16];
}

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

// ---- state kernel -------------------------------------------------------------------------------

// grid (slices * splits, 1 or 2): blockIdx.y == 1 reduces (Q, dO) to sum_i qhat_i^T dO_i instead
// of (K, V) under the key mask.  Partial states: row-major D x D floats per workgroup, the second
// kind `second_offset` floats behind the first (the layout of the vector-ALU path).
template <class F, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void wide_state_kernel(
    const unsigned char* __restrict__ Q, const unsigned char* __restrict__ K,
    const unsigned char* __restrict__ V, const unsigned char* __restrict__ dO,
    const uint8_t* __restrict__ mask, float* __restrict__ ws, int H, int N, int splits,
    int rows_per_split, size_t second_offset, float eps, Strides st) {
  constexpr int Dh = F::D, D = 2 * Dh, kRoundRows = WAVES * TR;
  static_assert(WAVES == 4 || WAVES == 8, "one or two waves per quadrant");
  unsigned char* round = smem;  // WAVES x [x half 0 | x half 1 | y half 0 | y half 1]
  const Lane L;
  const int split = blockIdx.x % splits, bh = blockIdx.x / splits;
  const bool second = blockIdx.y == 1;
  const size_t base = st.slice_base(bh, H);
  const WideSrc src((second ? Q : K) + base, (second ? dO : V) + base, N, st.row.stride);
  const uint8_t* __restrict__ m =
      (second || mask == nullptr) ? nullptr : mask + static_cast<size_t>(bh / H) * N;
  const int r_begin = split * rows_per_split;
  const int r_end = N < r_begin + rows_per_split ? N : r_begin + rows_per_split;
  // this wave's quadrant of the state, and (8 waves) which four tiles of a round it adds up
  const int quadrant = L.wave & 3, p = quadrant >> 1, q = quadrant & 1, part = L.wave >> 2;
  unsigned char* mine = round + L.wave * 4 * kTileBytes;

  typename F::Acc acc;
  acc.zero();
  WideRaw cur;
  load_wide<true>(cur, L, src, r_begin + L.wave * TR, row_bits(m, r_begin + L.wave * TR, r_end, L));
  int next_bits = row_bits(m, r_begin + kRoundRows + L.wave * TR, r_end, L);
  for (int r0 = r_begin; r0 < r_end; r0 += kRoundRows) {
    float inv[2];
    stage_wide<F, true, true>(cur, L, eps, mine, inv);
    // the wave's tile of the next round travels while this round is added up
    load_wide<true>(cur, L, src, r0 + kRoundRows + L.wave * TR, next_bits);
    next_bits = row_bits(m, r0 + 2 * kRoundRows + L.wave * TR, r_end, L);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const unsigned char* tile = round + (4 * part + t) * 4 * kTileBytes;
      acc.mfma(tile + p * kTileBytes, tile + (2 + q) * kTileBytes, L);
    }
    __syncthreads();  // the round's tiles are overwritten next
  }
  // 8 waves: the two sums of a quadrant meet in LDS (the round buffer is free), in a fixed order
  f32x4_t* meet = reinterpret_cast<f32x4_t*>(round) + quadrant * F::Acc::kGroups * 64 + L.lane;
  static_assert(4 * F::Acc::kGroups * 64 * 16 <= 8 * 4 * kTileBytes, "the sums fit the round buffer");
  if (WAVES == 8) {
    if (part == 1) {
#pragma unroll
      for (int g = 0; g < F::Acc::kGroups; ++g) meet[g * 64] = acc.group(g);
    }
    __syncthreads();
    if (part == 1) return;
  }
  float* __restrict__ out =
      ws + (second ? second_offset : 0) + static_cast<size_t>(blockIdx.x) * D * D;
#pragma unroll
  for (int g = 0; g < F::Acc::kGroups; ++g) {
    f32x4_t v = acc.group(g);
    if (WAVES == 8) v += meet[g * 64];
    const int row = p * Dh + F::Acc::group_row(g, L), col = q * Dh + F::Acc::group_col(g, L);
#pragma unroll
    for (int i = 0; i < 4; ++i) out[(row + i) * D + col] = v[i];
  }
}

// ---- operand images --------------------------------------------------------------------------------

// The four quadrant images of scale * M (M: a reduced state in global memory, row-major D x D),
// image (p, q) at images + (2 p + q) * F::kImageBytes:
//   natural     op[m][n] = M[p Dh + m][q Dh + n]     for products that contract over n
//   transposed  op[n][m] = M[p Dh + m][q Dh + n]     for products that contract over m
template <class F, int WAVES, bool TRANSPOSED>
__device__ __forceinline__ void build_images(const float* __restrict__ M, float scale,
                                             unsigned char* images) {
  constexpr int Dh = F::D, D = 2 * Dh, kThreads = 64 * WAVES;
  // element pairs; the loads of a batch travel together
  constexpr int kPairs = D * D / 2, kBatch = kPairs / kThreads < 8 ? kPairs / kThreads : 8;
  static_assert(kBatch >= 1 && kPairs % (kBatch * kThreads) == 0, "state size");
  for (int e0 = threadIdx.x; e0 < kPairs; e0 += kBatch * kThreads) {
    float v0[kBatch], v1[kBatch];
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int e = e0 + j * kThreads;
      if (TRANSPOSED) {  // the pair (m, m + 1) of column n: consecutive threads take consecutive n
        const int m = 2 * (e / D), n = e % D;
        v0[j] = M[m * D + n];
        v1[j] = M[(m + 1) * D + n];
      } else {           // the pair (n, n + 1) of row m
        const int m = e / (D / 2), n = 2 * (e % (D / 2));
        const float2 v = *reinterpret_cast<const float2*>(M + m * D + n);
        v0[j] = v.x;
        v1[j] = v.y;
      }
    }
#pragma unroll
    for (int j = 0; j < kBatch; ++j) {
      const int e = e0 + j * kThreads;
      const int m = TRANSPOSED ? 2 * (e / D) : e / (D / 2);
      const int n = TRANSPOSED ? e % D : 2 * (e % (D / 2));
      unsigned char* image = images + (2 * (m / Dh) + n / Dh) * F::kImageBytes;
      if (TRANSPOSED) F::write_image_pair(image, n % Dh, m % Dh, v0[j] * scale, v1[j] * scale);
      else F::write_image_pair(image, m % Dh, n % Dh, v0[j] * scale, v1[j] * scale);
    }
  }
}

// The four quadrant operands of a role: held in registers for all the tiles of the wave (HOLD:
// 4 x 32 registers for the 16-bit formats), or fetched from the images for every product (the
// backward roles share one kernel and do better at two waves per SIMD than with the operands
// held at one).
template <class F, bool HOLD>
struct Quadrants {
  typename F::Operand held[HOLD ? 4 : 1];
  const unsigned char* images;
  __device__ __forceinline__ Quadrants(const unsigned char* img, const Lane& L) : images(img) {
    if (HOLD) {
#pragma unroll
      for (int i = 0; i < 4; ++i) held[i].load(images + i * F::kImageBytes, L);
    }
  }
  // out = X[half 0] W(i0) + X[half 1] W(i1), images numbered 2 p + q
  __device__ __forceinline__ void apply(const typename F::TileRows (&X)[2], int i0, int i1,
                                        const Lane& L, float (&out)[2 * F::EPL]) const {
    f32x4_t a[F::NT], b[F::NT];
    if (HOLD) {
      F::apply(X[0], held[i0], a);
      F::apply(X[1], held[i1], b);
    } else {
      typename F::Operand W;
      W.load(images + i0 * F::kImageBytes, L);
      F::apply(X[0], W, a);
      W.load(images + i1 * F::kImageBytes, L);
      F::apply(X[1], W, b);
    }
#pragma unroll
    for (int nt = 0; nt < F::NT; ++nt) a[nt] += b[nt];
    product_rows<F>(a, out);
  }
};

// ---- apply roles ------------------------------------------------------------------------------------

struct ApplyArgs {
  const unsigned char* X;   // Q or K
  const unsigned char* Y;   // dO or V (projected role), unused otherwise
  const uint8_t* mask;      // key mask of the slice's batch row, or nullptr
  const float* state;       // reduced state of the slice, row-major D x D
  unsigned char* out;       // O, dQ, dK or dV
  int N, r_begin, r_end, stride;
  float scale, eps;
};

// LDS of the apply kernels: [four images][per wave: four tiles, 16 floats]
template <class F, int WAVES>
struct ApplyLds {
  static constexpr int kImages = 0;
  static constexpr int kWave = 4 * F::kImageBytes;
  static constexpr int kWaveBytes = 4 * kTileBytes + TR * 4;
  static constexpr int kBytes = kWave + WAVES * kWaveBytes;
};

// out rows = (x rows) M / r, contraction over the rows of M:  O = scale qhat S,  dV = scale khat dS.
template <class F, int WAVES, bool HOLD>
__device__ __forceinline__ void plain_role(const ApplyArgs& a) {
  constexpr int kRoundRows = WAVES * TR;  // rows between two tiles of a wave
  const Lane L;
  unsigned char* images = smem + ApplyLds<F, WAVES>::kImages;
  unsigned char* tiles = smem + ApplyLds<F, WAVES>::kWave + L.wave * ApplyLds<F, WAVES>::kWaveBytes;
  float* inv_slot = reinterpret_cast<float*>(tiles + 4 * kTileBytes);
  build_images<F, WAVES, true>(a.state, a.scale, images);
  __syncthreads();
  const Quadrants<F, HOLD> W(images, L);
  const WideSrc src(a.X, a.X, a.N, a.stride);
  int row0 = a.r_begin + L.wave * TR;
  WideRaw cur;
  load_wide<false>(cur, L, src, row0, row_bits(a.mask, row0, a.r_end, L));
  int next_bits = row_bits(a.mask, row0 + kRoundRows, a.r_end, L);
  for (; row0 < a.r_end; row0 += kRoundRows) {
    float inv[2];
    stage_wide<F, false, false>(cur, L, a.eps, tiles, inv);
    load_wide<false>(cur, L, src, row0 + kRoundRows, next_bits);
    next_bits = row_bits(a.mask, row0 + 2 * kRoundRows, a.r_end, L);
    const float inv_r = inv_by_row(inv_slot, L, inv);
    typename F::TileRows X[2];
    X[0].load(tiles, L);
    X[1].load(tiles + kTileBytes, L);
    const int row = row0 + L.i16;
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      float o[2 * F::EPL];
      W.apply(X, q, 2 + q, L, o);
#pragma unroll
      for (int i = 0; i < 2 * F::EPL; ++i) o[i] *= inv_r;
      if (row < a.r_end)
        store_product_row<F, kStoreStreamed>(a.out + q * kHalfBytes, row, RowAddr{a.stride, kHalfBytes}, L, o);
    }
    wave_lds_fence();
  }
}

// out rows = (g - xhat (xhat . g)) / r with g = (y rows) M^T, contraction over the columns of M:
//   dQ from (Q, dO) and scale S;   dK from (K, V) and scale dS (masked rows come out as zeros).
template <class F, int WAVES>
__device__ __forceinline__ void projected_role(const ApplyArgs& a) {
  constexpr int kRoundRows = WAVES * TR;
  const Lane L;
  unsigned char* images = smem + ApplyLds<F, WAVES>::kImages;
  unsigned char* tiles = smem + ApplyLds<F, WAVES>::kWave + L.wave * ApplyLds<F, WAVES>::kWaveBytes;
  float* inv_slot = reinterpret_cast<float*>(tiles + 4 * kTileBytes);
  build_images<F, WAVES, false>(a.state, a.scale, images);
  __syncthreads();
  const Quadrants<F, false> W(images, L);
  const WideSrc src(a.X, a.Y, a.N, a.stride);
  int row0 = a.r_begin + L.wave * TR;
  WideRaw cur;
  load_wide<true>(cur, L, src, row0, row_bits(a.mask, row0, a.r_end, L));
  int next_bits = row_bits(a.mask, row0 + kRoundRows, a.r_end, L);
  for (; row0 < a.r_end; row0 += kRoundRows) {
    float inv[2];
    stage_wide<F, true, true>(cur, L, a.eps, tiles, inv);
    load_wide<true>(cur, L, src, row0 + kRoundRows, next_bits);
    next_bits = row_bits(a.mask, row0 + 2 * kRoundRows, a.r_end, L);
    const float inv_r = inv_by_row(inv_slot, L, inv);
    typename F::TileRows Y[2], E[2];
    Y[0].load(tiles + 2 * kTileBytes, L);
    Y[1].load(tiles + 3 * kTileBytes, L);
    float g[2][2 * F::EPL];
#pragma unroll
    for (int p = 0; p < 2; ++p)
      W.apply(Y, 2 * p, 2 * p + 1, L, g[p]);
    E[0].load(tiles, L);
    E[1].load(tiles + kTileBytes, L);
    float proj = 0.0f;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      float u[2 * F::EPL];
      E[p].unpack(u);
#pragma unroll
      for (int c = 0; c < 2 * F::EPL; ++c) proj += u[c] * g[p][c];
      E[p].forget_unpacked();
    }
    proj = row_sum_groups(proj, L);
    const int row = row0 + L.i16;
#pragma unroll
    for (int p = 0; p < 2; ++p) {
      float u[2 * F::EPL];
      E[p].unpack(u);
#pragma unroll
      for (int c = 0; c < 2 * F::EPL; ++c) g[p][c] = (g[p][c] - u[c] * proj) * inv_r;
      if (row < a.r_end)
        store_product_row<F, kStoreStreamed>(a.out + p * kHalfBytes, row, RowAddr{a.stride, kHalfBytes}, L, g[p]);
    }
    wave_lds_fence();
  }
}

struct LaunchArgs {
  const unsigned char* Q;
  const unsigned char* K;
  const unsigned char* V;
  const unsigned char* dO;
  const uint8_t* mask;
  const float* states;   // reduced S of every slice
  const float* dstates;  // reduced sum_i qhat_i^T dO_i of every slice (backward)
  unsigned char* O;
  unsigned char* dQ;
  unsigned char* dK;
  unsigned char* dV;
  int H, N, splits, rows_per_split;
  float scale, eps;
  const float* slice_scale;
  Strides st;
};

__device__ __forceinline__ ApplyArgs role_args(const LaunchArgs& a, int dd) {
  ApplyArgs r{};
  const int split = blockIdx.x % a.splits, bh = blockIdx.x / a.splits;
  r.N = a.N;
  r.r_begin = split * a.rows_per_split;
  r.r_end = a.N < r.r_begin + a.rows_per_split ? a.N : r.r_begin + a.rows_per_split;
  r.stride = a.st.row.stride;
  r.scale = a.slice_scale != nullptr ? a.slice_scale[bh] : a.scale;
  r.eps = a.eps;
  return r;
}

template <class F, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void wide_fwd_kernel(const LaunchArgs a) {
  constexpr int D = 2 * F::D;
  const int bh = blockIdx.x / a.splits;
  const size_t base = a.st.slice_base(bh, a.H);
  ApplyArgs r = role_args(a, D * D);
  r.X = a.Q + base;
  r.mask = nullptr;  // queries are not masked
  r.state = a.states + static_cast<size_t>(bh) * D * D;
  r.out = a.O + base;
  plain_role<F, WAVES, true>(r);
}

// blockIdx.y: 0 dQ, 1 dV, 2 dK
template <class F, int WAVES>
__global__ __launch_bounds__(64 * WAVES) void wide_bwd_kernel(const LaunchArgs a) {
  constexpr int D = 2 * F::D;
  const int bh = blockIdx.x / a.splits;
  const size_t base = a.st.slice_base(bh, a.H);
  ApplyArgs r = role_args(a, D * D);
  const uint8_t* keys = a.mask == nullptr ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
  if (blockIdx.y == 0) {
    r.X = a.Q + base;
    r.Y = a.dO + base;
    r.mask = nullptr;
    r.state = a.states + static_cast<size_t>(bh) * D * D;
    r.out = a.dQ + base;
    projected_role<F, WAVES>(r);
  } else if (blockIdx.y == 1) {
    r.X = a.K + base;
    r.mask = keys;
    r.state = a.dstates + static_cast<size_t>(bh) * D * D;
    r.out = a.dV + base;
    plain_role<F, WAVES, false>(r);
  } else {
    r.X = a.K + base;
    r.Y = a.V + base;
    r.mask = keys;
    r.state = a.dstates + static_cast<size_t>(bh) * D * D;
    r.out = a.dK + base;
    projected_role<F, WAVES>(r);
  }
}

// ---- host side ------------------------------------------------------------------------------------

Strides byte_strides(const Problem& p) {
  return Strides{p.stride_batch * p.elem_bytes(), p.stride_head * p.elem_bytes(),
                 RowAddr{static_cast<int>(p.stride_row * p.elem_bytes()),
                         static_cast<int>(p.D * p.elem_bytes())}};
}

LaunchArgs launch_args(const Problem& p, const Plan& plan, const float* states, const float* dstates) {
  LaunchArgs a{};
  a.Q = static_cast<const unsigned char*>(p.Q);
  a.K = static_cast<const unsigned char*>(p.K);
  a.V = static_cast<const unsigned char*>(p.V);
  a.dO = static_cast<const unsigned char*>(p.dO);
  a.mask = p.mask;
  a.states = states;
  a.dstates = dstates;
  a.O = static_cast<unsigned char*>(p.O);
  a.dQ = static_cast<unsigned char*>(p.dQ);
  a.dK = static_cast<unsigned char*>(p.dK);
  a.dV = static_cast<unsigned char*>(p.dV);
  a.H = p.H;
  a.N = p.N;
  a.splits = plan.splits;
  a.rows_per_split = plan.rows_per_split;
  a.scale = p.scale;
  a.eps = p.eps;
  a.slice_scale = p.slice_scale;
  a.st = byte_strides(p);
  return a;
}

// Workgroups of 8 waves (the whole LDS of a compute unit at their disposal) when the launch has
// no more workgroups than there are compute units, of 4 waves (two per compute unit) otherwise.
constexpr int kUnits = 256;
template <int WAVES>
constexpr int max_lds_bytes() {
  return WAVES == 8 ? 160 * 1024 : 80 * 1024;
}

template <class F, int WAVES>
hipError_t states_w(const Problem& p, const Plan& plan, bool bwd) {
  constexpr int D = 2 * F::D;
  constexpr int lds = WAVES * 4 * kTileBytes;
  static_assert(lds <= max_lds_bytes<WAVES>(), "round buffer");
  const unsigned blocks = static_cast<unsigned>(p.B) * p.H * plan.splits;
  const size_t second = static_cast<size_t>(blocks) * D * D;
  const hipError_t err =
      grant_dynamic_lds(reinterpret_cast<const void*>(wide_state_kernel<F, WAVES>), max_lds_bytes<WAVES>());
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL((wide_state_kernel<F, WAVES>), dim3(blocks, bwd ? 2 : 1), dim3(64 * WAVES), lds,
                     p.stream, static_cast<const unsigned char*>(p.Q),
                     static_cast<const unsigned char*>(p.K), static_cast<const unsigned char*>(p.V),
                     static_cast<const unsigned char*>(p.dO), p.mask, p.workspace, p.H, p.N,
                     plan.splits, plan.rows_per_split, second, p.eps, byte_strides(p));
  return hipGetLastError();
}

template <class F, int WAVES>
hipError_t apply_w(const Problem& p, const Plan& plan, const float* st, const float* dst, bool bwd) {
  constexpr int lds = ApplyLds<F, WAVES>::kBytes;
  static_assert(lds <= max_lds_bytes<WAVES>(), "images and tiles");
  const LaunchArgs a = launch_args(p, plan, st, dst);
  const unsigned blocks = static_cast<unsigned>(p.B) * p.H * plan.splits;
  const void* kern = bwd ? reinterpret_cast<const void*>(wide_bwd_kernel<F, WAVES>)
                         : reinterpret_cast<const void*>(wide_fwd_kernel<F, WAVES>);
  const hipError_t err = grant_dynamic_lds(kern, max_lds_bytes<WAVES>());
  if (err != hipSuccess) return err;
  if (bwd)
    hipLaunchKernelGGL((wide_bwd_kernel<F, WAVES>), dim3(blocks, 3), dim3(64 * WAVES), lds, p.stream, a);
  else
    hipLaunchKernelGGL((wide_fwd_kernel<F, WAVES>), dim3(blocks), dim3(64 * WAVES), lds, p.stream, a);
  return hipGetLastError();
}

// `kinds`: workgroups per (slice, split) of the launch (states or roles)
inline bool few_workgroups(const Problem& p, const Plan& plan, int kinds) {
  return static_cast<long>(p.B) * p.H * plan.splits * kinds <= kUnits;
}

template <class F>
hipError_t states(const Problem& p, const Plan& plan, bool bwd) {
  return few_workgroups(p, plan, bwd ? 2 : 1) ? states_w<F, 8>(p, plan, bwd) : states_w<F, 4>(p, plan, bwd);
}

template <class F>
hipError_t apply(const Problem& p, const Plan& plan, const float* st, const float* dst, bool bwd) {
  return few_workgroups(p, plan, bwd ? 3 : 1) ? apply_w<F, 8>(p, plan, st, dst, bwd)
                                              : apply_w<F, 4>(p, plan, st, dst, bwd);
}

}  // namespace wide
}  // namespace

bool wide_supports(int dtype, int D) { return dtype == 0 ? D == 64 : D == 128; }

hipError_t launch_wide_states(const Problem& p, const Plan& plan, bool bwd) {
  using namespace mfma;
  return p.dtype == 0   ? wide::states<F32x32>(p, plan, bwd)
         : p.dtype == 1 ? wide::states<Bf16x64>(p, plan, bwd)
                        : wide::states<F16x64>(p, plan, bwd);
}

hipError_t launch_wide_apply(const Problem& p, const Plan& plan, const float* states,
                             const float* dstates, bool bwd) {
  using namespace mfma;
  return p.dtype == 0   ? wide::apply<F32x32>(p, plan, states, dstates, bwd)
         : p.dtype == 1 ? wide::apply<Bf16x64>(p, plan, states, dstates, bwd)
                        : wide::apply<F16x64>(p, plan, states, dstates, bwd);
}

}  // namespace cotten
