// Matrix-core kernels for 256-byte rows: fp32 I/O with d_h = 64, bf16 / fp16 I/O with d_h = 128
// (d_model = 128 or 256 with two heads, "Sequence Length and Embedding Size") - and, in their
// three-launch form, for the 512-byte rows of fp32 I/O with d_h = 128.
//
// A 256-byte row is handled as two 128-byte halves, a d_h x d_h state as four quadrants of
// the size the 128-byte-row formats work on (cotten_mfma_core.h), so that their tile layout,
// MFMA products, operand images and row epilogues serve unchanged:
//
//     S[p][q] = sum_j khat_j[half p]^T v_j[half q]           (state kernel)
//     O[half q] = sum_p Qhat[half p] S[p][q]                 (apply kernels; likewise dQ, dK, dV)
//
// with the row norm taken over both halves.  Three launches (partial states in the caller's
// workspace, [kinds][slices * splits][D * D] floats, then the reduced states):
//
//   wide_state_kernel   a workgroup of four (or eight) waves reduces a block of rows of one slice
//                       to a partial state: per round every wave stages one 16-row tile in LDS,
//                       then wave (p, q) adds four tiles of the round to its quadrant (with eight
//                       waves two waves share a quadrant and their sums meet at the end)
//   (the partial states of a slice are summed in split order by reduce_states_kernel)
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
//
// Template parameter P: the 128-byte pieces of a row.  2 for the 256-byte rows above; the kernels
// of the three-launch structure also exist for P = 4, fp32 rows of 512 bytes (d_h = 128): the
// state in 4 x 4 blocks of 32 x 32, four of them per wave of the state kernel, one set of sixteen
// operand images in the LDS of an apply workgroup of four waves.
constexpr int kHalfBytes = kRowBytes;    // one piece of a row

// A 16-row tile of a tensor pair in the load layout: piece [h][c] is bytes 128 c + 16 ch .. + 15 of
// row r8 + 8 h.  `live` bit h: the row takes part.
template <int P>
struct WideRawT {
  u32x4_t x[2][P], y[2][P];
  int live;
};
typedef WideRawT<2> WideRaw;

// The two tensors of a pass as buffer resources over one slice (see Src in cotten_mfma_core.h:
// lanes whose row does not take part get zeros and cause no traffic).
template <int P>
struct WideSrcT {
  __amdgpu_buffer_rsrc_t x, y;
  int stride;
  __device__ __forceinline__ WideSrcT(const unsigned char* X, const unsigned char* Y, int N, int stride_bytes)
      : stride(stride_bytes) {
    const int bytes = (N - 1) * stride + P * kHalfBytes;
    x = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(X), 0, bytes, 0x00020000);
    y = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(Y), 0, bytes, 0x00020000);
  }
};
typedef WideSrcT<2> WideSrc;

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

template <bool USE_Y, int P>
__device__ __forceinline__ void load_wide(WideRawT<P>& r, const Lane& L, const WideSrcT<P>& src, int row0,
                                          int bits) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const bool live = ((bits >> h) & 1) != 0;
    const uint32_t off =
        live ? static_cast<uint32_t>(row0 + L.r8 + 8 * h) * src.stride + L.ch * 16 : kOutOfBuffer;
#pragma unroll
    for (int c = 0; c < P; ++c) {
      r.x[h][c] = __builtin_amdgcn_raw_buffer_load_b128(src.x, off + c * kHalfBytes, 0, 0);
      if (USE_Y) r.y[h][c] = __builtin_amdgcn_raw_buffer_load_b128(src.y, off + c * kHalfBytes, 0, 0);
      else r.y[h][c] = u32x4_t{0, 0, 0, 0};
    }
  }
  r.live = bits;
}

// The tile into LDS as 2 P tiles of 16 x 128 bytes [x pieces | y pieces] (each in the layout of
// cotten_mfma_core.h); x raw, normalised over the whole row, or through the element-wise map of
// the format (XMODE, see stage() in cotten_mfma_core.h).
// inv[h] = 1/r of row r8 + 8 h (0 for a row that does not take part; with the element-wise map 1
// for a row that does, and a row that does not is written as zeros explicitly: phi(0) is not 0).
template <class F, int XMODE, bool USE_Y, int P>
__device__ __forceinline__ void stage_wide(const WideRawT<P>& r, const Lane& L, float eps,
                                           unsigned char* tiles, float (&inv)[2]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float f[P][F::EPL];
    const bool live = ((r.live >> h) & 1) != 0;
    const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
    if (XMODE == kXFeature) {
      inv[h] = live ? 1.0f : 0.0f;
#pragma unroll
      for (int c = 0; c < P; ++c) {
        F::unpack(r.x[h][c], f[c]);
#pragma unroll
        for (int i = 0; i < F::EPL; ++i) f[c][i] = live ? elu1(f[c][i]) : 0.0f;
        *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = F::pack(f[c]);
        if (USE_Y) *reinterpret_cast<u32x4_t*>(tiles + (P + c) * kTileBytes + off) = r.y[h][c];
      }
      continue;
    }
    float ss = 0.0f;
#pragma unroll
    for (int c = 0; c < P; ++c) {
      F::unpack(r.x[h][c], f[c]);
#pragma unroll
      for (int i = 0; i < F::EPL; ++i) ss += f[c][i] * f[c][i];
    }
    inv[h] = inv_norm_or_zero(row_sum8(ss), eps, live);
#pragma unroll
    for (int c = 0; c < P; ++c) {
      if (XMODE == kXNormalized) {
#pragma unroll
        for (int i = 0; i < F::EPL; ++i) f[c][i] *= inv[h];
        *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = F::pack(f[c]);
      } else {
        *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = r.x[h][c];
      }
      if (USE_Y) *reinterpret_cast<u32x4_t*>(tiles + (P + c) * kTileBytes + off) = r.y[h][c];
    }
  }
}

// How the x rows enter a product whose result is divided by r afterwards: raw under the cosine
// map (1/r applied to the result), mapped under the element-wise one (1/r is then 1).
template <class F>
constexpr int plain_mode() {
  return F::kMap == kMapElu1 ? kXFeature : kXRaw;
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

// No row of the tile takes part (all of them masked or beyond the sequence): the wave can write
// the zeros such rows come out as without computing them.
template <int P>
__device__ __forceinline__ bool tile_dead(const WideRawT<P>& r) {
  return __builtin_amdgcn_ballot_w64(r.live != 0) == 0;
}

template <class F, int P = 2>
__device__ __forceinline__ void store_zero_rows(unsigned char* out, int row0, int r_end, int stride,
                                                const Lane& L) {
  float z[2 * F::EPL];
#pragma unroll
  for (int i = 0; i < 2 * F::EPL; ++i) z[i] = 0.0f;
  const int row = row0 + L.i16;
  if (row < r_end) {
#pragma unroll
    for (int q = 0; q < P; ++q)
      store_product_row<F, kStoreStreamed>(out + q * kHalfBytes, row, RowAddr{stride, kHalfBytes}, L, z);
  }
}

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

// ---- state kernel -------------------------------------------------------------------------------

// grid (slices * splits, 1 or 2): blockIdx.y == 1 reduces (Q, dO) to sum_i qhat_i^T dO_i instead
// of (K, V) under the key mask.  Partial states: row-major D x D floats per workgroup, the second
// kind `second_offset` floats behind the first.
// The P x P blocks of the state are dealt to the waves 0-3 of a group, P*P/4 consecutive ones
// each (block i = piece i / P of x against piece i % P of y); with 8 waves two groups share the
// tiles of a round and their sums meet at the end.
template <class F, int WAVES, int P>
__global__ __launch_bounds__(64 * WAVES) void wide_state_kernel(
    const unsigned char* __restrict__ Q, const unsigned char* __restrict__ K,
    const unsigned char* __restrict__ V, const unsigned char* __restrict__ dO,
    const uint8_t* __restrict__ mask, float* __restrict__ ws, int H, int N, int splits,
    int rows_per_split, size_t second_offset, float eps, Strides st) {
  constexpr int Dh = F::D, D = P * Dh, kRoundRows = WAVES * TR, kBlocks = P * P / 4;
  constexpr int kSetBytes = 2 * P * kTileBytes;  // the tiles one wave stages per round
  static_assert(WAVES == 4 || WAVES == 8, "one or two groups of four waves");
  unsigned char* round = smem;  // WAVES x [x pieces | y pieces]
  const Lane L;
  const int split = blockIdx.x % splits, bh = blockIdx.x / splits;
  const bool second = blockIdx.y == 1;
  const size_t base = st.slice_base(bh, H);
  const WideSrcT<P> src((second ? Q : K) + base, (second ? dO : V) + base, N, st.row.stride);
  const uint8_t* __restrict__ m =
      (second || mask == nullptr) ? nullptr : mask + static_cast<size_t>(bh / H) * N;
  const int r_begin = split * rows_per_split;
  const int r_end = N < r_begin + rows_per_split ? N : r_begin + rows_per_split;
  // this wave's blocks of the state, and (8 waves) which four tiles of a round it adds up
  const int quadrant = L.wave & 3, part = L.wave >> 2;
  unsigned char* mine = round + L.wave * kSetBytes;

  typename F::Acc acc[kBlocks];
#pragma unroll
  for (int j = 0; j < kBlocks; ++j) acc[j].zero();
  WideRawT<P> cur;
  load_wide<true>(cur, L, src, r_begin + L.wave * TR, row_bits(m, r_begin + L.wave * TR, r_end, L));
  int next_bits = row_bits(m, r_begin + kRoundRows + L.wave * TR, r_end, L);
  for (int r0 = r_begin; r0 < r_end; r0 += kRoundRows) {
    float inv[2];
    stage_wide<F, mapped_mode<F>(), true>(cur, L, eps, mine, inv);
    // the wave's tile of the next round travels while this round is added up
    load_wide<true>(cur, L, src, r0 + kRoundRows + L.wave * TR, next_bits);
    next_bits = row_bits(m, r0 + 2 * kRoundRows + L.wave * TR, r_end, L);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const unsigned char* tile = round + (4 * part + t) * kSetBytes;
#pragma unroll
      for (int j = 0; j < kBlocks; ++j) {
        const int block = quadrant * kBlocks + j;
        acc[j].mfma(tile + (block / P) * kTileBytes, tile + (P + block % P) * kTileBytes, L);
      }
    }
    __syncthreads();  // the round's tiles are overwritten next
  }
  // 8 waves: the two sums of a block meet in LDS (the round buffer is free), in a fixed order
  f32x4_t* meet = reinterpret_cast<f32x4_t*>(round) + quadrant * kBlocks * F::Acc::kGroups * 64 + L.lane;
  static_assert(4 * kBlocks * F::Acc::kGroups * 64 * 16 <= 8 * kSetBytes, "the sums fit the round buffer");
  if (WAVES == 8) {
    if (part == 1) {
#pragma unroll
      for (int j = 0; j < kBlocks; ++j)
#pragma unroll
        for (int g = 0; g < F::Acc::kGroups; ++g) meet[(j * F::Acc::kGroups + g) * 64] = acc[j].group(g);
    }
    __syncthreads();
    if (part == 1) return;
  }
  float* __restrict__ out =
      ws + (second ? second_offset : 0) + static_cast<size_t>(blockIdx.x) * D * D;
#pragma unroll
  for (int j = 0; j < kBlocks; ++j) {
    const int block = quadrant * kBlocks + j;
#pragma unroll
    for (int g = 0; g < F::Acc::kGroups; ++g) {
      f32x4_t v = acc[j].group(g);
      if (WAVES == 8) v += meet[(j * F::Acc::kGroups + g) * 64];
      const int row = (block / P) * Dh + F::Acc::group_row(g, L);
      const int col = (block % P) * Dh + F::Acc::group_col(g, L);
#pragma unroll
      for (int i = 0; i < 4; ++i) out[(row + i) * D + col] = v[i];
    }
  }
}

// ---- operand images --------------------------------------------------------------------------------

// The P x P block images of scale * M (M: a reduced state in global memory, row-major D x D),
// image (p, q) at images + (P p + q) * F::kImageBytes:
//   natural     op[m][n] = M[p Dh + m][q Dh + n]     for products that contract over n
//   transposed  op[n][m] = M[p Dh + m][q Dh + n]     for products that contract over m
template <class F, int WAVES, bool TRANSPOSED, int P>
__device__ __forceinline__ void build_images(const float* __restrict__ M, float scale,
                                             unsigned char* images) {
  constexpr int Dh = F::D, D = P * Dh, kThreads = 64 * WAVES;
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
      unsigned char* image = images + (P * (m / Dh) + n / Dh) * F::kImageBytes;
      if (TRANSPOSED) F::write_image_pair(image, n % Dh, m % Dh, v0[j] * scale, v1[j] * scale);
      else F::write_image_pair(image, m % Dh, n % Dh, v0[j] * scale, v1[j] * scale);
    }
  }
}

// The P x P block operands of a role: held in registers for all the tiles of the wave (HOLD:
// 4 x 32 registers for the 16-bit formats with P = 2), or fetched from the images for every
// product (the backward roles share one kernel and do better at two waves per SIMD than with
// the operands held at one).
template <class F, bool HOLD, int P = 2>
struct Quadrants {
  typename F::Operand held[HOLD ? P * P : 1];
  const unsigned char* images;
  __device__ __forceinline__ Quadrants(const unsigned char* img, const Lane& L) : images(img) {
    if (HOLD) {
#pragma unroll
      for (int i = 0; i < P * P; ++i) held[i].load(images + i * F::kImageBytes, L);
    }
  }
  // out = sum_c X[piece c] W(first + c * step), images numbered P p + q
  __device__ __forceinline__ void apply(const typename F::TileRows (&X)[P], int first, int step,
                                        const Lane& L, float (&out)[2 * F::EPL]) const {
    f32x4_t a[F::NT];
#pragma unroll
    for (int c = 0; c < P; ++c) {
      if (HOLD) {
        if (c == 0) F::apply(X[c], held[first], a);
        else F::apply_onto(X[c], held[first + c * step], a);
      } else {
        typename F::Operand W;
        W.load(images + (first + c * step) * F::kImageBytes, L);
        if (c == 0) F::apply(X[c], W, a);
        else F::apply_onto(X[c], W, a);
      }
    }
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

// LDS of the apply kernels: [P x P images][per wave: 2 P tiles, 16 floats]
template <class F, int WAVES, int P = 2>
struct ApplyLds {
  static constexpr int kImages = 0;
  static constexpr int kWave = P * P * F::kImageBytes;
  static constexpr int kWaveBytes = 2 * P * kTileBytes + TR * 4;
  static constexpr int kBytes = kWave + WAVES * kWaveBytes;
};

// out rows = (x rows) M / r, contraction over the rows of M:  O = scale qhat S,  dV = scale khat dS.
// One tile of the plain role: `cur` staged raw into the wave's tile set, out rows = x W / r.
template <class F, bool HOLD, int P>
__device__ __forceinline__ void plain_tile(const Quadrants<F, HOLD, P>& W, const WideRawT<P>& cur, int row0,
                                           int r_end, unsigned char* out, int stride, float eps,
                                           unsigned char* tiles, const Lane& L) {
  if (tile_dead(cur)) {
    store_zero_rows<F, P>(out, row0, r_end, stride, L);
    return;
  }
  float* inv_slot = reinterpret_cast<float*>(tiles + 2 * P * kTileBytes);
  float inv[2];
  stage_wide<F, plain_mode<F>(), false>(cur, L, eps, tiles, inv);
  const float inv_r = inv_by_row(inv_slot, L, inv);
  typename F::TileRows X[P];
#pragma unroll
  for (int c = 0; c < P; ++c) X[c].load(tiles + c * kTileBytes, L);
  const int row = row0 + L.i16;
#pragma unroll
  for (int q = 0; q < P; ++q) {
    float o[2 * F::EPL];
    W.apply(X, q, P, L, o);
#pragma unroll
    for (int i = 0; i < 2 * F::EPL; ++i) o[i] *= inv_r;
    if (row < r_end)
      store_product_row<F, kStoreStreamed>(out + q * kHalfBytes, row, RowAddr{stride, kHalfBytes}, L, o);
  }
  wave_lds_fence();
}

// `images`: the transposed block images of scale * M; `tiles`: this wave's tile set.
// The wave's first tile: requested here, or (REQUESTED) by the caller with request_first_tile.
template <int WAVES, int P>
__device__ __forceinline__ void request_first_tile(WideRawT<P>& cur, const ApplyArgs& a, const Lane& L) {
  const WideSrcT<P> src(a.X, a.X, a.N, a.stride);
  const int row0 = a.r_begin + L.wave * TR;
  load_wide<false>(cur, L, src, row0, row_bits(a.mask, row0, a.r_end, L));
}

template <class F, int WAVES, bool HOLD, bool REQUESTED = false, int P = 2>
__device__ __forceinline__ void plain_tiles(const ApplyArgs& a, const unsigned char* images,
                                            unsigned char* tiles, const Lane& L,
                                            const WideRawT<P>* first = nullptr) {
  constexpr int kRoundRows = WAVES * TR;  // rows between two tiles of a wave
  const Quadrants<F, HOLD, P> W(images, L);
  const WideSrcT<P> src(a.X, a.X, a.N, a.stride);
  int row0 = a.r_begin + L.wave * TR;
  WideRawT<P> cur;
  if (REQUESTED) cur = *first;
  else request_first_tile<WAVES>(cur, a, L);
  int next_bits = row_bits(a.mask, row0 + kRoundRows, a.r_end, L);
  for (; row0 < a.r_end; row0 += kRoundRows) {
    const WideRawT<P> tile = cur;
    load_wide<false>(cur, L, src, row0 + kRoundRows, next_bits);
    next_bits = row_bits(a.mask, row0 + 2 * kRoundRows, a.r_end, L);
    plain_tile<F, HOLD>(W, tile, row0, a.r_end, a.out, a.stride, a.eps, tiles, L);
  }
}

template <class F, int WAVES, bool HOLD, int P>
__device__ __forceinline__ void plain_role(const ApplyArgs& a) {
  const Lane L;
  unsigned char* images = smem + ApplyLds<F, WAVES, P>::kImages;
  unsigned char* tiles = smem + ApplyLds<F, WAVES, P>::kWave + L.wave * ApplyLds<F, WAVES, P>::kWaveBytes;
  build_images<F, WAVES, true, P>(a.state, a.scale, images);
  __syncthreads();
  plain_tiles<F, WAVES, HOLD, false, P>(a, images, tiles, L);
}

// The row epilogue of dQ and dK over all pieces of a row, E holding the mapped rows (xhat, or
// phi(x)):  cosine map  g <- (g - xhat (xhat . g)) / r;   ELU + 1  g <- g * phi'(x), phi' = min(phi, 1).
template <class F, int P>
__device__ __forceinline__ void finish_projected(float (&g)[P][2 * F::EPL], typename F::TileRows (&E)[P],
                                                 float inv_r, const Lane& L) {
  if (F::kMap == kMapElu1) {
#pragma unroll
    for (int p = 0; p < P; ++p) feature_grad_rows<F>(g[p], E[p]);
    return;
  }
  float proj = 0.0f;
#pragma unroll
  for (int p = 0; p < P; ++p) {
    float u[2 * F::EPL];
    E[p].unpack(u);
#pragma unroll
    for (int c = 0; c < 2 * F::EPL; ++c) proj += u[c] * g[p][c];
    E[p].forget_unpacked();
  }
  proj = row_sum_groups(proj, L);
#pragma unroll
  for (int p = 0; p < P; ++p) {
    float u[2 * F::EPL];
    E[p].unpack(u);
#pragma unroll
    for (int c = 0; c < 2 * F::EPL; ++c) g[p][c] = (g[p][c] - u[c] * proj) * inv_r;
  }
}

// out rows = (g - xhat (xhat . g)) / r with g = (y rows) M^T, contraction over the columns of M:
//   dQ from (Q, dO) and scale S;   dK from (K, V) and scale dS (masked rows come out as zeros).
// `images`: the natural block images of scale * M.
template <class F, int WAVES, int P = 2>
__device__ __forceinline__ void projected_tiles(const ApplyArgs& a, const unsigned char* images,
                                                unsigned char* tiles, const Lane& L) {
  constexpr int kRoundRows = WAVES * TR;
  float* inv_slot = reinterpret_cast<float*>(tiles + 2 * P * kTileBytes);
  const Quadrants<F, false, P> W(images, L);
  const WideSrcT<P> src(a.X, a.Y, a.N, a.stride);
  int row0 = a.r_begin + L.wave * TR;
  WideRawT<P> cur;
  load_wide<true>(cur, L, src, row0, row_bits(a.mask, row0, a.r_end, L));
  int next_bits = row_bits(a.mask, row0 + kRoundRows, a.r_end, L);
  for (; row0 < a.r_end; row0 += kRoundRows) {
    if (tile_dead(cur)) {  // nothing was fetched: zeros
      load_wide<true>(cur, L, src, row0 + kRoundRows, next_bits);
      next_bits = row_bits(a.mask, row0 + 2 * kRoundRows, a.r_end, L);
      store_zero_rows<F, P>(a.out, row0, a.r_end, a.stride, L);
      continue;
    }
    float inv[2];
    stage_wide<F, mapped_mode<F>(), true>(cur, L, a.eps, tiles, inv);
    load_wide<true>(cur, L, src, row0 + kRoundRows, next_bits);
    next_bits = row_bits(a.mask, row0 + 2 * kRoundRows, a.r_end, L);
    const float inv_r = inv_by_row(inv_slot, L, inv);
    typename F::TileRows Y[P], E[P];
#pragma unroll
    for (int c = 0; c < P; ++c) Y[c].load(tiles + (P + c) * kTileBytes, L);
    float g[P][2 * F::EPL];
#pragma unroll
    for (int p = 0; p < P; ++p)
      W.apply(Y, P * p, 1, L, g[p]);
#pragma unroll
    for (int c = 0; c < P; ++c) E[c].load(tiles + c * kTileBytes, L);
    finish_projected<F>(g, E, inv_r, L);
    const int row = row0 + L.i16;
#pragma unroll
    for (int p = 0; p < P; ++p) {
      if (row < a.r_end)
        store_product_row<F, kStoreStreamed>(a.out + p * kHalfBytes, row, RowAddr{a.stride, kHalfBytes}, L, g[p]);
    }
    wave_lds_fence();
  }
}

template <class F, int WAVES, int P>
__device__ __forceinline__ void projected_role(const ApplyArgs& a) {
  const Lane L;
  unsigned char* images = smem + ApplyLds<F, WAVES, P>::kImages;
  unsigned char* tiles = smem + ApplyLds<F, WAVES, P>::kWave + L.wave * ApplyLds<F, WAVES, P>::kWaveBytes;
  build_images<F, WAVES, false, P>(a.state, a.scale, images);
  __syncthreads();
  projected_tiles<F, WAVES, P>(a, images, tiles, L);
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

__device__ __forceinline__ ApplyArgs role_args(const LaunchArgs& a) {
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

template <class F, int WAVES, int P>
__global__ __launch_bounds__(64 * WAVES) void wide_fwd_kernel(const LaunchArgs a) {
  constexpr int D = P * F::D;
  const int bh = blockIdx.x / a.splits;
  const size_t base = a.st.slice_base(bh, a.H);
  ApplyArgs r = role_args(a);
  r.X = a.Q + base;
  r.mask = nullptr;  // queries are not masked
  r.state = a.states + static_cast<size_t>(bh) * D * D;
  r.out = a.O + base;
  plain_role<F, WAVES, P == 2, P>(r);  // operands held in registers where they fit
}

// blockIdx.y: 0 dQ, 1 dV, 2 dK
template <class F, int WAVES, int P>
__global__ __launch_bounds__(64 * WAVES) void wide_bwd_kernel(const LaunchArgs a) {
  constexpr int D = P * F::D;
  const int bh = blockIdx.x / a.splits;
  const size_t base = a.st.slice_base(bh, a.H);
  ApplyArgs r = role_args(a);
  const uint8_t* keys = a.mask == nullptr ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
  if (blockIdx.y == 0) {
    r.X = a.Q + base;
    r.Y = a.dO + base;
    r.mask = nullptr;
    r.state = a.states + static_cast<size_t>(bh) * D * D;
    r.out = a.dQ + base;
    projected_role<F, WAVES, P>(r);
  } else if (blockIdx.y == 1) {
    r.X = a.K + base;
    r.mask = keys;
    r.state = a.dstates + static_cast<size_t>(bh) * D * D;
    r.out = a.dV + base;
    plain_role<F, WAVES, false, P>(r);
  } else {
    r.X = a.K + base;
    r.Y = a.V + base;
    r.mask = keys;
    r.state = a.dstates + static_cast<size_t>(bh) * D * D;
    r.out = a.dK + base;
    projected_role<F, WAVES, P>(r);
  }
}

// ---- one launch per direction: a workgroup of eight waves per slice ------------------------------
//
// When a sequence is not cut (one partial state per slice), the state need not leave the compute
// unit: the quadrant sums go from the accumulators straight into the operand images in LDS and
// the same workgroup streams the slice a second time through the apply roles.
//
//   forward   all eight waves reduce (K, V) to S (two waves per quadrant, rounds of 128 rows, the
//             sums meet in LDS), then stream Q through the transposed images of scale S.
//   backward  waves 0-3 reduce (K, V) to S, waves 4-7 (Q, dO) to dS, rounds of 64 rows each; then
//             all waves run dQ (natural images of S) and dV (transposed images of dS), and, the
//             images of S overwritten by the natural images of dS, dK.
//
// LDS: [SETS x four images][per wave: four tiles, 16 floats]; the tile sets double as the round
// buffer of the state phase and as the place where accumulators meet.
template <class F, int SETS>
struct FusedLds {
  static constexpr int kWaves = 8;
  static constexpr int kSetBytes = 4 * F::kImageBytes;
  static constexpr int kTiles = SETS * kSetBytes;
  static constexpr int kWaveBytes = 4 * kTileBytes + TR * 4;
  static constexpr int kBytes = kTiles + kWaves * kWaveBytes;
  static_assert(4 * F::Acc::kGroups * 64 * 16 + 64 <= kWaves * kWaveBytes, "accumulators meet in the tile sets");
};

// The state phase of a group of four waves (wave & 3: the quadrant): every wave stages the 16 rows
// from `first_row` on of each round into its own tile set and adds the four tile sets of its group
// (wave >> 2) to its quadrant - or, `swapped`, the transposed sum (y tile)^T (x tile) with the two
// operands changing places, from which the natural image is the one that can be written
// straight from the lane.  Rows at and beyond N, and masked rows, are never fetched.
template <class F, int WAVE_BYTES>
__device__ __forceinline__ void fused_state_pass(typename F::Acc& acc, const WideSrc& src,
                                                 const uint8_t* __restrict__ m, int N, int first_row,
                                                 int round_rows, float eps, unsigned char* sets,
                                                 const Lane& L, bool swapped = false, int limit = -1) {
  if (limit < 0) limit = N;  // rows that exist (0: the group has no slice and only keeps step)
  const int quadrant = L.wave & 3, p = quadrant >> 1, q = quadrant & 1, group = L.wave >> 2;
  const int left = (swapped ? 2 + q : p) * kTileBytes, right = (swapped ? p : 2 + q) * kTileBytes;
  unsigned char* mine = sets + L.wave * WAVE_BYTES;
  acc.zero();
  WideRaw cur;
  load_wide<true>(cur, L, src, first_row, row_bits(m, first_row, limit, L));
  int next_bits = row_bits(m, first_row + round_rows, limit, L);
  for (int r0 = 0; r0 < N; r0 += round_rows) {
    float inv[2];
    stage_wide<F, mapped_mode<F>(), true>(cur, L, eps, mine, inv);
    load_wide<true>(cur, L, src, r0 + round_rows + first_row, next_bits);
    next_bits = row_bits(m, r0 + 2 * round_rows + first_row, limit, L);
    __syncthreads();
#pragma unroll
    for (int t = 0; t < 4; ++t) {
      const unsigned char* tile = sets + (4 * group + t) * WAVE_BYTES;
      acc.mfma(tile + left, tile + right, L);
    }
    __syncthreads();  // the tile sets are overwritten next
  }
}

// A quadrant of scale * M from the accumulator layout (`get(g)`: group g, four consecutive rows of
// one column) into its operand image: transposed straight from the lane (two row pairs of its
// column), natural with the neighbouring lane's column (even lanes write the first two rows of a
// group, odd lanes the last two; each gets the other column of its rows from its neighbour).
template <class F, bool NATURAL, class Get>
__device__ __forceinline__ void quadrant_image(Get get, float scale, unsigned char* image, const Lane& L) {
  // (row, column) of the first value of a group = a part that depends on the lane only plus a
  // part that depends on the group only; the image offsets of the two add up, so the second
  // becomes the immediate offset of the write
  const int lane_row = F::Acc::group_row(0, L), lane_col = F::Acc::group_col(0, L);
  const bool odd = (lane_col & 1) != 0;
  Lane zero = L;
  zero.set(0);
  unsigned char* at = image + (NATURAL ? F::image_offset(lane_row + (odd ? 2 : 0), lane_col & ~1)
                                       : F::image_offset(lane_col, lane_row));
#pragma unroll
  for (int g = 0; g < F::Acc::kGroups; ++g) {
    const f32x4_t v = get(g) * scale;
    const int row = F::Acc::group_row(g, zero), col = F::Acc::group_col(g, zero);  // the group's part
    if (!NATURAL) {
      F::write_pair_at(at + F::image_offset(col, row), v[0], v[1]);
      F::write_pair_at(at + F::image_offset(col, row + 2), v[2], v[3]);
    } else {
      // The lane sends what its neighbour wants (the choice is made on the sending side: a
      // choice between two values received from the neighbour would be evaluated over there).
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const float mine = odd ? v[2 + i] : v[i];
        int sent = __builtin_bit_cast(int, odd ? v[i] : v[2 + i]);
        asm volatile("" : "+v"(sent));
        int got = __builtin_amdgcn_update_dpp(0, sent, 0xB1, 0xF, 0xF, true);  // lane ^ 1
        asm volatile("" : "+v"(got));
        const float other = __builtin_bit_cast(float, got);
        F::write_pair_at(at + F::image_offset(row + i, col), odd ? other : mine, odd ? mine : other);
      }
    }
  }
}

// End of the forward's state phase: the two sums of a quadrant meet in `meet_area` (free by then),
// in a fixed order; the waves of the first group write the transposed images of scale * S and, if
// asked, S itself (row-major, for the caller's backward call).  Ends with a barrier.
template <class F>
__device__ __forceinline__ void forward_images(const typename F::Acc& acc, float scale,
                                               unsigned char* images, unsigned char* meet_area,
                                               float* __restrict__ kept, const Lane& L) {
  constexpr int Dh = F::D, D = 2 * Dh;
  const int quadrant = L.wave & 3, part = L.wave >> 2;
  f32x4_t* meet = reinterpret_cast<f32x4_t*>(meet_area) + quadrant * F::Acc::kGroups * 64 + L.lane;
  if (part == 1) {
#pragma unroll
    for (int g = 0; g < F::Acc::kGroups; ++g) meet[g * 64] = acc.group(g);
  }
  __syncthreads();
  if (part == 0) {
    const auto sum = [&](int g) { return acc.group(g) + meet[g * 64]; };
    quadrant_image<F, false>(sum, scale, images + quadrant * F::kImageBytes, L);
    if (kept != nullptr) {
      const int p = quadrant >> 1, q = quadrant & 1;
#pragma unroll
      for (int g = 0; g < F::Acc::kGroups; ++g) {
        const f32x4_t v = sum(g);
        const int row = p * Dh + F::Acc::group_row(g, L), col = q * Dh + F::Acc::group_col(g, L);
#pragma unroll
        for (int i = 0; i < 4; ++i) kept[(row + i) * D + col] = v[i];
      }
    }
  }
  __syncthreads();
}

template <class F>
__global__ __launch_bounds__(512) void wide_fused_fwd_kernel(const LaunchArgs a, float* __restrict__ kept) {
  using Lds = FusedLds<F, 1>;
  constexpr int Dh = F::D, D = 2 * Dh;
  const Lane L;
  const int bh = blockIdx.x;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* images = smem;
  unsigned char* sets = smem + Lds::kTiles;
  typename F::Acc acc;
  {
    const WideSrc kv(a.K + base, a.V + base, a.N, a.st.row.stride);
    const uint8_t* keys = a.mask == nullptr ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
    fused_state_pass<F, Lds::kWaveBytes>(acc, kv, keys, a.N, L.wave * TR, 8 * TR, a.eps, sets, L);
  }
  const float scale = a.slice_scale != nullptr ? a.slice_scale[bh] : a.scale;
  ApplyArgs r{};
  r.X = a.Q + base;
  r.mask = nullptr;  // queries are not masked
  r.out = a.O + base;
  r.N = a.N;
  r.r_begin = 0;
  r.r_end = a.N;
  r.stride = a.st.row.stride;
  r.scale = scale;
  r.eps = a.eps;
  // the first tile of Q travels while the images are made
  WideRaw first;
  request_first_tile<8>(first, r, L);
  forward_images<F>(acc, scale, images, sets, kept == nullptr ? nullptr : kept + static_cast<size_t>(bh) * D * D, L);
  plain_tiles<F, 8, true, true>(r, images, sets + L.wave * Lds::kWaveBytes, L, &first);
}

// The forward with two slices per workgroup (waves 0-3 one slice, waves 4-7 the next), for
// launches with more slices than compute units: the LDS of a compute unit admits one of these
// workgroups at a time, and two slices that share it overlap their waits.  A group of four waves
// owns its slice completely (one quadrant per wave, rounds of 64 rows, no sums to meet), so the
// only thing the two groups share is the barriers of the state phase.
template <class F>
__global__ __launch_bounds__(512) void wide_paired_fwd_kernel(const LaunchArgs a, int slices,
                                                              float* __restrict__ kept) {
  using Lds = FusedLds<F, 2>;
  constexpr int Dh = F::D, D = 2 * Dh;
  const Lane L;
  const int quadrant = L.wave & 3, group = L.wave >> 2;
  const int slice = 2 * blockIdx.x + group;
  const bool exists = slice < slices;
  const int bh = exists ? slice : 0;
  const int rows = exists ? a.N : 0;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* images = smem + group * Lds::kSetBytes;
  unsigned char* sets = smem + Lds::kTiles;
  typename F::Acc acc;
  {
    const WideSrc kv(a.K + base, a.V + base, a.N, a.st.row.stride);
    const uint8_t* keys = a.mask == nullptr ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
    fused_state_pass<F, Lds::kWaveBytes>(acc, kv, keys, a.N, quadrant * TR, 4 * TR, a.eps, sets, L, false,
                                         rows);
  }
  const float scale = a.slice_scale != nullptr ? a.slice_scale[bh] : a.scale;
  Lane Lg = L;  // the wave's place in its group
  Lg.wave = quadrant;
  ApplyArgs r{};
  r.X = a.Q + base;
  r.mask = nullptr;  // queries are not masked
  r.out = a.O + base;
  r.N = a.N;
  r.r_begin = 0;
  r.r_end = rows;
  r.stride = a.st.row.stride;
  r.scale = scale;
  r.eps = a.eps;
  WideRaw first;
  request_first_tile<4>(first, r, Lg);
  const auto own = [&](int g) { return acc.group(g); };
  quadrant_image<F, false>(own, scale, images + quadrant * F::kImageBytes, L);
  if (kept != nullptr && exists) {  // S as it is, row-major, for the caller's backward call
    float* __restrict__ out = kept + static_cast<size_t>(bh) * D * D;
    const int p = quadrant >> 1, q = quadrant & 1;
#pragma unroll
    for (int g = 0; g < F::Acc::kGroups; ++g) {
      const f32x4_t v = acc.group(g);
      const int row = p * Dh + F::Acc::group_row(g, L), col = q * Dh + F::Acc::group_col(g, L);
#pragma unroll
      for (int i = 0; i < 4; ++i) out[(row + i) * D + col] = v[i];
    }
  }
  __syncthreads();
  plain_tiles<F, 4, true, true>(r, images, sets + L.wave * Lds::kWaveBytes, Lg, &first);
}

// d loss / d log(scale) = scale <S, dS> of the slice: the dS accumulators (waves 4-7) meet the S
// accumulators (waves 0-3) in `area` (free at that point), the sum in a fixed order.  Ends with
// a barrier.
template <class F>
__device__ __forceinline__ void state_dot(const typename F::Acc& acc, bool second, float scale,
                                          unsigned char* area, float* __restrict__ out, const Lane& L) {
  const int quadrant = L.wave & 3;
  f32x4_t* meet = reinterpret_cast<f32x4_t*>(area) + quadrant * F::Acc::kGroups * 64 + L.lane;
  float* partial = reinterpret_cast<float*>(area + 4 * F::Acc::kGroups * 64 * 16);
  if (second) {
#pragma unroll
    for (int g = 0; g < F::Acc::kGroups; ++g) meet[g * 64] = acc.group(g);
  }
  __syncthreads();
  if (!second) {
    float dot = 0.0f;
#pragma unroll
    for (int g = 0; g < F::Acc::kGroups; ++g) {
      const f32x4_t s = acc.group(g), d = meet[g * 64];
#pragma unroll
      for (int i = 0; i < 4; ++i) dot += s[i] * d[i];
    }
    dot = wave_sum(dot);
    if (L.lane == 0) partial[quadrant] = dot;
  }
  __syncthreads();
  if (threadIdx.x == 0) *out = (((partial[0] + partial[1]) + partial[2]) + partial[3]) * scale;
  __syncthreads();  // the area is written again next
}

template <class F>
__global__ __launch_bounds__(512) void wide_fused_bwd_kernel(const LaunchArgs a, float* __restrict__ dlog) {
  using Lds = FusedLds<F, 2>;
  const Lane L;
  const int bh = blockIdx.x;
  const size_t base = a.st.slice_base(bh, a.H);
  unsigned char* images_a = smem;                    // S natural, later dS natural
  unsigned char* images_b = smem + Lds::kSetBytes;   // dS transposed
  unsigned char* sets = smem + Lds::kTiles;
  const int quadrant = L.wave & 3;
  const bool second = L.wave >= 4;  // waves 4-7: dS = sum_i qhat_i^T dO_i
  const uint8_t* keys = a.mask == nullptr ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
  // S is needed as natural images only: its waves sum up the transposed quadrants, unless the
  // accumulators of S and dS are to meet lane by lane for <S, dS>
  const bool swapped = !second && dlog == nullptr;
  typename F::Acc acc;
  {
    const WideSrc src((second ? a.Q : a.K) + base, (second ? a.dO : a.V) + base, a.N, a.st.row.stride);
    fused_state_pass<F, Lds::kWaveBytes>(acc, src, second ? nullptr : keys, a.N, quadrant * TR, 4 * TR,
                                         a.eps, sets, L, swapped);
  }
  const float scale = a.slice_scale != nullptr ? a.slice_scale[bh] : a.scale;
  const auto own = [&](int g) { return acc.group(g); };
  if (dlog != nullptr) state_dot<F>(acc, second, scale, sets, dlog + bh, L);
  if (swapped) quadrant_image<F, false>(own, scale, images_a + quadrant * F::kImageBytes, L);
  else if (!second) quadrant_image<F, true>(own, scale, images_a + quadrant * F::kImageBytes, L);
  else quadrant_image<F, false>(own, scale, images_b + quadrant * F::kImageBytes, L);
  __syncthreads();

  unsigned char* tiles = sets + L.wave * Lds::kWaveBytes;
  ApplyArgs r{};
  r.N = a.N;
  r.r_begin = 0;
  r.r_end = a.N;
  r.stride = a.st.row.stride;
  r.scale = scale;
  r.eps = a.eps;
  // dQ
  r.X = a.Q + base;
  r.Y = a.dO + base;
  r.mask = nullptr;
  r.out = a.dQ + base;
  projected_tiles<F, 8>(r, images_a, tiles, L);
  __syncthreads();  // nobody reads the images of S any more
  if (second) quadrant_image<F, true>(own, scale, images_a + quadrant * F::kImageBytes, L);
  // dV
  r.X = a.K + base;
  r.mask = keys;
  r.out = a.dV + base;
  plain_tiles<F, 8, false>(r, images_b, tiles, L);
  __syncthreads();  // the natural images of dS are complete
  // dK
  r.Y = a.V + base;
  r.out = a.dK + base;
  projected_tiles<F, 8>(r, images_a, tiles, L);
}

// ---- short sequences (N <= 256), backward: every tile requested at once and kept in registers -----
//
// The backward for sequences of at most 256 rows: a wave asks for all its tiles at the start
// (everything the slice needs is in flight together) and keeps them in registers, so the apply
// roles read nothing again.  Waves 0-3, which hold (K, V) tiles, compute dV and dK for them and
// waves 4-7, which hold (Q, dO) tiles, dQ; all three image sets are written as
// soon as the states are complete (LDS: [S natural | dS natural | dS transposed][per wave: two
// tiles, 16 floats]; the unit rows and the other tensor's rows of a tile take turns in the two
// tiles), and the two round buffers of the state phase lie over the same memory.
constexpr int kKeptRows = 256;

template <class F>
struct KeptLds {
  static constexpr int kSetBytes = 4 * F::kImageBytes;
  static constexpr int kTiles = 3 * kSetBytes;
  static constexpr int kWaveBytes = 2 * kTileBytes + TR * 4;
  static constexpr int kRoundWave = 4 * kTileBytes;  // state phase: two round buffers from offset 0
  static constexpr int kRoundBuffer = 8 * kRoundWave;
  static constexpr int kBytes =
      kTiles + 8 * kWaveBytes > 2 * kRoundBuffer ? kTiles + 8 * kWaveBytes : 2 * kRoundBuffer;
  static_assert(4 * F::Acc::kGroups * 64 * 16 + 64 <= kBytes, "accumulators meet in the same memory");
};

// The state phase over tiles already in registers (see fused_state_pass); `rounds`: how many of
// them hold rows of the sequence.  Two round buffers (the second `SECOND_BUFFER` bytes behind the
// first) take turns: the tiles of the next round are staged while those of this one are added
// up, one barrier per round.  Ends with a barrier (the buffers are free).
template <class F, int ROUNDS, int WAVE_BYTES, int SECOND_BUFFER>
__device__ __forceinline__ void kept_state_pass(typename F::Acc& acc, const WideRaw (&kept)[ROUNDS],
                                                int rounds, float eps, unsigned char* sets,
                                                const Lane& L, bool swapped) {
  const int quadrant = L.wave & 3, p = quadrant >> 1, q = quadrant & 1, group = L.wave >> 2;
  const int left = (swapped ? 2 + q : p) * kTileBytes, right = (swapped ? p : 2 + q) * kTileBytes;
  unsigned char* mine = sets + L.wave * WAVE_BYTES;
  acc.zero();
  float inv[2];
  stage_wide<F, mapped_mode<F>(), true>(kept[0], L, eps, mine, inv);
#pragma unroll
  for (int r = 0; r < ROUNDS; ++r) {
    if (r < rounds) {
      __syncthreads();  // round r is staged; nobody reads the other buffer any more
      if (r + 1 < ROUNDS && r + 1 < rounds)
        stage_wide<F, mapped_mode<F>(), true>(kept[r + 1 < ROUNDS ? r + 1 : 0], L, eps,
                                  mine + ((r + 1) & 1) * SECOND_BUFFER, inv);
#pragma unroll
      for (int t = 0; t < 4; ++t) {
        const unsigned char* tile = sets + (r & 1) * SECOND_BUFFER + (4 * group + t) * WAVE_BYTES;
        acc.mfma(tile + left, tile + right, L);
      }
    }
  }
  __syncthreads();
}

// The y rows of a tile, as they are, into the two tiles of a wave.
__device__ __forceinline__ void stage_y(const WideRaw& r, const Lane& L, unsigned char* tiles) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
#pragma unroll
    for (int c = 0; c < 2; ++c) *reinterpret_cast<u32x4_t*>(tiles + c * kTileBytes + off) = r.y[h][c];
  }
}

// One kept tile in the backward: xhat rows staged, then (K tiles only) dV = khat (scale dS); the y
// rows staged over them, g = y (natural images)^T and out = (g - xhat (xhat . g)) / r.
template <class F>
__device__ __forceinline__ void kept_tile_bwd(const WideRaw& t, int row0, int N, bool plain_too,
                                              const unsigned char* natural,
                                              const unsigned char* transposed,
                                              unsigned char* out_projected, unsigned char* out_plain,
                                              int stride, float eps, unsigned char* tiles,
                                              const Lane& L) {
  if (tile_dead(t)) {
    if (plain_too) store_zero_rows<F>(out_plain, row0, N, stride, L);
    store_zero_rows<F>(out_projected, row0, N, stride, L);
    return;
  }
  float* inv_slot = reinterpret_cast<float*>(tiles + 2 * kTileBytes);
  float inv[2];
  stage_wide<F, mapped_mode<F>(), false>(t, L, eps, tiles, inv);
  const float inv_r = inv_by_row(inv_slot, L, inv);
  typename F::TileRows E[2];
  E[0].load(tiles, L);
  E[1].load(tiles + kTileBytes, L);
  const int row = row0 + L.i16;
  if (plain_too) {
    const Quadrants<F, false> W(transposed, L);
#pragma unroll
    for (int q = 0; q < 2; ++q) {
      float o[2 * F::EPL];
      W.apply(E, q, 2, L, o);
      if (row < N)
        store_product_row<F, kStoreStreamed>(out_plain + q * kHalfBytes, row, RowAddr{stride, kHalfBytes}, L, o);
    }
  }
  wave_lds_fence();
  stage_y(t, L, tiles);
  wave_lds_fence();
  typename F::TileRows Y[2];
  Y[0].load(tiles, L);
  Y[1].load(tiles + kTileBytes, L);
  const Quadrants<F, false> W(natural, L);
  float g[2][2 * F::EPL];
#pragma unroll
  for (int p = 0; p < 2; ++p) W.apply(Y, 2 * p, 1, L, g[p]);
  finish_projected<F>(g, E, inv_r, L);
#pragma unroll
  for (int p = 0; p < 2; ++p) {
    if (row < N)
      store_product_row<F, kStoreStreamed>(out_projected + p * kHalfBytes, row, RowAddr{stride, kHalfBytes}, L, g[p]);
  }
  wave_lds_fence();
}

template <class F>
__global__ __launch_bounds__(512) void wide_kept_bwd_kernel(const LaunchArgs a, float* __restrict__ dlog) {
  using Lds = KeptLds<F>;
  constexpr int kRounds = kKeptRows / (4 * TR);
  const Lane L;
  const int bh = blockIdx.x;
  const size_t base = a.st.slice_base(bh, a.H);
  const int stride = a.st.row.stride;
  const int quadrant = L.wave & 3;
  const bool second = L.wave >= 4;  // waves 4-7: (Q, dO) tiles, dS = sum_i qhat_i^T dO_i, dQ
  // which 16 rows of a round the wave holds: the two waves of a SIMD (w and w + 4) take different
  // ones, so that the round with a ragged end does not leave both with a tile more than the rest
  const int slot = second ? (quadrant + 2) & 3 : quadrant;
  WideRaw kept[kRounds];
  {
    const WideSrc src((second ? a.Q : a.K) + base, (second ? a.dO : a.V) + base, a.N, stride);
    const uint8_t* m = (second || a.mask == nullptr) ? nullptr : a.mask + static_cast<size_t>(bh / a.H) * a.N;
#pragma unroll
    for (int r = 0; r < kRounds; ++r) {
      const int row0 = (4 * r + slot) * TR;
      load_wide<true>(kept[r], L, src, row0, row_bits(m, row0, a.N, L));
    }
  }
  const int rounds = (a.N + 4 * TR - 1) / (4 * TR);
  typename F::Acc acc;
  // S is needed as natural images only: its waves sum up the transposed quadrants, unless the
  // accumulators of S and dS are to meet lane by lane for <S, dS>
  const bool swapped = !second && dlog == nullptr;
  kept_state_pass<F, kRounds, Lds::kRoundWave, Lds::kRoundBuffer>(acc, kept, rounds, a.eps, smem, L, swapped);
  const float scale = a.slice_scale != nullptr ? a.slice_scale[bh] : a.scale;
  if (dlog != nullptr) state_dot<F>(acc, second, scale, smem, dlog + bh, L);
  const auto own = [&](int g) { return acc.group(g); };
  if (swapped) {
    quadrant_image<F, false>(own, scale, smem + quadrant * F::kImageBytes, L);
  } else if (!second) {
    quadrant_image<F, true>(own, scale, smem + quadrant * F::kImageBytes, L);
  } else {
    quadrant_image<F, true>(own, scale, smem + Lds::kSetBytes + quadrant * F::kImageBytes, L);
    quadrant_image<F, false>(own, scale, smem + 2 * Lds::kSetBytes + quadrant * F::kImageBytes, L);
  }
  __syncthreads();
  unsigned char* tiles = smem + Lds::kTiles + L.wave * Lds::kWaveBytes;
  const unsigned char* natural = smem + (second ? 0 : Lds::kSetBytes);
  unsigned char* out_projected = (second ? a.dQ : a.dK) + base;
#pragma unroll 1
  for (int r = 0; r < rounds; ++r) {
    const int row0 = (4 * r + slot) * TR;
    if (row0 < a.N)
      kept_tile_bwd<F>(kept[0], row0, a.N, !second, natural, smem + 2 * Lds::kSetBytes, out_projected,
                       a.dV + base, stride, a.eps, tiles, L);
#pragma unroll
    for (int k = 0; k + 1 < kRounds; ++k) kept[k] = kept[k + 1];
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
// With rows of four pieces one set of images and four tile sets fill the LDS of a compute unit:
// the apply workgroups have 4 waves and a compute unit to themselves.
constexpr int kUnits = 256;
template <int WAVES, int P = 2>
constexpr int max_lds_bytes() {
  return (WAVES == 8 || P == 4) ? 160 * 1024 : 80 * 1024;
}

template <class F, int WAVES, int P>
hipError_t states_w(const Problem& p, const Plan& plan, bool bwd) {
  constexpr int D = P * F::D;
  constexpr int lds = WAVES * 2 * P * kTileBytes;
  static_assert(lds <= max_lds_bytes<WAVES, P>(), "round buffer");
  const unsigned blocks = static_cast<unsigned>(p.B) * p.H * plan.splits;
  const size_t second = static_cast<size_t>(blocks) * D * D;
  const hipError_t err = grant_dynamic_lds(reinterpret_cast<const void*>(wide_state_kernel<F, WAVES, P>),
                                           max_lds_bytes<WAVES, P>());
  if (err != hipSuccess) return err;
  hipLaunchKernelGGL((wide_state_kernel<F, WAVES, P>), dim3(blocks, bwd ? 2 : 1), dim3(64 * WAVES), lds,
                     p.stream, static_cast<const unsigned char*>(p.Q),
                     static_cast<const unsigned char*>(p.K), static_cast<const unsigned char*>(p.V),
                     static_cast<const unsigned char*>(p.dO), p.mask, p.workspace, p.H, p.N,
                     plan.splits, plan.rows_per_split, second, p.eps, byte_strides(p));
  return hipGetLastError();
}

template <class F, int WAVES, int P>
hipError_t apply_w(const Problem& p, const Plan& plan, const float* st, const float* dst, bool bwd) {
  constexpr int lds = ApplyLds<F, WAVES, P>::kBytes;
  static_assert(lds <= max_lds_bytes<WAVES, P>(), "images and tiles");
  const LaunchArgs a = launch_args(p, plan, st, dst);
  const unsigned blocks = static_cast<unsigned>(p.B) * p.H * plan.splits;
  const void* kern = bwd ? reinterpret_cast<const void*>(wide_bwd_kernel<F, WAVES, P>)
                         : reinterpret_cast<const void*>(wide_fwd_kernel<F, WAVES, P>);
  const hipError_t err = grant_dynamic_lds(kern, max_lds_bytes<WAVES, P>());
  if (err != hipSuccess) return err;
  if (bwd)
    hipLaunchKernelGGL((wide_bwd_kernel<F, WAVES, P>), dim3(blocks, 3), dim3(64 * WAVES), lds, p.stream, a);
  else
    hipLaunchKernelGGL((wide_fwd_kernel<F, WAVES, P>), dim3(blocks), dim3(64 * WAVES), lds, p.stream, a);
  return hipGetLastError();
}

// `kinds`: workgroups per (slice, split) of the launch (states or roles)
inline bool few_workgroups(const Problem& p, const Plan& plan, int kinds) {
  return static_cast<long>(p.B) * p.H * plan.splits * kinds <= kUnits;
}

template <class F, int P>
hipError_t states(const Problem& p, const Plan& plan, bool bwd) {
  return few_workgroups(p, plan, bwd ? 2 : 1) ? states_w<F, 8, P>(p, plan, bwd)
                                              : states_w<F, 4, P>(p, plan, bwd);
}

template <class F, int P>
hipError_t apply(const Problem& p, const Plan& plan, const float* st, const float* dst, bool bwd) {
  if (P == 4) return apply_w<F, 4, P>(p, plan, st, dst, bwd);
  return few_workgroups(p, plan, bwd ? 3 : 1) ? apply_w<F, 8, 2>(p, plan, st, dst, bwd)
                                              : apply_w<F, 4, 2>(p, plan, st, dst, bwd);
}

template <class F>
hipError_t fused(const Problem& p, const Plan& plan, bool bwd) {
  static_assert(FusedLds<F, 2>::kBytes <= max_lds_bytes<8>(), "two image sets and the tile sets");
  constexpr int lds_fwd = FusedLds<F, 1>::kBytes, lds_bwd = FusedLds<F, 2>::kBytes;
  const LaunchArgs a = launch_args(p, plan, nullptr, nullptr);
  const unsigned blocks = static_cast<unsigned>(p.B) * p.H;
  if (bwd && p.N <= kKeptRows) {
    constexpr int lds_kept = KeptLds<F>::kBytes;
    static_assert(lds_kept <= max_lds_bytes<8>(), "three image sets and the tile sets");
    const hipError_t err =
        grant_dynamic_lds(reinterpret_cast<const void*>(wide_kept_bwd_kernel<F>), max_lds_bytes<8>());
    if (err != hipSuccess) return err;
    hipLaunchKernelGGL((wide_kept_bwd_kernel<F>), dim3(blocks), dim3(512), lds_kept, p.stream, a,
                       p.dlog_scale);
    return hipGetLastError();
  }
  const void* kern = bwd ? reinterpret_cast<const void*>(wide_fused_bwd_kernel<F>)
                         : reinterpret_cast<const void*>(wide_fused_fwd_kernel<F>);
  const hipError_t err = grant_dynamic_lds(kern, max_lds_bytes<8>());
  if (err != hipSuccess) return err;
  if (!bwd && blocks > static_cast<unsigned>(kUnits)) {  // two slices per workgroup
    const hipError_t e2 =
        grant_dynamic_lds(reinterpret_cast<const void*>(wide_paired_fwd_kernel<F>), max_lds_bytes<8>());
    if (e2 != hipSuccess) return e2;
    hipLaunchKernelGGL((wide_paired_fwd_kernel<F>), dim3((blocks + 1) / 2), dim3(512), lds_bwd, p.stream,
                       a, static_cast<int>(blocks), p.saved_state);
    return hipGetLastError();
  }
  if (bwd)
    hipLaunchKernelGGL((wide_fused_bwd_kernel<F>), dim3(blocks), dim3(512), lds_bwd,
                       p.stream, a, p.dlog_scale);
  else
    hipLaunchKernelGGL((wide_fused_fwd_kernel<F>), dim3(blocks), dim3(512), lds_fwd,
                       p.stream, a, p.saved_state);
  return hipGetLastError();
}

}  // namespace wide
}  // namespace

bool wide_supports(int dtype, int D) { return dtype == 0 ? (D == 64 || D == 128) : D == 128; }

namespace {
// rows of four 128-byte pieces: fp32 d_h = 128 (three-launch structure only)
inline bool four_pieces(int dtype, int D) { return dtype == 0 && D == 128; }

// fn(F{}) for the element format of the problem, with the feature map of its params
template <class Fn>
hipError_t for_format(const Problem& p, Fn fn) {
  using namespace mfma;
  if (p.feature_map == kMapElu1)
    return p.dtype == 0   ? fn(WithElu1<F32x32>{})
           : p.dtype == 1 ? fn(WithElu1<Bf16x64>{})
                          : fn(WithElu1<F16x64>{});
  return p.dtype == 0 ? fn(F32x32{}) : p.dtype == 1 ? fn(Bf16x64{}) : fn(F16x64{});
}
}  // namespace

hipError_t launch_wide_states(const Problem& p, const Plan& plan, bool bwd) {
  using namespace mfma;
  if (four_pieces(p.dtype, p.D))
    return p.feature_map == kMapElu1 ? wide::states<WithElu1<F32x32>, 4>(p, plan, bwd)
                                     : wide::states<F32x32, 4>(p, plan, bwd);
  return for_format(p, [&](auto f) { return wide::states<decltype(f), 2>(p, plan, bwd); });
}

// One launch per direction whenever the sequence is not cut - except a backward over so few
// slices that its three roles as workgroups of their own are what fills the chip (64 slices of
// 200 rows, bf16 d_h = 128: 17.5 us against 19.4 us in one launch; the forward: 13.8 against 10.0),
// and except rows of four pieces, for which only the three-launch kernels exist.
bool wide_fused_applies(int dtype, int D, int B, int H, int splits, bool bwd) {
  return !four_pieces(dtype, D) && splits == 1 && !(bwd && static_cast<long>(B) * H * 3 <= wide::kUnits);
}

hipError_t launch_wide_fused(const Problem& p, const Plan& plan, bool bwd) {
  if (!wide_fused_applies(p.dtype, p.D, p.B, p.H, plan.splits, bwd)) return hipErrorInvalidValue;
  return for_format(p, [&](auto f) { return wide::fused<decltype(f)>(p, plan, bwd); });
}

hipError_t launch_wide_apply(const Problem& p, const Plan& plan, const float* states,
                             const float* dstates, bool bwd) {
  using namespace mfma;
  if (four_pieces(p.dtype, p.D))
    return p.feature_map == kMapElu1 ? wide::apply<WithElu1<F32x32>, 4>(p, plan, states, dstates, bwd)
                                     : wide::apply<F32x32, 4>(p, plan, states, dstates, bwd);
  return for_format(p, [&](auto f) { return wide::apply<decltype(f), 2>(p, plan, states, dstates, bwd); });
}

}  // namespace cotten
