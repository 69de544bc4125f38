// Resident kernels for short sequences of 16-bit elements (bf16 or fp16, N <= 208, d_h = 64).
//
// One persistent workgroup of 16 waves owns one slice at a time and keeps it in LDS: wave w
// loads and stages the 16-row tile w, so every global load of the slice is issued at once and
// nothing is read twice; the loads of the workgroup's next slice are issued as soon as the
// registers are free and travel while the current slice is worked on.  The d x d states are
// built by one wave per output block, each walking all resident tiles (no cross-wave
// reduction), and handed on as MFMA operand images in LDS.  Apply products are shared out
// over the waves by tile; their epilogue runs in the layout the product comes out in, next to
// the tile rows fetched from LDS in that same layout, and ends in 128-bit stores.
//
//   forward    stage K, V, Q | barrier | 4 waves: S | barrier | wave w: O rows of tile w
//   backward   see resident_bwd_kernel (dS is built while dQ is applied)
#include "cotten_launch.h"
#include "cotten_mfma_core.h"

namespace cotten {
namespace {

using namespace mfma;

constexpr int kWaves = 16;
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxTiles = 13;                  // N <= 208
constexpr int kBlockBytes = 4 * kTileBytes;    // [khat | v | q(hat) | dO] tiles of 16 rows
constexpr int kKt = 0, kVt = kTileBytes, kQt = 2 * kTileBytes, kGt = 3 * kTileBytes;

template <class F>
struct Lds {
  static constexpr int kImages = kMaxTiles * kBlockBytes;          // three operand images
  static constexpr int kLive = kImages + 3 * F::kImageBytes;       // one int per tile
  static constexpr int kInv = kLive + 16 * 4;                      // 1/r per tile: 16 q rows, 16 k rows
  static constexpr int kDots = kInv + kMaxTiles * 2 * TR * 4;     // <S, dS> per state block
  static constexpr int kBytes = kDots + 4 * 4;
};

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

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
  int H, N, slices;
  Strides st;
  float scale, eps;
  const float* scales;  // per-slice scale, or nullptr
  float* dlog;          // backward: <S, dS> per slice, or nullptr
  // S = sum_j m_j khat_j^T v_j of every slice as the caller keeps it from the forward to the
  // backward call ([slices][d][d] floats, row-major, without the scale), or nullptr
  float* saved;
  int d;                // head dimension (states are D x D, zero beyond d)
  // causal variant on sequences cut into chunks of kMaxTiles tiles: workgroup = (slice, chunk);
  // [slice][chunk][D*D] floats each, row-major, without the scale
  int chunks;
  const float* before;  // sum over the chunks before this one of khat^T v   (chunks > 1)
  const float* after;   // sum over the chunks after this one of qhat^T dO   (chunks > 1, backward)
};

// The wave's tile: rows 16*tile + r8 + 8h.  `want` bit h: the row takes part.
template <bool USE_Y>
__device__ __forceinline__ void load_tile(Raw& r, const Lane& L, const Src& src, int tile,
                                          int want) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = tile * TR + L.r8 + 8 * h;
    const uint32_t off =
        src.offset(row, (want >> h) & 1, L);
    r.x[h] = __builtin_amdgcn_raw_buffer_load_b128(src.x, off, 0, 0);
    if (USE_Y) r.y[h] = __builtin_amdgcn_raw_buffer_load_b128(src.y, off, 0, 0);
    else r.y[h] = u32x4_t{0, 0, 0, 0};
  }
  r.live = want;
}

// Valid-key bits of the wave's tile in a slice (bit h: row 16*tile + r8 + 8h); all rows
// count when there is no mask, none when the slice does not exist.
__device__ __forceinline__ int key_rows(const Args& a, const Lane& L, int slice, int tile) {
  if (slice >= a.slices) return 0;
  if (a.mask == nullptr) return 3;
  const uint8_t* mask = a.mask + static_cast<size_t>(slice / a.H) * a.N;
  int keys = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = tile * TR + L.r8 + 8 * h;
    if (row < a.N) keys |= static_cast<int>(mask[row] != 0) << h;
  }
  return keys;
}

// Issues the loads of the wave's tile of `slice` (none, at no cost, if the slice or the tile
// does not exist): PARTS bit 0 = K and V, of which rows that are not valid keys are not read;
// bit 1 = Q (and dO).
template <bool BWD, int PARTS = 3>
__device__ __forceinline__ void fetch(Raw& rq, Raw& rk, const Args& a, const Lane& L, int slice,
                                      int tile, int keys) {
  const bool ok = slice < a.slices;
  const size_t base = ok ? a.st.slice_base(slice, a.H) : 0;
  int rows = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h)
    rows |= static_cast<int>(ok && tile * TR + L.r8 + 8 * h < a.N) << h;
  if (PARTS & 1) {
    const Src kv_src(a.K + base, a.V + base, a.N, a.st.row);
    load_tile<true>(rk, L, kv_src, tile, rows & keys);
  }
  if (PARTS & 2) {
    const Src q_src(a.Q + base, (BWD ? a.dO : a.Q) + base, a.N, a.st.row);
    load_tile<BWD>(rq, L, q_src, tile, rows);
  }
}

// 1/r of the 16 tile rows, from the load layout to where any wave can pick them up by row.
__device__ __forceinline__ void publish_inv(float* dst, const Lane& L, const float (&inv)[2]) {
  if (L.ch == 0) {
    dst[L.r8] = inv[0];
    dst[L.r8 + 8] = inv[1];
  }
}

// One wave per state block: walks all kMaxTiles resident tiles and then writes its block into
// the images.  Tiles that contribute nothing must hold zeros.  The operands of the next
// kAhead tiles are requested from LDS before the matrix cores start on a tile (the scheduler
// is held to that order: left alone it funnels every tile through one register set, and each
// LDS read then waits for the product before it).
// Images are written with wide stores from an accumulator that holds the block the other way
// round: the natural image needs the transposed block, i.e. the operands swapped (a second
// accumulation, far cheaper than narrow image writes).
template <class F, bool NATURAL, bool TRANSPOSED>
__device__ __forceinline__ void build_state(const Lane& L, int block, int x_off, int y_off,
                                            float scale, unsigned char* natural,
                                            unsigned char* transposed,
                                            const unsigned char* other_natural = nullptr,
                                            float* dot_out = nullptr, float* save_to = nullptr,
                                            int d = 0) {
  typedef typename F::BlockAcc Acc;
  constexpr int kAhead = 3;
  static_assert(kAhead < kMaxTiles, "prefetch depth");
  Acc acc_t, acc_n;
  acc_t.zero();
  acc_n.zero();
  typename Acc::Frag ring[kAhead];
#pragma unroll
  for (int t = 0; t < kAhead; ++t)
    ring[t] = Acc::fetch(smem + t * kBlockBytes + x_off, smem + t * kBlockBytes + y_off, L, block);
#pragma unroll
  for (int t = 0; t < kMaxTiles; ++t) {
    const typename Acc::Frag f = ring[t % kAhead];
    __builtin_amdgcn_sched_barrier(0);
    if (t + kAhead < kMaxTiles) {
      const unsigned char* blk = smem + (t + kAhead) * kBlockBytes;
      ring[t % kAhead] = Acc::fetch(blk + x_off, blk + y_off, L, block);
    }
    __builtin_amdgcn_sched_barrier(0);
    if (TRANSPOSED) acc_t.mma(f);
    if (NATURAL) acc_n.mma_swapped(f);
  }
  const int r0 = Acc::block_row0(block), c0 = Acc::block_col0(block);
  if (TRANSPOSED) acc_t.write_image(L, r0, c0, scale, transposed);
  if (NATURAL) acc_n.write_image(L, c0, r0, scale, natural);
  // the block as it is (fp32, unscaled) into the caller's d x d array: the lane holds column
  // c0 + lane%32 of rows r0 + 8j + 4*(lane/32) .. +3, so 32 lanes write 128 contiguous bytes
  if (TRANSPOSED && save_to != nullptr) {
    const int c = c0 + (L.lane & 31);
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int r = r0 + 8 * j + 4 * (L.lane >> 5) + v;
        if (r < d && c < d) save_to[r * d + c] = acc_t.v[4 * j + v];
      }
  }
  // <this state, the state whose natural image is given>, this wave's block of it
  if (NATURAL && dot_out != nullptr) {
    const float dot = wave_sum(acc_n.dot_image(L, c0, r0, other_natural));
    if (L.lane == 0) *dot_out = dot;
  }
}

// Zero rows for the two tiles at Xt and Yt.
__device__ __forceinline__ void clear_tiles(const Lane& L, unsigned char* Xt, unsigned char* Yt) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
    *reinterpret_cast<u32x4_t*>(Xt + off) = u32x4_t{0, 0, 0, 0};
    *reinterpret_cast<u32x4_t*>(Yt + off) = u32x4_t{0, 0, 0, 0};
  }
}

// Both kernels are persistent: a workgroup takes slices blockIdx.x, blockIdx.x + gridDim.x, ...
// and, as soon as one slice is staged in LDS, issues the loads of its next one, which then
// travel while the states are built and the products applied.

template <class F>
__global__ __launch_bounds__(kThreads) void resident_fwd_kernel(const Args a) {
  const Lane L0;
  const int N = a.N, tile = L0.wave, stride = gridDim.x;
  const int n_tiles = (N + TR - 1) / TR;
  unsigned char* blk = smem + tile * kBlockBytes;
  unsigned char* img = smem + Lds<F>::kImages;
  float* invs = reinterpret_cast<float*>(smem + Lds<F>::kInv) + tile * 2 * TR;
  const bool mine = tile < n_tiles;
  if (!mine && tile < kMaxTiles) {  // absent tiles stay zero for the whole kernel
    clear_tiles(L0, blk + kKt, blk + kVt);
    clear_tiles(L0, blk + kQt, blk + kGt);
  }

  int slice = blockIdx.x;
  Raw rq, rk;
  // The first slice: only K and V are requested at once (every compute unit asks at the same
  // moment, and the first phase needs nothing else); Q follows when those have arrived.
  fetch<false, 1>(rq, rk, a, L0, slice, tile, key_rows(a, L0, slice, tile));
  int keys = key_rows(a, L0, slice + stride, tile);
  // Per slice (B = workgroup barrier):
  //   1  tile waves stage K, V                                                       B
  //   2  waves 12-15 build S (at raised priority: everyone waits for it); tile waves
  //      stage Q and issue the loads of the next slice                               B
  //   3  wave w finishes the O rows of tile w (phase 1 of the next slice may start at once:
  //      it writes only the K, V tiles, which nobody reads any more)
  for (int iter = 0; slice < a.slices; slice += stride, ++iter) {
    {
      const Lane L = L0.again();
      if (mine) {
        float inv[2];
        if (__ballot(rk.live != 0) != 0)
          stage<F, kXNormalized, true>(rk, L, a.eps, blk + kKt, blk + kVt, inv);
        else
          clear_tiles(L, blk + kKt, blk + kVt);
      }
      if (iter == 0) fetch<false, 2>(rq, rk, a, L, slice, tile, 0);
    }
    __syncthreads();
    {
      const Lane L = L0.again();
      constexpr int kB = F::BlockAcc::kBlocks;
      if (tile >= kWaves - kB) {  // O = qhat S: contraction over rows of S -> transposed image
        __builtin_amdgcn_s_setprio(3);
        const float scale = a.scales != nullptr ? a.scales[slice] : a.scale;
        build_state<F, false, true>(
            L, tile - (kWaves - kB), kKt, kVt, scale, nullptr, img, nullptr, nullptr,
            a.saved != nullptr ? a.saved + static_cast<size_t>(slice) * a.d * a.d : nullptr, a.d);
        __builtin_amdgcn_s_setprio(0);
      }
      if (mine) {
        float inv[2];
        stage<F, kXRaw, false>(rq, L, a.eps, blk + kQt, blk + kGt, inv);
        publish_inv(invs, L, inv);
        fetch<false>(rq, rk, a, L, slice + stride, tile, keys);
        keys = key_rows(a, L, slice + 2 * stride, tile);
      }
    }
    __syncthreads();
    if (mine) {
      const Lane L = L0.again();
      typename F::TileRows xq;
      xq.load(blk + kQt, L);
      const float inv_r = invs[L.i16];
      typename F::Operand W;
      W.load(img, L);
      f32x4_t out[F::NT];
      F::apply(xq, W, out);
      float o[2 * F::EPL];
      product_rows<F>(out, o);
#pragma unroll
      for (int i = 0; i < 2 * F::EPL; ++i) o[i] *= inv_r;
      const int row = tile * TR + L.i16;
      if (row < N)
        store_product_row<F, kStoreStreamed>(a.O + a.st.slice_base(slice, a.H), row, a.st.row, L, o);
    }
  }
}

// One tile of an apply product, finished and stored:
//   kind 0  dQ = (g - qhat (qhat.g)) / r_q,  g = dO W      (W = scale * S, natural image)
//   kind 1  dV = khat W                                     (W = scale * dS, transposed image;
//                                                            khat is zero on masked rows)
//   kind 2  dK = (h - khat (khat.h)) / r_k,  h = v W       (W = scale * dS, natural image;
//                                                            1/r_k is zero on masked rows)
// Tiles without a valid key get zero rows of dK and dV without touching LDS.
template <class F>
__device__ __forceinline__ void apply_tile(const Lane& L, int kind, int t, int N,
                                           const typename F::Operand& W, const int* live,
                                           const float* invs, unsigned char* dst,
                                           RowAddr row_addr) {
  const unsigned char* tb = smem + t * kBlockBytes;
  const int row = t * TR + L.i16;
  float p[2 * F::EPL];
  if (kind != 0 && live[t] == 0) {
#pragma unroll
    for (int c = 0; c < 2 * F::EPL; ++c) p[c] = 0.0f;
  } else {
    typename F::TileRows x;
    x.load(tb + (kind == 0 ? kGt : kind == 1 ? kKt : kVt), L);
    f32x4_t out[F::NT];
    F::apply(x, W, out);
    product_rows<F>(out, p);
    if (kind != 1) {
      typename F::TileRows e;
      e.load(tb + (kind == 0 ? kQt : kKt), L);
      project_rows<F, true>(p, e, invs[t * 2 * TR + (kind == 0 ? 0 : TR) + L.i16], L);
    }
  }
  if (row < N) store_product_row<F, kStoreStreamed>(dst, row, row_addr, L, p);
}

// Backward, per slice (B = workgroup barrier):
//   1  tile waves stage Q, dO and request Q, dO of the next slice                    B
//   2  waves 12-15 build dS (one block each, at raised priority: everyone waits for it);
//      tile waves stage K, V and request K, V of the next slice                      B
//   3  waves 12-15 build S;  waves 0-11 apply dV and dK, which need only dS: waves 2i, 2i+1
//      take tiles i, i+6, i+12, one product each, so that every SIMD gets both kinds    B
//   4  wave w applies dQ of tile w                                                    B
template <class F>
__global__ __launch_bounds__(kThreads) void resident_bwd_kernel(const Args a) {
  const Lane L0;
  const int N = a.N, tile = L0.wave, stride = gridDim.x;
  const int n_tiles = (N + TR - 1) / TR;
  unsigned char* blk = smem + tile * kBlockBytes;
  unsigned char* img_s = smem + Lds<F>::kImages;              // scale * S, natural
  unsigned char* img_ds = img_s + F::kImageBytes;             // scale * dS, natural
  unsigned char* img_dst = img_ds + F::kImageBytes;           // scale * dS, transposed
  int* live = reinterpret_cast<int*>(smem + Lds<F>::kLive);
  float* invs = reinterpret_cast<float*>(smem + Lds<F>::kInv);
  const bool mine = tile < n_tiles;
  if (!mine && tile < kMaxTiles) {  // absent tiles stay zero for the whole kernel
    clear_tiles(L0, blk + kKt, blk + kVt);
    clear_tiles(L0, blk + kQt, blk + kGt);
  }
  constexpr int kB = F::BlockAcc::kBlocks, kApplyWaves = kWaves - kB;
  static_assert(kB == 4 && kWaves == 16 && kMaxTiles <= 16, "wave roles below");
  const int kv_kind = 1 + ((tile + (tile >> 2)) & 1);  // phase 3: dV or dK

  int slice = blockIdx.x;
  Raw rq, rk;
  // Loads are requested as early as the registers that receive them are free: everything of the
  // first slice at once, Q and dO of the next slice as soon as those of the current one are
  // staged, its K and V as soon as the current ones are (measured against requesting the next
  // slice in one go after phase 2, and K, V of the first slice only after Q, dO: 18.3 against
  // 21.0 us at 512 slices of 200 rows).
  const int first_keys = key_rows(a, L0, slice, tile);
  fetch<true>(rq, rk, a, L0, slice, tile, first_keys);
  int keys = key_rows(a, L0, slice + stride, tile);
  float* dots = reinterpret_cast<float*>(smem + Lds<F>::kDots);
  for (int iter = 0; slice < a.slices; slice += stride, ++iter) {
    const size_t base = a.st.slice_base(slice, a.H);
    const float scale = a.scales != nullptr ? a.scales[slice] : a.scale;
    {
      const Lane L = L0.again();
      if (mine) {
        float inv[2];
        stage<F, kXNormalized, true>(rq, L, a.eps, blk + kQt, blk + kGt, inv);
        publish_inv(invs + tile * 2 * TR, L, inv);
      }
      // Q, dO of the next slice are requested as soon as their registers are free
      if (mine) fetch<true, 2>(rq, rk, a, L, slice + stride, tile, 0);
    }
    __syncthreads();
    {
      const Lane L = L0.again();
      if (tile >= kApplyWaves) {
        // dV = khat dS -> transposed image;  h = v dS^T -> natural image
        __builtin_amdgcn_s_setprio(3);  // the other waves wait for this at the next barrier
        build_state<F, true, true>(L, tile - kApplyWaves, kQt, kGt, scale, img_ds, img_dst);
        __builtin_amdgcn_s_setprio(0);
      }
      if (mine) {
        // A tile without a valid key adds nothing to S, and its dK, dV rows are plain zeros.
        const bool any_key = __ballot(rk.live != 0) != 0;
        if (any_key) {
          float inv[2];
          stage<F, kXNormalized, true>(rk, L, a.eps, blk + kKt, blk + kVt, inv);
          publish_inv(invs + tile * 2 * TR + TR, L, inv);
        } else {
          clear_tiles(L, blk + kKt, blk + kVt);
        }
        if (L.lane == 0) live[tile] = any_key;
        fetch<true, 1>(rq, rk, a, L, slice + stride, tile, keys);
        keys = key_rows(a, L, slice + 2 * stride, tile);
      }
    }
    __syncthreads();
    if (tile >= kApplyWaves) {
      // g = dO S^T: contraction over columns of S -> natural image.  With dlog wanted: this
      // block of <sum_j khat_j^T v_j, scale * dS (its image)>
      const Lane L = L0.again();
      __builtin_amdgcn_s_setprio(3);
      build_state<F, true, false>(L, tile - kApplyWaves, kKt, kVt, scale, img_s, nullptr, img_ds,
                     a.dlog != nullptr ? dots + (tile - kApplyWaves) : nullptr);
      __builtin_amdgcn_s_setprio(0);
    } else {
      const Lane L = L0.again();
      typename F::Operand W;
      W.load(kv_kind == 1 ? img_dst : img_ds, L);
      unsigned char* dst = (kv_kind == 1 ? a.dV : a.dK) + base;
#pragma unroll 1
      for (int t = tile >> 1; t < n_tiles; t += kApplyWaves / 2)
        apply_tile<F>(L, kv_kind, t, N, W, live, invs, dst, a.st.row);
    }
    __syncthreads();
    // d loss / d log(scale) = sum_i dO_i . O_i = <S, scale * dS>, blocks in order
    if (a.dlog != nullptr && threadIdx.x == 0)
      a.dlog[slice] = ((dots[0] + dots[1]) + dots[2]) + dots[3];
    if (mine) {
      const Lane L = L0.again();
      typename F::Operand W;
      W.load(img_s, L);
      apply_tile<F>(L, 0, tile, N, W, live, invs, a.dQ + base, a.st.row);
    }
    __syncthreads();  // the tiles and images are rewritten for the next slice
  }
}

// ---- causal variant on the matrix cores ------------------------------------------------------
// Row i attends the valid keys j <= i.  With the whole slice in LDS this is done tile pair by
// tile pair, (query tile t, key tile u <= t), all pairs independent:
//
//     P^T  = Khat_u Q_t^T          16 keys x 16 queries, two 16x16x32 MFMAs (contraction over d)
//     O_t^T += V_u^T P^T           16x16x16 MFMAs, one per 16 output columns
//
// A 16x16 MFMA result leaves lane (j, g) with rows 4g .. 4g+3 of column j - exactly the k a
// lane of a 16x16x16 B operand holds - so P (rounded to the element type, diagonal tile cut to
// its lower triangle) goes into the second product without moving between lanes; the A
// operand V_u^T comes from the transposing LDS read, with its columns picked so that the
// result lands in the product layout of the other kernels.  Wave t owns query tile t (and,
// in the backward, key tile t: t + 1 pairs in one role, n - t in the other, the same work for
// every wave).  Backward, with G^T = V_u dO_t^T on the same support:
//     dQhat_t^T += Khat_u^T G^T                         (as query tile t, over u <= t)
//     dV_u^T    += dO_t^T P,    H_u^T += Qhat_t^T G     (as key tile u, over t >= u)
// and the row-norm Jacobians as everywhere else.
//
// Longer sequences are cut into chunks of kMaxTiles tiles, one workgroup per chunk, wave w on
// tile w of the chunk.  The pairs inside the chunk are done as above; everything before the
// chunk reaches its queries through one state, S_before = sum of khat^T v over the earlier
// chunks (O_t += Q_t S_before, dQhat_t += dO_t S_before^T), and its keys are reached by everything
// after the chunk through T_after = sum of qhat^T dO over the later chunks (dV_u += Khat_u T_after,
// H_u += V_u T_after^T): apply products against operand images, as in the bidirectional kernels.

// The 2 x 2 block of a row-major D x D state in global memory that a thread carries into the
// operand images (threads beyond D*D/4 carry nothing).
template <class F>
struct StateBlock {
  float v[2][2];
  __device__ __forceinline__ void fetch(const float* __restrict__ M) {
    const int e = threadIdx.x;
    if (e >= F::D * F::D / 4) return;
    const int m = 2 * (e / (F::D / 2)), n = 2 * (e % (F::D / 2));
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const float2 r = *reinterpret_cast<const float2*>(M + (m + i) * F::D + n);
      v[i][0] = r.x;
      v[i][1] = r.y;
    }
  }
  // natural: op[m][n] = M[m][n] (products contracting over n); transposed: op[n][m] = M[m][n]
  __device__ __forceinline__ void write(unsigned char* natural, unsigned char* transposed) const {
    const int e = threadIdx.x;
    if (e >= F::D * F::D / 4) return;
    const int m = 2 * (e / (F::D / 2)), n = 2 * (e % (F::D / 2));
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      if (natural != nullptr) F::write_image_pair(natural, m + i, n, v[i][0], v[i][1]);
      if (transposed != nullptr) F::write_image_pair(transposed, n + i, m, v[0][i], v[1][i]);
    }
  }
};

// Which slice and chunk a workgroup of the causal kernels works on, and the wave's tile.
struct ChunkId {
  int slice, chunk, tile;  // tile: of the slice
  size_t state;            // offset of the chunk's states in Args::before / Args::after
  __device__ __forceinline__ ChunkId(const Args& a, int wave, int dd) {
    slice = blockIdx.x / a.chunks;
    chunk = blockIdx.x % a.chunks;
    tile = chunk * kMaxTiles + wave;
    state = static_cast<size_t>(blockIdx.x) * dd;
  }
};

template <class F>
__global__ __launch_bounds__(kThreads) void causal_fwd_kernel(const Args a) {
  const Lane L0;
  const ChunkId id(a, L0.wave, F::D * F::D);
  const int N = a.N, tile = L0.wave, slice = id.slice;
  const int n_tiles = (N + TR - 1) / TR;
  unsigned char* blk = smem + tile * kBlockBytes;
  unsigned char* image = smem + Lds<F>::kImages;
  int* live = reinterpret_cast<int*>(smem + Lds<F>::kLive);
  float* invs = reinterpret_cast<float*>(smem + Lds<F>::kInv) + tile * 2 * TR;
  const bool mine = tile < kMaxTiles && id.tile < n_tiles;  // the other waves only help with the image
  const bool carried = id.chunk > 0;  // uniform over the workgroup
  StateBlock<F> before;
  if (carried) before.fetch(a.before + id.state);
  Raw rq, rk;
  const int from = mine ? slice : a.slices;  // a slice that does not exist: nothing is loaded
  fetch<false>(rq, rk, a, L0, from, id.tile, key_rows(a, L0, from, id.tile));
  if (carried) before.write(nullptr, image);  // O = q S: contraction over the rows of S
  if (mine) {
    float inv[2];
    const bool any_key = __ballot(rk.live != 0) != 0;
    if (any_key) stage<F, kXNormalized, true>(rk, L0, a.eps, blk + kKt, blk + kVt, inv);
    if (L0.lane == 0) live[tile] = any_key;
    stage<F, kXRaw, false>(rq, L0, a.eps, blk + kQt, blk + kGt, inv);
    publish_inv(invs, L0, inv);
  }
  __syncthreads();
  if (!mine) return;
  const Lane L = L0.again();
  typename F::TileRows xq;
  xq.load(blk + kQt, L);
  f32x4_t out[F::NT];
  if (carried) {
    typename F::Operand S;
    S.load(image, L);
    F::apply(xq, S, out);
  } else {
#pragma unroll
    for (int nt = 0; nt < F::NT; ++nt) out[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  }
  for (int u = 0; u <= tile; ++u) {
    if (live[u] == 0) continue;  // no valid key in the tile (uniform)
    const unsigned char* ub = smem + u * kBlockBytes;
    typename F::TileRows xk;
    xk.load(ub + kKt, L);
    f32x4_t pt = F::dots(xk, xq);  // [key 4g+v][query i16]
    if (u == tile) {
#pragma unroll
      for (int v = 0; v < 4; ++v)
        if (4 * L.g16 + v > L.i16) pt[v] = 0.0f;
    }
    F::add_transposed_product(ub + kVt, L, pt, out);
  }
  float o[2 * F::EPL];
  product_rows<F>(out, o);
  const float factor = invs[L.i16] * (a.scales != nullptr ? a.scales[slice] : a.scale);
#pragma unroll
  for (int i = 0; i < 2 * F::EPL; ++i) o[i] *= factor;
  const int row = id.tile * TR + L.i16;
  if (row < N)
    store_product_row<F, kStoreStreamed>(a.O + a.st.slice_base(slice, a.H), row, a.st.row, L, o);
}

template <class F>
__global__ __launch_bounds__(kThreads) void causal_bwd_kernel(const Args a) {
  const Lane L0;
  const ChunkId id(a, L0.wave, F::D * F::D);
  const int N = a.N, tile = L0.wave, slice = id.slice;
  const int n_tiles = (N + TR - 1) / TR;
  // the tiles of the chunk that exist: the partners of a key tile end there
  const int chunk_tiles = n_tiles - id.chunk * kMaxTiles < kMaxTiles ? n_tiles - id.chunk * kMaxTiles
                                                                      : kMaxTiles;
  unsigned char* blk = smem + tile * kBlockBytes;
  unsigned char* image_s = smem + Lds<F>::kImages;         // S_before, natural
  unsigned char* image_tv = image_s + F::kImageBytes;      // T_after, transposed
  unsigned char* image_th = image_tv + F::kImageBytes;     // T_after, natural
  int* live = reinterpret_cast<int*>(smem + Lds<F>::kLive);
  float* invs = reinterpret_cast<float*>(smem + Lds<F>::kInv) + tile * 2 * TR;
  const bool mine = tile < chunk_tiles;  // the other waves only help with the images
  const bool carried = id.chunk > 0, followed = id.chunk < a.chunks - 1;  // uniform
  StateBlock<F> before, after;
  if (carried) before.fetch(a.before + id.state);
  if (followed) after.fetch(a.after + id.state);
  Raw rq, rk;
  const int from = mine ? slice : a.slices;  // a slice that does not exist: nothing is loaded
  fetch<true>(rq, rk, a, L0, from, id.tile, key_rows(a, L0, from, id.tile));
  if (carried) before.write(image_s, nullptr);    // dO S^T: contraction over the columns of S
  if (followed) after.write(image_th, image_tv);  // v T^T over columns, khat T over rows
  if (mine) {
    float inv[2];
    stage<F, kXNormalized, true>(rq, L0, a.eps, blk + kQt, blk + kGt, inv);
    publish_inv(invs, L0, inv);
    const bool any_key = __ballot(rk.live != 0) != 0;
    if (any_key) {
      stage<F, kXNormalized, true>(rk, L0, a.eps, blk + kKt, blk + kVt, inv);
      publish_inv(invs + TR, L0, inv);
    }
    if (L0.lane == 0) live[tile] = any_key;
  }
  __syncthreads();
  if (!mine) return;
  const Lane L = L0.again();
  const size_t base = a.st.slice_base(slice, a.H);
  const float scale = a.scales != nullptr ? a.scales[slice] : a.scale;
  const int row = id.tile * TR + L.i16;

  {  // as query tile: dQ
    typename F::TileRows xg;
    xg.load(blk + kGt, L);
    f32x4_t acc[F::NT];
    if (carried) {
      typename F::Operand S;
      S.load(image_s, L);
      F::apply(xg, S, acc);
    } else {
#pragma unroll
      for (int nt = 0; nt < F::NT; ++nt) acc[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
    }
    for (int u = 0; u <= tile; ++u) {
      if (live[u] == 0) continue;
      const unsigned char* ub = smem + u * kBlockBytes;
      typename F::TileRows xv;
      xv.load(ub + kVt, L);
      f32x4_t gt = F::dots(xv, xg);  // [key 4g+v][query i16] = v_key . dO_query
      if (u == tile) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
          if (4 * L.g16 + v > L.i16) gt[v] = 0.0f;
      }
      F::add_transposed_product(ub + kKt, L, gt, acc);
    }
    float g[2 * F::EPL];
    product_rows<F>(acc, g);
#pragma unroll
    for (int i = 0; i < 2 * F::EPL; ++i) g[i] *= scale;
    typename F::TileRows e;
    e.load(blk + kQt, L);
    project_rows<F, false>(g, e, invs[L.i16], L);
    if (row < N) store_product_row<F, kStoreStreamed>(a.dQ + base, row, a.st.row, L, g);
  }

  {  // as key tile: dK, dV
    float dk[2 * F::EPL], dv[2 * F::EPL];
    if (live[tile] == 0) {
#pragma unroll
      for (int i = 0; i < 2 * F::EPL; ++i) dk[i] = dv[i] = 0.0f;
    } else {
      typename F::TileRows xk, xv;
      xk.load(blk + kKt, L);
      xv.load(blk + kVt, L);
      f32x4_t av[F::NT], ah[F::NT];
      if (followed) {
        typename F::Operand T;
        T.load(image_tv, L);
        F::apply(xk, T, av);
        T.load(image_th, L);
        F::apply(xv, T, ah);
      } else {
#pragma unroll
        for (int nt = 0; nt < F::NT; ++nt) av[nt] = ah[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
      }
      for (int t = tile; t < chunk_tiles; ++t) {
        const unsigned char* tb = smem + t * kBlockBytes;
        typename F::TileRows xq, xg;
        xq.load(tb + kQt, L);
        xg.load(tb + kGt, L);
        f32x4_t p = F::dots(xq, xk);   // [query 4g+v][key i16] = qhat_query . khat_key
        f32x4_t gg = F::dots(xg, xv);  // [query 4g+v][key i16] = dO_query . v_key
        if (t == tile) {
#pragma unroll
          for (int v = 0; v < 4; ++v)
            if (L.i16 > 4 * L.g16 + v) p[v] = gg[v] = 0.0f;
        }
        F::add_transposed_product(tb + kGt, L, p, av);
        F::add_transposed_product(tb + kQt, L, gg, ah);
      }
      product_rows<F>(av, dv);
      product_rows<F>(ah, dk);
#pragma unroll
      for (int i = 0; i < 2 * F::EPL; ++i) {
        dv[i] *= scale;
        dk[i] *= scale;
      }
      // 1/r is zero on masked rows, whose khat and v rows are zero too: exact zeros there
      project_rows<F, false>(dk, xk, invs[TR + L.i16], L);
      if (invs[TR + L.i16] == 0.0f) {
#pragma unroll
        for (int i = 0; i < 2 * F::EPL; ++i) dv[i] = 0.0f;
      }
    }
    if (row < N) {
      store_product_row<F, kStoreStreamed>(a.dK + base, row, a.st.row, L, dk);
      store_product_row<F, kStoreStreamed>(a.dV + base, row, a.st.row, L, dv);
    }
  }
}

// Persistent workgroups: one per compute unit of the current device (the LDS admits no second
// one), 256 on MI355X.  Asked once per device.
int compute_units() {
  constexpr int kMaxDevices = 64;
  static int cached[kMaxDevices] = {};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return 256;
  if (cached[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cached[dev] = n;
  }
  return cached[dev];
}

Args make_args(const Problem& p) {
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
  a.H = p.H;
  a.N = p.N;
  a.slices = p.B * p.H;
  a.st = Strides{p.stride_batch * p.elem_bytes(), p.stride_head * p.elem_bytes(),
                 RowAddr{static_cast<int>(p.stride_row * p.elem_bytes()),
                         static_cast<int>(p.D * p.elem_bytes())}};
  a.scale = p.scale;
  a.eps = p.eps;
  a.scales = p.slice_scale;
  a.dlog = p.dlog_scale;
  a.saved = p.saved_state;
  a.d = p.D;
  return a;
}

template <class F>
hipError_t run(const Problem& p, bool bwd) {
  const Args a = make_args(p);
  const int units = compute_units();
  const dim3 grid(static_cast<unsigned>(a.slices < units ? a.slices : units));
  const size_t lds = Lds<F>::kBytes;
  // The backward never reads a kept state here: with the slice in LDS K and V are fetched once
  // whether S is rebuilt or not, and reading d x d floats per slice would only add traffic (at
  // d = 64 and 200 rows the state is 16 KB next to 25 KB per tensor: measured 23.1 against
  // 18.4 us at 512 slices).
  const void* kern = bwd ? reinterpret_cast<const void*>(resident_bwd_kernel<F>)
                         : reinterpret_cast<const void*>(resident_fwd_kernel<F>);
  const hipError_t err = grant_dynamic_lds(kern, static_cast<int>(lds));
  if (err != hipSuccess) return err;
  if (bwd)
    hipLaunchKernelGGL(resident_bwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  else
    hipLaunchKernelGGL(resident_fwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  return hipGetLastError();
}

}  // namespace

template <class F>
hipError_t run_causal(const Problem& p, bool bwd, int chunks) {
  Args a = make_args(p);
  a.chunks = chunks;
  if (chunks > 1) {
    if (p.workspace == nullptr) return hipErrorInvalidValue;
    a.before = p.workspace;
    a.after = p.workspace + static_cast<size_t>(a.slices) * chunks * F::D * F::D;
  }
  const dim3 grid(static_cast<unsigned>(a.slices) * chunks);
  const size_t lds = Lds<F>::kBytes;
  const void* kern = bwd ? reinterpret_cast<const void*>(causal_bwd_kernel<F>)
                         : reinterpret_cast<const void*>(causal_fwd_kernel<F>);
  const hipError_t err = grant_dynamic_lds(kern, static_cast<int>(lds));
  if (err != hipSuccess) return err;
  if (bwd)
    hipLaunchKernelGGL(causal_bwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  else
    hipLaunchKernelGGL(causal_fwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  return hipGetLastError();
}

bool resident_supports(int dtype, int D, int N) {
  return (dtype == 1 || dtype == 2) && (D == 64 || D == 32 || D == 16) && N <= kMaxTiles * mfma::TR;
}

static_assert(kCausalChunkRows == kMaxTiles * mfma::TR, "chunk = what the LDS holds");

bool causal_resident_supports(int dtype, int D) {
  return dtype == 0 ? (D == 32 || D == 16) : (D == 64 || D == 32 || D == 16);
}

hipError_t launch_resident_causal(const Problem& p, bool bwd, int chunks) {
  if (chunks != causal_chunks(p.N)) return hipErrorInvalidValue;
  return p.dtype == 0   ? run_causal<F32x32>(p, bwd, chunks)
         : p.dtype == 1 ? run_causal<Bf16x64>(p, bwd, chunks)
                        : run_causal<F16x64>(p, bwd, chunks);
}

hipError_t launch_resident_fwd(const Problem& p) {
  return p.dtype == 1 ? run<Bf16x64>(p, false) : run<F16x64>(p, false);
}

hipError_t launch_resident_bwd(const Problem& p) {
  return p.dtype == 1 ? run<Bf16x64>(p, true) : run<F16x64>(p, true);
}

}  // namespace cotten
