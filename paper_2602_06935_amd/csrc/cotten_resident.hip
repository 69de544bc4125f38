// Resident kernels for short sequences (N <= 208) with 128-byte rows.
//
// One workgroup of 16 waves owns one slice and keeps it in LDS: wave w loads, stages and
// later finishes the 16-row tile w, so every global load of the slice is issued at once and
// nothing is read twice.  Between staging and the apply phase the d x d states are built by
// one wave per output block, each walking all resident tiles (no cross-wave reduction):
//
//   load     mask bytes and (Q[,dO]) tile, then (K,V) tile with masked rows skipped
//   stage    khat, v, qhat (bwd) or q (fwd), dO  ->  LDS block of the tile;  1/r kept in registers
//   barrier
//   states   4 waves: S blocks;  backward: 4 more waves: dS blocks;  results -> operand images
//   barrier
//   apply    forward: wave w finishes tile w.  Backward: four waves per product (dQ, dV, dK)
//            share out the tiles, so an operand image is fetched once per three or four tiles.  The
//            epilogue runs in the layout the product comes out in, next to the tile rows
//            fetched from LDS in that same layout, and ends in 128-bit stores.
#include "cotten_launch.h"
#include "cotten_mfma_core.h"

// Optional phase timestamps for tuning builds (-DCOTTEN_TRACE), see cotten_mfma.hip.
#ifdef COTTEN_TRACE
__device__ long long cotten_rtrace_buf[2 * 16 * 16];
#define COTTEN_RTRACE(i)                                                                   \
  do {                                                                                     \
    if ((blockIdx.x == 0 || blockIdx.x == gridDim.x - 1) && (threadIdx.x & 63) == 0)       \
      cotten_rtrace_buf[((blockIdx.x != 0) * 16 + (threadIdx.x >> 6)) * 16 + (i)] = clock64(); \
  } while (0)
extern "C" int cotten_rtrace_read(long long* host, int n) {
  return static_cast<int>(hipMemcpyFromSymbol(host, HIP_SYMBOL(cotten_rtrace_buf), n * sizeof(long long)));
}
#define COTTEN_RTRACE_IT(i) do { if (iter < 2) COTTEN_RTRACE(8 * iter + (i)); } while (0)
#else
#define COTTEN_RTRACE(i) do {} while (0)
#define COTTEN_RTRACE_IT(i) do {} while (0)
#endif

namespace cotten {
namespace {

using namespace mfma;

constexpr int kWaves = 16;
constexpr int kWorkgroups = 256;                // one per compute unit (LDS admits no second)
constexpr int kThreads = 64 * kWaves;
constexpr int kMaxTiles = 13;                  // N <= 208
constexpr int kBlockBytes = 4 * kTileBytes;    // [khat | v | q(hat) | dO] tiles of 16 rows
constexpr int kKt = 0, kVt = kTileBytes, kQt = 2 * kTileBytes, kGt = 3 * kTileBytes;

template <class F>
struct Lds {
  static constexpr int kImages = kMaxTiles * kBlockBytes;          // three operand images
  static constexpr int kLive = kImages + 3 * F::kImageBytes;       // one int per tile
  static constexpr int kInv = kLive + 16 * 4;                      // 1/r per tile: 16 q rows, 16 k rows
  static constexpr int kBytes = kInv + kMaxTiles * 2 * TR * 4;
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
  float scale, eps;
};

// The wave's tile: rows 16*tile + r8 + 8h.  `want` bit h: the row takes part.
template <bool USE_Y>
__device__ __forceinline__ void load_tile(Raw& r, const Lane& L, const Src& src, int tile,
                                          int want) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = tile * TR + L.r8 + 8 * h;
    const uint32_t off =
        ((want >> h) & 1) ? static_cast<uint32_t>(row) * kRowBytes + L.ch * 16 : kOutOfBuffer;
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
// does not exist).  Rows of K and V that are not valid keys are not read.
template <bool BWD>
__device__ __forceinline__ void fetch(Raw& rq, Raw& rk, const Args& a, const Lane& L, int slice,
                                      int tile, int keys) {
  const bool ok = slice < a.slices;
  const size_t base = ok ? static_cast<size_t>(slice) * a.N * kRowBytes : 0;
  const Src q_src(a.Q + base, (BWD ? a.dO : a.Q) + base, a.N), kv_src(a.K + base, a.V + base, a.N);
  int rows = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h)
    rows |= static_cast<int>(ok && tile * TR + L.r8 + 8 * h < a.N) << h;
  load_tile<BWD>(rq, L, q_src, tile, rows);
  load_tile<true>(rk, L, kv_src, tile, rows & keys);
}

// 1/r of the 16 tile rows, from the load layout to where any wave can pick them up by row.
__device__ __forceinline__ void publish_inv(float* dst, const Lane& L, const float (&inv)[2]) {
  if (L.ch == 0) {
    dst[L.r8] = inv[0];
    dst[L.r8 + 8] = inv[1];
  }
}

// Bit t set: tile t holds a valid key.
__device__ __forceinline__ uint64_t live_tiles(const Lane& L, const int* live, int n_tiles) {
  const int lv = L.lane < n_tiles ? live[L.lane] : 0;
  return __ballot(lv != 0);
}

// One wave per state block: walks the given resident tiles (bit set), fetching the next
// tile's operands while the matrix core works on the current one, then writes its block into
// the images.
template <class F>
__device__ __forceinline__ void build_state(const Lane& L, int block, uint64_t tiles, int x_off,
                                            int y_off, float scale, unsigned char* natural,
                                            unsigned char* transposed) {
  typedef typename F::BlockAcc Acc;
  Acc acc;
  acc.zero();
  if (tiles != 0) {
    const unsigned char* blk = smem + __builtin_ctzll(tiles) * kBlockBytes;
    tiles &= tiles - 1;
    typename Acc::Frag cur = Acc::fetch(blk + x_off, blk + y_off, L, block);
    while (tiles != 0) {
      blk = smem + __builtin_ctzll(tiles) * kBlockBytes;
      tiles &= tiles - 1;
      const typename Acc::Frag nxt = Acc::fetch(blk + x_off, blk + y_off, L, block);
      acc.mma(cur);
      cur = nxt;
    }
    acc.mma(cur);
  }
  acc.write_images(L, block, scale, natural, transposed);
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
  int* live = reinterpret_cast<int*>(smem + Lds<F>::kLive);
  float* invs = reinterpret_cast<float*>(smem + Lds<F>::kInv) + tile * 2 * TR;
  const bool mine = tile < n_tiles;

  int slice = blockIdx.x;
  Raw rq, rk;
  fetch<false>(rq, rk, a, L0, slice, tile, key_rows(a, L0, slice, tile));
  int keys = key_rows(a, L0, slice + stride, tile);
  for (; slice < a.slices; slice += stride) {
    if (mine) {
      const Lane L = L0.again();
      float inv[2];
      const bool any_key = __ballot(rk.live != 0) != 0;
      if (any_key) stage<F, kXNormalized, true>(rk, L, a.eps, blk + kKt, blk + kVt, inv);
      if (L.lane == 0) live[tile] = any_key;
      stage<F, kXRaw, false>(rq, L, a.eps, blk + kQt, blk + kGt, inv);
      publish_inv(invs, L, inv);
    }
    __syncthreads();
    {
      const Lane L = L0.again();
      fetch<false>(rq, rk, a, L, slice + stride, tile, keys);
      keys = key_rows(a, L, slice + 2 * stride, tile);
    }
    if (tile < F::BlockAcc::kBlocks) {  // O = qhat S: contraction over rows of S -> transposed image
      const Lane L = L0.again();
      build_state<F>(L, tile, live_tiles(L, live, n_tiles), kKt, kVt, a.scale, nullptr, img);
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
        store_product_row<F>(a.O + static_cast<size_t>(slice) * N * kRowBytes, row, L, o);
    }
    __syncthreads();  // the tiles and images are rewritten for the next slice
  }
}

// Backward apply phase: wave w < 12 takes product w % 3 and every fourth tile from w / 3 on, so
// that each SIMD (waves w, w+4, w+8) gets one wave of each product.
constexpr int kProducts = 3, kWavesPerProduct = 4;

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

  // product 0: dQ = (g - qhat (qhat.g)) / r_q,  g = scale * dO S^T
  // product 1: dV = khat (scale * dS)             (khat is zero on masked rows)
  // product 2: dK = (h - khat (khat.h)) / r_k,  h = v (scale * dS)^T   (1/r_k = 0 on masked rows)
  const int product = tile < kProducts * kWavesPerProduct ? tile % kProducts : kProducts;
  const int x_off = product == 0 ? kGt : product == 1 ? kKt : kVt;
  const int e_off = product == 0 ? kQt : kKt;
  unsigned char* const dst0 = product == 0 ? a.dQ : product == 1 ? a.dV : a.dK;
  const unsigned char* const image = product == 0 ? img_s : product == 1 ? img_dst : img_ds;
  const float* inv_base = invs + (product == 0 ? 0 : TR);

  int slice = blockIdx.x;
  Raw rq, rk;
  COTTEN_RTRACE(0);
  fetch<true>(rq, rk, a, L0, slice, tile, key_rows(a, L0, slice, tile));
  int keys = key_rows(a, L0, slice + stride, tile);
  for (int iter = 0; slice < a.slices; slice += stride, ++iter) {
    COTTEN_RTRACE_IT(1);
    if (mine) {
      const Lane L = L0.again();
      float inv[2];
      stage<F, kXNormalized, true>(rq, L, a.eps, blk + kQt, blk + kGt, inv);
      publish_inv(invs + tile * 2 * TR, L, inv);
      // A tile without a valid key is never read again: the states skip it and its dK, dV
      // rows are plain zeros.
      const bool any_key = __ballot(rk.live != 0) != 0;
      if (any_key) {
        stage<F, kXNormalized, true>(rk, L, a.eps, blk + kKt, blk + kVt, inv);
        publish_inv(invs + tile * 2 * TR + TR, L, inv);
      }
      if (L.lane == 0) live[tile] = any_key;
    }
    COTTEN_RTRACE_IT(2);
    __syncthreads();
    COTTEN_RTRACE_IT(3);
    {
      const Lane L = L0.again();
      fetch<true>(rq, rk, a, L, slice + stride, tile, keys);
      keys = key_rows(a, L, slice + 2 * stride, tile);
    }
    constexpr int kB = F::BlockAcc::kBlocks;
    if (tile < 2 * kB) {
      const Lane L = L0.again();
      if (tile < kB)  // g = dO S^T: contraction over columns of S -> natural image
        build_state<F>(L, tile, live_tiles(L, live, n_tiles), kKt, kVt, a.scale, img_s, nullptr);
      else            // dV = khat dS -> transposed image;  h = v dS^T -> natural image
        build_state<F>(L, tile - kB, (1ull << n_tiles) - 1, kQt, kGt, a.scale, img_ds, img_dst);
    }
    COTTEN_RTRACE_IT(4);
    __syncthreads();
    COTTEN_RTRACE_IT(5);
    if (product < kProducts) {
      const Lane L = L0.again();
      unsigned char* dst = dst0 + static_cast<size_t>(slice) * N * kRowBytes;
      typename F::Operand W;
      W.load(image, L);
#pragma unroll 1
      for (int t = tile / kProducts; t < n_tiles; t += kWavesPerProduct) {
        const unsigned char* tb = smem + t * kBlockBytes;
        const int row = t * TR + L.i16;
        if (product != 0 && live[t] == 0) {  // no valid key in the tile: dK = dV = 0
          float zeros[2 * F::EPL];
#pragma unroll
          for (int c = 0; c < 2 * F::EPL; ++c) zeros[c] = 0.0f;
          if (row < N) store_product_row<F>(dst, row, L, zeros);
          continue;
        }
        typename F::TileRows x;
        x.load(tb + x_off, L);
        f32x4_t out[F::NT];
        F::apply(x, W, out);
        float p[2 * F::EPL];
        product_rows<F>(out, p);
        if (product != 1) {
          typename F::TileRows e;
          e.load(tb + e_off, L);
          project_rows<F>(p, e, inv_base[t * 2 * TR + L.i16], L);
        }
        if (row < N) store_product_row<F>(dst, row, L, p);
      }
    }
    COTTEN_RTRACE_IT(6);
    __syncthreads();  // the tiles and images are rewritten for the next slice
    COTTEN_RTRACE_IT(7);
  }
}

template <class F>
hipError_t run(const Problem& p, bool bwd) {
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
  a.scale = p.scale;
  a.eps = p.eps;
  const dim3 grid(static_cast<unsigned>(a.slices < kWorkgroups ? a.slices : kWorkgroups));
  const size_t lds = Lds<F>::kBytes;
  const void* kern = bwd ? reinterpret_cast<const void*>(resident_bwd_kernel<F>)
                         : reinterpret_cast<const void*>(resident_fwd_kernel<F>);
  const hipError_t err =
      hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(lds));
  if (err != hipSuccess) return err;
  if (bwd)
    hipLaunchKernelGGL(resident_bwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  else
    hipLaunchKernelGGL(resident_fwd_kernel<F>, grid, dim3(kThreads), lds, p.stream, a);
  return hipGetLastError();
}

}  // namespace

int resident_max_rows() { return kMaxTiles * mfma::TR; }

hipError_t launch_resident_fwd(const Problem& p) {
  return p.dtype == 1 ? run<Bf16x64>(p, false) : run<F32x32>(p, false);
}

hipError_t launch_resident_bwd(const Problem& p) {
  return p.dtype == 1 ? run<Bf16x64>(p, true) : run<F32x32>(p, true);
}

}  // namespace cotten
