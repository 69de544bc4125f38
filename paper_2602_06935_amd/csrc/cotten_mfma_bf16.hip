// MFMA path for bf16 I/O, d_h = 64 (gfx950).
//
// Work unit: one wavefront streams 16-row tiles of a slice.  A tile is loaded with
// 128-bit accesses (8 lanes per 128-byte row, 8 rows per instruction), normalised in
// fp32 registers, rounded to bf16 and parked in a wave-private LDS tile, from which
// the matrix cores are fed:
//   state products   S += Xhat^T Y   (contraction over rows):  32x32x16 bf16 MFMA,
//                    operands fetched with the transposing LDS read;
//   apply products   T = X W         (contraction over columns): 16x16x32 bf16 MFMA,
//                    X rows read straight from the tile, W held in registers.
// Products come back through a wave-private fp32 scratch tile into the load layout,
// where the epilogue (projection off the normalised row, 1/r, masking) runs in fp32
// next to the unrounded inputs and results leave with 128-bit stores.
//
// Fused kernels (one workgroup = 4 waves per slice) run all phases in one launch;
// split kernels cut long sequences over several workgroups per slice and pass
// partial states through the workspace.
#include "cotten_device.h"
#include "cotten_launch.h"

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

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint16_t lds_bf16;  // bf16 bit pattern in LDS

constexpr int D = 64;
constexpr int kWaves = 4;
constexpr int kThreads = 64 * kWaves;
constexpr int TR = 16;   // rows per wave tile
constexpr int RS = 72;   // row stride (elements) of bf16 LDS tiles and state operands
constexpr int SCS = 68;  // row stride (floats) of the fp32 scratch tile

// per-wave LDS working set
constexpr int kTileBytes = TR * RS * 2;       // 2304
constexpr int kScratchBytes = TR * SCS * 4;   // 4352
constexpr int kWaveBytes = 2 * kTileBytes + 2 * kScratchBytes;  // 13312
constexpr int kWorkBytes = kWaves * kWaveBytes;                 // 53248
constexpr int kOperandBytes = D * RS * 2;                       // one bf16 state operand
// LDS map: [working set / reduction buffers][operand 0][operand 1][mask bytes]
constexpr int kOp0Offset = kWorkBytes;
constexpr int kOp1Offset = kOp0Offset + kOperandBytes;
constexpr int kMaskOffset = kOp1Offset + kOperandBytes;

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2_t v;
  v[0] = static_cast<__bf16>(lo);
  v[1] = static_cast<__bf16>(hi);
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ void unpack8(const u32x4_t r, float (&f)[8]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[2 * i] = __uint_as_float(r[i] << 16);
    f[2 * i + 1] = __uint_as_float(r[i] & 0xffff0000u);
  }
}

__device__ __forceinline__ u32x4_t pack8(const float (&f)[8]) {
  u32x4_t r;
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = pack_bf16(f[2 * i], f[2 * i + 1]);
  return r;
}

// Sum over the 8 consecutive lanes that share one row, by lane-permuting adds (no LDS).
__device__ __forceinline__ float row_sum8(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // lane ^ 1
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // lane ^ 2
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // other quad of the 8
  return x;
}

// Sum of squares of the 8 bf16 values in a 128-bit register group (fp32 accumulation).
__device__ __forceinline__ float sumsq8(const u32x4_t r) {
  float s = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const float lo = __uint_as_float(r[i] << 16), hi = __uint_as_float(r[i] & 0xffff0000u);
    s += lo * lo;
    s += hi * hi;
  }
  return s;
}

// 1/sqrt(ss + eps) for a live row (hardware reciprocal square root, about 1 ulp), 0 otherwise.
__device__ __forceinline__ float inv_norm_or_zero(float ss, float eps, bool live) {
  return live ? __builtin_amdgcn_rsqf(ss + eps) : 0.0f;
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

// Lane geometry shared by every pass.
struct Lane {
  int lane, wave;
  int r8, ch;      // load layout: tile rows r8 and r8+8, columns 8*ch .. 8*ch+7
  int i16, g16;    // MFMA 16-lane groups: lane%16, lane/16
  __device__ __forceinline__ Lane() {
    lane = threadIdx.x & 63;
    wave = threadIdx.x >> 6;
    r8 = lane >> 3;
    ch = lane & 7;
    i16 = lane & 15;
    g16 = lane >> 4;
  }
};

// Raw 16-row tile in the load layout: x[h], y[h] hold row r8 + 8h; `live` bit h says the
// row takes part (in range and, where a mask applies, a valid key).
struct Raw {
  u32x4_t x[2], y[2];
  int live;
};

// Loads tile rows row0 .. row0+15.  A row takes part when it is below `row_limit` and, if
// `flags` is given, flags[row - m_base] != 0 (LDS copy of the key mask).  USE_Y: second tensor.
template <bool USE_Y>
__device__ __forceinline__ void load_raw(Raw& r, const Lane& L, const bf16* __restrict__ X,
                                         const bf16* __restrict__ Y, int row0,
                                         const uint8_t* flags, int m_base, int row_limit) {
  r.live = 0;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = row0 + L.r8 + 8 * h;
    bool live = row < row_limit;
    if (flags != nullptr) live = flags[row - m_base] != 0;
    r.x[h] = u32x4_t{0, 0, 0, 0};
    r.y[h] = u32x4_t{0, 0, 0, 0};
    if (live) {
      const size_t off = static_cast<size_t>(row) * D + L.ch * 8;
      r.x[h] = *reinterpret_cast<const u32x4_t*>(X + off);
      if (USE_Y) r.y[h] = *reinterpret_cast<const u32x4_t*>(Y + off);
      r.live |= 1 << h;
    }
  }
}

// What becomes of the x rows on their way to the LDS tile.
enum XMode { kXNone = 0, kXRaw = 1, kXNormalized = 2 };

// inv[h] = 1/r of row h (0 for rows that do not take part; their registers are zero).
// Xt receives nothing, the raw rows, or xhat rounded to bf16; Yt the raw y rows.
template <int XMODE, bool USE_Y>
__device__ __forceinline__ void stage(const Raw& r, const Lane& L, float eps, lds_bf16* Xt,
                                      lds_bf16* Yt, float (&inv)[2]) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    inv[h] = inv_norm_or_zero(row_sum8(sumsq8(r.x[h])), eps, (r.live >> h) & 1);
    const int off = (L.r8 + 8 * h) * RS + L.ch * 8;
    if (XMODE == kXNormalized) {
      float f[8];
      unpack8(r.x[h], f);
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] *= inv[h];
      *reinterpret_cast<u32x4_t*>(Xt + off) = pack8(f);
    } else if (XMODE == kXRaw) {
      *reinterpret_cast<u32x4_t*>(Xt + off) = r.x[h];
    }
    if (USE_Y) *reinterpret_cast<u32x4_t*>(Yt + off) = r.y[h];
  }
}

// Operand of the 32x32x16 MFMA for a contraction over the 16 tile rows: lane gets, for
// column cbase + lane%32, the 8 rows 8*(lane/32) .. +7 (two transposing reads of 4 rows).
__device__ __forceinline__ bf16x8_t rows_operand(const lds_bf16* T, const Lane& L, int cbase) {
  const int s = L.i16;
  const int row = 8 * (L.g16 >> 1) + (s >> 2);
  const int col = cbase + 16 * (L.g16 & 1) + 4 * (s & 3);
  typedef bf16x4_t __attribute__((address_space(3))) * lds_v4;
  const bf16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)(T + row * RS + col));
  const bf16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)(T + (row + 4) * RS + col));
  return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// acc[at][ct] += (X tile)^T (Y tile): rows at*32.., columns ct*32.. of the 64x64 state.
__device__ __forceinline__ void state_mfma(const lds_bf16* Xt, const lds_bf16* Yt, const Lane& L,
                                           f32x16_t (&acc)[2][2]) {
  bf16x8_t a[2], b[2];
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    a[t] = rows_operand(Xt, L, 32 * t);
    b[t] = rows_operand(Yt, L, 32 * t);
  }
#pragma unroll
  for (int at = 0; at < 2; ++at)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
      acc[at][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[at], b[ct], acc[at][ct], 0, 0, 0);
}

// State operand W held in registers for apply products T = X W (16x16x32 MFMA):
// frag[nt][ks] = 8 consecutive k (8*(lane/16) + 32*ks ..) of output column 16*nt + lane%16,
// read from an LDS image stored column-major in k: op[n][k].
struct Operand {
  bf16x8_t frag[4][2];
  __device__ __forceinline__ void load(const lds_bf16* op, const Lane& L) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        frag[nt][ks] = *reinterpret_cast<const bf16x8_t*>(op + (16 * nt + L.i16) * RS +
                                                           8 * L.g16 + 32 * ks);
  }
};

// out[nt] (16 rows x 16 columns, fp32) = (tile rows) x W
__device__ __forceinline__ void apply_mfma(const lds_bf16* T, const Operand& W, const Lane& L,
                                           f32x4_t (&out)[4]) {
  bf16x8_t a[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
    a[ks] = *reinterpret_cast<const bf16x8_t*>(T + L.i16 * RS + 8 * L.g16 + 32 * ks);
#pragma unroll
  for (int nt = 0; nt < 4; ++nt) {
    out[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
      out[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[ks], W.frag[nt][ks], out[nt], 0, 0, 0);
  }
}

// MFMA result layout -> scratch tile (row 4*(lane/16)+v, column 16*nt + lane%16)
__device__ __forceinline__ void to_scratch(const f32x4_t (&out)[4], float* Sc, const Lane& L) {
#pragma unroll
  for (int nt = 0; nt < 4; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) Sc[(4 * L.g16 + v) * SCS + 16 * nt + L.i16] = out[nt][v];
}

// scratch tile -> load layout: the 8 columns of row r8 + 8h this lane owns
__device__ __forceinline__ void from_scratch(const float* Sc, const Lane& L, int h, float (&f)[8]) {
  const f32x4_t* p = reinterpret_cast<const f32x4_t*>(Sc + (L.r8 + 8 * h) * SCS + 8 * L.ch);
  const f32x4_t a = p[0], b = p[1];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    f[i] = a[i];
    f[4 + i] = b[i];
  }
}

__device__ __forceinline__ void store_row(bf16* __restrict__ dst, int row, const Lane& L,
                                          const float (&f)[8]) {
  *reinterpret_cast<u32x4_t*>(dst + static_cast<size_t>(row) * D + 8 * L.ch) = pack8(f);
}

struct WaveLds {
  lds_bf16* Xt;
  lds_bf16* Yt;
  float* Sc0;
  float* Sc1;
  __device__ __forceinline__ WaveLds(unsigned char* smem, int wave) {
    unsigned char* base = smem + wave * kWaveBytes;
    Xt = reinterpret_cast<lds_bf16*>(base);
    Yt = reinterpret_cast<lds_bf16*>(base + kTileBytes);
    Sc0 = reinterpret_cast<float*>(base + 2 * kTileBytes);
    Sc1 = reinterpret_cast<float*>(base + 2 * kTileBytes + kScratchBytes);
  }
};

// Copies the key mask of rows [m_base, m_base + count) into LDS as "takes part" flags.
// mask == nullptr: every row below N takes part.
__device__ __forceinline__ void fill_flags(uint8_t* flags, const uint8_t* __restrict__ mask,
                                           int m_base, int count, int N) {
  for (int i = threadIdx.x; i < count; i += kThreads) {
    const int row = m_base + i;
    uint8_t f = 0;
    if (row < N) f = (mask == nullptr) ? 1 : (mask[row] != 0);
    flags[i] = f;
  }
}

// First tile of this wave (tile index = wave), issued early by the caller.
template <bool USE_Y>
__device__ __forceinline__ void load_first(Raw& a, const Lane& L, const bf16* __restrict__ X,
                                           const bf16* __restrict__ Y, int row_begin, int n_tiles,
                                           const uint8_t* flags, int m_base, int row_limit) {
  a.live = 0;
  if (L.wave < n_tiles)
    load_raw<USE_Y>(a, L, X, Y, row_begin + L.wave * TR, flags, m_base, row_limit);
}

// Walks the tiles wave, wave+kWaves, ... < n_tiles owned by this wave with the next tile's
// global loads in flight while the current one is processed.  `a` holds the first tile.
template <bool USE_Y, typename F>
__device__ __forceinline__ void for_each_tile(const Lane& L, const bf16* __restrict__ X,
                                              const bf16* __restrict__ Y, int row_begin,
                                              int n_tiles, const uint8_t* flags, int m_base,
                                              int row_limit, Raw& a, F&& body) {
  int t = L.wave;
  if (t >= n_tiles) return;
  Raw b;
  while (true) {
    bool more = t + kWaves < n_tiles;
    if (more) load_raw<USE_Y>(b, L, X, Y, row_begin + (t + kWaves) * TR, flags, m_base, row_limit);
    body(a, row_begin + t * TR);
    if (!more) break;
    t += kWaves;
    more = t + kWaves < n_tiles;
    if (more) load_raw<USE_Y>(a, L, X, Y, row_begin + (t + kWaves) * TR, flags, m_base, row_limit);
    body(b, row_begin + t * TR);
    if (!more) break;
    t += kWaves;
  }
}

// ---- passes -------------------------------------------------------------------------
// Every pass takes the wave's first tile already loaded in `first`.

// acc += sum over live rows of xhat^T y for rows [row_begin, row_begin + 16*n_tiles)
__device__ __forceinline__ void state_pass(const Lane& L, const WaveLds& W,
                                           const bf16* __restrict__ X, const bf16* __restrict__ Y,
                                           int row_begin, int n_tiles, const uint8_t* flags,
                                           int m_base, int row_limit, float eps, Raw& first,
                                           f32x16_t (&acc)[2][2]) {
  for_each_tile<true>(L, X, Y, row_begin, n_tiles, flags, m_base, row_limit, first,
                      [&](const Raw& r, int) {
    if (__ballot(r.live != 0) == 0) return;  // no live row in this tile (uniform)
    float inv[2];
    stage<kXNormalized, true>(r, L, eps, W.Xt, W.Yt, inv);
    wave_lds_fence();
    state_mfma(W.Xt, W.Yt, L, acc);
    wave_lds_fence();
  });
}

// O rows = (q rows x W) / r   (W = scale * S, operand image op[c][a])
__device__ __forceinline__ void fwd_apply_pass(const Lane& L, const WaveLds& W,
                                               const bf16* __restrict__ Q, bf16* __restrict__ O,
                                               int row_begin, int n_tiles, int row_limit,
                                               float eps, Raw& first, const Operand& Sop) {
  for_each_tile<false>(L, Q, Q, row_begin, n_tiles, nullptr, 0, row_limit, first,
                       [&](const Raw& r, int row0) {
    float inv[2];
    stage<kXRaw, false>(r, L, eps, W.Xt, W.Yt, inv);
    wave_lds_fence();
    f32x4_t out[4];
    apply_mfma(W.Xt, Sop, L, out);
    to_scratch(out, W.Sc0, L);
    wave_lds_fence();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float o[8];
      from_scratch(W.Sc0, L, h, o);
#pragma unroll
      for (int i = 0; i < 8; ++i) o[i] *= inv[h];
      if ((r.live >> h) & 1) store_row(O, row0 + L.r8 + 8 * h, L, o);
    }
    wave_lds_fence();
  });
}

// dQ rows from (Q, dO) and W = scale * S (operand image op[a][c]); with ACCUM also
// dsacc += qhat^T dO.
template <bool ACCUM>
__device__ __forceinline__ void bwd_q_pass(const Lane& L, const WaveLds& W,
                                           const bf16* __restrict__ Q, const bf16* __restrict__ dO,
                                           bf16* __restrict__ dQ, int row_begin, int n_tiles,
                                           int row_limit, float eps, Raw& first,
                                           const lds_bf16* Simage, f32x16_t (&dsacc)[2][2]) {
  // With the 64 accumulator registers live the operand is re-read from LDS for every tile;
  // without them it stays in registers.
  Operand held;
  if (!ACCUM) held.load(Simage, L);
  for_each_tile<true>(L, Q, dO, row_begin, n_tiles, nullptr, 0, row_limit, first,
                      [&](const Raw& r, int row0) {
    float inv[2];
    stage<ACCUM ? kXNormalized : kXNone, true>(r, L, eps, W.Xt, W.Yt, inv);
    wave_lds_fence();
    if (ACCUM) state_mfma(W.Xt, W.Yt, L, dsacc);
    f32x4_t out[4];
    if (ACCUM) {
      Operand fresh;
      fresh.load(Simage, L);
      apply_mfma(W.Yt, fresh, L, out);  // g = scale * dO S^T
    } else {
      apply_mfma(W.Yt, held, L, out);
    }
    to_scratch(out, W.Sc0, L);
    wave_lds_fence();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      float g[8], q[8];
      from_scratch(W.Sc0, L, h, g);
      unpack8(r.x[h], q);
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        q[i] *= inv[h];
        proj += q[i] * g[i];
      }
      proj = row_sum8(proj);
#pragma unroll
      for (int i = 0; i < 8; ++i) g[i] = (g[i] - q[i] * proj) * inv[h];
      if ((r.live >> h) & 1) store_row(dQ, row0 + L.r8 + 8 * h, L, g);
    }
    wave_lds_fence();
  });
}

// dK, dV rows from (K, V) and scale * dS: dV = (k dS)/r (operand image op[c][a]),
// h = v dS^T (operand image op[a][c]).  Rows below row_limit that are masked get zeros.
__device__ __forceinline__ void bwd_kv_pass(const Lane& L, const WaveLds& W,
                                            const bf16* __restrict__ K, const bf16* __restrict__ V,
                                            bf16* __restrict__ dK, bf16* __restrict__ dV,
                                            int row_begin, int n_tiles, const uint8_t* flags,
                                            int m_base, int row_limit, float eps, Raw& first,
                                            const Operand& dSop_v, const Operand& dSop_h) {
  for_each_tile<true>(L, K, V, row_begin, n_tiles, flags, m_base, row_limit, first,
                      [&](const Raw& r, int row0) {
    if (__ballot(r.live != 0) == 0) {  // nothing live: only the zero rows are due
      const float zeros[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int row = row0 + L.r8 + 8 * h;
        if (row < row_limit) {
          store_row(dK, row, L, zeros);
          store_row(dV, row, L, zeros);
        }
      }
      return;
    }
    float inv[2];
    stage<kXRaw, true>(r, L, eps, W.Xt, W.Yt, inv);
    wave_lds_fence();
    f32x4_t out[4];
    apply_mfma(W.Xt, dSop_v, L, out);
    to_scratch(out, W.Sc0, L);
    apply_mfma(W.Yt, dSop_h, L, out);
    to_scratch(out, W.Sc1, L);
    wave_lds_fence();
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int row = row0 + L.r8 + 8 * h;
      float gv[8], hh[8], k[8];
      from_scratch(W.Sc0, L, h, gv);
      from_scratch(W.Sc1, L, h, hh);
      unpack8(r.x[h], k);
      float proj = 0.0f;
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        k[i] *= inv[h];      // inv = 0 on masked rows: khat, dK and dV come out as exact zeros
        proj += k[i] * hh[i];
      }
      proj = row_sum8(proj);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        hh[i] = (hh[i] - k[i] * proj) * inv[h];
        gv[i] *= inv[h];
      }
      if (row < row_limit) {
        store_row(dK, row, L, hh);
        store_row(dV, row, L, gv);
      }
    }
    wave_lds_fence();
  });
}

// ---- workgroup-level state handling -------------------------------------------------

// Reduction buffers: two fp32 images of the 64x64 state stored column-major with a padded
// stride, R[n * kRStride + m], so that the 4 consecutive rows an accumulator register
// group holds move as one 128-bit LDS access.
constexpr int kRStride = 68;
constexpr int kRFloats = D * kRStride;
static_assert(2 * kRFloats * 4 <= kWorkBytes, "reduction buffers alias the working set");

__device__ __forceinline__ f32x4_t quad(const f32x16_t& a, int j) {
  return f32x4_t{a[4 * j], a[4 * j + 1], a[4 * j + 2], a[4 * j + 3]};
}

// Sums the four per-wave accumulators in the fixed order (w0 + w1) + (w2 + w3):
// afterwards R0 + R1 (at the start of LDS) is the total.
__device__ __forceinline__ void wg_reduce(const Lane& L, unsigned char* smem,
                                          const f32x16_t (&acc)[2][2]) {
  float* R = reinterpret_cast<float*>(smem) + (L.wave >> 1) * kRFloats;
  f32x4_t* dst[2][2][4];
#pragma unroll
  for (int at = 0; at < 2; ++at)
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int m = 32 * at + 8 * j + 4 * (L.lane >> 5);
        const int n = 32 * ct + (L.lane & 31);
        dst[at][ct][j] = reinterpret_cast<f32x4_t*>(R + n * kRStride + m);
      }
  __syncthreads();  // working set no longer in use
  if ((L.wave & 1) == 0) {
#pragma unroll
    for (int at = 0; at < 2; ++at)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *dst[at][ct][j] = quad(acc[at][ct], j);
  }
  __syncthreads();
  if ((L.wave & 1) == 1) {
    f32x4_t other[2][2][4];  // all reads first, so that they overlap
#pragma unroll
    for (int at = 0; at < 2; ++at)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j) other[at][ct][j] = *dst[at][ct][j];
#pragma unroll
    for (int at = 0; at < 2; ++at)
#pragma unroll
      for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *dst[at][ct][j] = other[at][ct][j] +
                            quad(acc[at][ct], j);
  }
  __syncthreads();
}

// Element (m, n) of the reduced state: from LDS (R0 + R1) or from a row-major global array.
struct StateSource {
  const float* lds;     // R0 (R1 follows) or nullptr
  const float* global;  // row-major 64x64 or nullptr
  __device__ __forceinline__ float at(int m, int n) const {
    if (lds != nullptr) return lds[n * kRStride + m] + lds[kRFloats + n * kRStride + m];
    return global[m * D + n];
  }
};

// Builds bf16 operand images of scale * M for the apply products:
//   natural    op[m][n] = M[m][n]   (products contracting over n)
//   transposed op[n][m] = M[m][n]   (products contracting over m)
// Two neighbouring elements are rounded together and leave as one 32-bit LDS write.
__device__ __forceinline__ void make_operands(const StateSource src, float scale,
                                              lds_bf16* natural, lds_bf16* transposed) {
  constexpr int kPer = D * D / 2 / kThreads;  // element pairs per thread
  if (natural != nullptr) {
    float lo[kPer], hi[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads, m = e >> 5, n = (e & 31) * 2;
      lo[i] = src.at(m, n);
      hi[i] = src.at(m, n + 1);
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads, m = e >> 5, n = (e & 31) * 2;
      *reinterpret_cast<uint32_t*>(natural + m * RS + n) = pack_bf16(lo[i] * scale, hi[i] * scale);
    }
  }
  if (transposed != nullptr) {
    float lo[kPer], hi[kPer];
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads, n = e & 63, m = (e >> 6) * 2;
      lo[i] = src.at(m, n);
      hi[i] = src.at(m + 1, n);
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
      const int e = threadIdx.x + i * kThreads, n = e & 63, m = (e >> 6) * 2;
      *reinterpret_cast<uint32_t*>(transposed + n * RS + m) =
          pack_bf16(lo[i] * scale, hi[i] * scale);
    }
  }
}

// ---- kernels --------------------------------------------------------------------------

extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

__device__ __forceinline__ void zero_acc(f32x16_t (&acc)[2][2]) {
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int c = 0; c < 2; ++c)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][c][v] = 0.0f;
}

__global__ __launch_bounds__(kThreads, 2) void fused_fwd_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const uint8_t* __restrict__ mask, bf16* __restrict__ O, int H, int N, float scale,
    float eps) {
  const Lane L;
  const WaveLds W(smem, L.wave);
  const int bh = blockIdx.x;
  const size_t base = static_cast<size_t>(bh) * N * D;
  const int n_tiles = (N + TR - 1) / TR;
  uint8_t* kflags = smem + kMaskOffset;  // valid keys
  lds_bf16* op0 = reinterpret_cast<lds_bf16*>(smem + kOp0Offset);

  Raw qfirst, kfirst;  // the query tile does not depend on the mask: issue it right away
  load_first<false>(qfirst, L, Q + base, Q + base, 0, n_tiles, nullptr, 0, N);
  fill_flags(kflags, mask == nullptr ? nullptr : mask + static_cast<size_t>(bh / H) * N, 0,
             n_tiles * TR, N);
  __syncthreads();
  load_first<true>(kfirst, L, K + base, V + base, 0, n_tiles, kflags, 0, N);

  f32x16_t acc[2][2];
  zero_acc(acc);
  state_pass(L, W, K + base, V + base, 0, n_tiles, kflags, 0, N, eps, kfirst, acc);
  wg_reduce(L, smem, acc);
  // O = qhat S: contraction over rows of S
  make_operands(StateSource{reinterpret_cast<const float*>(smem), nullptr}, scale, nullptr, op0);
  __syncthreads();
  Operand Sop;
  Sop.load(op0, L);
  fwd_apply_pass(L, W, Q + base, O + base, 0, n_tiles, N, eps, qfirst, Sop);
}

__global__ __launch_bounds__(kThreads, 2) void fused_bwd_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const uint8_t* __restrict__ mask, const bf16* __restrict__ dO, bf16* __restrict__ dQ,
    bf16* __restrict__ dK, bf16* __restrict__ dV, int H, int N, float scale, float eps) {
  const Lane L;
  const WaveLds W(smem, L.wave);
  const int bh = blockIdx.x;
  const size_t base = static_cast<size_t>(bh) * N * D;
  const int n_tiles = (N + TR - 1) / TR;
  uint8_t* kflags = smem + kMaskOffset;
  lds_bf16* op0 = reinterpret_cast<lds_bf16*>(smem + kOp0Offset);
  lds_bf16* op1 = reinterpret_cast<lds_bf16*>(smem + kOp1Offset);
  const StateSource reduced{reinterpret_cast<const float*>(smem), nullptr};

  COTTEN_TRACE_POINT(0);
  Raw qfirst, kfirst;
  load_first<true>(qfirst, L, Q + base, dO + base, 0, n_tiles, nullptr, 0, N);
  fill_flags(kflags, mask == nullptr ? nullptr : mask + static_cast<size_t>(bh / H) * N, 0,
             n_tiles * TR, N);
  __syncthreads();
  COTTEN_TRACE_POINT(1);
  load_first<true>(kfirst, L, K + base, V + base, 0, n_tiles, kflags, 0, N);

  f32x16_t acc[2][2];
  zero_acc(acc);
  state_pass(L, W, K + base, V + base, 0, n_tiles, kflags, 0, N, eps, kfirst, acc);
  COTTEN_TRACE_POINT(2);
  wg_reduce(L, smem, acc);
  COTTEN_TRACE_POINT(3);
  make_operands(reduced, scale, op0, nullptr);  // g = dO S^T: contraction over columns of S
  __syncthreads();
  zero_acc(acc);
  COTTEN_TRACE_POINT(4);
  bwd_q_pass<true>(L, W, Q + base, dO + base, dQ + base, 0, n_tiles, N, eps, qfirst, op0, acc);
  COTTEN_TRACE_POINT(5);
  // the key/value tiles are walked again: get the first one moving before the reduction
  load_first<true>(kfirst, L, K + base, V + base, 0, n_tiles, kflags, 0, N);
  wg_reduce(L, smem, acc);
  COTTEN_TRACE_POINT(6);
  make_operands(reduced, scale, op0, op1);  // op0 = dS natural, op1 = dS transposed
  __syncthreads();
  Operand dS_v, dS_h;
  dS_v.load(op1, L);  // dV = khat dS: contraction over rows of dS
  dS_h.load(op0, L);  // h = v dS^T: contraction over columns of dS
  COTTEN_TRACE_POINT(7);
  bwd_kv_pass(L, W, K + base, V + base, dK + base, dV + base, 0, n_tiles, kflags, 0, N, eps,
              kfirst, dS_v, dS_h);
  COTTEN_TRACE_POINT(8);
}

// Split path, step 1: partial states of a block of rows.  blockIdx.y = 0: (K,V) under
// the key mask -> partial S;  blockIdx.y = 1: (Q,dO) -> partial dS.
__global__ __launch_bounds__(kThreads, 2) void split_state_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const uint8_t* __restrict__ mask, float* __restrict__ ws, int H,
    int N, int splits, int rows_per_split, size_t second_offset, float eps) {
  const Lane L;
  const WaveLds W(smem, L.wave);
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const bool second = blockIdx.y == 1;
  const size_t base = static_cast<size_t>(bh) * N * D;
  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int n_tiles = (r_end - r_begin + TR - 1) / TR;
  const bool masked = !second && mask != nullptr;
  uint8_t* flags = masked ? smem + kMaskOffset : nullptr;
  const bf16* X = (second ? Q : K) + base;
  const bf16* Y = (second ? dO : V) + base;
  if (masked) {
    fill_flags(flags, mask + static_cast<size_t>(bh / H) * N, r_begin, n_tiles * TR, r_end);
    __syncthreads();
  }
  Raw first;
  load_first<true>(first, L, X, Y, r_begin, n_tiles, flags, r_begin, r_end);
  f32x16_t acc[2][2];
  zero_acc(acc);
  state_pass(L, W, X, Y, r_begin, n_tiles, flags, r_begin, r_end, eps, first, acc);
  wg_reduce(L, smem, acc);
  const StateSource reduced{reinterpret_cast<const float*>(smem), nullptr};
  float* out = ws + (second ? second_offset : 0) + static_cast<size_t>(blockIdx.x) * D * D;
  for (int e = threadIdx.x; e < D * D; e += kThreads) out[e] = reduced.at(e >> 6, e & 63);
}

__global__ __launch_bounds__(kThreads, 2) void split_apply_fwd_kernel(
    const bf16* __restrict__ Q, const float* __restrict__ states, bf16* __restrict__ O, int N,
    int splits, int rows_per_split, float scale, float eps) {
  const Lane L;
  const WaveLds W(smem, L.wave);
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const size_t base = static_cast<size_t>(bh) * N * D;
  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int n_tiles = (r_end - r_begin + TR - 1) / TR;
  lds_bf16* op0 = reinterpret_cast<lds_bf16*>(smem + kOp0Offset);
  Raw first;
  load_first<false>(first, L, Q + base, Q + base, r_begin, n_tiles, nullptr, 0, r_end);
  make_operands(StateSource{nullptr, states + static_cast<size_t>(bh) * D * D}, scale, nullptr,
                op0);
  __syncthreads();
  Operand Sop;
  Sop.load(op0, L);
  fwd_apply_pass(L, W, Q + base, O + base, r_begin, n_tiles, r_end, eps, first, Sop);
}

// blockIdx.y = 0: dQ of a block of rows;  blockIdx.y = 1: dK, dV of a block of rows.
__global__ __launch_bounds__(kThreads, 2) void split_apply_bwd_kernel(
    const bf16* __restrict__ Q, const bf16* __restrict__ K, const bf16* __restrict__ V,
    const bf16* __restrict__ dO, const uint8_t* __restrict__ mask,
    const float* __restrict__ states, const float* __restrict__ dstates, bf16* __restrict__ dQ,
    bf16* __restrict__ dK, bf16* __restrict__ dV, int H, int N, int splits, int rows_per_split,
    float scale, float eps) {
  const Lane L;
  const WaveLds W(smem, L.wave);
  const int split = blockIdx.x % splits;
  const int bh = blockIdx.x / splits;
  const size_t base = static_cast<size_t>(bh) * N * D;
  const int r_begin = split * rows_per_split;
  const int r_end = min(N, r_begin + rows_per_split);
  const int n_tiles = (r_end - r_begin + TR - 1) / TR;
  lds_bf16* op0 = reinterpret_cast<lds_bf16*>(smem + kOp0Offset);
  lds_bf16* op1 = reinterpret_cast<lds_bf16*>(smem + kOp1Offset);
  Raw first;
  if (blockIdx.y == 0) {
    load_first<true>(first, L, Q + base, dO + base, r_begin, n_tiles, nullptr, 0, r_end);
    make_operands(StateSource{nullptr, states + static_cast<size_t>(bh) * D * D}, scale, op0,
                  nullptr);
    __syncthreads();
    f32x16_t unused[2][2];
    bwd_q_pass<false>(L, W, Q + base, dO + base, dQ + base, r_begin, n_tiles, r_end, eps, first,
                      op0, unused);
  } else {
    uint8_t* flags = mask != nullptr ? smem + kMaskOffset : nullptr;
    if (flags != nullptr)
      fill_flags(flags, mask + static_cast<size_t>(bh / H) * N, r_begin, n_tiles * TR, r_end);
    make_operands(StateSource{nullptr, dstates + static_cast<size_t>(bh) * D * D}, scale, op0,
                  op1);
    __syncthreads();
    load_first<true>(first, L, K + base, V + base, r_begin, n_tiles, flags, r_begin, r_end);
    Operand dS_v, dS_h;
    dS_v.load(op1, L);
    dS_h.load(op0, L);
    bwd_kv_pass(L, W, K + base, V + base, dK + base, dV + base, r_begin, n_tiles, flags, r_begin,
                r_end, eps, first, dS_v, dS_h);
  }
}

// Dynamic LDS above 64 KB has to be granted per kernel first; two workgroups share a
// compute unit's 160 KB.
constexpr int kMaxLdsBytes = 80 * 1024;
template <typename Kern>
hipError_t allow_lds(Kern kern, size_t bytes) {
  if (bytes > static_cast<size_t>(kMaxLdsBytes)) return hipErrorInvalidValue;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                             hipFuncAttributeMaxDynamicSharedMemorySize, kMaxLdsBytes);
}

size_t lds_bytes(int flag_rows, int flag_sets) {
  return static_cast<size_t>(kMaskOffset) + static_cast<size_t>(flag_rows) * flag_sets + 16;
}

}  // namespace

bool mfma_bf16_supports(int dtype, int D) { return dtype == 1 && D == 64; }

hipError_t launch_mfma_bf16_fwd(const Problem& p, const Plan& plan) {
  const bf16* Q = static_cast<const bf16*>(p.Q);
  const bf16* K = static_cast<const bf16*>(p.K);
  const bf16* V = static_cast<const bf16*>(p.V);
  bf16* O = static_cast<bf16*>(p.O);
  const unsigned BH = static_cast<unsigned>(p.B) * p.H;
  hipError_t err;
  if (plan.path == Plan::kFused) {
    const size_t lds = lds_bytes((p.N + TR - 1) / TR * TR, 1);
    if ((err = allow_lds(fused_fwd_kernel, lds)) != hipSuccess) return err;
    hipLaunchKernelGGL(fused_fwd_kernel, dim3(BH), dim3(kThreads), lds, p.stream, Q, K, V, p.mask,
                       O, p.H, p.N, p.scale, p.eps);
    return hipGetLastError();
  }
  const size_t lds = lds_bytes(plan.rows_per_split, 1);
  if ((err = allow_lds(split_state_kernel, lds)) != hipSuccess) return err;
  if ((err = allow_lds(split_apply_fwd_kernel, lds)) != hipSuccess) return err;
  const dim3 grid(BH * plan.splits, 1, 1);
  hipLaunchKernelGGL(split_state_kernel, grid, dim3(kThreads), lds, p.stream, Q, K, V,
                     static_cast<const bf16*>(nullptr), p.mask, p.workspace, p.H, p.N, plan.splits,
                     plan.rows_per_split, size_t{0}, p.eps);
  const float* states = launch_reduce_states(p, plan, 1);
  hipLaunchKernelGGL(split_apply_fwd_kernel, grid, dim3(kThreads), lds, p.stream, Q, states, O,
                     p.N, plan.splits, plan.rows_per_split, p.scale, p.eps);
  return hipGetLastError();
}

hipError_t launch_mfma_bf16_bwd(const Problem& p, const Plan& plan) {
  const bf16* Q = static_cast<const bf16*>(p.Q);
  const bf16* K = static_cast<const bf16*>(p.K);
  const bf16* V = static_cast<const bf16*>(p.V);
  const bf16* dO = static_cast<const bf16*>(p.dO);
  bf16* dQ = static_cast<bf16*>(p.dQ);
  bf16* dK = static_cast<bf16*>(p.dK);
  bf16* dV = static_cast<bf16*>(p.dV);
  const unsigned BH = static_cast<unsigned>(p.B) * p.H;
  hipError_t err;
  if (plan.path == Plan::kFused) {
    const size_t lds = lds_bytes((p.N + TR - 1) / TR * TR, 1);
    if ((err = allow_lds(fused_bwd_kernel, lds)) != hipSuccess) return err;
    hipLaunchKernelGGL(fused_bwd_kernel, dim3(BH), dim3(kThreads), lds, p.stream, Q, K, V, p.mask,
                       dO, dQ, dK, dV, p.H, p.N, p.scale, p.eps);
    return hipGetLastError();
  }
  const size_t lds = lds_bytes(plan.rows_per_split, 1);
  if ((err = allow_lds(split_state_kernel, lds)) != hipSuccess) return err;
  if ((err = allow_lds(split_apply_bwd_kernel, lds)) != hipSuccess) return err;
  const dim3 grid(BH * plan.splits, 2, 1);
  const size_t second = static_cast<size_t>(BH) * plan.splits * D * D;
  hipLaunchKernelGGL(split_state_kernel, grid, dim3(kThreads), lds, p.stream, Q, K, V, dO, p.mask,
                     p.workspace, p.H, p.N, plan.splits, plan.rows_per_split, second, p.eps);
  const float* states = launch_reduce_states(p, plan, 2);
  const float* dstates = states + (plan.splits == 1 ? second : static_cast<size_t>(BH) * D * D);
  hipLaunchKernelGGL(split_apply_bwd_kernel, grid, dim3(kThreads), lds, p.stream, Q, K, V, dO,
                     p.mask, states, dstates, dQ, dK, dV, p.H, p.N, plan.splits,
                     plan.rows_per_split, p.scale, p.eps);
  return hipGetLastError();
}

}  // namespace cotten
