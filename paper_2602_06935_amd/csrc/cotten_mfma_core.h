// Device code shared by the MFMA kernels for 128-byte rows (bf16 d_h = 64, fp32 d_h = 32):
// lane geometry, the two element formats with their MFMA products, tile loads through
// buffer resources, staging into LDS tiles, and the epilogue helpers.
#pragma once
#include "cotten_device.h"

namespace cotten {
namespace mfma {

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x4_t __attribute__((ext_vector_type(4)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));

constexpr int TR = 16;               // rows per wave tile
constexpr int kRowBytes = 128;       // bytes of one tile row: d_h elements, or d_h/2 elements
                                     // followed by zeros (half-width rows)
constexpr int kTileStride = 144;     // bytes per row of an LDS tile (128 + 16 of padding)
constexpr int kTileBytes = TR * kTileStride;

// Sum over the 8 consecutive lanes that share one row, by lane-permuting adds (no LDS).
__device__ __forceinline__ float row_sum8(float x) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0xB1, 0xF, 0xF, true));   // lane ^ 1
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x4E, 0xF, 0xF, true));   // lane ^ 2
  x += __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, x), 0x141, 0xF, 0xF, true));  // other quad of the 8
  return x;
}

// 1/sqrt(ss + eps) for a live row (hardware reciprocal square root, about 1 ulp), 0 otherwise.
__device__ __forceinline__ float inv_norm_or_zero(float ss, float eps, bool live) {
  return live ? __builtin_amdgcn_rsqf(ss + eps) : 0.0f;
}

__device__ __forceinline__ void wave_lds_fence() {
  __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
  __builtin_amdgcn_wave_barrier();
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  bf16x2_t v;
  v[0] = static_cast<__bf16>(lo);
  v[1] = static_cast<__bf16>(hi);
  return __builtin_bit_cast(uint32_t, v);
}

__device__ __forceinline__ f32x4_t quad(const f32x16_t& a, int j) {
  return f32x4_t{a[4 * j], a[4 * j + 1], a[4 * j + 2], a[4 * j + 3]};
}

// Lane geometry shared by every pass.
struct Lane {
  int lane, wave;
  int r8, ch;    // load layout: tile rows r8 and r8+8, bytes 16*ch .. 16*ch+15 of the row
  int i16, g16;  // MFMA 16-lane groups: lane%16, lane/16
  __device__ __forceinline__ Lane() {
    set(threadIdx.x & 63);
    wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // uniform: lives in a scalar register
  }
  // The same geometry, recomputed from scratch where it is used: in a long kernel this keeps
  // the per-lane offsets derived from it from being carried (and spilled) across phases.
  __device__ __forceinline__ Lane again() const {
    Lane l = *this;
    int id = lane;
    asm volatile("" : "+v"(id));
    l.set(id);
    return l;
  }
  __device__ __forceinline__ void set(int id) {
    lane = id;
    r8 = lane >> 3;
    ch = lane & 7;
    i16 = lane & 15;
    g16 = lane >> 4;
  }
};

// ---- the two element formats ----------------------------------------------------------
//
// Common vocabulary of a format F:
//   F::D                  head dimension;  F::EPL = D/8 elements per lane in the load layout
//   F::unpack / F::pack   128-bit register group <-> EPL floats
//   F::Acc                accumulators of one D x D state per wave, with mfma() and the
//                         column-major image R[n*(D+4)+m] used for the cross-wave sum
//   F::Operand            a D x D matrix W held in registers for apply products, loaded from
//                         an LDS image op[n][k] (k contiguous); F::apply(tile, W, out)
//   F::write_image        builds such images from a reduced state

// The two 16-bit element types of the d_h = 64 format: how a pair sits in a 32-bit word, and
// the matrix-core and transposing-read instructions of the type.
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4_t __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8_t __attribute__((ext_vector_type(8)));

struct Bf16Elem {
  typedef bf16x8_t v8;
  typedef bf16x4_t v4;
  static __device__ __forceinline__ float lo(uint32_t w) { return __uint_as_float(w << 16); }
  static __device__ __forceinline__ float hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) { return pack_bf16(a, b); }
  static __device__ __forceinline__ f32x16_t mfma32(v8 a, v8 b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x4_t mfma16(v8 a, v8 b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ v4 read_tr(const unsigned char* p) {
    typedef v4 __attribute__((address_space(3))) * lds_v4;
    return __builtin_amdgcn_ds_read_tr16_b64_v4bf16((lds_v4)(p));
  }
  // 16x16x16: A lane (i = lane%16, k = 4*(lane/16) + e), B lane (j = lane%16, same k): the k
  // a lane holds is the row group it holds of a 16x16 result, so a result (rounded) can be fed
  // back as the B operand without moving between lanes
  static __device__ __forceinline__ f32x4_t mfma_k16(v4 a, v4 b, f32x4_t c) {
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    return __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(__builtin_bit_cast(s16x4_t, a),
                                                     __builtin_bit_cast(s16x4_t, b), c, 0, 0, 0);
  }
  static __device__ __forceinline__ v4 pack4(f32x4_t x) {
    u32x2_t r = {pack2(x[0], x[1]), pack2(x[2], x[3])};
    return __builtin_bit_cast(v4, r);
  }
};

struct F16Elem {
  typedef f16x8_t v8;
  typedef f16x4_t v4;
  static __device__ __forceinline__ float lo(uint32_t w) {
    return static_cast<float>(__builtin_bit_cast(f16x2_t, w)[0]);
  }
  static __device__ __forceinline__ float hi(uint32_t w) {
    return static_cast<float>(__builtin_bit_cast(f16x2_t, w)[1]);
  }
  static __device__ __forceinline__ uint32_t pack2(float a, float b) {  // round to nearest even
    f16x2_t v;
    v[0] = static_cast<_Float16>(a);
    v[1] = static_cast<_Float16>(b);
    return __builtin_bit_cast(uint32_t, v);
  }
  static __device__ __forceinline__ f32x16_t mfma32(v8 a, v8 b, f32x16_t c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x4_t mfma16(v8 a, v8 b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ v4 read_tr(const unsigned char* p) {
    typedef __fp16 raw4 __attribute__((ext_vector_type(4)));
    typedef raw4 __attribute__((address_space(3))) * lds_v4;
    return __builtin_bit_cast(v4, __builtin_amdgcn_ds_read_tr16_b64_v4f16((lds_v4)(p)));
  }
  static __device__ __forceinline__ f32x4_t mfma_k16(v4 a, v4 b, f32x4_t c) {
    return __builtin_amdgcn_mfma_f32_16x16x16f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ v4 pack4(f32x4_t x) {
    u32x2_t r = {pack2(x[0], x[1]), pack2(x[2], x[3])};
    return __builtin_bit_cast(v4, r);
  }
};

template <class E>
struct Half64 {
  typedef E Elem;
  static constexpr int kMap = 0;  // what is done to the rows of Q and K: see FeatureMap
  typedef typename E::v8 v8_t;
  typedef typename E::v4 v4_t;
  static constexpr int D = 64, EPL = 8, NT = 4;
  // tiles in flight ahead of the one being processed, per pass (register budget permitting)
  static constexpr int kDepthState = 3, kDepthFwd = 3, kDepthQ = 2, kDepthKV = 2, kDepthQAccum = 1;
  // keep-all-tiles-in-registers variants of the fused kernels: forward only (the backward
  // does not have the registers)
  static constexpr bool kShortFwd = true, kShortBwd = false;
  static constexpr int kImageStride = 72;                 // elements per image row
  static constexpr int kImageBytes = D * kImageStride * 2;
  // Apply products leave lane (i16, g16) with the columns 32j + 8*g16 .. +7 (j = 0, 1) of tile
  // row i16: value 4*nt + v of the lane is column out_col(nt, g16) + v.  Image row n (an
  // output column of the product) is therefore kept at position image_row(n), which puts the
  // 16 rows one MFMA operand needs next to each other.
  static __device__ __forceinline__ int out_col(int nt, int g16) {
    return 32 * (nt >> 1) + 8 * g16 + 4 * (nt & 1);
  }
  static __device__ __forceinline__ int image_row(int n) {
    return 16 * (2 * (n >> 5) + ((n >> 2) & 1)) + 4 * ((n >> 3) & 3) + (n & 3);
  }

  static __device__ __forceinline__ void unpack(const u32x4_t r, float (&f)[8]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      f[2 * i] = E::lo(r[i]);
      f[2 * i + 1] = E::hi(r[i]);
    }
  }
  static __device__ __forceinline__ u32x4_t pack(const float (&f)[8]) {
    u32x4_t r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = E::pack2(f[2 * i], f[2 * i + 1]);
    return r;
  }

  // Operand of the 32x32x16 MFMA for a contraction over the 16 tile rows: lane gets, for
  // column cbase + lane%32, the 8 rows 8*(lane/32) .. +7 (two transposing reads of 4 rows).
  static __device__ __forceinline__ v8_t rows_operand(const unsigned char* T, const Lane& L,
                                                          int cbase) {
    const int s = L.i16;
    const int row = 8 * (L.g16 >> 1) + (s >> 2);
    const int col = cbase + 16 * (L.g16 & 1) + 4 * (s & 3);
    const unsigned char* p = T + row * kTileStride + col * 2;
    const v4_t lo = E::read_tr(p);
    const v4_t hi = E::read_tr(p + 4 * kTileStride);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  }

  struct Acc {
    f32x16_t v[2][2];  // [row block of 32][column block of 32]
    __device__ __forceinline__ void zero() {
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int c = 0; c < 2; ++c)
#pragma unroll
          for (int i = 0; i < 16; ++i) v[a][c][i] = 0.0f;
    }
    // += (X tile)^T (Y tile)
    __device__ __forceinline__ void mfma(const unsigned char* Xt, const unsigned char* Yt,
                                         const Lane& L) {
      v8_t a[2], b[2];
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        a[t] = rows_operand(Xt, L, 32 * t);
        b[t] = rows_operand(Yt, L, 32 * t);
      }
#pragma unroll
      for (int at = 0; at < 2; ++at)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
          v[at][ct] = E::mfma32(a[at], b[ct], v[at][ct]);
    }
    // group g = 0..15 of four consecutive state rows held by this lane, and where it lives
    __device__ __forceinline__ f32x4_t group(int g) const { return quad(v[g >> 3][(g >> 2) & 1], g & 3); }
    static __device__ __forceinline__ int group_row(int g, const Lane& L) {
      return 32 * (g >> 3) + 8 * (g & 3) + 4 * (L.lane >> 5);
    }
    static __device__ __forceinline__ int group_col(int g, const Lane& L) {
      return 32 * ((g >> 2) & 1) + (L.lane & 31);
    }
    static constexpr int kGroups = 16;
  };

  struct Operand {
    v8_t frag[4][2];
    __device__ __forceinline__ void load(const unsigned char* image, const Lane& L) {
#pragma unroll
      for (int nt = 0; nt < 4; ++nt)
#pragma unroll
        for (int ks = 0; ks < 2; ++ks)
          frag[nt][ks] = *reinterpret_cast<const v8_t*>(
              image + ((16 * nt + L.i16) * kImageStride + 8 * L.g16 + 32 * ks) * 2);
    }
  };

  // The 16 rows of an LDS tile as the other operand of an apply product: lane (i16, g16)
  // holds bytes 64j + 16*g16 .. +15 (j = 0, 1) of row i16, the same columns an apply product
  // leaves it with, so a tile fetched this way also serves as the epilogue's row operand.
  struct TileRows {
    v8_t a[2];
    __device__ __forceinline__ void load(const unsigned char* T, const Lane& L) {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        a[ks] = *reinterpret_cast<const v8_t*>(T + L.i16 * kTileStride + (8 * L.g16 + 32 * ks) * 2);
    }
    __device__ __forceinline__ void unpack(float (&f)[16]) const {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        float h[8];
        Half64::unpack(__builtin_bit_cast(u32x4_t, a[ks]), h);
#pragma unroll
        for (int i = 0; i < 8; ++i) f[8 * ks + i] = h[i];
      }
    }
    // Makes the next unpack() a fresh computation, so that the 16 floats of the previous
    // one need not stay in registers in between.
    __device__ __forceinline__ void forget_unpacked() {
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) {
        u32x4_t r = __builtin_bit_cast(u32x4_t, a[ks]);
        asm volatile("" : "+v"(r));
        a[ks] = __builtin_bit_cast(v8_t, r);
      }
    }
  };
  // (tile rows) x W, computed transposed (W^T X^T) so that each lane ends up with runs of
  // neighbouring columns of one row: out[nt][v] = T[row i16][column out_col(nt, g16) + v]
  static __device__ __forceinline__ void apply(const TileRows& X, const Operand& W,
                                               f32x4_t (&out)[4]) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) {
      out[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int ks = 0; ks < 2; ++ks)
        out[nt] = E::mfma16(W.frag[nt][ks], X.a[ks], out[nt]);
    }
  }
  static __device__ __forceinline__ void apply(const unsigned char* T, const Operand& W,
                                               const Lane& L, f32x4_t (&out)[4]) {
    TileRows X;
    X.load(T, L);
    apply(X, W, out);
  }
  // out += (tile rows) x W
  static __device__ __forceinline__ void apply_onto(const TileRows& X, const Operand& W,
                                                    f32x4_t (&out)[4]) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
#pragma unroll
      for (int ks = 0; ks < 2; ++ks) out[nt] = E::mfma16(W.frag[nt][ks], X.a[ks], out[nt]);
  }

  // Products of two 16-row tiles, for the kernels that work tile pair by tile pair:
  // dots(a, b) = X_a X_b^T: lane (j, g) gets rows 4g .. 4g+3 (rows of a) of column j (row of b).
  static __device__ __forceinline__ f32x4_t dots(const TileRows& a, const TileRows& b) {
    f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) d = E::mfma16(a.a[ks], b.a[ks], d);
    return d;
  }
  // out += X^T P for the tile X at `T` and a 16 x 16 matrix P as dots() leaves it (rounded to
  // the element type): a 16x16 result leaves a lane with exactly the k it holds of a 16x16x16 B
  // operand, so P goes in without moving between lanes; X^T comes from the transposing LDS
  // read (lane i of a 16-lane group gets rows 4g .. 4g+3 of column out_col(nt, i/4) + i%4), so
  // the result lands in the product layout.
  static __device__ __forceinline__ void add_transposed_product(const unsigned char* T,
                                                                const Lane& L, f32x4_t p,
                                                                f32x4_t (&out)[4]) {
    const v4_t pb = E::pack4(p);
#pragma unroll
    for (int nt = 0; nt < 4; ++nt)
      out[nt] = E::mfma_k16(E::read_tr(T + (4 * L.g16 + (L.i16 >> 2)) * kTileStride +
                                       out_col(nt, L.i16 & 3) * 2),
                            pb, out[nt]);
  }

  // One 32x32 block of a state, accumulated by one wave over LDS-resident tiles
  // (block = 0..3: rows 32*(block/2).., columns 32*(block%2)..), and its way into operand images.
  struct BlockAcc {
    static constexpr int kBlocks = 4;
    f32x16_t v;
    __device__ __forceinline__ void zero() {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = 0.0f;
    }
    struct Frag {
      v8_t a, b;
    };
    static __device__ __forceinline__ Frag fetch(const unsigned char* Xt, const unsigned char* Yt,
                                                 const Lane& L, int block) {
      Frag f;
      f.a = rows_operand(Xt, L, 32 * (block >> 1));
      f.b = rows_operand(Yt, L, 32 * (block & 1));
      return f;
    }
    __device__ __forceinline__ void mma(const Frag& f) {
      v = E::mfma32(f.a, f.b, v);
    }
    // += (Y block)^T (X block): the transpose of what mma() adds
    __device__ __forceinline__ void mma_swapped(const Frag& f) {
      v = E::mfma32(f.b, f.a, v);
    }
    // The lane holds, of the accumulated block, column lane%32 and rows 8j + 4*(lane/32) .. +3:
    // four neighbours of image row (c0 + column), which go out as one 64-bit write.
    //   after mma():          r0 = 32*(block/2), c0 = 32*(block%2)  ->  image[n][m] (transposed)
    //   after mma_swapped():  r0 = 32*(block%2), c0 = 32*(block/2)  ->  image[m][n] (natural)
    __device__ __forceinline__ void write_image(const Lane& L, int r0, int c0, float scale,
                                                unsigned char* image) const {
      const int c = c0 + (L.lane & 31);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = r0 + 8 * j + 4 * (L.lane >> 5);
        uint32_t* p = reinterpret_cast<uint32_t*>(image + (image_row(c) * kImageStride + r) * 2);
        p[0] = E::pack2(v[4 * j] * scale, v[4 * j + 1] * scale);
        p[1] = E::pack2(v[4 * j + 2] * scale, v[4 * j + 3] * scale);
      }
    }
    // Sum over this lane's elements of (accumulated block) x (the block of another matrix
    // read back from an image written by write_image with the same r0, c0).
    __device__ __forceinline__ float dot_image(const Lane& L, int r0, int c0,
                                               const unsigned char* image) const {
      const int c = c0 + (L.lane & 31);
      float s = 0.0f;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int r = r0 + 8 * j + 4 * (L.lane >> 5);
        const uint32_t* p =
            reinterpret_cast<const uint32_t*>(image + (image_row(c) * kImageStride + r) * 2);
        const uint32_t lo = p[0], hi = p[1];
        s += v[4 * j] * E::lo(lo) + v[4 * j + 1] * E::hi(lo);
        s += v[4 * j + 2] * E::lo(hi) + v[4 * j + 3] * E::hi(hi);
      }
      return s;
    }
    static __device__ __forceinline__ int block_row0(int block) { return 32 * (block >> 1); }
    static __device__ __forceinline__ int block_col0(int block) { return 32 * (block & 1); }
  };

  // two neighbouring image elements (k, k+1) of image row n
  static __device__ __forceinline__ void write_image_pair(unsigned char* image, int n, int k,
                                                          float v0, float v1) {
    *reinterpret_cast<uint32_t*>(image + (image_row(n) * kImageStride + k) * 2) = E::pack2(v0, v1);
  }
  // The same in two steps, for writers that split (n, k) into a per-lane and a compile-time part:
  // image_offset is additive over parts that share no bit of n (a permutation of bits) and in k.
  static __device__ __forceinline__ int image_offset(int n, int k) {
    return (image_row(n) * kImageStride + k) * 2;
  }
  static __device__ __forceinline__ void write_pair_at(unsigned char* at, float v0, float v1) {
    *reinterpret_cast<uint32_t*>(at) = E::pack2(v0, v1);
  }
  // element k of image row n
  static __device__ __forceinline__ float image_at(const unsigned char* image, int n, int k) {
    const uint32_t h =
        *reinterpret_cast<const uint16_t*>(image + (image_row(n) * kImageStride + k) * 2);
    return E::lo(h);
  }
};

typedef Half64<Bf16Elem> Bf16x64;
typedef Half64<F16Elem> F16x64;

struct F32x32 {
  typedef float io_t;
  static constexpr int kMap = 0;
  static constexpr int D = 32, EPL = 4, NT = 2;
  static constexpr int kDepthState = 3, kDepthFwd = 3, kDepthQ = 3, kDepthKV = 2, kDepthQAccum = 2;
  static constexpr bool kShortFwd = true, kShortBwd = true;
  static constexpr int kImageStride = 36;
  static constexpr int kImageBytes = D * kImageStride * 4;
  // Apply products leave lane (i16, g16) with the columns 16j + 4*g16 .. +3 (j = 0, 1) of tile
  // row i16 (value 4*nt + v is column out_col(nt, g16) + v); image rows stay in place.
  static __device__ __forceinline__ int out_col(int nt, int g16) { return 16 * nt + 4 * g16; }
  static __device__ __forceinline__ int image_row(int n) { return n; }

  static __device__ __forceinline__ void unpack(const u32x4_t r, float (&f)[4]) {
#pragma unroll
    for (int i = 0; i < 4; ++i) f[i] = __uint_as_float(r[i]);
  }
  static __device__ __forceinline__ u32x4_t pack(const float (&f)[4]) {
    u32x4_t r;
#pragma unroll
    for (int i = 0; i < 4; ++i) r[i] = __float_as_uint(f[i]);
    return r;
  }

  struct Acc {
    f32x16_t v;
    __device__ __forceinline__ void zero() {
#pragma unroll
      for (int i = 0; i < 16; ++i) v[i] = 0.0f;
    }
    // += (X tile)^T (Y tile): 32x32x2 steps, lane = column, half-wave = row of the pair
    __device__ __forceinline__ void mfma(const unsigned char* Xt, const unsigned char* Yt,
                                         const Lane& L) {
      const int off = (L.lane >> 5) * kTileStride + (L.lane & 31) * 4;
      float a[8], b[8];
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        a[s] = *reinterpret_cast<const float*>(Xt + off + 2 * s * kTileStride);
        b[s] = *reinterpret_cast<const float*>(Yt + off + 2 * s * kTileStride);
      }
#pragma unroll
      for (int s = 0; s < 8; ++s) v = __builtin_amdgcn_mfma_f32_32x32x2f32(a[s], b[s], v, 0, 0, 0);
    }
    __device__ __forceinline__ f32x4_t group(int g) const { return quad(v, g); }
    static __device__ __forceinline__ int group_row(int g, const Lane& L) {
      return 8 * g + 4 * (L.lane >> 5);
    }
    static __device__ __forceinline__ int group_col(int, const Lane& L) { return L.lane & 31; }
    static constexpr int kGroups = 4;
  };

  // frag[nt][s] = W[k(s)][16*nt + i16], contraction step s taking column
  // k(s) = 16*(s/4) + 4*g16 + s%4: the columns a TileRows lane holds.
  struct Operand {
    float frag[2][8];
    __device__ __forceinline__ void load(const unsigned char* image, const Lane& L) {
#pragma unroll
      for (int nt = 0; nt < 2; ++nt) {
        const f32x4_t* p = reinterpret_cast<const f32x4_t*>(
            image + ((16 * nt + L.i16) * kImageStride + 4 * L.g16) * 4);
        const f32x4_t lo = p[0], hi = p[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          frag[nt][i] = lo[i];
          frag[nt][4 + i] = hi[i];
        }
      }
    }
  };

  // Lane (i16, g16) holds bytes 64j + 16*g16 .. +15 (j = 0, 1) of tile row i16: the columns
  // an apply product leaves it with.
  struct TileRows {
    float a[8];
    __device__ __forceinline__ void load(const unsigned char* T, const Lane& L) {
      const f32x4_t* p = reinterpret_cast<const f32x4_t*>(T + L.i16 * kTileStride + 16 * L.g16);
      const f32x4_t lo = p[0], hi = p[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        a[i] = lo[i];
        a[4 + i] = hi[i];
      }
    }
    __device__ __forceinline__ void unpack(float (&f)[8]) const {
#pragma unroll
      for (int i = 0; i < 8; ++i) f[i] = a[i];
    }
    __device__ __forceinline__ void forget_unpacked() {}
  };
  static __device__ __forceinline__ void apply(const TileRows& X, const Operand& W,
                                               f32x4_t (&out)[2]) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt) {
      out[nt] = f32x4_t{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s = 0; s < 8; ++s)
        out[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(W.frag[nt][s], X.a[s], out[nt], 0, 0, 0);
    }
  }
  static __device__ __forceinline__ void apply(const unsigned char* T, const Operand& W,
                                               const Lane& L, f32x4_t (&out)[2]) {
    TileRows X;
    X.load(T, L);
    apply(X, W, out);
  }
  // out += (tile rows) x W
  static __device__ __forceinline__ void apply_onto(const TileRows& X, const Operand& W,
                                                    f32x4_t (&out)[2]) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int s = 0; s < 8; ++s)
        out[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(W.frag[nt][s], X.a[s], out[nt], 0, 0, 0);
  }

  // Products of two 16-row tiles (see Half64): dots(a, b) = X_a X_b^T, lane (j, g) gets rows
  // 4g .. 4g+3 of column j; eight 16x16x4 steps, each lane feeding the column it holds.
  static __device__ __forceinline__ f32x4_t dots(const TileRows& a, const TileRows& b) {
    f32x4_t d = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int s = 0; s < 8; ++s) d = __builtin_amdgcn_mfma_f32_16x16x4f32(a.a[s], b.a[s], d, 0, 0, 0);
    return d;
  }
  // out += X^T P: step v contracts over the rows 4g + v (g = 0..3), which is the row of P a lane
  // of group g holds in p[v]; the matching element of X is read from the LDS tile directly.
  static __device__ __forceinline__ void add_transposed_product(const unsigned char* T,
                                                                const Lane& L, f32x4_t p,
                                                                f32x4_t (&out)[2]) {
#pragma unroll
    for (int nt = 0; nt < 2; ++nt)
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const float x = *reinterpret_cast<const float*>(T + (4 * L.g16 + v) * kTileStride +
                                                        (16 * nt + L.i16) * 4);
        out[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(x, p[v], out[nt], 0, 0, 0);
      }
  }

  static __device__ __forceinline__ void write_image_pair(unsigned char* image, int n, int k,
                                                          float v0, float v1) {
    float* p = reinterpret_cast<float*>(image + (n * kImageStride + k) * 4);
    p[0] = v0;
    p[1] = v1;
  }
  static __device__ __forceinline__ int image_offset(int n, int k) { return (n * kImageStride + k) * 4; }
  static __device__ __forceinline__ void write_pair_at(unsigned char* at, float v0, float v1) {
    float* p = reinterpret_cast<float*>(at);
    p[0] = v0;
    p[1] = v1;
  }
  static __device__ __forceinline__ float image_at(const unsigned char* image, int n, int k) {
    return *reinterpret_cast<const float*>(image + (n * kImageStride + k) * 4);
  }
};

// What a format does to the rows of Q and K before they enter the products:
//   kMapCosine  x / sqrt(|x|^2 + eps)   row-wise L2 normalisation (the paper's model)
//   kMapElu1    ELU(x) + 1              element-wise (the linear-attention comparison model of
//                                       "Linear Attention Models"); eps plays no part
// A format with the second map is the same format with kMap overridden: every pass picks the
// staging mode and the row epilogue from F::kMap.
enum FeatureMap { kMapCosine = 0, kMapElu1 = 1 };
template <class Base>
struct WithElu1 : Base {
  static constexpr int kMap = kMapElu1;
};

// phi(x) = ELU(x) + 1 with alpha = 1: x + 1 above zero, exp(x) below (hardware exp2, about
// 1 ulp).  Its derivative is 1 above zero and exp(x) below, i.e. min(phi(x), 1).
__device__ __forceinline__ float elu1(float x) {
  return x > 0.0f ? x + 1.0f : __builtin_amdgcn_exp2f(x * 1.44269504088896340736f);
}

// ---- tiles --------------------------------------------------------------------------------

// The tiles one workgroup walks: local tile lt = 0 .. n_tiles-1 is tile (tile0 + lt * stride)
// of the slice, i.e. rows 16*(tile0 + lt*stride) .. +15.  A fused workgroup has stride 1; in
// the split path the tiles of a slice are dealt round-robin to its `splits` workgroups, so
// that padding (which sits at one end of the sequence) is shared evenly.  Rows >= limit do
// not exist; `flags`, if given, is the LDS copy of the key mask: flags[16*lt + r].
struct Rows {
  int tile0, stride, n_tiles, limit;
  const uint8_t* flags;
  __device__ __forceinline__ int row0(int lt) const { return (tile0 + lt * stride) * TR; }
};

// Raw 16-row tile in the load layout: x[h], y[h] hold row r8 + 8h; `live` bit h says the
// row takes part (in range and, where a mask applies, a valid key).
struct Raw {
  u32x4_t x[2], y[2];
  int live;
};

// The two tensors a pass reads, as buffer resources over one slice each.  Buffer loads are
// used instead of flat loads because a lane whose offset lies outside the buffer gets zeros
// and causes no memory traffic: rows that do not take part are skipped without a branch, so
// every tile issues the same number of load instructions and the hardware's in-order load
// counter can tell "this tile has arrived" from "the tiles prefetched after it have not".
// How the rows of a slice are addressed in global memory: `stride` bytes apart, `bytes` bytes
// each (128, or 64 / 32 for narrower rows: d_h = 32 or 16 with 16-bit elements, d_h = 16 with
// fp32 - those run on the full-width formats with the rest of every tile row held at zero,
// which leaves all results unchanged).
struct RowAddr {
  int stride, bytes;
};

// Where the slices are (bytes): slice (b,h) starts at b*batch + h*head.
// [B,H,N,d]: batch = H*N*row bytes, head = N*row bytes, stride = row bytes;
// [B,N,H,d]: batch = N*H*row bytes, head = row bytes, stride = H*row bytes.
struct Strides {
  long long batch, head;
  RowAddr row;
  __device__ __forceinline__ size_t slice_base(int bh, int H) const {
    return static_cast<size_t>(bh / H) * batch + static_cast<size_t>(bh % H) * head;
  }
};

struct Src {
  __amdgpu_buffer_rsrc_t x, y;
  RowAddr row;
  __device__ __forceinline__ Src(const unsigned char* X, const unsigned char* Y, int N,
                                 RowAddr row_addr)
      : row(row_addr) {
    const int bytes = (N - 1) * row.stride + row.bytes;
    x = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(X), 0, bytes, 0x00020000);
    y = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(Y), 0, bytes, 0x00020000);
  }
  // byte offset of the lane's 16 bytes of `row`, outside the buffer (zeros, no traffic) when
  // the row does not take part or the lane's columns are padding
  __device__ __forceinline__ uint32_t offset(int row_index, bool live, const Lane& L) const;
};
constexpr uint32_t kOutOfBuffer = 0x80000000u;
__device__ __forceinline__ uint32_t Src::offset(int row_index, bool live, const Lane& L) const {
  return (live && L.ch * 16 < row.bytes) ? static_cast<uint32_t>(row_index) * row.stride + L.ch * 16
                                         : kOutOfBuffer;
}

// Loads local tile lt (all zeros, and no traffic, if lt is not one of the workgroup's tiles).
// A row takes part when it is below rows.limit and, if rows.flags is given, its flag is set.
template <bool USE_Y>
__device__ __forceinline__ void load_raw(Raw& r, const Lane& L, const Src& src, const Rows& rows,
                                         int lt) {
  r.live = 0;
  const bool tile_ok = lt < rows.n_tiles;
  const int row0 = rows.row0(lt);
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int row = row0 + L.r8 + 8 * h;
    bool live = tile_ok && row < rows.limit;
    if (rows.flags != nullptr) live = live && rows.flags[tile_ok ? lt * TR + L.r8 + 8 * h : 0] != 0;
    const uint32_t off = src.offset(row, live, L);
    r.x[h] = __builtin_amdgcn_raw_buffer_load_b128(src.x, off, 0, 0);
    if (USE_Y) r.y[h] = __builtin_amdgcn_raw_buffer_load_b128(src.y, off, 0, 0);
    else r.y[h] = u32x4_t{0, 0, 0, 0};
    r.live |= static_cast<int>(live) << h;
  }
}

// What becomes of the x rows on their way to the LDS tile.
enum XMode { kXNone = 0, kXRaw = 1, kXNormalized = 2, kXFeature = 3 };

// The staging mode of rows that enter a product through the feature map of the format.
template <class F>
constexpr int mapped_mode() {
  return F::kMap == kMapElu1 ? kXFeature : kXNormalized;
}

// inv[h] = 1/r of row h (0 for rows that do not take part; their registers are zero).
// Xt receives nothing, the raw rows, xhat, or phi(x) (kXFeature: then inv[h] is 1 for a row
// that takes part, and `cols` says whether the lane's columns exist - phi(0) is not 0, so
// padding columns and absent rows are written as zeros explicitly); Yt the raw y rows.
template <class F, int XMODE, bool USE_Y>
__device__ __forceinline__ void stage(const Raw& r, const Lane& L, float eps, unsigned char* Xt,
                                      unsigned char* Yt, float (&inv)[2], bool cols = true) {
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float f[F::EPL];
    F::unpack(r.x[h], f);
    if (XMODE == kXFeature) {
      const bool live = ((r.live >> h) & 1) != 0;
      inv[h] = live ? 1.0f : 0.0f;
#pragma unroll
      for (int i = 0; i < F::EPL; ++i) f[i] = (live && cols) ? elu1(f[i]) : 0.0f;
      const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
      *reinterpret_cast<u32x4_t*>(Xt + off) = F::pack(f);
      if (USE_Y) *reinterpret_cast<u32x4_t*>(Yt + off) = r.y[h];
      continue;
    }
    float ss = 0.0f;
#pragma unroll
    for (int i = 0; i < F::EPL; ++i) ss += f[i] * f[i];
    inv[h] = inv_norm_or_zero(row_sum8(ss), eps, (r.live >> h) & 1);
    const int off = (L.r8 + 8 * h) * kTileStride + L.ch * 16;
    if (XMODE == kXNormalized) {
#pragma unroll
      for (int i = 0; i < F::EPL; ++i) f[i] *= inv[h];
      *reinterpret_cast<u32x4_t*>(Xt + off) = F::pack(f);
    } else if (XMODE == kXRaw) {
      *reinterpret_cast<u32x4_t*>(Xt + off) = r.x[h];
    }
    if (USE_Y) *reinterpret_cast<u32x4_t*>(Yt + off) = r.y[h];
  }
}

// ---- epilogues in the product layout ------------------------------------------------------
// An apply product leaves lane (i16, g16) with 2*EPL values of tile row i16: the two 16-byte
// pieces of the row at bytes 64j + 16*g16.  TileRows::unpack gives any LDS tile in the same
// arrangement, so row-wise epilogues need no detour through an fp32 scratch tile.

template <class F>
__device__ __forceinline__ void product_rows(const f32x4_t (&out)[F::NT], float (&p)[2 * F::EPL]) {
  static_assert(4 * F::NT == 2 * F::EPL, "an apply product covers one row");
#pragma unroll
  for (int nt = 0; nt < F::NT; ++nt)
#pragma unroll
    for (int v = 0; v < 4; ++v) p[4 * nt + v] = out[nt][v];
}

// Sum over the 64 lanes of the wave, every lane gets it (fixed butterfly order).
__device__ __forceinline__ float wave_sum(float x) {
#pragma unroll
  for (int w = 1; w < 64; w <<= 1) x += __shfl_xor(x, w);
  return x;
}

// Sum over the four lanes (i16, 0..3) that share a row.
__device__ __forceinline__ float row_sum_groups(float x, const Lane& L) {
  x += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((L.lane ^ 16) << 2, __builtin_bit_cast(int, x)));
  x += __builtin_bit_cast(float, __builtin_amdgcn_ds_bpermute((L.lane ^ 32) << 2, __builtin_bit_cast(int, x)));
  return x;
}

// p <- (p - u (u.p)) / r for the lane's row, u being the unit row held in `e`: the tangent
// projection shared by dQ (u = qhat, p = g) and dK (u = khat, p = h).  With LAZY the unit row
// is unpacked twice instead of being kept in registers across the row sum.
template <class F, bool LAZY>
__device__ __forceinline__ void project_rows(float (&p)[2 * F::EPL], typename F::TileRows& e,
                                             float inv_r, const Lane& L) {
  float u[2 * F::EPL];
  e.unpack(u);
  float proj = 0.0f;
#pragma unroll
  for (int c = 0; c < 2 * F::EPL; ++c) proj += u[c] * p[c];
  proj = row_sum_groups(proj, L);
  if (LAZY) {
    e.forget_unpacked();
    e.unpack(u);
  }
#pragma unroll
  for (int c = 0; c < 2 * F::EPL; ++c) p[c] = (p[c] - u[c] * proj) * inv_r;
}

// p <- p * phi'(x) element-wise, with phi(x) of the lane's row held in `e`: the chain rule
// through the ELU + 1 map (phi' = min(phi, 1)).
template <class F>
__device__ __forceinline__ void feature_grad_rows(float (&p)[2 * F::EPL],
                                                  const typename F::TileRows& e) {
  float u[2 * F::EPL];
  e.unpack(u);
#pragma unroll
  for (int c = 0; c < 2 * F::EPL; ++c) p[c] *= fminf(u[c], 1.0f);
}

// The same with the raw row x = r * u in `e`:  (p - u (u.p)) / r = p/r - x (x.p) / r^3.
template <class F>
__device__ __forceinline__ void project_rows_raw(float (&p)[2 * F::EPL],
                                                 const typename F::TileRows& e, float inv_r,
                                                 const Lane& L) {
  float x[2 * F::EPL];
  e.unpack(x);
  float proj = 0.0f;
#pragma unroll
  for (int c = 0; c < 2 * F::EPL; ++c) proj += x[c] * p[c];
  proj = row_sum_groups(proj, L) * (inv_r * inv_r * inv_r);
#pragma unroll
  for (int c = 0; c < 2 * F::EPL; ++c) p[c] = p[c] * inv_r - x[c] * proj;
}

// Cache policy of the result stores.  Results are not read again by these kernels, and with
// the default policy the written lines displace the inputs still on their way through L2.
// Measured at N = 200 on the benchmark's alternating forward / backward steps (tokens/s of the
// step, fp32 fused and bf16 resident kernels): default 1.6 G and 0.77 G; nt 1.88 G and 0.90 G;
// sc0 sc1 nt 1.91 G and 0.93 G; sc0 sc1 without nt is the best for a forward run on its own
// but loses 8 % in the step.  The split kernels (N = 4096): default 0.64 G, nt 0.63 G, sc0 sc1
// 0.63 G, sc0 sc1 nt 0.67 G.  Loads are better left with the default policy everywhere.
constexpr int kStoreDefault = 0, kStoreStreamed = 19;  // aux bits: sc0 = 1, nt = 2, sc1 = 16

template <class F, int POLICY>
__device__ __forceinline__ void store_product_row(unsigned char* __restrict__ dst, int row,
                                                  RowAddr addr, const Lane& L,
                                                  const float (&p)[2 * F::EPL]) {
  // dst is a slice base: the byte offsets of its rows fit 31 bits (checked by the caller of
  // the library entry point)
  __amdgpu_buffer_rsrc_t out;
  if (POLICY != kStoreDefault) out = __builtin_amdgcn_make_buffer_rsrc(dst, 0, 0x7fffffff, 0x00020000);
#pragma unroll
  for (int j = 0; j < 2; ++j) {
    if (64 * j + 16 * L.g16 >= addr.bytes) break;  // narrower rows: the rest is padding
    float c[F::EPL];
#pragma unroll
    for (int i = 0; i < F::EPL; ++i) c[i] = p[F::EPL * j + i];
    const uint32_t off = static_cast<uint32_t>(row) * addr.stride + 64 * j + 16 * L.g16;
    if (POLICY != kStoreDefault) __builtin_amdgcn_raw_buffer_store_b128(F::pack(c), out, off, 0, POLICY);
    else *reinterpret_cast<u32x4_t*>(dst + off) = F::pack(c);
  }
}

}  // namespace mfma
}  // namespace cotten
