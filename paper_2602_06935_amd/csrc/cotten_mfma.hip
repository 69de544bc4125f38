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

// The implementation is compiled twice: 4 waves per workgroup (every kernel), and 8 waves per
// workgroup for the short fp32 kernels that keep their tiles in registers (half as many tiles
// per wave: the chain of a workgroup is that much shorter).
#define COTTEN_STREAM_WAVES 8
#define COTTEN_STREAM_NS stream8
#include "cotten_stream_impl.inc"
#undef COTTEN_STREAM_WAVES
#undef COTTEN_STREAM_NS
#define COTTEN_STREAM_WAVES 4
#define COTTEN_STREAM_NS stream4
#include "cotten_stream_impl.inc"
#undef COTTEN_STREAM_WAVES
#undef COTTEN_STREAM_NS

namespace cotten {

using namespace mfma;

// Full-width rows (128 bytes) and narrower rows (64 or 32 bytes, run zero-padded on the same
// formats).
bool mfma_supports(int dtype, int D) {
  return dtype == 0 ? (D == 32 || D == 16) : (D == 64 || D == 32 || D == 16);
}

int mfma_state_dim(int dtype) { return dtype == 0 ? F32x32::D : Bf16x64::D; }

hipError_t launch_mfma_fwd(const Problem& p, const Plan& plan) {
  if (p.feature_map == kMapElu1)
    return p.dtype == 1   ? stream4::run_fwd<WithElu1<Bf16x64>>(p, plan)
           : p.dtype == 2 ? stream4::run_fwd<WithElu1<F16x64>>(p, plan)
                          : stream4::run_fwd<WithElu1<F32x32>>(p, plan);
  return p.dtype == 1   ? stream4::run_fwd<Bf16x64>(p, plan)
         : p.dtype == 2 ? stream4::run_fwd<F16x64>(p, plan)
                        : stream4::run_fwd<F32x32>(p, plan);
}

hipError_t launch_mfma_bwd(const Problem& p, const Plan& plan) {
  if (p.feature_map == kMapElu1)
    return p.dtype == 1   ? stream4::run_bwd<WithElu1<Bf16x64>>(p, plan)
           : p.dtype == 2 ? stream4::run_bwd<WithElu1<F16x64>>(p, plan)
                          : stream4::run_bwd<WithElu1<F32x32>>(p, plan);
  return p.dtype == 1   ? stream4::run_bwd<Bf16x64>(p, plan)
         : p.dtype == 2 ? stream4::run_bwd<F16x64>(p, plan)
                        : stream4::run_bwd<F32x32>(p, plan);
}

hipError_t launch_chunk_states(const Problem& p, int chunk_tiles, int chunks, bool with_queries) {
  return p.dtype == 1   ? stream4::run_chunk_states<Bf16x64>(p, chunk_tiles, chunks, with_queries)
         : p.dtype == 2 ? stream4::run_chunk_states<F16x64>(p, chunk_tiles, chunks, with_queries)
                        : stream4::run_chunk_states<F32x32>(p, chunk_tiles, chunks, with_queries);
}

}  // namespace cotten
