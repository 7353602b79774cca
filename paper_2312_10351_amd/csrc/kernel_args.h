// Plain-data kernel argument records and the kernel list, shared by the host-side
// planner (which fills them at DAG build time) and the HIP translation unit (which
// launches them).  No HIP types here: the planner builds without a GPU toolchain.
#pragma once
#include <stdint.h>

namespace opara {

// Implicit-GEMM convolution / GEMM / strided batched GEMM.
//   D[n][m] = alpha * sum_k Wt[n][k] * Xg[m][k]   (n: output channel/column, m: pixel/row)
// Xg is either a plain matrix (gather == 0, row stride lda) or an on-the-fly patch
// gather from an [H][W][Cin] image with k = (i*kw + j)*Cin + ci (gather == 1).
struct IgemmArgs {
  const void *x, *w;
  const float *bias;
  void *y;
  const void *extra[3];
  int32_t n_extra;
  int32_t M, N, K;
  int32_t gather;
  int32_t H, W, Cin, Wo, kh, kw, sh, sw, ph, pw;
  int32_t HoWo;                 // output pixels per image; row m belongs to image m / HoWo
  int64_t img_stride;           // elements between consecutive input images (H*W*Cin)
  int64_t lda, ldb, ldy;        // row strides in elements
  int64_t a_bs, b_bs, y_bs;     // batch strides in elements (blockIdx.z)
  int32_t b_kmajor;             // second operand stored [K][N]
  int32_t relu;
  float alpha;
};

struct PoolArgs {
  const void *x;
  void *y;
  int32_t H, W, C, Ho, Wo, kh, kw, sh, sw, ph, pw;
  int32_t is_avg;
  int32_t B;                    // images
};

struct GapArgs {
  const void *x;
  void *y;
  int32_t HW, C;              // per image; blockIdx.y is the image
};

struct RowArgs {               // LayerNorm / softmax over rows of the summed inputs
  const void *in[8];
  void *y;
  int32_t n_in, rows, cols;
  float eps;
};

struct EltArgs {               // f(sum of inputs), f in {identity, relu, gelu}
  const void *in[8];
  void *y;
  int32_t n_in, op;            // op: 0 add, 1 relu, 2 gelu
  int64_t n;
};

struct ConcatArgs {
  const void *in[8];
  void *y;
  int32_t cols[8], col_off[8];
  int32_t n_in, rows, out_cols;
};

// X(name, ArgsType).  Order defines kernel ids.
#define OPARA_KERNEL_LIST(X)            \
  X(igemm_f16_t128x64, IgemmArgs)       \
  X(igemm_f16_t64x64, IgemmArgs)        \
  X(igemm_f16_direct4, IgemmArgs)       \
  X(igemm_f16_direct8, IgemmArgs)       \
  X(igemm_f16_quad4, IgemmArgs)         \
  X(igemm_f16_quad8, IgemmArgs)         \
  X(igemm_f16_quad64x4, IgemmArgs)      \
  X(igemm_f16_t64x64_scalar, IgemmArgs) \
  X(igemm_f32_t128x64, IgemmArgs)       \
  X(igemm_f32_t64x64, IgemmArgs)        \
  X(igemm_f32_direct4, IgemmArgs)       \
  X(igemm_f32_direct8, IgemmArgs)       \
  X(igemm_f32_quad4, IgemmArgs)         \
  X(igemm_f32_quad8, IgemmArgs)         \
  X(igemm_f32_quad64x4, IgemmArgs)      \
  X(igemm_f32_t64x64_scalar, IgemmArgs) \
  X(gemv_f16, IgemmArgs)                \
  X(gemv_f32, IgemmArgs)                \
  X(pool_f16_vec, PoolArgs)             \
  X(pool_f16_scalar, PoolArgs)          \
  X(pool_f32_vec, PoolArgs)             \
  X(pool_f32_scalar, PoolArgs)          \
  X(gap_f16, GapArgs)                   \
  X(gap_f32, GapArgs)                   \
  X(layernorm_f16_wave, RowArgs)        \
  X(layernorm_f16_block, RowArgs)       \
  X(layernorm_f16_generic, RowArgs)     \
  X(layernorm_f32_wave, RowArgs)        \
  X(layernorm_f32_block, RowArgs)       \
  X(layernorm_f32_generic, RowArgs)     \
  X(softmax_f16_wave, RowArgs)          \
  X(softmax_f16_block, RowArgs)         \
  X(softmax_f16_generic, RowArgs)       \
  X(softmax_f32_wave, RowArgs)          \
  X(softmax_f32_block, RowArgs)         \
  X(softmax_f32_generic, RowArgs)       \
  X(elt_f16_vec, EltArgs)               \
  X(elt_f16_scalar, EltArgs)            \
  X(elt_f32_vec, EltArgs)               \
  X(elt_f32_scalar, EltArgs)            \
  X(concat_f16_vec, ConcatArgs)         \
  X(concat_f16_scalar, ConcatArgs)      \
  X(concat_f32_vec, ConcatArgs)         \
  X(concat_f32_scalar, ConcatArgs)      \
  X(igemm_f16_direct4s, IgemmArgs)      \
  X(igemm_f16_quad4s, IgemmArgs)        \
  X(igemm_f32_direct4s, IgemmArgs)      \
  X(igemm_f32_quad4s, IgemmArgs)

enum KernelId : int32_t {
#define X(name, T) K_##name,
  OPARA_KERNEL_LIST(X)
#undef X
  K_COUNT
};

union KernelArgs {
  IgemmArgs igemm;
  PoolArgs pool;
  GapArgs gap;
  RowArgs row;
  EltArgs elt;
  ConcatArgs concat;
};

// One planned launch: which kernel, its grid and its arguments.
struct KernelPlan {
  int32_t kernel;
  uint32_t gx, gy, gz;
  uint32_t block;
  int32_t tag;                  // operator id: second kernel argument, slot of the operator timeline
  KernelArgs args;
};

// A group node: up to kGroupMaxOps mutually independent operators launched as ONE kernel
// whose grid is the sum of their grids.  Workgroup w serves the operator i with
// block_end[i-1] <= w < block_end[i]; each operator's range is padded to a multiple of the
// XCD count (padding workgroups leave at once), so that tile t of an operator runs on XCD
// t % 8 as in a launch of its own.  The record travels by value as the kernel argument.
constexpr int kGroupMaxOps = 16;
constexpr int kGroupAlign = 8;
struct GroupMeta {                                 // one member: read with one 32-byte scalar load
  int32_t kernel;                                  // KernelId of the operator's body
  int32_t gx, gy;                                  // the operator's own grid (x, y; z follows)
  int32_t tiles;                                   // gx * gy * gz
  int32_t tag;                                     // operator id (slot of the operator timeline)
  int32_t block_begin;                             // first block of the member's range
  int32_t reserved[2];
};
struct GroupArgs {
  int32_t n;
  int32_t reserved;
  unsigned long long *trace;                       // operator-timeline buffer, null = off
  int32_t block_end[kGroupMaxOps];
  GroupMeta meta[kGroupMaxOps];
  KernelArgs args[kGroupMaxOps];
};

// Tile geometry of the implicit-GEMM kernels (output columns x rows per workgroup).
struct IgemmTile { int bn, bm, threads; };
constexpr IgemmTile kTile128x64{128, 64, 256};   // 128 output columns x 64 rows
constexpr double kTiledMinFlops = 6.0e9;          // lighter contractions use the latency-oriented kernels
constexpr double kTiledMinFlopsPersistent = 2.0e9;   // inside the persistent kernel (four wavefronts per tile whatever K is)
constexpr int kTiledMinTiles = 80;               // ... and so do contractions with fewer 128x64 tiles
constexpr IgemmTile kTile64{64, 64, 256};
constexpr int64_t kQuadMinRowBytes = 1024;   // rows of K at least this long take the quad-coalesced variant
constexpr int kQuad64MinTiles = 128;             // GEMM-shaped operands with at least this many 64 x 64 tiles take them
constexpr double kQuad64MaxFlops = 4.0e10;       // ... up to this weight (measured up to 1.7e10)
constexpr int kQuadFourWaveTiles = 128;          // from this many 32 x 32 tiles on, four wavefronts per tile whatever K is
constexpr int kDirectTile = 32;       // output tile edge of the latency-oriented kernels
constexpr int kSmallTile = 16;        // ... of their small-tile forms, for operators with few 32 x 32 tiles
constexpr int kSmallTileMaxTiles32 = 100;   // at most this many 32 x 32 tiles: take 16 x 16 ones (four times as many workgroups)

constexpr int kRowGroupWave = 64;     // threads cooperating on one row (wave variant)
constexpr int kRowGroupBlock = 256;   // block variant
constexpr int kRowCacheChunks = 4;    // 16-byte chunks a thread keeps in registers
constexpr int kGemvMaxM = 4;

}  // namespace opara
