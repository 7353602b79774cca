// Kernel table and per-operator launch planning (host only, no HIP calls).
// The demand record of an operator (paper Sec. 3.2: threads, shared memory and
// registers of one block; Sec. 2.3: number of blocks) follows from the plan made
// here plus the static resources of the chosen kernel.
#include <cstring>
#include "opara_internal.h"

namespace opara {

// Generated at build time from the compiler's per-kernel resource report of
// kernels.hip; one row per entry of OPARA_KERNEL_LIST, same order.
const KernelResource kKernelResources[K_COUNT] = {
#include "kernel_resources.inc"
};

namespace {

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline uint32_t cdiv(int64_t a, int64_t b) { return (uint32_t)((a + b - 1) / b); }

int fail(const char *what, const opara_op_desc &op) {
  set_error("operator type %d: %s", op.op_type, what);
  return OPARA_EINVAL;
}

int plan_igemm(const opara_op_desc &op, const void *const *in, int kind, KernelPlan *out) {
  const bool persistent = kind == kPlanPersistent, group = kind == kPlanGroup;
  const opara_op_params &p = op.params;
  const bool f16 = op.dtype == OPARA_F16;
  const int ve = f16 ? 8 : 4;
  IgemmArgs a;
  std::memset(&a, 0, sizeof a);
  a.x = in[0];
  a.bias = op.bias;
  a.y = op.out;
  a.alpha = 1.0f;
  a.relu = (p.flags & OPARA_FLAG_RELU) ? 1 : 0;
  int64_t batch = 1;
  bool vec;
  if (op.op_type == OPARA_CONV2D) {
    if (op.n_inputs != 1 || !op.weight) return fail("convolution needs one input and a weight", op);
    if (p.h_in <= 0 || p.w_in <= 0 || p.c_in <= 0 || p.c_out <= 0 || p.kh <= 0 || p.kw <= 0 ||
        p.sh <= 0 || p.sw <= 0 || p.ph < 0 || p.pw < 0)
      return fail("bad convolution geometry", op);
    if (p.h_out != (p.h_in + 2 * p.ph - p.kh) / p.sh + 1 || p.w_out != (p.w_in + 2 * p.pw - p.kw) / p.sw + 1 ||
        p.h_out <= 0 || p.w_out <= 0)
      return fail("convolution output size does not match floor((in + 2*pad - k)/stride) + 1", op);
    if (p.batch < 0 || p.batch > 4096) return fail("bad image batch", op);
    const int images = p.batch > 0 ? p.batch : 1;
    a.w = op.weight;
    a.HoWo = p.h_out * p.w_out;
    a.img_stride = (int64_t)p.h_in * p.w_in * p.c_in;
    a.M = images * a.HoWo;
    a.N = p.c_out;
    a.K = p.kh * p.kw * p.c_in;
    a.gather = !(p.kh == 1 && p.kw == 1 && p.sh == 1 && p.sw == 1 && p.ph == 0 && p.pw == 0);
    a.H = p.h_in; a.W = p.w_in; a.Cin = p.c_in; a.Wo = p.w_out;
    a.kh = p.kh; a.kw = p.kw; a.sh = p.sh; a.sw = p.sw; a.ph = p.ph; a.pw = p.pw;
    if (p.c_row_stride != 0 && p.c_row_stride < p.c_out) return fail("output pixel stride below c_out", op);
    a.lda = p.c_in; a.ldb = a.K; a.ldy = p.c_row_stride ? p.c_row_stride : p.c_out;
    vec = (p.c_in % ve == 0);
  } else if (op.op_type == OPARA_GEMM) {
    if (!op.weight || op.n_inputs > 4) return fail("GEMM needs a weight and at most 3 extra inputs", op);
    if (p.m <= 0 || p.n <= 0 || p.k <= 0) return fail("bad GEMM shape", op);
    a.w = op.weight;
    a.M = p.m; a.N = p.n; a.K = p.k;
    if (p.c_row_stride != 0 && p.c_row_stride < p.n) return fail("output row stride below n", op);
    a.lda = p.k; a.ldb = p.k; a.ldy = p.c_row_stride ? p.c_row_stride : p.n;
    a.HoWo = p.m; a.Wo = 1;
    a.n_extra = op.n_inputs - 1;
    for (int i = 0; i < a.n_extra; ++i) a.extra[i] = in[i + 1];
    vec = (p.k % ve == 0);
  } else {  // BGEMM
    if (op.n_inputs != 2) return fail("batched GEMM needs two inputs", op);
    if (p.m <= 0 || p.n <= 0 || p.k <= 0 || p.batch <= 0 || p.batch > 65535) return fail("bad batched GEMM shape", op);
    if (p.a_row_stride < p.k || p.c_row_stride < p.n || p.a_batch_stride < 0 || p.b_batch_stride < 0 ||
        p.c_batch_stride < 0)
      return fail("bad batched GEMM strides", op);
    a.w = in[1];
    a.M = p.m; a.N = p.n; a.K = p.k;
    a.lda = p.a_row_stride; a.ldb = p.b_row_stride; a.ldy = p.c_row_stride;
    a.HoWo = p.m; a.Wo = 1;
    a.a_bs = p.a_batch_stride; a.b_bs = p.b_batch_stride; a.y_bs = p.c_batch_stride;
    a.b_kmajor = (p.flags & OPARA_FLAG_B_KMAJOR) ? 1 : 0;
    if (a.b_kmajor ? p.b_row_stride < p.n : p.b_row_stride < p.k) return fail("bad batched GEMM strides", op);
    a.alpha = p.alpha;
    batch = p.batch;
    vec = (p.k % ve == 0) && (a.lda % ve == 0) && (a.ldb % ve == 0) && (a.a_bs % ve == 0) && (a.b_bs % ve == 0) &&
          (!a.b_kmajor || p.n % ve == 0);
  }
  vec = vec && aligned16(a.x) && aligned16(a.w);
  int kernel;
  IgemmTile t = kTile64;
  if (vec && op.op_type == OPARA_GEMM && a.M <= kGemvMaxM) {
    kernel = f16 ? K_gemv_f16 : K_gemv_f32;
    out->kernel = kernel;
    out->gx = cdiv(a.N, 4);            // one wave per output column, four waves per workgroup
    out->gy = out->gz = 1;
    out->block = 256;
    out->args.igemm = a;
    return OPARA_OK;
  }
  if (!vec) {
    kernel = f16 ? K_igemm_f16_t64x64_scalar : K_igemm_f32_t64x64_scalar;
  } else {
    const int64_t n128 = (int64_t)cdiv(a.M, 128) * cdiv(a.N, 128) * batch;
    const double flops = 2.0 * a.M * a.N * a.K * (double)batch;
    const int64_t tiles = (int64_t)cdiv(a.M, kTile128x64.bm) * cdiv(a.N, kTile128x64.bn) * batch;
    (void)n128;
    const int64_t lim32 = (int64_t)1 << 31;
    const bool fits32 = (int64_t)a.M * a.lda < lim32 && (int64_t)a.N * a.ldb < lim32 &&
                        (!a.gather || (int64_t)(a.M / a.HoWo) * a.img_stride < lim32);
    const bool quad64 = !persistent && !a.b_kmajor && !a.gather && fits32 && flops < kQuad64MaxFlops &&
                        (int64_t)cdiv(a.M, 64) * cdiv(a.N, 64) * batch >= kQuad64MinTiles &&
                        (int64_t)a.K * (f16 ? 2 : 4) >= kQuadMinRowBytes;
    if (quad64) {
      // GEMM-shaped and at least one 64 x 64 tile per compute unit: the quad-coalesced
      // kernel whose wavefronts each multiply a whole tile over their share of K.
      // Four wavefronts whatever K is: two such workgroups share a CU (70 KB of LDS each),
      // which beat one eight-wavefront workgroup on every shape measured and leaves room
      // for workgroups of co-running operators.
      const int waves = 4;
      out->kernel = f16 ? K_igemm_f16_quad64x4 : K_igemm_f32_quad64x4;
      out->gx = cdiv(a.M, 64);
      out->gy = cdiv(a.N, 64);
      out->gz = (uint32_t)batch;
      out->block = waves * 64;
      out->args.igemm = a;
      return OPARA_OK;
    }
    if (!a.b_kmajor && tiles >= kTiledMinTiles && flops >= (persistent ? kTiledMinFlopsPersistent : kTiledMinFlops)) {
      // Throughput-oriented tiled kernel (128 output columns x 64 rows per workgroup):
      // pays once the contraction is heavy and has enough tiles to occupy the device.
      t = kTile128x64;
      kernel = f16 ? K_igemm_f16_t128x64 : K_igemm_f32_t128x64;
    } else if (a.b_kmajor) {           // [K][N] operand: staged (and transposed) through LDS
      t = kTile64;
      kernel = f16 ? K_igemm_f16_t64x64 : K_igemm_f32_t64x64;
    } else if (!fits32) {              // the latency-oriented kernel keeps 32-bit element offsets
      t = kTile64;
      kernel = f16 ? K_igemm_f16_t64x64 : K_igemm_f32_t64x64;
    } else {
      // Latency-oriented kernels, one 32 x 32 tile per workgroup, K split between its
      // wavefronts.  Deep contractions take the variant whose loads are coalesced in lane
      // groups of four (three times the load rate, paid for with a register transposition
      // per 256-byte step); shallow ones, where a wavefront walks a step or two, the
      // variant that loads MFMA fragments as they are.
      static const int ids[2][4] = {{K_igemm_f32_direct4, K_igemm_f32_direct8, K_igemm_f32_quad4, K_igemm_f32_quad8},
                                    {K_igemm_f16_direct4, K_igemm_f16_direct8, K_igemm_f16_quad4, K_igemm_f16_quad8}};
      // Convolutions with a tile or more for every other compute unit and rows of K up to 2 KiB
      // keep the fragment-loading kernel: with that many workgroups its four resident
      // workgroups per CU (105 registers against 211) hide more latency than the faster
      // loads of the quad-coalesced one save (GoogLeNet-like stem 3x3: 10.6 -> 9.2 us).  GEMMs
      // of that shape are better off with the quad-coalesced kernel (BERT-like FFN: measured).
      const int64_t row_bytes = (int64_t)a.K * (f16 ? 2 : 4);
      const int64_t tiles32q = (int64_t)cdiv(a.M, kDirectTile) * cdiv(a.N, kDirectTile) * batch;
      const bool quad = !persistent && row_bytes >= kQuadMinRowBytes &&
                        !(a.gather && tiles32q >= kQuadFourWaveTiles && row_bytes <= 2 * kQuadMinRowBytes);
      int waves;
      // Deep K on few tiles: eight wavefronts share it (latency).  With a tile or more per
      // compute unit, four: more workgroups per CU overlap better than longer ones.
      const int64_t tiles32 = (int64_t)cdiv(a.M, kDirectTile) * cdiv(a.N, kDirectTile) * batch;
      if (group) waves = 4;                                    // one workgroup size inside a group kernel
      else if (quad) waves = (cdiv(a.K, 16 * ve) <= 8 || tiles32 >= (int64_t)kQuadFourWaveTiles) ? 4 : 8;   // 256-byte steps
      else waves = cdiv(a.K, 8 * ve) <= 16 ? 4 : 8;            // 128-byte steps
      // Few tiles (the 14 x 14 and 7 x 7 stages of the CNNs): the load rate of ONE compute unit
      // bounds a workgroup, so 16 x 16 tiles on four times as many compute units finish sooner
      // although they move twice the operand bytes in total.
      static const int small_ids[2][2] = {{K_igemm_f32_direct4s, K_igemm_f32_quad4s}, {K_igemm_f16_direct4s, K_igemm_f16_quad4s}};
      if (!persistent && tiles32 <= kSmallTileMaxTiles32) {
        out->kernel = small_ids[f16][quad ? 1 : 0];
        out->gx = cdiv(a.M, kSmallTile);
        out->gy = cdiv(a.N, kSmallTile);
        out->gz = (uint32_t)batch;
        out->block = 256;
        out->args.igemm = a;
        return OPARA_OK;
      }
      out->kernel = ids[f16][(quad ? 2 : 0) + (waves == 8 ? 1 : 0)];
      out->gx = cdiv(a.M, kDirectTile);
      out->gy = cdiv(a.N, kDirectTile);
      out->gz = (uint32_t)batch;
      out->block = waves * 64;
      out->args.igemm = a;
      return OPARA_OK;
    }
  }
  out->kernel = kernel;
  out->gx = cdiv(a.M, t.bm);
  out->gy = cdiv(a.N, t.bn);
  out->gz = (uint32_t)batch;
  out->block = t.threads;
  out->args.igemm = a;
  return OPARA_OK;
}

int plan_pool(const opara_op_desc &op, const void *const *in, KernelPlan *out) {
  const opara_op_params &p = op.params;
  const bool f16 = op.dtype == OPARA_F16;
  const int ve = f16 ? 8 : 4;
  if (op.n_inputs != 1) return fail("pooling takes one input", op);
  if (p.h_in <= 0 || p.w_in <= 0 || p.c_in <= 0 || p.kh <= 0 || p.kw <= 0 || p.sh <= 0 || p.sw <= 0 ||
      p.ph < 0 || p.pw < 0 || p.ph >= p.kh || p.pw >= p.kw)
    return fail("bad pooling geometry", op);
  if (p.h_out != (p.h_in + 2 * p.ph - p.kh) / p.sh + 1 || p.w_out != (p.w_in + 2 * p.pw - p.kw) / p.sw + 1 ||
      p.h_out <= 0 || p.w_out <= 0)
    return fail("pooling output size does not match floor((in + 2*pad - k)/stride) + 1", op);
  PoolArgs a;
  std::memset(&a, 0, sizeof a);
  a.x = in[0]; a.y = op.out;
  a.H = p.h_in; a.W = p.w_in; a.C = p.c_in; a.Ho = p.h_out; a.Wo = p.w_out;
  a.kh = p.kh; a.kw = p.kw; a.sh = p.sh; a.sw = p.sw; a.ph = p.ph; a.pw = p.pw;
  a.is_avg = op.op_type == OPARA_AVGPOOL;
  if (p.batch < 0 || p.batch > 4096) return fail("bad image batch", op);
  a.B = p.batch > 0 ? p.batch : 1;
  const bool vec = (p.c_in % ve == 0) && aligned16(a.x) && aligned16(a.y);
  out->kernel = f16 ? (vec ? K_pool_f16_vec : K_pool_f16_scalar) : (vec ? K_pool_f32_vec : K_pool_f32_scalar);
  const int64_t items = (int64_t)a.B * p.h_out * p.w_out * (vec ? p.c_in / ve : p.c_in);
  out->gx = cdiv(items, 256); out->gy = out->gz = 1; out->block = 256;
  out->args.pool = a;
  return OPARA_OK;
}

int plan_gap(const opara_op_desc &op, const void *const *in, KernelPlan *out) {
  const opara_op_params &p = op.params;
  if (op.n_inputs != 1 || p.h_in <= 0 || p.w_in <= 0 || p.c_in <= 0) return fail("bad global pooling shape", op);
  GapArgs a;
  std::memset(&a, 0, sizeof a);
  a.x = in[0]; a.y = op.out; a.HW = p.h_in * p.w_in; a.C = p.c_in;
  out->kernel = op.dtype == OPARA_F16 ? K_gap_f16 : K_gap_f32;
  if (p.batch < 0 || p.batch > 4096) return fail("bad image batch", op);
  out->gx = cdiv(p.c_in, 64); out->gy = p.batch > 0 ? p.batch : 1; out->gz = 1; out->block = 256;
  out->args.gap = a;
  return OPARA_OK;
}

int plan_row(const opara_op_desc &op, const void *const *in, KernelPlan *out) {
  const opara_op_params &p = op.params;
  const bool f16 = op.dtype == OPARA_F16;
  const int ve = f16 ? 8 : 4;
  if (p.m <= 0 || p.n <= 0) return fail("bad row-wise shape", op);
  RowArgs a;
  std::memset(&a, 0, sizeof a);
  a.y = op.out; a.n_in = op.n_inputs; a.rows = p.m; a.cols = p.n; a.eps = p.eps;
  bool vec = (p.n % ve == 0) && aligned16(a.y);
  for (int i = 0; i < op.n_inputs; ++i) { a.in[i] = in[i]; vec = vec && aligned16(in[i]); }
  const bool ln = op.op_type == OPARA_LAYERNORM;
  int variant;  // 0 wave, 1 block, 2 generic
  if (vec && p.n <= kRowGroupWave * ve * 2) variant = 0;
  else if (vec && p.n <= kRowGroupBlock * ve * kRowCacheChunks) variant = 1;
  else variant = 2;
  static const int ids[2][2][3] = {
      {{K_softmax_f32_wave, K_softmax_f32_block, K_softmax_f32_generic},
       {K_softmax_f16_wave, K_softmax_f16_block, K_softmax_f16_generic}},
      {{K_layernorm_f32_wave, K_layernorm_f32_block, K_layernorm_f32_generic},
       {K_layernorm_f16_wave, K_layernorm_f16_block, K_layernorm_f16_generic}}};
  out->kernel = ids[ln][f16][variant];
  out->block = 256;
  out->gx = variant == 0 ? cdiv(p.m, 256 / kRowGroupWave) : (uint32_t)p.m;
  out->gy = out->gz = 1;
  out->args.row = a;
  return OPARA_OK;
}

int plan_elt(const opara_op_desc &op, const void *const *in, KernelPlan *out) {
  const opara_op_params &p = op.params;
  const bool f16 = op.dtype == OPARA_F16;
  const int ve = f16 ? 8 : 4;
  if (p.m <= 0 || p.n <= 0) return fail("bad element-wise shape", op);
  EltArgs a;
  std::memset(&a, 0, sizeof a);
  a.y = op.out; a.n_in = op.n_inputs; a.n = (int64_t)p.m * p.n;
  a.op = op.op_type == OPARA_ADD ? 0 : op.op_type == OPARA_RELU ? 1 : 2;
  bool vec = (a.n % ve == 0) && aligned16(a.y);
  for (int i = 0; i < op.n_inputs; ++i) { a.in[i] = in[i]; vec = vec && aligned16(in[i]); }
  out->kernel = f16 ? (vec ? K_elt_f16_vec : K_elt_f16_scalar) : (vec ? K_elt_f32_vec : K_elt_f32_scalar);
  out->gx = cdiv(vec ? a.n / ve : a.n, 256); out->gy = out->gz = 1; out->block = 256;
  out->args.elt = a;
  return OPARA_OK;
}

int plan_concat(const opara_op_desc &op, const void *const *in, KernelPlan *out) {
  const opara_op_params &p = op.params;
  const bool f16 = op.dtype == OPARA_F16;
  const int ve = f16 ? 8 : 4;
  if (p.m <= 0) return fail("bad concat shape", op);
  ConcatArgs a;
  std::memset(&a, 0, sizeof a);
  a.y = op.out; a.n_in = op.n_inputs; a.rows = p.m;
  bool vec = aligned16(a.y);
  int32_t off = 0, widest = 0;
  for (int i = 0; i < op.n_inputs; ++i) {
    if (p.in_cols[i] <= 0) return fail("concat input with no columns", op);
    a.in[i] = in[i]; a.cols[i] = p.in_cols[i]; a.col_off[i] = off;
    off += p.in_cols[i];
    if (p.in_cols[i] > widest) widest = p.in_cols[i];
    vec = vec && (p.in_cols[i] % ve == 0) && aligned16(in[i]);
  }
  if (p.n != off) return fail("concat: n must equal the sum of in_cols", op);
  a.out_cols = off;
  out->kernel = f16 ? (vec ? K_concat_f16_vec : K_concat_f16_scalar) : (vec ? K_concat_f32_vec : K_concat_f32_scalar);
  out->gx = cdiv((int64_t)p.m * (vec ? widest / ve : widest), 256);
  out->gy = (uint32_t)op.n_inputs; out->gz = 1; out->block = 256;
  out->args.concat = a;
  return OPARA_OK;
}

}  // namespace

int plan_op(const opara_op_desc &op, const void *const *in, int kind, KernelPlan *out) {
  std::memset(out, 0, sizeof *out);
  int rc;
  switch (op.op_type) {
    case OPARA_CONV2D: case OPARA_GEMM: case OPARA_BGEMM: rc = plan_igemm(op, in, kind, out); break;
    case OPARA_MAXPOOL: case OPARA_AVGPOOL: rc = plan_pool(op, in, out); break;
    case OPARA_GAVGPOOL: rc = plan_gap(op, in, out); break;
    case OPARA_LAYERNORM: case OPARA_SOFTMAX: rc = plan_row(op, in, out); break;
    case OPARA_GELU: case OPARA_RELU: case OPARA_ADD: rc = plan_elt(op, in, out); break;
    case OPARA_CONCAT: rc = plan_concat(op, in, out); break;
    default: set_error("unknown operator type %d", op.op_type); return OPARA_EINVAL;
  }
  if (rc != OPARA_OK) return rc;
  if (out->gx == 0 || out->gy == 0 || out->gz == 0 || out->gy > 65535u || out->gz > 65535u) {
    set_error("operator type %d: launch grid out of range", op.op_type);
    return OPARA_EUNSUPPORTED;
  }
  return OPARA_OK;
}

}  // namespace opara
