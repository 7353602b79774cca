/*
 * A C caller of the library: no Python, no PyTorch.  Builds a two-block Inception-style DAG
 * (1x1 | 1x1,3x3 | 1x1,3x3 | maxpool,1x1 -> channel concatenation, twice, then a global
 * average pool) with its own device buffers, and checks through the C ABI alone that
 *   - opara_elide_concats removes both concatenations,
 *   - the sequential graph of the full DAG and, on the rewritten DAG, the sequential graph,
 *     the validated multi-stream graph (opara_capture(OPARA_PARALLEL): validation in place)
 *     and the fused executor all produce bit-identical concatenated tensors and outputs,
 *   - replays are deterministic.
 * Exit status 0 and "abi_demo ok" on success.  Values are small integers in fp16, so every
 * result is exact whatever the summation order.
 */
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include "opara.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { fprintf(stderr, "%s: %s\n", #x, hipGetErrorString(e_)); exit(2); } } while (0)
#define CHECK(x) do { int rc_ = (x); if (rc_ != OPARA_OK) { fprintf(stderr, "%s -> %d: %s\n", #x, rc_, opara_last_error()); exit(3); } } while (0)

enum { H = 14, W = 14, C0 = 32 };

static uint16_t half_of_small_int(int v) {      /* exact fp16 encoding of an integer |v| <= 2048 */
  if (v == 0) return 0;
  uint16_t sign = v < 0 ? 0x8000u : 0u;
  unsigned a = (unsigned)(v < 0 ? -v : v);
  int e = 0;
  while ((a >> (e + 1)) != 0) ++e;
  unsigned mant = (a << (10 - e)) & 0x3ffu;
  return (uint16_t)(sign | ((unsigned)(e + 15) << 10) | mant);
}

static void *dev_alloc(size_t bytes) {
  void *p = NULL;
  CHECK_HIP(hipMalloc(&p, bytes));
  CHECK_HIP(hipMemset(p, 0, bytes));
  return p;
}

static uint32_t rng_state = 12345u;
static int small_rand(int lo, int hi) {         /* deterministic small integers */
  rng_state = rng_state * 1664525u + 1013904223u;
  return lo + (int)((rng_state >> 16) % (unsigned)(hi - lo + 1));
}

static void *dev_random_half(size_t n, int lo, int hi) {
  uint16_t *h = (uint16_t *)malloc(n * 2);
  for (size_t i = 0; i < n; ++i) h[i] = half_of_small_int(small_rand(lo, hi));
  void *d = dev_alloc(n * 2);
  CHECK_HIP(hipMemcpy(d, h, n * 2, hipMemcpyHostToDevice));
  free(h);
  return d;
}

typedef struct { opara_op_desc d[32]; size_t out_bytes[32]; int n; } dag_t;

static int add_conv(dag_t *g, int input, int cin, int cout, int k) {
  opara_op_desc *d = &g->d[g->n];
  memset(d, 0, sizeof *d);
  d->op_type = OPARA_CONV2D; d->op_class = OPARA_CLASS_DEFAULT; d->dtype = OPARA_F16;
  d->n_inputs = 1; d->inputs[0] = input;
  d->params.h_in = H; d->params.w_in = W; d->params.c_in = cin;
  d->params.h_out = H; d->params.w_out = W; d->params.c_out = cout;
  d->params.kh = d->params.kw = k; d->params.sh = d->params.sw = 1; d->params.ph = d->params.pw = k / 2;
  d->params.batch = 1; d->params.flags = OPARA_FLAG_RELU;
  d->weight = dev_random_half((size_t)cout * k * k * cin, -1, 1);
  d->bias = NULL;
  g->out_bytes[g->n] = (size_t)H * W * cout * 2;
  d->out = dev_alloc(g->out_bytes[g->n]);
  return g->n++;
}

static int add_pool(dag_t *g, int input, int c, int type, int global) {
  opara_op_desc *d = &g->d[g->n];
  memset(d, 0, sizeof *d);
  d->op_type = type; d->op_class = OPARA_CLASS_DEFAULT; d->dtype = OPARA_F16;
  d->n_inputs = 1; d->inputs[0] = input;
  d->params.h_in = H; d->params.w_in = W; d->params.c_in = c; d->params.batch = 1;
  if (!global) {
    d->params.h_out = H; d->params.w_out = W; d->params.c_out = c;
    d->params.kh = d->params.kw = 3; d->params.sh = d->params.sw = 1; d->params.ph = d->params.pw = 1;
  }
  g->out_bytes[g->n] = (size_t)(global ? 1 : H * W) * c * 2;
  d->out = dev_alloc(g->out_bytes[g->n]);
  return g->n++;
}

static int add_concat(dag_t *g, const int *in, const int *cols, int n_in) {
  opara_op_desc *d = &g->d[g->n];
  memset(d, 0, sizeof *d);
  d->op_type = OPARA_CONCAT; d->op_class = OPARA_CLASS_DEFAULT; d->dtype = OPARA_F16;
  d->n_inputs = n_in;
  int total = 0;
  for (int i = 0; i < n_in; ++i) { d->inputs[i] = in[i]; d->params.in_cols[i] = cols[i]; total += cols[i]; }
  d->params.m = H * W; d->params.n = total;
  g->out_bytes[g->n] = (size_t)H * W * total * 2;
  d->out = dev_alloc(g->out_bytes[g->n]);
  return g->n++;
}

static int add_block(dag_t *g, int input, int cin) {     /* returns the concatenation: 16 + 24 + 8 + 16 = 64 channels */
  int b1 = add_conv(g, input, cin, 16, 1);
  int b2 = add_conv(g, add_conv(g, input, cin, 8, 1), 8, 24, 3);
  int b3 = add_conv(g, add_conv(g, input, cin, 8, 1), 8, 8, 3);
  int b4 = add_conv(g, add_pool(g, input, cin, OPARA_MAXPOOL, 0), cin, 16, 1);
  int in[4] = {b1, b2, b3, b4}, cols[4] = {16, 24, 8, 16};
  return add_concat(g, in, cols, 4);
}

static void snapshot(const dag_t *g, const int *watch, int n_watch, uint16_t **out) {
  for (int i = 0; i < n_watch; ++i) {
    out[i] = (uint16_t *)malloc(g->out_bytes[watch[i]]);
    CHECK_HIP(hipMemcpy(out[i], g->d[watch[i]].out, g->out_bytes[watch[i]], hipMemcpyDeviceToHost));
  }
}

static void poison(const dag_t *g) {
  for (int v = 0; v < g->n; ++v) CHECK_HIP(hipMemset(g->d[v].out, 0x7e, g->out_bytes[v]));    /* fp16 NaN pattern */
}

int main(void) {
  CHECK_HIP(hipSetDevice(0));
  static dag_t g;
  void *x = dev_random_half((size_t)H * W * C0, -2, 2);
  void *ext[1] = {x};
  int cat1 = add_block(&g, -1, C0);
  int cat2 = add_block(&g, cat1, 64);
  int gap = add_pool(&g, cat2, 64, OPARA_GAVGPOOL, 1);
  const int watch[3] = {cat1, cat2, gap};
  uint16_t *want[3], *got[3];

  hipStream_t streams[16];
  for (int i = 0; i < 16; ++i) CHECK_HIP(hipStreamCreateWithFlags(&streams[i], hipStreamNonBlocking));

  /* the full DAG, sequential graph: the reference bits */
  opara_dag *full = NULL;
  opara_exec *seq = NULL;
  CHECK(opara_build_dag(g.d, g.n, ext, 1, NULL, &full));
  CHECK(opara_capture(full, (void *const *)streams, 1, OPARA_SEQUENTIAL, &seq));
  poison(&g);
  CHECK(opara_replay(seq, streams[0]));
  CHECK_HIP(hipStreamSynchronize(streams[0]));
  snapshot(&g, watch, 3, want);
  int nonzero = 0;
  for (size_t i = 0; i < g.out_bytes[gap] / 2; ++i) nonzero += (want[2][i] & 0x7fffu) != 0;
  if (nonzero < 8) { fprintf(stderr, "reference output is degenerate\n"); return 4; }

  /* the rewrite: both concatenations go */
  static opara_op_desc reduced[32];
  int32_t new_id[32], n_red = 0, n_ext = 0;
  void *ext_red[1 + 32];
  CHECK(opara_elide_concats(g.d, g.n, ext, 1, reduced, &n_red, new_id, ext_red, &n_ext));
  if (n_red != g.n - 2 || n_ext != 3 || new_id[cat1] != -1 || new_id[cat2] != -1) {
    fprintf(stderr, "unexpected rewrite: %d operators, %d external slots\n", n_red, n_ext);
    return 5;
  }
  opara_dag *dag = NULL;
  CHECK(opara_build_dag(reduced, n_red, ext_red, n_ext, NULL, &dag));
  int32_t stream_of[32], order[32], n_streams = 0;
  CHECK(opara_assign_streams(dag, stream_of, &n_streams));
  CHECK(opara_order_launch(dag, order));
  if (n_streams < 4 || n_streams > 16) { fprintf(stderr, "unexpected stream count %d\n", n_streams); return 6; }

  const int modes[3] = {OPARA_SEQUENTIAL, OPARA_PARALLEL, OPARA_FUSED};
  const char *names[3] = {"sequential graph", "multi-stream graph", "fused executor"};
  for (int m = 0; m < 3; ++m) {
    opara_exec *e = NULL;
    CHECK(opara_capture(dag, (void *const *)streams, n_streams, modes[m], &e));
    int32_t kind = -1, attempts = -1, nodes = 0, edges = 0;
    CHECK(opara_exec_validation(e, &kind, &attempts));
    CHECK(opara_exec_info(e, &nodes, &edges));
    if (modes[m] == OPARA_PARALLEL && kind == OPARA_NOT_VALIDATED) { fprintf(stderr, "multi-stream graph was not validated\n"); return 7; }
    for (int rep = 0; rep < 2; ++rep) {
      poison(&g);
      CHECK(opara_replay(e, streams[0]));
      CHECK_HIP(hipStreamSynchronize(streams[0]));
      snapshot(&g, watch, 3, got);
      for (int i = 0; i < 3; ++i) {
        if (memcmp(got[i], want[i], g.out_bytes[watch[i]]) != 0) {
          fprintf(stderr, "%s, replay %d: tensor %d differs from the full DAG's sequential graph\n", names[m], rep, i);
          return 8;
        }
        free(got[i]);
      }
    }
    printf("%s: %d nodes, %d edges, validation %d (%d instance(s)): bit-identical\n", names[m], nodes, edges, kind, attempts);
    opara_exec_destroy(e);
  }
  opara_exec_destroy(seq);
  opara_dag_destroy(dag);
  opara_dag_destroy(full);
  printf("abi_demo ok\n");
  return 0;
}
