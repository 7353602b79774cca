// Graph rewrites applied to an operator list before the DAG is built (host only, no HIP
// calls).  Zero-copy concatenation: the branches of a channel concatenation write their
// channel slices of the concatenated tensor themselves, and the concatenation operator
// (one more launch and one more synchronisation per block in the paper's cost model,
// Sec. 3.1 Eq. 3) disappears from the DAG.
#include <cstring>
#include <vector>
#include "opara_internal.h"

using namespace opara;

namespace {

int64_t conv_rows(const opara_op_params &p) {
  return (int64_t)(p.batch > 0 ? p.batch : 1) * p.h_out * p.w_out;
}

}  // namespace

extern "C" int opara_elide_concats(const opara_op_desc *ops, int32_t n_ops, void *const *ext_inputs, int32_t n_ext,
                                   opara_op_desc *out_ops, int32_t *n_out, int32_t *new_id, void **ext_out,
                                   int32_t *n_ext_out) {
  if (!ops || !out_ops || !n_out || !new_id || !ext_out || !n_ext_out || n_ops <= 0 || n_ext < 0 ||
      (n_ext > 0 && !ext_inputs)) {
    set_error("opara_elide_concats: null pointer or non-positive operator count");
    return OPARA_EINVAL;
  }
  try {
    // ---- validate what the rewrite itself relies on; opara_build_dag validates the rest
    for (int32_t v = 0; v < n_ops; ++v) {
      const opara_op_desc &op = ops[v];
      if (op.n_inputs < 1 || op.n_inputs > OPARA_MAX_INPUTS || op.n_deps < 0 || op.n_deps > OPARA_MAX_INPUTS) {
        set_error("opara_elide_concats: operator %d: bad n_inputs / n_deps", v);
        return OPARA_EINVAL;
      }
      for (int i = 0; i < op.n_inputs + op.n_deps; ++i) {
        const int32_t u = i < op.n_inputs ? op.inputs[i] : op.deps[i - op.n_inputs];
        if (u >= n_ops || (u < 0 && (i >= op.n_inputs || -(int64_t)u - 1 >= n_ext))) {
          set_error("opara_elide_concats: operator %d refers to %d, out of range", v, u);
          return OPARA_EINVAL;
        }
      }
    }
    // ---- uses of every operator's output (as argument or as dependency-only predecessor)
    std::vector<int32_t> uses(n_ops, 0);
    for (int32_t v = 0; v < n_ops; ++v)
      for (int i = 0; i < ops[v].n_inputs + ops[v].n_deps; ++i) {
        const int32_t u = i < ops[v].n_inputs ? ops[v].inputs[i] : ops[v].deps[i - ops[v].n_inputs];
        if (u >= 0) ++uses[u];
      }
    // ---- candidates: every input is the whole output of a distinct convolution nobody else reads
    std::vector<char> elide(n_ops, 0);
    for (int32_t c = 0; c < n_ops; ++c) {
      const opara_op_desc &cat = ops[c];
      if (cat.op_type != OPARA_CONCAT || !cat.out || cat.params.m <= 0) continue;
      bool ok = true;
      int64_t cols = 0;
      for (int i = 0; i < cat.n_inputs && ok; ++i) {
        const int32_t u = cat.inputs[i];
        if (u < 0) { ok = false; break; }
        const opara_op_desc &br = ops[u];
        ok = br.op_type == OPARA_CONV2D && br.dtype == cat.dtype && uses[u] == 1 && br.params.c_row_stride == 0 &&
             br.params.c_out == cat.params.in_cols[i] && conv_rows(br.params) == cat.params.m;
        cols += cat.params.in_cols[i];
      }
      ok = ok && cat.n_deps == 0 && cols == cat.params.n;
      elide[c] = ok;
    }
    // ---- a reader takes the branches as dependency-only predecessors; where they do not fit
    // into its record, the concatenations it reads stay (repeat until nothing changes)
    for (bool changed = true; changed;) {
      changed = false;
      for (int32_t v = 0; v < n_ops; ++v) {
        const opara_op_desc &op = ops[v];
        int extra = 0;
        for (int i = 0; i < op.n_inputs + op.n_deps; ++i) {
          const int32_t u = i < op.n_inputs ? op.inputs[i] : op.deps[i - op.n_inputs];
          if (u >= 0 && elide[u]) extra += ops[u].n_inputs;
        }
        if (extra == 0 || op.n_deps + extra <= OPARA_MAX_INPUTS) continue;
        for (int i = 0; i < op.n_inputs + op.n_deps; ++i) {
          const int32_t u = i < op.n_inputs ? op.inputs[i] : op.deps[i - op.n_inputs];
          if (u >= 0 && elide[u]) { elide[u] = 0; changed = true; }
        }
      }
    }
    // ---- numbering of the reduced list, one more external slot per elided concatenation
    std::vector<int32_t> slot_of(n_ops, -1);
    int32_t kept = 0, n_slots = n_ext;
    for (int32_t i = 0; i < n_ext; ++i) ext_out[i] = ext_inputs[i];
    for (int32_t v = 0; v < n_ops; ++v) {
      if (elide[v]) {
        new_id[v] = -1;
        slot_of[v] = n_slots;
        ext_out[n_slots++] = ops[v].out;
      } else {
        new_id[v] = kept++;
      }
    }
    // ---- where each branch writes: its channel slice of the concatenated tensor
    std::vector<const opara_op_desc *> cat_of(n_ops, nullptr);
    std::vector<int64_t> col_of(n_ops, 0);
    for (int32_t c = 0; c < n_ops; ++c) {
      if (!elide[c]) continue;
      int64_t off = 0;
      for (int i = 0; i < ops[c].n_inputs; ++i) {
        cat_of[ops[c].inputs[i]] = &ops[c];
        col_of[ops[c].inputs[i]] = off;
        off += ops[c].params.in_cols[i];
      }
    }
    for (int32_t v = 0; v < n_ops; ++v) {
      if (elide[v]) continue;
      opara_op_desc d = ops[v];
      if (cat_of[v]) {
        const size_t es = d.dtype == OPARA_F16 ? 2 : 4;
        d.out = (unsigned char *)cat_of[v]->out + (size_t)col_of[v] * es;
        d.params.c_row_stride = cat_of[v]->params.n;
      }
      int32_t nd = 0;
      int32_t deps[2 * OPARA_MAX_INPUTS];
      bool overflow = false;
      auto add_dep = [&](int32_t b) {
        for (int32_t j = 0; j < nd; ++j)
          if (deps[j] == b) return;
        if (nd < 2 * OPARA_MAX_INPUTS) deps[nd++] = b; else overflow = true;
      };
      auto add_branches = [&](int32_t cat) {
        for (int k = 0; k < ops[cat].n_inputs; ++k) add_dep(new_id[ops[cat].inputs[k]]);
      };
      for (int i = 0; i < d.n_deps; ++i) {
        const int32_t u = ops[v].deps[i];
        if (elide[u]) add_branches(u); else add_dep(new_id[u]);
      }
      for (int i = 0; i < d.n_inputs; ++i) {
        const int32_t u = ops[v].inputs[i];
        if (u < 0) continue;
        if (!elide[u]) { d.inputs[i] = new_id[u]; continue; }
        d.inputs[i] = -(slot_of[u] + 1);
        add_branches(u);
      }
      if (overflow || nd > OPARA_MAX_INPUTS) { set_error("opara_elide_concats: operator %d: dependency list overflow", v); return OPARA_EINVAL; }
      d.n_deps = nd;
      for (int32_t j = 0; j < OPARA_MAX_INPUTS; ++j) d.deps[j] = j < nd ? deps[j] : 0;
      out_ops[new_id[v]] = d;
    }
    *n_out = kept;
    *n_ext_out = n_slots;
  } catch (const std::bad_alloc &) {
    set_error("out of memory");
    return OPARA_ENOMEM;
  }
  return OPARA_OK;
}
