// Which tensors to make virtual: the virtual tensor opportunity graph (Sec. 5.1, Def. 6, Alg. 1)
// and the global greedy construction of a points-to graph (Sec. 5.2, Alg. 2).  Host logic.
//
// A computation graph is a list of statements over tensor numbers.  Data-movement statements
// create *bundles*: "tensor a can be made a virtual tensor of the tensors `targets` by eliminating
// exactly this one operator", in one of two directions:
//   read   a is an output of the operator and its elements are found in the operator's inputs
//          (the consumer of a reads through the map);
//   store  a is an input of the operator and lives inside the operator's output (the producer of
//          a writes through the map): inputs of Concat, the input of a Reshape, Permute or
//          Unsqueeze, the input of a Split (stitched from its outputs), the updates of a ScatterND.
// All edges of a bundle are taken together (the output of a Concat is a virtual tensor of all of
// its inputs at once).  The bundles of one tensor exclude each other: a tensor mapped into two
// places would break the one-to-one property (Sec. 4.1); that is the conflict set of Alg. 1.
#include <algorithm>
#include <string>
#include <vector>

#include "vt.h"
#include "vt_desc.h"

struct vt_vtog {
  struct Bundle {
    int tensor;
    std::vector<int> targets;
    int stmt;
    int direction;   // VT_DIR_READ or VT_DIR_STORE
  };
  int n_tensors = 0;
  std::vector<Bundle> bundles;                  // in statement order
  std::vector<std::vector<int>> by_tensor;      // tensor -> its bundles (pick at most one)
};

namespace {

using vt::fail;

bool is_bijective(int kind) { return kind == VT_OP_RESHAPE || kind == VT_OP_PERMUTE || kind == VT_OP_UNSQUEEZE; }

// Rules per operator (Sec. 4.4), both directions.
void rules(const vt_graph_stmt& st, int index, std::vector<vt_vtog::Bundle>* out) {
  const int k = st.kind;
  if (k < VT_OP_RESHAPE || k > VT_OP_SCATTER_ND) return;      // a compute operator: no opportunity
  if (k == VT_OP_SCATTER_ND) {
    // inputs: data, indices, updates.  The output starts as a clone of `data`: the output as a
    // virtual tensor of data, and the updates as a virtual tensor of the output
    out->push_back({st.out[0], {st.in[0]}, index, VT_DIR_READ});
    out->push_back({st.in[2], {st.out[0]}, index, VT_DIR_STORE});
    return;
  }
  if (k == VT_OP_SPLIT) {
    for (int i = 0; i < st.n_out; ++i) out->push_back({st.out[i], {st.in[0]}, index, VT_DIR_READ});
    out->push_back({st.in[0], std::vector<int>(st.out, st.out + st.n_out), index, VT_DIR_STORE});   // the input stitched from its outputs
    return;
  }
  if (k == VT_OP_CONCAT) {
    out->push_back({st.out[0], std::vector<int>(st.in, st.in + st.n_in), index, VT_DIR_READ});
    for (int i = 0; i < st.n_in; ++i) out->push_back({st.in[i], {st.out[0]}, index, VT_DIR_STORE});
    return;
  }
  out->push_back({st.out[0], {st.in[0]}, index, VT_DIR_READ});
  if (is_bijective(k)) out->push_back({st.in[0], {st.out[0]}, index, VT_DIR_STORE});
}

// Following the chosen bundles from every tensor must end at physical tensors: no cycle.
bool grounded(const vt_vtog& g, const int* bundle_of, int t, std::vector<char>& state) {
  if (bundle_of[t] < 0) return true;
  if (state[t] == 1) return false;
  if (state[t] == 2) return true;
  state[t] = 1;
  bool ok = true;
  for (int x : g.bundles[bundle_of[t]].targets) ok = ok && grounded(g, bundle_of, x, state);
  state[t] = 2;
  return ok;
}

}  // namespace

extern "C" {

int vt_vtog_build(const vt_graph_stmt* stmts, int n_stmts, int n_tensors, const uint8_t* pinned, int directions, vt_vtog** out) {
  if (!out || n_stmts < 0 || n_tensors < 1 || (n_stmts > 0 && !stmts) || !pinned) return fail(VT_ERR_INVALID_ARG, "vt_vtog_build: NULL argument or empty graph");
  if (!(directions & (VT_DIR_READ | VT_DIR_STORE))) return fail(VT_ERR_INVALID_ARG, "vt_vtog_build: no direction selected");
  vt_vtog* g = new vt_vtog;
  g->n_tensors = n_tensors;
  g->by_tensor.assign(n_tensors, {});
  for (int k = 0; k < n_stmts; ++k) {
    const vt_graph_stmt& st = stmts[k];
    bool ok = st.n_in >= 0 && st.n_in <= VT_MAX_OP_INPUTS && st.n_out >= 1 && st.n_out <= VT_MAX_OP_INPUTS;
    for (int i = 0; ok && i < st.n_in; ++i) ok = st.in[i] >= 0 && st.in[i] < n_tensors;
    for (int i = 0; ok && i < st.n_out; ++i) ok = st.out[i] >= 0 && st.out[i] < n_tensors;
    if (ok && st.kind >= VT_OP_RESHAPE && st.kind <= VT_OP_SCATTER_ND) ok = st.n_in >= (st.kind == VT_OP_SCATTER_ND ? 3 : 1);
    if (!ok) {
      delete g;
      return fail(VT_ERR_INVALID_ARG, "vt_vtog_build: statement " + std::to_string(k) + " names a tensor outside the graph or has no inputs");
    }
    std::vector<vt_vtog::Bundle> found;
    rules(st, k, &found);
    for (const vt_vtog::Bundle& b : found) {
      // tensors that are inputs or outputs of the graph stay physical: no edge leaves them (Alg. 1)
      if (!(b.direction & directions) || pinned[b.tensor]) continue;
      g->by_tensor[b.tensor].push_back((int)g->bundles.size());
      g->bundles.push_back(b);
    }
  }
  *out = g;
  return VT_OK;
}

int vt_vtog_free(vt_vtog* g) {
  delete g;
  return VT_OK;
}

int vt_vtog_size(const vt_vtog* g, int* n_tensors, int* n_bundles) {
  if (!g) return fail(VT_ERR_INVALID_ARG, "vt_vtog_size: NULL graph");
  if (n_tensors) *n_tensors = g->n_tensors;
  if (n_bundles) *n_bundles = (int)g->bundles.size();
  return VT_OK;
}

int vt_vtog_bundle(const vt_vtog* g, int b, int* tensor, int* n_targets, int* targets, int* stmt, int* direction) {
  if (!g || b < 0 || b >= (int)g->bundles.size()) return fail(VT_ERR_INVALID_ARG, "vt_vtog_bundle: no such bundle");
  const vt_vtog::Bundle& x = g->bundles[b];
  if (tensor) *tensor = x.tensor;
  if (n_targets) *n_targets = (int)x.targets.size();
  if (targets) std::copy(x.targets.begin(), x.targets.end(), targets);
  if (stmt) *stmt = x.stmt;
  if (direction) *direction = x.direction;
  return VT_OK;
}

int vt_vtog_is_points_to_graph(const vt_vtog* g, const int* bundle_of_tensor, int* ok) {
  if (!g || !bundle_of_tensor || !ok) return fail(VT_ERR_INVALID_ARG, "vt_vtog_is_points_to_graph: NULL argument");
  *ok = 0;
  for (int t = 0; t < g->n_tensors; ++t) {
    const int b = bundle_of_tensor[t];
    if (b < 0) continue;
    if (b >= (int)g->bundles.size() || g->bundles[b].tensor != t) return VT_OK;      // not one of the tensor's own bundles
  }
  std::vector<char> state(g->n_tensors, 0);
  for (int t = 0; t < g->n_tensors; ++t)
    if (!grounded(*g, bundle_of_tensor, t, state)) return VT_OK;
  *ok = 1;
  return VT_OK;
}

// Alg. 2.  Readings where the listing leaves room: MaxEdges(v, S(v), A) ranges over the empty set
// (v joins the anchor set as a physical tensor, saving 0) and the bundles of v whose targets all
// lie in the anchor set A (the bundles of one tensor exclude each other, so a non-empty
// conflict-free edge set is a single bundle); a bundle with a negative saving therefore loses to
// the empty set and is never taken.  Among equal savings a tensor one of whose bundles is ready
// goes first (all it could gain has been weighed: it stays physical, and the tensors behind it
// get their turn); otherwise the tensors are scanned from the graph's outputs towards its inputs
// and the first one found is taken: when no bundle is ready anywhere, the tensor nearest the
// outputs is anchored as physical, so that the tensors stored into it find it anchored (with this
// order the C3K2 block of Sec. 7 comes out as the paper reports it: a, b, c, e inside Y).  After
// a tensor joins with a bundle, the bundles that point to it are profiled again against the grown
// strategy.  The listing's exit on a negative maximum cannot fire under this reading (the empty
// set always offers 0); it is kept.
int vt_vtog_greedy(const vt_vtog* g, vt_saving_fn saving, void* user, int* bundle_of_tensor, double* total, int* order, int* n_order) {
  if (!g || !saving || !bundle_of_tensor) return fail(VT_ERR_INVALID_ARG, "vt_vtog_greedy: NULL argument");
  const int nt = g->n_tensors, nb = (int)g->bundles.size();
  std::vector<char> anchor(nt, 0);
  int n_anchor = 0;
  for (int t = 0; t < nt; ++t) {
    bundle_of_tensor[t] = -1;
    if (g->by_tensor[t].empty()) {
      anchor[t] = 1;
      ++n_anchor;
    }
  }
  std::vector<double> w(nb);
  for (int b = 0; b < nb; ++b) w[b] = saving(user, b, bundle_of_tensor);
  double sum = 0.0;
  int steps = 0;
  while (n_anchor < nt) {
    int v_c = -1, p_c = -1;
    double max_saving = 0.0;
    bool decided_c = false;
    for (int t = nt - 1; t >= 0; --t) {
      if (anchor[t]) continue;
      int p = -1;
      double s = 0.0;                              // the empty edge set
      bool decided = false;                        // some bundle of t is ready: its options have been weighed
      for (int b : g->by_tensor[t]) {
        bool ready = true;
        for (int x : g->bundles[b].targets) ready = ready && anchor[x];
        decided = decided || ready;
        if (ready && w[b] >= 0 && (p < 0 || w[b] > s)) {
          p = b;
          s = w[b];
        }
      }
      if (v_c < 0 || s > max_saving || (s == max_saving && decided && !decided_c)) {
        v_c = t;
        p_c = p;
        max_saving = s;
        decided_c = decided;
      }
    }
    if (v_c < 0 || max_saving < 0) break;
    anchor[v_c] = 1;
    ++n_anchor;
    if (p_c < 0) continue;                         // physical: the strategy did not change, nothing to profile again
    bundle_of_tensor[v_c] = p_c;
    sum += max_saving;
    if (order) order[steps] = p_c;
    ++steps;
    for (int b = 0; b < nb; ++b) {
      const vt_vtog::Bundle& x = g->bundles[b];
      if (!anchor[x.tensor] && std::find(x.targets.begin(), x.targets.end(), v_c) != x.targets.end()) w[b] = saving(user, b, bundle_of_tensor);
    }
  }
  if (total) *total = sum;
  if (n_order) *n_order = steps;
  return VT_OK;
}

}  // extern "C"
