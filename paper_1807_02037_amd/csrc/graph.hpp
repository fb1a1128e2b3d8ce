// Internal graph representation behind the C ABI: G = (V, E, lambda, tau) of Definition 1.
// Read edges are kept as each node's ordered input list, control edges as its control-input
// list, update edges as (from, variable) pairs.
#pragma once
#include <cstdint>
#include <string>
#include <utility>
#include <vector>

#include "lms.h"

namespace lms {

struct Node {
  int id = 0;
  std::string name;
  int op = LMS_OP_VARIABLE;
  lms_attr attr{};
  int phase = LMS_FWD;
  int placement = LMS_DEVICE;
  bool is_var = false;
  int var_kind = LMS_VAR_PARAM;
  int dtype = LMS_BF16;
  int ndim = 0;
  int64_t dims[5] = {1, 1, 1, 1, 1};
  int label = -1;             // order assigned by the rewriter to an inserted vertex (Figure 3)
  int clone_of = -1;          // inserted copy of an operation (recomputation): the vertex it repeats
  bool external = false;      // the output will be bound to caller memory: no arena block is planned for it
  std::vector<int> in;        // read edges, slot order
  std::vector<int> ctrl_in;   // control edges

  int64_t numel() const {
    int64_t n = 1;
    for (int i = 0; i < ndim; ++i) n *= dims[i];
    return n;
  }
  uint64_t bytes() const { return (uint64_t)numel() * (dtype == LMS_BF16 ? 2u : 4u); }
  int nsp() const { return ndim - 2; }
  int64_t channels() const { return dims[ndim - 1]; }
};

struct Graph {
  std::vector<Node> nodes;
  std::vector<std::pair<int, int>> updates;   // (from, variable)
};

void set_error(const char* fmt, ...);
const char* get_error();

// Orders of Definition 2 as minimal levels; false if the graph has a cycle.
bool topo_levels(const Graph& g, std::vector<int>& gamma);
// readers[u] = nodes with a read edge from u; outs[u] = readers plus control successors (sorted, unique).
void adjacency(const Graph& g, std::vector<std::vector<int>>& readers, std::vector<std::vector<int>>& outs);
// anc[v] = true if target is reachable from v along read/control edges (v != target).
void ancestors_of(const Graph& g, int target, std::vector<char>& anc);

lms_status add_variable(Graph& g, const char* name, int dtype, int ndim, const int64_t* dims, int kind, int* out);
lms_status add_op(Graph& g, const char* name, int op, const lms_attr* attr, int n_in, const int* inputs,
                  int phase, int* out);
lms_status build_backward(Graph& g, int loss_node);
lms_status build_update(Graph& g, float lr, float momentum, int* n_updates);

// ---- rewriting / planning -------------------------------------------------------------
lms_status rewrite_graph(Graph& g, const lms_params& p, lms_rewrite_stats* stats);

struct Block { uint64_t off = 0, size = 0; };
struct PlanResult {
  std::vector<int> order;                 // execution order of all nodes
  std::vector<int> pos;                   // position of node in order
  std::vector<int> last_use;              // position of the last reader of each node's tensor
  std::vector<Block> block;               // arena block of each node's output (size 0: not in the arena)
  std::vector<Block> wspace;              // transient workspace of each node
  // per node: earlier tenants of the address range of its output block / of its workspace; an entry v >= 0 is the
  // output block of node v, an entry ~v (negative) the workspace of node v
  std::vector<std::vector<int>> prev_tenants;
  std::vector<std::vector<int>> ws_prev_tenants;
  std::vector<uint64_t> host_off;         // per swap-out node: offset in the pinned pool
  std::vector<char> moved;                // block handed on to an in-place consumer instead of being released
  uint64_t arena_needed = 0, peak_live = 0, pinned_needed = 0;
  bool fits = true;
};
// Execution order: original operations in id order; a swap-out right after its producer; a
// swap-in right after its control operation.
bool schedule(const Graph& g, std::vector<int>& order);
// Offsets for every arena tensor for a sequential run in `order`; arena_limit 0 = unlimited.
// keep_all: no block is ever released.  external[v] = true: output lives outside the arena.
// encode_swaps: swapped tensors are parked in the encoded form (see swap_is_encoded / kernels.hpp), which
// needs a larger host slot.
// hold_swapped: with an arena limit, try to keep the blocks of swapped-out tensors taken until their copies are
// estimated to be over (all of them, else one after the other as far as the limit allows); false: the compact
// placement alone, which is what decides whether a graph fits.
void plan_memory(const Graph& g, uint64_t arena_limit, bool keep_all, const std::vector<char>* external,
                 PlanResult& out, bool encode_swaps = false, bool hold_swapped = true);
// true if a swap of this node's tensor can use the lossless encoding: 16-bit elements, count a multiple of 8
bool swap_is_encodable(const Node& n);
// Bytes a swap of this node's tensor is expected to put on the host link: all of them for a plain copy; encoded,
// half of a ReLU output's (every second element zero, the others 11 to 13 bits) and 0.7 of another tensor's.
double expected_link_bytes(const Graph& g, const Node& tensor, bool encode_swaps);
uint64_t workspace_bytes(const Graph& g, const Node& n);
// A COLSUM node whose output is bound to caller memory takes its result from the weight-gradient operation of the
// same layer, which reads the same dy anyway: colsum_host_wgrad gives that CONV_WGRAD node (or -1), wgrad_side_colsum
// the COLSUM node a CONV_WGRAD node serves (or -1).  The executor then skips the COLSUM node's own pass.
int colsum_host_wgrad(const Graph& g, int colsum_node);
int wgrad_side_colsum(const Graph& g, int wgrad_node);

}  // namespace lms
