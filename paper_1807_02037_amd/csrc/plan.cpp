// Execution order and static memory plan of a (possibly rewritten) graph.
//
// Shapes are static, so every tensor's arena offset is fixed before the first step.  The plan
// follows the lifetime rule of Section 3.5 (a tensor lives from the operation producing it to
// the last operation consuming it) over a sequential run in the order below, and records which
// earlier tenants each block overlaps so that the executor can order streams on reuse.
#include <algorithm>
#include <map>
#include <queue>
#include <tuple>
#include <utility>

#include "graph.hpp"
#include "kernels.hpp"

namespace lms {

// Operations keep their creation order; a swap-out runs right after its producer (Section 4.1 frees the device
// copy as soon as the producer is done) and a swap-in, or a recomputed copy, right after its control operation
// (Section 4.2.1); copies triggered by the same control operation run in their own creation order.
bool schedule(const Graph& g, std::vector<int>& order) {
  const int n = (int)g.nodes.size();
  typedef std::tuple<int, int, int> Key;
  std::vector<Key> key(n);
  std::vector<int> indeg(n, 0);
  std::vector<std::vector<int>> succ(n);
  for (const Node& v : g.nodes) {
    if (v.op == LMS_OP_SWAP_OUT) key[v.id] = Key(v.in[0], 1, v.id);
    else if (v.op == LMS_OP_SWAP_IN && !v.ctrl_in.empty()) key[v.id] = Key(*std::max_element(v.ctrl_in.begin(), v.ctrl_in.end()), 2, v.id);
    else if (v.op == LMS_OP_SWAP_IN) key[v.id] = Key(v.in[0], 3, v.id);
    else if (v.clone_of >= 0 && !v.ctrl_in.empty()) key[v.id] = Key(*std::max_element(v.ctrl_in.begin(), v.ctrl_in.end()), 2, v.id);
    else key[v.id] = Key(v.id, 0, v.id);
    if (v.is_var) continue;
    for (int u : v.in) { succ[u].push_back(v.id); ++indeg[v.id]; }
    for (int u : v.ctrl_in) { succ[u].push_back(v.id); ++indeg[v.id]; }
    // A column sum that comes out of a weight-gradient pass is written by that node: it is complete, for its readers
    // (the update phase), only after it.  In creation order the weight gradient comes first anyway; in a rewritten
    // graph it may have to wait for a swap-in or a recomputed copy while the column sum's own input is there already.
    const int host = colsum_host_wgrad(g, v.id);
    if (host >= 0) { succ[host].push_back(v.id); ++indeg[v.id]; }
  }
  // An operation reads the latest value of a variable (Section 3.2): the operation that updates a variable runs after
  // every reader of it that was created before (a recomputed copy counts as the operation it repeats) and before the
  // readers created after.  In creation order that holds by itself; in a rewritten graph an update operation is ready
  // as soon as its gradient is, long before a reader that still waits for a swap-in or a recomputed copy.
  if (!g.updates.empty()) {
    std::vector<std::vector<int>> readers_of_var(n);
    for (const Node& v : g.nodes)
      if (!v.is_var)
        for (int u : v.in)
          if (g.nodes[u].is_var) readers_of_var[u].push_back(v.id);
    for (const auto& up : g.updates) {
      const int from = up.first, var = up.second;
      for (int r : readers_of_var[var]) {
        if (r == from) continue;
        const int created = g.nodes[r].clone_of >= 0 ? g.nodes[r].clone_of : r;
        if (created < from) { succ[r].push_back(from); ++indeg[from]; }
        else { succ[from].push_back(r); ++indeg[r]; }
      }
    }
  }
  auto cmp = [&](int a, int b) { return key[a] > key[b]; };
  std::priority_queue<int, std::vector<int>, decltype(cmp)> ready(cmp);
  for (int i = 0; i < n; ++i)
    if (indeg[i] == 0) ready.push(i);
  order.clear();
  while (!ready.empty()) {
    int v = ready.top();
    ready.pop();
    order.push_back(v);
    for (int s : succ[v])
      if (--indeg[s] == 0) ready.push(s);
  }
  return (int)order.size() == n;
}

namespace {

constexpr uint64_t kAlign = 256;
inline uint64_t round_up(uint64_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// One arena allocation: the output of a node (or of a chain of nodes that accumulate in place), or
// the transient workspace of a node, live over the schedule positions [start, end].
struct Buf {
  bool ws = false;
  int start = 0, end = 0;
  uint64_t size = 0, off = 0;
  std::vector<int> members;
};

// Input whose block the output of n may take over: the gradient that n adds to its own result
// (each element is read and then written by the same thread).  -1 if there is none.
int inplace_source(const Graph& g, const Node& n) {
  const uint32_t f = n.attr.flags;
  int slot = -1;
  if (n.op == LMS_OP_CONV_DGRAD && (f & LMS_F_ADDEND)) slot = 2 + ((f & LMS_F_AFFINE) ? 1 : 0);
  else if (n.op == LMS_OP_TCONV_DGRAD && (f & LMS_F_ADDEND)) slot = 2;
  else if (n.op == LMS_OP_GRAD_SUM || n.op == LMS_OP_MSE_GRAD) slot = 0;   // element-wise
  if (slot < 0) return -1;
  const int src = n.in[slot];
  if (g.nodes[src].is_var || g.nodes[src].op == LMS_OP_SWAP_OUT) return -1;
  const bool elementwise = n.op == LMS_OP_GRAD_SUM || n.op == LMS_OP_MSE_GRAD;
  int uses = 0;
  for (int u : n.in) uses += (u == src);
  return (uses == 1 || elementwise) ? src : -1;
}

}  // namespace

// Lifetimes are known before the step runs, so offsets are assigned off line: buffers are placed
// largest first, each at the lowest offset that is free during its whole lifetime.
bool swap_is_encodable(const Node& n) { return n.dtype == LMS_BF16 && n.numel() % 8 == 0 && n.numel() > 0; }

double expected_link_bytes(const Graph& g, const Node& t, bool encode_swaps) {
  (void)g;
  const double bytes = (double)t.bytes();
  if (!encode_swaps || !swap_is_encodable(t)) return bytes;
  const bool relu_out = (t.op == LMS_OP_CONV || t.op == LMS_OP_TCONV) && (t.attr.flags & LMS_F_RELU);
  return bytes * (relu_out ? 0.5 : 0.7);
}

void plan_memory(const Graph& g, uint64_t arena_limit, bool keep_all, const std::vector<char>* external,
                 PlanResult& out, bool encode_swaps, bool hold_swapped) {
  const int n = (int)g.nodes.size();
  out = PlanResult();
  out.fits = schedule(g, out.order);
  out.pos.assign(n, -1);
  for (int i = 0; i < (int)out.order.size(); ++i) out.pos[out.order[i]] = i;
  out.last_use.assign(n, -1);
  out.block.assign(n, Block());
  out.wspace.assign(n, Block());
  out.prev_tenants.assign(n, {});
  out.ws_prev_tenants.assign(n, {});
  out.host_off.assign(n, 0);
  out.moved.assign(n, 0);
  if (!out.fits) return;
  for (const Node& v : g.nodes)
    for (int u : v.in) out.last_use[u] = std::max(out.last_use[u], out.pos[v.id]);

  std::vector<Buf> bufs;
  std::vector<int> buf_of(n, -1), ws_of(n, -1);
  for (int i = 0; i < n; ++i) {
    const int v = out.order[i];
    const Node& nv = g.nodes[v];
    if (nv.is_var) continue;
    if (nv.op == LMS_OP_SWAP_OUT) {
      out.host_off[v] = out.pinned_needed;
      out.pinned_needed += round_up(encode_swaps && swap_is_encodable(nv) ? swap_encoded_bytes((uint64_t)nv.numel()) : nv.bytes());
    } else if (!nv.external && !(external && (*external)[v])) {
      const uint64_t sz = round_up(nv.bytes());
      // a tensor nobody reads (the loss, an unbound gradient) stays until the step ends
      const int end = (keep_all || out.last_use[v] < 0) ? n - 1 : std::max(out.last_use[v], i);
      const int src = keep_all ? -1 : inplace_source(g, nv);
      if (src >= 0 && buf_of[src] >= 0 && out.last_use[src] == i && bufs[buf_of[src]].size == sz && !out.moved[src]) {
        // the gradient being added dies here: accumulate in place, the block changes owner
        Buf& b = bufs[buf_of[src]];
        b.end = end;
        b.members.push_back(v);
        buf_of[v] = buf_of[src];
        out.moved[src] = 1;
        out.prev_tenants[v].push_back(src);
      } else {
        Buf b;
        b.start = i;
        b.end = end;
        b.size = sz;
        b.members.push_back(v);
        buf_of[v] = (int)bufs.size();
        bufs.push_back(b);
      }
    }
    const uint64_t ws = round_up(workspace_bytes(g, nv));
    if (ws) {
      Buf b;
      b.ws = true;
      b.start = i;
      b.end = keep_all ? n - 1 : i;
      b.size = ws;
      b.members.push_back(v);
      ws_of[v] = (int)bufs.size();
      bufs.push_back(b);
    }
  }
  // peak of the sum of live bytes (what a perfect allocator would need)
  {
    std::vector<int64_t> delta(n + 1, 0);
    for (const Buf& b : bufs) { delta[b.start] += (int64_t)b.size; delta[b.end + 1] -= (int64_t)b.size; }
    int64_t live = 0;
    for (int i = 0; i < n; ++i) { live += delta[i]; out.peak_live = std::max<uint64_t>(out.peak_live, (uint64_t)live); }
  }
  // placement
  std::vector<int> by_size(bufs.size());
  for (size_t i = 0; i < bufs.size(); ++i) by_size[i] = (int)i;
  std::sort(by_size.begin(), by_size.end(), [&](int a, int b) {
    if (bufs[a].size != bufs[b].size) return bufs[a].size > bufs[b].size;
    if (bufs[a].start != bufs[b].start) return bufs[a].start < bufs[b].start;
    return a < b;
  });
  // A buffer is placed at the lowest offset that is free while its block is in use: from its start to until[bi].
  std::vector<std::pair<uint64_t, uint64_t>> busy;
  auto place = [&](const std::vector<int>& until) -> uint64_t {
    std::vector<int> placed;
    uint64_t need = 0;
    for (int bi : by_size) {
      Buf& b = bufs[bi];
      busy.clear();
      for (int pj : placed) {
        const Buf& a = bufs[pj];
        if (a.start <= until[bi] && b.start <= until[pj]) busy.emplace_back(a.off, a.off + a.size);
      }
      std::sort(busy.begin(), busy.end());
      uint64_t off = 0;
      for (const auto& iv : busy) {
        if (iv.first >= off + b.size) break;
        off = std::max(off, iv.second);
      }
      b.off = off;
      placed.push_back(bi);
      need = std::max(need, off + b.size);
    }
    return need;
  };
  std::vector<int> until(bufs.size());
  for (size_t bi = 0; bi < bufs.size(); ++bi) until[bi] = bufs[bi].end;
  // The block of a swapped-out tensor is free for the plan once its last reader has run, but the executor can only hand
  // it on when the copy to the host has finished as well; where the next tenant comes too early the compute stream
  // stands still for the rest of the copy.  With an arena limit to fill, the placement is therefore tried first with
  // such blocks held until their copy is over, by a rough clock: an operation takes its tensor bytes at 2 TB/s, a copy
  // the bytes it is expected to put on the link (expected_link_bytes) at 52 GB/s.  If that does not fit the limit, the blocks are
  // held one after the other, in schedule order, each for as much of its copy as the limit allows, and no longer than the plan needs otherwise
  // (the compact placement).  Offsets depend on sizes and positions only, so the
  // plan stays reproducible.
  bool relaxed = false;
  if (arena_limit && !keep_all && hold_swapped) {
    std::vector<double> clock(n + 1, 0.0);            // clock[i]: start of position i
    for (int i = 0; i < n; ++i) {
      const Node& nv = g.nodes[out.order[i]];
      double bytes = 0.0;
      if (!nv.is_var && nv.op != LMS_OP_SWAP_OUT && nv.op != LMS_OP_SWAP_IN) {
        bytes = (double)nv.bytes();
        for (int u : nv.in) bytes += (double)g.nodes[u].bytes();
      }
      clock[i + 1] = clock[i] + bytes / 2e12;
    }
    const double link = 52e9;
    std::vector<int> held = until;
    std::vector<int> longer;                          // buffers whose block would be held beyond its last reader
    double link_free = 0.0;                           // the copies leave one after the other
    for (int i = 0; i < n; ++i) {
      const Node& r = g.nodes[out.order[i]];
      if (r.op != LMS_OP_SWAP_OUT || buf_of[r.in[0]] < 0) continue;
      const int bi = buf_of[r.in[0]];
      const double done = std::max(clock[i], link_free) + expected_link_bytes(g, g.nodes[r.in[0]], encode_swaps) / link;
      link_free = done;
      int p = held[bi];
      while (p + 1 < n && clock[p + 1] < done) ++p;
      if (p > held[bi]) { held[bi] = p; longer.push_back(bi); }
    }
    if (!longer.empty() && place(held) <= arena_limit) relaxed = true;
    else if (longer.size() > 1) {
      // not all of them fit: hold one block after the other, in schedule order, as long as the arena still suffices
      std::vector<int> some = until;
      for (int bi : longer) {
        // as long as the limit allows: the whole copy, else the longest part of it found by bisection (a block given
        // up before its copy is over still makes the next tenant come later, and wait less)
        int lo = some[bi], hi = held[bi];             // lo fits (or nothing does), hi is wanted
        some[bi] = hi;
        if (place(some) <= arena_limit) { relaxed = true; continue; }
        for (int it = 0; it < 4 && hi - lo > 1; ++it) {
          const int mid = lo + (hi - lo) / 2;
          some[bi] = mid;
          if (place(some) <= arena_limit) { lo = mid; relaxed = true; }
          else hi = mid;
        }
        some[bi] = lo;
      }
      if (relaxed) {
        held = some;
        place(held);                                  // the offsets of the accepted set
      }
    }
  }
  if (!relaxed) out.arena_needed = place(until);
  else {
    out.arena_needed = 0;
    for (const Buf& bb : bufs) out.arena_needed = std::max(out.arena_needed, bb.off + bb.size);
  }
  if (arena_limit && out.arena_needed > arena_limit) out.fits = false;
  for (int v = 0; v < n; ++v) {
    if (buf_of[v] >= 0) out.block[v] = Block{bufs[buf_of[v]].off, bufs[buf_of[v]].size};
    if (ws_of[v] >= 0) out.wspace[v] = Block{bufs[ws_of[v]].off, bufs[ws_of[v]].size};
  }
  // earlier tenants of every buffer's address range: per sub-range only the most recent one matters
  std::vector<int> by_end(bufs.size());
  for (size_t i = 0; i < bufs.size(); ++i) by_end[i] = (int)i;
  std::sort(by_end.begin(), by_end.end(), [&](int a, int b) { return bufs[a].end > bufs[b].end; });
  for (size_t bi = 0; bi < bufs.size(); ++bi) {
    const Buf& b = bufs[bi];
    std::vector<std::pair<uint64_t, uint64_t>> open{{b.off, b.off + b.size}};   // parts without a known tenant yet
    std::vector<int>& prev = b.ws ? out.ws_prev_tenants[b.members[0]] : out.prev_tenants[b.members[0]];
    for (int aj : by_end) {
      if (open.empty()) break;
      const Buf& a = bufs[aj];
      if (a.end >= b.start) continue;
      const uint64_t lo = a.off, hi = a.off + a.size;
      bool hit = false;
      std::vector<std::pair<uint64_t, uint64_t>> rest;
      for (const auto& iv : open) {
        if (iv.second <= lo || iv.first >= hi) { rest.push_back(iv); continue; }
        hit = true;
        if (iv.first < lo) rest.emplace_back(iv.first, lo);
        if (iv.second > hi) rest.emplace_back(hi, iv.second);
      }
      if (hit) {
        // a workspace was touched by its operation alone, an output block by its producer and every reader
        for (int m : a.members) prev.push_back(a.ws ? ~m : m);
        open.swap(rest);
      }
    }
  }
}

}  // namespace lms
