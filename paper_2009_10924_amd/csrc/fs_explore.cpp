// Fusion exploration over a multi-pattern graph (paper Section 5): the search, and the making of
// an executable program from the plan it finds (fs_program.cpp runs it).
//   * candidate patterns per vertex, from the last vertex to the first, by PatternReduction
//     (Section 5.2): a vertex joins combinations of its consumers' candidate patterns, consumers
//     are handled in groups of two, only the top-k patterns by score survive;
//   * patterns with a cyclic dependence or that the code generator cannot process are discarded
//     (Section 5.2) -- "can process" here means: a hand-written kernel family matches it or it
//     compiles to a row program (a generated kernel, or the interpreter).  Computations outside the
//     graph that the graph names (Section 1: compute-intensive ops go to libraries and are not fused) order execution
//     like edges and are never inside a pattern;
//   * score f = T_reduced_mem + T_reduced_calls - T_penalty (Section 5.4, Eq. 3), with constants
//     measured on MI355X (launch cost, streaming rate) and the penalty from the kernel estimate
//     without compiled register figures;
//   * the overall plan by beam search over the vertices from producers to consumers (Section 5.3),
//     the final choice among the beam's plans by the full latency evaluator (Section 4.3);
//   * independent launch-bound patterns of the chosen plan are packed into one launch (remote
//     fusion / kernel packing, Section 5.2 and 4.1).
// The program runs the patterns in dependence order, in stages where external computations lie
// between them; tensors that cross from one pattern to another live in the caller's workspace,
// placed by lifetime; fold launches of column sums that nothing reads move behind the last step
// and run as one.
#include <algorithm>
#include <cstring>
#include <map>
#include <set>
#include <string>

#include "fs_internal.hpp"
#include "fs_program.hpp"

extern "C" {
fs_status fs_graph_create(fs_graph** out);
void fs_graph_destroy(fs_graph* g);
fs_tensor fs_graph_input(fs_graph* g, int32_t dtype, int32_t rank, const int64_t* dims);
fs_tensor fs_graph_op(fs_graph* g, int32_t opcode, int32_t n_in, const fs_tensor* in, const void* attr, size_t attr_bytes);
fs_status fs_graph_output(fs_graph* g, fs_tensor t, int32_t store_as);
fs_status fs_graph_finalize(fs_graph* g);
}

namespace fs {
namespace {

typedef std::vector<int> OpSet;   // sorted op indices

struct SubGraph {
  fs_graph* g = nullptr;
  std::vector<int32_t> in_tensor;    // sub input slot  -> tensor id in the big graph
  std::vector<int32_t> out_tensor;   // sub output slot -> tensor id in the big graph
  ~SubGraph() { fs_graph_destroy(g); }
  SubGraph() = default;
  SubGraph(const SubGraph&) = delete;
  SubGraph& operator=(const SubGraph&) = delete;
};

struct Scored {
  bool valid = false;
  int32_t why = FS_OK;     // FS_ERR_CYCLE / FS_ERR_UNSUPPORTED_PATTERN / FS_ERR_DTYPE when not valid
  double f = 0;            // microseconds
  double f_optimistic = 0; // what f would be if the ops ran as one kernel at streaming rate; set for every convex pattern
  double t_fused = 0, t_unfused = 0;
};

struct Explorer {
  const fs_graph& g;
  int n;                                     // ops
  std::vector<std::vector<int>> consumers;   // op -> ops that read its result (sorted, distinct)
  std::vector<std::vector<int>> waiting;     // op -> ops that wait for its result through an external computation
  std::vector<std::vector<uint64_t>> desc;   // op -> bitset of everything that runs after it because of it
  std::vector<std::vector<uint64_t>> reads_of;   // op -> bitset of its descendants through tensors of the graph alone
  std::map<OpSet, Scored> memo;
  int top_k = 3, beam_width = 3;

  explicit Explorer(const fs_graph& graph) : g(graph), n((int)graph.ops.size()) {
    consumers.resize(n);
    for (int i = 0; i < n; ++i) {
      std::set<int> c(g.tensors[g.ops[i].out].consumers.begin(), g.tensors[g.ops[i].out].consumers.end());
      consumers[i].assign(c.begin(), c.end());
    }
    waiting.resize(n);
    const std::vector<std::vector<int>> waits_for = g.external_producers();
    for (int i = 0; i < n; ++i)
      for (int p : waits_for[i]) waiting[p].push_back(i);
    const int words = (n + 63) / 64;
    desc.assign(n, std::vector<uint64_t>(words, 0));
    reads_of.assign(n, std::vector<uint64_t>(words, 0));
    for (int i = n - 1; i >= 0; --i) {
      for (int c : consumers[i]) {
        desc[i][c / 64] |= 1ull << (c % 64);
        reads_of[i][c / 64] |= 1ull << (c % 64);
        for (int w = 0; w < words; ++w) { desc[i][w] |= desc[c][w]; reads_of[i][w] |= reads_of[c][w]; }
      }
      for (int c : waiting[i]) {
        desc[i][c / 64] |= 1ull << (c % 64);
        for (int w = 0; w < words; ++w) desc[i][w] |= desc[c][w];
      }
    }
  }

  // An op and an op that waits for its result through an external computation cannot share a kernel.
  bool holds_external_dependence(const OpSet& p) const {
    for (int o : p)
      for (int c : waiting[o])
        if (std::binary_search(p.begin(), p.end(), c)) return true;
    return false;
  }

  // No path may leave the pattern and come back (Section 5.2, cyclic dependence).
  bool convex(const OpSet& p) const {
    const int words = (n + 63) / 64;
    std::vector<uint64_t> in(words, 0), below(words, 0);
    for (int o : p) in[o / 64] |= 1ull << (o % 64);
    for (int o : p)
      for (int w = 0; w < words; ++w) below[w] |= desc[o][w];
    for (int x = 0; x < n; ++x) {
      if ((in[x / 64] >> (x % 64)) & 1) continue;
      if (!((below[x / 64] >> (x % 64)) & 1)) continue;
      for (int w = 0; w < words; ++w)
        if (desc[x][w] & in[w]) return false;
    }
    return true;
  }

  // The pattern as a graph of its own: operands made outside become its inputs, results read
  // outside (or graph outputs) become its outputs.
  fs_status extract(const OpSet& p, SubGraph* sub) const {
    std::vector<char> inside(n, 0);
    for (int o : p) inside[o] = 1;
    if (fs_graph_create(&sub->g) != FS_OK) return FS_ERR_INVALID_ARG;
    std::map<int32_t, fs_tensor> local;   // big-graph tensor -> sub tensor
    for (int o : p) {
      const Op& op = g.ops[o];
      fs_tensor in[2] = {-1, -1};
      for (int k = 0; k < op.n_in; ++k) {
        const int32_t t = op.in[k];
        auto it = local.find(t);
        if (it == local.end()) {
          const Tensor& T = g.tensors[t];
          // what a neighbouring pattern wrote is what this one reads: an output stored in another dtype than it
          // was computed in cannot also feed a different pattern
          if (T.output_slot >= 0 && T.store_as != T.dtype) return FS_ERR_DTYPE;
          const fs_tensor id = fs_graph_input(sub->g, T.dtype, T.rank, T.dims);
          if (id < 0) return id;
          sub->in_tensor.push_back(t);
          it = local.emplace(t, id).first;
        }
        in[k] = it->second;
      }
      fs_tensor r;
      const Tensor& out = g.tensors[op.out];
      switch (op.opcode) {
        case FS_SCALE: case FS_ADD_SCALAR: {
          fs_attr_scalar a = {op.scalar};
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, &a, sizeof a);
          break;
        }
        case FS_BROADCAST: {
          fs_attr_dims a;
          a.rank = out.rank;
          for (int k = 0; k < FS_MAX_RANK; ++k) a.dims[k] = k < out.rank ? out.dims[k] : 1;
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, &a, sizeof a);
          break;
        }
        case FS_REDUCE_SUM: case FS_REDUCE_MAX: case FS_REDUCE_MEAN: {
          fs_attr_axis a = {op.axis};
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, &a, sizeof a);
          break;
        }
        case FS_TRANSPOSE: {
          fs_attr_perm a;
          for (int k = 0; k < FS_MAX_RANK; ++k) a.perm[k] = op.perm[k];
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, &a, sizeof a);
          break;
        }
        case FS_CONVERT: {
          fs_attr_dtype a = {op.to_dtype};
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, &a, sizeof a);
          break;
        }
        default:
          r = fs_graph_op(sub->g, op.opcode, op.n_in, in, nullptr, 0);
          break;
      }
      if (r < 0) return r;
      local[op.out] = r;
      bool read_outside = false;
      for (int c : out.consumers)
        if (!inside[c]) read_outside = true;
      if (out.output_slot >= 0 && read_outside && out.store_as != out.dtype) return FS_ERR_DTYPE;
      if (out.output_slot >= 0 || read_outside) {
        const fs_status s = fs_graph_output(sub->g, r, out.output_slot >= 0 ? out.store_as : out.dtype);
        if (s != FS_OK) return s;
        sub->out_tensor.push_back(op.out);
      }
    }
    return fs_graph_finalize(sub->g);
  }

  // per-op execution of one op: one launch and one dependent memory round trip, operands read and the result
  // written (float32 unless the op keeps a dtype)
  double t_single(int o) const {
    const DeviceModel& d = device();
    const Op& op = g.ops[o];
    double bytes = 0;
    for (int k = 0; k < op.n_in; ++k) bytes += (double)g.tensors[op.in[k]].numel() * dtype_bytes(g.tensors[op.in[k]].dtype);
    const Tensor& out = g.tensors[op.out];
    bytes += (double)out.numel() * dtype_bytes(out.output_slot >= 0 ? out.store_as : out.dtype);
    // a sum over rows that different workgroups own takes a second launch to fold their partial sums
    const bool across_rows = (op.opcode == FS_REDUCE_SUM || op.opcode == FS_REDUCE_MAX || op.opcode == FS_REDUCE_MEAN) &&
                             op.axis != g.tensors[op.in[0]].rank - 1;
    return d.launch_s * (across_rows ? 2.0 : 1.0) + d.mem_latency_s + bytes / (d.hbm_peak_Bps * d.stream_fraction);
  }

  // Delta-evaluator (Eq. 3): time saved by running the ops of `p` as one pattern.
  const Scored& score(const OpSet& p) {
    auto it = memo.find(p);
    if (it != memo.end()) return it->second;
    Scored s;
    for (int o : p) s.t_unfused += t_single(o);
    if (p.size() == 1) {
      s.valid = true;
      s.t_fused = s.t_unfused;
      s.f = 0;
    } else if (holds_external_dependence(p) || !convex(p)) {
      s.why = FS_ERR_CYCLE;
    } else {
      SubGraph sub;
      const fs_status st = extract(p, &sub);
      if (st == FS_OK) {
        const DeviceModel& d = device();
        s.f_optimistic = (s.t_unfused - (d.launch_s + d.mem_latency_s + (double)graph_bytes_min(*sub.g) / (d.hbm_peak_Bps * d.stream_fraction))) * 1e6;
      }
      std::vector<Candidate> cands;
      if (st != FS_OK) {
        s.why = st == FS_ERR_DTYPE ? FS_ERR_DTYPE : FS_ERR_UNSUPPORTED_PATTERN;
      } else if (build_stitched(*sub.g, &cands, nullptr).empty() || cands.empty()) {
        s.why = FS_ERR_UNSUPPORTED_PATTERN;
      } else {
        // T_penalty comes from the kernel estimate with register figures left at their estimates
        // (the expensive part of the latency evaluator is skipped during exploration)
        double best = 1e30;
        bool only_fallbacks = true;
        for (const Candidate& c : cands) only_fallbacks = only_fallbacks && c.fallback;
        for (const Candidate& c : cands) {
          if (c.fallback && !only_fallbacks) continue;   // the plan would not pick it either
          double t = evaluate(c.cost, 0).seconds;
          if (c.launches.size() > 1) t += device().launch_s * (double)(c.launches.size() - 1);
          best = std::min(best, t);
        }
        s.valid = true;
        s.t_fused = best;
        s.f = (s.t_unfused - s.t_fused) * 1e6;
      }
    }
    return memo.emplace(p, s).first->second;
  }

  // A candidate pattern.  `tentative`: no kernel can run it as it stands, but it is convex and may grow into
  // one that a kernel family covers; it takes part in the growth with its optimistic score and never in a plan.
  struct Pat {
    OpSet ops;
    double f = 0;
    bool tentative = false;
  };
  static bool better(const Pat& a, const Pat& b) {
    if (a.f != b.f) return a.f > b.f;
    return a.ops < b.ops;
  }
  // top-k runnable patterns and top-k tentative ones, each list by score
  void keep_top(std::vector<Pat>* v) const {
    std::sort(v->begin(), v->end(), better);
    v->erase(std::unique(v->begin(), v->end(), [](const Pat& a, const Pat& b) { return a.ops == b.ops; }), v->end());
    std::vector<Pat> kept;
    int n_real = 0, n_tent = 0;
    for (const Pat& p : *v) {
      int& count = p.tentative ? n_tent : n_real;
      if (count < top_k) { kept.push_back(p); ++count; }
    }
    v->swap(kept);
  }
  static OpSet unite(const OpSet& a, const OpSet& b) {
    OpSet r;
    std::set_union(a.begin(), a.end(), b.begin(), b.end(), std::back_inserter(r));
    return r;
  }
  // a scored pattern if it is valid and gains time; a tentative one if only the kernel is missing
  bool consider(const OpSet& ops, std::vector<Pat>* out) {
    const Scored& s = score(ops);
    if (s.valid) {
      if (!(s.f > 0)) return false;
      out->push_back(Pat{ops, s.f, false});
      return true;
    }
    if (s.why == FS_ERR_UNSUPPORTED_PATTERN && s.f_optimistic > 0 && (int)ops.size() <= max_tentative_ops &&
        !reads_own_output(ops)) {
      out->push_back(Pat{ops, s.f_optimistic, true});
      return true;
    }
    return false;
  }
  int max_tentative_ops = 24;
  // A graph output is written to memory whatever the plan: growing a speculative pattern across it gains little
  // and lets ever larger unrunnable merges crowd out the runnable pattern on either side.
  bool reads_own_output(const OpSet& p) const {
    for (int o : p) {
      const Tensor& T = g.tensors[g.ops[o].out];
      if (T.output_slot < 0) continue;
      for (int c : T.consumers)
        if (std::binary_search(p.begin(), p.end(), c)) return true;
    }
    return false;
  }

  std::vector<std::vector<Pat>> cand;   // per vertex: candidate patterns whose producer is the vertex (without the singleton)

  // Temporary candidates of vertex v from one group of its consumers (Section 5.2).
  std::vector<Pat> reduce_group(int v, const std::vector<int>& group) {
    std::vector<Pat> out;
    if (group.size() <= 2) {
      // every combination of "one candidate pattern or nothing" per consumer, plus v
      std::vector<std::vector<OpSet>> choices;
      for (int c : group) {
        std::vector<OpSet> ch;
        ch.push_back(OpSet());            // do not take this consumer
        ch.push_back(OpSet{c});           // the consumer alone
        for (const Pat& p : cand[c]) ch.push_back(p.ops);
        choices.push_back(ch);
      }
      std::vector<size_t> idx(choices.size(), 0);
      while (true) {
        OpSet u{v};
        bool any = false;
        for (size_t k = 0; k < choices.size(); ++k) {
          if (!choices[k][idx[k]].empty()) any = true;
          u = unite(u, choices[k][idx[k]]);
        }
        if (any) consider(u, &out);
        size_t k = 0;
        while (k < idx.size() && ++idx[k] == choices[k].size()) idx[k++] = 0;
        if (k == idx.size()) break;
      }
      keep_top(&out);
      return out;
    }
    // divide, conquer, and reduce: the halves' temporary candidates, and their pairwise unions
    const size_t half = group.size() / 2;
    const std::vector<Pat> a = reduce_group(v, std::vector<int>(group.begin(), group.begin() + half));
    const std::vector<Pat> b = reduce_group(v, std::vector<int>(group.begin() + half, group.end()));
    out = a;
    out.insert(out.end(), b.begin(), b.end());
    for (const Pat& x : a)
      for (const Pat& y : b) consider(unite(x.ops, y.ops), &out);
    keep_top(&out);
    return out;
  }

  void explore_patterns() {
    cand.assign(n, {});
    for (int v = n - 1; v >= 0; --v)
      if (!consumers[v].empty()) cand[v] = reduce_group(v, consumers[v]);
    // Seeds beyond the bottom-up growth.  The growth only reaches a pattern through smaller patterns that are
    // themselves runnable; a hand-written family (say a row pass that ends in a column reduction) is runnable
    // as a whole while some of its parts are not, and the top-k cut favours ever larger patterns.  So three whole
    // shapes are offered directly: everything downstream of a vertex, the same stopped at graph outputs, and the
    // connected component a vertex starts (ops joined by an edge or a shared operand).
    std::vector<int> comp(n, -1);
    for (int v = 0; v < n; ++v) {
      if (comp[v] >= 0) continue;
      std::vector<int> stack{v};
      comp[v] = v;
      while (!stack.empty()) {
        const int o = stack.back();
        stack.pop_back();
        std::vector<int> next = consumers[o];
        for (int k = 0; k < g.ops[o].n_in; ++k) {
          const Tensor& operand = g.tensors[g.ops[o].in[k]];
          if (operand.producer >= 0) next.push_back(operand.producer);
          for (int c : operand.consumers) next.push_back(c);   // ops that share an operand belong together too
        }
        for (int x : next)
          if (comp[x] < 0) { comp[x] = v; stack.push_back(x); }
      }
    }
    for (int v = 0; v < n; ++v) {
      std::vector<Pat> seeds;
      OpSet cone{v};
      for (int x = v + 1; x < n; ++x)
        if ((reads_of[v][x / 64] >> (x % 64)) & 1) cone.push_back(x);
      if (cone.size() > 1) consider(cone, &seeds);
      // the same cone, but not continued past a graph output: that tensor is written to memory anyway
      OpSet bounded{v};
      {
        std::vector<char> in(n, 0);
        in[v] = 1;
        for (int x = v; x < n; ++x) {
          if (!in[x]) continue;
          if (g.tensors[g.ops[x].out].output_slot >= 0) continue;
          for (int c : consumers[x]) in[c] = 1;
        }
        for (int x = v + 1; x < n; ++x)
          if (in[x]) bounded.push_back(x);
      }
      if (bounded.size() > 1 && bounded != cone) consider(bounded, &seeds);
      if (comp[v] == v) {
        OpSet whole;
        for (int x = 0; x < n; ++x)
          if (comp[x] == v) whole.push_back(x);
        if (whole.size() > 1 && whole != cone && whole != bounded) consider(whole, &seeds);
      }
      // seeds are not subject to the top-k cut (at most three per vertex)
      for (const Pat& sd : seeds) {
        bool have = false;
        for (const Pat& p : cand[v])
          if (p.ops == sd.ops) have = true;
        if (!have) cand[v].push_back(sd);
      }
      std::sort(cand[v].begin(), cand[v].end(), better);
    }
  }

  // Patterns that are convex one by one can still wait for each other in a circle (P = {a, d}, Q = {b, c} with edges
  // a -> b and c -> d and no path from b to c): Section 5.2's "no cyclic dependence" is a property of the plan, checked
  // on the graph whose vertices are the plan's patterns and the ops outside them.
  bool acyclic(const std::vector<OpSet>& groups) const {
    std::vector<int> gid(n, -1);
    int n_groups = 0;
    for (const OpSet& p : groups) {
      for (int o : p) gid[o] = n_groups;
      ++n_groups;
    }
    for (int o = 0; o < n; ++o)
      if (gid[o] < 0) gid[o] = n_groups++;
    std::vector<std::vector<int>> next(n_groups);
    std::vector<int> pending(n_groups, 0);
    for (int o = 0; o < n; ++o) {
      for (int c : consumers[o])
        if (gid[c] != gid[o]) next[gid[o]].push_back(gid[c]);
      for (int c : waiting[o])
        if (gid[c] != gid[o]) next[gid[o]].push_back(gid[c]);
    }
    for (int a = 0; a < n_groups; ++a) {
      std::sort(next[a].begin(), next[a].end());
      next[a].erase(std::unique(next[a].begin(), next[a].end()), next[a].end());
      for (int b : next[a]) ++pending[b];
    }
    std::vector<int> ready;
    for (int a = 0; a < n_groups; ++a)
      if (pending[a] == 0) ready.push_back(a);
    int done = 0;
    while (!ready.empty()) {
      const int a = ready.back();
      ready.pop_back();
      ++done;
      for (int b : next[a])
        if (--pending[b] == 0) ready.push_back(b);
    }
    return done == n_groups;
  }

  // Remote fusion (Section 5.2): patterns of a plan that are not adjacent in the graph -- no edge joins them --
  // may still share a kernel.  Greedy reading: among all pairs of the plan's patterns (single ops included)
  // whose union is a runnable pattern, merge the pair that gains the most over running the two apart; repeat
  // until no pair gains.  Returns the total gain (microseconds).
  double merge_remote(std::vector<OpSet>* groups) {
    if (groups->size() > 64) return 0.0;
    std::sort(groups->begin(), groups->end());
    auto f_of = [&](const OpSet& p) { return p.size() > 1 ? score(p).f : 0.0; };
    double total = 0.0;
    while (true) {
      double best_gain = 0.0;
      size_t bi = 0, bj = 0;
      for (size_t i = 0; i < groups->size(); ++i)
        for (size_t j = i + 1; j < groups->size(); ++j) {
          const OpSet u = unite((*groups)[i], (*groups)[j]);
          const Scored& s = score(u);
          if (!s.valid) continue;
          const double gain = s.f - f_of((*groups)[i]) - f_of((*groups)[j]);
          if (!(gain > best_gain)) continue;
          std::vector<OpSet> merged;
          for (size_t k = 0; k < groups->size(); ++k)
            if (k != i && k != j) merged.push_back((*groups)[k]);
          merged.push_back(u);
          if (!acyclic(merged)) continue;   // the union is convex, but the plan with it would wait for itself
          best_gain = gain;
          bi = i;
          bj = j;
        }
      if (!(best_gain > 0.0)) break;
      const OpSet u = unite((*groups)[bi], (*groups)[bj]);
      groups->erase(groups->begin() + bj);
      (*groups)[bi] = u;
      std::sort(groups->begin(), groups->end());
      total += best_gain;
    }
    return total;
  }

  struct PlanSet {
    std::vector<OpSet> patterns;      // multi-op patterns, in the order they were appended
    std::vector<uint64_t> covered;
    double f = 0;
  };
  // Beam search (Section 5.3).  Plans are ranked by their accumulated score plus a look-ahead for the part of the
  // graph not visited yet: every op still uncovered counts with the best score per op of any candidate pattern
  // that holds it.  Without the look-ahead a large pattern that swallows half of a neighbouring pattern pushes
  // out the plan that takes both neighbours whole; at the last vertex the look-ahead is zero and the ranking is
  // the paper's.
  std::vector<PlanSet> beam() {
    const int words = (n + 63) / 64;
    std::vector<double> per_op(n, 0.0);
    for (int v = 0; v < n; ++v)
      for (const Pat& p : cand[v]) {
        if (p.tentative) continue;
        const double share = p.f / (double)p.ops.size();
        for (int o : p.ops) per_op[o] = std::max(per_op[o], share);
      }
    auto rank = [&](const PlanSet& s, int v) {
      double r = s.f;
      for (int u = v + 1; u < n; ++u)
        if (!((s.covered[u / 64] >> (u % 64)) & 1)) r += per_op[u];
      return r;
    };
    std::vector<PlanSet> sets(1);
    sets[0].covered.assign(words, 0);
    for (int v = 0; v < n; ++v) {
      std::vector<PlanSet> next = sets;
      for (const PlanSet& s : sets) {
        for (const Pat& p : cand[v]) {
          if (p.tentative) continue;
          bool overlap = false;
          for (int o : p.ops)
            if ((s.covered[o / 64] >> (o % 64)) & 1) { overlap = true; break; }
          if (overlap) continue;
          PlanSet t = s;
          t.patterns.push_back(p.ops);
          if (!acyclic(t.patterns)) continue;
          for (int o : p.ops) t.covered[o / 64] |= 1ull << (o % 64);
          t.f += p.f;
          next.push_back(t);
        }
      }
      std::vector<std::pair<double, size_t>> order;
      for (size_t k = 0; k < next.size(); ++k) order.push_back({rank(next[k], v), k});
      std::stable_sort(order.begin(), order.end(), [&](const std::pair<double, size_t>& a, const std::pair<double, size_t>& b) {
        if (a.first != b.first) return a.first > b.first;
        return next[a.second].patterns < next[b.second].patterns;
      });
      std::vector<PlanSet> kept;
      for (size_t k = 0; k < order.size() && (int)k < beam_width; ++k) kept.push_back(next[order[k].second]);
      sets.swap(kept);
    }
    return sets;
  }
};

}  // namespace
}  // namespace fs

using namespace fs;


namespace {

int64_t align256(int64_t v) { return (v + 255) / 256 * 256; }

// first-fit placement of [begin, end] lifetimes (in steps) into one arena
struct Arena {
  struct Block { int64_t off, size; int begin, end; };
  std::vector<Block> blocks;
  int64_t top = 0;
  int64_t place(int64_t size, int begin, int end) {
    size = align256(size);
    std::vector<Block> live;
    for (const Block& b : blocks)
      if (!(b.end < begin || end < b.begin)) live.push_back(b);
    std::sort(live.begin(), live.end(), [](const Block& a, const Block& b) { return a.off < b.off; });
    int64_t off = 0;
    for (const Block& b : live) {
      if (off + size <= b.off) break;
      off = std::max(off, b.off + b.size);
    }
    blocks.push_back({off, size, begin, end});
    top = std::max(top, off + size);
    return off;
  }
};

struct BuiltPlan {
  std::vector<fs_program::Step> steps;
  double predicted = 0;   // latency-evaluator estimate, microseconds
  double f = 0;           // accumulated delta-evaluator score after remote fusion
  bool ok = false;
  void destroy() {
    for (fs_program::Step& s : steps) fs_plan_destroy(s.plan);
    steps.clear();
    ok = false;
  }
};

// One plan of the beam made executable: remote fusion, then a stitched plan per pattern and per op left alone.
fs_status build_steps(Explorer* ex, const Explorer::PlanSet& plan, bool remote_fusion, BuiltPlan* b, std::string* error_text) {
  std::vector<OpSet> groups = plan.patterns;
  for (int o = 0; o < ex->n; ++o)
    if (!((plan.covered[o / 64] >> (o % 64)) & 1)) groups.push_back(OpSet{o});
  b->f = plan.f + (remote_fusion ? ex->merge_remote(&groups) : 0.0);
  b->ok = true;
  for (const OpSet& p : groups) {
    SubGraph sub;
    fs_status st = ex->extract(p, &sub);
    if (st == FS_ERR_DTYPE)
      *error_text = "a tensor that is stored as a graph output in another dtype than it was computed in also feeds ops that "
                    "cannot join its pattern; add an explicit convert and read its result";
    else if (st != FS_OK)
      *error_text = fs_last_error();
    fs_program::Step step;
    if (st == FS_OK) {
      step.ops = p;
      step.f = p.size() > 1 ? ex->score(p).f : 0.0;
      st = create_plan(sub.g, FS_SCHEME_AUTO, nullptr, false, &step.plan);   // generated kernels are compiled for the winner only
      if (st != FS_OK) *error_text = fs_last_error();
    }
    if (st != FS_OK) {
      b->destroy();
      return st;
    }
    for (int32_t t : sub.in_tensor) {
      BufRef r;
      r.kind = BUF_INPUT;
      r.slot = t;           // tensor id in the whole graph for now; resolved once the order is known
      step.in.push_back(r);
    }
    for (int32_t t : sub.out_tensor) {
      BufRef r;
      r.kind = BUF_OUTPUT;
      r.slot = t;
      step.out.push_back(r);
    }
    b->predicted += step.plan->candidates[step.plan->chosen].info.predicted_us;
    b->steps.push_back(std::move(step));
  }
  return FS_OK;
}

std::vector<int> owners(const fs_graph& g, const std::vector<fs_program::Step>& steps) {
  std::vector<int> owner(g.ops.size(), -1);
  for (size_t s = 0; s < steps.size(); ++s)
    for (int o : steps[s].ops) owner[o] = (int)s;
  return owner;
}

// Dependence order: a pattern runs after every pattern that makes one of its operands.  False if none exists.
bool order_steps(const fs_graph& g, std::vector<fs_program::Step>* steps) {
  std::stable_sort(steps->begin(), steps->end(),
                   [](const fs_program::Step& a, const fs_program::Step& b) { return a.ops.back() < b.ops.back(); });
  const std::vector<int> owner = owners(g, *steps);
  const std::vector<std::vector<int>> waits_for = g.external_producers();
  const size_t ns = steps->size();
  std::vector<std::set<int>> deps(ns), across(ns);   // steps it reads from; steps it waits for through external computations
  for (size_t s = 0; s < ns; ++s)
    for (int o : (*steps)[s].ops) {
      for (int k = 0; k < g.ops[o].n_in; ++k) {
        const int32_t prod = g.tensors[g.ops[o].in[k]].producer;
        if (prod >= 0 && owner[prod] != (int)s) deps[s].insert(owner[prod]);
      }
      for (int prod : waits_for[o]) {
        if (owner[prod] == (int)s) return false;   // cannot happen: such a pattern has no score
        deps[s].insert(owner[prod]);
        across[s].insert(owner[prod]);
      }
    }
  std::vector<int> order;
  std::vector<char> done(ns, 0);
  while (order.size() < ns) {
    bool progressed = false;
    for (size_t s = 0; s < ns; ++s) {
      if (done[s]) continue;
      bool ready = true;
      for (int d : deps[s])
        if (!done[d]) ready = false;
      if (ready) { done[s] = 1; order.push_back((int)s); progressed = true; }
    }
    if (!progressed) return false;
  }
  // stages: a step runs in the stage after the latest one it waits for across an external computation, and never
  // before a step it reads from; the steps are issued stage by stage
  for (int s : order) {
    int32_t stage = 0;
    for (int d : deps[s]) stage = std::max(stage, (*steps)[d].stage + (across[s].count(d) ? 1 : 0));
    (*steps)[s].stage = stage;
  }
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return (*steps)[a].stage < (*steps)[b].stage; });
  std::vector<fs_program::Step> sorted;
  for (int s : order) sorted.push_back(std::move((*steps)[s]));
  steps->swap(sorted);
  return true;
}

// Launch-bound patterns with no dependence between them share one packed launch, issued where the first of them
// stands; a member joins only if everything it reads is made before that point (remote fusion as kernel packing).
void decide_packs(const fs_graph& g, fs_program* prog, std::vector<int>* pos) {
  const int ns = (int)prog->steps.size();
  const std::vector<int> owner = owners(g, prog->steps);
  std::vector<int> level(ns, 0);
  for (int s = 0; s < ns; ++s)
    for (int o : prog->steps[s].ops)
      for (int k = 0; k < g.ops[o].n_in; ++k) {
        const int32_t prod = g.tensors[g.ops[o].in[k]].producer;
        if (prod >= 0 && owner[prod] != s) level[s] = std::max(level[s], level[owner[prod]] + 1);
      }
  const double tiny_us = 3.0 * device().launch_s * 1e6;   // the launch is a third or more of the pattern's estimated time
  std::map<std::pair<int, int>, std::vector<int>> by_level;   // (stage, level): members of a pack are issued together
  for (int s = 0; s < ns; ++s) {
    const fs_plan* p = prog->steps[s].plan;
    if ((p->pack.spec >= 0 || p->generic.valid) && p->candidates[p->chosen].info.predicted_us <= tiny_us)
      by_level[{prog->steps[s].stage, level[s]}].push_back(s);
  }
  for (auto& kv : by_level) {
    if (kv.second.size() < 2) continue;
    std::vector<const fs_plan*> members;
    std::vector<int> chosen;
    const int first = kv.second.front();
    for (int s : kv.second) {
      bool ready = true;
      for (const BufRef& r : prog->steps[s].in) {
        const int32_t prod = g.tensors[r.slot].producer;
        if (prod >= 0 && owner[prod] >= first) ready = false;
      }
      if (ready) { members.push_back(prog->steps[s].plan); chosen.push_back(s); }
    }
    if (members.size() < 2 || members.size() > FS_PACK_MAX_MEMBERS) continue;
    fs_program::Pack pk;
    if (fs_pack_create(members.data(), (int32_t)members.size(), &pk.pack) != FS_OK) continue;
    pk.steps = chosen;
    for (int s : chosen) {
      prog->steps[s].pack = (int32_t)prog->packs.size();
      (*pos)[s] = first;
    }
    prog->packs.push_back(pk);
  }
  clear_error();
}

// Where tensors that cross patterns live: placed by lifetime, from the position their maker runs at to the position
// of their last reader; then every buffer reference of every step is resolved to a graph input, a graph output or
// a workspace offset.  Returns the workspace size.
int64_t place_buffers(const fs_graph& g, fs_program* prog, const std::vector<int>& pos) {
  const int ns = (int)prog->steps.size();
  std::map<int32_t, int> last_read;
  for (int s = 0; s < ns; ++s)
    for (const BufRef& r : prog->steps[s].in) {
      const int at = std::max(pos[s], s);
      auto it = last_read.find(r.slot);
      if (it == last_read.end() || it->second < at) last_read[r.slot] = at;
    }
  int64_t fixed = 0;   // the plans' own workspaces: never shared, so partial sums wait there untouched until the joint fold at the end
  for (int s = 0; s < ns; ++s) {
    const int64_t need = prog->steps[s].plan->candidates[prog->steps[s].plan->chosen].info.workspace_bytes;
    prog->steps[s].plan_ws_offset = fixed;
    fixed += align256(need);
  }
  Arena arena;
  std::map<int32_t, int64_t> where;
  for (int s = 0; s < ns; ++s)
    for (const BufRef& r : prog->steps[s].out) {
      const Tensor& T = g.tensors[r.slot];
      if (T.output_slot >= 0) continue;
      const int begin = pos[s];
      const int end = std::max(begin, last_read.count(r.slot) ? last_read[r.slot] : begin);
      where[r.slot] = fixed + arena.place(T.numel() * dtype_bytes(T.dtype), begin, end);
    }
  auto resolve = [&](BufRef* r) {
    const Tensor& T = g.tensors[r->slot];
    if (T.producer < 0) { r->kind = BUF_INPUT; r->slot = T.input_slot; }
    else if (T.output_slot >= 0) { r->kind = BUF_OUTPUT; r->slot = T.output_slot; }
    else { r->kind = BUF_WORKSPACE; r->offset = where[r->slot]; r->slot = 0; }
  };
  for (fs_program::Step& s : prog->steps) {
    for (BufRef& r : s.in) resolve(&r);
    for (BufRef& r : s.out) resolve(&r);
  }
  return fixed + arena.top;
}

// Column sums that nothing in the graph reads are finished by fold launches that only need to run before the
// program ends: instead of one tiny launch (or two) after each pattern, all of them run as one launch after the
// last step.  The plans' own workspaces, where the partial sums wait, are never shared between steps.
void join_folds(const fs_graph& g, fs_program* prog) {
  std::vector<fs_program::JointFold> found;
  for (size_t si = 0; si < prog->steps.size(); ++si) {
    fs_program::Step& s = prog->steps[si];
    const std::vector<Launch>& launches = s.plan->candidates[s.plan->chosen].launches;
    s.own_launches = launches.size();
    if (s.pack >= 0) continue;
    size_t first = launches.size();
    while (first > 1 && launches[first - 1].kernel == K_COLFOLD) {
      bool free_standing = true;
      for (int k = 0; k < 3; ++k) {
        const BufRef& r = launches[first - 1].ptr[k];
        if (r.kind != BUF_OUTPUT) continue;
        const int32_t t = s.out[r.slot].slot;
        const Tensor& T = g.tensors[t];
        if (T.output_slot < 0 || !T.consumers.empty()) free_standing = false;
        for (const std::pair<int32_t, int32_t>& e : g.external)
          if (e.first == t) free_standing = false;   // an external computation reads it before the program ends
      }
      if (!free_standing) break;
      --first;
    }
    for (size_t l = first; l < launches.size(); ++l) found.push_back({(int)si, l});
  }
  if (found.size() < 2) return;   // one fold alone gains nothing by moving
  for (const fs_program::JointFold& f : found) {
    fs_program::Step& s = prog->steps[f.step];
    s.own_launches = std::min(s.own_launches, f.launch);
    if (prog->joint_folds.empty() || prog->joint_folds.back().size() >= (size_t)kFoldManyMax) prog->joint_folds.emplace_back();
    prog->joint_folds.back().push_back(f);
  }
}

void fill_info(const Explorer& ex, fs_program* prog, int32_t beam_plans, double f_total_us, int64_t workspace_bytes) {
  fs_program_info& I = prog->info;
  I.n_ops = ex.n;
  I.beam_plans = beam_plans;
  I.workspace_bytes = workspace_bytes;
  I.bytes_min = graph_bytes_min(ex.g);
  I.f_total_us = f_total_us;
  std::set<int> counted_packs;
  for (const fs_program::Step& s : prog->steps) {
    const fs_plan_info& pi = s.plan->candidates[s.plan->chosen].info;
    if (s.ops.size() > 1) ++I.n_patterns; else ++I.n_single_ops;
    I.bytes_moved_model += pi.bytes_moved_model;
    if (s.pack >= 0) {
      if (counted_packs.insert(s.pack).second) {
        I.n_kernels += prog->packs[s.pack].pack->info.n_kernels;
        I.predicted_us += prog->packs[s.pack].pack->info.predicted_us;
        ++I.n_steps;
      }
    } else {
      I.n_kernels += pi.n_kernels;
      I.predicted_us += pi.predicted_us;
      ++I.n_steps;
    }
  }
  // joint folds: the steps they come from no longer issue a fold launch of their own; the estimate keeps the folds'
  // own times and drops the launches they no longer pay for
  int moved_from = 0;
  for (const fs_program::Step& s : prog->steps)
    if (s.pack < 0 && s.own_launches < s.plan->candidates[s.plan->chosen].launches.size()) ++moved_from;
  for (const std::vector<fs_program::JointFold>& j : prog->joint_folds) I.n_joint_folds += (int32_t)j.size();
  I.n_kernels += (int32_t)prog->joint_folds.size() - moved_from;
  I.predicted_us -= (double)(moved_from - (int)prog->joint_folds.size()) * device().launch_s * 1e6;
  I.n_packs = (int32_t)prog->packs.size();
  I.n_stages = 1;
  for (const fs_program::Step& s : prog->steps) I.n_stages = std::max(I.n_stages, s.stage + 1);
  for (int o = 0; o < ex.n; ++o) I.predicted_unfused_us += ex.t_single(o) * 1e6;
}

}  // namespace

extern "C" {

fs_status fs_explore_score(const fs_graph* g, const int32_t* ops, int32_t n, double* f_us, double* f_optimistic_us) try {
  clear_error();
  if (!g || !ops || !f_us) return fail(FS_ERR_INVALID_ARG, "fs_explore_score: null argument");
  if (!g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_explore_score: graph is not finalized");
  if (n < 1) return fail(FS_ERR_INVALID_ARG, "fs_explore_score: empty pattern");
  OpSet p(ops, ops + n);
  std::sort(p.begin(), p.end());
  if (std::adjacent_find(p.begin(), p.end()) != p.end() || p.front() < 0 || p.back() >= (int)g->ops.size())
    return fail(FS_ERR_INVALID_ARG, "fs_explore_score: op indices must be distinct and inside the graph");
  Explorer ex(*g);
  const Scored& s = ex.score(p);
  if (f_optimistic_us) *f_optimistic_us = s.f_optimistic;
  if (!s.valid) {
    if (s.why == FS_ERR_CYCLE) return fail(FS_ERR_CYCLE, "fs_explore_score: fusing these ops creates a cyclic dependence");
    if (s.why == FS_ERR_DTYPE)
      return fail(FS_ERR_DTYPE, "fs_explore_score: a tensor stored in another dtype than it was computed in crosses the pattern boundary");
    return fail(FS_ERR_UNSUPPORTED_PATTERN, "fs_explore_score: no stitched kernel can run these ops as one pattern");
  }
  *f_us = s.f;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_explore_score");
}

fs_status fs_explore(const fs_graph* g, const fs_explore_opts* opts, fs_program** out) try {
  clear_error();
  if (!g || !out) return fail(FS_ERR_INVALID_ARG, "fs_explore: null argument");
  if (!g->finalized) return fail(FS_ERR_INVALID_ARG, "fs_explore: graph is not finalized");
  Explorer ex(*g);
  bool pack_tiny = true, remote_fusion = true, joint_folds = true;
  if (opts) {
    if (opts->top_k < 0 || opts->beam_width < 0 || opts->top_k > 16 || opts->beam_width > 16)
      return fail(FS_ERR_INVALID_ARG, "fs_explore: top_k and beam_width must be 0 (default 3) or 1..16");
    if (opts->top_k > 0) ex.top_k = opts->top_k;
    if (opts->beam_width > 0) ex.beam_width = opts->beam_width;
    pack_tiny = opts->no_packing == 0;
    remote_fusion = opts->no_remote_fusion == 0;
    joint_folds = opts->no_joint_folds == 0;
  }
  ex.explore_patterns();
  const std::vector<Explorer::PlanSet> plans = ex.beam();

  // Final choice among the beam's plans by the full latency evaluator (Section 5.3): every pattern, and every op
  // left alone, is planned for real and the predicted times are added up.
  std::vector<BuiltPlan> built(plans.size());
  fs_status first_error = FS_OK;
  std::string first_text;
  for (size_t k = 0; k < plans.size(); ++k) {
    std::string text;
    const fs_status st = build_steps(&ex, plans[k], remote_fusion, &built[k], &text);
    if (st != FS_OK && first_error == FS_OK) { first_error = st; first_text = text; }
  }
  int best = -1;
  for (size_t k = 0; k < built.size(); ++k)
    if (built[k].ok && (best < 0 || built[k].predicted < built[best].predicted)) best = (int)k;
  for (size_t k = 0; k < built.size(); ++k)
    if ((int)k != best) built[k].destroy();
  if (best < 0) return fail(first_error != FS_OK ? first_error : FS_ERR_UNSUPPORTED_PATTERN, "fs_explore: %s", first_text.c_str());

  for (fs_program::Step& s : built[best].steps) {
    fs_status st = complete_plan(s.plan);
    if (st == FS_ERR_UNSUPPORTED_PATTERN) {
      // the pattern's only stitched form was a generated kernel that did not compile: it runs per op instead
      SubGraph sub;
      fs_plan* per_op = nullptr;
      st = ex.extract(s.ops, &sub);
      if (st == FS_OK) st = create_plan(sub.g, FS_SCHEME_UNFUSED, nullptr, true, &per_op);
      if (st == FS_OK) {
        fs_plan_destroy(s.plan);
        s.plan = per_op;
      }
    }
    if (st != FS_OK) {
      built[best].destroy();
      return st;
    }
  }
  fs_program* prog = new (std::nothrow) fs_program();
  if (!prog) { built[best].destroy(); return fail(FS_ERR_INVALID_ARG, "fs_explore: out of host memory"); }
  if (!order_steps(*g, &built[best].steps)) {   // cannot happen for convex patterns
    delete prog;
    built[best].destroy();
    return fail(FS_ERR_CYCLE, "fs_explore: the chosen patterns depend on each other cyclically");
  }
  prog->steps = std::move(built[best].steps);
  built[best].steps.clear();
  std::vector<int> pos(prog->steps.size());   // where in the order a step's kernel is issued (packed members: at the first member)
  for (size_t s = 0; s < pos.size(); ++s) pos[s] = (int)s;
  if (pack_tiny) decide_packs(*g, prog, &pos);
  for (fs_program::Step& s : prog->steps) s.own_launches = s.plan->candidates[s.plan->chosen].launches.size();
  if (joint_folds) join_folds(*g, prog);
  const int64_t workspace = place_buffers(*g, prog, pos);
  fill_info(ex, prog, (int32_t)plans.size(), built[best].f, workspace);
  prog->n_inputs = (int32_t)g->inputs.size();
  prog->n_outputs = (int32_t)g->outputs.size();
  *out = prog;
  return FS_OK;
} catch (...) {
  return fs::fail_caught("fs_explore");
}

}  // extern "C"
