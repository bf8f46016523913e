#include "fs_match.hpp"

#include <cctype>
#include <cmath>

namespace fs {

namespace {
struct Name { const char* text; int32_t opcode; };
const Name kNames[] = {
    {"add", FS_ADD}, {"sub", FS_SUB}, {"mul", FS_MUL}, {"div", FS_DIV}, {"max", FS_MAX},
    {"scale", FS_SCALE}, {"addc", FS_ADD_SCALAR}, {"square", FS_SQUARE}, {"exp", FS_EXP},
    {"rsqrt", FS_RSQRT}, {"tanh", FS_TANH}, {"gelu", FS_GELU_TANH}, {"gelugrad", FS_GELU_TANH_GRAD},
    {"bcast", FS_BROADCAST}, {"rsum", FS_REDUCE_SUM}, {"rmax", FS_REDUCE_MAX}, {"rmean", FS_REDUCE_MEAN},
    {"tr", FS_TRANSPOSE}, {"cvt", FS_CONVERT}, {"log", FS_LOG}, {"sigmoid", FS_SIGMOID}, {"relu", FS_RELU}, {"abs", FS_ABS},
    {"sqrt", FS_SQRT},
};
int32_t opcode_of(const std::string& s) {
  for (const Name& n : kNames)
    if (s == n.text) return n.opcode;
  return -1;
}
bool commutative(int32_t opc) { return opc == FS_ADD || opc == FS_MUL || opc == FS_MAX; }
}  // namespace

Pattern::Pattern(const std::string& text) {
  size_t pos = 0;
  root_ = parse(text, &pos);
  if (pos != text.size()) root_ = -1;
}

int Pattern::parse(const std::string& s, size_t* pos) {
  size_t& i = *pos;
  if (i >= s.size()) return -1;
  Node n;
  if (s[i] == '$') {
    size_t j = ++i;
    while (j < s.size() && (isalnum((unsigned char)s[j]) || s[j] == '_')) ++j;
    n.is_var = true;
    n.var = s.substr(i, j - i);
    i = j;
    nodes_.push_back(n);
    return (int)nodes_.size() - 1;
  }
  size_t j = i;
  while (j < s.size() && isalpha((unsigned char)s[j])) ++j;
  n.opcode = opcode_of(s.substr(i, j - i));
  if (n.opcode < 0) return -1;
  i = j;
  if (i < s.size() && s[i] == '[') {
    ++i;
    size_t e = s.find(']', i);
    if (e == std::string::npos) return -1;
    const std::string a = s.substr(i, e - i);
    if (!a.empty() && a[0] == '#') n.scalar_var = atoi(a.c_str() + 1);
    else if (!a.empty() && a[0] == '-') { n.has_axis = true; n.axis_from_end = atoi(a.c_str()); }
    else for (char c : a) n.perm.push_back(c - '0');
    i = e + 1;
  }
  if (i >= s.size() || s[i] != '(') return -1;
  ++i;
  for (;;) {
    const int c = parse(s, pos);
    if (c < 0 || n.n_child >= 2) return -1;
    n.child[n.n_child++] = c;
    if (i < s.size() && s[i] == ',') { ++i; continue; }
    break;
  }
  if (i >= s.size() || s[i] != ')') return -1;
  ++i;
  nodes_.push_back(n);
  return (int)nodes_.size() - 1;
}

bool Pattern::match(const fs_graph& g, int32_t t, MatchState* st) const {
  if (root_ < 0) return false;
  MatchState trial = *st;
  if (!match_node(g, root_, t, &trial)) return false;
  *st = trial;
  return true;
}

bool Pattern::match_node(const fs_graph& g, int node, int32_t t, MatchState* st) const {
  const Node& n = nodes_[node];
  if (n.is_var) {
    auto it = st->tensors.find(n.var);
    if (it != st->tensors.end()) return it->second == t;
    st->tensors[n.var] = t;
    return true;
  }
  const Tensor& x = g.tensors[t];
  if (x.producer < 0) return false;
  const Op& op = g.ops[x.producer];
  if (op.opcode != n.opcode || op.n_in != n.n_child) return false;
  if (n.has_axis && op.axis - g.tensors[op.in[0]].rank != n.axis_from_end) return false;
  if (!n.perm.empty()) {
    const int rank = g.tensors[op.in[0]].rank;
    if ((int)n.perm.size() != rank) return false;
    for (int k = 0; k < rank; ++k)
      if (op.perm[k] != n.perm[k]) return false;
  }
  if (n.scalar_var >= 0) {
    auto it = st->scalars.find(n.scalar_var);
    if (it != st->scalars.end()) { if (it->second != op.scalar) return false; }
    else st->scalars[n.scalar_var] = op.scalar;
  }
  if (op.opcode == FS_CONVERT) st->convert_dtype = op.to_dtype;

  auto try_order = [&](int first, int second) -> bool {
    MatchState trial = *st;
    if (!match_node(g, n.child[0], op.in[first], &trial)) return false;
    if (n.n_child == 2 && !match_node(g, n.child[1], op.in[second], &trial)) return false;
    trial.covered.insert(x.producer);
    *st = trial;
    return true;
  };
  if (try_order(0, 1)) return true;
  if (n.n_child == 2 && commutative(op.opcode) && try_order(1, 0)) return true;
  return false;
}

}  // namespace fs
