// Prefix index for probabilistic prefix deduplication (Sec. 7.3, "Trie-Based Prefix Index"): a trie over
// token sequences with insert, best-match lookup and evict, each linear in the prefix length.  A host-side
// structure (plain C++, no device code); see include/plc.h for the interface and the readings taken.
#include <cstdint>
#include <new>
#include <unordered_map>
#include <vector>

#include "plc.h"

namespace {

struct Node {
  int32_t parent = -1;
  int32_t token = 0;
  float bits = 0.0f;        // surprisal of `token` given the path above it
  int64_t id = -1;          // stored prefix that ends here, or -1
  int64_t below = 0;        // stored prefixes in this subtree (this node included)
  std::unordered_map<int32_t, int32_t> child;
};

}  // namespace

struct plc_trie {
  std::vector<Node> nodes;
  std::vector<int32_t> free_list;
  std::unordered_map<int64_t, int32_t> where;  // id -> node
  double max_bits;

  int32_t make(int32_t parent, int32_t token, float bits) {
    int32_t n;
    if (!free_list.empty()) {
      n = free_list.back();
      free_list.pop_back();
      nodes[n] = Node();
    } else {
      n = (int32_t)nodes.size();
      nodes.emplace_back();
    }
    nodes[n].parent = parent;
    nodes[n].token = token;
    nodes[n].bits = bits;
    return n;
  }
};

extern "C" plc_trie *plc_trie_create(double max_bits) {
  if (!(max_bits > 0.0)) return nullptr;
  plc_trie *t = new (std::nothrow) plc_trie();
  if (!t) return nullptr;
  t->max_bits = max_bits;
  t->nodes.emplace_back();  // the root: the empty prefix
  return t;
}

extern "C" void plc_trie_destroy(plc_trie *t) { delete t; }

extern "C" int64_t plc_trie_size(const plc_trie *t) { return t ? (int64_t)t->where.size() : -1; }

extern "C" int64_t plc_trie_nodes(const plc_trie *t) {
  return t ? (int64_t)(t->nodes.size() - t->free_list.size()) : -1;
}

extern "C" int plc_trie_insert(plc_trie *t, const int32_t *tokens, const float *bits, int64_t n, int64_t id,
                               int64_t *stored_len) {
  if (!t || n < 0 || (n > 0 && !tokens) || id < 0 || t->where.count(id)) return PLC_ERR_INVALID;
  // the stored path ends where the prefix's probability would fall below the threshold
  int64_t keep = 0;
  double total = 0.0;
  for (; keep < n; ++keep) {
    const double b = bits ? (double)bits[keep] : 0.0;
    if (!(b >= 0.0)) return PLC_ERR_INVALID;  // negative or NaN
    if (total + b > t->max_bits) break;
    total += b;
  }
  int32_t at = 0;
  for (int64_t i = 0; i < keep; ++i) {
    auto it = t->nodes[at].child.find(tokens[i]);
    int32_t next;
    if (it == t->nodes[at].child.end()) {
      next = t->make(at, tokens[i], bits ? bits[i] : 0.0f);
      t->nodes[at].child.emplace(tokens[i], next);
    } else {
      next = it->second;
    }
    at = next;
  }
  if (t->nodes[at].id >= 0) {  // another stored prefix already ends at this node: the two are the same entry
    if (stored_len) *stored_len = keep;
    return PLC_ERR_CAPACITY;
  }
  t->nodes[at].id = id;
  t->where.emplace(id, at);
  for (int32_t a = at; a >= 0; a = t->nodes[a].parent) t->nodes[a].below += 1;
  if (stored_len) *stored_len = keep;
  return PLC_OK;
}

extern "C" int plc_trie_best_match(const plc_trie *t, const int32_t *tokens, int64_t n, int64_t *id, int64_t *lcp,
                                   double *dist) {
  if (!t || n < 0 || (n > 0 && !tokens) || !id || !lcp || !dist) return PLC_ERR_INVALID;
  *id = -1;
  *lcp = 0;
  *dist = 0.0;
  if (t->nodes[0].below == 0) return PLC_OK;  // nothing stored
  int32_t at = 0;
  int64_t depth = 0;
  double total = 0.0;
  while (depth < n) {  // follow the query while stored paths go the same way
    auto it = t->nodes[at].child.find(tokens[depth]);
    if (it == t->nodes[at].child.end()) break;
    at = it->second;
    total += (double)t->nodes[at].bits;
    ++depth;
  }
  *lcp = depth;
  *dist = total;
  // a stored prefix through this node: the one ending here, else the first one found below
  int32_t down = at;
  while (t->nodes[down].id < 0) {
    int32_t next = -1;
    for (const auto &kv : t->nodes[down].child)
      if (t->nodes[kv.second].below > 0) {
        next = kv.second;
        break;
      }
    if (next < 0) return PLC_ERR_CORRUPT;  // cannot happen: every kept node has a stored prefix below it
    down = next;
  }
  *id = t->nodes[down].id;
  return PLC_OK;
}

extern "C" int plc_trie_evict(plc_trie *t, int64_t id) {
  if (!t) return PLC_ERR_INVALID;
  auto it = t->where.find(id);
  if (it == t->where.end()) return PLC_ERR_INVALID;
  int32_t at = it->second;
  t->where.erase(it);
  t->nodes[at].id = -1;
  for (int32_t a = at; a >= 0; a = t->nodes[a].parent) t->nodes[a].below -= 1;
  // prune the nodes that no stored prefix passes through any more
  while (at > 0 && t->nodes[at].below == 0) {
    const int32_t parent = t->nodes[at].parent;
    t->nodes[parent].child.erase(t->nodes[at].token);
    t->nodes[at].child.clear();
    t->free_list.push_back(at);
    at = parent;
  }
  return PLC_OK;
}
