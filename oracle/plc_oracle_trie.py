"""CPU oracle for the prefix index (Sec. 7.3, "Trie-Based Prefix Index").

TEST INFRASTRUCTURE ONLY.  No trie here: the stored prefixes are kept in a plain list and every
operation is the definition written out -- best match = the stored prefix with the longest common
prefix with the query, by comparing against all of them; d_T = -log2 P(common prefix) = the sum of
the per-token surprisals along it (Def. "PLT trie metric"); a prefix is stored only down to the last
token at which its surprisal sum stays within max_bits (the probability threshold of Sec. 7.3).
Where several stored prefixes share the longest common prefix, all of them are correct answers; the
oracle returns the whole set."""
from __future__ import annotations


class PrefixIndexOracle:
    def __init__(self, max_bits=float("inf")):
        self.max_bits = float(max_bits)
        self.stored = {}           # id -> (tokens kept, their bits)

    def kept_length(self, tokens, bits=None):
        total, keep = 0.0, 0
        for i in range(len(tokens)):
            b = 0.0 if bits is None else float(bits[i])
            if total + b > self.max_bits:
                break
            total += b
            keep += 1
        return keep

    def insert(self, tokens, ident, bits=None):
        """Returns the kept length, or None if an identical kept prefix is already stored."""
        keep = self.kept_length(tokens, bits)
        kept = tuple(int(t) for t in tokens[:keep])
        if ident in self.stored or any(k == kept for k, _ in self.stored.values()):
            return None
        kb = tuple(0.0 if bits is None else float(b) for b in (bits[:keep] if bits is not None else [0.0] * keep))
        self.stored[ident] = (kept, kb)
        return keep

    def evict(self, ident):
        del self.stored[ident]

    def best_match(self, tokens):
        """(set of ids, lcp, dist); (empty set, 0, 0.0) when nothing is stored."""
        best, ids, dist = -1, set(), 0.0
        for ident, (kept, kb) in self.stored.items():
            lcp = 0
            while lcp < len(kept) and lcp < len(tokens) and kept[lcp] == int(tokens[lcp]):
                lcp += 1
            if lcp > best:
                best, ids, dist = lcp, {ident}, sum(kb[:lcp])
            elif lcp == best:
                ids.add(ident)
        return ids, max(best, 0), dist

    def node_count(self):
        """Nodes of the trie over the kept prefixes, the root included."""
        nodes = {()}
        for kept, _ in self.stored.values():
            for i in range(1, len(kept) + 1):
                nodes.add(kept[:i])
        return len(nodes)
