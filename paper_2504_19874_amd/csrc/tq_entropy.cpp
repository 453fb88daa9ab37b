// Entropy coding of the codebook indices (Sec. 3.1, last paragraph): the
// probability p_l of index l is the mass of the coordinate law in its Voronoi
// cell; an optimal prefix code for {p_l} brings the average bit-width close to
// the entropy of that distribution (about 5 % below b at b = 4).  The paper
// leaves the technique out of the method; here it is an optional host-side
// codec for stored codes: Huffman lengths, canonical codewords, and a bit
// stream of one codeword per coordinate (most significant bit first, the
// coordinates of a vector in order, vectors back to back, with the bit offset
// of every vector returned so that any one vector can be decoded alone).
#include <cstring>
#include <vector>

#include "../../include/turboquant.h"

namespace {

struct Canonical {
  int max_len;
  uint32_t first_code[34];  // first codeword of each length
  int first_rank[34];       // rank (in (length, symbol) order) of that codeword
  int count[34];
  std::vector<int> by_rank;  // symbols in (length, symbol) order
};

bool make_canonical(int K, const uint8_t* lengths, Canonical* c) {
  c->max_len = 0;
  std::memset(c->count, 0, sizeof(c->count));
  for (int s = 0; s < K; ++s) {
    if (lengths[s] > 32 || (lengths[s] == 0 && K > 1)) return false;
    c->count[lengths[s]]++;
    if (lengths[s] > c->max_len) c->max_len = lengths[s];
  }
  c->by_rank.clear();
  for (int len = 0; len <= c->max_len; ++len)
    for (int s = 0; s < K; ++s)
      if (lengths[s] == len) c->by_rank.push_back(s);
  uint64_t code = 0;
  int rank = 0;
  for (int len = 1; len <= c->max_len; ++len) {
    code <<= 1;
    c->first_code[len] = (uint32_t)code;
    c->first_rank[len] = rank;
    code += (uint64_t)c->count[len];
    rank += c->count[len];
    if (code > ((uint64_t)1 << len)) return false;  // more codewords than the length holds
  }
  return true;
}

inline int index_of(const uint32_t* words, int bits, int j) {
  const uint32_t* g = words + (size_t)(j >> 5) * bits;
  int v = 0;
  for (int p = 0; p < bits; ++p) v |= (int)((g[p] >> (j & 31)) & 1u) << p;
  return v;
}

}  // namespace

extern "C" {

tq_status tq_prefix_code_build(int32_t K, const double* p, uint8_t* lengths, uint32_t* codewords, double* mean_bits) {
  if (K < 1 || K > 256 || p == nullptr || lengths == nullptr || codewords == nullptr) return TQ_ERR_INVALID_ARG;
  for (int s = 0; s < K; ++s)
    if (!(p[s] >= 0.0)) return TQ_ERR_INVALID_ARG;
  std::vector<int> len((size_t)K, 0);
  if (K > 1) {
    // Huffman: merge the two least probable nodes until one is left; ties go to the older node
    struct Node {
      double w;
      int age;
      std::vector<int> leaves;
    };
    std::vector<Node> nodes;
    for (int s = 0; s < K; ++s) nodes.push_back(Node{p[s], s, {s}});
    int age = K;
    while (nodes.size() > 1) {
      size_t a = 0, b = 1;
      auto less = [&](size_t x, size_t y) {
        return nodes[x].w < nodes[y].w || (nodes[x].w == nodes[y].w && nodes[x].age < nodes[y].age);
      };
      if (less(b, a)) std::swap(a, b);
      for (size_t i = 2; i < nodes.size(); ++i) {
        if (less(i, a)) {
          b = a;
          a = i;
        } else if (less(i, b)) {
          b = i;
        }
      }
      Node m{nodes[a].w + nodes[b].w, age++, nodes[a].leaves};
      m.leaves.insert(m.leaves.end(), nodes[b].leaves.begin(), nodes[b].leaves.end());
      for (int s : m.leaves) len[(size_t)s]++;
      const size_t hi = a > b ? a : b, lo = a > b ? b : a;
      nodes.erase(nodes.begin() + (long)hi);
      nodes.erase(nodes.begin() + (long)lo);
      nodes.push_back(std::move(m));
    }
  }
  double mean = 0.0;
  for (int s = 0; s < K; ++s) {
    if (len[(size_t)s] > 32) return TQ_ERR_UNSUPPORTED;  // codewords are kept in 32 bits
    lengths[s] = (uint8_t)len[(size_t)s];
    mean += p[s] * len[(size_t)s];
  }
  Canonical c;
  if (!make_canonical(K, lengths, &c)) return TQ_ERR_UNSUPPORTED;
  for (int len_i = 1, rank = 0; len_i <= c.max_len; ++len_i)
    for (int k = 0; k < c.count[len_i]; ++k, ++rank) codewords[c.by_rank[(size_t)(c.count[0] + rank)]] = c.first_code[len_i] + (uint32_t)k;
  if (K == 1) codewords[0] = 0;
  if (mean_bits != nullptr) *mean_bits = mean;
  return TQ_OK;
}

tq_status tq_entropy_encode(int32_t d, int32_t bits, const uint8_t* lengths, const uint32_t* codewords,
                            const uint32_t* idx, int64_t n, uint8_t* out, size_t out_capacity, size_t* out_bytes,
                            uint64_t* row_bit_offsets) {
  if (d <= 0 || bits < 1 || bits > 8 || n < 0 || lengths == nullptr || codewords == nullptr || out_bytes == nullptr)
    return TQ_ERR_INVALID_ARG;
  if (d % 32 != 0) return TQ_ERR_UNSUPPORTED;
  if (n > 0 && (idx == nullptr || (out == nullptr && out_capacity > 0))) return TQ_ERR_INVALID_ARG;
  const int K = 1 << bits;
  for (int s = 0; s < K; ++s)
    if (lengths[s] < 1 || lengths[s] > 32) return TQ_ERR_INVALID_ARG;
  const size_t words = (size_t)(d / 32) * bits;
  uint64_t pos = 0;  // bits written
  uint64_t acc = 0;  // bits not yet stored, right-aligned
  int held = 0;
  size_t at = 0;
  for (int64_t i = 0; i < n; ++i) {
    if (row_bit_offsets != nullptr) row_bit_offsets[i] = pos;
    const uint32_t* row = idx + (size_t)i * words;
    for (int j = 0; j < d; ++j) {
      const int v = index_of(row, bits, j);
      acc = (acc << lengths[v]) | codewords[v];
      held += lengths[v];
      pos += lengths[v];
      while (held >= 8) {
        if (at >= out_capacity) return TQ_ERR_WORKSPACE;
        out[at++] = (uint8_t)(acc >> (held - 8));
        held -= 8;
      }
    }
  }
  if (held > 0) {
    if (at >= out_capacity) return TQ_ERR_WORKSPACE;
    out[at++] = (uint8_t)(acc << (8 - held));
  }
  if (row_bit_offsets != nullptr) row_bit_offsets[n] = pos;
  *out_bytes = at;
  return TQ_OK;
}

tq_status tq_entropy_decode(int32_t d, int32_t bits, const uint8_t* lengths, const uint8_t* in, size_t in_bytes,
                            uint64_t first_bit, int64_t n, uint32_t* idx) {
  if (d <= 0 || bits < 1 || bits > 8 || n < 0 || lengths == nullptr) return TQ_ERR_INVALID_ARG;
  if (d % 32 != 0) return TQ_ERR_UNSUPPORTED;
  if (n > 0 && (in == nullptr || idx == nullptr)) return TQ_ERR_INVALID_ARG;
  const int K = 1 << bits;
  Canonical c;
  if (!make_canonical(K, lengths, &c) || c.count[0] != 0) return TQ_ERR_INVALID_ARG;
  const size_t words = (size_t)(d / 32) * bits;
  uint64_t pos = first_bit;
  const uint64_t end = (uint64_t)in_bytes * 8;
  for (int64_t i = 0; i < n; ++i) {
    uint32_t* row = idx + (size_t)i * words;
    std::memset(row, 0, words * sizeof(uint32_t));
    for (int j = 0; j < d; ++j) {
      uint32_t code = 0;
      int len = 0, sym = -1;
      while (sym < 0) {
        if (pos >= end || len >= c.max_len) return TQ_ERR_INVALID_ARG;  // truncated or not a stream of this code
        code = (code << 1) | ((in[pos >> 3] >> (7 - (pos & 7))) & 1u);
        ++pos;
        ++len;
        const uint32_t off = code - c.first_code[len];
        if (code >= c.first_code[len] && off < (uint32_t)c.count[len]) sym = c.by_rank[(size_t)(c.first_rank[len] + (int)off)];
      }
      uint32_t* g = row + (size_t)(j >> 5) * bits;
      for (int p = 0; p < bits; ++p) g[p] |= (uint32_t)((sym >> p) & 1) << (j & 31);
    }
  }
  return TQ_OK;
}

}  // extern "C"
