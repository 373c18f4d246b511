// Host-side hierarchical sequence partitioner (Sec. 3.1, Alg. 1 and Alg. 2): decides, from the lengths of a global
// batch, which sequences a device runs whole (local zone) and which it shares on a ring (intra-node / inter-node
// zone), i.e. what the attention engine's work list on each device is made of. Pure integer host code.
#include <algorithm>
#include <cstdint>
#include <map>
#include <numeric>
#include <vector>

#include "../../include/zeppelin_attn.h"

namespace {

struct NodeItem {
  int32_t seq;
  int32_t k;  // number of nodes the sequence spans (0: whole sequence placed in this node)
  int32_t m;  // index of this node among them
};

inline int64_t chunk_bound(int64_t len, int64_t c, int64_t G) { return (c * len) / (2 * G); }
// tokens ring rank r of G holds: chunks r and 2G-1-r of 2G equal-length chunks (Sec. 3.2)
inline int32_t ring_share(int64_t len, int64_t G, int64_t r) {
  return (int32_t)((chunk_bound(len, r + 1, G) - chunk_bound(len, r, G)) +
                   (chunk_bound(len, 2 * G - r, G) - chunk_bound(len, 2 * G - 1 - r, G)));
}
// ceil(a * b / den) exactly (the budgets s_avg and c_avg are rationals); an all-zero zone (den = 0) asks for one bucket
inline int64_t ceil_ratio(int64_t a, int64_t b, int64_t den) {
  if (den <= 0) return 1;
  const unsigned __int128 num = (unsigned __int128)a * (unsigned __int128)b;
  return (int64_t)((num + (unsigned __int128)(den - 1)) / (unsigned __int128)den);
}
template <class Load>
int argmin_load(const Load &load) {
  int best = 0;
  for (int i = 1; i < (int)load.size(); i++)
    if (load[i] < load[best]) best = i;
  return best;
}

}  // namespace

extern "C" int zp_partition(const int32_t *lengths, int32_t S, int32_t P, int32_t N, int32_t L, zp_placement *out,
                            int32_t max_out, int32_t *n_out, int32_t *s1_final, int32_t *s0_final) {
  if (!lengths || S < 0 || P < 1 || N < 1 || L < 1 || !out || !n_out) return ZP_EINVAL;
  for (int s = 0; s < S; s++)
    if (lengths[s] < 0) return ZP_EINVAL;
  std::vector<int32_t> order(S);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return lengths[a] > lengths[b]; });

  // ---- Alg. 1: inter-node partitioning. Lower the threshold s1 until every shorter sequence fits a node.
  const int64_t node_cap = (int64_t)P * L;
  int64_t s1 = node_cap;
  std::vector<std::vector<NodeItem>> node_items;
  for (;;) {
    node_items.assign(N, {});
    std::vector<int64_t> load(N, 0);
    // order is descending, so z2 is a prefix
    int split = 0;
    while (split < S && lengths[order[split]] >= s1) split++;
    if (split > 0) {
      int64_t total = 0;
      for (int i = 0; i < split; i++) total += lengths[order[i]];
      for (int i = 0; i < split; i++) {
        const int32_t s = order[i];
        // ceil(|s| / s_avg) with s_avg = total / N
        const int32_t k = (int32_t)std::max<int64_t>(1, std::min<int64_t>(N, ceil_ratio(lengths[s], N, total)));  // an empty sequence still gets a bucket
        std::vector<int> idx(N);
        std::iota(idx.begin(), idx.end(), 0);
        std::stable_sort(idx.begin(), idx.end(), [&](int a, int b) { return load[a] < load[b]; });
        idx.resize(k);
        std::sort(idx.begin(), idx.end());
        for (int m = 0; m < k; m++) {
          node_items[idx[m]].push_back({s, k, m});
          for (int p = 0; p < P; p++) load[idx[m]] += ring_share(lengths[s], (int64_t)k * P, (int64_t)m * P + p);
        }
      }
    }
    bool again = false;
    for (int i = split; i < S; i++) {
      const int32_t s = order[i];
      const int n = argmin_load(load);
      if (lengths[s] + load[n] > node_cap) {
        s1 = lengths[order[split]];  // the longest sequence still below the threshold joins the inter-node zone
        again = true;
        break;
      }
      node_items[n].push_back({s, 0, 0});
      load[n] += lengths[s];
    }
    if (!again) break;
  }
  if (s1_final) *s1_final = (int32_t)std::min<int64_t>(s1, INT32_MAX);

  // ---- Alg. 2: intra-node partitioning, node by node.
  int32_t n_written = 0;
  auto emit = [&](int32_t seq, int32_t zone, int32_t ring, int32_t rank, int32_t node, int32_t dev, int32_t tokens) {
    if (n_written < max_out) out[n_written] = zp_placement{seq, zone, ring, rank, node, dev, tokens};
    n_written++;
  };
  for (int n = 0; n < N; n++) {
    std::vector<int32_t> whole;  // descending length (node_items keeps the global order)
    for (const NodeItem &it : node_items[n])
      if (it.k == 0) whole.push_back(it.seq);
    int64_t s0 = L;
    std::vector<zp_placement> tmp;
    for (;;) {
      tmp.clear();
      std::vector<int64_t> load(P, 0);
      for (const NodeItem &it : node_items[n]) {
        if (it.k == 0) continue;
        const int64_t G = (int64_t)it.k * P;
        for (int p = 0; p < P; p++) {
          const int32_t t = ring_share(lengths[it.seq], G, (int64_t)it.m * P + p);
          tmp.push_back(zp_placement{it.seq, 2, (int32_t)G, (int32_t)(it.m * P + p), n, p, t});
          load[p] += t;
        }
      }
      int split = 0;  // whole[0 .. split) is z1 (length >= s0), the rest z0
      while (split < (int)whole.size() && lengths[whole[split]] >= s0) split++;
      if (split > 0) {
        // c_avg = c_sum / P, kept as an exact fraction (128 bits: squares of 31-bit lengths, summed)
        unsigned __int128 c_sum = 0;
        for (int i = 0; i < split; i++) c_sum += (unsigned __int128)((int64_t)lengths[whole[i]] * lengths[whole[i]]);
        int64_t next_slot = 0;
        for (int i = 0; i < split; i++) {
          const int32_t s = whole[i];
          // ceil(|s|^2 / c_avg) = ceil(|s|^2 * P / c_sum); at most P anyway, so the quotient is clamped before narrowing
          int64_t G = P;
          if (c_sum > 0) {
            const unsigned __int128 num = (unsigned __int128)((int64_t)lengths[s] * lengths[s]) * (unsigned __int128)P;
            const unsigned __int128 q = (num + c_sum - 1) / c_sum;
            G = q < (unsigned __int128)P ? (int64_t)q : (int64_t)P;
            if (G < 1) G = 1;  // an empty sequence still gets a bucket
          } else {
            G = 1;
          }
          for (int64_t r = 0; r < G; r++) {
            const int p = (int)(next_slot++ % P);
            const int32_t t = G > 1 ? ring_share(lengths[s], G, r) : lengths[s];
            tmp.push_back(zp_placement{s, 1, (int32_t)G, (int32_t)r, n, p, t});
            load[p] += t;
          }
        }
      }
      bool again = false;
      for (int i = split; i < (int)whole.size(); i++) {
        const int32_t s = whole[i];
        const int p = argmin_load(load);
        if (lengths[s] + load[p] > L) {
          s0 = lengths[whole[split]];
          again = true;
          break;
        }
        tmp.push_back(zp_placement{s, 0, 1, 0, n, p, lengths[s]});
        load[p] += lengths[s];
      }
      if (!again) break;
    }
    if (s0_final) s0_final[n] = (int32_t)s0;
    for (const zp_placement &pl : tmp) emit(pl.seq, pl.zone, pl.ring, pl.rank, pl.node, pl.device, pl.tokens);
  }
  *n_out = n_written;
  return n_written > max_out ? ZP_EWORKSPACE : ZP_OK;
}

// The attention layout that a placement list implies, as runs of consecutive tokens: devices in (node, device) order,
// on each device its placements in list order, a whole sequence as one run and ring rank r of G as the two runs
// chunk r and chunk 2G-1-r (Sec. 3.2).
extern "C" int zp_node_segments(const int32_t *lengths, int32_t S, const zp_placement *pl, int32_t n_pl, int32_t P,
                                int32_t N, zp_segment *out, int32_t max_out, int32_t *n_out, int32_t *tokens_per_rank) {
  if (!lengths || !pl || !out || !n_out || S < 0 || n_pl < 0 || P < 1 || N < 1) return ZP_EINVAL;
  for (int i = 0; i < n_pl; i++) {
    const zp_placement &x = pl[i];
    if (x.seq < 0 || x.seq >= S || x.node < 0 || x.node >= N || x.device < 0 || x.device >= P || x.ring < 1 ||
        x.rank < 0 || x.rank >= x.ring || lengths[x.seq] < 0)
      return ZP_EINVAL;
  }
  int32_t n = 0;
  int64_t tok = 0;
  for (int node = 0; node < N; node++)
    for (int dev = 0; dev < P; dev++) {
      const int64_t tok_rank0 = tok;
      for (int i = 0; i < n_pl; i++) {
        const zp_placement &x = pl[i];
        if (x.node != node || x.device != dev) continue;
        const int64_t len = lengths[x.seq], G = x.ring;
        const int n_runs = G == 1 ? 1 : 2;
        for (int k = 0; k < n_runs; k++) {
          const int64_t c = G == 1 ? 0 : (k == 0 ? x.rank : 2 * G - 1 - x.rank);
          const int64_t C = G == 1 ? 1 : 2 * G;
          const int64_t p0 = c * len / C, p1 = (c + 1) * len / C;
          if (n < max_out) {
            zp_segment &sg = out[n];
            sg.seq = x.seq; sg.chunk = (int32_t)c; sg.n_chunks = (int32_t)C;
            sg.pos0 = (int32_t)p0; sg.len = (int32_t)(p1 - p0); sg.tok0 = (int32_t)tok;
            sg.node = node; sg.device = dev;
          }
          n++;
          tok += p1 - p0;
        }
      }
      if (tok > INT32_MAX) return ZP_EINVAL;
      if (tokens_per_rank) tokens_per_rank[node * P + dev] = (int32_t)(tok - tok_rank0);
    }
  *n_out = n;
  return n > max_out ? ZP_EWORKSPACE : ZP_OK;
}

// The runs of one contiguous sequence cut into C equal-length chunks (Sec. 3.2).
extern "C" int zp_chunk_segments(int32_t seq, int32_t tok0, int32_t L, int32_t C, zp_segment *out, int32_t max_out) {
  if (!out || seq < 0 || tok0 < 0 || L < 0 || C < 1 || max_out < C || (int64_t)tok0 + L > INT32_MAX) return ZP_EINVAL;
  for (int32_t c = 0; c < C; c++) {
    const int64_t p0 = (int64_t)c * L / C, p1 = (int64_t)(c + 1) * L / C;
    out[c] = zp_segment{seq, c, C, (int32_t)p0, (int32_t)(p1 - p0), (int32_t)(tok0 + p0), 0, 0};
  }
  return C;
}

// Round t of the ring sequences among the runs: the pairs (qc, qc - t) (Sec. 3.2; grouping by chunk distance keeps
// every query run and every key run single inside a call).
extern "C" int zp_ring_round_pairs(const zp_segment *segs, int32_t n_segs, int32_t round, int32_t include_whole,
                                   zp_pair *pairs, int32_t max_pairs, int32_t *n_pairs, int32_t *n_rounds) {
  if (!segs || n_segs < 0 || round < 0 || !n_pairs || max_pairs < 0 || (max_pairs > 0 && !pairs)) return ZP_EINVAL;
  std::map<int32_t, std::vector<int32_t>> chunks;  // ring sequence -> index of the run of every chunk
  for (int32_t i = 0; i < n_segs; i++) {
    const zp_segment &sg = segs[i];
    if (sg.n_chunks < 1 || sg.chunk < 0 || sg.chunk >= sg.n_chunks || sg.len < 0 || sg.tok0 < 0 || sg.pos0 < 0 || sg.seq < 0)
      return ZP_EINVAL;
    if (sg.n_chunks == 1 && !include_whole) continue;
    auto &v = chunks[sg.seq];
    if (v.empty()) v.assign(sg.n_chunks, -1);
    if ((int32_t)v.size() != sg.n_chunks || v[sg.chunk] != -1) return ZP_EINVAL;
    v[sg.chunk] = i;
  }
  int32_t n = 0, rounds = 0;
  for (const auto &kv : chunks) {
    const std::vector<int32_t> &v = kv.second;
    const int32_t C = (int32_t)v.size();
    for (int32_t c = 0; c < C; c++)
      if (v[c] < 0) return ZP_EINVAL;
    rounds = std::max(rounds, C);
    for (int32_t qc = round; qc < C; qc++) {
      const zp_segment &sq = segs[v[qc]], &sk = segs[v[qc - round]];
      if (n < max_pairs) pairs[n] = zp_pair{sq.tok0, sq.len, sk.tok0, sk.len, sq.pos0, sk.pos0, 0};
      n++;
    }
  }
  *n_pairs = n;
  if (n_rounds) *n_rounds = rounds;
  return n > max_pairs ? ZP_EWORKSPACE : ZP_OK;
}

// Attention-layout token -> token of the batch as drawn.
extern "C" int zp_segment_positions(const int32_t *lengths, int32_t S, const zp_segment *segs, int32_t n_segs,
                                    int64_t *orig, int64_t n_tok) {
  if (!lengths || !segs || S < 0 || n_segs < 0 || n_tok < 0 || (n_tok > 0 && !orig)) return ZP_EINVAL;
  std::vector<int64_t> first(S + 1, 0);
  for (int s = 0; s < S; s++) {
    if (lengths[s] < 0) return ZP_EINVAL;
    first[s + 1] = first[s] + lengths[s];
  }
  std::vector<std::pair<int64_t, int64_t>> cover;
  for (int32_t i = 0; i < n_segs; i++) {
    const zp_segment &sg = segs[i];
    if (sg.seq < 0 || sg.seq >= S || sg.len < 0 || sg.pos0 < 0 || sg.tok0 < 0 || (int64_t)sg.pos0 + sg.len > lengths[sg.seq] ||
        (int64_t)sg.tok0 + sg.len > n_tok)
      return ZP_EINVAL;
    if (sg.len > 0) cover.push_back({sg.tok0, (int64_t)sg.tok0 + sg.len});
  }
  std::sort(cover.begin(), cover.end());
  int64_t at = 0;
  for (const auto &c : cover) {
    if (c.first != at) return ZP_EINVAL;
    at = c.second;
  }
  if (at != n_tok) return ZP_EINVAL;
  for (int32_t i = 0; i < n_segs; i++) {
    const zp_segment &sg = segs[i];
    for (int32_t j = 0; j < sg.len; j++) orig[(int64_t)sg.tok0 + j] = first[sg.seq] + sg.pos0 + j;
  }
  return ZP_OK;
}
