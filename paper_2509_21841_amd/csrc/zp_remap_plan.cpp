// Host-side planner of the remapping layer (Sec. 3.4, Eq. 2): which rank sends how many tokens to which rank when
// the attention layout (A_i tokens on rank i) is turned into the token-balanced layout of the linear modules, and
// the token permutation that goes with it. Pure integer host code.
//
// The objective of Eq. 2 counts, per sender, b_intra per token that stays in the node and b_inter per token that
// leaves it. Row sums are fixed, so a sender's cost is b_intra * s_i + (b_inter - b_intra) * x_i with x_i the tokens
// it sends across nodes. A node has to export exactly its excess E = max(surplus - deficit, 0) (exporting more only
// raises costs), and which remote rank receives a token does not enter the objective. The optimum is therefore found
// node by node: spread E over the node's senders so that the largest cost is smallest (water-filling on integers).
#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/zeppelin_attn.h"

namespace {

void balanced_targets(const int32_t *A, int32_t d, std::vector<int64_t> &B) {
  int64_t T = 0;
  for (int i = 0; i < d; i++) T += A[i];
  B.resize(d);
  for (int i = 0; i < d; i++) B[i] = T / d + (i < T % d ? 1 : 0);
}

// Tokens sender i exports when no sender's cost may exceed `level`: floor((level - base_i) / delta) clamped to [0, s_i].
int64_t exported_at(int64_t level, const std::vector<int64_t> &base, const std::vector<int64_t> &s, int64_t delta,
                    std::vector<int64_t> *x) {
  int64_t sum = 0;
  for (size_t i = 0; i < s.size(); i++) {
    int64_t v = level < base[i] ? 0 : std::min((level - base[i]) / delta, s[i]);
    if (x) (*x)[i] = v;
    sum += v;
  }
  return sum;
}

}  // namespace

extern "C" int zp_remap_plan(const int32_t *A, int32_t d, int32_t P, int32_t b_intra, int32_t b_inter, int32_t *M,
                             int64_t *objective) {
  if (!A || !M || d < 1 || P < 1 || b_intra < 1 || b_inter < b_intra) return ZP_EINVAL;
  for (int i = 0; i < d; i++)
    if (A[i] < 0) return ZP_EINVAL;
  std::vector<int64_t> B;
  balanced_targets(A, d, B);
  std::vector<int64_t> s(d), t(d), x(d, 0);
  for (int i = 0; i < d; i++) {
    s[i] = std::max<int64_t>(A[i] - B[i], 0);
    t[i] = std::max<int64_t>(B[i] - A[i], 0);
  }
  const int64_t delta = (int64_t)b_inter - b_intra;
  const int n_nodes = (d + P - 1) / P;
  for (int n = 0; n < n_nodes; n++) {
    const int lo = n * P, hi = std::min(d, lo + P);
    int64_t S = 0, Dn = 0;
    for (int i = lo; i < hi; i++) { S += s[i]; Dn += t[i]; }
    int64_t E = std::max<int64_t>(S - Dn, 0);
    if (E == 0) continue;
    std::vector<int64_t> sn(s.begin() + lo, s.begin() + hi), base(hi - lo), xn(hi - lo, 0);
    if (delta == 0) {  // crossing nodes costs nothing extra: export in rank order
      for (int i = 0; i < hi - lo && E > 0; i++) { xn[i] = std::min(sn[i], E); E -= xn[i]; }
    } else {
      for (int i = 0; i < hi - lo; i++) base[i] = (int64_t)b_intra * sn[i];
      // smallest cost level at which the senders can export E tokens between them
      int64_t l = 0, h = 0;
      for (int i = 0; i < hi - lo; i++) h = std::max(h, base[i] + delta * sn[i]);
      while (l < h) {
        const int64_t mid = l + (h - l) / 2;
        if (exported_at(mid, base, sn, delta, nullptr) >= E) h = mid; else l = mid + 1;
      }
      int64_t extra = exported_at(l, base, sn, delta, &xn) - E;
      // senders sitting exactly on the level each carry one token too many at most: take them back, highest rank first
      for (int i = hi - lo - 1; i >= 0 && extra > 0; i--)
        if (xn[i] > 0 && base[i] + delta * xn[i] == l) { xn[i]--; extra--; }
      if (extra != 0) return ZP_EINVAL;  // cannot happen: the level is minimal
    }
    for (int i = lo; i < hi; i++) x[i] = xn[i - lo];
  }

  std::fill(M, M + (size_t)d * d, 0);
  std::vector<int64_t> need(t);
  // inside each node: the tokens that stay, senders and receivers both in ascending rank order
  for (int n = 0; n < n_nodes; n++) {
    const int lo = n * P, hi = std::min(d, lo + P);
    int j = lo;
    for (int i = lo; i < hi; i++) {
      int64_t stay = s[i] - x[i];
      while (stay > 0) {
        while (j < hi && need[j] == 0) j++;
        if (j >= hi) return ZP_EINVAL;  // cannot happen: tokens that stay never exceed the node's deficit
        const int64_t m = std::min(stay, need[j]);
        M[(size_t)i * d + j] += (int32_t)m;
        stay -= m; need[j] -= m;
      }
    }
  }
  // across nodes: exported tokens meet the remaining deficits, both in ascending rank order
  {
    int j = 0;
    for (int i = 0; i < d; i++) {
      int64_t out = x[i];
      while (out > 0) {
        while (j < d && need[j] == 0) j++;
        if (j >= d) return ZP_EINVAL;
        const int64_t m = std::min(out, need[j]);
        M[(size_t)i * d + j] += (int32_t)m;
        out -= m; need[j] -= m;
      }
    }
  }
  if (objective) {
    int64_t worst = 0;
    for (int i = 0; i < d; i++) worst = std::max(worst, (int64_t)b_intra * (s[i] - x[i]) + (int64_t)b_inter * x[i]);
    *objective = worst;
  }
  return ZP_OK;
}

extern "C" int zp_remap_indices(const int32_t *A, const int32_t *M, int32_t d, int32_t *idx, int64_t n_idx) {
  if (!A || !M || d < 1 || (!idx && n_idx > 0)) return ZP_EINVAL;
  std::vector<int64_t> B, offA(d + 1, 0);
  for (int i = 0; i < d; i++) {
    if (A[i] < 0) return ZP_EINVAL;
    offA[i + 1] = offA[i] + A[i];
  }
  if (offA[d] != n_idx || offA[d] > INT32_MAX) return ZP_EINVAL;
  balanced_targets(A, d, B);
  // M has to move exactly the surplus of every sender and the deficit of every receiver
  for (int i = 0; i < d; i++) {
    int64_t row = 0, col = 0;
    for (int j = 0; j < d; j++) {
      if (M[(size_t)i * d + j] < 0) return ZP_EINVAL;
      row += M[(size_t)i * d + j];
      col += M[(size_t)j * d + i];
    }
    if (row != std::max<int64_t>(A[i] - B[i], 0) || col != std::max<int64_t>(B[i] - A[i], 0)) return ZP_EINVAL;
  }
  // a sender parts with the tail of its buffer, one run per destination in ascending rank order
  std::vector<int64_t> seg((size_t)d * d);
  for (int i = 0; i < d; i++) {
    int64_t p = std::min<int64_t>(A[i], B[i]);
    for (int j = 0; j < d; j++) { seg[(size_t)i * d + j] = p; p += M[(size_t)i * d + j]; }
  }
  // a receiver keeps its head and appends the arrivals in ascending source order
  int64_t w = 0;
  for (int r = 0; r < d; r++) {
    const int64_t kept = std::min<int64_t>(A[r], B[r]);
    for (int64_t p = 0; p < kept; p++) idx[w++] = (int32_t)(offA[r] + p);
    for (int i = 0; i < d; i++)
      for (int64_t p = 0; p < M[(size_t)i * d + r]; p++) idx[w++] = (int32_t)(offA[i] + seg[(size_t)i * d + r] + p);
  }
  return w == n_idx ? ZP_OK : ZP_EINVAL;
}
