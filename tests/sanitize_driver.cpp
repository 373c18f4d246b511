// Driver for the sanitizer build of the CPU side: the fp64 oracle (oracle/zeppelin_oracle.c) and the host planners of
// the library (zp_partition.cpp, zp_remap_plan.cpp) are compiled with -fsanitize=address,undefined and linked into
// this program, which reads one request file written by tests/test_sanitizers.py, calls every function on it and
// writes the results as raw arrays. The test compares them with what the ordinary builds return, and fails on any
// sanitizer report (non-zero exit, text on stderr).
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "../include/zeppelin_attn.h"

extern "C" {
typedef struct { int32_t q_tok0, q_len, k_tok0, k_len, q_pos0, k_pos0, out_row0; } zo_pair;
typedef struct { int32_t out_tok0, len, n_parts; int32_t part_row0[16]; } zo_merge;
int zo_varlen_attn_fwd(const double *q, const double *k, const double *v, int64_t T, int Hq, int Hkv, int d,
                       const int32_t *cu, int S, double scale, double *o, double *lse);
int zo_chunk_attn_partial(const double *q, const double *k, const double *v, int64_t T, int Hq, int Hkv, int d,
                          const zo_pair *pairs, int n_pairs, double scale, double *o_part, double *lse_part,
                          int64_t part_rows);
int zo_lse_merge(const double *o_part, const double *lse_part, int64_t part_rows, const zo_merge *merges, int n_merges,
                 int64_t T, int Hq, int d, double *o, double *lse);
int zo_varlen_attn_bwd(const double *dout, const double *q, const double *k, const double *v, int64_t T, int Hq, int Hkv,
                       int d, const int32_t *cu, int S, double scale, double *dq, double *dk, double *dv);
int zo_varlen_attn_bwd_sample(const double *dout, const double *q, const double *k, const double *v, int64_t T, int Hq,
                              int Hkv, int d, const int32_t *cu, int S, double scale, const int32_t *q_tok,
                              const int32_t *q_head, int n_q, double *dq_out, const int32_t *k_tok, const int32_t *k_head,
                              int n_k, double *dk_out, double *dv_out);
int zo_chunk_attn_partial_bwd(const double *dout, const double *q, const double *k, const double *v, int64_t T, int Hq,
                              int Hkv, int d, const zo_pair *pairs, int n_pairs, double scale, const double *lse,
                              const double *D, double *dq, double *dk, double *dv);
int zo_remap_tokens(const void *src, void *dst, int64_t row_bytes, const int32_t *idx, int64_t n_rows, int mode);
}

static FILE *fin, *fout;
template <class T> static std::vector<T> rd(size_t n) {
  std::vector<T> v(n);
  if (n && std::fread(v.data(), sizeof(T), n, fin) != n) { std::fprintf(stderr, "short read\n"); std::exit(3); }
  return v;
}
static int64_t rd1() { return rd<int64_t>(1)[0]; }
template <class T> static void wr(const std::vector<T> &v) {
  const int64_t n = (int64_t)v.size();
  std::fwrite(&n, 8, 1, fout);
  if (n) std::fwrite(v.data(), sizeof(T), v.size(), fout);
}
static void must(int rc, const char *what) {
  if (rc < 0) { std::fprintf(stderr, "%s failed: %d\n", what, rc); std::exit(4); }
}

static void run_oracle() {
  const int64_t T = rd1(), Hq = rd1(), Hkv = rd1(), d = rd1(), S = rd1(), n_pairs = rd1(), part_rows = rd1(), n_merges = rd1();
  const double scale = rd<double>(1)[0];
  auto cu = rd<int32_t>(S + 1);
  auto q = rd<double>(T * Hq * d), k = rd<double>(T * Hkv * d), v = rd<double>(T * Hkv * d), dout = rd<double>(T * Hq * d);
  auto pairs = rd<zo_pair>(n_pairs);
  auto merges = rd<zo_merge>(n_merges);
  auto idx = rd<int32_t>(T);
  std::vector<double> o(T * Hq * d), lse(Hq * T), dq(T * Hq * d), dk(T * Hkv * d), dv(T * Hkv * d);
  must(zo_varlen_attn_fwd(q.data(), k.data(), v.data(), T, Hq, Hkv, d, cu.data(), S, scale, o.data(), lse.data()), "fwd");
  wr(o); wr(lse);
  must(zo_varlen_attn_bwd(dout.data(), q.data(), k.data(), v.data(), T, Hq, Hkv, d, cu.data(), S, scale, dq.data(), dk.data(), dv.data()), "bwd");
  wr(dq); wr(dk); wr(dv);
  std::vector<double> op(part_rows * Hq * d), lp(Hq * part_rows);
  must(zo_chunk_attn_partial(q.data(), k.data(), v.data(), T, Hq, Hkv, d, pairs.data(), n_pairs, scale, op.data(), lp.data(), part_rows), "partial");
  wr(op); wr(lp);
  std::vector<double> om(T * Hq * d, 0.0), lm(Hq * T, 0.0);
  must(zo_lse_merge(op.data(), lp.data(), part_rows, merges.data(), n_merges, T, Hq, d, om.data(), lm.data()), "merge");
  wr(om); wr(lm);
  // sampled backward: first, middle and last token of the batch
  std::vector<int32_t> st = {0, (int32_t)(T / 2), (int32_t)(T - 1)}, sh = {0, (int32_t)(Hq - 1), 0}, skh = {0, (int32_t)(Hkv - 1), 0};
  std::vector<double> sdq(3 * d), sdk(3 * d), sdv(3 * d);
  must(zo_varlen_attn_bwd_sample(dout.data(), q.data(), k.data(), v.data(), T, Hq, Hkv, d, cu.data(), S, scale, st.data(), sh.data(), 3,
                                 sdq.data(), st.data(), skh.data(), 3, sdk.data(), sdv.data()), "bwd_sample");
  wr(sdq); wr(sdk); wr(sdv);
  // chunked backward over the same pairs with the whole-row statistics
  std::vector<double> D(Hq * T), cdq(T * Hq * d, 0.0), cdk(T * Hkv * d, 0.0), cdv(T * Hkv * d, 0.0);
  for (int64_t t = 0; t < T; t++)
    for (int64_t h = 0; h < Hq; h++) {
      double s = 0;
      for (int64_t c = 0; c < d; c++) s += dout[(t * Hq + h) * d + c] * o[(t * Hq + h) * d + c];
      D[h * T + t] = s;
    }
  must(zo_chunk_attn_partial_bwd(dout.data(), q.data(), k.data(), v.data(), T, Hq, Hkv, d, pairs.data(), n_pairs, scale, lse.data(), D.data(),
                                 cdq.data(), cdk.data(), cdv.data()), "partial_bwd");
  wr(cdq); wr(cdk); wr(cdv);
  std::vector<double> g(T * Hq * d), sc(T * Hq * d);
  must(zo_remap_tokens(q.data(), g.data(), Hq * d * 8, idx.data(), T, 0), "remap gather");
  must(zo_remap_tokens(q.data(), sc.data(), Hq * d * 8, idx.data(), T, 1), "remap scatter");
  wr(g); wr(sc);
}

static void run_planners() {
  const int64_t n_cases = rd1();
  for (int64_t c = 0; c < n_cases; c++) {
    const int32_t P = (int32_t)rd1(), N = (int32_t)rd1(), L = (int32_t)rd1(), S = (int32_t)rd1(), b_intra = (int32_t)rd1(), b_inter = (int32_t)rd1();
    auto lengths = rd<int32_t>(S);
    std::vector<zp_placement> pl((size_t)S * P * N + 1);
    int32_t n_pl = 0, s1 = 0;
    std::vector<int32_t> s0(N);
    must(zp_partition(lengths.data(), S, P, N, L, pl.data(), (int32_t)pl.size(), &n_pl, &s1, s0.data()), "zp_partition");
    pl.resize(n_pl);
    std::vector<int32_t> flat;
    for (auto &x : pl) for (int32_t f : {x.seq, x.zone, x.ring, x.rank, x.node, x.device, x.tokens}) flat.push_back(f);
    flat.push_back(s1);
    for (int32_t x : s0) flat.push_back(x);
    wr(flat);
    std::vector<zp_segment> segs(2 * (size_t)n_pl + 1);
    std::vector<int32_t> A((size_t)P * N);
    int32_t n_seg = 0;
    must(zp_node_segments(lengths.data(), S, pl.data(), n_pl, P, N, segs.data(), (int32_t)segs.size(), &n_seg, A.data()), "zp_node_segments");
    segs.resize(n_seg);
    flat.clear();
    for (auto &x : segs) for (int32_t f : {x.seq, x.chunk, x.n_chunks, x.pos0, x.len, x.tok0, x.node, x.device}) flat.push_back(f);
    wr(flat); wr(A);
    int64_t T = 0;
    for (int32_t x : lengths) T += x;
    std::vector<int64_t> orig(T);
    must(zp_segment_positions(lengths.data(), S, segs.data(), n_seg, orig.data(), T), "zp_segment_positions");
    wr(orig);
    int32_t n_pairs = 0, rounds = 0;
    int rc = zp_ring_round_pairs(segs.data(), n_seg, 0, 0, nullptr, 0, &n_pairs, &rounds);
    if (rc != ZP_OK && rc != ZP_EWORKSPACE) must(rc, "zp_ring_round_pairs");
    flat.clear();
    for (int32_t t = 0; t < rounds; t++) {
      std::vector<zp_pair> pr(n_pairs + 1);
      int32_t n = 0;
      must(zp_ring_round_pairs(segs.data(), n_seg, t, 0, pr.data(), (int32_t)pr.size(), &n, nullptr), "zp_ring_round_pairs");
      flat.push_back(n);
      for (int32_t i = 0; i < n; i++)
        for (int32_t f : {pr[i].q_tok0, pr[i].q_len, pr[i].k_tok0, pr[i].k_len, pr[i].q_pos0, pr[i].k_pos0}) flat.push_back(f);
    }
    wr(flat);
    const int32_t dd = P * N;
    std::vector<int32_t> M((size_t)dd * dd), idx(T);
    int64_t obj = 0;
    must(zp_remap_plan(A.data(), dd, P, b_intra, b_inter, M.data(), &obj), "zp_remap_plan");
    must(zp_remap_indices(A.data(), M.data(), dd, idx.data(), T), "zp_remap_indices");
    wr(M); wr(idx);
    wr(std::vector<int64_t>{obj});
    // a sequence cut into chunks where it lies, and its pair helper
    if (S > 0 && lengths[0] > 0) {
      std::vector<zp_segment> cs(5);
      must(zp_chunk_segments(0, 3, lengths[0], 5, cs.data(), 5), "zp_chunk_segments");
      flat.clear();
      for (auto &x : cs) for (int32_t f : {x.pos0, x.len, x.tok0}) flat.push_back(f);
      wr(flat);
    }
  }
}

int main(int argc, char **argv) {
  if (argc != 4) return 2;
  fin = std::fopen(argv[2], "rb");
  fout = std::fopen(argv[3], "wb");
  if (!fin || !fout) return 2;
  if (!std::strcmp(argv[1], "oracle")) run_oracle();
  else if (!std::strcmp(argv[1], "planners")) run_planners();
  else return 2;
  std::fclose(fin);
  std::fclose(fout);
  return 0;
}
