// C ABI of the attention engine: argument checks, the host planner (work lists ordered by cost), descriptor
// upload through pinned staging buffers, kernel launches. No device allocation, no synchronisation.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <string>
#include <vector>

#include "../../include/zeppelin_attn.h"
#include "zp_common.h"
#include "zp_pool.h"

extern "C" {
int zp_launch_attn_fwd(const zp_attn_params *p, int d, int partial, int block_rows, hipStream_t stream);
int zp_attn_fwd_block_rows(int d);
int zp_launch_remap(const void *src, void *dst, int64_t row_bytes, const int32_t *idx, int64_t n_rows, int mode,
                    hipStream_t stream);
int zp_merge_rows_per_item(void);
int zp_launch_lse_merge(const float *o_part, const float *lse_part, int64_t part_rows, const void *merges_dev,
                        const void *items_dev, int n_items, int Hq, int d, void *o, int64_t o_stride, float *lse,
                        int64_t T, int max_parts, hipStream_t stream);
struct zp_bwd_params {
  const __bf16 *q, *k, *v, *o, *dout;
  int64_t q_stride, k_stride, v_stride, o_stride, do_stride;
  const float *lse;
  float *dvec;
  float *lse2;
  const zp_tile *dq_tiles;
  const zp_tile *kv_tiles;
  const zp_tile *kv_tiles_short;  // key blocks with few query tiles: run by the two-workgroups-per-CU kernel (d = 128)
  int32_t n_dq_tiles, n_kv_tiles, n_kv_tiles_short, Hq, Hkv, grp, T;
  float scale_log2, scale;
  __bf16 *dq, *dk, *dv;
  int64_t dq_stride, dkv_stride;
  int32_t accumulate;
  zp_work_split work_dq, work_kv, work_kv_short;
};
int zp_launch_accum_to_bf16(const float *src, void *dst, int64_t n, hipStream_t stream);
int zp_launch_attn_bwd(const zp_bwd_params *p, int d, hipStream_t stream);
int zp_attn_bwd_block_rows(int d, int which);
}

namespace {

thread_local std::string g_hip_error = "HIP runtime error";

int hip_fail(hipError_t e, const char *what) {
  g_hip_error = std::string("HIP runtime error in ") + what + ": " + hipGetErrorString(e);
  return ZP_EHIP;
}
#define ZP_HIP(call, what)                       \
  do {                                           \
    hipError_t e__ = (call);                     \
    if (e__ != hipSuccess) return hip_fail(e__, what); \
  } while (0)

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- pinned staging pool -------------------------------------------------------------------------
// Descriptor tables are built in pinned host memory and copied with hipMemcpyAsync; a slot is reused only
// after the event recorded behind its copy has completed, so the host never overwrites bytes in flight
// (zp_pool.h holds the slot state machine; this is its HIP backend).
struct HipPoolBackend {
  typedef hipEvent_t event_t;
  typedef hipStream_t stream_t;
  static int alloc(void **p, size_t bytes) { return (int)hipHostMalloc(p, bytes, hipHostMallocDefault); }
  static void release(void *p) { (void)hipHostFree(p); }
  static int event_create(event_t *e) { return (int)hipEventCreateWithFlags(e, hipEventDisableTiming); }
  static int event_record(event_t e, stream_t s) { return (int)hipEventRecord(e, s); }
  static bool event_done(event_t e) { return hipEventQuery(e) == hipSuccess; }
};
zp_staging_pool<HipPoolBackend> g_pool;

int pool_acquire(size_t bytes, int *slot_out, void **host_out) {
  const int e = g_pool.acquire(bytes, slot_out, host_out);
  return e ? hip_fail((hipError_t)e, "staging buffer") : ZP_OK;
}
// Copy `bytes` from the slot to device memory on `stream` and mark the slot busy until the copy is done.
int pool_upload(int slot, const void *host, void *dev, size_t bytes, hipStream_t stream) {
  hipError_t e = hipMemcpyAsync(dev, host, bytes, hipMemcpyHostToDevice, stream);
  if (e != hipSuccess) {
    g_pool.abandon(slot);
    return hip_fail(e, "hipMemcpyAsync");
  }
  const int r = g_pool.submitted(slot, stream);
  return r ? hip_fail((hipError_t)r, "hipEventRecord") : ZP_OK;
}

// ---- per-kernel timing (measurement aid) -----------------------------------------------------------
// When enabled, every kernel launch is bracketed by a pair of hipEvents on the launch stream; the bench reads
// the elapsed times after it has synchronised. Off by default: no events are created or recorded.
struct ProfRec {
  const char *name;
  hipEvent_t a, b;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof;

// ---- checks --------------------------------------------------------------------------------------
int check_shape(const zp_shape *sh) {
  if (!sh) return ZP_EINVAL;
  if (sh->T < 0 || sh->S < 0 || sh->Hq <= 0 || sh->Hkv <= 0) return ZP_EINVAL;
  if (!(sh->scale >= 0.f) || std::isinf(sh->scale)) return ZP_EINVAL;
  if (sh->d != 64 && sh->d != 128) return ZP_EUNSUPPORTED;
  if (sh->Hq % sh->Hkv) return ZP_EUNSUPPORTED;
  return ZP_OK;
}
int check_cu(const int32_t *cu, const zp_shape *sh) {
  if (!cu) return ZP_EINVAL;
  if (cu[0] != 0) return ZP_EINVAL;
  for (int s = 0; s < sh->S; s++)
    if (cu[s + 1] < cu[s]) return ZP_EINVAL;
  if (cu[sh->S] != sh->T) return ZP_EINVAL;
  return ZP_OK;
}
// token strides: at least one token's heads, 16-byte aligned rows, and small enough that the byte offsets of a
// 64-row tile fit the 32-bit lane offsets of the asynchronous tile copy
int check_stride(int64_t stride, int H, int d) {
  return (stride < (int64_t)H * d || (stride % 8) || stride > (1 << 24)) ? ZP_EINVAL : ZP_OK;
}
bool aligned16(const void *p) { return ((uintptr_t)p & 15) == 0; }
int check_ws(const void *ws, size_t have, size_t need) {
  if (need == 0) return ZP_OK;
  if (!ws || ((uintptr_t)ws & 255) || have < need) return ZP_EWORKSPACE;
  return ZP_OK;
}
float eff_scale(const zp_shape *sh) { return sh->scale > 0.f ? sh->scale : 1.0f / std::sqrt((float)sh->d); }

// ---- planner -------------------------------------------------------------------------------------
// A tile's cost is the number of key tiles it visits: the per-block share of the quadratic cost |s|^2 that
// Alg. 2 balances. Lists of chunk-pair tiles are issued in descending cost so the heaviest start first.
struct CostTile {
  zp_tile t;
  int32_t cost;
};
inline int32_t tile_cost(const zp_tile &t) {
  int64_t n = (int64_t)t.q_pos0 + t.q_rows - 1 - t.k_pos0 + 1;
  if (n < 0) n = 0;
  if (n > t.k_len) n = t.k_len;
  return (int32_t)((n + 63) / 64);
}
void sort_by_cost(std::vector<CostTile> &v) {
  std::stable_sort(v.begin(), v.end(), [](const CostTile &a, const CostTile &b) { return a.cost > b.cost; });
}
int64_t count_blocks(const int32_t *cu, int S, int bm) {
  int64_t n = 0;
  for (int s = 0; s < S; s++) n += ((int64_t)cu[s + 1] - cu[s] + bm - 1) / bm;
  return n;
}
// Tiles of whole sequences: sequence by sequence, longest sequence first, and inside a sequence the last query block
// (the most expensive one) first. The heaviest tiles of the batch still start first and the cheap ones fill the tail,
// as a plain sort by cost would have it, but the query blocks of one (sequence, KV head) now run next to each other on
// one XCD and find the sequence's K/V rows in its L2 instead of re-reading them from HBM -- with many short sequences
// and one KV head per query head that re-reading, not the arithmetic, bounded the kernels.
void plan_whole(const int32_t *cu, int S, int bm, std::vector<CostTile> &out, const uint8_t *skip = nullptr) {
  std::vector<int> seq_order(S);
  for (int s = 0; s < S; s++) seq_order[s] = s;
  std::stable_sort(seq_order.begin(), seq_order.end(), [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
  for (int s : seq_order) {
    if (skip && skip[s]) continue;
    const int32_t L = cu[s + 1] - cu[s];
    for (int32_t r0 = ((L - 1) / bm) * bm; L > 0 && r0 >= 0; r0 -= bm) {
      CostTile c;
      c.t.q_tok0 = cu[s] + r0;
      c.t.q_rows = std::min(bm, L - r0);
      c.t.q_pos0 = r0;
      c.t.k_tok0 = cu[s];
      c.t.k_len = L;
      c.t.k_pos0 = 0;
      c.t.out_row0 = cu[s] + r0;
      c.t.aux = 0;
      c.cost = tile_cost(c.t);
      out.push_back(c);
    }
  }
}
int64_t count_pair_blocks(const zp_pair *pairs, int n, int bm) {
  int64_t c = 0;
  for (int i = 0; i < n; i++) c += ((int64_t)pairs[i].q_len + bm - 1) / bm;
  return c;
}

// Every tile table in a workspace is preceded by WS_HEADER bytes of work counters (three sets: a call launches at most
// three attention kernels), which travel with the table in the same copy and arrive as zeros.
constexpr size_t WS_HEADER = 3 * ZP_COUNTER_BYTES;
inline int32_t *ws_counters(void *ws) { return (int32_t *)ws; }
inline const zp_tile *ws_tiles(void *ws) { return (const zp_tile *)((char *)ws + WS_HEADER); }
inline size_t tile_table_bytes(size_t n_tiles) { return WS_HEADER + align256(n_tiles * sizeof(zp_tile)); }

// Share of a launch's items that workgroups claim at run time (zp_work_split): half when the items are heavy (32 key
// or query tiles and more on average, i.e. tens of microseconds each), an eighth when they are light.
int dyn_div_of(const std::vector<CostTile> &tiles, size_t first, size_t n, int weight) {
  if (n == 0) return 8;
  int64_t sum = 0;
  for (size_t i = first; i < first + n; i++) sum += tiles[i].cost;
  return sum * weight >= (int64_t)n * 32 ? 2 : 8;
}

int upload_tiles(const std::vector<CostTile> &tiles, void *ws, hipStream_t stream) {
  if (tiles.empty()) return ZP_OK;
  const size_t bytes = WS_HEADER + tiles.size() * sizeof(zp_tile);
  int slot;
  void *host;
  int rc = pool_acquire(bytes, &slot, &host);
  if (rc) return rc;
  std::memset(host, 0, WS_HEADER);
  zp_tile *h = (zp_tile *)((char *)host + WS_HEADER);
  for (size_t i = 0; i < tiles.size(); i++) h[i] = tiles[i].t;
  return pool_upload(slot, host, ws, bytes, stream);
}

// Sequences (or chunk pairs) whose key blocks loop over few (query tile, head) iterations go to the dK/dV kernel that
// runs two workgroups per CU (head dimension 128 only): a workgroup's fixed cost -- launch, row operands, first tiles,
// final stores -- is then covered by its neighbour, which is worth more than the other kernel's denser key loop below
// about 256 iterations of 64 queries (measured crossover: 8K tokens with one query head per KV head, 2K-4K tokens with
// 4-8). The choice is made per sequence, not per key block, so that the light last blocks of a long sequence stay in
// the long kernel's launch and fill its tail.
inline bool kv_rows_are_short(int64_t q_rows_max, int d, int grp) { return d == 128 && ((q_rows_max + 63) / 64) * grp < 256; }
// Moves the tiles marked short (aux = 1) behind the others, keeping the order inside both parts; returns the number of
// long tiles. When the short ones hold less than 30 % of the launch's work (query tiles to visit) they stay with the
// long ones instead: two launches have two tails, and a few light sequences are worth more as the filler of the long
// kernel's tail than they gain from the other kernel.
size_t split_kv_tiles(std::vector<CostTile> &kt) {
  int64_t work = 0, work_short = 0;
  for (const CostTile &c : kt) {
    work += c.cost;
    if (c.t.aux) work_short += c.cost;
  }
  if (work_short * 10 < work * 3)
    for (CostTile &c : kt) c.t.aux = 0;
  return (size_t)(std::stable_partition(kt.begin(), kt.end(), [](const CostTile &c) { return c.t.aux == 0; }) - kt.begin());
}

}  // namespace

extern "C" {

void zp_prof_begin(const char *name, hipStream_t stream) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!g_prof_on) return;
  ProfRec r{name, nullptr, nullptr};
  if (hipEventCreate(&r.a) != hipSuccess || hipEventCreate(&r.b) != hipSuccess) return;
  (void)hipEventRecord(r.a, stream);
  g_prof.push_back(r);
}
void zp_prof_end(hipStream_t stream) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (!g_prof_on || g_prof.empty()) return;
  (void)hipEventRecord(g_prof.back().b, stream);
}
int zp_profile_enable(int on) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  for (auto &r : g_prof) {
    (void)hipEventDestroy(r.a);
    (void)hipEventDestroy(r.b);
  }
  g_prof.clear();
  g_prof_on = on != 0;
  return ZP_OK;
}
int zp_profile_count(void) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  return (int)g_prof.size();
}
int zp_profile_get(int i, char *name, int name_cap, float *ms) {
  std::lock_guard<std::mutex> lk(g_prof_mu);
  if (i < 0 || i >= (int)g_prof.size() || !name || name_cap < 1 || !ms) return ZP_EINVAL;
  ZP_HIP(hipEventSynchronize(g_prof[i].b), "hipEventSynchronize");
  ZP_HIP(hipEventElapsedTime(ms, g_prof[i].a, g_prof[i].b), "hipEventElapsedTime");
  std::snprintf(name, (size_t)name_cap, "%s", g_prof[i].name);
  return ZP_OK;
}

// for the other translation units of the library: records the HIP error text and returns ZP_EHIP
int zp_report_hip_error(int hip_error, const char *what) { return hip_fail((hipError_t)hip_error, what); }

const char *zp_strerror(int code) {
  switch (code) {
    case ZP_OK: return "ok";
    case ZP_EINVAL: return "invalid argument";
    case ZP_EUNSUPPORTED: return "unsupported configuration";
    case ZP_EWORKSPACE: return "workspace missing, misaligned or too small";
    case ZP_EHIP: return g_hip_error.c_str();
    case ZP_ETOOLARGE: return "more sequences or tiles than the fixed limits of the no-allocation entry point";
    default: return "unknown error code";
  }
}

size_t zp_workspace_bytes(int which_fn, const zp_shape *sh, const int32_t *cu, int64_t n_desc) {
  if (check_shape(sh) != ZP_OK) return 0;
  switch (which_fn) {
    case ZP_FN_FWD: {
      if (check_cu(cu, sh) != ZP_OK) return 0;
      return tile_table_bytes((size_t)count_blocks(cu, sh->S, zp_attn_fwd_block_rows(sh->d))) + 256;
    }
    case ZP_FN_PARTIAL: {
      if (n_desc < 0) return 0;
      // a pair of q_len rows yields ceil(q_len / block_rows) tiles; bound it with T rows per pair... the exact
      // count needs the pairs, so this bound uses one tile per block_rows tokens of T plus one per pair, per pair
      const int bm = zp_attn_fwd_block_rows(sh->d);
      return tile_table_bytes((size_t)n_desc * ((size_t)sh->T / bm + 1)) + 256;
    }
    case ZP_FN_MERGE: {
      if (n_desc < 0) return 0;
      const int rpi = zp_merge_rows_per_item();
      return align256((size_t)n_desc * sizeof(zp_merge)) + align256(((size_t)sh->T / rpi + (size_t)n_desc + 1) * 8) + 256;
    }
    case ZP_FN_PARTIAL_BWD: {
      if (n_desc < 0) return 0;
      const size_t per_pair = (size_t)sh->T / zp_attn_bwd_block_rows(sh->d, 0) + (size_t)sh->T / zp_attn_bwd_block_rows(sh->d, 1) + 2;
      return tile_table_bytes((size_t)n_desc * per_pair) + 2 * align256((size_t)sh->Hq * (size_t)sh->T * sizeof(float)) + 512;
    }
    case ZP_FN_BWD: {
      if (check_cu(cu, sh) != ZP_OK) return 0;
      const size_t tiles = (size_t)count_blocks(cu, sh->S, zp_attn_bwd_block_rows(sh->d, 0)) +
                           (size_t)count_blocks(cu, sh->S, zp_attn_bwd_block_rows(sh->d, 1));
      return tile_table_bytes(tiles) + 2 * align256((size_t)sh->Hq * (size_t)sh->T * sizeof(float)) + 512;
    }
    default: return 0;
  }
}

int varlen_attn_fwd(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride, int64_t v_stride,
                    const int32_t *cu, const uint8_t *seq_skip, void *o, int64_t o_stride, float *lse,
                    const zp_shape *sh, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if ((rc = check_cu(cu, sh))) return rc;
  if (sh->T == 0) return ZP_OK;
  if (!q || !k || !v || !o || !lse) return ZP_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o)) return ZP_EINVAL;
  if (check_stride(q_stride, sh->Hq, sh->d) || check_stride(o_stride, sh->Hq, sh->d) ||
      check_stride(k_stride, sh->Hkv, sh->d) || check_stride(v_stride, sh->Hkv, sh->d))
    return ZP_EINVAL;
  const int bm = zp_attn_fwd_block_rows(sh->d);
  std::vector<CostTile> tiles;
  tiles.reserve((size_t)count_blocks(cu, sh->S, bm));
  plan_whole(cu, sh->S, bm, tiles, seq_skip);
  if (tiles.empty()) return ZP_OK;
  if ((rc = check_ws(ws, ws_bytes, tile_table_bytes(tiles.size())))) return rc;
  if ((rc = upload_tiles(tiles, ws, (hipStream_t)stream))) return rc;
  zp_attn_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride;
  p.tiles = ws_tiles(ws); p.n_tiles = (int32_t)tiles.size(); p.work.counters = ws_counters(ws); p.work.dyn_div = dyn_div_of(tiles, 0, tiles.size(), 1);
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv;
  p.scale = eff_scale(sh); p.scale_log2 = p.scale * 1.4426950408889634f;
  p.o = o; p.o_stride = o_stride; p.lse = lse; p.lse_stride = sh->T;
  hipError_t e = (hipError_t)zp_launch_attn_fwd(&p, sh->d, 0, bm, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "attn_fwd launch");
  return ZP_OK;
}

int chunk_attn_partial(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride,
                       int64_t v_stride, const zp_pair *pairs, int32_t n_pairs, float *o_part, float *lse_part,
                       int64_t part_rows, const zp_shape *sh, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if (n_pairs < 0 || part_rows < 0) return ZP_EINVAL;
  if (n_pairs == 0) return ZP_OK;
  if (!q || !k || !v || !o_part || !lse_part || !pairs) return ZP_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o_part)) return ZP_EINVAL;
  if (check_stride(q_stride, sh->Hq, sh->d) || check_stride(k_stride, sh->Hkv, sh->d) ||
      check_stride(v_stride, sh->Hkv, sh->d))
    return ZP_EINVAL;
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    if (pr.q_len < 0 || pr.k_len < 0 || pr.q_tok0 < 0 || pr.k_tok0 < 0 || pr.q_pos0 < 0 || pr.k_pos0 < 0 ||
        pr.out_row0 < 0)
      return ZP_EINVAL;
    if ((int64_t)pr.q_tok0 + pr.q_len > sh->T || (int64_t)pr.k_tok0 + pr.k_len > sh->T) return ZP_EINVAL;
    if ((int64_t)pr.out_row0 + pr.q_len > part_rows) return ZP_EINVAL;
  }
  const int bm = zp_attn_fwd_block_rows(sh->d);
  std::vector<CostTile> tiles;
  tiles.reserve((size_t)count_pair_blocks(pairs, n_pairs, bm));
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    for (int32_t r0 = 0; r0 < pr.q_len; r0 += bm) {
      CostTile c;
      c.t.q_tok0 = pr.q_tok0 + r0;
      c.t.q_rows = std::min(bm, pr.q_len - r0);
      c.t.q_pos0 = pr.q_pos0 + r0;
      c.t.k_tok0 = pr.k_tok0;
      c.t.k_len = pr.k_len;
      c.t.k_pos0 = pr.k_pos0;
      c.t.out_row0 = pr.out_row0 + r0;
      c.t.aux = 0;
      c.cost = tile_cost(c.t);
      tiles.push_back(c);
    }
  }
  sort_by_cost(tiles);
  if ((rc = check_ws(ws, ws_bytes, tile_table_bytes(tiles.size())))) return rc;
  if ((rc = upload_tiles(tiles, ws, (hipStream_t)stream))) return rc;
  zp_attn_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride;
  p.tiles = ws_tiles(ws); p.n_tiles = (int32_t)tiles.size(); p.work.counters = ws_counters(ws); p.work.dyn_div = dyn_div_of(tiles, 0, tiles.size(), 1);
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv;
  p.scale = eff_scale(sh); p.scale_log2 = p.scale * 1.4426950408889634f;
  p.o = o_part; p.o_stride = (int64_t)sh->Hq * sh->d; p.lse = lse_part; p.lse_stride = part_rows;
  hipError_t e = (hipError_t)zp_launch_attn_fwd(&p, sh->d, 1, bm, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "chunk_attn_partial launch");
  return ZP_OK;
}

int chunk_attn_update(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride, int64_t v_stride,
                      const zp_pair *pairs, int32_t n_pairs, float *o_run, float *lse_run, const zp_shape *sh,
                      void *ws, size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if (n_pairs < 0) return ZP_EINVAL;
  if (n_pairs == 0 || sh->T == 0) return ZP_OK;
  if (!q || !k || !v || !o_run || !lse_run || !pairs) return ZP_EINVAL;
  if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o_run)) return ZP_EINVAL;
  if (check_stride(q_stride, sh->Hq, sh->d) || check_stride(k_stride, sh->Hkv, sh->d) ||
      check_stride(v_stride, sh->Hkv, sh->d))
    return ZP_EINVAL;
  // the running rows are read, merged and written back without atomics: a query row may appear in one pair only
  std::vector<std::pair<int32_t, int32_t>> qr;
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    if (pr.q_len < 0 || pr.k_len < 0 || pr.q_tok0 < 0 || pr.k_tok0 < 0 || pr.q_pos0 < 0 || pr.k_pos0 < 0) return ZP_EINVAL;
    if ((int64_t)pr.q_tok0 + pr.q_len > sh->T || (int64_t)pr.k_tok0 + pr.k_len > sh->T) return ZP_EINVAL;
    if (pr.q_len > 0) qr.push_back({pr.q_tok0, pr.q_tok0 + pr.q_len});
  }
  std::sort(qr.begin(), qr.end());
  for (size_t i = 1; i < qr.size(); i++)
    if (qr[i].first < qr[i - 1].second) return ZP_EINVAL;
  const int bm = zp_attn_fwd_block_rows(sh->d);
  std::vector<CostTile> tiles;
  tiles.reserve((size_t)count_pair_blocks(pairs, n_pairs, bm));
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    for (int32_t r0 = 0; r0 < pr.q_len; r0 += bm) {
      CostTile c;
      c.t.q_tok0 = pr.q_tok0 + r0;
      c.t.q_rows = std::min(bm, pr.q_len - r0);
      c.t.q_pos0 = pr.q_pos0 + r0;
      c.t.k_tok0 = pr.k_tok0;
      c.t.k_len = pr.k_len;
      c.t.k_pos0 = pr.k_pos0;
      c.t.out_row0 = c.t.q_tok0;  // the running rows are the query's own token rows
      c.t.aux = 0;
      c.cost = tile_cost(c.t);
      if (c.cost > 0) tiles.push_back(c);  // a block that sees no key leaves its rows as they are
    }
  }
  if (tiles.empty()) return ZP_OK;
  sort_by_cost(tiles);
  if ((rc = check_ws(ws, ws_bytes, tile_table_bytes(tiles.size())))) return rc;
  if ((rc = upload_tiles(tiles, ws, (hipStream_t)stream))) return rc;
  zp_attn_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride;
  p.tiles = ws_tiles(ws); p.n_tiles = (int32_t)tiles.size(); p.work.counters = ws_counters(ws); p.work.dyn_div = dyn_div_of(tiles, 0, tiles.size(), 1);
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv;
  p.scale = eff_scale(sh); p.scale_log2 = p.scale * 1.4426950408889634f;
  p.o = o_run; p.o_stride = (int64_t)sh->Hq * sh->d; p.lse = lse_run; p.lse_stride = sh->T;
  p.update = 1;
  hipError_t e = (hipError_t)zp_launch_attn_fwd(&p, sh->d, 1, bm, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "chunk_attn_update launch");
  return ZP_OK;
}

int lse_merge(const float *o_part, const float *lse_part, int64_t part_rows, const zp_merge *merges, int32_t n_merges,
              void *o, int64_t o_stride, float *lse, const zp_shape *sh, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if (n_merges < 0 || part_rows < 0) return ZP_EINVAL;
  if (n_merges == 0) return ZP_OK;
  if (!o_part || !lse_part || !merges || !o || !lse) return ZP_EINVAL;
  if (!aligned16(o_part) || !aligned16(o)) return ZP_EINVAL;
  if (check_stride(o_stride, sh->Hq, sh->d)) return ZP_EINVAL;
  const int rpi = zp_merge_rows_per_item();
  size_t n_items = 0;
  for (int i = 0; i < n_merges; i++) {
    const zp_merge &m = merges[i];
    if (m.n_parts < 1 || m.n_parts > ZP_MAX_PARTS || m.len < 0 || m.out_tok0 < 0 ||
        (int64_t)m.out_tok0 + m.len > sh->T)
      return ZP_EINVAL;
    for (int p = 0; p < m.n_parts; p++)
      if (m.part_row0[p] < 0 || (int64_t)m.part_row0[p] + m.len > part_rows) return ZP_EINVAL;
    n_items += ((size_t)m.len + rpi - 1) / rpi;
  }
  const size_t desc_bytes = align256((size_t)n_merges * sizeof(zp_merge));
  const size_t item_bytes = n_items * 8;
  if ((rc = check_ws(ws, ws_bytes, desc_bytes + align256(item_bytes)))) return rc;
  if (n_items == 0) return ZP_OK;
  int slot;
  void *host;
  if ((rc = pool_acquire(desc_bytes + item_bytes, &slot, &host))) return rc;
  char *h = (char *)host;
  std::memcpy(h, merges, (size_t)n_merges * sizeof(zp_merge));
  int32_t *items = (int32_t *)(h + desc_bytes);
  size_t n = 0;
  for (int i = 0; i < n_merges; i++)
    for (int32_t r0 = 0; r0 < merges[i].len; r0 += rpi) {
      items[2 * n] = i;
      items[2 * n + 1] = r0;
      n++;
    }
  if ((rc = pool_upload(slot, host, ws, desc_bytes + item_bytes, (hipStream_t)stream))) return rc;
  int max_parts = 1;
  for (int i = 0; i < n_merges; i++) max_parts = std::max(max_parts, (int)merges[i].n_parts);
  hipError_t e = (hipError_t)zp_launch_lse_merge(o_part, lse_part, part_rows, ws, (char *)ws + desc_bytes, (int)n_items,
                                                 sh->Hq, sh->d, o, o_stride, lse, sh->T, max_parts, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "lse_merge launch");
  return ZP_OK;
}

int remap_tokens(const void *src, void *dst, int64_t row_bytes, const int32_t *idx_dev, int64_t n_rows, int32_t mode,
                 void *stream) {
  if (n_rows < 0 || row_bytes <= 0 || (mode != 0 && mode != 1)) return ZP_EINVAL;
  if (row_bytes % 16) return ZP_EUNSUPPORTED;
  if (n_rows == 0) return ZP_OK;
  if (!src || !dst || !idx_dev) return ZP_EINVAL;
  if (!aligned16(src) || !aligned16(dst)) return ZP_EINVAL;
  if (n_rows > 0x7fffffffLL || row_bytes > (1 << 20)) return ZP_EUNSUPPORTED;
  const char *s = (const char *)src;
  const char *d = (const char *)dst;
  const int64_t bytes = n_rows * row_bytes;
  if (s < d + bytes && d < s + bytes) return ZP_EINVAL;  // overlap
  hipError_t e = (hipError_t)zp_launch_remap(src, dst, row_bytes, idx_dev, n_rows, mode, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "remap_tokens launch");
  return ZP_OK;
}

int zp_chunk_pairs(int32_t tok0, int32_t L, int32_t C, int32_t rank, int32_t row0, zp_pair *pairs, int32_t max_pairs,
                   zp_merge *merges, int32_t max_merges, int32_t *n_merges, int64_t *rows_used) {
  if (L < 0 || C < 1 || tok0 < 0 || row0 < 0 || !pairs || !merges || !n_merges || !rows_used) return ZP_EINVAL;
  if (rank >= 0 && ((C & 1) || rank >= C / 2)) return ZP_EINVAL;
  auto bound = [&](int c) { return (int32_t)(((int64_t)c * L) / C); };
  int np = 0, nm = 0;
  int64_t row = row0;
  for (int qc = 0; qc < C; qc++) {
    if (rank >= 0 && qc != rank && qc != C - 1 - rank) continue;
    if (qc + 1 > ZP_MAX_PARTS) return ZP_EUNSUPPORTED;
    if (nm >= max_merges) return ZP_EINVAL;
    const int32_t qlen = bound(qc + 1) - bound(qc);
    zp_merge &m = merges[nm++];
    m.out_tok0 = tok0 + bound(qc);
    m.len = qlen;
    m.n_parts = qc + 1;
    for (int kc = 0; kc <= qc; kc++) {
      if (np >= max_pairs) return ZP_EINVAL;
      if (row + qlen > 0x7fffffffLL) return ZP_EINVAL;
      zp_pair &p = pairs[np++];
      p.q_tok0 = tok0 + bound(qc); p.q_len = qlen; p.q_pos0 = bound(qc);
      p.k_tok0 = tok0 + bound(kc); p.k_len = bound(kc + 1) - bound(kc); p.k_pos0 = bound(kc);
      p.out_row0 = (int32_t)row;
      m.part_row0[kc] = (int32_t)row;
      row += qlen;
    }
  }
  *n_merges = nm;
  *rows_used = row - row0;
  return np;
}

}  // extern "C"

extern "C" int varlen_attn_bwd(const void *dout, const void *q, const void *k, const void *v, const void *o,
                               const float *lse, int64_t do_stride, int64_t q_stride, int64_t k_stride,
                               int64_t v_stride, int64_t o_stride, const int32_t *cu, const uint8_t *seq_skip,
                               void *dq, void *dk, void *dv, int64_t dq_stride, int64_t dkv_stride,
                               const zp_shape *sh, void *ws, size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if ((rc = check_cu(cu, sh))) return rc;
  if (sh->T == 0) return ZP_OK;
  if (!dout || !q || !k || !v || !o || !lse || !dq || !dk || !dv) return ZP_EINVAL;
  if (!aligned16(dout) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(dq) ||
      !aligned16(dk) || !aligned16(dv))
    return ZP_EINVAL;
  if (check_stride(q_stride, sh->Hq, sh->d) || check_stride(o_stride, sh->Hq, sh->d) ||
      check_stride(do_stride, sh->Hq, sh->d) || check_stride(dq_stride, sh->Hq, sh->d) ||
      check_stride(k_stride, sh->Hkv, sh->d) || check_stride(v_stride, sh->Hkv, sh->d) ||
      check_stride(dkv_stride, sh->Hkv, sh->d))
    return ZP_EINVAL;
  const int bmq = zp_attn_bwd_block_rows(sh->d, 0), bnk = zp_attn_bwd_block_rows(sh->d, 1);
  std::vector<CostTile> qt, kt;
  qt.reserve((size_t)count_blocks(cu, sh->S, bmq));
  plan_whole(cu, sh->S, bmq, qt, seq_skip);
  kt.reserve((size_t)count_blocks(cu, sh->S, bnk));
  // Key-block tiles go sequence by sequence, longest sequence first, blocks in position order (descending
  // cost inside the sequence): workgroups that run side by side then walk the same Q/dO rows a few tiles
  // apart and find them in L2, and the cheap blocks of the short sequences still come last.
  std::vector<int> seq_order(sh->S);
  for (int s = 0; s < sh->S; s++) seq_order[s] = s;
  std::stable_sort(seq_order.begin(), seq_order.end(),
                   [&](int a, int b) { return cu[a + 1] - cu[a] > cu[b + 1] - cu[b]; });
  for (int s : seq_order) {
    if (seq_skip && seq_skip[s]) continue;
    const int32_t L = cu[s + 1] - cu[s];
    const int32_t short_rows = kv_rows_are_short(L, sh->d, sh->Hq / sh->Hkv) ? 1 : 0;
    for (int32_t j0 = 0; j0 < L; j0 += bnk) {
      CostTile c;
      c.t.k_tok0 = cu[s] + j0;
      c.t.k_len = std::min(bnk, L - j0);
      c.t.k_pos0 = j0;
      c.t.q_tok0 = cu[s] + j0;  // first query that sees the block's first key
      c.t.q_rows = L - j0;
      c.t.q_pos0 = j0;
      c.t.out_row0 = cu[s] + j0;
      c.t.aux = short_rows;
      c.cost = (c.t.q_rows + 63) / 64;
      kt.push_back(c);
    }
  }
  if (qt.empty() && kt.empty()) return ZP_OK;
  const size_t n_kv_long = split_kv_tiles(kt);
  const size_t tile_bytes = tile_table_bytes(qt.size() + kt.size());
  const size_t dvec_bytes = align256((size_t)sh->Hq * (size_t)sh->T * sizeof(float));
  if ((rc = check_ws(ws, ws_bytes, tile_bytes + 2 * dvec_bytes))) return rc;
  std::vector<CostTile> all(qt);
  all.insert(all.end(), kt.begin(), kt.end());
  if ((rc = upload_tiles(all, ws, (hipStream_t)stream))) return rc;
  zp_bwd_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v; p.o = (const __bf16 *)o;
  p.dout = (const __bf16 *)dout;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride; p.o_stride = o_stride; p.do_stride = do_stride;
  p.lse = lse;
  p.dvec = (float *)((char *)ws + tile_bytes);
  p.lse2 = (float *)((char *)ws + tile_bytes + dvec_bytes);
  p.dq_tiles = ws_tiles(ws);
  p.kv_tiles = ws_tiles(ws) + qt.size();
  p.work_dq.counters = ws_counters(ws);
  p.work_dq.dyn_div = dyn_div_of(all, 0, qt.size(), 1);
  p.work_kv.dyn_div = dyn_div_of(all, qt.size(), n_kv_long, sh->Hq / sh->Hkv);
  p.work_kv_short.dyn_div = dyn_div_of(all, qt.size() + n_kv_long, kt.size() - n_kv_long, sh->Hq / sh->Hkv);
  p.n_dq_tiles = (int32_t)qt.size(); p.n_kv_tiles = (int32_t)n_kv_long;
  p.kv_tiles_short = p.kv_tiles + n_kv_long; p.n_kv_tiles_short = (int32_t)(kt.size() - n_kv_long);
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv; p.T = sh->T;
  p.scale = eff_scale(sh); p.scale_log2 = p.scale * 1.4426950408889634f;
  p.dq = (__bf16 *)dq; p.dk = (__bf16 *)dk; p.dv = (__bf16 *)dv;
  p.dq_stride = dq_stride; p.dkv_stride = dkv_stride;
  hipError_t e = (hipError_t)zp_launch_attn_bwd(&p, sh->d, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "attn_bwd launch");
  return ZP_OK;
}

// Builds the dQ tiles (blocks of query rows of each pair's Q chunk against its KV chunk) and the dK/dV tiles (blocks
// of key rows of each pair's KV chunk against the Q-chunk rows that can see them) of one ring round.
static void plan_pairs_bwd(const zp_pair *pairs, int n_pairs, int bmq, int bnk, int d, int grp, std::vector<CostTile> &qt,
                           std::vector<CostTile> &kt) {
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    for (int32_t r0 = 0; r0 < pr.q_len; r0 += bmq) {
      CostTile c;
      c.t.q_tok0 = pr.q_tok0 + r0; c.t.q_rows = std::min(bmq, pr.q_len - r0); c.t.q_pos0 = pr.q_pos0 + r0;
      c.t.k_tok0 = pr.k_tok0; c.t.k_len = pr.k_len; c.t.k_pos0 = pr.k_pos0;
      c.t.out_row0 = c.t.q_tok0; c.t.aux = 0;
      c.cost = tile_cost(c.t);
      if (c.cost > 0) qt.push_back(c);
    }
    for (int32_t j0 = 0; j0 < pr.k_len; j0 += bnk) {
      // first query row of the chunk that sees the block's first key
      const int32_t off = std::max(0, pr.k_pos0 + j0 - pr.q_pos0);
      if (off >= pr.q_len) continue;
      CostTile c;
      c.t.k_tok0 = pr.k_tok0 + j0; c.t.k_len = std::min(bnk, pr.k_len - j0); c.t.k_pos0 = pr.k_pos0 + j0;
      c.t.q_tok0 = pr.q_tok0 + off; c.t.q_rows = pr.q_len - off; c.t.q_pos0 = pr.q_pos0 + off;
      c.t.out_row0 = c.t.k_tok0; c.t.aux = kv_rows_are_short(pr.q_len, d, grp) ? 1 : 0;
      c.cost = (c.t.q_rows + 63) / 64;
      kt.push_back(c);
    }
  }
  sort_by_cost(qt);
  sort_by_cost(kt);
}

extern "C" int chunk_attn_partial_bwd(const void *dout, const void *q, const void *k, const void *v, const void *o,
                                      const float *lse, int64_t do_stride, int64_t q_stride, int64_t k_stride,
                                      int64_t v_stride, int64_t o_stride, const zp_pair *pairs, int32_t n_pairs,
                                      float *dq_acc, float *dk_acc, float *dv_acc, const zp_shape *sh, void *ws,
                                      size_t ws_bytes, void *stream) {
  int rc = check_shape(sh);
  if (rc) return rc;
  if (n_pairs < 0) return ZP_EINVAL;
  if (n_pairs == 0 || sh->T == 0) return ZP_OK;
  if (!dout || !q || !k || !v || !o || !lse || !pairs || !dq_acc || !dk_acc || !dv_acc) return ZP_EINVAL;
  if (!aligned16(dout) || !aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(o) || !aligned16(dq_acc) ||
      !aligned16(dk_acc) || !aligned16(dv_acc))
    return ZP_EINVAL;
  if (check_stride(q_stride, sh->Hq, sh->d) || check_stride(o_stride, sh->Hq, sh->d) ||
      check_stride(do_stride, sh->Hq, sh->d) || check_stride(k_stride, sh->Hkv, sh->d) ||
      check_stride(v_stride, sh->Hkv, sh->d))
    return ZP_EINVAL;
  // one ring round: every Q row and every KV row may appear in at most one pair (the kernels add without atomics)
  std::vector<std::pair<int32_t, int32_t>> qr, kr;
  for (int i = 0; i < n_pairs; i++) {
    const zp_pair &pr = pairs[i];
    if (pr.q_len < 0 || pr.k_len < 0 || pr.q_tok0 < 0 || pr.k_tok0 < 0 || pr.q_pos0 < 0 || pr.k_pos0 < 0) return ZP_EINVAL;
    if ((int64_t)pr.q_tok0 + pr.q_len > sh->T || (int64_t)pr.k_tok0 + pr.k_len > sh->T) return ZP_EINVAL;
    if (pr.q_len > 0) qr.push_back({pr.q_tok0, pr.q_tok0 + pr.q_len});
    if (pr.k_len > 0) kr.push_back({pr.k_tok0, pr.k_tok0 + pr.k_len});
  }
  for (auto *ranges : {&qr, &kr}) {
    std::sort(ranges->begin(), ranges->end());
    for (size_t i = 1; i < ranges->size(); i++)
      if ((*ranges)[i].first < (*ranges)[i - 1].second) return ZP_EINVAL;
  }
  const int bmq = zp_attn_bwd_block_rows(sh->d, 0), bnk = zp_attn_bwd_block_rows(sh->d, 1);
  std::vector<CostTile> qt, kt;
  plan_pairs_bwd(pairs, n_pairs, bmq, bnk, sh->d, sh->Hq / sh->Hkv, qt, kt);
  const size_t n_kv_long = split_kv_tiles(kt);
  const size_t tile_bytes = tile_table_bytes(qt.size() + kt.size());
  const size_t dvec_bytes = align256((size_t)sh->Hq * (size_t)sh->T * sizeof(float));
  if ((rc = check_ws(ws, ws_bytes, tile_bytes + 2 * dvec_bytes))) return rc;
  std::vector<CostTile> all(qt);
  all.insert(all.end(), kt.begin(), kt.end());
  if ((rc = upload_tiles(all, ws, (hipStream_t)stream))) return rc;
  zp_bwd_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v; p.o = (const __bf16 *)o;
  p.dout = (const __bf16 *)dout;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride; p.o_stride = o_stride; p.do_stride = do_stride;
  p.lse = lse;
  p.dvec = (float *)((char *)ws + tile_bytes);
  p.lse2 = (float *)((char *)ws + tile_bytes + dvec_bytes);
  p.dq_tiles = ws_tiles(ws);
  p.kv_tiles = ws_tiles(ws) + qt.size();
  p.work_dq.counters = ws_counters(ws);
  p.work_dq.dyn_div = dyn_div_of(all, 0, qt.size(), 1);
  p.work_kv.dyn_div = dyn_div_of(all, qt.size(), n_kv_long, sh->Hq / sh->Hkv);
  p.work_kv_short.dyn_div = dyn_div_of(all, qt.size() + n_kv_long, kt.size() - n_kv_long, sh->Hq / sh->Hkv);
  p.n_dq_tiles = (int32_t)qt.size(); p.n_kv_tiles = (int32_t)n_kv_long;
  p.kv_tiles_short = p.kv_tiles + n_kv_long; p.n_kv_tiles_short = (int32_t)(kt.size() - n_kv_long);
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv; p.T = sh->T;
  p.scale = eff_scale(sh); p.scale_log2 = p.scale * 1.4426950408889634f;
  p.dq = (__bf16 *)dq_acc; p.dk = (__bf16 *)dk_acc; p.dv = (__bf16 *)dv_acc;
  p.dq_stride = (int64_t)sh->Hq * sh->d; p.dkv_stride = (int64_t)sh->Hkv * sh->d;
  p.accumulate = 1;
  hipError_t e = (hipError_t)zp_launch_attn_bwd(&p, sh->d, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "chunk_attn_partial_bwd launch");
  return ZP_OK;
}

extern "C" int zp_accum_to_bf16(const float *src, void *dst, int64_t n, void *stream) {
  if (n < 0 || (n % 8)) return ZP_EINVAL;
  if (n == 0) return ZP_OK;
  if (!src || !dst || !aligned16(src) || !aligned16(dst)) return ZP_EINVAL;
  hipError_t e = (hipError_t)zp_launch_accum_to_bf16(src, dst, n, (hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "accum_to_bf16 launch");
  return ZP_OK;
}
