// varlen_attn_fwd for callers that cannot allocate or upload: the ordered tile table of the forward kernel is
// built ON the device, from sequence boundaries passed by value in the launch arguments, into a file-scope device
// array. Nothing is allocated, no host buffer is read by the device, so the call can sit under HIP graph capture or in
// a serving loop that forbids hipMalloc. The attention kernel itself is the one varlen_attn_fwd launches.
#include <hip/hip_runtime.h>

#include <cmath>
#include <mutex>

#include "../../include/zeppelin_attn.h"
#include "zp_common.h"

extern "C" int zp_launch_attn_fwd(const zp_attn_params *p, int d, int partial, int block_rows, hipStream_t stream);
extern "C" int zp_attn_fwd_block_rows(int d);
extern "C" int zp_report_hip_error(int hip_error, const char *what);

// The forward kernel's work counters (ZP_COUNTER_BYTES) and its tile table: ZP_NOALLOC_MAX_TILES records of 32 bytes. One copy per GPU the library runs on, held until the
// process ends. In host code this name is only a handle for hipGetSymbolAddress, never a device address.
static __device__ __align__(256) unsigned char scratch[ZP_COUNTER_BYTES + (size_t)ZP_NOALLOC_MAX_TILES * sizeof(zp_tile)];

namespace {

constexpr int BM = 128;  // query rows per tile (the forward kernel's block)

// Launch arguments of the planning kernel: the batch description by value (under 4 KB of kernel arguments).
struct PlanArgs {
  int32_t S;
  int32_t n_tiles;
  int32_t cu[ZP_NOALLOC_MAX_SEQS + 1];
  uint32_t skip_bits[(ZP_NOALLOC_MAX_SEQS + 31) / 32];
};
static_assert(sizeof(PlanArgs) + sizeof(void *) <= 4096, "kernel arguments are limited to 4 KB");

// Query blocks of sequence s (none if it is flagged).
__device__ __forceinline__ void seq_blocks(const PlanArgs &a, int s, int &L, int &n_blk) {
  const bool skip = (a.skip_bits[s >> 5] >> (s & 31)) & 1u;
  L = a.cu[s + 1] - a.cu[s];
  n_blk = skip ? 0 : (L + BM - 1) / BM;
}

// One thread per tile, in the order the host planner of varlen_attn_fwd uses: sequence by sequence, longest first
// (equal lengths: lower index first), inside a sequence the last query block first. Tile (s, b) therefore sits behind
// all blocks of the sequences ordered before s and behind the later blocks of s -- a closed form, so no sort and no
// atomics, and the table is the same on every call.
__global__ __launch_bounds__(256) void plan_fwd_tiles_kernel(PlanArgs a, int32_t *counters, zp_tile *tiles) {
  __shared__ int first_tile[ZP_NOALLOC_MAX_SEQS + 1];
  // the attention kernel's work counters start from zero on every call
  if (blockIdx.x == 0 && threadIdx.x < 8) counters[threadIdx.x * ZP_COUNTER_STRIDE] = 0;
  for (int s = threadIdx.x; s < a.S; s += blockDim.x) {
    int L, nb;
    seq_blocks(a, s, L, nb);
    first_tile[s + 1] = nb;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    first_tile[0] = 0;
    for (int s = 0; s < a.S; s++) first_tile[s + 1] += first_tile[s];
  }
  __syncthreads();
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= a.n_tiles || i >= first_tile[a.S]) return;
  // the sequence that owns tile i in (sequence, block) numbering: last s with first_tile[s] <= i
  int lo = 0, hi = a.S - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (first_tile[mid] <= i) lo = mid; else hi = mid - 1;
  }
  const int s = lo, b = i - first_tile[s];
  int L, nb;
  seq_blocks(a, s, L, nb);
  int slot = nb - 1 - b;
  for (int s2 = 0; s2 < a.S; s2++) {
    int L2, nb2;
    seq_blocks(a, s2, L2, nb2);
    if (L2 > L || (L2 == L && s2 < s)) slot += nb2;
  }
  zp_tile t;
  t.q_tok0 = a.cu[s] + b * BM;
  t.q_rows = L - b * BM < BM ? L - b * BM : BM;
  t.q_pos0 = b * BM;
  t.k_tok0 = a.cu[s];
  t.k_len = L;
  t.k_pos0 = 0;
  t.out_row0 = t.q_tok0;
  t.aux = 0;
  tiles[slot] = t;
}

std::mutex g_mu;
constexpr int MAX_DEVICES = 64;
void *g_scratch_ptr[MAX_DEVICES] = {};

// Device address of this GPU's copy of the array, looked up once per device with that device current.
int scratch_for_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return zp_report_hip_error((int)e, "hipGetDevice");
  if (dev < 0 || dev >= MAX_DEVICES) return ZP_EUNSUPPORTED;
  std::lock_guard<std::mutex> lk(g_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return zp_report_hip_error((int)e, "hipGetSymbolAddress");
    if (!ptr) return zp_report_hip_error((int)hipErrorInvalidSymbol, "hipGetSymbolAddress");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return ZP_OK;
}

}  // namespace

extern "C" int varlen_attn_fwd_noalloc(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride,
                                       int64_t v_stride, const int32_t *cu, const uint8_t *seq_skip, void *o,
                                       int64_t o_stride, float *lse, const zp_shape *sh, void *stream) {
  // the same argument checks as varlen_attn_fwd, all before anything touches the device
  if (!sh) return ZP_EINVAL;
  if (sh->T < 0 || sh->S < 0 || sh->Hq <= 0 || sh->Hkv <= 0) return ZP_EINVAL;
  if (!(sh->scale >= 0.f) || std::isinf(sh->scale)) return ZP_EINVAL;
  if (sh->d != 64 && sh->d != 128) return ZP_EUNSUPPORTED;
  if (sh->Hq % sh->Hkv) return ZP_EUNSUPPORTED;
  if (!cu || cu[0] != 0) return ZP_EINVAL;
  for (int s = 0; s < sh->S; s++)
    if (cu[s + 1] < cu[s]) return ZP_EINVAL;
  if (cu[sh->S] != sh->T) return ZP_EINVAL;
  if (sh->T == 0) return ZP_OK;
  if (!q || !k || !v || !o || !lse) return ZP_EINVAL;
  if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return ZP_EINVAL;
  auto bad_stride = [&](int64_t st, int H) { return st < (int64_t)H * sh->d || (st % 8) || st > (1 << 24); };
  if (bad_stride(q_stride, sh->Hq) || bad_stride(o_stride, sh->Hq) || bad_stride(k_stride, sh->Hkv) ||
      bad_stride(v_stride, sh->Hkv))
    return ZP_EINVAL;
  // the fixed limits of this entry point
  if (sh->S > ZP_NOALLOC_MAX_SEQS) return ZP_ETOOLARGE;
  if (zp_attn_fwd_block_rows(sh->d) != BM) return ZP_EUNSUPPORTED;
  PlanArgs a;
  a.S = sh->S;
  for (size_t i = 0; i < sizeof(a.skip_bits) / sizeof(a.skip_bits[0]); i++) a.skip_bits[i] = 0;
  int64_t n_tiles = 0;
  for (int s = 0; s <= sh->S; s++) a.cu[s] = cu[s];
  for (int s = 0; s < sh->S; s++) {
    if (seq_skip && seq_skip[s]) { a.skip_bits[s >> 5] |= 1u << (s & 31); continue; }
    n_tiles += ((int64_t)cu[s + 1] - cu[s] + BM - 1) / BM;
  }
  if (n_tiles > ZP_NOALLOC_MAX_TILES) return ZP_ETOOLARGE;
  if (n_tiles == 0) return ZP_OK;
  a.n_tiles = (int32_t)n_tiles;

  void *tiles = nullptr;
  int rc = scratch_for_current_device(&tiles);
  if (rc) return rc;
  // Every slot the attention kernel reads is rewritten by the planning kernel of the same call, on the same stream,
  // and so are the work counters in front of the table: nothing of an earlier call survives into this one.
  hipLaunchKernelGGL(plan_fwd_tiles_kernel, dim3((unsigned)((n_tiles + 255) / 256)), dim3(256), 0, (hipStream_t)stream, a,
                     (int32_t *)tiles, (zp_tile *)((char *)tiles + ZP_COUNTER_BYTES));
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return zp_report_hip_error((int)e, "plan_fwd_tiles launch");

  zp_attn_params p{};
  p.q = (const __bf16 *)q; p.k = (const __bf16 *)k; p.v = (const __bf16 *)v;
  p.q_stride = q_stride; p.k_stride = k_stride; p.v_stride = v_stride;
  p.tiles = (const zp_tile *)((char *)tiles + ZP_COUNTER_BYTES); p.n_tiles = (int32_t)n_tiles; p.work.counters = (int32_t *)tiles;
  p.Hq = sh->Hq; p.Hkv = sh->Hkv; p.grp = sh->Hq / sh->Hkv;
  p.scale = sh->scale > 0.f ? sh->scale : 1.0f / std::sqrt((float)sh->d);
  p.scale_log2 = p.scale * 1.4426950408889634f;
  p.o = o; p.o_stride = o_stride; p.lse = lse; p.lse_stride = sh->T;
  e = (hipError_t)zp_launch_attn_fwd(&p, sh->d, 0, BM, (hipStream_t)stream);
  if (e != hipSuccess) return zp_report_hip_error((int)e, "attn_fwd launch");
  return ZP_OK;
}
