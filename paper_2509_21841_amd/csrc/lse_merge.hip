// Online-softmax combination of partial attention results (Sec. 3.2, ring attention rounds):
//   LSE = log sum_p exp(LSE_p),  O = sum_p exp(LSE_p - LSE) O_p.
// Elementwise and HBM-bound: each lane owns 4 consecutive head-dim elements of one (row, head), reads the
// n_parts partial LSEs (broadcast within the row) and n_parts float4, writes 4 bf16; two such items are in flight
// per lane.
#include "zp_common.h"

extern "C" void zp_prof_begin(const char *name, hipStream_t stream);
extern "C" void zp_prof_end(hipStream_t stream);

#define ZP_MAX_PARTS 16
struct zp_merge_dev {
  int32_t out_tok0, len, n_parts;
  int32_t part_row0[ZP_MAX_PARTS];
};
struct zp_merge_item { int32_t merge, row0; };  // a band of up to MERGE_ROWS rows of one merge

namespace {
// picked by a sweep over {256, 512, 1024} threads x {4, 8, 16} rows x {1, 2, 4} items in flight per lane (two where the
// registers of 1024 threads allow it, i.e. up to 8 parts)
constexpr int MERGE_NT = 1024;
constexpr int MERGE_ROWS = 8;

// MAXP: compile-time bound of n_parts for this launch (the host picks the smallest of 4, 8, 16 that covers every
// merge), so that the register arrays and the unrolled loops are no larger than needed.
template <int MAXP>
__global__ __launch_bounds__(MERGE_NT) void lse_merge_kernel(const float *__restrict__ o_part, const float *__restrict__ lse_part,
                                                             int64_t part_rows, const zp_merge_dev *__restrict__ merges,
                                                             const zp_merge_item *__restrict__ items, int Hq, int d,
                                                             __bf16 *__restrict__ o, int64_t o_stride, float *__restrict__ lse,
                                                             int64_t T) {
  const zp_merge_item it = items[blockIdx.x];
  const zp_merge_dev mg = merges[it.merge];
  int rows = mg.len - it.row0;
  if (rows > MERGE_ROWS) rows = MERGE_ROWS;
  const int d4 = d >> 2;
  const int per_row = Hq * d4;
  const int total = rows * per_row;
  constexpr int ILP = MAXP <= 8 ? 2 : 1;
  // ILP items per lane and trip: every load of all of them is issued before any arithmetic
  for (int w0 = threadIdx.x; w0 < total; w0 += ILP * MERGE_NT) {
    float lp[ILP][MAXP];
    f32x4 v[ILP][MAXP];
    int rr[ILP], h[ILP], c4[ILP];
#pragma unroll
    for (int u = 0; u < ILP; u++) {
      const int w = w0 + u * MERGE_NT;
      if (w < total) {
        const int r = w / per_row, rem = w - r * per_row;
        h[u] = rem / d4; c4[u] = rem - h[u] * d4; rr[u] = it.row0 + r;
#pragma unroll
        for (int p = 0; p < MAXP; p++)
          if (p < mg.n_parts) {
            lp[u][p] = lse_part[(int64_t)h[u] * part_rows + mg.part_row0[p] + rr[u]];
            v[u][p] = __builtin_nontemporal_load((const f32x4 *)(o_part + ((int64_t)(mg.part_row0[p] + rr[u]) * Hq + h[u]) * d) + c4[u]);
          }
      }
    }
#pragma unroll
    for (int u = 0; u < ILP; u++) {
      const int w = w0 + u * MERGE_NT;
      if (w < total) {
        float mx = -INFINITY;
#pragma unroll
        for (int p = 0; p < MAXP; p++)
          if (p < mg.n_parts) mx = fmaxf(mx, lp[u][p]);
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
        float L = -INFINITY;
        if (mx != -INFINITY) {
          float sum = 0.f;
#pragma unroll
          for (int p = 0; p < MAXP; p++)
            if (p < mg.n_parts) sum += __expf(lp[u][p] - mx);
          L = mx + __logf(sum);
#pragma unroll
          for (int p = 0; p < MAXP; p++)
            if (p < mg.n_parts && lp[u][p] != -INFINITY) acc += __expf(lp[u][p] - L) * v[u][p];
        }
        const int64_t t = (int64_t)mg.out_tok0 + rr[u];
        bf16x4 ob = {(__bf16)acc[0], (__bf16)acc[1], (__bf16)acc[2], (__bf16)acc[3]};
        __builtin_nontemporal_store(ob, (bf16x4 *)(o + t * o_stride + (int64_t)h[u] * d + 4 * c4[u]));
        if (c4[u] == 0) lse[(int64_t)h[u] * T + t] = L;
      }
    }
  }
}
}  // namespace


namespace {
// float accumulators -> bfloat16, 8 elements per lane
__global__ __launch_bounds__(256) void accum_to_bf16_kernel(const float *__restrict__ src, __bf16 *__restrict__ dst, int64_t n8) {
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < n8; i += (int64_t)gridDim.x * 256) {
    const f32x4 a = __builtin_nontemporal_load((const f32x4 *)src + 2 * i);
    const f32x4 b = __builtin_nontemporal_load((const f32x4 *)src + 2 * i + 1);
    bf16x8 o = {(__bf16)a[0], (__bf16)a[1], (__bf16)a[2], (__bf16)a[3], (__bf16)b[0], (__bf16)b[1], (__bf16)b[2], (__bf16)b[3]};
    *((bf16x8 *)dst + i) = o;
  }
}
}  // namespace

extern "C" int zp_launch_accum_to_bf16(const float *src, void *dst, int64_t n, hipStream_t stream) {
  if (n == 0) return 0;
  const int64_t n8 = n / 8;
  int64_t grid = (n8 + 255) / 256;
  if (grid > 256 * 64) grid = 256 * 64;
  zp_prof_begin("accum_to_bf16", stream);
  hipLaunchKernelGGL(accum_to_bf16_kernel, dim3((unsigned)grid), dim3(256), 0, stream, src, (__bf16 *)dst, n8);
  zp_prof_end(stream);
  return (int)hipGetLastError();
}

extern "C" int zp_merge_rows_per_item(void) { return MERGE_ROWS; }

extern "C" int zp_launch_lse_merge(const float *o_part, const float *lse_part, int64_t part_rows, const void *merges_dev,
                                   const void *items_dev, int n_items, int Hq, int d, void *o, int64_t o_stride,
                                   float *lse, int64_t T, int max_parts, hipStream_t stream) {
  if (n_items == 0) return 0;
  zp_prof_begin("lse_merge", stream);
#define ZP_MERGE_LAUNCH(MAXP)                                                                                      \
  hipLaunchKernelGGL(lse_merge_kernel<MAXP>, dim3(n_items), dim3(MERGE_NT), 0, stream, o_part, lse_part, part_rows, \
                     (const zp_merge_dev *)merges_dev, (const zp_merge_item *)items_dev, Hq, d, (__bf16 *)o, o_stride, \
                     lse, T)
  if (max_parts <= 4) ZP_MERGE_LAUNCH(4);
  else if (max_parts <= 8) ZP_MERGE_LAUNCH(8);
  else ZP_MERGE_LAUNCH(16);
#undef ZP_MERGE_LAUNCH
  zp_prof_end(stream);
  return (int)hipGetLastError();
}
