// Token move of the remapping layer (Sec. 3.4): a row gather / scatter on raw bytes, bound by HBM bandwidth.
// Every lane moves 16 bytes per access; a workgroup owns a band of consecutive index entries so the index
// array is read once, coalesced, and each row is copied by consecutive lanes (fully coalesced both ways).
#include "zp_common.h"

namespace {

constexpr int REMAP_NT = 1024;  // measured best on MI355X: 1024 threads, 4 x 16 B in flight per thread
constexpr int REMAP_UNROLL = 4;

// chunks_per_row = row_bytes / 16. Each block handles `rows_per_block` index entries.
template <bool SCATTER, bool POW2>
__global__ __launch_bounds__(REMAP_NT) void remap_kernel(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                          const int32_t *__restrict__ idx, int64_t n_rows,
                                                          int32_t cpr, int32_t cpr_shift, int32_t rows_per_block) {
  const int64_t row0 = (int64_t)blockIdx.x * rows_per_block;
  int64_t rows = n_rows - row0;
  if (rows > rows_per_block) rows = rows_per_block;
  const int total = (int)rows * cpr;  // chunks this block moves
  for (int base = threadIdx.x; base < total; base += REMAP_NT * REMAP_UNROLL) {
    u32x4 val[REMAP_UNROLL];
    int64_t doff[REMAP_UNROLL];
#pragma unroll
    for (int u = 0; u < REMAP_UNROLL; u++) {
      int lc = base + u * REMAP_NT;
      if (lc < total) {
        int r = POW2 ? (lc >> cpr_shift) : (lc / cpr);
        int c = lc - r * cpr;
        int64_t other = idx[row0 + r];
        int64_t s_row = SCATTER ? (row0 + r) : other;
        int64_t d_row = SCATTER ? other : (row0 + r);
        val[u] = __builtin_nontemporal_load(&src[s_row * cpr + c]);
        doff[u] = d_row * cpr + c;
      }
    }
#pragma unroll
    for (int u = 0; u < REMAP_UNROLL; u++) {
      int lc = base + u * REMAP_NT;
      if (lc < total) __builtin_nontemporal_store(val[u], &dst[doff[u]]);
    }
  }
}

}  // namespace

extern "C" void zp_prof_begin(const char *name, hipStream_t stream);
extern "C" void zp_prof_end(hipStream_t stream);

extern "C" int zp_launch_remap(const void *src, void *dst, int64_t row_bytes, const int32_t *idx, int64_t n_rows,
                               int mode, hipStream_t stream) {
  if (n_rows == 0) return 0;
  const int cpr = (int)(row_bytes / 16);
  int shift = -1;
  if ((cpr & (cpr - 1)) == 0) { shift = 0; while ((1 << shift) < cpr) shift++; }
  // 64 KiB per block for short rows, 128 KiB for long ones (measured), at least one row
  int rpb = (int)((row_bytes <= 4096 ? 65536 : 131072) / row_bytes);
  if (rpb < 1) rpb = 1;
  const int64_t grid = (n_rows + rpb - 1) / rpb;
  const u32x4 *s = (const u32x4 *)src;
  u32x4 *d = (u32x4 *)dst;
  zp_prof_begin("remap", stream);
  if (mode == 0) {
    if (shift >= 0) hipLaunchKernelGGL((remap_kernel<false, true>), dim3((unsigned)grid), dim3(REMAP_NT), 0, stream, s, d, idx, n_rows, cpr, shift, rpb);
    else hipLaunchKernelGGL((remap_kernel<false, false>), dim3((unsigned)grid), dim3(REMAP_NT), 0, stream, s, d, idx, n_rows, cpr, shift, rpb);
  } else {
    if (shift >= 0) hipLaunchKernelGGL((remap_kernel<true, true>), dim3((unsigned)grid), dim3(REMAP_NT), 0, stream, s, d, idx, n_rows, cpr, shift, rpb);
    else hipLaunchKernelGGL((remap_kernel<true, false>), dim3((unsigned)grid), dim3(REMAP_NT), 0, stream, s, d, idx, n_rows, cpr, shift, rpb);
  }
  zp_prof_end(stream);
  return (int)hipGetLastError();
}
