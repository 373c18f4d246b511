// Backward of causal varlen attention, deterministic and atomics-free: two kernels.
//   attn_bwd_dq   owns a block of query rows, walks the visible key tiles:  S^T = K Q^T, dP^T = V dO^T,
//                 dS^T = P^T o (dP^T - D), dQ^T += K^T dS^T.  Also computes D_i = dO_i . O_i and stores it.
//   attn_bwd_dkdv owns a block of key rows, walks the query tiles at or after it and the query heads of its
//                 KV group:  S = Q K^T, dP = dO V^T, dV^T += dO^T P, dK^T += Q^T dS.
// Both recompute P from the forward's LSE. In each kernel the accumulator of the first two products already
// has the register layout the third/fourth product needs as its B operand; the transposed A operands
// (K^T, Q^T, dO^T) come from the row-major LDS tiles through the transposing LDS read.
#include "zp_common.h"

struct zp_bwd_params {
  const __bf16 *q, *k, *v, *o, *dout;
  int64_t q_stride, k_stride, v_stride, o_stride, do_stride;
  const float *lse;   // [Hq][T]
  float *dvec;        // [Hq][T] scratch: D_i = dO_i . O_i
  const zp_tile *dq_tiles;
  const zp_tile *kv_tiles;
  int32_t n_dq_tiles, n_kv_tiles, Hq, Hkv, grp, T;
  float scale_log2, scale;
  __bf16 *dq, *dk, *dv;
  int64_t dq_stride, dkv_stride;
};

namespace {

constexpr int BWD_NT = 256;
constexpr float LOG2E = 1.4426950408889634f;

// cooperative global -> register -> LDS staging of a [64][D] bf16 tile (zp_swz layout)
template <int D>
struct TileStage {
  static constexpr int CPT = 64 * D / 8 / BWD_NT;  // 16-byte chunks per thread
  u32x4 r[CPT];
  __device__ __forceinline__ void load(const __bf16 *base, int64_t stride, int row0, int rows_total, int tid) {
#pragma unroll
    for (int n = 0; n < CPT; n++) {
      int id = tid + n * BWD_NT, rr = id / (D / 8), c = id % (D / 8);
      if (row0 + rr < rows_total) r[n] = *(const u32x4 *)(base + (int64_t)(row0 + rr) * stride + c * 8);
      else r[n] = u32x4{0, 0, 0, 0};
    }
  }
  __device__ __forceinline__ void store(char *lds, int tid) const {
#pragma unroll
    for (int n = 0; n < CPT; n++) {
      int id = tid + n * BWD_NT, rr = id / (D / 8), c = id % (D / 8);
      zp_lds_write16(lds, zp_swz<D>(rr, c), r[n]);
    }
  }
};

template <int D>
__device__ __forceinline__ void store_acc_rows(__bf16 *dst, const f32x16 (&acc)[D / 32], float mul) {
#pragma unroll
  for (int db = 0; db < D / 32; db++)
#pragma unroll
    for (int b = 0; b < 4; b++) {
      bf16x4 v4 = {(__bf16)(acc[db][4 * b] * mul), (__bf16)(acc[db][4 * b + 1] * mul),
                   (__bf16)(acc[db][4 * b + 2] * mul), (__bf16)(acc[db][4 * b + 3] * mul)};
      *(bf16x4 *)(dst + db * 32 + b * 8) = v4;
    }
}

// ------------------------------------------------------------------------------------------- dQ
template <int D>
__global__ __launch_bounds__(BWD_NT) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_bwd_dq_kernel(zp_bwd_params p) {
  constexpr int TILEB = 64 * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Ks = smem;               // [2][64][D]
  char *Vs = smem + 2 * TILEB;   // [2][64][D]

  int unit, hh;
  zp_block_to_unit(blockIdx.x, p.grp, unit, hh);
  if (unit >= p.n_dq_tiles * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const int h = g * p.grp + hh;
  const zp_tile t = p.dq_tiles[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ql = lane & 31, hi = lane >> 5;
  const int row = w * 32 + ql;
  const bool row_ok = row < t.q_rows;
  const int64_t tok = (int64_t)t.q_tok0 + row;

  auto nvis_of = [&](int r) {
    int n = t.q_pos0 + r - t.k_pos0 + 1;
    return n < 0 ? 0 : (n > t.k_len ? t.k_len : n);
  };
  const int nvis_lane = nvis_of(row);
  const int nvis_w_min = nvis_of(w * 32), nvis_w_max = nvis_of(w * 32 + 31);
  const int n_kt = (nvis_of(t.q_rows - 1) + 63) / 64;

  bf16x8 qreg[D / 16], doreg[D / 16];
  float dsum = 0.f;
  {
    const __bf16 *qp = p.q + tok * p.q_stride + (int64_t)h * D + 8 * hi;
    const __bf16 *dop = p.dout + tok * p.do_stride + (int64_t)h * D + 8 * hi;
    const __bf16 *op = p.o + tok * p.o_stride + (int64_t)h * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (row_ok) {
        qreg[kk] = *(const bf16x8 *)(qp + 16 * kk);
        doreg[kk] = *(const bf16x8 *)(dop + 16 * kk);
        bf16x8 ov = *(const bf16x8 *)(op + 16 * kk);
#pragma unroll
        for (int e = 0; e < 8; e++) dsum += (float)doreg[kk][e] * (float)ov[e];
      } else {
        qreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        doreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
  }
  const float Dq = zp_pair_sum(dsum);
  float lse2 = 0.f;
  if (row_ok) {
    lse2 = p.lse[(int64_t)h * p.T + tok] * LOG2E;
    if (hi == 0) p.dvec[(int64_t)h * p.T + tok] = Dq;
  }

  const __bf16 *kbase = p.k + (int64_t)t.k_tok0 * p.k_stride + (int64_t)g * D;
  const __bf16 *vbase = p.v + (int64_t)t.k_tok0 * p.v_stride + (int64_t)g * D;
  TileStage<D> kst, vst;

  f32x16 dq_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) dq_acc[i][r] = 0.f;
  const float c_log2 = p.scale_log2;

  if (n_kt > 0) {
    kst.load(kbase, p.k_stride, 0, t.k_len, tid);
    vst.load(vbase, p.v_stride, 0, t.k_len, tid);
    kst.store(Ks, tid);
    vst.store(Vs, tid);
  }
  __syncthreads();

  const int g16 = lane >> 4, i16 = lane & 15;
  const int trow = 4 * (g16 >> 1) + (i16 >> 2);
  const int tcol = 16 * (g16 & 1) + 4 * (i16 & 3);

  for (int it = 0; it < n_kt; it++) {
    const int j0 = it * 64, buf = it & 1;
    if (it + 1 < n_kt) {
      kst.load(kbase, p.k_stride, j0 + 64, t.k_len, tid);
      vst.load(vbase, p.v_stride, j0 + 64, t.k_len, tid);
    }
    if (j0 < nvis_w_max) {
      const char *Kb = Ks + buf * TILEB;
      const char *Vb = Vs + buf * TILEB;
      const bool need_mask = j0 + 64 > nvis_w_min;
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
          bf16x8 a = zp_lds_read16(Kb, zp_swz<D>(kb * 32 + ql, 2 * kk + hi));
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[kk], s, 0, 0, 0);
        }
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
          bf16x8 a = zp_lds_read16(Vb, zp_swz<D>(kb * 32 + ql, 2 * kk + hi));
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, doreg[kk], dp, 0, 0, 0);
        }
        bf16x8 dsb[2];
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float sv = s[r];
          if (need_mask) {
            int j = j0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (j >= nvis_lane) sv = -INFINITY;
          }
          float pv = zp_exp2(__builtin_fmaf(sv, c_log2, -lse2));
          dsb[r >> 3][r & 7] = (__bf16)(pv * (dp[r] - Dq));
        }
#pragma unroll
        for (int m = 0; m < 2; m++)
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            bf16x4 lo = zp_lds_read_tr(Kb, zp_swz_col<D>(kb * 32 + m * 16 + trow, db * 32 + tcol));
            bf16x4 hi4 = zp_lds_read_tr(Kb, zp_swz_col<D>(kb * 32 + m * 16 + 8 + trow, db * 32 + tcol));
            dq_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zp_cat(lo, hi4), dsb[m], dq_acc[db], 0, 0, 0);
          }
      }
    }
    if (it + 1 < n_kt) {
      kst.store(Ks + (buf ^ 1) * TILEB, tid);
      vst.store(Vs + (buf ^ 1) * TILEB, tid);
    }
    __syncthreads();
  }

  if (row_ok) store_acc_rows<D>(p.dq + tok * p.dq_stride + (int64_t)h * D + 4 * hi, dq_acc, p.scale);
}

// ------------------------------------------------------------------------------------------- dK, dV
// Tile fields: k_tok0/k_len/k_pos0 = this block of key rows; q_tok0/q_rows/q_pos0 = the query rows of the
// same sequence from the first one that can see the block's first key to the end of the sequence.
template <int D>
__global__ __launch_bounds__(BWD_NT) __attribute__((amdgpu_waves_per_eu(1, 1))) void attn_bwd_dkdv_kernel(zp_bwd_params p) {
  constexpr int TILEB = 64 * D * 2;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Qs = smem;                              // [2][64][D]
  char *Os = smem + 2 * TILEB;                  // [2][64][D]  (dO)
  float *Ls = (float *)(smem + 4 * TILEB);      // [2][64] LSE * log2(e)
  float *Ds = Ls + 128;                         // [2][64] D

  const int unit = blockIdx.x;
  if (unit >= p.n_kv_tiles * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const zp_tile t = p.kv_tiles[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int kl = lane & 31, hi = lane >> 5;
  const int krow = w * 32 + kl;
  const bool key_ok = krow < t.k_len;
  const int64_t ktok = (int64_t)t.k_tok0 + krow;
  const int kpos = t.k_pos0 + krow;

  bf16x8 kreg[D / 16], vreg[D / 16];
  {
    const __bf16 *kp = p.k + ktok * p.k_stride + (int64_t)g * D + 8 * hi;
    const __bf16 *vp = p.v + ktok * p.v_stride + (int64_t)g * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (key_ok) {
        kreg[kk] = *(const bf16x8 *)(kp + 16 * kk);
        vreg[kk] = *(const bf16x8 *)(vp + 16 * kk);
      } else {
        kreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
        vreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
      }
    }
  }

  f32x16 dk_acc[D / 32], dv_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) { dk_acc[i][r] = 0.f; dv_acc[i][r] = 0.f; }
  const float c_log2 = p.scale_log2;

  const int n_qt = (t.q_rows + 63) / 64;
  const int n_it = n_qt * p.grp;  // iterations: heads of the group outermost, query tiles innermost
  TileStage<D> qst, ost;
  float lpre = 0.f, dpre = 0.f;

  auto load_it = [&](int it) {
    const int hh = it / n_qt, i0 = (it - hh * n_qt) * 64;
    const int h = g * p.grp + hh;
    const __bf16 *qb = p.q + (int64_t)t.q_tok0 * p.q_stride + (int64_t)h * D;
    const __bf16 *ob = p.dout + (int64_t)t.q_tok0 * p.do_stride + (int64_t)h * D;
    qst.load(qb, p.q_stride, i0, t.q_rows, tid);
    ost.load(ob, p.do_stride, i0, t.q_rows, tid);
    if (tid < 64) {
      const bool ok = i0 + tid < t.q_rows;
      const int64_t idx = (int64_t)h * p.T + t.q_tok0 + i0 + tid;
      lpre = ok ? p.lse[idx] * LOG2E : 0.f;
      dpre = ok ? p.dvec[idx] : 0.f;
    }
  };
  auto store_it = [&](int buf) {
    qst.store(Qs + buf * TILEB, tid);
    ost.store(Os + buf * TILEB, tid);
    if (tid < 64) {
      Ls[buf * 64 + tid] = lpre;
      Ds[buf * 64 + tid] = dpre;
    }
  };

  if (n_it > 0) {
    load_it(0);
    store_it(0);
  }
  __syncthreads();

  const int g16 = lane >> 4, i16 = lane & 15;
  const int trow = 4 * (g16 >> 1) + (i16 >> 2);
  const int tcol = 16 * (g16 & 1) + 4 * (i16 & 3);
  const int kpos_w_min = t.k_pos0 + w * 32, kpos_w_max = t.k_pos0 + w * 32 + 31;

  for (int it = 0; it < n_it; it++) {
    const int buf = it & 1;
    const int hh = it / n_qt, i0 = (it - hh * n_qt) * 64;
    if (it + 1 < n_it) load_it(it + 1);

    const int qpos0 = t.q_pos0 + i0;  // position of the tile's first query
    if (qpos0 + 63 >= kpos_w_min) {   // otherwise every query of the tile precedes every key of this wave
      const char *Qb = Qs + buf * TILEB;
      const char *Ob = Os + buf * TILEB;
      const bool need_mask = qpos0 < kpos_w_max;
#pragma unroll
      for (int qb = 0; qb < 2; qb++) {
        f32x16 s, dp;
#pragma unroll
        for (int r = 0; r < 16; r++) { s[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
          bf16x8 a = zp_lds_read16(Qb, zp_swz<D>(qb * 32 + kl, 2 * kk + hi));
          s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kreg[kk], s, 0, 0, 0);
        }
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
          bf16x8 a = zp_lds_read16(Ob, zp_swz<D>(qb * 32 + kl, 2 * kk + hi));
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, vreg[kk], dp, 0, 0, 0);
        }
        bf16x8 pb[2], dsb[2];
#pragma unroll
        for (int b = 0; b < 4; b++) {
          const f32x4 l4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)(Ls + buf * 64) + (qb * 32 + 8 * b + 4 * hi) * 4);
          const f32x4 d4 = *(const ZP_LDS f32x4 *)((const ZP_LDS char *)(Ds + buf * 64) + (qb * 32 + 8 * b + 4 * hi) * 4);
#pragma unroll
          for (int c = 0; c < 4; c++) {
            const int r = 4 * b + c;
            float sv = s[r];
            if (need_mask) {
              const int qpos = qpos0 + qb * 32 + 8 * b + 4 * hi + c;
              if (qpos < kpos) sv = -INFINITY;
            }
            const float pv = zp_exp2(__builtin_fmaf(sv, c_log2, -l4[c]));
            pb[r >> 3][r & 7] = (__bf16)pv;
            dsb[r >> 3][r & 7] = (__bf16)(pv * (dp[r] - d4[c]));
          }
        }
#pragma unroll
        for (int m = 0; m < 2; m++)
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            bf16x4 lo = zp_lds_read_tr(Ob, zp_swz_col<D>(qb * 32 + m * 16 + trow, db * 32 + tcol));
            bf16x4 hi4 = zp_lds_read_tr(Ob, zp_swz_col<D>(qb * 32 + m * 16 + 8 + trow, db * 32 + tcol));
            dv_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zp_cat(lo, hi4), pb[m], dv_acc[db], 0, 0, 0);
            bf16x4 lo2 = zp_lds_read_tr(Qb, zp_swz_col<D>(qb * 32 + m * 16 + trow, db * 32 + tcol));
            bf16x4 hi2 = zp_lds_read_tr(Qb, zp_swz_col<D>(qb * 32 + m * 16 + 8 + trow, db * 32 + tcol));
            dk_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zp_cat(lo2, hi2), dsb[m], dk_acc[db], 0, 0, 0);
          }
      }
    }
    if (it + 1 < n_it) store_it(buf ^ 1);
    __syncthreads();
  }

  if (key_ok) {
    store_acc_rows<D>(p.dk + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dk_acc, p.scale);
    store_acc_rows<D>(p.dv + ktok * p.dkv_stride + (int64_t)g * D + 4 * hi, dv_acc, 1.0f);
  }
}

}  // namespace

extern "C" void zp_prof_begin(const char *name, hipStream_t stream);
extern "C" void zp_prof_end(hipStream_t stream);

extern "C" int zp_attn_bwd_block_rows(int d, int which) { (void)d; (void)which; return 128; }

extern "C" int zp_launch_attn_bwd(const zp_bwd_params *p, int d, hipStream_t stream) {
  const int dq_units = p->n_dq_tiles * p->Hkv;
  const int kv_units = p->n_kv_tiles * p->Hkv;
  if (dq_units > 0) {
    const int grid = ((dq_units + 7) / 8) * 8 * p->grp;
    zp_prof_begin("attn_bwd_dq", stream);
    if (d == 128) hipLaunchKernelGGL((attn_bwd_dq_kernel<128>), dim3(grid), dim3(BWD_NT), 4 * 64 * 128 * 2, stream, *p);
    else hipLaunchKernelGGL((attn_bwd_dq_kernel<64>), dim3(grid), dim3(BWD_NT), 4 * 64 * 64 * 2, stream, *p);
    zp_prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  if (kv_units > 0) {
    zp_prof_begin("attn_bwd_dkdv", stream);
    if (d == 128) hipLaunchKernelGGL((attn_bwd_dkdv_kernel<128>), dim3(kv_units), dim3(BWD_NT), 4 * 64 * 128 * 2 + 1024, stream, *p);
    else hipLaunchKernelGGL((attn_bwd_dkdv_kernel<64>), dim3(kv_units), dim3(BWD_NT), 4 * 64 * 64 * 2 + 1024, stream, *p);
    zp_prof_end(stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (int)e;
  }
  return 0;
}
