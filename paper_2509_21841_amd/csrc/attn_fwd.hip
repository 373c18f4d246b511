// Causal attention forward over a work list of (query block, key run) tiles: bf16 MFMA for K Q^T and V^T P^T,
// K/V tiles staged through LDS, online softmax kept per lane.
//
// Orientation. Scores are computed transposed, S^T = K Q^T with the 32x32x16 MFMA: the accumulator lane
// (l%32, l/32) then holds ONE query (column l%32) and 16 keys per 32-key block (rows 8b + 4(l/32) + c),
// so the row maximum and row sum of the softmax are in-lane reductions plus one exchange with lane l^32,
// and the rescale factor is a per-lane scalar. The bf16 probabilities are already laid out as the B
// operand of O^T += V^T P^T (k-slot i of MFMA m <-> accumulator register 8m+i), and V^T comes from the
// row-major V tile in LDS through the transposing LDS read with the matching key order.
#include "zp_common.h"

namespace {

constexpr int BN = 64;  // keys per LDS tile

template <int D, int NW>
struct FwdCfg {
  static constexpr int NT = NW * 64;
  static constexpr int BM = NW * 32;
  static constexpr int ROWB = D * 2;                   // bytes per tile row
  static constexpr int TILEB = BN * ROWB;              // bytes per K (or V) tile
  static constexpr int CHUNKS = BN * D / 8;            // 16-byte chunks per tile
  static constexpr int CPT = CHUNKS / NT;              // chunks per thread
  static_assert(CHUNKS % NT == 0, "tile chunks must divide over the threads");
};

template <int D, int NW, bool PARTIAL>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_kernel(zp_attn_params p) {
  using C = FwdCfg<D, NW>;
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Ks = smem;                  // [2][BN][D] bf16, row-read swizzle
  char *Vs = smem + 2 * C::TILEB;   // [2][BN][D] bf16, transposed-read swizzle

  int unit, hh;
  zp_block_to_unit(blockIdx.x, p.grp, unit, hh);
  if (unit >= p.n_tiles * p.Hkv) return;
  const int tile_idx = unit / p.Hkv, g = unit - tile_idx * p.Hkv;
  const int h = g * p.grp + hh;
  const zp_tile t = p.tiles[tile_idx];

  const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
  const int ql = lane & 31, hi = lane >> 5;
  const int row = w * 32 + ql;  // this lane's query row inside the block
  const bool row_ok = row < t.q_rows;

  // number of keys of the run visible to a query row r: clamp(q_pos0 + r - k_pos0 + 1, 0, k_len)
  auto nvis_of = [&](int r) {
    int n = t.q_pos0 + r - t.k_pos0 + 1;
    return n < 0 ? 0 : (n > t.k_len ? t.k_len : n);
  };
  const int nvis_lane = nvis_of(row);
  const int nvis_w_min = nvis_of(w * 32), nvis_w_max = nvis_of(w * 32 + 31);
  const int nvis_blk = nvis_of(t.q_rows - 1);
  const int n_kt = (nvis_blk + BN - 1) / BN;

  // Q^T operand: 8 consecutive head-dim elements of this lane's query per 16-wide k-step
  bf16x8 qreg[D / 16];
  {
    const __bf16 *qp = p.q + (int64_t)(t.q_tok0 + row) * p.q_stride + (int64_t)h * D + 8 * hi;
#pragma unroll
    for (int kk = 0; kk < D / 16; kk++) {
      if (row_ok) qreg[kk] = *(const bf16x8 *)(qp + 16 * kk);
      else qreg[kk] = bf16x8{0, 0, 0, 0, 0, 0, 0, 0};
    }
  }

  const __bf16 *kbase = p.k + (int64_t)t.k_tok0 * p.k_stride + (int64_t)g * D;
  const __bf16 *vbase = p.v + (int64_t)t.k_tok0 * p.v_stride + (int64_t)g * D;

  u32x4 kpre[C::CPT], vpre[C::CPT];
  auto load_tile = [&](int j0) {
#pragma unroll
    for (int n = 0; n < C::CPT; n++) {
      int id = tid + n * C::NT, r = id / (D / 8), c = id % (D / 8);
      if (j0 + r < t.k_len) {
        kpre[n] = *(const u32x4 *)(kbase + (int64_t)(j0 + r) * p.k_stride + c * 8);
        vpre[n] = *(const u32x4 *)(vbase + (int64_t)(j0 + r) * p.v_stride + c * 8);
      } else {
        kpre[n] = u32x4{0, 0, 0, 0};
        vpre[n] = u32x4{0, 0, 0, 0};
      }
    }
  };
  auto store_tile = [&](int buf) {
#pragma unroll
    for (int n = 0; n < C::CPT; n++) {
      int id = tid + n * C::NT, r = id / (D / 8), c = id % (D / 8);
      zp_lds_write16(Ks + buf * C::TILEB, zp_koff<D>(r, c), kpre[n]);
      zp_lds_write16(Vs + buf * C::TILEB, zp_voff<D>(r, c * 8), vpre[n]);
    }
  };

  f32x16 o_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) o_acc[i][r] = 0.f;
  float mc = -INFINITY;  // running reference maximum, in scaled log2 units
  float l_sum = 0.f;     // this lane's share of the row sum
  const float c_log2 = p.scale_log2;

  if (n_kt > 0) {
    load_tile(0);
    store_tile(0);
  }
  __syncthreads();

  for (int it = 0; it < n_kt; it++) {
    const int j0 = it * BN, buf = it & 1;
    if (it + 1 < n_kt) load_tile(j0 + BN);

    if (j0 < nvis_w_max) {  // otherwise every key of this tile is masked for the whole wave
      const char *Kb = Ks + buf * C::TILEB;
      const char *Vb = Vs + buf * C::TILEB;
      f32x16 s_acc[2];
#pragma unroll
      for (int kb = 0; kb < 2; kb++) {
#pragma unroll
        for (int r = 0; r < 16; r++) s_acc[kb][r] = 0.f;
#pragma unroll
        for (int kk = 0; kk < D / 16; kk++) {
          bf16x8 a = zp_lds_read16(Kb, zp_koff<D>(kb * 32 + ql, 2 * kk + hi));
          s_acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qreg[kk], s_acc[kb], 0, 0, 0);
        }
      }
      if (j0 + BN > nvis_w_min) {  // some lane has a masked key in this tile
#pragma unroll
        for (int kb = 0; kb < 2; kb++)
#pragma unroll
          for (int r = 0; r < 16; r++) {
            int j = j0 + kb * 32 + 8 * (r >> 2) + 4 * hi + (r & 3);
            if (j >= nvis_lane) s_acc[kb][r] = -INFINITY;
          }
      }
      float tmax = s_acc[0][0];
#pragma unroll
      for (int r = 1; r < 16; r++) tmax = fmaxf(tmax, s_acc[0][r]);
#pragma unroll
      for (int r = 0; r < 16; r++) tmax = fmaxf(tmax, s_acc[1][r]);
      tmax = zp_pair_max(tmax);
      const float tmc = tmax * c_log2;
      // the reference maximum moves only when the tile maximum exceeds it by more than 2^8
      if (__builtin_amdgcn_ballot_w64(tmc > mc + 8.0f) != 0) {
        const bool mv = tmc > mc + 8.0f;
        const float alpha = mv ? zp_exp2(mc - tmc) : 1.0f;
        mc = mv ? tmc : mc;
        l_sum *= alpha;
#pragma unroll
        for (int i = 0; i < D / 32; i++)
#pragma unroll
          for (int r = 0; r < 16; r++) o_acc[i][r] *= alpha;
      }
      const float neg_mc = (mc == -INFINITY) ? 0.f : -mc;
      bf16x8 pb[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int r = 0; r < 16; r++) {
          float pv = zp_exp2(__builtin_fmaf(s_acc[kb][r], c_log2, neg_mc));
          l_sum += pv;
          pb[kb][r >> 3][r & 7] = (__bf16)pv;
        }
      const int g16 = lane >> 4, i16 = lane & 15;
      const int vrow = 4 * (g16 >> 1) + (i16 >> 2);           // + 32kb + 16m + 8j
      const int vcol = 16 * (g16 & 1) + 4 * (i16 & 3);        // + 32 dblk
#pragma unroll
      for (int kb = 0; kb < 2; kb++)
#pragma unroll
        for (int m = 0; m < 2; m++)
#pragma unroll
          for (int db = 0; db < D / 32; db++) {
            bf16x4 lo = zp_lds_read_tr(Vb, zp_voff<D>(kb * 32 + m * 16 + vrow, db * 32 + vcol));
            bf16x4 hi4 = zp_lds_read_tr(Vb, zp_voff<D>(kb * 32 + m * 16 + 8 + vrow, db * 32 + vcol));
            o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(zp_cat(lo, hi4), pb[kb][m], o_acc[db], 0, 0, 0);
          }
    }

    if (it + 1 < n_kt) store_tile(buf ^ 1);
    __syncthreads();
  }

  // epilogue: normalise, write O and LSE
  const float l_tot = zp_pair_sum(l_sum);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  const float lse = l_tot > 0.f ? (mc * 0.6931471805599453f + __logf(l_tot)) : -INFINITY;
  if (row_ok) {
    const int64_t orow = (int64_t)t.out_row0 + row;
    if (hi == 0) p.lse[(int64_t)h * p.lse_stride + orow] = lse;
    if (PARTIAL) {
      float *op = (float *)p.o + orow * p.o_stride + (int64_t)h * D + 4 * hi;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          f32x4 v4 = {o_acc[db][4 * b] * inv, o_acc[db][4 * b + 1] * inv, o_acc[db][4 * b + 2] * inv,
                      o_acc[db][4 * b + 3] * inv};
          *(f32x4 *)(op + db * 32 + b * 8) = v4;
        }
    } else {
      __bf16 *op = (__bf16 *)p.o + orow * p.o_stride + (int64_t)h * D + 4 * hi;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          bf16x4 v4 = {(__bf16)(o_acc[db][4 * b] * inv), (__bf16)(o_acc[db][4 * b + 1] * inv),
                       (__bf16)(o_acc[db][4 * b + 2] * inv), (__bf16)(o_acc[db][4 * b + 3] * inv)};
          *(bf16x4 *)(op + db * 32 + b * 8) = v4;
        }
    }
  }
}

}  // namespace

extern "C" void zp_prof_begin(const char *name, hipStream_t stream);
extern "C" void zp_prof_end(hipStream_t stream);

// Host-side launcher used by the C ABI. Returns a hipError_t as int.
extern "C" int zp_launch_attn_fwd(const zp_attn_params *p, int d, int partial, int block_rows, hipStream_t stream) {
  const int units = p->n_tiles * p->Hkv;
  if (units == 0) return 0;
  const int grid = ((units + 7) / 8) * 8 * p->grp;
  (void)block_rows;
#define ZP_FWD_LAUNCH(D, NW, PART)                                                                      \
  do {                                                                                                  \
    size_t lds = 4 * (size_t)FwdCfg<D, NW>::TILEB;                                                      \
    zp_prof_begin(PART ? "attn_fwd_partial" : "attn_fwd", stream);                                      \
    hipLaunchKernelGGL((attn_fwd_kernel<D, NW, PART>), dim3(grid), dim3(NW * 64), lds, stream, *p);     \
    zp_prof_end(stream);                                                                                \
  } while (0)
  if (d == 128) {
    if (partial) ZP_FWD_LAUNCH(128, 4, true); else ZP_FWD_LAUNCH(128, 4, false);
  } else {
    if (partial) ZP_FWD_LAUNCH(64, 4, true); else ZP_FWD_LAUNCH(64, 4, false);
  }
#undef ZP_FWD_LAUNCH
  return (int)hipGetLastError();
}

extern "C" int zp_attn_fwd_block_rows(int d) { (void)d; return 128; }
