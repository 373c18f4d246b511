// Causal attention forward over a work list of (query block, key run) tiles: bf16 MFMA for K Q^T and V^T P^T,
// K/V tiles staged through LDS, online softmax kept per lane.
//
// Orientation. Scores are computed transposed, S^T = K Q^T with the 32x32x16 MFMA: the accumulator lane
// (l%32, l/32) then holds ONE query (column l%32) and 16 keys per 32-key block (rows 8b + 4(l/32) + c),
// so the row maximum and row sum of the softmax are in-lane reductions plus one exchange with lane l^32,
// and the rescale factor is a per-lane scalar. The bf16 probabilities are already laid out as the B
// operand of O^T += V^T P^T (k-slot i of MFMA m <-> accumulator register 8m+i), and V^T comes from the
// row-major V tile in LDS through the transposing LDS read with the matching key order.
#include <type_traits>
#include "zp_common.h"

namespace {

constexpr int BN = 64;  // keys per LDS tile

template <int D, int NW>
struct FwdCfg {
  static constexpr int NT = NW * 64;
  static constexpr int BM = NW * 32;
  static constexpr int TILEB = BN * D * 2;  // bytes per K (or V) tile
};

// One 64-key tile for one wave of 32 query rows. Kb, Vb: byte offsets of the K and V tile from the LDS base that
// the lane offsets in `lo` carry (compile-time at the call sites, so every read is a register plus an immediate).
// With PIECES, `piece(integral_constant<int, kk>)` is called once per 16-wide k-step of the score MFMAs: the caller
// issues one asynchronous copy of the next tile there. The steps are fenced, so the copies stay one MFMA pair apart
// -- far enough that none waits for the address unit behind the copies of the other waves, which is what issuing
// them back to back in front of the tile costs.
template <int D, bool MASK, bool PIECES, class Piece>
__device__ __forceinline__ void fwd_tile(int Kb, int Vb, const bf16x8 (&qreg)[D / 16],
                                         f32x16 (&o_acc)[D / 32], float &mc, float &l_sum, float c_log2, int j0,
                                         int hi, int nvis_lane, const zp_lds_offsets<D> &lo, Piece &&piece) {
  constexpr int KK = D / 16, DB = D / 32;
  const f32x16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  f32x16 s0 = zero, s1 = zero;
  if constexpr (PIECES) {
    // the K row operands stay two k-steps ahead of the MFMAs that use them
    bf16x8 k0[KK], k1[KK];
    k0[0] = lo.rows_at(Kb, 0, 0); k1[0] = lo.rows_at(Kb, 1, 0);
    k0[1] = lo.rows_at(Kb, 0, 1); k1[1] = lo.rows_at(Kb, 1, 1);
    zp_static_for<KK>([&](auto kk) {
      constexpr int k = kk.value;
      __builtin_amdgcn_sched_barrier(0);
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k0[k], qreg[k], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(k1[k], qreg[k], s1, 0, 0, 0);
      if constexpr (k + 2 < KK) { k0[k + 2] = lo.rows_at(Kb, 0, k + 2); k1[k + 2] = lo.rows_at(Kb, 1, k + 2); }
      piece(kk);
    });
    __builtin_amdgcn_sched_barrier(0);
  } else {
#pragma unroll
    for (int kk = 0; kk < KK; kk++) {
      s0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo.rows_at(Kb, 0, kk), qreg[kk], s0, 0, 0, 0);
      s1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo.rows_at(Kb, 1, kk), qreg[kk], s1, 0, 0, 0);
    }
  }
  if (MASK) {
#pragma unroll
    for (int r = 0; r < 16; r++) {
      const int j = j0 + 8 * (r >> 2) + 4 * hi + (r & 3);
      if (j >= nvis_lane) s0[r] = -INFINITY;
      if (j + 32 >= nvis_lane) s1[r] = -INFINITY;
    }
  }
  // Two chains of three-operand maxima over the lane's 32 scores. The compiler does not check the inline-assembly
  // v_max3 against the "MFMA result read too early" hazard, so both chains start from t0, an ordinary fmaxf of one
  // register of each accumulator: the wait states the compiler inserts before t0 cover every later read.
  const float t0 = fmaxf(s0[15], s1[15]);
  float ta = zp_max3(t0, s0[0], s0[1]);
  float tb = zp_max3(t0, s1[0], s1[1]);
#pragma unroll
  for (int r = 2; r < 14; r += 2) {
    ta = zp_max3(ta, s0[r], s0[r + 1]);
    tb = zp_max3(tb, s1[r], s1[r + 1]);
  }
  const float tmax = zp_pair_max(zp_max3(ta, tb, fmaxf(s0[14], s1[14])));
  const float tmc = tmax * c_log2;
  // the reference maximum moves only when the tile maximum exceeds it by more than 2^8
  if (__builtin_amdgcn_ballot_w64(tmc > mc + 8.0f) != 0) {
    const bool mv = tmc > mc + 8.0f;
    const float alpha = mv ? zp_exp2(mc - tmc) : 1.0f;
    mc = mv ? tmc : mc;
    l_sum *= alpha;
#pragma unroll
    for (int i = 0; i < DB; i++)
#pragma unroll
      for (int r = 0; r < 16; r++) o_acc[i][r] *= alpha;
  }
  const float neg_mc = (mc == -INFINITY) ? 0.f : -mc;
  // the row sum is taken over the unrounded probabilities: LSE has to hold to 1e-3 also for rows with few keys
  bf16x8 pb[2][2];
  float l1 = 0.f;
#pragma unroll
  for (int r = 0; r < 16; r++) {
    const float p0 = zp_exp2(__builtin_fmaf(s0[r], c_log2, neg_mc));
    const float p1 = zp_exp2(__builtin_fmaf(s1[r], c_log2, neg_mc));
    l_sum += p0;
    l1 += p1;
    pb[0][r >> 3][r & 7] = (__bf16)p0;
    pb[1][r >> 3][r & 7] = (__bf16)p1;
  }
  l_sum += l1;
#pragma unroll
  for (int kb = 0; kb < 2; kb++)
#pragma unroll
    for (int m = 0; m < 2; m++)
#pragma unroll
      for (int db = 0; db < DB; db++)
        o_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(lo.tr_at(Vb, kb, m, db), pb[kb][m], o_acc[db], 0, 0, 0);
}

template <int D, int NW, bool PARTIAL>
__global__ __launch_bounds__(NW * 64) __attribute__((amdgpu_waves_per_eu(2, 2))) void attn_fwd_kernel(zp_attn_params p) {
  using C = FwdCfg<D, NW>;
  static_assert(NW == 4, "the tile stager is laid out for four waves");
  extern __shared__ __attribute__((aligned(16))) char smem[];
  char *Ks = smem;                  // [2][BN][D] bf16
  char *Vs = smem + 2 * C::TILEB;   // [2][BN][D] bf16

  const int item = zp_item_of_block(p.work, (int *)(smem + 4 * C::TILEB));
  if (item < 0) return;
  int unit, hh;
  zp_block_to_unit(item, p.grp, unit, hh);
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
  const int n_kt = (nvis_of(t.q_rows - 1) + BN - 1) / BN;

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
  // No wait here: the first tile copy is issued right behind these loads so that the two memory latencies of the
  // prologue overlap; the explicit wait in front of the first barrier covers both (and tells the compiler that the
  // register operands have arrived: a wait of its own inside the key loop would drain the copies in flight).

  zp_stager<D> kst, vst;
  kst.init(p.k + (int64_t)t.k_tok0 * p.k_stride + (int64_t)g * D, p.k_stride, tid);
  vst.init(p.v + (int64_t)t.k_tok0 * p.v_stride + (int64_t)g * D, p.v_stride, tid);
  zp_lds_offsets<D> lo;
  lo.init_abs(lane, smem);

  f32x16 o_acc[D / 32];
#pragma unroll
  for (int i = 0; i < D / 32; i++)
#pragma unroll
    for (int r = 0; r < 16; r++) o_acc[i][r] = 0.f;
  float mc = -INFINITY;  // running reference maximum, in scaled log2 units
  float l_sum = 0.f;     // this lane's share of the row sum
  const float c_log2 = p.scale_log2;

  if (n_kt > 0) {
    kst.issue(Ks, 0, t.k_len);
    vst.issue(Vs, 0, t.k_len);
  }
  zp_wait_async();
  __syncthreads();

  constexpr int PW = zp_stager<D>::PER_WAVE;
  // one key tile out of LDS buffer BUF (a compile-time constant, so every LDS address is register + immediate)
  auto key_tile = [&](int it, auto BUF) {
    constexpr int buf = decltype(BUF)::value;
    const int j0 = it * BN;
    const bool compute = j0 < nvis_w_max;  // otherwise every key of this tile is masked for the whole wave
    const bool masked = j0 + BN > nvis_w_min;
    // the next tile is fetched inside this tile's score MFMAs when it has 64 valid keys and this wave computes an
    // unmasked tile (the common case), else in front of it
    const bool fetch = it + 1 < n_kt;
    const bool fused = fetch && compute && !masked && j0 + 2 * BN <= t.k_len;
    if (fetch && !fused) {
      kst.issue(Ks + (buf ^ 1) * C::TILEB, j0 + BN, t.k_len);
      vst.issue(Vs + (buf ^ 1) * C::TILEB, j0 + BN, t.k_len);
    }
    // the same copies one load at a time, K and V alternating (2 * PW loads = one per k-step); the sources are worked
    // out unconditionally: a value defined under a branch would not stay in scalar registers
    const void *pc_k = zp_uniform_ptr(kst.base + (int64_t)(j0 + BN) * kst.stride);
    const void *pc_v = zp_uniform_ptr(vst.base + (int64_t)(j0 + BN) * vst.stride);
    auto stage_piece = [&](auto n) {
      constexpr int N = decltype(n)::value, i = N / 2;
      static_assert(2 * PW == D / 16, "one copy per k-step");
      if constexpr (N % 2 == 0)
        zp_dma16_so(pc_k, kst.off[i], __builtin_amdgcn_readfirstlane(zp_lds_addr(Ks + (buf ^ 1) * C::TILEB) + (kst.w * PW + i) * 1024));
      else
        zp_dma16_so(pc_v, vst.off[i], __builtin_amdgcn_readfirstlane(zp_lds_addr(Vs + (buf ^ 1) * C::TILEB) + (vst.w * PW + i) * 1024));
    };
    if (compute) {
      constexpr int Kb = buf * C::TILEB, Vb = (2 + buf) * C::TILEB;  // byte offsets of the tiles from smem
      if (masked) fwd_tile<D, true, false>(Kb, Vb, qreg, o_acc, mc, l_sum, c_log2, j0, hi, nvis_lane, lo, stage_piece);
      else if (fused) fwd_tile<D, false, true>(Kb, Vb, qreg, o_acc, mc, l_sum, c_log2, j0, hi, nvis_lane, lo, stage_piece);
      else fwd_tile<D, false, false>(Kb, Vb, qreg, o_acc, mc, l_sum, c_log2, j0, hi, nvis_lane, lo, stage_piece);
    }
    zp_wait_async();
    __syncthreads();
  };
  int it = 0;
  for (; it + 1 < n_kt; it += 2) {
    key_tile(it, std::integral_constant<int, 0>{});
    key_tile(it + 1, std::integral_constant<int, 1>{});
  }
  if (it < n_kt) key_tile(it, std::integral_constant<int, 0>{});

  // epilogue: normalise, write O and LSE
  const float l_tot = zp_pair_sum(l_sum);
  const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
  const float lse = l_tot > 0.f ? (mc * 0.6931471805599453f + __logf(l_tot)) : -INFINITY;
  if (row_ok) {
    const int64_t orow = (int64_t)t.out_row0 + row;
    if (PARTIAL) {
      // weights of the running row (w_old) and of this partial (w_new, its 1/l folded in); without update: 0 and 1/l
      float w_old = 0.f, w_new = inv, lse_out = lse;
      if (p.update) {
        const float lse_old = p.lse[(int64_t)h * p.lse_stride + orow];
        const float mx = fmaxf(lse_old, lse);
        if (mx == -INFINITY) {
          w_new = 0.f;
        } else {
          const float e_old = __expf(lse_old - mx), e_new = __expf(lse - mx);
          const float tot = e_old + e_new;
          lse_out = mx + __logf(tot);
          w_old = e_old / tot;
          w_new = e_new / tot * inv;
        }
      }
      if (hi == 0) p.lse[(int64_t)h * p.lse_stride + orow] = lse_out;
      float *op = (float *)p.o + orow * p.o_stride + (int64_t)h * D + 4 * hi;
#pragma unroll
      for (int db = 0; db < D / 32; db++)
#pragma unroll
        for (int b = 0; b < 4; b++) {
          f32x4 v4 = {o_acc[db][4 * b] * w_new, o_acc[db][4 * b + 1] * w_new, o_acc[db][4 * b + 2] * w_new,
                      o_acc[db][4 * b + 3] * w_new};
          if (w_old > 0.f) {  // a row that has seen no key yet may hold anything
            const f32x4 old = *(const f32x4 *)(op + db * 32 + b * 8);
            v4[0] += w_old * old[0]; v4[1] += w_old * old[1]; v4[2] += w_old * old[2]; v4[3] += w_old * old[3];
          }
          *(f32x4 *)(op + db * 32 + b * 8) = v4;
        }
    } else {
      if (hi == 0) p.lse[(int64_t)h * p.lse_stride + orow] = lse;
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
  zp_attn_params q = *p;
  const int grid = zp_plan_work_split(q.work, p->work.counters, ((units + 7) / 8) * 8 * p->grp);
  p = &q;
  (void)block_rows;
#define ZP_FWD_LAUNCH(D, NW, PART)                                                                      \
  do {                                                                                                  \
    size_t lds = 4 * (size_t)FwdCfg<D, NW>::TILEB + 16;                                                    \
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
