/*
 * zeppelin_attn.h -- C ABI of the single-GPU attention engine over packed variable-length sequences
 * (the data-parallel hot path of Zeppelin, arXiv 2509.21841), hand-written HIP for gfx950 (MI355X).
 *
 * Common rules for every entry point
 *  - Returns ZP_OK (0) or a negative error code; zp_strerror() gives the text. All argument checks
 *    run on the host before anything is enqueued: on error nothing has been launched.
 *  - "device" pointers are HIP device memory owned by the caller and must stay valid until the work
 *    enqueued on `stream` has finished. "host" arrays are read before the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream). Calls only enqueue work:
 *    no device synchronisation, no device memory allocation. The library keeps a small pool of pinned
 *    host staging buffers (grown on demand) for its descriptor uploads.
 *  - `ws` is caller-provided device scratch of at least zp_workspace_bytes(...) bytes, 256-byte aligned.
 *    Its contents are undefined afterwards. Two calls that share one `ws` must be ordered on one stream.
 *  - Layouts: token-major packed tensors. Q, O, dO, dQ are [T][Hq][d]; K, V, dK, dV are [T][Hkv][d],
 *    bfloat16, head stride d, with an explicit token stride in ELEMENTS (so a fused QKV buffer works;
 *    a multiple of 8, at least H*d and at most 2^24).
 *    LSE is float32 [Hq][T], natural logarithm. Q head h reads KV head h / (Hq/Hkv).
 *  - Sequence s owns tokens cu_seqlens[s] .. cu_seqlens[s+1]-1; cu_seqlens[0] = 0, non-decreasing,
 *    cu_seqlens[S] = T. Zero-length sequences are legal. A token attends only to tokens of its own
 *    sequence at the same or an earlier position (Sec. 2.1: lower-triangular mask; Sec. 2.3 / 3.2:
 *    no cross-sequence attention, local sequences use a variable-length kernel).
 *  - Supported: d in {64, 128}; Hq % Hkv == 0; bfloat16 inputs, float32 accumulation.
 * Measurement aids (per-kernel timing, a device probe) are declared in zeppelin_attn_bench.h, not here.
 */
#ifndef ZEPPELIN_ATTN_H
#define ZEPPELIN_ATTN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ZP_OK 0
#define ZP_EINVAL (-1)       /* null pointer, bad cu_seqlens, descriptor out of range, bad stride */
#define ZP_EUNSUPPORTED (-2) /* head_dim not 64/128, Hq % Hkv != 0, row_bytes % 16 != 0 */
#define ZP_EWORKSPACE (-3)   /* ws is NULL, misaligned or smaller than zp_workspace_bytes() */
#define ZP_EHIP (-4)         /* a HIP runtime call failed; zp_strerror(ZP_EHIP) carries its text */
#define ZP_ETOOLARGE (-5)    /* more sequences or tiles than the fixed limits of varlen_attn_fwd_noalloc */

#define ZP_MAX_PARTS 16

/* Problem shape. T packed tokens, S sequences, Hq query heads, Hkv key/value heads, head dim d.
 * scale multiplies q.k before the softmax; 0 selects 1/sqrt(d). */
typedef struct {
  int32_t T, S, Hq, Hkv, d;
  float scale;
} zp_shape;

/* One (Q chunk, KV chunk) pair of one sequence (Sec. 3.2: a sequence on a ring of size G is cut into
 * 2G equal-length chunks; each round a rank computes its Q chunks against the KV chunks in hand).
 * q_tok0/k_tok0: first packed token of the Q / KV chunk; q_len/k_len: chunk lengths;
 * q_pos0/k_pos0: position of the chunk's first token inside its sequence; key j of the chunk is visible
 * to query i of the chunk iff k_pos0 + j <= q_pos0 + i; out_row0: the pair's first row in o_part/lse_part. */
typedef struct {
  int32_t q_tok0, q_len, k_tok0, k_len, q_pos0, k_pos0, out_row0;
} zp_pair;

/* One run of `len` output tokens starting at packed token out_tok0, each combined from n_parts partial
 * rows: part p contributes rows part_row0[p] .. part_row0[p]+len-1 of o_part / lse_part. */
typedef struct {
  int32_t out_tok0, len, n_parts;
  int32_t part_row0[ZP_MAX_PARTS];
} zp_merge;

/* Which entry point a workspace query is for. */
enum { ZP_FN_FWD = 0, ZP_FN_BWD = 1, ZP_FN_PARTIAL = 2, ZP_FN_MERGE = 3, ZP_FN_PARTIAL_BWD = 4 };

/* Bytes of `ws` an entry point needs. n_desc: number of pairs (ZP_FN_PARTIAL, ZP_FN_PARTIAL_BWD) or merges (ZP_FN_MERGE),
 * ignored otherwise. cu_seqlens_host may be NULL for ZP_FN_PARTIAL / ZP_FN_MERGE / ZP_FN_PARTIAL_BWD. Returns 0 on bad input. */
size_t zp_workspace_bytes(int which_fn, const zp_shape *sh, const int32_t *cu_seqlens_host, int64_t n_desc);

/* Causal softmax attention of every sequence of the packed batch (Sec. 3.2, local sequences; Sec. 2.1):
 *   O[i,h,:] = sum_{j<=i} softmax_j(scale q_i.k_j) v_j ,   LSE[h,i] = log sum_{j<=i} exp(scale q_i.k_j).
 * The host builds a work list of (sequence, query block) tiles by the quadratic cost model |s|^2 of Alg. 2:
 * sequences in descending length and, inside a sequence, query blocks in descending number of visible key
 * tiles, so that the heaviest tiles of the batch start first, the light ones fill the tail, and the blocks
 * of one sequence run side by side and share its K/V rows in the cache.
 * q,k,v: device bf16; o: device bf16 out; lse: device float32 [Hq][T] out; cu_seqlens_host: host [S+1].
 * seq_skip_host: NULL, or host [S] flags; a flagged sequence is left out (its O / LSE rows are not written)
 * so that the caller can compute it as chunk pairs instead (Sec. 3.2: ring sequences vs local sequences). */
int varlen_attn_fwd(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride, int64_t v_stride,
                    const int32_t *cu_seqlens_host, const uint8_t *seq_skip_host, void *o, int64_t o_stride, float *lse,
                    const zp_shape *sh, void *ws, size_t ws_bytes, void *stream);

/* varlen_attn_fwd for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc. Same arguments and same results (bit for bit) as varlen_attn_fwd without the workspace: the tile
 * table lives in a fixed device array inside the library (ZP_NOALLOC_MAX_TILES records of 32 bytes + 1 KiB of work
 * counters = 257 KiB, one copy
 * per GPU, held until the process ends) and is built on the device from the sequence boundaries, which travel by value
 * in the launch arguments. The call allocates nothing on host or device, reads no host memory from the device and
 * uploads nothing; it enqueues two kernels on `stream`. Limits: S <= ZP_NOALLOC_MAX_SEQS sequences and at most
 * ZP_NOALLOC_MAX_TILES blocks of 128 query rows (sum over unflagged sequences of ceil(len / 128)); beyond them the
 * call returns ZP_ETOOLARGE and enqueues nothing. Every call on a GPU uses that GPU's one table: calls on the same GPU
 * must be ordered on one stream (or otherwise not overlap), else they race. Keep zp_profile_enable off around it
 * (the timing aid creates events). */
#define ZP_NOALLOC_MAX_SEQS 768
#define ZP_NOALLOC_MAX_TILES 8192
int varlen_attn_fwd_noalloc(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride,
                            int64_t v_stride, const int32_t *cu_seqlens_host, const uint8_t *seq_skip_host, void *o,
                            int64_t o_stride, float *lse, const zp_shape *sh, void *stream);

/* Backward of varlen_attn_fwd (Sec. 5.4: the backward mirrors the forward with about twice the work).
 * Reads dO, Q, K, V and the forward's O and LSE; writes dQ [T][Hq][d], dK, dV [T][Hkv][d] (bf16). With
 * P_ij = exp(scale q_i.k_j - LSE_i), D_i = dO_i.O_i, dS_ij = P_ij (dO_i.v_j - D_i):
 *   dQ_i = scale sum_{j<=i} dS_ij k_j ;  dK_j = scale sum_{h in group} sum_{i>=j} dS_ij q_i ;
 *   dV_j = sum_{h in group} sum_{i>=j} P_ij dO_i.
 * Deterministic (no atomics): one kernel owns key/value rows, one owns query rows.
 * seq_skip_host: NULL, or host [S] flags; the dQ/dK/dV rows of a flagged sequence are not written (the caller runs
 * it as chunk pairs with chunk_attn_partial_bwd instead).
 * dq/dk/dv token strides are dq_stride (= for dQ) and dkv_stride (for dK and dV). */
int varlen_attn_bwd(const void *dout, const void *q, const void *k, const void *v, const void *o, const float *lse,
                    int64_t do_stride, int64_t q_stride, int64_t k_stride, int64_t v_stride, int64_t o_stride,
                    const int32_t *cu_seqlens_host, const uint8_t *seq_skip_host, void *dq, void *dk, void *dv,
                    int64_t dq_stride, int64_t dkv_stride, const zp_shape *sh, void *ws, size_t ws_bytes, void *stream);

/* Partial attention of (Q chunk, KV chunk) pairs (Sec. 3.2, the per-round compute of ring attention):
 * for each pair and head, softmax over only that KV chunk's causally visible keys, normalised by its
 * own sum, with its own LSE. Rows with no visible key get LSE = -inf and O = 0.
 * o_part: device float32 [part_rows][Hq][d]; lse_part: device float32 [Hq][part_rows]; every pair's row
 * range must lie inside part_rows; ranges of different pairs must not overlap (not checked).
 * sh->S is ignored, sh->T bounds the token offsets. pairs_host: host array of n_pairs. */
int chunk_attn_partial(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride,
                       int64_t v_stride, const zp_pair *pairs_host, int32_t n_pairs, float *o_part, float *lse_part,
                       int64_t part_rows, const zp_shape *sh, void *ws, size_t ws_bytes, void *stream);

/* Chunk-pair attention merged in place (Sec. 3.2: a ring rank folds every round's result into what it holds).
 * Like chunk_attn_partial, but instead of writing one partial per pair it combines each pair's result with the
 * running rows of its queries: o_run [T][Hq][d] fp32 (contiguous) holds outputs normalised by their own softmax sum,
 * lse_run [Hq][T] fp32 their natural-log LSE; after the call they hold the attention over the keys seen so far plus
 * this pair's keys (LSE = log(exp(LSE_run) + exp(LSE_pair)), O weighted by exp(LSE_x - LSE)). Start from
 * lse_run = -inf (o_run may then hold anything). out_row0 of the pairs is ignored. A query row may appear in ONE pair
 * of a call only (ZP_EINVAL otherwise): the rows are read, merged and written back without atomics. Workspace:
 * zp_workspace_bytes(ZP_FN_PARTIAL, ...). */
int chunk_attn_update(const void *q, const void *k, const void *v, int64_t q_stride, int64_t k_stride, int64_t v_stride,
                      const zp_pair *pairs_host, int32_t n_pairs, float *o_run, float *lse_run, const zp_shape *sh,
                      void *ws, size_t ws_bytes, void *stream);

/* Backward of one ring round of chunk pairs (Sec. 3.2 rounds, Sec. 5.4: the backward runs them in reverse): for
 * every pair and head, with P_ij = exp(scale q_i.k_j - LSE_i) over the pair's causally visible (i, j), LSE the
 * MERGED log-sum-exp of the whole row and D_i = dO_i.O_i from the merged O,
 *   dq_acc[i] += scale sum_j dS_ij k_j ;  dk_acc[j] += scale sum_{h in group} sum_i dS_ij q_i ;
 *   dv_acc[j] += sum_{h in group} sum_i P_ij dO_i ,   dS_ij = P_ij (dO_i.v_j - D_i).
 * dq_acc [T][Hq][d], dk_acc / dv_acc [T][Hkv][d] are device float accumulators the results are ADDED to (the caller
 * zeroes them before the first round); summed over all causal pairs of a sequence they equal varlen_attn_bwd's
 * result. Within one call the Q row ranges of the pairs must be pairwise disjoint and so must the KV row ranges
 * (checked; ZP_EINVAL): that is one ring round, and rounds are ordered by the stream. */
int chunk_attn_partial_bwd(const void *dout, const void *q, const void *k, const void *v, const void *o,
                           const float *lse, int64_t do_stride, int64_t q_stride, int64_t k_stride, int64_t v_stride,
                           int64_t o_stride, const zp_pair *pairs_host, int32_t n_pairs, float *dq_acc, float *dk_acc,
                           float *dv_acc, const zp_shape *sh, void *ws, size_t ws_bytes, void *stream);

/* Rounds n float accumulator values to bfloat16 (n % 8 == 0; src, dst 16-byte aligned device pointers). */
int zp_accum_to_bf16(const float *src, void *dst, int64_t n, void *stream);

/* Online-softmax combination of partial results (Sec. 3.2, "standard ring attention pattern"):
 *   LSE = log sum_p exp(LSE_p),  O = sum_p exp(LSE_p - LSE) O_p ; parts with LSE_p = -inf weigh 0 and a
 * row whose parts are all -inf gets LSE = -inf, O = 0. Writes O (bf16, token stride o_stride) and
 * LSE [Hq][T] only for the tokens the merges cover. merges_host: host array of n_merges. */
int lse_merge(const float *o_part, const float *lse_part, int64_t part_rows, const zp_merge *merges_host,
              int32_t n_merges, void *o, int64_t o_stride, float *lse, const zp_shape *sh, void *ws, size_t ws_bytes,
              void *stream);

/* Token move of the remapping layer (Sec. 3.4: attention layout <-> token-balanced layout, and back).
 * mode 0 (gather):  dst row i = src row idx[i];  mode 1 (scatter): dst row idx[i] = src row i.
 * Rows are raw bytes: row_bytes % 16 == 0, src/dst 16-byte aligned and not overlapping. idx_dev: device
 * int32 [n_rows], every entry in [0, n_rows) (a permutation for mode 1; not checked on the device). */
int remap_tokens(const void *src, void *dst, int64_t row_bytes, const int32_t *idx_dev, int64_t n_rows, int32_t mode,
                 void *stream);

/* Host-only helper (no device work): descriptors of one sequence cut into C equal-length chunks
 * (chunk c = positions [floor(cL/C), floor((c+1)L/C)) ). rank < 0: every causal pair (kc <= qc).
 * rank in [0, C/2): only the pairs ring rank `rank` computes, i.e. Q chunks {rank, C-1-rank} (C even).
 * tok0: first packed token of the sequence; row0: first free row of o_part. Fills pairs[] (capacity
 * max_pairs) and merges[] (capacity max_merges, one per Q chunk); returns the number of pairs, sets
 * *n_merges and *rows_used (partial rows consumed). Negative on error. */
int zp_chunk_pairs(int32_t tok0, int32_t L, int32_t C, int32_t rank, int32_t row0, zp_pair *pairs, int32_t max_pairs,
                   zp_merge *merges, int32_t max_merges, int32_t *n_merges, int64_t *rows_used);

/* One item of a device's work after partitioning: sequence `seq` runs on node `node`, device `device`, either
 * whole (zone 0, ring 1) or as ring rank `rank` of a ring of `ring` devices (zone 1: intra-node, zone 2:
 * inter-node), holding chunks `rank` and 2*ring-1-rank of 2*ring equal-length chunks; `tokens` of it live there. */
typedef struct {
  int32_t seq, zone, ring, rank, node, device, tokens;
} zp_placement;

/* Host-only: hierarchical sequence partitioner (Sec. 3.1, Alg. 1 inter-node then Alg. 2 intra-node) for S sequences
 * of the given lengths on N nodes of P devices with token capacity L per device. Sequences at or above the
 * inter-node threshold s1 (initially P*L, lowered until the rest fits node by node) are split evenly over
 * ceil(|s| / s_avg) of the least loaded nodes and over all P devices of each; inside a node, sequences at or above
 * s0 (initially L, lowered until the rest fits device by device) are split over ceil(|s|^2 / c_avg) <= P devices
 * assigned round-robin (c_avg = sum |s|^2 / P); the rest go whole to the least loaded device. A sequence on a ring of
 * G devices is cut into 2G equal-length chunks and rank r holds chunks r and 2G-1-r (Sec. 3.2).
 * Writes up to max_out placements (node-major), the count to *n_out, the final s1 to *s1_final and the final s0 of
 * every node to s0_final[N] (both optional). Returns ZP_EWORKSPACE if max_out was too small (*n_out = needed). */
int zp_partition(const int32_t *lengths, int32_t S, int32_t P, int32_t N, int32_t L, zp_placement *out,
                 int32_t max_out, int32_t *n_out, int32_t *s1_final, int32_t *s0_final);

/* Host helper: the attention layout a placement list implies (Sec. 3.1, 3.2), as runs of consecutive tokens of the
 * concatenated device buffers: devices in (node, device) order, on each its placements in list order; a whole
 * sequence is one run, ring rank r of G the two runs chunk r and chunk 2G-1-r of 2G equal-length chunks.
 * tok0 = first token of the run in the concatenation, pos0 = its first position inside its sequence.
 * Writes up to max_out runs, the count to *n_out and (optional) the tokens of every device to tokens_per_rank[N*P],
 * which is the vector A of the remap planner. Returns ZP_EWORKSPACE if max_out was too small (*n_out = needed). */
typedef struct {
  int32_t seq, chunk, n_chunks, pos0, len, tok0, node, device;
} zp_segment;
int zp_node_segments(const int32_t *lengths, int32_t S, const zp_placement *placements, int32_t n_placements, int32_t P,
                     int32_t N, zp_segment *out, int32_t max_out, int32_t *n_out, int32_t *tokens_per_rank);

/* Host helper: the runs of ONE sequence that lies contiguously at packed token tok0 and is cut into C equal-length
 * chunks (chunk c = positions [floor(cL/C), floor((c+1)L/C)), Sec. 3.2): out[c] = {seq, c, C, pos0, len, tok0 + pos0,
 * node 0, device 0}, the same records zp_node_segments writes for a ring sequence spread over devices. C >= 1,
 * max_out >= C. Returns C, or a negative error code. */
int zp_chunk_segments(int32_t seq, int32_t tok0, int32_t L, int32_t C, zp_segment *out, int32_t max_out);

/* Host helper: the chunk pairs of one round of the ring sequences among `segs` (records with n_chunks > 1, and, if
 * include_whole is non-zero, also whole sequences as "rings" of one chunk whose single pair (0, 0) is in round 0; a
 * sequence must be present with every chunk 0 .. n_chunks-1 exactly once, ZP_EINVAL otherwise). Sec. 3.2: a ring of G
 * devices over 2G chunks computes, over its G rounds, every causal pair (qc, kc), kc <= qc, once. On one GPU a call of
 * chunk_attn_update / chunk_attn_partial_bwd may hold a query run and a key run only once, so the same pairs are
 * grouped by their chunk distance: round t = the pairs (qc, qc - t), qc = t .. C-1, of every ring sequence (sequences
 * in ascending id, qc ascending); rounds 0 .. max C - 1 together are exactly the ring's pairs. Each pair takes
 * q_tok0/q_len/q_pos0 from the run of chunk qc and k_tok0/k_len/k_pos0 from the run of chunk qc - t; out_row0 = 0.
 * Writes up to max_pairs pairs, the count to *n_pairs and (optional) the number of rounds to *n_rounds.
 * Returns ZP_EWORKSPACE if max_pairs was too small (*n_pairs = needed). */
int zp_ring_round_pairs(const zp_segment *segs, int32_t n_segs, int32_t round, int32_t include_whole, zp_pair *pairs,
                        int32_t max_pairs, int32_t *n_pairs, int32_t *n_rounds);

/* Host helper: where every token of the attention layout sits in the batch as drawn (sequence after sequence in
 * `lengths` order): orig[run.tok0 + i] = (first drawn token of run.seq) + run.pos0 + i. n_tok must equal the tokens
 * the runs cover, and the runs must tile [0, n_tok) (ZP_EINVAL otherwise). */
int zp_segment_positions(const int32_t *lengths, int32_t S, const zp_segment *segs, int32_t n_segs, int64_t *orig,
                         int64_t n_tok);

/* Host helper: transfer plan of the remapping layer (Sec. 3.4, Eq. 2). A[d]: tokens per rank in the attention layout;
 * rank r sits in node r / P. The balanced target is B_i = floor(T/d) + (i < T mod d). Writes M[d*d] (row-major,
 * M[i*d+j] = tokens rank i sends to rank j) with row sums max(A-B,0), column sums max(B-A,0), minimising
 * max_i sum_j T_ij * M_ij where T_ij = b_inter across nodes and b_intra inside a node (integer costs per token,
 * 1 <= b_intra <= b_inter), and the minimum to *objective (optional). Among the optimal plans it picks the one that
 * exports from every node only its excess and matches senders to receivers in ascending rank order.
 * Returns ZP_EINVAL on null pointers, d < 1, P < 1, a negative count or costs out of order. */
int zp_remap_plan(const int32_t *A, int32_t d, int32_t P, int32_t b_intra, int32_t b_inter, int32_t *M,
                  int64_t *objective);

/* Host helper: the token permutation of a transfer plan, for remap_tokens. Positions count over the concatenation of
 * the rank buffers. A sender parts with the tail of its attention-layout buffer, cut into one run per destination in
 * ascending rank order; a rank's balanced buffer is its kept head followed by the arrivals in ascending source order.
 * Writes idx[n_idx] (n_idx = sum A): idx[balanced position] = attention-layout position, i.e. remap_tokens mode 0
 * takes the attention layout to the balanced one and mode 1 takes it back. Returns ZP_EINVAL if M does not move
 * exactly every surplus and deficit or n_idx != sum A. */
int zp_remap_indices(const int32_t *A, const int32_t *M, int32_t d, int32_t *idx, int64_t n_idx);

const char *zp_strerror(int code);

#ifdef __cplusplus
}
#endif
#endif
