/*
 * hstu_attn.h -- C ABI of the MI355X (gfx950) jagged HSTU attention library.
 *
 * The operation is the HSTU attention of the paper's section 2.1,
 *
 *     O = Mask( SiLU( alpha * Q K^T ) ) V / max_len
 *
 * with the bias term absent, SiLU(x) = x * sigmoid(x) applied pointwise, the
 * mask applied outside the SiLU (a masked pair contributes exactly zero), and
 * a plain 1/max_len normaliser (max_len = 1 gives the equation as printed).
 * Inputs are jagged tensors in the sense of section 2.2: a `values` buffer of
 * all sequences' rows back to back plus an int32 `seq_offsets` array; nothing
 * is padded.  The context-parallel entry point computes one rank's share under
 * the load-balanced split of section 2.3 (2*CP mini-chunks per sequence, rank r
 * owns mini-chunks r and 2*CP-1-r).  Because the nonlinearity is pointwise,
 * partial results over different key sets simply add.
 *
 * Conventions common to all entry points
 *   - Every data pointer is DEVICE memory owned by the caller; `seq_offsets`
 *     is device memory too and is never read by the host, so no call forces a
 *     host/device synchronisation (section 3 reports the cost of such syncs).
 *   - Layouts: q, k, dq, dk: [rows, num_heads, d_qk]; v, o, d_o, dv:
 *     [rows, num_heads, d_v]; row-major, contiguous.  Row t belongs to sequence
 *     b iff seq_offsets[b] <= t < seq_offsets[b+1]; seq_offsets[0] == 0,
 *     non-decreasing, seq_offsets[batch] == total_rows.  Rows at or beyond the
 *     row counts declared by the caller are never touched, even when the
 *     offsets on the device say otherwise.
 *   - All inputs of one call share `dtype`, all outputs share `out_dtype`.
 *     bf16 inputs are computed with bf16 MFMA operands and fp32 accumulation,
 *     the SiLU in fp32, and one rounding to bf16 at the output (none when
 *     out_dtype is fp32); fp32 inputs are computed in fp32 throughout.
 *   - `workspace` is caller-owned device scratch of at least
 *     hstu_jagged_attn_workspace_bytes() bytes, 256-byte aligned.  The library
 *     allocates no device memory and keeps no state between calls (the two
 *     exceptions are named where they are declared: the static scratch array of
 *     hstu_jagged_attn_fwd_static and the timing recorder); calls are
 *     asynchronous on `hip_stream` (a hipStream_t, NULL = the default stream)
 *     and calls on different streams with different workspaces may overlap.
 *   - Sizes: total_rows < 2^31; (rows / 128 + 2 * batch + 1) * num_heads < 2^31; and
 *     where a bf16 forward pass builds a transposed copy of V
 *     (HSTU_FLAG_FWD_TILE_128 / _256) the key side may hold at most 131071
 *     tiles of 64 rows, sequences' last tiles included (about 8.3 million rows).  Beyond: HSTU_ERR_BAD_SHAPE, and the
 *     workspace query returns 0.
 *   - Nothing in the process environment changes what a call does: the choices a caller (or a
 *     test) may want to force are bits of `params->flags` (hstu_flags below), and the same flags
 *     must be given to the workspace query and to the call.
 *   - Return value: HSTU_OK (0) or a negative hstu_status.  Nothing is launched
 *     when an error is returned.  batch == 0 or total_rows == 0 is HSTU_OK and
 *     launches nothing.  No exception or abort crosses this boundary.
 */
#ifndef HSTU_ATTN_H_
#define HSTU_ATTN_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HSTU_OK = 0,
  HSTU_ERR_NULL_PTR = -1,            /* a required pointer is NULL                         */
  HSTU_ERR_BAD_SHAPE = -2,           /* batch < 0, num_heads < 1, total_rows < 0 or
                                        >= 2^31, max_len < 1, alpha not finite              */
  HSTU_ERR_UNSUPPORTED = -3,         /* head dim not in {32,64,128}, unknown dtype, out_dtype
                                        neither dtype nor fp32, unknown bits in flags       */
  HSTU_ERR_WORKSPACE_TOO_SMALL = -4, /* workspace_bytes below the query function's answer   */
  HSTU_ERR_BAD_CP = -5,              /* cp_size < 1, a rank out of range, negative rows     */
  HSTU_ERR_HIP = -6,                 /* a HIP call failed; hipGetLastError() is left intact */
  HSTU_ERR_MISALIGNED = -7,          /* a data pointer is not 16-byte aligned               */
  HSTU_ERR_STATIC_SCRATCH = -8       /* hstu_jagged_attn_fwd_static: the problem needs more
                                        scratch than HSTU_STATIC_SCRATCH_BYTES                */
} hstu_status;

typedef enum { HSTU_BF16 = 0, HSTU_F32 = 1 } hstu_dtype;

typedef enum { HSTU_WS_FWD = 0, HSTU_WS_BWD = 1, HSTU_WS_CP = 2 } hstu_ws_kind;

/* Bits of hstu_attn_params.flags.  0 is the normal choice everywhere; the bits force one of the
 * library's forms where it would otherwise pick by problem size (testing, tuning, bit-for-bit
 * reproducibility).  Results are the same to rounding whatever the flags. */
typedef enum {
  HSTU_FLAG_NO_SPLIT = 1,       /* the forward and dQ passes never cut heavy query tiles along the keys
                                   (done when a problem has too few tiles to fill the chip); with it
                                   and HSTU_FLAG_NO_PACK a query row's result does not depend, bit for
                                   bit, on how many other rows the call has                        */
  HSTU_FLAG_NO_PACK = 2,        /* never tile across sequence boundaries ("packed tiles": bf16
                                   whole-batch calls whose mean length total_rows / batch is at
                                   most 256 tile the batch 128 rows at a time whatever sequences
                                   the rows belong to; the last bits of a row's result then depend
                                   on the sequences that share its tile)                          */
  HSTU_FLAG_PACK_SHORT = 4,     /* packed tiles up to a mean length of 1024 instead of 256         */
  HSTU_FLAG_FWD_TILE_128 = 8,   /* bf16 forward: the form that first builds a transposed copy of V in
                                   the workspace and reads that (one LDS instruction per matrix
                                   instruction instead of one and a half), with 128-row query tiles;
                                   the default reads V row-major and builds nothing               */
  HSTU_FLAG_FWD_TILE_256 = 16,  /* ... with 256-row query tiles                                    */
  HSTU_FLAG_DKDV_ONE_WAVE = 32, /* dk/dv pass at d_qk = d_v = 128: the kernel with one wave per 32
                                   keys instead of the one that splits the work over two          */
  HSTU_FLAG_BIAS_PER_PAIR = 64  /* calls with the timestamp bias (bf16): every block of pairs looks
                                   up the fp32 table entry of each pair; without it a block whose
                                   pairs share a bucket takes the entry as two bf16 halves (exact
                                   to 2^-16 of its value) through one matrix instruction          */
} hstu_flags;
#define HSTU_FLAGS_ALL 127

/* Problem description (section 2.1 for alpha and the mask, section 2.2 for the
 * jagged batch).  `total_rows` is passed by value so that grids and workspaces
 * can be sized without reading seq_offsets. */
typedef struct {
  int32_t batch;       /* B >= 0: number of sequences                                      */
  int32_t num_heads;   /* H >= 1: independent heads                                        */
  int32_t d_qk;        /* 32, 64 or 128                                                    */
  int32_t d_v;         /* 32, 64 or 128                                                    */
  int32_t max_len;     /* N >= 1: the normaliser 1/N; lengths above it are still computed  */
  float alpha;         /* scale inside the SiLU; the paper's 1/sqrt(d_k)                   */
  int32_t causal;      /* 1: key j visible to query i iff j <= i (in-sequence positions);
                          0: every key of the same sequence is visible                    */
  int32_t dtype;       /* hstu_dtype of the input tensors q, k, v, d_o                     */
  int64_t total_rows;  /* T = seq_offsets[batch], 0 <= T < 2^31                            */
  int32_t out_dtype;   /* hstu_dtype of the outputs o, dq, dk, dv: equal to dtype, or
                          HSTU_F32 to receive the fp32 accumulators unrounded (also the
                          precise choice for accumulate = 1 over several ring steps)      */
  int32_t flags;       /* 0, or an OR of hstu_flags; other bits HSTU_ERR_UNSUPPORTED            */
} hstu_attn_params;

/* One context-parallel step (section 2.3).  Local layout of rank r: for every
 * sequence in order, the rows of mini-chunk r followed by the rows of
 * mini-chunk 2*cp_size-1-r, where mini-chunk m of a sequence of length L holds
 * in-sequence positions [m*c, min((m+1)*c, L)) with c = ceil(L / (2*cp_size));
 * tail chunks may be short or empty and no padding row exists anywhere. */
typedef struct {
  int32_t cp_size;     /* CP >= 1                                                          */
  int32_t q_rank;      /* 0..CP-1: the rank whose query rows q_local holds                 */
  int32_t kv_rank;     /* 0..CP-1: k_part/v_part hold that rank's rows in local layout;
                          -1: they hold every row in the global (seq_offsets) layout      */
  int32_t accumulate;  /* 0: outputs are overwritten; 1: results are added to the outputs'
                          current contents (one ring step on top of the previous ones)    */
  int64_t q_rows;      /* rows in q_local / d_o_local / o_local / dq_local                 */
  int64_t kv_rows;     /* rows in k_part / v_part / dk_part / dv_part                      */
} hstu_cp_desc;

/* Forward over the whole jagged batch (section 2.1 equation, section 2.2 layout).
 *   q, k : [T, H, d_qk]   v : [T, H, d_v]   seq_offsets : int32 [B+1]   (inputs)
 *   o    : [T, H, d_v]    (output; every row of every sequence is written once, nothing else)
 */
int hstu_jagged_attn_fwd(const hstu_attn_params* params, const void* q, const void* k,
                         const void* v, const int32_t* seq_offsets, void* o, void* workspace,
                         size_t workspace_bytes, void* hip_stream);

/* hstu_jagged_attn_fwd for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, layouts, results (bit for bit) and errors, without the workspace: the schedule, the
 * transposed copy of V and the partial results of split tiles live in a static device array of
 * HSTU_STATIC_SCRATCH_BYTES inside the library, which every GPU the library runs on holds until
 * the process ends.  A problem whose hstu_jagged_attn_workspace_bytes(params, HSTU_WS_FWD) exceeds
 * that size is refused with HSTU_ERR_STATIC_SCRATCH and nothing is launched (a schedule needs a few
 * hundred bytes per sequence and 64 per 128 rows; a forced tile height adds a copy of V; from
 * max_len 4096 on a call may need up to
 * (rows / 128 + batch + 1024 / num_heads + 2) * num_heads * 128 * d_v * 4 bytes of partial results).
 * The call allocates nothing: no hipMalloc, hipFree or allocating library routine.  The device of
 * `hip_stream` must be the current device; the array's address on that device is looked up at the
 * first call there.  All calls on one GPU share that GPU's array: calls that overlap in time on
 * one GPU (different streams, or threads) race, and must be serialised by the caller.  Nothing
 * in the array has to survive between calls, and nothing in it is assumed to be zero. */
#define HSTU_STATIC_SCRATCH_BYTES (16u << 20)
size_t hstu_static_scratch_bytes(void);
int hstu_jagged_attn_fwd_static(const hstu_attn_params* params, const void* q, const void* k,
                                const void* v, const int32_t* seq_offsets, void* o, void* hip_stream);

/* Backward of the section 2.1 equation (the paper trains with it but does not print it; derived:
 * with x = alpha*<q_i,k_j>, sg = sigmoid(x), p = x*sg/N, dp = <d_o_i, v_j>/N, ds = dp*sg*(1+x*(1-sg)):
 * dv_j += p*d_o_i, dq_i += alpha*ds*k_j, dk_j += alpha*ds*q_i over the visible pairs): exact
 * gradients of sum(O * d_o) with respect to q, k, v.  S is recomputed from q and k; no forward
 * output or statistic is needed because the SiLU is pointwise.  dk and dv are accumulated per key tile without atomics;
 * dq is produced by a second pass over key tiles, so results are deterministic.
 *   d_o : [T, H, d_v] (input)    dq, dk : [T, H, d_qk]   dv : [T, H, d_v] (outputs)
 */
int hstu_jagged_attn_bwd(const hstu_attn_params* params, const void* q, const void* k,
                         const void* v, const void* d_o, const int32_t* seq_offsets, void* dq,
                         void* dk, void* dv, void* workspace, size_t workspace_bytes,
                         void* hip_stream);

/* Timestamp bias.  Section 2.1's equation has "+ Bias" inside the SiLU and describes the bias in
 * words only: differences of the rows' timestamps (of consecutive elements, the text says) are
 * transformed and grouped into bucket indices, which select entries of a learnable table.  The
 * transformation and the grouping are not given, and a term added to Q K^T needs a value per
 * (query, key) pair; this library's reading (PARITY WITH THE PAPER IS UNPINNED for it) takes the
 * difference of the pair's two timestamps:
 *     delta  = |timestamps[i] - timestamps[j]|                    (exact, up to 2^32 - 1)
 *     bucket = 0                                  if delta <= 1
 *            = min(num_buckets - 1, e * 2^f + m)  otherwise, e = floor(log2 delta), m = the f
 *              bits below delta's leading one (delta < 2^f: delta shifted up), f = groups_log2,
 *     x_ij   = alpha * (<Q_i, K_j> + ts_weights[bucket_ij])        (one table for all heads)
 * all in integer arithmetic, so no rounding decides a bucket.  With an all-zero table the
 * results equal those of the entry points without bias up to the order of fp32 additions.
 * Timestamps need not be sorted; blocks of pairs that fall into one bucket (the common case
 * for sorted timestamps away from the diagonal) take a faster path. */
typedef struct {
  const int32_t* timestamps;  /* device, [total_rows]: one per row, same layout as the rows     */
  const float* ts_weights;    /* device, [num_buckets] fp32: the table                          */
  float* d_ts_weights;        /* device, [num_buckets] fp32: backward output (overwritten: the
                                 sum over all visible pairs and heads of alpha * dS); NULL is
                                 allowed in the forward call.  Summed in 64-bit fixed point
                                 inside a workgroup (terms below 2^-32 of the unscaled dS are
                                 lost) and in double precision across workgroups             */
  int32_t num_buckets;        /* 1..512                                                         */
  int32_t groups_log2;        /* f: 0..8                                                        */
} hstu_ts_bias;

/* Workspace of the calls with bias (which: HSTU_WS_FWD, HSTU_WS_BWD, or HSTU_WS_CP for
 * hstu_jagged_attn_cp_partial_bias; 0 for invalid input). */
size_t hstu_jagged_attn_bias_workspace_bytes(const hstu_attn_params* params, int which);

/* hstu_jagged_attn_fwd / hstu_jagged_attn_bwd with the bias above; same arguments, layouts and
 * errors (fp32 inputs are computed in fp32 throughout, table and its gradient included), plus:
 * num_buckets or groups_log2 out of range HSTU_ERR_BAD_SHAPE, a NULL field of `bias` (other
 * than d_ts_weights in the forward call) HSTU_ERR_NULL_PTR.  dq, dk, dv are deterministic as in
 * hstu_jagged_attn_bwd; d_ts_weights is, up to the order of its double-precision additions. */
int hstu_jagged_attn_bias_fwd(const hstu_attn_params* params, const hstu_ts_bias* bias,
                              const void* q, const void* k, const void* v,
                              const int32_t* seq_offsets, void* o, void* workspace,
                              size_t workspace_bytes, void* hip_stream);
int hstu_jagged_attn_bias_bwd(const hstu_attn_params* params, const hstu_ts_bias* bias,
                              const void* q, const void* k, const void* v, const void* d_o,
                              const int32_t* seq_offsets, void* dq, void* dk, void* dv,
                              void* workspace, size_t workspace_bytes, void* hip_stream);

/* The timestamp bias for one context-parallel step: the two sides' timestamps in the layouts of
 * their buffers (see hstu_jagged_attn_cp_partial_bias). */
typedef struct {
  const int32_t* q_timestamps;   /* device, [q_rows]: the rows of q_local                          */
  const int32_t* kv_timestamps;  /* device, [kv_rows]: the rows of k_part / v_part                 */
  const float* ts_weights;       /* device, [num_buckets] fp32                                     */
  float* d_ts_weights;           /* device, [num_buckets] fp32; backward only (NULL otherwise):
                                    overwritten when cp->accumulate is 0, added to when it is 1    */
  int32_t num_buckets;           /* 1..512                                                         */
  int32_t groups_log2;           /* 0..8                                                           */
} hstu_cp_ts_bias;

/* One context-parallel rank's partial (section 2.3): the query rows of
 * `q_rank` against the keys of `kv_rank` (or all keys), masked on positions
 * inside the whole sequence, every visible (query chunk, key chunk) pair in one
 * launch.  `params->total_rows` and `seq_offsets_global` describe the full,
 * unsplit batch.
 *   q_local [q_rows,H,d_qk], k_part [kv_rows,H,d_qk], v_part [kv_rows,H,d_v]   (inputs)
 *   d_o_local [q_rows,H,d_v] or NULL for forward only
 *   o_local [q_rows,H,d_v] (output, may be NULL when d_o_local is given)
 *   dq_local [q_rows,H,d_qk], dk_part [kv_rows,H,d_qk], dv_part [kv_rows,H,d_v]
 *       (outputs, required iff d_o_local != NULL)
 * Summing o_local (dq_local) over kv_rank = 0..CP-1 gives q_rank's rows of the
 * full result; summing dk_part (dv_part) over q_rank gives kv_rank's rows.
 */
int hstu_jagged_attn_cp_partial(const hstu_attn_params* params, const hstu_cp_desc* cp,
                                const void* q_local, const void* k_part, const void* v_part,
                                const void* d_o_local, const int32_t* seq_offsets_global,
                                void* o_local, void* dq_local, void* dk_part, void* dv_part,
                                void* workspace, size_t workspace_bytes, void* hip_stream);

/* hstu_jagged_attn_cp_partial with the timestamp bias (same reading as hstu_jagged_attn_bias_fwd:
 * the bucket of |timestamp of the query row - timestamp of the key row|).  Same arguments and
 * errors, plus those of the calls with bias.  Workspace:
 * hstu_jagged_attn_bias_workspace_bytes(params, HSTU_WS_CP).  The partial table gradients of the
 * (query rank, key rank) pairs add up to the whole batch's. */
int hstu_jagged_attn_cp_partial_bias(const hstu_attn_params* params, const hstu_cp_desc* cp,
                                     const hstu_cp_ts_bias* bias, const void* q_local,
                                     const void* k_part, const void* v_part, const void* d_o_local,
                                     const int32_t* seq_offsets_global, void* o_local, void* dq_local,
                                     void* dk_part, void* dv_part, void* workspace,
                                     size_t workspace_bytes, void* hip_stream);

/* One rank's whole context-parallel pass as a ring of cp_size steps (section 3 names ring
 * attention as the variant for longer sequences; the partials are the ones of section 2.3).
 * Step s works on the K/V part of rank (q_rank - s) mod cp_size: the rank's own part first,
 * read in place, then the parts in the order they would arrive from the previous rank.  While a
 * step computes on `compute_stream`, the transfer of the next part runs on `copy_stream` into one
 * of two receive buffers (on one GPU a device-to-device copy stands in for the link; the
 * k_parts / v_parts pointers stand for the peers' memory).  o_local and dq_local are overwritten
 * by step 0 and accumulated by the later steps: give them fp32 (params->out_dtype) unless bf16
 * rounding between steps is acceptable.  The rank's contribution to the key-side gradients of
 * each part goes to dk_parts[r] / dv_parts[r] (added to them when accumulate_dkv != 0, as the
 * gradient buffer that travels with a part would be).
 * The call creates five HIP events (host objects, no device memory) for the ordering between the
 * two streams and destroys them before it returns; it is therefore not a call to make under
 * stream capture.
 * All arrays of the descriptor are host arrays of cp_size entries; the pointers in them are
 * device pointers.  Both streams must be distinct; on return everything is enqueued, the
 * compute stream carries the results, and the copy stream has been made to wait for the work
 * queued on the compute stream before the call.  Workspace as for hstu_jagged_attn_cp_partial.
 */
typedef struct hstu_cp_ring_desc {
  int32_t cp_size;
  int32_t q_rank;
  int32_t accumulate_dkv;        /* 0: overwrite dk_parts / dv_parts, 1: add to them */
  int32_t reserved;              /* must be 0 */
  int64_t q_rows;                /* rows of q_local (and d_o_local, o_local, dq_local) */
  int64_t recv_rows;             /* rows each receive buffer can hold (>= every other part) */
  const int64_t* part_rows;      /* rows of each rank's K/V part */
  const void* const* k_parts;    /* [part_rows[r], H, d_qk] */
  const void* const* v_parts;    /* [part_rows[r], H, d_v] */
  void* k_recv[2];               /* [recv_rows, H, d_qk] each */
  void* v_recv[2];               /* [recv_rows, H, d_v] each */
  void* const* dk_parts;         /* [part_rows[r], H, d_qk], out_dtype; NULL for forward only */
  void* const* dv_parts;         /* [part_rows[r], H, d_v] */
} hstu_cp_ring_desc;

int hstu_cp_ring_pass(const hstu_attn_params* params, const hstu_cp_ring_desc* ring,
                      const void* q_local, const void* d_o_local, const int32_t* seq_offsets_global,
                      void* o_local, void* dq_local, void* workspace, size_t workspace_bytes,
                      void* compute_stream, void* copy_stream);

/* The ring pass with the timestamp bias (hstu_jagged_attn_cp_partial_bias at every step): the
 * timestamps of a part's rows travel with its K and V.  Workspace:
 * hstu_jagged_attn_bias_workspace_bytes(params, HSTU_WS_CP).  d_ts_weights receives the rank's sum
 * over all its steps (overwritten). */
typedef struct hstu_cp_ring_ts_bias {
  const int32_t* q_timestamps;       /* [q_rows]: the rows of q_local                          */
  const int32_t* const* ts_parts;    /* per rank: [part_rows[r]] timestamps of its rows        */
  int32_t* ts_recv[2];               /* [recv_rows] each                                       */
  const float* ts_weights;           /* [num_buckets] fp32                                     */
  float* d_ts_weights;               /* [num_buckets] fp32, backward only (NULL otherwise)     */
  int32_t num_buckets;               /* 1..512                                                 */
  int32_t groups_log2;               /* 0..8                                                   */
} hstu_cp_ring_ts_bias;

int hstu_cp_ring_pass_bias(const hstu_attn_params* params, const hstu_cp_ring_desc* ring,
                           const hstu_cp_ring_ts_bias* bias, const void* q_local,
                           const void* d_o_local, const int32_t* seq_offsets_global, void* o_local,
                           void* dq_local, void* workspace, size_t workspace_bytes,
                           void* compute_stream, void* copy_stream);

/* Memory reorder for the load-balanced split (section 2.3: the "data shuffling ... memory
 * reordering" kernels that replace chunk + concatenate; section 3 credits them with +37 % QPS).
 * Moves whole rows between the global jagged layout and `rank`'s local layout (see hstu_cp_desc),
 * for up to four tensors at once (e.g. q, k, v, d_o), each with its own row length in bytes.
 *   scatter == 0 (gather):  dst[t][r] = src[t][g(r)]   dst: local [local_rows, ...], src: global
 *   scatter == 1:           dst[t][g(r)] = src[t][r]   dst: global, src: local (only the rank's
 *                           rows of dst are written; the gradient path back to the global layout)
 * where g(r) is the global row of local row r.  row_bytes[t] must be a multiple of 4 (multiples
 * of 16 move at full memory width; narrower rows, e.g. one int32 timestamp per row, word by
 * word); pointers 16-byte aligned.  Bit-exact copy; rows beyond local_rows / total_rows are never
 * touched.
 * One kernel launch on hip_stream; needs no workspace and allocates nothing.  seq_offsets is a
 * device pointer to batch + 1 int32 (the global offsets), read by the kernel only.
 */
int hstu_cp_reorder(int32_t batch, int64_t total_rows, int32_t cp_size, int32_t rank, int32_t scatter,
                    int32_t num_tensors, const void* const* src, void* const* dst,
                    const int64_t* row_bytes, int64_t local_rows, const int32_t* seq_offsets,
                    void* hip_stream);

/* Bytes of workspace the given entry point needs for `params` (an upper bound
 * that depends on batch, total_rows, num_heads, d_v and dtype only; 0 on invalid params).
 * Schedules, plus for bf16 forward passes with a forced tile height a transposed copy of V, plus
 * fp32 partial results where heavy
 * query tiles may be cut along the keys, plus 8 bytes per row for packed tiles.  The flags
 * change the answer: ask with the flags of the call.
 * `which` is a hstu_ws_kind. */
size_t hstu_jagged_attn_workspace_bytes(const hstu_attn_params* params, int which);

/* Host-side check of an offsets array the caller still has on the host:
 * HSTU_OK iff host_offsets[0] == 0, non-decreasing, host_offsets[batch] == total_rows. */
int hstu_validate_offsets_host(const int32_t* host_offsets, int32_t batch, int64_t total_rows);

/* Static, NUL-terminated description of a status code. */
const char* hstu_attn_status_string(int status);

/* ---- schedule inspection (for tests of the tile table, section 2.2 / 2.3) -------------------
 * Builds on the device, exactly as the attention entry points do (when they tile per sequence:
 * packed tiles have a schedule of their own, 128 consecutive rows per item in row order, which this
 * call does not show), the table of work items for one side of a problem and copies it to host
 * memory (this call synchronises the stream).
 *   side: 0 = items are query tiles streaming over key segments (forward, dq pass)
 *         1 = items are key tiles streaming over query segments (dk/dv pass)
 *   cp == NULL: whole-batch attention; else the context-parallel problem it describes
 *   items_host: room for max_items * 12 int32; per item
 *       {row0, nrows, pos0, nseg, seg_row0[2], seg_len[2], seg_pos0[2], cost, 0}
 *   returns the number of items (>= 0) in schedule order (non-increasing cost), or a status < 0.
 */
int hstu_debug_dump_schedule(const hstu_attn_params* params, const hstu_cp_desc* cp, int side,
                             const int32_t* seq_offsets, int32_t* items_host, int32_t max_items,
                             void* workspace, size_t workspace_bytes, void* hip_stream);

/* ---- per-launch timing (for benchmarks; the roofline figures of the measurement section) -----
 * Between hstu_debug_timing_begin() and hstu_debug_timing_end() every kernel the library
 * launches from the calling thread is bracketed by HIP events recorded on the stream it is
 * launched on.  This is the one piece of (thread-local) state the library ever keeps.
 *   begin: max_records in [1, 65536]; launches beyond it are not recorded.
 *   end:   waits for the recorded launches, writes per launch, in launch order, its kind
 *          (0 forward, 1 dk/dv pass, 2 dq pass, 3 schedule build, 4 transposed copy,
 *          5 reorder, 6 sum of the partial results of split tiles, 7 timestamp records,
 *          8 scaling of the bias table's gradient, 9 matrix-instruction loop, 10 atomic-rate kernel) and its duration in milliseconds; returns the number written (<= capacity) or a status < 0.
 */
int hstu_debug_timing_begin(int max_records);
int hstu_debug_timing_end(int32_t* kinds, float* milliseconds, int capacity);

/* ---- measurement kernels (the measurement section: what the attention kernels' rates are read
 * against) -----------------------------------------------------------------------------------
 * hstu_debug_mfma_loop: one launch of a kernel that issues nothing but v_mfma_f32_32x32x16_bf16 in
 * its loop (two workgroups of four waves per CU, four independent accumulators per wave,
 * `iterations` x 4 instructions per wave), with the same operand values in every lane
 * (random_operands = 0) or different ones (1: the chip's power limit, and with it the clock it
 * holds, depends on the data).  *flops_per_launch receives the flops of the launch (host pointer);
 * the caller times it (kind 9 of the timing recorder).  sink: device, 64 floats, never written in
 * practice.  This is the rate the matrix cores sustain on this machine; the published peak assumes
 * the 2.4 GHz clock.
 * hstu_debug_dq_atomic_rate: one launch of 256 workgroups (one per CU) that add 1.0 with fp32
 * atomics (no return value) to dq_f32 [rows, num_heads, 128] in the pattern a dk/dv pass would need
 * to produce dq itself: per 32-row block 16 KB per workgroup, each instruction covering two rows
 * of 128 contiguous bytes; head_per_xcd != 0 keeps every head's rows to one XCD (num_heads = 8).
 * *payload_bytes_per_launch receives the bytes added (host pointer); kind 10 of the recorder. */
int hstu_debug_mfma_loop(int random_operands, int iterations, float* sink, double* flops_per_launch,
                         void* hip_stream);
int hstu_debug_dq_atomic_rate(float* dq_f32, int64_t rows, int32_t num_heads, int32_t blocks,
                              int32_t head_per_xcd, double* payload_bytes_per_launch, void* hip_stream);

/* Rows per work item on the given side for a whole-batch problem described by `params` (the
 * tile height depends on the problem size: large problems use taller query tiles). */
int hstu_schedule_tile_rows(const hstu_attn_params* params, int side);

#ifdef __cplusplus
}
#endif
#endif /* HSTU_ATTN_H_ */
