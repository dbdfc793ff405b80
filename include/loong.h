/*
 * loong.h - C ABI of the per-device ring-step attention of Double-Ring-Attention.
 *
 * One GPU of a context-parallel group holds a local Q chunk and, at every ring
 * micro-step, one visiting K/V chunk.  Per micro-step it runs a blockwise softmax
 * attention of its Q against that chunk and folds the partial result into the running
 * output with a log-sum-exp update (paper: Alg. 2, the `Attention` and `Update` calls of
 * the inner loop).  The backward pass replays the chunks and, per micro-step, produces
 * the visiting chunk's dK/dV and this step's share of dQ from the stored attention
 * output and softmax_lse (paper: Sec. 3.1 last paragraph; Sec. "Selective Checkpoint++").
 *
 * Conventions for every entry point
 *   - plain C, no exceptions, returns 0 (LOONG_OK) or a negative LOONG_E_* code; the
 *     text of the last error of the calling thread is at loong_last_error().
 *   - every tensor pointer is a DEVICE pointer owned by the caller and must stay valid
 *     until the work enqueued on `stream` has finished; descriptors and the small
 *     arrays of loong_zigzag_mask are HOST memory read during the call.
 *   - nothing allocates, frees or synchronises, and the library keeps no state between
 *     calls (apart from the error text and a write-once table of device properties);
 *     kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = the default
 *     stream); scratch memory a call needs is handed in by the caller (`workspace`).
 *   - the kernels are built for gfx950 only: on any other device the step calls return
 *     LOONG_E_UNSUPPORTED; launch shapes follow the device's compute-unit count.
 *   - arguments are validated before anything is launched; on error nothing is enqueued.
 *   - layouts: 16-bit/fp32 inputs q,k,v,o,d_o are [batch, head, token, head_dim] with
 *     element strides given in the descriptor (head_dim stride 1).  fp32 results `out`
 *     and `dq` use o_stride; `dk`,`dv` are contiguous [batch, n_kv_heads, kv_len, head_dim];
 *     `lse` and `delta` are contiguous [batch, n_q_heads, q_len].
 */
#ifndef LOONG_H
#define LOONG_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__)
#define LOONG_API __attribute__((visibility("default")))
#else
#define LOONG_API
#endif

#define LOONG_OK              0
#define LOONG_E_NULL         -1   /* a required pointer is NULL */
#define LOONG_E_SHAPE        -2   /* negative/inconsistent sizes, bad rank/step/cp */
#define LOONG_E_UNSUPPORTED  -3   /* head_dim, head grouping or size outside the kernels' range */
#define LOONG_E_ALIGN        -4   /* pointer not 16-byte aligned or stride not vectorisable */
#define LOONG_E_DTYPE        -5   /* unknown dtype code */
#define LOONG_E_HIP          -6   /* the HIP runtime refused a launch */

/* storage type of q, k, v, o, d_o */
#define LOONG_BF16 0              /* bf16 MFMA kernels, head_dim 64 or 128 */
#define LOONG_FP32 1              /* fp32 storage, head_dim <= 128, multiple of 4: a correctness path for small
                                     cases (one wave per row, plain fp32 multiply-adds, no matrix cores, no
                                     tiling): far from any roofline and not meant for long sequences */
#define LOONG_FP16 2              /* the MFMA kernels on IEEE half storage (the 16-bit type Sec. "Performance
                                     Analysis" sizes the tensors in), head_dim 64 or 128 */

/* class of a (q half, k half) block of one micro-step */
#define LOONG_SKIP 0              /* key chunk lies after the query chunk: nothing visible */
#define LOONG_FULL 1              /* key chunk lies before the query chunk: everything visible */
#define LOONG_DIAG 2              /* same chunk: key offset <= query offset */

/* flags */
#define LOONG_FUSE_MERGE     1    /* fwd: out/lse hold the running result; the step is merged in-kernel */
#define LOONG_ACCUM_DKV      2    /* bwd: dk/dv are added to instead of overwritten */
#define LOONG_COMPUTE_DELTA  4    /* bwd: fill `delta` from o and d_o before the step */
#define LOONG_BWD_ONLY_DKV   8    /* bwd: compute dk/dv only (dq may be NULL and is not touched) */
#define LOONG_BWD_ONLY_DQ    16   /* bwd: compute this step's share of dq only (dk, dv may be NULL) */
/* Tuning/testing knob of the 16-bit kernels that own query rows (forward, dQ): bits 8..10 of
 * `flags` hold 1, 2 or 4 to force that many key splits per workgroup (waves that share the
 * same rows and divide every staged key tile); 0 = chosen from the shape and the device. */
#define LOONG_KEY_SPLITS_SHIFT 8
#define LOONG_KEY_SPLITS(n)  ((n) << LOONG_KEY_SPLITS_SHIFT)

typedef struct loong_step_desc {
  int32_t batch;
  int32_t n_q_heads;      /* local q heads; q head h reads kv head h / (n_q_heads / n_kv_heads) */
  int32_t n_kv_heads;     /* local kv heads (after any replication), divides n_q_heads */
  int32_t head_dim;
  int32_t q_len;          /* local q tokens;  causal: 2 * chunk_len */
  int32_t kv_len;         /* tokens of the visiting chunk; causal: 2 * chunk_len */
  int32_t chunk_len;      /* causal only: length c of one zigzag half */
  int32_t q_chunk[2];     /* causal only: global chunk ids of q rows [0,c) and [c,2c) */
  int32_t kv_chunk[2];    /* causal only: same for the visiting keys */
  int32_t causal;         /* 0: every key visible to every row (chunk fields ignored) */
  int32_t dtype;          /* LOONG_BF16 | LOONG_FP32 | LOONG_FP16 */
  float   softmax_scale;  /* multiplies q.k before the softmax (e.g. 1/sqrt(head_dim)) */
  int32_t flags;
  int64_t q_stride[3];    /* batch, head, token strides (elements) of q, o and d_o */
  int64_t kv_stride[3];   /* same for k and v */
  int64_t o_stride[3];    /* same for the fp32 out and dq */
} loong_step_desc;

/*
 * Zigzag layout and ring order (host only, pure).  Paper: Sec. 2 "Distributed Attention"
 * (load-balanced causal reorder) and Alg. 2 (outer loop of cp/inner_w steps around an
 * inner loop of inner_w micro-steps; sends go to the next rank, receives come from the
 * previous).  The sequence is cut into 2*cp chunks; rank r owns chunks r and 2cp-1-r.
 * Ranks are numbered i*inner_w + j for the j-th GPU of the i-th inner ring.
 * `step` counts micro-steps 0..cp-1 in execution order.  Outputs (any may be NULL):
 *   src_rank    rank whose chunk is held at that micro-step
 *   q_chunk     {rank, 2cp-1-rank};  kv_chunk  {src, 2cp-1-src}
 *   block_class [qhalf*2 + khalf] in {LOONG_SKIP, LOONG_FULL, LOONG_DIAG}
 * Errors: LOONG_E_SHAPE if cp < 1, inner_w < 1, cp % inner_w != 0, rank or step out of range.
 */
LOONG_API int loong_zigzag_mask(int32_t cp, int32_t inner_w, int32_t rank, int32_t step,
                      int32_t* src_rank, int32_t q_chunk[2], int32_t kv_chunk[2],
                      uint8_t block_class[4]);

/*
 * One micro-step forward: `Attention(Q, K, V)` of Alg. 2, optionally fused with `Update`.
 * q [B,Hq,q_len,d], k/v [B,Hkv,kv_len,d] in desc->dtype.
 * Without LOONG_FUSE_MERGE: out <- softmax(scale q k^T + mask) v over this chunk only,
 * lse <- natural-log sum of exp of the masked scaled scores; rows that see no key get
 * out = 0, lse = -inf.  With LOONG_FUSE_MERGE: (out, lse) is the running result (start
 * from out = 0, lse = -inf) and is replaced by its update with this step's partial;
 * rows that see no key are left untouched.  Fixed order of operations per row:
 * results are bit-reproducible run to run.
 */
LOONG_API int loong_attn_step_fwd(const loong_step_desc* desc, const void* q, const void* k, const void* v,
                        float* out, float* lse, void* stream);

/*
 * `Update(out, lse, block_out, block_lse)` of Alg. 2, in place on (out, lse):
 *   lse' = log(exp(lse) + exp(block_lse)),
 *   out' = exp(lse - lse') out + exp(block_lse - lse') block_out.
 * rows = batch*heads*tokens; out/block_out [rows, head_dim] fp32 contiguous, lse/block_lse
 * [rows].  A side with lse = -inf contributes nothing.  head_dim must be a multiple of 4.
 */
LOONG_API int loong_lse_merge(int64_t rows, int32_t head_dim, float* out, float* lse,
                    const float* block_out, const float* block_lse, void* stream);

/*
 * One micro-step backward (paper: Sec. 3.1, gradients of the visiting K/V travel with the
 * chunk; the kernel recomputes the probabilities from the stored softmax_lse).
 * Inputs: q, d_o [B,Hq,q_len,d] (q_stride), k, v the visiting chunk, lse and delta
 * [B,Hq,q_len] of the COMPLETE attention (all chunks merged), delta_i = sum_k d_o_ik o_ik.
 * With LOONG_COMPUTE_DELTA, `o` (stored output, same type/strides as q) must be given and
 * delta is written first; otherwise `o` may be NULL.
 * Outputs: dq [B,Hq,q_len,d] fp32 (o_stride) is ADDED to (zero it before the first
 * step); every row is updated by one thread group in a fixed order, so dq is
 * bit-reproducible.  dk, dv fp32 contiguous [B,Hkv,kv_len,d] are overwritten, or added to
 * with LOONG_ACCUM_DKV (a plain read-modify-write: two calls that add into the same dk, dv
 * must be ordered).  dk, dv are bit-reproducible too: when a step has too few key tiles to
 * fill the chip, several workgroups share a key tile's query loop and the last one to
 * arrive adds their partial sums in a fixed order.  Those partial sums and their arrival
 * counters live in `workspace`, device memory of the caller's, 16-byte aligned, at least
 * loong_workspace_bytes(desc) bytes (that may be 0: then `workspace` may be NULL).  It
 * may hold anything on entry (the call clears what it counts in with a kernel of its own on
 * `stream`) and holds nothing of value afterwards; calls that share one workspace must be
 * ordered on one stream.  A missing or too small workspace is LOONG_E_NULL / LOONG_E_SHAPE
 * and nothing is enqueued.  The bf16/fp16 kernels only; the fp32 kernels need none.
 * The two halves run as two kernels on `stream`; LOONG_BWD_ONLY_DKV / LOONG_BWD_ONLY_DQ
 * run one of them (both flags together: LOONG_E_UNSUPPORTED).
 */
LOONG_API int loong_attn_step_bwd(const loong_step_desc* desc, const void* q, const void* k, const void* v,
                        const void* o, const void* d_o, const float* lse, float* delta,
                        float* dq, float* dk, float* dv, void* workspace, int64_t workspace_bytes,
                        void* stream);

/*
 * loong_attn_step_bwd for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, semantics, results (bit for bit) and errors as loong_attn_step_bwd, except that
 * the scratch of the dK/dV kernel is an array of LOONG_STATIC_SCRATCH_BYTES inside the library's
 * device code (each GPU the library is used on holds its own copy until the process ends).
 * The call allocates and frees nothing and does not synchronise.  A step that needs more
 * scratch than the array holds (loong_workspace_bytes(desc) > LOONG_STATIC_SCRATCH_BYTES) is
 * refused with LOONG_E_UNSUPPORTED and nothing is enqueued: use loong_attn_step_bwd.  All
 * calls on one GPU share that GPU's array: calls that overlap on one GPU (two streams, two
 * threads) race on it and must be ordered by the caller; the array keeps the last call's
 * contents, and each call clears what it counts in on `stream` before its kernels use it.
 */
#define LOONG_STATIC_SCRATCH_BYTES (((int64_t)64 << 20) + 65536)
LOONG_API int loong_attn_step_bwd_static(const loong_step_desc* desc, const void* q, const void* k, const void* v,
                                         const void* o, const void* d_o, const float* lse, float* delta,
                                         float* dq, float* dk, float* dv, void* stream);

/* delta_i = sum_k d_o_ik * o_ik for every row; o, d_o in desc->dtype with q_stride. */
LOONG_API int loong_bwd_delta(const loong_step_desc* desc, const void* o, const void* d_o, float* delta,
                    void* stream);

/* Set a running result to the neutral element of Update: out = 0, lse = -inf. */
LOONG_API int loong_init_running(int64_t rows, int32_t head_dim, float* out, float* lse, void* stream);

/* Cast the merged fp32 output [rows, head_dim] to the stored activation type
 * (LOONG_BF16, LOONG_FP16: round to nearest even, fp16 overflow gives infinity; LOONG_FP32: copy),
 * contiguous. */
LOONG_API int loong_finalize_out(int64_t rows, int32_t head_dim, const float* out, void* o, int32_t dtype,
                       void* stream);

/* Bytes of workspace loong_attn_step_bwd needs for this step (0 when no query loop is shared).
 * Host-only; the answer depends on the compute-unit count of the current device (an MI355X's
 * 256 when there is none to ask), so ask on the device that will run the step.  An upper bound
 * over the steps of a replay is the maximum over its descriptors. */
LOONG_API int loong_workspace_bytes(const loong_step_desc* desc, int64_t* bytes);

/* Validate a descriptor exactly as the step calls do, without touching a device. */
LOONG_API int loong_validate_step(const loong_step_desc* desc);

/* Text of the calling thread's last error ("" if none). Never NULL. */
LOONG_API const char* loong_last_error(void);

/*
 * Row permutation: the local half of SeqAlltoAll and the KV replication of Alg. 1 (paper:
 * Sec. 3.1 steps 1 and 3; Sec. "KV Replication for GQA").  Copies n0*n1*n2 rows of
 * `row_bytes` bytes (a multiple of 16; rows 16-byte aligned): row (a, b, c) is read at
 * in + (a*in_stride[0] + b*in_stride[1] + c*in_stride[2]) bytes and written at the same
 * expression with out_stride.  Strides are in BYTES, multiples of 16; an input stride may be 0
 * (replication), output rows must not overlap.  Examples, with e = element size and
 * hl = H / d_hp:
 *   heads of (s, H, d) token-major into d_hp messages (d_hp, hl, s, d):
 *     n = {d_hp, hl, s}, in_stride = {hl*d*e, d*e, H*d*e}, out_stride = {hl*s*d*e, s*d*e, d*e}
 *   d_hp received messages (d_hp, hl, s, d) into (hl, d_hp*s, d):
 *     n = {d_hp, hl, s}, in_stride = {hl*s*d*e, s*d*e, d*e}, out_stride = {s*d*e, d_hp*s*d*e, d*e}
 *   replication (H_kv, s, d) -> (H_kv*rep, s, d): n = {H_kv, rep, s}, in_stride = {s*d*e, 0, d*e}
 * Errors: LOONG_E_NULL, LOONG_E_SHAPE (negative sizes), LOONG_E_ALIGN.
 */
LOONG_API int loong_permute_rows(const int64_t n[3], const int64_t in_stride[3], const int64_t out_stride[3],
                                 int64_t row_bytes, const void* in, void* out, void* stream);

/*
 * Gradient of the KV replication (paper: Sec. "KV Replication for GQA", backward pass): the fp32
 * gradients of the `rep` copies of every head are added in copy order.
 * in [heads*rep, rows_per_head*head_dim] fp32 contiguous -> out [heads, rows_per_head*head_dim].
 * `elems_per_head` = rows_per_head*head_dim must be a multiple of 4; pointers 16-byte aligned;
 * in and out must not overlap.  Errors: LOONG_E_NULL, LOONG_E_SHAPE, LOONG_E_ALIGN.
 */
LOONG_API int loong_reduce_replicas(int64_t heads, int32_t rep, int64_t elems_per_head, const float* in, float* out,
                                    void* stream);

/*
 * Performance model of 2D-Attention (paper: Sec. "Performance Analysis": "Computation
 * Analysis", "P2P Communication Analysis", "SeqAlltoAll Communication Analysis").  Host only.
 * Inputs: sequence length S and hidden size D (elements), H query heads, H_kv key/value
 * heads, the grid d_hp x d_cp, the inner ring size w (divides d_cp; d_hp divides H), the
 * forward compute constant alpha_fwd in seconds per unit of S^2 D (fit it to a measured
 * forward micro-step), the bandwidths in bytes per second of an inner-ring transfer, an
 * outer-ring transfer and the all-to-all, and a per-message latency in seconds.
 * Outputs, in the paper's notation (bytes and seconds):
 *   size_kv = max(H_kv, d_hp) / H * 4 S D / d_sp        size_q = 2 S D / d_sp
 *   alltoall_volume = sum over q, k, v, out of Size(i) * (d_hp - 1) / d_hp   (one phase)
 *   t_comp_fwd = alpha S^2 D / (d_cp d_sp)               t_comp_bwd = 3 t_comp_fwd
 *   t_p2p_* = latency + bytes / bandwidth; the backward moves the chunk and its gradient (2x)
 *   t_inner_ring = A (w - 1) + B,  A = max(t_comp, t_p2p_inner),  B = max(t_comp, t_p2p_outer)
 *   t_seq_alltoall = 2 * alltoall_volume / bw_alltoall   (forward and backward phase)
 *   objective = t_seq_alltoall + (t_inner_ring_fwd + t_inner_ring_bwd) * d_cp / w
 * Errors: LOONG_E_NULL; LOONG_E_SHAPE for non-positive sizes, bandwidths or alpha, d_hp not
 * dividing H, w not dividing d_cp, H_kv not dividing H.
 */
typedef struct loong_cost_in {
  double S, D;
  int32_t H, H_kv, d_hp, d_cp, w;
  double alpha_fwd;
  double bw_p2p_inner, bw_p2p_outer, bw_alltoall;
  double latency;
} loong_cost_in;

typedef struct loong_cost_out {
  double size_kv, size_q, alltoall_volume;
  double t_comp_fwd, t_comp_bwd;
  double t_p2p_inner_fwd, t_p2p_outer_fwd, t_p2p_inner_bwd, t_p2p_outer_bwd;
  double t_inner_ring_fwd, t_inner_ring_bwd, t_seq_alltoall, objective;
} loong_cost_out;

LOONG_API int loong_cost_model(const loong_cost_in* in, loong_cost_out* out);

/*
 * The grid with the smallest objective for d_sp GPUs: every d_hp that divides both d_sp and H,
 * d_cp = d_sp / d_hp, every w <= max_w that divides d_cp (ties: smaller d_hp, then smaller w).
 * `in->d_hp`, `in->d_cp`, `in->w` are ignored; the winner is written to `best_in` (the full
 * input with its grid) and `best_out`.  Errors as loong_cost_model, plus LOONG_E_SHAPE when no
 * grid is admissible.
 */
LOONG_API int loong_cost_search(const loong_cost_in* in, int32_t d_sp, int32_t max_w, loong_cost_in* best_in,
                                loong_cost_out* best_out);

/*
 * Measurement aid: a kernel of nothing but dependent-free v_mfma_f32_32x32x16_bf16 chains on
 * every SIMD of the device (`workgroups` x 4 waves x `iters` x 4 instructions).  It writes
 * one float per thread to `sink` (workgroups * 256 floats, device memory) so that the work
 * cannot be dropped.  Timing it gives the matrix-core rate the chip sustains at its real
 * clocks, the second ceiling `bench.py` prints beside the published peak.  That rate depends on
 * the operand VALUES (the clock the chip holds falls as more bits toggle): with `operands` NULL
 * the kernel uses nearly constant built-in operands; otherwise `operands` points at 2048 bytes
 * of device memory, 16-byte aligned, read only: lane l of every wave takes its eight A elements
 * from bytes [16 l, 16 l + 16) and its eight B elements from bytes [1024 + 16 l, +16), e.g. bf16
 * values drawn like the workload's.  FLOPs of a call: workgroups * 4 * iters * 4 * 32768.
 * Errors: LOONG_E_NULL (sink), LOONG_E_ALIGN (operands), LOONG_E_SHAPE (non-positive sizes).
 */
LOONG_API int loong_mfma_probe(int32_t workgroups, int32_t iters, const void* operands, float* sink, void* stream);

/* Library version, major*10000 + minor*100 + patch. */
LOONG_API int loong_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LOONG_H */
