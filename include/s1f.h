/* s1f — segment-wise causal attention for sequence-level 1F1B pipeline stages, MI355X (gfx950).
 *
 * C ABI of the library.  Plain pointers and sizes only; no framework types.
 *
 * The operations follow "Seq1F1B: Efficient Sequence-Level Pipeline Parallelism for Large Language
 * Model Training" (arXiv 2406.03488):
 *   - Section 3.1, Eq. 3: causal softmax attention; a token attends to itself and all earlier tokens,
 *     scores scaled by 1/sqrt(head_dim).
 *   - Section 3.1 (last paragraph) and Section 3.2: a sequence is cut into segments; the forward of a
 *     segment needs the keys/values of all preceding tokens (the "prefix"); backward passes run in
 *     reverse segment order and their gradients are accumulated so that the result equals that of the
 *     unsplit sequence.
 *   - Section 3.4, Eq. 7-8: segment lengths are chosen so that every segment costs the same FLOPs.
 *
 * Conventions common to all device entry points
 *   - All tensor pointers are DEVICE pointers owned by the caller; the library allocates nothing,
 *     keeps no caller pointer after return, and its only global state is what it asked the runtime once per
 *     device and kernel and remembers: that the kernel may use more than 64 KiB of LDS, how many of its
 *     workgroups the device holds at once, and the address of the scratch array built into the library
 *     (s1f_seg_attn_bwd_noalloc).  Calls are re-entrant.
 *   - Layout is [batch, head, sequence, head_dim] with head_dim contiguous; the other three strides
 *     are passed in ELEMENTS through s1f_desc.  q, out, dout, dq share the q_* strides; k, v share the
 *     kv_* strides; dk_prefix_acc, dv_prefix_acc share the kv_* strides too (in fp32 elements).
 *     lse is a dense fp32 array [batch, n_q_heads, seg_len].
 *   - Query head h reads key/value head h / (n_q_heads / n_kv_heads) (contiguous groups).
 *   - Kernels are enqueued on `hip_stream` (a hipStream_t passed as void*; NULL = default stream) and
 *     the call returns without synchronising.  Arguments are validated before anything is enqueued: on
 *     S1F_EINVAL, S1F_EUNSUPPORTED or S1F_ERANGE nothing has been launched and no output was touched.
 *     S1F_EDEVICE reports that the HIP runtime refused a launch of THIS call (errors left behind by the
 *     caller's earlier HIP work are not picked up); a call made of several launches (s1f_seg_attn_bwd, the
 *     cache calls with batch > 1) may then have enqueued its earlier ones, so its outputs are undefined.
 *   - Every entry point returns an s1f_status; nothing throws or aborts across this boundary.
 */
#ifndef S1F_H
#define S1F_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  S1F_OK = 0,
  S1F_EINVAL = 1,       /* null pointer, non-positive size, inconsistent descriptor */
  S1F_EUNSUPPORTED = 2, /* dtype / head_dim combination without a kernel, or a size beyond a kernel's limits */
  S1F_ERANGE = 3,       /* segment does not fit: seg_off < 0, seg_len < 1, seg_off + seg_len > kv_capacity */
  S1F_EDEVICE = 4,      /* the HIP runtime reported an error at launch */
  S1F_ESCRATCH = 5      /* s1f_seg_attn_bwd_noalloc only: the call needs more scratch than the built-in buffer holds */
} s1f_status;

typedef enum {
  S1F_F32 = 0, /* q, k, v, out, dout, dq are fp32; fp32 matrix arithmetic */
  S1F_BF16 = 1 /* q, k, v, out, dout, dq are bf16; bf16 MFMA with fp32 accumulation; probabilities and
                  score gradients are rounded to bf16 before their second product */
} s1f_dtype;

typedef struct {
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads; /* must divide n_q_heads */
  int32_t head_dim;   /* 64, 80 or 128 */
  int32_t dtype;      /* s1f_dtype; lse and the dK/dV accumulators are always fp32 */
  int32_t reserved;   /* must be 0 */
  int64_t q_stride_b, q_stride_h, q_stride_s;    /* elements; head_dim <= q_stride_s < 2^23 */
  int64_t kv_stride_b, kv_stride_h, kv_stride_s; /* elements; head_dim <= kv_stride_s < 2^23 (the kernels' asynchronous
                                                    copies use 32-bit byte offsets inside a tile; S1F_EUNSUPPORTED beyond) */
  int64_t kv_capacity; /* rows allocated per head in k, v, dk_prefix_acc, dv_prefix_acc */
} s1f_desc;

/* Computation-wise partition (Section 3.4, Eq. 7-8).  HOST function, no device work.
 *
 * Writes n_seg + 1 boundaries 0 = b[0] < b[1] < ... < b[n_seg] = seq_len into the caller-owned HOST
 * array `boundaries`; segment i (1-based) holds tokens b[i-1] .. b[i]-1.
 * Cost model: Eq. 8 with P/L = 12 hidden^2, made additive over tokens so that the k costs of Eq. 7 can
 * be equal: token t (1-based) costs w(t) = 6*hidden + t (units of 4*L*hidden FLOPs; the t is its
 * causal attention over t keys), the first x tokens cost W(x) = 6*hidden*x + x(x+1)/2.  b[i] is the
 * integer x minimising |n_seg*W(x) - i*W(seq_len)| (smaller x on a tie), then clamped so that every
 * segment keeps at least one token.  `heads` is validated (must divide hidden) and otherwise unused.
 * Errors: S1F_EINVAL for n_seg < 1, seq_len < n_seg, hidden < 1, heads < 1, hidden % heads != 0,
 * boundaries == NULL, or sizes whose cost would overflow 2^62. */
int s1f_partition(int64_t seq_len, int32_t n_seg, int32_t hidden, int32_t heads, int64_t *boundaries);

/* Variants of the partition (Section 3.4, Eq. 7-8).  HOST functions.
 *
 * cost_model S1F_COST_ADDITIVE is s1f_partition's rule.  S1F_COST_LITERAL takes the per-segment line of
 * Eq. 8 as printed: segment (a, b] costs (b - a) * (12*hidden + b) (units of 2*L*hidden FLOPs, its keys counted
 * up to and including the segment itself for every row).  That cost is not additive over tokens, so the k costs
 * cannot be made equal; the result is the composition whose largest cost is smallest, and among those the
 * lexicographically smallest boundaries.
 * `align` >= 1 restricts b[1] .. b[n_seg-1] to multiples of `align` (the paper does not align; 1 reproduces
 * s1f_partition).  Additive model: b[i] is the multiple of align in [0, seq_len] nearest in prefix cost to
 * i/n_seg of the total (smaller on a tie), clamped so that consecutive boundaries differ by at least `align`
 * and the last segment keeps a token.
 * Errors: as s1f_partition, plus S1F_EINVAL for align < 1, an unknown cost_model, or fewer than n_seg - 1
 * multiples of align in [align, seq_len - 1]. */
typedef enum { S1F_COST_ADDITIVE = 0, S1F_COST_LITERAL = 1 } s1f_cost_model;
int s1f_partition_ex(int64_t seq_len, int32_t n_seg, int32_t hidden, int32_t heads, int32_t cost_model,
                     int64_t align, int64_t *boundaries);

/* Re-balances a partition on MEASURED segment costs (Section 3.4's goal, equal time per segment, applied to
 * what a run actually took instead of the FLOP model of Eq. 8).  HOST function.
 *
 *   boundaries_in  [n_seg + 1]  current boundaries, 0 = b[0] < ... < b[n_seg] = sequence length
 *   seg_cost       [n_seg]      measured cost of each segment in any integer unit (e.g. nanoseconds), >= 0,
 *                               sum in [1, 2^48]
 *   boundaries_out [n_seg + 1]  caller-owned; may not alias boundaries_in
 * Every token of segment i is taken to cost seg_cost[i] / length_i; boundary j becomes the multiple of `align`
 * whose measured prefix cost is nearest to j/n_seg of the total (smaller on a tie, exact rational comparison),
 * clamped as in s1f_partition_ex.  Applying it again to the costs measured on its output converges on equal
 * measured time when the cost per token varies smoothly.
 * Errors: S1F_EINVAL for null pointers, n_seg < 1 or > 65536, boundaries not strictly increasing from 0,
 * a negative cost, a zero or too large sum, more than 2^30 tokens, align < 1 or too coarse for n_seg. */
int s1f_partition_rebalance(int32_t n_seg, const int64_t *boundaries_in, const int64_t *seg_cost, int64_t align,
                            int64_t *boundaries_out);

/* Forward of one segment (Section 3.1 Eq. 3 restricted to the segment's rows; Section 3.2).
 *
 *   q_seg     [batch, n_q_heads, seg_len, head_dim]  queries of absolute rows seg_off .. seg_off+seg_len-1
 *   k_prefix, v_prefix  point at row 0 of the caller's K/V cache; rows [0, seg_off+seg_len) must be
 *             valid and already include the segment's own keys/values
 *   out       [batch, n_q_heads, seg_len, head_dim]  overwritten (dtype of the descriptor)
 *   lse       [batch, n_q_heads, seg_len] fp32, overwritten: natural-log sum-exp of the scaled scores
 * Row r of the segment attends to keys j <= seg_off + r. */
int s1f_seg_attn_fwd(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix,
                     int64_t seg_off, int64_t seg_len, void *out, float *lse, void *hip_stream);

/* s1f_seg_attn_fwd with a caller-owned device workspace, which lets the library shorten the end of a launch: the
 * method turns one long launch into n_seg short ones (Sections 3.1-3.2), and a short launch ends with most of the
 * chip idle while its last few row tiles walk their whole prefix.  With a workspace the last row tiles are cut into
 * chunks along the keys that run side by side; each chunk leaves an unnormalised partial result there and a small
 * second kernel merges them by their log-sum-exp.  Same results up to fp32 rounding of that merge; bf16 only (fp32
 * descriptors run unsplit).
 *   workspace        device memory, 16-byte aligned, at least s1f_fwd_workspace_bytes(desc, seg_off, seg_len) bytes
 *                    (0 when this launch is not split: workspace may then be NULL); contents undefined afterwards
 * Errors as s1f_seg_attn_fwd, plus S1F_EINVAL if the workspace is too small, NULL or misaligned. */
int s1f_seg_attn_fwd_ws(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix,
                        int64_t seg_off, int64_t seg_len, void *out, float *lse, void *workspace,
                        size_t workspace_bytes, void *hip_stream);
/* Bytes s1f_seg_attn_fwd_ws needs for this call shape on the current device (0: none, or invalid arguments).  At most
 * 513 MiB.  The answer depends on the device's compute-unit count, so ask on the device that will run the call. */
size_t s1f_fwd_workspace_bytes(const s1f_desc *desc, int64_t seg_off, int64_t seg_len);

/* Backward of one segment (derivative of Eq. 3; order and accumulation per Sections 3.1-3.2).
 *
 *   dout, q_seg, out, lse : the segment's upstream gradient and the tensors saved by the forward
 *   dq        [batch, n_q_heads, seg_len, head_dim]  overwritten; complete after this call, since all
 *             keys a row of the segment can see are in the prefix
 *   dk_prefix_acc, dv_prefix_acc  fp32 [batch, n_kv_heads, kv_capacity, head_dim] (kv_* strides):
 *             rows [0, seg_off+seg_len) are updated with += (each element by exactly one workgroup, no
 *             atomics); rows beyond are not touched.  The caller zeroes them before the backward of the
 *             LAST segment and calls segments in reverse order; after the call for segment i, rows
 *             [seg_off, seg_off+seg_len) hold final gradients.
 *   workspace device scratch of at least s1f_bwd_workspace_bytes(desc, seg_off, seg_len) bytes
 *             (two fp32 values per query row and head: -lse/scale and -rowsum(dout * out), the row
 *             statistics the dK/dV kernel starts its products from; behind them up to 512 MiB of partial dQ
 *             rows when the dQ kernel cuts its last row tiles into chunks along the keys, as
 *             s1f_seg_attn_fwd_ws does); contents are undefined afterwards.
 * Errors as above, plus S1F_EINVAL if workspace is NULL or workspace_bytes is too small, and
 * S1F_EUNSUPPORTED if batch * n_q_heads * seg_len > 2^28 (the kernels' asynchronous copies use 32-bit byte
 * offsets inside the workspace). */
int s1f_seg_attn_bwd(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                     const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                     int64_t seg_len, void *dq, float *dk_prefix_acc, float *dv_prefix_acc,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/* The two halves of s1f_seg_attn_bwd as separate calls (same arguments, same validation), for callers
 * that schedule or time them separately; s1f_seg_attn_bwd is exactly _dq followed by _dkdv on one stream.
 *   s1f_seg_attn_bwd_dq    overwrites dq and writes the row statistics (-lse/scale, -rowsum(dout * out))
 *                          into workspace
 *   s1f_seg_attn_bwd_dkdv  reads the statistics left in workspace by _dq for the same segment (lse is
 *                          validated but not read) and updates dk_prefix_acc / dv_prefix_acc */
int s1f_seg_attn_bwd_dq(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                        const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                        int64_t seg_len, void *dq, void *workspace, size_t workspace_bytes, void *hip_stream);
int s1f_seg_attn_bwd_dkdv(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                          const void *v_prefix, const float *lse, int64_t seg_off, int64_t seg_len,
                          float *dk_prefix_acc, float *dv_prefix_acc, const void *workspace,
                          size_t workspace_bytes, void *hip_stream);

/* Bytes of device scratch s1f_seg_attn_bwd needs for this call shape on the current device (0 on invalid
 * arguments). */
size_t s1f_bwd_workspace_bytes(const s1f_desc *desc, int64_t seg_off, int64_t seg_len);

/* s1f_seg_attn_bwd for callers that cannot allocate device memory or pass a workspace: code under HIP graph
 * capture, tight serving or training loops, harnesses that forbid hipMalloc.  Same arguments (without the
 * workspace), same kernels; dK/dV bit-identical, dQ identical up to the rounding order of the key-split (the
 * built-in scratch leaves room for 32 MiB of partial dQ rows, s1f_seg_attn_bwd's workspace for 512 MiB, so the
 * two may cut a launch differently); the row statistics go to a device array built into the
 * library (48 MiB per GPU: 16 MiB of row statistics and 32 MiB for partial dQ rows; held until the process ends)
 * instead of a caller-owned workspace.  The call
 * allocates nothing and frees nothing.
 *   Limit: batch * n_q_heads * seg_len <= s1f_static_scratch_rows() (2^21); beyond it the call returns
 *   S1F_ESCRATCH before anything is launched.
 *   Every call on one GPU uses that GPU's one array: calls that overlap in time on the same GPU (different
 *   streams or threads) race; calls on one stream, or ordered by events, do not.  Nothing in the array has to
 *   start at zero and nothing in it is meaningful after the call.
 * The first call on a device looks up the array's device address (no allocation). */
int s1f_seg_attn_bwd_noalloc(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                             const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                             int64_t seg_len, void *dq, float *dk_prefix_acc, float *dv_prefix_acc,
                             void *hip_stream);
size_t s1f_static_scratch_rows(void);

/* The two data movements on either side of a segment's attention calls (Section 3.2: the keys and values of
 * all preceding tokens are retained; gradients of earlier tokens are accumulated until the backward passes
 * of all later segments have run).
 *
 * s1f_kv_append copies the segment's new rows k_seg, v_seg [batch, n_kv_heads, seg_len, head_dim] (strides
 * seg_stride_* in elements, head_dim contiguous) into rows [seg_off, seg_off + seg_len) of the caches k_cache,
 * v_cache (kv_* strides of desc), before s1f_seg_attn_fwd of that segment.
 * s1f_kv_grad_emit reads rows [seg_off, seg_off + seg_len) of the fp32 accumulators dk_prefix_acc,
 * dv_prefix_acc (kv_* strides) after s1f_seg_attn_bwd of that segment, when they are final, and writes them in
 * desc->dtype (bf16: round to nearest even) to dk_seg, dv_seg [batch, n_kv_heads, seg_len, head_dim]
 * (seg_stride_*).  n_q_heads, q_stride_* of desc are not used.
 * All pointers are device pointers, 16-byte aligned; all strides multiples of 8 elements; head_dim a multiple
 * of 8.  Errors: S1F_EINVAL (null/misaligned pointer, bad stride), S1F_EUNSUPPORTED (dtype, head_dim),
 * S1F_ERANGE (rows outside [0, kv_capacity)), S1F_EDEVICE. */
int s1f_kv_append(const s1f_desc *desc, const void *k_seg, const void *v_seg, int64_t seg_stride_b,
                  int64_t seg_stride_h, int64_t seg_stride_s, int64_t seg_off, int64_t seg_len, void *k_cache,
                  void *v_cache, void *hip_stream);
int s1f_kv_grad_emit(const s1f_desc *desc, const float *dk_prefix_acc, const float *dv_prefix_acc, int64_t seg_off,
                     int64_t seg_len, void *dk_seg, void *dv_seg, int64_t seg_stride_b, int64_t seg_stride_h,
                     int64_t seg_stride_s, void *hip_stream);

/* Order of passes of one pipeline device under the sequence-level 1F1B schedule (Section 3.2).  HOST
 * functions, no device work.
 *
 * pp_size = P devices, device = i in [1, P], n_micro = M micro-batches, n_seg = k segments per sequence.
 * s1f_seq1f1b_warmup writes the number of sub-sequences the device forwards before its first backward
 * pass, Eq. 4: P - i - 1 + k if M > P; otherwise every forward pass comes first (M * k sub-sequences: the
 * equation prints M, the micro-batch count of Eq. 1).  Never more than M * k.
 * s1f_seq1f1b_order writes the 2 * M * k passes in execution order into the caller-owned HOST array `order`
 * (capacity in elements) and their number into *n_passes (also when `order` is NULL or too small, which
 * returns S1F_EINVAL, so that a caller can size the array): the warm-up forward passes; then one forward
 * pass followed by one backward pass per step; then the remaining backward passes.  A backward pass takes
 * the tail segment of the earliest micro-batch that still has one (first-in-first-out over micro-batches,
 * last-in-first-out over the segments of a micro-batch), so for every micro-batch the calls of
 * s1f_seg_attn_fwd run for segments 0 .. k-1 and those of s1f_seg_attn_bwd for k-1 .. 0.
 * Errors: S1F_EINVAL for P < 1, i outside [1, P], M < 1, k < 1, M * k > 2^40 or a NULL result pointer. */
typedef struct {
  int32_t micro_batch; /* 0-based */
  int32_t segment;     /* 0-based */
  int32_t backward;    /* 0 = forward pass, 1 = backward pass */
} s1f_pass;
int s1f_seq1f1b_warmup(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, int64_t *warmup);
int s1f_seq1f1b_order(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, s1f_pass *order,
                      int64_t capacity, int64_t *n_passes);

/* Peak activation memory of one device (Section 3.1): with A the memory of all intermediate states of a batch,
 * device i holds A * w_i / sum_j w_j at its peak, w the warm-up counts (Eq. 1 for n_seg = 1, Eq. 4 otherwise).
 * Writes the exact fraction: *numerator = w_i, *denominator = sum over the P devices of w_j (not reduced).  HOST
 * function.  Errors: S1F_EINVAL as for s1f_seq1f1b_warmup, a NULL result pointer, or a zero sum (one device running
 * whole sequences has no warm-up phase; the formula is undefined there). */
int s1f_seq1f1b_peak_memory_share(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg,
                                  int64_t *numerator, int64_t *denominator);

/* Interleaved sequence-level schedule (Section 3.3): device i owns the n_chunks stages i, i + P, ..., and
 * switches to its next stage after P passes.  HOST functions, no device work.
 *
 * s1f_seq1f1b_interleaved_warmup writes Eq. 6, (P - i) * 2 + (n_chunks - 1) * P + k - 1 (Eq. 5 when k = 1), capped
 * at the device's M * k * n_chunks forward passes.
 * s1f_seq1f1b_interleaved_order writes the device's 2 * M * k * n_chunks passes (kind 0 or 1) in execution order,
 * sized and reported like s1f_seq1f1b_order.  The paper shows the order in a figure only; the reading built: the
 * M * k sub-sequences in forward order form groups of P; a group is forwarded through the device's first stage,
 * then its second, ...; backward passes take the groups in the same order, the stages from last to first, and
 * inside a group the tail segment of the earliest micro-batch first (Section 3.2's queue); warm-up forward passes,
 * then one forward and one backward per step, then the remaining backward passes.
 * Errors: S1F_EINVAL as for s1f_seq1f1b_order or n_chunks < 1; S1F_EUNSUPPORTED unless a group holds whole
 * micro-batches (k divides P) and P divides M * k.  That restriction belongs to this reading, not to the paper:
 * the text fixes the order only through a figure for k = 4 on P = 4 devices with two stages each, which the
 * reading reproduces; for other shapes the paper gives nothing to decide between the possible group layouts. */
typedef struct {
  int32_t kind;        /* 0 = forward pass, 1 = backward pass */
  int32_t micro_batch; /* 0-based */
  int32_t segment;     /* 0-based */
  int32_t chunk;       /* 0-based: which of the device's stages; its pipeline stage is chunk * P + i */
} s1f_stage_pass;
int s1f_seq1f1b_interleaved_warmup(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg,
                                   int32_t n_chunks, int64_t *warmup);
int s1f_seq1f1b_interleaved_order(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, int32_t n_chunks,
                                  s1f_stage_pass *order, int64_t capacity, int64_t *n_passes);

/* Timeline of a whole pipeline under these schedules: how long a batch takes, how busy each device is (the bubble
 * ratio is 1 - sum(busy) / (P * makespan)) and how many intermediate states it holds at its peak (Section 3.1:
 * warm-up, steady and cooling-down phases; Sections 3.2-3.3; Appendix A.1 for the split backward pass).  HOST
 * function; times are integers in any one unit.
 *
 * Every device walks its order (s1f_seq1f1b_order for n_chunks = 1, s1f_seq1f1b_interleaved_order otherwise;
 * n_seg = 1 gives 1F1B and 1F1B-I).  A pass starts when the device is free and its input has arrived: a forward
 * pass needs the sub-sequence forwarded by the previous stage, a backward pass needs it back-propagated by the next
 * stage (by its own forward pass on the last stage), plus t_comm when that stage is on another device.
 * split_weight_grad = 1: t_bwd is the input-gradient pass; each leaves a weight-gradient pass of t_wgrad pending,
 * and a device runs its oldest pending one whenever its next forward or backward pass still waits for its input or
 * more than max_pending_wgrad are waiting, the rest at the end (a reading: the appendix gives a figure only).
 * A sub-sequence's states count as held from its forward pass to its backward pass (to its weight-gradient pass
 * when split).
 * Results (caller-owned HOST memory): *makespan; busy[P]; peak_live[P] in units of seg_tokens (sub-sequences when
 * seg_tokens is NULL); peak_pending_wgrad[P] (may be NULL); *bubble_ratio = 1 - sum(busy) / (P * makespan), 0 for an
 * empty timeline (may be NULL).
 * Errors: S1F_EINVAL for null pointers, counts < 1, negative or > 2^36 times, reserved != 0, or
 * M * k * n_chunks * P > 2^24; S1F_EUNSUPPORTED where s1f_seq1f1b_interleaved_order returns it. */
typedef struct {
  int32_t pp_size, n_micro, n_seg, n_chunks;
  int32_t split_weight_grad; /* 0 or 1 */
  int32_t reserved;          /* must be 0 */
  int64_t max_pending_wgrad; /* >= 0; only read when split_weight_grad = 1 */
  int64_t t_comm;            /* >= 0 */
  const int64_t *t_fwd;      /* [n_seg] forward pass of segment j on one stage */
  const int64_t *t_bwd;      /* [n_seg] */
  const int64_t *t_wgrad;    /* [n_seg], or NULL when split_weight_grad = 0 */
  const int64_t *seg_tokens; /* [n_seg] weights of the held states, or NULL for 1 each */
} s1f_pipeline_desc;
int s1f_pipeline_simulate(const s1f_pipeline_desc *desc, int64_t *makespan, int64_t *busy, int64_t *peak_live,
                          int64_t *peak_pending_wgrad, double *bubble_ratio);

/* Static, NUL-terminated description of a status code. */
const char *s1f_strerror(int status);

/* Library version: major * 10000 + minor * 100 + patch. */
int s1f_version(void);

#ifdef __cplusplus
}
#endif
#endif /* S1F_H */
