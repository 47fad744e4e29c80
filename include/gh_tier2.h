/*
 * gh_tier2.h -- C ABI of the Tier-2 attention step on one MI355X (gfx950).
 *
 * The step is stage F2(C_k, qkv) -> C_k, x'_k of a transformer layer (paper
 * Section 2.1): the new key/value row of each sequence is appended to that
 * sequence's context slot, then the sequence's query heads attend over the
 * slot (Appendix A, Table 5, rows "Q_i^T.K_i" and "A_i^T.V_i"; Section 4.3:
 * multi-head attention with grouped-query support, FP32 arithmetic).  A
 * sequence is addressed by a context-slot id and the position of its latest
 * token (Section 4.1.3).  Sequences of one batch have different lengths.
 *
 * Conventions
 *   - gh_problem is read on the host.  Every other pointer is a DEVICE
 *     pointer unless stated otherwise.  The library allocates and frees
 *     nothing: the caller owns caches, inputs, outputs, the workspace, the
 *     index arrays and the stream.
 *   - All calls are asynchronous on `hip_stream` (a hipStream_t, 0 = the
 *     null stream).  append -> attention -> reduce in stream order gives
 *     "append before attending".
 *   - 16-bit tensors (q, k_new, v_new, caches) share one dtype (gh_dtype).
 *     Their base addresses and all three cache strides must be multiples of
 *     16 bytes (8 elements).
 *   - Cache element (slot s, kv head g, row r, column j) lives at index
 *     s*slot_stride + g*head_stride + r*row_stride + j (in elements); the
 *     `head_dim` elements of one row are contiguous.  K and V are separate
 *     allocations with the same geometry.
 *   - Blocked layout (block_rows > 0): row r of a head lives at
 *     (r / block_rows)*block_stride + (r % block_rows)*row_stride instead of
 *     r*row_stride.  It describes pages that hold block_rows consecutive rows of
 *     every kv head with each head's rows together ([slot][page][head][row][d]),
 *     which keeps a head's rows contiguous inside a page.
 *   - Query head h reads kv head h / (n_q_heads / n_kv_heads).
 *   - A cache that holds several layers (a Tier-1 node hosts a range of
 *     layers, Section 4.1.2) is addressed by passing the layer's base pointer:
 *     slots are then indexed by (layer, sequence) with no other change.
 *   - Host-checkable mistakes return a negative gh_status and launch
 *     nothing.  Conditions only visible on the device (slot id or position
 *     out of range) make the kernel skip that sequence and OR a bit into
 *     *dev_status when that pointer is non-null.  Nothing aborts or prints.
 *   - Caller guarantees (undefined otherwise): (slot id, position) pairs are
 *     unique within a batch, buffers do not alias, ctx_len[b] <= max_ctx_len.
 *   - Mixed prefill/decode batches (Appendix D): a batch entry is a token, and
 *     several entries may address the same slot with consecutive positions --
 *     the tokens of a prefill chunk of one prompt.  Each entry attends over
 *     rows [0, ctx_len) of its slot; since the append of the whole batch runs
 *     first, entry t of a chunk sees the chunk's earlier tokens and not the
 *     later ones: causal attention, with no other provision.
 *   - Token groups (tokens_per_group = T > 1): an optional declaration that
 *     lets the tokens of a prefill chunk share one pass over their slot.  Batch
 *     rows kT .. kT+T-1 form group k and address one slot; each row keeps its
 *     own ctx_len (and q, position, output row).  gh_decode_attention then
 *     fetches the slot's K/V rows from memory once per 128 of the T*G query
 *     heads a group has per kv head -- a wave carries 16 or 32 of them as the
 *     head columns of one or two matrix-core tiles fed from one stream of rows;
 *     beyond 32 the four waves of a workgroup stream the rows once between them
 *     (through LDS); each column is masked at its own token's length --
 *     instead of once per row.  A
 *     row with ctx_len 0, a bad slot id, or a slot other than that of the
 *     group's first live row gets no rows (output zero), so short groups are
 *     padded with ctx_len = 0 rows and a decode entry is a group with one live
 *     row.  Results are those of the undeclared batch up to fp32 rounding
 *     order.  gh_kv_append and the merge are unaffected (they work per row).
 *     Requires the matrix-core kernel with the library's split (chunk_rows =
 *     0); anything else returns GH_ERR_UNSUPPORTED.
 */
#ifndef GH_TIER2_H
#define GH_TIER2_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  GH_OK = 0,
  GH_ERR_NULL = -1,        /* a required pointer is null                        */
  GH_ERR_SHAPE = -2,       /* negative sizes, H % H_kv != 0, bad strides        */
  GH_ERR_UNSUPPORTED = -3, /* head_dim != 128, unknown dtype/kernel, alignment  */
  GH_ERR_WORKSPACE = -4,   /* workspace smaller than gh_decode_workspace_bytes  */
  GH_ERR_CAPACITY = -5,    /* max_ctx_len > slot_capacity                       */
  GH_ERR_HIP = -6,         /* the HIP runtime refused the launch                */
  GH_ERR_SCRATCH = -7      /* the problem needs more than GH_STATIC_SCRATCH_BYTES  */
} gh_status;

typedef enum { GH_F16 = 0, GH_BF16 = 1 } gh_dtype;

/* Which attention kernel gh_decode_attention launches. */
typedef enum {
  GH_KERNEL_AUTO = 0, /* the library's measured choice (currently always MFMA)   */
  GH_KERNEL_VALU = 1, /* fp32 vector arithmetic, passes of up to 8 heads          */
  GH_KERNEL_MFMA = 2, /* matrix-core tiles, passes of up to 16 heads, two at once  */
  GH_KERNEL_STRIPS = 3 /* gh_decode_step only (elsewhere: GH_KERNEL_AUTO): the same
                          tiles with one workgroup per (sequence, kv head) strip,
                          its four waves merged on chip -- no workspace traffic, no
                          partial records.  For batches of up to about a hundred
                          sequences whose contexts have about the same length (the
                          regime Appendix C profiles the attention in); with very
                          uneven lengths the longest strips finish alone and the
                          library's equal shares are the better split.           */
} gh_kernel;

/* Bits OR-ed into *dev_status by gh_kv_append. */
enum { GH_DEV_BAD_SLOT = 1, GH_DEV_BAD_POS = 2 };

typedef struct {
  int32_t batch;         /* B >= 0; 0 is a no-op returning GH_OK                 */
  int32_t n_q_heads;     /* H                                                    */
  int32_t n_kv_heads;    /* H_kv, divides H                                      */
  int32_t head_dim;      /* 128 (anything else: GH_ERR_UNSUPPORTED)              */
  int32_t dtype;         /* gh_dtype                                             */
  int32_t n_slots;       /* slots in each cache                                  */
  int32_t slot_capacity; /* rows per slot                                        */
  int32_t max_ctx_len;   /* host-known upper bound of ctx_len[]; sizes the grid  */
  int64_t slot_stride;   /* cache strides in elements, see above                 */
  int64_t head_stride;
  int64_t row_stride;
  float scale;           /* softmax scaling of the scores, e.g. 1/sqrt(head_dim) */
  int32_t chunk_rows;    /* > 0: fixed split, rows per context chunk, a multiple
                            of 64.  0: the library splits (see below).           */
  int32_t kernel;        /* gh_kernel                                            */
  int64_t q_batch_stride;   /* elements between the query rows of consecutive
                               sequences; 0 = contiguous [B, H, d] (H*d)          */
  int64_t new_batch_stride; /* the same for k_new and v_new; 0 = contiguous
                               [B, H_kv, d] (H_kv*d).  Multiples of 8.  With both
                               set to (H + 2*H_kv)*d the three inputs can be read
                               straight out of one packed per-sequence message
                               q | k | v (Section 5.4.3: what Tier 1 sends).      */
  int32_t block_rows;       /* 0, or a power of two >= 32: blocked cache layout   */
  int32_t tokens_per_group; /* T; 0 or 1: none.  T > 1 declares that batch rows
                               kT .. kT+T-1 address one slot (see above); batch
                               must be a multiple of T                            */
  int64_t block_stride;     /* elements between consecutive blocks of one head    */
} gh_problem;

/* Static text for a status code (host pointer, never null). */
const char* gh_status_string(int32_t status);

/*
 * Pure host functions: the split of the context (footnote of Section 2.2:
 * attention parallelised along the sequence).
 *
 * Fixed split (chunk_rows > 0, and always for GH_KERNEL_VALU, where 0 lets the
 * library pick the chunk size): record c of a head covers rows
 * [c*chunk_rows, (c+1)*chunk_rows) of its sequence.
 * Balanced split (chunk_rows == 0 with the MFMA kernel): the rows of the whole
 * batch -- of each slice of 4096 sequences, if it has more -- are cut into
 * equal shares, one per resident wave;
 * the non-empty records of a head cover consecutive row ranges that partition
 * [0, ctx_len) but whose borders depend on the other sequences' lengths.
 *
 *   gh_decode_chunk_rows  rows per chunk of the fixed split, 0 for the
 *                         balanced split; < 0 = gh_status.
 *   gh_decode_num_chunks  C = partial records per (sequence, head), >= 1;
 *                         < 0 = gh_status.
 *   gh_decode_workspace_bytes  bytes of workspace the two decode calls need
 *                         (0 if the problem is invalid or batch == 0).
 *
 * Workspace layout (base 16-byte aligned), with d = head_dim:
 *   float o[B][H][C][d], float m[B][H][C], float l[B][H][C], int32 n[B][H],
 *   int32 arrive[B][H] (gh_decode_step only)
 * n = how many of a head's C records are in use (records at index >= n are
 * unspecified and ignored by the merge); -1 = the head's result is already in
 * the output (gh_decode_attention_out).
 * For record c of (sequence b, head h), over the rows r it covers and with
 * t_r = scale * log2(e) * (q . K_r):
 *   l = sum_r 2^(t_r - m),  o[:] = sum_r 2^(t_r - m) * V_r[:]
 * where m is the exponent the sums are scaled by: max_r t_r - 8 <= m <= max_r t_r
 * (the matrix-core kernel lets it trail the running maximum by up to 2^8 to save
 * rescaling; any m in that range describes the same partial result, and the
 * merge only uses m as that common factor).
 * A record in use that covers no rows has m = -inf, l = 0, unspecified o.
 */
int32_t gh_decode_chunk_rows(const gh_problem* p);
int32_t gh_decode_num_chunks(const gh_problem* p);
size_t gh_decode_workspace_bytes(const gh_problem* p);

/*
 * The numbers behind the balanced split -- how the library parallelises the
 * attention along the sequence (footnote of Section 2.2) when the lengths of a
 * batch differ (Section 5.1: prompts of a batch have different lengths) -- for
 * callers and tests that want to reason about it (host function).  Every strip -- (group, kv head, set of
 * passes_per_strip * waves_per_worker passes of 16 head columns) -- counts ceil(rows / 32) tiles of
 * 32 rows, at least one; the strips are laid end to end in batch order, kv head
 * next, pass set fastest; worker w of n_workers takes tiles [w*share, (w+1)*share)
 * with share = max(ceil(total / n_workers), min_share); the record a wave
 * writes for a strip has index w - floor(first tile of the strip / share).
 * min_share is what keeps that index below gh_decode_num_chunks for every
 * batch whose lengths respect max_ctx_len.
 */
typedef struct {
  int32_t balanced;           /* 0: fixed split, the other fields are 0          */
  int32_t n_workers;          /* workers (waves, or workgroups of four waves)    */
  int32_t min_share;          /* least tiles per worker                          */
  int32_t passes_per_strip;   /* 1 or 2                                          */
  int32_t strips_per_kv_head; /* pass sets per (group, kv head)                  */
  int32_t n_chunks;           /* = gh_decode_num_chunks                          */
  int32_t waves_per_worker;   /* 1 or 4: the waves of a worker walk the same
                                 tiles, each with its own passes_per_strip passes
                                 (a strip then stands for their product of passes) */
  int32_t groups_per_launch;  /* a batch of more groups is launched in slices of
                                 this many (4096), each split as described, on
                                 its own                                          */
} gh_split_plan;
int32_t gh_decode_split_plan(const gh_problem* p, gh_split_plan* out);

/*
 * Append (the C_k update of F2).  For each sequence b and kv head g, copies
 * the head_dim elements k_new[b][g][:] / v_new[b][g][:] ([B, H_kv, d],
 * contiguous) to row pos[b] of slot slot_id[b] of k_cache / v_cache.  A bit
 * copy: no arithmetic touches the data.  Only those rows are written.
 * slot_id, pos: int32 [B].  dev_status: int32 on the device, may be null; the
 * caller clears it.  Sequences with slot_id outside [0, n_slots) or pos
 * outside [0, slot_capacity) are skipped and flagged there.
 */
int32_t gh_kv_append(const gh_problem* p, void* k_cache, void* v_cache,
                     const void* k_new, const void* v_new,
                     const int32_t* slot_id, const int32_t* pos,
                     int32_t* dev_status, void* hip_stream);

/*
 * Split-context attention (Table 5's Q.K and A.V, fused, softmax kept as a
 * running max and sum in fp32).  q: [B, H, d] contiguous.  ctx_len[b] = rows
 * attended for sequence b (pos[b] + 1 after an append); rows at or beyond it
 * are never read.  Writes n for every head, (m, l) of every record in use and
 * the o of every non-empty one.  A sequence with ctx_len <= 0 or a slot id out of range
 * produces only empty chunks.  ctx_len above min(max_ctx_len, slot_capacity)
 * is clamped to it.
 */
int32_t gh_decode_attention(const gh_problem* p, const void* q,
                            const void* k_cache, const void* v_cache,
                            const int32_t* slot_id, const int32_t* ctx_len,
                            void* workspace, size_t workspace_bytes,
                            void* hip_stream);

/*
 * gh_decode_attention that also finishes what it can (footnote of Section 2.2:
 * the split along the sequence is an option of the attention, not a need -- a
 * context that is not split has no partial results to merge, and its attention
 * is Table 5's Q.K, softmax, A.V as they stand).  A head whose rows one
 * wave covers alone (most heads of a large batch) has nothing to merge: its
 * result is normalised and stored straight into `out`, and its record count in
 * the workspace is set to -1, which makes the merges below leave that row of
 * `out` alone.  out_kind GH_OUT_F32: out is fp32 [B, H, d]; GH_OUT_NATIVE: the
 * model's 16-bit type, rounded as by gh_decode_reduce_native.  Call the
 * matching merge afterwards with the same `out` to complete the other heads;
 * the pair gives bit for bit what gh_decode_attention and the merge give.  With
 * a fixed split or the vector kernel no head is finished early and the call is
 * gh_decode_attention.  out: 16-byte aligned.
 */
typedef enum { GH_OUT_F32 = 0, GH_OUT_NATIVE = 1 } gh_out_kind;
int32_t gh_decode_attention_out(const gh_problem* p, const void* q,
                                const void* k_cache, const void* v_cache,
                                const int32_t* slot_id, const int32_t* ctx_len,
                                void* workspace, size_t workspace_bytes,
                                void* out, int32_t out_kind, void* hip_stream);

/*
 * Merge of the chunk partials (same footnote).  Per (b, h), over the records
 * in use with l > 0:  M = max_c m_c,
 *   out[b][h][:] = sum_c 2^(m_c - M) * o_c[:] / sum_c 2^(m_c - M) * l_c
 * and zeros when every chunk is empty.  out: fp32 [B, H, d] contiguous.
 * Deterministic: fixed summation order, no atomics.  ctx_len may be null (it
 * is not needed: empty chunks are recognised by l == 0).
 */
int32_t gh_decode_reduce(const gh_problem* p, const void* workspace,
                         const int32_t* ctx_len, float* out, void* hip_stream);

/*
 * The same merge with the result stored in the model's 16-bit type (p->dtype),
 * as the paper's kernels store it (Section 4.3) and as Tier 2 sends it back
 * (2*D bytes per token, Section 5.4.3).  out16: [B, H, d] contiguous, 16-byte
 * aligned.  The fp32 result is rounded to nearest even once, at the store.
 */
int32_t gh_decode_reduce_native(const gh_problem* p, const void* workspace,
                                const int32_t* ctx_len, void* out16, void* hip_stream);

/*
 * The whole stage F2(C_k, qkv) -> C_k, x'_k of Section 2.1 in ONE launch, for a
 * batch of one token per slot (plain decode): append, attention and merge.  It
 * computes what gh_kv_append + gh_decode_attention(ctx_len = pos + 1) +
 * gh_decode_reduce / gh_decode_reduce_native compute -- the appended rows bit
 * for bit, the result up to fp32 rounding order -- without the two extra
 * launches, which at the batch sizes of a Tier-2 node (tens of prompts,
 * Section 5.2 / Table 2) cost as much as the attention itself.
 *   - pos[b]: position of sequence b's new row; rows [0, pos[b]] are attended.
 *     The wave that reaches the end of a context reads the new row from k_new /
 *     v_new (never from the cache) and writes it to row pos[b] of the slot.
 *   - Slot ids must be UNIQUE within the batch (no prefill chunks here: a
 *     token's row would be appended while another token's wave reads the slot),
 *     and tokens_per_group must be 0 or 1 (GH_ERR_UNSUPPORTED).
 *   - A slot id outside [0, n_slots) or a position outside
 *     [0, min(slot_capacity, max_ctx_len)) skips the sequence: nothing is
 *     appended, its result is zero, and GH_DEV_BAD_SLOT / GH_DEV_BAD_POS is OR-ed
 *     into *dev_status when that is non-null (the caller clears it).
 *   - workspace: gh_decode_workspace_bytes(p) bytes.  Its arrival counters (one
 *     word per context strip; the wave that delivers the last partial record of
 *     a context merges them) must be zero when a launch begins: call
 *     gh_decode_step_init once on a fresh workspace; every gh_decode_step leaves
 *     them zero again.  Two steps that overlap in time need two workspaces.
 *   - out / out_kind as for gh_decode_attention_out; every row of `out` is
 *     written.  Deterministic for given inputs (fixed summation order).
 *   - With a fixed split (chunk_rows > 0), GH_KERNEL_VALU or more than 32 query
 *     heads per kv head the call issues the three kernels instead, same result.
 *     A batch of more than 4096 sequences is issued in slices of 4096.
 *   - kernel = GH_KERNEL_STRIPS (with chunk_rows = 0): one workgroup per strip,
 *     see gh_kernel; the workspace is then not touched.
 */
int32_t gh_decode_step_init(const gh_problem* p, void* workspace, size_t workspace_bytes,
                            void* hip_stream);
int32_t gh_decode_step(const gh_problem* p, const void* q, const void* k_new, const void* v_new,
                       void* k_cache, void* v_cache, const int32_t* slot_id, const int32_t* pos,
                       void* workspace, size_t workspace_bytes, void* out, int32_t out_kind,
                       int32_t* dev_status, void* hip_stream);

/*
 * For callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * gh_decode_attention_out followed by the matching merge, with the partial
 * records kept in a buffer that lives inside the library's code object instead of
 * a caller's workspace: GH_STATIC_SCRATCH_BYTES of device memory per GPU the
 * library runs on, held until the process ends.  Calls nothing that allocates.
 * `out` and `out_kind` as for gh_decode_attention_out; the result is bit for bit
 * that of gh_decode_attention_out + gh_decode_reduce / gh_decode_reduce_native.
 * A problem whose gh_decode_workspace_bytes exceeds GH_STATIC_SCRATCH_BYTES
 * returns GH_ERR_SCRATCH and launches nothing.  The first call on a device looks
 * up that device's copy of the buffer (a failure there is GH_ERR_HIP).  Every call
 * on one GPU shares that GPU's buffer, on whatever stream: calls that overlap in
 * time on one GPU race and give wrong results; calls ordered by a stream or by
 * events are fine.  Nothing in the buffer has to start at zero -- every word a
 * merge reads has been written by the attention kernel of the same call -- so
 * what an earlier, larger call left behind is harmless.
 */
#define GH_STATIC_SCRATCH_BYTES (64u << 20)
int32_t gh_decode_attention_static(const gh_problem* p, const void* q,
                                   const void* k_cache, const void* v_cache,
                                   const int32_t* slot_id, const int32_t* ctx_len,
                                   void* out, int32_t out_kind, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* GH_TIER2_H */
