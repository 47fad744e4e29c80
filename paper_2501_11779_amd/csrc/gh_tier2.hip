// C ABI of the Tier-2 attention step: host-side validation and kernel launches.
// Declarations and the contract of every entry point are in include/gh_tier2.h.
#include "gh_tier2.h"

#include "gh_append.hpp"
#include "gh_attn_mfma.hpp"
#include "gh_attn_valu.hpp"
#include "gh_common.hpp"
#include "gh_plan.hpp"
#include "gh_reduce.hpp"

#include <mutex>

// Partial records of gh_decode_attention_static: one copy per GPU the code object is loaded on.
// In host code this name is only a handle for hipGetSymbolAddress; the device address of each
// GPU's copy is looked up once per device (static_scratch_of) and that pointer is what the kernels get.
static __device__ __align__(256) unsigned char scratch[GH_STATIC_SCRATCH_BYTES];

namespace {

using namespace gh_plan;

// Instantiations of the balanced kernel: dtype x (token groups) x (one | two passes per wave) x
// (a wave per worker | a workgroup of four waves as one worker; the kernel also takes two, which
// was measured on groups of 17 to 32 head columns and is no faster than two passes per wave).
template <bool BF16, bool GROUPED, bool FUSED>
void launch_balanced_as(const gh::AttnArgs& a, int passes, int share, size_t lds, hipStream_t s) {
  const dim3 grid(share > 1 ? a.n_workers : a.n_workers / 4), block(share > 1 ? 64 * share : 256);
  if (passes == 1 && share == 1)
    hipLaunchKernelGGL((gh::attn_mfma_balanced_kernel<BF16, GROUPED, 1, 0, FUSED>), grid, block, lds, s, a);
  else if (passes == 2 && share == 1)
    hipLaunchKernelGGL((gh::attn_mfma_balanced_kernel<BF16, GROUPED, 2, 0, FUSED>), grid, block, lds, s, a);
  else if constexpr (!FUSED) {         // (the caller keeps the one-launch step off cooperative plans)
    if (passes == 1)
      hipLaunchKernelGGL((gh::attn_mfma_balanced_kernel<BF16, GROUPED, 1, 4, false>), grid, block, lds, s, a);
    else
      hipLaunchKernelGGL((gh::attn_mfma_balanced_kernel<BF16, GROUPED, 2, 4, false>), grid, block, lds, s, a);
  }
}
// fused: the one-launch step (never with token groups)
void launch_balanced(const gh::AttnArgs& a, bool bf16, bool grouped, bool fused, int passes,
                     int share, size_t lds, hipStream_t s) {
  if (fused) {
    if (bf16) launch_balanced_as<true, false, true>(a, passes, share, lds, s);
    else launch_balanced_as<false, false, true>(a, passes, share, lds, s);
  } else if (bf16 && grouped) launch_balanced_as<true, true, false>(a, passes, share, lds, s);
  else if (bf16) launch_balanced_as<true, false, false>(a, passes, share, lds, s);
  else if (grouped) launch_balanced_as<false, true, false>(a, passes, share, lds, s);
  else launch_balanced_as<false, false, false>(a, passes, share, lds, s);
}

template <bool BF16>
void launch_valu(const gh::AttnArgs& a, int per_pass, hipStream_t s) {
  const dim3 grid(a.n_items), block(256);
  switch (per_pass) {
    case 1: hipLaunchKernelGGL((gh::attn_valu_kernel<1, BF16>), grid, block, 0, s, a); break;
    case 2: hipLaunchKernelGGL((gh::attn_valu_kernel<2, BF16>), grid, block, 0, s, a); break;
    case 4: hipLaunchKernelGGL((gh::attn_valu_kernel<4, BF16>), grid, block, 0, s, a); break;
    default: hipLaunchKernelGGL((gh::attn_valu_kernel<8, BF16>), grid, block, 0, s, a); break;
  }
}

}  // namespace

extern "C" {

const char* gh_status_string(int32_t status) {
  switch (status) {
    case GH_OK: return "ok";
    case GH_ERR_NULL: return "a required pointer is null";
    case GH_ERR_SHAPE: return "inconsistent sizes, head counts, strides or chunk_rows";
    case GH_ERR_UNSUPPORTED: return "unsupported head_dim, dtype, kernel or alignment";
    case GH_ERR_WORKSPACE: return "workspace too small";
    case GH_ERR_CAPACITY: return "max_ctx_len exceeds slot_capacity";
    case GH_ERR_HIP: return "HIP launch failed";
    case GH_ERR_SCRATCH: return "problem needs more partial records than the library's static scratch holds";
    default: return "unknown status";
  }
}

int32_t gh_decode_chunk_rows(const gh_problem* p) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  return make_plan(p).chunk_rows;
}

int32_t gh_decode_num_chunks(const gh_problem* p) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  return make_plan(p).n_chunks;
}

int32_t gh_decode_split_plan(const gh_problem* p, gh_split_plan* out) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (!out) return GH_ERR_NULL;
  const Plan pl = make_plan(p);
  *out = gh_split_plan{};
  out->n_chunks = pl.n_chunks;
  if (pl.balanced) {
    out->balanced = 1;
    out->n_workers = pl.n_workers;
    out->min_share = pl.min_share;
    out->passes_per_strip = pl.passes_per_strip;
    out->strips_per_kv_head = pl.n_pass;
    out->waves_per_worker = pl.share;
    out->groups_per_launch = pl.launch_groups;
  }
  return GH_OK;
}

size_t gh_decode_workspace_bytes(const gh_problem* p) {
  if (check_problem(p) != GH_OK) return 0;
  return workspace_floats(p, make_plan(p)) * sizeof(float);
}

int32_t gh_kv_append(const gh_problem* p, void* k_cache, void* v_cache, const void* k_new,
                     const void* v_new, const int32_t* slot_id, const int32_t* pos,
                     int32_t* dev_status, void* hip_stream) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!k_cache || !v_cache || !k_new || !v_new || !slot_id || !pos) return GH_ERR_NULL;
  if (!aligned16(k_cache) || !aligned16(v_cache) || !aligned16(k_new) || !aligned16(v_new))
    return GH_ERR_UNSUPPORTED;
  gh::AppendArgs a;
  a.k_cache = static_cast<uint16_t*>(k_cache);
  a.v_cache = static_cast<uint16_t*>(v_cache);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.slot_id = slot_id;
  a.pos = pos;
  a.dev_status = dev_status;
  a.slot_stride = p->slot_stride;
  a.head_stride = p->head_stride;
  a.row_stride = p->row_stride;
  a.new_batch_stride =
      p->new_batch_stride ? p->new_batch_stride : (int64_t)p->n_kv_heads * p->head_dim;
  block_params(p, &a.block_stride, &a.block_shift, &a.block_mask);
  a.batch = p->batch;
  a.n_kv_heads = p->n_kv_heads;
  a.n_slots = p->n_slots;
  a.capacity = p->slot_capacity;
  const int64_t threads = (int64_t)p->batch * p->n_kv_heads * 32;
  const dim3 grid((unsigned)((threads + 255) / 256)), block(256);
  hipLaunchKernelGGL(gh::kv_append_kernel, grid, block, 0, static_cast<hipStream_t>(hip_stream), a);
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

}  // extern "C"

namespace {

// What the one-launch step adds to an attention launch (null k_new: an ordinary launch).
struct StepInputs {
  const void* k_new = nullptr;
  const void* v_new = nullptr;
  int32_t* dev_status = nullptr;
};

// A wave of the one-launch step covers at least this many tiles when the batch is small: fewer,
// longer pieces per strip keep the merge at its end short (it reads every piece's record).
constexpr int kStepMinShare = 8;

// out_kind: 0 = no early results, 1 = fp32, 2 = the problem's 16-bit type.  With `step` the array
// ctx_len holds the positions of the new rows.
int32_t launch_attention(const gh_problem* p, const void* q, const void* k_cache,
                         const void* v_cache, const int32_t* slot_id, const int32_t* ctx_len,
                         void* workspace, size_t workspace_bytes, void* out, int out_kind,
                         void* hip_stream, const StepInputs& step = StepInputs()) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!q || !k_cache || !v_cache || !slot_id || !ctx_len || !workspace) return GH_ERR_NULL;
  if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(workspace))
    return GH_ERR_UNSUPPORTED;
  const Plan pl = make_plan(p);
  if (tokens_per_group(p) > 1 && !pl.balanced) return GH_ERR_UNSUPPORTED;
  // the records of one (group, kv head) are addressed with 32-bit byte offsets from its first
  if ((int64_t)tokens_per_group(p) * p->n_q_heads * pl.n_chunks * gh::kHeadDim * 4 > 0x7fffffff)
    return GH_ERR_UNSUPPORTED;
  const size_t nrec = (size_t)p->batch * p->n_q_heads * pl.n_chunks;
  if (workspace_bytes < workspace_floats(p, pl) * sizeof(float)) return GH_ERR_WORKSPACE;
  const int64_t items = (int64_t)p->batch * p->n_kv_heads * pl.n_pass * pl.n_chunks;
  if (items > 0x7fffffff) return GH_ERR_SHAPE;

  gh::AttnArgs a;
  a.q = static_cast<const uint16_t*>(q);
  a.k_cache = static_cast<const uint16_t*>(k_cache);
  a.v_cache = static_cast<const uint16_t*>(v_cache);
  a.slot_id = slot_id;
  a.ctx_len = ctx_len;
  a.ws_o = static_cast<float*>(workspace);
  a.ws_m = a.ws_o + nrec * gh::kHeadDim;
  a.ws_l = a.ws_m + nrec;
  a.ws_n = reinterpret_cast<int32_t*>(a.ws_l + nrec);
  a.arrive = a.ws_n + (size_t)p->batch * p->n_q_heads;
  a.ctx_bias = step.k_new ? 1 : 0;
  a.k_new = static_cast<const uint16_t*>(step.k_new);
  a.v_new = static_cast<const uint16_t*>(step.v_new);
  a.new_batch_stride =
      p->new_batch_stride ? p->new_batch_stride : (int64_t)p->n_kv_heads * p->head_dim;
  a.dev_status = step.dev_status;
  a.slot_stride = p->slot_stride;
  a.head_stride = p->head_stride;
  a.row_stride = p->row_stride;
  a.q_batch_stride = p->q_batch_stride ? p->q_batch_stride : (int64_t)p->n_q_heads * p->head_dim;
  block_params(p, &a.block_stride, &a.block_shift, &a.block_mask);
  a.n_q_heads = p->n_q_heads;
  a.n_kv_heads = p->n_kv_heads;
  a.tokens = tokens_per_group(p);
  a.real_group = p->n_q_heads / p->n_kv_heads;
  a.group = a.real_group * a.tokens;
  a.n_slots = p->n_slots;
  a.row_limit = p->max_ctx_len < p->slot_capacity ? p->max_ctx_len : p->slot_capacity;
  a.chunk_rows = pl.chunk_rows;
  a.n_chunks = pl.n_chunks;
  a.heads_per_pass = pl.per_pass;
  a.n_pass = pl.n_pass;
  a.n_items = (int32_t)items;
  a.batch = p->batch / a.tokens;                 // groups
  a.n_workers = pl.n_workers;
  a.min_share = step.k_new && pl.min_share < kStepMinShare ? kStepMinShare : pl.min_share;
  a.share = pl.share;
  a.scale_log2e = p->scale * 1.44269504088896340736f;
  a.out = out;
  a.out_kind = out_kind == 0 ? 0 : out_kind == 1 ? 1 : p->dtype == GH_F16 ? 2 : 3;

  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = p->dtype == GH_BF16;
  if (pl.balanced) {
    // A batch of more groups than one launch takes goes in slices, each split on its own: every
    // per-entry array moves on by the slice's entries (the kernels index them from their bases).
    const int64_t groups = a.batch;
    const size_t esize = a.out_kind == 1 ? 4 : 2;
    for (int64_t g0 = 0; g0 < groups; g0 += pl.launch_groups) {
      gh::AttnArgs b = a;
      const int64_t e0 = g0 * a.tokens;                          // first batch entry of the slice
      b.batch = (int32_t)(groups - g0 < pl.launch_groups ? groups - g0 : pl.launch_groups);
      b.q = a.q + e0 * a.q_batch_stride;
      b.slot_id = a.slot_id + e0;
      b.ctx_len = a.ctx_len + e0;
      const int64_t h0 = e0 * p->n_q_heads;                      // first (entry, head) pair
      b.ws_o = a.ws_o + h0 * pl.n_chunks * gh::kHeadDim;
      b.ws_m = a.ws_m + h0 * pl.n_chunks;
      b.ws_l = a.ws_l + h0 * pl.n_chunks;
      b.ws_n = a.ws_n + h0;
      b.arrive = a.arrive + h0;
      if (a.k_new) {
        b.k_new = a.k_new + e0 * a.new_batch_stride;
        b.v_new = a.v_new + e0 * a.new_batch_stride;
      }
      if (a.out) b.out = static_cast<char*>(a.out) + h0 * gh::kHeadDim * esize;
      const size_t lds = (size_t)(3 * b.batch + 1) * sizeof(uint32_t);
      // (the one-launch step runs a wave per worker; with cooperative workers gh_decode_step
      // takes the three-kernel route, and this launch only reads positions instead of lengths)
      launch_balanced(b, bf16, a.tokens > 1, step.k_new != nullptr && pl.share == 1,
                      pl.passes_per_strip, pl.share, lds, s);
    }
  } else if (pl.kernel == GH_KERNEL_MFMA) {
    const dim3 grid(a.n_items), block(64);
    if (bf16)
      hipLaunchKernelGGL(gh::attn_mfma_kernel<true>, grid, block, 0, s, a);
    else
      hipLaunchKernelGGL(gh::attn_mfma_kernel<false>, grid, block, 0, s, a);
  } else {
    if (bf16)
      launch_valu<true>(a, pl.per_pass, s);
    else
      launch_valu<false>(a, pl.per_pass, s);
  }
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

// Device address of the current GPU's copy of `scratch`, looked up on the first call on that GPU
// and kept.  No allocation: the buffer is part of the loaded code object.
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

int32_t static_scratch_of(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return GH_ERR_HIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* found = nullptr;
    if (hipGetSymbolAddress(&found, HIP_SYMBOL(scratch)) != hipSuccess || !found) {
      (void)hipGetLastError();
      return GH_ERR_HIP;
    }
    g_scratch_ptr[dev] = found;
  }
  *ptr = g_scratch_ptr[dev];
  return GH_OK;
}

// The one-launch step with a workgroup per strip (small batches).  out_kind: 1 = fp32, 2 = 16-bit.
int32_t launch_strips(const gh_problem* p, const void* q, const void* k_new, const void* v_new,
                      void* k_cache, void* v_cache, const int32_t* slot_id, const int32_t* pos,
                      void* out, int out_kind, int32_t* dev_status, int waves, void* hip_stream) {
  gh::AttnArgs a = {};
  a.q = static_cast<const uint16_t*>(q);
  a.k_cache = static_cast<const uint16_t*>(k_cache);
  a.v_cache = static_cast<const uint16_t*>(v_cache);
  a.k_new = static_cast<const uint16_t*>(k_new);
  a.v_new = static_cast<const uint16_t*>(v_new);
  a.slot_id = slot_id;
  a.ctx_len = pos;
  a.ctx_bias = 1;
  a.dev_status = dev_status;
  a.slot_stride = p->slot_stride;
  a.head_stride = p->head_stride;
  a.row_stride = p->row_stride;
  a.q_batch_stride = p->q_batch_stride ? p->q_batch_stride : (int64_t)p->n_q_heads * p->head_dim;
  a.new_batch_stride =
      p->new_batch_stride ? p->new_batch_stride : (int64_t)p->n_kv_heads * p->head_dim;
  block_params(p, &a.block_stride, &a.block_shift, &a.block_mask);
  a.n_q_heads = p->n_q_heads;
  a.n_kv_heads = p->n_kv_heads;
  a.tokens = 1;
  a.real_group = a.group = p->n_q_heads / p->n_kv_heads;
  a.n_slots = p->n_slots;
  a.row_limit = p->max_ctx_len < p->slot_capacity ? p->max_ctx_len : p->slot_capacity;
  a.heads_per_pass = 16;
  a.n_pass = (a.group + 15) / 16;
  a.batch = p->batch;
  a.scale_log2e = p->scale * 1.44269504088896340736f;
  a.out = out;
  a.out_kind = out_kind == 1 ? 1 : p->dtype == GH_F16 ? 2 : 3;
  const dim3 grid((unsigned)((int64_t)p->batch * p->n_kv_heads * a.n_pass));
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  const bool bf16 = p->dtype == GH_BF16;
  if (waves == 8) {
    if (bf16) hipLaunchKernelGGL((gh::attn_mfma_strip_kernel<true, 8>), grid, dim3(512), 0, s, a);
    else hipLaunchKernelGGL((gh::attn_mfma_strip_kernel<false, 8>), grid, dim3(512), 0, s, a);
  } else {
    if (bf16) hipLaunchKernelGGL((gh::attn_mfma_strip_kernel<true, 4>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((gh::attn_mfma_strip_kernel<false, 4>), grid, dim3(256), 0, s, a);
  }
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

// out_kind: 0 = fp32, 1 = the problem's 16-bit type
int32_t launch_reduce(const gh_problem* p, const void* workspace, void* out, int out_kind,
                      void* hip_stream) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!workspace || !out) return GH_ERR_NULL;
  if (!aligned16(workspace) || !aligned16(out)) return GH_ERR_UNSUPPORTED;
  const Plan pl = make_plan(p);
  const size_t nrec = (size_t)p->batch * p->n_q_heads * pl.n_chunks;
  gh::ReduceArgs a;
  a.ws_o = static_cast<const float*>(workspace);
  a.ws_m = a.ws_o + nrec * gh::kHeadDim;
  a.ws_l = a.ws_m + nrec;
  a.ws_n = reinterpret_cast<const int32_t*>(a.ws_l + nrec);
  a.out = out;
  a.n_rows = (int64_t)p->batch * p->n_q_heads;
  a.n_chunks = pl.n_chunks;
  const dim3 grid((unsigned)((a.n_rows + 3) / 4)), block(256);
  hipStream_t s = static_cast<hipStream_t>(hip_stream);
  if (out_kind == 0)
    hipLaunchKernelGGL(gh::decode_reduce_kernel<0>, grid, block, 0, s, a);
  else if (p->dtype == GH_F16)
    hipLaunchKernelGGL(gh::decode_reduce_kernel<1>, grid, block, 0, s, a);
  else
    hipLaunchKernelGGL(gh::decode_reduce_kernel<2>, grid, block, 0, s, a);
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

}  // namespace

extern "C" {

int32_t gh_decode_attention(const gh_problem* p, const void* q, const void* k_cache,
                            const void* v_cache, const int32_t* slot_id, const int32_t* ctx_len,
                            void* workspace, size_t workspace_bytes, void* hip_stream) {
  return launch_attention(p, q, k_cache, v_cache, slot_id, ctx_len, workspace, workspace_bytes,
                          nullptr, 0, hip_stream);
}

int32_t gh_decode_attention_out(const gh_problem* p, const void* q, const void* k_cache,
                                const void* v_cache, const int32_t* slot_id, const int32_t* ctx_len,
                                void* workspace, size_t workspace_bytes, void* out,
                                int32_t out_kind, void* hip_stream) {
  if (out_kind != GH_OUT_F32 && out_kind != GH_OUT_NATIVE) return GH_ERR_UNSUPPORTED;
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!out) return GH_ERR_NULL;
  if (!aligned16(out)) return GH_ERR_UNSUPPORTED;
  // one row of `out` is addressed with 32-bit byte offsets from the first of its (group, kv head)
  if ((int64_t)tokens_per_group(p) * p->n_q_heads * gh::kHeadDim * 4 > 0x7fffffff)
    return GH_ERR_UNSUPPORTED;
  return launch_attention(p, q, k_cache, v_cache, slot_id, ctx_len, workspace, workspace_bytes,
                          out, out_kind == GH_OUT_F32 ? 1 : 2, hip_stream);
}

int32_t gh_decode_attention_static(const gh_problem* p, const void* q, const void* k_cache,
                                   const void* v_cache, const int32_t* slot_id,
                                   const int32_t* ctx_len, void* out, int32_t out_kind,
                                   void* hip_stream) {
  if (out_kind != GH_OUT_F32 && out_kind != GH_OUT_NATIVE) return GH_ERR_UNSUPPORTED;
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!q || !k_cache || !v_cache || !slot_id || !ctx_len || !out) return GH_ERR_NULL;
  const size_t need = workspace_floats(p, make_plan(p)) * sizeof(float);
  if (need > (size_t)GH_STATIC_SCRATCH_BYTES) return GH_ERR_SCRATCH;
  void* ws = nullptr;
  const int32_t sst = static_scratch_of(&ws);
  if (sst != GH_OK) return sst;
  const int32_t ast = gh_decode_attention_out(p, q, k_cache, v_cache, slot_id, ctx_len, ws, need,
                                              out, out_kind, hip_stream);
  if (ast != GH_OK) return ast;
  return launch_reduce(p, ws, out, out_kind == GH_OUT_F32 ? 0 : 1, hip_stream);
}

int32_t gh_decode_step_init(const gh_problem* p, void* workspace, size_t workspace_bytes,
                            void* hip_stream) {
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (p->batch == 0) return GH_OK;
  if (!workspace) return GH_ERR_NULL;
  if (!aligned16(workspace)) return GH_ERR_UNSUPPORTED;
  const Plan pl = make_plan(p);
  if (workspace_bytes < workspace_floats(p, pl) * sizeof(float)) return GH_ERR_WORKSPACE;
  const size_t rows = (size_t)p->batch * p->n_q_heads;
  int32_t* arrive = static_cast<int32_t*>(workspace) + rows * ((size_t)pl.n_chunks * (gh::kHeadDim + 2) + 1);
  hipLaunchKernelGGL(gh::zero_words_kernel, dim3((unsigned)((rows + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(hip_stream), arrive, (int64_t)rows);
  return hipGetLastError() == hipSuccess ? GH_OK : GH_ERR_HIP;
}

int32_t gh_decode_step(const gh_problem* p, const void* q, const void* k_new, const void* v_new,
                       void* k_cache, void* v_cache, const int32_t* slot_id, const int32_t* pos,
                       void* workspace, size_t workspace_bytes, void* out, int32_t out_kind,
                       int32_t* dev_status, void* hip_stream) {
  if (out_kind != GH_OUT_F32 && out_kind != GH_OUT_NATIVE) return GH_ERR_UNSUPPORTED;
  const int32_t st = check_problem(p);
  if (st != GH_OK) return st;
  if (tokens_per_group(p) > 1) return GH_ERR_UNSUPPORTED;
  if (p->batch == 0) return GH_OK;
  if (!q || !k_new || !v_new || !k_cache || !v_cache || !slot_id || !pos || !workspace || !out)
    return GH_ERR_NULL;
  if (!aligned16(k_new) || !aligned16(v_new) || !aligned16(out)) return GH_ERR_UNSUPPORTED;
  if ((int64_t)p->n_q_heads * gh::kHeadDim * 4 > 0x7fffffff) return GH_ERR_UNSUPPORTED;
  StepInputs step;
  step.k_new = k_new;
  step.v_new = v_new;
  step.dev_status = dev_status;
  const Plan pl = make_plan(p);
  // On request, a workgroup per strip, merged through LDS: for small batches whose contexts have
  // about the same length (measured at 2048 rows per context on 64 / 8 heads: 15-22% less step
  // time than the balanced split for 16 to 96 sequences, even at 128, behind it at 256; with
  // lengths between 256 and 4096 rows it is no faster than the three launches -- the longest
  // strips finish alone -- which is why it is not chosen automatically).
  if (p->kernel == GH_KERNEL_STRIPS && p->chunk_rows == 0)
    return launch_strips(p, q, k_new, v_new, k_cache, v_cache, slot_id, pos, out,
                         out_kind == GH_OUT_F32 ? 1 : 2, dev_status, 4, hip_stream);
  if (pl.balanced && pl.share == 1)
    return launch_attention(p, q, k_cache, v_cache, slot_id, pos, workspace, workspace_bytes, out,
                            out_kind == GH_OUT_F32 ? 1 : 2, hip_stream, step);
  // Fixed split, vector kernel, a batch beyond the balanced split or head groups so large that
  // workgroups work as one (more than 32 heads per kv head): the same result from the three
  // kernels, with the same rule for positions out of range.
  gh_problem bounded = *p;
  bounded.slot_capacity = p->max_ctx_len < p->slot_capacity ? p->max_ctx_len : p->slot_capacity;
  const int32_t ast = gh_kv_append(&bounded, k_cache, v_cache, k_new, v_new, slot_id, pos, dev_status,
                                   hip_stream);
  if (ast != GH_OK) return ast;
  StepInputs positions;                 // rows attended = position + 1; the rows are appended already
  positions.k_new = k_new;
  positions.v_new = v_new;
  const int32_t tst = launch_attention(p, q, k_cache, v_cache, slot_id, pos, workspace,
                                       workspace_bytes, nullptr, 0, hip_stream, positions);
  if (tst != GH_OK) return tst;
  return launch_reduce(p, workspace, out, out_kind == GH_OUT_F32 ? 0 : 1, hip_stream);
}

int32_t gh_decode_reduce(const gh_problem* p, const void* workspace, const int32_t* ctx_len,
                         float* out, void* hip_stream) {
  (void)ctx_len;
  return launch_reduce(p, workspace, out, 0, hip_stream);
}

int32_t gh_decode_reduce_native(const gh_problem* p, const void* workspace, const int32_t* ctx_len,
                                void* out16, void* hip_stream) {
  (void)ctx_len;
  return launch_reduce(p, workspace, out16, 1, hip_stream);
}

}  // extern "C"
