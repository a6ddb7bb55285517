// C ABI of the library: argument validation, launch-shape decisions, workspace layout.
// Every entry point is declared and documented in include/flexdraft.h.
#include "fd_common.h"
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>
#include <atomic>

namespace fd {
hipError_t run_attn_generic(const AttnParams& p, int dtype, hipStream_t st);
hipError_t run_attn_combine(const AttnParams& p, int dtype, int log2_units, int skip_single, hipStream_t st);
bool attn_mfma_supports(int dtype, int head_dim, int page_size);
size_t draft_select_workspace_bytes(int total_rows, int vocab);
hipError_t run_draft_select(const void* logits, int dt, long long row_stride, int vocab, float temperature,
                            float threshold, const int* row_indptr, int batch, int total_rows, int max_rows,
                            int* tokens, float* confidence, int* keep_len, void* ws, hipStream_t st);
hipError_t run_append_kv(const AttnParams& p, int dtype, void* k_cache, void* v_cache, const int* accept_len,
                         int* kv_len_out, hipStream_t st);
hipError_t run_select_branch(const int* block_tokens, const int* block_indptr, const int* mask_blocks,
                             const int* accept_len, const int* first_vis, const int* verify_len, int batch,
                             int total_tokens, int out_stride, int* out_tokens, int* out_block, hipStream_t st);
int attn_mfma_tile_keys();
int attn_mfma_rows_per_wg(int max_tile_rows);
hipError_t run_attn_mfma_plan(const AttnParams& p, void* workspace, int kv_chunk, hipStream_t st);
hipError_t run_attn_mfma(const AttnParams& p, void* workspace, int kv_chunk, bool planned, hipStream_t st);
hipError_t run_attn_mfma_combine(const AttnParams& p, void* workspace, hipStream_t st);
int attn_mfma_num_wgs();
size_t attn_mfma_workspace(int num_wgs, int rows_wg, size_t* off_ml, size_t* off_entries, size_t* off_plan);
size_t accept_workspace_bytes(int batch, int total_rows, int vocab, int sampling);
hipError_t run_accept_greedy(const void* logits, int dt, long long row_stride, int vocab, const int* row_indptr,
                             const int* toks, int batch, int total_rows, int max_rows, int* accept_len,
                             int* bonus, int* row_argmax, void* ws, hipStream_t st);
hipError_t run_accept_sample(const void* target, const void* draft, int dt, long long row_stride, int vocab,
                             float temperature, const int* row_indptr, const int* toks, const float* ua,
                             const float* ur, int batch, int total_rows, int max_rows, int* accept_len,
                             int* bonus, void* ws, hipStream_t st);
}  // namespace fd

namespace {

// FD_STATIC_SCRATCH_BYTES (flexdraft.h) covers the MFMA kernel's workspace at 128 tile rows per
// work-group on up to 304 compute units (35.7 MB at 256).

thread_local char g_err[512] = "";

fd_status fail(fd_status code, const char* fmt, ...) {
  va_list ap; va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return code;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

struct AttnPlan {
  bool use_mfma;
  int chunk, max_chunks, row_tiles;
  size_t acc_bytes, ml_bytes, total_bytes;
};

// Host-only checks of the scalar fields and the launch-shape plan.
fd_status plan_attn(const fd_attn_args* a, AttnPlan* plan) {
  if (!a) return fail(FD_ERR_INVALID_ARG, "args is NULL");
  if (a->batch < 0 || a->total_rows < 0 || a->max_kv_len < 0 || a->max_new_rows < 0 || a->num_pages < 0)
    return fail(FD_ERR_INVALID_ARG, "negative size (batch %d, total_rows %d, max_kv_len %d, max_new_rows %d, num_pages %d)",
                a->batch, a->total_rows, a->max_kv_len, a->max_new_rows, a->num_pages);
  if (a->num_q_heads <= 0 || a->num_kv_heads <= 0 || a->num_q_heads % a->num_kv_heads)
    return fail(FD_ERR_INVALID_ARG, "num_q_heads %d must be a positive multiple of num_kv_heads %d", a->num_q_heads, a->num_kv_heads);
  if (a->head_dim <= 0 || a->head_dim % 8) return fail(FD_ERR_INVALID_ARG, "head_dim %d must be a positive multiple of 8", a->head_dim);
  if (a->head_dim > 128) return fail(FD_ERR_UNSUPPORTED, "head_dim %d > 128 has no kernel", a->head_dim);
  if (a->page_size <= 0) return fail(FD_ERR_INVALID_ARG, "page_size %d must be positive", a->page_size);
  if (a->dtype != FD_F32 && a->dtype != FD_BF16) return fail(FD_ERR_INVALID_ARG, "unknown dtype %d", a->dtype);
  if (!(a->sm_scale >= 0.f) || isinf(a->sm_scale)) return fail(FD_ERR_INVALID_ARG, "sm_scale must be finite and >= 0");
  if (a->kv_chunk < 0 || a->kv_chunk % 64) return fail(FD_ERR_INVALID_ARG, "kv_chunk %d must be a non-negative multiple of 64", a->kv_chunk);
  if (a->page_indices_len < 0) return fail(FD_ERR_INVALID_ARG, "page_indices_len %d is negative", a->page_indices_len);
  if (a->batch > 65535) return fail(FD_ERR_UNSUPPORTED, "batch %d > 65535", a->batch);
  if (a->max_kv_len > (1 << 30)) return fail(FD_ERR_UNSUPPORTED, "max_kv_len %d too large", a->max_kv_len);

  const int G = a->num_q_heads / a->num_kv_heads;
  plan->use_mfma = fd::attn_mfma_supports(a->dtype, a->head_dim, a->page_size) && !(a->flags & FD_ATTN_FORCE_GENERIC);
  const int tile_keys = plan->use_mfma ? fd::attn_mfma_tile_keys() : 64;
  if (a->kv_chunk % tile_keys) return fail(FD_ERR_INVALID_ARG, "kv_chunk %d must be a multiple of %d for this kernel", a->kv_chunk, tile_keys);
  long long rows = (long long)a->max_new_rows * G;
  const int tile_rows = plan->use_mfma ? fd::attn_mfma_rows_per_wg((int)(rows > 128 ? 128 : rows)) : 16;
  plan->row_tiles = (int)((rows + tile_rows - 1) / tile_rows);
  if (plan->row_tiles < 1) plan->row_tiles = 1;
  if ((long long)plan->row_tiles * a->num_kv_heads > 65535)
    return fail(FD_ERR_UNSUPPORTED, "max_new_rows * heads too large for one launch");
  if (plan->use_mfma) {
    // the persistent kernel counts (sequence, head, row block, 64-key tile) units in 32 bits
    const long long tiles = (long long)(a->max_kv_len + tile_keys - 1) / tile_keys + (a->max_new_rows + tile_keys - 1) / tile_keys + 4;   // + start-up units
    const double units = (double)(a->batch > 0 ? a->batch : 1) * a->num_kv_heads * plan->row_tiles * (double)tiles;
    if (units >= 2147483648.0) return fail(FD_ERR_UNSUPPORTED, "batch x heads x rows x kv length too large for one launch");
  }

  int chunk = a->kv_chunk;
  if (chunk == 0) {
    // enough (sequence, head, chunk) work-groups to cover 256 CUs x 2 several times over,
    // but never chunks so short that the split partials rival the KV traffic
    long long pairs = (long long)(a->batch > 0 ? a->batch : 1) * a->num_kv_heads * plan->row_tiles;
    long long want = (2048 + pairs - 1) / pairs;
    if (want < 1) want = 1;
    long long c = ((long long)a->max_kv_len + want - 1) / want;
    c = (c + tile_keys - 1) / tile_keys * tile_keys;
    long long floor_c = 512;
    if (c < floor_c) c = floor_c;
    chunk = (int)c;
  }
  plan->chunk = chunk;
  long long mc = ((long long)a->max_kv_len + chunk - 1) / chunk;
  if (mc < 1) mc = 1;
  if (mc > 65535) return fail(FD_ERR_UNSUPPORTED, "kv_chunk %d gives %lld chunks (> 65535)", chunk, mc);
  plan->max_chunks = (int)mc;
  if (plan->use_mfma) {
    // persistent kernel: partial storage depends on the launch size only, not on the lengths
    plan->max_chunks = 1;
    plan->acc_bytes = plan->ml_bytes = 0;
    plan->total_bytes = fd::attn_mfma_workspace(fd::attn_mfma_num_wgs(), tile_rows, nullptr, nullptr, nullptr);
    return FD_OK;
  }
  size_t slots = (size_t)plan->max_chunks * (size_t)(a->total_rows > 0 ? a->total_rows : 1) * a->num_q_heads;
  plan->acc_bytes = (slots * a->head_dim * sizeof(float) + 255) / 256 * 256;
  plan->ml_bytes = (slots * 2 * sizeof(float) + 255) / 256 * 256;
  plan->total_bytes = plan->acc_bytes + plan->ml_bytes;
  return FD_OK;
}


// ---- static scratch of fd_verify_draft_attn_static ---------------------------------------------
// The array lives in device memory of every GPU the library's code object is loaded on, from then
// until the process ends.  On the host its name is only a handle: the device address is asked for
// once per device (with that device current) and kept; only that address is ever handed to kernels.
__device__ __align__(256) unsigned char scratch[FD_STATIC_SCRATCH_BYTES];

constexpr int MAX_DEVICES = 64;
std::atomic<void*> g_scratch_ptr[MAX_DEVICES];

fd_status static_scratch(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES)
    return fail(FD_ERR_HIP, "hipGetDevice failed or device index %d not below %d", dev, MAX_DEVICES);
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess || !ptr) return fail(FD_ERR_HIP, "hipGetSymbolAddress(scratch): %s", hipGetErrorString(e));
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);       // every thread would store the same address
  }
  *out = ptr;
  return FD_OK;
}

}  // namespace

extern "C" {

const char* fd_last_error(void) { return g_err; }
const char* fd_version(void) { return "flexdraft-gfx950 0.2"; }

size_t fd_verify_draft_attn_workspace(const fd_attn_args* a) {
  AttnPlan plan;
  if (plan_attn(a, &plan) != FD_OK) return 0;
  return plan.total_bytes;
}

// The attention call on the given workspace (the caller's, or the library's static scratch).
// what: 1 = plan only, 2 = attention only (the workspace holds the plan), 3 = both.
enum { DO_PLAN = 1, DO_ATTN = 2 };
static fd_status attn_call(const fd_attn_args* a, void* workspace, size_t workspace_bytes, void* hip_stream, int what) {
  AttnPlan plan;
  fd_status st = plan_attn(a, &plan);
  if (st != FD_OK) return st;
  g_err[0] = 0;
  if (a->batch == 0 || a->total_rows == 0) return FD_OK;          // nothing to compute
  const bool attn = (what & DO_ATTN) != 0;         // planning reads the lengths and the page lists only
  if (!a->page_indptr || !a->kv_len || !a->row_indptr || !a->verify_len ||
      (attn && (!a->q || !a->k_new || !a->v_new || !a->out)))
    return fail(FD_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (a->max_kv_len > 0 && (!a->page_indices || a->num_pages == 0 || (attn && (!a->k_cache || !a->v_cache))))
    return fail(FD_ERR_INVALID_ARG, "max_kv_len > 0 needs k_cache, v_cache, page_indices and num_pages > 0");
  if (a->max_new_rows == 0) return fail(FD_ERR_INVALID_ARG, "total_rows > 0 but max_new_rows == 0");
  if (a->cache_stride_page < 0 || a->cache_stride_head < 0 || a->cache_stride_token < a->head_dim ||
      a->cache_stride_page % 8 || a->cache_stride_head % 8 || a->cache_stride_token % 8)
    return fail(FD_ERR_INVALID_ARG, "cache strides must be non-negative multiples of 8 elements, token stride >= head_dim");
  if (a->cache_stride_token > (1 << 24)) return fail(FD_ERR_UNSUPPORTED, "cache_stride_token above 2^24 elements");
  if (plan.use_mfma && (a->cache_stride_page >= (1ll << 31) || a->cache_stride_head >= (1ll << 31) ||
                        (long long)a->page_size * a->cache_stride_token >= (1ll << 31)))
    return fail(FD_ERR_UNSUPPORTED, "cache strides of 2^31 elements or more");
  if (!workspace) return fail(FD_ERR_INVALID_ARG, "workspace is NULL");
  if (workspace_bytes < plan.total_bytes)
    return fail(FD_ERR_WORKSPACE_TOO_SMALL, "workspace %zu bytes, need %zu", workspace_bytes, plan.total_bytes);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(FD_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  if (attn && (!aligned16(a->q) || !aligned16(a->k_new) || !aligned16(a->v_new) || !aligned16(a->out) ||
               !aligned16(a->k_cache) || !aligned16(a->v_cache)))
    return fail(FD_ERR_INVALID_ARG, "q, k_new, v_new, out, k_cache and v_cache must be 16-byte aligned");

  fd::AttnParams p;
  p.B = a->batch; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads; p.D = a->head_dim;
  p.G = p.Hq / p.Hkv; p.page_size = a->page_size;
  p.total_rows = a->total_rows; p.max_kv_len = a->max_kv_len; p.max_new_rows = a->max_new_rows;
  p.num_pages = a->num_pages; p.page_entries = a->page_indices_len; p.chunk = plan.chunk; p.max_chunks = plan.max_chunks; p.row_tiles = plan.row_tiles;
  p.sm_scale = a->sm_scale > 0.f ? a->sm_scale : 1.0f / sqrtf((float)a->head_dim);
  p.k_cache = a->k_cache; p.v_cache = a->v_cache;
  p.sp = a->cache_stride_page; p.sh = a->cache_stride_head; p.st = a->cache_stride_token;
  p.page_indptr = a->page_indptr; p.page_indices = a->page_indices; p.kv_len = a->kv_len;
  p.row_indptr = a->row_indptr; p.verify_len = a->verify_len; p.mask_vis = a->mask_vis;
  p.mask_blocks = a->mask_blocks;
  p.q = a->q; p.k_new = a->k_new; p.v_new = a->v_new; p.out = a->out; p.lse = a->lse;
  p.part_acc = reinterpret_cast<float*>(workspace);
  p.part_ml = reinterpret_cast<float*>(reinterpret_cast<char*>(workspace) + plan.acc_bytes);
  p.status = a->status;

  hipStream_t stream = reinterpret_cast<hipStream_t>(hip_stream);
  if (plan.use_mfma) {
    if ((what & DO_ATTN) && !(what & DO_PLAN) && a->page_indices_len <= 0 && a->max_kv_len > 0)
      return fail(FD_ERR_INVALID_ARG, "a planned call needs page_indices_len (the plan's page list is checked against it)");
    if (what == DO_PLAN) {
      hipError_t e = fd::run_attn_mfma_plan(p, workspace, a->kv_chunk, stream);
      if (e != hipSuccess) return fail(FD_ERR_HIP, "planning kernel launch: %s", hipGetErrorString(e));
      return FD_OK;
    }
    // without a plan the streaming kernel finds its shares itself: no extra launch
    hipError_t e = fd::run_attn_mfma(p, workspace, a->kv_chunk, what == DO_ATTN, stream);
    if (e != hipSuccess) return fail(FD_ERR_HIP, "attention kernel launch: %s", hipGetErrorString(e));
    e = fd::run_attn_mfma_combine(p, workspace, stream);
    if (e != hipSuccess) return fail(FD_ERR_HIP, "combine kernel launch: %s", hipGetErrorString(e));
    return FD_OK;
  }
  if (!(what & DO_ATTN)) return FD_OK;            // the fp32 kernel has nothing to plan
  hipError_t e = fd::run_attn_generic(p, a->dtype, stream);
  if (e != hipSuccess) return fail(FD_ERR_HIP, "attention kernel launch: %s", hipGetErrorString(e));
  e = fd::run_attn_combine(p, a->dtype, 0, 0, stream);
  if (e != hipSuccess) return fail(FD_ERR_HIP, "combine kernel launch: %s", hipGetErrorString(e));
  return FD_OK;
}

fd_status fd_verify_draft_attn(const fd_attn_args* a, void* hip_stream) {
  if (!a) return fail(FD_ERR_INVALID_ARG, "args is NULL");
  return attn_call(a, a->workspace, a->workspace_bytes, hip_stream,
                   (a->flags & FD_ATTN_PLANNED) ? DO_ATTN : (DO_PLAN | DO_ATTN));
}

fd_status fd_verify_draft_plan(const fd_attn_args* a, void* hip_stream) {
  if (!a) return fail(FD_ERR_INVALID_ARG, "args is NULL");
  return attn_call(a, a->workspace, a->workspace_bytes, hip_stream, DO_PLAN);
}

fd_status fd_verify_draft_attn_static(const fd_attn_args* a, void* hip_stream) {
  if (!a) return fail(FD_ERR_INVALID_ARG, "args is NULL");
  AttnPlan plan;
  fd_status st = plan_attn(a, &plan);
  if (st != FD_OK) return st;
  if (plan.total_bytes > FD_STATIC_SCRATCH_BYTES)
    return fail(FD_ERR_WORKSPACE_TOO_SMALL, "this call needs %zu bytes of scratch, the static buffer holds %zu: use "
                "fd_verify_draft_attn with a workspace of your own", plan.total_bytes, (size_t)FD_STATIC_SCRATCH_BYTES);
  void* ptr = nullptr;
  st = static_scratch(&ptr);
  if (st != FD_OK) return st;
  return attn_call(a, ptr, FD_STATIC_SCRATCH_BYTES, hip_stream, DO_PLAN | DO_ATTN);   // never from a plan
}

size_t fd_accept_workspace(int32_t batch, int32_t total_rows, int32_t vocab, int32_t sampling) {
  return fd::accept_workspace_bytes(batch, total_rows, vocab, sampling);
}

static fd_status check_accept_common(const void* logits, fd_dtype dt, int64_t row_stride, int32_t vocab,
                                     const int32_t* row_indptr, const int32_t* toks, int32_t batch,
                                     int32_t total_rows, int32_t max_rows, const int32_t* accept_len,
                                     const int32_t* bonus, const void* ws, size_t ws_bytes, int sampling) {
  if (batch < 0 || total_rows < 0 || max_rows < 0) return fail(FD_ERR_INVALID_ARG, "negative size");
  if (vocab <= 0) return fail(FD_ERR_INVALID_ARG, "vocab %d must be positive", vocab);
  if (row_stride < vocab) return fail(FD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)row_stride, vocab);
  if (dt != FD_F32 && dt != FD_BF16) return fail(FD_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  if (batch > 0 && (!row_indptr || !accept_len || !bonus)) return fail(FD_ERR_INVALID_ARG, "row_indptr / outputs NULL");
  if (total_rows > 0 && (!logits || !toks)) return fail(FD_ERR_INVALID_ARG, "logits / input_tokens NULL");
  if (total_rows > 65535) return fail(FD_ERR_UNSUPPORTED, "total_rows %d > 65535", total_rows);
  if (batch > 0 && total_rows > 0 && max_rows == 0) return fail(FD_ERR_INVALID_ARG, "total_rows > 0 but max_rows_per_seq == 0");
  size_t need = fd::accept_workspace_bytes(batch, total_rows, vocab, sampling);
  if (batch > 0) {
    if (!ws) return fail(FD_ERR_INVALID_ARG, "workspace is NULL");
    if (ws_bytes < need) return fail(FD_ERR_WORKSPACE_TOO_SMALL, "workspace %zu bytes, need %zu", ws_bytes, need);
    if (reinterpret_cast<uintptr_t>(ws) & 255) return fail(FD_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  }
  return FD_OK;
}

fd_status fd_accept_greedy(const void* target_logits, fd_dtype dt, int64_t row_stride, int32_t vocab,
                           const int32_t* row_indptr, const int32_t* input_tokens,
                           int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                           int32_t* accept_len, int32_t* bonus_token, int32_t* row_argmax,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  fd_status st = check_accept_common(target_logits, dt, row_stride, vocab, row_indptr, input_tokens, batch,
                                     total_rows, max_rows_per_seq, accept_len, bonus_token, workspace,
                                     workspace_bytes, 0);
  if (st != FD_OK) return st;
  g_err[0] = 0;
  if (batch == 0) return FD_OK;
  hipError_t e = fd::run_accept_greedy(target_logits, dt, row_stride, vocab, row_indptr, input_tokens, batch,
                                       total_rows, max_rows_per_seq, accept_len, bonus_token, row_argmax,
                                       workspace, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(FD_ERR_HIP, "greedy acceptance launch: %s", hipGetErrorString(e));
  return FD_OK;
}

fd_status fd_accept_sample(const void* target_logits, const void* draft_logits, fd_dtype dt,
                           int64_t row_stride, int32_t vocab, float temperature,
                           const int32_t* row_indptr, const int32_t* input_tokens,
                           const float* u_accept, const float* u_resample,
                           int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                           int32_t* accept_len, int32_t* bonus_token,
                           void* workspace, size_t workspace_bytes, void* hip_stream) {
  fd_status st = check_accept_common(target_logits, dt, row_stride, vocab, row_indptr, input_tokens, batch,
                                     total_rows, max_rows_per_seq, accept_len, bonus_token, workspace,
                                     workspace_bytes, 1);
  if (st != FD_OK) return st;
  if (!(temperature > 0.f) || isinf(temperature)) return fail(FD_ERR_INVALID_ARG, "temperature must be finite and > 0");
  if (total_rows > 0 && (!draft_logits || !u_accept || !u_resample))
    return fail(FD_ERR_INVALID_ARG, "draft_logits / uniforms NULL");
  g_err[0] = 0;
  if (batch == 0) return FD_OK;
  hipError_t e = fd::run_accept_sample(target_logits, draft_logits, dt, row_stride, vocab, temperature, row_indptr,
                                       input_tokens, u_accept, u_resample, batch, total_rows, max_rows_per_seq,
                                       accept_len, bonus_token, workspace, reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(FD_ERR_HIP, "sampling acceptance launch: %s", hipGetErrorString(e));
  return FD_OK;
}

size_t fd_draft_select_workspace(int32_t total_rows, int32_t vocab) {
  if (total_rows < 0 || vocab <= 0) return 0;
  return fd::draft_select_workspace_bytes(total_rows, vocab);
}

fd_status fd_draft_select(const void* draft_logits, fd_dtype dt, int64_t row_stride, int32_t vocab,
                          float temperature, float threshold, const int32_t* row_indptr,
                          int32_t batch, int32_t total_rows, int32_t max_rows_per_seq,
                          int32_t* draft_tokens, float* confidence, int32_t* keep_len,
                          void* workspace, size_t workspace_bytes, void* hip_stream) {
  if (batch < 0 || total_rows < 0 || max_rows_per_seq < 0) return fail(FD_ERR_INVALID_ARG, "negative size");
  if (vocab <= 0) return fail(FD_ERR_INVALID_ARG, "vocab %d must be positive", vocab);
  if (dt != FD_F32 && dt != FD_BF16) return fail(FD_ERR_INVALID_ARG, "unknown dtype %d", (int)dt);
  if (row_stride < vocab) return fail(FD_ERR_INVALID_ARG, "row_stride %lld < vocab %d", (long long)row_stride, vocab);
  if (!(temperature > 0.f) || isinf(temperature)) return fail(FD_ERR_INVALID_ARG, "temperature must be finite and > 0");
  if (isnan(threshold) || isinf(threshold)) return fail(FD_ERR_INVALID_ARG, "threshold must be finite");
  if (batch > 65535 || total_rows > 65535) return fail(FD_ERR_UNSUPPORTED, "batch %d / total_rows %d > 65535", batch, total_rows);
  g_err[0] = 0;
  if (batch == 0) return FD_OK;
  if (!row_indptr || !keep_len || (total_rows > 0 && (!draft_logits || !draft_tokens)))
    return fail(FD_ERR_INVALID_ARG, "a required device pointer is NULL");
  const size_t need = fd::draft_select_workspace_bytes(total_rows, vocab);
  if (!workspace) return fail(FD_ERR_INVALID_ARG, "workspace is NULL");
  if (workspace_bytes < need) return fail(FD_ERR_WORKSPACE_TOO_SMALL, "workspace %zu bytes, need %zu", workspace_bytes, need);
  if (reinterpret_cast<uintptr_t>(workspace) & 255) return fail(FD_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
  hipError_t e = fd::run_draft_select(draft_logits, dt, row_stride, vocab, temperature, threshold, row_indptr, batch,
                                      total_rows, max_rows_per_seq, draft_tokens, confidence, keep_len, workspace,
                                      reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(FD_ERR_HIP, "draft select launch: %s", hipGetErrorString(e));
  return FD_OK;
}

fd_status fd_append_kv(const fd_attn_args* a, void* k_cache, void* v_cache, const int32_t* accept_len,
                       int32_t* kv_len_out, void* hip_stream) {
  if (!a) return fail(FD_ERR_INVALID_ARG, "args is NULL");
  if (a->batch < 0 || a->total_rows < 0 || a->max_kv_len < 0 || a->max_new_rows < 0 || a->num_pages < 0)
    return fail(FD_ERR_INVALID_ARG, "negative size");
  if (a->num_kv_heads <= 0 || a->head_dim <= 0 || a->head_dim % 8) return fail(FD_ERR_INVALID_ARG, "head_dim %d / num_kv_heads %d", a->head_dim, a->num_kv_heads);
  if (a->page_size <= 0) return fail(FD_ERR_INVALID_ARG, "page_size %d must be positive", a->page_size);
  if (a->dtype != FD_F32 && a->dtype != FD_BF16) return fail(FD_ERR_INVALID_ARG, "unknown dtype %d", a->dtype);
  if (a->batch > 65535) return fail(FD_ERR_UNSUPPORTED, "batch %d > 65535", a->batch);
  g_err[0] = 0;
  if (a->batch == 0) return FD_OK;
  if (!accept_len || !kv_len_out || !a->kv_len || !a->row_indptr || !a->page_indptr || !a->verify_len)
    return fail(FD_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (a->total_rows == 0 || a->max_new_rows == 0) {
    // nothing to commit: the lengths are copied
    if (kv_len_out != a->kv_len &&
        hipMemcpyAsync(kv_len_out, a->kv_len, sizeof(int32_t) * a->batch, hipMemcpyDeviceToDevice,
                       reinterpret_cast<hipStream_t>(hip_stream)) != hipSuccess)
      return fail(FD_ERR_HIP, "length copy failed");
    return FD_OK;
  }
  if (!k_cache || !v_cache || !a->page_indices || !a->k_new || !a->v_new || a->num_pages == 0)
    return fail(FD_ERR_INVALID_ARG, "k_cache, v_cache, page_indices, k_new, v_new and num_pages > 0 are needed");
  if (a->cache_stride_page < 0 || a->cache_stride_head < 0 || a->cache_stride_token < a->head_dim ||
      a->cache_stride_page % 8 || a->cache_stride_head % 8 || a->cache_stride_token % 8)
    return fail(FD_ERR_INVALID_ARG, "cache strides must be non-negative multiples of 8 elements, token stride >= head_dim");
  if (!aligned16(a->k_new) || !aligned16(a->v_new) || !aligned16(k_cache) || !aligned16(v_cache))
    return fail(FD_ERR_INVALID_ARG, "k_new, v_new, k_cache and v_cache must be 16-byte aligned");
  if (a->max_new_rows > 65535) return fail(FD_ERR_UNSUPPORTED, "max_new_rows %d > 65535", a->max_new_rows);
  fd::AttnParams p = {};
  p.B = a->batch; p.Hq = a->num_q_heads; p.Hkv = a->num_kv_heads; p.D = a->head_dim;
  p.G = a->num_kv_heads > 0 && a->num_q_heads > 0 ? a->num_q_heads / a->num_kv_heads : 1;
  p.page_size = a->page_size;
  p.total_rows = a->total_rows; p.max_kv_len = a->max_kv_len; p.max_new_rows = a->max_new_rows;
  p.num_pages = a->num_pages; p.page_entries = a->page_indices_len < 0 ? 0 : a->page_indices_len;
  p.k_cache = k_cache; p.v_cache = v_cache;
  p.sp = a->cache_stride_page; p.sh = a->cache_stride_head; p.st = a->cache_stride_token;
  p.page_indptr = a->page_indptr; p.page_indices = a->page_indices; p.kv_len = a->kv_len;
  p.row_indptr = a->row_indptr; p.verify_len = a->verify_len; p.mask_vis = a->mask_vis;
  p.mask_blocks = a->mask_blocks;
  p.k_new = a->k_new; p.v_new = a->v_new;
  p.status = a->status;
  hipError_t e = fd::run_append_kv(p, a->dtype, k_cache, v_cache, accept_len, kv_len_out,
                                   reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(FD_ERR_HIP, "append launch: %s", hipGetErrorString(e));
  return FD_OK;
}

fd_status fd_select_branch(const int32_t* block_tokens, const int32_t* block_indptr, const int32_t* mask_blocks,
                           const int32_t* accept_len, const int32_t* first_vis, const int32_t* verify_len,
                           int32_t batch, int32_t total_tokens,
                           int32_t out_stride, int32_t* out_tokens, int32_t* out_block, void* hip_stream) {
  if (batch < 0 || total_tokens < 0 || out_stride < 0) return fail(FD_ERR_INVALID_ARG, "negative size");
  g_err[0] = 0;
  if (batch == 0) return FD_OK;
  if (!block_indptr || !mask_blocks || !accept_len || (!out_tokens && out_stride > 0) || (!block_tokens && total_tokens > 0))
    return fail(FD_ERR_INVALID_ARG, "a required device pointer is NULL");
  if (!first_vis && !verify_len)
    return fail(FD_ERR_INVALID_ARG, "first_vis is NULL: verify_len is needed for its default");
  hipError_t e = fd::run_select_branch(block_tokens, block_indptr, mask_blocks, accept_len, first_vis, verify_len, batch,
                                       total_tokens, out_stride, out_tokens, out_block,
                                       reinterpret_cast<hipStream_t>(hip_stream));
  if (e != hipSuccess) return fail(FD_ERR_HIP, "select_branch launch: %s", hipGetErrorString(e));
  return FD_OK;
}

}  // extern "C"
