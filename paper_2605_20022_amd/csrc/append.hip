// Commit of verified rows to the paged KV cache (Sec. 4.3, decoupled execution: the cache
// written by target verification is what the next draft step reuses).
//
// grid (row j of the sequence, sequence): the work-group copies new row j's K and V, all KV
// heads, to logical position kv_len + j if j <= accept_len.  Only verify rows are ever written:
// mask tokens stay invisible to the clean prefix (Sec. 4.1), so a sequence without verify rows
// commits nothing and accept_len is held below the number of verify rows.  The lengths are
// updated by a second, tiny kernel so that the output array may be the input array.
#include "fd_common.h"

namespace fd {

template <typename T>
__global__ __launch_bounds__(256) void append_kv_kernel(AttnParams p, T* __restrict__ k_cache, T* __restrict__ v_cache,
                                                        const int* __restrict__ accept_len) {
  const int j = blockIdx.x, seq = blockIdx.y;
  const SeqInfo s = load_seq(p, seq);                         // clamps and reports bad lengths
  if (s.k <= 0) return;
  int acc = sload(accept_len, seq);
  if (acc < 0 || acc >= s.k) { if (j == 0 && threadIdx.x == 0) flag_status(p.status, FD_DEV_ROWS_RANGE); acc = clampi(acc, 0, s.k - 1); }
  if (j > acc) return;
  // kv_len is the length BEFORE the commit; load_seq checked that the page list covers it, the rows
  // added here need their own check
  const int pos = s.L + j;
  const int lp = pos / p.page_size, slot = pos - lp * p.page_size;
  if (lp >= s.npages) { if (threadIdx.x == 0) flag_status(p.status, FD_DEV_PAGE_RANGE); return; }
  const int phys = sload(p.page_indices, s.page0 + lp);
  if (phys < 0 || phys >= p.num_pages) { if (threadIdx.x == 0) flag_status(p.status, FD_DEV_PAGE_RANGE); return; }
  constexpr int VEC = 16 / sizeof(T);                          // elements per 16-byte vector
  const int vec_per_head = p.D / VEC;                          // head_dim is a multiple of 8
  const int nvec = p.Hkv * vec_per_head;
  const T* kn = reinterpret_cast<const T*>(p.k_new) + (long long)(s.row0 + j) * p.Hkv * p.D;
  const T* vn = reinterpret_cast<const T*>(p.v_new) + (long long)(s.row0 + j) * p.Hkv * p.D;
  T* kc = k_cache + (long long)phys * p.sp + (long long)slot * p.st;
  T* vc = v_cache + (long long)phys * p.sp + (long long)slot * p.st;
  for (int i = threadIdx.x; i < 2 * nvec; i += 256) {
    const bool is_v = i >= nvec;
    const int iv = is_v ? i - nvec : i;
    const int h = iv / vec_per_head, e = (iv - h * vec_per_head) * VEC;
    const u32x4 val = *reinterpret_cast<const u32x4*>((is_v ? vn : kn) + h * p.D + e);
    *reinterpret_cast<u32x4*>((is_v ? vc : kc) + (long long)h * p.sh + e) = val;
  }
}

__global__ __launch_bounds__(256) void append_len_kernel(AttnParams p, const int* __restrict__ accept_len, int* __restrict__ kv_len_out) {
  const int seq = blockIdx.x * 256 + threadIdx.x;
  if (seq >= p.B) return;
  const SeqInfo s = load_seq_t<false>(p, seq);
  int add = 0;
  if (s.k > 0) {
    add = clampi(accept_len[seq], 0, s.k - 1) + 1;
    const int room = s.npages * p.page_size - s.L;              // rows the page list can still take
    if (add > room) add = room < 0 ? 0 : room;
  }
  kv_len_out[seq] = s.L + add;
}

hipError_t run_append_kv(const AttnParams& p, int dtype, void* k_cache, void* v_cache, const int* accept_len,
                         int* kv_len_out, hipStream_t st) {
  dim3 grid(p.max_new_rows, p.B);
  if (dtype == FD_BF16)
    hipLaunchKernelGGL(append_kv_kernel<bf16_t>, grid, dim3(256), 0, st, p, reinterpret_cast<bf16_t*>(k_cache),
                       reinterpret_cast<bf16_t*>(v_cache), accept_len);
  else
    hipLaunchKernelGGL(append_kv_kernel<float>, grid, dim3(256), 0, st, p, reinterpret_cast<float*>(k_cache),
                       reinterpret_cast<float*>(v_cache), accept_len);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(append_len_kernel, dim3((p.B + 255) / 256), dim3(256), 0, st, p, accept_len, kv_len_out);
  return hipGetLastError();
}

}  // namespace fd
