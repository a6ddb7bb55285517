// Commit of verified rows to the paged KV cache (Sec. 4.3, decoupled execution: the cache
// written by target verification is what the next draft step reuses).
//
// One work-group per sequence, one launch: the work-group reads the sequence's length once, copies
// new rows 0 .. accept_len (K and V, all KV heads, 16-byte accesses) to logical positions
// kv_len + j, and writes the new length last -- so the output array may be the input array.  Only
// verify rows are ever written: mask tokens stay invisible to the clean prefix (Sec. 4.1), so a
// sequence without verify rows commits nothing and accept_len is held below the number of verify rows.
#include "fd_common.h"

namespace fd {

template <typename T>
__global__ __launch_bounds__(256) void append_kv_kernel(AttnParams p, T* __restrict__ k_cache, T* __restrict__ v_cache,
                                                        const int* __restrict__ accept_len, int* __restrict__ kv_len_out) {
  const int seq = blockIdx.x;
  const SeqInfo s = load_seq(p, seq);                         // clamps and reports bad lengths; reads kv_len[seq]
  int rows = 0;                                               // rows this sequence commits
  if (s.k > 0) {
    int acc = sload(accept_len, seq);
    if (acc < 0 || acc >= s.k) { if (threadIdx.x == 0) flag_status(p.status, FD_DEV_ROWS_RANGE); acc = clampi(acc, 0, s.k - 1); }
    rows = acc + 1;
    // kv_len is the length BEFORE the commit; load_seq checked that the page list covers it, the rows
    // added here need their own check: whatever the list has no room for is not committed
    const int room = s.npages * p.page_size - s.L;
    if (rows > room) { if (threadIdx.x == 0) flag_status(p.status, FD_DEV_PAGE_RANGE); rows = room < 0 ? 0 : room; }
  }
  constexpr int VEC = 16 / sizeof(T);                          // elements per 16-byte vector
  const int vec_per_head = p.D / VEC;                          // head_dim is a multiple of 8
  const int nvec = p.Hkv * vec_per_head;
  for (int j = 0; j < rows; ++j) {
    const int pos = s.L + j;
    const int lp = pos / p.page_size, slot = pos - lp * p.page_size;
    const int phys = sload(p.page_indices, s.page0 + lp);
    if (phys < 0 || phys >= p.num_pages) { if (threadIdx.x == 0) flag_status(p.status, FD_DEV_PAGE_RANGE); continue; }
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
  // every thread has read what it needs of this sequence's old length by now (s is in registers);
  // no other work-group reads kv_len[seq]
  if (threadIdx.x == 0) kv_len_out[seq] = s.L + rows;
}

hipError_t run_append_kv(const AttnParams& p, int dtype, void* k_cache, void* v_cache, const int* accept_len,
                         int* kv_len_out, hipStream_t st) {
  if (dtype == FD_BF16)
    hipLaunchKernelGGL(append_kv_kernel<bf16_t>, dim3(p.B), dim3(256), 0, st, p, reinterpret_cast<bf16_t*>(k_cache),
                       reinterpret_cast<bf16_t*>(v_cache), accept_len, kv_len_out);
  else
    hipLaunchKernelGGL(append_kv_kernel<float>, dim3(p.B), dim3(256), 0, st, p, reinterpret_cast<float*>(k_cache),
                       reinterpret_cast<float*>(v_cache), accept_len, kv_len_out);
  return hipGetLastError();
}

}  // namespace fd
