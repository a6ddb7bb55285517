// Shared device/host helpers of the gfx950 library (internal; not part of the C ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "flexdraft.h"

#define FD_WAVE 64

namespace fd {

typedef unsigned short bf16_t;                                   // raw bf16 bit pattern
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;  // 16-byte vector
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((unsigned)b) << 16); }

// round-to-nearest-even; inputs here are finite
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  unsigned u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((u >> 16) | 0x40);  // NaN stays NaN
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename T> struct Elem;
template <> struct Elem<float> {
  static __device__ __forceinline__ float load(const float* p) { return *p; }
  static __device__ __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  static __device__ __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Load through the scalar (constant) path: for read-only tables indexed uniformly across the
// wave (page ids, per-sequence lengths).  The pointer must not alias anything the kernel writes.
typedef const __attribute__((address_space(4))) int* const_int_ptr;
__device__ __forceinline__ int sload(const int* p, int idx) {
  return ((const_int_ptr)(uintptr_t)p)[idx];
}

__device__ __forceinline__ int clampi(int x, int lo, int hi) { return x < lo ? lo : (x > hi ? hi : x); }

__device__ __forceinline__ void flag_status(uint32_t* status, uint32_t bit) {
  if (status) atomicOr(status, bit);
}

// Per-sequence description every attention kernel derives from the device arrays,
// clamped to the host-declared bounds so that no later access leaves the buffers.
struct SeqInfo {
  int L;        // cached prefix tokens
  int row0;     // first packed row
  int n;        // new rows
  int k;        // verify rows
  int v;        // verify rows visible to mask block 0 (block b sees b more, at most k)
  int nb;       // mask blocks (n - k splits evenly into them)
  int page0;    // first entry in page_indices
  int npages;   // entries available
};

struct AttnParams {
  int B, Hq, Hkv, D, G, page_size;
  int total_rows, max_kv_len, max_new_rows, num_pages;
  int page_entries;   // length of page_indices, 0 = unknown (page_indptr is then trusted)
  int chunk;          // cached tokens per work-group
  int max_chunks;     // grid extent over chunks
  int row_tiles;      // grid extent over row tiles
  float sm_scale;
  const void* k_cache; const void* v_cache;
  long long sp, sh, st;                       // cache strides in elements
  const int* page_indptr; const int* page_indices; const int* kv_len;
  const int* row_indptr; const int* verify_len; const int* mask_vis; const int* mask_blocks;
  const void* q; const void* k_new; const void* v_new;
  void* out; float* lse;
  float* part_acc;    // [max_chunks][R][Hq][D]
  float* part_ml;     // [max_chunks][R][Hq][2]
  uint32_t* status;
};

// SCALAR: read through the scalar path (index uniform across the wave) and report bad data
// through the status word; otherwise plain per-lane loads and no reporting (used when lanes
// scan different sequences; `bad_out` then receives the FD_DEV_* bits).  Both give identical
// clamped values.
template <bool SCALAR>
__device__ __forceinline__ SeqInfo load_seq_t(const AttnParams& p, int i, uint32_t* bad_out = nullptr) {
  auto ld = [&](const int* a, int idx) { return SCALAR ? sload(a, idx) : a[idx]; };
  SeqInfo s;
  int L = ld(p.kv_len, i);
  int r0 = ld(p.row_indptr, i), r1 = ld(p.row_indptr, i + 1);
  int k = ld(p.verify_len, i);
  int pg0 = ld(p.page_indptr, i), pg1 = ld(p.page_indptr, i + 1);
  uint32_t bad = 0;
  if (L < 0 || L > p.max_kv_len) bad |= FD_DEV_KV_LEN_RANGE;
  s.L = clampi(L, 0, p.max_kv_len);
  if (r0 < 0 || r0 > p.total_rows || r1 < r0 || r1 > p.total_rows || r1 - r0 > p.max_new_rows) bad |= FD_DEV_ROWS_RANGE;
  s.row0 = clampi(r0, 0, p.total_rows);
  s.n = clampi(r1 - r0, 0, p.max_new_rows);
  if (s.row0 + s.n > p.total_rows) s.n = p.total_rows - s.row0;
  if (k < 0 || k > s.n) bad |= FD_DEV_ROWS_RANGE;
  s.k = clampi(k, 0, s.n);
  int nb = 1;
  if (p.mask_blocks) {
    nb = ld(p.mask_blocks, i);
    if (nb < 1 || (s.n - s.k) % (nb < 1 ? 1 : nb)) { bad |= FD_DEV_ROWS_RANGE; nb = 1; }
  }
  s.nb = nb;
  int v = s.k - nb + 1 < 0 ? 0 : s.k - nb + 1;
  if (p.mask_vis) {
    v = ld(p.mask_vis, i);
    if (v < 0 || v > s.k) bad |= FD_DEV_ROWS_RANGE;
    v = clampi(v, 0, s.k);
  }
  s.v = v;
  bool list_bad = pg0 < 0;
  if (p.page_entries > 0 && (pg0 > p.page_entries || pg1 > p.page_entries)) {      // list runs past the array
    list_bad = true;
    pg0 = pg0 > p.page_entries ? p.page_entries : pg0;
    pg1 = pg1 > p.page_entries ? p.page_entries : pg1;
  }
  s.page0 = pg0 < 0 ? 0 : pg0;
  s.npages = pg1 - s.page0 < 0 ? 0 : pg1 - s.page0;
  int need = (s.L + p.page_size - 1) / p.page_size;
  if (list_bad || need > s.npages) {      // page list shorter than kv_len claims
    bad |= FD_DEV_PAGE_RANGE;
    s.L = s.npages * p.page_size < s.L ? s.npages * p.page_size : s.L;
  }
  if (SCALAR && bad) flag_status(p.status, bad);
  if (bad_out) *bad_out = bad;
  return s;
}

__device__ __forceinline__ SeqInfo load_seq(const AttnParams& p, int i) { return load_seq_t<true>(p, i); }

// The same bounds applied to a description that came from somewhere else than the device arrays
// (a plan entry): whatever it holds, nothing derived from it leaves the caller's buffers.  The
// length of page_indices must be known (page_entries > 0).
__device__ __forceinline__ void clamp_seq(const AttnParams& p, SeqInfo& s) {
  s.L = clampi(s.L, 0, p.max_kv_len);
  s.row0 = clampi(s.row0, 0, p.total_rows);
  s.n = clampi(s.n, 0, p.max_new_rows < p.total_rows - s.row0 ? p.max_new_rows : p.total_rows - s.row0);
  s.k = clampi(s.k, 0, s.n);
  s.v = clampi(s.v, 0, s.k);
  if (s.nb < 1 || (s.n - s.k) % s.nb) s.nb = 1;
  s.page0 = clampi(s.page0, 0, p.page_entries);
  s.npages = clampi(s.npages, 0, p.page_entries - s.page0);
  const long long cap = (long long)s.npages * p.page_size;
  if (cap < s.L) s.L = (int)cap;
}

// What new row r (0-based within the sequence) sees among the new rows, Sec. 4.1: the rows
// t < vr, and the rows lo <= t < hi.  A verify row is causal (vr = r + 1, no second range); a
// mask row of block b sees the first min(v + b, k) verify rows and its own block.
struct RowWindow { int vr, lo, hi; };
__device__ __forceinline__ RowWindow row_window(int r, const SeqInfo& s) {
  RowWindow w;
  if (r < s.k) { w.vr = r + 1; w.lo = 0; w.hi = 0; return w; }
  const int mb = (s.n - s.k) / s.nb;                // >= 1 whenever a mask row exists
  const int b = (r - s.k) / (mb > 0 ? mb : 1);
  w.vr = s.v + b < s.k ? s.v + b : s.k;
  w.lo = s.k + b * mb;
  w.hi = w.lo + mb;
  return w;
}
__device__ __forceinline__ bool new_key_visible(const RowWindow& w, int t) {
  return (t < w.vr) | ((t >= w.lo) & (t < w.hi));
}

}  // namespace fd
