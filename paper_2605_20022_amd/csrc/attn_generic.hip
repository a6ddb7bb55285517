// Hybrid-mask verify+draft attention (Sec. 4.1), scalar fp32 kernel.
//
// This is the fp32 path (and the path for shapes the MFMA kernel does not take): every
// product and sum is an fp32 FMA, exponentials are accurate expf, so that an fp32 call
// stays within 1e-5 of the fp64 definition.  One work-group handles 16 tile rows (a tile
// row is one new row of one query head of the KV head's group) of one (sequence, KV head,
// KV chunk) and streams that chunk's keys 32 at a time through LDS.  The cached prefix
// needs no mask (every new row sees all of it, Sec. 4.1); only the ragged tail and the
// new-row tile are masked.  Results are left as split partials (running max, sum, and
// un-normalised output) that the combine kernel merges.
#include "fd_common.h"

namespace fd {

constexpr int GEN_BLOCK = 256;
constexpr int GEN_ROWS = 16;    // tile rows per work-group
constexpr int GEN_KEYS = 32;    // keys per LDS tile
constexpr int GEN_DMAX = 128;

template <typename T>
__global__ __launch_bounds__(GEN_BLOCK) void attn_generic_kernel(AttnParams p) {
  __shared__ float Qs[GEN_ROWS][GEN_DMAX];
  __shared__ float Ks[GEN_KEYS][GEN_DMAX + 1];
  __shared__ float Vs[GEN_KEYS][GEN_DMAX];
  __shared__ float Ps[GEN_ROWS][GEN_KEYS + 1];

  // Consecutive work-group ids go to different XCDs; rotating the chunk index by head and
  // sequence keeps any one XCD from collecting only the long (or only the short) chunks.
  const int chunk_id = (blockIdx.x + blockIdx.y + blockIdx.z) % gridDim.x;
  const int g = blockIdx.y % p.Hkv, rt = blockIdx.y / p.Hkv;
  const int seq = blockIdx.z;
  const SeqInfo s = load_seq(p, seq);
  const int nchunks = max(1, (s.L + p.chunk - 1) / p.chunk);
  const int rows_total = s.n * p.G;
  if (chunk_id >= nchunks || rt * GEN_ROWS >= rows_total) return;
  const int D = p.D, tid = threadIdx.x;
  const T* Kc = reinterpret_cast<const T*>(p.k_cache);
  const T* Vc = reinterpret_cast<const T*>(p.v_cache);
  const T* Q = reinterpret_cast<const T*>(p.q);
  const T* Kn = reinterpret_cast<const T*>(p.k_new);
  const T* Vn = reinterpret_cast<const T*>(p.v_new);

  // query tile: tile row T -> new row T / G, head g*G + T % G
  for (int idx = tid; idx < GEN_ROWS * D; idx += GEN_BLOCK) {
    int tr = idx / D, d = idx % D;
    int T_ = rt * GEN_ROWS + tr;
    float val = 0.f;
    if (T_ < rows_total) {
      int nn = T_ / p.G, hq = g * p.G + T_ % p.G;
      val = Elem<T>::load(Q + ((long long)(s.row0 + nn) * p.Hq + hq) * D + d);
    }
    Qs[tr][d] = val;
  }

  const int my_row = tid / 16;            // tile row owned in the score / softmax / PV phases
  const int sub = tid % 16;
  const int my_T = rt * GEN_ROWS + my_row;
  const int my_nn = my_T / p.G;           // new-row index of my tile row
  const RowWindow my_win = row_window(my_nn < s.n ? my_nn : 0, s);
  float m_run = -INFINITY, l_run = 0.f;
  float acc[GEN_DMAX / 16];
#pragma unroll
  for (int j = 0; j < GEN_DMAX / 16; ++j) acc[j] = 0.f;

  const int c0 = chunk_id * p.chunk;
  const int c1 = min(s.L, c0 + p.chunk);
  const bool has_new = (chunk_id == nchunks - 1);
  const int cached_tiles = c1 > c0 ? (c1 - c0 + GEN_KEYS - 1) / GEN_KEYS : 0;
  const int new_tiles = has_new ? (s.n + GEN_KEYS - 1) / GEN_KEYS : 0;

  for (int t = 0; t < cached_tiles + new_tiles; ++t) {
    const bool is_new = t >= cached_tiles;
    const int base = is_new ? (t - cached_tiles) * GEN_KEYS : c0 + t * GEN_KEYS;
    __syncthreads();                       // previous tile fully consumed (and Qs written)
    for (int idx = tid; idx < GEN_KEYS * D; idx += GEN_BLOCK) {
      int kk = idx / D, d = idx % D;
      int key = base + kk;
      float kv = 0.f, vv = 0.f;
      if (is_new) {
        if (key < s.n) {
          long long off = ((long long)(s.row0 + key) * p.Hkv + g) * D + d;
          kv = Elem<T>::load(Kn + off); vv = Elem<T>::load(Vn + off);
        }
      } else if (key < c1) {
        int lp = key / p.page_size, slot = key % p.page_size;
        int phys = p.page_indices[s.page0 + lp];
        if (phys < 0 || phys >= p.num_pages) { flag_status(p.status, FD_DEV_PAGE_RANGE); phys = 0; }
        long long off = (long long)phys * p.sp + (long long)g * p.sh + (long long)slot * p.st + d;
        kv = Elem<T>::load(Kc + off); vv = Elem<T>::load(Vc + off);
      }
      Ks[kk][d] = kv; Vs[kk][d] = vv;
    }
    __syncthreads();
    // scores: thread (my_row, sub) computes keys sub and sub+16
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      int kk = sub + 16 * h;
      float dot = 0.f;
      for (int d = 0; d < D; ++d) dot = fmaf(Qs[my_row][d], Ks[kk][d], dot);
      int key = base + kk;
      bool vis = is_new ? (new_key_visible(my_win, key) && key < s.n) : (key < c1);
      Ps[my_row][kk] = vis ? dot * p.sm_scale : -INFINITY;
    }
    __syncthreads();
    // online softmax for my row (the 16 threads of a row all hold the same state)
    float tmax = -INFINITY;
    for (int kk = 0; kk < GEN_KEYS; ++kk) tmax = fmaxf(tmax, Ps[my_row][kk]);
    float m_new = fmaxf(m_run, tmax);
    float alpha = (m_new == -INFINITY) ? 1.f : expf(m_run - m_new);   // exp(-inf) = 0 on the first real tile
    float p0 = 0.f, p1 = 0.f;
    if (m_new > -INFINITY) {
      p0 = expf(Ps[my_row][sub] - m_new);
      p1 = expf(Ps[my_row][sub + 16] - m_new);
    }
    float psum = p0 + p1;
#pragma unroll
    for (int off = 8; off >= 1; off >>= 1) psum += __shfl_xor(psum, off);
    __syncthreads();                       // everyone has read the scores
    Ps[my_row][sub] = p0; Ps[my_row][sub + 16] = p1;
    l_run = l_run * alpha + psum;
    m_run = m_new;
    __syncthreads();
    // output columns sub, sub+16, ... (D is a multiple of 8, not necessarily of 16)
    for (int j = 0; j * 16 < D; ++j) {
      int d = sub + 16 * j;
      if (d >= D) break;
      float a = acc[j] * alpha;
      for (int kk = 0; kk < GEN_KEYS; ++kk) a = fmaf(Ps[my_row][kk], Vs[kk][d], a);
      acc[j] = a;
    }
  }

  if (my_T < rows_total) {
    int hq = g * p.G + my_T % p.G;
    long long slot = ((long long)chunk_id * p.total_rows + (s.row0 + my_nn)) * p.Hq + hq;
    for (int j = 0; sub + 16 * j < D; ++j) p.part_acc[slot * D + sub + 16 * j] = acc[j];
    if (sub == 0) { p.part_ml[slot * 2] = m_run; p.part_ml[slot * 2 + 1] = l_run; }
  }
}

// ---------------------------------------------------------------------------------------
// Combine the per-chunk partials of every (row, head):
//   M = max_c m_c;  out = sum_c e^{m_c - M} acc_c / sum_c e^{m_c - M} l_c;  lse = M + log(sum)
// `log2_units` says the partial maxima are in base-2 exponent units (the MFMA kernel) or
// natural units (the scalar kernel).  `skip_single`: sequences that fit one chunk were already
// normalised and stored by the streaming kernel.  grid (ceil(Hq*D/256), max_new_rows, B).
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void attn_combine_kernel(AttnParams p, int log2_units, int skip_single) {
  const int seq = blockIdx.z, nn = blockIdx.y;
  const SeqInfo s = load_seq(p, seq);
  if (nn >= s.n) return;
  if (skip_single && s.L <= p.chunk) return;     // the streaming kernel already wrote these rows
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= p.Hq * p.D) return;
  const int hq = idx / p.D, d = idx % p.D;
  const int nchunks = max(1, (s.L + p.chunk - 1) / p.chunk);
  const long long row = s.row0 + nn;
  const long long stride = (long long)p.total_rows * p.Hq;     // partial slots per chunk
  const long long slot0 = row * p.Hq + hq;
  float M = -INFINITY;
  for (int c = 0; c < nchunks; ++c) M = fmaxf(M, p.part_ml[(slot0 + c * stride) * 2]);
  float num = 0.f, den = 0.f;
  for (int c = 0; c < nchunks; ++c) {
    long long sl = slot0 + c * stride;
    float mc = p.part_ml[sl * 2];
    if (mc == -INFINITY) continue;
    float w = log2_units ? exp2f(mc - M) : expf(mc - M);
    num = fmaf(w, p.part_acc[sl * p.D + d], num);
    den = fmaf(w, p.part_ml[sl * 2 + 1], den);
  }
  float o = den > 0.f ? num / den : 0.f;
  Elem<T>::store(reinterpret_cast<T*>(p.out) + (row * p.Hq + hq) * p.D + d, o);
  if (p.lse && d == 0)
    p.lse[row * p.Hq + hq] = log2_units ? (M + log2f(den)) * 0.6931471805599453f : M + logf(den);
}

hipError_t run_attn_generic(const AttnParams& p, int dtype, hipStream_t st) {
  dim3 grid(p.max_chunks, p.Hkv * ((p.max_new_rows * p.G + GEN_ROWS - 1) / GEN_ROWS), p.B);
  if (dtype == FD_BF16) hipLaunchKernelGGL(attn_generic_kernel<bf16_t>, grid, dim3(GEN_BLOCK), 0, st, p);
  else hipLaunchKernelGGL(attn_generic_kernel<float>, grid, dim3(GEN_BLOCK), 0, st, p);
  return hipGetLastError();
}

hipError_t run_attn_combine(const AttnParams& p, int dtype, int log2_units, int skip_single, hipStream_t st) {
  dim3 grid((p.Hq * p.D + 255) / 256, p.max_new_rows, p.B);
  if (dtype == FD_BF16) hipLaunchKernelGGL(attn_combine_kernel<bf16_t>, grid, dim3(256), 0, st, p, log2_units, skip_single);
  else hipLaunchKernelGGL(attn_combine_kernel<float>, grid, dim3(256), 0, st, p, log2_units, skip_single);
  return hipGetLastError();
}

}  // namespace fd
