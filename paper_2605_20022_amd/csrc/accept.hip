// Lossless acceptance kernels (Sec. 3): greedy arg-max / longest matching prefix / bonus
// token, and the speculative-sampling variant with supplied uniforms.
//
// Both are one streaming pass over [rows][vocab] logits, so the vocabulary of every row
// is cut into segments and one work-group reduces one (row, segment); a small epilogue
// per sequence merges the segment results and walks the verify rows.
#include "fd_common.h"
#include <float.h>

namespace fd {

constexpr int ACC_BLOCK = 256;

// 8 consecutive logits starting at element `e` of a row (e multiple of 8) as floats;
// entries at or beyond `vocab` come back as -inf.  `vec_ok` says the row base is 16-byte
// aligned so that one 16-byte load per lane can be used.
template <typename T>
__device__ __forceinline__ void load8(const T* row, int e, int vocab, bool vec_ok, float (&x)[8]);

template <>
__device__ __forceinline__ void load8<bf16_t>(const bf16_t* row, int e, int vocab, bool vec_ok, float (&x)[8]) {
  if (vec_ok && e + 8 <= vocab) {
    u32x4 w = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(row + e));
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[2 * i] = __uint_as_float(w[i] << 16);
      x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (e + i < vocab) ? bf16_to_f32(row[e + i]) : -INFINITY;
  }
}

template <>
__device__ __forceinline__ void load8<float>(const float* row, int e, int vocab, bool vec_ok, float (&x)[8]) {
  if (vec_ok && e + 8 <= vocab) {
    f32x4 a = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + e));
    f32x4 b = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(row + e + 4));
    x[0] = a[0]; x[1] = a[1]; x[2] = a[2]; x[3] = a[3];
    x[4] = b[0]; x[5] = b[1]; x[6] = b[2]; x[7] = b[3];
  } else {
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = (e + i < vocab) ? row[e + i] : -INFINITY;
  }
}

// (value, index) with "larger value wins, equal values: lower index wins"
__device__ __forceinline__ void amax_merge(float& v, int& i, float ov, int oi) {
  if (ov > v || (ov == v && oi < i)) { v = ov; i = oi; }
}

// ---------------------------------------------------------------------------------------
// Greedy, pass 1: arg-max of one vocabulary segment of one row.
//   grid (segments, rows); part_val/part_idx [rows][segments]
// A segment is at most ACC_BLOCK * 8 * ARG_ROUNDS logits, so a lane holds all of its share in
// registers.  First the segment's maximum (one max per logit), then only the lanes whose own
// maximum equals it look for the lowest index holding that value: comparing (value, index)
// pairs logit by logit would cost several times the instructions and bound the kernel by
// arithmetic rather than by the stream.
// ---------------------------------------------------------------------------------------
constexpr int ARG_ROUNDS = 5;
constexpr int ARG_SEG_MAX = ACC_BLOCK * 8 * ARG_ROUNDS;

template <typename T>
__global__ __launch_bounds__(ACC_BLOCK) void argmax_partial_kernel(
    const T* __restrict__ logits, long long row_stride, int vocab, int seg_len,
    float* __restrict__ part_val, int* __restrict__ part_idx) {
  const int seg = blockIdx.x, row = blockIdx.y, nseg = gridDim.x;
  const T* rp = logits + (long long)row * row_stride;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(rp) & 15) == 0;
  const int e0 = seg * seg_len;
  const int e1 = min(vocab, e0 + min(seg_len, ARG_SEG_MAX));
  __shared__ float sv[ACC_BLOCK / FD_WAVE]; __shared__ int si[ACC_BLOCK / FD_WAVE];
  float x[ARG_ROUNDS][8];
#pragma unroll
  for (int u = 0; u < ARG_ROUNDS; ++u) load8<T>(rp, e0 + (u * ACC_BLOCK + threadIdx.x) * 8, e1, vec_ok, x[u]);   // -inf past e1
  float m = -INFINITY;
#pragma unroll
  for (int u = 0; u < ARG_ROUNDS; ++u)
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, x[u][i]);
  float wm = m;
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) wm = fmaxf(wm, __shfl_xor(wm, off));
  if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = wm;
  __syncthreads();
  float M = sv[0];
#pragma unroll
  for (int w = 1; w < ACC_BLOCK / FD_WAVE; ++w) M = fmaxf(M, sv[w]);
  int bi = 0x7fffffff;
  if (m == M) {
#pragma unroll
    for (int u = ARG_ROUNDS - 1; u >= 0; --u)
#pragma unroll
      for (int i = 7; i >= 0; --i) {
        const int idx = e0 + (u * ACC_BLOCK + threadIdx.x) * 8 + i;
        if (x[u][i] == M && idx < e1) bi = idx;            // descending walk: the lowest index is kept
      }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) bi = min(bi, __shfl_xor(bi, off));
  if ((threadIdx.x & 63) == 0) si[threadIdx.x >> 6] = bi;
  __syncthreads();
  if (threadIdx.x == 0) {
#pragma unroll
    for (int w = 1; w < ACC_BLOCK / FD_WAVE; ++w) bi = min(bi, si[w]);
    part_val[(long long)row * nseg + seg] = M;
    part_idx[(long long)row * nseg + seg] = bi;
  }
}

// ---------------------------------------------------------------------------------------
// Greedy, pass 2: one wave per sequence.  Merge the segment results of each verify row,
// then count the leading rows whose arg-max equals the token fed at the next row.
// ---------------------------------------------------------------------------------------
constexpr int GE_GROUP = 16;                       // lanes that merge one row's segments
constexpr int GE_ROWS = ACC_BLOCK / GE_GROUP;     // rows merged at a time

__global__ __launch_bounds__(ACC_BLOCK) void accept_greedy_epilogue_kernel(
    const float* __restrict__ part_val, const int* __restrict__ part_idx, int nseg,
    const int* __restrict__ row_indptr, const int* __restrict__ input_tokens,
    int total_rows, int max_rows_per_seq,
    int* __restrict__ accept_len, int* __restrict__ bonus_token, int* __restrict__ row_argmax) {
  const int seq = blockIdx.x, grp = threadIdx.x / GE_GROUP, gl = threadIdx.x % GE_GROUP;
  int r0 = clampi(row_indptr[seq], 0, total_rows);
  int k = clampi(row_indptr[seq + 1] - r0, 0, min(max_rows_per_seq, total_rows - r0));
  if (k == 0) { if (threadIdx.x == 0) { accept_len[seq] = 0; bonus_token[seq] = -1; } return; }
  // Rows GE_ROWS at a time, in order: GE_GROUP lanes merge a row's segments (every load of a batch is
  // in flight together); the first row whose arg-max differs from the token fed at the next row --
  // or the last row -- ends the step and its arg-max is the bonus token.
  __shared__ int s_first_bad, s_bonus;
  if (threadIdx.x == 0) { s_first_bad = 0x7fffffff; s_bonus = -1; }
  __syncthreads();
  bool done = false;
  for (int j0 = 0; j0 < k; j0 += GE_ROWS) {
    const int j = j0 + grp;
    float bv = -INFINITY; int bi = 0x7fffffff;
    if (j < k)
      for (int s = gl; s < nseg; s += GE_GROUP)
        amax_merge(bv, bi, part_val[(long long)(r0 + j) * nseg + s], part_idx[(long long)(r0 + j) * nseg + s]);
#pragma unroll
    for (int off = GE_GROUP / 2; off >= 1; off >>= 1) {
      const float ov = __shfl_xor(bv, off); const int oi = __shfl_xor(bi, off);
      amax_merge(bv, bi, ov, oi);
    }
    if (gl == 0 && j < k) {
      if (row_argmax) row_argmax[r0 + j] = bi;
      if (!done && ((j == k - 1) || (bi != input_tokens[r0 + j + 1]))) atomicMin(&s_first_bad, j);
    }
    __syncthreads();
    if (!done && s_first_bad < j0 + GE_ROWS) {       // decided in this batch: its owner publishes the bonus token
      if (gl == 0 && j == s_first_bad) s_bonus = bi;
      done = true;
      if (!row_argmax) break;                        // (uniform) nothing else is wanted from the later rows
    }
  }
  __syncthreads();
  if (threadIdx.x == 0) { accept_len[seq] = s_first_bad; bonus_token[seq] = s_bonus; }
}

// ---------------------------------------------------------------------------------------
// Sampling, pass 1: per (row, segment) the maximum and the sum of exponentials of the
// temperature-scaled target and draft logits.  part [rows][segments][4] doubles:
// (max_t, sum_t, max_d, sum_d) with sum = sum exp(x*invT - max).
// ---------------------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off));
  return v;
}

// e^y for y <= 0.  e^y = 2^(y log2 e): the product is formed in two pieces, so that its rounding
// error (which grows with |y|) and the low part of log2 e enter as a first-order correction of
// the hardware exp2 (good to 1 ulp).  About a third of the instructions of the library expf,
// which is what the streaming passes below were spending their time on.
__device__ __forceinline__ float exp_neg(float y) {
  y = fmaxf(y, -104.f);                               // e^-104 is below the smallest normal float
  const float t = y * 1.44269502e+00f;
  float r = fmaf(y, 1.44269502e+00f, -t);             // rounding error of t, exactly
  r = fmaf(y, 1.92596299e-08f, r);                    // log2 e = 1.44269502 + 1.92596299e-8
  const float e = __builtin_amdgcn_exp2f(t);
  return fmaf(e, r * 0.693147182f, e);
}

// Sampling, pass 1: per (row, segment) the maximum of x / T and sum exp(x / T - max), for the
// target and the draft logits.  Both segments are requested up front and held in registers (one
// memory latency per work-group), the maximum is found first and the sum taken relative to it: the
// maximum's own term is exactly 1 and every other term's rounding error (|y| 2^-23 of itself,
// y = x / T - max <= 0) is weighted by its small size, so the plain hardware exp2 is accurate
// enough for a normaliser that is compared at 1e-5.
//   grid (segments, rows); part [rows][segments][4] = (max_t, sum_t, max_d, sum_d)
//   NR = rounds of ACC_BLOCK * 8 logits that cover a segment (registers held: 16 NR floats)
template <typename T, int NR>
__global__ __launch_bounds__(ACC_BLOCK) void softmax_stats_partial_kernel(
    const T* __restrict__ target, const T* __restrict__ draft, long long row_stride, int vocab, int seg_len,
    float inv_t, double* __restrict__ part) {
  constexpr int NW = ACC_BLOCK / FD_WAVE;
  __shared__ float s_max[2][NW]; __shared__ double s_sum[2][NW];
  const int seg = blockIdx.x, row = blockIdx.y, nseg = gridDim.x;
  const int e0 = seg * seg_len, e1 = min(vocab, e0 + min(seg_len, NR * ACC_BLOCK * 8));
  const T* tp = target + (long long)row * row_stride;
  const T* dp = draft + (long long)row * row_stride;
  const bool vt = (reinterpret_cast<uintptr_t>(tp) & 15) == 0, vd = (reinterpret_cast<uintptr_t>(dp) & 15) == 0;
  float xt[NR][8], xd[NR][8];
#pragma unroll
  for (int u = 0; u < NR; ++u) load8<T>(tp, e0 + (u * ACC_BLOCK + threadIdx.x) * 8, e1, vt, xt[u]);   // -inf past e1
#pragma unroll
  for (int u = 0; u < NR; ++u) load8<T>(dp, e0 + (u * ACC_BLOCK + threadIdx.x) * 8, e1, vd, xd[u]);
  float mt = -INFINITY, md = -INFINITY;
#pragma unroll
  for (int u = 0; u < NR; ++u)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      xt[u][i] *= inv_t; xd[u][i] *= inv_t;                       // padding stays -inf (1 / T > 0)
      mt = fmaxf(mt, xt[u][i]); md = fmaxf(md, xd[u][i]);
    }
  mt = wave_max(mt); md = wave_max(md);
  if ((threadIdx.x & 63) == 0) { s_max[0][threadIdx.x >> 6] = mt; s_max[1][threadIdx.x >> 6] = md; }
  __syncthreads();
  float Mt = s_max[0][0], Md = s_max[1][0];
#pragma unroll
  for (int w = 1; w < NW; ++w) { Mt = fmaxf(Mt, s_max[0][w]); Md = fmaxf(Md, s_max[1][w]); }
  float st = 0.f, sd = 0.f;
  const float L2E = 1.44269502e+00f;
  if (Mt > -INFINITY) {
#pragma unroll
    for (int u = 0; u < NR; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) st += __builtin_amdgcn_exp2f((xt[u][i] - Mt) * L2E);     // padding: 2^-inf = 0
  }
  if (Md > -INFINITY) {
#pragma unroll
    for (int u = 0; u < NR; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) sd += __builtin_amdgcn_exp2f((xd[u][i] - Md) * L2E);
  }
  const double wt = wave_sum((double)st), wd = wave_sum((double)sd);
  if ((threadIdx.x & 63) == 0) { s_sum[0][threadIdx.x >> 6] = wt; s_sum[1][threadIdx.x >> 6] = wd; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double tt = 0.0, td = 0.0;
#pragma unroll
    for (int w = 0; w < NW; ++w) { tt += s_sum[0][w]; td += s_sum[1][w]; }
    double* o = part + ((long long)row * nseg + seg) * 4;
    o[0] = (double)Mt; o[1] = tt; o[2] = (double)Md; o[3] = td;
  }
}

// ---------------------------------------------------------------------------------------
// Sampling, pass 2: grid (chunk groups, sequences).  Every work-group first repeats the
// (cheap) accept tests of its sequence to find the stopping row j*, then sums the bonus
// token's weights -- residual max(0,p-q), and p itself -- over its share of the
// vocabulary, one double per 512-token chunk (one wave, 8 tokens per lane).
//   decision [B][4] int: (stop row, rejected?, -, -) written by group 0
//   chunk_res, chunk_p [B][nchunks] doubles
// ---------------------------------------------------------------------------------------
constexpr int CHUNK_TOK = FD_WAVE * 8;   // 512 tokens per chunk

template <typename T>
__global__ __launch_bounds__(ACC_BLOCK) void accept_sample_weights_kernel(
    const T* __restrict__ target, const T* __restrict__ draft, long long row_stride, int vocab, float inv_t,
    const double* __restrict__ part, int nseg,
    const int* __restrict__ row_indptr, const int* __restrict__ input_tokens,
    const float* __restrict__ u_accept, int total_rows, int max_rows_per_seq, int nchunks,
    int* __restrict__ decision, double* __restrict__ row_stats /*[B][4]*/,
    double* __restrict__ chunk_res, double* __restrict__ chunk_p) {
  const int seq = blockIdx.y, grp = blockIdx.x, ngrp = gridDim.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NW = ACC_BLOCK / FD_WAVE;
  int r0 = clampi(row_indptr[seq], 0, total_rows);
  int k = clampi(row_indptr[seq + 1] - r0, 0, min(max_rows_per_seq, total_rows - r0));
  if (k == 0) { if (grp == 0 && threadIdx.x == 0) { decision[seq * 4] = -1; decision[seq * 4 + 1] = 0; } return; }

  // Accept tests: SG lanes per row merge that row's segment statistics, ROWS_AT_ONCE rows at a time
  // (every load of a batch is in flight together).  The statistics of a batch stay in LDS, so the
  // row the step stops at -- the first rejected draft, else the last row -- is at hand afterwards.
  constexpr int SG = 16, ROWS_AT_ONCE = ACC_BLOCK / SG;
  __shared__ int s_first_bad;
  __shared__ double s_rows[ROWS_AT_ONCE][4];
  __shared__ double s_stats[4];
  const int grp16 = threadIdx.x / SG, gl = threadIdx.x % SG;
  if (threadIdx.x == 0) s_first_bad = k - 1;
  __syncthreads();
  int stop = k - 1;
  for (int j0 = 0; j0 < k; j0 += ROWS_AT_ONCE) {
    const int j = min(j0 + grp16, k - 1);                          // surplus lane groups repeat the last row
    const double* pr = part + (long long)(r0 + j) * nseg * 4;
    double mt = -INFINITY, md = -INFINITY;
    for (int sg = gl; sg < nseg; sg += SG) { mt = fmax(mt, pr[sg * 4]); md = fmax(md, pr[sg * 4 + 2]); }
#pragma unroll
    for (int off = SG / 2; off >= 1; off >>= 1) { mt = fmax(mt, __shfl_xor(mt, off)); md = fmax(md, __shfl_xor(md, off)); }
    double zt = 0.0, zd = 0.0;
    for (int sg = gl; sg < nseg; sg += SG) {
      const double m0 = pr[sg * 4], s0 = pr[sg * 4 + 1], m1 = pr[sg * 4 + 2], s1 = pr[sg * 4 + 3];
      if (s0 > 0.0) zt += s0 * (double)exp_neg((float)(m0 - mt));     // maxima are floats held in doubles: the difference is exact
      if (s1 > 0.0) zd += s1 * (double)exp_neg((float)(m1 - md));
    }
#pragma unroll
    for (int off = SG / 2; off >= 1; off >>= 1) { zt += __shfl_xor(zt, off); zd += __shfl_xor(zd, off); }
    if (gl == 0 && j0 + grp16 < k) {
      s_rows[grp16][0] = mt; s_rows[grp16][1] = zt; s_rows[grp16][2] = md; s_rows[grp16][3] = zd;
      if (j < k - 1) {                                              // the last row has no draft to test
        const int d = input_tokens[r0 + j + 1];
        bool keep = false;
        if (d >= 0 && d < vocab) {
          const float xt = Elem<T>::load(target + (long long)(r0 + j) * row_stride + d);
          const float xd = Elem<T>::load(draft + (long long)(r0 + j) * row_stride + d);
          const double p = (double)expf(xt * inv_t - (float)mt) / zt;
          const double q = (double)expf(xd * inv_t - (float)md) / zd;
          keep = (double)u_accept[r0 + j] * q < p;
        }
        if (!keep) atomicMin(&s_first_bad, j);
      }
    }
    __syncthreads();
    stop = s_first_bad;
    if (stop < j0 + ROWS_AT_ONCE) {                                 // the stopping row is in this batch
      if (threadIdx.x < 4) s_stats[threadIdx.x] = s_rows[stop - j0][threadIdx.x];
      break;                                                        // (uniform: every thread read the same stop)
    }
    __syncthreads();                                                // s_rows is rewritten by the next batch
  }
  __syncthreads();
  const bool rejected = stop < k - 1 ? true : false;   // stop == k-1 only when every draft was kept
  // (a rejection at row k-1 cannot happen: that row has no draft to test)
  const float Mt = (float)s_stats[0], Md = (float)s_stats[2];
  const double iZt = 1.0 / s_stats[1], iZd = 1.0 / s_stats[3];
  if (grp == 0 && threadIdx.x == 0) {
    decision[seq * 4] = stop; decision[seq * 4 + 1] = rejected ? 1 : 0;
    row_stats[seq * 4 + 0] = s_stats[0]; row_stats[seq * 4 + 1] = s_stats[1];
    row_stats[seq * 4 + 2] = s_stats[2]; row_stats[seq * 4 + 3] = s_stats[3];
  }
  const T* tp = target + (long long)(r0 + stop) * row_stride;
  const T* dp = draft + (long long)(r0 + stop) * row_stride;
  const bool vt = (reinterpret_cast<uintptr_t>(tp) & 15) == 0, vd = (reinterpret_cast<uintptr_t>(dp) & 15) == 0;
  for (int c = grp * NW + wave; c < nchunks; c += ngrp * NW) {
    int e = c * CHUNK_TOK + lane * 8;
    double wres = 0.0, wp = 0.0;
    if (e < vocab) {
      float xt[8], xd[8];
      load8<T>(tp, e, vocab, vt, xt);
      load8<T>(dp, e, vocab, vd, xd);
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        double p = (double)expf(xt[i] * inv_t - Mt) * iZt;
        double q = (double)expf(xd[i] * inv_t - Md) * iZd;
        wp += p;
        wres += fmax(0.0, p - q);
      }
    }
    wres = wave_sum(wres); wp = wave_sum(wp);
    if (lane == 0) { chunk_res[(long long)seq * nchunks + c] = wres; chunk_p[(long long)seq * nchunks + c] = wp; }
  }
}

// ---------------------------------------------------------------------------------------
// Sampling, pass 3: one work-group per sequence.  Scan the chunk sums, find the chunk the
// scaled uniform falls into, then scan that chunk's 512 tokens with one wave.
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(ACC_BLOCK) void accept_sample_pick_kernel(
    const T* __restrict__ target, const T* __restrict__ draft, long long row_stride, int vocab, float inv_t,
    const int* __restrict__ row_indptr, const float* __restrict__ u_resample, int total_rows,
    int nchunks, const int* __restrict__ decision, const double* __restrict__ row_stats,
    const double* __restrict__ chunk_res, const double* __restrict__ chunk_p,
    int* __restrict__ accept_len, int* __restrict__ bonus_token) {
  const int seq = blockIdx.x;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int NW = ACC_BLOCK / FD_WAVE;
  const int stop = decision[seq * 4];
  if (stop < 0) { if (threadIdx.x == 0) { accept_len[seq] = 0; bonus_token[seq] = -1; } return; }
  const int r0 = clampi(row_indptr[seq], 0, total_rows);
  const bool rejected = decision[seq * 4 + 1] != 0;
  __shared__ double s_wsum[NW];
  __shared__ double s_tot[2];
  __shared__ int s_chunk; __shared__ double s_prefix;

  // totals of both weightings
  double a = 0.0, b = 0.0;
  for (int c = threadIdx.x; c < nchunks; c += ACC_BLOCK) { a += chunk_res[(long long)seq * nchunks + c]; b += chunk_p[(long long)seq * nchunks + c]; }
  a = wave_sum(a);
  if (lane == 0) s_wsum[wave] = a;
  __syncthreads();
  if (threadIdx.x == 0) { double t = 0; for (int w = 0; w < NW; ++w) t += s_wsum[w]; s_tot[0] = t; }
  __syncthreads();
  b = wave_sum(b);
  if (lane == 0) s_wsum[wave] = b;
  __syncthreads();
  if (threadIdx.x == 0) { double t = 0; for (int w = 0; w < NW; ++w) t += s_wsum[w]; s_tot[1] = t; }
  __syncthreads();
  const bool use_res = rejected && s_tot[0] > 0.0;      // residual identically zero -> draw from p
  const double* cw = (use_res ? chunk_res : chunk_p) + (long long)seq * nchunks;
  const double W = use_res ? s_tot[0] : s_tot[1];
  const double thr = (double)u_resample[r0 + stop] * W;

  // ordered scan over chunks by wave 0 (chunk counts are a few hundred)
  if (wave == 0) {
    double run = 0.0; int found = -1; double pre = 0.0;
    for (int base = 0; base < nchunks && found < 0; base += FD_WAVE) {
      int c = base + lane;
      double w = c < nchunks ? cw[c] : 0.0;
      double inc = w;                                   // inclusive scan across lanes
#pragma unroll
      for (int off = 1; off < FD_WAVE; off <<= 1) { double o = __shfl_up(inc, off); if (lane >= off) inc += o; }
      bool hit = c < nchunks && (run + inc > thr);
      unsigned long long m = __ballot(hit);
      if (m) {
        int src = __ffsll((long long)m) - 1;
        found = base + src;
        pre = run + __shfl(inc, src) - __shfl(w, src);
      }
      run += __shfl(inc, FD_WAVE - 1);
    }
    if (found < 0) {                                    // rounding corner: take the last non-empty chunk
      pre = 0.0; run = 0.0;
      for (int c = 0; c < nchunks; ++c) { double w = cw[c]; if (w > 0.0) { found = c; pre = run; } run += w; }
      if (found < 0) found = 0;
    }
    if (lane == 0) { s_chunk = found; s_prefix = pre; }
  }
  __syncthreads();
  if (wave != 0) return;
  const int c = s_chunk;
  const float Mt = (float)row_stats[seq * 4 + 0], Md = (float)row_stats[seq * 4 + 2];
  const double iZt = 1.0 / row_stats[seq * 4 + 1], iZd = 1.0 / row_stats[seq * 4 + 3];
  const T* tp = target + (long long)(r0 + stop) * row_stride;
  const T* dp = draft + (long long)(r0 + stop) * row_stride;
  const bool vt = (reinterpret_cast<uintptr_t>(tp) & 15) == 0, vd = (reinterpret_cast<uintptr_t>(dp) & 15) == 0;
  const int e = c * CHUNK_TOK + lane * 8;
  double w8[8]; double lsum = 0.0;
#pragma unroll
  for (int i = 0; i < 8; ++i) w8[i] = 0.0;
  if (e < vocab) {
    float xt[8], xd[8];
    load8<T>(tp, e, vocab, vt, xt);
    load8<T>(dp, e, vocab, vd, xd);
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      double p = (double)expf(xt[i] * inv_t - Mt) * iZt;
      double q = (double)expf(xd[i] * inv_t - Md) * iZd;
      w8[i] = use_res ? fmax(0.0, p - q) : p;
      lsum += w8[i];
    }
  }
  double inc = lsum;
#pragma unroll
  for (int off = 1; off < FD_WAVE; off <<= 1) { double o = __shfl_up(inc, off); if (lane >= off) inc += o; }
  double before = s_prefix + inc - lsum;
  int pick = -1;
  if (before + lsum > thr) {                            // the threshold is crossed inside this lane (or earlier)
    double run = before;
#pragma unroll
    for (int i = 0; i < 8; ++i) { run += w8[i]; if (pick < 0 && run > thr && w8[i] > 0.0) pick = e + i; }
  }
  unsigned long long m = __ballot(pick >= 0);
  int result;
  if (m) {
    result = __shfl(pick, __ffsll((long long)m) - 1);
  } else {                                              // rounding corner: last token of the chunk with weight
    int last = -1;
#pragma unroll
    for (int i = 0; i < 8; ++i) if (w8[i] > 0.0) last = e + i;
    unsigned long long m2 = __ballot(last >= 0);
    result = m2 ? __shfl(last, 63 - __clzll((long long)m2)) : min(vocab - 1, c * CHUNK_TOK);
  }
  if (lane == 0) { accept_len[seq] = stop; bonus_token[seq] = result; }
}

// ---------------------------------------------------------------------------------------
// Selective verification (Sec. 4.3, Eq. 5), pass 1: per (row, segment) of the drafter's logits the
// maximum, the lowest index holding it, and the sum of exp((x - max) / T) - the draft token and
// what its probability needs, in one pass with the segment held in registers.
//   grid (segments, rows); part_val/part_idx/part_sum [rows][segments]
// ---------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(ACC_BLOCK) void draft_stats_partial_kernel(
    const T* __restrict__ logits, long long row_stride, int vocab, int seg_len, float inv_t,
    float* __restrict__ part_val, int* __restrict__ part_idx, double* __restrict__ part_sum) {
  const int seg = blockIdx.x, row = blockIdx.y, nseg = gridDim.x;
  const T* rp = logits + (long long)row * row_stride;
  const bool vec_ok = (reinterpret_cast<uintptr_t>(rp) & 15) == 0;
  const int e0 = seg * seg_len;
  const int e1 = min(vocab, e0 + min(seg_len, ARG_SEG_MAX));
  __shared__ float sv[ACC_BLOCK / FD_WAVE]; __shared__ int si[ACC_BLOCK / FD_WAVE];
  __shared__ double sd[ACC_BLOCK / FD_WAVE];
  float x[ARG_ROUNDS][8];
#pragma unroll
  for (int u = 0; u < ARG_ROUNDS; ++u) load8<T>(rp, e0 + (u * ACC_BLOCK + threadIdx.x) * 8, e1, vec_ok, x[u]);   // -inf past e1
  float m = -INFINITY;
#pragma unroll
  for (int u = 0; u < ARG_ROUNDS; ++u)
#pragma unroll
    for (int i = 0; i < 8; ++i) m = fmaxf(m, x[u][i]);
  const float wm = wave_max(m);
  if ((threadIdx.x & 63) == 0) sv[threadIdx.x >> 6] = wm;
  __syncthreads();
  float M = sv[0];
#pragma unroll
  for (int w = 1; w < ACC_BLOCK / FD_WAVE; ++w) M = fmaxf(M, sv[w]);
  int bi = 0x7fffffff;
  float part = 0.f;
  if (M > -INFINITY) {
    if (m == M) {                                            // few threads hold the maximum: only they look for it
#pragma unroll
      for (int u = ARG_ROUNDS - 1; u >= 0; --u)
#pragma unroll
        for (int i = 7; i >= 0; --i)                         // descending walk: the lowest index is kept
          if (x[u][i] == M) bi = e0 + (u * ACC_BLOCK + threadIdx.x) * 8 + i;   // padding is -inf, never equal
    }
    // The terms are summed relative to the segment's maximum, so the term of the maximum is exactly
    // 1 and every other term's rounding error (|y| * 2^-23 of itself, y = (x - M) / T <= 0) is
    // weighted by its own small size: the plain hardware exp2 is accurate enough here, and the pass
    // stays below the cost of the memory traffic.
    const float c = inv_t * 1.44269502e+00f;
#pragma unroll
    for (int u = 0; u < ARG_ROUNDS; ++u)
#pragma unroll
      for (int i = 0; i < 8; ++i) part += __builtin_amdgcn_exp2f((x[u][i] - M) * c);   // padding: 2^-inf = 0
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) bi = min(bi, __shfl_xor(bi, off));
  const double ws = wave_sum((double)part);
  if ((threadIdx.x & 63) == 0) { si[threadIdx.x >> 6] = bi; sd[threadIdx.x >> 6] = ws; }
  __syncthreads();
  if (threadIdx.x == 0) {
    double tot = 0.0;
#pragma unroll
    for (int w = 0; w < ACC_BLOCK / FD_WAVE; ++w) { bi = min(bi, si[w]); tot += sd[w]; }
    const long long o = (long long)row * nseg + seg;
    part_val[o] = M; part_idx[o] = bi; part_sum[o] = tot;
  }
}

// ---------------------------------------------------------------------------------------
// Selective verification, pass 2: one work-group per sequence, DS_GROUP lanes per row, sixteen rows
// at a time.  A lane group merges its row's segments into the draft token and its probability
// p = 1 / sum_v exp((x_v - max) / T); thread 0 then walks the rows in order with the running
// product of the probabilities and counts the positions whose product is still at or above the
// threshold (Eq. 5); the first one below it ends the count.
// ---------------------------------------------------------------------------------------
constexpr int DS_GROUP = 16;
constexpr int DS_ROWS = ACC_BLOCK / DS_GROUP;

__global__ __launch_bounds__(ACC_BLOCK) void draft_select_epilogue_kernel(
    const float* __restrict__ part_val, const int* __restrict__ part_idx, const double* __restrict__ part_sum,
    int nseg, float inv_t, float threshold, const int* __restrict__ row_indptr, int total_rows, int max_rows_per_seq,
    int* __restrict__ draft_tokens, float* __restrict__ confidence, int* __restrict__ keep_len) {
  const int seq = blockIdx.x, grp = threadIdx.x / DS_GROUP, gl = threadIdx.x % DS_GROUP;
  const int r0 = clampi(row_indptr[seq], 0, total_rows);
  const int k = clampi(row_indptr[seq + 1] - r0, 0, min(max_rows_per_seq, total_rows - r0));
  __shared__ double s_p[DS_ROWS];
  double prod = 1.0;
  int keep = 0;
  bool open = true;
  for (int j0 = 0; j0 < k; j0 += DS_ROWS) {                  // k is uniform over the group
    const int j = min(j0 + grp, k - 1);                      // surplus lane groups repeat the last row, unwritten
    const long long base = (long long)(r0 + j) * nseg;
    float m = -INFINITY;
    for (int s = gl; s < nseg; s += DS_GROUP) m = fmaxf(m, part_val[base + s]);
#pragma unroll
    for (int off = DS_GROUP / 2; off >= 1; off >>= 1) m = fmaxf(m, __shfl_xor(m, off));
    int bi = 0x7fffffff; double z = 0.0;
    for (int s = gl; s < nseg; s += DS_GROUP) {
      const float v = part_val[base + s];
      if (v == m) bi = min(bi, part_idx[base + s]);
      if (v > -INFINITY) z += part_sum[base + s] * (double)exp_neg((v - m) * inv_t);
    }
#pragma unroll
    for (int off = DS_GROUP / 2; off >= 1; off >>= 1) {
      bi = min(bi, __shfl_xor(bi, off));
      z += __shfl_xor(z, off);
    }
    const double pj = z > 0.0 ? 1.0 / z : 0.0;
    if (gl == 0 && j0 + grp < k) {
      draft_tokens[r0 + j] = bi == 0x7fffffff ? -1 : bi;
      if (confidence) confidence[r0 + j] = (float)pj;
      s_p[grp] = pj;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      const int nrow = min(DS_ROWS, k - j0);
      for (int i = 0; i < nrow; ++i) {
        prod *= s_p[i];
        if (open && prod >= (double)threshold) ++keep; else open = false;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) keep_len[seq] = keep;
}

// ---------------------------------------------------------------------------------------
// Branch selection (Sec. 3, parallel speculative decoding): one wave per sequence copies the
// block drafted under the number of accepted drafts that verification arrived at.
// ---------------------------------------------------------------------------------------
__global__ __launch_bounds__(FD_WAVE) void select_branch_kernel(
    const int* __restrict__ block_tokens, const int* __restrict__ block_indptr, const int* __restrict__ mask_blocks,
    const int* __restrict__ accept_len, const int* __restrict__ first_vis, const int* __restrict__ verify_len,
    int total_tokens, int out_stride, int* __restrict__ out_tokens, int* __restrict__ out_block) {
  const int seq = blockIdx.x, lane = threadIdx.x;
  const int t0 = clampi(block_indptr[seq], 0, total_tokens);
  const int len = clampi(block_indptr[seq + 1] - t0, 0, total_tokens - t0);
  const int nb = mask_blocks[seq];
  int* o = out_tokens + (long long)seq * out_stride;
  const bool ok = nb >= 1 && len % (nb >= 1 ? nb : 1) == 0 && len / (nb >= 1 ? nb : 1) <= out_stride;
  const int mb = ok ? len / nb : 0;
  int b = -1;
  if (ok) {
    // without first_vis: the attention call's own default, the last block sees every verify row
    const int fv = first_vis ? first_vis[seq] : max(verify_len[seq] - nb + 1, 0);
    b = accept_len[seq] + 1 - fv;
    b = clampi(b, 0, nb - 1);
  }
  for (int j = lane; j < out_stride; j += FD_WAVE) o[j] = j < mb ? block_tokens[t0 + b * mb + j] : -1;
  if (out_block && lane == 0) out_block[seq] = b;
}

hipError_t run_select_branch(const int* block_tokens, const int* block_indptr, const int* mask_blocks,
                             const int* accept_len, const int* first_vis, const int* verify_len, int batch,
                             int total_tokens, int out_stride, int* out_tokens, int* out_block, hipStream_t st) {
  hipLaunchKernelGGL(select_branch_kernel, dim3(batch), dim3(FD_WAVE), 0, st, block_tokens, block_indptr,
                     mask_blocks, accept_len, first_vis, verify_len, total_tokens, out_stride, out_tokens, out_block);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------
// host-side launchers (called from api.hip)
// ---------------------------------------------------------------------------------------
static inline int pick_segments(int rows, int vocab) {
  // Around 2048 work-groups in all, each taking a whole number of rounds (ACC_BLOCK * 8 logits, one
  // 16-byte load per lane): at least two rounds, so that a group has 4096 logits to work on, and
  // never more than the passes hold in registers.
  int want = (2048 + rows - 1) / (rows > 0 ? rows : 1);
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  const long long round_len = (long long)ACC_BLOCK * 8;
  long long r = (vocab + want * round_len - 1) / (want * round_len);
  if (r < 2) r = 2;
  if (r > ARG_ROUNDS) r = ARG_ROUNDS;
  long long s = (vocab + r * round_len - 1) / (r * round_len);
  return (int)(s < 1 ? 1 : s);
}
static inline int seg_len_for(int vocab, int nseg) {
  int l = (vocab + nseg - 1) / nseg;
  return (l + 7) / 8 * 8;
}

// Sampling workspace layout (all blocks 256-byte aligned), shared by the size query and the launcher.
struct SampleLayout {
  size_t part, row_stats, chunk_res, chunk_p, decision, total;
  int nseg, nchunks;
};
static inline size_t align256(size_t x) { return (x + 255) / 256 * 256; }
static inline SampleLayout sample_layout(int batch, int total_rows, int vocab) {
  SampleLayout l;
  size_t rows = (size_t)(total_rows > 0 ? total_rows : 1), seqs = (size_t)(batch > 0 ? batch : 1);
  l.nseg = pick_segments(total_rows, vocab);
  l.nchunks = (vocab + CHUNK_TOK - 1) / CHUNK_TOK;
  size_t off = 0;
  l.part = off;      off += align256(rows * l.nseg * 4 * sizeof(double));
  l.row_stats = off; off += align256(seqs * 4 * sizeof(double));
  l.chunk_res = off; off += align256(seqs * l.nchunks * sizeof(double));
  l.chunk_p = off;   off += align256(seqs * l.nchunks * sizeof(double));
  l.decision = off;  off += align256(seqs * 4 * sizeof(int));
  l.total = off;
  return l;
}

size_t accept_workspace_bytes(int batch, int total_rows, int vocab, int sampling) {
  if (batch < 0 || total_rows < 0 || vocab <= 0) return 0;
  if (sampling) return sample_layout(batch, total_rows, vocab).total;
  size_t rows = (size_t)(total_rows > 0 ? total_rows : 1);
  return align256(rows * pick_segments(total_rows, vocab) * (sizeof(float) + sizeof(int)));
}

template <typename T>
static hipError_t launch_greedy(const T* logits, long long row_stride, int vocab, const int* row_indptr,
                                const int* toks, int batch, int total_rows, int max_rows, int* accept_len,
                                int* bonus, int* row_argmax, void* ws, hipStream_t st) {
  int nseg = pick_segments(total_rows, vocab);
  int sl = seg_len_for(vocab, nseg);
  float* pv = reinterpret_cast<float*>(ws);
  int* pi = reinterpret_cast<int*>(pv + (size_t)(total_rows > 0 ? total_rows : 1) * nseg);
  if (total_rows > 0)
    hipLaunchKernelGGL(argmax_partial_kernel<T>, dim3(nseg, total_rows), dim3(ACC_BLOCK), 0, st,
                       logits, row_stride, vocab, sl, pv, pi);
  if (batch > 0)
    hipLaunchKernelGGL(accept_greedy_epilogue_kernel, dim3(batch), dim3(ACC_BLOCK), 0, st,
                       pv, pi, nseg, row_indptr, toks, total_rows, max_rows, accept_len, bonus, row_argmax);
  return hipGetLastError();
}

template <typename T>
static hipError_t launch_sample(const T* target, const T* draft, long long row_stride, int vocab, float temperature,
                                const int* row_indptr, const int* toks, const float* ua, const float* ur,
                                int batch, int total_rows, int max_rows, int* accept_len, int* bonus,
                                void* ws, hipStream_t st) {
  const SampleLayout lay = sample_layout(batch, total_rows, vocab);
  const int nseg = lay.nseg, nchunks = lay.nchunks;
  const int sl = seg_len_for(vocab, nseg);
  char* base = reinterpret_cast<char*>(ws);
  double* part = reinterpret_cast<double*>(base + lay.part);
  double* row_stats = reinterpret_cast<double*>(base + lay.row_stats);
  double* chunk_res = reinterpret_cast<double*>(base + lay.chunk_res);
  double* chunk_p = reinterpret_cast<double*>(base + lay.chunk_p);
  int* decision = reinterpret_cast<int*>(base + lay.decision);
  float inv_t = 1.0f / temperature;
  if (total_rows > 0)
    switch ((sl + ACC_BLOCK * 8 - 1) / (ACC_BLOCK * 8)) {        // rounds that cover a segment (<= ARG_ROUNDS)
#define FD_STATS_CASE(NR)                                                                                          \
      case NR: hipLaunchKernelGGL((softmax_stats_partial_kernel<T, NR>), dim3(nseg, total_rows), dim3(ACC_BLOCK), 0, st, \
                                  target, draft, row_stride, vocab, sl, inv_t, part); break;
      FD_STATS_CASE(1) FD_STATS_CASE(2) FD_STATS_CASE(3) FD_STATS_CASE(4)
      default: hipLaunchKernelGGL((softmax_stats_partial_kernel<T, ARG_ROUNDS>), dim3(nseg, total_rows), dim3(ACC_BLOCK), 0, st,
                                  target, draft, row_stride, vocab, sl, inv_t, part); break;
#undef FD_STATS_CASE
    }
  if (batch > 0) {
    int groups = (nchunks + (ACC_BLOCK / FD_WAVE) - 1) / (ACC_BLOCK / FD_WAVE);
    int want = (1024 + batch - 1) / batch;
    if (groups > want) groups = want;
    if (groups < 1) groups = 1;
    hipLaunchKernelGGL(accept_sample_weights_kernel<T>, dim3(groups, batch), dim3(ACC_BLOCK), 0, st,
                       target, draft, row_stride, vocab, inv_t, part, nseg, row_indptr, toks, ua,
                       total_rows, max_rows, nchunks, decision, row_stats, chunk_res, chunk_p);
    hipLaunchKernelGGL(accept_sample_pick_kernel<T>, dim3(batch), dim3(ACC_BLOCK), 0, st,
                       target, draft, row_stride, vocab, inv_t, row_indptr, ur, total_rows, nchunks,
                       decision, row_stats, chunk_res, chunk_p, accept_len, bonus);
  }
  return hipGetLastError();
}

size_t draft_select_workspace_bytes(int total_rows, int vocab) {
  const size_t slots = (size_t)(total_rows > 0 ? total_rows : 1) * pick_segments(total_rows, vocab);
  return align256(slots * sizeof(float)) + align256(slots * sizeof(int)) + align256(slots * sizeof(double));
}

template <typename T>
static hipError_t launch_draft_select(const T* logits, long long row_stride, int vocab, float temperature, float threshold,
                                      const int* row_indptr, int batch, int total_rows, int max_rows, int* tokens,
                                      float* confidence, int* keep_len, void* ws, hipStream_t st) {
  const int nseg = pick_segments(total_rows, vocab);
  const int sl = seg_len_for(vocab, nseg);
  const size_t slots = (size_t)(total_rows > 0 ? total_rows : 1) * nseg;
  char* base = reinterpret_cast<char*>(ws);
  float* pv = reinterpret_cast<float*>(base);
  int* pi = reinterpret_cast<int*>(base + align256(slots * sizeof(float)));
  double* pd = reinterpret_cast<double*>(base + align256(slots * sizeof(float)) + align256(slots * sizeof(int)));
  const float inv_t = 1.0f / temperature;
  if (total_rows > 0)
    hipLaunchKernelGGL(draft_stats_partial_kernel<T>, dim3(nseg, total_rows), dim3(ACC_BLOCK), 0, st,
                       logits, row_stride, vocab, sl, inv_t, pv, pi, pd);
  if (batch > 0)
    hipLaunchKernelGGL(draft_select_epilogue_kernel, dim3(batch), dim3(ACC_BLOCK), 0, st, pv, pi, pd, nseg, inv_t,
                       threshold, row_indptr, total_rows, max_rows, tokens, confidence, keep_len);
  return hipGetLastError();
}

hipError_t run_draft_select(const void* logits, int dt, long long row_stride, int vocab, float temperature,
                            float threshold, const int* row_indptr, int batch, int total_rows, int max_rows,
                            int* tokens, float* confidence, int* keep_len, void* ws, hipStream_t st) {
  if (dt == FD_BF16)
    return launch_draft_select<bf16_t>((const bf16_t*)logits, row_stride, vocab, temperature, threshold, row_indptr,
                                       batch, total_rows, max_rows, tokens, confidence, keep_len, ws, st);
  return launch_draft_select<float>((const float*)logits, row_stride, vocab, temperature, threshold, row_indptr,
                                    batch, total_rows, max_rows, tokens, confidence, keep_len, ws, st);
}

hipError_t run_accept_greedy(const void* logits, int dt, long long row_stride, int vocab, const int* row_indptr,
                             const int* toks, int batch, int total_rows, int max_rows, int* accept_len,
                             int* bonus, int* row_argmax, void* ws, hipStream_t st) {
  if (dt == FD_BF16)
    return launch_greedy<bf16_t>((const bf16_t*)logits, row_stride, vocab, row_indptr, toks, batch, total_rows,
                                 max_rows, accept_len, bonus, row_argmax, ws, st);
  return launch_greedy<float>((const float*)logits, row_stride, vocab, row_indptr, toks, batch, total_rows,
                              max_rows, accept_len, bonus, row_argmax, ws, st);
}

hipError_t run_accept_sample(const void* target, const void* draft, int dt, long long row_stride, int vocab,
                             float temperature, const int* row_indptr, const int* toks, const float* ua,
                             const float* ur, int batch, int total_rows, int max_rows, int* accept_len,
                             int* bonus, void* ws, hipStream_t st) {
  if (dt == FD_BF16)
    return launch_sample<bf16_t>((const bf16_t*)target, (const bf16_t*)draft, row_stride, vocab, temperature,
                                 row_indptr, toks, ua, ur, batch, total_rows, max_rows, accept_len, bonus, ws, st);
  return launch_sample<float>((const float*)target, (const float*)draft, row_stride, vocab, temperature,
                              row_indptr, toks, ua, ur, batch, total_rows, max_rows, accept_len, bonus, ws, st);
}

}  // namespace fd
