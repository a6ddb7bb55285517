// Hybrid-mask verify+draft attention (Sec. 4.1), bf16 MFMA kernel for gfx950, head_dim 128.
//
// One work-group of four waves owns one (sequence, KV head, KV chunk, 128-tile-row block)
// and streams the chunk's keys and values 64 tokens at a time:
//
//   global --16-byte coalesced loads, one page slab per instruction--> registers
//          --> LDS (double buffered, one barrier per tile)
//   S^T = K Q^T        v_mfma_f32_32x32x16_bf16, A = K rows from LDS (ds_read_b128),
//                      B = Q fragments held in registers for the whole kernel
//   online softmax     in the accumulator layout: a lane owns ONE query row (column of
//                      S^T) and 16 of each 32 keys, so the row maximum needs one exchange
//                      with lane^32 and the row sum none until the end
//   O^T += V^T P^T     A = V^T fragments fetched with ds_read_b64_tr_b16 (the LDS transpose
//                      read of gfx950), B = P packed to bf16 straight from the S^T registers
//
// A tile row is (new row, query head of the group); wave w owns tile rows 32w..32w+31, so
// K and V are read from HBM once for all rows and all G heads of the KV head.  The cached
// prefix is unmasked (every new row sees all of it); only the ragged last tile and the
// tile of new rows apply the visibility rule, in registers.  Each work-group leaves split
// partials (base-2 running max, sum, un-normalised O) for the combine kernel.
#include "fd_common.h"

namespace fd {

constexpr int MF_BLOCK = 256;
constexpr int MF_TK = 64;                 // keys per LDS tile
constexpr int MF_D = 128;
constexpr int MF_ROWS = 128;              // tile rows per work-group
constexpr int MF_KSTR = MF_D + 8;         // LDS row pitch in bf16 elements (272 bytes)
constexpr int MF_VSTR = MF_D + 8;
constexpr int MF_TILE_ELEMS = MF_TK * MF_KSTR;
constexpr size_t MF_LDS_BYTES = (size_t)2 * 2 * MF_TILE_ELEMS * sizeof(bf16_t);   // K,V x 2 buffers

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

struct TileRegs { u32x4 k[4]; u32x4 v[4]; };

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);      // round to nearest even
  return __builtin_bit_cast(unsigned, b);
}

__global__ __launch_bounds__(MF_BLOCK, 2) void attn_mfma_kernel(AttnParams p) {
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];
  bf16_t* Ks = lds;                             // [2][MF_TK][MF_KSTR]
  bf16_t* Vs = lds + 2 * MF_TILE_ELEMS;         // [2][MF_TK][MF_VSTR]

  const int chunk_id = blockIdx.x;
  const int g = blockIdx.y % p.Hkv, rt = blockIdx.y / p.Hkv;
  const int seq = blockIdx.z;
  const SeqInfo s = load_seq(p, seq);
  const int nchunks = max(1, (s.L + p.chunk - 1) / p.chunk);
  const int rows_total = s.n * p.G;
  if (chunk_id >= nchunks || rt * MF_ROWS >= rows_total) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = lane >> 5, c32 = lane & 31, l16 = lane & 15;
  const bf16_t* Kc = reinterpret_cast<const bf16_t*>(p.k_cache);
  const bf16_t* Vc = reinterpret_cast<const bf16_t*>(p.v_cache);
  const bf16_t* Kn = reinterpret_cast<const bf16_t*>(p.k_new);
  const bf16_t* Vn = reinterpret_cast<const bf16_t*>(p.v_new);

  // ---- this lane's query row -----------------------------------------------------------
  const int T_row = rt * MF_ROWS + wave * 32 + c32;
  const bool row_valid = T_row < rows_total;
  const bool wave_active = (rt * MF_ROWS + wave * 32) < rows_total;
  const int nn = T_row / p.G;                                   // new-row index within the sequence
  const int hq = g * p.G + T_row % p.G;
  bf16x8 qf[8];
  {
    const bf16_t* qp = reinterpret_cast<const bf16_t*>(p.q) + ((long long)(s.row0 + (row_valid ? nn : 0)) * p.Hq + hq) * MF_D + 8 * h;
#pragma unroll
    for (int st = 0; st < 8; ++st) {
      u32x4 w = {0u, 0u, 0u, 0u};
      if (row_valid) w = *reinterpret_cast<const u32x4*>(qp + 16 * st);
      qf[st] = as_bf16x8(w);
    }
  }

  // ---- tile schedule -------------------------------------------------------------------
  const int c0 = chunk_id * p.chunk;
  const int c1 = min(s.L, c0 + p.chunk);
  const int n_ct = c1 > c0 ? (c1 - c0 + MF_TK - 1) / MF_TK : 0;
  const int n_nt = (chunk_id == nchunks - 1) ? (s.n + MF_TK - 1) / MF_TK : 0;
  const int NT = n_ct + n_nt;

  const int ld_key = tid >> 4;                 // 0..15: key within a 16-key group
  const int ld_col = (tid & 15) * 8;           // element offset of this thread's 16 bytes

  // physical page of each 16-key group of a cached tile (uniform across the work-group)
  auto fetch_pages = [&](int t, int (&pg)[4]) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int gs = c0 + t * MF_TK + 16 * j;        // first key of the group
      int ph = -1;
      if (t < n_ct && gs < c1) {
        ph = p.page_indices[s.page0 + gs / p.page_size];
        if (ph < 0 || ph >= p.num_pages) { flag_status(p.status, FD_DEV_PAGE_RANGE); ph = -1; }
      }
      pg[j] = ph;
    }
  };

  auto load_tile = [&](int t, const int (&pg)[4], TileRegs& r) {
    const u32x4 z = {0u, 0u, 0u, 0u};
    if (t < n_ct) {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int gs = c0 + t * MF_TK + 16 * j;
        int key = gs + ld_key;
        r.k[j] = z; r.v[j] = z;
        if (pg[j] >= 0 && key < c1) {
          long long off = (long long)pg[j] * p.sp + (long long)g * p.sh +
                          (long long)(gs % p.page_size + ld_key) * p.st + ld_col;
          r.k[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Kc + off));
          r.v[j] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(Vc + off));
        }
      }
    } else {
      int base = (t - n_ct) * MF_TK;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        int key = base + 16 * j + ld_key;
        r.k[j] = z; r.v[j] = z;
        if (key < s.n) {
          long long off = ((long long)(s.row0 + key) * p.Hkv + g) * MF_D + ld_col;
          r.k[j] = *reinterpret_cast<const u32x4*>(Kn + off);
          r.v[j] = *reinterpret_cast<const u32x4*>(Vn + off);
        }
      }
    }
  };

  auto store_tile = [&](int buf, const TileRegs& r) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      int row = 16 * j + ld_key;
      *reinterpret_cast<u32x4*>(Ks + buf * MF_TILE_ELEMS + row * MF_KSTR + ld_col) = r.k[j];
      *reinterpret_cast<u32x4*>(Vs + buf * MF_TILE_ELEMS + row * MF_VSTR + ld_col) = r.v[j];
    }
  };

  // ---- running softmax state: one query row per lane ------------------------------------
  const float cs = p.sm_scale * 1.4426950408889634f;           // scores are kept in base-2 units
  float m_run = -INFINITY, l_lane = 0.f;
  f32x16 o[4];
#pragma unroll
  for (int b = 0; b < 4; ++b)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[b][i] = 0.f;

  int pg[4];
  TileRegs regs;
  fetch_pages(0, pg);
  load_tile(0, pg, regs);
  fetch_pages(1, pg);
  store_tile(0, regs);
  __syncthreads();

  for (int t = 0; t < NT; ++t) {
    const int buf = t & 1;
    if (t + 1 < NT) {
      load_tile(t + 1, pg, regs);
      fetch_pages(t + 2, pg);
    }

    if (wave_active) {
      const bf16_t* Kb = Ks + buf * MF_TILE_ELEMS;
      const bf16_t* Vb = Vs + buf * MF_TILE_ELEMS;
      // ---- S^T = K Q^T : two 32-key blocks ----
      f32x16 sc[2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
        for (int i = 0; i < 16; ++i) sc[kb][i] = 0.f;
        const bf16_t* kp = Kb + (32 * kb + c32) * MF_KSTR + 8 * h;
#pragma unroll
        for (int st = 0; st < 8; ++st) {
          bf16x8 kf = as_bf16x8(*reinterpret_cast<const u32x4*>(kp + 16 * st));
          sc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[st], sc[kb], 0, 0, 0);
        }
      }
      // ---- visibility: ragged tail of the cache, or the new-row tile (Sec. 4.1 rules) ----
      const bool is_new = t >= n_ct;
      const int tile_base = is_new ? (t - n_ct) * MF_TK : c0 + t * MF_TK;
      if (is_new || tile_base + MF_TK > c1) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            int key = tile_base + 32 * kb + 8 * (i >> 2) + 4 * h + (i & 3);
            bool vis = is_new ? new_key_visible(nn, key, s.n, s.k, s.v) : (key < c1);
            if (!vis) sc[kb][i] = -INFINITY;
          }
      }
      // ---- online softmax (base 2) ----
      float mx = sc[0][0];
#pragma unroll
      for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sc[0][i]);
#pragma unroll
      for (int i = 0; i < 16; ++i) mx = fmaxf(mx, sc[1][i]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));
      const float m_new = fmaxf(m_run, mx * cs);
      const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;   // row with nothing visible yet
      const float alpha = __builtin_amdgcn_exp2f(m_run - m_sub);
      m_run = m_new;
      if (__any(alpha != 1.f)) {
        l_lane *= alpha;
#pragma unroll
        for (int b = 0; b < 4; ++b)
#pragma unroll
          for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
      }
      unsigned pk[2][8];                                         // P^T as packed bf16 pairs
#pragma unroll
      for (int kb = 0; kb < 2; ++kb) {
        float pr[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          pr[i] = __builtin_amdgcn_exp2f(fmaf(sc[kb][i], cs, -m_sub));
          l_lane += pr[i];
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) pk[kb][i] = pack_bf16x2(pr[2 * i], pr[2 * i + 1]);
      }
      // ---- O^T += V^T P^T ----
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          u32x4 pw = {pk[kb][4 * j], pk[kb][4 * j + 1], pk[kb][4 * j + 2], pk[kb][4 * j + 3]};
          const bf16x8 pf = as_bf16x8(pw);
          // keys of this k-step for lane-half h: base+4h+{0..3} and base+8+4h+{0..3}
          const bf16_t* vp = Vb + (32 * kb + 16 * j + 4 * h + (l16 >> 2)) * MF_VSTR + 16 * (c32 >> 4) + 4 * (l16 & 3);
#pragma unroll
          for (int b = 0; b < 4; ++b) {
            s16x4 v1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 32 * b));
            s16x4 v2 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 32 * b + 8 * MF_VSTR));
            typedef __attribute__((ext_vector_type(8))) short s16x8;
            s16x8 vv = {v1[0], v1[1], v1[2], v1[3], v2[0], v2[1], v2[2], v2[3]};
            o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), pf, o[b], 0, 0, 0);
          }
        }
    }

    if (t + 1 < NT) store_tile(buf ^ 1, regs);
    __syncthreads();
  }

  // ---- split partial: (m, l, O) per (chunk, row, head) ---------------------------------
  if (wave_active) {
    const float l_tot = l_lane + __shfl_xor(l_lane, 32);
    if (row_valid) {
      const long long slot = ((long long)chunk_id * p.total_rows + (s.row0 + nn)) * p.Hq + hq;
      float* ap = p.part_acc + slot * MF_D + 4 * h;
#pragma unroll
      for (int b = 0; b < 4; ++b)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          f32x4 w = {o[b][4 * a], o[b][4 * a + 1], o[b][4 * a + 2], o[b][4 * a + 3]};
          *reinterpret_cast<f32x4*>(ap + 32 * b + 8 * a) = w;
        }
      if (h == 0) { p.part_ml[slot * 2] = m_run; p.part_ml[slot * 2 + 1] = l_tot; }
    }
  }
}

size_t attn_mfma_lds_bytes() { return MF_LDS_BYTES; }

hipError_t run_attn_mfma(const AttnParams& p, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)MF_LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  dim3 grid(p.max_chunks, p.Hkv * p.row_tiles, p.B);
  hipLaunchKernelGGL(attn_mfma_kernel, grid, dim3(MF_BLOCK), MF_LDS_BYTES, st, p);
  return hipGetLastError();
}

}  // namespace fd
