// Hybrid-mask verify+draft attention (Sec. 4.1), bf16 MFMA kernel for gfx950, head_dim 128 or 64.
//
// Work decomposition.  An *item* is one (sequence, KV head, block of up to ROWS_WG tile
// rows); a tile row is (new row, query head of the group), so K and V are read from HBM once
// for all rows and all G heads of the KV head.  An item consists of ceil(L/64) tiles of 64
// cached keys followed by the tile(s) of the sequence's own new rows.  All tiles of all
// items, in (sequence, head, row block) order, form one line of work that is cut into equal
// shares, one per persistent work-group (two work-groups per CU), so that every CU streams
// the same number of bytes whatever the length mix of the batch.  A share is walked as a
// sequence of *pieces* (runs of tiles inside one item).  A piece that covers a whole item is
// normalised and stored; an item cut by a share boundary leaves one split partial (base-2
// running max, sum, un-normalised O as fp16 rows scaled by their largest entry) per work-group
// that touched it, and the work-group in which it ends leaves an entry for the combine kernel below.
//
// Where a share starts (sequence, offset, the page ids of its first two tiles) depends on the
// lengths only, so it can be found ahead of time by the planning kernel, once for every layer of a
// decoding step; the streaming kernel then starts from its plan entry -- one scalar load, then
// tiles are requested -- instead of scanning the batch itself.
//
// Streaming of one tile by the four waves of a work-group:
//   page ids           scalar loads, one tile ahead (they are uniform across the work-group)
//   global -> regs     one 16-key group per wave (a 4 KB K slab and a 4 KB V slab of one page at head
//                      dim 128), buffer_load_dwordx4 through a buffer descriptor built in scalar
//                      registers: no per-lane address arithmetic, and rows past the end of the
//                      prefix lie outside the descriptor and read as zero.  Two tiles are held
//                      in registers while a third is multiplied.
//   regs -> LDS        double buffered, K rows padded by 16 B, V rows by 64 B (272 / 320 B at head dim 128),
//                      one barrier per tile
//   S^T = K Q^T        v_mfma_f32_32x32x16_bf16, A = K rows from LDS (ds_read_b128),
//                      B = Q fragments held in registers for the whole item
//   online softmax     in the accumulator layout: a lane owns ONE query row (column of
//                      S^T) and 16 of each 32 keys, so the row maximum needs one exchange
//                      with lane^32 and the row sum none until the end
//   O^T += V^T P^T     A = V^T fragments fetched with ds_read_b64_tr_b16 (the LDS transpose
//                      read of gfx950), B = P packed to bf16 straight from the S^T registers
// The next piece's page ids are requested before the current piece's tile loop, its first two
// tiles and query rows before the current piece is merged and stored.
//
// Wave roles.  64-row variant: the tile rows in use form RB = 1 or 2 blocks of 32; wave w takes
// row block w % RB and, of each tile's two 32-key blocks, the one with index w / RB; waves that
// shared a row block merge their running (max, sum, O) through LDS at the end of the piece.
// 128-row variant: wave w owns row block w and every key block, no merge.
//
// The cached prefix is unmasked (every new row sees all of it, Sec. 4.1); only the ragged
// last tile and the tile of new rows apply the visibility rule, in registers.
#include "fd_common.h"
#include <atomic>
#include <type_traits>

// MFMAs by which the LDS fragment requests of S = K Q^T and O += V^T P^T run ahead of their use
// (3 and 3: measured best of 2..4; more costs registers the 64-row variant does not have)
#ifndef FD_PF_K
#define FD_PF_K 3
#endif
#ifndef FD_PF_V
#define FD_PF_V 3
#endif

namespace fd {

constexpr int MF_BLOCK = 256;
constexpr int MF_TK = 64;                 // keys per LDS tile
constexpr int MF_D_MAX = 128;             // head dims taken: 128 and 64
#ifndef FD_XCDS
#define FD_XCDS 8                         // accelerator dies of an MI355X; work-groups are dealt to them round-robin
#endif
#ifndef FD_WGS_PER_CU
#define FD_WGS_PER_CU 2                   // persistent work-groups per compute unit (two fit: registers and LDS)
#endif
#ifndef FD_DEFER_T1
#define FD_DEFER_T1 1
#endif
#ifndef FD_KPAD
#define FD_KPAD 8
#endif
#ifndef FD_VPAD
#define FD_VPAD 32
#endif
// LDS layout for head dim DH.  K rows are padded by 16 bytes (pitch 272 B for DH = 128, 144 B for 64: an odd
// number of 16-byte slots, so the 16 rows a ds_read_b128 touches at once fall into 16 different slots) and
// V rows by 64 bytes (pitch 320 / 192 B: four consecutive rows start 64 B apart modulo 256, so the 4 rows x 64 B
// of a transposing read cover every bank once; counter-checked for 128, where a 288 B pitch costs 2 cycles per read).
template <int DH> struct MfLds {
  static constexpr int KSTR = DH + FD_KPAD;                // K row pitch in bf16 elements
  static constexpr int VSTR = DH + FD_VPAD;                // V row pitch
  static constexpr int K_ELEMS = MF_TK * KSTR;
  static constexpr int V_ELEMS = MF_TK * VSTR;
  static constexpr int BUF_ELEMS = K_ELEMS + V_ELEMS;      // one K+V tile
  static constexpr size_t BYTES = (size_t)2 * BUF_ELEMS * sizeof(bf16_t);   // double buffered
};
constexpr int MF_BLOCKS = MF_TK / 32;     // 32-key MFMA blocks per tile
constexpr int MF_GROUPS = MF_TK / 16;     // 16-key load groups per tile
constexpr int MF_XCD_TILT = 40;           // per mille of a share that every share of an odd XCD hands to the even XCD before it
constexpr int MF_TILT_MIN_SHARE = 64;     // ... in launches whose shares are at least this many units long
constexpr float MF_LAZY = 6.f;            // the softmax reference follows the row maximum in steps of at least 2^6
// What starting an item costs a work-group, in tile times: measured ≈ 6.9 µs (request the next piece's
// tiles ≈ 2.4, merge and store ≈ 3.4, wait for the first tile ≈ 1.1) against 2.1 µs per tile in the
// 64-row variant, about half as many of the longer tiles of the 128-row variant.
constexpr int mf_start_cost(int maxrb) { return maxrb == 4 ? 2 : 4; }

typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

template <int NLD> struct TileRegsT { u32x4 k[NLD]; u32x4 v[NLD]; };      // one wave's 16-key group of a tile: NLD loads per tensor

// Launch-time scheduling parameters and the split-partial storage.
struct MfmaSched {
  int page_shift;
  int group_shift;    // log2(query heads per KV head), -1 if that is not a power of two
  int num_wgs;        // persistent work-groups launched
  int xcds;           // work-group x runs on XCD x % xcds (1: no such structure is assumed)
  int reuse;          // != 0: some sequence has several row blocks, i.e. its K/V tiles are read by several items
  int min_share;      // automatic shares are never smaller than this many tiles
  int fixed_share;    // > 0: tiles per work-group asked for by the caller
  unsigned short* part_acc;   // [2 * num_wgs][ROWS_WG][D] fp16: the un-normalised output row divided by its largest magnitude
  float* part_ml;             // [2 * num_wgs][ROWS_WG][4]: running maximum (base 2), row sum, that largest magnitude, unused
  int4* entries;      // [num_wgs + 1]: entry w: the split item that ends in the work-group of share w: (first packed row, head | row block << 16, tile rows, first slot); first < 0: none.  Entry num_wgs: (shares in use, -, -, -)
  struct PlanEntry* plan;     // [num_wgs]: written by the planning kernel, read by a planned streaming kernel
};

// What the planning kernel leaves for each persistent work-group (128 bytes, read through the scalar path).
struct PlanEntry {
  int seq;                    // sequence in which the share starts; < 0: nothing to do
  unsigned Pt;                // units of the line before that sequence
  unsigned g0, g1;            // the share: units [g0, g1) of the line
  int L, row0, n, k, v, nb, page0, npages;     // that sequence, clamped as load_seq clamps it
  unsigned sh_q, sh_r;        // share w starts at unit w sh_q + floor(w sh_r / W_eff)
  int W_eff;                  // shares in use (valid in every entry, also those without a share)
  int share;                  // which share this work-group takes
  int pg0[MF_GROUPS], pg1[MF_GROUPS];          // page ids of the first two tiles of the share's first piece
  int pad1[8];
};
static_assert(sizeof(PlanEntry) == 128, "one plan entry is 128 bytes");

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 x) { return __builtin_bit_cast(bf16x8, x); }

__device__ __forceinline__ unsigned pack_bf16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  f32x2 f = {lo, hi};
  bf16x2 b = __builtin_convertvector(f, bf16x2);      // round to nearest even
  return __builtin_bit_cast(unsigned, b);
}

__device__ __forceinline__ unsigned pack_f16x2(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
  typedef __attribute__((ext_vector_type(2))) float f32x2;
  f32x2 f = {lo, hi};
  f16x2 b = __builtin_convertvector(f, f16x2);        // round to nearest even
  return __builtin_bit_cast(unsigned, b);
}
__device__ __forceinline__ void unpack_f16x4(u32x2 w, float (&x)[4]) {
  typedef __attribute__((ext_vector_type(4))) _Float16 f16x4;
  const f16x4 hv = __builtin_bit_cast(f16x4, w);
#pragma unroll
  for (int e = 0; e < 4; ++e) x[e] = (float)hv[e];
}

// Tiles of one item of this sequence, and how many items (heads x row blocks) it has.
__device__ __forceinline__ void seq_shape(const AttnParams& p, const SeqInfo& s, int rows_wg, int& tiles, int& items) {
  if (s.n <= 0) { tiles = 0; items = 0; return; }
  tiles = (s.L + MF_TK - 1) / MF_TK + (s.n + MF_TK - 1) / MF_TK;
  items = p.Hkv * ((s.n * p.G + rows_wg - 1) / rows_wg);
}

// Work units of one item with `tiles` tiles.  The line of work is cut into shares of equal
// *time*, not of equal tile count: beginning an item (new query rows, new page list, the merge
// and the stores of the one before) costs about as much as streaming two tiles, so every item is
// preceded by `start_cost` units that stand for no tile.  A work-group whose share holds an
// item boundary gets that many tiles less.
__device__ __forceinline__ int item_units(int tiles, int start_cost) { return tiles > 0 ? tiles + start_cost : 0; }

// A 64-bit value known to be equal in every lane, moved to scalar registers.
__device__ __forceinline__ long long uniform_ll(long long v) {
  unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)(v & 0xffffffffll));
  unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)((unsigned long long)v >> 32));
  return (long long)(((unsigned long long)hi << 32) | lo);
}

__device__ __forceinline__ int wave_incl_scan(int v, int lane) {
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) { int o = __shfl_up(v, off); if (lane >= off) v += o; }
  return v;
}

// Where work-group w's share of the line starts.  Every thread of the work-group calls this; the
// results are uniform.  Tile counts fit 32 bits (the host checks the bound), so no 64-bit division
// is needed.  share w = [w q + floor(w r / W), ...) with q, r = total / W, total % W: equal to
// floor(w total / W).  Returns false if the work-group has nothing to do (W_eff is valid either way).
//
// Which share a work-group takes is XCD-aware.  Work-group x of a launch runs on XCD x % 8, each XCD
// has an L2 of its own, and neighbouring shares of the line often read the same K/V tiles at the same
// time: the row blocks of one (sequence, KV head) -- items that follow each other on the line -- start
// together and advance in step.  So the work-groups of one XCD take a CONTIGUOUS run of shares:
// work-group pw takes share (pw % xcds) * chunk + pw / xcds with chunk = ceil(W_eff / xcds), and the
// second reader of a tile finds it in its XCD's L2.
//
// The XCDs do not stream at one rate: with every one of them reading its equal part of a long batch, the
// odd-numbered ones (blockIdx.x odd) finish about 7 % after the even-numbered ones, launch after launch and
// whichever shares they are given (measured with per-work-group timestamps; whether the two XCDs of a
// pair share a port to the memory fabric is a guess).  So, on top of the equal cut floor(w total / W),
// every share of an odd XCD's run hands d = round(MF_XCD_TILT / 1000 of a share) units to the even run
// before it: boundary i of an even run of a shares, followed by an odd run of b <= a shares, moves up by
// floor(d b i / a), boundary i of that odd run by d (b - i); the ends of the pair stay where they were.
// Shares shorter than MF_TILT_MIN_SHARE units are left equal (such launches are not bound by the stream).
__device__ __forceinline__ unsigned share_begin(const MfmaSched& sc_, int ww, unsigned sh_q, unsigned sh_r, int W_eff) {
  unsigned g = (unsigned)ww * sh_q + ((unsigned)ww * sh_r) / (unsigned)W_eff;
  if (sc_.xcds > 1 && sh_q >= (unsigned)MF_TILT_MIN_SHARE) {
    const unsigned d = (sh_q * (unsigned)MF_XCD_TILT + 500u) / 1000u;
    const int chunk = (W_eff + sc_.xcds - 1) / sc_.xcds;
    const int run = ww / chunk, i = ww - run * chunk;
    const int ev = run & ~1;                                             // the even run of this pair
    const int a = max(0, min(chunk, W_eff - ev * chunk)), b = max(0, min(chunk, W_eff - (ev + 1) * chunk));
    if (a > 0 && b > 0) g += (run & 1) ? d * (unsigned)(b - i) : (d * (unsigned)b * (unsigned)i) / (unsigned)a;
  }
  return g;
}

template <int MAXRB>
__device__ __forceinline__ bool find_share(const AttnParams& p, const MfmaSched& sc_, int pw, int& w, int& seq, unsigned& Pt,
                                           SeqInfo& ws, unsigned& g0, unsigned& g1, unsigned& sh_q, unsigned& sh_r,
                                           int& W_eff) {
  constexpr int ROWS_WG = 32 * MAXRB;
  constexpr int MF_START_COST = mf_start_cost(MAXRB);
  __shared__ int sh_w[MF_BLOCK / 64];
  __shared__ int sh_found[12];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // ---- total work, this work-group's share, and the sequence in which the share starts -------
  // Tile counts fit 32 bits (the host checks the bound), so no 64-bit division is needed.
  // share w = [w q + floor(w r / W), ...) with q, r = total / W, total % W: equal to floor(w total / W)
  unsigned total = 0;
  sh_q = 0; sh_r = 0; W_eff = 0;
  auto plan_shares = [&]() {
    const unsigned want = sc_.fixed_share > 0 ? (unsigned)sc_.fixed_share
                                              : max((unsigned)sc_.min_share, (total + sc_.num_wgs - 1) / (unsigned)sc_.num_wgs);
    const unsigned weff = (total + want - 1) / want;
    W_eff = (int)min((unsigned)sc_.num_wgs, weff);
    sh_q = total / (unsigned)W_eff; sh_r = total % (unsigned)W_eff;
    const int chunk = (W_eff + sc_.xcds - 1) / sc_.xcds;
    w = pw / sc_.xcds < chunk ? (pw % sc_.xcds) * chunk + pw / sc_.xcds : W_eff;      // W_eff: no share
  };
  auto share_start = [&](int ww) -> unsigned { return share_begin(sc_, ww, sh_q, sh_r, W_eff); };
  g0 = 0; g1 = 0; Pt = 0; seq = -1; w = 0;
  if (p.B <= MF_BLOCK) {
    // one pass: thread i keeps sequence i in registers, the owner of tile g0 hands it over through LDS
    SeqInfo s_mine = {}; uint32_t bad = 0; int vt = 0;
    if (tid < p.B) {
      s_mine = load_seq_t<false>(p, tid, &bad);
      int T_, I_; seq_shape(p, s_mine, ROWS_WG, T_, I_);
      vt = item_units(T_, MF_START_COST) * I_;
    }
    const int it = wave_incl_scan(vt, lane);
    if (lane == 63) sh_w[wave] = it;
    if (tid == 0) sh_found[0] = -1;
    __syncthreads();
    int wt = 0;
#pragma unroll
    for (int q = 0; q < MF_BLOCK / 64; ++q) {
      if (q < wave) wt += sh_w[q];
      total += (unsigned)sh_w[q];
    }
    total = __builtin_amdgcn_readfirstlane(total);
    if (total == 0) return false;
    plan_shares();
    if (w >= W_eff) return false;
    g0 = share_start(w); g1 = share_start(w + 1);
    if (g1 <= g0) return false;
    const unsigned lo = (unsigned)(wt + it - vt), hi = (unsigned)(wt + it);
    if (lo <= g0 && g0 < hi) {
      sh_found[0] = tid; sh_found[1] = (int)lo;
      sh_found[2] = s_mine.L; sh_found[3] = s_mine.row0; sh_found[4] = s_mine.n; sh_found[5] = s_mine.k;
      sh_found[6] = s_mine.v; sh_found[7] = s_mine.page0; sh_found[8] = s_mine.npages; sh_found[9] = s_mine.nb;
    }
    if (bad) flag_status(p.status, bad);
    __syncthreads();
    seq = __builtin_amdgcn_readfirstlane(sh_found[0]);
    if (seq < 0) return false;                             // cannot happen for consistent data
    Pt = (unsigned)__builtin_amdgcn_readfirstlane(sh_found[1]);
    ws.L = __builtin_amdgcn_readfirstlane(sh_found[2]);      ws.row0 = __builtin_amdgcn_readfirstlane(sh_found[3]);
    ws.n = __builtin_amdgcn_readfirstlane(sh_found[4]);      ws.k = __builtin_amdgcn_readfirstlane(sh_found[5]);
    ws.v = __builtin_amdgcn_readfirstlane(sh_found[6]);      ws.page0 = __builtin_amdgcn_readfirstlane(sh_found[7]);
    ws.npages = __builtin_amdgcn_readfirstlane(sh_found[8]); ws.nb = __builtin_amdgcn_readfirstlane(sh_found[9]);
  } else {
    // larger batches: a first pass for the total, a second, block by block, for the owner of g0
    int part = 0;
    for (int i = tid; i < p.B; i += MF_BLOCK) {
      SeqInfo s = load_seq_t<false>(p, i);
      int T_, I_; seq_shape(p, s, ROWS_WG, T_, I_);
      part += item_units(T_, MF_START_COST) * I_;
    }
    part = wave_incl_scan(part, lane);
    if (lane == 63) sh_w[wave] = part;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < MF_BLOCK / 64; ++q) total += (unsigned)sh_w[q];
    total = __builtin_amdgcn_readfirstlane(total);
    if (tid == 0) sh_found[0] = -1;
    __syncthreads();
    if (total == 0) return false;
    plan_shares();
    if (w >= W_eff) return false;
    g0 = share_start(w); g1 = share_start(w + 1);
    if (g1 <= g0) return false;
    unsigned base_t = 0;
    for (int blk = 0; blk < p.B; blk += MF_BLOCK) {
      const int i = blk + tid;
      int T_ = 0, I_ = 0;
      if (i < p.B) { SeqInfo s = load_seq_t<false>(p, i); seq_shape(p, s, ROWS_WG, T_, I_); }
      const int vt = item_units(T_, MF_START_COST) * I_;
      const int it = wave_incl_scan(vt, lane);
      if (lane == 63) sh_w[wave] = it;
      __syncthreads();
      unsigned wt = 0, bt = 0;
#pragma unroll
      for (int q = 0; q < MF_BLOCK / 64; ++q) {
        if (q < wave) wt += (unsigned)sh_w[q];
        bt += (unsigned)sh_w[q];
      }
      const unsigned lo = base_t + wt + (unsigned)(it - vt), hi = base_t + wt + (unsigned)it;
      if (i < p.B && lo <= g0 && g0 < hi) { sh_found[0] = i; sh_found[1] = (int)lo; }
      base_t += bt;
      __syncthreads();
      if (sh_found[0] >= 0) break;
    }
    seq = __builtin_amdgcn_readfirstlane(sh_found[0]);
    if (seq < 0) return false;                             // cannot happen for consistent data
    Pt = (unsigned)__builtin_amdgcn_readfirstlane(sh_found[1]);
  }

  if (p.B > MF_BLOCK) ws = load_seq(p, seq);
  return true;
}

// Planning kernel: one work-group per persistent work-group of the streaming kernel.  Every one
// repeats the (cheap) scan over the batch, finds its own share and leaves its plan entry.
// MAXRB: 32-row blocks a work-group can own (2: up to 64 tile rows, 4: up to 128).
template <int MAXRB>
__global__ __launch_bounds__(MF_BLOCK) void attn_mfma_plan_kernel(AttnParams p, MfmaSched sc_) {
  constexpr int ROWS_WG = 32 * MAXRB;
  constexpr int MF_START_COST = mf_start_cost(MAXRB);
  const int tid = threadIdx.x;
  const int pw = blockIdx.x;                      // the entry is read by work-group pw of the streaming kernel
  PlanEntry* out = sc_.plan + pw;
  int w, seq, W_eff; unsigned Pt, g0, g1, sh_q, sh_r; SeqInfo ws;
  if (!find_share<MAXRB>(p, sc_, pw, w, seq, Pt, ws, g0, g1, sh_q, sh_r, W_eff)) {
    if (tid == 0) { out->seq = -1; out->W_eff = W_eff; }
    return;
  }
  // page ids of the first two tiles of the share's first piece (it lies in the item that holds unit g0)
  int T, I; seq_shape(p, ws, ROWS_WG, T, I);
  const int Tu = item_units(T, MF_START_COST);
  if (Tu <= 0) { if (tid == 0) { out->seq = -1; out->W_eff = W_eff; } return; }
  const int local = (int)(g0 - Pt);
  const int u = local - (local / Tu) * Tu;
  const int tile0 = max(u - MF_START_COST, 0);
  const int n_ct_all = (ws.L + MF_TK - 1) / MF_TK;
  if (tid < 2 * MF_GROUPS) {
    const int tau = tile0 + tid / MF_GROUPS, j = tid % MF_GROUPS;
    int id = 0;
    if (tau < n_ct_all) id = p.page_indices[ws.page0 + (min(tau * MF_TK + 16 * j, ws.L - 1) >> sc_.page_shift)];
    if (tid < MF_GROUPS) out->pg0[j] = id; else out->pg1[j] = id;
  }
  if (tid == 0) {
    out->seq = seq; out->Pt = Pt; out->g0 = g0; out->g1 = g1;
    out->L = ws.L; out->row0 = ws.row0; out->n = ws.n; out->k = ws.k; out->v = ws.v; out->nb = ws.nb;
    out->page0 = ws.page0; out->npages = ws.npages;
    out->sh_q = sh_q; out->sh_r = sh_r; out->W_eff = W_eff; out->share = w;
  }
}

// Streaming kernel.  MAXRB: 32-row blocks a work-group can own (2: up to 64 tile rows, 4: up to 128).
// PLANNED: the share comes from the plan entry the planning kernel left, else it is found here.
// DH: head dim (128 or 64).
template <int MAXRB, bool PLANNED, int DH>
__global__ __launch_bounds__(MF_BLOCK, 2) void attn_mfma_kernel(AttnParams p, MfmaSched sc_) {
  constexpr int ROWS_WG = 32 * MAXRB;
  constexpr int MF_D = DH;
  constexpr int MF_KSTR = MfLds<DH>::KSTR, MF_VSTR = MfLds<DH>::VSTR;
  constexpr int MF_K_ELEMS = MfLds<DH>::K_ELEMS, MF_BUF_ELEMS = MfLds<DH>::BUF_ELEMS;
  constexpr int NST = DH / 16;                   // MFMA steps over the head dim in S = K Q^T
  constexpr int NDB = DH / 32;                   // 32-wide blocks of the head dim in O
  constexpr int LPR = DH / 8;                    // lanes that load one row (16 bytes each)
  constexpr int RPL = 64 / LPR;                  // rows one load instruction of a wave covers
  constexpr int NLD = 16 / RPL;                  // load instructions per tensor for a wave's 16-key group
  typedef TileRegsT<NLD> TileRegs;
  constexpr int MF_START_COST = mf_start_cost(MAXRB);
  constexpr int PF_K = FD_PF_K, PF_V = FD_PF_V;   // LDS fragment requests run this many MFMAs ahead
  extern __shared__ __attribute__((aligned(16))) bf16_t lds[];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int h = lane >> 5, c32 = lane & 31, l16 = lane & 15;
  const int pw = blockIdx.x;
  const bool late_wg = pw >= (sc_.num_wgs >> 1);
  const bf16_t* Kc = reinterpret_cast<const bf16_t*>(p.k_cache);
  const bf16_t* Vc = reinterpret_cast<const bf16_t*>(p.v_cache);
  const bf16_t* Kn = reinterpret_cast<const bf16_t*>(p.k_new);
  const bf16_t* Vn = reinterpret_cast<const bf16_t*>(p.v_new);

  int w, seq, W_eff; unsigned Pt, g0, g1, sh_q, sh_r; SeqInfo ws;
  int nid0[MF_GROUPS], nid1[MF_GROUPS];          // page ids of the first two tiles of the piece to start
#pragma unroll
  for (int j = 0; j < MF_GROUPS; ++j) { nid0[j] = 0; nid1[j] = 0; }
  if (PLANNED) {
    // this work-group's plan entry: share, first sequence, first page ids (one scalar load)
    const int* pe = reinterpret_cast<const int*>(sc_.plan + pw);
    seq = sload(pe, 0); Pt = (unsigned)sload(pe, 1);
    g0 = (unsigned)sload(pe, 2); g1 = (unsigned)sload(pe, 3);
    ws.L = sload(pe, 4); ws.row0 = sload(pe, 5); ws.n = sload(pe, 6); ws.k = sload(pe, 7);
    ws.v = sload(pe, 8); ws.nb = sload(pe, 9); ws.page0 = sload(pe, 10); ws.npages = sload(pe, 11);
    sh_q = (unsigned)sload(pe, 12); sh_r = (unsigned)sload(pe, 13); W_eff = sload(pe, 14); w = sload(pe, 15);
#pragma unroll
    for (int j = 0; j < MF_GROUPS; ++j) { nid0[j] = sload(pe, 16 + j); nid1[j] = sload(pe, 20 + j); }
    // The plan is trusted to describe these arguments.  The checks below only keep a stale or foreign
    // plan from sending an access outside the caller's buffers (its results are then meaningless).
    W_eff = clampi(W_eff, 0, sc_.num_wgs);
    if (pw == 0 && tid == 0) sc_.entries[sc_.num_wgs] = make_int4(W_eff, 0, 0, 0);       // for the combine kernel
    if (seq < 0 || seq >= p.B || W_eff < 1 || w < 0 || w >= W_eff || g1 <= g0 || Pt > g0 || sh_q == 0) return;
    clamp_seq(p, ws);
  } else {
    const bool has = find_share<MAXRB>(p, sc_, pw, w, seq, Pt, ws, g0, g1, sh_q, sh_r, W_eff);
    if (pw == 0 && tid == 0) sc_.entries[sc_.num_wgs] = make_int4(W_eff, 0, 0, 0);
    if (!has) return;
  }
  // Slots, entries and every other per-share index below use the share's number w, not blockIdx.x.
  if (tid == 0) sc_.entries[w] = make_int4(-1, 0, 0, 0);
  auto share_start = [&](int ww) -> unsigned { return share_begin(sc_, ww, sh_q, sh_r, W_eff); };
  // the work-group whose share holds unit x of the line
  auto wg_of_unit = [&](unsigned x) -> int {
    int ww = (int)min(x / max(sh_q, 1u), (unsigned)(W_eff - 1));
    while (ww + 1 < W_eff && share_start(ww + 1) <= x) ++ww;
    while (ww > 0 && share_start(ww) > x) --ww;
    return ww;
  };

  // Tile loads: wave w fetches the w-th 16-key group of a tile (one page: one base address, one pair
  // of buffer descriptors per wave and tile); lane l takes 16-byte column l % LPR of keys l / LPR + RPL i
  // (head dim 128: column l & 15 of keys (l >> 4) + 4 i, four loads per tensor; 64: l & 7, (l >> 3) + 8 i, two).
  const int ld_row = lane / LPR;
  const int ld_col = (lane % LPR) * 8;         // element offset of this lane's 16 bytes
  const int page_mask = p.page_size - 1;
  const float cs = p.sm_scale * 1.4426950408889634f;           // scores are kept in base-2 units

  auto get_seq = [&](int i) {
    SeqInfo s = load_seq(p, i);
    s.L = __builtin_amdgcn_readfirstlane(s.L);       s.row0 = __builtin_amdgcn_readfirstlane(s.row0);
    s.n = __builtin_amdgcn_readfirstlane(s.n);       s.k = __builtin_amdgcn_readfirstlane(s.k);
    s.v = __builtin_amdgcn_readfirstlane(s.v);       s.page0 = __builtin_amdgcn_readfirstlane(s.page0);
    s.npages = __builtin_amdgcn_readfirstlane(s.npages); s.nb = __builtin_amdgcn_readfirstlane(s.nb);
    return s;
  };
  // ---- walk over the share, one piece (run of tiles inside one item) at a time ----------------
  // The walk state (sequence, its shape, tiles before it) only moves forward.
  int T, I; seq_shape(p, ws, ROWS_WG, T, I);

  struct Piece {
    SeqInfo s;                  // the sequence (scalar registers)
    int seq, head, rt;          // item
    int tile0, nt, T;           // tiles [tile0, tile0 + nt) of the item's T
    int units;                  // units of the line the piece covers
    int n_ct_all;               // cached tiles of the item (the rest are tiles of new rows)
    const bf16_t* kh;           // K cache and V cache advanced to the item's head
    const bf16_t* vh;
    const int* pi;              // the sequence's page list
    unsigned item_u;            // the item's first unit on the line
  };
  // descriptor of the piece that starts at unit g of the line (g < g1); false if the data ran out.
  // A piece may hold no tile at all (its units are start-up units only): pc.nt == 0.
  auto make_piece = [&](unsigned g, Piece& pc) -> bool {
    while (g >= Pt + (unsigned)(item_units(T, MF_START_COST) * I)) {
      Pt += (unsigned)(item_units(T, MF_START_COST) * I);
      ++seq;
      if (seq >= p.B) return false;
      ws = get_seq(seq);
      seq_shape(p, ws, ROWS_WG, T, I);
    }
    const int Tu = item_units(T, MF_START_COST);
    const int local = (int)(g - Pt);
    const int item = local / Tu;
    const int u = local - item * Tu;                               // unit within the item
    const int ue = min(Tu, u + (int)min(g1 - g, 0x3fffffffu));     // end of the piece, in units
    const int RT = I / p.Hkv;
    pc.s = ws; pc.seq = seq; pc.T = T;
    pc.head = item / RT; pc.rt = item - pc.head * RT;
    pc.tile0 = max(u - MF_START_COST, 0);
    pc.nt = max(ue - MF_START_COST, 0) - pc.tile0;
    pc.units = ue - u;
    pc.n_ct_all = (ws.L + MF_TK - 1) / MF_TK;
    pc.kh = Kc + (long long)pc.head * p.sh;
    pc.vh = Vc + (long long)pc.head * p.sh;
    pc.pi = p.page_indices + ws.page0;
    pc.item_u = Pt + (unsigned)(item * Tu);
    return true;
  };
  unsigned g = g0;                                  // next unit of the share to hand out
  auto next_piece = [&](Piece& pc) -> bool {       // the next piece that holds at least one tile
    while (g < g1) {
      if (!make_piece(g, pc)) return false;
      g += (unsigned)pc.units;
      if (pc.nt > 0) return true;
    }
    return false;
  };

  unsigned voff_c[NLD], voff_n[NLD];           // byte offsets of this lane's rows in a cached / a new 16-key group
  const long long new_pitch = (long long)p.Hkv * MF_D;
#pragma unroll
  for (int i = 0; i < NLD; ++i) {
    voff_c[i] = (unsigned)(2 * ((long long)(ld_row + RPL * i) * p.st + ld_col));
    voff_n[i] = (unsigned)(2 * ((long long)(ld_row + RPL * i) * new_pitch + ld_col));
  }

  // Physical page of each 16-key group of a cached tile: the same for every lane, so they are
  // fetched with scalar loads ahead of time and range-checked when the addresses are formed.
  auto fetch_pages = [&](const Piece& pc, int tau, int (&pg)[MF_GROUPS]) {
    if (tau < pc.n_ct_all) {
      const int base = tau * MF_TK, last = pc.s.L - 1;
      if (sc_.page_shift == 4 && base + MF_TK - 1 <= last) {
        // 16-token pages, full tile: four consecutive page ids, one scalar load
        typedef int i32x4_a4 __attribute__((ext_vector_type(4), aligned(4)));     // ids are only 4-byte aligned
        typedef const __attribute__((address_space(4))) i32x4_a4* const_i32x4_ptr;
        const int first = __builtin_amdgcn_readfirstlane(base >> 4);
        const i32x4_a4 v4 = *(const_i32x4_ptr)(uintptr_t)(pc.pi + first);
        pg[0] = v4[0]; pg[1] = v4[1]; pg[2] = v4[2]; pg[3] = v4[3];
      } else {
        // groups past the end of the prefix re-read its last page id (unused): no branch, so the
        // scalar loads of a tile go out back to back
#pragma unroll
        for (int j = 0; j < MF_GROUPS; ++j)
          pg[j] = sload(pc.pi, __builtin_amdgcn_readfirstlane(min(base + 16 * j, last) >> sc_.page_shift));
      }
    }
  };
  // One 16-key group = 16 rows of 256 B at a fixed pitch from a base that is the same for the
  // whole work-group.  It is read through a buffer descriptor built in scalar registers (base,
  // size) plus a per-lane 32-bit offset: no vector address arithmetic, and rows past the
  // descriptor's size read as zero.  `nrec` = bytes from the base to the end of the last valid row.
  auto load_rows = [&](const bf16_t* kbase, const bf16_t* vbase, int nrec, const unsigned (&voff)[NLD], TileRegs& r) {
    __amdgpu_buffer_rsrc_t rk_ = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(kbase), 0, nrec, 0x00020000);
    __amdgpu_buffer_rsrc_t rv_ = __builtin_amdgcn_make_buffer_rsrc(const_cast<bf16_t*>(vbase), 0, nrec, 0x00020000);
    if (sc_.reuse) {                               // the tile has other readers: let the L2 keep it
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(rk_, voff[i], 0, 0);
        r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv_, voff[i], 0, 0);
      }
    } else {
#pragma unroll
      for (int i = 0; i < NLD; ++i) {
        r.k[i] = __builtin_amdgcn_raw_buffer_load_b128(rk_, voff[i], 0, 2);      // aux 2: streaming (nt), read once
        r.v[i] = __builtin_amdgcn_raw_buffer_load_b128(rv_, voff[i], 0, 2);
      }
    }
  };
  auto nrec_of = [&](int valid, unsigned pitch) -> int {                 // valid rows of a 16-row group
    const int v16 = valid < 0 ? 0 : (valid > 16 ? 16 : valid);
    return v16 > 0 ? (int)(((unsigned)(v16 - 1) * pitch + MF_D) * 2u) : 0;
  };
  // strides as 32-bit values (the host checks the ranges): page id x page stride is then a
  // 32 x 32 -> 64 bit product instead of a 64 x 64 one
  const unsigned sp32 = (unsigned)p.sp, st32 = (unsigned)p.st;
  const int nrec_full = (int)((15u * st32 + MF_D) * 2u);
  auto load_tile = [&](const Piece& pc, int tau, const int (&pg)[MF_GROUPS], TileRegs& r) {
    const int gi = __builtin_amdgcn_readfirstlane(wave);   // this wave's 16-key group of the tile
    if (tau < pc.n_ct_all) {
      const int gs = tau * MF_TK + 16 * gi;
      unsigned ph = (unsigned)(gi == 0 ? pg[0] : gi == 1 ? pg[1] : gi == 2 ? pg[2] : pg[3]);
      const unsigned oob = ph >= (unsigned)p.num_pages ? 1u : 0u;
      if (oob & (gs < pc.s.L ? 1u : 0u)) flag_status(p.status, FD_DEV_PAGE_RANGE);
      ph = oob ? 0u : ph;
      const unsigned long long ub = (unsigned long long)ph * sp32 + (unsigned)(gs & page_mask) * st32;
      const int nrec = gs + 16 <= pc.s.L ? nrec_full : nrec_of(pc.s.L - gs, st32);   // rows past the prefix read as zero
      load_rows(pc.kh + ub, pc.vh + ub, nrec, voff_c, r);
    } else {
      const int key0 = (tau - pc.n_ct_all) * MF_TK + 16 * gi;
      const long long ub = ((long long)(pc.s.row0 + key0) * p.Hkv + pc.head) * MF_D;
      load_rows(Kn + ub, Vn + ub, nrec_of(pc.s.n - key0, (unsigned)new_pitch), voff_n, r);
    }
  };
  auto store_tile = [&](int buf, const TileRegs& r) {
    bf16_t* Kb = lds + buf * MF_BUF_ELEMS;
    bf16_t* Vb = Kb + MF_K_ELEMS;
#pragma unroll
    for (int i = 0; i < NLD; ++i) {
      const int row = 16 * wave + ld_row + RPL * i;
      *reinterpret_cast<u32x4*>(Kb + row * MF_KSTR + ld_col) = r.k[i];
      *reinterpret_cast<u32x4*>(Vb + row * MF_VSTR + ld_col) = r.v[i];
    }
  };

  // Per-lane view of a piece: which query row this lane owns and the wave's role.
  struct Lane {
    int RB, KQ, rb, kq, trow, nn, hq;
    RowWindow win;              // what this lane's row sees among the new rows
    bool row_valid, wave_has_rows;
  };
  auto make_lane = [&](const Piece& pc) {
    Lane ln;
    const int rows_total = pc.s.n * p.G;
    const int rows_here = min(ROWS_WG, rows_total - pc.rt * ROWS_WG);
    // 64-row variant: 1 or 2 row blocks, the waves of a row block split the tile's key blocks;
    // 128-row variant: wave w owns row block w and every key block (no key split, no merge)
    ln.RB = MAXRB == 4 ? 4 : (rows_here <= 32 ? 1 : 2);
    ln.KQ = MAXRB == 4 ? 1 : min(4 / ln.RB, MF_BLOCKS);
    ln.rb = wave % ln.RB; ln.kq = wave / ln.RB;                   // kq >= KQ: no block, idle
    ln.trow = ln.rb * 32 + c32;
    const int T_row = pc.rt * ROWS_WG + ln.trow;
    ln.row_valid = T_row < rows_total;
    ln.wave_has_rows = pc.rt * ROWS_WG + ln.rb * 32 < rows_total;
    if (sc_.group_shift >= 0) {                   // heads per KV head a power of two: no division
      ln.nn = T_row >> sc_.group_shift;
      ln.hq = pc.head * p.G + (T_row & (p.G - 1));
    } else {
      ln.nn = T_row / p.G;
      ln.hq = pc.head * p.G + T_row % p.G;
    }
    ln.win = row_window(ln.row_valid ? ln.nn : 0, pc.s);
    return ln;
  };

  bf16x8 qf[NST];
  int pg[MF_GROUPS];
#pragma unroll
  for (int j = 0; j < MF_GROUPS; ++j) pg[j] = 0;
  TileRegs rA, rB;
  // What a piece needs from memory before its first tile can be multiplied comes in two steps:
  // the page ids of its first two tiles (scalar loads), then, with those, the two tiles (into
  // rA, rB) and this lane's query row.  For every piece but the first, the ids are requested
  // before the previous piece's tile loop and the data before the previous piece is merged and
  // stored, so neither latency is exposed.
  auto start_ids = [&](const Piece& pc, int (&id0)[MF_GROUPS], int (&id1)[MF_GROUPS]) {
    fetch_pages(pc, pc.tile0, id0);
    if (pc.nt > 1) fetch_pages(pc, pc.tile0 + 1, id1);
  };
  auto start_loads = [&](const Piece& pc, const Lane& ln, const int (&id0)[MF_GROUPS], const int (&id1)[MF_GROUPS], bool second_tile) {
    const bf16_t* qp = reinterpret_cast<const bf16_t*>(p.q) + ((long long)(pc.s.row0 + (ln.row_valid ? ln.nn : 0)) * p.Hq + ln.hq) * MF_D + 8 * h;
    if (ln.row_valid) {
#pragma unroll
      for (int st = 0; st < NST; ++st) qf[st] = as_bf16x8(*reinterpret_cast<const u32x4*>(qp + 16 * st));
    } else {
      const u32x4 zero = {0u, 0u, 0u, 0u};
#pragma unroll
      for (int st = 0; st < NST; ++st) qf[st] = as_bf16x8(zero);
    }
    load_tile(pc, pc.tile0, id0, rA);
    if (pc.nt > 1 && second_tile) load_tile(pc, pc.tile0 + 1, id1, rB);
    fetch_pages(pc, pc.tile0 + 2, pg);
  };

  bool first_piece = true;
  Piece cur;
  if (!next_piece(cur)) return;
  Lane ln = make_lane(cur);
  if (!PLANNED) start_ids(cur, nid0, nid1);       // (a plan entry brings the first piece's page ids with it)
  start_loads(cur, ln, nid0, nid1, !FD_DEFER_T1);
#if FD_DEFER_T1
  // Every work-group starts at the same moment: with two tiles each in the first burst (33 MB) the memory
  // system queues them for 4-5 us and whoever is served last stays behind to the end.  The share's second
  // tile is requested when the first has landed.
  int t1ids[MF_GROUPS];
#pragma unroll
  for (int j = 0; j < MF_GROUPS; ++j) t1ids[j] = nid1[j];
#endif
  bool have = true;
  while (have) {
    // descriptor and page ids of the piece after this one: in flight during the tile loop
    Piece nxt;
    have = next_piece(nxt);
    if (have) start_ids(nxt, nid0, nid1);
    const SeqInfo& s = cur.s;
    const int tile0 = cur.tile0, nt = cur.nt, n_ct_all = cur.n_ct_all, c1 = cur.s.L;
    const bool whole = (tile0 == 0) && (nt == cur.T);
    const int slot = 2 * w + (first_piece ? 0 : 1);
    if (tid == 0 && tile0 > 0 && tile0 + nt == cur.T) {
      // this item started in an earlier work-group and ends here: leave it to the combine kernel.
      // Its first piece sits in the work-group wf that owns the item's first tile, in slot 2 wf
      // if nothing of wf's share precedes the item (a share that begins among the item's start-up
      // units has nothing before the item's first tile), else 2 wf + 1; later pieces are in slots 2 w'.
      const int wf = wg_of_unit(cur.item_u + MF_START_COST);
      const int first_slot = 2 * wf + (share_start(wf) >= cur.item_u ? 0 : 1);
      sc_.entries[w] = make_int4(cur.s.row0, cur.head | (cur.rt << 16), min(ROWS_WG, cur.s.n * p.G - cur.rt * ROWS_WG), first_slot);
    }
    const int RB = ln.RB, KQ = ln.KQ, rb = ln.rb, kq = ln.kq, trow = ln.trow, nn = ln.nn, hq = ln.hq;
    const bool row_valid = ln.row_valid, wave_has_rows = ln.wave_has_rows;

    // ---- running softmax state: one query row per lane ------------------------------------
    float m_run = -INFINITY, l_lane = 0.f;
    f32x16 o[NDB];
#pragma unroll
    for (int b = 0; b < NDB; ++b)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[b][i] = 0.f;

    store_tile(0, rA);                             // waits for the piece's first tile
#if FD_DEFER_T1
    if (first_piece && nt > 1) load_tile(cur, tile0 + 1, t1ids, rB);
#endif
    __syncthreads();

    // Two tiles are kept in registers: while tile t is multiplied out of LDS, tile t+2 is requested and
    // tile t+1 (requested an iteration earlier) is written to the other LDS buffer.  The request is
    // conditional and comes in two cache-policy variants, so the compiler's wait before that write
    // cannot count on it and drains the whole queue, tile t+2's loads included: the stream is in effect
    // one and a half tiles deep.  Making it exactly two deep was measured and is slower (more requests in
    // flight lengthen every queue, and a work-group that is behind falls further behind).
    auto iteration = [&](int t, TileRegs& r_store, TileRegs& r_load) {
      const int tau = tile0 + t;
      // The two work-groups of a CU take turns at the higher wave priority, one tile each.  At equal
      // priority the older wave wins every contested issue slot, and the CU's second work-group (the
      // upper half of blockIdx.x: dispatched once every CU has its first) would run about 10 % slower
      // than the first from start to end.
      if (((t & 1) != 0) != late_wg) __builtin_amdgcn_s_setprio(1); else __builtin_amdgcn_s_setprio(0);
      const bf16_t* Ks = lds + (t & 1) * MF_BUF_ELEMS;
      const bf16_t* Vs = Ks + MF_K_ELEMS;
      if (t + 2 < nt) {
        load_tile(cur, tau + 2, pg, r_load);
        fetch_pages(cur, tau + 3, pg);
      }

      // valid keys in this tile and whether the visibility rule has to be evaluated
      const bool is_new = tau >= n_ct_all;
      const int tile_base = is_new ? (tau - n_ct_all) * MF_TK : tau * MF_TK;
      const int tile_end = is_new ? s.n : c1;                     // keys at or beyond are invisible
      const bool masked = is_new | (tile_base + MF_TK > tile_end);

      if (wave_has_rows && kq < KQ) {
        // S^T = K Q^T for the 32 keys of block kb
        auto compute_S = [&](int kb) -> f32x16 {
          f32x16 sc;
#pragma unroll
          for (int i = 0; i < 16; ++i) sc[i] = 0.f;
          const bf16_t* kp = Ks + (32 * kb + c32) * MF_KSTR + 8 * h;
          // K fragments are requested PF_K MFMAs before the MFMA that consumes them
          u32x4 kf[NST];
#pragma unroll
          for (int f = 0; f < PF_K; ++f) kf[f] = *reinterpret_cast<const u32x4*>(kp + 16 * f);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int st = 0; st < NST; ++st) {
            sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(kf[st]), qf[st], sc, 0, 0, 0);
            if (st + PF_K < NST) kf[st + PF_K] = *reinterpret_cast<const u32x4*>(kp + 16 * (st + PF_K));
            __builtin_amdgcn_sched_barrier(0);                     // keep the requests where they are written
          }
          return sc;
        };
        // visibility + online softmax (base 2) of one block; returns P^T as packed bf16 pairs
        auto softmax_block = [&](f32x16 sc, int kb, unsigned (&pk)[8]) {
          if (masked) {
            // a prefix tile is the window "keys below the prefix length" (no second range)
            RowWindow wv = ln.win;
            if (!is_new) { wv.vr = c1; wv.lo = 0; wv.hi = 0; }
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              const int key = tile_base + 32 * kb + 8 * (i >> 2) + 4 * h + (i & 3);
              sc[i] = new_key_visible(wv, key) ? sc[i] : -INFINITY;
            }
          }
          float mx = fmaxf(sc[0], sc[1]);
#pragma unroll
          for (int i = 2; i < 16; ++i) mx = fmaxf(mx, sc[i]);
          // the other half of the row's keys is held by lane ^ 32: one v_permlane32_swap gives both
          // halves' maxima in every lane (no trip through LDS as a generic shuffle would make)
          {
            const unsigned mu = __builtin_bit_cast(unsigned, mx);
            const auto sw = __builtin_amdgcn_permlane32_swap(mu, mu, false, false);
            mx = fmaxf(__builtin_bit_cast(float, (unsigned)sw[0]), __builtin_bit_cast(float, (unsigned)sw[1]));
          }
          // The running reference m_run only follows the row maximum when that has moved up by more
          // than MF_LAZY (base-2 units): probabilities are then at most 2^MF_LAZY instead of 1, which
          // fp32 sums and bf16 P carry with the same relative precision, and the 64 accumulator
          // multiplications below run for a few tiles per item instead of for most of them.
          const float m_cand = fmaxf(m_run, mx * cs);
          const float m_new = m_cand > m_run + MF_LAZY ? m_cand : m_run;     // (-inf + MF_LAZY = -inf: first visible key)
          const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;  // row with nothing visible yet
          const float alpha = __builtin_amdgcn_exp2f(m_run - m_sub);
          m_run = m_new;
          if (__any(alpha != 1.f)) {
            l_lane *= alpha;
#pragma unroll
            for (int b = 0; b < NDB; ++b)
#pragma unroll
              for (int i = 0; i < 16; ++i) o[b][i] *= alpha;
          }
          float pr[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            pr[i] = __builtin_amdgcn_exp2f(fmaf(sc[i], cs, -m_sub));
            l_lane += pr[i];
          }
#pragma unroll
          for (int i = 0; i < 8; ++i) pk[i] = pack_bf16x2(pr[2 * i], pr[2 * i + 1]);
        };
        // O^T += V^T P^T for block kb
        auto compute_PV = [&](int kb, const unsigned (&pk)[8]) {
          // V^T fragment pair g: d-block g % NDB of k-step g / NDB; keys of a k-step for lane-half h are
          // base+4h+{0..3} and base+8+4h+{0..3}.  Pairs are requested PF_V MFMAs ahead.
          const bf16_t* vbase = Vs + (32 * kb + 4 * h + (l16 >> 2)) * MF_VSTR + 16 * (c32 >> 4) + 4 * (l16 & 3);
          s16x4 vf[4 * NDB];
          auto vread = [&](int g) {
            const bf16_t* vp = vbase + 16 * (g / NDB) * MF_VSTR + 32 * (g % NDB);
            vf[2 * g] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)vp);
            vf[2 * g + 1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(vp + 8 * MF_VSTR));
          };
#pragma unroll
          for (int g = 0; g < PF_V; ++g) vread(g);
#pragma unroll
          for (int g = 0; g < 2 * NDB; ++g) {
            const int q = g / NDB;
            u32x4 pw = {pk[4 * q], pk[4 * q + 1], pk[4 * q + 2], pk[4 * q + 3]};
            s16x8 vv = {vf[2 * g][0], vf[2 * g][1], vf[2 * g][2], vf[2 * g][3],
                        vf[2 * g + 1][0], vf[2 * g + 1][1], vf[2 * g + 1][2], vf[2 * g + 1][3]};
            o[g % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vv), as_bf16x8(pw), o[g % NDB], 0, 0, 0);
            if (g + PF_V < 2 * NDB) vread(g + PF_V);
          }
        };
        auto run_blocks = [&](auto nblk_c, int stride) {
          constexpr int NBLK = decltype(nblk_c)::value;
#pragma unroll
          for (int ib = 0; ib < NBLK; ++ib) {
            const int kb = kq + ib * stride;
            if (tile_base + 32 * kb >= tile_end) break;            // block entirely past the end
            f32x16 sc = compute_S(kb);
            unsigned pk[8];
            softmax_block(sc, kb, pk);
            compute_PV(kb, pk);
          }
        };
        if (tile_base + 32 * kq < tile_end) {
          if (MAXRB == 4 && RB == 4) run_blocks(std::integral_constant<int, MF_BLOCKS>{}, 1);   // all blocks of the tile
          else run_blocks(std::integral_constant<int, 1>{}, 0);                                // block kq only
        }
      }

      if (t + 1 < nt) store_tile((t + 1) & 1, r_store);
      __syncthreads();                           // tile t fully consumed, tile t+1 visible
    };
    for (int t = 0; t < nt; t += 2) {
      iteration(t, rB, rA);
      if (t + 1 < nt) iteration(t + 1, rA, rB);
    }

    // ---- next piece: get its loads going before this one is merged and stored --------------
    Lane ln_next = ln;
    if (have) { ln_next = make_lane(nxt); start_loads(nxt, ln_next, nid0, nid1, true); }

    // ---- merge the waves that shared a row block (through LDS, same register layout) ------
    constexpr int XQ = 4 * NDB;                                    // quads of O per lane
    f32x4* xch = reinterpret_cast<f32x4*>(lds);                    // [wave][XQ + 1][64] quads: XQ of O, then (m, l)
    static_assert((size_t)(MF_BLOCK / 64) * (XQ + 1) * 64 * sizeof(f32x4) <= MfLds<DH>::BYTES, "the merge area fits the tile buffers");
    if (MAXRB != 4 && KQ > 1) {
      if (kq > 0 && kq < KQ) {
        f32x4* dst = xch + (size_t)wave * (XQ + 1) * 64 + lane;
#pragma unroll
        for (int b = 0; b < NDB; ++b)
#pragma unroll
          for (int a = 0; a < 4; ++a) {
            f32x4 q4 = {o[b][4 * a], o[b][4 * a + 1], o[b][4 * a + 2], o[b][4 * a + 3]};
            dst[(4 * b + a) * 64] = q4;
          }
        f32x4 ml4 = {m_run, l_lane, 0.f, 0.f};
        dst[XQ * 64] = ml4;
      }
      __syncthreads();
      if (kq == 0) {
        for (int q2 = 1; q2 < KQ; ++q2) {
          const f32x4* src = xch + (size_t)(rb + q2 * RB) * (XQ + 1) * 64 + lane;
          const f32x4 ml4 = src[XQ * 64];
          const float m_o = ml4[0], l_o = ml4[1];
          const float m_new = fmaxf(m_run, m_o);
          const float m_sub = (m_new == -INFINITY) ? 0.f : m_new;
          const float a = __builtin_amdgcn_exp2f(m_run - m_sub), bsc = __builtin_amdgcn_exp2f(m_o - m_sub);
          l_lane = l_lane * a + l_o * bsc;
          m_run = m_new;
#pragma unroll
          for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int a4 = 0; a4 < 4; ++a4) {
              const f32x4 q4 = src[(4 * b + a4) * 64];
#pragma unroll
              for (int e = 0; e < 4; ++e) o[b][4 * a4 + e] = o[b][4 * a4 + e] * a + q4[e] * bsc;
            }
        }
      }
    }

    // ---- epilogue of the piece ------------------------------------------------------------
    if (kq == 0) {
      const float l_tot = l_lane + __shfl_xor(l_lane, 32);
      if (row_valid) {
        if (whole) {                              // whole item seen here: normalise and store
          const float inv = l_tot > 0.f ? 1.0f / l_tot : 0.f;
          bf16_t* op = reinterpret_cast<bf16_t*>(p.out) + ((long long)(s.row0 + nn) * p.Hq + hq) * MF_D + 4 * h;
#pragma unroll
          for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
              u32x2 wv = {pack_bf16x2(o[b][4 * a] * inv, o[b][4 * a + 1] * inv),
                          pack_bf16x2(o[b][4 * a + 2] * inv, o[b][4 * a + 3] * inv)};
              *reinterpret_cast<u32x2*>(op + 32 * b + 8 * a) = wv;
            }
          if (p.lse && h == 0)
            p.lse[(long long)(s.row0 + nn) * p.Hq + hq] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
        } else {
          // split partial for the combine kernel: the row scaled to [-1, 1] in fp16 (rounding 2^-11 of
          // the row's largest entry, a quarter of what the bf16 result carries) plus (max, sum, scale)
          float amax = 0.f;
#pragma unroll
          for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int i = 0; i < 16; ++i) amax = fmaxf(amax, fabsf(o[b][i]));
          amax = fmaxf(amax, __shfl_xor(amax, 32));
          const float rs = amax > 0.f ? 1.0f / amax : 0.f;
          const long long ps = (long long)slot * ROWS_WG + trow;
          unsigned short* ap = sc_.part_acc + ps * MF_D + 4 * h;
#pragma unroll
          for (int b = 0; b < NDB; ++b)
#pragma unroll
            for (int a = 0; a < 4; ++a) {
              u32x2 wv = {pack_f16x2(o[b][4 * a] * rs, o[b][4 * a + 1] * rs), pack_f16x2(o[b][4 * a + 2] * rs, o[b][4 * a + 3] * rs)};
              *reinterpret_cast<u32x2*>(ap + 32 * b + 8 * a) = wv;
            }
          if (h == 0) {
            f32x4 ml4 = {m_run, l_tot, amax, 0.f};
            *reinterpret_cast<f32x4*>(sc_.part_ml + ps * 4) = ml4;
          }
        }
      }
    }
    __syncthreads();                              // LDS is reused by the next piece
    first_piece = false;
    if (have) { cur = nxt; ln = ln_next; }
  }
}

// ---------------------------------------------------------------------------------------
// Merge the split partials of every item that was cut by a share boundary:
//   M = max m;  out = sum 2^{m - M} acc / sum 2^{m - M} l;  lse = (M + log2 sum) ln 2.
// The pieces of an item sit in its first slot, then in the first slot (2w) of every later
// work-group up to the one it ended in (which left the entry).  grid (num_wgs, ROWS_WG / 16):
// sixteen lanes per tile row, a lane owns eight adjacent output columns.
// ---------------------------------------------------------------------------------------
template <int MAXRB, int DH>
__global__ __launch_bounds__(256) void attn_mfma_combine_kernel(AttnParams p, MfmaSched sc_) {
  constexpr int ROWS_WG = 32 * MAXRB;
  constexpr int MF_D = DH;
  const int wl = blockIdx.x;                      // the work-group in which the split item ended
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l16 = lane & 15;                      // sixteen lanes own a tile row, a lane eight adjacent output columns
  const int* ep = reinterpret_cast<const int*>(sc_.entries + wl);
  const int shares = sload(reinterpret_cast<const int*>(sc_.entries + sc_.num_wgs), 0);     // entries beyond are nobody's
  const int row0 = sload(ep, 0), head_rt = sload(ep, 1), rows_here = sload(ep, 2), first_slot = sload(ep, 3);
  if (wl >= shares || row0 < 0) return;
  const int trow = blockIdx.y * 16 + wave * 4 + (lane >> 4);
  const int head = head_rt & 0xffff, rt = head_rt >> 16;
  const int wf = first_slot >> 1;
  if (rows_here > ROWS_WG || first_slot < 0 || wf >= wl || head >= p.Hkv) return;
  if (trow >= rows_here || l16 >= MF_D / 8) return;           // (head dim 64: half of the lanes have no column)
  const int T_row = rt * ROWS_WG + trow;
  const int nn = T_row / p.G, hq = head * p.G + T_row % p.G;
  if (row0 + nn >= p.total_rows) return;
  const int np = wl - wf + 1;                     // pieces: slot first_slot, then 2 (wf + 1) .. 2 wl
  auto ml_of = [&](int pi) -> const f32x4* {               // (max, sum, scale, -)
    const long long slot = pi == 0 ? first_slot : 2 * (wf + pi);
    return reinterpret_cast<const f32x4*>(sc_.part_ml + (slot * ROWS_WG + trow) * 4);
  };
  auto acc_of = [&](int pi) -> const u32x4* {               // eight fp16 columns of the scaled row
    const long long slot = pi == 0 ? first_slot : 2 * (wf + pi);
    return reinterpret_cast<const u32x4*>(sc_.part_acc + (slot * ROWS_WG + trow) * MF_D) + l16;
  };
  float num[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  float den = 0.f, M = -INFINITY;
  auto add_piece = [&](const f32x4& ml, const u32x4& a) {
    const float wgt = ml[0] == -INFINITY ? 0.f : exp2f(ml[0] - M);
    const float wa = wgt * ml[2];
    float x[8];
    { u32x2 lo = {a[0], a[1]}, hi = {a[2], a[3]}; float xl[4], xh[4]; unpack_f16x4(lo, xl); unpack_f16x4(hi, xh);
#pragma unroll
      for (int e = 0; e < 4; ++e) { x[e] = xl[e]; x[4 + e] = xh[e]; } }
#pragma unroll
    for (int e = 0; e < 8; ++e) num[e] = fmaf(wa, x[e], num[e]);
    den = fmaf(wgt, ml[1], den);
  };
  // up to 12 pieces: everything is requested at once (one memory latency), then reduced
  auto merge_at_once = [&](auto n_c) {
    constexpr int N = decltype(n_c)::value;
    f32x4 ml[N]; u32x4 a[N];
#pragma unroll
    for (int u = 0; u < N; ++u) {
      const int pu = min(u, np - 1);
      ml[u] = *ml_of(pu); a[u] = *acc_of(pu);
      if (u >= np) ml[u][0] = -INFINITY;
    }
    __builtin_amdgcn_sched_barrier(0);             // every request goes out before the first result is used
#pragma unroll
    for (int u = 0; u < N; ++u) M = fmaxf(M, ml[u][0]);
#pragma unroll
    for (int u = 0; u < N; ++u) add_piece(ml[u], a[u]);
  };
  if (np <= 4) merge_at_once(std::integral_constant<int, 4>{});
  else if (np <= 8) merge_at_once(std::integral_constant<int, 8>{});
  else if (np <= 12) merge_at_once(std::integral_constant<int, 12>{});
  else {
    // an item spread over more work-groups than that (cfg5: 17-18): twelve pieces at a time, all of a
    // batch requested together, with a running maximum (the sums are rescaled when it grows).  Larger
    // batches would need more registers than four blocks per CU leave, and most blocks of this grid
    // only look at their entry and return: how many of them a CU holds at once sets the kernel's floor.
    constexpr int NB = 12;
    for (int p0 = 0; p0 < np; p0 += NB) {
      f32x4 ml[NB]; u32x4 a[NB];
#pragma unroll
      for (int u = 0; u < NB; ++u) {
        const int pu = min(p0 + u, np - 1);
        ml[u] = *ml_of(pu); a[u] = *acc_of(pu);
        if (p0 + u >= np) ml[u][0] = -INFINITY;
      }
      __builtin_amdgcn_sched_barrier(0);
      float Mb = M;
#pragma unroll
      for (int u = 0; u < NB; ++u) Mb = fmaxf(Mb, ml[u][0]);
      if (Mb > M) {
        const float r = M == -INFINITY ? 0.f : exp2f(M - Mb);
#pragma unroll
        for (int e = 0; e < 8; ++e) num[e] *= r;
        den *= r;
        M = Mb;
      }
#pragma unroll
      for (int u = 0; u < NB; ++u) add_piece(ml[u], a[u]);
    }
  }
  const float inv = den > 0.f ? 1.0f / den : 0.f;
  const long long orow = (long long)(row0 + nn) * p.Hq + hq;
  u32x4 packed = {pack_bf16x2(num[0] * inv, num[1] * inv), pack_bf16x2(num[2] * inv, num[3] * inv),
                  pack_bf16x2(num[4] * inv, num[5] * inv), pack_bf16x2(num[6] * inv, num[7] * inv)};
  reinterpret_cast<u32x4*>(reinterpret_cast<bf16_t*>(p.out) + orow * MF_D)[l16] = packed;
  if (p.lse && l16 == 0) p.lse[orow] = (M + log2f(den)) * 0.6931471805599453f;
}

// ---------------------------------------------------------------------------------------
// host side
// ---------------------------------------------------------------------------------------
// The MFMA kernel takes bf16, head_dim 128 or 64 and power-of-two page sizes >= 16.
bool attn_mfma_supports(int dtype, int head_dim, int page_size) {
  return dtype == FD_BF16 && (head_dim == 128 || head_dim == 64) && page_size >= 16 && (page_size & (page_size - 1)) == 0;
}

int attn_mfma_tile_keys() { return MF_TK; }

// Tile rows one work-group covers for a launch whose largest sequence has `max_tile_rows`.
int attn_mfma_rows_per_wg(int max_tile_rows) { return max_tile_rows <= 64 ? 64 : 128; }

// Persistent work-groups: two per compute unit.
int attn_mfma_num_wgs() {
  static std::atomic<int> cached[64];              // per device; 0 = not asked yet
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 512;
  int n = cached[dev].load(std::memory_order_relaxed);
  if (n == 0) {
    int cus = 0;
    n = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0 ? FD_WGS_PER_CU * cus : 512;
    cached[dev].store(n, std::memory_order_relaxed);
  }
  return n;
}

// Workspace bytes for (num_wgs, rows per work-group) and the offsets of its parts: the partial
// rows, their (max, sum, scale), the combine entries, the plan entries.
size_t attn_mfma_workspace(int num_wgs, int rows_wg, size_t* off_ml, size_t* off_entries, size_t* off_plan) {
  auto al = [](size_t x) { return (x + 255) / 256 * 256; };
  size_t acc = al((size_t)2 * num_wgs * rows_wg * MF_D_MAX * sizeof(unsigned short));      // (sized for head dim 128)
  size_t ml = al((size_t)2 * num_wgs * rows_wg * 4 * sizeof(float));
  size_t en = al((size_t)(num_wgs + 1) * sizeof(int4));
  size_t pl = al((size_t)num_wgs * sizeof(PlanEntry));
  if (off_ml) *off_ml = acc;
  if (off_entries) *off_entries = acc + ml;
  if (off_plan) *off_plan = acc + ml + en;
  return acc + ml + en + pl;
}

static void fill_sched(const AttnParams& p, void* workspace, int kv_chunk, MfmaSched& sc, int& rows_wg) {
  sc.page_shift = 0;
  while ((1 << sc.page_shift) < p.page_size) ++sc.page_shift;
  sc.group_shift = -1;
  for (int b = 0; b < 16; ++b) if ((1 << b) == p.G) sc.group_shift = b;
  sc.num_wgs = attn_mfma_num_wgs();
  sc.xcds = sc.num_wgs % FD_XCDS == 0 ? FD_XCDS : 1;
  sc.min_share = 2;
  sc.fixed_share = kv_chunk > 0 ? (kv_chunk + MF_TK - 1) / MF_TK : 0;
  rows_wg = attn_mfma_rows_per_wg(p.max_new_rows * p.G > 128 ? 128 : p.max_new_rows * p.G);
  sc.reuse = (long long)p.max_new_rows * p.G > rows_wg ? 1 : 0;
  size_t off_ml, off_en, off_pl;
  attn_mfma_workspace(sc.num_wgs, rows_wg, &off_ml, &off_en, &off_pl);
  char* base = reinterpret_cast<char*>(workspace);
  sc.part_acc = reinterpret_cast<unsigned short*>(base);
  sc.part_ml = reinterpret_cast<float*>(base + off_ml);
  sc.entries = reinterpret_cast<int4*>(base + off_en);
  sc.plan = reinterpret_cast<PlanEntry*>(base + off_pl);
}

// The streaming kernel's LDS request is above the default limit: raised once per device.
template <int MAXRB, bool PLANNED, int DH>
static hipError_t configure_mfma() {
  static std::atomic<unsigned long long> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 64 && (done.load(std::memory_order_acquire) >> dev & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_mfma_kernel<MAXRB, PLANNED, DH>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)MfLds<DH>::BYTES);
  if (e == hipSuccess && dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
  return e;
}

// `workspace` must hold attn_mfma_workspace(...) bytes; kv_chunk > 0 asks for shares of that many keys.
// The plan: every persistent work-group's share, first sequence and first page ids.
hipError_t run_attn_mfma_plan(const AttnParams& p, void* workspace, int kv_chunk, hipStream_t st) {
  MfmaSched sc; int rows_wg;
  fill_sched(p, workspace, kv_chunk, sc, rows_wg);
  if (rows_wg == 64) hipLaunchKernelGGL(attn_mfma_plan_kernel<2>, dim3(sc.num_wgs), dim3(MF_BLOCK), 0, st, p, sc);
  else hipLaunchKernelGGL(attn_mfma_plan_kernel<4>, dim3(sc.num_wgs), dim3(MF_BLOCK), 0, st, p, sc);
  return hipGetLastError();
}

template <int MAXRB, bool PLANNED, int DH>
static hipError_t launch_mfma_d(const AttnParams& p, const MfmaSched& sc, hipStream_t st) {
  hipError_t e = configure_mfma<MAXRB, PLANNED, DH>();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_mfma_kernel<MAXRB, PLANNED, DH>), dim3(sc.num_wgs), dim3(MF_BLOCK), MfLds<DH>::BYTES, st, p, sc);
  return hipGetLastError();
}
template <int MAXRB, bool PLANNED>
static hipError_t launch_mfma(const AttnParams& p, const MfmaSched& sc, hipStream_t st) {
  if (p.D == 64) return launch_mfma_d<MAXRB, PLANNED, 64>(p, sc, st);
  if (p.D == 128) return launch_mfma_d<MAXRB, PLANNED, 128>(p, sc, st);
  return hipErrorInvalidValue;                  // (attn_mfma_supports keeps other head dims away)
}

// The streaming kernel; planned: the workspace holds the plan for these arguments.
hipError_t run_attn_mfma(const AttnParams& p, void* workspace, int kv_chunk, bool planned, hipStream_t st) {
  MfmaSched sc; int rows_wg;
  fill_sched(p, workspace, kv_chunk, sc, rows_wg);
  if (rows_wg == 64) return planned ? launch_mfma<2, true>(p, sc, st) : launch_mfma<2, false>(p, sc, st);
  return planned ? launch_mfma<4, true>(p, sc, st) : launch_mfma<4, false>(p, sc, st);
}

hipError_t run_attn_mfma_combine(const AttnParams& p, void* workspace, hipStream_t st) {
  MfmaSched sc; int rows_wg;
  fill_sched(p, workspace, 0, sc, rows_wg);
  dim3 grid(sc.num_wgs, rows_wg / 16);
  if (p.D != 64 && p.D != 128) return hipErrorInvalidValue;
  if (rows_wg == 64) {
    if (p.D == 64) hipLaunchKernelGGL((attn_mfma_combine_kernel<2, 64>), grid, dim3(256), 0, st, p, sc);
    else hipLaunchKernelGGL((attn_mfma_combine_kernel<2, 128>), grid, dim3(256), 0, st, p, sc);
  } else {
    if (p.D == 64) hipLaunchKernelGGL((attn_mfma_combine_kernel<4, 64>), grid, dim3(256), 0, st, p, sc);
    else hipLaunchKernelGGL((attn_mfma_combine_kernel<4, 128>), grid, dim3(256), 0, st, p, sc);
  }
  return hipGetLastError();
}

}  // namespace fd
