// Kernels of the HISA indexer (gfx950).  Notation follows the paper: B block size, m block
// budget, k token budget, H indexer heads, d head dimension, q/w/k indexing queries, gates, keys.
#pragma once

#include <type_traits>

#include "hisa_device.h"


namespace hisa {

// Fused Stage 2 kernel: waves per query and LDS tiles per wave.  Measured at the 64K bf16 prefill:
// 4 waves x 1 tile (two workgroups per CU) 8.9 ms; 8 waves x 1 or 2 tiles (one workgroup per CU,
// the select no longer overlaps another query's scoring) +25 %; 6 waves under a 168-register cap
// (three waves per SIMD, one accumulator live, no overlap inside a wave, no spills) +40 %: the
// MFMA-over-epilogue overlap inside a wave is worth more than a third wave.  Deeper rings do not
// help, neither do LDS reads requested half a tile early, a branch-free step with one DMA
// instruction per MFMA pair, a raised wave priority over the MFMAs, or touching the lines of the
// tiles two ahead (all within 2 % or slower), or a fixed grid of workgroups that each walk several
// queries (+10 % with 512 workgroups: the hardware's dynamic placement of one short workgroup
// per query balances better): with bf16 keys a tile is 8 KB through the CU's
// vector-memory path per 16 MFMAs, and that path (about 44 B/clk/CU measured, keys L2-resident)
// saturates together with the matrix cores.  fp8 keys run on the fp8 MFMA against the two-term
// e4m3 form of the query (no widening instructions, half the tile bytes): 7.7 ms; a ring of two
// fp8 tiles with the operand reads of tile j+1 requested before the MFMAs of tile j and awaited
// after them measured the same, and time grows by 1.5 ms per 16 kept blocks on top of 1.5 ms that
// does not depend on m (per query: fragment load and split, block table, top-k, output).
constexpr int kNBuf = 1;
constexpr int kFusedWaves = 4;

enum : int { DT_F32 = 0, DT_BF16 = 1, DT_FP8 = 2 };

// What a scoring kernel needs to know about queries, keys and where scores go.
struct ScoreArgs {
  const void* q;             // [T, H, d]
  const float* w;            // [T, H]
  const int32_t* q_seq;      // [T] or null
  const int32_t* q_pos;      // [T] or null
  const int32_t* q_lo;       // [T] first visible position (packed sequences) or null: 0
  int q_pos0;
  int H, d;
  const void* keys;          // [n_seq, rows_per_seq, d]: token keys, or pooled keys (pos_div = B)
  const float* k_scale;      // [n_seq, rows_per_seq] (fp8 token keys) or null
  const int32_t* seq_len;    // [n_seq]
  int n_seq;
  long rows_per_seq;
  int pos_div;               // 1: rows are tokens; B: rows are blocks (visible rows = pos / B + 1)
  const int32_t* block_idx;  // [T, m] => gather mode (Eq. 7: candidates = tokens of kept blocks)
  int m, B;
  float* out;                // [t_count, ld] scores, row = query - t_begin
  long ld;
  int t_begin, t_count;
  int tiles_per_wave;        // score_ranges: 32-key tiles each wave handles
  int groups;                // score_ranges: workgroups per query (the grid holds t_count * groups)
};

// Position and sequence of query t, clamped so that no key row past the sequence is visible.
__device__ __forceinline__ int query_pos(const ScoreArgs& a, int t, int& seq) {
  int s = a.q_seq ? a.q_seq[t] : 0;
  s = s < 0 ? 0 : (s >= a.n_seq ? a.n_seq - 1 : s);
  seq = s;
  int pos = a.q_pos ? a.q_pos[t] : a.q_pos0 + t;
  // a sequence cannot be longer than the padded row count of its key array (a bad seq_len must
  // not turn into an index past the arrays)
  const long cap = a.rows_per_seq * a.pos_div;
  int sl = a.seq_len[s];
  sl = sl < cap ? sl : (int)cap;
  return pos < sl ? pos : sl - 1;
}

__device__ __forceinline__ int visible_rows(const ScoreArgs& a, int pos) {
  return pos < 0 ? 0 : pos / a.pos_div + 1;
}

// First visible position of query t: its sequence's first token when sequences are packed into one
// key stream (Section 4.1: blocks may then straddle two sequences), else 0.  The query sees the
// positions lo .. pos; lo == pos + 1 means it sees nothing.
__device__ __forceinline__ int query_lo(const int32_t* q_lo, int t, int pos) {
  int lo = q_lo ? q_lo[t] : 0;
  lo = lo < 0 ? 0 : lo;
  return lo > pos + 1 ? pos + 1 : lo;
}

// Grids whose second dimension would be the query (row) index are launched one-dimensional, as
// rows * gx workgroups with the gx workgroups of a row adjacent: the y dimension of a grid stops at
// 65535, the x dimension at 2^31 - 1.
struct RowGroup {
  int row, x;
};
__device__ __forceinline__ RowGroup row_group(int gx) {
  const int b = (int)blockIdx.x;
  if (gx <= 1) return {b, 0};
  const int row = b / gx;
  return {row, b - row * gx};
}

// ------------------------------------------------------------------------------------------
// Eq. 4: block mean pooling.  One workgroup per (block, sequence).  VEC = elements per 16-byte
// load (4 fp32 / 8 bf16 / 16 fp8).  Thread (rl, col) sums rows rl, rl+RP, ... of its 16-byte
// column in fp32; the RP partial rows are then reduced through LDS and divided by the count.
// MAXP: per-dimension maximum instead of the mean (the other Pool of Section 4.1's generic Eq. 4).
template <int KDT, int PDT, bool MAXP = false>
__device__ __forceinline__ void pool_one_block(const void* __restrict__ keys,
                                               const float* __restrict__ k_scale, int sl, long s_max,
                                               int d, int B, int seq, int b, void* __restrict__ pooled,
                                               float* part) {
  constexpr int VEC = KDT == DT_F32 ? 4 : (KDT == DT_BF16 ? 8 : 16);
  const int tid = threadIdx.x;
  const int VC = d / VEC;               // 16-byte columns per key row (<= 256 checked on the host)
  const int RP = 256 / VC;              // rows in flight per pass
  const int rl = tid / VC, col = tid % VC;
  const long M = s_max / B;
  long lo = (long)b * B;
  int nb = (int)((sl - lo) < (long)B ? (sl - lo) : (long)B);
  if (nb < 0) nb = 0;
  float acc[VEC];
#pragma unroll
  for (int e = 0; e < VEC; ++e) acc[e] = MAXP ? neg_inf() : 0.f;
  auto add = [&](float& a, float v) { a = MAXP ? fmaxf(a, v) : a + v; };
  if (rl < RP) {
    const char* base = (const char*)keys + ((long)seq * s_max + lo) * d * (16 / VEC);
    for (int r = rl; r < nb; r += RP) {
      const uint4 v = *reinterpret_cast<const uint4*>(base + ((long)r * VC + col) * 16);
      if (KDT == DT_F32) {
        add(acc[0], __uint_as_float(v.x));
        add(acc[1], __uint_as_float(v.y));
        add(acc[2], __uint_as_float(v.z));
        add(acc[3], __uint_as_float(v.w));
      } else if (KDT == DT_BF16) {
        const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          add(acc[2 * e], __uint_as_float(ww[e] << 16));
          add(acc[2 * e + 1], __uint_as_float(ww[e] & 0xffff0000u));
        }
      } else if (MAXP) {
        const float sc = k_scale[(long)seq * s_max + lo + r];
        const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint2 h = fp8x4_to_bf16x4(ww[e]);
          add(acc[4 * e + 0], sc * __uint_as_float(h.x << 16));
          add(acc[4 * e + 1], sc * __uint_as_float(h.x & 0xffff0000u));
          add(acc[4 * e + 2], sc * __uint_as_float(h.y << 16));
          add(acc[4 * e + 3], sc * __uint_as_float(h.y & 0xffff0000u));
        }
      } else {
        const float sc = k_scale[(long)seq * s_max + lo + r];
        const uint32_t ww[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint2 h = fp8x4_to_bf16x4(ww[e]);
          acc[4 * e + 0] = __builtin_fmaf(sc, __uint_as_float(h.x << 16), acc[4 * e + 0]);
          acc[4 * e + 1] = __builtin_fmaf(sc, __uint_as_float(h.x & 0xffff0000u), acc[4 * e + 1]);
          acc[4 * e + 2] = __builtin_fmaf(sc, __uint_as_float(h.y << 16), acc[4 * e + 2]);
          acc[4 * e + 3] = __builtin_fmaf(sc, __uint_as_float(h.y & 0xffff0000u), acc[4 * e + 3]);
        }
      }
    }
#pragma unroll
    for (int e = 0; e < VEC; ++e) part[rl * d + col * VEC + e] = acc[e];
  }
  __syncthreads();
  for (int i = tid; i < d; i += 256) {
    float s = MAXP ? neg_inf() : 0.f;
    for (int r = 0; r < RP; ++r) add(s, part[r * d + i]);
    const float mean = nb > 0 ? (MAXP ? s : s / (float)nb) : 0.f;
    const long o = ((long)seq * M + b) * d + i;
    if (PDT == DT_F32)
      ((float*)pooled)[o] = mean;
    else
      ((uint16_t*)pooled)[o] = f32_to_bf16_rne(mean);
  }
}

template <int KDT, int PDT, bool MAXP = false>
__global__ __launch_bounds__(256) void k_pool(const void* __restrict__ keys,
                                              const float* __restrict__ k_scale,
                                              const int32_t* __restrict__ seq_len, long s_max, int d,
                                              int B, int blk_begin, void* __restrict__ pooled) {
  constexpr int VEC = KDT == DT_F32 ? 4 : (KDT == DT_BF16 ? 8 : 16);
  __shared__ float part[256 * VEC];
  const int seq = blockIdx.y;
  pool_one_block<KDT, PDT, MAXP>(keys, k_scale, seq_len[seq], s_max, d, B, seq, blk_begin + blockIdx.x,
                                 pooled, part);
}

// Incremental pooled-cache update (Section 4.1): workgroup (j, n) re-pools block prev_len[n]/B + j
// of sequence n if that block received tokens since the previous update.
template <int KDT, int PDT>
__global__ __launch_bounds__(256) void k_pool_append(const void* __restrict__ keys,
                                                     const float* __restrict__ k_scale,
                                                     const int32_t* __restrict__ seq_len,
                                                     const int32_t* __restrict__ prev_len, long s_max,
                                                     int d, int B, void* __restrict__ pooled) {
  constexpr int VEC = KDT == DT_F32 ? 4 : (KDT == DT_BF16 ? 8 : 16);
  __shared__ float part[256 * VEC];
  const int seq = blockIdx.y;
  int sl = seq_len[seq];
  sl = sl < 0 ? 0 : (sl > s_max ? (int)s_max : sl);
  int pl = prev_len[seq];
  pl = pl < 0 ? 0 : (pl > sl ? sl : pl);
  if (sl <= pl) return;                       // nothing appended (uniform per workgroup)
  const int b = pl / B + blockIdx.x;
  if (b > (sl - 1) / B) return;
  pool_one_block<KDT, PDT>(keys, k_scale, sl, s_max, d, B, seq, b, pooled, part);
}

// Block-Sparse baseline (Section 5): every visible token of the kept blocks.
__global__ __launch_bounds__(256) void k_block_sparse_tokens(ScoreArgs a, int32_t* __restrict__ tokens) {
  const RowGroup rg = row_group(a.groups);
  const int t = rg.row;
  int seq;
  const int pos = query_pos(a, t, seq);
  const int lo = query_lo(a.q_lo, t, pos);
  const int n_slots = a.m * a.B;
  const int n_blocks = (int)(a.rows_per_seq / a.B);
  for (int c = rg.x * 256 + threadIdx.x; c < n_slots; c += a.groups * 256) {
    const int slot = c / a.B;
    const int blk = a.block_idx[(long)t * a.m + slot];
    const int tok = blk * a.B + (c - slot * a.B);
    tokens[(long)t * n_slots + c] = (blk >= 0 && blk < n_blocks && tok <= pos && tok >= lo) ? tok : -1;
  }
}

// Eq. 12: one wave per row.  Both rows are ascending with -1 padding behind the valid entries: the
// valid lengths are counted, then every lane looks its share of row a up in row b by binary search
// (a row is a few KB and stays in the L1 / L2 for the walk).
// STAGED: row b is copied into this wave's k ints of LDS first (k <= 4096), where a probe costs an
// LDS access instead of a cache access.
template <bool STAGED>
__global__ __launch_bounds__(256) void k_index_iou(const int32_t* __restrict__ a_idx,
                                                   const int32_t* __restrict__ b_idx, int T, int k,
                                                   float* __restrict__ iou) {
  extern __shared__ int32_t iou_rows[];   // STAGED: [4][k]
  const int t = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (t >= T) return;
  const int32_t* pa = a_idx + (long)t * k;
  const int32_t* pb = b_idx + (long)t * k;
  int32_t* sb = iou_rows + (threadIdx.x >> 6) * k;
  // valid lengths: entries in front of the first negative one
  int first_a = k, first_b = k;
  for (int i = lane; i < k; i += 64) {
    const int y = pb[i];
    if (STAGED) sb[i] = y;
    if (pa[i] < 0 && i < first_a) first_a = i;
    if (y < 0 && i < first_b) first_b = i;
  }
  const int na = k - (int)wave_max((uint32_t)(k - first_a)), nb = k - (int)wave_max((uint32_t)(k - first_b));   // wave minima
  const int32_t* rb = STAGED ? sb : pb;   // (a wave reads only what it wrote itself: no barrier)
  int inter = 0;
  for (int i = lane; i < na; i += 64) {
    const int x = pa[i];
    int lo = 0, hi = nb;            // first position of b with b[pos] >= x
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (rb[mid] < x) lo = mid + 1;
      else hi = mid;
    }
    inter += (lo < nb && rb[lo] == x) ? 1 : 0;
  }
  inter = (int)wave_sum((uint32_t)inter);
  const int uni = na + nb - inter;
  if (lane == 0) iou[t] = uni == 0 ? 1.f : (float)inter / (float)uni;
}

// ------------------------------------------------------------------------------------------
// Attainable-peak probes (measurement aids, not part of the method): a streaming copy and a loop
// of nothing but MFMAs, so that a benchmark can quote its kernels against what this chip delivers.
__global__ __launch_bounds__(256) void k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst,
                                                    long n16) {
  // four 16-byte loads in flight per thread
  const long stride = (long)gridDim.x * 256;
  long i = (long)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 a = src[i], b = src[i + stride], c = src[i + 2 * stride], d = src[i + 3 * stride];
    dst[i] = a;
    dst[i + stride] = b;
    dst[i + 2 * stride] = c;
    dst[i + 3 * stride] = d;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

__global__ __launch_bounds__(256) void k_probe_mfma(float* out, int iters) {
  bf16x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = (__bf16)(float)(threadIdx.x & 3);
    b[e] = (__bf16)(float)(threadIdx.x & 1);
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
      for (int n = 0; n < 4; ++n) acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[n], 0, 0, 0);
  }
  out[(long)blockIdx.x * 256 + threadIdx.x] = (acc[0][0] + acc[1][5]) + (acc[2][9] + acc[3][15]);
}

__global__ __launch_bounds__(256) void k_probe_mfma_fp8(float* out, int iters) {
  i32x8 a, b;
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    a[e] = 0x38383838 + (int)(threadIdx.x & 3);   // e4m3 codes near 1.0
    b[e] = 0x30303030 + e;
  }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < 2; ++r)
#pragma unroll
      for (int n = 0; n < 4; ++n)
        acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(a, b, acc[n], 0, 0, 0, 0, 0, 0);
  }
  out[(long)blockIdx.x * 256 + threadIdx.x] = (acc[0][0] + acc[1][5]) + (acc[2][9] + acc[3][15]);
}

// The same two loops on operands that differ from lane to lane and from one MFMA to the next
// (pseudo-random signs and mantissas, exponents within a factor of 8 of one): what the matrix cores
// sustain when their inputs toggle as real data does.  With the constant small integers of the two
// probes above the chip holds its full clock; with these it does not.
__device__ __forceinline__ uint32_t probe_hash(uint32_t x) {
  x ^= x >> 16;
  x *= 0x7feb352dU;
  x ^= x >> 15;
  x *= 0x846ca68bU;
  x ^= x >> 16;
  return x;
}

template <bool FP8>
__global__ __launch_bounds__(256) void k_probe_mfma_toggling(float* out, int iters) {
  // four A and four B operands per lane, 32 bytes each (the bf16 instruction reads the first 16)
  i32x8 a[4], b[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const uint32_t h = probe_hash(threadIdx.x * 64u + n * 8u + e);
      const uint32_t g = probe_hash(h + 77u + blockIdx.x);
      if constexpr (FP8) {
        // e4m3 bytes: sign, exponent field 4..7 (2^-3 .. 1), three mantissa bits; never the NaN code
        a[n][e] = (int)((h & 0x87878787u) | 0x20202020u | ((h >> 1) & 0x18181818u));
        b[n][e] = (int)((g & 0x87878787u) | 0x20202020u | ((g >> 1) & 0x18181818u));
      } else {
        // bf16 halves: sign, exponent field 124..127, seven mantissa bits
        a[n][e] = (int)((h & 0x807f807fu) | 0x3e003e00u | ((h >> 2) & 0x01800180u));
        b[n][e] = (int)((g & 0x807f807fu) | 0x3e003e00u | ((g >> 2) & 0x01800180u));
      }
    }
  f32x16 acc[4];
#pragma unroll
  for (int n = 0; n < 4; ++n)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[n][i] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int r = 0; r < (FP8 ? 2 : 4); ++r)
#pragma unroll
      for (int n = 0; n < 4; ++n) {
        const i32x8 av = a[(n + r) & 3], bv = b[(n + 2 * r + 1) & 3];
        if constexpr (FP8) {
          acc[n] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(av, bv, acc[n], 0, 0, 0, 0, 0, 0);
        } else {
          const u32x4v a4 = {(uint32_t)av[0], (uint32_t)av[1], (uint32_t)av[2], (uint32_t)av[3]};
          const u32x4v b4 = {(uint32_t)bv[0], (uint32_t)bv[1], (uint32_t)bv[2], (uint32_t)bv[3]};
          acc[n] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a4),
                                                           __builtin_bit_cast(bf16x8, b4), acc[n], 0, 0, 0);
        }
      }
  }
  out[(long)blockIdx.x * 256 + threadIdx.x] = (acc[0][0] + acc[1][5]) + (acc[2][9] + acc[3][15]);
}

__global__ __launch_bounds__(256) void k_fill_f32(float* p, long n, float v) {
  for (long i = (long)blockIdx.x * 256 + threadIdx.x; i < n; i += (long)gridDim.x * 256) p[i] = v;
}

// ------------------------------------------------------------------------------------------
// Eq. 1 / Eq. 5 on the plain fp32 ALU, any H and d (the small fp32 configuration).  One workgroup
// per (chunk of keys, query); the query's heads and gates sit in LDS, each thread scores one key.
__global__ __launch_bounds__(256) void k_score_ranges_f32(ScoreArgs a, int keys_per_wg) {
  extern __shared__ float qs[];   // H*d query values, then H gates
  const RowGroup rg = row_group(a.groups);
  const int t = a.t_begin + rg.row;
  const int tid = threadIdx.x;
  int seq;
  const int pos = query_pos(a, t, seq);
  const int H = a.H, d = a.d;
  const float* q = (const float*)a.q + (long)t * H * d;
  for (int i = tid; i < H * d; i += 256) qs[i] = q[i];
  for (int i = tid; i < H; i += 256) qs[H * d + i] = a.w[(long)t * H + i];
  __syncthreads();
  const bool gather = a.block_idx != nullptr;
  const int n_total = gather ? a.m * a.B : visible_rows(a, pos);
  const int lo = query_lo(a.q_lo, t, pos);
  const int lo_row = lo / a.pos_div;   // first visible row when the rows are blocks or tokens in order
  const int c0 = rg.x * keys_per_wg;
  const int c1 = (c0 + keys_per_wg) < n_total ? (c0 + keys_per_wg) : n_total;
  const float* kbase = (const float*)a.keys + (long)seq * a.rows_per_seq * d;
  float* out = a.out + (long)rg.row * a.ld;
  for (int c = c0 + tid; c < c1; c += 256) {
    long row = c;
    bool valid = c >= lo_row;
    if (gather) {
      const int slot = c / a.B, off = c - slot * a.B;
      const int blk = a.block_idx[(long)t * a.m + slot];
      row = (long)blk * a.B + off;
      valid = blk >= 0 && row <= pos && row >= lo;
    }
    float s = neg_inf();
    if (valid) {
      const float4* kr = reinterpret_cast<const float4*>(kbase + row * d);
      s = 0.f;
      // Four heads per pass over the key row (its loads are then independent of each other and four
      // deep, instead of one dependent load per 4 multiply-adds); every head keeps its own four
      // partial sums in the order of the one-head loop below, so the grouping changes no bit.
      int j = 0;
      for (; j + 4 <= H; j += 4) {
        const float4* qr = reinterpret_cast<const float4*>(qs + j * d);
        const int dq = d >> 2;
        float p[4][4];
#pragma unroll
        for (int h = 0; h < 4; ++h)
#pragma unroll
          for (int e = 0; e < 4; ++e) p[h][e] = 0.f;
#pragma unroll 4
        for (int i = 0; i < dq; ++i) {
          const float4 kv = kr[i];
#pragma unroll
          for (int h = 0; h < 4; ++h) {
            const float4 qv = qr[h * dq + i];
            p[h][0] = __builtin_fmaf(qv.x, kv.x, p[h][0]);
            p[h][1] = __builtin_fmaf(qv.y, kv.y, p[h][1]);
            p[h][2] = __builtin_fmaf(qv.z, kv.z, p[h][2]);
            p[h][3] = __builtin_fmaf(qv.w, kv.w, p[h][3]);
          }
        }
#pragma unroll
        for (int h = 0; h < 4; ++h) {
          const float dot = (p[h][0] + p[h][1]) + (p[h][2] + p[h][3]);
          s = __builtin_fmaf(qs[H * d + j + h], __builtin_fmaxf(dot, 0.f), s);
        }
      }
      for (; j < H; ++j) {
        const float4* qr = reinterpret_cast<const float4*>(qs + j * d);
        float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
        for (int i = 0; i < d / 4; ++i) {
          const float4 kv = kr[i], qv = qr[i];
          d0 = __builtin_fmaf(qv.x, kv.x, d0);
          d1 = __builtin_fmaf(qv.y, kv.y, d1);
          d2 = __builtin_fmaf(qv.z, kv.z, d2);
          d3 = __builtin_fmaf(qv.w, kv.w, d3);
        }
        const float dot = (d0 + d1) + (d2 + d3);
        s = __builtin_fmaf(qs[H * d + j], __builtin_fmaxf(dot, 0.f), s);
      }
    }
    out[c] = s;
  }
}

// Where virtual tile v of a query lives: key rows [row0, row0+32), output slots [out0, out0+32).
// Flat / Stage 1: tile v covers rows 32v ..; gather (Stage 2): tile v is sub-tile v % (B/32) of
// the kept block in slot v / (B/32).  row0 < 0: the slot is empty (-1 padding).
struct TileLoc {
  long row0;
  long out0;
};

__device__ __forceinline__ TileLoc tile_loc(const ScoreArgs& a, int t, int v, bool gather) {
  TileLoc L;
  if (gather) {
    const int tpb = a.B >> 5;
    const int slot = v / tpb, sub = v - slot * tpb;
    const int blk = a.block_idx[(long)t * a.m + slot];
    L.out0 = (long)slot * a.B + sub * 32;
    L.row0 = blk < 0 ? -1 : (long)blk * a.B + sub * 32;
  } else {
    L.row0 = (long)v * 32;
    L.out0 = L.row0;
  }
  return L;
}

// ------------------------------------------------------------------------------------------
// The per-wave scoring pipeline shared by Stage 2 and the per-query scoring kernels.
//
// A wave owns one query (QFrag in registers) and a ring of NB LDS tiles.  For its j-th tile it
//   * DMAs the key rows global -> LDS NB tiles ahead (no registers involved),
//   * copies the staged tile into registers as MFMA B operands (which frees the LDS tile),
//   * runs the 16 MFMAs of tile j while the vector ALU does the ReLU / gate / head-sum epilogue of
//     tile j-1 (two accumulator sets swap roles, the loop is unrolled by two).
// (Measured and not kept: the operand reads of tile j+1 requested from LDS while the MFMAs of tile j
// run, into a second register set paid for by one accumulator set per head block, so that no MFMA of
// a wave waits on an LDS read: Stage 2 of the 64K prefill 3-4 % slower with bf16 and with fp8 keys,
// wherever in the step the next DMA was issued.  The step is not waiting on LDS latency.)
// row_at(j): first key row of tile j (wave-uniform, a row inside the sequence's key array);
// finish(j, s): lane l < 32 receives the score of key row_at(j) + l (fp8: already scaled).
template <int KDT>
struct TileGeom {
  static constexpr int kLoads = KDT == DT_BF16 ? 8 : 5;                 // DMA instructions per tile
  static constexpr int kBufBytes = KDT == DT_BF16 ? 8192 : 4096 + 256;  // LDS per staged tile
};

// The query fragment and the key-tile registers a key type computes with: bf16 keys on the bf16
// MFMA, fp8 keys (as stored) on the fp8 MFMA against the two-term e4m3 form of the query.
template <int HG, int KDT>
struct Operands {
  using Frag = QFrag<HG>;
  using Tile = u32x32;
  static __device__ __forceinline__ void make(const QFrag<HG>& f, Frag& o) { o = f; }
};
template <int HG>
struct Operands<HG, DT_FP8> {
  using Frag = QFrag8<HG>;
  using Tile = u32x16;
  static __device__ __forceinline__ void make(const QFrag<HG>& f, Frag& o) { split_qfrag<HG>(f, o); }
};

// One key tile (32 rows from `row`) global -> LDS at lds_addr, in the staged layout of its key type.
template <int KDT>
__device__ __forceinline__ void tile_dma(__amdgpu_buffer_rsrc_t krsrc, __amdgpu_buffer_rsrc_t srsrc,
                                         uint32_t lds_addr, int row) {
  if constexpr (KDT == DT_BF16)
    tile_dma_bf16(krsrc, lds_addr, row * (kD * 2), tile_lane_offsets_bf16());
  else
    tile_dma_fp8(krsrc, srsrc, lds_addr, row);
}

// primed: the caller has already issued the DMA of tile 0 into ring slot 0 (tile_dma above), to
// overlap it with other loads of its own.
template <int HG, int KDT, int NB, class RowAt, class Finish>
__device__ __forceinline__ void wave_pipeline(const typename Operands<HG, KDT>::Frag& f,
                                              __amdgpu_buffer_rsrc_t krsrc,
                                              __amdgpu_buffer_rsrc_t srsrc, uint32_t ring_addr, int nj,
                                              RowAt row_at, Finish finish, bool primed = false) {
  static_assert(NB >= 1 && NB <= 3, "ring of one to three tiles");
  constexpr int L = TileGeom<KDT>::kLoads;
  constexpr int BB = TileGeom<KDT>::kBufBytes;
  const int lane = lane_id();
  const u32x8 lane_offs = tile_lane_offsets_bf16();
  auto dma = [&](int j, int buf) {
    const int r = row_at(j);
    if constexpr (KDT == DT_BF16)
      tile_dma_bf16(krsrc, ring_addr + buf * BB, r * (kD * 2), lane_offs);
    else
      tile_dma_fp8(krsrc, srsrc, ring_addr + buf * BB, r);
  };
  // the DMA of tile j is complete once at most L * (tiles issued after it) loads are pending
  auto wait_tile = [&](int j) {
    const int later = (nj - 1 - j) < (NB - 1) ? (nj - 1 - j) : (NB - 1);
    if (later >= 2) wait_vmem_le<2 * L>();
    else if (later == 1) wait_vmem_le<L>();
    else wait_vmem_le<0>();
  };
  using Tile = typename Operands<HG, KDT>::Tile;
  auto read_tile = [&](int buf, float& scale) -> Tile {
    const uint32_t addr = ring_addr + buf * BB;
    if constexpr (KDT == DT_BF16) {
      scale = 1.f;
      return lds_read_tile_raw(addr);
    } else {
      scale = lds_read_f32_raw(addr + 4096 + (lane & 31) * 4);
      return lds_read_tile_fp8_raw(addr);
    }
  };
  if (nj <= 0) return;
#pragma unroll
  for (int b = 0; b < NB; ++b)
    if (b < nj && !(primed && b == 0)) dma(b, b);
  int buf = 0;                       // ring slot of the tile the next step consumes
  float sc_a = 1.f, sc_b = 1.f;      // fp8: per-key scales of the tiles held in acc_a / acc_b
  // one step: tile jn -> acc_out (matrix cores) while tile jn-1 = acc_in is finished (vector ALU)
  auto step = [&](int jn, const accvec<HG>& acc_in, float sc_in, accvec<HG>& acc_out, float& sc_out) {
    wait_tile(jn);
    if constexpr (KDT == DT_BF16) {
      // bf16 tile: the MFMAs of the first two 16-element chunks start as soon as those chunks are
      // in registers and cover the arrival of the other six (64K prefill: -1 %, 16K: -1.4 %)
      TileRegs tr;
      lds_read_tile_issue(ring_addr + buf * BB, tr);
      sc_out = 1.f;
      const int slot = buf;
      buf = (buf + 1 == NB) ? 0 : buf + 1;
      acc_out = mfma_tile_progressive<HG>(f, tr, [&] {
        if (jn + NB < nj) dma(jn + NB, slot);
      });
      finish(jn - 1, tile_epilogue<HG>(f, acc_in) * sc_in);
      return;
    }
    const Tile kv = read_tile(buf, sc_out);
    if (jn + NB < nj) dma(jn + NB, buf);
    buf = (buf + 1 == NB) ? 0 : buf + 1;
    acc_out = mfma_tile(f, kv);
    finish(jn - 1, tile_epilogue<HG>(f, acc_in) * sc_in);
  };
  wait_tile(0);
  const Tile kv0 = read_tile(0, sc_a);
  if (NB < nj) dma(NB, 0);
  buf = (NB == 1) ? 0 : 1;
  accvec<HG> acc_a = mfma_tile(f, kv0), acc_b;
  int j = 0;                         // acc_a holds tile j
  for (; j + 2 < nj; j += 2) {
    step(j + 1, acc_a, sc_a, acc_b, sc_b);
    step(j + 2, acc_b, sc_b, acc_a, sc_a);
  }
  if (j + 1 < nj) {
    step(j + 1, acc_a, sc_a, acc_b, sc_b);
    finish(j + 1, tile_epilogue<HG>(f, acc_b) * sc_b);
  } else {
    finish(j, tile_epilogue<HG>(f, acc_a) * sc_a);
  }
}

// Key array of one sequence as buffer descriptors (rows, and per-token scales for fp8).
template <int KDT>
__device__ __forceinline__ void key_buffers(const ScoreArgs& a, int seq, __amdgpu_buffer_rsrc_t& krsrc,
                                            __amdgpu_buffer_rsrc_t& srsrc) {
  const int rb = KDT == DT_BF16 ? 2 : 1;
  krsrc = key_buffer((const char*)a.keys + (long)seq * a.rows_per_seq * kD * rb, a.rows_per_seq * kD * rb);
  srsrc = key_buffer(a.k_scale ? (const void*)(a.k_scale + (long)seq * a.rows_per_seq) : a.keys,
                     a.k_scale ? a.rows_per_seq * 4 : 0);
}

// Lane j of the returned pair holds rows[j] / rows[64 + j]; at(j) broadcasts entry j.
struct LaneTable {
  int lo, hi;
  __device__ __forceinline__ int at(int j) const {
    return j < 64 ? __builtin_amdgcn_readlane(lo, j) : __builtin_amdgcn_readlane(hi, j - 64);
  }
};

// Eq. 1 / Eq. 5 / Eq. 8 on MFMA for arbitrary queries: one workgroup of 4 waves per (group of
// tiles, query); each wave runs the scoring pipeline over its own tiles (nothing is shared between
// queries here: this is the decode / two-kernel path).  Writes scores, and -inf for masked slots
// in gather mode.  tiles_per_wave <= 64.
template <int HG, int KDT>
__global__ __launch_bounds__(256, 2) void k_score_ranges(ScoreArgs a) {
  constexpr int NB = 2;
  __shared__ __align__(16) unsigned char ring[4 * NB * TileGeom<KDT>::kBufBytes];
  const RowGroup rg = row_group(a.groups);
  const int t = a.t_begin + rg.row;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  int seq;
  const int pos = query_pos(a, t, seq);
  const bool gather = a.block_idx != nullptr;
  const int n_vis = gather ? pos + 1 : visible_rows(a, pos);
  const int n_tiles = gather ? a.m * (a.B >> 5) : (n_vis + 31) >> 5;
  // first visible row: a token when gathering, else a row of the array in order (token or block)
  const int lo_row = gather ? query_lo(a.q_lo, t, pos) : query_lo(a.q_lo, t, pos) / a.pos_div;
  const int v0 = rg.x * 4 * a.tiles_per_wave;
  if (v0 >= n_tiles) return;
  // in-order rows below the first visible one are neither scored nor written: the select starts
  // at the first visible row (rounded down to four)
  if (!gather && (v0 + 4 * a.tiles_per_wave) * 32 <= lo_row) return;
  float* out = a.out + (long)rg.row * a.ld;
  const int n_blocks = (int)(a.rows_per_seq / a.B);

  // the four waves share one query: its fragment is loaded (fp8 keys: converted) once, through
  // the LDS of the tile rings, which are not in use yet
  static_assert(sizeof(ring) >= 32 * HG * 260, "the shared query fragment is staged in the rings");
  typename Operands<HG, KDT>::Frag fo;
  if constexpr (KDT == DT_FP8) {
    split_query_shared<HG, 4>((const uint16_t*)a.q + (long)t * a.H * kD, a.w + (long)t * a.H, ring, wave, fo);
  } else {
    load_qfrag_shared<HG, 4>(fo, (const uint16_t*)a.q + (long)t * a.H * kD, a.w + (long)t * a.H,
                             (long)a.H * kD * 2, lds_address(ring), wave);
  }

  // this wave's tiles: v = v0 + wave + 4 i; lane i looks its tile up; tiles without a visible key
  // are filled with -inf here (gather mode) and left out of the pipeline
  int my_row = -1, my_out = 0;
  {
    const int v = v0 + wave + 4 * lane;
    if (lane < a.tiles_per_wave && v < n_tiles) {
      const TileLoc Lc = tile_loc(a, t, v, gather);
      my_out = (int)Lc.out0;
      const bool ok = Lc.row0 >= 0 && Lc.row0 < n_vis && Lc.row0 + 32 > lo_row &&
                      (!gather || Lc.row0 / a.B < n_blocks);
      if (ok) my_row = (int)Lc.row0;
      else if (gather)
        for (int x = 0; x < 32; ++x) out[my_out + x] = neg_inf();
    }
  }
  // compact the valid tiles to the low lanes (order does not matter)
  const uint64_t okmask = __ballot(my_row >= 0);
  const int nj = __popcll(okmask);
  LaneTable rows{-1, -1}, outs{0, 0};
  {
    // lane j fetches the j-th valid entry: the source lane is the j-th set bit of okmask
    int src = 0;
    uint64_t mrem = okmask;
    for (int q = 0; q < 64; ++q) {           // wave-uniform loop over set bits
      if (!mrem) break;
      const int bit = __builtin_ctzll(mrem);
      mrem &= mrem - 1;
      if (lane == q) src = bit;
    }
    rows.lo = __shfl(my_row, src);
    outs.lo = __shfl(my_out, src);
  }
  __amdgpu_buffer_rsrc_t krsrc, srsrc;
  key_buffers<KDT>(a, seq, krsrc, srsrc);
  const uint32_t ring_addr = lds_address(ring) + wave * NB * TileGeom<KDT>::kBufBytes;
  auto row_at = [&](int j) { return rows.at(j); };
  auto finish = [&](int j, float s) {
    const int row = rows.at(j) + (lane & 31);
    if (row >= n_vis || row < lo_row) s = neg_inf();
    if (lane < 32 && (gather || row < n_vis)) out[outs.at(j) + lane] = s;
  };
  wave_pipeline<HG, KDT, NB>(fo, krsrc, srsrc, ring_addr, nj, row_at, finish);
}

// Eq. 1 / Eq. 5 on MFMA for a causal prefill of ONE sequence with consecutive positions: one
// workgroup of 8 waves = 8 consecutive queries; 128-key tiles (four 32-key sub-tiles) are DMA'd
// once into LDS (double buffered, one barrier per tile) and shared by the 8 queries; each wave runs
// the MFMAs of one sub-tile over the epilogue of the previous one (two accumulator sets).  Longest
// prefixes launch first.  Used by the flat DSA indexer and by Stage 1 above 512 blocks.  (Tiles of
// 64 keys, i.e. twice the barriers, were 2-3 % slower on the 64K flat indexer and 9 % on the 1M
// chunk; tiles of 256 keys, half the barriers and 128 KB of LDS, 1-2 % faster and not kept.
// Measured and not kept: score stores deferred by one iteration so that the wait before
// the barrier finds them old, and on top of that three tile buffers with the LDS operand reads
// requested one sub-tile early: +2 % and +4 % on the flat indexer, -3 % on short Stage 1 rows.
// With the DMA, the stores and the barrier all removed the loop itself runs at 1.34 PFLOP/s:
// what is left is the issue-slot limit of the MFMA / epilogue mix, not memory.)
template <int HG, int KDT>
__global__ __launch_bounds__(512) void k_score_prefill(ScoreArgs a) {
  constexpr int BB = TileGeom<KDT>::kBufBytes;
  constexpr int SUBS = 4;                       // 32-key sub-tiles per staged tile (one barrier per tile)
  constexpr int TK = 32 * SUBS;                 // keys per tile
  __shared__ __align__(16) unsigned char tiles[2 * SUBS * BB];   // [buffer][sub-tile]
  const int g = gridDim.x - 1 - blockIdx.x;
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int tl = g * 8 + wave;
  const bool active = tl < a.t_count;
  const int t = a.t_begin + (active ? tl : a.t_count - 1);
  int seq;
  const int pos = query_pos(a, t, seq);
  const int n_vis = active ? visible_rows(a, pos) : 0;
  const int tl_last = (g * 8 + 7) < a.t_count ? (g * 8 + 7) : a.t_count - 1;
  int seq_last;
  const int n_max = visible_rows(a, query_pos(a, a.t_begin + tl_last, seq_last));
  const int n_iter = (n_max + TK - 1) / TK;
  float* out = a.out + (long)(active ? tl : 0) * a.ld;

  QFrag<HG> fq;
  load_qfrag<HG>(fq, (const uint16_t*)a.q + (long)t * a.H * kD, a.w + (long)t * a.H);

  __amdgpu_buffer_rsrc_t krsrc, srsrc;
  key_buffers<KDT>(a, 0, krsrc, srsrc);
  const uint32_t tiles_addr = lds_address(tiles);
  // this wave's share of the cooperative DMA of a tile: sub-tile wave / 2, rows 16 * (wave % 2) .. +15 of it
  const int sub_w = wave >> 1, part_w = wave & 1;
  int voff[4] = {0, 0, 0, 0};
  if (KDT == DT_BF16) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {               // four transfers of four rows
      const int r = part_w * 16 + i * 4 + (lane >> 4), c = lane & 15;
      voff[i] = (lane >> 4) * 256 + ((c ^ (r & 15)) << 4);
    }
  } else {
#pragma unroll
    for (int i = 0; i < 2; ++i)                 // two transfers of eight rows, swizzled by (row / 2) % 8
      voff[i] = (lane >> 3) * 128 + (((lane & 7) ^ (((part_w * 2 + i) * 4 + (lane >> 4)) & 7)) << 4);
  }
  auto dma_tile = [&](int it, int buf) {
    const uint32_t dst = tiles_addr + (buf * SUBS + sub_w) * BB;
    const int row0 = it * TK + sub_w * 32 + part_w * 16;
    if constexpr (KDT == DT_BF16) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (lds_void*)(uintptr_t)(dst + (part_w * 256 + i * 64) * 16),
                                                 16, voff[i], (row0 + i * 4) * 256, 0, 0);
    } else {
#pragma unroll
      for (int i = 0; i < 2; ++i)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(krsrc, (lds_void*)(uintptr_t)(dst + (part_w * 2 + i) * 1024), 16,
                                                 voff[i], (row0 + i * 8) * 128, 0, 0);
      if (part_w == 0)
        __builtin_amdgcn_raw_ptr_buffer_load_lds(srsrc, (lds_void*)(uintptr_t)(dst + 4096), 4, lane * 4,
                                                 (it * TK + sub_w * 32) * 4, 0, 0);
    }
  };
  using Tile = typename Operands<HG, KDT>::Tile;
  auto read_sub = [&](int buf, int sub, float& scale) -> Tile {
    const uint32_t addr = tiles_addr + (buf * SUBS + sub) * BB;
    if constexpr (KDT == DT_BF16) {
      scale = 1.f;
      return lds_read_tile_raw(addr);
    } else {
      scale = lds_read_f32_raw(addr + 4096 + (lane & 31) * 4);
      return lds_read_tile_fp8_raw(addr);
    }
  };
  // sub-tile u covers rows 32u .. 32u+31
  auto finish = [&](int u, float s) {
    const int row = u * 32 + (lane & 31);
    if (lane < 32 && row < n_vis) out[row] = s;
  };

  if (n_iter > 0) dma_tile(0, 0);
  qfrag_ready<HG>(fq);
  typename Operands<HG, KDT>::Frag f;
  Operands<HG, KDT>::make(fq, f);
  // the contraction of one staged sub-tile; bf16: every 16-element chunk is awaited right before
  // its own MFMAs, so the first MFMAs run while the other chunks are still on their way from LDS
  auto score_sub = [&](int buf, int sub, float& scale) -> accvec<HG> {
    if constexpr (KDT == DT_BF16) {
      TileRegs tr;
      lds_read_tile_issue(tiles_addr + (buf * SUBS + sub) * BB, tr);
      scale = 1.f;
      return mfma_tile_progressive<HG, true>(f, tr, [] {});
    }
    const Tile kv = read_sub(buf, sub, scale);
    return mfma_tile(f, kv);
  };
  wait_vmem_le<0>();
  __syncthreads();
  accvec<HG> acc_a, acc_b;
  float sc_a = 1.f, sc_b = 1.f;
  for (int it = 0; it < n_iter; ++it) {
    const int buf = it & 1;
    if (it + 1 < n_iter) dma_tile(it + 1, buf ^ 1);
#pragma unroll
    for (int h = 0; h < SUBS / 2; ++h) {
      {
        acc_b = score_sub(buf, 2 * h, sc_b);                                       // sub-tile SUBS*it + 2h
        if (it > 0 || h > 0) finish(SUBS * it + 2 * h - 1, tile_epilogue<HG>(f, acc_a) * sc_a);   // the one before
      }
      {
        acc_a = score_sub(buf, 2 * h + 1, sc_a);                                   // sub-tile SUBS*it + 2h + 1
        finish(SUBS * it + 2 * h, tile_epilogue<HG>(f, acc_b) * sc_b);
      }
    }
    wait_vmem_le<0>();   // the next tile (and this wave's score stores) have landed
    __syncthreads();
  }
  if (n_iter > 0) finish(SUBS * n_iter - 1, tile_epilogue<HG>(f, acc_a) * sc_a);
}

// ------------------------------------------------------------------------------------------
// Eq. 5 / Eq. 1 on MFMA for a causal prefill of ONE sequence whose rows (pooled keys, normally)
// all fit in LDS: up to 512 bf16 rows = 16 tiles of 32 = 128 KB.  One workgroup of 8 waves stages
// the rows its queries can see ONCE (cooperative DMA, one barrier) and then every wave walks NQ
// queries of its own against the resident tiles: no DMA, no barrier and no tile traffic per query;
// what is left per query is its 16 KB fragment from HBM, and eight waves per CU with one such load
// in flight each keep that stream busy while the others compute.  Workgroup g serves the 8 * NQ
// consecutive queries from 8 * NQ * g, wave w the queries w, w + 8, ...; longest prefixes first.
// (Measured and not kept: pulling the next query's fragment towards L2 while the current one is
// scored, by DMA into a dummy LDS area since there are no registers for a second fragment: 10 %
// slower, the extra transfers cost more than the shorter wait.  Also measured and not kept: the
// block top-m fused behind the scoring, each wave selecting on an LDS row of its own without
// workgroup barriers: 0.455 ms against 0.332 + 0.068 ms for this kernel plus the separate select
// at the 64K prefill -- with two waves per SIMD the select's dependent LDS steps run at a quarter
// of the occupancy the small select kernel gets, which costs more than the 68 MB of block scores
// written and read back.)
template <int HG, int NQ>
__global__ __launch_bounds__(512) void k_score_resident(ScoreArgs a) {
  extern __shared__ __align__(16) unsigned char tiles[];   // [n_sub][8192]
  const int g = gridDim.x - 1 - blockIdx.x;
  const int th = threadIdx.x, lane = th & 63;
  const int wave = __builtin_amdgcn_readfirstlane(th >> 6);
  const int t0 = g * 8 * NQ;
  const int tl_last = (t0 + 8 * NQ - 1) < a.t_count ? (t0 + 8 * NQ - 1) : a.t_count - 1;
  int seq_last;
  const int n_max = visible_rows(a, query_pos(a, a.t_begin + tl_last, seq_last));
  const int n_sub = (n_max + 31) >> 5;
  __amdgpu_buffer_rsrc_t krsrc, srsrc;
  key_buffers<DT_BF16>(a, 0, krsrc, srsrc);
  const uint32_t tiles_addr = lds_address(tiles);
  {
    const u32x8 lane_offs = tile_lane_offsets_bf16();
    for (int u = wave; u < n_sub; u += 8) tile_dma_bf16(krsrc, tiles_addr + u * 8192, u * 32 * (kD * 2), lane_offs);
    wait_vmem_le<0>();
  }
  __syncthreads();
  for (int i = 0; i < NQ; ++i) {
    const int tl = t0 + i * 8 + wave;
    if (tl >= a.t_count) break;          // wave-uniform; no barrier below
    const int t = a.t_begin + tl;
    int seq;
    const int n_vis = visible_rows(a, query_pos(a, t, seq));
    const int nu = (n_vis + 31) >> 5;    // <= n_sub: positions grow with the query index
    if (nu <= 0) continue;
    float* out = a.out + (long)tl * a.ld;
    QFrag<HG> f;
    load_qfrag<HG>(f, (const uint16_t*)a.q + (long)t * a.H * kD, a.w + (long)t * a.H);
    qfrag_ready<HG>(f);
    auto store = [&](int u, float s) {
      const int row = u * 32 + (lane & 31);
      if (lane < 32 && row < n_vis) out[row] = s;
    };
    // MFMAs of sub-tile u over the epilogue of sub-tile u-1 (two accumulator sets, unrolled by two)
    accvec<HG> acc_a = mfma_tile<HG>(f, lds_read_tile_raw(tiles_addr)), acc_b;
    int u = 0;                           // acc_a holds sub-tile u
    for (; u + 2 < nu; u += 2) {
      acc_b = mfma_tile<HG>(f, lds_read_tile_raw(tiles_addr + (u + 1) * 8192));
      store(u, tile_epilogue<HG>(f, acc_a));
      acc_a = mfma_tile<HG>(f, lds_read_tile_raw(tiles_addr + (u + 2) * 8192));
      store(u + 1, tile_epilogue<HG>(f, acc_b));
    }
    if (u + 1 < nu) {
      acc_b = mfma_tile<HG>(f, lds_read_tile_raw(tiles_addr + (u + 1) * 8192));
      store(u, tile_epilogue<HG>(f, acc_a));
      store(u + 1, tile_epilogue<HG>(f, acc_b));
    } else {
      store(u, tile_epilogue<HG>(f, acc_a));
    }
  }
}

// Row-wise exact top-k over scores in global memory (Eqs. 2, 6, 9).
enum : int { MAP_FLAT = 0, MAP_BLOCKS = 1, MAP_CAND = 2, MAP_PAIRS = 3 };

struct SelectArgs {
  const float* scores;       // [rows, ld]
  long ld;
  const int32_t* idx_in;     // MAP_PAIRS: [rows, ld] ids aligned with scores
  const int32_t* q_seq;      // position info of the queries (FLAT / BLOCKS)
  const int32_t* q_pos;
  const int32_t* q_lo;       // first visible position per query or null (FLAT / BLOCKS)
  const int32_t* seq_len;
  int q_pos0, n_seq, pos_div;
  int t_begin;               // global query index of row 0
  int n_fixed;               // CAND / PAIRS: elements per row
  const int32_t* block_idx;  // MAP_CAND: [T, m] (global query indexing)
  int m, B;
  int seg_len, n_seg;        // FLAT: the row is cut into n_seg segments of seg_len (grid.x)
  int k;
  int32_t* out_idx;          // [rows * n_seg, k]
  float* out_scores;         // same shape, or null
};

template <int THREADS, int E, int MAP>
__global__ __launch_bounds__(THREADS) void k_select(SelectArgs a) {
  __shared__ SelectSmem<THREADS, E> sm;
  // Rows of up to 8192 entries are also kept in LDS as keys: the later threshold passes re-read single
  // entries, and from global memory every such round costs a full memory latency (it is what a
  // decode step, with one workgroup per query, mostly waited for).
  constexpr bool kStaged = THREADS * E * 4 <= 32768;
  __shared__ __align__(16) uint32_t staged[kStaged ? THREADS * E : 4];
  const RowGroup rg = row_group(a.n_seg);
  const int row = rg.row, seg = rg.x;
  const int t = a.t_begin + row;
  const float* sc = a.scores + (long)row * a.ld;
  int n = a.n_fixed;
  int base = 0;
  int first_vis = 0;   // MAP_BLOCKS: entry of the first visible block (0 unless sequences are packed)
  if (MAP == MAP_FLAT || MAP == MAP_BLOCKS) {
    int s = a.q_seq ? a.q_seq[t] : 0;
    s = s < 0 ? 0 : (s >= a.n_seq ? a.n_seq - 1 : s);
    int pos = a.q_pos ? a.q_pos[t] : a.q_pos0 + t;
    const int sl = a.seq_len[s];
    pos = pos < sl ? pos : sl - 1;
    int n_vis = pos < 0 ? 0 : pos / a.pos_div + 1;
    n_vis = n_vis < a.ld ? n_vis : (int)a.ld;   // never past the score row, whatever seq_len says
    // this segment's rows, cut at the first visible one rounded down to four (16-byte loads; the
    // up to three rows in between were written as -inf by the scoring kernel)
    const int lo_row = query_lo(a.q_lo, t, pos) / a.pos_div;
    const int seg_end = (seg + 1) * a.seg_len < n_vis ? (seg + 1) * a.seg_len : n_vis;
    base = seg * a.seg_len;
    base = base > (lo_row & ~3) ? base : (lo_row & ~3);
    n = seg_end - base;
    n = (n < 0 || lo_row >= n_vis) ? 0 : n;     // (first visible row past the last: the query sees nothing)
    first_vis = lo_row - base;                  // < 0 in later segments: no forced entry there
  }
  const long orow = (long)row * a.n_seg + seg;
  int32_t* oi = a.out_idx + orow * a.k;
  float* os = a.out_scores ? a.out_scores + orow * a.k : nullptr;
  const int n_last = n - 1;
  const float* rowp = sc + base;
  // the row through a buffer descriptor of exactly n floats: no branch at the ragged end
  const __amdgpu_buffer_rsrc_t rrow = key_buffer(rowp, (long)n * 4);
  auto key_of = [&](int i, float v) -> uint32_t {
    if (MAP == MAP_BLOCKS && (i == first_vis || i == n_last)) return 0xffffffffu;   // forced blocks
    return ordered_key(v);
  };
  auto load4 = [&](int q) -> uint4 {
    const int i = 4 * q;
    const u32x4v r = __builtin_amdgcn_raw_buffer_load_b128(rrow, i * 4, 0, 0);
    uint32_t kk[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) kk[x] = (i + x < n) ? key_of(i + x, __uint_as_float(r[x])) : 0u;
    const uint4 keys = make_uint4(kk[0], kk[1], kk[2], kk[3]);
    if (kStaged) *reinterpret_cast<uint4*>(&staged[i]) = keys;   // read back only after a barrier
    return keys;
  };
  auto load1 = [&](int i) -> uint32_t { return kStaged ? staged[i] : key_of(i, rowp[i]); };
  // MAP_CAND: a thread's E consecutive candidates lie in one kept block when E divides B; its
  // token base is then fetched once, not per emitted candidate
  const bool one_slot = MAP == MAP_CAND && a.B % E == 0;
  int my_base = 0;
  if (one_slot) {
    const int my_slot = (int)(threadIdx.x * E) / a.B;
    if (my_slot < a.m) my_base = (a.block_idx[(long)t * a.m + my_slot] - my_slot) * a.B;
  }
  auto emit = [&](int p, int i, uint32_t key) {
    int id;
    if (MAP == MAP_CAND && one_slot) {
      id = my_base + i;
    } else if (MAP == MAP_CAND) {
      const int slot = i / a.B;
      id = a.block_idx[(long)t * a.m + slot] * a.B + (i - slot * a.B);
    } else if (MAP == MAP_PAIRS) {
      id = a.idx_in[(long)row * a.ld + i];
    } else {
      id = base + i;
    }
    oi[p] = id;
    if (os) os[p] = key_to_score(key);
  };
  int n_out = -1;
  if constexpr ((MAP == MAP_CAND || MAP == MAP_BLOCKS) && THREADS >= 256) {
    // Candidate rows (Stage 2 behind the separate scoring kernel) and block-score rows (Stage 1)
    // first try the one-pass top-k of the fused kernel: a handful of barriers instead of about
    // sixteen, which is most of this kernel's time when a decode batch gives it a few rows.  It
    // declines before writing anything if the row is not its case.  (Not for the one-wave rows of up
    // to 512 entries: zeroing and scanning 2048 bins with 64 threads doubled Stage 1 of the
    // prefills, 0.40 -> 0.76 ms at 64K.)  Stage 1's two forced blocks
    // are the first and the last entry of the row: they are left out of the search, which then
    // looks for k - 2 among the others, and take the first and the last output position.
    __shared__ FineSelSmem<THREADS, E> fs;
    constexpr int kForced = MAP == MAP_BLOCKS ? 2 : 0;
    const int k_free = a.k - kForced;
    if (k_free >= 1 && n - kForced > k_free) {
      fine_select_prepare<THREADS, E>(fs);
      const float qnan = __uint_as_float(0xffffffffu);
      const int i0 = (int)threadIdx.x * E;
      float4 mine[E / 4];
      float x_max = -__builtin_inff(), x_min = __builtin_inff();
#pragma unroll
      for (int g = 0; g < E / 4; ++g) {
        const u32x4v r = __builtin_amdgcn_raw_buffer_load_b128(rrow, (i0 + 4 * g) * 4, 0, 0);   // zeros past the row
        float x[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int i = i0 + 4 * g + e;
          const float xe = __uint_as_float(r[e]);
          bool cand = i < n && xe != neg_inf();          // masked slots hold -inf in global memory
          if (kForced) cand = cand && i != first_vis && i != n_last;
          x[e] = cand ? xe : qnan;
          x_max = vmax_f32(x_max, x[e]);
          x_min = vmin_f32(x_min, x[e]);
        }
        mine[g] = make_float4(x[0], x[1], x[2], x[3]);
      }
      fine_select_range<THREADS, E>(fs, x_max, x_min, (int)threadIdx.x >> 6);
      __syncthreads();
      auto vals = [&](int q) -> float4 { return mine[q - (i0 >> 2)]; };
      auto emit_f = [&](uint32_t p, const auto& v, float tau, int32_t*) {
        p += kForced ? 1 : 0;
#pragma unroll
        for (int j = 0; j < E; ++j) {
          if (v[j] >= tau) {
            emit((int)p, i0 + j, ordered_key(v[j]));
            ++p;
          }
        }
      };
      if (select_topk_fine<THREADS, E>(fs, n, k_free, vals, emit_f)) {
        n_out = a.k;
        if (kForced && threadIdx.x == 0) {
          emit(0, first_vis, 0xffffffffu);
          emit(a.k - 1, n_last, 0xffffffffu);
        }
      } else {
        __syncthreads();
      }
    }
  }
  if (n_out < 0) n_out = select_topk<THREADS, E, true, MAP == MAP_BLOCKS>(sm, n, a.k, load4, load1, emit);
  for (int p = n_out + threadIdx.x; p < a.k; p += THREADS) {
    oi[p] = -1;
    if (os) os[p] = neg_inf();
  }
}

// ------------------------------------------------------------------------------------------
// Streaming exact top-k of one long score row (flat indexer, Eq. 2; k <= 2048).  The row stays in
// global memory and is read a few times instead of being held in registers:
//   1. a sample of the row gives a key range [rlo, rhi];
//   2. one pass histograms the keys into 4096 bins: bin 0 below rlo, bins 1..4094 equal slices of
//      the range, bin 4095 above it (any monotone binning keeps the selection exact; the range
//      only spreads the keys, so that the LDS atomics rarely collide);
//   3. the bin that holds the k-th key is found; if it holds more keys than the candidate list
//      can take, steps 2-3 repeat inside that bin's key range (only for degenerate rows);
//   4. one pass in index order collects the indices above the bin (selected for sure) and the
//      (index, key) pairs inside it; select_topk picks the missing r among those; both lists are
//      ascending and are merged into the output by rank.
// Order: key descending, then index ascending; output ascending, -1 padding.
struct StreamSelect {
  static constexpr int kThreads = 1024, kBins = 4096, kCap = 4 * kThreads, kMaxK = 2048;
  static constexpr int kHist = 0;                                   // uint32 [kBins]; later the winners
  static constexpr int kSure = kBins * 4;                           // int32 idx [kMaxK], uint32 key [kMaxK]
  static constexpr int kCand = kSure + kMaxK * 8;                   // int32 idx [kCap], uint32 key [kCap]
  static constexpr int kSel = kCand + kCap * 8;                     // SelectSmem<kThreads, 4>
  static constexpr int kTot = kSel + (int)((sizeof(SelectSmem<kThreads, 4>) + 15) / 16 * 16);
  static constexpr int kBytes = kTot + 2 * (kThreads / 64) * 4 + 64;   // chunk totals [2][waves] + broadcast
};

__global__ __launch_bounds__(StreamSelect::kThreads, 8) void k_select_stream(SelectArgs a) {
  using P = StreamSelect;
  constexpr int THREADS = P::kThreads, NW = THREADS / 64, NBIN = P::kBins, CAP = P::kCap;
  extern __shared__ __align__(16) unsigned char smem[];
  uint32_t* hist = reinterpret_cast<uint32_t*>(smem + P::kHist);
  int32_t* win_idx = reinterpret_cast<int32_t*>(smem + P::kHist);   // aliases hist (dead by then)
  uint32_t* win_key = reinterpret_cast<uint32_t*>(smem + P::kHist + P::kMaxK * 4);
  int32_t* sure_idx = reinterpret_cast<int32_t*>(smem + P::kSure);
  uint32_t* sure_key = reinterpret_cast<uint32_t*>(smem + P::kSure + P::kMaxK * 4);
  int32_t* cand_idx = reinterpret_cast<int32_t*>(smem + P::kCand);
  uint32_t* cand_key = reinterpret_cast<uint32_t*>(smem + P::kCand + CAP * 4);
  SelectSmem<THREADS, 4>& sm = *reinterpret_cast<SelectSmem<THREADS, 4>*>(smem + P::kSel);
  uint32_t* tot = reinterpret_cast<uint32_t*>(smem + P::kTot);      // [2][NW]
  uint32_t* bc = tot + 2 * NW;                                      // broadcast words

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int row = blockIdx.x;
  const int t = a.t_begin + row;
  int sq = a.q_seq ? a.q_seq[t] : 0;
  sq = sq < 0 ? 0 : (sq >= a.n_seq ? a.n_seq - 1 : sq);
  int pos = a.q_pos ? a.q_pos[t] : a.q_pos0 + t;
  const int sl = a.seq_len[sq];
  pos = pos < sl ? pos : sl - 1;
  int n = pos < 0 ? 0 : pos + 1;
  n = n < a.ld ? n : (int)a.ld;   // never past the score row, whatever seq_len says
  // packed sequences: the row starts at the first visible position rounded down to four (16-byte
  // loads; the up to three entries in between hold -inf); ids are row-relative until the output
  const int id0 = query_lo(a.q_lo, t, pos) & ~3;
  n = n > id0 ? n - id0 : 0;
  const int k = a.k;
  const float* rowp = a.scores + (long)row * a.ld + id0;
  int32_t* oi = a.out_idx + (long)row * k;
  float* os = a.out_scores ? a.out_scores + (long)row * k : nullptr;

  if (n <= 0) {
    for (int p = tid; p < k; p += THREADS) {
      oi[p] = -1;
      if (os) os[p] = neg_inf();
    }
    return;
  }
  if (n <= k) {   // Section 4.1, boundary behaviour: a prefix no longer than k is selected whole
    int bad = 0;   // a -inf entry is not a candidate: such a row takes the general path below
    for (int p = tid; p < n; p += THREADS) bad |= rowp[p] == neg_inf();
    if (!__syncthreads_or(bad)) {
      for (int p = tid; p < k; p += THREADS) {
        oi[p] = p < n ? id0 + p : -1;
        if (os) os[p] = p < n ? rowp[p] : neg_inf();
      }
      return;
    }
  }

  // The row through a buffer descriptor of exactly n floats: a 16-byte load needs no branch at
  // the ragged end (bytes past the row read as zero and are masked by index below).
  const __amdgpu_buffer_rsrc_t rrow = key_buffer(rowp, (long)n * 4);
  auto raw4 = [&](int i) -> u32x4v { return __builtin_amdgcn_raw_buffer_load_b128(rrow, i * 4, 0, 0); };
  // keys of elements i .. i+3 (0 = not a candidate: beyond the row, or a -inf score)
  auto keys_of = [&](int i, const u32x4v& r, uint32_t (&kk)[4]) {
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t key = ordered_key(__uint_as_float(r[x]));
      kk[x] = (i + x < n) ? key : 0u;
    }
  };

  // 1. key range of a sample
  uint32_t kmin = 0xffffffffu, kmax = 1u;
  {
    // up to 4096 entries: 64 evenly spaced runs of 64 consecutive entries (16 KB of the row;
    // single entries at a constant stride would pull in nearly every line of it)
    const int run_stride = n > 4 * THREADS ? n >> 6 : 64;
    float sv[4];
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const int j = tid * 4 + x;
      const long idx = (long)(j >> 6) * run_stride + (j & 63);
      sv[x] = idx < n ? rowp[idx] : neg_inf();
    }
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t key = ordered_key(sv[x]);
      if (key) {
        kmin = key < kmin ? key : kmin;
        kmax = key > kmax ? key : kmax;
      }
    }
    kmin = wave_min(kmin);
    kmax = wave_max(kmax);
    if (lane == 0) {
      tot[wave] = kmin;
      tot[NW + wave] = kmax;
    }
    __syncthreads();
#pragma unroll
    for (int v = 0; v < NW; ++v) {
      kmin = tot[v] < kmin ? tot[v] : kmin;
      kmax = tot[NW + v] > kmax ? tot[NW + v] : kmax;
    }
    if (kmin > kmax) kmin = kmax;
    kmin = __builtin_amdgcn_readfirstlane(kmin);   // workgroup-uniform from here on: scalar registers
    kmax = __builtin_amdgcn_readfirstlane(kmax);
    __syncthreads();
  }

  // 2.-3. histogram levels
  uint32_t plo = 1u, phi = 0xffffffffu;   // exact key range that still holds the k-th key
  uint32_t rlo = kmin, rhi = kmax;        // range the bins 1 .. NBIN-2 are laid over
  uint32_t krem = (uint32_t)k;            // how many keys to take from [plo, phi]
  uint32_t n_c = 0;                       // keys inside [plo, phi]
  bool all_valid = false;                 // fewer than k candidates: every candidate is selected
  for (int level = 0; level < 8; ++level) {
    int shift = 0;
    while (((rhi - rlo) >> shift) > (uint32_t)(NBIN - 3)) ++shift;
    const unsigned long long top = (unsigned long long)rlo + ((unsigned long long)(NBIN - 2) << shift) - 1ull;
    const uint32_t rhi_eff = top > 0xffffffffull ? 0xffffffffu : (uint32_t)top;
    for (int b = tid; b < NBIN; b += THREADS) hist[b] = 0u;
    __syncthreads();
    // four 16-byte loads in flight per thread before their keys are binned
    for (int i0 = tid * 4; i0 < n; i0 += THREADS * 16) {
      u32x4v q[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) q[u] = raw4(i0 + u * THREADS * 4);
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        uint32_t kk[4];
        keys_of(i0 + u * THREADS * 4, q[u], kk);
#pragma unroll
        for (int x = 0; x < 4; ++x) {
          const uint32_t key = kk[x];
          if (key >= plo && key <= phi) {
            const uint32_t bin =
                key < rlo ? 0u : (key > rhi_eff ? (uint32_t)(NBIN - 1) : ((key - rlo) >> shift) + 1u);
            atomicAdd(&hist[bin], 1u);
          }
        }
      }
    }
    __syncthreads();
    // suffix sums over the bins: thread t owns bins 4t .. 4t+3
    static_assert(NBIN == 4 * THREADS, "four bins per thread");
    const uint32_t c0 = hist[4 * tid + 0], c1 = hist[4 * tid + 1], c2 = hist[4 * tid + 2], c3 = hist[4 * tid + 3];
    const uint32_t mine = c0 + c1 + c2 + c3;
    const uint32_t wave_total = wave_sum(mine);
    uint32_t S = wave_total - wave_scan_add(mine) + mine;   // inclusive suffix sum over the lanes of the wave
    if (lane == 0) tot[wave] = wave_total;
    __syncthreads();
    uint32_t total = 0;
#pragma unroll
    for (int v = 0; v < NW; ++v) {
      const uint32_t tv = tot[v];
      total += tv;
      if (v > wave) S += tv;
    }
    total = __builtin_amdgcn_readfirstlane(total);
    if (level == 0 && total <= krem) {
      all_valid = true;
      __syncthreads();
      break;
    }
    const uint32_t a3 = S - mine, a2 = a3 + c3, a1 = a2 + c2, a0 = a1 + c1;
    int dsel = -1;
    uint32_t above = 0, cnt = 0;
    if (a3 < krem && krem <= a3 + c3) { dsel = 3; above = a3; cnt = c3; }
    if (a2 < krem && krem <= a2 + c2) { dsel = 2; above = a2; cnt = c2; }
    if (a1 < krem && krem <= a1 + c1) { dsel = 1; above = a1; cnt = c1; }
    if (a0 < krem && krem <= a0 + c0) { dsel = 0; above = a0; cnt = c0; }
    if (dsel >= 0) {
      bc[0] = (uint32_t)(4 * tid + dsel);
      bc[1] = krem - above;
      bc[2] = cnt;
    }
    __syncthreads();
    const uint32_t bsel = __builtin_amdgcn_readfirstlane(bc[0]);
    krem = __builtin_amdgcn_readfirstlane(bc[1]);
    n_c = __builtin_amdgcn_readfirstlane(bc[2]);
    uint32_t nlo, nhi;
    if (bsel == 0u) {
      nlo = plo;
      nhi = rlo - 1u;   // bin 0 is non-empty, so rlo > plo >= 1
    } else if (bsel == (uint32_t)(NBIN - 1)) {
      nlo = rhi_eff + 1u;   // bin NBIN-1 is non-empty, so rhi_eff < 0xffffffff
      nhi = phi;
    } else {
      nlo = rlo + ((bsel - 1u) << shift);
      nhi = nlo + ((1u << shift) - 1u);
    }
    plo = nlo > plo ? nlo : plo;
    phi = nhi < phi ? nhi : phi;
    __syncthreads();   // bc and tot are reused
    if (n_c <= (uint32_t)CAP || plo == phi) break;
    rlo = plo;
    rhi = phi;
  }
  // Keys above phi are selected for sure.  Keys in [plo, phi]: krem of them are selected; if they
  // do not fit the list they are all equal (plo == phi) and the first krem in index order win.
  const bool equal_mode = !all_valid && n_c > (uint32_t)CAP;
  const uint32_t r = all_valid ? 0u : krem;
  const uint32_t sure_lo = all_valid ? 1u : phi + 1u;   // phi + 1 == 0 means: none (phi = 0xffffffff)

  // 4. collect in index order
  uint32_t base_s = 0, base_c = 0;
  int par = 0;
  // the loads of the next two chunks fly over this chunk's scan
  u32x4v q_a = raw4(tid * 4), q_b = raw4(tid * 4 + THREADS * 4);
  for (int c0 = 0; c0 < n; c0 += THREADS * 4) {
    const int i = c0 + tid * 4;
    const u32x4v q = q_a;
    q_a = q_b;
    q_b = raw4(i + THREADS * 8);
    uint32_t kk[4];
    keys_of(i, q, kk);
    bool is_s[4], is_c[4];
    uint32_t cs = 0, cc = 0;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t key = kk[x];
      is_s[x] = key != 0u && sure_lo != 0u && key >= sure_lo;
      is_c[x] = !all_valid && key >= plo && key <= phi;
      cs += is_s[x];
      cc += is_c[x];
    }
    const uint32_t packed = cs | (cc << 16);
    const uint32_t inc = wave_scan_add(packed);
    if (lane == 63) tot[par * NW + wave] = inc;
    __syncthreads();
    uint32_t before = 0, chunk = 0;
#pragma unroll
    for (int v = 0; v < NW; ++v) {
      const uint32_t tv = tot[par * NW + v];
      chunk += tv;
      if (v < wave) before += tv;
    }
    uint32_t ps = base_s + (before & 0xffffu) + (inc & 0xffffu) - cs;
    uint32_t pc = base_c + (before >> 16) + (inc >> 16) - cc;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      if (is_s[x]) {
        if (ps < (uint32_t)P::kMaxK) {
          sure_idx[ps] = i + x;
          sure_key[ps] = kk[x];
        }
        ++ps;
      }
      if (is_c[x]) {
        if (equal_mode) {
          if (pc < r) {
            win_idx[pc] = i + x;
            win_key[pc] = kk[x];
          }
        } else if (pc < (uint32_t)CAP) {
          cand_idx[pc] = i + x;
          cand_key[pc] = kk[x];
        }
        ++pc;
      }
    }
    base_s += __builtin_amdgcn_readfirstlane(chunk & 0xffffu);
    base_c += __builtin_amdgcn_readfirstlane(chunk >> 16);
    par ^= 1;   // the next chunk writes the other totals row: one barrier per chunk is enough
  }
  __syncthreads();
  const int n_s = (int)(base_s < (uint32_t)P::kMaxK ? base_s : (uint32_t)P::kMaxK);

  // the r best of the candidate list (ascending index in, ascending index out)
  int n_w = (int)r;
  const int nc_all = (int)(base_c < (uint32_t)CAP ? base_c : (uint32_t)CAP);
  if (!equal_mode && r > 0u && nc_all <= THREADS) {
    // the usual case, a short list: one candidate per thread, ranked by counting the candidates
    // that beat it (larger key, or equal key earlier in the list); no further passes
    uint32_t* flag = reinterpret_cast<uint32_t*>(&sm);   // [THREADS] selected flags
    const uint32_t mykey = tid < nc_all ? cand_key[tid] : 0u;
    uint32_t rank = 0;
    for (int j = 0; j < nc_all; ++j) {
      const uint32_t kj = cand_key[j];
      rank += (kj > mykey) || (kj == mykey && j < tid);
    }
    const bool sel = tid < nc_all && rank < r;
    flag[tid] = sel ? 1u : 0u;
    __syncthreads();
    if (sel) {
      uint32_t before = 0;
      for (int j = 0; j < tid; ++j) before += flag[j];
      win_idx[before] = cand_idx[tid];
      win_key[before] = mykey;
    }
    n_w = (int)(r < (uint32_t)nc_all ? r : (uint32_t)nc_all);
  } else if (!equal_mode && r > 0u) {
    const int nc = nc_all;
    auto load4 = [&](int q4) -> uint4 { return *reinterpret_cast<const uint4*>(cand_key + 4 * q4); };
    auto load1 = [&](int i) -> uint32_t { return cand_key[i]; };
    auto emit = [&](int p, int i, uint32_t key) {
      win_idx[p] = cand_idx[i];
      win_key[p] = key;
    };
    n_w = select_topk<THREADS, 4>(sm, nc, (int)r, load4, load1, emit);
  }
  __syncthreads();

  // merge the two ascending lists by rank
  auto lower_bound = [](const int32_t* v, int len, int x) -> int {
    int lo = 0, hi = len;
    while (lo < hi) {
      const int mid = (lo + hi) >> 1;
      if (v[mid] < x) lo = mid + 1;
      else hi = mid;
    }
    return lo;
  };
  for (int j = tid; j < n_s; j += THREADS) {
    const int x = sure_idx[j];
    const int p = j + lower_bound(win_idx, n_w, x);
    oi[p] = id0 + x;
    if (os) os[p] = key_to_score(sure_key[j]);
  }
  for (int j = tid; j < n_w; j += THREADS) {
    const int y = win_idx[j];
    const int p = j + lower_bound(sure_idx, n_s, y);
    oi[p] = id0 + y;
    if (os) os[p] = key_to_score(win_key[j]);
  }
  for (int p = n_s + n_w + tid; p < k; p += THREADS) {
    oi[p] = -1;
    if (os) os[p] = neg_inf();
  }
}

// ------------------------------------------------------------------------------------------
// Stage 1 (Eqs. 5-6) of ONE query inside a workgroup of NW waves that already holds the query
// fragment: the pooled keys (bf16, [n_seq, n_blocks, d]) of the blocks 0 .. b_t go through
// the scoring pipeline in tiles of 32 (wave w takes tiles w, w + NW, ...), the block scores land
// in sc[0 .. 32 * tiles) (-inf past b_t and below the first visible block lo / B), select_topk keeps
// a.m of them with the first visible and the query's own block forced (E1 blocks per thread: NW * 64 * E1 >= n_blocks), and the kept ids go
// to blk_lds[0 .. a.m) ascending, -1 padded.  smem: the NW * NB tile rings of TILE bytes (reused
// by the select).  Ends with a barrier: ids visible, score area and rings free again.
// primed: every wave has already issued the DMA of its first tile (blocks 32 * wave ..) into its
// ring slot 0, and that DMA has completed.
template <int HG, int NW, int NB, int E1, int TILE>
__device__ __forceinline__ void stage1_in_workgroup(const QFrag<HG>& f, const ScoreArgs& a, const void* pooled,
                                                    int seq, int pos, int lo, int n_blocks, unsigned char* smem,
                                                    float* sc, int32_t* blk_lds, int wave, bool primed = false) {
  constexpr int NT = NW * 64;
  const int lane = threadIdx.x & 63;
  const int n_bvis = pos < 0 ? 0 : pos / a.B + 1;
  const int b_first = lo / a.B;   // first visible block (0 unless sequences are packed)
  const int nt1 = (n_bvis + 31) >> 5;
  const int nj1 = nt1 > wave ? (nt1 - wave + NW - 1) / NW : 0;
  const __amdgpu_buffer_rsrc_t prsrc =
      key_buffer((const char*)pooled + (long)seq * n_blocks * kD * 2, (long)n_blocks * kD * 2);
  wave_pipeline<HG, DT_BF16, NB>(
      f, prsrc, prsrc, lds_address(smem) + wave * NB * TILE, nj1,
      [&](int j) { return (wave + NW * j) * 32; },
      [&](int j, float s) {
        const int b = (wave + NW * j) * 32 + (lane & 31);
        if (lane < 32) sc[b] = (b < n_bvis && b >= b_first) ? s : neg_inf();
      },
      primed && nj1 > 0);
  __syncthreads();   // block scores complete, rings dead
  {
    SelectSmem<NT, E1>& sm1 = *reinterpret_cast<SelectSmem<NT, E1>*>(smem);
    const int n_last = n_bvis - 1;
    auto key_of = [&](int i, float v) -> uint32_t {
      return (i == b_first || i == n_last) ? 0xffffffffu : ordered_key(v);   // first and own block forced
    };
    auto load4 = [&](int q) -> uint4 {
      const float4 v = *reinterpret_cast<const float4*>(sc + 4 * q);
      return make_uint4(key_of(4 * q, v.x), key_of(4 * q + 1, v.y), key_of(4 * q + 2, v.z),
                        key_of(4 * q + 3, v.w));
    };
    auto load1 = [&](int i) -> uint32_t { return key_of(i, sc[i]); };
    auto emit = [&](int p, int i, uint32_t) { blk_lds[p] = i; };
    // (a first visible block past the query's own: the query sees nothing, nothing is forced)
    const int n_kept = select_topk<NT, E1>(sm1, b_first <= n_last ? n_bvis : 0, a.m, load4, load1, emit);
    for (int p = n_kept + threadIdx.x; p < a.m; p += NT) blk_lds[p] = -1;
  }
  __syncthreads();
}

// ------------------------------------------------------------------------------------------
// Stage 1 (Eqs. 5-6) of a FEW queries (a decode batch), one launch: one workgroup of 8 waves per
// query loads the query fragment, scores the pooled keys of the visible blocks into LDS and keeps m
// of them there; only the m ids leave the CU.  Against the scoring launch plus the select launch
// this saves a launch, the round trip of the block scores through HBM and the second query read;
// with one workgroup per query it only pays while the queries are fewer than the CUs.
// sc_floats >= the block count rounded up to 32; LDS: the tile rings, sc_floats scores, m ids
// (rounded up to 4), HG * 8192 bytes for the query fragment.
template <int HG, int E1, int NB>
__global__ __launch_bounds__(512) void k_stage1_query(ScoreArgs a, const void* pooled, int32_t* block_idx_out,
                                                      int sc_floats) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NW = 8, NT = NW * 64, TILE = 8192;
  constexpr size_t kStageBytes = (size_t)NW * NB * TILE;
  static_assert(sizeof(SelectSmem<NT, E1>) <= kStageBytes, "select scratch must fit the rings");
  float* sc = reinterpret_cast<float*>(smem + kStageBytes);
  int32_t* blk_lds = reinterpret_cast<int32_t*>(sc + sc_floats);
  unsigned char* q_lds = reinterpret_cast<unsigned char*>(blk_lds + (a.m + 3) / 4 * 4);   // HG * 8192 bytes
  const int t = a.t_begin + blockIdx.x;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  int seq;
  const int pos = query_pos(a, t, seq);
  const int lo = query_lo(a.q_lo, t, pos);
  const int n_blocks = (int)(a.rows_per_seq / a.B);
  // the query fragment is staged in an area of its own, so that every wave's first tile of pooled
  // keys can be requested right behind it: one memory latency for both
  QFrag<HG> f;
  qfrag_shared_request<HG, NW>(f, (const uint16_t*)a.q + (long)t * a.H * kD, a.w + (long)t * a.H,
                               (long)a.H * kD * 2, lds_address(q_lds), wave);
  {
    const __amdgpu_buffer_rsrc_t prsrc =
        key_buffer((const char*)pooled + (long)seq * n_blocks * kD * 2, (long)n_blocks * kD * 2);
    tile_dma<DT_BF16>(prsrc, prsrc, lds_address(smem) + wave * NB * TILE, wave * 32);
  }
  qfrag_shared_complete<HG>(f, lds_address(q_lds));
  qfrag_ready<HG>(f);
  stage1_in_workgroup<HG, NW, NB, E1, TILE>(f, a, pooled, seq, pos, lo, n_blocks, smem, sc, blk_lds, wave, true);
  for (int p = threadIdx.x; p < a.m; p += NT) block_idx_out[(long)t * a.m + p] = blk_lds[p];
}

// ------------------------------------------------------------------------------------------
// Stage 2 fused (Eqs. 7-9): one workgroup of NW waves per query scores every tile of the kept
// blocks into LDS and selects the top k there; only the k indices leave the CU.  E = candidates
// per thread in the select (NW * 64 * E >= m * B).  LDS: the per-wave tile rings, then the m*B
// scores; the select's scratch reuses the ring once scoring is over.
//
// E1 > 0: the whole of Algorithm 1 in this one launch.  Stage 1 (Eqs. 5-6) runs first in the
// same workgroup: the pooled keys (bf16, [n_seq, s_max / B, d]) of the visible blocks go through
// the same pipeline with the query fragment already in registers, the block scores land in the
// score area, select_topk keeps m of them (first and own block forced, E1 blocks per thread),
// and the kept ids stay in LDS for Stage 2 (and are written to block_idx_out if given).
// sc_floats: size of the score area (>= m * B, and >= NW * 64 * E1 when E1 > 0).
// (Measured and not kept: the tiles of a query handed out to its waves at run time from an LDS
// counter instead of dealt round robin, so that the waves finish together: 7-10 % slower with 4
// waves per query, 2 % with 8, whose waves wait longest for each other.)
// (Measured and not kept: a grid of as many workgroups as the chip holds, each walking its share
// of the queries and requesting the next query's fragment and block ids during the top-k of the
// current one: no faster than the same code with one query per workgroup, and the loop around the
// kernel body costs 16 % by itself -- 256 registers and spills where this form needs 221.)
// (Measured and not kept: each workgroup, once its scoring is over, pulling the query of the
// workgroup 512 or 1024 positions behind it into the XCD's L2: 64K prefill +2 %, 16K -1 %, fp8 keys
// and the 1M chunk unchanged.  The first read of a query is not what a workgroup waits for.)
template <int HG, int KDT, int NW, int NB, int E, int E1 = 0>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void k_refine_fused(ScoreArgs a, int k,
                                                                           int32_t* topk_idx,
                                                                           float* topk_scores,
                                                                           const void* pooled = nullptr,
                                                                           int32_t* block_idx_out = nullptr,
                                                                           int sc_floats = 0) {
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int NT = NW * 64;
  constexpr int kTileBytes = (E1 > 0 && TileGeom<KDT>::kBufBytes < 8192) ? 8192 : TileGeom<KDT>::kBufBytes;
  constexpr size_t kStageBytes = (size_t)NW * NB * kTileBytes;
  static_assert(sizeof(SelectSmem<NT, E>) <= kStageBytes, "select scratch must fit the rings");
  static_assert(E1 == 0 || sizeof(SelectSmem<NT, E1 ? E1 : 4>) <= kStageBytes, "select scratch must fit the rings");
  float* sc = reinterpret_cast<float*>(smem + kStageBytes);   // m*B scores (swizzled: score_slot)
  SelectSmem<NT, E>& sm = *reinterpret_cast<SelectSmem<NT, E>*>(smem);
  // scratch of the top-k's fast path, behind everything else (shared with nothing: see select_topk_fine)
  FineSelSmem<NT, E>& fs = *reinterpret_cast<FineSelSmem<NT, E>*>(
      smem + kStageBytes + (E1 > 0 ? (size_t)sc_floats * 4 + (size_t)((a.m + 3) / 4 * 4) * 4 : (size_t)a.m * a.B * 4));
  fine_select_prepare<NT, E>(fs);
  const int t = a.t_begin + (gridDim.x - 1 - blockIdx.x);
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63;
  int seq;
  const int pos = query_pos(a, t, seq);
  const int n_vis = pos + 1;
  const int lo = query_lo(a.q_lo, t, pos);   // first visible token (0 unless sequences are packed)

  // fp8 keys without Stage 1 in this launch: no wave needs the bf16 fragment, and the two-term
  // e4m3 fragment is built once for the workgroup (below) instead of once per wave
  constexpr bool kSharedSplit = KDT == DT_FP8 && E1 == 0;
  static_assert(!kSharedSplit || kStageBytes >= (size_t)32 * HG * 260, "the shared fragment is built in the rings");
  static_assert(kStageBytes >= (size_t)HG * 8192, "the shared query fragment is staged in the rings");
  // Without Stage 1 in this launch the fragment is staged in the score area when that is large
  // enough (it is free until the first score lands), which leaves the rings free: each wave then
  // issues its first key tile BEHIND the query request and waits for both at once.
  const uint16_t* q_t = (const uint16_t*)a.q + (long)t * a.H * kD;
  const float* w_t = a.w + (long)t * a.H;
  const bool q_in_sc = E1 == 0 && (long)a.m * a.B * 4 >= (long)32 * HG * 260;
  unsigned char* q_lds = q_in_sc ? reinterpret_cast<unsigned char*>(sc) : smem;
  QFrag<HG> f;
  SplitShare<HG, NW> q_share;
  if constexpr (kSharedSplit) {
    split_query_request<HG, NW>(q_share, q_t, w_t, wave);
  } else if constexpr (E1 == 0) {
    qfrag_shared_request<HG, NW>(f, q_t, w_t, (long)a.H * kD * 2, lds_address(q_lds), wave);
  } else {
    load_qfrag_shared<HG, NW>(f, q_t, w_t, (long)a.H * kD * 2, lds_address(smem), wave);
  }

  const int tpb = a.B >> 5;
  const int n_blocks = (int)(a.rows_per_seq / a.B);
  const int32_t* blk_ids = a.block_idx + (long)t * a.m;
  if constexpr (E1 > 0) {
    // ---- Stage 1 (Eqs. 5-6) in this workgroup; the kept ids stay in LDS behind the score area
    int32_t* blk_lds = reinterpret_cast<int32_t*>(sc + sc_floats);
    blk_ids = blk_lds;
    qfrag_ready<HG>(f);
    stage1_in_workgroup<HG, NW, NB, E1, kTileBytes>(f, a, pooled, seq, pos, lo, n_blocks, smem, sc, blk_lds, wave);
    if (block_idx_out)
      for (int p = threadIdx.x; p < a.m; p += NT) block_idx_out[(long)t * a.m + p] = blk_lds[p];
  }
  // Only the slots up to the last kept block are walked (a short prefix keeps few blocks).
  // Tile v = sub-tile v % tpb of slot v / tpb; wave w takes tiles w, w + NW, ...
  int n_used = 0;
  for (int i = lane; i < a.m; i += 64) {
    const int blk = blk_ids[i];
    if (blk >= 0 && blk < n_blocks) n_used = i + 1;
  }
  const int n_active = __builtin_amdgcn_readfirstlane((int)wave_max((uint32_t)n_used)) * tpb;
  // first key row of tile v, or -1 if its slot is empty / out of range / not visible
  auto row_of = [&](int v) -> int {
    const int slot = v / tpb;
    const int blk = blk_ids[slot];
    const int row0 = blk * a.B + (v - slot * tpb) * 32;
    return (blk < 0 || blk >= n_blocks || row0 >= n_vis) ? -1 : row0;
  };
  const int nj = n_active > wave ? (n_active - wave + NW - 1) / NW : 0;   // tiles of this wave
  // lane j holds the first key row of this wave's j-th tile (wave + NW * j)
  LaneTable rows;
  rows.lo = row_of(wave + NW * (lane < nj ? lane : 0));
  rows.hi = (nj > 64) ? row_of(wave + NW * (lane + 64 < nj ? lane + 64 : 0)) : -1;
  __amdgpu_buffer_rsrc_t krsrc, srsrc;
  key_buffers<KDT>(a, seq, krsrc, srsrc);
  auto row_at = [&](int j) {
    const int r = rows.at(j);
    return r < 0 ? 0 : r;   // a tile without visible keys still flows through, masked below
  };
  const uint32_t ring_addr = lds_address(smem) + wave * NB * kTileBytes;
  const bool primed = q_in_sc && nj > 0;
  if (primed) tile_dma<KDT>(krsrc, srsrc, ring_addr, row_at(0));
  typename Operands<HG, KDT>::Frag fo;
  if constexpr (kSharedSplit) {
    split_query_complete<HG, NW>(q_share, q_lds, wave, fo);
  } else if constexpr (E1 == 0) {
    qfrag_shared_complete<HG>(f, lds_address(q_lds));
    Operands<HG, KDT>::make(f, fo);
  } else {
    qfrag_ready<HG>(f);
    Operands<HG, KDT>::make(f, fo);
  }
  float s_max = -__builtin_inff(), s_min = __builtin_inff();   // this lane's largest / smallest score so far
  // score_slot of candidate tile * 32 + lane is tile * 32 + a lane pattern that depends on tile % 8
  // only, and this wave's tiles (wave + NW * j) alternate between two values of it
  static_assert((2 * NW) % 8 == 0, "a wave's tiles take two values modulo 8");
  const int l31 = lane & 31;
  const uint32_t pat0 = (uint32_t)(((((l31 >> 2) ^ wave) & 7) << 2) | (l31 & 3)) * 4u;
  const uint32_t pat1 = (uint32_t)(((((l31 >> 2) ^ (wave + NW)) & 7) << 2) | (l31 & 3)) * 4u;
  const uint32_t sc_addr = lds_address(sc);
  const int lane_lo = l31 - lo;
  auto finish = [&](int j, float s) {
    const int r = rows.at(j);
    // a masked slot holds the all-ones pattern, a NaN (ordered_key_plain sends it to "not a
    // candidate", the maximum / minimum below ignore it); a finished score is a sum that starts
    // from +0, so it is never -0.  Visible: lo <= row < n_vis, i.e. unsigned(row - lo) < n_vis - lo
    // (nothing, for a tile without a kept block).
    const int span = r < 0 ? 0 : (n_vis - lo > 0 ? n_vis - lo : 0);
    if ((uint32_t)((r < 0 ? 0 : r) + lane_lo) >= (uint32_t)span) s = __uint_as_float(kNoCandidateBits);
    const uint32_t addr = sc_addr + (uint32_t)(wave + NW * j) * 128u + ((j & 1) ? pat1 : pat0);
    if (lane < 32) asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(s) : "memory");
    s_max = vmax_f32(s_max, s);
    s_min = vmin_f32(s_min, s);
  };
  wave_pipeline<HG, KDT, NB>(fo, krsrc, srsrc, ring_addr, nj, row_at, finish, primed);
  fine_select_range<NT, E>(fs, s_max, s_min, wave);
  __syncthreads();   // scores complete, rings dead: the select scratch may overwrite them
  const int n_cand_slots = n_active * 32;   // score slots actually written

  int32_t* oi = topk_idx + (long)t * k;
  float* os = topk_scores ? topk_scores + (long)t * k : nullptr;
  auto load4 = [&](int q) -> uint4 {
    const uint4 v = *reinterpret_cast<const uint4*>(sc + score_slot(4 * q));
    return make_uint4(ordered_key_plain(v.x), ordered_key_plain(v.y), ordered_key_plain(v.z),
                      ordered_key_plain(v.w));
  };
  auto load1 = [&](int i) -> uint32_t { return ordered_key_plain(__float_as_uint(sc[score_slot(i)])); };
  // A thread's E consecutive candidates lie in one kept block when E divides B: its token base is
  // then fetched once, not per emitted candidate.
  const bool one_slot = a.B % E == 0;
  const int my_slot = (int)(threadIdx.x * E) / a.B;
  const int my_base = (one_slot && my_slot < a.m) ? (blk_ids[my_slot] - my_slot) * a.B : 0;
  // The selected indices are collected in LDS and leave as whole 16-byte rows: written straight
  // from the select, a wave's store would scatter a dozen dwords over as many cache lines.  The
  // score area serves as the collection buffer: by the time the select emits (after its last
  // barrier) every thread holds its candidates in registers and the scores are dead; k <= m * B.
  // (The optional score output keeps the direct path.)
  int32_t* stage = reinterpret_cast<int32_t*>(sc);
  auto emit = [&](int p, int i, uint32_t key) {
    int tok;
    if (one_slot) {
      tok = my_base + i;
    } else {
      const int slot = i / a.B;
      tok = blk_ids[slot] * a.B + (i - slot * a.B);
    }
    stage[p] = tok;
    if (os) os[p] = key_to_score(key);
  };
  // Fast path first (one fine histogram pass, exact by its own check); it declines -- before writing
  // anything -- whenever the row is not its case, and the general select takes over.
  int n_out = -1;
  if (n_cand_slots > k) {
    auto vals = [&](int q) -> float4 { return *reinterpret_cast<const float4*>(sc + score_slot(4 * q)); };
    // Without the score output the thread's E candidates are written without a branch: every
    // element is stored, the ones not selected into a dump word of the thread's own.
    auto emit_f = [&](uint32_t p, const auto& v, float tau, int32_t* dump) {
      const int i0 = (int)threadIdx.x * E;
      if (one_slot && !os) {
        const uint32_t dump_addr = lds_address(dump);
        const uint32_t stage_addr = lds_address(stage);
#pragma unroll
        for (int j = 0; j < E; ++j) {
          const bool take = v[j] >= tau;
          const uint32_t addr = take ? stage_addr + 4u * p : dump_addr;
          asm volatile("ds_write_b32 %0, %1" : : "v"(addr), "v"(my_base + i0 + j) : "memory");
          p += take;
        }
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // (the compiler does not count these writes)
        return;
      }
#pragma unroll
      for (int j = 0; j < E; ++j) {
        if (v[j] >= tau) {
          const int i = i0 + j;
          int tok;
          if (one_slot) {
            tok = my_base + i;
          } else {
            const int slot = i / a.B;
            tok = blk_ids[slot] * a.B + (i - slot * a.B);
          }
          stage[p] = tok;
          if (os) os[p] = v[j];
          ++p;
        }
      }
    };
    if (select_topk_fine<NT, E>(fs, n_cand_slots, k, vals, emit_f)) n_out = k;
  }
  if (n_out < 0) n_out = select_topk<NT, E, false, false>(sm, n_cand_slots, k, load4, load1, emit);
  for (int p = n_out + threadIdx.x; p < k; p += NT) {
    stage[p] = -1;
    if (os) os[p] = neg_inf();
  }
  __syncthreads();
  if ((k & 3) == 0 && (reinterpret_cast<uintptr_t>(oi) & 15) == 0) {
    // whole 16-byte rows, marked non-temporal: the indices are not read again by this kernel and
    // should not push key tiles out of the L2
    typedef int i32x4n __attribute__((ext_vector_type(4)));
    const i32x4n* srcv = reinterpret_cast<const i32x4n*>(stage);
    i32x4n* dstv = reinterpret_cast<i32x4n*>(oi);
    for (int p = threadIdx.x; p < (k >> 2); p += NT) __builtin_nontemporal_store(srcv[p], dstv + p);
  } else {
    for (int p = threadIdx.x; p < k; p += NT) oi[p] = stage[p];
  }
}

}  // namespace hisa
