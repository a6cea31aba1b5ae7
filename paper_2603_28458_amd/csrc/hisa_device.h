// Device-side building blocks of the HISA indexer kernels (gfx950 / CDNA4, wave64).
//
//  * wave_all / wave_scan_add: wave-wide reductions and prefix sums on DPP and lane swaps.
//  * QFrag / mfma_tile / tile_epilogue: the query-heads x key-tile contraction of Eq. 1 / Eq. 5 of
//    the paper on the 32x32x16 bf16 MFMA, with the ReLU, gate and head-sum epilogue in registers.
//  * QFrag8 / split_qfrag / split_query_shared: the same contraction for fp8 keys on the fp8 MFMA
//    (32x32x64, e4m3 x e4m3) against the bf16 query written as the sum of two e4m3 numbers.
//  * tile staging: a 32-key x 128-dim key tile in LDS as 16-byte chunks, XOR-swizzled so that
//    both the lane-contiguous global->LDS transfer and the MFMA-layout load are bank-conflict free;
//    load_qfrag_shared stages the query fragment the same way, once per workgroup.
//  * select_topk: exact per-row top-k (Eqs. 2, 6, 9) on order-preserving keys held in registers:
//    the threshold is bracketed by key ranges cut into 256 bins; ties go to the lower index,
//    output in ascending index order.
//  * score_slot: the swizzled LDS position of a candidate's score, conflict-free both for the
//    scoring waves (32 consecutive candidates) and for the selecting threads (E consecutive each).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace hisa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kWave = 64;
constexpr int kTileKeys = 32;      // keys per MFMA tile (N of the 32x32x16 MFMA)
constexpr int kD = 128;            // indexer head dimension of the MFMA path
constexpr int kTileChunks = 512;   // 16-byte chunks per staged tile: 32 keys x 256 B

__device__ __forceinline__ int lane_id() { return threadIdx.x & 63; }

__device__ __forceinline__ float neg_inf() { return -__builtin_inff(); }

union Pack128 {
  uint4 u;
  bf16x8 v;
};

__device__ __forceinline__ bf16x8 as_bf16x8(uint4 u) {
  Pack128 p;
  p.u = u;
  return p.v;
}

// ------------------------------------------------------------------------------------------
// Wave64 reductions and scans on the DPP / lane-swap paths of the vector ALU (a __shfl goes
// through the LDS crossbar and costs a memory-latency round trip per step).
template <int CTRL, int ROW_MASK = 0xf, int BANK_MASK = 0xf>
__device__ __forceinline__ uint32_t dpp_or0(uint32_t v) {   // lanes without a source read 0
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, ROW_MASK, BANK_MASK, false);
}
template <int CTRL>
__device__ __forceinline__ uint32_t dpp_perm(uint32_t v) {  // permutations: every lane has a source
  return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xf, 0xf, false);
}

// op (associative, commutative) over all 64 lanes, result in every lane.
template <class Op>
__device__ __forceinline__ uint32_t wave_all(uint32_t v, Op op) {
  v = op(v, dpp_perm<0xB1>(v));    // quad_perm [1,0,3,2]
  v = op(v, dpp_perm<0x4E>(v));    // quad_perm [2,3,0,1]
  v = op(v, dpp_perm<0x141>(v));   // row_half_mirror
  v = op(v, dpp_perm<0x140>(v));   // row_mirror
  {
    const auto sw = __builtin_amdgcn_permlane16_swap(v, v, false, false);
    v = op((uint32_t)sw[0], (uint32_t)sw[1]);
  }
  {
    const auto sw = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    v = op((uint32_t)sw[0], (uint32_t)sw[1]);
  }
  return v;
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
  return wave_all(v, [](uint32_t a, uint32_t b) { return a + b; });
}
__device__ __forceinline__ uint32_t wave_max(uint32_t v) {
  return wave_all(v, [](uint32_t a, uint32_t b) { return a > b ? a : b; });
}
__device__ __forceinline__ uint32_t wave_min(uint32_t v) {
  return wave_all(v, [](uint32_t a, uint32_t b) { return a < b ? a : b; });
}

// Inclusive prefix sum over the 64 lanes.
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t v) {
  v += dpp_or0<0x111>(v);        // row_shr:1
  v += dpp_or0<0x112>(v);        // row_shr:2
  v += dpp_or0<0x114>(v);        // row_shr:4
  v += dpp_or0<0x118>(v);        // row_shr:8
  v += dpp_or0<0x142, 0xa>(v);   // row_bcast:15 into rows 1 and 3
  v += dpp_or0<0x143, 0xc>(v);   // row_bcast:31 into rows 2 and 3
  return v;
}

// ------------------------------------------------------------------------------------------
// Query fragment: all H = 32*HG heads of one query in MFMA A-operand layout, plus the gates in
// the accumulator's row layout.  A operand of v_mfma_f32_32x32x16_bf16: lane l supplies row
// (l % 32) and the 8 contraction elements of half (l / 32); step kk covers d = 16*kk .. 16*kk+15.
// Accumulator: lane l holds column (l % 32); register i holds row 8*(i/4) + 4*(l/32) + (i%4).
template <int HG>
struct QFrag {
  bf16x8 a[HG][8];
  float w[HG][16];
};

template <int HG>
__device__ __forceinline__ void load_qfrag(QFrag<HG>& f, const uint16_t* __restrict__ q,
                                           const float* __restrict__ w) {
  const int lane = lane_id();
  const int half = lane >> 5;
  const int r = lane & 31;
#pragma unroll
  for (int g = 0; g < HG; ++g) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const uint4* p = reinterpret_cast<const uint4*>(q + (g * 32 + r) * kD + kk * 16 + half * 8);
      f.a[g][kk] = as_bf16x8(*p);
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) f.w[g][i] = w[g * 32 + 8 * (i >> 2) + 4 * half + (i & 3)];
  }
}

// Makes every load behind the fragment complete HERE.  Without it the first use sits inside the
// tile loop, and the in-order load counter then also waits there, every iteration, for the key
// rows that were just prefetched.
template <int HG>
__device__ __forceinline__ void qfrag_ready(QFrag<HG>& f) {
#pragma unroll
  for (int g = 0; g < HG; ++g) {
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) asm volatile("" : "+v"(f.a[g][kk]));
#pragma unroll
    for (int i = 0; i < 16; ++i) asm volatile("" : "+v"(f.w[g][i]));
  }
}

// max(x, 0) in one instruction (the float max costs a second one that quiets NaNs first).
__device__ __forceinline__ float relu(float x) {
  // as signed integers, every negative float (and -0) is below 0 and every positive float keeps
  // its bits: one integer max, with no NaN-quieting instruction in front of it
  const int b = __builtin_bit_cast(int, x);
  return __builtin_bit_cast(float, b > 0 ? b : 0);
}

// The same contraction and epilogue as two separate steps, so that a kernel can overlap the
// epilogue of one tile with the MFMAs of the next (software pipelining inside one wave).
template <int HG>
using accvec = float __attribute__((ext_vector_type(16 * HG)));
typedef uint32_t u32x32 __attribute__((ext_vector_type(32)));

// B operands of one staged tile: 8 chunks per lane, chunk kk = contraction step kk.  The reads
// are raw instructions: for a plain LDS load the compiler first waits for EVERY pending
// global->LDS transfer of the wave, which would undo the look-ahead of the tile ring.  The caller
// waits for the tile's DMA before calling; the data is complete on return.
typedef uint32_t u32x4e __attribute__((ext_vector_type(4)));

__device__ __forceinline__ u32x32 lds_read_tile_raw(uint32_t tile_addr) {
  const int lane = lane_id();
  const int half = lane >> 5;
  const int r = lane & 31;
  u32x32 kv;
  uint32_t ad[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    ad[kk] = tile_addr + (uint32_t)((r * 16 + ((2 * kk + half) ^ (r & 15))) << 4);
  u32x4e x0, x1, x2, x3, x4, x5, x6, x7;
  // the reads and the wait for their data are one unit, so nothing that uses the data can be
  // scheduled in front of the wait
  asm volatile(
      "ds_read_b128 %0, %8\n\t"
      "ds_read_b128 %1, %9\n\t"
      "ds_read_b128 %2, %10\n\t"
      "ds_read_b128 %3, %11\n\t"
      "ds_read_b128 %4, %12\n\t"
      "ds_read_b128 %5, %13\n\t"
      "ds_read_b128 %6, %14\n\t"
      "ds_read_b128 %7, %15\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3), "=&v"(x4), "=&v"(x5), "=&v"(x6), "=&v"(x7)
      : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7])
      : "memory");
  const u32x4e xs[8] = {x0, x1, x2, x3, x4, x5, x6, x7};
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    kv[4 * kk + 0] = xs[kk][0];
    kv[4 * kk + 1] = xs[kk][1];
    kv[4 * kk + 2] = xs[kk][2];
    kv[4 * kk + 3] = xs[kk][3];
  }
  return kv;
}

// The same eight reads WITHOUT the wait: the caller waits per chunk (tile_chunk_ready) right before
// the MFMAs that consume it, so the first MFMAs start as soon as the first chunk has arrived.  LDS
// operations complete in order, so "at most 7 - kk operations outstanding" implies that chunk kk is
// there, whatever else (score writes, scale reads) was issued behind the eight reads.
struct TileRegs {
  u32x4e x[8];
};

__device__ __forceinline__ void lds_read_tile_issue(uint32_t tile_addr, TileRegs& t) {
  const int lane = lane_id();
  const int half = lane >> 5;
  const int r = lane & 31;
  uint32_t ad[8];
#pragma unroll
  for (int kk = 0; kk < 8; ++kk)
    ad[kk] = tile_addr + (uint32_t)((r * 16 + ((2 * kk + half) ^ (r & 15))) << 4);
  asm volatile(
      "ds_read_b128 %0, %8\n\t"
      "ds_read_b128 %1, %9\n\t"
      "ds_read_b128 %2, %10\n\t"
      "ds_read_b128 %3, %11\n\t"
      "ds_read_b128 %4, %12\n\t"
      "ds_read_b128 %5, %13\n\t"
      "ds_read_b128 %6, %14\n\t"
      "ds_read_b128 %7, %15"
      : "=&v"(t.x[0]), "=&v"(t.x[1]), "=&v"(t.x[2]), "=&v"(t.x[3]), "=&v"(t.x[4]), "=&v"(t.x[5]), "=&v"(t.x[6]),
        "=&v"(t.x[7])
      : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3]), "v"(ad[4]), "v"(ad[5]), "v"(ad[6]), "v"(ad[7])
      : "memory");
}

template <int LEFT>
__device__ __forceinline__ void tile_chunk_ready(u32x4e& x) {
  asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(x) : "n"(LEFT));
}

// after_reads(): called once every read has left the LDS tile (from then on the tile may be
// overwritten), behind the MFMAs of the first two chunks, whose 128 cycles cover the rest of the reads.
template <int HG, bool EVERY_CHUNK = false, class AfterReads>
__device__ __forceinline__ accvec<HG> mfma_tile_progressive(const QFrag<HG>& f, TileRegs& t, AfterReads after_reads) {
  f32x16 acc[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
  auto chunk = [&](int kk) {
    const bf16x8 b = as_bf16x8(make_uint4(t.x[kk][0], t.x[kk][1], t.x[kk][2], t.x[kk][3]));
#pragma unroll
    for (int g = 0; g < HG; ++g)
      acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[g][kk], b, acc[g], 0, 0, 0);
  };
  tile_chunk_ready<7>(t.x[0]);
  chunk(0);
  tile_chunk_ready<6>(t.x[1]);
  chunk(1);
  if constexpr (EVERY_CHUNK) {
    // nothing waits for the tile to be free: every chunk is awaited right before its own MFMAs
    tile_chunk_ready<5>(t.x[2]);
    chunk(2);
    tile_chunk_ready<4>(t.x[3]);
    chunk(3);
    tile_chunk_ready<3>(t.x[4]);
    chunk(4);
    tile_chunk_ready<2>(t.x[5]);
    chunk(5);
    tile_chunk_ready<1>(t.x[6]);
    chunk(6);
    tile_chunk_ready<0>(t.x[7]);
    chunk(7);
    after_reads();
  } else {
    asm volatile("s_waitcnt lgkmcnt(0)"
                 : "+v"(t.x[2]), "+v"(t.x[3]), "+v"(t.x[4]), "+v"(t.x[5]), "+v"(t.x[6]), "+v"(t.x[7])
                 :
                 : "memory");
    after_reads();
#pragma unroll
    for (int kk = 2; kk < 8; ++kk) chunk(kk);
  }
  accvec<HG> out;
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) out[g * 16 + i] = acc[g][i];
  return out;
}

template <int HG>
__device__ __forceinline__ accvec<HG> mfma_tile(const QFrag<HG>& f, const u32x32& kv) {
  f32x16 acc[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
#pragma unroll
  for (int kk = 0; kk < 8; ++kk) {
    const bf16x8 b =
        as_bf16x8(make_uint4(kv[4 * kk + 0], kv[4 * kk + 1], kv[4 * kk + 2], kv[4 * kk + 3]));
#pragma unroll
    for (int g = 0; g < HG; ++g)
      acc[g] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[g][kk], b, acc[g], 0, 0, 0);
  }
  accvec<HG> out;
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) out[g * 16 + i] = acc[g][i];
  return out;
}

// Sum of both 32-lane halves in every lane (one swap of the halves, one add).
__device__ __forceinline__ float add_halves(float s) {
  const uint32_t b = __float_as_uint(s);
  const auto sw = __builtin_amdgcn_permlane32_swap(b, b, false, false);
  return __uint_as_float(sw[0]) + __uint_as_float(sw[1]);
}

template <int HG, class Frag>
__device__ __forceinline__ float tile_epilogue(const Frag& f, const accvec<HG>& acc) {
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
#pragma unroll
  for (int g = 0; g < HG; ++g) {
#pragma unroll
    for (int i = 0; i < 16; i += 4) {
      s0 = __builtin_fmaf(relu(acc[g * 16 + i + 0]), f.w[g][i + 0], s0);
      s1 = __builtin_fmaf(relu(acc[g * 16 + i + 1]), f.w[g][i + 1], s1);
      s2 = __builtin_fmaf(relu(acc[g * 16 + i + 2]), f.w[g][i + 2], s2);
      s3 = __builtin_fmaf(relu(acc[g * 16 + i + 3]), f.w[g][i + 3], s3);
    }
  }
  return add_halves((s0 + s1) + (s2 + s3));
}

// ------------------------------------------------------------------------------------------
// fp8 keys: the contraction runs on the fp8 MFMA (v_mfma_f32_32x32x64_f8f6f4, e4m3 x e4m3, twice the
// bf16 rate) with the key codes as they are stored, and the bf16 query written as a sum of two e4m3
// numbers.  Per head row the query is first multiplied by a power of two that puts its largest
// magnitude into [128, 256); hi = e4m3(q), lo = e4m3(q - hi): the 8 significant bits of a bf16
// value split 4 + 4, so hi + lo == q exactly for every element within 2^-9 of the row's largest,
// and within 2^-17 of that largest below (the e4m3 subnormal grid).  Two MFMAs (hi, lo) per 64
// contraction elements accumulate into the same registers; the power of two goes into the gate.
// Lane l keeps the contraction elements it holds in the bf16 fragment (d = 16*kk + 8*(l/32) + e):
// MFMA step ks takes kk = 4*ks .. 4*ks+3, and the key operand follows the same order, which an
// MFMA permits because A and B index the contraction dimension by the same (lane / 32, byte).
typedef int i32x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));

template <int HG>
struct QFrag8 {
  i32x8 hi[HG][2], lo[HG][2];
  float w[HG][16];
};

template <int HG>
__device__ __forceinline__ void split_qfrag(const QFrag<HG>& f, QFrag8<HG>& o) {
  const int half = lane_id() >> 5;
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    // largest bf16 magnitude (sign cleared) of head row g*32 + lane%32: 64 elements here, 64 in lane ^ 32
    uint32_t mag = 0;
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack128 p;
      p.v = f.a[g][kk];
      const uint32_t d[4] = {p.u.x, p.u.y, p.u.z, p.u.w};
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const uint32_t lo16 = d[c] & 0x7fffu, hi16 = (d[c] >> 16) & 0x7fffu;
        mag = mag > lo16 ? mag : lo16;
        mag = mag > hi16 ? mag : hi16;
      }
    }
    {
      const auto sw = __builtin_amdgcn_permlane32_swap(mag, mag, false, false);   // both halves of the row
      mag = sw[0] > sw[1] ? sw[0] : sw[1];
    }
    int e = (int)(mag >> 7);                  // biased exponent of the largest magnitude
    e = e < 8 ? 8 : (e > 254 ? 254 : e);      // (rows below 2^-119 lose their low bits: they score ~0)
    const float up = __uint_as_float((uint32_t)(261 - e) << 23);     // 2^(134 - e)
    const float down = __uint_as_float((uint32_t)(e - 7) << 23);     // 2^(e - 134)
    uint32_t whi[8][2], wlo[8][2];   // [kk]: the 8 codes of d = 16*kk + 8*half .. +7
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      Pack128 p;
      p.v = f.a[g][kk];
      const uint32_t d[4] = {p.u.x, p.u.y, p.u.z, p.u.w};
      whi[kk][0] = whi[kk][1] = wlo[kk][0] = wlo[kk][1] = 0u;
#pragma unroll
      for (int c = 0; c < 4; ++c) {
        const float x0 = __uint_as_float(d[c] << 16) * up;
        const float x1 = __uint_as_float(d[c] & 0xffff0000u) * up;
        const int h = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
        const auto back = __builtin_amdgcn_cvt_pk_f32_fp8(h, false);
        const int l = __builtin_amdgcn_cvt_pk_fp8_f32(x0 - back[0], x1 - back[1], 0, false);
        whi[kk][c >> 1] |= (uint32_t)(h & 0xffff) << (16 * (c & 1));
        wlo[kk][c >> 1] |= (uint32_t)(l & 0xffff) << (16 * (c & 1));
      }
    }
    // From halves of every 16-element chunk (the bf16 fragment's order) to whole chunks: for the
    // chunk pair (2j, 2j+1) lanes 0-31 hand the first half of the odd chunk to lanes 32-63 and
    // receive the second half of the even chunk: afterwards a lane of half h holds chunk 2j + h.
#pragma unroll
    for (int j = 0; j < 4; ++j) {
#pragma unroll
      for (int x = 0; x < 2; ++x) {
        const auto sh = __builtin_amdgcn_permlane32_swap(whi[2 * j][x], whi[2 * j + 1][x], false, false);
        const auto sl = __builtin_amdgcn_permlane32_swap(wlo[2 * j][x], wlo[2 * j + 1][x], false, false);
        whi[2 * j][x] = sh[0];
        whi[2 * j + 1][x] = sh[1];
        wlo[2 * j][x] = sl[0];
        wlo[2 * j + 1][x] = sl[1];
      }
      // chunk 2j + half as 16 bytes: (first half, second half) = (entry 2j, entry 2j+1)
      o.hi[g][j >> 1][4 * (j & 1) + 0] = (int)whi[2 * j][0];
      o.hi[g][j >> 1][4 * (j & 1) + 1] = (int)whi[2 * j][1];
      o.hi[g][j >> 1][4 * (j & 1) + 2] = (int)whi[2 * j + 1][0];
      o.hi[g][j >> 1][4 * (j & 1) + 3] = (int)whi[2 * j + 1][1];
      o.lo[g][j >> 1][4 * (j & 1) + 0] = (int)wlo[2 * j][0];
      o.lo[g][j >> 1][4 * (j & 1) + 1] = (int)wlo[2 * j][1];
      o.lo[g][j >> 1][4 * (j & 1) + 2] = (int)wlo[2 * j + 1][0];
      o.lo[g][j >> 1][4 * (j & 1) + 3] = (int)wlo[2 * j + 1][1];
    }
    // the gate of accumulator register i belongs to head row 8*(i/4) + 4*half + i%4, whose
    // power of two sits in the lane of that number
#pragma unroll
    for (int i = 0; i < 16; ++i)
      o.w[g][i] = f.w[g][i] * __shfl(down, 8 * (i >> 2) + 4 * half + (i & 3));
  }
}

// The same two-term fragment built ONCE per workgroup of NW waves instead of once per wave: wave w
// converts the heads w*H/NW .. (w+1)*H/NW - 1 (a head is spread over 64*NW/H consecutive lanes, so
// its largest magnitude is a DPP reduction inside a row), writes hi / lo in operand order and the
// scaled gates to LDS, and after one barrier every wave reads the whole fragment (16 reads of 16
// bytes, lane-contiguous).  lds: 32*HG*260 bytes that nothing else touches until the function
// returns (it ends with a second barrier).  q, w: this query's [H, d] bf16 and [H] gates.
template <int HG, int NW>
struct SplitShare {
  static constexpr int H = 32 * HG;
  static constexpr int HP = H / NW;     // heads per wave
  static constexpr int LPH = 64 / HP;   // lanes per head
  static constexpr int EPL = kD / LPH;  // elements per lane
  static_assert(H % NW == 0 && (LPH == 4 || LPH == 8 || LPH == 16), "a head must map to 4, 8 or 16 lanes");
  uint4 v[EPL / 8];   // this lane's share of its head, as loaded
  float gate;
};

// First half: the loads only, so that a caller can put other memory traffic behind them.
template <int HG, int NW>
__device__ __forceinline__ void split_query_request(SplitShare<HG, NW>& r, const uint16_t* __restrict__ q,
                                                    const float* __restrict__ w, int wave) {
  using S = SplitShare<HG, NW>;
  const int lane = lane_id();
  const int head = wave * S::HP + lane / S::LPH, seg = lane % S::LPH;
  const uint4* src = reinterpret_cast<const uint4*>(q + head * kD + seg * S::EPL);
#pragma unroll
  for (int c = 0; c < S::EPL / 8; ++c) r.v[c] = src[c];
  r.gate = w[head];
}

template <int HG, int NW>
__device__ __forceinline__ void split_query_complete(const SplitShare<HG, NW>& share, unsigned char* lds, int wave,
                                                     QFrag8<HG>& o) {
  using S = SplitShare<HG, NW>;
  constexpr int HP = S::HP, LPH = S::LPH, EPL = S::EPL;
  const int lane = lane_id();
  const int head = wave * HP + lane / LPH, seg = lane % LPH;
  const uint4* v = share.v;
  const float gate = share.gate;
  uint32_t mag = 0;
#pragma unroll
  for (int c = 0; c < EPL / 8; ++c) {
    const uint32_t d[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t lo16 = d[x] & 0x7fffu, hi16 = (d[x] >> 16) & 0x7fffu;
      mag = mag > lo16 ? mag : lo16;
      mag = mag > hi16 ? mag : hi16;
    }
  }
  auto mx = [](uint32_t a, uint32_t b) { return a > b ? a : b; };
  mag = mx(mag, dpp_perm<0xB1>(mag));                  // 2 lanes
  mag = mx(mag, dpp_perm<0x4E>(mag));                  // 4
  if (LPH >= 8) mag = mx(mag, dpp_perm<0x141>(mag));   // 8
  if (LPH >= 16) mag = mx(mag, dpp_perm<0x140>(mag));  // 16
  int e = (int)(mag >> 7);
  e = e < 8 ? 8 : (e > 254 ? 254 : e);
  const float up = __uint_as_float((uint32_t)(261 - e) << 23);
  const float down = __uint_as_float((uint32_t)(e - 7) << 23);
  const int g = head >> 5, r = head & 31;
  uint2* frag = reinterpret_cast<uint2*>(lds);
  float* gates = reinterpret_cast<float*>(lds + 32 * HG * 256);
#pragma unroll
  for (int c = 0; c < EPL / 8; ++c) {
    const uint32_t d[4] = {v[c].x, v[c].y, v[c].z, v[c].w};
    int whi[2] = {0, 0}, wlo[2] = {0, 0};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const float x0 = __uint_as_float(d[x] << 16) * up;
      const float x1 = __uint_as_float(d[x] & 0xffff0000u) * up;
      const int h = __builtin_amdgcn_cvt_pk_fp8_f32(x0, x1, 0, false);
      const auto back = __builtin_amdgcn_cvt_pk_f32_fp8(h, false);
      const int l = __builtin_amdgcn_cvt_pk_fp8_f32(x0 - back[0], x1 - back[1], 0, false);
      whi[x >> 1] |= (h & 0xffff) << (16 * (x & 1));
      wlo[x >> 1] |= (l & 0xffff) << (16 * (x & 1));
    }
    // elements 8*c8 .. 8*c8+7 of the head = half c8 % 2 of the 16-element chunk ch = c8 / 2, which
    // belongs to lane half ch % 2 as its chunk j = ch / 2 (see lds_read_tile_fp8_raw)
    const int c8 = seg * (EPL / 8) + c;
    const int ch = c8 >> 1, half = ch & 1, j = ch >> 1;
    // operand order: [g][ks = j / 2][piece][lane = half*32 + r] x 32 bytes, 8 bytes per (j % 2, c8 % 2)
    const int slot = (((g * 2 + (j >> 1)) * 2) * 64 + half * 32 + r) * 4 + (j & 1) * 2 + (c8 & 1);
    frag[slot] = make_uint2((uint32_t)whi[0], (uint32_t)whi[1]);
    frag[slot + 64 * 4] = make_uint2((uint32_t)wlo[0], (uint32_t)wlo[1]);
  }
  if (seg == 0) gates[head] = gate * down;
  __syncthreads();
  const int my_half = lane >> 5;
#pragma unroll
  for (int gg = 0; gg < HG; ++gg) {
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const uint4* ph = reinterpret_cast<const uint4*>(lds + ((((gg * 2 + ks) * 2 + 0) * 64 + lane) * 32));
      const uint4* pl = reinterpret_cast<const uint4*>(lds + ((((gg * 2 + ks) * 2 + 1) * 64 + lane) * 32));
      const uint4 h0 = ph[0], h1 = ph[1], l0 = pl[0], l1 = pl[1];
      o.hi[gg][ks] = i32x8{(int)h0.x, (int)h0.y, (int)h0.z, (int)h0.w, (int)h1.x, (int)h1.y, (int)h1.z, (int)h1.w};
      o.lo[gg][ks] = i32x8{(int)l0.x, (int)l0.y, (int)l0.z, (int)l0.w, (int)l1.x, (int)l1.y, (int)l1.z, (int)l1.w};
    }
#pragma unroll
    for (int a4 = 0; a4 < 4; ++a4) {
      const float4 gv = *reinterpret_cast<const float4*>(gates + gg * 32 + 8 * a4 + 4 * my_half);
      o.w[gg][4 * a4 + 0] = gv.x;
      o.w[gg][4 * a4 + 1] = gv.y;
      o.w[gg][4 * a4 + 2] = gv.z;
      o.w[gg][4 * a4 + 3] = gv.w;
    }
  }
  __syncthreads();
}

template <int HG, int NW>
__device__ __forceinline__ void split_query_shared(const uint16_t* __restrict__ q, const float* __restrict__ w,
                                                   unsigned char* lds, int wave, QFrag8<HG>& o) {
  SplitShare<HG, NW> r;
  split_query_request<HG, NW>(r, q, w, wave);
  split_query_complete<HG, NW>(r, lds, wave, o);
}

template <int HG>
__device__ __forceinline__ accvec<HG> mfma_tile(const QFrag8<HG>& f, const u32x16& kv) {
  f32x16 acc[HG];
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[g][i] = 0.f;
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    i32x8 b;
#pragma unroll
    for (int i = 0; i < 8; ++i) b[i] = (int)kv[8 * ks + i];
#pragma unroll
    for (int g = 0; g < HG; ++g)
      acc[g] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f.hi[g][ks], b, acc[g], 0, 0, 0, 0, 0, 0);
#pragma unroll
    for (int g = 0; g < HG; ++g)
      acc[g] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(f.lo[g][ks], b, acc[g], 0, 0, 0, 0, 0, 0);
  }
  accvec<HG> out;
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) out[g * 16 + i] = acc[g][i];
  return out;
}

// ------------------------------------------------------------------------------------------
// Tile staging.  Chunk (row r, 16-byte column c) of a tile lives at LDS chunk r*16 + (c ^ (r&15)).
// A staging step moves chunk position p = i*64 + lane, so consecutive lanes write consecutive
// 16-byte LDS words and read one 256-byte key row per 16 lanes.

// A tile's global address = a wave-uniform tile base plus eight per-lane byte offsets that do not
// depend on the tile (computed once per kernel).
typedef uint32_t u32x8 __attribute__((ext_vector_type(8)));

__device__ __forceinline__ u32x8 tile_lane_offsets_bf16() {
  const int lane = lane_id();
  u32x8 o;
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const int r = 4 * i + (lane >> 4), c = lane & 15;
    o[i] = (uint32_t)(r * 256 + ((c ^ (r & 15)) << 4));
  }
  return o;
}

// Key rows are read through a raw buffer descriptor: base = the sequence's first key, a
// wave-uniform byte offset picks the tile, the per-lane offsets stay in registers for the whole
// kernel, and reads past the end of the sequence's key array return zeros instead of faulting.
typedef uint32_t u32x4v __attribute__((__vector_size__(16)));

__device__ __forceinline__ __amdgpu_buffer_rsrc_t key_buffer(const void* base, long bytes) {
  return __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, (int)bytes, 0x00020000);
}

// Exact widening of 4 e4m3fn codes (one dword) to 4 bf16 (every e4m3 value is a bf16 value).
__device__ __forceinline__ uint2 fp8x4_to_bf16x4(uint32_t word) {
  union {
    bf16x2 h;
    uint32_t u;
  } lo, hi;
  lo.h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)word, 1.0f, false);
  hi.h = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8((int)word, 1.0f, true);
  return make_uint2(lo.u, hi.u);
}

// A tile moves global -> LDS directly (no registers): lane l of step i deposits its 16
// bytes at LDS byte address lds_addr + (i*64 + l)*16, which is the staged layout above.
typedef __attribute__((address_space(3))) void lds_void;

__device__ __forceinline__ uint32_t lds_address(const void* p) {
  return (uint32_t)reinterpret_cast<uintptr_t>(p);   // low 32 bits of a generic LDS pointer
}

__device__ __forceinline__ void tile_dma_bf16(__amdgpu_buffer_rsrc_t rsrc, uint32_t lds_addr,
                                              int tile_byte_off, const u32x8& o) {
#pragma unroll
  for (int i = 0; i < 8; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(uintptr_t)(lds_addr + i * 1024), 16,
                                         (int)o[i], tile_byte_off, 0, 0);
}

// fp8 keys by DMA: the 4 KB of a tile as 256 chunks of 16 codes; LDS chunk p = i*64 + lane holds
// global chunk (row r = p / 8, column (p % 8) xor ((r / 2) % 8)): 16 consecutive rows of one
// column then cover all 64 banks, which is what the 16-byte MFMA-layout reads below need (rows are
// 128 bytes, so two neighbours share the swizzle and differ in the upper half of the banks).
// A fifth transfer brings the 32 per-token scales (as 64 floats).
__device__ __forceinline__ void tile_dma_fp8(__amdgpu_buffer_rsrc_t rsrc, __amdgpu_buffer_rsrc_t srsrc,
                                             uint32_t lds_addr, int row0) {
  const int lane = lane_id();
  // row r = 8*i + lane/8, so (r/2) % 8 = (4*i + lane/16) % 8: transfers alternate between two offsets
  const int voff0 = (lane >> 3) * 128 + (((lane & 7) ^ (lane >> 4)) << 4);
  const int voff1 = voff0 ^ 64;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rsrc, (lds_void*)(uintptr_t)(lds_addr + i * 1024), 16,
                                             (i & 1) ? voff1 : voff0, row0 * 128 + i * 1024, 0, 0);
  __builtin_amdgcn_raw_ptr_buffer_load_lds(srsrc, (lds_void*)(uintptr_t)(lds_addr + 4096), 4, lane * 4,
                                           row0 * 4, 0, 0);
}

// B operands of an fp8 tile staged by tile_dma_fp8: four 16-byte reads per lane (raw
// instructions, see lds_read_tile_raw); read j brings the codes of d = 16*(2*j + lane/32) .. +15 of
// key row lane % 32 -- lanes 0-31 take the even 16-element chunks, lanes 32-63 the odd ones, the
// order split_qfrag gives the query operand.  Conflict-free.  Complete on return.
__device__ __forceinline__ u32x16 lds_read_tile_fp8_raw(uint32_t tile_addr) {
  const int lane = lane_id();
  const int half = lane >> 5;
  const int r = lane & 31;
  uint32_t ad[4];
#pragma unroll
  for (int j = 0; j < 4; ++j)
    ad[j] = tile_addr + (uint32_t)(r * 128 + (((2 * j + half) ^ ((r >> 1) & 7)) << 4));
  u32x4e x0, x1, x2, x3;
  asm volatile(
      "ds_read_b128 %0, %4\n\t"
      "ds_read_b128 %1, %5\n\t"
      "ds_read_b128 %2, %6\n\t"
      "ds_read_b128 %3, %7\n\t"
      "s_waitcnt lgkmcnt(0)"
      : "=&v"(x0), "=&v"(x1), "=&v"(x2), "=&v"(x3)
      : "v"(ad[0]), "v"(ad[1]), "v"(ad[2]), "v"(ad[3])
      : "memory");
  const u32x4e xs[4] = {x0, x1, x2, x3};
  u32x16 kv;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    kv[4 * j + 0] = xs[j][0];
    kv[4 * j + 1] = xs[j][1];
    kv[4 * j + 2] = xs[j][2];
    kv[4 * j + 3] = xs[j][3];
  }
  return kv;
}

// One float from LDS by raw instruction (same reason), complete on return.
__device__ __forceinline__ float lds_read_f32_raw(uint32_t addr) {
  float v;
  asm volatile("ds_read_b32 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=&v"(v) : "v"(addr) : "memory");
  return v;
}

// Wait until at most N global loads of this wave are outstanding (loads complete in order).
template <int N>
__device__ __forceinline__ void wait_vmem_le() {
  __builtin_amdgcn_s_waitcnt(0x0f70 | (N & 15) | ((N >> 4) << 14));
}

// The bf16 query fragment through LDS, loaded ONCE per workgroup of NW waves: the 32 heads of a
// group are 32 rows of 256 bytes, the geometry of a key tile, and the MFMA A operand of lane
// (row, half) at step kk is chunk 2*kk + half of its row, which is what lds_read_tile_raw returns.
// lds: HG * 8192 bytes nothing else touches until the function returns (it ends with a barrier).
template <int HG, int NW>
__device__ __forceinline__ void qfrag_shared_request(QFrag<HG>& f, const uint16_t* __restrict__ q,
                                                     const float* __restrict__ w, long q_bytes_left,
                                                     uint32_t lds_addr, int wave) {
  const int lane = lane_id();
  const int half = lane >> 5;
  const __amdgpu_buffer_rsrc_t qrsrc = key_buffer(q, q_bytes_left);
  const u32x8 lane_offs = tile_lane_offsets_bf16();
  // the 8 * HG transfers of 1 KB are dealt round robin to the waves
#pragma unroll
  for (int i = 0; i < 8 * HG; ++i)
    if (i % NW == wave)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(qrsrc, (lds_void*)(uintptr_t)(lds_addr + i * 1024), 16,
                                               (int)lane_offs[i & 7], (i >> 3) * 8192, 0, 2);   // aux 2 = non-temporal: a query is read once
#pragma unroll
  for (int g = 0; g < HG; ++g)
#pragma unroll
    for (int i = 0; i < 16; ++i) f.w[g][i] = w[g * 32 + 8 * (i >> 2) + 4 * half + (i & 3)];
}

// Second half: waits for everything this wave has in flight (the request above and whatever the
// caller issued since, e.g. its first key tile), then reads the fragment.  Ends with a barrier.
template <int HG>
__device__ __forceinline__ void qfrag_shared_complete(QFrag<HG>& f, uint32_t lds_addr) {
  wait_vmem_le<0>();
  __syncthreads();
#pragma unroll
  for (int g = 0; g < HG; ++g) {
    const u32x32 t = lds_read_tile_raw(lds_addr + g * 8192);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk)
      f.a[g][kk] = as_bf16x8(make_uint4(t[4 * kk + 0], t[4 * kk + 1], t[4 * kk + 2], t[4 * kk + 3]));
  }
  __syncthreads();
}

template <int HG, int NW>
__device__ __forceinline__ void load_qfrag_shared(QFrag<HG>& f, const uint16_t* __restrict__ q,
                                                  const float* __restrict__ w, long q_bytes_left,
                                                  uint32_t lds_addr, int wave) {
  qfrag_shared_request<HG, NW>(f, q, w, q_bytes_left, lds_addr, wave);
  qfrag_shared_complete<HG>(f, lds_addr);
}


// ------------------------------------------------------------------------------------------
// Order-preserving key of a score: larger score <=> larger key.  -0 counts as +0.  Key 0 is
// reserved for "not a candidate" (-inf or out of range); real candidates map to >= 1.
__device__ __forceinline__ uint32_t ordered_key(float s) {
  if (s == neg_inf()) return 0u;
  const uint32_t b = __float_as_uint(s + 0.0f);
  const uint32_t k = (b & 0x80000000u) ? ~b : (b | 0x80000000u);
  return k ? k : 1u;
}

// The same order-preserving map without the special cases, for score arrays whose writer
// guarantees that -0 does not occur and marks "not a candidate" with the all-ones bit pattern
// (which this map sends to 0): three instructions instead of seven.
constexpr uint32_t kNoCandidateBits = 0xffffffffu;
__device__ __forceinline__ uint32_t ordered_key_plain(uint32_t bits) {
  const uint32_t mask = (uint32_t)((int32_t)bits >> 31) | 0x80000000u;
  return bits ^ mask;
}

__device__ __forceinline__ float key_to_score(uint32_t k) {
  const uint32_t b = (k & 0x80000000u) ? (k & 0x7fffffffu) : ~k;
  return __uint_as_float(b);
}

__device__ __forceinline__ uint32_t lanes_below(uint64_t mask) {
  return __builtin_amdgcn_mbcnt_hi((uint32_t)(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo((uint32_t)mask, 0u));
}

// LDS word of candidate c in a score array: inside every row of 32 words, the eight 4-word
// groups are permuted by the row number, so that 8 lanes reading 16 bytes from 8 consecutive
// rows (one thread = one row in the select) hit 8 different bank groups.
__device__ __forceinline__ int score_slot(int c) {
  return (c & ~31) | ((((c >> 2) ^ (c >> 5)) & 7) << 2) | (c & 3);
}

template <int THREADS, int E>
struct SelectSmem {
  static constexpr int NW = THREADS / 64;
  static constexpr int CAP = 2048;   // entries of the threshold-bin list (fast path)
  uint32_t hist[256];
  uint32_t red[5 * NW];
  uint32_t bcast[4];
  uint32_t n_list;
  uint16_t list[CAP];
};

// Finds, in a 256-bin histogram of counts (bin 255 = largest keys), the bin that holds the
// krem-th largest element: counts above it < krem <= counts above it + its own.  Wave 0 only;
// publishes bcast[0] = bin, bcast[1] = krem - (count above), bcast[2] = count in that bin.
// If krem exceeds the histogram's total (the element lies below the binned range):
// bcast[0] = 0xffffffff, bcast[1] = krem - total, bcast[2] = total.
__device__ __forceinline__ void find_bin(const uint32_t* hist, uint32_t* bcast, uint32_t krem, int lane) {
  const uint32_t c0 = hist[4 * lane + 0], c1 = hist[4 * lane + 1];
  const uint32_t c2 = hist[4 * lane + 2], c3 = hist[4 * lane + 3];
  const uint32_t s = c0 + c1 + c2 + c3;
  const uint32_t total = wave_sum(s);
  const uint32_t S = total - wave_scan_add(s) + s;   // inclusive suffix sum over lanes
  const uint32_t a3 = S - s, a2 = a3 + c3, a1 = a2 + c2, a0 = a1 + c1;
  int dsel = -1;
  uint32_t above = 0, mine = 0;
  if (a3 < krem && krem <= a3 + c3) { dsel = 3; above = a3; mine = c3; }
  if (a2 < krem && krem <= a2 + c2) { dsel = 2; above = a2; mine = c2; }
  if (a1 < krem && krem <= a1 + c1) { dsel = 1; above = a1; mine = c1; }
  if (a0 < krem && krem <= a0 + c0) { dsel = 0; above = a0; mine = c0; }
  if (dsel >= 0) {
    bcast[0] = (uint32_t)(4 * lane + dsel);
    bcast[1] = krem - above;
    bcast[2] = mine;
  }
  if (lane == 0 && krem > total) {
    bcast[0] = 0xffffffffu;
    bcast[1] = krem - total;
    bcast[2] = total;
  }
}

// Exact top-k of one row by one workgroup of THREADS threads, n <= THREADS * E elements.
//   load4(q) -> keys of elements 4q .. 4q+3 (0: not a candidate); load1(i) -> key of element i.
//   Thread t holds the E consecutive elements t*E .. t*E+E-1 in registers.
//   emit(pos, i, key): element i is the pos-th selected, in ascending i.
// Returns the number selected: min(k, #candidates).  Order: key descending, then i ascending.
// Method: the threshold (the k-th largest key) is bracketed by key RANGES, each pass cutting the
// current range [lo, hi] into up to 256 equal bins, counting the candidates per bin (LDS atomics)
// and keeping the bin that holds the k-th.  Scores of one row crowd into one or two binades, so
// bins over the row's own range spread the counts where radix digits of the float bits would pile
// them onto a few addresses.  The first range is [largest of the per-thread minima, row maximum]:
// the low end sits near the row's 15th percentile whatever a few tiny scores do, and if the k-th
// lies below it the next pass bins [row minimum, that low end).  Keys equal to 0xffffffff (rows
// forced to the top by a caller) are counted apart and do not stretch the range.  The candidates
// of the bin kept by the first pass are listed in LDS and later passes run over that list only
// (if it overflows the list -- many equal keys -- they keep running over the registers); a pass
// whose bin is taken whole ends the search.  Positions come from one workgroup scan of
// per-thread counts: output is ascending, ties go to the lower index.
// Every thread of the workgroup must call it (it contains workgroup barriers).
// SAFE: load4(q) may be called for any q < THREADS * E / 4 (it returns anything beyond n); the
// loads of a thread are then issued back to back instead of one per guarded branch.
// FORCED: keys equal to 0xffffffff may occur (callers that force rows to the top); without it the
// per-element bookkeeping for them is left out.
template <int THREADS, int E, bool SAFE = false, bool FORCED = true, class Load4, class Load1, class Emit>
__device__ __forceinline__ int select_topk(SelectSmem<THREADS, E>& sm, int n, int k, Load4 load4,
                                           Load1 load1, Emit emit) {
  static_assert(E % 4 == 0, "elements per thread come in groups of four");
  constexpr int NW = THREADS / 64;
  constexpr int CAP = SelectSmem<THREADS, E>::CAP;
  constexpr uint32_t TOP = 0xffffffffu;
  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int wave = tid >> 6;
  const int i0 = tid * E;

  typedef uint32_t keyvec __attribute__((ext_vector_type(E)));
  keyvec key;   // one vector value, not an array (arrays that live across barriers go to scratch)
  uint32_t cnt = 0, n_top = 0, t_min = TOP, t_max = 0u;
  uint4 q4s[E / 4];
#pragma unroll
  for (int g = 0; g < E / 4; ++g) {
    if (SAFE) {
      q4s[g] = load4((i0 >> 2) + g);
    } else {
      q4s[g] = make_uint4(0u, 0u, 0u, 0u);
      if (i0 + 4 * g < n) q4s[g] = load4((i0 >> 2) + g);
    }
  }
  const bool whole = i0 + E <= n;   // every element of this thread lies inside the row (all but one thread)
#pragma unroll
  for (int g = 0; g < E / 4; ++g) {
    const uint4 q4 = q4s[g];
    const uint32_t kk[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      const uint32_t kj = (whole || i0 + 4 * g + x < n) ? kk[x] : 0u;
      key[4 * g + x] = kj;
      cnt += kj != 0u;
      // minimum over the keys in 1 .. TOP-1: 0 - 1 wraps to TOP and TOP - 1 stays large, so both
      // ends of the key space drop out of the minimum
      const uint32_t for_min = kj - 1u;
      t_min = for_min < t_min ? for_min : t_min;
      if (FORCED) {
        n_top += kj == TOP;
        const uint32_t for_max = kj + 1u;   // TOP + 1 wraps to 0 and drops out of the maximum
        t_max = for_max > t_max ? for_max : t_max;
      } else {
        t_max = kj > t_max ? kj : t_max;
      }
    }
  }
  // t_min = (smallest key in 1..TOP-1) - 1, or >= TOP - 1 if there is none; t_max = (largest such key) + 1, or 0/1
  uint32_t lo_est = t_min >= TOP - 1u ? 0u : t_min + 1u;   // this thread's minimum, 0 if it has none
  uint32_t k_min = t_min >= TOP - 1u ? TOP : t_min + 1u;
  uint32_t k_max = FORCED ? (t_max <= 1u ? 0u : t_max - 1u) : t_max;
  cnt = wave_sum(cnt);
  if (FORCED) n_top = wave_sum(n_top);
  lo_est = wave_max(lo_est);
  k_min = wave_min(k_min);
  k_max = wave_max(k_max);
  if (lane == 0) {
    sm.red[wave] = cnt;
    sm.red[NW + wave] = n_top;
    sm.red[2 * NW + wave] = lo_est;
    sm.red[3 * NW + wave] = k_min;
    sm.red[4 * NW + wave] = k_max;
  }
  if (tid == 0) sm.n_list = 0u;
  __syncthreads();
  cnt = 0;
  n_top = 0;
  lo_est = 0u;
  k_min = TOP;
  k_max = 0u;
#pragma unroll
  for (int v = 0; v < NW; ++v) {
    cnt += sm.red[v];
    n_top += sm.red[NW + v];
    const uint32_t a = sm.red[2 * NW + v], b = sm.red[3 * NW + v], c = sm.red[4 * NW + v];
    lo_est = a > lo_est ? a : lo_est;
    k_min = b < k_min ? b : k_min;
    k_max = c > k_max ? c : k_max;
  }
  const int n_valid = (int)cnt;

  uint32_t tau = 0u;   // threshold key: everything above is selected
  uint32_t r = 0u;     // how many elements equal to tau are selected (lowest indices first)
  if (n_valid > k && (uint32_t)k <= n_top) {
    tau = TOP;
    r = (uint32_t)k;
  } else if (n_valid > k) {
    uint32_t krem = (uint32_t)k - n_top;   // > 0; at least krem + 1 keys lie in [k_min, k_max]
    uint32_t lo = lo_est, hi = k_max;      // current range; k_min <= lo <= hi <= k_max < TOP
    bool on_list = false;
    uint32_t n_listed = 0;
    while (true) {
      const uint32_t width = hi - lo;
      const int s = width ? (32 - __builtin_clz(width) > 8 ? 32 - __builtin_clz(width) - 8 : 0) : 0;
      __syncthreads();   // list complete / previous result read by everyone
      for (int b = tid; b < 256; b += THREADS) sm.hist[b] = 0u;
      __syncthreads();
      if (on_list) {
        for (uint32_t p = tid; p < n_listed; p += THREADS) {
          const uint32_t dk = load1((int)sm.list[p]) - lo;   // keys below lo (and 0) wrap far above width
          if (dk <= width) atomicAdd(&sm.hist[dk >> s], 1u);
        }
      } else {
#pragma unroll
        for (int j = 0; j < E; ++j) {
          const uint32_t dk = key[j] - lo;
          if (dk <= width) atomicAdd(&sm.hist[dk >> s], 1u);
        }
      }
      __syncthreads();
      if (wave == 0) find_bin(sm.hist, sm.bcast, krem, lane);
      __syncthreads();
      const uint32_t D = sm.bcast[0];
      krem = sm.bcast[1];
      const uint32_t n_c = sm.bcast[2];
      if (D == TOP) {
        // the k-th lies below the range (first pass only: its low end is an estimate)
        hi = lo - 1u;
        lo = k_min;
        continue;
      }
      const uint32_t bin_lo = lo + (D << s);
      if (krem == n_c) {     // the whole bin is selected
        tau = bin_lo - 1u;
        r = 0u;
        break;
      }
      if (s == 0) {          // bins are single keys: krem of the n_c copies of this key are selected
        tau = bin_lo;
        r = krem;
        break;
      }
      const uint32_t span = (1u << s) - 1u;
      hi = (hi - bin_lo) > span ? bin_lo + span : hi;
      lo = bin_lo;
      if (!on_list && n_c <= (uint32_t)CAP) {
        on_list = true;
        n_listed = n_c;
#pragma unroll
        for (int j = 0; j < E; ++j)
          if (key[j] - lo <= hi - lo) sm.list[atomicAdd(&sm.n_list, 1u)] = (uint16_t)(i0 + j);
      }
    }
  }

  // Positions in index order: thread t's elements precede thread t+1's, so an exclusive scan of
  // the per-thread counts (selected-for-sure, equal-to-threshold) gives every thread its base.
  if (r == 0u) {
    // no key equal to the threshold is taken (the usual end of the search: a bin taken whole, or
    // everything selected): one count and one scan
    uint32_t g_cnt = 0;
#pragma unroll
    for (int j = 0; j < E; ++j) g_cnt += key[j] > tau;
    const uint32_t g_inc = wave_scan_add(g_cnt);
    __syncthreads();   // sm.red is free again
    if (lane == 63) sm.red[wave] = g_inc;
    __syncthreads();
    uint32_t g_run = g_inc - g_cnt;
#pragma unroll
    for (int v = 0; v < NW; ++v)
      if (v < wave) g_run += sm.red[v];
#pragma unroll
    for (int j = 0; j < E; ++j) {
      if (key[j] > tau) {
        emit((int)g_run, i0 + j, key[j]);
        ++g_run;
      }
    }
    return n_valid < k ? n_valid : k;
  }
  uint32_t g_cnt = 0, e_cnt = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) {
    g_cnt += key[j] > tau;
    e_cnt += key[j] == tau;   // (r > 0 implies tau != 0)
  }
  const uint32_t g_inc = wave_scan_add(g_cnt), e_inc = wave_scan_add(e_cnt);
  __syncthreads();   // sm.red is free again
  if (lane == 63) {
    sm.red[wave] = g_inc;
    sm.red[NW + wave] = e_inc;
  }
  __syncthreads();
  uint32_t g_run = g_inc - g_cnt, e_run = e_inc - e_cnt;
#pragma unroll
  for (int v = 0; v < NW; ++v) {
    if (v < wave) {
      g_run += sm.red[v];
      e_run += sm.red[NW + v];
    }
  }
#pragma unroll
  for (int j = 0; j < E; ++j) {
    const bool gt = key[j] > tau;
    const bool eq = key[j] == tau;
    if (gt || (eq && e_run < r)) emit((int)(g_run + (e_run < r ? e_run : r)), i0 + j, key[j]);
    g_run += gt;
    e_run += eq;
  }
  return n_valid < k ? n_valid : k;
}

// ------------------------------------------------------------------------------------------
// Fast path of the top-k behind the fused Stage 2 scoring: ONE histogram pass with bins fine enough
// (2048 or more over the row's own score range) that the bin holding the k-th score has a handful of
// entries, whose k-th is then found by counting.  The threshold tau is a score of the row, and the
// path emits only after it has CHECKED that exactly k scores are >= tau: then those k are the top
// k whatever the binning did (ties at tau are either all in or the check fails).  On any doubt -- a
// crowded bin, the k-th among the masked entries, ties across the threshold, a count that does not
// come out -- it returns false BEFORE writing anything, and the caller runs select_topk.
// Its scratch is NOT shared with anything else in the kernel, so that the bins can be zeroed at
// kernel start and the row's score range can be collected by the scoring waves as they go: the
// select itself then needs five workgroup barriers (the general select: about sixteen).
//   fine_select_prepare      at kernel start, every thread;
//   fine_select_range        after a wave's last score, every lane (x_max / x_min: the largest and
//                            smallest score the lane has produced, NaN entries ignored), BEFORE the
//                            barrier that ends scoring;
//   select_topk_fine         after that barrier, every thread.  vals(q) -> the scores of elements
//                            4q .. 4q+3 as stored (NaN: not a candidate); thread t owns the E
//                            consecutive elements from t*E; emit(pos, v, tau, dump): the thread's
//                            selected elements are those with v[j] >= tau, the first of them is the
//                            pos-th selected of the row (ascending element index); dump is an LDS
//                            word of the thread's own that may be overwritten.
template <int NT, int E>
struct FineSelSmem {
  static constexpr int NBIN = NT <= 512 ? 2048 : 4 * NT, LCAP = 64, NW = NT / 64;   // >= 4 bins per thread
  uint32_t hist[NBIN];
  float row_max[NW], row_min[NW];
  uint32_t tot_a[NW], tot_b[NW];
  uint32_t n_list;
  float list_v[LCAP];
};

__device__ __forceinline__ float vmax_f32(float a, float b) {   // IEEE maxNum in one instruction: a NaN operand is ignored
  float r;
  asm("v_max_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ float vmin_f32(float a, float b) {
  float r;
  asm("v_min_f32 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ __forceinline__ uint32_t cvt_u32_sat(float t) {      // floor for t >= 0; negatives and NaN give 0
  uint32_t r;
  asm("v_cvt_u32_f32 %0, %1" : "=v"(r) : "v"(t));
  return r;
}
__device__ __forceinline__ float wave_max_f32(float v) {
  return __uint_as_float(wave_all(__float_as_uint(v), [](uint32_t a, uint32_t b) {
    return __float_as_uint(vmax_f32(__uint_as_float(a), __uint_as_float(b)));
  }));
}

template <int NT, int E>
__device__ __forceinline__ void fine_select_prepare(FineSelSmem<NT, E>& sm) {
  uint4* h4 = reinterpret_cast<uint4*>(sm.hist);
  for (int b = threadIdx.x; b < FineSelSmem<NT, E>::NBIN / 4; b += NT) h4[b] = make_uint4(0u, 0u, 0u, 0u);
  if (threadIdx.x == 0) sm.n_list = 0u;
}

template <int NT, int E>
__device__ __forceinline__ void fine_select_range(FineSelSmem<NT, E>& sm, float x_max, float x_min, int wave) {
  const float w_max = wave_max_f32(x_max);
  const float w_min = -wave_max_f32(-x_min);
  if (lane_id() == 0) {
    sm.row_max[wave] = w_max;
    sm.row_min[wave] = w_min;
  }
}

template <int NT, int E, class Vals, class Emit>
__device__ __forceinline__ bool select_topk_fine(FineSelSmem<NT, E>& sm, int n, int k, Vals vals, Emit emit) {
  static_assert(E % 4 == 0, "elements per thread come in groups of four");
  using S = FineSelSmem<NT, E>;
  constexpr int NW = S::NW, NBIN = S::NBIN, BPT = NBIN / NT;
  static_assert(BPT % 4 == 0, "a thread scans whole 16-byte groups of bins");
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i0 = tid * E;
  const float qnan = __uint_as_float(0xffffffffu);
  const float inf = __builtin_inff();

  // ---- the thread's scores.  A thread lies wholly inside the row, wholly outside it (only NaN), or
  // -- one thread of the row at most -- across its end: only that one checks every element.
  typedef float valvec __attribute__((ext_vector_type(E)));
  valvec v;
  const bool whole = i0 + E <= n;
  const bool has_any = i0 < n;
#pragma unroll
  for (int j = 0; j < E; ++j) v[j] = qnan;
  if (whole) {
#pragma unroll
    for (int g = 0; g < E / 4; ++g) {
      const float4 q4 = vals((i0 >> 2) + g);
      v[4 * g + 0] = q4.x;
      v[4 * g + 1] = q4.y;
      v[4 * g + 2] = q4.z;
      v[4 * g + 3] = q4.w;
    }
  } else if (has_any) {
#pragma unroll
    for (int g = 0; g < E / 4; ++g) {
      float4 q4 = make_float4(qnan, qnan, qnan, qnan);
      if (i0 + 4 * g < n) q4 = vals((i0 >> 2) + g);
      const float x[4] = {q4.x, q4.y, q4.z, q4.w};
#pragma unroll
      for (int e = 0; e < 4; ++e) v[4 * g + e] = (i0 + 4 * g + e < n) ? x[e] : qnan;
    }
  }
  // ---- range of the bins: the row's own [minimum, maximum].  (A thread's E consecutive candidates
  // are a piece of one key block, whose scores move together: an estimate built from per-thread
  // extremes lands anywhere.)
  float hi = -inf, lo = inf;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    hi = vmax_f32(hi, sm.row_max[w]);
    lo = vmin_f32(lo, sm.row_min[w]);
  }
  if (!(hi > lo) || !(hi - lo < inf)) return false;          // empty, constant or overflowing range (uniform)
  // bin(x) = 1 + floor((x - lo) * scale) in 1 .. NBIN-1 for lo <= x <= hi, 0 for NaN: monotone in x, so
  // every score in a higher bin is larger than every score in a lower one.  scale stops a hair
  // short of (NBIN - 2) / (hi - lo), so the top bin needs no clamp.  A thread keeps, per element,
  // the LDS byte address of its bin (4 * bin + the histogram's base): one multiply-add, one
  // conversion that rounds down (negative and NaN give 0), one mask.
  const float scale4 = 4.0f * (float)(NBIN - 2) * (1.0f - 0x1p-18f) / (hi - lo);
  const uint32_t hist_base = lds_address(sm.hist);
  const float bias4 = 4.0f + (float)hist_base - lo * scale4;
  typedef uint32_t binvec __attribute__((ext_vector_type(E)));
  binvec bin;
#pragma unroll
  for (int j = 0; j < E; ++j) bin[j] = 0u;
  if (has_any) {                   // (threads past the row hold only NaN: they would all hit bin 0)
    uint32_t one;
    asm volatile("v_mov_b32 %0, 1" : "=v"(one));               // (kept in a register across the atomics below)
#pragma unroll
    for (int j = 0; j < E; ++j) {
      const uint32_t addr = cvt_u32_sat(__builtin_fmaf(v[j], scale4, bias4)) & ~3u;
      bin[j] = addr;
      // NaN: the conversion gives 0, below the histogram; it is counted in bin 0
      const uint32_t a_ok = addr > hist_base ? addr : hist_base;
      asm volatile("ds_add_u32 %0, %1" : : "v"(a_ok), "v"(one) : "memory");
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");         // (the compiler does not count these)
  }
  __syncthreads();                                             // 1: histogram complete
  // ---- the bin that holds the k-th largest: counts above it < k <= counts above it + its own.
  // Thread t owns bins t*BPT ..: wave totals first, then EVERY wave scans the bins of the wave that
  // holds the k-th, so that all of them know the bin without another barrier.
  auto bins_of = [&](int t, uint32_t (&c)[BPT]) -> uint32_t {
    uint32_t sum = 0;
#pragma unroll
    for (int g = 0; g < BPT / 4; ++g) {
      const uint4 c4 = *reinterpret_cast<const uint4*>(&sm.hist[t * BPT + 4 * g]);
      c[4 * g + 0] = c4.x;
      c[4 * g + 1] = c4.y;
      c[4 * g + 2] = c4.z;
      c[4 * g + 3] = c4.w;
      sum += (c4.x + c4.y) + (c4.z + c4.w);
    }
    return sum;
  };
  uint32_t c[BPT];
  {
    const uint32_t w_tot = wave_sum(bins_of(tid, c));
    if (lane == 0) sm.tot_a[wave] = w_tot;
  }
  __syncthreads();                                             // 2: wave totals visible
  int w_star = -1;
  uint32_t above_w = 0;
#pragma unroll
  for (int w = NW - 1; w >= 0; --w) {
    const uint32_t tw = sm.tot_a[w];
    if (w_star < 0) {
      if ((uint32_t)k <= above_w + tw) w_star = w;
      else above_w += tw;
    }
  }
  if (w_star < 0) return false;                                // (cannot happen: the bins hold NT * E >= n > k entries)
  const uint32_t mine = bins_of(w_star * 64 + lane, c);
  uint32_t above = above_w + (wave_sum(mine) - wave_scan_add(mine));   // entries in the bins above this lane's
  uint32_t f_bin = 0, f_rem = 0, f_cnt = 0;
  bool found = false;
#pragma unroll
  for (int b = BPT - 1; b >= 0; --b) {
    if (above < (uint32_t)k && (uint32_t)k <= above + c[b]) {
      found = true;
      f_bin = hist_base + 4u * (uint32_t)((w_star * 64 + lane) * BPT + b);   // the bin as its LDS address
      f_rem = (uint32_t)k - above;
      f_cnt = c[b];
    }
    above += c[b];
  }
  const uint64_t who_bin = __ballot(found);
  if (who_bin == 0ull) return false;
  const int src = __builtin_ctzll(who_bin);
  const uint32_t D = (uint32_t)__builtin_amdgcn_readlane((int)f_bin, src);
  const uint32_t krem = (uint32_t)__builtin_amdgcn_readlane((int)f_rem, src);
  const uint32_t n_c = (uint32_t)__builtin_amdgcn_readlane((int)f_cnt, src);
  if (D == hist_base || n_c > (uint32_t)S::LCAP) return false;  // the k-th among the masked entries, or a crowded bin
  // ---- the scores of that bin (a handful in the whole row): eight compares at a time are OR-ed in
  // scalar registers, and only a wave that holds one of them walks those eight elements
  constexpr int G = E >= 8 ? 8 : 4;
#pragma unroll
  for (int g = 0; g < E / G; ++g) {
    bool any = false;
#pragma unroll
    for (int j = g * G; j < (g + 1) * G; ++j) any |= bin[j] == D;
    if (__ballot(any) != 0ull) {
#pragma unroll
      for (int j = g * G; j < (g + 1) * G; ++j) {
        if (bin[j] == D) {
          const uint32_t slot = atomicAdd(&sm.n_list, 1u);
          if (slot < (uint32_t)S::LCAP) sm.list_v[slot] = v[j];
        }
      }
    }
  }
  __syncthreads();                                             // 3: list complete
  // their krem-th largest is the threshold: every wave ranks the list for itself (lane j takes
  // entry j, the others are handed round from lane to lane)
  const float x = lane < (int)n_c ? sm.list_v[lane] : qnan;
  uint32_t gt = 0, ge = 0;
  for (uint32_t i = 0; i < n_c; ++i) {
    const float y = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), (int)i));
    gt += y > x;
    ge += y >= x;
  }
  const bool is_kth = lane < (int)n_c && gt < krem && krem <= ge;
  const uint64_t who = __ballot(is_kth);
  if (who == 0ull) return false;
  const float tau = __uint_as_float(__builtin_amdgcn_readlane(__float_as_uint(x), __builtin_ctzll(who)));
  // ---- exactly k scores at or above tau?  (the check that makes the result exact)
  uint32_t cnt = 0;
#pragma unroll
  for (int j = 0; j < E; ++j) cnt += v[j] >= tau;
  const uint32_t c_incl = wave_scan_add(cnt);
  if (lane == 63) sm.tot_b[wave] = c_incl;
  __syncthreads();                                             // 4: counts visible
  uint32_t pos = c_incl - cnt, taken = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const uint32_t tw = sm.tot_b[w];
    taken += tw;
    if (w < wave) pos += tw;
  }
  if (taken != (uint32_t)k) return false;                      // ties across the threshold: not this path's case
  emit(pos, v, tau, reinterpret_cast<int32_t*>(&sm.hist[tid]));
  return true;
}

// fp32 -> bf16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint16_t f32_to_bf16_rne(float x) {
  const uint32_t b = __float_as_uint(x);
  return (uint16_t)((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

}  // namespace hisa
