// Host side of the C ABI declared in include/hisa.h: argument validation, workspace carving and
// kernel launches.  Nothing here allocates or synchronises.
#include "../../include/hisa.h"

#include <hip/hip_runtime.h>

#include <atomic>

#include "hisa_kernels.h"

using namespace hisa;

namespace {

inline long round_up(long x, long a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int launch_status() { return hipGetLastError() == hipSuccess ? HISA_OK : HISA_ERR_LAUNCH; }

constexpr int kMaxK = 8192, kMaxM = 1024, kMaxCand = 65536;
constexpr int kMaxT = 1 << 22;        // queries per call
constexpr int kMaxSeq = 65535;        // sequences per key array (the y extent of the pooling grids)
constexpr long kMaxGrid = 1L << 30;   // workgroups per launch (the x extent of a grid stops at 2^31 - 1)
constexpr int kMaxDevices = 64;

// A kernel that asks for more than 64 KB of dynamic LDS needs its limit raised first.  Done once
// per kernel instance and device (again only if a later call needs more than any earlier one), not
// on every call.
template <auto Kern>
int raise_lds_limit(size_t bytes) {
  static std::atomic<int> granted[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return HISA_ERR_LAUNCH;
  if ((int)bytes <= granted[dev].load(std::memory_order_acquire)) return HISA_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(Kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                          (int)bytes) != hipSuccess)
    return HISA_ERR_LAUNCH;
  granted[dev].store((int)bytes, std::memory_order_release);
  return HISA_OK;
}

// Flat top-k over rows longer than one select pass holds: the k best of every 65536-entry
// segment, then the k best of those.  (16384-entry segments were measured slower: 53.5 ms against
// 49.3 ms for the 64K prefill.)
inline int flat_seg_len(long, int) { return 65536; }

enum Path { PATH_NONE = 0, PATH_F32 = 1, PATH_MFMA = 2 };

// Which arithmetic path a dtype combination takes (see "Supported shapes" in hisa.h).
int pick_path(int q_dtype, int k_dtype, int H, int d, int* status) {
  if (q_dtype == HISA_F32 && k_dtype == HISA_F32) {
    if (H < 1 || H > 128 || d < 4 || d > 512 || d % 4) { *status = HISA_ERR_SHAPE; return PATH_NONE; }
    return PATH_F32;
  }
  if (q_dtype == HISA_BF16 && (k_dtype == HISA_BF16 || k_dtype == HISA_FP8_E4M3)) {
    if (d != 128 || (H != 32 && H != 64)) { *status = HISA_ERR_SHAPE; return PATH_NONE; }
    return PATH_MFMA;
  }
  *status = HISA_ERR_DTYPE;
  return PATH_NONE;
}

int check_queries(const hisa_queries* q) {
  if (!q || !q->q || !q->w) return HISA_ERR_NULL;
  if (q->T < 1 || q->T > kMaxT || q->H < 1) return HISA_ERR_SHAPE;
  if (!aligned16(q->q)) return HISA_ERR_ALIGN;
  return HISA_OK;
}

int check_keys(const hisa_keys* k, bool need_data) {
  if (!k || !k->seq_len) return HISA_ERR_NULL;
  if (k->n_seq < 1 || k->n_seq > kMaxSeq || k->s_max < 1 || k->d < 1) return HISA_ERR_SHAPE;
  if (k->k_dtype < HISA_F32 || k->k_dtype > HISA_FP8_E4M3) return HISA_ERR_DTYPE;
  // one sequence's key array is addressed with 32-bit byte offsets (buffer descriptors)
  const long elem = k->k_dtype == HISA_F32 ? 4 : (k->k_dtype == HISA_BF16 ? 2 : 1);
  if ((long)k->s_max * k->d * elem >= (1L << 31)) return HISA_ERR_SHAPE;
  if (need_data) {
    if (!k->k) return HISA_ERR_NULL;
    if (k->k_dtype == HISA_FP8_E4M3 && !k->k_scale) return HISA_ERR_NULL;
    if (!aligned16(k->k)) return HISA_ERR_ALIGN;
  }
  return HISA_OK;
}

ScoreArgs base_args(const hisa_queries* q, const hisa_keys* k) {
  ScoreArgs a{};
  a.q = q->q;
  a.w = q->w;
  a.q_seq = q->q_seq;
  a.q_pos = q->q_pos;
  a.q_lo = q->q_lo;
  a.q_pos0 = q->q_pos0;
  a.H = q->H;
  a.d = k->d;
  a.keys = k->k;
  a.k_scale = k->k_dtype == HISA_FP8_E4M3 ? k->k_scale : nullptr;
  a.seq_len = k->seq_len;
  a.n_seq = k->n_seq;
  a.rows_per_seq = k->s_max;
  a.pos_div = 1;
  a.block_idx = nullptr;
  a.m = 0;
  a.B = 1;
  a.tiles_per_wave = 1;
  a.groups = 1;
  return a;
}

// ---- scoring launches -------------------------------------------------------------------
template <int KDT>
void launch_ranges_mfma(ScoreArgs a, int n_tiles_max, hipStream_t st) {
  a.groups = (n_tiles_max + 4 * a.tiles_per_wave - 1) / (4 * a.tiles_per_wave);
  dim3 grid((unsigned)((long)a.groups * a.t_count));
  if (a.H == 64)
    hipLaunchKernelGGL((k_score_ranges<2, KDT>), grid, dim3(256), 0, st, a);
  else
    hipLaunchKernelGGL((k_score_ranges<1, KDT>), grid, dim3(256), 0, st, a);
}

template <int KDT>
void launch_prefill_mfma(const ScoreArgs& a, hipStream_t st) {
  dim3 grid((a.t_count + 7) / 8);
  if (a.H == 64)
    hipLaunchKernelGGL((k_score_prefill<2, KDT>), grid, dim3(512), 0, st, a);
  else
    hipLaunchKernelGGL((k_score_prefill<1, KDT>), grid, dim3(512), 0, st, a);
}

// Scores `a.t_count` queries against up to n_rows_max rows each (flat / Stage 1: rows of the
// key array; gather: m*B slots).  key_dt is the dtype of the rows.
void launch_score(int path, int key_dt, ScoreArgs a, long n_rows_max, bool consecutive,
                  hipStream_t st) {
  if (path == PATH_F32) {
    const int per_wg = 1024;
    a.groups = (int)((n_rows_max + per_wg - 1) / per_wg);
    dim3 grid((unsigned)((long)a.groups * a.t_count));
    const size_t sh = ((size_t)a.H * a.d + a.H) * sizeof(float);
    hipLaunchKernelGGL(k_score_ranges_f32, grid, dim3(256), sh, st, a, per_wg);
    return;
  }
  const bool gather = a.block_idx != nullptr;
  if (!gather && consecutive && a.t_count >= 2048 && key_dt == HISA_BF16 && a.rows_per_seq <= 512) {
    // all rows fit in LDS (Stage 1 up to 512 blocks): resident tiles, 64 queries per workgroup
    constexpr int NQ = 8;
    const size_t sh = (size_t)((a.rows_per_seq + 31) / 32) * 8192;
    dim3 grid((a.t_count + 8 * NQ - 1) / (8 * NQ));
    // (a refusal to raise the LDS limit makes the launch fail, which the entry point reports)
    if (a.H == 64) {
      (void)raise_lds_limit<k_score_resident<2, NQ>>(sh);
      hipLaunchKernelGGL((k_score_resident<2, NQ>), grid, dim3(512), sh, st, a);
    } else {
      (void)raise_lds_limit<k_score_resident<1, NQ>>(sh);
      hipLaunchKernelGGL((k_score_resident<1, NQ>), grid, dim3(512), sh, st, a);
    }
    return;
  }
  if (!gather && consecutive && a.t_count >= 64) {
    if (key_dt == HISA_BF16) launch_prefill_mfma<DT_BF16>(a, st);
    else launch_prefill_mfma<DT_FP8>(a, st);
    return;
  }
  const int n_tiles = (int)((n_rows_max + 31) / 32);
  // few queries: spread one query's tiles over many workgroups; many queries: amortise the
  // query-fragment load over more tiles
  int tpw = a.t_count >= 1024 ? 8 : (a.t_count >= 128 ? 4 : 2);
  if (gather) tpw = a.t_count >= 1024 ? 16 : 4;
  a.tiles_per_wave = tpw;
  if (key_dt == HISA_BF16) launch_ranges_mfma<DT_BF16>(a, n_tiles, st);
  else launch_ranges_mfma<DT_FP8>(a, n_tiles, st);
}

// ---- selection launches -----------------------------------------------------------------
template <int MAP>
int launch_select(const SelectArgs& a, int rows, int n_max, hipStream_t st) {
  dim3 grid((unsigned)((long)a.n_seg * rows));
  if (n_max <= 512)
    hipLaunchKernelGGL((k_select<64, 8, MAP>), grid, dim3(64), 0, st, a);
  else if (n_max <= 2048)
    hipLaunchKernelGGL((k_select<256, 8, MAP>), grid, dim3(256), 0, st, a);
  else if (n_max <= 8192 && rows * a.n_seg <= 256)
    // a decode batch: most CUs idle anyway, so a row gets 16 waves and a quarter of the work per thread
    hipLaunchKernelGGL((k_select<1024, 8, MAP>), grid, dim3(1024), 0, st, a);
  else if (n_max <= 8192)
    hipLaunchKernelGGL((k_select<256, 32, MAP>), grid, dim3(256), 0, st, a);
  else if (n_max <= 16384)
    hipLaunchKernelGGL((k_select<1024, 16, MAP>), grid, dim3(1024), 0, st, a);
  else if (n_max <= 65536)
    hipLaunchKernelGGL((k_select<1024, 64, MAP>), grid, dim3(1024), 0, st, a);
  else
    return HISA_ERR_SHAPE;
  return HISA_OK;
}

SelectArgs select_base(const hisa_queries* q, const hisa_keys* k) {
  SelectArgs s{};
  s.q_seq = q->q_seq;
  s.q_pos = q->q_pos;
  s.q_lo = q->q_lo;
  s.seq_len = k->seq_len;
  s.q_pos0 = q->q_pos0;
  s.n_seq = k->n_seq;
  s.pos_div = 1;
  s.seg_len = 1 << 30;
  s.n_seg = 1;
  return s;
}

// Fused Stage 2: kFusedWaves waves per query; EC = candidates per thread of a 256-thread select
// (16: up to 4096 candidates, 32: up to 8192, 64: up to 16384); with 8 waves the per-thread count halves.
template <int HG, int KDT, int EC>
int launch_fused_hg(const ScoreArgs& a, int k, int32_t* topk_idx, float* topk_scores,
                    hipStream_t st) {
  // more than 8192 candidates: their scores (64 KB) leave room for one workgroup per CU only, so
  // that one gets 8 waves (two per SIMD; and 32 instead of 64 candidates per thread in the select)
  constexpr int NW = EC > 32 ? 8 : kFusedWaves;
  constexpr int E = ((EC * 4 + NW - 1) / NW + 3) / 4 * 4;
  const size_t sh = (size_t)NW * kNBuf * TileGeom<KDT>::kBufBytes + (size_t)a.m * a.B * 4 +
                    sizeof(FineSelSmem<NW * 64, E>);
  constexpr auto kern = k_refine_fused<HG, KDT, NW, kNBuf, E>;
  if (raise_lds_limit<kern>(sh)) return HISA_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(a.t_count), dim3(NW * 64), sh, st, a, k, topk_idx, topk_scores,
                     (const void*)nullptr, (int32_t*)nullptr, 0);
  return HISA_OK;
}

template <int KDT, int EC>
int launch_fused(const ScoreArgs& a, int k, int32_t* topk_idx, float* topk_scores, hipStream_t st) {
  return a.H == 64 ? launch_fused_hg<2, KDT, EC>(a, k, topk_idx, topk_scores, st)
                   : launch_fused_hg<1, KDT, EC>(a, k, topk_idx, topk_scores, st);
}

// Single-launch HISA (Stage 1 + Stage 2 in k_refine_fused): NW waves per query; the Stage 1
// select holds E1 blocks per thread (NW * 64 * E1 >= 8192 blocks).
template <int HG, int KDT, int NW, int EC>
int launch_indexer_hg(const ScoreArgs& a, const void* pooled, int k, int32_t* block_idx_out,
                      int32_t* topk_idx, float* topk_scores, hipStream_t st) {
  constexpr int E = ((EC * 4 + NW - 1) / NW + 3) / 4 * 4;
  constexpr int E1 = NW == 4 ? 32 : 16;
  const int M = (int)(a.rows_per_seq / a.B);
  const int sc_floats = (int)round_up(a.m * a.B > M ? a.m * a.B : M, 32);
  const size_t tile = TileGeom<KDT>::kBufBytes < 8192 ? 8192 : TileGeom<KDT>::kBufBytes;
  const size_t sh = (size_t)NW * kNBuf * tile + (size_t)sc_floats * 4 + (size_t)round_up(a.m, 4) * 4 +
                    sizeof(FineSelSmem<NW * 64, E>);
  constexpr auto kern = k_refine_fused<HG, KDT, NW, kNBuf, E, E1>;
  if (raise_lds_limit<kern>(sh)) return HISA_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(a.t_count), dim3(NW * 64), sh, st, a, k, topk_idx, topk_scores, pooled,
                     block_idx_out, sc_floats);
  return HISA_OK;
}

template <int KDT, int NW>
int launch_indexer(const ScoreArgs& a, const void* pooled, int k, int32_t* block_idx_out,
                   int32_t* topk_idx, float* topk_scores, hipStream_t st) {
  const bool big = (long)a.m * a.B > 8192;
  if (a.H == 64)
    return big ? launch_indexer_hg<2, KDT, NW, 64>(a, pooled, k, block_idx_out, topk_idx, topk_scores, st)
               : launch_indexer_hg<2, KDT, NW, 32>(a, pooled, k, block_idx_out, topk_idx, topk_scores, st);
  return big ? launch_indexer_hg<1, KDT, NW, 64>(a, pooled, k, block_idx_out, topk_idx, topk_scores, st)
             : launch_indexer_hg<1, KDT, NW, 32>(a, pooled, k, block_idx_out, topk_idx, topk_scores, st);
}

// Stage 1 of a small batch in one launch (k_stage1_query): M blocks per sequence, E1 per thread.
template <int HG, int E1>
int launch_stage1_query_e(const ScoreArgs& a, const void* pooled, int M, int32_t* block_idx, hipStream_t st) {
  const int sc_floats = (int)round_up(M, 32);
  // up to 2048 blocks a ring of two tiles per wave fits beside the scores, above that a ring of one
  constexpr int NB = E1 <= 4 ? 2 : 1;
  const size_t sh = (size_t)8 * NB * 8192 + (size_t)sc_floats * 4 + (size_t)round_up(a.m, 4) * 4 + (size_t)HG * 8192;
  constexpr auto kern = k_stage1_query<HG, E1, NB>;
  if (raise_lds_limit<kern>(sh)) return HISA_ERR_LAUNCH;
  hipLaunchKernelGGL(kern, dim3(a.t_count), dim3(512), sh, st, a, pooled, block_idx, sc_floats);
  return HISA_OK;
}

constexpr int kStage1QueryMaxT = 256;    // one workgroup per query: while the queries are fewer than the CUs
constexpr int kStage1QueryMaxM = 8192;   // 512 threads x 16 blocks

int launch_stage1_query(const ScoreArgs& a, const void* pooled, int M, int32_t* block_idx, hipStream_t st) {
  if (M <= 2048)
    return a.H == 64 ? launch_stage1_query_e<2, 4>(a, pooled, M, block_idx, st)
                     : launch_stage1_query_e<1, 4>(a, pooled, M, block_idx, st);
  return a.H == 64 ? launch_stage1_query_e<2, 16>(a, pooled, M, block_idx, st)
                   : launch_stage1_query_e<1, 16>(a, pooled, M, block_idx, st);
}

// Flat indexer: rows of queries scored per chunk, and the size of the segment-merge area.
struct FlatPlan {
  long ld;          // score row stride (floats)
  int seg_len;      // entries per segment
  int n_seg;        // segments per row
  long per_query;   // workspace bytes per query in a chunk
};

// Rows longer than 16384 entries with k <= 2048 go through the streaming select, which takes a
// row of any length whole; other rows are selected from registers, in segments above 65536.
bool flat_streams(const hisa_keys* k, int kk) { return k->s_max > 16384 && kk <= StreamSelect::kMaxK; }

FlatPlan flat_plan(const hisa_keys* k, int kk) {
  FlatPlan p;
  p.ld = round_up(k->s_max, 64);
  p.seg_len = flat_streams(k, kk) ? k->s_max : flat_seg_len(k->s_max, kk);
  p.n_seg = (int)((k->s_max + p.seg_len - 1) / p.seg_len);
  p.per_query = p.ld * 4 + (p.n_seg > 1 ? (long)p.n_seg * kk * 8 : 0);
  return p;
}

}  // namespace

extern "C" {

const char* hisa_status_string(int status) {
  switch (status) {
    case HISA_OK: return "ok";
    case HISA_ERR_NULL: return "a required pointer is NULL";
    case HISA_ERR_SHAPE: return "shape outside the supported set";
    case HISA_ERR_DTYPE: return "unsupported dtype combination";
    case HISA_ERR_INFEASIBLE: return "infeasible budgets: need m >= 2 and m*B >= k";
    case HISA_ERR_WORKSPACE: return "workspace missing or too small";
    case HISA_ERR_ALIGN: return "tensor pointer not 16-byte aligned";
    case HISA_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
  }
}

const char* hisa_version(void) { return "0.4"; }


static int pool_blocks_impl(const hisa_keys* keys, int32_t B, int32_t blk_begin, int32_t blk_end,
                            void* pooled, int32_t pooled_dtype, bool max_pool, void* stream) {
  int st = check_keys(keys, true);
  if (st) return st;
  if (!pooled) return HISA_ERR_NULL;
  if (B < 1 || keys->s_max % B) return HISA_ERR_SHAPE;
  const int M = keys->s_max / B;
  if (blk_begin < 0 || blk_end > M || blk_begin > blk_end) return HISA_ERR_SHAPE;
  const int kd = keys->k_dtype, d = keys->d;
  const int vec = kd == HISA_F32 ? 4 : (kd == HISA_BF16 ? 8 : 16);
  if (d % vec || d / vec > 256) return HISA_ERR_SHAPE;
  if (!((kd == HISA_F32 && pooled_dtype == HISA_F32) ||
        (kd != HISA_F32 && (pooled_dtype == HISA_BF16 || pooled_dtype == HISA_F32))))
    return HISA_ERR_DTYPE;
  if (blk_begin == blk_end) return HISA_OK;
  hipStream_t s = (hipStream_t)stream;
  dim3 grid(blk_end - blk_begin, keys->n_seq);
#define POOL(KD, PD)                                                                             \
  do {                                                                                           \
    if (max_pool)                                                                                \
      hipLaunchKernelGGL((k_pool<KD, PD, true>), grid, dim3(256), 0, s, keys->k, keys->k_scale,  \
                         keys->seq_len, (long)keys->s_max, d, B, blk_begin, pooled);             \
    else                                                                                         \
      hipLaunchKernelGGL((k_pool<KD, PD, false>), grid, dim3(256), 0, s, keys->k, keys->k_scale, \
                         keys->seq_len, (long)keys->s_max, d, B, blk_begin, pooled);             \
  } while (0)
  if (kd == HISA_F32) POOL(DT_F32, DT_F32);
  else if (kd == HISA_BF16 && pooled_dtype == HISA_BF16) POOL(DT_BF16, DT_BF16);
  else if (kd == HISA_BF16) POOL(DT_BF16, DT_F32);
  else if (pooled_dtype == HISA_BF16) POOL(DT_FP8, DT_BF16);
  else POOL(DT_FP8, DT_F32);
#undef POOL
  return launch_status();
}

int hisa_pool_blocks(const hisa_keys* keys, int32_t B, int32_t blk_begin, int32_t blk_end,
                     void* pooled, int32_t pooled_dtype, void* stream) {
  return pool_blocks_impl(keys, B, blk_begin, blk_end, pooled, pooled_dtype, false, stream);
}

int hisa_pool_blocks_max(const hisa_keys* keys, int32_t B, int32_t blk_begin, int32_t blk_end,
                         void* pooled, int32_t pooled_dtype, void* stream) {
  return pool_blocks_impl(keys, B, blk_begin, blk_end, pooled, pooled_dtype, true, stream);
}

int hisa_pool_append(const hisa_keys* keys, int32_t B, const int32_t* prev_len, int32_t max_new_tokens,
                     void* pooled, int32_t pooled_dtype, void* stream) {
  int st = check_keys(keys, true);
  if (st) return st;
  if (!pooled || !prev_len) return HISA_ERR_NULL;
  if (B < 1 || keys->s_max % B || max_new_tokens < 0) return HISA_ERR_SHAPE;
  const int kd = keys->k_dtype, d = keys->d;
  const int vec = kd == HISA_F32 ? 4 : (kd == HISA_BF16 ? 8 : 16);
  if (d % vec || d / vec > 256) return HISA_ERR_SHAPE;
  if (!((kd == HISA_F32 && pooled_dtype == HISA_F32) ||
        (kd != HISA_F32 && (pooled_dtype == HISA_BF16 || pooled_dtype == HISA_F32))))
    return HISA_ERR_DTYPE;
  if (max_new_tokens == 0) return HISA_OK;
  // max_new_tokens appended tokens touch at most this many blocks (the first may be partial)
  const int n_blk = (max_new_tokens + B - 2) / B + 1;
  hipStream_t s = (hipStream_t)stream;
  dim3 grid(n_blk, keys->n_seq);
#define POOLA(KD, PD)                                                                            \
  hipLaunchKernelGGL((k_pool_append<KD, PD>), grid, dim3(256), 0, s, keys->k, keys->k_scale,     \
                     keys->seq_len, prev_len, (long)keys->s_max, d, B, pooled)
  if (kd == HISA_F32) POOLA(DT_F32, DT_F32);
  else if (kd == HISA_BF16 && pooled_dtype == HISA_BF16) POOLA(DT_BF16, DT_BF16);
  else if (kd == HISA_BF16) POOLA(DT_BF16, DT_F32);
  else if (pooled_dtype == HISA_BF16) POOLA(DT_FP8, DT_BF16);
  else POOLA(DT_FP8, DT_F32);
#undef POOLA
  return launch_status();
}

int hisa_block_sparse_tokens(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                             const int32_t* block_idx, int32_t* tokens, void* stream) {
  if (!queries || !keys || !keys->seq_len) return HISA_ERR_NULL;
  if (!block_idx || !tokens) return HISA_ERR_NULL;
  if (queries->T < 1 || keys->n_seq < 1 || keys->s_max < 1) return HISA_ERR_SHAPE;
  if (B < 1 || keys->s_max % B || m < 1 || m > kMaxM || (long)m * B > kMaxCand) return HISA_ERR_SHAPE;
  ScoreArgs a{};
  a.q_seq = queries->q_seq;
  a.q_pos = queries->q_pos;
  a.q_lo = queries->q_lo;
  a.q_pos0 = queries->q_pos0;
  a.seq_len = keys->seq_len;
  a.n_seq = keys->n_seq;
  a.rows_per_seq = keys->s_max;
  a.pos_div = 1;
  a.block_idx = block_idx;
  a.m = m;
  a.B = B;
  const int gx = (m * B + 255) / 256;
  a.groups = gx > 16 ? 16 : gx;
  hipLaunchKernelGGL(k_block_sparse_tokens, dim3((unsigned)((long)a.groups * queries->T)), dim3(256), 0,
                     (hipStream_t)stream, a, tokens);
  return launch_status();
}

int hisa_index_iou(const int32_t* a_idx, const int32_t* b_idx, int32_t T, int32_t k, float* iou,
                   void* stream) {
  if (!a_idx || !b_idx || !iou) return HISA_ERR_NULL;
  if (T < 1 || k < 1) return HISA_ERR_SHAPE;
  if (k <= 4096)
    hipLaunchKernelGGL(k_index_iou<true>, dim3((T + 3) / 4), dim3(256), (size_t)4 * k * sizeof(int32_t),
                       (hipStream_t)stream, a_idx, b_idx, T, k, iou);
  else
    hipLaunchKernelGGL(k_index_iou<false>, dim3((T + 3) / 4), dim3(256), 0, (hipStream_t)stream, a_idx, b_idx, T, k,
                       iou);
  return launch_status();
}

int hisa_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return HISA_ERR_NULL;
  if (bytes < 16 || bytes % 16) return HISA_ERR_SHAPE;
  if (!aligned16(src) || !aligned16(dst)) return HISA_ERR_ALIGN;
  hipLaunchKernelGGL(k_probe_copy, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const uint4*)src,
                     (uint4*)dst, (long)(bytes / 16));
  return launch_status();
}

int hisa_probe_mfma(float* out, int32_t iters, double* flop, void* stream) {
  if (!out || !flop) return HISA_ERR_NULL;
  if (iters < 1) return HISA_ERR_SHAPE;
  const int wgs = 512;   // two 4-wave workgroups per CU: two waves per SIMD
  hipLaunchKernelGGL(k_probe_mfma, dim3(wgs), dim3(256), 0, (hipStream_t)stream, out, iters);
  *flop = (double)wgs * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
  return launch_status();
}

int hisa_probe_mfma_fp8(float* out, int32_t iters, double* flop, void* stream) {
  if (!out || !flop) return HISA_ERR_NULL;
  if (iters < 1) return HISA_ERR_SHAPE;
  const int wgs = 512;
  hipLaunchKernelGGL(k_probe_mfma_fp8, dim3(wgs), dim3(256), 0, (hipStream_t)stream, out, iters);
  *flop = (double)wgs * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 64);
  return launch_status();
}

int hisa_probe_mfma_toggling(float* out, int32_t iters, int32_t fp8, double* flop, void* stream) {
  if (!out || !flop) return HISA_ERR_NULL;
  if (iters < 1 || (fp8 != 0 && fp8 != 1)) return HISA_ERR_SHAPE;
  const int wgs = 512;
  if (fp8) {
    hipLaunchKernelGGL(k_probe_mfma_toggling<true>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, out, iters);
    *flop = (double)wgs * 4.0 * iters * 8.0 * (2.0 * 32 * 32 * 64);
  } else {
    hipLaunchKernelGGL(k_probe_mfma_toggling<false>, dim3(wgs), dim3(256), 0, (hipStream_t)stream, out, iters);
    *flop = (double)wgs * 4.0 * iters * 16.0 * (2.0 * 32 * 32 * 16);
  }
  return launch_status();
}

int hisa_block_score_topk(const hisa_queries* queries, const hisa_keys* keys, const void* pooled,
                          int32_t pooled_dtype, int32_t B, int32_t m, int32_t* block_idx,
                          float* block_scores, void* ws, size_t ws_bytes, void* stream) {
  int st = check_queries(queries);
  if (st) return st;
  st = check_keys(keys, false);
  if (st) return st;
  if (!pooled || !block_idx) return HISA_ERR_NULL;
  if (!aligned16(pooled)) return HISA_ERR_ALIGN;
  if (B < 1 || keys->s_max % B) return HISA_ERR_SHAPE;
  if (m < 2) return HISA_ERR_INFEASIBLE;
  if (m > kMaxM) return HISA_ERR_SHAPE;
  const int M = keys->s_max / B;
  if (M > kMaxCand) return HISA_ERR_SHAPE;
  // pooled keys play the part of the keys here
  int path = pick_path(queries->q_dtype, pooled_dtype == HISA_F32 ? HISA_F32 : HISA_BF16, queries->H,
                       keys->d, &st);
  if (!path) return st;
  if (pooled_dtype != HISA_F32 && pooled_dtype != HISA_BF16) return HISA_ERR_DTYPE;
  const int T = queries->T;
  hipStream_t s = (hipStream_t)stream;
  ScoreArgs a = base_args(queries, keys);
  float* J = block_scores;
  if (!J) {
    if (!ws || ws_bytes < (size_t)T * M * 4) return HISA_ERR_WORKSPACE;
    J = (float*)ws;
  }
  if (path == PATH_MFMA && pooled_dtype == HISA_BF16 && !block_scores && T <= kStage1QueryMaxT &&
      M <= kStage1QueryMaxM) {
    // a decode batch: scoring and selection of a query in one workgroup, nothing through the workspace
    a.B = B;
    a.m = m;
    a.t_begin = 0;
    a.t_count = T;
    st = launch_stage1_query(a, pooled, M, block_idx, s);
    if (st) return st;
    return launch_status();
  }
  a.keys = pooled;
  a.k_scale = nullptr;
  a.rows_per_seq = M;
  a.pos_div = B;
  a.out = J;
  a.ld = M;
  a.t_begin = 0;
  a.t_count = T;
  if (block_scores) {
    const long n = (long)T * M;
    hipLaunchKernelGGL(k_fill_f32, dim3((unsigned)((n + 255) / 256 > 4096 ? 4096 : (n + 255) / 256)),
                       dim3(256), 0, s, J, n, -__builtin_inff());
  }
  launch_score(path, pooled_dtype, a, M, !queries->q_seq && !queries->q_pos && !queries->q_lo, s);

  SelectArgs sa = select_base(queries, keys);
  sa.scores = J;
  sa.ld = M;
  sa.pos_div = B;
  sa.t_begin = 0;
  sa.k = m;
  sa.out_idx = block_idx;
  sa.out_scores = nullptr;
  st = launch_select<MAP_BLOCKS>(sa, T, M, s);
  if (st) return st;
  return launch_status();
}

// ---- Stage 2 for callers that cannot allocate ---------------------------------------------
// The candidate scores of the two-kernel path go through this array instead of a caller workspace.
// Every GPU the library runs on holds its own copy, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)HISA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) __attribute__((used)) unsigned char scratch[kStaticScratchBytes];

// Device address of `scratch` on the current device (in host code the array's name is only a
// handle for the symbol, not an address a kernel can use), looked up once per device.
static void* static_scratch_ptr() {
  static std::atomic<void*> ptrs[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = ptrs[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) return nullptr;
  ptrs[dev].store(p, std::memory_order_release);
  return p;
}

static int token_refine_impl(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                             const int32_t* block_idx, int32_t k, int32_t* topk_idx,
                             float* topk_scores, float* cand_scores, void* ws, size_t ws_bytes,
                             bool static_ws, void* stream) {
  int st = check_queries(queries);
  if (st) return st;
  st = check_keys(keys, true);
  if (st) return st;
  if (!block_idx || !topk_idx) return HISA_ERR_NULL;
  if (B < 1 || keys->s_max % B || k < 1 || k > kMaxK || m > kMaxM) return HISA_ERR_SHAPE;
  if (m < 2 || (long)m * B < k) return HISA_ERR_INFEASIBLE;
  if ((long)m * B > kMaxCand) return HISA_ERR_SHAPE;
  int path = pick_path(queries->q_dtype, keys->k_dtype, queries->H, keys->d, &st);
  if (!path) return st;
  if (path == PATH_MFMA && B % 32) return HISA_ERR_SHAPE;
  const int T = queries->T;
  const int n_slots = m * B;
  hipStream_t s = (hipStream_t)stream;

  ScoreArgs a = base_args(queries, keys);
  a.block_idx = block_idx;
  a.m = m;
  a.B = B;
  a.t_begin = 0;
  a.t_count = T;
  a.ld = n_slots;

  const bool fused = path == PATH_MFMA && !cand_scores && T >= 256 && n_slots <= 16384;
  if (fused) {
    a.out = nullptr;
    const bool bf = keys->k_dtype == HISA_BF16;
    if (n_slots <= 4096)       // half the candidates: half as many per thread in the top-k
      st = bf ? launch_fused<DT_BF16, 16>(a, k, topk_idx, topk_scores, s)
              : launch_fused<DT_FP8, 16>(a, k, topk_idx, topk_scores, s);
    else if (n_slots <= 8192)
      st = bf ? launch_fused<DT_BF16, 32>(a, k, topk_idx, topk_scores, s)
              : launch_fused<DT_FP8, 32>(a, k, topk_idx, topk_scores, s);
    else
      st = bf ? launch_fused<DT_BF16, 64>(a, k, topk_idx, topk_scores, s)
              : launch_fused<DT_FP8, 64>(a, k, topk_idx, topk_scores, s);
    if (st) return st;
    return launch_status();
  }

  float* C = cand_scores;
  if (!C) {
    if (static_ws) {
      // every argument has passed validation; only now is the device asked for the array's address
      if ((size_t)T * n_slots * 4 > kStaticScratchBytes) return HISA_ERR_WORKSPACE;
      ws = static_scratch_ptr();
      if (!ws) return HISA_ERR_LAUNCH;
      ws_bytes = kStaticScratchBytes;
    }
    if (!ws || ws_bytes < (size_t)T * n_slots * 4) return HISA_ERR_WORKSPACE;
    C = (float*)ws;
  }
  a.out = C;
  launch_score(path, keys->k_dtype, a, n_slots, false, s);

  SelectArgs sa = select_base(queries, keys);
  sa.scores = C;
  sa.ld = n_slots;
  sa.n_fixed = n_slots;
  sa.block_idx = block_idx;
  sa.m = m;
  sa.B = B;
  sa.t_begin = 0;
  sa.k = k;
  sa.out_idx = topk_idx;
  sa.out_scores = topk_scores;
  st = launch_select<MAP_CAND>(sa, T, n_slots, s);
  if (st) return st;
  return launch_status();
}

int hisa_token_refine_topk(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                           const int32_t* block_idx, int32_t k, int32_t* topk_idx,
                           float* topk_scores, float* cand_scores, void* ws, size_t ws_bytes,
                           void* stream) {
  return token_refine_impl(queries, keys, B, m, block_idx, k, topk_idx, topk_scores, cand_scores, ws, ws_bytes,
                           false, stream);
}

int hisa_token_refine_topk_static(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                                  const int32_t* block_idx, int32_t k, int32_t* topk_idx,
                                  float* topk_scores, void* stream) {
  return token_refine_impl(queries, keys, B, m, block_idx, k, topk_idx, topk_scores, nullptr, nullptr, 0, true,
                           stream);
}

int hisa_indexer_topk(const hisa_queries* queries, const hisa_keys* keys, const void* pooled,
                      int32_t pooled_dtype, int32_t B, int32_t m, int32_t k, int32_t* block_idx,
                      int32_t* topk_idx, float* topk_scores, void* stream) {
  int st = check_queries(queries);
  if (st) return st;
  st = check_keys(keys, true);
  if (st) return st;
  if (!pooled || !topk_idx) return HISA_ERR_NULL;
  if (!aligned16(pooled)) return HISA_ERR_ALIGN;
  if (B < 1 || keys->s_max % B || k < 1 || k > kMaxK || m > kMaxM) return HISA_ERR_SHAPE;
  if (m < 2 || (long)m * B < k) return HISA_ERR_INFEASIBLE;
  int path = pick_path(queries->q_dtype, keys->k_dtype, queries->H, keys->d, &st);
  if (!path) return st;
  if (path != PATH_MFMA || pooled_dtype != HISA_BF16) return HISA_ERR_DTYPE;
  if (B % 32 || (long)m * B > 16384 || keys->s_max / B > 8192) return HISA_ERR_SHAPE;
  ScoreArgs a = base_args(queries, keys);
  a.block_idx = nullptr;
  a.m = m;
  a.B = B;
  a.t_begin = 0;
  a.t_count = queries->T;
  hipStream_t s = (hipStream_t)stream;
  // few queries (decode): 8 waves per query shorten the one workgroup a query has; many queries:
  // 4 waves and two workgroups per CU, as in the Stage 2 kernel
  const bool wide = queries->T < 256;
  if (keys->k_dtype == HISA_BF16)
    st = wide ? launch_indexer<DT_BF16, 8>(a, pooled, k, block_idx, topk_idx, topk_scores, s)
              : launch_indexer<DT_BF16, 4>(a, pooled, k, block_idx, topk_idx, topk_scores, s);
  else
    st = wide ? launch_indexer<DT_FP8, 8>(a, pooled, k, block_idx, topk_idx, topk_scores, s)
              : launch_indexer<DT_FP8, 4>(a, pooled, k, block_idx, topk_idx, topk_scores, s);
  if (st) return st;
  return launch_status();
}

int dsa_flat_indexer_topk(const hisa_queries* queries, const hisa_keys* keys, int32_t k,
                          int32_t* topk_idx, float* topk_scores, void* ws, size_t ws_bytes,
                          void* stream) {
  int st = check_queries(queries);
  if (st) return st;
  st = check_keys(keys, true);
  if (st) return st;
  if (!topk_idx) return HISA_ERR_NULL;
  if (k < 1 || k > kMaxK) return HISA_ERR_SHAPE;
  int path = pick_path(queries->q_dtype, keys->k_dtype, queries->H, keys->d, &st);
  if (!path) return st;
  const FlatPlan p = flat_plan(keys, k);
  if ((long)p.n_seg * k > kMaxCand) return HISA_ERR_SHAPE;
  const int T = queries->T;
  if (!ws) return HISA_ERR_WORKSPACE;
  long chunk = (long)(ws_bytes / (size_t)p.per_query);
  if (chunk > T) chunk = T;
  {
    // a chunk's scoring launch holds chunk * (workgroups per row) workgroups: keep it a legal grid
    const long groups = path == PATH_F32 ? (keys->s_max + 1023L) / 1024 : (keys->s_max + 255L) / 256;
    if (chunk > kMaxGrid / groups) chunk = kMaxGrid / groups;
  }
  if (chunk >= 8) chunk = chunk / 8 * 8;
  if (chunk < 1 || (chunk < 8 && chunk < T)) return HISA_ERR_WORKSPACE;
  hipStream_t s = (hipStream_t)stream;
  float* scores = (float*)ws;
  float* part_sc = (float*)((char*)ws + chunk * p.ld * 4);
  int32_t* part_id = (int32_t*)((char*)part_sc + chunk * (long)p.n_seg * k * 4);
  const bool consecutive = !queries->q_seq && !queries->q_pos && !queries->q_lo;

  for (long t0 = 0; t0 < T; t0 += chunk) {
    const int tc = (int)((T - t0) < chunk ? (T - t0) : chunk);
    ScoreArgs a = base_args(queries, keys);
    a.out = scores;
    a.ld = p.ld;
    a.t_begin = (int)t0;
    a.t_count = tc;
    launch_score(path, keys->k_dtype, a, keys->s_max, consecutive, s);

    SelectArgs sa = select_base(queries, keys);
    sa.scores = scores;
    sa.ld = p.ld;
    sa.t_begin = (int)t0;
    sa.k = k;
    if (flat_streams(keys, k)) {
      sa.out_idx = topk_idx + t0 * k;
      sa.out_scores = topk_scores ? topk_scores + t0 * k : nullptr;
      if (raise_lds_limit<k_select_stream>(StreamSelect::kBytes)) return HISA_ERR_LAUNCH;
      hipLaunchKernelGGL(k_select_stream, dim3(tc), dim3(StreamSelect::kThreads), StreamSelect::kBytes, s, sa);
    } else if (p.n_seg == 1) {
      sa.out_idx = topk_idx + t0 * k;
      sa.out_scores = topk_scores ? topk_scores + t0 * k : nullptr;
      st = launch_select<MAP_FLAT>(sa, tc, keys->s_max, s);
      if (st) return st;
    } else {
      // two levels: the k best of every segment, then the k best of those
      sa.seg_len = p.seg_len;
      sa.n_seg = p.n_seg;
      sa.out_idx = part_id;
      sa.out_scores = part_sc;
      st = launch_select<MAP_FLAT>(sa, tc, p.seg_len, s);
      if (st) return st;
      SelectArgs sm = select_base(queries, keys);
      sm.scores = part_sc;
      sm.idx_in = part_id;
      sm.ld = (long)p.n_seg * k;
      sm.n_fixed = p.n_seg * k;
      sm.t_begin = (int)t0;
      sm.k = k;
      sm.out_idx = topk_idx + t0 * k;
      sm.out_scores = topk_scores ? topk_scores + t0 * k : nullptr;
      st = launch_select<MAP_PAIRS>(sm, tc, p.n_seg * k, s);
      if (st) return st;
    }
  }
  return launch_status();
}

size_t hisa_workspace_bytes(int op, const hisa_queries* queries, const hisa_keys* keys, int32_t B,
                            int32_t m, int32_t k, int32_t want_scores) {
  if (!queries || !keys || queries->T < 1 || keys->s_max < 1) return 0;
  const size_t T = (size_t)queries->T;
  switch (op) {
    case HISA_OP_POOL:
      return 0;
    case HISA_OP_BLOCK_SCORE_TOPK:
      if (B < 1 || keys->s_max % B || want_scores) return 0;
      return round_up((long)(T * (size_t)(keys->s_max / B) * 4), 256);
    case HISA_OP_TOKEN_REFINE_TOPK: {
      if (B < 1 || m < 1 || want_scores) return 0;
      const size_t n_slots = (size_t)m * B;
      const bool mfma = queries->q_dtype == HISA_BF16;
      if (mfma && T >= 256 && n_slots <= 16384) return 0;   // fused path
      return round_up((long)(T * n_slots * 4), 256);
    }
    case HISA_OP_FLAT_TOPK: {
      if (k < 1) return 0;
      const FlatPlan p = flat_plan(keys, k);
      long chunk = (4L << 30) / p.per_query;      // aim at <= 4 GiB
      if (chunk < 8) chunk = 8;
      if (chunk > (long)T) chunk = (long)T;
      chunk = round_up(chunk, 8);
      return (size_t)round_up(chunk * p.per_query, 256);
    }
    default:
      return 0;
  }
}

}  // extern "C"
