/*
 * hisa.h -- C ABI of the HISA hierarchical indexer for AMD MI355X (gfx950).
 *
 * The library computes, per query t, the token-index set that Sparse MLA consumes, by the
 * two-stage search of the HISA paper (Section 4.1, Algorithm 1), and the flat DSA indexer
 * (Section 3, Eqs. 1-2) as the baseline at the same shapes.
 *
 * Conventions for every call
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, row-major, densely packed.
 *     The descriptor structs themselves live in HOST memory.
 *   - The library allocates nothing and keeps no state.  Scratch memory is a caller-provided
 *     device workspace `ws` of `ws_bytes` bytes (256-byte aligned); hisa_workspace_bytes() gives
 *     the size a call wants.  A call may be given more; it never touches bytes past ws_bytes.
 *   - A call only enqueues kernels on `stream` (a hipStream_t passed as void*, NULL = the null
 *     stream) and returns without synchronising.  Calls sharing one workspace must be ordered on
 *     one stream.
 *   - Return value: HISA_OK, or an error code.  Validation is done on the host BEFORE anything is
 *     launched: on an error other than HISA_ERR_LAUNCH nothing was enqueued and outputs are
 *     untouched.  Device-resident arrays (seq_len, q_seq, q_pos, block_idx) cannot be validated
 *     on the host; kernels clamp positions to the sequence length so a bad value cannot cause an
 *     out-of-bounds access, but the result for that query is then unspecified.
 *   - Positions are 0-based.  The query at position p sees keys s <= p of its own sequence
 *     (Section 4.1, boundary behaviour: a prefix no longer than k is selected whole).
 *   - Top-k / top-m order candidates by score descending, ties by lower index.  Index outputs
 *     hold the selected ids in ASCENDING order, then -1 padding when fewer than k (m) exist.
 *
 * Supported shapes
 *   - q F32  + k F32  (+ pooled F32):  any H <= 128, d % 4 == 0, d <= 512  (plain fp32 ALU path)
 *   - q BF16 + k BF16 or FP8_E4M3 (+ pooled BF16):  d == 128, H in {32, 64}, B % 32 == 0
 *     (MFMA path, fp32 accumulation.  bf16 keys: bf16 MFMA.  fp8 keys: the stored codes go into
 *     the fp8 MFMA against the bf16 query written as the sum of two e4m3 numbers per element,
 *     after a power-of-two scaling per head; that sum is the query exactly except for elements
 *     2^9 below their head's largest, which keep 2^-17 of that largest; the per-token scale
 *     multiplies the finished score, which equals Eq. 1 on the dequantised key because the scale
 *     is positive.  Scores agree with a double-precision evaluation of the same stored bits to
 *     about 2e-7 relative with bf16 keys and 2e-5 (6e-5 worst observed) with fp8 keys, the fp8 MFMA's
 *     own accumulation.)
 *   - top-k / candidate limits: k <= 8192, m <= 1024, m * B <= 65536; one sequence's key array
 *     (s_max * d elements) must stay below 2 GiB.
 *   - T <= 4194304 queries per call and n_seq <= 65535 sequences per key array (launch-grid limits;
 *     more queries: split the call); anything beyond returns HISA_ERR_SHAPE before a launch.
 */
#ifndef HISA_H_
#define HISA_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HISA_OK = 0,
  HISA_ERR_NULL = 1,        /* a required pointer is NULL                                        */
  HISA_ERR_SHAPE = 2,       /* H, d, B, m, k, T, s_max outside the supported set                 */
  HISA_ERR_DTYPE = 3,       /* unsupported dtype or dtype combination                            */
  HISA_ERR_INFEASIBLE = 4,  /* m * B < k (Section 4.1, feasibility constraint) or m < 2          */
  HISA_ERR_WORKSPACE = 5,   /* ws is NULL or smaller than the call's minimum                     */
  HISA_ERR_ALIGN = 6,       /* a tensor pointer is not 16-byte aligned                           */
  HISA_ERR_LAUNCH = 7       /* the HIP runtime refused a launch (hipGetLastError was non-zero)   */
} hisa_status;

typedef enum {
  HISA_F32 = 0,
  HISA_BF16 = 1,
  HISA_FP8_E4M3 = 2         /* OCP e4m3fn codes + one fp32 scale per token                       */
} hisa_dtype;

/* Token-level indexing keys k_s (Section 3): n_seq sequences padded to s_max rows each. */
typedef struct {
  const void*    k;         /* [n_seq, s_max, d] of k_dtype (device)                             */
  const float*   k_scale;   /* [n_seq, s_max] fp32, required iff k_dtype == FP8: key = scale*code */
  const int32_t* seq_len;   /* [n_seq] valid keys per sequence (device)                          */
  int32_t        n_seq;
  int32_t        s_max;
  int32_t        d;
  int32_t        k_dtype;   /* hisa_dtype */
} hisa_keys;

/* Indexing queries q_{t,j} and gates w_{t,j} (Section 3) for T packed queries. */
typedef struct {
  const void*    q;         /* [T, H, d] of q_dtype (device)                                     */
  const float*   w;         /* [T, H] fp32 gates, any sign (device)                              */
  const int32_t* q_seq;     /* [T] sequence id of each query, or NULL: all queries in sequence 0 */
  const int32_t* q_pos;     /* [T] position of each query, or NULL: q_pos[t] = q_pos0 + t        */
  const int32_t* q_lo;      /* [T] first visible position of each query, or NULL: 0.  For sequences
                               packed into one key stream without padding (Section 4.1: a block may
                               then straddle two sequences): q_lo[t] = first token of the query's
                               sequence in the stream, q_pos[t] its own position there; the query
                               sees the keys q_lo[t] .. q_pos[t].  Blocks stay multiples of B of the
                               stream and are pooled over everything they hold; the visible blocks
                               are q_lo/B .. q_pos/B, the first and the last of them forced.  (device) */
  int32_t        T;
  int32_t        H;
  int32_t        q_pos0;
  int32_t        q_dtype;   /* hisa_dtype: F32 or BF16 */
} hisa_queries;

/* Operation selector for hisa_workspace_bytes. */
enum { HISA_OP_POOL = 0, HISA_OP_BLOCK_SCORE_TOPK = 1, HISA_OP_TOKEN_REFINE_TOPK = 2,
       HISA_OP_FLAT_TOPK = 3 };

/*
 * Block pooling (Eq. 4; Algorithm 1, pooling loop): pooled[n, b, :] = mean of the keys of block
 * b of sequence n, for b in [blk_begin, blk_end) (blk_end <= s_max / B; pass 0, s_max / B for all).
 * A block holds tokens bB .. min((b+1)B, seq_len[n]) - 1 and is averaged over the tokens present;
 * a block with no token is written as zeros.  Accumulation in fp32, one rounding to pooled_dtype
 * (F32, or BF16 for BF16/FP8 keys).  pooled: [n_seq, s_max / B, d] device, written in the given
 * block range only.  Needs no workspace.
 */
int hisa_pool_blocks(const hisa_keys* keys, int32_t B, int32_t blk_begin, int32_t blk_end,
                     void* pooled, int32_t pooled_dtype, void* stream);

/*
 * The same call with the per-dimension MAXIMUM over the tokens present in a block instead of their
 * mean: Eq. 4 is written for a generic Pool, the paper uses the mean and names max-pooling as a
 * variant to explore.  Everything else as hisa_pool_blocks (a block with no token is zeros); the
 * later stages take either pooled array.  hisa_pool_append maintains the mean only.
 */
int hisa_pool_blocks_max(const hisa_keys* keys, int32_t B, int32_t blk_begin, int32_t blk_end,
                         void* pooled, int32_t pooled_dtype, void* stream);

/*
 * Stage 1 (Eqs. 5-6; Algorithm 1, block-level coarse filter).  For each query, scores the pooled
 * keys of the visible blocks 0 .. b_t (b_t = q_pos / B) and keeps min(m, b_t + 1) blocks: block 0
 * and block b_t always (Section 4.1: first and last block forced, counted inside the budget m),
 * the rest by score.  `keys` supplies shapes and seq_len only (keys->k may be NULL).
 *   pooled       [n_seq, s_max / B, d] of pooled_dtype (device, in)
 *   block_idx    [T, m] int32 (device, out): kept block ids ascending, then -1
 *   block_scores [T, s_max / B] fp32 (device, out) or NULL: J_{t,b} for b <= b_t, -inf beyond
 * Workspace: T * (s_max / B) floats when block_scores is NULL, else none.  (A batch of at most 256
 * queries with bf16 pooled keys and at most 8192 blocks per sequence -- a decode step -- is scored
 * and selected in one launch that keeps the block scores on chip; the workspace must still be
 * passed, and is then left untouched.)
 */
int hisa_block_score_topk(const hisa_queries* queries, const hisa_keys* keys, const void* pooled,
                          int32_t pooled_dtype, int32_t B, int32_t m, int32_t* block_idx,
                          float* block_scores, void* ws, size_t ws_bytes, void* stream);

/*
 * Stage 2 (Eqs. 7-9; Algorithm 1, token-level refinement).  Scores, with Eq. 1, the visible
 * tokens of the kept blocks and selects the k best.
 *   block_idx   [T, m] int32 (device, in): ascending block ids then -1, as Stage 1 writes them
 *   topk_idx    [T, k] int32 (device, out): selected token positions (within the query's
 *               sequence) ascending, then -1
 *   topk_scores [T, k] fp32 (device, out) or NULL: scores aligned with topk_idx (padding: -inf)
 *   cand_scores [T, m * B] fp32 (device, out) or NULL: every candidate score, slot c = kept block
 *               c / B, offset c % B; -inf where masked.  Requesting it selects the two-kernel path.
 * Workspace: none for the fused path (cand_scores NULL, T >= 256, m * B <= 16384), otherwise
 * T * m * B floats unless cand_scores is given.
 */
int hisa_token_refine_topk(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                           const int32_t* block_idx, int32_t k, int32_t* topk_idx,
                           float* topk_scores, float* cand_scores, void* ws, size_t ws_bytes,
                           void* stream);

/*
 * hisa_token_refine_topk for callers that cannot allocate device memory and have no workspace to
 * hand over: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same inputs, outputs and results as hisa_token_refine_topk with cand_scores == NULL; the
 * candidate scores of the two-kernel path (T < 256, or m * B > 16384) go through a static device
 * array of HISA_STATIC_SCRATCH_BYTES inside the library instead of a workspace.  The call
 * allocates and frees nothing and, like every other call, only enqueues kernels on `stream`.
 *   - Limit: T * m * B * 4 <= HISA_STATIC_SCRATCH_BYTES on that path (a decode batch of 512
 *     queries at m * B = 8192); beyond it the call returns HISA_ERR_WORKSPACE and launches nothing.
 *   - Every GPU the process uses holds its own copy of the array until the process ends.  The
 *     first call on a device looks its address up (make that call outside a graph capture).
 *   - All calls on one GPU share the array: calls that may overlap in time (different streams
 *     without an ordering between them) race on it.  Nothing in it has to be cleared between calls:
 *     the scoring kernel rewrites every slot the select reads.
 */
#define HISA_STATIC_SCRATCH_BYTES (16u << 20)
int hisa_token_refine_topk_static(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                                  const int32_t* block_idx, int32_t k, int32_t* topk_idx,
                                  float* topk_scores, void* stream);

/*
 * Flat DSA indexer (Eqs. 1-2): scores every visible key s <= q_pos and selects the k best.
 * Same outputs as Stage 2.  The scores of a chunk of queries go through the workspace (one row of
 * round_up(s_max, 64) floats per query) and are selected row by row; the library loops over
 * chunks sized to the workspace: minimum 8 rows (plus, only for k > 2048 with s_max > 65536,
 * 8 * k bytes per 65536-entry segment and query; hisa_workspace_bytes gives the size to pass).
 */
int dsa_flat_indexer_topk(const hisa_queries* queries, const hisa_keys* keys, int32_t k,
                          int32_t* topk_idx, float* topk_scores, void* ws, size_t ws_bytes,
                          void* stream);

/*
 * Algorithm 1 whole in one launch: Stage 1 (Eqs. 5-6) and Stage 2 (Eqs. 7-9) of each query run
 * back to back in one workgroup, the query is read once, the block scores and the kept block ids
 * never leave the CU.  Same results as hisa_block_score_topk followed by hisa_token_refine_topk.
 * A convenience for callers that want one call and no workspace, NOT the fast path: on MI355X the
 * two calls are quicker at every shape measured (prefill: the separate Stage 1 kernel shares each
 * pooled-key tile between 8 queries or keeps the tiles resident; decode: the two calls spread a
 * query's tiles over many compute units, one workgroup per query cannot), by 1 % (decode batch) to
 * 18 % (1M-context chunk).
 *   pooled     [n_seq, s_max / B, d] BF16 (device, in), as hisa_pool_blocks writes it
 *   block_idx  [T, m] int32 (device, out) or NULL: the kept block ids, ascending then -1
 *   topk_idx / topk_scores: as hisa_token_refine_topk
 * Supported: q BF16, k BF16 or FP8_E4M3, pooled BF16, d == 128, H in {32, 64}, B % 32 == 0,
 * m * B <= 16384, s_max / B <= 8192; anything else returns HISA_ERR_SHAPE / HISA_ERR_DTYPE (use the
 * two calls).  Needs no workspace.
 */
int hisa_indexer_topk(const hisa_queries* queries, const hisa_keys* keys, const void* pooled,
                      int32_t pooled_dtype, int32_t B, int32_t m, int32_t k, int32_t* block_idx,
                      int32_t* topk_idx, float* topk_scores, void* stream);

/*
 * Incremental maintenance of the pooled-key cache (Section 4.1, block pooling: the pooled keys are
 * a cache kept up to date next to the KV cache; Section 4.2 assumes it).  After sequence n grew
 * from prev_len[n] to keys->seq_len[n] tokens (appended at the end), recomputes exactly the pooled
 * keys of the blocks that received tokens: blocks prev_len[n] / B .. (seq_len[n] - 1) / B.  The
 * result is bit-identical to hisa_pool_blocks over the whole sequence.
 *   prev_len       [n_seq] int32 (device): lengths at the previous update (0 for a new sequence)
 *   max_new_tokens host bound on seq_len[n] - prev_len[n] over all sequences (sizes the launch);
 *                  growth beyond it is NOT pooled
 *   pooled         [n_seq, s_max / B, d] (device, in/out)
 */
int hisa_pool_append(const hisa_keys* keys, int32_t B, const int32_t* prev_len, int32_t max_new_tokens,
                     void* pooled, int32_t pooled_dtype, void* stream);

/*
 * Block-Sparse baseline of the paper's evaluation (Section 5: Stage 1 only, every token of the kept
 * blocks is attended): expands block_idx into token positions.
 *   tokens [T, m * B] int32 (device, out): slot c = block_idx[t, c / B] * B + c % B if that token
 *   is visible to the query (<= q_pos), else -1.  With block_idx as Stage 1 writes it (ascending,
 *   own block last) the valid entries are ascending and the -1 entries form the tail.
 */
int hisa_block_sparse_tokens(const hisa_queries* queries, const hisa_keys* keys, int32_t B, int32_t m,
                             const int32_t* block_idx, int32_t* tokens, void* stream);

/*
 * Selection-consistency diagnostic (Eq. 12): iou[t] = |A_t & B_t| / |A_t | B_t| for two index
 * tensors [T, k] whose rows are ascending with -1 padding at the end (as this library writes
 * them); two empty rows give 1.  iou: [T] fp32 (device, out).
 */
int hisa_index_iou(const int32_t* a_idx, const int32_t* b_idx, int32_t T, int32_t k, float* iou,
                   void* stream);

/*
 * Attainable-peak probes for benchmarks (measurement aids; nothing of the paper's method).
 * hisa_probe_copy: one streaming device-to-device copy of `bytes` (a multiple of 16; both pointers
 * device, 16-byte aligned) with a 4096-workgroup grid: bytes read + bytes written over its time is
 * the HBM rate this chip sustains.  hisa_probe_mfma: 512 workgroups of 4 waves each issue
 * iters * 16 v_mfma_f32_32x32x16_bf16 and nothing else; *flop (host) receives the flop count of the
 * launch, out (device, 512 * 256 floats) receives values that only keep the loop alive.
 * hisa_probe_mfma_fp8: the same with iters * 8 v_mfma_f32_32x32x64_f8f6f4 (e4m3 x e4m3), the
 * instruction the fp8-key scoring runs on.  hisa_probe_mfma_toggling: either loop (fp8 = 0 / 1) on
 * operands that differ per lane and per instruction (pseudo-random signs and mantissas): the rate
 * the matrix cores sustain once their inputs toggle as real data does, which on this chip is below
 * the rate of the two constant-operand probes because the clock drops under that load.
 */
int hisa_probe_copy(const void* src, void* dst, size_t bytes, void* stream);
int hisa_probe_mfma(float* out, int32_t iters, double* flop, void* stream);
int hisa_probe_mfma_fp8(float* out, int32_t iters, double* flop, void* stream);
int hisa_probe_mfma_toggling(float* out, int32_t iters, int32_t fp8, double* flop, void* stream);

/* Recommended workspace size in bytes for `op` (HISA_OP_*) at these shapes; 0 if none is needed
 * or the shapes are invalid.  `want_scores` != 0: the optional full score output of Stage 1 / 2
 * is requested (which then replaces the workspace). */
size_t hisa_workspace_bytes(int op, const hisa_queries* queries, const hisa_keys* keys, int32_t B,
                            int32_t m, int32_t k, int32_t want_scores);

/* Static description of a status code. */
const char* hisa_status_string(int status);

/* Library version, "major.minor". */
const char* hisa_version(void);

#ifdef __cplusplus
}
#endif
#endif /* HISA_H_ */
