// Host-side state and kernel launchers behind the C ABI of the DART drafting step.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/dart.h"
#include "../../include/dart_debug.h"

#define DART_SKINNY_ROWS 16   // rows one skinny-GEMM pass carries (one MFMA column block)
#define ATTN_KEY_CHUNK 128    // keys one attention workgroup walks (split-KV granularity)

// One weight matrix on the device.  fp32: row-major [N][Kd].  bf16: re-tiled for
// v_mfma_f32_16x16x32_bf16 (see pack_bf16_tiles in dart_api.hip): tile (strip s of 16
// output rows, k-step t of 32 inputs) is 1 KiB at ((s * Kd/32) + t) * 1024, and inside a
// tile lane l owns the 8 consecutive inputs 8*(l/16).. of output row l%16.
struct DeviceMatrix {
  void *data = nullptr;
  void *data16 = nullptr;   // bf16 matrices used by the multi-row path: fp16 copy of the tiles
  int N = 0;        // output features (padded to a multiple of 16 for bf16)
  int Kd = 0;       // input features
  int n_real = 0;   // unpadded output features
};

// One open-addressing slot: packed context (~0 when empty) and the row it maps to, 16 bytes so
// that a probe is a single memory access.
struct NgramSlot {
  uint64_t key;
  int32_t row;
  int32_t pad;
};

struct NgramTableDev {
  int n_gram;
  int S;                      // successors per row
  uint64_t slot_mask;         // n_slots - 1 (power of two)
  const NgramSlot *slots;
  const int32_t *succ_ids;    // [n_keys][S], -1 = unused
  const float *succ_logp;     // [n_keys][S]
  float logp_miss;
  // optional back-off table of order n_gram - 1 (same S; scores already carry the discount):
  // consulted with the context's newest n_gram - 2 tokens when the full context has no row.
  // Rows found there are reported with NGRAM_BACKOFF_ROW set.
  const NgramSlot *bo_slots;  // null = no back-off
  uint64_t bo_slot_mask;
  const int32_t *bo_succ_ids;
  const float *bo_succ_logp;
};
#define NGRAM_BACKOFF_ROW (1 << 30)   // row indices are < 2^30

struct dart_ngram {
  NgramTableDev dev;
  float eps = 0.f;
  void *slots = nullptr, *succ_ids = nullptr, *succ_logp = nullptr;
  void *bo_slots = nullptr, *bo_succ_ids = nullptr, *bo_succ_logp = nullptr;
};

struct PruneLevelWeights {
  float w_logit[DART_MAX_K];
  float w_level[DART_MAX_K];
};

// One pass of the layer over rows of up to DART_SEQ_GROUP sequences, passed to kernels by
// value.  The pass's rows are the concatenation, sequence after sequence, of positions
// [pos0[b], pos0[b] + rows_b); row_off[b] is the first row of sequence b (row_off[B] = total).
// The last K rows of every sequence are its query rows (K = 0: a K/V-only pass); query row j
// of sequence b has the compact index b*K + j in the q / residual / output buffers.
#define DART_SEQ_GROUP 16
struct SeqBatch {
  int B, K;
  const void *hidden[DART_SEQ_GROUP];   // [n][d] prefix representation of the sequence (front end:
                                        // [n][feat_dim] concatenated target hidden states)
  const int32_t *tokens[DART_SEQ_GROUP];  // front end: [n] token following each position
  int n[DART_SEQ_GROUP];                // prefix length
  int pos0[DART_SEQ_GROUP];             // first position of the sequence's rows in this pass
  int row_off[DART_SEQ_GROUP + 1];
  int slot[DART_SEQ_GROUP];             // K/V buffer slot
};

// Sequence b, position pos and query index qi (< 0 for a non-query row) of pass row r.
__host__ __device__ inline void seq_of_row(const SeqBatch &sb, int r, int &b, int &pos, int &qi) {
  b = 0;
  while (b + 1 < sb.B && r >= sb.row_off[b + 1]) ++b;
  const int local = r - sb.row_off[b];
  pos = sb.pos0[b] + local;
  qi = local - (sb.row_off[b + 1] - sb.row_off[b] - sb.K);
}

// Where key position pos sits in a row of the transposed V buffer: within every block of 32
// keys, key x is stored at 8*((x%16)/4) + 4*(x/16) + x%4, so that the 8 keys a lane of the
// P.V product contracts over (4*gq..+3 and 16+4*gq..+3, the layout the score product leaves
// the probabilities in) are 16 contiguous bytes.
__host__ __device__ inline int attn_vt_position(int pos) {
  const int x = pos & 31;
  return (pos & ~31) | (8 * ((x & 15) >> 2) + 4 * (x >> 4) + (x & 3));
}

// bf16 configuration: K and V^T of one (sequence, head) are stored chunk by chunk
// (ATTN_KEY_CHUNK keys) as the 1 KiB MFMA operand tiles the attention kernel copies to LDS, so
// that a tile copy reads 1 KiB of contiguous memory and a chunk is one contiguous block.
// K tile (kt, ks) of a chunk, tile index kt*(hd/32)+ks: 16 keys x 32 dims; lane (gq, col) holds
// dims 32ks+8gq..+7 of key 16kt+col.
__host__ __device__ inline size_t attn_k_index(int pos, int dim, int hd) {
  const int p = pos % ATTN_KEY_CHUNK;
  const int tile = (p / 16) * (hd / 32) + dim / 32;
  const int lane = ((dim % 32) / 8) * 16 + p % 16;
  return (size_t)(pos / ATTN_KEY_CHUNK) * ATTN_KEY_CHUNK * hd + ((size_t)tile * 64 + lane) * 8 + dim % 8;
}
// V^T tile (dt, blk), tile index dt*(ATTN_KEY_CHUNK/32)+blk: 16 dims x 32 keys; lane (gq, col)
// holds the keys stored at places 8gq..+7 of the block (attn_vt_position) for dim 16dt+col.
__host__ __device__ inline size_t attn_vt_index(int pos, int dim, int hd) {
  const int x = attn_vt_position(pos) & 31;
  const int tile = (dim / 16) * (ATTN_KEY_CHUNK / 32) + (pos % ATTN_KEY_CHUNK) / 32;
  const int lane = (x / 8) * 16 + dim % 16;
  return (size_t)(pos / ATTN_KEY_CHUNK) * ATTN_KEY_CHUNK * hd + ((size_t)tile * 64 + lane) * 8 + x % 8;
}

// Unit list of an attention launch (bf16 path).  A unit is one (sequence, K/V head, key chunk);
// units are numbered sequence-major, then head, then chunk: sequence b has cum[b+1] - cum[b]
// chunks per head and its units start at cum[b] * Hkv.  Workgroup w takes units
// [w * per, (w+1) * per); the partial it writes for a (sequence, head) pair is numbered
// w - (first unit of the pair) / per.
struct AttnWork {
  int cum[DART_SEQ_GROUP + 1];
  int per;
};

struct dart_ctx {
  dart_config cfg;
  int q_dim, kv_dim, qkv_dim;
  int t_cap;                     // K/V rows per (sequence, head): max_ctx + max_K - 1, padded to whole 128-key chunks
  // weights
  DeviceMatrix wqkv, wo, wgu, wdown, wlm;   // wgu: gate and up rows interleaved (see dart_api.hip)
  void *g_in = nullptr, *g_post = nullptr, *g_final = nullptr, *g_q = nullptr, *g_k = nullptr;
  void *mask_emb = nullptr;
  // front end (cfg.front_end): FC layer, frozen embedding table, gain of the embedding half;
  // in_dim = width of the layer's attention input (d, or 2d with the front end)
  int in_dim = 0;
  DeviceMatrix wfc;
  void *embed = nullptr, *g_emb = nullptr;
  float *feat32 = nullptr;        // [max(ws_rows, kv_rows)][feat_dim] features of a pass as fp32
  float *fc_part = nullptr;       // [chunks][max(ws_rows, kv_rows)][d] FC partial sums
  int split_fc = 1, gch_fc = 1, fc_rows = 0;
  float *rope_cos = nullptr, *rope_sin = nullptr;   // [t_cap][hd/2]
  // draft K/V buffers [batch][Hkv][t_cap * hd]: fp32 rows [t_cap][hd]; bf16 operand tiles (attn_k_index, attn_vt_index)
  void *kbuf = nullptr, *vbuf = nullptr;
  int *cached_rows = nullptr;     // host, [max_batch]
  // activations / workspaces (device, fp32 unless noted); ws_rows = rows one pass may carry
  int ws_rows = 16;
  float *xn = nullptr;            // [ws_rows][d] normed layer input
  float *resid = nullptr;         // [ws_rows][d] raw input rows of the query positions
  float *qkv = nullptr;           // [chunks][ws_rows][qkv_dim]
  void *qrot = nullptr;           // [ws_rows][q_dim] queries after norm + rotary (fp32 or fp16)
  float *att_part = nullptr;      // [ws_rows*Hq][splits][hd]
  float *att_ml = nullptr;        // [ws_rows*Hq][splits][2]
  float *att_out = nullptr;       // [ws_rows][q_dim]
  float *proj = nullptr;          // projection partial sums, [chunks][ws_rows][N] of the largest
  float *y = nullptr, *yn = nullptr, *hmid = nullptr, *u = nullptr;
  // LM head of the single-sequence calls when d is too long for one k-chunk of the skinny
  // kernel: chunk partials [split_lm][16][lm_stride], summed into the caller's logits
  int split_lm = 1;
  size_t lm_stride = 0;
  float *lm_part = nullptr;
  // K/V-only passes (prefix rows that are not query rows): up to kv_rows rows per pass
  int kv_rows = 16;
  bool kv_ordered = false;        // single-sequence K/V-only passes of many rows run on gemm_ordered_kernel
  float *xn_kv = nullptr;         // [kv_rows][d]
  float *kv_part = nullptr;       // [chunks][kv_rows][2*kv_dim]
  int split_qkv = 1, split_o = 1, split_gu = 1, split_down = 1;   // k-chunks per matrix (skinny kernel)
  int gch_qkv = 1, gch_o = 1, gch_gu = 1, gch_down = 1;           // k-chunks on the multi-row path
  void *xpack = nullptr;          // activations of one multi-row projection in MFMA operand order
  void *xpack2 = nullptr;         // ... of the down projection, written by the gate/up epilogue
  int max_rows;                   // max_batch * max_K
  int max_splits;                 // key splits the attention workspaces hold per query vector
  // top-k workspace
  uint64_t *topk_cand = nullptr;  // [rows][chunks][DART_MAX_TOPK]
  float *topk_ms = nullptr;       // [rows][chunks][2]
  int topk_chunks_max;
  int lm_select_wgs = 0;          // workgroups of the LM-head launch that selects its own candidates (0 = cannot)
  float *logits_tmp = nullptr;    // [max_K][vocab]: dart_draft_forward_topk without a logits buffer, unfused
};

namespace dart {

// Hash of a packed N-gram context; the host-side table build and the device probe share it.
__host__ __device__ inline uint64_t mix64(uint64_t x) {
  x ^= x >> 33;
  x *= 0xff51afd7ed558ccdULL;
  x ^= x >> 33;
  x *= 0xc4ceb9fe1a85ec53ULL;
  x ^= x >> 33;
  return x;
}

// Launch tunables: constants fixed after measurement.  Only a build with -DDART_TUNING (sweeps
// on a developer's box) makes them variables and exports dart_debug_set to change them; the
// product library has no mutable process-wide state on the hot path.
#ifdef DART_TUNING
#define DART_TUNABLE
#else
#define DART_TUNABLE const
#endif
extern DART_TUNABLE int g_gemm_ord_map, g_gemv_xcd, g_gemv_wgs_split, g_gemv_wgs, g_gemv_depth, g_gemv_nt, g_gemv_nt_min_mb, g_gemv_split, g_gemm_wgs, g_attn_seg;

// Raise a kernel's dynamic-LDS limit: a per-device property of the function, set the first time
// the function is launched on each device (thread-safe; a race only repeats the idempotent call).
hipError_t raise_dynamic_lds_once(const void *func, int bytes);

// All launchers only enqueue work on `st` and return the launch status.

// pack != null (bf16): the normed rows go to the packed operand tiles of a multi-row projection
// (launch_gemm_bf16 with X = null consumes them) instead of xn.
hipError_t launch_rmsnorm_gather(int dtype, const SeqBatch &sb, const void *mask_emb,
                                 const void *gain, int d, float eps, float *xn, float *resid,
                                 void *pack, int terms, hipStream_t st);

hipError_t launch_norm_pack_rows(const SeqBatch &sb, const void *mask_emb, const void *gain, int d,
                                 float eps, float *rstd, void *pack, hipStream_t st);

// Front end, step 1: the feature rows of a pass as fp32 (mask rows: zeros).
hipError_t launch_feature_rows(int dtype, const SeqBatch &sb, int feat_dim, float *out, hipStream_t st);
// Front end, step 2: per pass row, g = sum of the FC partials (prefix rows) and e = embedding
// of the row's next token, or the two halves of a mask slot; xn[r] = [RMSNorm(g) * gain_g ;
// RMSNorm(e) * gain_e] (2d wide), resid (query rows) = g.
hipError_t launch_front_norm(int dtype, const SeqBatch &sb, const float *fc_part, int chunks,
                             size_t chunk_stride, const void *embed, const void *mask_emb,
                             const void *gain_g, const void *gain_e, int d, float eps, float *xn,
                             float *resid, hipStream_t st);

// pack != null (bf16): yn is also written as the packed operand tiles of a multi-row projection
// of `rows` rows (launch_gemm_bf16 with X = null consumes them).
hipError_t launch_resid_norm(int dtype, const float *resid, const float *part, int chunks,
                             size_t chunk_stride, int row_stride, const void *gain, int rows, int d,
                             float eps, float *y, float *yn, void *pack, int terms, hipStream_t st);

hipError_t launch_gemv_f32(const DeviceMatrix &W, int row0, int nrows, const float *X, int M,
                           float *out, int out_stride, hipStream_t st);

// Candidate output of the skinny kernel when it selects its workgroups' top-k itself (the LM
// head with at most 8 rows): per (row, workgroup) k ordering keys and (max, sum exp), in the
// layout topk_merge_kernel reads with "chunks" = workgroups of the launch (gemv_bf16_select_wgs).
struct GemvTopk {
  uint64_t *cand;      // [row][workgroup][DART_MAX_TOPK] ordering keys, 0 = none
  float *ms;           // [row][workgroup][2]
  int k;
};

// bf16 skinny GEMM on packed weights; returns the number of k-chunks written through *chunks.
// tk != null: also write the workgroups' candidates; out may then be null.
hipError_t launch_gemv_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            float *out, int out_stride, size_t chunk_stride, int split, int *chunks,
                            hipStream_t st, const GemvTopk *tk = nullptr);
int gemv_bf16_select_wgs(const DeviceMatrix &W, int nstrips, int M);
int gemv_bf16_describe(const DeviceMatrix &W, int nstrips, int M, int nch, char *buf, int len,
                       bool topk = false);
int gemm_bf16_describe(const DeviceMatrix &W, int nstrips, int M, int nchunks, int epi, char *buf,
                       int len);
int gemv_bf16_chunks(int Kd);                 // k-chunks forced by the register budget
int gemv_bf16_split(int Kd, int nstrips);     // k-chunks that balance the workgroups (>= gemv_bf16_chunks)
int gemv_bf16_row_tiles(int Kd, int nch);     // 16-row tiles one launch may carry per row block

// bf16 multi-row GEMM on packed weights (any M); nchunks is fixed per matrix, see gemm_bf16_chunks.
// epi 1: the strips are interleaved gate/up rows and out receives silu(gate) * up, [M][out_stride].
// pack: scratch of gemm_bf16_pack_bytes(M, W.Kd) bytes for the activations in operand order
// (X == nullptr: pack already holds the operand tiles of these M rows; no conversion pass).
hipError_t launch_gemm_bf16(const DeviceMatrix &W, int strip0, int nstrips, const float *X, int M,
                            void *pack, float *out, int out_stride, size_t chunk_stride, int nchunks,
                            int epi, hipStream_t st,
                            void *out_pack = nullptr);
int gemm_bf16_chunks(int Kd, int nstrips);
hipError_t launch_pack_rows(const float *X, int M, int Kd, int terms, void *pack, hipStream_t st);
// Many rows with the skinny kernel's sums, bit for bit (the K/V build of a long prefix).
bool gemm_ordered_supported(const DeviceMatrix &W, int nch);
hipError_t launch_gemm_ordered(const DeviceMatrix &W, int strip0, int nstrips, int M, const void *pack,
                               float *out, int out_stride, int nch, hipStream_t st);
size_t gemm_bf16_pack_bytes(int M, int Kd);
int gemm_bf16_terms(const DeviceMatrix &W);   // format of the packed activations W's launches expect
hipError_t launch_tiles_to_f16(const void *src, void *dst, size_t n_elems, hipStream_t st);

// First k-step of k-chunk c when KT k-steps are cut into nchunks (multiples of 4 k-steps).
__host__ __device__ inline int gemm_chunk_begin(int KT, int nchunks, int c) {
  return c >= nchunks ? KT : (int)((int64_t)KT * c / nchunks) / 4 * 4;
}

hipError_t launch_sum_chunks(const float *part, int chunks, size_t chunk_stride, int row_stride,
                             int rows, int n, float *out, int out_stride, hipStream_t st);

hipError_t launch_swiglu(const float *gu, int chunks, size_t chunk_stride, int rows, int ffn,
                         int interleaved, float *h, hipStream_t st);

// qkv: [chunks][rows][row_stride] projection partials whose column 0 is column col0 of [q | k | v].
hipError_t launch_qkv_post(const dart_ctx *c, const SeqBatch &sb, const float *qkv, int chunks,
                           size_t chunk_stride, int row_stride, int col0, hipStream_t st);

// Attention of the B*K query rows of the pass (compact order) over their sequences' K/V.
hipError_t launch_attention(const dart_ctx *c, const SeqBatch &sb, void *pack, int terms, hipStream_t st);

int topk_chunks(int vocab);                   // vocabulary chunks of the top-k kernels
hipError_t launch_topk_merge(const uint64_t *cand, const float *ms, int rows, int k, int nlists, float eps,
                             int32_t *ids, float *scores, hipStream_t st);
hipError_t launch_topk(const dart_ctx *c, const float *logits, int rows, int vocab, int k, float eps,
                       int32_t *ids, float *scores, hipStream_t st);

hipError_t launch_tree_verify(int batch, const int32_t *tokens, const int32_t *parents,
                              const int32_t *n_nodes, const int32_t *target_next,
                              const int32_t *ctx_len, int budget, int path_cap,
                              int32_t *position_ids, int32_t *accept_path, int32_t *n_accepted,
                              int32_t *next_token, hipStream_t st);

hipError_t launch_prune(int batch, const int32_t *ids, const float *scores, int K,
                        const int32_t *ctx_tail, const NgramTableDev &tab,
                        const dart_prune_params &p, const PruneLevelWeights &lw, int32_t *tokens,
                        int32_t *parents, uint8_t *mask, int32_t *n_nodes, hipStream_t st);

}  // namespace dart
