// Per-position candidate extraction (paper Alg. 1 "Top-k_i tokens from l_i" and
// s_logit = log(softmax(l)_{i,t} + eps), App. D): one read of each logit row yields the
// k best tokens and the row's log-sum-exp together.
//
// Chunk kernel, grid: vocab chunks x rows.  A workgroup holds a 4096-logit chunk in registers,
// 1024 per wavefront.  Each wavefront computes its (max, sum exp) and selects its k largest
// entries; wavefront 0 then reduces the 4 x k winners to the chunk's k, combines the four
// statistics and writes both, while the other wavefronts have already left and made room for
// the next workgroup's loads.  Merge kernel, one wavefront per row: the chunk statistics give
// the row's log-sum-exp (fixed order) and the k largest of the chunk winners are the row's.
// A fused form (the workgroup that completes a row merges it, found through a device-scope
// counter) was slower at every row count: the wait for the stores and the counter sits inside
// every workgroup, and the merge's 40 keys per lane set the register count of the whole kernel
// (96 against 48, five wavefronts per SIMD against eight).
//
// Selection inside a wavefront (wave_select): the k-th largest of the 64 lane maxima is a
// lower bound T of the k-th largest value, found (to 16 bits) by a bitwise search with ballots;
// the entries >= T (at least k, in practice few more) are compacted into LDS and ranked by
// counting.  This replaces k dependent wavefront-wide max reductions by a handful of
// independent steps.  If ties make the candidate set overflow its LDS buffer the code falls
// back to the k sequential extractions.
// Ordering key: (logit descending, token id ascending), as one 64-bit integer
// (order-preserving float map << 32 | ~id), unique per entry, so the result is deterministic.
#include <mutex>

#include "common.h"
#include "dart_internal.h"
#include "topk_select.h"

namespace dart {

constexpr int TOPK_THREADS = 256;
constexpr int TOPK_WAVES = TOPK_THREADS / 64;
constexpr int TOPK_PER_THREAD = 16;
constexpr int TOPK_CHUNK = TOPK_THREADS * TOPK_PER_THREAD;   // 4096
constexpr int TOPK_MERGE_REGS = 40;                          // candidates per lane in the merge

// The row's log-sum-exp from the chunk statistics (fixed order) and the k best of the chunk
// winners, by one wavefront.
__device__ __forceinline__ void merge_row(int row, int k, int nchunks, float eps, const uint64_t *cand,
                                          const float *ms, uint64_t *buf, int32_t *__restrict__ ids,
                                          float *__restrict__ scores) {
  const int lane = threadIdx.x & 63;
  const uint64_t *csrc = cand + (size_t)row * nchunks * DART_MAX_TOPK;
  // Candidates first (the longest wait): winner j of the row's nchunks * k, lane by lane, so that
  // every lane holds a mixed handful (the selection's threshold is the k-th largest lane
  // maximum).  j / k by a multiplication: floor(j * ceil(2^32 / k) / 2^32) is exact while
  // j * (k - 1) < 2^32.
  const int total = nchunks * k;
  const bool in_regs = total <= 64 * TOPK_MERGE_REGS;
  uint64_t mine[TOPK_MERGE_REGS];
  if (in_regs) {
    const uint32_t inv_k = (uint32_t)((((uint64_t)1 << 32) + k - 1) / k);
#pragma unroll
    for (int e = 0; e < TOPK_MERGE_REGS; ++e) {
      const int j = e * 64 + lane;
      const int c = k == 1 ? j : (int)__umulhi((uint32_t)j, inv_k);
      mine[e] = j < total ? csrc[(size_t)c * DART_MAX_TOPK + (j - c * k)] : 0;
    }
  }
  // chunk statistics: read once (one chunk per lane up to 64 chunks), combined in lane order
  const float2 *ms2 = reinterpret_cast<const float2 *>(ms) + (size_t)row * nchunks;
  float rmx = -3.0e38f;
  float2 own = make_float2(-3.0e38f, 0.f);
  if (lane < nchunks) own = ms2[lane];
  rmx = own.x;
  for (int c = lane + 64; c < nchunks; c += 64) rmx = fmaxf(rmx, ms2[c].x);
  rmx = wave_max_dpp(rmx);
  float rse = lane < nchunks ? own.y * expf(own.x - rmx) : 0.f;
  for (int c = lane + 64; c < nchunks; c += 64) rse += ms2[c].y * expf(ms2[c].x - rmx);
  rse = wave_sum_dpp(rse);
  const float lse = rmx + logf(rse);
  auto emit = [&](int it, uint64_t best) {
    const float logit = f32_unsortable((uint32_t)(best >> 32));
    ids[(size_t)row * k + it] = (int32_t)(~(uint32_t)best);
    scores[(size_t)row * k + it] = fminf(0.f, logf(expf(logit - lse) + eps));
  };
  if (in_regs) {
    wave_select(mine, k, buf, emit);
  } else {                                          // very large vocab x k: re-read from memory
    uint64_t bound = ~(uint64_t)0;
    for (int it = 0; it < k; ++it) {
      uint64_t best = 0;
      for (int j = lane; j < total; j += 64) {
        const uint64_t kk = csrc[(size_t)(j / k) * DART_MAX_TOPK + j % k];
        if (kk < bound && kk > best) best = kk;
      }
      best = wave_max_u64(best);
      if (lane == 0) emit(it, best);
      bound = best;
    }
  }
}

__global__ __launch_bounds__(TOPK_THREADS) void topk_kernel(
    const float *__restrict__ logits, int vocab, int k, int nchunks,
    uint64_t *__restrict__ cand, float *__restrict__ ms) {
  __shared__ uint64_t wcand[TOPK_WAVES][DART_MAX_TOPK];
  __shared__ uint64_t sel[TOPK_WAVES][TOPK_CAP];
  __shared__ float wms[TOPK_WAVES][2];
  const int chunk = blockIdx.x, row = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const float *src = logits + (size_t)row * vocab;
  const int idx0 = chunk * TOPK_CHUNK + wave * (TOPK_CHUNK / TOPK_WAVES) + lane;
  // entries of this lane inside the row: indices idx0 + 64 e < vocab
  const int ne = idx0 < vocab ? min(TOPK_PER_THREAD, (vocab - idx0 + 63) >> 6) : 0;
  float val[TOPK_PER_THREAD];
  float mx = -3.0e38f;
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e) {
    val[e] = e < ne ? src[idx0 + e * 64] : -3.0e38f;
    mx = fmaxf(mx, val[e]);
  }
  mx = wave_max_dpp(mx);
  float se = 0.f;
  uint32_t v[TOPK_PER_THREAD];
#pragma unroll
  for (int e = 0; e < TOPK_PER_THREAD; ++e) {
    if (e < ne) se += __expf(val[e] - mx);      // 2 instructions; relative error 2^-21, far inside the score tolerance
    v[e] = f32_sortable(val[e]);
  }
  se = wave_sum_dpp(se);
  if (lane == 0) {
    wms[wave][0] = mx;
    wms[wave][1] = se;
  }
  wave_select_row(v, ne, idx0, k, sel[wave], [&](int r, uint64_t best) { wcand[wave][r] = best; });
  __syncthreads();
  // Wavefront 0 finishes the chunk alone; the others leave now.
  if (wave != 0) return;
  const size_t slot = (size_t)row * nchunks + chunk;
  // chunk statistics in wavefront order (deterministic), then the chunk's k best of 4 x k
  float cm = wms[0][0];
#pragma unroll
  for (int w = 1; w < TOPK_WAVES; ++w) cm = fmaxf(cm, wms[w][0]);
  float cs = 0.f;
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) cs += wms[w][1] * expf(wms[w][0] - cm);
  uint64_t mine[TOPK_WAVES];
#pragma unroll
  for (int w = 0; w < TOPK_WAVES; ++w) mine[w] = lane < k ? wcand[w][lane] : 0;
  if (lane == 0) {
    ms[slot * 2] = cm;
    ms[slot * 2 + 1] = cs;
  }
  wave_select(mine, k, sel[0], [&](int r, uint64_t best) {
    cand[slot * DART_MAX_TOPK + r] = best;                  // 0 when the chunk ran out
  });
}

// grid = rows, one wavefront each
__global__ __launch_bounds__(64) void topk_merge_kernel(int k, int nchunks, float eps, const uint64_t *cand,
                                                        const float *ms, int32_t *__restrict__ ids,
                                                        float *__restrict__ scores) {
  __shared__ uint64_t buf[TOPK_CAP];
  merge_row(blockIdx.x, k, nchunks, eps, cand, ms, buf, ids, scores);
}

int topk_chunks(int vocab) { return (vocab + TOPK_CHUNK - 1) / TOPK_CHUNK; }

// cand: [rows][chunks][DART_MAX_TOPK] keys, ms: [rows][chunks][2] floats of workspace.
static hipError_t launch_topk_on(uint64_t *cand, float *ms, const float *logits, int rows, int vocab,
                                 int k, float eps, int32_t *ids, float *scores, hipStream_t st) {
  const int nchunks = (vocab + TOPK_CHUNK - 1) / TOPK_CHUNK;
  hipLaunchKernelGGL(topk_kernel, dim3(nchunks, rows), dim3(TOPK_THREADS), 0, st, logits, vocab, k,
                     nchunks, cand, ms);
  hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(64), 0, st, k, nchunks, eps, cand, ms, ids,
                     scores);
  return hipGetLastError();
}

// Row merge alone, on lists some other kernel wrote in the chunk kernel's layout (the LM head
// that selects its workgroups' candidates itself): nlists lists per row.
hipError_t launch_topk_merge(const uint64_t *cand, const float *ms, int rows, int k, int nlists, float eps,
                             int32_t *ids, float *scores, hipStream_t st) {
  hipLaunchKernelGGL(topk_merge_kernel, dim3(rows), dim3(64), 0, st, k, nlists, eps, cand, ms, ids, scores);
  return hipGetLastError();
}

hipError_t launch_topk(const dart_ctx *c, const float *logits, int rows, int vocab, int k, float eps,
                       int32_t *ids, float *scores, hipStream_t st) {
  return launch_topk_on(c->topk_cand, c->topk_ms, logits, rows, vocab, k, eps, ids, scores, st);
}

}  // namespace dart

// ---- dart_topk_static: the same two kernels on a workspace that is part of the library image ----
//
// Workspace of the chunk kernel for up to DART_TOPK_STATIC_CELLS (row, vocabulary chunk) pairs:
// the chunk winners, then the chunk statistics.  One copy per GPU, held until the process ends.
namespace {

constexpr size_t STATIC_CAND_BYTES = (size_t)DART_TOPK_STATIC_CELLS * DART_MAX_TOPK * sizeof(uint64_t);
constexpr size_t STATIC_MS_BYTES = (size_t)DART_TOPK_STATIC_CELLS * 2 * sizeof(float);
static __device__ __align__(256) unsigned char scratch[STATIC_CAND_BYTES + STATIC_MS_BYTES];

// Device address of `scratch` on each GPU (the array's name is only a host-side handle; every
// device holds its own copy at its own address), resolved on the first call per device.
constexpr int STATIC_MAX_DEVICES = 64;
void *g_scratch_ptr[STATIC_MAX_DEVICES];
std::mutex g_scratch_lock;

hipError_t scratch_on_current_device(void **out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= STATIC_MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> hold(g_scratch_lock);
  if (!g_scratch_ptr[dev]) {
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!p) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = p;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

}  // namespace

extern "C" dart_status dart_topk_static(const float *logits, int rows, int vocab, int k, float eps,
                                        int32_t *ids_out, float *scores_out, void *stream) {
  if (!logits || !ids_out || !scores_out) return DART_ERR_ARG;
  if (rows < 1 || vocab < 1 || k < 1 || k > DART_MAX_TOPK || k > vocab) return DART_ERR_ARG;
  const int64_t cells = (int64_t)rows * dart::topk_chunks(vocab);
  if (cells > DART_TOPK_STATIC_CELLS) return DART_ERR_SHAPE;
  void *base = nullptr;
  if (scratch_on_current_device(&base) != hipSuccess) {
    (void)hipGetLastError();
    return DART_ERR_HIP;
  }
  // The chunk kernel writes every cell the merge kernel reads (all k winner slots and both
  // statistics of every (row, chunk) pair of this call), so nothing of an earlier call's
  // contents is read and nothing needs clearing.
  uint64_t *cand = reinterpret_cast<uint64_t *>(base);
  float *ms = reinterpret_cast<float *>(static_cast<unsigned char *>(base) + STATIC_CAND_BYTES);
  hipError_t e = dart::launch_topk_on(cand, ms, logits, rows, vocab, k, eps, ids_out, scores_out,
                                      (hipStream_t)stream);
  return e == hipSuccess ? DART_OK : DART_ERR_HIP;
}
