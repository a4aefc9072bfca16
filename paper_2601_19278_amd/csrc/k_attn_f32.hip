// Masked-position attention of the draft layer, fp32 storage (small parity configuration),
// and the split-merge kernel shared with the bf16 path.
//
// Query row i (0-based among the K read-out rows) sits at position n-1+i and sees keys
// 0..n-1+i: the whole prefix plus the mask rows up to itself -- the strictly causal mask
// of paper Sec. 3.1 restricted to one prefix (mask listing of App. B).
#include "common.h"
#include "dart_internal.h"

namespace dart {

// One wavefront per (key split, query vector).  Lane owns dims lane, lane+64.
// Query vector qv = (b*K + i)*Hq + h: query row i of sequence b (SeqBatch), head h.
// Partial result: unnormalised sum_j exp(s_j - m) v_j, with m and l = sum_j exp(s_j - m).
template <int HD>
__global__ __launch_bounds__(64) void attn_split_f32_kernel(
    SeqBatch sb, const float *__restrict__ q, const float *__restrict__ kbuf,
    const float *__restrict__ vbuf, size_t slot_elems, int t_cap, int Hq, int group, int chunk,
    float scale, int nsplit, float *__restrict__ o_part, float *__restrict__ ml_part) {
  constexpr int PER = HD / 64;
  const int split = blockIdx.x, qv = blockIdx.y, lane = threadIdx.x;
  const int row = qv / Hq, h = qv % Hq, g = h / group;
  const int b = row / sb.K, i = row % sb.K;
  const int last = sb.n[b] - 1 + i;                    // last visible key
  const int j0 = split * chunk;
  if (j0 >= sb.n[b] + sb.K - 1) return;                // beyond the sequence: the merge never reads it
  const int j1 = min(j0 + chunk, last + 1);
  float qr[PER], acc[PER];
#pragma unroll
  for (int p = 0; p < PER; ++p) {
    qr[p] = q[(size_t)qv * HD + lane + 64 * p];
    acc[p] = 0.f;
  }
  float m = -3.0e38f, l = 0.f;
  const float *kb = kbuf + sb.slot[b] * slot_elems + (size_t)g * t_cap * HD;
  const float *vb = vbuf + sb.slot[b] * slot_elems + (size_t)g * t_cap * HD;
  for (int j = j0; j < j1; ++j) {
    float s = 0.f;
#pragma unroll
    for (int p = 0; p < PER; ++p) s += qr[p] * kb[(size_t)j * HD + lane + 64 * p];
    s = wave_sum(s) * scale;
    const float mn = fmaxf(m, s);
    const float corr = expf(m - mn), pj = expf(s - mn);
    l = l * corr + pj;
#pragma unroll
    for (int p = 0; p < PER; ++p) acc[p] = acc[p] * corr + pj * vb[(size_t)j * HD + lane + 64 * p];
    m = mn;
  }
  const size_t slot = (size_t)qv * nsplit + split;
#pragma unroll
  for (int p = 0; p < PER; ++p) o_part[slot * HD + lane + 64 * p] = acc[p];
  if (lane == 0) {
    ml_part[slot * 2] = m;
    ml_part[slot * 2 + 1] = l;
  }
}

// out[qv][:] = sum_s e^{m_s - M} o_s / sum_s e^{m_s - M} l_s over the partials of the query's
// (sequence, K/V head) pair: one per workgroup run that holds units of the pair (AttnWork) and
// sub-range, out of the nsplit slots of the query vector.  A partial with l == 0 saw no visible
// key.  One wavefront per query vector (a lane holds output dims l and l + 64), no workgroup
// barrier: the weights are computed once across the lanes and kept in LDS, the reductions run
// on the DPP path, and the partial rows are then read with independent loads.
constexpr int ATTN_MAX_SPLITS = 1024;   // 256 key chunks x 4 sub-ranges

// pack != null: the result goes to the packed operand tiles of the multi-row O projection
// (row = query row, input = head * hd + dim; ntiles row tiles) instead of out.
constexpr int MERGE_VECS = 4;           // query vectors per workgroup, one wavefront each
__global__ __launch_bounds__(64 * MERGE_VECS) void attn_merge_kernel(
    SeqBatch sb, AttnWork work, int Hq, int group, int nsub, const float *__restrict__ o_part,
    const float *__restrict__ ml_part, int nsplit, int hd, int n_vecs, float *__restrict__ out,
    uint4 *__restrict__ pack, int ntiles, int terms) {
  __shared__ float w_all[MERGE_VECS][ATTN_MAX_SPLITS];
  __shared__ __align__(16) float row_all[MERGE_VECS][128];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int qv = blockIdx.x * MERGE_VECS + wave;
  if (qv >= n_vecs) return;                       // wave-uniform; no workgroup barrier below
  float *w = w_all[wave], *row_out = row_all[wave];
  const int b = qv / (Hq * sb.K), g = qv % Hq / group;
  const int cb = work.cum[b + 1] - work.cum[b];
  const int pair0 = work.cum[b] * (Hq / group) + g * cb;        // first unit of the pair
  const int used = ((pair0 + cb - 1) / work.per - pair0 / work.per + 1) * nsub;
  const float2 *ml2 = reinterpret_cast<const float2 *>(ml_part) + (size_t)qv * nsplit;
  // weights of the partials: exp(m_s - max m) over the partials that saw a key (l_s > 0)
  float mx = -3.0e38f;
  for (int s = lane; s < used; s += 64) {
    const float2 ml = ml2[s];
    if (ml.y > 0.f) mx = fmaxf(mx, ml.x);
  }
  mx = wave_max(mx);
  float den = 0.f;
  for (int s = lane; s < used; s += 64) {
    const float2 ml = ml2[s];
    const float ws = ml.y > 0.f ? expf(ml.x - mx) : 0.f;
    w[s] = ws;
    den += ws * ml.y;
  }
  den = wave_sum(den);
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  // lane l adds up elements l and l + 64 of the partial outputs, in index order (deterministic)
  const int t0 = min(lane, hd - 1), t1 = min(lane + 64, hd - 1);
  const float *src = o_part + (size_t)qv * nsplit * hd;
  float n0 = 0.f, n1 = 0.f;
  int s = 0;
  for (; s + 4 <= used; s += 4) {
    float a[4], c[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[i] = src[(size_t)(s + i) * hd + t0];
      c[i] = src[(size_t)(s + i) * hd + t1];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      n0 += w[s + i] * a[i];
      n1 += w[s + i] * c[i];
    }
  }
  for (; s < used; ++s) {
    n0 += w[s] * src[(size_t)s * hd + t0];
    n1 += w[s] * src[(size_t)s * hd + t1];
  }
  if (!pack) {
    if (lane < hd) out[(size_t)qv * hd + lane] = n0 / den;
    if (lane + 64 < hd) out[(size_t)qv * hd + lane + 64] = n1 / den;
    return;
  }
  if (lane < hd) row_out[lane] = n0 / den;
  if (lane + 64 < hd) row_out[lane + 64] = n1 / den;
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
  __builtin_amdgcn_wave_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  if (lane < hd / 8) {
    const int row = qv / Hq, h = qv % Hq;
    pack_store8(pack, ntiles, terms, row, h * hd + 8 * lane, &row_out[8 * lane]);
  }
}

hipError_t launch_attention_bf16(const dart_ctx *c, const SeqBatch &sb, const AttnWork &work,
                                 int nseg, hipStream_t st);

// Chunk units per attention workgroup of the bf16 path; 0 = chosen from the amount of work.
DART_TUNABLE int g_attn_seg = 0;

void gemm_bf16_pack_shape(int M, int Kd, int *ntiles, int *ksteps);

// pack: where the multi-row O projection expects its operand tiles (bf16 only), else null and
// the result goes to c->att_out.
hipError_t launch_attention(const dart_ctx *c, const SeqBatch &sb, void *pack, int terms,
                            hipStream_t st) {
  const dart_config &g = c->cfg;
  const int Hq = g.n_q_heads, Hkv = g.n_kv_heads, hd = g.head_dim;
  const int chunk = ATTN_KEY_CHUNK;                      // keys per chunk
  AttnWork work;
  work.cum[0] = 0;
  work.per = 1;
  int cb_max = 0;
  for (int b = 0; b < sb.B; ++b) {
    const int cb = (sb.n[b] + sb.K - 1 + chunk - 1) / chunk;
    work.cum[b + 1] = work.cum[b] + cb;
    cb_max = max(cb_max, cb);
  }
  const size_t slot_elems = (size_t)Hkv * c->t_cap * hd;
  const int QVT = sb.B * sb.K * Hq;                      // query vectors of the pass
  int nsub = 1, nseg = cb_max;
  if (g.dtype == DART_BF16) {
    // One unit per workgroup while there is at most one per compute unit (lowest latency);
    // beyond that, runs of several units over one double-buffered workgroup per compute unit
    // (128 KiB of LDS at head_dim 128; two fit at head_dim 64), so that copies overlap compute,
    // nothing queues behind a first round, and few partials are written and merged.
    const int units = work.cum[sb.B] * Hkv;
    const int resident = hd == 128 ? 256 : 512;
    work.per = g_attn_seg > 0 ? g_attn_seg : max(1, (units + resident - 1) / resident);
    nseg = (cb_max + work.per - 2) / work.per + 1;        // most runs a pair can touch
    nsub = 1;                                             // sub-ranges are merged in the kernel
    hipError_t e = launch_attention_bf16(c, sb, work, nseg, st);
    if (e != hipSuccess) return e;
  } else {
    const float scale = 1.0f / sqrtf((float)hd);
    dim3 grid(cb_max, QVT);
    if (hd == 64)
      hipLaunchKernelGGL(attn_split_f32_kernel<64>, grid, dim3(64), 0, st, sb,
                         (const float *)c->qrot, (const float *)c->kbuf, (const float *)c->vbuf,
                         slot_elems, c->t_cap, Hq, Hq / Hkv, chunk, scale, cb_max, c->att_part,
                         c->att_ml);
    else
      hipLaunchKernelGGL(attn_split_f32_kernel<128>, grid, dim3(64), 0, st, sb,
                         (const float *)c->qrot, (const float *)c->kbuf, (const float *)c->vbuf,
                         slot_elems, c->t_cap, Hq, Hq / Hkv, chunk, scale, cb_max, c->att_part,
                         c->att_ml);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  int ntiles = 0, ksteps = 0;
  if (pack) {
    // every input of every valid row is written; rows beyond the query rows only feed their own
    // (discarded) outputs.  An odd number of k-steps would need a zeroed extra step.
    gemm_bf16_pack_shape(sb.B * sb.K, Hq * hd, &ntiles, &ksteps);
    if (ksteps * 32 != Hq * hd) return hipErrorInvalidValue;
  }
  hipLaunchKernelGGL(attn_merge_kernel, dim3((QVT + MERGE_VECS - 1) / MERGE_VECS), dim3(64 * MERGE_VECS),
                     0, st, sb, work, Hq, Hq / Hkv, nsub, c->att_part, c->att_ml, nseg * nsub, hd, QVT,
                     c->att_out, (uint4 *)pack, ntiles, terms);
  return hipGetLastError();
}

}  // namespace dart
