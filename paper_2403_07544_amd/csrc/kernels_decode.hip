// Kernels of routed translation (paper section 3.2: a task is translated with its own modules):
// attention of one new query per row over cached keys and values, the greedy pick of the next
// token, and for beam search the selection of the next beam and the move of the token caches to
// their new hypotheses.  Everything else of a decoding step reuses the training kernels.
#include <hip/hip_runtime.h>

#include "mm_kernels.h"

namespace mm {
namespace {

template <typename T> __device__ inline float ldf(const T* p);
template <> __device__ inline float ldf<float>(const float* p) { return *p; }
template <> __device__ inline float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ inline void stf(T* p, float v);
template <> __device__ inline void stf<float>(float* p, float v) { *p = v; }
template <> __device__ inline void stf<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// 16 bytes of a row as floats: 8 bf16 or 4 fp32.
template <typename T> struct Vec16;
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  __device__ static void ld(const bf16_t* p, float* out) {
    const uint4 r = *reinterpret_cast<const uint4*>(p);
    const uint32_t w[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      out[2 * i] = __uint_as_float(w[i] << 16);
      out[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
  }
};
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ static void ld(const float* p, float* out) {
    const float4 r = *reinterpret_cast<const float4*>(p);
    out[0] = r.x; out[1] = r.y; out[2] = r.z; out[3] = r.w;
  }
};

// One workgroup per (head, sentence).  o = softmax(q K^T / sqrt(dh)) V over the sentence's `len`
// keys.  Keys of sentence b start at row cu[b] (len = cu[b+1]-cu[b]) or, with cu == null, at row
// b*seq_rows with len_uniform keys.  Scores and sums are fp32; the scores live in LDS.
// The head size is a power of two of 16-byte chunks (the library admits 16, 32 and 64):
// LPK = dh / Vec16::N lanes share one key, so a wavefront covers 64/LPK keys per pass with
// 16-byte loads that neighbouring lanes take from neighbouring addresses; four wavefronts and
// two passes in flight make a chunk of 8 * 64/LPK keys whose loads are all issued before the
// first is used (a sentence's keys are few: the kernel's time is memory latency, paid once
// per chunk instead of once per key).  The first chunk's values are fetched with its keys.
template <typename T, int LPK>
__global__ void __launch_bounds__(256)
attn_decode_vec_kernel(const T* __restrict__ q, int64_t q_stride, const T* __restrict__ k, const T* __restrict__ v,
                       int64_t ldkv, const int32_t* __restrict__ cu, int64_t seq_rows, int len_uniform,
                       T* __restrict__ o, int64_t o_stride, float scale, int rows_per_seq) {
  constexpr int N = Vec16<T>::N, KPP = 64 / LPK, dh = LPK * N, WAVES = 4, UNR = 2, CH = KPP * WAVES * UNR;
  extern __shared__ float smem[];
  float* red = smem;               // [2][WAVES] maxima, sums
  float* accs = smem + 2 * WAVES;  // [WAVES][dh]
  float* p = accs + WAVES * dh;    // [len] scaled scores
  const int h = blockIdx.x, b = blockIdx.y, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int c = lane % LPK, g = lane / LPK;
  // packed keys (cu given): rows_per_seq consecutive query rows (the hypotheses of one sentence)
  // attend to the same sentence's keys
  const int sb = b / rows_per_seq;
  const int64_t row0 = cu ? (int64_t)cu[sb] : (int64_t)b * seq_rows;
  const int len = cu ? cu[sb + 1] - cu[sb] : len_uniform;
  const int64_t col = (int64_t)h * dh + c * N;
  float qv[N], vv0[UNR][N];
  Vec16<T>::ld(q + (int64_t)b * q_stride + col, qv);
#pragma unroll
  for (int u = 0; u < UNR; ++u) {
    const int j = (u * WAVES + wave) * KPP + g;
    Vec16<T>::ld(v + (row0 + (j < len ? j : len - 1)) * ldkv + col, vv0[u]);
  }
  float mx = -INFINITY;
  for (int j0 = 0; j0 < len; j0 += CH) {
    float kv[UNR][N];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + (u * WAVES + wave) * KPP + g;
      Vec16<T>::ld(k + (row0 + (j < len ? j : len - 1)) * ldkv + col, kv[u]);
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + (u * WAVES + wave) * KPP + g;
      float s = 0.f;
#pragma unroll
      for (int e = 0; e < N; ++e) s = fmaf(qv[e], kv[u][e], s);
#pragma unroll
      for (int off = LPK / 2; off; off >>= 1) s += __shfl_xor(s, off);
      s *= scale;
      if (j < len) {
        if (c == 0) p[j] = s;
        mx = fmaxf(mx, s);
      }
    }
  }
#pragma unroll
  for (int off = 32; off; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  if (lane == 0) red[wave] = mx;
  __syncthreads();
  mx = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
  float acc[N];
#pragma unroll
  for (int e = 0; e < N; ++e) acc[e] = 0.f;
  float sum = 0.f;
  for (int j0 = 0; j0 < len; j0 += CH) {
    float vv[UNR][N];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + (u * WAVES + wave) * KPP + g;
      if (j0 == 0) {
#pragma unroll
        for (int e = 0; e < N; ++e) vv[u][e] = vv0[u][e];
      } else {
        Vec16<T>::ld(v + (row0 + (j < len ? j : len - 1)) * ldkv + col, vv[u]);
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int j = j0 + (u * WAVES + wave) * KPP + g;
      const float w = j < len ? __expf(p[j] - mx) : 0.f;
#pragma unroll
      for (int e = 0; e < N; ++e) acc[e] = fmaf(w, vv[u][e], acc[e]);
      if (c == 0) sum += w;
    }
  }
#pragma unroll
  for (int off = 32; off; off >>= 1) sum += __shfl_xor(sum, off);
#pragma unroll
  for (int off = 32; off >= LPK; off >>= 1) {
#pragma unroll
    for (int e = 0; e < N; ++e) acc[e] += __shfl_xor(acc[e], off);
  }
  if (g == 0) {
#pragma unroll
    for (int e = 0; e < N; ++e) accs[wave * dh + c * N + e] = acc[e];
  }
  if (lane == 0) red[WAVES + wave] = sum;
  __syncthreads();
  for (int e = tid; e < dh; e += 256) {
    const float tot = (red[WAVES] + red[WAVES + 1]) + (red[WAVES + 2] + red[WAVES + 3]);
    const float val = (accs[e] + accs[dh + e]) + (accs[2 * dh + e] + accs[3 * dh + e]);
    stf(o + (int64_t)b * o_stride + h * dh + e, val / tot);
  }
}

// One workgroup per sentence: the largest logit of row b, lowest index among equal ones.
// A sentence that has finished is left alone.  Otherwise the token is written to out_ids[b, t],
// becomes the next decoder input, and EOS marks the sentence finished (n_done counts them).
template <typename T>
__global__ void __launch_bounds__(256)
greedy_pick_kernel(const T* __restrict__ z, int V, int t, int max_new, int eos, int32_t* __restrict__ cur_tok,
                   int32_t* __restrict__ done, int32_t* __restrict__ out_ids, int32_t* __restrict__ out_len,
                   int32_t* __restrict__ n_done) {
  __shared__ float s_val[256];
  __shared__ int s_idx[256];
  const int b = blockIdx.x, tid = threadIdx.x;
  if (done[b]) return;
  const T* row = z + (int64_t)b * V;
  float best = -INFINITY;
  int best_i = V;   // stays V only if the row holds nothing comparable (all NaN)
  constexpr int N = Vec16<T>::N;
  if (V % N == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {   // rows start on 16-byte boundaries
    for (int i0 = tid * N; i0 < V; i0 += 4 * 256 * N) {       // four loads in flight
      float x[4][N];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * 256 * N;
        Vec16<T>::ld(row + (i < V ? i : i0), x[u]);
      }
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const int i = i0 + u * 256 * N;
        if (i < V) {
#pragma unroll
          for (int e = 0; e < N; ++e)
            if (x[u][e] > best || (x[u][e] == best && i + e < best_i)) { best = x[u][e]; best_i = i + e; }
        }
      }
    }
  } else {
    for (int i = tid; i < V; i += 256) {
      const float x = ldf(row + i);
      if (x > best || (x == best && i < best_i)) { best = x; best_i = i; }
    }
  }
  s_val[tid] = best; s_idx[tid] = best_i;
  __syncthreads();
  for (int w = 128; w; w >>= 1) {
    if (tid < w) {
      const float x = s_val[tid + w];
      const int i = s_idx[tid + w];
      if (x > s_val[tid] || (x == s_val[tid] && i < s_idx[tid])) { s_val[tid] = x; s_idx[tid] = i; }
    }
    __syncthreads();
  }
  if (tid == 0) {
    int tok = s_idx[0];
    if (tok >= V) tok = eos;   // a row without a largest entry ends the sentence
    out_ids[(int64_t)b * max_new + t] = tok;
    out_len[b] = t + 1;
    cur_tok[b] = tok;
    if (tok == eos) { done[b] = 1; atomicAdd(n_done, 1); }
  }
}


// ---- beam search -----------------------------------------------------------------------------
// One workgroup per sentence.  The sentence's `beam` hypotheses are rows r0 .. r0 + beam - 1 of z,
// best first.  Candidates: an unfinished hypothesis i extended by token v scores
// score[i] + (z[i, v] - logsumexp(z[i, :])); a finished one is carried at its score.  The `beam`
// best candidates, by (score descending, then hypothesis index, then token id), become the next
// beam.  Two sweeps over the rows: the softmax denominators, then the selection (each thread keeps
// its own best `beam` candidates, the workgroup merges the lists).  All arithmetic is fp32.
constexpr int BEAM_MAX = 8;
constexpr int BEAM_THREADS = 1024;   // per sentence: the sweeps over beam x V logits are the kernel's time
// (score, flat index) order of the candidates: higher score first, then the lower flat index
__device__ __forceinline__ bool cand_before(float sa, int fa, float sb, int fb) {
  return sa > sb || (sa == sb && fa < fb);
}
// K: entries of a thread's candidate list, a compile-time size >= beam (1, 2, 4 or 8).
template <typename T, int K>
__global__ void __launch_bounds__(BEAM_THREADS)
beam_select_kernel(const T* __restrict__ z, int V, int beam, int t, int eos, const float* __restrict__ score_in,
                   const int32_t* __restrict__ done_in, float* __restrict__ score_out, int32_t* __restrict__ done_out,
                   int32_t* __restrict__ next_tok, int32_t* __restrict__ parent_out, int32_t* __restrict__ hist_tok,
                   int32_t* __restrict__ hist_parent, int32_t* __restrict__ n_finished, int R) {
  __shared__ float s_val[BEAM_THREADS];
  __shared__ float s_aux[BEAM_THREADS];
  __shared__ int s_idx[BEAM_THREADS];
  __shared__ int s_who[BEAM_THREADS];
  __shared__ float s_lse[BEAM_MAX], s_score[BEAM_MAX];
  __shared__ int s_done[BEAM_MAX];
  constexpr int N = Vec16<T>::N;
  const int b = blockIdx.x, tid = threadIdx.x, r0 = b * beam;
  const bool vec = V % N == 0 && (reinterpret_cast<uintptr_t>(z) & 15) == 0;   // rows start on 16-byte boundaries
  if (tid < beam) { s_score[tid] = score_in[r0 + tid]; s_done[tid] = done_in[r0 + tid]; }
  __syncthreads();
  // Pass 1, per unfinished row: log of the softmax denominator, running maximum and rescaled sum
  // in one sweep; the threads' (max, sum) pairs are combined the same way.
  for (int i = 0; i < beam; ++i) {
    if (s_done[i]) continue;              // (uniform over the workgroup)
    const T* row = z + (int64_t)(r0 + i) * V;
    float mx = -INFINITY, sum = 0.f;
    auto take = [&](float x) {
      if (x > mx) { sum = sum * __expf(mx - x) + 1.f; mx = x; }
      else if (x == x && mx > -INFINITY) sum += __expf(x - mx);   // (NaN and a leading -inf contribute nothing)
    };
    if (vec) {
      // four loads in flight per thread: a sweep is bound by load latency, not by bytes
      for (int v0 = tid * N; v0 < V; v0 += 4 * BEAM_THREADS * N) {
        float x[4][N];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int v = v0 + u * BEAM_THREADS * N;
          Vec16<T>::ld(row + (v < V ? v : v0), x[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          if (v0 + u * BEAM_THREADS * N < V) {
#pragma unroll
            for (int e = 0; e < N; ++e) take(x[u][e]);
          }
        }
      }
    } else {
      for (int v = tid; v < V; v += BEAM_THREADS) take(ldf(row + v));
    }
    s_val[tid] = mx; s_aux[tid] = sum;
    __syncthreads();
    for (int w = BEAM_THREADS / 2; w; w >>= 1) {
      if (tid < w) {
        const float ma = s_val[tid], mb = s_val[tid + w];
        const float m = fmaxf(ma, mb);
        float acc = 0.f;
        if (ma > -INFINITY) acc += s_aux[tid] * __expf(ma - m);
        if (mb > -INFINITY) acc += s_aux[tid + w] * __expf(mb - m);
        s_val[tid] = m; s_aux[tid] = acc;
      }
      __syncthreads();
    }
    if (tid == 0) s_lse[i] = s_val[0] + __logf(s_aux[0]);
    __syncthreads();
  }
  // Pass 2: every thread keeps the best K >= beam of the candidates it sees (all rows), sorted, in
  // registers; then `beam` rounds of a block-wide arg-max over the threads' first entries, the
  // winner's list moving up by one.
  float cs[K];
  int cf[K];
#pragma unroll
  for (int q = 0; q < K; ++q) { cs[q] = -INFINITY; cf[q] = 0x7fffffff; }
  auto offer = [&](float sc, int flat) {
    // one comparison with the list's last entry decides for nearly every candidate (an empty slot
    // loses to everything; NaN compares false)
    if (!cand_before(sc, flat, cs[K - 1], cf[K - 1])) return;
    cs[K - 1] = sc; cf[K - 1] = flat;
#pragma unroll
    for (int q = K - 1; q > 0; --q) {                      // let it rise
      if (cand_before(cs[q], cf[q], cs[q - 1], cf[q - 1])) {
        const float ts = cs[q]; cs[q] = cs[q - 1]; cs[q - 1] = ts;
        const int tf = cf[q]; cf[q] = cf[q - 1]; cf[q - 1] = tf;
      }
    }
  };
  for (int i = 0; i < beam; ++i) {
    if (s_done[i]) { if (tid == 0) offer(s_score[i], i * V); continue; }   // carried at its score
    const T* row = z + (int64_t)(r0 + i) * V;
    const float base = s_score[i], lse = s_lse[i];
    if (vec) {
      for (int v0 = tid * N; v0 < V; v0 += 4 * BEAM_THREADS * N) {
        float x[4][N];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int v = v0 + u * BEAM_THREADS * N;
          Vec16<T>::ld(row + (v < V ? v : v0), x[u]);
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int v = v0 + u * BEAM_THREADS * N;
          if (v < V) {
#pragma unroll
            for (int e = 0; e < N; ++e) offer(base + (x[u][e] - lse), i * V + v + e);
          }
        }
      }
    } else {
      for (int v = tid; v < V; v += BEAM_THREADS) offer(base + (ldf(row + v) - lse), i * V + v);
    }
  }
  int all_done = 1;
  for (int j = 0; j < beam; ++j) {
    s_val[tid] = cs[0]; s_idx[tid] = cf[0]; s_who[tid] = tid;
    __syncthreads();
    for (int w = BEAM_THREADS / 2; w; w >>= 1) {
      if (tid < w && cand_before(s_val[tid + w], s_idx[tid + w], s_val[tid], s_idx[tid])) {
        s_val[tid] = s_val[tid + w]; s_idx[tid] = s_idx[tid + w]; s_who[tid] = s_who[tid + w];
      }
      __syncthreads();
    }
    const float win = s_val[0];
    const int flat = s_idx[0], who = s_who[0];
    __syncthreads();
    if (tid == who && flat != 0x7fffffff) {                // the winner's list moves up
#pragma unroll
      for (int q = 0; q + 1 < K; ++q) { cs[q] = cs[q + 1]; cf[q] = cf[q + 1]; }
      cs[K - 1] = -INFINITY; cf[K - 1] = 0x7fffffff;
    }
    if (tid == 0) {
      int i = 0, v = 0;
      if (flat != 0x7fffffff) { i = flat / V; v = flat - i * V; }        // (no candidate left: repeat row 0, finished)
      const int carried = flat == 0x7fffffff || s_done[i];
      const int fin = carried || v == eos;
      const int r = r0 + j;
      score_out[r] = flat == 0x7fffffff ? -INFINITY : win;
      done_out[r] = fin;
      next_tok[r] = carried ? 0 : v;
      parent_out[r] = r0 + i;
      hist_tok[(int64_t)t * R + r] = carried ? 0 : v;
      hist_parent[(int64_t)t * R + r] = r0 + i;
      all_done &= fin;
    }
  }
  if (tid == 0 && all_done) atomicAdd(&n_finished[t], 1);
}

// score[r] = 0 for the first row of every sentence's beam, -inf for the others (at the first step
// all rows of a beam hold the same hypothesis; only one of them may compete).
__global__ void beam_init_kernel(float* __restrict__ score, int R, int beam) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r < R) score[r] = (r % beam) == 0 ? 0.f : -INFINITY;
}

// Token caches follow their hypotheses: dst[l][r] = src[l][parent[r]] for the first `bytes` bytes of
// a row's cache (a multiple of 16), all decoder layers in one launch (grid: rows x layers).
struct CachePairs { const char* src[BEAM_LAYERS_MAX]; char* dst[BEAM_LAYERS_MAX]; };
__global__ void __launch_bounds__(256)
cache_gather_kernel(const CachePairs cp, const int32_t* __restrict__ parent, int64_t row_stride, int64_t bytes) {
  const int r = blockIdx.x, l = blockIdx.y;
  const uint4* s = reinterpret_cast<const uint4*>(cp.src[l] + (int64_t)parent[r] * row_stride);
  uint4* d = reinterpret_cast<uint4*>(cp.dst[l] + (int64_t)r * row_stride);
  for (int64_t i = threadIdx.x; i < bytes / 16; i += 256) d[i] = s[i];
}
}  // namespace

bool launch_attn_decode(hipStream_t st, Dtype dt, const void* q, int64_t q_stride, const void* k, const void* v,
                        int64_t ldkv, const int32_t* cu, int64_t seq_rows, int len_uniform, int max_len,
                        void* o, int64_t o_stride, int B, int H, int dh, int rows_per_seq) {
  if (rows_per_seq < 1) return false;
  const float scale = 1.0f / sqrtf((float)dh);
  const dim3 grid(H, B);
  const int n = dt == BF16 ? 8 : 4;                       // elements per 16 bytes
  const int lpk = dh / n;
  const auto al = [](const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; };
  const bool ok = (dh == 16 || dh == 32 || dh == 64) && al(q) && al(k) && al(v) && q_stride % n == 0 && ldkv % n == 0;
  if (!ok) return false;   // (mm_create admits no other head size and the runtime's buffers are aligned)
  const size_t lds = (size_t)(8 + 4 * dh + max_len) * sizeof(float);
#define MM_AD(T, L)                                                                                              \
  case L:                                                                                                        \
    attn_decode_vec_kernel<T, L><<<grid, 256, lds, st>>>((const T*)q, q_stride, (const T*)k, (const T*)v, ldkv, cu, \
                                                         seq_rows, len_uniform, (T*)o, o_stride, scale, rows_per_seq); \
    break;
  if (dt == BF16) {
    switch (lpk) { MM_AD(bf16_t, 2) MM_AD(bf16_t, 4) MM_AD(bf16_t, 8) }
  } else {
    switch (lpk) { MM_AD(float, 4) MM_AD(float, 8) MM_AD(float, 16) }
  }
#undef MM_AD
  return true;
}

void launch_greedy_pick(hipStream_t st, Dtype dt, const void* z, int B, int V, int t, int max_new, int eos,
                        int32_t* cur_tok, int32_t* done, int32_t* out_ids, int32_t* out_len, int32_t* n_done) {
  if (dt == BF16)
    greedy_pick_kernel<bf16_t><<<B, 256, 0, st>>>((const bf16_t*)z, V, t, max_new, eos, cur_tok, done, out_ids,
                                                  out_len, n_done);
  else
    greedy_pick_kernel<float><<<B, 256, 0, st>>>((const float*)z, V, t, max_new, eos, cur_tok, done, out_ids,
                                                 out_len, n_done);
}

bool launch_beam_select(hipStream_t st, Dtype dt, const void* z, int B, int V, int beam, int t, int eos,
                        const float* score_in, const int32_t* done_in, float* score_out, int32_t* done_out,
                        int32_t* next_tok, int32_t* parent_out, int32_t* hist_tok, int32_t* hist_parent,
                        int32_t* n_finished) {
  if (beam < 1 || beam > BEAM_MAX || (int64_t)beam * V > 0x7ffffffe) return false;
  const int R = B * beam;
#define MM_BS(T, K)                                                                                               \
  beam_select_kernel<T, K><<<B, BEAM_THREADS, 0, st>>>((const T*)z, V, beam, t, eos, score_in, done_in, score_out, \
                                                       done_out, next_tok, parent_out, hist_tok, hist_parent,      \
                                                       n_finished, R)
  if (dt == BF16) {
    if (beam == 1) MM_BS(bf16_t, 1); else if (beam == 2) MM_BS(bf16_t, 2); else if (beam <= 4) MM_BS(bf16_t, 4); else MM_BS(bf16_t, 8);
  } else {
    if (beam == 1) MM_BS(float, 1); else if (beam == 2) MM_BS(float, 2); else if (beam <= 4) MM_BS(float, 4); else MM_BS(float, 8);
  }
#undef MM_BS
  return true;
}

void launch_beam_init(hipStream_t st, float* score, int R, int beam) {
  beam_init_kernel<<<(R + 255) / 256, 256, 0, st>>>(score, R, beam);
}

bool launch_cache_gather(hipStream_t st, const char* const* src, char* const* dst, int n_layers, const int32_t* parent,
                         int R, int64_t row_stride_bytes, int64_t bytes) {
  if (n_layers < 1 || n_layers > BEAM_LAYERS_MAX || bytes % 16 || row_stride_bytes % 16) return false;
  CachePairs cp;
  for (int l = 0; l < n_layers; ++l) { cp.src[l] = src[l]; cp.dst[l] = dst[l]; }
  for (int l = n_layers; l < BEAM_LAYERS_MAX; ++l) { cp.src[l] = nullptr; cp.dst[l] = nullptr; }
  cache_gather_kernel<<<dim3(R, n_layers), 256, 0, st>>>(cp, parent, row_stride_bytes, bytes);
  return true;
}

}  // namespace mm
