// Kernels of routed greedy translation (paper section 3.2: a task is translated with its own
// modules): attention of one new query per sentence over cached keys and values, and the
// pick of the next token.  Everything else of a decoding step reuses the training kernels.
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

// One workgroup (64 lanes) per (head, sentence).  o = softmax(q K^T / sqrt(dh)) V over the
// sentence's `len` keys: scores one key per lane, the weighted sum one output element per lane.
// Keys of sentence b start at row cu[b] (len = cu[b+1]-cu[b]) or, with cu == null, at row
// b*seq_rows with len_uniform keys.  Scores and the sum are fp32; p[] lives in LDS.
template <typename T>
__global__ void __launch_bounds__(64)
attn_decode_kernel(const T* __restrict__ q, int64_t q_stride, const T* __restrict__ k, const T* __restrict__ v,
                   int64_t ldkv, const int32_t* __restrict__ cu, int64_t seq_rows, int len_uniform,
                   T* __restrict__ o, int64_t o_stride, int dh, float scale) {
  extern __shared__ float smem[];
  const int h = blockIdx.x, b = blockIdx.y, lane = threadIdx.x;
  const int64_t row0 = cu ? (int64_t)cu[b] : (int64_t)b * seq_rows;
  const int len = cu ? cu[b + 1] - cu[b] : len_uniform;
  float* qs = smem;        // [dh]
  float* p = smem + dh;    // [len]
  for (int e = lane; e < dh; e += 64) qs[e] = ldf(q + (int64_t)b * q_stride + h * dh + e);
  __syncthreads();
  float mx = -INFINITY;
  for (int j = lane; j < len; j += 64) {
    const T* kr = k + (row0 + j) * ldkv + h * dh;
    float s = 0.f;
    for (int e = 0; e < dh; ++e) s = fmaf(qs[e], ldf(kr + e), s);
    s *= scale;
    p[j] = s;
    mx = fmaxf(mx, s);
  }
  for (int off = 32; off; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
  float sum = 0.f;
  for (int j = lane; j < len; j += 64) {
    const float w = __expf(p[j] - mx);
    p[j] = w;
    sum += w;
  }
  for (int off = 32; off; off >>= 1) sum += __shfl_xor(sum, off);
  __syncthreads();
  const float inv = 1.f / sum;
  for (int e = lane; e < dh; e += 64) {
    const T* vc = v + row0 * ldkv + h * dh + e;
    float acc = 0.f;
    for (int j = 0; j < len; ++j) acc = fmaf(p[j], ldf(vc + (int64_t)j * ldkv), acc);
    stf(o + (int64_t)b * o_stride + h * dh + e, acc * inv);
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
  for (int i = tid; i < V; i += 256) {
    const float x = ldf(row + i);
    if (x > best || (x == best && i < best_i)) { best = x; best_i = i; }
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

}  // namespace

void launch_attn_decode(hipStream_t st, Dtype dt, const void* q, int64_t q_stride, const void* k, const void* v,
                        int64_t ldkv, const int32_t* cu, int64_t seq_rows, int len_uniform, int max_len,
                        void* o, int64_t o_stride, int B, int H, int dh) {
  const float scale = 1.0f / sqrtf((float)dh);
  const size_t lds = (size_t)(dh + max_len) * sizeof(float);
  const dim3 grid(H, B);
  if (dt == BF16)
    attn_decode_kernel<bf16_t><<<grid, 64, lds, st>>>((const bf16_t*)q, q_stride, (const bf16_t*)k, (const bf16_t*)v,
                                                      ldkv, cu, seq_rows, len_uniform, (bf16_t*)o, o_stride, dh, scale);
  else
    attn_decode_kernel<float><<<grid, 64, lds, st>>>((const float*)q, q_stride, (const float*)k, (const float*)v,
                                                     ldkv, cu, seq_rows, len_uniform, (float*)o, o_stride, dh, scale);
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

}  // namespace mm
