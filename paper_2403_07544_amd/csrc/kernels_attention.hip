// Fused masked attention, forward and backward, for packed (unpadded) sentences.
// One workgroup per (sentence, head); the sentence's K and V (and Q, dO in the backward) sit in
// LDS; one wavefront owns one query row (or key row) at a time and the softmax statistics are
// wavefront reductions.  Probabilities never reach HBM: the backward recomputes them from the
// saved row log-sum-exp.
//
// Masking: key j is blocked for query i iff j >= len_k (padding never exists in the packed
// layout, so this only bounds the loop) or, in causal mode, j > i.  Blocked keys get probability
// exactly 0 (they are skipped, not given a large negative score).
#include "mm_kernels.h"

namespace mm {
namespace {

constexpr int WAVE = 64;
constexpr int MAX_KEY_TILES = 4;  // sentences up to 256 tokens

template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }
template <typename T> __device__ __forceinline__ void stf(T* p, float v);
template <> __device__ __forceinline__ void stf<float>(float* p, float v) { *p = v; }
template <> __device__ __forceinline__ void stf<bf16_t>(bf16_t* p, float v) { *p = f32_to_bf16(v); }

__device__ __forceinline__ bool attn_blocked(int i, int j, int len_k, int causal) {
  return j >= len_k || (causal && j > i);
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, WAVE);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, WAVE));
  return v;
}

template <typename T> __host__ __device__ constexpr int row_pad() { return sizeof(T) == 2 ? 2 : 1; }

// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) attn_fwd_kernel(const AttnParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int dh = p.dh, ldr = dh + row_pad<T>();
  T* Ks = reinterpret_cast<T*>(smem_raw);
  T* Vs = Ks + (size_t)p.max_lk * ldr;
  float* qs = reinterpret_cast<float*>(Vs + (size_t)p.max_lk * ldr);  // [4][dh]
  float* ps = qs + 4 * dh;                                            // [4][max_lk]
  const int b = blockIdx.x / p.H, h = blockIdx.x % p.H;
  const int q0 = p.cu_q[b], lq = p.cu_q[b + 1] - q0;
  const int k0 = p.cu_k[b], lk = p.cu_k[b + 1] - k0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const T* qg = (const T*)p.q; const T* kg = (const T*)p.k; const T* vg = (const T*)p.v;
  for (int e = threadIdx.x; e < lk * dh; e += blockDim.x) {
    const int j = e / dh, c = e % dh;
    Ks[j * ldr + c] = kg[(int64_t)(k0 + j) * p.ldk + h * dh + c];
    Vs[j * ldr + c] = vg[(int64_t)(k0 + j) * p.ldv + h * dh + c];
  }
  const float scale = 1.0f / sqrtf((float)dh);
  const int ntile = (lk + WAVE - 1) / WAVE;
  float* myq = qs + wave * dh;
  float* myp = ps + wave * p.max_lk;
  for (int i0 = 0; i0 < lq; i0 += 4) {
    const int i = i0 + wave;
    const bool active = i < lq;
    __syncthreads();  // K/V loaded (first pass); previous row's ps/qs consumed
    if (active && lane < dh) myq[lane] = ldf<T>(qg + (int64_t)(q0 + i) * p.ldq + h * dh + lane);
    __syncthreads();
    if (active) {
      float s[MAX_KEY_TILES];
      float mx = -INFINITY;
#pragma unroll
      for (int t = 0; t < MAX_KEY_TILES; ++t) {
        s[t] = -INFINITY;
        const int j = lane + t * WAVE;
        if (t < ntile && !attn_blocked(i, j, lk, p.causal)) {
          float acc = 0.f;
          for (int c = 0; c < dh; ++c) acc = fmaf(myq[c], ldf<T>(&Ks[j * ldr + c]), acc);
          s[t] = acc * scale;
          mx = fmaxf(mx, s[t]);
        }
      }
      mx = wave_max(mx);
      float e[MAX_KEY_TILES], sum = 0.f;
#pragma unroll
      for (int t = 0; t < MAX_KEY_TILES; ++t) {
        e[t] = (s[t] == -INFINITY) ? 0.f : expf(s[t] - mx);
        sum += e[t];
      }
      sum = wave_sum(sum);
#pragma unroll
      for (int t = 0; t < MAX_KEY_TILES; ++t) {
        const int j = lane + t * WAVE;
        if (t < ntile && j < lk) myp[j] = e[t] / sum;
      }
      if (lane == 0) p.lse[(int64_t)h * p.rows_q + q0 + i] = mx + logf(sum);
    }
    __syncthreads();
    if (active && lane < dh) {
      const int jmax = p.causal ? min(lk, i + 1) : lk;
      float acc = 0.f;
      for (int j = 0; j < jmax; ++j) acc = fmaf(myp[j], ldf<T>(&Vs[j * ldr + lane]), acc);
      stf<T>((T*)p.o + (int64_t)(q0 + i) * p.ldo + h * dh + lane, acc);
    }
  }
}

// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) attn_bwd_kernel(const AttnParams p) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  const int dh = p.dh, ldr = dh + row_pad<T>();
  const int lmax = max(p.max_lq, p.max_lk);
  T* Qs = reinterpret_cast<T*>(smem_raw);
  T* dOs = Qs + (size_t)p.max_lq * ldr;
  T* Ks = dOs + (size_t)p.max_lq * ldr;
  T* Vs = Ks + (size_t)p.max_lk * ldr;
  float* Dd = reinterpret_cast<float*>(Vs + (size_t)p.max_lk * ldr);  // [max_lq]
  float* Ls = Dd + p.max_lq;                                          // [max_lq]
  float* buf1 = Ls + p.max_lq;                                        // [4][lmax]
  float* buf2 = buf1 + 4 * lmax;                                      // [4][lmax]
  const int b = blockIdx.x / p.H, h = blockIdx.x % p.H;
  const int q0 = p.cu_q[b], lq = p.cu_q[b + 1] - q0;
  const int k0 = p.cu_k[b], lk = p.cu_k[b + 1] - k0;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const T* qg = (const T*)p.q; const T* kg = (const T*)p.k; const T* vg = (const T*)p.v;
  const T* og = (const T*)p.o; const T* dog = (const T*)p.d_o;
  for (int e = threadIdx.x; e < lk * dh; e += blockDim.x) {
    const int j = e / dh, c = e % dh;
    Ks[j * ldr + c] = kg[(int64_t)(k0 + j) * p.ldk + h * dh + c];
    Vs[j * ldr + c] = vg[(int64_t)(k0 + j) * p.ldv + h * dh + c];
  }
  for (int e = threadIdx.x; e < lq * dh; e += blockDim.x) {
    const int i = e / dh, c = e % dh;
    Qs[i * ldr + c] = qg[(int64_t)(q0 + i) * p.ldq + h * dh + c];
    dOs[i * ldr + c] = dog[(int64_t)(q0 + i) * p.lddo + h * dh + c];
  }
  // D_i = sum_c dO[i][c] * O[i][c]  (= rowsum(dP * P)), one wave per row
  for (int i = wave; i < lq; i += 4) {
    float part = 0.f;
    for (int c = lane; c < dh; c += WAVE)
      part += ldf<T>(dog + (int64_t)(q0 + i) * p.lddo + h * dh + c) *
              ldf<T>(og + (int64_t)(q0 + i) * p.ldo + h * dh + c);
    part = wave_sum(part);
    if (lane == 0) { Dd[i] = part; Ls[i] = p.lse[(int64_t)h * p.rows_q + q0 + i]; }
  }
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)dh);
  float* my1 = buf1 + wave * lmax;
  float* my2 = buf2 + wave * lmax;

  // phase 1: dQ, one query row per wave
  {
    const int ntile = (lk + WAVE - 1) / WAVE;
    for (int i0 = 0; i0 < lq; i0 += 4) {
      const int i = i0 + wave;
      const bool active = i < lq;
      if (active) {
        const float Li = Ls[i], Di = Dd[i];
        for (int t = 0; t < ntile; ++t) {
          const int j = lane + t * WAVE;
          if (j < lk) {
            float ds = 0.f;
            if (!attn_blocked(i, j, lk, p.causal)) {
              float s = 0.f, dp = 0.f;
              for (int c = 0; c < dh; ++c) {
                s = fmaf(ldf<T>(&Qs[i * ldr + c]), ldf<T>(&Ks[j * ldr + c]), s);
                dp = fmaf(ldf<T>(&dOs[i * ldr + c]), ldf<T>(&Vs[j * ldr + c]), dp);
              }
              const float pr = expf(s * scale - Li);
              ds = pr * (dp - Di) * scale;
            }
            my1[j] = ds;
          }
        }
      }
      __syncthreads();
      if (active && lane < dh) {
        const int jmax = p.causal ? min(lk, i + 1) : lk;
        float acc = 0.f;
        for (int j = 0; j < jmax; ++j) acc = fmaf(my1[j], ldf<T>(&Ks[j * ldr + lane]), acc);
        stf<T>((T*)p.dq + (int64_t)(q0 + i) * p.lddq + h * dh + lane, acc);
      }
      __syncthreads();
    }
  }
  // phase 2: dK and dV, one key row per wave
  {
    const int ntile = (lq + WAVE - 1) / WAVE;
    for (int j0 = 0; j0 < lk; j0 += 4) {
      const int j = j0 + wave;
      const bool active = j < lk;
      if (active) {
        for (int t = 0; t < ntile; ++t) {
          const int i = lane + t * WAVE;
          if (i < lq) {
            float pr = 0.f, ds = 0.f;
            if (!attn_blocked(i, j, lk, p.causal)) {
              float s = 0.f, dp = 0.f;
              for (int c = 0; c < dh; ++c) {
                s = fmaf(ldf<T>(&Qs[i * ldr + c]), ldf<T>(&Ks[j * ldr + c]), s);
                dp = fmaf(ldf<T>(&dOs[i * ldr + c]), ldf<T>(&Vs[j * ldr + c]), dp);
              }
              pr = expf(s * scale - Ls[i]);
              ds = pr * (dp - Dd[i]) * scale;
            }
            my1[i] = pr;
            my2[i] = ds;
          }
        }
      }
      __syncthreads();
      if (active && lane < dh) {
        const int imin = p.causal ? j : 0;
        float av = 0.f, ak = 0.f;
        for (int i = imin; i < lq; ++i) {
          av = fmaf(my1[i], ldf<T>(&dOs[i * ldr + lane]), av);
          ak = fmaf(my2[i], ldf<T>(&Qs[i * ldr + lane]), ak);
        }
        stf<T>((T*)p.dv + (int64_t)(k0 + j) * p.lddv + h * dh + lane, av);
        stf<T>((T*)p.dk + (int64_t)(k0 + j) * p.lddk + h * dh + lane, ak);
      }
      __syncthreads();
    }
  }
}

template <typename T>
size_t lds_bytes_t(int dh, int max_lq, int max_lk, bool backward) {
  const size_t ldr = dh + row_pad<T>();
  if (!backward)
    return 2 * (size_t)max_lk * ldr * sizeof(T) + (4 * (size_t)dh + 4 * (size_t)max_lk) * sizeof(float) + 16;
  const size_t lmax = max_lq > max_lk ? max_lq : max_lk;
  return 2 * ((size_t)max_lq + max_lk) * ldr * sizeof(T) + (2 * (size_t)max_lq + 8 * lmax) * sizeof(float) + 16;
}

}  // namespace

size_t attn_lds_bytes(Dtype dt, int dh, int max_lq, int max_lk, bool backward) {
  return dt == BF16 ? lds_bytes_t<bf16_t>(dh, max_lq, max_lk, backward)
                    : lds_bytes_t<float>(dh, max_lq, max_lk, backward);
}

void launch_attn_fwd(hipStream_t st, Dtype dt, const AttnParams& p) {
  const size_t lds = attn_lds_bytes(dt, p.dh, p.max_lq, p.max_lk, false);
  if (dt == BF16) {
    hipFuncSetAttribute((const void*)attn_fwd_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attn_fwd_kernel<bf16_t><<<p.B * p.H, 256, lds, st>>>(p);
  } else {
    hipFuncSetAttribute((const void*)attn_fwd_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attn_fwd_kernel<float><<<p.B * p.H, 256, lds, st>>>(p);
  }
}

void launch_attn_bwd(hipStream_t st, Dtype dt, const AttnParams& p) {
  const size_t lds = attn_lds_bytes(dt, p.dh, p.max_lq, p.max_lk, true);
  if (dt == BF16) {
    hipFuncSetAttribute((const void*)attn_bwd_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attn_bwd_kernel<bf16_t><<<p.B * p.H, 256, lds, st>>>(p);
  } else {
    hipFuncSetAttribute((const void*)attn_bwd_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attn_bwd_kernel<float><<<p.B * p.H, 256, lds, st>>>(p);
  }
}

}  // namespace mm
