// HBM-bound kernels of the routed training step: token bookkeeping, embedding gather and its
// gradient, LayerNorm forward/backward, column sums (bias gradients), label-smoothed
// cross-entropy, Adam.  gfx950, 64-wide wavefronts, 16-byte accesses wherever rows allow.
#include "mm_kernels.h"

#include <hip/hip_ext.h>

namespace mm {

namespace {

constexpr int WAVE = 64;

template <typename T> struct Io;
template <> struct Io<float> {
  static __device__ __forceinline__ float ld(const float* p) { return *p; }
  static __device__ __forceinline__ void st(float* p, float v) { *p = v; }
  static __device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
  static __device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
};
template <> struct Io<bf16_t> {
  static __device__ __forceinline__ float ld(const bf16_t* p) { return bf16_to_f32(*p); }
  static __device__ __forceinline__ void st(bf16_t* p, float v) { *p = f32_to_bf16(v); }
  static __device__ __forceinline__ float4 ld4(const bf16_t* p) {
    uint2 r = *reinterpret_cast<const uint2*>(p);
    float4 f;
    f.x = __uint_as_float(r.x << 16); f.y = __uint_as_float(r.x & 0xffff0000u);
    f.z = __uint_as_float(r.y << 16); f.w = __uint_as_float(r.y & 0xffff0000u);
    return f;
  }
  static __device__ __forceinline__ void st4(bf16_t* p, float4 v) {
    uint2 r;
    r.x = pack2_bf16(v.x, v.y);
    r.y = pack2_bf16(v.z, v.w);
    *reinterpret_cast<uint2*>(p) = r;
  }
};

// streaming accesses (touched once per step): bypass-friendly nontemporal loads and stores
typedef float f32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 nt_ld4(const float* p) {
  const f32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t*>(p));
  return make_float4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ void nt_st4(float* p, float4 v) {
  const f32x4_t o = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(o, reinterpret_cast<f32x4_t*>(p));
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

// ----------------------------------------------------------------------------------------------
// token bookkeeping
// ----------------------------------------------------------------------------------------------
__global__ void pack_ids_kernel(const int32_t* __restrict__ src_ids, const int32_t* __restrict__ tgt_ids,
                                const int32_t* __restrict__ lens, const int32_t* __restrict__ cu_s,
                                const int32_t* __restrict__ cu_u, int S_max, int T_max, int V,
                                int32_t* src_tok, int32_t* src_pos, int32_t* dec_tok, int32_t* dec_pos,
                                int32_t* label, int32_t* flag) {
  const int b = blockIdx.x;
  const int s = lens[2 * b], t = lens[2 * b + 1];
  int bad = 0;
  for (int i = threadIdx.x; i < S_max; i += blockDim.x) {
    int id = src_ids[(int64_t)b * S_max + i];
    if (i < s) {
      if (id < 0 || id >= V) { bad |= 1; id = 0; }
      const int row = cu_s[b] + i;
      src_tok[row] = id;
      src_pos[row] = i;
    } else if (id != 0) {
      bad |= 2;
    }
  }
  for (int i = threadIdx.x; i < T_max; i += blockDim.x) {
    int id = tgt_ids[(int64_t)b * T_max + i];
    if (i < t) {
      if (id < 0 || id >= V) { bad |= 1; id = 0; }
      if (i < t - 1) {
        const int row = cu_u[b] + i;
        dec_tok[row] = id;
        dec_pos[row] = i;
      }
      if (i >= 1) label[cu_u[b] + i - 1] = id;
    } else if (id != 0) {
      bad |= 2;
    }
  }
  if (bad) atomicOr(flag, bad);
}

// The attention kernels use the same predicate (attn_blocked in kernels_attention.hip states it
// again for its own use; this kernel materialises it for bit-exact checks).
__global__ void mask_dump_kernel(const int32_t* __restrict__ cu_q, const int32_t* __restrict__ cu_k,
                                 int Lq, int Lk, int mode, uint8_t* out) {
  const int b = blockIdx.x;
  const int len_k = cu_k[b + 1] - cu_k[b];
  (void)cu_q;
  for (int e = threadIdx.x; e < Lq * Lk; e += blockDim.x) {
    const int i = e / Lk, j = e % Lk;
    const bool blocked = (j >= len_k) || (mode == 1 && j > i);
    out[(int64_t)b * Lq * Lk + e] = blocked ? 1 : 0;
  }
}

// ----------------------------------------------------------------------------------------------
// embedding gather + positional encoding
// ----------------------------------------------------------------------------------------------
template <typename T>
__global__ void embed_fwd_kernel(const T* __restrict__ E, const float* __restrict__ pe,
                                 const int32_t* __restrict__ tok, const int32_t* __restrict__ pos,
                                 float* __restrict__ x, int rows, int d, float sqrt_d, int pos_all) {
  const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // one float4 each
  const int per_row = d >> 2;
  if (q >= (int64_t)rows * per_row) return;
  const int row = (int)(q / per_row), c = (int)(q % per_row) << 2;
  const float4 e = Io<T>::ld4(E + (int64_t)tok[row] * d + c);
  const float4 p = Io<float>::ld4(pe + (int64_t)(pos ? pos[row] : pos_all) * d + c);
  float4 o;  // product rounded, then sum rounded (no fused multiply-add)
  o.x = __fadd_rn(__fmul_rn(sqrt_d, e.x), p.x);
  o.y = __fadd_rn(__fmul_rn(sqrt_d, e.y), p.y);
  o.z = __fadd_rn(__fmul_rn(sqrt_d, e.z), p.z);
  o.w = __fadd_rn(__fmul_rn(sqrt_d, e.w), p.w);
  Io<float>::st4(x + (int64_t)row * d + c, o);
}

// ----------------------------------------------------------------------------------------------
// embedding gradient: sort (token, row) keys, then one workgroup per run of equal tokens adds its
// rows in ascending row order.  No atomics: same bits every run.
// ----------------------------------------------------------------------------------------------
constexpr int ROW_BITS = 14;  // rows < 16384, tokens < 2^17

// Sorted position of key i = number of keys below it (keys are distinct: the row is part of the
// key).  A workgroup owns 64 keys, one per lane; its four wavefronts each compare them with a
// quarter of the batch's keys and the four counts are added through LDS.  The keys to compare
// against are fetched 64 at a time, one per lane (the next 64 are in flight meanwhile), and handed
// round lane by lane.  rows / 64 workgroups, no ordering between them, no atomics, exact.
__global__ void __launch_bounds__(256) rank_keys_kernel(const int32_t* __restrict__ tok, int rows,
                                                        uint32_t* __restrict__ keys) {
  __shared__ int part[4][64];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int i = blockIdx.x * 64 + lane;
  const uint32_t mine = i < rows ? (((uint32_t)tok[i] << ROW_BITS) | (uint32_t)i) : 0xffffffffu;
  const int quarter = (((rows + 3) >> 2) + 63) & ~63;         // whole groups of 64
  const int j0 = wave * quarter, j1 = min(rows, j0 + quarter);
  auto fetch = [&](int j) -> uint32_t {                        // past the end: a key below nobody
    const int g = j + lane;
    return g < j1 ? (((uint32_t)tok[g] << ROW_BITS) | (uint32_t)g) : 0xffffffffu;
  };
  int rank = 0;
  uint32_t cur = fetch(j0);
  for (int j = j0; j < j1; j += 64) {
    const uint32_t nxt = fetch(j + 64);
#pragma unroll
    for (int l = 0; l < 64; ++l) rank += (int)((uint32_t)__builtin_amdgcn_readlane((int)cur, l) < mine);
    cur = nxt;
  }
  part[wave][lane] = rank;
  __syncthreads();
  if (wave == 0 && i < rows) keys[(part[0][lane] + part[1][lane]) + (part[2][lane] + part[3][lane])] = mine;
}

// Two passes so that the run of the most frequent token (hundreds of rows under a Zipf law) is not
// one workgroup's serial loop.  Pass 1: runs are cut into chunks of EG_CHUNK sorted positions; the
// workgroup at a chunk's first position adds the chunk's rows (4 waves, fixed order).  A run that
// is a single chunk goes straight into the bucket; otherwise the chunk sum is parked in
// partial[position].  Pass 2: the workgroup at a multi-chunk run's first position adds the run's
// chunk sums in ascending order and updates the bucket.
constexpr int EG_CHUNK = 32;

template <int NV>
__device__ __forceinline__ void eg_block_reduce(float4 (&acc)[NV], float (*red)[NV * 256], int wave, int lane) {
  if (wave > 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      float* r = &red[wave - 1][v * 256 + (lane << 2)];
      r[0] = acc[v].x; r[1] = acc[v].y; r[2] = acc[v].z; r[3] = acc[v].w;
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v)
      for (int w = 0; w < 3; ++w) {
        const float* r = &red[w][v * 256 + (lane << 2)];
        acc[v].x += r[0]; acc[v].y += r[1]; acc[v].z += r[2]; acc[v].w += r[3];
      }
  }
}

template <int NV>  // float4 chunks per lane: d <= NV * 256
__global__ void __launch_bounds__(256) embed_grad_chunks_kernel(const uint32_t* __restrict__ keys,
                                                                const float* __restrict__ dx,
                                                                float* __restrict__ bucket,
                                                                float* __restrict__ partial, int rows, int d,
                                                                float sqrt_d) {
  const int p = blockIdx.x;
  const uint32_t token = keys[p] >> ROW_BITS;
  __shared__ int s_before, s_end;
  __shared__ float red[3][NV * 256];
  if (threadIdx.x == 0) { s_before = -1; s_end = min(rows, p + EG_CHUNK); }
  __syncthreads();
  // last position before p holding another token (keys are sorted: the first mismatch going back)
  for (int q = p - 1 - (int)threadIdx.x; q >= 0; q -= blockDim.x)
    if ((keys[q] >> ROW_BITS) != token) { atomicMax(&s_before, q); break; }
  if (threadIdx.x < EG_CHUNK) {
    const int q = p + 1 + threadIdx.x;
    if (q < rows && q < p + EG_CHUNK && (keys[q] >> ROW_BITS) != token) atomicMin(&s_end, q);
  }
  __syncthreads();
  const int run_start = s_before + 1;
  if ((p - run_start) % EG_CHUNK != 0) return;  // not the first position of a chunk (uniform)
  const int end = s_end;
  const bool whole_run = (p == run_start) && (end >= rows || (keys[end] >> ROW_BITS) != token);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float4 acc[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int q = p + wave; q < end; q += 4) {
    const int row = keys[q] & ((1u << ROW_BITS) - 1);
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (lane << 2) + v * 256;
      if (c < d) {
        const float4 g = Io<float>::ld4(dx + (int64_t)row * d + c);
        acc[v].x += g.x; acc[v].y += g.y; acc[v].z += g.z; acc[v].w += g.w;
      }
    }
  }
  eg_block_reduce<NV>(acc, red, wave, lane);
  if (wave == 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (lane << 2) + v * 256;
      if (c < d) {
        if (whole_run) {
          float* dst = bucket + (int64_t)token * d + c;
          float4 o = Io<float>::ld4(dst);
          o.x += sqrt_d * acc[v].x; o.y += sqrt_d * acc[v].y; o.z += sqrt_d * acc[v].z; o.w += sqrt_d * acc[v].w;
          Io<float>::st4(dst, o);
        } else {
          Io<float>::st4(partial + (int64_t)p * d + c, acc[v]);
        }
      }
    }
  }
}

template <int NV>
__global__ void __launch_bounds__(256) embed_grad_runs_kernel(const uint32_t* __restrict__ keys,
                                                              const float* __restrict__ partial,
                                                              float* __restrict__ bucket, int rows, int d,
                                                              float sqrt_d) {
  const int p = blockIdx.x;
  const uint32_t token = keys[p] >> ROW_BITS;
  if (p > 0 && (keys[p - 1] >> ROW_BITS) == token) return;                         // not a run head
  if (p + EG_CHUNK >= rows || (keys[p + EG_CHUNK] >> ROW_BITS) != token) return;   // single chunk: done in pass 1
  __shared__ float red[3][NV * 256];
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float4 acc[NV];
#pragma unroll
  for (int v = 0; v < NV; ++v) acc[v] = make_float4(0.f, 0.f, 0.f, 0.f);
  for (int q = p + wave * EG_CHUNK; q < rows && (keys[q] >> ROW_BITS) == token; q += 4 * EG_CHUNK) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (lane << 2) + v * 256;
      if (c < d) {
        const float4 g = Io<float>::ld4(partial + (int64_t)q * d + c);
        acc[v].x += g.x; acc[v].y += g.y; acc[v].z += g.z; acc[v].w += g.w;
      }
    }
  }
  eg_block_reduce<NV>(acc, red, wave, lane);
  if (wave == 0) {
#pragma unroll
    for (int v = 0; v < NV; ++v) {
      const int c = (lane << 2) + v * 256;
      if (c < d) {
        float* dst = bucket + (int64_t)token * d + c;
        float4 o = Io<float>::ld4(dst);
        o.x += sqrt_d * acc[v].x; o.y += sqrt_d * acc[v].y; o.z += sqrt_d * acc[v].z; o.w += sqrt_d * acc[v].w;
        Io<float>::st4(dst, o);
      }
    }
  }
}

// ----------------------------------------------------------------------------------------------
// LayerNorm
// ----------------------------------------------------------------------------------------------
template <typename T, int NV>
__global__ void __launch_bounds__(256) layernorm_fwd_kernel(const float* __restrict__ x,
                                                            const float* __restrict__ gamma,
                                                            const float* __restrict__ beta,
                                                            T* __restrict__ y, float* __restrict__ mean,
                                                            float* __restrict__ rstd, int rows, int d,
                                                            float eps, int x_parts, int64_t x_part_stride,
                                                            float* __restrict__ x_sum) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= rows) return;
  float4 v[NV];
  float s = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int c = (lane << 2) + k * 256;
    v[k] = c < d ? Io<float>::ld4(x + (int64_t)row * d + c) : make_float4(0.f, 0.f, 0.f, 0.f);
  }
  if (x_parts > 1) {   // x arrives as partial sums: add them in order, keep the sum
    for (int p0 = 1; p0 < x_parts; p0 += 4) {          // up to 4 * NV loads in flight
      float4 u[4][NV];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int pt = p0 + i < x_parts ? p0 + i : p0;
#pragma unroll
        for (int k = 0; k < NV; ++k) {
          const int c = (lane << 2) + k * 256;
          u[i][k] = c < d ? Io<float>::ld4(x + pt * x_part_stride + (int64_t)row * d + c) : make_float4(0.f, 0.f, 0.f, 0.f);
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        if (p0 + i < x_parts) {
#pragma unroll
          for (int k = 0; k < NV; ++k) { v[k].x += u[i][k].x; v[k].y += u[i][k].y; v[k].z += u[i][k].z; v[k].w += u[i][k].w; }
        }
      }
    }
    if (x_sum) {
#pragma unroll
      for (int k = 0; k < NV; ++k) {
        const int c = (lane << 2) + k * 256;
        if (c < d) Io<float>::st4(x_sum + (int64_t)row * d + c, v[k]);
      }
    }
  }
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    s += (v[k].x + v[k].y) + (v[k].z + v[k].w);
  }
  const float mu = wave_sum(s) / (float)d;
  float q = 0.f;
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int c = (lane << 2) + k * 256;
    if (c < d) {
      v[k].x -= mu; v[k].y -= mu; v[k].z -= mu; v[k].w -= mu;
      q += (v[k].x * v[k].x + v[k].y * v[k].y) + (v[k].z * v[k].z + v[k].w * v[k].w);
    }
  }
  const float var = wave_sum(q) / (float)d;
  const float rs = 1.0f / sqrtf(var + eps);
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int c = (lane << 2) + k * 256;
    if (c < d) {
      const float4 g = Io<float>::ld4(gamma + c), b = Io<float>::ld4(beta + c);
      float4 o;
      o.x = v[k].x * rs * g.x + b.x; o.y = v[k].y * rs * g.y + b.y;
      o.z = v[k].z * rs * g.z + b.z; o.w = v[k].w * rs * g.w + b.w;
      Io<T>::st4(y + (int64_t)row * d + c, o);
    }
  }
  if (lane == 0) { mean[row] = mu; rstd[row] = rs; }
}

// Each wavefront walks rows blockIdx*LNB_WAVES+wave, +gridDim*LNB_WAVES, ...; column sums for gamma/beta stay in
// registers and leave as one partial row per workgroup: partial[block][0][d] = dgamma part,
// partial[block][1][d] = dbeta part.
constexpr int LNB_WAVES = 8;   // wavefronts (rows in flight) per workgroup of the backward kernel
template <typename T, int NV>
__global__ void __launch_bounds__(64 * LNB_WAVES) layernorm_bwd_kernel(
    const float* __restrict__ dy, const float* __restrict__ x, const float* __restrict__ mean,
    const float* __restrict__ rstd, const float* __restrict__ gamma, const float* __restrict__ dres,
    float* __restrict__ dx_out, T* __restrict__ dxT_out, float* __restrict__ partial, int rows, int d, int dy_parts,
    int64_t dy_part_stride) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float4 g[NV], ag[NV], ab[NV];
#pragma unroll
  for (int k = 0; k < NV; ++k) {
    const int c = (lane << 2) + k * 256;
    g[k] = c < d ? Io<float>::ld4(gamma + c) : make_float4(0.f, 0.f, 0.f, 0.f);
    ag[k] = make_float4(0.f, 0.f, 0.f, 0.f);
    ab[k] = make_float4(0.f, 0.f, 0.f, 0.f);
  }
  const float inv_d = 1.0f / (float)d;
  for (int row = blockIdx.x * LNB_WAVES + wave; row < rows; row += gridDim.x * LNB_WAVES) {
    const float mu = mean[row], rs = rstd[row];
    float4 xh[NV], dh[NV], rv[NV];
    float s1 = 0.f, s2 = 0.f;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int c = (lane << 2) + k * 256;
      if (c < d) {
        const float4 xv = Io<float>::ld4(x + (int64_t)row * d + c);
        float4 dv = Io<float>::ld4(dy + (int64_t)row * d + c);
        if (dres) rv[k] = Io<float>::ld4(dres + (int64_t)row * d + c);   // in flight during the reductions
        for (int s = 1; s < dy_parts; ++s) {   // split-K partial sums of the producing product
          const float4 t = Io<float>::ld4(dy + s * dy_part_stride + (int64_t)row * d + c);
          dv.x += t.x; dv.y += t.y; dv.z += t.z; dv.w += t.w;
        }
        xh[k].x = (xv.x - mu) * rs; xh[k].y = (xv.y - mu) * rs;
        xh[k].z = (xv.z - mu) * rs; xh[k].w = (xv.w - mu) * rs;
        ag[k].x += dv.x * xh[k].x; ag[k].y += dv.y * xh[k].y;
        ag[k].z += dv.z * xh[k].z; ag[k].w += dv.w * xh[k].w;
        ab[k].x += dv.x; ab[k].y += dv.y; ab[k].z += dv.z; ab[k].w += dv.w;
        dh[k].x = dv.x * g[k].x; dh[k].y = dv.y * g[k].y;
        dh[k].z = dv.z * g[k].z; dh[k].w = dv.w * g[k].w;
        s1 += (dh[k].x + dh[k].y) + (dh[k].z + dh[k].w);
        s2 += (dh[k].x * xh[k].x + dh[k].y * xh[k].y) + (dh[k].z * xh[k].z + dh[k].w * xh[k].w);
      }
    }
    const float m1 = wave_sum(s1) * inv_d, m2 = wave_sum(s2) * inv_d;
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int c = (lane << 2) + k * 256;
      if (c < d) {
        float4 o;
        o.x = rs * (dh[k].x - m1 - xh[k].x * m2); o.y = rs * (dh[k].y - m1 - xh[k].y * m2);
        o.z = rs * (dh[k].z - m1 - xh[k].z * m2); o.w = rs * (dh[k].w - m1 - xh[k].w * m2);
        if (dres) { o.x += rv[k].x; o.y += rv[k].y; o.z += rv[k].z; o.w += rv[k].w; }
        Io<float>::st4(dx_out + (int64_t)row * d + c, o);
        if (dxT_out) Io<T>::st4(dxT_out + (int64_t)row * d + c, o);
      }
    }
  }
  // workgroup reduction of the waves' column sums, fixed order
  __shared__ float red[LNB_WAVES - 1][2][NV * 256];
  if (wave > 0) {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      float* r0 = &red[wave - 1][0][k * 256 + (lane << 2)];
      float* r1 = &red[wave - 1][1][k * 256 + (lane << 2)];
      r0[0] = ag[k].x; r0[1] = ag[k].y; r0[2] = ag[k].z; r0[3] = ag[k].w;
      r1[0] = ab[k].x; r1[1] = ab[k].y; r1[2] = ab[k].z; r1[3] = ab[k].w;
    }
  }
  __syncthreads();
  if (wave == 0) {
#pragma unroll
    for (int k = 0; k < NV; ++k) {
      const int c = (lane << 2) + k * 256;
      if (c < d) {
        float4 sg = ag[k], sb = ab[k];
        for (int w = 0; w < LNB_WAVES - 1; ++w) {
          const float* r0 = &red[w][0][k * 256 + (lane << 2)];
          const float* r1 = &red[w][1][k * 256 + (lane << 2)];
          sg.x += r0[0]; sg.y += r0[1]; sg.z += r0[2]; sg.w += r0[3];
          sb.x += r1[0]; sb.y += r1[1]; sb.z += r1[2]; sb.w += r1[3];
        }
        Io<float>::st4(partial + ((int64_t)blockIdx.x * 2 + 0) * d + c, sg);
        Io<float>::st4(partial + ((int64_t)blockIdx.x * 2 + 1) * d + c, sb);
      }
    }
  }
}

// dst[seg(n)] += sum_p partial[p * pstride + n] for n < N.  64 columns per workgroup; the four
// wavefronts each take every fourth partial row (loads independent, coalesced over columns) and
// are combined in a fixed order.  Columns n >= n_first go to dst2 (index n - n_first) instead.
__global__ void __launch_bounds__(256) reduce_partials_kernel(const float* __restrict__ partial, int n_partial,
                                                              int64_t pstride, int N, float* __restrict__ dst,
                                                              int split, int64_t seg_stride, float* __restrict__ dst2,
                                                              int n_first, int overwrite) {
  __shared__ float red[4][64];
  const int c = threadIdx.x & 63, r = threadIdx.x >> 6;
  const int n = blockIdx.x * 64 + c;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (n < N) {
    int p = r;
    for (; p + 12 < n_partial; p += 16) {
      s0 += partial[(int64_t)p * pstride + n];
      s1 += partial[(int64_t)(p + 4) * pstride + n];
      s2 += partial[(int64_t)(p + 8) * pstride + n];
      s3 += partial[(int64_t)(p + 12) * pstride + n];
    }
    for (; p < n_partial; p += 4) s0 += partial[(int64_t)p * pstride + n];
  }
  red[r][c] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (r == 0 && n < N) {
    const float s = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
    float* o;
    if (dst2 && n >= n_first) o = dst2 + (n - n_first);
    else o = split ? dst + (int64_t)(n / split) * seg_stride + (n % split) : dst + n;
    *o = overwrite ? s : *o + s;
  }
}

// All LayerNorm gain/shift gradients of a step in one launch: job j owns blocks
// [first_block, first_block + ceil(2d/64)); each block reduces 64 columns of the job's partial
// rows ([n_partial][2][d]) in the same fixed order as reduce_partials_kernel.
__global__ void __launch_bounds__(256) ln_reduce_grouped_kernel(const LnReduceJob* __restrict__ jobs, int n_jobs) {
  __shared__ float red[4][64];
  int lo = 0, hi = n_jobs - 1;
  const int blk = blockIdx.x;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (jobs[mid].first_block <= blk) lo = mid; else hi = mid - 1;
  }
  const LnReduceJob jb = jobs[lo];
  const int c = threadIdx.x & 63, r = threadIdx.x >> 6;
  const int n = (blk - jb.first_block) * 64 + c;
  const int N = 2 * jb.d;
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  if (n < N) {
    const float* part = jb.partial + n;
    int p = r;
    for (; p + 12 < jb.n_partial; p += 16) {
      s0 += part[(int64_t)p * N];
      s1 += part[(int64_t)(p + 4) * N];
      s2 += part[(int64_t)(p + 8) * N];
      s3 += part[(int64_t)(p + 12) * N];
    }
    for (; p < jb.n_partial; p += 4) s0 += part[(int64_t)p * N];
  }
  red[r][c] = (s0 + s1) + (s2 + s3);
  __syncthreads();
  if (r == 0 && n < N) {
    const float s = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
    float* o = n < jb.d ? jb.dgamma + n : jb.dbeta + (n - jb.d);
    *o = jb.overwrite ? s : *o + s;
  }
}

// ----------------------------------------------------------------------------------------------
// column sums: grid (ceil(N/256), chunks); each workgroup sums its row chunk for 256 columns
// ----------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(256) colsum_kernel(const T* __restrict__ Y, int64_t ldy, int M, int N,
                                                     int rows_per_chunk, float* __restrict__ partial) {
  const int n = blockIdx.x * 256 + threadIdx.x;
  if (n >= N) return;
  const int r0 = blockIdx.y * rows_per_chunk;
  const int r1 = min(M, r0 + rows_per_chunk);
  float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
  int r = r0;
  for (; r + 3 < r1; r += 4) {
    s0 += Io<T>::ld(Y + (int64_t)r * ldy + n);
    s1 += Io<T>::ld(Y + (int64_t)(r + 1) * ldy + n);
    s2 += Io<T>::ld(Y + (int64_t)(r + 2) * ldy + n);
    s3 += Io<T>::ld(Y + (int64_t)(r + 3) * ldy + n);
  }
  for (; r < r1; ++r) s0 += Io<T>::ld(Y + (int64_t)r * ldy + n);
  partial[(int64_t)blockIdx.y * N + n] = (s0 + s1) + (s2 + s3);
}

// ----------------------------------------------------------------------------------------------
// label-smoothed cross-entropy, one workgroup per row
// ----------------------------------------------------------------------------------------------
template <typename T>
__global__ void __launch_bounds__(1024) ce_kernel(T* __restrict__ z, const int32_t* __restrict__ label,
                                                  float* __restrict__ loss_rows, int V, float eps,
                                                  float scale, const int32_t* __restrict__ flag) {
  const int row = blockIdx.x;
  T* zr = z + (int64_t)row * V;
  const int tid = threadIdx.x, nthr = blockDim.x;
  const int wave = tid >> 6, lane = tid & 63, nwave = nthr >> 6;
  const int y = label[row];
  // the target logit, read before any wavefront starts overwriting the row with the gradient
  float zy = 0.f;
  if (tid == 0) zy = Io<T>::ld(zr + y);
  // pass 1: running max, rescaled sum of exponentials, plain sum
  float mx = -INFINITY, se = 0.f, sz = 0.f;
  for (int c = tid * 4; c < V; c += nthr * 4) {  // V % 4 == 0
    const float4 v = Io<T>::ld4(zr + c);
    const float m4 = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
    if (m4 > mx) { se *= __expf(mx - m4); mx = m4; }
    se += (__expf(v.x - mx) + __expf(v.y - mx)) + (__expf(v.z - mx) + __expf(v.w - mx));
    sz += (v.x + v.y) + (v.z + v.w);
  }
  __shared__ float s_mx[16], s_se[16], s_sz[16];
  __shared__ float s_lse, s_sumz;
  const float wmx = wave_max(mx);
  se = (mx == -INFINITY) ? 0.f : se * __expf(mx - wmx);
  se = wave_sum(se);
  sz = wave_sum(sz);
  if (lane == 0) { s_mx[wave] = wmx; s_se[wave] = se; s_sz[wave] = sz; }
  __syncthreads();
  if (tid == 0) {
    float gm = s_mx[0];
    for (int w = 1; w < nwave; ++w) gm = fmaxf(gm, s_mx[w]);
    float gs = 0.f, gz = 0.f;
    for (int w = 0; w < nwave; ++w) { gs += s_se[w] * __expf(s_mx[w] - gm); gz += s_sz[w]; }
    s_lse = gm + logf(gs);
    s_sumz = gz;
  }
  __syncthreads();
  const float lse = s_lse;
  if (tid == 0) loss_rows[row] = lse - (1.0f - eps) * zy - (eps / (float)V) * s_sumz;
  // pass 2 (the row was just read: served from cache): z <- (softmax - q) * scale * ok
  const float ok = (*flag == 0) ? scale : 0.0f;
  const float uni = eps / (float)V;
  for (int c = tid * 4; c < V; c += nthr * 4) {
    const float4 v = Io<T>::ld4(zr + c);
    float4 o;
    o.x = __expf(v.x - lse) - uni; o.y = __expf(v.y - lse) - uni;
    o.z = __expf(v.z - lse) - uni; o.w = __expf(v.w - lse) - uni;
    if (y >= c && y < c + 4) {
      const float one = 1.0f - eps;
      if (y == c) o.x -= one; else if (y == c + 1) o.y -= one; else if (y == c + 2) o.z -= one; else o.w -= one;
    }
    o.x *= ok; o.y *= ok; o.z *= ok; o.w *= ok;
    Io<T>::st4(zr + c, o);
  }
}

// The same for bf16 rows that fit a workgroup's registers (V a multiple of 8, at most
// 8 * THREADS * NCH): the row is read once with 16-byte loads and stays in registers, the maximum and
// the sums are plain (not online) reductions, and exp(z - max) is computed once and reused for the
// gradient.
template <int NCH, int THREADS>
__global__ void __launch_bounds__(THREADS) ce_rows_kernel(bf16_t* __restrict__ z, const int32_t* __restrict__ label,
                                                       float* __restrict__ loss_rows, int V, float eps, float scale,
                                                       const int32_t* __restrict__ flag) {
  const int row = blockIdx.x;
  bf16_t* zr = z + (int64_t)row * V;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int y = label[row];
  float zy = 0.f;
  if (tid == 0) zy = bf16_to_f32(zr[y]);   // before the row is overwritten
  float val[NCH][8];
  float mx = -INFINITY, sz = 0.f;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int c = (k * THREADS + tid) * 8;
    if (c < V) {
      const uint4 raw = *reinterpret_cast<const uint4*>(zr + c);
      const uint32_t* w = &raw.x;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        val[k][2 * e] = __uint_as_float(w[e] << 16);
        val[k][2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
      }
#pragma unroll
      for (int e = 0; e < 8; ++e) { mx = fmaxf(mx, val[k][e]); sz += val[k][e]; }
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) val[k][e] = -INFINITY;
    }
  }
  constexpr int NW = THREADS / 64;
  __shared__ float s_a[NW], s_b[NW];
  __shared__ float s_max, s_lse, s_inv, s_sumz;
  mx = wave_max(mx);
  if (lane == 0) s_a[wave] = mx;
  __syncthreads();
  if (tid == 0) {
    float gm = s_a[0];
    for (int w = 1; w < NW; ++w) gm = fmaxf(gm, s_a[w]);
    s_max = gm;
  }
  __syncthreads();
  const float gm = s_max;
  const float L2E = 1.44269504088896341f;
  const float off = -gm * L2E;
  float se = 0.f;
#pragma unroll
  for (int k = 0; k < NCH; ++k)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      val[k][e] = __builtin_amdgcn_exp2f(fmaf(val[k][e], L2E, off));   // past the row's end: exp2(-inf) = 0
      se += val[k][e];
    }
  se = wave_sum(se);
  sz = wave_sum(sz);
  if (lane == 0) { s_a[wave] = se; s_b[wave] = sz; }
  __syncthreads();
  if (tid == 0) {
    float gs = 0.f, gz = 0.f;
    for (int w = 0; w < NW; ++w) { gs += s_a[w]; gz += s_b[w]; }
    s_lse = gm + logf(gs);
    s_inv = 1.0f / gs;
    s_sumz = gz;
    loss_rows[row] = s_lse - (1.0f - eps) * zy - (eps / (float)V) * gz;
  }
  __syncthreads();
  const float ok = (*flag == 0) ? scale : 0.0f;
  const float inv = s_inv * ok, uni = (eps / (float)V) * ok, one = (1.0f - eps) * ok;
#pragma unroll
  for (int k = 0; k < NCH; ++k) {
    const int c = (k * THREADS + tid) * 8;
    if (c < V) {
      float o[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = val[k][e] * inv - uni;
      if (y >= c && y < c + 8) {
#pragma unroll
        for (int e = 0; e < 8; ++e) if (y == c + e) o[e] -= one;
      }
      uint4 r;
      r.x = pack2_bf16(o[0], o[1]); r.y = pack2_bf16(o[2], o[3]);
      r.z = pack2_bf16(o[4], o[5]); r.w = pack2_bf16(o[6], o[7]);
      *reinterpret_cast<uint4*>(zr + c) = r;
    }
  }
}

// host_out (may be null): pinned host memory that also receives the sum and, behind it, the word at
// flag - written from here, the result needs no device-to-host copy at the end of the step.
__global__ void __launch_bounds__(1024) sum_scaled_kernel(const float* __restrict__ v, int n, float scale,
                                                          float* __restrict__ out, float* __restrict__ host_out,
                                                          const int32_t* __restrict__ flag) {
  __shared__ float part[16];
  float s = 0.f;
  for (int i = threadIdx.x; i < n; i += blockDim.x) s += v[i];
  s = wave_sum(s);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    float t = 0.f;
    for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += part[w];
    out[0] = t * scale;
    if (host_out) {
      host_out[0] = t * scale;
      reinterpret_cast<int32_t*>(host_out)[1] = *flag;
    }
  }
}

// Copies n 4-byte words from pinned host memory (read by the kernel itself, across the bus) into
// device memory, and clears one more word if asked to.  For the few kilobytes of tables a step and
// an update need on the device: a copy command in their place left the stream idle for several
// microseconds on either side of it.
__global__ void __launch_bounds__(256) upload_words_kernel(const uint32_t* __restrict__ src, uint32_t* __restrict__ dst,
                                                           int n, int32_t* __restrict__ zero_word) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i < n) dst[i] = src[i];
  if (zero_word && i == 0) *zero_word = 0;
}

// ----------------------------------------------------------------------------------------------
// Adam over a segment list
// ----------------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256) adam_kernel(const AdamSegment* __restrict__ segs, int n_segs,
                                                   float lr, float beta1, float beta2, float eps,
                                                   const int32_t* __restrict__ step_flag) {
  // every product and sum below is rounded on its own (no fused multiply-add), so the update is
  // the same fp32 operation sequence as the textbook formulas written one operation at a time
#pragma clang fp contract(off)
  // find the segment of this chunk (n_segs is small)
  int lo = 0, hi = n_segs - 1;
  const int chunk = blockIdx.x;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (segs[mid].first_chunk <= chunk) lo = mid; else hi = mid - 1;
  }
  const AdamSegment sg = segs[lo];
  // the step that filled the buckets may still have been running when this update was enqueued:
  // had it found bad ids it counted for nothing, and a module it alone had used gets no update
  const float n_uses = (step_flag && *step_flag != 0) ? sg.n_uses_alt : sg.n_uses;
  if (n_uses == 0.f) return;
  const int64_t base = (int64_t)(chunk - sg.first_chunk) * ADAM_CHUNK;
  const float omb1 = 1.0f - beta1, omb2 = 1.0f - beta2;
  // all of the chunk's loads are issued before the first result is needed (16 x 16 bytes in
  // flight per thread); slots past the end of the segment re-read its last four elements and are
  // not stored
  constexpr int NIT = ADAM_CHUNK / 1024;
  float4 g[NIT], th[NIT], m[NIT], v[NIT];
  int64_t idx[NIT];
  bool rest[NIT];
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    idx[it] = base + it * 1024 + threadIdx.x * 4;
    const int64_t i = idx[it] < sg.len ? idx[it] : sg.len - 4;
    g[it] = nt_ld4(sg.g + i);
    m[it] = nt_ld4(sg.m + i); v[it] = nt_ld4(sg.v + i);
    if (sg.keep_g) th[it] = nt_ld4(sg.theta + i);
  }
  // Embedding tables (the modules whose bucket is cleared here): a row that has never received a
  // gradient has g = m = v = 0, and for those values the update changes nothing - m and v stay 0
  // and theta - lr * 0 / (0 + eps) is theta - so such pieces are left alone (nothing more is read,
  // nothing is written); under a Zipf law most rows of a table are in that state.  The other
  // pieces fetch theta now.
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    rest[it] = false;
    if (!sg.keep_g) {
      const uint32_t bits = (__float_as_uint(g[it].x) | __float_as_uint(g[it].y) | __float_as_uint(g[it].z) | __float_as_uint(g[it].w) |
                             __float_as_uint(m[it].x) | __float_as_uint(m[it].y) | __float_as_uint(m[it].z) | __float_as_uint(m[it].w) |
                             __float_as_uint(v[it].x) | __float_as_uint(v[it].y) | __float_as_uint(v[it].z) | __float_as_uint(v[it].w)) & 0x7fffffffu;
      rest[it] = bits == 0u;
      const int64_t i = idx[it] < sg.len ? idx[it] : sg.len - 4;
      if (!rest[it]) th[it] = nt_ld4(sg.theta + i);
    }
  }
#pragma unroll
  for (int it = 0; it < NIT; ++it) {
    if (rest[it]) continue;
    float* gp = &g[it].x; float* tp = &th[it].x; float* mp = &m[it].x; float* vp = &v[it].x;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float ge = gp[e] / n_uses;
      mp[e] = beta1 * mp[e] + omb1 * ge;
      vp[e] = beta2 * vp[e] + omb2 * ge * ge;
      const float mh = mp[e] / sg.bc1, vh = vp[e] / sg.bc2;
      tp[e] = tp[e] - lr * mh / (sqrtf(vh) + eps);
    }
    if (idx[it] < sg.len) {
      const int64_t i = idx[it];
      nt_st4(sg.theta + i, th[it]);
      nt_st4(sg.m + i, m[it]);
      nt_st4(sg.v + i, v[it]);
      // zero the bucket; a table's rows without gradient (most of them) are zero already
      const uint32_t any_bits = __float_as_uint(g[it].x) | __float_as_uint(g[it].y) | __float_as_uint(g[it].z) | __float_as_uint(g[it].w);
      if (!sg.keep_g && any_bits != 0u) nt_st4(sg.g + i, make_float4(0.f, 0.f, 0.f, 0.f));
      if (sg.w16) Io<bf16_t>::st4(sg.w16 + i, th[it]);
    }
  }
}

__global__ void to_bf16_kernel(const float* __restrict__ src, bf16_t* __restrict__ dst, int64_t n4) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n4) Io<bf16_t>::st4(dst + i * 4, Io<float>::ld4(src + i * 4));
}
__global__ void fill_f32_kernel(float* dst, int64_t n, float v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}
__global__ void fill_i32_kernel(int32_t* dst, int64_t n, int32_t v) {
  const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) dst[i] = v;
}

inline int nv_for(int d) { return d <= 256 ? 1 : d <= 512 ? 2 : d <= 1024 ? 4 : 8; }

}  // namespace

// ------------------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------------------
void launch_pack_ids(hipStream_t st, const int32_t* src_ids, const int32_t* tgt_ids, const int32_t* lens,
                     const int32_t* cu_s, const int32_t* cu_u, int B, int S_max, int T_max, int V,
                     int32_t* src_tok, int32_t* src_pos, int32_t* dec_tok, int32_t* dec_pos,
                     int32_t* label, int32_t* flag) {
  pack_ids_kernel<<<B, 128, 0, st>>>(src_ids, tgt_ids, lens, cu_s, cu_u, S_max, T_max, V, src_tok,
                                     src_pos, dec_tok, dec_pos, label, flag);
}

void launch_mask_dump(hipStream_t st, const int32_t* cu_q, const int32_t* cu_k, int B, int Lq, int Lk,
                      int mode, uint8_t* out) {
  mask_dump_kernel<<<B, 256, 0, st>>>(cu_q, cu_k, Lq, Lk, mode, out);
}

void launch_embed_fwd(hipStream_t st, Dtype dt, const void* E, const float* pe, const int32_t* tok,
                      const int32_t* pos, float* x, int rows, int d, float sqrt_d, int pos_all) {
  const int64_t n4 = (int64_t)rows * (d / 4);
  const int grid = (int)((n4 + 255) / 256);
  if (dt == BF16)
    embed_fwd_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)E, pe, tok, pos, x, rows, d, sqrt_d, pos_all);
  else
    embed_fwd_kernel<float><<<grid, 256, 0, st>>>((const float*)E, pe, tok, pos, x, rows, d, sqrt_d, pos_all);
}

void launch_sort_tokens(hipStream_t st, const int32_t* tok, int rows, uint32_t* keys) {
  if (rows > 0) rank_keys_kernel<<<(rows + 63) / 64, 256, 0, st>>>(tok, rows, keys);
}

void launch_embed_grad(hipStream_t st, const uint32_t* keys, const float* dx, float* bucket, float* partial,
                       int rows, int d, float sqrt_d) {
#define MM_EG(NV)                                                                                      \
  embed_grad_chunks_kernel<NV><<<rows, 256, 0, st>>>(keys, dx, bucket, partial, rows, d, sqrt_d);        \
  embed_grad_runs_kernel<NV><<<rows, 256, 0, st>>>(keys, partial, bucket, rows, d, sqrt_d);
  switch (nv_for(d)) {
    case 1: MM_EG(1) break;
    case 2: MM_EG(2) break;
    case 4: MM_EG(4) break;
    default: MM_EG(8) break;
  }
#undef MM_EG
}

#define MM_LN_DISPATCH(KERNEL, T, THREADS, ...)                               \
  switch (nv_for(d)) {                                                        \
    case 1: hipExtLaunchKernelGGL((KERNEL<T, 1>), dim3(grid), dim3(THREADS), 0, st, ev.start, ev.stop, 0, __VA_ARGS__); break;  \
    case 2: hipExtLaunchKernelGGL((KERNEL<T, 2>), dim3(grid), dim3(THREADS), 0, st, ev.start, ev.stop, 0, __VA_ARGS__); break;  \
    case 4: hipExtLaunchKernelGGL((KERNEL<T, 4>), dim3(grid), dim3(THREADS), 0, st, ev.start, ev.stop, 0, __VA_ARGS__); break;  \
    default: hipExtLaunchKernelGGL((KERNEL<T, 8>), dim3(grid), dim3(THREADS), 0, st, ev.start, ev.stop, 0, __VA_ARGS__); break; \
  }

void launch_layernorm_fwd(hipStream_t st, Dtype dt, const float* x, const float* gamma, const float* beta,
                          void* y, float* mean, float* rstd, int rows, int d, float eps, const LaunchEvents& ev,
                          int x_parts, int64_t x_part_stride, float* x_sum) {
  const int grid = (rows + 3) / 4;
  if (dt == BF16) {
    MM_LN_DISPATCH(layernorm_fwd_kernel, bf16_t, 256, x, gamma, beta, (bf16_t*)y, mean, rstd, rows, d, eps, x_parts,
                   x_part_stride, x_sum)
  } else {
    MM_LN_DISPATCH(layernorm_fwd_kernel, float, 256, x, gamma, beta, (float*)y, mean, rstd, rows, d, eps, x_parts,
                   x_part_stride, x_sum)
  }
}

int ln_bwd_partial_rows(int rows) {
  const int want = (rows + LNB_WAVES - 1) / LNB_WAVES;
  return want < 1024 ? want : 1024;
}

void launch_layernorm_bwd(hipStream_t st, Dtype dt, const float* dy, const float* x, const float* mean,
                          const float* rstd, const float* gamma, const float* dres, float* dx_out,
                          void* dxT_out, float* partial, int rows, int d, const LaunchEvents& ev, int dy_parts,
                          int64_t dy_part_stride) {
  const int grid = ln_bwd_partial_rows(rows);
  if (dt == BF16) {
    MM_LN_DISPATCH(layernorm_bwd_kernel, bf16_t, 64 * LNB_WAVES, dy, x, mean, rstd, gamma, dres, dx_out, (bf16_t*)dxT_out,
                   partial, rows, d, dy_parts, dy_part_stride)
  } else {
    MM_LN_DISPATCH(layernorm_bwd_kernel, float, 64 * LNB_WAVES, dy, x, mean, rstd, gamma, dres, dx_out, (float*)nullptr,
                   partial, rows, d, dy_parts, dy_part_stride)
  }
}

void launch_ln_reduce_grouped(hipStream_t st, const LnReduceJob* jobs_dev, int n_jobs, int total_blocks) {
  if (n_jobs > 0) ln_reduce_grouped_kernel<<<total_blocks, 256, 0, st>>>(jobs_dev, n_jobs);
}

int colsum_partial_rows(int M) {
  int chunks = (M + 127) / 128;
  return chunks < 32 ? chunks : 32;
}

void launch_colsum(hipStream_t st, Dtype dt, const void* Y, int y_f32, int64_t ldy, int M, int N,
                   float* partial, float* dst, int split, int64_t seg_stride, int overwrite) {
  const int chunks = colsum_partial_rows(M);
  const int rows_per_chunk = (M + chunks - 1) / chunks;
  dim3 grid((N + 255) / 256, chunks);
  if (y_f32 || dt == F32)
    colsum_kernel<float><<<grid, 256, 0, st>>>((const float*)Y, ldy, M, N, rows_per_chunk, partial);
  else
    colsum_kernel<bf16_t><<<grid, 256, 0, st>>>((const bf16_t*)Y, ldy, M, N, rows_per_chunk, partial);
  reduce_partials_kernel<<<(N + 63) / 64, 256, 0, st>>>(partial, chunks, N, N, dst, split, seg_stride, nullptr, 0, overwrite);
}

void launch_ce(hipStream_t st, Dtype dt, void* z, const int32_t* label, float* loss_rows, int U, int V,
               float eps, float scale, const int32_t* flag, const LaunchEvents& ev) {
  const int threads = V >= 16384 ? 1024 : V >= 2048 ? 256 : 64;
  if (dt == BF16 && V % 8 == 0 && V >= 16384 && V <= 8 * 1024 * 8 && (reinterpret_cast<uintptr_t>(z) & 15) == 0) {
    // measured: 512 threads x 8 chunks for rows up to 32768 logits (0.101 against 0.118 ms at V = 32000
    // with 1024 x 4), 1024 threads x 8 chunks above (0.217 against 0.282 ms at V = 64000 with 512 x 16)
    if (V <= 8 * 1024 * 4)
      hipExtLaunchKernelGGL((ce_rows_kernel<8, 512>), dim3(U), dim3(512), 0, st, ev.start, ev.stop, 0, (bf16_t*)z, label,
                            loss_rows, V, eps, scale, flag);
    else
      hipExtLaunchKernelGGL((ce_rows_kernel<8, 1024>), dim3(U), dim3(1024), 0, st, ev.start, ev.stop, 0, (bf16_t*)z, label,
                            loss_rows, V, eps, scale, flag);
    return;
  }
  if (dt == BF16)
    hipExtLaunchKernelGGL(ce_kernel<bf16_t>, dim3(U), dim3(threads), 0, st, ev.start, ev.stop, 0, (bf16_t*)z, label,
                          loss_rows, V, eps, scale, flag);
  else
    hipExtLaunchKernelGGL(ce_kernel<float>, dim3(U), dim3(threads), 0, st, ev.start, ev.stop, 0, (float*)z, label,
                          loss_rows, V, eps, scale, flag);
}

void launch_sum_scaled(hipStream_t st, const float* v, int n, float scale, float* out, float* host_out,
                       const int32_t* flag) {
  sum_scaled_kernel<<<1, 1024, 0, st>>>(v, n, scale, out, host_out, flag);
}

void launch_upload_words(hipStream_t st, const void* src_pinned, void* dst_dev, size_t n_bytes, int32_t* zero_word) {
  const int n = (int)((n_bytes + 3) / 4);
  if (n <= 0 && !zero_word) return;
  upload_words_kernel<<<n > 0 ? (n + 255) / 256 : 1, 256, 0, st>>>((const uint32_t*)src_pinned, (uint32_t*)dst_dev, n, zero_word);
}

void launch_adam(hipStream_t st, const AdamSegment* segs_dev, int n_segs, int total_chunks, float lr,
                 float beta1, float beta2, float eps, const int32_t* step_flag, const LaunchEvents& ev) {
  if (total_chunks > 0)
    hipExtLaunchKernelGGL(adam_kernel, dim3(total_chunks), dim3(256), 0, st, ev.start, ev.stop, 0, segs_dev, n_segs, lr,
                          beta1, beta2, eps, step_flag);
}

void launch_to_bf16(hipStream_t st, const float* src, bf16_t* dst, int64_t n) {
  const int64_t n4 = n / 4;
  if (n4 > 0) to_bf16_kernel<<<(unsigned)((n4 + 255) / 256), 256, 0, st>>>(src, dst, n4);
}
void launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v) {
  if (n > 0) fill_f32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(dst, n, v);
}
void launch_fill_i32(hipStream_t st, int32_t* dst, int64_t n, int32_t v) {
  if (n > 0) fill_i32_kernel<<<(unsigned)((n + 255) / 256), 256, 0, st>>>(dst, n, v);
}

}  // namespace mm
