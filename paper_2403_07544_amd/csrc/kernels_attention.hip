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

#include <hip/hip_ext.h>

#include <algorithm>

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


// =================================================================================================
// bf16 MFMA attention for head size 64.
//
// A wavefront owns 32 queries and keeps the whole score row of each in registers, so the softmax
// is the plain one (row maximum, exponentials, one division), not an online rescaling.  Scores
// are computed transposed, S^T = K Q^T (keys x queries): in the 32x32 accumulator layout a lane
// then holds, for ITS query (lane % 32), 16 of every 32 keys; the other 16 sit in lane ^ 32.  Row
// statistics are a register reduction plus one exchange with lane ^ 32.  The probabilities are
// already laid out as the B operand of O^T = V^T P^T: accumulator registers 8s..8s+7 of a key
// tile are the eight k-slots of MFMA step s.  Their key order within a block of 16 is
// 0-3, 8-11 (lanes 0-31) and 4-7, 12-15 (lanes 32-63); the fragments of V^T are read from the V
// tile in that same order (frag_tr), so no cross-lane shuffle is needed between the two products.
// =================================================================================================
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// Slot swizzle of a [rows][64] bf16 tile (eight 16-byte slots per 128-byte row; the LDS has 64
// banks, so rows of different parity never meet).  Two access shapes must both spread over the
// banks: a row fragment (one pass = 16 consecutive rows, the same chunk of each: the 8 rows of one
// parity need 8 different slots) and a transposing read (4 or 8 consecutive rows, the same two or
// four adjacent chunks of each: rows 2 apart must differ in the slot's top bit, rows 4 apart in
// the middle one).  Reversing the three bits of row / 2 does both (measured: no bank conflicts
// in either; the plain (row / 2) & 7 made every transposing read take two passes).
__device__ __forceinline__ int swz64(int row) { return ((row & 2) << 1) | ((row >> 1) & 2) | ((row >> 3) & 1); }
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {
  return pack2_bf16(a, b);
}
// Tile loading.  One work item = 4 consecutive rows x one 16-byte chunk (8 columns); a workgroup
// issues the loads of all its tiles back to back and only then starts storing, so a sentence costs
// one global-memory round trip rather than one per loop iteration.  A tile sits in LDS as
// [rows][64] bf16, 128-byte rows, 16-byte chunk c of row r in slot c ^ swz64(r); products that
// need its transpose read it with frag_tr, so each tile is kept once.
__device__ __forceinline__ void tile_fetch(uint4 (&v)[4], const bf16_t* g, int64_t ld, int row0, int len, int item) {
  const int cg = item & 7, tq = item >> 3;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = tq * 4 + j;
    v[j] = make_uint4(0, 0, 0, 0);
    if (row < len) v[j] = *reinterpret_cast<const uint4*>(g + (int64_t)(row0 + row) * ld + cg * 8);
  }
}
__device__ __forceinline__ void tile_store_natural(unsigned char* lds, const uint4 (&v)[4], int item) {
  const int cg = item & 7, tq = item >> 3;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int row = tq * 4 + j;
    *reinterpret_cast<uint4*>(lds + row * 128 + ((cg ^ swz64(row)) << 4)) = v[j];
  }
}
// dot product of two 8-element bf16 chunks
__device__ __forceinline__ float dot8(const uint4& a, const uint4& b) {
  const uint32_t* aw = &a.x; const uint32_t* bw = &b.x;
  float t = 0.f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    t += __uint_as_float(aw[e] << 16) * __uint_as_float(bw[e] << 16);
    t += __uint_as_float(aw[e] & 0xffff0000u) * __uint_as_float(bw[e] & 0xffff0000u);
  }
  return t;
}
__device__ __forceinline__ bf16x8_t frag_natural(const unsigned char* lds, int row, int chunk) {
  return *reinterpret_cast<const bf16x8_t*>(lds + row * 128 + ((chunk ^ swz64(row)) << 4));
}
// A-operand fragment of the transpose of a natural tile, formed by the transposing LDS read
// ds_read_b64_tr_b16 (within 16 lanes, lane j supplies the address of 4 columns of row j / 4 and
// lane i receives rows 0..3 of column i).  The lane that owns tile column ct*32 + (lane & 31)
// gets, for e = 0..7, the element of tile row rbase + 8 (e >> 2) + 4 hh + (e & 3), hh = lane >> 5:
// the order in which the accumulators of a 32x32 product hold their 16 rows (8 s2 .. 8 s2 + 7 of
// them make the other operand, see frag_from_regs), so the two k orders agree.
__device__ __forceinline__ bf16x8_t frag_tr(const unsigned char* lds, int rbase, int ct, int lane) {
  typedef short s16x4_t __attribute__((ext_vector_type(4)));
  typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
  const int jj = lane & 15, g2 = (lane >> 4) & 1, hh = lane >> 5;
  const int col = ct * 32 + 16 * g2 + 4 * (jj & 3);
  union { s16x4_t h[2]; bf16x8_t f; } u;
#pragma unroll
  for (int rd = 0; rd < 2; ++rd) {
    const int row = rbase + 8 * rd + 4 * hh + (jj >> 2);
    u.h[rd] = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        (lds_s16x4_ptr)(lds + row * 128 + (((col >> 3) ^ swz64(row)) << 4) + (((col >> 2) & 1) << 3)));
  }
  return u.f;
}
__device__ __forceinline__ bf16x8_t frag_from_regs(const float* v) {
  union { uint32_t u[4]; bf16x8_t f; } c;
  c.u[0] = pack_bf16(v[0], v[1]); c.u[1] = pack_bf16(v[2], v[3]);
  c.u[2] = pack_bf16(v[4], v[5]); c.u[3] = pack_bf16(v[6], v[7]);
  return c.f;
}

// Stores a wavefront's 32 x 64 result tile.  The accumulators hold it transposed: lane (lcol, hh)
// owns output row lcol and, per register group g4 of column tile ct, the four consecutive columns
// ct*32 + 8*g4 + 4*hh ...  Written from there each store instruction would put 16 bytes into each
// of 32 different rows.  Each half of the tile (32 columns) goes through the wavefront's own 2 KB
// LDS patch instead (rows of 64 bytes, the 8-byte piece p of row r at position p ^ ((r >> 1) & 7),
// so that the 16 rows one pass of a write touches use all banks) and leaves as 64-byte row
// pieces, four lanes per row.  Only LDS traffic of this wavefront is involved, so
// a wavefront-level fence orders the patch writes before the reads; no workgroup barrier.
constexpr int STORE_PATCH_BYTES = 2048;
__device__ __forceinline__ void store_tile_rows(unsigned char* patch, const f32x16_t (&acc)[2], bf16_t* dst0, int64_t ld,
                                                int rows_valid, int lane) {
  const int lcol = lane & 31, hh = lane >> 5;
#pragma unroll
  for (int ct = 0; ct < 2; ++ct) {
#pragma unroll
    for (int g4 = 0; g4 < 4; ++g4) {
      uint2 o;
      o.x = pack_bf16(acc[ct][4 * g4 + 0], acc[ct][4 * g4 + 1]);
      o.y = pack_bf16(acc[ct][4 * g4 + 2], acc[ct][4 * g4 + 3]);
      *reinterpret_cast<uint2*>(patch + lcol * 64 + ((((g4 << 1) | hh) ^ ((lcol >> 1) & 7)) << 3)) = o;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      const int row = 16 * i + (lane >> 2), c = lane & 3;
      // pieces 2c and 2c + 1 sit next to each other at positions (2c) ^ x and (2c + 1) ^ x: one
      // 16-byte read, halves exchanged when x is odd
      const int x = (row >> 1) & 7;
      uint4 v = *reinterpret_cast<const uint4*>(patch + row * 64 + ((c ^ (x >> 1)) << 4));
      if (x & 1) v = make_uint4(v.z, v.w, v.x, v.y);
      if (row < rows_valid) *reinterpret_cast<uint4*>(dst0 + (int64_t)row * ld + ct * 32 + c * 8) = v;
    }
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");   // the patch is free again once these reads are done
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  }
}

template <int NKT>
__global__ void __launch_bounds__(512, 1) attn_fwd_mfma_kernel(const AttnParams p_in) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  (void)p_in;
  const AttnParams p = kernarg_block<AttnParams>();
  const int b = blockIdx.x / p.H, h = blockIdx.x % p.H;
  const int q0 = p.cu_q[b], lq = p.cu_q[b + 1] - q0;
  const int k0 = p.cu_k[b], lk = p.cu_k[b + 1] - k0;
  const int nkt = (lk + 31) >> 5, Lp = nkt * 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lcol = lane & 31, hh = lane >> 5;
  const int nqt = (lq + 31) >> 5, Lqp = nqt * 32;
  unsigned char* Kn = smem_raw;
  unsigned char* Vn = Kn + Lp * 128;
  unsigned char* Qn = Vn + Lp * 128;
  unsigned char* patch = Qn + Lqp * 128 + wave * STORE_PATCH_BYTES;
  const bf16_t* qg = (const bf16_t*)p.q + h * 64;
  const float scale = 0.125f;  // 1 / sqrt(64)
  const int nwave = blockDim.x >> 6;
  // K, V and Q tiles of the sentence go to LDS with coalesced loads, all issued before the first store
  const int n_items = (Lp > Lqp ? Lp : Lqp) * 2;
  for (int base = 0; base < n_items; base += blockDim.x) {
    const int it = base + tid;
    uint4 vk[4], vv[4], vq[4];
    if (it < Lp * 2) {
      tile_fetch(vk, (const bf16_t*)p.k + h * 64, p.ldk, k0, lk, it);
      tile_fetch(vv, (const bf16_t*)p.v + h * 64, p.ldv, k0, lk, it);
    }
    if (it < Lqp * 2) tile_fetch(vq, qg, p.ldq, q0, lq, it);
    if (it < Lp * 2) {
      tile_store_natural(Kn, vk, it);
      tile_store_natural(Vn, vv, it);
    }
    if (it < Lqp * 2) tile_store_natural(Qn, vq, it);
  }
  __syncthreads();
  for (int qt = wave; qt < nqt; qt += nwave) {
    const int ql = qt * 32 + lcol;
    const bool valid_q = ql < lq;
    const int64_t grow = q0 + (valid_q ? ql : lq - 1);
    bf16x8_t qf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) qf[s] = frag_natural(Qn, ql, 2 * s + hh);
    const int kt_end = p.causal ? min(nkt, qt + 1) : nkt;
    f32x16_t sc[NKT];
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sc[kt][r] = 0.f;
      if (kt < kt_end) {
        // the four fragments of the key tile are requested together: with the read inside each
        // MFMA's operand the compiler waited for every one of them in turn
        bf16x8_t kfr[4];
#pragma unroll
        for (int s = 0; s < 4; ++s) kfr[s] = frag_natural(Kn, kt * 32 + lcol, 2 * s + hh);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int s = 0; s < 4; ++s)
          sc[kt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qf[s], sc[kt], 0, 0, 0);
      }
    }
    // softmax over keys: registers, then the other half of the keys in lane ^ 32.  The maximum is
    // taken over the raw products and the 1/sqrt(64) scale rides in the exponent's multiplier;
    // only tiles that hold keys past the sentence end or the causal diagonal are masked; the
    // probabilities go to the second product un-normalised and O is divided once at the end.
    const float cexp = scale * 1.44269504088896341f;   // exp(s * scale) = exp2(s * cexp)
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
      if (kt < kt_end) {
        if (kt * 32 + 32 > lk || (p.causal && kt == qt)) {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int key = kt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
            if (attn_blocked(ql, key, lk, p.causal)) sc[kt][r] = -INFINITY;
          }
        }
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sc[kt][r]);
      }
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, WAVE));
    const float moff = -mx * cexp;
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
      if (kt < kt_end) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float e = __builtin_amdgcn_exp2f(fmaf(sc[kt][r], cexp, moff));   // blocked: exp2(-inf) = 0
          sc[kt][r] = e;
          sum += e;
        }
      }
    }
    sum += __shfl_xor(sum, 32, WAVE);
    const float inv = 1.0f / sum;
    if (valid_q && hh == 0) p.lse[(int64_t)h * p.rows_q + q0 + ql] = mx * scale + __logf(sum);
    f32x16_t oc[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) oc[ct][r] = 0.f;
#pragma unroll
    for (int kt = 0; kt < NKT; ++kt) {
      if (kt < kt_end) {
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          float pv[8];
#pragma unroll
          for (int e = 0; e < 8; ++e) pv[e] = sc[kt][8 * s2 + e];
          bf16x8_t vtr[2];
#pragma unroll
          for (int ct = 0; ct < 2; ++ct) vtr[ct] = frag_tr(Vn, kt * 32 + s2 * 16, ct, lane);
          const bf16x8_t pf = frag_from_regs(pv);
#pragma unroll
          for (int ct = 0; ct < 2; ++ct)
            oc[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vtr[ct], pf, oc[ct], 0, 0, 0);
        }
      }
    }
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) oc[ct][r] *= inv;
    store_tile_rows(patch, oc, (bf16_t*)p.o + (int64_t)(q0 + qt * 32) * p.ldo + h * 64, p.ldo, lq - qt * 32, lane);
  }
}

inline size_t mfma_fwd_lds(int max_lq, int max_lk, int waves) {
  const int Lq = ((max_lq + 31) / 32) * 32, Lk = ((max_lk + 31) / 32) * 32;
  return (size_t)(2 * Lk + Lq) * 128 + (size_t)waves * STORE_PATCH_BYTES;   // K, V and Q tiles; one store patch per wavefront
}

// Backward with the same layouts, one workgroup per (sentence, head).  The Q, dO, K and V tiles of
// the sentence go to LDS once, with coalesced loads (D_i = sum_c dO[i][c] O[i][c] and the row
// log-sum-exp become two small tables on the way; O itself is not kept).  Every operand fragment
// then comes from LDS: rows of a tile with frag_natural, rows of its transpose with frag_tr.
// Phase A (dQ): a wavefront owns 32 queries and walks the key tiles: S^T = K Q^T, dP^T = V dO^T,
// dS^T = P^T * (dP^T - D) * scale, dQ^T += K^T dS^T.  Phase B (dK, dV): the wavefront owns 32 keys
// and walks the query tiles: S = Q K^T, dP = dO V^T, then dV^T += dO^T P and dK^T += Q^T dS.
// P is recomputed from the saved log-sum-exp in both phases; nothing is exchanged between them, and
// nothing is accumulated with atomics.
__global__ void __launch_bounds__(512, 1) attn_bwd_mfma_kernel(const AttnParams p_in) {
  extern __shared__ __align__(16) unsigned char smem_raw[];
  (void)p_in;
  const AttnParams p = kernarg_block<AttnParams>();
  const int b = blockIdx.x / p.H, h = blockIdx.x % p.H;
  const int q0 = p.cu_q[b], lq = p.cu_q[b + 1] - q0;
  const int k0 = p.cu_k[b], lk = p.cu_k[b + 1] - k0;
  const int nkt = (lk + 31) >> 5, Lkp = nkt * 32;
  const int nqt = (lq + 31) >> 5, Lqp = nqt * 32;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, lcol = lane & 31, hh = lane >> 5;
  const bf16_t* qg = (const bf16_t*)p.q + h * 64;
  const bf16_t* kg = (const bf16_t*)p.k + h * 64;
  const bf16_t* vg = (const bf16_t*)p.v + h * 64;
  const bf16_t* og = (const bf16_t*)p.o + h * 64;
  const bf16_t* dog = (const bf16_t*)p.d_o + h * 64;
  const float* lseg = p.lse + (int64_t)h * p.rows_q + q0;
  const float scale = 0.125f;
  const float cexp = scale * 1.44269504088896341f;   // exp(s * scale) = exp2(s * cexp)
  const int nwave = blockDim.x >> 6;

  float* Dd = reinterpret_cast<float*>(smem_raw);   // [Lqp] D_i * scale
  float* Ls = Dd + Lqp;                             // [Lqp] lse_i in base-2 units
  unsigned char* Qn = reinterpret_cast<unsigned char*>(Ls + Lqp);
  unsigned char* dOn = Qn + Lqp * 128;
  unsigned char* Kn = dOn + Lqp * 128;
  unsigned char* Vn = Kn + Lkp * 128;
  unsigned char* patch = Vn + Lkp * 128 + wave * STORE_PATCH_BYTES;

  // all loads of an iteration are issued before the first store
  const int n_items = (Lqp > Lkp ? Lqp : Lkp) * 2;
  for (int base = 0; base < n_items; base += blockDim.x) {
    const int it = base + tid;
    const bool has_q = it < Lqp * 2, has_k = it < Lkp * 2;
    uint4 vq[4], vdo[4], vo[4], vk[4], vv[4];
    float lse_r[4] = {0.f, 0.f, 0.f, 0.f};
    const int cg = it & 7, tq = it >> 3;
    if (has_q) {
      tile_fetch(vq, qg, p.ldq, q0, lq, it);
      tile_fetch(vdo, dog, p.lddo, q0, lq, it);
      tile_fetch(vo, og, p.ldo, q0, lq, it);
#pragma unroll
      for (int j = 0; j < 4; ++j) lse_r[j] = (cg == 0 && tq * 4 + j < lq) ? lseg[tq * 4 + j] : 0.f;
    }
    if (has_k) {
      tile_fetch(vk, kg, p.ldk, k0, lk, it);
      tile_fetch(vv, vg, p.ldv, k0, lk, it);
    }
    if (has_q) {
      tile_store_natural(Qn, vq, it);
      tile_store_natural(dOn, vdo, it);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        float part = dot8(vdo[j], vo[j]);   // rows past lq were loaded as zeros
        part += __shfl_xor(part, 1, WAVE);
        part += __shfl_xor(part, 2, WAVE);
        part += __shfl_xor(part, 4, WAVE);
        if (cg == 0) { Dd[tq * 4 + j] = part * scale; Ls[tq * 4 + j] = lse_r[j] * 1.44269504088896341f; }
      }
    }
    if (has_k) {
      tile_store_natural(Kn, vk, it);
      tile_store_natural(Vn, vv, it);
    }
  }
  __syncthreads();

  // ---------------- phase A: dQ ----------------
  for (int qt = wave; qt < nqt; qt += nwave) {
    const int ql = qt * 32 + lcol;
    const bool valid_q = ql < lq;
    bf16x8_t qf[4], dof[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      qf[s] = frag_natural(Qn, ql, 2 * s + hh);
      dof[s] = frag_natural(dOn, ql, 2 * s + hh);
    }
    const float lse_q = Ls[ql], Dq = Dd[ql];   // dS = P * (dP - D) * scale = P * (dP * scale - D * scale)
    f32x16_t dq[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) dq[ct][r] = 0.f;
    const int kt_end = p.causal ? min(nkt, qt + 1) : nkt;
    for (int kt = 0; kt < kt_end; ++kt) {
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
      // all fragments of the tile pair are requested before the first MFMA (see the forward kernel)
      bf16x8_t kfr[4], vfr[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        kfr[s] = frag_natural(Kn, kt * 32 + lcol, 2 * s + hh);
        vfr[s] = frag_natural(Vn, kt * 32 + lcol, 2 * s + hh);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr[s], qf[s], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr[s], dof[s], dp, 0, 0, 0);
      }
      // the transposed fragments of K for dQ travel while the exponentials are taken
      bf16x8_t ktr[2][2];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) ktr[s2][ct] = frag_tr(Kn, kt * 32 + s2 * 16, ct, lane);
      // Keys past the sentence end need no mask here: their rows of K are zeros in LDS, so
      // whatever dS holds for them adds nothing to dQ.  Only the causal diagonal tile is masked.
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(fmaf(sc[r], cexp, -lse_q));
        ds[r] = pr * fmaf(dp[r], scale, -Dq);
      }
      if (p.causal && kt == qt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (key > ql) ds[r] = 0.f;
        }
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8_t dsf = frag_from_regs(&ds[8 * s2]);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
          dq[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ktr[s2][ct], dsf, dq[ct], 0, 0, 0);
      }
    }
    store_tile_rows(patch, dq, (bf16_t*)p.dq + (int64_t)(q0 + qt * 32) * p.lddq + h * 64, p.lddq, lq - qt * 32, lane);
  }

  // ---------------- phase B: dK, dV ----------------
  for (int kt = wave; kt < nkt; kt += nwave) {
    const int kl = kt * 32 + lcol;
    const bool valid_k = kl < lk;
    bf16x8_t kf[4], vf[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      kf[s] = frag_natural(Kn, kl, 2 * s + hh);
      vf[s] = frag_natural(Vn, kl, 2 * s + hh);
    }
    f32x16_t dk[2], dv[2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
      for (int r = 0; r < 16; ++r) { dk[ct][r] = 0.f; dv[ct][r] = 0.f; }
    const int qt_begin = p.causal ? kt : 0;
    for (int qt = qt_begin; qt < nqt; ++qt) {
      f32x16_t sc, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sc[r] = 0.f; dp[r] = 0.f; }
      bf16x8_t qfr[4], dofr[4];
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        qfr[s] = frag_natural(Qn, qt * 32 + lcol, 2 * s + hh);
        dofr[s] = frag_natural(dOn, qt * 32 + lcol, 2 * s + hh);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        sc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qfr[s], kf[s], sc, 0, 0, 0);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dofr[s], vf[s], dp, 0, 0, 0);
      }
      bf16x8_t dotr[2][2], qtr[2][2];
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          dotr[s2][ct] = frag_tr(dOn, qt * 32 + s2 * 16, ct, lane);
          qtr[s2][ct] = frag_tr(Qn, qt * 32 + s2 * 16, ct, lane);
        }
      // Queries past the sentence end have zero rows of Q and dO in LDS and add nothing; this
      // wavefront's own keys past the end produce columns that are never stored.  Only the
      // causal diagonal tile is masked.
      float pr[16], ds[16];
#pragma unroll
      for (int g4 = 0; g4 < 4; ++g4) {
        // accumulator registers 4 g4 .. 4 g4 + 3 are four consecutive queries: one 16-byte read each
        const float4 l4 = *reinterpret_cast<const float4*>(Ls + qt * 32 + 8 * g4 + 4 * hh);
        const float4 d4 = *reinterpret_cast<const float4*>(Dd + qt * 32 + 8 * g4 + 4 * hh);
        const float lq4[4] = {l4.x, l4.y, l4.z, l4.w}, dq4[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const int r = 4 * g4 + e;
          pr[r] = __builtin_amdgcn_exp2f(fmaf(sc[r], cexp, -lq4[e]));
          ds[r] = pr[r] * fmaf(dp[r], scale, -dq4[e]);
        }
      }
      if (p.causal && qt == kt) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int qi = qt * 32 + 8 * (r >> 2) + 4 * hh + (r & 3);
          if (kl > qi) { pr[r] = 0.f; ds[r] = 0.f; }
        }
      }
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8_t pf = frag_from_regs(&pr[8 * s2]);
        const bf16x8_t dsf = frag_from_regs(&ds[8 * s2]);
#pragma unroll
        for (int ct = 0; ct < 2; ++ct) {
          dv[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(dotr[s2][ct], pf, dv[ct], 0, 0, 0);
          dk[ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qtr[s2][ct], dsf, dk[ct], 0, 0, 0);
        }
      }
    }
    store_tile_rows(patch, dk, (bf16_t*)p.dk + (int64_t)(k0 + kt * 32) * p.lddk + h * 64, p.lddk, lk - kt * 32, lane);
    store_tile_rows(patch, dv, (bf16_t*)p.dv + (int64_t)(k0 + kt * 32) * p.lddv + h * 64, p.lddv, lk - kt * 32, lane);
  }
}

inline size_t mfma_bwd_lds(int max_lq, int max_lk, int waves) {
  const size_t Lq = ((max_lq + 31) / 32) * 32, Lk = ((max_lk + 31) / 32) * 32;
  // D and lse tables; Q, dO, K, V tiles; one store patch per wavefront
  return 2 * Lq * sizeof(float) + 2 * Lq * 128 + 2 * Lk * 128 + (size_t)waves * STORE_PATCH_BYTES;
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

static bool mfma_ok(Dtype dt, const AttnParams& p) {
  return dt == BF16 && p.dh == 64 && p.max_lk <= 256 && p.max_lq <= 256 && p.ldq % 8 == 0 && p.ldk % 8 == 0 &&
         p.ldv % 8 == 0 && p.ldo % 8 == 0;
}

void launch_attn_fwd(hipStream_t st, Dtype dt, const AttnParams& p, const LaunchEvents& ev) {
  if (mfma_ok(dt, p)) {
    // one wavefront per 32 queries, up to eight: short sentences get small workgroups, so more of them share a CU
    const int threads = 64 * std::min(8, (p.max_lq + 31) / 32);
    const size_t lds = mfma_fwd_lds(p.max_lq, p.max_lk, threads / 64);
    if (p.max_lk <= 128) {
      hipFuncSetAttribute((const void*)attn_fwd_mfma_kernel<4>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipExtLaunchKernelGGL(attn_fwd_mfma_kernel<4>, dim3(p.B * p.H), dim3(threads), lds, st, ev.start, ev.stop, 0, p);
    } else {
      hipFuncSetAttribute((const void*)attn_fwd_mfma_kernel<8>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      hipExtLaunchKernelGGL(attn_fwd_mfma_kernel<8>, dim3(p.B * p.H), dim3(threads), lds, st, ev.start, ev.stop, 0, p);
    }
    return;
  }
  const size_t lds = attn_lds_bytes(dt, p.dh, p.max_lq, p.max_lk, false);
  if (dt == BF16) {
    hipFuncSetAttribute((const void*)attn_fwd_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipExtLaunchKernelGGL(attn_fwd_kernel<bf16_t>, dim3(p.B * p.H), dim3(256), lds, st, ev.start, ev.stop, 0, p);
  } else {
    hipFuncSetAttribute((const void*)attn_fwd_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipExtLaunchKernelGGL(attn_fwd_kernel<float>, dim3(p.B * p.H), dim3(256), lds, st, ev.start, ev.stop, 0, p);
  }
}

void launch_attn_bwd(hipStream_t st, Dtype dt, const AttnParams& p, const LaunchEvents& ev) {
  if (mfma_ok(dt, p) && p.lddo % 8 == 0 && p.lddq % 8 == 0 && p.lddk % 8 == 0 && p.lddv % 8 == 0) {
    int threads = 64 * std::min(8, (std::max(p.max_lq, p.max_lk) + 31) / 32);
    if (mfma_bwd_lds(p.max_lq, p.max_lk, threads / 64) > 160 * 1024) threads = 256;   // the longest sentences: four store patches
    const size_t lds = mfma_bwd_lds(p.max_lq, p.max_lk, threads / 64);
    hipFuncSetAttribute((const void*)attn_bwd_mfma_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipExtLaunchKernelGGL(attn_bwd_mfma_kernel, dim3(p.B * p.H), dim3(threads), lds, st, ev.start, ev.stop, 0, p);
    return;
  }
  const size_t lds = attn_lds_bytes(dt, p.dh, p.max_lq, p.max_lk, true);
  if (dt == BF16) {
    hipFuncSetAttribute((const void*)attn_bwd_kernel<bf16_t>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipExtLaunchKernelGGL(attn_bwd_kernel<bf16_t>, dim3(p.B * p.H), dim3(256), lds, st, ev.start, ev.stop, 0, p);
  } else {
    hipFuncSetAttribute((const void*)attn_bwd_kernel<float>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    hipExtLaunchKernelGGL(attn_bwd_kernel<float>, dim3(p.B * p.H), dim3(256), lds, st, ev.start, ev.stop, 0, p);
  }
}

}  // namespace mm
