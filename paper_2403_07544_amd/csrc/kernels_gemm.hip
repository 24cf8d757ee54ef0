// GEMM family of the routed training step (projections, FFN, vocabulary projection and their
// input-/weight-gradient products) with fused epilogues: bias, ReLU, ReLU mask, residual add,
// fp32 accumulate-into-bucket, segmented (Wq|Wk|Wv) operands.
//
//   gemm_simt_kernel : fp32-accumulate FMA kernel for any layout and dtype; the fp32 contexts'
//                      path and the fallback for shapes the MFMA kernel does not take.
//   gemm_mfma_kernel : bf16 MFMA kernel, LDS-staged 128x128 or 64x64 tiles.
#include "mm_kernels.h"

namespace mm {
namespace {

template <typename T> __device__ __forceinline__ float ldf(const T* p);
template <> __device__ __forceinline__ float ldf<float>(const float* p) { return *p; }
template <> __device__ __forceinline__ float ldf<bf16_t>(const bf16_t* p) { return bf16_to_f32(*p); }

// element (k, n) of the possibly segmented, possibly transposed B operand
template <typename T>
__device__ __forceinline__ float load_b(const GemmParams& p, int k, int n) {
  const T* B = (const T*)p.B;
  int kk = k, nn = n;
  if (p.b_split) {
    if (p.b_split_on_k) { B += (int64_t)(k / p.b_split) * p.b_seg_stride; kk = k % p.b_split; }
    else { B += (int64_t)(n / p.b_split) * p.b_seg_stride; nn = n % p.b_split; }
  }
  return p.transB ? ldf<T>(B + (int64_t)nn * p.ldb + kk) : ldf<T>(B + (int64_t)kk * p.ldb + nn);
}

// epilogue for one output element; shared by all GEMM kernels
template <typename T>
__device__ __forceinline__ void epilogue_store(const GemmParams& p, int m, int n, float acc) {
  int64_t seg = 0; int nn = n;
  if (p.c_split) { seg = n / p.c_split; nn = n % p.c_split; }
  if (p.bias) {
    if (p.bias_split) acc += p.bias[(int64_t)(n / p.bias_split) * p.bias_seg_stride + (n % p.bias_split)];
    else acc += p.bias[n];
  }
  if (p.relu) acc = fmaxf(acc, 0.f);
  if (p.relu_mask) {
    if (!(ldf<T>((const T*)p.relu_mask + (int64_t)m * p.ldm + n) > 0.f)) acc = 0.f;
  }
  if (p.residual) acc += p.residual[seg * p.c_seg_stride + (int64_t)m * p.ldr + nn];
  const int64_t off = seg * p.c_seg_stride + (int64_t)m * p.ldc + nn;
  if (p.out_f32) ((float*)p.C)[off] = acc;
  else if (sizeof(T) == 4) ((float*)p.C)[off] = acc;
  else ((bf16_t*)p.C)[off] = f32_to_bf16(acc);
}

constexpr int SB = 64;   // tile M = N
constexpr int SK = 16;   // tile K

template <typename T>
__global__ void __launch_bounds__(256) gemm_simt_kernel(const GemmParams p) {
  __shared__ float As[SK][SB + 4];
  __shared__ float Bs[SK][SB + 4];
  const int tid = threadIdx.x;
  const int tx = tid & 15, ty = tid >> 4;
  const int m0 = blockIdx.y * SB, n0 = blockIdx.x * SB;
  const T* A = (const T*)p.A;
  float acc[4][4] = {};
  for (int k0 = 0; k0 < p.K; k0 += SK) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int idx = tid + i * 256;
      int mm_, kk;
      if (p.transA) { mm_ = idx & 63; kk = idx >> 6; } else { kk = idx & 15; mm_ = idx >> 4; }
      const int m = m0 + mm_, k = k0 + kk;
      float v = 0.f;
      if (m < p.M && k < p.K)
        v = p.transA ? ldf<T>(A + (int64_t)k * p.lda + m) : ldf<T>(A + (int64_t)m * p.lda + k);
      As[kk][mm_] = v;
      int nn, kb;
      if (p.transB) { kb = idx & 15; nn = idx >> 4; } else { nn = idx & 63; kb = idx >> 6; }
      const int n = n0 + nn, k2 = k0 + kb;
      Bs[kb][nn] = (n < p.N && k2 < p.K) ? load_b<T>(p, k2, n) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < SK; ++kk) {
      const float4 a = *reinterpret_cast<const float4*>(&As[kk][ty * 4]);
      const float4 b = *reinterpret_cast<const float4*>(&Bs[kk][tx * 4]);
      const float av[4] = {a.x, a.y, a.z, a.w}, bv[4] = {b.x, b.y, b.z, b.w};
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = m0 + ty * 4 + i;
    if (m >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int n = n0 + tx * 4 + j;
      if (n < p.N) epilogue_store<T>(p, m, n, acc[i][j]);
    }
  }
}


// =================================================================================================
// bf16 MFMA kernel (v_mfma_f32_32x32x16_bf16), 256 threads = 4 wavefronts, K step 64, LDS double
// buffered.  Both operand tiles sit in LDS as [row][64 k] = 8 chunks of 16 bytes per row, where
// row = m (A) or n (B); chunk c of row r lives in slot c ^ swz(r) so that
//   * a wavefront's fragment reads (32 consecutive rows, one chunk each, 16 bytes per lane) and
//   * the k-contiguous loader's writes (8 lanes cover one row)
// touch every bank group once, and the transposing loader's 8-byte writes (16 lanes write rows
// 8 apart) collide at most pairwise.
// Operands that are k-contiguous in memory are copied 16 bytes at a time.  Operands whose
// contiguous axis is m or n (forward weights [K,N]; both operands of a weight gradient, whose
// reduction runs over tokens) are transposed on the way: a thread loads a 4(k) x 8(col) patch
// with four 16-byte loads, regroups it in registers and writes eight 8-byte k-quads.
// =================================================================================================
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

constexpr int BK = 64;

__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 7) ^ ((row >> 4) & 3); }

// Loads one operand tile (R rows x 64 k) from global memory into registers, then into LDS.
// KC: operand is k-contiguous in memory (element (row,k) at base + row*ld + k), else
// row-contiguous (element at base + k*ld + row).  split/seg_stride: see GemmParams.
template <int R, bool KC>
struct TileLoader {
  static constexpr int NL = KC ? R / 32 : (R >= 128 ? R / 128 : 1);  // work items per thread
  uint4 v[KC ? NL : NL * 4];
  const bf16_t* base; int64_t ld; int row0, row_lim, K;
  int split, split_on_k; int64_t seg_stride;

  __device__ __forceinline__ void load(int k0, int tid) {
    if (KC) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int q = tid + 256 * i, row = q >> 3, c = q & 7;
        const int gr = row0 + row, k = k0 + c * 8;
        uint4 val = make_uint4(0, 0, 0, 0);
        if (gr < row_lim && k < K) {
          const bf16_t* ptr = base;
          int kl = k, rl = gr;
          if (split) {
            if (split_on_k) { const int sg = k / split; kl = k - sg * split; ptr += (int64_t)sg * seg_stride; }
            else { const int sg = gr / split; rl = gr - sg * split; ptr += (int64_t)sg * seg_stride; }
          }
          val = *reinterpret_cast<const uint4*>(ptr + (int64_t)rl * ld + kl);
        }
        v[i] = val;
      }
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int q = tid + 256 * i;
        const int cg = q % (R / 8), kq = q / (R / 8);
        const int gc = row0 + cg * 8;
        const bf16_t* ptr = base;
        int cl = gc;
        bool ok = gc < row_lim && kq < 16;
        if (split && !split_on_k) { const int sg = gc / split; cl = gc - sg * split; ptr += (int64_t)sg * seg_stride; }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = k0 + kq * 4 + j;
          uint4 val = make_uint4(0, 0, 0, 0);
          if (ok && k < K) {
            const bf16_t* pk = ptr;
            int kl = k;
            if (split && split_on_k) { const int sg = k / split; kl = k - sg * split; pk += (int64_t)sg * seg_stride; }
            val = *reinterpret_cast<const uint4*>(pk + (int64_t)kl * ld + cl);
          }
          v[i * 4 + j] = val;
        }
      }
    }
  }

  __device__ __forceinline__ void store(unsigned char* lds, int tid) const {
    if (KC) {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int q = tid + 256 * i, row = q >> 3, c = q & 7;
        *reinterpret_cast<uint4*>(lds + row * 128 + ((c ^ swz(row)) << 4)) = v[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const int q = tid + 256 * i;
        const int cg = q % (R / 8), kq = q / (R / 8);
        if (kq >= 16) continue;
        const uint32_t* w0 = &v[i * 4 + 0].x; const uint32_t* w1 = &v[i * 4 + 1].x;
        const uint32_t* w2 = &v[i * 4 + 2].x; const uint32_t* w3 = &v[i * 4 + 3].x;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int row = cg * 8 + e;
          uint2 o;
          if (e & 1) {
            o.x = (w0[e >> 1] >> 16) | (w1[e >> 1] & 0xffff0000u);
            o.y = (w2[e >> 1] >> 16) | (w3[e >> 1] & 0xffff0000u);
          } else {
            o.x = (w0[e >> 1] & 0xffffu) | (w1[e >> 1] << 16);
            o.y = (w2[e >> 1] & 0xffffu) | (w3[e >> 1] << 16);
          }
          *reinterpret_cast<uint2*>(lds + row * 128 + (((kq >> 1) ^ swz(row)) << 4) + ((kq & 1) << 3)) = o;
        }
      }
    }
  }
};

// CS: also produce the column sums of B over the whole K range (the bias gradient that goes with a
// weight gradient: dW = X^T dY, db = column sums of dY).  Only the tiles of the first tile row do
// it, from the registers the transposing loader has just filled (4 k x 8 columns per thread).
template <int BM, int BN, int WM, int WN, bool KCA, bool KCB, bool CS = false>
__device__ __forceinline__ void gemm_mfma_tile(const GemmParams& p, const int m0, const int n0, unsigned char* lds) {
  static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts");
  constexpr int MT = WM / 32, NT = WN / 32;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wm = wave / (BN / WN), wn = wave % (BN / WN);

  TileLoader<BM, KCA> la;
  la.base = (const bf16_t*)p.A; la.ld = p.lda; la.row0 = m0; la.row_lim = p.M; la.K = p.K;
  la.split = 0; la.split_on_k = 0; la.seg_stride = 0;
  TileLoader<BN, KCB> lb;
  lb.base = (const bf16_t*)p.B; lb.ld = p.ldb; lb.row0 = n0; lb.row_lim = p.N; lb.K = p.K;
  lb.split = p.b_split; lb.split_on_k = p.b_split_on_k; lb.seg_stride = p.b_seg_stride;

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bool do_cs = CS && p.colsum_dst != nullptr && m0 == 0;
  auto add_colsum = [&]() {
    if (CS && !KCB && BN == 128) {
      if (do_cs) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const uint32_t* w = &lb.v[j].x;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            cs[2 * e] += __uint_as_float(w[e] << 16);
            cs[2 * e + 1] += __uint_as_float(w[e] & 0xffff0000u);
          }
        }
      }
    }
  };

  const int nk = (p.K + BK - 1) / BK;
  la.load(0, tid);
  lb.load(0, tid);
  add_colsum();
  la.store(lds, tid);
  lb.store(lds + A_BYTES, tid);
  __syncthreads();
  const int lrow = lane & 31, lhalf = lane >> 5;
  for (int kt = 0; kt < nk; ++kt) {
    const unsigned char* sA = lds + (kt & 1) * STAGE;
    const unsigned char* sB = sA + A_BYTES;
    if (kt + 1 < nk) {
      la.load((kt + 1) * BK, tid);
      lb.load((kt + 1) * BK, tid);
      add_colsum();
    }
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[MT], bfr[NT];
      const int c = kk * 2 + lhalf;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        const int row = wm * WM + i * 32 + lrow;
        af[i] = *reinterpret_cast<const bf16x8_t*>(sA + row * 128 + ((c ^ swz(row)) << 4));
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        const int row = wn * WN + j * 32 + lrow;
        bfr[j] = *reinterpret_cast<const bf16x8_t*>(sB + row * 128 + ((c ^ swz(row)) << 4));
      }
#pragma unroll
      for (int i = 0; i < MT; ++i)
#pragma unroll
        for (int j = 0; j < NT; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < nk) {
      unsigned char* dA = lds + ((kt + 1) & 1) * STAGE;
      la.store(dA, tid);
      lb.store(dA + A_BYTES, tid);
    }
    __syncthreads();
  }

  if (CS && !KCB && BN == 128) {
    if (do_cs) {  // uniform over the workgroup; LDS is free after the loop's last barrier
      float* red = reinterpret_cast<float*>(lds);  // [16 k-groups][128 columns]
      const int cg = tid & 15, kq = tid >> 4;
#pragma unroll
      for (int e = 0; e < 8; ++e) red[kq * 128 + cg * 8 + e] = cs[e];
      __syncthreads();
      if (tid < 128) {
        const int n = n0 + tid;
        if (n < p.N) {
          float t = 0.f;
#pragma unroll
          for (int g = 0; g < 16; ++g) t += red[g * 128 + tid];
          int64_t idx = n;
          if (p.c_split) { const int sg = n / p.c_split; idx = (int64_t)sg * p.c_seg_stride + (n - sg * p.c_split); }
          p.colsum_dst[idx] += t;
        }
      }
    }
  }

  // epilogue: lane holds column n = .. + lane%32 and rows 8*(r/4) + 4*(lane/32) + r%4 of each tile
#pragma unroll
  for (int j = 0; j < NT; ++j) {
    const int n = n0 + wn * WN + j * 32 + lrow;
    if (n >= p.N) continue;
    int64_t cbase = n; 
    if (p.c_split) { const int sg = n / p.c_split; cbase = (int64_t)sg * p.c_seg_stride + (n - sg * p.c_split); }
    float bias = 0.f;
    if (p.bias) {
      if (p.bias_split) { const int sg = n / p.bias_split; bias = p.bias[(int64_t)sg * p.bias_seg_stride + (n - sg * p.bias_split)]; }
      else bias = p.bias[n];
    }
#pragma unroll
    for (int i = 0; i < MT; ++i) {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int m = m0 + wm * WM + i * 32 + 8 * (r >> 2) + 4 * lhalf + (r & 3);
        if (m >= p.M) continue;
        float v = acc[i][j][r] + bias;
        if (p.relu) v = fmaxf(v, 0.f);
        if (p.relu_mask) {
          if (!(bf16_to_f32(((const bf16_t*)p.relu_mask)[(int64_t)m * p.ldm + n]) > 0.f)) v = 0.f;
        }
        if (p.residual) v += p.residual[cbase + (int64_t)m * p.ldr];
        const int64_t off = cbase + (int64_t)m * p.ldc;
        if (p.out_f32) ((float*)p.C)[off] = v;
        else ((bf16_t*)p.C)[off] = f32_to_bf16(v);
      }
    }
  }
}

template <int BM, int BN, int WM, int WN, bool KCA, bool KCB>
__global__ void __launch_bounds__(256) gemm_mfma_kernel(const GemmParams p) {
  extern __shared__ __align__(16) unsigned char lds[];
  gemm_mfma_tile<BM, BN, WM, WN, KCA, KCB>(p, blockIdx.y * BM, blockIdx.x * BN, lds);
}

// Many independent problems of one layout in one launch: workgroup -> (problem, tile) through a
// prefix table of tile counts.  Used for the weight-gradient products of a whole step, each of
// which alone has too few output tiles to fill 256 compute units.
template <int BM, int BN, int WM, int WN, bool KCA, bool KCB>
__global__ void __launch_bounds__(256) gemm_mfma_grouped_kernel(const GemmParams* __restrict__ table,
                                                                const int32_t* __restrict__ tile_start,
                                                                int n_problems) {
  extern __shared__ __align__(16) unsigned char lds[];
  __shared__ GemmParams prm;
  __shared__ int local_tile;
  if (threadIdx.x == 0) {
    int lo = 0, hi = n_problems - 1;
    const int t = blockIdx.x;
    while (lo < hi) {
      const int mid = (lo + hi + 1) >> 1;
      if (tile_start[mid] <= t) lo = mid; else hi = mid - 1;
    }
    prm = table[lo];
    local_tile = t - tile_start[lo];
  }
  __syncthreads();
  const int tiles_n = (prm.N + BN - 1) / BN;
  // consecutive workgroups walk down M first: they share the same columns of B (dY)
  const int tiles_m = (prm.M + BM - 1) / BM;
  const int tm = local_tile % tiles_m, tn = local_tile / tiles_m;
  (void)tiles_n;
  gemm_mfma_tile<BM, BN, WM, WN, KCA, KCB, true>(prm, tm * BM, tn * BN, lds);
}

template <int BM, int BN, int WM, int WN>
void launch_mfma_cfg(hipStream_t st, const GemmParams& p) {
  dim3 grid((p.N + BN - 1) / BN, (p.M + BM - 1) / BM);
  constexpr int LDS = 2 * (BM + BN) * 128;
  const bool kca = !p.transA, kcb = p.transB != 0;
#define MM_GO(KA, KB)                                                                               \
  do {                                                                                              \
    static bool attr_set = false;                                                                   \
    if (!attr_set) {                                                                                \
      hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, BN, WM, WN, KA, KB>,                    \
                          hipFuncAttributeMaxDynamicSharedMemorySize, LDS);                         \
      attr_set = true;                                                                              \
    }                                                                                               \
    gemm_mfma_kernel<BM, BN, WM, WN, KA, KB><<<grid, 256, LDS, st>>>(p);                            \
  } while (0)
  if (kca && kcb) MM_GO(true, true);
  else if (kca && !kcb) MM_GO(true, false);
  else if (!kca && kcb) MM_GO(false, true);
  else MM_GO(false, false);
#undef MM_GO
}

inline bool aligned16(const void* ptr) { return (reinterpret_cast<uintptr_t>(ptr) & 15) == 0; }

// The MFMA kernel takes 16-byte chunks along each operand's contiguous axis.
bool mfma_eligible(const GemmParams& p) {
  if (!aligned16(p.A) || !aligned16(p.B)) return false;
  if (p.lda % 8 || p.ldb % 8) return false;
  if (!p.transA ? p.K % 8 : p.M % 8) return false;       // A's contiguous extent
  if (p.transB ? p.K % 8 : p.N % 8) return false;        // B's contiguous extent
  if (p.b_split && (p.b_split % 8 || p.b_seg_stride % 8)) return false;
  return true;
}

}  // namespace

bool gemm_groupable(Dtype dt, const GemmParams& p) {
  return dt == BF16 && p.transA == 1 && p.transB == 0 && mfma_eligible(p);
}

int gemm_grouped_tiles(const GemmParams& p) { return ((p.M + 127) / 128) * ((p.N + 127) / 128); }

void launch_gemm_grouped_tn(hipStream_t st, const GemmParams* table_dev, const int32_t* tile_start_dev,
                            int n_problems, int total_tiles) {
  if (n_problems <= 0 || total_tiles <= 0) return;
  constexpr int LDS = 2 * (128 + 128) * 128;
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)gemm_mfma_grouped_kernel<128, 128, 64, 64, false, false>,
                        hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    attr_set = true;
  }
  gemm_mfma_grouped_kernel<128, 128, 64, 64, false, false><<<total_tiles, 256, LDS, st>>>(table_dev, tile_start_dev,
                                                                                          n_problems);
}

void launch_gemm_simt(hipStream_t st, Dtype dt, const GemmParams& p) {
  if (p.M <= 0 || p.N <= 0) return;
  dim3 grid((p.N + SB - 1) / SB, (p.M + SB - 1) / SB);
  if (dt == BF16) gemm_simt_kernel<bf16_t><<<grid, 256, 0, st>>>(p);
  else gemm_simt_kernel<float><<<grid, 256, 0, st>>>(p);
}

void launch_gemm(hipStream_t st, Dtype dt, const GemmParams& p) {
  if (p.M <= 0 || p.N <= 0) return;
  if (dt == BF16 && mfma_eligible(p)) {
    const long tiles_big = (long)((p.M + 127) / 128) * ((p.N + 127) / 128);
    if (tiles_big >= 192) launch_mfma_cfg<128, 128, 64, 64>(st, p);
    else launch_mfma_cfg<64, 64, 32, 32>(st, p);
    return;
  }
  launch_gemm_simt(st, dt, p);
}

}  // namespace mm
