// GEMM family of the routed training step (projections, FFN, vocabulary projection and their
// input-/weight-gradient products) with fused epilogues: bias, ReLU, ReLU mask, residual add,
// fp32 accumulate-into-bucket, segmented (Wq|Wk|Wv) operands.
//
//   gemm_simt_kernel : fp32-accumulate FMA kernel for any layout and dtype; the fp32 contexts'
//                      path and the fallback for shapes the MFMA kernel does not take.
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

}  // namespace

void launch_gemm(hipStream_t st, Dtype dt, const GemmParams& p) {
  if (p.M <= 0 || p.N <= 0) return;
  dim3 grid((p.N + SB - 1) / SB, (p.M + SB - 1) / SB);
  if (dt == BF16) gemm_simt_kernel<bf16_t><<<grid, 256, 0, st>>>(p);
  else gemm_simt_kernel<float><<<grid, 256, 0, st>>>(p);
}

}  // namespace mm
