// GEMM family of the routed training step (projections, FFN, vocabulary projection and their
// input-/weight-gradient products) with fused epilogues: bias, ReLU, ReLU mask, residual add,
// fp32 accumulate-into-bucket, segmented (Wq|Wk|Wv) operands.
//
//   gemm_simt_kernel : fp32-accumulate FMA kernel for any layout and dtype; the fp32 contexts'
//                      path and the fallback for shapes the MFMA kernel does not take.
//   gemm_mfma_kernel : bf16 MFMA kernel, LDS-staged 128x128 or 64x64 tiles.
#include "mm_kernels.h"
#include <algorithm>
#include <vector>

#include <hip/hip_ext.h>

#include <cstring>
#include <type_traits>

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
// buffered.  An operand that is k-contiguous in memory sits in LDS as [row][64 k] = 8 chunks of 16
// bytes per row, row = m (A) or n (B); chunk c of row r lives in slot c ^ swz(r) so that
//   * a wavefront's fragment reads (32 consecutive rows, one chunk each, 16 bytes per lane) and
//   * the loader's writes (8 lanes cover one row)
// touch every bank group once.  An operand whose contiguous axis is m or n (forward weights
// [K,N]; both operands of a weight gradient, whose reduction runs over tokens) is kept as it lies
// in memory, [64 k][rows], copied 16 bytes at a time like the other kind, and the MFMA fragments
// (8 consecutive k of one row per lane) are formed by the transposing LDS read ds_read_b64_tr_b16
// (two per fragment); chunk c of k row r lives in slot c ^ tr_swz(r).  Nothing is regrouped in
// registers and no transposed copy of a weight or an activation exists in HBM.
// =================================================================================================
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4_t* global_u4_ptr;

constexpr int BK = 64;

// 16-byte load from global memory through an address the optimiser cannot reason about: the load
// stays unconditional (no divergent branch around it), which keeps the count of outstanding loads
// exact, so a wait for one K step's data does not drain the prefetched ones.
__device__ __forceinline__ u32x4_t load16_global(const bf16_t* a) {
  uint64_t addr = reinterpret_cast<uint64_t>(a);
  asm volatile("" : "+v"(addr));
  return *reinterpret_cast<global_u4_ptr>(addr);
}

// Tells the compiler a value is the same in every lane (it then lives in scalar registers).
__device__ __forceinline__ uint64_t uniform64(uint64_t v) {
  const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
  const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(v >> 32));
  return ((uint64_t)hi << 32) | lo;
}

// s_waitcnt with only the vector-memory counter constrained: returns once at most N loads of this
// wavefront are still in flight (gfx9 encoding: vmcnt in bits 3:0 and 15:14, the others left open)
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
  __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

__device__ __forceinline__ int swz(int row) { return (row & 7) ^ ((row >> 3) & 7); }
// Chunk swizzle of a tile kept as it lies in memory, [64 k][R] (see gemm_mfma_tile): the four k rows
// that one transposing LDS read touches land in different banks.
template <int R>
__device__ __forceinline__ int tr_swz(int krow) { return R >= 128 ? (krow & 3) << 2 : ((krow >> 1) & 1) << 2; }

// Loads one operand tile (R rows x 64 k) from global memory into registers, then into LDS.
// KC: operand is k-contiguous in memory (element (row,k) at base + row*ld + k), else
// row-contiguous (element at base + k*ld + row).  Everything that does not change from one K step
// to the next (row pointers, bounds, LDS offsets, the segment a row belongs to) is worked out once
// in init(); a K step costs one address add, one compare, one load and one LDS store per item.
template <int R, bool KC>
struct TileLoader {
  static constexpr int NL = KC ? R / 32 : (R >= 128 ? R / 128 : 1);  // work items per thread
  static constexpr int NV = KC ? NL : NL * 4;                          // 16-byte registers per K step
  // row-contiguous tiles of 128 or 256 rows give every one of the 256 threads a k-row quad inside
  // the 64 k rows of a tile (R = 64 leaves half the threads without one): no test, no branch
  static constexpr bool ALL_ITEMS = KC || R >= 128;
  const bf16_t* ptr[NL];      // item address at k = 0
  int klim[NL];               // KC: item valid while k0 < klim; else: k row j valid while k0 + j < klim
  int off[KC ? NL : NL * 4];  // LDS byte offsets inside the tile (row-contiguous operand: one per k row)
  int64_t ld;
  int ksplit; int64_t seg_stride;  // KC only: segments along k (multiple of 64)
  const bf16_t* safe;              // any valid address: out-of-range items read it and are zeroed
  // fast path (tile fully inside the operand, K a multiple of 64, operand spans < 2 GiB): a
  // wave-uniform base pointer plus one 32-bit byte offset per item; a K step only moves the base
  const char* ubase;
  uint32_t voff[NL];
  // The same operand as a raw buffer: a fast-path load is then `buffer_load_dwordx4 v, voff, rsrc,
  // soffset` with the K step's byte offset in a scalar register - no vector instruction forms the
  // address (through a flat pointer the compiler folded base + voff into a 64-bit vector value and
  // added the K offset with a 64-bit vector multiply-add per load).
  __amdgpu_buffer_rsrc_t rsrc;

  __device__ __forceinline__ void init(const bf16_t* base, int64_t ld_, int row0, int row_lim, int K, int split,
                                       int split_on_k, int64_t seg_stride_, int tid) {
    ld = (int64_t)uniform64((uint64_t)ld_);
    safe = base;
    ubase = reinterpret_cast<const char*>(uniform64(reinterpret_cast<uint64_t>(base)));
    rsrc = __builtin_amdgcn_make_buffer_rsrc((void*)ubase, 0, 0x7fffffff, 0x00020000);   // fast path only: operand < 2 GiB
    ksplit = (KC && split && split_on_k) ? __builtin_amdgcn_readfirstlane(split) : 0;
    seg_stride = (int64_t)uniform64((uint64_t)seg_stride_);
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const int q = tid + 256 * i;
      if (KC) {
        const int row = q >> 3, c = q & 7;
        const int gr = row0 + row;
        const bf16_t* b = base;
        int rl = gr;
        if (split && !split_on_k) { const int sg = gr / split; rl = gr - sg * split; b += (int64_t)sg * seg_stride_; }
        ptr[i] = b + (int64_t)rl * ld_ + c * 8;
        voff[i] = (uint32_t)((ptr[i] - base) * 2);
        klim[i] = gr < row_lim ? K - c * 8 : 0;
        off[i] = row * 128 + ((c ^ swz(row)) << 4);
      } else {
        const int cg = q % (R / 8), kq = q / (R / 8);
        const int gc = row0 + cg * 8;
        const bf16_t* b = base;
        int cl = gc;
        if (split && !split_on_k) { const int sg = gc / split; cl = gc - sg * split; b += (int64_t)sg * seg_stride_; }
        ptr[i] = b + (int64_t)(kq * 4) * ld_ + cl;
        voff[i] = kq < 16 ? (uint32_t)((ptr[i] - base) * 2) : 0u;
        klim[i] = (gc < row_lim && kq < 16) ? K - kq * 4 : 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int krow = kq * 4 + j;
          off[i * 4 + j] = kq < 16 ? krow * (R * 2) + ((cg ^ tr_swz<R>(krow)) << 4) : -1;
        }
      }
    }
  }

  __device__ __forceinline__ void load(int k0, u32x4_t (&v)[NV]) const {
    if (KC) {
      int64_t koff = k0;
      if (ksplit) { const int sg = k0 / ksplit; koff = (int64_t)sg * seg_stride + (k0 - sg * ksplit); }
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        // no branch around the load: the compiler then counts outstanding loads exactly and the
        // stores to LDS wait only for the K step they need, not for the prefetched ones
        v[i] = load16_global(k0 < klim[i] ? ptr[i] + koff : safe);  // zeroed when stored if out of range
      }
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        const bf16_t* p0 = ptr[i] + (int64_t)k0 * ld;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          v[i * 4 + j] = load16_global(k0 + j < klim[i] ? p0 + (int64_t)j * ld : safe);
        }
      }
    }
  }

  __device__ __forceinline__ void load_fast(int k0, u32x4_t (&v)[NV]) const {
    if (KC) {
      int64_t koff = k0;
      if (ksplit) { const int sg = k0 / ksplit; koff = (int64_t)sg * seg_stride + (k0 - sg * ksplit); }
      const int so = (int)(koff * 2);
#pragma unroll
      for (int i = 0; i < NL; ++i) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff[i], so, 0);
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int so = (int)(((int64_t)(k0 + j) * ld) * 2);
#pragma unroll
        for (int i = 0; i < NL; ++i) v[i * 4 + j] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff[i], so, 0);
      }
    }
  }

  __device__ __forceinline__ void store_fast(unsigned char* lds, const u32x4_t (&v)[NV]) const {
    if (KC) {
#pragma unroll
      for (int i = 0; i < NL; ++i) *reinterpret_cast<u32x4_t*>(lds + off[i]) = v[i];
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        if (!ALL_ITEMS && off[i * 4] < 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) *reinterpret_cast<u32x4_t*>(lds + off[i * 4 + j]) = v[i * 4 + j];
      }
    }
  }

  // One quarter (Q of 4) of this thread's share of a K step: the LDS stores of tile k_st from v,
  // then the global loads of tile k_ld into the registers just freed.  Spread over the four MFMA
  // groups of a K step, the stores and loads issue while the matrix pipeline is busy.
  // element offset of k along a k-contiguous row (k segments, if any, taken into account)
  __device__ __forceinline__ int64_t k_offset(int k) const {
    if (KC && ksplit) { const int sg = k / ksplit; return (int64_t)sg * seg_stride + (k - sg * ksplit); }
    return k;
  }
  template <int Q, bool F>
  __device__ __forceinline__ void roll(unsigned char* lds, int k_st, int k_ld, int64_t koff, u32x4_t (&v)[NV]) const {
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    if (KC) {
      constexpr int I0 = NL >= 4 ? Q * (NL / 4) : Q, I1 = NL >= 4 ? (Q + 1) * (NL / 4) : (Q < NL ? Q + 1 : Q);
      if (I0 == I1) return;
      const int so = (int)(koff * 2);
#pragma unroll
      for (int i = I0; i < I1; ++i) {
        *reinterpret_cast<u32x4_t*>(lds + off[i]) = (F || k_st < klim[i]) ? v[i] : zero;
        if (F) v[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff[i], so, 0);
        else v[i] = load16_global(k_ld < klim[i] ? ptr[i] + koff : safe);
      }
    } else {
      // quarter Q moves k row Q of every item
      const int so = (int)(((int64_t)(k_ld + Q) * ld) * 2);
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        if (ALL_ITEMS || off[i * 4] >= 0)
          *reinterpret_cast<u32x4_t*>(lds + off[i * 4 + Q]) = (F || k_st + Q < klim[i]) ? v[i * 4 + Q] : zero;
        if (F) v[i * 4 + Q] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)voff[i], so, 0);
        else v[i * 4 + Q] = load16_global(k_ld + Q < klim[i] ? ptr[i] + (int64_t)(k_ld + Q) * ld : safe);
      }
    }
  }

  // k0: the K step these registers were loaded for (items beyond the operand's extent become 0)
  __device__ __forceinline__ void store(unsigned char* lds, int k0, const u32x4_t (&v)[NV]) const {
    const u32x4_t zero = {0u, 0u, 0u, 0u};
    if (KC) {
#pragma unroll
      for (int i = 0; i < NL; ++i) *reinterpret_cast<u32x4_t*>(lds + off[i]) = k0 < klim[i] ? v[i] : zero;
    } else {
#pragma unroll
      for (int i = 0; i < NL; ++i) {
        if (!ALL_ITEMS && off[i * 4] < 0) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j)
          *reinterpret_cast<u32x4_t*>(lds + off[i * 4 + j]) = k0 + j < klim[i] ? v[i * 4 + j] : zero;
      }
    }
  }
};

template <int I0, int I1, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I0 < I1) {
    f(std::integral_constant<int, I0>());
    static_for<I0 + 1, I1>(f);
  }
}

// CS: also produce the column sums of B over the whole K range (the bias gradient that goes with a
// weight gradient: dW = X^T dY, db = column sums of dY).  Only the tiles of the first tile row do
// it, from the registers the loader has just filled (4 k rows x 8 columns per thread).
// PF: K steps whose global loads are in flight ahead of the one being multiplied (register staged).
// DMA (both operands k-contiguous, K a multiple of 128): the tiles go from global memory straight
// into LDS (global_load_lds_dwordx4: lane l of a wavefront deposits its 16 bytes at base + 16 l, so
// one instruction fills eight 128-byte tile rows; the slot swizzle is applied by choosing which
// chunk each lane fetches).  No staging registers, no LDS store instructions.  DMA is the number of
// LDS stages: DMA - 1 tiles are in flight while one is multiplied.  Rows past the edge of an
// operand are read from its last row: they only feed outputs that are never stored.
// PIPE (with DMA >= 3 stages): the K loop is software-pipelined across K steps as well - the
// fragments of the next MFMA groups are read from LDS while the current group multiplies, also
// across the boundary between two tiles, so that the one barrier of a K step sits in the middle of
// a stream of MFMAs instead of in front of an LDS round trip (see run_dma_pipe).
template <int BM, int BN, int WM, int WN, bool KCA, bool KCB, int PF, bool CS = false, int DMA = 0, bool PIPE = false>
__device__ __forceinline__ void gemm_mfma_tile(const GemmParams& p, const int m0, const int n0, unsigned char* lds) {
  static_assert((BM / WM) * (BN / WN) == 4, "four wavefronts");
  constexpr int MT = WM / 32, NT = WN / 32;
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128, STAGE = A_BYTES + B_BYTES;
  // the wavefront's number is the same in all its lanes: held in a scalar register, so that what
  // derives from it (the LDS destination of a direct-to-LDS load goes through M0) needs no
  // lane-to-scalar moves inside the K loop
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int wm = wave / (BN / WN), wn = wave % (BN / WN);

  static_assert(!DMA || (KCA && !CS), "direct-to-LDS loads need a k-contiguous A");
  // An operand whose contiguous axis is m or n is kept in LDS as it lies in memory, [64 k][rows]
  // with 16-byte chunk c of k row r in slot c ^ tr_swz(r), and its MFMA fragments (8 consecutive k
  // of one row per lane) are formed by the transposing LDS read ds_read_b64_tr_b16: within 16
  // lanes, lane j supplies the address of 4 columns of k row j / 4 and lane i receives k rows 0..3
  // of column i.  The slot swizzle spreads the four k rows of one read over different banks.
  // (Register-staged and direct-to-LDS loads fill the same layout.)
  constexpr bool BTR = DMA && !KCB;
  constexpr bool TRA = !KCA, TRB = !KCB;                // operands kept [64 k][rows] in LDS (register path too)
  constexpr int AT_ROW = BM * 2, BT_ROW = BN * 2;       // bytes per k row of such a tile
  auto bt_swz = [](int krow) { return tr_swz<BN>(krow); };
  TileLoader<BM, KCA> la;
  TileLoader<BN, KCB> lb;
  if constexpr (!DMA) {
    la.init((const bf16_t*)p.A, p.lda, m0, p.M, p.K, 0, 0, 0, tid);
    lb.init((const bf16_t*)p.B, p.ldb, n0, p.N, p.K, p.b_split, p.b_split_on_k, p.b_seg_stride, tid);
  }
  // DMA: per-lane source addresses at k = 0, one per wavefront instruction (8 tile rows each)
  constexpr int NIA = BM / 32, NIB = BN / 32;
  const bf16_t* dma_a[DMA ? NIA : 1];
  const bf16_t* dma_b[DMA ? NIB : 1];
  int dma_ksplit = 0; int64_t dma_seg = 0;
  if constexpr (DMA) {
    const int slot = lane & 7;
#pragma unroll
    for (int i = 0; i < NIA; ++i) {
      const int row = (i * 4 + wave) * 8 + (lane >> 3);
      const int gr = min(m0 + row, p.M - 1);
      dma_a[i] = (const bf16_t*)p.A + (int64_t)gr * p.lda + ((slot ^ swz(row)) << 3);
    }
#pragma unroll
    for (int j = 0; j < NIB; ++j) {
      const int row = (j * 4 + wave) * 8 + (lane >> 3);
      const int gr = min(n0 + row, p.N - 1);
      const bf16_t* b = (const bf16_t*)p.B;
      int rl = gr;
      if (p.b_split && !p.b_split_on_k) { const int sg = gr / p.b_split; rl = gr - sg * p.b_split; b += (int64_t)sg * p.b_seg_stride; }
      dma_b[j] = b + (int64_t)rl * p.ldb + ((slot ^ swz(row)) << 3);
      if constexpr (BTR) {
        constexpr int CPR = BN / 8;                     // chunks per k row; one instruction = 64 / CPR rows
        const int krow = (j * 4 + wave) * (64 / CPR) + lane / CPR;
        const int col = min(n0 + (((lane % CPR) ^ bt_swz(krow)) << 3), p.N - 8);
        const bf16_t* bb = (const bf16_t*)p.B;
        int cl = col;
        if (p.b_split) { const int sg = col / p.b_split; cl = col - sg * p.b_split; bb += (int64_t)sg * p.b_seg_stride; }
        dma_b[j] = bb + (int64_t)krow * p.ldb + cl;
      }
    }
    if (p.b_split && p.b_split_on_k) { dma_ksplit = __builtin_amdgcn_readfirstlane(p.b_split); dma_seg = p.b_seg_stride; }
  }
  // quarter q (of 4) of this wavefront's loads of tile kt -> LDS stage at byte offset soff
  auto dma_kb = [&](int kt) -> int64_t {   // B's element offset of tile kt along k (k segments)
    const int k0 = kt * BK;
    if (dma_ksplit) { const int sg = k0 / dma_ksplit; return (int64_t)sg * dma_seg + (k0 - sg * dma_ksplit); }
    return k0;
  };
  auto dma_issue = [&](int soff, int kt, int64_t kb, int q) {
    if constexpr (DMA) {
      const int k0 = kt * BK;
#pragma unroll
      for (int i = 0; i < NIA; ++i)
        if ((i & 3) == q)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(dma_a[i] + k0),
                                           (__attribute__((address_space(3))) void*)(lds + soff + (i * 4 + wave) * 1024), 16, 0, 0);
#pragma unroll
      for (int j = 0; j < NIB; ++j)
        if (((j + NIA) & 3) == q)
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(dma_b[j] + (BTR ? (int64_t)k0 * p.ldb : kb)),
                                           (__attribute__((address_space(3))) void*)(lds + soff + A_BYTES + (j * 4 + wave) * 1024), 16, 0, 0);
    }
  };

  f32x16_t acc[MT][NT];
#pragma unroll
  for (int i = 0; i < MT; ++i)
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // A wavefront tile of 32 x 32 has one accumulator, and the four MFMAs of a K step on it would
  // form one dependent chain (an MFMA can issue every 8 passes, its result is ready after 16):
  // the odd MFMA groups of a K step go to a second accumulator, added in at the end.
  constexpr bool TWO_ACC = (MT * NT == 1);
  f32x16_t acc2;
  if constexpr (TWO_ACC) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc2[r] = 0.f;
  }

  float cs[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  const bool do_cs = CS && p.colsum_dst != nullptr && m0 == 0;
  static_assert(PF == 1 || PF == 2, "one or two K steps of global loads in flight");
  u32x4_t va[PF][TileLoader<BM, KCA>::NV];   // register sets: tile t travels in set t % PF
  u32x4_t vb[PF][TileLoader<BN, KCB>::NV];
  // every item of a thread covers the same 8 columns (items differ in their k rows only)
  constexpr bool CS_ON = CS && !KCB && (BN == 128 || BN == 256);
  auto add_colsum = [&](int k0, const u32x4_t (&v)[TileLoader<BN, KCB>::NV]) {
    if (CS_ON) {
      if (do_cs) {
#pragma unroll
        for (int i = 0; i < TileLoader<BN, KCB>::NL; ++i) {
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            if (k0 + j < lb.klim[i]) {
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                cs[2 * e] += __uint_as_float(v[i * 4 + j][e] << 16);
                cs[2 * e + 1] += __uint_as_float(v[i * 4 + j][e] & 0xffff0000u);
              }
            }
          }
        }
      }
    }
  };

  const int nk = (p.K + BK - 1) / BK;
  const int lrow = lane & 31, lhalf = lane >> 5;
  int a_off[MT][BK / 16], b_off[NT][BK / 16];
  // [64 k][rows] tiles: the two transposing reads (k 0..3, k 4..7) of a fragment
  int bt_off[TRB ? NT : 1][BK / 16][2];
  int at_off[TRA ? MT : 1][BK / 16][2];
  if constexpr (TRA || TRB) {
    const int jj = lane & 15, g2 = (lane >> 4) & 1;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk)
#pragma unroll
      for (int r = 0; r < 2; ++r) {
        const int krow = kk * 16 + lhalf * 8 + r * 4 + (jj >> 2);
        if constexpr (TRB) {
#pragma unroll
          for (int j = 0; j < NT; ++j) {
            const int col = wn * WN + j * 32 + 16 * g2 + 4 * (jj & 3);
            bt_off[j][kk][r] = A_BYTES + krow * BT_ROW + ((((col >> 3) ^ tr_swz<BN>(krow))) << 4) + (((col >> 2) & 1) << 3);
          }
        }
        if constexpr (TRA) {
#pragma unroll
          for (int i = 0; i < MT; ++i) {
            const int col = wm * WM + i * 32 + 16 * g2 + 4 * (jj & 3);
            at_off[i][kk][r] = krow * AT_ROW + ((((col >> 3) ^ tr_swz<BM>(krow))) << 4) + (((col >> 2) & 1) << 3);
          }
        }
      }
  }
#pragma unroll
  for (int kk = 0; kk < BK / 16; ++kk) {
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      const int row = wm * WM + i * 32 + lrow;
      a_off[i][kk] = row * 128 + (((kk * 2 + lhalf) ^ swz(row)) << 4);
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      const int row = wn * WN + j * 32 + lrow;
      b_off[j][kk] = A_BYTES + row * 128 + (((kk * 2 + lhalf) ^ swz(row)) << 4);
    }
  }
  // Multiplies the tile pair sitting in one LDS stage (compile-time: the stage offset folds into
  // the ds_read instructions' immediate field).  Fragments are read ahead of the MFMA group that
  // uses them: one group ahead when a group is four or more MFMAs (enough to cover the LDS
  // latency), all four groups at the top of the step when a group is only one or two.  After
  // each group, `between(kk)` may slot other work into the instruction stream, and a scheduling
  // fence keeps the compiler from gathering that work in one place.
  auto compute = [&](auto stage_tag, auto&& between) {
    constexpr int SOFF = decltype(stage_tag)::value * STAGE;
    constexpr int NBUF = (MT * NT <= 2) ? 4 : 2;
    // The transposing reads of a tile that direct-to-LDS loads fill are written as inline
    // assembly: through the builtin the compiler cannot tell them from the LDS locations the loads
    // still in flight will write and puts `s_waitcnt vmcnt(0)` in front of the first one, which
    // drains the prefetched tiles in every K step (the stage being read was waited for at the top
    // of the step; the loads in flight fill another one).  The compiler does not know when such a
    // read's result arrives, so the fragments pass through frag_wait() before the first MFMA.
    constexpr bool ASM_TR = BTR && NBUF == 4 && NT == 1;
    bf16x8_t af[NBUF][MT], bfr[NBUF][NT];
    auto read_frags = [&](auto buf_tag, int kk) {
      constexpr int BUF = decltype(buf_tag)::value % NBUF;
      typedef short s16x4_t __attribute__((ext_vector_type(4)));
      typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
#pragma unroll
      for (int i = 0; i < MT; ++i) {
        if constexpr (TRA) {
          union { s16x4_t h[2]; bf16x8_t f; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + at_off[i][kk][0] + SOFF));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + at_off[i][kk][1] + SOFF));
          af[BUF][i] = u.f;
        } else {
          af[BUF][i] = *reinterpret_cast<const bf16x8_t*>(lds + a_off[i][kk] + SOFF);
        }
      }
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if constexpr (ASM_TR) {
          union { s16x4_t h[2]; bf16x8_t f; } u;
          const uint32_t a0 = (uint32_t)(uintptr_t)(lds_s16x4_ptr)(lds + bt_off[j][kk][0]);
          const uint32_t a1 = (uint32_t)(uintptr_t)(lds_s16x4_ptr)(lds + bt_off[j][kk][1]);
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(u.h[0]) : "v"(a0), "n"(SOFF) : "memory");
          asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(u.h[1]) : "v"(a1), "n"(SOFF) : "memory");
          bfr[BUF][j] = u.f;
        } else if constexpr (TRB) {
          union { s16x4_t h[2]; bf16x8_t f; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][0] + SOFF));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][1] + SOFF));
          bfr[BUF][j] = u.f;
        } else {
          bfr[BUF][j] = *reinterpret_cast<const bf16x8_t*>(lds + b_off[j][kk] + SOFF);
        }
      }
    };
    // all LDS reads issued so far have arrived; the fragments are operands of the statement so that
    // no MFMA that uses them can be scheduled ahead of it
    auto frag_wait = [&]() {
      if constexpr (ASM_TR) {
        asm volatile("s_waitcnt lgkmcnt(0)"
                     : "+v"(bfr[0][0]), "+v"(bfr[1][0]), "+v"(bfr[2][0]), "+v"(bfr[3][0])
                     :
                     : "memory");
      }
    };
    auto mfmas = [&](auto buf_tag) {
      constexpr int BUF = decltype(buf_tag)::value % NBUF;
      if constexpr (TWO_ACC && (decltype(buf_tag)::value & 1)) {
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[BUF][0], bfr[BUF][0], acc2, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[BUF][i], bfr[BUF][j], acc[i][j], 0, 0, 0);
      }
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, 2> I2;
    typedef std::integral_constant<int, 3> I3;
    static_assert(BK == 64, "four MFMA groups per K step");
    __builtin_amdgcn_s_setprio(1);
    if constexpr (NBUF == 4) {
      read_frags(I0(), 0); read_frags(I1(), 1); read_frags(I2(), 2); read_frags(I3(), 3);
      frag_wait();
      mfmas(I0()); between(I0()); __builtin_amdgcn_sched_barrier(0);
      mfmas(I1()); between(I1()); __builtin_amdgcn_sched_barrier(0);
      mfmas(I2()); between(I2()); __builtin_amdgcn_sched_barrier(0);
      mfmas(I3()); between(I3());
    } else {
      read_frags(I0(), 0);
      read_frags(I1(), 1); mfmas(I0()); between(I0()); __builtin_amdgcn_sched_barrier(0);
      read_frags(I2(), 2); mfmas(I1()); between(I1()); __builtin_amdgcn_sched_barrier(0);
      read_frags(I3(), 3); mfmas(I2()); between(I2()); __builtin_amdgcn_sched_barrier(0);
      mfmas(I3()); between(I3());
    }
    __builtin_amdgcn_s_setprio(0);
  };
  // One K step = barrier, then, interleaved, (a) park the NEXT tile pair (already in registers) in
  // the other LDS stage, refilling each register with a later tile as soon as it is free, and (b)
  // multiply the current stage.  The barrier at the top
  // guarantees both that everybody has finished reading the stage (a) overwrites (it was multiplied
  // in the previous step) and that everybody's writes to the current stage have landed.
  // The K loop below runs in pairs of steps (one per LDS stage) with no conditional code around
  // the multiplications: the unmasked fast path therefore wants an even number of K steps; the
  // masked path rounds an odd count up, the extra step multiplying a tile the masks turn to zeros.
  const bool fast = (m0 + BM <= p.M) && (n0 + BN <= p.N) && (p.K % (2 * BK) == 0) && !p.wide;
  const int nk2 = (nk + 1) & ~1;
  auto stash = [&](auto stage_tag, auto set_tag, auto fast_tag, int kt) {  // registers (tile kt) -> LDS stage
    constexpr int SOFF = decltype(stage_tag)::value * STAGE;
    constexpr int SET = decltype(set_tag)::value;
    constexpr bool F = decltype(fast_tag)::value;
    if (F) { la.store_fast(lds + SOFF, va[SET]); lb.store_fast(lds + SOFF + A_BYTES, vb[SET]); }
    else { la.store(lds + SOFF, kt * BK, va[SET]); lb.store(lds + SOFF + A_BYTES, kt * BK, vb[SET]); }
    add_colsum(kt * BK, vb[SET]);
  };
  auto fetch = [&](auto set_tag, auto fast_tag, int kt) {                  // global tile kt -> registers
    constexpr int SET = decltype(set_tag)::value;
    constexpr bool F = decltype(fast_tag)::value;
    if (F) { la.load_fast(kt * BK, va[SET]); lb.load_fast(kt * BK, vb[SET]); }
    else { la.load(kt * BK, va[SET]); lb.load(kt * BK, vb[SET]); }
  };
  typedef std::integral_constant<int, 0> S0;
  typedef std::integral_constant<int, 1> S1;
  // set_tag: the register set of tile kt + 1 (parked now, then refilled with tile kt + 1 + PF).
  // Nothing in a step is conditional: past the end the last tile is fetched again and never
  // used.  With a branch around the loads the compiler could no longer tell how many are still
  // in flight at the next wait and would drain them all, which serialises the pipeline.
  // Register-staged loop with wavefront tiles of four or more MFMAs per group (XPIPE): the K steps
  // overlap.  A step's barrier sits in front of its LAST MFMA group instead of in front of its
  // first: by then this wavefront has parked its whole share of the next tile, so after the
  // barrier the next tile is complete in LDS, the fragments of the next step's first group are
  // requested at once, and the last group's MFMAs run while they travel.  (With the barrier at the
  // top of a step the first group waited for an LDS round trip with an idle matrix pipeline.)  The
  // two fragment buffers therefore live across steps: on entry to a step buffer 0 holds group 0.
  constexpr bool XPIPE = !DMA && (MT * NT >= 4);
  bf16x8_t xa[2][MT], xb[2][NT];
  auto xread = [&](auto buf_tag, int kk, auto stage_tag) {
    constexpr int BUF = decltype(buf_tag)::value, SOFF = decltype(stage_tag)::value * STAGE;
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
#pragma unroll
    for (int i = 0; i < MT; ++i) {
      if constexpr (TRA) {
        union { s16x4_t h[2]; bf16x8_t f; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + at_off[i][kk][0] + SOFF));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + at_off[i][kk][1] + SOFF));
        xa[BUF][i] = u.f;
      } else {
        xa[BUF][i] = *reinterpret_cast<const bf16x8_t*>(lds + a_off[i][kk] + SOFF);
      }
    }
#pragma unroll
    for (int j = 0; j < NT; ++j) {
      if constexpr (TRB) {
        union { s16x4_t h[2]; bf16x8_t f; } u;
        u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][0] + SOFF));
        u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][1] + SOFF));
        xb[BUF][j] = u.f;
      } else {
        xb[BUF][j] = *reinterpret_cast<const bf16x8_t*>(lds + b_off[j][kk] + SOFF);
      }
    }
  };
  auto xmm = [&](auto buf_tag) {
    constexpr int BUF = decltype(buf_tag)::value;
#pragma unroll
    for (int i = 0; i < MT; ++i)
#pragma unroll
      for (int j = 0; j < NT; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(xa[BUF][i], xb[BUF][j], acc[i][j], 0, 0, 0);
  };
  typedef std::integral_constant<int, 0> B0;
  typedef std::integral_constant<int, 1> B1;
  // before the first step: tile 0 is parked, wait for everybody's share and fetch group 0
  auto xprime = [&]() {
    if constexpr (XPIPE) {
      __syncthreads();
      xread(B0(), 0, S0());
    }
  };
  auto step = [&](auto cur_tag, auto nxt_tag, auto set_tag, auto fast_tag, int kt) {
    constexpr int SN = decltype(nxt_tag)::value * STAGE;
    constexpr int SET = decltype(set_tag)::value;
    constexpr bool F = decltype(fast_tag)::value;
    const int k_st = (kt + 1) * BK, k_ld = min(kt + 1 + PF, nk - 1) * BK;
    const int64_t koff_a = la.k_offset(k_ld), koff_b = lb.k_offset(k_ld);
    auto between = [&](auto q_tag) {
      constexpr int Q = decltype(q_tag)::value;
      la.template roll<Q, F>(lds + SN, k_st, k_ld, koff_a, va[SET]);
      lb.template roll<Q, F>(lds + SN + A_BYTES, k_st, k_ld, koff_b, vb[SET]);
    };
    if constexpr (XPIPE) {
      typedef std::integral_constant<int, 0> Q0;
      typedef std::integral_constant<int, 1> Q1;
      typedef std::integral_constant<int, 2> Q2;
      typedef std::integral_constant<int, 3> Q3;
      add_colsum(k_st, vb[SET]);
      __builtin_amdgcn_s_setprio(1);
      xread(B1(), 1, cur_tag); xmm(B0()); between(Q0()); __builtin_amdgcn_sched_barrier(0);
      xread(B0(), 2, cur_tag); xmm(B1()); between(Q1()); __builtin_amdgcn_sched_barrier(0);
      xread(B1(), 3, cur_tag); xmm(B0()); between(Q2()); __builtin_amdgcn_sched_barrier(0);
      between(Q3());
      __syncthreads();             // everybody's share of the next tile is in LDS; this stage is read out
      xread(B0(), 0, nxt_tag);
      xmm(B1());
      __builtin_amdgcn_s_setprio(0);
    } else {
      __syncthreads();
      add_colsum(k_st, vb[SET]);
      compute(cur_tag, between);
    }
  };
  auto last = [&](auto cur_tag) {
    if constexpr (XPIPE) {
      __builtin_amdgcn_s_setprio(1);
      xread(B1(), 1, cur_tag); xmm(B0());
      xread(B0(), 2, cur_tag); xmm(B1());
      xread(B1(), 3, cur_tag); xmm(B0());
      xmm(B1());
      __builtin_amdgcn_s_setprio(0);
    } else {
      __syncthreads();
      compute(cur_tag, [&](auto) {});
    }
  };
  auto run = [&](auto fast_tag) {
    typedef std::integral_constant<int, 1 % PF> SetOdd;   // tiles with odd index
    fetch(S0(), fast_tag, 0);
    if (PF > 1) fetch(SetOdd(), fast_tag, min(1, nk - 1));
    stash(S0(), S0(), fast_tag, 0);
    fetch(S0(), fast_tag, min(PF, nk - 1));
    xprime();
    int kt = 0;
    for (; kt + 2 < nk2; kt += 2) {
      step(S0(), S1(), SetOdd(), fast_tag, kt);
      step(S1(), S0(), S0(), fast_tag, kt + 1);
    }
    step(S0(), S1(), SetOdd(), fast_tag, kt);
    last(S1());
  };
  // A reduction whose length is not a multiple of 128 (weight gradients reduce over the batch's
  // tokens) on a tile that lies inside M and N: the unmasked steps for as long as the tile being
  // parked and the tile being fetched lie wholly inside K, the masked ones (per-load bounds, zero
  // fill) only for the last few.  Both kinds keep tiles in the same registers and LDS layout.
  // (Measured on 2048 x 512 x 3969: all steps masked 57.5 us, K = 4096 unmasked 46.3 us.)
  auto run_mixed = [&]() {
    typedef std::integral_constant<int, 1 % PF> SetOdd;
    const int nfull = p.K / BK;                         // tiles 0 .. nfull - 1 are whole
    fetch(S0(), std::true_type(), 0);
    if (PF > 1) fetch(SetOdd(), std::true_type(), 1);
    stash(S0(), S0(), std::true_type(), 0);
    fetch(S0(), std::true_type(), PF);
    xprime();
    int kt = 0;
    for (; kt + 2 < nk2 && kt + 2 + PF < nfull; kt += 2) {   // step kt + 1 parks tile kt + 2 and fetches tile kt + 2 + PF
      step(S0(), S1(), SetOdd(), std::true_type(), kt);
      step(S1(), S0(), S0(), std::true_type(), kt + 1);
    }
    for (; kt + 2 < nk2; kt += 2) {
      step(S0(), S1(), SetOdd(), std::false_type(), kt);
      step(S1(), S0(), S0(), std::false_type(), kt + 1);
    }
    step(S0(), S1(), SetOdd(), std::false_type(), kt);
    last(S1());
  };
  // DMA: at the top of step kt this wavefront waits until all but the loads of the DMA - 2 newest
  // tiles have landed (its part of tile kt is then in LDS), and the barrier extends that to the
  // whole workgroup and tells that everybody has finished multiplying stage (kt - 1) % DMA, which is
  // refilled with tile kt + DMA - 1 in four portions between the MFMA groups.  Every step issues
  // the same number of loads (past the end the last tile is fetched again into a stage nobody
  // reads), so the count in the wait is a constant.
  auto run_dma = [&]() {
    constexpr int LPW = NIA + NIB;               // loads per wavefront per tile
    constexpr int KEEP = (DMA - 2) * LPW;        // loads that may stay in flight at the top of a step
    for (int t = 0; t < DMA - 1; ++t)
      for (int q = 0; q < 4; ++q) dma_issue(t * STAGE, min(t, nk - 1), dma_kb(min(t, nk - 1)), q);
    // The stage of a step (kt % DMA) is a compile-time constant: the loop body is written out once
    // per stage, so that every LDS address in it is a register plus an immediate offset.
    constexpr int NS = DMA ? DMA : 1;
    auto one = [&](auto st_tag, int kt) {
      constexpr int ST = decltype(st_tag)::value;
      constexpr int ST_NEW = (ST + NS - 1) % NS;     // (kt + DMA - 1) % DMA
      wait_vmcnt<(KEEP > 0 ? KEEP : 0)>();
      __builtin_amdgcn_s_barrier();
      const int kt_new = min(kt + DMA - 1, nk - 1);
      const int64_t kb_new = dma_kb(kt_new);
      compute(st_tag, [&](auto q_tag) { dma_issue(ST_NEW * STAGE, kt_new, kb_new, decltype(q_tag)::value); });
    };
    int kt = 0;
    for (; kt + NS <= nk; kt += NS)
      static_for<0, NS>([&](auto s_tag) { one(s_tag, kt + decltype(s_tag)::value); });
    static_for<0, NS>([&](auto s_tag) {
      if (kt + decltype(s_tag)::value < nk) one(s_tag, kt + decltype(s_tag)::value);
    });
    wait_vmcnt<0>();   // the re-fetched tiles have landed before LDS is reused
  };
  // The same tiles, stages and loads as run_dma, but the fragment reads run D MFMA groups ahead of
  // the multiplications ACROSS K steps: while the last groups of tile kt multiply, the first
  // fragments of tile kt + 1 are already on their way from LDS.  The step's wait-and-barrier (tile
  // kt + 1 has landed for everybody; everybody has issued its last reads of tile kt - 1's stage,
  // which this step's loads refill) therefore sits in front of group 4 - D, not in front of an LDS
  // round trip with an idle matrix pipeline.  D = 1 when a group is four or more MFMAs, 3 when it
  // is one or two (an LDS read takes longer than two MFMAs).  A wavefront tile of 32 x 32 has one
  // accumulator; its four MFMAs of a K step would form one dependent chain (an MFMA can issue every
  // 8 passes but its result is ready after 16), so even and odd groups go to two accumulators that
  // are added at the end.
  auto run_dma_pipe = [&]() {
    static_assert(!PIPE || DMA >= 3, "the pipelined loop needs three or more LDS stages");
    constexpr int S = PIPE ? DMA : 3;                 // (the body is compiled for every configuration)
    constexpr int LPW = NIA + NIB;
    constexpr int D = (MT * NT >= 4) ? 1 : 3;
    constexpr int NB = D + 1;
    constexpr int GW = 4 - D;                         // first group whose look-ahead reads the next tile
    constexpr int PER = LPW / 4, REM = LPW % 4;       // loads per quarter: PER (+1 for the first REM quarters)
    constexpr int ISSUED = GW * PER + (GW < REM ? GW : REM);   // issued in quarters 0 .. GW-1 of this step
    constexpr int KEEP = (S - 3) * LPW + ISSUED;      // may stay in flight when tile kt + 1 is needed
    constexpr bool TWO = TWO_ACC;
    constexpr int RPG = MT + NT * (TRB ? 2 : 1);      // LDS read instructions per group
    bf16x8_t af[NB][MT], bfr[NB][NT];
    typedef short s16x4_t __attribute__((ext_vector_type(4)));
    typedef __attribute__((address_space(3))) s16x4_t* lds_s16x4_ptr;
    auto rd = [&](auto buf_tag, int kk, int soff) {
      constexpr int BUF = decltype(buf_tag)::value;
#pragma unroll
      for (int i = 0; i < MT; ++i) af[BUF][i] = *reinterpret_cast<const bf16x8_t*>(lds + a_off[i][kk] + soff);
#pragma unroll
      for (int j = 0; j < NT; ++j) {
        if constexpr (TRB) {
          union { s16x4_t h[2]; bf16x8_t f; } u;
          u.h[0] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][0] + soff));
          u.h[1] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_ptr)(lds + bt_off[j][kk][1] + soff));
          bfr[BUF][j] = u.f;
        } else {
          bfr[BUF][j] = *reinterpret_cast<const bf16x8_t*>(lds + b_off[j][kk] + soff);
        }
      }
    };
    auto mm_ = [&](auto buf_tag, auto g_tag) {
      constexpr int BUF = decltype(buf_tag)::value;
      if constexpr (TWO && (decltype(g_tag)::value & 1)) {
        acc2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[BUF][0], bfr[BUF][0], acc2, 0, 0, 0);
      } else {
#pragma unroll
        for (int i = 0; i < MT; ++i)
#pragma unroll
          for (int j = 0; j < NT; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[BUF][i], bfr[BUF][j], acc[i][j], 0, 0, 0);
      }
    };
    for (int t = 0; t < S - 1; ++t)
      for (int q = 0; q < 4; ++q) dma_issue(t * STAGE, min(t, nk - 1), dma_kb(min(t, nk - 1)), q);
    wait_vmcnt<(S - 2) * LPW>();
    __builtin_amdgcn_s_barrier();
    static_for<0, D>([&](auto g) { rd(g, decltype(g)::value, 0); });
    __builtin_amdgcn_s_setprio(1);
    // one K step with its stage (kt % S) known at compile time, see run_dma
    auto one = [&](auto st_tag, int kt) {
      constexpr int ST = decltype(st_tag)::value;
      constexpr int ST_NEXT = (ST + 1) % S;
      constexpr int ST_NEW = (ST + S - 1) % S;        // (kt + S - 1) % S: held tile kt - 1
      const int kt_new = min(kt + S - 1, nk - 1);
      const int64_t kb_new = dma_kb(kt_new);
      static_for<0, 4>([&](auto g_tag) {
        constexpr int G = decltype(g_tag)::value;
        constexpr int T = G + D;                      // the group whose fragments are read now
        if constexpr (T == 4) {
          wait_vmcnt<KEEP>();
          // this wavefront's fragment reads of the stage about to be refilled are done (only the
          // reads issued one group ago, which belong to a newer stage, may still be in flight)
          __builtin_amdgcn_s_waitcnt(0xC07F | ((RPG < 15 ? RPG : 15) << 8));
          __builtin_amdgcn_s_barrier();
        }
        if constexpr (T < 4) rd(std::integral_constant<int, T % NB>(), T, ST * STAGE);
        else rd(std::integral_constant<int, T % NB>(), T - 4, ST_NEXT * STAGE);
        mm_(std::integral_constant<int, G % NB>(), g_tag);
        dma_issue(ST_NEW * STAGE, kt_new, kb_new, G);
        __builtin_amdgcn_sched_barrier(0);
      });
    };
    int kt = 0;
    for (; kt + S <= nk; kt += S)
      static_for<0, S>([&](auto s_tag) { one(s_tag, kt + decltype(s_tag)::value); });
    static_for<0, S>([&](auto s_tag) {
      if (kt + decltype(s_tag)::value < nk) one(s_tag, kt + decltype(s_tag)::value);
    });
    __builtin_amdgcn_s_setprio(0);
    wait_vmcnt<0>();   // the re-fetched tiles have landed before LDS is reused
  };
  if constexpr (DMA && PIPE) run_dma_pipe();
  else if constexpr (DMA) run_dma();
  else {
    const bool inside = (m0 + BM <= p.M) && (n0 + BN <= p.N) && !p.wide;
    if (fast) run(std::true_type());
    else if (CS && inside && p.K / BK > PF + 3) run_mixed();
    else run(std::false_type());
  }
  if constexpr (TWO_ACC) {
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[0][0][r] += acc2[r];
  }
  __syncthreads();

  if (CS_ON) {
    if (do_cs) {  // uniform over the workgroup; LDS is free after the loop's last barrier
      constexpr int NCG = BN / 8, NKG = 256 / NCG;   // column groups, threads per column group
      float* red = reinterpret_cast<float*>(lds);    // [NKG][BN]
      const int cg = tid % NCG, kg = tid / NCG;
#pragma unroll
      for (int e = 0; e < 8; ++e) red[kg * BN + cg * 8 + e] = cs[e];
      __syncthreads();
      if (tid < BN) {
        const int n = n0 + tid;
        if (n < p.N) {
          float t = 0.f;
#pragma unroll
          for (int g = 0; g < NKG; ++g) t += red[g * BN + tid];
          int64_t idx = n;
          if (p.c_split) { const int sg = n / p.c_split; idx = (int64_t)sg * p.c_seg_stride + (n - sg * p.c_split); }
          p.colsum_dst[idx] = p.colsum_overwrite ? t : p.colsum_dst[idx] + t;
        }
      }
    }
  }

  // Epilogue.  In the accumulator a lane holds one column (lane % 32) and rows
  // 8*(r/4) + 4*(lane/32) + r%4 of each 32x32 tile: storing from there would write 2- or 4-byte
  // pieces.  Each wavefront instead passes 32 rows at a time through its own LDS patch and then
  // handles 8 consecutive columns of one row per lane: bias, mask and residual are 16/32-byte
  // loads and the result leaves as one 16-byte (bf16) or two 16-byte (fp32) stores.
  constexpr int PW = WN + 4;                       // patch row stride in floats
  float* patch = reinterpret_cast<float*>(lds) + wave * 32 * PW;   // (the loop's last barrier has passed)
  static_assert(4 * 32 * PW * 4 <= 2 * STAGE, "epilogue patch fits the tile buffers");
  if (CS_ON) __syncthreads();                      // the column-sum scratch above used the same memory
#pragma unroll
  for (int i = 0; i < MT; ++i) {
#pragma unroll
    for (int j = 0; j < NT; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        patch[(8 * (r >> 2) + 4 * lhalf + (r & 3)) * PW + j * 32 + lrow] = acc[i][j][r];
    __syncthreads();
#pragma unroll
    for (int it = 0; it < WN / 16; ++it) {
      const int q = lane + 64 * it;
      const int row = q / (WN / 8), c8 = q % (WN / 8);
      const int m = m0 + wm * WM + i * 32 + row;
      const int n = n0 + wn * WN + c8 * 8;
      if (m < p.M && n < p.N) {
        const float4 lo = *reinterpret_cast<const float4*>(patch + row * PW + c8 * 8);
        const float4 hi = *reinterpret_cast<const float4*>(patch + row * PW + c8 * 8 + 4);
        float v[8] = {lo.x, lo.y, lo.z, lo.w, hi.x, hi.y, hi.z, hi.w};
        if (p.bias) {
          const float* bp = p.bias + n;
          if (p.bias_split) { const int sg = n / p.bias_split; bp = p.bias + (int64_t)sg * p.bias_seg_stride + (n - sg * p.bias_split); }
          const float4 b0 = *reinterpret_cast<const float4*>(bp), b1 = *reinterpret_cast<const float4*>(bp + 4);
          v[0] += b0.x; v[1] += b0.y; v[2] += b0.z; v[3] += b0.w; v[4] += b1.x; v[5] += b1.y; v[6] += b1.z; v[7] += b1.w;
        }
        if (p.relu) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] = fmaxf(v[e], 0.f);
        }
        if (p.relu_mask) {
          const uint4 mk = *reinterpret_cast<const uint4*>((const bf16_t*)p.relu_mask + (int64_t)m * p.ldm + n);
          const uint32_t* mw = &mk.x;
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            if (!(__uint_as_float(mw[e] << 16) > 0.f)) v[2 * e] = 0.f;
            if (!(__uint_as_float(mw[e] & 0xffff0000u) > 0.f)) v[2 * e + 1] = 0.f;
          }
        }
        int64_t cbase = n;
        if (p.c_split) { const int sg = n / p.c_split; cbase = (int64_t)sg * p.c_seg_stride + (n - sg * p.c_split); }
        if (p.residual) {
          const float* rp = p.residual + cbase + (int64_t)m * p.ldr;
          const float4 r0 = *reinterpret_cast<const float4*>(rp), r1 = *reinterpret_cast<const float4*>(rp + 4);
          v[0] += r0.x; v[1] += r0.y; v[2] += r0.z; v[3] += r0.w; v[4] += r1.x; v[5] += r1.y; v[6] += r1.z; v[7] += r1.w;
        }
        const int64_t off = cbase + (int64_t)m * p.ldc;
        if (p.out_f32) {
          float* cp = (float*)p.C + off;
          *reinterpret_cast<float4*>(cp) = make_float4(v[0], v[1], v[2], v[3]);
          *reinterpret_cast<float4*>(cp + 4) = make_float4(v[4], v[5], v[6], v[7]);
        } else {
          uint4 o;
          o.x = pack2_bf16(v[0], v[1]);
          o.y = pack2_bf16(v[2], v[3]);
          o.z = pack2_bf16(v[4], v[5]);
          o.w = pack2_bf16(v[6], v[7]);
          *reinterpret_cast<uint4*>((bf16_t*)p.C + off) = o;
        }
      }
    }
    __syncthreads();
  }
}

// Workgroups are handed to the 8 XCDs round-robin by linear id, and each XCD has its own L2.
// remap_xcd() renumbers them so that the workgroups one XCD runs one after the other are
// consecutive logical tiles: neighbours that share an operand tile then share it through one L2
// instead of each XCD fetching its own copy.
__device__ __forceinline__ int remap_xcd(int bid, int total) {
  const int q = total >> 3, r = total & 7, x = bid & 7;
  return x * q + (x < r ? x : r) + (bid >> 3);
}

// Logical tile number -> tile coordinates.  The tiles an XCD runs at the same time are consecutive
// numbers (remap_xcd), a few dozen of them; they should share few operand panels, and the panels
// they share with the tiles that follow should still be in that XCD's L2 (4 MB).  So the output is
// walked in bands of TILE_BAND tile rows (or columns, along the axis with fewer tiles), within a
// band across the other axis, within that band-wide step along the band: 64 consecutive tiles
// cover 8 x 8 tiles, their 8 + 8 panels of K = 512 are 2 MB, and going on along the band keeps
// the band's panels while the other operand streams through once per band.  (Walking the whole
// short axis first, as an earlier version did, makes each XCD pull all of the smaller operand
// through its L2 for every two panels of the larger one: 714 MB read for the generator's 36 MB.)
constexpr int TILE_BAND = 8;
// (This runs in front of a workgroup's first load, and the GPU has no integer divide instruction:
// the band is found by subtraction when there are few, and a full band's split is a shift.)
__device__ __forceinline__ void tile_of(int L, int tiles_m, int tiles_n, int& tm, int& tn) {
  const bool along_m = tiles_m <= tiles_n;             // bands lie along the axis with more tiles
  const unsigned ts = along_m ? tiles_m : tiles_n, tl = along_m ? tiles_n : tiles_m;
  const unsigned per_band = TILE_BAND * tl;
  unsigned band = 0, r = (unsigned)L;
  if (ts <= 16 * TILE_BAND) {
    while (r >= per_band) { r -= per_band; ++band; }
  } else {
    band = r / per_band;
    r -= band * per_band;
  }
  const unsigned h = min((unsigned)TILE_BAND, ts - band * TILE_BAND);  // the last band may be lower
  unsigned s, l;
  static_assert(TILE_BAND == 8, "shift below");
  if (h == TILE_BAND) { s = r & (TILE_BAND - 1); l = r >> 3; }
  else { l = r / h; s = r - l * h; }
  s += band * TILE_BAND;
  tm = (int)(along_m ? s : l);
  tn = (int)(along_m ? l : s);
}

// For a launch of many tiles with long K: XCD x takes the groups of GROUPED_COHORT consecutive
// logical tiles numbered x, x + 8, x + 16, ...  An XCD (32 compute units, two workgroups each) runs
// one such group at a time, and tiles running at the same time share operand panels through its
// L2, so a product whose tiles fill one group exactly is read from HBM once.  The tail that does
// not fill a round of eight groups is split into eight contiguous ranges.
constexpr int GROUPED_COHORT = 64;
__device__ __forceinline__ int remap_cohort(int bid, int total) {
  const int full = total & ~(8 * GROUPED_COHORT - 1);
  if (bid < full) {
    const int x = bid & 7, i = bid >> 3;
    return ((i / GROUPED_COHORT) * 8 + x) * GROUPED_COHORT + i % GROUPED_COHORT;
  }
  return full + remap_xcd(bid - full, total - full);
}

template <int BM, int BN, int WM, int WN, bool KCA, bool KCB, int PF, int DMA, bool PIPE = false>
__global__ void __launch_bounds__(256) gemm_mfma_kernel(const GemmParams p_in) {
  extern __shared__ __align__(16) unsigned char lds[];
  // (kernarg_block: one group of scalar loads for all fields.  The grid size is recomputed from
  // the shape for the same reason: gridDim sits in the implicit arguments, another cache line away.)
  GemmParams p = kernarg_block<GemmParams>();
  (void)p_in;
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  int L = remap_xcd(blockIdx.x, tiles_m * tiles_n * (p.k_splits > 1 ? p.k_splits : 1));
  if (p.k_splits > 1) {   // this workgroup's share of K: shift the operands, shorten K, pick the part
    const int ks = L / (tiles_m * tiles_n);
    L -= ks * tiles_m * tiles_n;
    const int k0 = ks * p.k_chunk;
    p.A = (const bf16_t*)p.A + (KCA ? (int64_t)k0 : (int64_t)k0 * p.lda);
    p.B = (const bf16_t*)p.B + (KCB ? (int64_t)k0 : (int64_t)k0 * p.ldb);
    p.K = min(p.k_chunk, p.K - k0);
    p.C = (float*)p.C + (int64_t)ks * p.c_part_stride;
    if (ks > 0) { p.bias = nullptr; p.residual = nullptr; }
  }
  int tm, tn;
  tile_of(L, tiles_m, tiles_n, tm, tn);
  gemm_mfma_tile<BM, BN, WM, WN, KCA, KCB, PF, false, DMA, PIPE>(p, tm * BM, tn * BN, lds);
}

// Many independent problems of one layout in one launch: workgroup -> (problem, tile) through a
// prefix table of tile counts.  Used for the weight-gradient products of a whole step, each of
// which alone has too few output tiles to fill 256 compute units.
template <int BM, int BN, int WM, int WN, bool KCA, bool KCB, int PF>
__global__ void __launch_bounds__(256, (BM * BN <= 128 * 128) ? 2 : 1) gemm_mfma_grouped_kernel(const GemmParams* __restrict__ table,
                                                                const int32_t* __restrict__ tile_start,
                                                                int n_problems) {
  extern __shared__ __align__(16) unsigned char lds[];
  // Which problem this workgroup's tile belongs to: every thread compares the tile number with a
  // few entries of the (ascending) table of first tiles, and the count of entries that do not
  // exceed it, less one, is the problem - one memory round trip for the whole workgroup; then the
  // problem's parameter block is fetched a word per thread, a second one.  (A binary search by
  // one thread was seven or more dependent round trips in front of every tile.)
  __shared__ GemmParams prm;
  __shared__ int local_tile, n_below;
  const int t = remap_cohort(blockIdx.x, gridDim.x);
  if (threadIdx.x == 0) n_below = 0;
  __syncthreads();
  {
    int cnt = 0;
    for (int i = threadIdx.x; i < n_problems; i += blockDim.x) cnt += (tile_start[i] <= t) ? 1 : 0;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
    if ((threadIdx.x & 63) == 0 && cnt) atomicAdd(&n_below, cnt);
  }
  __syncthreads();
  {
    const int lo = n_below - 1;                  // tile_start[0] = 0, so there is at least one
    constexpr int NW = (int)(sizeof(GemmParams) / 4);
    static_assert(sizeof(GemmParams) % 4 == 0 && NW <= 256, "a word per thread");
    if ((int)threadIdx.x < NW)
      reinterpret_cast<uint32_t*>(&prm)[threadIdx.x] = reinterpret_cast<const uint32_t*>(table + lo)[threadIdx.x];
    if (threadIdx.x == 0) local_tile = t - tile_start[lo];
  }
  __syncthreads();
  const int tiles_n = (prm.N + BN - 1) / BN;
  // consecutive workgroups walk down M first: they share the same columns of B (dY)
  const int tiles_m = (prm.M + BM - 1) / BM;
  const int tm = local_tile % tiles_m, tn = local_tile / tiles_m;
  (void)tiles_n;
  gemm_mfma_tile<BM, BN, WM, WN, KCA, KCB, PF, true>(prm, tm * BM, tn * BN, lds);
}

// Several independent products in one launch, parameter blocks passed by value.
struct GemmMulti {
  GemmParams p[GEMM_MULTI_MAX];
  int32_t tile_start[GEMM_MULTI_MAX + 1];
  int32_t n;
};

template <int BM, int BN, int WM, int WN, bool KCA, bool KCB, int PF, int DMA>
__global__ void __launch_bounds__(256) gemm_mfma_multi_kernel(const GemmMulti mp) {
  extern __shared__ __align__(16) unsigned char lds[];
  const int t = remap_xcd(blockIdx.x, gridDim.x);
  int i = 0;
  while (i + 1 < mp.n && mp.tile_start[i + 1] <= t) ++i;   // uniform over the workgroup
  const GemmParams p = mp.p[i];
  const int L = t - mp.tile_start[i];
  const int tiles_m = (p.M + BM - 1) / BM, tiles_n = (p.N + BN - 1) / BN;
  int tm, tn;
  tile_of(L, tiles_m, tiles_n, tm, tn);
  gemm_mfma_tile<BM, BN, WM, WN, KCA, KCB, PF, false, DMA>(p, tm * BM, tn * BN, lds);
}

// An operand whose extent reaches 2 GiB cannot use the 32-bit per-lane offsets of the fast path.
void set_wide(GemmParams& p) {
  const int64_t lim = (int64_t)1 << 31;
  const int64_t a = (int64_t)(p.transA ? p.K : p.M) * p.lda * 2;
  int64_t b = (int64_t)(p.transB ? p.N : p.K) * p.ldb * 2;
  if (p.b_split) {
    const int64_t nseg = ((p.b_split_on_k ? p.K : p.N) + p.b_split - 1) / p.b_split;
    b = nseg * p.b_seg_stride * 2 + b;
  }
  p.wide = (a >= lim || b >= lim) ? 1 : 0;
}

template <int BM, int BN, int WM, int WN, int PF, int DMA = 0, bool PIPE = false>
void launch_mfma_cfg(hipStream_t st, const GemmParams& p_in, const LaunchEvents& ev = LaunchEvents()) {
  if (DMA && !(p_in.transA == 0 && p_in.K % BK == 0)) {
    launch_mfma_cfg<BM, BN, WM, WN, PF, 0>(st, p_in, ev);
    return;
  }
  GemmParams p = p_in;
  set_wide(p);
  dim3 grid(((p.N + BN - 1) / BN) * ((p.M + BM - 1) / BM) * (p.k_splits > 1 ? p.k_splits : 1));
  constexpr int LDS = (DMA ? DMA : 2) * (BM + BN) * 128;
  const bool kca = !p.transA, kcb = p.transB != 0;
#define MM_GO(KA, KB)                                                                               \
  do {                                                                                              \
    static bool attr_set = false;                                                                   \
    if (!attr_set) {                                                                                \
      hipFuncSetAttribute((const void*)gemm_mfma_kernel<BM, BN, WM, WN, KA, KB, PF, KA ? DMA : 0, KA && PIPE>, \
                          hipFuncAttributeMaxDynamicSharedMemorySize, LDS);                         \
      attr_set = true;                                                                              \
    }                                                                                               \
    hipExtLaunchKernelGGL((gemm_mfma_kernel<BM, BN, WM, WN, KA, KB, PF, KA ? DMA : 0, KA && PIPE>), grid, dim3(256), LDS, st, \
                          ev.start, ev.stop, 0, p);                                                 \
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
  if (p.K <= 0) return false;   // the K pipeline always loads its first tile
  if (p.k_splits > 1 && (!p.out_f32 || p.b_split || p.c_split || p.relu || p.relu_mask || p.k_chunk % BK ||
                         (int64_t)(p.k_splits - 1) * p.k_chunk >= p.K))
    return false;
  if (!aligned16(p.A) || !aligned16(p.B)) return false;
  if (p.lda % 8 || p.ldb % 8) return false;
  if (!p.transA ? p.K % 8 : p.M % 8) return false;       // A's contiguous extent
  if (p.transB ? p.K % 8 : p.N % 8) return false;        // B's contiguous extent
  if (p.b_split && (p.b_split % 8 || p.b_seg_stride % 8)) return false;
  if (p.b_split && p.b_split_on_k && (!p.transB || p.b_split % 64)) return false;  // k segments: whole K steps
  // the epilogue moves 8 columns at a time
  if (p.N % 8 || p.ldc % 8 || !aligned16(p.C)) return false;
  if (p.c_split && (p.c_split % 8 || p.c_seg_stride % 8)) return false;
  if (p.bias && (!aligned16(p.bias) || (p.bias_split && (p.bias_split % 8 || p.bias_seg_stride % 4)))) return false;
  if (p.residual && (!aligned16(p.residual) || p.ldr % 4)) return false;
  if (p.relu_mask && (!aligned16(p.relu_mask) || p.ldm % 8)) return false;
  return true;
}

}  // namespace

bool gemm_can_split_k(Dtype dt, const GemmParams& p) { return dt == BF16 && p.k_splits > 1 && mfma_eligible(p); }

bool gemm_groupable(Dtype dt, const GemmParams& p) {
  return dt == BF16 && p.transA == 1 && p.transB == 0 && mfma_eligible(p);
}

constexpr int MM_GROUPED_PF = 2;   // K steps of global loads in flight in the grouped weight-gradient launch
int gemm_grouped_tiles(const GemmParams& p) { return ((p.M + 127) / 128) * ((p.N + 127) / 128); }

void gemm_prepare_grouped(GemmParams& p) { set_wide(p); }

// Table order for the grouped launch: products whose tile count is a multiple of the group size
// first, then the smaller ones packed into whole groups (first fit, largest first), then the
// groups that stay partly empty, and last the large products that are no multiple of the group
// size - so that as many products as possible start and end on a group boundary
// (see remap_cohort).  The products are independent, so any order gives the same results.
void gemm_grouped_order(const int* tiles, int n, int* order) {
  constexpr int C = GROUPED_COHORT;
  std::vector<int> whole, small, big;
  for (int i = 0; i < n; ++i) (tiles[i] % C == 0 ? whole : tiles[i] < C ? small : big).push_back(i);
  std::stable_sort(small.begin(), small.end(), [&](int a, int b) { return tiles[a] > tiles[b]; });
  std::stable_sort(big.begin(), big.end(), [&](int a, int b) { return tiles[a] < tiles[b]; });
  struct Bin { int fill; std::vector<int> items; };
  std::vector<Bin> bins;
  for (int i : small) {
    size_t b = 0;
    while (b < bins.size() && bins[b].fill + tiles[i] > C) ++b;
    if (b == bins.size()) bins.push_back(Bin{0, {}});
    bins[b].fill += tiles[i];
    bins[b].items.push_back(i);
  }
  int k = 0;
  for (int i : whole) order[k++] = i;
  for (const Bin& b : bins) if (b.fill == C) for (int i : b.items) order[k++] = i;
  for (const Bin& b : bins) if (b.fill != C) for (int i : b.items) order[k++] = i;
  for (int i : big) order[k++] = i;
}

// 128x128 tiles: 256x256 ones (one workgroup per compute unit) were measured slower on the mix of
// products a training step defers, also when only the generator's product used them.
void launch_gemm_grouped_tn(hipStream_t st, const GemmParams* table_dev, const int32_t* tile_start_dev,
                            int n_problems, int total_tiles, const LaunchEvents& ev) {
  if (n_problems <= 0 || total_tiles <= 0) return;
  constexpr int LDS = 2 * (128 + 128) * 128;
  static bool attr_set = false;
  if (!attr_set) {
    hipFuncSetAttribute((const void*)gemm_mfma_grouped_kernel<128, 128, 64, 64, false, false, MM_GROUPED_PF>,
                        hipFuncAttributeMaxDynamicSharedMemorySize, LDS);
    attr_set = true;
  }
  hipExtLaunchKernelGGL((gemm_mfma_grouped_kernel<128, 128, 64, 64, false, false, MM_GROUPED_PF>), dim3(total_tiles), dim3(256), LDS,
                        st, ev.start, ev.stop, 0, table_dev, tile_start_dev, n_problems);
}

template <int BM, int BN, int WM, int WN, int PF, int DMA>
void launch_mfma_multi_cfg(hipStream_t st, const GemmMulti& mp, bool kcb, const LaunchEvents& ev) {
  constexpr int LDS = (DMA ? DMA : 2) * (BM + BN) * 128;
  const dim3 grid(mp.tile_start[mp.n]);
#define MM_GO(KB)                                                                                            \
  do {                                                                                                       \
    static bool attr_set = false;                                                                            \
    if (!attr_set) {                                                                                         \
      hipFuncSetAttribute((const void*)gemm_mfma_multi_kernel<BM, BN, WM, WN, true, KB, PF, DMA>,            \
                          hipFuncAttributeMaxDynamicSharedMemorySize, LDS);                                  \
      attr_set = true;                                                                                       \
    }                                                                                                        \
    hipExtLaunchKernelGGL((gemm_mfma_multi_kernel<BM, BN, WM, WN, true, KB, PF, DMA>), grid, dim3(256), LDS, st, \
                          ev.start, ev.stop, 0, mp);                                                         \
  } while (0)
  if (kcb) MM_GO(true); else MM_GO(false);
#undef MM_GO
}

bool launch_gemm_multi(hipStream_t st, Dtype dt, const GemmParams* ps, int n, const LaunchEvents& ev) {
  if (dt != BF16 || n < 1 || n > GEMM_MULTI_MAX) return false;
  GemmMulti mp;
  std::memset(&mp, 0, sizeof mp);
  long tiles128 = 0;
  bool k64 = true;
  int kmax = 0;
  for (int i = 0; i < n; ++i) {
    const GemmParams& p = ps[i];
    if (p.M <= 0 || p.N <= 0 || p.transA || p.transB != ps[0].transB || p.k_splits > 1 || !mfma_eligible(p)) return false;
    mp.p[i] = p;
    set_wide(mp.p[i]);
    tiles128 += (long)((p.M + 127) / 128) * ((p.N + 127) / 128);
    k64 = k64 && p.K % BK == 0;
    kmax = p.K > kmax ? p.K : kmax;
  }
  mp.n = n;
  const bool big = tiles128 >= 192;   // the rule of launch_gemm, applied to the whole set
  if (!big && !k64) return false;
  const int bm = big ? 128 : 64, bn = big ? 128 : 64;
  for (int i = 0; i < n; ++i)
    mp.tile_start[i + 1] = mp.tile_start[i] + ((ps[i].M + bm - 1) / bm) * ((ps[i].N + bn - 1) / bn);
  const bool kcb = ps[0].transB != 0;
  if (big) {
    if (tiles128 >= 1024 || kmax >= 1024) launch_mfma_multi_cfg<128, 128, 64, 64, 2, 0>(st, mp, kcb, ev);
    else launch_mfma_multi_cfg<128, 128, 64, 64, 1, 0>(st, mp, kcb, ev);
  } else {
    launch_mfma_multi_cfg<64, 64, 32, 32, 1, 3>(st, mp, kcb, ev);
  }
  return true;
}

void launch_gemm_simt(hipStream_t st, Dtype dt, const GemmParams& p, const LaunchEvents& ev) {
  if (p.M <= 0 || p.N <= 0) return;
  dim3 grid((p.N + SB - 1) / SB, (p.M + SB - 1) / SB);
  if (dt == BF16) hipExtLaunchKernelGGL(gemm_simt_kernel<bf16_t>, grid, dim3(256), 0, st, ev.start, ev.stop, 0, p);
  else hipExtLaunchKernelGGL(gemm_simt_kernel<float>, grid, dim3(256), 0, st, ev.start, ev.stop, 0, p);
}

void launch_gemm(hipStream_t st, Dtype dt, const GemmParams& p, const LaunchEvents& ev) {
  if (p.M <= 0 || p.N <= 0) return;
  if (dt == BF16 && mfma_eligible(p)) {
    // Measured on the step's shapes: 128x128 tiles once they fill the chip, with two K steps of
    // loads in flight when there are several rounds of tiles or a long K; otherwise 64x64.
    const long tiles_big = (long)((p.M + 127) / 128) * ((p.N + 127) / 128) * (p.k_splits > 1 ? p.k_splits : 1);
    const long tiles_small = (long)((p.M + 63) / 64) * ((p.N + 63) / 64) * (p.k_splits > 1 ? p.k_splits : 1);
    // A compute unit holds two workgroups of the 128x128 kernels and of the four-stage 64x64 kernel
    // (512 at a time on the chip), three of the three-stage 64x64 kernels (768).  A product with a
    // few tiles more than 512 - a batch of slightly more than 4096 tokens - would run a second,
    // nearly empty round; measured on such shapes the three-stage 64x64 kernels, which take all
    // tiles at once, are faster (K = 512, N = 2048, M = 4160: 21.6 against 24.1 us forward, 20.4
    // against 22.2 us for the input gradient; N = 512, K = 2048: 19.9 against 23.7 us).
    const bool dma_ok = p.transA == 0 && p.K % BK == 0;
    if (tiles_big > 512 && tiles_big <= 576 && dma_ok && p.K <= 512) {
      if (p.transB) launch_mfma_cfg<64, 64, 32, 32, 1, 3, true>(st, p, ev);
      else launch_mfma_cfg<64, 64, 32, 32, 1, 3>(st, p, ev);
    } else if (tiles_big >= 192) {
      if (tiles_big >= 1024 || p.K >= 1024) launch_mfma_cfg<128, 128, 64, 64, 2>(st, p, ev);
      else launch_mfma_cfg<128, 128, 64, 64, 1>(st, p, ev);
    } else if (p.transA == 0 && p.transB != 0 && p.K % BK == 0) {
      // both operands k-contiguous (input-gradient products): direct-to-LDS loads, four stages, the
      // K loop pipelined across K steps (measured 5-8 % faster than the loop below at K >= 1536)
      if (tiles_small > 512 && tiles_small <= 768) launch_mfma_cfg<64, 64, 32, 32, 1, 3, true>(st, p, ev);
      else launch_mfma_cfg<64, 64, 32, 32, 1, 4, true>(st, p, ev);
    } else {
      // (when A is k-contiguous and K is a multiple of 64 this runs the variant with direct-to-LDS
      // loads and three stages)
      launch_mfma_cfg<64, 64, 32, 32, 1, 3>(st, p, ev);
    }
    return;
  }
  launch_gemm_simt(st, dt, p, ev);
}

}  // namespace mm
