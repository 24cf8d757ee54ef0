// Internal launcher interface between the host runtime and the gfx950 kernels.
// Everything here runs on the stream it is given; nothing allocates.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace mm {

typedef uint16_t bf16_t;  // raw bfloat16 bits

enum Dtype { F32 = 0, BF16 = 1 };

__host__ __device__ inline float bf16_to_f32(bf16_t h) {
  union { uint32_t u; float f; } c;
  c.u = (uint32_t)h << 16;
  return c.f;
}
// round to nearest even; NaN stays NaN.  On the device this is gfx950's conversion instruction
// (v_cvt_pk_bf16_f32), which gives the same bits as the integer formula below for every input.
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  const __bf16 b = (__bf16)f;
  return __builtin_bit_cast(bf16_t, b);
#else
  union { uint32_t u; float f; } c;
  c.f = f;
  if ((c.u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)((c.u >> 16) | 0x40);
  c.u += 0x7fffu + ((c.u >> 16) & 1u);
  return (bf16_t)(c.u >> 16);
#endif
}
// two values in one instruction: a in the low half, b in the high half
__device__ inline uint32_t pack2_bf16(float a, float b) {
  typedef float f32x2_t __attribute__((ext_vector_type(2)));
  typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Timing handles for the launch being issued: when set, the launcher attaches them to its kernel
// (hipExtLaunchKernel), so they carry the kernel's own start and stop timestamps and no marker
// has to be queued around it.
struct LaunchEvents { hipEvent_t start = nullptr; hipEvent_t stop = nullptr; };

// ---------------------------------------------------------------------------------------------
// GEMM:  C[M,N] = epilogue( op(A)[M,K] * op(B)[K,N] )
//   transA = 0: A stored [M,K] row-major (lda = row stride); 1: stored [K,M] row-major.
//   transB = 0: B stored [K,N] row-major (ldb);              1: stored [N,K] row-major.
//   A and B hold the context's working dtype (float or bf16); accumulation is fp32.
//   Split operands: the canonical parameter layout keeps Wq, Wk, Wv (and their biases and
//   gradients) as separate tensors a fixed distance apart; a fused QKV product addresses them
//   as one matrix whose N (or K) axis is cut into segments of `*_split` indices, segment s
//   starting `s * *_seg_stride` elements after the base pointer.
// ---------------------------------------------------------------------------------------------
struct GemmParams {
  const void* A; const void* B; void* C;
  int M, N, K;
  int64_t lda, ldb, ldc;
  int transA, transB;
  int b_split;            // 0 = B is one matrix; else segment length along N (or K)
  int b_split_on_k;       // 1: segments along K (used by the fused QKV input-gradient product)
  int64_t b_seg_stride;
  int c_split;            // segments along N for C (and for the residual)
  int64_t c_seg_stride;
  const float* bias;      // [N] fp32 or null; added before relu
  int bias_split;         // segments along N for the bias vector
  int64_t bias_seg_stride;
  int relu;               // max(.,0)
  const void* relu_mask;  // working dtype [M,N], row stride ldm: result *= (mask > 0)
  int64_t ldm;
  const float* residual;  // fp32 [M,N], row stride ldr, same segmentation as C: added last
  int64_t ldr;
  int out_f32;            // 1: C is fp32; 0: C has the working dtype
  int wide;               // set by the launcher: an operand spans 2 GiB or more (32-bit offsets unusable)
  // Split K (a long reduction with too few output tiles to fill the chip): k_splits > 1 workgroups
  // per tile, split s reducing k in [s * k_chunk, (s+1) * k_chunk) into the fp32 partial result
  // C + s * c_part_stride; the consumer adds the parts.  Needs out_f32, no operand segments, and
  // k_chunk a multiple of 64; bias and residual go into part 0 only.
  int k_splits, k_chunk;
  int64_t c_part_stride;
  float* colsum_dst;      // grouped weight-gradient launch only: [N] (segmented like C) += column
                          // sums of B over K, i.e. the bias gradient belonging to this product
  int colsum_overwrite;   // the sums replace colsum_dst instead of being added (first use of a bucket)
};
void launch_gemm(hipStream_t st, Dtype dt, const GemmParams& p, const LaunchEvents& ev = LaunchEvents());
// true if a product with k_splits > 1 set can run that way (otherwise launch it with k_splits = 0)
bool gemm_can_split_k(Dtype dt, const GemmParams& p);
// Weight-gradient products (transA = 1, transB = 0) of a whole step in one launch.  table_dev and
// tile_start_dev are device arrays of n_problems entries; tile_start is the running sum of
// gemm_grouped_tiles() and total_tiles its total.  Every problem must satisfy gemm_groupable().
bool gemm_groupable(Dtype dt, const GemmParams& p);
int gemm_grouped_tiles(const GemmParams& p);
void gemm_prepare_grouped(GemmParams& p);  // call on each table entry before upload
// order[0..n): the table order that lets the most products begin and end on a boundary of the
// groups of tiles one XCD runs at a time; tiles[i] = gemm_grouped_tiles of product i.
void gemm_grouped_order(const int* tiles, int n, int* order);
void launch_gemm_grouped_tn(hipStream_t st, const GemmParams* table_dev, const int32_t* tile_start_dev,
                            int n_problems, int total_tiles, const LaunchEvents& ev = LaunchEvents());
// Up to GEMM_MULTI_MAX independent products of the same kind (transA = 0, same transB, no split K)
// in one launch; the parameter blocks travel as kernel arguments, no table upload.  Returns false
// and launches nothing when the set cannot run that way (fp32 context, mixed layouts, a shape the
// MFMA kernel does not take): the caller then launches the products one by one.
constexpr int GEMM_MULTI_MAX = 8;
bool launch_gemm_multi(hipStream_t st, Dtype dt, const GemmParams* ps, int n, const LaunchEvents& ev = LaunchEvents());
// Same contract, always the plain FMA kernel (cross-check of the MFMA path).
void launch_gemm_simt(hipStream_t st, Dtype dt, const GemmParams& p, const LaunchEvents& ev = LaunchEvents());

// ---------------------------------------------------------------------------------------------
// token bookkeeping
// ---------------------------------------------------------------------------------------------
// flag[0] |= 1 for an id outside [0,V) at a real position, |= 2 for a non-pad id after the end.
void launch_pack_ids(hipStream_t st, const int32_t* src_ids, const int32_t* tgt_ids,
                     const int32_t* lens, const int32_t* cu_s, const int32_t* cu_u, int B,
                     int S_max, int T_max, int V, int32_t* src_tok, int32_t* src_pos,
                     int32_t* dec_tok, int32_t* dec_pos, int32_t* label, int32_t* flag);
// mode 0: key j blocked iff j >= len_k; mode 1: also j > i.  out uint8 [B, Lq, Lk].
void launch_mask_dump(hipStream_t st, const int32_t* cu_q, const int32_t* cu_k, int B, int Lq,
                      int Lk, int mode, uint8_t* out);

// x[row,:] = sqrt_d * E[tok[row],:] + pe[pos[row],:]   (multiply, then add; fp32 out).
// pos null: every row sits at position pos_all.
void launch_embed_fwd(hipStream_t st, Dtype dt, const void* E, const float* pe, const int32_t* tok,
                      const int32_t* pos, float* x, int rows, int d, float sqrt_d, int pos_all = 0);
// keys[i] = (token << 14 | row), sorted ascending, rows entries.  Depends on the token ids only, so
// it can run ahead of the step on another stream.
void launch_sort_tokens(hipStream_t st, const int32_t* tok, int rows, uint32_t* keys);
// bucket[tok,:] += sqrt_d * sum over rows with that token of dx[row,:]; deterministic (fixed
// summation order, no atomics).  partial: scratch float [rows, d].
void launch_embed_grad(hipStream_t st, const uint32_t* keys, const float* dx, float* bucket,
                       float* partial, int rows, int d, float sqrt_d);

// ---------------------------------------------------------------------------------------------
// LayerNorm over the last axis, one row per wavefront
// ---------------------------------------------------------------------------------------------
// x may arrive as x_parts partial sums (x + s * x_part_stride, s < x_parts); they are added here
// and, with x_sum given, the sum is also written there.
void launch_layernorm_fwd(hipStream_t st, Dtype dt, const float* x, const float* gamma,
                          const float* beta, void* y, float* mean, float* rstd, int rows, int d,
                          float eps, const LaunchEvents& ev = LaunchEvents(), int x_parts = 1,
                          int64_t x_part_stride = 0, float* x_sum = nullptr);
// dx_out = dres + LN'(dy);  dxT_out (working dtype, may be null) = same, rounded.
// The column sums for the gain and shift gradients leave as ln_bwd_partial_rows(rows) partial
// rows, partial[p][0][d] (gain) and partial[p][1][d] (shift); launch_ln_reduce_grouped adds them
// into the buckets for many LayerNorms at once.
int ln_bwd_partial_rows(int rows);
// dy may arrive as dy_parts partial sums (dy + s * dy_part_stride, s < dy_parts) that are added here.
void launch_layernorm_bwd(hipStream_t st, Dtype dt, const float* dy, const float* x,
                          const float* mean, const float* rstd, const float* gamma,
                          const float* dres, float* dx_out, void* dxT_out, float* partial,
                          int rows, int d, const LaunchEvents& ev = LaunchEvents(), int dy_parts = 1,
                          int64_t dy_part_stride = 0);
struct LnReduceJob {
  const float* partial; float* dgamma; float* dbeta;
  int32_t n_partial, d, first_block, overwrite;   // first_block: running sum of ceil(2d/64); overwrite: = instead of +=
};
void launch_ln_reduce_grouped(hipStream_t st, const LnReduceJob* jobs_dev, int n_jobs, int total_blocks);

// dst[n] += sum_m Y[m,n] (= with overwrite); Y is fp32 (y_f32=1) or working dtype; dst segmented like GemmParams C.
int colsum_partial_rows(int M);
void launch_colsum(hipStream_t st, Dtype dt, const void* Y, int y_f32, int64_t ldy, int M, int N,
                   float* partial, float* dst, int split, int64_t seg_stride, int overwrite = 0);

// ---------------------------------------------------------------------------------------------
// attention, one (sentence, head) per workgroup; q/k/v/o rows are packed tokens
// ---------------------------------------------------------------------------------------------
struct AttnParams {
  const void* q; const void* k; const void* v; void* o;  // working dtype
  int64_t ldq, ldk, ldv, ldo;                              // row strides (elements)
  float* lse;                                              // [H, rows_q] log-sum-exp of scaled scores
  const int32_t* cu_q; const int32_t* cu_k;                // [B+1] row offsets per sentence
  int B, H, dh, causal, rows_q;
  int max_lq, max_lk;                                      // longest sentence in the batch
  // backward only
  const void* d_o; void* dq; void* dk; void* dv;
  int64_t lddo, lddq, lddk, lddv;
};
size_t attn_lds_bytes(Dtype dt, int dh, int max_lq, int max_lk, bool backward);
void launch_attn_fwd(hipStream_t st, Dtype dt, const AttnParams& p, const LaunchEvents& ev = LaunchEvents());
void launch_attn_bwd(hipStream_t st, Dtype dt, const AttnParams& p, const LaunchEvents& ev = LaunchEvents());

// ---------------------------------------------------------------------------------------------
// label-smoothed cross-entropy over the vocabulary, forward and backward in one pass
//   loss_rows[u] = lse - (1-eps) z[y] - (eps/V) sum_v z[v];  z <- (softmax(z) - q) * scale * ok
//   where ok = (flag[0] == 0).  z has the working dtype, [U, V] with row stride V.
// ---------------------------------------------------------------------------------------------
void launch_ce(hipStream_t st, Dtype dt, void* z, const int32_t* label, float* loss_rows, int U,
               int V, float eps, float scale, const int32_t* flag, const LaunchEvents& ev = LaunchEvents());
// out[0] = (sum of loss_rows) * scale
void launch_sum_scaled(hipStream_t st, const float* v, int n, float scale, float* out, float* host_out = nullptr,
                       const int32_t* flag = nullptr);
// n_bytes (rounded up to whole words; both buffers hold that many) from pinned host memory to device
// memory by a kernel that reads the host memory itself; zero_word (may be null) is cleared as well.
void launch_upload_words(hipStream_t st, const void* src_pinned, void* dst_dev, size_t n_bytes, int32_t* zero_word);

// ---------------------------------------------------------------------------------------------
// Adam over a list of module buckets, one launch
// ---------------------------------------------------------------------------------------------
struct AdamSegment {
  float* theta; float* m; float* v; float* g; bf16_t* w16;  // w16 null in fp32 contexts
  int64_t len;                                               // multiple of 64
  float n_uses, bc1, bc2;                                    // n_j, 1-beta1^t, 1-beta2^t
  float n_uses_alt;                                          // n_j to use instead when *step_flag != 0 (0: leave the segment alone)
  int32_t first_chunk;                                       // running chunk index of this segment
  int32_t keep_g;                                            // leave g as it is (its next use overwrites it)
};
static const int ADAM_CHUNK = 4096;
// step_flag (device, may be null): the word a training step still in flight sets when it finds bad
// ids.  The kernel reads it when it runs: nonzero selects n_uses_alt, the use counts without that
// step, and a segment whose count is then 0 is not touched at all.
void launch_adam(hipStream_t st, const AdamSegment* segs_dev, int n_segs, int total_chunks,
                 float lr, float beta1, float beta2, float eps, const int32_t* step_flag,
                 const LaunchEvents& ev = LaunchEvents());

// ---------------------------------------------------------------------------------------------
// greedy translation: one new query per sentence over cached keys/values; next-token pick
// ---------------------------------------------------------------------------------------------
// o[b, h*dh..] = softmax(q_b K_b^T / sqrt(dh)) V_b.  q row b at q + b*q_stride, o likewise.
// Keys/values: rows of stride ldkv; sentence b owns rows cu[b]..cu[b+1] or, with cu null, rows
// b*seq_rows .. b*seq_rows + len_uniform.  max_len bounds every sentence's key count.
// Head sizes 16, 32, 64 with 16-byte aligned operands; anything else returns false and launches nothing.
bool launch_attn_decode(hipStream_t st, Dtype dt, const void* q, int64_t q_stride, const void* k, const void* v,
                        int64_t ldkv, const int32_t* cu, int64_t seq_rows, int len_uniform, int max_len,
                        void* o, int64_t o_stride, int B, int H, int dh, int rows_per_seq = 1);
// (rows_per_seq, packed keys only: that many consecutive query rows -- the hypotheses of one
// sentence's beam -- share the keys of sentence row / rows_per_seq.)
// Row-wise arg-max of z [B, V] (lowest index among equal entries) for the sentences with
// done[b] == 0: out_ids[b, t] = cur_tok[b] = token, out_len[b] = t+1; EOS sets done[b] and
// adds one to n_done[0].
void launch_greedy_pick(hipStream_t st, Dtype dt, const void* z, int B, int V, int t, int max_new, int eos,
                        int32_t* cur_tok, int32_t* done, int32_t* out_ids, int32_t* out_len, int32_t* n_done);

// Beam search over summed log-probabilities.  Rows r0 = b*beam .. r0+beam-1 of z [B*beam, V] are
// sentence b's hypotheses, best first.  Writes the next beam: score_out, done_out, next_tok (the
// token a row feeds back; 0 for a carried finished hypothesis), parent_out (row of z the new row
// continues), the same two into hist_tok / hist_parent [t][B*beam], and adds one to n_finished[t]
// for every sentence whose new beam is finished throughout.  In and out arrays must differ.
// Order among equal scores: lower hypothesis row, then lower token id.  beam <= BEAM_MAX (8).
bool launch_beam_select(hipStream_t st, Dtype dt, const void* z, int B, int V, int beam, int t, int eos,
                        const float* score_in, const int32_t* done_in, float* score_out, int32_t* done_out,
                        int32_t* next_tok, int32_t* parent_out, int32_t* hist_tok, int32_t* hist_parent,
                        int32_t* n_finished);
// score[r] = 0 where r % beam == 0, -infinity elsewhere
void launch_beam_init(hipStream_t st, float* score, int R, int beam);
// dst[l] row r <- src[l] row parent[r], first `bytes` bytes of each row, for n_layers <= 32 buffers
constexpr int BEAM_LAYERS_MAX = 32;
bool launch_cache_gather(hipStream_t st, const char* const* src, char* const* dst, int n_layers, const int32_t* parent,
                         int R, int64_t row_stride_bytes, int64_t bytes);

// fp32 -> bf16 copy (working weights) and fill
void launch_to_bf16(hipStream_t st, const float* src, bf16_t* dst, int64_t n);
void launch_fill_f32(hipStream_t st, float* dst, int64_t n, float v);
void launch_fill_i32(hipStream_t st, int32_t* dst, int64_t n, int32_t v);


// The parameter block of a kernel whose only argument is one struct T passed by value, fetched
// from the kernel-argument segment by ONE group of scalar loads with one wait.  Left to the
// compiler the fields are fetched where they are first used, a scalar-cache round trip (about
// 0.2 us) at a time, several of them one after another in front of a workgroup's first load.
// Whole 64-byte pieces are read: up to 60 bytes past T, which lie in the implicit arguments that
// follow the explicit ones in the segment.
template <typename T>
__device__ __forceinline__ T kernarg_block() {
  static_assert(sizeof(T) % 4 == 0 && sizeof(T) <= 256, "one to four 16-dword loads");
#if defined(__HIP_DEVICE_COMPILE__)
  typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
  constexpr int NW = (int)(sizeof(T) / 4), NC = (NW + 15) / 16;
  const auto ka = __builtin_amdgcn_kernarg_segment_ptr();
  u32x16 c[4];
  if constexpr (NC == 1) {
    asm volatile("s_load_dwordx16 %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(c[0]) : "s"(ka) : "memory");
  } else if constexpr (NC == 2) {
    asm volatile("s_load_dwordx16 %0, %2, 0x0\n\ts_load_dwordx16 %1, %2, 0x40\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(c[0]), "=&s"(c[1]) : "s"(ka) : "memory");
  } else if constexpr (NC == 3) {
    asm volatile("s_load_dwordx16 %0, %3, 0x0\n\ts_load_dwordx16 %1, %3, 0x40\n\ts_load_dwordx16 %2, %3, 0x80\n\t"
                 "s_waitcnt lgkmcnt(0)"
                 : "=&s"(c[0]), "=&s"(c[1]), "=&s"(c[2]) : "s"(ka) : "memory");
  } else {
    asm volatile("s_load_dwordx16 %0, %4, 0x0\n\ts_load_dwordx16 %1, %4, 0x40\n\ts_load_dwordx16 %2, %4, 0x80\n\t"
                 "s_load_dwordx16 %3, %4, 0xc0\n\ts_waitcnt lgkmcnt(0)"
                 : "=&s"(c[0]), "=&s"(c[1]), "=&s"(c[2]), "=&s"(c[3]) : "s"(ka) : "memory");
  }
  uint32_t w[NW];
#pragma unroll
  for (int i = 0; i < NW; ++i) w[i] = c[i / 16][i % 16];
  T out;
  __builtin_memcpy(&out, w, sizeof(T));
  return out;
#else
  return T();   // (the host pass only parses kernels)
#endif
}

}  // namespace mm
