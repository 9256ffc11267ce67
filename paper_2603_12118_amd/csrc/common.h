// Shared declarations of the library's translation units (host side + kernel launchers).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <exception>
#include <new>
#include <string>

#include "../../include/cornenc.h"

namespace cs {

typedef uint16_t bf16_t;  // raw bf16 storage word

// ---- error plumbing -------------------------------------------------------------------
void set_error(const std::string& msg);
cs_status fail(cs_status s, const std::string& msg);

// No exception may cross the C boundary (host allocations can throw): the tail of a function-try-block
// around the body of an extern "C" function that returns a status.
inline cs_status fail_noexcept(cs_status s, const char* msg) noexcept {
  try {
    return fail(s, msg);
  } catch (...) {
    return s;
  }
}
#define CS_CATCH_ALL(who)                                                                                        \
  catch (const std::bad_alloc&) { return ::cs::fail_noexcept(CS_ERR_NO_MEMORY, who ": out of host memory"); }    \
  catch (const std::exception& ex) { return ::cs::fail_noexcept(CS_ERR_INVALID_ARG, ex.what()); }                \
  catch (...) { return ::cs::fail_noexcept(CS_ERR_INVALID_ARG, who ": unexpected exception"); }

#define CS_HIP(expr)                                                                          \
  do {                                                                                        \
    hipError_t _e = (expr);                                                                   \
    if (_e != hipSuccess)                                                                     \
      return ::cs::fail(CS_ERR_HIP, std::string(#expr) + ": " + hipGetErrorString(_e));       \
  } while (0)

static inline int64_t round_up(int64_t x, int64_t m) { return (x + m - 1) / m * m; }

// ---- GEMM  C = epilogue(A W^T) ----------------------------------------------------------
enum GemmEpilogue {
  EPI_BF16 = 0,       // (acc + bias) -> bf16
  EPI_F32 = 1,        // (acc + bias) -> fp32
  EPI_GELU_BF16 = 2,  // gelu(acc + bias) -> bf16
  EPI_GELU_F32 = 3,   // gelu(acc + bias) -> fp32
  EPI_RESADD_F32 = 4, // out += acc + bias   (fp32 residual stream)
  EPI_SWIGLU_BF16 = 5,// weight rows interleaved in blocks of 32: gate | up; out[:, j] = silu(g) * u
  EPI_QKV = 6,        // q,k: bias, rotary, (q: scale) -> bf16 row-major; v: bias -> bf16 transposed
  EPI_GELU_SPLIT = 7, // v = gelu(acc + bias) -> bf16 hi at column n and bf16 lo = v - hi at column N + n
  EPI_RESADD_SCALED_F32 = 8, // out += col_scale * (acc + bias)   (a learned per-channel scale on the branch)
  EPI_RESADD_SUMS_F32 = 9    // EPI_RESADD_F32 whose folded normalisation is a LayerNorm (plain sums as well);
                             // launch_gemm picks it for EPI_RESADD_F32 with s1_out set
};

struct GemmArgs {
  const bf16_t* A;   // [M, lda]
  int64_t lda;
  const bf16_t* W;   // [N, ldw], K % 64 == 0
  int64_t ldw;       // row pitch of W in elements; 0 means K
  const float* bias; // [N] or nullptr
  const float* col_scale;  // [N], EPI_RESADD_SCALED_F32 only
  void* out;         // [*, ldo]
  int64_t ldo;
  const int32_t* row_map;  // nullptr, or destination row per m (negative: skip)
  int32_t M, N, K;
  // split K: workgroups with blockIdx.y = s compute columns [s*K, (s+1)*K) of A and W (K is the length of
  // one part) and write to out + s * split_stride elements; splits <= 1: one part
  int32_t splits;
  int64_t split_stride;
  // EPI_QKV only
  bf16_t* vt;        // [hidden, ld_vt]
  int64_t ld_vt;
  const float* rope_cs;    // [M, head_dim/2, 2] = (cos, sin) per rotary pair, or nullptr (no rotary)
  int32_t hidden;    // q columns [0,hidden), k [hidden,2 hidden), v [2 hidden, 3 hidden)
  int32_t head_dim;
  float q_scale;
  // RMSNorm folded into the GEMMs on both sides of it (y = (x g / rms) W^T + b = (1/rms) ((x g) W^T) + b: a
  // row scale commutes with the product, and bf16(x g) carries the same relative rounding as bf16(x g / rms)).
  //  producer (the residual epilogues, on any tile of at most 256 columns): with ss_out set, the epilogue also
  //    writes xg[m, n] = bf16(x_new[m, n] * norm_gain[n]) and ss_out[(n0 / BN) * ss_stride + m] = the sum of
  //    x_new[m, n]^2 over the tile's BN columns (gemm_norm_fold_parts tells how many column tiles there are);
  //  consumer (EPI_QKV, EPI_SWIGLU_BF16): with ss_in set, row m of A W^T is multiplied by
  //    rsqrt(sum over ss_parts of ss_in[p * ss_stride + m] / norm_dim + norm_eps) before the bias is added.
  // LayerNorm folds the same way: LN(x) W^T + b = rs ((x g) W^T - mu c) + d with rs = 1/sqrt(var + eps),
  // c[n] = sum_k g[k] W[n, k] and d[n] = b[n] + sum_k beta[k] W[n, k], both made once from the weights.
  //  producer (also EPI_RESADD_SCALED_F32): with s1_out set it writes the sums of x_new[m, n] as well,
  //    laid out like ss_out;
  //  consumer (EPI_QKV, EPI_GELU_BF16): with s1_in set, mu = sum1 / norm_dim, var = sum2 / norm_dim - mu^2, and
  //    row m of A W^T becomes rs (A W^T)[m, n] - rs mu norm_shift[n] before the bias (= d) is added.
  //    (bf16(x g) is not centred: its rounding is relative to |x g|, so this is for rows whose mean is
  //    small against their deviation, as the rows of a pre-norm residual stream are.)
  const float* norm_gain;
  bf16_t* xg;
  int64_t ld_xg;
  float* ss_out;
  float* s1_out;
  const float* ss_in;
  const float* s1_in;
  const float* norm_shift;
  int32_t ss_parts;
  int64_t ss_stride;
  int32_t norm_dim;
  float norm_eps;
  // measurement aid: when set (host buffer of at least 96 bytes), launch_gemm writes the name of the kernel
  // instantiation it would run for these arguments there and launches nothing
  char* describe;
  // set by the launcher: the residual epilogue stores plainly (through the L2's write-back) instead of write-through
  int32_t plain_stores;
};

cs_status launch_gemm(int epilogue, const GemmArgs& g, hipStream_t stream);
// Column tiles (= partial sums of squares per row) of a residual GEMM that can fold the next RMSNorm into its
// epilogue for M rows and N columns, or 0 if that launch would not run on the tile that supports it.
int32_t gemm_norm_fold_parts(int64_t M, int64_t N, int64_t K, bool scaled = false, bool sums = false);

// ---- write-through global stores -----------------------------------------------------------
// Every XCD has its own L2, and the end of a kernel writes back whatever is dirty in it before the
// next kernel may read it from another XCD.  With plain stores that write-back (up to 4 MB per
// XCD) sits at the end of every kernel; stores of agent scope (sc1) go through the L2 as they are
// issued and leave it clean.  Measured: gate|up GEMM 153 -> 145 us, QKV GEMM -3.5 %, the kernels
// that read the data next unchanged.
// ONLY for 128-byte lines that a single workgroup (or workgroups of one XCD) writes completely:
// a line written in parts from two XCDs came out with stale bytes (seen with head rows of 160
// bytes written by one workgroup per head), and small strided pieces lose the L2's write
// combining (8-byte pieces of 32 rows per instruction: 50 % slower).  Callers pass `wt` = the
// destination's base and row pitch are multiples of 128 bytes and so is every workgroup's extent.
typedef float wt_f32x4 __attribute__((ext_vector_type(4)));
typedef float wt_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ void store_wt16(void* p, wt_f32x4 v) {
  asm volatile("global_store_dwordx4 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store_wt8(void* p, wt_f32x2 v) {
  asm volatile("global_store_dwordx2 %0, %1, off sc1" ::"v"(p), "v"(v) : "memory");
}
__device__ __forceinline__ void store16(void* p, wt_f32x4 v, bool wt) {
  if (wt) store_wt16(p, v);
  else *static_cast<wt_f32x4*>(p) = v;
}
__device__ __forceinline__ void store8(void* p, wt_f32x2 v, bool wt) {
  if (wt) store_wt8(p, v);
  else *static_cast<wt_f32x2*>(p) = v;
}
__host__ __device__ inline bool lines_exclusive(const void* base, int64_t pitch_bytes) {
  return ((reinterpret_cast<uintptr_t>(base) | static_cast<uintptr_t>(pitch_bytes)) & 127) == 0;
}

// GELU(z) = z Phi(z) with erfc from the five-term rational approximation of Abramowitz & Stegun
// 7.1.26 (absolute error below 1.5e-7): erfc(x) = t (a1 + t (a2 + ... t a5)) exp(-x^2), t = 1 / (1 + p x),
// x >= 0.  Phi(z) = erfc(|z| / sqrt 2) / 2 for z < 0 and one minus that otherwise, so the negative side
// has no cancellation.  A dozen instructions with the hardware reciprocal and exp2 where the library
// erff takes several times that, for every element of the audio MLP's widest epilogue.
__device__ __forceinline__ float gelu_erf(float z) {
  const float x = fabsf(z) * 0.70710678118654752f;
  const float t = __builtin_amdgcn_rcpf(1.0f + 0.3275911f * x);
  const float poly = t * (0.254829592f + t * (-0.284496736f + t * (1.421413741f + t * (-1.453152027f + t * 1.061405429f))));
  const float half_erfc = 0.5f * poly * __builtin_amdgcn_exp2f(-1.4426950408889634f * x * x);
  return z * (z < 0.f ? half_erfc : 1.0f - half_erfc);
}

// pixels -> patch rows (elementwise.hip): up to PATCHIFY_ITEMS items [F,3,H,W] per launch, described by value
constexpr int PATCHIFY_ITEMS = 32;
struct PatchifyItems {
  int32_t n;
  int32_t F[PATCHIFY_ITEMS], H[PATCHIFY_ITEMS], W[PATCHIFY_ITEMS];
  int64_t src_off[PATCHIFY_ITEMS];       // first pixel of the item, in elements
  int64_t dst_off[PATCHIFY_ITEMS];       // first output element of the item
  int64_t pair_cu[PATCHIFY_ITEMS + 1];   // running count of pixel pairs: item k owns [pair_cu[k], pair_cu[k+1])
};
cs_status launch_patchify(const void* frames, int in_bf16, void* out, int out_bf16, const PatchifyItems& items,
                          int32_t tp, int32_t patch, hipStream_t s);

// bare MFMA loop (probe.hip): blocks x 8 waves x iters x 32 MFMAs of 32x32x16; out holds blocks*512 floats
cs_status launch_mfma_loop(float* out, int blocks, int iters, int random_operands, hipStream_t stream);

// ---- attention ------------------------------------------------------------------------------
struct AttnWork {  // one workgroup: queries [q0,q1) against keys [kv0,kv1), token indices
  int32_t q0, q1, kv0, kv1;
};
struct AttnArgs {
  const bf16_t* qk;   // [n_tok, 2*hidden]
  const bf16_t* vt;   // [hidden, ld_vt]
  int64_t ld_vt;
  bf16_t* out;        // [n_tok, hidden]
  const AttnWork* work;
  int32_t n_work, n_tok, n_heads, head_dim;
  int32_t q_per_block;  // 64 or 256 queries per workgroup (work items are cut accordingly)
  int32_t single_tile;  // nonzero: no work item has more than 64 keys (64-query items only)
};
cs_status launch_attention(const AttnArgs& a, hipStream_t stream);

// ---- row-wise and copy kernels ----------------------------------------------------------
// Split-K partial sums of a residual GEMM that the next normalisation adds to x on its way through:
// x[r, n] += scale[n] * (sum over s of parts[s*stride + r*dim + n] + bias[n]), written back to x, then
// normalised.  parts == nullptr: nothing pending.  scale may be nullptr (1).
constexpr int PENDING_MAX_PARTS = 4;   // a split-K launch of the encoder leaves at most so many partial sums
struct PendingSum {
  const float* parts = nullptr;
  int32_t n_parts = 0;
  int64_t stride = 0;
  const float* bias = nullptr;
  const float* scale = nullptr;
};
cs_status launch_rmsnorm(float* x, const float* gain, float eps, bf16_t* y, int64_t rows, int32_t dim, hipStream_t s,
                         const PendingSum& add = PendingSum());
// y[g, 0:group*dim) = bf16 hi parts of `group` consecutive normalised rows, y[g, group*dim : 2*group*dim) = lo parts
cs_status launch_rmsnorm_split(float* x, const float* gain, float eps, bf16_t* y, int64_t rows, int32_t dim,
                               int32_t group, hipStream_t s, const PendingSum& add = PendingSum());
cs_status launch_layernorm(float* x, const float* gain, const float* bias, float eps, bf16_t* y, int64_t rows,
                           int32_t dim, hipStream_t s, const PendingSum& add = PendingSum());
// y[r] = layernorm(mean of `pool` consecutive rows of x)
cs_status launch_pool_layernorm(const float* x, const float* gain, const float* bias, float eps, bf16_t* y,
                                int64_t out_rows, int32_t dim, int32_t pool, hipStream_t s);
// dst[r, 0:dst_cols) = bf16(src[src_row[r], 0:src_cols)) padded with zeros; src_row < 0 gives a zero row
cs_status launch_gather_cast(const void* src, int src_is_bf16, int32_t src_cols, const int32_t* src_row,
                             bf16_t* dst, int32_t dst_cols, int64_t rows, hipStream_t s);
// out[n, j] = (cos, sin) of pos[n, axis[j]] * inv_freq[j]
cs_status launch_rope_table(const int32_t* pos, const int32_t* axis, const float* inv_freq, int32_t half,
                            float* cos_sin_out, int64_t n_tok, hipStream_t s);
// class-token towers: pos[r] >= 0: x[r] += table[pos[r]];  -1: x[r] = table[class_row];  -2: x[r] = 0
cs_status launch_place_tokens(float* x, const float* table, const int32_t* pos, int32_t class_row, int64_t rows,
                              int32_t dim, hipStream_t s);
// y[r, 0:dim) = bf16 hi parts of layernorm(x[r, 0:dim)), y[r, dim:2*dim) = lo parts; one workgroup per row, dim <= 8192
cs_status launch_layernorm_wide_split(const float* x, const float* gain, const float* bias, float eps, bf16_t* y,
                                      int64_t rows, int32_t dim, hipStream_t s);
// x[r, n] += scale[n] * (sum over s of parts[s*stride + r*dim + n] + bias[n]); scale / bias may be NULL (1 / 0)
cs_status launch_add_partials(float* x, const float* parts, int32_t n_parts, int64_t stride, const float* bias,
                              const float* scale, int64_t rows, int32_t dim, hipStream_t s);
// split-K sums of the merger's two GEMMs.  hidden: y = gelu(sum of parts + bias) written as bf16 hi at
// out[r, n] and bf16 lo = y - hi at out[r, dim + n] (rows of 2*dim).  store: out[row_map[r], n] = sum of
// parts + bias as fp32 or bf16 (out_bf16), rows of `dim`; row_map may be NULL, negative entries are skipped
cs_status launch_add_partials_gelu_split(bf16_t* out, const float* parts, int32_t n_parts, int64_t stride,
                                         const float* bias, int64_t rows, int32_t dim, hipStream_t s);
cs_status launch_add_partials_store(void* out, int out_bf16, const int32_t* row_map, const float* parts,
                                    int32_t n_parts, int64_t stride, const float* bias, int64_t rows, int32_t dim,
                                    hipStream_t s);
// x[r, :] += table[pos[r], :]
cs_status launch_add_rows(float* x, const float* table, const int32_t* pos, int64_t rows, int32_t dim,
                          hipStream_t s);
cs_status launch_zero_rows(bf16_t* buf, const int32_t* rows, int32_t n_rows, int32_t cols, hipStream_t s);
cs_status launch_scatter_rows(const void* src, const int64_t* index, void* dst, int64_t n_rows, int64_t dst_rows,
                              int64_t row_bytes, int32_t* err_flag, hipStream_t s);

}  // namespace cs
