// Bandwidth-bound kernels: normalisations, input gather/cast, rotary table, position add and the
// embedding hand-off (row scatter).  All are one pass over HBM with 16-byte (or 8-byte) accesses.
#include <algorithm>

#include "common.h"

namespace cs {

typedef float f32x2_e __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_e __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t pack2_e(float a, float b) {
  const f32x2_e v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_e));
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

constexpr int NORM_MAX_V4 = 8;  // a wave keeps a row of up to 64*4*8 = 2048 floats in registers

// One wave per row.  MODE 0: RMSNorm.  MODE 1: LayerNorm.  POOL rows of x are averaged first.
template <int MODE>
__global__ __launch_bounds__(256) void norm_kernel(float* __restrict__ x, const float* __restrict__ gain,
                                                   const float* __restrict__ bias, float eps,
                                                   bf16_t* __restrict__ y, int64_t rows, int dim, int pool, int split_group,
                                                   bool wt, PendingSum add) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  float4 v[NORM_MAX_V4];
  const int nv = dim >> 2;
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = lane + 64 * i;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < nv) {
      for (int p = 0; p < pool; ++p) {
        const float4 t = reinterpret_cast<const float4*>(x + (row * pool + p) * dim)[c];
        v[i].x += t.x; v[i].y += t.y; v[i].z += t.z; v[i].w += t.w;
      }
      if (pool > 1) {
        const float ip = 1.0f / pool;
        v[i].x *= ip; v[i].y *= ip; v[i].z *= ip; v[i].w *= ip;
      }
      if (add.parts) {   // pending split-K sums join the residual stream here (pool == 1)
        // all parts are requested before the first is used (a loop over a run-time count waits for every
        // load in turn); summed in part order as before
        float4 part[PENDING_MAX_PARTS];
#pragma unroll
        for (int s = 0; s < PENDING_MAX_PARTS; ++s)
          if (s < add.n_parts) part[s] = reinterpret_cast<const float4*>(add.parts + s * add.stride + row * dim)[c];
        float4 a = part[0];
#pragma unroll
        for (int s = 1; s < PENDING_MAX_PARTS; ++s)
          if (s < add.n_parts) { a.x += part[s].x; a.y += part[s].y; a.z += part[s].z; a.w += part[s].w; }
        if (add.bias) {
          const float4 t = reinterpret_cast<const float4*>(add.bias)[c];
          a.x += t.x; a.y += t.y; a.z += t.z; a.w += t.w;
        }
        if (add.scale) {
          const float4 t = reinterpret_cast<const float4*>(add.scale)[c];
          a.x *= t.x; a.y *= t.y; a.z *= t.z; a.w *= t.w;
        }
        v[i].x += a.x; v[i].y += a.y; v[i].z += a.z; v[i].w += a.w;
        reinterpret_cast<float4*>(x + row * dim)[c] = v[i];
      }
    }
  }
  float mean = 0.f;
  if (MODE == 1) {
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NORM_MAX_V4; ++i) s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    mean = wave_sum(s) / dim;
  }
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    if (lane + 64 * i < nv) {
      const float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      ss += (a * a + b * b) + (c * c + d * d);
    }
  }
  const float rstd = rsqrtf(wave_sum(ss) / dim + eps);
#pragma unroll
  for (int i = 0; i < NORM_MAX_V4; ++i) {
    const int c = lane + 64 * i;
    if (c < nv) {
      const float4 g = reinterpret_cast<const float4*>(gain)[c];
      float4 b = make_float4(0.f, 0.f, 0.f, 0.f);
      if (MODE == 1) b = reinterpret_cast<const float4*>(bias)[c];
      const float o0 = (v[i].x - mean) * rstd * g.x + b.x, o1 = (v[i].y - mean) * rstd * g.y + b.y;
      const float o2 = (v[i].z - mean) * rstd * g.z + b.z, o3 = (v[i].w - mean) * rstd * g.w + b.w;
      uint2 pk;
      pk.x = pack2_e(o0, o1);
      pk.y = pack2_e(o2, o3);
      if (split_group == 0) {
        store8(reinterpret_cast<uint2*>(y + row * dim) + c, __builtin_bit_cast(wt_f32x2, pk), wt);
      } else {
        // hi | lo halves of a row of `split_group` tokens: lo = value - hi, again rounded to bf16
        bf16_t* dst = y + (row / split_group) * (2 * split_group * dim) + (row % split_group) * dim;
        store8(reinterpret_cast<uint2*>(dst) + c, __builtin_bit_cast(wt_f32x2, pk), wt);
        uint2 lo;
        lo.x = pack2_e(o0 - __uint_as_float(pk.x << 16), o1 - __uint_as_float(pk.x & 0xFFFF0000u));
        lo.y = pack2_e(o2 - __uint_as_float(pk.y << 16), o3 - __uint_as_float(pk.y & 0xFFFF0000u));
        store8(reinterpret_cast<uint2*>(dst + split_group * dim) + c, __builtin_bit_cast(wt_f32x2, lo), wt);
      }
    }
  }
}

static cs_status norm_check(int64_t rows, int dim, const PendingSum& add = PendingSum()) {
  if (dim <= 0 || (dim & 3) || dim > 64 * 4 * NORM_MAX_V4)
    return fail(CS_ERR_UNSUPPORTED, "norm: dim must be a multiple of 4, at most 2048");
  if (add.parts && (add.n_parts < 1 || add.n_parts > PENDING_MAX_PARTS || (add.stride & 3)))
    return fail(CS_ERR_UNSUPPORTED, "norm: pending sums come in 1 to 4 parts, their stride a multiple of 4");
  if (rows > (int64_t)4 * 0x7fffffff) return fail(CS_ERR_UNSUPPORTED, "norm: too many rows");
  return CS_OK;
}

cs_status launch_rmsnorm(float* x, const float* gain, float eps, bf16_t* y, int64_t rows, int32_t dim, hipStream_t s,
                         const PendingSum& add) {
  if (rows <= 0) return CS_OK;
  if (cs_status st = norm_check(rows, dim, add)) return st;
  hipLaunchKernelGGL(norm_kernel<0>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x, gain, nullptr, eps, y,
                     rows, dim, 1, 0, lines_exclusive(y, (int64_t)dim * 2), add);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

cs_status launch_rmsnorm_split(float* x, const float* gain, float eps, bf16_t* y, int64_t rows, int32_t dim,
                               int32_t group, hipStream_t s, const PendingSum& add) {
  if (rows <= 0) return CS_OK;
  if (cs_status st = norm_check(rows, dim, add)) return st;
  if (group < 1 || rows % group) return fail(CS_ERR_INVALID_ARG, "rmsnorm_split: rows must be a multiple of the group");
  hipLaunchKernelGGL(norm_kernel<0>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x, gain, nullptr, eps, y,
                     rows, dim, 1, group, lines_exclusive(y, (int64_t)dim * 2), add);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

cs_status launch_layernorm(float* x, const float* gain, const float* bias, float eps, bf16_t* y, int64_t rows,
                           int32_t dim, hipStream_t s, const PendingSum& add) {
  if (rows <= 0) return CS_OK;
  if (cs_status st = norm_check(rows, dim, add)) return st;
  hipLaunchKernelGGL(norm_kernel<1>, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, x, gain, bias, eps, y, rows,
                     dim, 1, 0, lines_exclusive(y, (int64_t)dim * 2), add);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

cs_status launch_pool_layernorm(const float* x, const float* gain, const float* bias, float eps, bf16_t* y,
                                int64_t out_rows, int32_t dim, int32_t pool, hipStream_t s) {
  if (out_rows <= 0) return CS_OK;
  if (cs_status st = norm_check(out_rows, dim)) return st;
  if (pool < 1) return fail(CS_ERR_INVALID_ARG, "pool_layernorm: pool < 1");
  hipLaunchKernelGGL(norm_kernel<1>, dim3((unsigned)((out_rows + 3) / 4)), dim3(256), 0, s, const_cast<float*>(x), gain, bias,
                     eps, y, out_rows, dim, pool, 0, lines_exclusive(y, (int64_t)dim * 2), PendingSum());
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- gather + cast to bf16 with zero padding; 4 elements per thread
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void gather_cast_kernel(const void* __restrict__ src, int src_cols,
                                                          const int32_t* __restrict__ src_row,
                                                          bf16_t* __restrict__ dst, int dst_cols, int64_t rows, bool wt) {
  const int cpr = dst_cols >> 2;
  const int64_t total = rows * cpr;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / cpr;
    const int c = (int)(t - r * cpr) * 4;
    const int64_t sr = src_row ? src_row[r] : r;
    uint2 pk = make_uint2(0u, 0u);
    if (sr >= 0 && c < src_cols) {
      if (SRC_BF16) {
        pk = *reinterpret_cast<const uint2*>(static_cast<const bf16_t*>(src) + sr * src_cols + c);
      } else {
        const float4 v = *reinterpret_cast<const float4*>(static_cast<const float*>(src) + sr * src_cols + c);
        pk.x = pack2_e(v.x, v.y);
        pk.y = pack2_e(v.z, v.w);
      }
    }
    store8(dst + r * dst_cols + c, __builtin_bit_cast(wt_f32x2, pk), wt);
  }
}

cs_status launch_gather_cast(const void* src, int src_is_bf16, int32_t src_cols, const int32_t* src_row, bf16_t* dst,
                             int32_t dst_cols, int64_t rows, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if ((src_cols & 3) || (dst_cols & 3) || dst_cols < src_cols)
    return fail(CS_ERR_UNSUPPORTED, "gather_cast: column counts must be multiples of 4, dst >= src");
  const int64_t total = rows * (dst_cols >> 2);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
  if (src_is_bf16)
    hipLaunchKernelGGL(gather_cast_kernel<true>, dim3(blocks), dim3(256), 0, s, src, src_cols, src_row, dst, dst_cols, rows,
                       lines_exclusive(dst, 128));
  else
    hipLaunchKernelGGL(gather_cast_kernel<false>, dim3(blocks), dim3(256), 0, s, src, src_cols, src_row, dst, dst_cols, rows,
                       lines_exclusive(dst, 128));
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- rotary table: (cos, sin) interleaved per pair, so the QKV epilogue fetches two pairs in 16 bytes
__global__ __launch_bounds__(256) void rope_table_kernel(const int32_t* __restrict__ pos, const int32_t* __restrict__ axis,
                                                         const float* __restrict__ inv_freq, int half,
                                                         float2* __restrict__ out, int64_t total) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= total) return;
  const int64_t n = t / half;
  const int j = (int)(t - n * half);
  const float ang = (float)pos[n * 3 + axis[j]] * inv_freq[j];
  float sn, cs_;
  sincosf(ang, &sn, &cs_);
  out[t] = make_float2(cs_, sn);
}

cs_status launch_rope_table(const int32_t* pos, const int32_t* axis, const float* inv_freq, int32_t half, float* cos_sin_out,
                            int64_t n_tok, hipStream_t s) {
  const int64_t total = n_tok * half;
  if (total <= 0) return CS_OK;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, pos, axis, inv_freq, half,
                     reinterpret_cast<float2*>(cos_sin_out), total);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- split-K sums into the residual stream: x += scale * (sum of parts + bias), parts added in index order
__global__ __launch_bounds__(256) void add_partials_kernel(float* __restrict__ x, const float* __restrict__ parts, int n_parts,
                                                           int64_t stride, const float* __restrict__ bias,
                                                           const float* __restrict__ scale, int64_t rows, int dim) {
  const int cpr = dim >> 2;
  const int64_t total = rows * cpr;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / cpr;
    const int c = (int)(t - r * cpr);
    float4 a = reinterpret_cast<const float4*>(parts + r * dim)[c];
    for (int s = 1; s < n_parts; ++s) {
      const float4 p = reinterpret_cast<const float4*>(parts + s * stride + r * dim)[c];
      a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
    }
    if (bias) {
      const float4 b = reinterpret_cast<const float4*>(bias)[c];
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    if (scale) {
      const float4 g = reinterpret_cast<const float4*>(scale)[c];
      a.x *= g.x; a.y *= g.y; a.z *= g.z; a.w *= g.w;
    }
    float4 v = reinterpret_cast<float4*>(x + r * dim)[c];
    v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
    reinterpret_cast<float4*>(x + r * dim)[c] = v;
  }
}

cs_status launch_add_partials(float* x, const float* parts, int32_t n_parts, int64_t stride, const float* bias,
                              const float* scale, int64_t rows, int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if ((dim & 3) || n_parts < 1 || (stride & 3)) return fail(CS_ERR_UNSUPPORTED, "add_partials: dim and stride must be multiples of 4");
  const int64_t total = rows * (dim >> 2);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
  hipLaunchKernelGGL(add_partials_kernel, dim3(blocks), dim3(256), 0, s, x, parts, n_parts, stride, bias, scale, rows, dim);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// MODE 0: gelu, bf16 hi | lo.  MODE 1: plain store through the row map, fp32 or bf16.
template <int MODE>
__global__ __launch_bounds__(256) void add_partials_out_kernel(void* __restrict__ out, int out_bf16,
                                                               const int32_t* __restrict__ row_map,
                                                               const float* __restrict__ parts, int n_parts, int64_t stride,
                                                               const float* __restrict__ bias, int64_t rows, int dim) {
  const int cpr = dim >> 2;
  const int64_t total = rows * cpr;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / cpr;
    const int c = (int)(t - r * cpr);
    float4 a = reinterpret_cast<const float4*>(parts + r * dim)[c];
    for (int s = 1; s < n_parts; ++s) {
      const float4 p = reinterpret_cast<const float4*>(parts + s * stride + r * dim)[c];
      a.x += p.x; a.y += p.y; a.z += p.z; a.w += p.w;
    }
    if (bias) {
      const float4 b = reinterpret_cast<const float4*>(bias)[c];
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    if (MODE == 0) {
      const float y0 = gelu_erf(a.x), y1 = gelu_erf(a.y), y2 = gelu_erf(a.z), y3 = gelu_erf(a.w);
      uint2 hi, lo;
      hi.x = pack2_e(y0, y1);
      hi.y = pack2_e(y2, y3);
      lo.x = pack2_e(y0 - __uint_as_float(hi.x << 16), y1 - __uint_as_float(hi.x & 0xFFFF0000u));
      lo.y = pack2_e(y2 - __uint_as_float(hi.y << 16), y3 - __uint_as_float(hi.y & 0xFFFF0000u));
      bf16_t* dst = static_cast<bf16_t*>(out) + r * (2 * (int64_t)dim);
      reinterpret_cast<uint2*>(dst)[c] = hi;
      reinterpret_cast<uint2*>(dst + dim)[c] = lo;
    } else {
      const int64_t row = row_map ? row_map[r] : r;
      if (row < 0) continue;
      if (out_bf16) {
        uint2 pk;
        pk.x = pack2_e(a.x, a.y);
        pk.y = pack2_e(a.z, a.w);
        reinterpret_cast<uint2*>(static_cast<bf16_t*>(out) + row * dim)[c] = pk;
      } else {
        reinterpret_cast<float4*>(static_cast<float*>(out) + row * dim)[c] = a;
      }
    }
  }
}

static unsigned partials_blocks(int64_t rows, int dim) {
  const int64_t total = rows * (dim >> 2);
  return (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
}

cs_status launch_add_partials_gelu_split(bf16_t* out, const float* parts, int32_t n_parts, int64_t stride,
                                         const float* bias, int64_t rows, int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if ((dim & 3) || n_parts < 1 || (stride & 3)) return fail(CS_ERR_UNSUPPORTED, "add_partials: dim and stride must be multiples of 4");
  hipLaunchKernelGGL(add_partials_out_kernel<0>, dim3(partials_blocks(rows, dim)), dim3(256), 0, s, out, 1, nullptr, parts,
                     n_parts, stride, bias, rows, dim);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

cs_status launch_add_partials_store(void* out, int out_bf16, const int32_t* row_map, const float* parts, int32_t n_parts,
                                    int64_t stride, const float* bias, int64_t rows, int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if ((dim & 3) || n_parts < 1 || (stride & 3)) return fail(CS_ERR_UNSUPPORTED, "add_partials: dim and stride must be multiples of 4");
  hipLaunchKernelGGL(add_partials_out_kernel<1>, dim3(partials_blocks(rows, dim)), dim3(256), 0, s, out, out_bf16, row_map,
                     parts, n_parts, stride, bias, rows, dim);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- x[r,:] += table[pos[r],:]
__global__ __launch_bounds__(256) void add_rows_kernel(float* __restrict__ x, const float* __restrict__ table,
                                                       const int32_t* __restrict__ pos, int64_t rows, int dim) {
  const int cpr = dim >> 2;
  const int64_t total = rows * cpr;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / cpr;
    const int c = (int)(t - r * cpr);
    float4 v = reinterpret_cast<float4*>(x + r * dim)[c];
    const float4 p = reinterpret_cast<const float4*>(table + (int64_t)pos[r] * dim)[c];
    v.x += p.x; v.y += p.y; v.z += p.z; v.w += p.w;
    reinterpret_cast<float4*>(x + r * dim)[c] = v;
  }
}

cs_status launch_add_rows(float* x, const float* table, const int32_t* pos, int64_t rows, int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if (dim & 3) return fail(CS_ERR_UNSUPPORTED, "add_rows: dim must be a multiple of 4");
  const int64_t total = rows * (dim >> 2);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
  hipLaunchKernelGGL(add_rows_kernel, dim3(blocks), dim3(256), 0, s, x, table, pos, rows, dim);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- class-token towers: learned positions onto the patch embeddings, the class-token row, zero padding rows
__global__ __launch_bounds__(256) void place_tokens_kernel(float* __restrict__ x, const float* __restrict__ table,
                                                           const int32_t* __restrict__ pos, int class_row, int64_t rows,
                                                           int dim) {
  const int cpr = dim >> 2;
  const int64_t total = rows * cpr;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / cpr;
    const int c = (int)(t - r * cpr);
    const int p = pos[r];
    float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
    if (p >= 0) {
      v = reinterpret_cast<const float4*>(x + r * dim)[c];
      const float4 a = reinterpret_cast<const float4*>(table + (int64_t)p * dim)[c];
      v.x += a.x; v.y += a.y; v.z += a.z; v.w += a.w;
    } else if (p == -1) {
      v = reinterpret_cast<const float4*>(table + (int64_t)class_row * dim)[c];
    }
    reinterpret_cast<float4*>(x + r * dim)[c] = v;
  }
}

cs_status launch_place_tokens(float* x, const float* table, const int32_t* pos, int32_t class_row, int64_t rows,
                              int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if (dim & 3) return fail(CS_ERR_UNSUPPORTED, "place_tokens: dim must be a multiple of 4");
  const int64_t total = rows * (dim >> 2);
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 * 16 ? (total + 255) / 256 : 65536 * 16);
  hipLaunchKernelGGL(place_tokens_kernel, dim3(blocks), dim3(256), 0, s, x, table, pos, class_row, rows, dim);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- LayerNorm over wide rows (the concatenation of a merge group), one workgroup per row, output as
// bf16 hi | lo halves.  A thread keeps up to WIDE_MAX_V4 float4 of the row in registers.
constexpr int WIDE_MAX_V4 = 8;  // 256 threads * 8 * 4 = 8192 floats
__device__ __forceinline__ float block_sum_256(float v, float* red) {
  v = wave_sum(v);
  __syncthreads();                       // red may still be read from the previous reduction
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
  __syncthreads();
  return (red[0] + red[1]) + (red[2] + red[3]);
}

__global__ __launch_bounds__(256) void layernorm_wide_split_kernel(const float* __restrict__ x, const float* __restrict__ gain,
                                                                   const float* __restrict__ bias, float eps,
                                                                   bf16_t* __restrict__ y, int dim, bool wt) {
  __shared__ float red[4];
  const int64_t row = blockIdx.x;
  const int nv = dim >> 2;
  float4 v[WIDE_MAX_V4];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < WIDE_MAX_V4; ++i) {
    const int c = threadIdx.x + 256 * i;
    v[i] = make_float4(0.f, 0.f, 0.f, 0.f);
    if (c < nv) v[i] = reinterpret_cast<const float4*>(x + row * dim)[c];
    s += (v[i].x + v[i].y) + (v[i].z + v[i].w);
  }
  const float mean = block_sum_256(s, red) / dim;
  float ss = 0.f;
#pragma unroll
  for (int i = 0; i < WIDE_MAX_V4; ++i) {
    if (threadIdx.x + 256 * i < nv) {
      const float a = v[i].x - mean, b = v[i].y - mean, c = v[i].z - mean, d = v[i].w - mean;
      ss += (a * a + b * b) + (c * c + d * d);
    }
  }
  const float rstd = rsqrtf(block_sum_256(ss, red) / dim + eps);
  bf16_t* dst = y + row * (2 * (int64_t)dim);
#pragma unroll
  for (int i = 0; i < WIDE_MAX_V4; ++i) {
    const int c = threadIdx.x + 256 * i;
    if (c < nv) {
      const float4 g = reinterpret_cast<const float4*>(gain)[c];
      const float4 b = reinterpret_cast<const float4*>(bias)[c];
      const float o0 = (v[i].x - mean) * rstd * g.x + b.x, o1 = (v[i].y - mean) * rstd * g.y + b.y;
      const float o2 = (v[i].z - mean) * rstd * g.z + b.z, o3 = (v[i].w - mean) * rstd * g.w + b.w;
      uint2 pk;
      pk.x = pack2_e(o0, o1);
      pk.y = pack2_e(o2, o3);
      store8(reinterpret_cast<uint2*>(dst) + c, __builtin_bit_cast(wt_f32x2, pk), wt);
      uint2 lo;
      lo.x = pack2_e(o0 - __uint_as_float(pk.x << 16), o1 - __uint_as_float(pk.x & 0xFFFF0000u));
      lo.y = pack2_e(o2 - __uint_as_float(pk.y << 16), o3 - __uint_as_float(pk.y & 0xFFFF0000u));
      store8(reinterpret_cast<uint2*>(dst + dim) + c, __builtin_bit_cast(wt_f32x2, lo), wt);
    }
  }
}

cs_status launch_layernorm_wide_split(const float* x, const float* gain, const float* bias, float eps, bf16_t* y,
                                      int64_t rows, int32_t dim, hipStream_t s) {
  if (rows <= 0) return CS_OK;
  if (dim <= 0 || (dim & 3) || dim > 256 * 4 * WIDE_MAX_V4)
    return fail(CS_ERR_UNSUPPORTED, "layernorm_wide: dim must be a multiple of 4, at most 8192");
  if (rows > 0x7fffffff) return fail(CS_ERR_UNSUPPORTED, "layernorm_wide: too many rows");
  if (!gain || !bias) return fail(CS_ERR_INVALID_ARG, "layernorm_wide: gain and bias are needed");
  hipLaunchKernelGGL(layernorm_wide_split_kernel, dim3((unsigned)rows), dim3(256), 0, s, x, gain, bias, eps, y, dim,
                     lines_exclusive(y, (int64_t)dim * 2));
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- embedding hand-off: dst[index[i], :] = src[i, :], 16 bytes per thread, rows whole
__global__ __launch_bounds__(256) void scatter_rows_kernel(const uint4* __restrict__ src, const int64_t* __restrict__ index,
                                                           uint4* __restrict__ dst, int64_t n_rows, int64_t dst_rows,
                                                           int chunks_per_row, int32_t* err_flag, bool wt) {
  const int64_t total = n_rows * chunks_per_row;
  for (int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x; t < total; t += (int64_t)gridDim.x * 256) {
    const int64_t r = t / chunks_per_row;
    const int c = (int)(t - r * chunks_per_row);
    const int64_t d = index[r];
    if (d == -1) continue;
    if (d < -1 || d >= dst_rows) {
      if (err_flag && c == 0) *err_flag = 1;
      continue;
    }
    store16(dst + d * chunks_per_row + c, __builtin_bit_cast(wt_f32x4, src[t]), wt);
  }
}

cs_status launch_scatter_rows(const void* src, const int64_t* index, void* dst, int64_t n_rows, int64_t dst_rows,
                              int64_t row_bytes, int32_t* err_flag, hipStream_t s) {
  if (n_rows <= 0) return CS_OK;
  const int64_t cpr = row_bytes >> 4;
  const int64_t total = n_rows * cpr;
  const unsigned blocks = (unsigned)((total + 255) / 256 < 65536 * 8 ? (total + 255) / 256 : 65536 * 8);
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(blocks), dim3(256), 0, s, static_cast<const uint4*>(src), index,
                     static_cast<uint4*>(dst), n_rows, dst_rows, (int)cpr, err_flag, lines_exclusive(dst, row_bytes));
  CS_HIP(hipGetLastError());
  return CS_OK;
}

}  // namespace cs

namespace cs {

// ---- clear whole rows of a bf16 matrix (padding frames between audio clips)
__global__ __launch_bounds__(256) void zero_rows_kernel(bf16_t* __restrict__ buf, const int32_t* __restrict__ rows,
                                                        int n_rows, int cols) {
  const int cpr = cols >> 3;
  for (int t = blockIdx.x * 256 + threadIdx.x; t < n_rows * cpr; t += gridDim.x * 256) {
    const int r = t / cpr, c = t - r * cpr;
    reinterpret_cast<uint4*>(buf + (int64_t)rows[r] * cols)[c] = make_uint4(0u, 0u, 0u, 0u);
  }
}

cs_status launch_zero_rows(bf16_t* buf, const int32_t* rows, int32_t n_rows, int32_t cols, hipStream_t s) {
  if (n_rows <= 0) return CS_OK;
  if (cols & 7) return fail(CS_ERR_UNSUPPORTED, "zero_rows: cols must be a multiple of 8");
  const int total = n_rows * (cols >> 3);
  hipLaunchKernelGGL(zero_rows_kernel, dim3((total + 255) / 256), dim3(256), 0, s, buf, rows, n_rows, cols);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

// ---- pixels -> patch rows.  One thread per input pixel pair (x, x+1): reads run along image rows,
// writes are the 14-pixel runs of a patch row.  Output element order inside a patch: (channel,
// frame inside the temporal patch, py, px); patches in raster order (t, row, col).  An item with a
// single frame shows it tp times.  Up to PATCHIFY_ITEMS items per launch, described in the
// kernel arguments (no device-side table to allocate or copy).
template <bool IN_BF16, bool OUT_BF16>
__global__ __launch_bounds__(256) void patchify_kernel(const void* __restrict__ frames, void* __restrict__ out,
                                                       PatchifyItems it, int tp, int patch) {
  const int pdim = 3 * tp * patch * patch;
  const int64_t total = it.pair_cu[it.n];
  for (int64_t gi = (int64_t)blockIdx.x * 256 + threadIdx.x; gi < total; gi += (int64_t)gridDim.x * 256) {
    int k = 0;
    while (k + 1 < it.n && gi >= it.pair_cu[k + 1]) ++k;
    const int F = it.F[k], H = it.H[k], W = it.W[k];
    const int64_t i = gi - it.pair_cu[k];
    const int64_t half_w = W >> 1;
    const int h = H / patch, w = W / patch;
    const int x = (int)(i % half_w) * 2;
    int64_t r = i / half_w;
    const int y = (int)(r % H);
    r /= H;
    const int ch = (int)(r % 3), f = (int)(r / 3);
    float v0, v1;
    if (IN_BF16) {
      const uint32_t u = *reinterpret_cast<const uint32_t*>(static_cast<const bf16_t*>(frames) + it.src_off[k] + 2 * i);
      v0 = __uint_as_float(u << 16);
      v1 = __uint_as_float(u & 0xFFFF0000u);
    } else {
      const float2 u = *reinterpret_cast<const float2*>(static_cast<const float*>(frames) + it.src_off[k] + 2 * i);
      v0 = u.x;
      v1 = u.y;
    }
    const int row = y / patch, py = y - row * patch, col = x / patch, px = x - col * patch;   // px even: the pair stays in one patch
    const int t = F == 1 ? 0 : f / tp, tt0 = F == 1 ? 0 : f - t * tp, reps = F == 1 ? tp : 1;
    for (int rep = 0; rep < reps; ++rep) {
      const int64_t o = it.dst_off[k] + ((int64_t)(t * h + row) * w + col) * pdim + ((ch * tp + tt0 + rep) * patch + py) * patch + px;
      if (OUT_BF16) *reinterpret_cast<uint32_t*>(static_cast<bf16_t*>(out) + o) = pack2_e(v0, v1);
      else *reinterpret_cast<float2*>(static_cast<float*>(out) + o) = make_float2(v0, v1);
    }
  }
}

cs_status launch_patchify(const void* frames, int in_bf16, void* out, int out_bf16, const PatchifyItems& it, int32_t tp,
                          int32_t patch, hipStream_t s) {
  if (it.n <= 0 || it.n > PATCHIFY_ITEMS) return fail(CS_ERR_INVALID_ARG, "patchify: 1..32 items per launch");
  const int64_t total = it.pair_cu[it.n];
  if (total <= 0) return CS_OK;
  const unsigned blocks = (unsigned)std::min<int64_t>((total + 255) / 256, 65536 * 8);
  if (in_bf16 && out_bf16) hipLaunchKernelGGL((patchify_kernel<true, true>), dim3(blocks), dim3(256), 0, s, frames, out, it, tp, patch);
  else if (in_bf16) hipLaunchKernelGGL((patchify_kernel<true, false>), dim3(blocks), dim3(256), 0, s, frames, out, it, tp, patch);
  else if (out_bf16) hipLaunchKernelGGL((patchify_kernel<false, true>), dim3(blocks), dim3(256), 0, s, frames, out, it, tp, patch);
  else hipLaunchKernelGGL((patchify_kernel<false, false>), dim3(blocks), dim3(256), 0, s, frames, out, it, tp, patch);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

}  // namespace cs
