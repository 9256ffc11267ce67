// bf16 MFMA GEMM for gfx950:  C = epilogue(A W^T), A [M,K] and W [N,K] both K-contiguous.
//
// One workgroup owns a BM x BN tile of C and walks K in slices of 64.  Each slice of A and W
// is staged through LDS in 16-byte chunks whose position inside a 128-byte row is XOR-ed with
// (row / 2) % 8: measured on gfx950, ds_read_b128 serves 16 lanes per pass and the lanes of a pass
// are not consecutive (rows {0-3,12-15,20-23,24-27} of an operand read share one), and this is the
// XOR under which both the operand reads and the 16-byte staging stores run at full LDS rate.  Waves are laid out WGM x WGN
// over the tile; a wave accumulates (BM/WGM) x (BN/WGN) in fp32 with v_mfma_f32_32x32x16_bf16.
// Global loads for slice k+1 are issued before the MFMAs of slice k and written to the other
// LDS buffer afterwards, one barrier per slice.
#include "common.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t f2bf(float f) {  // round to nearest even
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }
// value held by the neighbouring lane (lane ^ 1)
__device__ __forceinline__ float lane_xor1(float v) {
  return __int_as_float(__builtin_amdgcn_mov_dpp(__float_as_int(v), 0xB1, 0xF, 0xF, true));
}

typedef __attribute__((address_space(3))) void lds_void;

// Issues the LDS-direct loads of one 64-wide K slice: every wave instruction moves 64 x 16 bytes
// from the lanes' global addresses to 1 KB of LDS starting at a wave-uniform address, in lane order.
template <int A_LOADS, int B_LOADS, int NWAVES, int BM>
__device__ __forceinline__ void issue_slice(const bf16_t* const* ap, const bf16_t* const* bp,
                                            int kt, unsigned char* stage, int wave) {
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i)
    __builtin_amdgcn_global_load_lds(ap[i] + kt * 64, (lds_void*)(uintptr_t)(stage + (i * NWAVES + wave) * 1024), 16, 0, 0);
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i)
    __builtin_amdgcn_global_load_lds(bp[i] + kt * 64, (lds_void*)(uintptr_t)(stage + BM * 128 + (i * NWAVES + wave) * 1024), 16, 0, 0);
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmArgs g) {
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int STAGE_BYTES = (BM + BN) * 128;
  static_assert(EPI != EPI_SWIGLU_BF16 || (TN % 2 == 0), "gate/up pairs need an even number of column tiles");

  extern __shared__ __align__(16) unsigned char smem[];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int M = g.M, N = g.N, K = g.K;

  // workgroup -> tile: consecutive workgroups land on different XCDs, so give each XCD a
  // contiguous range of tiles (they share A strips and W strips through that XCD's L2)
  const int tiles_n = (N + BN - 1) / BN;
  const int nb = gridDim.x;
  int bid = blockIdx.x;
  {
    const int xcd = bid & 7, idx = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    bid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int m0 = (bid / tiles_n) * BM, n0 = (bid % tiles_n) * BN;

  const int l31 = lane & 31, lhi = lane >> 5;
  const int a_rd = (wm * WM + l31) * 128;
  const int b_rd = BM * 128 + (wn * WN + l31) * 128;
  const int sw = (l31 >> 1) & 7;

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // ---- global -> LDS: 16-byte LDS-direct loads.  One wave instruction fills 1 KB of LDS in lane
  // order (8 rows of 128 bytes), so the XOR swizzle is applied on the global side: the lane that
  // fills chunk position c' of row r fetches chunk c' ^ ((r/2)%8) of that row.
  constexpr int NWAVES = WGM * WGN;
  constexpr int A_LOADS = BM / (8 * NWAVES), B_LOADS = BN / (8 * NWAVES);
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "tile vs waves");
  const int lr = lane >> 3;                 // row inside the 8-row group
  const bf16_t* ap[A_LOADS];
  const bf16_t* bp[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int rt = (i * NWAVES + wave) * 8 + lr;           // row inside the tile
    int r = m0 + rt;
    r = r < M ? r : M - 1;
    ap[i] = g.A + (int64_t)r * g.lda + (((lane & 7) ^ ((rt >> 1) & 7)) << 3);
  }
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i) {
    const int rt = (i * NWAVES + wave) * 8 + lr;
    int r = n0 + rt;
    r = r < N ? r : N - 1;
    bp[i] = g.W + (int64_t)r * K + (((lane & 7) ^ ((rt >> 1) & 7)) << 3);
  }
  const int KT = K >> 6;
  issue_slice<A_LOADS, B_LOADS, NWAVES, BM>(ap, bp, 0, smem, wave);
  for (int kt = 0; kt < KT; ++kt) {
    const unsigned char* cur = smem + (kt & 1) * STAGE_BYTES;
    unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of slice kt has landed
    __syncthreads();                                     // ... and everyone's; slice kt-1 fully consumed
    issue_slice<A_LOADS, B_LOADS, NWAVES, BM>(ap, bp, kt + 1 < KT ? kt + 1 : kt, nxt, wave);          // last iteration re-reads slice kt into the idle buffer
    bf16x8 af[2][TM], bfr[2][TN];
    {
      const int coff = ((0 * 2 + lhi) ^ sw) << 4;
#pragma unroll
      for (int i = 0; i < TM; ++i) af[0][i] = *reinterpret_cast<const bf16x8*>(cur + a_rd + i * 32 * 128 + coff);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8*>(cur + b_rd + j * 32 * 128 + coff);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      // MFMAs of k-step ks in source order, with one LDS read of k-step ks+1 issued after each of
      // the first TM+TN of them; scheduling barriers pin this order so that the reads' latency
      // is covered by the MFMAs that follow.
      const int coff = (((ks + 1) * 2 + lhi) ^ sw) << 4;
#pragma unroll
      for (int n = 0; n < TM * TN; ++n) {
        const int i = n / TN, j = n % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
        if (ks < 3) {
#pragma unroll
          for (int q = 2 * n; q < 2 * n + 2 && q < TM + TN; ++q) {   // two reads behind each of the first MFMAs
            if (q == 0) af[(ks + 1) & 1][0] = *reinterpret_cast<const bf16x8*>(cur + a_rd + coff);
            else if (q <= TN) bfr[(ks + 1) & 1][q - 1] = *reinterpret_cast<const bf16x8*>(cur + b_rd + (q - 1) * 32 * 128 + coff);
            else af[(ks + 1) & 1][q - TN] = *reinterpret_cast<const bf16x8*>(cur + a_rd + (q - TN) * 32 * 128 + coff);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");       // the redundant last prefetch must land before LDS is released

  // ---- epilogue.  Accumulator register r of lane l in a 32x32 tile is the element
  //      (row 8*(r/4) + 4*(l/32) + r%4, column l%32).
  const int mw = m0 + wm * WM + 4 * lhi;
  const int nw = n0 + wn * WN;

  if constexpr (EPI == EPI_SWIGLU_BF16) {
    bf16_t* out = static_cast<bf16_t*>(g.out);
    const int n_out = N >> 1;
#pragma unroll
    for (int j = 0; j < TN; j += 2) {
      const int ng = nw + j * 32 + l31, nu = ng + 32;
      const int jo = ((nw + j * 32) >> 1) + l31;
      const float bg = (g.bias && ng < N) ? g.bias[ng] : 0.f;
      const float bu = (g.bias && nu < N) ? g.bias[nu] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = mw + i * 32 + 8 * (r >> 2) + (r & 3);
          if (m < M && jo < n_out)
            out[(int64_t)m * g.ldo + jo] = (bf16_t)f2bf(silu_f(acc[i][j][r] + bg) * (acc[i][j + 1][r] + bu));
        }
    }
  } else if constexpr (EPI == EPI_QKV) {
    bf16_t* out = static_cast<bf16_t*>(g.out);
    const int half = g.head_dim >> 1;
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int nt0 = nw + j * 32;        // first column of this 32-wide tile (uniform in the wave)
      const int n = nt0 + l31;
      const float b = (g.bias && n < N) ? g.bias[n] : 0.f;
      if (nt0 >= 2 * g.hidden) {          // v: transposed store, 4 consecutive tokens per lane
        const int d = n - 2 * g.hidden;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int m = mw + i * 32 + 8 * q;
            if (m < M && n < N) {
              uint2 pk;
              pk.x = f2bf(acc[i][j][4 * q + 0] + b) | (f2bf(acc[i][j][4 * q + 1] + b) << 16);
              pk.y = f2bf(acc[i][j][4 * q + 2] + b) | (f2bf(acc[i][j][4 * q + 3] + b) << 16);
              *reinterpret_cast<uint2*>(g.vt + (int64_t)d * g.ld_vt + m) = pk;
            }
          }
      } else {                            // q or k: rotary on neighbouring columns (2j, 2j+1)
        const bool is_q = nt0 < g.hidden;
        const int pj = ((n % g.hidden) % g.head_dim) >> 1;
        const float sc = is_q ? g.q_scale : 1.0f;
        const bool odd = lane & 1;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const int m = mw + i * 32 + 8 * (r >> 2) + (r & 3);
            const int mc = m < M ? m : M - 1;
            float v = acc[i][j][r] + b;
            if (g.rope_cos) {
              const float c = g.rope_cos[(int64_t)mc * half + pj], s = g.rope_sin[(int64_t)mc * half + pj];
              const float o = lane_xor1(v);
              v = odd ? v * c + o * s : v * c - o * s;
            }
            if (m < M && n < N) out[(int64_t)m * g.ldo + n] = (bf16_t)f2bf(v * sc);
          }
      }
    }
  } else {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int n = nw + j * 32 + l31;
      const float b = (g.bias && n < N) ? g.bias[n] : 0.f;
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int m = mw + i * 32 + 8 * (r >> 2) + (r & 3);
          if (m >= M || n >= N) continue;
          int64_t row = m;
          if (g.row_map) {
            row = g.row_map[m];
            if (row < 0) continue;
          }
          float v = acc[i][j][r] + b;
          if constexpr (EPI == EPI_GELU_BF16 || EPI == EPI_GELU_F32) v = gelu_erf(v);
          if constexpr (EPI == EPI_BF16 || EPI == EPI_GELU_BF16) {
            static_cast<bf16_t*>(g.out)[row * g.ldo + n] = (bf16_t)f2bf(v);
          } else if constexpr (EPI == EPI_RESADD_F32) {
            float* p = static_cast<float*>(g.out) + row * g.ldo + n;
            *p = *p + v;
          } else {
            static_cast<float*>(g.out)[row * g.ldo + n] = v;
          }
        }
    }
  }
}

template <int BM, int BN, int WGM, int WGN, int EPI>
static cs_status launch_cfg(const GemmArgs& g, hipStream_t stream) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int LDS = 2 * (BM + BN) * 128;
  auto kern = gemm_kernel<BM, BN, WGM, WGN, EPI>;
  static bool attr_set = false;  // one attribute call per instantiation
  if (!attr_set) {
    CS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS));
    attr_set = true;
  }
  const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  hipLaunchKernelGGL(kern, dim3(tiles), dim3(NT), LDS, stream, g);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

template <int EPI>
static cs_status launch_epi(const GemmArgs& g, hipStream_t stream) {
  // Tile choice: 256x256 when that still gives every CU work twice over, else 128x128-ish.
  const int64_t big = (int64_t)((g.M + 255) / 256) * ((g.N + 255) / 256);
  if (big >= 384) return launch_cfg<256, 256, 2, 4, EPI>(g, stream);
  return launch_cfg<128, 128, 2, 2, EPI>(g, stream);
}

cs_status launch_gemm(int epilogue, const GemmArgs& g, hipStream_t stream) {
  if (g.M <= 0 || g.N <= 0) return CS_OK;
  if (g.K <= 0 || (g.K & 63)) return fail(CS_ERR_UNSUPPORTED, "gemm: K must be a positive multiple of 64");
  // lda < K is allowed: rows may overlap (a k=3 convolution reads three consecutive frames per row)
  if ((g.lda & 7) || (reinterpret_cast<uintptr_t>(g.A) & 15) || (reinterpret_cast<uintptr_t>(g.W) & 15))
    return fail(CS_ERR_INVALID_ARG, "gemm: A and W rows must be 16-byte aligned");
  switch (epilogue) {
    case EPI_BF16: return launch_epi<EPI_BF16>(g, stream);
    case EPI_F32: return launch_epi<EPI_F32>(g, stream);
    case EPI_GELU_BF16: return launch_epi<EPI_GELU_BF16>(g, stream);
    case EPI_GELU_F32: return launch_epi<EPI_GELU_F32>(g, stream);
    case EPI_RESADD_F32: return launch_epi<EPI_RESADD_F32>(g, stream);
    case EPI_SWIGLU_BF16:
      if (g.N & 63) return fail(CS_ERR_UNSUPPORTED, "gemm: swiglu needs N % 64 == 0");
      return launch_epi<EPI_SWIGLU_BF16>(g, stream);
    case EPI_QKV:
      if ((g.M & 3) || (g.hidden & 31) || (g.head_dim & 1) || g.N != 3 * g.hidden)
        return fail(CS_ERR_UNSUPPORTED, "gemm: qkv epilogue needs M % 4 == 0, hidden % 32 == 0, N == 3 hidden");
      return launch_epi<EPI_QKV>(g, stream);
    default: return fail(CS_ERR_INVALID_ARG, "gemm: unknown epilogue");
  }
}

}  // namespace cs
