// bf16 MFMA GEMM for gfx950:  C = epilogue(A W^T), A [M,K] and W [N,K] both K-contiguous.
//
// One workgroup owns a BM x BN tile of C and walks K in slices of 64.  Each slice of A and W is
// brought into LDS with 16-byte LDS-direct loads (no staging registers, no LDS store
// instructions), double-buffered: the loads of slice k+1 are issued one by one between the MFMAs
// of the first half of slice k and have the rest of that slice to land.
//
// LDS layout: rows of 128 bytes (64 bf16), the 16-byte chunk at position c of row r holds chunk
// c ^ ((r/2) % 8) of that row.  Measured on gfx950, ds_read_b128 serves 16 lanes per pass and the
// lanes of a pass are not consecutive (rows {0-3,12-15,20-23,24-27} of a 32-row operand read share
// one); this XOR is conflict-free for the operand reads, a plain row%8 XOR is 2-way conflicted.
// An LDS-direct load writes 64 lanes x 16 bytes in lane order, so the XOR is applied to the global
// address each lane fetches.
//
// Waves are laid out WGM x WGN over the tile; a wave accumulates (BM/WGM) x (BN/WGN) in fp32 with
// v_mfma_f32_32x32x16_bf16.  The products are formed transposed (W rows as the first operand), so
// that a lane owns one row m of C and its 16 accumulator registers of a 32x32 block walk the
// columns in groups of four consecutive n: bias, activations, rotary pairs and 8/16-byte stores
// all work on registers of one lane.  Inside a K slice the LDS reads of k-step s+1 are issued
// behind the first MFMAs of k-step s and scheduling barriers pin that order.
#include "common.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_void;

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
// four floats -> four bf16 (v_cvt_pk_bf16_f32, round to nearest even), as 8 bytes
__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d) {
  const f32x4 v = {a, b, c, d};
  const bf16x4 h = __builtin_convertvector(v, bf16x4);
  return __builtin_bit_cast(u32x2, h);
}
__device__ __forceinline__ float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752f)); }
__device__ __forceinline__ float silu_f(float z) { return z / (1.0f + __expf(-z)); }

// Issues the LDS-direct loads of one 64-wide K slice: every wave instruction moves 64 x 16 bytes
// from the lanes' global addresses to 1 KB of LDS starting at a wave-uniform address, in lane order.
template <int A_LOADS, int B_LOADS, int NWAVES, int BM>
__device__ __forceinline__ void issue_slice(const bf16_t* const* ap, const bf16_t* const* bp, int kt,
                                            unsigned char* stage, int wave) {
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i)
    __builtin_amdgcn_global_load_lds(ap[i] + kt * 64, (lds_void*)(uintptr_t)(stage + (i * NWAVES + wave) * 1024), 16, 0, 0);
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i)
    __builtin_amdgcn_global_load_lds(bp[i] + kt * 64, (lds_void*)(uintptr_t)(stage + BM * 128 + (i * NWAVES + wave) * 1024), 16, 0, 0);
}

// One of the A_LOADS + B_LOADS loads of a slice, by index.
template <int A_LOADS, int B_LOADS, int NWAVES, int BM>
__device__ __forceinline__ void issue_one(const bf16_t* const* ap, const bf16_t* const* bp, int l, int kt,
                                          unsigned char* stage, int wave) {
  if (l < A_LOADS)
    __builtin_amdgcn_global_load_lds(ap[l] + kt * 64, (lds_void*)(uintptr_t)(stage + (l * NWAVES + wave) * 1024), 16, 0, 0);
  else
    __builtin_amdgcn_global_load_lds(bp[l - A_LOADS] + kt * 64,
                                     (lds_void*)(uintptr_t)(stage + BM * 128 + ((l - A_LOADS) * NWAVES + wave) * 1024), 16, 0, 0);
}

// The K loop.  W_FIRST: accumulate C^T blocks (lane = row m, registers = columns n); otherwise
// C blocks (lane = column n, registers = rows m).
template <int BM, int BN, int WGM, int WGN, bool W_FIRST>
__device__ __forceinline__ void main_loop(const GemmArgs& g, unsigned char* smem, int m0, int n0,
                                          f32x16 (&acc)[BM / WGM / 32][BN / WGN / 32]) {
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  constexpr int STAGE_BYTES = (BM + BN) * 128;
  constexpr int NWAVES = WGM * WGN;
  constexpr int A_LOADS = BM / (8 * NWAVES), B_LOADS = BN / (8 * NWAVES);
  static_assert(BM % (8 * NWAVES) == 0 && BN % (8 * NWAVES) == 0, "tile vs waves");
  constexpr int RD_PER = 2;  // LDS reads of the next k-step issued behind each of the first MFMAs
  constexpr int SPREAD_KS = 2;  // k-steps over which the next slice's loads are spread (2 measured best of 1..4)
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int M = g.M, N = g.N, K = g.K;
  const int l31 = lane & 31, lhi = lane >> 5;
  const int a_rd = (wm * WM + l31) * 128;
  const int b_rd = BM * 128 + (wn * WN + l31) * 128;
  const int sw = (l31 >> 1) & 7;

#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int lr = lane >> 3;  // row inside an 8-row group
  const bf16_t* ap[A_LOADS];
  const bf16_t* bp[B_LOADS];
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i) {
    const int rt = (i * NWAVES + wave) * 8 + lr;  // row inside the tile
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
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's part of slice kt has landed
    __syncthreads();                                    // ... and everyone's; slice kt-1 fully consumed
    // The loads of slice kt+1 go out one at a time between the MFMAs of the first k-steps: issued
    // in one burst behind the barrier they queue in the texture-address unit (16 clocks each, all
    // waves at once) and every wave sits in the issue stall instead of feeding the MFMA pipe.
    // The last iteration re-reads slice kt into the idle buffer: no branch around the loads.
    const int kn = kt + 1 < KT ? kt + 1 : kt;
    bf16x8 af[2][TM], bfr[2][TN];
    {
      const int coff = (lhi ^ sw) << 4;
#pragma unroll
      for (int i = 0; i < TM; ++i) af[0][i] = *reinterpret_cast<const bf16x8*>(cur + a_rd + i * 32 * 128 + coff);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[0][j] = *reinterpret_cast<const bf16x8*>(cur + b_rd + j * 32 * 128 + coff);
    }
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      // MFMAs of k-step ks in source order, two LDS reads of k-step ks+1 behind each of the first
      // ones; the scheduling barriers keep the compiler from regrouping them, so the reads'
      // latency is covered by the MFMAs that follow.
      const int coff = (((ks + 1) * 2 + lhi) ^ sw) << 4;
#pragma unroll
      for (int n = 0; n < TM * TN; ++n) {
        const int i = n / TN, j = n % TN;
        if (W_FIRST)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
        else
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
        if (ks < SPREAD_KS) {
          constexpr int LT = A_LOADS + B_LOADS, SLOTS = SPREAD_KS * TM * TN;
#pragma unroll
          for (int l = 0; l < LT; ++l)
            if (l * SLOTS / LT == ks * TM * TN + n) issue_one<A_LOADS, B_LOADS, NWAVES, BM>(ap, bp, l, kn, nxt, wave);
        }
        if (ks < 3) {
#pragma unroll
          for (int q = RD_PER * n; q < RD_PER * n + RD_PER && q < TM + TN; ++q) {
            if (q == 0) af[(ks + 1) & 1][0] = *reinterpret_cast<const bf16x8*>(cur + a_rd + coff);
            else if (q <= TN) bfr[(ks + 1) & 1][q - 1] = *reinterpret_cast<const bf16x8*>(cur + b_rd + (q - 1) * 32 * 128 + coff);
            else af[(ks + 1) & 1][q - TN] = *reinterpret_cast<const bf16x8*>(cur + a_rd + (q - TN) * 32 * 128 + coff);
          }
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the redundant last prefetch lands before LDS is released
}

template <int BM, int BN, int WGM, int WGN, int EPI>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_kernel(GemmArgs g) {
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = WN / 32;
  static_assert(EPI != EPI_SWIGLU_BF16 || (TN % 2 == 0), "gate/up pairs need an even number of column tiles");

  extern __shared__ __align__(16) unsigned char smem[];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int M = g.M, N = g.N;
  const int l31 = lane & 31, lhi = lane >> 5;

  // workgroup -> tile.  Consecutive workgroups land on different XCDs (b % 8), each with its own
  // L2, so every XCD gets a contiguous range of tile ids; ids walk the tile grid in bands of GROUP_M
  // tile rows, row index fastest, so the ~32 tiles an XCD runs at a time form a GROUP_M x 8 block
  // that shares GROUP_M slices of A and 8 slices of W per k-step (an L2 miss on every W byte
  // otherwise: measured 427 clocks average L2 read latency and the L1 miss queue full 58 % of the time).
  constexpr int GROUP_M = 4;
  const int tiles_n = (N + BN - 1) / BN, tiles_m = (M + BM - 1) / BM;
  const int nb = gridDim.x;
  int bid = blockIdx.x;
  {
    const int xcd = bid & 7, idx = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    bid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  const int band = bid / (GROUP_M * tiles_n), in_band = bid - band * (GROUP_M * tiles_n);
  const int band_rows = tiles_m - band * GROUP_M < GROUP_M ? tiles_m - band * GROUP_M : GROUP_M;
  const int m0 = (band * GROUP_M + in_band % band_rows) * BM, n0 = (in_band / band_rows) * BN;

  f32x16 acc[TM][TN];

  if constexpr (EPI == EPI_QKV) {
    if (n0 >= 2 * g.hidden) {
      // v columns (the whole workgroup: 2*hidden is a multiple of BN).  Untransposed blocks: lane =
      // column n = one v dimension, registers = rows, four consecutive tokens per register group,
      // stored as 8 bytes into the transposed v buffer.
      main_loop<BM, BN, WGM, WGN, false>(g, smem, m0, n0, acc);
      const int mw = m0 + wm * WM + 4 * lhi;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int n = n0 + wn * WN + j * 32 + l31;
        if (n >= N) continue;
        const float b = g.bias ? g.bias[n] : 0.f;
        bf16_t* dst = g.vt + (int64_t)(n - 2 * g.hidden) * g.ld_vt;
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int m = mw + i * 32 + 8 * q;
            if (m < M)
              *reinterpret_cast<u32x2*>(dst + m) = pack4(acc[i][j][4 * q] + b, acc[i][j][4 * q + 1] + b,
                                                         acc[i][j][4 * q + 2] + b, acc[i][j][4 * q + 3] + b);
          }
      }
      return;
    }
  }

  main_loop<BM, BN, WGM, WGN, true>(g, smem, m0, n0, acc);

  // QKV: the (cos, sin) rows of this tile's BM tokens are staged in LDS (free after the K loop)
  // with coalesced 16-byte loads; read per lane from global they are 16-byte pieces of 32 different
  // rows per instruction, which cost 18 us of a 110 us launch.
  [[maybe_unused]] int rope_stride = 0;
  if constexpr (EPI == EPI_QKV) {
    if (g.rope_cs) {
      const int half = g.head_dim >> 1;
      const int cpr = half >> 1;                       // 16-byte chunks per token row (two pairs each)
      rope_stride = (cpr * 16 + 16) | 16;              // padded so that rows spread over the LDS banks
      const int64_t last = (int64_t)M * cpr - 1;
      __syncthreads();                                 // every wave is done reading the last K slice
      for (int c = threadIdx.x; c < BM * cpr; c += 64 * WGM * WGN) {
        int64_t src = (int64_t)m0 * cpr + c;
        src = src < last ? src : last;
        const f32x4 v = reinterpret_cast<const f32x4*>(g.rope_cs)[src];
        *reinterpret_cast<f32x4*>(smem + (c / cpr) * rope_stride + (c % cpr) * 16) = v;
      }
      __syncthreads();
    }
  }

  // ---- epilogue.  Register 4q+e of lane l in block (i,j) is the element
  //      (row m = i*32 + l%32, column n = j*32 + 8q + 4*(l/32) + e).
  const int nw = n0 + wn * WN + 4 * lhi;
  // QKV: byte offset of the first (cos, sin) pair of every 4-column group, once per lane (the
  // divisions by run-time sizes must not be redone for every row block)
  [[maybe_unused]] int rope_off[TN][4];
  if constexpr (EPI == EPI_QKV) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = nw + j * 32 + 8 * q;
        rope_off[j][q] = ((((n < g.hidden ? n : n - g.hidden)) % g.head_dim) >> 1) * 8;
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int m = m0 + wm * WM + i * 32 + l31;
    if (m >= M) continue;
    int64_t row = m;
    if (g.row_map) {
      row = g.row_map[m];
      if (row < 0) continue;
    }
    if constexpr (EPI == EPI_SWIGLU_BF16) {
      bf16_t* orow = static_cast<bf16_t*>(g.out) + row * g.ldo;
#pragma unroll
      for (int j = 0; j < TN; j += 2)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int ng = nw + j * 32 + 8 * q;         // gate columns ng..ng+3, up columns 32 further
          if (ng + 36 > N) continue;
          f32x4 bg = {0.f, 0.f, 0.f, 0.f}, bu = {0.f, 0.f, 0.f, 0.f};
          if (g.bias) {
            bg = *reinterpret_cast<const f32x4*>(g.bias + ng);
            bu = *reinterpret_cast<const f32x4*>(g.bias + ng + 32);
          }
          float o[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) o[e] = silu_f(acc[i][j][4 * q + e] + bg[e]) * (acc[i][j + 1][4 * q + e] + bu[e]);
          const int jo = ((n0 + wn * WN + j * 32) >> 1) + 4 * lhi + 8 * q;
          *reinterpret_cast<u32x2*>(orow + jo) = pack4(o[0], o[1], o[2], o[3]);
        }
    } else if constexpr (EPI == EPI_QKV) {
      // q and k columns: rotary on neighbouring columns (2p, 2p+1), both held by this lane
      bf16_t* orow = static_cast<bf16_t*>(g.out) + row * g.ldo;
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = nw + j * 32 + 8 * q;
          if (n >= N) continue;
          f32x4 b = {0.f, 0.f, 0.f, 0.f};
          if (g.bias) b = *reinterpret_cast<const f32x4*>(g.bias + n);
          float v0 = acc[i][j][4 * q] + b[0], v1 = acc[i][j][4 * q + 1] + b[1];
          float v2 = acc[i][j][4 * q + 2] + b[2], v3 = acc[i][j][4 * q + 3] + b[3];
          if (g.rope_cs) {
            const f32x4 cs = *reinterpret_cast<const f32x4*>(smem + (m - m0) * rope_stride + rope_off[j][q]);  // cos,sin,cos,sin
            const float r0 = v0 * cs[0] - v1 * cs[1], r1 = v1 * cs[0] + v0 * cs[1];
            const float r2 = v2 * cs[2] - v3 * cs[3], r3 = v3 * cs[2] + v2 * cs[3];
            v0 = r0; v1 = r1; v2 = r2; v3 = r3;
          }
          const float sc = n < g.hidden ? g.q_scale : 1.0f;
          *reinterpret_cast<u32x2*>(orow + n) = pack4(v0 * sc, v1 * sc, v2 * sc, v3 * sc);
        }
    } else {
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const int n = nw + j * 32 + 8 * q;
          if (n >= N) continue;
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][4 * q + e];
          if (g.bias) v += *reinterpret_cast<const f32x4*>(g.bias + n);
          if constexpr (EPI == EPI_GELU_BF16 || EPI == EPI_GELU_F32 || EPI == EPI_GELU_SPLIT) {
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = gelu_erf(v[e]);
          }
          if constexpr (EPI == EPI_GELU_SPLIT) {
            bf16_t* o = static_cast<bf16_t*>(g.out) + row * g.ldo + n;
            const u32x2 hi = pack4(v[0], v[1], v[2], v[3]);
            *reinterpret_cast<u32x2*>(o) = hi;
            *reinterpret_cast<u32x2*>(o + N) = pack4(v[0] - __uint_as_float(hi.x << 16), v[1] - __uint_as_float(hi.x & 0xFFFF0000u),
                                                     v[2] - __uint_as_float(hi.y << 16), v[3] - __uint_as_float(hi.y & 0xFFFF0000u));
          } else if constexpr (EPI == EPI_BF16 || EPI == EPI_GELU_BF16) {
            *reinterpret_cast<u32x2*>(static_cast<bf16_t*>(g.out) + row * g.ldo + n) = pack4(v[0], v[1], v[2], v[3]);
          } else if constexpr (EPI == EPI_RESADD_F32) {
            f32x4* p = reinterpret_cast<f32x4*>(static_cast<float*>(g.out) + row * g.ldo + n);
            *p = *p + v;
          } else {
            *reinterpret_cast<f32x4*>(static_cast<float*>(g.out) + row * g.ldo + n) = v;
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
  // Tile choice by the number of workgroups it yields for the 256 CUs.
  const int64_t tm = (g.M + 255) / 256;
  const int64_t big = tm * ((g.N + 255) / 256);
  const bool big_ok = EPI != EPI_QKV || (2 * g.hidden) % 256 == 0;
  if (big >= 384 && big_ok) return launch_cfg<256, 256, 2, 4, EPI>(g, stream);
  if constexpr (EPI != EPI_QKV && EPI != EPI_SWIGLU_BF16) {
    // narrow outputs (N = hidden = 1280): 256 x 160 tiles, four waves of 64 x 160, give M/256 * 8
    // workgroups, one round of the chip at M = 8192
    if (g.N % 160 == 0 && tm * (g.N / 160) >= 192) return launch_cfg<256, 160, 4, 1, EPI>(g, stream);
  }
  return launch_cfg<128, 128, 2, 2, EPI>(g, stream);
}

cs_status launch_gemm(int epilogue, const GemmArgs& g, hipStream_t stream) {
  if (g.M <= 0 || g.N <= 0) return CS_OK;
  if (g.K <= 0 || (g.K & 63)) return fail(CS_ERR_UNSUPPORTED, "gemm: K must be a positive multiple of 64");
  // lda < K is allowed: rows may overlap (a k=3 convolution reads three consecutive frames per row)
  if ((g.lda & 7) || (reinterpret_cast<uintptr_t>(g.A) & 15) || (reinterpret_cast<uintptr_t>(g.W) & 15))
    return fail(CS_ERR_INVALID_ARG, "gemm: A and W rows must be 16-byte aligned");
  if ((g.N & 3) || (g.ldo & 3) || (reinterpret_cast<uintptr_t>(g.out) & 15) || (reinterpret_cast<uintptr_t>(g.bias) & 15))
    return fail(CS_ERR_UNSUPPORTED, "gemm: N and the output row stride must be multiples of 4, out and bias 16-byte aligned");
  switch (epilogue) {
    case EPI_BF16: return launch_epi<EPI_BF16>(g, stream);
    case EPI_F32: return launch_epi<EPI_F32>(g, stream);
    case EPI_GELU_BF16: return launch_epi<EPI_GELU_BF16>(g, stream);
    case EPI_GELU_F32: return launch_epi<EPI_GELU_F32>(g, stream);
    case EPI_GELU_SPLIT: return launch_epi<EPI_GELU_SPLIT>(g, stream);
    case EPI_RESADD_F32: return launch_epi<EPI_RESADD_F32>(g, stream);
    case EPI_SWIGLU_BF16:
      if (g.N & 63) return fail(CS_ERR_UNSUPPORTED, "gemm: swiglu needs N % 64 == 0");
      return launch_epi<EPI_SWIGLU_BF16>(g, stream);
    case EPI_QKV:
      if ((g.M & 3) || (g.hidden & 63) || (g.head_dim & 3) || g.N != 3 * g.hidden || (g.ld_vt & 3) ||
          (reinterpret_cast<uintptr_t>(g.vt) & 7))
        return fail(CS_ERR_UNSUPPORTED, "gemm: qkv epilogue needs M % 4 == 0, hidden % 64 == 0, head_dim % 4 == 0, N == 3 hidden");
      return launch_epi<EPI_QKV>(g, stream);
    default: return fail(CS_ERR_INVALID_ARG, "gemm: unknown epilogue");
  }
}

}  // namespace cs
