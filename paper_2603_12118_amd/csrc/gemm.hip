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
#include <stdio.h>
#include <stdlib.h>

#include <atomic>

#include "common.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
typedef __attribute__((address_space(3))) void lds_void;

typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

// The MFMA shape (build-time switch for measurement: -DCS_GEMM_MFMA16=0 gives v_mfma_f32_32x32x16_bf16).
// Both do 1024 FLOP per SIMD and clock; on random operands at the board's power limit a bare loop of
// 16x16x32 sustains about 12 % more (see cs_mfma_ceiling and the measurement notes).
#ifndef CS_GEMM_MFMA16
#define CS_GEMM_MFMA16 1
#endif
// The 16x16x32 shape is used by the eight-wave tiles (two waves per SIMD).  With one wave per SIMD (the
// four-wave tiles) it is slower: every other instruction of the wave delays an MFMA of 16 clocks more
// than one of 32 (measured: down projection 67 -> 106 us).
// (The four-wave 128 x 160 tile is launched only where two of its workgroups share a CU, which again makes two
// waves per SIMD.)
template <int NWAVES, int BM = 256, int BN = 256>
constexpr bool use_mfma16() { return CS_GEMM_MFMA16 != 0 && (NWAVES >= 8 || (BM == 128 && BN == 160)); }

// A wave's accumulators are kept per 32 x 32 block of C^T (or C), 16 registers per lane = 4 groups q of
// 4 consecutive columns of one row.  Which row and columns a lane's group q holds depends on the MFMA:
//   32x32x16: one block per MFMA;      row lane % 32,                columns 8q + 4 (lane / 32) ...
//   16x16x32: four MFMAs per block;    row 16 (q / 2) + lane % 16,   columns 16 (q % 2) + 4 (lane / 16) ...
// ("row" is the second operand's index, "column" the first operand's.)
template <bool MFMA16>
__device__ __forceinline__ int blk_row(int q, int lane) { return MFMA16 ? 16 * (q >> 1) + (lane & 15) : (lane & 31); }
template <bool MFMA16>
__device__ __forceinline__ int blk_col(int q, int lane) { return MFMA16 ? 16 * (q & 1) + 4 * (lane >> 4) : 8 * q + 4 * (lane >> 5); }
// four floats -> four bf16 (v_cvt_pk_bf16_f32, round to nearest even), as 8 bytes
__device__ __forceinline__ u32x2 pack4(float a, float b, float c, float d) {
  const f32x4 v = {a, b, c, d};
  const bf16x4 h = __builtin_convertvector(v, bf16x4);
  return __builtin_bit_cast(u32x2, h);
}
// z * sigmoid(z) with the hardware exp2 and reciprocal (1 ulp each): five instructions, where the
// IEEE division costs a dozen, and this runs for every element of the widest GEMM's epilogue
__device__ __forceinline__ float silu_f(float z) {
  return z * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(-1.4426950408889634f * z));
}

// ---- epilogue through LDS.  A lane of an accumulator block owns one row and 4-column groups of
// it, so storing from registers writes 16-byte pieces of 32 different rows per instruction: measured,
// that way the stores cost a quarter of a K = 1280 launch.  Instead every wave passes its blocks
// through a private 32-row LDS chunk and writes them out as whole 64- or 128-byte row segments,
// 16 bytes per lane.  LDS serves one wave's instructions in order, so no wait is needed between a
// chunk's writes and reads beyond keeping the compiler from reordering them.
// What a tile may use behind its two stage buffers: 1 KB of per-column values, then the waves' per-row partial
// sums of a folded normalisation, [2][WGN][BM] floats (sums of squares, plain sums).  (The 128 x 160 tiles, of
// which the four-wave one must fit a CU twice, have 128 rows and two waves along N: 2 KB of sums.)
constexpr int EXTRA_LDS_BYTES = 1024 + 2 * 4 * 256 * 4;
constexpr int EXTRA_LDS_BYTES_PAIR = 1024 + 4 * 256 * 4;
// (Build-time switch for measurement: -DCS_GEMM_NARROW_STAGES=3 gives the eight-wave 256 x 160 tile of the plain
// residual epilogue a third stage buffer, see stages(); what is left of 160 KB then holds exactly its column
// values and one set of sums.  Measured on one box, alternated: slower, down projection 885 -> 816 TFLOP/s, the
// 8-image step 11.72 -> 12.02 ms, the 16 384-token step 26.35 -> 26.6 ms.)
#ifndef CS_GEMM_NARROW_STAGES
#define CS_GEMM_NARROW_STAGES 2
#endif
template <int BM, int BN, int NWAVES, int EPI>
constexpr bool third_stage() { return CS_GEMM_NARROW_STAGES == 3 && BM == 256 && BN == 160 && NWAVES == 8 && EPI == EPI_RESADD_F32; }
template <int BM, int BN, int NWAVES = 0, int EPI = -1>
constexpr int extra_lds_bytes() {
  return third_stage<BM, BN, NWAVES, EPI>() ? 1024 + 2 * 256 * 4 : BM == 128 && BN == 160 ? EXTRA_LDS_BYTES_PAIR : EXTRA_LDS_BYTES;
}
// Stage buffers of the K loop.  Two everywhere (a slice's MFMAs cover the next slice's loads where the tile is
// large, and more would not fit) except on the eight-wave 128 x 160 tile, which runs one workgroup per CU in
// launches that do not fill the chip: its slice of MFMAs is much shorter than the loads' latency, so it keeps
// CS_GEMM_SMALL_STAGES - 1 slices in flight, four stages being what 160 KB of LDS hold (build-time switch for
// measurement: 2 is the plain double buffer.  Measured on one box, 3072 tokens, 2 / 3 / 4 stages: out projection
// 31.4 / 32.1 / 28.5 us, down projection 60.3 / 61.8 / 52.0 us, the step 6.78 / 6.85 / 6.40 ms).
#ifndef CS_GEMM_SMALL_STAGES
#define CS_GEMM_SMALL_STAGES 4
#endif
template <int BM, int BN, int NWAVES, int EPI>
constexpr int stages() { return BM == 128 && BN == 160 && NWAVES == 8 ? CS_GEMM_SMALL_STAGES : third_stage<BM, BN, NWAVES, EPI>() ? 3 : 2; }
template <int BM, int BN, int NWAVES, int EPI>
constexpr int tile_lds_bytes() { return stages<BM, BN, NWAVES, EPI>() * (BM + BN) * 128 + extra_lds_bytes<BM, BN, NWAVES, EPI>(); }
constexpr int CHUNK_STRIDE = 144;               // bytes between chunk rows: 128 of data + 16 of padding
constexpr int CHUNK_BYTES_ = 32 * CHUNK_STRIDE;
// The 64-row tiles of a ragged last tile row run behind the full tiles, eight of them or so on an otherwise idle
// chip, each alone on its CU with next to no MFMA work per slice: their K loop goes at the pace of the loads
// (measured on 8224 x 1024 x 4096: the 32 extra rows cost 29 us on top of 65, 0.45 us per slice).  With eight
// waves they take as many stage buffers, up to four, as 160 KB of LDS hold (CS_GEMM_LIGHT_STAGES=2 at build time:
// two): 21 us, 0.33 us per slice, which is 75 GB/s, about what one CU draws; the 8-tile class-token step 9.82 ->
// 9.51 ms.
#ifndef CS_GEMM_LIGHT_STAGES
#define CS_GEMM_LIGHT_STAGES 4
#endif
template <int BN, int NWAVES, int EPI>
constexpr int light_lds_need(int st) {
  const int stage = (64 + BN) * 128, chunks = NWAVES * CHUNK_BYTES_;
  return st * stage + extra_lds_bytes<64, BN, NWAVES, EPI>() + (chunks > stage ? chunks : 0);
}
template <int BN, int NWAVES, int EPI>
constexpr int light_stages() {
  if (NWAVES != 8) return 2;
  for (int st = CS_GEMM_LIGHT_STAGES; st > 2; --st)
    if (light_lds_need<BN, NWAVES, EPI>(st) <= 160 * 1024) return st;
  return 2;
}
constexpr int CHUNK_BYTES = 32 * CHUNK_STRIDE;

// v[b][q] holds columns b*32 + blk_col(q) .. +3 of row blk_row(q) of a 32 x (NB*32) block.
// The block's element (r, c) goes to out[rowmap(row0 + r) * ld + col0 + c] for row0 + r < row_end,
// col0 + c < col_end (col_end - col0 a multiple of 4); ACCUM adds to what is there (fp32 only).
// Producer side of a folded RMSNorm: what the residual epilogue writes beside the updated stream.
struct NormFold {
  bf16_t* xg;             // [*, ld_xg] bf16(x_new * gain)
  int64_t ld_xg;
  const float* gain_lds;  // gain of the tile's columns, staged in LDS; index = column - n0
  int n0;
  float ssacc[4];         // this lane's sums of x_new^2, one per 8-row group of the 32-row block
  float s1acc[4];         // ... and of x_new (a LayerNorm needs the mean too)
};

template <int NB, typename T, bool ACCUM, bool MFMA16, bool SUMS = false>
__device__ __forceinline__ void store_block(unsigned char* chunk, const f32x4 (&v)[NB][4], T* out, int64_t ld,
                                            const int32_t* row_map, int row0, int row_end, int col0, int col_end,
                                            bool wide, bool wt, const f32x4* held = nullptr, NormFold* fold = nullptr) {
  constexpr int ES = (int)sizeof(T);
  static_assert(NB * 32 * ES <= 128, "a chunk row holds 128 bytes");
  static_assert(!ACCUM || ES == 4, "accumulation is for fp32 outputs");
  const int lane = threadIdx.x & 63;
  asm volatile("" ::: "memory");
#pragma unroll
  for (int b = 0; b < NB; ++b)
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      unsigned char* p = chunk + blk_row<MFMA16>(q, lane) * CHUNK_STRIDE + (b * 32 + blk_col<MFMA16>(q, lane)) * ES;
      if constexpr (ES == 2) *reinterpret_cast<u32x2*>(p) = pack4(v[b][q][0], v[b][q][1], v[b][q][2], v[b][q][3]);
      else *reinterpret_cast<f32x4*>(p) = v[b][q];
    }
  asm volatile("" ::: "memory");
  constexpr int LPR = NB * 32 * ES / 16;          // lanes per row
  constexpr int RPI = 64 / LPR;                   // rows per instruction
  constexpr int EPL = 16 / ES;                    // elements per lane
#pragma unroll
  for (int it = 0; it < 32 / RPI; ++it) {
    const int r = it * RPI + lane / LPR, c = (lane % LPR) * EPL;
    const f32x4 piece = *reinterpret_cast<const f32x4*>(chunk + r * CHUNK_STRIDE + (lane % LPR) * 16);
    const int m = row0 + r, n = col0 + c;
    if (m >= row_end || n >= col_end) continue;
    int64_t row = m;
    if (row_map) {
      row = row_map[m];
      if (row < 0) continue;
    }
    T* dst = out + row * ld + n;
    if constexpr (ES == 4) {
      f32x4* d4 = reinterpret_cast<f32x4*>(dst);
      if constexpr (ACCUM) {
        const f32x4 nx = (held ? held[it] : *d4) + piece;
        store16(d4, nx, wt);
        if constexpr (NB == 1) {
          if (fold) {
            const f32x4 gg = *reinterpret_cast<const f32x4*>(fold->gain_lds + (n - fold->n0));
            *reinterpret_cast<u32x2*>(fold->xg + row * fold->ld_xg + n) = pack4(nx[0] * gg[0], nx[1] * gg[1], nx[2] * gg[2], nx[3] * gg[3]);
            fold->ssacc[it] += (nx[0] * nx[0] + nx[1] * nx[1]) + (nx[2] * nx[2] + nx[3] * nx[3]);
            if constexpr (SUMS) fold->s1acc[it] += (nx[0] + nx[1]) + (nx[2] + nx[3]);
          }
        }
      } else {
        store16(d4, piece, wt);
      }
    } else {
      if (wide && n + 8 <= col_end) {
        store16(dst, piece, wt);
      } else {
        const f32x2 lo = {piece[0], piece[1]}, hi = {piece[2], piece[3]};
        *reinterpret_cast<f32x2*>(dst) = lo;
        if (n + 8 <= col_end) *reinterpret_cast<f32x2*>(dst + 4) = hi;
      }
    }
  }
  asm volatile("" ::: "memory");
}

// Cache-policy bits of the operand loads (build-time switches for measurement: -DCS_GEMM_W_AUX=2 marks the
// W loads non-temporal, 1 = sc0, 16 = sc1; likewise CS_GEMM_A_AUX for the A loads).
#ifndef CS_GEMM_W_AUX
#define CS_GEMM_W_AUX 0
#endif
#ifndef CS_GEMM_RESADD_WT     // 1: the residual-add epilogue stores write-through like the others
#define CS_GEMM_RESADD_WT 1
#endif
#ifndef CS_GEMM_A_AUX
#define CS_GEMM_A_AUX 0
#endif

// Issues the LDS-direct loads of one 64-wide K slice: every wave instruction moves 64 x 16 bytes
// from the lanes' global addresses to 1 KB of LDS starting at a wave-uniform address, in lane order.
// (A wave whose share of the W rows lies beyond the tile, where BN is not a multiple of 8 rows per wave,
// skips that load: wave-uniform.)
template <int A_LOADS, int B_LOADS, int NWAVES, int BM, int BN>
__device__ __forceinline__ void issue_slice(const bf16_t* const* ap, const bf16_t* const* bp, int kt,
                                            unsigned char* stage, int wave) {
#pragma unroll
  for (int i = 0; i < A_LOADS; ++i)
    __builtin_amdgcn_global_load_lds(ap[i] + kt * 64, (lds_void*)(uintptr_t)(stage + (i * NWAVES + wave) * 1024), 16, 0, CS_GEMM_A_AUX);
#pragma unroll
  for (int i = 0; i < B_LOADS; ++i)
    if (BN % (8 * NWAVES) == 0 || (i * NWAVES + wave) * 8 < BN)
    __builtin_amdgcn_global_load_lds(bp[i] + kt * 64, (lds_void*)(uintptr_t)(stage + BM * 128 + (i * NWAVES + wave) * 1024), 16, 0, CS_GEMM_W_AUX);
}

// One of the A_LOADS + B_LOADS loads of a slice, by index.
template <int A_LOADS, int B_LOADS, int NWAVES, int BM, int BN>
__device__ __forceinline__ void issue_one(const bf16_t* const* ap, const bf16_t* const* bp, int l, int kt,
                                          unsigned char* stage, int wave) {
  if (l < A_LOADS)
    __builtin_amdgcn_global_load_lds(ap[l] + kt * 64, (lds_void*)(uintptr_t)(stage + (l * NWAVES + wave) * 1024), 16, 0, CS_GEMM_A_AUX);
  else if (BN % (8 * NWAVES) == 0 || ((l - A_LOADS) * NWAVES + wave) * 8 < BN)
    __builtin_amdgcn_global_load_lds(bp[l - A_LOADS] + kt * 64,
                                     (lds_void*)(uintptr_t)(stage + BM * 128 + ((l - A_LOADS) * NWAVES + wave) * 1024), 16, 0, CS_GEMM_W_AUX);
}

// One 64-wide K slice of a wave's MFMAs.  PREFETCH: the loads of slice kn go out one at a time
// between the MFMAs of the first k-steps: issued in one burst behind the barrier they queue in the
// texture-address unit (16 clocks each, all waves at once) and every wave sits in the issue stall
// instead of feeding the MFMA pipe.  W_FIRST: accumulate C^T blocks (lane = row m, registers =
// columns n); otherwise C blocks (lane = column n, registers = rows m).
template <int BM, int BN, int WGM, int WGN, bool W_FIRST, bool PREFETCH>
__device__ __forceinline__ void k_slice(const bf16_t* const* ap, const bf16_t* const* bp, int kn,
                                        const unsigned char* cur, unsigned char* nxt, int a_rd, int b_rd, int sw,
                                        int lhi, int wave, f32x16 (&acc)[BM / WGM / 32][(BN / WGN + 31) / 32]) {
  constexpr int TM = BM / WGM / 32, TN = (BN / WGN + 31) / 32;
  constexpr int NWAVES = WGM * WGN;
  constexpr bool MFMA16 = use_mfma16<NWAVES, BM, BN>();
  constexpr int A_LOADS = BM / (8 * NWAVES), B_LOADS = (BN + 8 * NWAVES - 1) / (8 * NWAVES);
  constexpr int RD_PER = 2;     // LDS reads of the next k-step issued behind each of the first MFMAs
  constexpr int SPREAD_KS = 2;  // k-steps over which the next slice's loads are spread (2 measured best of 1..4)
  if constexpr (MFMA16) {
    // Two k-steps of 32 with v_mfma_f32_16x16x32_bf16; a_rd / b_rd address row lane % 16 of the wave's first
    // 16-row fragment and sw = (lane % 16) / 2; lhi = lane / 16 is the lane's 16-byte piece of a k-step's 64
    // bytes.  Fragment i of A pairs with fragment j of W into quarter 2 (i % 2) + j % 2 of block (i / 2, j / 2).
    // The operand with fewer fragments per wave is held, double-buffered over the two k-steps (the second
    // k-step's come in behind the first MFMAs); the other is streamed through a ring of four registers
    // sets, each fragment requested three rows of MFMAs before its turn, so 48 registers hold the operands
    // whatever the wave tile (a full double buffer of a 128 x 64 tile would take 96).
    constexpr int TM16 = 2 * TM, TN16 = BN / WGN / 16;   // a wave's columns may end in the middle of its last 32-block
    constexpr bool STREAM_A = TM16 >= TN16;
    constexpr int NO = STREAM_A ? TM16 : TN16;      // streamed fragments per k-step
    constexpr int NI = STREAM_A ? TN16 : TM16;      // held fragments per k-step
    const int s_rd = STREAM_A ? a_rd : b_rd, h_rd = STREAM_A ? b_rd : a_rd;
    const int coff0 = (lhi ^ sw) << 4, coff1 = ((4 + lhi) ^ sw) << 4;
    bf16x8 hf[2][NI], sf[4];
    auto read_streamed = [&](int r) {   // row r of the 2 * NO rows of this slice
      return *reinterpret_cast<const bf16x8*>(cur + s_rd + (r % NO) * 16 * 128 + (r < NO ? coff0 : coff1));
    };
#pragma unroll
    for (int j = 0; j < NI; ++j) hf[0][j] = *reinterpret_cast<const bf16x8*>(cur + h_rd + j * 16 * 128 + coff0);
#pragma unroll
    for (int r = 0; r < 3; ++r) sf[r] = read_streamed(r);
#pragma unroll
    for (int r = 0; r < 2 * NO; ++r) {
      const int ks = r / NO, o = r % NO;
#pragma unroll
      for (int in = 0; in < NI; ++in) {
        const int n = o * NI + in;
        const int i = STREAM_A ? o : in, j = STREAM_A ? in : o;
        const int quarter = 2 * (i & 1) + (j & 1);
        const bf16x8 fa = STREAM_A ? sf[r & 3] : hf[ks][in], fw = STREAM_A ? hf[ks][in] : sf[r & 3];
        f32x4 c;
#pragma unroll
        for (int e = 0; e < 4; ++e) c[e] = acc[i >> 1][j >> 1][4 * quarter + e];
        if (W_FIRST) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fw, fa, c, 0, 0, 0);
        else c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fa, fw, c, 0, 0, 0);
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i >> 1][j >> 1][4 * quarter + e] = c[e];
        if (PREFETCH && ks == 0) {
          constexpr int LT = A_LOADS + B_LOADS, SLOTS = NO * NI;
#pragma unroll
          for (int l = 0; l < LT; ++l)
            if (l * SLOTS / LT == n) issue_one<A_LOADS, B_LOADS, NWAVES, BM, BN>(ap, bp, l, kn, nxt, wave);
        }
        if (in == 0 && r + 3 < 2 * NO) sf[(r + 3) & 3] = read_streamed(r + 3);
        if (ks == 0 && n < NI) hf[1][n] = *reinterpret_cast<const bf16x8*>(cur + h_rd + n * 16 * 128 + coff1);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    return;
  }
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
      if (PREFETCH && ks < SPREAD_KS) {
        constexpr int LT = A_LOADS + B_LOADS, SLOTS = SPREAD_KS * TM * TN;
#pragma unroll
        for (int l = 0; l < LT; ++l)
          if (l * SLOTS / LT == ks * TM * TN + n) issue_one<A_LOADS, B_LOADS, NWAVES, BM, BN>(ap, bp, l, kn, nxt, wave);
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

// The K loop.  On return the stage buffer that does not hold the last slice is idle: every wave
// passed the last barrier after reading it and nothing was loaded into it since.
// before_last() runs between the last barrier and the last slice's MFMAs: global loads it issues
// are in flight while those execute.
template <int BM, int BN, int WGM, int WGN, bool W_FIRST, int STAGES, typename F>
__device__ __forceinline__ void main_loop(const GemmArgs& g, unsigned char* smem, int m0, int n0,
                                          f32x16 (&acc)[BM / WGM / 32][(BN / WGN + 31) / 32], F&& before_last) {
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = (WN + 31) / 32;
  constexpr int STAGE_BYTES = (BM + BN) * 128;
  constexpr int NWAVES = WGM * WGN;
  constexpr bool MFMA16 = use_mfma16<NWAVES, BM, BN>();
  constexpr int A_LOADS = BM / (8 * NWAVES), B_LOADS = (BN + 8 * NWAVES - 1) / (8 * NWAVES);
  static_assert(BM % (8 * NWAVES) == 0 && BN % 8 == 0, "tile vs waves");
  static_assert(WM % 32 == 0 && WN % (MFMA16 ? 16 : 32) == 0, "wave tile vs MFMA shape");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int M = g.M, N = g.N, K = g.K;
  // the lane's row inside an operand fragment (32 rows, or 16 for the 16x16x32 shape) and its 16-byte
  // piece of a k-step; sw = the row's share of the LDS chunk swizzle
  const int lrow = MFMA16 ? (lane & 15) : (lane & 31), lhi = MFMA16 ? (lane >> 4) : (lane >> 5);
  const int a_rd = (wm * WM + lrow) * 128;
  const int b_rd = BM * 128 + (wn * WN + lrow) * 128;
  const int sw = (lrow >> 1) & 7;

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
    bp[i] = g.W + (int64_t)r * g.ldw + (((lane & 7) ^ ((rt >> 1) & 7)) << 3);
  }
  const int KT = K >> 6;
  if constexpr (STAGES > 2) {
    // Slices kt + 1 .. kt + STAGES - 2 stay in flight while slice kt is consumed.  A wave's loads complete in the
    // order it issued them, so waiting until at most n * L of them are outstanding (L = its loads per slice) means
    // everything older than the newest n slices has landed.
    const int L = A_LOADS + (BN % (8 * NWAVES) == 0 || ((B_LOADS - 1) * NWAVES + wave) * 8 < BN ? B_LOADS : B_LOADS - 1);
    static_assert(STAGES <= 4, "the waits below cover up to two slices in flight");
    auto wait_newer = [&](int n) {   // n newer slices may still be in flight
      if (n <= 0) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      else if (L == A_LOADS + B_LOADS) {
        if (n == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(A_LOADS + B_LOADS) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (A_LOADS + B_LOADS)) : "memory");
      } else {
        if (n == 1) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(A_LOADS + B_LOADS - 1) : "memory");
        else asm volatile("s_waitcnt vmcnt(%0)" ::"n"(2 * (A_LOADS + B_LOADS - 1)) : "memory");
      }
    };
    static_assert(2 * (A_LOADS + B_LOADS) < 64, "vmcnt is a 6-bit counter");
#pragma unroll
    for (int st = 0; st < STAGES - 1; ++st)
      if (st < KT) issue_slice<A_LOADS, B_LOADS, NWAVES, BM, BN>(ap, bp, st, smem + st * STAGE_BYTES, wave);
    int cur_s = 0;                     // stage of slice kt
    for (int kt = 0; kt < KT - 1; ++kt) {
      const int ahead = KT - 1 - kt < STAGES - 2 ? KT - 1 - kt : STAGES - 2;   // newer slices already requested
      wait_newer(ahead);               // this wave's part of slice kt has landed
      // ... and everyone's; slice kt-1 fully consumed, so its stage is free.  A bare barrier: __syncthreads()
      // carries a fence that waits for every outstanding load, the newer slices' included.
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      asm volatile("" ::: "memory");
      const unsigned char* cur = smem + cur_s * STAGE_BYTES;
      const int nxt_s = cur_s == 0 ? STAGES - 1 : cur_s - 1;   // the stage slice kt-1 was in = that of slice kt + STAGES - 1
      if (kt + STAGES - 1 < KT)
        k_slice<BM, BN, WGM, WGN, W_FIRST, true>(ap, bp, kt + STAGES - 1, cur, smem + nxt_s * STAGE_BYTES, a_rd, b_rd, sw, lhi, wave, acc);
      else
        k_slice<BM, BN, WGM, WGN, W_FIRST, false>(ap, bp, 0, cur, nullptr, a_rd, b_rd, sw, lhi, wave, acc);
      cur_s = cur_s + 1 == STAGES ? 0 : cur_s + 1;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    before_last();
    k_slice<BM, BN, WGM, WGN, W_FIRST, false>(ap, bp, 0, smem + ((KT - 1) % STAGES) * STAGE_BYTES, nullptr, a_rd, b_rd, sw, lhi,
                                              wave, acc);
    return;
  }
  issue_slice<A_LOADS, B_LOADS, NWAVES, BM, BN>(ap, bp, 0, smem, wave);
  for (int kt = 0; kt < KT - 1; ++kt) {
    const unsigned char* cur = smem + (kt & 1) * STAGE_BYTES;
    unsigned char* nxt = smem + ((kt + 1) & 1) * STAGE_BYTES;
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // this wave's part of slice kt has landed
    __syncthreads();                                    // ... and everyone's; slice kt-1 fully consumed
    k_slice<BM, BN, WGM, WGN, W_FIRST, true>(ap, bp, kt + 1, cur, nxt, a_rd, b_rd, sw, lhi, wave, acc);
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  before_last();
  k_slice<BM, BN, WGM, WGN, W_FIRST, false>(ap, bp, 0, smem + ((KT - 1) & 1) * STAGE_BYTES, nullptr, a_rd, b_rd, sw, lhi,
                                            wave, acc);
}

template <int V>
struct int_tag { static constexpr int value = V; };

// A 64-row tile for the rows behind the last full tile row exists when every wave can own whole
// 32-column blocks of it (and the epilogue has no pairing of column blocks).
template <int BN, int WGM, int WGN, int EPI>
constexpr bool light_tail() {
  constexpr int WN = BN / (WGM * WGN);                           // columns per wave of the 64-row tile
  constexpr int UNIT = use_mfma16<WGM * WGN>() ? 16 : 32;          // (a 16x16x32 wave may own half a 32-column block)
  return EPI != EPI_SWIGLU_BF16 && WN % UNIT == 0 && WN >= UNIT && (EPI != EPI_QKV || WN % 32 == 0);
}

// One output tile: K loop and epilogue.
// LDS_ALLOC: bytes of LDS the launch has (that of its largest tile shape).
template <int BM, int BN, int WGM, int WGN, int EPI, int LDS_ALLOC = tile_lds_bytes<BM, BN, WGM * WGN, EPI>(), int STAGES_ARG = 0>
__device__ __forceinline__ void tile_body(const GemmArgs& g, unsigned char* smem, const int m0, const int n0) {
  constexpr int WM = BM / WGM, WN = BN / WGN;
  constexpr int TM = WM / 32, TN = (WN + 31) / 32;
  constexpr int STAGE_BYTES = (BM + BN) * 128;
  constexpr int NWAVES = WGM * WGN;
  constexpr bool MFMA16 = use_mfma16<NWAVES, BM, BN>();
  static_assert((EPI != EPI_SWIGLU_BF16 && EPI != EPI_QKV) || WN % 32 == 0, "these epilogues work on whole 32-column blocks");
  static_assert(EPI != EPI_SWIGLU_BF16 || (TN % 2 == 0), "gate/up pairs need an even number of column tiles");
  static_assert(EPI != EPI_QKV || (TM % 2 == 0), "v tiles leave through LDS two row blocks at a time");
  // the epilogue chunks live in the idle stage buffer; where that is too small for them (a 64-row tail tile of a
  // narrow launch) they go behind everything else this tile uses, inside what the launch's main tile shape allocated
  constexpr bool CHUNKS_BEHIND = NWAVES * CHUNK_BYTES > STAGE_BYTES;
  constexpr int XTRA = extra_lds_bytes<BM, BN, NWAVES, EPI>();
  constexpr int STAGES = STAGES_ARG ? STAGES_ARG : stages<BM, BN, NWAVES, EPI>();
  // (QKV: behind the K loop the rotary table and the chunks above it take the space of the first two stage buffers)
  static_assert(!CHUNKS_BEHIND || (STAGES * STAGE_BYTES + XTRA + NWAVES * CHUNK_BYTES <= LDS_ALLOC && EPI != EPI_QKV),
                "no room for the epilogue chunks");

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;
  const int M = g.M, N = g.N;
  // The extra LDS behind the stage buffers.  Consumer of a folded normalisation: BM row scales, BM row shifts
  // (LayerNorm: mean times scale) and BN column values of norm_shift.  Producer: the gain of the tile's columns
  // and, from float 256 on, the waves' sums of squares [WGN][BM] and plain sums [WGN][BM].
  float* extra_lds = reinterpret_cast<float*>(smem + STAGES * STAGE_BYTES);
  // consumer: thread t < BM gathers the partial sums of squares of row m0 + t while the last K slice runs
  // (thread BM + t the partial plain sums, for a LayerNorm), they are turned into 1 / rms (or 1 / sigma and
  // mean / sigma) behind the K loop and left in LDS for every wave
  constexpr bool CONSUMES_NORM = EPI == EPI_QKV || EPI == EPI_SWIGLU_BF16 || EPI == EPI_GELU_BF16;
  constexpr bool CONSUMES_LAYERNORM = EPI == EPI_QKV || EPI == EPI_GELU_BF16;
  static_assert(!CONSUMES_NORM || 64 * NWAVES >= BM, "one thread per tile row gathers its scale");
  static_assert(!CONSUMES_LAYERNORM || 64 * NWAVES >= 2 * BM || NWAVES <= 4, "a second thread per tile row gathers its sum");
  static_assert(!CONSUMES_NORM || (2 * BM + BN) * 4 <= XTRA, "extra LDS layout of a consumer");
  constexpr bool TWO_GATHERERS = 64 * NWAVES >= 2 * BM;
  [[maybe_unused]] float ss_part[8];
  [[maybe_unused]] float s1_part[(CONSUMES_LAYERNORM && !TWO_GATHERERS) ? 8 : 1];
  [[maybe_unused]] const bool layer_norm = CONSUMES_LAYERNORM && g.s1_in != nullptr;
  [[maybe_unused]] auto gather_scale = [&] {
    if (!g.ss_in) return;
    const int t = (int)threadIdx.x;
    if (t < BM) {
      int m = m0 + t;
      m = m < M ? m : M - 1;
#pragma unroll
      for (int k = 0; k < 8; ++k) ss_part[k] = k < g.ss_parts ? g.ss_in[(int64_t)k * g.ss_stride + m] : 0.f;
      if constexpr (CONSUMES_LAYERNORM && !TWO_GATHERERS) {
        if (layer_norm) {
#pragma unroll
          for (int k = 0; k < 8; ++k) s1_part[k] = k < g.ss_parts ? g.s1_in[(int64_t)k * g.ss_stride + m] : 0.f;
        }
      }
    } else if constexpr (CONSUMES_LAYERNORM && TWO_GATHERERS) {
      if (layer_norm && t < 2 * BM) {
        int m = m0 + t - BM;
        m = m < M ? m : M - 1;
#pragma unroll
        for (int k = 0; k < 8; ++k) ss_part[k] = k < g.ss_parts ? g.s1_in[(int64_t)k * g.ss_stride + m] : 0.f;
      }
    }
  };
  [[maybe_unused]] auto publish_scale = [&] {
    if (!g.ss_in) return;
    const int t = (int)threadIdx.x;
    const float tot = ((ss_part[0] + ss_part[1]) + (ss_part[2] + ss_part[3])) + ((ss_part[4] + ss_part[5]) + (ss_part[6] + ss_part[7]));
    if constexpr (CONSUMES_LAYERNORM) {
      if (layer_norm) {
        // the shift vector of the tile's columns, and the rows' statistics
        for (int c = t * 4; c < BN; c += 64 * NWAVES * 4) {
          int n = n0 + c;
          n = n < N ? n : N - 4;
          *reinterpret_cast<f32x4*>(extra_lds + 2 * BM + c) = *reinterpret_cast<const f32x4*>(g.norm_shift + n);
        }
        float sum1;
        if constexpr (TWO_GATHERERS) {
          if (t >= BM && t < 2 * BM) extra_lds[t] = tot;   // thread BM + r: the plain sum of row r
          __syncthreads();
          sum1 = t < BM ? extra_lds[BM + t] : 0.f;
        } else {
          sum1 = ((s1_part[0] + s1_part[1]) + (s1_part[2] + s1_part[3])) + ((s1_part[4] + s1_part[5]) + (s1_part[6] + s1_part[7]));
        }
        if (t < BM) {
          const float inv_d = 1.0f / (float)g.norm_dim;
          const float mean = sum1 * inv_d;
          const float var = fmaxf(tot * inv_d - mean * mean, 0.f);
          const float rs = rsqrtf(var + g.norm_eps);
          extra_lds[t] = rs;
          extra_lds[BM + t] = mean * rs;
        }
        __syncthreads();
        return;
      }
    }
    if (t < BM) extra_lds[t] = rsqrtf(tot / (float)g.norm_dim + g.norm_eps);
    __syncthreads();
  };

  f32x16 acc[TM][TN];
  // this wave's epilogue chunk, in the stage buffer the last K slice did not use
  unsigned char* chunk = CHUNKS_BEHIND ? smem + STAGES * STAGE_BYTES + XTRA + wave * CHUNK_BYTES
                                       : smem + ((g.K >> 6) % STAGES) * STAGE_BYTES + wave * CHUNK_BYTES;

  if constexpr (EPI == EPI_QKV) {
    if (n0 >= 2 * g.hidden) {
      // v columns (the whole workgroup: 2*hidden is a multiple of BN).  Untransposed blocks: a lane's
      // group holds one v dimension n (the block "row" here) and four consecutive tokens; written as
      // rows of the transposed v buffer, 64 tokens of one dimension per chunk row.  With the roles of
      // the operands swapped the two halves of a 16x16x32 group index swap too (vsub).
      float bv[TN][4];
      main_loop<BM, BN, WGM, WGN, false, STAGES>(g, smem, m0, n0, acc, [&] {
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int n = n0 + wn * WN + j * 32 + blk_row<MFMA16>(q, lane);
            bv[j][q] = (g.bias && n < N) ? g.bias[n] : 0.f;
          }
        gather_scale();
      });
      publish_scale();
      const bool wide = (g.ld_vt & 7) == 0;
      const bool wt_v = lines_exclusive(g.vt, g.ld_vt * 2);   // a workgroup writes 512-byte runs of a v^T row
#pragma unroll
      for (int j = 0; j < TN; ++j) {
#pragma unroll
        for (int i = 0; i < TM; i += 2) {
          f32x4 v[2][4];
#pragma unroll
          for (int ii = 0; ii < 2; ++ii)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
              const int vsub = MFMA16 ? (((q & 1) << 1) | (q >> 1)) : q;
              // the group's four values are four consecutive tokens: their row scales
              f32x4 rs = {1.f, 1.f, 1.f, 1.f}, sh = {0.f, 0.f, 0.f, 0.f};
              float cn = 0.f;   // LayerNorm: the shift of this v dimension
              if (g.ss_in) rs = *reinterpret_cast<const f32x4*>(extra_lds + wm * WM + (i + ii) * 32 + blk_col<MFMA16>(q, lane));
              if (layer_norm) {
                sh = *reinterpret_cast<const f32x4*>(extra_lds + BM + wm * WM + (i + ii) * 32 + blk_col<MFMA16>(q, lane));
                cn = extra_lds[2 * BM + wn * WN + j * 32 + blk_row<MFMA16>(q, lane)];
              }
#pragma unroll
              for (int e = 0; e < 4; ++e) v[ii][q][e] = acc[i + ii][j][4 * vsub + e] * rs[e] - sh[e] * cn + bv[j][q];
            }
          store_block<2, bf16_t, false, MFMA16>(chunk, v, g.vt, g.ld_vt, nullptr, n0 + wn * WN + j * 32 - 2 * g.hidden,
                                        N - 2 * g.hidden, m0 + wm * WM + i * 32, M, wide, wt_v);
        }
      }
      return;
    }
  }

  // Residual add: the old values are needed in the epilogue, where a load's latency would be
  // paid once per chunk (the stores in between keep the compiler from hoisting the loads).  With
  // four waves per workgroup (one per SIMD, or small tiles) the registers for the whole wave tile
  // are free, so every lane fetches the 16-byte pieces it will update before the last K slice.
  // With eight waves there is room for one row block before the last K slice; the second row block is
  // requested right behind the K loop, into the registers the operands leave, and from then on the pieces of
  // row block i + 2 are requested as soon as those of row block i are stored (into the same registers), so two
  // row blocks of x are in flight all through the epilogue (the narrow tiles: out projection 559 -> 575, down
  // projection 838 -> 870 TFLOP/s on 8192 tokens; the 256 x 256 tile, whose four row blocks per wave leave no
  // registers for it, stays with one: with two it spills more and gains nothing).
  constexpr bool RESADD = EPI == EPI_RESADD_F32 || EPI == EPI_RESADD_SCALED_F32 || EPI == EPI_RESADD_SUMS_F32;
  constexpr bool TWO_PER_SIMD = NWAVES > 4 || (BM == 128 && BN == 160);   // 256 registers per wave, not 512
  constexpr bool HOLD = RESADD && !TWO_PER_SIMD;
  constexpr bool HOLD_ROW = RESADD && TWO_PER_SIMD;
  constexpr bool HOLD_TWO = HOLD_ROW && TM > 1 && BN < 256;
  [[maybe_unused]] f32x4 held[HOLD ? TM : HOLD_TWO ? 2 : 1][(HOLD || HOLD_ROW) ? TN : 1][4];
  [[maybe_unused]] auto fetch_old = [&](int i, int j, f32x4 (&dst)[4]) {
    const int r = lane >> 3, c = (lane & 7) * 4;
    int n = n0 + wn * WN + j * 32 + c;
    n = n < N ? n : N - 4;
#pragma unroll
    for (int it = 0; it < 4; ++it) {
      int m = m0 + wm * WM + i * 32 + it * 8 + r;
      m = m < M ? m : M - 1;
      int64_t row = m;
      if (g.row_map) {
        row = g.row_map[m];
        row = row < 0 ? 0 : row;
      }
      dst[it] = *reinterpret_cast<const f32x4*>(static_cast<const float*>(g.out) + row * g.ldo + n);
    }
  };
  // The bias of the lane's columns is fetched there too (a load inside the epilogue waits out its
  // latency once per chunk).
  // (with the 16x16x32 shape groups q and q + 2 hold the same columns: two distinct column groups per block)
  constexpr int CQ = MFMA16 ? 2 : 4;
  f32x4 bias_r[TN][CQ];
  [[maybe_unused]] f32x4 scale_r[EPI == EPI_RESADD_SCALED_F32 ? TN : 1][CQ];
  main_loop<BM, BN, WGM, WGN, true, STAGES>(g, smem, m0, n0, acc, [&] {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < CQ; ++q) {
        const int n = n0 + wn * WN + j * 32 + blk_col<MFMA16>(q, lane);
        bias_r[j][q] = f32x4{0.f, 0.f, 0.f, 0.f};
        if (g.bias && n < N) bias_r[j][q] = *reinterpret_cast<const f32x4*>(g.bias + n);
        if constexpr (EPI == EPI_RESADD_SCALED_F32) {
          scale_r[j][q] = f32x4{0.f, 0.f, 0.f, 0.f};
          if (n < N) scale_r[j][q] = *reinterpret_cast<const f32x4*>(g.col_scale + n);
        }
      }
    if constexpr (HOLD) {
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) fetch_old(i, j, held[i][j]);
    } else if constexpr (HOLD_ROW) {
#pragma unroll
      for (int j = 0; j < TN; ++j) fetch_old(0, j, held[0][j]);
    }
    if constexpr (CONSUMES_NORM) gather_scale();
  });
  if constexpr (CONSUMES_NORM) publish_scale();
  if constexpr (HOLD_TWO) {
    if (m0 + wm * WM + 32 < M) {   // wave-uniform
#pragma unroll
      for (int j = 0; j < TN; ++j) fetch_old(1, j, held[1][j]);
    }
  }
  // producer of a folded RMSNorm: the gain of the tile's columns goes to LDS, from where the epilogue's
  // row-segment lanes read it
  constexpr bool FOLDS_NORM = RESADD;
  constexpr bool FOLDS_SUMS = (EPI == EPI_RESADD_SCALED_F32 || EPI == EPI_RESADD_SUMS_F32) && 1024 + 2 * WGN * BM * 4 <= XTRA;
  static_assert(!FOLDS_NORM || (BN <= 256 && 1024 + WGN * BM * 4 <= XTRA), "extra LDS layout");
  [[maybe_unused]] const bool folding = FOLDS_NORM && g.ss_out != nullptr;
  [[maybe_unused]] const bool folding_sums = FOLDS_SUMS && folding && g.s1_out != nullptr;
  if constexpr (FOLDS_NORM) {
    if (folding) {
      for (int c = threadIdx.x * 4; c < BN; c += 64 * NWAVES * 4) {
        int n = n0 + c;
        n = n < N ? n : N - 4;
        *reinterpret_cast<f32x4*>(extra_lds + c) = *reinterpret_cast<const f32x4*>(g.norm_gain + n);
      }
      __syncthreads();
    }
  }

  // QKV: the (cos, sin) rows of this tile's BM tokens are staged in LDS (free after the K loop)
  // with coalesced 16-byte loads; read per lane from global they are 16-byte pieces of 32 different
  // rows per instruction, which cost 18 us of a 110 us launch.  The table sits at the bottom of
  // LDS and the epilogue chunks move to the top.
  [[maybe_unused]] int rope_stride = 0;
  if constexpr (EPI == EPI_QKV) {
    if (g.rope_cs) {
      const int half = g.head_dim >> 1;
      const int cpr = half >> 1;                       // 16-byte pieces per token row (two pairs each)
      const int upr = (cpr + 1) | 1;                   // ... per padded LDS row: odd, so rows spread over the banks
      rope_stride = upr * 16;
      chunk = smem + 2 * STAGE_BYTES - (NWAVES - wave) * CHUNK_BYTES;
      __syncthreads();                                 // every wave is done reading the last K slice
      // LDS-direct loads, all in flight at once: piece u of the padded table comes from row u / upr
      // (the padding pieces repeat the row's last one; the tail of the last instruction runs up to
      // 1 KB past the table, below the chunks)
      for (int base = wave * 64; base < BM * upr; base += 64 * NWAVES) {
        const int u = base + lane;
        int r = u / upr, c = u - r * upr;
        c = c < cpr ? c : cpr - 1;
        r = m0 + r < M ? m0 + r : M - 1;
        __builtin_amdgcn_global_load_lds(g.rope_cs + ((int64_t)r * cpr + c) * 4, (lds_void*)(uintptr_t)(smem + base * 16), 16, 0, 0);
      }
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
    }
  }

  // ---- epilogue.  Register 4q+e of lane l in block (i,j) is the element
  //      (row m = i*32 + blk_row(q, l), column n = j*32 + blk_col(q, l) + e).
  const int nw = n0 + wn * WN;               // first column of this wave
  const int n_end = nw + WN < N ? nw + WN : N;   // one past its last (the wave's last 32-block may be half used)
  const bool wide = (g.ldo & 7) == 0;
  // write-through stores only where no 128-byte line of the output is shared with another workgroup:
  // aligned rows, and a tile's column extent in bytes a multiple of 128
  constexpr int OUT_ES = (EPI == EPI_F32 || EPI == EPI_GELU_F32 || RESADD) ? 4 : 2;
  constexpr int TILE_OUT_BYTES = (EPI == EPI_SWIGLU_BF16 ? BN / 2 : BN) * OUT_ES;
  const bool wt = TILE_OUT_BYTES % 128 == 0 && lines_exclusive(g.out, g.ldo * OUT_ES);
  // QKV: byte offset of the first (cos, sin) pair of every 4-column group, once per lane (the
  // divisions by run-time sizes must not be redone for every row block)
  [[maybe_unused]] int rope_off[TN][CQ];
  if constexpr (EPI == EPI_QKV) {
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int q = 0; q < CQ; ++q) {
        const int n = nw + j * 32 + blk_col<MFMA16>(q, lane);
        rope_off[j][q] = ((((n < g.hidden ? n : n - g.hidden)) % g.head_dim) >> 1) * 8;
      }
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    const int mrow = m0 + wm * WM + i * 32;  // first row of the block
    if (mrow >= M) continue;                 // wave-uniform
    // folded RMSNorm, consumer side: 1 / rms of the row each group q of this block holds
    [[maybe_unused]] float rsq[4] = {1.f, 1.f, 1.f, 1.f};
    [[maybe_unused]] float msq[CONSUMES_LAYERNORM ? 4 : 1] = {};   // LayerNorm: mean / sigma of those rows
    if constexpr (CONSUMES_NORM) {
      if (g.ss_in) {
#pragma unroll
        for (int q = 0; q < 4; ++q) rsq[q] = extra_lds[mrow - m0 + blk_row<MFMA16>(q, lane)];
      }
    }
    if constexpr (CONSUMES_LAYERNORM) {
      if (layer_norm) {
#pragma unroll
        for (int q = 0; q < 4; ++q) msq[q] = extra_lds[BM + mrow - m0 + blk_row<MFMA16>(q, lane)];
      }
    }
    // ... producer side: sums of squares of the updated rows, gathered by the residual store
    [[maybe_unused]] NormFold fold = {g.xg, g.ld_xg, extra_lds, n0, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
    if constexpr (EPI == EPI_SWIGLU_BF16) {
      // output column p*32 + c of the wave pairs gate column 2p*32 + c with up column (2p+1)*32 + c
      auto emit = [&](auto tag, int p0) {
        constexpr int NB = decltype(tag)::value;
        f32x4 v[NB][4];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int j = 2 * (p0 + b);
            const f32x4 bg = bias_r[j][q % CQ], bu = bias_r[j + 1][q % CQ];
#pragma unroll
            for (int e = 0; e < 4; ++e)
              v[b][q][e] = silu_f(acc[i][j][4 * q + e] * rsq[q] + bg[e]) * (acc[i][j + 1][4 * q + e] * rsq[q] + bu[e]);
          }
        store_block<NB, bf16_t, false, MFMA16>(chunk, v, static_cast<bf16_t*>(g.out), g.ldo, g.row_map, mrow, M,
                                       (nw >> 1) + p0 * 32, N >> 1, wide, wt);
      };
      constexpr int NP = TN / 2;
#pragma unroll
      for (int p0 = 0; p0 + 1 < NP; p0 += 2) emit(int_tag<2>{}, p0);
      if constexpr (NP & 1) emit(int_tag<1>{}, NP - 1);
    } else {
      constexpr bool OUT_F32 = EPI == EPI_F32 || EPI == EPI_GELU_F32 || RESADD;
      auto emit = [&](auto tag, int j0) {
        constexpr int NB = decltype(tag)::value;
        f32x4 v[NB][4];
#pragma unroll
        for (int b = 0; b < NB; ++b)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int j = j0 + b;
            const int n = nw + j * 32 + blk_col<MFMA16>(q, lane);
            f32x4 t;
#pragma unroll
            for (int e = 0; e < 4; ++e) t[e] = acc[i][j][4 * q + e];
            if constexpr (CONSUMES_NORM && EPI != EPI_SWIGLU_BF16) t *= rsq[q];
            if constexpr (CONSUMES_LAYERNORM) {
              if (layer_norm) t -= msq[q] * *reinterpret_cast<const f32x4*>(extra_lds + 2 * BM + (n - n0));
            }
            t += bias_r[j][q % CQ];
            if constexpr (EPI == EPI_RESADD_SCALED_F32) t *= scale_r[j][q % CQ];
            if constexpr (EPI == EPI_GELU_BF16 || EPI == EPI_GELU_F32 || EPI == EPI_GELU_SPLIT) {
#pragma unroll
              for (int e = 0; e < 4; ++e) t[e] = gelu_erf(t[e]);
            }
            if constexpr (EPI == EPI_QKV) {
              // q and k columns: rotary on neighbouring columns (2p, 2p+1), both held by this lane
              if (g.rope_cs) {
                const f32x4 cs = *reinterpret_cast<const f32x4*>(smem + (mrow - m0 + blk_row<MFMA16>(q, lane)) * rope_stride + rope_off[j][q % CQ]);  // cos,sin,cos,sin
                const float r0 = t[0] * cs[0] - t[1] * cs[1], r1 = t[1] * cs[0] + t[0] * cs[1];
                const float r2 = t[2] * cs[2] - t[3] * cs[3], r3 = t[3] * cs[2] + t[2] * cs[3];
                t[0] = r0; t[1] = r1; t[2] = r2; t[3] = r3;
              }
              t *= n < g.hidden ? g.q_scale : 1.0f;
            }
            v[b][q] = t;
          }
        const int col0 = nw + j0 * 32;
        if constexpr (RESADD) {
          store_block<NB, float, true, MFMA16, FOLDS_SUMS>(chunk, v, static_cast<float*>(g.out), g.ldo, g.row_map, mrow, M, col0, n_end, true,
                                       wt && CS_GEMM_RESADD_WT && !g.plain_stores,
                                       HOLD ? held[i][j0] : HOLD_TWO ? held[i & 1][j0] : HOLD_ROW ? held[0][j0] : nullptr,
                                       folding ? &fold : nullptr);
          if constexpr (HOLD_TWO) {
            if (i + 2 < TM) fetch_old(i + 2, j0, held[i & 1][j0]);
          } else if constexpr (HOLD_ROW) {
            if (i + 1 < TM) fetch_old(i + 1, j0, held[0][j0]);
          }
        } else if constexpr (OUT_F32) {
          store_block<NB, float, false, MFMA16>(chunk, v, static_cast<float*>(g.out), g.ldo, g.row_map, mrow, M, col0, n_end, true, wt);
        } else if constexpr (EPI == EPI_QKV) {
          store_block<NB, bf16_t, false, MFMA16>(chunk, v, static_cast<bf16_t*>(g.out), g.ldo, g.row_map, mrow, M, col0,
                                         2 * g.hidden, wide, wt);
        } else {
          store_block<NB, bf16_t, false, MFMA16>(chunk, v, static_cast<bf16_t*>(g.out), g.ldo, g.row_map, mrow, M, col0, n_end, wide, wt);
          if constexpr (EPI == EPI_GELU_SPLIT) {
            // second half of the row: what the bf16 rounding of the first half dropped
#pragma unroll
            for (int b = 0; b < NB; ++b)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const bf16x4 h = __builtin_convertvector(v[b][q], bf16x4);
                v[b][q] -= __builtin_convertvector(h, f32x4);
              }
            store_block<NB, bf16_t, false, MFMA16>(chunk, v, static_cast<bf16_t*>(g.out) + N, g.ldo, g.row_map, mrow, M, col0, n_end,
                                           wide && (N & 7) == 0, wt && (N & 63) == 0);
          }
        }
      };
      constexpr int PER = OUT_F32 ? 1 : 2;   // 32-column blocks per 128-byte chunk row
      if constexpr (PER == 2) {
#pragma unroll
        for (int j0 = 0; j0 + 1 < TN; j0 += 2) emit(int_tag<2>{}, j0);
        if constexpr (TN & 1) emit(int_tag<1>{}, TN - 1);
      } else {
#pragma unroll
        for (int j0 = 0; j0 < TN; ++j0) emit(int_tag<1>{}, j0);
      }
      if constexpr (FOLDS_NORM) {
        if (folding) {
          // eight lanes share a row of a 32-column fp32 block: their sums over the wave's columns, added
          // in a fixed order, are the tile's contribution to the row's sum of squares
#pragma unroll
          for (int it = 0; it < 4; ++it) {
            float s = fold.ssacc[it];
            s += __shfl_xor(s, 1);
            s += __shfl_xor(s, 2);
            s += __shfl_xor(s, 4);
            if ((lane & 7) == 0) extra_lds[256 + wn * BM + wm * WM + i * 32 + it * 8 + (lane >> 3)] = s;
          }
          if constexpr (FOLDS_SUMS) {
            if (folding_sums) {
#pragma unroll
              for (int it = 0; it < 4; ++it) {
                float s = fold.s1acc[it];
                s += __shfl_xor(s, 1);
                s += __shfl_xor(s, 2);
                s += __shfl_xor(s, 4);
                if ((lane & 7) == 0) extra_lds[256 + (WGN + wn) * BM + wm * WM + i * 32 + it * 8 + (lane >> 3)] = s;
              }
            }
          }
        }
      }
    }
  }
  if constexpr (FOLDS_NORM) {
    if (folding) {
      // the waves' sums over their columns, added in wave order: the tile's share of each row's sum of squares
      __syncthreads();
      const int t = threadIdx.x;
      if (t < BM && m0 + t < M) {
        float s = extra_lds[256 + t];
#pragma unroll
        for (int w2 = 1; w2 < WGN; ++w2) s += extra_lds[256 + w2 * BM + t];
        g.ss_out[(int64_t)(n0 / BN) * g.ss_stride + m0 + t] = s;
        if constexpr (FOLDS_SUMS) {
          if (folding_sums) {
            float s1 = extra_lds[256 + WGN * BM + t];
#pragma unroll
            for (int w2 = 1; w2 < WGN; ++w2) s1 += extra_lds[256 + (WGN + w2) * BM + t];
            g.s1_out[(int64_t)(n0 / BN) * g.ss_stride + m0 + t] = s1;
          }
        }
      }
    }
  }
}

// What a launch does with the tiles that would leave the chip mostly idle:
//  TAIL_LIGHT (M not a multiple of BM): the workgroups behind those of the full tile rows take the
//    remaining rows in 64-row tiles (same threads, every wave a 64 x BN/waves strip): they stream the
//    same W slices but do a quarter of the MFMAs, so that tile row costs microseconds instead of a round
//    of the chip.
//  TAIL_SPLIT (no light tail, the last round of the chip at most half full): the tiles of that
//    last round are cut in two along M and run as BM/2-row tiles by twice as many workgroups, so the
//    round takes little more than half as long.  A round costs the same however few of its tiles are
//    there (measured: 864 tiles of 256 x 256 take as long as 1024), and 8192 x 6912 is 3 3/8 rounds.
enum { TAIL_NONE = 0, TAIL_LIGHT = 1, TAIL_SPLIT = 2 };
constexpr int CHIP_CUS = 256;

// tile id -> first row / column.  Ids walk the tile grid in bands of GROUP_M tile rows, row index
// fastest, so the ~32 tiles an XCD runs at a time form a GROUP_M x 8 block that shares GROUP_M slices
// of A and 8 slices of W per k-step (an L2 miss on every W byte otherwise: measured 427 clocks average
// L2 read latency and the L1 miss queue full 58 % of the time).
template <int BM, int BN>
__device__ __forceinline__ void tile_origin(int id, int tiles_m, int tiles_n, int& m0, int& n0) {
  constexpr int GROUP_M = 4;   // (2: the same within noise; 8: 1 % slower on the 32-image batch; 16: 4 % slower)
  const int band = id / (GROUP_M * tiles_n), in_band = id - band * (GROUP_M * tiles_n);
  const int band_rows = tiles_m - band * GROUP_M < GROUP_M ? tiles_m - band * GROUP_M : GROUP_M;
  m0 = (band * GROUP_M + in_band % band_rows) * BM;
  n0 = (in_band / band_rows) * BN;
}

// LDS of a launch: that of its main tile, or what the deeper pipeline of its 64-row tail tiles needs.
template <int BM, int BN, int NWAVES, int EPI, int TAIL>
constexpr int launch_lds_bytes() {
  const int main_tile = tile_lds_bytes<BM, BN, NWAVES, EPI>();
  if (TAIL != 1 /* TAIL_LIGHT */) return main_tile;
  const int light = light_lds_need<BN, NWAVES, EPI>(light_stages<BN, NWAVES, EPI>());
  return light > main_tile ? light : main_tile;
}

template <int BM, int BN, int WGM, int WGN, int EPI, int TAIL>
__global__ __launch_bounds__(64 * WGM * WGN)
// (the four-wave 128 x 160 tile must leave room for a second workgroup on the CU: 256 registers, not 512)
__attribute__((amdgpu_waves_per_eu(BM == 128 && BN == 160 ? 2 : 1))) void gemm_kernel(GemmArgs g) {
  extern __shared__ __align__(16) unsigned char smem[];
  if (gridDim.y > 1) {   // split K (plain fp32 partial sums only): this workgroup's part of A, W and of the output
    g.A += (int64_t)blockIdx.y * g.K;
    g.W += (int64_t)blockIdx.y * g.K;
    g.out = static_cast<float*>(g.out) + (int64_t)blockIdx.y * g.split_stride;
  }
  const int M = g.M, N = g.N;
  const int tiles_n = (N + BN - 1) / BN;
  int tiles_m = (M + BM - 1) / BM;
  int nb = gridDim.x;
  constexpr bool LIGHT = TAIL == TAIL_LIGHT;
  static_assert(!LIGHT || light_tail<BN, WGM, WGN, EPI>(), "no 64-row tile for this shape");
  static_assert(TAIL != TAIL_SPLIT || (BM / 2 / WGM) % 32 == 0, "half tiles need whole 32-row blocks per wave");
  if constexpr (TAIL == TAIL_SPLIT) {
    // workgroups [0, n_main) run the full rounds; the rest each take half of a tile of the last round
    const int n_main = (tiles_m * tiles_n / CHIP_CUS) * CHIP_CUS;
    if ((int)blockIdx.x >= n_main) {
      // (the half tiles get the same treatment as the tiles: consecutive workgroups run on different XCDs,
      // so every XCD takes a contiguous run of half tiles, both halves of a tile among them)
      int t = blockIdx.x - n_main;
      {
        const int n_half = gridDim.x - n_main, xcd = t & 7, idx = t >> 3;
        const int per = n_half >> 3, rem = n_half & 7;
        t = xcd * per + (xcd < rem ? xcd : rem) + idx;
      }
      int m0, n0;
      tile_origin<BM, BN>(n_main + (t >> 1), tiles_m, tiles_n, m0, n0);
      m0 += (t & 1) * (BM / 2);
      if (m0 >= M) return;   // the lower half of a tile of a ragged last tile row may be empty
      tile_body<BM / 2, BN, WGM, WGN, EPI, tile_lds_bytes<BM, BN, WGM * WGN, EPI>()>(g, smem, m0, n0);
      return;
    }
    nb = n_main;
  }
  if constexpr (LIGHT) {
    const int full_m = M / BM, n_main = full_m * tiles_n;
    if ((int)blockIdx.x >= n_main) {
      const int t = blockIdx.x - n_main;
      const int tail_m = (M - full_m * BM + 63) / 64;
      tile_body<64, BN, 1, WGM * WGN, EPI, launch_lds_bytes<BM, BN, WGM * WGN, EPI, TAIL>(), light_stages<BN, WGM * WGN, EPI>()>(
          g, smem, full_m * BM + (t % tail_m) * 64, (t / tail_m) * BN);
      return;
    }
    tiles_m = full_m;
    nb = n_main;
  }

  // workgroup -> tile.  Consecutive workgroups land on different XCDs (b % 8), each with its own
  // L2, so every XCD gets a contiguous range of tile ids.
  int bid = blockIdx.x;
  {
    const int xcd = bid & 7, idx = bid >> 3;
    const int per = nb >> 3, rem = nb & 7;
    bid = xcd * per + (xcd < rem ? xcd : rem) + idx;
  }
  int m0, n0;
  tile_origin<BM, BN>(bid, tiles_m, tiles_n, m0, n0);
  tile_body<BM, BN, WGM, WGN, EPI>(g, smem, m0, n0);
}

// Measurement switch: CS_GEMM_NO_TAIL_SPLIT=1 in the environment keeps whole tiles in the last round, so
// the effect of the half tiles can be measured from the committed tree (read once).
static bool tail_split_off() {
  static const bool off = [] {
    const char* v = getenv("CS_GEMM_NO_TAIL_SPLIT");
    return v && *v && *v != '0';
  }();
  return off;
}

template <int BM, int BN, int WGM, int WGN, int EPI, int TAIL>
static cs_status launch_one(const GemmArgs& g, hipStream_t stream) {
  constexpr int NT = 64 * WGM * WGN;
  constexpr int LDS = launch_lds_bytes<BM, BN, WGM * WGN, EPI, TAIL>();
  static_assert(LDS <= 160 * 1024, "LDS of a CU");
  auto kern = gemm_kernel<BM, BN, WGM, WGN, EPI, TAIL>;
  if (g.describe) {
    snprintf(g.describe, 96, "gemm_kernel<%d, %d, %d, %d, %d, %d>%s", BM, BN, WGM, WGN, EPI, TAIL,
             use_mfma16<WGM * WGN, BM, BN>() ? " 16x16x32" : " 32x32x16");
    return CS_OK;
  }
  // one attribute call per instantiation (two threads that both see `false` repeat a harmless call)
  static std::atomic<bool> attr_set{false};
  if (!attr_set.load(std::memory_order_acquire)) {
    CS_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, LDS));
    attr_set.store(true, std::memory_order_release);
  }
  const int tiles_n = (g.N + BN - 1) / BN;
  int tiles = ((g.M + BM - 1) / BM) * tiles_n;
  if (TAIL == TAIL_LIGHT)   // full tile rows, then the remaining rows in 64-row tiles
    tiles = (g.M / BM) * tiles_n + ((g.M % BM + 63) / 64) * tiles_n;
  if (TAIL == TAIL_SPLIT)   // the tiles of the last round twice, as half tiles
    tiles += tiles % CHIP_CUS;
  GemmArgs ga = g;
  // The residual epilogue's stores are write-through except in launches of the narrow tiles that run more than
  // one round: there the next round's operand loads queue behind the first round's burst of stores, and stores
  // that stay in the L2's write-back do better (16 384 tokens: out projection 487 -> 521, down projection
  // 757 -> 775 TFLOP/s; one round and the 256 x 256 tile: 1 - 4 % worse).  CS_GEMM_RESADD_PLAIN in the environment
  // (read once) overrides the rule for measurement: 0 never plain, 1 always.
  {
    static const int mode = [] { const char* v = getenv("CS_GEMM_RESADD_PLAIN"); return v && *v >= '0' && *v <= '1' ? *v - '0' : 2; }();
    ga.plain_stores = mode == 1 || (mode == 2 && BN < 256 && tiles > CHIP_CUS);
  }
  hipLaunchKernelGGL(kern, dim3(tiles, g.splits > 1 ? g.splits : 1), dim3(NT), LDS, stream, ga);
  CS_HIP(hipGetLastError());
  return CS_OK;
}

template <int BM, int BN, int WGM, int WGN, int EPI>
static cs_status launch_cfg(const GemmArgs& g, hipStream_t stream) {
  // the light-tail variant where the last, partly empty tile row is at least 1/64 of the tile rows
  if constexpr (light_tail<BN, WGM, WGN, EPI>()) {
    if (g.M % BM != 0 && (g.M + BM - 1) / BM <= 64) return launch_one<BM, BN, WGM, WGN, EPI, TAIL_LIGHT>(g, stream);
  }
  // half tiles for a last round that is at most half full (the big tile only: that is where a round is long)
  if constexpr (BM == 256 && BN == 256) {
    const int tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN), tail = tiles % CHIP_CUS;
    if (g.splits <= 1 && tiles > CHIP_CUS && tail > 0 && tail <= CHIP_CUS / 2 && !tail_split_off())
      return launch_one<BM, BN, WGM, WGN, EPI, TAIL_SPLIT>(g, stream);
  }
  return launch_one<BM, BN, WGM, WGN, EPI, TAIL_NONE>(g, stream);
}

// Measurement switch: CS_GEMM_NARROW8 in the environment (read once) says when the 256 x 160 tile runs with
// eight waves of 64 x 80 instead of four of 64 x 160 (and the 256 x 128 tile with eight of 64 x 64 instead of four
// of 64 x 128): 0 never, 1 for long K loops, 2 (default) always.  Measured on the 8-image step: 11.92 / 11.88 /
// 11.84 ms for 0 / 1 / 2.
static int narrow8_mode() {
  static const int mode = [] {
    const char* v = getenv("CS_GEMM_NARROW8");
    return v && *v >= '0' && *v <= '2' ? *v - '0' : 2;
  }();
  return mode;
}

// CS_GEMM_RESADD_PAIR in the environment (read once): 1 runs the residual GEMMs with N = 1280 on 128 x 160 tiles
// of four waves, two workgroups per CU (independent of each other: one's barriers and epilogue run under the
// other's MFMAs), instead of one eight-wave 256 x 160 tile per CU; 0 does not.
static int resadd_pair_mode() {
  static const int mode = [] {
    const char* v = getenv("CS_GEMM_RESADD_PAIR");
    return v && *v >= '0' && *v <= '1' ? *v - '0' : 0;
  }();
  return mode;
}

// The fewest 256 x 256 tiles beyond one round of the chip for which a launch takes that tile: 257.  With the half
// tiles of a split last round such a launch never runs below 2/3 full (257 tiles: a round and a half round),
// which beats what the 128 x 128 tiles lose inside the CU (3072 tokens: gate|up 731 -> 872 TFLOP/s, the step 7.30
// -> 6.98 ms; 6144 tokens: 10.74 -> 10.33 ms).  CS_GEMM_BIG_MIN in the environment (read once) sets another
// threshold for measurement; 384, a round and a half, was the rule before the half tiles existed.
static int64_t big_tile_min() {
  static const int64_t v = [] {
    const char* e = getenv("CS_GEMM_BIG_MIN");
    const long x = e ? atol(e) : 0;
    return (int64_t)(x > 256 && x <= 4096 ? x : 257);
  }();
  return v;
}

static int small_resadd_pair() {
  static const int mode = [] {
    const char* v = getenv("CS_GEMM_SMALL_PAIR");
    return v && *v >= '0' && *v <= '2' ? *v - '0' : 2;
  }();
  return mode;
}

static bool narrow_resadd() {
  static const bool on = [] {
    const char* v = getenv("CS_GEMM_NARROW_RESADD");
    return v && *v && *v != '0';
  }();
  return on;
}

template <int EPI>
static cs_status launch_epi(const GemmArgs& g, hipStream_t stream) {
  // Tile choice by the number of workgroups it yields for the 256 CUs.
  const int64_t tm = (g.M + 255) / 256;
  const int64_t big = tm * ((g.N + 255) / 256);
  const bool big_ok = EPI != EPI_QKV || (2 * g.hidden) % 256 == 0;
  // (the scaled residual epilogue spills registers with eight waves and with 160-wide wave tiles: it
  // takes the 256 x 128 or 128 x 128 tiles)
  constexpr bool EIGHT_WAVES_OK = EPI != EPI_RESADD_SCALED_F32;
#ifdef CS_GEMM_FORCE_256      // measurement build: the 256 x 256 tile whatever the number of workgroups
  if constexpr (EIGHT_WAVES_OK) {
    if (big_ok) return launch_cfg<256, 256, 2, 4, EPI>(g, stream);
  }
#endif
  if constexpr (EIGHT_WAVES_OK) {
    // 256 x 256 for more than a round of the chip (CS_GEMM_NARROW_RESADD=1 in the environment makes the
    // residual add take the narrow tile below at any size, for measurement: the 32-image batch 166.5 -> 177.4 ms)
    const bool narrow_first = EPI == EPI_RESADD_F32 && g.N % 160 == 0 && narrow_resadd();
    // (the residual GEMMs keep a round and a half: below it their narrow tiles make whole rounds, e.g. two at 16 384 tokens)
    constexpr bool RES = EPI == EPI_RESADD_F32 || EPI == EPI_RESADD_SUMS_F32;
    if (big >= (RES ? 384 : big_tile_min()) && big_ok && !narrow_first) return launch_cfg<256, 256, 2, 4, EPI>(g, stream);
  }
  if constexpr (EPI != EPI_QKV && EPI != EPI_SWIGLU_BF16) {
    // narrow outputs (N = hidden = 1280): 256 x 160 tiles, four waves of 64 x 160, give M/256 * 8
    // workgroups, one round of the chip at M = 8192
    if constexpr (EIGHT_WAVES_OK) {
      if (g.N % 160 == 0 && tm * (g.N / 160) >= 192) {
#if CS_GEMM_MFMA16
        if constexpr (EPI == EPI_RESADD_F32) {
          if (resadd_pair_mode() == 1 && !g.s1_out) return launch_cfg<128, 160, 2, 2, EPI>(g, stream);
        }
        // eight waves of 64 x 80 (16x16x32 MFMAs, the wave's third 32-column block half used) where the K
        // loop is long: their main loop is 8 % faster, but with two waves per SIMD the residual epilogue can
        // prefetch only one row block of x at a time, which costs more than that at K = 1280 (measured:
        // K = 3456 74 -> 71 us, K = 1280 36.4 -> 37.5 us)
        if (narrow8_mode() == 2 || (narrow8_mode() == 1 && g.K >= 2560)) return launch_cfg<256, 160, 4, 2, EPI>(g, stream);
#endif
        return launch_cfg<256, 160, 4, 1, EPI>(g, stream);
      }
    }
    // the same for N = 1024: 256 x 128 tiles (eight waves of 64 x 64 leave room for the scaled residual epilogue too)
    // (not for N = 1280, which it would cut into ten column tiles, too many for the next normalisation to fold:
    // 5120 tokens, 9.73 -> 9.35 ms per step on the 128 x 160 tiles below)
    if (g.N % 128 == 0 && g.N % 160 != 0 && tm * (g.N / 128) >= 192) {
#if CS_GEMM_MFMA16
      if (narrow8_mode() == 2 || (narrow8_mode() == 1 && g.K >= 2560)) return launch_cfg<256, 128, 4, 2, EPI>(g, stream);
#endif
      return launch_cfg<256, 128, 4, 1, EPI>(g, stream);
    }
  }
  if constexpr (EIGHT_WAVES_OK) {
    // 256 x 256 also when it fills one round to 5/8 or more (batches of 2 - 4 images: 2 - 7 % faster than
    // 128 x 128 tiles; at 120 workgroups it loses)
    if (big >= 160 && big <= 256 && big_ok) return launch_cfg<256, 256, 2, 4, EPI>(g, stream);
  }
#if CS_GEMM_MFMA16
  // a residual GEMM with N = 1280 too small for the tiles above: 128 x 160 tiles rather than 128 x 128, which makes
  // eight column tiles instead of ten, so the next normalisation still folds into it (vision tower, 4096 tokens:
  // 8.32 -> 7.77 ms per step; audio tower, 3000 tokens: 8.08 -> 7.94 ms).  Up to one tile per CU they run with eight waves of 32 x 80, so that every SIMD has two waves to
  // alternate between (3072 tokens: 6.91 -> 6.73 ms, 4096: 7.58 -> 7.44); beyond that with four waves of 64 x 80,
  // two workgroups per CU.  CS_GEMM_SMALL_PAIR in the environment, for measurement: 0 keeps the 128 x 128 tiles,
  // 1 takes four waves at any size.
  if constexpr (EPI == EPI_RESADD_F32 || EPI == EPI_RESADD_SUMS_F32) {
    if (g.N % 160 == 0 && g.splits <= 1 && small_resadd_pair() > 0) {
      const int64_t tiles = ((g.M + 127) / 128) * (g.N / 160);
      if (small_resadd_pair() == 2 && tiles <= CHIP_CUS) return launch_cfg<128, 160, 4, 2, EPI>(g, stream);
      return launch_cfg<128, 160, 2, 2, EPI>(g, stream);
    }
  }
#endif
  return launch_cfg<128, 128, 2, 2, EPI>(g, stream);
}

int32_t gemm_norm_fold_parts(int64_t M, int64_t N, int64_t K, bool scaled, bool sums) {
  // ask the launcher itself which tile such a residual GEMM runs on: one partial sum per column tile
  if (M <= 0 || M > 0x7fffffff || N <= 0 || K <= 0 || (N & 3) || (K & 63)) return 0;
  char name[96] = {0};
  GemmArgs g = {};
  g.M = (int32_t)M; g.N = (int32_t)N; g.K = (int32_t)K; g.lda = K; g.ldo = N; g.describe = name;
  g.col_scale = scaled ? reinterpret_cast<const float*>(uintptr_t(16)) : nullptr;   // only its alignment is looked at
  g.s1_out = sums ? reinterpret_cast<float*>(uintptr_t(16)) : nullptr;              // a LayerNorm tower: sums as well
  int bm = 0, bn = 0;
  if (launch_gemm(scaled ? EPI_RESADD_SCALED_F32 : EPI_RESADD_F32, g, nullptr) != CS_OK ||
      sscanf(name, "gemm_kernel<%d, %d", &bm, &bn) != 2 || bn <= 0) return 0;
  const int64_t parts = (N + bn - 1) / bn;
  return parts <= 8 ? (int32_t)parts : 0;
}

cs_status launch_gemm(int epilogue, const GemmArgs& g_in, hipStream_t stream) {
  GemmArgs g = g_in;
  if (g.M <= 0 || g.N <= 0) return CS_OK;
  if (g.ldw == 0) g.ldw = (int64_t)g.K * (g.splits > 1 ? g.splits : 1);
  if (g.ldw < g.K || (g.ldw & 7)) return fail(CS_ERR_INVALID_ARG, "gemm: ldw must be at least K and a multiple of 8");
  if (g.splits > 1 && (epilogue != EPI_F32 || g.bias || g.row_map || g.splits > 16 ||
                       g.split_stride < (int64_t)g.M * g.ldo || (g.split_stride & 3)))
    return fail(CS_ERR_UNSUPPORTED, "gemm: split K writes plain fp32 partial sums (no bias, no row map), at most 16 parts");
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
    case EPI_RESADD_F32:
    case EPI_RESADD_SUMS_F32:
      return g.s1_out ? launch_epi<EPI_RESADD_SUMS_F32>(g, stream) : launch_epi<EPI_RESADD_F32>(g, stream);
    case EPI_RESADD_SCALED_F32:
      if (!g.col_scale || (reinterpret_cast<uintptr_t>(g.col_scale) & 15))
        return fail(CS_ERR_INVALID_ARG, "gemm: the scaled residual epilogue needs a 16-byte aligned col_scale");
      return launch_epi<EPI_RESADD_SCALED_F32>(g, stream);
    case EPI_SWIGLU_BF16:
      if (g.N & 63) return fail(CS_ERR_UNSUPPORTED, "gemm: swiglu needs N % 64 == 0");
      return launch_epi<EPI_SWIGLU_BF16>(g, stream);
    case EPI_QKV:
      if ((g.M & 3) || (g.hidden & 63) || (g.head_dim & 3) || g.N != 3 * g.hidden || (g.ld_vt & 3) ||
          (reinterpret_cast<uintptr_t>(g.vt) & 7))
        return fail(CS_ERR_UNSUPPORTED, "gemm: qkv epilogue needs M % 4 == 0, hidden % 64 == 0, head_dim % 4 == 0, N == 3 hidden");
      // the (cos, sin) table of a tile's tokens and the epilogue chunks share LDS behind the K loop
      if (g.rope_cs && g.head_dim > 80) return fail(CS_ERR_UNSUPPORTED, "gemm: rotary epilogue needs head_dim <= 80");
      return launch_epi<EPI_QKV>(g, stream);
    default: return fail(CS_ERR_INVALID_ARG, "gemm: unknown epilogue");
  }
}

}  // namespace cs
