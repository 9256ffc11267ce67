// Variable-length attention for gfx950, one kernel for window layers and full layers.
//
// A work item names a block of queries [q0,q1) and the keys [kv0,kv1) they attend to (both in
// token indices of the packed batch); a window layer has one item per window, a full layer
// cuts every sequence into query blocks.  Inside a workgroup every wave owns 64 queries and
// all waves walk the same 64-key tiles, which are staged in LDS once per workgroup.
//
// Scores are computed transposed, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16: a lane then holds
// one query column (lane % 32) and 16 of the 32 key rows of a tile, so the online-softmax state
// (running max, running sum, rescale factor) is per lane, and the exponentiated scores are
// already laid out as the B operand of the second product O^T = V^T P^T.  V is consumed
// transposed (token-contiguous), which is how the QKV projection stores it.  q arrives
// pre-multiplied by softmax_scale * log2(e); probabilities are exp2 of score differences.
#include "common.h"

namespace cs {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

typedef float f32x2_a __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_a __attribute__((ext_vector_type(2)));
// two floats -> packed bf16 pair (v_cvt_pk_bf16_f32, round to nearest even)
__device__ __forceinline__ uint32_t pack2_a(float a, float b) {
  const f32x2_a v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_a));
}

// Window layers launch thousands of two-wave workgroups, each a short chain load -> stage ->
// MFMA -> store: latency is hidden only by residency, so the single-tile variant is held to 168 registers
// (three waves per SIMD, six workgroups per CU, which is also what their LDS tiles allow).
// SINGLE: every work item has at most 64 keys (windows of up to 64 tokens): one tile, nothing to
// prefetch, so the staging registers are dead before the accumulators come alive.
template <int DH, int NW, int QT, bool SINGLE>
__global__ __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(SINGLE ? 3 : (NW == 8 ? 4 : 2), SINGLE ? 3 : (NW == 8 ? 4 : 2))))
void attn_kernel(AttnArgs a) {
  constexpr int NT = 64 * NW;
  constexpr int KS = DH / 16;            // k-steps of the score product
  constexpr int DT = (DH + 31) / 32;     // 32-row tiles of O^T
  constexpr int KSTR = DH * 2 + 16;      // LDS row stride of the K tile, bytes
  constexpr int VSTR = 64 * 2 + 8;       // LDS row stride of the V^T tile, bytes
  constexpr int KCH = DH / 8;            // 16-byte chunks per K row
  // Head dimension 80, eight waves: the query fragments wait in LDS (each lane's own 16-byte pieces, read
  // back in lane order: no conflicts) instead of 20 registers, which brings the kernel under 128 registers
  // and a second workgroup onto the CU.
  constexpr bool Q_IN_LDS = DH > 64 && NW == 8;
  __shared__ __align__(16) unsigned char k_lds[64 * KSTR];
  __shared__ __align__(16) unsigned char v_lds[DT * 32 * VSTR];
  __shared__ __align__(16) unsigned char q_lds[Q_IN_LDS ? QT * KS * NT * 16 : 16];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int l31 = lane & 31, lhi = lane >> 5;
  // Workgroup -> (work item, head).  Consecutive workgroups run on different XCDs (id % 8), each with its own L2.
  int head, item;
  {
    const int xcd = blockIdx.x & 7, r = blockIdx.x >> 3;
    if constexpr (SINGLE) {
      // window layers: an XCD takes every eighth window with all its heads one after the other, so the heads of a
      // window, which share the 128-byte lines of its token rows (a head is 128 or 160 bytes of a row), meet in one L2
      item = (r / a.n_heads) * 8 + xcd;
      head = r % a.n_heads;
      if (item >= a.n_work) return;   // (whole workgroup, before any barrier)
    } else {
      // full layers: the (head, item) pairs in head-major order, cut into eight equal runs: the query blocks of one
      // (item, head), which all read that head's K and V^T, run on one XCD at about the same time instead of on
      // all eight (the 32-image batch fetched 10.5 GB per full-attention layer for 0.85 GB of operands)
      const int pairs = a.n_work * a.n_heads, per = pairs >> 3, rem = pairs & 7;
      if (r >= per + (xcd < rem ? 1 : 0)) return;
      const int p = xcd * per + (xcd < rem ? xcd : rem) + r;
      head = p / a.n_work;
      item = p - head * a.n_work;
    }
  }
  const AttnWork w = a.work[item];
  const int hidden = a.n_heads * DH;
  const int64_t ldq = 2 * (int64_t)hidden;
  const bf16_t* qbase = a.qk + head * DH;
  const bf16_t* kbase = a.qk + hidden + head * DH;
  const bf16_t* vbase = a.vt + (int64_t)head * DH * a.ld_vt;
  const int last_tok = a.n_tok - 1;
  const int vt_last = ((a.n_tok + 3) & ~3) - 4;   // last 4-token chunk of a V^T row that was written

  // ---- this wave's queries as B operands: lane = query column, 8 consecutive dims per k-step
  const int qw = w.q0 + wave * (32 * QT);
  bf16x8 qf[QT][KS];
#pragma unroll
  for (int it = 0; it < QT; ++it) {
    int row = qw + it * 32 + l31;
    row = row < last_tok ? row : last_tok;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
      qf[it][ks] = *reinterpret_cast<const bf16x8*>(qbase + (int64_t)row * ldq + ks * 16 + lhi * 8);
  }
  if constexpr (Q_IN_LDS) {
#pragma unroll
    for (int it = 0; it < QT; ++it)
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) *reinterpret_cast<bf16x8*>(q_lds + ((it * KS + ks) * NT + tid) * 16) = qf[it][ks];
  }

  f32x16 o[QT][DT];
#pragma unroll
  for (int it = 0; it < QT; ++it)
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int r = 0; r < 16; ++r) o[it][dt][r] = 0.f;
  float mrun[QT], lrun[QT];
#pragma unroll
  for (int it = 0; it < QT; ++it) {
    mrun[it] = -INFINITY;
    lrun[it] = 0.f;
  }

  // ---- K / V^T tile staging: global -> registers (all loads of a tile in flight together, issued
  // before the MFMAs of the previous tile) -> LDS.
  constexpr int K_PT = (64 * KCH + NT - 1) / NT;   // 16-byte chunks of the K tile per thread
  constexpr int V_PT = (DH * 16 + NT - 1) / NT;    // 8-byte chunks of the V^T tile per thread
  typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
  typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
  u32x4 kreg[K_PT];
  u32x2 vreg[V_PT];
  auto load_tile = [&](int kv) {
#pragma unroll
    for (int u = 0; u < K_PT; ++u) {
      int c = tid + u * NT;
      c = c < 64 * KCH ? c : 64 * KCH - 1;
      const int r = c / KCH, ch = c % KCH;
      int row = kv + r;
      row = row < last_tok ? row : last_tok;
      kreg[u] = *reinterpret_cast<const u32x4*>(kbase + (int64_t)row * ldq + ch * 8);
    }
#pragma unroll
    for (int u = 0; u < V_PT; ++u) {
      int c = tid + u * NT;
      c = c < DH * 16 ? c : DH * 16 - 1;
      const int d = c >> 4, ch = c & 15;
      int tok = kv + ch * 4;
      tok = tok < vt_last ? tok : vt_last;
      vreg[u] = *reinterpret_cast<const u32x2*>(vbase + (int64_t)d * a.ld_vt + tok);
    }
  };
  auto store_tile = [&]() {
#pragma unroll
    for (int u = 0; u < K_PT; ++u) {
      const int c = tid + u * NT;
      if (c < 64 * KCH) *reinterpret_cast<u32x4*>(k_lds + (c / KCH) * KSTR + (c % KCH) * 16) = kreg[u];
    }
#pragma unroll
    for (int u = 0; u < V_PT; ++u) {
      const int c = tid + u * NT;
      if (c < DH * 16) *reinterpret_cast<u32x2*>(v_lds + (c >> 4) * VSTR + (c & 15) * 8) = vreg[u];
    }
  };

  // a wave whose queries lie beyond the item (the last query block of a sequence) only helps to stage the tiles
  const bool live = qw < w.q1;
  load_tile(w.kv0);
  for (int kv = w.kv0; kv < (SINGLE ? w.kv0 + 1 : w.kv1); kv += 64) {
    if (!SINGLE) __syncthreads();  // previous tile fully consumed
    store_tile();
    __syncthreads();
    if (!SINGLE && kv + 64 < w.kv1) load_tile(kv + 64);
    __builtin_amdgcn_sched_barrier(0);
    if (!SINGLE && !live) continue;

    // ---- S^T tiles: s[it][jt] covers keys kv + jt*32 .. +31 (rows) x queries it*32 .. +31 (lanes)
    // The accumulators start at minus the query's running maximum (a lane's scores all belong to one
    // query), so the products come out as score - maximum and the common case below needs no subtraction.
    const bool first = kv == w.kv0;
    f32x16 s[QT][2];
#pragma unroll
    for (int it = 0; it < QT; ++it) {
      const float init = first ? 0.f : -mrun[it];
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) s[it][jt][r] = init;
    }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
      for (int jt = 0; jt < 2; ++jt) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(k_lds + (jt * 32 + l31) * KSTR + ks * 32 + lhi * 16);
#pragma unroll
        for (int it = 0; it < QT; ++it) {
          bf16x8 q = qf[it][ks];
          if constexpr (Q_IN_LDS) q = *reinterpret_cast<const bf16x8*>(q_lds + ((it * KS + ks) * NT + tid) * 16);
          s[it][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, q, s[it][jt], 0, 0, 0);
        }
      }
    }
    // register r of a tile holds key row 8*(r/4) + 4*lhi + r%4
    if (kv + 64 > w.kv1) {
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kv + jt * 32 + 8 * (r >> 2) + 4 * lhi + (r & 3);
          if (key >= w.kv1) {
#pragma unroll
            for (int it = 0; it < QT; ++it) s[it][jt][r] = -INFINITY;
          }
        }
    }
    // ---- online softmax, per query column.  The running maximum is moved only when a tile's largest score
    // exceeds it by more than MAX_SLACK (in the log2 domain): probabilities are then at most 2^MAX_SLACK
    // instead of 1, which changes nothing in the quotient (softmax is invariant under a common shift, and
    // bf16 and fp32 keep their relative precision over that range), and the accumulators are rescaled
    // only on the first tile and on such a jump instead of on nearly every tile.
    constexpr float MAX_SLACK = 8.0f;
    bf16x8 pf[QT][4];
#pragma unroll
    for (int it = 0; it < QT; ++it) {
      float mx = s[it][0][0];
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[it][jt][r]);
      mx = fmaxf(mx, __shfl_xor(mx, 32));          // the tile's largest score minus the running maximum
      // v_exp_f32 directly: arguments are bounded above and results that would be denormal may flush to 0,
      // so the library exp2f's range scaling (four more instructions per score) buys nothing here
      const bool jump = first || mx > MAX_SLACK;   // every tile holds at least one valid key: mx is finite
      if (__any(jump)) {                           // some query of this wave takes a new maximum
        const float base = first ? 0.f : mrun[it];
        const float mnew = jump ? mx + base : mrun[it];
        const float alpha = first ? 0.f : __builtin_amdgcn_exp2f(mrun[it] - mnew);
        const float shift = mnew - base;           // 0 in the lanes whose query keeps its maximum
        mrun[it] = mnew;
        lrun[it] *= alpha;
#pragma unroll
        for (int jt = 0; jt < 2; ++jt)
#pragma unroll
          for (int r = 0; r < 16; ++r) s[it][jt][r] -= shift;
#pragma unroll
        for (int dt = 0; dt < DT; ++dt)
#pragma unroll
          for (int r = 0; r < 16; ++r) o[it][dt][r] *= alpha;
      }
      float sum = 0.f;
#pragma unroll
      for (int jt = 0; jt < 2; ++jt)
#pragma unroll
        for (int u = 0; u < 2; ++u) {
          uint32_t pk[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const float p0 = __builtin_amdgcn_exp2f(s[it][jt][8 * u + 2 * e]);
            const float p1 = __builtin_amdgcn_exp2f(s[it][jt][8 * u + 2 * e + 1]);
            sum += p0 + p1;
            pk[e] = pack2_a(p0, p1);
          }
          uint4 t = make_uint4(pk[0], pk[1], pk[2], pk[3]);
          pf[it][jt * 2 + u] = *reinterpret_cast<bf16x8*>(&t);
        }
      lrun[it] += sum;
    }
    // ---- O^T += V^T P^T.  k-slot e of lane-half lhi in step (jt,u) is key jt*32 + 16u + 8*(e/4) + 4*lhi + e%4
#pragma unroll
    for (int ku = 0; ku < 4; ++ku) {
#pragma unroll
      for (int dt = 0; dt < DT; ++dt) {
        const unsigned char* vp = v_lds + (dt * 32 + l31) * VSTR + (ku * 16 + 4 * lhi) * 2;
        uint4 t;
        const uint2 lo = *reinterpret_cast<const uint2*>(vp);
        const uint2 hi = *reinterpret_cast<const uint2*>(vp + 16);
        t.x = lo.x; t.y = lo.y; t.z = hi.x; t.w = hi.y;
        const bf16x8 vf = *reinterpret_cast<bf16x8*>(&t);
#pragma unroll
        for (int it = 0; it < QT; ++it)
          o[it][dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[it][ku], o[it][dt], 0, 0, 0);
      }
    }
  }

  // ---- normalise and store: register r of o[it][dt] is dim dt*32 + 8*(r/4) + 4*lhi + r%4 of query it*32 + lane%32
#pragma unroll
  for (int it = 0; it < QT; ++it) {
    const float l = lrun[it] + __shfl_xor(lrun[it], 32);
    const float inv = 1.0f / l;
    const int q = qw + it * 32 + l31;
    if (q >= w.q1) continue;
    bf16_t* orow = a.out + (int64_t)q * hidden + head * DH;
#pragma unroll
    for (int dt = 0; dt < DT; ++dt)
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const int d = dt * 32 + 8 * g + 4 * lhi;
        if (d < DH) {
          uint2 pk;
          pk.x = pack2_a(o[it][dt][4 * g + 0] * inv, o[it][dt][4 * g + 1] * inv);
          pk.y = pack2_a(o[it][dt][4 * g + 2] * inv, o[it][dt][4 * g + 3] * inv);
          *reinterpret_cast<uint2*>(orow + d) = pk;
        }
      }
  }
}

cs_status launch_attention(const AttnArgs& a, hipStream_t stream) {
  if (a.n_work <= 0) return CS_OK;
  if (a.n_tok < 4 || a.ld_vt < ((a.n_tok + 3) & ~3)) return fail(CS_ERR_INVALID_ARG, "attention: ld_vt too small");
  if (a.ld_vt & 3) return fail(CS_ERR_INVALID_ARG, "attention: ld_vt must be a multiple of 4");
  const int64_t pairs = (int64_t)a.n_work * a.n_heads;
  if (pairs + 8 * (int64_t)a.n_heads > 0x7fffffff) return fail(CS_ERR_UNSUPPORTED, "attention: too many work items");
  // (see the kernel: window layers give an XCD every eighth window, full layers an eighth of the (head, item) pairs)
  dim3 grid(a.single_tile ? (unsigned)(8 * ((a.n_work + 7) / 8) * a.n_heads) : (unsigned)(8 * ((pairs + 7) / 8)));
  // every wave owns 32 queries: two waves per 64-query work item (window layers), eight per 256-query item,
  // two waves per SIMD so that one wave's softmax arithmetic runs under the other's MFMAs
  if (a.single_tile && a.q_per_block != 64) return fail(CS_ERR_INVALID_ARG, "attention: single-tile items are 64-query items");
  if (a.head_dim == 80 && a.q_per_block == 64 && a.single_tile) hipLaunchKernelGGL((attn_kernel<80, 2, 1, true>), grid, dim3(128), 0, stream, a);
  else if (a.head_dim == 80 && a.q_per_block == 64) hipLaunchKernelGGL((attn_kernel<80, 2, 1, false>), grid, dim3(128), 0, stream, a);
  else if (a.head_dim == 80 && a.q_per_block == 256) hipLaunchKernelGGL((attn_kernel<80, 8, 1, false>), grid, dim3(512), 0, stream, a);
  else if (a.head_dim == 64 && a.q_per_block == 64 && a.single_tile) hipLaunchKernelGGL((attn_kernel<64, 2, 1, true>), grid, dim3(128), 0, stream, a);
  else if (a.head_dim == 64 && a.q_per_block == 64) hipLaunchKernelGGL((attn_kernel<64, 2, 1, false>), grid, dim3(128), 0, stream, a);
  else if (a.head_dim == 64 && a.q_per_block == 256) hipLaunchKernelGGL((attn_kernel<64, 8, 1, false>), grid, dim3(512), 0, stream, a);
  else return fail(CS_ERR_UNSUPPORTED, "attention: head_dim must be 64 or 80 and q_per_block 64 or 256");
  CS_HIP(hipGetLastError());
  return CS_OK;
}

}  // namespace cs
