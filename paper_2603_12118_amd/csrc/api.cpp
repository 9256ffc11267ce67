// C ABI of the library: error text, encoder creation (weight conversion and repacking on the
// host), batch query, the encoder task itself (a fixed sequence of kernel launches on the
// caller's stream) and the embedding hand-off.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <limits>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "common.h"
#include "plan.h"

namespace cs {

static thread_local std::string g_last_error;
void set_error(const std::string& msg) { g_last_error = msg; }
cs_status fail(cs_status s, const std::string& msg) {
  g_last_error = msg;
  return s;
}

static inline bf16_t host_f2bf(float f) {
  uint32_t u;
  memcpy(&u, &f, 4);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
static inline float host_bf2f(bf16_t b) {
  uint32_t u = (uint32_t)b << 16;
  float f;
  memcpy(&f, &u, 4);
  return f;
}

// A weight as the caller passed it, readable element by element as float.
struct SrcTensor {
  const void* data = nullptr;
  int64_t numel = 0;
  int dtype = CS_F32;
  float at(int64_t i) const {
    return dtype == CS_BF16 ? host_bf2f(static_cast<const bf16_t*>(data)[i]) : static_cast<const float*>(data)[i];
  }
  bf16_t bits(int64_t i) const {
    return dtype == CS_BF16 ? static_cast<const bf16_t*>(data)[i] : host_f2bf(static_cast<const float*>(data)[i]);
  }
};

// Host image of the device weight arena.
struct Arena {
  std::vector<unsigned char> host;
  size_t alloc(size_t bytes) {
    const size_t off = (size_t)round_up((int64_t)host.size(), 256);
    host.resize(off + bytes, 0);
    return off;
  }
  bf16_t* bf(size_t off) { return reinterpret_cast<bf16_t*>(host.data() + off); }
  float* f32(size_t off) { return reinterpret_cast<float*>(host.data() + off); }
};

struct LayerW {
  size_t wqkv, bqkv, wo, bo, w1, b1, w2, b2;  // w1: gate|up interleaved (vit) or fc1 (audio); w2: down / fc2
  size_t g1, be1, g2, be2;                    // norm gains and (LayerNorm towers) norm biases
  size_t ls1 = 0, ls2 = 0;                    // class-token tower: per-channel scales of the two branches
  // LayerNorm towers, for a LayerNorm folded into the GEMM behind it: shift vector c and bias d of that GEMM
  // (fold_vectors below); 0 where there are none
  size_t cqkv = 0, dqkv = 0, c1 = 0, d1 = 0;
};

}  // namespace cs

using namespace cs;

struct cs_encoder {
  cs_encoder_config cfg;
  int device = 0;
  // derived sizes
  int P_pad = 0, I_pad = 0, MH_pad = 0, half = 0;
  bool rope = false;
  // weights
  unsigned char* dev = nullptr;
  size_t dev_bytes = 0;
  std::vector<LayerW> layers;
  size_t w_pe = 0, g_m = 0, w_m1 = 0, b_m1 = 0, w_m2 = 0, b_m2 = 0;          // vit
  size_t w_c1 = 0, b_c1 = 0, w_c2 = 0, b_c2 = 0, g_p = 0, be_p = 0, w_p = 0, b_p = 0, pe_tab = 0;  // audio
  size_t inv_freq = 0, axis = 0;
  int pe_positions = 0;
  size_t b_pe = 0, be_m = 0, pos_tab = 0;    // class-token tower: patch-embed bias, projector norm bias, position table
  int n_positions = 0;                       // rows of its position table (1 + patches per tile); row n_positions = class token + row 0
  // plans of the batch shapes seen last (key: n_items, cu_seqlens, grid_thw), newest use = largest stamp
  struct CachedPlan {
    std::vector<int32_t> key;
    cs::BatchPlan plan;
    uint64_t stamp = 0;
  };
  mutable std::mutex plan_mu;
  mutable std::vector<CachedPlan> plans;
  mutable uint64_t plan_clock = 0;
  mutable uint64_t plan_hits = 0, plan_misses = 0;
  // pinned staging for the per-batch index tables, two slots used in turn
  void* stage[2] = {nullptr, nullptr};
  size_t stage_cap[2] = {0, 0};
  hipEvent_t stage_ev[2] = {nullptr, nullptr};
  bool stage_used[2] = {false, false};
  int stage_next = 0;
  bool capturing = false;            // a cs_encode_graph is being recorded: no timing events
  // optional per-step event timing
  int time_step = 0;
  int time_every = 1;                // of the launches of time_step, every time_every-th is timed
  int64_t time_seen = 0;
  std::vector<hipEvent_t> ev_pool;   // pairs: start, stop
  size_t ev_used = 0;

  template <class T>
  T* ptr(size_t off) const { return reinterpret_cast<T*>(dev + off); }
};

// ---- scratch of cs_encode_static: one array per GPU, in the code object's zero-initialised data, held
// until the process ends.  Host code never uses the array's name as an address (on the host it is
// only a handle for the lookup below); it uses the per-device address hipGetSymbolAddress returns.
static __device__ __align__(256) unsigned char scratch[CS_STATIC_SCRATCH_BYTES];

namespace cs {

constexpr int MAX_DEVICES = 64;
static std::mutex g_scratch_mu;
static void* g_scratch_ptr[MAX_DEVICES] = {};

// Address of the current device's copy of `scratch`, looked up once per device.
static cs_status static_scratch(void** out) {
  int dev = -1;
  CS_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= MAX_DEVICES) return fail(CS_ERR_UNSUPPORTED, "static scratch: device ordinal out of range");
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    CS_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(CS_ERR_HIP, "static scratch: hipGetSymbolAddress returned NULL");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return CS_OK;
}

static cs_status check_config(const cs_encoder_config& c) {
  if (c.struct_size != sizeof(cs_encoder_config)) return fail(CS_ERR_INVALID_ARG, "config.struct_size mismatch");
  if (c.input_order != CS_ORDER_RASTER && c.input_order != CS_ORDER_MERGE_MAJOR)
    return fail(CS_ERR_INVALID_ARG, "config.input_order");
  if (c.arch != CS_ARCH_VIT && c.arch != CS_ARCH_AUDIO && c.arch != CS_ARCH_VIT_CLS) return fail(CS_ERR_INVALID_ARG, "config.arch");
  if (c.input_order != CS_ORDER_RASTER && c.arch != CS_ARCH_VIT)
    return fail(CS_ERR_UNSUPPORTED, "config: input_order applies to vision encoders");
  if (c.attn_chunk < 0 || (c.attn_chunk & 3)) return fail(CS_ERR_INVALID_ARG, "config.attn_chunk must be a non-negative multiple of 4");
  if (c.attn_chunk != 0 && c.arch != CS_ARCH_AUDIO)
    return fail(CS_ERR_UNSUPPORTED, "config: attn_chunk applies to audio encoders");
  if ((c.dtype != CS_F32 && c.dtype != CS_BF16) || (c.out_dtype != CS_F32 && c.out_dtype != CS_BF16))
    return fail(CS_ERR_INVALID_ARG, "config.dtype / out_dtype");
  if (c.hidden <= 0 || c.n_heads <= 0 || c.head_dim <= 0 || c.n_heads * c.head_dim != c.hidden)
    return fail(CS_ERR_INVALID_ARG, "config: n_heads * head_dim must equal hidden");
  if (c.head_dim != 64 && c.head_dim != 80) return fail(CS_ERR_UNSUPPORTED, "config: head_dim must be 64 or 80");
  if (c.hidden % 64 || c.hidden > 2048) return fail(CS_ERR_UNSUPPORTED, "config: hidden must be a multiple of 64, at most 2048");
  if (c.n_layers <= 0 || c.n_layers > 64) return fail(CS_ERR_UNSUPPORTED, "config: 1..64 layers");
  if (c.mlp_dim <= 0 || c.out_hidden <= 0 || c.patch_dim <= 0) return fail(CS_ERR_INVALID_ARG, "config: sizes");
  if (c.patch_dim % 4) return fail(CS_ERR_UNSUPPORTED, "config: patch_dim must be a multiple of 4");
  if ((c.out_hidden * (c.out_dtype == CS_BF16 ? 2 : 4)) % 16)
    return fail(CS_ERR_UNSUPPORTED, "config: an output row must be a multiple of 16 bytes");
  if (c.arch == CS_ARCH_VIT) {
    if (c.merge != 2) return fail(CS_ERR_UNSUPPORTED, "config: merge must be 2");
    if (c.merger_hidden <= 0) return fail(CS_ERR_INVALID_ARG, "config: merger_hidden");
    if (c.window > 0 && c.window % c.merge) return fail(CS_ERR_UNSUPPORTED, "config: window must be a multiple of merge");
    const int s = c.rope_sections[0] + c.rope_sections[1] + c.rope_sections[2];
    if (c.rope_sections[0] < 0 || c.rope_sections[1] < 0 || c.rope_sections[2] < 0 || (s != 0 && s != c.head_dim / 2))
      return fail(CS_ERR_INVALID_ARG, "config: rope_sections must sum to head_dim/2 (or all be 0)");
    if (s && !(c.rope_theta > 0)) return fail(CS_ERR_INVALID_ARG, "config: rope_theta");
  } else if (c.arch == CS_ARCH_VIT_CLS) {
    if (c.merge != 2) return fail(CS_ERR_UNSUPPORTED, "config: merge must be 2");
    if (c.merger_hidden <= 0) return fail(CS_ERR_INVALID_ARG, "config: merger_hidden");
    if (c.window > 0 || c.rope_sections[0] || c.rope_sections[1] || c.rope_sections[2])
      return fail(CS_ERR_UNSUPPORTED, "config: a class-token tower has full attention and learned positions (window <= 0, no rotary sections)");
    if (4 * c.hidden > 8192) return fail(CS_ERR_UNSUPPORTED, "config: hidden of a class-token tower is at most 2048");
  } else {
    if (c.merge < 1 || c.merge > 8) return fail(CS_ERR_UNSUPPORTED, "config: pool must be 1..8");
    if (c.conv_kernel != 3) return fail(CS_ERR_UNSUPPORTED, "config: conv_kernel must be 3");
    if (c.patch_dim % 64) return fail(CS_ERR_UNSUPPORTED, "config: mel bins must be a multiple of 64");
  }
  if (!(c.norm_eps >= 0)) return fail(CS_ERR_INVALID_ARG, "config: norm_eps");
  return CS_OK;
}

struct WeightBook {
  std::map<std::string, SrcTensor> m;
  int dtype;
  cs_status get(const std::string& name, int64_t numel, SrcTensor& out, bool optional = false) const {
    auto it = m.find(name);
    if (it == m.end()) {
      if (optional) {
        out = SrcTensor();
        return CS_OK;
      }
      return fail(CS_ERR_MISSING_WEIGHT, "missing weight: " + name);
    }
    if (it->second.numel != numel)
      return fail(CS_ERR_SHAPE, "weight " + name + ": expected " + std::to_string(numel) + " elements, got " +
                                    std::to_string(it->second.numel));
    out = it->second;
    return CS_OK;
  }
};

// [rows, cols] -> bf16 [rows_pad, cols_pad] zero padded, row r taken from source row row_of(r)
template <class RowOf>
static size_t pack_matrix(Arena& A, const SrcTensor& t, int64_t rows_pad, int64_t cols, int64_t cols_pad, RowOf row_of) {
  const size_t off = A.alloc((size_t)rows_pad * cols_pad * 2);
  for (int64_t r = 0; r < rows_pad; ++r) {
    const int64_t sr = row_of(r);
    if (sr < 0) continue;
    bf16_t* d = A.bf(off) + r * cols_pad;
    if (t.dtype == CS_BF16) {
      memcpy(d, static_cast<const bf16_t*>(t.data) + sr * cols, (size_t)cols * 2);
    } else {
      const float* s = static_cast<const float*>(t.data) + sr * cols;
      for (int64_t c = 0; c < cols; ++c) d[c] = host_f2bf(s[c]);
    }
  }
  return off;
}

// LN(x) W^T + b = rs ((x g) W^T - mu c) + d with c[j] = sum_k g[k] W[j][k] and d[j] = b[j] + sum_k beta[k] W[j][k]:
// what a GEMM needs to take a LayerNorm's place (the product itself runs on bf16(x g); rs and mu come from
// per-row sums).  W, b as packed (bf16 rows in the GEMM's order, fp32 bias), g and beta fp32 [K].
static void fold_vectors(Arena& A, size_t w, size_t bias, size_t gain, size_t beta, int64_t rows, int64_t K, size_t* c_off,
                         size_t* d_off) {
  *c_off = A.alloc((size_t)rows * 4);
  *d_off = A.alloc((size_t)rows * 4);
  const bf16_t* W = A.bf(w);
  const float *b = A.f32(bias), *g = A.f32(gain), *be = beta ? A.f32(beta) : nullptr;
  for (int64_t j = 0; j < rows; ++j) {
    double c = 0.0, d = b[j];
    for (int64_t k = 0; k < K; ++k) {
      const double wv = host_bf2f(W[j * K + k]);
      c += wv * g[k];
      if (be) d += wv * be[k];
    }
    A.f32(*c_off)[j] = (float)c;
    A.f32(*d_off)[j] = (float)d;
  }
}

template <class RowOf>
static size_t pack_vector(Arena& A, const SrcTensor& t, int64_t n_pad, RowOf idx_of) {
  const size_t off = A.alloc((size_t)n_pad * 4);
  if (!t.data) return off;  // absent bias: zeros
  for (int64_t i = 0; i < n_pad; ++i) {
    const int64_t si = idx_of(i);
    if (si >= 0) A.f32(off)[i] = t.at(si);
  }
  return off;
}

static cs_status build_weights(cs_encoder* e, const WeightBook& wb, Arena& A) {
  const cs_encoder_config& c = e->cfg;
  const int64_t D = c.hidden, I = c.mlp_dim, dh = c.head_dim;
  auto ident = [](int64_t r) { return r; };
  SrcTensor t, b;
  // q and k rows are permuted inside every head so that the two members of rotary pair j
  // (dims j and j + dh/2) sit in neighbouring columns 2j, 2j+1; q.k is unchanged by a common permutation.
  auto qkv_row = [&](int64_t r) -> int64_t {
    if (!e->rope || r >= 2 * D) return r;
    const int64_t base = r - r % dh, p = r % dh;
    return base + ((p & 1) ? p / 2 + dh / 2 : p / 2);
  };
  e->layers.resize(c.n_layers);
  for (int l = 0; l < c.n_layers; ++l) {
    const std::string p = "blocks." + std::to_string(l) + ".";
    LayerW& L = e->layers[l];
    if (cs_status st = wb.get(p + "norm1.weight", D, t)) return st;
    L.g1 = pack_vector(A, t, D, ident);
    if (cs_status st = wb.get(p + "norm2.weight", D, t)) return st;
    L.g2 = pack_vector(A, t, D, ident);
    L.be1 = L.be2 = 0;
    if (c.arch != CS_ARCH_VIT) {
      if (cs_status st = wb.get(p + "norm1.bias", D, t, true)) return st;
      L.be1 = pack_vector(A, t, D, ident);
      if (cs_status st = wb.get(p + "norm2.bias", D, t, true)) return st;
      L.be2 = pack_vector(A, t, D, ident);
    }
    if (cs_status st = wb.get(p + "attn.qkv.weight", 3 * D * D, t)) return st;
    if (cs_status st = wb.get(p + "attn.qkv.bias", 3 * D, b, true)) return st;
    L.wqkv = pack_matrix(A, t, 3 * D, D, D, qkv_row);
    L.bqkv = pack_vector(A, b, 3 * D, qkv_row);
    if (cs_status st = wb.get(p + "attn.proj.weight", D * D, t)) return st;
    if (cs_status st = wb.get(p + "attn.proj.bias", D, b, true)) return st;
    L.wo = pack_matrix(A, t, D, D, D, ident);
    L.bo = pack_vector(A, b, D, ident);
    if (c.arch == CS_ARCH_VIT_CLS) {
      if (cs_status st = wb.get(p + "ls1", D, t)) return st;
      L.ls1 = pack_vector(A, t, D, ident);
      if (cs_status st = wb.get(p + "ls2", D, t)) return st;
      L.ls2 = pack_vector(A, t, D, ident);
    }
    if (c.arch == CS_ARCH_VIT) {
      // gate and up rows interleaved in blocks of 32 so that one lane holds gate_j and up_j
      SrcTensor tg, tu, bg, bu;
      if (cs_status st = wb.get(p + "mlp.gate.weight", I * D, tg)) return st;
      if (cs_status st = wb.get(p + "mlp.up.weight", I * D, tu)) return st;
      if (cs_status st = wb.get(p + "mlp.gate.bias", I, bg, true)) return st;
      if (cs_status st = wb.get(p + "mlp.up.bias", I, bu, true)) return st;
      const int64_t Ip = e->I_pad;
      L.w1 = A.alloc((size_t)2 * Ip * D * 2);
      L.b1 = A.alloc((size_t)2 * Ip * 4);
      for (int64_t r = 0; r < 2 * Ip; ++r) {
        const int64_t blk = r / 64, in = r % 64;
        const int64_t j = blk * 32 + (in & 31);
        if (j >= I) continue;
        const SrcTensor& w = in < 32 ? tg : tu;
        const SrcTensor& bb = in < 32 ? bg : bu;
        bf16_t* d = A.bf(L.w1) + r * D;
        for (int64_t k = 0; k < D; ++k) d[k] = w.bits(j * D + k);
        if (bb.data) A.f32(L.b1)[r] = bb.at(j);
      }
      if (cs_status st = wb.get(p + "mlp.down.weight", D * I, t)) return st;
      if (cs_status st = wb.get(p + "mlp.down.bias", D, b, true)) return st;
      L.w2 = pack_matrix(A, t, D, I, Ip, ident);
      L.b2 = pack_vector(A, b, D, ident);
    } else {
      const int64_t Ip = e->I_pad;
      if (cs_status st = wb.get(p + "mlp.fc1.weight", I * D, t)) return st;
      if (cs_status st = wb.get(p + "mlp.fc1.bias", I, b, true)) return st;
      L.w1 = pack_matrix(A, t, Ip, D, D, [&](int64_t r) { return r < I ? r : -1; });
      L.b1 = pack_vector(A, b, Ip, [&](int64_t r) { return r < I ? r : -1; });
      if (cs_status st = wb.get(p + "mlp.fc2.weight", D * I, t)) return st;
      if (cs_status st = wb.get(p + "mlp.fc2.bias", D, b, true)) return st;
      L.w2 = pack_matrix(A, t, D, I, Ip, ident);
      L.b2 = pack_vector(A, b, D, ident);
      fold_vectors(A, L.wqkv, L.bqkv, L.g1, L.be1, 3 * D, D, &L.cqkv, &L.dqkv);
      fold_vectors(A, L.w1, L.b1, L.g2, L.be2, Ip, D, &L.c1, &L.d1);
    }
  }
  if (c.arch == CS_ARCH_VIT || c.arch == CS_ARCH_VIT_CLS) {
    const int64_t P = c.patch_dim, G = (int64_t)c.merge * c.merge * D, MH = c.merger_hidden, H = c.out_hidden;
    if (cs_status st = wb.get("patch_embed.weight", D * P, t)) return st;
    e->w_pe = pack_matrix(A, t, D, P, e->P_pad, ident);
    if (c.arch == CS_ARCH_VIT) {
      if (cs_status st = wb.get("merger.norm.weight", D, t)) return st;
      e->g_m = pack_vector(A, t, D, ident);
    } else {
      // the projector's LayerNorm runs over the concatenation of a merge group
      if (cs_status st = wb.get("merger.norm.weight", G, t)) return st;
      e->g_m = pack_vector(A, t, G, ident);
      if (cs_status st = wb.get("merger.norm.bias", G, b, true)) return st;
      e->be_m = pack_vector(A, b, G, ident);
      if (cs_status st = wb.get("patch_embed.bias", D, b, true)) return st;
      e->b_pe = pack_vector(A, b, D, ident);
      // position table, and behind it the row the class token starts from (class token + position 0)
      SrcTensor cls, pe;
      if (cs_status st = wb.get("cls_token", D, cls)) return st;
      auto it = wb.m.find("pos_embed");
      if (it == wb.m.end()) return fail(CS_ERR_MISSING_WEIGHT, "missing weight: pos_embed");
      pe = it->second;
      if (pe.numel % D || pe.numel / D < 5 || pe.numel / D > (1 << 20))
        return fail(CS_ERR_SHAPE, "weight pos_embed: expected [1 + patches per tile, hidden]");
      e->n_positions = (int)(pe.numel / D);
      e->pos_tab = A.alloc((size_t)(e->n_positions + 1) * D * 4);
      for (int64_t i = 0; i < pe.numel; ++i) A.f32(e->pos_tab)[i] = pe.at(i);
      for (int64_t i = 0; i < D; ++i) A.f32(e->pos_tab)[pe.numel + i] = cls.at(i) + pe.at(i);
    }
    if (cs_status st = wb.get("merger.fc1.weight", MH * G, t)) return st;
    if (cs_status st = wb.get("merger.fc1.bias", MH, b, true)) return st;
    // The merger runs with split operands: its two inputs are carried as bf16 hi + bf16 lo
    // (value = hi + lo to ~16 bits), concatenated along K, against the weight matrix repeated twice.
    // It is 1.7 % of the FLOPs and the last stage before the output, where a plain bf16 rounding of
    // the normalised tokens alone costs a fifth of the error budget.
    e->w_m1 = A.alloc((size_t)e->MH_pad * 2 * G * 2);
    for (int64_t r = 0; r < MH; ++r)
      for (int rep = 0; rep < 2; ++rep)
        for (int64_t k = 0; k < G; ++k) A.bf(e->w_m1)[(r * 2 + rep) * G + k] = t.bits(r * G + k);
    e->b_m1 = pack_vector(A, b, e->MH_pad, [&](int64_t r) { return r < MH ? r : -1; });
    if (cs_status st = wb.get("merger.fc2.weight", H * MH, t)) return st;
    if (cs_status st = wb.get("merger.fc2.bias", H, b, true)) return st;
    e->w_m2 = A.alloc((size_t)H * 2 * e->MH_pad * 2);
    for (int64_t r = 0; r < H; ++r)
      for (int rep = 0; rep < 2; ++rep)
        for (int64_t k = 0; k < MH; ++k) A.bf(e->w_m2)[(r * 2 + rep) * e->MH_pad + k] = t.bits(r * MH + k);
    e->b_m2 = pack_vector(A, b, H, ident);
    // rotary: per pair j the axis it follows and its inverse frequency
    e->inv_freq = A.alloc((size_t)std::max(e->half, 1) * 4);
    e->axis = A.alloc((size_t)std::max(e->half, 1) * 4);
    if (e->rope) {
      int j = 0;
      for (int a = 0; a < 3; ++a)
        for (int i = 0; i < c.rope_sections[a]; ++i, ++j) {
          A.f32(e->inv_freq)[j] = (float)pow((double)c.rope_theta, -(double)i / c.rope_sections[a]);
          reinterpret_cast<int32_t*>(A.host.data() + e->axis)[j] = a;
        }
    }
  } else {
    const int64_t C = c.patch_dim, H = c.out_hidden;
    // conv weight [out, in, 3] -> [out, 3*in] with column d*in + c (tap-major), matching an input row
    // made of three consecutive frames
    auto pack_conv = [&](const SrcTensor& w, int64_t cin) {
      const size_t off = A.alloc((size_t)D * 3 * cin * 2);
      for (int64_t o = 0; o < D; ++o)
        for (int64_t d = 0; d < 3; ++d)
          for (int64_t ci = 0; ci < cin; ++ci) A.bf(off)[(o * 3 + d) * cin + ci] = w.bits((o * cin + ci) * 3 + d);
      return off;
    };
    if (cs_status st = wb.get("conv1.weight", D * C * 3, t)) return st;
    if (cs_status st = wb.get("conv1.bias", D, b, true)) return st;
    e->w_c1 = pack_conv(t, C);
    e->b_c1 = pack_vector(A, b, D, ident);
    if (cs_status st = wb.get("conv2.weight", D * D * 3, t)) return st;
    if (cs_status st = wb.get("conv2.bias", D, b, true)) return st;
    e->w_c2 = pack_conv(t, D);
    e->b_c2 = pack_vector(A, b, D, ident);
    if (cs_status st = wb.get("post.norm.weight", D, t)) return st;
    if (cs_status st = wb.get("post.norm.bias", D, b, true)) return st;
    e->g_p = pack_vector(A, t, D, ident);
    e->be_p = pack_vector(A, b, D, ident);
    if (cs_status st = wb.get("post.proj.weight", H * D, t)) return st;
    if (cs_status st = wb.get("post.proj.bias", H, b, true)) return st;
    e->w_p = pack_matrix(A, t, H, D, D, ident);
    e->b_p = pack_vector(A, b, H, ident);
    // sinusoidal positions: sin(pos w_i) | cos(pos w_i), w_i = exp(-i ln(10000)/(D/2-1))
    e->pe_positions = 4096;
    e->pe_tab = A.alloc((size_t)e->pe_positions * D * 4);
    const int64_t hD = D / 2;
    for (int64_t pos = 0; pos < e->pe_positions; ++pos)
      for (int64_t i = 0; i < hD; ++i) {
        const double a = (double)pos * exp(-(double)i * log(10000.0) / (double)(hD - 1));
        A.f32(e->pe_tab)[pos * D + i] = (float)sin(a);
        A.f32(e->pe_tab)[pos * D + hD + i] = (float)cos(a);
      }
  }
  return CS_OK;
}

// ---- workspace layout -----------------------------------------------------------------------
struct Workspace {
  size_t plan, rope, x, xn, attn, qk, vt, big, parts, ss, total;
  int64_t ld_vt, ss_stride;
  size_t s1 = 0;              // LayerNorm towers: per-row partial plain sums, laid out like ss
  int fold_proj, fold_down;   // column tiles of the two residual GEMMs when they fold the next RMSNorm (0: they do not)
  bool split_k;   // small batches: the residual GEMMs run split over K into `parts`
  int s_proj = 1, s_down = 1;   // ... the out projection and the down projection into so many
};

// Residual GEMMs of small batches (few workgroups, long K loops) are split over K: up to this many parts
constexpr int MAX_K_PARTS = PENDING_MAX_PARTS;
constexpr int64_t SPLIT_K_MAX_TOKENS = 2560;

// Parts for x += A W^T with M rows, N columns, K deep on 128 x 128 tiles: as many (at most MAX_K_PARTS)
// as divide the K slices evenly, leave four slices or more per part and keep the launch within 640 workgroups.
static int k_parts(int64_t M, int64_t N, int64_t K) {
  const int64_t wgs = ((M + 127) / 128) * ((N + 127) / 128);
  if (wgs > 160) return 1;
  const int64_t kt = K / 64;
  int best = 1;
  for (int s = 2; s <= MAX_K_PARTS; ++s)
    if (kt % s == 0 && kt / s >= 4 && wgs * s <= 640) best = s;
  return best;
}

// Measurement switch: CS_NO_NORM_FOLD=1 in the environment keeps every RMSNorm a kernel of its own (read once).
static bool fold_off() {
  static const bool off = [] {
    const char* v = getenv("CS_NO_NORM_FOLD");
    return v && *v && *v != '0';
  }();
  return off;
}

static Workspace layout_workspace(const cs_encoder* e, const BatchPlan& p) {
  const cs_encoder_config& c = e->cfg;
  const int64_t N = p.n_tok, D = c.hidden;
  Workspace w;
  size_t off = 0;
  auto take = [&](size_t bytes) {
    const size_t o = off;
    off = (size_t)round_up((int64_t)(off + bytes), 256);
    return o;
  };
  w.plan = take(p.blob.size() * 4);
  w.rope = take((size_t)N * std::max(e->half, 1) * 8);
  w.x = take((size_t)N * D * 4);
  w.xn = take((size_t)N * D * 4);            // bf16 tokens; twice that for the merger's hi|lo input
  w.attn = take((size_t)N * D * 2);
  w.qk = take((size_t)N * 2 * D * 2);
  w.ld_vt = round_up(N, 64);   // rows of v^T start on 128-byte lines (write-through stores need that)
  w.vt = take((size_t)D * w.ld_vt * 2);
  size_t big = (size_t)N * e->I_pad * 2;                                   // MLP activation
  if (c.arch != CS_ARCH_AUDIO) {
    big = std::max(big, (size_t)N * e->P_pad * 2);                          // gathered patches
    big = std::max(big, (size_t)p.n_groups * e->MH_pad * 4);                // merger hidden, hi|lo
  } else {
    // padded mel frames, then padded conv1 output, both alive during conv1
    big = std::max(big, (size_t)round_up(p.n_pad_rows * c.patch_dim * 2, 256) + (size_t)p.n_pad_rows * D * 2);
  }
  w.big = take(big);
  w.split_k = N <= SPLIT_K_MAX_TOKENS;
  // partial sums of the widest split GEMM: the residual ones (N x D) or the merger's (groups x its widths)
  size_t part = (size_t)N * D;
  if (c.arch != CS_ARCH_AUDIO) part = std::max(part, (size_t)p.n_groups * std::max<int64_t>(e->MH_pad, c.out_hidden));
  w.parts = take(w.split_k ? (size_t)MAX_K_PARTS * part * 4 : 0);
  // RMSNorm folded into the GEMMs around it (vision tower, unsplit residual GEMMs): per-row partial sums of
  // squares, one per column tile of the residual GEMM
  w.ss_stride = round_up(N, 64);
  // (a residual GEMM that runs split over K leaves its partial sums to the normalisation kernel: no fold)
  const bool ln = c.arch != CS_ARCH_VIT, scaled = c.arch == CS_ARCH_VIT_CLS;
  w.s_proj = w.split_k ? k_parts(N, D, D) : 1;
  w.s_down = w.split_k ? k_parts(N, D, e->I_pad) : 1;
  // The out projection's short K loop is not split once 128 x 160 tiles fill half the chip: unsplit, the launch
  // folds the next RMSNorm into its epilogue, which saves more than the split gains (2048 tokens: 5.33 -> 5.19 ms
  // per step; 1024 tokens: 3.95 -> 4.00 ms, so those stay split).
  if (w.s_proj > 1 && c.arch == CS_ARCH_VIT && D % 160 == 0 && ((N + 127) / 128) * (D / 160) >= 128 && !fold_off() &&
      gemm_norm_fold_parts(N, D, D, scaled, ln) > 0)
    w.s_proj = 1;
  w.fold_proj = w.s_proj == 1 && !fold_off() ? gemm_norm_fold_parts(N, D, D, scaled, ln) : 0;
  w.fold_down = w.s_down == 1 && !fold_off() ? gemm_norm_fold_parts(N, D, e->I_pad, scaled, ln) : 0;
  w.ss = take((w.fold_proj || w.fold_down) ? (size_t)8 * w.ss_stride * 4 : 0);
  w.s1 = take(ln && (w.fold_proj || w.fold_down) ? (size_t)8 * w.ss_stride * 4 : 0);
  w.total = off;
  return w;
}

// Records an event pair around the launches of one step when that step is being timed.
struct StepTimer {
  cs_encoder* e;
  hipStream_t stream;
  bool on;
  StepTimer(cs_encoder* enc, int step, hipStream_t s) : e(enc), stream(s), on(enc->time_step == step && !enc->capturing) {
    if (on) on = (e->time_seen++ % e->time_every) == 0;
    if (!on) return;
    if (e->ev_used + 2 > e->ev_pool.size()) {
      hipEvent_t a = nullptr, b = nullptr;
      if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) { on = false; return; }
      e->ev_pool.push_back(a);
      e->ev_pool.push_back(b);
    }
    (void)hipEventRecord(e->ev_pool[e->ev_used], stream);
  }
  ~StepTimer() {
    if (!on) return;
    (void)hipEventRecord(e->ev_pool[e->ev_used + 1], stream);
    e->ev_used += 2;
  }
};

static cs_status build_plan(const cs_encoder* e, const int32_t* cu, const int32_t* grid, int32_t n_items, BatchPlan& p) {
  if (e->cfg.arch == CS_ARCH_VIT) return build_vit_plan(e->cfg, cu, grid, n_items, p);
  if (e->cfg.arch == CS_ARCH_VIT_CLS) return build_cls_plan(e->cfg, e->n_positions, cu, grid, n_items, p);
  cs_status st = build_audio_plan(e->cfg, cu, grid, n_items, p);
  if (st) return st;
  for (int i = 0; i < n_items; ++i)
    if (grid[3 * i + 2] / 2 > e->pe_positions) return fail(CS_ERR_UNSUPPORTED, "audio clip longer than the position table");
  return CS_OK;
}

// The plan of a batch depends only on its description, and a serving loop sees the same few
// descriptions again and again (one image size, one clip length): the last PLAN_CACHE_ENTRIES distinct
// ones are kept per encoder.  The returned pointer stays valid until the next call on this encoder.
constexpr size_t PLAN_CACHE_ENTRIES = 8;
static cs_status get_plan(const cs_encoder* e, const int32_t* cu, const int32_t* grid, int32_t n_items,
                          const BatchPlan** out) {
  if (!cu || !grid) return fail(CS_ERR_INVALID_ARG, "cu_seqlens / grid_thw is NULL");
  if (n_items <= 0) return fail(CS_ERR_INVALID_ARG, "n_items must be positive");
  std::lock_guard<std::mutex> lock(e->plan_mu);
  for (cs_encoder::CachedPlan& c : e->plans) {
    if ((int64_t)c.key.size() != 4 * (int64_t)n_items + 2 || c.key[0] != n_items) continue;
    if (memcmp(c.key.data() + 1, cu, ((size_t)n_items + 1) * 4) != 0) continue;
    if (memcmp(c.key.data() + n_items + 2, grid, (size_t)n_items * 12) != 0) continue;
    c.stamp = ++e->plan_clock;
    ++e->plan_hits;
    *out = &c.plan;
    return CS_OK;
  }
  BatchPlan p;
  if (cs_status st = build_plan(e, cu, grid, n_items, p)) return st;
  ++e->plan_misses;
  cs_encoder::CachedPlan* slot = nullptr;
  if (e->plans.size() < PLAN_CACHE_ENTRIES) {
    e->plans.emplace_back();
    slot = &e->plans.back();
  } else {
    slot = &e->plans[0];
    for (cs_encoder::CachedPlan& c : e->plans)
      if (c.stamp < slot->stamp) slot = &c;
  }
  slot->key.resize(4 * (size_t)n_items + 2);
  slot->key[0] = n_items;
  memcpy(slot->key.data() + 1, cu, ((size_t)n_items + 1) * 4);
  memcpy(slot->key.data() + n_items + 2, grid, (size_t)n_items * 12);
  slot->plan = std::move(p);
  slot->stamp = ++e->plan_clock;
  *out = &slot->plan;
  return CS_OK;
}

// No exception may cross the C boundary: host allocations (vectors, strings, `new`) can throw.
template <class F>
static cs_status guarded(const char* who, F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return fail(CS_ERR_NO_MEMORY, std::string(who) + ": out of host memory");
  } catch (const std::exception& ex) {
    return fail(CS_ERR_INVALID_ARG, std::string(who) + ": " + ex.what());
  } catch (...) {
    return fail(CS_ERR_INVALID_ARG, std::string(who) + ": unknown exception");
  }
}

// What a pinned staging slot holds from create on: enough for the index tables of some 40 000 tokens
// (the tables take about 24 bytes per token).  Larger batches grow the slot in cs_encode, which blocks.
constexpr size_t STAGE_BYTES_AT_CREATE = (size_t)1 << 20;

}  // namespace cs

extern "C" {

const char* cs_status_string(cs_status s) {
  switch (s) {
    case CS_OK: return "ok";
    case CS_ERR_INVALID_ARG: return "invalid argument";
    case CS_ERR_SHAPE: return "inconsistent shapes";
    case CS_ERR_WORKSPACE: return "workspace too small";
    case CS_ERR_INDEX: return "index out of range";
    case CS_ERR_UNSUPPORTED: return "unsupported configuration";
    case CS_ERR_HIP: return "HIP runtime error";
    case CS_ERR_MISSING_WEIGHT: return "missing weight";
    case CS_ERR_BUSY: return "busy";
    case CS_ERR_NO_MEMORY: return "out of host memory";
    case CS_ERR_TIMEOUT: return "timed out";
  }
  return "unknown status";
}

const char* cs_last_error(void) { return g_last_error.c_str(); }

static cs_status encoder_create(const cs_encoder_config* config, const cs_tensor* weights, int32_t n_weights,
                                cs_encoder** out_encoder) {
  if (!config || !out_encoder || (!weights && n_weights > 0) || n_weights < 0)
    return fail(CS_ERR_INVALID_ARG, "cs_encoder_create: NULL argument");
  *out_encoder = nullptr;
  if (cs_status st = check_config(*config)) return st;
  WeightBook wb;
  wb.dtype = config->dtype;
  for (int i = 0; i < n_weights; ++i) {
    if (!weights[i].name || !weights[i].data || weights[i].numel <= 0)
      return fail(CS_ERR_INVALID_ARG, "cs_encoder_create: weight entry " + std::to_string(i) + " is incomplete");
    SrcTensor t;
    t.data = weights[i].data;
    t.numel = weights[i].numel;
    t.dtype = config->dtype;
    wb.m[weights[i].name] = t;
  }
  cs_encoder* e = new cs_encoder();
  e->cfg = *config;
  const cs_encoder_config& c = e->cfg;
  e->P_pad = (int)round_up(c.patch_dim, 64);
  e->I_pad = (int)round_up(c.mlp_dim, 64);
  e->MH_pad = c.arch != CS_ARCH_AUDIO ? (int)round_up(c.merger_hidden, 64) : 0;
  e->half = c.head_dim / 2;
  e->rope = c.arch == CS_ARCH_VIT && (c.rope_sections[0] + c.rope_sections[1] + c.rope_sections[2]) > 0;
  Arena A;
  A.alloc(256);  // offset 0 stays unused so that 0 can mean "absent"
  cs_status st = build_weights(e, wb, A);
  if (st == CS_OK) {
    hipError_t he = hipGetDevice(&e->device);
    if (he == hipSuccess) he = hipMalloc(reinterpret_cast<void**>(&e->dev), A.host.size());
    if (he == hipSuccess) he = hipMemcpy(e->dev, A.host.data(), A.host.size(), hipMemcpyHostToDevice);
    for (int s = 0; s < 2 && he == hipSuccess; ++s) he = hipEventCreateWithFlags(&e->stage_ev[s], hipEventDisableTiming);
    for (int s = 0; s < 2 && he == hipSuccess; ++s) {
      he = hipHostMalloc(&e->stage[s], STAGE_BYTES_AT_CREATE, hipHostMallocDefault);
      if (he == hipSuccess) e->stage_cap[s] = STAGE_BYTES_AT_CREATE;
    }
    if (he != hipSuccess) st = fail(CS_ERR_HIP, std::string("cs_encoder_create: ") + hipGetErrorString(he));
    e->dev_bytes = A.host.size();
    // the address of this device's copy of the static scratch array, for cs_encode_static
    if (st == CS_OK) {
      void* unused = nullptr;
      st = static_scratch(&unused);
    }
  }
  if (st != CS_OK) {
    cs_encoder_destroy(e);
    return st;
  }
  *out_encoder = e;
  return CS_OK;
}

cs_status cs_encoder_create(const cs_encoder_config* config, const cs_tensor* weights, int32_t n_weights,
                            cs_encoder** out_encoder) {
  return guarded("cs_encoder_create", [&] { return encoder_create(config, weights, n_weights, out_encoder); });
}

void cs_encoder_destroy(cs_encoder* e) {
  if (!e) return;
  if (e->dev) (void)hipFree(e->dev);
  for (hipEvent_t ev : e->ev_pool) (void)hipEventDestroy(ev);
  for (int s = 0; s < 2; ++s) {
    if (e->stage[s]) (void)hipHostFree(e->stage[s]);
    if (e->stage_ev[s]) (void)hipEventDestroy(e->stage_ev[s]);
  }
  delete e;
}

cs_status cs_encoder_time_step(cs_encoder* enc, int32_t step) {
  if (!enc || step < CS_STEP_NONE || step > CS_STEP_BACK) return fail(CS_ERR_INVALID_ARG, "cs_encoder_time_step");
  enc->time_step = step;
  enc->time_seen = 0;
  return CS_OK;
}

cs_status cs_encoder_time_every(cs_encoder* enc, int32_t every) {
  if (!enc || every < 1) return fail(CS_ERR_INVALID_ARG, "cs_encoder_time_every");
  enc->time_every = every;
  enc->time_seen = 0;
  return CS_OK;
}

cs_status cs_encoder_read_timing(cs_encoder* enc, double* total_ms, int64_t* launches) {
  if (!enc || !total_ms || !launches) return fail(CS_ERR_INVALID_ARG, "cs_encoder_read_timing: NULL argument");
  double sum = 0;
  for (size_t i = 0; i + 1 < enc->ev_used; i += 2) {
    CS_HIP(hipEventSynchronize(enc->ev_pool[i + 1]));
    float ms = 0;
    CS_HIP(hipEventElapsedTime(&ms, enc->ev_pool[i], enc->ev_pool[i + 1]));
    sum += ms;
  }
  *total_ms = sum;
  *launches = (int64_t)(enc->ev_used / 2);
  enc->ev_used = 0;
  return CS_OK;
}

cs_status cs_encoder_step_kernel(const cs_encoder* enc, int32_t step, int64_t n_tokens, char* out, size_t capacity) {
  if (!enc || !out || capacity < 96 || n_tokens <= 0 || n_tokens > 0x7fffffff)
    return fail(CS_ERR_INVALID_ARG, "cs_encoder_step_kernel: NULL argument, capacity below 96 or bad token count");
  const cs_encoder_config& c = enc->cfg;
  const int64_t D = c.hidden;
  GemmArgs g = {};
  g.describe = out;
  g.M = (int32_t)n_tokens;
  int epi = EPI_BF16;
  switch (step) {
    case CS_STEP_QKV:
      g.N = (int32_t)(3 * D); g.K = (int32_t)D; g.ldo = 2 * D; g.hidden = (int32_t)D; g.head_dim = c.head_dim; g.ld_vt = round_up(n_tokens, 64);
      g.M = (int32_t)round_up(n_tokens, 4);
      epi = EPI_QKV;
      break;
    case CS_STEP_PROJ:
      g.N = (int32_t)D; g.K = (int32_t)D; g.ldo = D;
      epi = c.arch == CS_ARCH_VIT_CLS ? EPI_RESADD_SCALED_F32 : EPI_RESADD_F32;
      break;
    case CS_STEP_MLP_UP:
      g.N = c.arch == CS_ARCH_VIT ? 2 * enc->I_pad : enc->I_pad; g.K = (int32_t)D; g.ldo = enc->I_pad;
      epi = c.arch == CS_ARCH_VIT ? EPI_SWIGLU_BF16 : EPI_GELU_BF16;
      break;
    case CS_STEP_MLP_DOWN:
      g.N = (int32_t)D; g.K = enc->I_pad; g.ldo = D;
      epi = c.arch == CS_ARCH_VIT_CLS ? EPI_RESADD_SCALED_F32 : EPI_RESADD_F32;
      break;
    default: return fail(CS_ERR_INVALID_ARG, "cs_encoder_step_kernel: step must be one of the four GEMM steps of a block");
  }
  // (an audio tower's residual GEMMs run the instantiation that also writes the plain sums of a folded LayerNorm)
  if (epi == EPI_RESADD_F32 && c.arch == CS_ARCH_AUDIO && !fold_off() &&
      (n_tokens > SPLIT_K_MAX_TOKENS || k_parts(n_tokens, D, g.K) == 1))
    g.s1_out = reinterpret_cast<float*>(uintptr_t(16));   // describe mode: only looked at, never written
  g.lda = g.K;
  if (epi == EPI_RESADD_SCALED_F32) g.col_scale = enc->ptr<float>(enc->layers[0].ls1);
  // (batches small enough for split K run other launches; this names the kernel of the unsplit path)
  return launch_gemm(epi, g, nullptr);
}

cs_status cs_encoder_query(const cs_encoder* enc, const int32_t* cu_seqlens, const int32_t* grid_thw, int32_t n_items,
                           int64_t* n_out_rows, size_t* workspace_bytes) {
  if (!enc) return fail(CS_ERR_INVALID_ARG, "cs_encoder_query: NULL encoder");
  return guarded("cs_encoder_query", [&]() -> cs_status {
    const BatchPlan* p = nullptr;
    if (cs_status st = get_plan(enc, cu_seqlens, grid_thw, n_items, &p)) return st;
    if (n_out_rows) *n_out_rows = p->n_out;
    if (workspace_bytes) *workspace_bytes = layout_workspace(enc, *p).total;
    return CS_OK;
  });
}

cs_status cs_encoder_plan_cache_stats(const cs_encoder* enc, int64_t* hits, int64_t* misses) {
  if (!enc) return fail(CS_ERR_INVALID_ARG, "cs_encoder_plan_cache_stats: NULL encoder");
  std::lock_guard<std::mutex> lock(enc->plan_mu);
  if (hits) *hits = (int64_t)enc->plan_hits;
  if (misses) *misses = (int64_t)enc->plan_misses;
  return CS_OK;
}

static cs_status plan_tokens(const cs_encoder_config* config, const int32_t* cu_seqlens, const int32_t* grid_thw,
                             int32_t n_items, int32_t* src_row, int32_t* out_row, int32_t* win_cu,
                             int32_t win_cu_capacity, int32_t* n_windows) {
  if (!config) return fail(CS_ERR_INVALID_ARG, "cs_plan_tokens: NULL config");
  if (cs_status st = check_config(*config)) return st;
  if (config->arch == CS_ARCH_AUDIO) return fail(CS_ERR_UNSUPPORTED, "cs_plan_tokens: vision encoders only");
  BatchPlan p;
  if (config->arch == CS_ARCH_VIT) {
    if (cs_status st = build_vit_plan(*config, cu_seqlens, grid_thw, n_items, p)) return st;
  } else {
    // without an encoder the position table is taken to fit the first tile
    if (!grid_thw || n_items <= 0) return fail(CS_ERR_INVALID_ARG, "cs_plan_tokens: no items");
    const int64_t n_pos = 1 + (int64_t)grid_thw[1] * grid_thw[2];
    if (n_pos < 5 || n_pos > (1 << 20)) return fail(CS_ERR_SHAPE, "cs_plan_tokens: tile size");
    if (cs_status st = build_cls_plan(*config, (int32_t)n_pos, cu_seqlens, grid_thw, n_items, p)) return st;
  }
  if (src_row) memcpy(src_row, p.blob.data() + p.off_src_row, (size_t)p.n_tok * 4);
  if (out_row) memcpy(out_row, p.blob.data() + p.off_out_row, (size_t)p.n_groups * 4);
  const int32_t nw = p.win_cu.empty() ? 0 : (int32_t)p.win_cu.size() - 1;
  if (n_windows) *n_windows = nw;
  if (win_cu && !p.win_cu.empty()) {
    if (win_cu_capacity < nw + 1) return fail(CS_ERR_INVALID_ARG, "cs_plan_tokens: win_cu_capacity too small");
    memcpy(win_cu, p.win_cu.data(), (size_t)(nw + 1) * 4);
  }
  return CS_OK;
}

cs_status cs_plan_tokens(const cs_encoder_config* config, const int32_t* cu_seqlens, const int32_t* grid_thw,
                         int32_t n_items, int32_t* src_row, int32_t* out_row, int32_t* win_cu,
                         int32_t win_cu_capacity, int32_t* n_windows) {
  return guarded("cs_plan_tokens", [&] {
    return plan_tokens(config, cu_seqlens, grid_thw, n_items, src_row, out_row, win_cu, win_cu_capacity, n_windows);
  });
}

// The encoder task.  may_grow: the pinned staging slots may be re-allocated for a batch whose index
// tables outgrow them (blocks the device); without it such a batch is refused and nothing allocates.
static cs_status encode_impl(cs_encoder* e, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                             int32_t n_items, void* out_embeddings, void* workspace, size_t workspace_bytes,
                             void* stream_, bool may_grow, const char* who, bool capturing = false) {
  if (!e || !patches || !out_embeddings || !workspace) return fail(CS_ERR_INVALID_ARG, std::string(who) + ": NULL argument");
  if ((reinterpret_cast<uintptr_t>(patches) | reinterpret_cast<uintptr_t>(out_embeddings) |
       reinterpret_cast<uintptr_t>(workspace)) & 15)
    return fail(CS_ERR_INVALID_ARG, std::string(who) + ": device pointers must be 16-byte aligned");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  const cs_encoder_config& c = e->cfg;
  const BatchPlan* plan_ptr = nullptr;
  if (cs_status st = get_plan(e, cu_seqlens, grid_thw, n_items, &plan_ptr)) return st;
  const BatchPlan& p = *plan_ptr;
  const Workspace w = layout_workspace(e, p);
  if (workspace_bytes < w.total)
    return fail(CS_ERR_WORKSPACE, std::string(who) + ": " + (may_grow ? "workspace" : "the static scratch") + " has " +
                                      std::to_string(workspace_bytes) + " bytes, this batch needs " + std::to_string(w.total));
  if (!may_grow && !capturing && p.blob.size() * 4 > std::min(e->stage_cap[0], e->stage_cap[1]))
    return fail(CS_ERR_WORKSPACE, std::string(who) + ": the index tables of this batch exceed the staging slots");
  unsigned char* ws = static_cast<unsigned char*>(workspace);

  // ---- index tables: host -> pinned slot -> workspace, one async copy (a stream under capture replays
  // launches only: the tables are already in the workspace from the eager call before the capture)
  if (!capturing) {
    const int s = e->stage_next;
    e->stage_next ^= 1;
    const size_t bytes = p.blob.size() * 4;
    if (e->stage_used[s]) CS_HIP(hipEventSynchronize(e->stage_ev[s]));  // the copy that last read this slot is done
    if (e->stage_cap[s] < bytes) {
      if (e->stage[s]) CS_HIP(hipHostFree(e->stage[s]));
      e->stage[s] = nullptr;
      e->stage_cap[s] = 0;
      CS_HIP(hipHostMalloc(&e->stage[s], bytes + bytes / 2, hipHostMallocDefault));
      e->stage_cap[s] = bytes + bytes / 2;
    }
    memcpy(e->stage[s], p.blob.data(), bytes);
    CS_HIP(hipMemcpyAsync(ws + w.plan, e->stage[s], bytes, hipMemcpyHostToDevice, stream));
    CS_HIP(hipEventRecord(e->stage_ev[s], stream));
    e->stage_used[s] = true;
  }
  const int32_t* plan = reinterpret_cast<const int32_t*>(ws + w.plan);
  const int64_t N = p.n_tok, D = c.hidden;
  float* x = reinterpret_cast<float*>(ws + w.x);
  bf16_t* xn = reinterpret_cast<bf16_t*>(ws + w.xn);
  bf16_t* attn = reinterpret_cast<bf16_t*>(ws + w.attn);
  bf16_t* qk = reinterpret_cast<bf16_t*>(ws + w.qk);
  bf16_t* vt = reinterpret_cast<bf16_t*>(ws + w.vt);
  bf16_t* big = reinterpret_cast<bf16_t*>(ws + w.big);
  float* rope_cs = reinterpret_cast<float*>(ws + w.rope);
  const bool vit = c.arch == CS_ARCH_VIT, cls = c.arch == CS_ARCH_VIT_CLS;
  const int out_epi = c.out_dtype == CS_BF16 ? EPI_BF16 : EPI_F32;

  auto gemm = [&](int epi, const bf16_t* A, int64_t lda, size_t W, size_t bias, void* out, int64_t ldo, int64_t M,
                  int64_t Nn, int64_t K, const int32_t* row_map) {
    GemmArgs g = {};
    g.A = A; g.lda = lda; g.W = e->ptr<bf16_t>(W); g.bias = bias ? e->ptr<float>(bias) : nullptr;
    g.out = out; g.ldo = ldo; g.row_map = row_map; g.M = (int32_t)M; g.N = (int32_t)Nn; g.K = (int32_t)K;
    return launch_gemm(epi, g, stream);
  };
  // x += [scale *] (A W^T + bias): a branch joining the residual stream (scale: class-token tower).
  // Small batches: partial sums over parts of K into the workspace (more workgroups, shorter K loops),
  // then one pass that adds them to x in a fixed order.
  float* parts = reinterpret_cast<float*>(ws + w.parts);
  PendingSum pending;
  auto take_pending = [&] {
    const PendingSum a = pending;
    pending = PendingSum();
    return a;
  };
  // for the consumers of x that cannot add pending sums themselves
  auto flush_pending = [&]() -> cs_status {
    if (!pending.parts) return CS_OK;
    const PendingSum a = take_pending();
    return launch_add_partials(x, a.parts, a.n_parts, a.stride, a.bias, a.scale, N, (int32_t)D, stream);
  };
  // RMSNorm folded into the GEMMs on both sides (vision tower): the residual GEMM in front of a norm also writes
  // xn = bf16(x * gain) and per-row sums of squares, the GEMM behind it scales its rows by 1 / rms.  folded > 0:
  // xn and ss are in that state, with so many partial sums per row.
  float* ss = reinterpret_cast<float*>(ws + w.ss);
  float* s1 = reinterpret_cast<float*>(ws + w.s1);
  int folded = 0;
  // shift, bias: the LayerNorm towers' vectors c and d of this GEMM (0 for the RMSNorm tower)
  auto consume_norm = [&](GemmArgs& g, size_t shift = 0, size_t bias = 0) {
    if (!folded) return;
    g.ss_in = ss; g.ss_parts = folded; g.ss_stride = w.ss_stride; g.norm_dim = (int32_t)D; g.norm_eps = c.norm_eps;
    if (!vit) {
      g.s1_in = s1; g.norm_shift = e->ptr<float>(shift); g.bias = e->ptr<float>(bias);
    }
    folded = 0;
  };
  auto gemm_residual = [&](const bf16_t* A, int64_t lda, size_t W, size_t bias, size_t scale, int64_t K, size_t next_gain,
                           int fold_parts, int S) -> cs_status {
    GemmArgs g = {};
    g.A = A; g.lda = lda; g.W = e->ptr<bf16_t>(W); g.ldo = D; g.M = (int32_t)N; g.N = (int32_t)D;
    if (S > 1) {
      g.ldw = K; g.K = (int32_t)(K / S); g.splits = S; g.split_stride = N * D; g.out = parts;
      if (cs_status st = launch_gemm(EPI_F32, g, stream)) return st;
      // the sums stay pending: the normalisation that reads x next adds them on its way through
      pending.parts = parts; pending.n_parts = S; pending.stride = N * D;
      pending.bias = e->ptr<float>(bias); pending.scale = scale ? e->ptr<float>(scale) : nullptr;
      return CS_OK;
    }
    g.bias = e->ptr<float>(bias); g.out = x; g.K = (int32_t)K;
    if (scale) g.col_scale = e->ptr<float>(scale);
    if (next_gain && fold_parts > 0) {
      g.norm_gain = e->ptr<float>(next_gain); g.xg = xn; g.ld_xg = D; g.ss_out = ss; g.ss_stride = w.ss_stride;
      if (!vit) g.s1_out = s1;
      folded = fold_parts;
    }
    return launch_gemm(scale ? EPI_RESADD_SCALED_F32 : EPI_RESADD_F32, g, stream);
  };

  // ---- front end: tokens into the fp32 residual stream x [N, D]
  {
    StepTimer tm(e, CS_STEP_FRONT, stream);
    if (vit) {
      if (cs_status st = launch_gather_cast(patches, c.dtype == CS_BF16, c.patch_dim, plan + p.off_src_row, big, e->P_pad, N, stream)) return st;
      if (e->rope)
        if (cs_status st = launch_rope_table(plan + p.off_pos, e->ptr<int32_t>(e->axis), e->ptr<float>(e->inv_freq), e->half, rope_cs, N, stream)) return st;
      if (cs_status st = gemm(EPI_F32, big, e->P_pad, e->w_pe, 0, x, D, N, D, e->P_pad, nullptr)) return st;
    } else if (cls) {
      // patch rows in internal order (zero rows where the class token and the padding go), embedded with
      // bias; then the positions are added and the class-token and padding rows are written
      if (cs_status st = launch_gather_cast(patches, c.dtype == CS_BF16, c.patch_dim, plan + p.off_src_row, big, e->P_pad, N, stream)) return st;
      if (cs_status st = gemm(EPI_F32, big, e->P_pad, e->w_pe, e->b_pe, x, D, N, D, e->P_pad, nullptr)) return st;
      if (cs_status st = launch_place_tokens(x, e->ptr<float>(e->pos_tab), plan + p.off_pos, e->n_positions, N, (int32_t)D, stream)) return st;
    } else {
      const int64_t R = p.n_pad_rows, C = c.patch_dim;
      bf16_t* melp = big;
      bf16_t* c1buf = reinterpret_cast<bf16_t*>(reinterpret_cast<unsigned char*>(big) + round_up(R * C * 2, 256));
      if (cs_status st = launch_gather_cast(patches, c.dtype == CS_BF16, (int32_t)C, plan + p.off_mel_src, melp, (int32_t)C, R, stream)) return st;
      if (cs_status st = launch_zero_rows(c1buf, plan + p.off_zero_rows, p.n_zero_rows, (int32_t)D, stream)) return st;
      if (cs_status st = gemm(EPI_GELU_BF16, melp, C, e->w_c1, e->b_c1, c1buf, D, R - 2, D, 3 * C, plan + p.off_c1_map)) return st;
      if (cs_status st = gemm(EPI_GELU_F32, c1buf, 2 * D, e->w_c2, e->b_c2, x, D, R / 2 - 1, D, 3 * D, plan + p.off_c2_map)) return st;
      if (cs_status st = launch_add_rows(x, e->ptr<float>(e->pe_tab), plan + p.off_pos, N, (int32_t)D, stream)) return st;
    }
  }

  // ---- transformer blocks
  AttnArgs aa = {};
  aa.qk = qk; aa.vt = vt; aa.ld_vt = w.ld_vt; aa.out = attn; aa.n_tok = (int32_t)N; aa.n_heads = c.n_heads; aa.head_dim = c.head_dim;
  const float q_scale = (float)(1.4426950408889634 / sqrt((double)c.head_dim));
  auto norm = [&](size_t gain, size_t bias) -> cs_status {
    if (folded) return CS_OK;      // the residual GEMM in front has written xn and the sums of squares
    StepTimer tm(e, CS_STEP_NORM, stream);
    if (vit) return launch_rmsnorm(x, e->ptr<float>(gain), c.norm_eps, xn, N, (int32_t)D, stream, take_pending());
    return launch_layernorm(x, e->ptr<float>(gain), e->ptr<float>(bias), c.norm_eps, xn, N, (int32_t)D, stream, take_pending());
  };
  for (int l = 0; l < c.n_layers; ++l) {
    const LayerW& L = e->layers[l];
    if (cs_status st = norm(L.g1, L.be1)) return st;
    {
      StepTimer tm(e, CS_STEP_QKV, stream);
      GemmArgs g = {};
      g.A = xn; g.lda = D; g.W = e->ptr<bf16_t>(L.wqkv); g.bias = e->ptr<float>(L.bqkv);
      g.out = qk; g.ldo = 2 * D; g.M = (int32_t)N; g.N = (int32_t)(3 * D); g.K = (int32_t)D;
      g.vt = vt; g.ld_vt = w.ld_vt; g.rope_cs = e->rope ? rope_cs : nullptr;
      g.hidden = (int32_t)D; g.head_dim = c.head_dim; g.q_scale = q_scale;
      consume_norm(g, L.cqkv, L.dqkv);
      if (cs_status st = launch_gemm(EPI_QKV, g, stream)) return st;
    }
    const bool full = !vit || c.window <= 0 || ((c.full_attn_layer_mask >> l) & 1);
    {
      StepTimer tm(e, full ? CS_STEP_ATTN_FULL : CS_STEP_ATTN_WINDOW, stream);
      if (full) {
        aa.work = reinterpret_cast<const AttnWork*>(plan + p.off_full_work); aa.n_work = p.n_full_work; aa.q_per_block = p.full_q_per_block; aa.single_tile = p.full_single_tile;
      } else {
        aa.work = reinterpret_cast<const AttnWork*>(plan + p.off_win_work); aa.n_work = p.n_win_work; aa.q_per_block = 64; aa.single_tile = p.win_single_tile;
      }
      if (cs_status st = launch_attention(aa, stream)) return st;
      if (full && p.n_tail_work > 0) {   // the short last query blocks of the items, as 64-query work items
        aa.work = reinterpret_cast<const AttnWork*>(plan + p.off_tail_work); aa.n_work = p.n_tail_work; aa.q_per_block = 64; aa.single_tile = 0;
        if (cs_status st = launch_attention(aa, stream)) return st;
      }
    }
    {
      StepTimer tm(e, CS_STEP_PROJ, stream);
      if (cs_status st = gemm_residual(attn, D, L.wo, L.bo, cls ? L.ls1 : 0, D, L.g2, w.fold_proj, w.s_proj)) return st;
    }
    if (cs_status st = norm(L.g2, L.be2)) return st;
    {
      StepTimer tm(e, CS_STEP_MLP_UP, stream);
      if (vit) {
        GemmArgs g = {};
        g.A = xn; g.lda = D; g.W = e->ptr<bf16_t>(L.w1); g.bias = e->ptr<float>(L.b1); g.out = big; g.ldo = e->I_pad;
        g.M = (int32_t)N; g.N = 2 * e->I_pad; g.K = (int32_t)D;
        consume_norm(g);
        if (cs_status st = launch_gemm(EPI_SWIGLU_BF16, g, stream)) return st;
      }
      else {
        GemmArgs g = {};
        g.A = xn; g.lda = D; g.W = e->ptr<bf16_t>(L.w1); g.bias = e->ptr<float>(L.b1); g.out = big; g.ldo = e->I_pad;
        g.M = (int32_t)N; g.N = e->I_pad; g.K = (int32_t)D;
        consume_norm(g, L.c1, L.d1);
        if (cs_status st = launch_gemm(EPI_GELU_BF16, g, stream)) return st;
      }
    }
    {
      StepTimer tm(e, CS_STEP_MLP_DOWN, stream);
      // (the norm behind the last block is the merger's, which splits its output: a kernel of its own)
      const size_t next_g1 = l + 1 < c.n_layers ? e->layers[l + 1].g1 : 0;
      if (cs_status st = gemm_residual(big, e->I_pad, L.w2, L.b2, cls ? L.ls2 : 0, e->I_pad, next_g1, w.fold_down, w.s_down)) return st;
    }
  }

  // ---- back end: merged / pooled tokens -> embedding rows
  {
    StepTimer tm(e, CS_STEP_BACK, stream);
    if (vit || cls) {
      const int64_t M = p.n_groups, G = (int64_t)c.merge * c.merge * D;
      if (vit) {
        if (cs_status st = launch_rmsnorm_split(x, e->ptr<float>(e->g_m), c.norm_eps, xn, N, (int32_t)D, c.merge * c.merge, stream, take_pending())) return st;
      } else {
        if (cs_status st = flush_pending()) return st;
        if (cs_status st = launch_layernorm_wide_split(x, e->ptr<float>(e->g_m), e->ptr<float>(e->be_m), c.norm_eps, xn, M, (int32_t)G, stream)) return st;
      }
      // small batches: both GEMMs split over K like the residual ones (a few merged rows against K = 2 * 4D)
      auto split_gemm = [&](const bf16_t* A, int64_t K, size_t W, int64_t Nn, int S) {
        GemmArgs g = {};
        g.A = A; g.lda = K; g.W = e->ptr<bf16_t>(W); g.ldw = K; g.K = (int32_t)(K / S); g.splits = S;
        g.split_stride = M * Nn; g.out = parts; g.ldo = Nn; g.M = (int32_t)M; g.N = (int32_t)Nn;
        return launch_gemm(EPI_F32, g, stream);
      };
      const int S1 = w.split_k ? k_parts(M, e->MH_pad, 2 * G) : 1, S2 = w.split_k ? k_parts(M, c.out_hidden, 2 * e->MH_pad) : 1;
      if (S1 > 1) {
        if (cs_status st = split_gemm(xn, 2 * G, e->w_m1, e->MH_pad, S1)) return st;
        if (cs_status st = launch_add_partials_gelu_split(big, parts, S1, M * e->MH_pad, e->ptr<float>(e->b_m1), M, e->MH_pad, stream)) return st;
      } else {
        if (cs_status st = gemm(EPI_GELU_SPLIT, xn, 2 * G, e->w_m1, e->b_m1, big, 2 * e->MH_pad, M, e->MH_pad, 2 * G, nullptr)) return st;
      }
      if (S2 > 1) {
        if (cs_status st = split_gemm(big, 2 * e->MH_pad, e->w_m2, c.out_hidden, S2)) return st;
        if (cs_status st = launch_add_partials_store(out_embeddings, c.out_dtype == CS_BF16, plan + p.off_out_row, parts, S2,
                                                     M * c.out_hidden, e->ptr<float>(e->b_m2), M, c.out_hidden, stream)) return st;
      } else {
        if (cs_status st = gemm(out_epi, big, 2 * e->MH_pad, e->w_m2, e->b_m2, out_embeddings, c.out_hidden, M, c.out_hidden, 2 * e->MH_pad, plan + p.off_out_row)) return st;
      }
    } else {
      if (cs_status st = flush_pending()) return st;
      if (cs_status st = launch_pool_layernorm(x, e->ptr<float>(e->g_p), e->ptr<float>(e->be_p), c.norm_eps, xn, p.n_out, (int32_t)D, c.merge, stream)) return st;
      if (cs_status st = gemm(out_epi, xn, D, e->w_p, e->b_p, out_embeddings, c.out_hidden, p.n_out, c.out_hidden, D, nullptr)) return st;
    }
  }
  return CS_OK;
}

cs_status cs_encode(cs_encoder* e, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                    int32_t n_items, void* out_embeddings, void* workspace, size_t workspace_bytes, void* stream) {
  return guarded("cs_encode", [&] {
    return encode_impl(e, patches, cu_seqlens, grid_thw, n_items, out_embeddings, workspace, workspace_bytes, stream,
                       true, "cs_encode");
  });
}

}  // extern "C"

// A recorded cs_encode: the launches of one batch on one set of buffers as an executable HIP graph.
struct cs_encode_graph {
  hipGraph_t graph = nullptr;
  hipGraphExec_t exec = nullptr;
};

extern "C" {

cs_status cs_encode_graph_create(cs_encoder* e, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                                 int32_t n_items, void* out_embeddings, void* workspace, size_t workspace_bytes,
                                 void* stream_, cs_encode_graph** out) {
  if (!out) return fail(CS_ERR_INVALID_ARG, "cs_encode_graph_create: NULL out");
  *out = nullptr;
  return guarded("cs_encode_graph_create", [&]() -> cs_status {
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (!stream) return fail(CS_ERR_INVALID_ARG, "cs_encode_graph_create: capture needs a stream of its own, not the default stream");
    // one eager call: validates, puts the index tables into the workspace, sets the kernels' attributes
    if (cs_status st = encode_impl(e, patches, cu_seqlens, grid_thw, n_items, out_embeddings, workspace, workspace_bytes,
                                   stream_, true, "cs_encode_graph_create"))
      return st;
    CS_HIP(hipStreamSynchronize(stream));
    cs_encode_graph* g = new cs_encode_graph();
    hipError_t he = hipStreamBeginCapture(stream, hipStreamCaptureModeThreadLocal);
    if (he != hipSuccess) {
      delete g;
      return fail(CS_ERR_HIP, std::string("cs_encode_graph_create: hipStreamBeginCapture: ") + hipGetErrorString(he));
    }
    e->capturing = true;
    const cs_status st = encode_impl(e, patches, cu_seqlens, grid_thw, n_items, out_embeddings, workspace, workspace_bytes,
                                     stream_, false, "cs_encode_graph_create", true);
    e->capturing = false;
    he = hipStreamEndCapture(stream, &g->graph);    // always ended, also after a failed launch
    if (st == CS_OK && he == hipSuccess) he = hipGraphInstantiate(&g->exec, g->graph, nullptr, nullptr, 0);
    if (st != CS_OK || he != hipSuccess) {
      if (g->graph) (void)hipGraphDestroy(g->graph);
      delete g;
      return st != CS_OK ? st : fail(CS_ERR_HIP, std::string("cs_encode_graph_create: ") + hipGetErrorString(he));
    }
    *out = g;
    return CS_OK;
  });
}

cs_status cs_encode_graph_launch(cs_encode_graph* g, void* stream) {
  if (!g || !g->exec) return fail(CS_ERR_INVALID_ARG, "cs_encode_graph_launch: NULL graph");
  CS_HIP(hipGraphLaunch(g->exec, static_cast<hipStream_t>(stream)));
  return CS_OK;
}

void cs_encode_graph_destroy(cs_encode_graph* g) {
  if (!g) return;
  if (g->exec) (void)hipGraphExecDestroy(g->exec);
  if (g->graph) (void)hipGraphDestroy(g->graph);
  delete g;
}

cs_status cs_encode_static(cs_encoder* e, const void* patches, const int32_t* cu_seqlens, const int32_t* grid_thw,
                           int32_t n_items, void* out_embeddings, void* stream) {
  return guarded("cs_encode_static", [&]() -> cs_status {
    void* ws = nullptr;
    if (cs_status st = static_scratch(&ws)) return st;
    return encode_impl(e, patches, cu_seqlens, grid_thw, n_items, out_embeddings, ws, CS_STATIC_SCRATCH_BYTES, stream,
                       false, "cs_encode_static");
  });
}

cs_status cs_forward_embeddings(const void* src, const int64_t* placeholder_index, void* dst_seq, int64_t n_rows,
                                int64_t dst_rows, int32_t hidden, int32_t dtype, int32_t* err_flag, void* stream) {
  if (n_rows < 0 || dst_rows < 0 || hidden <= 0) return fail(CS_ERR_INVALID_ARG, "cs_forward_embeddings: negative size");
  if (dtype != CS_F32 && dtype != CS_BF16) return fail(CS_ERR_INVALID_ARG, "cs_forward_embeddings: dtype");
  if (n_rows == 0) return CS_OK;
  if (!src || !placeholder_index || !dst_seq) return fail(CS_ERR_INVALID_ARG, "cs_forward_embeddings: NULL argument");
  const int64_t row_bytes = (int64_t)hidden * (dtype == CS_BF16 ? 2 : 4);
  if (row_bytes % 16) return fail(CS_ERR_UNSUPPORTED, "cs_forward_embeddings: a row must be a multiple of 16 bytes");
  if ((reinterpret_cast<uintptr_t>(src) | reinterpret_cast<uintptr_t>(dst_seq)) & 15)
    return fail(CS_ERR_INVALID_ARG, "cs_forward_embeddings: src and dst_seq must be 16-byte aligned");
  if ((reinterpret_cast<uintptr_t>(placeholder_index) & 7) || (reinterpret_cast<uintptr_t>(err_flag) & 3))
    return fail(CS_ERR_INVALID_ARG, "cs_forward_embeddings: misaligned index or flag pointer");
  return launch_scatter_rows(src, placeholder_index, dst_seq, n_rows, dst_rows, row_bytes, err_flag,
                             static_cast<hipStream_t>(stream));
}

cs_status cs_linear_bf16(const void* A, int64_t lda, const void* W, const float* bias, void* C, int32_t c_dtype,
                         int64_t M, int32_t N, int32_t K, void* stream) {
  if (!A || !W || !C) return fail(CS_ERR_INVALID_ARG, "cs_linear_bf16: NULL argument");
  if (M < 0 || M > 0x7fffffff || N < 0) return fail(CS_ERR_INVALID_ARG, "cs_linear_bf16: sizes");
  GemmArgs g = {};
  g.A = static_cast<const bf16_t*>(A); g.lda = lda; g.W = static_cast<const bf16_t*>(W); g.bias = bias;
  g.out = C; g.ldo = N; g.M = (int32_t)M; g.N = N; g.K = K;
  return launch_gemm(c_dtype == CS_BF16 ? EPI_BF16 : EPI_F32, g, static_cast<hipStream_t>(stream));
}

static cs_status attention_varlen(const void* qk, const void* vt, int64_t ld_vt, void* out, const int32_t* seg_cu,
                                  int32_t n_seg, int32_t n_heads, int32_t head_dim, void* stream_) {
  if (!qk || !vt || !out || !seg_cu || n_seg <= 0) return fail(CS_ERR_INVALID_ARG, "cs_attention_varlen: NULL argument");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  std::vector<int32_t> work;
  int max_len = 0;
  for (int s = 0; s < n_seg; ++s) {
    if (seg_cu[s] % 4 || seg_cu[s + 1] <= seg_cu[s]) return fail(CS_ERR_SHAPE, "cs_attention_varlen: segment boundaries");
    max_len = std::max(max_len, seg_cu[s + 1] - seg_cu[s]);
  }
  const int qpb = max_len <= 64 ? 64 : 256;
  for (int s = 0; s < n_seg; ++s)
    for (int q = seg_cu[s]; q < seg_cu[s + 1]; q += qpb) {
      work.push_back(q); work.push_back(std::min(q + qpb, seg_cu[s + 1])); work.push_back(seg_cu[s]); work.push_back(seg_cu[s + 1]);
    }
  // component call for tests and micro-benchmarks: the work list is uploaded synchronously
  AttnWork* dwork = nullptr;
  CS_HIP(hipMalloc(reinterpret_cast<void**>(&dwork), work.size() * 4));
  hipError_t he = hipMemcpy(dwork, work.data(), work.size() * 4, hipMemcpyHostToDevice);
  cs_status st = CS_OK;
  if (he != hipSuccess) st = fail(CS_ERR_HIP, hipGetErrorString(he));
  if (st == CS_OK) {
    AttnArgs a = {};
    a.qk = static_cast<const bf16_t*>(qk); a.vt = static_cast<const bf16_t*>(vt); a.ld_vt = ld_vt;
    a.out = static_cast<bf16_t*>(out); a.work = dwork; a.n_work = (int32_t)(work.size() / 4);
    a.n_tok = seg_cu[n_seg]; a.n_heads = n_heads; a.head_dim = head_dim; a.q_per_block = qpb; a.single_tile = max_len <= 64;
    st = launch_attention(a, stream);
    (void)hipStreamSynchronize(stream);
  }
  (void)hipFree(dwork);
  return st;
}

cs_status cs_attention_varlen(const void* qk, const void* vt, int64_t ld_vt, void* out, const int32_t* seg_cu,
                              int32_t n_seg, int32_t n_heads, int32_t head_dim, void* stream) {
  return guarded("cs_attention_varlen", [&] { return attention_varlen(qk, vt, ld_vt, out, seg_cu, n_seg, n_heads, head_dim, stream); });
}

static cs_status pack_batch(const int32_t* grid_thw, int32_t n_pending, int64_t row_budget, int32_t max_items,
                            int32_t* selected, int32_t* n_selected, int32_t* cu_seqlens, int32_t* packed_grid) {
  if (!grid_thw || !selected || !n_selected || n_pending <= 0 || max_items <= 0 || row_budget <= 0)
    return fail(CS_ERR_INVALID_ARG, "cs_pack_batch: NULL argument or non-positive count / budget");
  for (int i = 0; i < n_pending; ++i) {
    const int64_t t = grid_thw[3 * i], h = grid_thw[3 * i + 1], w = grid_thw[3 * i + 2];
    if (t <= 0 || h <= 0 || w <= 0 || t * h * w > (int64_t)1 << 28)
      return fail(CS_ERR_SHAPE, "cs_pack_batch: item " + std::to_string(i) + " has a non-positive or oversized grid");
  }
  int64_t rows = 0;
  int32_t taken = 0;
  if (cu_seqlens) cu_seqlens[0] = 0;
  for (int i = 0; i < n_pending && taken < max_items; ++i) {
    const int64_t r = (int64_t)grid_thw[3 * i] * grid_thw[3 * i + 1] * grid_thw[3 * i + 2];
    if (taken > 0 && rows + r > row_budget) continue;
    if (rows + r > (int64_t)1 << 28) return fail(CS_ERR_SHAPE, "cs_pack_batch: batch too large");
    rows += r;
    selected[taken] = i;
    if (packed_grid) for (int k = 0; k < 3; ++k) packed_grid[3 * taken + k] = grid_thw[3 * i + k];
    if (cu_seqlens) cu_seqlens[taken + 1] = (int32_t)rows;
    ++taken;
  }
  *n_selected = taken;
  return CS_OK;
}

cs_status cs_pack_batch(const int32_t* grid_thw, int32_t n_pending, int64_t row_budget, int32_t max_items,
                        int32_t* selected, int32_t* n_selected, int32_t* cu_seqlens, int32_t* packed_grid) {
  return guarded("cs_pack_batch", [&] {
    return pack_batch(grid_thw, n_pending, row_budget, max_items, selected, n_selected, cu_seqlens, packed_grid);
  });
}

static cs_status patchify(const void* frames, int32_t in_dtype, const int32_t* frame_dims, int32_t n_items,
                          int32_t temporal_patch, int32_t patch, void* patches, int32_t out_dtype, int32_t* grid_thw,
                          int32_t* cu_seqlens, void* stream_) {
  if (!frames || !frame_dims || !patches || n_items <= 0) return fail(CS_ERR_INVALID_ARG, "cs_patchify: NULL argument or no items");
  if ((in_dtype != CS_F32 && in_dtype != CS_BF16) || (out_dtype != CS_F32 && out_dtype != CS_BF16))
    return fail(CS_ERR_INVALID_ARG, "cs_patchify: dtype");
  if (temporal_patch < 1 || patch < 2 || (patch & 1)) return fail(CS_ERR_INVALID_ARG, "cs_patchify: patch sizes");
  if ((reinterpret_cast<uintptr_t>(frames) | reinterpret_cast<uintptr_t>(patches)) & 15)
    return fail(CS_ERR_INVALID_ARG, "cs_patchify: frames and patches must be 16-byte aligned");
  const int64_t in_sz = in_dtype == CS_BF16 ? 2 : 4;
  const int64_t pdim = 3 * (int64_t)temporal_patch * patch * patch;
  // validate everything before the first launch
  int64_t rows = 0;
  for (int i = 0; i < n_items; ++i) {
    const int64_t F = frame_dims[3 * i], H = frame_dims[3 * i + 1], W = frame_dims[3 * i + 2];
    if (F <= 0 || H <= 0 || W <= 0 || H % patch || W % patch || (F != 1 && F % temporal_patch))
      return fail(CS_ERR_SHAPE, "cs_patchify: item " + std::to_string(i) + ": sides must be multiples of the patch size, "
                                "frames 1 or a multiple of the temporal patch");
    if ((F * 3 * H * W * in_sz) % 16) return fail(CS_ERR_SHAPE, "cs_patchify: item " + std::to_string(i) + " does not end 16-byte aligned");
    rows += (F == 1 ? 1 : F / temporal_patch) * (H / patch) * (W / patch);
    if (rows > std::numeric_limits<int32_t>::max() / 8) return fail(CS_ERR_SHAPE, "cs_patchify: batch too large");
  }
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  int64_t src_el = 0, dst_el = 0;
  int32_t cu = 0;
  if (cu_seqlens) cu_seqlens[0] = 0;
  for (int i0 = 0; i0 < n_items; i0 += PATCHIFY_ITEMS) {
    PatchifyItems it = {};
    it.n = std::min(PATCHIFY_ITEMS, n_items - i0);
    for (int k = 0; k < it.n; ++k) {
      const int i = i0 + k;
      const int32_t F = frame_dims[3 * i], H = frame_dims[3 * i + 1], W = frame_dims[3 * i + 2];
      const int32_t T = F == 1 ? 1 : F / temporal_patch, h = H / patch, w = W / patch;
      it.F[k] = F; it.H[k] = H; it.W[k] = W;
      it.src_off[k] = src_el;
      it.dst_off[k] = dst_el;
      it.pair_cu[k + 1] = it.pair_cu[k] + (int64_t)F * 3 * H * (W / 2);
      src_el += (int64_t)F * 3 * H * W;
      dst_el += (int64_t)T * h * w * pdim;
      cu += T * h * w;
      if (grid_thw) { grid_thw[3 * i] = T; grid_thw[3 * i + 1] = h; grid_thw[3 * i + 2] = w; }
      if (cu_seqlens) cu_seqlens[i + 1] = cu;
    }
    if (cs_status st = launch_patchify(frames, in_dtype == CS_BF16, patches, out_dtype == CS_BF16, it, temporal_patch, patch, stream))
      return st;
  }
  return CS_OK;
}

cs_status cs_patchify(const void* frames, int32_t in_dtype, const int32_t* frame_dims, int32_t n_items,
                      int32_t temporal_patch, int32_t patch, void* patches, int32_t out_dtype, int32_t* grid_thw,
                      int32_t* cu_seqlens, void* stream) {
  return guarded("cs_patchify", [&] {
    return patchify(frames, in_dtype, frame_dims, n_items, temporal_patch, patch, patches, out_dtype, grid_thw, cu_seqlens, stream);
  });
}

cs_status cs_mfma_ceiling(void* scratch, size_t scratch_bytes, int32_t random_operands, int32_t iters, double* tflops,
                          void* stream_) {
  constexpr int kBlocks = 256;
  if (!scratch || !tflops || iters <= 0 || scratch_bytes < (size_t)kBlocks * 512 * 4)
    return fail(CS_ERR_INVALID_ARG, "cs_mfma_ceiling: scratch of at least 512 KiB, iters > 0");
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  CS_HIP(hipEventCreate(&e0));
  if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(e0); return fail(CS_ERR_HIP, "hipEventCreate"); }
  cs_status st = launch_mfma_loop(static_cast<float*>(scratch), kBlocks, 16, random_operands, stream);
  float ms = 0.f;
  if (st == CS_OK) {
    hipError_t he = hipEventRecord(e0, stream);
    if (he == hipSuccess) st = launch_mfma_loop(static_cast<float*>(scratch), kBlocks, iters, random_operands, stream);
    if (he == hipSuccess && st == CS_OK) he = hipEventRecord(e1, stream);
    if (he == hipSuccess && st == CS_OK) he = hipEventSynchronize(e1);
    if (he == hipSuccess && st == CS_OK) he = hipEventElapsedTime(&ms, e0, e1);
    if (he != hipSuccess) st = fail(CS_ERR_HIP, hipGetErrorString(he));
  }
  (void)hipEventDestroy(e0);
  (void)hipEventDestroy(e1);
  if (st != CS_OK) return st;
  *tflops = (double)kBlocks * 8 * iters * 32 * 32768.0 / ((double)ms * 1e-3) / 1e12;
  return CS_OK;
}

}  // extern "C"
