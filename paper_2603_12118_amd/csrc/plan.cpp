// Host-side batch planning.
//
// Vision batches are processed in an internal token order chosen so that every index pattern the
// encoder needs becomes a contiguous range: item, frame, attention window (row-major over the
// frame's window grid), 2x2 merge group (row-major inside the window), patch inside the group
// (row-major).  A window is then a run of consecutive tokens, an item is a run of windows, and the
// four patches that the merger concatenates are four consecutive rows, so [N, D] reinterpreted as
// [N/4, 4D] is the merger's input.  Windows tile a frame from its top-left corner; the last window
// of a row or column is smaller when the grid is not a multiple of the window.
#include "plan.h"

#include <algorithm>
#include <limits>

namespace cs {

static size_t blob_section(std::vector<int32_t>& blob, size_t words) {
  const size_t off = blob.size();
  blob.resize(off + (size_t)round_up((int64_t)words, 4), 0);
  return off;
}

static cs_status check_batch(const int32_t* cu, const int32_t* grid, int32_t n_items) {
  if (!cu || !grid) return fail(CS_ERR_INVALID_ARG, "cu_seqlens / grid_thw is NULL");
  if (n_items <= 0) return fail(CS_ERR_INVALID_ARG, "n_items must be positive");
  if (cu[0] != 0) return fail(CS_ERR_SHAPE, "cu_seqlens[0] must be 0");
  for (int i = 0; i < n_items; ++i) {
    const int64_t t = grid[3 * i], h = grid[3 * i + 1], w = grid[3 * i + 2];
    if (t <= 0 || h <= 0 || w <= 0) return fail(CS_ERR_SHAPE, "grid_thw entries must be positive");
    const int64_t n = t * h * w;
    if (n > std::numeric_limits<int32_t>::max() / 8) return fail(CS_ERR_SHAPE, "item too large");
    if ((int64_t)cu[i + 1] - cu[i] != n)
      return fail(CS_ERR_SHAPE, "cu_seqlens[" + std::to_string(i + 1) + "] - cu_seqlens[" + std::to_string(i) +
                                    "] != t*h*w of item " + std::to_string(i));
  }
  if ((int64_t)cu[n_items] > std::numeric_limits<int32_t>::max() / 8) return fail(CS_ERR_SHAPE, "batch too large");
  return CS_OK;
}

static void push_work(std::vector<int32_t>& v, int q0, int q1, int kv0, int kv1) {
  v.push_back(q0);
  v.push_back(q1);
  v.push_back(kv0);
  v.push_back(kv1);
}

// Query blocks of a full-attention segment: 256 queries per work item; a last block of at most 64 queries
// goes to the tail list (64-query work items).
static void push_full(std::vector<int32_t>& full, std::vector<int32_t>& tail, int q0, int q1, int kv0, int kv1) {
  for (int q = q0; q < q1; q += 256) {
    const int e = std::min(q + 256, q1);
    push_work(e - q <= 64 && q > q0 ? tail : full, q, e, kv0, kv1);
  }
}

cs_status build_vit_plan(const cs_encoder_config& cfg, const int32_t* cu, const int32_t* grid, int32_t n_items,
                         BatchPlan& p) {
  if (cs_status st = check_batch(cu, grid, n_items)) return st;
  const int mg = cfg.merge;
  for (int i = 0; i < n_items; ++i)
    if (grid[3 * i + 1] % mg || grid[3 * i + 2] % mg)
      return fail(CS_ERR_SHAPE, "item " + std::to_string(i) + ": h and w must be multiples of the merge size");
  const int64_t N = cu[n_items];
  p = BatchPlan();
  p.n_in = p.n_tok = N;
  p.n_out = p.n_groups = N / (mg * mg);
  std::vector<int32_t> src_row, pos, out_row, win_work, full_work, tail_work;
  src_row.reserve(N);
  pos.reserve(3 * N);
  out_row.reserve(p.n_out);
  p.win_cu.assign(1, 0);
  p.win_single_tile = true;
  int64_t out_base = 0;
  for (int i = 0; i < n_items; ++i) {
    const int T = grid[3 * i], h = grid[3 * i + 1], w = grid[3 * i + 2];
    const int win = cfg.window > 0 ? cfg.window : std::max(h, w);
    const int item_start = (int)src_row.size();
    for (int t = 0; t < T; ++t)
      for (int r0 = 0; r0 < h; r0 += win)
        for (int c0 = 0; c0 < w; c0 += win) {
          const int r1 = std::min(r0 + win, h), c1 = std::min(c0 + win, w);
          for (int R = r0; R < r1; R += mg)
            for (int C = c0; C < c1; C += mg) {
              out_row.push_back((int32_t)(out_base + ((int64_t)t * (h / mg) + R / mg) * (w / mg) + C / mg));
              for (int dr = 0; dr < mg; ++dr)
                for (int dc = 0; dc < mg; ++dc) {
                  const int r = R + dr, c = C + dc;
                  if (cfg.input_order == CS_ORDER_MERGE_MAJOR)
                    src_row.push_back(cu[i] + (((t * (h / mg) + R / mg) * (w / mg) + C / mg) * mg + dr) * mg + dc);
                  else
                    src_row.push_back(cu[i] + (t * h + r) * w + c);
                  pos.push_back(t);
                  pos.push_back(r);
                  pos.push_back(c);
                }
            }
          if (cfg.window > 0) {
            const int w0 = p.win_cu.back(), w1 = (int)src_row.size();
            p.win_cu.push_back(w1);
            if (w1 - w0 > 64) p.win_single_tile = false;
            for (int q = w0; q < w1; q += 64) push_work(win_work, q, std::min(q + 64, w1), w0, w1);
          }
        }
    const int item_end = (int)src_row.size();
    push_full(full_work, tail_work, item_start, item_end, item_start, item_end);
    out_base += (int64_t)T * (h / mg) * (w / mg);
  }
  p.off_src_row = blob_section(p.blob, src_row.size());
  std::copy(src_row.begin(), src_row.end(), p.blob.begin() + p.off_src_row);
  p.off_pos = blob_section(p.blob, pos.size());
  std::copy(pos.begin(), pos.end(), p.blob.begin() + p.off_pos);
  p.off_out_row = blob_section(p.blob, out_row.size());
  std::copy(out_row.begin(), out_row.end(), p.blob.begin() + p.off_out_row);
  p.off_win_work = blob_section(p.blob, win_work.size());
  std::copy(win_work.begin(), win_work.end(), p.blob.begin() + p.off_win_work);
  p.off_full_work = blob_section(p.blob, full_work.size());
  std::copy(full_work.begin(), full_work.end(), p.blob.begin() + p.off_full_work);
  p.off_tail_work = blob_section(p.blob, tail_work.size());
  std::copy(tail_work.begin(), tail_work.end(), p.blob.begin() + p.off_tail_work);
  p.n_win_work = (int32_t)(win_work.size() / 4);
  p.n_full_work = (int32_t)(full_work.size() / 4);
  p.n_tail_work = (int32_t)(tail_work.size() / 4);
  return CS_OK;
}

// Class-token tower: a tile of h x w patches becomes h*w + 4 internal tokens: the patches in
// merge-group order (2x2 groups row-major, row-major inside a group), then the class token, then
// three padding tokens, so that every tile starts on a multiple of four tokens and [n_tok, D] viewed
// as [n_tok/4, 4D] is the projector's input (one row per merge group, plus one row per tile made
// of the class token and the padding, which is computed and dropped).  Attention: every token of
// the tile is a query (the padding too, so that its rows stay finite), the keys are the patches and
// the class token.
cs_status build_cls_plan(const cs_encoder_config& cfg, int32_t n_positions, const int32_t* cu, const int32_t* grid,
                         int32_t n_items, BatchPlan& p) {
  if (cs_status st = check_batch(cu, grid, n_items)) return st;
  const int mg = cfg.merge;
  int64_t n_tok = 0;
  for (int i = 0; i < n_items; ++i) {
    const int64_t T = grid[3 * i], h = grid[3 * i + 1], w = grid[3 * i + 2];
    if (T != 1) return fail(CS_ERR_SHAPE, "item " + std::to_string(i) + ": tiles of a class-token tower have t == 1");
    if (h % mg || w % mg) return fail(CS_ERR_SHAPE, "item " + std::to_string(i) + ": h and w must be multiples of the merge size");
    if (1 + h * w != n_positions)
      return fail(CS_ERR_SHAPE, "item " + std::to_string(i) + ": 1 + h*w must equal the rows of the position table (" +
                                    std::to_string(n_positions) + ")");
    n_tok += h * w + 4;
  }
  if (n_tok > std::numeric_limits<int32_t>::max() / 8) return fail(CS_ERR_SHAPE, "batch too large");
  p = BatchPlan();
  p.n_in = cu[n_items];
  p.n_tok = n_tok;
  p.n_out = p.n_in / (mg * mg);
  p.n_groups = n_tok / 4;
  std::vector<int32_t> src_row, pos, out_row, full_work, tail_work;
  src_row.reserve(n_tok);
  pos.reserve(n_tok);
  out_row.reserve(p.n_groups);
  int64_t out_base = 0;
  for (int i = 0; i < n_items; ++i) {
    const int h = grid[3 * i + 1], w = grid[3 * i + 2];
    const int start = (int)src_row.size();
    for (int R = 0; R < h; R += mg)
      for (int C = 0; C < w; C += mg) {
        out_row.push_back((int32_t)(out_base + (int64_t)(R / mg) * (w / mg) + C / mg));
        for (int dr = 0; dr < mg; ++dr)
          for (int dc = 0; dc < mg; ++dc) {
            src_row.push_back(cu[i] + (R + dr) * w + C + dc);
            pos.push_back(1 + (R + dr) * w + C + dc);
          }
      }
    src_row.insert(src_row.end(), 4, -1);
    pos.push_back(-1);               // the class token
    pos.insert(pos.end(), 3, -2);    // padding
    out_row.push_back(-1);
    const int keys_end = start + h * w + 1, end = start + h * w + 4;
    push_full(full_work, tail_work, start, end, start, keys_end);
    out_base += (int64_t)(h / mg) * (w / mg);
  }
  auto put = [&](const std::vector<int32_t>& v) {
    const size_t o = blob_section(p.blob, v.size());
    std::copy(v.begin(), v.end(), p.blob.begin() + o);
    return o;
  };
  p.off_src_row = put(src_row);
  p.off_pos = put(pos);
  p.off_out_row = put(out_row);
  p.off_full_work = put(full_work);
  p.n_full_work = (int32_t)(full_work.size() / 4);
  p.off_tail_work = put(tail_work);
  p.n_tail_work = (int32_t)(tail_work.size() / 4);
  return CS_OK;
}

// Audio: item i has F_i mel frames.  The two k=3 convolutions run as GEMMs over zero-padded,
// frame-major buffers in which clip i owns F_i + 2 rows (one zero row before and after), so
// that output frame t reads three consecutive rows starting at padded row t (stride 1) or 2t
// (stride 2).  Rows of such a GEMM that straddle two clips are junk and are dropped by the row map.
cs_status build_audio_plan(const cs_encoder_config& cfg, const int32_t* cu, const int32_t* grid, int32_t n_items,
                           BatchPlan& p) {
  if (cs_status st = check_batch(cu, grid, n_items)) return st;
  for (int i = 0; i < n_items; ++i) {
    if (grid[3 * i] != 1 || grid[3 * i + 1] != 1) return fail(CS_ERR_SHAPE, "audio items are (1, 1, frames)");
    if (grid[3 * i + 2] % 8) return fail(CS_ERR_SHAPE, "audio frame counts must be multiples of 8");
    if (grid[3 * i + 2] % (2 * cfg.merge)) return fail(CS_ERR_SHAPE, "audio frame counts must be multiples of 2*pool");
  }
  p = BatchPlan();
  p.n_in = cu[n_items];
  p.n_tok = p.n_in / 2;
  p.n_out = p.n_groups = p.n_tok / cfg.merge;
  p.n_pad_rows = p.n_in + 2 * (int64_t)n_items;
  std::vector<int32_t> mel_src(p.n_pad_rows, -1), c1_map(p.n_pad_rows - 2, -1), c2_map(p.n_pad_rows / 2 - 1, -1);
  std::vector<int32_t> zero_rows, pos(p.n_tok), full_work;
  int off = 0, tok = 0;
  // short chunks: two-wave workgroups of 64 queries instead of eight waves of which most would idle
  const int qpb = cfg.attn_chunk > 0 && cfg.attn_chunk <= 128 ? 64 : 256;
  p.full_q_per_block = qpb;
  p.full_single_tile = cfg.attn_chunk > 0 && cfg.attn_chunk <= 64;
  for (int i = 0; i < n_items; ++i) {
    const int F = grid[3 * i + 2];
    zero_rows.push_back(off);
    zero_rows.push_back(off + F + 1);
    for (int t = 0; t < F; ++t) {
      mel_src[off + 1 + t] = cu[i] + t;
      c1_map[off + t] = off + 1 + t;
    }
    for (int t = 0; t < F / 2; ++t) {
      c2_map[off / 2 + t] = tok + t;
      pos[tok + t] = t;
    }
    // attention segments: the clip, or its chunks of attn_chunk tokens (the last one may be shorter)
    const int n_tok_i = F / 2, seg = cfg.attn_chunk > 0 ? cfg.attn_chunk : n_tok_i;
    for (int s0 = 0; s0 < n_tok_i; s0 += seg) {
      const int s1 = std::min(s0 + seg, n_tok_i);
      for (int q = s0; q < s1; q += qpb) push_work(full_work, tok + q, tok + std::min(q + qpb, s1), tok + s0, tok + s1);
    }
    off += F + 2;
    tok += F / 2;
  }
  auto put = [&](const std::vector<int32_t>& v) {
    const size_t o = blob_section(p.blob, v.size());
    std::copy(v.begin(), v.end(), p.blob.begin() + o);
    return o;
  };
  p.off_mel_src = put(mel_src);
  p.off_c1_map = put(c1_map);
  p.off_c2_map = put(c2_map);
  p.off_zero_rows = put(zero_rows);
  p.n_zero_rows = (int32_t)zero_rows.size();
  p.off_pos = put(pos);
  p.off_full_work = put(full_work);
  p.n_full_work = (int32_t)(full_work.size() / 4);
  return CS_OK;
}

}  // namespace cs
