// Host-side batch planning: validation of a packed batch and the index tables the kernels read.
#pragma once
#include <vector>

#include "common.h"

namespace cs {

// Index tables of one batch, packed into one int32 blob that is uploaded with a single copy.
// Offsets are in int32 words, each a multiple of 4 (16-byte aligned sections).
struct BatchPlan {
  int64_t n_in = 0;    // input rows (patches or mel frames)
  int64_t n_tok = 0;   // transformer tokens
  int64_t n_out = 0;   // embedding rows written
  int64_t n_groups = 0; // rows of the merger's GEMMs (class-token towers: n_out plus one dropped row per tile)
  std::vector<int32_t> blob;
  // vit
  size_t off_src_row = 0;   // [n_tok]   raster patch row of internal token i
  size_t off_pos = 0;       // [n_tok*3] (t,row,col) of internal token i      (audio: [n_tok] frame position)
  size_t off_out_row = 0;   // [n_out]   output row of internal merged token j
  size_t off_win_work = 0;  // [n_win_work*4] AttnWork, one window (or 64-query slice of it) each
  size_t off_full_work = 0; // [n_full_work*4] AttnWork, 256-query blocks of whole items
  size_t off_tail_work = 0; // [n_tail_work*4] AttnWork of the full layers: last query blocks of at most 64 queries,
                            // run by two-wave workgroups in a launch of their own (a 256-query workgroup for four
                            // queries would still walk every key tile and cost the launch a round of the chip)
  int32_t n_win_work = 0, n_full_work = 0, n_tail_work = 0;
  bool win_single_tile = false;  // no window has more than 64 tokens
  int32_t full_q_per_block = 256;   // queries per item of full_work: 256, or 64 when the segments are short chunks
  bool full_single_tile = false;    // no full_work item has more than 64 keys
  std::vector<int32_t> win_cu;  // host only: window boundaries in internal token order
  // audio
  int64_t n_pad_rows = 0;   // sum(frames_i + 2): rows of the zero-padded frame buffers
  size_t off_mel_src = 0;   // [n_pad_rows] mel frame feeding padded row r, -1 for padding
  size_t off_c1_map = 0;    // [n_pad_rows-2]  conv1 virtual row -> padded row of its output, -1 junk
  size_t off_c2_map = 0;    // [n_pad_rows/2-1] conv2 virtual row -> token, -1 junk
  size_t off_zero_rows = 0; // [2*n_items] padded rows that must be zero
  int32_t n_zero_rows = 0;
};

cs_status build_vit_plan(const cs_encoder_config& cfg, const int32_t* cu_seqlens, const int32_t* grid_thw,
                         int32_t n_items, BatchPlan& plan);
// Class-token tower: `n_positions` = rows of its position table (1 + patches per tile).
cs_status build_cls_plan(const cs_encoder_config& cfg, int32_t n_positions, const int32_t* cu_seqlens,
                         const int32_t* grid_thw, int32_t n_items, BatchPlan& plan);
cs_status build_audio_plan(const cs_encoder_config& cfg, const int32_t* cu_seqlens, const int32_t* grid_thw,
                           int32_t n_items, BatchPlan& plan);

}  // namespace cs
