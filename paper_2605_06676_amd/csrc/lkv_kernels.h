// Host-side launch interface of the kernels (internal to the library).
#pragma once

#include "lkv_common.h"

namespace lkv {

// score_linear.hip
void launch_score_linear(const SeqTable& tab, const uint16_t* w1, const float* b1, int heads_per_scorer_row,
                         hipStream_t stream);
int score_linear_blocks_per_head(int T);

// score_mlp.hip
hipError_t score_mlp_prepare();
void launch_score_mlp(const SeqTable& tab, const uint16_t* w1, const float* b1, const float* w2,
                      const float* b2, int hidden, int act, int heads_per_scorer_row, int rows_per_block,
                      hipStream_t stream, uint32_t* counts = nullptr, int seg_base = 0, int seg_stride = 0);
int score_mlp_rows_per_block(int T, int heads, int hidden);

// score_window.hip
int score_window_max_rows();
int score_window_rows_per_block(int64_t tokens_times_heads);
size_t score_window_pairs_bytes(int64_t heads, int T);
void launch_score_window(const WinTable& tab, int heads, int window, int group, int pool_width, int pool_kind,
                         int rows_per_block, float scale, hipStream_t stream);

// select.hip
hipError_t select_prepare();
int select_inline_capacity();
void launch_select(const SeqTable& tab, const int32_t* host_offsets, int n_total_segments, int32_t* offsets,
                   int32_t* idx, int seg_base, int seg_stride, hipStream_t stream,
                   const float* ragged_scores = nullptr, const int32_t* ragged_start = nullptr,
                   const int32_t* ragged_len = nullptr, uint32_t* counts = nullptr, uint32_t* pre_maps = nullptr,
                   int pre_words = 0);
int select_max_bitmap_tokens();

// counts.hip
void launch_clear_counts(uint32_t* counts, int64_t n_segments, hipStream_t stream);
void launch_count_level0(const SeqTable& tab, uint32_t* counts, int seg_base, int seg_stride, hipStream_t stream);
int count_level0_blocks_per_head(int T);

// compact.hip
void launch_compact(const SeqTable& tab, const int32_t* idx, const int32_t* offsets, int n_segments,
                    int heads_per_seq, int seq_lo, int head_lo, int n_heads_view, int64_t row_lo, int64_t row_hi,
                    void* kp, void* vp, hipStream_t stream, bool rows_of_own_sequences = false);

void launch_compact_grow(const SeqTable& tab, const int32_t* idx, const int32_t* offsets, int n_segments,
                         int heads_per_seq, int seq_lo, int64_t total_kept, int slack, void* kp, void* vp, float* up,
                         hipStream_t stream, bool rows_of_own_sequences = false);
void launch_compact_regrow(const int32_t* idx, const int32_t* offsets, int n_segments, int64_t total_kept, int slack,
                           const void* kp_old, const void* vp_old, const float* up_old, const int32_t* cap_old,
                           const int32_t* len_old, void* kp, void* vp, float* up, hipStream_t stream);
void launch_grown_layout(const int32_t* offsets, int n_segments, int slack, int32_t* cap, int32_t* len,
                         hipStream_t stream);

// append.hip
void launch_append(int n_segments, int heads_per_seq, int n_kv_heads, int scorer_kind, int act, int hidden,
                   int per_head, const uint16_t* w1, const float* b1, const float* w2, const float* b2,
                   const void* k_new, const void* v_new, void* kp, void* vp, float* up, const int32_t* cap,
                   int32_t* len, int32_t* overflow, hipStream_t stream);

// decode.hip
constexpr int kDecodeMaxGroup = 16;
hipError_t decode_prepare(int device);
size_t decode_workspace_bytes(int n_segments, int64_t total_kept, int G);
size_t decode_static_scratch_bytes();
void* decode_static_scratch(int device);
hipError_t launch_decode(int G, const void* q, const void* kp, const void* vp, const int32_t* offsets,
                         const int32_t* lengths, int n_segments, int64_t total_kept, float scale, float* out, float* lse, float* ws,
                         hipStream_t stream, const float* mask = nullptr);
void launch_uniform_offsets(int n_segments, int len, int32_t* offsets, hipStream_t stream);

// masked_attn.hip
hipError_t masked_attn_prepare();
void launch_masked_attn_fwd(const void* q, const void* k, const void* v, const float* m, int n_q_heads, int n_kv_heads,
                            int T, float scale, float* o, float* lse, hipStream_t stream);

// masked_attn_bwd.hip
hipError_t masked_attn_bwd_prepare();
size_t masked_attn_bwd_workspace_bytes(int n_q_heads, int n_kv_heads, int T);
void launch_masked_attn_bwd(const void* q, const void* k, const void* v, const float* m, const float* o,
                            const float* lse, const void* d_o, int n_q_heads, int n_kv_heads, int T, float scale,
                            float* dq, float* dk, float* dv, float* dm, float* workspace, hipStream_t stream);

// lkv_h.hip
hipError_t lkv_h_prepare();
int soft_topk_max_n(bool is_f64);
int head_scores_max_hidden();
void launch_soft_topk(const void* x, bool is_f64, int n, double k, double tau, double* y, double* info,
                      int32_t* budgets, double t, hipStream_t stream, int n_vec = 1, const double* k_vec = nullptr);
void launch_soft_topk_backward(const void* x, bool is_f64, int n, double tau, const double* info, const double* g,
                               double* dx, double* dk, hipStream_t stream, int n_vec = 1);
void launch_head_scores(const float* emb, const float* w1, const float* b1, const float* w2, const float* b2,
                        int n_heads, int d_e, int hidden, double* s, hipStream_t stream);

}  // namespace lkv
