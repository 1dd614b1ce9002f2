// Internal launch interface between the C ABI (api.hip) and the kernel files.
#pragma once

#include "common.hpp"

namespace maskkv {

// score.hip
size_t score_workspace_bytes(const maskkv_desc* d, const Lens& lens);
int launch_score(const maskkv_desc* d, const View& Q, const View& K, const Lens& lens, float scale, float* scores,
                 int64_t score_stride, float* prompt_mass, void* workspace, hipStream_t stream,
                 void* const* events, const float* row_lse = nullptr);

// select.hip
size_t select_workspace_bytes(const maskkv_desc* d);
int64_t select_max_prompt();
int launch_select(const maskkv_desc* d, const Lens& lens, const float* scores, int64_t score_stride, int window,
                  int mode, const int32_t* budgets, int32_t* idx, int32_t* cu_budget, int64_t capacity,
                  void* workspace, hipStream_t stream);
int launch_head_budgets(const maskkv_desc* d, const float* prompt_mass, int32_t k_l, float alpha, int32_t* budgets,
                        hipStream_t stream);

// compact.hip
int launch_compact(const maskkv_desc* d, const Lens& lens, const View& K, const View& V, const int32_t* idx, const int32_t* cu_budget,
                   int64_t capacity, void* Kc, void* Vc, hipStream_t stream);

// attend.hip
size_t attend_workspace_bytes(const maskkv_desc* d, bool full);
int launch_attend(const maskkv_desc* d, const Lens& lens, bool full, const View& Q, const void* Kc, const void* Vc,
                  const int32_t* cu_budget, int64_t capacity, const View& K2, const View& V2, float scale,
                  const View& O, float* lse, void* workspace, hipStream_t stream);

// layer.hip
size_t layer_importance_workspace_bytes();
int launch_layer_importance(const void* h_in, const void* h_out, int64_t n, int hidden, int dtype, int64_t row_bytes,
                            float* importance, void* workspace, hipStream_t stream);
int launch_value_shift(const void* v_now, const void* v_prev, int64_t n, int width, int dtype, int64_t row_bytes,
                       float delta, float* cos, int32_t* refresh, int32_t* count, hipStream_t stream);

// api.hip: the body of maskkv_score.  events: null, or four hipEvent_t (each may be null) recorded on the stream
// before pass 1, before the merge, before pass 2 and after pass 2; measurement harnesses link against this to time
// the stages of one call (the C entry point always passes null).
int score_entry(const maskkv_desc* desc, const maskkv_tensor* Q_mask, const maskkv_tensor* K_full, float scale,
                float* scores, int64_t score_stride, float* prompt_mass, void* workspace, size_t workspace_bytes,
                void* stream, void* const* events);

}  // namespace maskkv
