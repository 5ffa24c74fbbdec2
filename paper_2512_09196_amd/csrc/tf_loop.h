// Internal: the loop driver shared by tf_tune (profiles on the GPU) and tf_tune_replay
// (reads pre-made reports).
#pragma once
#include "tf.h"

namespace tf {
// Profile callback: BuildRun + parity gate + Profile of variant `id` into *out.
typedef tf_status (*profile_fn)(void* user, int32_t id, tf_report* out);

tf_status run_loop(const tf_problem_desc* prob, const tf_hw* hw, const tf_variant_desc* family, int32_t n,
                   const tf_theta* theta, profile_fn profile, void* user, int32_t* best_variant, tf_report* best,
                   tf_report* round_log, int32_t log_cap, int32_t* n_log);
}  // namespace tf
