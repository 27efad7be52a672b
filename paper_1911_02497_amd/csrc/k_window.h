// Sampled-window selection: one sweep over the weights per call instead of one per radix level.
#pragma once
#include "host.h"
namespace condensa {
constexpr int kSampleUnit = 32;        // consecutive elements read per sample position
template <bool LC, bool VEC>
static condensa_status launch_window_path(const DataArgs&, const Layout&, void*, hipStream_t) { return CONDENSA_OK; }
}  // namespace condensa
