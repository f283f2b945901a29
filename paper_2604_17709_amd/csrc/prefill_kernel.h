// Compute-bound ("prefill", T > 128 tokens) kernels for PACKED bf16 factor pairs.
#pragma once
#include "common.h"

namespace deinfer {
}  // namespace deinfer
