// Fused INT8 attention backward (paper Algorithm 2) for gfx950.
#pragma once
#include "common.h"
namespace sage {
}  // namespace sage
