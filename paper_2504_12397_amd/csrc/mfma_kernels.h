// Launchers of the MFMA (bf16, gfx950) kernels.
#pragma once
#include "common.h"

namespace alora {
}  // namespace alora
