// Launch-shape overrides for sweeps.  Inactive unless the environment variable SIRLLM_TUNE is
// set to a non-empty value when the library makes its first launch; then get() returns the
// integer value of the named environment variable if it is set, else the default.  Read at
// every launch, so a sweep can change a knob between calls of one process.
#pragma once

namespace sirllm {
namespace tuning {
int get(const char* name, int dflt);
}
}  // namespace sirllm
