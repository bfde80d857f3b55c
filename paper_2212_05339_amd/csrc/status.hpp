// Error reporting shared by every translation unit (no HIP types here: host-only files include just this).
#pragma once
#include "../../include/elixir_chunk.h"

namespace elixir {

// Stores the per-thread message returned by elixir_last_error() and hands back `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace elixir
