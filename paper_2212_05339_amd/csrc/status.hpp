// Error reporting shared by every translation unit (no HIP types here: host-only files include just this).
#pragma once
#include <exception>

#include "../../include/elixir_chunk.h"

namespace elixir {

// Stores the per-thread message returned by elixir_last_error() and hands back `code`.
int fail(int code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// Runs body() and turns a C++ exception (in practice std::bad_alloc from a host-side table) into a status: nothing
// throws across the C boundary.
template <typename F>
int no_throw(const char* what, F&& body) noexcept {
    try {
        return body();
    } catch (const std::exception& e) {
        return fail(ELIXIR_EINVAL, "%s: %s", what, e.what());
    } catch (...) {
        return fail(ELIXIR_EINVAL, "%s: C++ exception", what);
    }
}

}  // namespace elixir
