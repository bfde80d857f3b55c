// Streaming stores for data nobody reads again before the next kernel (gfx950).
//
// `nt` marks the line as streaming; `sc1` widens the scope of the store so that it is written through to
// memory instead of lingering in the L2 of the XCD.  On MI355X the pair measured ~1.5% faster than `nt`
// alone on the eight-stream AdamW update (presumably because lines written back later leave the L2 in bursts that compete
// with the read front).  The compiler's nontemporal builtin sets `nt` only, hence the instruction is
// written out here.  Stores are vector stores; they complete on their own after the wave has ended.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace elixir {

// W: any 4- or 8-byte trivially copyable type held in vector registers.  (Wider stores keep reading their data
// registers after issue and need padding that the compiler only adds for stores it emits itself; the kernels
// with 128-bit stores measured no gain from `sc1` and use the builtin.)
template <typename W>
__device__ __forceinline__ void stream_store(W v, W* p) {
    static_assert(sizeof(W) == 4 || sizeof(W) == 8, "unsupported width");
    if constexpr (sizeof(W) == 8) asm volatile("global_store_dwordx2 %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
    else asm volatile("global_store_dword %0, %1, off sc1 nt" ::"v"(p), "v"(v) : "memory");
}

}  // namespace elixir
