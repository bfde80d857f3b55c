"""Chunked mixed-precision AdamW step of Elixir (arXiv 2212.05339) for AMD MI355X.

The product is libelixir_chunk.so (HIP kernels behind a C ABI, see include/elixir_chunk.h);
this package is its thin Python binding.
"""
from .binding import *  # noqa: F401,F403
from .binding import EXPORTS, LIB_PATH, Ctx, ElixirError, elixir_adam_hparams, elixir_arena_array, elixir_hw_profile, lib, make_hparams  # noqa: F401
