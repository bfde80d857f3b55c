// Offloading benefit model and the placement rule built on it (host only, double precision).
//
// Paper Sec. 5.1: starting from one rCache block and every chunk in CPU memory, spare GPU memory can either
// hold one more rCache block, which saves the offloading traffic of one chunk in the backward pass
// (normalised benefit I(n), Eq. 1), or hold one more chunk together with its optimizer update, which saves
// that chunk's offloading traffic and replaces its CPU update by a GPU update (J(n), Eq. 2).  Whichever is
// larger gets the memory first; what is left goes to the other.
//   I(n) = 1/L_c * ( L_c*C/B_g2c(n) + L_c*C/B_c2g(n) )
//   J(n) = n/(L_c + L_os*F_os) * [ ( L_os*C/B_c2g(n) + L_c*I(n) + L_c*C/B_g2c(n) ) + ( C/V_c(n) - C/V_g(n) ) ]
// B in bytes per second, V in elements per second (both aggregate over the n processes), C in elements.
#include "status.hpp"

using namespace elixir;

extern "C" int elixir_offload_benefit(int n_procs, int64_t chunk_elems, int L_c, int L_os, int F_os,
                                      const elixir_hw_profile* hw, double* I_out, double* J_out) {
    static const char* what = "elixir_offload_benefit";
    if (!hw || !I_out || !J_out) return fail(ELIXIR_EINVAL, "%s: NULL argument", what);
    if (n_procs < 1 || chunk_elems < 1 || L_c < 1 || L_os < 1 || F_os < 1)
        return fail(ELIXIR_EINVAL, "%s: n_procs, chunk_elems and the precision lengths must be positive", what);
    if (!(hw->b_g2c > 0) || !(hw->b_c2g > 0) || !(hw->v_g > 0) || !(hw->v_c > 0))
        return fail(ELIXIR_EINVAL, "%s: bandwidths and velocities must be positive", what);
    const double C = (double)chunk_elems, lc = L_c, los = L_os, fos = F_os;
    const double I = (lc * C / hw->b_g2c + lc * C / hw->b_c2g) / lc;
    const double J = (double)n_procs / (lc + los * fos) *
                     ((los * C / hw->b_c2g + lc * I + lc * C / hw->b_g2c) + (C / hw->v_c - C / hw->v_g));
    *I_out = I;
    *J_out = J;
    return ELIXIR_OK;
}

extern "C" int elixir_offload_plan(int n_procs, int64_t chunk_elems, int64_t n_chunks, int64_t min_blocks, int L_c,
                                   int L_os, int F_os, const elixir_hw_profile* hw, double allowed_bytes,
                                   int64_t* n_blocks_out, int64_t* n_gpu_chunks_out) {
    static const char* what = "elixir_offload_plan";
    if (!n_blocks_out || !n_gpu_chunks_out) return fail(ELIXIR_EINVAL, "%s: NULL output", what);
    if (n_chunks < 0 || min_blocks < 1) return fail(ELIXIR_EINVAL, "%s: n_chunks must be >= 0 and min_blocks >= 1", what);
    double I, J;
    if (const int rc = elixir_offload_benefit(n_procs, chunk_elems, L_c, L_os, F_os, hw, &I, &J)) return rc;
    const double block_bytes = (double)L_c * (double)chunk_elems;                                  // one rCache block, per GPU
    const double chunk_bytes = ((double)L_c + (double)L_os * F_os) * (double)chunk_elems / n_procs;  // one uploaded chunk pair, per GPU
    int64_t blocks = min_blocks < n_chunks || n_chunks == 0 ? min_blocks : n_chunks;
    if (blocks < 1) blocks = 1;
    double left = allowed_bytes - (double)blocks * block_bytes;
    int64_t up = 0;
    if (left < 0) {  // not even the mandatory blocks fit: keep them, everything else stays in CPU memory
        *n_blocks_out = blocks;
        *n_gpu_chunks_out = 0;
        return ELIXIR_OK;
    }
    auto take = [&](double unit, int64_t room) -> int64_t {
        if (room <= 0) return 0;
        int64_t k = (int64_t)(left / unit);
        if (k > room) k = room;
        left -= (double)k * unit;
        return k;
    };
    if (J > I) {
        up = take(chunk_bytes, n_chunks);
        blocks += take(block_bytes, n_chunks - blocks);
    } else {
        blocks += take(block_bytes, n_chunks - blocks);
        up = take(chunk_bytes, n_chunks);
    }
    *n_blocks_out = blocks;
    *n_gpu_chunks_out = up;
    return ELIXIR_OK;
}
