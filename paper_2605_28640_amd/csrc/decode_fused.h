// Arguments of the persistent fused decode kernel (see decode_fused.hip).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace rs {

struct FusedParams {
    const void *q, *meta, *k_cache, *v_cache;
    void *out;
    float *lse_out;
    int32_t *idx_out;       // optional plain copy of the selection
    uint64_t *scores;       // [units][Np] tagged
    uint64_t *idx_tagged;   // [units][K] tagged
    uint64_t *partial;      // [units][S_att][D + 2] tagged
    uint32_t *ctr_score, *ctr_att, *ticket, *done, *err;
    int Hq, Hkv, units;
    long Tcap, Np_cap, T_valid;
    int P, Np, K, n_first, n_local;
    int S_score, S_att;
    int units_fine, S_att_fine;  // the last units_fine units (in ticket order) use S_att_fine slices
    int S_max;                   // slices the partial buffer holds per unit
    int reverse;            // walk the units from the last to the first
    int nt_kv;              // stream K/V pages with non-temporal loads
    float scale;
    uint32_t tag;
    int spin_limit;
    uint64_t *trace;  // builds with -DRS_FUSED_TRACE only: timeline [workgroup][64] of (time << 24 | item << 4 | phase); else NULL
    // replayable step: T_valid, Np and tag are read from the workspace's state words (T_valid =
    // tokens in the cache + 1: the step's append has run) and the last workgroup out advances them
    uint32_t *state;  // control words of the workspace, or NULL: T_valid, Np, tag above are used
    long T_max;       // replayable step: largest T_valid the buffers were sized for
};

// np_lds: page keys the dynamic LDS must hold (Np, or its largest value over the replays)
int decode_fused_dispatch(int dtype, int D, const FusedParams &prm, int np_lds, int grid, hipStream_t stream);

}  // namespace rs
