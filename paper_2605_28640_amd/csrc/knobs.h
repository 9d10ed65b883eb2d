// Tuning knobs: RATSPARSE_* environment variables, read ONCE per process (on the first call
// that needs one) into a table, so that no entry point touches the environment on its
// dispatch path.  The table is filled under std::call_once and is read-only afterwards:
// concurrent calls from several host threads see the same values.  A test that changes
// the environment afterwards asks for a re-read through ratsparse_debug_reload_knobs()
// (not thread-safe against calls in flight: a test hook, like the spin-limit one).
#pragma once

namespace rs {

constexpr int kKnobUnset = -2147483647 - 1;

struct Knobs {
    // decode (api.hip)
    int score_wgs, attend_wgs;
    int fused_grid, fused_sscore, fused_satt, fused_fine, fused_fine_pct, fused_nt, fused_pingpong;
    int fused_two_launch, fused_one_wg;
    // scan
    int scan_grid, scan_slab, scan_meta;
    // page metadata
    int meta_spw;
    // MoBA gate
    int gate_waves, gate_wgs, gate_shared;
    // prefill attention
    int prefill_masked, prefill_grid;
    // SnapKV
    int snap_one_wg;
};

// the table (filled on first use); a field holds kKnobUnset when its variable is not set
const Knobs &knobs();
// value of a field, or dflt when unset
inline int knob_or(int field, int dflt) { return field == kKnobUnset ? dflt : field; }
// test hook: read the environment again
void knobs_reload();

}  // namespace rs
