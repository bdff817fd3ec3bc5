// Tuning overrides: environment variables that force a kernel variant the planner would not pick by
// itself.  They exist for tests (every variant is parity-tested through its override) and for
// measurements; they are not part of the ABI contract.  The environment is read ONCE, at the first
// library call of the process, so a call costs no getenv; brg_tuning_reload() reads it again.
#pragma once

namespace brg {

struct Knob {
    bool set = false;
    int val = 0;
    bool on() const { return set && val != 0; }   // present and not "0"
};

struct Knobs {
    // name in the environment = BRG_ + the upper-case field name
    Knob conv_general, conv_pitch, conv_plane_pad, conv_kw, conv_no1x1, conv_zerofill, conv_nofuse;
    Knob conv_1x1_kw, conv_1x1_pg, conv_1x1_lds, conv_1x1_lds_ngw, conv_1x1_lds_pm, conv_1x1_split, conv_1x1_wf;
    Knob conv_small, conv_small_kw, conv_small_pg, conv_small_gz;
    Knob conv_stem_classes, conv_stem_gx;
    Knob conv_wgt_general, conv_wgt_ps, conv_wgt_target;
    Knob fc_general, fc_g64, fc_g128, fc_wgt_general;
    Knob gemm_general, no_ring, lstm_general, lstm_spin_limit;
    // presence alone switches these (any value, as before the table existed)
    bool flag(const Knob &k) const { return k.set; }
};

const Knobs &knobs();   // brg_host.cpp

}  // namespace brg
