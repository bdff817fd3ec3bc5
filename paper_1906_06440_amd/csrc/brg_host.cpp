// Host-only pieces of the C ABI: error text, version, tuning overrides.
#include <cstdlib>
#include <mutex>

#include "brg_common.hpp"
#include "brg_knobs.hpp"

namespace brg {
char *last_error_buf()
{
    static thread_local char buf[512] = {0};
    return buf;
}

static Knobs g_knobs;
static std::once_flag g_knobs_once;

static void read_knob(Knob &k, const char *name)
{
    const char *e = getenv(name);
    k.set = e != nullptr;
    k.val = e ? atoi(e) : 0;
}

static void load_knobs()
{
    Knobs &k = g_knobs;
#define BRG_KNOB(field, name) read_knob(k.field, name)
    BRG_KNOB(conv_general, "BRG_CONV_GENERAL");
    BRG_KNOB(conv_pitch, "BRG_CONV_PITCH");
    BRG_KNOB(conv_plane_pad, "BRG_CONV_PLANE_PAD");
    BRG_KNOB(conv_kw, "BRG_CONV_KW");
    BRG_KNOB(conv_no1x1, "BRG_CONV_NO1X1");
    BRG_KNOB(conv_zerofill, "BRG_CONV_ZEROFILL");
    BRG_KNOB(conv_nofuse, "BRG_CONV_NOFUSE");
    BRG_KNOB(conv_1x1_kw, "BRG_CONV_1X1_KW");
    BRG_KNOB(conv_1x1_pg, "BRG_CONV_1X1_PG");
    BRG_KNOB(conv_1x1_lds, "BRG_CONV_1X1_LDS");
    BRG_KNOB(conv_1x1_lds_ngw, "BRG_CONV_1X1_LDS_NGW");
    BRG_KNOB(conv_1x1_lds_pm, "BRG_CONV_1X1_LDS_PM");
    BRG_KNOB(conv_1x1_split, "BRG_CONV_1X1_SPLIT");
    BRG_KNOB(conv_1x1_wf, "BRG_CONV_1X1_WF");
    BRG_KNOB(conv_small, "BRG_CONV_SMALL");
    BRG_KNOB(conv_small_kw, "BRG_CONV_SMALL_KW");
    BRG_KNOB(conv_small_pg, "BRG_CONV_SMALL_PG");
    BRG_KNOB(conv_small_gz, "BRG_CONV_SMALL_GZ");
    BRG_KNOB(conv_stem_classes, "BRG_CONV_STEM_CLASSES");
    BRG_KNOB(conv_stem_gx, "BRG_CONV_STEM_GX");
    BRG_KNOB(conv_wgt_general, "BRG_CONV_WGT_GENERAL");
    BRG_KNOB(conv_wgt_ps, "BRG_CONV_WGT_PS");
    BRG_KNOB(conv_wgt_target, "BRG_CONV_WGT_TARGET");
    BRG_KNOB(fc_general, "BRG_FC_GENERAL");
    BRG_KNOB(fc_g64, "BRG_FC_G64");
    BRG_KNOB(fc_g128, "BRG_FC_G128");
    BRG_KNOB(fc_wgt_general, "BRG_FC_WGT_GENERAL");
    BRG_KNOB(gemm_general, "BRG_GEMM_GENERAL");
    BRG_KNOB(no_ring, "BRG_NO_RING");
    BRG_KNOB(lstm_general, "BRG_LSTM_GENERAL");
    BRG_KNOB(lstm_spin_limit, "BRG_LSTM_SPIN_LIMIT");
#undef BRG_KNOB
}

const Knobs &knobs()
{
    std::call_once(g_knobs_once, load_knobs);
    return g_knobs;
}
}  // namespace brg

extern "C" const char *brg_last_error(void) { return brg::last_error_buf(); }

extern "C" const char *brg_version(void) { return "brg 0.2 (gfx950)"; }

extern "C" void brg_tuning_reload(void)
{
    (void)brg::knobs();
    brg::load_knobs();
}
