// The table of behaviour switches: names, environment presets, run-time changes.
#include "tune.h"

#include <cctype>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <string>

namespace edl {

namespace {

struct Entry {
    const char* name;
    int64_t Tune::*field;
};

const Entry kEntries[] = {
    {"min128", &Tune::min128},
    {"min128_long", &Tune::min128_long},
    {"force_tile", &Tune::force_tile},
    {"bk64_kred", &Tune::bk64_kred},
    {"xcd", &Tune::xcd},
    {"order", &Tune::order},
    {"splitk_tiles", &Tune::splitk_tiles},
    {"splitk_target", &Tune::splitk_target},
    {"fused_stats", &Tune::fused_stats},
    {"held_stats", &Tune::held_stats},
    {"fused_mask", &Tune::fused_mask},
    {"fused_mask_cut", &Tune::fused_mask_cut},
    {"fused_mask_join", &Tune::fused_mask_join},
    {"join_tile", &Tune::join_tile},
    {"small_tail_from", &Tune::small_tail_from},
    {"small_tail_to", &Tune::small_tail_to},
    {"wgrad_blocks", &Tune::wgrad_blocks},
    {"wgrad_long_blocks", &Tune::wgrad_long_blocks},
    {"wgrad_long_ks", &Tune::wgrad_long_ks},
    {"wgrad_deep_max", &Tune::wgrad_deep_max},
    {"wgrad_stream", &Tune::wgrad_stream},
    {"wgrad_tail_main", &Tune::wgrad_tail_main},
    {"early_update", &Tune::early_update},
    {"early_blocks", &Tune::early_blocks},
    {"upd_vpt", &Tune::upd_vpt},
    {"upd_wide", &Tune::upd_wide},
    {"upd_nt", &Tune::upd_nt},
    {"upd_blocks", &Tune::upd_blocks},
    {"branch_stream", &Tune::branch_stream},
    {"transpose_stream", &Tune::transpose_stream},
    {"alias_shortcut", &Tune::alias_shortcut},
    {"bn_nt", &Tune::bn_nt},
    {"bn_nt_bytes", &Tune::bn_nt_bytes},
    {"spare0", &Tune::spare0},
    {"spare1", &Tune::spare1},
};

Tune g_tune;
std::once_flag g_once;

void load_env() {
    for (const Entry& e : kEntries) {
        std::string var = "EDL_TUNE_";
        for (const char* c = e.name; *c; ++c) var.push_back((char)toupper((unsigned char)*c));
        if (const char* v = getenv(var.c_str())) g_tune.*(e.field) = atoll(v);
    }
}

}  // namespace

Tune& tune() {
    std::call_once(g_once, load_env);
    return g_tune;
}

bool tune_set(const char* name, int64_t value) {
    if (!name) return false;
    Tune& t = tune();
    for (const Entry& e : kEntries)
        if (strcmp(e.name, name) == 0) {
            t.*(e.field) = value;
            return true;
        }
    return false;
}

bool tune_get(const char* name, int64_t* value) {
    if (!name || !value) return false;
    Tune& t = tune();
    for (const Entry& e : kEntries)
        if (strcmp(e.name, name) == 0) {
            *value = t.*(e.field);
            return true;
        }
    return false;
}

}  // namespace edl
