// Snapshot of the DWCONV_TUNE_* environment variables (see tune.hpp).
#include "tune.hpp"
#include <mutex>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

extern char **environ;

namespace dwc {

namespace {

constexpr int MAX_KNOBS = 96, NAME_LEN = 48, VALUE_LEN = 12;
struct Knob { char name[NAME_LEN]; char value[VALUE_LEN]; };
Knob g_knobs[MAX_KNOBS];
int g_count = 0;
std::once_flag g_once;

int snapshot()
{
    static const char prefix[] = "DWCONV_TUNE_";
    int n = 0;
    const char *master = getenv("DWCONV_TUNE");
    if (master && atoi(master) == 1 && environ) {
        for (char **e = environ; *e && n < MAX_KNOBS; ++e) {
            if (strncmp(*e, prefix, sizeof prefix - 1) != 0) continue;
            const char *eq = strchr(*e, '=');
            if (!eq || eq[1] == 0) continue;
            const size_t len = (size_t)(eq - *e);
            if (len >= NAME_LEN) continue;
            memcpy(g_knobs[n].name, *e, len);
            g_knobs[n].name[len] = 0;
            // values are small non-negative integers (tile sizes, counts, switches): anything else is
            // clamped into 0..65536 so that no consumer sees a negative or overflowing number
            long v = strtol(eq + 1, nullptr, 10);
            if (v < 0) v = 0;
            if (v > 65536) v = 65536;
            snprintf(g_knobs[n].value, VALUE_LEN, "%ld", v);
            ++n;
        }
    }
    g_count = n;
    return n;
}

}  // namespace

const char *tune_env(const char *name)
{
    std::call_once(g_once, [] { snapshot(); });
    for (int i = 0; i < g_count; ++i)
        if (strcmp(g_knobs[i].name, name) == 0) return g_knobs[i].value;
    return nullptr;
}

bool tune_active()
{
    std::call_once(g_once, [] { snapshot(); });
    return g_count > 0;
}

int tune_reload()
{
    std::call_once(g_once, [] {});
    return snapshot();
}

}  // namespace dwc
