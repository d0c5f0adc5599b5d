// Tuning overrides (DWCONV_TUNE_* environment variables) as an immutable snapshot.
//
// The dispatcher never reads the environment on a call.  The variables are copied once, when the
// library is first used, and only if the master switch DWCONV_TUNE=1 is set at that moment;
// without it the snapshot is empty and every lookup returns "unset" after one comparison.  A
// workspace query and the launch that follows it therefore always see the same values.  Tuning
// sweeps and the forced-tiling tests change the environment and then call dwconv_tuning_reload()
// (declared in include/dwconv.h), which takes a new snapshot; that call must not overlap any other
// call into the library.
#pragma once

namespace dwc {

// Value of the snapshot's variable `name` (full name, e.g. "DWCONV_TUNE_TH"), or nullptr if it
// was unset, empty, or the master switch was off.  The pointer stays valid until the next reload.
const char *tune_env(const char *name);

// Whether the snapshot holds any variable at all.
bool tune_active();

// Takes a new snapshot of the environment; returns the number of variables it holds.
int tune_reload();

}  // namespace dwc
