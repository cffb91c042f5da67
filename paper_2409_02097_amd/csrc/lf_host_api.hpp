// Small host-side helpers that linfusion.hip shares with the library's other translation units.
#pragma once

namespace lfh {

// LINFUSION_OK when the current device is a gfx950, else LINFUSION_ERR_DEVICE (cached per device)
int check_device();
// positive integer from the environment, `dflt` when unset or not positive (tuning aids)
int env_int(const char* name, int dflt);

}  // namespace lfh
