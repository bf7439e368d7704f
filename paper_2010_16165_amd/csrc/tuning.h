// Internal: the process-wide tuning switches behind fupr_tuning_set.  A switch
// selects among kernel instantiations (or schedules) that all compute the same
// operator; none changes what is computed.  Launchers read them through these
// two calls, never through the environment.
#pragma once
#include <cstddef>

namespace fupr {

// The switch's value parsed as an integer; `unset` when it has no value.
int tuning_int(const char* name, int unset);
// The switch's value copied into out (n bytes, always terminated); false when unset.
bool tuning_text(const char* name, char* out, size_t n);
// True when the switch is set to a value that starts with '0'.
bool tuning_off(const char* name);

}  // namespace fupr
