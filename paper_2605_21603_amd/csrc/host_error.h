// Thread-local error text shared by the host-side sources of the library.
#pragma once
#include "../../include/dynlayer.h"

namespace dyn {

// Stores the formatted text for dyn_last_error() on this thread and returns `st`.
dyn_status fail(dyn_status st, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

}  // namespace dyn
