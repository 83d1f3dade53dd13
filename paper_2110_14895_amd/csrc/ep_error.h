// Thread-local error text shared by the library's translation units.
#pragma once
#include "edgepipe.h"

// Records a formatted message as the calling thread's last error and returns `s`.
ep_status ep_fail(ep_status s, const char *fmt, ...) __attribute__((format(printf, 2, 3)));
void ep_clear_error();
