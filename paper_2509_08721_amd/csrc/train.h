// Internal declarations of the policy-update translation unit (gfx950 only).
#pragma once
#include "common.h"

namespace sapo {

// Sets the calling thread's error text (what sapo_last_error returns) and returns `code`.
int set_error(int code, const char* fmt, ...);

}  // namespace sapo
