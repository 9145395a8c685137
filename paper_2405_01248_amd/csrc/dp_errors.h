// Thread-local last-error message; error codes come from the public header.
#pragma once
#include "../../include/dpipe.h"
namespace dp {
// Records msg as the calling thread's last error and returns code.
int set_error(int code, const char* msg);
int set_errorf(int code, const char* fmt, ...);
}  // namespace dp
