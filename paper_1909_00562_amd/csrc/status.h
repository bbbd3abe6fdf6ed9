// Error reporting shared by the files that implement the C ABI: the calling thread's
// last message (read back through attn_softmax_last_error) and the code to return.
#pragma once
#include "../../include/attn_softmax.h"

namespace asx {
as_status set_error(as_status code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));
}
