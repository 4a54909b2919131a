// Internal helpers shared by the host packer and the device dispatcher.
#pragma once
#include <cstdarg>
#include <cstddef>
#include <cstdint>

#include "liquidgemm.h"

namespace lqq {

// Records a printf-style message for w4a8_last_error() and returns `code`.
int fail(int code, const char *fmt, ...);

// Shape rules of the packed layout (see lqq_layout.h).
inline bool shape_ok(int N, int K, int group)
{
    return N > 0 && K > 0 && N % 64 == 0 && K % 256 == 0 && (group == 64 || group == 128) &&
           K <= 131072 && N <= (1 << 26);
}

}  // namespace lqq
