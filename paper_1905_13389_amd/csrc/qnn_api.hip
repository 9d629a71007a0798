// Library-wide entry points: version, build id and the thread-local error message.
#include "qnn_host.h"

namespace qnn {
char *error_buffer()
{
    static thread_local char buf[kErrorBufferSize] = {0};
    return buf;
}
} // namespace qnn

extern "C" const char *qnn_last_error(void) { return qnn::error_buffer(); }

extern "C" int qnn_version(void) { return 0 * 10000 + 4 * 100 + 0; }

#ifndef QNN_BUILD_ID
#define QNN_BUILD_ID ""
#endif
extern "C" const char *qnn_build_id(void) { return QNN_BUILD_ID; }
