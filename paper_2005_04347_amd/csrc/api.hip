// Small parts of the C ABI that launch nothing: error strings, version.
#include "asnn_common.h"

namespace asnn {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(hipError_t e) { g_last_hip_error = (int)e; }
}  // namespace asnn

extern "C" int asnn_last_hip_error(void) { return asnn::g_last_hip_error; }

extern "C" int asnn_version(void) { return 1; }

extern "C" const char *asnn_strerror(int code) {
    switch (code) {
        case ASNN_OK: return "ok";
        case ASNN_ERR_NULL: return "a required pointer is NULL";
        case ASNN_ERR_SIZE: return "bad size argument";
        case ASNN_ERR_INDEX: return "node id or level out of range";
        case ASNN_ERR_INPUT_HAS_INEDGE: return "a connection ends in an input node";
        case ASNN_ERR_DUP_INPUT: return "an input id is listed twice";
        case ASNN_ERR_CYCLE: return "the connections contain a cycle";
        case ASNN_ERR_WORKSPACE: return "workspace too small or misaligned";
        case ASNN_ERR_HIP: return "a HIP runtime call failed (see asnn_last_hip_error)";
        case ASNN_ERR_LEVEL_ORDER: return "level[] does not increase along a connection";
        case ASNN_ERR_NO_DEVICE: return "no HIP device available";
        case ASNN_ERR_TIMEOUT: return "a dataflow wait exceeded its time limit";
        case ASNN_ERR_SCRATCH: return "network and batch need more scratch than asnn_activate_static holds";
        default: return "unknown error";
    }
}
