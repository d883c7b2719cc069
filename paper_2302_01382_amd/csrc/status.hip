// status.hip -- error reporting of libmpq.
#include "common.hpp"

namespace mpq {
static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }
}  // namespace mpq

extern "C" {

const char* mpq_strerror(int status) {
  switch (status) {
    case MPQ_OK: return "ok";
    case MPQ_ERR_NULL: return "a required pointer is NULL";
    case MPQ_ERR_SHAPE: return "invalid shape (non-positive, overflowing, or odd where even is required)";
    case MPQ_ERR_BITS: return "bit-width out of range (2..8; storage 4 or 8)";
    case MPQ_ERR_ALIGN: return "pointer alignment requirement not met";
    case MPQ_ERR_WORKSPACE: return "workspace missing or too small";
    case MPQ_ERR_GRAN: return "granularity not valid for this call";
    case MPQ_ERR_HIP: return "HIP runtime error on launch";
    case MPQ_ERR_TOO_LARGE: return "input needs more scratch than the library's built-in buffer holds";
    default: return "unknown status";
  }
}

int mpq_last_hip_error(void) { return mpq::g_last_hip_error; }

int mpq_version(void) { return 102; }  // 1.2: batched sweep calls, host functions, no-allocation sweep

}  // extern "C"
