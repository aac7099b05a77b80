// Status strings of the C ABI.
#include "swarm_stage.h"

extern "C" const char* swarm_status_string(swarm_status status) {
  switch (status) {
    case SWARM_OK: return "ok";
    case SWARM_ERR_NULL: return "null pointer";
    case SWARM_ERR_SHAPE: return "unsupported shape, size or alignment";
    case SWARM_ERR_DTYPE: return "unsupported dtype";
    case SWARM_ERR_WORKSPACE: return "workspace too small";
    case SWARM_ERR_LAUNCH: return "kernel launch failed";
  }
  return "unknown status";
}
