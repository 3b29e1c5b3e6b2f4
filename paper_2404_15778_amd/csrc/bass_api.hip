// Version and status strings of libbass.
#include "bass_common.h"

extern "C" int bass_version(void) { return 100; /* 0.1.0 */ }

extern "C" const char* bass_status_string(int code) {
  switch (code) {
    case BASS_OK: return "ok";
    case BASS_ERR_INVALID_ARG: return "invalid argument";
    case BASS_ERR_UNSUPPORTED: return "unsupported shape or dtype";
    case BASS_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case BASS_ERR_HIP: return "HIP launch error";
    default: return "unknown status";
  }
}
