// Status strings and version of libgnnagg.
#include "gnnagg.h"

extern "C" int gnnagg_version(void) { return 310; }  // major*10000 + minor*100 + patch

extern "C" const char* gnnagg_strerror(int status) {
  switch (status) {
    case GNNAGG_OK: return "ok";
    case GNNAGG_EINVAL: return "invalid argument";
    case GNNAGG_ENULL: return "required pointer is null";
    case GNNAGG_EUNSUPPORTED: return "not supported by the library";
    case GNNAGG_EWORKSPACE: return "workspace missing, too small or misaligned";
    case GNNAGG_EDEVICE: return "HIP runtime error";
    default: return "unknown status";
  }
}
