// Entry points of libplc that do not touch the device.
#include "plc_device.h"

extern "C" int plc_version(void) { return 100; }  // 0.1.0

extern "C" const char *plc_strerror(int code) {
  switch (code) {
    case PLC_OK: return "ok";
    case PLC_ERR_INVALID: return "invalid argument, probability row or table";
    case PLC_ERR_CAPACITY: return "output list too small";
    case PLC_ERR_CORRUPT: return "coded stream failed its integrity check";
    case PLC_ERR_HIP: return "HIP launch failed";
    default: return "unknown plc status";
  }
}
