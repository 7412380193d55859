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
    case PLC_ERR_SCRATCH: return "shape needs more scratch than the library's static buffer holds";
    default: return "unknown plc status";
  }
}

namespace plc {
TraceEvents g_trace[PLC_TRACE_COUNT] = {};
}

extern "C" int plc_trace_kernel_events(int kernel_id, void *start, void *stop) {
  if (kernel_id < 0 || kernel_id >= PLC_TRACE_COUNT) return PLC_ERR_INVALID;
  if ((start == nullptr) != (stop == nullptr)) return PLC_ERR_INVALID;
  plc::g_trace[kernel_id].start = static_cast<hipEvent_t>(start);
  plc::g_trace[kernel_id].stop = static_cast<hipEvent_t>(stop);
  return PLC_OK;
}
