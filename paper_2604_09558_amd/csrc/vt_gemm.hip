#include "vt_device.h"
using namespace vt;
extern "C" {
int vt_gemm(const vt_desc* const*, const vt_desc* const*, void* const*, int, int, int, float, void*) {
  return fail(VT_ERR_UNSUPPORTED, "vt_gemm: not built yet");
}
}
