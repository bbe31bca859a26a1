#include "vt_device.h"
using namespace vt;
extern "C" {
size_t vt_decode_attn_workspace(int B, int Hq, int D, int S, int n_splits) { (void)B; (void)Hq; (void)D; (void)S; (void)n_splits; return 0; }
int vt_decode_attn(const vt_desc*, const vt_desc*, const vt_desc*, float, void*, float*, void*, size_t, int, void*) {
  return fail(VT_ERR_UNSUPPORTED, "vt_decode_attn: not built yet");
}
}
