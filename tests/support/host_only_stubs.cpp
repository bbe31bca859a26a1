// Stand-ins for the parts of the library that need the GPU toolchain, for the host-only build
// that the sanitizer test makes of the descriptor builder, the device-form converter and the
// opportunity graph (tests/test_host_sanitizer.py).  Every kernel entry point answers "no device".
#include <cstddef>
#include <cstdint>

#include "vt.h"

extern "C" {
int hipGetLastError() { return 0; }
const char* hipGetErrorString(int) { return "no device in the host-only build"; }

#define VT_STUB(name, ...) int name(__VA_ARGS__) { return VT_ERR_DEVICE; }
VT_STUB(vt_materialize, const vt_desc*, void*, void*)
VT_STUB(vt_copy_op, const vt_source*, int, const vt_op*, void*, void*)
VT_STUB(vt_elementwise, int, const vt_desc*, const vt_desc*, float, void*, void*)
VT_STUB(vt_weighted_sum, const vt_desc*, const vt_desc*, const float*, void*, void*)
VT_STUB(vt_gemm, const vt_desc* const*, const vt_desc* const*, void* const*, int, int, int, float, void*)
VT_STUB(vt_decode_attn_plan, const vt_desc*, const vt_desc*, const vt_desc*, int, int*, int*, int*, int*)
VT_STUB(vt_decode_attn_workspace_init, void*, size_t, void*)
VT_STUB(vt_decode_attn, const vt_desc*, const vt_desc*, const vt_desc*, float, void*, float*, void*, size_t, int, void*)
VT_STUB(vt_decode_attn_static, const vt_desc*, const vt_desc*, const vt_desc*, float, void*, float*, int, void*)
VT_STUB(vt_scatter, const vt_desc*, const vt_desc*, void*)
VT_STUB(vt_gemm_store_workspace_init, void*, size_t, void*)
VT_STUB(vt_gemm_store, const vt_desc*, const vt_desc*, const vt_desc*, void*, size_t, void*)
size_t vt_decode_attn_workspace(int, int, int, int, int) { return 0; }
size_t vt_decode_attn_static_capacity(void) { return 0; }
size_t vt_gemm_store_workspace(int64_t, int64_t, int64_t) { return 0; }
}
