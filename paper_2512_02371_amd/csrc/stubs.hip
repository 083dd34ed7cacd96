// Entry points whose kernels are not written yet report HB_ERR_UNSUPPORTED.
#include "hb_host.hpp"
extern "C" {
size_t hb_sat2d_workspace_size(int, int) { return 0; }
hb_status hb_sat2d(const hb_half*, float*, int, int, int64_t, int64_t, void*, size_t, hb_stream) { return HB_ERR_UNSUPPORTED; }
hb_status hb_sat2d_valu(const hb_half*, float*, int, int, int64_t, int64_t, void*, size_t, hb_stream) { return HB_ERR_UNSUPPORTED; }
hb_status hb_conv3x3(const hb_half*, const hb_half*, hb_half*, int, int, int, int, int, hb_stream) { return HB_ERR_UNSUPPORTED; }
hb_status hb_conv3x3_valu(const hb_half*, const hb_half*, hb_half*, int, int, int, int, int, hb_stream) { return HB_ERR_UNSUPPORTED; }
}
