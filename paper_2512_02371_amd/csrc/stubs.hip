// Entry points whose kernels are not written yet report HB_ERR_UNSUPPORTED.
#include "hb_host.hpp"
extern "C" {
hb_status hb_conv3x3(const hb_half*, const hb_half*, hb_half*, int, int, int, int, int, hb_stream) { return HB_ERR_UNSUPPORTED; }
hb_status hb_conv3x3_valu(const hb_half*, const hb_half*, hb_half*, int, int, int, int, int, hb_stream) { return HB_ERR_UNSUPPORTED; }
}
