#include "device_common.h"
#include "launch.h"
namespace psdev {
int32_t launch_mfma_attention(const AttnParams&, const ps_geometry&, int, int, int, hipStream_t) { return PS_ERR_UNSUPPORTED; }
}
