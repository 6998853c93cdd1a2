#include "sp_common.h"
namespace sp {
sp_status launch_attn_bwd(const AttnArgs&, hipStream_t) { return SP_ERR_UNSUPPORTED; }
}
