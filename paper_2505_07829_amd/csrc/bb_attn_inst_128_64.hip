// attention kernel instantiations: head dimensions d = 128, dv = 64
#include "bb_attn_inst.h"
namespace bb {
template void attn_tiled_launch<128, 64>(int, int, int, dim3, dim3, hipStream_t, const AttnArgs&);
template void attn_decode_launch<128, 64>(dim3, hipStream_t, const AttnArgs&);
}
