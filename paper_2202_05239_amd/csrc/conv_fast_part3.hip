// Tile variants 12, 13, 14, 15 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part3(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 12: return launch_fast_tile<64, 256, 2, 2, 64, 2, 3>(p, ev, stream);
    case 13: return launch_fast_tile<128, 256, 2, 2, 128, 2, 2>(p, ev, stream);
    case 14: return launch_fast_tile<128, 128, 2, 2, 64, 3, 3>(p, ev, stream);
    case 15: return launch_fast_tile<128, 128, 2, 2, 64, 4, 2>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
