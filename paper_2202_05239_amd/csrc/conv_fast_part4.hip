// Tile variants 16, 17, 20, 21 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part4(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 16: return launch_fast_tile<128, 64, 2, 2, 64, 3, 4>(p, ev, stream);
    case 17: return launch_fast_tile<128, 64, 2, 2, 64, 4, 3>(p, ev, stream);
    case 20: return launch_fast_tile<256, 256, 2, 4, 64, 3, 1>(p, ev, stream);
    case 21: return launch_fast_tile<256, 128, 4, 2, 128, 2, 1>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
