// Tile variants 0, 1, 5, 6 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part0(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 0: return launch_fast_tile<256, 128, 2, 2, 64, 3, 2>(p, ev, stream);
    case 1: return launch_fast_tile<256, 64, 4, 1, 64, 3, 2>(p, ev, stream);
    case 5: return launch_fast_tile<256, 128, 2, 2, 128, 2, 1>(p, ev, stream);
    case 6: return launch_fast_tile<128, 128, 2, 2, 128, 3, 1>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
