// Tile variants 18, 19 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part5(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 18: return launch_fast_tile<256, 256, 2, 4, 128, 2, 1>(p, ev, stream);
    case 19: return launch_fast_tile<256, 256, 4, 2, 128, 2, 1>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
