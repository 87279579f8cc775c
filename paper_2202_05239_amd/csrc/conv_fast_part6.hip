// Tile variants 22, 23 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part6(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 22: return launch_fast_tile<256, 256, 2, 2, 128, 2, 1>(p, ev, stream);
    case 23: return launch_fast_tile<256, 256, 2, 2, 64, 3, 1>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
