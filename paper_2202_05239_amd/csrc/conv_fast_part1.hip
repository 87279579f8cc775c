// Tile variants 2, 3, 4, 7 of the LDS-direct dense kernel (conv_fast_kernel.h).
#include "conv_fast_kernel.h"
#include "conv_fast_parts.h"

namespace f8 {

int launch_conv_fast_part1(int variant, const ConvParams &p, int ev, hipStream_t stream) {
  switch (variant) {
    case 2: return launch_fast_tile<128, 128, 2, 2, 64, 2, 4>(p, ev, stream);
    case 3: return launch_fast_tile<128, 64, 2, 2, 64, 2, 4>(p, ev, stream);
    case 4: return launch_fast_tile<128, 128, 2, 2, 128, 2, 2>(p, ev, stream);
    case 7: return launch_fast_tile<128, 64, 2, 2, 128, 2, 3>(p, ev, stream);
    default: return -1;
  }
}

}  // namespace f8
