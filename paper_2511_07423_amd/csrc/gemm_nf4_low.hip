// Instantiations of the projection GEMM tile (gemm_tile.h): 256 columns, 16 .. 144 rows.
#include "gemm_tile.h"

hipError_t launch_proj_nf4_low(int mt, const GemmArgs& g, hipStream_t s) {
  switch (mt) {
    case 1: return launch_proj<1, 4>(g, s);
    case 2: return launch_proj<2, 4>(g, s);
    case 3: return launch_proj<3, 4>(g, s);
    case 4: return launch_proj<4, 4>(g, s);
    case 5: return launch_proj<5, 4>(g, s);
    case 6: return launch_proj<6, 4>(g, s);
    case 7: return launch_proj<7, 4>(g, s);
    case 8: return launch_proj<8, 4>(g, s);
    case 9: return launch_proj<9, 4>(g, s);
    default: return hipErrorInvalidValue;
  }
}
