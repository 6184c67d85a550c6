// Instantiations of the projection GEMM tile (gemm_tile.h): 128 columns, 16 .. 192 rows.
#include "gemm_tile.h"

hipError_t launch_proj_nf2(int mt, const GemmArgs& g, hipStream_t s) {
  switch (mt) {
    case 1: return launch_proj<1, 2>(g, s);
    case 2: return launch_proj<2, 2>(g, s);
    case 3: return launch_proj<3, 2>(g, s);
    case 4: return launch_proj<4, 2>(g, s);
    case 5: return launch_proj<5, 2>(g, s);
    case 6: return launch_proj<6, 2>(g, s);
    case 7: return launch_proj<7, 2>(g, s);
    case 8: return launch_proj<8, 2>(g, s);
    case 9: return launch_proj<9, 2>(g, s);
    case 10: return launch_proj<10, 2>(g, s);
    case 11: return launch_proj<11, 2>(g, s);
    case 12: return launch_proj<12, 2>(g, s);
    default: return hipErrorInvalidValue;
  }
}
