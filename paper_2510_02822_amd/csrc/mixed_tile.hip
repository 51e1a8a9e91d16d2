// One tile shape of the mixed GEMM / implicit-GEMM kernel: the four instantiations (linear or convolution,
// 4-bit weights from the packed codes or from the expanded copy).  Built once per shape with -DFQ_TILE=i.
#include "mixed_kernel.h"

#ifndef FQ_TILE
#error "compile with -DFQ_TILE=<0..7>"
#endif

namespace flexiq {

// waves along M, waves along N, 32x32 fragments per wave along M and N; then the measured cycles of one
// K-step of a block alone on its CU, the relative growth per co-resident block, and the epilogue cycles.
#if FQ_TILE == 0
TileShape tile_shape_0() { return make_shape<2, 2, 4, 4>(1530.0, 0.0, 11000.0); }  // 256 x 256
#elif FQ_TILE == 1
TileShape tile_shape_1() { return make_shape<1, 4, 7, 2>(1280.0, 0.0, 9000.0); }  // 224 x 256
#elif FQ_TILE == 2
TileShape tile_shape_2() { return make_shape<2, 2, 3, 4>(1150.0, 0.0, 8000.0); }  // 192 x 256
#elif FQ_TILE == 3
TileShape tile_shape_3() { return make_shape<1, 4, 5, 2>(1050.0, 0.0, 6500.0); }   // 160 x 256
#elif FQ_TILE == 4
TileShape tile_shape_4() { return make_shape<2, 2, 2, 4>(735.0, 0.35, 6500.0); }   // 128 x 256
#elif FQ_TILE == 5
TileShape tile_shape_5() { return make_shape<2, 2, 2, 2>(700.0, 0.35, 2900.0); }   // 128 x 128
#elif FQ_TILE == 6
TileShape tile_shape_6() { return make_shape<2, 2, 1, 2>(500.0, 0.37, 1500.0); }   //  64 x 128
#elif FQ_TILE == 7
TileShape tile_shape_7() { return make_shape<2, 2, 1, 1>(400.0, 0.45, 900.0); }     //  64 x  64
#else
#error "FQ_TILE out of range"
#endif

}  // namespace flexiq
