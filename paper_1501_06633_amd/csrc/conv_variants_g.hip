// Tile shapes of the FPROP convolution kernel, group g: the 48-row tile of 16 x 16 matrix blocks, and the wide tile for output-bound layers.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

//          WO WM RA RB KS NS VW JB MB
// four waves of 48 x 32: few registers, three workgroups per unit (a 48 x 256 tile on four waves of
// 48 x 64 reached 79 % where this one reaches 86 %; eight waves of 48 x 32 on 48 x 256: 81 %)
typedef Cfg<1, 4, 3, 2, 16, 3, 4, 2, 16> C_o48m128;
// eight waves of 32 x 128 (32 x 32 blocks): 2 KB of every output row per tile, for contractions so
// short that the layer is bound by writing its output
typedef Cfg<2, 4, 1, 4, 8, 3, 4, 2, 32> C_o64m512;

const VariantEntry kGroup[] = {
    // 34 KB ring + 8 KB table: three workgroups per CU
    // (48 filters of 3x3x96 over 57x57x128 outputs: 86 % against 62 % for the best of the 32-row-block tiles)
    // (with two or four row tiles -- 96, 192 filters -- it runs at 83-84 % where the 96-row tiles reach 86-88 %)
    make_entry<C_o48m128>("o48m128", 3, 0.83f, 0.78f, 1024),
    // chosen by rule (K <= 64), not by cost: rated so that the cost model never picks it elsewhere
    make_entry<C_o64m512>("o64m512", 2, 0.50f, 0.50f, 64),
};

}  // namespace

const VariantEntry* conv_variants_g(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
