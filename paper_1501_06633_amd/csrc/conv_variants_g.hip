// Tile shapes of the FPROP convolution kernel, group g: tiles of 16 x 16 matrix blocks: 48 filter rows.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

//          WO WM RA RB KS NS VW JB MB
typedef Cfg<1, 4, 3, 4, 16, 3, 4, 2, 16> C_o48m256;

const VariantEntry kGroup[] = {
    // 57 KB ring + 8 KB table: two workgroups per CU
    // (48 filters of 3x3x96 over 57x57x128 outputs: 79 % against 62 % for the best of the 32-row-block tiles)
    make_entry<C_o48m256>("o48m256", 2, 0.79f, 0.75f, 1024),
};

}  // namespace

const VariantEntry* conv_variants_g(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
