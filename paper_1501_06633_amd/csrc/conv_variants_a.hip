// Tile shapes of the FPROP convolution kernel, group a: the 128 x 128 tile with the deep slab, with its half, third and quarter pieces.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

//          WO WM RA RB KS NS VW
typedef Cfg<2, 2, 2, 2, 16, 3, 4> C_o128m128;

const VariantEntry kGroup[] = {
    make_entry<C_o128m128, 8, true>("o128m128", 2, 0.900f, 0.900f),
};

}  // namespace

const VariantEntry* conv_variants_a(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
