// Tile shapes of the FPROP convolution kernel, group i: 128 x 128 tiles for a minibatch that is no multiple of 4 beside a filter count that is.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy (41: filters 4, patches 1), barrier k-step,
// block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<2, 2, 2, 2, 16, 3, 41> C_o128m128b;
typedef Cfg<2, 2, 2, 2, 8, 4, 41> C_o128m128k8b;

const VariantEntry kGroup[] = {
    // 4-byte patch copies and stores, 16-byte filter copies; half and quarter pieces for the last
    // partial round of tiles.  A 3x3 256-channel layer at 56x56 with Nb = 50 / 30: 85.3 / 84.7 % of
    // the matrix rate (82.7 % with 4-byte copies of both operands)
    make_entry<C_o128m128b, 4>("o128m128b", 2, 0.85f, 0.80f, 2048),
    // the same on the 8-deep slab with three workgroups per unit: 86.6 / 87.5 %
    make_entry<C_o128m128k8b, 4>("o128m128k8b", 3, 0.865f, 0.79f, 2560),
};

}  // namespace

const VariantEntry* conv_variants_i(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
