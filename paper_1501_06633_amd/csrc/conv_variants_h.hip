// Tile shapes of the FPROP convolution kernel, group h: 128 x 128 tiles for sizes of which only one is no multiple of 4.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy (14: filters 1, patches 4; 41: filters 4,
// patches 1), barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<2, 2, 2, 2, 16, 3, 14> C_o128m128a;
typedef Cfg<2, 2, 2, 2, 16, 3, 41> C_o128m128b;

const VariantEntry kGroup[] = {
    // a filter count that is no multiple of 4 (rows of the K x No filter matrix start 4-byte
    // aligned only) beside a minibatch that is: 4-byte filter copies, everything else 16 bytes
    // wide.  A 3x3 256-channel layer at 56x56 with No = 250: 83.3 % of the matrix rate in required
    // FLOPs (79.6 % with 4-byte copies of both operands).
    make_entry<C_o128m128a>("o128m128a", 2, 0.855f, 0.81f, 2048),
    // the other way round: 4-byte patch copies and stores, 16-byte filter copies.  The same layer
    // with Nb = 50 / 30: 84.9 / 84.5 % (83.0 / 82.3 %).
    make_entry<C_o128m128b>("o128m128b", 2, 0.85f, 0.80f, 2048),
};

}  // namespace

const VariantEntry* conv_variants_h(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
