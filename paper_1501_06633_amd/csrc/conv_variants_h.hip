// Tile shapes of the FPROP convolution kernel, group h: 128 x 128 tiles for a filter count that is no multiple of 4 beside a minibatch that is.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy (14: filters 1, patches 4), barrier k-step,
// block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<2, 2, 2, 2, 16, 3, 14> C_o128m128a;
typedef Cfg<2, 2, 2, 2, 8, 4, 14> C_o128m128k8a;

const VariantEntry kGroup[] = {
    // a filter count that is no multiple of 4 (rows of the K x No filter matrix start 4-byte
    // aligned only) beside a minibatch that is: 4-byte filter copies, everything else 16 bytes
    // wide; half and quarter pieces for the last partial round of tiles.  A 3x3 256-channel layer
    // at 56x56 with No = 250 (3136 tiles): 87.7 % of the matrix rate in required FLOPs (79.4 % with
    // 4-byte copies of both operands and no pieces).
    make_entry<C_o128m128a, 4>("o128m128a", 2, 0.855f, 0.81f, 2048),
    // the same on the 8-deep slab with three workgroups per unit, for launches of many tiles:
    // 89.2 % on that layer; 1001 filters on 14x14 (784 tiles, 16 of them left over): 83.5 %
    // against 67 % without pieces
    make_entry<C_o128m128k8a, 4>("o128m128k8a", 3, 0.87f, 0.80f, 2560),
};

}  // namespace

const VariantEntry* conv_variants_h(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
