// Tile shapes of the FPROP convolution kernel, group e: the shallow 64 x 256 tile with its half and quarter pieces.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<1, 4, 2, 2, 8, 4, 4> C_o64m256k8;

const VariantEntry kGroup[] = {
    // 40 KB ring + 12 KB table: three workgroups per CU (+1 ... 2 % on 64-filter layers with many tiles)
    make_entry<C_o64m256k8, 4>("o64m256k8", 3, 0.900f, 0.85f, 1536),
};

}  // namespace

const VariantEntry* conv_variants_e(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
