// Tile shapes of the FPROP convolution kernel, group b: the 128 x 128 tile with the shallow slab (three workgroups per compute unit).
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<2, 2, 2, 2, 8, 4, 4> C_o128m128k8;

const VariantEntry kGroup[] = {
    // 32 KB ring + 20 KB table = 52 KB: three workgroups per CU whatever K is
    make_entry<C_o128m128k8, 8>("o128m128k8", 3, 0.905f, 0.870f, 2560),
};

}  // namespace

const VariantEntry* conv_variants_b(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
