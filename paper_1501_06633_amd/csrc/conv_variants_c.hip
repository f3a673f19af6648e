// Tile shapes of the FPROP convolution kernel, group c: the big tiles (one workgroup per compute unit) and the 96 x 128 tile.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<2, 2, 4, 2, 16, 3, 4> C_o256m128;
typedef Cfg<2, 2, 2, 4, 16, 3, 4> C_o128m256;
typedef Cfg<1, 4, 3, 1, 16, 3, 4> C_o96m128;

const VariantEntry kGroup[] = {
    make_entry<C_o256m128>("o256m128", 1, 0.83f, 0.83f),
    make_entry<C_o128m256>("o128m256", 1, 0.83f, 0.83f),
    // 42 KB ring + 10 KB table: three workgroups per CU whatever K is
    make_entry<C_o96m128>("o96m128", 3, 0.855f, 0.855f, 1280),
};

}  // namespace

const VariantEntry* conv_variants_c(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
