// Tile shapes of the FPROP convolution kernel, group f: the small tiles and the 4-byte-copy tile for sizes that are not multiples of 4.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

typedef Cfg<1, 4, 1, 1, 16, 3, 4> C_o32m128;
typedef Cfg<1, 2, 1, 1, 16, 3, 4> C_o32m64;
typedef Cfg<1, 1, 1, 1, 16, 3, 4> C_o32m32;
typedef Cfg<2, 2, 1, 1, 16, 3, 1> C_o64m64s;
typedef Cfg<2, 2, 2, 2, 16, 3, 1> C_o128m128s;

const VariantEntry kGroup[] = {
    make_entry<C_o32m128>("o32m128", 4, 0.80f, 0.80f, 1024),
    make_entry<C_o32m64>("o32m64", 8, 0.55f, 0.55f, 1024),
    make_entry<C_o32m32>("o32m32", 8, 0.35f, 0.35f, 1024),
    // 4-byte copies: any Nb and No.  Measured on a 3x3 256-channel layer at 56x56: 78 % of the matrix
    // rate with Nb = 50 or No = 250 (and with sizes the 16-byte tiles could take as well)
    make_entry<C_o64m64s>("o64m64s", 4, 0.76f, 0.70f),
    // the 128 x 128 tile fed by 4-byte copies, sixteen copies per thread and slab instead of four:
    // 83 % with Nb = 50, 79.5 % with No = 250
    make_entry<C_o128m128s, 4>("o128m128s", 2, 0.83f, 0.78f, 2048),
};

}  // namespace

const VariantEntry* conv_variants_f(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
