// Tile shapes of the FPROP convolution kernel, group d: the 96 x 256 tile (eight waves) with its halves, and the deep 64 x 256 tile.
// Columns of a shape: waves along filters x along columns, matrix blocks per wave along filters x
// along columns, slab depth, ring stages, floats per copy, barrier k-step, block edge.
// An entry: name, workgroups that fit one compute unit, measured fraction of the matrix rate with
// many tiles per unit / with few, offset-table entries kept in LDS (sized so that a long K does
// not cost a resident workgroup).
#include "conv_tile.h"

namespace mdnn {
namespace {

//          WO WM RA RB KS NS VW JB MB
// eight waves of 48 x 64 in 16 x 16 blocks: four waves of 96 x 64 need more than 200 registers each,
// which leaves two waves per SIMD however many workgroups fit; this shape runs four (a 3 -> 96
// channel first layer of 11 x 11 filters: 83.3 -> 85.9 % of peak)
typedef Cfg<2, 4, 3, 4, 16, 3, 4, 2, 16> C_o96m256;
typedef Cfg<1, 4, 2, 2, 16, 3, 4> C_o64m256;

const VariantEntry kGroup[] = {
    // with its half (48 x 256) and quarter (48 x 128) bodies for the last partial round of tiles:
    // 1568 tiles (six rounds + 32) 82.8 % with halves, 85.5 % with quarters.  Rated for few tiles
    // from a sweep of 272 ... 2320 tiles of a 96-filter 3x3 layer (with 0.82 the smaller tiles took
    // the layers under five rounds and lost 1 ... 4 points on most of them).
    make_entry<C_o96m256, 4>("o96m256", 2, 0.885f, 0.88f, 1536),
    make_entry<C_o64m256>("o64m256", 2, 0.885f, 0.86f, 2304),
};

}  // namespace

const VariantEntry* conv_variants_d(int* count)
{
    *count = (int)(sizeof(kGroup) / sizeof(kGroup[0]));
    return kGroup;
}

}  // namespace mdnn
