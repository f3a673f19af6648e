// Internal interface between the host API (mdnn_api.cpp) and the kernel
// translation unit (conv_fprop.hip).  Not installed; not part of the C ABI.
#ifndef MDNN_INTERNAL_H_
#define MDNN_INTERNAL_H_

#include <stdint.h>
#include "mdnn.h"

namespace mdnn {

constexpr int kMaxTabEntries = 4096;     // offset-table entries resident in LDS at once: 32 KB

// Everything a tile needs, passed by value as the single kernel argument.
struct ConvParams {
    const float* in;
    const float* filt;
    float*       out;
    int Nb, Wi, Hi, Nc, No, Sk, stride, pad;
    int Wo, Ho;
    int K;               // Nc*Sk*Sk: rows of the filter matrix / columns of a patch (Section 3)
    int SkSk;            // Sk*Sk
    // exact division of any n < 2^31 by SkSk and by Sk without a divide instruction:
    // q = (mulhi(n, magic) + ((n - mulhi(n, magic)) >> 1)) >> shift
    uint32_t sksk_magic, sksk_shift, sk_magic, sk_shift;
    uint32_t nb_magic, nb_shift, wo_magic, wo_shift;      // the same for Nb and Wo
    int M;               // Ho*Wo*Nb: columns of the output seen as a row-major No x M matrix
    int n_otiles;        // tiles along No
    int n_mtiles;        // tiles along M
    int n_tiles;         // n_otiles * n_mtiles
    // Tail balancing: tiles [0, n_whole) run whole; the last n_tiles - n_whole tiles are cut into
    // pieces that run as separate workgroups: first n_half tiles in halves, then n_third tiles in
    // thirds (48 + 48 + 32 filter rows of a 128-row tile), then n_quarter tiles in quarters.
    // Pieces are numbered within their class (halves, pieces of thirded tiles, quarters).
    int n_whole;
    int n_half, n_third, n_quarter, n_eighth;
    int n_pieces;        // 2 n_half + 3 n_third + 4 n_quarter + 8 n_eighth
    int tiles_per_xcd;   // ceil(n_whole / 8)
    // Launch order: the `front` pieces, the whole tiles, the `back` pieces.  Within a region the
    // classes follow each other, largest pieces first, and every class is dealt to the 8 XCDs in
    // contiguous runs of per_xcd pieces (so every XCD gets its share of every size).
    struct PieceRegion {
        int begin[4];    // first piece of class c (0 halves, 1 thirds, 2 quarters, 3 eighths) in this region
        int count[4];    // pieces of class c in this region
        int per_xcd[4];  // ceil(count / 8)
        int wgs;         // 8 * (sum of per_xcd): workgroups the region occupies in the grid
        int pieces;      // sum of count
    };
    PieceRegion front, back;
    // Column-tile order.  When a tile covers whole output pixels and a row of pixels is a whole
    // number of tiles (row_tiles > 0), column tiles are visited in strips of strip_rows image rows,
    // column by column inside a strip, so that the tiles in flight on one XCD form a compact 2-D
    // patch of the image and the overlapping input patches of neighbouring pixels meet in its L2.
    // row_tiles == 0: plain row-major order.
    int row_tiles;       // tiles per row of output pixels
    int strip_rows;
    int tab_cap;         // offset-table entries resident in LDS at once (multiple of the K slab)
    // Scatter mode of the epilogue (scat_stride > 0), used by the data gradient of strided layers:
    // the problem's "filters" are (residue class, channel) pairs, row o = cls * scat_Nc + c with
    // cls = ry * scat_stride + rx, and the value at output pixel (qy, qx) belongs to
    // out[c][qy * scat_stride + ry - scat_pad][qx * scat_stride + rx - scat_pad][n] of a
    // [scat_Nc][scat_Hi][scat_Wi][Nb] tensor (dropped where that pixel does not exist).
    int scat_stride, scat_Nc, scat_Hi, scat_Wi, scat_pad;
    int stream_out;      // 1: whole tiles store with the non-temporal hint (short contractions, large outputs)
    uint32_t in_bytes;   // byte size of in   (buffer-resource range: loads beyond it return 0)
    uint32_t filt_bytes; // byte size of filt
    float alpha;
};

// Static description of one tile variant (one template instantiation).
struct VariantInfo {
    const char* name;
    int tile_o;          // output filters per workgroup tile
    int tile_m;          // flat (coordinate, batch) columns per workgroup tile
    int kslab;           // patch columns (k) staged in LDS per pipeline step
    int threads;         // workgroup size
    int vec_a;           // 1: 16-byte filter copies, needs No % 4 == 0
    int vec_b;           // 1: 16-byte patch copies and stores, needs Nb % 4 == 0
    int est_wg_per_cu;   // workgroups expected to be co-resident on one compute unit
    float eff;           // sustained fraction of the matrix rate with many tiles per compute unit (measured)
    float eff_few;       // same with fewer than four tiles per compute unit: start-up and drain of
                         // co-resident workgroups coincide instead of overlapping (measured)
    int max_split;       // 1, 2, 4 or 8: finest even cut of a tile this variant's kernel can run
    int thirds;          // 1: the kernel can also run a tile as 48 + 48 + 32 filter rows
    int max_tab;         // most offset-table entries kept in LDS at once (longer K: several fills per tile)
};

// One instantiated kernel.  The translation units conv_variants_*.hip each hold a few of them
// (so that they compile side by side); conv_fprop.hip strings their lists together.
typedef void (*ConvKernelFn)(const ConvParams);
struct VariantEntry {
    VariantInfo  info;
    ConvKernelFn fn;
    uint32_t     ring_bytes;     // LDS of the operand ring; the offset table follows it
};
const VariantEntry* conv_variants_a(int* count);
const VariantEntry* conv_variants_b(int* count);
const VariantEntry* conv_variants_c(int* count);
const VariantEntry* conv_variants_d(int* count);
const VariantEntry* conv_variants_e(int* count);
const VariantEntry* conv_variants_f(int* count);
const VariantEntry* conv_variants_g(int* count);
const VariantEntry* conv_variants_h(int* count);
const VariantEntry* conv_variants_i(int* count);

int                variant_count();
const VariantInfo& variant_info(int i);

// LDS bytes variant i needs for a table of tab_cap entries.
uint32_t variant_lds_bytes(int i, int tab_cap);

// Enqueue variant i.  p.n_* / tab_cap must have been filled for that variant.
// Returns hipSuccess (0) or the HIP error code as int.
int launch_variant(int i, const ConvParams& p, void* stream);

int launch_mfma_probe(float* sink, int blocks, int waves_per_block, int iters, void* stream);

// Layout kernels of the data gradient (bprop_data.hip); return hipSuccess (0) or the HIP error code.
int launch_flip_transpose(const float* filt, float* ft, int Nc, int No, int SkSk, void* stream);
int launch_class_filters(const float* filt, float* fc, int Nc, int No, int Sk, int stride, int T, void* stream);
// din[c][iy][ix][n] = 0 for iy >= y_end or ix >= x_end (the pixels no window reaches)
int launch_zero_unreached(float* din, int Nc, int Hi, int Wi, int Nb, int y_end, int x_end, void* stream);

// Device address, on the current GPU, of the static array of MDNN_STATIC_SCRATCH_BYTES bytes behind
// mdnn_conv_bprop_data_static (bprop_data.hip); looked up once per GPU.  Returns 0 or a HIP error code.
int static_scratch(void** ptr);

// Filter gradient (bprop_filter.hip): everything a workgroup needs.
struct FilterGradParams {
    const float* in;
    const float* dout;
    float*       part;       // workspace: [splits][K][No] partial gradients
    int Nb, Wi, Hi, Nc, No, Sk, stride, pad;
    int Wo, Ho;
    int K, SkSk, M;
    uint32_t sksk_magic, sksk_shift, sk_magic, sk_shift;
    uint32_t nb_magic, nb_shift, wo_magic, wo_shift;
    int tile_o;              // columns of dfilt per workgroup: 128, 96, 64 or 32
    int n_otiles;            // tiles along No
    int n_tiles;             // tiles of the K x No gradient
    int splits;              // ranges the contraction index m is cut into
    int m_per_split;         // multiple of 16
    int per_xcd;             // ceil(n_tiles * splits / 8)
    int vec;                 // 1: 16-byte copies (Nb % 4 == 0)
    int uniform;             // 1: Nb % 16 == 0, a slab of 16 m never straddles output coordinates
    uint32_t in_bytes, dout_bytes;
};

// Enqueue the partial-gradient kernel and the kernel that sums the partials into dfilt.
int launch_bprop_filter(const FilterGradParams& p, float* dfilt, float alpha, void* stream);

}  // namespace mdnn
#endif
