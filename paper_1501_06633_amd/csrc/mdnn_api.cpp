// Host side of the C ABI: argument checks, geometry, the complexity formula,
// tile-variant choice.  No HIP call happens in this file; launches go through
// mdnn::launch_variant().
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <cstdlib>

#include "mdnn_internal.h"

namespace {

constexpr int     kComputeUnits = 256;          // MI355X
constexpr int     kStripRows = 8;               // image rows per strip of the 2-D tile order (measured: 4 and 8 fetch
                                                // least through L2, 2 and 16 about 15-35 % more, row-major 50 % more)
constexpr int64_t kFourGiB = (int64_t)1 << 32;
constexpr int     kWideTileMaxK = 64;           // ... and below this the 64 x 512 tile is taken
constexpr int     kStreamOutMaxK = 128;         // contractions this short are bound by writing the output
constexpr int64_t kStreamOutMinBytes = (int64_t)16 << 20;   // an output of half the 8 x 4 MB of L2 or more would not
                                                // stay there beside the operands: it is streamed past them
                                                // (never slower; 0 ... 2.6 points at K = 576 and 0 ... 0.8 on longer
                                                // contractions, depending on the machine the run landed on)
constexpr int     kMaxSlab = 64;                // no tile variant stages more rows of k than this at once

struct Geometry {
    int     Wo, Ho;
    int64_t K, M, in_bytes, filt_bytes, out_bytes;
};

mdnn_status check_geometry(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad,
                           Geometry* g)
{
    if (Nb < 1 || Wi < 1 || Hi < 1 || Nc < 1 || No < 1 || Sk < 1 || stride < 1 || pad < 0)
        return MDNN_EINVAL;
    const int64_t Wp = (int64_t)Wi + 2 * (int64_t)pad, Hp = (int64_t)Hi + 2 * (int64_t)pad;
    if (Sk > Wp || Sk > Hp) return MDNN_EINVAL;
    if (Wp >= ((int64_t)1 << 30) || Hp >= ((int64_t)1 << 30)) return MDNN_ETOOBIG;
    const int64_t Wo = (Wp - Sk) / stride + 1, Ho = (Hp - Sk) / stride + 1;
    // sizes in 64-bit, factor by factor, so that nothing wraps before the limit check
    auto bytes = [](int64_t a, int64_t b, int64_t c, int64_t d) -> int64_t {
        int64_t v = 4;
        const int64_t f[4] = {a, b, c, d};
        for (int64_t x : f) {
            if (v > kFourGiB / x) return kFourGiB;         // v*x would exceed 2^32
            v *= x;
        }
        return v;
    };
    g->in_bytes   = bytes(Nc, Hi, Wi, Nb);
    g->filt_bytes = bytes(Nc, Sk, Sk, No);
    g->out_bytes  = bytes(No, Ho, Wo, Nb);
    // The filter offsets advance one slab past the last row before the loop ends and must not
    // wrap back into the buffer: keep the filter bank under 2 GiB.
    if (g->in_bytes >= kFourGiB || g->filt_bytes >= kFourGiB / 2 || g->out_bytes >= kFourGiB)
        return MDNN_ETOOBIG;
    // Rows k >= K of the filter matrix read as zero because their byte offset lies beyond the end
    // of the buffer; that needs the offsets of up to kMaxSlab rows past the last one to stay below 2^32.
    if (((int64_t)Nc * Sk * Sk + kMaxSlab) * (int64_t)No * 4 >= kFourGiB) return MDNN_ETOOBIG;
    g->Wo = (int)Wo;
    g->Ho = (int)Ho;
    g->K  = (int64_t)Nc * Sk * Sk;
    g->M  = Ho * Wo * (int64_t)Nb;
    return MDNN_OK;
}

int div_up(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Division by an invariant d (Granlund & Montgomery, "Division by invariant integers using
// multiplication"): with l = ceil(log2 d) and magic = floor(2^32 (2^l - d) / d) + 1,
//     n / d = (t + ((n - t) >> 1)) >> (l - 1),   t = mulhi(n, magic),
// exact for every 32-bit n and every d >= 2.  d = 1 has no such pair and is encoded as magic 0,
// which the device code treats as "return n".
void division_magic(uint32_t d, uint32_t* magic, uint32_t* shift)
{
    if (d == 1) { *magic = 0; *shift = 0; return; }        // device code special-cases magic == 0
    uint32_t l = 0;
    while (((uint64_t)1 << l) < d) ++l;
    *magic = (uint32_t)(((((uint64_t)1 << l) - d) << 32) / d + 1);
    *shift = l - 1;
}

bool variant_usable(const mdnn::VariantInfo& v, int Nb, int No)
{
    return (!v.vec_a || No % 4 == 0) && (!v.vec_b || Nb % 4 == 0);
}

// Tail balancing.  With T tiles on 256 compute units the last T mod 256 tiles form
// a partial round that keeps a few units busy for a whole tile time.  Cutting
// them into pieces (less efficient, but short) can end the launch sooner.  The
// cuts a kernel may offer: halves and quarters of a tile, and for 128-row tiles
// eighths of 16 filter rows and "thirds" of 48 + 48 + 32.
// What was measured: workgroups that share a unit advance through the contraction
// at the same rate (the matrix pipe alternates between their waves), so a piece
// that starts beside a whole tile ends with it, whatever its height, and the two
// together take (128 + piece rows) / 128 tile times.  A second piece in the same
// slot starts when the unit is nearly empty and runs alone, at about half the
// matrix rate.  So the cut to take is the finest one that still leaves at most
// one piece per unit:
//   r <= 32 left-over tiles: eighths of 16 rows (1.125), where measured to pay (see choose_cut());
//   r <= 64: quarters (1.25 tile times for the round instead of 2);
//   r <= 85: thirds (1.375; 338 tiles of 128 x 128 on a 13 x 13 layer: 80 -> 86 % of peak);
//   r <= 128: halves (1.5);
//   r <= 192: quarters in chains of up to three, or -- where the whole tiles leave room for
//       two pieces per unit in front of them -- a half paired with an eighth or a quarter (see
//       choose_cut() for where that is);
// each weighed by the piece's relative efficiency and taken only if it beats the coarser
// choice by a margin.
struct Cut {
    int    n_whole, n_half, n_third, n_quarter, n_eighth;
    double cost;                       // of the partial round, in tile times (0 if there is none)
    bool   pair_up;                    // a half and a smaller piece per unit: all pieces go in front of the whole tiles
    int    pieces() const { return 2 * n_half + 3 * n_third + 4 * n_quarter + 8 * n_eighth; }
};

// `force`: 0 = choose; 'w' = no cutting; 'h', 't', 'q', 'e' = the left-over tiles in halves, thirds,
// quarters, eighths; 'H', 'T', 'Q', 'E' = every tile so; 'm', 'n' = 128 of the left-over tiles in halves
// and the rest in quarters ('m') or eighths ('n'), 'p' = 64 of them in quarters and the rest in eighths,
// all in front (tests and the block-size experiment pin a cut this way).  A kernel that lacks the
// cut asked for, or a tile count outside the range of a pairing, returns n_whole = -1.
Cut choose_cut(const mdnn::VariantInfo& v, int n_tiles, char force = 0)
{
    Cut c = {n_tiles, 0, 0, 0, 0, 0.0, false};
    if (force) {
        const bool all = force == 'H' || force == 'T' || force == 'Q' || force == 'E';
        const int  n = all ? n_tiles : n_tiles % kComputeUnits;
        const char f = all ? (char)(force - 'A' + 'a') : force;
        const bool has = f == 'w' || (f == 'h' && v.max_split >= 2) || (f == 't' && v.thirds) || (f == 'q' && v.max_split >= 4) ||
                         (f == 'e' && v.max_split >= 8) || (f == 'm' && v.max_split >= 4 && n > 128 && n <= 192) ||
                         (f == 'n' && v.max_split >= 8 && n > 128 && n <= 160) ||
                         (f == 'p' && v.max_split >= 8 && n > 64 && n <= 96);
        if (!has) { c.n_whole = -1; return c; }
        if (f == 'm') { c.n_half = 128;  c.n_quarter = n - 128;  c.pair_up = true; }
        if (f == 'n') { c.n_half = 128;  c.n_eighth = n - 128;  c.pair_up = true; }
        if (f == 'p') { c.n_quarter = 64;  c.n_eighth = n - 64;  c.pair_up = true; }
        if (f == 'e') c.n_eighth = n;
        if (f == 'h') c.n_half = n;
        if (f == 't') c.n_third = n;
        if (f == 'q') c.n_quarter = n;
        c.n_whole = n_tiles - (f == 'w' ? 0 : n);
        c.cost = n ? 1.0 : 0.0;
        return c;
    }
    const int r = n_tiles % kComputeUnits;
    if (r == 0) return c;
    c.cost = 1.0;
    if (v.max_split < 2) return c;
    const double e2 = 0.93, e3 = 0.90, e4 = 0.85, e8 = 0.70;   // a half, a 48-row third, a quarter, an eighth against a whole tile
    auto rounds_of = [&](int f) { return (double)((r * f + kComputeUnits - 1) / kComputeUnits) / f; };
    auto take = [&](double cost, int nh, int nt, int nq, int ne = 0, bool pair = false) {
        if (cost < c.cost - 0.05) { c.cost = cost;  c.n_half = nh;  c.n_third = nt;  c.n_quarter = nq;  c.n_eighth = ne;  c.pair_up = pair; }
    };
    const int R = n_tiles / kComputeUnits;
    if (v.max_split >= 8 && R >= 1) {
        // The two 128 x 128 kernels, which have every piece size.  Measured over R = 1 ... 8 rounds
        // and r = 8 ... 248 left-over tiles on five layer families (3x3 with 128, 256, 384
        // and 512 filters, 5x5 with 256), every cut pinned in turn.  With pieces of one size the best cut
        // follows the rows on the busiest unit at every R:
        //     r <= 32 eighths (16 rows) | <= 64 quarters (32) | <= 128 halves (64) | <= 192 quarters in
        //     chains of up to three | beyond: whole tiles,
        // with thirds (48 rows) for 64 < r <= 85 on the two-per-unit kernel when the whole tiles leave
        // half of their last wave of 512 free (R odd: +1.5 ... +6 points over halves; R even: 62 ... 80 %
        // against 81 ... 88 %).  Pairings of two sizes per
        // unit (<= 96: a quarter and an eighth; <= 160: a half and an eighth; <= 192: a half and a
        // quarter; all pieces in front) need room for up to 512 pieces beside the whole tiles:
        //   - three-per-unit kernel: the last wave of 768 must hold only 256 whole tiles (R mod 3 = 1;
        //     +1 ... +6 points over chains and halves on all five families); with 512 in it (R = 2, 5)
        //     the half pairings fall to 65 ... 82 %, the quarter-and-eighth pairing still holds;
        //   - two-per-unit kernel: the half and the eighth are steady at every R on all five families
        //     (84 ... 92 %, 3 ... 6 points over quarter chains) and are taken; so is the quarter and the
        //     eighth for two to eight rounds (0.3 ... 4.7 points over halves in all 24 measured cases; beside
        //     a single round it falls to 49 ... 52 % on three of the families); the half and the quarter
        //     fall to 79.8 % against 89.5 % and 84.5 % against 89.5 % on two 5x5 layers five rounds
        //     long -- not taken.
        // Whole tiles that fill their last wave exactly (three-per-unit kernel, R mod 3 = 0) leave
        // no room for any piece in front: halves swing between 75 and 91 % from shape to shape,
        // eighths between 67 and 82 %; quarters, alone or in chains, are the steady choice (83 ... 91 %).
        // (Beyond eight rounds, where nothing was measured and the tail is a few per cent of the
        // launch, a full last wave only rules out the eighths.)
        const bool three = v.est_wg_per_cu >= 3;
        const bool full_wave = three && R % 3 == 0;
        if (full_wave && R <= 8) {
            if (r <= 192) take(rounds_of(4) / e4, 0, 0, r);
        } else if (r <= 32 && !(three && R == 1) && !full_wave) take(0.125 / e8, 0, 0, 0, r);
        else if (r <= 64)                          take(0.25 / e4, 0, 0, r);
        else if (r <= 85 && v.thirds && R % 2 == 1) take(0.375 / e3, 0, r, 0);
        else if (r <= 96 && (three ? !full_wave : R >= 2 && R <= 8)) take(0.40, 0, 0, 64, r - 64, true);
        else if (r <= 128)                         take(0.5 / e2, r, 0, 0);
        else if (r <= 160 && (!three || R % 3 == 1)) take(three || R >= 2 ? 0.65 : 0.72, 128, 0, 0, r - 128, true);
        else if (r <= 192 && three && R % 3 == 1)  take(0.78, 128, 0, r - 128, 0, true);
        else if (r <= 192)                         take(rounds_of(4) / e4, 0, 0, r);
        if (c.pieces() > 0) c.n_whole = n_tiles - r;
        return c;
    }
    // The other kernels with pieces.  On the three-per-unit 64 x 256 kernel halves (one or two per
    // unit in front) lose to quarter chains at every round count but two -- by 2 ... 5 points at five
    // to eight rounds, by 15 at three (65 % against 80 %), where the whole tiles fill their last
    // wave and the halves displace them; beside two rounds the halves win by 4 ... 6.
    const bool halves = !(v.est_wg_per_cu >= 3 && v.max_split >= 4) || R == 0 || R == 2;
    if (halves) take(rounds_of(2) / e2, r, 0, 0);
    // Thirds only beside at most one round of whole tiles (kernels without eighths have none today).
    if (v.thirds && 3 * r <= kComputeUnits && n_tiles < 2 * kComputeUnits) take(0.375 / e3, 0, r, 0);
    if (v.max_split >= 4) take(rounds_of(4) / e4, 0, 0, r);
    if (c.pieces() > 0) c.n_whole = n_tiles - r;
    return c;
}

// Cost of a variant: tiles are dealt to 256 compute units, a unit works through
// its tiles one tile-time after another (co-resident workgroups share the
// matrix pipe, they do not add to it), and a tile costs its full area even
// when it hangs over the edge of the output matrix (Section 3.3's point about
// credit for unnecessary work).  The last, partial round costs what
// choose_cut() makes of it.
double variant_cost(const mdnn::VariantInfo& v, int No, int64_t M)
{
    const int64_t tiles = (int64_t)div_up(No, v.tile_o) * div_up(M, v.tile_m);
    if (tiles > ((int64_t)1 << 26)) return 1e300;
    const Cut cut = choose_cut(v, (int)tiles);
    const int n_whole = cut.n_whole;
    const double rounds = (double)(tiles / kComputeUnits) + cut.cost;
    // Which of the two measured efficiencies applies.  Tiles that hold two workgroups per unit: "few"
    // means fewer than 4 7/8 rounds.  Tiles that hold three or more: more than two rounds count as
    // many.  Exception for three per unit: when the whole tiles fill the 768 slots once and a part
    // of them a second time (up to 1248) with fewer than one piece per unit in front of them, the
    // tiles beyond the first wave land wherever slots free first, two on one unit while others
    // idle.  128x128: 73-82 % at 992 ... 1120 tiles against 93 % at 768, at 1088 with 256 pieces in
    // front (with 224 it is 75 ... 83 % on three families and 90 % on two), and from 1248 on;
    // 96x128: 91 % at 768 tiles, 74 % at 1024.  (The small tiles at four
    // and more per unit show no such dip: 32x128 follows plain rounds of 256.)
    const int64_t n_pieces = cut.pieces();
    double eff;
    if (v.est_wg_per_cu >= 3) {
        const int64_t slots = 3 * kComputeUnits;
        // (one piece per unit in front was measured to cure it on the 128 x 128 kernel only: the
        // 64 x 256 kernel with 320 quarter pieces in front of 1024 whole tiles still runs at 72 %)
        const bool partial_second_wave = v.est_wg_per_cu == 3 && n_whole > slots && 8 * (int64_t)n_whole < 13 * slots &&
                                         (n_pieces < kComputeUnits || v.max_split < 8);
        eff = tiles <= 2 * kComputeUnits ? v.eff_few : v.eff;
        if (partial_second_wave) eff = 0.82 * v.eff_few;
        // Whole tiles that fill their last wave of 768 exactly leave no room for the tail pieces
        // (see choose_cut()): up to six rounds the two-per-unit kernel is the steadier choice
        // (three or six rounds + 24 ... 48 tiles: 86 ... 88.5 % against 89.5 ... 91 %).
        const int64_t R = tiles / kComputeUnits;
        if (v.est_wg_per_cu == 3 && n_pieces > 0 && R % 3 == 0 && R <= 6) eff *= 0.985;
    } else {
        eff = 8 * tiles < 39 * kComputeUnits ? v.eff_few : v.eff;
    }
    return rounds * v.tile_o * v.tile_m / eff;
}

int find_variant(const char* name);

int choose(int Nb, int No, int64_t M, int64_t K)
{
    // Output-bound layers (a contraction of a few dozen terms: 54 FLOPs per 4 bytes written at
    // K = 27) want long contiguous pieces of every output row per tile and many waves in flight,
    // not matrix-core efficiency: the 64 x 512 tile (3 -> 64 channels at 224 x 224: 41 -> 45.6 %
    // of the matrix peak, which is 5.1 TB/s written).
    if (K <= kWideTileMaxK && No > 32 && Nb % 4 == 0 && No % 4 == 0 && M >= 512 * 2 * kComputeUnits) {
        const int wide = find_variant("o64m512");
        if (wide >= 0) return wide;
    }
    int    best = -1;
    double best_cost = 0;
    for (int i = 0; i < mdnn::variant_count(); ++i) {
        const mdnn::VariantInfo& v = mdnn::variant_info(i);
        if (!variant_usable(v, Nb, No)) continue;
        // 4-byte copies only where 16-byte ones cannot be used.  (With one size off the multiple of 4
        // the tiles that copy both operands 4 bytes at a time stay in the race: they are rated lower,
        // but the small one among them is the only small tile such a layer has.)
        if (Nb % 4 == 0 && No % 4 == 0 && !(v.vec_a && v.vec_b)) continue;
        if ((!v.vec_a && v.vec_b && No % 4 == 0) || (v.vec_a && !v.vec_b && Nb % 4 == 0)) continue;
        const double c = variant_cost(v, No, M);
        if (best < 0 || c < best_cost) { best = i; best_cost = c; }
    }
    return best;
}

int find_variant(const char* name)
{
    for (int i = 0; i < mdnn::variant_count(); ++i)
        if (std::strcmp(name, mdnn::variant_info(i).name) == 0) return i;
    return -1;
}

// Everything about a launch that does not depend on the pointers or alpha.
mdnn_status plan(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad,
                 const char* variant, mdnn::ConvParams* out, int* variant_index)
{
    Geometry g;
    const mdnn_status gs = check_geometry(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &g);
    if (gs != MDNN_OK) return gs;
    int  v;
    char force_cut = 0;
    if (!variant || !variant[0] || std::strcmp(variant, "auto") == 0) {
        v = choose(Nb, No, g.M, g.K);
    } else {
        // "name" or "name:c" with c one of w h t q e m n p H T Q E (see choose_cut)
        char name[32];
        const char* colon = std::strchr(variant, ':');
        const size_t len = colon ? (size_t)(colon - variant) : std::strlen(variant);
        if (len >= sizeof(name)) return MDNN_EINVAL;
        std::memcpy(name, variant, len);
        name[len] = 0;
        if (colon) {
            if (!colon[1] || colon[2] || !std::strchr("whtqemnpHTQE", colon[1])) return MDNN_EINVAL;
            force_cut = colon[1];
        }
        v = find_variant(name);
        if (v >= 0 && !variant_usable(mdnn::variant_info(v), Nb, No)) v = -1;
    }
    if (v < 0) return MDNN_EINVAL;
    const mdnn::VariantInfo& vi = mdnn::variant_info(v);

    mdnn::ConvParams p;
    p.in = nullptr;  p.filt = nullptr;  p.out = nullptr;
    p.Nb = Nb;  p.Wi = Wi;  p.Hi = Hi;  p.Nc = Nc;  p.No = No;
    p.Sk = Sk;  p.stride = stride;  p.pad = pad;
    p.Wo = g.Wo;  p.Ho = g.Ho;
    p.K = (int)g.K;  p.SkSk = Sk * Sk;  p.M = (int)g.M;
    division_magic((uint32_t)p.SkSk, &p.sksk_magic, &p.sksk_shift);
    division_magic((uint32_t)Sk, &p.sk_magic, &p.sk_shift);
    division_magic((uint32_t)Nb, &p.nb_magic, &p.nb_shift);
    division_magic((uint32_t)g.Wo, &p.wo_magic, &p.wo_shift);
    p.n_otiles = div_up(No, vi.tile_o);
    p.n_mtiles = div_up(g.M, vi.tile_m);
    const int64_t n_tiles = (int64_t)p.n_otiles * p.n_mtiles;
    if (n_tiles > ((int64_t)1 << 26)) return MDNN_ETOOBIG;
    p.n_tiles = (int)n_tiles;
    const Cut cut = choose_cut(vi, p.n_tiles, force_cut);
    if (cut.n_whole < 0) return MDNN_EINVAL;                  // this kernel cannot cut a tile that way
    p.n_whole = cut.n_whole;
    p.n_half = cut.n_half;  p.n_third = cut.n_third;  p.n_quarter = cut.n_quarter;  p.n_eighth = cut.n_eighth;
    p.n_pieces = cut.pieces();
    // Pieces go last, where the dispatcher deals them to whichever units free up first -- except
    // up to one per unit, which go FIRST.  A piece launched last runs alone on its unit, and a lone
    // small workgroup leaves the matrix pipe idle during every other instruction; launched first it
    // shares the unit with whole tiles, and the launch ends with whole tiles finishing together
    // (measured: +0.8 % on the 3x3 256-channel layer, +1 ... +3.4 % on layers with two to six rounds
    // of tiles; -0.6 % with a single round of whole tiles, hence the condition).  The largest
    // pieces are the ones that go first.
    {
        const int total[4] = {2 * p.n_half, 3 * p.n_third, 4 * p.n_quarter, 8 * p.n_eighth};
        int room = cut.pair_up ? 2 * kComputeUnits : p.n_whole >= 2 * kComputeUnits ? kComputeUnits : 0;
        for (int c = 0; c < 4; ++c) {
            const int f = std::min(total[c], room);
            room -= f;
            p.front.begin[c] = 0;         p.front.count[c] = f;            p.front.per_xcd[c] = div_up(f, 8);
            p.back.begin[c] = f;          p.back.count[c] = total[c] - f;  p.back.per_xcd[c] = div_up(total[c] - f, 8);
        }
        for (mdnn::ConvParams::PieceRegion* r : {&p.front, &p.back}) {
            r->wgs = 8 * (r->per_xcd[0] + r->per_xcd[1] + r->per_xcd[2] + r->per_xcd[3]);
            r->pieces = r->count[0] + r->count[1] + r->count[2] + r->count[3];
        }
    }
    p.tiles_per_xcd = div_up(p.n_whole, 8);
    // 2-D visiting order of the column tiles (see ConvParams): needs tiles aligned with pixel rows
    p.row_tiles = 0;
    p.strip_rows = 1;
    {
        const int64_t row_cols = (int64_t)g.Wo * Nb;             // flat columns per row of pixels
        const bool whole_pixels = (vi.tile_m % Nb == 0) || (Nb % vi.tile_m == 0);
        if (whole_pixels && row_cols % vi.tile_m == 0 && g.Ho > 1 && Sk > stride) {
            p.row_tiles = (int)(row_cols / vi.tile_m);
            p.strip_rows = g.Ho < kStripRows ? g.Ho : kStripRows;
        }
    }
    const int kpad = div_up(g.K, vi.kslab) * vi.kslab;
    p.tab_cap = kpad < vi.max_tab ? kpad : vi.max_tab;
    p.scat_stride = 0;  p.scat_Nc = 0;  p.scat_Hi = 0;  p.scat_Wi = 0;  p.scat_pad = 0;
    p.stream_out = (g.K <= kStreamOutMaxK || g.out_bytes >= kStreamOutMinBytes) ? 1 : 0;
    p.in_bytes = (uint32_t)g.in_bytes;
    p.filt_bytes = (uint32_t)g.filt_bytes;
    p.alpha = 0.0f;
    *out = p;
    *variant_index = v;
    return MDNN_OK;
}

}  // namespace

extern "C" {

mdnn_status mdnn_out_dims(int Wi, int Hi, int Sk, int stride, int pad, int* Wo, int* Ho)
{
    if (!Wo || !Ho) return MDNN_ENULL;
    Geometry g;
    // Nb = Nc = No = 1: only the spatial geometry matters here
    const mdnn_status s = check_geometry(1, Wi, Hi, 1, 1, Sk, stride, pad, &g);
    if (s != MDNN_OK) return s;
    *Wo = g.Wo;
    *Ho = g.Ho;
    return MDNN_OK;
}

uint64_t mdnn_conv_flops(int Nb, int Wo, int Ho, int Nc, int No, int Sk)
{
    if (Nb < 1 || Wo < 1 || Ho < 1 || Nc < 1 || No < 1 || Sk < 1) return 0;
    const uint64_t macs_per_output = (uint64_t)Nc * (uint64_t)Sk * (uint64_t)Sk + 1u;
    const uint64_t outputs = (uint64_t)Nb * (uint64_t)Wo * (uint64_t)Ho * (uint64_t)No;
    return 2u * outputs * macs_per_output;
}

const char* mdnn_status_string(mdnn_status s)
{
    // a C caller may pass any int: read the bits without going through the enumeration's value range
    int code;
    std::memcpy(&code, &s, sizeof code);
    switch (code) {
        case MDNN_OK:      return "ok";
        case MDNN_EINVAL:  return "invalid argument (dimension, stride, pad, alpha or variant name)";
        case MDNN_ENULL:   return "null pointer";
        case MDNN_EALIGN:  return "tensor pointer not 16-byte aligned";
        case MDNN_ETOOBIG: return "tensor of 4 GiB or more";
        case MDNN_ELAUNCH: return "kernel launch failed";
    }
    return "unknown status";
}

int mdnn_variant_count(void) { return mdnn::variant_count(); }

const char* mdnn_variant_name(int i)
{
    if (i < 0 || i >= mdnn::variant_count()) return nullptr;
    return mdnn::variant_info(i).name;
}

const char* mdnn_choose_variant(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad)
{
    Geometry g;
    if (check_geometry(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &g) != MDNN_OK) return nullptr;
    const int v = choose(Nb, No, g.M, g.K);
    return v < 0 ? nullptr : mdnn::variant_info(v).name;
}

mdnn_status mdnn_conv_fprop_variant(const float* in, const float* filt, float* out,
                                    int Nb, int Wi, int Hi, int Nc, int No,
                                    int Sk, int stride, int pad, float alpha,
                                    void* stream, const char* variant)
{
    if (!in || !filt || !out) return MDNN_ENULL;
    mdnn::ConvParams p;
    int v = -1;
    const mdnn_status ps = plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant, &p, &v);
    if (ps != MDNN_OK) return ps;
    if (!std::isfinite(alpha)) return MDNN_EINVAL;
    if (((uintptr_t)in | (uintptr_t)filt | (uintptr_t)out) & 15u) return MDNN_EALIGN;
    p.in = in;  p.filt = filt;  p.out = out;
    p.alpha = alpha;
    return mdnn::launch_variant(v, p, stream) == 0 ? MDNN_OK : MDNN_ELAUNCH;
}

mdnn_status mdnn_describe_launch(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad,
                                 const char* variant, char* text, size_t text_size)
{
    if (!text || text_size == 0) return MDNN_ENULL;
    mdnn::ConvParams p;
    int v = -1;
    const mdnn_status ps = plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, variant, &p, &v);
    if (ps != MDNN_OK) { text[0] = 0; return ps; }
    const mdnn::VariantInfo& vi = mdnn::variant_info(v);
    std::snprintf(text, text_size,
                  "variant=%s tile=%dx%d kslab=%d threads=%d K=%d M=%d tiles=%d whole=%d split=%d "
                  "halved=%d thirded=%d quartered=%d eighthed=%d pieces=%d "
                  "pieces_first=%d grid=%d lds_bytes=%u table_entries=%d",
                  vi.name, vi.tile_o, vi.tile_m, vi.kslab, vi.threads, p.K, p.M, p.n_tiles, p.n_whole,
                  // split: pieces per cut tile when all are cut alike (1 = none is cut), 0 = a mixture
                  p.n_pieces == 0 ? 1 : p.n_pieces == 2 * p.n_half ? 2 : p.n_pieces == 3 * p.n_third ? 3
                                    : p.n_pieces == 4 * p.n_quarter ? 4 : p.n_pieces == 8 * p.n_eighth ? 8 : 0,
                  p.n_half, p.n_third, p.n_quarter, p.n_eighth, p.n_pieces, p.front.pieces,
                  p.front.wgs + 8 * p.tiles_per_xcd + p.back.wgs,
                  mdnn::variant_lds_bytes(v, p.tab_cap), p.tab_cap);
    return MDNN_OK;
}

mdnn_status mdnn_conv_fprop(const float* in, const float* filt, float* out,
                            int Nb, int Wi, int Hi, int Nc, int No,
                            int Sk, int stride, int pad, float alpha, void* stream)
{
    return mdnn_conv_fprop_variant(in, filt, out, Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha,
                                   stream, nullptr);
}

// c (N x M) = alpha * a^T b: the 1 x 1, stride-1, unpadded convolution of one pixel of M images
// with K channels and N filters.
mdnn_status mdnn_sgemm_tn(const float* a, const float* b, float* c,
                          int N, int M, int K, float alpha, void* stream)
{
    return mdnn_conv_fprop_variant(b, a, c, /*Nb*/ M, /*Wi*/ 1, /*Hi*/ 1, /*Nc*/ K, /*No*/ N,
                                   /*Sk*/ 1, /*stride*/ 1, /*pad*/ 0, alpha, stream, nullptr);
}

namespace {

// Geometry of the forward convolution whose stride-1 run yields the data gradient.
// stride 1, pad <= Sk - 1: the turned-over bank (K' = No*Sk*Sk rows, Nc columns), pad Sk-1-pad, written to din.
// otherwise: T = ceil(Sk/s); the residue-class bank (No*T*T rows, s*s*Nc columns), pad T-1, over a grid
//           of (Ho+T-1) x (Wo+T-1) pixels per class, scattered into din by the kernel's epilogue.
struct BpropPlan {
    bool      direct;          // the first of the two forms
    int       T;               // taps per side of the transposed problem (Sk for the direct form)
    int       filters_t;       // its filter count (Nc, or s*s*Nc)
    int       pad_t;           // its pad
    int       He, We;          // its output extent (Hi x Wi for the direct form)
    size_t    bank_bytes;      // rearranged filter bank
    size_t    total_bytes;     // workspace: the bank, rounded up to 256 bytes
};

mdnn_status bprop_plan(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad, BpropPlan* b)
{
    Geometry g;
    const mdnn_status gs = check_geometry(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &g);
    if (gs != MDNN_OK) return gs;
    // Stride 1 with pad <= Sk - 1 is one forward convolution with pad Sk - 1 - pad.  A larger pad
    // would make that pad negative: such layers take the general form (one residue class, the
    // full correlation, of which the epilogue keeps what lies inside din), like every stride > 1.
    if (stride == 1 && pad <= Sk - 1) {
        b->direct = true;
        b->T = Sk;  b->filters_t = Nc;  b->pad_t = Sk - 1 - pad;
        b->He = Hi;  b->We = Wi;
        b->bank_bytes = (size_t)g.filt_bytes;
        b->total_bytes = (b->bank_bytes + 255) & ~(size_t)255;
        return MDNN_OK;
    }
    const int T = (int)(((int64_t)Sk + stride - 1) / stride);
    if ((int64_t)stride * stride >= ((int64_t)1 << 24)) return MDNN_ETOOBIG;      // (keeps the next product in range)
    const int64_t filters_t = (int64_t)stride * stride * Nc;
    if (filters_t >= ((int64_t)1 << 24)) return MDNN_ETOOBIG;
    b->direct = false;
    b->T = T;  b->filters_t = (int)filters_t;  b->pad_t = T - 1;
    b->He = g.Ho + T - 1;  b->We = g.Wo + T - 1;
    const int64_t bank_bytes = 4 * (int64_t)No * T * T * filters_t;
    // the per-class grid is only ever a column index of the kernel: it has to stay below 2^31 columns
    const int64_t columns = (int64_t)b->He * b->We * Nb;
    if (bank_bytes >= kFourGiB / 2 || columns * 4 >= kFourGiB) return MDNN_ETOOBIG;
    b->bank_bytes = (size_t)bank_bytes;
    b->total_bytes = (b->bank_bytes + 255) & ~(size_t)255;
    return MDNN_OK;
}

// Filter gradient: 128-row tiles of the K x No result, the contraction over m = (y,x,n) cut into
// `splits` ranges so that the launch fills the chip.
mdnn_status filter_grad_plan(int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad,
                             mdnn::FilterGradParams* f, size_t* workspace_bytes)
{
    Geometry g;
    const mdnn_status gs = check_geometry(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &g);
    if (gs != MDNN_OK) return gs;
    mdnn::FilterGradParams p;
    p.in = nullptr;  p.dout = nullptr;  p.part = nullptr;
    p.Nb = Nb;  p.Wi = Wi;  p.Hi = Hi;  p.Nc = Nc;  p.No = No;
    p.Sk = Sk;  p.stride = stride;  p.pad = pad;
    p.Wo = g.Wo;  p.Ho = g.Ho;
    p.K = (int)g.K;  p.SkSk = Sk * Sk;  p.M = (int)g.M;
    division_magic((uint32_t)p.SkSk, &p.sksk_magic, &p.sksk_shift);
    division_magic((uint32_t)Sk, &p.sk_magic, &p.sk_shift);
    division_magic((uint32_t)Nb, &p.nb_magic, &p.nb_shift);
    division_magic((uint32_t)g.Wo, &p.wo_magic, &p.wo_shift);
    // tile width: the least padded matrix work, narrower tiles rated a little slower per useful FLOP
    {
        const int   widths[4] = {128, 96, 64, 32};
        const float speed[4]  = {1.00f, 0.97f, 0.90f, 0.70f};
        float best = 0.f;
        p.tile_o = 128;
        for (int i = 0; i < 4; ++i) {
            const float cost = (float)(div_up(No, widths[i]) * widths[i]) / speed[i];
            if (best == 0.f || cost < best) { best = cost; p.tile_o = widths[i]; }
        }
    }
    p.n_otiles = div_up(No, p.tile_o);
    const int64_t n_tiles = (int64_t)div_up(g.K, 128) * p.n_otiles;
    if (n_tiles > ((int64_t)1 << 24)) return MDNN_ETOOBIG;
    p.n_tiles = (int)n_tiles;

    // How many ranges.  Workgroups are dealt evenly to the 256 compute units and a unit works
    // through its share at the matrix rate however many of them are resident at once (up to three
    // fit by LDS and registers), so a choice costs
    //     ceil(tiles * ranges / 256) * slabs per range,
    // a little more when fewer than three are resident (less latency hidden; measured), plus the
    // summing kernel's reads of one partial gradient per range at about 3.5 bytes/ns.  Measured on
    // the 5x5 layer with 38 tiles: 13 ranges (494 workgroups) 88 %, 14 (532) 64 %, 20 (760) 90 %,
    // 27 (1026) 73 %, 40 (1520) 88 %, as this model predicts.
    const int64_t slabs = (g.M + 15) / 16;
    const int64_t kMinSlabs = 8;
    const int64_t s_max = std::max<int64_t>(1, slabs / kMinSlabs);
    const int64_t s_cap = std::min<int64_t>(s_max, std::max<int64_t>(1, (12 * 256) / n_tiles + 1));
    // (a lone 96-wide workgroup per unit hides less: the 11x11 first layer with 96 filters runs at
    // 80.9 % of peak in 255 workgroups, 81.7 % in 510, 79.4 % in 765 with their larger partial sums)
    const double  rel_eff[3] = {p.tile_o == 96 ? 0.88 : 0.975, 0.99, 1.0};
    const double  n_bytes = (double)g.K * (double)No * 4.0;
    const double  slab_us = 0.85 * (double)p.tile_o / 128.0;
    const bool    small_gradient = g.K * (int64_t)No < ((int64_t)1 << 18);
    int64_t best_s = 1;
    double  best_cost = -1.0;
    for (int64_t s = 1; s <= s_cap; ++s) {
        const int64_t per    = (slabs + s - 1) / s;
        const int64_t real   = (slabs + per - 1) / per;            // ranges actually needed
        const int64_t per_cu = (n_tiles * real + 255) / 256;       // workgroups on the busiest unit
        // in microseconds: a slab of a lone 128-wide workgroup takes 0.85, narrower ones in proportion;
        // the summing kernel for small gradients walks the ranges in chains (latency, not bytes)
        const double  main_us = (double)(per_cu * per) * slab_us / rel_eff[std::min<int64_t>(per_cu, 3) - 1];
        const double  sum_us  = 2.0 + (double)real * n_bytes / 3.5e6 + (small_gradient ? 0.02 * (double)real : 0.0);
        const double  cost    = main_us + sum_us;
        if (best_cost < 0 || cost < best_cost - 1e-9) { best_cost = cost; best_s = real; }
    }
    p.m_per_split = (int)(((slabs + best_s - 1) / best_s) * 16);
    p.splits = (int)((g.M + p.m_per_split - 1) / p.m_per_split);
    p.per_xcd = div_up((int64_t)p.n_tiles * p.splits, 8);
    p.vec = (Nb % 4 == 0) ? 1 : 0;
    p.uniform = (Nb % 16 == 0) ? 1 : 0;
    p.in_bytes = (uint32_t)g.in_bytes;
    p.dout_bytes = (uint32_t)g.out_bytes;
    *f = p;
    *workspace_bytes = (size_t)p.splits * (size_t)g.K * (size_t)No * sizeof(float);
    return MDNN_OK;
}

// The kernels of one data-gradient call, enqueued on `stream`; every argument has been checked.
mdnn_status bprop_data_enqueue(const BpropPlan& b, const float* dout, const float* filt, float* din, void* workspace,
                               int Nb, int Wi, int Hi, int Nc, int No, int Sk, int stride, int pad,
                               float alpha, void* stream)
{
    Geometry g;
    check_geometry(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &g);       // succeeded inside bprop_plan
    float* bank = static_cast<float*>(workspace);

    // the transposed problem: No input channels of Ho x Wo, b.filters_t filters of T x T, stride 1
    mdnn::ConvParams p;
    int v = -1;
    const mdnn_status ps = plan(Nb, g.Wo, g.Ho, No, b.filters_t, b.T, 1, b.pad_t, nullptr, &p, &v);
    if (ps != MDNN_OK) return ps;
    if (p.Ho != b.He || p.Wo != b.We) return MDNN_EINVAL;          // cannot happen: Ho + 2 pad_t - T + 1 == He

    p.in = dout;  p.filt = bank;  p.out = din;
    p.alpha = alpha;
    if (b.direct) {
        if (mdnn::launch_flip_transpose(filt, bank, Nc, No, Sk * Sk, stream) != 0) return MDNN_ELAUNCH;
        return mdnn::launch_variant(v, p, stream) == 0 ? MDNN_OK : MDNN_ELAUNCH;
    }
    if (mdnn::launch_class_filters(filt, bank, Nc, No, Sk, stride, b.T, stream) != 0) return MDNN_ELAUNCH;
    // pixels with (iy + pad) / stride >= He (or the same along x) belong to no class's grid
    const int64_t y_end = (int64_t)stride * b.He - pad, x_end = (int64_t)stride * b.We - pad;
    if (mdnn::launch_zero_unreached(din, Nc, Hi, Wi, Nb, (int)std::max<int64_t>(0, std::min<int64_t>(y_end, Hi)),
                                    (int)std::max<int64_t>(0, std::min<int64_t>(x_end, Wi)), stream) != 0)
        return MDNN_ELAUNCH;
    p.scat_stride = stride;  p.scat_Nc = Nc;  p.scat_Hi = Hi;  p.scat_Wi = Wi;  p.scat_pad = pad;
    return mdnn::launch_variant(v, p, stream) == 0 ? MDNN_OK : MDNN_ELAUNCH;
}

}  // namespace

mdnn_status mdnn_conv_bprop_filter_workspace(int Nb, int Wi, int Hi, int Nc, int No,
                                             int Sk, int stride, int pad, size_t* bytes)
{
    if (!bytes) return MDNN_ENULL;
    mdnn::FilterGradParams f;
    return filter_grad_plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &f, bytes);
}

mdnn_status mdnn_conv_bprop_filter(const float* in, const float* dout, float* dfilt,
                                   void* workspace, size_t workspace_bytes,
                                   int Nb, int Wi, int Hi, int Nc, int No,
                                   int Sk, int stride, int pad, float alpha, void* stream)
{
    if (!in || !dout || !dfilt || !workspace) return MDNN_ENULL;
    mdnn::FilterGradParams f;
    size_t need = 0;
    const mdnn_status fs = filter_grad_plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &f, &need);
    if (fs != MDNN_OK) return fs;
    if (!std::isfinite(alpha)) return MDNN_EINVAL;
    if (workspace_bytes < need) return MDNN_EINVAL;
    if (((uintptr_t)in | (uintptr_t)dout | (uintptr_t)dfilt | (uintptr_t)workspace) & 15u) return MDNN_EALIGN;
    f.in = in;  f.dout = dout;  f.part = static_cast<float*>(workspace);
    return mdnn::launch_bprop_filter(f, dfilt, alpha, stream) == 0 ? MDNN_OK : MDNN_ELAUNCH;
}

mdnn_status mdnn_conv_bprop_data_workspace(int Nb, int Wi, int Hi, int Nc, int No,
                                           int Sk, int stride, int pad, size_t* bytes)
{
    if (!bytes) return MDNN_ENULL;
    BpropPlan b;
    const mdnn_status s = bprop_plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &b);
    if (s != MDNN_OK) return s;
    *bytes = b.total_bytes;
    return MDNN_OK;
}

mdnn_status mdnn_conv_bprop_data(const float* dout, const float* filt, float* din,
                                 void* workspace, size_t workspace_bytes,
                                 int Nb, int Wi, int Hi, int Nc, int No,
                                 int Sk, int stride, int pad, float alpha, void* stream)
{
    if (!dout || !filt || !din || !workspace) return MDNN_ENULL;
    BpropPlan b;
    const mdnn_status bs = bprop_plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &b);
    if (bs != MDNN_OK) return bs;
    if (!std::isfinite(alpha)) return MDNN_EINVAL;
    if (workspace_bytes < b.total_bytes) return MDNN_EINVAL;
    if (((uintptr_t)dout | (uintptr_t)filt | (uintptr_t)din | (uintptr_t)workspace) & 15u) return MDNN_EALIGN;
    return bprop_data_enqueue(b, dout, filt, din, workspace, Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha, stream);
}

mdnn_status mdnn_conv_bprop_data_static(const float* dout, const float* filt, float* din,
                                        int Nb, int Wi, int Hi, int Nc, int No,
                                        int Sk, int stride, int pad, float alpha, void* stream)
{
    if (!dout || !filt || !din) return MDNN_ENULL;
    BpropPlan b;
    const mdnn_status bs = bprop_plan(Nb, Wi, Hi, Nc, No, Sk, stride, pad, &b);
    if (bs != MDNN_OK) return bs;
    if (!std::isfinite(alpha)) return MDNN_EINVAL;
    if (b.total_bytes > (size_t)MDNN_STATIC_SCRATCH_BYTES) return MDNN_ETOOBIG;
    if (((uintptr_t)dout | (uintptr_t)filt | (uintptr_t)din) & 15u) return MDNN_EALIGN;
    void* scratch = nullptr;
    if (mdnn::static_scratch(&scratch) != 0 || !scratch) return MDNN_ELAUNCH;
    return bprop_data_enqueue(b, dout, filt, din, scratch, Nb, Wi, Hi, Nc, No, Sk, stride, pad, alpha, stream);
}

mdnn_status mdnn_mfma_peak_probe(float* sink, int blocks, int waves_per_block, int iters,
                                 uint64_t* flops, void* stream)
{
    if (!sink) return MDNN_ENULL;
    if (blocks < 1 || blocks > (1 << 20) || waves_per_block < 1 || waves_per_block > 4 || iters < 1)
        return MDNN_EINVAL;
    // 4 MFMA 32x32x2 per iteration per wave, 2*32*32*2 FLOPs each
    if (flops) *flops = (uint64_t)blocks * waves_per_block * (uint64_t)iters * 4u * 4096u;
    return mdnn::launch_mfma_probe(sink, blocks, waves_per_block, iters, stream) == 0 ? MDNN_OK
                                                                                      : MDNN_ELAUNCH;
}

}  // extern "C"
