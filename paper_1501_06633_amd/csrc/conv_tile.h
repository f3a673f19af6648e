// The FPROP convolution tile for gfx950 (MI355X): implicit GEMM on the FP32 matrix
// cores.  This header holds the kernel template; the translation units
// conv_variants_*.hip instantiate the tile shapes, conv_fprop.hip collects them.
//
// The output [No][Ho][Wo][Nb] is a row-major No x M matrix with
// M = Ho*Wo*Nb, and (maxDNN paper, Section 3) for each output coordinate its
// Nb columns are  filter-matrix^T (No x K)  times  patch (K x Nb),  K = Nc*Sk*Sk.
// A workgroup owns a TO x TM tile of that matrix: TO output filters by TM
// consecutive flat columns m = (y*Wo + x)*Nb + n, i.e. one output coordinate
// when TM == Nb, several when Nb is smaller (Section 3.2 uses one 64x64
// filter-image block per coordinate; Section 3.4 asks for other block sizes).
//
// Both GEMM operands are k-major with the lane-varying dimension contiguous in
// memory (filter row k = No consecutive floats, patch row k = Nb consecutive
// floats per coordinate), which is exactly what v_mfma_f32_32x32x2_f32 wants:
// lanes 0-31 carry the 32 rows (or columns) at k, lanes 32-63 the same at k+1.
// So global -> LDS is a straight row copy, LDS -> VGPR a read of consecutive
// floats, and nothing is ever transposed.  Filters sit on the MFMA rows and
// the flat column m on the MFMA columns, so the lane index of the result is
// the contiguous output index and stores are coalesced without a shuffle
// through LDS (the paper's Section 3.1 needs one).
//
// Gather (Section 3.2): the K patch-column offsets (c,ky,kx) -> byte offset
// are computed once per tile into an LDS table; an input address is
// patch base + table[k].  The image is not physically padded: a tap in the
// zero apron gets an out-of-range buffer offset, for which the hardware
// returns 0, so the inner loop has no boundary branch.
//
// Pipeline (the paper's Section 3.1 double buffering, re-cut for CDNA4):
// operand slabs of KS patch columns go global -> LDS directly
// (buffer_load ... lds, no staging registers) into a ring of NS stages, NS-1
// slabs ahead of the MFMAs; one workgroup barrier per slab; the LDS -> VGPR
// fragment reads run one MFMA k-step ahead of their use.  LDS reads inside the
// loop are issued through inline asm with hand-counted s_waitcnt: the compiler
// would otherwise drain every outstanding global -> LDS copy (vmcnt(0)) before
// each LDS read, which defeats the ring.
//
// What shapes the loop: on this chip a wave's MFMAs do not overlap that wave's
// other VALU/SALU instructions -- each one costs 4-5 matrix cycles (LDS reads
// are free) -- so the slab loop carries about twenty bookkeeping instructions
// per 32 MFMAs: incremental filter offsets, one add per patch copy, LDS
// addresses as immediates, no scalar tests in the steady state.
#ifndef MDNN_CONV_TILE_H_
#define MDNN_CONV_TILE_H_

#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "gfx950_util.h"
#include "mdnn_internal.h"

namespace mdnn {

namespace {

// How a wave treats taps that fall into the zero apron (chosen per tile and per wave):
constexpr int kTapNone = 0;   // none of the wave's patches touches the apron: no test at all
constexpr int kTapMask = 1;   // Sk*Sk <= 32: per-thread bit mask of apron taps, table carries the tap index
constexpr int kTapTest = 2;   // any Sk: table carries (ky,kx), two range compares per copy

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef f32x2 type; };
template <> struct VecOf<4> { typedef f32x4 type; };
template <class V> __device__ __forceinline__ float comp(const V& v, int i)
{
    if constexpr (sizeof(V) == sizeof(float)) return v;
    else return v[i];
}

// WO x WM waves per workgroup; each wave owns RA x RB matrix blocks of MB x MB
// (MB = 32: v_mfma_f32_32x32x2_f32, two k per instruction; MB = 16:
// v_mfma_f32_16x16x4_f32, four k per instruction -- the same FLOPs per cycle,
// half the block edge, which is what tile heights of 48 rows need); KS patch
// columns per slab; NS LDS stages; VW floats per global access: 4 or 1 for both
// operands, 14 = 4-byte filter copies and 16-byte patch copies (a filter count
// that is no multiple of 4), 41 = the other way round (such a minibatch).
template <int WO_, int WM_, int RA_, int RB_, int KS_, int NS_, int VW_, int JB_ = 2, int MB_ = 32>
struct Cfg {
    static constexpr int WO = WO_, WM = WM_, RA = RA_, RB = RB_, KS = KS_, NS = NS_, VW = VW_;
    static constexpr int JB = JB_;                    // k-step of a slab in front of which the barrier sits
    static constexpr int MB = MB_;                    // edge of a matrix block
    static constexpr int KB = 64 / MB;                // k consumed by one matrix instruction
    static constexpr int NT = 64 * WO * WM;           // threads
    static constexpr int TO = WO * RA * MB;           // tile rows (filters)
    static constexpr int TM = WM * RB * MB;           // tile columns (flat m)
    static constexpr int VWA = (VW == 4 || VW == 41) ? 4 : 1;   // floats per filter copy
    static constexpr int VWB = (VW == 4 || VW == 14) ? 4 : 1;   // floats per patch copy (and whether M is a multiple of 4)
    static constexpr int OG = TO / VWA;               // accesses per filter-slab row
    static constexpr int A_EL = KS * OG;              // accesses per filter slab
    static constexpr int NA = (A_EL + NT - 1) / NT;   // filter accesses per thread per slab
    static constexpr int MG = TM / VWB;               // accesses per patch-slab row
    static constexpr int BROWS = NT / MG;             // patch rows one pass of the workgroup covers
    static constexpr int NB = KS / BROWS;             // patch accesses per thread per slab
    // global -> LDS copies every wave issues per slab (waves past the end of a
    // short filter slab skip their filter copy, so only full passes count); the
    // vmcnt waits are phrased in these, which is exact for most tiles and merely
    // a little early for the waves that issue one more
    static constexpr int NL = A_EL / NT + NB;
    static constexpr int STAGE_FLOATS = KS * (TO + TM);
    static constexpr uint32_t ring_bytes = (uint32_t)NS * STAGE_FLOATS * sizeof(float);
    static_assert(VW == 1 || VW == 4 || VW == 14 || VW == 41, "VW");
    static_assert(MB == 32 || MB == 16, "MB");
    static_assert(NT % MG == 0 && KS % BROWS == 0 && KS % KB == 0, "tile shape");
    static_assert(A_EL % 32 == 0, "the filter copy masks off whole waves and, in the last wave that copies, the upper lanes");
    static_assert(RB == 1 || RB == 2 || RB == 4, "RB");
    static_assert(RA >= 1 && RA <= 4, "RA");
    // NS >= 3: slab s+1 must already be in flight when slab s reaches its barrier
    static_assert(NS >= 3 && (NS - 2) * NL <= 63, "ring depth / vmcnt range");
};

// One TO x TM output tile.  `lds` is the workgroup's dynamic LDS: ring, then table.
// CONTEXT only tells apart instantiations of one shape reached from different
// kernels (a quarter of the 128x128 tile is the 32x128 tile): hipcc's host pass
// rejects the second use of an identical specialisation of this function.
template <class C, int CONTEXT = 0>
__device__ __forceinline__ void conv_tile(const ConvParams& p, unsigned char* lds, const int o0, const int m0)
{
    constexpr int WO = C::WO, RA = C::RA, RB = C::RB, KS = C::KS, NS = C::NS, VWA = C::VWA, VWB = C::VWB;
    constexpr int MB = C::MB, KB = C::KB;
    constexpr int NV = MB * MB / 64;  // accumulator registers per matrix block
    typedef typename std::conditional<MB == 32, f32x16, f32x4>::type Acc;
    constexpr int NT = C::NT, TO = C::TO, TM = C::TM, OG = C::OG, MG = C::MG;
    constexpr int NA = C::NA, NB = C::NB, BROWS = C::BROWS, NL = C::NL;
    constexpr int STAGE_BYTES = C::STAGE_FLOATS * 4;
    constexpr int ACCESS_A = 4 * VWA, ACCESS_B = 4 * VWB;    // bytes per lane per global -> LDS copy
    typedef typename VecOf<RB>::type BVec;

    // A tile's start-up (column set-up, offset table, first copies) issues ahead of the older
    // workgroups' slab loops on the same SIMDs, which otherwise leave a young wave only the issue
    // cycles they do not use (a fifth of a tile's time passed before its first matrix instruction);
    // the priority drops back once the first slab is there.  +0.5 ... 1.2 % where K is a few hundred.
    __builtin_amdgcn_s_setprio(3);
    u32x2* tab = reinterpret_cast<u32x2*>(lds + C::ring_bytes);   // [tab_cap] {byte offset, tap id}
    const uint32_t lds_base = (uint32_t)(uintptr_t)LDS_PTR(lds);
    const uint32_t tab_base = lds_base + C::ring_bytes;

    const int t    = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wo   = wave % WO;
    const int wm   = wave / WO;
    const int kg   = lane / MB;      // which k of a matrix instruction's KB this lane supplies
    const int lb   = lane % MB;      // its row (filter operand) / column (patch operand) in the block

    const __amdgpu_buffer_rsrc_t rin =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.in), 0, (int)p.in_bytes, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rfl =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.filt), 0, (int)p.filt_bytes, kRsrcWord3);

    // ---- this thread's patch column group (VW adjacent columns, one output
    // coordinate because VW divides Nb): fixed for the whole tile.
    const int q    = t % MG;
    const int brow = t / MG;
    uint32_t  pbase;                  // byte offset of the patch origin (+n) in `in`, modulo 2^32
    int       iy0, ix0;               // image row/col of tap (0,0); far negative when the column is past M
    bool      col_inside;             // every tap of this column's patch lies inside the image
    {
        const int m = m0 + VWB * q;
        if (m < p.M) {
            const int pix = (int)fast_div((uint32_t)m, p.nb_magic, p.nb_shift);
            const int n   = m - pix * p.Nb;
            const int y   = (int)fast_div((uint32_t)pix, p.wo_magic, p.wo_shift);
            const int x   = pix - y * p.Wo;
            iy0 = y * p.stride - p.pad;
            ix0 = x * p.stride - p.pad;
            // modulo 2^32 on purpose: a negative apron origin wraps, and wraps back once a valid tap is added
            pbase = (((uint32_t)iy0 * (uint32_t)p.Wi + (uint32_t)ix0) * (uint32_t)p.Nb + (uint32_t)n) * 4u;
            col_inside = (iy0 >= 0) & (iy0 + p.Sk <= p.Hi) & (ix0 >= 0) & (ix0 + p.Sk <= p.Wi);
        } else {
            iy0 = -(1 << 30);
            ix0 = -(1 << 30);
            pbase = 0;
            col_inside = false;
        }
    }
    // Waves whose patches never touch the apron (most of them) take a loop
    // without the per-tap boundary test.  The choice only changes how a lane
    // forms its own copy offsets; barriers and counts are the same in every
    // mode, so it can differ from wave to wave.
    const bool interior = (__builtin_amdgcn_ballot_w64(col_inside) == __builtin_amdgcn_ballot_w64(true));
    const bool small_filter = (p.SkSk <= 32);
    uint32_t   apron_taps = 0;        // bit r set: tap r = ky*Sk + kx of this thread's patch is in the apron
    if (!interior && small_filter) {
        int ky = 0, kx = 0;
        for (int r = 0; r < p.SkSk; ++r) {
            const bool ok = ((uint32_t)(iy0 + ky) < (uint32_t)p.Hi) & ((uint32_t)(ix0 + kx) < (uint32_t)p.Wi);
            apron_taps |= (ok ? 0u : 1u) << r;
            if (++kx == p.Sk) { kx = 0; ++ky; }
        }
    }

    Acc acc[RA][RB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int v = 0; v < NV; ++v) acc[a][b][v] = 0.0f;

    // ---- global -> LDS copies.  Copy i of a slab covers accesses e = t + i*NT
    // of the row-major slab, so a wave's 64 lanes fill 64 consecutive slots of
    // LDS: what a global -> LDS load does (LDS address = wave-uniform base +
    // lane * size).  Every instruction issued inside the MFMA loop costs matrix
    // issue slots, so the per-slab address work is one add per copy.
    //
    // Filter slab: rows k0..k0+KS-1, columns o0..o0+TO-1 of the K x No matrix.
    // No predicate: a row k >= K lies beyond the end of the buffer and reads as
    // 0 (which also silences whatever the patch slab holds in that row), and a
    // column o >= No only feeds output rows that are never stored.
    uint32_t voffA[NA];
#pragma unroll
    for (int i = 0; i < NA; ++i) {
        const int e = t + i * NT;
        const int r = e / OG;
        const int c = e - r * OG;
        voffA[i] = ((uint32_t)r * (uint32_t)p.No + (uint32_t)(o0 + VWA * c)) * 4u;
    }
    const uint32_t strideA = (uint32_t)KS * (uint32_t)p.No * 4u;
    unsigned char* const dma_base_a = lds + wave * (64 * ACCESS_A);           // wave-uniform
    unsigned char* const dma_base_b = lds + wave * (64 * ACCESS_B);
    auto issue_A = [&](auto stc) {
        constexpr int st = decltype(stc)::value;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            if ((C::A_EL % NT) != 0 && wave * 64 + i * NT >= C::A_EL) continue;   // wave-uniform
            if (C::A_EL % 64 != 0 && wave * 64 + i * NT + lane >= C::A_EL) continue;   // last wave of the slab: lower lanes only
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rfl, LDS_PTR(dma_base_a + (st * STAGE_BYTES + i * NT * ACCESS_A)), C::VWA * 4,
                (int)voffA[i], 0, 0, 0);
            voffA[i] += strideA;
        }
    };
    // Patch slab: row k of the unrolled patch for this thread's columns, address
    // = patch base + table[k]; a tap in the apron gets an out-of-range offset
    // and reads as 0.  Table rows k >= K hold offset 0: they fetch finite data
    // (or 0) that meets a zero filter row.
    auto issue_B = [&](auto stc, auto modec, const u32x2 (&ent)[NB]) {
        constexpr int st   = decltype(stc)::value;
        constexpr int mode = decltype(modec)::value;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            uint32_t off = pbase + ent[i].x;
            if constexpr (mode == kTapMask) {
                // entry.y = tap index r; bit r of apron_taps set -> all ones -> out of range
                off |= (uint32_t)__builtin_amdgcn_sbfe((int)apron_taps, ent[i].y, 1u);
            } else if constexpr (mode == kTapTest) {
                const int  ky = (int)ent[i].y >> 16;
                const int  kx = (int)(ent[i].y & 0xFFFFu);
                const bool ok = ((uint32_t)(iy0 + ky) < (uint32_t)p.Hi) & ((uint32_t)(ix0 + kx) < (uint32_t)p.Wi);
                off = ok ? off : kOutOfRange;
            }
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rin, LDS_PTR(dma_base_b + (st * STAGE_BYTES + KS * TO * 4 + i * NT * ACCESS_B)), C::VWB * 4,
                (int)off, 0, 0, 0);
        }
    };
    // table entries of the rows this thread copies, slab after slab
    uint32_t ent_addr = tab_base + (uint32_t)brow * 8u;
    auto read_entries = [&](u32x2 (&ent)[NB]) {
        static_for<NB>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            lds_read<i * BROWS * 8>(ent[i], ent_addr);
        });
        ent_addr += KS * 8;
    };
    auto wait_entries = [&](u32x2 (&ent)[NB]) {
        if constexpr (NB == 1) lds_wait<0>(ent[0]);
        else if constexpr (NB == 2) lds_wait<0>(ent[0], ent[1]);
        else if constexpr (NB == 4) lds_wait<0>(ent[0], ent[1], ent[2], ent[3]);
        else if constexpr (NB == 8) {
            lds_wait<0>(ent[0], ent[1], ent[2], ent[3]);
            lds_wait<0>(ent[4], ent[5], ent[6], ent[7]);      // nothing left to wait for: ties the registers to the wait
        }
        else static_assert(NB == 1 || NB == 2 || NB == 4 || NB == 8, "NB");
    };

    // ---- the matrix-core loop.  An MB x MB x KB instruction: lane l supplies
    // A[l%MB][l/MB] and B[l/MB][l%MB]; rows = filters, columns = flat m.  Column
    // block b of a wave holds m = base + RB*(l%MB) + b, so one RB-wide LDS read
    // feeds all RB column blocks and the RB results of a lane are adjacent in memory.
    //
    // Schedule.  Slab s lives in stage s % NS; the slab loop is unrolled NS
    // times so that every LDS address is a constant offset from one register.
    // The fragments of k-step j+1 are requested from LDS before the MFMAs of
    // k-step j issue, across slab boundaries too, so the MFMA stream never waits
    // on LDS latency.  The one barrier per slab sits inside slab s, before
    // k-step JB: by then every wave has waited for its own share of slab s+1,
    // so after the barrier slab s+1 is complete and visible, and every wave is
    // done with slab s-1, whose stage is refilled with slab s+NS-1; the refill
    // is issued in between that k-step's MFMAs.
    constexpr int NSTEP = KS / KB;    // MFMA k-steps per slab
    constexpr int JB    = C::JB;      // k-step in front of which the barrier sits
    constexpr int NM    = RA * RB;    // MFMAs per k-step
    static_assert(NSTEP % 2 == 0 && JB < NSTEP, "fragment double-buffer parity must not depend on the slab");
    static_assert((NS - 1) * STAGE_BYTES + (KB * (NSTEP - 1) * TO + (RA - 1) * MB) * 4 < 65536 &&
                  (NS - 1) * STAGE_BYTES + KB * (NSTEP - 1) * TM * 4 < 65536, "LDS immediate offsets");
    const uint32_t a_addr = lds_base + (uint32_t)(kg * TO + wo * (RA * MB) + lb) * 4u;
    const uint32_t b_addr = lds_base + (uint32_t)(KS * TO + kg * TM + wm * (RB * MB) + lb * RB) * 4u;
    float av[2][RA];
    BVec  bv[2];
    auto request = [&](auto stc, auto jc, auto bufc) {
        constexpr int st = decltype(stc)::value, j = decltype(jc)::value, buf = decltype(bufc)::value;
        static_for<RA>([&](auto ac) {
            constexpr int a = decltype(ac)::value;
            lds_read<st * STAGE_BYTES + (KB * j * TO + a * MB) * 4>(av[buf][a], a_addr);
        });
        lds_read<st * STAGE_BYTES + KB * j * TM * 4>(bv[buf], b_addr);
    };
    auto await = [&](auto pendc, auto bufc) {
        constexpr int pend = decltype(pendc)::value, buf = decltype(bufc)::value;
        if constexpr (RA == 1) lds_wait<pend>(av[buf][0], bv[buf]);
        else if constexpr (RA == 2) lds_wait<pend>(av[buf][0], av[buf][1], bv[buf]);
        else if constexpr (RA == 3) lds_wait<pend>(av[buf][0], av[buf][1], av[buf][2], bv[buf]);
        else lds_wait<pend>(av[buf][0], av[buf][1], av[buf][2], av[buf][3], bv[buf]);
    };
    auto drain = [&]() {
        static_for<2>([&](auto bc) {
            constexpr int buf = decltype(bc)::value;
            if constexpr (RA == 1) lds_wait<0>(av[buf][0], bv[buf]);
            else if constexpr (RA == 2) lds_wait<0>(av[buf][0], av[buf][1], bv[buf]);
            else if constexpr (RA == 3) lds_wait<0>(av[buf][0], av[buf][1], av[buf][2], bv[buf]);
            else lds_wait<0>(av[buf][0], av[buf][1], av[buf][2], av[buf][3], bv[buf]);
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    typedef std::integral_constant<int, 0> I0;

    // table row k: {byte offset of (c,ky,kx) in `in`, tap id}; rows k >= K are {0, 0}
    auto table_entry = [&](int k) -> u32x2 {
        u32x2 e = {0u, 0u};
        if (k < p.K) {
            const uint32_t c  = fast_div((uint32_t)k, p.sksk_magic, p.sksk_shift);
            const uint32_t r  = (uint32_t)k - c * (uint32_t)p.SkSk;
            const uint32_t ky = fast_div(r, p.sk_magic, p.sk_shift);
            const uint32_t kx = r - ky * (uint32_t)p.Sk;
            e.x = ((c * (uint32_t)p.Hi + ky) * (uint32_t)p.Wi + kx) * (uint32_t)p.Nb * 4u;
            e.y = small_filter ? r : ((ky << 16) | kx);
        }
        return e;
    };

    auto main_loop = [&](auto modec) {
        // ---- over K, in table-sized chunks (one chunk unless K is huge)
        for (int kc = 0; kc < p.K; kc += p.tab_cap) {
            if (kc) __syncthreads();  // previous chunk has let go of the ring and the table
            const int kend = min(p.K, kc + p.tab_cap);
            const int ns   = (kend - kc + KS - 1) / KS;
            u32x2 ent[NB];

            // offset table, Section 3.2: k = (c*Sk + ky)*Sk + kx  ->  ((c*Hi + ky)*Wi + kx)*Nb floats
            for (int i = t; i < p.tab_cap; i += NT) tab[i] = table_entry(kc + i);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // table rows written ...
            bare_barrier();                                       // ... and visible

            // prologue: slabs 0 .. NS-2 in flight, entries of slab NS-1 requested,
            // slab 0 complete and visible, its first fragments requested
            ent_addr = tab_base + (uint32_t)brow * 8u;
            static_for<NS - 1>([&](auto sc) {
                constexpr int s = decltype(sc)::value;
                if (s < ns) {
                    read_entries(ent);
                    wait_entries(ent);
                    issue_A(sc);
                    issue_B(sc, modec, ent);
                }
            });
            if (NS - 1 < ns) read_entries(ent);
            {
                const int younger = min(NS - 2, ns - 1);
                static_for<NS - 1>([&](auto yc) {
                    constexpr int y = decltype(yc)::value;
                    if (younger == y) vmem_wait<y * NL>();
                });
            }
            bare_barrier();
            __builtin_amdgcn_s_setprio(0);
            request(I0{}, I0{}, I0{});

            // One slab.  `steady` = slabs s+1 .. s+NS all exist, so the barrier, the
            // refill and the entry prefetch are unconditional (no scalar tests
            // inside the MFMA stream); the last slabs of a chunk take the tested form.
            auto slab = [&](auto uc, auto steadyc, const int s) {
                constexpr int  u      = decltype(uc)::value;         // stage of this slab
                constexpr int  unext  = (u + 1) % NS;                // stage of slab s+1
                constexpr int  ufill  = (u + NS - 1) % NS;           // stage slab s-1 leaves, slab s+NS-1 enters
                constexpr bool steady = decltype(steadyc)::value;
                const bool has_next = steady || (s + 1 < ns);
                const bool refill   = steady || (s + NS - 1 < ns);
                const bool more_ent = steady || (s + NS < ns);

                static_for<NSTEP>([&](auto jc) {
                    constexpr int j = decltype(jc)::value, cur = j & 1;
                    if constexpr (j == JB) {
                        if (has_next) {
                            // own share of slab s+1 landed: slabs s+2 .. s+NS-2 may still be in flight
                            if constexpr (steady) {
                                vmem_wait<(NS - 3 > 0 ? NS - 3 : 0) * NL>();
                            } else {
                                const int younger = min(NS - 3, ns - 2 - s);
                                static_for<(NS > 2 ? NS - 2 : 1)>([&](auto yc) {
                                    constexpr int y = decltype(yc)::value;
                                    if (younger == y) vmem_wait<y * NL>();
                                });
                            }
                            bare_barrier();
                        }
                        // entries were requested a slab ago, the current fragments a k-step ago: no stall
                        if (refill) wait_entries(ent);
                    }
                    if constexpr (j + 1 < NSTEP) {
                        request(uc, std::integral_constant<int, j + 1>{}, std::integral_constant<int, cur ^ 1>{});
                        await(std::integral_constant<int, RA + 1>{}, std::integral_constant<int, cur>{});
                    } else {
                        // Always the same request/await pair, also behind the last slab (where it
                        // fetches values nobody uses): a branch here would let the compiler copy
                        // a fragment register on one path before the wait that makes it valid.
                        request(std::integral_constant<int, unext>{}, I0{}, std::integral_constant<int, cur ^ 1>{});
                        await(std::integral_constant<int, RA + 1>{}, std::integral_constant<int, cur>{});
                    }
                    static_for<NM>([&](auto mc) {
                        constexpr int mi = decltype(mc)::value, a = mi / RB, b = mi % RB;
                        if constexpr (MB == 32)
                            acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][a], comp(bv[cur], b), acc[a][b], 0, 0, 0);
                        else
                            acc[a][b] = __builtin_amdgcn_mfma_f32_16x16x4f32(av[cur][a], comp(bv[cur], b), acc[a][b], 0, 0, 0);
                        if constexpr (j == JB) {
                            // refill, spread behind the MFMAs of this k-step
                            if constexpr (mi == 0) {
                                __builtin_amdgcn_sched_barrier(0);
                                if (refill) issue_A(std::integral_constant<int, ufill>{});
                                __builtin_amdgcn_sched_barrier(0);
                            }
                            if constexpr (mi == (NM > 1 ? 1 : 0)) {
                                __builtin_amdgcn_sched_barrier(0);
                                if (refill) issue_B(std::integral_constant<int, ufill>{}, modec, ent);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                            if constexpr (mi == (NM > 2 ? 2 : NM - 1)) {
                                __builtin_amdgcn_sched_barrier(0);
                                if (more_ent) read_entries(ent);
                                __builtin_amdgcn_sched_barrier(0);
                            }
                        }
                    });
                    // keep the written order request / wait / MFMAs k-step by k-step: the MFMAs are
                    // free to move across the asm statements otherwise, and a build that sinks
                    // them below the next wait serialises LDS latency with the matrix work
                    __builtin_amdgcn_sched_barrier(0);
                });
            };
            int s0 = 0;
            for (; s0 + 2 * NS - 1 < ns; s0 += NS)
                static_for<NS>([&](auto uc) { slab(uc, std::true_type{}, s0 + decltype(uc)::value); });
            for (; s0 < ns; s0 += NS)
                static_for<NS>([&](auto uc) {
                    if (s0 + decltype(uc)::value < ns) slab(uc, std::false_type{}, s0 + decltype(uc)::value);
                });
            // the fragment request behind the last slab is still in flight: let it land before
            // anything else may use those registers
            drain();
        }
    };
    if (interior)          main_loop(std::integral_constant<int, kTapNone>{});
    else if (small_filter) main_loop(std::integral_constant<int, kTapMask>{});
    else                   main_loop(std::integral_constant<int, kTapTest>{});

    // ---- epilogue: out = alpha * acc.  Accumulator register v of lane l in
    // block (a,b) is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of a 32 x 32 block
    // and row 4*(l/16) + v, column l%16 of a 16 x 16 block, so a lane's RB values
    // of one row are adjacent in memory.  Like the loop, the
    // epilogue is written to cost few instructions: a tile that lies wholly
    // inside the output (nearly all do) stores through a wave-uniform row
    // pointer plus one per-lane 32-bit offset, with no per-row address
    // arithmetic or bounds test in vector instructions.
    const int o_wave = o0 + wo * (RA * MB);
    const int m_wave = m0 + wm * (RB * MB);
    auto block_row = [](int a, int v) { return MB == 32 ? a * 32 + 8 * (v >> 2) + (v & 3) : a * 16 + v; };
    if (p.scat_stride) {
        // Scatter mode (see ConvParams): row o of the problem is a (residue class, channel) pair and
        // column m a (pixel, image) of the class's own grid; the value goes straight to its place in
        // the interleaved tensor, so the per-class results never exist in memory.  Where each row of
        // the tile goes is worked out once per tile into LDS (the operand ring is free by now).
        int* const row_c  = reinterpret_cast<int*>(lds);          // channel, or -1 for a row past the last
        int* const row_dy = row_c + TO;                           // ry - pad
        int* const row_dx = row_dy + TO;                          // rx - pad
        static_assert(3 * TO * 4 <= (int)C::ring_bytes, "row table fits the ring");
        __syncthreads();
        for (int r = t; r < TO; r += NT) {
            const int o = o0 + r;
            int c = -1, dy = 0, dx = 0;
            if (o < p.No) {
                const int cls = o / p.scat_Nc;
                const int ry  = cls / p.scat_stride;
                c  = o - cls * p.scat_Nc;
                dy = ry - p.scat_pad;
                dx = (cls - ry * p.scat_stride) - p.scat_pad;
            }
            row_c[r] = c;  row_dy[r] = dy;  row_dx[r] = dx;
        }
        __syncthreads();
        // this lane's columns: with 16-byte copies its RB columns are images of one pixel
        constexpr int NCOL = (VWB == 4) ? 1 : RB;
        int  cy[NCOL], cx[NCOL], cn[NCOL];
        bool cok[NCOL];
#pragma unroll
        for (int b = 0; b < NCOL; ++b) {
            const int m = m_wave + lb * RB + b;
            cok[b] = m < p.M;
            const int pix = (int)fast_div((uint32_t)(cok[b] ? m : 0), p.nb_magic, p.nb_shift);
            const int qy  = (int)fast_div((uint32_t)pix, p.wo_magic, p.wo_shift);
            cn[b] = (cok[b] ? m : 0) - pix * p.Nb;
            cy[b] = qy * p.scat_stride;
            cx[b] = (pix - qy * p.Wo) * p.scat_stride;
        }
#pragma unroll
        for (int a = 0; a < RA; ++a) {
#pragma unroll
            for (int v = 0; v < NV; ++v) {
                const int r  = wo * (RA * MB) + block_row(a, v) + 4 * kg;
                const int c  = row_c[r];
                const int dy = row_dy[r], dx = row_dx[r];
#pragma unroll
                for (int b = 0; b < NCOL; ++b) {
                    const int iy = cy[b] + dy, ix = cx[b] + dx;
                    const bool ok = cok[b] & (c >= 0) & ((uint32_t)iy < (uint32_t)p.scat_Hi) & ((uint32_t)ix < (uint32_t)p.scat_Wi);
                    if (!ok) continue;
                    // fewer than 2^30 elements: 32-bit index arithmetic cannot wrap
                    const uint32_t e = (((uint32_t)c * (uint32_t)p.scat_Hi + (uint32_t)iy) * (uint32_t)p.scat_Wi + (uint32_t)ix) *
                                           (uint32_t)p.Nb + (uint32_t)cn[b];
                    if constexpr (VWB == 4) {
                        BVec w;
#pragma unroll
                        for (int bb = 0; bb < RB; ++bb) {
                            if constexpr (RB == 1) w = p.alpha * acc[a][0][v];
                            else w[bb] = p.alpha * acc[a][bb][v];
                        }
                        *reinterpret_cast<BVec*>(p.out + e) = w;
                    } else {
                        p.out[e] = p.alpha * acc[a][b][v];
                    }
                }
            }
        }
        return;
    }
    if (o0 + TO <= p.No && m0 + TM <= p.M) {
        const uint32_t lane_off = ((uint32_t)(4 * kg) * (uint32_t)p.M + (uint32_t)(lb * RB)) * 4u;
        const size_t   row_bytes = (size_t)p.M * 4u;
        char* const    wave_base = reinterpret_cast<char*>(p.out) + ((size_t)o_wave * (size_t)p.M + (size_t)m_wave) * 4u;
        auto store_rows = [&](auto unitc, auto streamc) {
            constexpr bool unit = decltype(unitc)::value;       // alpha == 1: store the accumulators as they are
            constexpr bool streaming = decltype(streamc)::value;
#pragma unroll
            for (int a = 0; a < RA; ++a) {
#pragma unroll
                for (int v = 0; v < NV; ++v) {
                    char* row = wave_base + (size_t)block_row(a, v) * row_bytes;   // uniform
                    BVec w;
#pragma unroll
                    for (int b = 0; b < RB; ++b) {
                        const float x = unit ? acc[a][b][v] : p.alpha * acc[a][b][v];
                        if constexpr (RB == 1) w = x;
                        else w[b] = x;
                    }
                    if constexpr (streaming) __builtin_nontemporal_store(w, reinterpret_cast<BVec*>(row + lane_off));
                    else *reinterpret_cast<BVec*>(row + lane_off) = w;
                }
            }
        };
        // Short contractions are bound by writing the output (Section 3.4's first-layer case taken
        // to its end: K = 27 does 54 FLOPs per 4 bytes written).  There, and wherever the output is
        // too large to stay in L2, the stores carry the non-temporal hint, so the result streams to
        // memory instead of displacing the operands in L2: 4.1 -> 5.0 TB/s on a 3 -> 64 channel
        // layer; on matrix-bound layers never slower and up to 2.6 points faster (K = 576), depending
        // on the machine.
        if (p.stream_out) {
            if (p.alpha == 1.0f) store_rows(std::true_type{}, std::true_type{});
            else                 store_rows(std::false_type{}, std::true_type{});
        } else {
            if (p.alpha == 1.0f) store_rows(std::true_type{}, std::false_type{});
            else                 store_rows(std::false_type{}, std::false_type{});
        }
        return;
    }
    // ragged tile: per-row and per-column tests
    const int ocol = m_wave + lb * RB;
#pragma unroll
    for (int a = 0; a < RA; ++a) {
#pragma unroll
        for (int v = 0; v < NV; ++v) {
            const int o = o_wave + block_row(a, v) + 4 * kg;
            if (o >= p.No) continue;
            float* dst = p.out + (size_t)o * (size_t)p.M + ocol;
            if constexpr (VWB == 4) {
                if (ocol < p.M) {                 // M % 4 == 0 and RB | 4: all or nothing
                    BVec w;
#pragma unroll
                    for (int b = 0; b < RB; ++b) {
                        if constexpr (RB == 1) w = p.alpha * acc[a][0][v];
                        else w[b] = p.alpha * acc[a][b][v];
                    }
                    *reinterpret_cast<BVec*>(dst) = w;
                }
            } else {
#pragma unroll
                for (int b = 0; b < RB; ++b)
                    if (ocol + b < p.M) dst[b] = p.alpha * acc[a][b][v];
            }
        }
    }
}

// Position in visiting order -> column-tile index (see ConvParams::row_tiles).
__device__ __forceinline__ int column_tile(const ConvParams& p, int seq)
{
    if (p.row_tiles == 0) return seq;
    const int per_strip = p.strip_rows * p.row_tiles;
    const int strip = seq / per_strip;
    const int r     = seq - strip * per_strip;
    const int rows  = min(p.strip_rows, p.Ho - strip * p.strip_rows);   // last strip may be short
    const int xt    = r / rows;
    const int y     = strip * p.strip_rows + (r - xt * rows);
    return y * p.row_tiles + xt;
}

// A tile cut into SPLIT pieces of equal area: same threads, same ring depth and
// slab.  Along the filter dimension where the wave layout allows it (same
// columns, TO / SPLIT filters); a tile with an odd number of filter blocks per
// wave is halved along the columns instead.
template <class C, int SPLIT> struct PieceOf;
template <class C> struct PieceOf<C, 2> {
    static_assert(C::RA % 2 == 0 || C::RB % 2 == 0, "no way to halve this tile");
    typedef typename std::conditional<C::RA % 2 == 0,
        Cfg<C::WO, C::WM, C::RA / 2, C::RB, C::KS, C::NS, C::VW, C::JB, C::MB>,            // half the filter blocks per wave
        typename std::conditional<C::WO == 2,
            Cfg<1, C::WM * 2, C::RA, C::RB / 2, C::KS, C::NS, C::VW, C::JB, C::MB>,        // half the filter waves, moved to the column side
            Cfg<C::WO, C::WM, C::RA, C::RB / 2, C::KS, C::NS, C::VW, C::JB, C::MB>>::type  // half the columns
        >::type type;
};
template <class C> struct PieceOf<C, 4> {
    typedef typename PieceOf<typename PieceOf<C, 2>::type, 2>::type type;
};

// A 128-row tile cut 48 + 48 + 32 along the filters ("thirds"): two pieces of three 16-row matrix
// blocks per wave and the quarter piece.  This is the cut for launches whose last round leaves
// between a quarter and a third of a tile per compute unit (338 tiles on 256 units: one whole
// tile and one 48-row piece each end 8 % sooner than one whole and a half).
template <class C> struct ThirdOf {
    static_assert(C::TO == 128 && C::MB == 32 && C::KS % 4 == 0, "thirds exist for 128-row tiles");
    static constexpr int NSTEP16 = C::KS / 4;
    typedef Cfg<1, C::WO * C::WM, 3, C::TM / (C::WO * C::WM) / 16, C::KS, C::NS, C::VW,
                (C::JB < NSTEP16 ? C::JB : NSTEP16 - 1), 16> big;       // 48 x TM
    static_assert(big::TM == C::TM && PieceOf<C, 4>::type::TM == C::TM && PieceOf<C, 4>::type::TO == 32,
                  "the last 32 rows run as the fourth quarter piece");
};

// A 128-row tile cut into eight pieces of 16 rows: one 16-row matrix block per wave, all waves
// side by side along the columns.  For launches that leave a CU a sixteenth to an eighth of a tile
// beyond the pieces it already has (392 tiles on 256 units: a whole tile, a half and, on a quarter
// of the units, one of these).
template <class C> struct EighthOf {
    static_assert(C::TO == 128 && C::MB == 32 && C::KS % 4 == 0, "eighths exist for 128-row tiles");
    static constexpr int NSTEP16 = C::KS / 4;
    typedef Cfg<1, C::WO * C::WM, 1, C::TM / (C::WO * C::WM) / 16, C::KS, C::NS, C::VW,
                (C::JB < NSTEP16 ? C::JB : NSTEP16 - 1), 16> type;      // 16 x TM
    static_assert(type::TM == C::TM && type::TO == 16, "eight pieces stacked along the filters");
};

// Run piece `part` of the tile at (o0, m0) of the whole-tile shape C as shape P.
template <class C, class P>
__device__ __forceinline__ void conv_piece(const ConvParams& p, unsigned char* lds, int o0, int m0, int part)
{
    static_assert(P::NT == C::NT && P::TO * P::TM * (C::TO / P::TO) * (C::TM / P::TM) == C::TO * C::TM, "piece shape");
    constexpr int along_m = C::TM / P::TM;                 // pieces side by side along the columns
    const int pm = part % along_m, po = part / along_m;
    conv_tile<P, C::TO * 4096 + C::TM>(p, lds, o0 + po * P::TO, m0 + pm * P::TM);     // one CONTEXT per parent shape
}

// SPLITS: 1 = whole tiles only; 2 = the kernel also carries the half-tile body; 4 = half and quarter;
// 8 = half, quarter and the 16-row eighth.
// THIRDS: it carries the 48-row body as well.
template <class C, int SPLITS, bool THIRDS = false>
__global__ void __launch_bounds__(C::NT) conv_fprop_kernel(const ConvParams p)
{
    extern __shared__ __align__(16) unsigned char lds_raw[];
    // ---- tile map.  Workgroups are dealt round-robin to the 8 XCDs, each with
    // its own L2: give every XCD a contiguous run of tiles so that neighbouring
    // output coordinates (overlapping patches) and the filter tiles of one
    // coordinate (same patch) meet in the same L2.  Launch order: up to one
    // piece per CU, then the whole tiles, then the remaining pieces of the
    // last, partial round of tiles -- so that the tail of the launch is made of
    // short workgroups on every CU instead of long ones on a few (Section 3.4's
    // smaller blocks, used only where they pay), and so that, where one piece
    // per CU is all there is, no piece runs alone on its CU (see the host's
    // plan()).  Every region is a multiple of 8 workgroups long, which keeps
    // workgroup id mod 8 = XCD.
    const int front = p.front.wgs;
    const int whole = 8 * p.tiles_per_xcd;
    int       bid   = (int)blockIdx.x - front;
    if (bid >= 0 && bid < whole) {
        const int tile = (bid & 7) * p.tiles_per_xcd + (bid >> 3);
        if (tile >= p.n_whole) return;                       // uniform per workgroup
        const int ms = tile / p.n_otiles;
        const int ot = tile - ms * p.n_otiles;
        conv_tile<C>(p, lds_raw, ot * C::TO, column_tile(p, ms) * C::TM);
        return;
    }
    if constexpr (SPLITS > 1) {
        // Scalar selects with constant indices only: a variable index, or a reference that may name
        // either region, would move the argument block to scratch memory.
        const bool in_front = bid < 0;
        bid = in_front ? (int)blockIdx.x : bid - whole;
        int cls = 0, per = 0, cnt = 0, beg = 0;
        auto pick = [&](auto cc) {
            constexpr int c = decltype(cc)::value;
            per = in_front ? p.front.per_xcd[c] : p.back.per_xcd[c];
            cnt = in_front ? p.front.count[c] : p.back.count[c];
            beg = in_front ? p.front.begin[c] : p.back.begin[c];
        };
        pick(std::integral_constant<int, 0>{});
        static_for<3>([&](auto cc) {
            constexpr int c = decltype(cc)::value;
            if (cls == c && bid >= 8 * per) {
                bid -= 8 * per;
                cls = c + 1;
                pick(std::integral_constant<int, c + 1>{});
            }
        });
        const int j = (bid & 7) * per + (bid >> 3);
        if (j >= cnt) return;                                // uniform per workgroup
        const int q = beg + j;                               // piece number within its class
        // The cut tiles follow the whole ones: first those cut in halves, then those cut in thirds,
        // in quarters, in eighths.
        int cut = cls == 3 ? 8 : cls + 2, tile, part;
        if (cls == 0)      { tile = q >> 1;  part = q & 1; }
        else if (cls == 1) { tile = q / 3;   part = q - tile * 3;  tile += p.n_half; }
        else if (cls == 2) { tile = q >> 2;  part = q & 3;  tile += p.n_half + p.n_third; }
        else               { tile = q >> 3;  part = q & 7;  tile += p.n_half + p.n_third + p.n_quarter; }
        tile += p.n_whole;
        const int ms = tile / p.n_otiles;
        const int ot = tile - ms * p.n_otiles;
        const int o0 = ot * C::TO, m0 = column_tile(p, ms) * C::TM;
        if (cut == 2) {
            conv_piece<C, typename PieceOf<C, 2>::type>(p, lds_raw, o0, m0, part);
            return;
        }
        if constexpr (THIRDS) {
            static_assert(SPLITS >= 4, "the 32-row third is the quarter piece");
            if (cut == 3) {
                if (part < 2) {
                    conv_tile<typename ThirdOf<C>::big, C::TO * 4096 + C::TM>(p, lds_raw, o0 + 48 * part, m0);
                    return;
                }
                cut = 4;  part = 3;      // rows 96 .. 127: the fourth quarter piece
            }
        }
        if constexpr (SPLITS >= 4) {
            if (cut == 4) {
                conv_piece<C, typename PieceOf<C, 4>::type>(p, lds_raw, o0, m0, part);
                return;
            }
        }
        if constexpr (SPLITS >= 8) {
            if (cut == 8) conv_tile<typename EighthOf<C>::type, C::TO * 4096 + C::TM>(p, lds_raw, o0 + 16 * part, m0);
        }
    }
}

// ---- one registry entry per instantiated kernel
template <class C, int SPLITS = 1, bool THIRDS = false>
constexpr VariantEntry make_entry(const char* name, int wg_per_cu, float eff, float eff_few,
                                  int max_tab = kMaxTabEntries)
{
    return VariantEntry{VariantInfo{name, C::TO, C::TM, C::KS, C::NT, C::VWA == 4 ? 1 : 0, C::VWB == 4 ? 1 : 0, wg_per_cu, eff, eff_few,
                                    SPLITS, THIRDS ? 1 : 0, max_tab},
                        &conv_fprop_kernel<C, SPLITS, THIRDS>, C::ring_bytes};
}

}  // namespace

}  // namespace mdnn
#endif
