// Filter gradient (BPROP with respect to the weights) for gfx950 (MI355X) on
// the FP32 matrix cores.
//
// The maxDNN paper only states the belief that its approach carries over to
// BPROP (abstract, Section 3.5).  For the weights it does, with the roles of
// the GEMM dimensions rotated.  Section 3 multiplies, per output coordinate, a
// patch (K columns, K = Nc*Sk*Sk) by the filter matrix (K x No).  The gradient
// of that filter matrix is
//     dfilt[k][o] = alpha * sum_m  P[k][m] * G[o][m],      m = (y*Wo + x)*Nb + n,
// where P[k][m] is element k of the patch at output coordinate (y,x) of image n
// (zero in the apron, gathered with the same (c,ky,kx) -> offset arithmetic as
// in Section 3.2) and G = dout seen as a row-major No x M matrix.  The result is
// small (K x No) and the contraction is long (M = Ho*Wo*Nb), so the work is cut
// along m as well: a workgroup owns a 128 x 128 tile of dfilt and one range of
// m, writes its partial tile to the caller's workspace, and a second small
// kernel adds the partial tiles in a fixed order and scales by alpha
// (deterministic; no atomics).
//
// MFMA 32x32x2 wants lane l to supply P[row l%32][m + l/32] and
// G[row l%32][m + l/32]; in memory both operands are contiguous along m (the
// batch index is innermost in both tensors).  So in LDS a slab keeps, for each
// of its 128 + 128 rows, 16 consecutive m as four 16-byte chunks, and a lane
// reads one whole chunk (ds_read_b128) that feeds four MFMA steps: lanes 0-31
// take chunk 2g, lanes 32-63 chunk 2g+1, and step q multiplies element q of
// both -- any pairing of m values between the two lane halves is a valid
// contraction order as long as P and G use the same one.  Rows are 64 bytes
// apart and LDS has 64 banks (256 bytes); a 16-byte read is served 16 lanes at a
// time, the lanes of a half-wave grouped by the parity of (lane/4)'s bits:
// {0-3,12-15,20-27} and {4-11,16-19,28-31} (measured with two-lane probes and the
// bank-conflict counter).  With one lane per row, four lanes of such a group
// have the same row%4 and would meet in the same banks; they differ in
// (row/8)%4, so the chunk position inside a row is XOR-ed with (row/8)%4.
// Global -> LDS copies write lane-contiguous LDS, so the swizzle is applied on
// the global side: the lane that fills position u of a row fetches chunk
// u ^ (row/8)%4 of that row.
//
// Pipeline, waits and barrier placement follow the forward kernel: a ring of
// NS slabs filled by global -> LDS copies, LDS reads through inline asm with
// hand-counted waits, one fence-free barrier per slab.
#include <hip/hip_runtime.h>

#include "gfx950_util.h"
#include "mdnn_internal.h"

namespace mdnn {
namespace {

constexpr int kTileK     = 128;   // rows of dfilt (k) per workgroup
constexpr int kSlabM     = 16;    // m per slab and row
constexpr int kRowBytes  = kSlabM * 4;
constexpr int kOperBytes = 128 * kRowBytes;       // one operand's slab
constexpr int kStageBytes = 2 * kOperBytes;

// VW: floats per global -> LDS copy (4 needs Nb % 4 == 0).  UNIFORM: Nb % 16 == 0,
// so the 16 m of a slab share one output coordinate and the walk over
// coordinates is scalar work done once per coordinate instead of per copy.
// WK x (4/WK) waves, each owning RA x RB MFMA blocks: WK*RA*32 = 128 rows k and
// (4/WK)*RB*32 <= 128 columns o (Section 3.4's other block sizes, for layers with
// few filters).  The G slab in LDS always has 128 rows; a narrower tile leaves
// the surplus rows out of range (zero-filled, never read).
//
// The body is a device function, not the kernel itself: the host pass checks a
// kernel's body against the host's idea of the target and rejects the 16-byte
// form of the global -> LDS copy there.
template <int VW, bool UNIFORM, int NS, int WK, int RA, int RB>
__device__ __forceinline__ void filter_grad_workgroup(const FilterGradParams& p, unsigned char* lds)
{
    constexpr int WO = 4 / WK;
    constexpr int TO = WO * RB * 32;          // columns of dfilt (o) per workgroup
    static_assert(WK * RA * 32 == kTileK && TO <= 128 && RA + RB <= 4, "tile shape");
    static_assert(VW == 4 || (VW == 1 && !UNIFORM), "VW");
    static_assert(NS >= 3, "slab s+1 must be in flight when slab s reaches its barrier");
    constexpr int CPR = 16 / VW;              // lanes per row in one copy
    constexpr int RPI = 64 / CPR;             // rows one copy covers
    constexpr int NI  = 128 / RPI / 4;        // copies per operand, wave and slab
    constexpr int NL  = 2 * NI;               // copies per wave and slab
    constexpr int COPY_BYTES = 64 * 4 * VW;
    typedef std::integral_constant<int, 4 * VW> CopySize;   // a plain constant is not one inside the lambdas below
    static_assert((NS - 2) * NL <= 63, "vmcnt range");

    // ---- which tile, which range of m.  Workgroups are dealt round-robin to the
    // 8 XCDs; consecutive work items (all tiles of one range of m, which read the
    // same slices of `in` and `dout`) go to the same XCD and so share its L2.
    const int bid = blockIdx.x;
    const int w   = (bid & 7) * p.per_xcd + (bid >> 3);
    if (w >= p.n_tiles * p.splits) return;
    const int sp   = w / p.n_tiles;
    const int tile = w - sp * p.n_tiles;
    const int kt   = tile / p.n_otiles;
    const int k0   = kt * kTileK;
    const int o0   = (tile - kt * p.n_otiles) * TO;
    const int m_begin = sp * p.m_per_split;
    const int m_end   = min(p.M, m_begin + p.m_per_split);
    const int ns      = (m_end - m_begin + kSlabM - 1) / kSlabM;

    const uint32_t lds_base = (uint32_t)(uintptr_t)LDS_PTR(lds);
    const int t    = threadIdx.x;
    const int lane = t & 63;
    const int wave = __builtin_amdgcn_readfirstlane(t >> 6);
    const int wk   = wave % WK;
    const int wo   = wave / WK;
    const int half = lane >> 5;
    const int l32  = lane & 31;

    const __amdgpu_buffer_rsrc_t rin =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.in), 0, (int)p.in_bytes, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rdo =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.dout), 0, (int)p.dout_bytes, kRsrcWord3);

    // ---- copy roles.  Copy i of this wave covers rows (wave*NI + i)*RPI ... of an
    // operand slab; this lane fills position u of row `rsub` of those.
    const int u    = lane % CPR;
    const int rsub = lane / CPR;
    int      dm[NI];           // m of this lane's datum relative to the slab start
    uint32_t rowoff[NI];       // P side: byte offset of (c,ky,kx) in `in`
    int      ky[NI], kx[NI];   // P side: tap of the row; far out of range for rows k >= K
    uint32_t offg[NI];         // G side: running byte offset in `dout`
    uint32_t incg[NI];         // G side: 64 per slab; 0 for rows o >= No, which stay out of range
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int row = (wave * NI + i) * RPI + rsub;
        const int pos = (VW == 4) ? u : (u >> 2);
        const int el  = (VW == 4) ? 0 : (u & 3);
        dm[i] = 4 * (pos ^ ((row >> 3) & 3)) + el;
        const int k = k0 + row;
        if (k < p.K) {
            const uint32_t c  = fast_div((uint32_t)k, p.sksk_magic, p.sksk_shift);
            const uint32_t r  = (uint32_t)k - c * (uint32_t)p.SkSk;
            const uint32_t yy = fast_div(r, p.sk_magic, p.sk_shift);
            const uint32_t xx = r - yy * (uint32_t)p.Sk;
            rowoff[i] = ((c * (uint32_t)p.Hi + yy) * (uint32_t)p.Wi + xx) * (uint32_t)p.Nb * 4u;
            ky[i] = (int)yy;
            kx[i] = (int)xx;
        } else {
            rowoff[i] = 0;
            ky[i] = 1 << 20;
            kx[i] = 1 << 20;
        }
        const int o = o0 + row;
        if (row < TO && o < p.No) {
            offg[i] = (uint32_t)(((size_t)o * (size_t)p.M + (size_t)(m_begin + dm[i])) * 4u);
            incg[i] = kRowBytes;
        } else {
            offg[i] = kOutOfRange;
            incg[i] = 0;
        }
    }

    // ---- the walk over m of the copies (runs NS-1 slabs ahead of the MFMAs)
    int cur_m = m_begin;                      // general path: slab start
    // uniform path: the slab's output coordinate and batch offset, all scalar
    int      cur_n = 0, cur_x = 0, cur_y = 0;
    uint32_t cur_off = 0;                     // ((iy0*Wi + ix0)*Nb + n)*4 mod 2^32
    bool     okp[NI];                         // this row's tap is inside the image at the current coordinate
    auto enter_coordinate = [&]() {
        const int iy0 = cur_y * p.stride - p.pad;
        const int ix0 = cur_x * p.stride - p.pad;
        cur_off = (((uint32_t)iy0 * (uint32_t)p.Wi + (uint32_t)ix0) * (uint32_t)p.Nb + (uint32_t)cur_n) * 4u;
#pragma unroll
        for (int i = 0; i < NI; ++i)
            okp[i] = ((uint32_t)(iy0 + ky[i]) < (uint32_t)p.Hi) & ((uint32_t)(ix0 + kx[i]) < (uint32_t)p.Wi);
    };
    if constexpr (UNIFORM) {
        const int pix = (int)fast_div((uint32_t)m_begin, p.nb_magic, p.nb_shift);
        cur_n = m_begin - pix * p.Nb;
        cur_y = (int)fast_div((uint32_t)pix, p.wo_magic, p.wo_shift);
        cur_x = pix - cur_y * p.Wo;
        enter_coordinate();
#pragma unroll
        for (int i = 0; i < NI; ++i) rowoff[i] += (uint32_t)dm[i] * 4u;
    }

    unsigned char* const dma_base = lds + wave * (NI * COPY_BYTES);      // wave-uniform
    auto issue_P = [&](auto stc) {
        constexpr int st = decltype(stc)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            uint32_t off;
            if constexpr (UNIFORM) {
                off = okp[i] ? rowoff[i] + cur_off : kOutOfRange;
            } else {
                const int m = cur_m + dm[i];
                off = kOutOfRange;
                if (m < m_end) {
                    const int pix = (int)fast_div((uint32_t)m, p.nb_magic, p.nb_shift);
                    const int n   = m - pix * p.Nb;
                    const int y   = (int)fast_div((uint32_t)pix, p.wo_magic, p.wo_shift);
                    const int x   = pix - y * p.Wo;
                    const int iy0 = y * p.stride - p.pad;
                    const int ix0 = x * p.stride - p.pad;
                    const bool ok = ((uint32_t)(iy0 + ky[i]) < (uint32_t)p.Hi) & ((uint32_t)(ix0 + kx[i]) < (uint32_t)p.Wi);
                    if (ok)
                        off = rowoff[i] +
                              (((uint32_t)iy0 * (uint32_t)p.Wi + (uint32_t)ix0) * (uint32_t)p.Nb + (uint32_t)n) * 4u;
                }
            }
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rin, LDS_PTR(dma_base + (st * kStageBytes + i * COPY_BYTES)),
                                                     CopySize::value, (int)off, 0, 0, 0);
        }
    };
    auto issue_G = [&](auto stc) {
        constexpr int st = decltype(stc)::value;
#pragma unroll
        for (int i = 0; i < NI; ++i) {
            uint32_t off = offg[i];
            if constexpr (!UNIFORM) off = (cur_m + dm[i] < m_end) ? off : kOutOfRange;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(
                rdo, LDS_PTR(dma_base + (st * kStageBytes + kOperBytes + i * COPY_BYTES)), CopySize::value, (int)off, 0, 0, 0);
            offg[i] += incg[i];
        }
        // step the walk to the next slab
        if constexpr (UNIFORM) {
            cur_n += kSlabM;
            cur_off += kRowBytes;
            if (cur_n == p.Nb) {
                cur_n = 0;
                if (++cur_x == p.Wo) { cur_x = 0; ++cur_y; }
                enter_coordinate();
            }
        } else {
            cur_m += kSlabM;
        }
    };

    // ---- fragments.  Block row r of operand X lives at X + r*64; chunk c of it at
    // position c ^ (r/8)%4.  Group g of a slab: lanes 0-31 chunk 2g, lanes 32-63 chunk 2g+1.
    const int rowA = wk * (RA * 32) + l32;
    const int rowB = wo * (RB * 32) + l32;
    uint32_t a_addr[2], b_addr[2];
#pragma unroll
    for (int g = 0; g < 2; ++g) {
        a_addr[g] = lds_base + (uint32_t)(rowA * kRowBytes + (((2 * g + half) ^ ((rowA >> 3) & 3)) * 16));
        b_addr[g] = lds_base + (uint32_t)(kOperBytes + rowB * kRowBytes + (((2 * g + half) ^ ((rowB >> 3) & 3)) * 16));
    }
    f32x4 fa[2][RA], fb[2][RB];               // [buffer][block]
    auto request = [&](auto stc, auto gc, auto bufc) {
        constexpr int st = decltype(stc)::value, g = decltype(gc)::value, buf = decltype(bufc)::value;
        static_for<RA>([&](auto ac) {
            constexpr int a = decltype(ac)::value;
            lds_read<st * kStageBytes + a * 32 * kRowBytes>(fa[buf][a], a_addr[g]);
        });
        static_for<RB>([&](auto bc) {
            constexpr int b = decltype(bc)::value;
            lds_read<st * kStageBytes + b * 32 * kRowBytes>(fb[buf][b], b_addr[g]);
        });
    };
    auto await = [&](auto pendc, auto bufc) {
        constexpr int pend = decltype(pendc)::value, buf = decltype(bufc)::value;
        if constexpr (RA == 2 && RB == 2)      lds_wait<pend>(fa[buf][0], fa[buf][1], fb[buf][0], fb[buf][1]);
        else if constexpr (RA == 1 && RB == 3) lds_wait<pend>(fa[buf][0], fb[buf][0], fb[buf][1], fb[buf][2]);
        else if constexpr (RA == 1 && RB == 2) lds_wait<pend>(fa[buf][0], fb[buf][0], fb[buf][1]);
        else if constexpr (RA == 1 && RB == 1) lds_wait<pend>(fa[buf][0], fb[buf][0]);
        else static_assert(RA == 0, "no wait written for this block shape");
    };
    typedef std::integral_constant<int, 0> I0;
    typedef std::integral_constant<int, 1> I1;
    typedef std::integral_constant<int, RA + RB> IReq;   // LDS reads one request issues
    constexpr int NM = RA * RB;                          // MFMAs per step

    f32x16 acc[RA][RB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    // ---- prologue: slabs 0 .. NS-2 in flight, slab 0 complete and visible
    static_for<NS - 1>([&](auto sc) {
        if (decltype(sc)::value < ns) {
            issue_P(sc);
            issue_G(sc);
        }
    });
    {
        const int younger = min(NS - 2, ns - 1);
        static_for<NS - 1>([&](auto yc) {
            constexpr int y = decltype(yc)::value;
            if (younger == y) vmem_wait<y * NL>();
        });
    }
    bare_barrier();
    request(I0{}, I0{}, I0{});

    // One slab = two groups of four MFMA steps.  The barrier sits after the first
    // step: by then this wave has waited for its own copies of slab s+1, so
    // behind the barrier slab s+1 is complete and every wave is done with slab
    // s-1, whose stage the copies of slab s+NS-1 (issued between the next MFMAs)
    // may overwrite.
    auto slab = [&](auto uc, auto steadyc, const int s) {
        constexpr int  st     = decltype(uc)::value;
        constexpr int  unext  = (st + 1) % NS;
        constexpr int  ufill  = (st + NS - 1) % NS;
        constexpr bool steady = decltype(steadyc)::value;
        const bool has_next = steady || (s + 1 < ns);
        const bool refill   = steady || (s + NS - 1 < ns);

        // sched_barrier(0): keep the written order of requests, waits and MFMA groups -- the MFMAs
        // are free to move across the asm statements otherwise, and a build that sinks them below
        // the next wait serialises LDS latency and the barrier with the matrix work
        request(uc, I1{}, I1{});
        await(IReq{}, I0{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            if constexpr (q == 1) {
                __builtin_amdgcn_sched_barrier(0);
                if (has_next) {
                    if constexpr (steady) {
                        vmem_wait<(NS - 3) * NL>();
                    } else {
                        const int younger = min(NS - 3, ns - 2 - s);
                        static_for<NS - 2>([&](auto yc) {
                            constexpr int y = decltype(yc)::value;
                            if (younger == y) vmem_wait<y * NL>();
                        });
                    }
                    bare_barrier();
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            static_for<NM>([&](auto mc) {
                constexpr int mi = decltype(mc)::value, a = mi / RB, b = mi % RB;
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[0][a][q], fb[0][b][q], acc[a][b], 0, 0, 0);
                if constexpr (q == 1 && mi == 0) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (refill) issue_P(std::integral_constant<int, ufill>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (q == 1 && mi == (NM > 1 ? 1 : 0)) {
                    __builtin_amdgcn_sched_barrier(0);
                    if (refill) issue_G(std::integral_constant<int, ufill>{});
                    __builtin_amdgcn_sched_barrier(0);
                }
            });
        });
        // always the same request/await pair, also behind the last slab (where it fetches values
        // nobody uses): a branch here would let the compiler copy a fragment register on one path
        // before the wait that makes it valid
        __builtin_amdgcn_sched_barrier(0);
        request(std::integral_constant<int, unext>{}, I0{}, I0{});
        await(IReq{}, I1{});
        __builtin_amdgcn_sched_barrier(0);
        static_for<4>([&](auto qc) {
            constexpr int q = decltype(qc)::value;
            static_for<NM>([&](auto mc) {
                constexpr int mi = decltype(mc)::value, a = mi / RB, b = mi % RB;
                acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(fa[1][a][q], fb[1][b][q], acc[a][b], 0, 0, 0);
            });
        });
        __builtin_amdgcn_sched_barrier(0);
    };
    int s0 = 0;
    for (; s0 + 2 * NS - 1 < ns; s0 += NS)
        static_for<NS>([&](auto uc) { slab(uc, std::true_type{}, s0 + decltype(uc)::value); });
    for (; s0 < ns; s0 += NS)
        static_for<NS>([&](auto uc) {
            if (s0 + decltype(uc)::value < ns) slab(uc, std::false_type{}, s0 + decltype(uc)::value);
        });

    // the fragment request behind the last slab is still in flight: let it land before anything
    // else may use those registers
    await(I0{}, I0{});
    await(I0{}, I1{});
    __builtin_amdgcn_sched_barrier(0);

    // ---- partial tile -> workspace [split][K][No].  Accumulator register v of lane
    // l in block (a,b) is row 8*(v/4) + 4*(l/32) + v%4, column l%32: 32 lanes
    // store 32 consecutive o.
    float* const dst = p.part + (size_t)sp * (size_t)p.K * (size_t)p.No;
    const int    o   = o0 + wo * (RB * 32) + l32;
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int k = k0 + wk * (RA * 32) + a * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (k >= p.K) continue;
#pragma unroll
            for (int b = 0; b < RB; ++b)
                if (o + 32 * b < p.No) dst[(size_t)k * (size_t)p.No + o + 32 * b] = acc[a][b][v];
        }
}

template <int VW, bool UNIFORM, int NS, int WK, int RA, int RB>
__global__ void __launch_bounds__(256) conv_bprop_filter_kernel(const FilterGradParams p)
{
    extern __shared__ __align__(64) unsigned char lds_raw[];
    filter_grad_workgroup<VW, UNIFORM, NS, WK, RA, RB>(p, lds_raw);
}

// dfilt[e] = alpha * sum over the ranges of part[range][e], in a fixed order (same
// bits on every run).  Small gradients with many ranges: a block owns 32
// consecutive elements; eight threads per element each add every eighth range
// in ascending order (several loads in flight), and the eight chains are then
// added in ascending order.
__global__ void __launch_bounds__(256) sum_partial_gradients(const float* __restrict__ part,
                                                             float* __restrict__ dfilt,
                                                             size_t n, int splits, float alpha)
{
    __shared__ float chain[8][32];
    const int    el = threadIdx.x & 31;
    const int    ch = threadIdx.x >> 5;
    const size_t e  = (size_t)blockIdx.x * 32 + el;
    float s = 0.0f;
    if (e < n) {
        int i = ch;
        for (; i + 24 < splits; i += 32) {
            const float v0 = part[(size_t)i * n + e];
            const float v1 = part[(size_t)(i + 8) * n + e];
            const float v2 = part[(size_t)(i + 16) * n + e];
            const float v3 = part[(size_t)(i + 24) * n + e];
            s += v0;
            s += v1;
            s += v2;
            s += v3;
        }
        for (; i < splits; i += 8) s += part[(size_t)i * n + e];
    }
    chain[ch][el] = s;
    __syncthreads();
    if (ch == 0 && e < n) {
        float r = chain[0][el];
#pragma unroll
        for (int c = 1; c < 8; ++c) r += chain[c][el];
        dfilt[e] = alpha * r;
    }
}

// Large gradients (n % 4 == 0): plenty of elements to fill the chip, so one
// thread adds all ranges of four adjacent elements with 16-byte accesses.
__global__ void __launch_bounds__(256) sum_partial_gradients_wide(const f32x4* __restrict__ part,
                                                                  f32x4* __restrict__ dfilt,
                                                                  size_t n4, int splits, float alpha)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= n4) return;
    f32x4 s = part[e];
    int i = 1;
    for (; i + 3 < splits; i += 4) {
        const f32x4 v0 = part[(size_t)i * n4 + e];
        const f32x4 v1 = part[(size_t)(i + 1) * n4 + e];
        const f32x4 v2 = part[(size_t)(i + 2) * n4 + e];
        const f32x4 v3 = part[(size_t)(i + 3) * n4 + e];
        s += v0;
        s += v1;
        s += v2;
        s += v3;
    }
    for (; i < splits; ++i) s += part[(size_t)i * n4 + e];
    dfilt[e] = alpha * s;
}

typedef void (*FilterGradFn)(const FilterGradParams);
constexpr int kRingStages = 3;
template <int VW, bool UNIFORM, int WK, int RA, int RB>
constexpr FilterGradFn kernel_of()
{
    return &conv_bprop_filter_kernel<VW, UNIFORM, kRingStages, WK, RA, RB>;
}
// [tile width 128, 96, 64, 32][16-byte copies with the scalar walk / 16-byte copies, per-lane walk /
// 4-byte copies]
const FilterGradFn kKernels[4][3] = {
    {kernel_of<4, true, 2, 2, 2>(), kernel_of<4, false, 2, 2, 2>(), kernel_of<1, false, 2, 2, 2>()},
    {kernel_of<4, true, 4, 1, 3>(), kernel_of<4, false, 4, 1, 3>(), kernel_of<1, false, 4, 1, 3>()},
    {kernel_of<4, true, 4, 1, 2>(), kernel_of<4, false, 4, 1, 2>(), kernel_of<1, false, 4, 1, 2>()},
    {kernel_of<4, true, 4, 1, 1>(), kernel_of<4, false, 4, 1, 1>(), kernel_of<1, false, 4, 1, 1>()},
};

}  // namespace

int launch_bprop_filter(const FilterGradParams& p, float* dfilt, float alpha, void* stream)
{
    const int shape = p.tile_o == 128 ? 0 : p.tile_o == 96 ? 1 : p.tile_o == 64 ? 2 : p.tile_o == 32 ? 3 : -1;
    if (shape < 0) return (int)hipErrorInvalidValue;
    const FilterGradFn fn = kKernels[shape][(p.vec && p.uniform) ? 0 : p.vec ? 1 : 2];
    const uint32_t lds = (uint32_t)kRingStages * kStageBytes;
    hipError_t err = hipSuccess;
    if (lds > 48u * 1024u) {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(fn), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)lds);
        if (err != hipSuccess) return (int)err;
    }
    hipLaunchKernelGGL(fn, dim3((unsigned)(8 * p.per_xcd)), dim3(256), lds, static_cast<hipStream_t>(stream), p);
    err = hipGetLastError();
    if (err != hipSuccess) return (int)err;
    const size_t n = (size_t)p.K * (size_t)p.No;
    if (n % 4 == 0 && n >= ((size_t)1 << 18)) {
        const size_t n4 = n / 4;
        hipLaunchKernelGGL(sum_partial_gradients_wide, dim3((unsigned)((n4 + 255) / 256)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), reinterpret_cast<const f32x4*>(p.part),
                           reinterpret_cast<f32x4*>(dfilt), n4, p.splits, alpha);
    } else {
        hipLaunchKernelGGL(sum_partial_gradients, dim3((unsigned)((n + 31) / 32)), dim3(256), 0,
                           static_cast<hipStream_t>(stream), p.part, dfilt, n, p.splits, alpha);
    }
    return (int)hipGetLastError();
}

}  // namespace mdnn
