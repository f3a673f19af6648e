// FPROP convolution kernels for gfx950 (MI355X): implicit GEMM on the FP32
// matrix cores.
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
#include <hip/hip_runtime.h>

#include "mdnn_internal.h"

namespace mdnn {

typedef float    f32x16 __attribute__((ext_vector_type(16)));
typedef float    f32x4  __attribute__((ext_vector_type(4)));
typedef float    f32x2  __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4  __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kOutOfRange = 0xFFFFFFFFu;   // beyond any buffer of < 2^32 bytes
constexpr int      kRsrcWord3  = 0x00020000;    // raw 32-bit-data buffer descriptor, gfx9 family

__device__ __forceinline__ f32x4 buf_load4(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)byte_off, 0, 0));
}
__device__ __forceinline__ float buf_load1(__amdgpu_buffer_rsrc_t r, uint32_t byte_off)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)byte_off, 0, 0));
}

template <int N> struct VecOf;
template <> struct VecOf<1> { typedef float type; };
template <> struct VecOf<2> { typedef f32x2 type; };
template <> struct VecOf<4> { typedef f32x4 type; };

// WO x WM waves per workgroup; each wave owns RA x RB MFMA blocks of 32x32;
// KS patch columns per pipeline step; VEC = 16-byte global accesses.
template <int WO_, int WM_, int RA_, int RB_, int KS_, bool VEC_>
struct Cfg {
    static constexpr int  WO = WO_, WM = WM_, RA = RA_, RB = RB_, KS = KS_;
    static constexpr bool VEC = VEC_;
    static constexpr int  NT = 64 * WO * WM;          // threads
    static constexpr int  TO = WO * RA * 32;          // tile rows (filters)
    static constexpr int  TM = WM * RB * 32;          // tile columns (flat m)
    static constexpr int  OG = TO / 4;                // float4 groups per filter-slab row
    static constexpr int  A_V4 = KS * OG;             // float4s in a filter slab
    static constexpr int  NA = (A_V4 + NT - 1) / NT;  // filter float4s per thread per slab
    static constexpr int  MG = TM / 4;                // float4 column groups of the patch slab
    static constexpr int  BROWS = NT / MG;            // patch rows covered by one pass of the WG
    static constexpr int  NB = KS / BROWS;            // patch float4s per thread per slab
    static constexpr int  CS = VEC ? 1 : 4;           // column states per thread
    static_assert(NT % MG == 0 && KS % BROWS == 0 && KS % 2 == 0, "tile shape");
    static_assert(RB == 1 || RB == 2 || RB == 4, "RB");
    static constexpr uint32_t stage_bytes = 2u * KS * (TO + TM) * sizeof(float);
};

template <class C>
__global__ void __launch_bounds__(C::NT) conv_fprop_kernel(const ConvParams p)
{
    constexpr int WO = C::WO, WM = C::WM, RA = C::RA, RB = C::RB, KS = C::KS;
    constexpr int NT = C::NT, TO = C::TO, TM = C::TM, OG = C::OG, MG = C::MG;
    constexpr int NA = C::NA, NB = C::NB, BROWS = C::BROWS, CS = C::CS;
    constexpr bool VEC = C::VEC;
    (void)WM;

    extern __shared__ __align__(16) unsigned char lds_raw[];
    float* As  = reinterpret_cast<float*>(lds_raw);          // [2][KS][TO]
    float* Bs  = As + 2 * KS * TO;                           // [2][KS][TM]
    int2*  tab = reinterpret_cast<int2*>(Bs + 2 * KS * TM);  // [tab_cap] {byte offset, ky<<16|kx}

    // ---- tile map.  Workgroups are dealt round-robin to the 8 XCDs, each with
    // its own L2: give every XCD a contiguous run of tiles so that neighbouring
    // output coordinates (overlapping patches) and the filter tiles of one
    // coordinate (same patch) meet in the same L2.
    const int bid  = blockIdx.x;
    const int tile = (bid & 7) * p.tiles_per_xcd + (bid >> 3);
    if (tile >= p.n_tiles) return;                           // uniform per workgroup
    const int mt = tile / p.n_otiles;
    const int ot = tile - mt * p.n_otiles;
    const int o0 = ot * TO;
    const int m0 = mt * TM;

    const int t    = threadIdx.x;
    const int lane = t & 63;
    const int wave = t >> 6;
    const int wo   = wave % WO;
    const int wm   = wave / WO;

    const __amdgpu_buffer_rsrc_t rin =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.in), 0, (int)p.in_bytes, kRsrcWord3);
    const __amdgpu_buffer_rsrc_t rfl =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(p.filt), 0, (int)p.filt_bytes, kRsrcWord3);

    // ---- this thread's patch columns: fixed for the whole tile.
    const int q    = t % MG;          // float4 column group inside the tile
    const int brow = t / MG;          // first patch row this thread copies in each pass
    uint32_t pbase[CS];               // byte offset of the patch origin (+n) in `in`, mod 2^32
    int      iy0[CS], ix0[CS];        // image row/col of tap (0,0); far negative when the column is past M
#pragma unroll
    for (int cs = 0; cs < CS; ++cs) {
        const int m = m0 + 4 * q + cs;
        if (m < p.M) {
            const int pix = m / p.Nb;
            const int n   = m - pix * p.Nb;
            const int y   = pix / p.Wo;
            const int x   = pix - y * p.Wo;
            iy0[cs] = y * p.stride - p.pad;
            ix0[cs] = x * p.stride - p.pad;
            // modulo 2^32 on purpose: negative apron origins wrap and wrap back once a valid tap is added
            pbase[cs] = (((uint32_t)iy0[cs] * (uint32_t)p.Wi + (uint32_t)ix0[cs]) * (uint32_t)p.Nb + (uint32_t)n) * 4u;
        } else {
            iy0[cs] = -(1 << 30);
            ix0[cs] = -(1 << 30);
            pbase[cs] = 0;
        }
    }

    f32x16 acc[RA][RB];
#pragma unroll
    for (int a = 0; a < RA; ++a)
#pragma unroll
        for (int b = 0; b < RB; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    f32x4 ga[NA], gb[NB];             // global -> LDS staging registers

    // filter slab rows k0..k0+KS-1, columns o0..o0+TO-1 (plain GEMM operand)
    auto load_A = [&](int k0) {
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int e = t + i * NT;
            const int r = e / OG;
            const int c = e - r * OG;
            const int k = k0 + r;
            const int o = o0 + 4 * c;
            if ((C::A_V4 % NT) != 0 && e >= C::A_V4) { ga[i] = f32x4{0, 0, 0, 0}; continue; }
            if (VEC) {
                const bool ok = (k < p.K) && (o < p.No);
                ga[i] = buf_load4(rfl, ok ? (uint32_t)(k * p.No + o) * 4u : kOutOfRange);
            } else {
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const bool ok = (k < p.K) && (o + j < p.No);
                    ga[i][j] = buf_load1(rfl, ok ? (uint32_t)(k * p.No + o + j) * 4u : kOutOfRange);
                }
            }
        }
    };
    // patch slab: row k of the unrolled patch for this thread's columns,
    // address = patch base + table[k]; zero when the tap is in the apron.
    auto load_B = [&](int k0, int kc) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const int  k  = k0 + brow + i * BROWS;
            const int2 e  = tab[k - kc];
            const int  ky = e.y >> 16;
            const int  kx = e.y & 0xFFFF;
#pragma unroll
            for (int cs = 0; cs < CS; ++cs) {
                const bool ok = (k < p.K) && ((uint32_t)(iy0[cs] + ky) < (uint32_t)p.Hi) &&
                                ((uint32_t)(ix0[cs] + kx) < (uint32_t)p.Wi);
                const uint32_t off = ok ? pbase[cs] + (uint32_t)e.x : kOutOfRange;
                if (VEC) gb[i] = buf_load4(rin, off);
                else     gb[i][cs] = buf_load1(rin, off);
            }
        }
    };
    auto store_AB = [&](int stage) {
        float* as = As + stage * KS * TO;
        float* bs = Bs + stage * KS * TM;
#pragma unroll
        for (int i = 0; i < NA; ++i) {
            const int e = t + i * NT;
            if ((C::A_V4 % NT) != 0 && e >= C::A_V4) continue;
            *reinterpret_cast<f32x4*>(as + 4 * e) = ga[i];          // row-major [KS][TO], e*4 == r*TO + 4c
        }
#pragma unroll
        for (int i = 0; i < NB; ++i)
            *reinterpret_cast<f32x4*>(bs + (brow + i * BROWS) * TM + 4 * q) = gb[i];
    };

    // One slab on the matrix cores.  MFMA 32x32x2: lane l supplies A[l%32][l/32]
    // and B[l/32][l%32]; rows = filters, columns = flat m.  Column block b of a
    // wave holds m = base + RB*(l%32) + b, so one RB-wide LDS read feeds all RB
    // column blocks and the RB results of a lane are adjacent in memory.
    const int half = lane >> 5;
    const int l32  = lane & 31;
    auto compute = [&](int stage) {
        const float* as = As + stage * KS * TO + half * TO + wo * (RA * 32) + l32;
        const float* bs = Bs + stage * KS * TM + half * TM + wm * (RB * 32) + l32 * RB;
#pragma unroll
        for (int kk = 0; kk < KS; kk += 2) {
            float av[RA];
            typename VecOf<RB>::type bv;
#pragma unroll
            for (int a = 0; a < RA; ++a) av[a] = as[kk * TO + a * 32];
            bv = *reinterpret_cast<const typename VecOf<RB>::type*>(bs + kk * TM);
#pragma unroll
            for (int a = 0; a < RA; ++a)
#pragma unroll
                for (int b = 0; b < RB; ++b) {
                    float bval;
                    if constexpr (RB == 1) bval = bv; else bval = bv[b];
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a], bval, acc[a][b], 0, 0, 0);
                }
        }
    };

    // ---- main loop over K, in table-sized chunks (one chunk unless K is huge)
    for (int kc = 0; kc < p.K; kc += p.tab_cap) {
        if (kc) __syncthreads();
        // offset table, Section 3.2: k = (c*Sk + ky)*Sk + kx  ->  ((c*Hi + ky)*Wi + kx)*Nb floats
        for (int i = t; i < p.tab_cap; i += NT) {
            const int k = kc + i;
            int2 e = make_int2(0, 0);
            if (k < p.K) {
                const int c  = k / p.SkSk;
                const int r  = k - c * p.SkSk;
                const int ky = r / p.Sk;
                const int kx = r - ky * p.Sk;
                e.x = (int)((uint32_t)((c * p.Hi + ky) * p.Wi + kx) * (uint32_t)p.Nb * 4u);
                e.y = (ky << 16) | kx;
            }
            tab[i] = e;
        }
        __syncthreads();

        const int kend = min(p.K, kc + p.tab_cap);
        const int ns   = (kend - kc + KS - 1) / KS;
        load_A(kc);
        load_B(kc, kc);
        store_AB(0);
        __syncthreads();
        for (int s = 0; s < ns; ++s) {
            const bool more = (s + 1 < ns);
            if (more) {                           // next slab's global loads fly during the MFMAs
                load_A(kc + (s + 1) * KS);
                load_B(kc + (s + 1) * KS, kc);
            }
            compute(s & 1);
            if (more) store_AB((s + 1) & 1);      // other stage: last read one barrier ago
            __syncthreads();
        }
    }

    // ---- epilogue: out = alpha * acc.  Accumulator register v of lane l in
    // block (a,b) is row 8*(v/4) + 4*(l/32) + v%4, column l%32 of the block.
    const int ocol = m0 + wm * (RB * 32) + l32 * RB;
#pragma unroll
    for (int a = 0; a < RA; ++a) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int o = o0 + wo * (RA * 32) + a * 32 + 8 * (v >> 2) + 4 * half + (v & 3);
            if (o >= p.No) continue;
            float* dst = p.out + (size_t)o * (size_t)p.M + ocol;
            if (VEC) {
                if (ocol < p.M) {                 // M % 4 == 0 and RB | 4: all or nothing
                    typename VecOf<RB>::type w;
#pragma unroll
                    for (int b = 0; b < RB; ++b) {
                        if constexpr (RB == 1) w = p.alpha * acc[a][0][v];
                        else w[b] = p.alpha * acc[a][b][v];
                    }
                    *reinterpret_cast<typename VecOf<RB>::type*>(dst) = w;
                }
            } else {
#pragma unroll
                for (int b = 0; b < RB; ++b)
                    if (ocol + b < p.M) dst[b] = p.alpha * acc[a][b][v];
            }
        }
    }
}

// ---- register-only FP32 MFMA loop: the sustained matrix rate with no memory traffic
__global__ void __launch_bounds__(256) mfma_probe_kernel(float* sink, int iters)
{
    f32x16 c0, c1, c2, c3;
#pragma unroll
    for (int v = 0; v < 16; ++v) { c0[v] = 0.f; c1[v] = 0.f; c2[v] = 0.f; c3[v] = 0.f; }
    const float a = 1.0f + (threadIdx.x & 3) * 0.25f;
    const float b = 1.0f / (float)(1 + (threadIdx.x & 7));
    for (int i = 0; i < iters; ++i) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, a, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x2f32(a, a, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x2f32(b, b, c3, 0, 0, 0);
    }
    float s = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) s += c0[v] + c1[v] + c2[v] + c3[v];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// ---- variant registry -----------------------------------------------------
typedef void (*KernelFn)(const ConvParams);

struct Entry {
    VariantInfo info;
    KernelFn    fn;
    uint32_t    stage_bytes;
};

template <class C>
constexpr Entry make_entry(const char* name, int wg_per_cu, float eff)
{
    return Entry{VariantInfo{name, C::TO, C::TM, C::KS, C::NT, C::VEC ? 1 : 0, wg_per_cu, eff},
                 &conv_fprop_kernel<C>, C::stage_bytes};
}

//                         WO WM RA RB KS  VEC
typedef Cfg<2, 2, 2, 2, 16, true>  C_o128m128;
typedef Cfg<2, 2, 4, 2, 16, true>  C_o256m128;
typedef Cfg<2, 2, 2, 4, 16, true>  C_o128m256;
typedef Cfg<1, 4, 3, 2, 16, true>  C_o96m256;
typedef Cfg<1, 4, 2, 2, 16, true>  C_o64m256;
typedef Cfg<1, 4, 1, 1, 16, true>  C_o32m128;
typedef Cfg<2, 2, 1, 1, 16, false> C_o64m64s;

const Entry kEntries[] = {
    make_entry<C_o128m128>("o128m128", 2, 0.85f),
    make_entry<C_o256m128>("o256m128", 2, 0.88f),
    make_entry<C_o128m256>("o128m256", 2, 0.88f),
    make_entry<C_o96m256>("o96m256", 2, 0.85f),
    make_entry<C_o64m256>("o64m256", 2, 0.80f),
    make_entry<C_o32m128>("o32m128", 4, 0.50f),
    make_entry<C_o64m64s>("o64m64s", 4, 0.30f),
};
constexpr int kNumEntries = (int)(sizeof(kEntries) / sizeof(kEntries[0]));

}  // namespace

int variant_count() { return kNumEntries; }
const VariantInfo& variant_info(int i) { return kEntries[i].info; }
uint32_t variant_lds_bytes(int i, int tab_cap)
{
    return kEntries[i].stage_bytes + (uint32_t)tab_cap * (uint32_t)sizeof(int2);
}

int launch_variant(int i, const ConvParams& p, void* stream)
{
    const Entry& e = kEntries[i];
    const uint32_t lds = variant_lds_bytes(i, p.tab_cap);
    hipError_t err = hipSuccess;
    if (lds > 48u * 1024u) {
        err = hipFuncSetAttribute(reinterpret_cast<const void*>(e.fn),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (err != hipSuccess) return (int)err;
    }
    const dim3 grid((unsigned)(8 * p.tiles_per_xcd)), block((unsigned)e.info.threads);
    hipLaunchKernelGGL(e.fn, grid, block, lds, static_cast<hipStream_t>(stream), p);
    err = hipGetLastError();
    return (int)err;
}

int launch_mfma_probe(float* sink, int blocks, int waves_per_block, int iters, void* stream)
{
    hipLaunchKernelGGL(mfma_probe_kernel, dim3((unsigned)blocks), dim3((unsigned)(64 * waves_per_block)),
                       0, static_cast<hipStream_t>(stream), sink, iters);
    return (int)hipGetLastError();
}

}  // namespace mdnn
