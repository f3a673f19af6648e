// Data gradient (BPROP with respect to the input) built on the FPROP kernels.
//
// The maxDNN paper only states the belief that its techniques carry over to
// BPROP (abstract, Section 3.5).  For the gradient with respect to the input
// they carry over literally: with the filter bank turned over and its channel
// and filter roles swapped,
//     F'[o][ky'][kx'][c] = filt[c][Sk-1-ky'][Sk-1-kx'][o],
// the gradient is itself a stride-1 forward convolution (Section 2) of the
// output gradient -- zero-dilated by the forward stride -- with pad Sk-1-pad:
//     din[c][iy][ix][n] = alpha * sum_{o,ky',kx'} D[o][iy-(Sk-1-pad)+ky'][ix-(Sk-1-pad)+kx'][n] * F'[o][ky'][kx'][c],
//     D[o][stride*y][stride*x][n] = dout[o][y][x][n], zero elsewhere.
// So the implicit-GEMM kernel, its offset table and its zero-apron handling are
// reused unchanged; this file only holds the small layout kernels around it.
// Stride 1: one transpose of the filter bank into the caller's workspace.
// Stride s > 1: dilating dout would make the matrix cores multiply s*s - 1
// inserted zeros per value; instead the input pixels are split by the residue
// class of (iy + pad, ix + pad) modulo s, every class is a stride-1 correlation
// of dout with its own ceil(Sk/s)^2 sub-filter, all classes run as one forward
// convolution with s*s*Nc filters, and that convolution's epilogue stores every
// value straight to its interleaved place in din (the kernel's scatter mode), so
// the per-class results never exist in memory; the few pixels beyond the last
// window, which no class reaches, are set to zero by a small kernel here.
#include <hip/hip_runtime.h>

#include <mutex>

#include "mdnn_internal.h"

namespace mdnn {
namespace {

// Workspace of the allocation-free data-gradient entry point: the rearranged filter bank of one call.  One copy per GPU, held from the moment
// the library's code is loaded there until the process ends.  In host code this name is only a
// handle for hipGetSymbolAddress(); the device address it yields is what kernels are given.
constexpr size_t kStaticScratchBytes = MDNN_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
std::mutex scratch_lock;
void*      scratch_addr[kMaxDevices];      // device address of `scratch` on each GPU, once looked up

// F'[(o*SkSk + t')*Nc + c] = filt[(c*SkSk + SkSk-1-t')*No + o]: per tap a No x Nc
// transpose, through a padded LDS tile so that both sides are coalesced.
__global__ void __launch_bounds__(256) flip_transpose_filters(const float* __restrict__ filt,
                                                              float* __restrict__ ft,
                                                              int Nc, int No, int SkSk)
{
    __shared__ float tile[32][33];
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
    // blockIdx.x walks the 32 x 32 blocks of the No x Nc matrix of every tap (grids are limited to
    // 65535 in y and z, which a large filter's tap count or channel count could exceed)
    const int o_blocks = (No + 31) / 32, c_blocks = (Nc + 31) / 32;
    const int per_tap = o_blocks * c_blocks;
    const int tap = (int)(blockIdx.x / (unsigned)per_tap);      // destination tap t'
    const int rem = (int)(blockIdx.x - (unsigned)tap * (unsigned)per_tap);
    const int src_tap = SkSk - 1 - tap;
    const int c0 = (rem / o_blocks) * 32, o0 = (rem % o_blocks) * 32;
#pragma unroll
    for (int j = 0; j < 32; j += 8) {
        const int c = c0 + ty + j, o = o0 + tx;
        tile[ty + j][tx] = (c < Nc && o < No) ? filt[((size_t)c * SkSk + src_tap) * No + o] : 0.0f;
    }
    __syncthreads();
#pragma unroll
    for (int j = 0; j < 32; j += 8) {
        const int o = o0 + ty + j, c = c0 + tx;
        if (o < No && c < Nc) ft[((size_t)o * SkSk + tap) * Nc + c] = tile[tx][ty + j];
    }
}

// Stride s > 1.  An input row iy only meets the taps ky = ry + s*t with ry = (iy + pad) % s, and
// then the output rows y = (iy + pad)/s - t: per residue class (ry, rx) the gradient is a
// stride-1 correlation of dout with a T x T sub-filter, T = ceil(Sk/s).  All s*s classes read the
// same dout with the same geometry, so they run as ONE forward convolution with s*s*Nc "filters":
// row k' = (o*T + ty')*T + tx', column cls*Nc + c of the bank built here holds
// filt[c][ry + s*(T-1-ty')][rx + s*(T-1-tx')][o], or 0 where that tap does not exist.
__global__ void __launch_bounds__(256) class_filters(const float* __restrict__ filt, float* __restrict__ fc,
                                                     int Nc, int No, int Sk, int stride, int T)
{
    const int    cols  = stride * stride * Nc;
    const size_t total = (size_t)No * T * T * cols;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int    col = (int)(i % cols);
        const size_t k   = i / cols;
        const int    cls = col / Nc, c = col - cls * Nc;
        const int    ry  = cls / stride, rx = cls - ry * stride;
        const int    o   = (int)(k / (T * T));
        const int    r   = (int)(k - (size_t)o * T * T);
        const int    ty  = r / T, tx = r - ty * T;
        const int    ky  = ry + stride * (T - 1 - ty);
        const int    kx  = rx + stride * (T - 1 - tx);
        fc[i] = (ky < Sk && kx < Sk) ? filt[(((size_t)c * Sk + ky) * Sk + kx) * No + o] : 0.0f;
    }
}

// din[c][iy][ix][n] = 0 for the pixels beyond the last window (iy >= y_end or ix >= x_end): no
// residue class has a value for them, so the scattering convolution never writes them.
__global__ void __launch_bounds__(256) zero_unreached(float* __restrict__ din, int Nc, int Hi, int Wi, int Nb,
                                                      int y_end, int x_end)
{
    // the bottom strip of every channel (whole rows), then the right strip of the rows above it
    const size_t bottom = (size_t)(Hi - y_end) * Wi * Nb;             // per channel
    const size_t right  = (size_t)y_end * (Wi - x_end) * Nb;          // per channel
    const size_t total  = (size_t)Nc * (bottom + right);
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const size_t c = i / (bottom + right);
        size_t       r = i - c * (bottom + right);
        size_t       e;
        if (r < bottom) {
            e = ((size_t)c * Hi + y_end) * Wi * Nb + r;
        } else {
            r -= bottom;
            const size_t per_row = (size_t)(Wi - x_end) * Nb;
            const size_t iy = r / per_row;
            e = (((size_t)c * Hi + iy) * Wi + x_end) * Nb + (r - iy * per_row);
        }
        din[e] = 0.0f;
    }
}

}  // namespace

int static_scratch(void** ptr)
{
    int dev = 0;
    hipError_t err = hipGetDevice(&dev);
    if (err != hipSuccess) return (int)err;
    if (dev < 0 || dev >= kMaxDevices) return (int)hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(scratch_lock);
    if (!scratch_addr[dev]) {
        // each GPU has its own copy of the array at its own address: look it up with that GPU current
        void* p = nullptr;
        err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (err != hipSuccess) return (int)err;
        scratch_addr[dev] = p;
    }
    *ptr = scratch_addr[dev];
    return 0;
}

int launch_flip_transpose(const float* filt, float* ft, int Nc, int No, int SkSk, void* stream)
{
    // one workgroup per 32 x 32 block and tap: the bank holds fewer than 2^29 floats, so fewer than 2^31 blocks
    const dim3 grid((unsigned)((size_t)((No + 31) / 32) * ((Nc + 31) / 32) * SkSk));
    hipLaunchKernelGGL(flip_transpose_filters, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       filt, ft, Nc, No, SkSk);
    return (int)hipGetLastError();
}

int launch_class_filters(const float* filt, float* fc, int Nc, int No, int Sk, int stride, int T, void* stream)
{
    const size_t total = (size_t)No * T * T * stride * stride * Nc;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256u * 64u) blocks = 256u * 64u;          // grid-stride beyond that
    hipLaunchKernelGGL(class_filters, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       filt, fc, Nc, No, Sk, stride, T);
    return (int)hipGetLastError();
}

int launch_zero_unreached(float* din, int Nc, int Hi, int Wi, int Nb, int y_end, int x_end, void* stream)
{
    if (y_end > Hi) y_end = Hi;
    if (x_end > Wi) x_end = Wi;
    const size_t total = (size_t)Nc * ((size_t)(Hi - y_end) * Wi + (size_t)y_end * (Wi - x_end)) * Nb;
    if (total == 0) return 0;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256u * 64u) blocks = 256u * 64u;          // grid-stride beyond that
    hipLaunchKernelGGL(zero_unreached, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       din, Nc, Hi, Wi, Nb, y_end, x_end);
    return (int)hipGetLastError();
}

}  // namespace mdnn
