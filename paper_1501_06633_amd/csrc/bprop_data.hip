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
// reused unchanged; this file only holds the two small layout kernels that
// prepare F' and D in the caller's workspace.  For stride 1, D is dout itself.
// For stride s > 1 the matrix cores also multiply the inserted zeros (s*s times
// the necessary work): correct, not yet efficient.
#include <hip/hip_runtime.h>

#include "mdnn_internal.h"

namespace mdnn {
namespace {

// F'[(o*SkSk + t')*Nc + c] = filt[(c*SkSk + SkSk-1-t')*No + o]: per tap a No x Nc
// transpose, through a padded LDS tile so that both sides are coalesced.
__global__ void __launch_bounds__(256) flip_transpose_filters(const float* __restrict__ filt,
                                                              float* __restrict__ ft,
                                                              int Nc, int No, int SkSk)
{
    __shared__ float tile[32][33];
    const int tap = blockIdx.z;                 // destination tap t'
    const int src_tap = SkSk - 1 - tap;
    const int c0 = blockIdx.y * 32, o0 = blockIdx.x * 32;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;     // 32 x 8
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

// D[o][ty][tx][n] = dout[o][ty/s][tx/s][n] where both are multiples of s and inside, else 0.
__global__ void __launch_bounds__(256) dilate_gradient(const float* __restrict__ dout,
                                                       float* __restrict__ d,
                                                       int No, int Ho, int Wo, int Hd, int Wd, int Nb, int stride)
{
    const size_t total = (size_t)No * Hd * Wd * Nb;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total;
         i += (size_t)gridDim.x * blockDim.x) {
        const int    n   = (int)(i % Nb);
        const size_t pix = i / Nb;
        const int    tx  = (int)(pix % Wd);
        const size_t r   = pix / Wd;
        const int    ty  = (int)(r % Hd);
        const int    o   = (int)(r / Hd);
        float v = 0.0f;
        if (ty % stride == 0 && tx % stride == 0) {
            const int y = ty / stride, x = tx / stride;
            if (y < Ho && x < Wo) v = dout[(((size_t)o * Ho + y) * Wo + x) * Nb + n];
        }
        d[i] = v;
    }
}

}  // namespace

int launch_flip_transpose(const float* filt, float* ft, int Nc, int No, int SkSk, void* stream)
{
    const dim3 grid((unsigned)((No + 31) / 32), (unsigned)((Nc + 31) / 32), (unsigned)SkSk);
    hipLaunchKernelGGL(flip_transpose_filters, grid, dim3(256), 0, static_cast<hipStream_t>(stream),
                       filt, ft, Nc, No, SkSk);
    return (int)hipGetLastError();
}

int launch_dilate(const float* dout, float* d, int No, int Ho, int Wo, int Hd, int Wd, int Nb, int stride,
                  void* stream)
{
    const size_t total = (size_t)No * Hd * Wd * Nb;
    size_t blocks = (total + 255) / 256;
    if (blocks > 256u * 64u) blocks = 256u * 64u;          // grid-stride beyond that
    hipLaunchKernelGGL(dilate_gradient, dim3((unsigned)blocks), dim3(256), 0, static_cast<hipStream_t>(stream),
                       dout, d, No, Ho, Wo, Hd, Wd, Nb, stride);
    return (int)hipGetLastError();
}

}  // namespace mdnn
