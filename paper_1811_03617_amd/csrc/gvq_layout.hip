// Gradient flattening of GradiVeQ (Section 2, first paragraphs, and Fig. 2a): the gradient of a
// convolution layer with F filters of depth D, height H, width W is laid out so that the F
// gradients at the same (depth, row, column) position of the F filters are adjacent; these
// groups follow each other along the depth first, then the width, then the height:
//     flat[((h*W + w)*D + d)*F + f] = grad[f][d][h][w]          (grad stored [F][D][H][W])
// That is the order in which neighbouring numbers are linearly correlated, which is what the
// slice-wise PCA lives on.  Pure permutation; bound by HBM.
//
// One work-group moves a tile of TF filters x TD depths x all H*W positions through LDS: it
// reads, for each filter, the contiguous run grad[f][d0 .. d0+TD) (TD*H*W numbers) and writes,
// for each (h, w, d), the TF adjacent numbers of the flat layout.  LDS rows get an odd stride,
// so both directions are free of bank conflicts.
#include "gvq_internal.h"

#define LAYOUT_THREADS 256
#define LAYOUT_TF 64
#define LAYOUT_LDS_ELEMS 8192   // 32-bit words of LDS per work-group

struct LayoutArgs {
    const void* src;
    void* dst;
    int F, D, HW, TD, RS;   // RS: LDS row stride (odd, >= TD*HW)
    int n_dtiles;
};

template <typename T, bool FLATTEN>
__global__ __launch_bounds__(LAYOUT_THREADS) void conv_layout_kernel(LayoutArgs a)
{
    extern __shared__ unsigned int tile_raw[];
    T* tile = (T*)tile_raw;   // [TF][RS]
    const int ft = blockIdx.x / a.n_dtiles, dt = blockIdx.x % a.n_dtiles;
    const int f0 = ft * LAYOUT_TF, d0 = dt * a.TD;
    const int nf = a.F - f0 < LAYOUT_TF ? a.F - f0 : LAYOUT_TF;
    const int nd = a.D - d0 < a.TD ? a.D - d0 : a.TD;
    const int run = nd * a.HW;                 // contiguous numbers per filter in the [F][D][H][W] layout
    const T* grad = (const T*)(FLATTEN ? a.src : a.dst);   // the [F][D][H][W] side
    const T* flat = (const T*)(FLATTEN ? a.dst : a.src);   // the flat side
    if (FLATTEN) {
        for (int i = threadIdx.x; i < nf * run; i += LAYOUT_THREADS) {
            const int f = i / run, r = i - f * run;
            tile[f * a.RS + r] = grad[((size_t)(f0 + f) * a.D + d0) * a.HW + r];
        }
        __syncthreads();
        for (int i = threadIdx.x; i < run * nf; i += LAYOUT_THREADS) {
            const int g = i / nf, f = i - g * nf;            // g = (hw, d) group, f innermost
            const int hw = g / nd, dd = g - hw * nd;
            ((T*)a.dst)[((size_t)hw * a.D + d0 + dd) * a.F + f0 + f] = tile[f * a.RS + dd * a.HW + hw];
        }
    } else {
        for (int i = threadIdx.x; i < run * nf; i += LAYOUT_THREADS) {
            const int g = i / nf, f = i - g * nf;
            const int hw = g / nd, dd = g - hw * nd;
            tile[f * a.RS + dd * a.HW + hw] = flat[((size_t)hw * a.D + d0 + dd) * a.F + f0 + f];
        }
        __syncthreads();
        for (int i = threadIdx.x; i < nf * run; i += LAYOUT_THREADS) {
            const int f = i / run, r = i - f * run;
            ((T*)a.dst)[((size_t)(f0 + f) * a.D + d0) * a.HW + r] = tile[f * a.RS + r];
        }
    }
}

// H*W too large for an LDS tile: one thread per number (correct, not fast).
template <typename T, bool FLATTEN>
__global__ void conv_layout_direct_kernel(const T* src, T* dst, int F, int D, int HW)
{
    const size_t n = (size_t)F * D * HW;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
        const int f = (int)(i % F);          // i indexes the flat side
        const size_t g = i / F;
        const int dd = (int)(g % D), hw = (int)(g / D);
        const size_t j = ((size_t)f * D + dd) * HW + hw;
        if (FLATTEN) dst[i] = src[j]; else dst[j] = src[i];
    }
}

template <typename T, bool FLATTEN>
static int launch_layout(const void* src, void* dst, int F, int D, int HW, hipStream_t st)
{
    if ((int64_t)LAYOUT_TF * HW > LAYOUT_LDS_ELEMS) {
        const size_t n = (size_t)F * D * HW;
        int grid = (int)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
        hipLaunchKernelGGL((conv_layout_direct_kernel<T, FLATTEN>), dim3(grid), dim3(256), 0, st, (const T*)src,
                           (T*)dst, F, D, HW);
        GVQ_HIP(hipGetLastError());
        return GVQ_OK;
    }
    LayoutArgs a;
    a.src = src; a.dst = dst; a.F = F; a.D = D; a.HW = HW;
    int td = LAYOUT_LDS_ELEMS / (LAYOUT_TF * HW);
    if (td > 16) td = 16;
    if (td > D) td = D;
    while (td > 1 && (int64_t)LAYOUT_TF * ((td * HW) | 1) > LAYOUT_LDS_ELEMS) --td;
    a.TD = td;
    a.RS = (td * HW) | 1;
    a.n_dtiles = (D + td - 1) / td;
    const int n_ftiles = (F + LAYOUT_TF - 1) / LAYOUT_TF;
    const size_t lds = sizeof(unsigned int) * (size_t)LAYOUT_TF * a.RS;
    hipLaunchKernelGGL((conv_layout_kernel<T, FLATTEN>), dim3(n_ftiles * a.n_dtiles), dim3(LAYOUT_THREADS), lds, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

int gvq_launch_layout(const void* src, void* dst, int F, int D, int HW, gvq_dtype_t dtype, bool flatten,
                      hipStream_t st)
{
    if (dtype == GVQ_BF16)
        return flatten ? launch_layout<unsigned short, true>(src, dst, F, D, HW, st)
                       : launch_layout<unsigned short, false>(src, dst, F, D, HW, st);
    return flatten ? launch_layout<unsigned int, true>(src, dst, F, D, HW, st)
                   : launch_layout<unsigned int, false>(src, dst, F, D, HW, st);
}
