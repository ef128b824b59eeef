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

typedef float f4 __attribute__((ext_vector_type(4)));

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

// 16-byte aligned sides, F and D*H*W multiples of V = 16 / sizeof(T) (4 for fp32, 8 for bf16): the same tile scheme
// with 128-bit global accesses and no division per element.  LDS holds the tile in the flat order, tile[g][f],
// g = hw * nd + dd the position inside the tile and f fastest (row stride TF + V elements: 128-bit rows, and 8 lanes x
// 128 bits cover all banks).  On the [F][D][H][W] side a thread moves V consecutive numbers of one filter's run (and
// scatters them to, or gathers them from, V rows of the tile); on the flat side a thread moves V adjacent filters of
// one row.  A tile is TD depths x all H*W positions, or, when H*W alone is longer than a tile (and a multiple of V),
// one depth x a piece of H*W; either way a filter's part of it is one contiguous run.
#define LF_BYTES 32768          // LDS per work-group

struct LayoutFastArgs {
    const void* src;
    void* dst;
    int F, D, HW, TD;           // TD * HWT is a multiple of V and at most LF_BYTES / sizeof(T) / (TF + V)
    int n_dtiles;
    int HWT, n_hwtiles;         // positions per tile: H*W (one tile over them), or a multiple of V when H*W is too long
                                // for one tile (then TD = 1)
};

typedef unsigned int lu4 __attribute__((ext_vector_type(4)));

// TF: filters per tile (a row of the flat side is TF elements contiguous)
template <typename T, bool FLATTEN, int TF>
__global__ __launch_bounds__(LAYOUT_THREADS) void conv_layout_fast_kernel(LayoutFastArgs a)
{
    extern __shared__ lu4 ftile_raw[];
    T* ftile = (T*)ftile_raw;   // [run][RS]
    constexpr int V = 16 / sizeof(T), RS = TF + V, QF = TF / V, ROWS = LAYOUT_THREADS / QF;
    union Vec { lu4 v; T e[V]; };
    const int tid = threadIdx.x;
    const int ht = blockIdx.x % a.n_hwtiles, fd = blockIdx.x / a.n_hwtiles;
    const int ft = fd / a.n_dtiles, dt = fd % a.n_dtiles;
    const int f0 = ft * TF, d0 = dt * a.TD, hw0 = ht * a.HWT;
    const int nf = a.F - f0 < TF ? a.F - f0 : TF;             // a multiple of V
    const int nd = a.D - d0 < a.TD ? a.D - d0 : a.TD;
    const int nhw = a.HW - hw0 < a.HWT ? a.HW - hw0 : a.HWT;
    const int run = nd * nhw, rq = run / V;                  // run: a multiple of V, contiguous in a filter (nd = 1 or nhw = H*W)
    const T* grad = (const T*)(FLATTEN ? a.src : a.dst);
    const T* flat = (const T*)(FLATTEN ? a.dst : a.src);
    // the [F][D][H][W] side: this thread's chunk c of a run, for filters fsub, fsub + fpp, ...
    const int fpp = LAYOUT_THREADS / rq, fsub = tid / rq, c = tid - fsub * rq;
    int g[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
        const int r = V * c + i, dd = r / nhw, hw = r - dd * nhw;
        g[i] = (hw * nd + dd) * RS;
    }
    // the flat side: V adjacent filters q of rows gr, gr + ROWS, ...
    const int q = tid % QF, gr = tid / QF;
    auto grad_ptr = [&](int f) { return (T*)grad + ((size_t)(f0 + f) * a.D + d0) * a.HW + hw0 + V * c; };
    auto flat_rows = [&](auto&& body) {
        int hw = gr / nd, dd = gr - hw * nd;
        for (int gg = gr; gg < run; gg += ROWS) {
            if (V * q < nf) body(gg, (T*)flat + ((size_t)(hw0 + hw) * a.D + d0 + dd) * a.F + f0 + V * q);
            dd += ROWS;
            while (dd >= nd) { dd -= nd; ++hw; }
        }
    };
    if (FLATTEN) {
        if (fsub < fpp)
            for (int f = fsub; f < nf; f += fpp) {
                Vec x;
                x.v = __builtin_nontemporal_load((const lu4*)grad_ptr(f));
#pragma unroll
                for (int i = 0; i < V; ++i) ftile[g[i] + f] = x.e[i];
            }
        __syncthreads();
        flat_rows([&](int gg, T* p) { __builtin_nontemporal_store(*(const lu4*)(ftile + gg * RS + V * q), (lu4*)p); });
    } else {
        flat_rows([&](int gg, T* p) { *(lu4*)(ftile + gg * RS + V * q) = __builtin_nontemporal_load((const lu4*)p); });
        __syncthreads();
        if (fsub < fpp)
            for (int f = fsub; f < nf; f += fpp) {
                Vec x;
#pragma unroll
                for (int i = 0; i < V; ++i) x.e[i] = ftile[g[i] + f];
                __builtin_nontemporal_store(x.v, (lu4*)grad_ptr(f));
            }
    }
}

// Depths per tile for the kernel above with at most max_run rows (a multiple of V), or 0 when the shape does not fit
// it; *hwt: the positions per tile.
static int layout_fast_td(const void* src, const void* dst, int F, int D, int HW, int V, int max_run, int* hwt)
{
    *hwt = HW;
    if ((((uintptr_t)src | (uintptr_t)dst) & 15) || F % V || ((int64_t)D * HW) % V) return 0;
    if (HW > max_run) {   // one depth per tile, H*W in pieces
        if (HW % V) return 0;
        *hwt = max_run;
        return 1;
    }
    int step = V;                                  // TD * HW must be a multiple of V: TD of V / gcd(HW, V)
    while (step > 1 && (HW * (step / 2)) % V == 0) step /= 2;
    int td = max_run / HW / step * step;
    if (td < step) return 0;
    if (td >= D) return D;                         // one depth tile: D * HW is a multiple of V
    return td;
}

template <typename T, bool FLATTEN, int TF>
static int launch_layout_fast(const void* src, void* dst, int F, int D, int HW, int td, int hwt, hipStream_t st)
{
    LayoutFastArgs a;
    a.src = src; a.dst = dst; a.F = F; a.D = D; a.HW = HW; a.TD = td;
    a.n_dtiles = (D + td - 1) / td;
    a.HWT = hwt; a.n_hwtiles = (HW + hwt - 1) / hwt;
    const int n_ftiles = (F + TF - 1) / TF;
    const size_t lds = sizeof(T) * (size_t)td * hwt * (TF + 16 / sizeof(T));
    const int64_t grid = (int64_t)n_ftiles * a.n_dtiles * a.n_hwtiles;
    if (grid > 0x7fffffff) return GVQ_EINVAL;
    hipLaunchKernelGGL((conv_layout_fast_kernel<T, FLATTEN, TF>), dim3((unsigned)grid), dim3(LAYOUT_THREADS), lds,
                       st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

// H*W too large for an LDS tile and not a multiple of the vector width: one thread per number (correct, not fast).
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
    {
        // 64 filters per tile; 128 for a fully connected layer when it is flattened or holds bf16 (measured on 67 - 411 MB
        // layers: fp32 flatten 4.2 - 4.6 against 3.9 TB/s, bf16 3.5 / 3.2 against 2.7 / 2.6; with H*W > 1, and for the
        // fp32 unflatten, 128 is 15 - 30 % slower)
        constexpr int V = 16 / sizeof(T);
        const int tf = HW == 1 && F >= 128 && (FLATTEN || sizeof(T) == 2) ? 128 : 64;
        int hwt = HW;
        const int td = layout_fast_td(src, dst, F, D, HW, V, LF_BYTES / (int)sizeof(T) / (tf + V) / V * V, &hwt);
        if (td > 0) {
            if (tf == 128) return launch_layout_fast<T, FLATTEN, 128>(src, dst, F, D, HW, td, hwt, st);
            return launch_layout_fast<T, FLATTEN, 64>(src, dst, F, D, HW, td, hwt, st);
        }
    }
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
