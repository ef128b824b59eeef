// Moments of the basis refresh for every slice length other than 16, 32, 64 and 128, up to
// GVQ_MAX_D (GradiVeQ Section 3, "slice size": the slice is a multiple of a layer's filters x
// depth, e.g. 768 for a (3,3,16,16) layer): sum x x^T in 64 x 64 blocks on the fp64 matrix pipe,
// one wave per (block, sample chunk), fixed-order sum of the chunks afterwards.  The
// eigendecomposition of the result is in gvq_eigen_block.hip.
#include "gvq_internal.h"

typedef double d4 __attribute__((ext_vector_type(4)));
typedef unsigned int lu4 __attribute__((ext_vector_type(4)));
typedef unsigned int lu2 __attribute__((ext_vector_type(2)));

#define LG 64                       // elements per group (one 64 x 64 block of the matrix per wave)
#define LBLOCK (LG * LG + LG)       // doubles per partial: the block, then the sums of its row group

struct MomLargeArgs {
    gvq_ptrs grads;
    int L;
    const int64_t* offs;
    int64_t M;
    int d, ng, npairs, chunks;
    int accumulate;
    double* part;   // [B][npairs][chunks][LBLOCK]
    unsigned long long* nsamp;   // [B] += the sample slices this launch took in (counted by the waves of block pair 0)
};

__device__ __forceinline__ float large_elem(const void* g, bool bf16, int64_t idx)
{
    if (bf16) return __uint_as_float((unsigned int)((const unsigned short*)g)[idx] << 16);
    return ((const float*)g)[idx];
}

// v_mfma_f64_16x16x4_f64: A lane l = (row l%16, step l/16), B lane l = (step l/16, column l%16),
// result register r of lane l = (row 4r + l/16, column l%16); the 4 steps are 4 samples.
// A "tile" may be any 16 elements of the slice: lane (m, kk) loads elements 4m..4m+3 of its
// group of 64 as one word, and register c of that word is element m of tile c, i.e. element
// 4m + c of the group.  acc[c1][c2] is then the 16 x 16 block (tile c1 of group ga) x (tile c2
// of group gb).  VEC: d is a multiple of 4, so a word lies wholly inside or outside the slice and
// slices stay word-aligned.
template <bool BF16, bool VEC>
__global__ __launch_bounds__(256, 2) void moments_large_kernel(MomLargeArgs a)
{
    const int lane = threadIdx.x & 63, m = lane & 15, kk = lane >> 4;
    const int b = blockIdx.y;
    const int64_t task = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (task >= (int64_t)a.npairs * a.chunks) return;
    const int chunk = (int)(task / a.npairs), pair = (int)(task - (int64_t)chunk * a.npairs);
    int ga = 0, rem = pair;
    while (rem >= a.ng - ga) { rem -= a.ng - ga; ++ga; }
    const int gb = ga + rem;
    const int d = a.d;

    const int64_t full = a.M / d;
    int64_t lo = a.offs[b], hi = a.offs[b + 1] < full ? a.offs[b + 1] : full;
    if (hi < lo) hi = lo;
    const int64_t cnt = hi - lo;
    const int64_t j0 = lo + cnt * chunk / a.chunks, j1 = lo + cnt * (chunk + 1) / a.chunks;

    d4 acc[4][4];
    double ssum[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = d4{0.0, 0.0, 0.0, 0.0};

    const int ea = ga * LG + 4 * m, eb = gb * LG + 4 * m;   // first element of this lane's words
    auto load_word = [&](const void* g, int64_t j, int e0, float (&x)[4]) {
        x[0] = x[1] = x[2] = x[3] = 0.f;
        if (j >= j1) return;
        if (VEC) {
            if (e0 >= d) return;
            if (BF16) {
                const lu2 v = *(const lu2*)((const unsigned short*)g + j * d + e0);
                x[0] = __uint_as_float(v.x << 16);
                x[1] = __uint_as_float(v.x & 0xffff0000u);
                x[2] = __uint_as_float(v.y << 16);
                x[3] = __uint_as_float(v.y & 0xffff0000u);
            } else {
                const lu4 v = *(const lu4*)((const float*)g + j * d + e0);
                x[0] = __uint_as_float(v.x);
                x[1] = __uint_as_float(v.y);
                x[2] = __uint_as_float(v.z);
                x[3] = __uint_as_float(v.w);
            }
        } else {
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (e0 + c < d) x[c] = large_elem(g, BF16, j * d + e0 + c);
        }
    };

    // PF groups of 4 samples are in flight ahead of the one being multiplied (one group is 1024
    // matrix-pipe cycles, a load from HBM takes several times that)
    constexpr int PF = 4;
    unsigned int taken = 0;   // samples multiplied by this lane's slot
    for (int l = 0; l < a.L; ++l) {
        const void* g = a.grads.p[l];
        float xa[PF][4], xb[PF][4];
#pragma unroll
        for (int u = 0; u < PF; ++u) {
            load_word(g, j0 + 4 * u + kk, ea, xa[u]);
            load_word(g, j0 + 4 * u + kk, eb, xb[u]);
        }
        for (int64_t j = j0; j < j1; j += 4 * PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                taken += (pair == 0 && m == 0 && j + 4 * u + kk < j1) ? 1u : 0u;
                double da[4], db[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    da[c] = (double)xa[u][c];
                    db[c] = (double)xb[u][c];
                    ssum[c] += da[c];
                }
                // this group's registers are free again: ask for the group PF further on (zeros past the range)
                load_word(g, j + 4 * (u + PF) + kk, ea, xa[u]);
                load_word(g, j + 4 * (u + PF) + kk, eb, xb[u]);
#pragma unroll
                for (int c1 = 0; c1 < 4; ++c1)
#pragma unroll
                    for (int c2 = 0; c2 < 4; ++c2)
                        acc[c1][c2] = __builtin_amdgcn_mfma_f64_16x16x4f64(da[c1], db[c2], acc[c1][c2], 0, 0, 0);
            }
        }
    }

    if (pair == 0) {
        unsigned int cnt = taken;
        cnt += __shfl_xor(cnt, 16, 64);
        cnt += __shfl_xor(cnt, 32, 64);
        if (lane == 0 && cnt) atomicAdd(a.nsamp + b, (unsigned long long)cnt);
    }
    double* out = a.part + (((size_t)b * a.npairs + pair) * a.chunks + chunk) * LBLOCK;
#pragma unroll
    for (int c1 = 0; c1 < 4; ++c1)
#pragma unroll
        for (int c2 = 0; c2 < 4; ++c2)
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                double* o = out + ((c1 * 4 + c2) * 4 + r) * 64 + lane;
                *o = a.accumulate ? *o + acc[c1][c2][r] : acc[c1][c2][r];
            }
    // sums of group ga's elements (used from the diagonal blocks only): add the 4 sample lanes
#pragma unroll
    for (int c = 0; c < 4; ++c) {
        double v = ssum[c];
        v += __shfl_xor(v, 16, 64);
        v += __shfl_xor(v, 32, 64);
        if (kk == 0) {
            double* o = out + LG * LG + 4 * m + c;
            *o = a.accumulate ? *o + v : v;
        }
    }
}

// mom[b] (d*d + d: sum x x^T, both triangles, then sum x) from the per-chunk blocks, chunks
// added in index order.
__global__ __launch_bounds__(256) void reduce_large_kernel(const double* part, double* mom, int d, int ng,
                                                           int npairs, int chunks)
{
    const int b = blockIdx.z, pair = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= LBLOCK) return;
    int ga = 0, rem = pair;
    while (rem >= ng - ga) { rem -= ng - ga; ++ga; }
    const int gb = ga + rem;
    if (i >= LG * LG && ga != gb) return;
    const double* src = part + ((size_t)b * npairs + pair) * chunks * LBLOCK + i;
    double v = 0.0;
    for (int c = 0; c < chunks; ++c) v += src[(size_t)c * LBLOCK];
    double* o = mom + (size_t)b * ((size_t)d * d + d);
    if (i >= LG * LG) {
        const int e = ga * LG + (i - LG * LG);
        if (e < d) o[(size_t)d * d + e] = v;
        return;
    }
    const int lane = i & 63, r = (i >> 6) & 3, c2 = (i >> 8) & 3, c1 = i >> 10;
    const int row = ga * LG + 4 * (4 * r + (lane >> 4)) + c1, col = gb * LG + 4 * (lane & 15) + c2;
    if (row >= d || col >= d) return;
    o[(size_t)row * d + col] = v;
    if (ga != gb) o[(size_t)col * d + row] = v;   // a diagonal block holds both of its triangles itself
}

int gvq_large_groups(int d) { return (d + LG - 1) / LG; }
size_t gvq_large_partial_doubles(int d, int chunks)
{
    const size_t ng = (size_t)gvq_large_groups(d);
    return ng * (ng + 1) / 2 * (size_t)chunks * LBLOCK;
}

int gvq_launch_moments_large(gvq_basis* h, const void* const* grads, int L, hipStream_t st)
{
    const int d = h->d, ng = gvq_large_groups(d), npairs = ng * (ng + 1) / 2;
    for (int l0 = 0; l0 < L; l0 += GVQ_MAX_PTRS) {
        MomLargeArgs a;
        a.L = L - l0 < GVQ_MAX_PTRS ? L - l0 : GVQ_MAX_PTRS;
        for (int i = 0; i < a.L; ++i) a.grads.p[i] = grads[l0 + i];
        a.offs = h->d_offs; a.M = h->M; a.d = d; a.ng = ng; a.npairs = npairs; a.chunks = h->P;
        a.accumulate = l0 > 0; a.part = h->d_part; a.nsamp = h->d_nsamp;
        const int64_t tasks = (int64_t)npairs * h->P;
        dim3 grid((unsigned)((tasks + 3) / 4), h->B);
        const bool bf = h->dtype == GVQ_BF16, vec = (d & 3) == 0;
        if (bf && vec) hipLaunchKernelGGL((moments_large_kernel<true, true>), grid, dim3(256), 0, st, a);
        else if (bf) hipLaunchKernelGGL((moments_large_kernel<true, false>), grid, dim3(256), 0, st, a);
        else if (vec) hipLaunchKernelGGL((moments_large_kernel<false, true>), grid, dim3(256), 0, st, a);
        else hipLaunchKernelGGL((moments_large_kernel<false, false>), grid, dim3(256), 0, st, a);
        GVQ_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(reduce_large_kernel, dim3((LBLOCK + 255) / 256, npairs, h->B), dim3(256), 0, st,
                       h->d_part, h->d_mom, d, ng, npairs, h->P);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}
