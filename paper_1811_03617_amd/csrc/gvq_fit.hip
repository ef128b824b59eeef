// Basis refresh kernels for gfx950 (GradiVeQ Section 2, PCA paragraph after Eq. 4):
//   1. moments:  per basis, sum x and sum x x^T over the sample slices, in float64
//                (fp32/bf16 inputs widen exactly and their products are exact in float64);
//   2. reduce:   fixed-order sum of the per-workgroup partials (bit-reproducible);
//   3. eigen:    mu = s/n, C = G/n - mu mu^T, parallel-order two-sided Jacobi in float64,
//                one workgroup per basis; sort, keep k columns, fix signs.
#include "gvq_internal.h"

__device__ __forceinline__ float load_elem(const void* g, bool bf16, int64_t idx)
{
    if (bf16) return __uint_as_float((unsigned int)((const unsigned short*)g)[idx] << 16);
    return ((const float*)g)[idx];
}

// --------------------------------------------------------------------------------------
// moments on the fp64 matrix pipe, d in {16,32,64,128}.
//
// sum x x^T over samples is a (d x n)(n x d) product with the samples as the contraction
// index, so v_mfma_f64_16x16x4_f64 fits directly: A and B operands have the same lane layout
// (lane l holds row/column l%16 for contraction step l/16), i.e. lane (m, kk) holds element m
// of a 16-element tile of sample kk of the current group of 4 samples -- both operands of a
// tile pair come from the same registers.  Result register r of lane l is entry
// (row 4r + l/16, column l%16) of the 16x16 block.  Only tile pairs T1 <= T2 are computed (the
// matrix is symmetric): 36 blocks at d = 128, all held in one wave's accumulators (288
// registers, which is why a wave has a SIMD to itself here); the four waves of a work-group
// take different samples.
// A "tile" is any 16 elements, so it is chosen to suit the loads: for d >= 64 a lane loads
// 128-bit chunk m + 16q of its sample's slice and register c of that chunk belongs to tile
// T = 4q + c, whose element m is 4(m + 16q) + c; for d < 64 tile T is elements 16T..16T+15.
// Packed partial layout per wave: [pair][r][lane] blocks of 256 doubles, then the d sums.
// --------------------------------------------------------------------------------------
typedef double d4 __attribute__((ext_vector_type(4)));
typedef unsigned int mu4 __attribute__((ext_vector_type(4)));
typedef unsigned int mu2 __attribute__((ext_vector_type(2)));

__host__ __device__ constexpr int mom_pairs(int D) { return (D / 16) * (D / 16 + 1) / 2; }
__host__ __device__ constexpr int mom_packed_width(int D) { return mom_pairs(D) * 256 + D; }
// element index of entry m of tile T
__host__ __device__ inline int mom_elem(int D, int T, int m)
{
    return D >= 64 ? 4 * (m + 16 * (T / 4)) + (T % 4) : 16 * T + m;
}

struct MomMfmaArgs {
    gvq_ptrs grads;
    int L;
    const int64_t* offs;
    int64_t M;
    int wgs;         // work-groups per basis (each holds 4 sample streams, 2 at d = 128)
    int accumulate;  // 0: overwrite the partials, 1: add to them
    double* part;    // [B][wgs * streams][packed width]
    unsigned long long* nsamp;   // [B] += the sample slices this launch took in
};

// HALF selects which tile pairs this wave accumulates: with SPLIT = 2 (d = 128) the 36 pairs
// are shared by two waves that read the same samples (pairs 0..17 and 18..35), so that the
// accumulators of one wave fit the accumulation registers; otherwise every wave has all pairs.
template <int D, bool BF16, int SPLIT, int HALF>
__device__ __forceinline__ void moments_mfma_body(const MomMfmaArgs& a, int stream, int nstreams)
{
    constexpr int NTL = D / 16, NPAIR = mom_pairs(D), WP = mom_packed_width(D);
    constexpr int P0 = SPLIT == 2 ? (HALF ? NPAIR / 2 : 0) : 0;          // first pair of this wave
    constexpr int P1 = SPLIT == 2 ? (HALF ? NPAIR : NPAIR / 2) : NPAIR;  // one past its last pair
    constexpr int NLD = D >= 64 ? D / 64 : NTL;   // loads per lane per sample group
    const int lane = threadIdx.x & 63;
    const int m = lane & 15, kk = lane >> 4;
    const int b = blockIdx.y, p = blockIdx.x;

    const int64_t full = a.M / D;
    int64_t lo = a.offs[b], hi = a.offs[b + 1] < full ? a.offs[b + 1] : full;
    if (hi < lo) hi = lo;
    const int64_t cnt = hi - lo;
    const int64_t nw = (int64_t)a.wgs * nstreams, w = (int64_t)p * nstreams + stream;
    const int64_t j0 = lo + cnt * w / nw, j1 = lo + cnt * (w + 1) / nw;   // this wave's samples

    d4 acc[P1 - P0];
    double sacc[NTL];
#pragma unroll
    for (int i = 0; i < P1 - P0; ++i) acc[i] = d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < NTL; ++i) sacc[i] = 0.0;

    // raw loads of one group of 4 samples: this lane's sample is j = first + kk
    unsigned int taken = 0;   // samples this lane's group slot held (lanes with m = 0 of the counting waves)
    auto load_group = [&](const void* g, int64_t first, float (&x)[NTL]) {
        const int64_t j = first + kk;
        const bool ok = j < j1;
        taken += ok ? 1u : 0u;
        if (D >= 64) {
#pragma unroll
            for (int q = 0; q < NLD; ++q) {
                const int64_t e = j * D + 4 * (m + 16 * q);
                if (BF16) {
                    mu2 v = {0u, 0u};
                    if (ok) v = *(const mu2*)((const unsigned short*)g + e);
                    x[4 * q + 0] = __uint_as_float(v.x << 16);
                    x[4 * q + 1] = __uint_as_float(v.x & 0xffff0000u);
                    x[4 * q + 2] = __uint_as_float(v.y << 16);
                    x[4 * q + 3] = __uint_as_float(v.y & 0xffff0000u);
                } else {
                    mu4 v = {0u, 0u, 0u, 0u};
                    if (ok) v = *(const mu4*)((const float*)g + e);
                    x[4 * q + 0] = __uint_as_float(v.x);
                    x[4 * q + 1] = __uint_as_float(v.y);
                    x[4 * q + 2] = __uint_as_float(v.z);
                    x[4 * q + 3] = __uint_as_float(v.w);
                }
            }
        } else {
#pragma unroll
            for (int T = 0; T < NTL; ++T) {
                const int64_t e = j * D + 16 * T + m;
                float v = 0.f;
                if (ok) v = BF16 ? __uint_as_float((unsigned int)((const unsigned short*)g)[e] << 16)
                                 : ((const float*)g)[e];
                x[T] = v;
            }
        }
    };
    auto consume = [&](const float (&x)[NTL]) {
        double xd[NTL];
#pragma unroll
        for (int T = 0; T < NTL; ++T) {
            xd[T] = (double)x[T];
            if (HALF == 0) sacc[T] += xd[T];
        }
        int pi = 0;
#pragma unroll
        for (int T1 = 0; T1 < NTL; ++T1)
#pragma unroll
            for (int T2 = T1; T2 < NTL; ++T2) {
                if (pi >= P0 && pi < P1)
                    acc[pi - P0] = __builtin_amdgcn_mfma_f64_16x16x4f64(xd[T1], xd[T2], acc[pi - P0], 0, 0, 0);
                ++pi;
            }
    };

    for (int l = 0; l < a.L; ++l) {
        const void* g = a.grads.p[l];
        float xa[NTL], xb[NTL], na[NTL], nb[NTL];
        int64_t j = j0;
        if (j < j1) {
            load_group(g, j, xa);
            load_group(g, j + 4, xb);
        }
        for (; j < j1; j += 8) {
            load_group(g, j + 8, na);     // two groups ahead; past the range they read as zero
            load_group(g, j + 12, nb);
            consume(xa);
            consume(xb);
#pragma unroll
            for (int T = 0; T < NTL; ++T) { xa[T] = na[T]; xb[T] = nb[T]; }
        }
    }

    double* out = a.part + ((size_t)b * nw + w) * WP;
#pragma unroll
    for (int pi = P0; pi < P1; ++pi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double* o = out + pi * 256 + r * 64 + lane;
            *o = a.accumulate ? *o + acc[pi - P0][r] : acc[pi - P0][r];
        }
    if (HALF == 0) {
        // every group that was loaded inside the range was also multiplied: count its samples once
        unsigned int cnt = m == 0 ? taken : 0u;
        cnt += __shfl_xor(cnt, 16, 64);
        cnt += __shfl_xor(cnt, 32, 64);
        if (lane == 0 && cnt) atomicAdd(a.nsamp + b, (unsigned long long)cnt);
        // sums: add the four sample lanes kk of every element
#pragma unroll
        for (int T = 0; T < NTL; ++T) {
            double v = sacc[T];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (kk == 0) {
                double* o = out + NPAIR * 256 + T * 16 + m;
                *o = a.accumulate ? *o + v : v;
            }
        }
    }
}

template <int D, bool BF16>
__global__ __launch_bounds__(256, 2) void moments_mfma_kernel(MomMfmaArgs a)
{
    const int wave = threadIdx.x >> 6;
    if constexpr (D == 128) {
        if (wave & 1) moments_mfma_body<D, BF16, 2, 1>(a, wave >> 1, 2);
        else moments_mfma_body<D, BF16, 2, 0>(a, wave >> 1, 2);
    } else {
        moments_mfma_body<D, BF16, 1, 0>(a, wave, 4);
    }
}

// --------------------------------------------------------------------------------------
// d = 128: the same products with the samples staged through LDS.  The 36 tile pairs are split over
// the four waves of a work-group (9 each: 72 accumulation registers, so two work-groups share a
// compute unit), which all work on the SAME samples: a block of 32 consecutive slices (one contiguous
// run of 32 * 128 elements) is loaded once with full-width loads, two blocks ahead of the one being
// multiplied, parked in LDS as it is, and every wave fetches its operands from there -- lane (m, kk)
// reads elements 4(m + 16q) .. +3 of sample kk of the current group of four with one LDS access and
// has element m of tiles 4q .. 4q+3.  Each input byte crosses HBM once; one barrier per block.
// Wave 0 (whose pairs touch every tile) also keeps the sums of x and counts the samples.
// --------------------------------------------------------------------------------------
#define MOM_BLOCK 32   // slices per LDS block

template <bool BF16, int WAVE>
__device__ __forceinline__ void moments128_wave(const MomMfmaArgs& a, const unsigned int* lds_u32)
{
    constexpr int D = 128, NTL = 8, NPAIR = 36, WP = mom_packed_width(D);
    constexpr int P0 = 9 * WAVE, P1 = P0 + 9;
    constexpr int ROW = BF16 ? D / 2 : D;        // 32-bit words per slice in LDS
    const int lane = threadIdx.x & 63, tid = threadIdx.x;
    const int m = lane & 15, kk = lane >> 4;
    const int b = blockIdx.y, p = blockIdx.x;

    const int64_t full = a.M / D;
    int64_t lo = a.offs[b], hi = a.offs[b + 1] < full ? a.offs[b + 1] : full;
    if (hi < lo) hi = lo;
    const int64_t cnt = hi - lo;
    const int64_t j0 = lo + cnt * p / a.wgs, j1 = lo + cnt * (p + 1) / a.wgs;   // this work-group's samples
    const int64_t nblk = (j1 - j0 + MOM_BLOCK - 1) / MOM_BLOCK;

    d4 acc[9];
    double sacc[NTL];
#pragma unroll
    for (int i = 0; i < 9; ++i) acc[i] = d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll
    for (int i = 0; i < NTL; ++i) sacc[i] = 0.0;
    unsigned int taken = 0;

    // which tiles this wave's pairs touch (compile time)
    bool need[NTL] = {false, false, false, false, false, false, false, false};
    {
        int pi = 0;
#pragma unroll
        for (int T1 = 0; T1 < NTL; ++T1)
#pragma unroll
            for (int T2 = T1; T2 < NTL; ++T2) {
                if (pi >= P0 && pi < P1) { need[T1] = true; need[T2] = true; }
                ++pi;
            }
    }

    // a block = MOM_BLOCK slices = 128-bit words w = 0 .. WPB-1, thread t moves words t, t + 256, ...
    constexpr int WPB = MOM_BLOCK * ROW / 4;     // 1024 (fp32) or 512 (bf16)
    constexpr int NLD = WPB / 256;               // 4 or 2 loads per thread and block
    mu4 stage[NLD];
    unsigned int* ldsw = const_cast<unsigned int*>(lds_u32);
    auto load_block = [&](const void* g, int64_t blk) {
        const int64_t first = j0 + blk * MOM_BLOCK;                    // first slice of the block
        const int64_t words_left = (j1 - first) * (ROW / 4);           // 128-bit words that exist
        const mu4* src = (const mu4*)((const char*)g + first * (int64_t)(ROW * 4));
#pragma unroll
        for (int r = 0; r < NLD; ++r) {
            const int wi = tid + 256 * r;
            mu4 v = {0u, 0u, 0u, 0u};
            if (blk < nblk && wi < words_left) v = __builtin_nontemporal_load(src + wi);
            stage[r] = v;
        }
    };
    auto park_block = [&](int buf) {
#pragma unroll
        for (int r = 0; r < NLD; ++r) *(mu4*)(ldsw + buf * (WPB * 4) + 4 * (tid + 256 * r)) = stage[r];
    };

    for (int l = 0; l < a.L; ++l) {
        const void* g = a.grads.p[l];
        if (nblk == 0) break;
        load_block(g, 0);
        __syncthreads();          // the previous gradient's last block is no longer being read
        park_block(0);
        load_block(g, 1);
        for (int64_t blk = 0; blk < nblk; ++blk) {
            __syncthreads();      // block blk is parked; everyone is done with the buffer that takes block blk + 1
            if (blk + 1 < nblk) park_block((int)((blk + 1) & 1));
            load_block(g, blk + 2);
            const unsigned int* cur = lds_u32 + (blk & 1) * (WPB * 4);
            const int64_t first = j0 + blk * MOM_BLOCK;
#pragma unroll 2
            for (int grp = 0; grp < MOM_BLOCK / 4; ++grp) {
                const int s = 4 * grp + kk;                              // this lane's sample in the block
                double xd[NTL];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    if (!need[4 * q] && !need[4 * q + 1] && !need[4 * q + 2] && !need[4 * q + 3]) continue;
                    if (BF16) {
                        const mu2 v = *(const mu2*)(cur + s * ROW + 2 * (m + 16 * q));
                        xd[4 * q + 0] = (double)__uint_as_float(v.x << 16);
                        xd[4 * q + 1] = (double)__uint_as_float(v.x & 0xffff0000u);
                        xd[4 * q + 2] = (double)__uint_as_float(v.y << 16);
                        xd[4 * q + 3] = (double)__uint_as_float(v.y & 0xffff0000u);
                    } else {
                        const mu4 v = *(const mu4*)(cur + s * ROW + 4 * (m + 16 * q));
                        xd[4 * q + 0] = (double)__uint_as_float(v.x);
                        xd[4 * q + 1] = (double)__uint_as_float(v.y);
                        xd[4 * q + 2] = (double)__uint_as_float(v.z);
                        xd[4 * q + 3] = (double)__uint_as_float(v.w);
                    }
                }
                if (WAVE == 0) {
#pragma unroll
                    for (int T = 0; T < NTL; ++T) sacc[T] += xd[T];
                    taken += (m == 0 && first + s < j1) ? 1u : 0u;
                }
                int pi = 0;
#pragma unroll
                for (int T1 = 0; T1 < NTL; ++T1)
#pragma unroll
                    for (int T2 = T1; T2 < NTL; ++T2) {
                        if (pi >= P0 && pi < P1)
                            acc[pi - P0] = __builtin_amdgcn_mfma_f64_16x16x4f64(xd[T1], xd[T2], acc[pi - P0], 0, 0, 0);
                        ++pi;
                    }
            }
        }
    }

    double* out = a.part + ((size_t)b * a.wgs + p) * WP;
#pragma unroll
    for (int pi = P0; pi < P1; ++pi)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            double* o = out + pi * 256 + r * 64 + lane;
            *o = a.accumulate ? *o + acc[pi - P0][r] : acc[pi - P0][r];
        }
    if (WAVE == 0) {
        unsigned int c = taken;
        c += __shfl_xor(c, 16, 64);
        c += __shfl_xor(c, 32, 64);
        if (lane == 0 && c) atomicAdd(a.nsamp + b, (unsigned long long)c);
#pragma unroll
        for (int T = 0; T < NTL; ++T) {
            double v = sacc[T];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (kk == 0) {
                double* o = out + NPAIR * 256 + T * 16 + m;
                *o = a.accumulate ? *o + v : v;
            }
        }
    }
}

template <bool BF16>
__global__ __launch_bounds__(256, 2) void moments128_kernel(MomMfmaArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned int lds[2 * MOM_BLOCK * (BF16 ? 64 : 128)];
    switch (threadIdx.x >> 6) {
    case 0: moments128_wave<BF16, 0>(a, lds); break;
    case 1: moments128_wave<BF16, 1>(a, lds); break;
    case 2: moments128_wave<BF16, 2>(a, lds); break;
    default: moments128_wave<BF16, 3>(a, lds); break;
    }
}

// dst[b][g][i] = src[b][g*G][i] + src[b][g*G+1][i] + ... (at most G terms, fixed order)
__global__ void reduce_groups_kernel(const double* src, double* dst, int P, int G, int W)
{
    const int b = blockIdx.z, g = blockIdx.y;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= W) return;
    const int nG = (P + G - 1) / G;
    const int p0 = g * G, p1 = p0 + G < P ? p0 + G : P;
    const double* s = src + ((size_t)b * P + p0) * W + i;
    double acc = 0.0;
    for (int p = p0; p < p1; ++p, s += W) acc += *s;
    dst[((size_t)b * nG + g) * W + i] = acc;
}

// packed [B][packed width] -> mom [B][d*d + d] (both triangles written)
__global__ void unpack_moments_kernel(const double* packed, double* mom, int D)
{
    const int b = blockIdx.y;
    const int NTL = D / 16, NPAIR = NTL * (NTL + 1) / 2, WP = NPAIR * 256 + D;
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= WP) return;
    const double v = packed[(size_t)b * WP + i];
    double* o = mom + (size_t)b * (D * D + D);
    if (i >= NPAIR * 256) {
        const int t = i - NPAIR * 256;
        o[D * D + mom_elem(D, t / 16, t % 16)] = v;
        return;
    }
    int pi = i / 256, rem = i % 256, r = rem / 64, lane = rem % 64;
    int T1 = 0, T2 = 0, c = 0;
    for (int t1 = 0; t1 < NTL; ++t1)
        for (int t2 = t1; t2 < NTL; ++t2) {
            if (c == pi) { T1 = t1; T2 = t2; }
            ++c;
        }
    const int e1 = mom_elem(D, T1, 4 * r + lane / 16), e2 = mom_elem(D, T2, lane % 16);
    o[e1 * D + e2] = v;
    if (T1 != T2) o[e2 * D + e1] = v;
}

// --------------------------------------------------------------------------------------
// Eigensolver: two-sided Jacobi with the round-robin ("chess tournament") ordering.  In one
// step the n/2 disjoint index pairs (p_i, q_i) are rotated at once: A <- J^T A J with J the
// product of the n/2 plane rotations, which maps every 2x2 block A[{p_i,q_i}][{p_j,q_j}] to
// R_i^T (block) R_j independently of all other blocks -- one thread per block, no ordering
// needed inside the step.  A rotation R = [[c, s], [-s, c]] annihilates a_pq with
// theta = (a_qq - a_pp) / (2 a_pq), t = sign(theta) / (|theta| + sqrt(theta^2 + 1)),
// c = 1/sqrt(1 + t^2), s = t c.  The matrix lives in LDS, the eigenvectors V (V <- V J) in
// global memory.  n = d rounded up to even; a padding index has a zero row/column and is
// never rotated.
// --------------------------------------------------------------------------------------
struct EigArgs {
    const double* mom;     // [B][d*d+d]
    const unsigned long long* nsamp;   // [B] samples behind the moments
    int d, k;
    double* cov;           // [B][d][d]
    double* V;             // [B][n][n]
    double* eig;           // [B][d]
    float* U;              // [B][d][k]
    float* mu;             // [B][d]
    int* sweeps;           // [B]
    int max_sweeps;
    double tol;
};

__device__ double block_sum(double v, double* red)
{
    // red: LDS array of at least blockDim.x / 64 doubles
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, nw = blockDim.x >> 6;
    __syncthreads();
    if (lane == 0) red[wave] = v;
    __syncthreads();
    double tot = 0.0;
    for (int i = 0; i < nw; ++i) tot += red[i];
    return tot;
}

// The sweeps of the parallel-order Jacobi on the n x n matrix A in LDS (n even), V <- V J in
// global memory (n x n, row-major), all threads of the work-group.  fro2 = squared Frobenius
// norm of A.  Returns the number of sweeps used, -1 if the off-diagonal mass did not fall below
// tol^2 fro2 within max_sweeps (or turned NaN).
__device__ __forceinline__ int jacobi_lds_sweeps(double* A, double* V, int n, double* cs, double* sn, double* red, int* pp, int* qq,
                                 double fro2, int max_sweeps, double tol)
{
    const int half = n >> 1, tid = threadIdx.x, nth = blockDim.x;
    int sweeps_used = -1;
    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        double off2 = 0.0;
        for (int i = tid; i < n * n; i += nth) {
            int r = i / n, c = i - r * n;
            if (r != c) off2 += A[i] * A[i];
        }
        off2 = block_sum(off2, red);
        if (off2 != off2 || fro2 != fro2) break;  // NaN: no convergence (sweeps_used stays -1)
        if (!(off2 > tol * tol * fro2)) { sweeps_used = sweep; break; }
        if (sweep == max_sweeps) break;

        for (int round = 0; round < n - 1; ++round) {
            if (tid < half) {
                int p, q;
                if (tid == 0) { p = round; q = n - 1; }
                else { p = (round + tid) % (n - 1); q = (round - tid + (n - 1)) % (n - 1); }
                if (p > q) { int t = p; p = q; q = t; }
                double apq = A[p * n + q], c = 1.0, s = 0.0;
                if (apq != 0.0) {
                    double theta = (A[q * n + q] - A[p * n + p]) / (2.0 * apq);
                    double t = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                    c = 1.0 / sqrt(1.0 + t * t);
                    s = t * c;
                }
                pp[tid] = p; qq[tid] = q; cs[tid] = c; sn[tid] = s;
            }
            __syncthreads();
            // eigenvector pairs of this round: start their (global memory) loads first, so the
            // latency runs under the LDS work on the matrix; at most 8 pairs per thread for
            // every launch shape used (n*half <= 8 * blockDim)
            double vr[8], vt[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + u * nth;
                if (idx < n * half) {
                    const int row = idx / half, j = idx - row * half;
                    vr[u] = V[row * n + pp[j]];
                    vt[u] = V[row * n + qq[j]];
                }
            }
            for (int idx = tid; idx < half * half; idx += nth) {
                const int i = idx / half, j = idx - i * half;
                const int p = pp[i], q = qq[i], r = pp[j], t = qq[j];
                const double ci = cs[i], si = sn[i], cj = cs[j], sj = sn[j];
                double apr = A[p * n + r], apt = A[p * n + t], aqr = A[q * n + r], aqt = A[q * n + t];
                // rows: R_i^T * block
                double xpr = ci * apr - si * aqr, xpt = ci * apt - si * aqt;
                double xqr = si * apr + ci * aqr, xqt = si * apt + ci * aqt;
                // columns: * R_j
                double ypr = cj * xpr - sj * xpt, ypt = sj * xpr + cj * xpt;
                double yqr = cj * xqr - sj * xqt, yqt = sj * xqr + cj * xqt;
                if (i == j) { ypt = 0.0; yqr = 0.0; }
                A[p * n + r] = ypr; A[p * n + t] = ypt; A[q * n + r] = yqr; A[q * n + t] = yqt;
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int idx = tid + u * nth;
                if (idx < n * half) {
                    const int row = idx / half, j = idx - row * half;
                    const double cj = cs[j], sj = sn[j];
                    V[row * n + pp[j]] = cj * vr[u] - sj * vt[u];
                    V[row * n + qq[j]] = sj * vr[u] + cj * vt[u];
                }
            }
            __syncthreads();
        }
    }
    return sweeps_used;
}

__global__ void eigen_kernel(EigArgs a)
{
    extern __shared__ double smem[];
    const int d = a.d, n = d + (d & 1), half = n >> 1;
    double* A = smem;                       // [n][n]
    double* cs = A + n * n;                 // [half]
    double* sn = cs + half;                 // [half]
    double* red = sn + half;                // [32]
    double* lam = red + 32;                 // [n]
    int* pp = (int*)(lam + n);              // [half]
    int* qq = pp + half;                    // [half]
    int* order = qq + half;                 // [n]
    const int b = blockIdx.x, tid = threadIdx.x, nth = blockDim.x;

    const int W = d * d + d;
    const double* mom = a.mom + (size_t)b * W;
    const double ns = (double)a.nsamp[b];

    double* V = a.V + (size_t)b * n * n;
    double* cov = a.cov + (size_t)b * d * d;
    double fro2 = 0.0;
    for (int i = tid; i < n * n; i += nth) {
        int r = i / n, c = i - r * n;
        double v = 0.0;
        if (r < d && c < d) {
            // upper and lower halves of the Gram sum are bit-identical (same products, same order)
            // true divisions: a constant gradient then gives exactly C = 0
            v = ns > 0.0 ? mom[r * d + c] / ns - (mom[d * d + r] / ns) * (mom[d * d + c] / ns) : 0.0;
            cov[r * d + c] = v;
        }
        A[i] = v;
        V[i] = r == c ? 1.0 : 0.0;
        fro2 += v * v;
    }
    for (int i = tid; i < d; i += nth) a.mu[(size_t)b * d + i] = ns > 0.0 ? (float)(mom[d * d + i] / ns) : 0.0f;
    fro2 = block_sum(fro2, red);

    const int sweeps_used = jacobi_lds_sweeps(A, V, n, cs, sn, red, pp, qq, fro2, a.max_sweeps, a.tol);

    // eigenvalues in decreasing order (ties: lower index first)
    for (int i = tid; i < d; i += nth) lam[i] = A[i * n + i];
    __syncthreads();
    for (int i = tid; i < d; i += nth) {
        // NaN sorts last: compare with NaN replaced by -inf
        const double li = lam[i] == lam[i] ? lam[i] : -INFINITY;
        int rank = 0;
        for (int j = 0; j < d; ++j) {
            const double lj = lam[j] == lam[j] ? lam[j] : -INFINITY;
            if (lj > li || (lj == li && j < i)) ++rank;
        }
        order[rank] = i;
    }
    __syncthreads();
    for (int i = tid; i < d; i += nth) a.eig[(size_t)b * d + i] = lam[order[i]];
    // kept eigenvectors, sign: largest-magnitude entry (lowest index on ties) positive
    for (int i = tid; i < a.k; i += nth) {
        const int col = order[i];
        int arg = 0;
        double big = -1.0;
        for (int e = 0; e < d; ++e) {
            double m = fabs(V[e * n + col]);
            if (m > big) { big = m; arg = e; }
        }
        const double sign = V[arg * n + col] < 0.0 ? -1.0 : 1.0;
        for (int e = 0; e < d; ++e) a.U[((size_t)b * d + e) * a.k + i] = (float)(sign * V[e * n + col]);
    }
    if (tid == 0) a.sweeps[b] = sweeps_used;
}

// --------------------------------------------------------------------------------------
// First-slice sampling with fewer samples than dimensions (Section 3: L time samples of one slice,
// slice sizes in the hundreds).  The covariance C = Xc^T Xc / L (Xc: the L centred samples as
// rows) has rank < L, and its non-zero eigenpairs are those of the small L x L matrix
// K = Xc Xc^T / L: K v = lambda v  =>  C (Xc^T v) = lambda (Xc^T v).  So the Jacobi runs on K in
// LDS whatever d is, and the kept directions are u_i = Xc^T v_i, normalised and cleaned with one
// round of Gram-Schmidt against the columns before them.  Directions beyond the rank of the data
// (eigenvalue <= 1e-12 of the largest) are not determined by it; they are completed with unit
// vectors made orthogonal to the columns so far, so that U always has orthonormal columns.
// One work-group per basis.  work[b]: [m*m] eigenvectors of K, then [k][d] the columns of U in
// float64.
// --------------------------------------------------------------------------------------
#define GVQ_GRAM_MAX_L 128
#define GVQ_GRAM_MAX_K 256
struct GramArgs {
    gvq_ptrs grads[GVQ_GRAM_MAX_L / GVQ_MAX_PTRS];
    int L;
    const double* mom;     // [B][d*d+d] from first_slice_moments_kernel
    const unsigned long long* nsamp;   // [B] samples behind the moments (L, or 0 without a full first slice)
    const int64_t* offs;
    int64_t M;
    int d, k, bf16;
    double* cov;           // [B][d][d]
    double* work;          // [B][work_stride]
    size_t work_stride;
    double* eig;           // [B][d]
    float* U;              // [B][d][k]
    float* mu;             // [B][d]
    int* sweeps;           // [B]
    int max_sweeps;
    double tol;
};

size_t gvq_gram_lds_bytes(int L, int k)
{
    const int m = L + (L & 1), half = m / 2;
    return sizeof(double) * ((size_t)m * m + 2 * half + 32 + m + k) + sizeof(int) * (2 * half + m);
}

__global__ __launch_bounds__(1024) void gram_eigen_kernel(GramArgs a)
{
    extern __shared__ double smem[];
    const int d = a.d, k = a.k, L = a.L, m = L + (L & 1), half = m >> 1;
    double* A = smem;                       // [m][m]
    double* cs = A + m * m;                 // [half]
    double* sn = cs + half;                 // [half]
    double* red = sn + half;                // [32]
    double* lam = red + 32;                 // [m]
    double* dots = lam + m;                 // [k]
    int* pp = (int*)(dots + k);             // [half]
    int* qq = pp + half;                    // [half]
    int* order = qq + half;                 // [m]
    const int b = blockIdx.x, tid = threadIdx.x, nth = blockDim.x, lane = tid & 63, wave = tid >> 6, nw = nth >> 6;

    const double* mom = a.mom + (size_t)b * ((size_t)d * d + d);
    double* cov = a.cov + (size_t)b * d * d;
    double* V = a.work + (size_t)b * a.work_stride;   // [m][m]
    double* Uw = V + (size_t)m * m;                   // [k][d]
    const int64_t j = a.offs[b];
    if (a.nsamp[b] == 0) {
        // no full first slice: the trivial basis, as in the general solver
        for (int i = tid; i < d * d; i += nth) cov[i] = 0.0;
        for (int i = tid; i < d; i += nth) { a.mu[(size_t)b * d + i] = 0.f; a.eig[(size_t)b * d + i] = 0.0; }
        for (int i = tid; i < d * k; i += nth) a.U[(size_t)b * d * k + i] = (i / k == i % k) ? 1.f : 0.f;
        if (tid == 0) a.sweeps[b] = 0;
        return;
    }
    const double ns = (double)a.nsamp[b];   // = L
    for (int i = tid; i < d * d; i += nth) {
        const int r = i / d, c = i - r * d;
        cov[i] = mom[i] / ns - (mom[(size_t)d * d + r] / ns) * (mom[(size_t)d * d + c] / ns);
    }
    for (int i = tid; i < d; i += nth) a.mu[(size_t)b * d + i] = (float)(mom[(size_t)d * d + i] / ns);
    auto xc = [&](int l, int e) {   // centred sample l, element e
        return (double)load_elem(a.grads[l / GVQ_MAX_PTRS].p[l % GVQ_MAX_PTRS], a.bf16 != 0, j * d + e) -
               mom[(size_t)d * d + e] / ns;
    };
    // K (upper triangle computed, mirrored), zero row/column for the padding index
    for (int i = tid; i < m * m; i += nth) {
        const int r = i / m, c = i - r * m;
        if (r > c) continue;
        double v = 0.0;
        if (c < L) {
            for (int e = 0; e < d; ++e) v = fma(xc(r, e), xc(c, e), v);
            v /= ns;
        }
        A[r * m + c] = v;
        A[c * m + r] = v;
    }
    for (int i = tid; i < m * m; i += nth) V[i] = (i / m == i % m) ? 1.0 : 0.0;
    __syncthreads();
    double fro2 = 0.0;
    for (int i = tid; i < m * m; i += nth) fro2 += A[i] * A[i];
    fro2 = block_sum(fro2, red);
    const int sweeps_used = jacobi_lds_sweeps(A, V, m, cs, sn, red, pp, qq, fro2, a.max_sweeps, a.tol);
    __syncthreads();

    // eigenvalues of K in decreasing order (ties: lower index first, NaN last)
    // K is positive semi-definite: a negative eigenvalue is rounding noise around zero
    for (int i = tid; i < L; i += nth) lam[i] = A[i * m + i] < 0.0 ? 0.0 : A[i * m + i];
    __syncthreads();
    for (int i = tid; i < L; i += nth) {
        const double li = lam[i] == lam[i] ? lam[i] : -INFINITY;
        int rank = 0;
        for (int q = 0; q < L; ++q) {
            const double lq = lam[q] == lam[q] ? lam[q] : -INFINITY;
            if (lq > li || (lq == li && q < i)) ++rank;
        }
        order[rank] = i;
    }
    __syncthreads();
    for (int i = tid; i < d; i += nth) a.eig[(size_t)b * d + i] = i < L ? lam[order[i]] : 0.0;
    const double top = lam[order[0]];

    // raw directions Xc^T v_i for the columns the data determines, zero for the others
    for (int i = tid; i < k * d; i += nth) {
        const int col = i / d, e = i - col * d;
        double v = 0.0;
        if (col < L && lam[order[col]] > 1e-12 * top) {
            const int vc = order[col];
            for (int l = 0; l < L; ++l) v = fma(V[l * m + vc], xc(l, e), v);
        }
        Uw[i] = v;
    }
    __syncthreads();

    // columns one after the other: orthogonalise against the earlier ones (twice), normalise
    int next_unit = 0;
    for (int col = 0; col < k; ++col) {
        double* w = Uw + (size_t)col * d;
        const bool determined = col < L && lam[order[col]] > 1e-12 * top;   // uniform
        for (;;) {   // ends: every retry takes a new unit vector, and there are d of them
            if (!determined) {
                for (int e = tid; e < d; e += nth) w[e] = e == next_unit ? 1.0 : 0.0;
                ++next_unit;
                __syncthreads();
            }
            for (int pass = 0; pass < 2; ++pass) {
                for (int q = wave; q < col; q += nw) {
                    const double* u = Uw + (size_t)q * d;
                    double acc = 0.0;
                    for (int e = lane; e < d; e += 64) acc = fma(u[e], w[e], acc);
                    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
                    if (lane == 0) dots[q] = acc;
                }
                __syncthreads();
                for (int e = tid; e < d; e += nth) {
                    double v = w[e];
                    for (int q = 0; q < col; ++q) v = fma(-dots[q], Uw[(size_t)q * d + e], v);
                    w[e] = v;
                }
                __syncthreads();
            }
            double n2 = 0.0;
            for (int e = tid; e < d; e += nth) n2 += w[e] * w[e];
            n2 = block_sum(n2, red);
            // a unit vector that lies almost inside the span so far is a poor start: take the next one
            if (!determined && n2 < 0.25 && next_unit < d) continue;
            const double inv = n2 > 0.0 ? 1.0 / sqrt(n2) : 0.0;
            for (int e = tid; e < d; e += nth) w[e] *= inv;
            __syncthreads();
            break;
        }
    }
    // sign: largest-magnitude entry (lowest index on ties) positive
    for (int col = tid; col < k; col += nth) {
        const double* w = Uw + (size_t)col * d;
        int arg = 0;
        double big = -1.0;
        for (int e = 0; e < d; ++e) {
            const double mag = fabs(w[e]);
            if (mag > big) { big = mag; arg = e; }
        }
        const double sign = w[arg] < 0.0 ? -1.0 : 1.0;
        for (int e = 0; e < d; ++e) a.U[((size_t)b * d + e) * k + col] = (float)(sign * w[e]);
    }
    if (tid == 0) a.sweeps[b] = sweeps_used;
}

// The small-matrix route is taken when it applies and its scratch fits the eigenvector work space.
bool gvq_gram_shape(int d, int k, int L)
{
    // scratch: (L rounded up to even)^2 + k d doubles inside the d x d eigenvector work space
    const int64_t m = L + (L & 1);
    return L >= 2 && L <= GVQ_GRAM_MAX_L && 2 * L <= d && k <= GVQ_GRAM_MAX_K &&
           m * m + (int64_t)k * d <= (int64_t)d * d;
}

// Section 3, "compressor reuse": moments of the first slice of every basis only -- L samples of d
// numbers per basis, a few KB; one work-group per basis, one thread per matrix entry.
__global__ void first_slice_moments_kernel(gvq_ptrs grads, int L, const int64_t* offs, int64_t M, int d, int bf16,
                                           int accumulate, double* mom, unsigned long long* nsamp)
{
    const int b = blockIdx.x, W = d * d + d;
    const int64_t j = offs[b];
    const bool ok = (j + 1) * d <= M;     // the first slice must be a full one
    if (blockIdx.y == 0 && threadIdx.x == 0 && ok) atomicAdd(nsamp + b, (unsigned long long)L);
    for (int i = blockIdx.y * blockDim.x + threadIdx.x; i < W; i += gridDim.y * blockDim.x) {
        const int r = i < d * d ? i / d : i - d * d, c = i < d * d ? i % d : -1;
        double acc = 0.0;
        if (ok)
            for (int l = 0; l < L; ++l) {
                const double xr = (double)load_elem(grads.p[l], bf16 != 0, j * d + r);
                acc += c >= 0 ? xr * (double)load_elem(grads.p[l], bf16 != 0, j * d + c) : xr;
            }
        double* o = mom + (size_t)b * W + i;
        *o = accumulate ? *o + acc : acc;
    }
}

// Section 3, Eq. (5): smallest k with (eig[0] + .. + eig[k-1]) / sum(eig) >= 1 - lambda; one
// thread per basis, partial sums from the largest eigenvalue down, in double.
__global__ void select_k_kernel(const double* eig, int d, int B, double lambda, int* k_out)
{
    const int b = blockIdx.x * blockDim.x + threadIdx.x;
    if (b >= B) return;
    const double* e = eig + (size_t)b * d;
    double total = 0.0;
    for (int i = 0; i < d; ++i) total += e[i];
    int k = d;
    if (!(total > 0.0)) {
        k = 1;
    } else {
        double cum = 0.0;
        for (int i = 1; i <= d; ++i) {
            cum += e[i - 1];
            if (cum / total >= 1.0 - lambda) { k = i; break; }
        }
    }
    k_out[b] = k;
}

int gvq_launch_select_k(const gvq_basis* h, double lambda, hipStream_t st)
{
    hipLaunchKernelGGL(select_k_kernel, dim3((h->B + 63) / 64), dim3(64), 0, st, h->d_eig, h->d, h->B, lambda,
                       h->d_ksel);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

// ======================================================================================
size_t gvq_eigen_lds_bytes(int d)
{
    const int n = d + (d & 1), half = n / 2;
    return sizeof(double) * ((size_t)n * n + 2 * half + 32 + n) + sizeof(int) * (2 * half + n);
}

template <int D>
static void launch_moments_mfma(const gvq_basis* h, const MomMfmaArgs& a, hipStream_t st)
{
    dim3 grid(h->mom_wgs, h->B);
    if constexpr (D == 128) {
        if (h->dtype == GVQ_BF16)
            hipLaunchKernelGGL((moments128_kernel<true>), grid, dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL((moments128_kernel<false>), grid, dim3(256), 0, st, a);
        return;
    }
    if (h->dtype == GVQ_BF16)
        hipLaunchKernelGGL((moments_mfma_kernel<D, true>), grid, dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL((moments_mfma_kernel<D, false>), grid, dim3(256), 0, st, a);
}

bool gvq_moments_mfma_shape(int d) { return d == 16 || d == 32 || d == 64 || d == 128; }
int gvq_moments_packed_width(int d) { return mom_packed_width(d); }
int gvq_moments_streams(int d) { return d == 128 ? 1 : 4; }   // d = 128: the four waves share one stream

// A fill kernel rather than a memset, so that a fit can be captured into a HIP graph.
__global__ void zero_counts_kernel(unsigned long long* p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0ull;
}

int gvq_launch_fit(gvq_basis* h, const void* const* grads, int L, bool first_slice_only, hipStream_t st)
{
    const int d = h->d, W = d * d + d;
    hipLaunchKernelGGL(zero_counts_kernel, dim3((h->B + 255) / 256), dim3(256), 0, st, h->d_nsamp, h->B);
    GVQ_HIP(hipGetLastError());
    if (first_slice_only) {
        for (int l0 = 0; l0 < L; l0 += GVQ_MAX_PTRS) {
            gvq_ptrs p;
            const int n = L - l0 < GVQ_MAX_PTRS ? L - l0 : GVQ_MAX_PTRS;
            for (int i = 0; i < n; ++i) p.p[i] = grads[l0 + i];
            hipLaunchKernelGGL(first_slice_moments_kernel, dim3(h->B, (W + 4095) / 4096), dim3(256), 0, st, p, n,
                               h->d_offs, h->M, d,
                               h->dtype == GVQ_BF16 ? 1 : 0, l0 > 0 ? 1 : 0, h->d_mom, h->d_nsamp);
            GVQ_HIP(hipGetLastError());
        }
    } else if (!gvq_moments_mfma_shape(d)) {
        const int rc = gvq_launch_moments_large(h, grads, L, st);
        if (rc != GVQ_OK) return rc;
    } else {
        const int WP = mom_packed_width(d);
        for (int l0 = 0; l0 < L; l0 += GVQ_MAX_PTRS) {
            MomMfmaArgs a;
            a.L = L - l0 < GVQ_MAX_PTRS ? L - l0 : GVQ_MAX_PTRS;
            for (int i = 0; i < a.L; ++i) a.grads.p[i] = grads[l0 + i];
            a.offs = h->d_offs; a.M = h->M; a.wgs = h->mom_wgs; a.accumulate = l0 > 0; a.part = h->d_part;
            a.nsamp = h->d_nsamp;
            switch (d) {
            case 16: launch_moments_mfma<16>(h, a, st); break;
            case 32: launch_moments_mfma<32>(h, a, st); break;
            case 64: launch_moments_mfma<64>(h, a, st); break;
            default: launch_moments_mfma<128>(h, a, st); break;
            }
            GVQ_HIP(hipGetLastError());
        }
        // fixed-order tree: P partials -> groups of 32 -> one, then to the d x d layout
        const int P = h->P, G = 32, nG = (P + G - 1) / G;
        hipLaunchKernelGGL(reduce_groups_kernel, dim3((WP + 255) / 256, nG, h->B), dim3(256), 0, st,
                           h->d_part, h->d_part2, P, G, WP);
        GVQ_HIP(hipGetLastError());
        hipLaunchKernelGGL(reduce_groups_kernel, dim3((WP + 255) / 256, 1, h->B), dim3(256), 0, st,
                           h->d_part2, h->d_part, nG, nG, WP);   // result: d_part[b][0][:] with stride WP
        GVQ_HIP(hipGetLastError());
        hipLaunchKernelGGL(unpack_moments_kernel, dim3((WP + 255) / 256, h->B), dim3(256), 0, st,
                           h->d_part, h->d_mom, d);
        GVQ_HIP(hipGetLastError());
    }

    if (first_slice_only && gvq_gram_shape(d, h->k, L)) {
        GramArgs g;
        for (int l = 0; l < L; ++l) g.grads[l / GVQ_MAX_PTRS].p[l % GVQ_MAX_PTRS] = grads[l];
        g.L = L; g.mom = h->d_mom; g.nsamp = h->d_nsamp; g.offs = h->d_offs; g.M = h->M; g.d = d; g.k = h->k;
        g.bf16 = h->dtype == GVQ_BF16 ? 1 : 0;
        g.cov = h->d_cov; g.work = h->d_V; g.work_stride = (size_t)(d + (d & 1)) * (d + (d & 1));
        g.eig = h->d_eig; g.U = h->d_U; g.mu = h->d_mu; g.sweeps = h->d_sweeps; g.max_sweeps = 60; g.tol = 1e-15;
        static gvq_once_per_device gram_once;
        if (gram_once.first(h->device))
            GVQ_HIP(hipFuncSetAttribute((const void*)gram_eigen_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                        (int)gvq_gram_lds_bytes(GVQ_GRAM_MAX_L, GVQ_GRAM_MAX_K)));
        hipLaunchKernelGGL(gram_eigen_kernel, dim3(h->B), dim3(1024), gvq_gram_lds_bytes(L, h->k), st, g);
        GVQ_HIP(hipGetLastError());
        return gvq_launch_pack(h, st);
    }
    if (d > GVQ_LDS_EIGEN_MAX_D) {
        const int rc = gvq_launch_eigen_block(h, st);
        return rc != GVQ_OK ? rc : gvq_launch_pack(h, st);
    }
    EigArgs e;
    e.mom = h->d_mom; e.nsamp = h->d_nsamp; e.d = d; e.k = h->k;
    e.cov = h->d_cov; e.V = h->d_V; e.eig = h->d_eig; e.U = h->d_U; e.mu = h->d_mu;
    e.sweeps = h->d_sweeps; e.max_sweeps = 60; e.tol = 1e-15;
    const size_t lds = gvq_eigen_lds_bytes(d);
    static gvq_once_per_device once;
    if (once.first(h->device))
        GVQ_HIP(hipFuncSetAttribute((const void*)eigen_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)gvq_eigen_lds_bytes(GVQ_LDS_EIGEN_MAX_D)));
    const int threads = d > 16 ? 256 : 64;
    hipLaunchKernelGGL(eigen_kernel, dim3(h->B), dim3(threads), lds, st, e);
    GVQ_HIP(hipGetLastError());
    return gvq_launch_pack(h, st);
}
