// Basis refresh for long slices, 128 < d <= GVQ_MAX_D (GradiVeQ Section 3, "slice size": the
// slice is a multiple of a layer's filters x depth, e.g. 768 for a (3,3,16,16) layer).  The
// d x d matrix no longer fits one work-group's LDS, so both stages work out of global memory:
//   moments: sum x x^T in 64 x 64 blocks on the fp64 matrix pipe, one wave per (block, sample
//            chunk), fixed-order sum of the chunks afterwards (any d: also used for the short
//            slice lengths other than 16, 32, 64 and 128);
//   eigen:   the same parallel-order two-sided Jacobi as for short slices, one kernel launch per
//            round of disjoint rotations (the launch boundary is the grid-wide barrier), the
//            matrix ping-ponging between two buffers so that a round reads only old values.
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

// ======================================================================================
// Jacobi out of global memory.  state[b] = {done, sweeps used (-1: not converged), buffer that
// holds the final matrix, unused}.
// ======================================================================================
struct JacArgs {
    const double* mom;     // [B][d*d+d]
    const unsigned long long* nsamp;   // [B] samples behind the moments
    int d, n, k;
    double* cov;           // [B][d][d]
    double* jac;           // [B][2][n][n]
    double* V;             // [B][n][n]
    double* eig;           // [B][d]
    float* U;              // [B][d][k]
    float* mu;             // [B][d]
    int* sweeps;           // [B]
    int* state;            // [B][4]
    double tol;
};

// mu = s/n, C = G/n - mu mu^T (true divisions: a constant gradient gives exactly C = 0),
// matrix buffer 0 <- C padded to n x n, V <- identity.
__global__ __launch_bounds__(256) void jacobi_init_kernel(JacArgs a)
{
    const int b = blockIdx.y, d = a.d, n = a.n;
    const double* mom = a.mom + (size_t)b * ((size_t)d * d + d);
    const double ns = (double)a.nsamp[b];
    double* A = a.jac + (size_t)b * 2 * n * n;
    double* V = a.V + (size_t)b * n * n;
    double* cov = a.cov + (size_t)b * d * d;
    const int gtid = blockIdx.x * blockDim.x + threadIdx.x, gsz = gridDim.x * blockDim.x;
    for (int i = gtid; i < n * n; i += gsz) {
        const int r = i / n, c = i - r * n;
        double v = 0.0;
        if (r < d && c < d) {
            v = ns > 0.0 ? mom[(size_t)r * d + c] / ns - (mom[(size_t)d * d + r] / ns) * (mom[(size_t)d * d + c] / ns)
                         : 0.0;
            cov[(size_t)r * d + c] = v;
        }
        A[i] = v;
        V[i] = r == c ? 1.0 : 0.0;
    }
    for (int i = gtid; i < d; i += gsz)
        a.mu[(size_t)b * d + i] = ns > 0.0 ? (float)(mom[(size_t)d * d + i] / ns) : 0.0f;
    if (gtid == 0) {
        a.state[4 * b + 0] = 0;
        a.state[4 * b + 1] = -1;
        a.state[4 * b + 2] = 0;
    }
}

// Start of sweep `sweep`: stop when the off-diagonal mass is below tol^2 of the whole, on NaN,
// or when the sweep budget is used up.  One work-group per basis, fixed summation order.
__global__ __launch_bounds__(1024) void jacobi_check_kernel(JacArgs a, int sweep, int src, int max_sweeps)
{
    __shared__ double red_off[16], red_all[16];
    const int b = blockIdx.x, n = a.n, tid = threadIdx.x;
    if (a.state[4 * b]) return;
    const double* A = a.jac + ((size_t)b * 2 + src) * n * n;
    double off2 = 0.0, all2 = 0.0;
    for (int i = tid; i < n * n; i += 1024) {
        const int r = i / n, c = i - r * n;
        const double v = A[i], v2 = v * v;
        all2 += v2;
        if (r != c) off2 += v2;
    }
    for (int o = 32; o > 0; o >>= 1) {
        off2 += __shfl_down(off2, o, 64);
        all2 += __shfl_down(all2, o, 64);
    }
    if ((tid & 63) == 0) { red_off[tid >> 6] = off2; red_all[tid >> 6] = all2; }
    __syncthreads();
    if (tid == 0) {
        double so = 0.0, sa = 0.0;
        for (int i = 0; i < 16; ++i) { so += red_off[i]; sa += red_all[i]; }
        int done = 0, used = -1;
        if (!(so > a.tol * a.tol * sa)) { done = 1; used = sweep; }   // also taken when so is NaN ...
        if (so != so || sa != sa) { done = 1; used = -1; }             // ... which is no convergence
        if (!done && sweep >= max_sweeps) done = 1;
        if (done) {
            a.state[4 * b + 1] = used;
            a.state[4 * b + 2] = src;
            __threadfence();
            a.state[4 * b + 0] = 1;
        }
    }
}

// Index pair i of the round-robin schedule in round `round` (n even): pair 0 is (round, n-1),
// pair i is ((round + i) mod (n-1), (round - i) mod (n-1)); returned with p < q.
__device__ __forceinline__ void jacobi_pair(int n, int round, int i, int& p, int& q)
{
    if (i == 0) { p = round; q = n - 1; }
    else { p = (round + i) % (n - 1); q = (round - i + (n - 1)) % (n - 1); }
    if (p > q) { const int u = p; p = q; q = u; }
}

// One round: the n/2 disjoint rotations (p_i, q_i) of the round-robin schedule, applied as
// dst[{p_i,q_i}][{p_j,q_j}] = R_i^T src[..][..] R_j, one thread per 2 x 2 block, and V <- V J for
// the rows 2i, 2i+1 and column pair j.  R = [[c, s], [-s, c]], theta = (a_qq - a_pp) / (2 a_pq),
// t = sign(theta) / (|theta| + sqrt(theta^2 + 1)), c = 1/sqrt(1 + t^2), s = t c.  A work-group
// covers 16 x 16 blocks.
__global__ __launch_bounds__(256) void jacobi_round_kernel(JacArgs a, int round, int src)
{
    __shared__ double sc[2][16], ss[2][16];
    const int b = blockIdx.z;
    if (a.state[4 * b]) return;
    const int n = a.n, half = n >> 1, tid = threadIdx.x;
    const double* A = a.jac + ((size_t)b * 2 + src) * n * n;
    double* Bm = a.jac + ((size_t)b * 2 + (src ^ 1)) * n * n;
    double* V = a.V + (size_t)b * n * n;
    // The pair indices are arithmetic, so a thread asks for its 2 x 2 block and its eigenvector
    // entries right away; the 16 + 16 rotations of the work-group are worked out meanwhile by its
    // first 32 threads (from the old matrix) and handed over through LDS: one memory round trip.
    const int ti = tid >> 4, tj = tid & 15;
    const int i = blockIdx.y * 16 + ti, j = blockIdx.x * 16 + tj;
    const bool active = i < half && j < half;
    int p = 0, q = 0, r = 0, t = 0;
    double apr = 0.0, apt = 0.0, aqr = 0.0, aqt = 0.0, v0r = 0.0, v0t = 0.0, v1r = 0.0, v1t = 0.0;
    const int r0 = 2 * i, r1 = 2 * i + 1;
    if (active) {
        jacobi_pair(n, round, i, p, q);
        jacobi_pair(n, round, j, r, t);
        apr = A[(size_t)p * n + r]; apt = A[(size_t)p * n + t];
        aqr = A[(size_t)q * n + r]; aqt = A[(size_t)q * n + t];
        v0r = V[(size_t)r0 * n + r]; v0t = V[(size_t)r0 * n + t];
        v1r = V[(size_t)r1 * n + r]; v1t = V[(size_t)r1 * n + t];
    }
    if (tid < 32) {
        const int side = tid >> 4, u = tid & 15;
        const int pi = (side ? blockIdx.x : blockIdx.y) * 16 + u;
        double c = 1.0, s = 0.0;
        if (pi < half) {
            int pp, qq;
            jacobi_pair(n, round, pi, pp, qq);
            const double apq = A[(size_t)pp * n + qq];
            if (apq != 0.0) {
                const double theta = (A[(size_t)qq * n + qq] - A[(size_t)pp * n + pp]) / (2.0 * apq);
                const double tt = (theta >= 0.0 ? 1.0 : -1.0) / (fabs(theta) + sqrt(theta * theta + 1.0));
                c = 1.0 / sqrt(1.0 + tt * tt);
                s = tt * c;
            }
        }
        sc[side][u] = c; ss[side][u] = s;
    }
    __syncthreads();
    if (!active) return;
    const double ci = sc[0][ti], si = ss[0][ti], cj = sc[1][tj], sj = ss[1][tj];
    // rows: R_i^T * block
    const double xpr = ci * apr - si * aqr, xpt = ci * apt - si * aqt;
    const double xqr = si * apr + ci * aqr, xqt = si * apt + ci * aqt;
    // columns: * R_j
    double ypr = cj * xpr - sj * xpt, ypt = sj * xpr + cj * xpt;
    double yqr = cj * xqr - sj * xqt, yqt = sj * xqr + cj * xqt;
    if (i == j) { ypt = 0.0; yqr = 0.0; }
    Bm[(size_t)p * n + r] = ypr; Bm[(size_t)p * n + t] = ypt;
    Bm[(size_t)q * n + r] = yqr; Bm[(size_t)q * n + t] = yqt;
    V[(size_t)r0 * n + r] = cj * v0r - sj * v0t; V[(size_t)r0 * n + t] = sj * v0r + cj * v0t;
    V[(size_t)r1 * n + r] = cj * v1r - sj * v1t; V[(size_t)r1 * n + t] = sj * v1r + cj * v1t;
}

// Eigenvalues in decreasing order (ties: lower index first, NaN last), the k leading
// eigenvectors with the largest-magnitude entry (lowest index on ties) made positive.
__global__ __launch_bounds__(1024) void jacobi_finish_kernel(JacArgs a)
{
    __shared__ double lam[GVQ_MAX_D];
    __shared__ int order[GVQ_MAX_D];
    const int b = blockIdx.x, d = a.d, n = a.n, tid = threadIdx.x;
    const double* A = a.jac + ((size_t)b * 2 + a.state[4 * b + 2]) * n * n;
    const double* V = a.V + (size_t)b * n * n;
    for (int i = tid; i < d; i += 1024) lam[i] = A[(size_t)i * n + i];
    __syncthreads();
    for (int i = tid; i < d; i += 1024) {
        const double li = lam[i] == lam[i] ? lam[i] : -INFINITY;
        int rank = 0;
        for (int j = 0; j < d; ++j) {
            const double lj = lam[j] == lam[j] ? lam[j] : -INFINITY;
            if (lj > li || (lj == li && j < i)) ++rank;
        }
        order[rank] = i;
    }
    __syncthreads();
    for (int i = tid; i < d; i += 1024) a.eig[(size_t)b * d + i] = lam[order[i]];
    for (int i = tid; i < a.k; i += 1024) {
        const int col = order[i];
        int arg = 0;
        double big = -1.0;
        for (int e = 0; e < d; ++e) {
            const double mag = fabs(V[(size_t)e * n + col]);
            if (mag > big) { big = mag; arg = e; }
        }
        const double sign = V[(size_t)arg * n + col] < 0.0 ? -1.0 : 1.0;
        for (int e = 0; e < d; ++e)
            a.U[((size_t)b * d + e) * a.k + i] = (float)(sign * V[(size_t)e * n + col]);
    }
    if (tid == 0) a.sweeps[b] = a.state[4 * b] ? a.state[4 * b + 1] : -1;
}

int gvq_launch_eigen_large(gvq_basis* h, int L, bool first_slice_only, hipStream_t st)
{
    const int d = h->d, n = d + (d & 1), half = n / 2;
    JacArgs a;
    a.mom = h->d_mom; a.nsamp = h->d_nsamp; a.d = d; a.n = n; a.k = h->k;
    (void)L; (void)first_slice_only;
    a.cov = h->d_cov; a.jac = h->d_jac; a.V = h->d_V; a.eig = h->d_eig; a.U = h->d_U; a.mu = h->d_mu;
    a.sweeps = h->d_sweeps; a.state = h->d_jstate; a.tol = 1e-15;
    const int max_sweeps = 24;
    hipLaunchKernelGGL(jacobi_init_kernel, dim3(256, h->B), dim3(256), 0, st, a);
    GVQ_HIP(hipGetLastError());
    const dim3 rgrid((half + 15) / 16, (half + 15) / 16, h->B);
    int src = 0;
    for (int sweep = 0; sweep <= max_sweeps; ++sweep) {
        hipLaunchKernelGGL(jacobi_check_kernel, dim3(h->B), dim3(1024), 0, st, a, sweep, src, max_sweeps);
        GVQ_HIP(hipGetLastError());
        if (sweep == max_sweeps) break;
        for (int round = 0; round < n - 1; ++round) {
            hipLaunchKernelGGL(jacobi_round_kernel, rgrid, dim3(256), 0, st, a, round, src);
            src ^= 1;
        }
        GVQ_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(jacobi_finish_kernel, dim3(h->B), dim3(1024), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}
