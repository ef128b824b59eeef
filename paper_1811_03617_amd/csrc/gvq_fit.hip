// Basis refresh kernels for gfx950 (GradiVeQ Section 2, PCA paragraph after Eq. 4):
//   1. moments:  per basis, sum x and sum x x^T over the sample slices, in float64
//                (fp32/bf16 inputs widen exactly and their products are exact in float64);
//   2. reduce:   fixed-order sum of the per-workgroup partials (bit-reproducible);
//   3. eigen:    mu = s/n, C = G/n - mu mu^T, parallel-order two-sided Jacobi in float64,
//                one workgroup per basis; sort, keep k columns, fix signs.
#include "gvq_internal.h"

#define MOM_THREADS 256
#define MOM_TILE 32  // slices staged in LDS per step

struct MomArgs {
    gvq_ptrs grads;
    int L;
    const int64_t* offs;
    int64_t M;
    int d, P;
    double* part;  // [B][P][d*d+d]
};

__device__ __forceinline__ float load_elem(const void* g, bool bf16, int64_t idx)
{
    if (bf16) return __uint_as_float((unsigned int)((const unsigned short*)g)[idx] << 16);
    return ((const float*)g)[idx];
}

// Thread (ti, tj) of a 16x16 thread grid owns the TB x TB block of sum x x^T with rows
// ti*TB.. and columns tj*TB..; d is padded with zeros to 16*TB.
template <int TB, bool BF16>
__global__ __launch_bounds__(MOM_THREADS) void moments_kernel(MomArgs a)
{
    constexpr int DP = 16 * TB;
    __shared__ float xs[MOM_TILE][DP];
    const int tid = threadIdx.x, ti = tid >> 4, tj = tid & 15;
    const int b = blockIdx.y, p = blockIdx.x;
    const int d = a.d;

    const int64_t full = a.M / d;  // full slices in a gradient
    int64_t lo = a.offs[b], hi = a.offs[b + 1] < full ? a.offs[b + 1] : full;
    if (hi < lo) hi = lo;
    const int64_t cnt = hi - lo;
    const int64_t j0 = lo + cnt * p / a.P, j1 = lo + cnt * (p + 1) / a.P;

    double acc[TB][TB];
    double sacc[TB];
#pragma unroll
    for (int i = 0; i < TB; ++i) {
        sacc[i] = 0.0;
#pragma unroll
        for (int j = 0; j < TB; ++j) acc[i][j] = 0.0;
    }
    for (int i = tid; i < MOM_TILE * DP; i += MOM_THREADS) (&xs[0][0])[i] = 0.f;

    for (int l = 0; l < a.L; ++l) {
        const void* g = a.grads.p[l];
        for (int64_t c0 = j0; c0 < j1; c0 += MOM_TILE) {
            const int ns = (int)(j1 - c0 < MOM_TILE ? j1 - c0 : MOM_TILE);
            __syncthreads();
            for (int i = tid; i < ns * d; i += MOM_THREADS) {
                int s = i / d, e = i - s * d;
                xs[s][e] = load_elem(g, BF16, c0 * d + i);
            }
            __syncthreads();
            for (int s = 0; s < ns; ++s) {
                double xr[TB], xc[TB];
#pragma unroll
                for (int i = 0; i < TB; ++i) {
                    xr[i] = (double)xs[s][ti * TB + i];
                    xc[i] = (double)xs[s][tj * TB + i];
                }
#pragma unroll
                for (int i = 0; i < TB; ++i)
#pragma unroll
                    for (int j = 0; j < TB; ++j) acc[i][j] = fma(xr[i], xc[j], acc[i][j]);
                if (ti == 0) {
#pragma unroll
                    for (int j = 0; j < TB; ++j) sacc[j] += xc[j];
                }
            }
        }
    }
    double* out = a.part + ((size_t)b * a.P + p) * (size_t)(d * d + d);
#pragma unroll
    for (int i = 0; i < TB; ++i)
#pragma unroll
        for (int j = 0; j < TB; ++j) {
            int r = ti * TB + i, c = tj * TB + j;
            if (r < d && c < d) out[r * d + c] += acc[i][j];
        }
    if (ti == 0) {
#pragma unroll
        for (int j = 0; j < TB; ++j) {
            int c = tj * TB + j;
            if (c < d) out[d * d + c] += sacc[j];
        }
    }
}

__global__ void fill_zero_kernel(double* p, int64_t n)
{
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x)
        p[i] = 0.0;
}

// mom[b][e] = part[b][0][e] + part[b][1][e] + ... in that order.
__global__ void reduce_partials_kernel(const double* part, double* mom, int P, int W)
{
    const int b = blockIdx.y;
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= W) return;
    const double* src = part + (size_t)b * P * W + e;
    double acc = 0.0;
    for (int p = 0; p < P; ++p) acc += src[(size_t)p * W];
    mom[(size_t)b * W + e] = acc;
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
    const int64_t* offs;
    int64_t M;
    int L, d, k;
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
    const int64_t full = a.M / d;
    int64_t lo = a.offs[b], hi = a.offs[b + 1] < full ? a.offs[b + 1] : full;
    const double ns = hi > lo ? (double)((hi - lo) * (int64_t)a.L) : 0.0;
    const double inv = ns > 0.0 ? 1.0 / ns : 0.0;

    double* V = a.V + (size_t)b * n * n;
    double* cov = a.cov + (size_t)b * d * d;
    double fro2 = 0.0;
    for (int i = tid; i < n * n; i += nth) {
        int r = i / n, c = i - r * n;
        double v = 0.0;
        if (r < d && c < d) {
            // upper and lower halves of the Gram sum are bit-identical (same products, same order)
            v = mom[r * d + c] * inv - (mom[d * d + r] * inv) * (mom[d * d + c] * inv);
            cov[r * d + c] = v;
        }
        A[i] = v;
        V[i] = r == c ? 1.0 : 0.0;
        fro2 += v * v;
    }
    for (int i = tid; i < d; i += nth) a.mu[(size_t)b * d + i] = (float)(mom[d * d + i] * inv);
    fro2 = block_sum(fro2, red);

    int sweeps_used = -1;
    for (int sweep = 0; sweep <= a.max_sweeps; ++sweep) {
        double off2 = 0.0;
        for (int i = tid; i < n * n; i += nth) {
            int r = i / n, c = i - r * n;
            if (r != c) off2 += A[i] * A[i];
        }
        off2 = block_sum(off2, red);
        if (!(off2 > a.tol * a.tol * fro2)) { sweeps_used = sweep; break; }
        if (off2 != off2) break;  // NaN: give up
        if (sweep == a.max_sweeps) break;

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
            for (int idx = tid; idx < n * half; idx += nth) {
                const int row = idx / half, j = idx - row * half;
                const int r = pp[j], t = qq[j];
                const double cj = cs[j], sj = sn[j];
                double vr = V[row * n + r], vt = V[row * n + t];
                V[row * n + r] = cj * vr - sj * vt;
                V[row * n + t] = sj * vr + cj * vt;
            }
            __syncthreads();
        }
    }

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

// ======================================================================================
template <int TB>
static void launch_moments(const gvq_basis* h, const MomArgs& a, hipStream_t st)
{
    dim3 grid(h->P, h->B);
    if (h->dtype == GVQ_BF16)
        hipLaunchKernelGGL((moments_kernel<TB, true>), grid, dim3(MOM_THREADS), 0, st, a);
    else
        hipLaunchKernelGGL((moments_kernel<TB, false>), grid, dim3(MOM_THREADS), 0, st, a);
}

size_t gvq_eigen_lds_bytes(int d)
{
    const int n = d + (d & 1), half = n / 2;
    return sizeof(double) * ((size_t)n * n + 2 * half + 32 + n) + sizeof(int) * (2 * half + n);
}

int gvq_launch_fit(gvq_basis* h, const void* const* grads, int L, hipStream_t st)
{
    const int d = h->d, W = d * d + d;
    const int64_t npart = (int64_t)h->B * h->P * W;
    hipLaunchKernelGGL(fill_zero_kernel, dim3(1024), dim3(256), 0, st, h->d_part, npart);
    GVQ_HIP(hipGetLastError());

    for (int l0 = 0; l0 < L; l0 += GVQ_MAX_PTRS) {
        MomArgs a;
        a.L = L - l0 < GVQ_MAX_PTRS ? L - l0 : GVQ_MAX_PTRS;
        for (int i = 0; i < a.L; ++i) a.grads.p[i] = grads[l0 + i];
        a.offs = h->d_offs; a.M = h->M; a.d = d; a.P = h->P; a.part = h->d_part;
        if (d <= 16) launch_moments<1>(h, a, st);
        else if (d <= 32) launch_moments<2>(h, a, st);
        else if (d <= 64) launch_moments<4>(h, a, st);
        else launch_moments<8>(h, a, st);
        GVQ_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(reduce_partials_kernel, dim3((W + 255) / 256, h->B), dim3(256), 0, st,
                       h->d_part, h->d_mom, h->P, W);
    GVQ_HIP(hipGetLastError());

    EigArgs e;
    e.mom = h->d_mom; e.offs = h->d_offs; e.M = h->M; e.L = L; e.d = d; e.k = h->k;
    e.cov = h->d_cov; e.V = h->d_V; e.eig = h->d_eig; e.U = h->d_U; e.mu = h->d_mu;
    e.sweeps = h->d_sweeps; e.max_sweeps = 60; e.tol = 1e-15;
    const size_t lds = gvq_eigen_lds_bytes(d);
    static bool attr_set = false;
    if (!attr_set) {
        GVQ_HIP(hipFuncSetAttribute((const void*)eigen_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)gvq_eigen_lds_bytes(GVQ_MAX_D)));
        attr_set = true;
    }
    const int threads = d > 64 ? 1024 : (d > 16 ? 256 : 64);
    hipLaunchKernelGGL(eigen_kernel, dim3(h->B), dim3(threads), lds, st, e);
    GVQ_HIP(hipGetLastError());
    return gvq_launch_pack(h, st);
}
