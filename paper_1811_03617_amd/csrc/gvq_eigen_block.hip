// Eigensolver of the basis refresh for d > 64 (GradiVeQ Section 2, PCA paragraph: "applies SVD to
// obtain the eigen matrix U and eigen vector s"; Section 3, "slice size": the covariance is K x K
// with K up to several hundred): the cyclic two-sided Jacobi method in float64 with its rotations
// regrouped by blocks, any number of bases side by side.
//
// The n x n matrix (n = d rounded up to a multiple of 64, zero padded) is cut into p = n / 32 blocks
// of 32 indices.  A sweep visits every pair of blocks once, in p - 1 rounds of p / 2 disjoint pairs
// (the round-robin "tournament" order).  For a block pair (I, J)
//   solve: one work-group gathers the 64 x 64 matrix S = [[A_II, A_IJ], [A_JI, A_JJ]] into LDS and
//          rotates its index pairs once, in rounds of 32 disjoint pairs (all pairs of the 64 indices in
//          the first round of a sweep, afterwards only those across the two blocks: a sweep then
//          rotates every index pair of the matrix exactly once), accumulating the rotations in Q
//          (64 x 64, LDS).  S goes back into A (its annihilated entries exactly zero), Q into a
//          per-pair buffer;
//   apply: A <- Q_all^T A Q_all and V <- V Q_all with Q_all the direct sum of the round's Q's: block
//          (i, j) of the pair grid becomes Q_i^T A_(i,j) Q_j, which reads nothing but itself, so the
//          update is in place; one work-group per block with i < j (the mirror image is written
//          along) and one per 64 rows x pair of V, the two products on the fp64 matrix pipe.
// The next round's S of a block pair lies inside ONE block of this round's pair grid (plus diagonal
// blocks that this round does not touch), so the work-group that applies that block goes straight on
// to the next round's solve: a round is one launch, a sweep p + 1 of them (the convergence check, the
// first solve, p - 1 rounds), a refresh a few hundred instead of the tens of thousands that one
// launch per round of scalar rotations took.  Launches after convergence see a per-basis flag and
// return at once.  Convergence: squared off-diagonal mass <= tol^2 of the whole, checked once per
// sweep with a fixed summation order; NaN stops with "not converged".
// A padding index has a zero row and column, is never rotated (its pivot is exactly zero), and
// stays in its place beyond index d.
#include "gvq_internal.h"

#define BJ_MAX_OUTER 30     // outer sweeps enqueued (12-14 used on full-rank data; a sweep is p + 1 launches)

struct BjArgs {
    const double* mom;                 // [B][d*d+d]
    const unsigned long long* nsamp;   // [B] samples behind the moments
    int d, n, k, p;                    // p = n / 32 blocks, even
    int cgroups;                       // work-groups per basis of the convergence check (<= BJ_CHECK_GROUPS)
    double* cov;                       // [B][d][d]
    double* A;                         // [B][n][n]
    double* V;                         // [B][n][n]
    double* Q;                         // [2][B][p/2][64][64] rotations of the current round and of the next
    double* fro2;                      // [B] squared Frobenius norm of A (from the sweep's check)
    double* part;                      // [B][BJ_CHECK_GROUPS][2] partial sums of the check
    double* eig;                       // [B][d]
    float* U;                          // [B][d][k]
    float* mu;                         // [B][d]
    int* sweeps;                       // [B]
    int* state;                        // [B][4] {done, sweeps used or -1, arrivals at the check, -}
    double tol;
};

// Index pair i of the round-robin schedule in round `round` over m items (m even): pair 0 is
// (round, m-1), pair i is ((round + i) mod (m-1), (round - i) mod (m-1)); returned with a < b.
__device__ __forceinline__ void bj_pair(int m, int round, int i, int& a, int& b)
{
    if (i == 0) { a = round; b = m - 1; }
    else { a = (round + i) % (m - 1); b = (round - i + (m - 1)) % (m - 1); }
    if (a > b) { const int u = a; a = b; b = u; }
}

// mu = s/n, C = G/n - mu mu^T (true divisions: a constant gradient gives exactly C = 0),
// A <- C padded to n x n, V <- identity.
__global__ __launch_bounds__(256) void bj_init_kernel(BjArgs a)
{
    const int b = blockIdx.y, d = a.d, n = a.n;
    const double* mom = a.mom + (size_t)b * ((size_t)d * d + d);
    const double ns = (double)a.nsamp[b];
    double* A = a.A + (size_t)b * n * n;
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

// Start of outer sweep `sweep`: stop when the off-diagonal mass is below tol^2 of the whole, on NaN,
// or when the sweep budget is used up.  a.cgroups work-groups per basis sum a share of the rows
// each; the one that finishes last adds the partial sums in their fixed order and decides.
#define BJ_CHECK_GROUPS 32
__global__ __launch_bounds__(256) void bj_check_kernel(BjArgs a, int sweep, int max_sweeps)
{
    __shared__ double red_off[4], red_all[4];
    __shared__ int last;
    const int b = blockIdx.y, g = blockIdx.x, n = a.n, tid = threadIdx.x;
    if (a.state[4 * b]) return;
    const double* A = a.A + (size_t)b * n * n;
    const int G = a.cgroups;
    const int r0 = (int)((int64_t)n * g / G), r1 = (int)((int64_t)n * (g + 1) / G);
    double off2 = 0.0, all2 = 0.0;
    for (int i = r0 * n + tid; i < r1 * n; i += 256) {
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
        double* part = a.part + ((size_t)b * BJ_CHECK_GROUPS + g) * 2;
        part[0] = (red_off[0] + red_off[1]) + (red_off[2] + red_off[3]);
        part[1] = (red_all[0] + red_all[1]) + (red_all[2] + red_all[3]);
        __threadfence();
        last = atomicAdd(a.state + 4 * b + 2, 1) == G - 1;
    }
    __syncthreads();
    if (!last || tid != 0) return;
    __threadfence();
    double so = 0.0, sa = 0.0;
    for (int i = 0; i < G; ++i) {
        const volatile double* part = a.part + ((size_t)b * BJ_CHECK_GROUPS + i) * 2;
        so += part[0];
        sa += part[1];
    }
    int done = 0, used = -1;
    if (so != so || sa != sa) { done = 1; used = -1; }                    // NaN: no convergence
    else if (!(so > a.tol * a.tol * sa)) { done = 1; used = sweep; }
    else if (sweep >= max_sweeps) done = 1;
    a.fro2[b] = sa;
    a.state[4 * b + 2] = 0;   // the counter, for the next sweep's check
    if (done) {
        a.state[4 * b + 1] = used;
        __threadfence();
        a.state[4 * b + 0] = 1;
    }
}

// Global index of local index x (0 .. 2nb-1) of the block pair (I, J).
__device__ __forceinline__ int bj_global(int nb, int I, int J, int x)
{
    return x < nb ? I * nb + x : J * nb + (x - nb);
}

// 1 / sqrt(x) in full double precision for x in the range where x and 1/x are normal numbers: the
// hardware's approximation (v_rsq_f64) and two Newton steps.
__device__ __forceinline__ double bj_rsqrt(double x)
{
    double y = __builtin_amdgcn_rsq(x);
    const double h = 0.5 * x;
    y = y * (1.5 - h * y * y);
    y = y * (1.5 - h * y * y);
    return y;
}

// Rotation (c, s) that annihilates a_pq: tan of the angle is the smaller root of t^2 + 2 t theta - 1 = 0,
// theta = (a_qq - a_pp) / (2 a_pq).  With dd = a_qq - a_pp and h = sqrt(dd^2 + 4 a_pq^2):
//     c^2 = (1 + |dd| / h) / 2,   s = sgn(dd) a_pq / (h c)        (dd = 0 counts as positive),
// which needs two reciprocal square roots and no division: this runs on 32 lanes between two barriers of
// every inner round, with the whole work-group waiting for it.  Outside the range where dd^2 + 4 a_pq^2
// is safely a normal number the textbook form with its divisions is used.
__device__ __forceinline__ void bj_rotation(double app, double aqq, double apq, double& c, double& s)
{
    c = 1.0; s = 0.0;
    if (apq == 0.0) return;
    const double dd = aqq - app;
    const double x = dd * dd + 4.0 * apq * apq;
    if (x > 1e-280 && x < 1e280) {
        const double rh = bj_rsqrt(x);
        const double c2 = 0.5 + 0.5 * fabs(dd) * rh;
        const double rc = bj_rsqrt(c2);
        c = c2 * rc;
        s = (dd >= 0.0 ? apq : -apq) * rh * rc;
        return;
    }
    const double r = hypot(dd, 2.0 * apq);
    const double t = (dd >= 0.0 ? 2.0 : -2.0) * apq / (fabs(dd) + r);
    c = 1.0 / sqrt(1.0 + t * t);
    s = t * c;
}

// Pair i of inner round t.  full: the round-robin order over all m = 2nb local indices (m - 1 rounds);
// else only the pairs with one index in each block (nb rounds): (i, nb + (i + t) mod nb).
__device__ __forceinline__ void bj_inner_pair(bool full, int nb, int t, int i, int& p, int& q)
{
    if (full) {
        bj_pair(2 * nb, t, i, p, q);
    } else {
        p = i;
        q = nb + (i + t) % nb;
    }
}

#define BJ_NB 32
#define BJ_M 64
#define BJ_LD 66            // row stride of the LDS matrices of the apply step (doubles)
typedef double bj_d4 __attribute__((ext_vector_type(4)));

// One pass over the index pairs of the block pair (I, J) (see the file comment), 256 threads.
// LDS: S and Q (64 x 64 each) and two sets of rotation parameters.  Per inner round: every thread
// updates 2 x 2 blocks of S; then, between two barriers, the first wave works out the next round's
// rotations from the new S while the other waves apply this round's to Q.  qout: where Q goes.
__device__ __forceinline__ void bj_solve_pair(const BjArgs& a, double* smem, double* A, int I, int J, bool full,
                                              double* qout)
{
    constexpr int nb = BJ_NB, m = BJ_M, half = BJ_NB;
    const int n = a.n, tid = threadIdx.x;
    double* S = smem;                    // [m][m]
    double* Q = S + m * m;               // [m][m]
    double* cs = Q + m * m;              // [2][half]
    double* sn = cs + 2 * half;          // [2][half]
    int* pp = (int*)(sn + 2 * half);     // [2][half]
    int* qq = pp + 2 * half;             // [2][half]
    const int rounds = full ? m - 1 : nb;

    for (int i = tid; i < m * m; i += 256) {
        const int r = i / m, c = i - r * m;
        S[i] = A[(size_t)bj_global(nb, I, J, r) * n + bj_global(nb, I, J, c)];
        Q[i] = r == c ? 1.0 : 0.0;
    }
    __syncthreads();
    auto params = [&](int t) {           // threads 0 .. half-1
        int p, q;
        bj_inner_pair(full, nb, t, tid, p, q);
        double c, s;
        bj_rotation(S[p * m + p], S[q * m + q], S[p * m + q], c, s);
        const int o = (t & 1) * half + tid;
        pp[o] = p; qq[o] = q; cs[o] = c; sn[o] = s;
    };
    if (tid < half) params(0);
    __syncthreads();
    // Thread layout of a round: rotation j = tid % 32 on the column side for every thread (its parameters are read
    // once per round), rotations i = tid / 32 + 8 u on the row side of S (four 2 x 2 blocks per thread), rows
    // (tid - 64) / 32 + 6 v of Q for the three waves that update it.  All loops unrolled: the LDS reads of a
    // thread's blocks are in flight together instead of one round trip after the other.
    const int j = tid & (half - 1), i0 = tid >> 5, qrow0 = (tid - 64) >> 5;
    for (int t = 0; t < rounds; ++t) {
        const int o = (t & 1) * half;
        const int r = pp[o + j], u = qq[o + j];
        const double cj = cs[o + j], sj = sn[o + j];
        // S <- J^T S J: one 2 x 2 block per (rotation i, rotation j), in place (a block reads only itself)
        int p4[4], q4[4];
        double ci4[4], si4[4], apr[4], apu[4], aqr[4], aqu[4];
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const int i = i0 + 8 * v;
            p4[v] = pp[o + i]; q4[v] = qq[o + i]; ci4[v] = cs[o + i]; si4[v] = sn[o + i];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            apr[v] = S[p4[v] * m + r]; apu[v] = S[p4[v] * m + u];
            aqr[v] = S[q4[v] * m + r]; aqu[v] = S[q4[v] * m + u];
        }
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            const double ci = ci4[v], si = si4[v];
            const double xpr = ci * apr[v] - si * aqr[v], xpu = ci * apu[v] - si * aqu[v];
            const double xqr = si * apr[v] + ci * aqr[v], xqu = si * apu[v] + ci * aqu[v];
            double ypr = cj * xpr - sj * xpu, ypu = sj * xpr + cj * xpu;
            double yqr = cj * xqr - sj * xqu, yqu = sj * xqr + cj * xqu;
            if (i0 + 8 * v == j) { ypu = 0.0; yqr = 0.0; }
            S[p4[v] * m + r] = ypr; S[p4[v] * m + u] = ypu; S[q4[v] * m + r] = yqr; S[q4[v] * m + u] = yqu;
        }
        __syncthreads();
        if (tid < 64) {
            if (tid < half && t + 1 < rounds) params(t + 1);
        } else {
            // Q <- Q J, columns r and u of rows qrow0 + 6 v
            double vr[11], vu[11];
#pragma unroll
            for (int v = 0; v < 11; ++v) {
                const int row = qrow0 + 6 * v;
                if (row < m) { vr[v] = Q[row * m + r]; vu[v] = Q[row * m + u]; }
            }
#pragma unroll
            for (int v = 0; v < 11; ++v) {
                const int row = qrow0 + 6 * v;
                if (row < m) {
                    Q[row * m + r] = cj * vr[v] - sj * vu[v];
                    Q[row * m + u] = sj * vr[v] + cj * vu[v];
                }
            }
        }
        __syncthreads();
    }
    for (int i = tid; i < m * m; i += 256) {
        const int r = i / m, c = i - r * m;
        A[(size_t)bj_global(nb, I, J, r) * n + bj_global(nb, I, J, c)] = S[i];
        qout[i] = Q[i];
    }
}

// The first solve of a sweep (all index pairs of every block pair).  grid (p/2, B), 256 threads.
__global__ __launch_bounds__(256) void bj_solve_kernel(BjArgs a, int qbuf)
{
    extern __shared__ double bj_smem[];
    const int b = blockIdx.y;
    if (a.state[4 * b]) return;
    int I, J;
    bj_pair(a.p, 0, blockIdx.x, I, J);
    const int P2 = a.p / 2;
    bj_solve_pair(a, bj_smem, a.A + (size_t)b * a.n * a.n, I, J, true,
                  a.Q + (((size_t)qbuf * gridDim.y + b) * P2 + blockIdx.x) * BJ_M * BJ_M);
}

// Which pair of round `round` holds block `blk` (inverse of bj_pair over p blocks).
__device__ __forceinline__ int bj_pair_of_block(int p, int round, int blk)
{
    if (blk == p - 1 || blk == round) return 0;
    const int delta = (blk - round + (p - 1)) % (p - 1);      // 1 .. p-2
    return delta <= p / 2 - 1 ? delta : (p - 1) - delta;
}

// One round: apply (see the file comment) and, for the work-group whose block holds the next round's
// S of a block pair, that pair's solve (`next` = next round of the same sweep, -1 = none).
// Work items: first the (p/2)(p/2 - 1)/2 blocks (i < j) of A, then the (n / 64) x (p/2) blocks of V.
// 256 threads = 4 waves; wave w owns rows 16w .. 16w+15 of the 64 x 64 products, which run on
// v_mfma_f64_16x16x4_f64: A operand lane l = (row l%16, step l/16), B operand lane l = (step l/16,
// column l%16), result register r of lane l = (row 4r + l/16, column l%16).
// Q of round r is read from buffer r % 2, the next round's is written to the other one.
__global__ __launch_bounds__(256) void bj_round_kernel(BjArgs a, int round, int next)
{
    extern __shared__ double bj_smem[];
    constexpr int M = BJ_M, NB = BJ_NB, LD = BJ_LD;
    const int b = blockIdx.y;
    if (a.state[4 * b]) return;
    const int n = a.n, tid = threadIdx.x, lane = tid & 63, w = tid >> 6, lm = lane & 15, lk = lane >> 4;
    const int P2 = a.p / 2, NA = P2 * (P2 - 1) / 2;
    double* X = bj_smem;                 // [M][LD] the block, then T = X Q_j, then the result
    double* Ql = X + M * LD;             // [M][LD] Q_j, then Q_i
    double* A = a.A + (size_t)b * n * n;
    double* V = a.V + (size_t)b * n * n;
    const double* Qround = a.Q + ((size_t)(round & 1) * gridDim.y + b) * P2 * M * M;

    int item = blockIdx.x, pi = 0, pj = 0, rowblk = 0;
    const bool isA = item < NA;
    if (isA) {
        int rem = item;                  // item -> (pi < pj): row pi holds P2 - 1 - pi items
        while (rem >= P2 - 1 - pi) { rem -= P2 - 1 - pi; ++pi; }
        pj = pi + 1 + rem;
    } else {
        item -= NA;
        rowblk = item / P2;
        pj = item - rowblk * P2;
    }
    int Ii = 0, Ji = 0, Ij, Jj;
    bj_pair(a.p, round, pj, Ij, Jj);
    if (isA) bj_pair(a.p, round, pi, Ii, Ji);

    double* src = isA ? A : V;
    for (int i = tid; i < M * M; i += 256) {
        const int r = i / M, c = i - r * M;
        const int gr = isA ? bj_global(NB, Ii, Ji, r) : rowblk * M + r;
        X[r * LD + c] = src[(size_t)gr * n + bj_global(NB, Ij, Jj, c)];
        Ql[r * LD + c] = Qround[(size_t)pj * M * M + i];
    }
    __syncthreads();
    // T = X Q_j
    bj_d4 acc[4];
#pragma unroll
    for (int ct = 0; ct < 4; ++ct) acc[ct] = bj_d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
    for (int kk = 0; kk < M / 4; ++kk) {
        const double av = X[(16 * w + lm) * LD + 4 * kk + lk];
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
            acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, Ql[(4 * kk + lk) * LD + 16 * ct + lm], acc[ct], 0, 0, 0);
    }
    __syncthreads();   // everyone is done reading X and Q_j
#pragma unroll
    for (int ct = 0; ct < 4; ++ct)
#pragma unroll
        for (int r = 0; r < 4; ++r) X[(16 * w + 4 * r + lk) * LD + 16 * ct + lm] = acc[ct][r];
    if (isA) {
        for (int i = tid; i < M * M; i += 256) Ql[(i / M) * LD + (i % M)] = Qround[(size_t)pi * M * M + i];
        __syncthreads();
        // Y = Q_i^T T
#pragma unroll
        for (int ct = 0; ct < 4; ++ct) acc[ct] = bj_d4{0.0, 0.0, 0.0, 0.0};
#pragma unroll 4
        for (int kk = 0; kk < M / 4; ++kk) {
            const double av = Ql[(4 * kk + lk) * LD + 16 * w + lm];
#pragma unroll
            for (int ct = 0; ct < 4; ++ct)
                acc[ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, X[(4 * kk + lk) * LD + 16 * ct + lm], acc[ct], 0, 0, 0);
        }
        __syncthreads();   // everyone is done reading T
#pragma unroll
        for (int ct = 0; ct < 4; ++ct)
#pragma unroll
            for (int r = 0; r < 4; ++r) X[(16 * w + 4 * r + lk) * LD + 16 * ct + lm] = acc[ct][r];
    }
    __syncthreads();
    // write the block back (rows of 32 consecutive numbers), for A also its mirror image
    for (int i = tid; i < M * M; i += 256) {
        const int r = i / M, c = i - r * M;
        const int gr = isA ? bj_global(NB, Ii, Ji, r) : rowblk * M + r;
        src[(size_t)gr * n + bj_global(NB, Ij, Jj, c)] = X[r * LD + c];
    }
    if (!isA) return;
    for (int i = tid; i < M * M; i += 256) {
        const int c = i / M, r = i - c * M;     // consecutive threads along r: rows of the mirror image
        A[(size_t)bj_global(NB, Ij, Jj, c) * n + bj_global(NB, Ii, Ji, r)] = X[r * LD + c];
    }
    if (next < 0) return;
    // the next round's block pairs whose S lies in this block (its other entries are on the diagonal
    // of this round's pair grid, which the apply step leaves alone): solve them here
    __syncthreads();   // this work-group's writes to A are visible to all its threads
    for (int x = 0; x < P2; ++x) {
        int In, Jn;
        bj_pair(a.p, next, x, In, Jn);
        int lo = bj_pair_of_block(a.p, round, In), hi = bj_pair_of_block(a.p, round, Jn);
        if (lo > hi) { const int u = lo; lo = hi; hi = u; }
        if (lo != pi || hi != pj) continue;   // uniform over the work-group
        bj_solve_pair(a, bj_smem, A, In, Jn, false,
                      a.Q + (((size_t)(next & 1) * gridDim.y + b) * P2 + x) * M * M);
        __syncthreads();
    }
}

// Eigenvalues in decreasing order (ties: lower index first, NaN last), the k leading
// eigenvectors with the largest-magnitude entry (lowest index on ties) made positive.
__global__ __launch_bounds__(1024) void bj_finish_kernel(BjArgs a)
{
    __shared__ double lam[GVQ_MAX_D];
    __shared__ int order[GVQ_MAX_D];
    const int b = blockIdx.x, d = a.d, n = a.n, tid = threadIdx.x;
    const double* A = a.A + (size_t)b * n * n;
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

// ======================================================================================
int gvq_bj_padded(int d) { return (d + BJ_M - 1) / BJ_M * BJ_M; }
size_t gvq_bj_q_doubles(int d)   // per basis: two buffers of p/2 rotations
{
    return (size_t)2 * (gvq_bj_padded(d) / BJ_M) * BJ_M * BJ_M;
}

int gvq_launch_eigen_block(gvq_basis* h, hipStream_t st)
{
    const int d = h->d, n = gvq_bj_padded(d), p = n / BJ_NB, P2 = p / 2;
    BjArgs a;
    a.mom = h->d_mom; a.nsamp = h->d_nsamp; a.d = d; a.n = n; a.k = h->k; a.p = p;
    a.cov = h->d_cov; a.A = h->d_bjA; a.V = h->d_V; a.Q = h->d_bjQ; a.fro2 = h->d_bjfro; a.part = h->d_bjfro + h->B;
    a.eig = h->d_eig; a.U = h->d_U; a.mu = h->d_mu; a.sweeps = h->d_sweeps; a.state = h->d_jstate; a.tol = 1e-15;
    a.cgroups = 2 * h->num_cu / h->B;   // the check's launch fills the chip once
    if (a.cgroups > BJ_CHECK_GROUPS) a.cgroups = BJ_CHECK_GROUPS;
    if (a.cgroups > n / 8) a.cgroups = n / 8;
    if (a.cgroups < 1) a.cgroups = 1;
    const size_t lds = sizeof(double) * 2 * BJ_M * BJ_LD + 2048;   // either step's matrices, the rotation parameters
    static gvq_once_per_device once;
    if (once.first(h->device)) {
        GVQ_HIP(hipFuncSetAttribute((const void*)bj_solve_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        GVQ_HIP(hipFuncSetAttribute((const void*)bj_round_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    }
    hipLaunchKernelGGL(bj_init_kernel, dim3(n >= 512 ? 256 : 32, h->B), dim3(256), 0, st, a);
    GVQ_HIP(hipGetLastError());
    const int items = P2 * (P2 - 1) / 2 + (n / BJ_M) * P2;
    for (int sweep = 0; sweep <= BJ_MAX_OUTER; ++sweep) {
        hipLaunchKernelGGL(bj_check_kernel, dim3(a.cgroups, h->B), dim3(256), 0, st, a, sweep, BJ_MAX_OUTER);
        GVQ_HIP(hipGetLastError());
        if (sweep == BJ_MAX_OUTER) break;
        hipLaunchKernelGGL(bj_solve_kernel, dim3(P2, h->B), dim3(256), lds, st, a, 0);
        for (int round = 0; round < p - 1; ++round)
            hipLaunchKernelGGL(bj_round_kernel, dim3(items, h->B), dim3(256), lds, st, a, round,
                               round + 1 < p - 1 ? round + 1 : -1);
        GVQ_HIP(hipGetLastError());
    }
    hipLaunchKernelGGL(bj_finish_kernel, dim3(h->B), dim3(1024), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}
