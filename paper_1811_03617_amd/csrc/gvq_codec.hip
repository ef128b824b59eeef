// Codec kernels for gfx950: compress (Eq. 2), aggregate (Eq. 3), decompress (Eq. 4) of
// GradiVeQ, Section 2.  All three stream the gradient once; U and mu live in registers.
//
// The two projections are tall-skinny contractions (inner dimension d <= 128 or k <= 32).
// At d = 128, k = 32 they need ~13 flop per HBM byte, more than the fp32 vector units
// deliver at HBM speed, so the contraction runs on v_mfma_f32_16x16x4_f32.  Operand layout
// of that instruction on a 64-lane wave, lane l:
//     A (16x4):  A[m = l%16][kk = l/16]        B (4x16):  B[kk = l/16][n = l%16]
//     D (16x16): register r of lane l holds D[m = 4*(l/16) + r][n = l%16]
// Slices always sit on the n side (lane l%16 = slice within a 16-slice tile), so each lane
// ends with 4 consecutive outputs of one slice in its 4 result registers and stores them
// as one 128-bit word.
#include "gvq_internal.h"

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

#define WAVES_PER_WG 4
#define WG_THREADS (64 * WAVES_PER_WG)
#define TILE_SLICES 16

struct CodecArgs {
    const void* in;       // compress: gradient; decompress: compressed [S][k]
    void* out;            // compress: compressed [S][k]; decompress: gradient
    const float* U;       // [B][d][k]
    const float* mu;      // [B][d]
    const int64_t* offs;  // [B+1] slice offsets of the bases
    int64_t M, S;
    int B, d, k;
    float n_workers;      // compress only
};

// Largest b with offs[b] <= j (offs[0] = 0, offs[B] = S > j).
__device__ __forceinline__ int find_block(const int64_t* offs, int B, int64_t j)
{
    int lo = 0, hi = B - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (offs[mid] <= j) lo = mid; else hi = mid - 1;
    }
    return lo;
}

__device__ __forceinline__ float bf16_to_f32(unsigned int hi16)
{
    return __uint_as_float(hi16 << 16);
}

// Round-to-nearest-even fp32 -> bf16 bit pattern (NaN kept quiet).
__device__ __forceinline__ unsigned int f32_to_bf16_rne(float f)
{
    unsigned int u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x40u;
    return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// --------------------------------------------------------------------------------------
// compress, MFMA path.  D in {16,32,64,128}, NT = ceil(k/16) in {1,2}.
//
// One wave owns a contiguous range of 16-slice tiles.  Per tile: every lane loads 128-bit
// words of the tile in memory order (fully coalesced: the tile is one contiguous run of
// 16*D elements), subtracts mu/N, and parks them in the wave's private LDS region; the
// lanes then read the same data back in the B-operand order (lane = slice, 4 consecutive
// elements per 128-bit read).  Chunk c (4 floats) of slice s lives at 128-bit slot
// s*CPS + (c ^ swz(s)), a XOR swizzle that keeps 8 consecutive lanes on 8 distinct
// 128-bit bank groups for the transposed read.
// The contraction index may be visited in any order as long as U follows: MFMA step
// (q, j) multiplies elements e = 4*(4q + kk) + j, kk = l/16.
// --------------------------------------------------------------------------------------
template <int D>
__device__ __forceinline__ int swz(int s)
{
    return (D >= 32) ? (s & 7) : ((s >> 1) & 3);
}

template <int D, int NT, bool BF16>
__global__ __launch_bounds__(WG_THREADS) void compress_mfma_kernel(CodecArgs a)
{
    constexpr int CPS = D / 4;                    // fp32 128-bit chunks per slice
    constexpr int EPL = BF16 ? 8 : 4;             // elements per 128-bit global load
    constexpr int LCPS = D / EPL;                 // load chunks per slice
    constexpr int TILE_LOADS = TILE_SLICES * LCPS;  // 128-bit loads per tile
    constexpr int NL = (TILE_LOADS + 63) / 64;    // loads per lane per tile
    constexpr int NQ = CPS / 4;                   // 128-bit LDS reads per lane per tile

    __shared__ f4 lds_all[WAVES_PER_WG][TILE_SLICES * CPS];
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    f4* lds = lds_all[wave];

    const int64_t T = (a.S + TILE_SLICES - 1) / TILE_SLICES;
    const int64_t W = (int64_t)gridDim.x * WAVES_PER_WG;
    const int64_t w = (int64_t)blockIdx.x * WAVES_PER_WG + wave;
    const int64_t t0 = w * T / W, t1 = (w + 1) * T / W;
    if (t0 >= t1) return;

    const int n_ = lane & 15, kk = lane >> 4;
    // this lane's fixed position inside every tile, for the coalesced loads
    const int lc = lane % LCPS;                   // load chunk within the slice

    // ---- per-basis state -------------------------------------------------------------
    int cur_b = find_block(a.offs, a.B, t0 * TILE_SLICES);
    int64_t blk_begin = a.offs[cur_b], blk_end = a.offs[cur_b + 1];
    float ufrag[NQ][4][NT];
    float mun[EPL];

    auto load_basis = [&](int b) {
        const float* Ub = a.U + (size_t)b * D * a.k;
        const float* mub = a.mu + (size_t)b * D;
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    int e = 4 * (4 * q + kk) + j, c = 16 * nt + n_;
                    ufrag[q][j][nt] = c < a.k ? Ub[e * a.k + c] : 0.0f;
                }
#pragma unroll
        for (int i = 0; i < EPL; ++i) mun[i] = mub[lc * EPL + i] / a.n_workers;
    };
    load_basis(cur_b);

    // ---- tile loads --------------------------------------------------------------------
    u4 regs[NL];
    auto load_tile = [&](int64_t t) {
        const int64_t base = t * TILE_SLICES * (int64_t)D;  // first element of the tile
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            int g = r * 64 + lane;
            u4 v = {0u, 0u, 0u, 0u};
            if (g < TILE_LOADS) {
                int64_t e0 = base + (int64_t)g * EPL;
                if (e0 + EPL <= a.M) {
                    v = *(const u4*)((const char*)a.in + e0 * (BF16 ? 2 : 4));
                } else if (e0 < a.M) {
                    if (BF16) {
                        const unsigned short* p = (const unsigned short*)a.in;
                        unsigned int h[8];
#pragma unroll
                        for (int i = 0; i < 8; ++i) h[i] = e0 + i < a.M ? p[e0 + i] : 0u;
                        v = u4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16),
                               h[6] | (h[7] << 16)};
                    } else {
                        const unsigned int* p = (const unsigned int*)a.in;
                        v = u4{p[e0], e0 + 1 < a.M ? p[e0 + 1] : 0u, e0 + 2 < a.M ? p[e0 + 2] : 0u,
                               e0 + 3 < a.M ? p[e0 + 3] : 0u};
                    }
                }
            }
            regs[r] = v;
        }
    };
    // park the loaded tile in LDS as fp32, minus mu/N
    auto stage_tile = [&]() {
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            int g = r * 64 + lane;
            if (g < TILE_LOADS) {
                int s = g / LCPS;
                u4 v = regs[r];
                if (BF16) {
                    f4 lo = {bf16_to_f32(v.x & 0xffffu) - mun[0], bf16_to_f32(v.x >> 16) - mun[1],
                             bf16_to_f32(v.y & 0xffffu) - mun[2], bf16_to_f32(v.y >> 16) - mun[3]};
                    f4 hi = {bf16_to_f32(v.z & 0xffffu) - mun[4 % EPL], bf16_to_f32(v.z >> 16) - mun[5 % EPL],
                             bf16_to_f32(v.w & 0xffffu) - mun[6 % EPL], bf16_to_f32(v.w >> 16) - mun[7 % EPL]};
                    lds[s * CPS + ((2 * lc) ^ swz<D>(s))] = lo;
                    lds[s * CPS + ((2 * lc + 1) ^ swz<D>(s))] = hi;
                } else {
                    f4 x = {__uint_as_float(v.x) - mun[0], __uint_as_float(v.y) - mun[1],
                            __uint_as_float(v.z) - mun[2], __uint_as_float(v.w) - mun[3]};
                    lds[s * CPS + (lc ^ swz<D>(s))] = x;
                }
            }
        }
    };

    load_tile(t0);
    for (int64_t t = t0; t < t1; ++t) {
        const int64_t s0 = t * TILE_SLICES;
        const int64_t s1 = s0 + TILE_SLICES < a.S ? s0 + TILE_SLICES : a.S;
        if (s0 >= blk_end) {  // the previous tile ended exactly on a basis boundary, or bases were skipped
            cur_b = find_block(a.offs, a.B, s0);
            blk_begin = a.offs[cur_b];
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        __builtin_amdgcn_wave_barrier();
        stage_tile();
        __builtin_amdgcn_wave_barrier();
        if (t + 1 < t1) load_tile(t + 1);

        for (;;) {
            f4 acc[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q) {
                f4 x = lds[n_ * CPS + ((4 * q + kk) ^ swz<D>(n_))];
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(ufrag[q][j][nt], x[j], acc[nt], 0, 0, 0);
            }
            // lane holds comps 16*nt + 4*kk + r of slice s0 + n_
            const int64_t j = s0 + n_;
            const int64_t lo = s0 > blk_begin ? s0 : blk_begin, hi = s1 < blk_end ? s1 : blk_end;
            if (j >= lo && j < hi) {
                float* o = (float*)a.out + j * a.k;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) {
                    int c0 = 16 * nt + 4 * kk;
                    if ((a.k & 3) == 0) {
                        if (c0 < a.k) *(f4*)(o + c0) = acc[nt];
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (c0 + r < a.k) o[c0 + r] = acc[nt][r];
                    }
                }
            }
            if (blk_end >= s1) break;
            // the tile continues into the next basis: re-centre the parked data and redo it
            float old[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i) old[i] = mun[i];
            cur_b += 1;
            blk_begin = blk_end;
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int r = 0; r < NL; ++r) {
                int g = r * 64 + lane;
                if (g < TILE_LOADS) {
                    int s = g / LCPS;
                    if (BF16) {
                        f4* p0 = &lds[s * CPS + ((2 * lc) ^ swz<D>(s))];
                        f4* p1 = &lds[s * CPS + ((2 * lc + 1) ^ swz<D>(s))];
                        f4 v0 = *p0, v1 = *p1;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            v0[i] += old[i] - mun[i];
                            v1[i] += old[(4 + i) % EPL] - mun[(4 + i) % EPL];
                        }
                        *p0 = v0;
                        *p1 = v1;
                    } else {
                        f4* p0 = &lds[s * CPS + (lc ^ swz<D>(s))];
                        f4 v0 = *p0;
#pragma unroll
                        for (int i = 0; i < 4; ++i) v0[i] += old[i] - mun[i];
                        *p0 = v0;
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    }
}

// compress, any d <= 128 and k <= d: one thread per output number.  Correct, not fast.
template <bool BF16>
__global__ __launch_bounds__(256) void compress_generic_kernel(CodecArgs a)
{
    const int64_t total = a.S * a.k;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
         o += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = o / a.k;
        const int c = (int)(o - j * a.k);
        const int b = find_block(a.offs, a.B, j);
        const float* Ub = a.U + (size_t)b * a.d * a.k;
        const float* mub = a.mu + (size_t)b * a.d;
        float acc = 0.f;
        for (int e = 0; e < a.d; ++e) {
            int64_t idx = j * a.d + e;
            float x = 0.f;
            if (idx < a.M)
                x = BF16 ? bf16_to_f32(((const unsigned short*)a.in)[idx]) : ((const float*)a.in)[idx];
            acc = fmaf(Ub[e * a.k + c], x - mub[e] / a.n_workers, acc);
        }
        ((float*)a.out)[o] = acc;
    }
}

// --------------------------------------------------------------------------------------
// decompress, MFMA path.  D in {16,32,64,128}, NQ = ceil(k/16) in {1,2}.
// A = U tile (16 elements x 4 comps), B = Y (4 comps x 16 slices): lane (n = l%16, kk = l/16)
// loads comps 16q + 4kk + {0..3} of slice n as one 128-bit word and MFMA step (q, j)
// contracts comp 16q + 4kk + j.  Result register r of element tile et is element
// 16et + 4kk + r of slice n, so each lane stores 4 consecutive outputs per tile.
// --------------------------------------------------------------------------------------
template <int D, int NQ, bool OUT_BF16>
__global__ __launch_bounds__(WG_THREADS) void decompress_mfma_kernel(CodecArgs a)
{
    constexpr int ET = D / 16;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int64_t T = (a.S + TILE_SLICES - 1) / TILE_SLICES;
    const int64_t W = (int64_t)gridDim.x * WAVES_PER_WG;
    const int64_t w = (int64_t)blockIdx.x * WAVES_PER_WG + wave;
    const int64_t t0 = w * T / W, t1 = (w + 1) * T / W;
    if (t0 >= t1) return;
    const int n_ = lane & 15, kk = lane >> 4;
    const float* Y = (const float*)a.in;

    int cur_b = find_block(a.offs, a.B, t0 * TILE_SLICES);
    int64_t blk_begin = a.offs[cur_b], blk_end = a.offs[cur_b + 1];
    float ufrag[ET][NQ][4];
    f4 mu4[ET];
    auto load_basis = [&](int b) {
        const float* Ub = a.U + (size_t)b * D * a.k;
        const float* mub = a.mu + (size_t)b * D;
#pragma unroll
        for (int et = 0; et < ET; ++et) {
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    int c = 16 * q + 4 * kk + j;
                    ufrag[et][q][j] = c < a.k ? Ub[(16 * et + n_) * a.k + c] : 0.0f;
                }
#pragma unroll
            for (int r = 0; r < 4; ++r) mu4[et][r] = mub[16 * et + 4 * kk + r];
        }
    };
    load_basis(cur_b);

    f4 y[NQ];
    auto load_tile = [&](int64_t t) {
        const int64_t j = t * TILE_SLICES + n_;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int c0 = 16 * q + 4 * kk;
            f4 v = {0.f, 0.f, 0.f, 0.f};
            if (j < a.S) {
                const float* p = Y + j * a.k + c0;
                if ((a.k & 3) == 0) {
                    if (c0 < a.k) v = *(const f4*)p;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (c0 + r < a.k) v[r] = p[r];
                }
            }
            y[q] = v;
        }
    };

    load_tile(t0);
    for (int64_t t = t0; t < t1; ++t) {
        const int64_t s0 = t * TILE_SLICES;
        const int64_t s1 = s0 + TILE_SLICES < a.S ? s0 + TILE_SLICES : a.S;
        if (s0 >= blk_end) {
            cur_b = find_block(a.offs, a.B, s0);
            blk_begin = a.offs[cur_b];
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        f4 yc[NQ];
#pragma unroll
        for (int q = 0; q < NQ; ++q) yc[q] = y[q];
        if (t + 1 < t1) load_tile(t + 1);

        for (;;) {
            const int64_t j = s0 + n_;
            const int64_t lo = s0 > blk_begin ? s0 : blk_begin, hi = s1 < blk_end ? s1 : blk_end;
            const bool mine = j >= lo && j < hi;
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                f4 acc = mu4[et];
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(ufrag[et][q][jj], yc[q][jj], acc, 0, 0, 0);
                if (mine) {
                    const int64_t e0 = j * D + 16 * et + 4 * kk;
                    if (OUT_BF16) {
                        unsigned short* o = (unsigned short*)a.out;
                        if (e0 + 4 <= a.M) {
                            u2 pk = {f32_to_bf16_rne(acc[0]) | (f32_to_bf16_rne(acc[1]) << 16),
                                     f32_to_bf16_rne(acc[2]) | (f32_to_bf16_rne(acc[3]) << 16)};
                            *(u2*)(o + e0) = pk;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (e0 + r < a.M) o[e0 + r] = (unsigned short)f32_to_bf16_rne(acc[r]);
                        }
                    } else {
                        float* o = (float*)a.out;
                        if (e0 + 4 <= a.M) {
                            *(f4*)(o + e0) = acc;
                        } else {
#pragma unroll
                            for (int r = 0; r < 4; ++r)
                                if (e0 + r < a.M) o[e0 + r] = acc[r];
                        }
                    }
                }
            }
            if (blk_end >= s1) break;
            cur_b += 1;
            blk_begin = blk_end;
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
    }
}

// decompress, any d, k: one thread per output element.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void decompress_generic_kernel(CodecArgs a)
{
    const float* Y = (const float*)a.in;
    for (int64_t o = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < a.M;
         o += (int64_t)gridDim.x * blockDim.x) {
        const int64_t j = o / a.d;
        const int e = (int)(o - j * a.d);
        const int b = find_block(a.offs, a.B, j);
        const float* Ub = a.U + (size_t)b * a.d * a.k + (size_t)e * a.k;
        float acc = 0.f;
        for (int c = 0; c < a.k; ++c) acc = fmaf(Ub[c], Y[j * a.k + c], acc);
        acc += a.mu[(size_t)b * a.d + e];
        if (OUT_BF16)
            ((unsigned short*)a.out)[o] = (unsigned short)f32_to_bf16_rne(acc);
        else
            ((float*)a.out)[o] = acc;
    }
}

// --------------------------------------------------------------------------------------
// aggregate: out[i] = ((in0[i] + in1[i]) + in2[i]) + ...   128 bits per lane per input.
// --------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void aggregate_kernel(gvq_ptrs in, int n, float* out, int64_t len)
{
    const int64_t len4 = len >> 2;
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
    for (int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < len4; i += stride) {
        f4 acc = ((const f4*)in.p[0])[i];
        for (int w = 1; w < n; ++w) acc += ((const f4*)in.p[w])[i];
        ((f4*)out)[i] = acc;
    }
    // up to 3 trailing numbers
    const int64_t i = (len4 << 2) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.x == 0 && i < len) {
        float acc = ((const float*)in.p[0])[i];
        for (int w = 1; w < n; ++w) acc += ((const float*)in.p[w])[i];
        out[i] = acc;
    }
}

// ======================================================================================
// host side
// ======================================================================================
static CodecArgs make_args(const gvq_basis* h, const void* in, void* out, int n_workers)
{
    CodecArgs a;
    a.in = in; a.out = out; a.U = h->d_U; a.mu = h->d_mu; a.offs = h->d_offs;
    a.M = h->M; a.S = h->S; a.B = h->B; a.d = h->d; a.k = h->k;
    a.n_workers = (float)n_workers;
    return a;
}

template <typename K>
static int streaming_grid(const gvq_basis* h, K kernel, int64_t tiles)
{
    int per_cu = gvq_opt_wg_per_cu();
    if (per_cu <= 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, WG_THREADS, 0) != hipSuccess || occ < 1)
            occ = 2;
        per_cu = occ;
    }
    int64_t want = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;  // at least one tile per wave
    int64_t cap = (int64_t)h->num_cu * per_cu;
    int64_t g = want < cap ? want : cap;
    return (int)(g < 1 ? 1 : g);
}

template <int D, int NT, bool BF16>
static int launch_compress_t(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    auto kern = compress_mfma_kernel<D, NT, BF16>;
    int64_t tiles = (h->S + TILE_SLICES - 1) / TILE_SLICES;
    int grid = streaming_grid(h, kern, tiles);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, bool BF16>
static int launch_compress_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    return h->k <= 16 ? launch_compress_t<D, 1, BF16>(h, a, st) : launch_compress_t<D, 2, BF16>(h, a, st);
}

int gvq_launch_compress(const gvq_basis* h, const void* grad, int n_workers, float* out, hipStream_t st)
{
    CodecArgs a = make_args(h, grad, out, n_workers);
    const bool bf = h->dtype == GVQ_BF16;
    if (h->k <= 32) {
        switch (h->d) {
        case 16: return bf ? launch_compress_d<16, true>(h, a, st) : launch_compress_d<16, false>(h, a, st);
        case 32: return bf ? launch_compress_d<32, true>(h, a, st) : launch_compress_d<32, false>(h, a, st);
        case 64: return bf ? launch_compress_d<64, true>(h, a, st) : launch_compress_d<64, false>(h, a, st);
        case 128: return bf ? launch_compress_d<128, true>(h, a, st) : launch_compress_d<128, false>(h, a, st);
        default: break;
        }
    }
    int64_t total = h->S * h->k;
    int64_t want = (total + 255) / 256, cap = (int64_t)h->num_cu * 16;
    int grid = (int)(want < cap ? want : cap);
    if (bf)
        hipLaunchKernelGGL(compress_generic_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(compress_generic_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, int NQ, bool OBF>
static int launch_decompress_t(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    auto kern = decompress_mfma_kernel<D, NQ, OBF>;
    int64_t tiles = (h->S + TILE_SLICES - 1) / TILE_SLICES;
    int grid = streaming_grid(h, kern, tiles);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, bool OBF>
static int launch_decompress_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    return h->k <= 16 ? launch_decompress_t<D, 1, OBF>(h, a, st) : launch_decompress_t<D, 2, OBF>(h, a, st);
}

int gvq_launch_decompress(const gvq_basis* h, const float* comp, void* out, gvq_dtype_t odt, hipStream_t st)
{
    CodecArgs a = make_args(h, comp, out, 1);
    const bool bf = odt == GVQ_BF16;
    if (h->k <= 32) {
        switch (h->d) {
        case 16: return bf ? launch_decompress_d<16, true>(h, a, st) : launch_decompress_d<16, false>(h, a, st);
        case 32: return bf ? launch_decompress_d<32, true>(h, a, st) : launch_decompress_d<32, false>(h, a, st);
        case 64: return bf ? launch_decompress_d<64, true>(h, a, st) : launch_decompress_d<64, false>(h, a, st);
        case 128: return bf ? launch_decompress_d<128, true>(h, a, st) : launch_decompress_d<128, false>(h, a, st);
        default: break;
        }
    }
    int64_t want = (h->M + 255) / 256, cap = (int64_t)h->num_cu * 16;
    int grid = (int)(want < cap ? want : cap);
    if (bf)
        hipLaunchKernelGGL(decompress_generic_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(decompress_generic_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

int gvq_launch_aggregate(const gvq_basis* h, const float* const* comps, int N, float* out, hipStream_t st)
{
    const int64_t len = h->S * h->k;
    int64_t want = ((len >> 2) + 255) / 256, cap = (int64_t)h->num_cu * 8;
    int grid = (int)(want < cap ? want : cap);
    if (grid < 1) grid = 1;
    // out = comps[0] + ... in groups of at most GVQ_MAX_PTRS; later groups start from out
    int done = 0;
    while (done < N) {
        gvq_ptrs p;
        int n = 0;
        if (done > 0) p.p[n++] = out;
        while (n < GVQ_MAX_PTRS && done < N) p.p[n++] = comps[done++];
        hipLaunchKernelGGL(aggregate_kernel, dim3(grid), dim3(256), 0, st, p, n, out, len);
        GVQ_HIP(hipGetLastError());
    }
    return GVQ_OK;
}
