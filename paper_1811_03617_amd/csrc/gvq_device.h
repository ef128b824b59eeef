// Device-side helpers shared by the codec and monitor kernels (gfx950).
#pragma once
#include "gvq_internal.h"
#include <type_traits>

typedef float f4 __attribute__((ext_vector_type(4)));
typedef unsigned int u4 __attribute__((ext_vector_type(4)));
typedef unsigned int u2 __attribute__((ext_vector_type(2)));

#define WAVES_PER_WG 4
#define WG_THREADS (64 * WAVES_PER_WG)
#define TILE_SLICES 16
#ifndef GVQ_NONTEMPORAL
#define GVQ_NONTEMPORAL 1  // gradients are touched once: keep them out of the way of the caches
#endif

struct CodecArgs {
    const void* in;       // compress: gradient; decompress: compressed [S][k]
    void* out;            // compress: compressed [S][k]; decompress: gradient
    const float* U;       // [B][d][k]
    const f4* Upack;      // MFMA-operand order copy of U for this kernel, see pack_basis_kernel
    const f4* Upack2;     // local-loss kernel only: the decompress-order copy
    const float* Umu;     // bf16 compress kernel only: [B][16 NT] U^T mu
    const float* acc_in;  // compress only, may be null: [S][k] added to the result (ring step of Algorithm 1)
    int64_t seg_begin, seg_end;  // only the slices [seg_begin, seg_end) are produced
    const float* mu;      // [B][d]
    const int64_t* offs;  // [B+1] slice offsets of the bases
    int64_t M, S;
    int B, d, k;
    float n_workers;      // compress only
    const int* tile_block;  // [T] basis of the first slice of every 16-slice tile (B > 1 only)
    int run_tiles;        // tile schedule, see TileIter
    // Fast phase of the register-resident kernels: "super-tiles" of whole slices of ONE basis that lie
    // wholly inside the gradient and the requested range (2048 gradient elements each, i.e. 128/d
    // consecutive 16-slice tiles for fp32 input; 256/d for the bf16-pipe compress).  Everything else is a
    // "rest" tile and goes through the bounds-checked general phase.
    int64_t n_super;          // super-tiles (0 = no fast phase)
    int64_t sup_first;        // sup_tile == null: super-tile p starts at 16-slice tile sup_first + p * G
    const int64_t* sup_tile;  // many bases: [n_super] first 16-slice tile of every super-tile
    const int* sup_basis;     // many bases: [n_super] its basis
    int64_t rest_lo0, rest_lo1, rest_hi0, rest_hi1;   // rest_list == null: the rest tiles are [lo0, lo1) and [hi0, hi1)
    const int64_t* rest_list; // many bases: [n_rest] the rest tiles
    int64_t n_rest;
    int rest_run;             // rest tiles per run, see RestIter
    int il;                   // fast phase, one basis: il consecutive super-tiles interleave their 1 KB rows (row r of
                              // super-tile p of a group is row r il + p % il of the group's il times as many rows), so that
                              // consecutive waves, which take consecutive super-tiles, read and write one compact window of
                              // memory at any moment; 1 = none (a super-tile is 2048 consecutive elements).  Whole groups only.
    int keep_y;               // compress: the launcher picks the kernel whose fast phase writes the results with ordinary
                              // stores (they stay in the last-level cache for whoever reads them next) instead of
                              // non-temporal ones
    int pace;                 // fast phase: bit 0 = wait for all memory work before a super-tile is parked,
                              // bit 1 = also after its matrix products (fewer requests in flight per wave), bit 2 = the matrix
                              // products of a super-tile wait for the next one's loads one by one
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

// Two fp32 -> packed bf16 (round to nearest even) in one v_cvt_pk_bf16_f32; low half = a.
typedef __bf16 gvq_bf2 __attribute__((ext_vector_type(2)));
typedef float gvq_f2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ unsigned int pack_bf16x2(float a, float b)
{
    const gvq_f2 v = {a, b};
    return __builtin_bit_cast(unsigned int, __builtin_convertvector(v, gvq_bf2));
}

typedef __bf16 lbf8 __attribute__((ext_vector_type(8)));

// 8 floats -> their two bf16 terms, packed in operand order (element 2i in the low half of word i)
__device__ __forceinline__ void split8(const f4& v0, const f4& v1, u4& hi, u4& lo)
{
    float r[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const unsigned int h = pack_bf16x2(r[2 * i], r[2 * i + 1]);
        hi[i] = h;
        lo[i] = pack_bf16x2(r[2 * i] - __uint_as_float(h << 16), r[2 * i + 1] - __uint_as_float(h & 0xffff0000u));
    }
}

// Orders this wave's LDS traffic for the compiler: what one lane wrote is read by another
// lane of the same wave afterwards.  The hardware executes a wave's LDS instructions in
// order, so no s_barrier is needed; this only stops the compiler from moving LDS accesses
// across the exchange point.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

template <typename T>
__device__ __forceinline__ T stream_load(const T* p)
{
#if GVQ_NONTEMPORAL
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void stream_store(T* p, T v)
{
#if GVQ_NONTEMPORAL
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

// Which tiles a wave works on: runs of R consecutive 16-slice tiles, run r = w, w+W, w+2W, ...
// for wave w of W.  R = 1 interleaves single tiles, so that at any moment the whole chip
// reads one compact window of memory (what HBM likes best); a longer run keeps a wave inside
// one basis for longer when there are many bases; R = ceil(T/W) gives every wave one
// contiguous chunk.
struct TileIter {
    int64_t t, run, run_end, T0, T1, W;
    int R;
    // tiles [T0, T1)
    __device__ __forceinline__ bool init(int64_t T0_, int64_t T1_, int R_)
    {
        T0 = T0_; T1 = T1_; R = R_;
        W = (int64_t)gridDim.x * WAVES_PER_WG;
        run = (int64_t)blockIdx.x * WAVES_PER_WG + (threadIdx.x >> 6);
        t = T0 + run * R;
        run_end = t + R < T1 ? t + R : T1;
        return t < T1;
    }
    __device__ __forceinline__ bool advance()
    {
        if (++t < run_end) return true;
        run += W;
        t = T0 + run * R;
        run_end = t + R < T1 ? t + R : T1;
        return t < T1;
    }
};

// This wave's index in the grid and the number of waves, as scalars (wave-uniform values the
// compiler would otherwise keep in vector registers because they derive from threadIdx).
__device__ __forceinline__ int64_t grid_wave()
{
    return (int64_t)blockIdx.x * WAVES_PER_WG + __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
}
__device__ __forceinline__ int64_t grid_waves() { return (int64_t)gridDim.x * WAVES_PER_WG; }

// The super-tiles of one wave in the fast phase: runs of R consecutive ones, runs interleaved
// across the grid (see TileIter), all scalar.
struct SuperIter {
    int64_t p, run, run_end, N, W;
    int R;
    __device__ __forceinline__ bool init(int64_t N_, int R_)
    {
        N = N_; R = R_;
        W = grid_waves();
        run = grid_wave();
        p = run * R;
        run_end = p + R < N ? p + R : N;
        return p < N;
    }
    __device__ __forceinline__ bool advance()
    {
        if (++p < run_end) return true;
        run += W;
        p = run * R;
        run_end = p + R < N ? p + R : N;
        return p < N;
    }
};

// The rest tiles of one wave (general phase): runs of R consecutive items, runs interleaved across the
// grid, counted from the far end so that the waves with the fewest super-tiles take them first.
struct RestIter {
    int64_t t, i, run, run_end, n, W, lo0, nlo, hi0;
    int R;
    const int64_t* list;
    __device__ __forceinline__ int64_t tile_of(int64_t j) const
    {
        if (list) return list[j];
        return j < nlo ? lo0 + j : hi0 + (j - nlo);
    }
    __device__ __forceinline__ bool init(const CodecArgs& a)
    {
        list = a.rest_list;
        lo0 = a.rest_lo0; nlo = a.rest_lo1 - a.rest_lo0; hi0 = a.rest_hi0;
        n = list ? a.n_rest : nlo + (a.rest_hi1 - a.rest_hi0);
        R = a.rest_run;
        W = grid_waves();
        run = W - 1 - grid_wave();
        i = run * R;
        run_end = i + R < n ? i + R : n;
        if (i >= n) return false;
        t = tile_of(i);
        return true;
    }
    __device__ __forceinline__ bool advance()
    {
        if (++i >= run_end) {
            run += W;
            i = run * R;
            run_end = i + R < n ? i + R : n;
            if (i >= n) return false;
        }
        t = tile_of(i);
        return true;
    }
};

// Load through the scalar cache: the address must be the same for the whole wave and the memory must
// not change while the kernel runs (tables the host wrote before the launch).  Scalar loads count on
// their own counter, so they do not disturb the bookkeeping of the vector loads and stores around them.
template <typename T>
__device__ __forceinline__ T uniform_load(const T* p)
{
    typedef const T __attribute__((address_space(4))) CT;
    return *(CT*)(uintptr_t)p;
}

// Compile-time loop: f(integral_constant<int, I>) for I = 0 .. N-1.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// At most N of this wave's vector-memory requests are still outstanding (they complete in order).
template <int N>
__device__ __forceinline__ void wait_vmem_at_most()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));   // expcnt, lgkmcnt untouched
}

// Everything this wave asked of memory has arrived (loads) or been accepted (stores); also tells the
// compiler's wait-count bookkeeping so, which keeps a loop that follows free of inherited waits.
__device__ __forceinline__ void drain_memory()
{
    __builtin_amdgcn_s_waitcnt(0x0070);   // vmcnt(0) lgkmcnt(0), expcnt untouched
}

// Ring step of Algorithm 1: the partial sum that arrived from the predecessor, in the register
// layout of a result tile (lane (n, kk) holds comps 16 nt + 4 kk + r of slice j); zero where
// there is nothing to add.
template <int NT>
__device__ __forceinline__ void load_acc_in(const CodecArgs& a, int64_t j, int kk, bool row_ok, f4 (&v)[NT])
{
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        v[nt] = f4{0.f, 0.f, 0.f, 0.f};
        if (a.acc_in && row_ok) {
            const int c0 = 16 * nt + 4 * kk;
            const float* p = a.acc_in + j * a.k + c0;
            if ((a.k & 3) == 0) {
                if (c0 < a.k) v[nt] = *(const f4*)p;
            } else {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (c0 + r < a.k) v[nt][r] = p[r];
            }
        }
    }
}

// Rows of the tile [s0, s1) that belong to the current basis and to the requested range.
__device__ __forceinline__ void row_range(const CodecArgs& a, int64_t s0, int64_t s1, int64_t blk_begin,
                                          int64_t blk_end, int64_t& lo, int64_t& hi)
{
    lo = s0 > blk_begin ? s0 : blk_begin;
    hi = s1 < blk_end ? s1 : blk_end;
    if (lo < a.seg_begin) lo = a.seg_begin;
    if (hi > a.seg_end) hi = a.seg_end;
}

__device__ __forceinline__ int block_of_tile(const CodecArgs& a, int64_t t)
{
    return a.B > 1 ? a.tile_block[t] : 0;
}

// XOR swizzle of the 128-bit LDS slots of a 16-row tile with D/4 slots per row: slot
// s*CPS + (c ^ swz(s)) keeps 8 consecutive lanes on 8 distinct 128-bit bank groups both for
// row-major (memory order) and for column-major (one row per lane) accesses.
template <int D>
__device__ __forceinline__ int swz(int s)
{
    return (D >= 32) ? (s & 7) : ((s >> 1) & 3);
}

