// Codec kernels for long slices, 128 < d <= GVQ_MAX_D and k <= 128 (GradiVeQ Eqs. 2 and 4 with
// the slice sizes of Section 3, e.g. d = 768), also used for every shorter shape that the
// register-resident kernels do not take (d not in {16,32,64,128}, or k > 32).  U (d x k floats, up
// to 512 KB) does not fit a wave's registers, so these are LDS-tiled contractions on the matrix
// pipes (first the exact fp32 products on v_mfma_f32_16x16x4_f32, further down the bf16 split):
//   a work-group of 4 waves owns LW_SLICES = 128 consecutive slices of one basis, 32 per wave
//   (two 16-slice MFMA column tiles);  U is streamed through LDS in chunks of LC = 64 elements,
//   double-buffered, one s_barrier per chunk, shared by the 4 waves;  the gradient side goes
//   straight between global memory and registers in MFMA operand order (lane (n, kk) moves 4
//   consecutive elements of slice n with one 128-bit access).
// Tiles never straddle two bases: the tiles of basis b are tstart[b] .. tstart[b+1]-1.
#include "gvq_device.h"

#define LW_SLICES 128
#define LC 64
// first element (inside a chunk) of word i of lane group kk in the compress kernels
#define LWORD(i, kk) (32 * ((i) >> 1) + 16 * ((i) & 1) + 4 * (kk))

struct LongArgs {
    const void* in;
    void* out;
    const float* acc_in;     // compress only, may be null
    const f4* Upack;         // [B][nchunk][4][NT][64] f4 in the kernel's operand order
    const f4* Upack2;        // loss kernel only: the decompress-order copy
    const float* mu;         // [B][d]
    const int64_t* offs;     // [B+1]
    const int64_t* tstart;   // [B+1] first tile of each basis (B > 1 only)
    int64_t M, S, seg_begin, seg_end, t0, t1;
    int B, d, k, nchunk;     // k: the comps of THIS column pass (at most 128)
    int kfull, c0;           // row length of the compressed vector, first comp of this pass (k > 128: several passes)
    int accum;               // decompress: add to what grad_out holds (passes after the first; fp32 output only)
    int upack_stride;        // packed-U words (f4 / u4) from one basis to the next
    float n_workers;
};

__device__ __forceinline__ void long_tile(const LongArgs& a, int64_t tile, int& b, int64_t& first, int64_t& end)
{
    if (a.B == 1) {
        b = 0;
        first = tile * LW_SLICES;
        end = first + LW_SLICES < a.S ? first + LW_SLICES : a.S;
        return;
    }
    int lo = 0, hi = a.B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.tstart[mid] <= tile) lo = mid; else hi = mid;
    }
    b = lo;
    first = a.offs[b] + (tile - a.tstart[b]) * LW_SLICES;
    end = first + LW_SLICES < a.offs[b + 1] ? first + LW_SLICES : a.offs[b + 1];
}

// 4 consecutive gradient elements starting at element e of slice s, zero where the slice or the
// gradient ends (the zero padding of the last slice).  FAST: the caller guarantees that d is a
// multiple of 4 and that every slice of the tile lies wholly inside the gradient; the load is
// then unconditional from `row` (the start of the lane's slice, or of the tile's last slice for
// lanes past its end, whose results are dropped), which keeps the number of loads in flight
// known to the compiler, so that it waits for the words it needs and not for the requests
// behind them.
template <bool BF16, bool FAST>
__device__ __forceinline__ f4 load_x4(const LongArgs& a, bool row_ok, int64_t s, const void* row, int e)
{
    f4 v = {0.f, 0.f, 0.f, 0.f};
    if (FAST) {
        const bool inside = e < a.d;            // past the slice (last chunk, d not a multiple of 64):
        const int ec = inside ? e : a.d - 4;    // read its last word instead and drop the value
        if (BF16) {
            const u2 w = *(const u2*)((const unsigned short*)row + ec);
            v[0] = __uint_as_float(w.x << 16);
            v[1] = __uint_as_float(w.x & 0xffff0000u);
            v[2] = __uint_as_float(w.y << 16);
            v[3] = __uint_as_float(w.y & 0xffff0000u);
        } else {
            v = *(const f4*)((const float*)row + ec);
        }
#pragma unroll
        for (int r = 0; r < 4; ++r) v[r] = inside ? v[r] : 0.f;
        return v;
    }
    if (!row_ok || e >= a.d) return v;
    const int64_t idx = s * a.d + e;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (e + r < a.d && idx + r < a.M)
            v[r] = BF16 ? bf16_to_f32(((const unsigned short*)a.in)[idx + r]) : ((const float*)a.in)[idx + r];
    return v;
}

// Comps c0 .. c0+3 of slice s of the compressed output (plus the ring step's partial sum when
// there is one); nothing past comp k.
__device__ __forceinline__ void store_y4(const LongArgs& a, int64_t s, int c0, f4 v)
{
    if (c0 >= a.k) return;
    float* Y = (float*)a.out;
    const int64_t o = s * a.kfull + a.c0 + c0;
    if ((a.kfull & 3) == 0) {
        if (a.acc_in) v += *(const f4*)(a.acc_in + o);
        *(f4*)(Y + o) = v;
    } else {
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (c0 + r < a.k) Y[o + r] = a.acc_in ? v[r] + a.acc_in[o + r] : v[r];
    }
}

// Elements e0 .. e0+3 of slice s of the reconstructed gradient; `vec`: the whole tile lies inside
// the gradient and d is a multiple of 4, so the word is stored whole.
template <bool OUT_BF16>
__device__ __forceinline__ void store_x4(const LongArgs& a, bool vec, int64_t s, int e0, f4 v)
{
    const int64_t idx = s * a.d + e0;
    if (!OUT_BF16 && a.accum) {   // a later column pass: add to the earlier passes' sum
        if (vec) {
            f4* o = (f4*)((float*)a.out + idx);
            *o = *o + v;
        } else {
#pragma unroll
            for (int r = 0; r < 4; ++r)
                if (e0 + r < a.d && idx + r < a.M) ((float*)a.out)[idx + r] += v[r];
        }
        return;
    }
    if (vec) {
        if (OUT_BF16) {
            u2 w2;
            w2.x = pack_bf16x2(v[0], v[1]);
            w2.y = pack_bf16x2(v[2], v[3]);
            *(u2*)((unsigned short*)a.out + idx) = w2;
        } else {
            *(f4*)((float*)a.out + idx) = v;
        }
        return;
    }
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (e0 + r < a.d && idx + r < a.M) {
            if (OUT_BF16) ((unsigned short*)a.out)[idx + r] = (unsigned short)f32_to_bf16_rne(v[r]);
            else ((float*)a.out)[idx + r] = v[r];
        }
}

// --------------------------------------------------------------------------------------
// compress: D[comp][slice] += U[elem][comp] x[slice][elem].  For chunk c, word i (0..3) and
// step j (0..3), lane (m, kk) of the A operand holds U[64c + w(i, kk) + j][16nt + m] and lane
// (n, kk) of the B operand x[slice n][64c + w(i, kk) + j] - mu/N with w(i, kk) = 32(i/2) + 16(i%2)
// + 4kk: one 128-bit word of x feeds four steps, and the four lanes of a slice read 64 contiguous
// bytes per load instruction (the order of the contraction is free).  Result register r of
// lane (n, kk) is comp 16nt + 4kk + r of slice n.
// Upack[b][c][i][nt][lane] = the four U values (j = 0..3) of that lane, zero past d and k.
// --------------------------------------------------------------------------------------
template <int NT, bool BF16, bool FAST, bool LOSS>
__device__ __forceinline__ void compress_long_tile(const LongArgs& a, f4* Us, const float* mus, const f4* Ub,
                                                   const f4* Ub2, int64_t first, int64_t end, int64_t lo, int64_t hi)
{
    constexpr int CH4 = 4 * NT * 64;              // 128-bit words of one U chunk
    constexpr int G = NT <= 4 ? NT : (NT == 6 ? 3 : 4);   // comp tiles per group of MFMAs
    constexpr int NG = NT / G, STEPS = 4 * NG;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_ = lane & 15, kk = lane >> 4;

    int64_t s[2];
    const void* sc[2];
    bool ok[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        s[t] = first + wave * 32 + 16 * t + n_;
        ok[t] = s[t] >= lo && s[t] < hi;
        const int64_t row = (s[t] < end ? s[t] : end - 1) * a.d;
        sc[t] = BF16 ? (const void*)((const unsigned short*)a.in + row) : (const void*)((const float*)a.in + row);
    }
    f4 acc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[t][nt] = f4{0.f, 0.f, 0.f, 0.f};
    // a word of x is requested again, for the next chunk, as soon as the MFMAs of its last use
    // are issued, so the load has most of a chunk's MFMA time to arrive.  All requests are
    // unconditional (in the last chunk the same words are simply fetched again).
    const int last = a.nchunk - 1;
    f4 xr[2][4], ur[NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int i = 0; i < 4; ++i) xr[t][i] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], LWORD(i, kk));

    for (int c = 0; c < a.nchunk; ++c) {
        const int cn = c < last ? c + 1 : last;
#pragma unroll
        for (int q = 0; q < NT; ++q) ur[q] = Ub[(size_t)cn * CH4 + tid + 256 * q];
        const f4* Uc = Us + (c & 1) * CH4;
        const float* mc = mus + c * LC;
        // MFMA steps (i, g): the LDS operands of step st + 1 are requested before the MFMAs of
        // step st are issued; inside a step the accumulators are innermost, 2 G independent
        // chains between two uses of one
        f4 uw[2][G], mw[2];
#pragma unroll
        for (int q = 0; q < G; ++q) uw[0][q] = Uc[q * 64 + lane];
        mw[0] = *(const f4*)(mc + LWORD(0, kk));
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            const int i = st / NG, g = st % NG;
            if (st + 1 < STEPS) {
                const int i1 = (st + 1) / NG, g1 = (st + 1) % NG;
#pragma unroll
                for (int q = 0; q < G; ++q) uw[(st + 1) & 1][q] = Uc[(i1 * NT + g1 * G + q) * 64 + lane];
                if (g1 == 0) mw[i1 & 1] = *(const f4*)(mc + LWORD(i1, kk));
            }
            const f4 x0 = xr[0][i] - mw[i & 1], x1 = xr[1][i] - mw[i & 1];
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int q = 0; q < G; ++q) {
                    const int nt = g * G + q;
                    acc[0][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[st & 1][q][j], x0[j], acc[0][nt], 0, 0, 0);
                    acc[1][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[st & 1][q][j], x1[j], acc[1][nt], 0, 0, 0);
                }
            if (g == NG - 1) {   // word i is used up
#pragma unroll
                for (int t = 0; t < 2; ++t)
                    xr[t][i] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], cn * LC + LWORD(i, kk));
            }
        }
        __builtin_amdgcn_s_setprio(0);
        if (c < last) {
            f4* Un = Us + ((c + 1) & 1) * CH4;   // last read one chunk ago, before the previous barrier
#pragma unroll
            for (int q = 0; q < NT; ++q) Un[tid + 256 * q] = ur[q];
            __syncthreads();
        }
    }

    if constexpr (LOSS) {
        // Eq. (6): the residual (x - mu/N) - U y of the same tile.  The accumulators already are
        // the B operand of the reconstruction product (lane (n, kk) holds comps 16w + 4kk + j of
        // slice n), and the product's result registers cover the same elements as the x words
        // of the projection (element tile et <-> word i), so x is simply read once more, chunk by
        // chunk, and nothing but the squared sum leaves the registers.
        __syncthreads();   // every wave is done with the projection's last U chunk
#pragma unroll
        for (int q = 0; q < NT; ++q) Us[tid + 256 * q] = Ub2[tid + 256 * q];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int i = 0; i < 4; ++i) xr[t][i] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], 16 * i + 4 * kk);
        __syncthreads();
        float sq[2] = {0.f, 0.f};
        for (int c = 0; c < a.nchunk; ++c) {
            const int cn = c < last ? c + 1 : last;
#pragma unroll
            for (int q = 0; q < NT; ++q) ur[q] = Ub2[(size_t)cn * CH4 + tid + 256 * q];
            const f4* Uc = Us + (c & 1) * CH4;
            f4 rec[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int et = 0; et < 4; ++et) rec[t][et] = f4{0.f, 0.f, 0.f, 0.f};
            f4 uw[2][4];
#pragma unroll
            for (int et = 0; et < 4; ++et) uw[0][et] = Uc[(et * NT) * 64 + lane];
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int w = 0; w < NT; ++w) {
                if (w + 1 < NT) {
#pragma unroll
                    for (int et = 0; et < 4; ++et) uw[(w + 1) & 1][et] = Uc[(et * NT + w + 1) * 64 + lane];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int et = 0; et < 4; ++et) {
                        rec[0][et] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[w & 1][et][j], acc[0][w][j], rec[0][et], 0, 0, 0);
                        rec[1][et] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[w & 1][et][j], acc[1][w][j], rec[1][et], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_s_setprio(0);
#pragma unroll
            for (int et = 0; et < 4; ++et) {
                const int e0 = c * LC + 16 * et + 4 * kk;
                const f4 mw = *(const f4*)(mus + e0);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const f4 res = (xr[t][et] - mw) - rec[t][et];
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // only elements that exist count (not the zero padding of the last slice)
                        const bool real = FAST ? e0 < a.d : (e0 + r < a.d && s[t] * a.d + e0 + r < a.M);
                        if (real) sq[t] = fmaf(res[r], res[r], sq[t]);
                    }
                    xr[t][et] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], cn * LC + 16 * et + 4 * kk);
                }
            }
            if (c < last) {
                f4* Un = Us + ((c + 1) & 1) * CH4;
#pragma unroll
                for (int q = 0; q < NT; ++q) Un[tid + 256 * q] = ur[q];
                __syncthreads();
            }
        }
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            float v = sq[t];
            v += __shfl_xor(v, 16, 64);
            v += __shfl_xor(v, 32, 64);
            if (kk == 0 && ok[t]) ((float*)a.out)[s[t]] = v;
        }
        return;
    }
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (!ok[t]) continue;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) store_y4(a, s[t], 16 * nt + 4 * kk, acc[t][nt]);
    }
}

template <int NT, bool BF16, bool LOSS>
__global__ __launch_bounds__(256, 2) void compress_long_kernel(LongArgs a)
{
    extern __shared__ f4 smem[];
    constexpr int CH4 = 4 * NT * 64;
    f4* Us = smem;                                // [2][CH4]
    float* mus = (float*)(smem + 2 * CH4);        // [nchunk * LC]  mu / N, zero past d
    const int tid = threadIdx.x;

    for (int64_t tile = a.t0 + blockIdx.x; tile < a.t1; tile += gridDim.x) {
        int b;
        int64_t first, end;
        long_tile(a, tile, b, first, end);
        const int64_t lo = first > a.seg_begin ? first : a.seg_begin, hi = end < a.seg_end ? end : a.seg_end;
        const f4* Ub = a.Upack + (size_t)b * a.upack_stride;
        __syncthreads();   // the previous tile's readers are done with mus and Us
        for (int e = tid; e < a.nchunk * LC; e += 256)
            mus[e] = e < a.d ? a.mu[(size_t)b * a.d + e] / a.n_workers : 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) Us[tid + 256 * q] = Ub[tid + 256 * q];
        __syncthreads();
        const f4* Ub2 = LOSS ? a.Upack2 + (size_t)b * a.upack_stride : nullptr;
        if ((a.d & 3) == 0 && end * a.d <= a.M)
            compress_long_tile<NT, BF16, true, LOSS>(a, Us, mus, Ub, Ub2, first, end, lo, hi);
        else
            compress_long_tile<NT, BF16, false, LOSS>(a, Us, mus, Ub, Ub2, first, end, lo, hi);
    }
}

// --------------------------------------------------------------------------------------
// decompress: D[elem][slice] = sum_comp U[elem][comp] Y[slice][comp], then + mu.  The wave keeps
// its 32 slices of Y in registers (lane (n, kk) holds comps 16w + 4kk + j, w < NT) and walks
// over the element chunks; for element tile et (0..3) of chunk c and comp group w, lane (m, kk)
// of the A operand holds U[64c + 16et + m][16w + 4kk + j].  Result register r of lane (n, kk) is
// element 64c + 16et + 4kk + r of slice n: one 128-bit store.
// Upack[b][c][et][w][lane] = the four U values (j = 0..3) of that lane, zero past d and k.
// --------------------------------------------------------------------------------------
template <int NT, bool OUT_BF16>
__global__ __launch_bounds__(256, 2) void decompress_long_kernel(LongArgs a)
{
    extern __shared__ f4 smem[];
    constexpr int CH4 = 4 * NT * 64;
    f4* Us = smem;
    float* mus = (float*)(smem + 2 * CH4);        // [nchunk * LC]  mu, zero past d
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_ = lane & 15, kk = lane >> 4;
    const float* Y = (const float*)a.in;

    for (int64_t tile = a.t0 + blockIdx.x; tile < a.t1; tile += gridDim.x) {
        int b;
        int64_t first, end;
        long_tile(a, tile, b, first, end);
        const int64_t lo = first > a.seg_begin ? first : a.seg_begin, hi = end < a.seg_end ? end : a.seg_end;
        const f4* Ub = a.Upack + (size_t)b * a.upack_stride;
        __syncthreads();
        for (int e = tid; e < a.nchunk * LC; e += 256) mus[e] = (e < a.d && !a.accum) ? a.mu[(size_t)b * a.d + e] : 0.f;
        f4 ur[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) Us[tid + 256 * q] = Ub[tid + 256 * q];
        __syncthreads();

        int64_t s[2];
        bool ok[2];
        f4 yr[2][NT];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            s[t] = first + wave * 32 + 16 * t + n_;
            ok[t] = s[t] >= lo && s[t] < hi;
#pragma unroll
            for (int w = 0; w < NT; ++w) {
                yr[t][w] = f4{0.f, 0.f, 0.f, 0.f};
                const int c0 = 16 * w + 4 * kk;
                if (!ok[t] || c0 >= a.k) continue;
                const float* p = Y + s[t] * a.kfull + a.c0 + c0;
                if ((a.kfull & 3) == 0) {
                    yr[t][w] = *(const f4*)p;
                } else {
#pragma unroll
                    for (int r = 0; r < 4; ++r)
                        if (c0 + r < a.k) yr[t][w][r] = p[r];
                }
            }
        }
        const bool vec = (a.d & 3) == 0 && end * a.d <= a.M;   // every store of the tile is a whole word

        for (int c = 0; c < a.nchunk; ++c) {
            const int cn = c + 1 < a.nchunk ? c + 1 : c;   // unconditional: the last chunk is fetched twice
#pragma unroll
            for (int q = 0; q < NT; ++q) ur[q] = Ub[(size_t)cn * CH4 + tid + 256 * q];
            const f4* Uc = Us + (c & 1) * CH4;
            f4 acc[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int et = 0; et < 4; ++et) acc[t][et] = f4{0.f, 0.f, 0.f, 0.f};
            // comp group w + 1's operands are requested before the MFMAs of group w; the 8
            // accumulators are innermost
            f4 uw[2][4];
#pragma unroll
            for (int et = 0; et < 4; ++et) uw[0][et] = Uc[(et * NT) * 64 + lane];
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int w = 0; w < NT; ++w) {
                if (w + 1 < NT) {
#pragma unroll
                    for (int et = 0; et < 4; ++et) uw[(w + 1) & 1][et] = Uc[(et * NT + w + 1) * 64 + lane];
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int et = 0; et < 4; ++et) {
                        acc[0][et] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[w & 1][et][j], yr[0][w][j], acc[0][et], 0, 0, 0);
                        acc[1][et] = __builtin_amdgcn_mfma_f32_16x16x4f32(uw[w & 1][et][j], yr[1][w][j], acc[1][et], 0, 0, 0);
                    }
            }
            __builtin_amdgcn_s_setprio(0);
            // the next U chunk goes to LDS before this chunk's stores are issued, so that waiting
            // for its loads does not wait for the stores
            if (c + 1 < a.nchunk) {
                f4* Un = Us + ((c + 1) & 1) * CH4;
#pragma unroll
                for (int q = 0; q < NT; ++q) Un[tid + 256 * q] = ur[q];
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (!ok[t]) continue;
#pragma unroll
                for (int et = 0; et < 4; ++et) {
                    const int e0 = c * LC + 16 * et + 4 * kk;
                    if (e0 >= a.d) continue;
                    store_x4<OUT_BF16>(a, vec, s[t], e0, acc[t][et] + *(const f4*)(mus + e0));
                }
            }
            if (c + 1 < a.nchunk) __syncthreads();
        }
    }
}

// ======================================================================================
// The same two contractions on the bf16 matrix pipe, for shapes whose 2dk flop per slice would
// keep the fp32 pipe busy for longer than HBM needs for the slice's bytes (d = 768, k = 96: 43
// flop per byte).  Every fp32 number is split into two bf16 terms, a = a1 + a2 with
// a1 = bf16(a), a2 = bf16(a - a1) (round to nearest even; |a - a1 - a2| <= 2^-18 |a|), and a
// product x u is taken as x1 u1 + x1 u2 + x2 u1 on v_mfma_f32_16x16x32_bf16 with fp32
// accumulation: the three dropped terms are each below 2^-18 |x u|, i.e. a product is good to
// about 1e-5 of its magnitude, an order of magnitude inside the codec's 1e-4 tolerance.  One
// MFMA contracts 32 elements, so the matrix work falls to about a seventh and the kernels are
// bound by memory again.  U is split once per basis (pack_long_split_kernel), x (after x - mu/N)
// and Y in registers.  Tiling, U streaming through LDS and tile ownership are as above; NT is
// even here (an MFMA step of decompress contracts 32 comps).
//   compress:   chunk c, step st (0,1): A lane (m, kk) = U[64c + 32st + r(kk, j)][16nt + m], j = 0..7,
//               B lane (n, kk) = x[slice n][64c + 32st + r(kk, j)], r(kk, j) = 16(j/4) + 4kk + j%4: the
//               contraction order is free, and this one makes the four lanes of a slice read 64
//               contiguous bytes per load instruction;
//               Upack[b][c][st][p][nt][lane] = 8 bf16 of term p;
//   decompress: chunk c, element tile et, comp step ks: A lane (m, kk) = U[64c + 16et + m][32ks + r(kk, j)],
//               B lane (n, kk) = Y[slice n][32ks + r(kk, j)];  Upack[b][c][et][ks][p][lane].
// ======================================================================================
template <int NT, bool BF16, bool FAST>
__device__ __forceinline__ void compress_split_tile(const LongArgs& a, u4* Us, const float* mus, const u4* Ub,
                                                    int64_t first, int64_t end, int64_t lo, int64_t hi)
{
    constexpr int CH4 = 4 * NT * 64;   // 128-bit words of one U chunk: [st 2][p 2][NT][64]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_ = lane & 15, kk = lane >> 4;

    int64_t s[2];
    const void* sc[2];
    bool ok[2];
#pragma unroll
    for (int t = 0; t < 2; ++t) {
        s[t] = first + wave * 32 + 16 * t + n_;
        ok[t] = s[t] >= lo && s[t] < hi;
        const int64_t row = (s[t] < end ? s[t] : end - 1) * a.d;
        sc[t] = BF16 ? (const void*)((const unsigned short*)a.in + row) : (const void*)((const float*)a.in + row);
    }
    f4 acc[2][NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[t][nt] = f4{0.f, 0.f, 0.f, 0.f};
    const int last = a.nchunk - 1;
    // raw x of the next chunk: word (st, h) of tile t = elements 32st + 16h + 4kk .. +3
    f4 xr[2][2][2];
    u4 ur[NT];
#pragma unroll
    for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                xr[t][st][h] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], 32 * st + 16 * h + 4 * kk);

    for (int c = 0; c < a.nchunk; ++c) {
        const int cn = c < last ? c + 1 : last;
#pragma unroll
        for (int q = 0; q < NT; ++q) ur[q] = Ub[(size_t)cn * CH4 + tid + 256 * q];
        // centre and split this chunk's x, then ask for the next chunk's (unconditionally)
        u4 xh[2][2], xl[2][2];
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const float* mc = mus + c * LC + 32 * st + 4 * kk;
            const f4 m0 = *(const f4*)mc, m1 = *(const f4*)(mc + 16);
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                split8(xr[t][st][0] - m0, xr[t][st][1] - m1, xh[t][st], xl[t][st]);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    xr[t][st][h] = load_x4<BF16, FAST>(a, ok[t], s[t], sc[t], cn * LC + 32 * st + 16 * h + 4 * kk);
            }
        }
        const u4* Uc = Us + (c & 1) * CH4;
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int st = 0; st < 2; ++st)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const lbf8 u1 = __builtin_bit_cast(lbf8, Uc[((st * 2 + 0) * NT + nt) * 64 + lane]);
                const lbf8 u2 = __builtin_bit_cast(lbf8, Uc[((st * 2 + 1) * NT + nt) * 64 + lane]);
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const lbf8 bh = __builtin_bit_cast(lbf8, xh[t][st]), bl = __builtin_bit_cast(lbf8, xl[t][st]);
                    acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u1, bl, acc[t][nt], 0, 0, 0);
                    acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u2, bh, acc[t][nt], 0, 0, 0);
                    acc[t][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u1, bh, acc[t][nt], 0, 0, 0);
                }
            }
        __builtin_amdgcn_s_setprio(0);
        if (c < last) {
            u4* Un = Us + ((c + 1) & 1) * CH4;
#pragma unroll
            for (int q = 0; q < NT; ++q) Un[tid + 256 * q] = ur[q];
            __syncthreads();
        }
    }

#pragma unroll
    for (int t = 0; t < 2; ++t) {
        if (!ok[t]) continue;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) store_y4(a, s[t], 16 * nt + 4 * kk, acc[t][nt]);
    }
}

template <int NT, bool BF16>
__global__ __launch_bounds__(256, 2) void compress_split_kernel(LongArgs a)
{
    extern __shared__ f4 smem[];
    constexpr int CH4 = 4 * NT * 64;
    u4* Us = (u4*)smem;                           // [2][CH4]
    float* mus = (float*)(smem + 2 * CH4);        // [nchunk * LC]  mu / N, zero past d
    const int tid = threadIdx.x;
    for (int64_t tile = a.t0 + blockIdx.x; tile < a.t1; tile += gridDim.x) {
        int b;
        int64_t first, end;
        long_tile(a, tile, b, first, end);
        const int64_t lo = first > a.seg_begin ? first : a.seg_begin, hi = end < a.seg_end ? end : a.seg_end;
        const u4* Ub = (const u4*)a.Upack + (size_t)b * a.upack_stride;
        __syncthreads();
        for (int e = tid; e < a.nchunk * LC; e += 256)
            mus[e] = e < a.d ? a.mu[(size_t)b * a.d + e] / a.n_workers : 0.f;
#pragma unroll
        for (int q = 0; q < NT; ++q) Us[tid + 256 * q] = Ub[tid + 256 * q];
        __syncthreads();
        if ((a.d & 3) == 0 && end * a.d <= a.M)
            compress_split_tile<NT, BF16, true>(a, Us, mus, Ub, first, end, lo, hi);
        else
            compress_split_tile<NT, BF16, false>(a, Us, mus, Ub, first, end, lo, hi);
    }
}

template <int NT, bool OUT_BF16>
__global__ __launch_bounds__(256, 2) void decompress_split_kernel(LongArgs a)
{
    extern __shared__ f4 smem[];
    constexpr int CH4 = 4 * NT * 64;              // [et 4][ks NT/2][p 2][64]
    constexpr int NKS = NT / 2;
    u4* Us = (u4*)smem;
    float* mus = (float*)(smem + 2 * CH4);        // [nchunk * LC]  mu, zero past d
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, n_ = lane & 15, kk = lane >> 4;
    const float* Y = (const float*)a.in;

    for (int64_t tile = a.t0 + blockIdx.x; tile < a.t1; tile += gridDim.x) {
        int b;
        int64_t first, end;
        long_tile(a, tile, b, first, end);
        const int64_t lo = first > a.seg_begin ? first : a.seg_begin, hi = end < a.seg_end ? end : a.seg_end;
        const u4* Ub = (const u4*)a.Upack + (size_t)b * a.upack_stride;
        __syncthreads();
        for (int e = tid; e < a.nchunk * LC; e += 256) mus[e] = (e < a.d && !a.accum) ? a.mu[(size_t)b * a.d + e] : 0.f;
        u4 ur[NT];
#pragma unroll
        for (int q = 0; q < NT; ++q) Us[tid + 256 * q] = Ub[tid + 256 * q];
        __syncthreads();

        int64_t s[2];
        bool ok[2];
        u4 yh[2][NKS], yl[2][NKS];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            s[t] = first + wave * 32 + 16 * t + n_;
            ok[t] = s[t] >= lo && s[t] < hi;
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks) {
                f4 v[2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    v[h] = f4{0.f, 0.f, 0.f, 0.f};
                    const int c0 = 32 * ks + 16 * h + 4 * kk;
                    if (!ok[t] || c0 >= a.k) continue;
                    const float* p = Y + s[t] * a.kfull + a.c0 + c0;
                    if ((a.kfull & 3) == 0) {
                        v[h] = *(const f4*)p;
                    } else {
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (c0 + r < a.k) v[h][r] = p[r];
                    }
                }
                split8(v[0], v[1], yh[t][ks], yl[t][ks]);
            }
        }
        const bool vec = (a.d & 3) == 0 && end * a.d <= a.M;

        for (int c = 0; c < a.nchunk; ++c) {
            const int cn = c + 1 < a.nchunk ? c + 1 : c;
#pragma unroll
            for (int q = 0; q < NT; ++q) ur[q] = Ub[(size_t)cn * CH4 + tid + 256 * q];
            const u4* Uc = Us + (c & 1) * CH4;
            f4 acc[2][4];
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int et = 0; et < 4; ++et) acc[t][et] = f4{0.f, 0.f, 0.f, 0.f};
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
                for (int et = 0; et < 4; ++et) {
                    const lbf8 u1 = __builtin_bit_cast(lbf8, Uc[((et * NKS + ks) * 2 + 0) * 64 + lane]);
                    const lbf8 u2 = __builtin_bit_cast(lbf8, Uc[((et * NKS + ks) * 2 + 1) * 64 + lane]);
#pragma unroll
                    for (int t = 0; t < 2; ++t) {
                        const lbf8 bh = __builtin_bit_cast(lbf8, yh[t][ks]), bl = __builtin_bit_cast(lbf8, yl[t][ks]);
                        acc[t][et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u1, bl, acc[t][et], 0, 0, 0);
                        acc[t][et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u2, bh, acc[t][et], 0, 0, 0);
                        acc[t][et] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(u1, bh, acc[t][et], 0, 0, 0);
                    }
                }
            __builtin_amdgcn_s_setprio(0);
            if (c + 1 < a.nchunk) {
                u4* Un = Us + ((c + 1) & 1) * CH4;
#pragma unroll
                for (int q = 0; q < NT; ++q) Un[tid + 256 * q] = ur[q];
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                if (!ok[t]) continue;
#pragma unroll
                for (int et = 0; et < 4; ++et) {
                    const int e0 = c * LC + 16 * et + 4 * kk;
                    if (e0 >= a.d) continue;
                    store_x4<OUT_BF16>(a, vec, s[t], e0, acc[t][et] + *(const f4*)(mus + e0));
                }
            }
            if (c + 1 < a.nchunk) __syncthreads();
        }
    }
}

// The two-term bf16 copies of U for the split kernels, 8 values per 128-bit word in operand order
// (layouts above); term 0 = bf16(U), term 1 = bf16(U - term 0); zero where e >= d or comp >= k.
__global__ void pack_long_split_kernel(const float* U, unsigned short* Upc, unsigned short* Upd, int d, int k, int NT,
                                       int nchunk, int c0, int npass, int pass)
{
    const int b = blockIdx.y, NKS = NT / 2;
    const float* Ub = U + (size_t)b * d * k + c0;          // this column pass starts at comp c0
    const size_t per = (size_t)nchunk * 4 * NT * 64 * 8;   // bf16 values per basis and pass in either copy
    Upc += ((size_t)b * npass + pass) * per - (size_t)b * per;
    Upd += ((size_t)b * npass + pass) * per - (size_t)b * per;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < per; i += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(i & 7), lane = (int)((i >> 3) & 63), m = lane & 15, kk = lane >> 4;
        const size_t word = i >> 9;                         // index of the 64-lane word group
        const int c = (int)(word / (4 * NT)), w = (int)(word % (4 * NT));
        auto term = [&](int e, int comp, int p) -> unsigned short {
            if (e >= d || c0 + comp >= k) return 0;
            const float u = Ub[(size_t)e * k + comp];
            const unsigned int t0 = f32_to_bf16_rne(u);
            if (p == 0) return (unsigned short)t0;
            return (unsigned short)f32_to_bf16_rne(u - bf16_to_f32(t0));
        };
        {   // compress: w = (st * 2 + p) * NT + nt
            const int nt = w % NT, p = (w / NT) & 1, st = w / (2 * NT);
            Upc[(size_t)b * per + i] = term(c * LC + 32 * st + 16 * (j >> 2) + 4 * kk + (j & 3), 16 * nt + m, p);
        }
        {   // decompress: w = ((et * NKS + ks) * 2 + p)
            const int p = w & 1, ks = (w >> 1) % NKS, et = (w >> 1) / NKS;
            Upd[(size_t)b * per + i] = term(c * LC + 16 * et + m, 32 * ks + 16 * (j >> 2) + 4 * kk + (j & 3), p);
        }
    }
}

// Upc / Upd for the kernels above; one thread per float, zero where e >= d or comp >= k.
__global__ void pack_long_kernel(const float* U, float* Upc, float* Upd, int d, int k, int NT, int nchunk, int c0,
                                 int npass, int pass)
{
    const int b = blockIdx.y;
    const float* Ub = U + (size_t)b * d * k + c0;          // this column pass starts at comp c0
    const size_t per = (size_t)nchunk * 4 * NT * 64 * 4;   // floats per basis and pass in either copy
    Upc += ((size_t)b * npass + pass) * per - (size_t)b * per;
    Upd += ((size_t)b * npass + pass) * per - (size_t)b * per;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < per; i += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(i & 3), lane = (int)((i >> 2) & 63), m = lane & 15, kk = lane >> 4;
        const size_t hi = i >> 8;
        const int inner = (int)(hi % NT), outer = (int)((hi / NT) & 3), c = (int)(hi / (4 * NT));
        {   // compress order: outer = i (load), inner = nt
            const int e = c * LC + LWORD(outer, kk) + j, comp = 16 * inner + m;
            Upc[(size_t)b * per + i] = (e < d && c0 + comp < k) ? Ub[(size_t)e * k + comp] : 0.0f;
        }
        {   // decompress order: outer = et, inner = w
            const int e = c * LC + 16 * outer + m, comp = 16 * inner + 4 * kk + j;
            Upd[(size_t)b * per + i] = (e < d && c0 + comp < k) ? Ub[(size_t)e * k + comp] : 0.0f;
        }
    }
}

// ======================================================================================
// host side
// ======================================================================================
// Every shape the register-resident kernels for d in {16,32,64,128}, k <= 32 do not take.  A kernel launch
// handles at most 128 comps (8 column tiles of 16); more than that takes ceil(k / 128) column passes
// over the gradient: each compress pass writes its own comps, each decompress pass after the first adds
// to the reconstruction so far (fp32 output; bf16 output of k > 128 keeps the any-shape kernel).
bool gvq_long_shape(int d, int k) { return !gvq_mfma_shape(d, k); }
int gvq_long_passes(int k) { return (k + 127) / 128; }
int gvq_long_nt(int k) { return k <= 16 ? 1 : k <= 32 ? 2 : k <= 64 ? 4 : k <= 96 ? 6 : 8; }
int gvq_long_chunks(int d) { return (d + LC - 1) / LC; }
int64_t gvq_long_tiles(int64_t slices) { return (slices + LW_SLICES - 1) / LW_SLICES; }

static int pass_k(int k, int pass) { return k - 128 * pass < 128 ? k - 128 * pass : 128; }
static int pack_nt(int k) { return k > 128 ? 8 : gvq_long_nt(k); }          // column tiles per pass as packed
static int split_nt(int k) { const int nt = pack_nt(k); return nt < 2 ? 2 : nt; }
// floats per basis in either operand-order copy of U (all passes)
size_t gvq_long_pack_floats(int d, int k)
{
    return (size_t)gvq_long_passes(k) * gvq_long_chunks(d) * LC * 16 * pack_nt(k);
}
// bf16 values per basis in either split copy of U (all passes)
size_t gvq_long_split_pack_halves(int d, int k)
{
    return (size_t)gvq_long_passes(k) * gvq_long_chunks(d) * 4 * split_nt(k) * 64 * 8;
}

// Which matrix pipe: exact fp32 products while they keep up with memory (2dk / (4(d + k)) below 10
// flop per byte; at 14, d = 256 and k = 32, the fp32 decompress already falls a quarter behind the
// split one), the bf16 split above that.  Option 2 overrides: 1 = always fp32 products, 2 = always
// the split, 3 = the split without the basis-stationary compress kernel (gvq_codec_ws.hip), which otherwise
// takes the fp32 gradients of every shape it can run on.
bool gvq_long_split(const gvq_basis* h)
{
    const int mode = gvq_opt_long_mode();
    if (mode == 1) return false;
    if (mode >= 2) return true;
    const int k = h->k < 128 ? h->k : 128;   // per pass
    return 2.0 * h->d * k / (4.0 * (h->d + k)) >= 10.0;
}

int gvq_launch_pack_long(const gvq_basis* h, hipStream_t st)
{
    const int nchunk = gvq_long_chunks(h->d), np = gvq_long_passes(h->k);
    unsigned short* Upd = h->d_Upb + (size_t)h->B * gvq_long_split_pack_halves(h->d, h->k);
    for (int p = 0; p < np; ++p) {
        hipLaunchKernelGGL(pack_long_kernel, dim3(64, h->B), dim3(256), 0, st, h->d_U, h->d_Upc, h->d_Upd, h->d, h->k,
                           pack_nt(h->k), nchunk, 128 * p, np, p);
        GVQ_HIP(hipGetLastError());
        hipLaunchKernelGGL(pack_long_split_kernel, dim3(64, h->B), dim3(256), 0, st, h->d_U, h->d_Upb, Upd, h->d, h->k,
                           split_nt(h->k), nchunk, 128 * p, np, p);
        GVQ_HIP(hipGetLastError());
    }
    if (gvq_ws_shape(h) || gvq_wsd_shape(h)) return gvq_launch_pack_ws(h, st);
    return GVQ_OK;
}

static int64_t tile_of_slice(const gvq_basis* h, int64_t s)
{
    if (h->B == 1) return s / LW_SLICES;
    int lo = 0, hi = h->B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) / 2;
        if (h->h_offs[mid] <= s) lo = mid; else hi = mid;
    }
    return h->h_ltile[lo] + (s - h->h_offs[lo]) / LW_SLICES;
}

static LongArgs long_args(const gvq_basis* h, const void* in, void* out, const float* upack, int64_t first_slice,
                          int64_t n_slices)
{
    LongArgs a;
    a.in = in; a.out = out; a.acc_in = nullptr; a.Upack = (const f4*)upack; a.Upack2 = nullptr; a.mu = h->d_mu; a.offs = h->d_offs;
    a.tstart = h->d_ltile; a.M = h->M; a.S = h->S; a.seg_begin = first_slice; a.seg_end = first_slice + n_slices;
    a.t0 = tile_of_slice(h, a.seg_begin);
    a.t1 = tile_of_slice(h, a.seg_end - 1) + 1;
    a.B = h->B; a.d = h->d; a.k = h->k; a.nchunk = gvq_long_chunks(h->d);
    a.kfull = h->k; a.c0 = 0; a.accum = 0; a.upack_stride = 0;
    a.n_workers = 1.f;
    return a;
}

// Arguments of column pass `pass`: its comps, and its packed U (`upack`: the copy of all bases and passes,
// nt column tiles per pass as packed; both copies count 4 * nt * 64 128-bit words per chunk).
static LongArgs pass_args(const gvq_basis* h, const LongArgs& a0, const void* upack, int nt, int pass)
{
    LongArgs a = a0;
    const size_t per = (size_t)a.nchunk * 4 * nt * 64;
    a.k = pass_k(h->k, pass);
    a.c0 = 128 * pass;
    a.upack_stride = (int)(per * gvq_long_passes(h->k));
    a.Upack = (const f4*)upack + per * pass;
    return a;
}

template <auto KERN>
static int launch_long(const gvq_basis* h, const LongArgs& a, int NT, hipStream_t st, int most = 0)
{
    const size_t lds = sizeof(f4) * 2 * 4 * NT * 64 + sizeof(float) * (size_t)a.nchunk * LC;
    static gvq_once_per_device once;
    if (once.first(h->device)) {
        // the largest slice needs 8 KB NT + 4 KB: allow it once, for every later launch
        GVQ_HIP(hipFuncSetAttribute((const void*)KERN, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)(sizeof(f4) * 2 * 4 * NT * 64 + sizeof(float) * GVQ_MAX_D)));
    }
    int per_cu = gvq_opt_wg_per_cu();
    if (per_cu <= 0) {
        // asked once per kernel and LDS size (the size changes with the slice length only)
        static size_t known_lds = 0;
        static int known_per_cu = 0;
        if (known_per_cu == 0 || known_lds != lds) {
            int occ = 0;
            GVQ_HIP(hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, (const void*)KERN, 256, lds));
            known_per_cu = occ < 1 ? 1 : occ;
            known_lds = lds;
        }
        per_cu = most > 0 && known_per_cu > most ? most : known_per_cu;
    }
    const int64_t tiles = a.t1 - a.t0, cap = (int64_t)h->num_cu * per_cu;
    const int grid = (int)(tiles < cap ? tiles : cap);
    hipLaunchKernelGGL(KERN, dim3(grid), dim3(256), lds, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <bool BF16, bool LOSS>
static int compress_long_nt(const gvq_basis* h, const LongArgs& a, int NT, hipStream_t st)
{
    switch (NT) {
    case 1: return launch_long<compress_long_kernel<1, BF16, LOSS>>(h, a, 1, st);
    case 2: return launch_long<compress_long_kernel<2, BF16, LOSS>>(h, a, 2, st);
    case 4: return launch_long<compress_long_kernel<4, BF16, LOSS>>(h, a, 4, st);
    case 6: return launch_long<compress_long_kernel<6, BF16, LOSS>>(h, a, 6, st);
    default: return launch_long<compress_long_kernel<8, BF16, LOSS>>(h, a, 8, st);
    }
}

// Work-groups per compute unit of the decompress kernels, at most.  Their waves spend half their time getting
// stores accepted, and more work-groups storing at once make that worse: on 138 M elements two per compute unit
// give 4.95 TB/s at d = 256, k = 32 where the four that fit give 4.35 (d = 512, k = 64: 4.5 against 4.1); with
// six or more column tiles the matrix work needs a third (d = 768, k = 96: 3.85 against 3.65 with two), and so
// does bf16 output.
static int decompress_most(int NT, bool out_bf16) { return NT >= 6 || out_bf16 ? 3 : 2; }

template <bool BF16>
static int decompress_long_nt(const gvq_basis* h, const LongArgs& a, int NT, hipStream_t st)
{
    switch (NT) {
    case 1: return launch_long<decompress_long_kernel<1, BF16>>(h, a, 1, st, decompress_most(1, BF16));
    case 2: return launch_long<decompress_long_kernel<2, BF16>>(h, a, 2, st, decompress_most(2, BF16));
    case 4: return launch_long<decompress_long_kernel<4, BF16>>(h, a, 4, st, decompress_most(4, BF16));
    case 6: return launch_long<decompress_long_kernel<6, BF16>>(h, a, 6, st, decompress_most(6, BF16));
    default: return launch_long<decompress_long_kernel<8, BF16>>(h, a, 8, st, decompress_most(8, BF16));
    }
}

template <bool BF16>
static int compress_split_nt(const gvq_basis* h, const LongArgs& a, int NT, hipStream_t st)
{
    switch (NT) {
    case 2: return launch_long<compress_split_kernel<2, BF16>>(h, a, 2, st);
    case 4: return launch_long<compress_split_kernel<4, BF16>>(h, a, 4, st);
    case 6: return launch_long<compress_split_kernel<6, BF16>>(h, a, 6, st);
    default: return launch_long<compress_split_kernel<8, BF16>>(h, a, 8, st);
    }
}

template <bool BF16>
static int decompress_split_nt(const gvq_basis* h, const LongArgs& a, int NT, hipStream_t st)
{
    switch (NT) {
    case 2: return launch_long<decompress_split_kernel<2, BF16>>(h, a, 2, st, decompress_most(2, BF16));
    case 4: return launch_long<decompress_split_kernel<4, BF16>>(h, a, 4, st, decompress_most(4, BF16));
    case 6: return launch_long<decompress_split_kernel<6, BF16>>(h, a, 6, st, decompress_most(6, BF16));
    default: return launch_long<decompress_split_kernel<8, BF16>>(h, a, 8, st, decompress_most(8, BF16));
    }
}

int gvq_launch_compress_long(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice,
                             int64_t n_slices, const float* comp_in, float* out, hipStream_t st)
{
    const bool split = gvq_long_split(h), bf = h->dtype == GVQ_BF16;
    // the shapes it takes (one basis, d a multiple of 256): the kernel that keeps U in registers (option 2 = 3: never).
    // bf16 storage on the split pipe only.  With exact
    // fp32 products only from d = 512 up: at d = 256 its two accumulator chains per wave leave the fp32 matrix pipe
    // waiting, and the LDS-tiled kernel is 13 - 20 % faster (d = 768, k = 16: 5.2 against 4.5 TB/s; d = 1024: 5.2
    // against 3.5; d = 512: level).
    const int mode = gvq_opt_long_mode();
    if (gvq_ws_shape(h) && mode != 3 && (split || (!bf && h->d >= 512))) {
        int64_t done = 0;
        const int rc = gvq_launch_compress_ws(h, grad, n_workers, first_slice, n_slices, comp_in, out, !split, st, &done);
        if (rc != GVQ_OK) return rc;
        first_slice += done;
        n_slices -= done;
        if (n_slices <= 0) return GVQ_OK;
    }
    LongArgs a0 = long_args(h, grad, out, h->d_Upc, first_slice, n_slices);
    a0.acc_in = comp_in;
    a0.n_workers = (float)n_workers;
    for (int p = 0; p < gvq_long_passes(h->k); ++p) {
        int rc;
        if (split) {
            const LongArgs a = pass_args(h, a0, h->d_Upb, split_nt(h->k), p);
            rc = bf ? compress_split_nt<true>(h, a, split_nt(h->k), st) : compress_split_nt<false>(h, a, split_nt(h->k), st);
        } else {
            const LongArgs a = pass_args(h, a0, h->d_Upc, pack_nt(h->k), p);
            rc = bf ? compress_long_nt<true, false>(h, a, pack_nt(h->k), st)
                    : compress_long_nt<false, false>(h, a, pack_nt(h->k), st);
        }
        if (rc != GVQ_OK) return rc;
    }
    return GVQ_OK;
}

// Per-slice squared residuals of Eq. (6) into loss_slice[S]; the caller sums them per basis.  k <= 128.
int gvq_launch_loss_long(const gvq_basis* h, const void* grad, int n_workers, float* loss_slice, hipStream_t st)
{
    LongArgs a0 = long_args(h, grad, loss_slice, h->d_Upc, 0, h->S);
    a0.n_workers = (float)n_workers;
    const int NT = gvq_long_nt(h->k);
    LongArgs a = pass_args(h, a0, h->d_Upc, NT, 0);
    a.Upack2 = (const f4*)h->d_Upd;
    return h->dtype == GVQ_BF16 ? compress_long_nt<true, true>(h, a, NT, st)
                                : compress_long_nt<false, true>(h, a, NT, st);
}

// k > 128 needs fp32 output (the passes add up in grad_out).
int gvq_launch_decompress_long(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices,
                               void* out, gvq_dtype_t odt, hipStream_t st)
{
    const bool split = gvq_long_split(h), bf = odt == GVQ_BF16;
    // the shapes it takes (one basis, d a multiple of 256): the kernel that keeps U in registers (option 2 = 3: never); with exact fp32
    // products from d = 512 up, like compress (d = 1024, k = 16: 5.2 against 3.0 TB/s, d = 512, k = 16: 5.2 against 4.5)
    if (gvq_wsd_shape(h) && gvq_opt_long_mode() != 3 && (split || h->d >= 512)) {
        int64_t done = 0;
        const int rc = gvq_launch_decompress_ws(h, comp, first_slice, n_slices, out, bf, !split, st, &done);
        if (rc != GVQ_OK) return rc;
        first_slice += done;
        n_slices -= done;
        if (n_slices <= 0) return GVQ_OK;
    }
    const LongArgs a0 = long_args(h, comp, out, h->d_Upd, first_slice, n_slices);
    const unsigned short* Upd_split = h->d_Upb + (size_t)h->B * gvq_long_split_pack_halves(h->d, h->k);
    for (int p = 0; p < gvq_long_passes(h->k); ++p) {
        int rc;
        if (split) {
            LongArgs a = pass_args(h, a0, Upd_split, split_nt(h->k), p);
            a.accum = p > 0;
            rc = bf ? decompress_split_nt<true>(h, a, split_nt(h->k), st) : decompress_split_nt<false>(h, a, split_nt(h->k), st);
        } else {
            LongArgs a = pass_args(h, a0, h->d_Upd, pack_nt(h->k), p);
            a.accum = p > 0;
            rc = bf ? decompress_long_nt<true>(h, a, pack_nt(h->k), st) : decompress_long_nt<false>(h, a, pack_nt(h->k), st);
        }
        if (rc != GVQ_OK) return rc;
    }
    return GVQ_OK;
}
