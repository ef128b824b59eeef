// Codec kernels for gfx950: compress (Eq. 2), aggregate (Eq. 3), decompress (Eq. 4) of
// GradiVeQ, Section 2, for the shapes whose basis fits a wave's registers (d in {16,32,64,128},
// k <= 32); every other shape with k <= 128 goes to the LDS-tiled kernels of gvq_codec_long.hip,
// k > 128 to the one-thread-per-output kernels here.  All stream the gradient once.
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
#include "gvq_device.h"

#include <mutex>

// --------------------------------------------------------------------------------------
// Fast phase shared by the register-resident kernels.
//
// The bounds-checked loops further down serve every tile, but their branches (partial tiles,
// slices of two bases in one tile, basis reloads) make the compiler's wait-count bookkeeping give
// up: it then waits for *everything* in flight at the top of every tile -- the prefetched next
// tile and the stores just issued -- and a wave has nothing in flight while it multiplies.  So the
// bulk of the work, whole tiles of one basis, runs in a loop without a single branch around a
// memory instruction: every load and store is unconditional (lanes with nothing to do repeat the
// last valid address; duplicate stores write the same bytes), the basis is loaded outside the
// tile loop and waited for explicitly, and the next super-tile's loads are issued right after the
// current one is parked in LDS.  The compiler then counts exactly: the wait before parking a tile
// leaves the previous tile's stores in flight.
// A super-tile is 2048 consecutive gradient elements (128/D 16-slice tiles): 8 loads of 128 bits
// per lane whatever the slice length, so short slices move as many bytes per loop trip as long ones.
// --------------------------------------------------------------------------------------
// MANY: the handle has several bases and the super-tiles come from its tables; otherwise they are
// consecutive and all of basis 0.  G: 16-slice tiles per super-tile.
template <int G, bool MANY>
__device__ __forceinline__ int64_t super_tile(const CodecArgs& a, int64_t p)
{
    if constexpr (MANY) return uniform_load(a.sup_tile + p);
    else return a.sup_first + p * G;
}
template <bool MANY>
__device__ __forceinline__ int super_basis(const CodecArgs& a, int64_t p)
{
    if constexpr (MANY) return uniform_load(a.sup_basis + p);
    else return 0;
}

// NSO = 128-bit result words per lane and super-tile: ceil(8 k / D), a template value so that the
// stores can be counted (YS picks it: the largest possible number, G * NT, shifted right by YS).
// LOSS: Eq. (6) instead of Eq. (2): the per-slice squared residual is written (a.out: one float per slice), see the
// general phase of the kernel for how the reconstruction comes out of the accumulators; a.il must be 1.
template <int D, int NT, bool BF16, int VAR, int YS, bool MANY, bool LOSS = false>
__device__ __forceinline__ void compress_fast_phase(const CodecArgs& a, f4* lds)
{
    constexpr int G = 128 / D;                    // 16-slice tiles per super-tile
    constexpr int CPS = D / 4;                    // fp32 128-bit chunks per slice
    constexpr int EPL = BF16 ? 8 : 4;             // elements per 128-bit global load
    constexpr int LCPS = D / EPL;                 // load chunks per slice
    constexpr int NL = 2048 / EPL / 64;           // loads per lane per super-tile
    constexpr int NQ = CPS / 4;
    constexpr int KC = 4 * NT;                    // 128-bit chunks per slice of the padded result tile
    constexpr int NSO = ((G * NT) >> YS) > 0 ? ((G * NT) >> YS) : 1;
    constexpr bool RING = (VAR & 4) != 0;
    constexpr bool KEEP = (VAR & 8) != 0;         // results written with ordinary instead of non-temporal stores

    SuperIter it;
    if (!it.init(a.n_super, a.run_tiles)) return;

    const int lane = threadIdx.x & 63, n_ = lane & 15, kk = lane >> 4;
    const int kc = a.k >> 2, cnt = G * TILE_SLICES * kc;   // result words of a super-tile
    // result word gi of a super-tile belongs to the input row gi / orw (a row: 1 KB of input, a whole number of
    // slices, orw 128-bit words of result)
    const int orw = (1024 / (D * (BF16 ? 2 : 4))) * kc;
    int so_slot[NSO], so_row[NSO], so_in[NSO];
#pragma unroll
    for (int r = 0; r < NSO; ++r) {
        int gi = r * 64 + lane;
        if (gi > cnt - 1) gi = cnt - 1;
        const int s = gi / kc, c = gi - s * kc;
        so_slot[r] = s * KC + (c ^ swz<16 * NT>(s & 15));
        so_row[r] = gi / orw;
        so_in[r] = 4 * (gi - so_row[r] * orw);
    }
    const int lc = lane % LCPS;
    int in_slot[NL];
#pragma unroll
    for (int r = 0; r < NL; ++r) {
        const int row = (r * 64 + lane) / LCPS;
        in_slot[r] = row * CPS + ((BF16 ? 2 * lc : lc) ^ swz<D>(row & 15));
    }

    f4 uf[NQ][NT];
    f4 ud[LOSS ? NQ : 1][NT];   // LOSS only: ud[et][q][j] = U[16et + n_][16q + 4kk + j]
    float mun[EPL];
    auto load_basis = [&](int b) {
        const f4* Up = a.Upack + (size_t)b * (NQ * NT * 64) + lane;
        const float* mub = a.mu + (size_t)b * D;
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) uf[q][nt] = Up[(q * NT + nt) * 64];
        if constexpr (LOSS) {
            const f4* Up2 = a.Upack2 + (size_t)b * (NQ * NT * 64) + lane;
#pragma unroll
            for (int et = 0; et < NQ; ++et)
#pragma unroll
                for (int q = 0; q < NT; ++q) ud[et][q] = Up2[(et * NT + q) * 64];
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i) mun[i] = mub[lc * EPL + i] / a.n_workers;
    };

    u4 regs[NL];
    f4 prev[RING ? NSO : 1];
    // Where super-tile p lies.  A super-tile is NL rows of 1 KB (a row: 64 lanes x 128 bits, a whole number of
    // slices).  One basis: each group of a.il consecutive super-tiles covers a.il * NL consecutive rows and member j
    // takes rows j, j + a.il, j + 2 a.il, ... of them, so that the waves that run side by side read and write one
    // compact window row by row; the super-tiles past the last whole group keep their own NL consecutive rows.
    constexpr int ES = BF16 ? 2 : 4;
    const int64_t n_il = (!MANY && a.il > 1) ? a.n_super / a.il * a.il : 0;
    struct Where { int64_t in_byte, out_word; int rstride; };   // first input byte, first result word, rows between rows
    auto where = [&](int64_t p) {
        Where w;
        if (!MANY && p < n_il) {
            const int64_t g = p / a.il, j = p - g * a.il;
            const int64_t row = g * a.il * NL + j;                    // from the first super-tile's start
            w.in_byte = a.sup_first * (int64_t)(TILE_SLICES * D * ES) + row * 1024;
            w.out_word = a.sup_first * (int64_t)(TILE_SLICES) * kc + row * orw;
            w.rstride = a.il;
        } else {
            const int64_t t0 = super_tile<G, MANY>(a, p);
            w.in_byte = t0 * (int64_t)(TILE_SLICES * D * ES);
            w.out_word = t0 * (int64_t)(TILE_SLICES) * kc;
            w.rstride = 1;
        }
        return w;
    };
    // `rows`: false when there is no next super-tile (the loads stay so that they can be counted, but all
    // fetch one row that was just read)
    auto load_super = [&](const Where& w, bool rows) {
        const char* base = (const char*)a.in + w.in_byte + lane * 16;
        const int64_t stride = rows ? (int64_t)w.rstride * 1024 : 0;
#pragma unroll
        for (int r = 0; r < NL; ++r) regs[r] = stream_load((const u4*)(base + r * stride));
        if constexpr (RING) {
            const float* pin = a.acc_in + 4 * w.out_word;
#pragma unroll
            for (int r = 0; r < NSO; ++r) prev[r] = stream_load((const f4*)(pin + 4 * so_row[r] * w.rstride * orw + so_in[r]));
        }
    };

    int64_t cur = it.p;
    int b = super_basis<MANY>(a, cur);
    Where wc = where(cur);
    load_super(wc, true);
    for (;;) {
        load_basis(b);
        drain_memory();
        int nb;
        do {
            const bool more = it.advance();
            const int64_t nxt = more ? it.p : cur;
            nb = more ? super_basis<MANY>(a, nxt) : -1;
            const Where wn = where(nxt);

            if (a.pace & 1) drain_memory();
            // park the super-tile in LDS as fp32, minus mu/N
            wave_lds_sync();
#pragma unroll
            for (int r = 0; r < NL; ++r) {
                const u4 v = regs[r];
                if (BF16) {
                    f4 lo = {bf16_to_f32(v.x & 0xffffu) - mun[0], bf16_to_f32(v.x >> 16) - mun[1],
                             bf16_to_f32(v.y & 0xffffu) - mun[2], bf16_to_f32(v.y >> 16) - mun[3]};
                    f4 hi = {bf16_to_f32(v.z & 0xffffu) - mun[4 % EPL], bf16_to_f32(v.z >> 16) - mun[5 % EPL],
                             bf16_to_f32(v.w & 0xffffu) - mun[6 % EPL], bf16_to_f32(v.w >> 16) - mun[7 % EPL]};
                    lds[in_slot[r]] = lo;
                    lds[in_slot[r] ^ 1] = hi;
                } else {
                    f4 x = {__uint_as_float(v.x) - mun[0], __uint_as_float(v.y) - mun[1],
                            __uint_as_float(v.z) - mun[2], __uint_as_float(v.w) - mun[3]};
                    lds[in_slot[r]] = x;
                }
            }
            f4 pv[RING ? NSO : 1];
            if constexpr (RING) {
#pragma unroll
                for (int r = 0; r < NSO; ++r) pv[r] = prev[r];
            }
            load_super(wn, more);   // the next super-tile (or one row of this one, unused, when there is none)
            wave_lds_sync();
            f4 x[G][NQ];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int q = 0; q < NQ; ++q) x[g][q] = lds[(g * 16 + n_) * CPS + ((4 * q + kk) ^ swz<D>(n_))];
            f4 acc[G][NT];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[g][nt] = f4{0.f, 0.f, 0.f, 0.f};
            __builtin_amdgcn_s_setprio(3);
            // NQ * G = 8 = NL groups of products; with pacing, group i waits for load i of the next super-tile
            static_for<0, NQ * G>([&](auto ic) {
                constexpr int i = decltype(ic)::value, q = i / G, g = i % G;
                if constexpr (NQ * G == NL) {
                    if (a.pace & 4) wait_vmem_at_most<NL - 1 - i + (RING ? NSO : 0)>();
                }
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[g][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(uf[q][nt][j], x[g][q][j], acc[g][nt], 0, 0, 0);
            });
            if constexpr (LOSS) {
                // whole slices inside the gradient: every element counts
                const int64_t s0 = super_tile<G, MANY>(a, cur) * TILE_SLICES;
#pragma unroll
                for (int g = 0; g < G; ++g) {
                    float sq = 0.f;
#pragma unroll
                    for (int et = 0; et < NQ; ++et) {
                        f4 rec = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                        for (int q = 0; q < NT; ++q)
#pragma unroll
                            for (int jj = 0; jj < 4; ++jj)
                                rec = __builtin_amdgcn_mfma_f32_16x16x4f32(ud[et][q][jj], acc[g][q][jj], rec, 0, 0, 0);
#pragma unroll
                        for (int r = 0; r < 4; ++r) {
                            const float df = x[g][et][r] - rec[r];
                            sq = fmaf(df, df, sq);
                        }
                    }
                    sq += __shfl_xor(sq, 16, 64);
                    sq += __shfl_xor(sq, 32, 64);
                    if (kk == 0) ((float*)a.out)[s0 + g * 16 + n_] = sq;
                }
                __builtin_amdgcn_s_setprio(0);
            } else {
            __builtin_amdgcn_s_setprio(0);
            if (a.pace & 2) drain_memory();
            // the result tiles leave through the same LDS region (every x is in registers by now) as
            // full-width stores in memory order
            wave_lds_sync();
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    lds[(g * 16 + n_) * KC + ((4 * nt + kk) ^ swz<16 * NT>(n_))] = acc[g][nt];
            wave_lds_sync();
            float* o = (float*)a.out + 4 * wc.out_word;
#pragma unroll
            for (int r = 0; r < NSO; ++r) {
                f4 v = lds[so_slot[r]];
                if constexpr (RING) v += pv[r];
                f4* dst = (f4*)(o + 4 * so_row[r] * wc.rstride * orw + so_in[r]);
                if constexpr (KEEP) *dst = v;
                else stream_store(dst, v);
            }
            }
            cur = nxt;
            wc = wn;
        } while (nb == b);
        if (nb < 0) break;
        b = nb;
    }
    drain_memory();
}

// --------------------------------------------------------------------------------------
// compress, MFMA path.  D in {16,32,64,128}, NT = ceil(k/16) in {1,2}.
//
// Per 16-slice tile a wave loads 128-bit words in memory order (fully coalesced: the tile
// is one contiguous run of 16*D elements), subtracts mu/N, and parks them in its private
// LDS region; the lanes then read the data back in the B-operand order (lane = slice, 4
// consecutive elements per 128-bit read).  Chunk c (4 floats) of slice s lives at 128-bit
// slot s*CPS + (c ^ swz(s)), a XOR swizzle that keeps 8 consecutive lanes on 8 distinct
// 128-bit bank groups for the transposed read.  The loads of the next tile are in flight
// while the current one is multiplied.
// The contraction index may be visited in any order as long as U follows: MFMA step
// (q, j) multiplies elements e = 4*(4q + kk) + j, kk = l/16.
// --------------------------------------------------------------------------------------
template <int D, int NT, bool BF16, int VAR, bool LOSS, int YS>
__global__ __launch_bounds__(WG_THREADS, LOSS ? 1 : 2) void compress_mfma_kernel(CodecArgs a)
{
    constexpr int CPS = D / 4;                    // fp32 128-bit chunks per slice
    constexpr int EPL = BF16 ? 8 : 4;             // elements per 128-bit global load
    constexpr int LCPS = D / EPL;                 // load chunks per slice
    constexpr int TILE_LOADS = TILE_SLICES * LCPS;  // 128-bit loads per tile
    constexpr int NL = (TILE_LOADS + 63) / 64;    // loads per lane per tile
    constexpr int NQ = CPS / 4;                   // 128-bit LDS reads per lane per tile
    constexpr int64_t TILE_ELEMS = (int64_t)TILE_SLICES * D;

    constexpr int KC = 4 * NT;                    // 128-bit chunks per slice of the padded result tile

    __shared__ f4 lds_all[WAVES_PER_WG][512];     // one super-tile of the fast phase (8 KB per wave)
    __shared__ f4 ldso_all[WAVES_PER_WG][TILE_SLICES * KC];
    const int lane = threadIdx.x & 63;
    f4* lds = lds_all[threadIdx.x >> 6];
    f4* ldso = ldso_all[threadIdx.x >> 6];

    if (a.sup_tile) compress_fast_phase<D, NT, BF16, VAR, YS, true, LOSS>(a, lds);
    else compress_fast_phase<D, NT, BF16, VAR, YS, false, LOSS>(a, lds);

    // ---- general phase: the tiles the fast phase leaves out, every check in place ----------
    RestIter it;
    if (!it.init(a)) return;

    const int n_ = lane & 15, kk = lane >> 4;
    // result tile in memory order: 16 slices x k floats, contiguous; this lane's 128-bit pieces
    const int kc = a.k >> 2;
    int so_s[NT], so_c[NT];
#pragma unroll
    for (int r = 0; r < NT; ++r) {
        const int g = r * 64 + lane;
        so_s[r] = kc ? g / kc : 0;
        so_c[r] = kc ? g - so_s[r] * kc : 0;
    }
    const int lc = lane % LCPS;                   // this lane's load chunk within a slice
    const bool loads = lane < TILE_LOADS;         // false only for the upper lanes at D = 16, bf16

    // ---- per-basis state -------------------------------------------------------------
    int cur_b = block_of_tile(a, it.t);
    int64_t blk_begin = a.offs[cur_b], blk_end = a.offs[cur_b + 1];
    f4 uf[NQ][NT];   // uf[q][nt][j] = U[4*(4q + kk) + j][16nt + n_], zero past column k
    f4 ud[LOSS ? NQ : 1][NT];   // LOSS only: ud[et][q][j] = U[16et + n_][16q + 4kk + j]
    float mun[EPL];

    auto load_basis = [&](int b) {
        const f4* Up = a.Upack + (size_t)b * (NQ * NT * 64) + lane;
        const float* mub = a.mu + (size_t)b * D;
#pragma unroll
        for (int q = 0; q < NQ; ++q)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) uf[q][nt] = Up[(q * NT + nt) * 64];
        if constexpr (LOSS) {
            const f4* Up2 = a.Upack2 + (size_t)b * (NQ * NT * 64) + lane;
#pragma unroll
            for (int et = 0; et < NQ; ++et)
#pragma unroll
                for (int q = 0; q < NT; ++q) ud[et][q] = Up2[(et * NT + q) * 64];
        }
#pragma unroll
        for (int i = 0; i < EPL; ++i) mun[i] = mub[lc * EPL + i] / a.n_workers;
    };
    load_basis(cur_b);

    // ---- tile loads --------------------------------------------------------------------
    u4 regs[NL];
    auto load_tile = [&](int64_t t) {
        const int64_t base = t * TILE_ELEMS;  // first element of the tile
        if (base + TILE_ELEMS <= a.M) {       // interior tile: no bounds checks
#pragma unroll
            for (int r = 0; r < NL; ++r) {
                const int g = r * 64 + lane;
                if (NL * 64 == TILE_LOADS || loads)
                    regs[r] = stream_load((const u4*)((const char*)a.in + (base + (int64_t)g * EPL) * (BF16 ? 2 : 4)));
            }
            return;
        }
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            const int g = r * 64 + lane;
            u4 v = {0u, 0u, 0u, 0u};
            const int64_t e0 = base + (int64_t)g * EPL;
            if (g < TILE_LOADS && e0 < a.M) {
                if (e0 + EPL <= a.M) {
                    v = *(const u4*)((const char*)a.in + e0 * (BF16 ? 2 : 4));
                } else if (BF16) {
                    const unsigned short* p = (const unsigned short*)a.in;
                    unsigned int h[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) h[i] = e0 + i < a.M ? p[e0 + i] : 0u;
                    v = u4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                } else {
                    const unsigned int* p = (const unsigned int*)a.in;
                    v = u4{p[e0], e0 + 1 < a.M ? p[e0 + 1] : 0u, e0 + 2 < a.M ? p[e0 + 2] : 0u,
                           e0 + 3 < a.M ? p[e0 + 3] : 0u};
                }
            }
            regs[r] = v;
        }
    };
    // park the loaded tile in LDS as fp32, minus mu/N
    auto stage_tile = [&]() {
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            const int g = r * 64 + lane;
            if (NL * 64 == TILE_LOADS || loads) {
                const int s = g / LCPS;
                const u4 v = regs[r];
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

    load_tile(it.t);
    for (bool more = true; more;) {
        const int64_t t = it.t;
        const int64_t s0 = t * TILE_SLICES;
        const int64_t s1 = s0 + TILE_SLICES < a.S ? s0 + TILE_SLICES : a.S;
        if (s0 >= blk_end || s0 < blk_begin) {  // this tile starts in another basis
            cur_b = block_of_tile(a, t);
            blk_begin = a.offs[cur_b];
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        wave_lds_sync();
        stage_tile();
        wave_lds_sync();
        more = it.advance();
        if (more) load_tile(it.t);
        if constexpr ((VAR & 2) != 0) __builtin_amdgcn_s_setprio(3);

        for (;;) {
            int64_t lo, hi;
            row_range(a, s0, s1, blk_begin, blk_end, lo, hi);
            f4 x[NQ];
#pragma unroll
            for (int q = 0; q < NQ; ++q) x[q] = lds[n_ * CPS + ((4 * q + kk) ^ swz<D>(n_))];
            f4 acc[NT], prev[NT];
            if constexpr ((VAR & 4) != 0) load_acc_in<NT>(a, s0 + n_, kk, s0 + n_ >= lo && s0 + n_ < hi, prev);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(uf[q][nt][j], x[q][j], acc[nt], 0, 0, 0);
            if constexpr ((VAR & 4) != 0) {   // ring step: add the predecessor's partial sum
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] += prev[nt];
            }
            // lane holds comps 16*nt + 4*kk + r of slice s0 + n_
            if constexpr (LOSS) {
                // Eq. (6): reconstruct U y from the accumulators (they already sit in the
                // B-operand order of the second product) and compare with the parked x - mu/N;
                // x[et][r] and the result register r of tile et are the same element 16et + 4kk + r
                const int64_t j = s0 + n_;
                float sq = 0.f;
#pragma unroll
                for (int et = 0; et < NQ; ++et) {
                    f4 rec = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int q = 0; q < NT; ++q)
#pragma unroll
                        for (int jj = 0; jj < 4; ++jj)
                            rec = __builtin_amdgcn_mfma_f32_16x16x4f32(ud[et][q][jj], acc[q][jj], rec, 0, 0, 0);
                    const int64_t e0 = j * D + 16 * et + 4 * kk;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        const float df = x[et][r] - rec[r];
                        if (e0 + r < a.M) sq = fmaf(df, df, sq);   // padding is not part of the gradient
                    }
                }
                sq += __shfl_xor(sq, 16, 64);
                sq += __shfl_xor(sq, 32, 64);
                if (kk == 0 && j >= lo && j < hi) ((float*)a.out)[j] = sq;
            } else if ((a.k & 3) == 0 && (VAR & 1) == 0) {
                const int64_t j = s0 + n_;
                if (j >= lo && j < hi) {
                    float* o = (float*)a.out + j * a.k;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        if (16 * nt + 4 * kk < a.k) stream_store((f4*)(o + 16 * nt + 4 * kk), acc[nt]);
                }
            } else if ((a.k & 3) == 0) {
                // through LDS, so that the tile leaves as full-width stores in memory order
                wave_lds_sync();
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) ldso[n_ * KC + ((4 * nt + kk) ^ swz<16 * NT>(n_))] = acc[nt];
                wave_lds_sync();
                float* o = (float*)a.out + s0 * a.k;
#pragma unroll
                for (int r = 0; r < NT; ++r) {
                    const int g = r * 64 + lane;
                    const int64_t j = s0 + so_s[r];
                    if (g < TILE_SLICES * kc && j >= lo && j < hi)
                        stream_store((f4*)(o + 4 * g), ldso[so_s[r] * KC + (so_c[r] ^ swz<16 * NT>(so_s[r]))]);
                }
            } else {
                const int64_t j = s0 + n_;
                if (j >= lo && j < hi) {
                    float* o = (float*)a.out + j * a.k;
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (16 * nt + 4 * kk + r < a.k) o[16 * nt + 4 * kk + r] = acc[nt][r];
                }
            }
            if constexpr ((VAR & 2) != 0) __builtin_amdgcn_s_setprio(0);
            if (blk_end >= s1) break;
            // the tile continues into the next basis: re-centre the parked data and redo it
            float old[EPL];
#pragma unroll
            for (int i = 0; i < EPL; ++i) old[i] = mun[i];
            cur_b += 1;
            blk_begin = blk_end;
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
            wave_lds_sync();
            if (loads) {
#pragma unroll
                for (int r = 0; r < NL; ++r) {
                    const int s = (r * 64 + lane) / LCPS;
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
            wave_lds_sync();
        }
    }
}

// --------------------------------------------------------------------------------------
// compress for bf16-stored gradients on the bf16 matrix pipe, D in {32,64,128}.
//
// A bf16 input needs no conversion at all: 8 consecutive elements of a slice are exactly one
// B operand of v_mfma_f32_16x16x32_bf16.  U is fp32; it is split once per basis into three
// bf16 terms u1 + u2 + u3 (each the bf16 rounding of what the previous terms left over, which
// reproduces all 24 mantissa bits), so three MFMAs give the fp32-exact products and the
// accumulation stays fp32 -- a sixth of the fp32 pipe's cycles, no VALU conversion work, half
// the LDS traffic.  Eq. (2)'s centring cannot be applied to the bf16 operand, so it becomes
// the accumulator's start value: y = U^T x - U^T mu / N (algebraically the same; it costs
// digits only when |mu|/N exceeds the spread of x by ~1e3, far beyond what bf16 storage
// itself resolves).
// Tile staging is the same as in the fp32 kernel (memory-order 128-bit loads, swizzled LDS,
// lane = slice on the way back); MFMA step st of lane (n, kk) contracts elements
// 8(4 st + kk) .. +7.
// --------------------------------------------------------------------------------------
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));

// Fast phase of the bf16-pipe compress (see compress_fast_phase).  A super-tile is G2 = 2 (D = 128) or 4
// 16-slice tiles: 8 loads of 128 bits per lane at D >= 64, 4 at D = 32.
template <int D> constexpr int bf16_super_tiles() { return D == 128 ? 2 : 4; }

template <int D, int NT, bool ACC, int YS, bool MANY>
__device__ __forceinline__ void compress_bf16_fast_phase(const CodecArgs& a, u4* lds)
{
    constexpr int G = bf16_super_tiles<D>();
    constexpr int C8 = D / 8, NST = D / 32, KC = 4 * NT;
    constexpr int NL = G * TILE_SLICES * C8 / 64;
    constexpr int NSO = ((G * NT) >> YS) > 0 ? ((G * NT) >> YS) : 1;
    f4* ldsf = (f4*)lds;

    SuperIter it;
    if (!it.init(a.n_super, a.run_tiles)) return;

    const int lane = threadIdx.x & 63, n_ = lane & 15, kk = lane >> 4;
    const int kc = a.k >> 2, cnt = G * TILE_SLICES * kc;
    const int orw = (1024 / (D * 2)) * kc;   // result words of one 1 KB input row (see compress_fast_phase)
    int so_slot[NSO], so_row[NSO], so_in[NSO];
#pragma unroll
    for (int r = 0; r < NSO; ++r) {
        int gi = r * 64 + lane;
        if (gi > cnt - 1) gi = cnt - 1;
        const int s = gi / kc, c = gi - s * kc;
        so_slot[r] = s * KC + (c ^ swz<16 * NT>(s & 15));
        so_row[r] = gi / orw;
        so_in[r] = 4 * (gi - so_row[r] * orw);
    }
    int in_slot[NL];
#pragma unroll
    for (int r = 0; r < NL; ++r) {
        const int g = r * 64 + lane, row = g / C8, c = g % C8;
        in_slot[r] = row * C8 + (c ^ swz<D / 2>(row & 15));
    }

    u4 ua[NST][3][NT];
    f4 bias[NT];
    auto load_basis = [&](int b) {
        const u4* Up = (const u4*)a.Upack + (size_t)b * (NST * 3 * NT * 64) + lane;
#pragma unroll
        for (int st = 0; st < NST; ++st)
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) ua[st][p][nt] = Up[((st * 3 + p) * NT + nt) * 64];
        const f4* um = (const f4*)(a.Umu + (size_t)b * 16 * NT) + kk;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bias[nt] = um[4 * nt] / a.n_workers;
    };
    u4 regs[NL];
    f4 prev[ACC ? NSO : 1];
    // Where super-tile p lies: see compress_fast_phase.
    const int64_t n_il = (!MANY && a.il > 1) ? a.n_super / a.il * a.il : 0;
    struct Where { int64_t in_byte, out_word; int rstride; };
    auto where = [&](int64_t p) {
        Where w;
        if (!MANY && p < n_il) {
            const int64_t g = p / a.il, j = p - g * a.il;
            const int64_t row = g * a.il * NL + j;
            w.in_byte = a.sup_first * (int64_t)(TILE_SLICES * D * 2) + row * 1024;
            w.out_word = a.sup_first * (int64_t)(TILE_SLICES) * kc + row * orw;
            w.rstride = a.il;
        } else {
            const int64_t t0 = super_tile<G, MANY>(a, p);
            w.in_byte = t0 * (int64_t)(TILE_SLICES * D * 2);
            w.out_word = t0 * (int64_t)(TILE_SLICES) * kc;
            w.rstride = 1;
        }
        return w;
    };
    auto load_super = [&](const Where& w, bool rows) {   // rows: see compress_fast_phase
        const char* base = (const char*)a.in + w.in_byte + lane * 16;
        const int64_t stride = rows ? (int64_t)w.rstride * 1024 : 0;
#pragma unroll
        for (int r = 0; r < NL; ++r) regs[r] = stream_load((const u4*)(base + r * stride));
        if constexpr (ACC) {
            const float* pin = a.acc_in + 4 * w.out_word;
#pragma unroll
            for (int r = 0; r < NSO; ++r)
                prev[r] = stream_load((const f4*)(pin + 4 * so_row[r] * w.rstride * orw + so_in[r]));
        }
    };

    int64_t cur = it.p;
    int b = super_basis<MANY>(a, cur);
    Where wc = where(cur);
    load_super(wc, true);
    for (;;) {
        load_basis(b);
        drain_memory();
        int nb;
        do {
            const bool more = it.advance();
            const int64_t nxt = more ? it.p : cur;
            nb = more ? super_basis<MANY>(a, nxt) : -1;
            const Where wn = where(nxt);

            if (a.pace & 1) drain_memory();
            wave_lds_sync();
#pragma unroll
            for (int r = 0; r < NL; ++r) lds[in_slot[r]] = regs[r];
            f4 pv[ACC ? NSO : 1];
            if constexpr (ACC) {
#pragma unroll
                for (int r = 0; r < NSO; ++r) pv[r] = prev[r];
            }
            load_super(wn, more);
            wave_lds_sync();
            u4 xb[G][NST];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int st = 0; st < NST; ++st) xb[g][st] = lds[(g * 16 + n_) * C8 + ((4 * st + kk) ^ swz<D / 2>(n_))];
            f4 acc[G][NT];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[g][nt] = -bias[nt];
            __builtin_amdgcn_s_setprio(3);
            // NST * G = NL groups of products; with pacing, group i waits for load i of the next super-tile
            static_for<0, NST * G>([&](auto ic) {
                constexpr int i = decltype(ic)::value, st = i / G, g = i % G;
                if (a.pace & 4) wait_vmem_at_most<NL - 1 - i + (ACC ? NSO : 0)>();
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[g][nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf8, ua[st][p][nt]), __builtin_bit_cast(bf8, xb[g][st]), acc[g][nt], 0, 0, 0);
            });
            __builtin_amdgcn_s_setprio(0);
            if (a.pace & 2) drain_memory();
            wave_lds_sync();   // every xb is in registers: the region now takes the result tiles
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    ldsf[(g * 16 + n_) * KC + ((4 * nt + kk) ^ swz<16 * NT>(n_))] = acc[g][nt];
            wave_lds_sync();
            float* o = (float*)a.out + 4 * wc.out_word;
#pragma unroll
            for (int r = 0; r < NSO; ++r) {
                f4 v = ldsf[so_slot[r]];
                if constexpr (ACC) v += pv[r];
                stream_store((f4*)(o + 4 * so_row[r] * wc.rstride * orw + so_in[r]), v);
            }
            cur = nxt;
            wc = wn;
        } while (nb == b);
        if (nb < 0) break;
        b = nb;
    }
    drain_memory();
}

template <int D, int NT, bool ACC, int YS>
__global__ __launch_bounds__(WG_THREADS, 2) void compress_bf16_kernel(CodecArgs a)
{
    constexpr int C8 = D / 8;                        // 128-bit chunks (8 bf16) per slice
    constexpr int TILE_LOADS = TILE_SLICES * C8;
    constexpr int NL = (TILE_LOADS + 63) / 64;
    constexpr int NST = D / 32;                      // MFMA steps per tile
    constexpr int64_t TILE_ELEMS = (int64_t)TILE_SLICES * D;

    __shared__ u4 lds_all[WAVES_PER_WG][512];        // one super-tile of the fast phase (8 KB per wave)
    const int lane = threadIdx.x & 63;
    u4* lds = lds_all[threadIdx.x >> 6];

    if (a.sup_tile) compress_bf16_fast_phase<D, NT, ACC, YS, true>(a, lds);
    else compress_bf16_fast_phase<D, NT, ACC, YS, false>(a, lds);

    // ---- general phase: the tiles the fast phase leaves out, every check in place ----------
    RestIter it;
    if (!it.init(a)) return;
    const int n_ = lane & 15, kk = lane >> 4;
    const bool loads = lane < TILE_LOADS;            // false only for the upper lanes at D = 32

    int cur_b = block_of_tile(a, it.t);
    int64_t blk_begin = a.offs[cur_b], blk_end = a.offs[cur_b + 1];
    u4 ua[NST][3][NT];   // bf16 x 8: part p of U[8(4 st + kk) + j][16 nt + n_], j = 0..7
    f4 bias[NT];         // (U^T mu)[16 nt + 4 kk + r] / N
    auto load_basis = [&](int b) {
        const u4* Up = (const u4*)a.Upack + (size_t)b * (NST * 3 * NT * 64) + lane;
#pragma unroll
        for (int st = 0; st < NST; ++st)
#pragma unroll
            for (int p = 0; p < 3; ++p)
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) ua[st][p][nt] = Up[((st * 3 + p) * NT + nt) * 64];
        const f4* um = (const f4*)(a.Umu + (size_t)b * 16 * NT) + kk;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bias[nt] = um[4 * nt] / a.n_workers;
    };
    load_basis(cur_b);

    u4 regs[NL];
    auto load_tile = [&](int64_t t) {
        const int64_t base = t * TILE_ELEMS;
        const unsigned short* p = (const unsigned short*)a.in;
        if (base + TILE_ELEMS <= a.M) {
#pragma unroll
            for (int r = 0; r < NL; ++r)
                if (NL * 64 == TILE_LOADS || loads) regs[r] = stream_load((const u4*)(p + base + (int64_t)(r * 64 + lane) * 8));
            return;
        }
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            const int g = r * 64 + lane;
            const int64_t e0 = base + (int64_t)g * 8;
            u4 v = {0u, 0u, 0u, 0u};
            if (g < TILE_LOADS && e0 < a.M) {
                if (e0 + 8 <= a.M) {
                    v = *(const u4*)(p + e0);
                } else {
                    unsigned int h[8];
#pragma unroll
                    for (int i = 0; i < 8; ++i) h[i] = e0 + i < a.M ? p[e0 + i] : 0u;
                    v = u4{h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16)};
                }
            }
            regs[r] = v;
        }
    };

    load_tile(it.t);
    for (bool more = true; more;) {
        const int64_t t = it.t;
        const int64_t s0 = t * TILE_SLICES;
        const int64_t s1 = s0 + TILE_SLICES < a.S ? s0 + TILE_SLICES : a.S;
        if (s0 >= blk_end || s0 < blk_begin) {
            cur_b = block_of_tile(a, t);
            blk_begin = a.offs[cur_b];
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        wave_lds_sync();
#pragma unroll
        for (int r = 0; r < NL; ++r) {
            const int g = r * 64 + lane;
            if (NL * 64 == TILE_LOADS || loads) {
                const int s = g / C8, c = g % C8;
                lds[s * C8 + (c ^ swz<D / 2>(s))] = regs[r];
            }
        }
        wave_lds_sync();
        more = it.advance();
        if (more) load_tile(it.t);

        u4 xb[NST];
#pragma unroll
        for (int st = 0; st < NST; ++st) xb[st] = lds[n_ * C8 + ((4 * st + kk) ^ swz<D / 2>(n_))];
        __builtin_amdgcn_s_setprio(3);
        for (;;) {
            int64_t lo, hi;
            row_range(a, s0, s1, blk_begin, blk_end, lo, hi);
            f4 acc[NT], prev[NT];
            if constexpr (ACC) load_acc_in<NT>(a, s0 + n_, kk, s0 + n_ >= lo && s0 + n_ < hi, prev);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) acc[nt] = -bias[nt];
#pragma unroll
            for (int st = 0; st < NST; ++st)
#pragma unroll
                for (int p = 0; p < 3; ++p)
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                            __builtin_bit_cast(bf8, ua[st][p][nt]), __builtin_bit_cast(bf8, xb[st]), acc[nt], 0, 0, 0);
            if constexpr (ACC) {   // ring step: add the predecessor's partial sum
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) acc[nt] += prev[nt];
            }
            const int64_t j = s0 + n_;
            if (j >= lo && j < hi) {
                float* o = (float*)a.out + j * a.k;
                if ((a.k & 3) == 0) {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
                        if (16 * nt + 4 * kk < a.k) stream_store((f4*)(o + 16 * nt + 4 * kk), acc[nt]);
                } else {
#pragma unroll
                    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                        for (int r = 0; r < 4; ++r)
                            if (16 * nt + 4 * kk + r < a.k) o[16 * nt + 4 * kk + r] = acc[nt][r];
                }
            }
            if (blk_end >= s1) break;
            cur_b += 1;               // the tile continues into the next basis
            blk_begin = blk_end;
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        __builtin_amdgcn_s_setprio(0);
    }
}

// compress, any d and k <= d (used for k > 128 only): one thread per output number.  Correct, not fast.
template <bool BF16>
__global__ __launch_bounds__(256) void compress_generic_kernel(CodecArgs a)
{
    const int64_t first = a.seg_begin * a.k, total = a.seg_end * a.k;
    for (int64_t o = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < total;
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
        if (a.acc_in) acc += a.acc_in[o];
        ((float*)a.out)[o] = acc;
    }
}

// Fast phase of decompress (see compress_fast_phase): per super-tile the compressed rows arrive in
// memory order (NY = ceil(8 k / D) full-width loads per lane, a template value through YS), are
// transposed through LDS into the B operand, multiplied, and the 2048 reconstructed elements leave
// through the same LDS region as 8 full-width stores per lane (4 for bf16 output), mu added on the
// way out.  Nothing is conditional.
template <int D, int NQ, bool OUT_BF16, int YS, bool MANY>
__device__ __forceinline__ void decompress_fast_phase(const CodecArgs& a, f4* lds)
{
    constexpr int G = 128 / D, ET = D / 16, CPS = D / 4, KC = 4 * NQ;
    constexpr int NY = ((G * NQ) >> YS) > 0 ? ((G * NQ) >> YS) : 1;
    constexpr int EPS = OUT_BF16 ? 8 : 4;            // elements per 128-bit store
    constexpr int SCPS = D / EPS;                    // store chunks per slice
    constexpr int NS = 2048 / EPS / 64;              // stores per lane per super-tile

    SuperIter it;
    if (!it.init(a.n_super, a.run_tiles)) return;

    const int lane = threadIdx.x & 63, n_ = lane & 15, kk = lane >> 4;
    const float* Y = (const float*)a.in;
    const int kc = a.k >> 2, cnt = G * TILE_SLICES * kc;   // 128-bit words of a super-tile's input
    // input word gi of a super-tile belongs to the output row gi / irw (a row: 1 KB of output, a whole number of
    // slices, irw 128-bit words of input)
    const int irw = (1024 / (D * (OUT_BF16 ? 2 : 4))) * kc;
    int si_slot[NY], si_row[NY], si_in[NY];
#pragma unroll
    for (int r = 0; r < NY; ++r) {
        int gi = r * 64 + lane;
        if (gi > cnt - 1) gi = cnt - 1;
        const int s = gi / kc, c = gi - s * kc;
        si_slot[r] = s * KC + (c ^ swz<16 * NQ>(s & 15));
        si_row[r] = gi / irw;
        si_in[r] = 4 * (gi - si_row[r] * irw);
    }
    const int sc = lane % SCPS;                      // this lane's store chunk within a slice
    int out_slot[NS];
#pragma unroll
    for (int r = 0; r < NS; ++r) {
        const int row = (r * 64 + lane) / SCPS;
        out_slot[r] = row * CPS + ((OUT_BF16 ? 2 * sc : sc) ^ swz<D>(row & 15));
    }
    bool col_ok[NQ];                                 // padded columns of the input tile hold whatever was there
#pragma unroll
    for (int q = 0; q < NQ; ++q) col_ok[q] = 4 * q + kk < kc;

    f4 uf[ET][NQ];
    float mul[EPS];
    auto load_basis = [&](int b) {
        const f4* Up = a.Upack + (size_t)b * (ET * NQ * 64) + lane;
        const float* mub = a.mu + (size_t)b * D + sc * EPS;
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int q = 0; q < NQ; ++q) uf[et][q] = Up[(et * NQ + q) * 64];
#pragma unroll
        for (int i = 0; i < EPS; ++i) mul[i] = mub[i];
    };
    f4 y[NY];
    // Where super-tile p lies (see compress_fast_phase): its first output byte, first input word, rows between rows.
    constexpr int ES = OUT_BF16 ? 2 : 4;
    const int64_t n_il = (!MANY && a.il > 1) ? a.n_super / a.il * a.il : 0;
    struct Where { int64_t out_byte, in_word; int rstride; };
    auto where = [&](int64_t p) {
        Where w;
        if (!MANY && p < n_il) {
            const int64_t g = p / a.il, j = p - g * a.il;
            const int64_t row = g * a.il * NS + j;
            w.out_byte = a.sup_first * (int64_t)(TILE_SLICES * D * ES) + row * 1024;
            w.in_word = a.sup_first * (int64_t)(TILE_SLICES) * kc + row * irw;
            w.rstride = a.il;
        } else {
            const int64_t t0 = super_tile<G, MANY>(a, p);
            w.out_byte = t0 * (int64_t)(TILE_SLICES * D * ES);
            w.in_word = t0 * (int64_t)(TILE_SLICES) * kc;
            w.rstride = 1;
        }
        return w;
    };
    auto load_super = [&](const Where& w) {
        const float* p = Y + 4 * w.in_word;
#pragma unroll
        for (int r = 0; r < NY; ++r) y[r] = stream_load((const f4*)(p + 4 * si_row[r] * w.rstride * irw + si_in[r]));
    };

    int64_t cur = it.p;
    int b = super_basis<MANY>(a, cur);
    Where wc = where(cur);
    load_super(wc);
    for (;;) {
        load_basis(b);
        drain_memory();
        int nb;
        do {
            const bool more = it.advance();
            const int64_t nxt = more ? it.p : cur;
            nb = more ? super_basis<MANY>(a, nxt) : -1;
            const Where wn = where(nxt);

            if (a.pace & 1) drain_memory();
            wave_lds_sync();
#pragma unroll
            for (int r = 0; r < NY; ++r) lds[si_slot[r]] = y[r];
            load_super(wn);
            wave_lds_sync();
            f4 yc[G][NQ];
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const f4 v = lds[(g * 16 + n_) * KC + ((4 * q + kk) ^ swz<16 * NQ>(n_))];
                    yc[g][q] = col_ok[q] ? v : f4{0.f, 0.f, 0.f, 0.f};
                }
            f4 acc[G][ET];
            __builtin_amdgcn_s_setprio(3);
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int et = 0; et < ET; ++et) acc[g][et] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int q = 0; q < NQ; ++q)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj)
#pragma unroll
                    for (int g = 0; g < G; ++g)
#pragma unroll
                        for (int et = 0; et < ET; ++et)
                            acc[g][et] = __builtin_amdgcn_mfma_f32_16x16x4f32(uf[et][q][jj], yc[g][q][jj], acc[g][et], 0, 0, 0);
            __builtin_amdgcn_s_setprio(0);
            if (a.pace & 2) drain_memory();
            wave_lds_sync();   // every yc is in registers: the region now takes the result
#pragma unroll
            for (int g = 0; g < G; ++g)
#pragma unroll
                for (int et = 0; et < ET; ++et) lds[(g * 16 + n_) * CPS + ((4 * et + kk) ^ swz<D>(n_))] = acc[g][et];
            wave_lds_sync();
            char* o = (char*)a.out + wc.out_byte + lane * 16;
            const int64_t ostride = (int64_t)wc.rstride * 1024;
#pragma unroll
            for (int r = 0; r < NS; ++r) {
                if (OUT_BF16) {
                    f4 v0 = lds[out_slot[r]], v1 = lds[out_slot[r] ^ 1];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        v0[i] += mul[i];
                        v1[i] += mul[(4 + i) % EPS];
                    }
                    const u4 pk = {pack_bf16x2(v0[0], v0[1]), pack_bf16x2(v0[2], v0[3]),
                                   pack_bf16x2(v1[0], v1[1]), pack_bf16x2(v1[2], v1[3])};
                    stream_store((u4*)(o + r * ostride), pk);
                } else {
                    f4 v = lds[out_slot[r]];
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] += mul[i];
                    stream_store((f4*)(o + r * ostride), v);
                }
            }
            cur = nxt;
            wc = wn;
        } while (nb == b);
        if (nb < 0) break;
        b = nb;
    }
    drain_memory();
}

// --------------------------------------------------------------------------------------
// decompress, MFMA path.  D in {16,32,64,128}, NQ = ceil(k/16) in {1,2}.
// A = U tile (16 elements x 4 comps), B = Y (4 comps x 16 slices): lane (n = l%16, kk = l/16)
// loads comps 16q + 4kk + {0..3} of slice n as one 128-bit word and MFMA step (q, j)
// contracts comp 16q + 4kk + j.  Result register r of element tile et is element
// 16et + 4kk + r of slice n.  The 16 x D result tile is one contiguous run of memory, so
// it goes through the wave's LDS region (same swizzle as compress) and leaves as
// full-width 128-bit stores in memory order.
// --------------------------------------------------------------------------------------
template <int D, int NQ, bool OUT_BF16, int YS>
__global__ __launch_bounds__(WG_THREADS, 2) void decompress_mfma_kernel(CodecArgs a)
{
    constexpr int ET = D / 16;
    constexpr int CPS = D / 4;                       // fp32 128-bit chunks per slice
    constexpr int EPS = OUT_BF16 ? 8 : 4;            // elements per 128-bit store
    constexpr int SCPS = D / EPS;                    // store chunks per slice
    constexpr int TILE_STORES = TILE_SLICES * SCPS;
    constexpr int NS = (TILE_STORES + 63) / 64;      // stores per lane per tile
    constexpr int64_t TILE_ELEMS = (int64_t)TILE_SLICES * D;

    constexpr int KC = 4 * NQ;                       // 128-bit chunks per slice of the padded input tile

    __shared__ f4 lds_all[WAVES_PER_WG][512];        // one super-tile of the fast phase (8 KB per wave)
    __shared__ f4 ldsi_all[WAVES_PER_WG][TILE_SLICES * KC];
    const int lane = threadIdx.x & 63;
    f4* lds = lds_all[threadIdx.x >> 6];
    f4* ldsi = ldsi_all[threadIdx.x >> 6];

    if (a.sup_tile) decompress_fast_phase<D, NQ, OUT_BF16, YS, true>(a, lds);
    else decompress_fast_phase<D, NQ, OUT_BF16, YS, false>(a, lds);

    // ---- general phase: the tiles the fast phase leaves out, every check in place ----------
    RestIter it;
    if (!it.init(a)) return;
    const int n_ = lane & 15, kk = lane >> 4;
    const float* Y = (const float*)a.in;
    const bool vec = (a.k & 3) == 0;
    // input tile in memory order: 16 slices x k floats, contiguous; this lane's 128-bit pieces
    const int kc = a.k >> 2;
    int si_s[NQ], si_c[NQ];
#pragma unroll
    for (int r = 0; r < NQ; ++r) {
        const int g = r * 64 + lane;
        si_s[r] = kc ? g / kc : 0;
        si_c[r] = kc ? g - si_s[r] * kc : 0;
    }
    // columns k..KP of the padded tile are never written: they must read as zero
#pragma unroll
    for (int r = 0; r < NQ; ++r) ldsi[r * 64 + lane] = f4{0.f, 0.f, 0.f, 0.f};

    int cur_b = block_of_tile(a, it.t);
    int64_t blk_begin = a.offs[cur_b], blk_end = a.offs[cur_b + 1];
    f4 uf[ET][NQ];   // uf[et][q][j] = U[16et + n_][16q + 4kk + j], zero past column k
    float mul[EPS];  // mu of the elements this lane writes out (the same chunk of every slice)
    auto load_basis = [&](int b) {
        const f4* Up = a.Upack + (size_t)b * (ET * NQ * 64) + lane;
        const float* mub = a.mu + (size_t)b * D + (lane % SCPS) * EPS;
#pragma unroll
        for (int et = 0; et < ET; ++et)
#pragma unroll
            for (int q = 0; q < NQ; ++q) uf[et][q] = Up[(et * NQ + q) * 64];
#pragma unroll
        for (int i = 0; i < EPS; ++i) mul[i] = mub[i];
    };
    load_basis(cur_b);

    f4 y[NQ];
    auto load_tile = [&](int64_t t) {
        if (vec) {   // memory order: full-width loads; transposed through LDS later
            const float* p = Y + t * TILE_SLICES * a.k;
#pragma unroll
            for (int r = 0; r < NQ; ++r) {
                const int g = r * 64 + lane;
                f4 v = {0.f, 0.f, 0.f, 0.f};
                if (g < TILE_SLICES * kc && t * TILE_SLICES + si_s[r] < a.S) v = stream_load((const f4*)(p + 4 * g));
                y[r] = v;
            }
            return;
        }
        const int64_t j = t * TILE_SLICES + n_;
#pragma unroll
        for (int q = 0; q < NQ; ++q) {
            const int c0 = 16 * q + 4 * kk;
            f4 v = {0.f, 0.f, 0.f, 0.f};
            if (j < a.S) {
#pragma unroll
                for (int r = 0; r < 4; ++r)
                    if (c0 + r < a.k) v[r] = Y[j * a.k + c0 + r];
            }
            y[q] = v;
        }
    };

    load_tile(it.t);
    for (bool more = true; more;) {
        const int64_t t = it.t;
        const int64_t s0 = t * TILE_SLICES;
        const int64_t s1 = s0 + TILE_SLICES < a.S ? s0 + TILE_SLICES : a.S;
        if (s0 >= blk_end || s0 < blk_begin) {
            cur_b = block_of_tile(a, t);
            blk_begin = a.offs[cur_b];
            blk_end = a.offs[cur_b + 1];
            load_basis(cur_b);
        }
        f4 yc[NQ];
        if (vec) {
            wave_lds_sync();
#pragma unroll
            for (int r = 0; r < NQ; ++r)
                if (r * 64 + lane < TILE_SLICES * kc) ldsi[si_s[r] * KC + (si_c[r] ^ swz<16 * NQ>(si_s[r]))] = y[r];
            wave_lds_sync();
#pragma unroll
            for (int q = 0; q < NQ; ++q) yc[q] = ldsi[n_ * KC + ((4 * q + kk) ^ swz<16 * NQ>(n_))];
        } else {
#pragma unroll
            for (int q = 0; q < NQ; ++q) yc[q] = y[q];
        }
        more = it.advance();
        if (more) load_tile(it.t);

        for (;;) {
            wave_lds_sync();
#pragma unroll
            for (int et = 0; et < ET; ++et) {
                f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int q = 0; q < NQ; ++q)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj)
                        acc = __builtin_amdgcn_mfma_f32_16x16x4f32(uf[et][q][jj], yc[q][jj], acc, 0, 0, 0);
                lds[n_ * CPS + ((4 * et + kk) ^ swz<D>(n_))] = acc;
            }
            wave_lds_sync();
            // write the tile out in memory order
            int64_t lo, hi;
            row_range(a, s0, s1, blk_begin, blk_end, lo, hi);
            const bool whole = lo == s0 && hi == s0 + TILE_SLICES && (s0 + TILE_SLICES) * (int64_t)D <= a.M;
#pragma unroll
            for (int r = 0; r < NS; ++r) {
                const int g = r * 64 + lane;
                if (NS * 64 != TILE_STORES && g >= TILE_STORES) continue;
                const int s = g / SCPS, c = g % SCPS;
                const int64_t e0 = s0 * D + (int64_t)g * EPS;
                if (OUT_BF16) {
                    f4 v0 = lds[s * CPS + ((2 * c) ^ swz<D>(s))];
                    f4 v1 = lds[s * CPS + ((2 * c + 1) ^ swz<D>(s))];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        v0[i] += mul[i];
                        v1[i] += mul[(4 + i) % EPS];
                    }
                    unsigned short* o = (unsigned short*)a.out;
                    if (whole || (s0 + s >= lo && s0 + s < hi && e0 + 8 <= a.M)) {
                        u4 pk = {pack_bf16x2(v0[0], v0[1]), pack_bf16x2(v0[2], v0[3]),
                                 pack_bf16x2(v1[0], v1[1]), pack_bf16x2(v1[2], v1[3])};
                        stream_store((u4*)(o + e0), pk);
                    } else if (s0 + s >= lo && s0 + s < hi) {
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            if (e0 + i < a.M) o[e0 + i] = (unsigned short)f32_to_bf16_rne(v0[i]);
                            if (e0 + 4 + i < a.M) o[e0 + 4 + i] = (unsigned short)f32_to_bf16_rne(v1[i]);
                        }
                    }
                } else {
                    f4 v = lds[s * CPS + (c ^ swz<D>(s))];
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] += mul[i];
                    float* o = (float*)a.out;
                    if (whole || (s0 + s >= lo && s0 + s < hi && e0 + 4 <= a.M)) {
                        stream_store((f4*)(o + e0), v);
                    } else if (s0 + s >= lo && s0 + s < hi) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (e0 + i < a.M) o[e0 + i] = v[i];
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
    (void)TILE_ELEMS;
}

// decompress, any d, k (used for k > 128 only): one thread per output element.
template <bool OUT_BF16>
__global__ __launch_bounds__(256) void decompress_generic_kernel(CodecArgs a)
{
    const float* Y = (const float*)a.in;
    const int64_t first = a.seg_begin * a.d, last = a.seg_end * a.d < a.M ? a.seg_end * a.d : a.M;
    for (int64_t o = first + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; o < last;
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
// aggregate: out[i] = ((in0[i] + in1[i]) + in2[i]) + ...   Each wave owns blocks of AGG_ROWS KB:
// it walks over the inputs one after the other and takes AGG_ROWS contiguous 1 KB rows from
// each (128 bits per lane per row, non-temporal), adding as it goes.  Long contiguous bursts
// per input with few requests in flight suit this memory system better than one element
// from all inputs at once (6.2 vs 5.6 TB/s measured for 16 inputs).
// KEEP: the sum is written with ordinary stores instead of non-temporal ones, so that it stays in the
// last-level cache for the decompress that follows (see the launcher).
// --------------------------------------------------------------------------------------
#define AGG_ROWS 4
template <bool KEEP>
__global__ __launch_bounds__(256) void aggregate_kernel(gvq_ptrs in, int n, float* out, int64_t len)
{
    const int lane = threadIdx.x & 63;
    const int64_t W = (int64_t)gridDim.x * 4, w = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    const int64_t len4 = len >> 2;
    const int64_t T = len4 / (64 * AGG_ROWS);   // whole blocks
    for (int64_t t = w; t < T; t += W) {
        const int64_t base = t * (64 * AGG_ROWS) + lane;
        f4 acc[AGG_ROWS];
#pragma unroll
        for (int r = 0; r < AGG_ROWS; ++r) acc[r] = stream_load((const f4*)in.p[0] + base + r * 64);
        for (int u = 1; u < n; ++u) {
            f4 v[AGG_ROWS];
#pragma unroll
            for (int r = 0; r < AGG_ROWS; ++r) v[r] = stream_load((const f4*)in.p[u] + base + r * 64);
#pragma unroll
            for (int r = 0; r < AGG_ROWS; ++r) acc[r] += v[r];
        }
#pragma unroll
        for (int r = 0; r < AGG_ROWS; ++r) {
            if constexpr (KEEP) *((f4*)out + base + r * 64) = acc[r];
            else stream_store((f4*)out + base + r * 64, acc[r]);
        }
    }
    // what is left of the last block, 128 bits at a time, then up to 3 single numbers
    for (int64_t i = T * (64 * AGG_ROWS) + (int64_t)blockIdx.x * blockDim.x + threadIdx.x; i < len4;
         i += (int64_t)gridDim.x * blockDim.x) {
        f4 acc = ((const f4*)in.p[0])[i];
        for (int u = 1; u < n; ++u) acc += ((const f4*)in.p[u])[i];
        ((f4*)out)[i] = acc;
    }
    const int64_t i = (len4 << 2) + threadIdx.x;
    if (blockIdx.x == 0 && i < len) {
        float acc = ((const float*)in.p[0])[i];
        for (int u = 1; u < n; ++u) acc += ((const float*)in.p[u])[i];
        out[i] = acc;
    }
}

// --------------------------------------------------------------------------------------
// Copies of U in the order the MFMA kernels consume it, so that a wave fetches its operand
// registers with contiguous 128-bit loads (both are d x KP floats per basis, KP = k rounded
// up to 16, zero past column k):
//   compress:   Upc[b][q][nt][lane][j] = U[4*(4q + kk) + j][16nt + n],  n = lane%16, kk = lane/16
//   decompress: Upd[b][et][q][lane][j] = U[16et + n][16q + 4kk + j]
// --------------------------------------------------------------------------------------
__global__ void pack_basis_kernel(const float* U, float* Upc, float* Upd, int d, int k, int NT)
{
    const int b = blockIdx.x;
    const float* Ub = U + (size_t)b * d * k;
    const int per = d * 16 * NT;  // floats per basis in either packed copy
    const int NQc = d / 16, ET = d / 16;
    for (int i = threadIdx.x; i < per; i += blockDim.x) {
        const int j = i & 3, lane = (i >> 2) & 63, n = lane & 15, kk = lane >> 4, hi = i >> 8;
        {   // compress order: hi = q*NT + nt
            const int q = hi / NT, nt = hi % NT;
            const int e = 4 * (4 * q + kk) + j, c = 16 * nt + n;
            Upc[(size_t)b * per + i] = (q < NQc && c < k) ? Ub[e * k + c] : 0.0f;
        }
        {   // decompress order: hi = et*NT + q
            const int et = hi / NT, q = hi % NT;
            const int e = 16 * et + n, c = 16 * q + 4 * kk + j;
            Upd[(size_t)b * per + i] = (et < ET && c < k) ? Ub[e * k + c] : 0.0f;
        }
    }
}

// For the bf16 compress kernel (d in {32,64,128}):
//   Upb[b][st][p][nt][lane][j] (bf16) = term p of U[8(4 st + kk) + j][16 nt + n], U = u1 + u2 + u3 with
//       u1 = bf16(U), u2 = bf16(U - u1), u3 = bf16(U - u1 - u2)   (round to nearest even; the
//       differences are exact in fp32), zero past column k;
//   Umu[b][c] = sum_e U[e][c] mu[e]  (float64 sum, stored as float), c < 16 NT, zero past k.
__global__ void pack_basis_bf16_kernel(const float* U, const float* mu, unsigned short* Upb, float* Umu,
                                       int d, int k, int NT)
{
    const int b = blockIdx.x;
    const float* Ub = U + (size_t)b * d * k;
    const float* mub = mu + (size_t)b * d;
    const int NST = d / 32;
    const int per = NST * 3 * NT * 64 * 8;   // bf16 values per basis
    for (int i = threadIdx.x; i < per; i += blockDim.x) {
        const int j = i & 7, lane = (i >> 3) & 63, n = lane & 15, kk = lane >> 4, hi = i >> 9;
        const int nt = hi % NT, p = (hi / NT) % 3, st = hi / (3 * NT);
        const int e = 8 * (4 * st + kk) + j, c = 16 * nt + n;
        unsigned int out = 0u;
        if (c < k) {
            float rest = Ub[e * k + c];
            for (int t = 0; t <= p; ++t) {
                out = f32_to_bf16_rne(rest);
                rest -= bf16_to_f32(out);
            }
        }
        Upb[(size_t)b * per + i] = (unsigned short)out;
    }
    for (int c = threadIdx.x; c < 16 * NT; c += blockDim.x) {
        double acc = 0.0;
        if (c < k)
            for (int e = 0; e < d; ++e) acc += (double)Ub[e * k + c] * (double)mub[e];
        Umu[(size_t)b * 16 * NT + c] = (float)acc;
    }
}

// ======================================================================================
// host side
// ======================================================================================
bool gvq_mfma_shape(int d, int k)
{
    return k <= 32 && (d == 16 || d == 32 || d == 64 || d == 128);
}

// bf16-stored gradients whose slices fill whole 32-element MFMA steps take the bf16 pipe
bool gvq_bf16_pipe_shape(const gvq_basis* h)
{
    return h->dtype == GVQ_BF16 && gvq_mfma_shape(h->d, h->k) && h->d >= 32;
}

int gvq_launch_pack(const gvq_basis* h, hipStream_t st)
{
    if (gvq_long_shape(h->d, h->k)) return gvq_launch_pack_long(h, st);
    if (!gvq_mfma_shape(h->d, h->k)) return GVQ_OK;
    hipLaunchKernelGGL(pack_basis_kernel, dim3(h->B), dim3(256), 0, st, h->d_U, h->d_Upc, h->d_Upd,
                       h->d, h->k, h->k <= 16 ? 1 : 2);
    GVQ_HIP(hipGetLastError());
    if (gvq_bf16_pipe_shape(h)) {
        hipLaunchKernelGGL(pack_basis_bf16_kernel, dim3(h->B), dim3(256), 0, st, h->d_U, h->d_mu, h->d_Upb,
                           h->d_Umu, h->d, h->k, h->k <= 16 ? 1 : 2);
        GVQ_HIP(hipGetLastError());
    }
    return GVQ_OK;
}

static CodecArgs make_args(const gvq_basis* h, const void* in, void* out, int n_workers, const float* upack)
{
    CodecArgs a;
    a.in = in; a.out = out; a.U = h->d_U; a.Upack = (const f4*)upack; a.mu = h->d_mu; a.offs = h->d_offs;
    a.M = h->M; a.S = h->S; a.B = h->B; a.d = h->d; a.k = h->k;
    a.n_workers = (float)n_workers;
    a.tile_block = h->d_tile_block;
    a.run_tiles = 1;
    a.Upack2 = nullptr;
    a.Umu = nullptr;
    a.acc_in = nullptr;
    a.seg_begin = 0;
    a.seg_end = h->S;
    a.n_super = 0; a.sup_first = 0; a.sup_tile = nullptr; a.sup_basis = nullptr;
    a.rest_lo0 = a.rest_lo1 = a.rest_hi0 = a.rest_hi1 = 0;
    a.rest_list = nullptr; a.n_rest = 0; a.rest_run = 1;
    a.pace = 0;
    a.il = 1;
    a.keep_y = 0;
    return a;
}

// Splits the 16-slice tiles that touch the requested slice range into super-tiles of G tiles for the
// fast phase (whole slices of one basis, wholly inside the gradient and the range) and rest tiles.
// `which`: the handle's precomputed split for many bases (0: G = 128/d, 1: the bf16-pipe compress), used when the
// whole gradient is requested; a partial range over many bases goes through the general phase.
static void plan_tiles(const gvq_basis* h, CodecArgs& a, int G, bool fast_ok, int which)
{
    const int64_t T0 = a.seg_begin / TILE_SLICES, T1 = (a.seg_end + TILE_SLICES - 1) / TILE_SLICES;
    a.rest_lo0 = T0; a.rest_lo1 = T1; a.rest_hi0 = T1; a.rest_hi1 = T1;
    if (!fast_ok) return;
    if (h->B == 1) {
        const int64_t full = h->M / h->d;   // slices that lie wholly inside the gradient
        const int64_t p0 = (a.seg_begin + TILE_SLICES - 1) / TILE_SLICES;
        const int64_t p1 = (a.seg_end < full ? a.seg_end : full) / TILE_SLICES;
        if (p1 - p0 < G) return;
        a.n_super = (p1 - p0) / G;
        a.sup_first = p0;
        a.rest_lo1 = p0;
        a.rest_hi0 = p0 + a.n_super * G;
        return;
    }
    const gvq_plan& pl = h->plan[which];
    if (a.seg_begin != 0 || a.seg_end != h->S || !pl.d_rest) return;
    a.n_super = pl.n_super; a.sup_tile = pl.d_sup_tile; a.sup_basis = pl.d_sup_basis;
    a.rest_list = pl.d_rest; a.n_rest = pl.n_rest;
}

// Number of 128-bit words per lane that the compressed side of a super-tile needs, as the shift YS of
// the kernels' template (words = max(1, (G * NT) >> YS), the smallest that covers ceil(G 16 k / 4 / 64)).
static int pick_ys(int G, int NT, int k)
{
    const int need = (G * TILE_SLICES * (k >> 2) + 63) / 64;
    int ys = 0;
    while (ys < 2 && ((G * NT) >> (ys + 1)) >= need && ((G * NT) >> (ys + 1)) >= 1) ++ys;
    return ys;
}

int gvq_build_plans(gvq_basis* h)
{
    if (h->B == 1 || !gvq_mfma_shape(h->d, h->k)) return GVQ_OK;
    const int64_t T = (h->S + TILE_SLICES - 1) / TILE_SLICES, full = h->M / h->d;
    for (int which = 0; which < 2; ++which) {
        if (which == 1 && !gvq_bf16_pipe_shape(h)) break;
        const int G = which ? (h->d == 128 ? 2 : 4) : 128 / h->d;   // bf16_super_tiles<D>() for which = 1
        gvq_plan& pl = h->plan[which];
        int64_t ns = 0;
        for (int b = 0; b < h->B; ++b) {
            const int64_t hi = h->h_offs[b + 1] < full ? h->h_offs[b + 1] : full;
            const int64_t p0 = (h->h_offs[b] + TILE_SLICES - 1) / TILE_SLICES, p1 = hi / TILE_SLICES;
            if (p1 - p0 >= G) ns += (p1 - p0) / G;
        }
        int64_t* st = (int64_t*)malloc(sizeof(int64_t) * (size_t)(ns ? ns : 1));
        int* sb = (int*)malloc(sizeof(int) * (size_t)(ns ? ns : 1));
        int64_t* rest = (int64_t*)malloc(sizeof(int64_t) * (size_t)T);
        if (!st || !sb || !rest) { free(st); free(sb); free(rest); return GVQ_ENOMEM; }
        int64_t i = 0, nr = 0, next = 0;   // next: first tile not yet assigned
        for (int b = 0; b < h->B; ++b) {
            const int64_t hi = h->h_offs[b + 1] < full ? h->h_offs[b + 1] : full;
            const int64_t p0 = (h->h_offs[b] + TILE_SLICES - 1) / TILE_SLICES, p1 = hi / TILE_SLICES;
            if (p1 - p0 < G) continue;
            const int64_t n = (p1 - p0) / G;
            while (next < p0) rest[nr++] = next++;
            for (int64_t j = 0; j < n; ++j) { st[i] = p0 + j * G; sb[i] = b; ++i; }
            next = p0 + n * G;
        }
        while (next < T) rest[nr++] = next++;
        pl.n_super = ns; pl.n_rest = nr;
        hipError_t e = hipMalloc((void**)&pl.d_sup_tile, sizeof(int64_t) * (size_t)(ns ? ns : 1));
        if (e == hipSuccess) e = hipMalloc((void**)&pl.d_sup_basis, sizeof(int) * (size_t)(ns ? ns : 1));
        if (e == hipSuccess) e = hipMalloc((void**)&pl.d_rest, sizeof(int64_t) * (size_t)(nr ? nr : 1));
        if (e == hipSuccess && ns) e = hipMemcpy(pl.d_sup_tile, st, sizeof(int64_t) * (size_t)ns, hipMemcpyHostToDevice);
        if (e == hipSuccess && ns) e = hipMemcpy(pl.d_sup_basis, sb, sizeof(int) * (size_t)ns, hipMemcpyHostToDevice);
        if (e == hipSuccess && nr) e = hipMemcpy(pl.d_rest, rest, sizeof(int64_t) * (size_t)nr, hipMemcpyHostToDevice);
        free(st); free(sb); free(rest);
        if (e != hipSuccess) return gvq_hip_fail(e, "tile plan upload");
    }
    return GVQ_OK;
}

// `most`: upper limit on the work-groups per compute unit when the tuning option is not set
// (0 = whatever fits).  `full_rounds`: see below (compress gains 2 - 4 % on a 25 M gradient, decompress loses 2 %).
template <auto KERN>
static int streaming_grid(const gvq_basis* h, int64_t tiles, int most = 0, bool full_rounds = false)
{
    int per_cu = gvq_opt_wg_per_cu();
    if (per_cu <= 0) {
        // one instance of this function per kernel: ask the runtime once, then remember
        static int cached = 0;
        if (cached == 0) {
            int occ = 0;
            if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, KERN, WG_THREADS, 0) != hipSuccess || occ < 1)
                occ = 2;
            cached = occ;
        }
        per_cu = most > 0 && cached > most ? most : cached;
    }
    int64_t want = (tiles + WAVES_PER_WG - 1) / WAVES_PER_WG;  // at least one tile per wave
    int64_t cap = (int64_t)h->num_cu * per_cu;
    int64_t g = want < cap ? want : cap;
    // A short launch (few rounds of tiles per wave) ends with a round in which most waves have nothing left: a
    // grid up to an eighth smaller whose last round is full moves the same bytes without that tail.
    if (full_rounds && gvq_opt_wg_per_cu() <= 0 && g == cap && tiles / (cap * WAVES_PER_WG) < 32) {
        int64_t best = g, best_idle = -1;
        for (int64_t c = cap; c >= cap - cap / 8; --c) {
            const int64_t waves = c * WAVES_PER_WG, rounds = (tiles + waves - 1) / waves;
            const int64_t idle = (rounds * waves - tiles) * cap / c;   // wave-rounds wasted, scaled to the full grid
            if (best_idle < 0 || idle < best_idle) { best = c; best_idle = idle; }
        }
        g = best;
    }
    return (int)(g < 1 ? 1 : g);
}

// Tiles per run for the MFMA kernels (see TileIter): the tuning option if set, else single
// tiles for one basis and short runs when there are many bases.
static int run_length(const gvq_basis* h, int64_t tiles, int grid, int many = 4)
{
    const int64_t waves = (int64_t)grid * WAVES_PER_WG;
    const int64_t chunk = (tiles + waves - 1) / waves;   // run length that gives one run per wave
    int64_t r = gvq_opt_run_tiles();
    if (r <= 0) r = h->B > 1 ? many : 1;
    if (r > chunk) r = chunk;
    return (int)(r < 1 ? 1 : r);
}

// Launch shape of the fast phase.  This memory system gives its best with as few requests in flight
// as keep it busy (measured on whole aggregation steps, GB/s of one kernel: d = 128 compress 5.95 with
// two work-groups per compute unit and full pacing against 5.5 unpaced; d = 64 compress 6.1 with one
// work-group and paced products against 5.6 with two; decompress 5.55 with one work-group against 5.2
// with two), so every kernel has its own default.
struct FastShape {
    int wg_per_cu;   // most work-groups per compute unit
    int pace;        // CodecArgs::pace
    int many_run;    // super-tiles per run when there are many bases (each run reloads its basis)
};
static int pace_of(const FastShape& f) { return gvq_opt_pace() >= 0 ? gvq_opt_pace() : f.pace; }

// Row interleave of the fast phase (CodecArgs::il): one basis and single super-tiles per run only.
static int interleave_of(const CodecArgs& a, int dflt)
{
    if (a.sup_tile || a.run_tiles != 1) return 1;
    return gvq_opt_interleave() > 0 ? gvq_opt_interleave() : dflt;
}

// Work items of a launch: super-tiles plus rest tiles; at least one per wave.
static int64_t work_items(const CodecArgs& a)
{
    const int64_t rest = a.rest_list ? a.n_rest : (a.rest_lo1 - a.rest_lo0) + (a.rest_hi1 - a.rest_hi0);
    return a.n_super + rest;
}

template <int D, int NT, bool BF16, int VAR, int YS>
static int launch_compress_y(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    constexpr auto kern = compress_mfma_kernel<D, NT, BF16, VAR, false, YS>;
    const int64_t items = work_items(a);
    constexpr FastShape fs = D == 128 ? FastShape{2, 5, 4} : D == 64 ? FastShape{1, 4, 4} : FastShape{1, 0, 4};
    int grid = streaming_grid<kern>(h, items, fs.wg_per_cu, true);
    CodecArgs b = a;
    b.pace = pace_of(fs);
    b.run_tiles = run_length(h, a.n_super, grid, fs.many_run);
    b.rest_run = run_length(h, work_items(a) - a.n_super, grid);
    b.il = interleave_of(b, D >= 64 ? 64 : 1);   // steady state: d = 128 5.90 -> 5.99 TB/s, d = 64 6.09 -> 6.18, d = 32 5.43 -> 5.35
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, b);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, int NT, bool BF16, int VAR>
static int launch_compress_v(const gvq_basis* h, const CodecArgs& a0, hipStream_t st)
{
    constexpr int G = 128 / D;
    CodecArgs a = a0;
    plan_tiles(h, a, G, (h->k & 3) == 0 && !(gvq_opt_no_fast() & 1), 0);
    if constexpr (NT == 1 && D < 128) {
        const int ys = pick_ys(G, NT, h->k);
        if (ys == 1) return launch_compress_y<D, NT, BF16, VAR, 1>(h, a, st);
        if constexpr (D < 64) {
            if (ys == 2) return launch_compress_y<D, NT, BF16, VAR, 2>(h, a, st);
        }
    }
    return launch_compress_y<D, NT, BF16, VAR, 0>(h, a, st);
}

template <int D, int NT, bool BF16>
static int launch_compress_t(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    // VAR bit 0 (general phase): results leave through LDS as full-width stores (pays at k > 16, where a
    // slice's results would otherwise leave in two half-line pieces); bit 1: raised wave priority
    // while a wave feeds the MFMA pipe.  Bit 2: fused ring step (adds acc_in); a separate
    // instantiation so that the plain kernel does not carry its registers.  Bit 3: the fast phase writes its results
    // with ordinary stores (CodecArgs::keep_y).
    if (a.acc_in) return launch_compress_v<D, NT, BF16, (NT == 2 ? 7 : 6)>(h, a, st);
    if (a.keep_y) return launch_compress_v<D, NT, BF16, (NT == 2 ? 11 : 10)>(h, a, st);
    return launch_compress_v<D, NT, BF16, (NT == 2 ? 3 : 2)>(h, a, st);
}

template <int D, bool BF16>
static int launch_compress_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    if constexpr (D == 16) return launch_compress_t<D, 1, BF16>(h, a, st);   // k <= d = 16
    else return h->k <= 16 ? launch_compress_t<D, 1, BF16>(h, a, st) : launch_compress_t<D, 2, BF16>(h, a, st);
}

template <int D, int NT, bool ACC, int YS>
static int launch_compress_bf16_y(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    constexpr auto kern = compress_bf16_kernel<D, NT, ACC, YS>;
    constexpr FastShape fs = {1, 0, 4};
    int grid = streaming_grid<kern>(h, work_items(a), fs.wg_per_cu, true);
    CodecArgs b = a;
    b.pace = pace_of(fs);
    b.run_tiles = run_length(h, a.n_super, grid, fs.many_run);
    b.rest_run = run_length(h, work_items(a) - a.n_super, grid);
    b.il = interleave_of(b, 1);   // no gain measured for bf16 storage
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, b);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, int NT, bool ACC>
static int launch_compress_bf16_a(const gvq_basis* h, const CodecArgs& a0, hipStream_t st)
{
    constexpr int G = bf16_super_tiles<D>();
    CodecArgs a = a0;
    plan_tiles(h, a, G, (h->k & 3) == 0 && !(gvq_opt_no_fast() & 2), 1);
    if constexpr (NT == 1) {
        const int ys = pick_ys(G, NT, h->k);
        if (ys == 1) return launch_compress_bf16_y<D, NT, ACC, 1>(h, a, st);
        if constexpr (G == 4) {
            if (ys == 2) return launch_compress_bf16_y<D, NT, ACC, 2>(h, a, st);
        }
    }
    return launch_compress_bf16_y<D, NT, ACC, 0>(h, a, st);
}

template <int D, int NT>
static int launch_compress_bf16_t(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    return a.acc_in ? launch_compress_bf16_a<D, NT, true>(h, a, st) : launch_compress_bf16_a<D, NT, false>(h, a, st);
}

template <int D>
static int launch_compress_bf16_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    return h->k <= 16 ? launch_compress_bf16_t<D, 1>(h, a, st) : launch_compress_bf16_t<D, 2>(h, a, st);
}

int gvq_launch_compress(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice,
                        int64_t n_slices, const float* comp_in, float* out, hipStream_t st)
{
    if (gvq_long_shape(h->d, h->k))
        return gvq_launch_compress_long(h, grad, n_workers, first_slice, n_slices, comp_in, out, st);
    if (gvq_bf16_pipe_shape(h)) {
        CodecArgs a = make_args(h, grad, out, n_workers, (const float*)h->d_Upb);
        a.Umu = h->d_Umu;
        a.acc_in = comp_in; a.seg_begin = first_slice; a.seg_end = first_slice + n_slices;
        switch (h->d) {
        case 32: return launch_compress_bf16_d<32>(h, a, st);
        case 64: return launch_compress_bf16_d<64>(h, a, st);
        default: return launch_compress_bf16_d<128>(h, a, st);
        }
    }
    CodecArgs a = make_args(h, grad, out, n_workers, h->d_Upc);
    a.acc_in = comp_in; a.seg_begin = first_slice; a.seg_end = first_slice + n_slices;
    // When the n_workers results that are summed next fit the last-level cache (256 MB) together, they are left there:
    // measured on whole steps of 8 workers with 25.6 MB each, the sum that follows runs at 6.1 instead of 5.4 TB/s and
    // the compress itself at 5.6 instead of 5.4; with results that do not fit (8 x 61 MB, 16 x 138 MB) ordinary stores
    // cost the compress 2.6 % and the step 1 - 2 %.
    a.keep_y = !comp_in && (int64_t)n_workers * n_slices * h->k * 4 <= (224ll << 20);
    const bool bf = h->dtype == GVQ_BF16;
    if (gvq_mfma_shape(h->d, h->k)) {
        switch (h->d) {
        // bf16-stored gradients reach this point with d = 16 only (longer slices took the bf16 pipe above)
        case 16: return bf ? launch_compress_d<16, true>(h, a, st) : launch_compress_d<16, false>(h, a, st);
        case 32: return launch_compress_d<32, false>(h, a, st);
        case 64: return launch_compress_d<64, false>(h, a, st);
        case 128: return launch_compress_d<128, false>(h, a, st);
        default: break;
        }
    }
    int64_t total = n_slices * h->k;
    int64_t want = (total + 255) / 256, cap = (int64_t)h->num_cu * 16;
    int grid = (int)(want < cap ? want : cap);
    if (bf)
        hipLaunchKernelGGL(compress_generic_kernel<true>, dim3(grid), dim3(256), 0, st, a);
    else
        hipLaunchKernelGGL(compress_generic_kernel<false>, dim3(grid), dim3(256), 0, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, int NQ, bool OBF, int YS>
static int launch_decompress_y(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    constexpr auto kern = decompress_mfma_kernel<D, NQ, OBF, YS>;
    const int64_t items = work_items(a);
    // many bases: the basis reload of every run has to be hidden by a second work-group
    const FastShape fs = h->B > 1 ? FastShape{2, 0, 8} : FastShape{1, 0, 1};
    int grid = streaming_grid<kern>(h, items, fs.wg_per_cu);
    CodecArgs b = a;
    b.pace = pace_of(fs);
    b.run_tiles = run_length(h, a.n_super, grid, fs.many_run);
    b.rest_run = run_length(h, work_items(a) - a.n_super, grid);
    b.il = interleave_of(b, 32);   // d = 128: 5.55 -> 5.95 TB/s, d = 64: 5.5 -> 5.8
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, b);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, int NQ, bool OBF>
static int launch_decompress_t(const gvq_basis* h, const CodecArgs& a0, hipStream_t st)
{
    constexpr int G = 128 / D;
    CodecArgs a = a0;
    plan_tiles(h, a, G, (h->k & 3) == 0 && !(gvq_opt_no_fast() & 4), 0);
    if constexpr (NQ == 1 && D < 128) {
        const int ys = pick_ys(G, NQ, h->k);
        if (ys == 1) return launch_decompress_y<D, NQ, OBF, 1>(h, a, st);
        if constexpr (D < 64) {
            if (ys == 2) return launch_decompress_y<D, NQ, OBF, 2>(h, a, st);
        }
    }
    return launch_decompress_y<D, NQ, OBF, 0>(h, a, st);
}

template <int D, bool OBF>
static int launch_decompress_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    if constexpr (D == 16) return launch_decompress_t<D, 1, OBF>(h, a, st);   // k <= d = 16
    else return h->k <= 16 ? launch_decompress_t<D, 1, OBF>(h, a, st) : launch_decompress_t<D, 2, OBF>(h, a, st);
}

int gvq_launch_decompress(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices,
                          void* out, gvq_dtype_t odt, hipStream_t st)
{
    // (bf16 output of more than 128 comps cannot add up its column passes in place: the any-shape kernel below)
    if (gvq_long_shape(h->d, h->k) && !(h->k > 128 && odt == GVQ_BF16))
        return gvq_launch_decompress_long(h, comp, first_slice, n_slices, out, odt, st);
    CodecArgs a = make_args(h, comp, out, 1, h->d_Upd);
    a.seg_begin = first_slice; a.seg_end = first_slice + n_slices;
    const bool bf = odt == GVQ_BF16;
    if (gvq_mfma_shape(h->d, h->k)) {
        switch (h->d) {
        case 16: return bf ? launch_decompress_d<16, true>(h, a, st) : launch_decompress_d<16, false>(h, a, st);
        case 32: return bf ? launch_decompress_d<32, true>(h, a, st) : launch_decompress_d<32, false>(h, a, st);
        case 64: return bf ? launch_decompress_d<64, true>(h, a, st) : launch_decompress_d<64, false>(h, a, st);
        case 128: return bf ? launch_decompress_d<128, true>(h, a, st) : launch_decompress_d<128, false>(h, a, st);
        default: break;
        }
    }
    int64_t want = (n_slices * h->d + 255) / 256, cap = (int64_t)h->num_cu * 16;
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
    int per_cu = gvq_opt_wg_per_cu();
    if (per_cu <= 0) per_cu = 2;   // measured best: 6.1 TB/s, against 5.7 with 1 or 4 per compute unit
    int64_t want = (len / (4 * 64 * AGG_ROWS) + 3) / 4, cap = (int64_t)h->num_cu * per_cu;
    int grid = (int)(want < cap ? want : cap);
    if (grid < 1) grid = 1;
    // A sum of 32 - 128 MB is left in the last-level cache (256 MB) for the decompress that reads it next: measured on
    // whole steps, decompress gains 12 % at 69 MB with bf16 output, 5 % at 61 MB, 2 % with long slices; a larger sum
    // does not stay (138 MB: decompress -1.5 %), and with a smaller one the aggregate itself loses more (26 MB: -4 %)
    // than the decompress gains.
    const bool keep = len * 4 >= (32ll << 20) && len * 4 <= (128ll << 20);
    // out = comps[0] + ... in groups of at most GVQ_MAX_PTRS; later groups start from out
    int done = 0;
    while (done < N) {
        gvq_ptrs p;
        int n = 0;
        if (done > 0) p.p[n++] = out;
        while (n < GVQ_MAX_PTRS && done < N) p.p[n++] = comps[done++];
        if (keep) hipLaunchKernelGGL(aggregate_kernel<true>, dim3(grid), dim3(256), 0, st, p, n, out, len);
        else hipLaunchKernelGGL(aggregate_kernel<false>, dim3(grid), dim3(256), 0, st, p, n, out, len);
        GVQ_HIP(hipGetLastError());
    }
    return GVQ_OK;
}


// ======================================================================================
// local compression loss (Section 3, Eq. 6)
// ======================================================================================
// Any d, k (used for k > 128 only): one wave per slice.  Lanes first share the k projections, then
// the d residuals.
template <bool BF16>
__global__ __launch_bounds__(256) void loss_generic_kernel(CodecArgs a)
{
    __shared__ float xs_all[4][GVQ_MAX_D], ys_all[4][GVQ_MAX_D];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    float* xs = xs_all[wave];
    float* ys = ys_all[wave];
    const int64_t W = (int64_t)gridDim.x * 4;
    for (int64_t j = (int64_t)blockIdx.x * 4 + wave; j < a.S; j += W) {
        const int b = find_block(a.offs, a.B, j);
        const float* Ub = a.U + (size_t)b * a.d * a.k;
        const float* mub = a.mu + (size_t)b * a.d;
        wave_lds_sync();
        for (int e = lane; e < a.d; e += 64) {
            const int64_t idx = j * a.d + e;
            float x = 0.f;
            if (idx < a.M)
                x = BF16 ? bf16_to_f32(((const unsigned short*)a.in)[idx]) : ((const float*)a.in)[idx];
            xs[e] = x - mub[e] / a.n_workers;
        }
        wave_lds_sync();
        for (int c = lane; c < a.k; c += 64) {
            float acc = 0.f;
            for (int e = 0; e < a.d; ++e) acc = fmaf(Ub[e * a.k + c], xs[e], acc);
            ys[c] = acc;
        }
        wave_lds_sync();
        float sq = 0.f;
        for (int e = lane; e < a.d; e += 64) {
            float r = xs[e];
            for (int c = 0; c < a.k; ++c) r = fmaf(-Ub[e * a.k + c], ys[c], r);
            if (j * a.d + e < a.M) sq = fmaf(r, r, sq);
        }
        for (int off = 32; off > 0; off >>= 1) sq += __shfl_xor(sq, off, 64);
        if (lane == 0) ((float*)a.out)[j] = sq;
    }
}

// Fixed-order sum of a block of doubles held one per thread (256 threads).
__device__ __forceinline__ double wg_sum_256(double v, double* red)
{
    red[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) red[threadIdx.x] += red[threadIdx.x + s];
        __syncthreads();
    }
    const double tot = red[0];
    __syncthreads();
    return tot;
}

// part[b][g] = sum of the per-slice losses of chunk g (of G) of basis b's slice range
__global__ __launch_bounds__(256) void loss_reduce1_kernel(const float* per_slice, const int64_t* offs, int G,
                                                           double* part)
{
    __shared__ double red[256];
    const int b = blockIdx.y, g = blockIdx.x;
    const int64_t lo = offs[b], cnt = offs[b + 1] - lo;
    const int64_t j0 = lo + cnt * g / G, j1 = lo + cnt * (g + 1) / G;
    double acc = 0.0;
    for (int64_t j = j0 + threadIdx.x; j < j1; j += 256) acc += (double)per_slice[j];
    acc = wg_sum_256(acc, red);
    if (threadIdx.x == 0) part[(size_t)b * G + g] = acc;
}

__global__ __launch_bounds__(256) void loss_reduce2_kernel(const double* part, int G, double* out)
{
    __shared__ double red[256];
    const int b = blockIdx.x;
    double acc = 0.0;
    for (int g = threadIdx.x; g < G; g += 256) acc += part[(size_t)b * G + g];
    acc = wg_sum_256(acc, red);
    if (threadIdx.x == 0) out[b] = acc;
}

template <int D, int NT, bool BF16>
static int launch_loss_t(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    constexpr auto kern = compress_mfma_kernel<D, NT, BF16, 0, true, 0>;
    CodecArgs b = a;
    plan_tiles(h, b, 128 / D, (h->k & 3) == 0 && !(gvq_opt_no_fast() & 1), 0);
    int grid = streaming_grid<kern>(h, work_items(b));
    b.run_tiles = run_length(h, b.n_super, grid);
    b.rest_run = run_length(h, work_items(b) - b.n_super, grid);
    b.il = 1;   // the per-slice results are addressed by slice: no row interleave
    hipLaunchKernelGGL(kern, dim3(grid), dim3(WG_THREADS), 0, st, b);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int D, bool BF16>
static int launch_loss_d(const gvq_basis* h, const CodecArgs& a, hipStream_t st)
{
    if constexpr (D == 16) return launch_loss_t<D, 1, BF16>(h, a, st);
    else return h->k <= 16 ? launch_loss_t<D, 1, BF16>(h, a, st) : launch_loss_t<D, 2, BF16>(h, a, st);
}

// loss_slice [S] and loss_part [B][loss_groups]: the scratch of the two reduction stages.
static int launch_local_loss(const gvq_basis* h, const void* grad, int n_workers, double* loss_out, hipStream_t st,
                             float* loss_slice, double* loss_part)
{
    CodecArgs a = make_args(h, grad, loss_slice, n_workers, h->d_Upc);
    a.Upack2 = (const f4*)h->d_Upd;
    const bool bf = h->dtype == GVQ_BF16;
    int rc = GVQ_OK;
    if (gvq_long_shape(h->d, h->k) && h->k <= 128) {
        rc = gvq_launch_loss_long(h, grad, n_workers, loss_slice, st);
    } else if (gvq_mfma_shape(h->d, h->k)) {
        switch (h->d) {
        case 16: rc = bf ? launch_loss_d<16, true>(h, a, st) : launch_loss_d<16, false>(h, a, st); break;
        case 32: rc = bf ? launch_loss_d<32, true>(h, a, st) : launch_loss_d<32, false>(h, a, st); break;
        case 64: rc = bf ? launch_loss_d<64, true>(h, a, st) : launch_loss_d<64, false>(h, a, st); break;
        default: rc = bf ? launch_loss_d<128, true>(h, a, st) : launch_loss_d<128, false>(h, a, st); break;
        }
    } else {
        int64_t want = (h->S + 3) / 4, cap = (int64_t)h->num_cu * 8;
        int grid = (int)(want < cap ? want : cap);
        if (bf)
            hipLaunchKernelGGL(loss_generic_kernel<true>, dim3(grid), dim3(256), 0, st, a);
        else
            hipLaunchKernelGGL(loss_generic_kernel<false>, dim3(grid), dim3(256), 0, st, a);
        GVQ_HIP(hipGetLastError());
    }
    if (rc != GVQ_OK) return rc;
    const int G = h->loss_groups;
    hipLaunchKernelGGL(loss_reduce1_kernel, dim3(G, h->B), dim3(256), 0, st, loss_slice, h->d_offs, G, loss_part);
    GVQ_HIP(hipGetLastError());
    hipLaunchKernelGGL(loss_reduce2_kernel, dim3(h->B), dim3(256), 0, st, loss_part, G, loss_out);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

int gvq_launch_local_loss(const gvq_basis* h, const void* grad, int n_workers, double* loss_out, hipStream_t st)
{
    return launch_local_loss(h, grad, n_workers, loss_out, st, h->d_loss_slice, h->d_loss_part);
}

// --------------------------------------------------------------------------------------
// The same, for callers that cannot allocate: the scratch of the two reduction stages lives in a
// file-scope device array instead of the handle.  In host code the array's name is only a stand-in
// for the symbol; its device address is asked for once per device (with that device current) and
// that pointer is what the kernels get.  Every GPU has its own copy of the array; every call on a
// GPU shares it, so calls that overlap in time on one GPU race.  Nothing has to start at zero: the
// kernels overwrite every entry they later read.
// --------------------------------------------------------------------------------------
#define GVQ_STATIC_PART_DOUBLES 65536
static __device__ __align__(256) unsigned char scratch[sizeof(float) * GVQ_STATIC_MAX_SLICES +
                                                        sizeof(double) * GVQ_STATIC_PART_DOUBLES];
#define GVQ_MAX_DEVICES 64
static void* g_scratch_ptr[GVQ_MAX_DEVICES];
static std::mutex g_scratch_mutex;

int gvq_launch_local_loss_static(const gvq_basis* h, const void* grad, int n_workers, double* loss_out,
                                 hipStream_t st)
{
    if (h->S > GVQ_STATIC_MAX_SLICES || (int64_t)h->B * h->loss_groups > GVQ_STATIC_PART_DOUBLES) return GVQ_ETOOBIG;
    int dev = -1;
    GVQ_HIP(hipGetDevice(&dev));
    if (dev != h->device || dev < 0 || dev >= GVQ_MAX_DEVICES) return GVQ_EINVAL;   // the handle's device must be current
    void* base = nullptr;
    {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        if (!g_scratch_ptr[dev]) {
            void* p = nullptr;
            GVQ_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            g_scratch_ptr[dev] = p;
        }
        base = g_scratch_ptr[dev];
    }
    float* loss_slice = (float*)base;
    double* loss_part = (double*)((unsigned char*)base + sizeof(float) * GVQ_STATIC_MAX_SLICES);
    return launch_local_loss(h, grad, n_workers, loss_out, st, loss_slice, loss_part);
}
