// Basis-stationary kernels for long slices (Section 3, "slice size": d = 768 in the paper's example):
// Eq. (2), y = U^T (x - mu/N), first; Eq. (4) further down.  Products on the bf16 matrix pipe (two-term split) or,
// EXACT, on the fp32 one; fp32 or bf16 storage.
//
// The LDS-tiled kernels of gvq_codec_long.hip stream U through LDS once per 128-slice tile and walk over the
// gradient in 256-byte strips of 128 rows.  Here the roles are swapped.  A compute unit's register files hold
// 512 KB, more than the two-term bf16 copy of a whole basis (4dk bytes: 288 KB at d = 768, k = 96), so one
// work-group of 8 waves per compute unit keeps U in registers for the whole launch, an eighth of the slice's
// elements per wave (all column tiles), and the gradient streams past it in tiles of 16 whole slices, each tile
// one contiguous run of 64d bytes: the memory system sees a plain sequential stream and U costs no traffic after
// the first microseconds.  A tile's 16 x d floats are copied global -> LDS by the load unit itself
// (global_load_lds: no registers in between, up to two tiles in flight while one is worked on); a wave reads its
// strip in B-operand order, centres and splits it, and accumulates the 16 x k partial products of its strip; the
// 8 partial results meet in LDS, each in the strip of the tile that its wave alone reads, and are added.
//
// Products as in the split kernels: a = a1 + a2 in bf16, x u = x1 u1 + x1 u2 + x2 u1 with fp32 accumulation on
// v_mfma_f32_16x16x32_bf16.  Shapes: one basis, d a multiple of 256, k of 4, and the limits of gvq_ws_shape.  The slices after the last whole 16-slice tile of a range (and the slice that ends past the gradient's
// end) are one more tile, fetched with bounds-checked loads by one work-group: a second launch for them would cost a
// fifth of the whole kernel's time (one work-group of the LDS-tiled kernel walking through all of U: 33 us).
// Eq. (4) has a kernel of the same kind further down (decompress_ws_kernel): there a wave owns an eighth of the
// slice's elements for all comps, nothing has to be added up, and what matters is how the 16 x d results leave.
#include "gvq_internal.h"

#include <type_traits>

#include "gvq_device.h"

typedef unsigned int u2 __attribute__((ext_vector_type(2)));

struct WsArgs {
    const void* in;          // gradient
    void* out;               // y
    const float* acc_in;     // partial sum of the ring step to add, or null
    const u4* Upack;         // the operand-order copy of U (layout at the pack kernel)
    const float* mu;         // [d]
    int64_t first;           // first slice
    int64_t ntiles;          // whole 16-slice tiles inside the gradient
    int64_t M;               // elements of the gradient
    int tail_rows;           // slices after the last whole tile (0 .. 16; the last one may end past M)
    int d, k;
    float n_workers;
};

#define WS_WAVES 8
#define WS_ROWPAD 4          // floats between LDS rows of the x tile: 16 lanes x 128 bits then cover all banks

// 1 KB, 16 bytes per lane, global -> LDS without passing through registers.  lds_off: wave-uniform
// byte offset of the first lane's bytes inside the work-group's LDS.  Written as inline assembly so
// that the compiler does not pair the copy with the LDS reads of the *other* buffer (it would wait
// for the copy before every such read).
// (m0 carries the LDS offset and is named as clobbered on purpose; the compiler remarks on every instance that m0 is
// a reserved register, which it sets itself right before each of its own uses.)
#pragma clang diagnostic push
#pragma clang diagnostic ignored "-Winline-asm"
__device__ __forceinline__ void copy_1k_to_lds(const void* src_lane, unsigned int lds_off)
{
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(src_lane), "s"(lds_off)
                 : "memory", "m0");
}
#pragma clang diagnostic pop

// 128 bits global -> registers that the compiler does not count either (it would wait for every copy in flight before
// the first use): the caller waits by hand and then passes the value through claim_loaded before using it.
__device__ __forceinline__ void load_uncounted(f4& v, const float* p)
{
    asm volatile("global_load_dwordx4 %0, %1, off nt" : "=&v"(v) : "v"(p) : "memory");
}
__device__ __forceinline__ void claim_loaded(f4& v) { asm volatile("" : "+v"(v)); }

// --------------------------------------------------------------------------------------
// compress.  LDS: xs[nbuf][16][d + 4] floats (the partial results reuse the strips of the tile), mus[d] floats; for
// bf16 storage see BIN below.
// --------------------------------------------------------------------------------------
// EXACT: fp32 products on v_mfma_f32_16x16x4_f32 instead of the bf16 split; U then sits in the same registers as
// floats (word [st][nt][h], register r: U[EW w + 32 st + 16 h + 4 kk + r][16 nt + m] for lane (m, kk)), and each of a
// lane's 8 floats of x per step is the B operand of one product.
// BIN: the gradient is stored as bf16.  A tile is then 16 rows of D bf16 without padding, its 16-byte chunks
// swizzled inside each row (chunk c of row r sits at chunk c ^ (r & 7): the copies place them so, and 8 lanes reading
// the same chunk of 8 rows hit 8 different bank groups); a lane widens its 8 numbers to fp32 and goes on as for fp32
// storage.  The strips of such a tile are too small for the partial results, which get a region of their own:
// part[8][16][16 NT + 4] floats.
template <int STEPS, int NT, bool EXACT, bool BIN>
__global__ __launch_bounds__(512) void compress_ws_kernel(WsArgs a, int nbuf)
{
    extern __shared__ f4 smem[];
    constexpr int D = 256 * STEPS, RS = D + WS_ROWPAD, EW = 32 * STEPS;
    constexpr int XT = BIN ? 8 * D : 16 * RS;   // floats of LDS per tile buffer
    constexpr int PS = 16 * NT + 4;             // BIN: floats per row of a wave's partial result
    constexpr int NCP = BIN ? STEPS : 2 * STEPS;   // 1 KB copies per wave and tile
    static_assert(16 * NT <= EW, "a wave's partial result must fit the strip of the tile it alone reads");
    float* xs = (float*)smem;                 // [nbuf][16][RS], or [nbuf][16][D] bf16
    float* part = xs + nbuf * XT;             // BIN only: [8][16][PS]
    float* mus = part + (BIN ? WS_WAVES * 16 * PS : 0);   // [D]
    const int tid = threadIdx.x, lane = tid & 63, n_ = lane & 15, kk = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    u4 us[STEPS][NT][2];
#pragma unroll
    for (int st = 0; st < STEPS; ++st)
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int p = 0; p < 2; ++p) us[st][nt][p] = a.Upack[((((size_t)w * STEPS + st) * NT + nt) * 2 + p) * 64 + lane];
    for (int e = tid; e < D; e += 512) mus[e] = a.mu[e] / a.n_workers;

    const unsigned int xs_off = (unsigned int)(size_t)(__attribute__((address_space(3))) void*)xs;
    // Piece i (0 .. NCP - 1) of this wave's share of a tile: 1 KB of row 2w + i / STEPS, into buffer buf; BIN: the 64
    // chunks from chunk 64 (w STEPS + i) of the tile on, each fetched from where the swizzle says
    auto copy_piece = [&](int64_t tile, int buf, int i) {
        if constexpr (BIN) {
            const int P = 64 * (w * STEPS + i) + lane, row = P / (D / 8), c = (P - row * (D / 8)) ^ (row & 7);
            const unsigned short* g = (const unsigned short*)a.in + ((a.first + 16 * tile + row) * (int64_t)D + 8 * c);
            copy_1k_to_lds(g, xs_off + 4u * (unsigned int)(buf * XT) + 1024u * (unsigned int)(w * STEPS + i));
        } else {
            const int row = 2 * w + i / STEPS, q = i % STEPS;
            const float* g = (const float*)a.in + ((a.first + 16 * tile + row) * (int64_t)D + q * 256 + lane * 4);
            copy_1k_to_lds(g, xs_off + 4u * (unsigned int)((buf * 16 + row) * RS + q * 256));
        }
    };

    // Wave v adds up column tile v when that tile holds a comp below k; it then issues exactly one store per tile.
    const bool adds = 16 * w < a.k;
    const bool ring = a.acc_in != nullptr;
    // nbuf - 1 tiles are in flight while one is worked on
    const int ahead = nbuf - 1;
    int64_t t = blockIdx.x;
    for (int p = 0; p < ahead; ++p) {
        const int64_t tp = t + (int64_t)p * gridDim.x;
        if (tp < a.ntiles) {
#pragma unroll
            for (int i = 0; i < NCP; ++i) copy_piece(tp, p, i);
        }
    }
    drain_memory();   // U and the first tiles have arrived: the loop below inherits no wait

    // One tile out of buffer `buf`: products, partial results, their sum, and the store of its first `rows` slices.
    // AHEAD: the pieces of tile `ta` are copied into buffer `bufa` between the products.
    auto work_tile = [&](auto ahead_c, int buf, int64_t tile, int rows, int64_t ta, int bufa) {
        constexpr bool AHEAD = decltype(ahead_c)::value;
        // ring step: this lane's word of the partial sum, asked for before the tile's copies and used after them
        f4 prev = {0.f, 0.f, 0.f, 0.f};
        if (adds && ring) {
            const int rr = n_ < rows ? n_ : rows - 1, cc = 16 * w + 4 * kk < a.k ? 16 * w + 4 * kk : a.k - 4;
            load_uncounted(prev, a.acc_in + (a.first + 16 * tile + rr) * a.k + cc);
        }
        f4 acc[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = f4{0.f, 0.f, 0.f, 0.f};
        float* xrow = xs + (buf * 16 + n_) * RS + EW * w + 4 * kk;
        const unsigned short* xrow16 = (const unsigned short*)(xs + buf * XT) + n_ * D;   // BIN
        const float* mrow = mus + EW * w + 4 * kk;
#pragma unroll
        for (int st = 0; st < STEPS; ++st) {
            // lane (n, kk): elements EW w + 32 st + 16 h + 4 kk .. + 3, h = 0, 1, of slice n
            f4 x0, x1;
            if constexpr (BIN) {
                const int e0 = EW * w + 32 * st + 4 * kk, e1 = e0 + 16;
                const u2 h0 = *(const u2*)(xrow16 + 8 * ((e0 >> 3) ^ (n_ & 7)) + (e0 & 4));
                const u2 h1 = *(const u2*)(xrow16 + 8 * ((e1 >> 3) ^ (n_ & 7)) + (e1 & 4));
                x0 = f4{__uint_as_float(h0.x << 16), __uint_as_float(h0.x & 0xffff0000u), __uint_as_float(h0.y << 16),
                        __uint_as_float(h0.y & 0xffff0000u)};
                x1 = f4{__uint_as_float(h1.x << 16), __uint_as_float(h1.x & 0xffff0000u), __uint_as_float(h1.y << 16),
                        __uint_as_float(h1.y & 0xffff0000u)};
            } else {
                x0 = *(const f4*)(xrow + 32 * st);
                x1 = *(const f4*)(xrow + 32 * st + 16);
            }
            const f4 m0 = *(const f4*)(mrow + 32 * st), m1 = *(const f4*)(mrow + 32 * st + 16);
            // the pieces of the tile ahead, between the products: every wave is past the second barrier of the tile
            // that used that buffer
            if constexpr (AHEAD) {
                if constexpr (BIN) copy_piece(ta, bufa, st);
                else {
                    copy_piece(ta, bufa, 2 * st);
                    copy_piece(ta, bufa, 2 * st + 1);
                }
            }
            if constexpr (EXACT) {
                const f4 xc[2] = {x0 - m0, x1 - m1};
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int nt = 0; nt < NT; ++nt)
                            acc[nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(us[st][nt][h][r]), xc[h][r],
                                                                           acc[nt], 0, 0, 0);
            } else {
                u4 xh, xl;
                split8(x0 - m0, x1 - m1, xh, xl);
                const lbf8 bh = __builtin_bit_cast(lbf8, xh), bl = __builtin_bit_cast(lbf8, xl);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, us[st][nt][0]), bl, acc[nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, us[st][nt][1]), bh, acc[nt], 0, 0, 0);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
                    acc[nt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, us[st][nt][0]), bh, acc[nt], 0, 0, 0);
            }
        }
        // The partial result goes where this wave's strip of x was: nobody else reads that strip, and this wave
        // is done with it.  Register r of lane (n, kk) of column tile nt: row n, float EW w + 16 nt + 4 kk + r.
        float* pw = BIN ? part + (w * 16 + n_) * PS + 4 * kk : xrow;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) *(f4*)(pw + 16 * nt) = acc[nt];
        __syncthreads();
        // wave v adds the 8 partial results of column tile v (comps 16 v + 4 kk + r of slice n).  The
        // buffer is next written by the copy of a later tile, which every wave asks for after the next barrier.
        if (adds) {
            const float* prow = BIN ? part + n_ * PS + 16 * w + 4 * kk : xs + (buf * 16 + n_) * RS + 16 * w + 4 * kk;
            constexpr int PV = BIN ? 16 * PS : EW;   // from one wave's partial result to the next
            f4 s = *(const f4*)prow;
#pragma unroll
            for (int v = 1; v < WS_WAVES; ++v) s += *(const f4*)(prow + PV * v);
            const int c0 = 16 * w + 4 * kk;
            const int64_t o = (a.first + 16 * tile + n_) * a.k + c0;
            float* Y = (float*)a.out;
            if (ring) {
                // younger than the word asked for: this tile's copies
                if constexpr (AHEAD) wait_vmem_at_most<NCP>(); else wait_vmem_at_most<0>();
                claim_loaded(prev);
                s += prev;
            }
            if (c0 < a.k && n_ < rows) stream_store((f4*)(Y + o), s);   // k is a multiple of 4; true for kk = 0 at least
        }
    };

    for (int buf = 0; t < a.ntiles; t += gridDim.x, buf = buf + 1 == nbuf ? 0 : buf + 1) {
        // the tile to ask for (the current one again when there is none: the count in flight stays the same)
        // and the buffer it goes to, which held the tile before this one
        const int64_t ta = t + (int64_t)ahead * gridDim.x < a.ntiles ? t + (int64_t)ahead * gridDim.x : t;
        const int bufa = buf == 0 ? nbuf - 1 : buf - 1;
        // This wave's rows of the current tile: memory operations retire in order, and the requests younger
        // than them are the copies of the tiles between (NCP each) and one store per tile for the waves
        // that add up a column tile.
        if (ahead == 2) {
            if (adds && ring) wait_vmem_at_most<NCP + 3>();   // ... and the word of the partial sum in between
            else if (adds) wait_vmem_at_most<NCP + 2>();
            else wait_vmem_at_most<NCP>();
        } else {
            if (adds) wait_vmem_at_most<1>(); else wait_vmem_at_most<0>();
        }
        __syncthreads();
        work_tile(std::true_type{}, buf, t, 16, ta, bufa);
    }
    drain_memory();   // the last copies have no reader: let them land before the buffers are used again or released

    // The slices after the last whole tile (fewer than 16, or 16 of which the last ends past M): one work-group
    // fetches them with bounds-checked loads, zeros where there is nothing, and works on them like on any tile.
    if (a.tail_rows > 0 && (int64_t)blockIdx.x == a.ntiles % gridDim.x) {
        __syncthreads();   // every wave has read its last partial results
        const int64_t s0 = a.first + 16 * a.ntiles;
        if constexpr (BIN) {
            const unsigned short* in16 = (const unsigned short*)a.in;
            for (int P = tid; P < 2 * D; P += 512) {   // the tile's 16-byte chunks, in LDS order
                const int row = P / (D / 8), c = (P - row * (D / 8)) ^ (row & 7);
                const int64_t e = (s0 + row) * (int64_t)D + 8 * c;
                unsigned int hw[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
                if (row < a.tail_rows) {
#pragma unroll
                    for (int i = 0; i < 8; ++i)
                        if (e + i < a.M) hw[i] = in16[e + i];
                }
                *(u4*)((unsigned short*)xs + 8 * P) = u4{hw[0] | (hw[1] << 16), hw[2] | (hw[3] << 16), hw[4] | (hw[5] << 16),
                                                        hw[6] | (hw[7] << 16)};
            }
        } else
        for (int i = tid; i < 16 * (D / 4); i += 512) {
            const int row = i / (D / 4), c4 = i - row * (D / 4);
            const int64_t e = (s0 + row) * (int64_t)D + 4 * c4;
            f4 v = {0.f, 0.f, 0.f, 0.f};
            if (row < a.tail_rows) {
                const float* g = (const float*)a.in + e;
                if (e + 3 < a.M) v = *(const f4*)g;
                else {
                    if (e < a.M) v.x = g[0];
                    if (e + 1 < a.M) v.y = g[1];
                    if (e + 2 < a.M) v.z = g[2];
                }
            }
            *(f4*)(xs + row * RS + 4 * c4) = v;
        }
        __syncthreads();
        work_tile(std::false_type{}, 0, a.ntiles, a.tail_rows, 0, 0);
    }
}

// --------------------------------------------------------------------------------------
// The operand-order copy of U, 8 bf16 per 128-bit word, term p = 0: bf16(U), p = 1: bf16(U - term 0); zero where
// comp >= k.  Uc[w][st][nt][p][lane (m, kk)][j] = U[EW w + 32 st + r(kk, j)][16 nt + m], EW = d/8,
// r(kk, j) = 16 (j / 4) + 4 kk + j % 4 (the order in which a lane reads its strip of x).
// --------------------------------------------------------------------------------------
__global__ void pack_ws_kernel(const float* U, unsigned short* Uc, int d, int k, int NT)
{
    const int EW = d / 8, STEPS = d / 256;
    const size_t n = (size_t)WS_WAVES * STEPS * NT * 2 * 512;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(q & 7), lane = (int)((q >> 3) & 63), m = lane & 15, kk = lane >> 4, p = (int)((q >> 9) & 1);
        size_t g = q >> 10;
        const int nt = (int)(g % NT); g /= NT;
        const int st = (int)(g % STEPS), w = (int)(g / STEPS);
        const int e = EW * w + 32 * st + 16 * (j >> 2) + 4 * kk + (j & 3), comp = 16 * nt + m;
        unsigned short v = 0;
        if (comp < k) {
            const float u = U[(size_t)e * k + comp];
            const unsigned int t0 = f32_to_bf16_rne(u);
            v = (unsigned short)(p == 0 ? t0 : f32_to_bf16_rne(u - __uint_as_float(t0 << 16)));
        }
        Uc[q] = v;
    }
}

// --------------------------------------------------------------------------------------
// decompress, Eq. (4): x = U y + mu, fp32 output.  Wave w keeps the rows 2 STEPS x 16 of U that belong to its
// eighth of the slice (all comps) and produces that eighth of all 16 slices of a tile from the whole y tile: no
// partial results to add.  The 16 x d results meet in LDS so that they leave as whole rows: wave w stores rows
// 2w and 2w + 1 in runs of 1 KB.  Groups of WSD_IL consecutive tiles (which run side by side on neighbouring
// compute units) interleave their slices: tile j of a group takes slices j, j + WSD_IL, ... of the group's
// 16 WSD_IL, so that the chip writes one compact window row by row (a write-only probe of this pattern: 5.8 TB/s
// against 4.9 - 5.1 for 48 KB runs per work-group and 3.4 - 4.4 for 64-byte pieces).  One barrier per tile: the
// result tile is double-buffered, the y tiles sit in a ring of WSD_NY, and a tile's rows are stored between the
// products of the tile after it, so that the store unit and the matrix pipe work at the same time (one burst of
// stores per tile, with nothing computed meanwhile, was 13 % slower).
// A tile's y (16 rows of k floats) is gathered global -> LDS by the load unit, one 128-bit word per lane: LDS word
// YW row + c holds comps 4c .. 4c + 3 of the row's slice, YW = 8 NKS + 1 (odd: 16 lanes x 128 bits cover all banks),
// and the words past k come from a zero word in global memory, so that a row reads as zeros up to 32 NKS comps.
// LDS: os[2][16][d + 4] floats, ys[WSD_NY][YT] 128-bit words (YT: 16 YW rounded up to whole 64-lane copies), mus[d].
// --------------------------------------------------------------------------------------
struct WsdArgs {
    const float* y;          // compressed gradient
    void* out;               // gradient (fp32, or bf16 for OBF)
    const u4* Upack;         // the operand-order copy of U (layout at the pack kernel)
    const float* zero;       // 4 floats of zeros
    const float* mu;         // [d]
    int64_t first;           // first slice
    int64_t ntiles;          // whole 16-slice tiles inside the gradient
    int64_t M;               // elements of the gradient
    int tail_rows;           // slices after the last whole tile (0 .. 16; the last one may end past M)
    int d, k;
    int il;                  // tiles per interleave group
};

#define WSD_IL 16
#define WSD_NY 4   // y tiles in LDS: one in use, three on their way

// EXACT: fp32 products on v_mfma_f32_16x16x4_f32; U's words then hold floats, word [ti][ks][h], register r:
// U[EW w + 16 ti + m][32 ks + 16 h + 4 kk + r] for lane (m, kk).
// OBF: the output is bf16 (round to nearest even at the row stores, 8 numbers per lane and store).
template <int STEPS, int NKS, bool EXACT, bool OBF>
__global__ __launch_bounds__(512) void decompress_ws_kernel(WsdArgs a)
{
    extern __shared__ f4 smem[];
    constexpr int D = 256 * STEPS, RS = D + WS_ROWPAD, EW = 32 * STEPS, NTI = 2 * STEPS;
    constexpr int YW = 8 * NKS + 1, YC = (16 * YW + 63) / 64, YT = 64 * YC;   // words per row, 64-word copies, words
    float* os = (float*)smem;            // [2][16][RS]
    f4* ys = (f4*)(os + 2 * 16 * RS);    // [WSD_NY][YT]
    float* mus = (float*)(ys + WSD_NY * YT);  // [D]
    const int tid = threadIdx.x, lane = tid & 63, n_ = lane & 15, kk = lane >> 4;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    u4 ua[NTI][NKS][2];
#pragma unroll
    for (int ti = 0; ti < NTI; ++ti)
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks)
#pragma unroll
            for (int p = 0; p < 2; ++p) ua[ti][ks][p] = a.Upack[((((size_t)w * NTI + ti) * NKS + ks) * 2 + p) * 64 + lane];
    for (int e = tid; e < D; e += 512) mus[e] = a.mu[e];

    // Slice `row` of tile `tile`, counted from a.first (see above); the tiles past the last whole group, and the
    // tail tile, keep 16 consecutive slices.
    const int64_t n_il = a.ntiles / a.il * a.il;
    auto slice_of = [&](int64_t tile, int row) -> int64_t {
        if (tile >= n_il) return 16 * tile + row;
        const int64_t g = tile / a.il, j = tile - g * a.il;
        return 16 * a.il * g + (int64_t)row * a.il + j;
    };
    // This wave's copies of a tile's y: the 64 words from 64 c on, c = w and w + 8 (the latter only exists for
    // wave 0, and only when a tile has more than 512 words).
    const int kq = a.k >> 2;
    const unsigned int ys_off = (unsigned int)(size_t)(__attribute__((address_space(3))) void*)ys;
    auto copy_y = [&](int64_t tile, int buf, int rows) {
        for (int c = w; c < YC; c += 8) {
            const int word = 64 * c + lane, row = word / YW, col = word - row * YW;
            const float* src = a.zero;
            if (row < rows && col < kq) src = a.y + (a.first + slice_of(tile, row)) * a.k + 4 * col;
            copy_1k_to_lds(src, ys_off + 16u * (unsigned int)(buf * YT + 64 * c));
        }
    };

    // Rows 2w and 2w + 1 of the result tile in os[buf] leave whole, piece i = 0 .. NST - 1 at a time: 1 KB of output
    // per piece, i.e. 256 fp32 or 512 bf16 numbers of the two rows taken as one run of 2 D numbers.
    constexpr int NST = OBF ? STEPS : 2 * STEPS, PER = OBF ? 8 : 4;
    auto store_piece = [&](int buf, int64_t tile, int i) {
        const int e = (256 * PER / 4) * i + PER * lane, row = 2 * w + e / D, col = e % D;
        const float* src = os + (buf * 16 + row) * RS + col;
        const int64_t o = (a.first + slice_of(tile, row)) * (int64_t)D + col;
        if constexpr (OBF) {
            const f4 v0 = *(const f4*)src, v1 = *(const f4*)(src + 4);
            const u4 pk = {f32_to_bf16_rne(v0.x) | (f32_to_bf16_rne(v0.y) << 16), f32_to_bf16_rne(v0.z) | (f32_to_bf16_rne(v0.w) << 16),
                           f32_to_bf16_rne(v1.x) | (f32_to_bf16_rne(v1.y) << 16), f32_to_bf16_rne(v1.z) | (f32_to_bf16_rne(v1.w) << 16)};
            stream_store((u4*)((unsigned short*)a.out + o), pk);
        } else {
            stream_store((f4*)((float*)a.out + o), *(const f4*)src);
        }
    };
    // The products of one tile out of ys[ybuf] into os[buf]; between them, when there is one, the stores of the tile
    // before (`prev`, in the other result buffer): the store unit takes them while the matrix pipe works, instead of
    // one burst per tile during which nothing is computed.
    auto products = [&](int buf, int ybuf, bool have_prev, int64_t prev) {
        f4 acc[NTI];
        const float* mrow = mus + EW * w + 4 * kk;
#pragma unroll
        for (int ti = 0; ti < NTI; ++ti) acc[ti] = *(const f4*)(mrow + 16 * ti);
        const f4* yr = ys + ybuf * YT + n_ * YW + kk;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
            // lane (n, kk): comps 32 ks + 16 h + 4 kk .. + 3, h = 0, 1, of slice n
            if constexpr (EXACT) {
                const f4 yc[2] = {yr[8 * ks], yr[8 * ks + 4]};
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    if (32 * ks + 16 * h >= a.k) continue;   // 16 comps that do not exist (k = 16: half the products)
#pragma unroll
                    for (int r = 0; r < 4; ++r)
#pragma unroll
                        for (int ti = 0; ti < NTI; ++ti)
                            acc[ti] = __builtin_amdgcn_mfma_f32_16x16x4f32(__uint_as_float(ua[ti][ks][h][r]), yc[h][r],
                                                                           acc[ti], 0, 0, 0);
                }
            } else {
                u4 yh, yl;
                split8(yr[8 * ks], yr[8 * ks + 4], yh, yl);
                const lbf8 bh = __builtin_bit_cast(lbf8, yh), bl = __builtin_bit_cast(lbf8, yl);
#pragma unroll
                for (int ti = 0; ti < NTI; ++ti)
                    acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, ua[ti][ks][0]), bl, acc[ti], 0, 0, 0);
#pragma unroll
                for (int ti = 0; ti < NTI; ++ti)
                    acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, ua[ti][ks][1]), bh, acc[ti], 0, 0, 0);
#pragma unroll
                for (int ti = 0; ti < NTI; ++ti)
                    acc[ti] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(lbf8, ua[ti][ks][0]), bh, acc[ti], 0, 0, 0);
            }
            if (have_prev) {
#pragma unroll
                for (int i = 0; i < NST; ++i)
                    if (i * NKS / NST == ks) store_piece(buf ^ 1, prev, i);
            }
        }
        // register r of lane (n, kk) of row tile ti: element EW w + 16 ti + 4 kk + r of slice n
        float* orow = os + (buf * 16 + n_) * RS + EW * w + 4 * kk;
#pragma unroll
        for (int ti = 0; ti < NTI; ++ti) *(f4*)(orow + 16 * ti) = acc[ti];
    };

    // this wave's copies per tile
    const int ncopy = (w < YC ? 1 : 0) + (w + 8 < YC ? 1 : 0);
    int64_t t = blockIdx.x;
    if (t < a.ntiles) {
        for (int p = 0; p < WSD_NY; ++p) {
            const int64_t tp = t + (int64_t)p * gridDim.x;
            copy_y(tp < a.ntiles ? tp : t, p, 16);
        }
    }
    drain_memory();   // U, and the first y tiles: the loop below inherits no wait
    __syncthreads();
    int buf = 0;
    for (int ybuf = 0; t < a.ntiles; t += gridDim.x, buf ^= 1, ybuf = ybuf + 1 == WSD_NY ? 0 : ybuf + 1) {
        products(buf, ybuf, t != (int64_t)blockIdx.x, t - gridDim.x);
        // The y tile after this one was asked for WSD_NY - 1 tiles ago.  Requests retire in order, and the younger
        // ones are the stores of WSD_NY - 1 tiles and the copies of the WSD_NY - 2 y tiles between.
        constexpr int younger = (WSD_NY - 1) * NST;
        if (ncopy == 0) wait_vmem_at_most<younger>();
        else if (ncopy == 1) wait_vmem_at_most<younger + (WSD_NY - 2)>();
        else wait_vmem_at_most<younger + 2 * (WSD_NY - 2)>();
        __syncthreads();
        // WSD_NY tiles on, into the buffer that this tile's products have just read
        const int64_t ta = t + (int64_t)WSD_NY * gridDim.x;
        copy_y(ta < a.ntiles ? ta : t, ybuf, 16);
    }
    // the last tile's rows (its barrier has passed)
    if ((int64_t)blockIdx.x < a.ntiles) {
#pragma unroll
        for (int i = 0; i < NST; ++i) store_piece(buf ^ 1, t - gridDim.x, i);
    }
    drain_memory();   // the last copies have no reader: let them land before the buffers are used again or released

    // The slices after the last whole tile: the same work by one work-group, with bounds-checked stores.
    if (a.tail_rows > 0 && (int64_t)blockIdx.x == a.ntiles % gridDim.x) {
        __syncthreads();   // every wave is past its last reads of both buffers
        copy_y(a.ntiles, 0, a.tail_rows);
        drain_memory();
        __syncthreads();
        products(0, 0, false, 0);
        __syncthreads();
        for (int i = 0; i < 2 * STEPS; ++i) {
            const int row = 2 * w + i / STEPS, q = i % STEPS;
            if (row >= a.tail_rows) continue;
            const f4 v = *(const f4*)(os + row * RS + q * 256 + lane * 4);
            const int64_t e = (a.first + 16 * a.ntiles + row) * (int64_t)D + q * 256 + lane * 4;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                if (e + r >= a.M) break;
                if constexpr (OBF) ((unsigned short*)a.out)[e + r] = (unsigned short)f32_to_bf16_rne(v[r]);
                else ((float*)a.out)[e + r] = v[r];
            }
        }
    }
}

// The operand-order copy of U for the kernel above, 8 bf16 per 128-bit word, terms as in pack_ws_kernel.
// Ud[w][ti][ks][p][lane (m, kk)][j] = U[EW w + 16 ti + m][32 ks + r(kk, j)], r(kk, j) = 16 (j / 4) + 4 kk + j % 4.
__global__ void pack_wsd_kernel(const float* U, unsigned short* Ud, int d, int k, int NKS, size_t zero_at)
{
    const int EW = d / 8, NTI = d / 128;
    const size_t n = (size_t)WS_WAVES * NTI * NKS * 2 * 512;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += (size_t)gridDim.x * blockDim.x) {
        const int j = (int)(q & 7), lane = (int)((q >> 3) & 63), m = lane & 15, kk = lane >> 4, p = (int)((q >> 9) & 1);
        size_t g = q >> 10;
        const int ks = (int)(g % NKS); g /= NKS;
        const int ti = (int)(g % NTI), w = (int)(g / NTI);
        const int e = EW * w + 16 * ti + m, comp = 32 * ks + 16 * (j >> 2) + 4 * kk + (j & 3);
        unsigned short v = 0;
        if (comp < k) {
            const float u = U[(size_t)e * k + comp];
            const unsigned int t0 = f32_to_bf16_rne(u);
            v = (unsigned short)(p == 0 ? t0 : f32_to_bf16_rne(u - __uint_as_float(t0 << 16)));
        }
        Ud[q] = v;
    }
    if (blockIdx.x == 0 && threadIdx.x < 8) Ud[zero_at + threadIdx.x] = 0;   // the zero word of WsdArgs, after both copies
}

// The fp32 copy of U for decompress_ws_kernel<.., EXACT = true>.
// Ude[w][ti][ks][h][lane (m, kk)][r] = U[EW w + 16 ti + m][32 ks + 16 h + 4 kk + r]; zero where comp >= k.
__global__ void pack_wsd_exact_kernel(const float* U, float* Ue, int d, int k, int NKS)
{
    const int EW = d / 8, NTI = d / 128;
    const size_t n = (size_t)WS_WAVES * NTI * NKS * 2 * 256;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(q & 3), lane = (int)((q >> 2) & 63), m = lane & 15, kk = lane >> 4, h = (int)((q >> 8) & 1);
        size_t g = q >> 9;
        const int ks = (int)(g % NKS); g /= NKS;
        const int ti = (int)(g % NTI), w = (int)(g / NTI);
        const int e = EW * w + 16 * ti + m, comp = 32 * ks + 16 * h + 4 * kk + r;
        Ue[q] = comp < k ? U[(size_t)e * k + comp] : 0.f;
    }
}

// The fp32 copy of U for compress_ws_kernel<.., EXACT = true>: same words as the bf16 copy, each holding 4 floats.
// Ue[w][st][nt][h][lane (m, kk)][r] = U[EW w + 32 st + 16 h + 4 kk + r][16 nt + m]; zero where comp >= k.
__global__ void pack_ws_exact_kernel(const float* U, float* Ue, int d, int k, int NT)
{
    const int EW = d / 8, STEPS = d / 256;
    const size_t n = (size_t)WS_WAVES * STEPS * NT * 2 * 256;
    for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < n; q += (size_t)gridDim.x * blockDim.x) {
        const int r = (int)(q & 3), lane = (int)((q >> 2) & 63), m = lane & 15, kk = lane >> 4, h = (int)((q >> 8) & 1);
        size_t g = q >> 9;
        const int nt = (int)(g % NT); g /= NT;
        const int st = (int)(g % STEPS), w = (int)(g / STEPS);
        const int e = EW * w + 32 * st + 16 * h + 4 * kk + r, comp = 16 * nt + m;
        Ue[q] = comp < k ? U[(size_t)e * k + comp] : 0.f;
    }
}

// ======================================================================================
// host side
// ======================================================================================
static int ws_nt(int k) { const int nt = (k + 15) / 16; return nt + (nt & 1); }   // column tiles, even

// LDS: nbuf tiles of 16 padded rows, and mu
static size_t ws_lds(int d, int nbuf, bool bin = false, int nt = 0)
{
    if (bin) return sizeof(float) * ((size_t)nbuf * 8 * d + (size_t)WS_WAVES * 16 * (16 * nt + 4) + d);
    return sizeof(float) * ((size_t)nbuf * 16 * (d + WS_ROWPAD) + d);
}
// Tiles of x in LDS: three (two in flight) where they fit 160 KB (d <= 768), else two (with two, d = 256 is 20 %
// slower, d = 768 2 %; d = 512 measures 3 % faster, within what one box differs from the next)
static int ws_nbuf(int d) { return ws_lds(d, 3) <= 160 * 1024 ? 3 : 2; }

// One basis, d in {256, 512, 768, 1024}, k a multiple of 4, U fits the registers of 8 waves (d/256 x NT words of
// 8 registers, at most 18), and a wave's partial result fits its strip of the tile (16 floats per column tile,
// d/8 per strip).  Wherever it can run it beats the LDS-tiled split kernel on 138 M elements: d = 256, k = 32: 5.5 against
// 4.7 TB/s, d = 512, k = 64: 5.1 against 4.4, d = 768, k = 96: 5.05 against 3.6, d = 1024, k = 64: 5.2 against 3.25.
bool gvq_ws_shape(const gvq_basis* h)
{
    if (h->B != 1 || h->d % 256 != 0 || h->d > 1024 || h->k % 4 != 0) return false;
    return (h->d / 256) * ws_nt(h->k) <= 18 && 16 * ws_nt(h->k) <= h->d / 8;
}

// bf16 values of the operand-order copy
size_t gvq_ws_pack_halves(int d, int k) { return (size_t)WS_WAVES * (d / 256) * ws_nt(k) * 2 * 512; }

// decompress: one basis, d in {256, 512, 768, 1024}, k a multiple of 4 up to 128 (a tile's y is one 128-bit word
// per thread), U fits the registers of 8 waves (d/128 x ceil(k/32) words of 8 registers, at most 18).
static int wsd_nks(int k) { return (k + 31) / 32; }
bool gvq_wsd_shape(const gvq_basis* h)
{
    if (h->B != 1 || h->d % 256 != 0 || h->d > 1024 || h->k % 4 != 0 || h->k > 128) return false;
    return (h->d / 128) * wsd_nks(h->k) <= 18;
}
// ... and 8 more for a 128-bit word of zeros
static size_t wsd_copy_halves(int d, int k) { return (size_t)WS_WAVES * (d / 128) * wsd_nks(k) * 2 * 512; }
size_t gvq_wsd_pack_halves(int d, int k) { return 2 * wsd_copy_halves(d, k) + 8; }   // bf16 split, fp32, zeros
// d_Uws holds the two compress copies (bf16 split, then fp32; if that kernel takes the shape), then the decompress copy
static size_t wsd_offset_halves(const gvq_basis* h) { return gvq_ws_shape(h) ? 2 * gvq_ws_pack_halves(h->d, h->k) : 0; }
size_t gvq_ws_alloc_halves(const gvq_basis* h)
{
    return wsd_offset_halves(h) + (gvq_wsd_shape(h) ? gvq_wsd_pack_halves(h->d, h->k) : 0);
}

int gvq_launch_pack_ws(const gvq_basis* h, hipStream_t st)
{
    if (gvq_ws_shape(h)) {
        hipLaunchKernelGGL(pack_ws_kernel, dim3(256), dim3(256), 0, st, h->d_U, h->d_Uws, h->d, h->k, ws_nt(h->k));
        GVQ_HIP(hipGetLastError());
        hipLaunchKernelGGL(pack_ws_exact_kernel, dim3(256), dim3(256), 0, st, h->d_U,
                           (float*)(h->d_Uws + gvq_ws_pack_halves(h->d, h->k)), h->d, h->k, ws_nt(h->k));
        GVQ_HIP(hipGetLastError());
    }
    if (gvq_wsd_shape(h)) {
        hipLaunchKernelGGL(pack_wsd_kernel, dim3(256), dim3(256), 0, st, h->d_U, h->d_Uws + wsd_offset_halves(h), h->d,
                           h->k, wsd_nks(h->k), 2 * wsd_copy_halves(h->d, h->k));
        GVQ_HIP(hipGetLastError());
        hipLaunchKernelGGL(pack_wsd_exact_kernel, dim3(256), dim3(256), 0, st, h->d_U,
                           (float*)(h->d_Uws + wsd_offset_halves(h) + wsd_copy_halves(h->d, h->k)), h->d, h->k,
                           wsd_nks(h->k));
        GVQ_HIP(hipGetLastError());
    }
    return GVQ_OK;
}

// Whole 16-slice tiles at the start of [first_slice, first_slice + n_slices) that lie inside the gradient.
static int64_t ws_tiles(const gvq_basis* h, int64_t first_slice, int64_t n_slices)
{
    const int64_t full = h->M / h->d;
    const int64_t end = first_slice + n_slices < full ? first_slice + n_slices : full;
    return end > first_slice ? (end - first_slice) / 16 : 0;
}

template <auto KERN>
static int launch_ws(const gvq_basis* h, const WsArgs& a, size_t lds, int nbuf, hipStream_t st)
{
    static gvq_once_per_device once;   // per kernel
    if (once.first(h->device))
        GVQ_HIP(hipFuncSetAttribute((const void*)KERN, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024));
    int64_t grid = a.ntiles < h->num_cu ? a.ntiles : h->num_cu;   // one work-group per compute unit
    if (grid < 1) grid = 1;   // only the slices after the last whole tile
    hipLaunchKernelGGL(KERN, dim3((unsigned)grid), dim3(512), lds, st, a, nbuf);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int STEPS, bool EXACT, bool BIN>
static int compress_ws_nt(const gvq_basis* h, const WsArgs& a, hipStream_t st)
{
    const int NT = ws_nt(h->k), nbuf = BIN ? 3 : ws_nbuf(256 * STEPS);
    const size_t lds = ws_lds(256 * STEPS, nbuf, BIN, NT);
    // the shapes gvq_ws_shape lets through: 16 NT <= 32 STEPS, and STEPS x NT <= 18
    if constexpr (STEPS == 4) {
        if (NT == 4) return launch_ws<compress_ws_kernel<4, 4, EXACT, BIN>>(h, a, lds, nbuf, st);
    }
    if constexpr (STEPS == 3) {
        if (NT == 6) return launch_ws<compress_ws_kernel<3, 6, EXACT, BIN>>(h, a, lds, nbuf, st);
        if (NT == 4) return launch_ws<compress_ws_kernel<3, 4, EXACT, BIN>>(h, a, lds, nbuf, st);
    }
    if constexpr (STEPS == 2) {
        if (NT == 4) return launch_ws<compress_ws_kernel<2, 4, EXACT, BIN>>(h, a, lds, nbuf, st);
    }
    return launch_ws<compress_ws_kernel<STEPS, 2, EXACT, BIN>>(h, a, lds, nbuf, st);
}

template <bool EXACT, bool BIN>
static int compress_ws_steps(const gvq_basis* h, const WsArgs& a, hipStream_t st)
{
    switch (h->d / 256) {
    case 1: return compress_ws_nt<1, EXACT, BIN>(h, a, st);
    case 2: return compress_ws_nt<2, EXACT, BIN>(h, a, st);
    case 3: return compress_ws_nt<3, EXACT, BIN>(h, a, st);
    default: return compress_ws_nt<4, EXACT, BIN>(h, a, st);
    }
}

// Compresses the range (as far as the gradient has slices); *done = the slices it took.
int gvq_launch_compress_ws(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice, int64_t n_slices,
                           const float* comp_in, float* out, bool exact, hipStream_t st, int64_t* done)
{
    WsArgs a;
    a.in = grad; a.out = out; a.acc_in = comp_in; a.mu = h->d_mu;
    a.Upack = (const u4*)(h->d_Uws + (exact ? gvq_ws_pack_halves(h->d, h->k) : 0));
    a.first = first_slice; a.ntiles = ws_tiles(h, first_slice, n_slices); a.d = h->d; a.k = h->k;
    a.n_workers = (float)n_workers;
    a.M = h->M;
    const int64_t end = first_slice + n_slices < h->S ? first_slice + n_slices : h->S;
    const int64_t tail = end - (first_slice + 16 * a.ntiles);   // 0 .. 15 whole slices and the one that ends past M
    a.tail_rows = tail > 0 ? (int)tail : 0;
    *done = 16 * a.ntiles + a.tail_rows;
    if (*done == 0) return GVQ_OK;
    if (h->dtype == GVQ_BF16) return exact ? GVQ_EINVAL : compress_ws_steps<false, true>(h, a, st);   // bf16 storage: split pipe only
    return exact ? compress_ws_steps<true, false>(h, a, st) : compress_ws_steps<false, false>(h, a, st);
}

template <int STEPS, int NKS, bool EXACT, bool OBF>
static int launch_wsd(const gvq_basis* h, const WsdArgs& a, hipStream_t st)
{
    constexpr int D = 256 * STEPS;
    constexpr size_t lds = sizeof(float) * (2 * 16 * (D + WS_ROWPAD) + WSD_NY * 4 * 64 * ((16 * (8 * NKS + 1) + 63) / 64) + D);
    static_assert(lds <= 160 * 1024, "LDS");
    static gvq_once_per_device once;
    if (once.first(h->device))
        GVQ_HIP(hipFuncSetAttribute((const void*)decompress_ws_kernel<STEPS, NKS, EXACT, OBF>,
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
    int64_t grid = a.ntiles < h->num_cu ? a.ntiles : h->num_cu;   // one work-group per compute unit
    if (grid < 1) grid = 1;
    hipLaunchKernelGGL((decompress_ws_kernel<STEPS, NKS, EXACT, OBF>), dim3((unsigned)grid), dim3(512), lds, st, a);
    GVQ_HIP(hipGetLastError());
    return GVQ_OK;
}

template <int STEPS, bool EXACT, bool OBF>
static int decompress_ws_nks(const gvq_basis* h, const WsdArgs& a, hipStream_t st)
{
    // the shapes gvq_wsd_shape lets through: 2 STEPS x NKS <= 18, NKS <= 4
    switch (wsd_nks(h->k)) {
    case 1: return launch_wsd<STEPS, 1, EXACT, OBF>(h, a, st);
    case 2: return launch_wsd<STEPS, 2, EXACT, OBF>(h, a, st);
    case 3: if constexpr (STEPS <= 3) return launch_wsd<STEPS, 3, EXACT, OBF>(h, a, st); else break;
    case 4: if constexpr (STEPS <= 2) return launch_wsd<STEPS, 4, EXACT, OBF>(h, a, st); else break;
    }
    return GVQ_EINVAL;
}

template <bool EXACT, bool OBF>
static int decompress_ws_steps(const gvq_basis* h, const WsdArgs& a, hipStream_t st)
{
    switch (h->d / 256) {
    case 1: return decompress_ws_nks<1, EXACT, OBF>(h, a, st);
    case 2: return decompress_ws_nks<2, EXACT, OBF>(h, a, st);
    case 3: return decompress_ws_nks<3, EXACT, OBF>(h, a, st);
    default: return decompress_ws_nks<4, EXACT, OBF>(h, a, st);
    }
}

// Decompresses the range (as far as the gradient has slices) into fp32 or bf16; *done = the slices it took.
int gvq_launch_decompress_ws(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices, void* out,
                             bool out_bf16, bool exact, hipStream_t st, int64_t* done)
{
    WsdArgs a;
    const size_t copy = wsd_copy_halves(h->d, h->k);
    a.y = comp; a.out = out; a.Upack = (const u4*)(h->d_Uws + wsd_offset_halves(h) + (exact ? copy : 0)); a.mu = h->d_mu;
    a.zero = (const float*)(h->d_Uws + wsd_offset_halves(h) + 2 * copy);
    a.first = first_slice; a.ntiles = ws_tiles(h, first_slice, n_slices); a.M = h->M; a.d = h->d; a.k = h->k;
    const int64_t end = first_slice + n_slices < h->S ? first_slice + n_slices : h->S;
    const int64_t tail = end - (first_slice + 16 * a.ntiles);
    a.tail_rows = tail > 0 ? (int)tail : 0;
    a.il = gvq_opt_interleave() > 0 ? gvq_opt_interleave() : WSD_IL;
    *done = 16 * a.ntiles + a.tail_rows;
    if (*done == 0) return GVQ_OK;
    if (out_bf16) return exact ? decompress_ws_steps<true, true>(h, a, st) : decompress_ws_steps<false, true>(h, a, st);
    return exact ? decompress_ws_steps<true, false>(h, a, st) : decompress_ws_steps<false, false>(h, a, st);
}
