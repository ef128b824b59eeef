// Internal declarations shared by the translation units of libgvq (host side only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gvq.h"

#define GVQ_MAX_PTRS 32  // device pointers passed by value in one kernel launch
#define GVQ_LDS_EIGEN_MAX_D 64   // longest slice that goes to the one-work-group eigensolver with the matrix in LDS;
                                 // longer ones take the block Jacobi method (gvq_eigen_block.hip)

// Many bases: the split of the gradient's 16-slice tiles into super-tiles (G consecutive tiles of
// whole slices of one basis, for the branch-free fast phase of the register-resident codec kernels)
// and the rest, made once per handle.
struct gvq_plan {
    int64_t n_super = 0, n_rest = 0;
    int64_t* d_sup_tile = nullptr;   // [n_super] first 16-slice tile
    int* d_sup_basis = nullptr;      // [n_super] basis
    int64_t* d_rest = nullptr;       // [n_rest] the tiles no super-tile covers
};

struct gvq_basis {
    int64_t M = 0, S = 0;       // elements, slices
    int d = 0, k = 0, B = 0;    // slice length, kept components, number of bases
    gvq_dtype_t dtype = GVQ_F32;
    int device = 0;
    int num_cu = 0;
    int64_t* h_offs = nullptr;  // host [B+1]
    int64_t* d_offs = nullptr;  // device [B+1]
    int* d_tile_block = nullptr;  // device [ceil(S/16)]: basis of the first slice of each 16-slice tile (B > 1)
    gvq_plan plan[2];             // B > 1, register-resident shapes: G = 128/d, and the bf16-pipe compress's G
    int64_t* h_ltile = nullptr; // host [B+1]: first 128-slice tile of each basis (long slices, B > 1)
    int64_t* d_ltile = nullptr; // device copy
    float* d_U = nullptr;       // [B][d][k]
    float* d_mu = nullptr;      // [B][d]
    float* d_Upc = nullptr;     // [B][d][KP] U in compress-MFMA operand order (MFMA shapes only; long slices:
                                // d rounded up to 64, KP = 16 * gvq_long_nt(k))
    float* d_Upd = nullptr;     // [B][d][KP] U in decompress-MFMA operand order
    unsigned short* d_Upb = nullptr;  // [B][d/32][3][NT][64][8] bf16 three-term split of U (bf16 gradients);
                                      // long slices: the two-term copies, compress order then decompress order
    unsigned short* d_Uws = nullptr;  // basis-stationary compress kernel (gvq_ws_shape): two-term bf16 copy of U in its
                                      // operand order, per wave
    float* d_Umu = nullptr;     // [B][KP] U^T mu (bf16 gradients)
    double* d_eig = nullptr;    // [B][d]
    double* d_cov = nullptr;    // [B][d][d]
    double* d_V = nullptr;      // [B][dp][dp] eigenvector work space, dp = d rounded up to even (block Jacobi: to
                                // a whole number of block pairs)
    double* d_part = nullptr;   // moment partials: [B][P][packed width] for d in {16,32,64,128}, else
                                // [B][block pairs][P][64*64+64] (64 x 64 blocks, P sample chunks)
    double* d_part2 = nullptr;  // [B][ceil(P/32)][width] second level of the partial sum (MFMA path)
    int mom_wgs = 0;            // work-groups per basis of the MFMA moments kernel (P = streams * mom_wgs there)
    double* d_mom = nullptr;    // [B][d*d+d] reduced moments (sum x x^T, then sum x)
    unsigned long long* d_nsamp = nullptr;  // [B] sample slices the moment kernels of the last fit took in, counted by them
    double* d_bjA = nullptr;    // block Jacobi (d > 64): [B][n][n] the matrix, n = d padded to whole block pairs
    double* d_bjQ = nullptr;    // [B][pairs per round][2nb][2nb] rotations of the current round
    double* d_bjfro = nullptr;  // [B] squared Frobenius norm of the matrix, then [B][32][2] partial sums of its check
    int* d_jstate = nullptr;    // [B][4] its per-basis state
    int* d_sweeps = nullptr;    // [B] Jacobi sweeps used, -1 = not converged
    int* d_ksel = nullptr;      // [B] result of the last gvq_select_k
    float* d_loss_slice = nullptr;  // [S] per-slice squared residual of the last gvq_local_loss
    double* d_loss_part = nullptr;  // [B][loss_groups] partial sums of those
    int loss_groups = 1;
    int P = 0;                  // moment partials per basis
    int fit_L = 0;              // gradients of the last fit
    bool fit_first_slice = false;  // the last fit sampled only the first slice of every basis
    bool fitted = false;        // basis usable (fit or import)
    bool has_cov = false;       // d_cov / d_eig hold a fit's results
};

struct gvq_ptrs {
    const void* p[GVQ_MAX_PTRS];
};

// Records the HIP error text for gvq_strerror and returns GVQ_EHIP.
int gvq_hip_fail(hipError_t e, const char* what);

#define GVQ_HIP(call)                                         \
    do {                                                      \
        hipError_t e__ = (call);                              \
        if (e__ != hipSuccess) return gvq_hip_fail(e__, #call); \
    } while (0)

// Workgroups per compute unit for the streaming kernels (0 = pick from occupancy).
int gvq_opt_wg_per_cu();
// hipFuncSetAttribute acts on the current device: a launcher keeps one of these per kernel and raises the kernel's
// dynamic LDS limit the first time it runs on each device (devices 0 .. 63; not synchronised, like the launch options).
struct gvq_once_per_device {
    unsigned long long done = 0;
    bool first(int device)
    {
        const unsigned long long bit = 1ull << (device & 63);
        if (done & bit) return false;
        done |= bit;
        return true;
    }
};

// Tiles per run in the MFMA kernels' schedule (0 = default).
int gvq_opt_run_tiles();
// LDS-tiled codec kernels: 0 = pick the matrix pipe from the shape, 1 = fp32 products, 2 = the bf16 split,
// 3 = the bf16 split without the basis-stationary compress kernel.
int gvq_opt_long_mode();
// Bit mask: send every tile through the bounds-checked general phase (1: fp32-pipe compress, 2: bf16-pipe
// compress, 4: decompress).
int gvq_opt_no_fast();
// Pacing of the fast phase (CodecArgs::pace), -1 = each kernel's default.
int gvq_opt_pace();
// Super-tiles whose 1 KB rows interleave in the fast phase (CodecArgs::il), 0 = each kernel's default, 1 = none.
int gvq_opt_interleave();

// Kernel launchers (each only enqueues on `st`; returns GVQ_OK or GVQ_EHIP).
int gvq_launch_compress(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice,
                        int64_t n_slices, const float* comp_in, float* out, hipStream_t st);
int gvq_launch_aggregate(const gvq_basis* h, const float* const* comps, int N, float* out,
                         hipStream_t st);
int gvq_launch_decompress(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices,
                          void* out, gvq_dtype_t odt, hipStream_t st);
int gvq_launch_fit(gvq_basis* h, const void* const* grads, int L, bool first_slice_only, hipStream_t st);
int gvq_launch_local_loss(const gvq_basis* h, const void* grad, int n_workers, double* loss_out,
                          hipStream_t st);
int gvq_launch_local_loss_static(const gvq_basis* h, const void* grad, int n_workers, double* loss_out,
                                 hipStream_t st);
int gvq_launch_layout(const void* src, void* dst, int F, int D, int HW, gvq_dtype_t dtype, bool flatten,
                      hipStream_t st);
int gvq_launch_select_k(const gvq_basis* h, double lambda, hipStream_t st);
// Refresh the operand-order copies of U after d_U changed (no-op for non-MFMA shapes).
int gvq_launch_pack(const gvq_basis* h, hipStream_t st);
bool gvq_mfma_shape(int d, int k);
int gvq_build_plans(gvq_basis* h);   // fills h->plan (needs h_offs; no-op for one basis or other shapes)
bool gvq_bf16_pipe_shape(const gvq_basis* h);
bool gvq_moments_mfma_shape(int d);
int gvq_moments_packed_width(int d);
int gvq_moments_streams(int d);   // sample streams (partial slots) per work-group
// Moments in 64 x 64 blocks (every d other than 16, 32, 64, 128).
bool gvq_long_shape(int d, int k);            // codec: the LDS-tiled MFMA kernels take this shape (d > 128, or any
                                              // shape with k <= 128 that the register-resident kernels do not)
size_t gvq_long_pack_floats(int d, int k);    // floats per basis in either operand-order copy of U
size_t gvq_long_split_pack_halves(int d, int k);   // bf16 values per basis in either two-term copy of U
int64_t gvq_long_tiles(int64_t slices);       // 128-slice tiles that cover this many slices of one basis
int gvq_launch_pack_long(const gvq_basis* h, hipStream_t st);
int gvq_launch_compress_long(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice,
                             int64_t n_slices, const float* comp_in, float* out, hipStream_t st);
int gvq_launch_loss_long(const gvq_basis* h, const void* grad, int n_workers, float* loss_slice, hipStream_t st);
int gvq_launch_decompress_long(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices,
                               void* out, gvq_dtype_t odt, hipStream_t st);
// Basis-stationary compress kernel (gvq_codec_ws.hip): U stays in registers, the gradient streams past in tiles
// of 16 whole slices.  The launcher reports the slices done (the whole range, as far as the gradient has slices).
bool gvq_ws_shape(const gvq_basis* h);   // it can take this handle's shape
size_t gvq_ws_pack_halves(int d, int k);   // bf16 values of its operand-order copy of U
bool gvq_wsd_shape(const gvq_basis* h);  // the decompress kernel of the same kind can take the shape
size_t gvq_ws_alloc_halves(const gvq_basis* h);   // bf16 values of d_Uws: both kernels' copies
int gvq_launch_decompress_ws(const gvq_basis* h, const float* comp, int64_t first_slice, int64_t n_slices, void* out,
                             bool out_bf16, bool exact, hipStream_t st, int64_t* done);
int gvq_launch_pack_ws(const gvq_basis* h, hipStream_t st);
int gvq_launch_compress_ws(const gvq_basis* h, const void* grad, int n_workers, int64_t first_slice, int64_t n_slices,
                           const float* comp_in, float* out, bool exact, hipStream_t st, int64_t* done);
int gvq_large_groups(int d);
size_t gvq_large_partial_doubles(int d, int chunks);   // per basis
int gvq_launch_moments_large(gvq_basis* h, const void* const* grads, int L, hipStream_t st);
int gvq_bj_padded(int d);                  // block Jacobi: matrix size
size_t gvq_bj_q_doubles(int d);            // doubles per basis of its rotation buffer
int gvq_launch_eigen_block(gvq_basis* h, hipStream_t st);
