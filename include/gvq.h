/*
 * gvq.h -- C ABI of libgvq: the GradiVeQ slice-wise linear PCA gradient codec for
 * AMD MI355X (gfx950).
 *
 * Notation.  A flattened gradient of M numbers is cut into S = ceil(M/d) slices of d
 * adjacent numbers (the paper's slice size K); each slice is projected onto k basis
 * vectors (the paper's d), so the compression ratio is d/k.  N is the number of workers
 * whose gradients are summed, L the number of gradients a basis is fitted on (the
 * paper's L_t).  A "basis" is the triple (U, mu, eig): U is d x k with orthonormal
 * columns, mu the length-d whitening vector, eig the d eigenvalues of the sample
 * covariance in decreasing order.  A gradient may be covered by several bases: basis b
 * serves the contiguous slice range [block_slice_offsets[b], block_slice_offsets[b+1]).
 *
 * Conventions for every entry point
 *   - return value: 0 (GVQ_OK) or a negative gvq_status_t; nothing throws or aborts;
 *   - "device" pointers are HIP device memory on the device that was current when the
 *     handle was created, owned by the caller, 16-byte aligned (else GVQ_EALIGN);
 *     "host" pointers are ordinary host memory, read or written before the call returns;
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  fit, compress,
 *     aggregate and decompress only enqueue kernels on it and never synchronise the device;
 *     buffers must stay valid until that work has finished;
 *   - the library owns the handle and the scratch memory inside it (allocated by
 *     gvq_basis_create, released by gvq_basis_destroy) and nothing else;
 *   - calls on one handle must not overlap in time on different streams;
 *   - the first launch of a kernel in a process asks the runtime once for its occupancy and,
 *     for some kernels, raises its LDS limit; these queries are not stream work, so call an
 *     entry point once on the shapes in use before capturing it into a HIP graph.
 *
 * Layouts
 *   gradient    : M elements, fp32 or bf16 (bit pattern in 16 bits), slice j = elements
 *                 [j*d, j*d+d); the last slice may be partial and is treated as zero-padded;
 *   compressed  : float [S][k], slice-major, so any range of slices is one contiguous
 *                 byte range (what a ring all-reduce segment needs);
 *   U           : float [B][d][k] row-major (B = number of bases);  mu: float [B][d];
 *   eig, cov    : double [B][d], double [B][d][d].
 */
#ifndef GVQ_H
#define GVQ_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gvq_basis gvq_basis_t; /* opaque */

typedef enum { GVQ_F32 = 0, GVQ_BF16 = 1 } gvq_dtype_t;

typedef enum {
    GVQ_OK = 0,
    GVQ_EINVAL = -1,     /* null pointer, size or count out of range, bad block offsets */
    GVQ_EALIGN = -2,     /* a device pointer is not 16-byte aligned */
    GVQ_ENOTFIT = -3,    /* compress / decompress / export before fit or import */
    GVQ_EHIP = -4,       /* a HIP call failed; gvq_strerror gives the HIP text */
    GVQ_ENOMEM = -5,     /* host or device allocation failed */
    GVQ_ENONFINITE = -6, /* gvq_fit_status: a fitted eigenvalue is NaN or Inf */
    GVQ_ENOCONV = -7,    /* gvq_fit_status: the eigensolver hit its sweep limit */
    GVQ_ETOOBIG = -8     /* gvq_local_loss_static: more slices or bases than its fixed scratch buffer holds */
} gvq_status_t;

#define GVQ_MAX_D 1024      /* largest supported slice length */
#define GVQ_STATIC_MAX_SLICES 2097152 /* most slices gvq_local_loss_static takes (2^21) */
#define GVQ_MAX_BASES 65535 /* most bases per handle (the basis index is a grid dimension of the fit kernels) */

/*
 * Create the codec state for gradients of n_elems (M >= 1) elements of grad_dtype, slice
 * length d in [2, GVQ_MAX_D], k in [1, d] kept components (the paper requires k < d; k = d
 * is accepted and makes the codec lossless), n_blocks in [1, GVQ_MAX_BASES] bases.  block_slice_offsets: host array of
 * n_blocks+1 strictly increasing slice indices, first 0, last S; NULL means one basis for
 * the whole gradient (n_blocks must then be 1).  Allocates the device copies of U, mu,
 * eig and the fit scratch on the current device.  Section 2 (slicing; one compressor per
 * group of slices, Section 3 "compressor reuse").
 * Speed by shape: d in {16,32,64,128} with k <= 32 runs register-resident kernels; every other
 * shape runs LDS-tiled kernels that take 128 comps per pass over the gradient, so k > 128 costs
 * ceil(k/128) passes (compress, and decompress to fp32).  Two calls keep slow any-shape kernels
 * when k > 128: decompress to bf16 output and gvq_local_loss.  The paper's setting (compression
 * ratio d/k >= 8, Section 4) never reaches k > 128 at d <= GVQ_MAX_D.
 */
int gvq_basis_create(gvq_basis_t** out, int64_t n_elems, int d, int k, int n_blocks,
                     const int64_t* block_slice_offsets, gvq_dtype_t grad_dtype);

/* Release the handle (the state of Section 2's compressor: U, mu, eig) and its device memory.
 * Synchronises the device first.  NULL is OK. */
int gvq_basis_destroy(gvq_basis_t* h);

/* S = ceil(M/d), the number of slices of Section 2 ("each gradient vector is cut into slices"), or
 * GVQ_EINVAL for a NULL handle. */
int64_t gvq_num_slices(const gvq_basis_t* h);

/*
 * Basis refresh (Section 2, PCA paragraph after Eq. 4).  grads: host array of L >= 1
 * device pointers, each a gradient of M elements of the handle's dtype; they are taken
 * as samples of the *aggregated* gradient.  For every basis b the sample set is every
 * full slice of its range in each of the L gradients (a partial tail slice is not a
 * sample): mu_b = sample mean, C_b = covariance with normaliser 1/n, accumulated in
 * float64 from exact products; C_b is eigendecomposed in float64 (Jacobi rotations),
 * eigenvalues sorted in decreasing order, U_b = eigenvectors of the k largest, each
 * negated if needed so that its largest-magnitude entry (lowest index on ties) is
 * positive.  Results stay on the device inside the handle.  A basis whose range holds
 * no full slice gets mu = 0, eig = 0 and U = the first k unit vectors.
 * Asynchronous on `stream`; the handle counts as fitted once this returns GVQ_OK.
 */
int gvq_fit_basis(gvq_basis_t* h, const void* const* grads, int L, void* stream);

/*
 * The paper's own sampling (Section 3, "compressor reuse"): like gvq_fit_basis, but the sample
 * set of basis b is its FIRST slice only -- L samples, one per gradient -- and the resulting
 * compressor is reused for the remaining slices of the range.  With L <= d the covariance is
 * rank deficient (rank <= L - 1): the trailing eigenvalues are zero and only the first
 * min(k, L - 1) columns of U are determined by the data.
 */
int gvq_fit_basis_first_slice(gvq_basis_t* h, const void* const* grads, int L, void* stream);

/*
 * Waits for `stream`'s work, then reports on the last fit: *max_sweeps (may be NULL)
 * receives the largest Jacobi sweep count over the bases.  Returns GVQ_ENOCONV if a basis
 * hit the sweep limit, GVQ_ENONFINITE if an eigenvalue is not finite (e.g. NaN/Inf in a
 * fit gradient), GVQ_ENOTFIT if no fit was run.
 */
int gvq_fit_status(const gvq_basis_t* h, int* max_sweeps, void* stream);

/*
 * Eq. (2): comp_out[j][:] = U_b^T (x_j - mu_b / n_workers) for every slice j of `grad`
 * (device, M elements of the handle's dtype), b the basis of slice j, the tail slice
 * zero-padded.  comp_out: device float [S][k].  n_workers >= 1 must equal the number of
 * vectors later summed by gvq_aggregate (only then do the mu/N terms add up to mu, Eq. 3);
 * the library cannot check this.  fp32 arithmetic, fp32 accumulation.  n_workers also sets the
 * cache policy of comp_out: when n_workers vectors of S*k floats fit the last-level cache together
 * (224 MB), comp_out is written so that it stays there for the sum that follows, otherwise with
 * non-temporal stores; the values are the same either way.
 */
int gvq_compress(const gvq_basis_t* h, const void* grad, int n_workers, float* comp_out,
                 void* stream);

/*
 * Eq. (3): comp_sum = comps[0] + comps[1] + ... + comps[N-1], element-wise over S*k
 * floats, added in that order in fp32.  comps: host array of N >= 1 device pointers.
 * comp_sum may alias comps[0] only.
 */
int gvq_aggregate(const gvq_basis_t* h, const float* const* comps, int N, float* comp_sum,
                  void* stream);

/*
 * Eq. (4): grad_out[j*d + e] = (U_b comp_sum[j][:])[e] + mu_b[e], for the first M elements.
 * grad_out: device, M elements of out_dtype (bf16 is rounded to nearest even).
 */
int gvq_decompress(const gvq_basis_t* h, const float* comp_sum, void* grad_out,
                   gvq_dtype_t out_dtype, void* stream);

/*
 * Section 2 (gradient packing, Fig. 2a): reorder the gradient of one convolution layer, stored
 * [F][D][H][W] (filters, depth, height, width -- the usual weight layout), into the flat order
 * the codec slices:  flat[((h*W + w)*D + d)*F + f] = grad[f][d][h][w], i.e. the F collocated
 * gradients of the F filters are adjacent and the groups run along depth, then width, then
 * height.  gvq_unflatten_conv is the inverse.  Both pointers are device memory of F*D*H*W
 * elements of `dtype`, aligned to the element size, not overlapping.  No handle: a model's
 * layers are flattened one call each into their places of the big gradient vector.
 */
int gvq_flatten_conv(const void* grad, void* flat, int F, int D, int H, int W, gvq_dtype_t dtype,
                     void* stream);
int gvq_unflatten_conv(const void* flat, void* grad, int F, int D, int H, int W, gvq_dtype_t dtype,
                       void* stream);

/*
 * Building blocks of Algorithm 1 (compression overlapped with the ring all-reduce): the same
 * operations restricted to the slices [first_slice, first_slice + n_slices), one ring segment.
 * All buffers are the full-size ones; only the segment's rows (elements) are read and written,
 * at their usual positions, so a segment of the compressed vector is the contiguous byte range
 * comp + first_slice*k.  0 <= first_slice, first_slice + n_slices <= S.
 *
 * gvq_compress_segment: comp_out[j][:] = Q(x_j) (Eq. 2) + comp_in[j][:] for j in the segment;
 * comp_in (device, may be NULL = nothing to add, may equal comp_out) is the partial sum
 * received from the predecessor -- one fused step of Algorithm 1's compression round, which
 * saves a separate pass over the compressed data.
 * gvq_decompress_segment: Eq. (4) on the segment's slices (decompression round).
 */
int gvq_compress_segment(const gvq_basis_t* h, const void* grad, int n_workers, int64_t first_slice,
                         int64_t n_slices, const float* comp_in, float* comp_out, void* stream);
int gvq_decompress_segment(const gvq_basis_t* h, const float* comp_sum, int64_t first_slice,
                           int64_t n_slices, void* grad_out, gvq_dtype_t out_dtype, void* stream);

/*
 * Section 3, Eq. (6): the local compression loss of one worker's gradient,
 *     loss_out[b] = sum over the slices of basis b of || x - (U_b y + mu_b/N) ||^2,
 *     y = U_b^T (x - mu_b/N)   (Eq. 2),
 * which a node watches to decide when the basis needs a refresh.  grad: device, M elements
 * of the handle's dtype; loss_out: device double [B] (8-byte aligned).  The tail slice is
 * projected zero-padded but only its real elements count.  The gradient is read once;
 * nothing else of its size is written.  fp32 arithmetic per slice, float64 sums over slices
 * in a fixed order.  Asynchronous on `stream`.
 */
int gvq_local_loss(const gvq_basis_t* h, const void* grad, int n_workers, double* loss_out,
                   void* stream);

/*
 * gvq_local_loss for callers that cannot allocate device memory and cannot let a library do it for
 * them: code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, same kernels and same result as gvq_local_loss, but the scratch of the two reduction
 * stages (one float per slice, then a few partial sums per basis) lives in a fixed buffer inside the
 * library, about 8.5 MB per GPU, held until the process ends, instead of in the handle.  The call
 * allocates and frees nothing.  Limits: S <= GVQ_STATIC_MAX_SLICES slices and (bases x partial sums
 * per basis) <= 65536, else GVQ_ETOOBIG; the handle's device must be the current device (GVQ_EINVAL).
 * All calls on one GPU share the buffer, whatever the handle or stream: calls that overlap in time on
 * one GPU race, and the buffer keeps the last call's contents (every entry a call reads it has
 * written itself).  As for every entry point, call it once on the shapes in use before capturing it
 * into a HIP graph.
 */
int gvq_local_loss_static(const gvq_basis_t* h, const void* grad, int n_workers, double* loss_out,
                          void* stream);

/*
 * Section 3, Eq. (5): for every basis of the last fit, the smallest k such that
 * (eig[0] + ... + eig[k-1]) / (eig[0] + ... + eig[d-1]) >= 1 - lambda, 0 <= lambda < 1 (1 when
 * the eigenvalue sum is not positive).  k_out: host int [B].  Advisory: the handle keeps the
 * k it was created with.  Waits for `stream`.  GVQ_ENOTFIT unless gvq_fit_basis ran.
 */
int gvq_select_k(const gvq_basis_t* h, double lambda, int* k_out, void* stream);

/*
 * Checkpoint of the codec state that the PCA paragraph of Section 2 defines (the eigen matrix cut to
 * its first k columns, the whitening vector, the eigenvalue vector): copy the basis to host arrays
 * (any may be NULL): U float [B][d][k], mu float [B][d], eig double [B][d].  Synchronises the device.
 * eig is all zero after gvq_basis_import.
 */
int gvq_basis_export(const gvq_basis_t* h, float* U, float* mu, double* eig);

/*
 * Diagnostics of the last fit (Section 2, PCA paragraph): host copy of the covariance matrices,
 * double [B][d][d] (what the eigensolver was given), and of the per-basis sample counts, int64 [B],
 * as the moment kernels counted the slices they took in (either may be NULL).  Synchronises the
 * device.  GVQ_ENOTFIT unless gvq_fit_basis ran on this handle.
 */
int gvq_basis_export_cov(const gvq_basis_t* h, double* cov, int64_t* n_samples);

/*
 * Restore of that checkpoint: replace the basis by host arrays U float [B][d][k] and mu float [B][d]
 * (the two parts of the state that Eqs. 2 and 4 use; also lets a test inject a basis).  U is used as
 * given: no orthonormality check.  Synchronous.
 */
int gvq_basis_import(gvq_basis_t* h, const float* U, const float* mu);

/*
 * Text for a status code.  For GVQ_EHIP the text includes the message of the most recent
 * failed HIP call in this process.  The pointer stays valid until the next call.
 */
const char* gvq_strerror(int status);

/*
 * Launch tuning (benchmarks only), process-wide; value 0 restores the default.
 *   option 0: workgroups per compute unit for the streaming kernels;
 *   option 1: consecutive 16-slice tiles a wave takes before it jumps ahead by the width
 *             of the whole grid (1 = interleave single tiles, large = one chunk per wave);
 *   option 2: matrix pipe of the long-slice codec kernels (slices longer than 128 elements, and
 *             shorter shapes other than d in {16,32,64,128} with k <= 32): 0 = exact fp32
 *             products where they keep up with memory (2dk/(4(d+k)) < 10 flop per byte),
 *             else products of two-term bf16 splits with fp32 accumulation (each product good to
 *             about 1e-5 of its magnitude, results within 1e-5 of the exact ones relative to the
 *             largest value, up to 2 times faster); 1 = always exact products; 2 = always the split;
 *             3 = always the split, and never the kernels that keep U in registers (the default
 *             for fp32 gradients with one basis and d a multiple of 256; for A/B timing);
 *   option 3: bit mask that sends every tile of a kernel family through its bounds-checked general loop
 *             instead of the branch-free loop over whole tiles (1: fp32-pipe compress, 2: bf16-pipe
 *             compress, 4: decompress); results are identical, for A/B timing;
 *   option 4: pacing of the branch-free loop, -1 = each kernel's default: bit 0 = a wave waits for all its
 *             memory work before it parks the next tile, bit 1 = also after a tile's matrix products,
 *             bit 2 = the matrix products wait for the next tile's loads one by one;
 *   option 5: with one basis, the number of consecutive super-tiles (2048 elements each) of the branch-free
 *             loop whose 1 KB rows interleave, so that the waves running side by side sweep one compact
 *             window of memory row by row; 1 = none, at most 4096; results are identical.
 * The options are plain process-wide variables read at launch time: set them while no other thread is
 * inside a libgvq call.  Returns GVQ_EINVAL for unknown options or values out of range.
 */
int gvq_set_option(int option, int value);

#ifdef __cplusplus
}
#endif
#endif /* GVQ_H */
