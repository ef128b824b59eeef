// C ABI of libgvq: argument checking, handle life cycle, host<->device copies of the basis.
// All arithmetic of the codec runs in the HIP kernels (gvq_codec.hip, gvq_fit.hip).
#include <math.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <new>

#include "gvq_internal.h"

static thread_local char g_hip_msg[256] = "no HIP error recorded";
static thread_local char g_msg[320];
static int g_wg_per_cu = 0;
static int g_run_tiles = 0;
static int g_long_mode = 0;
static int g_no_fast = 0;
static int g_pace = -1;
static int g_interleave = 0;

int gvq_hip_fail(hipError_t e, const char* what)
{
    snprintf(g_hip_msg, sizeof g_hip_msg, "%s: %s", what, hipGetErrorString(e));
    (void)hipGetLastError();  // clear the sticky error
    return GVQ_EHIP;
}

int gvq_opt_wg_per_cu() { return g_wg_per_cu; }
int gvq_opt_run_tiles() { return g_run_tiles; }
int gvq_opt_long_mode() { return g_long_mode; }
int gvq_opt_no_fast() { return g_no_fast; }
int gvq_opt_pace() { return g_pace; }
int gvq_opt_interleave() { return g_interleave; }

static bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

extern "C" {

const char* gvq_strerror(int status)
{
    switch (status) {
    case GVQ_OK: return "ok";
    case GVQ_EINVAL: return "invalid argument";
    case GVQ_EALIGN: return "device pointer is not 16-byte aligned";
    case GVQ_ENOTFIT: return "basis not fitted or imported";
    case GVQ_EHIP:
        snprintf(g_msg, sizeof g_msg, "HIP call failed (%s)", g_hip_msg);
        return g_msg;
    case GVQ_ENOMEM: return "out of memory";
    case GVQ_ENONFINITE: return "fit produced a non-finite eigenvalue";
    case GVQ_ENOCONV: return "eigensolver did not converge";
    case GVQ_ETOOBIG: return "size exceeds the static scratch buffer of this entry point";
    default: return "unknown status";
    }
}

int gvq_set_option(int option, int value)
{
    if (option == 0 && value >= 0 && value <= 64) { g_wg_per_cu = value; return GVQ_OK; }
    if (option == 1 && value >= 0) { g_run_tiles = value; return GVQ_OK; }
    if (option == 2 && value >= 0 && value <= 3) { g_long_mode = value; return GVQ_OK; }
    if (option == 3 && value >= 0 && value <= 7) { g_no_fast = value; return GVQ_OK; }
    if (option == 4 && value >= -1 && value <= 7) { g_pace = value; return GVQ_OK; }
    if (option == 5 && value >= 0 && value <= 4096) { g_interleave = value; return GVQ_OK; }
    return GVQ_EINVAL;
}

int gvq_basis_destroy(gvq_basis_t* h)
{
    if (!h) return GVQ_OK;
    (void)hipDeviceSynchronize();
    void* dev[] = {h->d_offs, h->d_tile_block, h->d_U, h->d_Upc, h->d_Upd, h->d_Upb, h->d_Uws, h->d_Umu, h->d_mu, h->d_eig, h->d_cov, h->d_V, h->d_part, h->d_part2, h->d_mom, h->d_nsamp, h->d_bjA, h->d_bjQ, h->d_bjfro, h->d_jstate, h->d_ltile, h->d_sweeps, h->d_ksel, h->d_loss_slice, h->d_loss_part};
    for (void* p : dev)
        if (p) (void)hipFree(p);
    for (gvq_plan& pl : h->plan) {
        if (pl.d_sup_tile) (void)hipFree(pl.d_sup_tile);
        if (pl.d_sup_basis) (void)hipFree(pl.d_sup_basis);
        if (pl.d_rest) (void)hipFree(pl.d_rest);
    }
    free(h->h_offs);
    free(h->h_ltile);
    delete h;
    (void)hipGetLastError();
    return GVQ_OK;
}

int gvq_basis_create(gvq_basis_t** out, int64_t n_elems, int d, int k, int n_blocks,
                     const int64_t* offs, gvq_dtype_t dtype)
{
    if (!out) return GVQ_EINVAL;
    *out = nullptr;
    if (n_elems < 1 || d < 2 || d > GVQ_MAX_D || k < 1 || k > d || n_blocks < 1 || n_blocks > GVQ_MAX_BASES)
        return GVQ_EINVAL;
    if (dtype != GVQ_F32 && dtype != GVQ_BF16) return GVQ_EINVAL;
    const int64_t S = (n_elems + d - 1) / d;
    if (!offs && n_blocks != 1) return GVQ_EINVAL;
    if (offs) {
        if (n_blocks > S || offs[0] != 0 || offs[n_blocks] != S) return GVQ_EINVAL;
        for (int b = 0; b < n_blocks; ++b)
            if (offs[b + 1] <= offs[b]) return GVQ_EINVAL;
    }
    gvq_basis* h = new (std::nothrow) gvq_basis();
    if (!h) return GVQ_ENOMEM;
    h->M = n_elems; h->S = S; h->d = d; h->k = k; h->B = n_blocks; h->dtype = dtype;
    h->h_offs = (int64_t*)malloc(sizeof(int64_t) * (n_blocks + 1));
    if (!h->h_offs) { delete h; return GVQ_ENOMEM; }
    if (offs) memcpy(h->h_offs, offs, sizeof(int64_t) * (n_blocks + 1));
    else { h->h_offs[0] = 0; h->h_offs[1] = S; }

    // moment partials per basis: enough workgroups to fill the chip, never more than one
    // per 64 sample slices of the largest basis
    int64_t longest = 0;
    for (int b = 0; b < n_blocks; ++b)
        if (h->h_offs[b + 1] - h->h_offs[b] > longest) longest = h->h_offs[b + 1] - h->h_offs[b];

    int rc = GVQ_OK;
    hipError_t e;
#define TRY(call) do { e = (call); if (e != hipSuccess) { rc = gvq_hip_fail(e, #call); goto fail; } } while (0)
    {
        hipDeviceProp_t prop;
        TRY(hipGetDevice(&h->device));
        TRY(hipGetDeviceProperties(&prop, h->device));
        h->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
        size_t width = (size_t)d * d + d;
        size_t part_doubles = 0;   // per basis, when not P * width
        if (!gvq_moments_mfma_shape(d)) {
            // one wave per (64 x 64 block, sample chunk): as many chunks as fill, but do not exceed, the
            // two waves per SIMD the kernel runs at (one wave more would cost a whole second round),
            // never less than 64 sample slices per chunk
            const int64_t ng = gvq_large_groups(d), npairs = ng * (ng + 1) / 2;
            int64_t chunks = (8LL * h->num_cu) / (npairs * n_blocks);
            if (chunks > (longest + 63) / 64) chunks = (longest + 63) / 64;
            if (chunks < 1) chunks = 1;
            h->P = (int)chunks;
            part_doubles = gvq_large_partial_doubles(d, h->P);
        } else {
            // two work-groups of 4 waves per compute unit, spread over the bases (rounded down: every
            // work-group runs for the whole launch, so a few more than fit would cost a second
            // round as long as the first); never less than 64 sample slices per stream
            const int streams = gvq_moments_streams(d);
            int64_t wgs = (2LL * h->num_cu) / n_blocks;
            if (wgs > (longest + 64LL * streams - 1) / (64LL * streams)) wgs = (longest + 64LL * streams - 1) / (64LL * streams);
            if (wgs < 1) wgs = 1;
            h->mom_wgs = (int)wgs;
            h->P = (int)wgs * streams;
            width = (size_t)gvq_moments_packed_width(d);
        }
        const size_t B = (size_t)n_blocks, W = (size_t)d * d + d, n = (size_t)(d + (d & 1));
        TRY(hipMalloc((void**)&h->d_offs, sizeof(int64_t) * (B + 1)));
        TRY(hipMalloc((void**)&h->d_U, sizeof(float) * B * d * k));
        TRY(hipMalloc((void**)&h->d_mu, sizeof(float) * B * d));
        if (gvq_long_shape(d, k)) {
            const size_t pf = gvq_long_pack_floats(d, k);
            TRY(hipMalloc((void**)&h->d_Upc, sizeof(float) * B * pf));
            TRY(hipMalloc((void**)&h->d_Upd, sizeof(float) * B * pf));
            TRY(hipMalloc((void**)&h->d_Upb, sizeof(unsigned short) * B * 2 * gvq_long_split_pack_halves(d, k)));
            if (gvq_ws_alloc_halves(h)) TRY(hipMalloc((void**)&h->d_Uws, sizeof(unsigned short) * gvq_ws_alloc_halves(h)));
            if (n_blocks > 1) {
                h->h_ltile = (int64_t*)malloc(sizeof(int64_t) * (B + 1));
                if (!h->h_ltile) { rc = GVQ_ENOMEM; goto fail; }
                h->h_ltile[0] = 0;
                for (int b = 0; b < n_blocks; ++b)
                    h->h_ltile[b + 1] = h->h_ltile[b] + gvq_long_tiles(h->h_offs[b + 1] - h->h_offs[b]);
                TRY(hipMalloc((void**)&h->d_ltile, sizeof(int64_t) * (B + 1)));
                TRY(hipMemcpy(h->d_ltile, h->h_ltile, sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice));
            }
        } else if (gvq_mfma_shape(d, k)) {
            const size_t kp = k <= 16 ? 16 : 32;
            TRY(hipMalloc((void**)&h->d_Upc, sizeof(float) * B * d * kp));
            TRY(hipMalloc((void**)&h->d_Upd, sizeof(float) * B * d * kp));
            if (gvq_bf16_pipe_shape(h)) {
                TRY(hipMalloc((void**)&h->d_Upb, sizeof(unsigned short) * B * d * kp * 3));
                TRY(hipMalloc((void**)&h->d_Umu, sizeof(float) * B * kp));
            }
        }
        TRY(hipMalloc((void**)&h->d_eig, sizeof(double) * B * d));
        TRY(hipMalloc((void**)&h->d_cov, sizeof(double) * B * d * d));
        if (d > GVQ_LDS_EIGEN_MAX_D) {
            const size_t np = (size_t)gvq_bj_padded(d);
            TRY(hipMalloc((void**)&h->d_V, sizeof(double) * B * np * np));
            TRY(hipMalloc((void**)&h->d_bjA, sizeof(double) * B * np * np));
            TRY(hipMalloc((void**)&h->d_bjQ, sizeof(double) * B * gvq_bj_q_doubles(d)));
            TRY(hipMalloc((void**)&h->d_bjfro, sizeof(double) * B * (1 + 2 * 32)));   // norm, then the check's partial sums
            TRY(hipMalloc((void**)&h->d_jstate, sizeof(int) * B * 4));
        } else {
            TRY(hipMalloc((void**)&h->d_V, sizeof(double) * B * n * n));
        }
        if (part_doubles) {
            TRY(hipMalloc((void**)&h->d_part, sizeof(double) * B * part_doubles));
        } else {
            TRY(hipMalloc((void**)&h->d_part, sizeof(double) * B * (size_t)h->P * width));
            TRY(hipMalloc((void**)&h->d_part2, sizeof(double) * B * (size_t)((h->P + 31) / 32) * width));
        }
        TRY(hipMalloc((void**)&h->d_mom, sizeof(double) * B * W));
        TRY(hipMalloc((void**)&h->d_nsamp, sizeof(unsigned long long) * B));
        TRY(hipMalloc((void**)&h->d_sweeps, sizeof(int) * B));
        TRY(hipMalloc((void**)&h->d_ksel, sizeof(int) * B));
        TRY(hipMalloc((void**)&h->d_loss_slice, sizeof(float) * (size_t)S));
        h->loss_groups = (int)((longest + 4095) / 4096);
        if (h->loss_groups > 256) h->loss_groups = 256;
        if (h->loss_groups < 1) h->loss_groups = 1;
        TRY(hipMalloc((void**)&h->d_loss_part, sizeof(double) * B * (size_t)h->loss_groups));
        TRY(hipMemcpy(h->d_offs, h->h_offs, sizeof(int64_t) * (B + 1), hipMemcpyHostToDevice));
        if (n_blocks > 1) {
            const int64_t T = (S + 15) / 16;
            int* tb = (int*)malloc(sizeof(int) * (size_t)T);
            if (!tb) { rc = GVQ_ENOMEM; goto fail; }
            int b = 0;
            for (int64_t t = 0; t < T; ++t) {
                while (h->h_offs[b + 1] <= t * 16) ++b;
                tb[t] = b;
            }
            e = hipMalloc((void**)&h->d_tile_block, sizeof(int) * (size_t)T);
            if (e == hipSuccess) e = hipMemcpy(h->d_tile_block, tb, sizeof(int) * (size_t)T, hipMemcpyHostToDevice);
            free(tb);
            if (e != hipSuccess) { rc = gvq_hip_fail(e, "tile_block upload"); goto fail; }
        }
        TRY(hipMemset(h->d_eig, 0, sizeof(double) * B * d));
        rc = gvq_build_plans(h);
        if (rc != GVQ_OK) goto fail;
    }
#undef TRY
    *out = h;
    return GVQ_OK;
fail:
    gvq_basis_destroy(h);
    return rc;
}

int64_t gvq_num_slices(const gvq_basis_t* h) { return h ? h->S : (int64_t)GVQ_EINVAL; }

static int fit_call(gvq_basis_t* h, const void* const* grads, int L, bool first_slice_only, void* stream)
{
    if (!h || !grads || L < 1) return GVQ_EINVAL;
    for (int l = 0; l < L; ++l) {
        if (!grads[l]) return GVQ_EINVAL;
        if (!aligned16(grads[l])) return GVQ_EALIGN;
    }
    int rc = gvq_launch_fit(h, grads, L, first_slice_only, (hipStream_t)stream);
    if (rc != GVQ_OK) return rc;
    h->fitted = true;
    h->has_cov = true;
    h->fit_L = L;
    h->fit_first_slice = first_slice_only;
    return GVQ_OK;
}

int gvq_fit_basis(gvq_basis_t* h, const void* const* grads, int L, void* stream)
{
    return fit_call(h, grads, L, false, stream);
}

int gvq_fit_basis_first_slice(gvq_basis_t* h, const void* const* grads, int L, void* stream)
{
    return fit_call(h, grads, L, true, stream);
}

int gvq_fit_status(const gvq_basis_t* h, int* max_sweeps, void* stream)
{
    if (!h) return GVQ_EINVAL;
    if (!h->has_cov) return GVQ_ENOTFIT;
    GVQ_HIP(hipStreamSynchronize((hipStream_t)stream));
    const size_t B = (size_t)h->B;
    int* sw = (int*)malloc(sizeof(int) * B);
    double* eig = (double*)malloc(sizeof(double) * B * h->d);
    if (!sw || !eig) { free(sw); free(eig); return GVQ_ENOMEM; }
    hipError_t e1 = hipMemcpy(sw, h->d_sweeps, sizeof(int) * B, hipMemcpyDeviceToHost);
    hipError_t e2 = hipMemcpy(eig, h->d_eig, sizeof(double) * B * h->d, hipMemcpyDeviceToHost);
    int rc = GVQ_OK;
    if (e1 != hipSuccess) rc = gvq_hip_fail(e1, "hipMemcpy(sweeps)");
    else if (e2 != hipSuccess) rc = gvq_hip_fail(e2, "hipMemcpy(eig)");
    else {
        int mx = 0;
        bool noconv = false, nonfinite = false;
        for (size_t b = 0; b < B; ++b) {
            if (sw[b] < 0) noconv = true;
            else if (sw[b] > mx) mx = sw[b];
        }
        for (size_t i = 0; i < B * h->d; ++i)
            if (!isfinite(eig[i])) nonfinite = true;
        if (max_sweeps) *max_sweeps = mx;
        if (nonfinite) rc = GVQ_ENONFINITE;
        else if (noconv) rc = GVQ_ENOCONV;
    }
    free(sw); free(eig);
    return rc;
}

int gvq_compress(const gvq_basis_t* h, const void* grad, int n_workers, float* comp_out, void* stream)
{
    if (!h || !grad || !comp_out || n_workers < 1) return GVQ_EINVAL;
    if (!aligned16(grad) || !aligned16(comp_out)) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    return gvq_launch_compress(h, grad, n_workers, 0, h->S, nullptr, comp_out, (hipStream_t)stream);
}

int gvq_compress_segment(const gvq_basis_t* h, const void* grad, int n_workers, int64_t first_slice,
                         int64_t n_slices, const float* comp_in, float* comp_out, void* stream)
{
    if (!h || !grad || !comp_out || n_workers < 1) return GVQ_EINVAL;
    if (first_slice < 0 || n_slices < 0 || first_slice > h->S || n_slices > h->S - first_slice) return GVQ_EINVAL;
    if (!aligned16(grad) || !aligned16(comp_out) || (comp_in && !aligned16(comp_in))) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    if (n_slices == 0) return GVQ_OK;
    return gvq_launch_compress(h, grad, n_workers, first_slice, n_slices, comp_in, comp_out, (hipStream_t)stream);
}

int gvq_aggregate(const gvq_basis_t* h, const float* const* comps, int N, float* comp_sum, void* stream)
{
    if (!h || !comps || !comp_sum || N < 1) return GVQ_EINVAL;
    if (!aligned16(comp_sum)) return GVQ_EALIGN;
    for (int n = 0; n < N; ++n) {
        if (!comps[n]) return GVQ_EINVAL;
        if (!aligned16(comps[n])) return GVQ_EALIGN;
        if (n > 0 && comps[n] == comp_sum) return GVQ_EINVAL;  // only comps[0] may alias the output
    }
    return gvq_launch_aggregate(h, comps, N, comp_sum, (hipStream_t)stream);
}

int gvq_decompress(const gvq_basis_t* h, const float* comp_sum, void* grad_out, gvq_dtype_t out_dtype,
                   void* stream)
{
    if (!h || !comp_sum || !grad_out) return GVQ_EINVAL;
    if (out_dtype != GVQ_F32 && out_dtype != GVQ_BF16) return GVQ_EINVAL;
    if (!aligned16(comp_sum) || !aligned16(grad_out)) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    return gvq_launch_decompress(h, comp_sum, 0, h->S, grad_out, out_dtype, (hipStream_t)stream);
}

int gvq_decompress_segment(const gvq_basis_t* h, const float* comp_sum, int64_t first_slice, int64_t n_slices,
                           void* grad_out, gvq_dtype_t out_dtype, void* stream)
{
    if (!h || !comp_sum || !grad_out) return GVQ_EINVAL;
    if (out_dtype != GVQ_F32 && out_dtype != GVQ_BF16) return GVQ_EINVAL;
    if (first_slice < 0 || n_slices < 0 || first_slice > h->S || n_slices > h->S - first_slice) return GVQ_EINVAL;
    if (!aligned16(comp_sum) || !aligned16(grad_out)) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    if (n_slices == 0) return GVQ_OK;
    return gvq_launch_decompress(h, comp_sum, first_slice, n_slices, grad_out, out_dtype, (hipStream_t)stream);
}

int gvq_local_loss(const gvq_basis_t* h, const void* grad, int n_workers, double* loss_out, void* stream)
{
    if (!h || !grad || !loss_out || n_workers < 1) return GVQ_EINVAL;
    if (!aligned16(grad) || ((uintptr_t)loss_out & 7u)) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    return gvq_launch_local_loss(h, grad, n_workers, loss_out, (hipStream_t)stream);
}

int gvq_local_loss_static(const gvq_basis_t* h, const void* grad, int n_workers, double* loss_out, void* stream)
{
    if (!h || !grad || !loss_out || n_workers < 1) return GVQ_EINVAL;
    if (!aligned16(grad) || ((uintptr_t)loss_out & 7u)) return GVQ_EALIGN;
    if (!h->fitted) return GVQ_ENOTFIT;
    return gvq_launch_local_loss_static(h, grad, n_workers, loss_out, (hipStream_t)stream);
}

int gvq_select_k(const gvq_basis_t* h, double lambda, int* k_out, void* stream)
{
    if (!h || !k_out || !(lambda >= 0.0) || !(lambda < 1.0)) return GVQ_EINVAL;
    if (!h->has_cov) return GVQ_ENOTFIT;
    int rc = gvq_launch_select_k(h, lambda, (hipStream_t)stream);
    if (rc != GVQ_OK) return rc;
    GVQ_HIP(hipStreamSynchronize((hipStream_t)stream));
    GVQ_HIP(hipMemcpy(k_out, h->d_ksel, sizeof(int) * (size_t)h->B, hipMemcpyDeviceToHost));
    return GVQ_OK;
}

static int layout_call(const void* src, void* dst, int F, int D, int H, int W, gvq_dtype_t dtype, bool flatten,
                       void* stream)
{
    if (!src || !dst || src == dst || F < 1 || D < 1 || H < 1 || W < 1) return GVQ_EINVAL;
    if (dtype != GVQ_F32 && dtype != GVQ_BF16) return GVQ_EINVAL;
    if ((int64_t)H * W > (1 << 20) || (int64_t)F * D * H * W > ((int64_t)1 << 40)) return GVQ_EINVAL;
    const uintptr_t mask = dtype == GVQ_BF16 ? 1u : 3u;
    if (((uintptr_t)src & mask) || ((uintptr_t)dst & mask)) return GVQ_EALIGN;
    return gvq_launch_layout(src, dst, F, D, H * W, dtype, flatten, (hipStream_t)stream);
}

int gvq_flatten_conv(const void* grad, void* flat, int F, int D, int H, int W, gvq_dtype_t dtype, void* stream)
{
    return layout_call(grad, flat, F, D, H, W, dtype, true, stream);
}

int gvq_unflatten_conv(const void* flat, void* grad, int F, int D, int H, int W, gvq_dtype_t dtype, void* stream)
{
    return layout_call(flat, grad, F, D, H, W, dtype, false, stream);
}

int gvq_basis_export(const gvq_basis_t* h, float* U, float* mu, double* eig)
{
    if (!h) return GVQ_EINVAL;
    if (!h->fitted) return GVQ_ENOTFIT;
    GVQ_HIP(hipDeviceSynchronize());
    const size_t B = (size_t)h->B;
    if (U) GVQ_HIP(hipMemcpy(U, h->d_U, sizeof(float) * B * h->d * h->k, hipMemcpyDeviceToHost));
    if (mu) GVQ_HIP(hipMemcpy(mu, h->d_mu, sizeof(float) * B * h->d, hipMemcpyDeviceToHost));
    if (eig) GVQ_HIP(hipMemcpy(eig, h->d_eig, sizeof(double) * B * h->d, hipMemcpyDeviceToHost));
    return GVQ_OK;
}

int gvq_basis_export_cov(const gvq_basis_t* h, double* cov, int64_t* n_samples)
{
    if (!h) return GVQ_EINVAL;
    if (!h->has_cov) return GVQ_ENOTFIT;
    GVQ_HIP(hipDeviceSynchronize());
    const size_t B = (size_t)h->B;
    if (cov) GVQ_HIP(hipMemcpy(cov, h->d_cov, sizeof(double) * B * h->d * h->d, hipMemcpyDeviceToHost));
    if (n_samples) {
        static_assert(sizeof(unsigned long long) == sizeof(int64_t), "sample counters are copied as they are");
        GVQ_HIP(hipMemcpy(n_samples, h->d_nsamp, sizeof(int64_t) * B, hipMemcpyDeviceToHost));
    }
    return GVQ_OK;
}

int gvq_basis_import(gvq_basis_t* h, const float* U, const float* mu)
{
    if (!h || !U || !mu) return GVQ_EINVAL;
    GVQ_HIP(hipDeviceSynchronize());
    const size_t B = (size_t)h->B;
    GVQ_HIP(hipMemcpy(h->d_U, U, sizeof(float) * B * h->d * h->k, hipMemcpyHostToDevice));
    GVQ_HIP(hipMemcpy(h->d_mu, mu, sizeof(float) * B * h->d, hipMemcpyHostToDevice));
    GVQ_HIP(hipMemset(h->d_eig, 0, sizeof(double) * B * h->d));
    {
        int rc = gvq_launch_pack(h, nullptr);
        if (rc != GVQ_OK) return rc;
    }
    GVQ_HIP(hipDeviceSynchronize());
    h->fitted = true;
    h->has_cov = false;
    return GVQ_OK;
}

}  // extern "C"
