// clip.hip -- gradient clipping by global norm, per worker (App. C of arXiv 2310.14423:
// threshold 1 for parallel AdamW, 4 for Local AdamW with a constant period in the linear and
// step-decay runs, off in the QSR runs).  Two small kernels produce, for each of the K rows of
// the gradient buffer, the factor min(1, c / (||g_k||_2 + 1e-6)); the update kernels multiply
// the gradient by it as they read it, so clipping costs one more read of the gradients (4 B per
// replica-parameter) and no write.
// The sum of squares is deterministic: every lane adds its elements in index order with an
// error-free transformation of each addition, a workgroup combines its lanes in a fixed tree in
// double precision, and one workgroup per row adds the partial sums in index order.
#include <mutex>

#include "opt_elem.h"
#include "qsr_internal.h"

namespace qsr {

constexpr int CLIP_THREADS = 256;

// partial[k * nb + b] = sum of squares of the b-th chunk of row k
__global__ __launch_bounds__(CLIP_THREADS) void sqnorm_partial_kernel(
    const float *__restrict__ g, long long P, long long chunk, double *__restrict__ partial)
{
    __shared__ double red[CLIP_THREADS];
    const int k = blockIdx.y, b = blockIdx.x, nb = gridDim.x;
    const float *row = g + (long long)k * P;
    const long long i0 = (long long)b * chunk, i1 = min(P, i0 + chunk);
    float s = 0.f, c = 0.f;
    if ((((uintptr_t)(row + i0)) & 15) == 0) {
        const long long n4 = (i1 - i0) / 4;
        const float4 *r4 = (const float4 *)(row + i0);
        for (long long i = threadIdx.x; i < n4; i += CLIP_THREADS) {
            const float4 v = ld_nt4(r4 + i);
            add_comp(s, c, v.x * v.x); add_comp(s, c, v.y * v.y);
            add_comp(s, c, v.z * v.z); add_comp(s, c, v.w * v.w);
        }
        for (long long i = i0 + n4 * 4 + threadIdx.x; i < i1; i += CLIP_THREADS) add_comp(s, c, row[i] * row[i]);
    } else {
        for (long long i = i0 + threadIdx.x; i < i1; i += CLIP_THREADS) add_comp(s, c, row[i] * row[i]);
    }
    red[threadIdx.x] = (double)s + (double)c;
    __syncthreads();
    for (int w = CLIP_THREADS / 2; w > 0; w >>= 1) {
        if ((int)threadIdx.x < w) red[threadIdx.x] += red[threadIdx.x + w];
        __syncthreads();
    }
    if (threadIdx.x == 0) partial[(long long)k * nb + b] = red[0];
}

// coef[k] = min(1, max_norm / (sqrt(sum_b partial[k][b]) + 1e-6)); norm[k] = that square root
__global__ void clip_coef_kernel(const double *__restrict__ partial, int nb, float max_norm,
                                 float *__restrict__ coef, float *__restrict__ norm)
{
    if (threadIdx.x != 0) return;
    const int k = blockIdx.x;
    double ss = 0.0;
    for (int b = 0; b < nb; ++b) ss += partial[(long long)k * nb + b];
    const double nrm = sqrt(ss);
    const double cf = (double)max_norm / (nrm + 1e-6);
    coef[k] = cf < 1.0 ? (float)cf : 1.0f;
    norm[k] = (float)nrm;
}

int clip_blocks_per_row(long long P)
{
    long long nb = (P + 16383) / 16384;
    if (nb > 1024) nb = 1024;
    if (nb < 1) nb = 1;
    return (int)nb;
}

hipError_t launch_clip_coef(const float *g, int K, long long P, float max_norm, double *partial, float *coef,
                            float *norm, hipStream_t s)
{
    const int nb = clip_blocks_per_row(P);
    long long chunk = (P + nb - 1) / nb;
    chunk = (chunk + 3) / 4 * 4;                    // chunk starts stay 16-byte aligned where the row is
    sqnorm_partial_kernel<<<dim3((unsigned)nb, (unsigned)K), CLIP_THREADS, 0, s>>>(g, P, chunk, partial);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    clip_coef_kernel<<<K, 64, 0, s>>>(partial, nb, max_norm, coef, norm);
    return hipGetLastError();
}

}  // namespace qsr

// Stateless form for callers that hold gradients of their own (like qsr_average_rows for the
// All-Reduce line): the K factors and norms of a [K][P] gradient buffer, with the partial sums in a
// workspace the caller brings in.
extern "C" int qsr_clip_workspace_bytes(int32_t K, int64_t P, size_t *bytes)
{
    if (!bytes) return QSR_EINVAL;
    *bytes = 0;
    if (K < 1 || K > 65535 || P < 1 || P > ((long long)1 << 34)) return QSR_EINVAL;
    *bytes = (size_t)K * (size_t)qsr::clip_blocks_per_row(P) * sizeof(double);
    return QSR_OK;
}

static int clip_args_ok(const float *grads, int32_t K, int64_t P, float max_norm, const float *coef, const float *norm)
{
    if (!grads || !coef || !norm || K < 1 || K > 65535 || P < 1 || P > ((long long)1 << 34)) return 0;
    if (!(max_norm > 0.0f) || !(max_norm < INFINITY)) return 0;
    return 1;
}

extern "C" int qsr_clip_factors(const float *grads, int32_t K, int64_t P, float max_norm, void *workspace,
                                size_t workspace_bytes, float *coef, float *norm, void *stream)
{
    if (!clip_args_ok(grads, K, P, max_norm, coef, norm)) return QSR_EINVAL;
    if (!workspace || ((uintptr_t)workspace & 7) != 0) return QSR_EINVAL;
    size_t need = 0;
    (void)qsr_clip_workspace_bytes(K, P, &need);
    if (workspace_bytes < need) return QSR_ENOMEM;
    hipError_t e = qsr::launch_clip_coef(grads, K, P, max_norm, (double *)workspace, coef, norm, (hipStream_t)stream);
    if (e != hipSuccess) { qsr::set_last_hip_error((int)e); return QSR_EHIP; }
    return QSR_OK;
}


// ---------------------------------------------------------------------------------------------
// The same for callers that cannot allocate (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): the partial sums live in an array inside the library's device
// image, K * min(1024, ceil(P / 16384)) doubles, K <= 64: 512 KiB that every GPU the library runs
// on holds until the process ends.  All calls on one GPU share it: calls that overlap there
// (different streams, different threads) race on the partial sums.  Nothing has to start at zero:
// the first kernel writes every partial sum the second one reads.
// ---------------------------------------------------------------------------------------------
constexpr int CLIP_STATIC_MAX_K = 64;
constexpr int CLIP_STATIC_DOUBLES = CLIP_STATIC_MAX_K * 1024;
static __device__ __align__(256) double scratch[CLIP_STATIC_DOUBLES];

// In host code `scratch` is only a handle: the array's device address is asked for once per device,
// with that device current, and kept; each GPU holds its own copy at its own address.
constexpr int CLIP_MAX_DEVICES = 64;
static std::mutex g_scratch_mutex;
static double *g_scratch_ptr[CLIP_MAX_DEVICES];

int qsr::clip_static_setup(double **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { qsr::set_last_hip_error((int)e); return QSR_EHIP; }
    if (dev < 0 || dev >= CLIP_MAX_DEVICES) return QSR_ELIMIT;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        double *p = nullptr;
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) { qsr::set_last_hip_error((int)e); return QSR_EHIP; }
        if (!p) return QSR_EHIP;
        g_scratch_ptr[dev] = p;
    }
    if (out) *out = g_scratch_ptr[dev];
    return QSR_OK;
}

extern "C" int qsr_clip_factors_static(const float *grads, int32_t K, int64_t P, float max_norm, float *coef,
                                       float *norm, void *stream)
{
    if (!clip_args_ok(grads, K, P, max_norm, coef, norm)) return QSR_EINVAL;
    if (K > CLIP_STATIC_MAX_K) return QSR_ELIMIT;
    if ((long long)K * qsr::clip_blocks_per_row(P) > CLIP_STATIC_DOUBLES) return QSR_ELIMIT;
    double *partial = nullptr;
    const int rc = qsr::clip_static_setup(&partial);
    if (rc != QSR_OK) return rc;
    hipError_t e = qsr::launch_clip_coef(grads, K, P, max_norm, partial, coef, norm, (hipStream_t)stream);
    if (e != hipSuccess) { qsr::set_last_hip_error((int)e); return QSR_EHIP; }
    return QSR_OK;
}
