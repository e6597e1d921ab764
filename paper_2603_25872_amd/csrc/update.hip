// Elementwise sampler updates: guidance combine, the refinement chain of standard
// denoising updates, and the skip transitions that draft the next block, fused into
// one pass over the latent fields (Algorithm 1 / Algorithm 2, everything except the
// predictor).  HBM-bound: every input element is read once, every output written once.
#include "common.h"

namespace drf {

namespace {

template <typename V> struct VecTraits;
template <> struct VecTraits<float> { static constexpr int N = 1; };
template <> struct VecTraits<float4> { static constexpr int N = 4; };

__device__ inline float comp(const float& v, int) { return v; }
__device__ inline float comp(const float4& v, int i) { return i == 0 ? v.x : i == 1 ? v.y : i == 2 ? v.z : v.w; }
__device__ inline void setc(float& v, int, float s) { v = s; }
__device__ inline void setc(float4& v, int i, float s)
{
    if (i == 0) v.x = s; else if (i == 1) v.y = s; else if (i == 2) v.z = s; else v.w = s;
}

// Noise field f at vector index i, with guidance eps = eps_null + w (eps_cond - eps_null)
// when the pass carried (cond, null) slot pairs.
template <typename V>
__device__ inline V load_noise(const UpdateArgs& a, int f, size_t i, size_t nvec)
{
    const V* base = reinterpret_cast<const V*>(a.eps) + (size_t)f * a.g * nvec;
    V c = base[i];
    if (a.g == 2) {
        V u = base[nvec + i];
#pragma unroll
        for (int k = 0; k < VecTraits<V>::N; ++k) {
            float uu = comp(u, k);
            setc(c, k, fmaf(a.w, comp(c, k) - uu, uu));
        }
    }
    return c;
}

template <typename V>
__global__ void __launch_bounds__(256) update_kernel(const UpdateArgs a, size_t nvec)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < nvec; i += stride) {
        V y = reinterpret_cast<const V*>(a.x_base)[i];
        // refinement: standard updates replayed from the first draft (or anchor)
        for (int c = 0; c < a.n_chain; ++c) {
            V e = load_noise<V>(a, c, i, nvec);
#pragma unroll
            for (int k = 0; k < VecTraits<V>::N; ++k) setc(y, k, fmaf(a.cA[c], comp(y, k), a.cB[c] * comp(e, k)));
        }
        if (a.x_out) reinterpret_cast<V*>(a.x_out)[i] = y;
        // drafts for the next block by skip transitions from (y, anchor noise)
        if (a.n_draft > 0) {
            V e = load_noise<V>(a, a.anchor_field, i, nvec);
            for (int j = 0; j < a.n_draft; ++j) {
                V d;
#pragma unroll
                for (int k = 0; k < VecTraits<V>::N; ++k) setc(d, k, fmaf(a.dA[j], comp(y, k), a.dB[j] * comp(e, k)));
                reinterpret_cast<V*>(a.draft_out)[(size_t)j * nvec + i] = d;
            }
        }
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

drf_status launch_update(const UpdateArgs& a, hipStream_t st)
{
    if (a.field == 0) return DRF_OK;
    const bool vec = a.field % 4 == 0 && aligned16(a.x_base) && aligned16(a.eps) && aligned16(a.x_out) &&
                     aligned16(a.draft_out);
    const size_t nvec = vec ? a.field / 4 : a.field;
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;      // grid-stride beyond 32 blocks per CU
    if (vec)
        hipLaunchKernelGGL(update_kernel<float4>, dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    else
        hipLaunchKernelGGL(update_kernel<float>, dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf

using namespace drf;

extern "C" drf_status drf_skip_transition(const drf_sched_config* sched, const float* x_from, const float* eps_from,
                                          int s_from, const int* s_to, int m, int batch, size_t elems_per_sample,
                                          float* x_to, void* hip_stream)
{
    Schedule sch;
    drf_status rc = make_schedule(sched, &sch);
    if (rc != DRF_OK) return rc;
    if (m < 0 || batch < 0) DRF_FAIL(DRF_EINVAL, "m and batch must be >= 0");
    if (m == 0 || batch == 0 || elems_per_sample == 0) return DRF_OK;
    if (!x_from || !eps_from || !s_to || !x_to) DRF_FAIL(DRF_EINVAL, "NULL buffer");
    if (s_from < 0 || s_from > sch.steps) DRF_FAIL(DRF_EINVAL, "s_from %d outside [0, %d]", s_from, sch.steps);
    for (int j = 0; j < m; ++j)
        if (s_to[j] < 0 || s_to[j] > sch.steps) DRF_FAIL(DRF_EINVAL, "s_to[%d] = %d outside [0, %d]", j, s_to[j], sch.steps);
    const size_t field = (size_t)batch * elems_per_sample;
    for (int j0 = 0; j0 < m; j0 += kMaxBlock) {
        UpdateArgs a{};
        a.x_base = x_from; a.eps = eps_from; a.x_out = nullptr;
        a.draft_out = x_to + (size_t)j0 * field;
        a.field = field; a.g = 1; a.w = 0.f; a.n_chain = 0; a.anchor_field = 0;
        a.n_draft = m - j0 < kMaxBlock ? m - j0 : kMaxBlock;
        for (int j = 0; j < a.n_draft; ++j) sch.coef(s_from, s_to[j0 + j], &a.dA[j], &a.dB[j]);
        rc = launch_update(a, (hipStream_t)hip_stream);
        if (rc != DRF_OK) return rc;
    }
    return DRF_OK;
}

extern "C" drf_status drf_refine_step(const drf_sched_config* sched, const float* x, const float* eps, int s_from,
                                      int batch, size_t elems_per_sample, float* x_out, void* hip_stream)
{
    if (s_from < 1) DRF_FAIL(DRF_EINVAL, "s_from must be >= 1 (got %d)", s_from);
    const int to = s_from - 1;
    return drf_skip_transition(sched, x, eps, s_from, &to, 1, batch, elems_per_sample, x_out, hip_stream);
}
