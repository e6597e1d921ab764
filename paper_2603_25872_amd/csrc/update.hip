// Elementwise sampler updates: guidance combine, the refinement chain of standard
// denoising updates, and the skip transitions that draft the next block, fused into
// one pass over the latent fields (Algorithm 1 / Algorithm 2, everything except the
// predictor).  HBM-bound: every input element is read once, every output written once.
#include "common.h"
#include "../../include/drf_measure.h"

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

// Philox4x32 with 10 rounds (Salmon et al., SC'11): a keyed bijection of the 128-bit counter.
__device__ inline uint4 philox4x32_10(uint4 c, uint32_t k0, uint32_t k1)
{
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hi0 = __umulhi(0xD2511F53u, c.x), lo0 = 0xD2511F53u * c.x;
        const uint32_t hi1 = __umulhi(0xCD9E8D57u, c.z), lo1 = 0xCD9E8D57u * c.z;
        c = make_uint4(hi1 ^ c.y ^ k0, lo1, hi0 ^ c.w ^ k1, lo0);
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return c;
}

// Two standard normals from two random words (Box-Muller).  u = ((r >> 9) + 1/2) 2^-23 has 24
// significant bits, so it is the same number in every precision and lies strictly inside (0, 1).
__device__ inline void box_muller(uint32_t ra, uint32_t rb, float* n0, float* n1)
{
    const float ua = ((float)(ra >> 9) + 0.5f) * 0x1p-23f;
    const float ub = ((float)(rb >> 9) + 0.5f) * 0x1p-23f;
    const float rad = sqrtf(-2.f * logf(ua));
    float sn, cs;
    sincospif(2.f * ub, &sn, &cs);
    *n0 = rad * cs;
    *n1 = rad * sn;
}

// The four normals of block q of noise field `field` (elements 4q .. 4q+3 of that field).
__device__ inline float4 normal_block(uint64_t seed, uint32_t field, size_t q)
{
    const uint4 r = philox4x32_10(make_uint4((uint32_t)q, (uint32_t)((uint64_t)q >> 32), field, 0u), (uint32_t)seed,
                                  (uint32_t)(seed >> 32));
    float4 z;
    box_muller(r.x, r.y, &z.x, &z.y);
    box_muller(r.z, r.w, &z.z, &z.w);
    return z;
}

// Fresh noise field `ordinal` of this call at vector index i.
template <typename V> __device__ inline V load_fresh(const UpdateArgs& a, int ordinal, size_t i, size_t nvec);
template <> __device__ inline float4 load_fresh<float4>(const UpdateArgs& a, int ordinal, size_t i, size_t nvec)
{
    if (a.noise_mode == NOISE_EXPLICIT) return reinterpret_cast<const float4*>(a.z)[(size_t)ordinal * nvec + i];
    return normal_block(a.seed, a.z_field0 + (uint32_t)ordinal, i);
}
template <> __device__ inline float load_fresh<float>(const UpdateArgs& a, int ordinal, size_t i, size_t nvec)
{
    if (a.noise_mode == NOISE_EXPLICIT) return a.z[(size_t)ordinal * nvec + i];
    return comp(normal_block(a.seed, a.z_field0 + (uint32_t)ordinal, i >> 2), (int)(i & 3));
}

template <typename V, bool NOISE>
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
            if (NOISE && a.cC[c] != 0.f) {
                V z = load_fresh<V>(a, a.cz[c], i, nvec);
#pragma unroll
                for (int k = 0; k < VecTraits<V>::N; ++k) setc(y, k, fmaf(a.cC[c], comp(z, k), comp(y, k)));
            }
        }
        if (a.x_out) reinterpret_cast<V*>(a.x_out)[i] = y;
        // drafts for the next block by skip transitions from (y, anchor noise)
        if (a.n_draft > 0) {
            V e = load_noise<V>(a, a.anchor_field, i, nvec);
            for (int j = 0; j < a.n_draft; ++j) {
                V d;
#pragma unroll
                for (int k = 0; k < VecTraits<V>::N; ++k) setc(d, k, fmaf(a.dA[j], comp(y, k), a.dB[j] * comp(e, k)));
                if (NOISE && a.dC[j] != 0.f) {
                    V z = load_fresh<V>(a, a.dz[j], i, nvec);
#pragma unroll
                    for (int k = 0; k < VecTraits<V>::N; ++k) setc(d, k, fmaf(a.dC[j], comp(z, k), comp(d, k)));
                }
                reinterpret_cast<V*>(a.draft_out)[(size_t)j * nvec + i] = d;
            }
        }
    }
}

__global__ void __launch_bounds__(256) normal_fill_kernel(uint64_t seed, uint32_t field0, size_t n_fields, size_t F,
                                                          float* out)
{
    const size_t blocks_per_field = (F + 3) / 4, total = n_fields * blocks_per_field;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
        const size_t f = i / blocks_per_field, q = i - f * blocks_per_field;
        const float4 z = normal_block(seed, field0 + (uint32_t)f, q);
        float* o = out + f * F + 4 * q;
        const size_t left = F - 4 * q;
        o[0] = z.x;
        if (left > 1) o[1] = z.y;
        if (left > 2) o[2] = z.z;
        if (left > 3) o[3] = z.w;
    }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

}  // namespace

drf_status launch_update(const UpdateArgs& a, hipStream_t st)
{
    if (a.field == 0) return DRF_OK;
    const bool vec = a.field % 4 == 0 && aligned16(a.x_base) && aligned16(a.eps) && aligned16(a.x_out) &&
                     aligned16(a.draft_out) && aligned16(a.z);
    const size_t nvec = vec ? a.field / 4 : a.field;
    size_t blocks = (nvec + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;      // grid-stride beyond 32 blocks per CU
    const bool noise = a.noise_mode != NOISE_NONE;
    if (vec && noise)
        hipLaunchKernelGGL((update_kernel<float4, true>), dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    else if (vec)
        hipLaunchKernelGGL((update_kernel<float4, false>), dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    else if (noise)
        hipLaunchKernelGGL((update_kernel<float, true>), dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    else
        hipLaunchKernelGGL((update_kernel<float, false>), dim3((unsigned)blocks), dim3(256), 0, st, a, nvec);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf

using namespace drf;

extern "C" drf_status drf_skip_transition_noise(const drf_sched_config* sched, const float* x_from,
                                                const float* net_from, int s_from, const int* s_to, int m, int batch,
                                                size_t elems_per_sample, const drf_noise* noise, float* x_to,
                                                void* hip_stream)
{
    Schedule sch;
    drf_status rc = make_schedule(sched, &sch);
    if (rc != DRF_OK) return rc;
    if (m < 0 || batch < 0) DRF_FAIL(DRF_EINVAL, "m and batch must be >= 0");
    if (m == 0 || batch == 0 || elems_per_sample == 0) return DRF_OK;
    if (!x_from || !net_from || !s_to || !x_to) DRF_FAIL(DRF_EINVAL, "NULL buffer");
    if (s_from < 0 || s_from > sch.steps) DRF_FAIL(DRF_EINVAL, "s_from %d outside [0, %d]", s_from, sch.steps);
    for (int j = 0; j < m; ++j)
        if (s_to[j] < 0 || s_to[j] > sch.steps) DRF_FAIL(DRF_EINVAL, "s_to[%d] = %d outside [0, %d]", j, s_to[j], sch.steps);
    const size_t field = (size_t)batch * elems_per_sample;
    // all argument blocks are validated before the first launch
    std::vector<UpdateArgs> launches;
    for (int j0 = 0; j0 < m; j0 += kMaxBlock) {
        UpdateArgs a{};
        a.x_base = x_from; a.eps = net_from; a.x_out = nullptr;
        a.draft_out = x_to + (size_t)j0 * field;
        a.field = field; a.g = 1; a.w = 0.f; a.n_chain = 0; a.anchor_field = 0;
        a.n_draft = m - j0 < kMaxBlock ? m - j0 : kMaxBlock;
        for (int j = 0; j < a.n_draft; ++j) {
            rc = sch.coef(s_from, s_to[j0 + j], &a.dA[j], &a.dB[j], &a.dC[j]);
            if (rc != DRF_OK) return rc;
            a.dz[j] = j0 + j;
        }
        rc = set_noise_source(&a, noise);
        if (rc != DRF_OK) return rc;
        launches.push_back(a);
    }
    for (const UpdateArgs& a : launches) {
        rc = launch_update(a, (hipStream_t)hip_stream);
        if (rc != DRF_OK) return rc;
    }
    return DRF_OK;
}

extern "C" drf_status drf_skip_transition(const drf_sched_config* sched, const float* x_from, const float* eps_from,
                                          int s_from, const int* s_to, int m, int batch, size_t elems_per_sample,
                                          float* x_to, void* hip_stream)
{
    return drf_skip_transition_noise(sched, x_from, eps_from, s_from, s_to, m, batch, elems_per_sample, nullptr, x_to,
                                     hip_stream);
}

extern "C" drf_status drf_normal_fill(uint64_t seed, uint32_t field0, size_t n_fields, size_t field_elems, float* out,
                                      void* hip_stream)
{
    if (n_fields == 0 || field_elems == 0) return DRF_OK;
    if (!out) DRF_FAIL(DRF_EINVAL, "out is NULL");
    if ((uint64_t)field0 + n_fields > 0x100000000ull) DRF_FAIL(DRF_EINVAL, "field numbers must stay below 2^32");
    const size_t total = n_fields * ((field_elems + 3) / 4);
    size_t blocks = (total + 255) / 256;
    if (blocks > 256 * 32) blocks = 256 * 32;
    hipLaunchKernelGGL(normal_fill_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream, seed, field0,
                       n_fields, field_elems, out);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

extern "C" drf_status drf_refine_step(const drf_sched_config* sched, const float* x, const float* eps, int s_from,
                                      int batch, size_t elems_per_sample, float* x_out, void* hip_stream)
{
    if (s_from < 1) DRF_FAIL(DRF_EINVAL, "s_from must be >= 1 (got %d)", s_from);
    const int to = s_from - 1;
    return drf_skip_transition(sched, x, eps, s_from, &to, 1, batch, elems_per_sample, x_out, hip_stream);
}

extern "C" drf_status drf_probe_update_fused(const drf_sched_config* sched, int s_from, int n_chain, int n_draft, int g,
                                             float w, size_t field, const float* x_base, const float* eps, float* x_out,
                                             float* draft_out, void* hip_stream)
{
    Schedule sch;
    drf_status rc = make_schedule(sched, &sch);
    if (rc != DRF_OK) return rc;
    if (sch.stochastic()) DRF_FAIL(DRF_EINVAL, "the probe takes samplers without variance");
    if (n_chain < 0 || n_draft < 0 || n_chain > kMaxBlock || n_draft > kMaxBlock || (g != 1 && g != 2))
        DRF_FAIL(DRF_EINVAL, "bad chain / draft / guidance counts");
    if (s_from < 0 || s_from > sch.steps || s_from - n_chain - n_draft < 0) DRF_FAIL(DRF_EINVAL, "chain and drafts run past index 0");
    if (field == 0) return DRF_OK;
    if (!x_base || !eps || (n_draft > 0 && !draft_out) || (!x_out && n_draft == 0)) DRF_FAIL(DRF_EINVAL, "NULL buffer");
    UpdateArgs a{};
    a.x_base = x_base; a.eps = eps; a.x_out = x_out; a.draft_out = n_draft > 0 ? draft_out : nullptr;
    a.field = field; a.g = g; a.w = w; a.n_chain = n_chain; a.n_draft = n_draft;
    a.anchor_field = n_chain > 0 ? n_chain - 1 : 0;
    float c_unused = 0.f;
    for (int i = 0; i < n_chain; ++i)
        if ((rc = sch.coef(s_from - i, s_from - i - 1, &a.cA[i], &a.cB[i], &c_unused)) != DRF_OK) return rc;
    const int s_mid = s_from - n_chain;
    for (int j = 0; j < n_draft; ++j)
        if ((rc = sch.coef(s_mid, s_mid - j - 1, &a.dA[j], &a.dB[j], &c_unused)) != DRF_OK) return rc;
    if ((rc = set_noise_source(&a, nullptr)) != DRF_OK) return rc;
    return launch_update(a, (hipStream_t)hip_stream);
}
