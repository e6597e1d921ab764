// Multi-head attention softmax(q k^T / sqrt(d)) v without mask.
// bf16 path: flash-style, one wave per 32 queries, scores computed transposed
// (S^T = K Q^T) so that each lane owns one query column and the online softmax needs a
// single cross-lane exchange; P^T feeds the second MFMA straight from registers.
// fp32 path: one thread per query, for the fp32 configuration.
#include "common.h"

namespace drf {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kKvb = 64;            // kv rows staged per step
constexpr int kQPerBlock = 128;     // 4 waves x 32 queries

// KS = ceil(d / 16) k-steps of the score MFMA; DT = ceil(d / 32) row tiles of O^T.
template <int KS, int DT>
__global__ void __launch_bounds__(256) attn_bf16_kernel(const AttnArgs a, float scale_log2)
{
    constexpr int DK = KS * 16, LDKS = DK + 8, LDV = kKvb + 8;
    __shared__ __attribute__((aligned(16))) bf16_t sK[kKvb * LDKS];        // [kv][d padded]
    __shared__ __attribute__((aligned(16))) bf16_t sVt[DT * 32 * LDV];      // [d padded][kv]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int slot = blockIdx.z, h = blockIdx.y, d = a.d;
    const int kvb = a.kv_mod ? slot % a.kv_mod : slot;
    const bf16_t* Q = (const bf16_t*)a.q + (size_t)slot * a.Nq * a.ldq + h * d;
    const bf16_t* Kp = (const bf16_t*)a.k + (size_t)kvb * a.Nk * a.ldk + h * d;
    const bf16_t* Vp = (const bf16_t*)a.v + (size_t)kvb * a.Nk * a.ldk + h * d;

    // zero the padding that loads never touch: K columns [d, DK), V^T rows [d, DT*32)
    for (int i = tid; i < kKvb * LDKS; i += 256) sK[i] = (bf16_t)0.f;
    for (int i = tid; i < DT * 32 * LDV; i += 256) sVt[i] = (bf16_t)0.f;

    // this lane's query column and its Q fragments (B operand: 8 consecutive d per k-step half)
    const int q = blockIdx.x * kQPerBlock + wave * 32 + l32;
    const int qc = q < a.Nq ? q : a.Nq - 1;
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int dd = ks * 16 + half * 8;
        bf16x8 z = { 0, 0, 0, 0, 0, 0, 0, 0 };
        qf[ks] = dd < d ? *reinterpret_cast<const bf16x8*>(Q + (size_t)qc * a.ldq + dd) : z;
    }
    f32x16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;
    const int dch = d / 8;                  // 16-byte chunks per row

    for (int kv0 = 0; kv0 < a.Nk; kv0 += kKvb) {
        __syncthreads();                    // previous tile fully consumed (and zero fill done)
        for (int id = tid; id < kKvb * dch; id += 256) {
            const int r = id / dch, c = id % dch, kv = kv0 + r;
            bf16x8 kk = { 0, 0, 0, 0, 0, 0, 0, 0 }, vv = kk;
            if (kv < a.Nk) {
                kk = *reinterpret_cast<const bf16x8*>(Kp + (size_t)kv * a.ldk + c * 8);
                vv = *reinterpret_cast<const bf16x8*>(Vp + (size_t)kv * a.ldk + c * 8);
            }
            *reinterpret_cast<bf16x8*>(sK + r * LDKS + c * 8) = kk;
#pragma unroll
            for (int e = 0; e < 8; ++e) sVt[(c * 8 + e) * LDV + r] = vv[e];
        }
        __syncthreads();
#pragma unroll
        for (int t = 0; t < kKvb / 32; ++t) {
            if (kv0 + t * 32 >= a.Nk) break;          // uniform: whole sub-tile past the end
            // S^T[kv][q] = sum_d K[kv][d] Q[q][d]
            f32x16 s;
#pragma unroll
            for (int r = 0; r < 16; ++r) s[r] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + (t * 32 + l32) * LDKS + ks * 16 + half * 8);
                s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s, 0, 0, 0);
            }
            // register r of this lane holds kv row 8*(r/4) + 4*half + r%4 of the sub-tile
            float mx = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int kv = kv0 + t * 32 + 8 * (r >> 2) + 4 * half + (r & 3);
                s[r] = kv < a.Nk ? s[r] * scale_log2 : -INFINITY;
                mx = fmaxf(mx, s[r]);
            }
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run, mx);
            const float alpha = exp2f(m_run - m_new);
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) { s[r] = exp2f(s[r] - m_new); psum += s[r]; }
            psum += __shfl_xor(psum, 32, 64);
            l_run = l_run * alpha + psum;
            m_run = m_new;
#pragma unroll
            for (int tt = 0; tt < DT; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[tt][r] *= alpha;
            // O^T[d][q] += sum_kv V^T[d][kv] P^T[kv][q]; element e of a lane's k-slice is kv row
            // 16c + 4*half + e (e < 4) or 16c + 8 + 4*half + e - 4, for both operands alike.
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                bf16x8 pf;
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) pf[e2] = (bf16_t)s[8 * c + e2];
#pragma unroll
                for (int tt = 0; tt < DT; ++tt) {
                    const bf16_t* vp = sVt + (tt * 32 + l32) * LDV + t * 32 + 16 * c + 4 * half;
                    bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vp);
                    bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vp + 8);
                    bf16x8 vf = { v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3] };
                    o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[tt], 0, 0, 0);
                }
            }
        }
    }
    if (q >= a.Nq) return;
    const float inv = 1.f / l_run;
    bf16_t* op = (bf16_t*)a.out + ((size_t)slot * a.Nq + q) * a.ldo + h * d;
#pragma unroll
    for (int tt = 0; tt < DT; ++tt)
#pragma unroll
        for (int g4 = 0; g4 < 4; ++g4) {
            const int dd = tt * 32 + 8 * g4 + 4 * half;
            if (dd < d) {
                bf16x4 w = { (bf16_t)(o[tt][4 * g4] * inv), (bf16_t)(o[tt][4 * g4 + 1] * inv),
                             (bf16_t)(o[tt][4 * g4 + 2] * inv), (bf16_t)(o[tt][4 * g4 + 3] * inv) };
                *reinterpret_cast<bf16x4*>(op + dd) = w;
            }
        }
}

// fp32: one thread per query, online softmax over kv rows read through the cache.
constexpr int kF32MaxD = 128;
__global__ void __launch_bounds__(128) attn_f32_kernel(const AttnArgs a, float scale)
{
    const int slot = blockIdx.z, h = blockIdx.y, d = a.d;
    const int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q >= a.Nq) return;
    const int kvb = a.kv_mod ? slot % a.kv_mod : slot;
    const float* Q = (const float*)a.q + ((size_t)slot * a.Nq + q) * a.ldq + h * d;
    const float* Kp = (const float*)a.k + (size_t)kvb * a.Nk * a.ldk + h * d;
    const float* Vp = (const float*)a.v + (size_t)kvb * a.Nk * a.ldk + h * d;
    float qv[kF32MaxD], o[kF32MaxD];
    for (int e = 0; e < d; ++e) { qv[e] = Q[e] * scale; o[e] = 0.f; }
    float m_run = -INFINITY, l_run = 0.f;
    for (int j = 0; j < a.Nk; ++j) {
        const float* kr = Kp + (size_t)j * a.ldk;
        float s = 0.f;
        for (int e = 0; e < d; ++e) s = fmaf(qv[e], kr[e], s);
        const float m_new = fmaxf(m_run, s);
        const float alpha = expf(m_run - m_new), p = expf(s - m_new);
        l_run = l_run * alpha + p;
        m_run = m_new;
        const float* vr = Vp + (size_t)j * a.ldk;
        for (int e = 0; e < d; ++e) o[e] = fmaf(o[e], alpha, p * vr[e]);
    }
    float* op = (float*)a.out + ((size_t)slot * a.Nq + q) * a.ldo + h * d;
    const float inv = 1.f / l_run;
    for (int e = 0; e < d; ++e) op[e] = o[e] * inv;
}

template <int KS, int DT>
drf_status launch_bf16_inst(const AttnArgs& a, float scale_log2, hipStream_t st)
{
    const dim3 grid((a.Nq + kQPerBlock - 1) / kQPerBlock, a.heads, a.slots);
    hipLaunchKernelGGL((attn_bf16_kernel<KS, DT>), grid, dim3(256), 0, st, a, scale_log2);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace

drf_status launch_attn_bf16(const AttnArgs& a, hipStream_t st)
{
    if (a.slots == 0 || a.Nq == 0) return DRF_OK;
    if (a.Nk < 1 || a.d % 8 != 0 || a.d > 96 || a.ldq % 8 != 0 || a.ldk % 8 != 0 || a.ldo % 4 != 0)
        DRF_FAIL(DRF_ESHAPE, "bf16 attention needs head dim %% 8 == 0 and <= 96 (got %d)", a.d);
    const float sl2 = 1.4426950408889634f / sqrtf((float)a.d);
    switch ((a.d + 15) / 16) {
    case 1: return launch_bf16_inst<1, 1>(a, sl2, st);
    case 2: return launch_bf16_inst<2, 1>(a, sl2, st);
    case 3: return launch_bf16_inst<3, 2>(a, sl2, st);
    case 4: return launch_bf16_inst<4, 2>(a, sl2, st);
    case 5: return launch_bf16_inst<5, 3>(a, sl2, st);
    default: return launch_bf16_inst<6, 3>(a, sl2, st);
    }
}

drf_status launch_attn_f32(const AttnArgs& a, hipStream_t st)
{
    if (a.slots == 0 || a.Nq == 0) return DRF_OK;
    if (a.Nk < 1 || a.d > kF32MaxD) DRF_FAIL(DRF_ESHAPE, "fp32 attention needs head dim <= %d (got %d)", kF32MaxD, a.d);
    const dim3 grid((a.Nq + 127) / 128, a.heads, a.slots);
    hipLaunchKernelGGL(attn_f32_kernel, grid, dim3(128), 0, st, a, 1.f / sqrtf((float)a.d));
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf
