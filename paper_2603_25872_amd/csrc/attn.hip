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
// max of three without the canonicalisation the generic fmaxf lowering adds per operand
__device__ inline float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
constexpr float kTau = 8.f;         // lazy-rescale headroom of the online softmax, in log2 units

// KS = ceil(d / 16) k-steps of the score MFMA; DT = ceil(d / 32) row tiles of O^T.
// Per step 64 kv rows: two 32 x 32 score tiles, one online-softmax update, four PV k-chunks.
// The next K/V tile is fetched into registers while the current one is being used.
template <int KS, int DT>
__global__ void __launch_bounds__(256) attn_bf16_kernel(const AttnArgs a, float scale_log2)
{
    constexpr int DK = KS * 16, LDKS = DK + 8, LDV = kKvb + 8;
    constexpr int MAXCH = (kKvb * (KS * 2) + 255) / 256;                   // 16-byte chunks of a tile per thread
    __shared__ __attribute__((aligned(16))) bf16_t sK[kKvb * LDKS];        // [kv][d padded]
    __shared__ __attribute__((aligned(16))) bf16_t sVt[DT * 32 * LDV];      // [d padded][kv]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int slot = blockIdx.z, h = blockIdx.y, d = a.d;
    const int kvb = a.kv_mod ? slot % a.kv_mod : slot;
    const bf16_t* Q = (const bf16_t*)a.q + slot * a.q_slot_stride + h * a.q_head_stride;
    const bf16_t* Kp = (const bf16_t*)a.k + kvb * a.kv_batch_stride + h * a.kv_head_stride;
    const bf16_t* Vp = (const bf16_t*)a.v + kvb * a.kv_batch_stride + h * a.kv_head_stride;

    // zero the padding that loads never touch: K columns [d, DK), V^T rows [d, DT*32)
    for (int i = tid; i < kKvb * LDKS; i += 256) sK[i] = (bf16_t)0.f;
    for (int i = tid; i < DT * 32 * LDV; i += 256) sVt[i] = (bf16_t)0.f;
    // When the head width leaves a padding row in O^T, V^T row d is set to ones: the PV MFMA
    // then accumulates the softmax denominator there for free.
    const bool ones_row = d < DT * 32;
    __syncthreads();
    if (ones_row)
        for (int i = tid; i < LDV; i += 256) sVt[d * LDV + i] = (bf16_t)1.f;

    // this lane's query column and its Q fragments (B operand: 8 consecutive d per k-step half)
    const int q = blockIdx.x * kQPerBlock + wave * 32 + l32;
    const int qc = q < a.Nq ? q : a.Nq - 1;
    const bf16x8 zero8 = { 0, 0, 0, 0, 0, 0, 0, 0 };
    bf16x8 qf[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        const int dd = ks * 16 + half * 8;
        qf[ks] = dd < d ? *reinterpret_cast<const bf16x8*>(Q + (size_t)qc * a.ldq + dd) : zero8;
    }
    f32x16 o[DT];
#pragma unroll
    for (int t = 0; t < DT; ++t)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;      // running max of the raw scores, running sum
    const int dch = d / 8, nch = kKvb * dch;    // 16-byte chunks per row / per tile

    // K chunks: consecutive threads take consecutive 16-byte chunks of a row (coalesced loads,
    // 16-byte LDS writes).  V chunks: consecutive threads take consecutive kv rows of one chunk
    // column, so that the transposing 2-byte LDS writes of a wave fall on consecutive addresses.
    bf16x8 rk[MAXCH], rv[MAXCH];
    auto fetch = [&](int kv0) {
#pragma unroll
        for (int c = 0; c < MAXCH; ++c) {
            const int id = tid + c * 256;
            const int rk_r = id / dch, rk_c = id % dch, rv_c = id / kKvb, rv_r = id % kKvb;
            rk[c] = zero8; rv[c] = zero8;
            if (id < nch) {
                if (kv0 + rk_r < a.Nk) rk[c] = *reinterpret_cast<const bf16x8*>(Kp + (size_t)(kv0 + rk_r) * a.ldk + rk_c * 8);
                if (kv0 + rv_r < a.Nk) rv[c] = *reinterpret_cast<const bf16x8*>(Vp + (size_t)(kv0 + rv_r) * a.ldk + rv_c * 8);
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int c = 0; c < MAXCH; ++c) {
            const int id = tid + c * 256;
            const int rk_r = id / dch, rk_c = id % dch, rv_c = id / kKvb, rv_r = id % kKvb;
            if (id < nch) {
                *reinterpret_cast<bf16x8*>(sK + rk_r * LDKS + rk_c * 8) = rk[c];
#pragma unroll
                for (int e = 0; e < 8; ++e) sVt[(rv_c * 8 + e) * LDV + rv_r] = rv[c][e];
            }
        }
    };

    fetch(0);
    for (int kv0 = 0; kv0 < a.Nk; kv0 += kKvb) {
        __syncthreads();                    // previous tile fully consumed (and zero fill done)
        stage();
        __syncthreads();
        if (kv0 + kKvb < a.Nk) fetch(kv0 + kKvb);
        // S^T[kv][q] = sum_d K[kv][d] Q[q][d] for the two 32-row halves of the tile
        f32x16 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const f32x16 zero16 = { 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f };
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                bf16x8 kf = *reinterpret_cast<const bf16x8*>(sK + (t * 32 + l32) * LDKS + ks * 16 + half * 8);
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], ks == 0 ? zero16 : s[t], 0, 0, 0);
            }
        }
        // register r of s[t] holds kv row t*32 + 8*(r/4) + 4*half + r%4 of the tile
        if (kv0 + kKvb > a.Nk) {            // ragged last tile: rows past the end do not take part
#pragma unroll
            for (int t = 0; t < 2; ++t)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (kv0 + t * 32 + 8 * (r >> 2) + 4 * half + (r & 3) >= a.Nk) s[t][r] = -INFINITY;
        }
        float mx = max3(s[0][0], s[1][0], s[0][1]);
#pragma unroll
        for (int r = 1; r < 16; ++r) mx = r < 15 ? max3(mx, s[1][r], s[0][r + 1]) : fmaxf(mx, s[1][15]);
        mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
        // Lazy rescaling: exponents are taken against a reference m_run that only moves when some
        // query of the wave would otherwise exceed 2^kTau; until then P stays <= 2^kTau (fine for
        // bf16 operands and fp32 sums) and the accumulators need no rescale.
        if (__any((mx - m_run) * scale_log2 > kTau)) {
            const float m_new = fmaxf(m_run, mx);
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);   // 0 on the first tile
            m_run = m_new;
            l_run *= alpha;
#pragma unroll
            for (int tt = 0; tt < DT; ++tt)
#pragma unroll
                for (int r = 0; r < 16; ++r) o[tt][r] *= alpha;
        }
        const float ms = m_run * scale_log2;
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) s[t][r] = __builtin_amdgcn_exp2f(fmaf(s[t][r], scale_log2, -ms));
        if (!ones_row) {
            float psum = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) psum += s[0][r] + s[1][r];
            l_run += psum;                  // this half's share; the halves are added at the end
        }
        // O^T[d][q] += sum_kv V^T[d][kv] P^T[kv][q]; element e of a lane's k-slice is kv row
        // 16c + 4*half + e (e < 4) or 16c + 8 + 4*half + e - 4 of the 32-row half, for both operands.
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                bf16x8 pf;
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) pf[e2] = (bf16_t)s[t][8 * c + e2];
#pragma unroll
                for (int tt = 0; tt < DT; ++tt) {
                    const bf16_t* vp = sVt + (tt * 32 + l32) * LDV + t * 32 + 16 * c + 4 * half;
                    bf16x4 v0 = *reinterpret_cast<const bf16x4*>(vp);
                    bf16x4 v1 = *reinterpret_cast<const bf16x4*>(vp + 8);
                    bf16x8 vf = __builtin_shufflevector(v0, v1, 0, 1, 2, 3, 4, 5, 6, 7);
                    o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf, o[tt], 0, 0, 0);
                }
            }
    }
    // denominator: from the ones row (kept by the lanes of one half) or the two halves' partial sums
    float l_tot;
    if (ones_row) {
        const int tt = d >> 5, lr = d & 31, r = 4 * (lr >> 3) + (lr & 3), owner = (lr >> 2) & 1;
        float mine = 0.f;
#pragma unroll
        for (int t2 = 0; t2 < DT; ++t2)
#pragma unroll
            for (int r2 = 0; r2 < 16; ++r2) mine = (t2 == tt && r2 == r) ? o[t2][r2] : mine;
        const float other = __shfl_xor(mine, 32, 64);
        l_tot = half == owner ? mine : other;
    } else {
        l_tot = l_run + __shfl_xor(l_run, 32, 64);
    }
    if (q >= a.Nq) return;
    const float inv = 1.f / l_tot;
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
    const float* Q = (const float*)a.q + slot * a.q_slot_stride + h * a.q_head_stride + (size_t)q * a.ldq;
    const float* Kp = (const float*)a.k + kvb * a.kv_batch_stride + h * a.kv_head_stride;
    const float* Vp = (const float*)a.v + kvb * a.kv_batch_stride + h * a.kv_head_stride;
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
