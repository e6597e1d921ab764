// Bandwidth-bound pieces of the DiT forward: conditioning front-end, patch embedding,
// LayerNorm + adaLN modulation, final projection + unpatchify.
#include "common.h"

namespace drf {

namespace {

constexpr int kWave = 64;
constexpr int kTFreq = 256;

__device__ inline float wave_sum(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

__device__ inline float silu(float v) { return v / (1.f + __expf(-v)); }

__device__ inline int slot_tau(const SlotMap& m, int slot) { return m.t_dev ? m.t_dev[slot] : m.taus[slot / m.group]; }
__device__ inline int slot_xrow(const SlotMap& m, int slot) { return (slot / m.x_group) * m.x_batch + slot % m.x_batch; }
__device__ inline int slot_crow(const SlotMap& m, int slot) { return m.cond_mod ? slot % m.cond_mod : slot; }

// One block per slot.  femb(tau) -> Linear -> SiLU -> Linear (+ cond embedding) -> SiLU.
// Each wave owns output rows; lanes stride over the input so weight reads coalesce.
__global__ void __launch_bounds__(256) cond_embed_kernel(const CondArgs a)
{
    extern __shared__ float sm[];          // femb[256] | h1[D] | cvec (vector cond) [cond_dim]
    float* femb = sm;
    float* h1 = sm + kTFreq;
    float* cv = h1 + a.D;
    const int slot = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, nw = blockDim.x >> 6;
    const int tau = slot_tau(a.map, slot);
    // sinusoid in double: tau * f reaches ~1e3 rad, beyond what fp32 range reduction keeps to 1e-7
    if (tid < kTFreq / 2) {
        double f = exp(-9.210340371976184 * (double)tid / (double)(kTFreq / 2));
        double ang = (double)tau * f;
        femb[tid] = (float)cos(ang);
        femb[kTFreq / 2 + tid] = (float)sin(ang);
    }
    const int crow = slot_crow(a.map, slot);
    if (a.cond_kind == DRF_COND_VECTOR)
        for (int i = tid; i < a.cond_dim; i += blockDim.x) cv[i] = ((const float*)a.cond)[(size_t)crow * a.cond_dim + i];
    __syncthreads();
    for (int j = wave; j < a.D; j += nw) {
        const float* wr = a.t_w1 + (size_t)j * kTFreq;
        float acc = 0.f;
        for (int k = lane; k < kTFreq; k += kWave) acc = fmaf(femb[k], wr[k], acc);
        acc = wave_sum(acc);
        if (lane == 0) h1[j] = silu(acc + a.t_b1[j]);
    }
    __syncthreads();
    int cls = 0;
    if (a.cond_kind == DRF_COND_CLASS) {
        cls = ((const int32_t*)a.cond)[crow];
        if (cls < 0 || cls > a.cond_dim) cls = a.cond_dim;
    }
    for (int j = wave; j < a.D; j += nw) {
        const float* wr = a.t_w2 + (size_t)j * a.D;
        float acc = 0.f;
        for (int k = lane; k < a.D; k += kWave) acc = fmaf(h1[k], wr[k], acc);
        if (a.cond_kind == DRF_COND_VECTOR) {
            const float* cr = a.c_w + (size_t)j * a.cond_dim;
            for (int k = lane; k < a.cond_dim; k += kWave) acc = fmaf(cv[k], cr[k], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            float c = acc + a.t_b2[j];
            if (a.cond_kind == DRF_COND_VECTOR) c += a.c_b[j];
            else if (a.cond_kind == DRF_COND_CLASS) c += a.table[(size_t)cls * a.D + j];
            float s = silu(c);
            a.act_f32[(size_t)slot * a.D + j] = s;
            if (a.act_bf16) a.act_bf16[(size_t)slot * a.D + j] = (bf16_t)s;
        }
    }
}

// resid[m][j] = sum_k token[m][k] w[j][k] + b[j] + pos[token][j].  One block per kTok tokens.
constexpr int kTok = 8;
__global__ void __launch_bounds__(256) patch_embed_kernel(const float* __restrict__ x, const SlotMap map,
                                                          const float* __restrict__ w, const float* __restrict__ b,
                                                          const float* __restrict__ pos, const DitDims dm, int M,
                                                          float* __restrict__ resid)
{
    extern __shared__ float tok[];         // [kTok][P]
    const int m0 = blockIdx.x * kTok, tid = threadIdx.x;
    const size_t E = (size_t)dm.C * dm.H * dm.W;
    for (int i = tid; i < kTok * dm.P; i += blockDim.x) {
        const int tl = i / dm.P, k = i % dm.P, m = m0 + tl;
        float v = 0.f;
        if (m < M) {
            const int slot = m / dm.T, t = m % dm.T, py = t / dm.gw, px = t % dm.gw;
            const int pp = dm.patch * dm.patch, ch = k / pp, dy = (k % pp) / dm.patch, dx = k % dm.patch;
            v = x[(size_t)slot_xrow(map, slot) * E + ((size_t)ch * dm.H + py * dm.patch + dy) * dm.W + px * dm.patch + dx];
        }
        tok[i] = v;
    }
    __syncthreads();
    for (int j = tid; j < dm.D; j += blockDim.x) {
        const float* wr = w + (size_t)j * dm.P;
        const float bj = b[j];
        float acc[kTok];
#pragma unroll
        for (int tl = 0; tl < kTok; ++tl) acc[tl] = 0.f;
        for (int k = 0; k < dm.P; ++k) {
            const float wv = wr[k];
#pragma unroll
            for (int tl = 0; tl < kTok; ++tl) acc[tl] = fmaf(tok[tl * dm.P + k], wv, acc[tl]);
        }
#pragma unroll
        for (int tl = 0; tl < kTok; ++tl) {
            const int m = m0 + tl;
            if (m < M) resid[(size_t)m * dm.D + j] = acc[tl] + bj + pos[(size_t)(m % dm.T) * dm.D + j];
        }
    }
}

// One wave per row; the row stays in registers between the statistics and the output.
constexpr int kLnMaxPer = 32;              // hidden <= 64 * 32
template <typename OutT>
__global__ void __launch_bounds__(256) ln_modulate_kernel(const float* __restrict__ resid, const float* __restrict__ shift,
                                                          const float* __restrict__ scale, int mod_ld, int rows_per_slot,
                                                          int M, int D, OutT* __restrict__ out)
{
    const int lane = threadIdx.x & 63, row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const float* xr = resid + (size_t)row * D;
    float v[kLnMaxPer];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        v[i] = j < D ? xr[j] : 0.f;
        sum += v[i];
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        const float dlt = j < D ? v[i] - mean : 0.f;
        sq = fmaf(dlt, dlt, sq);
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)D + 1e-6f);
    const size_t mrow = (size_t)(row / rows_per_slot) * mod_ld;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        if (j < D) {
            float y = (v[i] - mean) * rstd;
            if (shift) y = fmaf(y, 1.f + scale[mrow + j], shift[mrow + j]);
            out[(size_t)row * D + j] = (OutT)y;
        }
    }
}

// Final layer: LN + modulate, Linear(D -> P), scatter to [C][H][W].  One wave per token.
__global__ void __launch_bounds__(256) final_kernel(const float* __restrict__ resid, const float* __restrict__ shift,
                                                    const float* __restrict__ scale, int mod_ld,
                                                    const float* __restrict__ w, const float* __restrict__ b,
                                                    const DitDims dm, int M, float* __restrict__ eps_out)
{
    const int lane = threadIdx.x & 63, row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const int D = dm.D;
    const float* xr = resid + (size_t)row * D;
    float v[kLnMaxPer];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        v[i] = j < D ? xr[j] : 0.f;
        sum += v[i];
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        const float dlt = j < D ? v[i] - mean : 0.f;
        sq = fmaf(dlt, dlt, sq);
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)D + 1e-6f);
    const int slot = row / dm.T, t = row % dm.T, py = t / dm.gw, px = t % dm.gw;
    const size_t mrow = (size_t)slot * mod_ld;
#pragma unroll
    for (int i = 0; i < kLnMaxPer; ++i) {
        const int j = i * kWave + lane;
        v[i] = j < D ? fmaf((v[i] - mean) * rstd, 1.f + scale[mrow + j], shift[mrow + j]) : 0.f;
    }
    const size_t E = (size_t)dm.C * dm.H * dm.W;
    const int pp = dm.patch * dm.patch;
    for (int k = 0; k < dm.P; ++k) {
        const float* wr = w + (size_t)k * D;
        float acc = 0.f;
#pragma unroll
        for (int i = 0; i < kLnMaxPer; ++i) {
            const int j = i * kWave + lane;
            if (j < D) acc = fmaf(v[i], wr[j], acc);
        }
        acc = wave_sum(acc);
        if (lane == 0) {
            const int ch = k / pp, dy = (k % pp) / dm.patch, dx = k % dm.patch;
            eps_out[(size_t)slot * E + ((size_t)ch * dm.H + py * dm.patch + dy) * dm.W + px * dm.patch + dx] = acc + b[k];
        }
    }
}

__global__ void f32_to_bf16_kernel(const float* __restrict__ in, bf16_t* __restrict__ out, size_t n)
{
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) out[i] = (bf16_t)in[i];
}

}  // namespace

drf_status launch_cond_embed(const CondArgs& a, hipStream_t st)
{
    if (a.slots == 0) return DRF_OK;
    const size_t smem = sizeof(float) * (size_t)(kTFreq + a.D + (a.cond_kind == DRF_COND_VECTOR ? a.cond_dim : 0));
    hipLaunchKernelGGL(cond_embed_kernel, dim3(a.slots), dim3(256), smem, st, a);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

drf_status launch_patch_embed(const float* x, const SlotMap& map, const float* w, const float* b, const float* pos,
                              const DitDims& dm, int slots, float* resid, hipStream_t st)
{
    const int M = slots * dm.T;
    if (M == 0) return DRF_OK;
    hipLaunchKernelGGL(patch_embed_kernel, dim3((M + kTok - 1) / kTok), dim3(256), sizeof(float) * kTok * dm.P, st, x, map,
                       w, b, pos, dm, M, resid);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

drf_status launch_ln_modulate(const float* resid, const float* shift, const float* scale, int mod_ld, int rows_per_slot,
                              int M, int D, void* out, int out_f32, hipStream_t st)
{
    if (M == 0) return DRF_OK;
    if (D > kWave * kLnMaxPer) DRF_FAIL(DRF_ESHAPE, "hidden %d exceeds LayerNorm kernel limit %d", D, kWave * kLnMaxPer);
    const dim3 grid((M + 3) / 4), block(256);
    if (out_f32)
        hipLaunchKernelGGL(ln_modulate_kernel<float>, grid, block, 0, st, resid, shift, scale, mod_ld, rows_per_slot, M, D,
                           (float*)out);
    else
        hipLaunchKernelGGL(ln_modulate_kernel<bf16_t>, grid, block, 0, st, resid, shift, scale, mod_ld, rows_per_slot, M, D,
                           (bf16_t*)out);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

drf_status launch_final(const float* resid, const float* shift, const float* scale, int mod_ld, const float* w,
                        const float* b, const DitDims& dm, int slots, float* eps_out, hipStream_t st)
{
    const int M = slots * dm.T;
    if (M == 0) return DRF_OK;
    hipLaunchKernelGGL(final_kernel, dim3((M + 3) / 4), dim3(256), 0, st, resid, shift, scale, mod_ld, w, b, dm, M, eps_out);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

drf_status launch_f32_to_bf16(const float* in, bf16_t* out, size_t n, hipStream_t st)
{
    if (n == 0) return DRF_OK;
    size_t blocks = (n + 255) / 256;
    if (blocks > 65536) blocks = 65536;
    hipLaunchKernelGGL(f32_to_bf16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, in, out, n);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf
