// GEMM C[M][N] = A[M][K] . W[N][K]^T with fused epilogues (bias, GELU-tanh, gated
// residual).  bf16 path: MFMA 32x32x16 tiles fed from LDS, fp32 accumulate.
// fp32 path: plain LDS-tiled FMA kernel for the fp32 configuration.
#include "common.h"

namespace drf {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

__device__ inline float gelu_tanh(float x)
{
    const float u = 0.7978845608028654f * (x + 0.044715f * x * x * x);
    // tanh(u) = 1 - 2 / (exp(2u) + 1)
    const float t = 1.f - 2.f / (__expf(2.f * u) + 1.f);
    return 0.5f * x * (1.f + t);
}

// Applies the epilogue to 4 consecutive columns n..n+3 of row m (n % 4 == 0, n + 3 < N).
__device__ inline void epilogue4(const Epilogue& e, int m, int n, float v0, float v1, float v2, float v3)
{
    const float4 b = *reinterpret_cast<const float4*>(e.bias + n);
    v0 += b.x; v1 += b.y; v2 += b.z; v3 += b.w;
    if (e.mode == EPI_RESID) {
        float4* xp = reinterpret_cast<float4*>((float*)e.out + (size_t)m * e.ldo + n);
        float4 x = *xp;
        if (e.gate) {
            const float4 g = *reinterpret_cast<const float4*>(e.gate + (size_t)(m / e.rows_per_slot) * e.gate_ld + n);
            x.x = fmaf(g.x, v0, x.x); x.y = fmaf(g.y, v1, x.y); x.z = fmaf(g.z, v2, x.z); x.w = fmaf(g.w, v3, x.w);
        } else {
            x.x += v0; x.y += v1; x.z += v2; x.w += v3;
        }
        *xp = x;
        return;
    }
    if (e.mode == EPI_STORE_GELU) { v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3); }
    if (e.out_f32) {
        *reinterpret_cast<float4*>((float*)e.out + (size_t)m * e.ldo + n) = make_float4(v0, v1, v2, v3);
    } else {
        bf16x4 o = { (bf16_t)v0, (bf16_t)v1, (bf16_t)v2, (bf16_t)v3 };
        *reinterpret_cast<bf16x4*>((bf16_t*)e.out + (size_t)m * e.ldo + n) = o;
    }
}

// ------------------------------------------------------------------ bf16 MFMA
// Block tile BM x BN x 64, WM x WN waves, each wave (BM/WM) x (BN/WN) as 32x32 MFMA tiles.
// The weight tile is the MFMA "A" operand and the activation tile the "B" operand, so a
// lane ends up with 4 consecutive output columns per register quad (vector stores).
template <int BM, int BN, int WM, int WN>
__global__ void __launch_bounds__(WM * WN * 64)
gemm_bf16_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, int M, int N, int K, const Epilogue e)
{
    constexpr int BK = 64, LDK = BK + 8, NT = WM * WN * 64;
    constexpr int TM = BM / WM, TN = BN / WN, MI = TM / 32, NI = TN / 32;
    constexpr int ACH = BM * (BK / 8) / NT, WCH = BN * (BK / 8) / NT;   // 16-byte chunks per thread
    static_assert(BM * (BK / 8) % NT == 0 && BN * (BK / 8) % NT == 0, "tile/threads mismatch");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* sA = reinterpret_cast<bf16_t*>(smem_raw);                 // [2][BM][LDK]
    bf16_t* sW = sA + 2 * BM * LDK;                                     // [2][BN][LDK]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave % WM, wn = wave / WM;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    const int l32 = lane & 31, half = lane >> 5;

    bf16x8 ra[ACH], rw[WCH];
    auto load_global = [&](int kt) {
#pragma unroll
        for (int c = 0; c < ACH; ++c) {
            const int id = tid + c * NT, row = id >> 3, kc = id & 7;
            int gm = m0 + row; gm = gm < M ? gm : M - 1;               // clamp: rows past M are never stored
            ra[c] = *reinterpret_cast<const bf16x8*>(A + (size_t)gm * K + kt * BK + kc * 8);
        }
#pragma unroll
        for (int c = 0; c < WCH; ++c) {
            const int id = tid + c * NT, row = id >> 3, kc = id & 7;
            int gn = n0 + row; gn = gn < N ? gn : N - 1;
            rw[c] = *reinterpret_cast<const bf16x8*>(W + (size_t)gn * K + kt * BK + kc * 8);
        }
    };
    auto store_lds = [&](int buf) {
#pragma unroll
        for (int c = 0; c < ACH; ++c) {
            const int id = tid + c * NT, row = id >> 3, kc = id & 7;
            *reinterpret_cast<bf16x8*>(sA + (buf * BM + row) * LDK + kc * 8) = ra[c];
        }
#pragma unroll
        for (int c = 0; c < WCH; ++c) {
            const int id = tid + c * NT, row = id >> 3, kc = id & 7;
            *reinterpret_cast<bf16x8*>(sW + (buf * BN + row) * LDK + kc * 8) = rw[c];
        }
    };

    f32x16 acc[NI][MI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < MI; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int nk = K / BK;
    load_global(0);
    store_lds(0);
    __syncthreads();
    for (int kt = 0; kt < nk; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < nk) load_global(kt + 1);
        const bf16_t* pa = sA + (buf * BM + wm * TM + l32) * LDK + half * 8;
        const bf16_t* pw = sW + (buf * BN + wn * TN + l32) * LDK + half * 8;
#pragma unroll
        for (int ks = 0; ks < BK / 16; ++ks) {
            bf16x8 fa[MI], fw[NI];
#pragma unroll
            for (int j = 0; j < MI; ++j) fa[j] = *reinterpret_cast<const bf16x8*>(pa + j * 32 * LDK + ks * 16);
#pragma unroll
            for (int i = 0; i < NI; ++i) fw[i] = *reinterpret_cast<const bf16x8*>(pw + i * 32 * LDK + ks * 16);
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < MI; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[i], fa[j], acc[i][j], 0, 0, 0);
        }
        if (kt + 1 < nk) store_lds(buf ^ 1);
        __syncthreads();
    }

    // acc[i][j][r]: n = n0 + wn*TN + i*32 + 8*(r/4) + 4*half + r%4,  m = m0 + wm*TM + j*32 + l32
#pragma unroll
    for (int j = 0; j < MI; ++j) {
        const int m = m0 + wm * TM + j * 32 + l32;
        if (m >= M) continue;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int n = n0 + wn * TN + i * 32 + 8 * q + 4 * half;
                if (n < N) epilogue4(e, m, n, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
            }
    }
}

// ------------------------------------------------------------------------ fp32
// 64 x 64 x 16 tile, 256 threads, 4 x 4 outputs per thread (columns n consecutive).
__global__ void __launch_bounds__(256)
gemm_f32_kernel(const float* __restrict__ A, const float* __restrict__ W, int M, int N, int K, const Epilogue e)
{
    constexpr int BM = 64, BN = 64, BK = 16;
    __shared__ float sA[BK][BM + 1], sW[BK][BN + 1];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += BK) {
        for (int i = tid; i < BM * BK; i += 256) {
            const int r = i / BK, k = i % BK;
            sA[k][r] = (m0 + r < M && k0 + k < K) ? A[(size_t)(m0 + r) * K + k0 + k] : 0.f;
            sW[k][r] = (n0 + r < N && k0 + k < K) ? W[(size_t)(n0 + r) * K + k0 + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int k = 0; k < BK; ++k) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) { a[i] = sA[k][ty * 4 + i]; w[i] = sW[k][tx * 4 + i]; }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i, n = n0 + tx * 4;
        if (m < M && n < N) epilogue4(e, m, n, acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    }
}

template <int BM, int BN, int WM, int WN>
drf_status launch_bf16_tile(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st)
{
    constexpr size_t smem = (size_t)2 * (BM + BN) * (64 + 8) * sizeof(bf16_t);
    static bool attr_set = false;
    auto kern = gemm_bf16_kernel<BM, BN, WM, WN>;
    if (!attr_set) {
        DRF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const dim3 grid((N + BN - 1) / BN, (M + BM - 1) / BM);
    hipLaunchKernelGGL(kern, grid, dim3(WM * WN * 64), smem, st, A, W, M, N, K, e);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace

drf_status launch_gemm_bf16(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st)
{
    if (M == 0 || N == 0) return DRF_OK;
    if (K % 64 != 0 || N % 4 != 0 || e.ldo % 4 != 0) DRF_FAIL(DRF_ESHAPE, "bf16 GEMM needs K %% 64 == 0 and N %% 4 == 0 (M=%d N=%d K=%d)", M, N, K);
    return launch_bf16_tile<128, 128, 2, 2>(A, W, M, N, K, e, st);
}

drf_status launch_gemm_f32(const float* A, const float* W, int M, int N, int K, const Epilogue& e, hipStream_t st)
{
    if (M == 0 || N == 0) return DRF_OK;
    if (N % 4 != 0 || e.ldo % 4 != 0) DRF_FAIL(DRF_ESHAPE, "fp32 GEMM needs N %% 4 == 0 (N=%d)", N);
    const dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(256), 0, st, A, W, M, N, K, e);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf
