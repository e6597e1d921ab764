// Bandwidth-bound pieces of the DiT forward: conditioning front-end, patch embedding,
// LayerNorm + adaLN modulation, final projection + unpatchify.
#include "common.h"

namespace drf {

namespace {

constexpr int kWave = 64;
constexpr int kTFreq = 256;

// Sum over the 64 lanes with DPP adds (no LDS traffic): inclusive scan inside each row of 16
// lanes (row_shr 1, 2, 4, 8 with zero fill), then the row totals are passed on with
// row_bcast:15 (into rows 1 and 3) and row_bcast:31 (into rows 2 and 3); lane 63 ends with
// the wave total, which readlane hands to every lane.
template <int CTRL, int ROW_MASK>
__device__ inline float dpp_add(float v)
{
    return v + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, ROW_MASK, 0xf, true));
}
__device__ inline float wave_sum(float v)
{
    v = dpp_add<0x111, 0xf>(v);
    v = dpp_add<0x112, 0xf>(v);
    v = dpp_add<0x114, 0xf>(v);
    v = dpp_add<0x118, 0xf>(v);
    v = dpp_add<0x142, 0xa>(v);
    v = dpp_add<0x143, 0xc>(v);
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
}

__device__ inline float silu(float v) { return v / (1.f + __expf(-v)); }

__device__ inline int slot_tau(const SlotMap& m, int slot) { return m.t_dev ? m.t_dev[slot] : m.taus[slot / m.group]; }
__device__ inline int slot_xrow(const SlotMap& m, int slot) { return (slot / m.x_group) * m.x_batch + slot % m.x_batch; }
__device__ inline int slot_crow(const SlotMap& m, int slot) { return m.cond_mod ? slot % m.cond_mod : slot; }

// Conditioning front-end, four small launches that each fill the chip:
//   femb(tau) per slot -> skinny Linear + SiLU -> skinny Linear -> add cond embedding, SiLU.

// femb[slot][256] = [cos(tau f_i) | sin(tau f_i)], f_i = 10000^(-i/128).  Double precision:
// tau * f reaches ~1e3 rad, beyond what fp32 range reduction keeps to 1e-7.
__global__ void __launch_bounds__(kTFreq / 2) time_features_kernel(const SlotMap map, int slots, float* __restrict__ femb)
{
    const int slot = blockIdx.x, i = threadIdx.x;
    if (slot >= slots) return;
    const double f = exp(-9.210340371976184 * (double)i / (double)(kTFreq / 2));
    const double ang = (double)slot_tau(map, slot) * f;
    femb[(size_t)slot * kTFreq + i] = (float)cos(ang);
    femb[(size_t)slot * kTFreq + kTFreq / 2 + i] = (float)sin(ang);
}

// y[r][j] = act(sum_k x[row(r)][k] w[j][k] + b[j]) for a handful of rows r (one per slot).
// A block owns kSkinnyCols output columns of one 64-row chunk (grid.y walks the chunks) and
// walks K in pieces staged through LDS: thread (row, column pair) accumulates two outputs.
constexpr int kSkinnyCols = 8, kSkinnyChunk = 128;
template <bool SILU>
__global__ void __launch_bounds__(256) skinny_linear_kernel(const float* __restrict__ x, int ldx, int row_mod,
                                                            const float* __restrict__ w, const float* __restrict__ b,
                                                            int rows, int K, int N, float* __restrict__ y)
{
    __shared__ float xs[64][kSkinnyChunk + 1];
    __shared__ float ws[kSkinnyCols][kSkinnyChunk + 1];
    const int tid = threadIdx.x, rl = tid & 63, cg = tid >> 6;
    const int j0 = blockIdx.x * kSkinnyCols;
    for (int r0 = blockIdx.y * 64; r0 < rows; r0 += gridDim.y * 64) {
        float acc0 = 0.f, acc1 = 0.f;
        for (int k0 = 0; k0 < K; k0 += kSkinnyChunk) {
            __syncthreads();
            for (int i = tid; i < 64 * kSkinnyChunk; i += 256) {
                const int r = i / kSkinnyChunk, k = i % kSkinnyChunk, rr = r0 + r;
                float v = 0.f;
                if (rr < rows && k0 + k < K) v = x[(size_t)(row_mod ? rr % row_mod : rr) * ldx + k0 + k];
                xs[r][k] = v;
            }
            for (int i = tid; i < kSkinnyCols * kSkinnyChunk; i += 256) {
                const int c = i / kSkinnyChunk, k = i % kSkinnyChunk;
                ws[c][k] = (j0 + c < N && k0 + k < K) ? w[(size_t)(j0 + c) * K + k0 + k] : 0.f;
            }
            __syncthreads();
#pragma unroll 8
            for (int k = 0; k < kSkinnyChunk; ++k) {
                const float xv = xs[rl][k];
                acc0 = fmaf(xv, ws[2 * cg][k], acc0);
                acc1 = fmaf(xv, ws[2 * cg + 1][k], acc1);
            }
        }
        const int r = r0 + rl;
        if (r < rows) {
            const int ja = j0 + 2 * cg, jb = ja + 1;
            if (ja < N) { const float v = acc0 + b[ja]; y[(size_t)r * N + ja] = SILU ? silu(v) : v; }
            if (jb < N) { const float v = acc1 + b[jb]; y[(size_t)r * N + jb] = SILU ? silu(v) : v; }
        }
    }
}

// c = t_emb + cond embedding; writes SiLU(c) as float and, if asked, bf16.
__global__ void __launch_bounds__(256) cond_finish_kernel(const float* __restrict__ temb, const float* __restrict__ vemb,
                                                          const float* __restrict__ table, const int32_t* __restrict__ cls,
                                                          const SlotMap map, int n_classes, int slots, int D,
                                                          float* __restrict__ act_f32, bf16_t* __restrict__ act_bf16)
{
    const int slot = blockIdx.y, j = blockIdx.x * blockDim.x + threadIdx.x;
    if (slot >= slots || j >= D) return;
    float c = temb[(size_t)slot * D + j];
    if (vemb) c += vemb[(size_t)slot * D + j];
    if (table) {
        int k = cls[slot_crow(map, slot)];
        if (k < 0 || k > n_classes) k = n_classes;
        c += table[(size_t)k * D + j];
    }
    const float s = silu(c);
    act_f32[(size_t)slot * D + j] = s;
    if (act_bf16) act_bf16[(size_t)slot * D + j] = (bf16_t)s;
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
// Lanes hold pairs of adjacent columns (8-byte loads, 4- or 8-byte stores); PER pairs per lane.
template <typename OutT> struct Pair;
template <> struct Pair<float> { typedef float2 type; };
template <> struct Pair<bf16_t> { typedef bf16_t type __attribute__((ext_vector_type(2))); };

template <int PER, typename OutT>
__global__ void __launch_bounds__(256) ln_modulate_kernel(float* __restrict__ resid, const bf16_t* __restrict__ add,
                                                          const bf16_t* __restrict__ add2, int write_back,
                                                          const float* __restrict__ shift,
                                                          const float* __restrict__ scale, int mod_ld, int rows_per_slot,
                                                          int M, int D, OutT* __restrict__ out)
{
    typedef typename Pair<OutT>::type out2;
    typedef bf16_t bf16x2 __attribute__((ext_vector_type(2)));
    const int lane = threadIdx.x & 63, row = blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6);
    if (row >= M) return;
    const int D2 = D >> 1;
    float2* xr = reinterpret_cast<float2*>(resid + (size_t)row * D);
    float2 v[PER];
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = i * kWave + lane;
        v[i] = j < D2 ? xr[j] : make_float2(0.f, 0.f);
        if (add && j < D2) {                   // pending branch outputs: x = resid + add (+ add2), stored if asked
            const bf16x2 a2 = reinterpret_cast<const bf16x2*>(add + (size_t)row * D)[j];
            v[i].x += (float)a2.x; v[i].y += (float)a2.y;
            if (add2) {
                const bf16x2 b2 = reinterpret_cast<const bf16x2*>(add2 + (size_t)row * D)[j];
                v[i].x += (float)b2.x; v[i].y += (float)b2.y;
            }
            if (write_back) xr[j] = v[i];
        }
        sum += v[i].x + v[i].y;
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = i * kWave + lane;
        const float dx = j < D2 ? v[i].x - mean : 0.f, dy = j < D2 ? v[i].y - mean : 0.f;
        sq = fmaf(dx, dx, fmaf(dy, dy, sq));
    }
    const float rstd = rsqrtf(wave_sum(sq) / (float)D + 1e-6f);
    const size_t mrow = (size_t)(row / rows_per_slot) * mod_ld;
    const float2* sh = shift ? reinterpret_cast<const float2*>(shift + mrow) : nullptr;
    const float2* sc = shift ? reinterpret_cast<const float2*>(scale + mrow) : nullptr;
    out2* orow = reinterpret_cast<out2*>(out + (size_t)row * D);
#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int j = i * kWave + lane;
        if (j < D2) {
            float y0 = (v[i].x - mean) * rstd, y1 = (v[i].y - mean) * rstd;
            if (sh) {
                const float2 s2 = sc[j], h2 = sh[j];
                y0 = fmaf(y0, 1.f + s2.x, h2.x);
                y1 = fmaf(y1, 1.f + s2.y, h2.y);
            }
            out2 o;
            o.x = (OutT)y0; o.y = (OutT)y1;
            orow[j] = o;
        }
    }
}

// Same operation for hidden sizes that are multiples of 128: half a wave per row, 16-byte loads
// of the residual row (PER4 float4 per lane) and 8-byte (bf16) or 16-byte (fp32) stores.
__device__ inline float half_wave_sum(float v)
{
#pragma unroll
    for (int o = 16; o >= 1; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
template <int PER4, typename OutT, int ADD, bool WB>
__global__ void __launch_bounds__(256) ln_modulate4_kernel(float* __restrict__ resid, const bf16_t* __restrict__ add,
                                                           const bf16_t* __restrict__ add2,
                                                           const float* __restrict__ shift,
                                                           const float* __restrict__ scale, int mod_ld, int rows_per_slot,
                                                           int M, OutT* __restrict__ out)
{
    constexpr int D = PER4 * 128;
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    typedef float f32x4n __attribute__((ext_vector_type(4)));
    const int l32 = threadIdx.x & 31, row = blockIdx.x * (blockDim.x >> 5) + (threadIdx.x >> 5);
    if (row >= M) return;                       // M is even here or the spare half wave idles: no block barrier below
    float4* xr = reinterpret_cast<float4*>(resid + (size_t)row * D);
    float4 v[PER4];
    bf16x4 a4[ADD >= 1 ? PER4 : 1], b4[ADD >= 2 ? PER4 : 1];
#pragma unroll
    for (int i = 0; i < PER4; ++i) {
        // The residual stream and the pending branch outputs are streaming data here: each is next needed a
        // few hundred microseconds and several hundred megabytes of other traffic later, so they are read and
        // written with the non-temporal hint and leave the caches to the activations that the next kernel
        // consumes (the GEMMs of a call run 2 % faster for it, this launch 5 % slower).
        { const f32x4n t4 = __builtin_nontemporal_load(reinterpret_cast<const f32x4n*>(xr) + i * 32 + l32); v[i] = make_float4(t4[0], t4[1], t4[2], t4[3]); }
        if constexpr (ADD >= 1) a4[i] = __builtin_nontemporal_load(&reinterpret_cast<const bf16x4*>(add + (size_t)row * D)[i * 32 + l32]);
        if constexpr (ADD >= 2) b4[i] = __builtin_nontemporal_load(&reinterpret_cast<const bf16x4*>(add2 + (size_t)row * D)[i * 32 + l32]);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < PER4; ++i) {
        if constexpr (ADD >= 1) {               // pending branch outputs: x = resid + add (+ add2), stored if WB
            v[i].x += (float)a4[i][0]; v[i].y += (float)a4[i][1]; v[i].z += (float)a4[i][2]; v[i].w += (float)a4[i][3];
            if constexpr (ADD >= 2) {
                v[i].x += (float)b4[i][0]; v[i].y += (float)b4[i][1]; v[i].z += (float)b4[i][2]; v[i].w += (float)b4[i][3];
            }
        }
        sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
    }
    // Every load of the kernel is issued before its first store: loads and stores share one in-order counter, so a
    // load behind a store is only seen once the memory system has taken the store.  The modulation rows are asked
    // for here, all at once, and arrive during the two reductions; the stream's write-back waits until the end.
    // (132-170 registers, two or three waves per SIMD: capping the kernel at 168 or 128 registers for more waves
    // was measured 2 % and 50 % slower for these launches.)
    float4 s4[PER4], h4[PER4];
    if (shift) {
        const size_t mrow = (size_t)(row / rows_per_slot) * mod_ld;
        const float4* sh = reinterpret_cast<const float4*>(shift + mrow);
        const float4* sc = reinterpret_cast<const float4*>(scale + mrow);
#pragma unroll
        for (int i = 0; i < PER4; ++i) { s4[i] = sc[i * 32 + l32]; h4[i] = sh[i * 32 + l32]; }
    } else {
#pragma unroll
        for (int i = 0; i < PER4; ++i) { s4[i] = make_float4(0.f, 0.f, 0.f, 0.f); h4[i] = s4[i]; }
    }
    const float mean = half_wave_sum(sum) * (1.f / (float)D);
    float sq = 0.f;
#pragma unroll
    for (int i = 0; i < PER4; ++i) {
        const float dx = v[i].x - mean, dy = v[i].y - mean, dz = v[i].z - mean, dw = v[i].w - mean;
        sq = fmaf(dx, dx, fmaf(dy, dy, fmaf(dz, dz, fmaf(dw, dw, sq))));
    }
    const float rstd = rsqrtf(half_wave_sum(sq) * (1.f / (float)D) + 1e-6f);
#pragma unroll
    for (int i = 0; i < PER4; ++i) {
        const int j = i * 32 + l32;
        float y0 = (v[i].x - mean) * rstd, y1 = (v[i].y - mean) * rstd, y2 = (v[i].z - mean) * rstd, y3 = (v[i].w - mean) * rstd;
        if (shift) {                            // (without modulation y * 1 + 0 would be the same value; kept exact in form)
            y0 = fmaf(y0, 1.f + s4[i].x, h4[i].x); y1 = fmaf(y1, 1.f + s4[i].y, h4[i].y);
            y2 = fmaf(y2, 1.f + s4[i].z, h4[i].z); y3 = fmaf(y3, 1.f + s4[i].w, h4[i].w);
        }
        if constexpr (sizeof(OutT) == 4) {
            reinterpret_cast<float4*>(out + (size_t)row * D)[j] = make_float4(y0, y1, y2, y3);
        } else {
            const bf16x4 o = { (bf16_t)y0, (bf16_t)y1, (bf16_t)y2, (bf16_t)y3 };
            reinterpret_cast<bf16x4*>(out + (size_t)row * D)[j] = o;
        }
        if constexpr (ADD >= 1 && WB) { const f32x4n t4 = { v[i].x, v[i].y, v[i].z, v[i].w }; __builtin_nontemporal_store(t4, reinterpret_cast<f32x4n*>(xr) + i * 32 + l32); }
    }
}

// Final layer: LN + modulate, Linear(D -> P), scatter to [C][H][W].  A block of 4 waves takes
// kFinalRowsPerBlock token rows; wave w keeps the weights of outputs w, w+4, w+8, w+12 (of each
// group of 16) in registers and sweeps the rows, so nothing but the residual rows is re-read.
constexpr int kFinalRowsPerBlock = 16;
template <int PER>
__global__ void __launch_bounds__(256) final_kernel(const float* __restrict__ resid, const float* __restrict__ shift,
                                                    const float* __restrict__ scale, int mod_ld,
                                                    const float* __restrict__ w, const float* __restrict__ b,
                                                    const DitDims dm, int M, float* __restrict__ eps_out)
{
    const int D = dm.D, P = dm.P;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t E = (size_t)dm.C * dm.H * dm.W;
    const int pp = dm.patch * dm.patch;
    const int row0 = blockIdx.x * kFinalRowsPerBlock, row_end = min(M, row0 + kFinalRowsPerBlock);
    for (int kbase = 0; kbase < P; kbase += 16) {
        float wr[4][PER], bias[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int k = kbase + wave + 4 * q;
            bias[q] = k < P ? b[k] : 0.f;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int j = i * kWave + lane;
                wr[q][i] = (k < P && j < D) ? w[(size_t)k * D + j] : 0.f;
            }
        }
        for (int row = row0; row < row_end; ++row) {
            const float* xr = resid + (size_t)row * D;
            float v[PER];
            float sum = 0.f;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int j = i * kWave + lane;
                v[i] = j < D ? xr[j] : 0.f;
                sum += v[i];
            }
            const float mean = wave_sum(sum) / (float)D;
            float sq = 0.f;
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int j = i * kWave + lane;
                const float dlt = j < D ? v[i] - mean : 0.f;
                sq = fmaf(dlt, dlt, sq);
            }
            const float rstd = rsqrtf(wave_sum(sq) / (float)D + 1e-6f);
            const int slot = row / dm.T, t = row % dm.T, py = t / dm.gw, px = t % dm.gw;
            const size_t mrow = (size_t)slot * mod_ld;
            float acc[4] = { 0.f, 0.f, 0.f, 0.f };
#pragma unroll
            for (int i = 0; i < PER; ++i) {
                const int j = i * kWave + lane;
                const float y = j < D ? fmaf((v[i] - mean) * rstd, 1.f + scale[mrow + j], shift[mrow + j]) : 0.f;
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = fmaf(y, wr[q][i], acc[q]);
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float tot = wave_sum(acc[q]);
                const int k = kbase + wave + 4 * q;
                if (lane == 0 && k < P) {
                    const int ch = k / pp, dy = (k % pp) / dm.patch, dx = k % dm.patch;
                    eps_out[(size_t)slot * E + ((size_t)ch * dm.H + py * dm.patch + dy) * dm.W + px * dm.patch + dx] = tot + bias[q];
                }
            }
        }
    }
}

// Final layer for hidden sizes that are multiples of 128 and weights [P][D] that fit LDS: the weights are
// staged once per block, half a wave takes a row (16-byte loads, the row stays in registers through the
// statistics, the modulation and the P dot products), and 16 partial sums per lane are reduced across
// the half wave by a transposing butterfly (8 + 4 + 2 + 1 + 1 exchanges) that leaves output k on the lane
// whose bits 4..1 spell k.
template <int PER4>
__global__ void __launch_bounds__(256) final4_kernel(const float* __restrict__ resid, const float* __restrict__ shift,
                                                     const float* __restrict__ scale, int mod_ld,
                                                     const float* __restrict__ w, const float* __restrict__ b,
                                                     const DitDims dm, int M, int rows_per_block, float* __restrict__ eps_out)
{
    constexpr int D = PER4 * 128;
    extern __shared__ __attribute__((aligned(16))) float fin_w[];            // [P][D]
    const int P = dm.P, tid = threadIdx.x, l32 = tid & 31, hw = tid >> 5;
    for (int i = tid; i < P * (D / 4); i += 256) reinterpret_cast<float4*>(fin_w)[i] = reinterpret_cast<const float4*>(w)[i];
    __syncthreads();
    const size_t E = (size_t)dm.C * dm.H * dm.W;
    const int pp = dm.patch * dm.patch;
    const int row0 = blockIdx.x * rows_per_block, row_end = min(M, row0 + rows_per_block);
    for (int row = row0 + hw; row < row_end; row += 8) {
        const float4* xr = reinterpret_cast<const float4*>(resid + (size_t)row * D);
        float4 v[PER4];
        float sum = 0.f;
#pragma unroll
        for (int i = 0; i < PER4; ++i) {
            v[i] = xr[i * 32 + l32];
            sum += (v[i].x + v[i].y) + (v[i].z + v[i].w);
        }
        const float mean = half_wave_sum(sum) * (1.f / (float)D);
        float sq = 0.f;
#pragma unroll
        for (int i = 0; i < PER4; ++i) {
            const float dx = v[i].x - mean, dy = v[i].y - mean, dz = v[i].z - mean, dw = v[i].w - mean;
            sq = fmaf(dx, dx, fmaf(dy, dy, fmaf(dz, dz, fmaf(dw, dw, sq))));
        }
        const float rstd = rsqrtf(half_wave_sum(sq) * (1.f / (float)D) + 1e-6f);
        const int slot = row / dm.T, t = row % dm.T, py = t / dm.gw, px = t % dm.gw;
        const float4* sh = reinterpret_cast<const float4*>(shift + (size_t)slot * mod_ld);
        const float4* sc = reinterpret_cast<const float4*>(scale + (size_t)slot * mod_ld);
#pragma unroll
        for (int i = 0; i < PER4; ++i) {
            const float4 s4 = sc[i * 32 + l32], h4 = sh[i * 32 + l32];
            v[i].x = fmaf((v[i].x - mean) * rstd, 1.f + s4.x, h4.x); v[i].y = fmaf((v[i].y - mean) * rstd, 1.f + s4.y, h4.y);
            v[i].z = fmaf((v[i].z - mean) * rstd, 1.f + s4.z, h4.z); v[i].w = fmaf((v[i].w - mean) * rstd, 1.f + s4.w, h4.w);
        }
        for (int kbase = 0; kbase < P; kbase += 16) {
            float acc[16];
#pragma unroll
            for (int q = 0; q < 16; ++q) {
                acc[q] = 0.f;
                if (kbase + q < P) {                        // uniform over the block
                    const float4* wk = reinterpret_cast<const float4*>(fin_w + (size_t)(kbase + q) * D);
#pragma unroll
                    for (int i = 0; i < PER4; ++i) {
                        const float4 w4 = wk[i * 32 + l32];
                        acc[q] = fmaf(v[i].x, w4.x, fmaf(v[i].y, w4.y, fmaf(v[i].z, w4.z, fmaf(v[i].w, w4.w, acc[q]))));
                    }
                }
            }
            float a8[8], a4[4], a2[2];
            const bool b16 = l32 & 16, b8 = l32 & 8, b4 = l32 & 4, b2 = l32 & 2;
#pragma unroll
            for (int q = 0; q < 8; ++q) a8[q] = (b16 ? acc[q + 8] : acc[q]) + __shfl_xor(b16 ? acc[q] : acc[q + 8], 16, 64);
#pragma unroll
            for (int q = 0; q < 4; ++q) a4[q] = (b8 ? a8[q + 4] : a8[q]) + __shfl_xor(b8 ? a8[q] : a8[q + 4], 8, 64);
#pragma unroll
            for (int q = 0; q < 2; ++q) a2[q] = (b4 ? a4[q + 2] : a4[q]) + __shfl_xor(b4 ? a4[q] : a4[q + 2], 4, 64);
            const float a1 = (b2 ? a2[1] : a2[0]) + __shfl_xor(b2 ? a2[0] : a2[1], 2, 64);
            const float tot = a1 + __shfl_xor(a1, 1, 64);
            const int k = kbase + (b16 ? 8 : 0) + (b8 ? 4 : 0) + (b4 ? 2 : 0) + (b2 ? 1 : 0);
            if (!(l32 & 1) && k < P) {
                const int ch = k / pp, dy = (k % pp) / dm.patch, dx = k % dm.patch;
                eps_out[(size_t)slot * E + ((size_t)ch * dm.H + py * dm.patch + dy) * dm.W + px * dm.patch + dx] = tot + b[k];
            }
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
    const int D = a.D, S = a.slots;
    // scratch rows: femb [S][256] | h1 [S][D] | temb [S][D] | vemb [S][D]
    float* femb = a.scratch;
    float* h1 = femb + (size_t)S * kTFreq;
    float* temb = h1 + (size_t)S * D;
    float* vemb = temb + (size_t)S * D;
    const dim3 gcol((D + kSkinnyCols - 1) / kSkinnyCols, (S + 63) / 64 < 64 ? (S + 63) / 64 : 64);
    hipLaunchKernelGGL(time_features_kernel, dim3(S), dim3(kTFreq / 2), 0, st, a.map, S, femb);
    hipLaunchKernelGGL(skinny_linear_kernel<true>, gcol, dim3(256), 0, st, femb, kTFreq, 0, a.t_w1, a.t_b1, S, kTFreq, D, h1);
    hipLaunchKernelGGL(skinny_linear_kernel<false>, gcol, dim3(256), 0, st, h1, D, 0, a.t_w2, a.t_b2, S, D, D, temb);
    const bool vec = a.cond_kind == DRF_COND_VECTOR;
    if (vec)
        hipLaunchKernelGGL(skinny_linear_kernel<false>, gcol, dim3(256), 0, st, (const float*)a.cond, a.cond_dim,
                           a.map.cond_mod, a.c_w, a.c_b, S, a.cond_dim, D, vemb);
    const bool cls = a.cond_kind == DRF_COND_CLASS;
    hipLaunchKernelGGL(cond_finish_kernel, dim3((D + 255) / 256, S), dim3(256), 0, st, temb, vec ? vemb : nullptr,
                       cls ? a.table : nullptr, cls ? (const int32_t*)a.cond : nullptr, a.map, a.cond_dim, S, D,
                       a.act_f32, a.act_bf16);
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

template <int PER>
static void launch_ln_inst(float* resid, const bf16_t* add, const bf16_t* add2, int write_back, const float* shift, const float* scale,
                           int mod_ld, int rows_per_slot, int M, int D, void* out, int out_f32, hipStream_t st)
{
    const dim3 grid((M + 3) / 4), block(256);
    if (out_f32)
        hipLaunchKernelGGL((ln_modulate_kernel<PER, float>), grid, block, 0, st, resid, add, add2, write_back, shift, scale, mod_ld,
                           rows_per_slot, M, D, (float*)out);
    else
        hipLaunchKernelGGL((ln_modulate_kernel<PER, bf16_t>), grid, block, 0, st, resid, add, add2, write_back, shift, scale, mod_ld,
                           rows_per_slot, M, D, (bf16_t*)out);
}

template <int PER4>
void launch_ln4_inst(float* resid, const bf16_t* add, const bf16_t* add2, int write_back, const float* shift, const float* scale,
                     int mod_ld, int rows_per_slot, int M, void* out, int out_f32, hipStream_t st)
{
    const dim3 grid((M + 7) / 8), block(256);
#define DRF_LN4(OUT, ADD, WB) \
    hipLaunchKernelGGL((ln_modulate4_kernel<PER4, OUT, ADD, WB>), grid, block, 0, st, resid, add, add2, shift, scale, mod_ld, \
                       rows_per_slot, M, (OUT*)out)
    if (out_f32) DRF_LN4(float, 0, false);
    else if (!add) DRF_LN4(bf16_t, 0, false);
    else if (!add2 && write_back) DRF_LN4(bf16_t, 1, true);
    else if (!add2) DRF_LN4(bf16_t, 1, false);
    else if (write_back) DRF_LN4(bf16_t, 2, true);
    else DRF_LN4(bf16_t, 2, false);
#undef DRF_LN4
}

drf_status launch_ln_modulate(float* resid, const bf16_t* add, const bf16_t* add2, bool write_back, const float* shift,
                              const float* scale, int mod_ld, int rows_per_slot, int M, int D, void* out, int out_f32,
                              hipStream_t st)
{
    if (M == 0) return DRF_OK;
    if (add && out_f32) DRF_FAIL(DRF_ESHAPE, "the pending-branch add is a bf16-path feature");
    if (add2 && !add) DRF_FAIL(DRF_EINVAL, "a second pending branch output needs a first one");
    if (D > 2048 || D % 2 != 0 || mod_ld % 2 != 0) DRF_FAIL(DRF_ESHAPE, "LayerNorm kernel needs even hidden <= 2048 (got %d)", D);
    const int wb = write_back ? 1 : 0;
    const bool al16 = mod_ld % 4 == 0 && ((reinterpret_cast<uintptr_t>(resid) | reinterpret_cast<uintptr_t>(out) |
                                           reinterpret_cast<uintptr_t>(shift) | reinterpret_cast<uintptr_t>(scale) |
                                           reinterpret_cast<uintptr_t>(add) | reinterpret_cast<uintptr_t>(add2)) & 15u) == 0;
    if (al16 && (D == 1152 || D == 384 || D == 768 || D == 1024 || D == 128)) {
        switch (D / 128) {
        case 1: launch_ln4_inst<1>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, out, out_f32, st); break;
        case 3: launch_ln4_inst<3>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, out, out_f32, st); break;
        case 6: launch_ln4_inst<6>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, out, out_f32, st); break;
        case 8: launch_ln4_inst<8>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, out, out_f32, st); break;
        default: launch_ln4_inst<9>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, out, out_f32, st); break;
        }
        DRF_HIP(hipGetLastError());
        return DRF_OK;
    }
    const int per = (D / 2 + kWave - 1) / kWave;      // column pairs per lane
    if (per <= 1) launch_ln_inst<1>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, D, out, out_f32, st);
    else if (per <= 3) launch_ln_inst<3>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, D, out, out_f32, st);
    else if (per <= 5) launch_ln_inst<5>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, D, out, out_f32, st);
    else if (per <= 9) launch_ln_inst<9>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, D, out, out_f32, st);
    else launch_ln_inst<16>(resid, add, add2, wb, shift, scale, mod_ld, rows_per_slot, M, D, out, out_f32, st);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

drf_status launch_final(const float* resid, const float* shift, const float* scale, int mod_ld, const float* w,
                        const float* b, const DitDims& dm, int slots, float* eps_out, hipStream_t st)
{
    const int M = slots * dm.T;
    if (M == 0) return DRF_OK;
    if (dm.D > 2048) DRF_FAIL(DRF_ESHAPE, "final layer needs hidden <= 2048");
    const size_t wbytes = (size_t)dm.P * dm.D * sizeof(float);
    const bool al16 = mod_ld % 4 == 0 && ((reinterpret_cast<uintptr_t>(resid) | reinterpret_cast<uintptr_t>(shift) |
                                           reinterpret_cast<uintptr_t>(scale) | reinterpret_cast<uintptr_t>(w)) & 15u) == 0;
    if (al16 && wbytes <= 96 * 1024 && (dm.D == 1152 || dm.D == 384 || dm.D == 768 || dm.D == 1024 || dm.D == 128)) {
        const int rpb = M >= 8192 ? 32 : 16;
        const dim3 grid4((M + rpb - 1) / rpb), block4(256);
        auto go = [&](auto kern) -> drf_status {
            static bool attr_set = false;                   // one flag per kernel instantiation
            if (!attr_set) {
                DRF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024));
                attr_set = true;
            }
            hipLaunchKernelGGL(kern, grid4, block4, wbytes, st, resid, shift, scale, mod_ld, w, b, dm, M, rpb, eps_out);
            DRF_HIP(hipGetLastError());
            return DRF_OK;
        };
        switch (dm.D / 128) {
        case 1: return go(final4_kernel<1>);
        case 3: return go(final4_kernel<3>);
        case 6: return go(final4_kernel<6>);
        case 8: return go(final4_kernel<8>);
        default: return go(final4_kernel<9>);
        }
    }
    const dim3 grid((M + kFinalRowsPerBlock - 1) / kFinalRowsPerBlock), block(256);
    const int per = (dm.D + kWave - 1) / kWave;
    if (per <= 6) hipLaunchKernelGGL(final_kernel<6>, grid, block, 0, st, resid, shift, scale, mod_ld, w, b, dm, M, eps_out);
    else if (per <= 18) hipLaunchKernelGGL(final_kernel<18>, grid, block, 0, st, resid, shift, scale, mod_ld, w, b, dm, M, eps_out);
    else hipLaunchKernelGGL(final_kernel<32>, grid, block, 0, st, resid, shift, scale, mod_ld, w, b, dm, M, eps_out);
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
