// GEMM C[M][N] = A[M][K] . W[N][K]^T with fused epilogues (bias, GELU-tanh, gated
// residual).  bf16 path: the wide-tile kernel (16x16x32 MFMAs, operands by LDS-DMA) for the
// DiT's big GEMMs and a small 32x32x16-MFMA kernel for short or ragged problems, fp32
// accumulate.  fp32 path: plain LDS-tiled FMA kernel for the fp32 configuration.
#include <type_traits>

#include "common.h"

namespace drf {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// GELU (tanh form): 0.5 x (1 + tanh(u)) = x * sigmoid(2u), u = sqrt(2/pi) (x + 0.044715 x^3).
// One exp2 and one reciprocal (both hardware transcendental ops, ~1 ulp).
__device__ inline float gelu_tanh(float x)
{
    const float t = x * x;
    const float m2u_log2e = x * fmaf(t, -0.1029432f, -2.3022082f);   // -2 u log2(e)
    return x * __builtin_amdgcn_rcpf(1.f + __builtin_amdgcn_exp2f(m2u_log2e));
}

// floor(n / d) for 0 <= n < 2^31 with a host-made magic number (d >= 1).
__device__ inline int fast_div(int n, uint32_t magic, int shift)
{
    return magic ? (int)(__umulhi((uint32_t)n, magic) >> shift) : (n >> shift);
}

// Element offset of (row m, column n) in the head-major q | k | v planes (n is a multiple of 4 or 8
// and the head width a multiple of 8, so a vector never straddles a head).
__device__ inline size_t heads_offset(const Epilogue& e, int m, int n)
{
    const int which = fast_div(n, e.hid_magic, e.hid_shift), c = n - which * e.hid;
    const int head = fast_div(c, e.hd_magic, e.hd_shift), dd = c - head * e.hd;
    const int slot = fast_div(m, e.rps_magic, e.rps_shift), t = m - slot * e.rows_per_slot;
    return (size_t)which * e.plane + ((size_t)(slot * e.heads + head) * e.rows_per_slot + t) * e.hd + dd;
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
            const float4 g = *reinterpret_cast<const float4*>(e.gate + (size_t)fast_div(m, e.rps_magic, e.rps_shift) * e.gate_ld + n);
            x.x = fmaf(g.x, v0, x.x); x.y = fmaf(g.y, v1, x.y); x.z = fmaf(g.z, v2, x.z); x.w = fmaf(g.w, v3, x.w);
        } else {
            x.x += v0; x.y += v1; x.z += v2; x.w += v3;
        }
        *xp = x;
        return;
    }
    if (e.mode == EPI_STORE_GELU) { v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3); }
    if (e.mode == EPI_STORE_GATED) {
        const float4 g = *reinterpret_cast<const float4*>(e.gate + (size_t)fast_div(m, e.rps_magic, e.rps_shift) * e.gate_ld + n);
        v0 *= g.x; v1 *= g.y; v2 *= g.z; v3 *= g.w;
    }
    if (e.out_f32) {
        *reinterpret_cast<float4*>((float*)e.out + (size_t)m * e.ldo + n) = make_float4(v0, v1, v2, v3);
    } else {
        bf16x4 o = { (bf16_t)v0, (bf16_t)v1, (bf16_t)v2, (bf16_t)v3 };
        const size_t off = e.mode == EPI_STORE_HEADS ? heads_offset(e, m, n) : (size_t)m * e.ldo + n;
        *reinterpret_cast<bf16x4*>((bf16_t*)e.out + off) = o;
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

#define DRF_GLOBAL_AS __attribute__((address_space(1)))
#define DRF_LDS_AS __attribute__((address_space(3)))
template <int N> __device__ inline void wait_vmcnt() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }
template <int N> __device__ inline void wait_lgkmcnt() { asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory"); }
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
// 16 bytes per lane from LDS byte address addr + OFF, asynchronously: dst is valid only after an
// s_waitcnt lgkmcnt that covers it.
template <int OFF> __device__ inline void lds_read16(u32x4& dst, uint32_t addr)
{
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF));
}
// Waits until at most N LDS reads are outstanding.  The fragments that the following MFMAs consume
// pass through the statement as in/out operands, so no use of them can be scheduled above the wait.
template <int N> __device__ inline void wait_frag(u32x4& w) { asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(w) : "n"(N)); }
template <int N, int MI> __device__ inline void wait_frags(u32x4& w, u32x4 (&a)[MI])
{
    static_assert(MI == 2 || MI == 4, "activation fragments per k-step");
    if constexpr (MI == 2) asm volatile("s_waitcnt lgkmcnt(%3)" : "+v"(w), "+v"(a[0]), "+v"(a[1]) : "n"(N));
    else asm volatile("s_waitcnt lgkmcnt(%5)" : "+v"(w), "+v"(a[0]), "+v"(a[1]), "+v"(a[2]), "+v"(a[3]) : "n"(N));
}
template <int I, int N, typename F> __device__ __forceinline__ void static_for(F&& f)
{
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// ------------------------------------------------ bf16 MFMA 16x16x32, wide tiles
// The main kernel for the DiT's big GEMMs.  BM x BN x 64 block tile (256 x 288 for hidden
// 1152: 1152, 3456 and 4608 are all multiples of 288, so at 64 row tiles every GEMM of the
// block is a whole number of 256-tile rounds), 8 waves as WM x WN, wave tile (BM/WM) x
// (BN/WN) built from 16x16x32 MFMAs so that widths only need to be multiples of 16.
//  - operands go HBM -> LDS directly (global_load_lds_dwordx4: every lane supplies its own
//    global address and the wave's 64 x 16 bytes land contiguously in LDS), NS stages (two
//    for the wide tiles: all that 160 KB of LDS hold), so the copy of the next k-tiles overlaps
//    the MFMAs of k-tile t.  A tile row is 128 bytes = 8
//    chunks; chunk c of row r sits at position c ^ ((r / 2) % 8), which keeps both the DMA
//    writes and the ds_read_b128 operand fetches free of bank conflicts;
//  - workgroup ids are remapped so that each XCD (ids are dealt round-robin over the 8 XCDs)
//    works on a compact group of tiles and shares A/W slices through its own L2;
//  - the weight tile is the MFMA A operand: a lane ends with 4 consecutive columns n of one
//    row m per accumulator;
//  - epilogue: each wave transposes its accumulators through its own slice of the (now
//    idle) LDS stages and then touches global memory in whole rows: 16 bytes per lane,
//    consecutive lanes on consecutive addresses.
typedef float f32x4 __attribute__((ext_vector_type(4)));
// copy instructions issued per MFMA group by the in-loop copy of the two-stage kernels (1: measured best; 2, 3 and
// the whole copy at once are 0.8 % slower per call, one every other group lands too late: 3 % slower)
constexpr int kSpreadPer = 1;
// split K across workgroups: at most this many workgroups per launch (one round of the GPU's CUs), and only
// when the problem has at least this many 64-wide k-tiles (shorter ones do not repay the reduction launch:
// 36 -> 18 was measured, another 4.5 % off a batch-1 call)
constexpr int kSplitKMaxGroups = 256, kSplitKMinKTiles = 18;

//  - SK (split K across workgroups, for problems with few tiles and a long K: the out-projection of the MLP at
//    one or two samples per pass): tiles_n counts sk.splits column-tile rows, workgroup (tm, tn) takes k-range
//    tn / sk.tiles_n of column tile tn % sk.tiles_n and leaves its fp32 partial tile in sk.part
//    ([split][tiles_m * BM][sk.tiles_n * BN], padded, so no bounds are needed); splitk_reduce_kernel adds the
//    partial tiles in a fixed order and applies the epilogue.
struct SplitK { int splits, tiles_n, ksub; float* part; };

template <int BM, int BN, int BK, int NS, int WM, int WN, int WK = 1, bool SK = false>
__global__ void __launch_bounds__(WM * WN * WK * 64)
gemm_bf16_xl_kernel(const bf16_t* __restrict__ A, const bf16_t* __restrict__ W, int M, int N, int K, const Epilogue e,
                    int tiles_m, int tiles_n, const SplitK sk)
{
    // WK > 1: the waves form WK groups that share the output tile and split K between them (group g
    // takes the k-tiles g, g + WK, ...); the groups' partial sums are added through LDS before the
    // epilogue.  This doubles the waves per CU for shapes that only yield one small tile per CU.
    constexpr int NWT = WM * WN, NW = NWT * WK, TM = BM / WM, TN = BN / WN, MI = TM / 16, NI = TN / 16, KS = BK / 32;
    constexpr int CPR = BK / 8, RPI = 64 / CPR, RB = 256 / (BK * 2);
    constexpr int STAGE1 = (BM + BN) * BK, STAGE = WK * STAGE1;
    constexpr int SEG1 = (BM + BN) / RPI, SEG = WK * SEG1, LPT = (SEG + NW - 1) / NW;
    constexpr int GROUP_M = 8;
    static_assert(TM % 16 == 0 && TN % 16 == 0 && (BM + BN) % RPI == 0 && BM % 16 == 0, "tile shape");
    extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
    bf16_t* smem = reinterpret_cast<bf16_t*>(smem_raw);

    const int nb = tiles_m * tiles_n, b = blockIdx.x;
    const int xcd = b & 7, local = b >> 3, q = nb >> 3, rem = nb & 7;
    const int idx = xcd * q + (xcd < rem ? xcd : rem) + local;
    const int per_group = GROUP_M * tiles_n, group = idx / per_group, first_m = group * GROUP_M;
    const int gsz = tiles_m - first_m < GROUP_M ? tiles_m - first_m : GROUP_M;
    const int tm = first_m + (idx % per_group) % gsz, tn = (idx % per_group) / gsz;
    const int split = SK ? tn / sk.tiles_n : 0;
    const int m0 = tm * BM, n0 = (SK ? tn - split * sk.tiles_n : tn) * BN;
    if constexpr (SK) { A += split * sk.ksub; W += split * sk.ksub; }   // row stride stays K

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);      // wave-uniform, kept in a scalar register
    const int wk = wave / NWT, wl = wave % NWT, wm = wl % WM, wn = wl / WM;
    const int l16 = lane & 15, quarter = lane >> 4;

    // Cache warm-up for a later launch (see Epilogue::warm): the lines are dealt over the workgroups of
    // the last round, a thread loads one word per line; the values are only consumed by an empty asm
    // after the first barrier, so the loads complete together with the first operand tiles.
    unsigned warm_val = 0;
    if (e.warm_lines) {
        const uint32_t first = nb > 256 ? (uint32_t)nb - 256u : 0u, cnt = (uint32_t)nb - first;
        const uint32_t per = (e.warm_lines + cnt - 1u) / cnt;
        if ((uint32_t)b >= first)
            for (uint32_t t = (uint32_t)tid; t < per; t += NW * 64) {
                const uint32_t line = ((uint32_t)b - first) * per + t;
                if (line < e.warm_lines) warm_val ^= reinterpret_cast<const unsigned*>(e.warm)[(size_t)line * 32];
            }
    }

    // DMA: the A rows and W rows of a k-tile form one row space [0, BM + BN), and a stage holds WK
    // k-tiles one after the other.  A wave-wide instruction covers RPI rows (never straddling the
    // A/W boundary).  Every wave issues LPT instructions; when SEG is not a multiple of the wave
    // count the surplus ones repeat the last segment (same bytes, same place).  Per lane only a
    // 32-bit byte offset is kept; the matrix base and the LDS destination are wave-uniform.
    const int prow = lane / CPR, ppos = lane % CPR;
    uint32_t voff[LPT];
#pragma unroll
    for (int i = 0; i < LPT; ++i) {
        int g = wave * LPT + i; g = g < SEG ? g : SEG - 1;
        const int gl = g % SEG1, r = gl * RPI + prow;
        const int chunk = ppos ^ ((r / RB) & (CPR - 1));
        int row;
        if (gl * RPI < BM) { row = m0 + r; row = row < M ? row : M - 1; }
        else { row = n0 + r - BM; row = row < N ? row : N - 1; }
        voff[i] = ((uint32_t)row * (uint32_t)K + (uint32_t)chunk * 8u) * 2u;
    }
    const uint32_t lds_base = (uint32_t)(uintptr_t)(DRF_LDS_AS unsigned char*)smem_raw;
    // instruction i (of this wave's LPT) of the copy of k-tile kt into `stage`
    auto issue_one = [&](auto ic, int kt, int stage) {
        constexpr int i = decltype(ic)::value;
        int g = wave * LPT + i; g = g < SEG ? g : SEG - 1;
        const int sub = g / SEG1, gl = g % SEG1;
        // written by hand in the scalar-base form (uniform 64-bit base in SGPRs + the lane's 32-bit byte offset),
        // which needs no 64-bit address registers per lane; M0 carries the wave-uniform LDS destination
        const bf16_t* base = (gl * RPI < BM ? A : W) + (kt * WK + sub) * BK;
        const uint32_t dst = lds_base + (uint32_t)(stage * STAGE + sub * STAGE1 + gl * RPI * BK) * 2u;
        const uint32_t vo = voff[i];
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(dst), "v"(vo), "s"(base) : "memory");
    };
    auto issue = [&](int kt, int stage) {
        static_for<0, LPT>([&](auto ic) { issue_one(ic, kt, stage); });
    };

    f32x4 acc[NI][MI];
#pragma unroll
    for (int i = 0; i < NI; ++i)
#pragma unroll
        for (int j = 0; j < MI; ++j) acc[i][j] = (f32x4){ 0.f, 0.f, 0.f, 0.f };

    int koff[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) koff[ks] = l16 * BK + (((ks * 4 + quarter) ^ ((l16 / RB) & (CPR - 1))) << 3);

    // Main loop, software-pipelined at the granularity of one weight fragment.  The MFMAs of a k-tile
    // are G = KS * NI groups (one 16-column weight fragment against the MI activation fragments); the
    // LDS read of the fragment for group g + D is issued just before the MFMAs of group g, into a ring
    // of R = D + 1 register sets, and the activation fragments of a k-step are double-buffered the
    // same way.  The block barrier that hands over the next k-tile (its DMA has landed, every wave has
    // finished reading the current one) sits D groups before the end of the current tile, so each wave
    // leaves it with D groups of MFMAs whose operands are already in registers while the first reads
    // of the new tile are in flight: no LDS latency is exposed at the tile boundary.
    // The fragment reads and their waits are written by hand (ds_read_b128 / s_waitcnt lgkmcnt(n)):
    // with LDS-DMA in the loop the compiler's own wait insertion falls back to lgkmcnt(0), which
    // exposes a full LDS round trip several times per tile.  LDS reads return in order, so before the
    // MFMAs of group g it is enough that at most the reads issued after position g's remain.
    static_assert(NS >= 2 && KS == 2, "the pipelined loop assumes LDS stages of two k-steps");
    constexpr int G = KS * NI;
    constexpr int R = G % 6 == 0 ? 6 : G % 4 == 0 ? 4 : G % 5 == 0 ? 5 : G % 3 == 0 ? 3 : 2, D = R - 1;
    static_assert(G % R == 0 && D < NI && D + MI <= 15, "ring size");
    // With two stages the copy of tile kt + 2 is not issued as one burst after the barrier of tile kt (72
    // wave-wide loads that the vector-memory path takes one per ~17 cycles, during which the issuing waves
    // cannot issue MFMAs) but one instruction per MFMA group: the first HEAD of them in the groups after the
    // barrier, the remaining TAIL in the first groups of the next tile.  All of them are issued long before
    // the next barrier, whose vmcnt(0) covers them as before.
    constexpr int PER = kSpreadPer;                 // copy instructions per MFMA group
    constexpr int HEAD0 = D * PER < LPT ? D * PER : LPT;
    constexpr bool kSpread = NS == 2 && WK == 1 && (LPT - HEAD0 + PER - 1) / PER <= G - D;
    constexpr int HEAD = kSpread ? HEAD0 : LPT, TAIL = LPT - HEAD;
    const int nk = (SK ? sk.ksub : K) / (BK * WK);
    u32x4 fa[2][MI], fw[R];
    const uint32_t lds0 = (uint32_t)(uintptr_t)(DRF_LDS_AS unsigned char*)smem_raw;
    uint32_t a_addr[KS], w_addr[KS];                // byte addresses of this lane's fragments in stage 0
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
        a_addr[ks] = lds0 + (uint32_t)(wk * STAGE1 + wm * TM * BK + koff[ks]) * 2u;
        w_addr[ks] = lds0 + (uint32_t)(wk * STAGE1 + BM * BK + wn * TN * BK + koff[ks]) * 2u;
    }
    // reads of stream position p (0 <= p < G) of a k-tile; aa / wa: this lane's fragment addresses in its stage
    auto fetch = [&](auto pc, const uint32_t (&aa)[KS], const uint32_t (&wa)[KS]) {
        constexpr int p = decltype(pc)::value, ks = p / NI, i = p % NI;
        if constexpr (i == 0)
            static_for<0, MI>([&](auto jc) {
                constexpr int j = decltype(jc)::value;
                lds_read16<j * 16 * BK * 2>(fa[ks & 1][j], aa[ks]);
            });
        lds_read16<i * 16 * BK * 2>(fw[p % R], wa[ks]);
    };

    // tiles 0 .. NS-2 are in flight before the loop; tile kt + NS - 1 is requested once tile kt - 1 has been read
    issue(0, 0);
    // Gated store, all rows of the tile in one slot (the slot length is a multiple of BM): the tile's BN gate
    // values go to LDS behind the stages, once, and the epilogue reads them from there.  Read from global memory
    // in the epilogue they would be loaded per 16 x 16 piece, each load waited for on the spot (and, from the
    // second transposition pass on, behind the stores of the pass before: loads and stores share a counter).
    const bool gate_lds = e.mode == EPI_STORE_GATED && e.rows_per_slot % BM == 0;
    float* sgate = reinterpret_cast<float*>(smem_raw + NS * STAGE * 2);
    if (gate_lds && tid < BN / 4) {
        const int n = n0 + tid * 4;
        const float4 gv = *reinterpret_cast<const float4*>(e.gate + (size_t)fast_div(m0, e.rps_magic, e.rps_shift) * e.gate_ld + (n < N ? n : 0));
        *reinterpret_cast<float4*>(sgate + tid * 4) = gv;   // (the compiler waits for every load before this write:
    }                                                       //  the later stages are requested only now)
#pragma unroll
    for (int t = 1; t < NS - 1; ++t)
        if (t < nk) issue(t, t);
    if (NS > 2 && nk >= NS - 1) wait_vmcnt<LPT * (NS - 2)>(); else wait_vmcnt<0>();
    asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
    asm volatile("" ::"v"(warm_val));
    if (NS - 1 < nk) issue(NS - 1, NS - 1);
    static_for<0, D>([&](auto pc) { fetch(pc, a_addr, w_addr); });
    int cs = 0;                                     // stage of tile kt
    for (int kt = 0; kt < nk; ++kt) {
        const int ns = cs + 1 == NS ? 0 : cs + 1;
        const uint32_t co = (uint32_t)cs * (uint32_t)(STAGE * 2), no = (uint32_t)ns * (uint32_t)(STAGE * 2);
        uint32_t ca[KS], cw[KS], na[KS], nw[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) { ca[ks] = a_addr[ks] + co; cw[ks] = w_addr[ks] + co; na[ks] = a_addr[ks] + no; nw[ks] = w_addr[ks] + no; }
        static_for<0, G>([&](auto gc) {
            constexpr int g = decltype(gc)::value;
            if constexpr (g + D == G) {
                // tile kt+1 has landed (vmcnt 0) and this wave's reads of tile kt are complete (lgkmcnt 0), for
                // every wave after the barrier: the stage of tile kt may be refilled
                // (the NS - 2 younger tiles may still be in flight; near the end fewer are, so wait for all)
                if (NS > 2 && kt + NS - 1 < nk) wait_vmcnt<LPT * (NS - 2)>(); else wait_vmcnt<0>();
                asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory");
                if constexpr (!kSpread) {
                    if (kt + NS < nk) issue(kt + NS, cs);
                }
            }
            if constexpr (kSpread) {
                static_for<0, PER>([&](auto uc) {
                    constexpr int u = decltype(uc)::value;
                    if constexpr (g >= G - D && (g - (G - D)) * PER + u < HEAD) {
                        if (kt + NS < nk) issue_one(std::integral_constant<int, (g - (G - D)) * PER + u>{}, kt + NS, cs);
                    } else if constexpr (g < G - D && g * PER + u < TAIL) {
                        // the rest of the copy that the previous tile's last groups started: tile kt + 1, into the other stage
                        if (kt >= 1 && kt + 1 < nk) issue_one(std::integral_constant<int, HEAD + g * PER + u>{}, kt + 1, ns);
                    }
                });
            }
            {
                // on the last tile the positions beyond it read the idle stage: valid LDS, values unused
                // (drained by the wait after the loop)
                if constexpr (g + D < G) fetch(std::integral_constant<int, g + D>{}, ca, cw);
                else fetch(std::integral_constant<int, g + D - G>{}, na, nw);
                __builtin_amdgcn_sched_barrier(0);
                // reads issued after position g's: one per later position, plus the activation fragments
                // of a k-step that starts among them
                constexpr int later = D + (((g + D) / NI) != (g / NI) ? MI : 0);
                if constexpr (g % NI == 0) wait_frags<later, MI>(fw[g % R], fa[(g / NI) & 1]);
                else wait_frag<later>(fw[g % R]);
                static_for<0, MI>([&](auto jc) {
                    constexpr int j = (g & 1) ? MI - 1 - decltype(jc)::value : decltype(jc)::value;   // snake: one operand changes per MFMA
                    acc[g % NI][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, fw[g % R]),
                                                                             __builtin_bit_cast(bf16x8, fa[(g / NI) & 1][j]),
                                                                             acc[g % NI][j], 0, 0, 0);
                });
                __builtin_amdgcn_sched_barrier(0);
            }
        });
        cs = ns;
    }
    wait_lgkmcnt<0>();                              // the last tile's look-ahead reads

    if constexpr (SK) {
        // partial tile, straight from the accumulators: acc[i][j][r] is (m = j*16 + l16, n = i*16 + 4*quarter + r)
        static_assert(WK == 1, "split K across workgroups or across wave groups, not both");
        float* pt = sk.part + ((size_t)split * tiles_m * BM + m0 + wm * TM) * ((size_t)sk.tiles_n * BN) + n0 + wn * TN;
#pragma unroll
        for (int i = 0; i < NI; ++i)
#pragma unroll
            for (int j = 0; j < MI; ++j)
                *reinterpret_cast<f32x4*>(pt + (size_t)(j * 16 + l16) * ((size_t)sk.tiles_n * BN) + i * 16 + 4 * quarter) = acc[i][j];
        return;
    }
    // ---- epilogue through LDS: acc[i][j][r] is (m = j*16 + l16, n = i*16 + 4*quarter + r) of the wave tile
    __syncthreads();
    constexpr int PART = (WK - 1) * NWT * TM * TN * 4;              // partial sums of the other K groups
    if constexpr (WK > 1) {
        static_assert(PART < NS * STAGE * 2, "LDS too small for the split-K partial sums");
        f32x4* part = reinterpret_cast<f32x4*>(smem_raw);
        if (wk > 0) {
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < MI; ++j) part[(((wk - 1) * NWT + wl) * NI * MI + i * MI + j) * 64 + lane] = acc[i][j];
        }
        __syncthreads();
        if (wk > 0) return;                                         // the first group finishes the tile
#pragma unroll
        for (int g = 0; g < WK - 1; ++g)
#pragma unroll
            for (int i = 0; i < NI; ++i)
#pragma unroll
                for (int j = 0; j < MI; ++j) acc[i][j] += part[((g * NWT + wl) * NI * MI + i * MI + j) * 64 + lane];
    }
    constexpr int WBYTES = (NS * STAGE * 2 - PART) / NWT / 16 * 16; // this wave's private slice of the stages
    unsigned char* wbuf = smem_raw + PART + wl * WBYTES;
    const int mw = m0 + wm * TM, nw = n0 + wn * TN;
    // bias of this lane's columns, fetched in one batch (kept in registers: reading it from LDS per 16 x 16 piece
    // like the gate was measured 1 % slower per call)
    float4 bb[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int n = nw + i * 16 + 4 * quarter;
        bb[i] = *reinterpret_cast<const float4*>(e.bias + (n < N ? n : 0));
    }
    if (e.mode == EPI_RESID || e.out_f32) {
        constexpr int ROWB = TN * 4 + ((TN * 4) % 128 == 0 ? 16 : 0);
        constexpr int RPP = (WBYTES / ROWB) / 16 * 16 < TM ? (WBYTES / ROWB) / 16 * 16 : TM;   // rows per pass
        static_assert(RPP >= 16, "LDS slice too small for the fp32 epilogue");
        constexpr int CH = TN / 4, IT = (RPP * CH + 63) / 64;       // float4 chunks per row, chunks per lane and pass
        auto run = [&](auto mode_c) {
            constexpr int MODE = decltype(mode_c)::value;
#pragma unroll
            for (int j0 = 0; j0 < MI; j0 += RPP / 16) {
#pragma unroll
                for (int jj = 0; jj < RPP / 16; ++jj) {
                    const int j = j0 + jj;
                    if (j < MI) {
#pragma unroll
                        for (int i = 0; i < NI; ++i) {
                            float4 v = make_float4(acc[i][j][0] + bb[i].x, acc[i][j][1] + bb[i].y, acc[i][j][2] + bb[i].z,
                                                   acc[i][j][3] + bb[i].w);
                            if (MODE == EPI_STORE_GELU) { v.x = gelu_tanh(v.x); v.y = gelu_tanh(v.y); v.z = gelu_tanh(v.z); v.w = gelu_tanh(v.w); }
                            *reinterpret_cast<float4*>(wbuf + (jj * 16 + l16) * ROWB + (i * 16 + 4 * quarter) * 4) = v;
                        }
                    }
                }
                // rows back out, kBatch chunks per lane at a time: their loads are all issued before
                // the first dependent store
                constexpr int kBatch = 3;
#pragma unroll
                for (int it0 = 0; it0 < IT; it0 += kBatch) {
                    float4 vv[kBatch], xx[kBatch], gg[kBatch];
                    bool ok[kBatch];
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        const int id = lane + (it0 + u) * 64, rl = id / CH, c = id % CH;
                        const int m = mw + j0 * 16 + rl, n = nw + c * 4;
                        ok[u] = it0 + u < IT && id < RPP * CH && j0 * 16 + rl < TM && m < M && n < N;
                        if (ok[u]) {
                            vv[u] = *reinterpret_cast<const float4*>(wbuf + rl * ROWB + c * 16);
                            if (MODE == EPI_RESID) {
                                xx[u] = *reinterpret_cast<const float4*>((const float*)e.out + (size_t)m * e.ldo + n);
                                gg[u] = e.gate ? *reinterpret_cast<const float4*>(e.gate + (size_t)fast_div(m, e.rps_magic, e.rps_shift) * e.gate_ld + n)
                                               : make_float4(1.f, 1.f, 1.f, 1.f);
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < kBatch; ++u) {
                        const int id = lane + (it0 + u) * 64, rl = id / CH, c = id % CH;
                        const int m = mw + j0 * 16 + rl, n = nw + c * 4;
                        if (ok[u]) {
                            float4 o = vv[u];
                            if (MODE == EPI_RESID) {
                                o.x = fmaf(gg[u].x, vv[u].x, xx[u].x); o.y = fmaf(gg[u].y, vv[u].y, xx[u].y);
                                o.z = fmaf(gg[u].z, vv[u].z, xx[u].z); o.w = fmaf(gg[u].w, vv[u].w, xx[u].w);
                            }
                            *reinterpret_cast<float4*>((float*)e.out + (size_t)m * e.ldo + n) = o;
                        }
                    }
                }
            }
        };
        if (e.mode == EPI_RESID) run(std::integral_constant<int, EPI_RESID>{});
        else if (e.mode == EPI_STORE_GELU) run(std::integral_constant<int, EPI_STORE_GELU>{});
        else run(std::integral_constant<int, EPI_STORE>{});
    } else {
        constexpr int ROWB = TN * 2 + ((TN * 2) % 128 == 0 ? 16 : 0);
        constexpr int RPP = (WBYTES / ROWB) / 16 * 16 < TM ? (WBYTES / ROWB) / 16 * 16 : TM;
        static_assert(RPP >= 16, "LDS slice too small for the bf16 epilogue");
        constexpr int CH = TN / 8, IT = (RPP * CH + 63) / 64;       // 16-byte chunks per row, chunks per lane and pass
        auto run = [&](auto mode_c, auto gate_lds_c) {
            constexpr int MODE = decltype(mode_c)::value;
            constexpr bool GLDS = decltype(gate_lds_c)::value;
#pragma unroll
            for (int j0 = 0; j0 < MI; j0 += RPP / 16) {
#pragma unroll
                for (int jj = 0; jj < RPP / 16; ++jj) {
                    const int j = j0 + jj;
                    if (j < MI) {
                        // EPI_STORE_GATED: the gate row of this lane's output row (rows past M use the last one)
                        const float* grow = nullptr;
                        if constexpr (MODE == EPI_STORE_GATED && !GLDS) {
                            const int mr = mw + j * 16 + l16;
                            grow = e.gate + (size_t)fast_div(mr < M ? mr : M - 1, e.rps_magic, e.rps_shift) * e.gate_ld;
                        }
#pragma unroll
                        for (int i = 0; i < NI; ++i) {
                            float v0 = acc[i][j][0] + bb[i].x, v1 = acc[i][j][1] + bb[i].y, v2 = acc[i][j][2] + bb[i].z, v3 = acc[i][j][3] + bb[i].w;
                            if (MODE == EPI_STORE_GELU) { v0 = gelu_tanh(v0); v1 = gelu_tanh(v1); v2 = gelu_tanh(v2); v3 = gelu_tanh(v3); }
                            if constexpr (MODE == EPI_STORE_GATED) {
                                float4 g;
                                if constexpr (GLDS) {
                                    g = *reinterpret_cast<const float4*>(sgate + wn * TN + i * 16 + 4 * quarter);
                                } else {
                                    const int ng = nw + i * 16 + 4 * quarter;
                                    g = *reinterpret_cast<const float4*>(grow + (ng < N ? ng : 0));
                                }
                                v0 *= g.x; v1 *= g.y; v2 *= g.z; v3 *= g.w;
                            }
                            bf16x4 o = { (bf16_t)v0, (bf16_t)v1, (bf16_t)v2, (bf16_t)v3 };
                            *reinterpret_cast<bf16x4*>(wbuf + (jj * 16 + l16) * ROWB + (i * 16 + 4 * quarter) * 2) = o;
                        }
                    }
                }
                // rows back out: all of a pass's LDS reads first (reading is harmless where nothing is stored), then the stores
                constexpr int kRB = 4;                                  // LDS reads in flight before their stores
#pragma unroll
                for (int it0 = 0; it0 < IT; it0 += kRB) {
                    bf16x8 rv[kRB];
#pragma unroll
                    for (int u = 0; u < kRB; ++u) {
                        const int id = lane + (it0 + u) * 64, idc = id < RPP * CH ? id : RPP * CH - 1;
                        if (it0 + u < IT) rv[u] = *reinterpret_cast<const bf16x8*>(wbuf + (idc / CH) * ROWB + (idc % CH) * 16);
                    }
#pragma unroll
                    for (int u = 0; u < kRB; ++u) {
                        const int id = lane + (it0 + u) * 64, rl = id / CH, c = id % CH;
                        const int m = mw + j0 * 16 + rl, n = nw + c * 8;
                        if (it0 + u < IT && id < RPP * CH && j0 * 16 + rl < TM && m < M && n < N) {
                            const size_t off = MODE == EPI_STORE_HEADS ? heads_offset(e, m, n) : (size_t)m * e.ldo + n;
                            if (n + 8 <= N)
                                *reinterpret_cast<bf16x8*>((bf16_t*)e.out + off) = rv[u];
                            else            // N is a multiple of 4: the last chunk of a row may be half valid
                                *reinterpret_cast<bf16x4*>((bf16_t*)e.out + off) = __builtin_shufflevector(rv[u], rv[u], 0, 1, 2, 3);
                        }
                    }
                }
            }
        };
        if (e.mode == EPI_STORE_GELU) run(std::integral_constant<int, EPI_STORE_GELU>{}, std::false_type{});
        else if (e.mode == EPI_STORE_HEADS) run(std::integral_constant<int, EPI_STORE_HEADS>{}, std::false_type{});
        else if (e.mode == EPI_STORE_GATED && gate_lds) run(std::integral_constant<int, EPI_STORE_GATED>{}, std::true_type{});
        else if (e.mode == EPI_STORE_GATED) run(std::integral_constant<int, EPI_STORE_GATED>{}, std::false_type{});
        else run(std::integral_constant<int, EPI_STORE>{}, std::false_type{});
    }
}

// Sum of the split-K partial tiles (fixed order: deterministic), then the epilogue; one thread per 4 columns.
__global__ void __launch_bounds__(256)
splitk_reduce_kernel(const float* __restrict__ part, int splits, size_t split_stride, int ldp, int M, int N, const Epilogue e)
{
    const int n4 = N / 4, id = blockIdx.x * 256 + threadIdx.x;
    if (id >= M * n4) return;
    const int m = id / n4, n = (id - m * n4) * 4;
    const float* p = part + (size_t)m * ldp + n;
    float4 v = *reinterpret_cast<const float4*>(p);
    for (int s2 = 1; s2 < splits; ++s2) {
        const float4 u = *reinterpret_cast<const float4*>(p + (size_t)s2 * split_stride);
        v.x += u.x; v.y += u.y; v.z += u.z; v.w += u.w;
    }
    epilogue4(e, m, n, v.x, v.y, v.z, v.w);
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

template <int BM, int BN, int BK, int NS, int WM, int WN, int WK = 1>
drf_status launch_bf16_xl(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st)
{
    constexpr size_t smem = (size_t)NS * WK * (BM + BN) * BK * sizeof(bf16_t) + BN * sizeof(float);   // stages + gate row
    static_assert(smem <= 160 * 1024, "LDS of a CU");
    static bool attr_set = false;
    auto kern = gemm_bf16_xl_kernel<BM, BN, BK, NS, WM, WN, WK>;
    if (K % (BK * WK) != 0) DRF_FAIL(DRF_ESHAPE, "bf16 GEMM tile needs K %% %d == 0 (K=%d)", BK * WK, K);
    if (!attr_set) {
        DRF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(WM * WN * WK * 64), smem, st, A, W, M, N, K, e, tiles_m, tiles_n, SplitK{});
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

// Split-K form of the 128 x 128 tile: `splits` workgroups per output tile, partial tiles in `part`
// (splits * tiles * 128 * 128 floats), then the reduction with the epilogue.
drf_status launch_bf16_splitk(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st,
                              int splits, float* part)
{
    constexpr int BM = 128, BN = 128, BK = 64;
    constexpr int NS = 4;
    constexpr size_t smem = (size_t)NS * (BM + BN) * BK * sizeof(bf16_t) + BN * sizeof(float);
    static bool attr_set = false;
    auto kern = gemm_bf16_xl_kernel<BM, BN, BK, NS, 2, 2, 1, true>;
    if (!attr_set) {
        DRF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const int tiles_m = (M + BM - 1) / BM, tiles_n = (N + BN - 1) / BN;
    SplitK sk{ splits, tiles_n, K / splits, part };
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n * splits), dim3(256), smem, st, A, W, M, N, K, e, tiles_m, tiles_n * splits, sk);
    DRF_HIP(hipGetLastError());
    const int ldp = tiles_n * BN;
    const long long quads = (long long)M * (N / 4);
    hipLaunchKernelGGL(splitk_reduce_kernel, dim3((unsigned)((quads + 255) / 256)), dim3(256), 0, st, part, splits,
                       (size_t)tiles_m * BM * ldp, ldp, M, N, e);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace

size_t gemm_splitk_scratch_bytes() { return (size_t)kSplitKMaxGroups * 128 * 128 * sizeof(float); }

drf_status launch_gemm_bf16(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st,
                            int variant, float* splitk_scratch)
{
    if (M == 0 || N == 0) return DRF_OK;
    if (K % 64 != 0 || N % 4 != 0 || e.ldo % 4 != 0) DRF_FAIL(DRF_ESHAPE, "bf16 GEMM needs K %% 64 == 0 and N %% 4 == 0 (M=%d N=%d K=%d)", M, N, K);
    if (e.mode == EPI_STORE_HEADS && (e.out_f32 || e.hd % 8 != 0 || N % e.hid != 0))
        DRF_FAIL(DRF_ESHAPE, "head-major store needs bf16 output and head width %% 8 == 0");
    if (e.mode == EPI_STORE_GATED && (e.out_f32 || !e.gate)) DRF_FAIL(DRF_ESHAPE, "gated store needs bf16 output and a gate");
    if ((size_t)M * K >= ((size_t)1 << 31) || (size_t)N * K >= ((size_t)1 << 31))
        DRF_FAIL(DRF_ESHAPE, "bf16 GEMM operand exceeds 2^31 elements");
    int v = variant;
    if (v == 0) {
        // Pick the tile shape that wastes the least MFMA work: padding of the last tile row /
        // column, and the idle CUs of the last round of 256 concurrent tiles.
        struct Cand { int id, bm, bn; double eff; };
        const Cand cands[] = { { 2, 256, 288, 1.0 }, { 3, 256, 256, 0.97 }, { 4, 128, 288, 0.8 }, { 7, 128, 144, 0.6 },
                               { 5, 128, 128, 0.55 } };
        double best = 0.0;
        v = 1;
        if (M >= 512) {
            for (const Cand& c : cands) {
                const double tm = (M + c.bm - 1) / c.bm, tn = (N + c.bn - 1) / c.bn, tiles = tm * tn;
                const double rounds = (double)((long long)(tiles + 255) / 256);
                const double score = c.eff * ((double)M * N) / (rounds * 256.0 * c.bm * c.bn);
                if (score > best) { best = score; v = c.id; }
            }
            // one small tile per CU: let two wave groups split K inside the block
            if (v == 7 && K % 128 == 0 && K >= 1024) v = 8;
        }
    }
    // Few 128 x 128 tiles and a long K (one or two samples per pass: the MLP's out-projection is 36 tiles of 72
    // k-tiles on 256 CUs, the attention out-projection 36 of 18): split K over as many workgroups as fit one
    // round, the k-tiles dividing evenly and at least six to a workgroup.
    if (v == 10) v = 5;
    if ((v == 5 || v == 1) && (variant == 0 || variant == 10) && splitk_scratch && K / 64 >= kSplitKMinKTiles) {
        const int tiles = ((M + 127) / 128) * ((N + 127) / 128), nk = K / 64;
        int splits = 0;
        for (int s2 = 2; s2 <= 8 && s2 * tiles <= kSplitKMaxGroups; ++s2)
            if (nk % s2 == 0 && nk / s2 >= 6) splits = s2;
        if (splits) return launch_bf16_splitk(A, W, M, N, K, e, st, splits, splitk_scratch);
    }
    switch (v) {
    case 2: return launch_bf16_xl<256, 288, 64, 2, 4, 2>(A, W, M, N, K, e, st);
    case 3: return launch_bf16_xl<256, 256, 64, 2, 4, 2>(A, W, M, N, K, e, st);
    case 4: return launch_bf16_xl<128, 288, 64, 2, 2, 2>(A, W, M, N, K, e, st);
    case 5: return launch_bf16_xl<128, 128, 64, 4, 2, 2>(A, W, M, N, K, e, st);
    case 6: return launch_bf16_xl<256, 288, 64, 2, 4, 3>(A, W, M, N, K, e, st);
    case 7: return launch_bf16_xl<128, 144, 64, 4, 4, 1>(A, W, M, N, K, e, st);
    case 8: return launch_bf16_xl<128, 144, 64, 2, 4, 1, 2>(A, W, M, N, K, e, st);
    default: return launch_bf16_tile<128, 128, 2, 2>(A, W, M, N, K, e, st);
    }
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
