// Multi-head attention softmax(q k^T / sqrt(d)) v without mask.
// bf16 path: flash-style, one wave per 32 queries, scores computed transposed
// (S^T = K Q^T) so that each lane owns one query column and the online softmax needs a
// single cross-lane exchange; P^T feeds the second MFMA straight from registers.
// fp32 path: a few lanes per query over kv rows read through the cache, for the fp32 configuration.
#include <type_traits>

#include "common.h"

namespace drf {

namespace {

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
#define DRF_LDS_PTR __attribute__((address_space(3)))

constexpr int kKvb = 64;            // kv rows per online-softmax step
// max of three without the canonicalisation the generic fmaxf lowering adds per operand
__device__ inline float max3(float a, float b, float c)
{
    float r;
    asm("v_max3_f32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
    return r;
}
constexpr int kPersistGroups = 256;  // workgroups of a persistent launch: one per CU of the MI355X
constexpr float kTau = 8.f;         // lazy-rescale headroom of the online softmax, in log2 units

// KS = ceil(d / 16) k-steps of the score MFMA; DT = ceil(d / 32) row tiles of O^T; NW waves of 32
// queries per block, all sharing the staged K / V (NW = 8 covers the 256 tokens of a DiT-XL head
// with one block, so K and V are read and transposed once per head).
// K and V^T are staged in chunks of KC kv rows, NB chunk buffers: a sequence of up to KC rows is
// staged once (NB = 1) and the waves then run their steps without any block barrier; longer
// sequences alternate two buffers with one barrier per chunk.  Between barriers the two waves of
// a SIMD drift apart, so the MFMAs of one overlap the softmax arithmetic of the other; a barrier
// per 64-row step would keep every wave in the same phase and leave either the matrix or the
// vector unit idle.
// Per step 64 kv rows: two 32 x 32 score tiles, one online-softmax update, four PV k-chunks.
// V^T is stored with the 16 kv rows of each k-chunk permuted to [0-3, 8-11 | 4-7, 12-15]: that is
// the order in which the score MFMA leaves a lane's P values, so the PV operand is one 16-byte read,
// and the transposing store of four kv rows of one d is one 8-byte write.
// VTR: V is staged as stored instead (row-major, contiguous 16-byte pieces like K: coalesced loads and
// 16-byte LDS writes) and the V^T operand is produced by the LDS transpose read, whose groups of four kv
// rows are the ones in which the score MFMA leaves a lane's P values.  Cheaper between the steps, dearer
// inside them (two 8-byte reads per operand): it wins where a chunk is a single step (sequences of up to
// 256 rows: -3.7 % for those launches) and loses on long sequences (+3 % at 4096 rows).
// The grid is one-dimensional over work items (query block, head, slot), query block fastest.  With
// PERSIST a workgroup takes items blockIdx.x, blockIdx.x + gridDim.x, ... and, while it runs the steps
// of an item's last chunk, already has the next item's Q fragments and first K / V chunk in flight, so
// only the first item of a workgroup waits for its first loads with nothing else to do.
template <int KS, int DT, int NW, int KC, int NB, bool PERSIST, bool VTR>
__global__ void __launch_bounds__(NW * 64) attn_bf16_kernel(const AttnArgs a, float scale_log2, int nqb, int n_items)
{
    static_assert(!PERSIST || NB == 2, "the cross-item prefetch needs two chunk buffers");
    constexpr int NT = NW * 64;
    // VTR row stride of V: 4 consecutive rows x 32 bytes tile the 32 banks
    constexpr int DK = KS * 16, LDKS = DK + 8, LDV = VTR ? DT * 32 + 16 : KC + 8;
    constexpr int KBUF = KC * LDKS, VBUF = VTR ? KC * LDV : DT * 32 * LDV;
    constexpr int MAXK = (KC * (KS * 2) + NT - 1) / NT;                   // 16-byte K pieces of a chunk per thread
    constexpr int MAXV = VTR ? MAXK : ((KC / 4) * (KS * 2) + NT - 1) / NT;  // (4 kv rows x 8 d) V blocks per thread (VTR: pieces as for K)
    extern __shared__ __attribute__((aligned(16))) unsigned char attn_smem[];
    bf16_t* sK = reinterpret_cast<bf16_t*>(attn_smem);                    // [buf][kv][d padded]
    bf16_t* sVt = sK + NB * KBUF;                                         // [buf][d padded][kv, permuted]; VTR: [buf][kv][d padded]
    constexpr int LDO = DT * 32 + 8;                                      // row stride of a wave's output tile
    bf16_t* sOut = sVt + NB * VBUF + (threadIdx.x >> 6) * (32 * LDO);     // [wave][32 queries][d padded]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, l32 = lane & 31, half = lane >> 5;
    const int d = a.d;
    const bf16x8 zero8 = { 0, 0, 0, 0, 0, 0, 0, 0 };
    // where a work item's rows are, and this lane's query in it
    struct Item { const bf16_t *Q, *Kp, *Vp; int slot, h, q; };
    auto locate = [&](int item) {
        Item it;
        const int qb = item % nqb, hs = item / nqb;
        it.h = hs % a.heads; it.slot = hs / a.heads;
        const int kvb = a.kv_mod ? it.slot % a.kv_mod : it.slot;
        it.Q = (const bf16_t*)a.q + it.slot * a.q_slot_stride + it.h * a.q_head_stride;
        it.Kp = (const bf16_t*)a.k + kvb * a.kv_batch_stride + it.h * a.kv_head_stride;
        it.Vp = (const bf16_t*)a.v + kvb * a.kv_batch_stride + it.h * a.kv_head_stride;
        it.q = qb * (NW * 32) + wave * 32 + l32;
        return it;
    };
    // this lane's Q fragments of an item (B operand: 8 consecutive d per k-step half)
    auto load_q = [&](const Item& it, bf16x8 (&f)[KS]) {
        const int qc = it.q < a.Nq ? it.q : a.Nq - 1;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int dd = ks * 16 + half * 8;
            f[ks] = dd < d ? *reinterpret_cast<const bf16x8*>(it.Q + (size_t)qc * a.ldq + dd) : zero8;
        }
    };
    // Workgroup ids are dealt round-robin over the 8 XCDs, each with its own L2.  The query blocks of one
    // (slot, head) read the same K / V rows, so position v of the launch order takes the item that puts
    // consecutive items on one XCD: its L2 then fetches a head's K / V once, not once per XCD.
    auto item_at = [&](int v) {
        const int q8 = n_items >> 3, rem = n_items & 7, xcd = v & 7;
        return nqb > 1 ? xcd * q8 + (xcd < rem ? xcd : rem) + (v >> 3) : v;
    };
    int vpos = blockIdx.x, item = item_at(vpos);
    Item cur = locate(item);

    // zero the padding that loads never touch: K columns [d, DK), V^T rows [d, DT*32)
    for (int i = tid; i < NB * (KBUF + VBUF) / 8; i += NT) reinterpret_cast<bf16x8*>(sK)[i] = zero8;
    // When the head width leaves a padding row in O^T, V^T row d is set to ones: the PV MFMA
    // then accumulates the softmax denominator there for free.  (VTR: the last padding column of V, so that the
    // accumulator register that ends up holding the denominator is known at compile time: -4.5 % for the
    // 256-row launches; the same move in the V^T layout made the 4096-row launches 3.5 % slower.)
    const bool ones_row = d < DT * 32;
    __syncthreads();
    if (ones_row) {
        if constexpr (VTR) {
            for (int i = tid; i < NB * KC; i += NT) sVt[(i / KC) * VBUF + (i % KC) * LDV + DT * 32 - 1] = (bf16_t)1.f;
        } else {
            for (int i = tid; i < NB * LDV; i += NT) sVt[(i / LDV) * VBUF + d * LDV + i % LDV] = (bf16_t)1.f;
        }
    }

    bf16x8 qf[KS];
    load_q(cur, qf);
    f32x16 o[DT];
    float m_run, l_run;                         // running max of the raw scores, running sum
    const int dch = d / 8, nch = KC * dch, nvb = (KC / 4) * dch;

    // K: consecutive threads take consecutive 16-byte pieces of a row (coalesced loads, 16-byte LDS
    // writes).  V: a thread takes 4 consecutive kv rows of one 8-wide d piece and writes, for each
    // of the 8 d, the 4 kv values as one 8-byte piece of the V^T row.
    bf16x8 rk[MAXK], rv[MAXV][VTR ? 1 : 4];
    auto fetch = [&](const Item& it, int kv0) {
#pragma unroll
        for (int c = 0; c < MAXK; ++c) {
            const int id = tid + c * NT, r = id / dch, cc = id % dch;
            rk[c] = zero8;
            if (id < nch && kv0 + r < a.Nk) rk[c] = *reinterpret_cast<const bf16x8*>(it.Kp + (size_t)(kv0 + r) * a.ldk + cc * 8);
        }
        if constexpr (VTR) {
#pragma unroll
            for (int c = 0; c < MAXV; ++c) {
                const int id = tid + c * NT, r = id / dch, cc = id % dch;
                rv[c][0] = zero8;
                if (id < nch && kv0 + r < a.Nk) rv[c][0] = *reinterpret_cast<const bf16x8*>(it.Vp + (size_t)(kv0 + r) * a.ldk + cc * 8);
            }
        } else {
#pragma unroll
            for (int c = 0; c < MAXV; ++c) {
                const int id = tid + c * NT, g4 = id % (KC / 4), cc = id / (KC / 4);
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    rv[c][j] = zero8;
                    if (id < nvb && kv0 + 4 * g4 + j < a.Nk)
                        rv[c][j] = *reinterpret_cast<const bf16x8*>(it.Vp + (size_t)(kv0 + 4 * g4 + j) * a.ldk + cc * 8);
                }
            }
        }
    };
    auto stage = [&](int buf) {
        bf16_t* bk = sK + buf * KBUF;
        bf16_t* bv = sVt + buf * VBUF;
#pragma unroll
        for (int c = 0; c < MAXK; ++c) {
            const int id = tid + c * NT, r = id / dch, cc = id % dch;
            if (id < nch) *reinterpret_cast<bf16x8*>(bk + r * LDKS + cc * 8) = rk[c];
        }
        if constexpr (VTR) {
#pragma unroll
            for (int c = 0; c < MAXV; ++c) {
                const int id = tid + c * NT, r = id / dch, cc = id % dch;
                if (id < nch) *reinterpret_cast<bf16x8*>(bv + r * LDV + cc * 8) = rv[c][0];
            }
        } else {
#pragma unroll
            for (int c = 0; c < MAXV; ++c) {
                const int id = tid + c * NT, g4 = id % (KC / 4), cc = id / (KC / 4);
                // kv rows 4 g4 .. 4 g4 + 3 of the chunk: position of row r16 inside its 16-row group is
                // 8 * ((r16 >> 2) & 1) + (r16 & 3) + 4 * (r16 >> 3)
                const int k4 = g4 & 3, pos = 16 * (g4 >> 2) + 8 * (k4 & 1) + 4 * (k4 >> 1);
                if (id < nvb) {
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const bf16x4 w = { rv[c][0][e], rv[c][1][e], rv[c][2][e], rv[c][3][e] };
                        *reinterpret_cast<bf16x4*>(bv + (cc * 8 + e) * LDV + pos) = w;
                    }
                }
            }
        }
    };

    // one online-softmax step over the 64 kv rows at row `row0` of a staged chunk (global row kv0)
    auto step = [&](const bf16_t* bk, const bf16_t* bv, int row0, int kv0) {
        // S^T[kv][q] = sum_d K[kv][d] Q[q][d] for the two 32-row halves.  All K fragments of the step
        // are requested before the first MFMA, and the V^T fragments right after the score MFMAs, so
        // that they land while the softmax runs.
        bf16x8 kf[2][KS];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                kf[t][ks] = *reinterpret_cast<const bf16x8*>(bk + (row0 + t * 32 + l32) * LDKS + ks * 16 + half * 8);
        f32x16 s[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const f32x16 zero16 = { 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f };
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                s[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[t][ks], qf[ks], ks == 0 ? zero16 : s[t], 0, 0, 0);
        }
        bf16x8 vf[2][2][DT];
        // VTR: the 16 lanes of a group point at 4 kv rows x 16 d (8 bytes each) and lane i receives column i of
        // the 4 rows; two reads per operand: kv rows 16 c + 4 half + (0..3) and the same + 8, the two groups of
        // four kv rows that a lane's P values of k-chunk c belong to
        const bf16_t* vl = bv + (row0 + 4 * half + ((lane & 15) >> 2)) * LDV + (l32 & 16) + 4 * (lane & 3);
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c)
#pragma unroll
                for (int tt = 0; tt < DT; ++tt) {
                    if constexpr (VTR) {
                        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((DRF_LDS_PTR s16x4*)(vl + (t * 32 + 16 * c) * LDV + tt * 32));
                        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((DRF_LDS_PTR s16x4*)(vl + (t * 32 + 16 * c + 8) * LDV + tt * 32));
                        vf[t][c][tt] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
                    } else {
                        vf[t][c][tt] = *reinterpret_cast<const bf16x8*>(bv + (tt * 32 + l32) * LDV + row0 + t * 32 + 16 * c + 8 * half);
                    }
                }
        __builtin_amdgcn_sched_barrier(0);
        // register r of s[t] holds kv row t*32 + 8*(r/4) + 4*half + r%4 of the step
        if (kv0 + kKvb > a.Nk) {            // ragged last step: rows past the end do not take part
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
            const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * scale_log2);   // 0 on the first step
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
        // 16c + 4*half + e (e < 4) or 16c + 8 + 4*half + e - 4 of the 32-row half, for both operands:
        // in the permuted V^T row these are the 8 consecutive values at 16c + 8*half.
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int c = 0; c < 2; ++c) {
                bf16x8 pf;
#pragma unroll
                for (int e2 = 0; e2 < 8; ++e2) pf[e2] = (bf16_t)s[t][8 * c + e2];
#pragma unroll
                for (int tt = 0; tt < DT; ++tt) o[tt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[t][c][tt], pf, o[tt], 0, 0, 0);
            }
    };

    // The Q fragments are settled here, before any chunk is in flight behind them: a first use inside
    // the chunk loop would make the compiler wait for every outstanding load (vmcnt(0)) at each step,
    // which would expose the loads of the chunk being prefetched.
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
    fetch(cur, 0);
    __syncthreads();                            // zero fill and ones row done
    stage(0);
    __syncthreads();
    int buf = 0;
    for (;;) {
        const int vnxt = vpos + (int)gridDim.x;
        const bool has_next = PERSIST && vnxt < n_items;
        const int nxt = has_next ? item_at(vnxt) : item;
        Item np = cur;
#pragma unroll
        for (int t = 0; t < DT; ++t)
#pragma unroll
            for (int r = 0; r < 16; ++r) o[t][r] = 0.f;
        m_run = -INFINITY; l_run = 0.f;
        for (int c0 = 0; c0 < a.Nk; c0 += KC) {
            // chunk c0 is visible in `buf`; with two buffers the next chunk (of this item, or the first
            // one of the workgroup's next item together with that item's Q fragments) is fetched now and
            // staged after this chunk's steps (the other buffer was last read before the previous barrier)
            const bool more = c0 + KC < a.Nk;
            if (NB == 2 && more) fetch(cur, c0 + KC);
            if (PERSIST && !more && has_next) {
                np = locate(nxt);
                fetch(np, 0);
            }
            const bf16_t* bk = sK + buf * KBUF;
            const bf16_t* bv = sVt + buf * VBUF;
            for (int r0 = 0; r0 < KC && c0 + r0 < a.Nk; r0 += kKvb) step(bk, bv, r0, c0 + r0);
            if (PERSIST && !more && has_next) {     // the old fragments are dead: the next item's take their place
                load_q(np, qf);
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) asm volatile("" : "+v"(qf[ks]));
            }
            if (more || has_next) {
                if (NB == 2) {
                    stage(buf ^ 1);
                    buf ^= 1;
                } else {                        // single buffer: refill in place
                    __syncthreads();
                    fetch(cur, c0 + KC);
                    stage(0);
                }
                __syncthreads();
            }
        }
        // denominator: from the ones row (kept by the lanes of one half) or the two halves' partial sums
        float l_tot;
        if (ones_row && VTR) {
            // O^T row 31 of the last row tile: register 4 * (31 >> 3) + (31 & 3) = 15 of the lanes of half (31 >> 2) & 1 = 1
            const float mine = o[DT - 1][15];
            const float other = __shfl_xor(mine, 32, 64);
            l_tot = half == 1 ? mine : other;
        } else if (ones_row) {
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
        // The wave's 32 x d output tile goes through its own LDS slice so that global memory is written
        // in 16-byte pieces of whole rows (a lane holds 4 consecutive d of one query: stored directly,
        // every instruction would touch 32 different rows).  LDS operations of a wave complete in order,
        // so the reads below see the writes without a barrier.
        {
            const float inv = 1.f / l_tot;
#pragma unroll
            for (int tt = 0; tt < DT; ++tt)
#pragma unroll
                for (int g4 = 0; g4 < 4; ++g4) {
                    const int dd = tt * 32 + 8 * g4 + 4 * half;
                    const bf16x4 w = { (bf16_t)(o[tt][4 * g4] * inv), (bf16_t)(o[tt][4 * g4 + 1] * inv),
                                       (bf16_t)(o[tt][4 * g4 + 2] * inv), (bf16_t)(o[tt][4 * g4 + 3] * inv) };
                    *reinterpret_cast<bf16x4*>(sOut + l32 * LDO + dd) = w;
                }
            const int q0 = cur.q - l32;                                   // first query of the wave's tile
            bf16_t* op = (bf16_t*)a.out + ((size_t)cur.slot * a.Nq + q0) * a.ldo + cur.h * d;
            for (int id = lane; id < 32 * dch; id += 64) {
                const int r = id / dch, c = id % dch;
                if (q0 + r < a.Nq)
                    *reinterpret_cast<bf16x8*>(op + (size_t)r * a.ldo + c * 8) = *reinterpret_cast<const bf16x8*>(sOut + r * LDO + c * 8);
            }
        }
        if (!has_next) break;
        vpos = vnxt;
        item = nxt;
        cur = np;
    }
}

// fp32: kLanesPerQuery lanes share a query and split the kv rows between them (lane t takes rows
// t, t + kLanesPerQuery, ...), each with its own online-softmax state; the states are merged with
// cross-lane exchanges at the end.  The head width is a template bound so that the per-lane query and
// output vectors stay in registers.
constexpr int kF32MaxD = 128, kLanesPerQuery = 8, kF32Threads = 256;
template <int DMAX>
__global__ void __launch_bounds__(kF32Threads) attn_f32_kernel(const AttnArgs a, float scale)
{
    const int h = blockIdx.y, d = a.d;
    const int sub = threadIdx.x % kLanesPerQuery;
    const int q = blockIdx.x * (kF32Threads / kLanesPerQuery) + threadIdx.x / kLanesPerQuery;
    const bool live = q < a.Nq;
    const int qc = live ? q : a.Nq - 1;             // lanes past the end keep their group's exchanges in step
    for (int slot = blockIdx.z; slot < a.slots; slot += gridDim.z) {
        const int kvb = a.kv_mod ? slot % a.kv_mod : slot;
        const float* Q = (const float*)a.q + slot * a.q_slot_stride + h * a.q_head_stride + (size_t)qc * a.ldq;
        const float* Kp = (const float*)a.k + kvb * a.kv_batch_stride + h * a.kv_head_stride;
        const float* Vp = (const float*)a.v + kvb * a.kv_batch_stride + h * a.kv_head_stride;
        float qv[DMAX], o[DMAX];
#pragma unroll
        for (int e = 0; e < DMAX; ++e) { qv[e] = e < d ? Q[e] * scale : 0.f; o[e] = 0.f; }
        float m_run = -INFINITY, l_run = 0.f;
        for (int j = sub; j < a.Nk; j += kLanesPerQuery) {
            const float* kr = Kp + (size_t)j * a.ldk;
            float s = 0.f;
#pragma unroll
            for (int e = 0; e < DMAX; ++e)
                if (e < d) s = fmaf(qv[e], kr[e], s);
            const float m_new = fmaxf(m_run, s);
            const float alpha = expf(m_run - m_new), p = expf(s - m_new);
            l_run = l_run * alpha + p;
            m_run = m_new;
            const float* vr = Vp + (size_t)j * a.ldk;
#pragma unroll
            for (int e = 0; e < DMAX; ++e)
                if (e < d) o[e] = fmaf(o[e], alpha, p * vr[e]);
        }
        // merge the kLanesPerQuery partial states (a lane that saw no row has m = -inf, l = 0)
#pragma unroll
        for (int off = 1; off < kLanesPerQuery; off <<= 1) {
            const float m_o = __shfl_xor(m_run, off, 64), l_o = __shfl_xor(l_run, off, 64);
            const float m_new = fmaxf(m_run, m_o);
            const float ca = m_run == -INFINITY ? 0.f : expf(m_run - m_new), cb = m_o == -INFINITY ? 0.f : expf(m_o - m_new);
            l_run = l_run * ca + l_o * cb;
#pragma unroll
            for (int e = 0; e < DMAX; ++e) {
                const float o_o = __shfl_xor(o[e], off, 64);
                o[e] = o[e] * ca + o_o * cb;
            }
            m_run = m_new;
        }
        if (live) {
            float* op = (float*)a.out + ((size_t)slot * a.Nq + q) * a.ldo + h * d;
            const float inv = 1.f / l_run;
#pragma unroll
            for (int e = 0; e < DMAX; ++e)
                if (e < d && e % kLanesPerQuery == sub) op[e] = o[e] * inv;
        }
    }
}

template <int KS, int DT, int NW, int KC, int NB, bool PERSIST = false, bool VTR = false>
drf_status launch_bf16_cfg(const AttnArgs& a, float scale_log2, hipStream_t st)
{
    constexpr int LDKS = KS * 16 + 8, LDV = VTR ? DT * 32 + 16 : KC + 8;
    constexpr size_t smem = ((size_t)NB * (KC * LDKS + (VTR ? KC : DT * 32) * LDV) + (size_t)NW * 32 * (DT * 32 + 8)) * sizeof(bf16_t);
    static_assert(smem <= 160 * 1024 && smem % 16 == 0, "LDS budget");
    auto kern = attn_bf16_kernel<KS, DT, NW, KC, NB, PERSIST, VTR>;
    static bool attr_set = false;
    if (!attr_set) {
        DRF_HIP(hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem));
        attr_set = true;
    }
    const int nqb = (a.Nq + NW * 32 - 1) / (NW * 32);
    const long long n_items = (long long)nqb * a.heads * a.slots;
    if (n_items > 0x7fffffffLL) DRF_FAIL(DRF_ESHAPE, "attention: too many (query block, head, slot) items");
    // persistent: one workgroup per CU-sized share (a workgroup of 8 waves fills a CU)
    const int grid = PERSIST && n_items > kPersistGroups ? kPersistGroups : (int)n_items;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), smem, st, a, scale_log2, nqb, (int)n_items);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

template <int KS, int DT>
drf_status launch_bf16_inst(const AttnArgs& a, float scale_log2, hipStream_t st)
{
    // 8 waves (256 queries) share each staged chunk when there are that many queries.  Up to 256 kv rows
    // go through two buffers of 64 rows (the first MFMAs start after a quarter of the loads and every
    // later chunk is fetched during the steps of the one before; measured the fastest of the 64 / 128 /
    // 256-row, one / two-buffer combinations), longer sequences through two buffers of 128 rows.
    if (a.Nq > 128) {
        if (a.Nk <= 256) {
            // more items than workgroups that fit the chip at once: persistent workgroups hide each next
            // item's first loads; otherwise the plain kernel (fewer registers) is the faster one
            const long long n_items = (long long)((a.Nq + 255) / 256) * a.heads * a.slots;
            if (n_items > kPersistGroups) return launch_bf16_cfg<KS, DT, 8, 64, 2, true, true>(a, scale_log2, st);
            return launch_bf16_cfg<KS, DT, 8, 64, 2, false, true>(a, scale_log2, st);
        }
        return launch_bf16_cfg<KS, DT, 8, 128, 2>(a, scale_log2, st);
    }
    if (a.Nk <= 256) return launch_bf16_cfg<KS, DT, 4, 256, 1>(a, scale_log2, st);
    return launch_bf16_cfg<KS, DT, 4, 128, 2>(a, scale_log2, st);
}

}  // namespace

drf_status launch_attn_bf16(const AttnArgs& a, hipStream_t st)
{
    if (a.slots == 0 || a.Nq == 0) return DRF_OK;
    if (a.Nk < 1 || a.d % 8 != 0 || a.d > 96 || a.ldq % 8 != 0 || a.ldk % 8 != 0 || a.ldo % 8 != 0 ||
        (reinterpret_cast<uintptr_t>(a.out) & 15u) != 0)
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
    constexpr int qpb = kF32Threads / kLanesPerQuery;
    // slots beyond the grid's z limit are covered by a stride loop inside the kernel
    const dim3 grid((a.Nq + qpb - 1) / qpb, a.heads, a.slots < 65535 ? a.slots : 65535);
    const float scale = 1.f / sqrtf((float)a.d);
    if (a.d <= 32) hipLaunchKernelGGL(attn_f32_kernel<32>, grid, dim3(kF32Threads), 0, st, a, scale);
    else if (a.d <= 64) hipLaunchKernelGGL(attn_f32_kernel<64>, grid, dim3(kF32Threads), 0, st, a, scale);
    else hipLaunchKernelGGL(attn_f32_kernel<128>, grid, dim3(kF32Threads), 0, st, a, scale);
    DRF_HIP(hipGetLastError());
    return DRF_OK;
}

}  // namespace drf
