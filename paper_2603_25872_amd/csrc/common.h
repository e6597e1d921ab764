// Internal declarations shared by the translation units of libdrf.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>
#include <string>
#include <vector>

#include "../../include/drf.h"

namespace drf {

// ---- errors -----------------------------------------------------------------
void set_error(const char* fmt, ...);
#define DRF_FAIL(code, ...) do { ::drf::set_error(__VA_ARGS__); return (code); } while (0)
#define DRF_HIP(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { \
    ::drf::set_error("%s failed: %s (%s:%d)", #expr, hipGetErrorString(e_), __FILE__, __LINE__); \
    return DRF_EHIP; } } while (0)

// ---- schedule / plan (host) ---------------------------------------------------
struct Schedule {
    std::vector<double> abar;   // cumulative alpha per training timestep
    int steps = 0, stride = 0, train_steps = 0;
    drf_sampler sampler = DRF_DDIM;
    double eta = 0.0, shift = 1.0;
    int tau(int s) const { return (s - 1) * stride; }
    double abar_at(int s) const { return s == 0 ? 1.0 : abar[(size_t)tau(s)]; }
    // Euler: ODE time of sampling index s
    double sigma_at(int s) const;
    // integer time fed to the network at sampling index s >= 1
    int net_time(int s) const;
    // true when some transition of this sampler adds fresh noise
    bool stochastic() const { return sampler == DRF_DDPM || (sampler == DRF_DDIM && eta != 0.0); }
    // x_to = A x_from + B net + C z.  Fails for a transition with variance that is not a move towards data.
    drf_status coef(int s_from, int s_to, float* A, float* B, float* C) const;
};
drf_status make_schedule(const drf_sched_config* sc, Schedule* out);

// One batched predictor pass of drf_sample and the elementwise update after it.
struct Pass {
    int round = 0;
    bool solo = false;              // stand-alone evaluation of the anchor state
    int s_anchor = 0;               // anchor index the evaluated states were drafted from
    std::vector<int> eval_s;        // sampling indices evaluated, one per slot group
    bool base_is_draft = false;     // chain starts from the first draft, else from the anchor state
    std::vector<std::pair<int, int>> chain;   // standard updates (s_from -> s_to); update i uses noise field i
    std::vector<int> chain_z;       // per update: ordinal of its fresh-noise field among the call's draws
    int anchor_field = -1;          // noise field that pairs with the state after the chain (-1: none)
    std::vector<int> draft_to;      // skip targets drafted from (state after chain, anchor noise)
    std::vector<int> draft_z;       // per draft: ordinal of its fresh-noise field
    int s_after = 0;                // index of the state after the chain
    bool writes_x0 = false;         // the state after the chain (or the lone draft to 0) is x_0
};
// rows: plan table in the documented row format (may be NULL).  n_noise (may be NULL): number of
// fresh-noise fields the call draws (kind-1 plus kind-2 rows).
drf_status build_plan(const Schedule& sch, drf_mode mode, int n, std::vector<Pass>* passes,
                      std::vector<int32_t>* rows, size_t* n_noise = nullptr);

// ---- elementwise update kernel --------------------------------------------------
constexpr int kMaxBlock = 64;       // largest block size n the update kernel's argument block holds
struct UpdateArgs {
    const float* x_base;   // [field]
    const float* eps;      // [n_fields][g][field]
    float* x_out;          // [field] or NULL: state after the chain
    float* draft_out;      // [n_draft][field] or NULL
    size_t field;          // batch * elems_per_sample
    int g;                 // 1, or 2 = (cond, null) pairs combined by guidance
    float w;               // guidance scale
    int n_chain, anchor_field, n_draft;
    float cA[kMaxBlock], cB[kMaxBlock], dA[kMaxBlock], dB[kMaxBlock];
    // fresh noise: y += cC[i] * z(field cz[i]) after chain update i, d_j += dC[j] * z(field dz[j]);
    // a zero coefficient means the field is not touched
    int noise_mode;        // 0 none | 1 explicit fields at z | 2 generated from (seed, z_field0 + ordinal)
    const float* z;        // [..][field]
    uint64_t seed;
    uint32_t z_field0;
    float cC[kMaxBlock], dC[kMaxBlock];
    int cz[kMaxBlock], dz[kMaxBlock];
};
enum { NOISE_NONE = 0, NOISE_EXPLICIT = 1, NOISE_PHILOX = 2 };
// Fills noise_mode / z / seed / z_field0 from the caller's source; fails when a nonzero cC / dC has no source.
drf_status set_noise_source(UpdateArgs* a, const drf_noise* noise);
drf_status launch_update(const UpdateArgs& a, hipStream_t st);

// ---- DiT kernels ------------------------------------------------------------------
typedef __bf16 bf16_t;

// How slot j of a pass finds its inputs.
struct SlotMap {
    const int32_t* t_dev;   // per-slot training timesteps, or NULL: use taus[j / group]
    int group;              // slots per draft group (g * batch)
    int taus[kMaxBlock];
    int x_group, x_batch;   // x row of slot j = (j / x_group) * x_batch + j % x_batch
    int cond_mod;           // cond row of slot j = cond_mod ? j % cond_mod : j
};

enum EpiMode { EPI_STORE = 0, EPI_STORE_GELU = 1, EPI_RESID = 2, EPI_STORE_HEADS = 3, EPI_STORE_GATED = 4 };
struct Epilogue {
    int mode;
    void* out;              // EPI_STORE*: [M][ldo] of out type; EPI_RESID: float [M][ldo], read-modify-write
    int ldo;
    int out_f32;            // EPI_STORE*: 1 = float output, 0 = bf16 output
    const float* bias;      // [N]
    const float* gate;      // EPI_RESID, EPI_STORE_GATED: gate[(m / rows_per_slot) * gate_ld + n]; EPI_RESID: NULL = ungated
                            // EPI_STORE_GATED (bf16 only): out = gate * (acc + bias), the branch output that the next
                            // LayerNorm launch adds to the residual stream
    int gate_ld, rows_per_slot;
    uint32_t rps_magic; int rps_shift;   // m / rows_per_slot == fast_div(m, rps_magic, rps_shift), see set_rows_per_slot
    // EPI_STORE_HEADS (bf16 only): column n = which * hid + head * hd + dd of row m = slot * rows_per_slot + t goes to
    //   out[which * plane + ((slot * heads + head) * rows_per_slot + t) * hd + dd]     (q | k | v planes, head-major)
    int hid, hd, heads; size_t plane;
    uint32_t hid_magic, hd_magic; int hid_shift, hd_shift;
    // Optional (bf16 wide-tile kernel only): the last 256 workgroups of the launch (the ones that run in
    // its final round) each load one word of their share of the warm_lines 128-byte lines at `warm`,
    // typically the weights of the GEMM that runs next, so that those are already on the near side of
    // HBM when that GEMM asks for them.  Values are not used.
    const void* warm; uint32_t warm_lines;
};
// Division constants for floor(n / d), 0 <= n < 2^31 (see fast_div in gemm.hip).
void make_fast_div(int d, uint32_t* magic, int* shift);
// Fills rows_per_slot and its division constants (exact for 0 <= m < 2^31).
void set_rows_per_slot(Epilogue* e, int rows_per_slot);
// C[M][N] = A[M][K] . W[N][K]^T, then the epilogue.  bf16: K % 64 == 0.
// variant 0: the tile shape is chosen from the problem size; > 0 forces one (measurement and tile tests).
// splitk_scratch: gemm_splitk_scratch_bytes() of device memory, or NULL; with it, problems of few tiles and a long
// K are split across workgroups (variant 10 forces the 128 x 128 tile, split when the rule allows).
drf_status launch_gemm_bf16(const bf16_t* A, const bf16_t* W, int M, int N, int K, const Epilogue& e, hipStream_t st,
                            int variant = 0, float* splitk_scratch = nullptr);
size_t gemm_splitk_scratch_bytes();
drf_status launch_gemm_f32(const float* A, const float* W, int M, int N, int K, const Epilogue& e, hipStream_t st);

struct AttnArgs {
    // query i of (slot, head h) starts at q + slot * q_slot_stride + h * q_head_stride + i * ldq  (elements);
    // key/value j at k|v + kv_batch * kv_batch_stride + h * kv_head_stride + j * ldk.
    // Packed rows [row][.. head h at column h*d ..]: slot stride N * ld, head stride d.
    // Head-major [slot][head][row][d]: slot stride heads * N * d, head stride N * d, ld = d.
    const void* q; int ldq; size_t q_slot_stride, q_head_stride;
    const void* k; const void* v; int ldk; size_t kv_batch_stride, kv_head_stride;
    void* out; int ldo;             // out row (slot * Nq + i), head h at column h * d
    int Nq, Nk, heads, d, slots;
    int kv_mod;                     // kv_batch = kv_mod ? slot % kv_mod : slot
};
drf_status launch_attn_bf16(const AttnArgs& a, hipStream_t st);
drf_status launch_attn_f32(const AttnArgs& a, hipStream_t st);

struct DitDims { int D, P, T, gh, gw, C, H, W, patch, heads, d, R, L; };

// c = MLP(femb(tau)) + cond embedding; writes SiLU(c) as float [slots][D] and, if act_bf16 != NULL, bf16.
struct CondArgs {
    const float *t_w1, *t_b1, *t_w2, *t_b2, *c_w, *c_b, *table;
    const void* cond; int cond_kind, cond_dim;
    int D, slots;
    SlotMap map;
    float* act_f32; bf16_t* act_bf16;
    float* scratch;          // slots * (256 + 3 D) floats
};
drf_status launch_cond_embed(const CondArgs& a, hipStream_t st);

drf_status launch_patch_embed(const float* x, const SlotMap& map, const float* w, const float* b, const float* pos,
                              const DitDims& dm, int slots, float* resid, hipStream_t st);
// out = LN(resid) * (1 + scale) + shift (shift == NULL: plain LN); mod rows are per slot.
// add != NULL (bf16 [M][D], and add2 likewise if also != NULL): the rows normalised are x = (resid + add) + add2;
// write_back stores x over resid, otherwise resid is left as it was and the caller passes the same `add`
// again (with the next branch output as add2) to the launch that does write back.
drf_status launch_ln_modulate(float* resid, const bf16_t* add, const bf16_t* add2, bool write_back, const float* shift,
                              const float* scale, int mod_ld, int rows_per_slot, int M, int D, void* out, int out_f32,
                              hipStream_t st);
drf_status launch_final(const float* resid, const float* shift, const float* scale, int mod_ld, const float* w,
                        const float* b, const DitDims& dm, int slots, float* eps_out, hipStream_t st);
drf_status launch_f32_to_bf16(const float* in, bf16_t* out, size_t n, hipStream_t st);

}  // namespace drf
