// Internal declarations shared by the translation units of libflashsink.
// Nothing here is part of the C ABI (see include/flashsink.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <string>
#include <vector>

#include "flashsink.h"

namespace fs {

// ---------------------------------------------------------------------------------------
// constants
// ---------------------------------------------------------------------------------------
constexpr double kLog2e = 1.4426950408889634074;   // log2(e)
constexpr double kLn2 = 0.69314718055994530942;    // ln(2)
constexpr float kNegInit = -3.0e38f;               // finite "-inf" seed of the running max
constexpr int kLowdMaxD = 16;                      // d <= 16: fp32 vector-ALU path
// Most column splits of one streaming pass over `n_res` resident rows: as many as fill the chip
// even for a handful of rows (n << m), as long as the [splits][rows] partial records stay at 64 MB.
// (`budget`: bytes the records may take; the context's Ctx::partial_budget)
inline int max_splits(size_t budget, int64_t n_res)
{
    const int64_t pad = (n_res + 1023) / 1024 * 1024;
    const int64_t s = (int64_t)budget / (pad * 16);
    return s < 1 ? 1 : (s > 1024 ? 1024 : (int)s);
}

// fp32-accurate scores on the bf16 matrix cores (low-d path).  A float v is the sum of three bf16
// pieces v1 + v2 + v3 (each the bf16 rounding of what the previous ones leave).  A product c x_k y_k
// is then the sum of the eight piece products of relative size >= 2^-24,
//     x1 y1, x1 y2, x2 y1, x1 y3, x2 y2, x3 y1, x2 y3, x3 y2,
// so a point is stored as one 16-byte "piece" of eight bf16 per coordinate:
//     streamed role, coordinate k:  y1 y2 y1 y3 y2 y1 y3 y2      resident role:  x1 x1 x2 x1 x2 x3 x2 x3
//     piece d (streamed):           b1 b2 b3  1  1  1  0  0      (resident):      1  1  1 m1 m2 m3  0  0
// with b = the point's bias and m = minus the resident row's running max (an integer, exact in
// three pieces).  One row of MFMA 32x32x16 steps over 16 ks = 8 (d + 1) padded slots then yields
// score - max directly, with fp32 accumulation; measured error equals that of an fp32 FMA chain.
// Direct global -> LDS loads (no registers in between): lane l's 16 (4) bytes land at
// lds_off + 16 l (4 l); lds_off must be wave-uniform.  Issued as inline assembly so that the
// compiler does not serialise them against the LDS reads of OTHER ring slots; completion is
// tracked by hand with s_waitcnt vmcnt (VMEM operations retire in order).
__device__ inline void dma16(const void *g, unsigned lds_off)
{
    unsigned m = __builtin_amdgcn_readfirstlane(lds_off);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" ::"v"(g), "s"(m) : "memory", "m0");
}
__device__ inline void dma4(const void *g, unsigned lds_off)
{
    unsigned m = __builtin_amdgcn_readfirstlane(lds_off);
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %0, off" ::"v"(g), "s"(m) : "memory", "m0");
}

// The same with a wave-uniform base address (it stays in scalar registers, and so does all the
// arithmetic that leads to it) and a per-lane byte offset.
__device__ inline void dma16s(const void *g_uniform, unsigned lane_off, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(g_uniform), "s"(lds_off)
                 : "memory", "m0");
}
__device__ inline void dma4s(const void *g_uniform, unsigned lane_off, unsigned lds_off)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dword %0, %1" ::"v"(lane_off), "s"(g_uniform), "s"(lds_off)
                 : "memory", "m0");
}

inline int split_ksteps(int64_t d) { return (int)(8 * d + 6 + 15) / 16; }   // 1..9 for d = 1..16
// Position (in 16-byte units) of piece `piece` inside the record of point `point`: 64-byte records
// (ks = 2) are rotated so that sixteen consecutive lanes read sixteen different 16-byte bank groups
// of a 256-byte line when 32 consecutive records are read at one piece; HBM holds the records already rotated,
// so tiles are copied to LDS linearly.
__host__ __device__ inline int split_piece_pos(int ks, int64_t point, int piece)
{
    return ks == 2 ? (piece ^ (int)((point >> 2) & 3)) : piece;
}
__device__ inline void split3(float v, __bf16 (&p)[3])
{
    p[0] = (__bf16)v;
    const bool fin = fabsf(v) < INFINITY;   // an infinite bias (padding) stays in the first piece
    float r = fin ? v - (float)p[0] : 0.0f;
    p[1] = (__bf16)r;
    r -= (float)p[1];
    p[2] = (__bf16)r;
}
__device__ inline void split3d(double v, __bf16 (&p)[3])   // three bf16 pieces of a finite double
{
    p[0] = (__bf16)(float)v;
    double r = v - (double)(float)p[0];
    p[1] = (__bf16)(float)r;
    r -= (double)(float)p[1];
    p[2] = (__bf16)(float)r;
}
// Grids of the leading digits of the "precise" split records (d <= 3, see k_lse_lowd_split):
// gy = 2^(Ey-7) with 2^Ey > max |y_k| (from rho_max, the largest squared norm after centring) and
// gx = 2^(Ex-7) with 2^Ex > (2 log2e/eps) max |x_k|; leading digits are multiples of the grid with
// at most 8 significant bits.
__host__ __device__ inline void split_grids(double rho_max, double eps, double *gx, double *gy)
{
    const double r = sqrt(rho_max > 1e-60 ? rho_max : 1e-60);
    *gy = exp2(floor(log2(r)) + 1.0 - 7.0);
    *gx = exp2(floor(log2(r * 2.0 * kLog2e / eps)) + 1.0 - 7.0);
}
__device__ inline uint32_t bf16_pair(__bf16 lo, __bf16 hi)
{
    return (uint32_t)__builtin_bit_cast(uint16_t, lo) | ((uint32_t)__builtin_bit_cast(uint16_t, hi) << 16);
}

enum class Path { LowD, F64, BF16 };

// ---------------------------------------------------------------------------------------
// context
// ---------------------------------------------------------------------------------------
struct Ctx {
    int device = 0;
    hipStream_t stream = nullptr;
    int num_cu = 256;
    // grow-only device workspace
    char *ws = nullptr;
    size_t ws_bytes = 0;
    bool ws_static = false;          // ws is the library's static scratch array for the duration of a call: never freed or grown
    char *static_ws = nullptr;       // this device's address of the static scratch array (resolved in fs_create)
    size_t partial_budget = size_t(64) << 20;   // bytes the [splits][rows] partial records of a pass may take
    // grow-only second buffer for entry points that call other entry points (which lay the workspace out anew)
    char *aux = nullptr;
    size_t aux_bytes = 0;
    std::string err;
    // Derived copies kept across entry calls (fs_points_keep): what identifies the clouds the caller has declared
    // unchanged, whether the workspace currently holds their derived copies, and the host-side value that belongs
    // to them (largest squared norm after centring, low-d path)
    struct PointsKey {
        const void *x = nullptr, *y = nullptr;
        int dtype = 0, compute = 0;
        int64_t n = 0, m = 0, d = 0, ldx = 0, ldy = 0;
        const char *ws = nullptr;      // the workspace the copies live in
        size_t partial_budget = 0;     // (the offsets of the device scalars depend on it)
        bool same(const PointsKey &o) const
        {
            return x == o.x && y == o.y && dtype == o.dtype && compute == o.compute && n == o.n && m == o.m && d == o.d &&
                   ldx == o.ldx && ldy == o.ldy && ws == o.ws && partial_budget == o.partial_budget;
        }
    };
    bool keep_on = false;
    PointsKey keep_key;                // declared by the caller (ws and partial_budget unset)
    bool kept_valid = false;
    PointsKey kept_key;
    double kept_rho_max = -1.0;
    // test and experiment switches of this context (fs_debug_set); 0 = the library decides
    int dbg_lowd_splits = 0;         // forced split count of the streamed side of a low-d pass
    int dbg_lowd_score = 0;          // 32: fp32 scores, 64: float64 scores in every low-d half-step
    int dbg_lowd_precise_valu = 0;   // 1: float64 scores at d <= 3 on the vector ALU instead of the precise records
    int dbg_lowd_any_bias = 0;       // 1: the precise records also for biases beyond their digit range (tests of that case)
    // profiling of the streaming LSE launches
    bool prof_on = false;
    std::vector<hipEvent_t> ev_pool;   // pairs (start, stop)
    size_t ev_used = 0;
    std::vector<int> ev_kind;          // per recorded launch: which kernel it was (0 = the path's main
                                       // kernel, 1 = the low-d float64-score kernel)
    std::vector<double> ev_pairs;      // per recorded launch: pair evaluations
};

fs_status fail(Ctx *c, fs_status s, const char *fmt, ...);

#define FS_HIP(ctx, expr)                                                                     \
    do {                                                                                      \
        hipError_t e__ = (expr);                                                              \
        if (e__ != hipSuccess)                                                                \
            return fs::fail((ctx), FS_ERR_DEVICE, "%s failed: %s", #expr, hipGetErrorString(e__)); \
    } while (0)

// Linear sub-allocator over the workspace (256-byte aligned pieces).
struct Arena {
    size_t off = 0;
    size_t take(size_t bytes)
    {
        size_t o = off;
        off += (bytes + 255) & ~size_t(255);
        return o;
    }
};

inline int64_t round_up(int64_t v, int64_t q) { return (v + q - 1) / q * q; }
inline int64_t ceil_div(int64_t v, int64_t q) { return (v + q - 1) / q; }

// ---------------------------------------------------------------------------------------
// One side (x or y) of a prepared problem: the derived copy the kernels read, its squared
// norms, the shifted potential and the bias it contributes when it is the streamed side.
// ---------------------------------------------------------------------------------------
struct Side {
    int64_t cnt = 0;       // real points
    int64_t cnt_pad = 0;   // rows of the derived copy (padding rows: zero coordinates, bias -inf)
    const float *w = nullptr;   // weights (device) or nullptr = uniform
    double log_uniform = 0.0;   // log(1/cnt)
    // LowD: packed [cnt_pad][dp] floats, dp = round_up(d+1, 4), and [cnt_pad][dpd] doubles,
    // dpd = round_up(d+1, 2); slot d of each point holds its bias
    float *packed = nullptr;
    double *packed_d = nullptr;
    double *norm_f = nullptr;  // [cnt_pad] squared norms of the float-rounded centred points
    // LowD: the packed floats again as [cnt_pad][16 ks] bf16 "split" records for the
    // matrix cores (layout: see split_ksteps)
    uint16_t *split = nullptr;
    // LowD, d <= 3: "precise" split records [cnt_pad][48] bf16 built from the float64 copy
    uint16_t *split_p = nullptr;
    // F64: double [cnt_pad][kp], kp = round_up(d, 32) (zero filled), bias in bias_d[cnt_pad].
    // LowD with d > 3 keeps the same two arrays (centred coordinates, kp = 32) for its float64-score
    // passes, which run on the fp64 matrix-core kernels.
    double *pts_d = nullptr;
    double *bias_d = nullptr;
    // BF16: uint16 [cnt_pad][kp], kp = round_up(d, 32), bias in bias_f[cnt_pad]
    uint16_t *pts_b = nullptr;
    float *bias_f = nullptr;
    double *norm = nullptr;   // [cnt_pad] squared norms of the derived points
    double *pot = nullptr;    // [cnt_pad] UNSHIFTED potential (f or g) in float64
};

struct Prepared {
    Path path = Path::LowD;
    int64_t d = 0;
    int dp = 0;   // LowD: floats per packed point
    int dpd = 0;  // LowD: doubles per packed point (float64 score mode)
    int ks = 0;   // LowD: 16-wide contraction steps of a split record
    double rho_max = 0.0;   // LowD: largest squared norm of a centred point (host copy)
    // LowD: size of the biases that the caller's potentials give, in base-2 units:
    //   |bias| <= pot_mag_eps / eps + logw_mag   (potential part, scaling like 1/eps, and log-weight part)
    double pot_mag_eps = 0.0, logw_mag = 0.0;
    int halfsteps_per_eps = 2;    // LowD: half-steps the caller runs at one eps (error budget)
    bool force_precise = false;   // LowD: float64 scores regardless (marginal error evaluation)
    int dbg_score = 0;            // LowD: the context's score switch (see Ctx::dbg_lowd_score)
    bool dbg_precise_valu = false;   // LowD: the context's kernel switch (see Ctx::dbg_lowd_precise_valu)
    bool dbg_any_bias = false;       // LowD: see Ctx::dbg_lowd_any_bias
    int kp = 0;   // F64 / BF16: padded contraction length
    Side X, Y;
    // partial reductions of a streaming pass: [splits][max(n,m)_pad] records
    void *partial = nullptr;
    size_t partial_bytes = 0;
    double *dev_part = nullptr;  // [ceil(max(n,m)/256)] per-block sums of the marginal deviation
    double *gauge_part = nullptr;   // [2][ceil(max(n,m)/256)] per-block sums of the plan's mass seen by a g-update
    double *gauge_part_x = nullptr; // the same for an f-update (averaged schedule: both passes measure, halves by parity)
    double *scalars = nullptr;   // [16] device doubles (marginal errors, centring sums...; [8], [9]: gauge drift, see GaugeMode)
    double *mean = nullptr;      // [kLowdMaxD] common mean (LowD)
    char *extra = nullptr;       // entry-point specific scratch (plan application partials)
    size_t extra_bytes = 0;
};

// ---------------------------------------------------------------------------------------
// kernel launchers (implemented in the path-specific translation units)
// ---------------------------------------------------------------------------------------

// Launch-shape decision of one streaming pass.
struct PassShape {
    int rows_per_block = 0;
    int row_blocks = 0;
    int splits = 1;
    int64_t cols_per_split = 0;   // multiple of the column tile
};

// fs_prep.hip
fs_status launch_prepare(Ctx *c, const fs_problem *p, Prepared *P);
// `first` / `last`: an entry point that brings in both potentials passes (true, false) and then
// (false, true); the low-d read-back of the sizes that choose the score arithmetic (largest squared
// norm, size of the biases) happens once, in the call with last = true.
fs_status launch_bias_from_user(Ctx *c, Prepared *P, Side *side, const float *pot_user, double eps, bool first = true,
                                bool last = true);
// `res_norm` is the norm array matching the coordinates the pass used (Side::norm or norm_f).
// `mix`: the new potential is (1 - mix) * old + mix * update (1: plain update, 1/2: averaged schedule).
// `abs_dev_sum` != nullptr measures the marginal deviation instead of storing the update; with
// `save_old` it does both and leaves the replaced potential in save_old[0..cnt).
// Drift of the alternating iteration along its neutral direction (f + t, g - t), and how it is taken out.
// The exact iterates keep the plan's total mass at 1: after "f from g" the row marginals are exact.  A g-update
// measures that mass on its way (Prop. 3: c_j = b_j exp((g_j - g_j^+)/eps) are the column sums of the plan that
// (f, g) induce).  When the f-pass and the g-pass carry different systematic rounding biases u_f, u_g (the matrix
// cores truncate when they align the products of a score), the computed mass is exp((u_f - u_g)/eps), and the
// difference is exactly what one iteration adds to t: a random error would be damped, this one accumulates linearly
// (measured on the annealed low-dimension workload: 8e-5 eps at n = 16384, 2.5e-4 eps at n = 32768 after 200
// iterations, with a scatter around that constant of 8e-6).  So a solve adds up eps ln(mass) over its g-updates
// (scalars[8]; scalars[9] keeps the sum without the last term) and hands f - scalars[9], g + scalars[8] to the caller.
//   Measure: this merge is a g-update of an alternating solve: leave the block sums of c_j in gauge_part
//   Collect: this merge is the f-update after one: its first workgroup adds eps_prev ln(sum gauge_part) to scalars[8]
enum class GaugeMode { None, Measure, Collect };
fs_status launch_finalize(Ctx *c, const Prepared *P, Side *res, const double *res_norm, int splits,
                          double eps_cur, double eps_next_bias, float *user_out, double *abs_dev_sum,
                          double mix = 1.0, double *save_old = nullptr, GaugeMode gauge = GaugeMode::None,
                          int64_t gauge_prev_cnt = 0, double gauge_prev_eps = 0.0);
// the last g-update's term, then f_user = (float)(X.pot - scalars[9]) and g_user = (float)(Y.pot + scalars[8])
// (x_pot: the f to hand out, X.pot or a saved copy of it)
fs_status launch_gauge_export(Ctx *c, const Prepared *P, bool collect_last, double eps_last, const double *x_pot,
                              float *f_user, float *g_user);
// `gauge`: the averaged schedule's form of the drift removal (see GaugeMode): both passes of an iteration read the
// same old potentials, so the plan's mass as the f-pass sees it (row sums) and as the g-pass sees it (column sums)
// differ by exp((u_f - u_g)/eps) exactly, and an averaged iteration moves t by a quarter of u_f - u_g.  With
// gauge_parity >= 0 (the iteration number) both merges leave their block sums in half `gauge_parity & 1` of
// gauge_part_x / gauge_part, and, `collect_prev`, the first workgroup adds the previous iteration's term
// eps (ln mass_g - ln mass_f) / 4 to scalars[8] and [9] from the other half; the caller hands out f - scalars[9],
// g + scalars[8] (launch_gauge_collect_pair for the last iteration, then launch_gauge_export with collect_last = false).
fs_status launch_finalize_pair(Ctx *c, const Prepared *P, Side *X, const double *norm_x, const void *partial_x, int splits_x,
                               float *f_out, Side *Y, const double *norm_y, const void *partial_y, int splits_y,
                               float *g_out, double eps_cur, double eps_next_bias, double mix, int gauge_parity = -1,
                               bool collect_prev = false);
fs_status launch_gauge_collect_pair(Ctx *c, const Prepared *P, double eps, int gauge_parity);
fs_status launch_export_f32(Ctx *c, const double *src, int64_t cnt, float *dst);
// label-augmented cost: augmented copy [rows][d + V] of one cloud (see k_label_augment) and the map between the
// potentials of the labelled and of the augmented problem
fs_status launch_label_augment(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld,
                               const int32_t *labels, const float *W, int V, bool target_side, double l1, double l2,
                               bool round_bf16, float *out, float *vconst, unsigned *bad);
fs_status launch_label_potential(Ctx *c, const float *src, const float *vconst, double cshift, double l1, bool to_augmented,
                                 int64_t cnt, float *dst);
fs_status launch_pts_to_f32(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, float *dst);
fs_status launch_grad_assemble(Ctx *c, float *g, int64_t ldg, const void *pts, int dtype, int64_t ld, int64_t rows,
                               int64_t d, const float *w, const float *mass, int mode);
fs_status launch_value_terms(Ctx *c, const Prepared *P, const Side *res, const double *res_norm, const Side *str,
                             int splits, double eps, double *scratch, double *dst);
fs_status launch_row_norms(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld,
                           float *out);
fs_status launch_fill_f64(Ctx *c, double *dst, double v, int64_t cnt);
fs_status launch_weight_stats(Ctx *c, const float *w, int64_t cnt, double *scratch, double *dst);
fs_status launch_count_nonfinite(Ctx *c, const float *v, int64_t cnt, double *scratch, double *dst);
// merge the splits of an application pass (partial (max,sum) + opart[split][row][PC]) and apply
// the epilogue  out_i = w_i exp(pot_shifted_i/eps + m_i) O_i  for columns p0 .. p0+PC-1
fs_status launch_apply_finalize(Ctx *c, const Prepared *P, const Side *res, const double *res_norm, int splits,
                                double eps, const float *opart, int PC, int p0, int p, float *out, int64_t ldo,
                                float *mass_out);

// fs_hvp.hip
size_t hvp_scratch_bytes(int64_t n, int64_t m, int64_t d);
fs_status hvp_run(Ctx *c, Prepared *P, const float *x, int64_t ldx, const float *y, int64_t ldy, double eps,
                  const float *A, int64_t lda, double tau, double eta, int max_cg, float *out, int64_t ldo,
                  char *scratch, int *cg_iters);

// out (n x p, ldo) += <A_i, mean> PV_i (PV: n x p, dense): the mean's share of the Hadamard weights
fs_status launch_add_mean_share(Ctx *c, const float *A, int64_t lda, const double *mean, const float *PV, int64_t n, int d,
                                int p, float *out, int64_t ldo);

// fs_lowd.hip
PassShape lowd_shape(const Ctx *c, int64_t n_res, int64_t n_str);
// true: this half-step runs the low-d pass with float64 scores (norm), false: float (norm_f)
bool lowd_precise(const Prepared *P, double eps);
fs_status lowd_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps,
                   int *splits_out);
// both half-steps of an averaged iteration (Eq. 4-5) in one launch; *done = false: not applicable
fs_status lowd_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x,
                        int *splits_y, bool *done);
size_t lowd_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t d, int64_t p);
// had_A != nullptr: Hadamard-weighted transport (Alg. 5), every plan entry times <had_A row i, centred
// streamed point j>; had_A is [res->cnt][lda] floats.
fs_status lowd_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps,
                     const float *V, int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out,
                     const float *had_A = nullptr, int64_t lda = 0);

// fs_f64.hip
// (prof_kind: how the launch is booked by the profiling hooks, see Ctx::ev_kind)
fs_status f64_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps,
                  int *splits_out, int prof_kind = 0);
fs_status f64_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x,
                       int *splits_y);
size_t f64_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t d, int64_t p);
fs_status f64_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps,
                    const float *V, int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out,
                    const float *hadA = nullptr, int64_t lda = 0);

// fs_bf16.hip
fs_status bf16_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps,
                   int *splits_out);
fs_status bf16_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x,
                        int *splits_y);
// plan application in bf16 mode (Alg. 2 / Alg. 4): workspace bytes and the pass itself
size_t bf16_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str);
fs_status bf16_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V, int64_t p,
                     int64_t ldv, float *out, int64_t ldo, float *mass_out);

// profiling helpers (fs_api.hip)
void prof_begin(Ctx *c, double pairs, int kind = 0);
void prof_end(Ctx *c);

}  // namespace fs
