// Low-dimension (d <= 16) streaming passes on the vector ALU.
//
// With three coordinates there is no dense contraction to give to the matrix
// cores: a score costs d FMAs and the pass is bound by the exp2 rate.  Mapping:
// every lane owns R resident rows (their pre-scaled coordinates and the running
// (max, sum) live in registers, so the row reduction never crosses lanes); the
// streamed points are staged in LDS in tiles of 256, packed as
// (coord_0..coord_{d-1}, bias), so that one broadcast LDS read serves all 64 lanes
// of a wave and all R rows of a lane.
//
// Scores are in base 2:  s_ij = (2 log2e / eps) <x_i, y_j> + bias_j  (Alg. 1, line "score tile
// + bias", times log2 e), so exp and log are single v_exp_f32 / v_log_f32 instructions.
// The online LSE of Alg. 1 is applied per register chunk of T columns; the running max is
// kept integer-valued, so every rescale factor is an exact power of two.
//
// Score type S: float when (log2e/eps) * max|x|^2 is small enough for fp32 scores to hold the
// 1e-4 target, double otherwise (a score of magnitude 500 has an fp32 ulp of 6e-5).  In both
// cases the exponent s_ij - m is formed in S and only then rounded to float.
#include "fs_internal.h"

#include <stdlib.h>

namespace fs {
namespace {

constexpr int kBlock = 256;   // threads per workgroup
constexpr int kTJ = 256;      // streamed points per LDS tile
constexpr int kT = 8;         // columns per register chunk
constexpr float kLazyMax = 1.152921504606846976e18f;   // 2^60: largest chunk sum taken without rescaling

__device__ inline float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

template <typename S> struct Pack;   // how a point (d coords + bias) of type S is padded to 16-byte units
template <> struct Pack<float> {
    static constexpr int per16 = 4;
};
template <> struct Pack<double> {
    static constexpr int per16 = 2;
};

// 16-byte unit as stored in LDS / loaded from global
struct alignas(16) Unit {
    uint32_t w[4];
};

template <typename S, int DP> __device__ inline void unpack(const Unit *u, S (&v)[DP])
{
    constexpr int Q = DP / Pack<S>::per16;
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        Unit t = u[q];
        if constexpr (sizeof(S) == 4) {
            v[4 * q + 0] = __uint_as_float(t.w[0]);
            v[4 * q + 1] = __uint_as_float(t.w[1]);
            v[4 * q + 2] = __uint_as_float(t.w[2]);
            v[4 * q + 3] = __uint_as_float(t.w[3]);
        } else {
            v[2 * q + 0] = __hiloint2double((int)t.w[1], (int)t.w[0]);
            v[2 * q + 1] = __hiloint2double((int)t.w[3], (int)t.w[2]);
        }
    }
}

template <typename S, int D, int R, int T = kT>
__global__ __launch_bounds__(kBlock) void k_lse_lowd(const S *__restrict__ res, const S *__restrict__ str, S cscale,
                                                     int tiles_per_split, int n_tiles, double2 *__restrict__ partial,
                                                     int64_t partial_stride)
{
    constexpr int P16 = Pack<S>::per16;
    constexpr int DP = (D + 1 + P16 - 1) / P16 * P16;
    constexpr int Q = DP / P16;               // 16-byte units per packed point
    __shared__ Unit tile[2][kTJ * Q];

    const int tid = threadIdx.x;
    const int64_t row0 = (int64_t)blockIdx.x * (kBlock * R);

    S xs[R][D];
    // running max, running sum over finished tiles, and the sum inside the current tile: adding
    // tile totals instead of single terms keeps the fp32 summation error at the 1e-6 level
    float mrun[R], srun[R], stile[R];
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const S *px = res + (row0 + r * kBlock + tid) * DP;
#pragma unroll
        for (int k = 0; k < D; ++k) xs[r][k] = px[k] * cscale;
        mrun[r] = kNegInit;
        srun[r] = 0.0f;
        stile[r] = 0.0f;
    }

    const int t_begin = blockIdx.y * tiles_per_split;
    const int t_end = min(n_tiles, t_begin + tiles_per_split);
    const Unit *gsrc = reinterpret_cast<const Unit *>(str);

    Unit pre[Q];
    if (t_begin < t_end) {
#pragma unroll
        for (int q = 0; q < Q; ++q) pre[q] = gsrc[(int64_t)t_begin * (kTJ * Q) + q * kBlock + tid];
#pragma unroll
        for (int q = 0; q < Q; ++q) tile[0][q * kBlock + tid] = pre[q];
    }
    __syncthreads();

    int buf = 0;
    for (int t = t_begin; t < t_end; ++t) {
        const bool more = (t + 1 < t_end);
        if (more) {
#pragma unroll
            for (int q = 0; q < Q; ++q) pre[q] = gsrc[(int64_t)(t + 1) * (kTJ * Q) + q * kBlock + tid];
        }
        const Unit *tl = tile[buf];
#pragma unroll 1
        for (int j = 0; j < kTJ; j += T) {
            S sc[R][T];
#pragma unroll
            for (int c = 0; c < T; ++c) {
                S yv[DP];
                unpack<S, DP>(tl + (j + c) * Q, yv);
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    S acc = yv[D];   // bias
#pragma unroll
                    for (int k = 0; k < D; ++k) acc = xs[r][k] * yv[k] + acc;   // contracted to FMA
                    sc[r][c] = acc;
                }
            }
            // Lazy stabiliser: exponents are taken against the CURRENT (integer) running max, which
            // may be exceeded by up to 2^60 before anything is rescaled.  Only when a chunk sum
            // leaves that range (or the max is still the initial sentinel) does the wave take the
            // slow branch: lift the max to ceil(chunk max) and rescale by an exact power of two.
            float csum[R];
            bool bad = false;
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const S mS = (S)mrun[r];
                float acc = fast_exp2((float)(sc[r][0] - mS));
#pragma unroll
                for (int c = 1; c < T; ++c) acc += fast_exp2((float)(sc[r][c] - mS));
                csum[r] = acc;
                bad = bad || !(acc < kLazyMax);
            }
            if (__any(bad)) {
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    float mx = (float)sc[r][0];
#pragma unroll
                    for (int c = 1; c < T; ++c) mx = fmaxf(mx, (float)sc[r][c]);
                    float mnew = fmaxf(mrun[r], ceilf(mx));
                    float scale = fast_exp2(mrun[r] - mnew);
                    const S mS = (S)mnew;
                    float acc = fast_exp2((float)(sc[r][0] - mS));
#pragma unroll
                    for (int c = 1; c < T; ++c) acc += fast_exp2((float)(sc[r][c] - mS));
                    csum[r] = acc;
                    srun[r] *= scale;
                    stile[r] *= scale;
                    mrun[r] = mnew;
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r) stile[r] += csum[r];
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            srun[r] += stile[r];
            stile[r] = 0.0f;
        }
        if (more) {
#pragma unroll
            for (int q = 0; q < Q; ++q) tile[buf ^ 1][q * kBlock + tid] = pre[q];
        }
        __syncthreads();
        buf ^= 1;
    }

#pragma unroll
    for (int r = 0; r < R; ++r) {
        int64_t row = row0 + r * kBlock + tid;
        partial[(int64_t)blockIdx.y * partial_stride + row] = make_double2((double)mrun[r], (double)srun[r]);
    }
}

// ---- plan application (Alg. 2 / Alg. 4): the same pass with a value accumulator ----------
// Every lane owns ONE resident row and PC columns of the output; the streamed tile carries
// the PC values of each streamed point next to its coordinates.
template <typename S, int D, int PC>
__global__ __launch_bounds__(kBlock) void k_apply_lowd(const S *__restrict__ res, const S *__restrict__ str,
                                                       const float *__restrict__ V, int64_t ldv, int p0, int p,
                                                       int64_t n_str, S cscale, int tiles_per_split, int n_tiles,
                                                       double2 *__restrict__ partial, int64_t partial_stride,
                                                       float *__restrict__ opart, int64_t opart_stride)
{
    constexpr int P16 = Pack<S>::per16;
    constexpr int DP = (D + 1 + P16 - 1) / P16 * P16;
    constexpr int Q = DP / P16;
    __shared__ Unit tile[kTJ * Q];
    __shared__ float vt[kTJ][PC];

    const int tid = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * kBlock + tid;

    S xs[D];
    {
        const S *px = res + row * DP;
#pragma unroll
        for (int k = 0; k < D; ++k) xs[k] = px[k] * cscale;
    }
    float mrun = kNegInit, srun = 0.0f;
    float O[PC];
#pragma unroll
    for (int c = 0; c < PC; ++c) O[c] = 0.0f;

    const int t_begin = blockIdx.y * tiles_per_split;
    const int t_end = min(n_tiles, t_begin + tiles_per_split);
    const Unit *gsrc = reinterpret_cast<const Unit *>(str);

    for (int t = t_begin; t < t_end; ++t) {
        __syncthreads();
#pragma unroll
        for (int q = 0; q < Q; ++q) tile[q * kBlock + tid] = gsrc[(int64_t)t * (kTJ * Q) + q * kBlock + tid];
        {
            int64_t j = (int64_t)t * kTJ + tid;
#pragma unroll
            for (int c = 0; c < PC; ++c) vt[tid][c] = (j < n_str && p0 + c < p) ? V[j * ldv + p0 + c] : 0.0f;
        }
        __syncthreads();
#pragma unroll 1
        for (int j = 0; j < kTJ; j += kT) {
            S sc[kT];
#pragma unroll
            for (int c = 0; c < kT; ++c) {
                S yv[DP];
                unpack<S, DP>(tile + (j + c) * Q, yv);
                S acc = yv[D];
#pragma unroll
                for (int k = 0; k < D; ++k) acc = xs[k] * yv[k] + acc;
                sc[c] = acc;
            }
            float mx = (float)sc[0];
#pragma unroll
            for (int c = 1; c < kT; ++c) mx = fmaxf(mx, (float)sc[c]);
            float mnew = fmaxf(mrun, ceilf(mx));
            float scale = fast_exp2(mrun - mnew);
            srun *= scale;
#pragma unroll
            for (int c = 0; c < PC; ++c) O[c] *= scale;
            const S mS = (S)mnew;
#pragma unroll
            for (int c = 0; c < kT; ++c) {
                float e = fast_exp2((float)(sc[c] - mS));
                srun += e;
#pragma unroll
                for (int q = 0; q < PC; ++q) O[q] = fmaf(e, vt[j + c][q], O[q]);
            }
            mrun = mnew;
        }
    }
    partial[(int64_t)blockIdx.y * partial_stride + row] = make_double2((double)mrun, (double)srun);
#pragma unroll
    for (int c = 0; c < PC; ++c) opart[((int64_t)blockIdx.y * opart_stride + row) * PC + c] = O[c];
}

constexpr int kApplyPC = 4;   // output columns per application pass

template <typename S, int D>
void launch_lse_d(int R, dim3 grid, hipStream_t st, const S *res, const S *str, S cscale, int tps, int n_tiles,
                  double2 *partial, int64_t stride)
{
    if (R == 2)
        hipLaunchKernelGGL((k_lse_lowd<S, D, 2>), grid, dim3(kBlock), 0, st, res, str, cscale, tps, n_tiles, partial, stride);
    else
        hipLaunchKernelGGL((k_lse_lowd<S, D, 1>), grid, dim3(kBlock), 0, st, res, str, cscale, tps, n_tiles, partial, stride);
}

template <typename S, int D>
void launch_apply_d(dim3 grid, hipStream_t st, const S *res, const S *str, const float *V, int64_t ldv, int p0, int p,
                    int64_t n_str, S cscale, int tps, int n_tiles, double2 *partial, int64_t stride, float *opart)
{
    hipLaunchKernelGGL((k_apply_lowd<S, D, kApplyPC>), grid, dim3(kBlock), 0, st, res, str, V, ldv, p0, p, n_str, cscale,
                       tps, n_tiles, partial, stride, opart, stride);
}

#define FS_LOWD_DISPATCH(D_, CALL)                                                                       \
    switch (D_) {                                                                                        \
    case 1: { constexpr int DD = 1; CALL; } break;   case 2: { constexpr int DD = 2; CALL; } break;     \
    case 3: { constexpr int DD = 3; CALL; } break;   case 4: { constexpr int DD = 4; CALL; } break;     \
    case 5: { constexpr int DD = 5; CALL; } break;   case 6: { constexpr int DD = 6; CALL; } break;     \
    case 7: { constexpr int DD = 7; CALL; } break;   case 8: { constexpr int DD = 8; CALL; } break;     \
    case 9: { constexpr int DD = 9; CALL; } break;   case 10: { constexpr int DD = 10; CALL; } break;   \
    case 11: { constexpr int DD = 11; CALL; } break; case 12: { constexpr int DD = 12; CALL; } break;   \
    case 13: { constexpr int DD = 13; CALL; } break; case 14: { constexpr int DD = 14; CALL; } break;   \
    case 15: { constexpr int DD = 15; CALL; } break; default: { constexpr int DD = 16; CALL; } break;   \
    }

PassShape shape_for(const Ctx *c, int64_t n_res, int64_t n_str, int R)
{
    PassShape s;
    s.rows_per_block = kBlock * R;
    s.row_blocks = (int)ceil_div(n_res, s.rows_per_block);
    int n_tiles = (int)ceil_div(n_str, kTJ);
    // measured at n = m = 262144: the pass time falls from 12.2 ms at 4 workgroups per CU to a
    // plateau of ~10.6 ms at 24..64 (more waves to hide LDS latency, finer load balance)
    int target = 32 * c->num_cu;
    int splits = (int)ceil_div(target, s.row_blocks);
    if (splits > n_tiles) splits = n_tiles;
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
    int tps = (int)ceil_div(n_tiles, splits);
    s.splits = (int)ceil_div(n_tiles, tps);
    s.cols_per_split = (int64_t)tps * kTJ;
    return s;
}

}  // namespace

// Score precision of a half-step.  An fp32 score carries roundings of relative size 2^-24 at
// magnitude Mag = 2 k rho_max (k = log2e/eps, rho_max = largest squared norm after centring);
// measured against the float64 reference, a run of T half-steps at one eps accumulates about
// 0.05 * T * 2^-24 * Mag in units of eps.  fp32 scores are used while that estimate stays
// below 1.5e-5, i.e. Mag * T <= 5000; otherwise the scores are formed in float64.
// FS_LOWD_SCORE=f32|f64 overrides the choice (experiments and tests only).
bool lowd_precise(const Prepared *P, double eps)
{
    static const char *force = getenv("FS_LOWD_SCORE");
    if (force && force[0] == 'f' && force[1] == '3') return false;
    if (force && force[0] == 'f' && force[1] == '6') return true;
    if (P->force_precise) return true;
    const double k = kLog2e / eps;
    return 2.0 * k * P->rho_max * (double)(P->halfsteps_per_eps > 0 ? P->halfsteps_per_eps : 1) > 5000.0;
}

PassShape lowd_shape(const Ctx *c, int64_t n_res, int64_t n_str)
{
    // two rows per lane halve the LDS reads per pair; four cost occupancy and were slower
    int R = n_res >= 32768 ? 2 : 1;
    return shape_for(c, n_res, n_str, R);
}

fs_status lowd_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out)
{
    PassShape s = lowd_shape(c, res->cnt, str->cnt);
    const int R = s.rows_per_block / kBlock;
    const int n_tiles = (int)ceil_div(str->cnt, kTJ);
    const int tps = (int)(s.cols_per_split / kTJ);
    // host-side shape checks: every access of the kernel stays inside the padded copies
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)n_tiles * kTJ > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes)
        return fail(c, FS_ERR_DEVICE, "internal: low-d launch shape exceeds the padded buffers");
    const double cscale = 2.0 * kLog2e / eps;
    dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
    prof_begin(c, (double)res->cnt * (double)str->cnt);
    if (lowd_precise(P, eps)) {
        FS_LOWD_DISPATCH((int)P->d, (launch_lse_d<double, DD>(R, grid, c->stream, res->packed_d, str->packed_d, cscale,
                                                              tps, n_tiles, (double2 *)P->partial, res->cnt_pad)));
    } else {
        FS_LOWD_DISPATCH((int)P->d, (launch_lse_d<float, DD>(R, grid, c->stream, res->packed, str->packed,
                                                             (float)cscale, tps, n_tiles, (double2 *)P->partial,
                                                             res->cnt_pad)));
    }
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = s.splits;
    return FS_OK;
}

size_t lowd_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t p)
{
    (void)p;
    PassShape s = shape_for(c, n_res, n_str, 1);
    return (size_t)s.splits * (size_t)round_up(n_res, 1024) * kApplyPC * 4;
}

fs_status lowd_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V,
                     int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out)
{
    PassShape s = shape_for(c, res->cnt, str->cnt, 1);
    const int n_tiles = (int)ceil_div(str->cnt, kTJ);
    const int tps = (int)(s.cols_per_split / kTJ);
    if ((int64_t)s.row_blocks * kBlock > res->cnt_pad || (int64_t)n_tiles * kTJ > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes ||
        (size_t)s.splits * res->cnt_pad * kApplyPC * 4 > P->extra_bytes)
        return fail(c, FS_ERR_DEVICE, "internal: low-d apply launch shape exceeds the padded buffers");
    const double cscale = 2.0 * kLog2e / eps;
    const bool precise = lowd_precise(P, eps);
    dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
    float *opart = (float *)P->extra;
    for (int p0 = 0; p0 < p; p0 += kApplyPC) {
        if (precise) {
            FS_LOWD_DISPATCH((int)P->d, (launch_apply_d<double, DD>(grid, c->stream, res->packed_d, str->packed_d, V, ldv,
                                                                    p0, (int)p, str->cnt, cscale, tps, n_tiles,
                                                                    (double2 *)P->partial, res->cnt_pad, opart)));
        } else {
            FS_LOWD_DISPATCH((int)P->d, (launch_apply_d<float, DD>(grid, c->stream, res->packed, str->packed, V, ldv, p0,
                                                                   (int)p, str->cnt, (float)cscale, tps, n_tiles,
                                                                   (double2 *)P->partial, res->cnt_pad, opart)));
        }
        fs_status st = launch_apply_finalize(c, P, res, precise ? res->norm : res->norm_f, s.splits, eps, opart,
                                             kApplyPC, p0, (int)p, out, ldo, mass_out);
        if (st != FS_OK) return st;
    }
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
