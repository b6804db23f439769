// fp32-accuracy path for d > 16: the score contraction <x_i, y_j> runs on the fp64 matrix
// cores (v_mfma_f64_16x16x4_f64).
//
// Why fp64: with d = 64 and eps = 0.1 a score (2<x,y> - |y|^2 + g)/eps reaches ~2e3, where an
// fp32 ulp is 1.2e-4 -- the whole error budget of 1e-4.  MI355X has 78.6 TFLOP/s of fp64 MFMA,
// so the exact route costs 2x the fp32-MFMA time instead of the accuracy.
//
// Mapping of one 16x16x4 MFMA (a wrong assumption here fails every parity test of this path):
//   A operand: lane l supplies A[i = l%16][k = l/16]        -> i = STREAMED point
//   B operand: lane l supplies B[k = l/16][j = l%16]        -> j = RESIDENT row
//   D result : lane l, register r holds D[i = 4r + l/16][j = l%16]
// so the four accumulator registers of a lane are four streamed points of ONE resident row:
// the online LSE of Alg. 1 runs inside the lane, and lanes are merged only once, at the end.
// For plan application (Alg. 2/4) the exponentiated tile is, register by register, already
// in A-operand layout for the second contraction  O[j][c] += sum_i E[i][j] V[i][c]  (k = l/16
// <-> i = 4r + k), so P never leaves the registers.
//
// Workgroup: 256 threads = 4 waves; 64 resident rows (4 column blocks j of 16) x tiles of 64
// streamed points (16 per wave).  The resident block lives in LDS for the whole pass when
// d <= 64; streamed points go through LDS in contraction chunks of 32.
#include "fs_internal.h"

namespace fs {
namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));   // staging registers: a plain vector type, so that they stay registers

constexpr int BC = 64;      // streamed points per tile: one 16-point block per wave (two per wave were slower)
constexpr int KC = 32;     // contraction chunk staged for the streamed points
constexpr int KRES = 64;   // resident coordinates kept in LDS across the pass
// leading dimensions = 2 (mod 32) doubles: the 32 lanes of a half-wave (16 points x 2 adjacent
// coordinates) then read 32 different 8-byte bank pairs, and rows stay 16-byte aligned for the
// 128-bit stores of the staging
constexpr int LDR = KRES + 2;
constexpr int LDS_ = KC + 2;
constexpr int kReadAhead = 8;   // the operand reads run one contraction step ahead of the MFMAs: slack behind the arrays
constexpr int PCH = 64;    // value columns per application pass

__device__ inline float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

struct PassArgs {
    const double *res;       // [res_pad][kp]
    const double *str;       // [str_pad][kp]
    const double *bias;      // [str_pad], base-2 bias of the streamed points (-inf on padding)
    int kp;                  // row stride of res / str: coordinates rounded up to KC, zero filled
    int kc;                  // contraction length: coordinates rounded up to 8
    double cscale;           // 2 log2(e) / eps
    int tiles_per_split, n_tiles;
    double2 *partial;        // [splits][partial_stride] (max, sum)
    int64_t partial_stride;
    // application only
    const float *V;          // [n_str][ldv]
    int64_t ldv, n_str;
    int p0, p;
    float *opart;            // [splits][partial_stride][PCH]
    // Hadamard-weighted application only (Alg. 5): every plan entry times <hadA row of the
    // resident point, streamed point>
    const float *hadA;       // [n_res][lda]
    int64_t lda, n_res;
    int d;                   // real number of coordinates (columns of hadA)
};

// (two workgroups per CU for the LSE pass: with at most 256 registers per lane the compiler keeps
// the MFMA accumulators in ordinary VGPRs; with more it parks them in AGPRs and copies all of them
// in and out around every group of MFMAs)
// NCT: 16-column blocks of the value matrix this launch produces (1..4); transport-vector products
// (one column) then do a quarter of the second contraction
// JT: 16-row resident blocks per workgroup (4: 64 rows; 2: 32 rows, which lets the plan application
// run two workgroups per CU without parking accumulators in AGPRs)
template <bool APPLY, bool HAD = false, int NCT = 4, int JT = 4>
__global__ __launch_bounds__(256, (APPLY && JT == 4) ? 1 : 2) void k_pass_f64(PassArgs a)
{
    constexpr int BR = 16 * JT;   // resident rows per workgroup
    // Two buffers for the streamed chunk: the next stage is stored while other waves may still be
    // reading the current one, which leaves one barrier per stage.  The Hadamard variant keeps one
    // buffer (and a second barrier) so that two workgroups still fit in a CU's LDS.
    constexpr int NSB = HAD ? 1 : 2;
    constexpr int kStrBuf = BC * LDS_;
    __shared__ __attribute__((aligned(16))) double res_lds[BR * LDR + kReadAhead];   // 33.8 KB (JT = 4); reused for the final merge
    __shared__ __attribute__((aligned(16))) double str_lds[NSB * kStrBuf + kReadAhead];  // 17.4 KB per buffer
    __shared__ double bias_lds[3][BC];            // by tile number mod 3 (a tile's epilogue may run after the next stage is stored)
    __shared__ float vt[APPLY ? BC * PCH : 1];    // 16,384 B (application)
    __shared__ __attribute__((aligned(16))) double had_lds[HAD ? BR * LDR + kReadAhead : 1];  // rows of hadA, laid out like res_lds
    __shared__ float mw[4][BR];                   // per-wave running max (final merge)
    __shared__ float sred[BR][17];                // per-(wave, lane group) sums (final merge)

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lg = l >> 4, lj = l & 15;
    const int kld = a.kp;         // row stride of the records: a multiple of KC, zero beyond the coordinates
    const int kc = a.kc;          // contraction length: coordinates rounded up to 8
    const int64_t row0 = (int64_t)blockIdx.x * BR;
    const bool res_cached = kc <= KRES;
    const int n_chunks = (kc + KC - 1) / KC;

    if (res_cached) {
        const int per_row = kc >> 1;   // double2 per row
        for (int e = tid; e < BR * per_row; e += 256) {
            int r = e / per_row, kk = (e - r * per_row) * 2;
            *reinterpret_cast<d2 *>(res_lds + r * LDR + kk) = *reinterpret_cast<const d2 *>(a.res + (row0 + r) * kld + kk);
        }
        if constexpr (HAD) {
            for (int e = tid; e < BR * kc; e += 256) {
                int r = e / kc, kk = e - r * kc;
                had_lds[r * LDR + kk] = (row0 + r < a.n_res && kk < a.d) ? (double)a.hadA[(row0 + r) * a.lda + kk] : 0.0;
            }
        }
    }

    float mrun[JT], srun[JT];
    d4 O[APPLY ? JT : 1][APPLY ? NCT : 1];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
        mrun[jt] = kNegInit;
        srun[jt] = 0.0f;
    }
    if constexpr (APPLY) {
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) O[jt][ct] = d4{0.0, 0.0, 0.0, 0.0};
    }

    const int t_begin = blockIdx.y * a.tiles_per_split;
    const int t_end = min(a.n_tiles, t_begin + a.tiles_per_split);

    // Staging of one (tile, chunk) stage goes through registers: its global loads are issued
    // before the MFMAs of the previous stage and stored to LDS after them, so the memory latency
    // is covered by matrix work.  Addresses are a uniform base plus a per-thread offset that never
    // changes: thread (point tid / 16 of every group of 16 points, coordinates 2 (tid % 16) ..+1).
    d2 pre_s[4], pre_r[JT], pre_a[HAD ? JT : 1];
    double pre_b = 0.0;
    // value rows of the tile go through registers too, except in the Hadamard variant, which has
    // no registers to spare and loads them between the barriers instead
    constexpr bool VPRE = APPLY && !HAD;
    float pre_v[VPRE ? BC * PCH / 256 : 1];
    const int sp = tid >> 4, sk = (tid & 15) * 2;
    const int toff = sp * kld + sk;
    auto fetch = [&](int t, int ch) __attribute__((always_inline)) {
        const int64_t col0 = (int64_t)t * BC;
        const int kc0 = ch * KC;
        const double *gs = a.str + col0 * kld + kc0;
#pragma unroll
        for (int q = 0; q < 4; ++q) pre_s[q] = *reinterpret_cast<const d2 *>(gs + (int64_t)(16 * q) * kld + toff);
        if (!res_cached) {
            const double *gr = a.res + row0 * kld + kc0;
#pragma unroll
            for (int q = 0; q < JT; ++q) {
                pre_r[q] = *reinterpret_cast<const d2 *>(gr + (int64_t)(16 * q) * kld + toff);
                if constexpr (HAD) {
                    const int64_t rr = row0 + 16 * q + sp;
                    const int k0 = kc0 + sk;
                    pre_a[q].x = (rr < a.n_res && k0 < a.d) ? (double)a.hadA[rr * a.lda + k0] : 0.0;
                    pre_a[q].y = (rr < a.n_res && k0 + 1 < a.d) ? (double)a.hadA[rr * a.lda + k0 + 1] : 0.0;
                }
            }
        }
        if (ch == 0 && tid < BC) pre_b = a.bias[col0 + tid];
        if constexpr (VPRE) {
            if (ch == 0) {
#pragma unroll
                for (int q = 0; q < BC * PCH / 256; ++q) {
                    const int e = tid + 256 * q;
                    const int cidx = e >> 6, cc = e & 63;
                    const int64_t j = col0 + cidx;
                    pre_v[q] = (j < a.n_str && a.p0 + cc < a.p) ? a.V[j * a.ldv + a.p0 + cc] : 0.0f;
                }
            }
        }
    };
    // store the fetched stage: streamed chunk into buffer `buf`, the resident chunk (when it is not
    // cached) into columns [32 buf, 32 buf + 32) of its rows, bias and values of a tile's first stage
    auto stash = [&](int buf, int t_st, int ch, int tile_mod3) __attribute__((always_inline)) {
        double *sd = str_lds + buf * kStrBuf + sp * LDS_ + sk;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<d2 *>(sd + 16 * q * LDS_) = pre_s[q];
        if (!res_cached) {
#pragma unroll
            for (int q = 0; q < JT; ++q) {
                *reinterpret_cast<d2 *>(res_lds + (16 * q + sp) * LDR + KC * buf + sk) = pre_r[q];
                if constexpr (HAD) *reinterpret_cast<d2 *>(had_lds + (16 * q + sp) * LDR + KC * buf + sk) = pre_a[q];
            }
        }
        if (ch == 0 && tid < BC) bias_lds[tile_mod3][tid] = pre_b;
        if constexpr (VPRE) {
            if (ch == 0) {
#pragma unroll
                for (int q = 0; q < BC * PCH / 256; ++q) vt[tid + 256 * q] = pre_v[q];
            }
        } else if constexpr (APPLY) {
            if (ch == 0) {
                const int64_t col0 = (int64_t)t_st * BC;
                for (int e = tid; e < BC * PCH; e += 256) {
                    const int cidx = e >> 6, cc = e & 63;
                    const int64_t j = col0 + cidx;
                    vt[e] = (j < a.n_str && a.p0 + cc < a.p) ? a.V[j * a.ldv + a.p0 + cc] : 0.0f;
                }
            }
        }
    };

    d4 acc[JT];
    d4 accW[HAD ? JT : 1];   // <hadA row, streamed point> (Hadamard weights)
    auto zero_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            acc[jt] = d4{0.0, 0.0, 0.0, 0.0};
            if constexpr (HAD) accW[jt] = d4{0.0, 0.0, 0.0, 0.0};
        }
    };

    // ---- tile epilogue: scores of this lane = cscale * acc + bias of its four streamed points
    auto epilogue = [&](int tile_mod3) __attribute__((always_inline)) {
        const int sp0 = 16 * w;   // first streamed point of this wave's block within the tile
        double bias[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bias[r] = bias_lds[tile_mod3][sp0 + 4 * r + lg];

        if constexpr (!APPLY) {
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                double sc[4];
                float mx = kNegInit;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    sc[r] = fma(acc[jt][r], a.cscale, bias[r]);
                    mx = fmaxf(mx, (float)sc[r]);
                }
                float mnew = fmaxf(mrun[jt], ceilf(mx));
                float scale = fast_exp2(mrun[jt] - mnew);
                double md = (double)mnew;
                float csum = 0.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r) csum += fast_exp2((float)(sc[r] - md));
                srun[jt] = fmaf(srun[jt], scale, csum);
                mrun[jt] = mnew;
            }
        } else {
            double sc[JT][4];
            float mx[JT];
            bool raise = false;
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                float m = kNegInit;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    sc[jt][r] = fma(acc[jt][r], a.cscale, bias[r]);
                    m = fmaxf(m, (float)sc[jt][r]);
                }
                // the stabiliser of a resident row must be common to the four lane groups,
                // because the second MFMA sums over them
                m = fmaxf(m, __shfl_xor(m, 16, 64));
                m = fmaxf(m, __shfl_xor(m, 32, 64));
                mx[jt] = m;
                raise = raise || (m > mrun[jt] + 40.0f);
            }
            if (__any(raise)) {
                // rare: lift the (integer) stabilisers and rescale sums and accumulators exactly
#pragma unroll
                for (int jt = 0; jt < JT; ++jt) {
                    float mnew = fmaxf(mrun[jt], ceilf(mx[jt]));
                    float scale = fast_exp2(mrun[jt] - mnew);
                    srun[jt] *= scale;
                    mrun[jt] = mnew;
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // accumulator register r holds resident row 4r + lg of this column block
                        double scd = (double)__shfl(scale, 4 * r + lg, 64);
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct) O[jt][ct][r] *= scd;
                    }
                }
            }
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) {
                double md = (double)mrun[jt];
                double E[4];
                float csum = 0.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float e = fast_exp2((float)(sc[jt][r] - md));
                    csum += e;
                    E[r] = (double)e;
                    if constexpr (HAD) E[r] *= accW[jt][r];
                }
                srun[jt] += csum;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        double vv = (double)vt[(sp0 + 4 * r + lg) * PCH + 16 * ct + lj];
                        O[jt][ct] = __builtin_amdgcn_mfma_f64_16x16x4f64(E[r], vv, O[jt][ct], 0, 0, 0);
                    }
                }
            }
        }
    };

    // ---- the stages (tile, chunk) of this workgroup's split, in order ---------------------------
    auto advance = [&](int &t, int &ch, int &m3) __attribute__((always_inline)) {
        if (++ch == n_chunks) {
            ch = 0;
            ++t;
            m3 = m3 == 2 ? 0 : m3 + 1;
        }
    };
    int t = t_begin, ch = 0, m3 = 0;     // stage being contracted (m3: its tile's number mod 3)
    int tn = t, chn = 0, m3n = 0;        // stage stored next
    advance(tn, chn, m3n);
    int par = 0;                         // buffer of the stage being contracted
    if (t < t_end) {
        fetch(t, 0);
        stash(0, t, 0, 0);
    }
    __syncthreads();
    if (tn < t_end) fetch(tn, chn);
    zero_acc();

    while (t < t_end) {
        const int kc0 = ch * KC;
        const int kw = min(KC, kc - kc0);
        const int kbase = res_cached ? kc0 : KC * par;
        const double *sa = str_lds + par * kStrBuf + (16 * w + lj) * LDS_ + lg;
        const double *sb = res_lds + lj * LDR + kbase + lg;
        const double *sw = had_lds + lj * LDR + kbase + lg;
        // Operands of contraction step k+1 are read from LDS before the MFMAs of step k are
        // issued (two register sets, ping-pong): otherwise every group of MFMAs starts by
        // waiting out the LDS latency with an idle matrix pipe.  The last trip reads one step
        // past the chunk (never used; it stays inside the arrays' slack).
        double av0, av1, bv0[JT], bv1[JT], wv0[HAD ? JT : 1], wv1[HAD ? JT : 1];
        auto rd = [&](int kk, double &av, double (&bv)[JT], double (&wv)[HAD ? JT : 1]) {
            av = sa[kk];
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) bv[jt] = sb[jt * 16 * LDR + kk];
            if constexpr (HAD) {
#pragma unroll
                for (int jt = 0; jt < JT; ++jt) wv[jt] = sw[jt * 16 * LDR + kk];
            }
        };
        auto mm = [&](double av, const double (&bv)[JT], const double (&wv)[HAD ? JT : 1]) {
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) acc[jt] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, bv[jt], acc[jt], 0, 0, 0);
            if constexpr (HAD) {
#pragma unroll
                for (int jt = 0; jt < JT; ++jt) accW[jt] = __builtin_amdgcn_mfma_f64_16x16x4f64(av, wv[jt], accW[jt], 0, 0, 0);
            }
        };
        rd(0, av0, bv0, wv0);
        for (int kk = 0; kk < kw; kk += 8) {   // kw is a multiple of 8
            rd(kk + 4, av1, bv1, wv1);
            __builtin_amdgcn_sched_barrier(0);
            mm(av0, bv0, wv0);
            __builtin_amdgcn_sched_barrier(0);
            rd(kk + 8, av0, bv0, wv0);
            __builtin_amdgcn_sched_barrier(0);
            mm(av1, bv1, wv1);
            __builtin_amdgcn_sched_barrier(0);
        }

        const bool last = ch == n_chunks - 1;
        if constexpr (APPLY) {
            // the epilogue reads the tile's values and bias, which the store below replaces
            if (last) {
                epilogue(m3);
                zero_acc();
                __syncthreads();
            } else if (NSB == 1) {
                __syncthreads();
            }
        } else if (NSB == 1) {
            __syncthreads();
        }
        if (tn < t_end) stash(NSB == 2 ? par ^ 1 : 0, tn, chn, m3n);
        __syncthreads();
        int t2 = tn, ch2 = chn, m32 = m3n;
        advance(t2, ch2, m32);
        if (t2 < t_end) fetch(t2, ch2);
        if constexpr (!APPLY) {
            if (last) {
                epilogue(m3);
                zero_acc();
            }
        }
        t = tn;
        ch = chn;
        m3 = m3n;
        tn = t2;
        chn = ch2;
        m3n = m32;
        if (NSB == 2) par ^= 1;
    }

    // ---- merge the 4 waves x 4 lane groups of every resident row ---------------------------
    __syncthreads();
    if constexpr (APPLY) {
        if (lg == 0) {
#pragma unroll
            for (int jt = 0; jt < JT; ++jt) mw[w][16 * jt + lj] = mrun[jt];
        }
    } else {
        // per-lane maxima differ: reduce them over the lane groups first
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            float m = mrun[jt];
            m = fmaxf(m, __shfl_xor(m, 16, 64));
            m = fmaxf(m, __shfl_xor(m, 32, 64));
            srun[jt] *= fast_exp2(mrun[jt] - m);
            mrun[jt] = m;
            if (lg == 0) mw[w][16 * jt + lj] = m;
        }
    }
    __syncthreads();
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
        int r = 16 * jt + lj;
        float M = fmaxf(fmaxf(mw[0][r], mw[1][r]), fmaxf(mw[2][r], mw[3][r]));
        sred[r][4 * w + lg] = srun[jt] * fast_exp2(mrun[jt] - M);
    }
    if constexpr (APPLY) {
        double *obuf = res_lds;   // [BR][PCH] doubles = 32 KB <= sizeof(res_lds)
        for (int ww = 0; ww < 4; ++ww) {
            if (w == ww) {
#pragma unroll
                for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int row = 16 * jt + 4 * r + lg;
                        float M = fmaxf(fmaxf(mw[0][row], mw[1][row]), fmaxf(mw[2][row], mw[3][row]));
                        double sc = (double)fast_exp2(mw[w][row] - M);
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct) {
                            int idx = row * PCH + 16 * ct + lj;
                            double v = O[jt][ct][r] * sc;
                            obuf[idx] = (ww == 0) ? v : obuf[idx] + v;
                        }
                    }
            }
            __syncthreads();
        }
        for (int e = tid; e < BR * PCH; e += 256) {
            int r = e >> 6, cc = e & 63;
            a.opart[((int64_t)blockIdx.y * a.partial_stride + row0 + r) * PCH + cc] = cc < 16 * NCT ? (float)obuf[e] : 0.0f;
        }
    }
    __syncthreads();
    if (tid < BR) {
        float M = fmaxf(fmaxf(mw[0][tid], mw[1][tid]), fmaxf(mw[2][tid], mw[3][tid]));
        double S = 0.0;
#pragma unroll
        for (int k = 0; k < 16; ++k) S += (double)sred[tid][k];
        a.partial[(int64_t)blockIdx.y * a.partial_stride + row0 + tid] = make_double2((double)M, S);
    }
}

constexpr int kLseJT = 4, kApplyJT = 2;   // resident blocks per workgroup of the two passes

PassShape shape_f64(const Ctx *c, int64_t n_res, int64_t n_str, int br)
{
    PassShape s;
    s.rows_per_block = br;
    s.row_blocks = (int)ceil_div(n_res, br);
    int n_tiles = (int)ceil_div(n_str, BC);
    int target = 2 * c->num_cu;
    int splits = (int)ceil_div(target, s.row_blocks);
    if (splits > n_tiles) splits = n_tiles;
    if (splits > max_splits(n_res)) splits = max_splits(n_res);
    if (splits < 1) splits = 1;
    int tps = (int)ceil_div(n_tiles, splits);
    s.splits = (int)ceil_div(n_tiles, tps);
    s.cols_per_split = (int64_t)tps * BC;
    return s;
}

}  // namespace

fs_status f64_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out)
{
    PassShape s = shape_f64(c, res->cnt, str->cnt, 16 * kLseJT);
    PassArgs a{};
    a.res = res->pts_d;
    a.str = str->pts_d;
    a.bias = str->bias_d;
    a.kp = P->kp;
    a.kc = (int)round_up(P->d, 8);
    a.cscale = 2.0 * kLog2e / eps;
    a.n_tiles = (int)ceil_div(str->cnt, BC);
    a.tiles_per_split = (int)(s.cols_per_split / BC);
    a.partial = (double2 *)P->partial;
    a.partial_stride = res->cnt_pad;
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)a.n_tiles * BC > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp % KC) != 0 || a.kc > a.kp)
        return fail(c, FS_ERR_DEVICE, "internal: fp64 launch shape exceeds the padded buffers");
    prof_begin(c, (double)res->cnt * (double)str->cnt);
    hipLaunchKernelGGL((k_pass_f64<false, false, 4, kLseJT>), dim3((unsigned)s.row_blocks, (unsigned)s.splits), dim3(256), 0, c->stream, a);
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = s.splits;
    return FS_OK;
}

size_t f64_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t d, int64_t p)
{
    (void)d;
    (void)p;
    PassShape s = shape_f64(c, n_res, n_str, 16 * kApplyJT);
    return (size_t)s.splits * (size_t)round_up(n_res, 1024) * PCH * 4;
}

fs_status f64_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V,
                    int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out, const float *hadA, int64_t lda)
{
    PassShape s = shape_f64(c, res->cnt, str->cnt, 16 * kApplyJT);
    PassArgs a{};
    a.res = res->pts_d;
    a.str = str->pts_d;
    a.bias = str->bias_d;
    a.kp = P->kp;
    a.kc = (int)round_up(P->d, 8);
    a.cscale = 2.0 * kLog2e / eps;
    a.n_tiles = (int)ceil_div(str->cnt, BC);
    a.tiles_per_split = (int)(s.cols_per_split / BC);
    a.partial = (double2 *)P->partial;
    a.partial_stride = res->cnt_pad;
    a.V = V;
    a.ldv = ldv;
    a.n_str = str->cnt;
    a.p = (int)p;
    a.opart = (float *)P->extra;
    a.hadA = hadA;
    a.lda = lda;
    a.n_res = res->cnt;
    a.d = (int)P->d;
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)a.n_tiles * BC > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp % KC) != 0 || a.kc > a.kp ||
        (size_t)s.splits * res->cnt_pad * PCH * 4 > P->extra_bytes)
        return fail(c, FS_ERR_DEVICE, "internal: fp64 apply launch shape exceeds the padded buffers");
    for (int p0 = 0; p0 < p; p0 += PCH) {
        a.p0 = p0;
        const dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
        const int nct = (int)ceil_div((p - p0 < PCH ? p - p0 : (int64_t)PCH), 16);
#define FS_F64_APPLY(H, N) hipLaunchKernelGGL((k_pass_f64<true, H, N, kApplyJT>), grid, dim3(256), 0, c->stream, a)
        if (hadA) {
            switch (nct) {
            case 1: FS_F64_APPLY(true, 1); break;
            case 2: FS_F64_APPLY(true, 2); break;
            case 3: FS_F64_APPLY(true, 3); break;
            default: FS_F64_APPLY(true, 4); break;
            }
        } else {
            switch (nct) {
            case 1: FS_F64_APPLY(false, 1); break;
            case 2: FS_F64_APPLY(false, 2); break;
            case 3: FS_F64_APPLY(false, 3); break;
            default: FS_F64_APPLY(false, 4); break;
            }
        }
#undef FS_F64_APPLY
        fs_status st = launch_apply_finalize(c, P, res, res->norm, s.splits, eps, a.opart, PCH, p0, (int)p, out, ldo,
                                             mass_out);
        if (st != FS_OK) return st;
    }
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
