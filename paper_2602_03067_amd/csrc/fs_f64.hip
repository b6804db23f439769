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
// <-> i = 4r + k), so P never leaves the registers.  That second contraction runs on the fp32 matrix
// cores (v_mfma_f32_16x16x4_f32, operands laid out as above, D: lane l, register r holds
// D[4 (l/16) + r][l%16]): exponentials and values are floats, and fp32 accumulators take half the
// time and half the registers.
//
// Workgroup: 4 or 8 waves; 64 (LSE) or 32 (application) resident rows in column blocks j of 16 x
// tiles of 16 streamed points per wave.  The resident block lives in LDS for the whole pass when
// d <= 64; streamed points go through LDS in contraction chunks of 32.
#include "fs_internal.h"

namespace fs {
namespace {

typedef double d4 __attribute__((ext_vector_type(4)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef double d2 __attribute__((ext_vector_type(2)));   // staging registers: a plain vector type, so that they stay registers

constexpr int KC = 32;     // contraction chunk staged for the streamed points
constexpr int KRES = 64;   // resident coordinates kept in LDS across the pass
// leading dimensions = 2 (mod 32) doubles: the 32 lanes of a half-wave (16 points x 2 adjacent
// coordinates) then read 32 different 8-byte bank pairs, and rows stay 16-byte aligned for the
// 128-bit stores of the staging
constexpr int LDR = KRES + 2;
constexpr int LDS_ = KC + 2;
constexpr int kReadAhead = 16;  // the operand reads run one contraction step ahead of the MFMAs: slack behind the arrays
constexpr int PCH = 64;    // value columns per application pass (128 in the wide form, see the kernel)

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

// (never more than 256 registers per lane: with at most 256 the compiler keeps the MFMA
// accumulators in ordinary VGPRs; with more it parks them in AGPRs and copies all of them in and
// out around every group of MFMAs.  The LSE pass needs ~120 and 52 KB of LDS: three workgroups per CU.)
// NCT: 16-column blocks of the value matrix this launch produces (1..4); transport-vector products
// (one column) then do a quarter of the second contraction
// JT: 16-row resident blocks per workgroup (4: 64 rows; 2: 32 rows, which lets the plan application
// run two workgroups per CU without parking accumulators in AGPRs)
// NW: waves per workgroup; a wave owns 16 streamed points of every tile (two 16-point blocks per
// wave were slower), so a tile has 16 NW points.  The LSE pass runs 8 waves over one resident
// block (4 waves per SIMD with two workgroups per CU), the application 4.
// LAZY: the stabiliser of the epilogue (see there); the LSE pass uses it for the short contractions it
// runs on behalf of the low-dimension path, whose scores spread little.
template <bool APPLY, bool HAD = false, int NCT = 4, int JT = 4, int NW = 4, bool LAZY = APPLY>
__device__ __forceinline__ void pass_f64_body(const PassArgs &a, const int bx, const int by)
{
    static_assert(LAZY || !APPLY, "the application has the lazy stabiliser only");
    constexpr int NT = 64 * NW;   // threads
    constexpr int BC = 16 * NW;   // streamed points per tile
    constexpr int BR = 16 * JT;   // resident rows per workgroup
    __shared__ __attribute__((aligned(16))) double res_lds[BR * LDR + kReadAhead];   // 33.8 KB (JT = 4); reused for the final merge
    __shared__ __attribute__((aligned(16))) double str_lds[BC * LDS_ + kReadAhead];  // 17.4 KB: 16 points per wave, wave-private
    __shared__ double bias_lds[BC];
    // value columns of a pass: 64, or 128 in the wide form (NCT > 4: twice the output registers, two workgroups
    // per CU), which halves the passes -- and the repeated score contractions -- of an application with p > 64
    constexpr int PCH = NCT > 4 ? 128 : 64;
    constexpr int NVQ = PCH / 64;                 // value columns per lane and streamed point
    static_assert(NCT >= 1 && NCT <= 8 && (!HAD || NCT <= 4), "column blocks of a pass");
    __shared__ __attribute__((aligned(16))) float vt[APPLY ? BC * PCH : 1];    // 16 or 32 KB (application)
    __shared__ __attribute__((aligned(16))) double had_lds[HAD ? BR * LDR + kReadAhead : 1];  // rows of hadA, laid out like res_lds
    // final merge: per-wave running max and per-(wave, lane group) sums, on top of the streamed
    // staging area, which is free by then (this keeps the LSE pass at three workgroups per CU)
    static_assert(sizeof(float) * (NW * BR + BR * (4 * NW + 1)) <= sizeof(double) * BC * LDS_, "merge scratch exceeds the staging area");
    float (*mw)[BR] = reinterpret_cast<float (*)[BR]>(str_lds);
    float (*sred)[4 * NW + 1] = reinterpret_cast<float (*)[4 * NW + 1]>(reinterpret_cast<float *>(str_lds) + NW * BR);

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63, lg = l >> 4, lj = l & 15;
    const int kld = a.kp;         // row stride of the records: a multiple of KC, zero beyond the coordinates
    const int kc = a.kc;          // contraction length: coordinates rounded up to 8
    const int64_t row0 = (int64_t)bx * BR;
    const bool res_cached = kc <= KRES;
    const int n_chunks = (kc + KC - 1) / KC;

    if (res_cached) {
        const int per_row = kc >> 1;   // double2 per row
        for (int e = tid; e < BR * per_row; e += NT) {
            int r = e / per_row, kk = (e - r * per_row) * 2;
            *reinterpret_cast<d2 *>(res_lds + r * LDR + kk) = *reinterpret_cast<const d2 *>(a.res + (row0 + r) * kld + kk);
        }
        if constexpr (HAD) {
            for (int e = tid; e < BR * kc; e += NT) {
                int r = e / kc, kk = e - r * kc;
                had_lds[r * LDR + kk] = (row0 + r < a.n_res && kk < a.d) ? (double)a.hadA[(row0 + r) * a.lda + kk] : 0.0;
            }
        }
    }

    float mrun[JT], srun[JT];
    // Output accumulators of the second contraction, in fp32: E <= 2^60 and V are floats, a register adds a
    // few thousand products, and fp32 MFMAs take half the time and half the registers of fp64 ones.
    // v_mfma_f32_16x16x4_f32: A and B as in the fp64 form, D: lane l, register r holds D[4 (l / 16) + r][l % 16].
    f4 O[APPLY ? JT : 1][APPLY ? NCT : 1];
#pragma unroll
    for (int jt = 0; jt < JT; ++jt) {
        mrun[jt] = kNegInit;
        srun[jt] = 0.0f;
    }
    if constexpr (APPLY) {
#pragma unroll
        for (int jt = 0; jt < JT; ++jt)
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) O[jt][ct] = f4{0.0f, 0.0f, 0.0f, 0.0f};
    }

    const int t_begin = by * a.tiles_per_split;
    const int t_end = min(a.n_tiles, t_begin + a.tiles_per_split);

    // Staging of one (tile, chunk) stage goes through registers: its global loads are issued
    // before the MFMAs of the previous stage and stored to LDS after them, so the memory latency
    // is covered by matrix work.  Everything that belongs to the streamed points (coordinates,
    // bias, value rows) is WAVE-PRIVATE: a wave loads, stores and reads only its own 16 points, so
    // program order within the wave is all the synchronisation these need.  When the resident rows
    // fit in LDS for the whole pass (d <= 64) the loop therefore has no barrier at all, and the
    // four waves drift apart freely, which lets one wave's epilogue overlap the others' MFMAs.
    // Only a resident block that has to be staged chunk by chunk (d > 64) is shared: it alternates
    // between the two column halves of res_lds, with one barrier per stage.
    // Addresses are a uniform base plus a per-thread offset that never changes.
    constexpr int RP = NT / 16;        // resident rows one staging pass of the workgroup covers
    constexpr int NRQ = BR / RP;       // passes per resident chunk
    static_assert(BR % RP == 0 && NRQ >= 1, "resident block and workgroup size do not match");
    d2 pre_s[4], pre_r[NRQ], pre_a[HAD ? NRQ : 1];
    double pre_b = 0.0;
    // value rows of the tile go through registers too, except in the Hadamard variant, which has
    // no registers to spare and loads them at the store instead
    constexpr bool VPRE = APPLY && !HAD;
    float pre_v[VPRE ? 16 * NVQ : 1];
    const int sk = (l & 15) * 2;                  // coordinate pair of this thread within a chunk
    const int toff_s = (16 * w + lg) * kld + sk;  // streamed: point 16 w + 4 q + lg of the tile
    const int sp = tid >> 4;
    const int toff_r = sp * kld + sk;             // resident: row (NT / 16) q + sp of the block
    auto fetch = [&](int t, int ch) __attribute__((always_inline)) {
        const int64_t col0 = (int64_t)t * BC;
        const int kc0 = ch * KC;
        const double *gs = a.str + col0 * kld + kc0;
#pragma unroll
        for (int q = 0; q < 4; ++q) pre_s[q] = *reinterpret_cast<const d2 *>(gs + (int64_t)(4 * q) * kld + toff_s);
        if (!res_cached) {
            const double *gr = a.res + row0 * kld + kc0;
#pragma unroll
            for (int q = 0; q < NRQ; ++q) {
                pre_r[q] = *reinterpret_cast<const d2 *>(gr + (int64_t)(RP * q) * kld + toff_r);
                if constexpr (HAD) {
                    const int64_t rr = row0 + RP * q + sp;
                    const int k0 = kc0 + sk;
                    pre_a[q].x = (rr < a.n_res && k0 < a.d) ? (double)a.hadA[rr * a.lda + k0] : 0.0;
                    pre_a[q].y = (rr < a.n_res && k0 + 1 < a.d) ? (double)a.hadA[rr * a.lda + k0 + 1] : 0.0;
                }
            }
        }
        if (ch == 0 && l < 16) pre_b = a.bias[col0 + 16 * w + l];
        if constexpr (VPRE) {
            if (ch == 0) {
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    const int64_t j = col0 + 16 * w + q;
#pragma unroll
                    for (int h = 0; h < NVQ; ++h) {
                        const int cc = a.p0 + l + 64 * h;
                        pre_v[q * NVQ + h] = (j < a.n_str && cc < a.p) ? a.V[j * a.ldv + cc] : 0.0f;
                    }
                }
            }
        }
    };
    // store the fetched stage; `half` = column half of res_lds the shared resident chunk goes to
    auto stash = [&](int half, int t_st, int ch) __attribute__((always_inline)) {
        double *sd = str_lds + (16 * w + lg) * LDS_ + sk;
#pragma unroll
        for (int q = 0; q < 4; ++q) *reinterpret_cast<d2 *>(sd + 4 * q * LDS_) = pre_s[q];
        if (!res_cached) {
#pragma unroll
            for (int q = 0; q < NRQ; ++q) {
                *reinterpret_cast<d2 *>(res_lds + (RP * q + sp) * LDR + KC * half + sk) = pre_r[q];
                if constexpr (HAD) *reinterpret_cast<d2 *>(had_lds + (RP * q + sp) * LDR + KC * half + sk) = pre_a[q];
            }
        }
        if (ch == 0 && l < 16) bias_lds[16 * w + l] = pre_b;
        if constexpr (VPRE) {
            if (ch == 0) {
#pragma unroll
                for (int q = 0; q < 16; ++q)
#pragma unroll
                    for (int h = 0; h < NVQ; ++h) vt[(16 * w + q) * PCH + l + 64 * h] = pre_v[q * NVQ + h];
            }
        } else if constexpr (APPLY) {
            if (ch == 0) {
                const int64_t col0 = (int64_t)t_st * BC;
#pragma unroll 4
                for (int q = 0; q < 16; ++q) {
                    const int64_t j = col0 + 16 * w + q;
                    vt[(16 * w + q) * PCH + l] = (j < a.n_str && a.p0 + l < a.p) ? a.V[j * a.ldv + a.p0 + l] : 0.0f;
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
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int sp0 = 16 * w;   // first streamed point of this wave's block within the tile
        double bias[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) bias[r] = bias_lds[sp0 + 4 * r + lg];

        if constexpr (!LAZY) {
            // every tile lifts the running max (an integer) to the ceiling of its largest score
            // (at d = 64 the lazy scheme below was measured slower: 0.605 against 0.587 ms at n = m = 16384
            // with one check per block, 0.623 with one per tile; scores that spread over hundreds of
            // base-2 units send some lane of the wave through its recompute path in many tiles)
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
            return;
        }
        // Lazy stabiliser: the running max (an integer) is not tracked tile by tile.  The
        // exponentials are taken against the current one and their sum is checked against 2^60;
        // only when that fails (the first tile, and the few times a row meets much larger scores)
        // is the max lifted to the ceiling of the tile's largest score, the running sums rescaled
        // by the exact power of two and the tile's exponentials redone.  Terms below 2^-126 of a
        // sum that has held a term above 1/2 are lost, which is far below fp32 resolution.
#pragma unroll
        for (int jt = 0; jt < JT; ++jt) {
            double sc[4];
            float e[4];
            double md = (double)mrun[jt];
            float csum = 0.0f;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                sc[r] = fma(acc[jt][r], a.cscale, bias[r]);
                e[r] = fast_exp2((float)(sc[r] - md));
                csum += e[r];
            }
            if (__any(!(csum < 0x1p60f))) {
                float m = kNegInit;
#pragma unroll
                for (int r = 0; r < 4; ++r) m = fmaxf(m, (float)sc[r]);
                if constexpr (APPLY) {
                    // the stabiliser of a resident row must be common to the four lane groups,
                    // because the second MFMA sums over them
                    m = fmaxf(m, __shfl_xor(m, 16, 64));
                    m = fmaxf(m, __shfl_xor(m, 32, 64));
                }
                const float mnew = fmaxf(mrun[jt], ceilf(m));
                const float scale = fast_exp2(mrun[jt] - mnew);
                srun[jt] *= scale;
                mrun[jt] = mnew;
                if constexpr (APPLY) {
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        // output register r holds resident row 4 lg + r of this column block
                        const float scr = __shfl(scale, 4 * lg + r, 64);
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct) O[jt][ct][r] *= scr;
                    }
                }
                md = (double)mnew;
                csum = 0.0f;
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    e[r] = fast_exp2((float)(sc[r] - md));
                    csum += e[r];
                }
            }
            srun[jt] += csum;
            if constexpr (APPLY) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    float E = e[r];
                    if constexpr (HAD) E *= (float)accW[jt][r];
#pragma unroll
                    for (int ct = 0; ct < NCT; ++ct) {
                        const float vv = vt[(sp0 + 4 * r + lg) * PCH + 16 * ct + lj];
                        O[jt][ct] = __builtin_amdgcn_mfma_f32_16x16x4f32(E, vv, O[jt][ct], 0, 0, 0);
                    }
                }
            }
        }
    };

    // ---- the stages (tile, chunk) of this workgroup's split, in order ---------------------------
    auto advance = [&](int &t, int &ch) __attribute__((always_inline)) {
        if (++ch == n_chunks) {
            ch = 0;
            ++t;
        }
    };
    int t = t_begin, ch = 0;     // stage being contracted
    int tn = t, chn = 0;         // stage stored next
    advance(tn, chn);
    int par = 0;                 // column half of a staged resident chunk
    if (t < t_end) {
        fetch(t, 0);
        stash(0, t, 0);
    }
    __syncthreads();             // resident rows (cached or first chunk) are in place
    if (tn < t_end) fetch(tn, chn);
    zero_acc();

    while (t < t_end) {
        const int kc0 = ch * KC;
        const int kw = min(KC, kc - kc0);
        const int kbase = res_cached ? kc0 : KC * par;
        const double *sa = str_lds + (16 * w + lj) * LDS_ + lg;
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

        if (ch == n_chunks - 1) {
            epilogue();
            zero_acc();
        }
        // the wave is done reading its part of the staging arrays: store the next stage
        __builtin_amdgcn_wave_barrier();
        if (tn < t_end) stash(par ^ 1, tn, chn);
        __builtin_amdgcn_wave_barrier();
        if (!res_cached) __syncthreads();   // uniform over the workgroup: the shared resident chunk
        int t2 = tn, ch2 = chn;
        advance(t2, ch2);
        if (t2 < t_end) fetch(t2, ch2);
        t = tn;
        ch = chn;
        tn = t2;
        chn = ch2;
        par ^= 1;
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
        float M = mw[0][r];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, mw[ww][r]);
        sred[r][4 * w + lg] = srun[jt] * fast_exp2(mrun[jt] - M);
    }
    if constexpr (APPLY) {
        // [BR][PCH] doubles: on top of the resident rows, or (wide form) of the value rows
        static_assert(NCT > 4 ? sizeof(double) * BR * PCH <= sizeof(float) * BC * PCH : sizeof(double) * BR * PCH <= sizeof(double) * BR * LDR,
                      "merge buffer of the outputs");
        double *obuf = NCT > 4 ? reinterpret_cast<double *>(vt) : res_lds;
        for (int ww = 0; ww < NW; ++ww) {
            if (w == ww) {
#pragma unroll
                for (int jt = 0; jt < JT; ++jt)
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        int row = 16 * jt + 4 * lg + r;
                        float M = mw[0][row];
#pragma unroll
                        for (int w2 = 1; w2 < NW; ++w2) M = fmaxf(M, mw[w2][row]);
                        double sc = (double)fast_exp2(mw[w][row] - M);
#pragma unroll
                        for (int ct = 0; ct < NCT; ++ct) {
                            int idx = row * PCH + 16 * ct + lj;
                            double v = (double)O[jt][ct][r] * sc;
                            obuf[idx] = (ww == 0) ? v : obuf[idx] + v;
                        }
                    }
            }
            __syncthreads();
        }
        for (int e = tid; e < BR * PCH; e += NT) {
            int r = e / PCH, cc = e % PCH;
            a.opart[((int64_t)by * a.partial_stride + row0 + r) * PCH + cc] = cc < 16 * NCT ? (float)obuf[e] : 0.0f;
        }
    }
    __syncthreads();
    if (tid < BR) {
        float M = mw[0][tid];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) M = fmaxf(M, mw[ww][tid]);
        double S = 0.0;
#pragma unroll
        for (int k = 0; k < 4 * NW; ++k) S += (double)sred[tid][k];
        a.partial[(int64_t)by * a.partial_stride + row0 + tid] = make_double2((double)M, S);
    }
}

// (the plain application needs at most 158 registers and 51 KB of LDS: three workgroups per CU)
template <bool APPLY, bool HAD = false, int NCT = 4, int JT = 4, int NW = 4, bool LAZY = APPLY>
__global__ __launch_bounds__(64 * NW, (APPLY && !HAD && NCT <= 4) ? 3 : 2) void k_pass_f64(PassArgs a)
{
    pass_f64_body<APPLY, HAD, NCT, JT, NW, LAZY>(a, blockIdx.x, blockIdx.y);
}

// Both LSE passes of one iteration of the averaged schedule (Eq. 4-5) in one launch: they read the same
// old potentials, so the row blocks of the f-pass (a0, the first rb0 of the grid) and of the g-pass (a1)
// share a grid; grid.y covers the larger of the two split counts.
template <int JT, int NW, bool LAZY>
__global__ __launch_bounds__(64 * NW, 2) void k_pass_f64_pair(PassArgs a0, PassArgs a1, int rb0, int splits0, int splits1)
{
    const bool second = (int)blockIdx.x >= rb0;   // uniform over the workgroup
    if ((int)blockIdx.y >= (second ? splits1 : splits0)) return;
    pass_f64_body<false, false, 4, JT, NW, LAZY>(second ? a1 : a0, (int)blockIdx.x - (second ? rb0 : 0), blockIdx.y);
}

constexpr int kLseJT = 4, kApplyJT = 2;   // resident blocks per workgroup of the two passes
constexpr int kLseNW = 8, kApplyNW = 4;   // waves per workgroup
constexpr int kLseWgPerCu = 2, kApplyWgPerCu = 3;   // as in the kernels' launch bounds (the Hadamard variant: 2)

// Launch shape: row blocks x splits of the streamed side.  The split count minimises a makespan
// model in units of the time a CU needs for one tile: workgroups are dealt to the CUs evenly, a CU
// with w of them takes w (tiles per split + start-up) tile times (two resident workgroups share the
// matrix pipe, so each runs at half speed; one alone cannot fill the CU and is charged 1.4x), and
// every split adds a record per row to the merge.  Filling "twice the CUs" regardless of the size, as
// the first version did, gave e.g. 628 workgroups on 512 slots at n = 10000: a second round at a
// quarter of the chip.
PassShape shape_f64(const Ctx *c, int64_t n_res, int64_t n_str, int br, int bc, int64_t kc, int wg_per_cu)
{
    PassShape s;
    s.rows_per_block = br;
    s.row_blocks = (int)ceil_div(n_res, br);
    const int n_tiles = (int)ceil_div(n_str, bc);
    int cap = max_splits(c->partial_budget, n_res);
    if (cap > n_tiles) cap = n_tiles;
    if (cap < 1) cap = 1;
    const double startup = 64.0 / (double)(kc < 8 ? 8 : kc);   // ~5 us of start-up and wind-down in tile times
    double best = 0.0;
    int best_tps = n_tiles;
    for (int sp = 1; sp <= cap; ++sp) {
        const int tps = (int)ceil_div(n_tiles, sp);
        const int eff = (int)ceil_div(n_tiles, tps);
        if (eff != sp) continue;   // the same shape as a smaller count
        const int64_t w = ceil_div((int64_t)s.row_blocks * eff, (int64_t)c->num_cu);
        // workgroups of a CU run wg_per_cu at a time; an incomplete last batch cannot fill the CU: one
        // workgroup alone is charged 1.4x, two of three 1.08x (measured on the plan application)
        // (with two per CU the charge applies to a single workgroup only: a third one running alone at the
        // end measured cheaper than the coarser split that avoids it, n = m = 10000, d = 64: 0.46 against 0.49 ms)
        const int64_t rem = (w < wg_per_cu || wg_per_cu >= 3) ? w % wg_per_cu : 0;
        const double units = (double)(w - rem) + (double)rem * (rem == 1 ? 1.4 : 1.08);
        const double cost = units * ((double)tps + startup) + 0.02 * eff;
        if (sp == 1 || cost < best * 0.995) {
            best = cost;
            best_tps = tps;
        }
    }
    s.splits = (int)ceil_div(n_tiles, best_tps);
    s.cols_per_split = (int64_t)best_tps * bc;
    return s;
}

}  // namespace

// arguments and launch shape of an LSE pass (res resident, str streamed) writing its records to `partial`
static fs_status lse_pass_args(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, void *partial,
                               PassArgs *out, PassShape *shape)
{
    const PassShape s = shape_f64(c, res->cnt, str->cnt, 16 * kLseJT, 16 * kLseNW, P->d, kLseWgPerCu);
    constexpr int BC = 16 * kLseNW;
    PassArgs a{};
    a.res = res->pts_d;
    a.str = str->pts_d;
    a.bias = str->bias_d;
    a.kp = P->kp;
    a.kc = (int)round_up(P->d, 8);
    a.cscale = 2.0 * kLog2e / eps;
    a.n_tiles = (int)ceil_div(str->cnt, BC);
    a.tiles_per_split = (int)(s.cols_per_split / BC);
    a.partial = (double2 *)partial;
    a.partial_stride = res->cnt_pad;
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)a.n_tiles * BC > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp % KC) != 0 || a.kc > a.kp)
        return fail(c, FS_ERR_DEVICE, "internal: fp64 launch shape exceeds the padded buffers");
    *out = a;
    *shape = s;
    return FS_OK;
}

fs_status f64_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out, int prof_kind)
{
    PassArgs a;
    PassShape s;
    fs_status st = lse_pass_args(c, P, res, str, eps, P->partial, &a, &s);
    if (st != FS_OK) return st;
    prof_begin(c, (double)res->cnt * (double)str->cnt, prof_kind);
    const dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
    if (P->path == Path::LowD)
        hipLaunchKernelGGL((k_pass_f64<false, false, 4, kLseJT, kLseNW, true>), grid, dim3(64 * kLseNW), 0, c->stream, a);
    else
        hipLaunchKernelGGL((k_pass_f64<false, false, 4, kLseJT, kLseNW, false>), grid, dim3(64 * kLseNW), 0, c->stream, a);
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = s.splits;
    return FS_OK;
}

// The f-pass (records to partial_x) and the g-pass (records to partial_y) of one iteration of the averaged
// schedule (Eq. 4-5) in ONE launch.
fs_status f64_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x, int *splits_y)
{
    PassArgs ax, ay;
    PassShape sx, sy;
    fs_status st;
    if ((st = lse_pass_args(c, P, &P->X, &P->Y, eps, partial_x, &ax, &sx)) != FS_OK) return st;
    if ((st = lse_pass_args(c, P, &P->Y, &P->X, eps, partial_y, &ay, &sy)) != FS_OK) return st;
    const dim3 grid((unsigned)(sx.row_blocks + sy.row_blocks), (unsigned)(sx.splits > sy.splits ? sx.splits : sy.splits));
    prof_begin(c, 2.0 * (double)P->X.cnt * (double)P->Y.cnt, P->path == Path::LowD ? 1 : 0);
    if (P->path == Path::LowD)
        hipLaunchKernelGGL((k_pass_f64_pair<kLseJT, kLseNW, true>), grid, dim3(64 * kLseNW), 0, c->stream, ax, ay, sx.row_blocks,
                           sx.splits, sy.splits);
    else
        hipLaunchKernelGGL((k_pass_f64_pair<kLseJT, kLseNW, false>), grid, dim3(64 * kLseNW), 0, c->stream, ax, ay, sx.row_blocks,
                           sx.splits, sy.splits);
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_x = sx.splits;
    *splits_y = sy.splits;
    return FS_OK;
}

constexpr int kWidePCH = 128;   // value columns of a pass of the wide form

size_t f64_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t d, int64_t p)
{
    (void)p;
    // the larger of the shapes of the plain and of the Hadamard-weighted / wide application, at the wide row length
    const PassShape s1 = shape_f64(c, n_res, n_str, 16 * kApplyJT, 16 * kApplyNW, d, kApplyWgPerCu);
    const PassShape s2 = shape_f64(c, n_res, n_str, 16 * kApplyJT, 16 * kApplyNW, d, 2);
    return (size_t)(s1.splits > s2.splits ? s1.splits : s2.splits) * (size_t)round_up(n_res, 1024) * kWidePCH * 4;
}

fs_status f64_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V,
                    int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out, const float *hadA, int64_t lda)
{
    constexpr int BC = 16 * kApplyNW;
    PassArgs a{};
    a.res = res->pts_d;
    a.str = str->pts_d;
    a.bias = str->bias_d;
    a.kp = P->kp;
    a.kc = (int)round_up(P->d, 8);
    a.cscale = 2.0 * kLog2e / eps;
    a.n_tiles = (int)ceil_div(str->cnt, BC);
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
    for (int p0 = 0; p0 < p;) {
        a.p0 = p0;
        // more than 64 columns left: a wide pass (128 columns) -- every pass repeats the score contraction
        const bool wide = !hadA && p - p0 > PCH;
        const int width = wide ? kWidePCH : PCH;
        const int cols = (int)(p - p0 < width ? p - p0 : width);
        const int nct = (int)ceil_div(cols, 16);
        const PassShape s = shape_f64(c, res->cnt, str->cnt, 16 * kApplyJT, BC, P->d, (hadA || wide) ? 2 : kApplyWgPerCu);
        a.tiles_per_split = (int)(s.cols_per_split / BC);
        if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)a.n_tiles * BC > str->cnt_pad ||
            (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp % KC) != 0 || a.kc > a.kp ||
            (size_t)s.splits * res->cnt_pad * width * 4 > P->extra_bytes)
            return fail(c, FS_ERR_DEVICE, "internal: fp64 apply launch shape exceeds the padded buffers");
        const dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
#define FS_F64_APPLY(H, N) hipLaunchKernelGGL((k_pass_f64<true, H, N, kApplyJT, kApplyNW>), grid, dim3(64 * kApplyNW), 0, c->stream, a)
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
            case 4: FS_F64_APPLY(false, 4); break;
            case 5: FS_F64_APPLY(false, 5); break;
            case 6: FS_F64_APPLY(false, 6); break;
            case 7: FS_F64_APPLY(false, 7); break;
            default: FS_F64_APPLY(false, 8); break;
            }
        }
#undef FS_F64_APPLY
        fs_status st = launch_apply_finalize(c, P, res, res->norm, s.splits, eps, a.opart, width, p0, (int)p, out, ldo,
                                             mass_out);
        if (st != FS_OK) return st;
        p0 += width;
    }
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
