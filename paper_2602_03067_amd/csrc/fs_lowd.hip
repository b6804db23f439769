// Low-dimension (d <= 16) streaming passes.
//
// The pass is bound by the exp2 rate of the vector ALU (one quarter-rate v_exp_f32 per pair), so
// everything else is kept off that ALU as far as possible:
//  * fp32-accuracy half-steps (k_lse_lowd_split) form the scores on the bf16 matrix cores from
//    operands split into three bf16 pieces; the vector ALU does one exp2 and one add per pair;
//  * float64-score half-steps and the plan application (k_lse_lowd<double>, k_apply_lowd) run on
//    the vector ALU: every lane owns R resident rows (pre-scaled coordinates and the running
//    (max, sum) in registers, so the row reduction never crosses lanes); the streamed points are
//    staged in LDS in tiles of 256, packed as (coord_0..coord_{d-1}, bias), so that one broadcast
//    LDS read serves all 64 lanes of a wave and all R rows of a lane.
//
// Scores are in base 2:  s_ij = (2 log2e / eps) <x_i, y_j> + bias_j  (Alg. 1, line "score tile
// + bias", times log2 e), so exp and log are single v_exp_f32 / v_log_f32 instructions.
// The online LSE of Alg. 1 is applied per chunk of streamed points; the running max is kept
// integer-valued, so every rescale factor is an exact power of two.
//
// Score precision: fp32 when (log2e/eps) * max|x|^2 is small enough for fp32 scores to hold the
// 1e-4 target, float64 otherwise (a score of magnitude 500 has an fp32 ulp of 6e-5).
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

// ---- fp32-accurate scores on the bf16 matrix cores ("split" records) -------------------------
// On the vector ALU the d FMAs of a score cost as much as its exp2.  The fp32 matrix instructions
// do not help: measured, their time adds to the vector ALU's (a K = 4 fp32 MFMA variant of this
// pass gained 10 %).  The bf16 ones are 16 times faster and take only ~13 cycles of vector issue
// each.  With the operands split into three bf16 pieces (see split_ksteps), KS = (8 d + 6)/16
// rounded up MFMA 32x32x16 per 32 x 32 pairs (two for d = 3) deliver score - max at fp32 accuracy,
// and the vector ALU is left with one exp2 and one add per pair.
// A = 32 streamed points (lane l: point l%32, slots 8(l/32)..+7 of the K-step), B = 32 resident
// rows, so a lane's 16 result registers are 16 streamed points of ONE resident row (l%32); the two
// lane halves of a row are merged once at the end.  The running max sits in the operand B itself
// (three slots against ones in A), so the lazy stabiliser costs nothing in the common path: when a
// chunk sum leaves [0, 2^60), the wave zeroes those slots, recomputes the chunk's raw scores,
// lifts the integer max, writes it back into B and takes the chunk's sums again.
typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf2 __attribute__((ext_vector_type(2)));
typedef float f16v __attribute__((ext_vector_type(16)));

//
// PRECISE = true is the variant for half-steps that need better than fp32 scores (d <= 3): the
// operands come from the float64 copies, and the leading part of every term is put on a fixed
// grid so that the large, mutually cancelling contributions are summed EXACTLY:
//   c x_k = X1 + rx, X1 a multiple of gx = 2^(Ex-7) (|X1| <= 2^Ex), y_k = Y1 + ry likewise with gy,
//   bias = (Ba + Bb + Bc) + rb with three 8-bit digits on the grid q = gx gy, max = integer >= q.
// K-step 0 holds X1 Y1 (three slots), the bias digits against ones and the max pieces against
// ones: all multiples of q inside a 2^24 q window, so the MFMA's aligned adder loses nothing, and
// their sum is already within ~2^-6 of the largest term's size of the final score - max.  K-steps 1
// and 2 add the residual products X1 ry, rx Y1, rx ry (residuals in three bf16 pieces) and rb, whose
// fp32 accumulation error is relative to that small size.  Measured: error of score - max below
// 2 ulp of the result for |score| up to 3e4 (an fp32 chain is off by 3.5e-3 there).
struct SplitArgs {
    const void *res;        // resident side: packed floats [.][dp] (fp32 variant) or doubles [.][dp] (precise)
    const uint16_t *str;    // streamed side: split records
    double cscale;          // 2 log2e / eps
    double gx;              // precise: grid of the leading digit of c x
    int d, dp;
    int tiles_per_split, n_tiles;
    int row_blocks, splits;  // extent of this pass in the grid
    double2 *partial;
    int64_t partial_stride;
    // plan application (PC > 0): value matrix [n_str][ldv], its columns p0 .. p0+PC-1 of p, and the
    // [splits][partial_stride][PC] accumulators
    const float *V;
    int64_t ldv, n_str;
    int p0, p;
    float *opart;
    const unsigned char *vimg;   // PC == 8: value images of the streamed tiles (see k_vimg_lowd)
};

// one workgroup of the pass: row block bx, column split by.
// PC > 0 makes it the plan application (Alg. 2 / Alg. 4) for PC value columns, in one of two forms.
// PC == 4: every exponential also multiplies the value row of its streamed point, which all lanes of a
// half-wave share (a lane's registers are streamed points, its lane index the resident row), so the
// value row comes as one broadcast LDS read per exponential and the products stay on the vector ALU
// in fp32: 4 FMAs and an LDS read per exponential.
// PC == 8: the products go to the matrix cores as well.  The sixteen exponentials of a lane ARE the B
// operand of an MFMA whose contraction runs over the streamed points (k-step 0 = registers 0..7,
// k-step 1 = registers 8..15), once split into a bf16 head (E rounded) and a bf16 tail (E - head, exact
// in fp32, then rounded: E is kept to 2^-17, the size of the error that fp32 scores of a few hundred
// base-2 units leave in E anyway).  The A operand is an image of the tile's
// value rows in the matching order, 32 rows = 8 columns x (three bf16 pieces of the value, exact to
// 24 bits, + a spare row, the first of which holds ones and so yields the row sum):
//     O[c'][j] += sum_i A2[c'][i] (Eh[i][j] + El[i][j]),   c' = 8 (col / 2) + 4 (col % 2) + piece,
// so in the accumulator layout lane half h of resident row j ends up with columns h, 2 + h, 4 + h, 6 + h
// in its registers 4 q + piece, and half 0 with the row sum in register 3.  Per 32 x 32 pairs that
// is 48 simple vector instructions and 4 MFMAs instead of 64 FMAs and 16 LDS reads, for twice the columns.
template <int KS, int R, int TJ, int CH, bool PRECISE, int PC = 0, int PCU = PC>
__device__ __forceinline__ void lse_split_body(const SplitArgs &a, const int bx, const int by)
{
    // PCU <= PC: value columns actually wanted (the others are not multiplied; zeros are stored for them)
    constexpr bool APPLY = PC > 0;
    constexpr bool MM = PC == 8 || PC == 16;   // products on the matrix cores
    // PC == 16: fifteen columns with TWO bf16 pieces per value (values to 2^-17, like the exponentials): rows
    // 2 col + piece, row 30 the ones, so the row sum lands in register 14 of lane half 1
    constexpr bool V2 = PC == 16;
    static_assert(PC == 0 || PC == 4 || PC == 8 || PC == 16, "one float4 of values per streamed point, or an image of 8 / 15 columns");
    constexpr int VBYTES = MM ? (TJ / 32) * 2048 : (APPLY ? TJ * PC * 4 : 16);   // values of a tile in LDS
    __shared__ __attribute__((aligned(1024))) unsigned char vbuf[APPLY ? 2 : 1][VBYTES];
    constexpr int NP = 2 * KS;               // 16-byte pieces per record
    constexpr int UPT = TJ * NP / kBlock;    // pieces each thread moves per tile
    constexpr int NG = TJ / 32;              // groups of 32 streamed points per tile
    static_assert(TJ * NP % kBlock == 0 && NG % CH == 0, "tile shape");
    static_assert(!PRECISE || KS == 3, "the precise record has three K-steps");
    __shared__ Unit tile[2][TJ * NP];

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63;
    const int lj = l & 31, lh = l >> 5;
    const int d = a.d;
    const int tiles_per_split = a.tiles_per_split, n_tiles = a.n_tiles;
    double2 *__restrict__ partial = a.partial;
    const int64_t partial_stride = a.partial_stride;
    const uint16_t *__restrict__ str = a.str;
    const int64_t row0 = (int64_t)bx * (128 * R) + w * (32 * R);
    // the piece with the ones and the max slots: piece d = 2 (KS-1) + (d & 1) in the fp32 record,
    // piece 1 in the precise one
    constexpr int MK = PRECISE ? 0 : KS - 1;
    const bool holds_max = PRECISE ? (lh == 1) : (lh == (d & 1));
    auto lds_pos = [](int point, int piece) { return point * NP + split_piece_pos(KS, point, piece); };

    bf8 b[R][KS];
    float mrun[R], srun[R], stile[R];
    float orun[APPLY && !MM ? R : 1][APPLY && !MM ? PC : 1], otile[APPLY && !MM ? R : 1][APPLY && !MM ? PC : 1];
    f16v omm[MM ? R : 1];   // PC == 8: running outputs in the accumulator layout
    if constexpr (APPLY && !MM) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int c = 0; c < PC; ++c) orun[r][c] = otile[r][c] = 0.0f;
    }
    if constexpr (MM) {
#pragma unroll
        for (int r = 0; r < R; ++r)
#pragma unroll
            for (int e = 0; e < 16; ++e) omm[r][e] = 0.0f;
    }
    auto set_max = [&](int r, float neg_m) {   // slots 3..5 of that piece <- pieces of -max
        __bf16 q[3];
        split3(neg_m, q);
        if (holds_max) {
            b[r][MK][3] = q[0];
            b[r][MK][4] = q[1];
            b[r][MK][5] = q[2];
        }
    };
    const int t_begin = by * tiles_per_split;
    const int t_end = min(n_tiles, t_begin + tiles_per_split);
    const Unit *gsrc = reinterpret_cast<const Unit *>(str);

    // a tile is a linear 16 KS TJ / 8 byte copy, moved by direct global -> LDS loads (no registers)
    const unsigned tile_off = (unsigned)(size_t)&tile[0][0];
    const unsigned vtile_off = (unsigned)(size_t)&vbuf[0][0];
    auto fetch = [&](int t, int bufi) {
        // each wave brings UPT consecutive KB of the tile, in runs of up to four loads behind one write of the LDS
        // base to m0 (immediate offsets advance the memory and the LDS address alike; a write to m0 waits for the
        // wave's earlier direct loads to leave for the address unit)
        const Unit *src = gsrc + (int64_t)t * (TJ * NP) + (w * UPT) * 64 + l;
        const unsigned dst = tile_off + (bufi * (TJ * NP) + (w * UPT) * 64) * 16;
#pragma unroll
        for (int q = 0; q < UPT; ++q) {
            if (q % 4 == 0) {
                const unsigned m = __builtin_amdgcn_readfirstlane(dst + q * 1024);
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(m) : "memory", "m0");
            }
            asm volatile("global_load_lds_dwordx4 %0, off offset:%1" ::"v"(src + (q / 4) * 256), "n"((q % 4) * 1024) : "memory");
        }
        if constexpr (MM) {
            // the tile's value image: VBYTES / 1024 consecutive KB, this wave's share as one run
            constexpr int VPW = VBYTES / 1024 / 4;
            static_assert(VBYTES % 4096 == 0 && VPW <= 4, "a run of at most four loads per wave");
            const unsigned char *vsrc = a.vimg + (int64_t)t * VBYTES + (w * VPW) * 1024 + l * 16;
            const unsigned m = __builtin_amdgcn_readfirstlane(vtile_off + bufi * VBYTES + (w * VPW) * 1024);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0" ::"s"(m) : "memory", "m0");
#pragma unroll
            for (int q = 0; q < VPW; ++q) asm volatile("global_load_lds_dwordx4 %0, off offset:%1" ::"v"(vsrc), "n"(q * 1024) : "memory");
        } else if constexpr (APPLY) {
            // value rows of the tile, one dword per lane; entries outside the matrix are read from a
            // valid address instead (their exponentials are zero / their columns are not stored)
#pragma unroll
            for (int q = 0; q < TJ * PC / kBlock; ++q) {
                const int e = q * kBlock + tid;
                const int64_t j = (int64_t)t * TJ + e / PC;
                const int cc = a.p0 + e % PC;
                const float *src = a.V + (j < a.n_str ? j : 0) * a.ldv + (cc < a.p ? cc : a.p0);
                dma4(src, vtile_off + (bufi * (TJ * PC) + q * kBlock + w * 64) * 4);
            }
        }
    };
    // the first tile is on its way while the resident operands are built
    if (t_begin < t_end) fetch(t_begin, 0);

    const __bf16 one = (__bf16)1.0f, zero = (__bf16)0.0f;
#pragma unroll
    for (int r = 0; r < R; ++r) {
        if constexpr (!PRECISE) {
            const float *px = static_cast<const float *>(a.res) + (row0 + 32 * r + lj) * a.dp;
            const float cscale = (float)a.cscale;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int c = 2 * ks + lh;
                __bf16 x[3];
                split3(c < d ? px[c] * cscale : 0.0f, x);
                bf8 v = {x[0], x[0], x[1], x[0], x[1], x[2], x[1], x[2]};
                if (c == d) v = bf8{one, one, one, zero, zero, zero, zero, zero};
                b[r][ks] = v;
            }
        } else {
            const double *px = static_cast<const double *>(a.res) + (row0 + 32 * r + lj) * a.dp;
            __bf16 X1[3], rx[3][3];
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const double cx = c < d ? px[c] * a.cscale : 0.0;
                const double x1 = rint(cx / a.gx) * a.gx;
                X1[c] = (__bf16)(float)x1;
                split3d(cx - x1, rx[c]);
            }
            // pieces 0..5 (piece = 2 ks + lh); see split_precise_record for the streamed counterparts
            const bf8 p0 = {X1[0], X1[1], X1[2], zero, zero, zero, zero, zero};
            const bf8 p1 = {one, one, one, zero, zero, zero, zero, zero};
            const bf8 p5 = {one, one, one, zero, zero, rx[0][1], rx[1][1], rx[2][1]};
            bf8 pc[3];
#pragma unroll
            for (int c = 0; c < 3; ++c) pc[c] = bf8{X1[c], X1[c], X1[c], rx[c][0], rx[c][1], rx[c][2], rx[c][0], rx[c][0]};
            b[r][0] = lh ? p1 : p0;
            b[r][1] = lh ? pc[1] : pc[0];
            b[r][2] = lh ? p5 : pc[2];
        }
        mrun[r] = kNegInit;
        srun[r] = 0.0f;
        stile[r] = 0.0f;
        set_max(r, -kNegInit);
    }

    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();

    auto load_a = [&](const Unit *tl, int grp, bf8(&av)[KS]) {
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) av[ks] = *reinterpret_cast<const bf8 *>(tl + lds_pos(grp * 32 + lj, 2 * ks + lh));
    };
    auto scores = [&](const bf8(&av)[KS], f16v(&dd)[R]) {
#pragma unroll
        for (int r = 0; r < R; ++r) {
            f16v z;
#pragma unroll
            for (int e = 0; e < 16; ++e) z[e] = 0.0f;
            dd[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0], b[r][0], z, 0, 0, 0);
#pragma unroll
            for (int ks = 1; ks < KS; ++ks) dd[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[ks], b[r][ks], dd[r], 0, 0, 0);
        }
    };
    // Sums of exp2(score - max) over one chunk of CH x 32 streamed points.  The chunk is a pipeline
    // of CH x R steps (32 streamed points x 32 resident rows each): while the vector ALU takes the
    // exponentials of step s, the matrix pipe computes step s + 1, its KS instructions spread evenly
    // between them.  (Instructions of one wave overlap across the two pipes only if they alternate
    // at this grain; a wave that issues its MFMAs back to back stalls the vector ALU.)
    auto chunk_sums = [&](const Unit *tl, const float *vt, int c0, float(&csum)[R], float(&co)[APPLY ? R : 1][APPLY ? PC : 1]) {
        constexpr int NS = CH * R;
        bf8 av[2][KS];
        f16v dd[2];
        f16v z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.0f;
        load_a(tl, c0, av[0]);
        if (CH > 1 && R == 1) load_a(tl, c0 + 1, av[1]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            dd[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0][ks], b[0][ks], ks == 0 ? z : dd[0], 0, 0, 0);
#pragma unroll
        for (int st = 0; st < NS; ++st) {
            const int g = st / R, r = st % R;
            const int sn = st + 1, gn = sn / R, rn = sn % R;
            // request the A operands of a later group into the buffer whose group is fully produced
            if (R == 1) {
                if (g + 2 < CH) load_a(tl, c0 + g + 2, av[g & 1]);
            } else if (r == 0 && g + 1 < CH) {
                load_a(tl, c0 + g + 1, av[(g + 1) & 1]);
            }
            float acc = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                if (sn < NS)
                    dd[sn & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[gn & 1][ks], b[rn][ks], ks == 0 ? z : dd[sn & 1], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
                const int e0 = 16 * ks / KS, e1 = 16 * (ks + 1) / KS;
                float part = 0.0f;
#pragma unroll
                for (int e = e0; e < e1; ++e) {
                    const float ev = fast_exp2(dd[st & 1][e]);
                    part = e == e0 ? ev : part + ev;
                    if constexpr (APPLY) {
                        // register e of lane half lh is streamed point 8 (e / 4) + 4 lh + e % 4 of group c0 + g
                        const float4 vv = *reinterpret_cast<const float4 *>(vt + (32 * (c0 + g) + 8 * (e >> 2) + 4 * lh + (e & 3)) * PC);
                        const float vcol[4] = {vv.x, vv.y, vv.z, vv.w};
#pragma unroll
                        for (int c = 0; c < PC; ++c) {
                            if (c >= PCU)
                                co[r][c] = 0.0f;
                            else if (g == 0 && e == 0)
                                co[r][c] = ev * vcol[c];
                            else
                                co[r][c] = fmaf(ev, vcol[c], co[r][c]);
                        }
                    }
                }
                acc = ks == 0 ? part : acc + part;
                __builtin_amdgcn_sched_barrier(0);
            }
            csum[r] = g == 0 ? acc : csum[r] + acc;
        }
    };

    // PC == 8: the same pipeline with the products on the matrix cores.  dch[r] receives, for the chunk alone,
    // sum_i A2[c'][i] E[i][j]; the four product MFMAs of a step (two k-steps x head/tail) are issued between
    // the exponentials of the NEXT step, like the score MFMAs, so that the two pipes alternate.
    auto load_va = [&](const unsigned char *vi, int grp, bf8(&va)[2]) {
#pragma unroll
        for (int k2 = 0; k2 < 2; ++k2) va[k2] = *reinterpret_cast<const bf8 *>(vi + ((((grp * 2 + k2) * 2 + lh) * 32 + lj) << 4));
    };
    // the pairs (-1, 0) and (0, -1) in bf16, held in vector registers (written as constants the compiler turns them
    // into inline operands, which this instruction does not read as a bf16 pair)
    uint32_t ksel0 = 0x0000bf80u, ksel1 = 0xbf800000u;
    if constexpr (MM) {
        asm("v_mov_b32 %0, 0xbf80" : "=v"(ksel0));
        asm("v_mov_b32 %0, 0xbf800000" : "=v"(ksel1));
    }
    auto chunk_mm = [&](const Unit *tl, const unsigned char *vi, int c0, f16v(&dch)[MM ? R : 1]) {
        constexpr int NS = CH * R;
        bf8 av[2][KS], va[2][2];
        bf8 eh[2], el[2];   // heads and tails of the previous step's exponentials, per k-step
        f16v dd[2];
        f16v z;
#pragma unroll
        for (int e = 0; e < 16; ++e) z[e] = 0.0f;
        load_a(tl, c0, av[0]);
        if (CH > 1 && R == 1) load_a(tl, c0 + 1, av[1]);
        load_va(vi, c0, va[0]);
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            dd[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[0][ks], b[0][ks], ks == 0 ? z : dd[0], 0, 0, 0);
#pragma unroll
        for (int st = 0; st <= NS; ++st) {
            const int g = st / R, r = st % R;
            const int sn = st + 1, gn = sn / R, rn = sn % R;
            const int pst = st > 0 ? st - 1 : 0;
            const int pg = pst / R, pr = pst % R;   // the step whose products are pending
            if (st < NS) {
                if (R == 1) {
                    if (g + 2 < CH) load_a(tl, c0 + g + 2, av[g & 1]);
                } else if (r == 0 && g + 1 < CH) {
                    load_a(tl, c0 + g + 1, av[(g + 1) & 1]);
                }
            }
            // four quarters, each: one pending product MFMA, its share of the next step's score MFMAs, four
            // exponentials (consecutive MFMAs into one accumulator are a dependent chain: the exponentials between
            // them cover its latency)
            float ev[16];
#pragma unroll
            for (int qd = 0; qd < 4; ++qd) {
                if (st > 0)
                    dch[pr] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(va[pg & 1][qd >> 1], (qd & 1) ? el[qd >> 1] : eh[qd >> 1],
                                                                      (pg == 0 && qd == 0) ? z : dch[pr], 0, 0, 0);
                if (sn < NS) {
#pragma unroll
                    for (int ks = 0; ks < KS; ++ks)
                        if (ks * 4 / KS == qd)
                            dd[sn & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[gn & 1][ks], b[rn][ks], ks == 0 ? z : dd[sn & 1], 0, 0, 0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (st < NS) {
#pragma unroll
                    for (int e = 4 * qd; e < 4 * qd + 4; ++e) ev[e] = fast_exp2(dd[st & 1][e]);
                }
                __builtin_amdgcn_sched_barrier(0);
            }
            if (st < NS) {
                // the value image of the next group, once the pending products of the group before it are issued
                if (r == 0 && g + 1 < CH) load_va(vi, c0 + g + 1, va[(g + 1) & 1]);
#pragma unroll
                for (int k2 = 0; k2 < 2; ++k2) {
                    uint32_t hp[4];
#pragma unroll
                    for (int q = 0; q < 8; q += 2) {
                        // heads: the two exponentials rounded to bf16, packed; tails: what the heads leave, rounded
                        const float x0 = ev[8 * k2 + q], x1 = ev[8 * k2 + q + 1];
                        const bf2 hd = {(__bf16)x0, (__bf16)x1};
                        const uint32_t pk = __builtin_bit_cast(uint32_t, hd);
                        hp[q >> 1] = pk;
                        // x - head in one instruction each: the bf16 dot product of the packed heads with (-1, 0) or
                        // (0, -1), accumulated onto x (products and sum are exact here)
                        el[k2][q] = (__bf16)__builtin_amdgcn_fdot2_f32_bf16(hd, __builtin_bit_cast(bf2, ksel0), x0, false);
                        el[k2][q + 1] = (__bf16)__builtin_amdgcn_fdot2_f32_bf16(hd, __builtin_bit_cast(bf2, ksel1), x1, false);
                    }
                    const uint4 u = make_uint4(hp[0], hp[1], hp[2], hp[3]);
                    eh[k2] = __builtin_bit_cast(bf8, u);
                }
            }
        }
    };

    int buf = 0;
    for (int t = t_begin; t < t_end; ++t) {
        if (t + 1 < t_end) fetch(t + 1, buf ^ 1);   // that buffer was last read before the previous barrier
        const Unit *tl = tile[buf];
        const float *vt = reinterpret_cast<const float *>(vbuf[APPLY ? buf : 0]);
        const unsigned char *vi = vbuf[APPLY ? buf : 0];
#pragma unroll 1
        for (int c0 = 0; c0 < NG; c0 += CH) {
            float csum[R];
            float co[APPLY && !MM ? R : 1][APPLY && !MM ? PC : 1];
            f16v dch[MM ? R : 1];
            if constexpr (MM) {
                chunk_mm(tl, vi, c0, dch);
                // (the row sum of the chunk sits in register 3 of lane half 0; the other half has a zero row there.
                // With two pieces per value: register 14 of lane half 1, and a product row in the other half)
#pragma unroll
                for (int r = 0; r < R; ++r) csum[r] = V2 ? (lh == 1 ? dch[r][14] : 0.0f) : dch[r][3];
            } else {
                chunk_sums(tl, vt, c0, csum, co);
            }
            if constexpr (APPLY && !MM) {
                // pin the products to this point: left alone, the compiler sinks all of them behind the
                // branch below (they are only needed when the chunk is accepted) and keeps 64
                // exponentials and 64 value rows alive for that, in scratch memory
#pragma unroll
                for (int r = 0; r < R; ++r)
#pragma unroll
                    for (int c = 0; c < PC; ++c) asm volatile("" ::"v"(co[r][c]));
            }
            bool bad = false;
#pragma unroll
            for (int r = 0; r < R; ++r) bad = bad || !(csum[r] < kLazyMax);
            if (__any(bad)) {
                float mx[R];
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    mx[r] = kNegInit;
                    set_max(r, 0.0f);
                }
#pragma unroll
                for (int g = 0; g < CH; ++g) {
                    bf8 av[KS];
                    f16v dd[R];
                    load_a(tl, c0 + g, av);
                    scores(av, dd);
#pragma unroll
                    for (int r = 0; r < R; ++r)
#pragma unroll
                        for (int e = 0; e < 16; ++e) mx[r] = fmaxf(mx[r], dd[r][e]);
                }
#pragma unroll
                for (int r = 0; r < R; ++r) {
                    // the max of a row sits once in B and serves both lane halves: lift it for both
                    const float mrow = fmaxf(mx[r], __shfl_xor(mx[r], 32));
                    const float mnew = fmaxf(mrun[r], ceilf(mrow));
                    const float scale = fast_exp2(mrun[r] - mnew);
                    srun[r] *= scale;
                    stile[r] *= scale;
                    if constexpr (APPLY && !MM) {
#pragma unroll
                        for (int c = 0; c < PC; ++c) {
                            orun[r][c] *= scale;
                            otile[r][c] *= scale;
                        }
                    }
                    if constexpr (MM) {
#pragma unroll
                        for (int e = 0; e < 16; ++e) omm[r][e] *= scale;
                    }
                    mrun[r] = mnew;
                    set_max(r, -mnew);
                }
                // all exponents are <= 0 now: no second check
                if constexpr (MM)
                    chunk_mm(tl, vi, c0, dch);
                else
                    chunk_sums(tl, vt, c0, csum, co);
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {
                if constexpr (MM) {
#pragma unroll
                    for (int e = 0; e < 16; ++e) omm[r][e] += dch[r][e];
                } else {
                    stile[r] += csum[r];
                }
                if constexpr (APPLY && !MM) {
#pragma unroll
                    for (int c = 0; c < PC; ++c) otile[r][c] += co[r][c];
                }
            }
        }
#pragma unroll
        for (int r = 0; r < R; ++r) {
            srun[r] += stile[r];
            stile[r] = 0.0f;
            if constexpr (APPLY && !MM) {
#pragma unroll
                for (int c = 0; c < PC; ++c) {
                    orun[r][c] += otile[r][c];
                    otile[r][c] = 0.0f;
                }
            }
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this wave's part of the next tile has landed
        __syncthreads();
        buf ^= 1;
    }

    if constexpr (MM) {
        // the second contraction has already summed over both lane halves' streamed points; the max of a row is
        // common to its two lanes
#pragma unroll
        for (int r = 0; r < R; ++r) {
            const int64_t row = row0 + 32 * r + lj;
            if constexpr (V2) {
                if (lh == 1) partial[(int64_t)by * partial_stride + row] = make_double2((double)mrun[r], (double)omm[r][14]);
                // rows 8 q + 4 h + s of this lane half: columns 4 q + 2 h and 4 q + 2 h + 1 (column 15 does not exist)
                float *o = a.opart + ((int64_t)by * partial_stride + row) * PC + 2 * lh;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    o[4 * q] = omm[r][4 * q] + omm[r][4 * q + 1];
                    o[4 * q + 1] = (q == 3 && lh == 1) ? 0.0f : omm[r][4 * q + 2] + omm[r][4 * q + 3];
                }
            } else {
                if (lh == 0) partial[(int64_t)by * partial_stride + row] = make_double2((double)mrun[r], (double)omm[r][3]);
                float *o = a.opart + ((int64_t)by * partial_stride + row) * PC + lh;
#pragma unroll
                for (int q = 0; q < 4; ++q) o[2 * q] = (omm[r][4 * q] + omm[r][4 * q + 1]) + omm[r][4 * q + 2];
            }
        }
        return;
    }
    // merge the two lane halves (streamed points 8q+4h .. of every 32) of each resident row
#pragma unroll
    for (int r = 0; r < R; ++r) {
        const float m = mrun[r], sv = srun[r];
        const float mo = __shfl_xor(m, 32), so = __shfl_xor(sv, 32);
        const float M = fmaxf(m, mo);
        const float S = sv * fast_exp2(m - M) + so * fast_exp2(mo - M);
        if (lh == 0) partial[(int64_t)by * partial_stride + row0 + 32 * r + lj] = make_double2((double)M, (double)S);
        if constexpr (APPLY && !MM) {
            float4 o;
            o.x = orun[r][0] * fast_exp2(m - M) + __shfl_xor(orun[r][0], 32) * fast_exp2(mo - M);
            o.y = orun[r][1] * fast_exp2(m - M) + __shfl_xor(orun[r][1], 32) * fast_exp2(mo - M);
            o.z = orun[r][2] * fast_exp2(m - M) + __shfl_xor(orun[r][2], 32) * fast_exp2(mo - M);
            o.w = orun[r][3] * fast_exp2(m - M) + __shfl_xor(orun[r][3], 32) * fast_exp2(mo - M);
            if (lh == 0)
                *reinterpret_cast<float4 *>(a.opart + ((int64_t)by * partial_stride + row0 + 32 * r + lj) * PC) = o;
        }
    }
}

template <int KS, int R, int TJ, int CH, bool PRECISE>
__global__ __launch_bounds__(kBlock, 2) void k_lse_lowd_split(SplitArgs a)
{
    lse_split_body<KS, R, TJ, CH, PRECISE>(a, blockIdx.x, blockIdx.y);
}

// plan application on the split records (PC value columns per launch)
template <int KS, int R, int TJ, int CH, bool PRECISE, int PC, int PCU>
__global__ __launch_bounds__(kBlock, 2) void k_apply_lowd_split(SplitArgs a)
{
    lse_split_body<KS, R, TJ, CH, PRECISE, PC, PCU>(a, blockIdx.x, blockIdx.y);
}

// Both half-steps of one iteration of the averaged schedule (Eq. 4-5) in one launch: they read the
// same old potentials, so the row blocks of the f-pass (a0) and of the g-pass (a1) share a grid;
// grid.y covers the larger of the two split counts.
template <int KS, int R, int TJ, int CH, bool PRECISE>
__global__ __launch_bounds__(kBlock, 2) void k_lse_lowd_split_pair(SplitArgs a0, SplitArgs a1)
{
    const bool second = (int)blockIdx.x >= a0.row_blocks;   // uniform over the workgroup
    const SplitArgs &a = second ? a1 : a0;
    if ((int)blockIdx.y >= a.splits) return;
    lse_split_body<KS, R, TJ, CH, PRECISE>(a, (int)blockIdx.x - (second ? a0.row_blocks : 0), blockIdx.y);
}

// ---- plan application (Alg. 2 / Alg. 4): the same pass with a value accumulator ----------
// Every lane owns ONE resident row and PC columns of the output; the streamed tile carries
// the PC values of each streamed point next to its coordinates.
// HAD = true is the Hadamard-weighted transport of Alg. 5, (P o (A Yc^T)) V: every plan entry is
// multiplied by <A_i, yc_j> with A_i the resident row of a second matrix and yc_j the streamed
// point as stored (centred at the common mean; the caller adds the mean's share).
template <typename S, int D, int PC, bool HAD>
__global__ __launch_bounds__(kBlock) void k_apply_lowd(const S *__restrict__ res, const S *__restrict__ str,
                                                       const float *__restrict__ V, int64_t ldv, int p0, int p,
                                                       int64_t n_str, S cscale, int tiles_per_split, int n_tiles,
                                                       double2 *__restrict__ partial, int64_t partial_stride,
                                                       float *__restrict__ opart, int64_t opart_stride,
                                                       const float *__restrict__ had_A, int64_t lda, int64_t n_res)
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
    float ar[HAD ? D : 1];
    if constexpr (HAD) {
#pragma unroll
        for (int k = 0; k < D; ++k) ar[k] = row < n_res ? had_A[row * lda + k] : 0.0f;
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
            float wv[HAD ? kT : 1];
#pragma unroll
            for (int c = 0; c < kT; ++c) {
                S yv[DP];
                unpack<S, DP>(tile + (j + c) * Q, yv);
                S acc = yv[D];
#pragma unroll
                for (int k = 0; k < D; ++k) acc = xs[k] * yv[k] + acc;
                sc[c] = acc;
                if constexpr (HAD) {
                    float wsum = 0.0f;
#pragma unroll
                    for (int k = 0; k < D; ++k) wsum = fmaf(ar[k], (float)yv[k], wsum);
                    wv[c] = wsum;
                }
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
                if constexpr (HAD) e *= wv[c];
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

template <int D>
void launch_lse_d(int R, dim3 grid, hipStream_t st, const double *res, const double *str, double cscale, int tps,
                  int n_tiles, double2 *partial, int64_t stride)
{
    // float64 scores on the vector ALU exist for d <= 3 only (above, those half-steps run on the fp64
    // matrix cores and never come here)
    if constexpr (D <= 3) {
        if (R == 2)
            hipLaunchKernelGGL((k_lse_lowd<double, D, 2>), grid, dim3(kBlock), 0, st, res, str, cscale, tps, n_tiles, partial, stride);
        else
            hipLaunchKernelGGL((k_lse_lowd<double, D, 1>), grid, dim3(kBlock), 0, st, res, str, cscale, tps, n_tiles, partial, stride);
    }
}

template <typename S, int D>
void launch_apply_d(dim3 grid, hipStream_t st, const S *res, const S *str, const float *V, int64_t ldv, int p0, int p,
                    int64_t n_str, S cscale, int tps, int n_tiles, double2 *partial, int64_t stride, float *opart,
                    const float *had_A, int64_t lda, int64_t n_res)
{
    // (the float64 form exists for d <= 3 only, see launch_lse_d)
    if constexpr (sizeof(S) == 4 || D <= 3) {
        if (had_A)
            hipLaunchKernelGGL((k_apply_lowd<S, D, kApplyPC, true>), grid, dim3(kBlock), 0, st, res, str, V, ldv, p0, p, n_str,
                               cscale, tps, n_tiles, partial, stride, opart, stride, had_A, lda, n_res);
        else
            hipLaunchKernelGGL((k_apply_lowd<S, D, kApplyPC, false>), grid, dim3(kBlock), 0, st, res, str, V, ldv, p0, p, n_str,
                               cscale, tps, n_tiles, partial, stride, opart, stride, had_A, lda, n_res);
    }
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

// Column splits of a streaming pass.  Model (in units of the time a CU needs for one tile): a CU
// works through its ceil(W / CUs) workgroups one tile at a time (the vector ALU is the shared
// resource, two resident workgroups only interleave), and every round of 2 CUs workgroups pays
// the start-up and wind-down latency of a workgroup (resident operands, first tile, merge,
// partial store: ~5 us measured, about 7 tile times of the split kernel) once:
//     cost(s) = ceil(W / CUs) * tiles_per_split + ceil(W / (2 CUs)) * startup + 0.3 s,   W = row_blocks * s
// (the last term: the merge kernel that follows reads s records per row).
// Among the split counts within 2 % of the cheapest the one closest to 32 workgroups per CU from
// below is taken (finer load balance at large sizes; measured at n = m = 262144), else the smallest.
// One tile per workgroup, which filling the chip 32 times over used to give at n ~ 10^4, made the
// pass four times slower than this choice.  The context's "lowd_splits" switch overrides (tests and experiments).
PassShape shape_for(const Ctx *c, int64_t n_res, int64_t n_str, int rows_per_block, int tj = kTJ, int startup_tiles = 7)
{
    PassShape s;
    s.rows_per_block = rows_per_block;
    s.row_blocks = (int)ceil_div(n_res, s.rows_per_block);
    const int n_tiles = (int)ceil_div(n_str, tj);
    const int cap_splits = max_splits(c->partial_budget, n_res);
    int smax = n_tiles < cap_splits ? n_tiles : cap_splits;
    if (smax < 1) smax = 1;
    int legacy = (int)ceil_div(32 * c->num_cu, s.row_blocks);
    if (legacy > smax) legacy = smax;
    auto cost = [&](int sp) {
        const int64_t tps = ceil_div(n_tiles, sp);
        const int64_t w = (int64_t)s.row_blocks * ceil_div(n_tiles, tps);
        return (double)(ceil_div(w, c->num_cu) * tps + ceil_div(w, 2 * c->num_cu) * startup_tiles) + 0.3 * (double)(w / s.row_blocks);
    };
    double best = cost(1);
    for (int sp = 2; sp <= smax; ++sp) best = cost(sp) < best ? cost(sp) : best;
    int splits = 0;
    for (int sp = legacy; sp >= 1 && !splits; --sp)
        if (cost(sp) <= 1.02 * best) splits = sp;
    for (int sp = legacy + 1; sp <= smax && !splits; ++sp)
        if (cost(sp) <= 1.02 * best) splits = sp;
    if (c->dbg_lowd_splits >= 1) splits = c->dbg_lowd_splits < smax ? c->dbg_lowd_splits : smax;
    const int tps = (int)ceil_div(n_tiles, splits);
    s.splits = (int)ceil_div(n_tiles, tps);
    s.cols_per_split = (int64_t)tps * tj;
    return s;
}

}  // namespace

// Score precision of a half-step.  An fp32 score carries roundings of relative size 2^-24 at
// magnitude Mag = max(2 k rho_max, largest |bias| the caller's potentials give), k = log2e/eps,
// rho_max = largest squared norm after centring.  A single half-step can be off by about
// 1.5 * 2^-24 * Mag * ln2 in units of eps when few terms dominate a row (no averaging), and,
// measured against the float64 reference, a run of T half-steps at one eps accumulates about
// 0.05..0.07 * T * 2^-24 * Mag in single rows (small clouds with outlying points, where the iteration
// damps little).  fp32 scores are used while both stay below ~3e-5 and 2e-5, i.e.
// Mag <= 480 and Mag * T <= 5000; otherwise the scores are formed in float64.
// (The part of these errors that is common to all rows and differs between the two passes is a
// different matter: it adds up along the iteration's neutral direction and grows with the size of the
// clouds; the solvers measure and remove it, see GaugeMode.)
// The context's "lowd_score" switch overrides the choice (tests and experiments), except for the
// measurements that always take float64 scores.
bool lowd_precise(const Prepared *P, double eps)
{
    if (P->force_precise) return true;
    if (P->dbg_score == 32) return false;
    if (P->dbg_score == 64) return true;
    const double k = kLog2e / eps;
    const double mag = fmax(2.0 * k * P->rho_max, P->pot_mag_eps / eps + P->logw_mag);
    return mag > 480.0 || mag * (double)(P->halfsteps_per_eps > 0 ? P->halfsteps_per_eps : 1) > 5000.0;
}

PassShape lowd_shape(const Ctx *c, int64_t n_res, int64_t n_str)
{
    // two rows per lane halve the LDS reads per pair; four cost occupancy and were slower
    int R = n_res >= 32768 ? 2 : 1;
    return shape_for(c, n_res, n_str, kBlock * R);
}

// split-record pass: a wave owns kSplitR groups of 32 resident rows, a workgroup 128 kSplitR rows;
// streamed tiles of kSplitTJ points (two LDS buffers of 32 KS kSplitTJ bytes), chunks of kSplitCH x 32
// streamed points between two checks of the lazy stabiliser.  Measured at n = m = 262144, d = 3:
// (R, TJ, CH) = (2,128,4) 6.62 ms, (2,256,4) 6.69, (4,256,2) 6.68, (2,256,8) 6.71, (1,128,4) 7.03.
constexpr int kSplitR = 2, kSplitTJ = 128, kSplitCH = 4;

template <int KS>
void launch_lse_split(dim3 grid, hipStream_t st, const SplitArgs &a)
{
    hipLaunchKernelGGL((k_lse_lowd_split<KS, kSplitR, kSplitTJ, kSplitCH, false>), grid, dim3(kBlock), 0, st, a);
}

// Can a float64-score half-step run on the matrix cores from the precise split records?
// d <= 3; integers (the running max) must be multiples of the grid q = gx gy of the exact part,
// and the three 8-bit bias digits must cover the largest bias that can come up (the size the
// caller's potentials give, or four times the cost scale for potentials the iteration produces).
static bool precise_on_matrix_cores(const Prepared *P, const Side *res, const Side *str, double eps, double *gx_out)
{
    if (P->dbg_precise_valu) return false;   // the context's "lowd_precise_valu" switch
    if (P->d > 3 || !str->split_p || !res->packed_d) return false;
    double gx, gy;
    split_grids(P->rho_max, eps, &gx, &gy);
    const double q = gx * gy;
    const double mag = 2.0 * (kLog2e / eps) * P->rho_max;
    const double bias_bound = fmax(4.0 * mag, P->pot_mag_eps / eps + P->logw_mag);
    *gx_out = gx;
    // (beyond the digit range the records still sum to the bias, at fp32-grade accuracy of the score: the context's
    // "lowd_precise_any_bias" switch lets tests run that case, which otherwise only potentials that outgrow the bound
    // during a solve can reach)
    return q <= 1.0 && (bias_bound < 2097152.0 * q || P->dbg_any_bias);
}

// Arguments of a split-record pass (res resident, str streamed) writing its records to `partial`;
// false when this half-step does not run on the split-record kernels (float64 scores off the
// matrix cores) or its shape does not fit the padded copies (*st says which).
static bool split_pass_args(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, void *partial,
                            SplitArgs *a, bool *precise_out, fs_status *st, int rblocks = kSplitR)
{
    *st = FS_OK;
    const bool precise = lowd_precise(P, eps);
    double gx = 0.0;
    if (precise && !precise_on_matrix_cores(P, res, str, eps, &gx)) return false;
    // (rblocks: blocks of 32 resident rows per wave of the kernel that will run)
    const PassShape s = shape_for(c, res->cnt, str->cnt, 128 * rblocks, kSplitTJ);
    const int n_tiles = (int)ceil_div(str->cnt, kSplitTJ);
    // host-side shape checks: every access of the kernel stays inside the padded copies
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)n_tiles * kSplitTJ > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes || (!precise && P->ks != split_ksteps(P->d)) ||
        (!precise && (P->ks < 1 || P->ks > 9))) {
        *st = fail(c, FS_ERR_DEVICE, "internal: low-d launch shape exceeds the padded buffers");
        return false;
    }
    *a = SplitArgs{};
    a->cscale = 2.0 * kLog2e / eps;
    a->d = (int)P->d;
    a->tiles_per_split = (int)(s.cols_per_split / kSplitTJ);
    a->n_tiles = n_tiles;
    a->row_blocks = s.row_blocks;
    a->splits = s.splits;
    a->partial = (double2 *)partial;
    a->partial_stride = res->cnt_pad;
    if (precise) {
        a->res = res->packed_d;
        a->dp = P->dpd;
        a->str = str->split_p;
        a->gx = gx;
    } else {
        a->res = res->packed;
        a->dp = P->dp;
        a->str = str->split;
    }
    *precise_out = precise;
    return true;
}

template <int KS>
void launch_lse_split_pair(dim3 grid, hipStream_t st, const SplitArgs &a0, const SplitArgs &a1)
{
    hipLaunchKernelGGL((k_lse_lowd_split_pair<KS, kSplitR, kSplitTJ, kSplitCH, false>), grid, dim3(kBlock), 0, st, a0, a1);
}

#define FS_SPLIT_KS_DISPATCH(ks, CALL)                                                                       \
    switch (ks) {                                                                                            \
    case 1: { constexpr int KS_ = 1; CALL; } break;                                                          \
    case 2: { constexpr int KS_ = 2; CALL; } break;                                                          \
    case 3: { constexpr int KS_ = 3; CALL; } break;                                                          \
    case 4: { constexpr int KS_ = 4; CALL; } break;                                                          \
    case 5: { constexpr int KS_ = 5; CALL; } break;                                                          \
    case 6: { constexpr int KS_ = 6; CALL; } break;                                                          \
    case 7: { constexpr int KS_ = 7; CALL; } break;                                                          \
    case 8: { constexpr int KS_ = 8; CALL; } break;                                                          \
    default: { constexpr int KS_ = 9; CALL; } break;                                                         \
    }

fs_status lowd_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out)
{
    // fp32-accuracy half-steps run on the bf16 matrix cores from the split records; float64-score
    // ones too when d <= 3 (precise records); other float64-score half-steps are handled further down
    SplitArgs a;
    bool precise = false;
    fs_status st;
    if (split_pass_args(c, P, res, str, eps, P->partial, &a, &precise, &st)) {
        const dim3 grid((unsigned)a.row_blocks, (unsigned)a.splits);
        prof_begin(c, (double)res->cnt * (double)str->cnt, precise ? 1 : 0);
        if (precise) {
            hipLaunchKernelGGL((k_lse_lowd_split<3, kSplitR, kSplitTJ, kSplitCH, true>), grid, dim3(kBlock), 0, c->stream, a);
        } else {
            FS_SPLIT_KS_DISPATCH(P->ks, (launch_lse_split<KS_>(grid, c->stream, a)));
        }
        prof_end(c);
        FS_HIP(c, hipGetLastError());
        *splits_out = a.splits;
        return FS_OK;
    }
    if (st != FS_OK) return st;
    // float64 scores outside the reach of the split records: on the fp64 matrix cores for d > 3 (from
    // the centred float64 records the prologue wrote for that kernel), else on the vector ALU
    if (res->pts_d && str->pts_d && str->bias_d) return f64_lse(c, P, res, str, eps, splits_out, 1);
    if (P->d > 3) return fail(c, FS_ERR_DEVICE, "internal: float64-score pass at d > 3 without its records");
    PassShape s = lowd_shape(c, res->cnt, str->cnt);
    const int n_tiles = (int)ceil_div(str->cnt, kTJ);
    const int tps = (int)(s.cols_per_split / kTJ);
    if ((int64_t)s.row_blocks * s.rows_per_block > res->cnt_pad || (int64_t)n_tiles * kTJ > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes)
        return fail(c, FS_ERR_DEVICE, "internal: low-d launch shape exceeds the padded buffers");
    const double cscale = 2.0 * kLog2e / eps;
    dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
    double2 *part = (double2 *)P->partial;
    prof_begin(c, (double)res->cnt * (double)str->cnt, 1);
    const int R = s.rows_per_block / kBlock;
    FS_LOWD_DISPATCH((int)P->d, (launch_lse_d<DD>(R, grid, c->stream, res->packed_d, str->packed_d, cscale, tps, n_tiles,
                                                  part, res->cnt_pad)));
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = s.splits;
    return FS_OK;
}

// The f-pass (records to partial_x) and the g-pass (records to partial_y) of one iteration of the
// averaged schedule (Eq. 4-5) in ONE launch.  *done = false (nothing launched) when the half-steps
// of this problem do not run on the split-record kernels; the caller then runs them one by one.
fs_status lowd_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x,
                        int *splits_y, bool *done)
{
    *done = false;
    SplitArgs ax, ay;
    bool px = false, py = false;
    fs_status st;
    if (!split_pass_args(c, P, &P->X, &P->Y, eps, partial_x, &ax, &px, &st)) return st;
    if (!split_pass_args(c, P, &P->Y, &P->X, eps, partial_y, &ay, &py, &st)) return st;
    if (px != py) return FS_OK;
    const dim3 grid((unsigned)(ax.row_blocks + ay.row_blocks), (unsigned)(ax.splits > ay.splits ? ax.splits : ay.splits));
    prof_begin(c, 2.0 * (double)P->X.cnt * (double)P->Y.cnt, px ? 1 : 0);
    if (px) {
        hipLaunchKernelGGL((k_lse_lowd_split_pair<3, kSplitR, kSplitTJ, kSplitCH, true>), grid, dim3(kBlock), 0, c->stream, ax, ay);
    } else {
        FS_SPLIT_KS_DISPATCH(P->ks, (launch_lse_split_pair<KS_>(grid, c->stream, ax, ay)));
    }
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_x = ax.splits;
    *splits_y = ay.splits;
    *done = true;
    return FS_OK;
}

// Value image for the matrix-core application (PC == 8): per tile of kSplitTJ streamed points and group of 32
// of them, [k-step 0/1][lane half h][row c' 0..31][8 bf16]; slot e of (k-step ks, half h) is streamed point
// 8 (2 ks + e / 4) + 4 h + e % 4 of the group, i.e. the order in which a lane of the score MFMA holds its sixteen
// exponentials.  Row c' = 8 (col / 2) + 4 (col % 2) + piece holds bf16 piece `piece` (0..2) of value column
// p0 + col; row 3 holds ones (the row sum), the other spare rows zeros.  One thread per 16-byte unit.
constexpr int kApplyMM = 8;   // value columns per pass of the matrix-core application (values in three bf16 pieces)
constexpr int kApplyMM2 = 15;  // ... with values in two pieces (kept to 2^-17 like the exponentials): for more than 8 columns
// `pieces` == 2: fifteen columns, row 2 col + piece, row 30 the ones, row 31 zeros.
__global__ __launch_bounds__(256) void k_vimg_lowd(const float *__restrict__ V, int64_t ldv, int64_t n_str, int p0, int p,
                                                   int64_t units, unsigned char *__restrict__ img, int pieces)
{
    const int64_t u = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (u >= units) return;
    const int cr = (int)(u & 31), h = (int)(u >> 5) & 1, ks = (int)(u >> 6) & 1;
    const int64_t grp = u >> 7;   // group of 32 streamed points
    // piece 3 = a spare row (ones in row `ones_row`, zeros elsewhere)
    const int piece = pieces == 2 ? (cr >= 30 ? 3 : (cr & 1)) : (cr & 3);
    const int col = pieces == 2 ? (cr >> 1) : 2 * (cr >> 3) + ((cr >> 2) & 1);
    const int ones_row = pieces == 2 ? 30 : 3;
    uint32_t w[4];
#pragma unroll
    for (int e = 0; e < 8; e += 2) {
        __bf16 v[2];
#pragma unroll
        for (int k = 0; k < 2; ++k) {
            const int64_t i = grp * 32 + 8 * (2 * ks + ((e + k) >> 2)) + 4 * h + ((e + k) & 3);
            float x = 0.0f;
            if (i < n_str) {
                if (piece == 3) {
                    x = cr == ones_row ? 1.0f : 0.0f;
                } else if (p0 + col < p) {
                    __bf16 q[3];
                    split3(V[i * ldv + p0 + col], q);
                    x = (float)q[piece];
                }
            }
            v[k] = (__bf16)x;
        }
        w[e >> 1] = bf16_pair(v[0], v[1]);
    }
    *reinterpret_cast<uint4 *>(img + u * 16) = make_uint4(w[0], w[1], w[2], w[3]);
}

// workspace of an application: [splits][rows][columns per pass] float accumulators, then the value images
static size_t lowd_opart_bytes(int splits, int64_t res_pad) { return ((size_t)splits * (size_t)res_pad * 16 * 4 + 1023) & ~size_t(1023); }
static size_t lowd_vimg_bytes(int64_t n_str) { return (size_t)ceil_div(n_str, kSplitTJ) * (kSplitTJ / 32) * 2048; }

size_t lowd_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str, int64_t d, int64_t p)
{
    // the largest of the launch shapes an application can take (split records with one or two row blocks per
    // wave / vector ALU / fp64 matrix cores)
    const PassShape s1 = shape_for(c, n_res, n_str, kBlock);
    const PassShape s2 = shape_for(c, n_res, n_str, 128 * kSplitR, kSplitTJ);
    const PassShape s3 = shape_for(c, n_res, n_str, 128, kSplitTJ);
    int splits = s1.splits > s2.splits ? s1.splits : s2.splits;
    splits = splits > s3.splits ? splits : s3.splits;
    const size_t own = lowd_opart_bytes(splits, round_up(n_res, 1024)) + lowd_vimg_bytes(n_str);
    const size_t f64 = d > 3 ? f64_apply_ws(c, n_res, n_str, d, p) : 0;
    return own > f64 ? own : f64;
}

// Matrix-core application on the split records: eight value columns per pass.  Two blocks of 32 resident rows per
// wave while the records are short; one block for KS > 4, where two would not leave registers for the operands.
// (One block per wave and three workgroups per CU instead of two, which the registers allow for KS <= 4, measured
// 4-6 % slower at d = 2..4 and 15 % slower at d = 6.)
template <int KS>
void launch_apply_split(dim3 grid, hipStream_t st, const SplitArgs &a, bool two_pieces)
{
    if (two_pieces)
        hipLaunchKernelGGL((k_apply_lowd_split<KS, (KS <= 4 ? kSplitR : 1), kSplitTJ, kSplitCH, false, 16, 16>), grid, dim3(kBlock), 0,
                           st, a);
    else
        hipLaunchKernelGGL((k_apply_lowd_split<KS, (KS <= 4 ? kSplitR : 1), kSplitTJ, kSplitCH, false, kApplyMM, kApplyMM>), grid,
                           dim3(kBlock), 0, st, a);
}
// The form with the products on the vector ALU (four columns per pass) is kept where it measured faster
// (n = m = 65536): a single column on short records, where a kernel copy multiplies one column only
// (d = 3: 0.71 against 0.89 ms), and up to four columns at d = 16, where the matrix-core form runs one
// workgroup per CU (1.8 against 2.2 ms).  Everywhere else the matrix-core form wins: 0.92 against 1.06 ms
// for three columns at d = 3, 0.97 against 2.02 ms for eight.
static bool apply_on_valu(int ks, bool precise, int64_t p) { return (p == 1 && (precise || ks <= 3)) || (!precise && ks == 9 && p <= 4); }
template <int KS>
void launch_apply_split_valu(dim3 grid, hipStream_t st, const SplitArgs &a, int cols)
{
    if constexpr (KS <= 3) {
        if (cols == 1) {
            hipLaunchKernelGGL((k_apply_lowd_split<KS, kSplitR, kSplitTJ, kSplitCH, false, kApplyPC, 1>), grid, dim3(kBlock), 0, st, a);
            return;
        }
    }
    hipLaunchKernelGGL((k_apply_lowd_split<KS, kSplitR, kSplitTJ, kSplitCH, false, kApplyPC, kApplyPC>), grid, dim3(kBlock), 0, st, a);
}

fs_status lowd_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V,
                     int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass_out, const float *had_A, int64_t lda)
{
    float *opart = (float *)P->extra;
    // Plain applications run on the split records (scores and products on the matrix cores);
    // the Hadamard-weighted form and float64 scores outside the matrix cores' reach stay on the
    // vector-ALU kernel below.
    if (!had_A) {
        SplitArgs a;
        bool precise = false;
        fs_status st;
        const bool valu = apply_on_valu(P->ks, lowd_precise(P, eps), p);
        const int rblocks = (valu || lowd_precise(P, eps) || P->ks <= 4) ? kSplitR : 1;
        if (split_pass_args(c, P, res, str, eps, P->partial, &a, &precise, &st, rblocks)) {
            const size_t ob = lowd_opart_bytes(a.splits, res->cnt_pad);
            const int64_t units = (int64_t)a.n_tiles * (kSplitTJ / 32) * 128;
            if (!opart || ob + (size_t)units * 16 > P->extra_bytes) return fail(c, FS_ERR_DEVICE, "internal: low-d apply workspace");
            unsigned char *vimg = reinterpret_cast<unsigned char *>(opart) + ob;
            a.V = V;
            a.ldv = ldv;
            a.n_str = str->cnt;
            a.p = (int)p;
            a.opart = opart;
            a.vimg = vimg;
            const dim3 grid((unsigned)a.row_blocks, (unsigned)a.splits);
            for (int p0 = 0; valu && p0 < p; p0 += kApplyPC) {
                a.p0 = p0;
                const int cols = (int)(p - p0 < kApplyPC ? p - p0 : kApplyPC);
                if (precise) {
                    hipLaunchKernelGGL((k_apply_lowd_split<3, kSplitR, kSplitTJ, kSplitCH, true, kApplyPC, 1>), grid, dim3(kBlock), 0,
                                       c->stream, a);
                } else {
                    FS_SPLIT_KS_DISPATCH(P->ks, (launch_apply_split_valu<KS_>(grid, c->stream, a, cols)));
                }
                FS_HIP(c, hipGetLastError());
                st = launch_apply_finalize(c, P, res, precise ? res->norm : res->norm_f, a.splits, eps, opart, kApplyPC, p0,
                                           (int)p, out, ldo, mass_out);
                if (st != FS_OK) return st;
            }
            if (valu) return FS_OK;
            // up to eight columns: values in three bf16 pieces (exact); more: passes of fifteen columns with two pieces
            const bool two = p > kApplyMM;
            const int step = two ? kApplyMM2 : kApplyMM, width = two ? 16 : kApplyMM;
            for (int p0 = 0; p0 < p; p0 += step) {
                a.p0 = p0;
                const int p_end = (int)(p0 + step < p ? p0 + step : p);   // columns of this pass: p0 .. p_end - 1
                hipLaunchKernelGGL(k_vimg_lowd, dim3((unsigned)ceil_div(units, 256)), dim3(256), 0, c->stream, V, ldv, str->cnt, p0,
                                   p_end, units, vimg, two ? 2 : 3);
                if (precise) {
                    if (two)
                        hipLaunchKernelGGL((k_apply_lowd_split<3, kSplitR, kSplitTJ, kSplitCH, true, 16, 16>), grid, dim3(kBlock), 0,
                                           c->stream, a);
                    else
                        hipLaunchKernelGGL((k_apply_lowd_split<3, kSplitR, kSplitTJ, kSplitCH, true, kApplyMM, kApplyMM>), grid,
                                           dim3(kBlock), 0, c->stream, a);
                } else {
                    FS_SPLIT_KS_DISPATCH(P->ks, (launch_apply_split<KS_>(grid, c->stream, a, two)));
                }
                FS_HIP(c, hipGetLastError());
                st = launch_apply_finalize(c, P, res, precise ? res->norm : res->norm_f, a.splits, eps, opart, width, p0, p_end, out,
                                           ldo, mass_out);
                if (st != FS_OK) return st;
            }
            return FS_OK;
        }
        if (st != FS_OK) return st;
    }
    // float64 scores at d > 3 (plain or Hadamard-weighted): the fp64 matrix-core application
    if (lowd_precise(P, eps) && res->pts_d && str->pts_d && str->bias_d)
        return f64_apply(c, P, res, str, eps, V, p, ldv, out, ldo, mass_out, had_A, lda);
    if (P->d > 3 && lowd_precise(P, eps)) return fail(c, FS_ERR_DEVICE, "internal: float64-score application at d > 3 without its records");
    PassShape s = shape_for(c, res->cnt, str->cnt, kBlock);
    const int n_tiles = (int)ceil_div(str->cnt, kTJ);
    const int tps = (int)(s.cols_per_split / kTJ);
    if ((int64_t)s.row_blocks * kBlock > res->cnt_pad || (int64_t)n_tiles * kTJ > str->cnt_pad ||
        (size_t)s.splits * res->cnt_pad * 16 > P->partial_bytes ||
        (size_t)s.splits * res->cnt_pad * kApplyPC * 4 > P->extra_bytes)
        return fail(c, FS_ERR_DEVICE, "internal: low-d apply launch shape exceeds the padded buffers");
    const double cscale = 2.0 * kLog2e / eps;
    const bool precise = lowd_precise(P, eps);
    dim3 grid((unsigned)s.row_blocks, (unsigned)s.splits);
    for (int p0 = 0; p0 < p; p0 += kApplyPC) {
        if (precise) {
            FS_LOWD_DISPATCH((int)P->d, (launch_apply_d<double, DD>(grid, c->stream, res->packed_d, str->packed_d, V, ldv,
                                                                    p0, (int)p, str->cnt, cscale, tps, n_tiles,
                                                                    (double2 *)P->partial, res->cnt_pad, opart, had_A, lda,
                                                                    res->cnt)));
        } else {
            FS_LOWD_DISPATCH((int)P->d, (launch_apply_d<float, DD>(grid, c->stream, res->packed, str->packed, V, ldv, p0,
                                                                   (int)p, str->cnt, (float)cscale, tps, n_tiles,
                                                                   (double2 *)P->partial, res->cnt_pad, opart, had_A, lda,
                                                                   res->cnt)));
        }
        fs_status st = launch_apply_finalize(c, P, res, precise ? res->norm : res->norm_f, s.splits, eps, opart,
                                             kApplyPC, p0, (int)p, out, ldo, mass_out);
        if (st != FS_OK) return st;
    }
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
