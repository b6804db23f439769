// bf16 matrix-core path (d >= 16): the score tile 2<x_i, y_j> of Alg. 1 / Alg. 3 is a dense
// contraction over d, computed with v_mfma_f32_32x32x16_bf16 (bf16 in, fp32 accumulate); bias,
// online LSE and potentials stay in fp32/fp64.
//
// Shape of the work.  A resident row block at d = 784..1024 does not fit on chip (256 rows x
// 800 x 2 B = 400 KB), so unlike Alg. 1 the pass is organised as a GEMM with an LSE epilogue:
// a workgroup owns 256 resident rows (j) and a group of streamed tiles (i); for every streamed
// tile of 256 points it runs the full contraction over d in chunks of 32 through a four-stage
// LDS ring filled by direct global->LDS loads (three stages in flight), then folds
// the 256 x 256 scores into the per-row running (max, sum).  Groups of streamed tiles ("splits")
// are merged afterwards.  Concurrent workgroups of one XCD form 8 x 8 super-tiles, so each panel
// chunk fetched into that XCD's L2 is shared by eight workgroups.
//
// MFMA operand roles (32x32x16): A = streamed points (i), B = resident rows (j);
//   A: lane l holds A[i = l%32][k = 8*(l/32) .. +7],  B likewise with j = l%32,
//   D: lane l, register r holds D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32],
// i.e. the 16 accumulator registers of a lane are 16 streamed points of ONE resident row, so
// the row-wise LSE runs inside the lane; lanes/waves are merged once per workgroup.
#include <type_traits>

#include "fs_internal.h"

namespace fs {
namespace {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int BI = 256;          // streamed points per tile (4 waves x 64)
constexpr int KC = 32;           // contraction chunk per pipeline stage (bf16 elements) = 64 B per row
constexpr int NBIAS = 8;         // ring of bias tiles (one per stage, deeper than the data ring)
constexpr float kLazyMax = 1.152921504606846976e18f;   // 2^60

__device__ inline float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

// all LDS reads of this wave have returned, then the workgroup barrier
__device__ inline void lds_done_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
template <int N> __device__ inline void wait_vm() { asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory"); }

// N consecutive 1 KB pieces (N <= 4) by direct global -> LDS loads behind ONE write of the LDS base to m0, the
// pieces addressed by immediate offsets (they advance the memory and the LDS address alike).  A write to m0 waits
// until the wave's earlier direct loads have left for the address unit, so a load with its own m0 write between the
// MFMAs of the contraction loop stalls the wave behind the queue of all eight waves' loads: issuing a stage's loads
// as one run took the pass at n = m = 70000, d = 784 from 7.7 to 6.6 ms.
template <int N>
__device__ inline void dma16_run(const void *g_uniform, unsigned lane_off, unsigned lds_off)
{
    static_assert(N >= 1 && N <= 4, "immediate offsets reach 3 KB");
    if constexpr (N == 1)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1" ::"v"(lane_off), "s"(g_uniform), "s"(lds_off)
                     : "memory", "m0");
    else if constexpr (N == 2)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024" ::"v"(
                         lane_off),
                     "s"(g_uniform), "s"(lds_off)
                     : "memory", "m0");
    else if constexpr (N == 3)
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024\n\t"
                     "global_load_lds_dwordx4 %0, %1 offset:2048" ::"v"(lane_off),
                     "s"(g_uniform), "s"(lds_off)
                     : "memory", "m0");
    else
        asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1\n\tglobal_load_lds_dwordx4 %0, %1 offset:1024\n\t"
                     "global_load_lds_dwordx4 %0, %1 offset:2048\n\tglobal_load_lds_dwordx4 %0, %1 offset:3072" ::"v"(lane_off),
                     "s"(g_uniform), "s"(lds_off)
                     : "memory", "m0");
}
// (n is uniform over the wave)
__device__ inline void dma16_run_n(int n, const void *g_uniform, unsigned lane_off, unsigned lds_off)
{
    switch (n) {
    case 1: dma16_run<1>(g_uniform, lane_off, lds_off); break;
    case 2: dma16_run<2>(g_uniform, lane_off, lds_off); break;
    case 3: dma16_run<3>(g_uniform, lane_off, lds_off); break;
    case 4: dma16_run<4>(g_uniform, lane_off, lds_off); break;
    default: break;
    }
}

struct BfArgs {
    const uint16_t *res;     // resident side, tiled bf16 copy (see k_prep_bf16)
    const uint16_t *str;     // streamed side, tiled bf16 copy
    const float *bias;       // [str_pad] base-2 bias of the streamed points (-inf on padding)
    int kp;                  // multiple of 32
    float cscale;            // 2 log2(e) / eps
    int n_jtiles, n_itiles, splits, tiles_per_split;
    double2 *partial;
    int64_t partial_stride;
    // plan application only
    const unsigned char *vimg;   // [n_itiles] value images (see k_vimg_bf16)
    float *opart;                // [splits][partial_stride][PC]
};

// Workgroup shapes (WJ = waves along the resident side, each owning 128 resident rows; four waves
// along the streamed side, each owning 64 of the tile's 256 streamed points):
//   WJ = 2: 512 threads, 256 x 256 tile, ring of 4 stages x 32 KB, one workgroup per CU;
//   WJ = 1: 256 threads, 256 x 128 tile, ring of 3 stages x 24 KB, two workgroups per CU, which
//           run out of phase: one's tile epilogue (vector ALU only) and barrier waits are covered by
//           the other's MFMAs, at the price of 1.5x the operand traffic per flop.  Measured slower
//           (8.8 against 7.9 ms at n = m = 70000, d = 784): the operand traffic costs more than the
//           overlap brings.  The LSE pass is built with WJ = 2 only; the template keeps the parameter.
//
// LDS layout of a stage: row r (0..255 streamed, then the resident rows) occupies 64 bytes = four
// 16-byte pieces; piece p is stored at position p ^ ((r >> 2) & 3): sixteen consecutive rows then read
// one MFMA fragment from sixteen different 16-byte bank groups of a 256-byte line (measured fragment-read
// rate 179 B/clk/CU, against 120 with a rotation by (r >> 1) & 3 and 63 without one).
// The derived bf16 copies in HBM already have this layout in 1 KB tiles (16 rows x 32 coordinates),
// so every direct load is a linear 1 KB copy: measured 52 B/clk/CU from L2 against 26 B/clk/CU for
// 64-byte row segments, and a 256 x 256 tile needs 32 B/clk/CU at full MFMA rate.
//
// Schedule of one stage g in every wave (F0/F1 = fragment registers of the two 16-wide k-steps):
//     4 MFMA on F0(g) | read F1(g), issue the loads of stage g + NS - 1 | 4 MFMA on F0(g) | 4 MFMA on F1(g) |
//     wait "stage g+1 landed" + barrier | read F0(g+1) | 4 MFMA on F1(g)
// A wave's loads of a stage (its 1 KB pieces, consecutive in memory and in LDS) go out as ONE run behind a
// single write of m0; the biases of a streamed tile come with the tile's first stage.  The barrier and the
// LDS latency of the next fragments hide behind the last MFMAs.
// Ceiling: with random operands the matrix cores sustain ~1.83 PFLOP/s here (a loop of nothing but
// this MFMA: 2.42 PFLOP/s on constant operands, 1.83 on uniform random ones), i.e. the chip is
// power-limited well below the 2.5 PFLOP/s peak that the roofline fraction is quoted against; the
// shipped pass runs at 1.84 GHz with the matrix pipe 67 % busy.
//
// PC > 0 is the plan application (Alg. 2 / Alg. 4) in this mode: a fused matmul - softmax - matmul.
// A wave then owns JTW = 2 blocks of 32 resident rows (64 x 64 scores per tile, 256 x 128 per
// workgroup), which leaves registers for the output accumulators O[resident row][PC value columns].
// After the contraction over d the exponentials exp2(score - max) of a tile are rounded to bf16 IN
// the accumulator layout, which is exactly the B operand of a second MFMA whose contraction runs
// over the streamed points:   O^T[c][j] += sum_i Vt[c][i] E[i][j].   The value rows of the tile
// arrive as a bf16 image Vt[c][i] (rows padded to 520 bytes: conflict-free 8-byte fragment reads)
// by direct loads issued at the start of the tile's contraction.  The running max of a resident
// row is common to the two lane halves here (the second MFMA sums over them).
constexpr int kVRow = 520;                       // bytes per value column in the LDS image (256 points + pad)
constexpr int kVImgBytes(int pc) { return (pc * kVRow + 1023) / 1024 * 1024; }

template <int WJ, int NS, int JTW, int PC, bool HALF = false>
__device__ __forceinline__ void lse_bf16_body(const BfArgs &a, const int block)
{
    constexpr bool APPLY = PC > 0;
    constexpr int BJ = 32 * JTW * WJ;            // resident rows per workgroup
    constexpr int ROWS = BI + BJ;
    constexpr int STAGE_BYTES = ROWS * KC * 2;   // 32 KB / 24 KB
    constexpr int NW = 4 * WJ;                   // waves
    constexpr int PPW = (ROWS / 16) / NW;        // 1 KB pieces of a stage per wave
    constexpr int D = NS - 1;                    // stages in flight
    constexpr int NCB = APPLY ? PC / 32 : 1;     // 32-column blocks of the value matrix
    constexpr int VIMG = APPLY ? kVImgBytes(PC) : 16;
    constexpr int NVP = VIMG / 1024;             // 1 KB pieces of a value image
    static_assert((ROWS / 16) % NW == 0 && PPW <= 4 && D >= 2 && D <= 3, "pipeline shape");
    static_assert(JTW == 4 || JTW == 2, "MFMA schedules below");
    static_assert(!APPLY || (PC % 32 == 0 && BJ * PC * 4 + BJ * 64 <= NS * STAGE_BYTES), "merge buffers fit the ring");
    __shared__ __attribute__((aligned(1024))) unsigned char ring[NS * STAGE_BYTES];
    __shared__ __attribute__((aligned(256))) float bias_ring[NBIAS][BI];                 // 8,192 B
    __shared__ __attribute__((aligned(1024))) unsigned char vimg[VIMG];

    // ---- which (resident tile, split) this workgroup owns.  Workgroups go to XCDs round-robin;
    // each XCD gets a contiguous, equally long run of the work list, which is ordered in patches of
    // 8 resident tiles x 8 splits (clipped at the edges), so that the workgroups running on an
    // XCD at any time share their panels through that XCD's L2.
    const int b = block;
    const int total = a.n_jtiles * a.splits;
    const int per = (total + 7) >> 3;
    const int lb = b >> 3;
    const int idx = (b & 7) * per + lb;
    if (lb >= per || idx >= total) return;
    int jtile, split;
    {
        const int NJ = a.n_jtiles, full = a.splits >> 3, gsz = NJ * 8;
        int gs, rem, h;
        if (idx < full * gsz) {
            gs = idx / gsz;
            rem = idx - gs * gsz;
            h = 8;
        } else {
            gs = full;
            rem = idx - full * gsz;
            h = a.splits - 8 * full;
        }
        const int pj = rem / (8 * h);
        const int r = rem - pj * 8 * h;
        const int wp = min(8, NJ - 8 * pj);
        jtile = 8 * pj + r % wp;
        split = 8 * gs + r / wp;
    }

    const int tid = threadIdx.x;
    // (the wave number as a scalar: stage, piece and address arithmetic of the loads below then runs on
    // the scalar unit instead of taking vector-ALU issue slots from the MFMA loop)
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6), l = tid & 63;
    const int wi = w & 3, wj = w >> 2;
    const int lh = l >> 5, lr = l & 31;
    const int n_chunks = a.kp / KC;
    const int64_t row0 = (int64_t)jtile * BJ;
    const int t_begin = split * a.tiles_per_split;
    const int t_end = min(a.n_itiles, t_begin + a.tiles_per_split);
    const int G = (t_end - t_begin) * n_chunks;   // pipeline stages of this workgroup

    const unsigned ring_off = (unsigned)(size_t)ring;
    const unsigned bias_off = (unsigned)(size_t)&bias_ring[0][0];
    const unsigned vimg_off = (unsigned)(size_t)vimg;

    // The bf16 copies are stored as 1 KB tiles (16 rows x 32 coordinates, already swizzled); the sixteen
    // tiles of a group of 256 rows at one chunk are contiguous (16 KB) and the chunks of a group follow
    // each other: a stage is ROWS/16 linear 1 KB copies, PPW consecutive ones per wave (pieces w PPW + q;
    // 0..15 streamed rows, then the resident rows), so a wave's loads of a stage, and of the next, walk
    // through memory linearly.
    const unsigned char *res_tiles = reinterpret_cast<const unsigned char *>(a.res) +
                                     (((int64_t)(row0 >> 8) * n_chunks * 16 + ((row0 >> 4) & 15)) << 10);
    const unsigned char *str_tiles = reinterpret_cast<const unsigned char *>(a.str);
    const unsigned l16 = l * 16, l4 = l * 4;

    int pg = 0, pch = 0, pt = t_begin;   // next stage this wave issues: number, chunk, tile
    // This wave's share of the next stage: PPW consecutive pieces starting at piece w PPW, i.e. one run of the
    // streamed group and / or one of the resident group; with the first stage of a tile also the wave's quarter of the
    // tile's biases (with two waves per streamed quarter both write the same 256 bytes: harmless).
    auto issue_stage = [&]() {
        if (pch == 0) dma4s(a.bias + (int64_t)pt * BI + wi * 64, l4, bias_off + ((pt - t_begin) & (NBIAS - 1)) * (BI * 4) + wi * 256);
        const int s0 = w * PPW;
        const int n_str = s0 >= 16 ? 0 : (16 - s0 < PPW ? 16 - s0 : PPW);
        const unsigned lds = ring_off + (pg % NS) * STAGE_BYTES;
        if (n_str > 0)
            dma16_run_n(n_str, str_tiles + ((((int64_t)pt * n_chunks + pch) * 16 + s0) << 10), l16, lds + s0 * 1024);
        if (n_str < PPW)
            dma16_run_n(PPW - n_str, res_tiles + (((int64_t)pch * 16 + (s0 + n_str - 16)) << 10), l16, lds + (s0 + n_str) * 1024);
        ++pg;
        if (++pch == n_chunks) {
            pch = 0;
            ++pt;
        }
    };

    float mrun[JTW], srun[JTW];
    f16v O[APPLY ? JTW : 1][NCB];
#pragma unroll
    for (int jt = 0; jt < JTW; ++jt) {
        mrun[jt] = kNegInit;
        srun[jt] = 0.0f;
    }
    if constexpr (APPLY) {
#pragma unroll
        for (int jt = 0; jt < JTW; ++jt)
#pragma unroll
            for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                for (int r = 0; r < 16; ++r) O[jt][cb][r] = 0.0f;
    }

    // fragment addressing inside a stage
    const int sw = (lr >> 2) & 3;
    const int offA = (64 * wi + lr) * 64, offB = (BI + 32 * JTW * wj + lr) * 64;
    const int pk0 = ((0 + lh) ^ sw) * 16, pk1 = ((2 + lh) ^ sw) * 16;
    bf8 a0[2], b0[JTW], a1[2], b1[JTW];
    auto read_frags = [&](bf8(&af)[2], bf8(&bf)[JTW], int stage, int pk) {
        const unsigned char *sb = ring + (stage % NS) * STAGE_BYTES + pk;
#pragma unroll
        for (int it = 0; it < 2; ++it) af[it] = *reinterpret_cast<const bf8 *>(sb + offA + it * 32 * 64);
#pragma unroll
        for (int jt = 0; jt < JTW; ++jt) bf[jt] = *reinterpret_cast<const bf8 *>(sb + offB + jt * 32 * 64);
    };
    // this wave's loads of stage `upto` and older have landed, given that it has issued stages up to `issued`
    // (loads of a value image issued in between only make these waits stricter)
    auto wait_landed = [&](int upto, int issued) {
        const int newer = issued - upto;   // whole stages issued after `upto`
        // (a stage has PPW loads of this wave, the first stage of a tile one more: counting PPW per newer stage
        // can only wait for more than necessary)
        if (newer >= 2)
            wait_vm<2 * PPW>();
        else if (newer == 1)
            wait_vm<PPW>();
        else
            wait_vm<0>();
    };
    int vstamp = 0;   // pg when this wave issued its pieces of the current tile's value image
    auto issue_vimg = [&](int t) {
        if constexpr (APPLY) {
            const unsigned char *src = reinterpret_cast<const unsigned char *>(a.vimg) + (int64_t)t * VIMG;
            // consecutive pieces per wave, in runs of up to four behind one LDS base each
            constexpr int VPW = (NVP + NW - 1) / NW;
            const int p0 = w * VPW;
            const int cnt = p0 >= NVP ? 0 : (NVP - p0 < VPW ? NVP - p0 : VPW);
#pragma unroll
            for (int r0 = 0; r0 < VPW; r0 += 4) {
                const int n = cnt - r0 < 4 ? cnt - r0 : 4;
                if (n > 0) dma16_run_n(n, src + (p0 + r0) * 1024, l16, vimg_off + (p0 + r0) * 1024);
            }
            vstamp = pg;
        }
    };

    // ---- prologue: D stages in flight, stage 0 landed, its first fragments on the way ----
    while (pg < D && pg < G) issue_stage();
    wait_landed(0, pg - 1);
    lds_done_barrier();
    read_frags(a0, b0, 0, pk0);

    int g = 0;
    for (int t = t_begin; t < t_end; ++t) {
        f16v acc[2][JTW];
        if constexpr (APPLY) {
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int jt = 0; jt < JTW; ++jt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[it][jt][r] = 0.0f;
        }

        if constexpr (!APPLY) {
            // One stage of the LSE pass.  The first chunk of a tile has a code copy of its own, in which the first
            // eight MFMAs start from a zero accumulator operand: no registers to clear per tile.
            //     4 MFMA on F0(g) | read F1(g), issue stage g+3 | 4 MFMA on F0(g) | 4 MFMA on F1(g) |
            //     wait "stage g+1 landed" + barrier | read F0(g+1) | 4 MFMA on F1(g)
            // Stage g + D goes to the ring slot of stage g - 1, which nobody reads any more: every
            // wave had its reads of that stage back before it passed the barrier of stage g - 1.
            auto stage = [&](auto first_c, auto half_c) {
                constexpr bool FIRST = decltype(first_c)::value;
                constexpr bool skip_second = decltype(half_c)::value;
                const f16v zero = {0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f, 0.0f};
#define FS_MFMA0(IT, JT) acc[IT][JT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0[IT], b0[JT], FIRST ? zero : acc[IT][JT], 0, 0, 0)
#define FS_MFMA1(IT, JT) acc[IT][JT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1[IT], b1[JT], acc[IT][JT], 0, 0, 0)
                // (only F0(g) is pending here, so the wait the compiler puts before the first MFMA is
                // exactly "F0 has arrived"; F1 is requested behind the first MFMA group)
                FS_MFMA0(0, 0);
                FS_MFMA0(0, 1);
                FS_MFMA0(0, 2);
                FS_MFMA0(0, 3);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!skip_second) read_frags(a1, b1, g, pk1);
                if (g + D < G) issue_stage();
                __builtin_amdgcn_sched_barrier(0);
                FS_MFMA0(1, 0);
                FS_MFMA0(1, 1);
                FS_MFMA0(1, 2);
                FS_MFMA0(1, 3);
                // (the second 16 coordinates of a tile's last chunk are zero padding when d ends in its first half:
                // 784 = 49 x 16 saves 2 % of the MFMAs this way)
                if constexpr (!skip_second) {
                    FS_MFMA1(0, 0);
                    FS_MFMA1(0, 1);
                    FS_MFMA1(0, 2);
                    FS_MFMA1(0, 3);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (g + 1 < G) {
                    wait_landed(g + 1, pg - 1);   // this wave's pieces of stage g+1 have landed ...
                    lds_done_barrier();           // ... and after the barrier everybody's; F0 may be refilled
                    read_frags(a0, b0, g + 1, pk0);
                }
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (!skip_second) {
                    FS_MFMA1(1, 0);
                    FS_MFMA1(1, 1);
                    FS_MFMA1(1, 2);
                    FS_MFMA1(1, 3);
                }
#undef FS_MFMA0
#undef FS_MFMA1
                ++g;
            };
            using yes = std::integral_constant<bool, true>;
            using no = std::integral_constant<bool, false>;
            // (HALF: the launcher has checked that d ends in the first 16 coordinates of the last chunk and that a
            // tile has at least two chunks; the three code copies follow each other without a branch between them)
            stage(yes{}, no{});
            if constexpr (HALF) {
                for (int ch = 1; ch + 1 < n_chunks; ++ch) stage(no{}, no{});
                stage(no{}, yes{});
            } else {
                for (int ch = 1; ch < n_chunks; ++ch) stage(no{}, no{});
            }
        }
        for (int ch = 0; APPLY && ch < n_chunks; ++ch, ++g) {
            const bool issue = g + D < G;
#define FS_MFMA(IT, JT, AF, BF) acc[IT][JT] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(AF[IT], BF[JT], acc[IT][JT], 0, 0, 0)
#define FS_PIECE(Q)                          \
    __builtin_amdgcn_sched_barrier(0);       \
    if (Q == 0 && issue) issue_stage();      \
    __builtin_amdgcn_sched_barrier(0)
            // (plan application: 64 x 64 scores per wave)
            //     2 MFMA on F0(g) | read F1(g), issue stage g+3 | 2 MFMA on F0(g) | 2 MFMA on F1(g) |
            //     wait "stage g+1 landed" + barrier | read F0(g+1) | 2 MFMA on F1(g)
            static_assert(!APPLY || JTW == 2, "schedule of the application");
            FS_MFMA(0, 0, a0, b0);
            FS_MFMA(0, 1, a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            read_frags(a1, b1, g, pk1);
            FS_PIECE(0);
            FS_MFMA(1, 0, a0, b0);
            FS_MFMA(1, 1, a0, b0);
            FS_MFMA(0, 0, a1, b1);
            FS_MFMA(0, 1, a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            if (g + 1 < G) {
                // this wave's pieces of stage g+1 have landed ...
                wait_landed(g + 1, pg - 1);
                // ... and after the barrier everybody's; F0 may be refilled
                lds_done_barrier();
                read_frags(a0, b0, g + 1, pk0);
            }
            if constexpr (APPLY) {
                // every wave is past the previous tile's use of the value image now
                if (ch == 0) {
                    if (g + 1 >= G) lds_done_barrier();
                    issue_vimg(t);
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            FS_MFMA(1, 0, a1, b1);
            FS_MFMA(1, 1, a1, b1);
#undef FS_MFMA
#undef FS_PIECE
        }

        // ---- epilogue: fold 2 x 16 streamed points per resident row into (max, sum) ----------
        // lazy stabiliser: exponents against the current integer running max; the slow branch
        // (lift the max, rescale by an exact power of two) runs only when a sum leaves [0, 2^60)
        const int bslot = (t - t_begin) & (NBIAS - 1);   // the first stage of this tile carried its biases
        float bias[2][16];
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float4 bv = *reinterpret_cast<const float4 *>(&bias_ring[bslot][64 * wi + 32 * it + 8 * g4 + 4 * lh]);
                bias[it][4 * g4 + 0] = bv.x;
                bias[it][4 * g4 + 1] = bv.y;
                bias[it][4 * g4 + 2] = bv.z;
                bias[it][4 * g4 + 3] = bv.w;
            }
        if constexpr (!APPLY) {
            float csum[JTW];
            bool bad = false;
#pragma unroll
            for (int jt = 0; jt < JTW; ++jt) {
                const float m = mrun[jt];
                float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    s0 += fast_exp2(fmaf(acc[0][jt][r], a.cscale, bias[0][r]) - m);
                    s1 += fast_exp2(fmaf(acc[1][jt][r], a.cscale, bias[1][r]) - m);
                }
                csum[jt] = s0 + s1;
                bad = bad || !(csum[jt] < kLazyMax);
            }
            if (__any(bad)) {
#pragma unroll
                for (int jt = 0; jt < JTW; ++jt) {
                    float mx = kNegInit;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        mx = fmaxf(mx, fmaf(acc[0][jt][r], a.cscale, bias[0][r]));
                        mx = fmaxf(mx, fmaf(acc[1][jt][r], a.cscale, bias[1][r]));
                    }
                    float mnew = fmaxf(mrun[jt], ceilf(mx));
                    float s0 = 0.0f, s1 = 0.0f;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        s0 += fast_exp2(fmaf(acc[0][jt][r], a.cscale, bias[0][r]) - mnew);
                        s1 += fast_exp2(fmaf(acc[1][jt][r], a.cscale, bias[1][r]) - mnew);
                    }
                    csum[jt] = s0 + s1;
                    srun[jt] *= fast_exp2(mrun[jt] - mnew);
                    mrun[jt] = mnew;
                }
            }
#pragma unroll
            for (int jt = 0; jt < JTW; ++jt) srun[jt] += csum[jt];
        } else {
            // scores in place of the accumulators
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int jt = 0; jt < JTW; ++jt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[it][jt][r] = fmaf(acc[it][jt][r], a.cscale, bias[it][r]);
            // the stabiliser must keep every exponential representable in bf16 next to the row's
            // largest one and the fp32 sums finite: lift it when a score exceeds it by more than 60
            bool lift = false;
            float mx[JTW];
#pragma unroll
            for (int jt = 0; jt < JTW; ++jt) {
                float m = kNegInit;
#pragma unroll
                for (int r = 0; r < 16; ++r) m = fmaxf(m, fmaxf(acc[0][jt][r], acc[1][jt][r]));
                m = fmaxf(m, __shfl_xor(m, 32, 64));   // common to the two lane halves of the row
                mx[jt] = m;
                lift = lift || (m > mrun[jt] + 60.0f);
            }
            if (__any(lift)) {
#pragma unroll
                for (int jt = 0; jt < JTW; ++jt) {
                    const float mnew = fmaxf(mrun[jt], ceilf(mx[jt]));
                    const float scale = fast_exp2(mrun[jt] - mnew);   // exact power of two (or 0)
                    srun[jt] *= scale;
                    mrun[jt] = mnew;
                    // accumulator column n = lr is this lane's resident row: one factor per lane
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) O[jt][cb][r] *= scale;
                }
            }
            // this wave's pieces of the value image have landed, then everybody's
            {
                const int newer = pg - vstamp;
                if (newer >= 2)
                    wait_vm<2 * PPW>();
                else if (newer == 1)
                    wait_vm<PPW>();
                else
                    wait_vm<0>();
            }
            lds_done_barrier();
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int s = 0; s < 2; ++s) {
                    // A fragments: Vt[c = 32 cb + lr][the eight streamed points of this lane half]
                    bf8 vf[NCB];
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb) {
                        const unsigned char *vp = vimg + (32 * cb + lr) * kVRow + 2 * (64 * wi + 32 * it + 16 * s + 4 * lh);
                        const uint2 lo = *reinterpret_cast<const uint2 *>(vp);
                        const uint2 hi = *reinterpret_cast<const uint2 *>(vp + 16);
                        const uint4 u = make_uint4(lo.x, lo.y, hi.x, hi.y);
                        vf[cb] = *reinterpret_cast<const bf8 *>(&u);
                    }
#pragma unroll
                    for (int jt = 0; jt < JTW; ++jt) {
                        bf8 e;
                        float part = 0.0f;
#pragma unroll
                        for (int q = 0; q < 8; ++q) {
                            const float ev = fast_exp2(acc[it][jt][8 * s + q] - mrun[jt]);
                            part += ev;
                            e[q] = (__bf16)ev;
                        }
                        srun[jt] += part;
#pragma unroll
                        for (int cb = 0; cb < NCB; ++cb)
                            O[jt][cb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[cb], e, O[jt][cb], 0, 0, 0);
                    }
                }
        }
    }

    // ---- merge the 2 lane halves x 4 streamed-side waves of every resident row -------------
    lds_done_barrier();   // the ring is free: reuse it for the merge
    float2 *red = reinterpret_cast<float2 *>(ring);   // [BJ][8]: 4 streamed-side waves x 2 lane halves per row
#pragma unroll
    for (int jt = 0; jt < JTW; ++jt)
        red[(32 * JTW * wj + 32 * jt + lr) * 8 + 2 * wi + lh] = make_float2(mrun[jt], srun[jt]);
    __syncthreads();
    if constexpr (APPLY) {
        // output accumulators: scaled to the row's common max and added wave by wave (fixed order)
        float *obuf = reinterpret_cast<float *>(ring + BJ * 64);   // [BJ][PC]
        for (int ww = 0; ww < 4; ++ww) {
            if (wi == ww) {
#pragma unroll
                for (int jt = 0; jt < JTW; ++jt) {
                    const int j = 32 * JTW * wj + 32 * jt + lr;
                    float M = kNegInit;
#pragma unroll
                    for (int k = 0; k < 8; ++k) M = fmaxf(M, red[j * 8 + k].x);
                    const float sc = fast_exp2(mrun[jt] - M);
#pragma unroll
                    for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int cc = 32 * cb + 8 * (r >> 2) + 4 * lh + (r & 3);
                            const float v = O[jt][cb][r] * sc;
                            obuf[j * PC + cc] = ww == 0 ? v : obuf[j * PC + cc] + v;
                        }
                }
            }
            __syncthreads();
        }
        for (int e = tid; e < BJ * PC; e += 256 * WJ) {
            const int j = e / PC, cc = e - j * PC;
            a.opart[((int64_t)split * a.partial_stride + row0 + j) * PC + cc] = obuf[e];
        }
    }
    if (tid < BJ) {
        float M = kNegInit;
#pragma unroll
        for (int k = 0; k < 8; ++k) M = fmaxf(M, red[tid * 8 + k].x);
        double S = 0.0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            float2 q = red[tid * 8 + k];
            S += (double)(q.y * fast_exp2(q.x - M));
        }
        a.partial[(int64_t)split * a.partial_stride + row0 + tid] = make_double2((double)M, S);
    }
}

template <int WJ, int NS, int JTW, int PC, bool HALF = false>
__global__ __launch_bounds__(256 * WJ, WJ == 2 ? 1 : 2) void k_lse_bf16(BfArgs a)
{
    lse_bf16_body<WJ, NS, JTW, PC, HALF>(a, blockIdx.x);
}

// Both LSE passes of one iteration of the averaged schedule (Eq. 4-5) in one launch: the first `blocks0`
// workgroups (a multiple of 8, so that the dealing to XCDs is the same as in a launch of its own) run the
// f-pass, the others the g-pass.
template <int WJ, int NS, int JTW>
__global__ __launch_bounds__(256 * WJ, WJ == 2 ? 1 : 2) void k_lse_bf16_pair(BfArgs a0, BfArgs a1, int blocks0)
{
    const bool second = (int)blockIdx.x >= blocks0;   // uniform over the workgroup
    lse_bf16_body<WJ, NS, JTW, 0>(second ? a1 : a0, (int)blockIdx.x - (second ? blocks0 : 0));
}

// Value image of every streamed tile for the plan application: bf16 Vt[c][i], c < pc value columns
// starting at p0, i < 256 points of tile t, rows of kVRow bytes, one image per img_bytes; zero
// outside the matrix.  (The pad bytes are copied to LDS with the rest and never read.)
__global__ __launch_bounds__(BI) void k_vimg_bf16(const float *V, int64_t ldv, int64_t n_str, int p0, int p, int pc,
                                                   int img_bytes, unsigned char *img)
{
    const int i = threadIdx.x;
    const int64_t row = (int64_t)blockIdx.x * BI + i;
    unsigned char *dst = img + (int64_t)blockIdx.x * img_bytes;
    for (int cc = 0; cc < pc; ++cc) {
        const float v = (row < n_str && p0 + cc < p) ? V[row * ldv + p0 + cc] : 0.0f;
        *reinterpret_cast<__bf16 *>(dst + cc * kVRow + 2 * i) = (__bf16)v;
    }
}

// Number of splits of the streamed side that minimises  rounds x tiles-per-workgroup
// (rounds = ceil(workgroups / workgroups the chip holds at a time)), i.e. the time including the
// idle tail of the last round; prefer fewer, longer workgroups on near-ties.
int choose_splits(const Ctx *c, int n_jtiles, int n_itiles, int cap, int per_cu)
{
    int best_s = 1;
    double best_cost = 1e300;
    const int smax = n_itiles < cap ? n_itiles : cap;
    for (int sp = 1; sp <= smax; ++sp) {
        int tps = (int)ceil_div(n_itiles, sp);
        int seff = (int)ceil_div(n_itiles, tps);
        if (seff != sp) continue;
        double rounds = (double)ceil_div((int64_t)n_jtiles * seff, (int64_t)c->num_cu * per_cu);
        double cost = rounds * (tps + 0.25);   // 0.25: pipeline fill and merge of a workgroup
        if (cost < best_cost * 0.99) {
            best_cost = cost;
            best_s = sp;
        }
    }
    return best_s;
}

constexpr int kApplyPC = 64;    // value columns per application pass
constexpr int kApplyPCWide = 96;   // ... when there are more than 64 (every pass repeats the score contraction)
constexpr int kApplyBJ = 128;   // resident rows per workgroup of the application kernel

}  // namespace

// arguments of an LSE pass (res resident, str streamed) writing its records to `partial`; *blocks = its grid
static fs_status lse_pass_args(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, void *partial, BfArgs *out,
                               int *blocks)
{
    // (a 256 x 128 workgroup tile, two workgroups per CU, was measured slower and is not built)
    const int bj = 256, per_cu = 1;
    BfArgs a{};
    a.res = res->pts_b;
    a.str = str->pts_b;
    a.bias = str->bias_f;
    a.kp = P->kp;
    a.cscale = (float)(2.0 * kLog2e / eps);
    a.n_jtiles = (int)ceil_div(res->cnt, bj);
    a.n_itiles = (int)ceil_div(str->cnt, BI);
    a.splits = choose_splits(c, a.n_jtiles, a.n_itiles, max_splits(c->partial_budget, res->cnt), per_cu);
    a.tiles_per_split = (int)ceil_div(a.n_itiles, a.splits);
    const int total = a.n_jtiles * a.splits;
    a.partial = (double2 *)partial;
    a.partial_stride = res->cnt_pad;
    if ((int64_t)a.n_jtiles * bj > res->cnt_pad || (int64_t)a.n_itiles * BI > str->cnt_pad ||
        (size_t)a.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp & 31) != 0 || a.kp < 32)
        return fail(c, FS_ERR_DEVICE, "internal: bf16 launch shape exceeds the padded buffers");
    *out = a;
    *blocks = (total + 7) / 8 * 8;
    return FS_OK;
}

fs_status bf16_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out)
{
    BfArgs a;
    int blocks = 0;
    fs_status st = lse_pass_args(c, P, res, str, eps, P->partial, &a, &blocks);
    if (st != FS_OK) return st;
    // the coordinates end in the first 16 of a tile's last chunk (d = 784 = 49 x 16): the kernel copy that leaves
    // out that chunk's second, all-zero k-step (2 % of the MFMAs at d = 784)
    const bool half = (P->d % 32) >= 1 && (P->d % 32) <= 16 && a.kp >= 64;
    prof_begin(c, (double)res->cnt * (double)str->cnt);
    if (half)
        hipLaunchKernelGGL((k_lse_bf16<2, 4, 4, 0, true>), dim3((unsigned)blocks), dim3(512), 0, c->stream, a);
    else
        hipLaunchKernelGGL((k_lse_bf16<2, 4, 4, 0>), dim3((unsigned)blocks), dim3(512), 0, c->stream, a);
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = a.splits;
    return FS_OK;
}

// The f-pass (records to partial_x) and the g-pass (records to partial_y) of one iteration of the averaged
// schedule (Eq. 4-5) in ONE launch.
fs_status bf16_lse_pair(Ctx *c, const Prepared *P, double eps, void *partial_x, void *partial_y, int *splits_x, int *splits_y)
{
    BfArgs ax, ay;
    int bx = 0, by = 0;
    fs_status st;
    if ((st = lse_pass_args(c, P, &P->X, &P->Y, eps, partial_x, &ax, &bx)) != FS_OK) return st;
    if ((st = lse_pass_args(c, P, &P->Y, &P->X, eps, partial_y, &ay, &by)) != FS_OK) return st;
    if (bx + by <= 4 * c->num_cu) {
        prof_begin(c, 2.0 * (double)P->X.cnt * (double)P->Y.cnt);
        hipLaunchKernelGGL((k_lse_bf16_pair<2, 4, 4>), dim3((unsigned)(bx + by)), dim3(512), 0, c->stream, ax, ay, bx);
        prof_end(c);
    } else {
        // many rounds of workgroups: one launch saves nothing there, and two passes of different shape in one
        // grid share the L2 of an XCD worse than one after the other (n = 50000, m = 20000, d = 1024: 4 % slower)
        prof_begin(c, (double)P->X.cnt * (double)P->Y.cnt);
        hipLaunchKernelGGL((k_lse_bf16<2, 4, 4, 0>), dim3((unsigned)bx), dim3(512), 0, c->stream, ax);
        prof_end(c);
        prof_begin(c, (double)P->X.cnt * (double)P->Y.cnt);
        hipLaunchKernelGGL((k_lse_bf16<2, 4, 4, 0>), dim3((unsigned)by), dim3(512), 0, c->stream, ay);
        prof_end(c);
    }
    FS_HIP(c, hipGetLastError());
    *splits_x = ax.splits;
    *splits_y = ay.splits;
    return FS_OK;
}

// workspace of bf16_apply: [splits][rows][kApplyPC] float accumulators, then the value images
size_t bf16_apply_ws(const Ctx *c, int64_t n_res, int64_t n_str)
{
    const int n_jtiles = (int)ceil_div(n_res, kApplyBJ), n_itiles = (int)ceil_div(n_str, BI);
    const int splits = choose_splits(c, n_jtiles, n_itiles, max_splits(c->partial_budget, n_res), 1);
    const size_t opart = (size_t)splits * (size_t)round_up(n_res, 1024) * kApplyPCWide * 4;
    return ((opart + 1023) & ~size_t(1023)) + (size_t)n_itiles * kVImgBytes(kApplyPCWide);
}

fs_status bf16_apply(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, const float *V, int64_t p,
                     int64_t ldv, float *out, int64_t ldo, float *mass_out)
{
    BfArgs a{};
    a.res = res->pts_b;
    a.str = str->pts_b;
    a.bias = str->bias_f;
    a.kp = P->kp;
    a.cscale = (float)(2.0 * kLog2e / eps);
    a.n_jtiles = (int)ceil_div(res->cnt, kApplyBJ);
    a.n_itiles = (int)ceil_div(str->cnt, BI);
    a.splits = choose_splits(c, a.n_jtiles, a.n_itiles, max_splits(c->partial_budget, res->cnt), 1);
    a.tiles_per_split = (int)ceil_div(a.n_itiles, a.splits);
    a.partial = (double2 *)P->partial;
    a.partial_stride = res->cnt_pad;
    // 96 columns per pass when there are more than 64 (the registers allow three 32-column accumulator blocks), 64 else
    const int pc = p > kApplyPC ? kApplyPCWide : kApplyPC;
    const size_t opart_bytes = ((size_t)a.splits * res->cnt_pad * pc * 4 + 1023) & ~size_t(1023);
    const size_t vimg_bytes = (size_t)a.n_itiles * kVImgBytes(pc);
    a.opart = reinterpret_cast<float *>(P->extra);
    unsigned char *vimg = reinterpret_cast<unsigned char *>(P->extra) + opart_bytes;
    a.vimg = vimg;
    // host-side shape checks: every access of the kernels stays inside the padded buffers
    if ((int64_t)a.n_jtiles * kApplyBJ > res->cnt_pad || (int64_t)a.n_itiles * BI > str->cnt_pad ||
        (size_t)a.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp & 31) != 0 || a.kp < 32 ||
        opart_bytes + vimg_bytes > P->extra_bytes || !P->extra)
        return fail(c, FS_ERR_DEVICE, "internal: bf16 apply launch shape exceeds the padded buffers");
    const int total = a.n_jtiles * a.splits;
    const int per = (total + 7) / 8;
    for (int p0 = 0; p0 < p; p0 += pc) {
        hipLaunchKernelGGL(k_vimg_bf16, dim3((unsigned)a.n_itiles), dim3(BI), 0, c->stream, V, ldv, str->cnt, p0, (int)p, pc,
                           kVImgBytes(pc), vimg);
        if (pc == kApplyPCWide)
            hipLaunchKernelGGL((k_lse_bf16<2, 4, 2, kApplyPCWide>), dim3((unsigned)(per * 8)), dim3(512), 0, c->stream, a);
        else
            hipLaunchKernelGGL((k_lse_bf16<2, 4, 2, kApplyPC>), dim3((unsigned)(per * 8)), dim3(512), 0, c->stream, a);
        FS_HIP(c, hipGetLastError());
        fs_status st = launch_apply_finalize(c, P, res, res->norm, a.splits, eps, a.opart, pc, p0, (int)p, out, ldo, mass_out);
        if (st != FS_OK) return st;
    }
    return FS_OK;
}

}  // namespace fs
