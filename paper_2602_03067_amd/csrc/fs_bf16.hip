// bf16 matrix-core path (d >= 16): the score tile 2<x_i, y_j> of Alg. 1 / Alg. 3 is a dense
// contraction over d, computed with v_mfma_f32_32x32x16_bf16 (bf16 in, fp32 accumulate); bias,
// online LSE and potentials stay in fp32/fp64.
//
// Shape of the work.  A resident row block at d = 784..1024 does not fit on chip (256 rows x
// 800 x 2 B = 400 KB), so unlike Alg. 1 the pass is organised as a GEMM with an LSE epilogue:
// a workgroup owns 256 resident rows (j) and a group of streamed tiles (i); for every streamed
// tile of 128 points it runs the full contraction over d in chunks of 64 through LDS, then folds
// the 128 x 256 scores into the per-row running (max, sum).  Groups of streamed tiles ("splits")
// are merged afterwards.  Concurrent workgroups of one XCD form 8 x 8 super-tiles, so each panel
// chunk fetched into that XCD's L2 is shared by eight workgroups.
//
// MFMA operand roles (32x32x16): A = streamed points (i), B = resident rows (j);
//   A: lane l holds A[i = l%32][k = 8*(l/32) .. +7],  B likewise with j = l%32,
//   D: lane l, register r holds D[i = 8*(r/4) + 4*(l/32) + r%4][j = l%32],
// i.e. the 16 accumulator registers of a lane are 16 streamed points of ONE resident row, so
// the row-wise LSE runs inside the lane; lanes/waves are merged once per workgroup.
#include "fs_internal.h"

namespace fs {
namespace {

typedef __bf16 bf8 __attribute__((ext_vector_type(8)));
typedef float f16v __attribute__((ext_vector_type(16)));

constexpr int BI = 128;          // streamed points per tile (2 waves x 64)
constexpr int BJ = 256;          // resident rows per workgroup (2 waves x 128)
constexpr int KC = 64;           // contraction chunk (bf16 elements)
constexpr int ROWB = KC * 2 + 16;   // LDS bytes per row: 128 data + 16 pad -> conflict-free b128 reads
constexpr int PIECES = (BI + BJ) * (KC * 2 / 16) / 256;   // 16-byte pieces per thread per chunk = 12

__device__ inline float fast_exp2(float v) { return __builtin_amdgcn_exp2f(v); }

struct BfArgs {
    const uint16_t *res;     // [res_pad][kp] bf16
    const uint16_t *str;     // [str_pad][kp] bf16
    const float *bias;       // [str_pad] base-2 bias of the streamed points (-inf on padding)
    int kp;                  // multiple of 32
    float cscale;            // 2 log2(e) / eps
    int n_jtiles, n_itiles, splits, tiles_per_split;
    int work_per_xcd;        // work items assigned to one XCD (contiguous range)
    double2 *partial;
    int64_t partial_stride;
};

__global__ __launch_bounds__(256, 2) void k_lse_bf16(BfArgs a)
{
    __shared__ __attribute__((aligned(16))) unsigned char lds[(BI + BJ) * ROWB];   // 55,296 B
    __shared__ float bias_lds[BI];
    __shared__ float2 red[BJ][4];

    // ---- which (resident tile, split) this workgroup owns: XCD-contiguous, 8 x 8 super-tiles
    const int b = blockIdx.x;
    const int wk = (b & 7) * a.work_per_xcd + (b >> 3);
    const int sj = (a.n_jtiles + 7) >> 3;
    const int sup = wk >> 6, within = wk & 63;
    const int jtile = (sup % sj) * 8 + (within & 7);
    const int split = (sup / sj) * 8 + (within >> 3);
    if ((b >> 3) >= a.work_per_xcd || jtile >= a.n_jtiles || split >= a.splits) return;

    const int tid = threadIdx.x;
    const int w = tid >> 6, l = tid & 63;
    const int wi = w & 1, wj = w >> 1;
    const int lh = l >> 5, lr = l & 31;
    const int kp = a.kp;
    const int n_chunks = (kp + KC - 1) / KC;
    const int64_t row0 = (int64_t)jtile * BJ;

    float mrun[4], srun[4];
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) {
        mrun[jt] = kNegInit;
        srun[jt] = 0.0f;
    }

    // per-thread pieces of a chunk: piece e = tid + 256 q covers row e/8, bytes (e%8)*16..+15
    const int t_begin = split * a.tiles_per_split;
    const int t_end = min(a.n_itiles, t_begin + a.tiles_per_split);

    for (int t = t_begin; t < t_end; ++t) {
        const int64_t col0 = (int64_t)t * BI;
        f16v acc[2][4];
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int jt = 0; jt < 4; ++jt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[it][jt][r] = 0.0f;

        uint4 pre[PIECES];
        auto load_chunk = [&](int ch) {
            const int kc0 = ch * KC;
            const int kw16 = min(KC, kp - kc0) >> 3;   // valid 16-byte pieces per row (4 or 8)
#pragma unroll
            for (int q = 0; q < PIECES; ++q) {
                int e = tid + 256 * q;
                int row = e >> 3, part = e & 7;
                const uint16_t *src = row < BI ? a.str + (col0 + row) * kp : a.res + (row0 + row - BI) * kp;
                uint4 v = make_uint4(0u, 0u, 0u, 0u);
                if (part < kw16) v = *reinterpret_cast<const uint4 *>(src + kc0 + part * 8);
                pre[q] = v;
            }
        };
        load_chunk(0);

        for (int ch = 0; ch < n_chunks; ++ch) {
            __syncthreads();   // everyone is done reading the previous chunk
#pragma unroll
            for (int q = 0; q < PIECES; ++q) {
                int e = tid + 256 * q;
                *reinterpret_cast<uint4 *>(lds + (e >> 3) * ROWB + (e & 7) * 16) = pre[q];
            }
            if (ch == 0 && tid < BI) bias_lds[tid] = a.bias[col0 + tid];
            __syncthreads();
            if (ch + 1 < n_chunks) load_chunk(ch + 1);

            const int ksteps = min(KC, kp - ch * KC) >> 4;   // 2 or 4
            const unsigned char *pa = lds + (64 * wi + lr) * ROWB + lh * 16;
            const unsigned char *pb = lds + (BI + 128 * wj + lr) * ROWB + lh * 16;
            for (int ks = 0; ks < ksteps; ++ks) {
                bf8 af[2], bfr[4];
#pragma unroll
                for (int it = 0; it < 2; ++it)
                    af[it] = *reinterpret_cast<const bf8 *>(pa + it * 32 * ROWB + ks * 32);
#pragma unroll
                for (int jt = 0; jt < 4; ++jt)
                    bfr[jt] = *reinterpret_cast<const bf8 *>(pb + jt * 32 * ROWB + ks * 32);
#pragma unroll
                for (int it = 0; it < 2; ++it)
#pragma unroll
                    for (int jt = 0; jt < 4; ++jt)
                        acc[it][jt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[it], bfr[jt], acc[it][jt], 0, 0, 0);
            }
        }

        // ---- epilogue: fold 2 x 16 streamed points per resident row into (max, sum) ----------
        float bias[2][16];
#pragma unroll
        for (int it = 0; it < 2; ++it)
#pragma unroll
            for (int g4 = 0; g4 < 4; ++g4) {
                float4 bv = *reinterpret_cast<const float4 *>(&bias_lds[64 * wi + 32 * it + 8 * g4 + 4 * lh]);
                bias[it][4 * g4 + 0] = bv.x;
                bias[it][4 * g4 + 1] = bv.y;
                bias[it][4 * g4 + 2] = bv.z;
                bias[it][4 * g4 + 3] = bv.w;
            }
#pragma unroll
        for (int jt = 0; jt < 4; ++jt) {
            float sc[2][16];
            float mx = kNegInit;
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; r += 2) {
                    sc[it][r] = fmaf(acc[it][jt][r], a.cscale, bias[it][r]);
                    sc[it][r + 1] = fmaf(acc[it][jt][r + 1], a.cscale, bias[it][r + 1]);
                    mx = fmaxf(mx, fmaxf(sc[it][r], sc[it][r + 1]));
                }
            float mnew = fmaxf(mrun[jt], ceilf(mx));
            float scale = fast_exp2(mrun[jt] - mnew);
            float csum = 0.0f;
#pragma unroll
            for (int it = 0; it < 2; ++it)
#pragma unroll
                for (int r = 0; r < 16; ++r) csum += fast_exp2(sc[it][r] - mnew);
            srun[jt] = fmaf(srun[jt], scale, csum);
            mrun[jt] = mnew;
        }
    }

    // ---- merge the 2 lane halves x 2 streamed-side waves of every resident row -------------
#pragma unroll
    for (int jt = 0; jt < 4; ++jt) red[128 * wj + 32 * jt + lr][2 * wi + lh] = make_float2(mrun[jt], srun[jt]);
    __syncthreads();
    {
        float2 p0 = red[tid][0], p1 = red[tid][1], p2 = red[tid][2], p3 = red[tid][3];
        float M = fmaxf(fmaxf(p0.x, p1.x), fmaxf(p2.x, p3.x));
        double S = (double)(p0.y * fast_exp2(p0.x - M)) + (double)(p1.y * fast_exp2(p1.x - M)) +
                   (double)(p2.y * fast_exp2(p2.x - M)) + (double)(p3.y * fast_exp2(p3.x - M));
        a.partial[(int64_t)split * a.partial_stride + row0 + tid] = make_double2((double)M, S);
    }
}

}  // namespace

fs_status bf16_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits_out)
{
    BfArgs a{};
    a.res = res->pts_b;
    a.str = str->pts_b;
    a.bias = str->bias_f;
    a.kp = P->kp;
    a.cscale = (float)(2.0 * kLog2e / eps);
    a.n_jtiles = (int)ceil_div(res->cnt, BJ);
    a.n_itiles = (int)ceil_div(str->cnt, BI);
    // enough (resident tile, split) work items for ~8 rounds over 2 workgroups per CU
    int target = 16 * c->num_cu;
    int splits = (int)ceil_div(target, a.n_jtiles);
    if (splits > a.n_itiles) splits = a.n_itiles;
    if (splits > kMaxSplits) splits = kMaxSplits;
    if (splits < 1) splits = 1;
    a.tiles_per_split = (int)ceil_div(a.n_itiles, splits);
    a.splits = (int)ceil_div(a.n_itiles, a.tiles_per_split);
    const int sj = (a.n_jtiles + 7) / 8, sg = (a.splits + 7) / 8;
    const int work = sj * sg * 64;                 // super-tile grid, including idle corners
    a.work_per_xcd = (work + 7) / 8;
    a.partial = (double2 *)P->partial;
    a.partial_stride = res->cnt_pad;
    if ((int64_t)a.n_jtiles * BJ > res->cnt_pad || (int64_t)a.n_itiles * BI > str->cnt_pad ||
        (size_t)a.splits * res->cnt_pad * 16 > P->partial_bytes || (a.kp & 31) != 0 || a.kp < 32)
        return fail(c, FS_ERR_DEVICE, "internal: bf16 launch shape exceeds the padded buffers");
    prof_begin(c, (double)res->cnt * (double)str->cnt);
    hipLaunchKernelGGL(k_lse_bf16, dim3((unsigned)(a.work_per_xcd * 8)), dim3(256), 0, c->stream, a);
    prof_end(c);
    FS_HIP(c, hipGetLastError());
    *splits_out = a.splits;
    return FS_OK;
}

}  // namespace fs
