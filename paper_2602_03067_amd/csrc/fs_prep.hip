// O(n d) kernels around the streaming passes: derived copies of the point
// clouds and their squared norms (Prop. 1: alpha, beta), the per-point bias
// (Alg. 1, "precompute bias"), and the merge of the per-split LSE statistics into
// the new shifted potential.
#include "fs_internal.h"

namespace fs {
namespace {

__device__ inline float bf16_to_float(uint16_t h) { return __uint_as_float(((uint32_t)h) << 16); }

// round-to-nearest-even float -> bfloat16 bits (NaN kept quiet)
__device__ inline uint16_t float_to_bf16(float v)
{
    uint32_t u = __float_as_uint(v);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ inline float load_pt(const void *pts, int dtype, int64_t idx)
{
    return dtype == FS_BF16 ? bf16_to_float(((const uint16_t *)pts)[idx]) : ((const float *)pts)[idx];
}

// block-wide sum of one double per thread (blockDim.x == 256); result valid in thread 0
__device__ inline double block_sum_256(double v, double *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = 128; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    return sh[0];
}

__global__ void k_fill_f64(double *dst, double v, int64_t cnt)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cnt) dst[i] = v;
}

// ---- squared row norms, float64 accumulation --------------------------------------------
__global__ void k_row_norms(const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, float *out)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    double s = 0.0;
    for (int64_t k = 0; k < d; ++k) {
        double v = (double)load_pt(pts, dtype, i * ld + k);
        s += v * v;
    }
    out[i] = (float)s;
}

// ---- common mean of both clouds (low-d path), deterministic two-stage reduction ---------
// stage 1: block b writes the coordinate sums of its slice to part[b][0..15]
// (blockIdx.y: 0 = the x cloud, 1 = the y cloud)
struct CloudIn {
    const void *pts;
    int64_t rows, ld;
    double *part;
};
__global__ __launch_bounds__(256) void k_coord_sums(CloudIn c0, CloudIn c1, int dtype, int d)
{
    const CloudIn &cl = blockIdx.y ? c1 : c0;
    const void *pts = cl.pts;
    const int64_t rows = cl.rows, ld = cl.ld;
    double *part = cl.part;
    __shared__ double sh[256];
    double acc[kLowdMaxD];
    for (int k = 0; k < kLowdMaxD; ++k) acc[k] = 0.0;
    for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < rows; i += (int64_t)gridDim.x * 256)
        for (int k = 0; k < d; ++k) acc[k] += (double)load_pt(pts, dtype, i * ld + k);
    for (int k = 0; k < kLowdMaxD; ++k) {
        double t = block_sum_256(acc[k], sh);
        if (threadIdx.x == 0) part[(int64_t)blockIdx.x * kLowdMaxD + k] = t;
        __syncthreads();
    }
}

// stage 2: mean[k] = (sum of partX[.][k] + sum of partY[.][k]) / (n + m).  One block of 256: thread
// (group g, coordinate k) sums the blocks b = g mod 16, then coordinate k's 16 group sums are added
// in a fixed order.  Also clears zeroed[0..2] (the slots the next kernels take maxima into).
__global__ __launch_bounds__(256) void k_mean_final(const double *partX, const double *partY, int blocks, double inv_cnt,
                                                    double *mean, double *zeroed)
{
    static_assert(kLowdMaxD == 16, "thread mapping below");
    __shared__ double sh[16][kLowdMaxD];
    const int k = threadIdx.x & 15, g = threadIdx.x >> 4;
    double s = 0.0;
    for (int b = g; b < blocks; b += 16) s += partX[(int64_t)b * kLowdMaxD + k] + partY[(int64_t)b * kLowdMaxD + k];
    sh[g][k] = s;
    __syncthreads();
    if (threadIdx.x < kLowdMaxD) {
        double t = 0.0;
        for (int q = 0; q < 16; ++q) t += sh[q][threadIdx.x];
        mean[threadIdx.x] = t * inv_cnt;
    }
    if (threadIdx.x < 3) zeroed[threadIdx.x] = 0.0;
}

// piece d of a streamed-role split record: the bias in three bf16 pieces, then the three ones
// that pick up the resident row's (negated) running max
__device__ inline uint4 split_bias_piece(float bias)
{
    __bf16 b[3];
    split3(bias, b);
    const __bf16 one = (__bf16)1.0f;
    return make_uint4(bf16_pair(b[0], b[1]), bf16_pair(b[2], one), bf16_pair(one, one), 0u);
}

// ---- low-d derived copies: coordinates centred at the common mean, packed with a bias slot;
//      float (rounded once) and double (exact difference), each with its own squared norms ----
// (blockIdx.y: 0 = the x cloud, 1 = the y cloud; a cloud's cnt_pad is a multiple of the block size, so a
// block is either entirely inside it or leaves as a whole)
struct PrepLowdSide {
    const void *pts;
    int64_t cnt, cnt_pad, ld;
    float *packed;
    double *packed_d, *norm_f, *norm;
    uint16_t *split;
    double *pts_d, *bias_d;   // d > 3: records of the fp64 matrix-core pass ([cnt_pad][kp] centred coordinates, bias), else null
};
__global__ __launch_bounds__(256) void k_prep_lowd(PrepLowdSide s0, PrepLowdSide s1, int dtype, int d, int dp, int dpd, int kp,
                                                   const double *mean, int ks, unsigned long long *rho_max_bits)
{
    const PrepLowdSide &sd = blockIdx.y ? s1 : s0;
    if ((int64_t)blockIdx.x * 256 >= sd.cnt_pad) return;
    const void *pts = sd.pts;
    const int64_t cnt = sd.cnt, ld = sd.ld;
    float *packed = sd.packed;
    double *packed_d = sd.packed_d, *norm_f = sd.norm_f, *norm = sd.norm;
    uint16_t *split = sd.split;
    __shared__ double shmax[256];
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    float *o = packed + i * dp;
    double *od = packed_d + i * dpd;
    double nf = 0.0, nd = 0.0;
    for (int k = 0; k < dp; ++k) o[k] = 0.0f;
    for (int k = 0; k < dpd; ++k) od[k] = 0.0;
    if (i < cnt) {
        for (int k = 0; k < d; ++k) {
            double v = (double)load_pt(pts, dtype, i * ld + k) - mean[k];
            float vf = (float)v;
            o[k] = vf;
            od[k] = v;
            nf += (double)vf * (double)vf;
            nd += v * v;
        }
    }
    o[d] = -INFINITY;   // bias slots: padding rows never contribute; real rows are set per half-step
    od[d] = -INFINITY;
    if (sd.pts_d) {
        double *op = sd.pts_d + i * kp;
        for (int k = 0; k < kp; ++k) op[k] = k < d ? od[k] : 0.0;
        sd.bias_d[i] = -INFINITY;
    }
    norm_f[i] = nf;
    norm[i] = nd;
    if (split) {   // streamed-role split record of the float copy
        uint4 *rec = reinterpret_cast<uint4 *>(split) + i * (2 * ks);
        for (int k = 0; k < 2 * ks; ++k) {
            uint4 u = make_uint4(0, 0, 0, 0);
            if (k < d) {
                __bf16 y[3];
                split3(o[k], y);
                u = make_uint4(bf16_pair(y[0], y[1]), bf16_pair(y[0], y[2]), bf16_pair(y[1], y[0]), bf16_pair(y[2], y[1]));
            } else if (k == d) {
                u = split_bias_piece(-INFINITY);
            }
            rec[split_piece_pos(ks, i, k)] = u;
        }
    }
    // largest squared norm after centring, over both clouds: non-negative doubles order like their
    // bit patterns, and a maximum does not depend on the order of the atomics
    shmax[threadIdx.x] = nd;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) shmax[threadIdx.x] = fmax(shmax[threadIdx.x], shmax[threadIdx.x + st]);
        __syncthreads();
    }
    if (threadIdx.x == 0 && shmax[0] > 0.0) atomicMax(rho_max_bits, (unsigned long long)__double_as_longlong(shmax[0]));
}

// ---- "precise" split records (d <= 3) from the float64 copy; layout of the six 16-byte pieces
//      (resident counterparts in k_lse_lowd_split):
//   0: Y1_0 Y1_1 Y1_2 0 0 0 0 0          leading digits on the grid gy          x  X1_0 X1_1 X1_2
//   1: Ba Bb Bc 1 1 1 0 0                bias digits on the grid gx gy, ones    x  1 1 1 m1 m2 m3
//   2+k: ry1 ry2 ry3 Y1 Y1 Y1 ry1 ry2    residual pieces of coordinate k        x  X1 X1 X1 rx1 rx2 rx3 rx1 rx1
//   5: rb1 rb2 rb3 0 0 ry1_0 ry1_1 ry1_2 bias residual, second-order terms      x  1 1 1 0 0 rx2_0 rx2_1 rx2_2
// The three 8-bit digits of a bias on the grid q and what they leave.  Inside the digit range (|bias| < 2^21 q: the
// launcher checks the biases it can foresee) every digit is exact in bf16 and the residual is bias - rint(bias/q) q.
// Each digit is taken from what the ROUNDED digits before it leave, and the residual from all three as stored, so a
// bias beyond the range (potentials that grew during a solve) still has pieces that sum to it to double precision:
// the exact window of the first k-step is lost there and the score falls back to fp32-grade accuracy instead of
// carrying a silently rounded digit.
__device__ inline void split_precise_bias(double bias, double q, uint4 *digits, uint2 *residual)
{
    const __bf16 one = (__bf16)1.0f, z = (__bf16)0.0f;
    if (!(fabs(bias) < INFINITY)) {   // padding and zero-weight points: -inf
        *digits = make_uint4(bf16_pair((__bf16)(float)bias, z), bf16_pair(z, one), bf16_pair(one, one), 0u);
        if (residual) *residual = make_uint2(0u, 0u);
        return;
    }
    const double B = rint(bias / q);
    const __bf16 da = (__bf16)(float)(rint(B * (1.0 / 65536.0)) * 65536.0 * q);
    const double ra = B * q - (double)(float)da;
    const __bf16 db = (__bf16)(float)(rint(ra / (256.0 * q)) * 256.0 * q);
    const double rb = ra - (double)(float)db;
    const __bf16 dc = (__bf16)(float)rb;
    *digits = make_uint4(bf16_pair(da, db), bf16_pair(dc, one), bf16_pair(one, one), 0u);
    if (residual) {
        __bf16 r[3];
        split3d(bias - ((double)(float)da + (double)(float)db + (double)(float)dc), r);
        *residual = make_uint2(bf16_pair(r[0], r[1]), bf16_pair(r[2], z));
    }
}

// `rho_max`: device scalar (largest squared norm after centring): the grid comes from it
// (blockIdx.y: 0 = the x cloud, 1 = the y cloud)
__global__ void k_prep_split_precise(const double *packed_d0, int64_t cnt_pad0, uint16_t *out0, const double *packed_d1,
                                     int64_t cnt_pad1, uint16_t *out1, int d, int dpd, const double *rho_max)
{
    const double *packed_d = blockIdx.y ? packed_d1 : packed_d0;
    const int64_t cnt_pad = blockIdx.y ? cnt_pad1 : cnt_pad0;
    uint16_t *out = blockIdx.y ? out1 : out0;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt_pad) return;
    double gx_unused, gy;
    split_grids(*rho_max, 1.0, &gx_unused, &gy);
    __bf16 Y1[3], ry[3][3];
    for (int k = 0; k < 3; ++k) {
        const double y = k < d ? packed_d[i * dpd + k] : 0.0;
        const double y1 = rint(y / gy) * gy;
        Y1[k] = (__bf16)(float)y1;
        split3d(y - y1, ry[k]);
    }
    const __bf16 z = (__bf16)0.0f;
    uint4 *rec = reinterpret_cast<uint4 *>(out) + i * 6;
    rec[0] = make_uint4(bf16_pair(Y1[0], Y1[1]), bf16_pair(Y1[2], z), 0u, 0u);
    split_precise_bias(-INFINITY, 1.0, rec + 1, nullptr);
    for (int k = 0; k < 3; ++k)
        rec[2 + k] = make_uint4(bf16_pair(ry[k][0], ry[k][1]), bf16_pair(ry[k][2], Y1[k]), bf16_pair(Y1[k], Y1[k]),
                                bf16_pair(ry[k][0], ry[k][1]));
    rec[5] = make_uint4(0u, 0u, bf16_pair(z, ry[0][0]), bf16_pair(ry[1][0], ry[2][0]));
}

// ---- float64 derived copy (fp64 matrix-core path) ----------------------------------------
__global__ void k_prep_f64(const void *pts, int dtype, int64_t cnt, int64_t cnt_pad, int64_t d, int64_t ld, int kp,
                           double *out, double *bias, double *norm)
{
    // one wave-sized group of 64 threads per row, strided over the coordinates
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (row >= cnt_pad) return;
    double nrm = 0.0;
    for (int k = lane; k < kp; k += 64) {
        double v = 0.0;
        if (row < cnt && k < d) v = (double)load_pt(pts, dtype, row * ld + k);
        out[row * kp + k] = v;
        nrm += v * v;
    }
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
    if (lane == 0) {
        norm[row] = nrm;
        bias[row] = -INFINITY;
    }
}

// ---- bfloat16 derived copy (bf16 matrix-core path); norms of the ROUNDED points ----------
// Layout: the copy is stored in 1 KB tiles of 16 rows x 32 coordinates; the sixteen tiles of a group
// of 256 rows at one chunk of 32 coordinates are contiguous (16 KB), and the groups of one row group
// follow each other chunk by chunk: tile (rb, ch) sits at (((rb / 16) * n_chunks + ch) * 16 + rb % 16) KB.
// Inside a tile row r occupies 64 bytes and its 16-byte piece p (coordinates 8p..8p+7 of the chunk)
// sits at position p ^ ((r >> 2) & 3).  A 16 KB group is exactly the image that half a pipeline stage
// needs in LDS, so the streaming kernel fills LDS with linear direct loads, each wave a contiguous run
// of it, and reads MFMA fragments without bank conflicts; the contraction loop of a tile walks through
// memory linearly.
__global__ void k_prep_bf16(const void *pts, int dtype, int64_t cnt, int64_t cnt_pad, int64_t d, int64_t ld, int kp,
                            uint16_t *out, float *bias, double *norm)
{
    int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    int lane = threadIdx.x & 63;
    if (row >= cnt_pad) return;
    const int n_chunks = kp >> 5;
    const int64_t rb = row >> 4;
    const int rl = (int)(row & 15);
    double nrm = 0.0;
    for (int pi = lane; pi < (kp >> 3); pi += 64) {   // one 16-byte piece = 8 coordinates
        uint16_t h[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            int k = pi * 8 + e;
            h[e] = 0;
            if (row < cnt && k < d) {
                h[e] = dtype == FS_BF16 ? ((const uint16_t *)pts)[row * ld + k]
                                        : float_to_bf16(((const float *)pts)[row * ld + k]);
                double v = (double)bf16_to_float(h[e]);
                nrm += v * v;
            }
        }
        const int ch = pi >> 2, piece = pi & 3;
        const int pos = piece ^ ((rl >> 2) & 3);
        uint4 v;
        v.x = (uint32_t)h[0] | ((uint32_t)h[1] << 16);
        v.y = (uint32_t)h[2] | ((uint32_t)h[3] << 16);
        v.z = (uint32_t)h[4] | ((uint32_t)h[5] << 16);
        v.w = (uint32_t)h[6] | ((uint32_t)h[7] << 16);
        *reinterpret_cast<uint4 *>(reinterpret_cast<unsigned char *>(out) +
                                   ((((rb >> 4) * n_chunks + ch) * 16 + (rb & 15)) << 10) + rl * 64 + pos * 16) = v;
    }
    for (int off = 32; off > 0; off >>= 1) nrm += __shfl_xor(nrm, off, 64);
    if (lane == 0) {
        norm[row] = nrm;
        bias[row] = -INFINITY;
    }
}

// Where the bias of point i of a side lives, by path, and the squared norms that turn the
// unshifted potential into the shifted one of Prop. 1 (fhat = f - alpha, ghat = g - beta).
struct BiasSink {
    float *packed;          // LowD float copy: packed[i*dp + d], shifted by norm_f
    uint16_t *split;        // LowD split records (same value as the float copy), ks > 0
    int ks;
    uint16_t *split_p;      // LowD precise split records (d <= 3) and the grid of their bias digits:
    double q;               // q itself, or (q == 0) the device scalar rho_max and the eps it is derived from
    const double *rho_dev;
    double q_eps;
    double *packed_d;       // LowD double copy: packed_d[i*dpd + d], shifted by norm
    int dp, dpd, d;
    float *bias_f;          // BF16 path
    double *bias_d;         // F64 path
    const double *norm_f;
    const double *norm;
};

// bias in base-2 units of a streamed point:  ((pot_shifted)/eps + log w) * log2(e)
// (Alg. 1: (ghat_j + delta_j)/eps with delta = eps*log b)
__device__ inline void store_bias(const BiasSink &s, int64_t i, double pot, double inv_eps, double lw)
{
    double b = ((pot - s.norm[i]) * inv_eps + lw) * kLog2e;
    if (s.packed) {
        const float bf = (float)(((pot - s.norm_f[i]) * inv_eps + lw) * kLog2e);
        s.packed[i * s.dp + s.d] = bf;
        if (s.split) reinterpret_cast<uint4 *>(s.split)[i * (2 * s.ks) + split_piece_pos(s.ks, i, s.d)] = split_bias_piece(bf);
    }
    if (s.packed_d) s.packed_d[i * s.dpd + s.d] = b;
    if (s.split_p) {
        double q = s.q;
        if (!(q > 0.0)) {
            double gx, gy;
            split_grids(*s.rho_dev, s.q_eps, &gx, &gy);
            q = gx * gy;
        }
        uint4 *rec = reinterpret_cast<uint4 *>(s.split_p) + i * 6;
        split_precise_bias(b, q, rec + 1, reinterpret_cast<uint2 *>(rec + 5));
    }
    if (s.bias_f) s.bias_f[i] = (float)b;
    if (s.bias_d) s.bias_d[i] = b;
}

// ---- workspace potential (float64, unshifted) + bias from a user potential (float) -------
// `absmax` (optional) receives the largest finite |(pot - norm)/eps| log2e in absmax[1] and the
// largest finite |log w| log2e in absmax[0] (the two parts of a bias, which scale differently with
// eps), as bit patterns of non-negative doubles (for those, the order of the bit patterns is the
// order of the values)
__global__ void k_bias_from_user(const float *pot_user, int64_t cnt, double inv_eps, const float *w,
                                 double log_uniform, double *pot, BiasSink sink, unsigned long long *absmax)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    double mag_pot = 0.0, mag_w = 0.0;
    if (i < cnt) {
        double pu = (double)pot_user[i];
        pot[i] = pu;
        double lw = w ? log((double)w[i]) : log_uniform;
        store_bias(sink, i, pu, inv_eps, lw);
        mag_pot = fabs((pu - sink.norm[i]) * inv_eps) * kLog2e;
        mag_w = fabs(lw) < INFINITY ? fabs(lw) * kLog2e : 0.0;   // zero-weight points never contribute
    }
    if (absmax) {   // one pair of atomics per workgroup (256 threads)
        __shared__ double shm[2][4];
        for (int off = 32; off > 0; off >>= 1) {
            mag_pot = fmax(mag_pot, __shfl_xor(mag_pot, off));
            mag_w = fmax(mag_w, __shfl_xor(mag_w, off));
        }
        if ((threadIdx.x & 63) == 0) {
            shm[0][threadIdx.x >> 6] = mag_w;
            shm[1][threadIdx.x >> 6] = mag_pot;
        }
        __syncthreads();
        if (threadIdx.x == 0) {
            mag_w = fmax(fmax(shm[0][0], shm[0][1]), fmax(shm[0][2], shm[0][3]));
            mag_pot = fmax(fmax(shm[1][0], shm[1][1]), fmax(shm[1][2], shm[1][3]));
            if (mag_w > 0.0) atomicMax(absmax + 0, (unsigned long long)__double_as_longlong(mag_w));
            if (mag_pot > 0.0) atomicMax(absmax + 1, (unsigned long long)__double_as_longlong(mag_pot));
        }
    }
}

// Rescaling of a split's sums to the common maximum.  Every streaming kernel keeps integer-valued
// running maxima (and -3e38 for "nothing seen"), so the factor 2^(m_k - M) is an exact ldexp.
__device__ inline double rescale_split(double v, double mk, double M)
{
    const double dlt = mk - M;
    return dlt >= -1100.0 ? ldexp(v, (int)dlt) : 0.0;   // also 0 for a NaN difference (-inf - -inf)
}

// ---- merge the per-split (max, sum) statistics of a streaming pass -----------------------
//   LSE_2 = M + log2(sum_k s_k 2^(m_k - M)),  pot_new = -eps * ln2 * LSE_2      (Alg. 1, last lines)
// and, as asked: store pot_new, the bias for the pass that streams this side next, the
// unshifted potential for the caller, or the marginal deviation |w e^((pot_old-pot_new)/eps) - w|.
struct FinalizeArgs {
    const double2 *partial;
    int64_t stride;
    int splits;
    int64_t cnt;
    double eps, inv_eps_next;
    const float *w;
    double log_uniform;
    const double *res_norm;
    double *pot;
    BiasSink sink;
    float *user_out;
    double *dev_part;
    double mix;
    double *save_old;
    int blocks;   // workgroups of this side
    // gauge drift (see GaugeMode): where a g-update leaves the block sums of the plan's column marginals, and what
    // the first workgroup of the following f-update collects
    double *gauge_out;
    const double *gauge_prev;
    int64_t gauge_prev_cnt;
    double gauge_prev_eps;
    double *gauge_scalars;   // [0]: the sum so far, [1]: the sum without its last term
    const double *gauge_prev_x;   // averaged schedule: the f-pass's block sums of the previous iteration
    int64_t gauge_prev_x_cnt;
};

// one workgroup: scalars[1] <- scalars[0], scalars[0] += eps ln(sum of part[0..cnt)), in a fixed order
__device__ inline void gauge_collect(const double *part, int64_t cnt, double eps, double *scalars, double *sh)
{
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < cnt; i += 256) acc += part[i];
    const double t = block_sum_256(acc, sh);
    if (threadIdx.x == 0) {
        const double prev = scalars[0];
        scalars[1] = prev;
        scalars[0] = prev + ((t > 0.0 && t < INFINITY) ? eps * log(t) : 0.0);
    }
    __syncthreads();
}

// averaged schedule, one workgroup: scalars[0] = scalars[1] += eps (ln sum(part_y) - ln sum(part_x)) / 4
__device__ inline void gauge_collect_pair(const double *part_x, int64_t cnt_x, const double *part_y, int64_t cnt_y, double eps,
                                          double *scalars, double *sh)
{
    double ax = 0.0, ay = 0.0;
    for (int64_t i = threadIdx.x; i < cnt_x; i += 256) ax += part_x[i];
    for (int64_t i = threadIdx.x; i < cnt_y; i += 256) ay += part_y[i];
    const double sx = block_sum_256(ax, sh);
    __syncthreads();
    const double sy = block_sum_256(ay, sh);
    if (threadIdx.x == 0) {
        const bool ok = sx > 0.0 && sx < INFINITY && sy > 0.0 && sy < INFINITY;
        const double v = scalars[0] + (ok ? 0.25 * eps * (log(sy) - log(sx)) : 0.0);
        scalars[0] = v;
        scalars[1] = v;
    }
    __syncthreads();
}

__device__ __forceinline__ void finalize_body(const FinalizeArgs &a, const int bx)
{
    // dev_part == nullptr: store the update.  dev_part != nullptr: measure the marginal deviation
    // only, unless save_old is given: then measure AND store, keeping the old potential in save_old.
    __shared__ double sh[256];
    if (a.gauge_prev && bx == 0) {
        if (a.gauge_prev_x)
            gauge_collect_pair(a.gauge_prev_x, a.gauge_prev_x_cnt, a.gauge_prev, a.gauge_prev_cnt, a.gauge_prev_eps,
                               a.gauge_scalars, sh);
        else
            gauge_collect(a.gauge_prev, a.gauge_prev_cnt, a.gauge_prev_eps, a.gauge_scalars, sh);
    }
    const int64_t i = (int64_t)bx * 256 + threadIdx.x;
    double dev = 0.0, mass = 0.0;
    if (i < a.cnt) {
        double M = -INFINITY;
#pragma unroll 8
        for (int k = 0; k < a.splits; ++k) {
            double mk = a.partial[(int64_t)k * a.stride + i].x;
            M = mk > M ? mk : M;
        }
        double S = 0.0;
#pragma unroll 8
        for (int k = 0; k < a.splits; ++k) {
            double2 ms = a.partial[(int64_t)k * a.stride + i];
            S += rescale_split(ms.y, ms.x, M);
        }
        // fhat = -eps * LSE (Alg. 1), f = fhat + alpha (Prop. 1)
        double pot_new = -a.eps * kLn2 * (M + log2(S)) + a.res_norm[i];
        const double pot_upd = pot_new;
        if (a.mix != 1.0) pot_new = (1.0 - a.mix) * a.pot[i] + a.mix * pot_new;   // averaged schedule (Eq. 4-5)
        if (a.dev_part) {
            double wi = a.w ? (double)a.w[i] : exp(a.log_uniform);
            dev = fabs(wi * exp((a.pot[i] - pot_new) / a.eps) - wi);   // Prop. 3: r = a exp((fhat - fhat+)/eps)
        }
        if (a.gauge_out) {
            // Prop. 3: the plan's column (row) sum, from the UPDATE itself also where the stored potential is an average
            const double wi = a.w ? (double)a.w[i] : exp(a.log_uniform);
            mass = wi > 0.0 ? wi * exp((a.pot[i] - pot_upd) / a.eps) : 0.0;
        }
        if (!a.dev_part || a.save_old) {
            if (a.save_old) a.save_old[i] = a.pot[i];
            a.pot[i] = pot_new;
            if (a.inv_eps_next > 0.0)
                store_bias(a.sink, i, pot_new, a.inv_eps_next, a.w ? log((double)a.w[i]) : a.log_uniform);
            if (a.user_out) a.user_out[i] = (float)pot_new;
        }
    }
    if (a.dev_part) {
        double t = block_sum_256(dev, sh);
        if (threadIdx.x == 0) a.dev_part[bx] = t;
    }
    if (a.gauge_out) {
        __syncthreads();
        double t = block_sum_256(mass, sh);
        if (threadIdx.x == 0) a.gauge_out[bx] = t;
    }
}

__global__ __launch_bounds__(256) void k_gauge_collect(const double *part, int64_t cnt, double eps, double *scalars)
{
    __shared__ double sh[256];
    gauge_collect(part, cnt, eps, scalars, sh);
}

__global__ __launch_bounds__(256) void k_gauge_collect_pair(const double *part_x, int64_t cnt_x, const double *part_y,
                                                            int64_t cnt_y, double eps, double *scalars)
{
    __shared__ double sh[256];
    gauge_collect_pair(part_x, cnt_x, part_y, cnt_y, eps, scalars, sh);
}

// f_user = (float)(x_pot - scalars[1]) for i < n, g_user = (float)(y_pot + scalars[0]) for the next m indices
__global__ void k_gauge_export(const double *x_pot, int64_t n, const double *y_pot, int64_t m, const double *scalars,
                               float *f_user, float *g_user)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n)
        f_user[i] = (float)(x_pot[i] - scalars[1]);
    else if (i < n + m)
        g_user[i - n] = (float)(y_pot[i - n] + scalars[0]);
}

__global__ __launch_bounds__(256) void k_finalize(FinalizeArgs a) { finalize_body(a, blockIdx.x); }

// the merges of the two passes of an averaged iteration (Eq. 4-5) in one launch
__global__ __launch_bounds__(256) void k_finalize_pair(FinalizeArgs a0, FinalizeArgs a1)
{
    if ((int)blockIdx.x < a0.blocks)
        finalize_body(a0, blockIdx.x);
    else
        finalize_body(a1, (int)blockIdx.x - a0.blocks);
}

__global__ void k_export_f32(const double *src, int64_t cnt, float *dst)
{
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cnt) dst[i] = (float)src[i];
}

// sum of `cnt` doubles by one block, fixed order
__global__ __launch_bounds__(256) void k_sum_to(const double *part, int64_t cnt, double *dst)
{
    __shared__ double sh[256];
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < cnt; i += 256) acc += part[i];
    double t = block_sum_256(acc, sh);
    if (threadIdx.x == 0) *dst = t;
}

// the five sums of the dual objective's terms in one launch: block k < 3 sums pr[k][0..br), block 3 + k
// sums ps[k][0..bs), each in a fixed order
__global__ __launch_bounds__(256) void k_sum_value_terms(const double *pr, int64_t br, const double *ps, int64_t bs, double *dst)
{
    __shared__ double sh[256];
    const int k = blockIdx.x;
    const double *part = k < 3 ? pr + (int64_t)k * br : ps + (int64_t)(k - 3) * bs;
    const int64_t cnt = k < 3 ? br : bs;
    double acc = 0.0;
    for (int64_t i = threadIdx.x; i < cnt; i += 256) acc += part[i];
    const double t = block_sum_256(acc, sh);
    if (threadIdx.x == 0) dst[k] = t;
}

// ---- terms of the dual objective (App. B) -------------------------------------------------
// After an LSE pass over `res`: mass_i = w_i exp((pot_i - pot_i^+)/eps) is the row sum of the plan
// that the CURRENT potentials induce (Prop. 3).  Block sums of mass_i, w_i pot_i and w_i go to
// part[0][.], part[1][.], part[2][.] (part has 3 * gridDim.x doubles).
__global__ __launch_bounds__(256) void k_value_terms(const double2 *partial, int64_t stride, int splits, int64_t cnt,
                                                     double eps, const float *w, double log_uniform,
                                                     const double *res_norm, const double *pot, double *part)
{
    __shared__ double sh[256];
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double t[3] = {0.0, 0.0, 0.0};
    if (i < cnt) {
        double M = -INFINITY;
#pragma unroll 8
        for (int k = 0; k < splits; ++k) {
            double mk = partial[(int64_t)k * stride + i].x;
            M = mk > M ? mk : M;
        }
        double S = 0.0;
#pragma unroll 8
        for (int k = 0; k < splits; ++k) {
            double2 ms = partial[(int64_t)k * stride + i];
            S += rescale_split(ms.y, ms.x, M);
        }
        const double pot_new = -eps * kLn2 * (M + log2(S)) + res_norm[i];
        const double wi = w ? (double)w[i] : exp(log_uniform);
        t[0] = wi > 0.0 ? wi * exp((pot[i] - pot_new) / eps) : 0.0;
        t[1] = wi * pot[i];
        t[2] = wi;
    }
    for (int k = 0; k < 3; ++k) {
        double v = block_sum_256(t[k], sh);
        if (threadIdx.x == 0) part[(int64_t)k * gridDim.x + blockIdx.x] = v;
        __syncthreads();
    }
}

// block counts of the entries that are NaN or infinite
__global__ __launch_bounds__(256) void k_count_nonfinite(const float *v, int64_t cnt, double *part)
{
    __shared__ double sh[256];
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const double t = (i < cnt && !(fabsf(v[i]) < INFINITY)) ? 1.0 : 0.0;
    const double s = block_sum_256(t, sh);
    if (threadIdx.x == 0) part[blockIdx.x] = s;
}

// block sums of the weights (part[0][.]) and of the indicator "not positive and finite" (part[1][.])
__global__ __launch_bounds__(256) void k_weight_stats(const float *w, int64_t cnt, double *part)
{
    __shared__ double sh[256];
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double t[2] = {0.0, 0.0};
    if (i < cnt) {
        const float v = w[i];
        const bool ok = v > 0.0f && v < INFINITY;
        t[0] = ok ? (double)v : 0.0;
        t[1] = ok ? 0.0 : 1.0;
    }
    for (int k = 0; k < 2; ++k) {
        double s = block_sum_256(t[k], sh);
        if (threadIdx.x == 0) part[(int64_t)k * gridDim.x + blockIdx.x] = s;
        __syncthreads();
    }
}

// block sums of w_i pot_i and w_i: part[0][.], part[1][.]
__global__ __launch_bounds__(256) void k_weighted_sums(int64_t cnt, const float *w, double log_uniform, const double *pot,
                                                       double *part)
{
    __shared__ double sh[256];
    int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    double t[2] = {0.0, 0.0};
    if (i < cnt) {
        const double wi = w ? (double)w[i] : exp(log_uniform);
        t[0] = wi * pot[i];
        t[1] = wi;
    }
    for (int k = 0; k < 2; ++k) {
        double v = block_sum_256(t[k], sh);
        if (threadIdx.x == 0) part[(int64_t)k * gridDim.x + blockIdx.x] = v;
        __syncthreads();
    }
}

// merge the splits of an application pass and apply the epilogue of Alg. 2:
//   out_i = a_i * exp(fhat_i/eps + m_i) * O_i   with everything in base 2;  mass_i = same with s.
// A block of 256 threads covers 256 / PC rows; thread (row, c) produces one output entry, so the
// reads of the [splits][rows][PC] accumulators are contiguous; the row's max and factor are
// computed once (by its thread c = 0) and shared.  (When PC does not divide 256 the last 256 % PC threads idle.)
__global__ __launch_bounds__(256) void k_apply_finalize(const double2 *partial, int64_t stride, const float *opart,
                                                        int64_t opart_stride, int PC, int splits, int64_t cnt,
                                                        double inv_eps, const float *w, double log_uniform,
                                                        const double *pot, const double *res_norm, int p0, int p,
                                                        float *out, int64_t ldo, float *mass_out)
{
    __shared__ double shM[256], shFac[256];
    const int rows_per_block = 256 / PC;
    const int rl = threadIdx.x / PC, c = threadIdx.x - rl * PC;
    const int64_t i = rl < rows_per_block ? (int64_t)blockIdx.x * rows_per_block + rl : cnt;   // (idle threads: no row)
    if (c == 0 && i < cnt) {
        double M = -INFINITY;
#pragma unroll 8
        for (int k = 0; k < splits; ++k) {
            double mk = partial[(int64_t)k * stride + i].x;
            M = mk > M ? mk : M;
        }
        double lw = w ? log((double)w[i]) : log_uniform;
        // row factor  a_i * exp(fhat_i/eps + m_i): add the exponents BEFORE exponentiating
        const double fac = exp2(((pot[i] - res_norm[i]) * inv_eps + lw) * kLog2e + M);
        shM[rl] = M;
        shFac[rl] = fac;
        if (mass_out && p0 == 0) {
            double S = 0.0;
#pragma unroll 8
            for (int k = 0; k < splits; ++k) {
                double2 ms = partial[(int64_t)k * stride + i];
                S += rescale_split(ms.y, ms.x, M);
            }
            mass_out[i] = (float)(fac * S);
        }
    }
    __syncthreads();
    if (i >= cnt || p0 + c >= p) return;
    const double M = shM[rl];
    double acc = 0.0;
#pragma unroll 4
    for (int k = 0; k < splits; ++k) {
        const double mk = partial[(int64_t)k * stride + i].x;
        acc += rescale_split((double)opart[((int64_t)k * opart_stride + i) * PC + c], mk, M);
    }
    out[i * ldo + p0 + c] = (float)(shFac[rl] * acc);
}

// `eps`: the eps of the pass that will stream these biases
// `rho_on_device`: the host does not know rho_max yet (prologue of an entry call): the kernel
// derives the grid from the device scalar
BiasSink sink_of(const Prepared *P, const Side *s, double eps, bool rho_on_device = false)
{
    BiasSink k{};
    k.split_p = s->split_p;
    if (s->split_p && eps > 0.0) {
        if (rho_on_device) {
            k.q = 0.0;
            k.rho_dev = P->scalars + 7;
            k.q_eps = eps;
        } else {
            double gx, gy;
            split_grids(P->rho_max, eps, &gx, &gy);
            k.q = gx * gy;
        }
    } else {
        k.split_p = nullptr;
    }
    k.packed = s->packed;
    k.packed_d = s->packed_d;
    k.split = s->split;
    k.ks = P->ks;
    k.dp = P->dp;
    k.dpd = P->dpd;
    k.d = (int)P->d;
    k.bias_f = s->bias_f;
    k.bias_d = s->bias_d;
    k.norm_f = s->norm_f;
    k.norm = s->norm;
    return k;
}

}  // namespace

fs_status launch_apply_finalize(Ctx *c, const Prepared *P, const Side *res, const double *res_norm, int splits,
                                double eps, const float *opart, int PC, int p0, int p, float *out, int64_t ldo,
                                float *mass_out)
{
    if (PC < 1 || PC > 256) return fail(c, FS_ERR_DEVICE, "internal: accumulator width of the application merge");
    hipLaunchKernelGGL(k_apply_finalize, dim3((unsigned)ceil_div(res->cnt, 256 / PC)), dim3(256), 0, c->stream,
                       (const double2 *)P->partial, res->cnt_pad, opart, res->cnt_pad, PC, splits, res->cnt, 1.0 / eps,
                       res->w, res->log_uniform, res->pot, res_norm, p0, p, out, ldo, mass_out);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// float copy of a point matrix (bf16 storage) for use as the value matrix of a plan application
__global__ void k_pts_to_f32(const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, float *dst)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * d) return;
    const int64_t i = e / d, k = e - i * d;
    dst[e] = load_pt(pts, dtype, i * ld + k);
}

// Gradient assembly on top of T = (plan applied to the other cloud), in place in `g` (rows x d):
//   mode 0: 2 (w_i z_i - T_i)        Cor. 4, w the given weights (uniform 1/rows when NULL)
//   mode 1: 2 (mass_i z_i - T_i)     the same with the plan's own marginal (appendix on gradients)
//   mode 2: z_i - T_i / w_i          displacement to the barycentric image
__global__ void k_grad_assemble(float *g, int64_t ldg, const void *pts, int dtype, int64_t ld, int64_t rows, int64_t d,
                                const float *w, double uniform_w, const float *mass, int mode)
{
    const int64_t e = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= rows * d) return;
    const int64_t i = e / d, k = e - i * d;
    const double z = (double)load_pt(pts, dtype, i * ld + k);
    const double t = (double)g[i * ldg + k];
    const double wi = w ? (double)w[i] : uniform_w;
    double r;
    if (mode == 0)
        r = 2.0 * (wi * z - t);
    else if (mode == 1)
        r = 2.0 * ((double)mass[i] * z - t);
    else
        r = z - t / wi;
    g[i * ldg + k] = (float)r;
}

// ---- label-augmented cost  l1 |x_i - y_j|^2 + l2 W[lx_i, ly_j]  (Section 3.1's remark on generalised costs; the
// appendix on the dataset-distance application).  The table lookup is itself a contraction,
// W[lx, ly] = <onehot(lx), W[:, ly]>, so V more coordinates carry it through the score contraction of every kernel:
//     xa_i = [x_i, onehot(lx_i)],   ya_j = [y_j, u_j],  u_j = -(l2 / 2 l1) W[:, ly_j]
//     l1 |xa_i - ya_j|^2 = l1 |x_i - y_j|^2 + l2 W[lx_i, ly_j] + l1 + v_j,   v_j = l1 |u_j|^2,
// a cost that differs from the wanted one by per-point constants only, which the potentials absorb exactly.
// In bf16 mode u is rounded to bfloat16 here, so that v_j is taken from the values the matrix cores will see.
// Labels outside [0, V) are counted in *bad (and read as class 0).
__global__ void k_label_augment(const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, const int32_t *labels,
                                const float *W, int V, int target_side, double half_ratio, double l1, int round_bf16,
                                float *out, float *vconst, unsigned *bad)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= rows) return;
    int lab = labels[i];
    if (lab < 0 || lab >= V) {
        atomicAdd(bad, 1u);
        lab = 0;
    }
    float *o = out + i * (d + V);
    for (int64_t k = 0; k < d; ++k) o[k] = load_pt(pts, dtype, i * ld + k);
    double v = 0.0;
    for (int k = 0; k < V; ++k) {
        float u;
        if (target_side) {
            u = (float)(-half_ratio * (double)W[(int64_t)k * V + lab]);
            if (round_bf16) u = bf16_to_float(float_to_bf16(u));
            v += (double)u * (double)u;
        } else {
            u = k == lab ? 1.0f : 0.0f;
        }
        o[d + k] = u;
    }
    if (vconst) vconst[i] = (float)(l1 * v);
}

// potentials of the labelled problem <-> potentials of the augmented one:  p' = (p + shift) / l1  and back
__global__ void k_label_potential(const float *src, const float *vconst, double cshift, double l1, int to_augmented,
                                  int64_t cnt, float *dst)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= cnt) return;
    const double sh = cshift + (vconst ? (double)vconst[i] : 0.0);
    dst[i] = to_augmented ? (float)(((double)src[i] + sh) / l1) : (float)((double)src[i] * l1 - sh);
}

fs_status launch_label_augment(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld,
                               const int32_t *labels, const float *W, int V, bool target_side, double l1, double l2,
                               bool round_bf16, float *out, float *vconst, unsigned *bad)
{
    hipLaunchKernelGGL(k_label_augment, dim3((unsigned)ceil_div(rows, 128)), dim3(128), 0, c->stream, pts, dtype, rows, d, ld,
                       labels, W, V, target_side ? 1 : 0, l2 / (2.0 * l1), l1, round_bf16 ? 1 : 0, out, vconst, bad);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_label_potential(Ctx *c, const float *src, const float *vconst, double cshift, double l1, bool to_augmented,
                                 int64_t cnt, float *dst)
{
    hipLaunchKernelGGL(k_label_potential, dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, c->stream, src, vconst, cshift, l1,
                       to_augmented ? 1 : 0, cnt, dst);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_pts_to_f32(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, float *dst)
{
    hipLaunchKernelGGL(k_pts_to_f32, dim3((unsigned)ceil_div(rows * d, 256)), dim3(256), 0, c->stream, pts, dtype, rows, d,
                       ld, dst);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_grad_assemble(Ctx *c, float *g, int64_t ldg, const void *pts, int dtype, int64_t ld, int64_t rows,
                               int64_t d, const float *w, const float *mass, int mode)
{
    hipLaunchKernelGGL(k_grad_assemble, dim3((unsigned)ceil_div(rows * d, 256)), dim3(256), 0, c->stream, g, ldg, pts, dtype,
                       ld, rows, d, w, 1.0 / (double)rows, mass, mode);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_export_f32(Ctx *c, const double *src, int64_t cnt, float *dst)
{
    hipLaunchKernelGGL(k_export_f32, dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, c->stream, src, cnt, dst);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_fill_f64(Ctx *c, double *dst, double v, int64_t cnt)
{
    hipLaunchKernelGGL(k_fill_f64, dim3((unsigned)ceil_div(cnt, 256)), dim3(256), 0, c->stream, dst, v, cnt);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_row_norms(Ctx *c, const void *pts, int dtype, int64_t rows, int64_t d, int64_t ld, float *out)
{
    hipLaunchKernelGGL(k_row_norms, dim3((unsigned)ceil_div(rows, 256)), dim3(256), 0, c->stream, pts, dtype, rows, d,
                       ld, out);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_prepare(Ctx *c, const fs_problem *p, Prepared *P)
{
    const int dtype = p->dtype;
    struct In { const void *pts; int64_t ld; Side *S; };
    In in[2] = {{p->x, p->ldx, &P->X}, {p->y, p->ldy, &P->Y}};
    if (P->path == Path::LowD) {
        // the reserved area holds 16 doubles (mean) + 2 x 128 x 16 doubles (per-block sums of x, of y)
        const int half = 128;
        double *partX = P->mean + kLowdMaxD;
        double *partY = partX + (size_t)half * kLowdMaxD;
        const CloudIn cx{p->x, p->n, p->ldx, partX}, cy{p->y, p->m, p->ldy, partY};
        hipLaunchKernelGGL(k_coord_sums, dim3(half, 2), dim3(256), 0, c->stream, cx, cy, dtype, (int)p->d);
        // (also clears scalars[5..7]: the sizes of the biases and the largest squared norm, all taken by atomic maxima)
        hipLaunchKernelGGL(k_mean_final, dim3(1), dim3(256), 0, c->stream, partX, partY, half,
                           1.0 / (double)(p->n + p->m), P->mean, P->scalars + 5);
        const int64_t pad_max = P->X.cnt_pad > P->Y.cnt_pad ? P->X.cnt_pad : P->Y.cnt_pad;
        PrepLowdSide sd[2];
        for (int k = 0; k < 2; ++k) {
            const Side *S = in[k].S;
            sd[k] = PrepLowdSide{in[k].pts, S->cnt, S->cnt_pad, in[k].ld, S->packed, S->packed_d, S->norm_f, S->norm, S->split,
                                 S->pts_d,   S->bias_d};
        }
        hipLaunchKernelGGL(k_prep_lowd, dim3((unsigned)ceil_div(pad_max, 256), 2), dim3(256), 0, c->stream, sd[0], sd[1], dtype,
                           (int)p->d, P->dp, P->dpd, P->kp, P->mean, P->ks, reinterpret_cast<unsigned long long *>(P->scalars + 7));
        // (the host reads rho_max back together with the sizes of the biases, see launch_bias_from_user)
        P->rho_max = -1.0;
        if (p->d <= 3)   // the grid of the precise records' leading digits depends on rho_max
            hipLaunchKernelGGL(k_prep_split_precise, dim3((unsigned)ceil_div(pad_max, 256), 2), dim3(256), 0, c->stream,
                               P->X.packed_d, P->X.cnt_pad, P->X.split_p, P->Y.packed_d, P->Y.cnt_pad, P->Y.split_p, (int)p->d,
                               P->dpd, P->scalars + 7);
        FS_HIP(c, hipGetLastError());
    } else if (P->path == Path::F64) {
        for (auto &s : in)
            hipLaunchKernelGGL(k_prep_f64, dim3((unsigned)ceil_div(s.S->cnt_pad, 4)), dim3(256), 0, c->stream, s.pts,
                               dtype, s.S->cnt, s.S->cnt_pad, p->d, s.ld, P->kp, s.S->pts_d, s.S->bias_d, s.S->norm);
    } else {
        for (auto &s : in)
            hipLaunchKernelGGL(k_prep_bf16, dim3((unsigned)ceil_div(s.S->cnt_pad, 4)), dim3(256), 0, c->stream, s.pts,
                               dtype, s.S->cnt, s.S->cnt_pad, p->d, s.ld, P->kp, s.S->pts_b, s.S->bias_f, s.S->norm);
    }
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_bias_from_user(Ctx *c, Prepared *P, Side *side, const float *pot_user, double eps, bool first, bool last)
{
    // low-d problems: the size of the bias enters the choice of the score precision (lowd_precise),
    // so it is measured where a caller's potential comes in; it is read back together with the
    // largest squared norm, once per entry call (three doubles)
    unsigned long long *absmax = nullptr;
    if (P->path == Path::LowD) {
        absmax = reinterpret_cast<unsigned long long *>(P->scalars + 5);   // scalars[5], [6]
        if (first && !(P->rho_max < 0.0)) {   // (a fresh prologue has cleared them already)
            fs_status st = launch_fill_f64(c, P->scalars + 5, 0.0, 2);
            if (st != FS_OK) return st;
        }
    }
    hipLaunchKernelGGL(k_bias_from_user, dim3((unsigned)ceil_div(side->cnt, 256)), dim3(256), 0, c->stream, pot_user,
                       side->cnt, 1.0 / eps, side->w, side->log_uniform, side->pot, sink_of(P, side, eps, P->rho_max < 0.0),
                       absmax);
    FS_HIP(c, hipGetLastError());
    if (absmax && last) {
        double h[3] = {0.0, 0.0, 0.0};   // |log w| part, potential part, rho_max
        FS_HIP(c, hipMemcpyAsync(h, P->scalars + 5, sizeof h, hipMemcpyDeviceToHost, c->stream));
        FS_HIP(c, hipStreamSynchronize(c->stream));
        if (h[0] > P->logw_mag) P->logw_mag = h[0];
        if (h[1] * eps > P->pot_mag_eps) P->pot_mag_eps = h[1] * eps;
        P->rho_max = h[2];
        if (c->kept_valid) c->kept_rho_max = h[2];   // belongs to the kept derived copies (no-op when they are another problem's)
    }
    return FS_OK;
}

static FinalizeArgs finalize_args(const Prepared *P, const void *partial, Side *res, const double *res_norm, int splits,
                                  double eps_cur, double eps_next_bias, float *user_out, double *dev_part, double mix,
                                  double *save_old)
{
    FinalizeArgs a{};
    a.partial = (const double2 *)partial;
    a.stride = res->cnt_pad;
    a.splits = splits;
    a.cnt = res->cnt;
    a.eps = eps_cur;
    a.inv_eps_next = eps_next_bias > 0.0 ? 1.0 / eps_next_bias : 0.0;
    a.w = res->w;
    a.log_uniform = res->log_uniform;
    a.res_norm = res_norm;
    a.pot = res->pot;
    a.sink = sink_of(P, res, eps_next_bias);
    a.user_out = user_out;
    a.dev_part = dev_part;
    a.mix = mix;
    a.save_old = save_old;
    a.blocks = (int)ceil_div(res->cnt, 256);
    return a;
}

fs_status launch_gauge_export(Ctx *c, const Prepared *P, bool collect_last, double eps_last, const double *x_pot,
                              float *f_user, float *g_user)
{
    if (collect_last)
        hipLaunchKernelGGL(k_gauge_collect, dim3(1), dim3(256), 0, c->stream, P->gauge_part, (int64_t)ceil_div(P->Y.cnt, 256),
                           eps_last, P->scalars + 8);
    hipLaunchKernelGGL(k_gauge_export, dim3((unsigned)ceil_div(P->X.cnt + P->Y.cnt, 256)), dim3(256), 0, c->stream, x_pot,
                       P->X.cnt, P->Y.pot, P->Y.cnt, P->scalars + 8, f_user, g_user);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

fs_status launch_finalize(Ctx *c, const Prepared *P, Side *res, const double *res_norm, int splits, double eps_cur,
                          double eps_next_bias, float *user_out, double *abs_dev_sum, double mix, double *save_old,
                          GaugeMode gauge, int64_t gauge_prev_cnt, double gauge_prev_eps)
{
    double *dev_part = abs_dev_sum ? P->dev_part : nullptr;   // per-block sums of the marginal deviation
    FinalizeArgs a = finalize_args(P, P->partial, res, res_norm, splits, eps_cur, eps_next_bias, user_out, dev_part,
                                   mix, save_old);
    if (gauge == GaugeMode::Measure) a.gauge_out = P->gauge_part;
    if (gauge == GaugeMode::Collect && gauge_prev_cnt > 0) {
        a.gauge_prev = P->gauge_part;
        a.gauge_prev_cnt = (int64_t)ceil_div(gauge_prev_cnt, 256);
        a.gauge_prev_eps = gauge_prev_eps;
        a.gauge_scalars = P->scalars + 8;
    }
    hipLaunchKernelGGL(k_finalize, dim3((unsigned)a.blocks), dim3(256), 0, c->stream, a);
    if (abs_dev_sum)
        hipLaunchKernelGGL(k_sum_to, dim3(1), dim3(256), 0, c->stream, dev_part, (int64_t)a.blocks, abs_dev_sum);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// merges of the f-pass (records in partial_x) and of the g-pass (partial_y) in one launch
fs_status launch_finalize_pair(Ctx *c, const Prepared *P, Side *X, const double *norm_x, const void *partial_x, int splits_x,
                               float *f_out, Side *Y, const double *norm_y, const void *partial_y, int splits_y,
                               float *g_out, double eps_cur, double eps_next_bias, double mix, int gauge_parity, bool collect_prev)
{
    FinalizeArgs ax = finalize_args(P, partial_x, X, norm_x, splits_x, eps_cur, eps_next_bias, f_out, nullptr, mix, nullptr);
    FinalizeArgs ay = finalize_args(P, partial_y, Y, norm_y, splits_y, eps_cur, eps_next_bias, g_out, nullptr, mix, nullptr);
    if (gauge_parity >= 0) {
        // the sums of this iteration go to one half of the two arrays while the first workgroup of the f side
        // collects the previous iteration's from the other half
        const int64_t nbx = ceil_div(X->cnt, 256), nby = ceil_div(Y->cnt, 256);
        const int64_t half = nbx > nby ? nbx : nby;
        ax.gauge_out = P->gauge_part_x + (gauge_parity & 1) * half;
        ay.gauge_out = P->gauge_part + (gauge_parity & 1) * half;
        if (collect_prev) {
            ax.gauge_prev = P->gauge_part + ((gauge_parity & 1) ^ 1) * half;
            ax.gauge_prev_cnt = nby;
            ax.gauge_prev_x = P->gauge_part_x + ((gauge_parity & 1) ^ 1) * half;
            ax.gauge_prev_x_cnt = nbx;
            ax.gauge_prev_eps = eps_cur;
            ax.gauge_scalars = P->scalars + 8;
        }
    }
    hipLaunchKernelGGL(k_finalize_pair, dim3((unsigned)(ax.blocks + ay.blocks)), dim3(256), 0, c->stream, ax, ay);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// the term of the last averaged iteration (its sums sit in half `gauge_parity` of the two arrays)
fs_status launch_gauge_collect_pair(Ctx *c, const Prepared *P, double eps, int gauge_parity)
{
    const int64_t nbx = ceil_div(P->X.cnt, 256), nby = ceil_div(P->Y.cnt, 256);
    const int64_t half = nbx > nby ? nbx : nby;
    hipLaunchKernelGGL(k_gauge_collect_pair, dim3(1), dim3(256), 0, c->stream, P->gauge_part_x + (gauge_parity & 1) * half, nbx,
                       P->gauge_part + (gauge_parity & 1) * half, nby, eps, P->scalars + 8);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// dst[0] <- how many of the cnt floats are NaN or infinite; `scratch` holds one double per 256 values
fs_status launch_count_nonfinite(Ctx *c, const float *v, int64_t cnt, double *scratch, double *dst)
{
    const unsigned nb = (unsigned)ceil_div(cnt, 256);
    hipLaunchKernelGGL(k_count_nonfinite, dim3(nb), dim3(256), 0, c->stream, v, cnt, scratch);
    hipLaunchKernelGGL(k_sum_to, dim3(1), dim3(256), 0, c->stream, scratch, (int64_t)nb, dst);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// dst[0] <- sum of the weights, dst[1] <- how many of them are not positive and finite; `scratch` holds
// 2 * blocks doubles
fs_status launch_weight_stats(Ctx *c, const float *w, int64_t cnt, double *scratch, double *dst)
{
    const unsigned nb = (unsigned)ceil_div(cnt, 256);
    hipLaunchKernelGGL(k_weight_stats, dim3(nb), dim3(256), 0, c->stream, w, cnt, scratch);
    hipLaunchKernelGGL(k_sum_to, dim3(1), dim3(256), 0, c->stream, scratch, (int64_t)nb, dst);
    hipLaunchKernelGGL(k_sum_to, dim3(1), dim3(256), 0, c->stream, scratch + nb, (int64_t)nb, dst + 1);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

// dst[0..4] <- sum_i mass_i, <w_res, pot_res>, sum w_res, <w_str, pot_str>, sum w_str  (see k_value_terms);
// `scratch` holds 3 * blocks(res) + 2 * blocks(str) doubles
fs_status launch_value_terms(Ctx *c, const Prepared *P, const Side *res, const double *res_norm, const Side *str,
                             int splits, double eps, double *scratch, double *dst)
{
    const unsigned br = (unsigned)ceil_div(res->cnt, 256), bs = (unsigned)ceil_div(str->cnt, 256);
    double *pr = scratch, *ps = scratch + 3 * (size_t)br;
    hipLaunchKernelGGL(k_value_terms, dim3(br), dim3(256), 0, c->stream, (const double2 *)P->partial, res->cnt_pad, splits,
                       res->cnt, eps, res->w, res->log_uniform, res_norm, res->pot, pr);
    hipLaunchKernelGGL(k_weighted_sums, dim3(bs), dim3(256), 0, c->stream, str->cnt, str->w, str->log_uniform, str->pot, ps);
    hipLaunchKernelGGL(k_sum_value_terms, dim3(5), dim3(256), 0, c->stream, pr, (int64_t)br, ps, (int64_t)bs, dst);
    FS_HIP(c, hipGetLastError());
    return FS_OK;
}

}  // namespace fs
