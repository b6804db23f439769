// C ABI of libflashsink: argument validation, workspace management and the
// orchestration of the streaming passes.  All arithmetic of the method runs in
// the kernels of fs_prep.hip / fs_lowd.hip / fs_f64.hip / fs_bf16.hip.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include <new>

#include "fs_internal.h"

namespace fs {

fs_status fail(Ctx *c, fs_status s, const char *fmt, ...)
{
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return s;
}

void prof_begin(Ctx *c, double pairs, int kind)
{
    if (!c->prof_on) return;
    if (c->ev_used + 2 > c->ev_pool.size()) {
        for (int k = 0; k < 2; ++k) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return;
            c->ev_pool.push_back(e);
        }
    }
    (void)hipEventRecord(c->ev_pool[c->ev_used], c->stream);
    c->ev_kind.resize(c->ev_used / 2 + 1);
    c->ev_pairs.resize(c->ev_used / 2 + 1);
    c->ev_kind[c->ev_used / 2] = kind;
    c->ev_pairs[c->ev_used / 2] = pairs;
}

void prof_end(Ctx *c)
{
    if (!c->prof_on || c->ev_used + 2 > c->ev_pool.size()) return;
    (void)hipEventRecord(c->ev_pool[c->ev_used + 1], c->stream);
    c->ev_used += 2;
}

namespace {

// Workspace of the entry point that allocates nothing (fs_solve_noalloc): every GPU the library runs on holds
// its own copy of this array, at its own address, until the process ends.  In host code the name is only a
// handle for hipGetSymbolAddress (fs_create resolves it, with the context's device current); kernels and
// copies get the resolved address.
constexpr size_t kStaticScratchBytes = size_t(32) << 20;
constexpr size_t kStaticPartialBudget = size_t(8) << 20;   // of which the partial records of a pass may take
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// Makes the context's device current for the duration of an entry call and restores the caller's.
struct DeviceGuard {
    int prev = -1;
    bool active = false;
    explicit DeviceGuard(const Ctx *c)
    {
        if (c && c->device >= 0 && hipGetDevice(&prev) == hipSuccess && prev != c->device)
            active = hipSetDevice(c->device) == hipSuccess;
    }
    ~DeviceGuard()
    {
        if (active) (void)hipSetDevice(prev);
    }
    DeviceGuard(const DeviceGuard &) = delete;
    DeviceGuard &operator=(const DeviceGuard &) = delete;
};

Path choose_path(const fs_problem *p)
{
    if (p->compute == FS_COMPUTE_BF16_MFMA) return Path::BF16;
    return p->d <= kLowdMaxD ? Path::LowD : Path::F64;
}

fs_status validate_problem(Ctx *c, const fs_problem *p)
{
    if (!c) return FS_ERR_INVALID_ARG;
    c->err.clear();
    if (!p) return fail(c, FS_ERR_INVALID_ARG, "problem is NULL");
    if (!p->x || !p->y) return fail(c, FS_ERR_INVALID_ARG, "x or y is NULL");
    if (p->dtype != FS_F32 && p->dtype != FS_BF16)
        return fail(c, FS_ERR_INVALID_ARG, "unknown dtype %d", (int)p->dtype);
    if (p->compute != FS_COMPUTE_FP32 && p->compute != FS_COMPUTE_BF16_MFMA)
        return fail(c, FS_ERR_INVALID_ARG, "unknown compute mode %d", (int)p->compute);
    if (p->n <= 0 || p->m <= 0 || p->d <= 0)
        return fail(c, FS_ERR_BAD_SHAPE, "n, m, d must be positive (got %lld, %lld, %lld)",
                    (long long)p->n, (long long)p->m, (long long)p->d);
    if (p->n > (int64_t(1) << 24) || p->m > (int64_t(1) << 24) || p->d > 8192)
        return fail(c, FS_ERR_BAD_SHAPE, "n, m <= 2^24 and d <= 8192 are supported");
    if (p->ldx < p->d || p->ldy < p->d)
        return fail(c, FS_ERR_BAD_SHAPE, "leading dimension smaller than d");
    if (p->compute == FS_COMPUTE_BF16_MFMA && p->d < 16)
        return fail(c, FS_ERR_UNSUPPORTED,
                    "bf16 matrix-core mode needs d >= 16 (d = %lld is not a dense contraction)",
                    (long long)p->d);
    return FS_OK;
}

fs_status validate_eps(Ctx *c, float eps)
{
    if (!(eps > 0.0f) || !isfinite(eps)) return fail(c, FS_ERR_BAD_EPS, "eps must be positive and finite");
    return FS_OK;
}

bool overlap(const void *p, size_t pb, const void *q, size_t qb)
{
    if (!p || !q) return false;
    const char *a = (const char *)p, *b = (const char *)q;
    return a < b + qb && b < a + pb;
}

size_t pts_bytes(const fs_problem *p, bool is_x)
{
    size_t es = p->dtype == FS_BF16 ? 2 : 4;
    int64_t rows = is_x ? p->n : p->m;
    int64_t ld = is_x ? p->ldx : p->ldy;
    return (size_t)((rows - 1) * ld + p->d) * es;
}

// An output may not overlap x, y, a, b.
fs_status check_out(Ctx *c, const fs_problem *p, const void *out, size_t bytes, const char *name)
{
    if (!out) return fail(c, FS_ERR_INVALID_ARG, "%s is NULL", name);
    if (overlap(out, bytes, p->x, pts_bytes(p, true)) || overlap(out, bytes, p->y, pts_bytes(p, false)) ||
        overlap(out, bytes, p->a, (size_t)p->n * 4) || overlap(out, bytes, p->b, (size_t)p->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "%s overlaps an input of the problem", name);
    return FS_OK;
}

double stage_eps(double e0, double e1, int stages, int s)
{
    if (stages <= 1 || s >= stages - 1) return (double)(float)e1;
    if (s <= 0) return (double)(float)e0;
    return (double)(float)(e0 * pow(e1 / e0, (double)s / (double)(stages - 1)));
}

// Lay the prepared problem out in the workspace; returns bytes needed.  With base == nullptr
// only the size is computed.
size_t layout(const Ctx *c, const fs_problem *p, Prepared *P, char *base, size_t extra)
{
    Arena A;
    P->path = choose_path(p);
    P->d = p->d;
    auto side = [&](Side &S, int64_t cnt, const float *w) {
        S.cnt = cnt;
        S.w = w;
        S.log_uniform = -log((double)cnt);
        S.cnt_pad = round_up(cnt, 1024);
        size_t o;
        switch (P->path) {
        case Path::LowD:
            P->dp = (int)round_up(p->d + 1, 4);
            P->dpd = (int)round_up(p->d + 1, 2);
            o = A.take((size_t)S.cnt_pad * P->dp * 4);
            S.packed = base ? (float *)(base + o) : nullptr;
            o = A.take((size_t)S.cnt_pad * P->dpd * 8);
            S.packed_d = base ? (double *)(base + o) : nullptr;
            o = A.take((size_t)S.cnt_pad * 8);
            S.norm_f = base ? (double *)(base + o) : nullptr;
            P->ks = split_ksteps(p->d);
            o = A.take((size_t)S.cnt_pad * P->ks * 32);
            S.split = (base && P->ks) ? (uint16_t *)(base + o) : nullptr;
            o = A.take(p->d <= 3 ? (size_t)S.cnt_pad * 96 : 0);
            S.split_p = (base && p->d <= 3) ? (uint16_t *)(base + o) : nullptr;
            // d > 3: float64-score half-steps run on the fp64 matrix cores, from records of that path
            P->kp = 32;
            o = A.take(p->d > 3 ? (size_t)S.cnt_pad * P->kp * 8 : 0);
            S.pts_d = (base && p->d > 3) ? (double *)(base + o) : nullptr;
            o = A.take(p->d > 3 ? (size_t)S.cnt_pad * 8 : 0);
            S.bias_d = (base && p->d > 3) ? (double *)(base + o) : nullptr;
            break;
        case Path::F64:
            P->kp = (int)round_up(p->d, 32);
            o = A.take((size_t)S.cnt_pad * P->kp * 8);
            S.pts_d = base ? (double *)(base + o) : nullptr;
            o = A.take((size_t)S.cnt_pad * 8);
            S.bias_d = base ? (double *)(base + o) : nullptr;
            break;
        case Path::BF16:
            P->kp = (int)round_up(p->d, 32);
            o = A.take((size_t)S.cnt_pad * P->kp * 2);
            S.pts_b = base ? (uint16_t *)(base + o) : nullptr;
            o = A.take((size_t)S.cnt_pad * 4);
            S.bias_f = base ? (float *)(base + o) : nullptr;
            break;
        }
        o = A.take((size_t)S.cnt_pad * 8);
        S.norm = base ? (double *)(base + o) : nullptr;
        o = A.take((size_t)S.cnt_pad * 8);
        S.pot = base ? (double *)(base + o) : nullptr;
    };
    side(P->X, p->n, p->a);
    side(P->Y, p->m, p->b);
    int64_t big = P->X.cnt_pad > P->Y.cnt_pad ? P->X.cnt_pad : P->Y.cnt_pad;
    // [splits][rows] records of the pass over either side
    const size_t pbx = (size_t)max_splits(c->partial_budget, p->n) * P->X.cnt_pad * 16, pby = (size_t)max_splits(c->partial_budget, p->m) * P->Y.cnt_pad * 16;
    P->partial_bytes = pbx > pby ? pbx : pby;
    size_t o = A.take(P->partial_bytes);
    P->partial = base ? (void *)(base + o) : nullptr;
    o = A.take((size_t)ceil_div(big, 256) * 8);
    P->dev_part = base ? (double *)(base + o) : nullptr;
    o = A.take((size_t)ceil_div(big, 256) * 16);
    P->gauge_part = base ? (double *)(base + o) : nullptr;
    o = A.take((size_t)ceil_div(big, 256) * 16);
    P->gauge_part_x = base ? (double *)(base + o) : nullptr;
    o = A.take(16 * 8);
    P->scalars = base ? (double *)(base + o) : nullptr;
    o = A.take((size_t)(256 + 1) * 16 * 8);
    P->mean = base ? (double *)(base + o) : nullptr;
    o = A.take(extra);
    (void)o;
    return A.off;
}

fs_status ensure_ws(Ctx *c, size_t need)
{
    if (need <= c->ws_bytes) return FS_OK;
    if (c->ws_static) return fail(c, FS_ERR_BAD_SHAPE, "the problem needs %zu bytes of workspace, the static scratch holds %zu", need, c->ws_bytes);
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (c->ws) {
        FS_HIP(c, hipFree(c->ws));
        c->ws = nullptr;
        c->ws_bytes = 0;
    }
    void *pnew = nullptr;
    hipError_t e = hipMalloc(&pnew, need);
    if (e != hipSuccess)
        return fail(c, FS_ERR_ALLOC, "workspace of %zu bytes: %s", need, hipGetErrorString(e));
    c->ws = (char *)pnew;
    c->ws_bytes = need;
    return FS_OK;
}

// Validate, size the workspace, lay the problem out and run the prologue kernels.
// `extra` bytes are reserved after the prepared problem; *extra_ptr receives their address.
fs_status prepare(Ctx *c, const fs_problem *p, Prepared *P, size_t extra, char **extra_ptr)
{
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    size_t need = layout(c, p, P, nullptr, extra);
    fs_status st = ensure_ws(c, need);
    if (st != FS_OK) return st;
    layout(c, p, P, c->ws, extra);
    P->dbg_score = c->dbg_lowd_score;
    P->dbg_precise_valu = c->dbg_lowd_precise_valu != 0;
    P->dbg_any_bias = c->dbg_lowd_any_bias != 0;
    if (extra_ptr) *extra_ptr = c->ws + (need - ((extra + 255) & ~size_t(255)));
    // The prepared part of the layout comes first and depends on the problem alone, so the derived copies of the clouds
    // sit at the same place in every entry call on the same problem.  When the caller has declared the clouds unchanged
    // (fs_points_keep) and the workspace still holds their copies, the part of the prologue that reads the clouds
    // (coordinate sums, mean, derived copies, norms) is skipped; biases and potentials are written anew by every call.
    Ctx::PointsKey key;
    key.x = p->x; key.y = p->y; key.dtype = (int)p->dtype; key.compute = (int)p->compute;
    key.n = p->n; key.m = p->m; key.d = p->d; key.ldx = p->ldx; key.ldy = p->ldy;
    Ctx::PointsKey declared = key;
    key.ws = c->ws;
    key.partial_budget = c->partial_budget;
    if (c->keep_on && c->kept_valid && key.same(c->kept_key)) {
        P->rho_max = c->kept_rho_max;
        return FS_OK;
    }
    c->kept_valid = false;   // whatever was kept is overwritten now
    fs_status st2 = launch_prepare(c, p, P);
    // (not in the static scratch array: other contexts on this GPU write there too)
    if (st2 == FS_OK && c->keep_on && !c->ws_static && declared.same(c->keep_key)) {
        c->kept_key = key;
        c->kept_rho_max = -1.0;   // (low-d path: set when the host reads it back, see launch_bias_from_user)
        c->kept_valid = true;
    }
    return st2;
}

// merge the splits of the pass that just ran over `res` (see launch_finalize)
fs_status finalize(Ctx *c, const Prepared *P, Side *res, int splits, double eps, double eps_next_bias, float *user_out,
                   double *abs_dev_sum, double mix = 1.0, double *save_old = nullptr, GaugeMode gauge = GaugeMode::None,
                   int64_t gauge_prev_cnt = 0, double gauge_prev_eps = 0.0)
{
    const double *nrm = (P->path == Path::LowD && !lowd_precise(P, eps)) ? res->norm_f : res->norm;
    return launch_finalize(c, P, res, nrm, splits, eps, eps_next_bias, user_out, abs_dev_sum, mix, save_old, gauge,
                           gauge_prev_cnt, gauge_prev_eps);
}

fs_status run_lse(Ctx *c, const Prepared *P, const Side *res, const Side *str, double eps, int *splits)
{
    switch (P->path) {
    case Path::LowD: return lowd_lse(c, P, res, str, eps, splits);
    case Path::F64: return f64_lse(c, P, res, str, eps, splits);
    case Path::BF16: return bf16_lse(c, P, res, str, eps, splits);
    }
    return FS_ERR_UNSUPPORTED;
}

// Plan application in two phases, so that a caller can place data in the workspace in between:
// apply_begin validates, sizes the workspace (with `tail_bytes` more for the caller, at *tail),
// prepares the problem and the biases of both sides; apply_run streams.
fs_status apply_begin(Ctx *c, const fs_problem *prob, float eps, const float *f, const float *g, int64_t p,
                      bool transposed, size_t tail_bytes, Prepared *P, char **tail)
{
    fs_status st;
    const int64_t n_res = transposed ? prob->m : prob->n;
    const int64_t n_str = transposed ? prob->n : prob->m;
    size_t extra = 0;
    switch (choose_path(prob)) {
    case Path::LowD: extra = lowd_apply_ws(c, n_res, n_str, prob->d, p); break;
    case Path::F64: extra = f64_apply_ws(c, n_res, n_str, prob->d, p); break;
    case Path::BF16: extra = bf16_apply_ws(c, n_res, n_str); break;
    }
    extra = (extra + 255) & ~size_t(255);
    if ((st = prepare(c, prob, P, extra + tail_bytes, &P->extra)) != FS_OK) return st;
    P->extra_bytes = extra;
    if (tail) *tail = P->extra + extra;
    if ((st = launch_bias_from_user(c, P, &P->X, f, eps, true, false)) != FS_OK) return st;
    return launch_bias_from_user(c, P, &P->Y, g, eps, false, true);
}

fs_status apply_run(Ctx *c, Prepared *P, float eps, bool transposed, const float *V, int64_t p, int64_t ldv, float *out,
                    int64_t ldo, float *mass)
{
    Side *res = transposed ? &P->Y : &P->X;
    Side *str = transposed ? &P->X : &P->Y;
    switch (P->path) {
    case Path::LowD: return lowd_apply(c, P, res, str, eps, V, p, ldv, out, ldo, mass);
    case Path::F64: return f64_apply(c, P, res, str, eps, V, p, ldv, out, ldo, mass);
    case Path::BF16: return bf16_apply(c, P, res, str, eps, V, p, ldv, out, ldo, mass);
    }
    return FS_ERR_UNSUPPORTED;
}

fs_status apply_common(Ctx *c, const fs_problem *prob, float eps, const float *f, const float *g,
                       const float *V, int64_t p, int64_t ldv, float *out, int64_t ldo, float *mass,
                       bool transposed)
{
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g || !V) return fail(c, FS_ERR_INVALID_ARG, "f, g or the matrix to apply is NULL");
    if (p <= 0 || p > 4096 || ldv < p || ldo < p) return fail(c, FS_ERR_BAD_SHAPE, "need 0 < p <= 4096, ld >= p");
    int64_t out_rows = transposed ? prob->m : prob->n;
    int64_t in_rows = transposed ? prob->n : prob->m;
    if ((st = check_out(c, prob, out, (size_t)((out_rows - 1) * ldo + p) * 4, "out")) != FS_OK) return st;
    if (mass && (st = check_out(c, prob, mass, (size_t)out_rows * 4, "mass output")) != FS_OK) return st;
    if (overlap(out, (size_t)((out_rows - 1) * ldo + p) * 4, V, (size_t)((in_rows - 1) * ldv + p) * 4) ||
        overlap(out, (size_t)((out_rows - 1) * ldo + p) * 4, f, (size_t)prob->n * 4) ||
        overlap(out, (size_t)((out_rows - 1) * ldo + p) * 4, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "out overlaps an input");
    Prepared P;
    if ((st = apply_begin(c, prob, eps, f, g, p, transposed, 0, &P, nullptr)) != FS_OK) return st;
    return apply_run(c, &P, eps, transposed, V, p, ldv, out, ldo, mass);
}

// a9: gradient of the OT value with respect to one cloud, assembled in the library on top of
// the plan applied to the other cloud
fs_status grad_common(Ctx *c, const fs_problem *prob, float eps, const float *f, const float *g, int32_t mode,
                      float *grad, int64_t ldg, bool wrt_y)
{
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g) return fail(c, FS_ERR_INVALID_ARG, "f or g is NULL");
    if (mode < 0 || mode > 2) return fail(c, FS_ERR_INVALID_ARG, "mode must be 0, 1 or 2");
    const int64_t d = prob->d;
    if (d > 4096 || ldg < d) return fail(c, FS_ERR_BAD_SHAPE, "need d <= 4096 and ldg >= d");
    const int64_t rows = wrt_y ? prob->m : prob->n;          // the cloud differentiated
    const int64_t orows = wrt_y ? prob->n : prob->m;         // the cloud the plan is applied to
    const size_t gbytes = (size_t)((rows - 1) * ldg + d) * 4;
    if ((st = check_out(c, prob, grad, gbytes, "grad")) != FS_OK) return st;
    if (overlap(grad, gbytes, f, (size_t)prob->n * 4) || overlap(grad, gbytes, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "grad overlaps an input");
    const void *opts = wrt_y ? prob->x : prob->y;
    const int64_t old = wrt_y ? prob->ldx : prob->ldy;
    const bool convert = prob->dtype != FS_F32;              // the value matrix of an application is float
    const size_t mass_bytes = ((size_t)rows * 4 + 255) & ~size_t(255);
    const size_t tail_bytes = mass_bytes + (convert ? (size_t)orows * d * 4 : 0);
    Prepared P;
    char *tail = nullptr;
    if ((st = apply_begin(c, prob, eps, f, g, d, wrt_y, tail_bytes, &P, &tail)) != FS_OK) return st;
    float *mass = reinterpret_cast<float *>(tail);
    const float *V = static_cast<const float *>(opts);
    int64_t ldv = old;
    if (convert) {
        float *vf = reinterpret_cast<float *>(tail + mass_bytes);
        if ((st = launch_pts_to_f32(c, opts, prob->dtype, orows, d, old, vf)) != FS_OK) return st;
        V = vf;
        ldv = d;
    }
    if ((st = apply_run(c, &P, eps, wrt_y, V, d, ldv, grad, ldg, mode == 1 ? mass : nullptr)) != FS_OK) return st;
    return launch_grad_assemble(c, grad, ldg, wrt_y ? prob->y : prob->x, prob->dtype, wrt_y ? prob->ldy : prob->ldx, rows, d,
                                wrt_y ? prob->b : prob->a, mass, mode);
}

// the context's second buffer (kept across the entry points that lay the workspace out anew), at least `need` bytes
fs_status ensure_aux(Ctx *c, size_t need)
{
    if (need <= c->aux_bytes) return FS_OK;
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (c->aux) {
        FS_HIP(c, hipFree(c->aux));
        c->aux = nullptr;
        c->aux_bytes = 0;
    }
    void *pnew = nullptr;
    hipError_t e = hipMalloc(&pnew, need);
    if (e != hipSuccess) return fail(c, FS_ERR_ALLOC, "buffer of %zu bytes: %s", need, hipGetErrorString(e));
    c->aux = (char *)pnew;
    c->aux_bytes = need;
    return FS_OK;
}

}  // namespace
}  // namespace fs

using namespace fs;

extern "C" {

const char *fs_version(void) { return "flashsink 0.1 gfx950"; }

const char *fs_status_str(fs_status s)
{
    switch (s) {
    case FS_OK: return "ok";
    case FS_ERR_INVALID_ARG: return "invalid argument";
    case FS_ERR_BAD_SHAPE: return "bad shape";
    case FS_ERR_BAD_EPS: return "bad eps or iteration count";
    case FS_ERR_BAD_WEIGHTS: return "bad weights";
    case FS_ERR_UNSUPPORTED: return "unsupported";
    case FS_ERR_ALLOC: return "device allocation failed";
    case FS_ERR_DEVICE: return "device error";
    case FS_ERR_NONFINITE: return "non-finite value";
    }
    return "unknown status";
}

const char *fs_last_error(const fs_ctx *ctx)
{
    return ctx ? reinterpret_cast<const Ctx *>(ctx)->err.c_str() : "";
}

fs_status fs_create(fs_ctx **ctx, int device, void *hip_stream)
{
    if (!ctx) return FS_ERR_INVALID_ARG;
    *ctx = nullptr;
    if (device == -1) {   // host-only context: argument validation works, nothing can be launched
        Ctx *h = new (std::nothrow) Ctx;
        if (!h) return FS_ERR_ALLOC;
        h->device = -1;
        *ctx = reinterpret_cast<fs_ctx *>(h);
        return FS_OK;
    }
    int count = 0;
    if (hipGetDeviceCount(&count) != hipSuccess || device < 0 || device >= count) return FS_ERR_DEVICE;
    Ctx *c = new (std::nothrow) Ctx;
    if (!c) return FS_ERR_ALLOC;
    c->device = device;
    c->stream = (hipStream_t)hip_stream;
    int prev = -1;
    const bool had_prev = hipGetDevice(&prev) == hipSuccess;
    if (hipSetDevice(device) != hipSuccess) {
        delete c;
        return FS_ERR_DEVICE;
    }
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, device) == hipSuccess && cu > 0)
        c->num_cu = cu;
    // this device's copy of the static scratch array (the device is current here)
    void *sp = nullptr;
    const hipError_t se = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
    if (had_prev && prev != device) (void)hipSetDevice(prev);
    if (se != hipSuccess || !sp) {
        delete c;
        return FS_ERR_DEVICE;
    }
    c->static_ws = static_cast<char *>(sp);
    *ctx = reinterpret_cast<fs_ctx *>(c);
    return FS_OK;
}

fs_status fs_destroy(fs_ctx *ctx)
{
    if (!ctx) return FS_OK;
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (c->device >= 0) {
        DeviceGuard device_guard(c);
        (void)hipStreamSynchronize(c->stream);
        for (hipEvent_t e : c->ev_pool) (void)hipEventDestroy(e);
        if (c->ws) (void)hipFree(c->ws);
        if (c->aux) (void)hipFree(c->aux);
    }
    delete c;
    return FS_OK;
}

fs_status fs_row_norms(fs_ctx *ctx, const void *pts, int32_t dtype, int64_t rows, int64_t d, int64_t ld,
                       float *out)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (!c) return FS_ERR_INVALID_ARG;
    c->err.clear();
    if (!pts || !out) return fail(c, FS_ERR_INVALID_ARG, "pts or out is NULL");
    if (dtype != FS_F32 && dtype != FS_BF16) return fail(c, FS_ERR_INVALID_ARG, "unknown dtype");
    if (rows <= 0 || d <= 0 || ld < d) return fail(c, FS_ERR_BAD_SHAPE, "rows, d must be positive and ld >= d");
    size_t es = dtype == FS_BF16 ? 2 : 4;
    if (overlap(out, (size_t)rows * 4, pts, (size_t)((rows - 1) * ld + d) * es))
        return fail(c, FS_ERR_INVALID_ARG, "out overlaps pts");
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    return launch_row_norms(c, pts, dtype, rows, d, ld, out);
}

fs_status fs_update_f(fs_ctx *ctx, const fs_problem *prob, float eps, const float *g, float *f_out)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!g) return fail(c, FS_ERR_INVALID_ARG, "g is NULL");
    if ((st = check_out(c, prob, f_out, (size_t)prob->n * 4, "f_out")) != FS_OK) return st;
    if (overlap(f_out, (size_t)prob->n * 4, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "f_out overlaps g");
    Prepared P;
    if ((st = prepare(c, prob, &P, 0, nullptr)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps)) != FS_OK) return st;
    int splits = 1;
    if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
    return finalize(c, &P, &P.X, splits, eps, 0.0, f_out, nullptr);
}

fs_status fs_update_g(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, float *g_out)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f) return fail(c, FS_ERR_INVALID_ARG, "f is NULL");
    if ((st = check_out(c, prob, g_out, (size_t)prob->m * 4, "g_out")) != FS_OK) return st;
    if (overlap(g_out, (size_t)prob->m * 4, f, (size_t)prob->n * 4))
        return fail(c, FS_ERR_INVALID_ARG, "g_out overlaps f");
    Prepared P;
    if ((st = prepare(c, prob, &P, 0, nullptr)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.X, f, eps)) != FS_OK) return st;
    int splits = 1;
    if ((st = run_lse(c, &P, &P.Y, &P.X, eps, &splits)) != FS_OK) return st;
    return finalize(c, &P, &P.Y, splits, eps, 0.0, g_out, nullptr);
}

// fs_solve and fs_solve_noalloc: `static_only` runs in the library's static scratch array and fails instead of allocating
static fs_status solve_impl(Ctx *c, const fs_problem *prob, float eps_start, float eps_end, int32_t n_stages,
                            int32_t iters_per_stage, float *f, float *g, bool static_only)
{
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps_end)) != FS_OK) return st;
    if (n_stages < 1 || iters_per_stage < 0)
        return fail(c, FS_ERR_BAD_EPS, "need n_stages >= 1 and iters_per_stage >= 0");
    if (n_stages > 1 && (st = validate_eps(c, eps_start)) != FS_OK) return st;
    if ((st = check_out(c, prob, f, (size_t)prob->n * 4, "f")) != FS_OK) return st;
    if ((st = check_out(c, prob, g, (size_t)prob->m * 4, "g")) != FS_OK) return st;
    if (overlap(f, (size_t)prob->n * 4, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "f overlaps g");
    // The workspace of a call that may not allocate is the static scratch array: sizes beyond it are refused here,
    // on the host, before anything is launched (also on a host-only context).
    struct StaticWs {   // swaps the static array in as the context's workspace for this call
        Ctx *c;
        char *ws;
        size_t bytes, budget;
        explicit StaticWs(Ctx *c_) : c(c_), ws(c_->ws), bytes(c_->ws_bytes), budget(c_->partial_budget)
        {
            c->ws = c->static_ws;
            c->ws_bytes = kStaticScratchBytes;
            c->ws_static = true;
            c->partial_budget = kStaticPartialBudget;
        }
        ~StaticWs()
        {
            c->ws = ws;
            c->ws_bytes = bytes;
            c->ws_static = false;
            c->partial_budget = budget;
        }
    };
    struct Maybe {   // (no heap: the guard lives in this frame)
        alignas(StaticWs) unsigned char buf[sizeof(StaticWs)];
        StaticWs *p = nullptr;
        ~Maybe()
        {
            if (p) p->~StaticWs();
        }
    } sw;
    if (static_only) {
        sw.p = new (sw.buf) StaticWs(c);
        Prepared sizing;
        const size_t need = layout(c, prob, &sizing, nullptr, 0);
        if (need > kStaticScratchBytes)
            return fail(c, FS_ERR_BAD_SHAPE,
                        "this problem needs %zu bytes of workspace; fs_solve_noalloc holds %zu (use fs_solve)", need,
                        kStaticScratchBytes);
    }
    if (iters_per_stage == 0) return c->device < 0 ? fail(c, FS_ERR_DEVICE, "host-only context") : FS_OK;

    Prepared P;
    P.halfsteps_per_eps = 2 * iters_per_stage;
    if ((st = prepare(c, prob, &P, 0, nullptr)) != FS_OK) return st;
    double eps0 = stage_eps(eps_start, eps_end, n_stages, 0);
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps0)) != FS_OK) return st;
    // the drift along (f + t, g - t) that the g-updates measure (see GaugeMode) is summed up on the device and taken
    // out when the potentials are handed to the caller
    if ((st = launch_fill_f64(c, P.scalars + 8, 0.0, 2)) != FS_OK) return st;
    double eps_prev = 0.0;
    double eps = eps0;
    for (int s = 0; s < n_stages; ++s) {
        eps = stage_eps(eps_start, eps_end, n_stages, s);
        for (int t = 0; t < iters_per_stage; ++t) {
            bool last = (s == n_stages - 1) && (t == iters_per_stage - 1);
            double eps_next = eps;
            if (t == iters_per_stage - 1 && !last) eps_next = stage_eps(eps_start, eps_end, n_stages, s + 1);
            int splits = 1;
            // Alg. 1: f from g
            if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
            if ((st = finalize(c, &P, &P.X, splits, eps, eps, nullptr, nullptr, 1.0, nullptr,
                               eps_prev > 0.0 ? GaugeMode::Collect : GaugeMode::None, prob->m, eps_prev)) != FS_OK)
                return st;
            // Alg. 3: g from the new f
            if ((st = run_lse(c, &P, &P.Y, &P.X, eps, &splits)) != FS_OK) return st;
            if ((st = finalize(c, &P, &P.Y, splits, eps, last ? 0.0 : eps_next, nullptr, nullptr, 1.0, nullptr,
                               GaugeMode::Measure)) != FS_OK)
                return st;
            eps_prev = eps;
        }
    }
    return launch_gauge_export(c, &P, true, eps, P.X.pot, f, g);
}

fs_status fs_solve(fs_ctx *ctx, const fs_problem *prob, float eps_start, float eps_end, int32_t n_stages,
                   int32_t iters_per_stage, float *f, float *g)
{
    return solve_impl(reinterpret_cast<Ctx *>(ctx), prob, eps_start, eps_end, n_stages, iters_per_stage, f, g, false);
}

fs_status fs_solve_noalloc(fs_ctx *ctx, const fs_problem *prob, float eps_start, float eps_end, int32_t n_stages,
                           int32_t iters_per_stage, float *f, float *g)
{
    return solve_impl(reinterpret_cast<Ctx *>(ctx), prob, eps_start, eps_end, n_stages, iters_per_stage, f, g, true);
}

fs_status fs_solve_labeled(fs_ctx *ctx, const fs_problem *prob, const int32_t *lx, const int32_t *ly, const float *W,
                           int32_t V, float lambda1, float lambda2, float eps, int32_t iters, float *f, float *g)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (iters < 0) return fail(c, FS_ERR_BAD_EPS, "need iters >= 0");
    if (!lx || !ly || !W) return fail(c, FS_ERR_INVALID_ARG, "lx, ly or W is NULL");
    if (V < 1 || prob->d + V > 8192) return fail(c, FS_ERR_BAD_SHAPE, "need V >= 1 and d + V <= 8192");
    if (!(lambda1 > 0.0f) || !isfinite(lambda1) || !isfinite(lambda2))
        return fail(c, FS_ERR_INVALID_ARG, "need lambda1 > 0 and both weights finite");
    if ((st = check_out(c, prob, f, (size_t)prob->n * 4, "f")) != FS_OK) return st;
    if ((st = check_out(c, prob, g, (size_t)prob->m * 4, "g")) != FS_OK) return st;
    if (overlap(f, (size_t)prob->n * 4, g, (size_t)prob->m * 4)) return fail(c, FS_ERR_INVALID_ARG, "f overlaps g");
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    if (iters == 0) return FS_OK;

    // augmented clouds, the per-point constants and the augmented potentials live in the context's second buffer (the
    // solve below lays the workspace out anew)
    const int64_t n = prob->n, m = prob->m, da = prob->d + V;
    auto al = [](size_t b) { return (b + 255) & ~size_t(255); };
    const size_t bx = al((size_t)n * da * 4), by = al((size_t)m * da * 4), bv = al((size_t)m * 4), bf = al((size_t)n * 4),
                 bg = al((size_t)m * 4);
    if ((st = ensure_aux(c, bx + by + bv + bf + bg + 256)) != FS_OK) return st;
    char *p = c->aux;
    float *xa = reinterpret_cast<float *>(p);
    float *ya = reinterpret_cast<float *>(p + bx);
    float *vc = reinterpret_cast<float *>(p + bx + by);
    float *fa = reinterpret_cast<float *>(p + bx + by + bv);
    float *ga = reinterpret_cast<float *>(p + bx + by + bv + bf);
    unsigned *bad = reinterpret_cast<unsigned *>(p + bx + by + bv + bf + bg);
    const double l1 = (double)lambda1, l2 = (double)lambda2;
    const bool bf16 = prob->compute == FS_COMPUTE_BF16_MFMA;
    if ((st = launch_fill_f64(c, reinterpret_cast<double *>(bad), 0.0, 1)) != FS_OK) return st;
    if ((st = launch_label_augment(c, prob->x, prob->dtype, n, prob->d, prob->ldx, lx, W, V, false, l1, l2, bf16, xa, nullptr,
                                   bad)) != FS_OK)
        return st;
    if ((st = launch_label_augment(c, prob->y, prob->dtype, m, prob->d, prob->ldy, ly, W, V, true, l1, l2, bf16, ya, vc, bad)) !=
        FS_OK)
        return st;
    // |xa - ya|^2 = (C + l1 + v_j) / l1: the augmented problem at eps / l1 with potentials ((f + l1) / l1, (g + v) / l1)
    if ((st = launch_label_potential(c, f, nullptr, l1, l1, true, n, fa)) != FS_OK) return st;
    if ((st = launch_label_potential(c, g, vc, 0.0, l1, true, m, ga)) != FS_OK) return st;
    fs_problem aug = *prob;
    aug.x = xa;
    aug.y = ya;
    aug.dtype = FS_F32;
    aug.d = da;
    aug.ldx = aug.ldy = da;
    const float eps_a = (float)((double)eps / l1);
    if ((st = solve_impl(c, &aug, eps_a, eps_a, 1, iters, fa, ga, false)) != FS_OK) return st;
    if ((st = launch_label_potential(c, fa, nullptr, l1, l1, false, n, f)) != FS_OK) return st;
    if ((st = launch_label_potential(c, ga, vc, 0.0, l1, false, m, g)) != FS_OK) return st;
    unsigned nbad = 0;
    FS_HIP(c, hipMemcpyAsync(&nbad, bad, sizeof nbad, hipMemcpyDeviceToHost, c->stream));
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (nbad) return fail(c, FS_ERR_INVALID_ARG, "%u labels are outside [0, V)", nbad);
    return FS_OK;
}

fs_status fs_solve_tol(fs_ctx *ctx, const fs_problem *prob, float eps_in, int32_t max_iters, int32_t check_every,
                       float tol, float *f, float *g, int32_t *iters_done, float *err_row_l1)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps_in)) != FS_OK) return st;
    if (max_iters < 1 || check_every < 1 || !(tol >= 0.0f))
        return fail(c, FS_ERR_BAD_EPS, "need max_iters >= 1, check_every >= 1 and tol >= 0");
    if ((st = check_out(c, prob, f, (size_t)prob->n * 4, "f")) != FS_OK) return st;
    if ((st = check_out(c, prob, g, (size_t)prob->m * 4, "g")) != FS_OK) return st;
    if (overlap(f, (size_t)prob->n * 4, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "f overlaps g");
    if (!iters_done || !err_row_l1) return fail(c, FS_ERR_INVALID_ARG, "iters_done or err_row_l1 is NULL");

    const double eps = (double)eps_in;
    Prepared P;
    P.halfsteps_per_eps = 2 * max_iters;
    char *extra = nullptr;
    if ((st = prepare(c, prob, &P, (size_t)prob->n * 8, &extra)) != FS_OK) return st;
    double *f_before = reinterpret_cast<double *>(extra);   // f of the last completed iteration at a check
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps)) != FS_OK) return st;
    if ((st = launch_fill_f64(c, P.scalars, 0.0, 1)) != FS_OK) return st;
    if ((st = launch_fill_f64(c, P.scalars + 8, 0.0, 2)) != FS_OK) return st;   // drift along (f + t, g - t), see GaugeMode
    bool gauge_pending = false;   // a g-update's measurement waits for the next f-update to collect it
    // The row marginal error of (f_t, g_t) is a by-product of the f-update that starts iteration
    // t + 1 (Prop. 3: r = a exp((f_t - f_{t+1})/eps)), so a check costs no extra pass unless it stops
    // the iteration.  `pending`: that f-update has already been done.
    bool pending = false;
    int t = 0;
    double err = -1.0;
    while (true) {
        int splits = 1;
        if (!pending) {   // Alg. 1: f from g
            if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
            if ((st = finalize(c, &P, &P.X, splits, eps, eps, nullptr, nullptr, 1.0, nullptr,
                               gauge_pending ? GaugeMode::Collect : GaugeMode::None, prob->m, eps)) != FS_OK)
                return st;
            gauge_pending = false;
        }
        pending = false;
        // Alg. 3: g from the new f
        if ((st = run_lse(c, &P, &P.Y, &P.X, eps, &splits)) != FS_OK) return st;
        if ((st = finalize(c, &P, &P.Y, splits, eps, eps, nullptr, nullptr, 1.0, nullptr, GaugeMode::Measure)) != FS_OK) return st;
        gauge_pending = true;
        ++t;
        if (t % check_every != 0 && t != max_iters) continue;
        // the next f-update, measuring the error of (f_t, g_t) on the way
        if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
        if ((st = finalize(c, &P, &P.X, splits, eps, eps, nullptr, P.scalars, 1.0, f_before, GaugeMode::Collect, prob->m, eps)) !=
            FS_OK)
            return st;
        gauge_pending = false;
        FS_HIP(c, hipMemcpyAsync(&err, P.scalars, sizeof(double), hipMemcpyDeviceToHost, c->stream));
        FS_HIP(c, hipStreamSynchronize(c->stream));
        if (err <= (double)tol || t == max_iters) break;
        pending = true;
    }
    // f_t sat before the last g-update's term entered the sum, g_t behind it
    if ((st = launch_gauge_export(c, &P, false, eps, f_before, f, g)) != FS_OK) return st;
    FS_HIP(c, hipStreamSynchronize(c->stream));
    *iters_done = t;
    *err_row_l1 = (float)err;
    return FS_OK;
}

fs_status fs_solve_symmetric(fs_ctx *ctx, const fs_problem *prob, float eps_in, int32_t iters, float *f, float *g)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps_in)) != FS_OK) return st;
    if (iters < 0) return fail(c, FS_ERR_BAD_EPS, "need iters >= 0");
    if ((st = check_out(c, prob, f, (size_t)prob->n * 4, "f")) != FS_OK) return st;
    if ((st = check_out(c, prob, g, (size_t)prob->m * 4, "g")) != FS_OK) return st;
    if (overlap(f, (size_t)prob->n * 4, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "f overlaps g");
    if (iters == 0) return c->device < 0 ? fail(c, FS_ERR_DEVICE, "host-only context") : FS_OK;

    const double eps = (double)eps_in;
    Prepared P;
    P.halfsteps_per_eps = 2 * iters;
    // Both passes of an iteration read the old potentials, so the second one must not overwrite
    // the split partials of the first before they are merged: it gets a partial buffer of its own.
    Prepared sizing;
    layout(c, prob, &sizing, nullptr, 0);
    const size_t second = sizing.partial_bytes;
    char *second_partial = nullptr;
    if ((st = prepare(c, prob, &P, second, &second_partial)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.X, f, eps, true, false)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps, false, true)) != FS_OK) return st;
    void *const first_partial = P.partial;
    if ((st = launch_fill_f64(c, P.scalars + 8, 0.0, 2)) != FS_OK) return st;
    for (int t = 0; t < iters; ++t) {
        const bool last = t == iters - 1;
        int splits_f = 1, splits_g = 1;
        const double eps_bias = last ? 0.0 : eps;
        if (P.path == Path::LowD) {
            // both passes in one launch and both merges in another, when the half-steps run on the
            // split-record kernels: at small n an iteration is bound by launch latency
            bool done = false;
            P.partial = first_partial;
            if ((st = lowd_lse_pair(c, &P, eps, first_partial, second_partial, &splits_f, &splits_g, &done)) != FS_OK)
                return st;
            if (done) {
                const bool pr = lowd_precise(&P, eps);
                if ((st = launch_finalize_pair(c, &P, &P.X, pr ? P.X.norm : P.X.norm_f, first_partial, splits_f, nullptr, &P.Y,
                                               pr ? P.Y.norm : P.Y.norm_f, second_partial, splits_g, nullptr, eps, eps_bias, 0.5, t,
                                               t > 0)) != FS_OK)
                    return st;
                continue;
            }
        }
        P.partial = first_partial;
        const bool f64_kernels = P.path == Path::F64 || (P.path == Path::LowD && P.X.pts_d && P.Y.pts_d);
        if (f64_kernels) {
            // (fp64 matrix-core passes, also on behalf of the low-d path at d > 3: both in one launch)
            if ((st = f64_lse_pair(c, &P, eps, first_partial, second_partial, &splits_f, &splits_g)) != FS_OK) return st;
        } else if (P.path == Path::BF16) {
            if ((st = bf16_lse_pair(c, &P, eps, first_partial, second_partial, &splits_f, &splits_g)) != FS_OK) return st;
        } else {
            if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits_f)) != FS_OK) return st;   // Eq. 4: from the old g
            P.partial = second_partial;
            if ((st = run_lse(c, &P, &P.Y, &P.X, eps, &splits_g)) != FS_OK) return st;   // Eq. 5: from the old f
        }
        // only now are the potentials (and the biases the next iteration streams) replaced: both merges in one launch
        P.partial = first_partial;
        {
            const bool fl = P.path == Path::LowD && !lowd_precise(&P, eps);   // which norms the pass was biased with
            if ((st = launch_finalize_pair(c, &P, &P.X, fl ? P.X.norm_f : P.X.norm, first_partial, splits_f, nullptr, &P.Y,
                                           fl ? P.Y.norm_f : P.Y.norm, second_partial, splits_g, nullptr, eps, eps_bias, 0.5, t,
                                           t > 0)) != FS_OK)
                return st;
        }
    }
    // the drift along (f + t, g - t) that the iterations measured (see launch_finalize_pair), taken out on the way out
    if ((st = launch_gauge_collect_pair(c, &P, eps, iters - 1)) != FS_OK) return st;
    return launch_gauge_export(c, &P, false, eps, P.X.pot, f, g);
}

fs_status fs_marginal_err(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                          float *err_row_l1, float *err_col_l1)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g) return fail(c, FS_ERR_INVALID_ARG, "f or g is NULL");
    Prepared P;
    P.force_precise = true;   // a measurement: always the accurate score arithmetic
    if ((st = prepare(c, prob, &P, 0, nullptr)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.X, f, eps, true, false)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps, false, true)) != FS_OK) return st;
    // (the two error sums only: slots 5..7 belong to the prologue and, with kept derived copies, to later calls)
    if ((st = launch_fill_f64(c, P.scalars, 0.0, 2)) != FS_OK) return st;
    int splits = 1;
    if (err_row_l1) {
        if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
        if ((st = finalize(c, &P, &P.X, splits, eps, 0.0, nullptr, P.scalars + 0)) != FS_OK) return st;
    }
    if (err_col_l1) {
        if ((st = run_lse(c, &P, &P.Y, &P.X, eps, &splits)) != FS_OK) return st;
        if ((st = finalize(c, &P, &P.Y, splits, eps, 0.0, nullptr, P.scalars + 1)) != FS_OK) return st;
    }
    double host[2] = {0.0, 0.0};
    FS_HIP(c, hipMemcpyAsync(host, P.scalars, sizeof host, hipMemcpyDeviceToHost, c->stream));
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (err_row_l1) *err_row_l1 = (float)host[0];
    if (err_col_l1) *err_col_l1 = (float)host[1];
    return FS_OK;
}

fs_status fs_ot_value(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g, double *value)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g || !value) return fail(c, FS_ERR_INVALID_ARG, "f, g or value is NULL");
    Prepared P;
    P.force_precise = true;   // a measurement: always the accurate score arithmetic
    const size_t scratch_bytes = (3 * (size_t)ceil_div(prob->n, 256) + 2 * (size_t)ceil_div(prob->m, 256)) * 8;
    char *scratch = nullptr;
    if ((st = prepare(c, prob, &P, scratch_bytes, &scratch)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.X, f, eps, true, false)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps, false, true)) != FS_OK) return st;
    int splits = 1;
    if ((st = run_lse(c, &P, &P.X, &P.Y, eps, &splits)) != FS_OK) return st;
    const double *nrm = (P.path == Path::LowD && !lowd_precise(&P, eps)) ? P.X.norm_f : P.X.norm;
    if ((st = launch_value_terms(c, &P, &P.X, nrm, &P.Y, splits, eps, reinterpret_cast<double *>(scratch), P.scalars)) !=
        FS_OK)
        return st;
    double h[5] = {0.0, 0.0, 0.0, 0.0, 0.0};
    FS_HIP(c, hipMemcpyAsync(h, P.scalars, sizeof h, hipMemcpyDeviceToHost, c->stream));
    FS_HIP(c, hipStreamSynchronize(c->stream));
    // App. B: <a,f> + <b,g> - eps (sum_ij P_ij - sum_ij a_i b_j)
    *value = h[1] + h[3] - (double)eps * (h[0] - h[2] * h[4]);
    return FS_OK;
}

fs_status fs_check_finite(fs_ctx *ctx, const float *v, int64_t cnt, int64_t *bad_count)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (!c) return FS_ERR_INVALID_ARG;
    c->err.clear();
    if (!v) return fail(c, FS_ERR_INVALID_ARG, "v is NULL");
    if (cnt < 1) return fail(c, FS_ERR_BAD_SHAPE, "cnt must be >= 1");
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    const size_t nb = (size_t)ceil_div(cnt, 256);
    fs_status st = ensure_aux(c, (nb + 1) * sizeof(double));
    if (st != FS_OK) return st;
    double *res = reinterpret_cast<double *>(c->aux);
    if ((st = launch_count_nonfinite(c, v, cnt, res + 1, res)) != FS_OK) return st;
    double h = 0.0;
    FS_HIP(c, hipMemcpyAsync(&h, res, sizeof h, hipMemcpyDeviceToHost, c->stream));
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (bad_count) *bad_count = (int64_t)h;
    if (h > 0.0) return fail(c, FS_ERR_NONFINITE, "%.0f of %lld values are not finite", h, (long long)cnt);
    return FS_OK;
}

fs_status fs_check_weights(fs_ctx *ctx, const fs_problem *prob, float tol, double *sum_a, double *sum_b)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if (!(tol >= 0.0f) || !(tol < INFINITY)) return fail(c, FS_ERR_INVALID_ARG, "tol must be finite and >= 0");
    if (sum_a) *sum_a = 1.0;
    if (sum_b) *sum_b = 1.0;
    if (!prob->a && !prob->b) return FS_OK;   // uniform weights on both sides
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    const size_t ba = (size_t)ceil_div(prob->n, 256), bb = (size_t)ceil_div(prob->m, 256);
    if ((st = ensure_aux(c, (2 * (ba + bb) + 4) * sizeof(double))) != FS_OK) return st;
    double *res = reinterpret_cast<double *>(c->aux), *scratch = res + 4;
    double h[4] = {1.0, 0.0, 1.0, 0.0};
    if (prob->a && (st = launch_weight_stats(c, prob->a, prob->n, scratch, res)) != FS_OK) return st;
    if (prob->b && (st = launch_weight_stats(c, prob->b, prob->m, scratch + 2 * ba, res + 2)) != FS_OK) return st;
    if (prob->a) FS_HIP(c, hipMemcpyAsync(h, res, 2 * sizeof(double), hipMemcpyDeviceToHost, c->stream));
    if (prob->b) FS_HIP(c, hipMemcpyAsync(h + 2, res + 2, 2 * sizeof(double), hipMemcpyDeviceToHost, c->stream));
    FS_HIP(c, hipStreamSynchronize(c->stream));
    if (sum_a) *sum_a = h[0];
    if (sum_b) *sum_b = h[2];
    if (h[1] > 0.0) return fail(c, FS_ERR_BAD_WEIGHTS, "%.0f weights of a are not positive and finite", h[1]);
    if (h[3] > 0.0) return fail(c, FS_ERR_BAD_WEIGHTS, "%.0f weights of b are not positive and finite", h[3]);
    if (fabs(h[0] - 1.0) > (double)tol) return fail(c, FS_ERR_BAD_WEIGHTS, "a sums to %.9g", h[0]);
    if (fabs(h[2] - 1.0) > (double)tol) return fail(c, FS_ERR_BAD_WEIGHTS, "b sums to %.9g", h[2]);
    return FS_OK;
}

fs_status fs_divergence(fs_ctx *ctx, const fs_problem *prob, float eps, int32_t iters, float *f, float *g, double *value,
                        double *terms)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (iters < 1) return fail(c, FS_ERR_BAD_EPS, "need iters >= 1");
    if (!value) return fail(c, FS_ERR_INVALID_ARG, "value is NULL");
    if ((st = check_out(c, prob, f, (size_t)prob->n * 4, "f")) != FS_OK) return st;
    if ((st = check_out(c, prob, g, (size_t)prob->m * 4, "g")) != FS_OK) return st;
    if (overlap(f, (size_t)prob->n * 4, g, (size_t)prob->m * 4)) return fail(c, FS_ERR_INVALID_ARG, "f overlaps g");
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context: arguments are valid, nothing was launched");
    // potentials of the two self-terms: the entry points called below lay the workspace out anew, so
    // these live in a buffer of their own
    const int64_t big = prob->n > prob->m ? prob->n : prob->m;
    if ((st = ensure_aux(c, (size_t)2 * big * sizeof(float))) != FS_OK) return st;
    float *sf = reinterpret_cast<float *>(c->aux), *sg = sf + big;
    double v[3] = {0.0, 0.0, 0.0};
    // cross term: OT(a, b)
    FS_HIP(c, hipMemsetAsync(f, 0, (size_t)prob->n * 4, c->stream));
    FS_HIP(c, hipMemsetAsync(g, 0, (size_t)prob->m * 4, c->stream));
    if ((st = fs_solve(ctx, prob, eps, eps, 1, iters, f, g)) != FS_OK) return st;
    if ((st = fs_ot_value(ctx, prob, eps, f, g, &v[0])) != FS_OK) return st;
    // self terms: OT(a, a) and OT(b, b)
    for (int k = 0; k < 2; ++k) {
        fs_problem self = *prob;
        if (k == 0) {
            self.y = prob->x;
            self.m = prob->n;
            self.ldy = prob->ldx;
            self.b = prob->a;
        } else {
            self.x = prob->y;
            self.n = prob->m;
            self.ldx = prob->ldy;
            self.a = prob->b;
        }
        FS_HIP(c, hipMemsetAsync(sf, 0, (size_t)self.n * 4, c->stream));
        FS_HIP(c, hipMemsetAsync(sg, 0, (size_t)self.m * 4, c->stream));
        if ((st = fs_solve(ctx, &self, eps, eps, 1, iters, sf, sg)) != FS_OK) return st;
        if ((st = fs_ot_value(ctx, &self, eps, sf, sg, &v[1 + k])) != FS_OK) return st;
    }
    *value = v[0] - 0.5 * v[1] - 0.5 * v[2];
    if (terms) {
        terms[0] = v[0];
        terms[1] = v[1];
        terms[2] = v[2];
    }
    return FS_OK;
}

fs_status fs_apply_plan(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                        const float *V, int64_t p, int64_t ldv, float *out, int64_t ldo, float *r_out)
{
    return apply_common(reinterpret_cast<Ctx *>(ctx), prob, eps, f, g, V, p, ldv, out, ldo, r_out, false);
}

fs_status fs_apply_plan_T(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                          const float *U, int64_t p, int64_t ldu, float *out, int64_t ldo, float *c_out)
{
    return apply_common(reinterpret_cast<Ctx *>(ctx), prob, eps, f, g, U, p, ldu, out, ldo, c_out, true);
}

fs_status fs_grad_x(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g, int32_t mode,
                    float *grad, int64_t ldg)
{
    return grad_common(reinterpret_cast<Ctx *>(ctx), prob, eps, f, g, mode, grad, ldg, false);
}

fs_status fs_grad_y(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g, int32_t mode,
                    float *grad, int64_t ldg)
{
    return grad_common(reinterpret_cast<Ctx *>(ctx), prob, eps, f, g, mode, grad, ldg, true);
}

fs_status fs_hvp(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g, const float *A,
                 int64_t lda, float tau, float eta, int32_t max_cg, float *out, int64_t ldo, int32_t *cg_iters)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g || !A) return fail(c, FS_ERR_INVALID_ARG, "f, g or A is NULL");
    if (lda < prob->d || ldo < prob->d) return fail(c, FS_ERR_BAD_SHAPE, "lda and ldo must be at least d");
    if (!(tau >= 0.0f) || !(eta >= 0.0f) || max_cg < 0)
        return fail(c, FS_ERR_BAD_EPS, "need tau >= 0, eta >= 0 and max_cg >= 0");
    if (prob->dtype != FS_F32 || prob->compute != FS_COMPUTE_FP32)
        return fail(c, FS_ERR_UNSUPPORTED, "the Hessian-vector product is available for float32 points and FS_COMPUTE_FP32");
    const size_t out_bytes = (size_t)((prob->n - 1) * ldo + prob->d) * 4;
    if ((st = check_out(c, prob, out, out_bytes, "out")) != FS_OK) return st;
    if (overlap(out, out_bytes, A, (size_t)((prob->n - 1) * lda + prob->d) * 4) ||
        overlap(out, out_bytes, f, (size_t)prob->n * 4) || overlap(out, out_bytes, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "out overlaps an input");
    Prepared P;
    const bool lowd = choose_path(prob) == Path::LowD;
    const size_t ws_f = lowd ? lowd_apply_ws(c, prob->n, prob->m, prob->d, prob->d) : f64_apply_ws(c, prob->n, prob->m, prob->d, prob->d);
    const size_t ws_g = lowd ? lowd_apply_ws(c, prob->m, prob->n, prob->d, prob->d) : f64_apply_ws(c, prob->m, prob->n, prob->d, prob->d);
    const size_t apply_ws = ((ws_f > ws_g ? ws_f : ws_g) + 255) & ~size_t(255);
    char *extra = nullptr;
    if ((st = prepare(c, prob, &P, apply_ws + hvp_scratch_bytes(prob->n, prob->m, prob->d), &extra)) != FS_OK) return st;
    P.extra = extra;
    P.extra_bytes = apply_ws;
    if ((st = launch_bias_from_user(c, &P, &P.X, f, eps, true, false)) != FS_OK) return st;
    if ((st = launch_bias_from_user(c, &P, &P.Y, g, eps, false, true)) != FS_OK) return st;
    int iters = 0;
    st = hvp_run(c, &P, static_cast<const float *>(prob->x), prob->ldx, static_cast<const float *>(prob->y), prob->ldy,
                 (double)eps, A, lda, (double)tau, (double)eta, max_cg, out, ldo, extra + apply_ws, &iters);
    if (cg_iters) *cg_iters = iters;
    return st;
}

fs_status fs_apply_plan_hadamard(fs_ctx *ctx, const fs_problem *prob, float eps, const float *f, const float *g,
                                 const float *A, int64_t lda, const float *V, int64_t p, int64_t ldv, float *out, int64_t ldo)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    if ((st = validate_eps(c, eps)) != FS_OK) return st;
    if (!f || !g || !A || !V) return fail(c, FS_ERR_INVALID_ARG, "f, g, A or V is NULL");
    if (p <= 0 || p > 4096 || ldv < p || ldo < p || lda < prob->d)
        return fail(c, FS_ERR_BAD_SHAPE, "need 0 < p <= 4096, ldv >= p, ldo >= p and lda >= d");
    if (prob->dtype != FS_F32 || prob->compute != FS_COMPUTE_FP32)
        return fail(c, FS_ERR_UNSUPPORTED, "the Hadamard-weighted transport is available for float32 points and FS_COMPUTE_FP32");
    const size_t out_bytes = (size_t)((prob->n - 1) * ldo + p) * 4;
    if ((st = check_out(c, prob, out, out_bytes, "out")) != FS_OK) return st;
    if (overlap(out, out_bytes, A, (size_t)((prob->n - 1) * lda + prob->d) * 4) ||
        overlap(out, out_bytes, V, (size_t)((prob->m - 1) * ldv + p) * 4) || overlap(out, out_bytes, f, (size_t)prob->n * 4) ||
        overlap(out, out_bytes, g, (size_t)prob->m * 4))
        return fail(c, FS_ERR_INVALID_ARG, "out overlaps an input");
    // The low-d kernels form the weights against the points centred at the common mean; the mean's share,
    // <A_i, mean> (P V)_i, comes from a plain application into the workspace.  Above d = 16 nothing is centred.
    const bool lowd = choose_path(prob) == Path::LowD;
    Prepared P;
    char *tail = nullptr;
    if ((st = apply_begin(c, prob, eps, f, g, p, false, lowd ? (size_t)prob->n * p * 4 : 0, &P, &tail)) != FS_OK) return st;
    if (lowd) {
        if ((st = lowd_apply(c, &P, &P.X, &P.Y, eps, V, p, ldv, out, ldo, nullptr, A, lda)) != FS_OK) return st;
        float *PV = reinterpret_cast<float *>(tail);
        if ((st = lowd_apply(c, &P, &P.X, &P.Y, eps, V, p, ldv, PV, p, nullptr)) != FS_OK) return st;
        return launch_add_mean_share(c, A, lda, P.mean, PV, prob->n, (int)prob->d, (int)p, out, ldo);
    }
    return f64_apply(c, &P, &P.X, &P.Y, eps, V, p, ldv, out, ldo, nullptr, A, lda);
}

fs_status fs_points_keep(fs_ctx *ctx, const fs_problem *prob)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    if (!c) return FS_ERR_INVALID_ARG;
    fs_status st = validate_problem(c, prob);
    if (st != FS_OK) return st;
    Ctx::PointsKey k;
    k.x = prob->x; k.y = prob->y; k.dtype = (int)prob->dtype; k.compute = (int)prob->compute;
    k.n = prob->n; k.m = prob->m; k.d = prob->d; k.ldx = prob->ldx; k.ldy = prob->ldy;
    c->keep_key = k;
    c->keep_on = true;
    c->kept_valid = false;   // the copies are built by the next entry call on these clouds
    return FS_OK;
}

fs_status fs_points_release(fs_ctx *ctx)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    if (!c) return FS_ERR_INVALID_ARG;
    c->err.clear();
    c->keep_on = false;
    c->kept_valid = false;
    return FS_OK;
}

fs_status fs_debug_set(fs_ctx *ctx, const char *key, int64_t value)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (!c) return FS_ERR_INVALID_ARG;
    c->err.clear();
    if (!key) return fail(c, FS_ERR_INVALID_ARG, "key is NULL");
    const std::string k(key);
    if (k == "lowd_splits" && value >= 0 && value <= 1024)
        c->dbg_lowd_splits = (int)value;
    else if (k == "lowd_score" && (value == 0 || value == 32 || value == 64))
        c->dbg_lowd_score = (int)value;
    else if (k == "lowd_precise_valu" && (value == 0 || value == 1))
        c->dbg_lowd_precise_valu = (int)value;
    else if (k == "lowd_precise_any_bias" && (value == 0 || value == 1))
        c->dbg_lowd_any_bias = (int)value;
    else
        return fail(c, FS_ERR_INVALID_ARG, "unknown switch or value out of range: %s = %lld", key, (long long)value);
    return FS_OK;
}

fs_status fs_profile_enable(fs_ctx *ctx, int32_t on)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (!c) return FS_ERR_INVALID_ARG;
    c->prof_on = on != 0;
    return FS_OK;
}

fs_status fs_profile_read(fs_ctx *ctx, double *avg_ms, int64_t *launches, double *pairs_per_launch)
{
    Ctx *c = reinterpret_cast<Ctx *>(ctx);
    DeviceGuard device_guard(c);
    if (!c) return FS_ERR_INVALID_ARG;
    if (c->device < 0) return fail(c, FS_ERR_DEVICE, "host-only context");
    FS_HIP(c, hipStreamSynchronize(c->stream));
    // per kernel kind; the one with the largest total time is the dominant kernel
    double total[2] = {0.0, 0.0}, pairs[2] = {0.0, 0.0};
    int64_t cnt[2] = {0, 0};
    for (size_t k = 0; k + 1 < c->ev_used; k += 2) {
        float ms = 0.0f;
        if (hipEventElapsedTime(&ms, c->ev_pool[k], c->ev_pool[k + 1]) == hipSuccess) {
            const int kind = c->ev_kind[k / 2] ? 1 : 0;
            total[kind] += ms;
            pairs[kind] += c->ev_pairs[k / 2];
            ++cnt[kind];
        }
    }
    const int dom = total[1] > total[0] ? 1 : 0;
    if (avg_ms) *avg_ms = cnt[dom] ? total[dom] / (double)cnt[dom] : 0.0;
    if (launches) *launches = cnt[dom];
    if (pairs_per_launch) *pairs_per_launch = cnt[dom] ? pairs[dom] / (double)cnt[dom] : 0.0;
    c->ev_used = 0;
    return FS_OK;
}

}  // extern "C"
