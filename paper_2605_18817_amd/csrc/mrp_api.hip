// C ABI of libmrp (see include/mrp.h): context, argument validation and the
// chain driver that enqueues one denoising step's K-head chain on one stream.
#include "../../include/mrp.h"

#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <vector>

#include "mrp_kernels.h"

using namespace mrp;

struct mrp_ctx {
    mrp_dims dims;
    int device;
    int nIb;            // activation row blocks per k block (multiple of 8)
    long plane;         // uint4 per activation plane
    int nT_max;         // partial tiles per row
    size_t part_rows;   // capacity of the k-split partial buffer, in rows of d floats
    int maxB;
    bool use_tiled;     // 256 x 256 tiled GEMMs for M >= 768
    bool lm_persist;    // the persistent LM-head kernel for M <= 512 (launches of at most 256 rows)
    int nCU;            // compute units of the device (workgroups of the persistent LM-head kernel)
    char *ws;
    size_t ws_bytes;
    uint4 *XH, *XE, *S, *Y;
    float *PART, *pm, *ps;
    int *pi;
    float *vwm;
    int *vwi;
    float *kl_part, *kl_lse;   // KL loss: 5 partial arrays [max_rows * tiles], row log-sum-exps [2][max_rows]
    size_t kl_stride;
    double *rms_part;          // residual magnitudes: per-workgroup sums of squares
    int *err_flag;             // device error word (MRP_FLAG_* bits), read and cleared by mrp_poll_error
    // transformer head body (mrp_tbody_create): its own allocation
    bool tb_on;
    mrp_tbody_dims tb;
    char *tb_ws;
    float *tb_U;               // residual stream [max_rows][d]
    uint4 *tb_P;               // NSPLIT activation planes, tb_plane uint4 each (widest of d, nh*hd, d_ff columns)
    long tb_plane;
    float *tb_part;            // partial sums, tb_part_floats floats
    size_t tb_part_floats;
    float2 *tb_rope;           // [max_rows][64]
    float *tb_attn;            // attention partials, attention_scratch_floats() floats
    char err[512];
    bool prof_on;
    std::vector<hipEvent_t> ev;  // pairs
    int ev_used;
};

namespace {

constexpr int PROF_PAIRS = 4096;

size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct Layout {
    int nIb;
    long plane;
    int nT_max;
    size_t part_rows;
    int maxB;
    size_t off_XH, off_XE, off_S, off_Y, off_PART, off_pm, off_ps, off_pi, off_vwm, off_vwi, off_klp, off_kll, off_rms, off_err, total;
    size_t kl_stride;
};

bool dims_ok(const mrp_dims *d) {
    return d && d->d >= 128 && d->d % 128 == 0 && d->d <= 8192 && d->V >= 1 && d->max_rows >= 1 &&
           d->max_rows <= 65535 && d->block_len >= 1 && d->block_len <= MRP_MAX_BLOCK_LEN &&
           d->max_rows % d->block_len == 0 && d->rms_eps >= 0.f;
}

Layout make_layout(const mrp_dims *dm, int nCU) {
    Layout l;
    const int ib = (dm->max_rows + 31) / 32;
    l.nIb = (ib + 7) / 8 * 8;
    l.plane = (long)(dm->d / 16) * l.nIb * 64;
    const int nT_lm = ((dm->V + 31) / 32 + WG_WAVES - 1) / WG_WAVES;
    const int nT_0 = reduce_rows_tiles(dm->V);
    l.nT_max = nT_lm > nT_0 ? nT_lm : nT_0;
    const int nT_p = nCU;  // persistent LM-head kernel: one slot per workgroup
    if (nT_p > l.nT_max) l.nT_max = nT_p;
    // (k-split partial sums: 16 parts at up to 128 rows; beyond, 4096 rows hold 4 parts of 1024 rows or 2 of 2048)
    l.part_rows = dm->max_rows <= 128 ? (size_t)dm->max_rows * 16 : (dm->max_rows < 4096 ? 4096 : dm->max_rows);
    l.maxB = dm->max_rows / dm->block_len;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
    l.off_XH = take((size_t)NSPLIT * l.plane * 16);
    l.off_XE = take((size_t)l.plane * 16);
    l.off_S = take((size_t)NSPLIT * l.plane * 16);
    l.off_Y = take((size_t)l.plane * 16);
    l.off_PART = take(l.part_rows * dm->d * sizeof(float));
    l.off_pm = take((size_t)l.nT_max * dm->max_rows * 4);
    l.off_ps = take((size_t)l.nT_max * dm->max_rows * 4);
    l.off_pi = take((size_t)l.nT_max * dm->max_rows * 4);
    const size_t vw = (size_t)l.maxB * MRP_MAX_HEADS * verify_chunks(dm->V);
    l.off_vwm = take(vw * 4);
    l.off_vwi = take(vw * 4);
    l.kl_stride = (size_t)dm->max_rows * kl_tiles(dm->V);
    l.off_klp = take(5 * l.kl_stride * 4);
    l.off_kll = take((size_t)2 * dm->max_rows * 4);
    l.off_rms = take(residual_rms_part_bytes());
    l.off_err = take(256);
    l.total = o;
    return l;
}

int fail(mrp_ctx *c, int code, const char *fmt, ...) {
    if (c) {
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(c->err, sizeof(c->err), fmt, ap);
        va_end(ap);
    }
    return code;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

#define HIP_TRY(ctx, expr)                                                                      \
    do {                                                                                        \
        hipError_t e_ = (expr);                                                                 \
        if (e_ != hipSuccess) return fail(ctx, MRP_ERR_HIP, "%s: %s", #expr, hipGetErrorString(e_)); \
    } while (0)

// k splits for a partial-sum GEMM so that small row counts still fill the chip
int pick_ksplit(int nVt, int nMg, int G, size_t part_rows, int M) {
    int want = (512 + nVt * nMg - 1) / (nVt * nMg);
    if (want > 16) want = 16;
    if (want > G / 2) want = G / 2;
    if ((size_t)want * M > part_rows) want = (int)(part_rows / M);
    return want < 1 ? 1 : want;
}

// Which GEMM kernel the head body (and the transformer body's projections) take for M rows and operands of
// width Kc.  The 256 x 256 tile kernel (with its k split when the tiles are few) from 768 rows, for wide
// operands from 513; below, the kernels that reduce their k split inside the workgroup (no partial sums in
// memory).  Measured per head of the MLP body, small-row kernels against the tile kernel: d = 4096 153 / 156 /
// 208 / 254 / 294 us at 192 / 256 / 384 / 512 / 640 rows against 248 / 272 / 240 / 258 / 226 us; d = 2048 63 /
// 103 / 128 us at 256 / 512 / 640 rows against 119 / 120 / 145 us.  (The streaming kernel with its partial
// sums is behind both: d = 2048 102 / 133 / 160 us at 256 / 512 / 640 rows, d = 4096 202 / 268 / 329 us at
// 256 / 512 / 752 rows.)
bool body_on_tiles(int M, int Kc) { return M >= 768 || (Kc > 2048 && M > 512); }
bool small_rows_kernel(int M, int Kc) { return !body_on_tiles(M, Kc); }

// Weight row blocks per tile of the small-row GEMM kernels: two (64 features), so that a workgroup's
// activation fragments serve twice the weights, once there are more 32-feature tiles than CUs and at least
// six row tiles (measured per head: d = 4096 at 384 rows 209 us against 227, d = 2048 at 256 rows 63 us
// against 70; but at 128 rows, d = 4096, 110 us against 100: with four row tiles the 512 smaller workgroups,
// two per CU, keep more requests in flight)
int small_tile_blocks(int R, int nrt, int nCU) { return (R % 64 == 0 && (R / 32) * nrt > nCU && nrt >= 6) ? 2 : 1; }

// out[ks][M][R] = partial sums of W [R][Kc] (packed) times the activation planes; returns the number
// of k splits written (1 for the tiled kernel) or -1 after a launch error (*err set).
int gemm_partial(mrp_ctx *c, hipStream_t st, const void *Wp, int R, int Kc, const uint4 *act, long plane_stride,
                 int nplanes, int M, float *out, size_t out_floats, hipError_t *err) {
    if (c->use_tiled && body_on_tiles(M, Kc) && R % 256 == 0) {
        TiledGemmArgs tg;
        memset(&tg, 0, sizeof(tg));
        tg.Wp = static_cast<const uint4 *>(Wp);
        tg.KBw = Kc / 16; tg.n_rb = R / 32; tg.nIb = c->nIb; tg.M = M; tg.R = R;
        tg.seg[0] = TiledSeg{act, plane_stride, Kc / 64, nplanes};
        tg.nseg = 1;
        tg.nMt = (M + 255) / 256; tg.nVt = R / 256;
        tg.nKs = tiled_ksplit(tg.nMt * tg.nVt, (Kc / 64) * nplanes, c->nCU, out_floats / (size_t)R, M);
        tg.out = out;
        *err = launch_tiled_gemm(tg, EPI_PARTIAL, st);
        return *err == hipSuccess ? tg.nKs : -1;
    }
    if (small_rows_kernel(M, Kc) && M > 64 && R % 64 == 0 && nplanes <= 2) {
        // 65 .. 512 rows: 64-feature x 128-row tiles with k split over workgroups
        const int nrg = (M + 127) / 128;
        // 128-feature tiles halve the activation bytes a CU pulls in per output; they pay once there are enough of
        // them (measured at 128 rows, d = 2048: the 12288-feature gate/up projection, 96 tiles, 26.5 -> 24 us; with 32
        // or 16 tiles, the qkv and o / down projections, the step is 2 - 5 % slower)
        const int nf = (R % 128 == 0 && (R / 128) * nrg >= 96) ? 4 : 2;
        const int nft = R / (32 * nf);
        const int ks = wide_gemm_ksplit(nft * nrg, Kc / 16, c->nCU, out_floats / (size_t)R, M, nf);
        if (ks > 0) {
            WideGemmArgs wg;
            wg.Wp = static_cast<const uint4 *>(Wp); wg.X = act; wg.plane = plane_stride; wg.nplanes = nplanes;
            wg.out = out; wg.nIb = c->nIb; wg.M = M; wg.R = R; wg.Kc = Kc; wg.nKs = ks; wg.nft = nft; wg.nrg = nrg;
            wg.nf = nf;
            *err = launch_wide_gemm(wg, st);
            return *err == hipSuccess ? ks : -1;
        }
    }
    if (small_rows_kernel(M, Kc) && R % 32 == 0 && Kc % 128 == 0 && nplanes <= 2) {
        SmallGemmArgs sg;
        sg.Wp = static_cast<const uint4 *>(Wp); sg.X = act; sg.plane = plane_stride; sg.nplanes = nplanes;
        sg.out = out; sg.nIb = c->nIb; sg.M = M; sg.R = R; sg.Kc = Kc;
        sg.nrt = (M + 31) / 32;
        sg.nf = small_tile_blocks(R, sg.nrt, c->nCU);
        sg.nct = R / (32 * sg.nf);
        *err = launch_small_gemm(sg, st);
        return *err == hipSuccess ? 1 : -1;
    }
    const int IT = stream_gemm_it(M);
    StreamGemmArgs g;
    memset(&g, 0, sizeof(g));
    g.Wp = static_cast<const uint4 *>(Wp);
    g.KBw = Kc / 16; g.n_rb = R / 32; g.nIb = c->nIb; g.M = M; g.R = R;
    g.seg[0] = ActSeg{act, plane_stride, Kc / (16 * KSTEP), nplanes};
    g.nseg = 1;
    g.nVt = R / WG_ROWS; g.nMg = ((M + 31) / 32 + IT - 1) / IT; g.G = Kc / (16 * KSTEP);
    g.nKs = pick_ksplit(g.nVt, g.nMg, g.G, out_floats / (size_t)R, M);
    g.out = out;
    *err = launch_stream_gemm(g, EPI_PARTIAL, st);
    return *err == hipSuccess ? g.nKs : -1;
}

}  // namespace

extern "C" {

size_t mrp_workspace_bytes(const mrp_dims *dims) {
    if (!dims_ok(dims)) return 0;
    int dev = 0, nCU = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&nCU, hipDeviceAttributeMultiprocessorCount, dev);
    return make_layout(dims, nCU > 0 ? nCU : 256).total;
}

int mrp_create(mrp_ctx **out, const mrp_dims *dims) {
    if (!out || !dims) return MRP_ERR_NULL;
    *out = nullptr;
    if (!dims_ok(dims)) return MRP_ERR_SHAPE;
    mrp_ctx *c = new mrp_ctx();
    c->dims = *dims;
    c->err[0] = 0;
    c->prof_on = false;
    c->ev_used = 0;
    c->tb_on = false;
    c->tb_ws = nullptr;
    c->lm_persist = true;
    c->use_tiled = true;
    if (hipGetDevice(&c->device) != hipSuccess ||
        hipDeviceGetAttribute(&c->nCU, hipDeviceAttributeMultiprocessorCount, c->device) != hipSuccess || c->nCU < 1) {
        delete c;
        return MRP_ERR_HIP;
    }
    const Layout l = make_layout(dims, c->nCU);
    c->nIb = l.nIb; c->plane = l.plane; c->nT_max = l.nT_max; c->part_rows = l.part_rows; c->maxB = l.maxB;
    c->ws_bytes = l.total;
    (void)verify_static_scratch();   // resolve this device's scratch address of mrp_verify_accept_static now
    if (stream_gemm_configure() != hipSuccess || lm_persist_configure() != hipSuccess) {
        delete c;
        return MRP_ERR_HIP;
    }
    c->ws = nullptr;
    if (hipMalloc(reinterpret_cast<void **>(&c->ws), l.total) != hipSuccess ||
        hipMemset(c->ws, 0, l.total) != hipSuccess || hipDeviceSynchronize() != hipSuccess) {
        if (c->ws) (void)hipFree(c->ws);
        delete c;
        return MRP_ERR_HIP;
    }
    c->XH = reinterpret_cast<uint4 *>(c->ws + l.off_XH);
    c->XE = reinterpret_cast<uint4 *>(c->ws + l.off_XE);
    c->S = reinterpret_cast<uint4 *>(c->ws + l.off_S);
    c->Y = reinterpret_cast<uint4 *>(c->ws + l.off_Y);
    c->PART = reinterpret_cast<float *>(c->ws + l.off_PART);
    c->pm = reinterpret_cast<float *>(c->ws + l.off_pm);
    c->ps = reinterpret_cast<float *>(c->ws + l.off_ps);
    c->pi = reinterpret_cast<int *>(c->ws + l.off_pi);
    c->vwm = reinterpret_cast<float *>(c->ws + l.off_vwm);
    c->vwi = reinterpret_cast<int *>(c->ws + l.off_vwi);
    c->kl_part = reinterpret_cast<float *>(c->ws + l.off_klp);
    c->kl_lse = reinterpret_cast<float *>(c->ws + l.off_kll);
    c->kl_stride = l.kl_stride;
    c->rms_part = reinterpret_cast<double *>(c->ws + l.off_rms);
    c->err_flag = reinterpret_cast<int *>(c->ws + l.off_err);
    *out = c;
    return MRP_OK;
}

int mrp_destroy(mrp_ctx *c) {
    if (!c) return MRP_ERR_NULL;
    for (hipEvent_t e : c->ev) (void)hipEventDestroy(e);
    (void)hipFree(c->ws);
    if (c->tb_ws) (void)hipFree(c->tb_ws);
    delete c;
    return MRP_OK;
}

const char *mrp_last_error(const mrp_ctx *c) { return c ? c->err : "null context"; }

size_t mrp_packed_bytes(int rows, int cols) {
    if (rows < 1 || cols < 16 || cols % 16) return 0;
    return ((size_t)rows + 31) / 32 * 32 * (size_t)cols * 2;
}

static int pack_impl(void *stream, const void *src, int rows, int cols, void *dst, bool to_f16) {
    if (!src || !dst) return MRP_ERR_NULL;
    if (rows < 1 || cols < 16 || cols % 16) return MRP_ERR_SHAPE;
    if (!aligned16(src) || !aligned16(dst)) return MRP_ERR_ALIGN;
    hipError_t e = launch_pack_weight(static_cast<const uint16_t *>(src), rows, cols, static_cast<uint4 *>(dst), to_f16,
                                      static_cast<hipStream_t>(stream));
    return e == hipSuccess ? MRP_OK : MRP_ERR_HIP;
}

int mrp_pack_weight(void *stream, const void *src, int rows, int cols, void *dst) {
    return pack_impl(stream, src, rows, cols, dst, false);
}

int mrp_pack_body_weight(void *stream, const void *src, int rows, int cols, void *dst) {
    return pack_impl(stream, src, rows, cols, dst, true);
}

int mrp_kl_loss(mrp_ctx *c, void *stream, int M, const float *teacher, const float *student, const uint8_t *row_mask,
                float scale, float *loss_rows, float *grad) {
    if (!c) return MRP_ERR_NULL;
    if (!teacher || !student || !loss_rows) return fail(c, MRP_ERR_NULL, "mrp_kl_loss: NULL pointer");
    if (M < 0 || M > c->dims.max_rows) return fail(c, MRP_ERR_WORKSPACE, "mrp_kl_loss: M=%d exceeds max_rows", M);
    if (c->dims.V % 4 == 0 && (!aligned16(teacher) || !aligned16(student) || (grad && !aligned16(grad))))
        return fail(c, MRP_ERR_ALIGN, "mrp_kl_loss: tensors must be 16-byte aligned");
    if (M == 0) return MRP_OK;
    HIP_TRY(c, launch_kl_loss(M, c->dims.V, teacher, student, row_mask, scale, c->kl_part, c->kl_stride, c->kl_lse,
                              loss_rows, grad, static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

int mrp_residual_rms(mrp_ctx *c, void *stream, int n_blocks, int S, long N, const void *X, int dtype,
                     double *rms_pair, double *rms_delta) {
    if (!c) return MRP_ERR_NULL;
    if (!X || !rms_pair || !rms_delta) return fail(c, MRP_ERR_NULL, "mrp_residual_rms: NULL pointer");
    if (!residual_rms_supported(S))
        return fail(c, MRP_ERR_SHAPE, "mrp_residual_rms: S=%d states (block + 1) must be 3, 5, 9 or 17", S);
    if (dtype != MRP_DTYPE_F32 && dtype != MRP_DTYPE_BF16)
        return fail(c, MRP_ERR_SHAPE, "mrp_residual_rms: dtype %d is neither fp32 nor bf16", dtype);
    if (n_blocks < 0 || N < 1 || n_blocks > residual_rms_max_blocks())
        return fail(c, MRP_ERR_SHAPE, "mrp_residual_rms: n_blocks=%d (max %d), N=%ld", n_blocks,
                    residual_rms_max_blocks(), N);
    if ((reinterpret_cast<uintptr_t>(X) & (dtype == MRP_DTYPE_F32 ? 3u : 1u)) ||
        (reinterpret_cast<uintptr_t>(rms_pair) & 7u) || (reinterpret_cast<uintptr_t>(rms_delta) & 7u))
        return fail(c, MRP_ERR_ALIGN, "mrp_residual_rms: pointers must be aligned to their element size");
    if (n_blocks == 0) return MRP_OK;
    HIP_TRY(c, launch_residual_rms(n_blocks, S, N, X, dtype == MRP_DTYPE_BF16, c->rms_part, rms_pair, rms_delta,
                                   static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

int mrp_tbody_create(mrp_ctx *c, const mrp_tbody_dims *t) {
    if (!c || !t) return MRP_ERR_NULL;
    if (c->tb_on) return fail(c, MRP_ERR_SHAPE, "mrp_tbody_create: already configured");
    const int L = c->dims.block_len, d = c->dims.d;
    if (t->D < 1 || t->D > MRP_MAX_TLAYERS || !tbody_shape_ok(t->n_heads, t->n_kv_heads, t->head_dim, L))
        return fail(c, MRP_ERR_SHAPE,
                    "mrp_tbody_create: need 1 <= D <= %d, head_dim 128, n_heads a multiple of n_kv_heads, block_len <= 16 "
                    "and (n_heads / n_kv_heads) * block_len <= 64",
                    MRP_MAX_TLAYERS);
    if (t->d_ff < 128 || t->d_ff % 128 || t->d_ff > 65536 || t->max_prefix < 0 || !(t->rope_theta > 1.f))
        return fail(c, MRP_ERR_SHAPE, "mrp_tbody_create: d_ff must be a multiple of 128, max_prefix >= 0, rope_theta > 1");
    if (tbody_configure() != hipSuccess) return fail(c, MRP_ERR_HIP, "mrp_tbody_create: kernel attributes");
    const int qd = t->n_heads * t->head_dim, qkvd = qd + 2 * t->n_kv_heads * t->head_dim;
    int cmax = d > qd ? d : qd;
    if (t->d_ff > cmax) cmax = t->d_ff;
    int rmax = qkvd > 2 * t->d_ff ? qkvd : 2 * t->d_ff;
    if (d > rmax) rmax = d;
    c->tb_plane = (long)(cmax / 16) * c->nIb * 64;
    c->tb_part_floats = c->part_rows * (size_t)rmax;
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t r = o; o = align_up(o + bytes, 256); return r; };
    const size_t off_U = take((size_t)c->dims.max_rows * d * sizeof(float));
    const size_t off_P = take((size_t)NSPLIT * c->tb_plane * 16);
    const size_t off_part = take(c->tb_part_floats * sizeof(float));
    const size_t off_rope = take((size_t)c->dims.max_rows * 64 * sizeof(float2));
    const size_t off_attn = take(attention_scratch_floats() * sizeof(float));
    if (hipMalloc(reinterpret_cast<void **>(&c->tb_ws), o) != hipSuccess || hipMemset(c->tb_ws, 0, o) != hipSuccess ||
        hipDeviceSynchronize() != hipSuccess) {
        if (c->tb_ws) (void)hipFree(c->tb_ws);
        c->tb_ws = nullptr;
        return fail(c, MRP_ERR_HIP, "mrp_tbody_create: allocating %zu bytes failed", o);
    }
    c->tb_U = reinterpret_cast<float *>(c->tb_ws + off_U);
    c->tb_P = reinterpret_cast<uint4 *>(c->tb_ws + off_P);
    c->tb_part = reinterpret_cast<float *>(c->tb_ws + off_part);
    c->tb_rope = reinterpret_cast<float2 *>(c->tb_ws + off_rope);
    c->tb_attn = reinterpret_cast<float *>(c->tb_ws + off_attn);
    c->tb = *t;
    c->tb_on = true;
    return MRP_OK;
}

int mrp_profile_enable(mrp_ctx *c, int on) {
    if (!c) return MRP_ERR_NULL;
    if (on && c->ev.empty()) {
        c->ev.resize(2 * PROF_PAIRS);
        for (auto &e : c->ev) HIP_TRY(c, hipEventCreate(&e));
    }
    c->prof_on = on != 0;
    c->ev_used = 0;
    return MRP_OK;
}

int mrp_profile_read(mrp_ctx *c, float *ms_out, int cap) {
    if (!c || !ms_out) return MRP_ERR_NULL;
    int n = 0;
    for (int p = 0; p < c->ev_used && n < cap; ++p) {
        HIP_TRY(c, hipEventSynchronize(c->ev[2 * p + 1]));
        HIP_TRY(c, hipEventElapsedTime(&ms_out[n], c->ev[2 * p], c->ev[2 * p + 1]));
        ++n;
    }
    c->ev_used = 0;
    return n;
}

}  // extern "C"

// layers == nullptr: MLP head body; else head k's transformer layers are layers[(k - 1) * D ..]
static int chain_impl(mrp_ctx *c, void *stream, int B, int K, const void *h, float *h_run, const void *E,
                      const void *W_lm_packed, const mrp_head *heads, const mrp_tlayer *layers,
                      const int32_t *prefix_len, float *z, const mrp_reveal_cfg *cfg, const mrp_step_io *io) {
    if (!c) return MRP_ERR_NULL;
    if (!h_run || !E || !W_lm_packed || !z || !cfg || !io || (K > 0 && !heads))
        return fail(c, MRP_ERR_NULL, "mrp_chain_step: required pointer is NULL");
    if (!io->tok || !io->conf || !io->lse || !io->revealed_at || !io->masked || !io->cond_tok ||
        !io->protect_pos || !io->draft_pos || !io->draft_tok)
        return fail(c, MRP_ERR_NULL, "mrp_chain_step: required mrp_step_io pointer is NULL");
    const int L = c->dims.block_len, d = c->dims.d, V = c->dims.V;
    if (B < 0 || K < 0 || K > MRP_MAX_HEADS) return fail(c, MRP_ERR_SHAPE, "B=%d K=%d out of range", B, K);
    if (cfg->r_min < 0 || cfg->state_offset < 0 || cfg->state_offset + K > 120 || !(cfg->tau == cfg->tau) ||
        cfg->remask_mode < 0 || cfg->remask_mode > 1)
        return fail(c, MRP_ERR_SHAPE, "bad reveal configuration");
    if (cfg->remask_mode == 1 && cfg->tau_remask >= 0.f && !io->x_tok)
        return fail(c, MRP_ERR_NULL, "remask_mode 1 needs mrp_step_io.x_tok");
    const long Ml = (long)B * L;
    if (Ml > c->dims.max_rows) return fail(c, MRP_ERR_WORKSPACE, "rows %ld exceed max_rows %d", Ml, c->dims.max_rows);
    for (int k = 0; k < K; ++k) {
        if (!heads[k].W1_packed || (!layers && !heads[k].W2_packed) || !heads[k].gamma)
            return fail(c, MRP_ERR_NULL, "head %d has a NULL weight", k);
        if (!aligned16(heads[k].W1_packed) || (!layers && !aligned16(heads[k].W2_packed)) || !aligned16(heads[k].gamma))
            return fail(c, MRP_ERR_ALIGN, "head %d weights must be 16-byte aligned", k);
    }
    if (layers) {
        if (!c->tb_on) return fail(c, MRP_ERR_WORKSPACE, "transformer body: call mrp_tbody_create first");
        if (!prefix_len) return fail(c, MRP_ERR_NULL, "transformer body: prefix_len is NULL");
        for (int n = 0; n < K * c->tb.D; ++n) {
            const mrp_tlayer &l = layers[n];
            const void *ptrs[8] = {l.Wqkv_packed, l.Wo_packed, l.Wgu_packed, l.Wdown_packed, l.g1, l.g2, l.k_cache, l.v_cache};
            for (int q = 0; q < 8; ++q) {
                if (!ptrs[q] && !(q >= 6 && c->tb.max_prefix == 0))
                    return fail(c, MRP_ERR_NULL, "transformer layer %d has a NULL pointer", n);
                if (!aligned16(ptrs[q])) return fail(c, MRP_ERR_ALIGN, "transformer layer %d: pointers must be 16-byte aligned", n);
            }
        }
    }
    if ((h && !aligned16(h)) || !aligned16(h_run) || !aligned16(E) || !aligned16(W_lm_packed) || !aligned16(z))
        return fail(c, MRP_ERR_ALIGN, "tensor base pointers must be 16-byte aligned");
    if (B == 0) return MRP_OK;

    const int M = (int)Ml;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const uint16_t *Eb = static_cast<const uint16_t *>(E);
    const int IT = stream_gemm_it(M);
    const int nMg = ((M + 31) / 32 + IT - 1) / IT;
    const int off = cfg->state_offset;
    // MLP body at small row counts: the first GEMM also reads the conditioning embeddings from the table
    // itself (no gathered copy is made) and applies the SiLU
    const bool fused = !layers && d % 128 == 0 && small_rows_kernel(M, d);

    SelectArgs sa;
    memset(&sa, 0, sizeof(sa));
    sa.pm = c->pm; sa.ps = c->ps; sa.pi = c->pi;
    sa.M = M; sa.B = B; sa.L = L; sa.d = d; sa.V = V;
    sa.tau = cfg->tau; sa.r_min = cfg->r_min; sa.max_accept = cfg->max_accept;
    sa.revealed_at = io->revealed_at; sa.masked = io->masked;
    sa.cond_tok = io->cond_tok; sa.protect_pos = io->protect_pos;
    sa.draft_stride = K + 1;
    sa.xe = c->XE; sa.nIb = c->nIb;
    sa.x_tok = io->x_tok; sa.remask_mode = cfg->remask_mode; sa.z = z;
    sa.err_flag = c->err_flag;

    if (cfg->run_state0) {
        int nT0 = 0;
        HIP_TRY(c, launch_reduce_rows(z, M, V, c->pm, c->ps, c->pi, &nT0, st));
        sa.nT = nT0;
        sa.slot_stride = 1; sa.row_stride = nT0;
        sa.state = off; sa.do_reveal = 1; sa.fresh = cfg->fresh_block; sa.write_protect = 1;
        sa.tau_remask = -1.f;
        sa.tok = io->tok; sa.conf = io->conf; sa.lse = io->lse;
        sa.draft_pos = io->draft_pos; sa.draft_tok = io->draft_tok;
        sa.remasked = io->remasked;
        sa.E = (K > 0 && !fused) ? Eb : nullptr;
        HIP_TRY(c, launch_merge_select(sa, st));
    } else if (K > 0 && !fused) {
        HIP_TRY(c, launch_gather_e(Eb, io->cond_tok, c->XE, c->nIb, B, L, d, V, c->err_flag, st));
    }
    if (K == 0) return MRP_OK;

    HIP_TRY(c, launch_init_hidden(static_cast<const uint16_t *>(h), h_run, c->XH, c->plane, c->nIb, M, d,
                                  h != nullptr, st));
    int np_h = h ? 1 : NSPLIT;
    const int nkr_d = d / (16 * KSTEP);

    for (int k = 1; k <= K; ++k) {
        const mrp_head &hd = heads[k - 1];
        StreamGemmArgs g;
        // The LM head has V / 256 tiles per 256 rows and takes the tile kernel beyond 512 rows (measured at
        // d = 4096, V = 151936: 931 / 955 / 1031 / 1074 us at 272 / 512 / 752 / 768 rows); below, the persistent
        // kernel in launches of at most 256 rows is ahead (see there).  The streaming kernel is left with
        // vocabularies that are not a multiple of 4.
        const bool tiled = c->use_tiled && body_on_tiles(M, d);
        const bool tiled_lm = c->use_tiled && M > 512;
        int nks1 = 1, nks2 = 1;
        bool silu_done = false;   // the first GEMM's epilogue already wrote s = SiLU(a) as activation planes
        const float *resid = nullptr;   // transformer body: residual stream added to the last projection
        if (fused) {
            // s = SiLU(W1 [h ; e]) with e read from the embedding table, then u = W2 s
            HeadFusedArgs fa;
            memset(&fa, 0, sizeof(fa));
            fa.W1p = static_cast<const uint4 *>(hd.W1_packed);
            fa.W2p = static_cast<const uint4 *>(hd.W2_packed);
            fa.XH = c->XH; fa.plane = c->plane; fa.np_h = np_h;
            fa.E = Eb; fa.cond_tok = io->cond_tok; fa.L = L; fa.V = V;
            fa.S = c->S; fa.U = c->PART;
            fa.nIb = c->nIb; fa.M = M; fa.d = d;
            fa.err_flag = c->err_flag;
            fa.nrt = (M + 31) / 32;
            fa.nf = small_tile_blocks(d, fa.nrt, c->nCU);
            fa.nct = d / (32 * fa.nf);
            HIP_TRY(c, launch_head_fused(fa, st));
        } else {
        // a = W1 [h_run ; e]
        if (tiled) {
            TiledGemmArgs tg;
            memset(&tg, 0, sizeof(tg));
            tg.Wp = static_cast<const uint4 *>(hd.W1_packed);
            tg.KBw = 2 * d / 16; tg.n_rb = d / 32; tg.nIb = c->nIb; tg.M = M; tg.R = d;
            tg.seg[0] = TiledSeg{c->XH, c->plane, d / 64, np_h};
            tg.seg[1] = TiledSeg{c->XE, 0, d / 64, 1};
            tg.nseg = 2;
            tg.nMt = (M + 255) / 256; tg.nVt = (d + 255) / 256;
            tg.nKs = tiled_ksplit(tg.nMt * tg.nVt, (d / 64) * (np_h + 1), c->nCU, c->part_rows, M);
            nks1 = tg.nKs;
            tg.out = c->PART;
            // a single k part of the MLP body: SiLU and the fp16 split sit in the tile epilogue
            silu_done = !layers && tg.nKs == 1;
            tg.planes = c->S; tg.plane_stride = c->plane;
            HIP_TRY(c, launch_tiled_gemm(tg, silu_done ? EPI_SILU : EPI_PARTIAL, st));
        } else {
            memset(&g, 0, sizeof(g));
            g.Wp = static_cast<const uint4 *>(hd.W1_packed);
            g.KBw = 2 * d / 16; g.n_rb = d / 32; g.nIb = c->nIb; g.M = M; g.R = d;
            g.seg[0] = ActSeg{c->XH, c->plane, nkr_d, np_h};
            g.seg[1] = ActSeg{c->XE, 0, nkr_d, 1};
            g.nseg = 2;
            g.nVt = d / WG_ROWS; g.nMg = nMg; g.G = 2 * nkr_d;
            g.nKs = pick_ksplit(g.nVt, nMg, g.G, c->part_rows, M);
            g.out = c->PART;
            nks1 = g.nKs;
            HIP_TRY(c, launch_stream_gemm(g, EPI_PARTIAL, st));
        }
        if (layers) {
            const mrp_tbody_dims &tb = c->tb;
            const int qd = tb.n_heads * tb.head_dim, qkvd = qd + 2 * tb.n_kv_heads * tb.head_dim, ff = tb.d_ff;
            const size_t part_d = c->part_rows * (size_t)d;
            hipError_t ge = hipSuccess;
            if (k == 1)
                HIP_TRY(c, launch_rope_table(prefix_len, B, L, tb.max_prefix, (double)tb.rope_theta, c->tb_rope,
                                             c->err_flag, st));
            // u_0 = fuse projection; planes <- RMSNorm(u_0) g1 of layer 0
            int nks = nks1;
            for (int l = 0; l < tb.D; ++l) {
                const mrp_tlayer &ly = layers[(size_t)(k - 1) * tb.D + l];
                HIP_TRY(c, launch_resid_norm_split(c->PART, nks, l == 0 ? nullptr : c->tb_U, c->tb_U,
                                                   static_cast<const uint16_t *>(ly.g1), c->dims.rms_eps, c->tb_P,
                                                   c->tb_plane, c->nIb, M, d, st));
                nks = gemm_partial(c, st, ly.Wqkv_packed, qkvd, d, c->tb_P, c->tb_plane, NSPLIT, M, c->tb_part,
                                   c->tb_part_floats, &ge);
                HIP_TRY(c, ge);
                HIP_TRY(c, launch_attention(c->tb_part, nks, M, B, L, tb.n_heads, tb.n_kv_heads, c->tb_rope,
                                            static_cast<const uint16_t *>(ly.k_cache),
                                            static_cast<const uint16_t *>(ly.v_cache), prefix_len, tb.max_prefix,
                                            c->tb_P, c->tb_plane, c->nIb, c->tb_attn, st));
                nks = gemm_partial(c, st, ly.Wo_packed, d, qd, c->tb_P, c->tb_plane, NSPLIT, M, c->PART, part_d, &ge);
                HIP_TRY(c, ge);
                // a = u + Wo o; planes <- RMSNorm(a) g2
                HIP_TRY(c, launch_resid_norm_split(c->PART, nks, c->tb_U, c->tb_U, static_cast<const uint16_t *>(ly.g2),
                                                   c->dims.rms_eps, c->tb_P, c->tb_plane, c->nIb, M, d, st));
                nks = gemm_partial(c, st, ly.Wgu_packed, 2 * ff, d, c->tb_P, c->tb_plane, NSPLIT, M, c->tb_part,
                                   c->tb_part_floats, &ge);
                HIP_TRY(c, ge);
                HIP_TRY(c, launch_swiglu_split(c->tb_part, nks, c->tb_P, c->tb_plane, c->nIb, M, ff, st));
                nks = gemm_partial(c, st, ly.Wdown_packed, d, ff, c->tb_P, c->tb_plane, NSPLIT, M, c->PART, part_d, &ge);
                HIP_TRY(c, ge);
                // u' = a + (down projection): folded into the next layer's norm or into the final norm below
            }
            nks2 = nks;
            resid = c->tb_U;
        } else {
        if (!silu_done) HIP_TRY(c, launch_silu_split(c->PART, nks1, c->S, c->plane, c->nIb, M, d, st));
        // u = W2 s
        if (tiled) {
            TiledGemmArgs tg;
            memset(&tg, 0, sizeof(tg));
            tg.Wp = static_cast<const uint4 *>(hd.W2_packed);
            tg.KBw = d / 16; tg.n_rb = d / 32; tg.nIb = c->nIb; tg.M = M; tg.R = d;
            tg.seg[0] = TiledSeg{c->S, c->plane, d / 64, NSPLIT};
            tg.nseg = 1;
            tg.nMt = (M + 255) / 256; tg.nVt = (d + 255) / 256;
            tg.nKs = tiled_ksplit(tg.nMt * tg.nVt, (d / 64) * NSPLIT, c->nCU, c->part_rows, M);
            nks2 = tg.nKs;
            tg.out = c->PART;
            HIP_TRY(c, launch_tiled_gemm(tg, EPI_PARTIAL, st));
        } else {
            memset(&g, 0, sizeof(g));
            g.Wp = static_cast<const uint4 *>(hd.W2_packed);
            g.KBw = d / 16; g.n_rb = d / 32; g.nIb = c->nIb; g.M = M; g.R = d;
            g.seg[0] = ActSeg{c->S, c->plane, nkr_d, NSPLIT};
            g.nseg = 1;
            g.nVt = d / WG_ROWS; g.nMg = nMg; g.G = nkr_d;
            g.nKs = pick_ksplit(g.nVt, nMg, g.G, c->part_rows, M);
            g.out = c->PART;
            nks2 = g.nKs;
            HIP_TRY(c, launch_stream_gemm(g, EPI_PARTIAL, st));
        }
        }
        }
        // h_run += u ; y = bf16(RMSNorm(u) * gamma)
        HIP_TRY(c, launch_norm(c->PART, nks2, resid, static_cast<const uint16_t *>(hd.gamma), c->dims.rms_eps, h_run,
                               cfg->carry_hidden != 0, c->Y, c->XH, c->plane, c->nIb, M, d, st));
        if (cfg->carry_hidden) np_h = NSPLIT;
        // z += W_lm y, fused with the split-vocabulary (max, sum-exp, argmax) partials
        const bool prof = c->prof_on && c->ev_used < PROF_PAIRS;
        if (prof) HIP_TRY(c, hipEventRecord(c->ev[2 * c->ev_used], st));
        int nT_lm = 0;
        bool lm_rowmajor = false;  // partial layout [M][nT] (persistent kernel) or [nT][M]
        if (c->lm_persist && M <= 512 && V % 4 == 0) {
            // up to 256 rows per launch; a second launch for the rows beyond streams W_lm again, which up to
            // 512 rows is still cheaper than the tile kernel (measured at d = 4096: 392 us for 256 rows,
            // 281 us for 128, against 931-955 us for the tile kernel at 272-512 rows)
            int chunk = 0;
            for (int row0 = 0; row0 < M; row0 += 256, ++chunk) {
                LmPersistArgs la;
                memset(&la, 0, sizeof(la));
                la.Wp = static_cast<const uint4 *>(W_lm_packed);
                la.Y = c->Y + (size_t)(row0 / 32) * 64;      // (planes are [k block][row block][lane])
                la.KB = d / 16; la.n_rb = (V + 31) / 32; la.nIb = c->nIb;
                la.M = M - row0 < 256 ? M - row0 : 256; la.V = V;
                la.nWG = c->nCU;
                // consecutive launches walk the vocabulary in opposite directions: what the previous one
                // touched last (W_lm is shared by all heads) is still in the L2s when this one starts
                la.reverse = (off + k + chunk) & 1;
                la.z = z + (size_t)row0 * V;
                la.pm = c->pm + (size_t)row0 * la.nWG; la.ps = c->ps + (size_t)row0 * la.nWG;
                la.pi = c->pi + (size_t)row0 * la.nWG;
                HIP_TRY(c, launch_lm_persist(la, st));
            }
            nT_lm = c->nCU;
            lm_rowmajor = true;
        } else if (tiled_lm && V % 4 == 0) {
            TiledGemmArgs tg;
            memset(&tg, 0, sizeof(tg));
            tg.Wp = static_cast<const uint4 *>(W_lm_packed);
            tg.KBw = d / 16; tg.n_rb = (V + 31) / 32; tg.nIb = c->nIb; tg.M = M; tg.R = V;
            tg.seg[0] = TiledSeg{c->Y, 0, d / 64, 1};
            tg.nseg = 1;
            tg.nMt = (M + 255) / 256; tg.nVt = (V + 255) / 256;
            tg.nKs = 1;
            tg.z = z; tg.pm = c->pm; tg.ps = c->ps; tg.pi = c->pi;
            HIP_TRY(c, launch_tiled_gemm(tg, EPI_LM, st));
            nT_lm = tg.nVt;
        } else {
            memset(&g, 0, sizeof(g));
            g.Wp = static_cast<const uint4 *>(W_lm_packed);
            g.KBw = d / 16; g.n_rb = (V + 31) / 32; g.nIb = c->nIb; g.M = M; g.R = V;
            g.seg[0] = ActSeg{c->Y, 0, nkr_d, 1};
            g.nseg = 1;
            g.nVt = (g.n_rb + WG_WAVES - 1) / WG_WAVES; g.nMg = nMg; g.nKs = 1; g.G = nkr_d;
            g.z = z; g.pm = c->pm; g.ps = c->ps; g.pi = c->pi;
            HIP_TRY(c, launch_stream_gemm(g, EPI_LM, st));
            nT_lm = g.nVt;
        }
        if (prof) {
            HIP_TRY(c, hipEventRecord(c->ev[2 * c->ev_used + 1], st));
            ++c->ev_used;
        }
        // merge partials, reveal / draft / remask, gather the next conditioning embedding
        sa.nT = nT_lm;
        sa.slot_stride = lm_rowmajor ? 1 : M;
        sa.row_stride = lm_rowmajor ? nT_lm : 1;
        sa.state = off + k; sa.do_reveal = cfg->head_reveal; sa.fresh = 0; sa.write_protect = 0;
        sa.tau_remask = cfg->tau_remask;
        sa.tok = io->tok + (size_t)k * M; sa.conf = io->conf + (size_t)k * M; sa.lse = io->lse + (size_t)k * M;
        sa.draft_pos = io->draft_pos + k; sa.draft_tok = io->draft_tok + k;
        sa.remasked = io->remasked ? io->remasked + (size_t)k * M : nullptr;
        sa.E = (k < K && !fused) ? Eb : nullptr;
        HIP_TRY(c, launch_merge_select(sa, st));
    }
    return MRP_OK;
}

extern "C" {

int mrp_chain_step(mrp_ctx *c, void *stream, int B, int K, const void *h, float *h_run, const void *E,
                   const void *W_lm_packed, const mrp_head *heads, float *z, const mrp_reveal_cfg *cfg,
                   const mrp_step_io *io) {
    return chain_impl(c, stream, B, K, h, h_run, E, W_lm_packed, heads, nullptr, nullptr, z, cfg, io);
}

int mrp_chain_step_tf(mrp_ctx *c, void *stream, int B, int K, const void *h, float *h_run, const void *E,
                      const void *W_lm_packed, const mrp_head *heads, const mrp_tlayer *layers,
                      const int32_t *prefix_len, float *z, const mrp_reveal_cfg *cfg, const mrp_step_io *io) {
    if (!c) return MRP_ERR_NULL;
    if (K > 0 && !layers) return fail(c, MRP_ERR_NULL, "mrp_chain_step_tf: layers is NULL");
    return chain_impl(c, stream, B, K, h, h_run, E, W_lm_packed, heads, K > 0 ? layers : nullptr, prefix_len, z, cfg, io);
}

int mrp_remask(mrp_ctx *c, void *stream, int B, int state, const float *conf_new, float tau_remask,
               const int32_t *protect_pos, int8_t *revealed_at, uint8_t *masked, uint8_t *remasked_out) {
    if (!c) return MRP_ERR_NULL;
    if (!conf_new || !revealed_at || !masked || !remasked_out) return fail(c, MRP_ERR_NULL, "mrp_remask: NULL pointer");
    if (B < 0 || (long)B * c->dims.block_len > c->dims.max_rows || state < 0 || state > 126)
        return fail(c, MRP_ERR_SHAPE, "mrp_remask: B=%d state=%d out of range", B, state);
    if (B == 0) return MRP_OK;
    HIP_TRY(c, launch_remask(B, c->dims.block_len, state, conf_new, tau_remask, protect_pos, revealed_at, masked,
                             remasked_out, static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

int mrp_commit(mrp_ctx *c, void *stream, int B, const int32_t *x_tok, int8_t *revealed_at, const uint8_t *masked,
               int32_t *x_out, int32_t *n_masked) {
    if (!c) return MRP_ERR_NULL;
    if (!x_tok || !revealed_at || !masked || !x_out || !n_masked) return fail(c, MRP_ERR_NULL, "mrp_commit: NULL pointer");
    if (B < 0 || (long)B * c->dims.block_len > c->dims.max_rows)
        return fail(c, MRP_ERR_SHAPE, "mrp_commit: B=%d out of range", B);
    if (B == 0) return MRP_OK;
    HIP_TRY(c, launch_commit(B, c->dims.block_len, x_tok, revealed_at, masked, x_out, n_masked,
                             static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

static int verify_impl(mrp_ctx *c, void *stream, int B, int K, int joint, const float *verify, const int32_t *draft_pos,
                      const int32_t *draft_tok, int draft_stride, uint8_t *match, int32_t *accept_len,
                      int32_t *correction_tok) {
    if (!c) return MRP_ERR_NULL;
    if (!verify || !draft_pos || !draft_tok || !match || !accept_len || !correction_tok)
        return fail(c, MRP_ERR_NULL, "mrp_verify_accept: NULL pointer");
    if (B < 0 || B > c->maxB || K < 1 || K > MRP_MAX_HEADS || draft_stride < K || (long)B * K > 65535)
        return fail(c, MRP_ERR_SHAPE, "mrp_verify_accept: B=%d K=%d stride=%d out of range", B, K, draft_stride);
    if (c->dims.V % 4 == 0 && !aligned16(verify)) return fail(c, MRP_ERR_ALIGN, "verify must be 16-byte aligned");
    if (B == 0) return MRP_OK;
    HIP_TRY(c, launch_verify(B, c->dims.block_len, c->dims.V, K, joint, verify, draft_pos, draft_tok, draft_stride, c->vwm,
                             c->vwi, match, accept_len, correction_tok, c->err_flag, static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

int mrp_verify_accept(mrp_ctx *c, void *stream, int B, int K, const float *verify, const int32_t *draft_pos,
                      const int32_t *draft_tok, int draft_stride, uint8_t *match, int32_t *accept_len,
                      int32_t *correction_tok) {
    return verify_impl(c, stream, B, K, 0, verify, draft_pos, draft_tok, draft_stride, match, accept_len,
                       correction_tok);
}

int mrp_verify_accept_joint(mrp_ctx *c, void *stream, int B, int K, const float *verify, const int32_t *draft_pos,
                            const int32_t *draft_tok, int draft_stride, uint8_t *match, int32_t *accept_len,
                            int32_t *correction_tok) {
    return verify_impl(c, stream, B, K, 1, verify, draft_pos, draft_tok, draft_stride, match, accept_len,
                       correction_tok);
}

int mrp_build_candidates(mrp_ctx *c, void *stream, int B, int K, const int32_t *x_t, const uint8_t *masked_t,
                         const int32_t *draft_pos, const int32_t *draft_tok, int draft_stride, int32_t mask_token,
                         int32_t *cand_tok, uint8_t *cand_masked) {
    if (!c) return MRP_ERR_NULL;
    if (!x_t || !masked_t || !draft_pos || !draft_tok || !cand_tok || !cand_masked)
        return fail(c, MRP_ERR_NULL, "mrp_build_candidates: NULL pointer");
    if (B < 0 || B > c->maxB || K < 0 || K > MRP_MAX_HEADS || draft_stride < K)
        return fail(c, MRP_ERR_SHAPE, "mrp_build_candidates: B=%d K=%d stride=%d out of range", B, K, draft_stride);
    if (B == 0) return MRP_OK;
    HIP_TRY(c, launch_build_candidates(B, c->dims.block_len, K, x_t, masked_t, draft_pos, draft_tok, draft_stride,
                                       mask_token, cand_tok, cand_masked, c->err_flag,
                                       static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

int mrp_poll_error(mrp_ctx *c, void *stream) {
    if (!c) return MRP_ERR_NULL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    int flags = 0;
    HIP_TRY(c, hipStreamSynchronize(st));
    HIP_TRY(c, hipMemcpy(&flags, c->err_flag, sizeof(int), hipMemcpyDeviceToHost));
    if (flags) {
        HIP_TRY(c, hipMemset(c->err_flag, 0, sizeof(int)));
        snprintf(c->err, sizeof(c->err), "device error word 0x%x:%s%s%s%s", (unsigned)flags,
                 (flags & MRP_FLAG_COND_TOK) ? " cond_tok out of range (clamped)" : "",
                 (flags & MRP_FLAG_DRAFT_POS) ? " draft position >= block length (taken as missing)" : "",
                 (flags & MRP_FLAG_PREFIX_LEN) ? " prefix_len outside [0, max_prefix] (clamped)" : "",
                 (flags & MRP_FLAG_X_TOK) ? " recorded token >= V (clamped)" : "");
    }
    return flags;
}

int mrp_probe_lm_traffic(mrp_ctx *c, void *stream, int mode, int M, const void *W_lm_packed, float *z) {
    if (!c) return MRP_ERR_NULL;
    if (!W_lm_packed || (mode >= 1 && !z)) return fail(c, MRP_ERR_NULL, "mrp_probe_lm_traffic: NULL pointer");
    if (mode < 0 || mode > 2 || M < 1 || M > 128 || M > c->dims.max_rows || c->dims.V % 4 != 0 || c->dims.d % 256 != 0)
        return fail(c, MRP_ERR_SHAPE, "mrp_probe_lm_traffic: mode 0..2, 1 <= M <= 128, V %% 4 == 0, d %% 256 == 0");
    if (!aligned16(W_lm_packed) || (z && !aligned16(z))) return fail(c, MRP_ERR_ALIGN, "mrp_probe_lm_traffic: 16-byte alignment");
    HIP_TRY(c, launch_lm_traffic(mode, static_cast<const uint4 *>(W_lm_packed), z, c->dims.d / 16, (c->dims.V + 31) / 32, M,
                                 c->dims.V, c->nCU, reinterpret_cast<unsigned *>(c->err_flag + 8),
                                 static_cast<hipStream_t>(stream)));
    return MRP_OK;
}

}  // extern "C"
