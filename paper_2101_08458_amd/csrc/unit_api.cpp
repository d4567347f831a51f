// C boundary of libunit: argument validation, workspace carving, tile selection and
// kernel dispatch.  Every error path returns before the first HIP call.
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "../../include/unit.h"
#include "unit_internal.h"

namespace unit {
hipError_t launch_igemm_i8(int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);
hipError_t launch_igemm_f16(int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);
hipError_t launch_igemm_bf16(int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);
hipError_t launch_igemm_u8(int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);
hipError_t launch_igemm_fp8(int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st);

// dtype is the public unit_dtype
hipError_t launch_igemm(int dtype, int bsrc, int tile, const IgemmArgs &a, int split_k, hipStream_t st)
{
    switch (dtype) {
    case UNIT_I8:   return launch_igemm_i8(bsrc, tile, a, split_k, st);
    case UNIT_F16:  return launch_igemm_f16(bsrc, tile, a, split_k, st);
    case UNIT_BF16: return launch_igemm_bf16(bsrc, tile, a, split_k, st);
    case UNIT_U8I8: return bsrc == BSRC_NCHW ? hipErrorInvalidValue : launch_igemm_u8(bsrc, tile, a, split_k, st);
    case UNIT_FP8:  return launch_igemm_fp8(bsrc, tile, a, split_k, st);
    default:        return hipErrorInvalidValue;
    }
}
}  // namespace unit

using namespace unit;

namespace {

thread_local char g_hip_err[256] = "";
#ifdef UNIT_PROBE
void *g_probe_ptr = nullptr;        // instrumented build: where the next launches write their time stamps
#endif

// Internal problem description: conv2d is the depth-1 case of conv3d (the only thing that
// changes between them is the address generator of the gather).
struct ConvND {
    int n, c, d, h, w;
    int k, t, r, s;
    int stride_d, stride_h, stride_w, pad_d, pad_h, pad_w;
    ConvND() : n(0), c(0), d(0), h(0), w(0), k(0), t(0), r(0), s(0),
               stride_d(0), stride_h(0), stride_w(0), pad_d(0), pad_h(0), pad_w(0) {}
    explicit ConvND(const unit_conv2d_desc *p) : ConvND() {
        if (!p) return;
        n = p->n; c = p->c; d = 1; h = p->h; w = p->w; k = p->k; t = 1; r = p->r; s = p->s;
        stride_d = 1; stride_h = p->stride_h; stride_w = p->stride_w; pad_d = 0; pad_h = p->pad_h; pad_w = p->pad_w;
    }
    explicit ConvND(const unit_conv3d_desc *p) : ConvND() {
        if (!p) return;
        n = p->n; c = p->c; d = p->d; h = p->h; w = p->w; k = p->k; t = p->t; r = p->r; s = p->s;
        stride_d = p->stride_d; stride_h = p->stride_h; stride_w = p->stride_w;
        pad_d = p->pad_d; pad_h = p->pad_h; pad_w = p->pad_w;
    }
};

int hip_fail(hipError_t e)
{
    std::snprintf(g_hip_err, sizeof g_hip_err, "%s", hipGetErrorString(e));
    return UNIT_EHIP;
}
#define UNIT_HIP(call) do { hipError_t e_ = (call); if (e_ != hipSuccess) return hip_fail(e_); } while (0)

inline size_t align256(size_t v) { return (v + 255) & ~(size_t)255; }
inline bool dtype_ok(int dtype) { return dtype >= UNIT_I8 && dtype <= UNIT_FP8; }
inline bool byte_type(int dtype) { return dtype == UNIT_I8 || dtype == UNIT_U8I8; }   // integer sums
inline int elem_size(int dtype) { return (byte_type(dtype) || dtype == UNIT_FP8) ? 1 : 2; }
// what the layout kernels need to know: one- or two-byte elements
inline int storage_dtype(int dtype) { return elem_size(dtype) == 1 ? DT_I8 : DT_F16; }
inline long max_reduction(int dtype)
{
    return dtype == UNIT_I8 ? UNIT_MAX_REDUCTION_I8 : dtype == UNIT_U8I8 ? UNIT_MAX_REDUCTION_U8I8 : 0x7fffffffL;
}
inline int chunk_elems(int dtype) { return 16 / elem_size(dtype); }
inline int pad_channels(int c, int dtype) { int ch = chunk_elems(dtype); return (c + ch - 1) / ch * ch; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline bool aligned256(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 255) == 0; }

bool desc_ok(const ConvND *d)
{
    if (!d) return false;
    if (d->n <= 0 || d->c <= 0 || d->d <= 0 || d->h <= 0 || d->w <= 0) return false;
    if (d->k <= 0 || d->t <= 0 || d->r <= 0 || d->s <= 0) return false;
    if (d->stride_d <= 0 || d->stride_h <= 0 || d->stride_w <= 0) return false;
    if (d->pad_d < 0 || d->pad_h < 0 || d->pad_w < 0) return false;
    if (d->d + 2 * d->pad_d < d->t || d->h + 2 * d->pad_h < d->r || d->w + 2 * d->pad_w < d->s) return false;
    return true;
}

size_t packed_act_bytes_nd(const struct ConvND *d, int dtype);
size_t packed_weights_bytes_nd(const struct ConvND *d, int dtype);

struct ConvGeom {
    int o, p, q, cp, kchunks, rows;
    long cols;
    long out_elems;
};

int conv_geom(const ConvND *d, int dtype, ConvGeom *g)
{
    if (!dtype_ok(dtype)) return UNIT_EINVAL;
    if (!desc_ok(d)) return UNIT_EINVAL;
    if (d->n > 65535) return UNIT_ENOTSUP;        // the layout kernels put the image index in grid.z
    g->o = (d->d + 2 * d->pad_d - d->t) / d->stride_d + 1;
    g->p = (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
    g->q = (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
    g->cp = pad_channels(d->c, dtype);
    long red = (long)d->c * d->t * d->r * d->s;
    if (red > max_reduction(dtype)) return UNIT_EOVERFLOW;
    long kbytes = (long)d->t * d->r * d->s * g->cp * elem_size(dtype);
    g->kchunks = (int)(kbytes / 16);
    g->rows = d->k;
    g->cols = (long)d->n * g->o * g->p * g->q;
    g->out_elems = g->cols * d->k;
    // index arithmetic in the kernels is 32-bit for rows/cols/chunks
    if (g->cols > 0x7fffffffL || kbytes > 0x7fffffffL || g->out_elems > (1L << 40)) return UNIT_ENOTSUP;
    // buffer descriptors address at most 2 GiB per tensor
    if ((long)d->n * d->d * d->h * d->w * g->cp * elem_size(dtype) >= 0x7fffffffL) return UNIT_ENOTSUP;
    if (g->out_elems * 4 >= 0x7fffffffL || kbytes * 256 >= 0x7fffffffL) return UNIT_ENOTSUP;
    return UNIT_OK;
}

void fill_tile_info(const RangePlan &p, int dtype, unit_tile_info *out)
{
    const TileChoice &ch = p.choice[0];
    const TileCfg *tiles = dtype == UNIT_FP8 ? g_tiles_fp8 : g_tiles;
    const TileCfg &c = tiles[ch.tile];
    out->block_m = c.bm;  out->block_n = c.bn;  out->block_k_bytes = c.bkb;
    out->waves_m = c.wgm; out->waves_n = c.wgn; out->waves_k = c.wgk;
    out->mfma = c.mf;     out->split_k = ch.split_k;  out->workgroups = ch.workgroups;
    out->tail_block_n = p.n > 1 ? tiles[p.choice[1].tile].bn : 0;
    out->tail_workgroups = p.n > 1 ? p.choice[1].workgroups : 0;
    out->tail_first_col = p.n > 1 ? p.col_begin[1] : 0;
}

// divisor + truncated reciprocal for the kernels' divisions (IgemmArgs::dv_*)
static DivU make_div(long d)
{
    DivU x;
    x.d = d > 1 ? (unsigned)d : 1u;
    x.m = d > 1 ? (unsigned)((1ULL << 32) / (unsigned long long)d) : 0xffffffffu;
    return x;
}

// Runs the main kernel (+ the split reduce when the selector splits across workgroups).
int run_igemm(int dtype, int bsrc, IgemmArgs a, long out_elems, int K, int PQ,
              void *ws, size_t ws_bytes, hipStream_t st, bool allow_split = true)
{
    const bool conv = bsrc != BSRC_PLAIN;
    // (column ranges need tiles that may start anywhere in an image: not with per-image tiling)
    const RangePlan plan = plan_ranges(a.rows, a.cols, a.kchunks, dtype, bsrc, allow_split, conv ? a.CB : 0,
                                       !(conv && a.per_img));
    const TileChoice ch = plan.choice[0];
    for (int r = 0; r < plan.n; ++r)
        if (!tile_fits(plan.choice[r].tile, dtype, bsrc)) return UNIT_ENOTSUP;     // (only a forced tile can fail this)
    // Tile order inside an XCD's run: while the whole B operand is small (<= 8 MiB: every XCD can afford its own
    // copy in L2) a run walks the column tiles of one row tile, so A (the weights) is fetched once in total; large
    // problems walk bands of 8 row tiles, which bounds the re-fetching of both operands.
    a.row_runs = ((long)a.cols * a.kchunks * 16 <= (8L << 20)) ? 1 : 0;
#ifdef UNIT_PROBE
    a.probe = static_cast<unsigned long long *>(g_probe_ptr);
#endif
    {   // divisors of the index arithmetic that do not depend on the tile
        a.nimg = (int)(a.cols / (a.PQ > 0 ? a.PQ : 1));
        a.dv_pq = make_div(a.PQ);
        a.dv_ppq = make_div((long)a.P * a.Q);
        a.dv_q = make_div(a.Q);
        a.dv_w = make_div(a.W);
        a.dv_cpi = make_div(a.cols_per_img);
        a.dv_cb = make_div(a.CB);
        a.dv_s = make_div(a.S);
        a.dv_r = make_div(a.R);
    }
    // ... and the ones of a launch's tile coordinates
    auto set_range = [&](IgemmArgs &x, int r) {
        const TileCfg &t = g_tiles[plan.choice[r].tile];
        const long pq = x.PQ > 0 ? x.PQ : 1;
        const long tiles_img = (pq + t.bn - 1) / t.bn;
        x.col_base = plan.col_begin[r];
        x.col_limit = plan.col_end[r];
        const long tiles_n = (conv && x.per_img) ? tiles_img * x.nimg
                                                 : ((long)x.col_limit - x.col_base + t.bn - 1) / t.bn;
        x.dv_tiles_n = make_div(tiles_n);
        x.dv_band = make_div(8 * tiles_n);
        x.dv_tiles_img = make_div(tiles_img);
        x.ksteps_per_split = plan.choice[r].ksteps_per_split;
    };
    if (ch.split_k == 1) {
        a.split_stride = 0;
        for (int r = 0; r < plan.n; ++r) {
            set_range(a, r);
            UNIT_HIP(launch_igemm(dtype, bsrc, plan.choice[r].tile, a, 1, st));
        }
        return UNIT_OK;
    }
    set_range(a, 0);                               // (a split reduction is always one range)
    const long slice = (out_elems + 3) & ~3L;     // 16-byte aligned slices for the reduce kernel
    size_t need = (size_t)ch.split_k * slice * 4;
    if (!ws || ws_bytes < need) return UNIT_EWORKSPACE;
    IgemmArgs m = a;
    m.out = ws;
    m.split_stride = slice;
    m.epi = EPI_RAW;
    m.store_raw = 1;
    if (!conv) {                                   // partials of a matmul are dense [rows][cols]
        m.row_stride = a.cols;
    }
    UNIT_HIP(launch_igemm(dtype, bsrc, ch.tile, m, ch.split_k, st));
    ReduceArgs r;
    std::memset(&r, 0, sizeof r);
    r.partials = ws;  r.nsplit = ch.split_k;  r.split_stride = slice;
    r.dtype = byte_type(dtype) ? DT_I8 : DT_F16;               // integer or float sums
    r.total = out_elems;  r.K = K;  r.PQ = PQ;
    r.out = (a.epi == EPI_RAW || a.store_raw) ? a.out : nullptr;
    r.epi = a.epi;  r.scale = a.scale;  r.bias = a.bias;  r.residual = a.residual;  r.relu = a.relu;
    r.res_packed = a.res_packed;  r.res_mult = a.res_mult;
    r.out_i8 = a.out_i8;  r.out_packed = a.out_packed;  r.packed_ld = a.packed_ld;
    UNIT_HIP(launch_splitk_reduce(r, st));
    return UNIT_OK;
}

// A 1x1, stride-1, unpadded conv can read its NCHW input directly: the
// channel rows are DMAed as they are and transposed between LDS and the fragments, which
// saves the separate pack_act launch.  The 16-byte global -> LDS loads take any byte offset, so
// the channel rows need no alignment; with several images whose pixel count is not a whole number
// of 16-byte chunks the columns are tiled per image (conv_packed sets per_img).
// The range check of those loads works per dword (a dword that is not wholly inside the buffer reads as
// zero), so with rows that do not start on 4-byte boundaries the chunk that crosses the tensor's end would
// lose valid bytes.  The kernel then does not load that chunk at all and takes its pixels (last channel only)
// from a copy of the tensor's last 16 bytes (IgemmArgs::edge); that needs whole steps of channels and an
// image of at least one chunk.
bool nchw_rows_unaligned(const ConvND *d, int dtype)
{
    return ((long)d->d * d->h * d->w * elem_size(dtype)) % 4 != 0;
}

bool nchw_direct_ok(const ConvND *d, int dtype, const void *x, const unit_requant *rq)
{
    ConvGeom g;
    if (conv_geom(d, dtype, &g) != UNIT_OK) return false;
    TileChoice ch = select_tile(g.rows, (int)g.cols, g.kchunks, dtype, BSRC_NCHW, true, g.cp * elem_size(dtype) / 16);
    if (!tile_fits(ch.tile, dtype, BSRC_NCHW)) return false;
    if (nchw_rows_unaligned(d, dtype)) {
        if (((long)d->c * elem_size(dtype)) % g_tiles[ch.tile].bkb != 0) return false;
        if ((long)d->d * d->h * d->w < chunk_elems(dtype)) return false;
    }
    return d->t == 1 && d->r == 1 && d->s == 1 &&
           d->stride_d == 1 && d->stride_h == 1 && d->stride_w == 1 &&
           d->pad_d == 0 && d->pad_h == 0 && d->pad_w == 0 && rq == nullptr && dtype != UNIT_U8I8 && (reinterpret_cast<uintptr_t>(x) & 15) == 0;
}

// The general direct read (BSRC_NCHWS): stride 1, output grid equal to the input grid
// ("same" padding), whole steps inside one tap, and a tile shape that has a kernel in this mode.
bool nchw_shift_ok(const ConvND *d, int dtype, const ConvGeom &g, const void *x, const unit_requant *rq)
{
    if (rq || dtype == UNIT_U8I8 || d->d != 1 || d->t != 1) return false;
    if (d->stride_h != 1 || d->stride_w != 1) return false;
    if (2 * d->pad_h != d->r - 1 || 2 * d->pad_w != d->s - 1) return false;
    if (reinterpret_cast<uintptr_t>(x) & 15) return false;
    // only the first and the last channel may have needed pixels in a 16-byte chunk that crosses the
    // tensor's start or end (the kernel patches exactly those): true once an image holds a chunk more
    // than the largest tap offset
    const long px = (long)d->h * d->w;
    if (px < (long)d->pad_h * d->w + d->pad_w + chunk_elems(dtype)) return false;
    if ((long)d->n * d->c * px * elem_size(dtype) >= (1L << 31)) return false;    // byte offsets are 32-bit
    // The unaligned loads and the border masks make a step of this mode a little dearer than a gather step; what it
    // saves is the pack_act launch.  That pays while the layer is launch-bound (one image, a few small ones);
    // measured on the 3x3 layers of the ResNet-50 set, fp16: at batch 16 packing first is 5-25 % faster.
    if ((long)g.rows * g.cols * g.kchunks * 16 > (256L << 20)) return false;
    TileChoice ch = select_tile(g.rows, (int)g.cols, g.kchunks, dtype, BSRC_NCHWS, true, g.cp * elem_size(dtype) / 16);
    if (!tile_fits(ch.tile, dtype, BSRC_NCHWS)) return false;
    const TileCfg &t = g_tiles[ch.tile];
    // several images whose pixels are not whole 16-byte chunks are tiled one image at a time: not worth it
    // when the tiles of an image would be more than half empty
    if (d->n > 1 && px % chunk_elems(dtype) != 0 && (px + t.bn - 1) / t.bn * t.bn > 2 * px) return false;
    return ((long)d->c * elem_size(dtype)) % t.bkb == 0;
}

// `xp` is the packed activation tensor, or (direct modes) the caller's NCHW tensor itself.
int conv_packed(const ConvND *d, int dtype, const void *xp, const void *wp,
                void *y_raw, const unit_requant *rq, int8_t *y_i8, void *y_packed,
                void *ws, size_t ws_bytes, void *stream, int bsrc = BSRC_GATHER,
                const int32_t *fix = nullptr)       // fix: per-channel correction of an unsigned operand
{
    const bool nchw_direct = bsrc != BSRC_GATHER;   // xp is the caller's NCHW tensor
    ConvGeom g;
    int rc = conv_geom(d, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!xp || !wp) return UNIT_EINVAL;
    if (!aligned16(xp) || !aligned16(wp)) return UNIT_EINVAL;
    if (rq) {
        if (dtype != UNIT_I8 || !rq->scale || (!y_i8 && !y_packed)) return UNIT_EINVAL;
        if (rq->residual_packed && !aligned16(rq->residual_packed)) return UNIT_EINVAL;
    } else {
        if (!y_raw || y_i8 || y_packed) return UNIT_EINVAL;
    }
    if (ws && !aligned256(ws)) return UNIT_EINVAL;
    if (y_packed && !aligned16(y_packed)) return UNIT_EINVAL;     // written with 32-bit stores, read back as 16-byte chunks
    if ((dtype == UNIT_U8I8) != (fix != nullptr)) return UNIT_EINVAL;

    IgemmArgs a;
    std::memset(&a, 0, sizeof a);
    const int es = elem_size(dtype);
    a.A = static_cast<const uint8_t *>(wp);  a.lda = (long)g.kchunks * 16;  a.rows = d->k;
    a.B = static_cast<const uint8_t *>(xp);  a.ldb = 0;                      a.cols = (int)g.cols;
    a.kchunks = g.kchunks;
    a.D = d->d;  a.H = d->h;  a.W = d->w;  a.CB = g.cp * es / 16;
    a.P = g.p;  a.Q = g.q;  a.PQ = g.o * g.p * g.q;
    a.b_bytes = nchw_direct ? (long)d->n * d->c * d->d * d->h * d->w * es : (long)d->n * d->d * d->h * d->w * g.cp * es;
    a.Cin = d->c;
    a.edge = (bsrc == BSRC_NCHW && nchw_rows_unaligned(d, dtype)) ? 1 : 0;
    a.per_img = (nchw_direct && d->n > 1 && ((long)d->d * d->h * d->w) % chunk_elems(dtype) != 0) ? 1 : 0;
    a.T = d->t;  a.R = d->r;  a.S = d->s;
    a.sd = d->stride_d;  a.sh = d->stride_h;  a.sw = d->stride_w;  a.pd = d->pad_d;  a.ph = d->pad_h;  a.pw = d->pad_w;
    a.out = y_raw;  a.row_stride = a.PQ;  a.img_stride = (long)d->k * a.PQ;  a.cols_per_img = a.PQ;
    if (rq) {
        a.epi = EPI_REQUANT;  a.scale = rq->scale;  a.bias = rq->bias;  a.residual = rq->residual;
        a.relu = rq->relu ? 1 : 0;
        a.res_packed = static_cast<const int8_t *>(rq->residual_packed);
        a.res_mult = rq->residual_packed ? rq->residual_mult : 0;
        a.out_i8 = y_i8;  a.out_packed = static_cast<int8_t *>(y_packed);
        a.packed_ld = pad_channels(d->k, UNIT_I8);
        a.store_raw = y_raw ? 1 : 0;
    } else {
        a.epi = EPI_RAW;  a.store_raw = 1;  a.bias = fix;
    }
    return run_igemm(dtype, bsrc, a, g.out_elems, d->k, a.PQ, ws, ws_bytes,
                     static_cast<hipStream_t>(stream));
}

size_t packed_act_bytes_nd(const ConvND *d, int dtype)
{
    return align256((size_t)d->n * d->d * d->h * d->w * pad_channels(d->c, dtype) * elem_size(dtype));
}
size_t packed_weights_bytes_nd(const ConvND *d, int dtype)
{
    return align256((size_t)d->k * d->t * d->r * d->s * pad_channels(d->c, dtype) * elem_size(dtype));
}

size_t conv_fix_bytes(const ConvND *d, int dtype)
{
    return dtype == UNIT_U8I8 ? align256((size_t)d->k * 4) : 0;
}

size_t conv_split_bytes(const ConvGeom &g, int dtype, int bsrc)
{
    TileChoice ch = select_tile(g.rows, (int)g.cols, g.kchunks, dtype, bsrc, true, g.cp * elem_size(dtype) / 16);
    return ch.split_k > 1 ? align256((size_t)ch.split_k * ((g.out_elems + 3) & ~3L) * 4) : 0;
}
// what a caller who does not know the input mode yet must provide
size_t conv_split_bytes_any(const ConvGeom &g, int dtype)
{
    size_t a = conv_split_bytes(g, dtype, BSRC_GATHER), b = conv_split_bytes(g, dtype, BSRC_NCHWS);
    return a > b ? a : b;
}

int conv_wpacked(const ConvND *d, int dtype, const void *x, const void *wp,
                 void *y_raw, const unit_requant *rq, int8_t *y_i8,
                 void *ws, size_t ws_bytes, void *stream, const int32_t *fix = nullptr);
bool nchw_direct_ok(const ConvND *d, int dtype, const void *x, const unit_requant *rq);

// workspace conv_wpacked needs for this call (after the packed weights, if any)
size_t wpacked_need(const ConvND *d, int dtype, const ConvGeom &g, const void *x, const unit_requant *rq)
{
    if (nchw_direct_ok(d, dtype, x, rq)) return conv_split_bytes(g, dtype, BSRC_NCHW);
    if (nchw_shift_ok(d, dtype, g, x, rq)) return conv_split_bytes(g, dtype, BSRC_NCHWS);
    return packed_act_bytes_nd(d, dtype) + conv_split_bytes(g, dtype, BSRC_GATHER);
}

int static_scratch(void **ptr);

int conv_plain(const ConvND *d, int dtype, const void *x, const void *w,
               void *y_raw, const unit_requant *rq, int8_t *y_i8,
               void *ws, size_t ws_bytes, void *stream)
{
    ConvGeom g;
    int rc = conv_geom(d, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!x || !w) return UNIT_EINVAL;
    if (rq) {
        if (dtype != UNIT_I8 || !rq->scale || !y_i8) return UNIT_EINVAL;
    } else if (!y_raw || y_i8) {
        return UNIT_EINVAL;
    }
    size_t wt_b = packed_weights_bytes_nd(d, dtype);
    size_t fix_b = conv_fix_bytes(d, dtype);
    if (!ws || ws_bytes < wt_b + fix_b + wpacked_need(d, dtype, g, x, rq)) return UNIT_EWORKSPACE;
    if (!aligned256(ws)) return UNIT_EINVAL;
    uint8_t *wp = static_cast<uint8_t *>(ws);
    hipStream_t st = static_cast<hipStream_t>(stream);
    UNIT_HIP(launch_pack_weights(storage_dtype(dtype), d->k, d->c, d->t * d->r, d->s, w, wp, st));
    int32_t *fix = nullptr;
    if (fix_b) {            // unsigned activations: 128 * (sum of each filter's weights)
        fix = reinterpret_cast<int32_t *>(wp + wt_b);
        UNIT_HIP(launch_rowsum128_i8(wp, (long)g.kchunks * 16, d->k, g.kchunks, fix, st));
    }
    return conv_wpacked(d, dtype, x, wp, y_raw, rq, y_i8, wp + wt_b + fix_b, ws_bytes - wt_b - fix_b, stream, fix);
}

// NCHW activations + packed weights: fused direct read when possible, else pack_act into the
// workspace followed by the packed kernel.
int conv_wpacked(const ConvND *d, int dtype, const void *x, const void *wp,
                 void *y_raw, const unit_requant *rq, int8_t *y_i8,
                 void *ws, size_t ws_bytes, void *stream, const int32_t *fix)
{
    ConvGeom g;
    int rc = conv_geom(d, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!x || !wp) return UNIT_EINVAL;
    if (ws && !aligned256(ws)) return UNIT_EINVAL;
    if (!aligned16(wp)) return UNIT_EINVAL;
    size_t split_b = conv_split_bytes(g, dtype, BSRC_NCHW);
    if (nchw_direct_ok(d, dtype, x, rq)) {
        if (split_b && (!ws || ws_bytes < split_b)) return UNIT_EWORKSPACE;
        return conv_packed(d, dtype, x, wp, y_raw, rq, y_i8, nullptr, ws, ws_bytes, stream, BSRC_NCHW);
    }
    if (nchw_shift_ok(d, dtype, g, x, rq)) {
        split_b = conv_split_bytes(g, dtype, BSRC_NCHWS);
        if (split_b && (!ws || ws_bytes < split_b)) return UNIT_EWORKSPACE;
        return conv_packed(d, dtype, x, wp, y_raw, rq, y_i8, nullptr, ws, ws_bytes, stream, BSRC_NCHWS);
    }
    split_b = conv_split_bytes(g, dtype, BSRC_GATHER);
    size_t act_b = packed_act_bytes_nd(d, dtype);
    if (!ws || ws_bytes < act_b + split_b) return UNIT_EWORKSPACE;
    uint8_t *xp = static_cast<uint8_t *>(ws);
    // A strided 1x1 conv reads one pixel in stride_h*stride_w: pack only those and run the
    // unit-stride 1x1 conv on the subsampled tensor (same reduction, same output).
    if (d->d == 1 && d->t == 1 && d->r == 1 && d->s == 1 && d->pad_h == 0 && d->pad_w == 0 &&
        (d->stride_h > 1 || d->stride_w > 1)) {
        ConvND sub = *d;
        sub.h = g.p;  sub.w = g.q;  sub.stride_h = sub.stride_w = 1;
        UNIT_HIP(launch_pack_act_sub(storage_dtype(dtype), d->n, d->c, d->h, d->w, d->stride_h, d->stride_w,
                                     g.p, g.q, x, xp, static_cast<hipStream_t>(stream)));
        return conv_packed(&sub, dtype, xp, wp, y_raw, rq, y_i8, nullptr, split_b ? xp + act_b : nullptr, split_b,
                           stream, BSRC_GATHER, fix);
    }
    UNIT_HIP(launch_pack_act(storage_dtype(dtype), d->n, d->c, d->d * d->h, d->w, x, xp, static_cast<hipStream_t>(stream)));
    return conv_packed(d, dtype, xp, wp, y_raw, rq, y_i8, nullptr, split_b ? xp + act_b : nullptr, split_b, stream,
                       BSRC_GATHER, fix);
}

struct MatmulGeom {
    int kpad_bytes, kchunks;
    bool pad_a, pad_b;
    bool gemv;                 // at most GEMV_MAX_ROWS rows: the dot-product kernel instead of the matrix units
    size_t a_bytes, b_bytes, fix_bytes, split_bytes;
};

int matmul_geom(int m, int n, int k, long lda, long ldb, int dtype, MatmulGeom *g)
{
    if (!dtype_ok(dtype)) return UNIT_EINVAL;
    if (m <= 0 || n <= 0 || k <= 0 || lda < k || ldb < k) return UNIT_EINVAL;
    if (k > max_reduction(dtype)) return UNIT_EOVERFLOW;
    const int es = elem_size(dtype);
    // a 256-row tile of either operand and of C must stay below 2 GiB (buffer descriptors)
    if (lda * es * 256 >= 0x7fffffffL || ldb * es * 256 >= 0x7fffffffL) return UNIT_ENOTSUP;
    g->kpad_bytes = (int)(((long)k * es + 15) / 16 * 16);
    g->kchunks = g->kpad_bytes / 16;
    bool ktail = ((long)k * es) % 16 != 0;
    g->pad_a = ktail || (lda * es) % 16 != 0;
    g->pad_b = ktail || (ldb * es) % 16 != 0;
    g->a_bytes = g->pad_a ? align256((size_t)m * g->kpad_bytes) : 0;
    g->b_bytes = g->pad_b ? align256((size_t)n * g->kpad_bytes) : 0;
    g->fix_bytes = dtype == UNIT_U8I8 ? align256((size_t)n * 4) : 0;
    g->gemv = m <= GEMV_MAX_ROWS && (dtype == UNIT_I8 || dtype == UNIT_F16) && !tile_is_forced();
    TileChoice ch = select_tile(m, n, g->kchunks, dtype, BSRC_PLAIN);
    g->split_bytes = (ch.split_k > 1 && !g->gemv) ? align256((size_t)ch.split_k * (((long)m * n + 3) & ~3L) * 4) : 0;
    return UNIT_OK;
}

int matmul_any(int dtype, int m, int n, int k, const void *A, long lda, const void *B, long ldb,
               void *C, long ldc, void *ws, size_t ws_bytes, void *stream)
{
    MatmulGeom g;
    int rc = matmul_geom(m, n, k, lda, ldb, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!A || !B || !C || ldc < n) return UNIT_EINVAL;
    if (ldc * 4 * 256 >= 0x7fffffffL) return UNIT_ENOTSUP;
    const int es = elem_size(dtype);
    if ((!g.pad_a && !aligned16(A)) || (!g.pad_b && !aligned16(B))) return UNIT_EINVAL;
    if (reinterpret_cast<uintptr_t>(C) & 3) return UNIT_EINVAL;
    size_t need = g.a_bytes + g.b_bytes + g.fix_bytes + g.split_bytes;
    if (need && (!ws || ws_bytes < need)) return UNIT_EWORKSPACE;
    if (need && !aligned256(ws)) return UNIT_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    uint8_t *wsp = static_cast<uint8_t *>(ws);
    const uint8_t *Ap = static_cast<const uint8_t *>(A);
    const uint8_t *Bp = static_cast<const uint8_t *>(B);
    long lda_b = lda * es, ldb_b = ldb * es;
    if (g.pad_a) {
        UNIT_HIP(launch_pad_rows(A, lda_b, m, k * es, wsp, g.kpad_bytes, st));
        Ap = wsp;  lda_b = g.kpad_bytes;  wsp += g.a_bytes;
    }
    if (g.pad_b) {
        UNIT_HIP(launch_pad_rows(B, ldb_b, n, k * es, wsp, g.kpad_bytes, st));
        Bp = wsp;  ldb_b = g.kpad_bytes;  wsp += g.b_bytes;
    }
    if (g.gemv) {
        UNIT_HIP(launch_gemv(dtype == UNIT_I8 ? DT_I8 : DT_F16, Ap, lda_b, Bp, ldb_b, m, n, g.kchunks, C, ldc, st));
        return UNIT_OK;
    }
    IgemmArgs a;
    std::memset(&a, 0, sizeof a);
    a.A = Ap;  a.lda = lda_b;  a.rows = m;
    a.B = Bp;  a.ldb = ldb_b;  a.cols = n;
    a.kchunks = g.kchunks;
    a.out = C;  a.row_stride = ldc;  a.img_stride = 0;  a.cols_per_img = n;
    a.epi = EPI_RAW;  a.store_raw = 1;
    if (g.fix_bytes) {      // unsigned A: 128 * (sum of each column of B) corrects every output column
        int32_t *fix = reinterpret_cast<int32_t *>(wsp);
        UNIT_HIP(launch_rowsum128_i8(Bp, ldb_b, n, g.kchunks, fix, st));
        a.bias = fix;  wsp += g.fix_bytes;
    }
    // the split reduce writes a dense [m][n] result: only usable when ldc == n
    return run_igemm(dtype, BSRC_PLAIN, a, (long)m * n, 1, n, g.split_bytes ? wsp : nullptr, g.split_bytes, st,
                     ldc == n);
}

}  // namespace

// Scratch of unit_conv2d_wpacked_i8_static: one copy per GPU the library's code object is loaded on,
// held until the process ends.  In host code the name is only a handle for hipGetSymbolAddress; the
// device address it yields (per device) is what kernels and copies are given.
static __device__ __align__(256) unsigned char scratch[UNIT_STATIC_SCRATCH_BYTES];

namespace {
enum { MAX_DEVICES = 64 };
void *g_scratch_ptr[MAX_DEVICES];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device, looked up once per device.
int static_scratch(void **ptr)
{
    int dev = -1;
    UNIT_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return UNIT_ENOTSUP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        UNIT_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return UNIT_EHIP;
        g_scratch_ptr[dev] = p;
    }
    *ptr = g_scratch_ptr[dev];
    return UNIT_OK;
}
}  // namespace

extern "C" {

#ifdef UNIT_PROBE
// Instrumented build only: main-kernel launches from now on write their per-wave time stamps to `buf`
// (device memory, (workgroups * waves) * 128 bytes for the largest launch; NULL switches it off).
void unit_probe_set(void *buf) { g_probe_ptr = buf; }
#endif

int unit_version(void) { return 110; }

const char *unit_status_str(int status)
{
    switch (status) {
    case UNIT_OK:         return "ok";
    case UNIT_EINVAL:     return "invalid argument";
    case UNIT_ENOTSUP:    return "unsupported shape";
    case UNIT_EOVERFLOW:  return "byte reduction too long for an exact int32 sum";
    case UNIT_EWORKSPACE: return "workspace missing or too small";
    case UNIT_EHIP:       return "HIP runtime error";
    case UNIT_ESCRATCH:   return "problem needs more scratch than the static buffer of the *_static entry point holds";
    default:              return "unknown status";
    }
}

const char *unit_last_hip_error(void) { return g_hip_err; }

int unit_conv2d_out_dims(const unit_conv2d_desc *d, int32_t *p, int32_t *q)
{
    ConvND nd(d);
    if (!desc_ok(&nd) || !p || !q) return UNIT_EINVAL;
    *p = (d->h + 2 * d->pad_h - d->r) / d->stride_h + 1;
    *q = (d->w + 2 * d->pad_w - d->s) / d->stride_w + 1;
    return UNIT_OK;
}

size_t unit_packed_act_bytes(int32_t n, int32_t c, int32_t h, int32_t w, int dtype)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || !dtype_ok(dtype)) return 0;
    return align256((size_t)n * h * w * pad_channels(c, dtype) * elem_size(dtype));
}

size_t unit_packed_weights_bytes(const unit_conv2d_desc *d, int dtype)
{
    ConvND nd(d);
    if (!desc_ok(&nd) || !dtype_ok(dtype)) return 0;
    return packed_weights_bytes_nd(&nd, dtype);
}

size_t unit_conv2d_packed_workspace(const unit_conv2d_desc *d, int dtype)
{
    ConvGeom g;
    ConvND nd(d);
    if (conv_geom(&nd, dtype, &g) != UNIT_OK) return 0;
    return conv_split_bytes(g, dtype, BSRC_GATHER);
}

size_t unit_conv2d_workspace(const unit_conv2d_desc *d, int dtype)
{
    ConvGeom g;
    ConvND nd(d);
    if (conv_geom(&nd, dtype, &g) != UNIT_OK) return 0;
    return packed_act_bytes_nd(&nd, dtype) + packed_weights_bytes_nd(&nd, dtype) + conv_fix_bytes(&nd, dtype) +
           conv_split_bytes_any(g, dtype);
}

size_t unit_matmul_workspace(int32_t m, int32_t n, int32_t k, int64_t lda, int64_t ldb, int dtype)
{
    MatmulGeom g;
    if (matmul_geom(m, n, k, lda, ldb, dtype, &g) != UNIT_OK) return 0;
    return g.a_bytes + g.b_bytes + g.fix_bytes + g.split_bytes;
}

int unit_select_conv2d(const unit_conv2d_desc *d, int dtype, unit_tile_info *out)
{
    ConvGeom g;
    ConvND nd(d);
    int rc = conv_geom(&nd, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!out) return UNIT_EINVAL;
    fill_tile_info(plan_ranges(g.rows, (int)g.cols, g.kchunks, dtype, BSRC_GATHER, true, g.cp * elem_size(dtype) / 16, true), dtype, out);
    return UNIT_OK;
}

int unit_select_conv2d_input(const unit_conv2d_desc *d, int dtype, int input_mode, unit_tile_info *out)
{
    ConvGeom g;
    ConvND nd(d);
    int rc = conv_geom(&nd, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!out || input_mode < UNIT_INPUT_PACKED || input_mode > UNIT_INPUT_DIRECT_SHIFTED) return UNIT_EINVAL;
    const int bsrc = input_mode == UNIT_INPUT_DIRECT ? BSRC_NCHW : input_mode == UNIT_INPUT_DIRECT_SHIFTED ? BSRC_NCHWS : BSRC_GATHER;
    fill_tile_info(plan_ranges(g.rows, (int)g.cols, g.kchunks, dtype, bsrc, true, g.cp * elem_size(dtype) / 16, true), dtype, out);
    return UNIT_OK;
}

int unit_conv2d_input_mode(const unit_conv2d_desc *d, int dtype, const void *x)
{
    ConvGeom g;
    ConvND nd(d);
    int rc = conv_geom(&nd, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!x) return UNIT_EINVAL;
    if (nchw_direct_ok(&nd, dtype, x, nullptr)) return UNIT_INPUT_DIRECT;
    if (nchw_shift_ok(&nd, dtype, g, x, nullptr)) return UNIT_INPUT_DIRECT_SHIFTED;
    return UNIT_INPUT_PACKED;
}

int unit_debug_force_tile(int32_t tile, int32_t split_k)
{
    if (tile >= NUM_TILES) return UNIT_EINVAL;
    force_tile(tile < 0 ? -1 : tile, split_k < 1 ? -1 : split_k);
    return UNIT_OK;
}

int unit_measure_mfma(int dtype, int32_t steps, int32_t random_operands, void *counters, size_t counters_bytes,
                      void *stream)
{
    if (dtype < UNIT_I8 || dtype > UNIT_BF16 || steps <= 0 || !counters) return UNIT_EINVAL;
    if (counters_bytes < (size_t)UNIT_MEASURE_COUNTERS_BYTES) return UNIT_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(counters) & 7) return UNIT_EINVAL;
    UNIT_HIP(launch_mfma_ceiling(dtype, steps, random_operands ? 1 : 0, counters, static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_select_matmul(int32_t m, int32_t n, int32_t k, int dtype, unit_tile_info *out)
{
    MatmulGeom g;
    int rc = matmul_geom(m, n, k, k, k, dtype, &g);
    if (rc != UNIT_OK) return rc;
    if (!out) return UNIT_EINVAL;
    fill_tile_info(plan_ranges(m, n, g.kchunks, dtype, BSRC_PLAIN, true, 0, true), dtype, out);
    if (g.gemv) {               // one wave per output column on the vector ALU's dot-product instructions
        out->block_m = m == 1 ? 1 : m == 2 ? 2 : m <= 4 ? 4 : 8;  out->block_n = 4;  out->block_k_bytes = 2048;
        out->waves_m = 1;  out->waves_n = 4;  out->waves_k = 1;  out->mfma = 0;
        out->split_k = 1;  out->workgroups = (n + 3) / 4;
        out->tail_block_n = out->tail_workgroups = out->tail_first_col = 0;
    }
    return UNIT_OK;
}

int unit_conv2d_i8(const unit_conv2d_desc *d, const int8_t *x, const int8_t *w,
                   int32_t *y_i32, const unit_requant *rq, int8_t *y_i8,
                   void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_I8, x, w, y_i32, rq, y_i8, ws, ws_bytes, stream);
}

int unit_conv2d_f16(const unit_conv2d_desc *d, const uint16_t *x, const uint16_t *w,
                    float *y, void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_F16, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_matmul_i8(int32_t m, int32_t n, int32_t k, const int8_t *A, int64_t lda,
                   const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc,
                   void *ws, size_t ws_bytes, void *stream)
{
    return matmul_any(UNIT_I8, m, n, k, A, lda, B, ldb, C, ldc, ws, ws_bytes, stream);
}

int unit_matmul_f16(int32_t m, int32_t n, int32_t k, const uint16_t *A, int64_t lda,
                    const uint16_t *B, int64_t ldb, float *C, int64_t ldc,
                    void *ws, size_t ws_bytes, void *stream)
{
    return matmul_any(UNIT_F16, m, n, k, A, lda, B, ldb, C, ldc, ws, ws_bytes, stream);
}

int unit_conv2d_bf16(const unit_conv2d_desc *d, const uint16_t *x, const uint16_t *w,
                     float *y, void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_BF16, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_matmul_bf16(int32_t m, int32_t n, int32_t k, const uint16_t *A, int64_t lda,
                     const uint16_t *B, int64_t ldb, float *C, int64_t ldc,
                     void *ws, size_t ws_bytes, void *stream)
{
    return matmul_any(UNIT_BF16, m, n, k, A, lda, B, ldb, C, ldc, ws, ws_bytes, stream);
}

int unit_conv2d_fp8(const unit_conv2d_desc *d, const uint8_t *x, const uint8_t *w,
                    float *y, void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_FP8, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_matmul_fp8(int32_t m, int32_t n, int32_t k, const uint8_t *A, int64_t lda,
                    const uint8_t *B, int64_t ldb, float *C, int64_t ldc,
                    void *ws, size_t ws_bytes, void *stream)
{
    return matmul_any(UNIT_FP8, m, n, k, A, lda, B, ldb, C, ldc, ws, ws_bytes, stream);
}

int unit_conv2d_u8i8(const unit_conv2d_desc *d, const uint8_t *x, const int8_t *w,
                     int32_t *y, void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_U8I8, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_matmul_u8i8(int32_t m, int32_t n, int32_t k, const uint8_t *A, int64_t lda,
                     const int8_t *B, int64_t ldb, int32_t *C, int64_t ldc,
                     void *ws, size_t ws_bytes, void *stream)
{
    return matmul_any(UNIT_U8I8, m, n, k, A, lda, B, ldb, C, ldc, ws, ws_bytes, stream);
}

static int pack_act_any(int dtype, int32_t n, int32_t c, int32_t h, int32_t w, const void *x,
                        void *xp, size_t bytes, void *stream)
{
    size_t need = unit_packed_act_bytes(n, c, h, w, dtype);
    if (!need || !x || !xp) return UNIT_EINVAL;
    if (n > 65535) return UNIT_ENOTSUP;           // the image index is grid.z
    if (bytes < need) return UNIT_EWORKSPACE;
    if (!aligned16(xp)) return UNIT_EINVAL;
    UNIT_HIP(launch_pack_act(dtype, n, c, h, w, x, xp, static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_pack_act_i8(int32_t n, int32_t c, int32_t h, int32_t w, const int8_t *x,
                     void *xp, size_t bytes, void *stream)
{
    return pack_act_any(UNIT_I8, n, c, h, w, x, xp, bytes, stream);
}

int unit_pack_act_f16(int32_t n, int32_t c, int32_t h, int32_t w, const uint16_t *x,
                      void *xp, size_t bytes, void *stream)
{
    return pack_act_any(UNIT_F16, n, c, h, w, x, xp, bytes, stream);
}

static int pack_w_any(int dtype, const unit_conv2d_desc *d, const void *w, void *wp, size_t bytes, void *stream)
{
    size_t need = unit_packed_weights_bytes(d, dtype);
    if (!need || !w || !wp) return UNIT_EINVAL;
    if (bytes < need) return UNIT_EWORKSPACE;
    if (!aligned16(wp)) return UNIT_EINVAL;
    UNIT_HIP(launch_pack_weights(dtype, d->k, d->c, d->r, d->s, w, wp, static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_pack_weights_i8(const unit_conv2d_desc *d, const int8_t *w, void *wp, size_t bytes, void *stream)
{
    return pack_w_any(UNIT_I8, d, w, wp, bytes, stream);
}

int unit_pack_weights_f16(const unit_conv2d_desc *d, const uint16_t *w, void *wp, size_t bytes, void *stream)
{
    return pack_w_any(UNIT_F16, d, w, wp, bytes, stream);
}

int unit_unpack_act_i8(int32_t n, int32_t c, int32_t h, int32_t w, const void *xp, int8_t *x, void *stream)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || !xp || !x) return UNIT_EINVAL;
    UNIT_HIP(launch_unpack_act_i8(n, c, h, w, xp, x, static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_conv2d_packed_i8(const unit_conv2d_desc *d, const void *xp, const void *wp,
                          int32_t *y_i32, const unit_requant *rq, int8_t *y_i8, void *y_packed,
                          void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_packed(&nd, UNIT_I8, xp, wp, y_i32, rq, y_i8, y_packed, ws, ws_bytes, stream);
}

size_t unit_conv2d_wpacked_workspace(const unit_conv2d_desc *d, int dtype)
{
    ConvGeom g;
    ConvND nd(d);
    if (conv_geom(&nd, dtype, &g) != UNIT_OK) return 0;
    return packed_act_bytes_nd(&nd, dtype) + conv_split_bytes_any(g, dtype);
}

int unit_conv2d_wpacked_i8(const unit_conv2d_desc *d, const int8_t *x, const void *wp,
                           int32_t *y_i32, const unit_requant *rq, int8_t *y_i8,
                           void *ws, size_t ws_bytes, void *stream)
{
    if (rq ? (!rq->scale || !y_i8) : (!y_i32 || y_i8)) return UNIT_EINVAL;
    ConvND nd(d);
    return conv_wpacked(&nd, UNIT_I8, x, wp, y_i32, rq, y_i8, ws, ws_bytes, stream);
}

int unit_conv2d_wpacked_i8_static(const unit_conv2d_desc *d, const int8_t *x, const void *wp,
                                  int32_t *y_i32, const unit_requant *rq, int8_t *y_i8, void *stream)
{
    if (rq ? (!rq->scale || !y_i8) : (!y_i32 || y_i8)) return UNIT_EINVAL;
    ConvND nd(d);
    ConvGeom g;
    int rc = conv_geom(&nd, UNIT_I8, &g);
    if (rc != UNIT_OK) return rc;
    if (!x || !wp) return UNIT_EINVAL;
    // the size test comes before the first HIP call, like every other argument error
    if (wpacked_need(&nd, UNIT_I8, g, x, rq) > (size_t)UNIT_STATIC_SCRATCH_BYTES) return UNIT_ESCRATCH;
    void *ws = nullptr;
    rc = static_scratch(&ws);
    if (rc != UNIT_OK) return rc;
    return conv_wpacked(&nd, UNIT_I8, x, wp, y_i32, rq, y_i8, ws, UNIT_STATIC_SCRATCH_BYTES, stream);
}

int unit_conv2d_wpacked_f16(const unit_conv2d_desc *d, const uint16_t *x, const void *wp,
                            float *y, void *ws, size_t ws_bytes, void *stream)
{
    if (!y) return UNIT_EINVAL;
    ConvND nd(d);
    return conv_wpacked(&nd, UNIT_F16, x, wp, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_conv2d_packed_f16(const unit_conv2d_desc *d, const void *xp, const void *wp,
                           float *y, void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_packed(&nd, UNIT_F16, xp, wp, y, nullptr, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_maxpool_packed_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                           int32_t window, int32_t stride, int32_t pad,
                           const void *xp, void *yp, void *stream)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || window <= 0 || stride <= 0 || pad < 0 || !xp || !yp)
        return UNIT_EINVAL;
    if (pad >= window || h + 2 * pad < window || w + 2 * pad < window) return UNIT_EINVAL;
    if (!aligned16(xp) || !aligned16(yp)) return UNIT_EINVAL;
    int p = (h + 2 * pad - window) / stride + 1, q = (w + 2 * pad - window) / stride + 1;
    const long cpl = pad_channels(c, UNIT_I8);
    if ((long)n * h * w * cpl >= (1L << 31)) return UNIT_ENOTSUP;     // addressed through a buffer descriptor
    UNIT_HIP(launch_maxpool_packed_i8(n, pad_channels(c, UNIT_I8), h, w, window, stride, pad, p, q,
                                      xp, yp, static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_global_avgpool_packed_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                                  const void *xp, const float *scale, int8_t *y, void *stream)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || !xp || !scale || !y) return UNIT_EINVAL;
    if (!aligned16(xp)) return UNIT_EINVAL;
    if ((long)h * w > 16777216L) return UNIT_EOVERFLOW;
    UNIT_HIP(launch_avgpool_packed_i8(n, c, pad_channels(c, UNIT_I8), h * w, xp, scale, y,
                                      static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_widen_residual_i8(int32_t n, int32_t c, int32_t h, int32_t w,
                           const void *xp, int32_t mult, int32_t *residual, void *stream)
{
    if (n <= 0 || c <= 0 || h <= 0 || w <= 0 || !xp || !residual) return UNIT_EINVAL;
    UNIT_HIP(launch_widen_residual_i8(n, c, pad_channels(c, UNIT_I8), h * w, xp, mult, residual,
                                      static_cast<hipStream_t>(stream)));
    return UNIT_OK;
}

int unit_conv3d_out_dims(const unit_conv3d_desc *d, int32_t *o, int32_t *p, int32_t *q)
{
    ConvND nd(d);
    if (!desc_ok(&nd) || !o || !p || !q) return UNIT_EINVAL;
    *o = (nd.d + 2 * nd.pad_d - nd.t) / nd.stride_d + 1;
    *p = (nd.h + 2 * nd.pad_h - nd.r) / nd.stride_h + 1;
    *q = (nd.w + 2 * nd.pad_w - nd.s) / nd.stride_w + 1;
    return UNIT_OK;
}

size_t unit_conv3d_workspace(const unit_conv3d_desc *d, int dtype)
{
    ConvGeom g;
    ConvND nd(d);
    if (conv_geom(&nd, dtype, &g) != UNIT_OK) return 0;
    return packed_act_bytes_nd(&nd, dtype) + packed_weights_bytes_nd(&nd, dtype) + conv_fix_bytes(&nd, dtype) +
           conv_split_bytes_any(g, dtype);
}

int unit_conv3d_i8(const unit_conv3d_desc *d, const int8_t *x, const int8_t *w, int32_t *y,
                   void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_I8, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

int unit_conv3d_f16(const unit_conv3d_desc *d, const uint16_t *x, const uint16_t *w, float *y,
                    void *ws, size_t ws_bytes, void *stream)
{
    ConvND nd(d);
    return conv_plain(&nd, UNIT_F16, x, w, y, nullptr, nullptr, ws, ws_bytes, stream);
}

}  // extern "C"
