// Host side of libhgc: descriptor validation, problem geometry, choice of
// algorithm and tiling, and the launches.  Everything up to the launch is plain
// integer work on the host; nothing here allocates, copies or synchronises
// (the paper's rules: scalars stay host scalars, Section 3.2; no host<->device
// traffic or conversions on the path, Section 3.3).
#include <algorithm>
#include <atomic>
#include <climits>
#include <cstring>

#include "hgc_internal.h"

namespace hgc {

static std::atomic<int> g_forced_path{HGC_PATH_AUTO};
static std::atomic<int> g_forced_variant{-1};
static thread_local int g_last_hip_error = 0;

static constexpr long long kMaxLds = 160 * 1024;

static hgc_status validate(const hgc_conv2d_desc *d, Geometry *g)
{
    if (d->N < 1 || d->C < 1 || d->H < 1 || d->W < 1 || d->num_output < 1 || d->kernel < 1 ||
        d->stride < 1 || d->pad < 0 || d->group < 1)
        return HGC_ERR_BAD_DESC;
    if (d->C % d->group || d->num_output % d->group) return HGC_ERR_BAD_DESC;
    if (d->bias != 0 && d->bias != 1) return HGC_ERR_BAD_DESC;
    if (d->relu != 0 && d->relu != 1) return HGC_ERR_BAD_DESC;
    const long long Hp = (long long)d->H + 2LL * d->pad, Wp = (long long)d->W + 2LL * d->pad;
    if (Hp < d->kernel || Wp < d->kernel) return HGC_ERR_BAD_DESC;
    if (Hp > INT_MAX || Wp > INT_MAX) return HGC_ERR_TOO_LARGE;
    g->N = d->N; g->C = d->C; g->H = d->H; g->W = d->W; g->M = d->num_output;
    g->k = d->kernel; g->s = d->stride; g->p = d->pad; g->G = d->group;
    g->bias = d->bias; g->relu = d->relu;
    g->Ho = (int)((Hp - d->kernel) / d->stride) + 1;
    g->Wo = (int)((Wp - d->kernel) / d->stride) + 1;
    g->Cg = d->C / d->group;
    g->Mg = d->num_output / d->group;
    g->Kg = (long long)g->Cg * g->k * g->k;
    g->P = (long long)g->N * g->Ho * g->Wo;
    // kernels index tensors with 32-bit element counts
    const long long lim = INT_MAX;
    const long long nx = (long long)g->N * g->C;
    if (nx > lim || nx * g->H > lim || nx * g->H * g->W > lim) return HGC_ERR_TOO_LARGE;
    if ((long long)g->M * g->Cg > lim || (long long)g->M * g->Kg > lim) return HGC_ERR_TOO_LARGE;
    const long long ny = (long long)g->N * g->M;
    if (ny > lim || ny * g->Ho > lim || ny * g->Ho * g->Wo > lim) return HGC_ERR_TOO_LARGE;
    return HGC_OK;
}

struct Plan {
    hgc_plan pub;
    ConvArgs args;
    const IgemmVariant *variant;
};

static void base_args(const Geometry &g, ConvArgs *a)
{
    std::memset(a, 0, sizeof(*a));
    a->N = g.N; a->C = g.C; a->H = g.H; a->W = g.W; a->M = g.M; a->Ho = g.Ho; a->Wo = g.Wo;
    a->Cg = g.Cg; a->Mg = g.Mg; a->G = g.G;
    a->ks = g.k; a->stride = g.s; a->pad = g.p; a->bias = g.bias; a->relu = g.relu;
    a->split_k = 1;
}

static int ceil_div(long long a, long long b) { return (int)((a + b - 1) / b); }

// Pick the output-window shape (tile_w = 2^j columns, tile_h = BN / tile_w rows)
// that wastes the fewest accumulator columns on pixels outside the image, and fits LDS.
static bool choose_window(const Geometry &g, const IgemmVariant &v, ConvArgs *a, long long *lds_out)
{
    const int BN = v.BN();
    double best = 1e30;
    bool found = false;
    for (int j = 2; (1 << j) <= BN && j <= 6; ++j) {
        const int TW = 1 << j, TH = BN >> j;
        const int tiles_w = ceil_div(g.Wo, TW), tiles_h = ceil_div(g.Ho, TH);
        const int PH = (TH - 1) * g.s + g.k;
        const int PW = (TW - 1) * g.s + g.k;
        const int PWU = (v.xvec == 2) ? 2 * ((PW + 2) / 2) : PW;
        const long long lds = (long long)v.lds_bytes + 16LL * v.npl * PH * PWU;
        if (lds > kMaxLds) continue;
        // cost: padded pixel slots, with a mild preference for wide rows (coalesced stores)
        double cost = (double)tiles_w * TW * tiles_h * TH / ((double)g.Wo * g.Ho);
        cost *= 1.0 + 0.02 * (6 - j);
        if (cost < best) {
            best = cost; found = true;
            a->log2_tw = j; a->tiles_w = tiles_w; a->tiles_h = tiles_h;
            a->PH = PH; a->PWU = PWU;
            *lds_out = lds;
        }
    }
    return found;
}

static bool plan_igemm(const Geometry &g, bool with_ws, bool x_al4, bool w_al16, int forced_variant,
                       bool force_split, Plan *pl)
{
    int nv = 0;
    const IgemmVariant *vs = igemm_variants(&nv);
    const int want_xvec = (g.W % 2 == 0 && x_al4) ? 2 : 1;
    const int want_cal = (g.Cg % 8 == 0 && w_al16) ? 1 : 0;
    const IgemmVariant *pick = nullptr;
    if (forced_variant >= 0) {
        if (forced_variant >= nv) return false;
        const IgemmVariant &v = vs[forced_variant];
        if (v.ks != g.k) return false;
        if (v.xvec == 2 && want_xvec != 2) return false;
        if (v.calign && !want_cal) return false;
        pick = &v;
    } else {
        for (int i = 0; i < nv; ++i) {
            const IgemmVariant &v = vs[i];
            if (v.ks != g.k || v.xvec != want_xvec || v.calign != want_cal) continue;
            if (!pick) { pick = &v; continue; }
            // prefer the tile with less channel padding; ties go to the larger tile
            const long long pad_new = (long long)ceil_div(g.Mg, v.BM()) * v.BM();
            const long long pad_old = (long long)ceil_div(g.Mg, pick->BM()) * pick->BM();
            if (pad_new < pad_old) pick = &v;
        }
    }
    if (!pick) return false;
    ConvArgs *a = &pl->args;
    long long lds = 0;
    if (!choose_window(g, *pick, a, &lds)) return false;
    a->tiles_m = ceil_div(g.Mg, pick->BM());
    a->nsteps = ceil_div(g.Cg, 8 * pick->npl);
    long long grid = (long long)a->tiles_m * a->tiles_w * a->tiles_h * g.G * g.N;
    int split = 1;
    if (with_ws && a->nsteps >= 2) {
        // too few workgroups for 256 CUs: slice the channel blocks
        if (grid < 192 || force_split) {
            split = (int)((384 + grid - 1) / grid);
            if (split > a->nsteps) split = a->nsteps;
            if (split > 32) split = 32;
            if (force_split && split < 2) split = 2;
        }
    }
    a->steps_per_split = ceil_div(a->nsteps, split);
    a->split_k = ceil_div(a->nsteps, a->steps_per_split);
    if (grid * a->split_k > INT_MAX) return false;
    pl->variant = pick;
    pl->pub.path = a->split_k > 1 ? HGC_PATH_IGEMM_SPLITK : HGC_PATH_IGEMM;
    pl->pub.tile_m = pick->BM();
    pl->pub.tile_w = 1 << a->log2_tw;
    pl->pub.tile_h = pick->BN() >> a->log2_tw;
    pl->pub.split_k = a->split_k;
    pl->pub.variant = (int)(pick - vs);
    pl->pub.grid = (int)(grid * a->split_k);
    pl->pub.block = 256;
    pl->pub.lds_bytes = lds;
    pl->pub.workspace_bytes =
        a->split_k > 1 ? 4LL * a->split_k * g.N * g.M * g.Ho * g.Wo : 0;
    return true;
}

static void make_plan(const Geometry &g, bool with_ws, bool x_al4, bool w_al16, Plan *pl)
{
    std::memset(pl, 0, sizeof(*pl));
    base_args(g, &pl->args);
    pl->pub.Ho = g.Ho; pl->pub.Wo = g.Wo;
    pl->pub.split_k = 1;
    const int forced = g_forced_path.load(std::memory_order_relaxed);
    const int fvar = g_forced_variant.load(std::memory_order_relaxed);
    const bool depthwise_ok = (g.G == g.C && g.M == g.C && (g.k == 3 || g.k == 5));

    int path = forced;
    if (path == HGC_PATH_AUTO) {
        if (depthwise_ok) path = HGC_PATH_DEPTHWISE;
        else if (g.Mg >= 16) path = HGC_PATH_IGEMM;
        else path = HGC_PATH_DIRECT;
    }
    if (path == HGC_PATH_DEPTHWISE && depthwise_ok) {
        pl->pub.path = HGC_PATH_DEPTHWISE;
        pl->pub.block = 256;
        pl->pub.grid = (int)std::min<long long>(1048576, (long long)g.N * g.C * ceil_div(g.Ho * g.Wo, 256));
        return;
    }
    if (path == HGC_PATH_IGEMM || path == HGC_PATH_IGEMM_SPLITK) {
        const bool ws = with_ws && (forced != HGC_PATH_IGEMM);
        if (plan_igemm(g, ws, x_al4, w_al16, fvar, forced == HGC_PATH_IGEMM_SPLITK && with_ws, pl))
            return;
        base_args(g, &pl->args);
    }
    pl->pub.path = HGC_PATH_DIRECT;
    pl->pub.block = 256;
    pl->pub.grid = (int)std::min<long long>(1048576, ((long long)g.N * g.M * g.Ho * g.Wo + 255) / 256);
}

static hgc_status run(const hgc_conv2d_desc *desc, const void *x, const void *w, const void *b,
                      void *y, void *ws, size_t ws_bytes, bool with_ws, void *stream)
{
    if (!desc || !x || !w || !y) return HGC_ERR_NULL;
    if (desc->bias == 1 && !b) return HGC_ERR_NULL;
    Geometry g;
    hgc_status st = validate(desc, &g);
    if (st != HGC_OK) return st;
    Plan pl;
    const bool x_al4 = ((uintptr_t)x & 3) == 0;
    const bool w_al16 = ((uintptr_t)w & 15) == 0;
    make_plan(g, with_ws, x_al4, w_al16, &pl);
    if (pl.pub.workspace_bytes > 0) {
        // the size reported to the caller assumed aligned tensors; an unaligned call
        // may need the same or less, never more (same tiles, same split rule)
        if (!ws || (long long)ws_bytes < pl.pub.workspace_bytes) return HGC_ERR_WORKSPACE;
    }
    ConvArgs &a = pl.args;
    a.x = static_cast<const uint16_t *>(x);
    a.w = static_cast<const uint16_t *>(w);
    a.b = static_cast<const uint16_t *>(b);
    a.y = static_cast<uint16_t *>(y);
    a.ws = static_cast<float *>(ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipError_t e;
    switch (pl.pub.path) {
    case HGC_PATH_DEPTHWISE:
        e = launch_depthwise(a, s);
        break;
    case HGC_PATH_IGEMM:
    case HGC_PATH_IGEMM_SPLITK:
        e = pl.variant->launch(a, dim3((unsigned)pl.pub.grid), s);
        if (e == hipSuccess && a.split_k > 1) e = launch_splitk_reduce(a, s);
        break;
    default:
        e = launch_direct(a, s);
        break;
    }
    g_last_hip_error = (int)e;
    return e == hipSuccess ? HGC_OK : HGC_ERR_LAUNCH;
}

}  // namespace hgc

using namespace hgc;

extern "C" {

hgc_status hgc_conv2d_forward(const hgc_conv2d_desc *desc, const void *x, const void *w,
                              const void *b, void *y, void *stream)
{
    return run(desc, x, w, b, y, nullptr, 0, false, stream);
}

hgc_status hgc_conv2d_forward_ws(const hgc_conv2d_desc *desc, const void *x, const void *w,
                                 const void *b, void *y, void *workspace, size_t workspace_bytes,
                                 void *stream)
{
    return run(desc, x, w, b, y, workspace, workspace_bytes, true, stream);
}

hgc_status hgc_conv2d_workspace_size(const hgc_conv2d_desc *desc, size_t *bytes_out)
{
    if (!desc || !bytes_out) return HGC_ERR_NULL;
    Geometry g;
    hgc_status st = validate(desc, &g);
    if (st != HGC_OK) return st;
    Plan pl;
    make_plan(g, true, true, true, &pl);
    long long need = pl.pub.workspace_bytes;
    // an unaligned tensor base selects a different instantiation with its own tiles
    Plan alt;
    make_plan(g, true, false, false, &alt);
    if (alt.pub.workspace_bytes > need) need = alt.pub.workspace_bytes;
    make_plan(g, true, true, false, &alt);
    if (alt.pub.workspace_bytes > need) need = alt.pub.workspace_bytes;
    make_plan(g, true, false, true, &alt);
    if (alt.pub.workspace_bytes > need) need = alt.pub.workspace_bytes;
    *bytes_out = (size_t)need;
    return HGC_OK;
}

hgc_status hgc_conv2d_plan(const hgc_conv2d_desc *desc, int32_t with_workspace, hgc_plan *plan_out)
{
    if (!desc || !plan_out) return HGC_ERR_NULL;
    Geometry g;
    hgc_status st = validate(desc, &g);
    if (st != HGC_OK) return st;
    Plan pl;
    make_plan(g, with_workspace != 0, true, true, &pl);
    *plan_out = pl.pub;
    return HGC_OK;
}

int32_t hgc_set_forced_path(int32_t path, int32_t tile_variant)
{
    if (path < HGC_PATH_AUTO || path > HGC_PATH_DEPTHWISE) path = HGC_PATH_AUTO;
    g_forced_variant.store(tile_variant, std::memory_order_relaxed);
    return g_forced_path.exchange(path, std::memory_order_relaxed);
}

const char *hgc_status_string(hgc_status status)
{
    switch (status) {
    case HGC_OK: return "ok";
    case HGC_ERR_NULL: return "a required pointer is NULL";
    case HGC_ERR_BAD_DESC: return "descriptor field out of range or empty output";
    case HGC_ERR_TOO_LARGE: return "a tensor has more than 2^31-1 elements";
    case HGC_ERR_WORKSPACE: return "workspace missing or too small";
    case HGC_ERR_LAUNCH: return "HIP launch failed";
    default: return "unknown status";
    }
}

int32_t hgc_version(void) { return 100; }

const char *hgc_last_launch_error(void)
{
    return hipGetErrorString((hipError_t)g_last_hip_error);
}

}  // extern "C"
