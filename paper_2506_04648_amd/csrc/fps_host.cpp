// Host side of libfps: argument validation, error text, the step-aware schedule (Eq. 6), the host
// statement of the tile neighbourhood (Eq. 2), and the extern "C" entry points that forward to
// the kernel launchers.
#include "fps_internal.h"

#include <stdio.h>
#include <string.h>

namespace fps {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int hip_fail(hipError_t e, const char* what) {
    set_error("%s: %s", what, hipGetErrorString(e));
    return FPS_ERR_HIP;
}

int check_ptr(const void* p, const char* name) {
    if (!p) { set_error("%s is NULL", name); return FPS_ERR_INVALID_ARG; }
    if (reinterpret_cast<uintptr_t>(p) & 15u) {
        set_error("%s is not 16-byte aligned", name);
        return FPS_ERR_INVALID_ARG;
    }
    return FPS_OK;
}

int check_shape(const fps_shape* s, Geom* g) {
    if (!s) { set_error("shape is NULL"); return FPS_ERR_INVALID_ARG; }
    if (s->B <= 0 || s->heads <= 0 || s->T <= 0 || s->H <= 0 || s->W <= 0 || s->Tt <= 0 ||
        s->Th <= 0 || s->Tw <= 0 || s->head_dim <= 0) {
        set_error("shape has a non-positive dimension");
        return FPS_ERR_INVALID_ARG;
    }
    const long long bh = (long long)s->B * s->heads;
    const long long ts = (long long)s->Tt * s->Th * s->Tw;
    const int nT = (s->T + s->Tt - 1) / s->Tt, nH = (s->H + s->Th - 1) / s->Th,
              nW = (s->W + s->Tw - 1) / s->Tw;
    const long long m = (long long)nT * nH * nW;
    if (s->head_dim != kHeadDim) {
        set_error("head_dim %d unsupported (only 128)", s->head_dim);
        return FPS_ERR_UNSUPPORTED;
    }
    if (ts > kMaxTileTokens) {
        set_error("tile of %lld tokens unsupported (at most %d)", ts, kMaxTileTokens);
        return FPS_ERR_UNSUPPORTED;
    }
    int qt = s->Qt, qh = s->Qh, qw = s->Qw;
    if (qt == 0 && qh == 0 && qw == 0) { qt = s->Tt; qh = s->Th; qw = s->Tw; }
    if (qt <= 0 || qh <= 0 || qw <= 0 || s->Tt % qt || s->Th % qh || s->Tw % qw) {
        set_error("quantisation sub-tile (%d,%d,%d) must be all zero or divide the tile (%d,%d,%d)",
                  s->Qt, s->Qh, s->Qw, s->Tt, s->Th, s->Tw);
        return FPS_ERR_INVALID_ARG;
    }
    const int qs = qt * qh * qw;
    const int ns = (s->Tt / qt) * (s->Th / qh) * (s->Tw / qw);
    // 32-slot blocks when they waste fewer slots than 128-slot blocks (sub-tiles of <= 96 tokens)
    const int bs = (qs <= 128 && (qs + 31) / 32 * 32 < 128) ? 32 : 128;
    const int kbs = (qs + bs - 1) / bs;
    const long long kb = (long long)ns * kbs;
    if (kb * bs > 4LL * kMaxTileTokens) {
        set_error("tile of %lld slots after padding its %d sub-tiles to whole blocks is too large", kb * bs, ns);
        return FPS_ERR_UNSUPPORTED;
    }
    if (bh > (1 << 20) || m > (1 << 20) || bh * m * kb >= (1LL << 30)) {
        set_error("shape too large (B*heads*M*blocks-per-tile must stay below 2^30)");
        return FPS_ERR_INVALID_ARG;
    }
    if (!g) return FPS_OK;
    g->BH = (int)bh;
    g->T = s->T; g->H = s->H; g->W = s->W;
    g->Tt = s->Tt; g->Th = s->Th; g->Tw = s->Tw;
    g->nT = nT; g->nH = nH; g->nW = nW;
    g->M = (int)m; g->TS = (int)ts;
    g->Qt = qt; g->Qh = qh; g->Qw = qw;
    g->nsT = s->Tt / qt; g->nsH = s->Th / qh; g->nsW = s->Tw / qw;
    g->NS = ns; g->QS = qs;
    g->inv_qplane = 1.0f / (float)(qh * qw);
    g->inv_qw = 1.0f / (float)qw;
    g->BS = bs; g->KBS = kbs; g->QSP = kbs * bs; g->KB = (int)kb; g->TSP = (int)kb * bs;
    g->lastT = s->T - (nT - 1) * s->Tt;
    g->lastH = s->H - (nH - 1) * s->Th;
    g->lastW = s->W - (nW - 1) * s->Tw;
    // sub-tile layers along t that hold a real plane of a last-along-T tile; within the last such
    // layer the padding-only blocks form a suffix only if the layer is a single sub-tile
    const int layers = (g->lastT + qt - 1) / qt;
    if (g->nsH * g->nsW == 1)
        g->kb_last = (layers - 1) * kbs + ((g->lastT - (layers - 1) * qt) * qh * qw + bs - 1) / bs;
    else
        g->kb_last = layers * g->nsH * g->nsW * kbs;
    return FPS_OK;
}

static int check_window(const fps_window* w) {
    if (!w) { set_error("window is NULL"); return FPS_ERR_INVALID_ARG; }
    if (w->wt <= 0 || w->wh <= 0 || w->ww <= 0) {
        set_error("window sizes must be positive");
        return FPS_ERR_INVALID_ARG;
    }
    if (w->edge != FPS_EDGE_TRUNCATE && w->edge != FPS_EDGE_SHIFT) {
        set_error("window.edge has invalid value %d", (int)w->edge);
        return FPS_ERR_INVALID_ARG;
    }
    return FPS_OK;
}

static int check_enum(int v, int hi, const char* name) {
    if (v < 0 || v > hi) { set_error("%s has invalid value %d", name, v); return FPS_ERR_INVALID_ARG; }
    return FPS_OK;
}

}  // namespace fps

using namespace fps;

#define FPS_TRY(expr) do { int _rc = (expr); if (_rc != FPS_OK) return _rc; } while (0)

extern "C" {

const char* fps_last_error(void) { return g_err; }

int fps_schedule_select(const fps_step_cfg* cfg, fps_regime* out) {
    if (!cfg || !out) { set_error("cfg or out is NULL"); return FPS_ERR_INVALID_ARG; }
    if (cfg->num_steps <= 0 || cfg->step < 1 || cfg->step > cfg->num_steps) {
        set_error("step %d outside 1..%d", cfg->step, cfg->num_steps);
        return FPS_ERR_INVALID_ARG;
    }
    if (!(cfg->alpha1 > 0.f && cfg->alpha1 < cfg->alpha2 && cfg->alpha2 < 1.f)) {
        set_error("need 0 < alpha1 < alpha2 < 1");
        return FPS_ERR_INVALID_ARG;
    }
    for (int i = 0; i < 3; ++i) {
        FPS_TRY(check_enum(cfg->regime[i].prec, FPS_PREC_FP8, "regime.prec"));
        FPS_TRY(check_window(&cfg->regime[i].win));
        const fps_regime& r = cfg->regime[i];
        const bool none = r.Tt == 0 && r.Th == 0 && r.Tw == 0;
        if (!none && (r.Tt <= 0 || r.Th <= 0 || r.Tw <= 0)) {
            set_error("regime %d: tile (%d,%d,%d) must be all zero or all positive", i, r.Tt, r.Th, r.Tw);
            return FPS_ERR_INVALID_ARG;
        }
        const bool qnone = r.Qt == 0 && r.Qh == 0 && r.Qw == 0;
        if (!qnone && (r.Qt <= 0 || r.Qh <= 0 || r.Qw <= 0)) {
            set_error("regime %d: sub-tile (%d,%d,%d) must be all zero or all positive", i, r.Qt, r.Qh, r.Qw);
            return FPS_ERR_INVALID_ARG;
        }
    }
    const float t1 = cfg->alpha1 * (float)cfg->num_steps;
    const float t2 = cfg->alpha2 * (float)cfg->num_steps;
    const float t = (float)cfg->step;
    *out = cfg->regime[t <= t1 ? 0 : (t <= t2 ? 1 : 2)];
    return FPS_OK;
}

size_t fps_num_tiles(const fps_shape* shape) {
    Geom g;
    if (check_shape(shape, &g) != FPS_OK) return 0;
    return (size_t)g.M;
}

size_t fps_num_groups(const fps_shape* shape) {
    Geom g;
    if (check_shape(shape, &g) != FPS_OK) return 0;
    return (size_t)g.M * g.NS;
}

size_t fps_tile_slots(const fps_shape* shape) {
    Geom g;
    if (check_shape(shape, &g) != FPS_OK) return 0;
    return (size_t)g.TSP;
}

size_t fps_block_slots(const fps_shape* shape) {
    Geom g;
    if (check_shape(shape, &g) != FPS_OK) return 0;
    return (size_t)g.BS;
}

size_t fps_packed_bytes(const fps_shape* shape, fps_precision prec) {
    Geom g;
    if (check_shape(shape, &g) != FPS_OK) return 0;
    if (check_enum(prec, FPS_PREC_FP8, "prec") != FPS_OK) return 0;
    const size_t n = (size_t)g.BH * g.M * g.TSP * kHeadDim;
    return prec == FPS_PREC_FP8 ? n : 2 * n;
}

int fps_tile_mask_host(const fps_shape* shape, const fps_window* win, uint8_t* mask,
                       uint64_t* pairs_or_null) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_window(win));
    if (!mask) { set_error("mask is NULL"); return FPS_ERR_INVALID_ARG; }
    const int rt = win->wt / 2, rh = win->wh / 2, rw = win->ww / 2;
    const bool shift = win->edge == FPS_EDGE_SHIFT;
    // kept range [lo, hi] along one axis
    auto lo_of = [shift](int u, int r, int n) {
        if (!shift) return u - r > 0 ? u - r : 0;
        if (n <= 2 * r + 1) return 0;
        const int c = u < r ? r : (u > n - 1 - r ? n - 1 - r : u);
        return c - r;
    };
    auto hi_of = [shift](int u, int r, int n) {
        if (!shift) return u + r < n - 1 ? u + r : n - 1;
        if (n <= 2 * r + 1) return n - 1;
        const int c = u < r ? r : (u > n - 1 - r ? n - 1 - r : u);
        return c + r;
    };
    uint64_t pairs = 0;
    for (int u = 0; u < g.M; ++u) {
        const int uw = u % g.nW, uh = (u / g.nW) % g.nH, ut = u / (g.nW * g.nH);
        for (int v = 0; v < g.M; ++v) {
            const int vw = v % g.nW, vh = (v / g.nW) % g.nH, vt = v / (g.nW * g.nH);
            const uint8_t keep = (vt >= lo_of(ut, rt, g.nT) && vt <= hi_of(ut, rt, g.nT) &&
                                  vh >= lo_of(uh, rh, g.nH) && vh <= hi_of(uh, rh, g.nH) &&
                                  vw >= lo_of(uw, rw, g.nW) && vw <= hi_of(uw, rw, g.nW)) ? 1 : 0;
            mask[(size_t)u * g.M + v] = keep;
            pairs += keep;
        }
    }
    if (pairs_or_null) *pairs_or_null = pairs;
    return FPS_OK;
}

int fps_tile_order(const fps_shape* shape, const void* x_raster_bf16, void* x_tiled_bf16,
                   void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_ptr(x_raster_bf16, "x_raster_bf16"));
    FPS_TRY(check_ptr(x_tiled_bf16, "x_tiled_bf16"));
    return launch_tile_order(g, x_raster_bf16, x_tiled_bf16, (hipStream_t)stream);
}

int fps_tile_unorder(const fps_shape* shape, const void* o_tiled, fps_out_dtype dt, void* o_raster,
                     void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(dt, FPS_OUT_F32, "dt"));
    FPS_TRY(check_ptr(o_tiled, "o_tiled"));
    FPS_TRY(check_ptr(o_raster, "o_raster"));
    return launch_tile_unorder(g, o_tiled, dt == FPS_OUT_F32 ? 4 : 2, o_raster,
                               (hipStream_t)stream);
}

int fps_quantize_tiles(const fps_shape* shape, const void* x_tiled_bf16, fps_role role,
                       fps_vscale vscale, void* xq_out, float* scales_out, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(role, FPS_ROLE_V, "role"));
    FPS_TRY(check_enum(vscale, FPS_VSCALE_CHANNEL, "vscale"));
    FPS_TRY(check_ptr(x_tiled_bf16, "x_tiled_bf16"));
    FPS_TRY(check_ptr(xq_out, "xq_out"));
    FPS_TRY(check_ptr(scales_out, "scales_out"));
    const int vs = role == FPS_ROLE_V ? (int)vscale : (int)FPS_VSCALE_TILE;
    return launch_quantize(g, x_tiled_bf16, 0, role, vs, xq_out, scales_out, (hipStream_t)stream);
}

int fps_quantize_raster(const fps_shape* shape, const void* x_raster_bf16, fps_role role,
                        fps_vscale vscale, void* xq_out, float* scales_out, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(role, FPS_ROLE_V, "role"));
    FPS_TRY(check_enum(vscale, FPS_VSCALE_CHANNEL, "vscale"));
    FPS_TRY(check_ptr(x_raster_bf16, "x_raster_bf16"));
    FPS_TRY(check_ptr(xq_out, "xq_out"));
    FPS_TRY(check_ptr(scales_out, "scales_out"));
    const int vs = role == FPS_ROLE_V ? (int)vscale : (int)FPS_VSCALE_TILE;
    return launch_quantize(g, x_raster_bf16, 1, role, vs, xq_out, scales_out, (hipStream_t)stream);
}

int fps_pack_tiles_bf16(const fps_shape* shape, const void* x_tiled_bf16, fps_role role,
                        void* xp_out, float* vscale_out, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(role, FPS_ROLE_V, "role"));
    FPS_TRY(check_ptr(x_tiled_bf16, "x_tiled_bf16"));
    FPS_TRY(check_ptr(xp_out, "xp_out"));
    if (role == FPS_ROLE_V) FPS_TRY(check_ptr(vscale_out, "vscale_out"));
    return launch_pack_bf16(g, x_tiled_bf16, 0, role, xp_out, vscale_out, (hipStream_t)stream);
}

int fps_pack_raster_bf16(const fps_shape* shape, const void* x_raster_bf16, fps_role role,
                         void* xp_out, float* vscale_out, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(role, FPS_ROLE_V, "role"));
    FPS_TRY(check_ptr(x_raster_bf16, "x_raster_bf16"));
    FPS_TRY(check_ptr(xp_out, "xp_out"));
    if (role == FPS_ROLE_V) FPS_TRY(check_ptr(vscale_out, "vscale_out"));
    return launch_pack_bf16(g, x_raster_bf16, 1, role, xp_out, vscale_out, (hipStream_t)stream);
}

int fps_debug_unpack_q8(const fps_shape* shape, const void* xq, fps_role role,
                        uint8_t* codes_rowmajor, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_enum(role, FPS_ROLE_V, "role"));
    FPS_TRY(check_ptr(xq, "xq"));
    FPS_TRY(check_ptr(codes_rowmajor, "codes_rowmajor"));
    return launch_unpack_q8(g, xq, role, codes_rowmajor, (hipStream_t)stream);
}

int fps_debug_copy(const void* src, void* dst, size_t bytes, void* stream) {
    FPS_TRY(check_ptr(src, "src"));
    FPS_TRY(check_ptr(dst, "dst"));
    if (bytes == 0 || (bytes & 15u) || bytes > ((size_t)1 << 40)) {
        set_error("bytes must be a positive multiple of 16");
        return FPS_ERR_INVALID_ARG;
    }
    return launch_copy(src, dst, (long long)bytes, (hipStream_t)stream);
}

int fps_debug_mfma_rate(int workgroups, int iters, float* sink, void* stream) {
    FPS_TRY(check_ptr(sink, "sink"));
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24)) {
        set_error("workgroups must be in 1..2^20 and iters in 1..2^24");
        return FPS_ERR_INVALID_ARG;
    }
    return launch_mfma_rate(workgroups, iters, sink, (hipStream_t)stream);
}

int fps_debug_issue_mix(int matrix_kind, int valu_per_mfma, int valu_kind, int workgroups_per_cu,
                        int workgroups, int iters, float* sink, unsigned long long* cycles,
                        void* stream) {
    FPS_TRY(check_ptr(sink, "sink"));
    FPS_TRY(check_ptr(cycles, "cycles"));
    if (matrix_kind < 0 || matrix_kind > 4 || valu_kind < 0 || valu_kind > 1) {
        set_error("matrix_kind must be 0 (E4M3 16x16x128), 1 (bf16 16x16x32), 2 (none), 3 (E4M3 32x32x64) or 4 (bf16 32x32x16); valu_kind 0 (fma) or 1 (exp2)");
        return FPS_ERR_INVALID_ARG;
    }
    if (workgroups_per_cu < 1 || workgroups_per_cu > 8) {
        set_error("workgroups_per_cu must be in 1..8");
        return FPS_ERR_INVALID_ARG;
    }
    if (workgroups <= 0 || workgroups > (1 << 20) || iters <= 0 || iters > (1 << 24)) {
        set_error("workgroups must be in 1..2^20 and iters in 1..2^24");
        return FPS_ERR_INVALID_ARG;
    }
    return launch_issue_mix(matrix_kind, valu_per_mfma, valu_kind, workgroups_per_cu, workgroups, iters,
                            sink, cycles, (hipStream_t)stream);
}

int fps_debug_scores_q8(const fps_shape* shape, const void* q, const void* k, int bh, int u, int v,
                        float* scores, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_ptr(q, "q"));
    FPS_TRY(check_ptr(k, "k"));
    FPS_TRY(check_ptr(scores, "scores"));
    if (bh < 0 || bh >= g.BH || u < 0 || u >= g.M || v < 0 || v >= g.M) {
        set_error("bh/u/v out of range");
        return FPS_ERR_INVALID_ARG;
    }
    if (g.TSP > kMaxScoreSlots) {
        set_error("score debug call refused for tiles of more than %d slots", kMaxScoreSlots);
        return FPS_ERR_UNSUPPORTED;
    }
    return launch_scores_fp8(g, q, k, bh, u, v, scores, (hipStream_t)stream);
}

int fps_debug_scores_block_q8(const fps_shape* shape, const void* q, const void* k, int bh, int u,
                              int jq, int v, int jk, float* scores, int* bs_or_null, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    FPS_TRY(check_ptr(q, "q"));
    FPS_TRY(check_ptr(k, "k"));
    FPS_TRY(check_ptr(scores, "scores"));
    if (bh < 0 || bh >= g.BH || u < 0 || u >= g.M || v < 0 || v >= g.M || jq < 0 || jq >= g.KB ||
        jk < 0 || jk >= g.KB) {
        set_error("bh/u/v/jq/jk out of range");
        return FPS_ERR_INVALID_ARG;
    }
    if (bs_or_null) *bs_or_null = g.BS;
    return launch_scores_block_fp8(g, q, k, bh, u, jq, v, jk, scores, (hipStream_t)stream);
}

int fps_attn_fwd(const fps_shape* shape, const fps_window* win, fps_precision prec,
                 const fps_step_cfg* step, const void* q, const void* k, const void* v,
                 const float* sq, const float* sk, const float* sv, fps_vscale vscale, void* out,
                 fps_out_dtype out_dt, fps_layout out_layout, uint8_t* visited, void* stream) {
    Geom g;
    FPS_TRY(check_shape(shape, &g));
    fps_regime sel;
    if (step) {
        FPS_TRY(fps_schedule_select(step, &sel));
        if (sel.Tt != 0 && (sel.Tt != shape->Tt || sel.Th != shape->Th || sel.Tw != shape->Tw)) {
            set_error("step %d selects tile (%d,%d,%d) but the shape of the call has (%d,%d,%d)",
                      step->step, sel.Tt, sel.Th, sel.Tw, shape->Tt, shape->Th, shape->Tw);
            return FPS_ERR_INVALID_ARG;
        }
        if (sel.Qt != 0 && (sel.Qt != g.Qt || sel.Qh != g.Qh || sel.Qw != g.Qw)) {
            set_error("step %d selects sub-tile (%d,%d,%d) but the shape of the call has (%d,%d,%d)",
                      step->step, sel.Qt, sel.Qh, sel.Qw, g.Qt, g.Qh, g.Qw);
            return FPS_ERR_INVALID_ARG;
        }
    } else {
        FPS_TRY(check_window(win));
        FPS_TRY(check_enum(prec, FPS_PREC_FP8, "prec"));
        sel.prec = prec;
        sel.win = *win;
        sel.Tt = sel.Th = sel.Tw = 0;
        sel.Qt = sel.Qh = sel.Qw = 0;
    }
    FPS_TRY(check_enum(vscale, FPS_VSCALE_CHANNEL, "vscale"));
    FPS_TRY(check_enum(out_dt, FPS_OUT_F32, "out_dt"));
    FPS_TRY(check_enum(out_layout, FPS_LAYOUT_RASTER, "out_layout"));
    FPS_TRY(check_ptr(q, "q"));
    FPS_TRY(check_ptr(k, "k"));
    FPS_TRY(check_ptr(v, "v"));
    FPS_TRY(check_ptr(out, "out"));
    if (sel.prec == FPS_PREC_FP8) {
        FPS_TRY(check_ptr(sq, "sq"));
        FPS_TRY(check_ptr(sk, "sk"));
    }
    FPS_TRY(check_ptr(sv, "sv"));
    return launch_attn(g, sel.win, sel.prec, q, k, v, sq, sk, sv, vscale, out,
                       out_dt == FPS_OUT_F32, out_layout == FPS_LAYOUT_RASTER, visited,
                       (hipStream_t)stream);
}

}  // extern "C"
