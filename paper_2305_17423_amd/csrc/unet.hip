// Masked UNet step: host-side plan (module walk, flat weight / cache / context
// layouts) and the launch sequence.  Every module is a short chain of the gathered
// GEMM, row LayerNorm and active-query attention kernels, all enqueued on the
// caller's stream; nothing here allocates or synchronises.
#include <algorithm>
#include <cmath>
#include <map>
#include <string>
#include <vector>
#include "igemm.h"

namespace fise {
IgemmArgs linear_args(const void* A, int rows_per_b, int B, int Cin, const void* W, const void* bias, int N);
int run_conv(const void* a0, int C0, int B, int Hin, int Win, int stride, int ups, const void* w, const void* bias, int N,
             const int* idx, int n_active, int tile, void* out, const IgemmWorkspace* iw, hipStream_t st, const GnView* views,
             int nview);
int run_resnet(const fise_resnet_args* a, void* ws, const IgemmWorkspace* iw, hipStream_t st, const BlockDerived* dv);
int run_transformer(const fise_transformer_args* a, void* workspace, const IgemmWorkspace* iw, hipStream_t st, const BlockDerived* dv);
size_t resnet_ws_bytes(const fise_resnet_args* a);
size_t transformer_ws_bytes(const fise_transformer_args* a);
}

using namespace fise;

namespace {
// One pixel-addressed cache tensor for the cache-moving kernels.  rows: [B, H*W, row_bytes] (a map, or K);
// vt: [B, C, H*W] two-byte elements (V transposed).
struct MoveEntry { long long off; int row_bytes; short lvl; short vt; };
struct Tensor { std::string name; int64_t off; int64_t numel; };
enum Kind { K_CONV_IN, K_RES, K_TR, K_DS, K_US, K_OUT };
// A consumer of a module's output map that normalises it first: consumer module, and whether the map is the
// consumer's skip source (second part of the channel concatenation).
struct ViewSpec { int consumer; bool as_skip; };
struct Module {
    Kind kind; std::string name; int lvl; int cin, cskip, cout;   // tr/ds/us: cin == cout == c
    std::string in_map, skip_map;                                 // cache tensors read ("" = latent)
    int temb_off;                                                 // column offset in the stacked time projection
    std::vector<ViewSpec> views;                                  // who wants this module's output normalised
};
}  // namespace

struct fise_unet {
    fise_unet_desc d;
    std::vector<Module> mods;
    std::vector<Tensor> tensors[4];                  // 0 weights, 1 stored cache tensors, 2 context K/V, 3 derived cache tensors
    std::map<std::string, int> index[4];
    int64_t weight_elems = 0; size_t cache_bytes = 0, ctxkv_bytes = 0;
    int temb_total = 0, n_stride = 0;
    fise_unet_cache_layout layout{};                 // byte ranges of the groups of cache tensors
    std::vector<MoveEntry> move_maps, move_k, move_vt;   // pixel-addressed tensors of the stored part, by group

    int64_t add(int kind, const std::string& name, int64_t numel, int64_t& cursor, int64_t align) {
        cursor = (cursor + align - 1) / align * align;
        index[kind][name] = (int)tensors[kind].size();
        tensors[kind].push_back({name, cursor, numel});
        const int64_t off = cursor; cursor += numel;
        return off;
    }
    int64_t off(int kind, const std::string& name) const { return tensors[kind][index[kind].at(name)].off; }
};

static void build_plan(fise_unet* u) {
    const fise_unet_desc& d = u->d;
    const int nl = d.n_levels, L = d.layers, base = d.base, te = 4 * base;
    std::vector<Module>& mods = u->mods;
    std::vector<std::pair<std::string, int>> skips;
    auto S = [](const char* fmt, int a, int b = 0) { char buf[64]; snprintf(buf, sizeof buf, fmt, a, b); return std::string(buf); };
    mods.push_back({K_CONV_IN, "conv_in", 0, d.in_ch, 0, base, "", "", 0});
    std::string cur = "conv_in.out";
    skips.push_back({cur, base});
    int ch = base;
    for (int l = 0; l < nl; ++l) {
        const int co = base * d.mults[l];
        for (int i = 0; i < L; ++i) {
            std::string n = S("down.%d.res.%d", l, i);
            mods.push_back({K_RES, n, l, ch, 0, co, cur, "", 0});
            ch = co; cur = n + ".out";
            if (d.attn[l]) { n = S("down.%d.tr.%d", l, i); mods.push_back({K_TR, n, l, ch, 0, ch, cur, "", 0}); cur = n + ".out"; }
            skips.push_back({cur, ch});
        }
        if (l != nl - 1) {
            std::string n = S("down.%d.ds", l);
            mods.push_back({K_DS, n, l + 1, ch, 0, ch, cur, "", 0});
            cur = n + ".out"; skips.push_back({cur, ch});
        }
    }
    const int lb = nl - 1;
    mods.push_back({K_RES, "mid.res.0", lb, ch, 0, ch, cur, "", 0}); cur = "mid.res.0.out";
    mods.push_back({K_TR, "mid.tr.0", lb, ch, 0, ch, cur, "", 0}); cur = "mid.tr.0.out";
    mods.push_back({K_RES, "mid.res.1", lb, ch, 0, ch, cur, "", 0}); cur = "mid.res.1.out";
    for (int j = 0; j < nl; ++j) {
        const int l = nl - 1 - j, co = base * d.mults[l];
        for (int i = 0; i <= L; ++i) {
            auto sk = skips.back(); skips.pop_back();
            std::string n = S("up.%d.res.%d", j, i);
            mods.push_back({K_RES, n, l, ch, sk.second, co, cur, sk.first, 0});
            ch = co; cur = n + ".out";
            if (d.attn[l]) { n = S("up.%d.tr.%d", j, i); mods.push_back({K_TR, n, l, ch, 0, ch, cur, "", 0}); cur = n + ".out"; }
        }
        if (l != 0) { std::string n = S("up.%d.us", j); mods.push_back({K_US, n, l - 1, ch, 0, ch, cur, "", 0}); cur = n + ".out"; }
    }
    mods.push_back({K_OUT, "out", 0, ch, 0, d.out_ch, cur, "", 0});

    // ---- weights (bf16 elements, every tensor 8-element aligned).  The time projections of all
    // ResNet blocks are stacked into one [sum C_out, te] matrix so one launch serves the step.
    int64_t wc = 0;
    u->add(0, "time.l1.w", (int64_t)te * base, wc, 8); u->add(0, "time.l1.b", te, wc, 8);
    u->add(0, "time.l2.w", (int64_t)te * te, wc, 8);   u->add(0, "time.l2.b", te, wc, 8);
    int toff = 0;
    for (Module& m : mods) if (m.kind == K_RES) { m.temb_off = toff; u->add(0, m.name + ".temb.w", (int64_t)m.cout * te, wc, 8); toff += m.cout; }
    u->temb_total = toff;
    for (Module& m : mods) if (m.kind == K_RES) u->add(0, m.name + ".temb.b", m.cout, wc, 8);
    for (const Module& m : mods) {
        const std::string& n = m.name;
        const int64_t ci = m.cin + m.cskip, co = m.cout, c = m.cout, cd = d.ctx_dim;
        switch (m.kind) {
        case K_CONV_IN: u->add(0, n + ".w", co * 9 * ci, wc, 8); u->add(0, n + ".b", co, wc, 8); break;
        case K_RES:
            u->add(0, n + ".gn1.g", ci, wc, 8); u->add(0, n + ".gn1.b", ci, wc, 8);
            u->add(0, n + ".conv1.w", co * 9 * ci, wc, 8); u->add(0, n + ".conv1.b", co, wc, 8);
            u->add(0, n + ".gn2.g", co, wc, 8); u->add(0, n + ".gn2.b", co, wc, 8);
            u->add(0, n + ".conv2.w", co * 9 * co, wc, 8); u->add(0, n + ".conv2.b", co, wc, 8);
            if (ci != co) { u->add(0, n + ".sc.w", co * ci, wc, 8); u->add(0, n + ".sc.b", co, wc, 8); }
            break;
        case K_TR:
            u->add(0, n + ".gn.g", c, wc, 8); u->add(0, n + ".gn.b", c, wc, 8);
            u->add(0, n + ".pin.w", c * c, wc, 8); u->add(0, n + ".pin.b", c, wc, 8);
            u->add(0, n + ".ln1.g", c, wc, 8); u->add(0, n + ".ln1.b", c, wc, 8);
            u->add(0, n + ".a1.q.w", c * c, wc, 8); u->add(0, n + ".a1.k.w", c * c, wc, 8); u->add(0, n + ".a1.v.w", c * c, wc, 8);
            u->add(0, n + ".a1.o.w", c * c, wc, 8); u->add(0, n + ".a1.o.b", c, wc, 8);
            u->add(0, n + ".ln2.g", c, wc, 8); u->add(0, n + ".ln2.b", c, wc, 8);
            u->add(0, n + ".a2.q.w", c * c, wc, 8); u->add(0, n + ".a2.k.w", c * cd, wc, 8); u->add(0, n + ".a2.v.w", c * cd, wc, 8);
            u->add(0, n + ".a2.o.w", c * c, wc, 8); u->add(0, n + ".a2.o.b", c, wc, 8);
            u->add(0, n + ".ln3.g", c, wc, 8); u->add(0, n + ".ln3.b", c, wc, 8);
            u->add(0, n + ".ff1.w", 8 * c * c, wc, 8); u->add(0, n + ".ff1.b", 8 * c, wc, 8);
            u->add(0, n + ".ff2.w", c * 4 * c, wc, 8); u->add(0, n + ".ff2.b", c, wc, 8);
            u->add(0, n + ".pout.w", c * c, wc, 8); u->add(0, n + ".pout.b", c, wc, 8);
            break;
        case K_DS: case K_US: u->add(0, n + ".w", c * 9 * c, wc, 8); u->add(0, n + ".b", c, wc, 8); break;
        case K_OUT:
            u->add(0, n + ".gn.g", ci, wc, 8); u->add(0, n + ".gn.b", ci, wc, 8);
            u->add(0, n + ".conv.w", co * 9 * ci, wc, 8); u->add(0, n + ".conv.b", co, wc, 8);
            break;
        }
    }
    u->weight_elems = (wc + 7) / 8 * 8;

    // ---- per-step cache (bytes, 256-byte aligned): maps bf16, statistics float.  Tensors are grouped so that each
    // group is one contiguous byte range: [stored maps][K, V^T][statistics][scale / shift tables][derived maps].
    // The first three groups are what the method stores, the last two are derived from them.
    int64_t cc = 0;
    const int64_t B = d.B, G = d.groups;
    auto HW = [&](const Module& m) { return (int64_t)(d.H >> m.lvl) * (d.W >> m.lvl); };
    auto map_entry = [&](int64_t off, const Module& m, int C) { u->move_maps.push_back({off, C * 2, (short)m.lvl, 0}); };
    for (const Module& m : mods) {
        const std::string& n = m.name;
        const int64_t hw = HW(m);
        if (m.kind == K_RES) map_entry(u->add(1, n + ".h1", B * hw * m.cout * 2, cc, 256), m, m.cout);
        map_entry(u->add(1, m.kind == K_OUT ? std::string("eps") : n + ".out", B * hw * m.cout * 2, cc, 256), m, m.cout);
    }
    u->layout.maps_off = 0; u->layout.maps_bytes = cc = (cc + 255) / 256 * 256;
    for (const Module& m : mods)
        if (m.kind == K_TR) {
            u->move_k.push_back({u->add(1, m.name + ".k", B * HW(m) * m.cout * 2, cc, 256), m.cout * 2, (short)m.lvl, 0});
            u->move_vt.push_back({u->add(1, m.name + ".v", B * HW(m) * m.cout * 2, cc, 256), m.cout, (short)m.lvl, 1});
        }
    cc = (cc + 255) / 256 * 256;
    u->layout.kv_off = u->layout.maps_bytes; u->layout.kv_bytes = cc - u->layout.kv_off;
    u->layout.small_off = cc;
    for (const Module& m : mods) {
        const std::string& n = m.name;
        auto stat = [&](const std::string& g) { u->add(1, n + "." + g + ".mean", B * G * 4, cc, 256); u->add(1, n + "." + g + ".rstd", B * G * 4, cc, 256); };
        if (m.kind == K_RES) { stat("gn1"); stat("gn2"); }
        else if (m.kind == K_TR || m.kind == K_OUT) stat("gn");
    }
    cc = (cc + 255) / 256 * 256;
    u->layout.stored_bytes = cc;
    // ---- derived tensors, in the same buffer behind the stored ones (bytes): what the masked step would otherwise
    // recompute from stored maps + cached statistics at every call.  ResNet: activated inputs of both convolutions
    // and the scale / shift tables of both GroupNorms; transformer: the normalised input of the 1x1 in and its table.
    for (const Module& m : mods) {
        const std::string& n = m.name;
        if (m.kind == K_RES) { u->add(3, n + ".gn1.ss", B * (m.cin + m.cskip) * 8, cc, 256);  u->add(3, n + ".gn2.ss", B * m.cout * 8, cc, 256); }
        else if (m.kind == K_TR) u->add(3, n + ".gn.ss", B * m.cout * 8, cc, 256);
    }
    cc = (cc + 255) / 256 * 256;
    u->layout.small_bytes = cc - u->layout.small_off;
    u->layout.derived_maps_off = cc;
    for (const Module& m : mods) {
        const std::string& n = m.name;
        const int64_t hw = HW(m), ci = m.cin + m.cskip;
        if (m.kind == K_RES) { u->add(3, n + ".a1", B * hw * ci * 2, cc, 256); u->add(3, n + ".a2", B * hw * m.cout * 2, cc, 256); }
        else if (m.kind == K_TR) u->add(3, n + ".gx", B * hw * m.cout * 2, cc, 256);
    }
    u->cache_bytes = (size_t)((cc + 255) / 256 * 256);
    u->layout.derived_maps_bytes = (int64_t)u->cache_bytes - u->layout.derived_maps_off;
    // ---- who normalises whose output
    std::map<std::string, int> producer;
    for (int i = 0; i < (int)mods.size(); ++i) producer[mods[i].kind == K_OUT ? std::string("eps") : mods[i].name + ".out"] = i;
    for (int i = 0; i < (int)mods.size(); ++i) {
        const Module& m = mods[i];
        if (m.kind != K_RES && m.kind != K_TR) continue;
        if (!m.in_map.empty()) mods[producer.at(m.in_map)].views.push_back({i, false});
        if (!m.skip_map.empty()) mods[producer.at(m.skip_map)].views.push_back({i, true});
    }

    // ---- context K/V (bytes): per transformer block K[B,n_ctx,C], Vt[B,C,n_stride]
    u->n_stride = (d.n_ctx + 7) / 8 * 8;
    int64_t kc = 0;
    for (const Module& m : mods)
        if (m.kind == K_TR) {
            u->add(2, m.name + ".ctx_k", B * d.n_ctx * m.cout * 2, kc, 256);
            u->add(2, m.name + ".ctx_vt", B * m.cout * u->n_stride * 2, kc, 256);
        }
    u->ctxkv_bytes = (size_t)((kc + 255) / 256 * 256);
}

extern "C" int fise_unet_create(const fise_unet_desc* desc, fise_unet** out) {
    if (!desc || !out) return fail(FISE_ERR_NULL, "fise_unet_create: null pointer");
    const fise_unet_desc& d = *desc;
    if (d.n_levels < 1 || d.n_levels > FISE_MAX_LEVELS || d.layers < 1 || d.B < 1 || d.in_ch < 1 || d.out_ch < 1)
        return fail(FISE_ERR_SHAPE, "fise_unet_create: bad levels/layers/batch");
    if (d.base < 32 || d.base % 32 || d.groups < 1 || d.heads < 1 || d.ctx_dim % 32 || d.ctx_dim < 32 || d.n_ctx < 1)
        return fail(FISE_ERR_SHAPE, "fise_unet_create: base and ctx_dim must be positive multiples of 32");
    if (d.H < 1 || d.W < 1 || d.H % (1 << (d.n_levels - 1)) || d.W % (1 << (d.n_levels - 1)))
        return fail(FISE_ERR_SHAPE, "fise_unet_create: H, W must be divisible by 2^(levels-1)");
    for (int l = 0; l < d.n_levels; ++l) {
        const int c = d.base * d.mults[l];
        if (d.mults[l] < 1 || c % d.groups || c % d.heads || (c / d.heads) % 8 || c / d.heads > 160)
            return fail(FISE_ERR_SHAPE, "fise_unet_create: level %d width %d vs groups %d / heads %d", l, c, d.groups, d.heads);
        if (d.attn[l] && ((d.H >> l) * (d.W >> l)) % 8) return fail(FISE_ERR_SHAPE, "fise_unet_create: level %d token count not a multiple of 8", l);
    }
    for (int l = 0; l + 1 < d.n_levels; ++l) {      // concatenated widths must keep whole groups
        (void)l;
    }
    fise_unet* u = new fise_unet();
    u->d = d;
    build_plan(u);
    for (const Module& m : u->mods) {
        if (m.kind == K_RES && (m.cin + m.cskip) % d.groups) { delete u; return fail(FISE_ERR_SHAPE, "fise_unet_create: %s input width %d %% groups", m.name.c_str(), m.cin + m.cskip); }
        if (m.views.size() > 2) { delete u; return fail(FISE_ERR_SHAPE, "fise_unet_create: %s feeds %zu normalising consumers", m.name.c_str(), m.views.size()); }
    }
    *out = u;
    return FISE_OK;
}

extern "C" void fise_unet_destroy(fise_unet* u) { delete u; }

extern "C" int fise_unet_desc_get(const fise_unet* u, fise_unet_desc* out) {
    if (!u || !out) return fail(FISE_ERR_NULL, "fise_unet_desc_get: null pointer");
    *out = u->d;
    return FISE_OK;
}

extern "C" int fise_unet_num_tensors(const fise_unet* u, int kind) {
    if (!u || kind < 0 || kind > 3) return fail(FISE_ERR_NULL, "fise_unet_num_tensors: bad arguments");
    return (int)u->tensors[kind].size();
}

extern "C" int fise_unet_tensor_info(const fise_unet* u, int kind, int i, char* name, int64_t* offset, int64_t* numel) {
    if (!u || !name || !offset || !numel) return fail(FISE_ERR_NULL, "fise_unet_tensor_info: null pointer");
    if (kind < 0 || kind > 3 || i < 0 || i >= (int)u->tensors[kind].size()) return fail(FISE_ERR_CAPACITY, "fise_unet_tensor_info: index");
    const Tensor& t = u->tensors[kind][i];
    snprintf(name, 64, "%s", t.name.c_str());
    *offset = t.off; *numel = t.numel;
    return FISE_OK;
}

extern "C" int64_t fise_unet_weight_elems(const fise_unet* u) { return u ? u->weight_elems : 0; }
extern "C" size_t fise_unet_cache_bytes(const fise_unet* u) { return u ? u->cache_bytes : 0; }
extern "C" size_t fise_unet_ctxkv_bytes(const fise_unet* u) { return u ? u->ctxkv_bytes : 0; }

namespace {
struct WsLayout { size_t idx_full, emb_a, emb_b, temb, block, igemm, total; };

// active tiles of level l: the caller's list, or every tile when the level runs dense
inline int level_tiles(const fise_unet_desc& d, int base_tile, int n_active, bool dense) {
    return dense ? (d.H / base_tile) * (d.W / base_tile) : n_active;
}

WsLayout ws_layout(const fise_unet* u, int n_tiles, int base_tile, const int* level_dense) {
    const fise_unet_desc& d = u->d;
    WsLayout w{};
    size_t c = 0;
    auto take = [&](size_t bytes) { size_t o = c; c += align256(bytes); return o; };
    const int tiles_total = (d.H / base_tile) * (d.W / base_tile);
    w.idx_full = take((size_t)tiles_total * 4);
    const int te = 4 * d.base;
    w.emb_a = take((size_t)d.B * te * 4); w.emb_b = take((size_t)d.B * te * 4);
    w.temb = take((size_t)d.B * u->temb_total * 4);
    size_t blk = 256;
    for (const Module& m : u->mods) {
        const bool dense = level_dense && level_dense[m.lvl];
        if (m.kind == K_TR) {
            fise_transformer_args t{};
            t.B = d.B; t.H = d.H >> m.lvl; t.W = d.W >> m.lvl; t.C = m.cout; t.G = d.groups; t.heads = d.heads;
            t.n_active = level_tiles(d, base_tile, n_tiles, dense); t.tile = base_tile >> m.lvl;
            blk = std::max(blk, transformer_ws_bytes(&t));
        } else if (m.kind == K_RES) {
            fise_resnet_args r{};
            r.B = d.B; r.H = d.H >> m.lvl; r.W = d.W >> m.lvl; r.G = d.groups; r.C0 = m.cin; r.C1 = m.cskip; r.Cout = m.cout;
            blk = std::max(blk, resnet_ws_bytes(&r));
        }
    }
    w.block = take(blk);
    w.igemm = take(igemm_workspace_bytes());
    w.total = c;
    return w;
}
}  // namespace

extern "C" size_t fise_unet_workspace_bytes(const fise_unet* u, int max_active_tiles, int base_tile) {
    if (!u || base_tile < 1 || max_active_tiles < 0 || (base_tile >> (u->d.n_levels - 1)) < 1) return 0;
    return ws_layout(u, max_active_tiles, base_tile, nullptr).total;
}

extern "C" int fise_unet_context_kv(const fise_unet* u, const void* weights, const void* ctx, void* ctxkv, void* workspace,
                                    size_t workspace_bytes, void* stream) {
    (void)workspace; (void)workspace_bytes;
    if (!u || !weights || !ctx || !ctxkv) return fail(FISE_ERR_NULL, "fise_unet_context_kv: null pointer");
    const fise_unet_desc& d = u->d;
    const bf16_t* Wt = (const bf16_t*)weights;
    hipStream_t st = as_stream(stream);
    for (const Module& m : u->mods) {
        if (m.kind != K_TR) continue;
        const int C = m.cout;
        // k.w and v.w are adjacent: one launch, two output sections
        IgemmArgs g = linear_args(ctx, d.n_ctx, d.B, d.ctx_dim, Wt + u->off(0, m.name + ".a2.k.w"), nullptr, 2 * C);
        g.nsect = 2; g.sect_n = C; g.Ho = 1; g.Wo = u->n_stride;
        g.out[0] = (bf16_t*)((char*)ctxkv + u->off(2, m.name + ".ctx_k")); g.out_mode[0] = OUT_COMPACT;
        g.out[1] = (bf16_t*)((char*)ctxkv + u->off(2, m.name + ".ctx_vt")); g.out_mode[1] = OUT_TOKENS_T;
        if (int e = launch_igemm(g, nullptr, st)) return e;
    }
    return FISE_OK;
}

extern "C" int fise_unet_num_modules(const fise_unet* u) { return u ? (int)u->mods.size() : 0; }

extern "C" int fise_unet_module_name(const fise_unet* u, int i, char* name) {
    if (!u || !name) return fail(FISE_ERR_NULL, "fise_unet_module_name: null pointer");
    if (i < 0 || i >= (int)u->mods.size()) return fail(FISE_ERR_CAPACITY, "fise_unet_module_name: index %d", i);
    snprintf(name, 64, "%s", u->mods[i].name.c_str());
    return FISE_OK;
}

static int unet_run(const fise_unet* u, const void* weights, void* cache, const void* latent, const float* t_sin, const void* ctxkv,
                    const int32_t* tile_idx, int n_active, int base_tile, int stats_mode, const int* level_dense, int first_module,
                    int n_modules, int trust_derived, void* workspace, size_t workspace_bytes, void* stream);

extern "C" int fise_masked_unet_step(const fise_unet* u, const void* weights, void* cache, const void* latent,
                                     const float* t_sin, const void* ctxkv, const int32_t* tile_idx, int n_active,
                                     int base_tile, int stats_mode, const int* level_dense, void* workspace,
                                     size_t workspace_bytes, void* stream) {
    return unet_run(u, weights, cache, latent, t_sin, ctxkv, tile_idx, n_active, base_tile, stats_mode, level_dense, 0,
                    u ? (int)u->mods.size() : 0, 1, workspace, workspace_bytes, stream);
}

extern "C" int fise_masked_unet_modules(const fise_unet* u, const void* weights, void* cache, const void* latent,
                                        const float* t_sin, const void* ctxkv, const int32_t* tile_idx, int n_active,
                                        int base_tile, int stats_mode, const int* level_dense, int first_module,
                                        int n_modules, void* workspace, size_t workspace_bytes, void* stream) {
    // module i reads its input MAPS as they stand: their normalised copies are recomputed, not trusted
    return unet_run(u, weights, cache, latent, t_sin, ctxkv, tile_idx, n_active, base_tile, stats_mode, level_dense, first_module,
                    n_modules, 0, workspace, workspace_bytes, stream);
}

static int unet_run(const fise_unet* u, const void* weights, void* cache, const void* latent, const float* t_sin, const void* ctxkv,
                    const int32_t* tile_idx, int n_active, int base_tile, int stats_mode, const int* level_dense, int first_module,
                    int n_modules, int trust_derived, void* workspace, size_t workspace_bytes, void* stream) {
    if (!u || !weights || !cache || !latent || !t_sin || !ctxkv) return fail(FISE_ERR_NULL, "fise_masked_unet_step: null pointer");
    const fise_unet_desc& d = u->d;
    const int nl = d.n_levels;
    if (base_tile < 1 || base_tile % (1 << (nl - 1)) || d.H % base_tile || d.W % base_tile)
        return fail(FISE_ERR_SHAPE, "fise_masked_unet_step: base_tile %d must divide H, W and be a multiple of %d", base_tile, 1 << (nl - 1));
    const int tiles_total = (d.W / base_tile) * (d.H / base_tile);
    if (n_active < 0 || n_active > tiles_total) return fail(FISE_ERR_CAPACITY, "fise_masked_unet_step: n_active %d of %d tiles", n_active, tiles_total);
    if (stats_mode != FISE_STATS_CACHED && stats_mode != FISE_STATS_FRESH) return fail(FISE_ERR_SHAPE, "fise_masked_unet_step: stats_mode %d", stats_mode);
    bool any_dense = false;
    if (level_dense) for (int l = 0; l < nl; ++l) any_dense |= level_dense[l] != 0;
    if (first_module < 0 || n_modules < 0 || first_module + n_modules > (int)u->mods.size())
        return fail(FISE_ERR_CAPACITY, "fise_masked_unet_modules: modules [%d, %d) of %zu", first_module, first_module + n_modules, u->mods.size());
    if ((n_active == 0 && !any_dense) || n_modules == 0) return FISE_OK;
    if (n_active > 0 && !tile_idx) return fail(FISE_ERR_NULL, "fise_masked_unet_step: null tile_idx");
    const WsLayout wl = ws_layout(u, n_active, base_tile, level_dense);
    if (!workspace || workspace_bytes < wl.total) return fail(FISE_ERR_CAPACITY, "fise_masked_unet_step: workspace %zu < %zu bytes", workspace_bytes, wl.total);
    const void* chk[] = {weights, cache, latent, ctxkv, workspace};
    for (const void* p : chk) if (!aligned16(p)) return fail(FISE_ERR_ALIGN, "fise_masked_unet_step: pointer %p not 16-byte aligned", p);

    hipStream_t st = as_stream(stream);
    const bf16_t* Wt = (const bf16_t*)weights;
    char* cb = (char*)cache; char* ws = (char*)workspace; const char* kv = (const char*)ctxkv;
    auto Wp = [&](const std::string& n) { return (const void*)(Wt + u->off(0, n)); };
    auto Cp = [&](const std::string& n) { return (void*)(cb + u->off(1, n)); };
    auto Cf = [&](const std::string& n) { return (float*)(cb + u->off(1, n)); };
    auto Dp = [&](const std::string& n) { return (void*)(cb + u->off(3, n)); };
    // the normalised copies the consumers of module m's output want, and m's own derived tensors
    auto derived = [&](const Module& m) {
        BlockDerived dv{};
        if (m.kind == K_RES) {
            dv.act_in = Dp(m.name + ".a1"); dv.act_mid = Dp(m.name + ".a2");
            dv.ss_in = (float2*)Dp(m.name + ".gn1.ss"); dv.ss_mid = (float2*)Dp(m.name + ".gn2.ss");
        } else if (m.kind == K_TR) {
            dv.act_in = Dp(m.name + ".gx"); dv.ss_in = (float2*)Dp(m.name + ".gn.ss");
        }
        dv.trust = trust_derived;
        for (const ViewSpec& v : m.views) {
            const Module& c = u->mods[v.consumer];
            GnView w{};
            if (c.kind == K_RES) {
                w.dst = (bf16_t*)Dp(c.name + ".a1"); w.ss = (const float2*)Dp(c.name + ".gn1.ss");
                w.dstC = c.cin + c.cskip; w.c_off = v.as_skip ? c.cin : 0; w.silu = 1;
            } else {
                w.dst = (bf16_t*)Dp(c.name + ".gx"); w.ss = (const float2*)Dp(c.name + ".gn.ss");
                w.dstC = c.cout; w.c_off = 0; w.silu = 0;
            }
            dv.out_view[dv.n_out_view++] = w;
        }
        return dv;
    };
    int* idx_full = (int*)(ws + wl.idx_full);
    float* emb_a = (float*)(ws + wl.emb_a); float* emb_b = (float*)(ws + wl.emb_b); float* temb = (float*)(ws + wl.temb);
    void* blockws = ws + wl.block;
    const int B = d.B, G = d.groups, te = 4 * d.base;
    const int fresh = stats_mode == FISE_STATS_FRESH;

    IgemmWorkspace iws; const IgemmWorkspace* iw = &iws;
    if (int e = igemm_workspace_init(ws + wl.igemm, igemm_workspace_bytes(), &iws, st)) return e;
    if (any_dense) if (int e = launch_iota(idx_full, tiles_total, st)) return e;
    // time embedding MLP and the stacked per-block projections (dense, a few rows)
    if (int e = launch_small_linear(t_sin, B, d.base, Wp("time.l1.w"), Wp("time.l1.b"), te, 1, emb_a, st)) return e;
    if (int e = launch_small_linear(emb_a, B, te, Wp("time.l2.w"), Wp("time.l2.b"), te, 1, emb_b, st)) return e;
    for (const Module& m : u->mods)
        if (m.kind == K_RES) {
            if (int e = launch_small_linear(emb_b, B, te, Wp(m.name + ".temb.w"), Wp(m.name + ".temb.b"), u->temb_total, 0, temb, st)) return e;
            break;
        }

    for (int mi = first_module; mi < first_module + n_modules; ++mi) {
        const Module& m = u->mods[mi];
        const bool dense = level_dense && level_dense[m.lvl];
        const int* idx = dense ? idx_full : tile_idx;
        const int nt = dense ? tiles_total : n_active;
        if (nt == 0) continue;
        const int tile = base_tile >> m.lvl;
        const int H = d.H >> m.lvl, W = d.W >> m.lvl;
        const std::string& n = m.name;
        const void* in0 = m.in_map.empty() ? latent : Cp(m.in_map);
        const void* in1 = m.skip_map.empty() ? nullptr : Cp(m.skip_map);
        const BlockDerived dv = derived(m);
        const int nview = fresh ? 0 : dv.n_out_view;       // with fresh statistics the consumers normalise for themselves
        switch (m.kind) {
        case K_CONV_IN: {
            fise_conv_args a{};
            a.x0 = latent; a.C0 = d.in_ch; a.B = B; a.H = H; a.W = W; a.w = Wp(n + ".w"); a.bias = Wp(n + ".b"); a.Cout = m.cout;
            a.ksize = 3; a.stride = 1; a.tile_idx = idx; a.n_active = nt; a.tile = tile; a.y_cache = Cp(n + ".out"); a.dtype = FISE_BF16;
            if (int e = conv_dispatch(&a, nullptr, 0, st, dv.out_view, nview)) return e;
        } break;
        case K_RES: {
            fise_resnet_args r{};
            r.x0 = in0; r.x1 = in1; r.C0 = m.cin; r.C1 = m.cskip; r.B = B; r.H = H; r.W = W; r.Cout = m.cout; r.G = G;
            r.gn1_mean = Cf(n + ".gn1.mean"); r.gn1_rstd = Cf(n + ".gn1.rstd"); r.gn1_gamma = Wp(n + ".gn1.g"); r.gn1_beta = Wp(n + ".gn1.b");
            r.conv1_w = Wp(n + ".conv1.w"); r.conv1_b = Wp(n + ".conv1.b"); r.temb = temb + m.temb_off; r.temb_stride = u->temb_total;
            r.gn2_mean = Cf(n + ".gn2.mean"); r.gn2_rstd = Cf(n + ".gn2.rstd"); r.gn2_gamma = Wp(n + ".gn2.g"); r.gn2_beta = Wp(n + ".gn2.b");
            r.conv2_w = Wp(n + ".conv2.w"); r.conv2_b = Wp(n + ".conv2.b");
            if (m.cin + m.cskip != m.cout) { r.sc_w = Wp(n + ".sc.w"); r.sc_b = Wp(n + ".sc.b"); }
            r.tile_idx = idx; r.n_active = nt; r.tile = tile; r.h1_cache = Cp(n + ".h1"); r.out_cache = Cp(n + ".out"); r.stats_fresh = fresh;
            if (int e = run_resnet(&r, blockws, iw, st, &dv)) return e;
        } break;
        case K_TR: {
            fise_transformer_args t{};
            t.x = in0; t.B = B; t.H = H; t.W = W; t.C = m.cout; t.G = G; t.heads = d.heads;
            t.gn_mean = Cf(n + ".gn.mean"); t.gn_rstd = Cf(n + ".gn.rstd"); t.gn_gamma = Wp(n + ".gn.g"); t.gn_beta = Wp(n + ".gn.b");
            t.pin_w = Wp(n + ".pin.w"); t.pin_b = Wp(n + ".pin.b");
            t.ln1_g = Wp(n + ".ln1.g"); t.ln1_b = Wp(n + ".ln1.b"); t.qkv_w = Wp(n + ".a1.q.w"); t.o1_w = Wp(n + ".a1.o.w"); t.o1_b = Wp(n + ".a1.o.b");
            t.ln2_g = Wp(n + ".ln2.g"); t.ln2_b = Wp(n + ".ln2.b"); t.q2_w = Wp(n + ".a2.q.w"); t.o2_w = Wp(n + ".a2.o.w"); t.o2_b = Wp(n + ".a2.o.b");
            t.K_ctx = kv + u->off(2, n + ".ctx_k"); t.Vt_ctx = kv + u->off(2, n + ".ctx_vt"); t.n_ctx = d.n_ctx; t.n_ctx_stride = u->n_stride;
            t.ln3_g = Wp(n + ".ln3.g"); t.ln3_b = Wp(n + ".ln3.b"); t.ff1_w = Wp(n + ".ff1.w"); t.ff1_b = Wp(n + ".ff1.b");
            t.ff2_w = Wp(n + ".ff2.w"); t.ff2_b = Wp(n + ".ff2.b"); t.pout_w = Wp(n + ".pout.w"); t.pout_b = Wp(n + ".pout.b");
            t.K_cache = Cp(n + ".k"); t.Vt_cache = Cp(n + ".v"); t.out_cache = Cp(n + ".out");
            t.tile_idx = idx; t.n_active = nt; t.tile = tile; t.stats_fresh = fresh;
            if (int e = run_transformer(&t, blockws, iw, st, &dv)) return e;
        } break;
        case K_DS:
            if (int e = run_conv(in0, m.cin, B, 2 * H, 2 * W, 2, 0, Wp(n + ".w"), Wp(n + ".b"), m.cout, idx, nt, tile, Cp(n + ".out"), iw, st, dv.out_view, nview)) return e;
            break;
        case K_US:
            if (int e = run_conv(in0, m.cin, B, H / 2, W / 2, 1, 1, Wp(n + ".w"), Wp(n + ".b"), m.cout, idx, nt, tile, Cp(n + ".out"), iw, st, dv.out_view, nview)) return e;
            break;
        case K_OUT: {
            fise_conv_args a{};
            a.x0 = in0; a.C0 = m.cin; a.B = B; a.H = H; a.W = W; a.w = Wp(n + ".conv.w"); a.bias = Wp(n + ".conv.b"); a.Cout = m.cout;
            a.ksize = 3; a.stride = 1; a.gn_mean = Cf(n + ".gn.mean"); a.gn_rstd = Cf(n + ".gn.rstd"); a.gn_gamma = Wp(n + ".gn.g");
            a.gn_beta = Wp(n + ".gn.b"); a.G = G; a.gn_silu = 1; a.tile_idx = idx; a.n_active = nt; a.tile = tile; a.y_cache = Cp("eps");
            a.dtype = FISE_BF16;
            if (fresh)
                if (int e = fise_groupnorm_stats(in0, nullptr, FISE_BF16, B, H, W, m.cin, 0, G, 1e-5f, Cf(n + ".gn.mean"), Cf(n + ".gn.rstd"), blockws, st)) return e;
            if (int e = conv_dispatch(&a, ws + wl.igemm, igemm_workspace_bytes(), st, nullptr, 0)) return e;
        } break;
        }
    }
    return FISE_OK;
}

// ---- derived tensors from the stored ones: scale / shift tables from the cached statistics, then every activated
// map over the whole image (one tile per launch block row: the map's own tile grid at edge 2^(levels-1-level))
extern "C" size_t fise_unet_refresh_derived_workspace_bytes(const fise_unet* u) {
    if (!u) return 0;
    const int t0 = 1 << (u->d.n_levels - 1);
    return align256((size_t)(u->d.H / t0) * (u->d.W / t0) * sizeof(int));
}

extern "C" int fise_unet_refresh_derived(const fise_unet* u, const void* weights, void* cache, void* workspace, size_t workspace_bytes,
                                         void* stream) {
    const char* fn = "fise_unet_refresh_derived";
    if (!u || !weights || !cache || !workspace) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    if (workspace_bytes < fise_unet_refresh_derived_workspace_bytes(u)) return fail(FISE_ERR_CAPACITY, "%s: workspace too small", fn);
    if (!aligned16(weights) || !aligned16(cache) || !aligned16(workspace)) return fail(FISE_ERR_ALIGN, "%s: pointers must be 16-byte aligned", fn);
    const fise_unet_desc& d = u->d;
    hipStream_t st = as_stream(stream);
    const bf16_t* Wt = (const bf16_t*)weights;
    char* cb = (char*)cache;
    auto Wp = [&](const std::string& n) { return (const void*)(Wt + u->off(0, n)); };
    auto Cp = [&](const std::string& n) { return (void*)(cb + u->off(1, n)); };
    auto Cf = [&](const std::string& n) { return (float*)(cb + u->off(1, n)); };
    auto Dp = [&](const std::string& n) { return (void*)(cb + u->off(3, n)); };
    const int t0 = 1 << (d.n_levels - 1);
    const int ntiles = (d.H / t0) * (d.W / t0);
    int* idx_full = (int*)workspace;
    if (int e = launch_iota(idx_full, ntiles, st)) return e;
    const int B = d.B, G = d.groups;
    for (const Module& m : u->mods) {
        const std::string& n = m.name;
        const int H = d.H >> m.lvl, W = d.W >> m.lvl, tile = t0 >> m.lvl;
        if (m.kind == K_RES) {
            const int Ci = m.cin + m.cskip;
            const void* in0 = Cp(m.in_map); const void* in1 = m.skip_map.empty() ? nullptr : Cp(m.skip_map);
            if (int e = launch_gn_scale_shift(Cf(n + ".gn1.mean"), Cf(n + ".gn1.rstd"), Wp(n + ".gn1.g"), Wp(n + ".gn1.b"), B, Ci, G, (float2*)Dp(n + ".gn1.ss"), st)) return e;
            if (int e = launch_gn_scale_shift(Cf(n + ".gn2.mean"), Cf(n + ".gn2.rstd"), Wp(n + ".gn2.g"), Wp(n + ".gn2.b"), B, m.cout, G, (float2*)Dp(n + ".gn2.ss"), st)) return e;
            if (int e = launch_gn_act_halo(in0, in1, m.cin, m.cskip, B, H, W, Cf(n + ".gn1.mean"), Cf(n + ".gn1.rstd"), Wp(n + ".gn1.g"), Wp(n + ".gn1.b"), G, 1,
                                           idx_full, ntiles, tile, Dp(n + ".a1"), st)) return e;
            if (int e = launch_gn_act_halo(Cp(n + ".h1"), nullptr, m.cout, 0, B, H, W, Cf(n + ".gn2.mean"), Cf(n + ".gn2.rstd"), Wp(n + ".gn2.g"), Wp(n + ".gn2.b"), G, 1,
                                           idx_full, ntiles, tile, Dp(n + ".a2"), st)) return e;
        } else if (m.kind == K_TR) {
            if (int e = launch_gn_scale_shift(Cf(n + ".gn.mean"), Cf(n + ".gn.rstd"), Wp(n + ".gn.g"), Wp(n + ".gn.b"), B, m.cout, G, (float2*)Dp(n + ".gn.ss"), st)) return e;
            if (int e = launch_gn_act_halo(Cp(m.in_map), nullptr, m.cout, 0, B, H, W, Cf(n + ".gn.mean"), Cf(n + ".gn.rstd"), Wp(n + ".gn.g"), Wp(n + ".gn.b"), G, 0,
                                           idx_full, ntiles, tile, Dp(n + ".gx"), st)) return e;
        }
    }
    return FISE_OK;
}

// ---------------------------------------------------------------------------
// Moving the part of a cache that a masked step reads or writes (see the header).
// ---------------------------------------------------------------------------
namespace {
constexpr int MOVE_BATCH = 64;          // entries per launch (they travel as kernel arguments)
// Workgroups per entry; each lane strides over the entry's pieces.  Kept small on purpose: these kernels run beside
// the step's own launches on another stream, and lanes waiting on the host link would otherwise fill every wave slot of
// the device (64 workgroups per entry slowed the concurrent step by a third); 8 x 256 lanes x 16 bytes per entry and
// ~60 entries in flight are far more than the link's bandwidth-delay product.
constexpr int MOVE_GX = 8;
struct MoveLevels { int list_off[FISE_MAX_LEVELS]; int hw[FISE_MAX_LEVELS]; };
struct MoveArgs { MoveEntry e[MOVE_BATCH]; MoveLevels lv; int B; };

// Workgroup l lists, ascending, the pixels of level l that lie in an active tile (halo 0) or within one pixel of
// one (halo 1): tile flags in LDS, then an ordered compaction (wave ballot + popcount prefix) 256 pixels at a time.
__global__ __launch_bounds__(256) void cache_pixel_list_kernel(const int* __restrict__ tile_idx, int n_active, int tiles_w, int tiles_h,
                                                               int base_tile, int H, int W, int halo, const MoveLevels lv,
                                                               int* __restrict__ lists, int* __restrict__ counts) {
    extern __shared__ unsigned char tmask[];
    __shared__ int wave_cnt[4];
    const int l = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int nt = tiles_w * tiles_h;
    for (int i = tid; i < nt; i += 256) tmask[i] = 0;
    __syncthreads();
    for (int i = tid; i < n_active; i += 256) {
        const int t = tile_idx[i];
        if ((unsigned)t < (unsigned)nt) tmask[t] = 1;
    }
    __syncthreads();
    const int t = base_tile >> l, Hl = H >> l, Wl = W >> l, n = Hl * Wl;
    int* list = lists + lv.list_off[l];
    int base = 0;
    for (int c0 = 0; c0 < n; c0 += 256) {
        const int p = c0 + tid;
        bool need = false;
        if (p < n) {
            const int y = p / Wl, x = p % Wl;
            for (int dy = -halo; dy <= halo; ++dy)
                for (int dx = -halo; dx <= halo; ++dx) {
                    const int yy = y + dy, xx = x + dx;
                    if (yy >= 0 && yy < Hl && xx >= 0 && xx < Wl) need |= tmask[(yy / t) * tiles_w + xx / t] != 0;
                }
        }
        const unsigned long long bal = __ballot(need);
        const int before = __popcll(bal & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wave] = __popcll(bal);
        __syncthreads();
        int off = base, total = 0;
        for (int w = 0; w < 4; ++w) {
            if (w < wave) off += wave_cnt[w];
            total += wave_cnt[w];
        }
        if (need) list[off + before] = p;
        base += total;
        __syncthreads();
    }
    if (tid == 0) counts[l] = base;
}

// dst[addr] = src[addr] for every listed pixel of every entry: 16-byte pieces of a pixel's row (two-byte pieces when
// the row is not a multiple of 16 bytes), or one two-byte element per (channel, pixel) of a transposed tensor.
__global__ __launch_bounds__(256) void cache_move_kernel(const MoveArgs a, const int* __restrict__ lists, const int* __restrict__ counts,
                                                         const unsigned char* __restrict__ src, unsigned char* __restrict__ dst) {
    const MoveEntry e = a.e[blockIdx.y];
    const unsigned cnt = (unsigned)counts[e.lvl], hw = (unsigned)a.lv.hw[e.lvl];
    if (cnt == 0) return;
    const int* list = lists + a.lv.list_off[e.lvl];
    const unsigned stride = gridDim.x * 256u, w0 = blockIdx.x * 256u + threadIdx.x;
    if (e.vt) {
        const unsigned total = cnt * (unsigned)a.B * (unsigned)e.row_bytes;         // row_bytes = channels here
        for (unsigned w = w0; w < total; w += stride) {
            const unsigned pi = w % cnt, bc = w / cnt;
            const size_t addr = (size_t)e.off + ((size_t)bc * hw + (unsigned)list[pi]) * 2;
            *(unsigned short*)(dst + addr) = *(const unsigned short*)(src + addr);
        }
    } else if ((e.row_bytes & 15) == 0) {
        const unsigned pieces = (unsigned)e.row_bytes >> 4, total = cnt * (unsigned)a.B * pieces;
        for (unsigned w = w0; w < total; w += stride) {
            const unsigned piece = w % pieces, pb = w / pieces, pi = pb % cnt, b = pb / cnt;
            const size_t addr = (size_t)e.off + ((size_t)b * hw + (unsigned)list[pi]) * (unsigned)e.row_bytes + piece * 16u;
            *(uint4*)(dst + addr) = *(const uint4*)(src + addr);
        }
    } else {
        const unsigned pieces = (unsigned)e.row_bytes >> 1, total = cnt * (unsigned)a.B * pieces;
        for (unsigned w = w0; w < total; w += stride) {
            const unsigned piece = w % pieces, pb = w / pieces, pi = pb % cnt, b = pb / cnt;
            const size_t addr = (size_t)e.off + ((size_t)b * hw + (unsigned)list[pi]) * (unsigned)e.row_bytes + piece * 2u;
            *(unsigned short*)(dst + addr) = *(const unsigned short*)(src + addr);
        }
    }
}

// The address under which the GPU reaches p: device memory as it is, pinned host memory through its mapping.
int gpu_address(const char* fn, const char* what, const void* p, void** out) {
    hipPointerAttribute_t at{};
    if (hipPointerGetAttributes(&at, p) != hipSuccess) {
        (void)hipGetLastError();
        return fail(FISE_ERR_ALIGN, "%s: %s %p is neither device memory nor pinned host memory", fn, what, p);
    }
    if (at.type == hipMemoryTypeDevice) { *out = const_cast<void*>(p); return FISE_OK; }
    if (at.type == hipMemoryTypeHost && at.devicePointer) { *out = at.devicePointer; return FISE_OK; }
    return fail(FISE_ERR_ALIGN, "%s: %s %p is neither device memory nor pinned host memory", fn, what, p);
}

size_t move_lists_ints(const fise_unet_desc& d) {
    size_t n = 0;
    for (int l = 0; l < d.n_levels; ++l) n += (size_t)(d.H >> l) * (d.W >> l);
    return n;
}
}  // namespace

extern "C" int fise_unet_cache_layout_get(const fise_unet* u, fise_unet_cache_layout* out) {
    if (!u || !out) return fail(FISE_ERR_NULL, "fise_unet_cache_layout_get: null pointer");
    *out = u->layout;
    return FISE_OK;
}

extern "C" size_t fise_unet_cache_move_workspace_bytes(const fise_unet* u) {
    if (!u) return 0;
    return align256((move_lists_ints(u->d) + FISE_MAX_LEVELS) * sizeof(int));
}

extern "C" int fise_unet_cache_move_active(const fise_unet* u, const void* src, void* dst, const int32_t* tile_idx, int n_active,
                                           int base_tile, int halo, int what, void* workspace, size_t workspace_bytes, void* stream) {
    const char* fn = "fise_unet_cache_move_active";
    if (!u || !src || !dst) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    const fise_unet_desc& d = u->d;
    const int nl = d.n_levels;
    if (base_tile < 1 || base_tile % (1 << (nl - 1)) || d.H % base_tile || d.W % base_tile)
        return fail(FISE_ERR_SHAPE, "%s: base_tile %d must divide H, W and be a multiple of %d", fn, base_tile, 1 << (nl - 1));
    const int tiles_w = d.W / base_tile, tiles_h = d.H / base_tile, tiles_total = tiles_w * tiles_h;
    if (n_active < 0 || n_active > tiles_total) return fail(FISE_ERR_CAPACITY, "%s: n_active %d of %d tiles", fn, n_active, tiles_total);
    if (halo != 0 && halo != 1) return fail(FISE_ERR_SHAPE, "%s: halo %d (0 or 1)", fn, halo);
    if (what & ~(FISE_MOVE_MAPS | FISE_MOVE_K | FISE_MOVE_VT)) return fail(FISE_ERR_SHAPE, "%s: unknown bits in what = %d", fn, what);
    if (n_active == 0 || what == 0) return FISE_OK;
    if (!tile_idx || !workspace) return fail(FISE_ERR_NULL, "%s: null tile_idx or workspace", fn);
    if (workspace_bytes < fise_unet_cache_move_workspace_bytes(u)) return fail(FISE_ERR_CAPACITY, "%s: workspace too small", fn);
    if (tiles_total > 48 * 1024) return fail(FISE_ERR_CAPACITY, "%s: %d tiles exceed the tile-flag table of 48 K entries", fn, tiles_total);
    int cmax = std::max(d.in_ch, d.out_ch);
    for (int l = 0; l < nl; ++l) cmax = std::max(cmax, d.base * d.mults[l]);
    if ((size_t)d.B * d.H * d.W * cmax >= ((size_t)1 << 32))          // the kernels count pieces in 32 bits
        return fail(FISE_ERR_CAPACITY, "%s: maps too large for 32-bit piece counters", fn);
    if (!aligned16(src) || !aligned16(dst) || !aligned16(workspace)) return fail(FISE_ERR_ALIGN, "%s: pointers must be 16-byte aligned", fn);
    const char* sb = (const char*)src; const char* db = (const char*)dst;
    if (sb < db + u->cache_bytes && db < sb + u->cache_bytes) return fail(FISE_ERR_SHAPE, "%s: src and dst overlap", fn);
    void* gsrc = nullptr; void* gdst = nullptr;
    if (int e = gpu_address(fn, "src", src, &gsrc)) return e;
    if (int e = gpu_address(fn, "dst", dst, &gdst)) return e;

    hipStream_t st = as_stream(stream);
    MoveArgs args{};
    int off = 0;
    for (int l = 0; l < nl; ++l) { args.lv.list_off[l] = off; args.lv.hw[l] = (d.H >> l) * (d.W >> l); off += args.lv.hw[l]; }
    args.B = d.B;
    int* lists = (int*)workspace;
    int* counts = lists + off;
    hipLaunchKernelGGL(cache_pixel_list_kernel, dim3(nl), dim3(256), (size_t)tiles_total, st, tile_idx, n_active, tiles_w, tiles_h, base_tile,
                       d.H, d.W, halo, args.lv, lists, counts);
    FISE_CHECK_LAUNCH("cache pixel lists");
    const std::vector<MoveEntry>* groups[3] = {&u->move_maps, &u->move_k, &u->move_vt};
    for (int g = 0; g < 3; ++g) {
        if (!(what & (1 << g))) continue;
        const std::vector<MoveEntry>& v = *groups[g];
        for (size_t i0 = 0; i0 < v.size(); i0 += MOVE_BATCH) {
            const int n = (int)std::min<size_t>(MOVE_BATCH, v.size() - i0);
            for (int i = 0; i < n; ++i) args.e[i] = v[i0 + i];
            hipLaunchKernelGGL(cache_move_kernel, dim3(MOVE_GX, n), dim3(256), 0, st, args, lists, counts, (const unsigned char*)gsrc,
                               (unsigned char*)gdst);
            FISE_CHECK_LAUNCH("cache move");
        }
    }
    return FISE_OK;
}

// The same move by the copy engines: whole pixel rows of the map levels, one asynchronous copy per (tensor, batch
// element, run of rows).  No kernel runs, so nothing competes with the step's launches for the compute units or sits
// in front of their end-of-kernel cache maintenance (measured: lanes of a concurrent kernel waiting on the host link
// make every launch of the step 2-3x longer while they are in flight; copy-engine transfers do not).
extern "C" int fise_unet_cache_move_tile_rows(const fise_unet* u, const void* src, void* dst, const int32_t* tile_rows, int n_ranges,
                                              int base_tile, int halo, int what, void* stream) {
    const char* fn = "fise_unet_cache_move_tile_rows";
    if (!u || !src || !dst) return fail(FISE_ERR_NULL, "%s: null pointer", fn);
    const fise_unet_desc& d = u->d;
    const int nl = d.n_levels;
    if (base_tile < 1 || base_tile % (1 << (nl - 1)) || d.H % base_tile || d.W % base_tile)
        return fail(FISE_ERR_SHAPE, "%s: base_tile %d must divide H, W and be a multiple of %d", fn, base_tile, 1 << (nl - 1));
    if (halo != 0 && halo != 1) return fail(FISE_ERR_SHAPE, "%s: halo %d (0 or 1)", fn, halo);
    if (what & ~(FISE_MOVE_MAPS | FISE_MOVE_K)) return fail(FISE_ERR_SHAPE, "%s: what = %d (maps and K rows only; V^T is not row-addressed)", fn, what);
    if (n_ranges < 0) return fail(FISE_ERR_CAPACITY, "%s: n_ranges %d", fn, n_ranges);
    if (n_ranges == 0 || what == 0) return FISE_OK;
    if (!tile_rows) return fail(FISE_ERR_NULL, "%s: null tile_rows", fn);
    const int tiles_h = d.H / base_tile;
    for (int r = 0; r < n_ranges; ++r) {
        const int a = tile_rows[2 * r], b = tile_rows[2 * r + 1];
        if (a < 0 || b <= a || b > tiles_h || (r > 0 && a < tile_rows[2 * r - 1]))
            return fail(FISE_ERR_SHAPE, "%s: range %d = [%d, %d) must be non-empty, ascending, disjoint and inside %d tile rows", fn, r, a, b, tiles_h);
    }
    const char* sb = (const char*)src; char* db = (char*)dst;
    if (sb < db + u->cache_bytes && db < sb + u->cache_bytes) return fail(FISE_ERR_SHAPE, "%s: src and dst overlap", fn);
    hipStream_t st = as_stream(stream);
    // runs of pixel rows per level (ranges that touch after the ring is added are merged)
    std::vector<std::pair<int, int>> runs[FISE_MAX_LEVELS];
    for (int l = 0; l < nl; ++l) {
        const int t = base_tile >> l, Hl = d.H >> l;
        for (int r = 0; r < n_ranges; ++r) {
            const int y0 = std::max(0, tile_rows[2 * r] * t - halo), y1 = std::min(Hl, tile_rows[2 * r + 1] * t + halo);
            if (!runs[l].empty() && y0 <= runs[l].back().second) runs[l].back().second = std::max(runs[l].back().second, y1);
            else runs[l].push_back({y0, y1});
        }
    }
    const std::vector<MoveEntry>* groups[2] = {&u->move_maps, &u->move_k};
    for (int g = 0; g < 2; ++g) {
        if (!(what & (1 << g))) continue;
        for (const MoveEntry& e : *groups[g]) {
            const size_t Hl = (size_t)(d.H >> e.lvl), row = (size_t)(d.W >> e.lvl) * e.row_bytes;
            for (int b = 0; b < d.B; ++b)
                for (const auto& run : runs[e.lvl]) {
                    const size_t off = (size_t)e.off + ((size_t)b * Hl + run.first) * row;
                    if (hipMemcpyAsync(db + off, sb + off, (size_t)(run.second - run.first) * row, hipMemcpyDefault, st) != hipSuccess) {
                        (void)hipGetLastError();
                        return fail(FISE_ERR_HIP, "%s: hipMemcpyAsync failed", fn);
                    }
                }
        }
    }
    return FISE_OK;
}
