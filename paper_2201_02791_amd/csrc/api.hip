// Per-step entry points of the C ABI: argument checks, workspace carving and the launch
// sequence of one training step (Algorithm 1: GNNmodel, loss, backward) on one stream.
#include <string.h>

#include <vector>

#include "common.h"

// ------------------------------------------------------------------ event profiling
namespace {
struct ProfRec { const char *name; hipEvent_t a, b; };
bool g_prof_on = false;
std::vector<ProfRec> g_prof_recs;
std::vector<hipEvent_t> g_prof_pool;
hipEvent_t prof_event()
{
    if (!g_prof_pool.empty()) { hipEvent_t e = g_prof_pool.back(); g_prof_pool.pop_back(); return e; }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}
}  // namespace

KgeProfScope::KgeProfScope(const char *name, hipStream_t s) : slot(-1), st(s)
{
    if (!g_prof_on) return;
    ProfRec r{name, prof_event(), prof_event()};
    if (!r.a || !r.b) return;
    (void)hipEventRecord(r.a, st);
    slot = (int)g_prof_recs.size();
    g_prof_recs.push_back(r);
}
KgeProfScope::~KgeProfScope()
{
    if (slot >= 0) (void)hipEventRecord(g_prof_recs[slot].b, st);
}

extern "C" int kge_profile_enable(int32_t on)
{
    g_prof_on = on != 0;
    return KGE_OK;
}

extern "C" int kge_profile_collect(kge_prof_entry *out, int32_t max_entries, int32_t *n_entries)
{
    KGE_REQUIRE(out && n_entries && max_entries > 0, KGE_EINVAL, "NULL argument");
    int n = 0;
    for (const ProfRec &r : g_prof_recs) {
        float ms = 0.f;
        KGE_HIP(hipEventSynchronize(r.b));
        KGE_HIP(hipEventElapsedTime(&ms, r.a, r.b));
        int k = 0;
        for (; k < n; ++k) if (strncmp(out[k].name, r.name, sizeof out[k].name) == 0) break;
        if (k == n) {
            if (n == max_entries) continue;
            memset(&out[n], 0, sizeof out[n]);
            strncpy(out[n].name, r.name, sizeof(out[n].name) - 1);
            ++n;
        }
        out[k].total_ms += ms;
        out[k].calls += 1;
        g_prof_pool.push_back(r.a);
        g_prof_pool.push_back(r.b);
    }
    g_prof_recs.clear();
    *n_entries = n;
    return KGE_OK;
}

namespace {

struct WsLayout {
    std::vector<size_t> off_P, off_H;   // per layer: projected messages, layer output
    std::vector<size_t> off_Hbf, off_Wbf, off_WbfT;   // bf16 workloads: bf16 copies of layer input and weights
    std::vector<size_t> off_Z;          // relation-weight layers: run means [S][d_in]
    size_t off_C = 0;                   // relation-weight layers: C [2R][d_in*d_out] (shared)
    // relation-weight layers: W_r fp32 [2R][d_in*d_out] and, for bf16 workloads, its bf16 copies in both
    // orientations; U / dZ [S][max(d_in, d_out)] (shared)
    std::vector<size_t> off_Wrel, off_Wrb, off_WrbT;
    size_t off_U = 0;
    std::vector<size_t> off_Hd;         // layers with dropout: the input as the layer reads it, fp32 [N][d_in]
    size_t off_self = 0, off_G = 0, off_dP = 0, off_dHa = 0, off_dHb = 0, off_seg = 0, off_part = 0, total = 0;
};

int check_layers(const kge_partition *p, const kge_layer *layers, int32_t n_layers, int32_t msg_dtype)
{
    KGE_REQUIRE(p && layers, KGE_EINVAL, "NULL partition or layers");
    KGE_REQUIRE(n_layers >= 1 && n_layers <= 16, KGE_EINVAL, "n_layers must be in [1, 16]");
    KGE_REQUIRE(msg_dtype == KGE_MSG_F32 || msg_dtype == KGE_MSG_BF16, KGE_EINVAL, "bad msg_dtype");
    const int mult = msg_dtype == KGE_MSG_BF16 ? 8 : 4;
    const int dmax = msg_dtype == KGE_MSG_BF16 ? 512 : 256;
    for (int l = 0; l < n_layers; ++l) {
        const kge_layer &L = layers[l];
        KGE_REQUIRE(L.V && L.a && L.W0, KGE_EINVAL, "layer %d has a NULL parameter pointer", l);
        KGE_REQUIRE(L.d_in > 0 && L.d_out > 0 && L.n_bases > 0 && L.n_bases <= 256, KGE_EINVAL,
                    "layer %d: d_in, d_out must be positive and n_bases in [1, 256]", l);
        KGE_REQUIRE(L.d_in % mult == 0 && L.d_out % mult == 0, KGE_EINVAL,
                    "layer %d: d_in and d_out must be multiples of %d", l, mult);
        KGE_REQUIRE(L.d_out <= dmax && L.d_in <= 512, KGE_EINVAL,
                    "layer %d: d_out must be at most %d and d_in at most 512", l, dmax);
        // the transposed gather of the project-first order holds a row of d_out floats in one wavefront's lanes
        KGE_REQUIRE(L.order != KGE_ORDER_PROJECT_FIRST || L.d_out <= 256, KGE_EINVAL,
                    "layer %d: the project-first order needs d_out <= 256", l);
        KGE_REQUIRE(L.act == KGE_ACT_IDENTITY || L.act == KGE_ACT_RELU, KGE_EINVAL, "layer %d: bad act", l);
        KGE_REQUIRE(L.dropout >= 0.0f && L.dropout < 1.0f, KGE_EINVAL, "layer %d: dropout must be in [0, 1)", l);
        KGE_REQUIRE(L.order == KGE_ORDER_PROJECT_FIRST || L.order == KGE_ORDER_RELATION_WEIGHTS, KGE_EINVAL,
                    "layer %d: bad order", l);
        KGE_REQUIRE(L.order != KGE_ORDER_RELATION_WEIGHTS || L.d_in <= dmax, KGE_EINVAL,
                    "layer %d: the relation-weight order needs d_in <= %d", l, dmax);
        KGE_REQUIRE(l == 0 || L.d_in == layers[l - 1].d_out, KGE_EINVAL,
                    "layer %d: d_in does not match the previous layer's d_out", l);
        KGE_REQUIRE(((uintptr_t)L.V % 16) == 0 && ((uintptr_t)L.W0 % 16) == 0, KGE_EINVAL,
                    "layer %d: V and W0 must be 16-byte aligned", l);
    }
    return KGE_OK;
}

void layout(const kge_partition *p, const kge_layer *layers, int32_t n_layers, int32_t msg_dtype, WsLayout *w)
{
    const size_t N = (size_t)p->n_vert, ep = msg_dtype == KGE_MSG_BF16 ? 2 : 4;
    size_t cur = 0, max_dout = 0, max_din = 0, max_bd = 0, max_B = 0;
    const bool bf = msg_dtype == KGE_MSG_BF16;
    size_t max_nc = 0;
    w->off_P.assign(n_layers, 0); w->off_H.resize(n_layers); w->off_Z.assign(n_layers, 0);
    w->off_Wrel.assign(n_layers, 0); w->off_Wrb.assign(n_layers, 0); w->off_WrbT.assign(n_layers, 0);
    size_t max_u = 0;
    size_t max_c = 0, max_zd = 0;
    w->off_Hbf.assign(n_layers, 0); w->off_Wbf.assign(n_layers, 0); w->off_WbfT.assign(n_layers, 0);
    w->off_Hd.assign(n_layers, 0);
    for (int l = 0; l < n_layers; ++l) {
        const kge_layer &L = layers[l];
        if (L.order == KGE_ORDER_RELATION_WEIGHTS) {
            const size_t dd = (size_t)L.d_in * L.d_out, R2 = (size_t)2 * p->n_relations;
            // bf16: the run means follow the bf16 copy of the layer input without a gap, so that the two are
            // one matrix [X; Z] whose rows the partition's seg_zrow addresses
            if (bf) { w->off_Hbf[l] = cur; cur += N * L.d_in * 2; }
            w->off_Z[l] = cur; cur = align_up(cur + (size_t)p->n_seg * L.d_in * ep, 256);
            if (!bf) {
                w->off_Wrel[l] = cur; cur = align_up(cur + R2 * dd * 4, 256);
            } else {
                w->off_Wrb[l] = cur; cur = align_up(cur + R2 * dd * 2, 256);
                w->off_WrbT[l] = cur; cur = align_up(cur + R2 * dd * 2, 256);
            }
            const size_t dm = (size_t)(L.d_in > L.d_out ? L.d_in : L.d_out);
            if ((size_t)p->n_seg * dm * ep > max_u) max_u = (size_t)p->n_seg * dm * ep;
            if (R2 * dd * 4 > max_c) max_c = R2 * dd * 4;
            if ((size_t)L.d_in > max_zd) max_zd = L.d_in;
            if ((size_t)L.d_in > max_dout) max_dout = L.d_in;      // Self also holds the self-loop part of dH
        } else {
            w->off_P[l] = cur; cur = align_up(cur + N * L.n_bases * L.d_out * ep, 256);
        }
        w->off_H[l] = cur; cur = align_up(cur + N * L.d_out * 4, 256);
        if (L.dropout > 0.0f) { w->off_Hd[l] = cur; cur = align_up(cur + N * L.d_in * 4, 256); }
        if ((size_t)L.d_out > max_dout) max_dout = L.d_out;
        if ((size_t)L.d_in > max_din) max_din = L.d_in;
        if ((size_t)L.n_bases * L.d_out > max_bd) max_bd = (size_t)L.n_bases * L.d_out;
        if ((size_t)L.n_bases > max_B) max_B = L.n_bases;
        const size_t nc = (size_t)(L.n_bases + 1) * L.d_out;
        if (nc > max_nc) max_nc = nc;
        if (bf) {
            if (L.order != KGE_ORDER_RELATION_WEIGHTS) { w->off_Hbf[l] = cur; cur = align_up(cur + N * L.d_in * 2, 256); }
            w->off_Wbf[l] = cur; cur = align_up(cur + nc * L.d_in * 2, 256);
            w->off_WbfT[l] = cur; cur = align_up(cur + nc * L.d_in * 2, 256);
        }
    }
    w->off_C = cur; cur = align_up(cur + max_c, 256);
    w->off_U = cur; cur = align_up(cur + max_u, 256);
    w->off_self = cur; cur = align_up(cur + N * max_dout * 4, 256);
    w->off_G = cur; cur = align_up(cur + N * max_dout * 4, 256);
    // dP; bf16 workloads append G behind it so that X = [dP | G] is one bf16 matrix
    w->off_dP = cur; cur = align_up(cur + (bf ? N * max_nc * 2 : N * max_bd * ep), 256);
    w->off_dHa = cur; cur = align_up(cur + N * max_din * 4, 256);
    w->off_dHb = cur; cur = align_up(cur + N * max_din * 4, 256);
    w->off_seg = cur; cur = align_up(cur + (size_t)p->n_seg * max_B * 4, 256);
    // partial results of the units of heavy rows; the three users never overlap in time
    size_t part = (size_t)p->hv_dm.n_units * max_dout;
    if ((size_t)p->hv_sm.n_units * max_bd > part) part = (size_t)p->hv_sm.n_units * max_bd;
    if ((size_t)p->hv_seg.n_units * max_B > part) part = (size_t)p->hv_seg.n_units * max_B;
    if ((size_t)p->hv_seg.n_units * max_zd > part) part = (size_t)p->hv_seg.n_units * max_zd;
    if (max_u > 0 && (size_t)p->hv_dr.n_units * max_dout > part) part = (size_t)p->hv_dr.n_units * max_dout;
    if (max_u > 0 && (size_t)p->hv_sm.n_units * max_dout > part) part = (size_t)p->hv_sm.n_units * max_dout;
    w->off_part = cur; cur = align_up(cur + part * 4, 256);
    w->total = cur > 0 ? cur : 256;
}

int check_ws(const kge_partition *p, const kge_layer *layers, int32_t n_layers, int32_t msg_dtype,
             void *workspace, size_t ws_bytes, WsLayout *w)
{
    int rc = check_layers(p, layers, n_layers, msg_dtype);
    if (rc != KGE_OK) return rc;
    layout(p, layers, n_layers, msg_dtype, w);
    KGE_REQUIRE(workspace && ((uintptr_t)workspace % 256) == 0, KGE_EINVAL, "workspace must be 256-byte aligned");
    KGE_REQUIRE(ws_bytes >= w->total, KGE_ENOMEM, "workspace has %zu bytes, %zu needed", ws_bytes, w->total);
    return KGE_OK;
}

}  // namespace

extern "C" size_t kge_workspace_bytes(const kge_partition *p, const kge_layer *layers, int32_t n_layers,
                                      int32_t msg_dtype)
{
    if (check_layers(p, layers, n_layers, msg_dtype) != KGE_OK) return 0;
    WsLayout w;
    layout(p, layers, n_layers, msg_dtype, &w);
    return w.total;
}

extern "C" int kge_workspace_slice(const kge_partition *p, const kge_layer *layers, int32_t n_layers,
                                   int32_t msg_dtype, int32_t which, int32_t layer, size_t *offset,
                                   size_t *bytes)
{
    int rc = check_layers(p, layers, n_layers, msg_dtype);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(offset && bytes, KGE_EINVAL, "NULL argument");
    KGE_REQUIRE(layer >= 0 && layer < n_layers, KGE_EINVAL, "layer out of range");
    WsLayout w;
    layout(p, layers, n_layers, msg_dtype, &w);
    const size_t N = (size_t)p->n_vert, ep = msg_dtype == KGE_MSG_BF16 ? 2 : 4;
    const kge_layer &L = layers[layer];
    switch (which) {
    case KGE_WS_P:
        KGE_REQUIRE(L.order == KGE_ORDER_PROJECT_FIRST, KGE_EINVAL, "a relation-weight layer keeps no projected messages");
        *offset = w.off_P[layer]; *bytes = N * L.n_bases * L.d_out * ep; break;
    case KGE_WS_Z:
        KGE_REQUIRE(L.order != KGE_ORDER_PROJECT_FIRST, KGE_EINVAL, "a project-first layer keeps no run means");
        *offset = w.off_Z[layer]; *bytes = (size_t)p->n_seg * L.d_in * ep; break;
    case KGE_WS_U:
        KGE_REQUIRE(L.order == KGE_ORDER_RELATION_WEIGHTS, KGE_EINVAL, "only relation-weight layers have per-run products");
        *offset = w.off_U; *bytes = (size_t)p->n_seg * (size_t)(L.d_in > L.d_out ? L.d_in : L.d_out) * ep; break;
    case KGE_WS_H: *offset = w.off_H[layer]; *bytes = N * L.d_out * 4; break;
    case KGE_WS_HD:
        KGE_REQUIRE(L.dropout > 0.0f, KGE_EINVAL, "layer %d has no dropout", layer);
        *offset = w.off_Hd[layer]; *bytes = N * L.d_in * 4; break;
    case KGE_WS_G: *offset = w.off_G; *bytes = N * L.d_out * 4; break;
    case KGE_WS_DP:
        *offset = w.off_dP;
        *bytes = N * (size_t)(msg_dtype == KGE_MSG_BF16 ? L.n_bases + 1 : L.n_bases) * L.d_out * ep;
        break;
    case KGE_WS_DH:
        KGE_REQUIRE(layer >= 1, KGE_EINVAL, "layer 0's input gradient is the caller's dH0");
        *offset = (layer & 1) ? w.off_dHb : w.off_dHa; *bytes = N * L.d_in * 4; break;
    default: KGE_REQUIRE(false, KGE_EINVAL, "unknown workspace slice %d", which);
    }
    return KGE_OK;
}

extern "C" int kge_rgcn_forward(const kge_partition *p, const kge_cgraph *cg, const kge_layer *layers,
                                int32_t n_layers, int32_t msg_dtype, const float *H0, void *workspace,
                                size_t ws_bytes, float *H_out, void *stream)
{
    WsLayout w;
    int rc = check_ws(p, layers, n_layers, msg_dtype, workspace, ws_bytes, &w);
    if (rc != KGE_OK) return rc;
    rc = kge_cgraph_check(p, cg, n_layers);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(H0 && H_out, KGE_EINVAL, "H0 or H_out is NULL");
    KGE_REQUIRE(((uintptr_t)H0 % 16) == 0 && ((uintptr_t)H_out % 16) == 0, KGE_EINVAL, "H0 and H_out must be 16-byte aligned");
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int bf = msg_dtype == KGE_MSG_BF16;
    const float *Hin = H0;
    float *Self = (float *)(ws + w.off_self);
    float *part = (float *)(ws + w.off_part);
    bool hbf_written = false;        // the previous layer has written this layer's bf16 input already
    for (int l = 0; l < n_layers; ++l) {
        const kge_layer &L = layers[l];
        void *P = ws + w.off_P[l];
        float *Hl = (float *)(ws + w.off_H[l]);
        // The last layer's output goes to the caller's H_out; the workspace keeps a copy of it only when
        // backward reads it (the ReLU mask).
        const bool last = l == n_layers - 1;
        float *out1 = last && L.act == KGE_ACT_IDENTITY ? H_out : Hl;
        float *out2 = last && L.act != KGE_ACT_IDENTITY ? H_out : nullptr;
        if (L.dropout > 0.0f) {      // everything below reads the dropped copy; backward regenerates the mask
            float *Hd = (float *)(ws + w.off_Hd[l]);
            rc = launch_dropout(Hin, p->n_vert, L.d_in, L.dropout, L.drop_seed, L.drop_step, l, Hd, st);
            if (rc != KGE_OK) return rc;
            Hin = Hd;
        }
        if (L.order == KGE_ORDER_RELATION_WEIGHTS) {
            void *Z = ws + w.off_Z[l], *U = ws + w.off_U;
            float *Wrel = (float *)(ws + w.off_Wrel[l]);
            const uint8_t *act_l = kge_cgraph_layer(cg, l);
            const int32_t R2 = 2 * p->n_relations;
            // bf16 messages: the relation matrices are rounded as they are summed; the fp32 ones are never stored
            if (bf) rc = launch_relation_weights_bf16(L.a, R2, L.n_bases, L.V, L.d_in, L.d_out, ws + w.off_Wrb[l], ws + w.off_WrbT[l], st);
            else rc = launch_relation_weights(L.a, R2, L.n_bases, L.V, (int64_t)L.d_in * L.d_out, Wrel, st);
            if (rc != KGE_OK) return rc;
            if (bf) {
                void *Hbf = ws + w.off_Hbf[l], *Wbf = ws + w.off_Wbf[l], *WbfT = ws + w.off_WbfT[l];
                if (!hbf_written) rc = launch_cvt_rows_bf16(Hin, p->n_vert * (int64_t)L.d_in, Hbf, st);
                if (rc != KGE_OK) return rc;
                rc = launch_cvt_weights_bf16(L.V, L.W0, L.d_in, L.d_out, 0, Wbf, WbfT, st);     // W0 alone, both orientations
                if (rc != KGE_OK) return rc;
                // a run of one edge has its source's row of Hbf as its mean: those rows of Z are neither written
                // nor read (Hbf and Z are adjacent, seg_zrow says which row of [Hbf; Z] holds run s)
                const int32_t *zrow = p->seg_zrow;
                rc = launch_run_mean(p, Hbf, L.d_in, Z, 1, part, act_l, zrow != nullptr, st);
                if (rc != KGE_OK) return rc;
                rc = launch_apply_relation_weights_bf16(p, zrow ? Hbf : Z, zrow, ws + w.off_WrbT[l], L.d_in, L.d_out, U, st);
                if (rc != KGE_OK) return rc;
                rc = launch_project_bf16(Hbf, p->n_vert, L.d_in, L.d_out, 0, WbfT, nullptr, Self, st);
            } else {
                rc = launch_run_mean(p, Hin, L.d_in, Z, 0, part, act_l, 0, st);
                if (rc != KGE_OK) return rc;
                rc = launch_apply_relation_weights(p, (const float *)Z, Wrel, L.d_in, L.d_out, (float *)U, st);
                if (rc != KGE_OK) return rc;
                rc = launch_project(Hin, p->n_vert, L.d_in, L.d_out, 0, L.V, L.W0, nullptr, Self, st);
            }
            if (rc != KGE_OK) return rc;
            // the next layer's bf16 input is written by this layer's sums when that layer reads this output as
            // it is (same order, no dropout in between)
            hbf_written = bf && !last && layers[l + 1].order == KGE_ORDER_RELATION_WEIGHTS && layers[l + 1].dropout == 0.0f;
            rc = launch_sum_runs(p, U, bf, L.d_out, Self, L.act, out1, out2, hbf_written ? ws + w.off_Hbf[l + 1] : nullptr,
                                 part, act_l, st);
            if (rc != KGE_OK) return rc;
            Hin = Hl;
            continue;
        }
        if (bf) {
            void *Hbf = ws + w.off_Hbf[l], *Wbf = ws + w.off_Wbf[l], *WbfT = ws + w.off_WbfT[l];
            rc = launch_cvt_rows_bf16(Hin, p->n_vert * (int64_t)L.d_in, Hbf, st);
            if (rc != KGE_OK) return rc;
            rc = launch_cvt_weights_bf16(L.V, L.W0, L.d_in, L.d_out, L.n_bases, Wbf, WbfT, st);
            if (rc != KGE_OK) return rc;
            rc = launch_project_bf16(Hbf, p->n_vert, L.d_in, L.d_out, L.n_bases, WbfT, P, Self, st);
        } else {
            rc = launch_project(Hin, p->n_vert, L.d_in, L.d_out, L.n_bases, L.V, L.W0, (float *)P, Self, st);
        }
        if (rc != KGE_OK) return rc;
        rc = launch_gather_forward(p, P, bf, L.a, L.n_bases, L.d_out, Self, L.act, out1, out2, part,
                                   kge_cgraph_layer(cg, l), st);
        if (rc != KGE_OK) return rc;
        Hin = Hl;
    }
    return KGE_OK;
}

extern "C" int kge_rgcn_backward(const kge_partition *p, const kge_cgraph *cg, const kge_layer *layers,
                                 int32_t n_layers, int32_t msg_dtype, const float *H0, void *workspace,
                                 size_t ws_bytes, const float *dH_out, const kge_layer_grad *grads, float *dH0,
                                 void *stream)
{
    WsLayout w;
    int rc = check_ws(p, layers, n_layers, msg_dtype, workspace, ws_bytes, &w);
    if (rc != KGE_OK) return rc;
    rc = kge_cgraph_check(p, cg, n_layers);
    if (rc != KGE_OK) return rc;
    KGE_REQUIRE(H0 && dH_out && grads, KGE_EINVAL, "H0, dH_out or grads is NULL");
    KGE_REQUIRE(((uintptr_t)H0 % 16) == 0 && ((uintptr_t)dH_out % 16) == 0 && ((uintptr_t)dH0 % 16) == 0,
                KGE_EINVAL, "H0, dH_out and dH0 must be 16-byte aligned");
    for (int l = 0; l < n_layers; ++l)
        KGE_REQUIRE(grads[l].dV && grads[l].da && grads[l].dW0 && ((uintptr_t)grads[l].dV % 4) == 0 &&
                        ((uintptr_t)grads[l].da % 4) == 0 && ((uintptr_t)grads[l].dW0 % 4) == 0,
                    KGE_EINVAL, "layer %d: NULL or misaligned gradient pointer", l);
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace;
    const int bf = msg_dtype == KGE_MSG_BF16;
    float *G = (float *)(ws + w.off_G);
    void *dP = ws + w.off_dP;
    float *dHbuf[2] = {(float *)(ws + w.off_dHa), (float *)(ws + w.off_dHb)};
    float *seg = (float *)(ws + w.off_seg);
    float *part = (float *)(ws + w.off_part);
    const float *gin = dH_out;
    for (int l = n_layers - 1; l >= 0; --l) {
        const kge_layer &L = layers[l];
        const void *P = ws + w.off_P[l];
        const float *Hl = (const float *)(ws + w.off_H[l]);
        const float *Hprev = L.dropout > 0.0f ? (const float *)(ws + w.off_Hd[l])
                                              : l > 0 ? (const float *)(ws + w.off_H[l - 1]) : H0;
        const float *Gl = gin;
        bool g_bf = false;           // the bf16 copy of G is already behind dP's columns
        if (L.act != KGE_ACT_IDENTITY) {
            if (bf) {
                rc = launch_act_backward_append_bf16(gin, Hl, L.act, p->n_vert, L.d_out,
                                                     L.order == KGE_ORDER_RELATION_WEIGHTS ? 0 : L.n_bases, G, dP, st);
                g_bf = true;
            } else {
                rc = launch_act_backward(gin, Hl, L.act, p->n_vert * (int64_t)L.d_out, G, st);
            }
            if (rc != KGE_OK) return rc;
            Gl = G;
        }
        float *C = (float *)(ws + w.off_C);
        if (L.order == KGE_ORDER_RELATION_WEIGHTS) {
            // W_r = sum_b a_rb V_b was applied per (relation, destination) run: dW_r = C_r = sum_runs z^T G,
            // da_rb = <C_r, V_b>, dV_b = sum_r a_rb C_r, dz_s = G_dst W_r^T, dh_j = sum_{e out of j} dz/c + G_j W_0^T
            const int32_t R2 = 2 * p->n_relations;
            const int64_t dd = (int64_t)L.d_in * L.d_out;
            const void *Z = ws + w.off_Z[l];
            void *dZ = ws + w.off_U;
            float *Self = (float *)(ws + w.off_self);
            const bool need_in = l > 0 || dH0;
            float *dst = l > 0 ? dHbuf[l & 1] : dH0;
            if (bf) {
                if (!g_bf) rc = launch_append_g_bf16(Gl, p->n_vert, L.d_out, 0, dP, st);          // Gbf [N][d_out]
                if (rc != KGE_OK) return rc;
                rc = launch_rel_outer_bf16(p, p->seg_zrow ? ws + w.off_Hbf[l] : Z, p->seg_zrow, dP, L.d_out, L.d_in, L.d_out, C, st);
            } else {
                rc = launch_rel_outer(p, (const float *)Z, Gl, L.d_in, L.d_out, C, st);
            }
            if (rc != KGE_OK) return rc;
            rc = launch_coeff_contract(p, C, L.V, L.d_in, L.d_out, L.n_bases, grads[l].da, st);
            if (rc != KGE_OK) return rc;
            rc = launch_basis_grad_from_relations(L.a, R2, L.n_bases, C, dd, grads[l].dV, st);
            if (rc != KGE_OK) return rc;
            if (bf) rc = launch_weight_grad_bf16(ws + w.off_Hbf[l], p->n_vert, L.d_in, L.d_out, 0, dP, grads[l].dV, grads[l].dW0, st);
            else rc = launch_weight_grad(Hprev, p->n_vert, L.d_in, L.d_out, 0, nullptr, Gl, grads[l].dV, grads[l].dW0, st);
            if (rc != KGE_OK) return rc;
            if (need_in) {
                if (bf) {
                    rc = launch_input_grad_bf16(dP, p->n_vert, L.d_in, L.d_out, 0, ws + w.off_Wbf[l], Self, st);
                    if (rc != KGE_OK) return rc;
                    rc = launch_apply_relation_weights_t_bf16(p, dP, L.d_out, ws + w.off_Wrb[l], L.d_in, L.d_out, dZ, st);
                } else {
                    rc = launch_input_grad(nullptr, Gl, p->n_vert, L.d_in, L.d_out, 0, L.V, L.W0, Self, st);
                    if (rc != KGE_OK) return rc;
                    rc = launch_apply_relation_weights_t(p, Gl, (const float *)(ws + w.off_Wrel[l]), L.d_in, L.d_out,
                                                         (float *)dZ, st);
                }
                if (rc != KGE_OK) return rc;
                rc = launch_sum_edges_out(p, dZ, bf, L.d_in, Self, dst, part, kge_cgraph_layer(cg, l - 1), st);
                if (rc != KGE_OK) return rc;
                if (L.dropout > 0.0f) {
                    rc = launch_dropout(dst, p->n_vert, L.d_in, L.dropout, L.drop_seed, L.drop_step, l, dst, st);
                    if (rc != KGE_OK) return rc;
                }
                gin = dst;
            }
            continue;
        }
        rc = launch_coeff_grad(p, P, bf, Gl, L.n_bases, L.d_out, seg, part, grads[l].da, kge_cgraph_layer(cg, l), st);
        if (rc != KGE_OK) return rc;
        const int64_t bd = (int64_t)L.n_bases * L.d_out;
        if (bf && gather_transpose_bf16_supported(L.n_bases, L.d_out)) {
            // the bf16 copy of G first (behind the dP columns of the same matrix): the transposed sums gather it
            if (!g_bf) rc = launch_append_g_bf16(Gl, p->n_vert, L.d_out, L.n_bases, dP, st);
            if (rc != KGE_OK) return rc;
            rc = launch_gather_transpose_bf16(p, (const uint16_t *)dP + bd, bd + L.d_out, L.a, L.n_bases, L.d_out, dP,
                                              bd + L.d_out, part, kge_cgraph_layer(cg, l), st);
            if (rc != KGE_OK) return rc;
        } else {
            rc = launch_gather_transpose(p, Gl, L.a, L.n_bases, L.d_out, dP, bf ? bd + L.d_out : bd, bf, part,
                                         kge_cgraph_layer(cg, l), st);
            if (rc != KGE_OK) return rc;
            if (bf && !g_bf) rc = launch_append_g_bf16(Gl, p->n_vert, L.d_out, L.n_bases, dP, st);
            if (rc != KGE_OK) return rc;
        }
        if (bf) {
            rc = launch_weight_grad_bf16(ws + w.off_Hbf[l], p->n_vert, L.d_in, L.d_out, L.n_bases, dP,
                                         grads[l].dV, grads[l].dW0, st);
        } else {
            rc = launch_weight_grad(Hprev, p->n_vert, L.d_in, L.d_out, L.n_bases, (const float *)dP, Gl,
                                    grads[l].dV, grads[l].dW0, st);
        }
        if (rc != KGE_OK) return rc;
        if (l > 0 || dH0) {
            float *dst = l > 0 ? dHbuf[l & 1] : dH0;
            if (bf) rc = launch_input_grad_bf16(dP, p->n_vert, L.d_in, L.d_out, L.n_bases, ws + w.off_Wbf[l], dst, st);
            else rc = launch_input_grad((const float *)dP, Gl, p->n_vert, L.d_in, L.d_out, L.n_bases, L.V, L.W0, dst, st);
            if (rc != KGE_OK) return rc;
            if (L.dropout > 0.0f) {      // chain rule through out = mask * h / (1 - p): the same mask and scale
                rc = launch_dropout(dst, p->n_vert, L.d_in, L.dropout, L.drop_seed, L.drop_step, l, dst, st);
                if (rc != KGE_OK) return rc;
            }
            gin = dst;
        }
    }
    return KGE_OK;
}

extern "C" int kge_sample_negatives(const kge_partition *p, const int32_t *pos_core_idx, int64_t n_pos,
                                    int32_t n_neg, int32_t mode, uint64_t seed, uint64_t step,
                                    int32_t *neg_ent, uint8_t *neg_side, void *stream)
{
    KGE_REQUIRE(p, KGE_EINVAL, "NULL partition");
    KGE_REQUIRE(n_pos >= 0 && n_neg >= 0, KGE_EINVAL, "negative count");
    KGE_REQUIRE(mode == KGE_NEG_TAIL || mode == KGE_NEG_HEAD_OR_TAIL, KGE_EINVAL, "bad mode");
    KGE_REQUIRE(n_pos * (int64_t)n_neg == 0 || (pos_core_idx && neg_ent && neg_side), KGE_EINVAL, "NULL array");
    return launch_sample_negatives(p, pos_core_idx, n_pos, n_neg, mode, seed, step, neg_ent, neg_side,
                                   (hipStream_t)stream);
}

extern "C" int kge_distmult_score_loss(const kge_partition *p, kge_score_index *index, const float *H, const float *M,
                                       int32_t d, const int32_t *pos_core_idx, int64_t n_pos, const int32_t *neg_ent,
                                       const uint8_t *neg_side, int32_t n_neg, float *scores, float *loss,
                                       float *dH, float *dM, void *stream)
{
    KGE_REQUIRE(p && H && M && loss && dH && dM, KGE_EINVAL, "NULL argument");
    KGE_REQUIRE(d > 0 && d <= 512 && d % 4 == 0, KGE_EINVAL, "d must be a multiple of 4 in [4, 512]");
    KGE_REQUIRE(n_pos >= 0 && n_neg >= 0, KGE_EINVAL, "negative count");
    KGE_REQUIRE(n_pos == 0 || pos_core_idx, KGE_EINVAL, "pos_core_idx is NULL");
    KGE_REQUIRE(n_pos * (int64_t)n_neg == 0 || (neg_ent && neg_side), KGE_EINVAL, "negatives are NULL");
    KGE_REQUIRE(n_pos == 0 || p->n_core > 0, KGE_EINVAL, "the partition has no core edge to score");
    KGE_REQUIRE(((uintptr_t)dH % 4) == 0 && ((uintptr_t)dM % 4) == 0 && ((uintptr_t)loss % 4) == 0, KGE_EINVAL,
                "misaligned output");
    if (index)
        return launch_distmult_indexed(p, index, H, M, d, pos_core_idx, n_pos, neg_ent, neg_side, n_neg, scores, loss,
                                       dH, dM, (hipStream_t)stream);
    return launch_distmult(p, H, M, d, pos_core_idx, n_pos, neg_ent, neg_side, n_neg, scores, loss, dH, dM,
                           (hipStream_t)stream);
}
