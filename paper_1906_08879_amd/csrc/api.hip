// C ABI of the library (declared in include/placeto.h): handles, uploads, scratch buffers
// and the sequence of kernel launches that makes one policy forward pass (Section 2.2
// steps 1-3 and the policy head of Appendix A.7).
#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "internal.h"

// Intermediate buffers of pl_embed_forward_static: device memory that exists from the moment the
// library is loaded on a device, 32 MiB per device, shared by every call on that device.
static __device__ __align__(256) unsigned char scratch[static_cast<size_t>(32) << 20];

namespace pl {

namespace {
thread_local std::string g_error;
}

void set_error(const std::string &msg) { g_error = msg; }

int fail(int code, const std::string &msg)
{
    g_error = msg;
    return code;
}

int hip_fail(hipError_t e, const char *what)
{
    g_error = std::string(what) + ": " + hipGetErrorString(e);
    (void)hipGetLastError();
    return PL_ERR_HIP;
}

namespace {

template <typename T>
int upload(const std::vector<T> &host, T **dev)
{
    *dev = nullptr;
    const size_t bytes = sizeof(T) * (host.empty() ? 1 : host.size());
    PL_HIP(hipMalloc(reinterpret_cast<void **>(dev), bytes));
    if (!host.empty())
        PL_HIP(hipMemcpy(*dev, host.data(), sizeof(T) * host.size(), hipMemcpyHostToDevice));
    return PL_OK;
}

struct StageTimer {
    std::vector<hipEvent_t> ev[PL_STAGE_COUNT];   // start/stop pairs not yet read
    std::vector<hipEvent_t> pool;                 // created events that are free for reuse
    double ms_sum[PL_STAGE_COUNT] = {};
    int64_t launches[PL_STAGE_COUNT] = {};
    bool on = false;

    // An event from the pool (filled when timing is switched on, so that no event is created
    // between two timed launches), or a new one when the pool is empty.
    bool take(hipEvent_t *e)
    {
        if (!pool.empty()) {
            *e = pool.back();
            pool.pop_back();
            return true;
        }
        return hipEventCreate(e) == hipSuccess;
    }
};

}  // namespace
}  // namespace pl

struct pl_graph_batch {
    pl::HostLayout host;
    bool on_device = false;
    int device = -1;
    // device arrays
    int32_t *d_node_off = nullptr, *d_lvl_off = nullptr, *d_node_graph = nullptr;
    int32_t *d_nbr_ptr[2] = {nullptr, nullptr}, *d_nbr_idx[2] = {nullptr, nullptr};
    int32_t *d_order[2] = {nullptr, nullptr}, *d_lvl_ptr[2] = {nullptr, nullptr};
    int32_t *d_ck_off[2] = {nullptr, nullptr}, *d_ck_ovf[2] = {nullptr, nullptr};
    int32_t *d_pos[2] = {nullptr, nullptr}, *d_tmpl = nullptr;
    uint32_t *d_ck_rec[2] = {nullptr, nullptr};
    pl::GraphView view{};
    pl::Workspace ws;
    pl::GradWorkspace gw;
    // timeline of the simulator (pl_simulate_reward): op_start, op_end [n_tot]; arrival, alloc, free
    // [n_tot, sim_D]; run times [B]
    float *sim_start = nullptr, *sim_end = nullptr, *sim_arrival = nullptr, *sim_arrival_last = nullptr,
          *sim_alloc = nullptr, *sim_free = nullptr, *sim_rt = nullptr;
    int sim_D = 0;
    pl::StageTimer timer;
};

struct pl_weights {
    pl_model_cfg cfg{};
    pl::ModelView view{};
    float *d_blob = nullptr;
    float *d_blob_t = nullptr;      // same offsets, every matrix transposed to [out, in] (gradient pass)
    std::vector<float> host_blob;   // values as stored (bf16-rounded when asked)
    // matrix-core sweep: packed A fragments and biases (null when the shape is not covered)
    uint16_t *d_wfrag = nullptr;
    uint16_t *d_wfrag_bw = nullptr;  // the same for the reverse pass (transposed, f before g)
    float *d_sweep_bias = nullptr;
    uint16_t *d_pool_frag = nullptr;
    uint16_t *d_pool_afrag = nullptr;   // the streaming pooling kernel's fragments (null when not covered)
    uint16_t *d_pool_bwfrag = nullptr;  // ... and those of its reverse
    float *d_pool_bias = nullptr;
    int sweep_ws = 0;               // bf16 parts per weight: 1 (bf16 weights) or 3 (fp32)
    int path = 0;                   // 0 = fastest available kernels, 1 = generic fp32 kernels
};

namespace pl {
namespace {

bool cfg_ok(const pl_model_cfg *c)
{
    return c && c->D >= 1 && c->D <= kMaxD && c->H >= 1 && c->H <= kMaxH && c->n_layers >= 1 &&
           c->n_layers <= kMaxLayers && c->k_sweeps >= 0 && c->k_sweeps <= kMaxSweeps &&
           (c->group_by_device == 0 || c->group_by_device == 1) &&
           (c->single_set == 0 || c->single_set == 1) &&
           (c->weight_dtype == PL_WEIGHTS_FP32 || c->weight_dtype == PL_WEIGHTS_BF16);
}

// Lays out the blob: fills every LayerRef and returns the total number of floats.
size_t plan_weights(const pl_model_cfg &c, ModelView *mv)
{
    ModelView m{};
    m.D = c.D;
    m.H = c.H;
    m.L = c.n_layers;
    m.G = c.group_by_device ? c.D : 1;
    m.F = c.D + 4;
    m.single_set = c.single_set;
    m.Z = (2 + 3 * m.G) * c.H;
    size_t pos = 0;
    auto take = [&pos](int n_in, int n_out) {
        LayerRef r;
        r.w = static_cast<int32_t>(pos);
        r.b = static_cast<int32_t>(pos + static_cast<size_t>(n_in) * n_out);
        r.n_in = n_in;
        r.n_out = n_out;
        pos += static_cast<size_t>(n_in) * n_out + n_out;
        return r;
    };
    auto take_mlp = [&](int n_in) {
        MlpRef r{};
        for (int l = 0; l < c.n_layers; ++l) r.layer[l] = take(l == 0 ? n_in : c.H, c.H);
        return r;
    };
    m.proj = take(m.F, c.H);
    m.f[0] = take_mlp(c.H);
    m.g[0] = take_mlp(c.H);
    m.f[1] = take_mlp(c.H);
    m.g[1] = take_mlp(c.H);
    for (int i = 0; i < 3; ++i) m.l[i] = take_mlp(2 * c.H);
    for (int i = 0; i < 3; ++i) m.h[i] = take_mlp(c.H);
    m.pol1 = take(m.Z, c.H);
    m.pol2 = take(c.H, c.D);
    if (mv) *mv = m;
    return pos;
}

// fp32 -> nearest bfloat16 (ties to even), returned widened back to fp32.
float round_bf16(float x)
{
    uint32_t u;
    std::memcpy(&u, &x, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return x;   // inf / nan unchanged
    u += 0x7FFFu + ((u >> 16) & 1u);
    u &= 0xFFFF0000u;
    std::memcpy(&x, &u, 4);
    return x;
}

void round_layer(std::vector<float> &blob, const LayerRef &r)
{
    for (int64_t i = 0; i < static_cast<int64_t>(r.n_in) * r.n_out; ++i)
        blob[r.w + i] = round_bf16(blob[r.w + i]);
}

int upload_batch(pl_graph_batch *g);

// Device copies of the batch's index data, made once.  Host allocations of the conversion are
// guarded: no exception crosses the C boundary.
int ensure_on_device(pl_graph_batch *g)
{
    if (g->on_device) return PL_OK;
    try {
        return upload_batch(g);
    } catch (const std::bad_alloc &) {
        return fail(PL_ERR_NOMEM, "out of host memory");
    }
}

int upload_batch(pl_graph_batch *g)
{
    const HostLayout &L = g->host;
    PL_HIP(hipGetDevice(&g->device));
    std::vector<int32_t> node_off(L.node_off.begin(), L.node_off.end());
    std::vector<int32_t> lvl_off(L.lvl_off.begin(), L.lvl_off.end());
    std::vector<int32_t> node_graph(L.n_tot);
    std::vector<int32_t> ptr[2], idx[2], order[2], lvl[2];
    for (int dir = 0; dir < 2; ++dir) {
        const auto &hp = dir ? L.chi_ptr : L.par_ptr;
        const auto &hi = dir ? L.chi_idx : L.par_idx;
        const auto &ho = dir ? L.bu_order : L.td_order;
        const auto &hl = dir ? L.bu_lvl_ptr : L.td_lvl_ptr;
        ptr[dir].assign(hp.begin(), hp.end());
        idx[dir].resize(L.e_tot);
        order[dir].resize(L.n_tot);
        lvl[dir].resize(hl.size());
        for (int32_t b = 0; b < L.B; ++b) {
            const int32_t n0 = static_cast<int32_t>(L.node_off[b]);
            for (int64_t v = L.node_off[b]; v < L.node_off[b + 1]; ++v) {
                node_graph[v] = b;
                order[dir][v] = n0 + ho[v];
                for (int64_t p = hp[v]; p < hp[v + 1]; ++p) idx[dir][p] = n0 + hi[p];
            }
            for (int64_t q = L.lvl_off[b]; q < L.lvl_off[b + 1]; ++q) lvl[dir][q] = n0 + hl[q];
        }
    }
    int rc;
    if ((rc = upload(node_off, &g->d_node_off))) return rc;
    if ((rc = upload(lvl_off, &g->d_lvl_off))) return rc;
    if ((rc = upload(node_graph, &g->d_node_graph))) return rc;
    if ((rc = upload(L.tmpl, &g->d_tmpl))) return rc;
    for (int dir = 0; dir < 2; ++dir) {
        if ((rc = upload(ptr[dir], &g->d_nbr_ptr[dir]))) return rc;
        if ((rc = upload(idx[dir], &g->d_nbr_idx[dir]))) return rc;
        if ((rc = upload(order[dir], &g->d_order[dir]))) return rc;
        if ((rc = upload(lvl[dir], &g->d_lvl_ptr[dir]))) return rc;
        SweepPlanHost plan;
        if ((rc = build_sweep_plan(L, dir, &plan))) return rc;
        if ((rc = upload(plan.ck_off, &g->d_ck_off[dir]))) return rc;
        if ((rc = upload(plan.rec, &g->d_ck_rec[dir]))) return rc;
        if ((rc = upload(plan.ovf, &g->d_ck_ovf[dir]))) return rc;
        std::vector<int32_t> pos(L.n_tot);
        for (int64_t p = 0; p < L.n_tot; ++p) pos[order[dir][p]] = static_cast<int32_t>(p);
        if ((rc = upload(pos, &g->d_pos[dir]))) return rc;
    }
    GraphView &v = g->view;
    v.B = L.B;
    v.n_tot = static_cast<int32_t>(L.n_tot);
    v.node_off = g->d_node_off;
    v.lvl_off = g->d_lvl_off;
    v.node_graph = g->d_node_graph;
    v.tmpl = g->d_tmpl;
    for (int dir = 0; dir < 2; ++dir) {
        v.nbr_ptr[dir] = g->d_nbr_ptr[dir];
        v.nbr_idx[dir] = g->d_nbr_idx[dir];
        v.order[dir] = g->d_order[dir];
        v.lvl_ptr[dir] = g->d_lvl_ptr[dir];
        v.plan[dir].ck_off = g->d_ck_off[dir];
        v.plan[dir].rec = reinterpret_cast<const uint4 *>(g->d_ck_rec[dir]);
        v.plan[dir].ovf = g->d_ck_ovf[dir];
        v.pos[dir] = g->d_pos[dir];
    }
    g->on_device = true;
    return PL_OK;
}

void free_workspace(Workspace &ws)
{
    (void)hipFree(ws.base);
    (void)hipFree(ws.reach);
    ws = Workspace();
}

// Lays the intermediate buffers of one forward pass out in one block starting at `base` (which
// may be null: then only the size is computed) and returns the block's size in bytes.  Every
// buffer starts on a 256-byte boundary.  With `with_reach` the reachability bytes are part of
// the block, otherwise ws->reach is left alone.
// Rows past the data (matrix-core sweep): emb row n, msg row 2n + 1, xb row 2n and reach byte
// 2n + 1 take the stores of a chunk's unused rows; msg row 2n and reach byte 2n are never
// written, must read as zero, and are the target of dummy loads.
size_t carve_workspace(unsigned char *base, size_t n, size_t B, const ModelView &mv, bool with_reach, Workspace *ws)
{
    size_t at = 0;
    auto take = [&](size_t bytes) {
        unsigned char *p = base ? base + at : nullptr;
        at += (bytes + 255) / 256 * 256;
        return p;
    };
    const size_t H = mv.H;
    ws->n_chunks = 8;
    ws->emb = reinterpret_cast<float *>(take(sizeof(float) * ((n + 1) * 2 * H + 4)));
    ws->msg = reinterpret_cast<float *>(take(sizeof(float) * ((2 * n + 2) * H + 4)));
    ws->xb = reinterpret_cast<float *>(take(sizeof(float) * ((2 * n + 1) * H + 4)));
    ws->featb = reinterpret_cast<float4 *>(take(sizeof(float4) * (n + 1)));
    ws->partial = reinterpret_cast<float *>(take(sizeof(float) * (B * ws->n_chunks * 3 * mv.G * H + 4)));
    ws->zbuf = reinterpret_cast<float *>(take(sizeof(float) * (B * mv.Z + 4)));
    ws->hidp = reinterpret_cast<double *>(take(sizeof(double) * (static_cast<size_t>((mv.Z + 255) / 256) * B * H + 4)));
    ws->klist = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (n + 16)));
    ws->koff = reinterpret_cast<int32_t *>(take(sizeof(int32_t) * (B * (3 * kMaxD + 1) + 4)));
    if (with_reach) ws->reach = take(2 * n + 32);
    ws->H = mv.H;
    ws->G = mv.G;
    return at;
}

void free_grad_workspace(GradWorkspace &gw)
{
    float *all[] = {gw.fact, gw.gact, gw.agg, gw.dagg, gw.dfg, gw.keep, gw.snap_emb, gw.snap_msg, gw.lact, gw.dl, gw.demb, gw.dx, gw.phi,
                    gw.pooled, gw.dP, gw.hin, gw.hact, gw.dh, gw.dz, gw.hid, gw.dpre, gw.dlogit, gw.partial};
    for (float *p : all) (void)hipFree(p);
    (void)hipFree(gw.cls);
    (void)hipFree(gw.mask4);
    (void)hipFree(gw.counts);
    (void)hipFree(gw.blk_cnt);
    (void)hipFree(gw.lists);
    gw = GradWorkspace();
}

int ensure_reach(pl_graph_batch *g)
{
    if (g->ws.reach) return PL_OK;
    const size_t n = static_cast<size_t>(g->host.n_tot);
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->ws.reach), 2 * n + 16));
    PL_HIP(hipMemset(g->ws.reach, 0, 2 * n + 16));
    return PL_OK;
}

int ensure_workspace(pl_graph_batch *g, const ModelView &mv)
{
    Workspace &ws = g->ws;
    if (ws.emb && ws.H == mv.H && ws.G == mv.G) return PL_OK;
    uint8_t *keep = ws.reach;
    ws.reach = nullptr;
    free_workspace(ws);
    ws.reach = keep;
    const size_t n = static_cast<size_t>(g->host.n_tot), B = static_cast<size_t>(g->host.B);
    int rc = ensure_reach(g);
    if (rc) return rc;
    Workspace sized;
    const size_t bytes = carve_workspace(nullptr, n, B, mv, false, &sized);
    unsigned char *base = nullptr;
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&base), bytes));
    ws.base = base;
    carve_workspace(base, n, B, mv, false, &ws);
    PL_HIP(hipMemset(ws.msg, 0, sizeof(float) * ((2 * n + 2) * mv.H + 4)));
    return PL_OK;
}

int ensure_grad_workspace(pl_graph_batch *g, const ModelView &mv)
{
    GradWorkspace &gw = g->gw;
    if (gw.demb && gw.H == mv.H && gw.G == mv.G && gw.L == mv.L && gw.D == mv.D) return PL_OK;
    free_grad_workspace(gw);
    const size_t n = static_cast<size_t>(g->host.n_tot), H = mv.H, L = mv.L, B = g->host.B;
    const size_t NH = n * H, BG = B * mv.G;
    auto take = [](float **p, size_t floats) {
        return hipMalloc(reinterpret_cast<void **>(p), sizeof(float) * (floats + 4));
    };
    PL_HIP(take(&gw.fact, 2 * L * NH));
    PL_HIP(take(&gw.gact, 2 * L * NH));
    PL_HIP(take(&gw.agg, 2 * NH));
    // the matrix-core chain kernel reads row 2 n of dagg as an all-zero row and stores the rows
    // of unused chunk slots to row 2 n + 1, to row n of demb and to the spare floats of dfg
    PL_HIP(take(&gw.dagg, 2 * NH + 2 * H));
    PL_HIP(hipMemset(gw.dagg, 0, sizeof(float) * (2 * NH + 2 * H)));
    gw.dfg_stride = 2 * L * NH + H;
    PL_HIP(take(&gw.dfg, 2 * gw.dfg_stride));
    PL_HIP(take(&gw.keep, 2 * gw.dfg_stride));
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&gw.mask4), 2 * NH + H + 16));
    PL_HIP(take(&gw.lact, L * NH));
    PL_HIP(take(&gw.dl, L * NH));
    PL_HIP(take(&gw.demb, 2 * NH + 2 * H));
    PL_HIP(take(&gw.dx, NH));
    PL_HIP(take(&gw.phi, n * 32));   // F <= 20 columns, padded to 32 on the matrix-core path
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&gw.cls), n + 16));
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&gw.counts), 64));
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&gw.blk_cnt), sizeof(int32_t) * (3 * ((n + 255) / 256) + 4)));
    PL_HIP(hipMalloc(reinterpret_cast<void **>(&gw.lists), sizeof(int32_t) * (3 * n + 4)));
    PL_HIP(take(&gw.pooled, 3 * BG * H));
    PL_HIP(take(&gw.dP, 3 * BG * H));
    PL_HIP(take(&gw.hin, 3 * BG * H));
    PL_HIP(take(&gw.hact, 3 * L * BG * H));
    PL_HIP(take(&gw.dh, 3 * L * BG * H));
    PL_HIP(take(&gw.dz, B * mv.Z));
    PL_HIP(take(&gw.hid, B * H));
    PL_HIP(take(&gw.dpre, B * H));
    PL_HIP(take(&gw.dlogit, B * mv.D));
    // (three times: the gradients of l's layers are taken for the three node sets in one launch)
    size_t part = 3 * wgrad_partial_floats(static_cast<int64_t>(n), 2 * mv.H, mv.H);
    part = std::max(part, wgrad_partial_floats(static_cast<int64_t>(n), 32, mv.H));
    part = std::max(part, wgrad_partial_floats(static_cast<int64_t>(BG), mv.H, mv.H));
    part = std::max(part, wgrad_partial_floats(static_cast<int64_t>(B), mv.Z, mv.H));
    part = std::max(part, wgrad_partial_floats(static_cast<int64_t>(B), mv.H, mv.D));
    PL_HIP(take(&gw.partial, part));
    gw.H = mv.H;
    gw.G = mv.G;
    gw.L = mv.L;
    gw.D = mv.D;
    return PL_OK;
}

// PL_VALIDATE=1 in the environment: the device-resident state of a call is copied to the host
// and range-checked before any kernel is launched (a debugging aid: it synchronises the stream).
bool validate_enabled()
{
    const char *e = std::getenv("PL_VALIDATE");
    return e && e[0] == '1' && e[1] == '\0';
}

// allow_finished: a cur_node of -1 (the marker pl_episode_step leaves when a graph's episode is
// over) is accepted, and so is an action of -1 for such a graph.
int validate_state(const pl_graph_batch *g, int D, const int32_t *placement, const int32_t *cur_node,
                   const int32_t *actions, bool allow_finished, hipStream_t s)
{
    try {
        const HostLayout &L = g->host;
        std::vector<int32_t> pl_h(static_cast<size_t>(L.n_tot)), cur_h(static_cast<size_t>(L.B)), act_h;
        PL_HIP(hipStreamSynchronize(s));
        if (placement)
            PL_HIP(hipMemcpy(pl_h.data(), placement, sizeof(int32_t) * pl_h.size(), hipMemcpyDeviceToHost));
        if (cur_node)
            PL_HIP(hipMemcpy(cur_h.data(), cur_node, sizeof(int32_t) * cur_h.size(), hipMemcpyDeviceToHost));
        if (actions) {
            act_h.resize(static_cast<size_t>(L.B));
            PL_HIP(hipMemcpy(act_h.data(), actions, sizeof(int32_t) * act_h.size(), hipMemcpyDeviceToHost));
        }
        if (placement)
            for (int64_t v = 0; v < L.n_tot; ++v)
                if (pl_h[v] < 0 || pl_h[v] >= D)
                    return fail(PL_ERR_RANGE, "PL_VALIDATE: placement[" + std::to_string(v) + "] = " +
                                                  std::to_string(pl_h[v]) + " is outside [0, " + std::to_string(D) + ")");
        for (int32_t b = 0; b < L.B; ++b) {
            const int64_t n_b = L.node_off[b + 1] - L.node_off[b];
            const bool finished = allow_finished && cur_node && cur_h[b] == -1;
            if (finished) continue;
            if (cur_node && (cur_h[b] < 0 || cur_h[b] >= n_b))
                return fail(PL_ERR_RANGE, "PL_VALIDATE: cur_node[" + std::to_string(b) + "] = " +
                                              std::to_string(cur_h[b]) + " is outside the graph's " +
                                              std::to_string(n_b) + " nodes");
            if (actions && (act_h[b] < 0 || act_h[b] >= D))
                return fail(PL_ERR_RANGE, "PL_VALIDATE: actions[" + std::to_string(b) + "] = " +
                                              std::to_string(act_h[b]) + " is outside [0, " + std::to_string(D) + ")");
        }
    } catch (const std::bad_alloc &) {
        return fail(PL_ERR_NOMEM, "out of host memory");
    }
    return PL_OK;
}

struct StageScope {
    StageTimer &t;
    int stage;
    hipStream_t s;
    StageScope(StageTimer &timer, int st, hipStream_t stream) : t(timer), stage(st), s(stream)
    {
        if (!t.on) return;
        hipEvent_t e;
        if (t.take(&e)) {
            (void)hipEventRecord(e, s);
            t.ev[stage].push_back(e);
        }
    }
    ~StageScope()
    {
        if (!t.on || (t.ev[stage].size() & 1u) == 0) return;
        hipEvent_t e;
        if (t.take(&e)) {
            (void)hipEventRecord(e, s);
            t.ev[stage].push_back(e);
        } else {
            t.pool.push_back(t.ev[stage].back());
            t.ev[stage].pop_back();
        }
    }
};

// Nodes and edges of the batch's largest graph.
struct GraphExtent {
    int n_max, e_max;
};
GraphExtent graph_extent(const HostLayout &h)
{
    int64_t n_max = 0, e_max = 0;
    for (int32_t b = 0; b < h.B; ++b) {
        n_max = std::max<int64_t>(n_max, h.node_off[b + 1] - h.node_off[b]);
        e_max = std::max<int64_t>(e_max, h.edge_off[b + 1] - h.edge_off[b]);
    }
    return {static_cast<int>(n_max), static_cast<int>(e_max)};
}

// StageMarks hook over a batch's timer: an event at the beginning and at the end of a stage.
void stage_mark(void *ctx, int stage, bool begin, hipStream_t s)
{
    StageTimer &t = *static_cast<StageTimer *>(ctx);
    if (!t.on) return;
    auto &ev = t.ev[stage];
    if (!begin && (ev.size() & 1u) == 0) return;    // no open pair
    hipEvent_t e;
    if (t.take(&e)) {
        (void)hipEventRecord(e, s);
        ev.push_back(e);
    } else if (!begin) {
        t.pool.push_back(ev.back());
        ev.pop_back();
    }
}

// static_ws: the intermediate buffers of a call that must not allocate (the batch is on the
// device already, stage timing is off); otherwise the batch's own buffers are used, allocated on
// the first call.
int forward_impl(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                 const int32_t *cur_node, const pl_weights *w, float *out_logits, float *out_probs,
                 float *out_node_emb, float *out_pooled, uint8_t *out_class, void *stream, bool validate,
                 float *keep = nullptr, size_t keep_stride = 0, float *keep_pool = nullptr,
                 bool *pool_kept = nullptr, float *snap_emb = nullptr, float *snap_msg = nullptr,
                 const Workspace *static_ws = nullptr, uint8_t *gates = nullptr)
{
    if (!g || !w) return fail(PL_ERR_NULL, "graph batch or weights handle is NULL");
    if (g->host.B == 0) return PL_OK;
    if (!node_feats || !placement || !cur_node || !out_logits)
        return fail(PL_ERR_NULL, "node_feats, placement, cur_node and out_logits are required");
    hipStream_t s = static_cast<hipStream_t>(stream);
    int rc;
    if (validate && validate_enabled() &&
        (rc = validate_state(g, w->cfg.D, placement, cur_node, nullptr, false, s)))
        return rc;
    const ModelView &mv = w->view;
    if (!static_ws) {
        if ((rc = ensure_on_device(g))) return rc;
        if ((rc = ensure_workspace(g, mv))) return rc;
    }
    const Workspace &ws = static_ws ? *static_ws : g->ws;
    StageTimer off;
    StageTimer &timer = static_ws ? off : g->timer;
    ForwardArgs fa{node_feats, placement, cur_node, out_logits, out_probs, out_pooled};
    const GraphView &gv = g->view;
    // the matrix-core sweep addresses its buffers with 32-bit offsets
    const bool fits32 = (static_cast<double>(g->host.n_tot) + 2) * 2 * mv.H * sizeof(float) < 4.0e9;
    const bool mfma = w->d_wfrag && w->path == 0 && w->cfg.k_sweeps > 0 && fits32;
    {
        // the matrix-core sweep computes x_v itself from the raw features (first sweep)
        StageScope scope(timer, PL_STAGE_PROJECT, s);
        if (!mfma) launch_project(gv, mv, ws, fa, true, false, s);
    }
    {
        StageScope scope(timer, PL_STAGE_SWEEP, s);
        // without sweeps the node sets still need reachability from v*, unless there is one set
        // (one set without sweeps needs none, unless the caller asks for the sets themselves)
        if (w->cfg.k_sweeps == 0 && (!w->cfg.single_set || out_class)) {
            const GraphExtent x = graph_extent(g->host);
            launch_reach_only(gv, cur_node, ws.reach, x.n_max, x.e_max, g->host.max_depth, s);
        }
        for (int k = 0; k < w->cfg.k_sweeps; ++k) {
            if (mfma)
                launch_sweep_mfma(gv, mv, ws, fa, reinterpret_cast<const uint4 *>(w->d_wfrag),
                                  w->d_sweep_bias, w->sweep_ws, k == 0, k + 1 < w->cfg.k_sweeps, keep, keep_stride,
                                  gates, s);
            else
                launch_sweep_generic(gv, mv, ws, fa, k == 0, s);
            if (snap_emb && k + 1 < w->cfg.k_sweeps) {
                // the reverse pass of a multi-sweep network needs the states and messages after this sweep
                const size_t span = static_cast<size_t>(g->host.n_tot) * 2 * mv.H;
                PL_HIP(hipMemcpyAsync(snap_emb + k * span, ws.emb, sizeof(float) * span, hipMemcpyDeviceToDevice, s));
                PL_HIP(hipMemcpyAsync(snap_msg + k * span, ws.msg, sizeof(float) * span, hipMemcpyDeviceToDevice, s));
            }
        }
    }
    // the node sets as the pooling below reads them: from the reachability bits the sweeps left
    if (out_class) launch_classes(gv, cur_node, ws.reach, out_class, s);
    const bool pool_mfma = w->d_pool_frag && w->path == 0;
    int pool_slices = ws.n_chunks;
    {
        StageScope scope(timer, PL_STAGE_POOL, s);
        if (pool_mfma)
            pool_slices = launch_pool_mfma(gv, mv, ws, fa, reinterpret_cast<const uint4 *>(w->d_pool_frag),
                                           reinterpret_cast<const uint4 *>(w->d_pool_afrag), w->d_pool_bias,
                                           w->sweep_ws, keep_pool, s);
        else
            launch_pool_generic(gv, mv, ws, fa, s);
        if (pool_kept) *pool_kept = pool_mfma && keep_pool;
    }
    {
        StageScope scope(timer, PL_STAGE_HEAD, s);
        launch_head_generic(gv, mv, ws, fa, pool_slices, s);
    }
    if (out_node_emb)
        PL_HIP(hipMemcpyAsync(out_node_emb, ws.emb,
                              sizeof(float) * static_cast<size_t>(g->host.n_tot) * 2 * mv.H,
                              hipMemcpyDeviceToDevice, s));
    PL_HIP(hipGetLastError());
    return PL_OK;
}

// ---- intermediate buffers for callers that cannot allocate: one fixed block per device
constexpr size_t kStaticScratchBytes = static_cast<size_t>(32) << 20;
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch`, looked up once per device.
int scratch_address(void **out)
{
    int dev = -1;
    PL_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return fail(PL_ERR_SHAPE, "device index beyond the supported range");
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        PL_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return PL_OK;
}

}  // namespace
}  // namespace pl

using namespace pl;

extern "C" {

int pl_graph_batch_create(int32_t B, const int32_t *n_nodes, const int32_t *n_edges,
                          const int32_t *edge_src, const int32_t *edge_dst, pl_graph_batch **out)
{
    if (!out) return fail(PL_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (B < 0) return fail(PL_ERR_SHAPE, "B is negative");
    if (B > 0 && (!n_nodes || !n_edges)) return fail(PL_ERR_NULL, "n_nodes / n_edges are NULL");
    pl_graph_batch *g = new (std::nothrow) pl_graph_batch();
    if (!g) return fail(PL_ERR_NOMEM, "out of host memory");
    int rc;
    try {
        rc = build_layout(B, n_nodes, n_edges, edge_src, edge_dst, &g->host);
    } catch (const std::bad_alloc &) {
        rc = fail(PL_ERR_NOMEM, "out of host memory");
    }
    if (rc) {
        delete g;
        return rc;
    }
    *out = g;
    return PL_OK;
}

int pl_graph_batch_create_replicated(int32_t n_nodes, int32_t n_edges, const int32_t *edge_src,
                                     const int32_t *edge_dst, int32_t R, pl_graph_batch **out)
{
    if (!out) return fail(PL_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (R < 1) return fail(PL_ERR_SHAPE, "the number of copies must be at least 1");
    pl_graph_batch *g = new (std::nothrow) pl_graph_batch();
    if (!g) return fail(PL_ERR_NOMEM, "out of host memory");
    int rc;
    try {
        HostLayout one;
        rc = build_layout(1, &n_nodes, &n_edges, edge_src, edge_dst, &one);
        if (!rc) rc = replicate_layout(one, R, &g->host);
    } catch (const std::bad_alloc &) {
        rc = fail(PL_ERR_NOMEM, "out of host memory");
    }
    if (rc) {
        delete g;
        return rc;
    }
    *out = g;
    return PL_OK;
}

int pl_graph_batch_destroy(pl_graph_batch *g)
{
    if (!g) return PL_OK;
    if (g->on_device) {
        (void)hipFree(g->d_node_off);
        (void)hipFree(g->d_lvl_off);
        (void)hipFree(g->d_node_graph);
        (void)hipFree(g->d_tmpl);
        for (int dir = 0; dir < 2; ++dir) {
            (void)hipFree(g->d_nbr_ptr[dir]);
            (void)hipFree(g->d_nbr_idx[dir]);
            (void)hipFree(g->d_order[dir]);
            (void)hipFree(g->d_lvl_ptr[dir]);
            (void)hipFree(g->d_ck_off[dir]);
            (void)hipFree(g->d_ck_rec[dir]);
            (void)hipFree(g->d_ck_ovf[dir]);
            (void)hipFree(g->d_pos[dir]);
        }
    }
    free_workspace(g->ws);
    free_grad_workspace(g->gw);
    for (float *p : {g->sim_start, g->sim_end, g->sim_arrival, g->sim_arrival_last, g->sim_alloc, g->sim_free, g->sim_rt})
        (void)hipFree(p);
    for (auto &v : g->timer.ev)
        for (hipEvent_t e : v) (void)hipEventDestroy(e);
    for (hipEvent_t e : g->timer.pool) (void)hipEventDestroy(e);
    delete g;
    return PL_OK;
}

int pl_graph_batch_info(const pl_graph_batch *g, int32_t *B, int64_t *n_tot, int64_t *e_tot,
                        int32_t *max_depth)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    if (B) *B = g->host.B;
    if (n_tot) *n_tot = g->host.n_tot;
    if (e_tot) *e_tot = g->host.e_tot;
    if (max_depth) *max_depth = g->host.max_depth;
    return PL_OK;
}

int pl_graph_batch_levels(const pl_graph_batch *g, int32_t *td_level, int32_t *bu_level)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    const size_t bytes = sizeof(int32_t) * static_cast<size_t>(g->host.n_tot);
    if (td_level && bytes) std::memcpy(td_level, g->host.td_level.data(), bytes);
    if (bu_level && bytes) std::memcpy(bu_level, g->host.bu_level.data(), bytes);
    return PL_OK;
}

int pl_graph_batch_layout(const pl_graph_batch *g, int64_t *par_ptr, int32_t *par_idx,
                          int64_t *chi_ptr, int32_t *chi_idx, int32_t *td_order,
                          int32_t *bu_order)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    const HostLayout &L = g->host;
    auto copy = [](auto *dst, const auto &src) {
        if (dst && !src.empty()) std::memcpy(dst, src.data(), sizeof(src[0]) * src.size());
    };
    copy(par_ptr, L.par_ptr);
    copy(par_idx, L.par_idx);
    copy(chi_ptr, L.chi_ptr);
    copy(chi_idx, L.chi_idx);
    copy(td_order, L.td_order);
    copy(bu_order, L.bu_order);
    return PL_OK;
}

int pl_node_classes(pl_graph_batch *g, const int32_t *cur_node, uint8_t *out_class, void *stream)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    if (g->host.B == 0) return PL_OK;
    if (!cur_node || !out_class) return fail(PL_ERR_NULL, "cur_node / out_class are NULL");
    int rc = ensure_on_device(g);
    if (rc) return rc;
    if ((rc = ensure_reach(g))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const GraphExtent x = graph_extent(g->host);
    launch_reach_only(g->view, cur_node, g->ws.reach, x.n_max, x.e_max, g->host.max_depth, s);
    launch_classes(g->view, cur_node, g->ws.reach, out_class, s);
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_debug_node_classes(pl_graph_batch *g, const int32_t *cur_node, uint8_t *out_class, void *stream)
{
    return pl_node_classes(g, cur_node, out_class, stream);
}

size_t pl_weights_count(const pl_model_cfg *cfg)
{
    if (!cfg_ok(cfg)) return 0;
    return plan_weights(*cfg, nullptr);
}

int pl_weights_create(const pl_model_cfg *cfg, const float *host_blob, size_t n_floats,
                      pl_weights **out)
{
    if (!out) return fail(PL_ERR_NULL, "out is NULL");
    *out = nullptr;
    if (!cfg || !host_blob) return fail(PL_ERR_NULL, "cfg / host_blob are NULL");
    if (!cfg_ok(cfg)) return fail(PL_ERR_SHAPE, "model configuration out of the supported range");
    pl_weights *w = new (std::nothrow) pl_weights();
    if (!w) return fail(PL_ERR_NOMEM, "out of host memory");
    w->cfg = *cfg;
    const size_t need = plan_weights(*cfg, &w->view);
    if (n_floats != need) {
        delete w;
        return fail(PL_ERR_SHAPE, "weight blob has " + std::to_string(n_floats) + " floats, expected " +
                                      std::to_string(need));
    }
    w->host_blob.assign(host_blob, host_blob + n_floats);
    if (cfg->weight_dtype == PL_WEIGHTS_BF16) {
        const ModelView &m = w->view;
        round_layer(w->host_blob, m.proj);
        for (int l = 0; l < m.L; ++l) {
            for (int d = 0; d < 2; ++d) {
                round_layer(w->host_blob, m.f[d].layer[l]);
                round_layer(w->host_blob, m.g[d].layer[l]);
            }
            for (int i = 0; i < 3; ++i) {
                round_layer(w->host_blob, m.l[i].layer[l]);
                round_layer(w->host_blob, m.h[i].layer[l]);
            }
        }
        round_layer(w->host_blob, m.pol1);
        round_layer(w->host_blob, m.pol2);
    }
    int rc = upload(w->host_blob, &w->d_blob);
    if (rc) {
        delete w;
        return rc;
    }
    w->view.blob = w->d_blob;
    {
        std::vector<float> t(w->host_blob);
        auto flip = [&](const LayerRef &r) {
            for (int i = 0; i < r.n_in; ++i)
                for (int j = 0; j < r.n_out; ++j)
                    t[r.w + static_cast<size_t>(j) * r.n_in + i] = w->host_blob[r.w + static_cast<size_t>(i) * r.n_out + j];
        };
        const ModelView &m = w->view;
        flip(m.proj);
        for (int l = 0; l < m.L; ++l) {
            for (int d = 0; d < 2; ++d) {
                flip(m.f[d].layer[l]);
                flip(m.g[d].layer[l]);
            }
            for (int i = 0; i < 3; ++i) {
                flip(m.l[i].layer[l]);
                flip(m.h[i].layer[l]);
            }
        }
        flip(m.pol1);
        flip(m.pol2);
        if ((rc = upload(t, &w->d_blob_t))) {
            pl_weights_destroy(w);
            return rc;
        }
    }
    if (sweep_mfma_supported(cfg->H, cfg->n_layers, cfg->weight_dtype)) {
        std::vector<uint16_t> frag;
        std::vector<float> sweep_bias;
        w->sweep_ws = cfg->weight_dtype == PL_WEIGHTS_BF16 ? 1 : 3;
        pack_sweep_weights(w->view, w->host_blob.data(), w->sweep_ws, &frag, &sweep_bias);
        if ((rc = upload(frag, &w->d_wfrag)) || (rc = upload(sweep_bias, &w->d_sweep_bias))) {
            pl_weights_destroy(w);
            return rc;
        }
        std::vector<float> unused;
        pack_sweep_weights(w->view, w->host_blob.data(), w->sweep_ws, &frag, &unused, true);
        if ((rc = upload(frag, &w->d_wfrag_bw))) {
            pl_weights_destroy(w);
            return rc;
        }
    }
    if (pool_mfma_supported(cfg->H, cfg->n_layers, cfg->weight_dtype)) {
        std::vector<uint16_t> frag;
        std::vector<float> pool_bias;
        w->sweep_ws = cfg->weight_dtype == PL_WEIGHTS_BF16 ? 1 : 3;
        pack_pool_weights(w->view, w->host_blob.data(), w->sweep_ws, &frag, &pool_bias);
        if ((rc = upload(frag, &w->d_pool_frag)) || (rc = upload(pool_bias, &w->d_pool_bias))) {
            pl_weights_destroy(w);
            return rc;
        }
        if (pool_stream_supported(cfg->H, cfg->n_layers, cfg->weight_dtype)) {
            pack_pool_stream_weights(w->view, w->host_blob.data(), &frag);
            if ((rc = upload(frag, &w->d_pool_afrag))) {
                pl_weights_destroy(w);
                return rc;
            }
            if (pool_stream_bw_supported(cfg->H, cfg->n_layers, cfg->weight_dtype)) {
                pack_pool_stream_bw_weights(w->view, w->host_blob.data(), &frag);
                if ((rc = upload(frag, &w->d_pool_bwfrag))) {
                    pl_weights_destroy(w);
                    return rc;
                }
            }
        }
    }
    *out = w;
    return PL_OK;
}

int pl_weights_set_path(pl_weights *w, int32_t path)
{
    if (!w) return fail(PL_ERR_NULL, "weights handle is NULL");
    if (path != 0 && path != 1) return fail(PL_ERR_SHAPE, "path must be 0 or 1");
    w->path = path;
    return PL_OK;
}

int pl_weights_destroy(pl_weights *w)
{
    if (!w) return PL_OK;
    (void)hipFree(w->d_blob);
    (void)hipFree(w->d_blob_t);
    (void)hipFree(w->d_wfrag);
    (void)hipFree(w->d_wfrag_bw);
    (void)hipFree(w->d_sweep_bias);
    (void)hipFree(w->d_pool_frag);
    (void)hipFree(w->d_pool_afrag);
    (void)hipFree(w->d_pool_bwfrag);
    (void)hipFree(w->d_pool_bias);
    delete w;
    return PL_OK;
}

int pl_embed_forward(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                     const int32_t *cur_node, const pl_weights *w, float *out_logits, void *stream)
{
    return forward_impl(g, node_feats, placement, cur_node, w, out_logits, nullptr, nullptr,
                        nullptr, nullptr, stream, true);
}

int pl_embed_forward_ex(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                        const int32_t *cur_node, const pl_weights *w, float *out_logits,
                        float *out_probs, float *out_node_emb, float *out_pooled, uint8_t *out_class,
                        void *stream)
{
    return forward_impl(g, node_feats, placement, cur_node, w, out_logits, out_probs, out_node_emb,
                        out_pooled, out_class, stream, true);
}

int pl_graph_batch_upload(pl_graph_batch *g)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    void *unused = nullptr;
    int rc = scratch_address(&unused);
    if (rc) return rc;
    if (g->host.B == 0) return PL_OK;
    return ensure_on_device(g);
}

size_t pl_embed_forward_static_limit(void) { return kStaticScratchBytes; }

size_t pl_embed_forward_static_bytes(const pl_graph_batch *g, const pl_weights *w)
{
    if (!g || !w) return 0;
    Workspace sized;
    return carve_workspace(nullptr, static_cast<size_t>(g->host.n_tot), static_cast<size_t>(g->host.B), w->view,
                           true, &sized);
}

int pl_embed_forward_static(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                            const int32_t *cur_node, const pl_weights *w, float *out_logits,
                            float *out_probs, void *stream)
{
    if (!g || !w) return fail(PL_ERR_NULL, "graph batch or weights handle is NULL");
    if (g->host.B == 0) return PL_OK;
    if (!g->on_device)
        return fail(PL_ERR_STATE, "the batch is not on the device yet: call pl_graph_batch_upload first "
                                  "(this entry point allocates nothing)");
    int dev = -1;
    PL_HIP(hipGetDevice(&dev));
    if (dev != g->device) return fail(PL_ERR_STATE, "the batch lives on another device than the current one");
    const size_t n = static_cast<size_t>(g->host.n_tot), B = static_cast<size_t>(g->host.B);
    Workspace ws;
    const size_t need = carve_workspace(nullptr, n, B, w->view, true, &ws);
    if (need > kStaticScratchBytes)
        return fail(PL_ERR_SHAPE, "this batch and model need " + std::to_string(need) +
                                      " bytes of intermediate buffers, more than the fixed block of " +
                                      std::to_string(kStaticScratchBytes) + " bytes: use pl_embed_forward");
    void *ptr = nullptr;
    int rc = scratch_address(&ptr);
    if (rc) return rc;
    carve_workspace(static_cast<unsigned char *>(ptr), n, B, w->view, true, &ws);
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the block keeps the last call's contents: the rows and bytes that the kernels read as zero
    // without ever writing them are cleared by a fill kernel (a memset node must not be captured)
    launch_fill_zero(ws.msg + 2 * n * w->view.H, 2 * static_cast<size_t>(w->view.H), s);
    launch_fill_zero(reinterpret_cast<float *>(ws.reach + (2 * n) / 4 * 4), 5, s);
    return forward_impl(g, node_feats, placement, cur_node, w, out_logits, out_probs, nullptr, nullptr, nullptr,
                        stream, false, nullptr, 0, nullptr, nullptr, nullptr, nullptr, &ws);
}

int pl_episode_step(pl_graph_batch *g, int32_t D, const float *logits, const float *uniforms,
                    const int32_t *order, int32_t t, float *node_feats, int32_t *placement,
                    int32_t *cur_node, int32_t *out_action, float *out_logp, void *stream)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    if (D < 1 || D > kMaxD || t < 0) return fail(PL_ERR_SHAPE, "D must be in [1, 16] and t >= 0");
    if (g->host.B == 0) return PL_OK;
    if (!logits || !uniforms || !order || !node_feats || !placement || !cur_node)
        return fail(PL_ERR_NULL, "a required device array is NULL");
    int rc = ensure_on_device(g);
    if (rc) return rc;
    launch_episode_step(g->view, D, logits, uniforms, order, t, node_feats, placement, cur_node, out_action,
                        out_logp, static_cast<hipStream_t>(stream));
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_episode_run(pl_graph_batch *g, const pl_weights *w, float *node_feats, int32_t *placement,
                   int32_t *cur_node, const int32_t *order, const float *uniforms, int32_t t0,
                   int32_t n_steps, float *logits, int32_t keep_logits, int32_t *out_actions,
                   float *out_logp, void *stream)
{
    if (!g || !w) return fail(PL_ERR_NULL, "graph batch or weights handle is NULL");
    if (t0 < 0 || n_steps < 0) return fail(PL_ERR_SHAPE, "t0 and n_steps must not be negative");
    if (g->host.B == 0 || n_steps == 0) return PL_OK;
    if (!logits || !uniforms || !order || !node_feats || !placement || !cur_node)
        return fail(PL_ERR_NULL, "a required device array is NULL");
    if (validate_enabled()) {
        const int rc = validate_state(g, w->cfg.D, placement, cur_node, nullptr, true, static_cast<hipStream_t>(stream));
        if (rc) return rc;
    }
    const size_t B = static_cast<size_t>(g->host.B), D = static_cast<size_t>(w->cfg.D);
    for (int32_t i = 0; i < n_steps; ++i) {
        float *l = keep_logits ? logits + static_cast<size_t>(i) * B * D : logits;
        int rc = forward_impl(g, node_feats, placement, cur_node, w, l, nullptr, nullptr, nullptr, nullptr, stream,
                              false);
        if (rc) return rc;
        launch_episode_step(g->view, w->cfg.D, l, uniforms + static_cast<size_t>(i) * B, order, t0 + i,
                            node_feats, placement, cur_node, out_actions ? out_actions + static_cast<size_t>(i) * B : nullptr,
                            out_logp ? out_logp + static_cast<size_t>(i) * B : nullptr,
                            static_cast<hipStream_t>(stream));
    }
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_reinforce_coeff(int32_t T, int32_t B, const float *rewards, const int32_t *group, int32_t n_groups,
                       float *out_coeff, float *out_baseline, void *stream)
{
    if (T < 0 || B < 0 || n_groups < 0) return fail(PL_ERR_SHAPE, "T, B and n_groups must not be negative");
    if (static_cast<double>(T) * std::max(B, n_groups) >= 2.0e9)
        return fail(PL_ERR_SHAPE, "T x B is too large");
    if (T == 0 || B == 0) return PL_OK;
    if (!rewards || !out_coeff) return fail(PL_ERR_NULL, "rewards and out_coeff are required");
    if (n_groups > 0 && (!group || !out_baseline))
        return fail(PL_ERR_NULL, "group and out_baseline are required when n_groups > 0");
    launch_reinforce_coeff(T, B, n_groups, rewards, group, out_coeff, out_baseline,
                           static_cast<hipStream_t>(stream));
    PL_HIP(hipGetLastError());
    return PL_OK;
}

static int policy_gradient_impl(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                                const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                                const float *coeff, const float *entropy_coeff, int32_t accumulate, float *grad,
                                float *out_logits, float *out_logp, float *out_entropy, void *stream,
                                bool allow_finished);

int pl_episode_gradient(pl_graph_batch *g, const pl_weights *w, float *node_feats, int32_t *placement,
                        int32_t *cur_node, const int32_t *order, const int32_t *actions, const float *coeff,
                        const float *entropy_coeff, int32_t t0, int32_t n_steps, int32_t accumulate, float *grad,
                        float *logits, float *out_logp, void *stream)
{
    if (!g || !w) return fail(PL_ERR_NULL, "graph batch or weights handle is NULL");
    if (t0 < 0 || n_steps < 0) return fail(PL_ERR_SHAPE, "t0 and n_steps must not be negative");
    if (g->host.B == 0) return PL_OK;
    if (!node_feats || !placement || !cur_node || !order || !actions || !coeff || !grad || !logits)
        return fail(PL_ERR_NULL, "a required device array is NULL");
    const size_t B = static_cast<size_t>(g->host.B);
    if (n_steps == 0 && !accumulate) {
        launch_fill_zero(grad, plan_weights(w->cfg, nullptr), static_cast<hipStream_t>(stream));
        PL_HIP(hipGetLastError());
        return PL_OK;
    }
    for (int32_t i = 0; i < n_steps; ++i) {
        int rc = policy_gradient_impl(g, node_feats, placement, cur_node, w, actions + i * B, coeff + i * B,
                                      entropy_coeff ? entropy_coeff + i * B : nullptr,
                                      (accumulate || i > 0) ? 1 : 0, grad, logits,
                                      out_logp ? out_logp + i * B : nullptr, nullptr, stream, true);
        if (rc) return rc;
        launch_episode_apply(g->view, w->cfg.D, actions + i * B, order, t0 + i, node_feats, placement, cur_node,
                             static_cast<hipStream_t>(stream));
    }
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_policy_gradient(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                       const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                       const float *coeff, int32_t accumulate, float *grad, float *out_logits,
                       float *out_logp, void *stream)
{
    return pl_policy_gradient_ex(g, node_feats, placement, cur_node, w, actions, coeff, nullptr, accumulate, grad,
                                 out_logits, out_logp, nullptr, stream);
}

static int policy_gradient_impl(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                                const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                                const float *coeff, const float *entropy_coeff, int32_t accumulate, float *grad,
                                float *out_logits, float *out_logp, float *out_entropy, void *stream,
                                bool allow_finished)
{
    if (!g || !w) return fail(PL_ERR_NULL, "graph batch or weights handle is NULL");
    if (g->host.B == 0) return PL_OK;
    if (!node_feats || !placement || !cur_node || !actions || !coeff || !grad || !out_logits)
        return fail(PL_ERR_NULL, "a required device array is NULL");
    int rc;
    if (validate_enabled() && (rc = validate_state(g, w->cfg.D, placement, cur_node, actions, allow_finished,
                                                   static_cast<hipStream_t>(stream))))
        return rc;
    if ((rc = ensure_on_device(g))) return rc;
    const ModelView &mv = w->view;
    if ((rc = ensure_grad_workspace(g, mv))) return rc;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // the chain kernel addresses the delta arrays with 32-bit element offsets
    const bool fits = (2.0 * mv.L * static_cast<double>(g->host.n_tot) + 1) * mv.H < 2.0e9 &&
                      (static_cast<double>(g->host.n_tot) + 2) * 2 * mv.H * sizeof(float) < 4.0e9;
    const bool chain_cores = w->d_wfrag_bw && w->path == 0 && w->cfg.k_sweeps >= 1 && fits;
    // on that path a single forward sweep keeps a_v and the layer outputs, so nothing is computed twice
    float *keep = (chain_cores && w->cfg.k_sweeps == 1) ? g->gw.keep : nullptr;
    // several sweeps: the states and messages after every sweep but the last are copied aside
    if (w->cfg.k_sweeps > 1 && g->gw.snap_sweeps < w->cfg.k_sweeps - 1) {
        (void)hipFree(g->gw.snap_emb);
        (void)hipFree(g->gw.snap_msg);
        g->gw.snap_emb = g->gw.snap_msg = nullptr;
        g->gw.snap_sweeps = 0;
        const size_t span = static_cast<size_t>(g->host.n_tot) * 2 * mv.H * (w->cfg.k_sweeps - 1);
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->gw.snap_emb), sizeof(float) * (span + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->gw.snap_msg), sizeof(float) * (span + 4)));
        g->gw.snap_sweeps = w->cfg.k_sweeps - 1;
    }
    // likewise the matrix-core pooling kernel keeps the outputs of l's layers
    bool pool_kept = false;
    rc = forward_impl(g, node_feats, placement, cur_node, w, out_logits, nullptr, nullptr, g->gw.pooled, nullptr,
                      stream, false, keep, g->gw.dfg_stride, w->path == 0 ? g->gw.lact : nullptr, &pool_kept,
                      w->cfg.k_sweeps > 1 ? g->gw.snap_emb : nullptr, g->gw.snap_msg, nullptr, g->gw.mask4);
    if (rc) return rc;
    if (!accumulate) launch_fill_zero(grad, plan_weights(w->cfg, nullptr), s);
    ForwardArgs fa{node_feats, placement, cur_node, out_logits, nullptr, g->gw.pooled};
    const StageMarks marks{&g->timer, stage_mark};
    const BackwardArgs ba{actions, coeff, entropy_coeff, grad, out_logp, out_entropy, g->gw.snap_emb, g->gw.snap_msg,
                          w->path == 0 ? reinterpret_cast<const uint4 *>(w->d_pool_bwfrag) : nullptr};
    launch_backward(g->view, mv, w->d_blob_t, g->ws, g->gw, fa, ba, w->cfg.k_sweeps, g->ws.n_chunks, w->path,
                    chain_cores ? reinterpret_cast<const uint4 *>(w->d_wfrag_bw) : nullptr, w->d_sweep_bias,
                    w->sweep_ws, keep, pool_kept, &marks, s);
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_policy_gradient_ex(pl_graph_batch *g, const float *node_feats, const int32_t *placement,
                          const int32_t *cur_node, const pl_weights *w, const int32_t *actions,
                          const float *coeff, const float *entropy_coeff, int32_t accumulate, float *grad,
                          float *out_logits, float *out_logp, float *out_entropy, void *stream)
{
    return policy_gradient_impl(g, node_feats, placement, cur_node, w, actions, coeff, entropy_coeff, accumulate,
                                grad, out_logits, out_logp, out_entropy, stream, false);
}

int pl_simulate_runtime(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                        float inv_bandwidth, float *out_runtime, int32_t *out_events, void *stream)
{
    return pl_simulate_runtime_ex(g, D, node_feats, placement, inv_bandwidth, 0, out_runtime, out_events, stream);
}

int pl_simulate_runtime_ex(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                           float inv_bandwidth, int32_t per_child_transfers, float *out_runtime,
                           int32_t *out_events, void *stream)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    if (D < 1 || D > kMaxD) return fail(PL_ERR_SHAPE, "D must be in [1, 16]");
    if (!(inv_bandwidth >= 0.0f)) return fail(PL_ERR_SHAPE, "inv_bandwidth must not be negative");
    if (g->host.B == 0) return PL_OK;
    if (!node_feats || !placement || !out_runtime) return fail(PL_ERR_NULL, "a required device array is NULL");
    int64_t n_max = 0, e_max = 0;
    for (int32_t b = 0; b < g->host.B; ++b) {
        n_max = std::max<int64_t>(n_max, g->host.node_off[b + 1] - g->host.node_off[b]);
        e_max = std::max<int64_t>(e_max, g->host.edge_off[b + 1] - g->host.edge_off[b]);
    }
    // graph-local ids and queue links are 16-bit in LDS; the whole graph must fit the 160 KB of a CU
    if (n_max >= 0xFFFF || e_max >= 0xFFFF ||
        simulator_lds_bytes(static_cast<int>(n_max), static_cast<int>(e_max)) > 160 * 1024)
        return fail(PL_ERR_SHAPE, "a graph is too large for the simulator (its state must fit in 160 KB of LDS)");
    int rc = ensure_on_device(g);
    if (rc) return rc;
    rc = launch_simulate(g->view, D, static_cast<int>(n_max), static_cast<int>(e_max), node_feats, placement,
                         inv_bandwidth, per_child_transfers != 0, out_runtime, out_events,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_simulate_reward(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                       float inv_bandwidth, float mem_limit, float mem_penalty, float *out_reward,
                       float *out_runtime, float *out_peak_mem, int32_t *out_events, void *stream)
{
    return pl_simulate_reward_ex(g, D, node_feats, placement, inv_bandwidth, 0, mem_limit, mem_penalty, out_reward,
                                 out_runtime, out_peak_mem, out_events, stream);
}

int pl_simulate_reward_ex(pl_graph_batch *g, int32_t D, const float *node_feats, const int32_t *placement,
                          float inv_bandwidth, int32_t per_child_transfers, float mem_limit, float mem_penalty,
                          float *out_reward, float *out_runtime, float *out_peak_mem, int32_t *out_events,
                          void *stream)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    if (D < 1 || D > kMaxD) return fail(PL_ERR_SHAPE, "D must be in [1, 16]");
    if (!(inv_bandwidth >= 0.0f)) return fail(PL_ERR_SHAPE, "inv_bandwidth must not be negative");
    if (!(mem_penalty >= 0.0f) || mem_limit != mem_limit)
        return fail(PL_ERR_SHAPE, "mem_penalty must not be negative and mem_limit must be a number");
    if (g->host.B == 0) return PL_OK;
    if (!node_feats || !placement || !out_reward) return fail(PL_ERR_NULL, "a required device array is NULL");
    int64_t n_max = 0, e_max = 0;
    for (int32_t b = 0; b < g->host.B; ++b) {
        n_max = std::max<int64_t>(n_max, g->host.node_off[b + 1] - g->host.node_off[b]);
        e_max = std::max<int64_t>(e_max, g->host.edge_off[b + 1] - g->host.edge_off[b]);
    }
    if (n_max >= 0xFFFF || e_max >= 0xFFFF ||
        simulator_lds_bytes(static_cast<int>(n_max), static_cast<int>(e_max)) > 160 * 1024)
        return fail(PL_ERR_SHAPE, "a graph is too large for the simulator (its state must fit in 160 KB of LDS)");
    int rc = ensure_on_device(g);
    if (rc) return rc;
    const size_t n = static_cast<size_t>(g->host.n_tot);
    if (!g->sim_start || g->sim_D < D) {
        for (float **p : {&g->sim_start, &g->sim_end, &g->sim_arrival, &g->sim_arrival_last, &g->sim_alloc,
                          &g->sim_free, &g->sim_rt}) {
            (void)hipFree(*p);
            *p = nullptr;
        }
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_start), sizeof(float) * (n + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_end), sizeof(float) * (n + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_arrival), sizeof(float) * (n * D + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_arrival_last), sizeof(float) * (n * D + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_alloc), sizeof(float) * (n * D + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_free), sizeof(float) * (n * D + 4)));
        PL_HIP(hipMalloc(reinterpret_cast<void **>(&g->sim_rt), sizeof(float) * (g->host.B + 4)));
        g->sim_D = D;
    }
    rc = launch_simulate_reward(g->view, D, static_cast<int>(n_max), static_cast<int>(e_max), node_feats, placement,
                                inv_bandwidth, per_child_transfers != 0, mem_limit, mem_penalty, g->sim_start,
                                g->sim_end, g->sim_arrival, g->sim_arrival_last, g->sim_alloc, g->sim_free,
                                out_runtime ? out_runtime : g->sim_rt, out_peak_mem,
                                out_reward, out_events, static_cast<hipStream_t>(stream));
    if (rc) return rc;
    PL_HIP(hipGetLastError());
    return PL_OK;
}

int pl_profile_enable(pl_graph_batch *g, int32_t on)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    g->timer.on = on != 0;
    // events for a few hundred timed calls are created now, not between the launches they time
    constexpr size_t kPooled = 2048;
    try {
        while (on && g->timer.pool.size() < kPooled) {
            hipEvent_t e;
            PL_HIP(hipEventCreate(&e));
            g->timer.pool.push_back(e);
        }
    } catch (const std::bad_alloc &) {
        return fail(PL_ERR_NOMEM, "out of host memory");
    }
    return PL_OK;
}

int pl_profile_read(pl_graph_batch *g, double *ms_sum, int64_t *launches, int32_t reset)
{
    if (!g) return fail(PL_ERR_NULL, "graph batch is NULL");
    StageTimer &t = g->timer;
    try {
    for (int st = 0; st < PL_STAGE_COUNT; ++st) {
        auto &ev = t.ev[st];
        for (size_t i = 0; i + 1 < ev.size(); i += 2) {
            float ms = 0.0f;
            PL_HIP(hipEventSynchronize(ev[i + 1]));
            PL_HIP(hipEventElapsedTime(&ms, ev[i], ev[i + 1]));
            t.ms_sum[st] += ms;
            t.launches[st] += 1;
        }
        for (hipEvent_t e : ev) t.pool.push_back(e);     // kept for the next timed calls
        ev.clear();
        if (ms_sum) ms_sum[st] = t.ms_sum[st];
        if (launches) launches[st] = t.launches[st];
        if (reset) {
            t.ms_sum[st] = 0.0;
            t.launches[st] = 0;
        }
    }
    } catch (const std::bad_alloc &) {
        return fail(PL_ERR_NOMEM, "out of host memory");
    }
    return PL_OK;
}

const char *pl_last_error(void) { return g_error.c_str(); }

const char *pl_version(void) { return "placeto-mi355x 0.1 (gfx950)"; }

}  // extern "C"
