// C ABI of the RainFusion library: argument checks, the cache of device-resident block
// lists, and the two entry points.  All checks run before the first HIP call, so they can
// be exercised on a machine without a GPU.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstring>
#include <memory>
#include <mutex>
#include <vector>

#include "rf_internal.h"

namespace rf {
namespace {

struct CachedPlan {
    Geometry g;
    int block;  // 0 for the ARM sample tables
    int device;
    void* blob = nullptr;
    DevicePlan dev{};
    // ARM tables (block == 0)
    const int32_t* local_pos = nullptr;   // [HW]   in-frame position of first-frame sample a
    const int32_t* global_pos = nullptr;  // [nG]   in-frame position of equal-interval sample a
    const int32_t* global_frame = nullptr;  // [nG] frame of equal-interval sample a
    const int32_t* local_pos_range = nullptr;  // per 64-sample tile of each table: {min, max}
    const int32_t* global_pos_range = nullptr;
    const int32_t* global_frame_range = nullptr;
    int nG = 0;
};

std::mutex g_mu;
std::vector<std::unique_ptr<CachedPlan>> g_plans;

bool same_geometry(const Geometry& a, const Geometry& b) { return std::memcmp(&a, &b, sizeof(Geometry)) == 0; }

CachedPlan* find_plan(const Geometry& g, int block, int device) {
    for (auto& p : g_plans)
        if (p->block == block && p->device == device && same_geometry(p->g, g)) return p.get();
    return nullptr;
}

// Uploads `words` and returns the device address; segments are 256-byte aligned inside one blob.
struct BlobBuilder {
    std::vector<int32_t> words;
    size_t add(const std::vector<int32_t>& v) {
        while (words.size() % 64) words.push_back(0);
        const size_t off = words.size();
        words.insert(words.end(), v.begin(), v.end());
        if (v.empty()) words.push_back(0);
        return off;
    }
    int upload(void** blob) {
        if (hipMalloc(blob, words.size() * sizeof(int32_t)) != hipSuccess) return RF_ERR_HIP;
        if (hipMemcpy(*blob, words.data(), words.size() * sizeof(int32_t), hipMemcpyHostToDevice) != hipSuccess) {
            (void)hipFree(*blob);
            *blob = nullptr;
            return RF_ERR_HIP;
        }
        return RF_OK;
    }
};

int get_attention_plan(const Geometry& g, int block, const DevicePlan** out) {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return RF_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    CachedPlan* cp = find_plan(g, block, device);
    if (!cp) {
        HostPlan hp;
        build_plan(g, block, &hp);
        BlobBuilder bb;
        size_t off_rp[kLists], off_co[kLists], off_at[kLists], off_qo[kLists], off_fe[kLists];
        for (int c = 0; c < kLists; ++c) {
            off_rp[c] = bb.add(hp.row_ptr[c]);
            off_co[c] = bb.add(hp.cols[c]);
            off_at[c] = bb.add(hp.attr[c]);
            off_qo[c] = bb.add(hp.qorder[c]);
            off_fe[c] = bb.add(hp.first_entry[c]);
        }
        const size_t off_ci = bb.add(hp.cidx), off_pm = bb.add(hp.pm_token);
        auto p = std::make_unique<CachedPlan>();
        p->g = g;
        p->block = block;
        p->device = device;
        const int st = bb.upload(&p->blob);
        if (st != RF_OK) return st;
        const int32_t* base = static_cast<const int32_t*>(p->blob);
        DevicePlan& d = p->dev;
        for (int c = 0; c < kLists; ++c) {
            d.row_ptr[c] = base + off_rp[c];
            d.cols[c] = base + off_co[c];
            d.attr[c] = base + off_at[c];
            d.qorder[c] = base + off_qo[c];
            d.first_entry[c] = base + off_fe[c];
        }
        d.cidx = base + off_ci;
        d.pm_token = base + off_pm;
        d.radius[RF_SPATIAL] = g.r_spatial;
        d.radius[RF_TEMPORAL] = g.r_temporal;
        d.radius[RF_TEXTURAL] = 0;
        d.radius[kListTemporalPM] = g.r_temporal;
        d.video_shift = g.video_shift();
        d.text_shift = g.text_shift();
        d.N = g.N; d.Nv = g.Nv; d.Nc = hp.Nc;
        d.block = block; d.nQB = hp.nQB; d.nKT = hp.nKT; d.nCT = hp.nCT;
        d.first_text_qb = hp.first_text_qb;
        cp = p.get();
        g_plans.push_back(std::move(p));
    }
    *out = &cp->dev;
    return RF_OK;
}

int global_sample_count(const Geometry& g) { return (g.Nv + g.omega - 1) / g.omega; }

int get_arm_tables(const Geometry& g, const CachedPlan** out) {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return RF_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    CachedPlan* cp = find_plan(g, 0, device);
    if (!cp) {
        const int nG = global_sample_count(g);
        std::vector<int32_t> lp(g.HW), gp(nG), gf(nG);
        for (int a = 0; a < g.HW; ++a) lp[a] = a;
        for (int a = 0; a < nG; ++a) {
            const int64_t tok = static_cast<int64_t>(a) * g.omega;
            gp[a] = static_cast<int32_t>(tok % g.HW);
            gf[a] = static_cast<int32_t>(tok / g.HW);
        }
        auto tile_ranges = [](const std::vector<int32_t>& v) {
            std::vector<int32_t> r;
            for (size_t t0 = 0; t0 < v.size(); t0 += kTileK) {
                const size_t t1 = std::min(v.size(), t0 + kTileK);
                r.push_back(*std::min_element(v.begin() + t0, v.begin() + t1));
                r.push_back(*std::max_element(v.begin() + t0, v.begin() + t1));
            }
            return r;
        };
        BlobBuilder bb;
        const size_t o0 = bb.add(lp), o1 = bb.add(gp), o2 = bb.add(gf);
        const size_t r0 = bb.add(tile_ranges(lp)), r1 = bb.add(tile_ranges(gp)), r2 = bb.add(tile_ranges(gf));
        auto p = std::make_unique<CachedPlan>();
        p->g = g;
        p->block = 0;
        p->device = device;
        const int st = bb.upload(&p->blob);
        if (st != RF_OK) return st;
        const int32_t* base = static_cast<const int32_t*>(p->blob);
        p->local_pos = base + o0;
        p->global_pos = base + o1;
        p->global_frame = base + o2;
        p->local_pos_range = base + r0;
        p->global_pos_range = base + r1;
        p->global_frame_range = base + r2;
        p->nG = nG;
        cp = p.get();
        g_plans.push_back(std::move(p));
    }
    *out = cp;
    return RF_OK;
}

// Work-queue counters of the attention kernel: 8 ints per call, taken round-robin from a small
// per-device ring so that calls in flight on different streams do not share a set.
constexpr int kQueueSets = 64, kQueueStride = 64;  // ints; a set per 256 bytes
struct QueueRing {
    int device;
    int* base;
    unsigned next;
};
std::vector<QueueRing> g_queues;

int next_queue(int** out) {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return RF_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_mu);
    for (auto& r : g_queues)
        if (r.device == device) {
            *out = r.base + (r.next++ % kQueueSets) * kQueueStride;
            return RF_OK;
        }
    void* p = nullptr;
    if (hipMalloc(&p, kQueueSets * kQueueStride * sizeof(int)) != hipSuccess) return RF_ERR_HIP;
    g_queues.push_back(QueueRing{device, static_cast<int*>(p), 1});
    *out = static_cast<int*>(p);
    return RF_OK;
}

bool valid_block(int block) { return block == 64 || block == 128 || block == 256; }  // query rows per block

int check_shape(int B, int nH, int D, const Geometry& g) {
    if (B < 1 || nH < 1) return RF_ERR_SHAPE;
    if (D != 64 && D != 96 && D != 128) return RF_ERR_SHAPE;
    if (static_cast<int64_t>(B) * nH > (1 << 20)) return RF_ERR_SHAPE;
    (void)g;
    return RF_OK;
}

size_t arm_rows(const Geometry& g) { return static_cast<size_t>(std::max(g.HW, global_sample_count(g))); }

}  // namespace
}  // namespace rf

using namespace rf;

extern "C" {

int rf_version(void) { return 100; }

const char* rf_status_string(int status) {
    switch (status) {
        case RF_OK: return "ok";
        case RF_ERR_NULL: return "null pointer";
        case RF_ERR_SHAPE: return "bad tensor shape";
        case RF_ERR_LAYOUT: return "bad video layout";
        case RF_ERR_PARAM: return "bad parameter";
        case RF_ERR_BLOCK: return "block must be 64, 128 or 256";
        case RF_ERR_WORKSPACE: return "workspace missing or too small";
        case RF_ERR_HIP: return "HIP runtime error";
        default: return "unknown status";
    }
}

size_t rf_arm_workspace_bytes(int B, int nH, const rf_layout* layout, const rf_params* params) {
    Geometry g;
    if (resolve_geometry(layout, params, &g) != RF_OK || B < 1 || nH < 1) return 0;
    return static_cast<size_t>(B) * nH * 2 * arm_rows(g) * sizeof(float);
}

// Geometry of `params` with both band widths replaced by bw.
static int geometry_with_bandwidth(const rf_layout* layout, const rf_params* params, float bw, Geometry* g) {
    rf_params p = params ? *params : rf_params{0.25f, 0.25f, 2, 0, 0};
    p.bw_spatial = bw;
    p.bw_temporal = bw;
    return resolve_geometry(layout, &p, g);
}

static int check_bandwidths(const float* bandwidths, int n_bw) {
    if (!bandwidths) return RF_ERR_NULL;
    if (n_bw < 1 || n_bw > RF_MAX_BANDWIDTHS) return RF_ERR_PARAM;
    for (int k = 0; k < n_bw; ++k)
        if (!(bandwidths[k] >= 0.f && bandwidths[k] <= 1.f)) return RF_ERR_PARAM;
    return RF_OK;
}

// Shared by rf_arm_classify (bandwidths == null: the widths of params) and rf_arm_classify_plus.
static int arm_classify_impl(const void* Q, const void* K, int B, int nH, int D, const rf_layout* layout,
                             const rf_params* params, int sample_mode, float threshold, const float* bandwidths,
                             int n_bw, int32_t* head_class, int32_t* head_bw, float* recalls, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!Q || !K || !head_class || !layout) return RF_ERR_NULL;
    Geometry g;
    int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    st = check_shape(B, nH, D, g);
    if (st != RF_OK) return st;
    if (sample_mode != RF_SAMPLE_FIRST_FRAME && sample_mode != RF_SAMPLE_EQUAL_INTERVAL) return RF_ERR_PARAM;
    if (!(threshold >= 0.f && threshold <= 1.f)) return RF_ERR_PARAM;
    if (bandwidths) {
        st = check_bandwidths(bandwidths, n_bw);
        if (st != RF_OK) return st;
    }
    if (!workspace || workspace_bytes < n_bw * rf_arm_workspace_bytes(B, nH, layout, params)) return RF_ERR_WORKSPACE;

    int r_temporal[kMaxBw] = {g.r_temporal}, r_spatial[kMaxBw] = {g.r_spatial};
    ArmArgs a{};
    a.n_bw = n_bw;
    for (int k = 0; k < n_bw; ++k) a.by_width[k] = k;
    if (bandwidths) {
        for (int k = 0; k < n_bw; ++k) {
            Geometry gk;
            st = geometry_with_bandwidth(layout, params, bandwidths[k], &gk);
            if (st != RF_OK) return st;
            r_temporal[k] = gk.r_temporal;
            r_spatial[k] = gk.r_spatial;
        }
        std::stable_sort(a.by_width, a.by_width + n_bw, [&](int x, int y) { return bandwidths[x] < bandwidths[y]; });
    }

    const CachedPlan* tb = nullptr;
    st = get_arm_tables(g, &tb);
    if (st != RF_OK) return st;

    a.Q = static_cast<const uint16_t*>(Q);
    a.K = static_cast<const uint16_t*>(K);
    a.BH = B * nH;
    a.N = g.N;
    a.first_video_row = g.video_shift();
    a.scale_log2 = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(D)));
    if (sample_mode == RF_SAMPLE_FIRST_FRAME) a.pass[0] = ArmPass{tb->local_pos, tb->local_pos_range, g.HW, 1, {0}};
    else a.pass[0] = ArmPass{tb->global_pos, tb->global_pos_range, tb->nG, g.omega, {0}};
    a.pass[1] = ArmPass{tb->global_frame, tb->global_frame_range, tb->nG, g.omega, {0}};
    for (int k = 0; k < n_bw; ++k) {
        a.pass[0].radius[k] = r_temporal[k];
        a.pass[1].radius[k] = r_spatial[k];
    }
    a.row_recall = static_cast<float*>(workspace);
    a.max_n = static_cast<int>(arm_rows(g));
    a.threshold = threshold;
    a.fallback_class = g.two_head ? RF_DENSE : RF_TEXTURAL;
    a.head_class = head_class;
    a.head_bw = head_bw;
    a.recalls = recalls;
    return launch_arm(a, D, stream) == 0 ? RF_OK : RF_ERR_HIP;
}

int rf_arm_classify(const void* Q, const void* K, int B, int nH, int D, const rf_layout* layout,
                    const rf_params* params, int sample_mode, float threshold, int32_t* head_class,
                    float* recalls, void* workspace, size_t workspace_bytes, void* stream) {
    return arm_classify_impl(Q, K, B, nH, D, layout, params, sample_mode, threshold, nullptr, 1, head_class, nullptr,
                             recalls, workspace, workspace_bytes, stream);
}

int rf_arm_classify_plus(const void* Q, const void* K, int B, int nH, int D, const rf_layout* layout,
                         const rf_params* params, int sample_mode, float threshold, const float* bandwidths,
                         int n_bw, int32_t* head_class, int32_t* head_bw, float* recalls, void* workspace,
                         size_t workspace_bytes, void* stream) {
    if (!head_bw) return RF_ERR_NULL;
    const int st = check_bandwidths(bandwidths, n_bw);
    if (st != RF_OK) return st;
    return arm_classify_impl(Q, K, B, nH, D, layout, params, sample_mode, threshold, bandwidths, n_bw, head_class,
                             head_bw, recalls, workspace, workspace_bytes, stream);
}

size_t rf_attention_workspace_bytes(int B, int nH, int D, const rf_layout* layout, const rf_params* params) {
    Geometry g;
    if (resolve_geometry(layout, params, &g) != RF_OK || check_shape(B, nH, D, g) != RF_OK) return 0;
    return 2 * static_cast<size_t>(B) * nH * g.N * D * sizeof(uint16_t);
}

static int sparse_attention_impl(const void* Q, const void* K, const void* V, const int32_t* head_class,
                                 const int32_t* head_bw, const float* bandwidths, int n_bw, int B, int nH, int D,
                                 const rf_layout* layout, const rf_params* params, int block, void* O, void* workspace,
                                 size_t workspace_bytes, void* stream) {
    if (!Q || !K || !V || !O || !layout) return RF_ERR_NULL;
    const bool force_dense = params && (params->flags & RF_FLAG_FORCE_DENSE);
    if (!head_class && !force_dense) return RF_ERR_NULL;
    Geometry g;
    int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    st = check_shape(B, nH, D, g);
    if (st != RF_OK) return st;
    if (!valid_block(block)) return RF_ERR_BLOCK;
    if (workspace && workspace_bytes < rf_attention_workspace_bytes(B, nH, D, layout, params)) return RF_ERR_WORKSPACE;
    if (workspace && (reinterpret_cast<uintptr_t>(workspace) & 15)) return RF_ERR_WORKSPACE;

    AttnArgs a{};
    a.n_plans = bandwidths ? n_bw : 1;
    for (int k = 0; k < a.n_plans; ++k) {
        Geometry gk = g;
        if (bandwidths) {
            st = geometry_with_bandwidth(layout, params, bandwidths[k], &gk);
            if (st != RF_OK) return st;
        }
        const DevicePlan* dp = nullptr;
        st = get_attention_plan(gk, block, &dp);
        if (st != RF_OK) return st;
        a.plan[k] = *dp;
    }
    a.Q = static_cast<const uint16_t*>(Q);
    a.K = static_cast<const uint16_t*>(K);
    a.V = static_cast<const uint16_t*>(V);
    a.O = static_cast<uint16_t*>(O);
    st = next_queue(&a.queue);
    if (st != RF_OK) return st;
    a.head_class = force_dense ? nullptr : head_class;
    a.head_bw = bandwidths ? head_bw : nullptr;
    a.BH = B * nH;
    a.scale_log2 = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(D)));
    if (workspace && !force_dense) {
        a.packed_k = static_cast<uint16_t*>(workspace);
        a.packed_v = a.packed_k + static_cast<size_t>(B) * nH * g.N * D;
        if (launch_pack_textural(a, D, stream) != 0) return RF_ERR_HIP;
    }
    return launch_attention(a, D, stream) == 0 ? RF_OK : RF_ERR_HIP;
}

int rf_sparse_attention(const void* Q, const void* K, const void* V, const int32_t* head_class, int B, int nH,
                        int D, const rf_layout* layout, const rf_params* params, int block, void* O,
                        void* workspace, size_t workspace_bytes, void* stream) {
    return sparse_attention_impl(Q, K, V, head_class, nullptr, nullptr, 1, B, nH, D, layout, params, block, O,
                                 workspace, workspace_bytes, stream);
}

int rf_sparse_attention_plus(const void* Q, const void* K, const void* V, const int32_t* head_class,
                             const int32_t* head_bw, const float* bandwidths, int n_bw, int B, int nH, int D,
                             const rf_layout* layout, const rf_params* params, int block, void* O, void* workspace,
                             size_t workspace_bytes, void* stream) {
    if (!head_bw) return RF_ERR_NULL;
    const int st = check_bandwidths(bandwidths, n_bw);
    if (st != RF_OK) return st;
    return sparse_attention_impl(Q, K, V, head_class, head_bw, bandwidths, n_bw, B, nH, D, layout, params, block, O,
                                 workspace, workspace_bytes, stream);
}

int rf_plan_host(const rf_layout* layout, const rf_params* params, int block, int cls, int32_t* row_ptr,
                 int32_t* cols, size_t cap, size_t* needed) {
    if (!layout || !needed) return RF_ERR_NULL;
    Geometry g;
    const int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    if (!valid_block(block)) return RF_ERR_BLOCK;
    if (cls < RF_SPATIAL || cls > RF_LIST_TEMPORAL_POSITION_MAJOR) return RF_ERR_PARAM;
    HostPlan hp;
    build_plan(g, block, &hp);
    std::vector<int32_t> rp, co;
    flatten_class(hp, cls, &rp, &co);
    *needed = co.size();
    if (row_ptr) std::memcpy(row_ptr, rp.data(), rp.size() * sizeof(int32_t));
    if (cols) {
        if (cap < co.size()) return RF_ERR_WORKSPACE;
        std::memcpy(cols, co.data(), co.size() * sizeof(int32_t));
    }
    return RF_OK;
}

int rf_plan_order(const rf_layout* layout, const rf_params* params, int block, int cls, int32_t* order,
                  int32_t* first_entry) {
    if (!layout || !order) return RF_ERR_NULL;
    Geometry g;
    const int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    if (!valid_block(block)) return RF_ERR_BLOCK;
    if (cls < RF_SPATIAL || cls > RF_LIST_TEMPORAL_POSITION_MAJOR) return RF_ERR_PARAM;
    HostPlan hp;
    build_plan(g, block, &hp);
    const int list = cls == RF_LIST_TEMPORAL_POSITION_MAJOR ? kListTemporalPM : cls;
    // dense heads: the same scheme with plain token order for the blocks without text rows
    for (int i = 0; i < hp.nQB; ++i) order[i] = hp.qorder[cls == RF_DENSE ? RF_SPATIAL : list][i];
    if (first_entry)
        for (int i = 0; i < hp.nQB; ++i) first_entry[i] = cls == RF_DENSE ? 0 : hp.first_entry[list][i];
    return RF_OK;
}

int rf_plan_position_major(const rf_layout* layout, const rf_params* params, int32_t* token_of) {
    if (!layout || !token_of) return RF_ERR_NULL;
    Geometry g;
    const int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    for (int n = 0; n < g.Nv; ++n) token_of[n] = g.row_of((n % g.T) * g.HW + n / g.T);
    for (int n = g.Nv; n < g.N; ++n) token_of[n] = g.row_of(n);
    return RF_OK;
}

int rf_plan_clear(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (g_plans.empty() && g_queues.empty()) return RF_OK;
    int st = RF_OK;
    if (hipDeviceSynchronize() != hipSuccess) st = RF_ERR_HIP;
    for (auto& p : g_plans)
        if (p->blob && hipFree(p->blob) != hipSuccess) st = RF_ERR_HIP;
    g_plans.clear();
    for (auto& r : g_queues)
        if (hipFree(r.base) != hipSuccess) st = RF_ERR_HIP;
    g_queues.clear();
    return st;
}

}  // extern "C"
