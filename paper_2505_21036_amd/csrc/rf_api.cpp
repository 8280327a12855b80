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
    Geometry g;  // with the fields the lists do not depend on zeroed (see list_key)
    int block;
    int device;
    unsigned long long last_use = 0;
    void* blob = nullptr;
    DevicePlan dev{};
};

std::mutex g_mu;
std::vector<std::unique_ptr<CachedPlan>> g_plans;
unsigned long long g_use_counter = 0;
constexpr size_t kMaxCachedPlans = 16;  // per process; the least recently used one makes room

// The block lists depend on the layout, the band widths, the checkerboard stride and the placement
// of the text tokens, not on the ARM's sampling interval or its fallback class.
Geometry list_key(Geometry g) {
    g.omega = 0;
    g.two_head = 0;
    return g;
}

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

// out receives a COPY of the plan: the cache entry may be evicted by a later call (its device memory
// is only freed after the device has drained, so kernels already launched keep reading valid lists).
int get_attention_plan(const Geometry& geometry, int block, DevicePlan* out) {
    int device = 0;
    if (hipGetDevice(&device) != hipSuccess) return RF_ERR_HIP;
    const Geometry g = list_key(geometry);
    std::lock_guard<std::mutex> lock(g_mu);
    CachedPlan* cp = find_plan(g, block, device);
    if (!cp) {
        if (g_plans.size() >= kMaxCachedPlans) {
            size_t oldest = 0;
            for (size_t i = 1; i < g_plans.size(); ++i)
                if (g_plans[i]->last_use < g_plans[oldest]->last_use) oldest = i;
            if (hipDeviceSynchronize() != hipSuccess) return RF_ERR_HIP;
            if (g_plans[oldest]->blob && hipFree(g_plans[oldest]->blob) != hipSuccess) return RF_ERR_HIP;
            g_plans.erase(g_plans.begin() + static_cast<std::ptrdiff_t>(oldest));
        }
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
    cp->last_use = ++g_use_counter;
    *out = cp->dev;
    return RF_OK;
}

int global_sample_count(const Geometry& g) { return (g.Nv + g.omega - 1) / g.omega; }

bool valid_block(int block) { return block == 64 || block == 128 || block == 256 || block == 384; }  // query rows per block

// (token counts that overflow int32 indices were already refused by resolve_geometry)
int check_shape(int B, int nH, int D) {
    if (B < 1 || nH < 1) return RF_ERR_SHAPE;
    if (D != 64 && D != 96 && D != 128) return RF_ERR_SHAPE;
    if (static_cast<int64_t>(B) * nH > (1 << 20)) return RF_ERR_SHAPE;
    return RF_OK;
}

// The kernels read and write the tensors 16 bytes at a time.
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

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
        case RF_ERR_BLOCK: return "block must be 64, 128, 256 or 384";
        case RF_ERR_WORKSPACE: return "workspace missing or too small";
        case RF_ERR_HIP: return "HIP runtime error";
        case RF_ERR_ALIGN: return "tensor or workspace pointer misaligned";
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
    st = check_shape(B, nH, D);
    if (st != RF_OK) return st;
    if (!aligned16(Q) || !aligned16(K)) return RF_ERR_ALIGN;
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

    a.Q = static_cast<const uint16_t*>(Q);
    a.K = static_cast<const uint16_t*>(K);
    a.BH = B * nH;
    a.N = g.N;
    a.first_video_row = g.video_shift();
    a.scale_log2 = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(D)));
    const int nG = global_sample_count(g);
    if (sample_mode == RF_SAMPLE_FIRST_FRAME) a.pass[0] = ArmPass{0, g.HW, 1, g.HW, {0}};
    else a.pass[0] = ArmPass{0, nG, g.omega, g.HW, {0}};
    a.pass[1] = ArmPass{1, nG, g.omega, g.HW, {0}};
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

int rf_arm_classify_noalloc(const void* Q, const void* K, int B, int nH, int D, const rf_layout* layout,
                            const rf_params* params, int sample_mode, float threshold, int32_t* head_class,
                            float* recalls, void* stream) {
    // every argument check, and the size limit, before any HIP call
    if (!Q || !K || !head_class || !layout) return RF_ERR_NULL;
    Geometry g;
    int st = resolve_geometry(layout, params, &g);
    if (st != RF_OK) return st;
    st = check_shape(B, nH, D);
    if (st != RF_OK) return st;
    if (!aligned16(Q) || !aligned16(K)) return RF_ERR_ALIGN;
    if (sample_mode != RF_SAMPLE_FIRST_FRAME && sample_mode != RF_SAMPLE_EQUAL_INTERVAL) return RF_ERR_PARAM;
    if (!(threshold >= 0.f && threshold <= 1.f)) return RF_ERR_PARAM;
    if (rf_arm_workspace_bytes(B, nH, layout, params) > kArmStaticScratchBytes) return RF_ERR_WORKSPACE;
    void* scratch = nullptr;
    size_t scratch_bytes = 0;
    if (arm_static_scratch(&scratch, &scratch_bytes) != 0) return RF_ERR_HIP;
    return arm_classify_impl(Q, K, B, nH, D, layout, params, sample_mode, threshold, nullptr, 1, head_class, nullptr,
                             recalls, scratch, scratch_bytes, stream);
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
    if (resolve_geometry(layout, params, &g) != RF_OK || check_shape(B, nH, D) != RF_OK) return 0;
    return RF_ATTENTION_MIN_WORKSPACE + 2 * static_cast<size_t>(B) * nH * g.N * D * sizeof(uint16_t);
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
    st = check_shape(B, nH, D);
    if (st != RF_OK) return st;
    if (!valid_block(block)) return RF_ERR_BLOCK;
    if (params && (params->flags & RF_FLAG_WIDE_ROWS) && (block != 256 || D != 128)) return RF_ERR_PARAM;
    if (!aligned16(Q) || !aligned16(K) || !aligned16(V) || !aligned16(O)) return RF_ERR_ALIGN;
    // the work-queue counters live in the first RF_ATTENTION_MIN_WORKSPACE bytes; a workspace of the
    // full size also has room for the packed copies of K and V
    if (!workspace || workspace_bytes < RF_ATTENTION_MIN_WORKSPACE) return RF_ERR_WORKSPACE;
    if (reinterpret_cast<uintptr_t>(workspace) & 255) return RF_ERR_ALIGN;
    const bool room_to_pack = workspace_bytes >= rf_attention_workspace_bytes(B, nH, D, layout, params);

    AttnArgs a{};
    a.n_plans = bandwidths ? n_bw : 1;
    for (int k = 0; k < a.n_plans; ++k) {
        Geometry gk = g;
        if (bandwidths) {
            st = geometry_with_bandwidth(layout, params, bandwidths[k], &gk);
            if (st != RF_OK) return st;
        }
        st = get_attention_plan(gk, block, &a.plan[k]);
        if (st != RF_OK) return st;
    }
    a.Q = static_cast<const uint16_t*>(Q);
    a.K = static_cast<const uint16_t*>(K);
    a.V = static_cast<const uint16_t*>(V);
    a.O = static_cast<uint16_t*>(O);
    a.queue = static_cast<int*>(workspace);
    a.join_sweep = (params && (params->flags & RF_FLAG_FIXED_ORDER)) ? 0 : 1;
    a.wide_rows = (params && (params->flags & RF_FLAG_WIDE_ROWS)) ? 1 : 0;
    a.head_class = force_dense ? nullptr : head_class;
    a.head_bw = bandwidths ? head_bw : nullptr;
    a.BH = B * nH;
    a.scale_log2 = static_cast<float>(1.4426950408889634 / std::sqrt(static_cast<double>(D)));
    if (room_to_pack && !force_dense) {
        a.packed_k = reinterpret_cast<uint16_t*>(static_cast<unsigned char*>(workspace) + RF_ATTENTION_MIN_WORKSPACE);
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
    if (g_plans.empty()) return RF_OK;
    int st = RF_OK;
    if (hipDeviceSynchronize() != hipSuccess) st = RF_ERR_HIP;
    for (auto& p : g_plans)
        if (p->blob && hipFree(p->blob) != hipSuccess) st = RF_ERR_HIP;
    g_plans.clear();
    return st;
}

}  // extern "C"
