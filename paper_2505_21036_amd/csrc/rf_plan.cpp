// Host-side block lists for RainFusion's three head patterns (Sec. 3.2).
//
// The masks are token-level predicates; this file only decides, for a tiling of the N x N
// score matrix into query blocks of `block` rows and key tiles of 64 columns, which pairs
// contain at least one kept token pair (they are visited) and which of those contain a dropped
// pair or run past the last token (the kernel re-applies the predicate there).  Everything is exact integer interval
// arithmetic on frame indices and in-frame positions.
#include <algorithm>
#include <cmath>
#include <utility>

#include "rf_internal.h"

namespace rf {

static int band_radius(float bw, int n) {
    double r = std::floor(static_cast<double>(bw) * static_cast<double>(n));
    if (r < 0) r = 0;
    if (r > n) r = n;
    return static_cast<int>(r);
}

int resolve_geometry(const rf_layout* L, const rf_params* P, Geometry* g) {
    if (!L) return RF_ERR_NULL;
    if (L->T < 1 || L->H < 1 || L->W < 1 || L->text_len < 0) return RF_ERR_LAYOUT;
    const int64_t HW = static_cast<int64_t>(L->H) * L->W;
    const int64_t Nv = HW * L->T;
    const int64_t N = Nv + L->text_len;
    if (N > (int64_t{1} << 24)) return RF_ERR_SHAPE;  // keeps every index and block count in int32
    rf_params def = {0.25f, 0.25f, 2, 0, 0};
    const rf_params* p = P ? P : &def;
    if (!(p->bw_spatial >= 0.f && p->bw_spatial <= 1.f)) return RF_ERR_PARAM;
    if (!(p->bw_temporal >= 0.f && p->bw_temporal <= 1.f)) return RF_ERR_PARAM;
    if (p->tex_stride < 1 || p->sample_interval < 0) return RF_ERR_PARAM;
    if (p->flags & ~(RF_FLAG_TWO_HEAD | RF_FLAG_TEXT_FIRST | RF_FLAG_FORCE_DENSE | RF_FLAG_FIXED_ORDER | RF_FLAG_WIDE_ROWS)) return RF_ERR_PARAM;
    g->T = L->T; g->H = L->H; g->W = L->W; g->text_len = L->text_len;
    g->HW = static_cast<int>(HW); g->Nv = static_cast<int>(Nv); g->N = static_cast<int>(N);
    g->r_spatial = band_radius(p->bw_spatial, L->T);
    g->r_temporal = band_radius(p->bw_temporal, g->HW);
    g->tau = p->tex_stride;
    g->omega = p->sample_interval > 0 ? p->sample_interval : L->T;
    g->two_head = (p->flags & RF_FLAG_TWO_HEAD) ? 1 : 0;
    g->text_first = (p->flags & RF_FLAG_TEXT_FIRST) && L->text_len > 0 ? 1 : 0;
    return RF_OK;
}

namespace {

struct Span { int lo, hi; };  // inclusive

// In-frame positions covered by video tokens [s, e): one span per frame touched.
void position_spans(int s, int e, int HW, std::vector<Span>* out) {
    out->clear();
    if (s >= e) return;
    const int fs = s / HW, fe = (e - 1) / HW;
    for (int f = fs; f <= fe; ++f) {
        Span sp{f == fs ? s % HW : 0, f == fe ? (e - 1) % HW : HW - 1};
        out->push_back(sp);
        if (sp.lo == 0 && sp.hi == HW - 1) { out->assign(1, sp); return; }  // a whole frame covers all
    }
}

inline int span_gap(Span a, Span b) { return std::max(0, std::max(b.lo - a.hi, a.lo - b.hi)); }
inline int span_reach(Span a, Span b) { return std::max(b.hi - a.lo, a.hi - b.lo); }

}  // namespace

// How a head's query blocks are handed to workgroups.  The attention kernel runs one queue of
// (head, query block) items per XCD (each XCD has its own L2) and a workgroup takes items from other
// XCDs' queues once its own is empty, so the queues need not hold equal work.  Two things matter:
//  - The blocks that hold text rows are the long items (text queries see every key, so such a block
//    walks the whole sequence under every pattern).  They come first in the order, and the kernel
//    hands them out, for all heads, before anything else: the launch must not end waiting for one.
//  - The other blocks follow in a locality order, of which XCD x owns the x-th eighth, head after
//    head: blocks that run together (an XCD has about kConcurrentRows query rows in flight, a
//    generation) should walk the same key tiles at the same time, so that a tile is fetched into
//    the XCD's L2 once.  That order is token order (under the Temporal pattern in token order,
//    whose lists depend only on the in-frame position: grouped by position across frames); and in
//    the banded lists (Spatial; Temporal in position-major order), where a block's tiles are one
//    contiguous range that slides with the block, the blocks of a generation all start their walk
//    at the same tile, the first tile of the generation's last block, and wrap around: they then
//    sweep the same tiles in step instead of each trailing its neighbour by the slide.
static void order_query_blocks(HostPlan* plan) {
    HostPlan& P = *plan;
    const int nQB = P.nQB, block = P.block, HW = P.g.HW;
    const int nVB = P.first_text_qb, nTB = nQB - nVB;  // video-only blocks, text-holding blocks
    const int per_share = (nVB + 7) / 8;
    constexpr int kConcurrentRows = 8192;  // 32 CUs x 256 rows
    const int generation = std::max(1, kConcurrentRows / block);
    for (int cls = 0; cls < kLists; ++cls) {
        std::vector<int32_t>& ord = P.qorder[cls];
        ord.resize(nQB);
        for (int i = 0; i < nTB; ++i) ord[i] = nVB + i;
        for (int qb = 0; qb < nVB; ++qb) ord[nTB + qb] = qb;
        if (cls == RF_TEMPORAL) {
            auto key = [&](int qb) { return (static_cast<int64_t>(qb) * block % HW) / block; };
            std::stable_sort(ord.begin() + nTB, ord.end(), [&](int a, int b) { return key(a) < key(b); });
        }
        std::vector<int32_t>& fe = P.first_entry[cls];
        fe.assign(nQB, 0);
        if (cls != RF_SPATIAL && cls != kListTemporalPM) continue;
        auto tile_of = [&](int e) { return P.cols[cls][e] & kTileIndexMask; };
        for (int s0 = 0; s0 < nVB; s0 += per_share)
            for (int g0 = s0; g0 < std::min(s0 + per_share, nVB); g0 += generation) {
                const int g1 = std::min({g0 + generation, s0 + per_share, nVB});
                int start_tile = 0;
                for (int o = g0; o < g1; ++o) {
                    const int qb = ord[nTB + o];
                    if (P.row_ptr[cls][qb] < P.row_ptr[cls][qb + 1]) start_tile = std::max(start_tile, tile_of(P.row_ptr[cls][qb]));
                }
                for (int o = g0; o < g1; ++o) {
                    const int qb = ord[nTB + o], e0 = P.row_ptr[cls][qb], e1 = P.row_ptr[cls][qb + 1];
                    int e = e0;
                    while (e < e1 && tile_of(e) < start_tile) ++e;
                    fe[qb] = e < e1 ? e - e0 : 0;
                }
            }
    }
}

void build_plan(const Geometry& g, int block, HostPlan* plan) {
    HostPlan& P = *plan;
    P.g = g;
    P.block = block;
    const int N = g.N, Nv = g.Nv, HW = g.HW;
    P.nQB = (N + block - 1) / block;
    P.nKT = (N + kTileK - 1) / kTileK;
    P.first_text_qb = g.text_len > 0 ? Nv / block : P.nQB;

    // per-token attributes
    for (auto& a : P.attr) a.assign(N, 0);
    P.cidx.clear();
    P.pm_token.resize(N);
    for (int n = 0; n < Nv; ++n) {  // position-major row n = p*T + f
        const int p = n / g.T, f = n % g.T;
        P.pm_token[n] = g.row_of(f * HW + p);
        P.attr[kListTemporalPM][n] = p;
    }
    for (int n = Nv; n < N; ++n) P.pm_token[n] = g.row_of(n);
    for (int n = 0; n < Nv; ++n) {
        const int f = n / HW, p = n % HW, y = p / g.W, x = p % g.W;
        P.attr[RF_SPATIAL][n] = f;
        P.attr[RF_TEMPORAL][n] = p;
        const bool kept = ((y - x) % g.tau) == 0;
        P.attr[RF_TEXTURAL][n] = kept ? 0 : 1;
        if (kept) P.cidx.push_back(g.row_of(n));
    }
    for (int n = Nv; n < N; ++n) P.cidx.push_back(g.row_of(n));
    P.Nc = static_cast<int>(P.cidx.size());
    P.nCT = (P.Nc + kTileK - 1) / kTileK;

    std::vector<Span> qs, ks;
    for (int cls = 0; cls < kLists; ++cls) {
        // a band over groups of consecutive rows: frames of HW tokens (Spatial), positions of T tokens
        // (Temporal in position-major order)
        const bool banded = cls == RF_SPATIAL || cls == kListTemporalPM;
        const int group = cls == RF_SPATIAL ? HW : g.T, group_radius = cls == RF_SPATIAL ? g.r_spatial : g.r_temporal;
        auto& rp = P.row_ptr[cls];
        auto& co = P.cols[cls];
        rp.assign(P.nQB + 1, 0);
        co.clear();
        for (int qb = 0; qb < P.nQB; ++qb) {
            const int q0 = qb * block, q1 = std::min(N, q0 + block);
            const int qv1 = std::min(q1, Nv);  // video part [q0, qv1)
            const bool q_text = q1 > Nv, q_video = q0 < Nv;
            if (cls == RF_TEXTURAL && !q_text) { rp[qb + 1] = static_cast<int32_t>(co.size()); continue; }
            if (cls == RF_TEMPORAL && q_video) position_spans(q0, qv1, HW, &qs);
            for (int kb = 0; kb < P.nKT; ++kb) {
                const int k0 = kb * kTileK, k1 = std::min(N, k0 + kTileK);
                const int kv1 = std::min(k1, Nv);
                const bool k_text = k1 > Nv, k_video = k0 < Nv;
                bool any = q_text || k_text, all = true;
                if (q_video && k_video) {
                    if (banded) {
                        Span a{q0 / group, (qv1 - 1) / group}, b{k0 / group, (kv1 - 1) / group};
                        any = any || span_gap(a, b) <= group_radius;
                        all = span_reach(a, b) <= group_radius;
                    } else if (cls == RF_TEMPORAL) {
                        position_spans(k0, kv1, HW, &ks);
                        for (Span a : qs)
                            for (Span b : ks) {
                                any = any || span_gap(a, b) <= g.r_temporal;
                                all = all && span_reach(a, b) <= g.r_temporal;
                            }
                    } else {  // Textural rows of a block that also holds text rows
                        bool every_kept = true, some_kept = false;
                        for (int j = k0; j < kv1; ++j) {
                            const bool kept = P.attr[RF_TEXTURAL][j] == 0;
                            every_kept = every_kept && kept;
                            some_kept = some_kept || kept;
                        }
                        any = any || some_kept;
                        all = every_kept;
                    }
                }
                if (!any) continue;
                const bool tail = k0 + kTileK > N;
                // a tile of text keys only is never partial; one that mixes text and video keys, or
                // runs past N, needs the position checks as well as the pattern's band check
                const bool boundary = tail || (k_text && k_video && !all);
                co.push_back(kb | ((!all || tail) ? RF_PLAN_PARTIAL : 0) | (boundary ? kTileBoundary : 0));
            }
            rp[qb + 1] = static_cast<int32_t>(co.size());
        }
    }
    order_query_blocks(plan);
}

// cls in the public numbering: a head class, or RF_LIST_TEMPORAL_POSITION_MAJOR
void flatten_class(const HostPlan& P, int cls, std::vector<int32_t>* row_ptr, std::vector<int32_t>* cols) {
    const int list = cls == RF_LIST_TEMPORAL_POSITION_MAJOR ? kListTemporalPM : cls;
    row_ptr->assign(P.nQB + 1, 0);
    cols->clear();
    for (int qb = 0; qb < P.nQB; ++qb) {
        if (cls == RF_DENSE || (cls == RF_TEXTURAL && qb < P.first_text_qb)) {
            const int nt = cls == RF_DENSE ? P.nKT : P.nCT;
            const int len = cls == RF_DENSE ? P.g.N : P.Nc;
            for (int kt = 0; kt < nt; ++kt)
                cols->push_back(kt | ((kt + 1) * kTileK > len ? RF_PLAN_PARTIAL : 0));
        } else {
            for (int e = P.row_ptr[list][qb]; e < P.row_ptr[list][qb + 1]; ++e)
                cols->push_back(P.cols[list][e] & ~kTileBoundary);
        }
        (*row_ptr)[qb + 1] = static_cast<int32_t>(cols->size());
    }
}

}  // namespace rf
