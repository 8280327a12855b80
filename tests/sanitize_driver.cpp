// Host-only driver for the AddressSanitizer / UndefinedBehaviorSanitizer test: builds the block
// lists of the named layouts at every block size through the library's host code (rf_plan.cpp),
// checks their basic shape, and runs every oracle entry point on a small head.  Compiled and run
// by tests/test_sanitizers.py; prints "sanitize ok" when everything ran.
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rf_internal.h"

extern "C" {
typedef struct { int32_t T, H, W, text_len; } rfo_layout;
typedef struct { double bw_spatial, bw_temporal; int32_t tex_stride, sample_interval, two_head, text_first; } rfo_params;
int64_t rfo_num_tokens(const rfo_layout*);
int rfo_keep(int, int64_t, int64_t, const rfo_layout*, const rfo_params*);
void rfo_attention_rows(const float*, const float*, const float*, int, int, const rfo_layout*, const rfo_params*, const int64_t*, int64_t, double*, double*);
void rfo_attention_blockskip(const float*, const float*, const float*, int, int, const rfo_layout*, const rfo_params*, int, double*, int64_t*, int64_t*);
double rfo_arm_recall(const float*, const float*, int, const rfo_layout*, const rfo_params*, int, int, double*);
int rfo_arm_classify(const float*, const float*, int, const rfo_layout*, const rfo_params*, int, double, double*);
int rfo_arm_classify_plus(const float*, const float*, int, const rfo_layout*, const rfo_params*, int, double, const double*, int, int*, double*);
double rfo_kept_fraction(int, const rfo_layout*, const rfo_params*);
void rfo_keep_matrix(int, const rfo_layout*, const rfo_params*, uint8_t*);
}

static int fail(const char* what) {
    std::fprintf(stderr, "sanitize driver: %s\n", what);
    return 1;
}

static int check_plans() {
    const rf_layout layouts[] = {{13, 30, 45, 226}, {33, 45, 80, 256}, {24, 45, 80, 0}, {4, 8, 8, 0},
                                 {1, 5, 5, 0}, {1, 3, 3, 40}, {2, 2, 2, 1}, {3, 7, 9, 0}, {1, 1, 1, 0}, {5, 6, 11, 19}};
    const rf_params params[] = {{0.25f, 0.25f, 2, 0, 0}, {0.f, 0.f, 1, 0, 0}, {1.f, 1.f, 3, 0, 0}, {0.13f, 0.18f, 4, 7, RF_FLAG_TEXT_FIRST}};
    long long lists = 0, entries = 0;
    for (const rf_layout& L : layouts)
        for (const rf_params& P : params) {
            const bool big = static_cast<long long>(L.T) * L.H * L.W > 50000;
            if (big && &P != &params[0] && &P != &params[3]) continue;  // the paper-sized layouts: two settings are enough
            rf::Geometry g;
            if (rf::resolve_geometry(&L, &P, &g) != RF_OK) return fail("resolve_geometry refused a valid layout");
            for (int block : {64, 128, 256, 384}) {
                rf::HostPlan hp;
                rf::build_plan(g, block, &hp);
                for (int cls = RF_SPATIAL; cls <= RF_LIST_TEMPORAL_POSITION_MAJOR; ++cls) {
                    std::vector<int32_t> rp, co;
                    rf::flatten_class(hp, cls, &rp, &co);
                    if (static_cast<int>(rp.size()) != hp.nQB + 1 || rp[0] != 0 || rp.back() != static_cast<int32_t>(co.size()))
                        return fail("row_ptr does not frame the entries");
                    const int limit = (cls == RF_TEXTURAL) ? std::max(hp.nKT, hp.nCT) : hp.nKT;
                    for (int qb = 0; qb < hp.nQB; ++qb) {
                        if (rp[qb] > rp[qb + 1]) return fail("row_ptr decreases");
                        if (rp[qb] == rp[qb + 1]) return fail("a query block with no key tile");
                    }
                    for (int32_t e : co)
                        if ((e & rf::kTileIndexMask) >= limit) return fail("tile index out of range");
                    ++lists;
                    entries += static_cast<long long>(co.size());
                }
                for (int list = 0; list < rf::kLists; ++list) {
                    std::vector<char> seen(hp.nQB, 0);
                    for (int32_t qb : hp.qorder[list]) {
                        if (qb < 0 || qb >= hp.nQB || seen[qb]) return fail("block order is not a permutation");
                        seen[qb] = 1;
                    }
                }
            }
        }
    std::printf("plans: %lld lists, %lld entries\n", lists, entries);
    return 0;
}

static int check_oracle() {
    const rfo_layout L = {3, 4, 5, 7};
    const int D = 8;
    const int64_t N = rfo_num_tokens(&L);
    std::vector<float> Q(N * D), K(N * D), V(N * D);
    unsigned s = 12345u;
    auto rnd = [&]() { s = s * 1664525u + 1013904223u; return static_cast<float>((s >> 8) & 0xffff) / 65536.f - 0.5f; };
    for (auto* t : {&Q, &K, &V})
        for (float& x : *t) x = rnd();
    std::vector<int64_t> rows(N);
    for (int64_t i = 0; i < N; ++i) rows[i] = i;
    for (int text_first = 0; text_first < 2; ++text_first)
        for (int two_head = 0; two_head < 2; ++two_head) {
            const rfo_params P = {0.25, 0.3, 2, text_first ? 3 : 0, two_head, text_first};
            for (int cls = 0; cls < 4; ++cls) {
                std::vector<double> O(N * D), O2(N * D), prob(N * N);
                rfo_attention_rows(Q.data(), K.data(), V.data(), D, cls, &L, &P, rows.data(), N, O.data(), prob.data());
                int64_t visited = 0, total = 0;
                rfo_attention_blockskip(Q.data(), K.data(), V.data(), D, cls, &L, &P, 16, O2.data(), &visited, &total);
                if (visited < 1 || visited > total) return fail("block-skipping oracle visited an impossible number of blocks");
                std::vector<uint8_t> mask(N * N);
                rfo_keep_matrix(cls, &L, &P, mask.data());
                if (mask[0] != rfo_keep(cls, 0, 0, &L, &P)) return fail("keep matrix disagrees with the predicate");
                const double f = rfo_kept_fraction(cls, &L, &P);
                if (!(f > 0.0 && f <= 1.0)) return fail("kept fraction out of range");
            }
            for (int mode = 0; mode < 2; ++mode) {
                double rec[2], recp[2 * 3];
                std::vector<double> row_recall(64);
                rfo_arm_recall(Q.data(), K.data(), D, &L, &P, mode, 1, row_recall.data());
                const int c = rfo_arm_classify(Q.data(), K.data(), D, &L, &P, mode, 0.5, rec);
                const double bws[3] = {0.5, 0.25, 0.125};
                int idx = -2;
                const int cp = rfo_arm_classify_plus(Q.data(), K.data(), D, &L, &P, mode, 0.5, bws, 3, &idx, recp);
                if (c < 0 || c > 3 || cp < 0 || cp > 3 || idx < -1 || idx > 2) return fail("ARM oracle returned an impossible class");
            }
        }
    std::printf("oracle: every entry point ran\n");
    return 0;
}

int main() {
    if (check_plans() || check_oracle()) return 1;
    std::printf("sanitize ok\n");
    return 0;
}
