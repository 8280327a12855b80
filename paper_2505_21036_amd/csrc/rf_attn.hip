// Block-sparse attention forward for RainFusion's head patterns (Eq. 1-5; Fig. 2a), gfx950.
//
// Work item = one query block (64, 128, 256 or 384 rows) of one head; a resident set of workgroups
// takes items from per-XCD queues.  For its item a workgroup reads the head's class on the device,
// walks that class's list of 64-key tiles (skipped tiles cost no traffic), loads K and V tiles
// global -> LDS one tile ahead without staging registers, forms the transposed score tile with
// bf16 MFMA, runs the online softmax in fp32 with exp2, and accumulates O^T = V^T P^T with bf16
// MFMA.  In tiles flagged partial the token-level predicate of the pattern is re-applied to each
// score.
#include <algorithm>
#include <mutex>
#include <type_traits>

#include "rf_device.h"

namespace rf {

// How a query block finds its key tiles.
enum : int {
    MODE_ALL = 0,      // every key tile of the sequence in order (dense heads)
    MODE_COMPACT = 1,  // every tile of the compacted key sequence; rows go through the index table (Eq. 5)
    MODE_LISTED = 2    // the CSR list of the head's pattern; partial tiles re-apply the predicate
};

// K/V tiles kept in flight ahead of the one being consumed.  Two (with a third buffer) measured no
// faster than one at any shape: the loads are not what the wavefronts wait for.
#ifndef RF_TILES_AHEAD
#define RF_TILES_AHEAD 1
#endif

template <int D, int NW>
struct AttnSmem {
    using ST = DirectTile<D, NW>;
    // K/V tiles resident at a time: the one being consumed plus AHEAD on their way
    static constexpr int AHEAD = RF_TILES_AHEAD;
    static constexpr int DEPTH = AHEAD + 1;
    static constexpr int SIDE_SLOTS = DEPTH + 1;  // side data runs one tile further ahead than K/V
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = DEPTH * ST::K_BYTES;
    static constexpr int SIDE_OFF = V_OFF + DEPTH * ST::V_BYTES;  // ring of 64-int slots: key indices or key attributes
    static constexpr int ITEM_OFF = SIDE_OFF + SIDE_SLOTS * kTileK * 4;  // two ints: the work item just taken
    static constexpr int BYTES = ITEM_OFF + 16;
    static_assert(K_OFF % 256 == 0 && V_OFF % 256 == 0 && ST::K_BYTES % 256 == 0 && ST::V_BYTES % 256 == 0,
                  "tile buffers must start at multiples of 256 bytes (see DirectTile::k_address)");
};

struct QueryBlock {
    int bh, qb, cls;
    int list;                    // MODE_LISTED: which of the plan's lists (a class, or Temporal position-major)
    const int32_t* row_token;    // null, or: row of the walked order -> token (queries are gathered, O scattered)
    const unsigned char* kbase;  // K and V rows of the key sequence walked (the head's, or its compacted copy)
    const unsigned char* vbase;
    // tensor row of walked index n = n + (n < Nv ? video_shift : text_shift); both 0 unless the text
    // tokens come first in the tensors, and 0 when kbase/vbase are packed copies (already in walked order)
    int video_shift, text_shift;
    const int32_t* cols;  // MODE_LISTED: this query block's tile entries
    int first;            // entry (tile, for the unlisted walks) the cyclic walk starts at
    int ntiles;           // key tiles to visit
    int* sweep;           // null, or: where this workgroup publishes how far its walk has come (see join_sweep)
    int sweep_tag;        // which key sequence the published tile index refers to
    int keyN;             // length of the key sequence walked (N, or Nc when compacted)
};

// Workgroups of one XCD share that XCD's L2, so they should walk the same key tiles at the same time.
// Items are handed out one by one as workgroups finish, so a workgroup that starts an item finds the
// others somewhere in the middle of theirs: it joins them.  Every workgroup publishes, every few
// tiles, the tile its walk has reached (with a tag naming the head and the key sequence) in one of
// kSweepSlots words per XCD next to the work-queue counters (an XCD is usually on two or three heads
// at a time: the slot is the head's index modulo kSweepSlots); a starting workgroup whose item walks
// the same sequence begins its cyclic walk at that tile if the tile is in its list.  This only moves
// where the walk starts: every tile of the list is still visited exactly once.
constexpr int kSweepTileBits = 18, kSweepTileMask = (1 << kSweepTileBits) - 1;  // N <= 2^24 tokens: tile indices below 2^18
constexpr int kSweepSlots = 8, kQueueWords = 8 + 8 * kSweepSlots;
static_assert(kQueueWords * 4 <= RF_ATTENTION_MIN_WORKSPACE, "counters and sweep words live in the minimum workspace");
__device__ __forceinline__ int* sweep_word(int* queue, int xcd, int bh) { return queue + 8 + xcd * kSweepSlots + (bh & (kSweepSlots - 1)); }

// exp2 arguments may exceed 0 by at most this much before the running reference is moved: the
// softmax is invariant to the reference, so a stale one only costs range, which fp32/bf16 have.
constexpr float kRescaleSlack = 8.f;

}  // namespace rf

#include "rf_attn_wide.h"

namespace rf {

// QH: 32-query halves a wavefront owns (1, or 2: every K and V slab read from LDS then feeds two MFMAs).
template <int D, int NW, int MODE, int QH = 1>
__device__ __forceinline__ void attend(const AttnArgs& a, const DevicePlan& pl, const QueryBlock& qk, unsigned char* smem) {
    constexpr int BQ = 32 * NW * QH;
    using ST = DirectTile<D, NW>;
    using SM = AttnSmem<D, NW>;
    constexpr int DEPTH = SM::DEPTH;
    // how many slabs ahead of their MFMAs the LDS operand reads run: with two halves every slab feeds two
    // MFMAs and the registers are all in use, and two measured best (dense CogVideoX-shaped layer 4.25 ->
    // 3.99 ms against the depths of the one-half loop); twelve wavefronts at head_dim 128 have 168
    // registers each, which the loops fit without spills at depth two
    constexpr int AK = (QH == 2 || (NW == 12 && D == 128)) ? 2 : kAheadK, AV = (QH == 2 || (NW == 12 && D == 128)) ? 2 : kAheadV;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;
    const int N = pl.N, Nv = pl.Nv, keyN = qk.keyN, ntiles = qk.ntiles;
    // per-key side data staged through LDS two tiles ahead: the token index of each key of the
    // compacted sequence, or the pattern attribute (frame / position / kept flag) of each key
    const int32_t* side_src = MODE == MODE_COMPACT ? pl.cidx : (MODE == MODE_LISTED ? pl.attr[qk.list] : nullptr);
    int* side = reinterpret_cast<int*>(smem + SM::SIDE_OFF);

    const unsigned char* Kh = qk.kbase;
    const unsigned char* Vh = qk.vbase;
    const uint16_t* Qh = a.Q + static_cast<size_t>(qk.bh) * N * D;

    // this lane's queries, one per half
    int qrow[QH], qtok[QH];
    bf16x8 qf[QH][D / 16];
    uint32_t q_lo[QH], q_span[QH];
#pragma unroll
    for (int h = 0; h < QH; ++h) {
        qrow[h] = qk.qb * BQ + wave * (32 * QH) + 32 * h + m;  // row of the walked order
        const int qrow_c = min(qrow[h], N - 1);
        qtok[h] = (MODE == MODE_LISTED && qk.row_token) ? qk.row_token[qrow_c]
                                                        : qrow_c + (qrow_c < Nv ? pl.video_shift : pl.text_shift);
        load_q_frags<D>(Qh, qtok[h], hf, qf[h]);
        int q_attr = 0, q_rad = 0x3fffffff;  // text queries keep everything
        if (MODE == MODE_LISTED) {
            // Spatial / Temporal compare the query's frame / position with the key's; the Textural
            // table is 0 on kept keys and 1 on dropped ones, compared against 0 with radius 0
            if (qk.cls != RF_TEXTURAL) q_attr = side_src[qrow_c];
            if (qrow_c < Nv) q_rad = pl.radius[qk.list];
        }
        q_lo[h] = static_cast<uint32_t>(q_rad - q_attr);
        q_span[h] = 2u * static_cast<uint32_t>(q_rad);
    }

    f32x16 oacc[QH][D / 32];
#pragma unroll
    for (int h = 0; h < QH; ++h)
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[h][db] = f32x16{0};
    // m_ref: reference subtracted inside exp2 (raw score units), finite from the start; has_ref: it has
    // been taken from real scores of this row; l_run: this lane's share of the softmax denominator
    float m_ref[QH], l_run[QH];
    bool has_ref[QH];
#pragma unroll
    for (int h = 0; h < QH; ++h) {
        m_ref[h] = 0.f;
        l_run[h] = 0.f;
        has_ref[h] = false;
    }
    const float c = a.scale_log2;

    ST st;
    st.init(tid);
    int side_reg = 0;

    // Tile entries of a listed query block are read 64 at a time, one per lane, and handed out with
    // v_readlane: no scalar-load latency in the loop.  ent_cur covers [ent_base, ent_base + 64).
    int ent_cur = 0, ent_nxt = 0, ent_base = 0;
    auto load_entries = [&](int from) {
        const int j = min(from + lane, ntiles - 1) + qk.first;  // the walk starts at entry qk.first and wraps
        return qk.cols[j < ntiles ? j : j - ntiles];
    };
    if (MODE == MODE_LISTED && ntiles > 0) {
        ent_cur = load_entries(0);
        ent_nxt = load_entries(64);
    }
    // entries must be asked for in increasing t
    auto entry_of = [&](int t) -> int {
        if (MODE == MODE_LISTED) {
            if (t >= ent_base + 64) {
                ent_base += 64;
                ent_cur = ent_nxt;
                ent_nxt = load_entries(ent_base + 64);
            }
            return __builtin_amdgcn_readlane(ent_cur, t - ent_base);
        }
        int tile = t + qk.first;  // the walk starts at tile qk.first and wraps
        if (tile >= ntiles) tile -= ntiles;
        return tile | ((tile + 1) * kTileK > keyN ? (RF_PLAN_PARTIAL | kTileBoundary) : 0);
    };
    // side data is needed for every tile of the compacted sequence, and for partial listed tiles
    auto wants_side = [&](int entry) { return MODE == MODE_COMPACT || (MODE == MODE_LISTED && (entry & RF_PLAN_PARTIAL)); };
    auto load_side = [&](int entry) {
        if (!wants_side(entry)) return;
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (tid < kTileK) side_reg = side_src[min(k0 + tid, keyN - 1)];
    };
    auto stash_side = [&](int t, int entry) {
        if (!wants_side(entry)) return;
        if (tid < kTileK) side[(t % SM::SIDE_SLOTS) * kTileK + tid] = side_reg;
    };
    auto k_lds = [&](int t) { return smem + SM::K_OFF + (t % DEPTH) * ST::K_BYTES; };
    auto v_lds = [&](int t) { return smem + SM::V_OFF + (t % DEPTH) * ST::V_BYTES; };
    auto fetch_tile = [&](int t, int entry) {
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (MODE == MODE_COMPACT) {
            const int* idx = side + (t % SM::SIDE_SLOTS) * kTileK;
            st.issue(Kh, Vh, k_lds(t), v_lds(t), [&](int row) { return idx[row]; });
        } else if (k0 + kTileK <= keyN && !(qk.text_shift != 0 && k0 < Nv && k0 + kTileK > Nv)) {
            // full tile of consecutive tensor rows: everything but the tile origin is loop invariant
            const int r0 = k0 + (k0 < Nv ? qk.video_shift : qk.text_shift);
            const size_t origin = static_cast<size_t>(r0) * (2 * D);
            st.issue_consecutive(Kh + origin, Vh + origin, k_lds(t), v_lds(t));
        } else {
            st.issue(Kh, Vh, k_lds(t), v_lds(t), [&](int row) {
                const int n = min(k0 + row, keyN - 1);
                return n + (n < Nv ? qk.video_shift : qk.text_shift);
            });
        }
    };

    // S^T of tile t (64 keys x this lane's query of each half), predicate applied where the tile is partial
    auto scores = [&](int t, int entry, f32x16 (&s)[QH][2]) {
        if (QH == 1) {
            st.template scores<AK>(st.k_address(k_lds(t)), qf[0], s[0]);
        } else {
            // as DirectTile::scores, every K slab feeding one MFMA per half
            constexpr int NQK = 2 * (D / 16);
            const uint32_t ka = st.k_address(k_lds(t));
            bf16x8 frag[NQK];
#pragma unroll
            for (int i = 0; i < AK; ++i) frag[i] = st.k_frag(ka, i & 1, i >> 1);
#pragma unroll
            for (int h = 0; h < QH; ++h) {
                s[h][0] = f32x16{0};
                s[h][1] = f32x16{0};
            }
#pragma unroll
            for (int j = 0; j < NQK; ++j) {
                if (j + AK < NQK) frag[j + AK] = st.k_frag(ka, (j + AK) & 1, (j + AK) >> 1);
#pragma unroll
                for (int h = 0; h < QH; ++h) {
                    s[h][j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[j], qf[h][j >> 1], s[h][j & 1], 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        }
        if (entry & RF_PLAN_PARTIAL) {
            const int k0 = (entry & kTileIndexMask) * kTileK;
            const int* al = side + (t % SM::SIDE_SLOTS) * kTileK;
#pragma unroll
            for (int h = 0; h < QH; ++h) {
                // this lane's keys come in runs of eight: keys 32*kb2 + 16*u + 8*hf .. +7 sit in registers 8*u .. 8*u+7
                typedef __attribute__((address_space(3))) const u32x4 lds_u32x4;
                const bool band_only = MODE == MODE_LISTED && !(entry & kTileBoundary);  // all 64 keys are video tokens
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        const int base = 32 * kb2 + 16 * u + 8 * hf;
                        uint32_t at[8] = {};
                        if (MODE == MODE_LISTED) {
                            const u32x4 a0 = *(lds_u32x4*)(uintptr_t)ST::lds_offset(reinterpret_cast<const unsigned char*>(al + base));
                            const u32x4 a1 = *(lds_u32x4*)(uintptr_t)ST::lds_offset(reinterpret_cast<const unsigned char*>(al + base + 4));
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                at[i] = a0[i];
                                at[4 + i] = a1[i];
                            }
                        }
#pragma unroll
                        for (int i = 0; i < 8; ++i) {
                            const int kidx = k0 + base + i;
                            bool ok = band_only || kidx < keyN;
                            if (MODE == MODE_LISTED) ok = ok & ((at[i] + q_lo[h] <= q_span[h]) | (!band_only && kidx >= Nv));
                            s[h][kb2][8 * u + i] = ok ? s[h][kb2][8 * u + i] : -INFINITY;
                        }
                    }
            }
        }
    };

    // O^T += V^T P^T for tile t, P (bf16) in pf
    bf16x8 pf[QH][4];
    auto accumulate = [&](int t) {
        const uint32_t va = st.v_address(v_lds(t));
        // consecutive MFMAs go to different accumulators (channel blocks, halves): no back-to-back
        // dependence; operand reads kAheadV slabs ahead, order fenced as for the scores
        constexpr int NPV = 4 * (D / 32), NDB = D / 32;
        bf16x8 frag[NPV];
#pragma unroll
        for (int i = 0; i < AV; ++i) frag[i] = ST::v_frag(va, i % NDB, i / NDB);
#pragma unroll
        for (int j = 0; j < NPV; ++j) {
            if (j + AV < NPV) frag[j + AV] = ST::v_frag(va, (j + AV) % NDB, (j + AV) / NDB);
#pragma unroll
            for (int h = 0; h < QH; ++h) {
                oacc[h][j % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[j], pf[h][j / NDB], oacc[h][j % NDB], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
    };
    // Software pipeline.  While tile t is consumed, the loads of tiles t+1 .. t+AHEAD are in flight
    // or landed, and the side data of tile t+DEPTH is on its way to its ring slot (one tile further,
    // because the loads of a compacted tile take their row indices from it).  e[i] = entry of tile t+i.
    constexpr int AHEAD = SM::AHEAD;
    int e[DEPTH + 1] = {};
#pragma unroll
    for (int i = 0; i < DEPTH; ++i)
        if (i < ntiles) {
            e[i] = entry_of(i);
            load_side(e[i]);
            stash_side(i, e[i]);
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < AHEAD; ++i)
        if (i < ntiles) fetch_tile(i, e[i]);
    ST::template wait_landed<0>();
    __syncthreads();
    // The compiler cannot see the tile loads above, so its own wait for the Q loads, if left inside
    // the loop, would count them out too and wait for the tiles in flight; make it wait here.
#pragma unroll
    for (int h = 0; h < QH; ++h)
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, qf[h][cc])));

    for (int t = 0; t < ntiles; ++t) {
        // the buffer of tile t+AHEAD held tile t+AHEAD-DEPTH, which every wavefront left before the last barrier
        if (t + DEPTH < ntiles) e[DEPTH] = entry_of(t + DEPTH);
        if (t + AHEAD < ntiles) fetch_tile(t + AHEAD, e[AHEAD]);
        if (t + DEPTH < ntiles) load_side(e[DEPTH]);
        const int e_cur = e[0];
        // every eighth tile, tell the workgroups that start an item on this XCD where this walk is
        if (qk.sweep && (t & 7) == 0 && tid == 0)
            __hip_atomic_store(qk.sweep, (qk.sweep_tag << kSweepTileBits) | (e_cur & kSweepTileMask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);

        // Online softmax (Eq. 1) in base 2 with 1/sqrt(D) folded into c.  The reference subtracted in
        // the exponent is moved, and the accumulators rescaled, only when a row outgrows it by more
        // than 2^kRescaleSlack (or has none yet): the softmax does not depend on the reference.
        f32x16 s[QH][2];
        scores(t, e_cur, s);
        // With eight wavefronts at head_dim 128 the softmax section (VALU only) runs at raised
        // priority and the two MFMA sections at the default: the wavefront that shares the SIMD is
        // then served in the gaps of this one's VALU work rather than the other way round (measured
        // +1 % there; neutral at head_dim 96 and 1-4 % slower with four wavefronts, so not there).
        constexpr bool kSoftmaxPriority = D == 128 && NW == 8;
        if (kSoftmaxPriority) __builtin_amdgcn_s_setprio(1);
#pragma unroll
        for (int h = 0; h < QH; ++h) {
            float mt = s[h][0][0];
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) mt = fmaxf(mt, s[h][kb2][r]);
            // the two halves of the wavefront hold different keys of the same 32 queries: their maxima
            // are exchanged only when some lane asks for the reference to move
            const bool grow = has_ref[h] ? (mt - m_ref[h]) * c > kRescaleSlack : mt > -INFINITY;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                mt = fmaxf(mt, other_half(mt));
                if (mt > -INFINITY) {
                    const float m_new = has_ref[h] ? fmaxf(m_ref[h], mt) : mt;
                    const float alpha = has_ref[h] ? fast_exp2((m_ref[h] - m_new) * c) : 0.f;  // nothing accumulated before
                    l_run[h] *= alpha;
#pragma unroll
                    for (int db = 0; db < D / 32; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[h][db][r] *= alpha;
                    m_ref[h] = m_new;
                    has_ref[h] = true;
                }
            }
            // p = exp2((s - m_ref) * c) in place
            const float mc = m_ref[h] * c;
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[h][kb2][r] = fast_exp2(fmaf(s[h][kb2][r], c, -mc));
            // P is rounded to bf16 for the second MFMA; the denominator sums those same rounded values
            // (two per v_dot2c_f32_bf16), so numerator and denominator of Eq. 2 see identical weights
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int u2 = 0; u2 < 2; ++u2) {
                    u32x4 w;
                    w.x = pack_bf16(s[h][kb2][8 * u2 + 0], s[h][kb2][8 * u2 + 1]);
                    w.y = pack_bf16(s[h][kb2][8 * u2 + 2], s[h][kb2][8 * u2 + 3]);
                    w.z = pack_bf16(s[h][kb2][8 * u2 + 4], s[h][kb2][8 * u2 + 5]);
                    w.w = pack_bf16(s[h][kb2][8 * u2 + 6], s[h][kb2][8 * u2 + 7]);
                    l_run[h] = add_bf16_pair(add_bf16_pair(add_bf16_pair(add_bf16_pair(l_run[h], w.x), w.y), w.z), w.w);
                    pf[h][2 * kb2 + u2] = as_bf16x8(w);
                }
        }
        if (kSoftmaxPriority) __builtin_amdgcn_s_setprio(0);
        accumulate(t);

        // tile t+1 must be in LDS at the barrier; the loads of the tiles after it may stay in flight
        if (AHEAD > 1 && t + AHEAD < ntiles) ST::template wait_landed<AHEAD - 1>();
        else ST::template wait_landed<0>();
        if (t + DEPTH < ntiles) stash_side(t + DEPTH, e[DEPTH]);
#pragma unroll
        for (int i = 0; i < DEPTH; ++i) e[i] = e[i + 1];
        __syncthreads();
    }
    // Eq. 2: divide by the softmax denominator and store.  Lane (hf, m) owns query m and, per
    // 32-channel block, channels 8*(r/4) + 4*hf + r%4.
#pragma unroll
    for (int h = 0; h < QH; ++h) {
        const float l_tot = l_run[h] + other_half(l_run[h]);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        if (qrow[h] < N) {
            uint16_t* orow = a.O + static_cast<size_t>(qk.bh) * N * D + static_cast<size_t>(qtok[h]) * D;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int rq = 0; rq < 4; ++rq) {
                    u32x2 w;
                    w.x = pack_bf16(oacc[h][db][4 * rq + 0] * inv, oacc[h][db][4 * rq + 1] * inv);
                    w.y = pack_bf16(oacc[h][db][4 * rq + 2] * inv, oacc[h][db][4 * rq + 3] * inv);
                    *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * rq + 4 * hf) = w;
                }
        }
    }
}

// Which tile loop a kernel instance runs.
enum : int {
    LOOP_32 = 0,           // wavefronts of 32 query rows (attend)
    LOOP_64_PIPELINED = 1, // wavefronts of 64 rows, one per SIMD, software-pipelined (attend_wide)
    LOOP_64 = 2            // wavefronts of 64 rows on the plain loop (attend with two halves): head_dim 64 only, where two fit a SIMD
};
constexpr int rows_per_wave(int LOOP) { return LOOP == LOOP_32 ? 32 : 64; }

// Wavefronts per SIMD the register allocation is held to: three for head_dim 64 with 128-row
// blocks of 32-row wavefronts (measured best; its accumulators are half the size) and for the
// twelve-wavefront workgroups of 384-row blocks, two otherwise; one for the pipelined 64-row loop,
// which needs the whole register file.
constexpr int attn_waves_per_simd(int D, int NW, int LOOP) {
    return LOOP == LOOP_64_PIPELINED ? 1 : (LOOP == LOOP_32 && ((D == 64 && NW == 4) || NW == 12)) ? 3 : 2;
}

template <int D, int NW, int LOOP>
using SmemOf = std::conditional_t<LOOP == LOOP_64_PIPELINED, WideSmem<D, NW>, AttnSmem<D, NW>>;

// Items of one launch.  Queue x holds first its share of the long items (the nTB text-holding blocks
// of every head: global index i = head * nTB + k goes to queue i mod 8), then, head after head, the
// ordinals [x * per_xcd, (x+1) * per_xcd) of the order of the nVB other blocks.
struct Queues {
    int BH, nVB, nTB, per_xcd;
    __device__ __forceinline__ int long_items(int x) const { return (nTB * BH - x + 7) >> 3; }
    __device__ __forceinline__ int share(int x) const { return max(0, min(per_xcd, nVB - x * per_xcd)); }
    __device__ __forceinline__ int items(int x) const { return long_items(x) + share(x) * BH; }
};

// The next item for a workgroup whose home queue is `home`, or -1 when every queue is empty.
// ctr[x] counts how many items of queue x have been handed out.  A workgroup drains its home queue
// first (its neighbours on the XCD are on the same part of the same head, which is what the L2
// wants) and then helps whichever queue has the most left.  Every path ends: counters only grow, a
// failed take means another workgroup took that item, and once all are taken -1 is returned.
__device__ __forceinline__ int take_item(int* ctr, int home, const Queues& qs, int* queue) {
    auto taken = [&](int x) { return __hip_atomic_load(ctr + x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT); };
    int q = home;
    for (;;) {
        if (taken(q) < qs.items(q)) {
            const int j = __hip_atomic_fetch_add(ctr + q, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (j < qs.items(q)) {
                *queue = q;
                return j;
            }
        }
        int best = -1, best_left = 0;
        for (int x = 0; x < 8; ++x) {
            const int left = qs.items(x) - taken(x);
            if (left > best_left) {
                best_left = left;
                best = x;
            }
        }
        if (best < 0) return -1;
        q = best;
    }
}

// head of the item-th item of queue xcd (see Queues)
__device__ __forceinline__ int item_head(int item, int xcd, const Queues& qs) {
    const int longs = qs.long_items(xcd);
    return item < longs ? (item * 8 + xcd) / qs.nTB : (item - longs) / qs.share(xcd);
}

template <int D, int NW, int LOOP>
__device__ __forceinline__ void process_item(const AttnArgs& a, int item, int xcd, int seen, const Queues& qs, unsigned char* smem);

// Eight queue counters, then the sweep words (-1: nothing published yet).
__global__ void reset_queue_kernel(int* ctr) {
    if (threadIdx.x < kQueueWords) ctr[threadIdx.x] = threadIdx.x < 8 ? 0 : -1;
}

// NW wavefronts of rows_per_wave(LOOP) query rows each.
template <int D, int NW, int LOOP>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(attn_waves_per_simd(D, NW, LOOP), attn_waves_per_simd(D, NW, LOOP)))) attn_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];  // the kernel's only LDS: starts at address 0
    int* item_box = reinterpret_cast<int*>(smem + SmemOf<D, NW, LOOP>::ITEM_OFF);
    // A resident set of workgroups (as many as fit on the chip) works through the (head, query
    // block) items.  Workgroup ids go to the 8 XCDs round-robin; XCD x's queue is one eighth of every
    // head's block order, head after head (neighbours in that order walk nearly the same key tiles,
    // which they share through the XCD's L2), so all XCDs move through the heads together and the
    // K/V of the head in flight (tens of MB) stays resident in the memory-side cache for whatever
    // misses L2.  XCDs differ in speed by several per cent and shares in work; an XCD whose queue is
    // empty takes items from the others.
    Queues qs;
    qs.BH = a.BH;
    qs.nVB = a.plan[0].first_text_qb;
    qs.nTB = a.plan[0].nQB - qs.nVB;
    qs.per_xcd = (qs.nVB + 7) >> 3;
    for (;;) {
        if (threadIdx.x == 0) {
            int q = 0;
            item_box[0] = take_item(a.queue, blockIdx.x & 7, qs, &q);
            item_box[1] = q;
            // the sweep word for the item's head on this workgroup's XCD (it serves its own L2, whichever queue
            // the item came from), read ONCE for the whole workgroup: it changes all the time
            const int it = item_box[0];
            item_box[2] = (a.join_sweep && it >= 0)
                              ? __hip_atomic_load(sweep_word(a.queue, blockIdx.x & 7, item_head(it, q, qs)), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)
                              : -1;
        }
        __syncthreads();
        // wavefront-uniform by construction; say so, so that everything derived stays in scalar registers
        const int item = __builtin_amdgcn_readfirstlane(item_box[0]), xcd = __builtin_amdgcn_readfirstlane(item_box[1]);
        const int seen = __builtin_amdgcn_readfirstlane(item_box[2]);
        __syncthreads();
        if (item < 0) break;
        process_item<D, NW, LOOP>(a, item, xcd, seen, qs, smem);
    }
}

// One (head, query block) item: item-th of queue xcd.  seen: the sweep word of this workgroup's XCD
// (it serves its own L2, whichever queue the item came from), or -1.
template <int D, int NW, int LOOP>
__device__ __forceinline__ void process_item(const AttnArgs& a, int item, int xcd, int seen, const Queues& qs, unsigned char* smem) {
    auto run = [&](auto mode, const DevicePlan& plan, const QueryBlock& block) {
        constexpr int MODE = decltype(mode)::value;
        if constexpr (LOOP == LOOP_64_PIPELINED) attend_wide<D, NW, MODE>(a, plan, block, smem);
        else attend<D, NW, MODE, rows_per_wave(LOOP) / 32>(a, plan, block, smem);
    };
    // position in the block order, and the head
    int ordinal, bh;
    const int longs = qs.long_items(xcd);
    if (item < longs) {
        const int i = item * 8 + xcd;
        bh = i / qs.nTB;
        ordinal = i % qs.nTB;
    } else {
        const int share = qs.share(xcd), j = item - longs;
        bh = j / share;
        ordinal = qs.nTB + xcd * qs.per_xcd + j % share;
    }
    QueryBlock qk;
    qk.bh = bh;
    // per-head bandwidth: the plans differ only in the Spatial / Temporal lists, radii and block order
    int which = 0;
    if (a.head_bw) {
        which = a.head_bw[qk.bh];
        if (static_cast<unsigned>(which) >= static_cast<unsigned>(a.n_plans)) which = 0;
    }
    const DevicePlan& pl = a.plan[which];
    int cls = a.head_class ? a.head_class[qk.bh] : RF_DENSE;
    if (static_cast<unsigned>(cls) > 3u) cls = RF_DENSE;
    qk.cls = cls;
    // a Temporal head walks the position-major copy of its K and V if the caller gave room for one
    const bool temporal_pm = cls == RF_TEMPORAL && a.packed_k;
    const int list = temporal_pm ? kListTemporalPM : cls;
    // dense heads: text-holding blocks first, then token order
    qk.qb = cls == RF_DENSE ? (ordinal < qs.nTB ? qs.nVB + ordinal : ordinal - qs.nTB) : pl.qorder[list][ordinal];
    qk.first = 0;
    qk.cols = nullptr;
    qk.sweep = a.join_sweep ? sweep_word(a.queue, blockIdx.x & 7, bh) : nullptr;
    auto same_sequence = [&]() { return seen >= 0 && (seen >> kSweepTileBits) == qk.sweep_tag; };
    qk.list = cls;
    qk.row_token = nullptr;
    qk.video_shift = pl.video_shift;
    qk.text_shift = pl.text_shift;
    const size_t head_bytes = static_cast<size_t>(qk.bh) * pl.N * D * 2;
    qk.kbase = reinterpret_cast<const unsigned char*>(a.K) + head_bytes;
    qk.vbase = reinterpret_cast<const unsigned char*>(a.V) + head_bytes;
    // tag: the head and which of its key sequences is walked (token order, compacted, position-major)
    const int kTagBits = 31 - kSweepTileBits;
    auto tag_of = [&](int sequence) { return (qk.bh * 4 + sequence) & ((1 << kTagBits) - 1); };
    if (cls == RF_DENSE) {
        qk.ntiles = pl.nKT;
        qk.keyN = pl.N;
        qk.sweep_tag = tag_of(0);
        if (same_sequence() && (seen & kSweepTileMask) < qk.ntiles) qk.first = seen & kSweepTileMask;
        run(std::integral_constant<int, MODE_ALL>{}, pl, qk);
    } else if (cls == RF_TEXTURAL && qk.qb < pl.first_text_qb) {
        // Textural query blocks made only of video tokens see the compacted key sequence (Eq. 5):
        // as a packed copy made by pack_textural_kernel if the caller gave room for one, else
        // gathered row by row through the index table
        qk.ntiles = pl.nCT;
        qk.keyN = pl.Nc;
        qk.sweep_tag = tag_of(1);
        if (same_sequence() && (seen & kSweepTileMask) < qk.ntiles) qk.first = seen & kSweepTileMask;
        if (a.packed_k) {
            const size_t packed_bytes = head_bytes;
            qk.kbase = reinterpret_cast<const unsigned char*>(a.packed_k) + packed_bytes;
            qk.vbase = reinterpret_cast<const unsigned char*>(a.packed_v) + packed_bytes;
            qk.video_shift = qk.text_shift = 0;
            run(std::integral_constant<int, MODE_ALL>{}, pl, qk);
        } else {
            run(std::integral_constant<int, MODE_COMPACT>{}, pl, qk);
        }
    } else {
        qk.list = list;
        if (temporal_pm) {
            qk.row_token = pl.pm_token;
            qk.kbase = reinterpret_cast<const unsigned char*>(a.packed_k) + head_bytes;
            qk.vbase = reinterpret_cast<const unsigned char*>(a.packed_v) + head_bytes;
            qk.video_shift = qk.text_shift = 0;
        }
        const int e0 = pl.row_ptr[list][qk.qb];
        qk.ntiles = pl.row_ptr[list][qk.qb + 1] - e0;
        qk.cols = pl.cols[list] + e0;
        qk.first = pl.first_entry[list][qk.qb];
        qk.keyN = pl.N;
        qk.sweep_tag = tag_of(temporal_pm ? 2 : 0);
        if (same_sequence() && qk.ntiles > 0) {
            // banded lists are one run of consecutive tiles (then the text tiles): the published tile,
            // if it is in the run, sits at entry (tile - first tile of the run)
            const int tile = seen & kSweepTileMask, at = tile - (qk.cols[0] & kTileIndexMask);
            // if it is not (the others are just outside this block's band, which overlaps theirs almost
            // entirely), the start of the run is where they will be next
            qk.first = (at >= 0 && at < qk.ntiles && (qk.cols[at] & kTileIndexMask) == tile) ? at : 0;
        }
        run(std::integral_constant<int, MODE_LISTED>{}, pl, qk);
    }
}

// Copies of K and V in the order their head walks them, into the caller's workspace: for a
// Textural head the kept keys' rows, then the text rows (K_C, V_C of Eq. 5 made physical); for a
// Temporal head every row, in position-major order.  One workgroup per (64 copied rows, head).
template <int D>
__global__ void __launch_bounds__(256) pack_textural_kernel(AttnArgs a) {
    const DevicePlan& pl = a.plan[0];
    const int bh = blockIdx.y, cls = a.head_class[bh];
    if (cls != RF_TEXTURAL && cls != RF_TEMPORAL) return;
    const int32_t* token_of = cls == RF_TEXTURAL ? pl.cidx : pl.pm_token;
    const int rows = cls == RF_TEXTURAL ? pl.Nc : pl.N;
    constexpr int CH = D / 8;  // 16-byte chunks per row
    const size_t head = static_cast<size_t>(bh) * pl.N * D;
    for (int i = threadIdx.x; i < kTileK * CH; i += 256) {
        const int c = blockIdx.x * kTileK + i / CH, ch = i % CH;
        if (c >= rows) break;
        const size_t src = head + static_cast<size_t>(token_of[c]) * D + 8 * ch;
        const size_t dst = head + static_cast<size_t>(c) * D + 8 * ch;
        *reinterpret_cast<u32x4*>(a.packed_k + dst) = *reinterpret_cast<const u32x4*>(a.K + src);
        *reinterpret_cast<u32x4*>(a.packed_v + dst) = *reinterpret_cast<const u32x4*>(a.V + src);
    }
}

int launch_pack_textural(const AttnArgs& a, int D, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const dim3 grid(a.plan[0].nKT, a.BH);
    if (D == 64) hipLaunchKernelGGL(pack_textural_kernel<64>, grid, dim3(256), 0, st, a);
    else if (D == 96) hipLaunchKernelGGL(pack_textural_kernel<96>, grid, dim3(256), 0, st, a);
    else if (D == 128) hipLaunchKernelGGL(pack_textural_kernel<128>, grid, dim3(256), 0, st, a);
    else return static_cast<int>(hipErrorInvalidValue);
    return static_cast<int>(hipGetLastError());
}

template <int D, int NW, int LOOP = LOOP_32>
static int launch_one(const AttnArgs& a, hipStream_t st) {
    constexpr int NT = 64 * NW;
    constexpr int smem = SmemOf<D, NW, LOOP>::BYTES;
    // workgroups each device holds at once, found on first use there (which also raises the kernel's dynamic-LDS limit)
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static int resident_on[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    int resident = 0;
    {
        std::lock_guard<std::mutex> lock(mu);
        if (resident_on[dev] == 0) {
            const void* fn = reinterpret_cast<const void*>(&attn_kernel<D, NW, LOOP>);
            e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, smem);
            if (e != hipSuccess) return static_cast<int>(e);
            int cus = 0, per_cu = 0;
            if ((e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev)) != hipSuccess) return static_cast<int>(e);
            if ((e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, attn_kernel<D, NW, LOOP>, NT, smem)) != hipSuccess)
                return static_cast<int>(e);
            if (cus < 1 || per_cu < 1) return static_cast<int>(hipErrorInvalidValue);
            resident_on[dev] = cus * per_cu;
        }
        resident = resident_on[dev];
    }
    const long long items = static_cast<long long>(a.plan[0].nQB) * a.BH;
    const int grid = static_cast<int>(std::min<long long>(resident, items));
    hipLaunchKernelGGL(reset_queue_kernel, dim3(1), dim3(64), 0, st, a.queue);
    e = hipGetLastError();
    if (e != hipSuccess) return static_cast<int>(e);
    hipLaunchKernelGGL((attn_kernel<D, NW, LOOP>), dim3(grid), dim3(NT), smem, st, a);
    return static_cast<int>(hipGetLastError());
}

int launch_attention(const AttnArgs& a, int D, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nw = a.plan[0].block / 32;
    if (a.wide_rows) {  // the pipelined loop for 64-row wavefronts: 256-row blocks as four wavefronts, head_dim 128
        if (D == 128 && nw == 8) return launch_one<128, 4, LOOP_64_PIPELINED>(a, st);
        return static_cast<int>(hipErrorInvalidValue);
    }
    if (D == 64 && nw == 2) return launch_one<64, 2>(a, st);
    if (D == 64 && nw == 4) return launch_one<64, 4>(a, st);
    if (D == 96 && nw == 2) return launch_one<96, 2>(a, st);
    if (D == 96 && nw == 4) return launch_one<96, 4>(a, st);
    if (D == 128 && nw == 2) return launch_one<128, 2>(a, st);
    if (D == 128 && nw == 4) return launch_one<128, 4>(a, st);
    // 256-row blocks at head_dim 64: four wavefronts of 64 rows (two still fit a SIMD; measured 8-15 %
    // faster than eight of 32: half the LDS operand reads and half the per-tile bookkeeping per MFMA)
    if (D == 64 && nw == 8) return launch_one<64, 4, LOOP_64>(a, st);
    if (D == 96 && nw == 8) return launch_one<96, 8>(a, st);
    if (D == 128 && nw == 8) return launch_one<128, 8>(a, st);
    // 384-row blocks: twelve wavefronts, three per SIMD at 168 registers (3-7 % faster than eight on 256
    // rows for every class at head_dim 96 and 128; even with the 64-row wavefronts at head_dim 64)
    if (D == 64 && nw == 12) return launch_one<64, 12>(a, st);
    if (D == 96 && nw == 12) return launch_one<96, 12>(a, st);
    if (D == 128 && nw == 12) return launch_one<128, 12>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace rf
