// The tile loop for wavefronts that own 64 query rows (included by rf_attn.hip; gfx950 only).
//
// A wavefront holds two 32-query halves.  Every K slab and every transposed V slab it reads from
// LDS feeds two MFMAs, one per half, so the LDS operand traffic per MFMA is half that of the
// 32-row loop; the price is twice the accumulators, so one wavefront per SIMD (512 registers), and
// with nobody else on the SIMD to fill the gaps, the overlap of matrix and vector work has to come
// from inside the wavefront: the loop is software-pipelined, iteration t issuing the MFMAs of
// O^T += V^T P(t-1)^T and of S(t+1)^T = K(t+1) Q^T with the pieces of the softmax of S(t) dropped
// between them.
#pragma once
#include <type_traits>

namespace rf {

// element e (0 .. 31) of a tile's scores held as two 16-register blocks
#define RF_AT(s, e) s[(e) >> 4][(e) & 15]

template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
    if constexpr (I < N) {
        f(std::integral_constant<int, I>{});
        static_for<I + 1, N>(f);
    }
}

// One lane's query (the transposed score tile puts ONE query in a lane): its running softmax state
// (Eq. 1-2).  The softmax of a tile is cut into kChunks pieces of four to twelve vector instructions
// (chunk()), which the tile loop drops between its MFMAs.
template <int D, int MODE>
struct QueryLane {
    static constexpr int kMaxChunks = 4, kCheckChunk = 4, kExpChunk0 = 5, kExpChunks = 8;
    static constexpr int kChunks = kExpChunk0 + kExpChunks;

    f32x16 oacc[D / 32];
    u32x4 pw[4];  // P of the tile last exponentiated, bf16 pairs, in the operand layout of the second MFMA
    // ref2: reference subtracted inside exp2, in units of the exponent (score * c), always an integer so
    // that moving it rescales by an exact power of two; has_ref: it has been taken from real scores of this
    // row; l_run: this lane's share of the softmax denominator
    float ref2, l_run, c;
    bool has_ref;
    uint32_t q_lo, q_span;  // the band test |attr_q - attr_k| <= r as one unsigned compare: attr_k + q_lo <= q_span
    int hf;
    float mx[4];  // partial maxima of the tile being worked on

    __device__ __forceinline__ void init(float scale_log2, int q_attr, int q_rad, int half) {
#pragma unroll
        for (int db = 0; db < D / 32; ++db) oacc[db] = f32x16{0};
#pragma unroll
        for (int u = 0; u < 4; ++u) pw[u] = u32x4{0, 0, 0, 0};
        ref2 = 0.f;
        l_run = 0.f;
        has_ref = false;
        c = scale_log2;
        q_lo = static_cast<uint32_t>(q_rad - q_attr);
        q_span = 2u * static_cast<uint32_t>(q_rad);
        hf = half;
    }

    // Partial tile: scores of dropped (or non-existent) keys become -inf.  al: the tile's 64 key
    // attributes in LDS (MODE_LISTED).
    __device__ __forceinline__ void mask(int entry, const int* al, int keyN, int Nv, f32x16 (&s)[2]) const {
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (MODE == MODE_LISTED && !(entry & kTileBoundary)) {
            // all 64 keys are video tokens: only the pattern's band decides
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const uint32_t d = static_cast<uint32_t>(al[32 * kb2 + key_of_reg(r, hf)]) + q_lo;
                    s[kb2][r] = d <= q_span ? s[kb2][r] : -INFINITY;
                }
        } else {
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int koff = 32 * kb2 + key_of_reg(r, hf);
                    const int kidx = k0 + koff;
                    bool ok = kidx < keyN;
                    if (MODE == MODE_LISTED) {
                        const uint32_t d = static_cast<uint32_t>(al[koff]) + q_lo;
                        ok = ok & ((d <= q_span) | (kidx >= Nv));
                    }
                    s[kb2][r] = ok ? s[kb2][r] : -INFINITY;
                }
        }
    }

    static __device__ __forceinline__ float max3(float a, float b, float d) { return fmaxf(fmaxf(a, b), d); }

    // Piece I of the online softmax (Eq. 1) of one tile's scores s, in base 2 with 1/sqrt(D) folded
    // into c.  Pieces 0-3 form the row maximum; piece 4 moves the reference if some row has outgrown
    // it by more than 2^kRescaleSlack (or has none yet), rescaling everything accumulated so far (the
    // softmax does not depend on the reference, so it is moved rarely); pieces 5-12 exponentiate four
    // scores each, round P to bf16 for the second MFMA and add it to the denominator.
    template <int I>
    __device__ __forceinline__ void chunk(f32x16 (&s)[2]) {
        // The pieces are pure arithmetic, which the compiler would otherwise gather next to its first
        // use; the empty assembly statements tie each piece's results to its place in the stream.
        if constexpr (I == 0) {
#pragma unroll
            for (int k = 0; k < 4; ++k) mx[k] = max3(RF_AT(s, 3 * k), RF_AT(s, 3 * k + 1), RF_AT(s, 3 * k + 2));
            asm volatile("" : "+v"(mx[0]), "+v"(mx[1]), "+v"(mx[2]), "+v"(mx[3]));
        } else if constexpr (I < 3) {
#pragma unroll
            for (int k = 0; k < 4; ++k) mx[k] = max3(mx[k], RF_AT(s, 12 + 8 * (I - 1) + 2 * k), RF_AT(s, 12 + 8 * (I - 1) + 2 * k + 1));
            asm volatile("" : "+v"(mx[0]), "+v"(mx[1]), "+v"(mx[2]), "+v"(mx[3]));
        } else if constexpr (I == 3) {
            mx[0] = max3(mx[0], RF_AT(s, 28), RF_AT(s, 29));
            mx[1] = max3(mx[1], RF_AT(s, 30), RF_AT(s, 31));
            mx[0] = max3(mx[0], mx[1], fmaxf(mx[2], mx[3]));
            asm volatile("" : "+v"(mx[0]));
        } else if constexpr (I == kCheckChunk) {
            float mt = mx[0];
            // the two halves of the wavefront hold different keys of the same 32 queries: their maxima
            // are exchanged only when some lane asks for the reference to move
            const bool grow = has_ref ? fmaf(mt, c, -ref2) > kRescaleSlack : mt > -INFINITY;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                mt = fmaxf(mt, other_half(mt));
                if (mt > -INFINITY) {
                    const float want = ceilf(mt * c);
                    const float ref_new = has_ref ? fmaxf(ref2, want) : want;
                    // an exact power of two (or 0 while nothing has been accumulated), so the bf16 weights
                    // of the tile whose P V product is still to come can be rescaled without rounding
                    const float alpha = has_ref ? fast_exp2(ref2 - ref_new) : 0.f;
                    l_run *= alpha;
#pragma unroll
                    for (int db = 0; db < D / 32; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
#pragma unroll
                    for (int u = 0; u < 4; ++u)
#pragma unroll
                        for (int w = 0; w < 4; ++w) {
                            const float lo = __builtin_bit_cast(float, pw[u][w] << 16) * alpha;
                            const float hi = __builtin_bit_cast(float, pw[u][w] & 0xffff0000u) * alpha;
                            pw[u][w] = pack_bf16(lo, hi);
                        }
                    ref2 = ref_new;
                    has_ref = true;
                }
            }
        } else {
            // Four scores: exponentiate, round P to bf16 for the second MFMA and add it to the denominator,
            // which sums those same rounded values (two per v_dot2c_f32_bf16), so numerator and denominator
            // of Eq. 2 see identical weights.  The fp32 exponentials go nowhere else: the scores sit in
            // accumulation registers, which vector instructions reach only through copies.
            constexpr int k = I - kExpChunk0, g = k >> 1, h = k & 1;
            float x0 = RF_AT(s, 4 * k), x1 = RF_AT(s, 4 * k + 1), x2 = RF_AT(s, 4 * k + 2), x3 = RF_AT(s, 4 * k + 3);
            asm volatile("" : "+v"(x0), "+v"(x1), "+v"(x2), "+v"(x3));
            x0 = fast_exp2(fmaf(x0, c, -ref2));
            x1 = fast_exp2(fmaf(x1, c, -ref2));
            x2 = fast_exp2(fmaf(x2, c, -ref2));
            x3 = fast_exp2(fmaf(x3, c, -ref2));
            uint32_t w0 = pack_bf16(x0, x1), w1 = pack_bf16(x2, x3);
            l_run = add_bf16_pair(add_bf16_pair(l_run, w0), w1);
            asm volatile("" : "+v"(w0), "+v"(w1), "+v"(l_run));
            pw[g][2 * h] = w0;
            pw[g][2 * h + 1] = w1;
        }
    }

    // Eq. 2: divide by the softmax denominator and store.  Lane (hf, m) owns query m and, per
    // 32-channel block, channels 8*(r/4) + 4*hf + r%4.
    __device__ __forceinline__ void store(uint16_t* orow) const {
        const float l_tot = l_run + other_half(l_run);
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        if (!orow) return;
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int rq = 0; rq < 4; ++rq) {
                u32x2 w;
                w.x = pack_bf16(oacc[db][4 * rq + 0] * inv, oacc[db][4 * rq + 1] * inv);
                w.y = pack_bf16(oacc[db][4 * rq + 2] * inv, oacc[db][4 * rq + 3] * inv);
                *reinterpret_cast<u32x2*>(orow + 32 * db + 8 * rq + 4 * hf) = w;
            }
    }
};
// The walk of one query block over its key tiles: which tile comes t-th, where its rows are, and the
// per-key side data (token indices of a compacted tile, or the pattern attribute of each key).
template <int D, int NW, int MODE>
struct TileWalk {
    using ST = DirectTile<D, NW>;
    const QueryBlock& qk;
    const int32_t* side_src;
    int Nv, lane, tid;
    // Tile entries of a listed query block are read 64 at a time, one per lane, and handed out with
    // v_readlane: no scalar-load latency in the loop.  ent_cur covers [ent_base, ent_base + 64).
    int ent_cur = 0, ent_nxt = 0, ent_base = 0;
    int side_reg = 0;

    __device__ __forceinline__ TileWalk(const QueryBlock& q, const DevicePlan& pl, int tid_)
        : qk(q), side_src(MODE == MODE_COMPACT ? pl.cidx : (MODE == MODE_LISTED ? pl.attr[q.list] : nullptr)), Nv(pl.Nv),
          lane(tid_ & 63), tid(tid_) {
        if (MODE == MODE_LISTED && qk.ntiles > 0) {
            ent_cur = load_entries(0);
            ent_nxt = load_entries(64);
        }
    }
    __device__ __forceinline__ int load_entries(int from) const {
        const int j = min(from + lane, qk.ntiles - 1) + qk.first;  // the walk starts at entry qk.first and wraps
        return qk.cols[j < qk.ntiles ? j : j - qk.ntiles];
    }
    // entries must be asked for in increasing t
    __device__ __forceinline__ int entry_of(int t) {
        if (MODE == MODE_LISTED) {
            if (t >= ent_base + 64) {
                ent_base += 64;
                ent_cur = ent_nxt;
                ent_nxt = load_entries(ent_base + 64);
            }
            return __builtin_amdgcn_readlane(ent_cur, t - ent_base);
        }
        int tile = t + qk.first;  // the walk starts at tile qk.first and wraps
        if (tile >= qk.ntiles) tile -= qk.ntiles;
        return tile | ((tile + 1) * kTileK > qk.keyN ? (RF_PLAN_PARTIAL | kTileBoundary) : 0);
    }
    // side data is needed for every tile of the compacted sequence, and for partial listed tiles
    static __device__ __forceinline__ bool wants_side(int entry) {
        return MODE == MODE_COMPACT || (MODE == MODE_LISTED && (entry & RF_PLAN_PARTIAL));
    }
    __device__ __forceinline__ void load_side(int entry) {
        if (!wants_side(entry)) return;
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (tid < kTileK) side_reg = side_src[min(k0 + tid, qk.keyN - 1)];
    }
    __device__ __forceinline__ void stash_side(int entry, int* slot) const {
        if (!wants_side(entry)) return;
        if (tid < kTileK) slot[tid] = side_reg;
    }
    // Issues the loads of the tile of `entry` into kl / vl; idx: the tile's side slot (MODE_COMPACT).
    template <bool WITH_K, bool WITH_V>
    __device__ __forceinline__ void fetch(ST& st, int entry, const int* idx, unsigned char* kl, unsigned char* vl) const {
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (MODE == MODE_COMPACT) {
            st.template issue<WITH_V, WITH_K>(qk.kbase, qk.vbase, kl, vl, [&](int row) { return idx[row]; });
        } else if (k0 + kTileK <= qk.keyN && !(qk.text_shift != 0 && k0 < Nv && k0 + kTileK > Nv)) {
            // full tile of consecutive tensor rows: everything but the tile origin is loop invariant
            const int r0 = k0 + (k0 < Nv ? qk.video_shift : qk.text_shift);
            const size_t origin = static_cast<size_t>(r0) * (2 * D);
            st.template issue_consecutive<WITH_V, WITH_K>(qk.kbase + origin, qk.vbase + origin, kl, vl);
        } else {
            st.template issue<WITH_V, WITH_K>(qk.kbase, qk.vbase, kl, vl, [&](int row) {
                const int n = min(k0 + row, qk.keyN - 1);
                return n + (n < Nv ? qk.video_shift : qk.text_shift);
            });
        }
    }
};


// LDS layout of the 64-row loop: rings of K tiles and V tiles (those being read and those on their
// way) and a ring of per-key side data.  Iteration t reads K(t+1) and V(t-1) and issues the loads of
// K(t+K_AHEAD) and V(t+V_AHEAD); one workgroup per CU, so the rings can be deep.
template <int D, int NW>
struct WideSmem {
    using ST = DirectTile<D, NW>;
    static constexpr int K_AHEAD = 3, V_AHEAD = 1;
    static constexpr int K_RING = K_AHEAD, V_RING = V_AHEAD + 2;  // the slot of K(t+K_AHEAD) held K(t), that of V(t+V_AHEAD) held V(t-2)
    // side data of tile u is written at the end of iteration u-SIDE_AHEAD (before K(u) is loaded in
    // iteration u-K_AHEAD) and last read in iteration u
    static constexpr int SIDE_AHEAD = K_AHEAD + 1, SIDE_SLOTS = 8;
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = K_RING * ST::K_BYTES;
    static constexpr int SIDE_OFF = V_OFF + V_RING * ST::V_BYTES;
    static constexpr int ITEM_OFF = SIDE_OFF + SIDE_SLOTS * kTileK * 4;  // the work item just taken
    static constexpr int BYTES = ITEM_OFF + 16;
    static_assert(K_OFF % 256 == 0 && V_OFF % 256 == 0 && ST::K_BYTES % 256 == 0 && ST::V_BYTES % 256 == 0,
                  "tile buffers must start at multiples of 256 bytes (see DirectTile::k_address)");
    static_assert(SIDE_SLOTS > SIDE_AHEAD, "a side slot is rewritten only after every wavefront has left the iteration that read it");
};

// softmax pieces (of 2 * QueryLane::kChunks per iteration) after which an iteration issues its V and its K loads
#ifndef RF_WIDE_V_LOAD_AT
#define RF_WIDE_V_LOAD_AT 8
#endif
#ifndef RF_WIDE_K_LOAD_AT
#define RF_WIDE_K_LOAD_AT 20
#endif
#ifndef RF_WIDE_PRE
#define RF_WIDE_PRE 3
#endif

// Half h of this lane's queries: tensor row, Q operand, band test; returns the row of O (null past the end).
template <int D, int NW, int MODE>
__device__ __forceinline__ uint16_t* load_query_half(const AttnArgs& a, const DevicePlan& pl, const QueryBlock& qk,
                                                     const int32_t* side_src, int wave, int h, int m, int hf, bf16x8 (&qf)[D / 16],
                                                     QueryLane<D, MODE>& ql) {
    constexpr int BQ = 64 * NW;
    const int N = pl.N, Nv = pl.Nv;
    const uint16_t* Qh = a.Q + static_cast<size_t>(qk.bh) * N * D;
    const int qrow = qk.qb * BQ + wave * 64 + 32 * h + m;  // row of the walked order
    const int qrow_c = min(qrow, N - 1);
    const int qtok = (MODE == MODE_LISTED && qk.row_token) ? qk.row_token[qrow_c]
                                                           : qrow_c + (qrow_c < Nv ? pl.video_shift : pl.text_shift);
    load_q_frags<D>(Qh, qtok, hf, qf);
    int q_attr = 0, q_rad = 0x3fffffff;  // text queries keep everything
    if (MODE == MODE_LISTED) {
        // Spatial / Temporal compare the query's frame / position with the key's; the Textural
        // table is 0 on kept keys and 1 on dropped ones, compared against 0 with radius 0
        if (qk.cls != RF_TEXTURAL) q_attr = side_src[qrow_c];
        if (qrow_c < Nv) q_rad = pl.radius[qk.list];
    }
    ql.init(a.scale_log2, q_attr, q_rad, hf);
    return qrow < N ? a.O + static_cast<size_t>(qk.bh) * N * D + static_cast<size_t>(qtok) * D : nullptr;
}

// The tile loop of one query block of 64 * NW rows.
//
// Iteration t, as one instruction stream: per V slab of tile t-1 two MFMAs (one per half) of
// O^T += V^T P^T, then per K slab of tile t+1 two MFMAs of S^T = K Q^T, with the pieces of the softmax
// of S(t), alternating between the halves, dropped between them, and with the loads of K(t+K_AHEAD)
// and V(t+V_AHEAD) issued from two points inside the stream.  Then the loads that the next iteration
// reads are awaited and a barrier publishes them.  Scores live in two register sets that swap roles
// from one iteration to the next (the loop is unrolled by two for that).
template <int D, int NW, int MODE>
__device__ __forceinline__ void attend_wide(const AttnArgs& a, const DevicePlan& pl, const QueryBlock& qk, unsigned char* smem) {
    using ST = DirectTile<D, NW>;
    using SM = WideSmem<D, NW>;
    using QL = QueryLane<D, MODE>;
    constexpr int KA = SM::K_AHEAD, VA = SM::V_AHEAD, SA = SM::SIDE_AHEAD;
    constexpr int NPV = 4 * (D / 32), NDB = D / 32, NQK = 2 * (D / 16);
    constexpr int PRE = RF_WIDE_PRE;  // operand reads run this many slabs ahead of their use
    constexpr int V_LOAD_AT = RF_WIDE_V_LOAD_AT, K_LOAD_AT = RF_WIDE_K_LOAD_AT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;
    const int ntiles = qk.ntiles;
    int* side = reinterpret_cast<int*>(smem + SM::SIDE_OFF);

    TileWalk<D, NW, MODE> walk(qk, pl, tid);
    bf16x8 qf[2][D / 16];
    QL ql[2];
    uint16_t* orow[2];
#pragma unroll
    for (int h = 0; h < 2; ++h) orow[h] = load_query_half<D, NW, MODE>(a, pl, qk, walk.side_src, wave, h, m, hf, qf[h], ql[h]);

    ST st;
    st.init(tid);
    const int loads_per_tensor = st.loads_per_tensor();
    static_assert(2 * ST::PER_WAVE <= 8, "wait_all_but() knows counts up to 8");
    auto k_lds = [&](int t) { return smem + SM::K_OFF + (t % SM::K_RING) * ST::K_BYTES; };
    auto v_lds = [&](int t) { return smem + SM::V_OFF + (t % SM::V_RING) * ST::V_BYTES; };
    auto side_slot = [&](int t) { return side + (t % SM::SIDE_SLOTS) * kTileK; };

    // e[i] = entry of tile t+i
    int e[SA + 1] = {};

    // The MFMAs of one iteration as one operand stream: first the V slabs of tile t-1 (if WITH_PV), then
    // the K slabs of tile t+1 (scores into s_out); slab f is read from LDS PRE slabs before its use and
    // feeds MFMAs 2f (half 0) and 2f+1 (half 1).  Before softmax piece i, ceil((i + 1) * NM / pieces)
    // of the NM MFMAs have been issued.
    auto pipelined = [&](auto with_pv, int t, f32x16 (&s_in)[2][2], f32x16 (&s_out)[2][2]) {
        constexpr bool PV = decltype(with_pv)::value;
        constexpr int NA = PV ? NPV : 0, NF = NA + NQK, NM = 2 * NF, NCH = 2 * QL::kChunks;
        const uint32_t va = PV ? st.v_address(v_lds(t - 1)) : 0, ka = st.k_address(k_lds(t + 1));
        bf16x8 frag[NF];
        auto operand = [&](auto fc) {
            constexpr int f = decltype(fc)::value;
            if constexpr (f < NA) frag[f] = ST::v_frag(va, f % NDB, f / NDB);
            else frag[f] = st.k_frag(ka, (f - NA) & 1, (f - NA) >> 1);
        };
        auto mfma = [&](auto jc) {
            constexpr int j = decltype(jc)::value, f = j >> 1, h = j & 1;
            if constexpr (h == 0 && f + PRE < NF) operand(std::integral_constant<int, f + PRE>{});
            if constexpr (f < NA) {
                ql[h].oacc[f % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f], as_bf16x8(ql[h].pw[f / NDB]), ql[h].oacc[f % NDB], 0, 0, 0);
            } else {
                constexpr int i = f - NA;
                s_out[h][i & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[f], qf[h][i >> 1], i < 2 ? f32x16{0} : s_out[h][i & 1], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        static_for<0, (PRE < NF ? PRE : NF)>(operand);
        static_for<0, NCH>([&](auto ic) {
            constexpr int i = decltype(ic)::value;
            constexpr int lo = (i * NM + NCH - 1) / NCH, hi = ((i + 1) * NM + NCH - 1) / NCH;
            static_for<lo, hi>(mfma);
            ql[i & 1].template chunk<(i >> 1)>(s_in[i & 1]);
            if constexpr (i == V_LOAD_AT) {
                if (t + VA < ntiles) walk.template fetch<false, true>(st, e[VA], side_slot(t + VA), nullptr, v_lds(t + VA));
            }
            if constexpr (i == K_LOAD_AT) {
                if (t + KA < ntiles) walk.template fetch<true, false>(st, e[KA], side_slot(t + KA), k_lds(t + KA), nullptr);
            }
            __builtin_amdgcn_sched_barrier(0);
        });
    };

#pragma unroll
    for (int i = 0; i <= SA; ++i)
        if (i < ntiles) e[i] = walk.entry_of(i);
    // side data of the first SA tiles goes straight to its slots
#pragma unroll
    for (int i = 0; i < SA; ++i)
        if (i < ntiles) {
            walk.load_side(e[i]);
            walk.stash_side(e[i], side_slot(i));
        }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < KA; ++i)
        if (i < ntiles) walk.template fetch<true, false>(st, e[i], side_slot(i), k_lds(i), nullptr);
#pragma unroll
    for (int i = 0; i < VA; ++i)
        if (i < ntiles) walk.template fetch<false, true>(st, e[i], side_slot(i), nullptr, v_lds(i));
    ST::template wait_landed<0>();
    __syncthreads();
    // The compiler cannot see the tile loads, so its own wait for the Q loads, if left inside the
    // loop, would count them out too and wait for the tiles in flight; make it wait here.
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int cc = 0; cc < D / 16; ++cc) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, qf[h][cc])));

    f32x16 sa[2][2], sb[2][2];
    if (ntiles > 0) {
        const uint32_t ka0 = st.k_address(k_lds(0));
#pragma unroll
        for (int h = 0; h < 2; ++h) st.template scores<kAheadK>(ka0, qf[h], sa[h]);
    }

    // One iteration (see above).  In the last one the scores of the tile after the last are formed from
    // whatever its buffer holds and never used.
    auto iteration = [&](int t, auto with_pv, f32x16 (&s_in)[2][2], f32x16 (&s_out)[2][2]) {
        if (t + SA < ntiles) walk.load_side(e[SA]);
        // every eighth tile, tell the workgroups that start an item on this XCD where this walk is
        if (qk.sweep && (t & 7) == 0 && tid == 0)
            __hip_atomic_store(qk.sweep, (qk.sweep_tag << kSweepTileBits) | (e[0] & kSweepTileMask), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (e[0] & RF_PLAN_PARTIAL) {
#pragma unroll
            for (int h = 0; h < 2; ++h) ql[h].mask(e[0], side_slot(t), qk.keyN, pl.Nv, s_in[h]);
        }
        pipelined(with_pv, t, s_in, s_out);
        // K(t+2) and V(t) must have landed; those are loads of the iteration before, so this iteration's
        // own (counted exactly: fewer near the end of the walk) may stay in flight
        ST::wait_all_but(((t + KA < ntiles) + (t + VA < ntiles)) * loads_per_tensor);
        if (t + SA < ntiles) walk.stash_side(e[SA], side_slot(t + SA));
#pragma unroll
        for (int i = 0; i < SA; ++i) e[i] = e[i + 1];
        if (t + SA + 1 < ntiles) e[SA] = walk.entry_of(t + SA + 1);
        __syncthreads();
    };
    if (ntiles > 0) {
        iteration(0, std::false_type{}, sa, sb);
        int t = 1;
        for (; t + 1 < ntiles; t += 2) {
            iteration(t, std::true_type{}, sb, sa);
            iteration(t + 1, std::true_type{}, sa, sb);
        }
        if (t < ntiles) iteration(t, std::true_type{}, sb, sa);
        // P V of the last tile
        const uint32_t va = st.v_address(v_lds(ntiles - 1));
        bf16x8 frag[NPV];
#pragma unroll
        for (int i = 0; i < kAheadV; ++i) frag[i] = ST::v_frag(va, i % NDB, i / NDB);
#pragma unroll
        for (int j = 0; j < NPV; ++j) {
            if (j + kAheadV < NPV) frag[j + kAheadV] = ST::v_frag(va, (j + kAheadV) % NDB, (j + kAheadV) / NDB);
#pragma unroll
            for (int h = 0; h < 2; ++h)
                ql[h].oacc[j % NDB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[j], as_bf16x8(ql[h].pw[j / NDB]), ql[h].oacc[j % NDB], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        // the workgroup's next use of these V buffers comes after the barriers of the item hand-out
    }
#pragma unroll
    for (int h = 0; h < 2; ++h) ql[h].store(orow[h]);
}

}  // namespace rf
