// Block-sparse attention forward for RainFusion's head patterns (Eq. 1-5; Fig. 2a), gfx950.
//
// One workgroup = one query block (64 or 128 rows) of one head.  It reads the head's class on
// the device, walks that class's list of 64-key tiles (skipped tiles cost no traffic), stages K
// and V^T tiles through LDS with one tile of prefetch held in registers, forms the transposed
// score tile with bf16 MFMA, runs the online softmax in fp32 with exp2, and accumulates
// O^T = V^T P^T with bf16 MFMA.  In tiles flagged partial the token-level predicate of the
// pattern is re-applied to each score.
#include "rf_device.h"

namespace rf {

// How a query block finds its key tiles.
enum : int {
    MODE_ALL = 0,      // every key tile of the sequence in order (dense heads)
    MODE_COMPACT = 1,  // every tile of the compacted key sequence; rows go through the index table (Eq. 5)
    MODE_LISTED = 2    // the CSR list of the head's pattern; partial tiles re-apply the predicate
};

// Two ways of getting a 64-key tile of K and V from global memory into LDS and of reading
// MFMA operands back out.  Both expose: init(), issue(), commit(), k_frag(), v_frag().

typedef short s16x4 __attribute__((ext_vector_type(4)));

// (1) DirectTile, head_dim 64 and 128: global_load_lds writes the tile straight into LDS (no
// staging registers).  A wavefront instruction fills 1 KiB of consecutive LDS, lane l bytes
// 16*l .. 16*l+15, so rows are unpadded; bank conflicts are avoided by permuting, per row, which
// 16-byte chunk of the row a slot holds (slot position = chunk ^ X(row)), which costs nothing
// because every lane chooses its own global address.  K is read back 16 bytes per lane as the A
// operand of S^T = K Q^T; V stays row-major [key][channel] and ds_read_b64_tr_b16 transposes it
// on the way out into the A operand of O^T = V^T P^T (8 consecutive keys of one channel per lane).
template <int D, int NW>
struct DirectTile {
    static_assert(D == 64 || D == 128, "row length must be a power of two number of 16-byte chunks");
    static constexpr int NT = 64 * NW, CH = D / 8, ROW = 2 * D;
    static constexpr int K_BYTES = kTileK * ROW, V_BYTES = kTileK * ROW;
    static constexpr int SEGS = kTileK * CH / 64;  // 1 KiB segments per tile
    static constexpr int V_READS_PER_FRAG = 2;
    static constexpr int PER_WAVE = SEGS / NW;     // load instructions per tensor per thread

    // chunk permutation of a row: K spreads the 16 rows a read phase touches over all banks,
    // V spreads the 4 rows a transposing read phase touches over the four 64-byte bank groups
    static __device__ __forceinline__ int xk(int row) { return D == 128 ? (row & 15) : ((row >> 1) & 7); }
    static __device__ __forceinline__ int xv(int row) { return D == 128 ? 4 * (row & 3) : 4 * ((row >> 1) & 1); }

    static __device__ __forceinline__ uint32_t lds_offset(const unsigned char* p) {
        return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const unsigned char*)p));
    }
    // One 16-byte-per-lane load from  base + lane offset  into LDS at  lds_addr + 16*lane; completion
    // is awaited in commit().
    static __device__ __forceinline__ void dma16(const unsigned char* base, uint32_t lane_off, uint32_t lds_addr) {
        __builtin_amdgcn_global_load_lds(base + lane_off, (__attribute__((address_space(3))) void*)(uintptr_t)lds_addr, 16,
                                         0, 0);
    }

    int wave, lane;
    int k_base;          // byte offset of this lane's K operand for kb2 = 0, c = 0
    int v_base[D / 32];  // byte offset of this lane's V operand for u = 0, first half, per channel block
    static constexpr int ROWS_PER_LOAD = 64 * NW / CH;  // tile rows between a thread's successive loads
    // X(row) has period 16 for K and 4 for V, so V's lane offset never depends on the load index j
    // and K's only when a load covers fewer than 16 rows
    static constexpr int K_VARIANTS = (ROWS_PER_LOAD % 16 == 0) ? 1 : PER_WAVE;
    static_assert(ROWS_PER_LOAD % 4 == 0, "V row permutation must not change between loads");
    uint32_t k_lane_off[K_VARIANTS], v_lane_off;  // global byte offsets of this lane's slot within a load

    __device__ __forceinline__ void init(int tid) {
        lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int hf = lane >> 5, m = lane & 31, g4 = lane >> 4, i = lane & 15;
        const int krow = key_of_mfma_row(m);
        k_base = krow * ROW + 16 * (hf ^ xk(krow));
        {
            // slot of load j: tile row  j*ROWS_PER_LOAD + row0, position pos; X(row) is the same for all j
            const int slot = wave * 64 + lane, row0 = slot / CH, pos = slot % CH;
#pragma unroll
            for (int j = 0; j < K_VARIANTS; ++j) k_lane_off[j] = row0 * ROW + 16 * (pos ^ xk(row0 + j * ROWS_PER_LOAD));
            v_lane_off = row0 * ROW + 16 * (pos ^ xv(row0));
        }
        const int vrow = 8 * hf + (i >> 2);  // + 16*u + 4*half: multiples of 4, invisible to xv()
#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
            const int chunk = 4 * db + 2 * (g4 & 1) + ((i & 3) >> 1);
            v_base[db] = vrow * ROW + 16 * (chunk ^ xv(vrow)) + 8 * (i & 1);
        }
    }

    // tok(row): token whose K/V row goes to tile row `row`; kh/vh: byte pointers the tokens index
    template <typename F>
    __device__ __forceinline__ void issue(const unsigned char* kh, const unsigned char* vh, unsigned char* kl,
                                          unsigned char* vl, F tok) {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int seg = j * NW + wave;
            const int slot = seg * 64 + lane, row = slot / CH, pos = slot % CH;
            const uint32_t row_off = static_cast<uint32_t>(tok(row)) * ROW;
            const uint32_t k_off = row_off + 16u * (pos ^ xk(row)), v_off = row_off + 16u * (pos ^ xv(row));
            dma16(kh, k_off, lds_offset(kl) + seg * 1024);
            dma16(vh, v_off, lds_offset(vl) + seg * 1024);
        }
    }
    // same for a tile of 64 consecutive tokens starting at kh / vh: only uniform bases move
    __device__ __forceinline__ void issue_consecutive(const unsigned char* kh, const unsigned char* vh, unsigned char* kl,
                                                      unsigned char* vl) {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int seg = j * NW + wave;
            dma16(kh + j * ROWS_PER_LOAD * ROW, k_lane_off[j % K_VARIANTS], lds_offset(kl) + seg * 1024);
            dma16(vh + j * ROWS_PER_LOAD * ROW, v_lane_off, lds_offset(vl) + seg * 1024);
        }
    }
    // the tile is in LDS once this thread's loads have landed (the barrier that follows publishes it)
    __device__ __forceinline__ void commit(unsigned char*, unsigned char*) { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

    __device__ __forceinline__ bf16x8 k_frag(const unsigned char* kl, int kb2, int c) const {
        return as_bf16x8(*reinterpret_cast<const u32x4*>(kl + ((k_base ^ (32 * c)) + kb2 * 32 * ROW)));
    }
    __device__ __forceinline__ bf16x8 v_frag(const unsigned char* vl, int db, int u) const {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const unsigned char* p = vl + v_base[db] + 16 * u * ROW;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(p + 4 * ROW));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
};

// (2) StagedTile, any head_dim (used for 96): global -> registers -> LDS.  K rows are padded by
// 16 bytes; V is transposed in registers and stored one LDS row per channel.  A thread owns
// "units": unit (kg, dc) covers keys 8*kg .. 8*kg+7; from V it loads channels 4*dc .. 4*dc+3 of
// those rows (8 bytes each), from K four of the same rows, 16 bytes each.
template <int D, int NW>
struct StagedTile {
    static constexpr int NT = 64 * NW;
    static constexpr int K_ROW = 2 * D + 16;       // bytes; +16 pad: conflict-free 16-B reads down a column
    static constexpr int V_ROW = 2 * kTileK + 16;  // bytes
    static constexpr int K_BYTES = kTileK * K_ROW;
    static constexpr int V_BYTES = D * V_ROW;
    static constexpr int DC = D / 4;               // units per key group
    static constexpr int V_READS_PER_FRAG = 1;
    static constexpr int UNITS = (kTileK / 8) * DC;
    static constexpr int PER_THREAD = (UNITS + NT - 1) / NT;
    static constexpr bool EXACT = UNITS % NT == 0;

    int tid, hf, m;
    u32x4 kreg[PER_THREAD][4];
    u32x2 vreg[PER_THREAD][8];

    __device__ __forceinline__ void init(int t) {
        tid = t;
        hf = (t & 63) >> 5;
        m = t & 31;
    }
    static __device__ __forceinline__ int k_row_in_group(int dc) { return 4 * (dc / (D / 8)); }
    static __device__ __forceinline__ int k_chunk(int dc) { return dc % (D / 8); }

    template <typename F>
    __device__ __forceinline__ void issue(const unsigned char* kh, const unsigned char* vh, unsigned char*,
                                          unsigned char*, F tok) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (EXACT || u < UNITS) {
                const int kg = u / DC, dc = u % DC;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const uint32_t row_off = static_cast<uint32_t>(tok(8 * kg + e)) * (2u * D);
                    vreg[i][e] = *reinterpret_cast<const u32x2*>(vh + row_off + 8u * dc);
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const uint32_t row_off = static_cast<uint32_t>(tok(8 * kg + k_row_in_group(dc) + j)) * (2u * D);
                    kreg[i][j] = *reinterpret_cast<const u32x4*>(kh + row_off + 16u * k_chunk(dc));
                }
            }
        }
    }

    __device__ __forceinline__ void issue_consecutive(const unsigned char* kh, const unsigned char* vh, unsigned char* kl,
                                                      unsigned char* vl) {
        issue(kh, vh, kl, vl, [](int row) { return row; });
    }

    __device__ __forceinline__ void commit(unsigned char* kl, unsigned char* vl) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (EXACT || u < UNITS) {
                const int kg = u / DC, dc = u % DC;
                const int r0 = 8 * kg + k_row_in_group(dc);
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    *reinterpret_cast<u32x4*>(kl + (r0 + j) * K_ROW + 16 * k_chunk(dc)) = kreg[i][j];
                uint32_t o[4][4];  // [channel][key pair]
#pragma unroll
                for (int w = 0; w < 4; ++w) {  // keys 2w, 2w+1 side by side, one channel per output row
                    const u32x2 a = vreg[i][2 * w], b = vreg[i][2 * w + 1];
                    o[0][w] = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u);
                    o[1][w] = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
                    o[2][w] = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u);
                    o[3][w] = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
                }
                // 16-byte key chunk kg of channel row d sits at chunk position kg ^ ((d >> 4) & 3):
                // with the 36-dword row pitch this spreads the 16 lanes of a write phase over all banks
                const int pos = kg ^ ((dc >> 2) & 3);
#pragma unroll
                for (int dd = 0; dd < 4; ++dd)
                    *reinterpret_cast<u32x4*>(vl + (4 * dc + dd) * V_ROW + 16 * pos) =
                        u32x4{o[dd][0], o[dd][1], o[dd][2], o[dd][3]};
            }
        }
    }

    // A operand of S^T = K Q^T: keys 32*kb2 .. +31 (permuted per lane), channels 16*c + 8*hf .. +7
    __device__ __forceinline__ bf16x8 k_frag(const unsigned char* kl, int kb2, int c) const {
        const int row = 32 * kb2 + key_of_mfma_row(m);
        return as_bf16x8(*reinterpret_cast<const u32x4*>(kl + row * K_ROW + 32 * c + 16 * hf));
    }
    // A operand of O^T = V^T P^T: channels 32*db + m, keys 16*u + 8*hf .. +7
    __device__ __forceinline__ bf16x8 v_frag(const unsigned char* vl, int db, int u) const {
        const int row = 32 * db + m;
        const int pos = (2 * u + hf) ^ ((row >> 4) & 3);
        return as_bf16x8(*reinterpret_cast<const u32x4*>(vl + row * V_ROW + 16 * pos));
    }
};

template <int D, int NW>
struct TileFor {
    using type = StagedTile<D, NW>;
};
template <int NW>
struct TileFor<64, NW> {
    using type = DirectTile<64, NW>;
};
template <int NW>
struct TileFor<128, NW> {
    using type = DirectTile<128, NW>;
};

template <int D, int NW>
struct AttnSmem {
    using ST = typename TileFor<D, NW>::type;
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = 2 * ST::K_BYTES;
    static constexpr int SIDE_OFF = V_OFF + 2 * ST::V_BYTES;  // ring of 3 x 64 ints: key indices or key attributes
    static constexpr int BYTES = SIDE_OFF + 3 * kTileK * 4;
};

struct QueryBlock {
    int bh, qb, cls;
    const int32_t* cols;  // MODE_LISTED: this query block's tile entries
    int ntiles;           // key tiles to visit
    int keyN;             // length of the key sequence walked (N, or Nc when compacted)
};

// exp2 arguments may exceed 0 by at most this much before the running reference is moved: the
// softmax is invariant to the reference, so a stale one only costs range, which fp32/bf16 have.
constexpr float kRescaleSlack = 8.f;

template <int D, int NW, int MODE>
__device__ __forceinline__ void attend(const AttnArgs& a, const QueryBlock& qk, unsigned char* smem) {
    constexpr int BQ = 32 * NW;
    using ST = typename TileFor<D, NW>::type;
    using SM = AttnSmem<D, NW>;
    const DevicePlan& pl = a.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;
    const int N = pl.N, Nv = pl.Nv, keyN = qk.keyN, ntiles = qk.ntiles;
    // per-key side data staged through LDS two tiles ahead: the token index of each key of the
    // compacted sequence, or the pattern attribute (frame / position / kept flag) of each key
    const int32_t* side_src = MODE == MODE_COMPACT ? pl.cidx : (MODE == MODE_LISTED ? pl.attr[qk.cls] : nullptr);
    int* side = reinterpret_cast<int*>(smem + SM::SIDE_OFF);

    const size_t head_bytes = static_cast<size_t>(qk.bh) * N * D * 2;
    const unsigned char* Kh = reinterpret_cast<const unsigned char*>(a.K) + head_bytes;
    const unsigned char* Vh = reinterpret_cast<const unsigned char*>(a.V) + head_bytes;
    const uint16_t* Qh = a.Q + static_cast<size_t>(qk.bh) * N * D;

    // this lane's query
    const int qrow = qk.qb * BQ + wave * 32 + m;
    const int qtok = min(qrow, N - 1);
    bf16x8 qf[D / 16];
    load_q_frags<D>(Qh, qtok, hf, qf);
    int q_attr = 0, q_rad = 0x3fffffff;  // text queries keep everything
    if (MODE == MODE_LISTED) {
        // Spatial / Temporal compare the query's frame / position with the key's; the Textural
        // table is 0 on kept keys and 1 on dropped ones, compared against 0 with radius 0
        if (qk.cls != RF_TEXTURAL) q_attr = side_src[qtok];
        if (qtok < Nv) q_rad = pl.radius[qk.cls];
    }
    const uint32_t q_lo = static_cast<uint32_t>(q_rad - q_attr), q_span = 2u * static_cast<uint32_t>(q_rad);

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) oacc[db] = f32x16{0};
    // m_ref: reference subtracted inside exp2 (raw score units), finite from the start; has_ref: it has
    // been taken from real scores of this row; l_run: this lane's share of the softmax denominator
    float m_ref = 0.f, l_run = 0.f;
    bool has_ref = false;
    const float c = a.scale_log2;

    ST st;
    st.init(tid);
    int side_reg = 0;

    // Tile entries of a listed query block are read 64 at a time, one per lane, and handed out with
    // v_readlane: no scalar-load latency in the loop.  ent_cur covers [ent_base, ent_base + 64).
    int ent_cur = 0, ent_nxt = 0, ent_base = 0;
    auto load_entries = [&](int first) { return qk.cols[min(first + lane, ntiles - 1)]; };
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
        return t | ((t + 1) * kTileK > keyN ? (RF_PLAN_PARTIAL | kTileBoundary) : 0);
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
        if (tid < kTileK) side[(t % 3) * kTileK + tid] = side_reg;
    };
    auto k_lds = [&](int t) { return smem + SM::K_OFF + (t & 1) * ST::K_BYTES; };
    auto v_lds = [&](int t) { return smem + SM::V_OFF + (t & 1) * ST::V_BYTES; };
    auto fetch_tile = [&](int t, int entry) {
        const int k0 = (entry & kTileIndexMask) * kTileK;
        if (MODE == MODE_COMPACT) {
            const int* idx = side + (t % 3) * kTileK;
            st.issue(Kh, Vh, k_lds(t), v_lds(t), [&](int row) { return idx[row]; });
        } else if (k0 + kTileK <= keyN) {
            // full tile: rows are consecutive tokens, everything but the tile origin is loop invariant
            const size_t origin = static_cast<size_t>(k0) * (2 * D);
            st.issue_consecutive(Kh + origin, Vh + origin, k_lds(t), v_lds(t));
        } else {
            st.issue(Kh, Vh, k_lds(t), v_lds(t), [&](int row) { return min(k0 + row, keyN - 1); });
        }
    };
    auto stash_tile = [&](int t) { st.commit(k_lds(t), v_lds(t)); };

    // S^T of tile t (64 keys x this lane's query), predicate applied where the tile is partial
    auto scores = [&](int t, int entry, f32x16 (&s)[2]) {
        const unsigned char* kl = k_lds(t);
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            f32x16 acc = {0};
#pragma unroll
            for (int cc = 0; cc < D / 16; ++cc)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(st.k_frag(kl, kb2, cc), qf[cc], acc, 0, 0, 0);
            s[kb2] = acc;
        }
#ifdef RF_SCHED_QK
        // keep RF_SCHED_QK operand reads in flight ahead of the MFMA that consumes them
        __builtin_amdgcn_sched_group_barrier(0x100, RF_SCHED_QK, 0);
#pragma unroll
        for (int i = 0; i < 2 * (D / 16) - RF_SCHED_QK; ++i) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, RF_SCHED_QK, 0);
#endif
        if (entry & RF_PLAN_PARTIAL) {
            const int k0 = (entry & kTileIndexMask) * kTileK;
            const int* al = side + (t % 3) * kTileK;
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
    };
    // p = exp2((s - m_ref) * c) in place; returns this lane's sum
    auto exponentiate = [&](f32x16 (&s)[2]) {
        const float mc = m_ref * c;
        float sum = 0.f;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[kb2][r] = fast_exp2(fmaf(s[kb2][r], c, -mc));
                sum += s[kb2][r];
            }
        return sum;
    };

    // software pipeline: side data runs two tiles ahead of the compute, K/V one tile ahead
    int e_cur = 0, e_nxt = 0, e_nx2 = 0;
    if (ntiles > 0) {
        e_cur = entry_of(0);
        if (ntiles > 1) e_nxt = entry_of(1);
        load_side(e_cur);
        stash_side(0, e_cur);
        if (ntiles > 1) {
            load_side(e_nxt);
            stash_side(1, e_nxt);
        }
    }
    __syncthreads();
    if (ntiles > 0) {
        fetch_tile(0, e_cur);
        stash_tile(0);
    }
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        if (t + 2 < ntiles) e_nx2 = entry_of(t + 2);
        if (t + 1 < ntiles) fetch_tile(t + 1, e_nxt);
        if (t + 2 < ntiles) load_side(e_nx2);

        // Online softmax (Eq. 1) in base 2 with 1/sqrt(D) folded into c.  The reference subtracted in
        // the exponent is moved, and the accumulators rescaled, only when a row outgrows it by more
        // than 2^kRescaleSlack (or has none yet): the softmax does not depend on the reference.
        f32x16 s[2];
        scores(t, e_cur, s);
        float mt = s[0][0];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) mt = fmaxf(mt, s[kb2][r]);
        // the two halves of the wavefront hold different keys of the same 32 queries: their maxima
        // are exchanged only when some lane asks for the reference to move
        const bool grow = has_ref ? (mt - m_ref) * c > kRescaleSlack : mt > -INFINITY;
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            mt = fmaxf(mt, other_half(mt));
            if (mt > -INFINITY) {
                const float m_new = has_ref ? fmaxf(m_ref, mt) : mt;
                const float alpha = has_ref ? fast_exp2((m_ref - m_new) * c) : 0.f;  // nothing accumulated before
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < D / 32; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
                m_ref = m_new;
                has_ref = true;
            }
        }
        const float psum = exponentiate(s);
        l_run += psum;

        bf16x8 pf[4];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int u2 = 0; u2 < 2; ++u2) {
                u32x4 w;
                w.x = pack_bf16(s[kb2][8 * u2 + 0], s[kb2][8 * u2 + 1]);
                w.y = pack_bf16(s[kb2][8 * u2 + 2], s[kb2][8 * u2 + 3]);
                w.z = pack_bf16(s[kb2][8 * u2 + 4], s[kb2][8 * u2 + 5]);
                w.w = pack_bf16(s[kb2][8 * u2 + 6], s[kb2][8 * u2 + 7]);
                pf[2 * kb2 + u2] = as_bf16x8(w);
            }

        const unsigned char* vl = v_lds(t);
#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(st.v_frag(vl, db, u), pf[u], oacc[db], 0, 0, 0);
#ifdef RF_SCHED_PV
        {
            constexpr int PER = ST::V_READS_PER_FRAG, TOTAL = 4 * (D / 32);
            __builtin_amdgcn_sched_group_barrier(0x100, RF_SCHED_PV * PER, 1);
#pragma unroll
            for (int i = 0; i < TOTAL - RF_SCHED_PV; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 1);
                __builtin_amdgcn_sched_group_barrier(0x100, PER, 1);
            }
            __builtin_amdgcn_sched_group_barrier(0x008, RF_SCHED_PV, 1);
        }
#endif

        if (t + 1 < ntiles) stash_tile(t + 1);
        if (t + 2 < ntiles) stash_side(t + 2, e_nx2);
        e_cur = e_nxt;
        e_nxt = e_nx2;
        __syncthreads();
    }

    // Eq. 2: divide by the softmax denominator and store.  Lane (hf, m) owns query m and, per
    // 32-channel block, channels 8*(r/4) + 4*hf + r%4.
    const float l_tot = l_run + other_half(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (qrow < N) {
        uint16_t* orow = a.O + static_cast<size_t>(qk.bh) * N * D + static_cast<size_t>(qrow) * D;
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
}

// Wavefronts per SIMD the register allocation is held to: three for head_dim 64 (measured
// best; its accumulators are half the size), two for 96 and 128, one for the 64-row blocks of
// the larger head dims, whose two-unit staging would otherwise spill.
constexpr int attn_waves_per_simd(int D, int NW) { return NW == 4 ? (D == 64 ? 3 : 2) : (D == 64 ? 2 : 1); }

template <int D, int NW>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(attn_waves_per_simd(D, NW), attn_waves_per_simd(D, NW)))) attn_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const DevicePlan& pl = a.plan;
    // Workgroup ids go to the 8 XCDs round-robin.  Every XCD takes one eighth of a head's query
    // blocks, a contiguous run of the pattern's block order (neighbours in that order walk nearly
    // the same key tiles, which they then share through the XCD's L2), and all XCDs move through
    // the heads together, so the K/V of the head in flight (tens of MB) stays resident in the
    // memory-side cache for whatever misses L2.
    const int per_xcd = (pl.nQB + 7) >> 3;
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int ordinal = xcd * per_xcd + slot % per_xcd;
    if (ordinal >= pl.nQB) return;
    QueryBlock qk;
    qk.bh = slot / per_xcd;
    int cls = a.head_class[qk.bh];
    if (static_cast<unsigned>(cls) > 3u) cls = RF_DENSE;
    qk.cls = cls;
    qk.qb = cls == RF_DENSE ? ordinal : pl.qorder[cls][ordinal];
    qk.cols = nullptr;
    if (cls == RF_DENSE) {
        qk.ntiles = pl.nKT;
        qk.keyN = pl.N;
        attend<D, NW, MODE_ALL>(a, qk, smem);
    } else if (cls == RF_TEXTURAL && qk.qb < pl.first_text_qb) {
        // Textural query blocks made only of video tokens see the compacted key sequence
        qk.ntiles = pl.nCT;
        qk.keyN = pl.Nc;
        attend<D, NW, MODE_COMPACT>(a, qk, smem);
    } else {
        const int e0 = pl.row_ptr[cls][qk.qb];
        qk.ntiles = pl.row_ptr[cls][qk.qb + 1] - e0;
        qk.cols = pl.cols[cls] + e0;
        qk.keyN = pl.N;
        attend<D, NW, MODE_LISTED>(a, qk, smem);
    }
}

template <int D, int NW>
static int launch_one(const AttnArgs& a, hipStream_t st) {
    constexpr int NT = 64 * NW;
    constexpr int smem = AttnSmem<D, NW>::BYTES;
    static bool configured = false;  // raising the dynamic-LDS limit is per function, once
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<D, NW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return static_cast<int>(e);
        configured = true;
    }
    const int grid = 8 * ((a.plan.nQB + 7) / 8) * a.BH;
    hipLaunchKernelGGL((attn_kernel<D, NW>), dim3(grid), dim3(NT), smem, st, a);
    return static_cast<int>(hipGetLastError());
}

int launch_attention(const AttnArgs& a, int D, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int nw = a.plan.block / 32;
    if (D == 64 && nw == 2) return launch_one<64, 2>(a, st);
    if (D == 64 && nw == 4) return launch_one<64, 4>(a, st);
    if (D == 96 && nw == 2) return launch_one<96, 2>(a, st);
    if (D == 96 && nw == 4) return launch_one<96, 4>(a, st);
    if (D == 128 && nw == 2) return launch_one<128, 2>(a, st);
    if (D == 128 && nw == 4) return launch_one<128, 4>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace rf
