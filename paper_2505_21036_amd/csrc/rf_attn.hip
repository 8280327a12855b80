// Block-sparse attention forward for RainFusion's head patterns (Eq. 1-5; Fig. 2a), gfx950.
//
// One workgroup = one query block of one head.  It reads the head's class on the device,
// walks that class's list of key blocks (skipped blocks cost no traffic), stages K and V^T
// tiles of 64 keys through LDS with one tile of prefetch held in registers, forms the
// transposed score tile with bf16 MFMA, runs the online softmax in fp32 with exp2, and
// accumulates O^T = V^T P^T with bf16 MFMA.  In key blocks flagged partial the token-level
// predicate of the pattern is re-applied to each score.
#include "rf_device.h"

namespace rf {

// V tile stored transposed in LDS: one row per channel holding the tile's 64 keys, so the
// A operand of O^T = V^T P^T (8 consecutive keys of one channel) is a single 16-byte read.
template <int D, int NT>
struct VtTile {
    static constexpr int ROW_BYTES = 2 * kTileK + 16;
    static constexpr int BYTES = D * ROW_BYTES;
    static constexpr int UNITS = (kTileK / 8) * (D / 4);  // a unit = 8 keys x 4 channels
    static constexpr int PER_THREAD = (UNITS + NT - 1) / NT;
    u32x2 reg[PER_THREAD][8];

    template <typename F>
    __device__ __forceinline__ void fetch(const uint16_t* base, int tid, F row_token) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int kg = u / (D / 4), dc = u % (D / 4);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    reg[i][e] = *reinterpret_cast<const u32x2*>(base + static_cast<size_t>(row_token(8 * kg + e)) * D + 4 * dc);
            }
        }
    }
    __device__ __forceinline__ void stash(unsigned char* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int kg = u / (D / 4), dc = u % (D / 4);
                uint32_t o[4][4];  // [channel][key pair]
#pragma unroll
                for (int w = 0; w < 4; ++w) {  // keys 2w, 2w+1 side by side, one channel per output row
                    const u32x2 a = reg[i][2 * w], b = reg[i][2 * w + 1];
                    o[0][w] = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u);
                    o[1][w] = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
                    o[2][w] = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u);
                    o[3][w] = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
                }
#pragma unroll
                for (int dd = 0; dd < 4; ++dd)
                    *reinterpret_cast<u32x4*>(lds + (4 * dc + dd) * ROW_BYTES + 16 * kg) =
                        u32x4{o[dd][0], o[dd][1], o[dd][2], o[dd][3]};
            }
        }
    }
    // A operand of O^T = V^T P^T: channels 32*db + m, keys 16*u + 8*hf .. +7
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int db, int u, int m, int hf) {
        return as_bf16x8(*reinterpret_cast<const u32x4*>(lds + (32 * db + m) * ROW_BYTES + 32 * u + 16 * hf));
    }
};

template <int D, int NT>
struct AttnSmem {
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = 2 * KTile<D, NT>::BYTES;
    static constexpr int A_OFF = V_OFF + 2 * VtTile<D, NT>::BYTES;
    static constexpr int BYTES = A_OFF + 2 * kTileK * 4;
};

// How a query block finds its key tiles.
enum : int {
    MODE_ALL = 0,      // every key block of the sequence in order (dense heads)
    MODE_COMPACT = 1,  // every block of the compacted key sequence; rows go through the index table (Eq. 5)
    MODE_LISTED = 2    // the CSR list of the head's pattern; partial blocks re-apply the predicate
};

struct QueryBlock {
    int bh, qb, cls;
    const int32_t* cols;  // MODE_LISTED: this query block's entries
    int nblk;             // key blocks to visit
    int keyN;             // length of the key sequence walked (N, or Nc when compacted)
};

// exp2 arguments may exceed 0 by at most this much before the running reference is moved: the
// softmax is invariant to the reference, so a stale one only costs range, which fp32/bf16 have.
constexpr float kRescaleSlack = 8.f;

template <int D, int NW, int MODE>
__device__ __forceinline__ void attend(const AttnArgs& a, const QueryBlock& qk, unsigned char* smem) {
    constexpr int NT = 64 * NW, BQ = 32 * NW, SUB = BQ / kTileK;
    using KT = KTile<D, NT>;
    using VT = VtTile<D, NT>;
    using SM = AttnSmem<D, NT>;
    const DevicePlan& pl = a.plan;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;
    const int N = pl.N, Nv = pl.Nv, keyN = qk.keyN;
    const int ntiles = qk.nblk * SUB;
    const int32_t* cidx = pl.cidx;
    const int32_t* attr = MODE == MODE_LISTED ? pl.attr[qk.cls] : nullptr;

    const size_t head_off = static_cast<size_t>(qk.bh) * N * D;
    const uint16_t* Qh = a.Q + head_off;
    const uint16_t* Kh = a.K + head_off;
    const uint16_t* Vh = a.V + head_off;

    // this lane's query
    const int qrow = qk.qb * BQ + wave * 32 + m;
    const int qtok = min(qrow, N - 1);
    bf16x8 qf[D / 16];
    load_q_frags<D>(Qh, qtok, hf, qf);
    int q_attr = 0, q_rad = 0x3fffffff;  // text queries keep everything
    if (MODE == MODE_LISTED) {
        // Spatial / Temporal compare the query's frame / position with the key's; the Textural
        // table is 0 on kept keys and 1 on dropped ones, compared against 0 with radius 0
        if (qk.cls != RF_TEXTURAL) q_attr = attr[qtok];
        if (qtok < Nv) q_rad = pl.radius[qk.cls];
    }

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) oacc[db] = f32x16{0};
    // m_ref: reference subtracted inside exp2 (in units of raw score); l_run: this lane's share of the denominator
    float m_ref = -INFINITY, l_run = 0.f;
    const float c = a.scale_log2;

    KT kt;
    VT vt;
    int attr_reg = 0;

    // tile t -> (first key position, partial flag)
    auto tile_info = [&](int t, int* k0, bool* partial) {
        const int blk = t / SUB, s = t % SUB;
        int entry;
        if (MODE == MODE_LISTED) entry = qk.cols[blk];
        else entry = blk | ((blk + 1) * BQ > keyN ? RF_PLAN_PARTIAL : 0);
        *k0 = (entry & ~RF_PLAN_PARTIAL) * BQ + s * kTileK;
        *partial = (entry & RF_PLAN_PARTIAL) != 0;
    };
    auto fetch_tile = [&](int t) {
        int k0;
        bool partial;
        tile_info(t, &k0, &partial);
        auto row_token = [&](int r) {
            const int key = min(k0 + r, keyN - 1);
            return MODE == MODE_COMPACT ? cidx[key] : key;
        };
        kt.fetch(Kh, tid, row_token);
        vt.fetch(Vh, tid, row_token);
        if (MODE == MODE_LISTED && partial && tid < kTileK) attr_reg = attr[min(k0 + tid, N - 1)];
    };
    auto stash_tile = [&](int t) {
        const int buf = t & 1;
        kt.stash(smem + SM::K_OFF + buf * KT::BYTES, tid);
        vt.stash(smem + SM::V_OFF + buf * VT::BYTES, tid);
        if (MODE == MODE_LISTED && tid < kTileK) reinterpret_cast<int*>(smem + SM::A_OFF)[buf * kTileK + tid] = attr_reg;
    };

    if (ntiles > 0) {
        fetch_tile(0);
        stash_tile(0);
    }
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        if (t + 1 < ntiles) fetch_tile(t + 1);

        int k0;
        bool partial;
        tile_info(t, &k0, &partial);
        const unsigned char* kl = smem + SM::K_OFF + buf * KT::BYTES;
        const unsigned char* vl = smem + SM::V_OFF + buf * VT::BYTES;

        f32x16 s[2];
        score_tile<D, NT>(kl, qf, m, hf, s);

        if (partial) {
            const int* al = reinterpret_cast<const int*>(smem + SM::A_OFF) + buf * kTileK;
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int koff = 32 * kb2 + key_of_reg(r, hf);
                    const int kidx = k0 + koff;
                    bool ok = kidx < keyN;
                    if (MODE == MODE_LISTED) {
                        const int d = q_attr - al[koff];
                        ok = ok && ((d < 0 ? -d : d) <= q_rad || kidx >= Nv);
                    }
                    s[kb2][r] = ok ? s[kb2][r] : -INFINITY;
                }
        }

        // online softmax (Eq. 1), base-2 exponent with 1/sqrt(D) folded into c
        float mt = s[0][0];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) mt = fmaxf(mt, s[kb2][r]);
        mt = fmaxf(mt, other_half(mt));
        // move the reference only when some row of this wavefront outgrew it by more than the slack
        const bool grow = (mt - m_ref) * c > kRescaleSlack || (m_ref == -INFINITY && mt > -INFINITY);
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            const float m_new = fmaxf(m_ref, mt);
            const float m_use = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = fast_exp2((m_ref - m_use) * c);
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < D / 32; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
            m_ref = m_new;
        }
        const float mc = (m_ref == -INFINITY ? 0.f : m_ref) * c;
        float psum = 0.f;
        bf16x8 pf[4];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2) {
            float p[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                p[r] = fast_exp2(fmaf(s[kb2][r], c, -mc));
                psum += p[r];
            }
#pragma unroll
            for (int u2 = 0; u2 < 2; ++u2) {
                u32x4 w;
                w.x = pack_bf16(p[8 * u2 + 0], p[8 * u2 + 1]);
                w.y = pack_bf16(p[8 * u2 + 2], p[8 * u2 + 3]);
                w.z = pack_bf16(p[8 * u2 + 4], p[8 * u2 + 5]);
                w.w = pack_bf16(p[8 * u2 + 6], p[8 * u2 + 7]);
                pf[2 * kb2 + u2] = as_bf16x8(w);
            }
        }
        l_run += psum;

#pragma unroll
        for (int db = 0; db < D / 32; ++db)
#pragma unroll
            for (int u = 0; u < 4; ++u)
                oacc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VT::frag(vl, db, u, m, hf), pf[u], oacc[db], 0, 0, 0);

        if (t + 1 < ntiles) stash_tile(t + 1);
        __syncthreads();
    }

    // Eq. 2: divide by the softmax denominator and store.  Lane (hf, m) owns query m and, per
    // 32-channel block, channels 8*(r/4) + 4*hf + r%4.
    const float l_tot = l_run + other_half(l_run);
    const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
    if (qrow < N) {
        uint16_t* orow = a.O + head_off + static_cast<size_t>(qrow) * D;
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

template <int D, int NW>
__global__ void __launch_bounds__(64 * NW) __attribute__((amdgpu_waves_per_eu(2))) attn_kernel(AttnArgs a) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    const DevicePlan& pl = a.plan;
    const int item = xcd_contiguous_item(blockIdx.x, pl.nQB * a.BH);
    if (item < 0) return;
    QueryBlock qk;
    qk.bh = item / pl.nQB;
    qk.qb = item % pl.nQB;
    int cls = a.head_class[qk.bh];
    if (static_cast<unsigned>(cls) > 3u) cls = RF_DENSE;
    qk.cls = cls;
    qk.cols = nullptr;
    if (cls == RF_DENSE) {
        qk.nblk = pl.nKB;
        qk.keyN = pl.N;
        attend<D, NW, MODE_ALL>(a, qk, smem);
    } else if (cls == RF_TEXTURAL && qk.qb < pl.first_text_qb) {
        // Textural query blocks made only of video tokens see the compacted key sequence
        qk.nblk = pl.nCB;
        qk.keyN = pl.Nc;
        attend<D, NW, MODE_COMPACT>(a, qk, smem);
    } else {
        const int e0 = pl.row_ptr[cls][qk.qb];
        qk.nblk = pl.row_ptr[cls][qk.qb + 1] - e0;
        qk.cols = pl.cols[cls] + e0;
        qk.keyN = pl.N;
        attend<D, NW, MODE_LISTED>(a, qk, smem);
    }
}

template <int D, int NW>
static int launch_one(const AttnArgs& a, hipStream_t st) {
    constexpr int NT = 64 * NW;
    constexpr int smem = AttnSmem<D, NT>::BYTES;
    static bool configured = false;  // raising the dynamic-LDS limit is per function, once
    if (!configured) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_kernel<D, NW>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, smem);
        if (e != hipSuccess) return static_cast<int>(e);
        configured = true;
    }
    const int total = a.plan.nQB * a.BH;
    const int grid = 8 * ((total + 7) / 8);
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
