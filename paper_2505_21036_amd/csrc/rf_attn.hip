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
    uint2 reg[PER_THREAD][8];

    template <typename F>
    __device__ __forceinline__ void fetch(const uint16_t* base, int tid, F row_token) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int kg = u / (D / 4), dc = u % (D / 4);
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    reg[i][e] = *reinterpret_cast<const uint2*>(base + static_cast<size_t>(row_token(8 * kg + e)) * D + 4 * dc);
            }
        }
    }
    __device__ __forceinline__ void stash(unsigned char* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int u = tid + i * NT;
            if (UNITS % NT == 0 || u < UNITS) {
                const int kg = u / (D / 4), dc = u % (D / 4);
                uint4 out[4];
#pragma unroll
                for (int w = 0; w < 4; ++w) {  // keys 2w, 2w+1 side by side, one channel per output row
                    const uint2 a = reg[i][2 * w], b = reg[i][2 * w + 1];
                    (&out[0].x)[w] = __builtin_amdgcn_perm(b.x, a.x, 0x05040100u);
                    (&out[1].x)[w] = __builtin_amdgcn_perm(b.x, a.x, 0x07060302u);
                    (&out[2].x)[w] = __builtin_amdgcn_perm(b.y, a.y, 0x05040100u);
                    (&out[3].x)[w] = __builtin_amdgcn_perm(b.y, a.y, 0x07060302u);
                }
#pragma unroll
                for (int dd = 0; dd < 4; ++dd)
                    *reinterpret_cast<uint4*>(lds + (4 * dc + dd) * ROW_BYTES + 16 * kg) = out[dd];
            }
        }
    }
    // A operand of O^T = V^T P^T: channels 32*db + m, keys 16*u + 8*hf .. +7
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int db, int u, int m, int hf) {
        return as_bf16x8(*reinterpret_cast<const uint4*>(lds + (32 * db + m) * ROW_BYTES + 32 * u + 16 * hf));
    }
};

template <int D, int NT>
struct AttnSmem {
    static constexpr int K_OFF = 0;
    static constexpr int V_OFF = 2 * KTile<D, NT>::BYTES;
    static constexpr int A_OFF = V_OFF + 2 * VtTile<D, NT>::BYTES;
    static constexpr int BYTES = A_OFF + 2 * kTileK * 4;
};

template <int D, int NW>
__global__ void __launch_bounds__(64 * NW) attn_kernel(AttnArgs a) {
    constexpr int NT = 64 * NW, BQ = 32 * NW, SUB = BQ / kTileK;
    using KT = KTile<D, NT>;
    using VT = VtTile<D, NT>;
    using SM = AttnSmem<D, NT>;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

    const DevicePlan& pl = a.plan;
    const int item = xcd_contiguous_item(blockIdx.x, pl.nQB * a.BH);
    if (item < 0) return;
    const int bh = item / pl.nQB, qb = item % pl.nQB;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;
    const int N = pl.N, Nv = pl.Nv;

    int cls = a.head_class[bh];
    if (static_cast<unsigned>(cls) > 3u) cls = RF_DENSE;
    // Textural query blocks made only of video tokens see the compacted key sequence (Eq. 5)
    const bool compact = cls == RF_TEXTURAL && qb < pl.first_text_qb;
    const bool listed = cls != RF_DENSE && !compact;
    const int keyN = compact ? pl.Nc : N;
    const int32_t* cols = nullptr;
    int nblk;
    if (listed) {
        const int e0 = pl.row_ptr[cls][qb];
        nblk = pl.row_ptr[cls][qb + 1] - e0;
        cols = pl.cols[cls] + e0;
    } else {
        nblk = compact ? pl.nCB : pl.nKB;
    }
    const int ntiles = nblk * SUB;
    const int32_t* cidx = pl.cidx;
    const int32_t* attr = listed ? pl.attr[cls] : nullptr;

    const size_t head_off = static_cast<size_t>(bh) * N * D;
    const uint16_t* Qh = a.Q + head_off;
    const uint16_t* Kh = a.K + head_off;
    const uint16_t* Vh = a.V + head_off;

    // this lane's query
    const int qrow = qb * BQ + wave * 32 + m;
    const int qtok = min(qrow, N - 1);
    bf16x8 qf[D / 16];
    load_q_frags<D>(Qh, qtok, hf, qf);
    int q_attr = 0, q_rad = 0x3fffffff;  // text queries keep everything
    if (listed) {
        // Spatial / Temporal compare the query's frame / position with the key's; the Textural
        // table is 0 on kept keys and 1 on dropped ones, compared against 0 with radius 0
        if (cls != RF_TEXTURAL) q_attr = attr[qtok];
        if (qtok < Nv) q_rad = pl.radius[cls];
    }

    f32x16 oacc[D / 32];
#pragma unroll
    for (int db = 0; db < D / 32; ++db) oacc[db] = f32x16{0};
    float m_run = -INFINITY, l_run = 0.f;
    const float c = a.scale_log2;

    KT kt;
    VT vt;
    int attr_reg = 0;

    // tile t -> (first key position, partial flag)
    auto tile_info = [&](int t, int* k0, bool* partial) {
        const int blk = t / SUB, s = t % SUB;
        int entry;
        if (listed) entry = cols[blk];
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
            return compact ? cidx[key] : key;
        };
        kt.fetch(Kh, tid, row_token);
        vt.fetch(Vh, tid, row_token);
        if (listed && partial && tid < kTileK) attr_reg = attr[min(k0 + tid, N - 1)];
    };
    auto stash_tile = [&](int t) {
        const int buf = t & 1;
        kt.stash(smem + SM::K_OFF + buf * KT::BYTES, tid);
        vt.stash(smem + SM::V_OFF + buf * VT::BYTES, tid);
        if (tid < kTileK) reinterpret_cast<int*>(smem + SM::A_OFF)[buf * kTileK + tid] = attr_reg;
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
                    if (listed) {
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
        const float m_new = fmaxf(m_run, mt);
        const float m_use = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = fast_exp2((m_run - m_use) * c);
        const float mc = m_use * c;
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
                uint4 w;
                w.x = pack_bf16(p[8 * u2 + 0], p[8 * u2 + 1]);
                w.y = pack_bf16(p[8 * u2 + 2], p[8 * u2 + 3]);
                w.z = pack_bf16(p[8 * u2 + 4], p[8 * u2 + 5]);
                w.w = pack_bf16(p[8 * u2 + 6], p[8 * u2 + 7]);
                pf[2 * kb2 + u2] = as_bf16x8(w);
            }
        }
        l_run = l_run * alpha + psum;
        m_run = m_new;

#pragma unroll
        for (int db = 0; db < D / 32; ++db) {
            f32x16 acc = oacc[db];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] *= alpha;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(VT::frag(vl, db, u, m, hf), pf[u], acc, 0, 0, 0);
            oacc[db] = acc;
        }

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
                uint2 w;
                w.x = pack_bf16(oacc[db][4 * rq + 0] * inv, oacc[db][4 * rq + 1] * inv);
                w.y = pack_bf16(oacc[db][4 * rq + 2] * inv, oacc[db][4 * rq + 3] * inv);
                *reinterpret_cast<uint2*>(orow + 32 * db + 8 * rq + 4 * hf) = w;
            }
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
