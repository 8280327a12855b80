// ARM head classifier (Sec. 3.3, Eq. 6, Alg. 1) on gfx950.
//
// Pass 0 measures the recall of the Temporal mask (R-hat), pass 1 that of the Spatial mask
// (R-tilde).  A pass is described by its sample (sample a is token a * stride), an integer
// attribute per sample (in-frame position, resp. frame index) and a radius: the mask keeps
// |attr[a] - attr[b]| <= radius.  The scores Q'K'^T / sqrt(D) are formed tile by tile with
// bf16 MFMA and never stored; the sampled K' rows go global -> LDS one tile ahead, gathered by
// index arithmetic (no copy of Q', K' is made).  Per sampled query the kernel keeps a reference for
// the exponent, the softmax denominator over all sampled keys (M_init) and the part of it on kept
// keys (M').  The masks are bands on the attribute, so for most (32 queries, 64 keys) pairs every
// entry is kept or every entry is dropped; the kernel tells from the attribute ranges of the two
// sides and applies the mask entry by entry only where the band's edge crosses the pair.
// A sample's attribute (in-frame position or frame) follows from its index by arithmetic; no table of
// samples exists anywhere.  Per-row recalls go to scratch and are reduced in a fixed order by
// arm_finish_kernel, which also applies the decision rule.
#include <mutex>

#include "rf_device.h"

namespace rf {

// Wavefronts per workgroup, 32 sampled queries each.  A workgroup walks all sampled keys, so the
// launch has (samples / 32 / waves) workgroups per head and pass: 8 waves when the passes run apart,
// 4 when one workgroup serves both (half as many items, each twice as long: the finer grain keeps
// the 256 CUs evenly loaded).
constexpr int kArmWavesApart = 8, kArmWavesBoth = 4;
// as in the attention kernel: the reference in the exponent moves only when a row outgrows it by this
constexpr float kArmRescaleSlack = 8.f;

template <int D, int NW>
struct ArmSmem {
    using ST = DirectTile<D, NW>;
    static constexpr int K_OFF = 0;                      // two K' tiles
    static constexpr int ATTR_OFF = 2 * ST::K_BYTES;     // per tile and pass: the 64 samples' attributes, then bounds on them (lowest, highest)
    static constexpr int ATTR_SLOT = kTileK + 2;
    static constexpr int BYTES = ATTR_OFF + 2 * 2 * ATTR_SLOT * 4 + 16;
    static_assert(ST::K_BYTES % 256 == 0, "tile buffers must start at multiples of 256 bytes (see DirectTile::k_address)");
};

// BOTH: the two passes use the same sample (equal-interval sampling), so one workgroup forms each
// score tile once and keeps the kept-key sums of both masks; the arithmetic per pass, and so every
// recall, is the same as when the passes run apart.
template <int D, bool BOTH>
__global__ void __launch_bounds__(64 * (BOTH ? kArmWavesBoth : kArmWavesApart)) arm_recall_kernel(ArmArgs a, int nQB) {
    constexpr int NW = BOTH ? kArmWavesBoth : kArmWavesApart, BQ = 32 * NW, NP = BOTH ? 2 : 1;
    using SM = ArmSmem<D, NW>;
    using ST = typename SM::ST;
    extern __shared__ __attribute__((aligned(256))) unsigned char smem[];  // the kernel's only LDS: starts at address 0
    int* abuf = reinterpret_cast<int*>(smem + SM::ATTR_OFF);

    const int item = xcd_contiguous_item(blockIdx.x, nQB * (2 / NP) * a.BH);
    if (item < 0) return;
    const int qb = item % nQB, pass0 = BOTH ? 0 : (item / nQB) & 1, bh = item / ((2 / NP) * nQB);
    ArmPass ps[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) ps[i] = a.pass[pass0 + i];
    const int n = ps[0].n, stride = ps[0].stride;  // BOTH: the same in the two passes (the host checks)
    if (qb * BQ >= n) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, m = lane & 31;

    // samples are video tokens; first_video_row is where those start in the tensors
    const size_t head_off = (static_cast<size_t>(bh) * a.N + a.first_video_row) * D;
    const uint16_t* Qh = a.Q + head_off;
    const unsigned char* Kh = reinterpret_cast<const unsigned char*>(a.K + head_off);

    const int qs = qb * BQ + wave * 32 + m;  // this lane's sampled query
    const int qsc = min(qs, n - 1);
    bf16x8 qf[D / 16];
    load_q_frags<D>(Qh, qsc * stride, hf, qf);
    auto attr_of = [&](int i, int sample) {
        const int token = sample * stride;
        return ps[i].by_frame ? token / ps[i].HW : token % ps[i].HW;
    };
    // attribute of this lane's query and its range over the wavefront's 32 queries (both halves hold
    // the same queries)
    int q_attr[NP], q_min[NP], q_max[NP];
#pragma unroll
    for (int i = 0; i < NP; ++i) {
        q_attr[i] = attr_of(i, qsc);
        int lo = q_attr[i], hi = q_attr[i];
#pragma unroll
        for (int w = 1; w < 32; w <<= 1) {
            lo = min(lo, __shfl_xor(lo, w, 64));
            hi = max(hi, __shfl_xor(hi, w, 64));
        }
        q_min[i] = __builtin_amdgcn_readfirstlane(lo);
        q_max[i] = __builtin_amdgcn_readfirstlane(hi);
    }

    // m_ref: reference subtracted inside exp2 (raw score units); l_all / l_kept: this lane's share of
    // the denominator over all sampled keys and over the kept ones, both relative to m_ref
    float m_ref = 0.f, l_all = 0.f, l_kept[NP][kMaxBw];
    bool has_ref = false;
#pragma unroll
    for (int i = 0; i < NP; ++i)
#pragma unroll
        for (int b = 0; b < kMaxBw; ++b) l_kept[i][b] = 0.f;
    const int n_bw = a.n_bw;
    const float c = a.scale_log2;
    const int ntiles = (n + kTileK - 1) / kTileK;

    ST st;
    st.init(tid);
    auto k_lds = [&](int t) { return smem + SM::K_OFF + (t & 1) * ST::K_BYTES; };
    auto attr_slot = [&](int t, int i) { return abuf + ((t & 1) * 2 + i) * SM::ATTR_SLOT; };
    int attr_reg[NP] = {};
    auto fetch_tile = [&](int t) {
        const int k0 = t * kTileK;
        if (stride == 1 && k0 + kTileK <= n)
            st.template issue_consecutive<false>(Kh + static_cast<size_t>(k0) * (2 * D), nullptr, k_lds(t), nullptr);
        else
            st.template issue<false>(Kh, nullptr, k_lds(t), nullptr, [&](int r) { return min(k0 + r, n - 1) * stride; });
        // the tile's attributes (first wavefront, one sample per lane)
        if (tid < kTileK) {
#pragma unroll
            for (int i = 0; i < NP; ++i) attr_reg[i] = attr_of(i, min(k0 + tid, n - 1));
        }
    };
    // Also bounds on the tile's attributes: samples are in token order, so frames never decrease, and
    // positions do not either as long as the tile stays inside one frame; a tile that crosses into
    // another frame gets the widest bounds (the caller then masks it entry by entry, which is exact).
    auto stash_attr = [&](int t) {
        if (tid >= kTileK) return;
        const int first = t * kTileK * stride, last = min(t * kTileK + kTileK - 1, n - 1) * stride;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            int* slot = attr_slot(t, i);
            slot[tid] = attr_reg[i];
            int lo = __builtin_amdgcn_readlane(attr_reg[i], 0), hi = __builtin_amdgcn_readlane(attr_reg[i], kTileK - 1);
            if (!ps[i].by_frame && first / ps[i].HW != last / ps[i].HW) {
                lo = 0;
                hi = ps[i].HW - 1;
            }
            if (tid == 0) {
                slot[kTileK] = lo;
                slot[kTileK + 1] = hi;
            }
        }
    };
    fetch_tile(0);
    stash_attr(0);
    ST::template wait_landed<0>();
    __syncthreads();
    // the compiler cannot see the tile loads; make its own wait for the Q loads happen here, not in the loop
#pragma unroll
    for (int cc = 0; cc < D / 16; ++cc) asm volatile("" ::"v"(__builtin_bit_cast(u32x4, qf[cc])));

    for (int t = 0; t < ntiles; ++t) {
        if (t + 1 < ntiles) fetch_tile(t + 1);
        const int k0 = t * kTileK;

        f32x16 s[2];
        st.template scores<kAheadK>(st.k_address(k_lds(t)), qf, s);
        if (k0 + kTileK > n) {  // ragged last tile: samples past the end do not exist
#pragma unroll
            for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (k0 + 32 * kb2 + key_of_reg(r, hf) >= n) s[kb2][r] = -INFINITY;
        }
        float mt = s[0][0];
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) mt = fmaxf(mt, s[kb2][r]);
        // the two halves of the wavefront hold different keys of the same 32 queries: their maxima are
        // exchanged, and the sums rescaled, only when some lane asks for the reference to move
        const bool grow = has_ref ? (mt - m_ref) * c > kArmRescaleSlack : mt > -INFINITY;
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            mt = fmaxf(mt, other_half(mt));
            if (mt > -INFINITY) {
                const float m_new = has_ref ? fmaxf(m_ref, mt) : mt;
                const float alpha = has_ref ? fast_exp2((m_ref - m_new) * c) : 0.f;  // nothing accumulated before
                l_all *= alpha;
#pragma unroll
                for (int i = 0; i < NP; ++i)
#pragma unroll
                    for (int b = 0; b < kMaxBw; ++b) l_kept[i][b] *= alpha;
                m_ref = m_new;
                has_ref = true;
            }
        }
        const float mc = m_ref * c;
        // the tile's terms of the denominator, summed in register order whatever the masks need
        float sum_all = 0.f;
#pragma unroll
        for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                s[kb2][r] = fast_exp2(fmaf(s[kb2][r], c, -mc));
                sum_all += s[kb2][r];
            }
        l_all += sum_all;
#pragma unroll
        for (int i = 0; i < NP; ++i) {
            // Where does the band's edge fall for this (wavefront, tile) pair?  inside: bit b set if every
            // pair is within radius b; mixed: some candidate has both kept and dropped pairs here.
            const int* al = attr_slot(t, i);
            const int k_min = __builtin_amdgcn_readfirstlane(al[kTileK]), k_max = __builtin_amdgcn_readfirstlane(al[kTileK + 1]);
            const int reach = max(k_max - q_min[i], q_max[i] - k_min), gap = max(k_min - q_max[i], q_min[i] - k_max);
            int inside = 0;
            bool mixed = false;
#pragma unroll
            for (int b = 0; b < kMaxBw; ++b) {
                if (b >= n_bw) break;
                if (reach <= ps[i].radius[b]) inside |= 1 << b;
                else if (gap <= ps[i].radius[b]) mixed = true;
            }
            if (!mixed) {
#pragma unroll
                for (int b = 0; b < kMaxBw; ++b) l_kept[i][b] += ((inside >> b) & 1) ? sum_all : 0.f;
            } else {
                float sum_kept[kMaxBw];
#pragma unroll
                for (int b = 0; b < kMaxBw; ++b) sum_kept[b] = 0.f;
#pragma unroll
                for (int kb2 = 0; kb2 < 2; ++kb2)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float p = s[kb2][r];
                        const int d = q_attr[i] - al[32 * kb2 + key_of_reg(r, hf)];
                        const int dist = d < 0 ? -d : d;
                        sum_kept[0] += dist <= ps[i].radius[0] ? p : 0.f;
                        if (n_bw > 1) {  // uniform: the per-head bandwidth variant measures every candidate at once
#pragma unroll
                            for (int b = 1; b < kMaxBw; ++b) sum_kept[b] += (b < n_bw && dist <= ps[i].radius[b]) ? p : 0.f;
                        }
                    }
#pragma unroll
                for (int b = 0; b < kMaxBw; ++b) l_kept[i][b] += sum_kept[b];
            }
        }

        if (t + 1 < ntiles) stash_attr(t + 1);
        ST::template wait_landed<0>();
        __syncthreads();
    }
    l_all += other_half(l_all);
#pragma unroll
    for (int i = 0; i < NP; ++i)
#pragma unroll
        for (int b = 0; b < kMaxBw; ++b) {
            if (b >= n_bw) break;
            const float kept = l_kept[i][b] + other_half(l_kept[i][b]);
            if (hf == 0 && qs < n)
                a.row_recall[((static_cast<size_t>(bh) * 2 + pass0 + i) * n_bw + b) * a.max_n + qs] = kept / l_all;  // Eq. 6, one row
        }
}

// Mean of the per-row recalls in a fixed summation order, then Alg. 1's rule (with several
// candidate bandwidths: the narrowest one that holds the threshold, Temporal before Spatial).
__global__ void __launch_bounds__(256) arm_finish_kernel(ArmArgs a) {
    __shared__ float red[256];
    __shared__ float rec[2][kMaxBw];
    const int bh = blockIdx.x, tid = threadIdx.x, n_bw = a.n_bw;
    for (int pass = 0; pass < 2; ++pass)
        for (int b = 0; b < n_bw; ++b) {
            const int n = a.pass[pass].n;
            const float* rr = a.row_recall + ((static_cast<size_t>(bh) * 2 + pass) * n_bw + b) * a.max_n;
            float acc = 0.f;
            for (int i = tid; i < n; i += 256) acc += rr[i];
            red[tid] = acc;
            __syncthreads();
            for (int w = 128; w > 0; w >>= 1) {
                if (tid < w) red[tid] += red[tid + w];
                __syncthreads();
            }
            if (tid == 0) rec[pass][b] = red[0] / static_cast<float>(n);
            __syncthreads();
        }
    if (tid == 0) {
        int cls = a.fallback_class, chosen = -1;
        for (int pass = 0; pass < 2 && chosen < 0; ++pass)  // Temporal (pass 0) has priority
            for (int i = 0; i < n_bw && chosen < 0; ++i) {
                const int b = a.by_width[i];
                if (rec[pass][b] >= a.threshold) {
                    chosen = b;
                    cls = pass == 0 ? RF_TEMPORAL : RF_SPATIAL;
                }
            }
        a.head_class[bh] = cls;
        if (a.head_bw) a.head_bw[bh] = chosen;
        if (a.recalls)
            for (int pass = 0; pass < 2; ++pass)
                for (int b = 0; b < n_bw; ++b) a.recalls[(bh * 2 + pass) * n_bw + b] = rec[pass][b];
    }
}

template <int D>
static int launch_arm_d(const ArmArgs& a, hipStream_t st) {
    const bool both = a.pass[0].n == a.pass[1].n && a.pass[0].stride == a.pass[1].stride;  // one sample for the two passes
    const int NW = both ? kArmWavesBoth : kArmWavesApart;
    const int nQB = (a.max_n + 32 * NW - 1) / (32 * NW);
    const int total = nQB * (both ? 1 : 2) * a.BH;
    const dim3 grid(8 * ((total + 7) / 8)), block(64 * NW);
    constexpr int lds_both = ArmSmem<D, kArmWavesBoth>::BYTES, lds_apart = ArmSmem<D, kArmWavesApart>::BYTES;
    if (both)
        hipLaunchKernelGGL((arm_recall_kernel<D, true>), grid, block, lds_both, st, a, nQB);
    else
        hipLaunchKernelGGL((arm_recall_kernel<D, false>), grid, block, lds_apart, st, a, nQB);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return static_cast<int>(e);
    hipLaunchKernelGGL(arm_finish_kernel, dim3(a.BH), dim3(256), 0, st, a);
    return static_cast<int>(hipGetLastError());
}

// Scratch for callers that cannot allocate (rf_arm_classify_noalloc): lives in the library's image on
// every GPU the library runs on, at an address that differs from device to device.
static __device__ __align__(256) unsigned char scratch[kArmStaticScratchBytes];

int arm_static_scratch(void** ptr, size_t* bytes) {
    constexpr int kMaxDevices = 64;
    static std::mutex mu;
    static void* address[kMaxDevices] = {};
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return static_cast<int>(e);
    if (dev < 0 || dev >= kMaxDevices) return static_cast<int>(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(mu);
    if (!address[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));  // with device `dev` current: that device's copy
        if (e != hipSuccess) return static_cast<int>(e);
        address[dev] = p;
    }
    *ptr = address[dev];
    *bytes = kArmStaticScratchBytes;
    return 0;
}

int launch_arm(const ArmArgs& a, int D, void* stream) {
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (D == 64) return launch_arm_d<64>(a, st);
    if (D == 96) return launch_arm_d<96>(a, st);
    if (D == 128) return launch_arm_d<128>(a, st);
    return static_cast<int>(hipErrorInvalidValue);
}

}  // namespace rf
