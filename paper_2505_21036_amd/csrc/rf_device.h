// Device-side building blocks shared by the attention and ARM kernels (gfx950 only).
//
// Both kernels form score tiles TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the A operand is a 32-key x 16-channel slab of K read from LDS (DirectTile below), the B operand
// a 16-channel x 32-query slab of Q held in registers.  In the 32x32 fp32 result a lane
// owns ONE query (column lane%32) and 16 keys, so the row statistics of the softmax
// (running maximum, running sum) are per-lane scalars and need a single exchange
// between the two 32-lane halves of the wavefront.
#pragma once
#include <hip/hip_runtime.h>

#include "rf_internal.h"

namespace rf {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

// MFMA result register r of lane half hf holds matrix row 8*(r/4) + 4*hf + r%4.  Letting the
// lane that feeds matrix row m read key  swap_bits23(m)  makes register r of half hf hold key
// 16*(r/8) + 8*hf + r%8: eight consecutive keys per half, which is exactly the operand
// layout the second MFMA (P V) wants, so P never leaves registers.
__device__ __forceinline__ int key_of_mfma_row(int m) {
    return (m & 0x13) | ((m & 8) >> 1) | ((m & 4) << 1);
}
__device__ __forceinline__ int key_of_reg(int r, int hf) { return 16 * (r >> 3) + 8 * hf + (r & 7); }

__device__ __forceinline__ bf16x8 as_bf16x8(u32x4 v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// acc + lo + hi of a packed pair of bf16 values, in fp32 (v_dot2c_f32_bf16 against {1, 1})
__device__ __forceinline__ float add_bf16_pair(float acc, uint32_t pair) {
    const bf16x2 ones = {static_cast<__bf16>(1.0f), static_cast<__bf16>(1.0f)};
    return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, pair), ones, acc, false);
}

__device__ __forceinline__ float other_half(float x) { return __shfl_xor(x, 32, 64); }

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Workgroup id -> logical work item such that each of the 8 XCDs (which take workgroup ids
// round-robin) walks one contiguous range of items, so neighbouring query blocks of one
// head share K/V through that XCD's L2.  Returns -1 for padding workgroups.
__device__ __forceinline__ int xcd_contiguous_item(int wg, int total) {
    const int chunk = (total + 7) >> 3;
    const int item = (wg & 7) * chunk + (wg >> 3);
    return ((wg >> 3) < chunk && item < total) ? item : -1;
}

// Q operand (B of S^T = K Q^T) for one lane: row `token`, channels 16*c + 8*hf .. +7.
template <int D>
__device__ __forceinline__ void load_q_frags(const uint16_t* base, int token, int hf, bf16x8 (&qf)[D / 16]) {
#pragma unroll
    for (int c = 0; c < D / 16; ++c)
        qf[c] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + static_cast<size_t>(token) * D + 16 * c + 8 * hf));
}

typedef short s16x4 __attribute__((ext_vector_type(4)));

// MFMA operand reads from LDS are issued this many MFMAs ahead of their use (K: one 16-byte read per
// operand; V: two transposing 8-byte reads per operand).
#ifndef RF_AHEAD_K
#define RF_AHEAD_K 4
#endif
#ifndef RF_AHEAD_V
#define RF_AHEAD_V 3
#endif
constexpr int kAheadK = RF_AHEAD_K, kAheadV = RF_AHEAD_V;

// A 64-key tile of K and of V in LDS, filled by global_load_lds (global -> LDS without staging
// registers) and read back as MFMA operands.
//
// A wavefront load instruction fills 1 KiB of consecutive LDS, lane l bytes 16*l .. 16*l+15, so
// rows are unpadded; bank conflicts are avoided by permuting, per row, which 16-byte chunk of the
// row a slot holds, which costs nothing because every lane chooses its own global address.  K is
// read back 16 bytes per lane as the A operand of S^T = K Q^T; V stays row-major [key][channel]
// and ds_read_b64_tr_b16 transposes it on the way out into the A operand of O^T = V^T P^T
// (8 consecutive keys of one channel per lane).
//
// Chunk permutations (chunk = 16 bytes = 8 channels; a row has CH = D/8 of them):
//   K: the 16 lanes of a read phase take one chunk index from 16 different rows; they must hit 16
//      different 16-byte bank groups.  head_dim 128 / 64: slot = chunk ^ X(row), X = row % 16, resp.
//      (row / 2) % 8.  head_dim 96 (12 chunks, rows start 48 banks apart): slot = (chunk + (row/4) % 4) mod 12.
//   V: the 32 lanes of a transposing read phase take one 64-byte block from 4 consecutive rows;
//      head_dim 128 / 64: slot = chunk ^ 4*(row % 4), resp. ^ 4*((row/2) % 2); head_dim 96 needs
//      none, its 192-byte rows already rotate through the four 64-byte bank groups.
template <int D, int NW>
struct DirectTile {
    static_assert(D == 64 || D == 96 || D == 128, "unsupported head_dim");
    static constexpr bool POW2 = D != 96;
    static constexpr int NT = 64 * NW, CH = D / 8, ROW = 2 * D;
    static constexpr int K_BYTES = kTileK * ROW, V_BYTES = kTileK * ROW;
    static constexpr int SEGS = kTileK * CH / 64;  // 1 KiB segments per tile
    static constexpr int V_READS_PER_FRAG = 2;
    static constexpr int PER_WAVE = (SEGS + NW - 1) / NW;  // load instructions per tensor per thread (at most)
    static constexpr bool EVEN = SEGS % NW == 0;           // else the last round is taken by the first wavefronts only

    static __device__ __forceinline__ int k_slot(int row, int chunk) {
        if (D == 128) return chunk ^ (row & 15);
        if (D == 64) return chunk ^ ((row >> 1) & 7);
        const int p = chunk + ((row >> 2) & 3);
        return p >= CH ? p - CH : p;
    }
    static __device__ __forceinline__ int k_chunk(int row, int slot) {  // inverse of k_slot
        if (POW2) return k_slot(row, slot);
        const int ch = slot - ((row >> 2) & 3);
        return ch < 0 ? ch + CH : ch;
    }
    static __device__ __forceinline__ int v_slot(int row, int chunk) {  // its own inverse
        if (D == 128) return chunk ^ (4 * (row & 3));
        if (D == 64) return chunk ^ (4 * ((row >> 1) & 1));
        return chunk;
    }

    static __device__ __forceinline__ uint32_t lds_offset(const unsigned char* p) {
        return static_cast<uint32_t>(reinterpret_cast<uintptr_t>((__attribute__((address_space(3))) const unsigned char*)p));
    }
    // One 16-byte-per-lane load from  base + lane offset  into LDS at  lds_addr + 16*lane (lds_addr
    // wavefront-uniform, handed over in M0); completion is awaited in wait_landed().
    //
    // Written as inline assembly rather than with the compiler's builtin on purpose: while a builtin
    // LDS load is in flight the compiler's wait-count insertion treats it as a pending access to both
    // memories and degrades every LDS wait in the loop to "all outstanding" (lgkmcnt(0)), and it puts
    // a full vmcnt(0) in front of the transposing LDS reads, which rules out keeping a second tile in
    // flight.  Here the waits are explicit instead.  M0 is otherwise unused by the generated code of
    // this file (a host-side test inspects the assembly for that); the wait state the hardware needs
    // between the write of M0 and the load is the s_nop.
    static __device__ __forceinline__ void dma16(const unsigned char* base, uint32_t lane_off, uint32_t lds_addr) {
        const unsigned char* p = base + lane_off;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(p) : "memory", "m0");
    }

    int wave, lane;
    int k_base;          // byte offset of this lane's K operand for kb2 = 0 (chunk 0 of its row when !POW2)
    int k_rot;           // !POW2: hf + rotation of this lane's K row
    int v_base;          // byte offset of this lane's V operand for u = 0, first half, channel block 0
    // Loads of a tile of consecutive tokens: load j of a lane reads  base + j*STEP + lane_off[j].
    // With power-of-two rows a lane keeps its slot position and moves down ROWS_PER_LOAD rows per
    // load, and the permutations have period 16 (K) and 4 (V) rows, so one offset serves every j
    // (K: only if a load covers a multiple of 16 rows); 12-chunk rows need an offset per load.
    static constexpr int ROWS_PER_LOAD = 64 * NW / CH;
    static constexpr int STEP = POW2 ? ROWS_PER_LOAD * ROW : 0;
    static constexpr int K_VARIANTS = (POW2 && ROWS_PER_LOAD % 16 == 0) ? 1 : PER_WAVE;
    static constexpr int V_VARIANTS = POW2 ? 1 : PER_WAVE;
    static_assert(!POW2 || ROWS_PER_LOAD % 4 == 0, "V row permutation must not change between loads");
    uint32_t k_lane_off[K_VARIANTS], v_lane_off[V_VARIANTS];

    __device__ __forceinline__ void init(int tid) {
        lane = tid & 63;
        wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        const int hf = lane >> 5, m = lane & 31, g4 = lane >> 4, i = lane & 15;
        const int krow = key_of_mfma_row(m);  // + 32*kb2: invisible to the K permutation
        k_base = POW2 ? krow * ROW + 16 * k_slot(krow, hf) : krow * ROW;
        k_rot = hf + ((krow >> 2) & 3);
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int slot = min((j * NW + wave) * 64 + lane, kTileK * CH - 1), row = slot / CH, pos = slot % CH;
            if (j < K_VARIANTS) k_lane_off[j] = row * ROW + 16 * k_chunk(row, pos) - j * STEP;
            if (j < V_VARIANTS) v_lane_off[j] = row * ROW + 16 * v_slot(row, pos) - j * STEP;
        }
        // V operand of channel block db: chunk 4*db + r of row vrow (+ 16*u + 4*half: multiples of 4,
        // invisible to the V permutation).  With the XOR permutation the chunk lands in slot
        // 4*(db ^ y) + r, i.e. at v_base ^ 64*db; unpermuted (head_dim 96) at v_base + 64*db.
        const int vrow = 8 * hf + (i >> 2);
        const int chunk0 = 2 * (g4 & 1) + ((i & 3) >> 1);
        v_base = vrow * ROW + 16 * v_slot(vrow, chunk0) + 8 * (i & 1);
    }

    // tok(row): token whose K/V row goes to tile row `row`; kh/vh: byte pointers the tokens index.
    // WITH_V = false: K only (the ARM needs no V); WITH_K = false: V only (the attention loop for 64-row
    // wavefronts loads the K and V of different tiles).
    template <bool WITH_V = true, bool WITH_K = true, typename F>
    __device__ __forceinline__ void issue(const unsigned char* kh, const unsigned char* vh, unsigned char* kl,
                                          unsigned char* vl, F tok) {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int seg = j * NW + wave;
            if (!EVEN && seg >= SEGS) break;
            const int slot = seg * 64 + lane, row = slot / CH, pos = slot % CH;
            const uint32_t row_off = static_cast<uint32_t>(tok(row)) * ROW;
            if (WITH_K) dma16(kh, row_off + 16u * k_chunk(row, pos), lds_offset(kl) + seg * 1024);
            if (WITH_V) dma16(vh, row_off + 16u * v_slot(row, pos), lds_offset(vl) + seg * 1024);
        }
    }
    // same for a tile of 64 consecutive tokens starting at kh / vh
    template <bool WITH_V = true, bool WITH_K = true>
    __device__ __forceinline__ void issue_consecutive(const unsigned char* kh, const unsigned char* vh, unsigned char* kl,
                                                      unsigned char* vl) {
#pragma unroll
        for (int j = 0; j < PER_WAVE; ++j) {
            const int seg = j * NW + wave;
            if (!EVEN && seg >= SEGS) break;
            if (WITH_K) dma16(kh + j * STEP, k_lane_off[j % K_VARIANTS], lds_offset(kl) + seg * 1024);
            if (WITH_V) dma16(vh + j * STEP, v_lane_off[j % V_VARIANTS], lds_offset(vl) + seg * 1024);
        }
    }
    // load instructions per tensor and tile this wavefront issues (the first SEGS % NW wavefronts take the odd round)
    __device__ __forceinline__ int loads_per_tensor() const { return EVEN ? PER_WAVE : (SEGS / NW + (wave < SEGS % NW ? 1 : 0)); }
    // Loads land in issue order.  A tile is in LDS once all but the loads issued after its own have
    // landed (the barrier that follows publishes it): LATER = how many whole tiles were issued after
    // it.  Every wavefront issues at least MIN_LOADS_PER_TILE loads per tile.
    static constexpr int MIN_LOADS_PER_TILE = 2 * (SEGS / NW);  // K and V; callers that load K only wait for all
    template <int LATER>
    static __device__ __forceinline__ void wait_landed() {
        static_assert(LATER * MIN_LOADS_PER_TILE < 64, "vmcnt is a 6-bit counter");
        asm volatile("s_waitcnt vmcnt(%0)" ::"n"(LATER * MIN_LOADS_PER_TILE) : "memory");
    }

    // The same wait with a wavefront-uniform run-time count: all but the newest n loads have landed.
    static __device__ __forceinline__ void wait_all_but(int n) {
        switch (n) {
            case 1: asm volatile("s_waitcnt vmcnt(1)" ::: "memory"); break;
            case 2: asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); break;
            case 3: asm volatile("s_waitcnt vmcnt(3)" ::: "memory"); break;
            case 4: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
            case 5: asm volatile("s_waitcnt vmcnt(5)" ::: "memory"); break;
            case 6: asm volatile("s_waitcnt vmcnt(6)" ::: "memory"); break;
            case 7: asm volatile("s_waitcnt vmcnt(7)" ::: "memory"); break;
            case 8: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
            default: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
        }
    }

    // Per-tile LDS addresses of this lane's operands.  Both are made opaque once per tile, so that what
    // the loop carries is one K and one V register per lane rather than a hoisted register per
    // (chunk, channel block): the tile buffers start at multiples of 256 bytes, so the XORs that
    // select a chunk commute with adding the buffer's address.
    __device__ __forceinline__ uint32_t k_address(const unsigned char* kl) const {
        uint32_t ka = lds_offset(kl) + k_base;
        asm volatile("" : "+v"(ka));
        return ka;
    }
    __device__ __forceinline__ uint32_t v_address(const unsigned char* vl) const {
        uint32_t va = lds_offset(vl) + v_base;
        asm volatile("" : "+v"(va));
        return va;
    }
    // A operand of S^T = K Q^T: keys 32*kb2 .. +31 (permuted per lane), channels 16*c + 8*hf .. +7
    __device__ __forceinline__ bf16x8 k_frag(uint32_t ka, int kb2, int c) const {
        typedef __attribute__((address_space(3))) u32x4 lds_u32x4;
        uint32_t addr;
        if (POW2) {
            addr = ka ^ (32 * c);  // chunk 2c + hf: the permutation is an XOR, so c toggles address bits
        } else {
            const int p = 2 * c + k_rot;
            addr = ka + 16 * (p >= CH ? p - CH : p);
        }
        return as_bf16x8(*(lds_u32x4*)(uintptr_t)(addr + kb2 * 32 * ROW));
    }
    // S^T of one tile (64 keys x this lane's query) = two 32x32 MFMA blocks, the two 32-key halves as
    // independent accumulation chains taken in turn.  Operand reads run AHEAD MFMAs ahead of their use;
    // the fences keep the compiler's scheduler from undoing that order (left to itself it sometimes
    // issues read, wait, MFMA, read, wait, ...).
    template <int AHEAD>
    __device__ __forceinline__ void scores(uint32_t ka, const bf16x8 (&qf)[D / 16], f32x16 (&s)[2]) const {
        constexpr int NQK = 2 * (D / 16);
        bf16x8 frag[NQK];
#pragma unroll
        for (int i = 0; i < AHEAD; ++i) frag[i] = k_frag(ka, i & 1, i >> 1);
        s[0] = f32x16{0};
        s[1] = f32x16{0};
#pragma unroll
        for (int j = 0; j < NQK; ++j) {
            if (j + AHEAD < NQK) frag[j + AHEAD] = k_frag(ka, (j + AHEAD) & 1, (j + AHEAD) >> 1);
            s[j & 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(frag[j], qf[j >> 1], s[j & 1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    // A operand of O^T = V^T P^T: channels 32*db + lane%32, keys 16*u + 8*hf .. +7
    static __device__ __forceinline__ bf16x8 v_frag(uint32_t va, int db, int u) {
        typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
        const uint32_t p = (POW2 ? va ^ (64 * db) : va + 64 * db) + 16 * u * ROW;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(p));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)(uintptr_t)(p + 4 * ROW));
        typedef short s16x8 __attribute__((ext_vector_type(8)));
        const s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
        return __builtin_bit_cast(bf16x8, v);
    }
};

}  // namespace rf
