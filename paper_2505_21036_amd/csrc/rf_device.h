// Device-side building blocks shared by the attention and ARM kernels (gfx950 only).
//
// Both kernels form score tiles TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16_bf16:
// the A operand is a 32-key x 16-channel slab of K read from LDS, the B operand a
// 16-channel x 32-query slab of Q held in registers.  In the 32x32 fp32 result a lane
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

// One K tile (kTileK keys x D channels, bf16) staged through registers into padded LDS rows.
template <int D, int NT>
struct KTile {
    static constexpr int ROW_BYTES = 2 * D + 16;  // +16 B pad: conflict-free 16-B reads down a column
    static constexpr int BYTES = kTileK * ROW_BYTES;
    static constexpr int CHUNKS = kTileK * D / 8;  // 16-byte pieces
    static constexpr int PER_THREAD = (CHUNKS + NT - 1) / NT;
    u32x4 reg[PER_THREAD];

    // row_token(r) gives the token whose K row goes to tile row r (already clamped in range)
    template <typename F>
    __device__ __forceinline__ void fetch(const uint16_t* base, int tid, F row_token) {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int c = tid + i * NT;
            if (CHUNKS % NT == 0 || c < CHUNKS) {
                const int row = c / (D / 8), col = c % (D / 8);
                reg[i] = *reinterpret_cast<const u32x4*>(base + static_cast<size_t>(row_token(row)) * D + col * 8);
            }
        }
    }
    __device__ __forceinline__ void stash(unsigned char* lds, int tid) const {
#pragma unroll
        for (int i = 0; i < PER_THREAD; ++i) {
            const int c = tid + i * NT;
            if (CHUNKS % NT == 0 || c < CHUNKS) {
                const int row = c / (D / 8), col = c % (D / 8);
                *reinterpret_cast<u32x4*>(lds + row * ROW_BYTES + col * 16) = reg[i];
            }
        }
    }
    // A operand of S^T = K Q^T: keys 32*kb2 .. +31 (permuted per lane), channels 16*c + 8*hf .. +7
    static __device__ __forceinline__ bf16x8 frag(const unsigned char* lds, int kb2, int c, int m, int hf) {
        const int row = 32 * kb2 + key_of_mfma_row(m);
        return as_bf16x8(*reinterpret_cast<const u32x4*>(lds + row * ROW_BYTES + 32 * c + 16 * hf));
    }
};

// Q operand (B of S^T = K Q^T) for one lane: row `token`, channels 16*c + 8*hf .. +7.
template <int D>
__device__ __forceinline__ void load_q_frags(const uint16_t* base, int token, int hf, bf16x8 (&qf)[D / 16]) {
#pragma unroll
    for (int c = 0; c < D / 16; ++c)
        qf[c] = as_bf16x8(*reinterpret_cast<const u32x4*>(base + static_cast<size_t>(token) * D + 16 * c + 8 * hf));
}

// S^T tile (64 keys x 32 queries per wavefront) = two 32x32 MFMA blocks.
template <int D, int NT>
__device__ __forceinline__ void score_tile(const unsigned char* kl, const bf16x8 (&qf)[D / 16], int m, int hf,
                                           f32x16 (&s)[2]) {
#pragma unroll
    for (int kb2 = 0; kb2 < 2; ++kb2) {
        f32x16 acc = {0};
#pragma unroll
        for (int c = 0; c < D / 16; ++c)
            acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(KTile<D, NT>::frag(kl, kb2, c, m, hf), qf[c], acc, 0, 0, 0);
        s[kb2] = acc;
    }
}

}  // namespace rf
