// Internal declarations shared by the host side (argument checks, block lists) and the
// HIP kernels of the RainFusion library.  Not part of the public ABI.
#pragma once
#include <cstddef>
#include <cstdint>
#include <vector>

#include "rainfusion.h"

namespace rf {

constexpr int kTileK = 64;  // keys per LDS tile of the attention and ARM kernels
constexpr int kMaxBw = RF_MAX_BANDWIDTHS;  // candidate bandwidths of the per-head bandwidth variant

// Flags on a key-tile entry of a block list (RF_PLAN_PARTIAL is public).
constexpr int32_t kTileBoundary = 0x20000000;  // tile holds text keys or runs past the last key
constexpr int32_t kTileIndexMask = 0x1fffffff;

// Resolved, validated problem description.
struct Geometry {
    int T, H, W, text_len;
    int HW, Nv, N;
    int r_spatial, r_temporal;  // band half-widths in frames / in-frame positions
    int tau;                    // checkerboard stride (Eq. 4)
    int omega;                  // global sampling interval (Sec. 3.3)
    int two_head;               // ARM fallback class is DENSE instead of TEXTURAL
    int text_first;             // text tokens are the first rows of the tensors instead of the last

    // Lists, attributes and orders are all built on the WALKED order: video tokens 0 .. Nv-1, then
    // text.  row_of() gives the tensor row of a walked index (the identity unless text_first).
    int video_shift() const { return text_first ? text_len : 0; }  // added to a walked video index
    int text_shift() const { return text_first ? -Nv : 0; }        // added to a walked text index
    int row_of(int n) const { return n + (n < Nv ? video_shift() : text_shift()); }
};

// Lists: 0/1/2 = Spatial / Temporal / Textural in token order; 3 = Temporal in POSITION-MAJOR
// order (video token (frame f, position p) sits at p*T + f, text tokens stay last), where the
// Temporal band |p_i - p_j| <= r is one contiguous run of keys per query block.
constexpr int kLists = 4;
constexpr int kListTemporalPM = 3;

// Host copy of everything the attention kernel needs besides the tensors.
struct HostPlan {
    Geometry g;
    int block;     // query rows per block (64 or 128) = rows one workgroup owns
    int nQB;       // ceil(N / block)
    int nKT;       // ceil(N / kTileK): key tiles of the token sequence
    int Nc;        // compacted key count of the Textural pattern: kept video keys + text keys
    int nCT;       // ceil(Nc / kTileK): key tiles of the compacted sequence
    int first_text_qb;  // first query block holding a text row (nQB if there is none)
    // CSR lists of key tiles per query block; Textural: text-holding query blocks only
    std::vector<int32_t> row_ptr[kLists], cols[kLists];
    // Scheduling of a head's query blocks (affects cache behaviour only, never the result), per list:
    // qorder = the order in which blocks are handed out (a permutation; XCD x takes ordinals
    // [x * ceil(nQB/8), (x+1) * ceil(nQB/8)) of it), first_entry = the entry of its list a block starts
    // its (cyclic) walk at.
    std::vector<int32_t> qorder[kLists];
    std::vector<int32_t> first_entry[kLists];
    // per row of the list's order: frame index / in-frame index / 0 if kept by Eq. 4 else 1 / in-frame index
    std::vector<int32_t> attr[kLists];
    std::vector<int32_t> cidx;      // compacted position -> tensor row (Textural)
    std::vector<int32_t> pm_token;  // position-major row -> tensor row
};

// Fills g from layout/params (params may be null -> paper defaults). Returns an rf_status.
int resolve_geometry(const rf_layout* layout, const rf_params* params, Geometry* g);

// Builds the block lists. Pure host code.
void build_plan(const Geometry& g, int block, HostPlan* plan);

// Block list of one class as the kernel walks it (see rf_plan_host in rainfusion.h).
void flatten_class(const HostPlan& plan, int cls, std::vector<int32_t>* row_ptr, std::vector<int32_t>* cols);

// Device-resident plan: raw device pointers into one allocation.
struct DevicePlan {
    const int32_t* row_ptr[kLists];
    const int32_t* cols[kLists];
    const int32_t* attr[kLists];
    const int32_t* qorder[kLists];
    const int32_t* first_entry[kLists];
    const int32_t* cidx;
    const int32_t* pm_token;
    int radius[kLists];
    int video_shift, text_shift;  // tensor row = walked index + (index < Nv ? video_shift : text_shift)
    int N, Nv, Nc;
    int block, nQB, nKT, nCT, first_text_qb;
};

// All plans of one call share the layout and the checkerboard; they differ in the band widths.
struct AttnArgs {
    const uint16_t* Q;
    const uint16_t* K;
    const uint16_t* V;
    uint16_t* O;
    const int32_t* head_class;  // null: every head dense
    int BH;            // B * nH
    float scale_log2;  // log2(e) / sqrt(D)
    // optional: packed copies of K and V, [BH][N][D] each: the kept rows of Textural heads (first Nc rows),
    // all rows of Temporal heads in position-major order; null: no packing
    uint16_t* packed_k;
    uint16_t* packed_v;
    const int32_t* head_bw;  // optional per-head index into plan[]; null or out of range: plan[0]
    int* queue;              // 8 work-queue counters and 8 sweep words (one each per XCD) at the start of the caller's workspace, reset by the launcher
    int wide_rows;           // 1: wavefronts of 64 query rows (256-row blocks only)
    int join_sweep;          // 1: a starting item joins the tile walk of the workgroups already running on its XCD; 0: fixed start
    int n_plans;
    DevicePlan plan[kMaxBw];
};

// One ARM pass = one (sampling, mask) pair: sample a -> video token a * stride, whose attribute is its
// in-frame position (token mod HW) or its frame (token div HW); the mask keeps |attr[a] - attr[b]| <= radius.
struct ArmPass {
    int by_frame;         // 0: attribute = in-frame position (Temporal mask), 1: attribute = frame (Spatial mask)
    int n;                // number of samples
    int stride;           // token stride between samples
    int HW;               // tokens per frame
    int radius[kMaxBw];   // one band half-width per candidate bandwidth
};

struct ArmArgs {
    const uint16_t* Q;
    const uint16_t* K;
    int BH, N;
    int first_video_row;  // tensor row of video token 0
    float scale_log2;
    ArmPass pass[2];   // 0: Temporal mask (R_hat), 1: Spatial mask (R_tilde)
    int n_bw;          // candidate bandwidths (1 for plain Alg. 1)
    int by_width[kMaxBw];  // candidate indices from the narrowest bandwidth to the widest
    float* row_recall; // device [BH][2][n_bw][max_n]
    int max_n;
    float threshold;
    int fallback_class;   // class of a head that matches neither mask
    int32_t* head_class;  // device [BH]
    int32_t* head_bw;     // device [BH] or null: chosen candidate index, -1 for Textural heads
    float* recalls;       // device [BH][2][n_bw] or null
};

// Kernel launchers (defined in the .hip files). Return a hipError_t as int.
int launch_attention(const AttnArgs& a, int D, void* stream);
int launch_pack_textural(const AttnArgs& a, int D, void* stream);
int launch_arm(const ArmArgs& a, int D, void* stream);
// Device address and size of the library's static scratch array on the current device (rf_arm.hip).
int arm_static_scratch(void** ptr, size_t* bytes);
constexpr size_t kArmStaticScratchBytes = RF_ARM_STATIC_SCRATCH_BYTES;

}  // namespace rf
