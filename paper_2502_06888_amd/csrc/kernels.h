// Internal interface between the C-ABI host code and the HIP kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kmoe {

constexpr int kLanes = 64;
constexpr int kRowBlk = 32;        // rows (tokens) per MFMA block
constexpr int kTileBlks = 8;       // row blocks per tile (256 rows)
constexpr int kPlanChunk = 1024;   // assignments per block of the dispatch kernels
constexpr int kMaxExperts = 256;
constexpr int kMaxTopK = 8;
constexpr int kMaxBatches = 64;

// Capacity of the tile tables for a context.
inline int max_tiles_for(int max_rowblks, int E, int S, int max_tokens) {
    return max_rowblks / kTileBlks + E + S * ((max_tokens + kTileBlks * kRowBlk - 1) / (kTileBlks * kRowBlk) + 1) + 1;
}

struct BatchOffsets {
    int32_t n;
    int32_t v[kMaxBatches + 1];
};

// Device pointers of one context's dispatch plan (all inside the caller's workspace).
struct PlanPtrs {
    int32_t* topk_idx;    // [A]
    float* topk_w;        // [A]
    int32_t* counts;      // [E]
    int32_t* offsets;     // [E+1]
    int32_t* poff;        // [E+1]  32-padded row offsets by expert id
    int32_t* nbatch;      // [E]
    int32_t* exec_order;  // [E]
    int32_t* meta;        // [0] n_active  [1] n_tiles  [2] routed row blocks  [3] n_tokens
    int32_t* perm;        // [A]
    int32_t* inv_perm;    // [A]
    int32_t* blk_counts;  // [nchunks][E]
    int32_t* blk_base;    // [nchunks][E]
    unsigned long long* blk_mask;  // [nchunks][E]
    int32_t* tile_expert; // [max_tiles]   expert id (E+s for shared)
    int32_t* tile_xblk;   // [max_tiles]   first row block in the packed activations
    int32_t* tile_hblk;   // [max_tiles]   first row block in H / O
    int32_t* tile_nblk;   // [max_tiles]   row blocks in this tile (1..8)
    int32_t* exp_tile0;   // [E+S] first tile of an expert
    int32_t* exp_ntiles;  // [E+S]
    int32_t* blk_expert;  // [max_rowblks] routed expert owning a row block
    int32_t* mail;        // [2E+1] counts, exec_order, n_active: the host's mailbox (pinned, written by the plan)
};

struct Shape {
    int32_t N, d, f, E, k, S;
    int32_t renorm;
    int32_t max_rowblks;   // capacity of the routed padded-row space, in row blocks
};

// ---- router -------------------------------------------------------------------------------
void launch_router(hipStream_t st, int dtype, const void* x, const void* wg, const Shape& s,
                   float* logits_out, int32_t* idx_out, float* w_out);

// ---- dispatch plan ------------------------------------------------------------------------
void launch_plan(hipStream_t st, const Shape& s, const BatchOffsets& bo, const PlanPtrs& p,
                 int max_tiles);

// ---- bf16 path ----------------------------------------------------------------------------
// Offline packing of one expert (W1,W3 [f,d]; W2 [d,f]) into the fragment-ordered blob.  The
// down section holds W2 * w2_scale as fp16 (w2_scale a power of two chosen from launch_w2_stats).
void launch_pack_expert_bf16(hipStream_t st, const void* w1, const void* w3, const void* w2,
                             int d, int f, void* blob, float w2_scale);
// out2[0] = bits of max |w2|, out2[1] = bits of the largest row sum of squares; out2 zeroed by the caller.
void launch_w2_stats(hipStream_t st, const void* w2, int d, int f, uint32_t* out2);
void launch_zero_u64(hipStream_t st, unsigned long long* p, size_t n);
// The same for a 4-bit group-quantised expert: codes [rows, cols/2] (even column in the low
// nibble), scales and zero points [rows, cols/64] as bf16, for W1, W3 ([f, d]) and W2 ([d, f]).
// w2_scale (a power of two) multiplies the scales of W2's groups, so that the dequantised weights
// fit the fp16 range of the down projection (launch_w2_stats_q4 gives the range).
void launch_pack_expert_q4(hipStream_t st, const uint8_t* q1, const uint16_t* s1, const uint16_t* z1,
                           const uint8_t* q3, const uint16_t* s3, const uint16_t* z3, const uint8_t* q2,
                           const uint16_t* s2, const uint16_t* z2, int d, int f, void* blob, float w2_scale);
// As launch_w2_stats for a 4-bit W2 [d, f]: the dequantised weights bf16(fma(code, s, -z*s)).
void launch_w2_stats_q4(hipStream_t st, const uint8_t* q2, const uint16_t* s2, const uint16_t* z2, int d, int f,
                        uint32_t* out2);
// Gather token rows per expert (and the plain rows for shared experts) into fragment order.
// Also zeroes herr (remainder energy per H row of this call).
void launch_gather_bf16(hipStream_t st, const void* x, const Shape& s, const PlanPtrs& p,
                        void* xp, unsigned long long* herr);

constexpr int kMaxLaunchGroup = 8;  // streamed experts whose tiles one launch may cover

struct FfnArgs {
    const uint8_t* const* wtab;  // device table: blob of expert id e (may hold nulls for streamed)
    const uint8_t* w_single;     // non-null: use this blob for every tile of the launch
    const uint8_t* w_group[kMaxLaunchGroup];  // n_group > 0: blobs (window slots) of the experts group_expert[i];
    int32_t group_expert[kMaxLaunchGroup];    // any other expert of the launch is looked up in wtab
    int32_t n_group;
    const void* act;             // packed activations (Xp for up, Hp for down)
    void* out;                   // Hp (up) or O partials (down)
    const int32_t* tile_expert;
    const int32_t* tile_xblk;
    const int32_t* tile_hblk;
    const int32_t* tile_nblk;
    const int32_t* tile_first;   // device: index of the first tile of this launch (null = tile_first_v)
    const int32_t* tile_count;   // device: number of tiles of this launch (null = tile_count_v)
    int32_t tile_first_v, tile_count_v;  // the same by value, from the host's mirror of the tile tables
    int32_t max_tiles;           // tiles the grid was sized for
    int32_t est_tiles;           // tiles the host expects to be live (launch-shape heuristic)
    int32_t d, f;
    int32_t h_mode;              // H travels as an fp16 value plane + an fp16 remainder plane.  0: the remainder
                                 // is multiplied only by tiles whose recorded remainder energy asks for it;
                                 // 1: always
    int64_t h_plane_units;       // 16-byte units between the value plane and the remainder plane of H
    unsigned long long* herr;    // per H row: remainder energy in units of threshold / 2^20 (h_mode 0)
    const float2* wmeta;         // per expert of the layer: (output scale of the down projection, 1 / threshold)
    int32_t* sat_count;          // device counters: [0] H values clamped to the fp16 range, [1] down-projection
                                 // workgroups that multiplied the remainder plane on their own finding (h_mode 0)
    int32_t variant;             // kernel shape (waves per workgroup x units per wave); 0 = default
    int32_t panel;               // full tiles: 1 + log2 of the tiles per panel of the workgroup order (0 = default)
    int32_t full_tiles;          // host estimate: most tiles are full (more than 160 rows per expert)
    int32_t weight_bits;         // 0/16: bf16 weights; 4: 4-bit codes in groups of 64 with (s, z)
    int32_t split_k;             // down projection only
    int64_t o_split_stride;      // elements between split-K partials of O
};
void launch_ffn_up_bf16(hipStream_t st, const FfnArgs& a);
void launch_ffn_down_bf16(hipStream_t st, const FfnArgs& a);
void launch_corr_update(hipStream_t st, const int32_t* idx_prev, const int32_t* idx_cur, int N, int k,
                        int E, int32_t* table);
int ffn_configure();  // one-time function attributes (dynamic LDS); returns hipError_t

// Y[t] = sum_j w[t,j] * sum_s O[s][row(t,j)] + shared rows; one rounding to the output type.
void launch_combine(hipStream_t st, int out_dtype, const Shape& s, const PlanPtrs& p,
                    const float* o, int split_k, int64_t o_split_stride, void* y);

// ---- f32 path (plain row-major blobs: W1 | W3 | W2) ------------------------------------------
void launch_pack_expert_f32(hipStream_t st, const void* w1, const void* w3, const void* w2, int d,
                            int f, void* blob);
void launch_ffn_f32(hipStream_t st, const float* x, const Shape& s, const PlanPtrs& p,
                    const uint8_t* const* wtab, const uint8_t* w_single, int32_t only_expert,
                    float* h, float* o);

}  // namespace kmoe
