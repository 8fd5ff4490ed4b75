// Internal interface between the attention layer's C-ABI host code and its HIP kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kattn {

constexpr int kRowBlk = 32;   // rows (sequences) per MFMA block
constexpr int kMaxSplit = 16; // split-K partials of a projection, at most

// Fragment order (shared by activations and weights): a [rows, K] bf16 matrix is cut into
// units of 32 rows x 16 reduction steps; unit (rb, s) is 1 KiB at ((rb * K/16) + s) * 64 lanes
// x 16 bytes; lane l holds row rb*32 + l%32, elements s*16 + (l/32)*8 .. +8.

struct Dims {
    int32_t d, Hq, Hkv, hd;
    int32_t max_len;
};

// The batches one launch serves, passed by value as a kernel argument: batch b owns the rows
// row0[b] .. row0[b+1]-1 of the activation buffers, its sequences hold pos[b] cached positions.
constexpr int kMaxGroup = 64;
struct GroupTab {
    int32_t n;
    int32_t row0[kMaxGroup + 1];
    int32_t pos[kMaxGroup];
    const void* h_in[kMaxGroup];
    void* h_out[kMaxGroup];
    void* kc[kMaxGroup];        // [n_seq, Hkv, max_len, hd] bf16
    void* vc[kMaxGroup];
    void* new_rows[kMaxGroup];  // [2, n_seq, Hkv, hd] bf16 or null
};

// W [rows, K] row-major bf16 -> fragment order at `out` (rows multiple of 32, K multiple of 16).
void launch_pack_weight(hipStream_t st, const void* w, int rows, int K, void* out);

// xn = x / sqrt(mean(x^2) + eps) * g as bf16 in fragment order for all rows of the table; the
// padding rows of the last row block are not written.
void launch_rmsnorm(hipStream_t st, const GroupTab& tab, const void* g, int d, float eps, void* a_frag);

// out[sp][row][col] (fp32, row stride n_out) = A[rows, K] . W[n_out, K]^T over split sp of K.
// row_blocks = ceil(rows / 32); the A buffer must hold row_blocks rounded up to the row tile.
void launch_proj(hipStream_t st, const void* a_frag, const void* w_frag, int row_blocks, int K,
                 int n_out, int splits, float* out, int64_t split_stride);
int pick_row_tile(int row_blocks);                 // row blocks per wavefront (1, 2 or 4)
int pick_splits(int row_blocks, int K, int n_out); // split-K factor the launcher should be given

// Sums the split-K partials of the fused q|k|v projection, rotates q and k to position pos,
// writes q (fp32, [rows, Hq, hd], already multiplied by log2(e)/sqrt(hd)), the new k and v rows as
// bf16 into each batch's caches at its position and into its `new_rows` (when not null).
void launch_qkv_finish(hipStream_t st, const float* part, int splits, int64_t split_stride,
                       const Dims& dm, const GroupTab& tab, const double* inv_freq, float* q);

// Softmax attention of the new token of every sequence over its batch's cache positions 0..pos;
// output as bf16 in fragment order ([rows, Hq*hd] as the A operand of the output projection).
int launch_attention(hipStream_t st, const float* q, const Dims& dm, const GroupTab& tab, void* o_frag);

// y = x + sum of the split-K partials of the output projection, one rounding to bf16.
void launch_out_finish(hipStream_t st, const float* part, int splits, int64_t split_stride,
                       const GroupTab& tab, int d);

}  // namespace kattn
