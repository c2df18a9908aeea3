// Internal device-side types and launcher prototypes of the user-side network of libaif (gfx950 only).
#pragma once
#include "aif_dev.h"

namespace aif {

constexpr int USER_PROJ_ROWS = 32;      // rows of one projection block
constexpr int USER_FFN_ROWS = 64;       // positions of one FFN / pooling block

// One user of a call.  Its rows in the workspace X (row-major, [q | a], 2 d wide): rows
// row_base .. row_base + seq_len - 1 are the projected sequence positions, row row_base + seq_len is the
// projected profile -- one more query of the same attention over the same sequence (Eq. 3 is Eq. 2's
// attention with the profile in the place of a position).
struct UserDesc {
    const void *profile;
    const void *seq;
    void *user_vec_out;
    void *seq_out;
    int32_t seq_len;
    int32_t row_base;           // multiple of ROW_BLOCK
};

struct UserWeights {
    const float *wseq_t;        // [d_raw, d] fp32: W_seq transposed
    const float *wprof;         // [d, d_raw] fp32: W_profile as given (row-major)
    const float *wffn_t;        // [d, d]
    const float *b_ffn;         // [d] or null
    int32_t d_raw, d, dtype;
    // bf16 MFMA variants of the projection and the FFN (d = 32, 64 or 128, d_raw a multiple of 16): the
    // weights as A fragments, [row tile][k-step][lane][8], as pack_frag lays them out; null = not used
    const void *wseq_frag, *wffn_frag;
    int32_t part_rows;          // positions summed into one partial of the pooling (USER_FFN_ROWS, or 32 with MFMA)
};

// Eq. 1: X[row, 0:d] = W x for every sequence position and the profile; U^_seq also to the user's seq_out.
hipError_t launch_user_project(const UserWeights &w, const UserDesc *users /*device*/, const int32_t *blk_req /*device*/,
                               int n_blk, void *X, hipStream_t s);
size_t user_project_lds_bytes(int d_raw);

// FFN of Eq. 2 on the attention rows X[row, d:2d] of the sequence positions and their sum over each block of
// USER_FFN_ROWS positions: part[(row / USER_FFN_ROWS), 0:d].
hipError_t launch_user_ffn_partial(const UserWeights &w, const UserDesc *users, const int32_t *blk_req, int n_blk,
                                   const void *X, float *part, hipStream_t s);
size_t user_ffn_lds_bytes(int d);

// Pooling of Eq. 2 (mean of the partial sums, in block order) and the combined vector
// [U_self_attention | U_profile_attention] to each user's user_vec_out.
hipError_t launch_user_combine(const UserWeights &w, const UserDesc *users, int n_users, const void *X, const float *part,
                               hipStream_t s);

}  // namespace aif
