// Internal device-side types and launcher prototypes of the LSH path of libaif (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace aif {

constexpr int LSH_BLOCK = 256;          // candidates per scheduling block
constexpr int LSH_TCHUNK = 512;         // history items whose user-side sums one block forms (more for a long history)
constexpr int LSH_MAX_CHUNKS = 64;      // chunks of one history at most
// Chunk length of a history of L items: LSH_TCHUNK times the smallest whole factor that keeps the chunks within
// LSH_MAX_CHUNKS -- every chunk's partial sums (2 d' d floats) are written to memory and read back, which a history of
// 10^5 items would otherwise do 196 times.  A function of the request's own history only, like everything that
// decides the order of its sums.
__host__ __device__ inline int lsh_chunk_len(int L)
{
    const int chunks = (L + LSH_TCHUNK - 1) / LSH_TCHUNK;
    return LSH_TCHUNK * ((chunks + LSH_MAX_CHUNKS - 1) / LSH_MAX_CHUNKS > 1 ? (chunks + LSH_MAX_CHUNKS - 1) / LSH_MAX_CHUNKS : 1);
}
__host__ __device__ inline int lsh_chunks(int L)
{
    const int len = lsh_chunk_len(L);
    return (L + len - 1) / len;
}
constexpr int LSH_MAX_TIERS = 8;

struct LshReqDesc {
    const uint8_t *seq_sigs;
    const void *seq_emb;
    const int32_t *cand_ids;
    float *din_out;
    int32_t *tier_out;
    int32_t seq_len;
    int32_t n_cand;
    int32_t cand_base;          // first candidate slot of this request in the batch (multiple of LSH_BLOCK)
    int32_t index;
};

struct LshBatch {
    const LshReqDesc *reqs;     // device, [n_req]
    const int32_t *blk_req;     // device, [n_blk]: request owning each block of LSH_BLOCK candidate slots
    int32_t n_req;
    int32_t n_blk;
};

struct LshModel {
    int64_t n_items;
    int32_t d_bits, d_out, n_tiers;
    int32_t dtype;              // storage of U~: 0 fp32, 1 bf16
    int32_t tier_mul;           // ceil(2^20 / d_bits): (x * tier_mul) >> 20 == x / d_bits for x <= 2048
};

// a2 of this path -- per request and chunk of the history:
// part[r][chunk][s][k][j] = sum over the chunk's t with bit k of signature t equal to s of U~[t][j]   (s = 0, 1)
// (grid_chunks: chunks of the longest history in the batch; max_chunks: chunk stride of `part`)
hipError_t launch_lsh_user_partial(const LshModel &m, const LshBatch &b, int grid_chunks, int max_chunks, float *part,
                                   hipStream_t s);
// A[r][s][k][j] = sum of the partial sums over the chunks, in chunk order
hipError_t launch_lsh_user_reduce(const LshModel &m, const LshBatch &b, int max_chunks, const float *part, float *A,
                                  hipStream_t s);
// Eq. 8: din[i][j] = (1 / d') sum_k A[b_ik][k][j]
hipError_t launch_lsh_din(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, const float *A, int32_t *bad,
                          hipStream_t s);
// Eq. 8 on the matrix cores (d a multiple of 32 up to 128): the candidates' bits one-hot against the tables cut into three
// bf16 pieces.  pieces: workspace of lsh_din_pieces_stride() 16-byte pieces per request, written by the launch itself.
bool lsh_din_on_mfma(const LshModel &m);
size_t lsh_din_pieces_stride(const LshModel &m);
hipError_t launch_lsh_din_mfma(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, const float *A, void *pieces,
                               int32_t *bad, hipStream_t s);
// Eq. 6, 7, 9: equal-bit counts against every history item, counted into tiers
hipError_t launch_lsh_simtier(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, hipStream_t s);
// The same with the equal-bit counts formed on the matrix cores (signatures of 32, 64 or 128 bits; 2 d' / N a power of
// two up to 256).  hist: workspace of lsh_hist_stride() 16-byte pieces per request, written by the launch itself (the
// history signatures as the matrix instruction's operand); longest: the longest history of the batch; parts: workspace
// of lsh_simtier_parts_bytes() for the partial counts of a batch too small to fill the chip uncut.
bool lsh_simtier_on_mfma(const LshModel &m);
size_t lsh_hist_stride(const LshModel &m, int max_seq_len);
size_t lsh_simtier_parts_bytes();
hipError_t launch_lsh_simtier_mfma(const LshModel &m, const LshBatch &b, const uint8_t *sig_table, void *hist, size_t req_stride,
                                   int longest, void *parts, hipStream_t s);

}  // namespace aif
