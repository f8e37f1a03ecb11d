// Internal declarations shared by the host side of the library and its kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace ca {

constexpr int kMaxSeqsPerLaunch = 64;  // per-conversation arguments travel in the kernel-argument block
constexpr int kPageSize = 16;
constexpr int kXcds = 8;               // MI355X: 8 accelerator dies, workgroup i runs on die i % 8

// ---------------------------------------------------------------------------------------
// paged pool <-> contiguous rows (Section 3.2: layer-wise load / save are data movement)
// ---------------------------------------------------------------------------------------
// One entry per conversation handled by a launch.  "contig" is [token][n_kv_heads][head_dim];
// token (contig_tok0 + i) <-> context token (ctx_tok0 + i) for i < count.
struct MoveArgs {
    uint8_t *contig_k[kMaxSeqsPerLaunch];
    uint8_t *contig_v[kMaxSeqsPerLaunch];
    int64_t contig_tok0[kMaxSeqsPerLaunch];
    int32_t ctx_tok0[kMaxSeqsPerLaunch];
    int32_t count[kMaxSeqsPerLaunch];
    int32_t seq[kMaxSeqsPerLaunch];  // row of the block table
};

// Second contiguous destination of a launch that writes what it reads twice (the new turn's K/V go into the pool AND
// to the tier in one pass): token (contig_tok0 + i) of the source also lands at token (dst2_tok0 + i) of dst2.
struct MoveArgs2 {
    uint8_t *dst2_k[kMaxSeqsPerLaunch];
    uint8_t *dst2_v[kMaxSeqsPerLaunch];
    int64_t dst2_tok0[kMaxSeqsPerLaunch];
};

constexpr int kMoveUnroll = 2;   // 16-byte loads in flight per lane of the move kernel (one pass = kMoveUnroll*256 vectors)

struct MoveShape {
    const int32_t *block_table;  // device [n_seqs][max_pages]
    int32_t max_pages;
    int32_t n_kv_heads;
    int32_t vecs_per_row;        // head_dim * esize / 16
    int32_t heads_per_wg;        // heads one workgroup moves (grid.x slices the heads, and K/V)
    int32_t n_in_launch;
    int32_t max_pages_touched;   // largest number of pages a range of this launch touches
    int32_t max_grid_y;          // 0: one workgroup row per page; > 0: at most this many rows, each walking several pages
                                 // (a kernel that stores over the host link is bound by the link and should hold few compute units)
};

// to_pool = true: contiguous -> pages (unpack / append); false: pages -> contiguous (pack).
hipError_t launch_move(bool to_pool, const MoveArgs &args, const MoveShape &shape, uint8_t *k_pool,
                       uint8_t *v_pool, hipStream_t stream);
// contiguous -> pages as launch_move(true, ...), and every vector is also stored to the second destination
hipError_t launch_move_dual(const MoveArgs &args, const MoveArgs2 &second, const MoveShape &shape, uint8_t *k_pool,
                            uint8_t *v_pool, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Section 3.4: per-token metadata of the rebased plan
// ---------------------------------------------------------------------------------------
struct RebaseArgs {
    int32_t n_seqs;
    int32_t max_pages;
    const int32_t *block_table;  // device
    const int32_t *n_keep;       // device [n_seqs]
    const int32_t *cu_q;         // device [n_seqs+1]
    const int32_t *cu_k;         // device [n_seqs+1]
    int32_t *q_pos;              // device [sum new]
    int32_t *q_seq;              // device [sum new]
    int32_t *slot_map;           // device [sum context]
    int32_t total_q, total_k;
};
hipError_t launch_rebase(const RebaseArgs &args, hipStream_t stream);

// ---------------------------------------------------------------------------------------
// Sections 2.1 / 3.1 / 3.4: attention of the new tokens over [kept history | new tokens]
// ---------------------------------------------------------------------------------------
struct WorkItem {      // one tile of stacked query rows of one (conversation, kv head)
    int32_t seq;       // -1: padding, the workgroup exits
    int32_t kv_head;
    int32_t row0;      // first stacked row; row r <-> new token r / G, query head kv_head*G + r % G
    int32_t n_rows;
    int32_t key_begin; // the item's share of the keys: [key_begin, min(key_end, what its rows see));
    int32_t key_end;   // the whole range unless the row tile was split; cuts are multiples of 64
    int32_t part;      // -1: the item writes `out`; else index of its share in the partial-result buffer
    int32_t reserved;
};

struct CombineItem {   // a row tile whose keys were split: shares first_part .. first_part + n_parts - 1
    int32_t seq, kv_head, row0, n_rows;
    int32_t first_part, n_parts;
    int32_t reserved[2];
};

struct AttnArgs {
    const uint16_t *q;       // bf16 bits
    uint16_t *out;
    const uint16_t *k_pool;
    const uint16_t *v_pool;
    const int32_t *block_table;
    const int32_t *n_keep;
    const int32_t *cu_q;
    const int32_t *q_pos;    // [total_q] rebased position of every new token
    const int32_t *q_seq;    // [total_q] its conversation
    const WorkItem *items;
    const CombineItem *combine;   // row tiles to merge after the walk (n_combine of them)
    float *partial;          // shares of split row tiles: per part [tile_rows][head_dim] sums, [tile_rows] maxima,
                             // [tile_rows] denominators (fp32)
    const float2 *rope;      // [max_positions][head_dim/2] (cos, sin)
    // keys rotated once per batch and layer instead of in every row tile (prerotate != 0):
    uint16_t *k_rot;             // scratch copy of the keys, dense pages [n_dense_pages][n_kv_heads][16][head_dim]
    uint16_t *v_t;               // scratch copy of the values, same pages, each block transposed (pipelined != 0 only)
    const int32_t *rot_nvalid;   // [n_dense_pages] context tokens in the page (16 except a conversation's last page)
    int32_t pipelined;            // the scratch copies have the layouts of ca_attn_pp.hip and its kernel runs
    const int32_t *dense_page0;  // [n_seqs] first dense page of a conversation
    const int32_t *rot_src_page; // [n_dense_pages] pool page a dense page is rotated from
    const int32_t *rot_pos0;     // [n_dense_pages] position of its first token
    int32_t n_dense_pages;
    int32_t prerotate;
    int32_t max_positions;
    int32_t n_items;
    int32_t n_combine;
    int32_t total_q;
    int32_t max_pages;
    int32_t n_q_heads, n_kv_heads, head_dim;
    int32_t rope_style;
    int32_t tile_rows;       // stacked query rows per workgroup: 128 (4 wavefronts) or 256 (8)
    float softmax_scale;
};

constexpr int kAttnTileRowsMin = 128;   // smallest tile of stacked query rows (4 wavefronts x 32)
constexpr int kRopeMinRows = 256;       // the kernels read table rows below this whatever the window

hipError_t launch_attn_ref(const AttnArgs &args, hipStream_t stream);
hipError_t launch_attn_dma(const AttnArgs &args, hipStream_t stream);
// head_dim 128, 256-row tiles, keys rotated and values transposed once per layer into scratch copies; inside every
// wavefront the matrix instructions of one key tile are pipelined with the softmax of the previous one
hipError_t launch_attn_pp(const AttnArgs &args, hipStream_t stream);
// merges the shares of split row tiles (args.combine) into args.out; used by every kernel that writes shares
hipError_t launch_attn_combine(const AttnArgs &args, hipStream_t stream);
// decode steps: every item has at most kAttnDecodeMaxRows stacked rows starting at row 0; streams K/V through
// registers instead of matrix-core tiles
constexpr int kAttnDecodeMaxRows = 2;
hipError_t launch_attn_decode(const AttnArgs &args, int max_rows, hipStream_t stream);
constexpr int kAttnMaxParts = 1024;           // shares of split row tiles per batch (sizes the partial-result buffer)
constexpr int kAttnMaxPartsPerTile = 16;
constexpr int kAttnMinPartKeys = 256;         // a share is at least this many keys

}  // namespace ca
