// Host-side launchers of the gfx950 kernels (internal to the library; the
// public boundary is include/allocmoe.h).  Every pointer is a device pointer.
// Launchers only enqueue; they return hipGetLastError() of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace allocmoe {

// rows per tile of the grouped-GEMM tile map written by the plan kernel
constexpr int kTileRowsSmall = 32;

// tile_info layout: [0] = number of tiles; [1] = how many of them, at the end of the
// list, are the only tile of an expert with at most 64 rows; entry i at
// [kTileHdr + 4*i]: expert, first row, rows in tile, number of tiles of this expert.
//
// An expert's rows are split evenly over its ceil(rows / bm) tiles, so the tiles
// of one expert cost the same.  Experts are listed by decreasing rows per tile
// (ties: expert ascending), an expert's tiles next to each other: a launch that
// takes tiles in this order starts with its longest workgroups and ends on its
// cheapest, and neighbouring tiles mostly read the same expert's weights.
constexpr int kTileHdr = 4;
inline size_t tile_info_ints(int64_t max_tiles) { return kTileHdr + 4 * static_cast<size_t>(max_tiles); }

// ---- route.hip
hipError_t launch_route(int dtype, const void* X, const void* Wg, const float* bias,
                        const void* w_sg, int T, int d, int E, int K, float* scores,
                        int32_t* topk_ids, float* topk_s, float* sgate, hipStream_t stream);
// bf16 gate GEMM on the matrix cores from the re-tiled gate matrix
// (kGateBlocks 16-column blocks: 64 expert columns + the shared-gate column)
constexpr int kGateBlocks = 5;
inline size_t gate_packed_elems(int d) { return static_cast<size_t>(kGateBlocks) * 16 * d; }
hipError_t launch_route_mfma(const void* X, const void* gate_packed, const float* bias,
                             bool with_gate, int T, int d, int E, int K, float* scores,
                             int32_t* topk_ids, float* topk_s, float* sgate, hipStream_t stream);
hipError_t launch_pack_gate(const void* Wg, const void* w_sg, int d, int E, void* out,
                            hipStream_t stream);
hipError_t launch_topk_from_scores(const float* scores, int T, int E, int K, int32_t* topk_ids,
                                   float* topk_s, hipStream_t stream);

// ---- plan.hip
// keys of the alternative selectors (mode: allocmoe_selector, 1 or 2) from the sorted
// candidate scores [T,K]
hipError_t launch_selector_keys(const float* topk_s, int T, int K, int mode, float* keys,
                                hipStream_t stream);
// From kPlanSpreadTokens tokens on, selection and dispatch run as a sequence of launches
// over many workgroups; the selection then needs plan_spread_bytes(T) bytes of device
// scratch (`spread`, 256-byte aligned; null: one workgroup does the work, whatever T).
// Every launch of the sequence costs 5-10 us whatever its size (a chain of dependent
// memory round trips), five of them 42 us at 8192 tokens and 36 us at 4096, against 82 us
// and 50 us for the single workgroup; at 2048 tokens both take 32 us.
// `alone`: nothing else wants the compute units while the plan runs; below the spread
// size the one launch then has several workgroups that repeat the selection and share
// out the placement (beside other work extra workgroups would only queue behind it).
constexpr int kPlanSpreadTokens = 4096;
size_t plan_spread_bytes(int T);
hipError_t launch_select(const float* topk_s, int T, int K, int Kb, int64_t B,
                         int32_t* keep_count, void* spread, hipStream_t stream);
hipError_t launch_dispatch(const int32_t* topk_ids, const int32_t* keep_count, int T, int K,
                           int E, int64_t B, int32_t* expert_offsets, int32_t* row_token,
                           int32_t* row_rank, int32_t* inv_row, uint64_t* words, int32_t* prefix,
                           int bm, int32_t* tile_info, bool alone, hipStream_t stream);
hipError_t launch_plan(const float* topk_s, const int32_t* topk_ids, int T, int K, int Kb,
                       int64_t B, int E, int32_t* keep_count, int32_t* expert_offsets,
                       int32_t* row_token, int32_t* row_rank, int32_t* inv_row, uint64_t* words,
                       int32_t* prefix, int bm, int32_t* tile_info, void* spread, bool alone,
                       hipStream_t stream);

// ---- ffn_f32.hip : C = A B (or silu(A B1) * (A B3)) over row tiles, fp32, row-major B
// A rows are taken through row_map when it is not null.  With tile_info null the
// rows 0..M_dense-1 form one group (group 0).  B1/B3: [G][Kd][N].
hipError_t launch_ffn_f32(bool swiglu, const float* A, int lda, const int32_t* row_map,
                          const float* B1, const float* B3, int Kd, int N,
                          const int32_t* tile_info, int64_t max_tiles, int M_dense, float* C,
                          int ldc, hipStream_t stream);

// ---- ffn_bf16.hip : the same contraction on the matrix cores from packed weights
// One group of row tiles: A rows (through row_map when not null) times packed
// B.  With tile_info null the rows 0..M_dense-1 form one group.  A == nullptr
// marks an absent group.
struct StreamGroup {
    const void* A = nullptr;
    int lda = 0;
    const int32_t* row_map = nullptr;
    const void* Bp = nullptr;
    size_t group_stride = 0;   // elements between consecutive experts in Bp
    int Kd = 0, N = 0;
    const int32_t* tile_info = nullptr;
    int64_t max_tiles = 0;
    int M_dense = 0;
    void* C = nullptr;
    int ldc = 0;
    int64_t n_wg = 0;          // filled by the launcher
    int xr = 1;                // dense group: XCDs along the row tiles (filled by the launcher)
    int dense_rows = 256;      // dense group, tile kernel: rows per tile (filled by the launcher)
    // 8-bit weights: Bp holds E4M3 codes, one byte per element
    // (group_stride in bytes), and scale[g][stream][n] the fp32 scale of every output
    // column (stream: W1, W3 for the SwiGLU half; one for the plain half)
    const float* scale = nullptr;
};
// routed experts' tiles and the shared expert's tiles in one launch
hipError_t launch_ffn_bf16_stream(bool swiglu, StreamGroup routed, StreamGroup shared,
                                  hipStream_t stream);

// Register-blocked 256 x 256 tile kernel for prefill-shaped groups (tile map with
// kTileRowsLarge rows per tile): weights straight from global memory into
// registers, activations through LDS; needs Kd % 128 == 0 and N % 128 == 0
// (swiglu) or N % 256 == 0 (plain).
constexpr int kTileRowsLarge = 256;
hipError_t launch_ffn_bf16_t256(bool swiglu, StreamGroup routed, StreamGroup shared,
                                hipStream_t stream);

// ---- pack.hip : row-major [G][Kd][N] bf16 -> MFMA fragment order
// 8-bit variant: per output column a scale (max |w| / 448, 1 for a zero column) and E4M3
// codes of w / scale (nearest, ties to even mantissa, saturating), in fragments of
// 32 k x 32 n: lane l holds 16 bytes, k = 32 kb + 8 (l/32) + i in bytes i = 0..7 and
// k = 32 kb + 16 + 8 (l/32) + i in bytes 8 + i, column 32 nb + l%32.  Destination of
// fragment (g, nb, kb): out + g*group_stride + nb*nblock_stride + base_off + kb*1024
// (bytes).  scale_out[g*scale_stride + n].
hipError_t launch_pack_b_fp8(const void* W, int G, int Kd, int N, void* out, size_t group_stride,
                             size_t nblock_stride, size_t base_off, float* scale_out,
                             size_t scale_stride, hipStream_t stream);
hipError_t launch_pack_b(const void* W, int G, int Kd, int N, void* out,
                         size_t group_stride_elems, size_t nblock_stride_elems,
                         size_t base_off_elems, hipStream_t stream);

// ---- stats.hip : routing analytics; metrics: 5 floats (see allocmoe_routing_metrics)
hipError_t launch_routing_stats(const float* scores, const int32_t* topk_ids, const float* topk_s,
                                const int32_t* keep_count, int T, int E, int K,
                                int32_t* load_orig, int32_t* load_kept, float* wload_orig,
                                float* wload_kept, float* token_entropy, int32_t* entropy_rank2,
                                float* metrics, hipStream_t stream);

// ---- combine.hip : y_t = sum_j s[t,j] O[inv_row[t,j]] + g_t Os[t]
hipError_t launch_combine(int dtype, const void* O, const void* Os, const int32_t* inv_row,
                          const float* topk_s, const int32_t* keep_count, const float* sgate,
                          int T, int d, int K, void* Y, hipStream_t stream);

}  // namespace allocmoe
