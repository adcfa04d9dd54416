// bf16 expert networks on the matrix cores for prefill-shaped layers (Section
// 3.1: one feed-forward execution per selected pair), fp32 accumulation:
//   H = silu(A W1) * (A W3)   (SWIGLU)    or    O = A W2,   both stored as bf16.
//
// Register-blocked 256 x 256 tile on 4 waves (one per SIMD, all 512 registers).
//
// A workgroup owns <= 256 rows of one expert times 128 SwiGLU columns (128 of
// W1 and the same 128 of W3) or 256 columns of W2.  Wave w owns 64 of those
// weight columns (two 32-column MFMA fragments: W1|W3 of the same columns, or
// two neighbouring W2 blocks) times every 32-row block of the tile: up to
// 8 x 2 accumulators of 32x32, 256 registers.
//
//  * The weights never pass through LDS: they were re-tiled once into MFMA
//    B-fragment order, a wave is the only consumer of its columns, so each lane
//    loads its 16 bytes per fragment straight from global memory (1 KB
//    contiguous per wave-load) into a ring of 8 fragment pairs (8 k16 steps =
//    128 k ahead of use).
//  * The activation rows go global -> LDS directly (no VGPR staging) into a ring
//    of 4 slots of 256 rows x 64 k; lanes 8r..8r+7 fetch the eight 16-byte
//    chunks of row r (one 128-byte line per row), XOR-swizzled so that every
//    MFMA A-operand read is one conflict-free ds_read_b128.  Loads run three
//    slots ahead; one workgroup barrier per 64 k.
//  * Per 16 k a wave issues 2*NRB MFMAs for NRB LDS reads + 2 global loads, so a
//    tile with fewer than 256 rows costs in proportion to its 32-row blocks.
//  * 8-bit weights (E4M3 codes with one fp32 scale per output column): a lane's
//    16-byte load holds its fragments of two k16 steps, so the ring of 8 loads per
//    stream reaches 16 steps ahead (as many bytes in flight as with bf16) and a
//    loop pass covers 16 steps; the codes are widened to bf16 (exactly) right
//    before the MFMAs that use them and the column scales multiply the fp32 sums
//    in the epilogue.
#include <algorithm>
#include <type_traits>

#include "common.hpp"
#include "kernels.hpp"

namespace allocmoe {

namespace {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));

constexpr int kRows = kTileRowsLarge;   // rows per tile
constexpr int kStepK = 64;              // contraction elements per ring slot
constexpr int kSlots = 4;
constexpr int kWaves = 4;
constexpr int kSlotBytes = kRows * kStepK * 2;
constexpr int kXcds = 8;                // accelerator dies (one L2 each) of an MI355X
constexpr int kBRing = 8;               // 16-byte units of weight fragments held per stream (k16 steps with bf16)
constexpr int kBRingDeep = 24;          // the same for tiles of at most kLightRowBlocks row blocks
constexpr int kLightRowBlocks = 2;


// 8 rows x 128 B of activations, global -> LDS directly: lane l's 16 bytes land
// at lds_addr + 16 l (M0 holds the wave-uniform LDS base; one idle state between
// writing M0 and the load that reads it).  Written as asm, hidden from the
// compiler's wait-count insertion: it treats a direct-to-LDS load as touching
// both memory paths and then drains *all* outstanding loads (vmcnt(0)) at the
// next use of any loaded register, which would serialise the weight prefetch.
// Hidden, these loads still count in vmcnt, in issue order: every wait the
// compiler emits for a weight register is then stricter than needed, never
// weaker, and the waits for the slots themselves are written by hand.
__device__ __forceinline__ void load_rows_to_lds(const bf16x8* g, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off"
                 :
                 : "v"(g), "s"(lds_addr)
                 : "memory", "m0");
}

// Workgroup barrier without the memory fence of __syncthreads(): the fence
// would wait for every outstanding load, i.e. also for the prefetched slots.
// What a step needs is awaited explicitly (vmcnt) before the barrier.
__device__ __forceinline__ void wg_barrier_nofence() {
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt_le() {
    // s_waitcnt with expcnt/lgkmcnt unconstrained; vmcnt is bits [3:0] and [15:14]
    __builtin_amdgcn_s_waitcnt(0x0F70 | (N & 15) | ((N >> 4) << 14));
}

// 8 E4M3 codes (byte i = element i) -> 8 bf16 values, exactly
__device__ __forceinline__ bf16x8 widen_fp8x8(uint2 q) {
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
    const bf16x2 p0 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q.x, 1.0f, false);
    const bf16x2 p1 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q.x, 1.0f, true);
    const bf16x2 p2 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q.y, 1.0f, false);
    const bf16x2 p3 = __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(q.y, 1.0f, true);
    const u32x4 w = {__builtin_bit_cast(uint32_t, p0), __builtin_bit_cast(uint32_t, p1),
                     __builtin_bit_cast(uint32_t, p2), __builtin_bit_cast(uint32_t, p3)};
    return __builtin_bit_cast(bf16x8, w);
}

// b0, b1: the wave's two weight streams (bf16 fragments, or with FP8 the codes: a lane's
// 16 bytes per 32 k hold its fragment of the even k16 step, then of the odd one);
// sc0, sc1: with FP8 the scales of the 32 columns of each stream.
template <bool SWIGLU, int NRB, bool STREAM_ONCE, bool FP8, int RING>
__device__ __forceinline__ void t256_body(char* lds, const bf16_t* A, size_t lda,
                                          const int32_t* row_map, const void* b0,
                                          const void* b1, const float* sc0, const float* sc1,
                                          int KT, int wave, int lane, int row0,
                                          int rows, int nt, void* C, int ldc) {
    f32x16 acc[NRB][2];
#pragma unroll
    for (int i = 0; i < NRB; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = f32x16{0};

    // A: per slot, wave w stages rows 32 i + 8 w .. + 7 of every row block i that
    // holds real rows (NRB wave-loads): lane 8 r + p fetches the chunk that belongs
    // at position p of row r.  Rows past the tile's end re-read its last row (in
    // bounds, never stored).
    const bf16x8* arow[NRB];
#pragma unroll
    for (int i = 0; i < NRB; ++i) {
        const int R = 32 * i + 8 * wave + lane / 8;
        const int my_row = row0 + min(R, rows - 1);
        const long src = row_map ? row_map[my_row] : my_row;
        arow[i] = reinterpret_cast<const bf16x8*>(A + static_cast<size_t>(src) * lda) +
                  ((lane % 8) ^ ((R >> 1) & 7));
    }
    const uint32_t lds_wave = __builtin_amdgcn_readfirstlane(
        static_cast<uint32_t>(reinterpret_cast<uintptr_t>(lds)) + wave * 1024);
    auto issue_a = [&](int s, int slot) {
#pragma unroll
        for (int i = 0; i < NRB; ++i)
            load_rows_to_lds(arow[i] + s * (kStepK / 8), lds_wave + slot * kSlotBytes + i * 4096);
    };
    typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;
    i32x4 breg[RING][2];
    // Weight fragments come through buffer loads: a scalar descriptor per stream
    // (base, size), the lane's offset in a VGPR and the k16 step's offset in an SGPR,
    // so a load costs no address arithmetic on the vector unit; a step past the end
    // of the stream reads zeros instead of faulting.  Weights that no other tile
    // reads are marked non-temporal: they need not displace what the caches hold
    // for tiles that share theirs.
    const int stream_bytes = KT * kStepK * 32 * (FP8 ? 1 : 2);
    const __amdgpu_buffer_rsrc_t rs0 = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(b0), 0, stream_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs1 = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<void*>(b1), 0, stream_bytes, 0x00020000);
    const int lane_off = lane * 16;
    // ring entry r <- 16-byte unit q of both streams (bf16: k16 step q; FP8: steps 2q, 2q+1)
    auto load_b = [&](int q, int r) {
        constexpr int kAux = STREAM_ONCE ? 2 : 0;   // nt
        breg[r][0] = __builtin_amdgcn_raw_buffer_load_b128(rs0, lane_off, q * 1024, kAux);
        breg[r][1] = __builtin_amdgcn_raw_buffer_load_b128(rs1, lane_off, q * 1024, kAux);
    };
    // A operand of row block i, k16 chunk kc of a slot: lane l reads row m = l%32 of
    // the block, 16-byte chunk c = 2 kc + l/32 of that row, stored at position
    // c ^ ((m/2) % 8) of the row's 128 bytes.
    const int m = lane % 32, sw = (m >> 1) & 7;
    int a_off[4];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) a_off[kc] = (m * 8 + ((2 * kc + lane / 32) ^ sw)) * 16;
    auto read_a = [&](int slot, int kc, bf16x8 (&a)[NRB]) {
        const char* base = lds + slot * kSlotBytes + a_off[kc];
#pragma unroll
        for (int i = 0; i < NRB; ++i) a[i] = *reinterpret_cast<const bf16x8*>(base + i * (32 * 128));
    };
    // The weight fragment is the first MFMA operand and the activation fragment the
    // second, i.e. the unit forms the transposed 32x32 block: register r of lane l then
    // holds the output of token row l%32 at column 8*(r/4) + 4*(l/32) + r%4, four
    // consecutive columns per register quad, which the epilogue stores as one 8-byte
    // word of bf16.
    // this wave's two weight fragments of step u of a loop pass
    auto weights_of = [&](int u, bf16x8 (&b)[2]) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            if constexpr (FP8) {
                const i32x4 q = breg[u / 2][j];
                b[j] = widen_fp8x8((u & 1) ? uint2{static_cast<uint32_t>(q[2]), static_cast<uint32_t>(q[3])}
                                           : uint2{static_cast<uint32_t>(q[0]), static_cast<uint32_t>(q[1])});
            } else {
                b[j] = __builtin_bit_cast(bf16x8, breg[u][j]);
            }
        }
    };
    // step u of a loop pass
    auto multiply = [&](const bf16x8 (&a)[NRB], int u) {
        bf16x8 b[2];
        weights_of(u, b);
#pragma unroll
        for (int i = 0; i < NRB; ++i) {
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0], a[i], acc[i][0], 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[1], a[i], acc[i][1], 0, 0, 0);
        }
    };

    // the same, with the loads of activation slot `slot` (k step sl) between the MFMAs
    auto multiply_and_issue = [&](const bf16x8 (&a)[NRB], int u, int sl, int slot) {
        bf16x8 b[2];
        weights_of(u, b);
#pragma unroll
        for (int i = 0; i < NRB; ++i) {
            acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[0], a[i], acc[i][0], 0, 0, 0);
            acc[i][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b[1], a[i], acc[i][1], 0, 0, 0);
            __builtin_amdgcn_sched_barrier(0);
            load_rows_to_lds(arow[i] + sl * (kStepK / 8), lds_wave + slot * kSlotBytes + i * 4096);
            __builtin_amdgcn_sched_barrier(0);
        }
    };

    // Load schedule.  Per k16 step u (8 per loop pass = 2 slots): the step's MFMAs,
    // then 2 loads refilling its weight registers for step u + 8 (the compiler
    // inserts the waits for those registers); after the barrier behind the third
    // k16 of a slot additionally NRB loads refilling the slot used one step ago with
    // the slot three ahead (issued between the MFMAs of the fourth k16, before that
    // step's weight loads).  Slot s+1 is awaited after the third k16 of slot s: it
    // was issued two slots earlier, followed by 2 + (6 + NRB + 2) + 6 loads -> kWaitA.
    // The prologue issues slot 0 and then exactly the sequence of one loop pass
    // (weights of steps 0-2, slot 1, steps 3-6, slot 2, step 7), so that count
    // holds from the first pass on.  Loads past the end of the contraction re-read
    // the last step (in bounds, never multiplied) or, for the weights, read zeros
    // past the end of the buffer, which keeps the count uniform.
    // FP8: 16 steps per pass (4 slots), 2 weight loads after every second step (the
    // ring entry both steps used, refilled for 16 steps later); between the loads of
    // slot s+1 and the wait for it: 2 + (2 + NRB + 2) + 2.  The prologue keeps that
    // count by placing the surplus weight loads before slot 1.
    // A deeper ring (RING k16 steps, bf16 only) changes nothing in these counts: the loads
    // of slot j sit right before the weight loads of step 4 j - 9 + RING in the steady
    // state, and so they do in the prologue.  At most 63 loads can be outstanding per wave
    // (2 RING + 3 NRB here), which bounds RING for the row-block counts that use it.
    static_assert(!FP8 || RING == 8, "8-bit weights: ring of 8 units = 16 steps");
    static_assert(2 * RING + 3 * NRB <= 63, "outstanding loads per wave");
    constexpr int kPass = FP8 ? 16 : RING;
    constexpr int kWaitA = FP8 ? 8 + NRB : 16 + NRB;
    issue_a(0, 0);
#pragma unroll
    for (int r = 0; r < RING; ++r) {
        load_b(r, r);
        if (r == (FP8 ? 4 : RING - 6)) issue_a(min(1, KT - 1), 1);
        if (r == RING - 2) issue_a(min(2, KT - 1), 2);
    }
    wait_vmcnt_le<2 * RING + 2 * NRB>();   // slot 0 has landed (this wave's part)
    wg_barrier_nofence();
    bf16x8 af[2][NRB];
    read_a(0, 0, af[0]);

    // steps [4 s2, 4 s2 + STEPS) of the contraction
    auto pass = [&](int s2, auto steps_const) {
        constexpr int STEPS = decltype(steps_const)::value;
#pragma unroll
        for (int u = 0; u < STEPS; ++u) {
            const int s = s2 + u / 4, kc = u % 4;
            __builtin_amdgcn_sched_barrier(0);
            __builtin_amdgcn_sched_barrier(0);
            // next step's A fragments are read under the first MFMAs of this step
            if (kc < 3)
                read_a(s & 3, kc + 1, af[(u + 1) & 1]);
            else
                read_a((s + 1) & 3, 0, af[(u + 1) & 1]);
            if (kc == 3) {
                // the loads of the slot three ahead (its predecessor was released by the
                // barrier of the step before) go out between this step's MFMAs, one row
                // block's after the two MFMAs of that row block: issued as one run behind
                // the barrier they leave the matrix unit idle for ~40 instructions
                const int sl = min(s + 3, KT - 1), slot = (s + 3) & 3;
                multiply_and_issue(af[u & 1], u, sl, slot);
            } else {
                multiply(af[u & 1], u);
#pragma unroll
                for (int i = 0; i < NRB; ++i) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);   // one MFMA
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);   // one LDS read
                }
                __builtin_amdgcn_sched_group_barrier(0x008, NRB, 0);     // the remaining MFMAs
            }
            __builtin_amdgcn_sched_barrier(0);
            if constexpr (!FP8)
                load_b(4 * s2 + u + RING, u);
            else if (u & 1)
                load_b(2 * s2 + u / 2 + RING, u / 2);
            if (kc == 2) {
                // this wave's part of the next slot has landed; after the barrier
                // everybody's has, and everybody is done with the slot before this one
                wait_vmcnt_le<kWaitA>();
                wg_barrier_nofence();
            }
        }
    };
    int s2 = 0;
    for (; s2 + kPass / 4 <= KT; s2 += kPass / 4) pass(s2, std::integral_constant<int, kPass>{});
    // (KT is even, so what remains of the contraction is a multiple of 8 steps below kPass)
    if constexpr (kPass >= 16) {
        if (KT - s2 == 2) pass(s2, std::integral_constant<int, 8>{});
    }
    if constexpr (kPass >= 24) {
        if (KT - s2 == 4) pass(s2, std::integral_constant<int, 16>{});
    }
    static_assert(kPass == 8 || kPass == 16 || kPass == 24, "remainder passes");
    __builtin_amdgcn_sched_barrier(0);
    wait_vmcnt_le<0>();   // the surplus loads have landed before registers and LDS are reused

    // epilogue: lane l owns token row l%32 of every row block; register quad g of
    // fragment j holds columns 32 j + 8 g + 4 (l/32) .. + 3 of the wave's columns.
    // SwiGLU: the two fragments are the W1 and W3 halves of the same 32 columns.
    // Lanes l and l + 32 hold the two halves of 8 consecutive columns of one row: quads
    // are taken in pairs (g, g + 1) and one lane-half swap per register gives lane l the 8
    // columns of quad g and lane l + 32 those of quad g + 1, stored as 16 bytes each (half
    // as many store instructions and row segments as 8-byte stores; a store's cost here is
    // the number of distinct row segments it touches).
    const int half = lane / 32, cq = 4 * half;
    f32x4 scale[2][4];   // FP8: of the lane's columns, [fragment][quad]
    if constexpr (FP8) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            scale[0][g] = *reinterpret_cast<const f32x4*>(sc0 + 8 * g + cq);
            scale[1][g] = *reinterpret_cast<const f32x4*>(sc1 + 8 * g + cq);
        }
    }
    // w0: quad g, w1: quad g + 1 of the same fragment -> 16 bytes at column 8 (g + half)
    auto store_pair = [&](bf16_t* at, uint2 w0, uint2 w1) {
        const auto x = __builtin_amdgcn_permlane32_swap(w0.x, w1.x, false, false);
        const auto y = __builtin_amdgcn_permlane32_swap(w0.y, w1.y, false, false);
        *reinterpret_cast<uint4*>(at) = make_uint4(x[0], y[0], x[1], y[1]);
    };
#pragma unroll
    for (int i = 0; i < NRB; ++i) {
        const int mr = i * 32 + lane % 32;
        if (mr >= rows) continue;   // (the same for lanes l and l + 32)
        bf16_t* out = static_cast<bf16_t*>(C) + static_cast<size_t>(row0 + mr) * ldc +
                      nt * (SWIGLU ? 128 : 256) + wave * (SWIGLU ? 32 : 64) + 8 * half;
        if (SWIGLU) {
            uint2 w[4];
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                float h[4];
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    float av = acc[i][0][4 * g + c], bv = acc[i][1][4 * g + c];
                    if constexpr (FP8) {
                        av *= scale[0][g][c];
                        bv *= scale[1][g][c];
                    }
                    h[c] = av * bv * __builtin_amdgcn_rcpf(1.f + __expf(-av));
                }
                // round-to-nearest-even in the conversion unit (v_cvt_pk_bf16_f32)
                w[g] = __builtin_bit_cast(uint2, __builtin_convertvector(f32x4{h[0], h[1], h[2], h[3]}, bf16x4));
            }
            store_pair(out, w[0], w[1]);
            store_pair(out + 16, w[2], w[3]);
        } else {
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                uint2 w[4];
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    f32x4 v = {acc[i][j][4 * g], acc[i][j][4 * g + 1], acc[i][j][4 * g + 2],
                               acc[i][j][4 * g + 3]};
                    if constexpr (FP8) v *= scale[j][g];
                    w[g] = __builtin_bit_cast(uint2, __builtin_convertvector(v, bf16x4));
                }
                store_pair(out + 32 * j, w[0], w[1]);
                store_pair(out + 32 * j + 16, w[2], w[3]);
            }
        }
    }
}

// How many tiles at the end of the tile map form the light class (single tiles of at most
// kLightRowBlocks row blocks, spread among the others and run with the deeper weight ring):
// all of them if they are the minority, else none.  8-bit weights: none (no deeper ring for
// them, and without it spreading the light tiles only costs).
__device__ __forceinline__ int light_class_of(const int32_t* tile_info, bool fp8) {
    const int tiles = tile_info[0], light = tile_info[1];
    return (!fp8 && 2 * light <= tiles) ? light : 0;
}

template <bool SWIGLU, bool FP8>
__global__ __launch_bounds__(kWaves* kWave, 1) void ffn_bf16_t256_kernel(StreamGroup g0,
                                                                        StreamGroup g1) {
    __shared__ __attribute__((aligned(1024))) char lds[kSlots * kSlotBytes];

    // Work order.  Workgroups are dealt to the 8 XCDs round-robin by blockIdx, and
    // each XCD has its own L2: workgroup i is item i/8 of XCD i%8's list.
    //  * The dense (shared-expert) group comes first.  The XCDs form an
    //    xr x (8/xr) grid over its (row tiles, column tiles), interleaved, and an
    //    XCD's items are ordered (column tile, row tile): the workgroups of the
    //    first round start together and stay in step, so a weight stream is fetched
    //    into an L2 once for all the XCD's row tiles, an activation tile once for
    //    all its column tiles.
    //  * Then the routed tiles in the tile map's order (longest first), in pairs of
    //    neighbours: pair p runs on XCD p % 8, its items ordered (column tile, tile
    //    of the pair).  Neighbouring tiles mostly belong to one expert and cost the
    //    same, so the two workgroups of a column tile start together and share one
    //    pass over the weight stream; the column tiles that share the gathered
    //    activation rows follow within a few items.
    constexpr int kColsPerTile = SWIGLU ? 128 : 256;
    const int xcd = blockIdx.x % kXcds, idx = blockIdx.x / kXcds;
    const int nt0 = g0.A ? g0.N / kColsPerTile : 1, nt1 = g1.A ? g1.N / kColsPerTile : 1;
    int S = 0, s_rows = 1;     // dense group: items and row tiles of this XCD
    const int xr = g1.xr, xc = kXcds / xr, xri = xcd % xr, xci = xcd / xr;
    if (g1.A != nullptr) {
        const int tiles = (g1.M_dense + g1.dense_rows - 1) / g1.dense_rows;
        s_rows = (tiles - xri + xr - 1) / xr;
        S = s_rows * ((nt1 - xci + xc - 1) / xc);
    }
    const bool first = idx >= S;
    const StreamGroup& g = first ? g0 : g1;
    int tile, nt;
    if (first) {
        if (g0.A == nullptr) return;
        int sub = idx - S;
        if (g0.tile_info != nullptr) {
            // (8-bit weights: no deeper ring for the light tiles, and without it spreading
            // them only costs: they stay at the end)
            const int tiles = g0.tile_info[0];
            const int light = light_class_of(g0.tile_info, FP8), heavy = tiles - light;
            // (pairs dealt in serpentine order: even rounds left to right, odd rounds
            // right to left, which evens out the XCDs' totals of the sorted tile costs)
            const int round = sub / (2 * nt0), in_pair = sub % (2 * nt0);
            const int q = round * kXcds + ((round & 1) ? kXcds - 1 - xcd : xcd);
            // The light tiles (single tiles of at most kLightRowBlocks row blocks: the end
            // of the tile map) wait for their weights, the others for the matrix unit:
            // their pairs are spread evenly among the pairs of the others, so that both
            // kinds run side by side through the whole launch.  Of the first q + 1 pair
            // positions floor((q + 1) n_light / n_pairs) hold light pairs.
            const int hp = (heavy + 1) / 2, lp = (light + 1) / 2, np = hp + lp;
            if (q >= np) return;   // the grid is sized for the host's bound
            const int lq = static_cast<int>(static_cast<int64_t>(q + 1) * lp / np);
            const int lq0 = static_cast<int>(static_cast<int64_t>(q) * lp / np);
            int first_of_pair, end;
            if (lq > lq0) {
                first_of_pair = heavy + 2 * lq0;
                end = tiles;
            } else {
                first_of_pair = 2 * (q - lq0);
                end = heavy;
            }
            tile = first_of_pair + in_pair % 2;
            nt = in_pair / 2;
            if (tile >= end) return;
        } else {   // a dense group in the first slot: its row tiles striped over the XCDs
            const int tiles = (g0.M_dense + g0.dense_rows - 1) / g0.dense_rows;
            tile = sub / nt0 * kXcds + xcd;
            nt = sub % nt0;
            if (tile >= tiles) return;
        }
    } else {
        tile = xri + xr * (idx % s_rows);
        nt = xci + xc * (idx / s_rows);
    }

    const bf16_t* __restrict__ A = static_cast<const bf16_t*>(g.A);
    const char* __restrict__ Bp = static_cast<const char*>(g.Bp);
    const int32_t* __restrict__ row_map = g.row_map;
    const int32_t* __restrict__ tile_info = g.tile_info;
    const int lda = g.lda, Kd = g.Kd, ldc = g.ldc, M_dense = g.M_dense;
    int e, row0, rows;
    bool only_tile;   // of its expert: nobody else reads these weights
    if (tile_info != nullptr) {
        const int32_t* ent = tile_info + kTileHdr + 4 * static_cast<size_t>(tile);
        e = ent[0];
        row0 = ent[1];
        rows = ent[2];
        only_tile = ent[3] == 1;
    } else {
        e = 0;
        row0 = tile * g.dense_rows;
        rows = min(g.dense_rows, M_dense - row0);
        only_tile = M_dense <= g.dense_rows;
    }
    const int lane = lane_id(), wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n_rb = (rows + 31) / 32;   // 32-row blocks that hold real rows
    const bool deep_ring = tile_info != nullptr && only_tile && light_class_of(tile_info, FP8) > 0;
    const int KT = Kd / kStepK;

    // B: the two fragment streams of this wave's 64 weight columns; a stream is
    // Kd/16 fragments of 64 lanes x 16 B (FP8: Kd/32), contiguous
    constexpr size_t kElemBytes = FP8 ? 1 : 2;
    const size_t stream_elems = static_cast<size_t>(Kd) * 32;
    const size_t sidx = SWIGLU ? static_cast<size_t>(4 * nt + wave) * 2
                               : static_cast<size_t>(8 * nt + 2 * wave);
    // (wave-uniform pointers: the loads take a scalar base and the lane's offset)
    const char* b0 = Bp + (static_cast<size_t>(e) * g.group_stride + sidx * stream_elems) * kElemBytes;
    const char* b1 = b0 + stream_elems * kElemBytes;
    // FP8: scale[expert][stream][N]; SwiGLU: W1 and W3 scales of the wave's 32 columns,
    // plain: of its two neighbouring 32-column blocks
    const float* sc0 = nullptr;
    const float* sc1 = nullptr;
    if (FP8) {
        const float* sc = g.scale + static_cast<size_t>(e) * (SWIGLU ? 2 : 1) * g.N;
        sc0 = sc + nt * kColsPerTile + wave * (SWIGLU ? 32 : 64);
        sc1 = SWIGLU ? sc0 + g.N : sc0 + 32;
    }

    // The deeper weight ring is for light tiles that run among matrix-bound ones; where
    // most tiles are light (few tokens) the launch as a whole is bound by the memory
    // system, which more loads in flight per unit only crowd (measured: +3 % step time at
    // 256 tokens, +17 % on a layer whose experts all hold 128 rows).
#define ALLOCMOE_T256_BODY(n, ring)                                                                 \
    do {                                                                                            \
        if (only_tile)                                                                              \
            t256_body<SWIGLU, n, true, FP8, ring>(lds, A, lda, row_map, b0, b1, sc0, sc1, KT,       \
                                                  wave, lane, row0, rows, nt, g.C, ldc);            \
        else                                                                                        \
            t256_body<SWIGLU, n, false, FP8, ring>(lds, A, lda, row_map, b0, b1, sc0, sc1, KT,      \
                                                   wave, lane, row0, rows, nt, g.C, ldc);           \
    } while (0)
#define ALLOCMOE_T256_CASE(n)                                                                       \
    case n:                                                                                         \
        if constexpr (!FP8 && n <= kLightRowBlocks) {                                               \
            if (deep_ring) {                                                                        \
                ALLOCMOE_T256_BODY(n, kBRingDeep);                                                  \
                break;                                                                              \
            }                                                                                       \
        }                                                                                           \
        ALLOCMOE_T256_BODY(n, kBRing);                                                              \
        break;
    switch (n_rb) {   // uniform over the workgroup
        ALLOCMOE_T256_CASE(1)
        ALLOCMOE_T256_CASE(2)
        ALLOCMOE_T256_CASE(3)
        ALLOCMOE_T256_CASE(4)
        ALLOCMOE_T256_CASE(5)
        ALLOCMOE_T256_CASE(6)
        ALLOCMOE_T256_CASE(7)
        default: ALLOCMOE_T256_CASE(8)
    }
#undef ALLOCMOE_T256_CASE
#undef ALLOCMOE_T256_BODY
}

}  // namespace

// Rows per tile of a dense group (every row tile reads the same weights): full
// 256-row tiles where those fill the chip; with fewer tokens the smallest multiple of
// 32 rows that still gives at most one workgroup per two compute units, so that the
// group is one round of short workgroups instead of a few long ones (a tile costs in
// proportion to its 32-row blocks; the weights it re-reads come from L2).  Measured on
// DeepSeek-V2-Lite shapes, targets of 64 to 192 workgroups differ by < 2 %, 256 and
// more lose 1-5 % from 2048 tokens on; against fixed 256-row tiles the step is 4-6 %
// shorter at 128-512 tokens with bf16 weights, 9-13 % with 8-bit weights.
int dense_tile_rows(int M, int col_tiles) {
    constexpr int kTargetWorkgroups = 128;
    int h = 32;
    while (h < kRows && static_cast<int64_t>((M + h - 1) / h) * col_tiles > kTargetWorkgroups) h += 32;
    return h;
}

hipError_t launch_ffn_bf16_t256(bool swiglu, StreamGroup routed, StreamGroup shared,
                                hipStream_t stream) {
    const int cols = swiglu ? 128 : 256;
    if (routed.A != nullptr && routed.tile_info == nullptr)
        routed.dense_rows = dense_tile_rows(routed.M_dense, routed.N / cols);
    if (shared.A != nullptr) shared.dense_rows = dense_tile_rows(shared.M_dense, shared.N / cols);
    // items per XCD; for the routed group an upper bound (the real tile count is
    // known on the device only)
    int64_t per_xcd = 0;
    if (routed.A != nullptr) {
        int64_t tiles;   // per XCD
        if (routed.tile_info != nullptr)
            // whole pairs; light and other tiles pair among themselves: one pair more
            tiles = 2 * (((routed.max_tiles + 1) / 2 + 1 + kXcds - 1) / kXcds);
        else
            tiles = ((routed.M_dense + routed.dense_rows - 1) / routed.dense_rows + kXcds - 1) / kXcds;
        per_xcd += tiles * (routed.N / cols);
    }
    if (shared.A != nullptr) {
        // XCD grid over (row tiles, column tiles): xr x 8/xr, chosen to minimise the
        // bytes the 8 L2s fetch in total: (8/xr) x activations + xr x weights
        const int64_t rt = (shared.M_dense + shared.dense_rows - 1) / shared.dense_rows, ct = shared.N / cols;
        const double a_bytes = static_cast<double>(shared.M_dense) * shared.Kd;
        const double b_bytes = static_cast<double>(shared.N) * shared.Kd * (swiglu ? 2 : 1);
        int best = 1;
        double best_cost = 0;
        for (int xr = 1; xr <= kXcds; xr *= 2) {
            const double cost = (kXcds / xr) * a_bytes + xr * b_bytes;
            if (xr == 1 || cost < best_cost) {
                best = xr;
                best_cost = cost;
            }
        }
        shared.xr = best;
        const int xc = kXcds / best;
        per_xcd += ((rt + best - 1) / best) * ((ct + xc - 1) / xc);
    }
    if (per_xcd <= 0) return hipSuccess;
    const dim3 grid(static_cast<unsigned>(per_xcd * kXcds)), block(kWaves * kWave);
    const bool fp8 = (routed.A ? routed.scale : shared.scale) != nullptr;
    if (routed.A && shared.A && (routed.scale != nullptr) != (shared.scale != nullptr))
        return hipErrorInvalidValue;   // one weight format per launch
    if (swiglu && fp8)
        hipLaunchKernelGGL((ffn_bf16_t256_kernel<true, true>), grid, block, 0, stream, routed, shared);
    else if (swiglu)
        hipLaunchKernelGGL((ffn_bf16_t256_kernel<true, false>), grid, block, 0, stream, routed, shared);
    else if (fp8)
        hipLaunchKernelGGL((ffn_bf16_t256_kernel<false, true>), grid, block, 0, stream, routed, shared);
    else
        hipLaunchKernelGGL((ffn_bf16_t256_kernel<false, false>), grid, block, 0, stream, routed, shared);
    return hipGetLastError();
}

}  // namespace allocmoe
