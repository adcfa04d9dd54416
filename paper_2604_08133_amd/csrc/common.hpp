// Device-side helpers shared by the gfx950 kernels: element types, wave64
// reductions, ordered keys.  Wavefronts are 64 lanes wide throughout.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace allocmoe {

constexpr int kWave = 64;

typedef uint16_t bf16_t;  // bfloat16 bit pattern

__device__ __forceinline__ float bf16_to_f32(bf16_t v) {
    return __uint_as_float(static_cast<uint32_t>(v) << 16);
}

// round-to-nearest-even; inputs are finite in this library
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return static_cast<bf16_t>(u >> 16);
}

__device__ __forceinline__ float load_f32(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float load_f32(const bf16_t* p, size_t i) { return bf16_to_f32(p[i]); }
__device__ __forceinline__ void store_elem(float* p, size_t i, float v) { p[i] = v; }
__device__ __forceinline__ void store_elem(bf16_t* p, size_t i, float v) { p[i] = f32_to_bf16(v); }

__device__ __forceinline__ int lane_id() { return threadIdx.x & (kWave - 1); }

// The value of lane (l ^ S), S a power of two.  Within a row of 16 lanes the exchange is
// done by the vector unit's lane permutations (DPP) instead of a trip through the LDS
// crossbar: l^1 and l^2 are permutations inside a quad; reversing a quad is l^3,
// reversing 8 lanes l^7, reversing 16 lanes l^15, so l^4 = (l^7)^3 and l^8 = (l^15)^7.
// Across rows: the row swaps of gfx950 (v_permlane16_swap exchanges the odd rows of its
// first operand with the even rows of its second, v_permlane32_swap the upper half with
// the lower half); given the same value twice, the first result holds rows (0,0,2,2)
// resp. halves (lo,lo), the second rows (1,1,3,3) resp. (hi,hi), and a lane takes the
// one that holds its partner's row.
// All 64 lanes must be active.
template <int S>
__device__ __forceinline__ uint32_t lane_xor(uint32_t v) {
    static_assert(S == 1 || S == 2 || S == 4 || S == 8 || S == 16 || S == 32, "power of two");
    const int x = static_cast<int>(v);
    constexpr int kQuad1 = 0xB1, kQuad2 = 0x4E, kQuadRev = 0x1B;    // quad_perm [1,0,3,2] [2,3,0,1] [3,2,1,0]
    constexpr int kRowMirror = 0x140, kRowHalfMirror = 0x141;
    if (S == 1) return __builtin_amdgcn_mov_dpp(x, kQuad1, 0xF, 0xF, false);
    if (S == 2) return __builtin_amdgcn_mov_dpp(x, kQuad2, 0xF, 0xF, false);
    if (S == 4)
        return __builtin_amdgcn_mov_dpp(__builtin_amdgcn_mov_dpp(x, kRowHalfMirror, 0xF, 0xF, false),
                                        kQuadRev, 0xF, 0xF, false);
    if (S == 8)
        return __builtin_amdgcn_mov_dpp(__builtin_amdgcn_mov_dpp(x, kRowMirror, 0xF, 0xF, false),
                                        kRowHalfMirror, 0xF, 0xF, false);
    if (S == 16) {
        const auto r = __builtin_amdgcn_permlane16_swap(v, v, false, false);
        return (lane_id() & 16) ? r[0] : r[1];
    }
    const auto r = __builtin_amdgcn_permlane32_swap(v, v, false, false);
    return (lane_id() & 32) ? r[0] : r[1];
}
template <int S>
__device__ __forceinline__ float lane_xor(float v) {
    return __uint_as_float(lane_xor<S>(__float_as_uint(v)));
}
template <int S>
__device__ __forceinline__ uint64_t lane_xor(uint64_t v) {
    return static_cast<uint64_t>(lane_xor<S>(static_cast<uint32_t>(v))) |
           (static_cast<uint64_t>(lane_xor<S>(static_cast<uint32_t>(v >> 32))) << 32);
}

// Reductions over the 64 lanes (all active), result in every lane, without LDS permutes:
// inside a row of 16 lanes by DPP permutations (lane ^ 1, lane ^ 2, mirror of 8, mirror
// of 16: afterwards every lane holds its row's result), across the rows by the two row
// broadcasts (lane 15 of a row into the next row, lane 31 into the upper half), after
// which lane 63 holds the whole wave's result.  `identity` is what a lane combines with
// where a broadcast does not reach it.  The order of the combination is fixed.
template <typename Op>
__device__ __forceinline__ uint32_t wave_reduce_bits(uint32_t v, uint32_t identity, Op op) {
    constexpr int kQuad1 = 0xB1, kQuad2 = 0x4E, kRowMirror = 0x140, kRowHalfMirror = 0x141;
    constexpr int kBcast15 = 0x142, kBcast31 = 0x143;
#define ALLOCMOE_DPP(x, ctrl) \
    static_cast<uint32_t>(__builtin_amdgcn_mov_dpp(static_cast<int>(x), ctrl, 0xF, 0xF, false))
    v = op(v, ALLOCMOE_DPP(v, kQuad1));
    v = op(v, ALLOCMOE_DPP(v, kQuad2));
    v = op(v, ALLOCMOE_DPP(v, kRowHalfMirror));
    v = op(v, ALLOCMOE_DPP(v, kRowMirror));
#undef ALLOCMOE_DPP
    v = op(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
                  static_cast<int>(identity), static_cast<int>(v), kBcast15, 0xA, 0xF, false)));
    v = op(v, static_cast<uint32_t>(__builtin_amdgcn_update_dpp(
                  static_cast<int>(identity), static_cast<int>(v), kBcast31, 0xC, 0xF, false)));
    return static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(v), kWave - 1));
}
__device__ __forceinline__ float wave_sum(float v) {
    return __uint_as_float(wave_reduce_bits(__float_as_uint(v), __float_as_uint(0.f), [](uint32_t a, uint32_t b) {
        return __float_as_uint(__uint_as_float(a) + __uint_as_float(b));
    }));
}
__device__ __forceinline__ float wave_max(float v) {
    return __uint_as_float(wave_reduce_bits(__float_as_uint(v), __float_as_uint(-INFINITY), [](uint32_t a, uint32_t b) {
        return __float_as_uint(fmaxf(__uint_as_float(a), __uint_as_float(b)));
    }));
}
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t v) {
    return wave_reduce_bits(v, 0xFFFFFFFFu, [](uint32_t a, uint32_t b) { return b < a ? b : a; });
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
    return wave_reduce_bits(v, 0u, [](uint32_t a, uint32_t b) { return b > a ? b : a; });
}
// (64-bit: a butterfly, one exchange per power of two, largest first)
__device__ __forceinline__ uint64_t wave_max_u64(uint64_t v) {
    auto mx = [](uint64_t a, uint64_t b) { return b > a ? b : a; };
    v = mx(v, lane_xor<32>(v));
    v = mx(v, lane_xor<16>(v));
    v = mx(v, lane_xor<8>(v));
    v = mx(v, lane_xor<4>(v));
    v = mx(v, lane_xor<2>(v));
    v = mx(v, lane_xor<1>(v));
    return v;
}
// inclusive prefix sum over the 64 lanes (all active): inside each row of 16 lanes by
// DPP shifts that fill with zero, then the totals of the rows before (lane 15 of a row
// broadcast to the next row, lane 31 to the upper half)
__device__ __forceinline__ int wave_scan_incl(int v) {
    constexpr int kRowShr = 0x110, kBcast15 = 0x142, kBcast31 = 0x143;
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr + 1, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr + 2, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr + 4, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kRowShr + 8, 0xF, 0xF, true);
    v += __builtin_amdgcn_update_dpp(0, v, kBcast15, 0xA, 0xF, false);
    v += __builtin_amdgcn_update_dpp(0, v, kBcast31, 0xC, 0xF, false);
    return v;
}

// Monotone map from finite fp32 to u32: a < b  <=>  key(a) < key(b); -0.0 and
// +0.0 map to the same key.
__device__ __forceinline__ uint32_t ordered_key(float f) {
    uint32_t u = __float_as_uint(f + 0.0f);
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

__device__ __forceinline__ uint64_t lanemask_lt() {
    return (1ull << lane_id()) - 1ull;
}

}  // namespace allocmoe
