// C ABI of the library (include/allocmoe.h): argument validation on the host,
// workspace carving, and the launch sequence of the layer.  Nothing here
// allocates, synchronises or copies to the host.
#include "../../include/allocmoe.h"

#include "kernels.hpp"

#include <algorithm>
#include <mutex>

namespace {

using namespace allocmoe;

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline size_t elem_size(int dtype) { return dtype == ALLOCMOE_F32 ? 4u : 2u; }

struct Scratch {       // offsets inside the scratch region (which starts the workspace)
    size_t words, prefix, tile_info, spread, bytes;
    int64_t max_tiles;
};

inline int64_t max_tiles_for(const allocmoe_layer_desc* d, int bm) {
    // >= sum_e ceil(M_e / bm) for any split of B rows over the experts: an expert with
    // rows has one tile plus one per further bm rows, and at most min(E, B) have rows
    const int64_t active = std::min<int64_t>(d->E, d->budget);
    return active + (d->budget - active) / bm;
}

Scratch scratch_of(const allocmoe_layer_desc* d) {
    Scratch s;
    const size_t nb = (static_cast<size_t>(d->T) + 63) / 64;
    size_t off = 0;
    s.words = off;
    off = align_up(off + nb * 64 * sizeof(uint64_t));
    s.prefix = off;
    off = align_up(off + nb * 64 * sizeof(int32_t));
    s.tile_info = off;
    s.max_tiles = max_tiles_for(d, kTileRowsSmall);
    off = align_up(off + tile_info_ints(s.max_tiles) * sizeof(int32_t));
    s.spread = off;   // partial histograms of the many-workgroup selection
    off = align_up(off + plan_spread_bytes(d->T));
    s.bytes = off;
    return s;
}

inline int selector_of(const allocmoe_layer_desc* d) { return d->flags & 0xFF; }
inline bool fp8_of(const allocmoe_layer_desc* d) { return (d->flags & ALLOCMOE_WEIGHTS_FP8) != 0; }

allocmoe_status check_desc(const allocmoe_layer_desc* d) {
    if (d == nullptr) return ALLOCMOE_EINVAL;
    if (d->dtype != ALLOCMOE_F32 && d->dtype != ALLOCMOE_BF16) return ALLOCMOE_EINVAL;
    if ((d->flags & ~(0xFF | ALLOCMOE_WEIGHTS_FP8)) != 0) return ALLOCMOE_EINVAL;
    if (selector_of(d) > ALLOCMOE_SELECT_RELATIVE) return ALLOCMOE_EINVAL;
    if (fp8_of(d) && d->dtype != ALLOCMOE_BF16) return ALLOCMOE_EINVAL;
    if (d->T < 1 || d->d < 1 || d->E < 1 || d->I < 1 || d->K < 1) return ALLOCMOE_EINVAL;
    if (d->K_base < 0 || d->K_base > d->K || d->K > d->E) return ALLOCMOE_EINVAL;
    if (d->I_shared < 0 || (d->shared_gate != 0 && d->shared_gate != 1)) return ALLOCMOE_EINVAL;
    if (d->shared_gate && d->I_shared == 0) return ALLOCMOE_EINVAL;
    if (d->E > 64 || d->K > 16) return ALLOCMOE_ESHAPE;
    if (static_cast<int64_t>(d->T) * d->K >= (1ll << 31)) return ALLOCMOE_ESHAPE;
    if (d->dtype == ALLOCMOE_BF16 && (d->d % 64 || d->I % 64 || d->I_shared % 64))
        return ALLOCMOE_ESHAPE;
    if (fp8_of(d) && (d->d % 128 || d->I % 128 || d->I_shared % 128)) return ALLOCMOE_ESHAPE;
    if (d->budget < static_cast<int64_t>(d->T) * d->K_base ||
        d->budget > static_cast<int64_t>(d->T) * d->K)
        return ALLOCMOE_EBUDGET;
    return ALLOCMOE_OK;
}

allocmoe_status layout_of(const allocmoe_layer_desc* d, allocmoe_ws_layout* L) {
    const allocmoe_status st = check_desc(d);
    if (st != ALLOCMOE_OK) return st;
    const size_t T = d->T, E = d->E, K = d->K, B = static_cast<size_t>(d->budget);
    const size_t es = elem_size(d->dtype);
    size_t off = 0;
    auto take = [&off](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    L->scratch = take(scratch_of(d).bytes);
    L->sel_keys = take(selector_of(d) != ALLOCMOE_SELECT_SCORE ? T * K * 4 : 0);
    L->scores = take(T * E * 4);
    L->topk_ids = take(T * K * 4);
    L->topk_s = take(T * K * 4);
    L->keep_count = take(T * 4);
    L->shared_gate = take(T * 4);
    L->expert_offsets = take((E + 1) * 4);
    L->row_token = take(B * 4);
    L->row_rank = take(B * 4);
    L->inv_row = take(T * K * 4);
    L->H = take(B * d->I * es);
    L->Hs = take(T * d->I_shared * es);
    L->O = take(B * d->d * es);   // the experts' outputs are kept in the layer's dtype
    L->Os = take(d->I_shared ? T * d->d * es : 0);
    L->total = off;
    return ALLOCMOE_OK;
}

struct PackedLayout {   // element offsets inside the packed buffer
    size_t p13, p2, ps13, ps2, gate, total_elems;
};

PackedLayout packed_of(const allocmoe_layer_desc* d) {
    PackedLayout p;
    const size_t E = d->E, dd = d->d, I = d->I, Is = d->I_shared;
    p.p13 = 0;
    p.p2 = p.p13 + E * 2 * dd * I;
    p.ps13 = p.p2 + E * I * dd;
    p.ps2 = p.ps13 + 2 * dd * Is;
    p.gate = p.ps2 + Is * dd;
    p.total_elems = p.gate + gate_packed_elems(d->d);
    return p;
}

// 8-bit expert weights: byte offsets.  The code regions keep the order and the
// element counts of the bf16 layout (one byte per element); then the bf16 gate
// matrix, then the fp32 column scales [E][2][I], [E][d], [2][I_shared], [d].
struct PackedFp8 {
    size_t q13, q2, qs13, qs2, gate, sc13, sc2, scs13, scs2, total;
};

PackedFp8 packed_fp8_of(const allocmoe_layer_desc* d) {
    PackedFp8 p;
    const size_t E = d->E, dd = d->d, I = d->I, Is = d->I_shared;
    size_t off = 0;
    auto take = [&off](size_t bytes) {
        const size_t at = off;
        off = align_up(off + bytes);
        return at;
    };
    p.q13 = take(E * 2 * dd * I);
    p.q2 = take(E * I * dd);
    p.qs13 = take(2 * dd * Is);
    p.qs2 = take(Is * dd);
    p.gate = take(gate_packed_elems(d->d) * 2);
    p.sc13 = take(E * 2 * I * 4);
    p.sc2 = take(E * dd * 4);
    p.scs13 = take(2 * Is * 4);
    p.scs2 = take(Is ? dd * 4 : 0);
    p.total = off;
    return p;
}

// the re-tiled gate matrix inside the packed buffer
inline const uint16_t* packed_gate(const allocmoe_layer_desc* d, const void* packed) {
    if (fp8_of(d))
        return reinterpret_cast<const uint16_t*>(static_cast<const char*>(packed) + packed_fp8_of(d).gate);
    return static_cast<const uint16_t*>(packed) + packed_of(d).gate;
}

inline bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline allocmoe_status hip_status(hipError_t e) { return e == hipSuccess ? ALLOCMOE_OK : ALLOCMOE_EHIP; }

template <typename T>
inline T* at(void* base, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(base) + off); }

#define ALLOCMOE_TRY(expr)                                  \
    do {                                                    \
        const allocmoe_status st_ = hip_status(expr);       \
        if (st_ != ALLOCMOE_OK) return st_;                 \
    } while (0)

}  // namespace

extern "C" {

const char* allocmoe_status_string(allocmoe_status status) {
    switch (status) {
        case ALLOCMOE_OK: return "ok";
        case ALLOCMOE_EINVAL: return "invalid argument";
        case ALLOCMOE_EBUDGET: return "budget outside [T*K_base, T*K]";
        case ALLOCMOE_ESHAPE: return "unsupported size";
        case ALLOCMOE_EWORKSPACE: return "workspace or packed buffer too small or misaligned";
        case ALLOCMOE_EHIP: return "HIP runtime error";
    }
    return "unknown status";
}

allocmoe_status allocmoe_workspace_layout(const allocmoe_layer_desc* desc,
                                          allocmoe_ws_layout* layout) {
    if (layout == nullptr) return ALLOCMOE_EINVAL;
    return layout_of(desc, layout);
}

allocmoe_status allocmoe_workspace_bytes(const allocmoe_layer_desc* desc, size_t* bytes) {
    if (bytes == nullptr) return ALLOCMOE_EINVAL;
    allocmoe_ws_layout L;
    const allocmoe_status st = layout_of(desc, &L);
    if (st == ALLOCMOE_OK) *bytes = L.total;
    return st;
}

allocmoe_status allocmoe_packed_bytes(const allocmoe_layer_desc* desc, size_t* bytes) {
    if (bytes == nullptr) return ALLOCMOE_EINVAL;
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (desc->dtype != ALLOCMOE_BF16) return ALLOCMOE_EINVAL;
    *bytes = fp8_of(desc) ? packed_fp8_of(desc).total : align_up(packed_of(desc).total_elems * 2);
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_pack_weights(const allocmoe_layer_desc* desc,
                                      const allocmoe_weights* w, void* packed,
                                      size_t packed_bytes, allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (desc->dtype != ALLOCMOE_BF16 || w == nullptr || packed == nullptr) return ALLOCMOE_EINVAL;
    if (!w->Wg || !w->W1 || !w->W3 || !w->W2) return ALLOCMOE_EINVAL;
    if (desc->I_shared && (!w->Ws1 || !w->Ws3 || !w->Ws2)) return ALLOCMOE_EINVAL;
    if (desc->shared_gate && !w->w_sg) return ALLOCMOE_EINVAL;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int E = desc->E, d = desc->d, I = desc->I, Is = desc->I_shared;
    if (fp8_of(desc)) {
        const PackedFp8 q = packed_fp8_of(desc);
        if (packed_bytes < q.total || !aligned(packed, kAlign)) return ALLOCMOE_EWORKSPACE;
        char* out = static_cast<char*>(packed);
        const size_t dd = d, II = I, SS = Is;
        float* sc13 = at<float>(out, q.sc13);
        ALLOCMOE_TRY(launch_pack_b_fp8(w->W1, E, d, I, out + q.q13, 2 * dd * II, 2 * dd * 32, 0, sc13,
                                       2 * II, stream));
        ALLOCMOE_TRY(launch_pack_b_fp8(w->W3, E, d, I, out + q.q13, 2 * dd * II, 2 * dd * 32, dd * 32,
                                       sc13 + II, 2 * II, stream));
        ALLOCMOE_TRY(launch_pack_b_fp8(w->W2, E, I, d, out + q.q2, II * dd, II * 32, 0,
                                       at<float>(out, q.sc2), dd, stream));
        ALLOCMOE_TRY(launch_pack_gate(w->Wg, desc->shared_gate ? w->w_sg : nullptr, d, E,
                                      out + q.gate, stream));
        if (Is) {
            float* scs13 = at<float>(out, q.scs13);
            ALLOCMOE_TRY(launch_pack_b_fp8(w->Ws1, 1, d, Is, out + q.qs13, 2 * dd * SS, 2 * dd * 32, 0,
                                           scs13, 2 * SS, stream));
            ALLOCMOE_TRY(launch_pack_b_fp8(w->Ws3, 1, d, Is, out + q.qs13, 2 * dd * SS, 2 * dd * 32,
                                           dd * 32, scs13 + SS, 2 * SS, stream));
            ALLOCMOE_TRY(launch_pack_b_fp8(w->Ws2, 1, Is, d, out + q.qs2, SS * dd, SS * 32, 0,
                                           at<float>(out, q.scs2), dd, stream));
        }
        return ALLOCMOE_OK;
    }
    const PackedLayout p = packed_of(desc);
    if (packed_bytes < p.total_elems * 2 || !aligned(packed, kAlign)) return ALLOCMOE_EWORKSPACE;
    uint16_t* out = static_cast<uint16_t*>(packed);
    const size_t dd = d, II = I;
    ALLOCMOE_TRY(launch_pack_b(w->W1, E, d, I, out + p.p13, 2 * dd * II, 2 * dd * 32, 0, stream));
    ALLOCMOE_TRY(launch_pack_b(w->W3, E, d, I, out + p.p13, 2 * dd * II, 2 * dd * 32, dd * 32, stream));
    ALLOCMOE_TRY(launch_pack_b(w->W2, E, I, d, out + p.p2, II * dd, II * 32, 0, stream));
    ALLOCMOE_TRY(launch_pack_gate(w->Wg, desc->shared_gate ? w->w_sg : nullptr, d, E, out + p.gate,
                                  stream));
    if (Is) {
        const size_t SS = Is;
        ALLOCMOE_TRY(launch_pack_b(w->Ws1, 1, d, Is, out + p.ps13, 2 * dd * SS, 2 * dd * 32, 0, stream));
        ALLOCMOE_TRY(launch_pack_b(w->Ws3, 1, d, Is, out + p.ps13, 2 * dd * SS, 2 * dd * 32, dd * 32, stream));
        ALLOCMOE_TRY(launch_pack_b(w->Ws2, 1, Is, d, out + p.ps2, SS * dd, SS * 32, 0, stream));
    }
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_route(const allocmoe_layer_desc* desc, const void* X,
                               const allocmoe_weights* w, float* scores, int32_t* topk_ids,
                               float* topk_s, int32_t* keep_count, void* ws, size_t ws_bytes,
                               allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (!X || !w || !w->Wg || !topk_ids || !topk_s || !keep_count) return ALLOCMOE_EINVAL;
    // one workgroup selects out of LDS; the selector keys need device scratch, and so does
    // the many-workgroup selection (used when the workspace has room for it)
    const bool keyed = selector_of(desc) != ALLOCMOE_SELECT_SCORE;
    const size_t key_bytes = keyed ? align_up(static_cast<size_t>(desc->T) * desc->K * 4) : 0;
    if (keyed && (ws == nullptr || ws_bytes < key_bytes || !aligned(ws, kAlign)))
        return ALLOCMOE_EWORKSPACE;
    void* spread = nullptr;
    if (ws != nullptr && aligned(ws, kAlign) && plan_spread_bytes(desc->T) > 0 &&
        ws_bytes >= key_bytes + plan_spread_bytes(desc->T))
        spread = static_cast<char*>(ws) + key_bytes;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (desc->dtype == ALLOCMOE_BF16 && w->packed != nullptr) {
        if (!aligned(w->packed, kAlign) || !aligned(X, 16)) return ALLOCMOE_EINVAL;
        const uint16_t* gp = packed_gate(desc, w->packed);
        ALLOCMOE_TRY(launch_route_mfma(X, gp, w->gate_bias, false, desc->T, desc->d, desc->E,
                                       desc->K, scores, topk_ids, topk_s, nullptr, stream));
    } else {
        ALLOCMOE_TRY(launch_route(desc->dtype, X, w->Wg, w->gate_bias, nullptr, desc->T, desc->d,
                                  desc->E, desc->K, scores, topk_ids, topk_s, nullptr, stream));
    }
    const float* keys = topk_s;
    if (keyed) {
        ALLOCMOE_TRY(launch_selector_keys(topk_s, desc->T, desc->K, selector_of(desc),
                                          static_cast<float*>(ws), stream));
        keys = static_cast<const float*>(ws);
    }
    ALLOCMOE_TRY(launch_select(keys, desc->T, desc->K, desc->K_base, desc->budget, keep_count,
                               spread, stream));
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_route_from_scores(const allocmoe_layer_desc* desc, const float* scores,
                                           int32_t* topk_ids, float* topk_s,
                                           int32_t* keep_count, void* ws, size_t ws_bytes,
                                           allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (!scores || !topk_ids || !topk_s || !keep_count) return ALLOCMOE_EINVAL;
    const bool keyed = selector_of(desc) != ALLOCMOE_SELECT_SCORE;
    const size_t key_bytes = keyed ? align_up(static_cast<size_t>(desc->T) * desc->K * 4) : 0;
    if (keyed && (ws == nullptr || ws_bytes < key_bytes || !aligned(ws, kAlign)))
        return ALLOCMOE_EWORKSPACE;
    void* spread = nullptr;
    if (ws != nullptr && aligned(ws, kAlign) && plan_spread_bytes(desc->T) > 0 &&
        ws_bytes >= key_bytes + plan_spread_bytes(desc->T))
        spread = static_cast<char*>(ws) + key_bytes;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ALLOCMOE_TRY(launch_topk_from_scores(scores, desc->T, desc->E, desc->K, topk_ids, topk_s, stream));
    const float* keys = topk_s;
    if (keyed) {
        ALLOCMOE_TRY(launch_selector_keys(topk_s, desc->T, desc->K, selector_of(desc),
                                          static_cast<float*>(ws), stream));
        keys = static_cast<const float*>(ws);
    }
    ALLOCMOE_TRY(launch_select(keys, desc->T, desc->K, desc->K_base, desc->budget, keep_count,
                               spread, stream));
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_dispatch(const allocmoe_layer_desc* desc, const int32_t* topk_ids,
                                  const int32_t* keep_count, int32_t* expert_offsets,
                                  int32_t* row_token, int32_t* row_rank, int32_t* inv_row,
                                  void* ws, size_t ws_bytes, allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (!topk_ids || !keep_count || !expert_offsets || !inv_row) return ALLOCMOE_EINVAL;
    if (desc->budget > 0 && (!row_token || !row_rank)) return ALLOCMOE_EINVAL;
    const Scratch s = scratch_of(desc);
    if (ws == nullptr || ws_bytes < s.bytes || !aligned(ws, kAlign)) return ALLOCMOE_EWORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ALLOCMOE_TRY(launch_dispatch(topk_ids, keep_count, desc->T, desc->K, desc->E, desc->budget,
                                 expert_offsets, row_token, row_rank, inv_row,
                                 at<uint64_t>(ws, s.words), at<int32_t>(ws, s.prefix),
                                 kTileRowsSmall, nullptr, true, stream));
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_routing_stats(const allocmoe_layer_desc* desc, const float* scores,
                                       const int32_t* topk_ids, const float* topk_s,
                                       const int32_t* keep_count, int32_t* load_orig,
                                       int32_t* load_kept, float* wload_orig, float* wload_kept,
                                       float* token_entropy, allocmoe_routing_metrics* metrics,
                                       void* ws, size_t ws_bytes, allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (!scores || !topk_ids || !topk_s || !keep_count || !load_orig || !load_kept ||
        !wload_orig || !wload_kept || !token_entropy || !metrics)
        return ALLOCMOE_EINVAL;
    if (ws == nullptr || ws_bytes < static_cast<size_t>(desc->T) * 4 || !aligned(ws, kAlign))
        return ALLOCMOE_EWORKSPACE;
    ALLOCMOE_TRY(launch_routing_stats(scores, topk_ids, topk_s, keep_count, desc->T, desc->E,
                                      desc->K, load_orig, load_kept, wload_orig, wload_kept,
                                      token_entropy, static_cast<int32_t*>(ws),
                                      reinterpret_cast<float*>(metrics),
                                      static_cast<hipStream_t>(stream_)));
    return ALLOCMOE_OK;
}

}  // extern "C"

namespace {

// Host-side objects the library keeps per device, created on first use and kept for
// the life of the process: one extra stream (default priority, not synchronising with
// the null stream) and two events without timing, for running the shared expert's GEMMs
// beside the selection; the timing events of the measurement variant.  `lock` is held
// for the whole enqueue sequence of a forward call, so that two host threads calling on
// one device cannot interleave their records and waits on the shared events.
constexpr int kTimedEvents = 9;   // main stream: before each of the 5 stages + end; side stream: 3
struct DeviceState {
    std::mutex lock;
    hipStream_t side = nullptr;
    hipEvent_t fork = nullptr, join = nullptr;
    hipEvent_t ev[kTimedEvents] = {};
    bool have_ev = false;
    unsigned char* static_scratch = nullptr;   // this device's copy of `scratch` (below)
};

// Scratch of allocmoe_dispatch_static.  In host code this name is only a handle for
// hipGetSymbolAddress: every device holds its own copy at its own address, kept in
// DeviceState::static_scratch.
static __device__ __align__(256) unsigned char scratch[ALLOCMOE_STATIC_SCRATCH_BYTES];

allocmoe_status device_state_of_current_device(DeviceState** out) {
    constexpr int kMaxDevices = 64;
    static DeviceState table[kMaxDevices];
    int dev = 0;
    ALLOCMOE_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return ALLOCMOE_EHIP;
    *out = &table[dev];
    return ALLOCMOE_OK;
}

// (state.lock held)
allocmoe_status ensure_side_stream(DeviceState& s) {
    if (s.side != nullptr) return ALLOCMOE_OK;
    hipStream_t st = nullptr;
    ALLOCMOE_TRY(hipStreamCreateWithFlags(&st, hipStreamNonBlocking));
    ALLOCMOE_TRY(hipEventCreateWithFlags(&s.fork, hipEventDisableTiming));
    ALLOCMOE_TRY(hipEventCreateWithFlags(&s.join, hipEventDisableTiming));
    s.side = st;
    return ALLOCMOE_OK;
}

// Records ev[i] (when ev is not null) on a stream.
#define ALLOCMOE_MARK_ON(i, st)                                          \
    do {                                                                 \
        if (ev != nullptr) ALLOCMOE_TRY(hipEventRecord(ev[i], st));      \
    } while (0)
#define ALLOCMOE_MARK(i) ALLOCMOE_MARK_ON(i, stream)
// indices of the side-stream events
constexpr int kEvSide0 = 6, kEvSide1 = 7, kEvSide2 = 8;

// Host-side argument checks of the forward entry points (nothing is enqueued and no
// HIP call is made before they pass).
allocmoe_status validate_forward(const allocmoe_layer_desc* desc, const void* X,
                                 const allocmoe_weights* w, const void* Y, const void* ws,
                                 size_t ws_bytes, allocmoe_ws_layout* L) {
    const allocmoe_status st = layout_of(desc, L);
    if (st != ALLOCMOE_OK) return st;
    if (!X || !Y || !w || !w->Wg) return ALLOCMOE_EINVAL;
    if (desc->dtype == ALLOCMOE_BF16) {
        if (!w->packed || !aligned(w->packed, kAlign)) return ALLOCMOE_EINVAL;
    } else {
        if (!w->W1 || !w->W3 || !w->W2) return ALLOCMOE_EINVAL;
        if (desc->I_shared && (!w->Ws1 || !w->Ws3 || !w->Ws2)) return ALLOCMOE_EINVAL;
    }
    if (desc->shared_gate && !w->w_sg) return ALLOCMOE_EINVAL;
    if (ws == nullptr || ws_bytes < L->total || !aligned(ws, kAlign)) return ALLOCMOE_EWORKSPACE;
    // rows are read and written in 16-byte pieces
    if (!aligned(X, 16) || !aligned(Y, 16)) return ALLOCMOE_EINVAL;
    return ALLOCMOE_OK;
}

// (state.lock held)
allocmoe_status forward_impl(const allocmoe_layer_desc* desc, const void* X,
                             const allocmoe_weights* w, void* Y, void* ws, size_t ws_bytes,
                             allocmoe_stream stream_, DeviceState& state, hipEvent_t* ev) {
    allocmoe_ws_layout L;
    const allocmoe_status st = validate_forward(desc, X, w, Y, ws, ws_bytes, &L);
    if (st != ALLOCMOE_OK) return st;
    const bool bf16 = desc->dtype == ALLOCMOE_BF16;
    const int Is = desc->I_shared;

    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int T = desc->T, d = desc->d, E = desc->E, I = desc->I, K = desc->K;
    const int64_t B = desc->budget;
    const Scratch s = scratch_of(desc);
    char* base = static_cast<char*>(ws);
    char* scr = base + L.scratch;
    float* scores = at<float>(base, L.scores);
    int32_t* topk_ids = at<int32_t>(base, L.topk_ids);
    float* topk_s = at<float>(base, L.topk_s);
    int32_t* keep_count = at<int32_t>(base, L.keep_count);
    float* sgate = desc->shared_gate ? at<float>(base, L.shared_gate) : nullptr;
    int32_t* expert_offsets = at<int32_t>(base, L.expert_offsets);
    int32_t* row_token = at<int32_t>(base, L.row_token);
    int32_t* row_rank = at<int32_t>(base, L.row_rank);
    int32_t* inv_row = at<int32_t>(base, L.inv_row);
    int32_t* tile_info = at<int32_t>(scr, s.tile_info);
    void* H = base + L.H;
    void* Hs = base + L.Hs;
    void* O = base + L.O;
    void* Os = Is ? base + L.Os : nullptr;

    // Kernel choice for step 5 (bf16): experts that see about eight rows or more on
    // average use the register-blocked tile kernel (256-row tiles), otherwise the
    // weight-streaming kernel (32-row tiles); decided per group from the descriptor
    // alone.  Measured on DeepSeek-V2-Lite shapes the two kernels cross between 6
    // and 9 rows per expert for the routed group (B = 6E: 174 us a step streaming,
    // 182 tiled; B = 9E: 200 against 193; B = 12E: 227 against 201), and at about
    // 128 tokens for the shared expert.
    constexpr int64_t kRoutedTiledRowsPerExpert = 8;
    constexpr int kSharedTiledTokens = 128;
    // Both kernels read bf16 or 8-bit weights (one format per layer).
    const bool fp8 = fp8_of(desc);
    const bool tiled_shapes = bf16 && d % 256 == 0 && I % 128 == 0 && Is % 128 == 0;
    const bool routed_tiled = tiled_shapes && B >= kRoutedTiledRowsPerExpert * static_cast<int64_t>(E);
    const bool shared_tiled = tiled_shapes && T >= kSharedTiledTokens;
    const int bm = routed_tiled ? kTileRowsLarge : kTileRowsSmall;
    const int64_t max_tiles = max_tiles_for(desc, bm);
    // The shared expert depends on nothing but X.  Where a group uses the tile kernel
    // (prefill shapes), the shared expert's two GEMMs run on a side stream beside
    // selection and the routed experts' GEMMs, and the streams meet again before the
    // combine: the side stream starts after the routing kernel and the
    // single-workgroup plan kernel is enqueued first, so that it gets a compute unit
    // at once.  Decode shapes (both groups on the weight-streaming kernel) keep one
    // stream and one launch per half for both groups: there the two event waits of a
    // fork and join cost more than the overlap gains.
    const bool overlap = bf16 && Is > 0 && B > 0 && (routed_tiled || shared_tiled);
    struct { hipStream_t stream; hipEvent_t fork, join; } side_{}, *side = &side_;
    StreamGroup s1, s2;   // the shared expert's two GEMMs
    if (bf16 && Is) {
        const PackedLayout p = packed_of(desc);
        const uint16_t* pk = static_cast<const uint16_t*>(w->packed);
        const size_t dd = d, SS = Is;
        s1.A = X; s1.lda = d; s1.Bp = pk + p.ps13; s1.group_stride = 2 * dd * SS; s1.Kd = d;
        s1.N = Is; s1.M_dense = T; s1.C = Hs; s1.ldc = Is;
        s2.A = Hs; s2.lda = Is; s2.Bp = pk + p.ps2; s2.group_stride = SS * dd; s2.Kd = Is;
        s2.N = d; s2.M_dense = T; s2.C = Os; s2.ldc = d;
        if (fp8) {
            const PackedFp8 q = packed_fp8_of(desc);
            const char* pq = static_cast<const char*>(w->packed);
            s1.Bp = pq + q.qs13; s1.scale = reinterpret_cast<const float*>(pq + q.scs13);
            s2.Bp = pq + q.qs2; s2.scale = reinterpret_cast<const float*>(pq + q.scs2);
        }
    }
    const StreamGroup none;
    auto fork_shared_expert = [&]() -> allocmoe_status {
        ALLOCMOE_TRY(hipEventRecord(side->fork, stream));
        ALLOCMOE_TRY(hipStreamWaitEvent(side->stream, side->fork, 0));
        for (int half = 0; half < 2; ++half) {
            const StreamGroup& sh = half == 0 ? s1 : s2;
            ALLOCMOE_MARK_ON(half == 0 ? kEvSide0 : kEvSide1, side->stream);
            ALLOCMOE_TRY(shared_tiled ? launch_ffn_bf16_t256(half == 0, none, sh, side->stream)
                                      : launch_ffn_bf16_stream(half == 0, sh, none, side->stream));
        }
        ALLOCMOE_MARK_ON(kEvSide2, side->stream);
        ALLOCMOE_TRY(hipEventRecord(side->join, side->stream));
        return ALLOCMOE_OK;
    };
    if (overlap) {
        const allocmoe_status sst = ensure_side_stream(state);
        if (sst != ALLOCMOE_OK) return sst;
        side_.stream = state.side;
        side_.fork = state.fork;
        side_.join = state.join;
        if (!shared_tiled) {
            const allocmoe_status fst = fork_shared_expert();
            if (fst != ALLOCMOE_OK) return fst;
        }
    }

    // steps 1-2: scores and sorted candidates
    ALLOCMOE_MARK(ALLOCMOE_STAGE_ROUTE);
    if (bf16) {
        const uint16_t* gp = packed_gate(desc, w->packed);
        ALLOCMOE_TRY(launch_route_mfma(X, gp, w->gate_bias, desc->shared_gate != 0, T, d, E, K,
                                       scores, topk_ids, topk_s, sgate, stream));
    } else {
        ALLOCMOE_TRY(launch_route(desc->dtype, X, w->Wg, w->gate_bias,
                                  desc->shared_gate ? w->w_sg : nullptr, T, d, E, K, scores,
                                  topk_ids, topk_s, sgate, stream));
    }
    if (overlap && shared_tiled) {   // the fork point; the kernels follow the plan kernel
        ALLOCMOE_TRY(hipEventRecord(side->fork, stream));
        ALLOCMOE_TRY(hipStreamWaitEvent(side->stream, side->fork, 0));
    }
    // steps 3-4: Alloc-T selection, dispatch, tile map.  Beside the shared expert's GEMMs
    // (which hide it, and whose workgroups hold every compute unit for tens of
    // microseconds at a time) one workgroup does it in one launch, enqueued before them;
    // otherwise, from kPlanSpreadTokens tokens on, a sequence of short launches over many
    // workgroups.
    const bool spread_plan = plan_spread_bytes(T) > 0 && !overlap;
    ALLOCMOE_MARK(ALLOCMOE_STAGE_PLAN);
    const float* sel_keys = topk_s;   // Alloc-T selects on the scores themselves
    if (selector_of(desc) != ALLOCMOE_SELECT_SCORE) {
        ALLOCMOE_TRY(launch_selector_keys(topk_s, T, K, selector_of(desc), at<float>(base, L.sel_keys),
                                          stream));
        sel_keys = at<float>(base, L.sel_keys);
    }
    ALLOCMOE_TRY(launch_plan(sel_keys, topk_ids, T, K, desc->K_base, B, E, keep_count,
                             expert_offsets, row_token, row_rank, inv_row,
                             at<uint64_t>(scr, s.words), at<int32_t>(scr, s.prefix), bm, tile_info,
                             spread_plan ? scr + s.spread : nullptr, !overlap, stream));
    if (overlap && shared_tiled) {
        for (int half = 0; half < 2; ++half) {
            ALLOCMOE_MARK_ON(half == 0 ? kEvSide0 : kEvSide1, side->stream);
            ALLOCMOE_TRY(launch_ffn_bf16_t256(half == 0, none, half == 0 ? s1 : s2, side->stream));
        }
        ALLOCMOE_MARK_ON(kEvSide2, side->stream);
        ALLOCMOE_TRY(hipEventRecord(side->join, side->stream));
    }
    // step 5: expert networks over the selected rows, then the shared expert
    if (bf16) {
        const PackedLayout p = packed_of(desc);
        const uint16_t* pk = static_cast<const uint16_t*>(w->packed);
        const size_t dd = d, II = I;
        // without the side stream, routed rows and the shared expert's rows share one
        // launch per half where they use the same kernel
        StreamGroup r1, r2;
        if (B > 0) {
            r1.A = X; r1.lda = d; r1.row_map = row_token; r1.Bp = pk + p.p13;
            r1.group_stride = 2 * dd * II; r1.Kd = d; r1.N = I; r1.tile_info = tile_info;
            r1.max_tiles = max_tiles; r1.C = H; r1.ldc = I;
            r2.A = H; r2.lda = I; r2.Bp = pk + p.p2; r2.group_stride = II * dd; r2.Kd = I;
            r2.N = d; r2.tile_info = tile_info; r2.max_tiles = max_tiles; r2.C = O; r2.ldc = d;
            if (fp8) {
                const PackedFp8 q = packed_fp8_of(desc);
                const char* pq = static_cast<const char*>(w->packed);
                r1.Bp = pq + q.q13; r1.scale = reinterpret_cast<const float*>(pq + q.sc13);
                r2.Bp = pq + q.q2; r2.scale = reinterpret_cast<const float*>(pq + q.sc2);
            }
        }
        for (int half = 0; half < 2; ++half) {
            const bool swiglu = half == 0;
            const StreamGroup& r = swiglu ? r1 : r2;
            const StreamGroup& sh = swiglu ? s1 : s2;
            ALLOCMOE_MARK(swiglu ? ALLOCMOE_STAGE_FFN1 : ALLOCMOE_STAGE_FFN2);
            if (overlap) {
                ALLOCMOE_TRY(routed_tiled ? launch_ffn_bf16_t256(swiglu, r, none, stream)
                                          : launch_ffn_bf16_stream(swiglu, r, none, stream));
            } else if (routed_tiled == shared_tiled) {   // one launch covers both groups
                ALLOCMOE_TRY(routed_tiled ? launch_ffn_bf16_t256(swiglu, r, sh, stream)
                                          : launch_ffn_bf16_stream(swiglu, r, sh, stream));
            } else {
                ALLOCMOE_TRY(routed_tiled ? launch_ffn_bf16_t256(swiglu, r, none, stream)
                                          : launch_ffn_bf16_stream(swiglu, r, none, stream));
                ALLOCMOE_TRY(shared_tiled ? launch_ffn_bf16_t256(swiglu, sh, none, stream)
                                          : launch_ffn_bf16_stream(swiglu, sh, none, stream));
            }
        }
        if (overlap) ALLOCMOE_TRY(hipStreamWaitEvent(stream, side->join, 0));
    } else {
        const float* Xf = static_cast<const float*>(X);
        ALLOCMOE_MARK(ALLOCMOE_STAGE_FFN1);
        if (B > 0)
            ALLOCMOE_TRY(launch_ffn_f32(true, Xf, d, row_token, static_cast<const float*>(w->W1),
                                        static_cast<const float*>(w->W3), d, I, tile_info,
                                        s.max_tiles, 0, static_cast<float*>(H), I, stream));
        if (Is)
            ALLOCMOE_TRY(launch_ffn_f32(true, Xf, d, nullptr, static_cast<const float*>(w->Ws1),
                                        static_cast<const float*>(w->Ws3), d, Is, nullptr, 0, T,
                                        static_cast<float*>(Hs), Is, stream));
        ALLOCMOE_MARK(ALLOCMOE_STAGE_FFN2);
        if (B > 0)
            ALLOCMOE_TRY(launch_ffn_f32(false, static_cast<const float*>(H), I, nullptr,
                                        static_cast<const float*>(w->W2), nullptr, I, d, tile_info,
                                        s.max_tiles, 0, static_cast<float*>(O), d, stream));
        if (Is)
            ALLOCMOE_TRY(launch_ffn_f32(false, static_cast<const float*>(Hs), Is, nullptr,
                                        static_cast<const float*>(w->Ws2), nullptr, Is, d, nullptr,
                                        0, T, static_cast<float*>(Os), d, stream));
    }
    // step 6: Eq. (2)
    ALLOCMOE_MARK(ALLOCMOE_STAGE_COMBINE);
    ALLOCMOE_TRY(launch_combine(desc->dtype, O, Os, inv_row, topk_s, keep_count, sgate, T, d, K, Y,
                                stream));
    ALLOCMOE_MARK(5);
    if (ev != nullptr && !overlap)   // nothing ran beside the caller's stream: empty intervals
        for (int i = kEvSide0; i <= kEvSide2; ++i) ALLOCMOE_MARK(i);
    return ALLOCMOE_OK;
}

}  // namespace

extern "C" {

allocmoe_status allocmoe_dispatch_static(const allocmoe_layer_desc* desc, const int32_t* topk_ids,
                                         const int32_t* keep_count, int32_t* expert_offsets,
                                         int32_t* row_token, int32_t* row_rank, int32_t* inv_row,
                                         allocmoe_stream stream_) {
    const allocmoe_status st = check_desc(desc);
    if (st != ALLOCMOE_OK) return st;
    if (!topk_ids || !keep_count || !expert_offsets || !inv_row) return ALLOCMOE_EINVAL;
    if (desc->budget > 0 && (!row_token || !row_rank)) return ALLOCMOE_EINVAL;
    if (desc->T > ALLOCMOE_STATIC_MAX_TOKENS) return ALLOCMOE_ESHAPE;
    const Scratch s = scratch_of(desc);
    if (s.tile_info > ALLOCMOE_STATIC_SCRATCH_BYTES) return ALLOCMOE_ESHAPE;   // words + prefixes
    DeviceState* state = nullptr;
    const allocmoe_status dst = device_state_of_current_device(&state);
    if (dst != ALLOCMOE_OK) return dst;
    unsigned char* base = nullptr;
    {
        std::lock_guard<std::mutex> guard(state->lock);
        if (state->static_scratch == nullptr) {   // once per device, with that device current
            void* p = nullptr;
            ALLOCMOE_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
            if (p == nullptr) return ALLOCMOE_EHIP;
            state->static_scratch = static_cast<unsigned char*>(p);
        }
        base = state->static_scratch;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    ALLOCMOE_TRY(launch_dispatch(topk_ids, keep_count, desc->T, desc->K, desc->E, desc->budget,
                                 expert_offsets, row_token, row_rank, inv_row,
                                 at<uint64_t>(base, s.words), at<int32_t>(base, s.prefix),
                                 kTileRowsSmall, nullptr, true, stream));
    return ALLOCMOE_OK;
}

allocmoe_status allocmoe_moe_forward(const allocmoe_layer_desc* desc, const void* X,
                                     const allocmoe_weights* w, void* Y, void* ws,
                                     size_t ws_bytes, allocmoe_stream stream) {
    allocmoe_ws_layout L;
    const allocmoe_status vst = validate_forward(desc, X, w, Y, ws, ws_bytes, &L);
    if (vst != ALLOCMOE_OK) return vst;
    DeviceState* state = nullptr;
    const allocmoe_status st = device_state_of_current_device(&state);
    if (st != ALLOCMOE_OK) return st;
    std::lock_guard<std::mutex> guard(state->lock);
    return forward_impl(desc, X, w, Y, ws, ws_bytes, stream, *state, nullptr);
}

allocmoe_status allocmoe_moe_forward_timed(const allocmoe_layer_desc* desc, const void* X,
                                           const allocmoe_weights* w, void* Y, void* ws,
                                           size_t ws_bytes, allocmoe_stream stream,
                                           float* stage_ms) {
    if (stage_ms == nullptr) return ALLOCMOE_EINVAL;
    allocmoe_ws_layout L;
    const allocmoe_status vst = validate_forward(desc, X, w, Y, ws, ws_bytes, &L);
    if (vst != ALLOCMOE_OK) return vst;
    DeviceState* state = nullptr;
    const allocmoe_status dst = device_state_of_current_device(&state);
    if (dst != ALLOCMOE_OK) return dst;
    std::lock_guard<std::mutex> guard(state->lock);
    if (!state->have_ev) {
        for (int i = 0; i < kTimedEvents; ++i) ALLOCMOE_TRY(hipEventCreate(&state->ev[i]));
        state->have_ev = true;
    }
    hipEvent_t* ev = state->ev;
    const allocmoe_status st = forward_impl(desc, X, w, Y, ws, ws_bytes, stream, *state, ev);
    if (st != ALLOCMOE_OK) return st;
    // (the end mark of the caller's stream follows the join with the side stream)
    ALLOCMOE_TRY(hipEventSynchronize(ev[5]));
    ALLOCMOE_TRY(hipEventSynchronize(ev[kEvSide2]));
    for (int i = 0; i < 5; ++i) ALLOCMOE_TRY(hipEventElapsedTime(&stage_ms[i], ev[i], ev[i + 1]));
    ALLOCMOE_TRY(hipEventElapsedTime(&stage_ms[ALLOCMOE_STAGE_SHARED_FFN1], ev[kEvSide0], ev[kEvSide1]));
    ALLOCMOE_TRY(hipEventElapsedTime(&stage_ms[ALLOCMOE_STAGE_SHARED_FFN2], ev[kEvSide1], ev[kEvSide2]));
    ALLOCMOE_TRY(hipEventElapsedTime(&stage_ms[ALLOCMOE_STAGE_EXPERT_SPAN], ev[ALLOCMOE_STAGE_PLAN],
                                     ev[ALLOCMOE_STAGE_COMBINE]));
    ALLOCMOE_TRY(hipEventElapsedTime(&stage_ms[ALLOCMOE_STAGE_TOTAL], ev[0], ev[5]));
    return ALLOCMOE_OK;
}

}  // extern "C"
