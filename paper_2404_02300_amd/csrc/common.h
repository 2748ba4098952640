// Internal helpers shared by the HIP translation units of libsdt.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>

#include "../../include/sdt.h"

namespace sdt {

constexpr int WAVE = 64;

// Thread-local error text behind sdt_last_error().
void set_error(const char* fmt, ...);

#define SDT_REQUIRE(cond, code, ...)          \
    do {                                      \
        if (!(cond)) {                        \
            ::sdt::set_error(__VA_ARGS__);    \
            return (code);                    \
        }                                     \
    } while (0)

// Call right after a kernel launch: turns a launch failure into SDT_ERR_HIP.
#define SDT_CHECK_LAUNCH(name)                                                     \
    do {                                                                           \
        hipError_t e__ = hipGetLastError();                                        \
        if (e__ != hipSuccess) {                                                   \
            ::sdt::set_error("%s: launch failed: %s", name, hipGetErrorString(e__)); \
            return SDT_ERR_HIP;                                                    \
        }                                                                          \
    } while (0)

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }

// Bump allocator over a caller-provided workspace (all chunks 256-byte aligned).
struct Arena {
    char* base;
    size_t off = 0;
    explicit Arena(void* p) : base(static_cast<char*>(p)) {}
    template <typename T>
    T* take(size_t count) {
        T* r = base ? reinterpret_cast<T*>(base + off) : nullptr;
        off += align_up(count * sizeof(T), 256);
        return r;
    }
    size_t take_off(size_t bytes) {
        size_t r = off;
        off += align_up(bytes, 256);
        return r;
    }
};

// ---- bf16 <-> fp32 (round to nearest even on the way down) -------------------
struct bf16_t {
    uint16_t bits;
};

__device__ __forceinline__ float bf16_to_f32(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
    uint32_t x = __float_as_uint(f);
    if ((x & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((x >> 16) | 0x40u);  // NaN stays NaN
    x += 0x7FFFu + ((x >> 16) & 1u);
    return (uint16_t)(x >> 16);
}

template <typename T>
__device__ __forceinline__ float to_f32(T v);
template <>
__device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v.bits); }

template <typename T>
__device__ __forceinline__ T from_f32(float v);
template <>
__device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <>
__device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return bf16_t{f32_to_bf16(v)}; }

__device__ __forceinline__ int dev_count(int cap, const int32_t* n_d) {
    int n = n_d ? *n_d : cap;
    return n < cap ? n : cap;
}

inline size_t dtype_size(int32_t dt) { return dt == SDT_BF16 ? 2 : 4; }
inline bool dtype_ok(int32_t dt) { return dt == SDT_F32 || dt == SDT_BF16; }

// ---- internal entry points shared between translation units -------------------
// Sampling of one layer; `map_ready` says the node->local-id map in the
// workspace already holds the destination nodes (chained layers of one step).
struct SampleWs {
    int32_t* map;      // [n_nodes]   global id -> local id in the current frontier, -1 = absent
    uint32_t* bitmap;  // [ceil(n_nodes/32)]  newly reached nodes (all zero between calls)
    int32_t* e_pad;    // [cap_dst*fanout]    sampled global ids, row-padded
    int32_t* m;        // [cap_dst]           sampled count per row
    int32_t* part;     // scan partials
    int32_t* cursor;   // [cap_src] fill cursors of the transposed block
    int32_t* longlist; // [cap_src+1] segments left to the cooperative sorter (+ counter)
};
size_t sample_ws_carve(Arena& a, int64_t n_nodes, int32_t cap_dst, int32_t fanout, SampleWs* out);
int32_t sample_layer(const sdt_csr& g, const int32_t* dst_nodes, int32_t n_dst_cap, const int32_t* n_dst_d,
                     int32_t fanout, uint64_t seed, uint32_t step, uint32_t layer, const sdt_block& out,
                     const SampleWs& ws, bool map_ready, hipStream_t st);
int32_t sample_init_map(const SampleWs& ws, int64_t n_nodes, const int32_t* dst_nodes, int32_t n_dst_cap,
                        const int32_t* n_dst_d, hipStream_t st);

int32_t softmax_xent(const float* logits, int64_t ld, int32_t B, int32_t C, const int32_t* labels,
                     const int32_t* seeds, float* dZ, float* row_loss, float* loss_d, hipStream_t st);
int32_t sgd_update(const sdt_model& m, float* const* dW, float* const* db, float lr, hipStream_t st);

}  // namespace sdt
