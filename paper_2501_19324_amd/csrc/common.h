// Shared device helpers: bf16 storage type, 8-element loads, wave reductions.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <type_traits>

#define RSD_WAVE 64

struct bf16_t { uint16_t v; };

__device__ __forceinline__ float bf2f(uint16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// fp32 -> bf16, round to nearest even (inputs are finite)
__device__ __forceinline__ uint16_t f2bf(float f) {
    uint32_t u = __float_as_uint(f);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

__device__ __forceinline__ void load8(const float* __restrict__ p, float o[8]) {
    const float4 a = *reinterpret_cast<const float4*>(p);
    const float4 b = *reinterpret_cast<const float4*>(p + 4);
    o[0] = a.x; o[1] = a.y; o[2] = a.z; o[3] = a.w;
    o[4] = b.x; o[5] = b.y; o[6] = b.z; o[7] = b.w;
}

__device__ __forceinline__ void unpack8(const uint4 r, float o[8]) {
    o[0] = __uint_as_float(r.x << 16); o[1] = __uint_as_float(r.x & 0xFFFF0000u);
    o[2] = __uint_as_float(r.y << 16); o[3] = __uint_as_float(r.y & 0xFFFF0000u);
    o[4] = __uint_as_float(r.z << 16); o[5] = __uint_as_float(r.z & 0xFFFF0000u);
    o[6] = __uint_as_float(r.w << 16); o[7] = __uint_as_float(r.w & 0xFFFF0000u);
}

__device__ __forceinline__ void load8(const bf16_t* __restrict__ p, float o[8]) {
    unpack8(*reinterpret_cast<const uint4*>(p), o);
}

__device__ __forceinline__ float ld1(const float* p) { return *p; }
__device__ __forceinline__ float ld1(const bf16_t* p) { return bf2f(p->v); }
__device__ __forceinline__ void st1(float* p, float v) { *p = v; }
__device__ __forceinline__ void st1(bf16_t* p, float v) { p->v = f2bf(v); }

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, RSD_WAVE);
    return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, RSD_WAVE));
    return v;
}

// Sum over the 64 lanes with cross-lane register moves (no LDS traffic).  All 64 lanes must be
// active; every lane gets the result.
__device__ __forceinline__ float wave_sum_dpp(float v) {
    auto dpp_add = [](float x, auto ctrl) {
        return x + __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), decltype(ctrl)::value, 0xF, 0xF, true));
    };
    v = dpp_add(v, std::integral_constant<int, 0xB1>{});    // quad_perm [1,0,3,2]
    v = dpp_add(v, std::integral_constant<int, 0x4E>{});    // quad_perm [2,3,0,1]
    v = dpp_add(v, std::integral_constant<int, 0x141>{});   // row_half_mirror
    v = dpp_add(v, std::integral_constant<int, 0x140>{});   // row_mirror: each row of 16 lanes holds its sum
    const int bits = __float_as_int(v);
    return (__int_as_float(__builtin_amdgcn_readlane(bits, 0)) + __int_as_float(__builtin_amdgcn_readlane(bits, 16))) +
           (__int_as_float(__builtin_amdgcn_readlane(bits, 32)) + __int_as_float(__builtin_amdgcn_readlane(bits, 48)));
}

// Reductions over the four 16-lane rows of a wave (lanes l, l+16, l+32, l+48), register moves only:
// a swap of odd/even rows, then of the two wave halves.  Every lane gets the result.
__device__ __forceinline__ float rows4_max(float v) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = fmaxf(__uint_as_float(a[0]), __uint_as_float(a[1]));
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return fmaxf(__uint_as_float(b[0]), __uint_as_float(b[1]));
}
__device__ __forceinline__ float rows4_sum(float v) {
    const auto a = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = __uint_as_float(a[0]) + __uint_as_float(a[1]);
    const auto b = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return __uint_as_float(b[0]) + __uint_as_float(b[1]);
}

// Sum over a 256-thread block; `red` is 4 floats of LDS. All threads get the result.
__device__ __forceinline__ float block256_sum(float v, float* red) {
    v = wave_sum(v);
    __syncthreads();
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = v;
    __syncthreads();
    return red[0] + red[1] + red[2] + red[3];
}

// Row descriptor shared by the per-row kernels.  Chunked prefill passes give
// explicit (sequence, position) arrays; single-token decode passes leave them
// null: row r is sequence r, fed at position kv_len[r], skipped when inactive.
// Which sequence and which position a row of a pass stands for.
//   chunked pass:   row_seq[r], row_pos[r] (every row is in use)
//   decode, dense:  row r is sequence r at position kv_len[r], in use while active[r]
//   decode, packed: row r is sequence row_seq[r] (< 0: unused row) at kv_len[seq], in use while active[seq]
struct RowMap {
    const int* row_seq;
    const int* row_pos;
    const int* kv_len;
    const int* active;
};
__device__ __forceinline__ bool row_lookup(const RowMap& rm, int r, int& seq, int& pos) {
    if (rm.row_seq) {
        seq = rm.row_seq[r];
        if (rm.row_pos) { pos = rm.row_pos[r]; return true; }
        if (seq < 0) return false;
        pos = rm.kv_len[seq];
        return rm.active[seq] != 0;
    }
    seq = r; pos = rm.kv_len[r];
    return rm.active[r] != 0;
}
