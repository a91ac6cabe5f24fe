// Device-side building blocks shared by the kernels: the counter-based hash, the
// 64-bit (distance, id) sort key, and wave-level sort / merge networks.
// gfx950 only: wavefronts are 64 lanes wide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
typedef unsigned int u32;

#define TG_WAVE 64
#define TG_EMPTY_KEY 0xFFFFFFFFFFFFFFFFull
#define TG_GOLDEN 0x9E3779B97F4A7C15ull
#define TG_ID_MASK 0x7FFFFFFFu     // list word: id in bits 0..30, "fresh" mark in bit 31

// tags of the three random decisions (initial lists, reverse priority, candidate slot)
#define TG_TAG_INIT 1ull
#define TG_TAG_REV(round) (2ull + 4ull * (u64)(round))
#define TG_TAG_SLOT(round) (3ull + 4ull * (u64)(round))

// SplitMix64 output function (Steele, Lea, Flood 2014).
__host__ __device__ inline u64 tg_mix64(u64 z)
{
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// hash(seed, tag, x, y) = mix(mix(mix(seed + tag*golden) + x) + y); the first mix is
// done once on the host per round and passed in as `hs`.
__host__ __device__ inline u64 tg_hash_seed(u64 seed, u64 tag) { return tg_mix64(seed + tag * TG_GOLDEN); }
__device__ inline u64 tg_hash_xy(u64 hs, u64 x, u64 y) { return tg_mix64(tg_mix64(hs + x) + y); }

// Order-preserving map fp32 -> u32 (works for negative values; -0 is folded into +0).
__device__ inline u32 tg_ord(float f)
{
    f += 0.0f;
    u32 b = __float_as_uint(f);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float tg_unord(u32 o)
{
    u32 b = (o & 0x80000000u) ? (o & 0x7FFFFFFFu) : ~o;
    return __uint_as_float(b);
}

// 64-bit key: [63:32] ordered distance bits, [31:2] id, [1] came-from-candidate, [0] fresh.
// Ids are distinct inside any one comparison set, so the two low bits never decide.
__device__ inline u64 tg_key(float dist, u32 id, u32 low2) { return ((u64)tg_ord(dist) << 32) | (u64)((id << 2) | low2); }
__device__ inline u32 tg_key_id(u64 key) { return ((u32)key) >> 2; }
__device__ inline float tg_key_dist(u64 key) { return tg_unord((u32)(key >> 32)); }

__device__ inline int tg_lane() { return (int)__lane_id(); }

__device__ inline u64 tg_shfl64(u64 x, int src)
{
    u32 lo = (u32)__shfl((int)(u32)x, src);
    u32 hi = (u32)__shfl((int)(u32)(x >> 32), src);
    return ((u64)hi << 32) | lo;
}
__device__ inline u64 tg_shfl_xor64(u64 x, int mask)
{
    u32 lo = (u32)__shfl_xor((int)(u32)x, mask);
    u32 hi = (u32)__shfl_xor((int)(u32)(x >> 32), mask);
    return ((u64)hi << 32) | lo;
}
__device__ inline u64 tg_min64(u64 a, u64 b) { return a < b ? a : b; }
__device__ inline u64 tg_max64(u64 a, u64 b) { return a < b ? b : a; }

// Ascending bitonic sort of one key per lane across the wave.
__device__ inline u64 tg_wave_sort(u64 key)
{
    const int lane = tg_lane();
#pragma unroll
    for (int size = 2; size <= TG_WAVE; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            u64 other = tg_shfl_xor64(key, stride);
            bool up = (lane & size) == 0;
            bool lower = (lane & stride) == 0;
            key = (up == lower) ? tg_min64(key, other) : tg_max64(key, other);
        }
    }
    return key;
}

// a and b are ascending across the wave; returns the 64 smallest keys of their union,
// ascending (the wave-level form of the rank merge of section 4.2).
__device__ inline u64 tg_wave_merge_low(u64 a, u64 b)
{
    const int lane = tg_lane();
    u64 x = tg_min64(a, tg_shfl64(b, TG_WAVE - 1 - lane));
#pragma unroll
    for (int stride = TG_WAVE / 2; stride > 0; stride >>= 1) {
        u64 other = tg_shfl_xor64(x, stride);
        x = ((lane & stride) == 0) ? tg_min64(x, other) : tg_max64(x, other);
    }
    return x;
}

__device__ inline u64 tg_lanemask_lt() { return (1ull << tg_lane()) - 1ull; }
