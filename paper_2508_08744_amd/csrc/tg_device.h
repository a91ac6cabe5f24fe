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

// Value held by lane (lane ^ XOR).  Inside a row of 16 lanes this is one or two DPP moves
// (quad permutations, mirrors of 8 and 16 lanes, rotation by 8); across rows it goes through
// the LDS crossbar.
template <int CTRL>
__device__ inline u64 tg_dpp64(u64 x)
{
    // every lane has a source inside its row for the controls used here, so no fill value is needed
    const u32 lo = (u32)__builtin_amdgcn_mov_dpp((int)(u32)x, CTRL, 0xF, 0xF, true);
    const u32 hi = (u32)__builtin_amdgcn_mov_dpp((int)(u32)(x >> 32), CTRL, 0xF, 0xF, true);
    return ((u64)hi << 32) | lo;
}
template <int XOR>
__device__ inline u64 tg_partner(u64 x)
{
    if (XOR == 1) return tg_dpp64<0xB1>(x);                     // quad_perm 1,0,3,2
    if (XOR == 2) return tg_dpp64<0x4E>(x);                     // quad_perm 2,3,0,1
    if (XOR == 3) return tg_dpp64<0x1B>(x);                     // quad_perm 3,2,1,0
    if (XOR == 4) return tg_dpp64<0x1B>(tg_dpp64<0x141>(x));    // mirror of 8, then of 4: 7 ^ 3
    if (XOR == 7) return tg_dpp64<0x141>(x);                    // row_half_mirror
    if (XOR == 8) return tg_dpp64<0x128>(x);                    // row_ror 8
    if (XOR == 15) return tg_dpp64<0x140>(x);                   // row_mirror
    return tg_shfl_xor64(x, XOR);
}
// one compare-exchange: the lane keeps the smaller of (key, other) if keep_min, else the larger
__device__ inline u64 tg_cmpx(u64 key, u64 other, bool keep_min)
{
    const bool lt = key < other;
    return (lt != keep_min) ? other : key;
}
template <int SIZE>
__device__ inline u64 tg_sort_level(u64 key, int lane)
{
    // blocks of SIZE lanes: fold each block onto itself, then clean its halves
    key = tg_cmpx(key, tg_partner<SIZE - 1>(key), (lane & (SIZE >> 1)) == 0);
    if (SIZE >= 64) key = tg_cmpx(key, tg_partner<16>(key), (lane & 16) == 0);
    if (SIZE >= 32) key = tg_cmpx(key, tg_partner<8>(key), (lane & 8) == 0);
    if (SIZE >= 16) key = tg_cmpx(key, tg_partner<4>(key), (lane & 4) == 0);
    if (SIZE >= 8) key = tg_cmpx(key, tg_partner<2>(key), (lane & 2) == 0);
    if (SIZE >= 4) key = tg_cmpx(key, tg_partner<1>(key), (lane & 1) == 0);
    return key;
}
// Ascending bitonic sort of one key per lane across the wave.
__device__ inline u64 tg_wave_sort(u64 key)
{
    const int lane = tg_lane();
    key = tg_sort_level<2>(key, lane);
    key = tg_sort_level<4>(key, lane);
    key = tg_sort_level<8>(key, lane);
    key = tg_sort_level<16>(key, lane);
    key = tg_sort_level<32>(key, lane);
    key = tg_sort_level<64>(key, lane);
    return key;
}

// a and b are ascending across the wave; returns the 64 smallest keys of their union,
// ascending (the wave-level form of the rank merge of section 4.2).
__device__ inline u64 tg_wave_merge_low(u64 a, u64 b)
{
    const int lane = tg_lane();
    u64 x = tg_min64(a, tg_partner<63>(b));
    x = tg_cmpx(x, tg_partner<32>(x), (lane & 32) == 0);
    x = tg_cmpx(x, tg_partner<16>(x), (lane & 16) == 0);
    x = tg_cmpx(x, tg_partner<8>(x), (lane & 8) == 0);
    x = tg_cmpx(x, tg_partner<4>(x), (lane & 4) == 0);
    x = tg_cmpx(x, tg_partner<2>(x), (lane & 2) == 0);
    x = tg_cmpx(x, tg_partner<1>(x), (lane & 1) == 0);
    return x;
}

// The same network on 32-bit keys: compare-exchange is one v_min / v_max with a DPP operand.
template <int CTRL>
__device__ inline u32 tg_dpp32(u32 x)
{
    return (u32)__builtin_amdgcn_mov_dpp((int)x, CTRL, 0xF, 0xF, true);
}
template <int XOR>
__device__ inline u32 tg_partner32(u32 x)
{
    if (XOR == 1) return tg_dpp32<0xB1>(x);
    if (XOR == 2) return tg_dpp32<0x4E>(x);
    if (XOR == 3) return tg_dpp32<0x1B>(x);
    if (XOR == 4) return tg_dpp32<0x1B>(tg_dpp32<0x141>(x));
    if (XOR == 7) return tg_dpp32<0x141>(x);
    if (XOR == 8) return tg_dpp32<0x128>(x);
    if (XOR == 15) return tg_dpp32<0x140>(x);
    return (u32)__shfl_xor((int)x, XOR);
}
__device__ inline u32 tg_cmpx32(u32 key, u32 other, bool keep_min) { return keep_min ? min(key, other) : max(key, other); }
template <int SIZE>
__device__ inline u32 tg_sort_level32(u32 key, int lane)
{
    key = tg_cmpx32(key, tg_partner32<SIZE - 1>(key), (lane & (SIZE >> 1)) == 0);
    if (SIZE >= 64) key = tg_cmpx32(key, tg_partner32<16>(key), (lane & 16) == 0);
    if (SIZE >= 32) key = tg_cmpx32(key, tg_partner32<8>(key), (lane & 8) == 0);
    if (SIZE >= 16) key = tg_cmpx32(key, tg_partner32<4>(key), (lane & 4) == 0);
    if (SIZE >= 8) key = tg_cmpx32(key, tg_partner32<2>(key), (lane & 2) == 0);
    if (SIZE >= 4) key = tg_cmpx32(key, tg_partner32<1>(key), (lane & 1) == 0);
    return key;
}
// Ascending bitonic sort of one 32-bit key per lane across the wave.
__device__ inline u32 tg_wave_sort32(u32 key)
{
    const int lane = tg_lane();
    key = tg_sort_level32<2>(key, lane);
    key = tg_sort_level32<4>(key, lane);
    key = tg_sort_level32<8>(key, lane);
    key = tg_sort_level32<16>(key, lane);
    key = tg_sort_level32<32>(key, lane);
    key = tg_sort_level32<64>(key, lane);
    return key;
}

__device__ inline u64 tg_lanemask_lt() { return (1ull << tg_lane()) - 1ull; }
