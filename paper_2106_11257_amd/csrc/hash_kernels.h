// Partition hashes hash(g_i[j]) / hash(g^[j]) (the commitments of Alg. 2, lines 2 and 6).
//
// The paper asks for "a cryptographic hash function" and names none.  Here it is SHA-256
// (FIPS 180-4) arranged as a tree so that a partition of megabytes is hashed by thousands
// of lanes instead of one:
//   level 0: the partition's bytes (fp32 values as they lie in memory, little-endian) are
//            cut into chunks of 1024 bytes (the last one may be shorter; an empty partition
//            is one empty chunk); every chunk's SHA-256 is a node;
//   level k + 1: if a partition has more than one node at level k, every run of 32
//            consecutive node digests (the last run may be shorter) is hashed into one node:
//            SHA-256 of their concatenation; a partition with a single node keeps it;
//   the hash of the partition is its single remaining node.  A partition of at most 1024
//   bytes is therefore hashed by plain SHA-256.  (No node hashes more than 1 KiB: a lane's
//   chain of dependent compressions stays short, which is what bounds the time for a single
//   row such as the aggregate.)
// One lane hashes one node.  All message lengths are multiples of 4 bytes, so the padding
// starts on a word boundary.  The work is bound by the 32-bit integer ALU (about 31
// instructions per byte, 22 on gfx950 with its three-input bit operations), not by memory.
#pragma once

#include "kernels_common.h"

namespace btard {

constexpr int kHashChunkBytes = 1024;
constexpr int kHashFanout = 32;
constexpr int kDigestBytes = 32;
constexpr int kDigestWords = 8;

__device__ __constant__ uint32_t kSha256K[64] = {
    0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u,
    0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u,
    0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau,
    0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u,
    0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u,
    0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u,
    0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u,
    0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u};

// (dword-aligned 128-bit access, as for the rows of the slab)
typedef uint32_t u32x4_u __attribute__((ext_vector_type(4), aligned(4)));

__device__ __forceinline__ uint32_t rotr32(uint32_t x, int r) { return (x >> r) | (x << (32 - r)); }

// Three-input bitwise functions in one v_bitop3_b32 each; the truth table's bit
// (4 a + 2 b + c) is the result for the input bits (a, b, c).
__device__ __forceinline__ uint32_t xor3(uint32_t a, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)a, (int)b, (int)c, 0x96);
}
__device__ __forceinline__ uint32_t choose(uint32_t e, uint32_t f, uint32_t g)      // e ? f : g
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)e, (int)f, (int)g, 0xCA);
}
__device__ __forceinline__ uint32_t majority(uint32_t a, uint32_t b, uint32_t c)
{
    return (uint32_t)__builtin_amdgcn_bitop3_b32((int)a, (int)b, (int)c, 0xE8);
}

// One SHA-256 compression: state += F(state, the 16 big-endian words w[]).
__device__ __forceinline__ void sha256_compress(uint32_t (&st)[8], uint32_t (&w)[16])
{
    uint32_t a = st[0], b = st[1], c = st[2], d = st[3], e = st[4], f = st[5], g = st[6], h = st[7];
#pragma unroll
    for (int t = 0; t < 64; ++t) {
        if (t >= 16) {
            const uint32_t w15 = w[(t + 1) & 15], w2 = w[(t + 14) & 15];
            const uint32_t s0 = xor3(rotr32(w15, 7), rotr32(w15, 18), w15 >> 3);
            const uint32_t s1 = xor3(rotr32(w2, 17), rotr32(w2, 19), w2 >> 10);
            w[t & 15] = w[t & 15] + s0 + w[(t + 9) & 15] + s1;
        }
        const uint32_t S1 = xor3(rotr32(e, 6), rotr32(e, 11), rotr32(e, 25));
        const uint32_t ch = choose(e, f, g);
        const uint32_t t1 = h + S1 + ch + kSha256K[t] + w[t & 15];
        const uint32_t S0 = xor3(rotr32(a, 2), rotr32(a, 13), rotr32(a, 22));
        const uint32_t maj = majority(a, b, c);
        const uint32_t t2 = S0 + maj;
        h = g; g = f; f = e; e = d + t1; d = c; c = b; b = a; a = t1 + t2;
    }
    st[0] += a; st[1] += b; st[2] += c; st[3] += d; st[4] += e; st[5] += f; st[6] += g; st[7] += h;
}

// SHA-256 of `words` 32-bit words at p (4-byte aligned device memory, read as bytes in
// memory order); the digest as 8 words whose bytes in memory order are the digest's bytes.
__device__ __forceinline__ void sha256_words(const uint32_t *__restrict__ p, int64_t words,
                                             uint32_t (&out)[8])
{
    uint32_t st[8] = {0x6a09e667u, 0xbb67ae85u, 0x3c6ef372u, 0xa54ff53au,
                      0x510e527fu, 0x9b05688cu, 0x1f83d9abu, 0x5be0cd19u};
    uint32_t w[16];
    const int64_t full = words / 16;
#pragma unroll 1
    for (int64_t b = 0; b < full; ++b) {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4_u t = *reinterpret_cast<const u32x4_u *>(p + b * 16 + q * 4);
            w[4 * q + 0] = __builtin_bswap32(t.x);
            w[4 * q + 1] = __builtin_bswap32(t.y);
            w[4 * q + 2] = __builtin_bswap32(t.z);
            w[4 * q + 3] = __builtin_bswap32(t.w);
        }
        sha256_compress(st, w);
    }
    // the last block(s): the remaining words, 0x80, zeros, the length in bits
    const int rem = (int)(words - full * 16);
#pragma unroll
    for (int k = 0; k < 16; ++k) {
        uint32_t x = 0u;
        if (k < rem) x = __builtin_bswap32(p[full * 16 + k]);
        else if (k == rem) x = 0x80000000u;
        w[k] = x;
    }
    const uint64_t bits = (uint64_t)words * 32u;
    if (rem >= 14) {                     // no room for the length: it goes into one more block
        sha256_compress(st, w);
#pragma unroll
        for (int k = 0; k < 16; ++k) w[k] = 0u;
    }
    w[14] = (uint32_t)(bits >> 32);
    w[15] = (uint32_t)bits;
    sha256_compress(st, w);
#pragma unroll
    for (int k = 0; k < 8; ++k) out[k] = __builtin_bswap32(st[k]);
}

struct HashArgs {
    // level 0 input: the slab
    const float *g;
    int64_t ld;
    const int64_t *off;          // [P + 1] partition offsets (coordinates)
    // level k > 0 input: the digests of level k - 1, [n][total_in] x 32 bytes
    const uint32_t *in;
    const int64_t *node_in;      // [P + 1] prefix sums of the partitions' node counts at level k - 1
    int64_t total_in;
    // output: [n][total_out] x 32 bytes
    uint32_t *out;
    const int64_t *node_out;     // [P + 1] prefix sums at this level
    int64_t total_out;
    int32_t n, P, level;
};

// partition j with node[j] <= r < node[j + 1] (node counts are >= 1, so it is unique)
__device__ __forceinline__ int hash_find_partition(const int64_t *node, int P, int64_t r)
{
    int lo = 0, hi = P;                  // invariant: node[lo] <= r < node[hi]
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (node[mid] <= r) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ __launch_bounds__(kBlock) void hash_level_kernel(HashArgs a)
{
    const int64_t t = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (t >= (int64_t)a.n * a.total_out) return;
    const int i = (int)(t / a.total_out);
    const int64_t r = t - (int64_t)i * a.total_out;
    const int j = hash_find_partition(a.node_out, a.P, r);
    const int64_t m = r - a.node_out[j];                         // node index within the partition
    uint32_t dig[8];
    if (a.level == 0) {
        const int64_t words = a.off[j + 1] - a.off[j];
        const int64_t first = m * (kHashChunkBytes / 4);
        int64_t len = words - first;
        if (len > kHashChunkBytes / 4) len = kHashChunkBytes / 4;
        if (len < 0) len = 0;
        const uint32_t *p = reinterpret_cast<const uint32_t *>(a.g + (int64_t)i * a.ld + a.off[j]) + first;
        sha256_words(p, len, dig);
    } else {
        const int64_t cnt_in = a.node_in[j + 1] - a.node_in[j];
        const uint32_t *src = a.in + ((int64_t)i * a.total_in + a.node_in[j]) * kDigestWords;
        if (cnt_in <= 1) {
#pragma unroll
            for (int k = 0; k < 8; ++k) dig[k] = src[k];         // a single node is kept
        } else {
            const int64_t first = m * kHashFanout;
            int64_t len = cnt_in - first;
            if (len > kHashFanout) len = kHashFanout;
            sha256_words(src + first * kDigestWords, len * kDigestWords, dig);
        }
    }
    uint32_t *dst = a.out + ((int64_t)i * a.total_out + r) * kDigestWords;
#pragma unroll
    for (int k = 0; k < 8; ++k) dst[k] = dig[k];
}

}  // namespace btard
