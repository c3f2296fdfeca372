// vt_sha256.h -- SHA-256 (FIPS 180-4) on 32-bit integer registers, for one lane.
//
// The method hashes the model weights at every checkpoint (Method, primitive hash_sha256) and
// keeps the digests in a Merkle tree (primitive tree; Algorithms "train" and "audit" append a
// leaf every k steps and return the root).  SHA-256 itself is sequential over its 64-byte
// blocks, so a lane hashes one byte range from start to end; parallelism comes from hashing
// many ranges at once (chunks of the weights, pairs of tree nodes).
//
// The message schedule lives in 16 registers and the 64 rounds are unrolled, so the round
// constants are instruction literals and no array is indexed dynamically.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace vt {

struct Sha256State {
    uint32_t h[8];
};

static __host__ __device__ __forceinline__ void sha256_init(Sha256State &s)
{
    s.h[0] = 0x6a09e667u; s.h[1] = 0xbb67ae85u; s.h[2] = 0x3c6ef372u; s.h[3] = 0xa54ff53au;
    s.h[4] = 0x510e527fu; s.h[5] = 0x9b05688cu; s.h[6] = 0x1f83d9abu; s.h[7] = 0x5be0cd19u;
}

static __host__ __device__ __forceinline__ uint32_t sha_rotr(uint32_t x, uint32_t n) { return (x >> n) | (x << (32u - n)); }
static __host__ __device__ __forceinline__ uint32_t sha_bswap(uint32_t x) { return __builtin_bswap32(x); }
// a ^ b ^ c: one three-input bit operation on the GPU (truth table 0x96); the host build of this
// header (CPU checks of the routines) takes two.
static __host__ __device__ __forceinline__ uint32_t sha_xor3(uint32_t a, uint32_t b, uint32_t c)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_bitop3_b32(a, b, c, 0x96);
#else
    return a ^ b ^ c;
#endif
}
// Ch(e, f, g): f where e is set, g elsewhere (truth table 0xCA with inputs 0xF0, 0xCC, 0xAA).
static __host__ __device__ __forceinline__ uint32_t sha_ch(uint32_t e, uint32_t f, uint32_t g)
{
#if defined(__HIP_DEVICE_COMPILE__)
    return __builtin_amdgcn_bitop3_b32(e, f, g, 0xCA);
#else
    return g ^ (e & (f ^ g));
#endif
}

// One round with the working variables renamed instead of moved: the caller rotates the
// argument order, so nothing is copied between rounds.
#define VT_SHA_ROUND(a, b, c, d, e, f, g, h, k, w)                                              \
    do {                                                                                        \
        const uint32_t t1 = (h) + sha_xor3(sha_rotr((e), 6), sha_rotr((e), 11), sha_rotr((e), 25)) + \
                            sha_ch((e), (f), (g)) + (k) + (w);                                  \
        const uint32_t t2 = sha_xor3(sha_rotr((a), 2), sha_rotr((a), 13), sha_rotr((a), 22)) +  \
                            (((a) & (b)) | ((c) & ((a) | (b))));                                \
        (d) += t1;                                                                              \
        (h) = t1 + t2;                                                                          \
    } while (0)

// w[i & 15] becomes W[i] for i >= 16: sigma1(W[i-2]) + W[i-7] + sigma0(W[i-15]) + W[i-16]
#define VT_SHA_SCHED(w, i)                                                                       \
    ((w)[(i) & 15] += sha_xor3(sha_rotr((w)[((i) - 2) & 15], 17), sha_rotr((w)[((i) - 2) & 15], 19), \
                               (w)[((i) - 2) & 15] >> 10) +                                      \
                      (w)[((i) - 7) & 15] +                                                      \
                      sha_xor3(sha_rotr((w)[((i) - 15) & 15], 7), sha_rotr((w)[((i) - 15) & 15], 18), \
                               (w)[((i) - 15) & 15] >> 3))

#define VT_SHA_8ROUNDS(i, k0, k1, k2, k3, k4, k5, k6, k7)  \
    VT_SHA_ROUND(a, b, c, d, e, f, g, h, k0, w[(i) + 0]);  \
    VT_SHA_ROUND(h, a, b, c, d, e, f, g, k1, w[(i) + 1]);  \
    VT_SHA_ROUND(g, h, a, b, c, d, e, f, k2, w[(i) + 2]);  \
    VT_SHA_ROUND(f, g, h, a, b, c, d, e, k3, w[(i) + 3]);  \
    VT_SHA_ROUND(e, f, g, h, a, b, c, d, k4, w[(i) + 4]);  \
    VT_SHA_ROUND(d, e, f, g, h, a, b, c, k5, w[(i) + 5]);  \
    VT_SHA_ROUND(c, d, e, f, g, h, a, b, k6, w[(i) + 6]);  \
    VT_SHA_ROUND(b, c, d, e, f, g, h, a, k7, w[(i) + 7])

#define VT_SHA_8SCHED(i)                                                                       \
    VT_SHA_SCHED(w, (i) + 0); VT_SHA_SCHED(w, (i) + 1); VT_SHA_SCHED(w, (i) + 2); VT_SHA_SCHED(w, (i) + 3); \
    VT_SHA_SCHED(w, (i) + 4); VT_SHA_SCHED(w, (i) + 5); VT_SHA_SCHED(w, (i) + 6); VT_SHA_SCHED(w, (i) + 7)

// The compression function on one 64-byte block given as 16 big-endian words (w is consumed).
static __host__ __device__ __forceinline__ void sha256_compress(Sha256State &s, uint32_t (&w)[16])
{
    uint32_t a = s.h[0], b = s.h[1], c = s.h[2], d = s.h[3], e = s.h[4], f = s.h[5], g = s.h[6], h = s.h[7];
    VT_SHA_8ROUNDS(0, 0x428a2f98u, 0x71374491u, 0xb5c0fbcfu, 0xe9b5dba5u, 0x3956c25bu, 0x59f111f1u, 0x923f82a4u, 0xab1c5ed5u);
    VT_SHA_8ROUNDS(8, 0xd807aa98u, 0x12835b01u, 0x243185beu, 0x550c7dc3u, 0x72be5d74u, 0x80deb1feu, 0x9bdc06a7u, 0xc19bf174u);
    VT_SHA_8SCHED(16); VT_SHA_8SCHED(24);
    VT_SHA_8ROUNDS(0, 0xe49b69c1u, 0xefbe4786u, 0x0fc19dc6u, 0x240ca1ccu, 0x2de92c6fu, 0x4a7484aau, 0x5cb0a9dcu, 0x76f988dau);
    VT_SHA_8ROUNDS(8, 0x983e5152u, 0xa831c66du, 0xb00327c8u, 0xbf597fc7u, 0xc6e00bf3u, 0xd5a79147u, 0x06ca6351u, 0x14292967u);
    VT_SHA_8SCHED(32); VT_SHA_8SCHED(40);
    VT_SHA_8ROUNDS(0, 0x27b70a85u, 0x2e1b2138u, 0x4d2c6dfcu, 0x53380d13u, 0x650a7354u, 0x766a0abbu, 0x81c2c92eu, 0x92722c85u);
    VT_SHA_8ROUNDS(8, 0xa2bfe8a1u, 0xa81a664bu, 0xc24b8b70u, 0xc76c51a3u, 0xd192e819u, 0xd6990624u, 0xf40e3585u, 0x106aa070u);
    VT_SHA_8SCHED(48); VT_SHA_8SCHED(56);
    VT_SHA_8ROUNDS(0, 0x19a4c116u, 0x1e376c08u, 0x2748774cu, 0x34b0bcb5u, 0x391c0cb3u, 0x4ed8aa4au, 0x5b9cca4fu, 0x682e6ff3u);
    VT_SHA_8ROUNDS(8, 0x748f82eeu, 0x78a5636fu, 0x84c87814u, 0x8cc70208u, 0x90befffau, 0xa4506cebu, 0xbef9a3f7u, 0xc67178f2u);
    s.h[0] += a; s.h[1] += b; s.h[2] += c; s.h[3] += d; s.h[4] += e; s.h[5] += f; s.h[6] += g; s.h[7] += h;
}

// The block that ends a message whose length is a multiple of 64 bytes: 0x80, zeros, and the
// length in bits as a 64-bit big-endian integer.
static __host__ __device__ __forceinline__ void sha256_pad_block(Sha256State &s, uint64_t total_bytes)
{
    uint32_t w[16];
#pragma unroll
    for (int i = 1; i < 14; ++i) w[i] = 0;
    w[0] = 0x80000000u;
    w[14] = (uint32_t)((total_bytes << 3) >> 32);
    w[15] = (uint32_t)(total_bytes << 3);
    sha256_compress(s, w);
}

// Ends a message of total_bytes whose last rem = total_bytes % 64 bytes (rem > 0) start at `tail`.
// Byte loads: this runs once per ragged range, not in the streaming loop.
static __host__ __device__ inline void sha256_finish_ragged(Sha256State &s, const uint8_t *tail, uint32_t rem,
                                                            uint64_t total_bytes)
{
    uint32_t w[16];
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        uint32_t v = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const uint32_t p = 4u * (uint32_t)i + (uint32_t)j;
            const uint32_t byte = p < rem ? (uint32_t)tail[p] : (p == rem ? 0x80u : 0u);
            v = (v << 8) | byte;
        }
        w[i] = v;
    }
    if (rem >= 56) {                  // no room for the length: it goes into a block of its own
        sha256_compress(s, w);
#pragma unroll
        for (int i = 0; i < 14; ++i) w[i] = 0;
    }
    w[14] = (uint32_t)((total_bytes << 3) >> 32);
    w[15] = (uint32_t)(total_bytes << 3);
    sha256_compress(s, w);
}

}  // namespace vt
