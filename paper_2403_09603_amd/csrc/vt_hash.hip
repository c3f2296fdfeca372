// vt_hash.hip -- SHA-256 of the model weights and the Merkle root over checkpoint digests (gfx950).
//
// Method, primitives hash_sha256 and tree; Algorithms "train" / "audit" (a leaf every k steps,
// the root at the end).  A SHA-256 stream is sequential, so the weights are hashed as a tree of
// chunks: every lane hashes one chunk from start to end, the digests of a level are laid out in
// chunk order and become the next level's data, until one chunk is left.  The work is integer
// ALU (about 24 operations per byte), not memory: a lane reads its chunk with 16-byte loads and
// keeps the next block's loads in flight while it compresses the current one.
#include "vt_kernels.h"
#include "vt_sha256.h"

namespace vt {
namespace {

constexpr int kHashThreads = 64;     // one wave per workgroup: chunks spread over all CUs

__device__ __forceinline__ void load_block(const uint4 *p, uint32_t (&w)[16])
{
    const uint4 q0 = p[0], q1 = p[1], q2 = p[2], q3 = p[3];
    w[0] = q0.x; w[1] = q0.y; w[2] = q0.z; w[3] = q0.w;
    w[4] = q1.x; w[5] = q1.y; w[6] = q1.z; w[7] = q1.w;
    w[8] = q2.x; w[9] = q2.y; w[10] = q2.z; w[11] = q2.w;
    w[12] = q3.x; w[13] = q3.y; w[14] = q3.z; w[15] = q3.w;
}

// The digest as bytes: the eight state words, big-endian.
__device__ __forceinline__ void store_digest(const Sha256State &s, uint32_t *out)
{
#pragma unroll
    for (int i = 0; i < 8; ++i) out[i] = sha_bswap(s.h[i]);
}

// Lane t hashes bytes [t * chunk, min((t + 1) * chunk, nbytes)) of `in` and writes the digest to
// out[8 t ..].  `in` is 16-byte aligned and chunk a multiple of 64, so every whole block is four
// aligned 16-byte loads; a ragged end (only the last range can have one) is read byte by byte.
__global__ __launch_bounds__(kHashThreads) void sha256_chunks_kernel(const uint8_t *__restrict__ in, uint64_t nbytes,
                                                                     uint64_t chunk, uint64_t n_chunks,
                                                                     uint32_t *__restrict__ out)
{
    const uint64_t t = (uint64_t)blockIdx.x * kHashThreads + threadIdx.x;
    if (t >= n_chunks) return;
    const uint64_t off = t * chunk;
    const uint64_t len = nbytes - off < chunk ? nbytes - off : chunk;
    const uint64_t blocks = len >> 6;
    const uint4 *p = (const uint4 *)(in + off);
    Sha256State s;
    sha256_init(s);
    uint32_t nxt[16];
    if (blocks) load_block(p, nxt);
#pragma unroll 1
    for (uint64_t b = 0; b < blocks; ++b) {
        uint32_t w[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) w[i] = sha_bswap(nxt[i]);
        if (b + 1 < blocks) load_block(p + 4 * (b + 1), nxt);      // in flight during the 64 rounds below
        sha256_compress(s, w);
    }
    const uint32_t rem = (uint32_t)(len & 63);
    if (rem) sha256_finish_ragged(s, in + off + (blocks << 6), rem, len);
    else sha256_pad_block(s, len);
    store_digest(s, out + 8 * t);
}

// One level of the Merkle tree: parent i = SHA-256(node 2i || node 2i+1); a last node without a
// sibling moves up unchanged.  A 64-byte message is one data block and one constant padding block.
__global__ __launch_bounds__(kHashThreads) void merkle_level_kernel(const uint32_t *__restrict__ nodes, uint64_t n,
                                                                    uint32_t *__restrict__ parents)
{
    const uint64_t t = (uint64_t)blockIdx.x * kHashThreads + threadIdx.x;
    const uint64_t pairs = n >> 1;
    if (t < pairs) {
        uint32_t w[16];
#pragma unroll
        for (int i = 0; i < 16; ++i) w[i] = sha_bswap(nodes[16 * t + i]);
        Sha256State s;
        sha256_init(s);
        sha256_compress(s, w);
        sha256_pad_block(s, 64);
        store_digest(s, parents + 8 * t);
    } else if (t == pairs && (n & 1)) {
#pragma unroll
        for (int i = 0; i < 8; ++i) parents[8 * t + i] = nodes[8 * (n - 1) + i];
    }
}

__global__ void copy_digest_kernel(const uint32_t *__restrict__ src, uint32_t *__restrict__ dst)
{
    if (threadIdx.x < 8) dst[threadIdx.x] = src[threadIdx.x];
}

inline uint64_t ceil_div(uint64_t a, uint64_t b) { return (a + b - 1) / b; }
inline size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

}  // namespace

size_t sha256_tree_bytes(uint64_t nbytes, uint64_t chunk)
{
    if (chunk == 0 || nbytes <= chunk) return 256;
    const uint64_t c0 = ceil_div(nbytes, chunk);                 // digests of the first level
    const uint64_t c1 = ceil_div(32 * c0, chunk);                // and of the second: the two ping-pong buffers
    return align256(32 * c0) + align256(32 * c1);
}

hipError_t launch_sha256_tree(const uint8_t *data, uint64_t nbytes, uint64_t chunk, uint32_t *digest, void *ws,
                              hipStream_t s)
{
    if (chunk == 0) chunk = nbytes > 64 ? (nbytes + 63) & ~(uint64_t)63 : 64;    // flat: one range holds everything
    const uint8_t *level = data;
    uint64_t level_bytes = nbytes;
    uint32_t *buf[2];
    buf[0] = (uint32_t *)ws;
    buf[1] = (uint32_t *)((char *)ws + align256(32 * ceil_div(nbytes > 0 ? nbytes : 1, chunk)));
    int which = 0;
    while (level_bytes > chunk) {
        const uint64_t n_chunks = ceil_div(level_bytes, chunk);
        hipLaunchKernelGGL(sha256_chunks_kernel, dim3((unsigned)ceil_div(n_chunks, kHashThreads)), dim3(kHashThreads), 0, s,
                           level, level_bytes, chunk, n_chunks, buf[which]);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        level = (const uint8_t *)buf[which];
        level_bytes = 32 * n_chunks;
        which ^= 1;
    }
    hipLaunchKernelGGL(sha256_chunks_kernel, dim3(1), dim3(kHashThreads), 0, s, level, level_bytes, chunk, (uint64_t)1, digest);
    return hipGetLastError();
}

size_t merkle_root_bytes(uint64_t n_leaves) { return 2 * align256(32 * ceil_div(n_leaves > 0 ? n_leaves : 1, 2)); }

hipError_t launch_merkle_root(const uint32_t *leaves, uint64_t n_leaves, uint32_t *root, void *ws, hipStream_t s)
{
    const uint32_t *level = leaves;
    uint64_t n = n_leaves;
    uint32_t *buf[2];
    buf[0] = (uint32_t *)ws;
    buf[1] = (uint32_t *)((char *)ws + align256(32 * ceil_div(n_leaves, 2)));
    int which = 0;
    while (n > 1) {
        const uint64_t parents = ceil_div(n, 2);
        uint32_t *dst = parents == 1 ? root : buf[which];
        hipLaunchKernelGGL(merkle_level_kernel, dim3((unsigned)ceil_div(parents, kHashThreads)), dim3(kHashThreads), 0, s,
                           level, n, dst);
        const hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        level = dst;
        n = parents;
        which ^= 1;
    }
    if (n_leaves == 1) {
        hipLaunchKernelGGL(copy_digest_kernel, dim3(1), dim3(64), 0, s, leaves, root);
        return hipGetLastError();
    }
    return hipSuccess;
}

}  // namespace vt
