// Measurement aid, not part of the library: what HBM rate can ANY kernel with the codec's byte mix reach on
// this device?  Copy kernels that move the bytes of one fused step of the 1-bit channel-scale codec on
// [4096, 3072] bf16 tensors (per element: read x and recon, 2 + 2 bytes; write err fp32 and recon, 4 + 2 bytes;
// optionally 1/8 byte of codes) with no arithmetic to speak of, no reduction and no waiting, in the two shapes
// the library uses:
//   row-local      a lane loads one 16-byte vector of x and of recon and stores at once (the shape of k_encode);
//   item-resident  a workgroup of 256 lanes loads a whole item of 256 rows x 128 channels (32 vectors per lane),
//                  passes a barrier, then stores (the shape of k_single_pass), with the items dealt to the
//                  workgroups in index order or XCD-major, and the item's code bytes not written, written as
//                  the 16-byte pieces of the wire layout, or written as one contiguous block per item.
// And the receiver's mix (cf_decompress: read recon and the 1-bit codes, write recon in place).
// For scale, two kernels that only read (x and recon) or only write (err and recon) the same buffers.
// Prints one line per variant.  Usage: stream_ceiling [n_tensors, default 114]
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstdlib>

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
#define GLOBAL __attribute__((address_space(1)))
#define CHECK(x)                                                                      \
    do {                                                                              \
        hipError_t err_ = (x);                                                        \
        if (err_ != hipSuccess) {                                                     \
            printf("HIP error %s at line %d\n", hipGetErrorString(err_), __LINE__);   \
            exit(1);                                                                  \
        }                                                                             \
    } while (0)

constexpr int kTokens = 4096, kChannels = 3072, kRowsPerLane = 16;
constexpr size_t kRowVecs = kChannels * 2 / 16;     // 16-byte vectors per row of x or recon (384)
constexpr int kChunkLanes = 16, kRowLanes = 16;     // 16 lanes across the 256-byte row segment, 16 down the rows
constexpr int kItemRows = kRowLanes * kRowsPerLane, kRowBlocks = kTokens / kItemRows, kStripes = (int)(kRowVecs / kChunkLanes);
enum Codes { NONE = 0, WIRE_PIECES = 1, ITEM_BLOCK = 2 };

__global__ __launch_bounds__(256) void k_row_local(const u32x4 *x, u32x4 *r, u32x4 *e, size_t n_vecs)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vecs) return;
    const u32x4 a = __builtin_nontemporal_load((const GLOBAL u32x4 *)(x + i));
    const u32x4 b = __builtin_nontemporal_load((const GLOBAL u32x4 *)(r + i));     // written back below: the hint pays
    *(GLOBAL u32x4 *)(e + 2 * i) = a - b;
    *(GLOBAL u32x4 *)(e + 2 * i + 1) = a ^ b;
    *(GLOBAL u32x4 *)(r + i) = a + b;
}

// 4 vectors of x and of recon per lane, folded into a value that is (practically) never stored
__global__ __launch_bounds__(256) void k_read_only(const u32x4 *x, const u32x4 *r, u32x4 *sink, size_t n_vecs)
{
    const size_t i0 = (size_t)blockIdx.x * 1024 + threadIdx.x;
    u32x4 acc = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        const size_t i = i0 + (size_t)k * 256;
        if (i < n_vecs) acc ^= __builtin_nontemporal_load((const GLOBAL u32x4 *)(x + i)) + *(const GLOBAL u32x4 *)(r + i);
    }
    if (acc.x == 0x9e3779b9u && acc.y == 0x7f4a7c15u && acc.z == 0xf39cc060u) *(GLOBAL u32x4 *)sink = acc;
}

__global__ __launch_bounds__(256) void k_write_only(u32x4 *r, u32x4 *e, size_t n_vecs)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vecs) return;
    const u32x4 v = {(unsigned)i, 1u, 2u, 3u};
    *(GLOBAL u32x4 *)(e + 2 * i) = v;
    *(GLOBAL u32x4 *)(e + 2 * i + 1) = v;
    *(GLOBAL u32x4 *)(r + i) = v;
}

// the receiver: a lane reads one vector of recon and its code byte and writes the vector back
__global__ __launch_bounds__(256) void k_row_local_decode(u32x4 *r, const unsigned char *codes, size_t n_vecs)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vecs) return;
    const u32x4 b = __builtin_nontemporal_load((const GLOBAL u32x4 *)(r + i));
    const unsigned c = *(const GLOBAL unsigned char *)(codes + i);
    *(GLOBAL u32x4 *)(r + i) = b + c;
}

template <bool XCD_MAJOR, int CODES>
__global__ __launch_bounds__(256, 2) void k_item_resident(const u32x4 *x, u32x4 *r, u32x4 *e, unsigned char *codes)
{
    unsigned item = blockIdx.x;
    if (XCD_MAJOR) {
        const unsigned q = gridDim.x >> 3, rem = gridDim.x & 7u, xcd = blockIdx.x & 7u;
        item = xcd * q + (xcd < rem ? xcd : rem) + (blockIdx.x >> 3);
    }
    const int t = item / (kRowBlocks * kStripes), local = item % (kRowBlocks * kStripes);
    const int stripe = local / kRowBlocks, rb = local % kRowBlocks;
    const int cl = threadIdx.x % kChunkLanes, rl = threadIdx.x / kChunkLanes;
    const size_t row0 = (size_t)t * kTokens + (size_t)rb * kItemRows + (size_t)rl * kRowsPerLane;
    const size_t col = (size_t)stripe * kChunkLanes + cl;
    u32x4 a[kRowsPerLane], b[kRowsPerLane];
#pragma unroll
    for (int k = 0; k < kRowsPerLane; ++k) {
        a[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(x + (row0 + k) * kRowVecs + col));
        b[k] = __builtin_nontemporal_load((const GLOBAL u32x4 *)(r + (row0 + k) * kRowVecs + col));
    }
    __shared__ unsigned mix[256];
    unsigned acc = 0;
#pragma unroll
    for (int k = 0; k < kRowsPerLane; ++k) acc ^= a[k].x ^ b[k].y;
    mix[threadIdx.x] = acc;
    __syncthreads();
    const unsigned s = mix[(threadIdx.x * 7) & 255];
#pragma unroll
    for (int k = 0; k < kRowsPerLane; ++k) {
        const size_t i = (row0 + k) * kRowVecs + col;
        u32x4 d = a[k] - b[k];
        d.x ^= s;
        *(GLOBAL u32x4 *)(e + 2 * i) = d;
        *(GLOBAL u32x4 *)(e + 2 * i + 1) = a[k] ^ b[k];
        *(GLOBAL u32x4 *)(r + i) = a[k] + b[k];
        if (CODES == WIRE_PIECES && (cl & 3) == 0)      // one code byte per lane and row; four lanes share a dword
            *(GLOBAL unsigned *)(codes + (row0 + k) * kRowVecs + col) = d.y;
        if (CODES == ITEM_BLOCK && k == kRowsPerLane - 1) *(GLOBAL u32x4 *)(codes + ((size_t)item * 256 + threadIdx.x) * 16) = d;
    }
}

struct Buffers {
    u32x4 *x, *r, *e;
    unsigned char *codes;
    int n_tensors;
    size_t n_vecs;
    hipEvent_t e0, e1;
};

template <typename Launch> void time_it(const char *what, const Buffers &b, double bytes_per_element, Launch launch)
{
    for (int i = 0; i < 2; ++i) launch();
    CHECK(hipDeviceSynchronize());
    const int iters = 5;
    CHECK(hipEventRecord(b.e0));
    for (int i = 0; i < iters; ++i) launch();
    CHECK(hipEventRecord(b.e1));
    CHECK(hipEventSynchronize(b.e1));
    CHECK(hipGetLastError());
    float ms = 0.0f;
    CHECK(hipEventElapsedTime(&ms, b.e0, b.e1));
    const double bytes = (double)b.n_tensors * kTokens * kChannels * bytes_per_element;
    const double gbps = bytes / 1e9 / (ms / iters * 1e-3);
    printf("%-72s %7.3f ms  %7.1f GB/s  %.1f %% of 8 TB/s\n", what, ms / iters, gbps, gbps / 80.0);
    fflush(stdout);
}

template <bool XCD_MAJOR, int CODES> void item_resident(const char *what, const Buffers &b)
{
    const int grid = b.n_tensors * kRowBlocks * kStripes;
    time_it(what, b, 10.0 + (CODES == NONE ? 0.0 : 0.125),
            [&] { hipLaunchKernelGGL((k_item_resident<XCD_MAJOR, CODES>), dim3(grid), dim3(256), 0, 0, b.x, b.r, b.e, b.codes); });
}

int main(int argc, char **argv)
{
    Buffers b;
    b.n_tensors = argc > 1 ? atoi(argv[1]) : 114;
    if (b.n_tensors < 1 || b.n_tensors > 400) {
        printf("n_tensors must be in [1, 400]\n");
        return 1;
    }
    b.n_vecs = (size_t)b.n_tensors * kTokens * kRowVecs;
    CHECK(hipEventCreate(&b.e0));
    CHECK(hipEventCreate(&b.e1));
    CHECK(hipMalloc(&b.x, b.n_vecs * 16));
    CHECK(hipMalloc(&b.r, b.n_vecs * 16));
    CHECK(hipMalloc(&b.e, b.n_vecs * 32));
    CHECK(hipMalloc(&b.codes, b.n_vecs));          // one byte per vector of 8 elements: the 1-bit codes
    CHECK(hipMemset(b.x, 1, b.n_vecs * 16));
    CHECK(hipMemset(b.r, 2, b.n_vecs * 16));
    CHECK(hipMemset(b.e, 0, b.n_vecs * 32));
    CHECK(hipMemset(b.codes, 0, b.n_vecs));
    printf("%d tensors of [%d, %d] bf16; 10 bytes per element (+ 1/8 with codes)\n", b.n_tensors, kTokens, kChannels);
    time_it("read only (x and recon; 4 bytes per element)", b, 4.0, [&] {
        hipLaunchKernelGGL(k_read_only, dim3((unsigned)((b.n_vecs / 4 + 255) / 256)), dim3(256), 0, 0, b.x, b.r, (u32x4 *)b.codes, b.n_vecs);
    });
    time_it("write only (err and recon; 6 bytes per element)", b, 6.0,
            [&] { hipLaunchKernelGGL(k_write_only, dim3((unsigned)((b.n_vecs + 255) / 256)), dim3(256), 0, 0, b.r, b.e, b.n_vecs); });
    time_it("row-local, no codes", b, 10.0,
            [&] { hipLaunchKernelGGL(k_row_local, dim3((unsigned)((b.n_vecs + 255) / 256)), dim3(256), 0, 0, b.x, b.r, b.e, b.n_vecs); });
    time_it("row-local receiver (recon in place + codes; 4.125 bytes per element)", b, 4.125,
            [&] { hipLaunchKernelGGL(k_row_local_decode, dim3((unsigned)((b.n_vecs + 255) / 256)), dim3(256), 0, 0, b.r, b.codes, b.n_vecs); });
    item_resident<false, NONE>("item-resident, index order, no codes", b);
    item_resident<true, NONE>("item-resident, XCD-major, no codes", b);
    item_resident<false, WIRE_PIECES>("item-resident, index order, codes as 16-byte wire pieces", b);
    item_resident<true, WIRE_PIECES>("item-resident, XCD-major, codes as 16-byte wire pieces", b);
    item_resident<false, ITEM_BLOCK>("item-resident, index order, codes as one block per item", b);
    item_resident<true, ITEM_BLOCK>("item-resident, XCD-major, codes as one block per item", b);
    return 0;
}
