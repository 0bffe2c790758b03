// Huffman-coded size of a tensor of level indices (Sec. V-A, eq. Nofbits: the paper measures the
// compressed size of weights and activations as the average Huffman code length per entry).
//
// Two kernels: a histogram of the int8 indices (16 bytes per thread and trip; per-wave LDS histograms with
// eight interleaved copies of every bin, so that lanes collide only when they share copy and bin; one
// plain row of 256 counts per block), and a single-block kernel that adds the rows, sorts the counts
// (bitonic, in LDS) and runs the two-queue form of Huffman's algorithm: the total code length is the sum
// of the weights of all merged nodes, which no choice among equal weights can change.
#include "cdl_internal.h"

namespace cdl {

namespace {

constexpr int kHistThreads = 256;
constexpr int kHistCopies = 8;
constexpr int kHistMaxBlocks = 1024;

__global__ __launch_bounds__(kHistThreads)
void index_hist_kernel(const int8_t *__restrict__ idx, int64_t n, unsigned int *__restrict__ rows /* [gridDim.x][256] */)
{
    __shared__ unsigned int hist[kHistThreads / 64][256 * kHistCopies];
    for (int i = threadIdx.x; i < (kHistThreads / 64) * 256 * kHistCopies; i += kHistThreads) (&hist[0][0])[i] = 0u;
    __syncthreads();
    unsigned int *mine = &hist[threadIdx.x >> 6][threadIdx.x & (kHistCopies - 1)];
    const int64_t n16 = n >> 4;
    const int64_t stride = (int64_t)gridDim.x * kHistThreads;
    for (int64_t v = (int64_t)blockIdx.x * kHistThreads + threadIdx.x; v < n16; v += stride) {
        const uint4 w = reinterpret_cast<const uint4 *>(idx)[v];
        const unsigned int ws[4] = {w.x, w.y, w.z, w.w};
#pragma unroll
        for (int d = 0; d < 4; ++d)
#pragma unroll
            for (int b = 0; b < 4; ++b) atomicAdd(mine + ((ws[d] >> (8 * b)) & 0xffu) * kHistCopies, 1u);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0)
        for (int64_t e = n16 << 4; e < n; ++e) atomicAdd(mine + (unsigned int)(uint8_t)idx[e] * kHistCopies, 1u);
    __syncthreads();
    // bin b = the index byte as an unsigned number
    unsigned int s = 0u;
    for (int w = 0; w < kHistThreads / 64; ++w)
#pragma unroll
        for (int c = 0; c < kHistCopies; ++c) s += hist[w][threadIdx.x * kHistCopies + ((c + threadIdx.x) & (kHistCopies - 1))];
    rows[(size_t)blockIdx.x * 256 + threadIdx.x] = s;
}

__global__ __launch_bounds__(1024)
void huffman_kernel(const unsigned int *__restrict__ rows, int nrows, int64_t n, int lo, int n_levels,
                    unsigned long long *__restrict__ counts /* [n_levels], nullable */,
                    unsigned long long *__restrict__ total_bits /* nullable */, float *__restrict__ bits_per_entry /* nullable */)
{
    __shared__ unsigned long long key[256];
    __shared__ unsigned long long merged[256];
    __shared__ unsigned long long part[16][256];
    // 1024 threads = 16 groups of 64: a group takes every sixteenth row, a thread four neighbouring bins
    // (one 16-byte load), four loads in flight each (one thread per bin walking all rows one after the other
    // is nothing but memory latency)
    {
        const int q = threadIdx.x & 63, grp = threadIdx.x >> 6;
        unsigned long long c[4][4] = {};
        const uint4 *rows4 = reinterpret_cast<const uint4 *>(rows);
        int r = grp;
        for (; r + 48 < nrows; r += 64) {
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const uint4 v = rows4[(size_t)(r + 16 * u) * 64 + q];
                c[u][0] += v.x; c[u][1] += v.y; c[u][2] += v.z; c[u][3] += v.w;
            }
        }
        for (; r < nrows; r += 16) {
            const uint4 v = rows4[(size_t)r * 64 + q];
            c[0][0] += v.x; c[0][1] += v.y; c[0][2] += v.z; c[0][3] += v.w;
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) part[grp][4 * q + e] = (c[0][e] + c[1][e]) + (c[2][e] + c[3][e]);
    }
    __syncthreads();
    // from here on the first 256 threads work, thread t on byte value t, i.e. level (int8)t; the others
    // only keep the barriers company
    const int t = threadIdx.x;
    const bool act = t < 256;
    if (act) {
        unsigned long long c = 0ull;
#pragma unroll
        for (int g = 0; g < 16; ++g) c += part[g][t];
        const int level = (int)(int8_t)(uint8_t)t;
        const bool in_set = level >= lo && level < lo + n_levels;
        if (counts && in_set) counts[level - lo] = c;
        key[t] = in_set ? c : 0ull;
    }
    __syncthreads();
    // bitonic sort, ascending
    for (int k = 2; k <= 256; k <<= 1)
        for (int j = k >> 1; j > 0; j >>= 1) {
            const int p = t ^ j;
            if (act && p > t) {
                const unsigned long long a = key[t], b = key[p];
                const bool up = (t & k) == 0;
                if ((a > b) == up) { key[t] = b; key[p] = a; }
            }
            __syncthreads();
        }
    if (t != 0) return;
    // two queues: the sorted leaves (zeros skipped) and the merged nodes, which come out in nondecreasing order
    int i = 0;
    while (i + 8 <= 256 && key[i + 7] == 0ull) i += 8;     // the zeros sort to the front
    while (i < 256 && key[i] == 0ull) ++i;
    const int leaves = 256 - i;
    unsigned long long total = 0ull;
    if (leaves == 1) {
        total = key[i];          // a single level that occurs: one bit per entry
    } else if (leaves > 1) {
        int mh = 0, mt = 0;      // head and tail of the merged queue
        for (int step = 0; step < leaves - 1; ++step) {
            unsigned long long w2[2];
            for (int s = 0; s < 2; ++s) {
                const bool take_leaf = i < 256 && (mh >= mt || key[i] <= merged[mh]);
                w2[s] = take_leaf ? key[i] : merged[mh];
                if (take_leaf) ++i; else ++mh;
            }
            merged[mt++] = w2[0] + w2[1];
            total += w2[0] + w2[1];
        }
    }
    if (total_bits) *total_bits = total;
    if (bits_per_entry) *bits_per_entry = n > 0 ? (float)((double)total / (double)n) : 0.0f;
}

int hist_blocks(int64_t n)
{
    int64_t b = (n / 16 + (int64_t)kHistThreads * 8 - 1) / ((int64_t)kHistThreads * 8);
    if (b < 1) b = 1;
    if (b > kHistMaxBlocks) b = kHistMaxBlocks;
    return (int)b;
}

}  // namespace

size_t huffman_workspace_bytes(int64_t n)
{
    return align_up((size_t)hist_blocks(n) * 256 * sizeof(unsigned int), 256);
}

int launch_huffman_bits(const int8_t *idx, int64_t n, int lo, int n_levels, unsigned long long *counts,
                        unsigned long long *total_bits, float *bits_per_entry, void *ws, hipStream_t stream)
{
    const int blocks = hist_blocks(n);
    unsigned int *rows = reinterpret_cast<unsigned int *>(ws);
    CDL_LAUNCH("index_hist_kernel", stream, index_hist_kernel, dim3(blocks), dim3(kHistThreads), 0, idx, n, rows);
    CDL_LAUNCH("huffman_kernel", stream, huffman_kernel, dim3(1), dim3(1024), 0, rows, blocks, n, lo, n_levels, counts, total_bits,
               bits_per_entry);
    return check_launch();
}

}  // namespace cdl
