// Sparsity of a tensor (Section VI, "Sparsity"): the number of its values that are zero, counted on the
// quantized codes (a code is zero when its exponent and mantissa fields are, whatever the sign bit) or on
// fp32 values (+0 and -0), so that the ratio between a quantized tensor and its full-precision original
// can be formed.  One read of the tensor, 16 bytes per lane and step; HBM-bound.
#include "fpq_dev.h"
#include "fpq_host.h"

namespace fpq {

namespace {

enum { ZK_BYTE = 0, ZK_NIBBLE = 1, ZK_F32 = 2 };
typedef uint32_t v4u __attribute__((ext_vector_type(4)));

// Zero elements in one 32-bit word.  Codes: `field` holds the magnitude mask of one element replicated
// over the word; a masked byte is at most 0x7f (a nibble at most 7), so adding 0x7f (7) sets the element's
// top bit exactly when it is non-zero, without a carry into its neighbour.
template <int KIND>
__device__ __forceinline__ int zeros_in_word(uint32_t w, uint32_t field)
{
    if (KIND == ZK_F32) return (w & 0x7fffffffu) == 0u;
    if (KIND == ZK_BYTE) return 4 - __popc(((w & field) + 0x7f7f7f7fu) & 0x80808080u);
    return 8 - __popc(((w & field) + 0x77777777u) & 0x88888888u);
}

// Block b counts its contiguous share of the 16-byte groups of the aligned body; block 0 also takes the
// bytes before and after it one at a time (fewer than 16 before, at most 16 after).
template <int KIND>
__global__ __launch_bounds__(256) void count_zeros_kernel(const uint8_t* __restrict__ p, size_t nbytes, size_t head,
                                                          uint32_t field, int odd_nibbles,
                                                          unsigned long long* __restrict__ partial)
{
    // with an odd number of nibbles the last byte is kept out of the 16-byte groups: its high nibble is no element
    const size_t avail = nbytes - head;
    const size_t body = (avail > (size_t)odd_nibbles ? avail - odd_nibbles : 0) / 16;
    const v4u* __restrict__ v = reinterpret_cast<const v4u*>(p + head);
    unsigned long long cnt = 0;
    const size_t share = (body + gridDim.x - 1) / gridDim.x;
    const size_t first = (size_t)blockIdx.x * share;
    const size_t last = first + share < body ? first + share : body;
    for (size_t i = first + threadIdx.x; i < last; i += 1024) {   // four independent streaming loads per lane in flight
        v4u q[4];
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < last) q[u] = __builtin_nontemporal_load(v + i + u * 256);
#pragma unroll
        for (int u = 0; u < 4; ++u)
            if (i + u * 256 < last)
                cnt += zeros_in_word<KIND>(q[u].x, field) + zeros_in_word<KIND>(q[u].y, field) +
                       zeros_in_word<KIND>(q[u].z, field) + zeros_in_word<KIND>(q[u].w, field);
    }
    if (blockIdx.x == 0 && KIND != ZK_F32) {
        const size_t tail0 = head + body * 16;
        const size_t loose = head + (nbytes - tail0);   // bytes outside the body, at most 31
        if (threadIdx.x < loose) {
            const size_t at = threadIdx.x < head ? threadIdx.x : tail0 + (threadIdx.x - head);
            const uint32_t byte = p[at];
            if (KIND == ZK_BYTE) {
                cnt += (byte & field & 0xffu) == 0u;
            } else {
                cnt += (byte & field & 0x0fu) == 0u;
                if (!(odd_nibbles && at == nbytes - 1)) cnt += (byte & field & 0xf0u) == 0u;
            }
        }
    }
    if (blockIdx.x == 0 && KIND == ZK_F32) {
        // fp32 input is 4-byte aligned: head and tail are whole words
        const size_t tail0 = head + body * 16;
        const size_t loose = (head + (nbytes - tail0)) / 4;
        if (threadIdx.x < loose) {
            const size_t at = threadIdx.x < head / 4 ? (size_t)threadIdx.x * 4 : tail0 + (threadIdx.x - head / 4) * 4;
            cnt += (*reinterpret_cast<const uint32_t*>(p + at) & 0x7fffffffu) == 0u;
        }
    }
    // 64-bit sums across the wavefront, then across the four wavefronts through LDS
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off, 64);
    __shared__ unsigned long long wsum[4];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) partial[blockIdx.x] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

__global__ __launch_bounds__(256) void count_zeros_final_kernel(const unsigned long long* __restrict__ partial, int nparts,
                                                                unsigned long long* __restrict__ out)
{
    unsigned long long cnt = 0;
    for (int i = threadIdx.x; i < nparts; i += 256) cnt += partial[i];
    for (int off = 32; off > 0; off >>= 1) cnt += __shfl_down(cnt, off, 64);
    __shared__ unsigned long long wsum[4];
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = cnt;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = wsum[0] + wsum[1] + wsum[2] + wsum[3];
}

}  // namespace

int launch_count_zeros(const void* x, int is_fp32, size_t n, int em, bool four_bit, unsigned long long* out,
                       unsigned long long* partial, hipStream_t st)
{
    const uint8_t* p = static_cast<const uint8_t*>(x);
    const size_t nbytes = is_fp32 ? n * 4 : (four_bit ? (n + 1) / 2 : n);
    size_t head = (size_t)(-(intptr_t)reinterpret_cast<uintptr_t>(p)) & 15;
    if (head > nbytes) head = nbytes;
    const int nparts = count_zeros_parts(nbytes);
    const uint32_t m1 = (1u << em) - 1u;
    if (is_fp32) {
        hipLaunchKernelGGL(count_zeros_kernel<ZK_F32>, dim3(nparts), dim3(256), 0, st, p, nbytes, head, 0u, 0, partial);
    } else if (four_bit) {
        hipLaunchKernelGGL(count_zeros_kernel<ZK_NIBBLE>, dim3(nparts), dim3(256), 0, st, p, nbytes, head,
                           m1 * 0x11111111u, (int)(n & 1), partial);
    } else {
        hipLaunchKernelGGL(count_zeros_kernel<ZK_BYTE>, dim3(nparts), dim3(256), 0, st, p, nbytes, head,
                           m1 * 0x01010101u, 0, partial);
    }
    hipLaunchKernelGGL(count_zeros_final_kernel, dim3(1), dim3(256), 0, st, partial, nparts, out);
    return hipGetLastError() == hipSuccess ? FPQ_OK : FPQ_ERR_LAUNCH;
}

}  // namespace fpq
