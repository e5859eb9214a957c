// HilbertCurve permutation (Sec. 3.7; App. A): the visual tokens of a T x H x W grid are flattened along
// a Hilbert curve before attention and the output is put back in the original order.  The order is
// computed on the host (it depends on the grid only); the token gathers are bandwidth-bound kernels.
#include <algorithm>
#include <vector>

#include "common.hpp"

namespace sparge {

namespace {

// Hilbert index of a grid cell inside the 2^bits cube, encoding direction of Skilling's transform
// ("Programming the Hilbert curve", 2004): from the coarsest level down, axis 0 is inverted below a set
// bit of axis i, or exchanges its low bits with axis i below a clear one; then a Gray code across the
// axes; the index interleaves the axes' bits, axis 0 first.
uint64_t hilbert_index(const uint32_t* cell, int ndim, int bits) {
    uint32_t x[3];
    for (int i = 0; i < ndim; ++i) x[i] = cell[i];
    for (uint32_t q = 1u << (bits - 1); q > 1; q >>= 1) {
        const uint32_t low = q - 1;
        for (int i = 0; i < ndim; ++i) {
            if (x[i] & q) {
                x[0] ^= low;
            } else {
                const uint32_t swap = (x[0] ^ x[i]) & low;
                x[0] ^= swap;
                x[i] ^= swap;
            }
        }
    }
    for (int i = 1; i < ndim; ++i) x[i] ^= x[i - 1];
    uint32_t flip = 0;
    for (uint32_t q = 1u << (bits - 1); q > 1; q >>= 1)
        if (x[ndim - 1] & q) flip ^= q - 1;
    for (int i = 0; i < ndim; ++i) x[i] ^= flip;
    uint64_t idx = 0;
    for (int b = bits - 1; b >= 0; --b)
        for (int i = 0; i < ndim; ++i) idx = (idx << 1) | ((x[i] >> b) & 1u);
    return idx;
}

// dst[.., off + s, :] = src[.., off + perm[s], :] (INVERSE: dst[.., off + perm[s], :] = src[.., off + s, :]);
// tokens outside [off, off + L) are copied in place.  One 16-byte piece per thread.
template <bool INVERSE>
__global__ __launch_bounds__(256) void permute_tokens_kernel(const uint16_t* __restrict__ src, Shape s,
                                                             const int32_t* __restrict__ perm, int L, int off,
                                                             uint16_t* __restrict__ dst) {
    const int cpr = s.d / 8;                       // 16-byte pieces per token
    const int rows_per_wg = 256 / cpr;
    const int row = blockIdx.x * rows_per_wg + threadIdx.x / cpr, col = threadIdx.x % cpr;
    if (row >= s.N) return;
    const long long base = (long long)blockIdx.z * s.sb + (long long)blockIdx.y * s.sh;
    int from = row, to = row;
    if (row >= off && row < off + L) {
        const unsigned e = static_cast<unsigned>(perm[row - off]);
        const int other = e < static_cast<unsigned>(L) ? off + static_cast<int>(e) : row;  // a bad entry moves nothing
        if (INVERSE) to = other; else from = other;
    }
    const uint4 v = *reinterpret_cast<const uint4*>(src + base + (long long)from * s.sn + col * 8);
    *reinterpret_cast<uint4*>(dst + base + (long long)to * s.sn + col * 8) = v;
}

}  // namespace

void hilbert_order_host(int T, int H, int W, int32_t* perm) {
    const int dims[3] = {T, H, W};
    const int first = T == 1 ? 1 : 0, ndim = 3 - first;  // a single frame: the two-dimensional curve over (H, W)
    int bits = 1;
    while ((1 << bits) < std::max(T, std::max(H, W))) ++bits;
    const long long n = (long long)T * H * W;
    std::vector<std::pair<uint64_t, int32_t>> key(n);
    long long cellno = 0;
    for (int t = 0; t < dims[0]; ++t)
        for (int h = 0; h < dims[1]; ++h)
            for (int w = 0; w < dims[2]; ++w, ++cellno) {
                const uint32_t cell[3] = {(uint32_t)t, (uint32_t)h, (uint32_t)w};
                key[cellno] = {hilbert_index(cell + first, ndim, bits), (int32_t)cellno};
            }
    std::sort(key.begin(), key.end());
    for (long long sidx = 0; sidx < n; ++sidx) perm[sidx] = key[sidx].second;
}

hipError_t launch_permute_tokens(const void* src, const Shape& s, const int32_t* perm, int L, int off, int inverse,
                                 void* dst, hipStream_t st) {
    const int rows_per_wg = 256 / (s.d / 8);
    dim3 grid((s.N + rows_per_wg - 1) / rows_per_wg, s.H, s.B);
    const uint16_t* a = static_cast<const uint16_t*>(src);
    uint16_t* b = static_cast<uint16_t*>(dst);
    if (inverse) hipLaunchKernelGGL(permute_tokens_kernel<true>, grid, dim3(256), 0, st, a, s, perm, L, off, b);
    else hipLaunchKernelGGL(permute_tokens_kernel<false>, grid, dim3(256), 0, st, a, s, perm, L, off, b);
    return hipGetLastError();
}

}  // namespace sparge
