// Instantiations and launcher of the row-packed softmax (both element types).
#include "packed_kernels.h"

namespace turbo {

namespace {

template <typename T, int VEC>
hipError_t packed_tv(const PackedSoftmaxArgs& a, int max_len, hipStream_t s) {
    const int nvec = (max_len + VEC - 1) / VEC;
    const int per_lane = (nvec + kWave - 1) / kWave;
    const dim3 block(kWave * kPackedWaves);
    auto grid = [&](int nv) {  // rows per workgroup = wavefronts x rows in flight per wavefront
        const long long per_wg = (long long)kPackedWaves * packed_rows_in_flight(nv, VEC);
        return dim3((unsigned)((a.n_rows + per_wg - 1) / per_wg));
    };
    if (per_lane <= 1)
        hipLaunchKernelGGL((softmax_packed_kernel<T, VEC, 1>), grid(1), block, 0, s, a);
    else if (per_lane <= 2)
        hipLaunchKernelGGL((softmax_packed_kernel<T, VEC, 2>), grid(2), block, 0, s, a);
    else if (per_lane <= 4)
        hipLaunchKernelGGL((softmax_packed_kernel<T, VEC, 4>), grid(4), block, 0, s, a);
    else if (per_lane <= 8)
        hipLaunchKernelGGL((softmax_packed_kernel<T, VEC, 8>), grid(8), block, 0, s, a);
    else if (per_lane <= 16)
        hipLaunchKernelGGL((softmax_packed_kernel<T, VEC, 16>), grid(16), block, 0, s, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_packed(const PackedSoftmaxArgs& a, int elem_size, int max_len, hipStream_t s) {
    return elem_size == 4 ? packed_tv<float, 4>(a, max_len, s) : packed_tv<_Float16, 8>(a, max_len, s);
}

}  // namespace turbo
