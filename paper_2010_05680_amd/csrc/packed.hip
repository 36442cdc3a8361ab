// Instantiations and launcher of the row-packed softmax (both element types).
#include "packed_kernels.h"

namespace turbo {

namespace {

template <typename T, int VEC>
hipError_t packed_groups_tv(const PackedSoftmaxArgs& a, int max_len, int num_cus, int grid_cap_per_cu, hipStream_t s) {
    const int nvec = (max_len + VEC - 1) / VEC;
    const int per_lane = (nvec + kWave - 1) / kWave;
    // every request has at most 1 + (its rows / rows per task of the longest request) tasks
    const long long task_rows = packed_task_rows<VEC>(max_len);
    long long waves = (a.n_rows + task_rows - 1) / task_rows + a.B;
    long long wgs = (waves + kPackedWaves - 1) / kPackedWaves;
    if (grid_cap_per_cu > 0 && wgs > (long long)num_cus * grid_cap_per_cu) wgs = (long long)num_cus * grid_cap_per_cu;
    const dim3 grid((unsigned)wgs), block(kWave * kPackedWaves);
    if (per_lane <= 1)
        hipLaunchKernelGGL((softmax_packed_groups_kernel<T, VEC, 1>), grid, block, 0, s, a);
    else if (per_lane <= 2)
        hipLaunchKernelGGL((softmax_packed_groups_kernel<T, VEC, 2>), grid, block, 0, s, a);
    else if (per_lane <= 4)
        hipLaunchKernelGGL((softmax_packed_groups_kernel<T, VEC, 4>), grid, block, 0, s, a);
    else if (per_lane <= 8)
        hipLaunchKernelGGL((softmax_packed_groups_kernel<T, VEC, 8>), grid, block, 0, s, a);
    else if (per_lane <= 16)
        hipLaunchKernelGGL((softmax_packed_groups_kernel<T, VEC, 16>), grid, block, 0, s, a);
    else
        return hipErrorInvalidValue;
    return hipGetLastError();
}

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

hipError_t launch_softmax_packed(const PackedSoftmaxArgs& a, int elem_size, int max_len, int num_cus, int grid_cap_per_cu,
                                 bool rows_kernel, hipStream_t s) {
    // the request-shaped kernel keeps the length table in the lanes of a wavefront: up to 63 requests
    if (a.B < kWave && !rows_kernel)
        return elem_size == 4 ? packed_groups_tv<float, 4>(a, max_len, num_cus, grid_cap_per_cu, s)
                              : packed_groups_tv<_Float16, 8>(a, max_len, num_cus, grid_cap_per_cu, s);
    return elem_size == 4 ? packed_tv<float, 4>(a, max_len, s) : packed_tv<_Float16, 8>(a, max_len, s);
}

}  // namespace turbo
