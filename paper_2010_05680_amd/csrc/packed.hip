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

// Rows beyond one wavefront's registers span more than 1024 vectors, so the workgroup is always the largest one (16
// wavefronts) and max_len only decides the vectors per lane (2, 3, 4 or 8: at most 32 elements).
template <typename T, int VEC>
hipError_t packed_block_tv(const PackedSoftmaxArgs& a, int max_len, hipStream_t s) {
    constexpr int waves = kBlockMaxWaves;
    const int nvec = (max_len + VEC - 1) / VEC;
    const int per_lane = (nvec + kWave * waves - 1) / (kWave * waves);
    const int nv = per_lane <= 2 ? 2 : per_lane <= 3 ? 3 : per_lane <= 4 ? 4 : 8;
    if ((long long)kWave * waves * nv * VEC < max_len || nv * VEC > 32) return hipErrorInvalidValue;
    const dim3 grid((unsigned)a.n_rows), block(kWave * waves);
    switch (nv) {
        case 2: hipLaunchKernelGGL((softmax_packed_block_kernel<T, VEC, 2>), grid, block, 0, s, a); break;
        case 3: hipLaunchKernelGGL((softmax_packed_block_kernel<T, VEC, 3>), grid, block, 0, s, a); break;
        case 4: hipLaunchKernelGGL((softmax_packed_block_kernel<T, VEC, 4>), grid, block, 0, s, a); break;
        case 8:
            if constexpr (8 * VEC <= 32) {
                hipLaunchKernelGGL((softmax_packed_block_kernel<T, VEC, 8>), grid, block, 0, s, a);
                break;
            }
            return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_softmax_packed(const PackedSoftmaxArgs& a, int elem_size, int max_len, int num_cus, int grid_cap_per_cu,
                                 bool rows_kernel, hipStream_t s) {
    const int wave_max = elem_size == 4 ? packed_wave_max_len<float>() : packed_wave_max_len<_Float16>();
    const int short_len = max_len < wave_max ? max_len : wave_max;  // what the wavefront-per-row kernels are sized for
    hipError_t err;
    // the request-shaped kernel keeps the length table in the lanes of a wavefront: up to 63 requests
    if (a.B < kWave && !rows_kernel)
        err = elem_size == 4 ? packed_groups_tv<float, 4>(a, short_len, num_cus, grid_cap_per_cu, s)
                             : packed_groups_tv<_Float16, 8>(a, short_len, num_cus, grid_cap_per_cu, s);
    else
        err = elem_size == 4 ? packed_tv<float, 4>(a, short_len, s) : packed_tv<_Float16, 8>(a, short_len, s);
    if (err != hipSuccess || max_len <= wave_max) return err;
    // requests beyond a wavefront's registers: a second launch over the same batch, a workgroup per long row
    PackedSoftmaxArgs b = a;
    b.long_from = wave_max;
    return elem_size == 4 ? packed_block_tv<float, 4>(b, max_len, s) : packed_block_tv<_Float16, 8>(b, max_len, s);
}

}  // namespace turbo
