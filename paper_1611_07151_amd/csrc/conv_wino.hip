// Kernel transform of the minimal-filtering convolution: host launch (both input types).
#include "conv_wino_kernel.h"

namespace sq {

size_t wino_transformed_bytes(int Cout, int Cin)
{
    const size_t mtiles = ((size_t)Cout + mfma::kWinoBM - 1) / mfma::kWinoBM;
    return mtiles * ((size_t)Cin / mfma::kWinoCC) * mfma::kWinoImage * sizeof(float);
}

// the second layout (conv_wino_auto_kernel.h) follows the first in the same scratch area
size_t wino_auto_offset(int Cout, int Cin) { return align_up(wino_transformed_bytes(Cout, Cin), 256); }
size_t wino_auto_bytes(int Cout, int Cin)
{
    return (size_t)((Cout + 31) / 32) * (Cin / 4) * mfma::kWinoAutoStep * sizeof(float);
}

int conv_prepare_kernels(const KernelPrepJob *jobs, int n, int dtype)
{
    using namespace mfma;
    if (n <= 0 || n > kWinoMaxJobs) return SQ_ERR_SHAPE;
    WinoJobs wj;
    double bytes = 0;
    wj.n = n;
    wj.first[0] = 0;
    for (int j = 0; j < kWinoMaxJobs; ++j) {
        const KernelPrepJob &job = jobs[j < n ? j : n - 1];
        wj.w[j] = job.w; wj.u[j] = (float *)job.ws; wj.u2[j] = (float *)((char *)job.ws + wino_auto_offset(job.Cout, job.Cin)); wj.Cout[j] = job.Cout; wj.Cin[j] = job.Cin;
        if (j < n) {
            const long long padded = (long long)((job.Cout + kWinoBM - 1) / kWinoBM * kWinoBM) * job.Cin;
            if (wj.first[j] + padded >= (1ll << 30)) return SQ_ERR_UNSUPPORTED;
            wj.first[j + 1] = wj.first[j] + (int)padded;
            bytes += (dtype == SQ_BF16 ? 2.0 : 4.0) * 9.0 * job.Cout * job.Cin + 4.0 * 16.0 * ((double)padded + (double)job.Cout * job.Cin);
        } else {
            wj.first[j + 1] = wj.first[j];
        }
    }
    const unsigned blocks = (unsigned)((wj.first[n] + 255) / 256);
    LaunchScope scope("f2x2_kernel_transform", 0.0, bytes);
    if (dtype == SQ_BF16)
        hipLaunchKernelGGL(wino_kernel_transform<uint16_t>, dim3(blocks), dim3(256), 0, current_stream(), wj);
    else
        hipLaunchKernelGGL(wino_kernel_transform<float>, dim3(blocks), dim3(256), 0, current_stream(), wj);
    return check_launch();
}

}  // namespace sq
