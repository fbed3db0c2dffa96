// The filters of many layers packed for the specialised forward / layer-gradient kernels in one launch
// (q8t_qconv_pack_multi): the weights of a step are quantized once, so their packed forms and column sums (the
// zero-point correction of Section 4's products) can be made once, ahead of the products, instead of by a small
// dependent launch in front of every product.
#include "q8t_common.h"
#include "q8t_internal.h"
#include "repack.h"

namespace {

struct PackTable {
    Q8tPackJob job[kPackMaxJobs];
    int n;
};

__global__ __launch_bounds__(kRepackThreads) void repack_multi(const PackTable t)
{
    __shared__ int red[kRepackThreads / 64];
    // the job whose run of blocks holds this one (jobs are few: a uniform scan)
    int j = 0;
    for (int i = 1; i < t.n; ++i)
        if ((int)blockIdx.x >= t.job[i].first_block) j = i;
    const Q8tPackJob &b = t.job[j];
    const int oc = (int)blockIdx.x - b.first_block;
    if (b.layout == Q8T_PACK_TILE64)
        q8t_repack_tile64(b.w, b.Kf, b.Cf, b.R, b.S, b.dgrad, b.out, b.colsum, oc, red);
    else
        q8t_repack_wide(b.w, b.Kf, b.Cf, b.dgrad, b.layout == Q8T_PACK_WIDE256 ? 256 : 128, b.out, b.colsum, oc, red);
}

}  // namespace

int q8t_pack_launch(const Q8tPackJob *jobs, int n, hipStream_t st)
{
    for (int at = 0; at < n; at += kPackMaxJobs) {
        PackTable t;
        t.n = n - at < kPackMaxJobs ? n - at : kPackMaxJobs;
        int blocks = 0;
        for (int i = 0; i < t.n; ++i) {
            t.job[i] = jobs[at + i];
            t.job[i].first_block = blocks;
            blocks += jobs[at + i].dgrad ? jobs[at + i].Cf : jobs[at + i].Kf;   // one workgroup per output channel of the product
        }
        if (blocks == 0) continue;
        hipLaunchKernelGGL(repack_multi, dim3((unsigned)blocks), dim3(kRepackThreads), 0, st, t);
        Q8T_LAUNCH_CHECK();
    }
    return Q8T_OK;
}
