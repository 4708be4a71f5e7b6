// Per-program segmented sum of row scores (CSR offsets), order preserving.
//
// A candidate program's score is the sum of the model's outputs over its statement rows;
// the additions are sequential fp32 in ascending row order starting from +0, so the
// result is reproducible bit for bit.  One lane owns one program.  A wavefront streams
// the contiguous row range of its 64 programs through registers 64 rows at a time
// (coalesced loads) and every lane pulls the rows it owns out of the current window with
// wavefront shuffles, one row per step, in order.  That suits very short programs (many
// programs per 64-row window).  When the wavefront's programs average more than 4 rows (measured:
// from 8 rows per program on the shuffles lose), every lane reads its own rows straight from
// memory instead, four loads in flight, still adding them in ascending order.
#include "fs_internal.h"

namespace fs {

__global__ void __launch_bounds__(kSegProgsPerBlock)
segsum_kernel(const FamDesc *__restrict__ descs, int n_families)
{
    int lo = 0, hi = n_families - 1;
    while (lo < hi) {
        int mid = (lo + hi + 1) >> 1;
        if (descs[mid].seg_block0 <= (int)blockIdx.x)
            lo = mid;
        else
            hi = mid - 1;
    }
    const FamDesc &d = descs[lo];
    const int n_programs = d.n_programs;
    const int32_t *__restrict__ off = d.prog_off;
    const float *__restrict__ rs = d.row_score;
    const int lane = threadIdx.x & 63;
    const int p_wave = (blockIdx.x - d.seg_block0) * kSegProgsPerBlock + (threadIdx.x & ~63);
    if (p_wave >= n_programs)
        return;                                     // whole wavefront leaves together
    const int p = p_wave + lane;
    const int p_last = min(p_wave + 64, n_programs);
    const int n_rows = d.n_rows;
    // Lanes past the family's last program own no rows but keep taking part in the shuffles.
    int begin = 0, end = 0;
    if (p < n_programs) {
        begin = min(max(off[p], 0), n_rows);
        end = min(max(off[p + 1], begin), n_rows);
    }
    const int w_begin = min(max(off[p_wave], 0), n_rows);
    const int w_end = min(max(off[p_last], w_begin), n_rows);

    float acc = 0.0f;
    int cur = begin;
    if (w_end - w_begin > 4 * (p_last - p_wave)) {         // longer programs: per-lane reads
        while (__any(cur < end)) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u)
                v[u] = (cur + u < end) ? rs[cur + u] : 0.0f;
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (cur + u < end)
                    acc = acc + v[u];
            cur += 4;
        }
        if (p < n_programs)
            d.prog_score[p] = acc;
        return;
    }
    for (int base = w_begin; base < w_end; base += 64) {
        const int idx = base + lane;
        const float v = (idx < w_end) ? rs[idx] : 0.0f;
        const int win_end = min(base + 64, w_end);
        while (true) {
            const bool active = (cur < end) && (cur < win_end) && (cur >= base);
            if (!__any(active))
                break;
            const float t = __shfl(v, active ? (cur - base) : 0, 64);
            if (active) {
                acc = acc + t;
                ++cur;
            }
        }
    }
    if (p < n_programs)
        d.prog_score[p] = acc;
}

int launch_segsum(const FamDesc *d_desc, int n_families, int total_blocks, hipStream_t stream)
{
    hipLaunchKernelGGL(segsum_kernel, dim3(total_blocks), dim3(kSegProgsPerBlock), 0, stream,
                       d_desc, n_families);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail_hip(e, "segsum_kernel launch");
    return FS_OK;
}

}  // namespace fs
