// Head reduction of the visual mass (Sec. 3.2: last-row attention on the visual keys, here
// averaged over heads), shared by the decode finish kernel and by the eviction-plan kernel, which
// finishes the mass of the attention launch that preceded it.
#pragma once

#include "st3_attend.h"

namespace st3 {

#if defined(__HIPCC__)

// Row maximum and reciprocal row sum of every head of sequence b, rebuilt from the per-chunk
// (max, sum) pairs in chunk order, into two LDS arrays of H entries.  Ends with a barrier.
__device__ __forceinline__ void head_norms(const float* part_ml, int b, int H, int ns, int nsplit_cap, float* sm_m,
                                           float* sm_rl) {
    for (int h = threadIdx.x; h < H; h += blockDim.x) {
        const float* ml = part_ml + ((int64_t)b * H + h) * nsplit_cap * 2;
        float m = -INFINITY, l = 0.f;
        if (ns > 0) {
            m = ml[0];
            for (int s = 1; s < ns; ++s) m = fmaxf(m, ml[2 * s]);
            for (int s = 0; s < ns; ++s) l = fmaf(ml[2 * s + 1], exp2_fast(ml[2 * s] - m), l);
        }
        sm_m[h] = m;
        sm_rl[h] = ns > 0 ? 1.0f / l : 0.f;
    }
    __syncthreads();
}

// mass_row[j] = (1/H) sum_h exp2(logit[b,h,j] - m_h) / l_h for j in [j0, j1); heads are added in
// index order so the result does not depend on scheduling.
__device__ __forceinline__ void finish_mass(const float* logits, int b, int H, int capacity, const float* sm_m,
                                            const float* sm_rl, int j0, int j1, float* mass_row) {
    const float* lgb = logits + (int64_t)b * H * capacity;
    const float inv_h = 1.0f / (float)H;
    for (int j = j0 + threadIdx.x; j < j1; j += blockDim.x) {
        float acc = 0.f;
        for (int h = 0; h < H; ++h) acc += exp2_fast(lgb[(int64_t)h * capacity + j] - sm_m[h]) * sm_rl[h];
        mass_row[j] = acc * inv_h;
    }
}

#endif  // __HIPCC__

}  // namespace st3
