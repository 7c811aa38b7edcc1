// Arguments shared by the two prefill attention kernels (float32 row kernel, bf16 MFMA kernel).
#pragma once

#include "st3_common.h"

namespace st3 {

struct PrefillArgs {
    const void* q; const void* k; const void* v; void* out;
    int64_t q_sb, q_sh, q_st;       // strides in elements
    int64_t k_sb, k_sh, k_st;
    int64_t v_sb, v_sh, v_st;
    int64_t o_sb, o_sh, o_st;
    int32_t n, sys_len, vis_len, window, H;
    int32_t B, n_qt;                // batch and query tiles per strip (filled in by the MFMA launcher)
    int32_t q_shift;                // rows by which the query tiles start before row 0 (MFMA launcher)
    float scale_l2;                 // softmax scale times log2(e)
    float* pre_logits;              // [B,H,W,vis_len] log2-domain logits of the last W rows (null: no mass)
    float* pre_ml;                  // [B,H,W,2] row max and row sum of those rows
};

// bf16 only; returns ST3_ERR_UNSUPPORTED for shapes it does not handle.
st3_status launch_prefill_mfma(const PrefillArgs& a, int B, int D, hipStream_t st);

}  // namespace st3
