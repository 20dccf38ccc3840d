// Backward of the segmented LoRA update for fine-tune segments.
#include "lq_common.h"

extern "C" size_t lora_backward_workspace_bytes(int32_t n_tokens, int32_t max_rank, int32_t d_in, int32_t d_out)
{
    (void)n_tokens; (void)max_rank; (void)d_in; (void)d_out;
    return lq::kWsHeaderBytes;
}

extern "C" lq_status lora_segmented_backward(const void* x, int64_t ldx, const void* dy, int64_t lddy, void* dx,
                                             int64_t lddx, int32_t d_in, int32_t d_out,
                                             const void* const* A_ptrs, const void* const* B_ptrs,
                                             float* const* dA_ptrs, float* const* dB_ptrs,
                                             const int32_t* ranks, const float* scales, int32_t n_adapters,
                                             int32_t max_rank, const int32_t* perm, int32_t n_tokens,
                                             const int32_t* seg_starts, const int32_t* seg_adapter,
                                             const uint8_t* seg_kind, const int32_t* n_segments, int32_t max_segments,
                                             const float* h_saved, const int64_t* h_offsets,
                                             void* workspace, size_t workspace_bytes, void* stream)
{
    (void)x; (void)ldx; (void)dy; (void)lddy; (void)dx; (void)lddx; (void)d_in; (void)d_out; (void)A_ptrs; (void)B_ptrs;
    (void)dA_ptrs; (void)dB_ptrs; (void)ranks; (void)scales; (void)n_adapters; (void)max_rank; (void)perm;
    (void)n_tokens; (void)seg_starts; (void)seg_adapter; (void)seg_kind; (void)n_segments; (void)max_segments;
    (void)h_saved; (void)h_offsets; (void)workspace; (void)workspace_bytes; (void)stream;
    return LQ_ERR_UNSUPPORTED;
}
