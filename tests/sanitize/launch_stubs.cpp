// Stand-ins for the kernel launchers of libhbmm, for the host-only sanitizer build of the C-ABI layer
// (csrc/api.hip): every launcher counts the call and reports success, so that the argument checking
// and dispatch code of api.hip runs under AddressSanitizer / UBSan on a machine without a GPU.
// Test infrastructure only: nothing in the product links this file.
#include "../../paper_1905_10759_amd/csrc/kernels.h"

static int g_launches = 0;
extern "C" int hbmm_stub_launches(void) { return g_launches; }

namespace hbmm {
hipError_t launch_pack_rows(const float *, int64_t, int64_t, int64_t, int, uint32_t *, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_pack_cols(const float *, int64_t, int64_t, int64_t, int, uint32_t *, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_pack_activations_any(const float *, int64_t, int64_t, int, uint32_t *, float *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_pack_any(const float *, int64_t, int64_t, int64_t, int, int, uint32_t *, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_binarize_backward_any(const float *, const float *, int64_t, int64_t, int64_t, int64_t, int, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_binarize_backward(const float *, const float *, int64_t, int64_t, int64_t, int64_t, int, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_popcount_gemm(const PopcountGemmArgs &, int, int, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_split_gemm(const SplitGemmOperand &, const SplitGemmOperand &, int64_t, float *, int64_t, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_split_any(const SplitGemmOperand &, const SplitGemmOperand &, int64_t, float *, int64_t, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_split_conv(const ConvActivations &, const SplitGemmOperand &, const ConvGeometry &, float *, hipStream_t) { ++g_launches; return hipSuccess; }
int64_t conv_filter_pieces_bytes(int64_t N, int64_t C, int KH, int KW, int form) { return ((N + 31) / 32) * ((C + 31) / 32) * KH * KW * (form ? 4096 : 6144) + (form ? (N + 31) / 32 * 128 : 0); }
hipError_t launch_conv_prepare_filters(const uint32_t *, const float *, int64_t, int64_t, int, int64_t, int64_t, int, int, int, void *, hipStream_t) { ++g_launches; return hipSuccess; }
bool conv_direct_fits(const ConvGeometry &g)
{
    // the documented limits: OW <= 128 and ((OW - 1) * stride + KW) * KH <= 640
    const int64_t OW = (g.W + 2 * g.pad - g.KW) / g.stride + 1;
    return OW <= 128 && ((OW - 1) * g.stride + g.KW) * g.KH <= 640;
}
hipError_t launch_conv_direct(const ConvActivations &, const void *, int64_t, const ConvGeometry &, int, float *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_i8_gemm(const uint32_t *, const float *, int64_t, int64_t, int, const uint32_t *, const float *, int64_t, int64_t, int, int64_t, int64_t, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_fp4_gemm(const uint32_t *, const float *, int64_t, int64_t, int, const uint32_t *, const float *, int64_t, int64_t, int, int64_t, int64_t, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_mfma_fp8_gemm(const uint32_t *, const float *, int64_t, int64_t, int, const uint32_t *, const float *, int64_t, int64_t, int, int64_t, int64_t, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_probe_mfma(int, int, float *, hipStream_t) { ++g_launches; return hipSuccess; }
hipError_t launch_dense_ref(const void *, int64_t, const void *, int64_t, int, int64_t, int64_t, int64_t, float *, int64_t, hipStream_t) { ++g_launches; return hipSuccess; }
}  // namespace hbmm
