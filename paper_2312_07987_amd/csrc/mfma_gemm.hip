#include "common.h"
namespace sh {
bool mfma_row_gemm_supported(const RowGemmArgs&) { return false; }
void launch_mfma_row_gemm(const RowGemmArgs&, hipStream_t) {}
bool mfma_wgrad_supported(const WgradArgs&) { return false; }
void launch_mfma_wgrad(const WgradArgs&, hipStream_t) {}
}
