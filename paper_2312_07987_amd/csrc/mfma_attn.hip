#include "common.h"
namespace sh {
bool mfma_attn_supported(int, int) { return false; }
void launch_mfma_attn_fwd(const AttnArgs&, hipStream_t) {}
void launch_mfma_attn_bwd(const AttnBwdArgs&, hipStream_t) {}
}
