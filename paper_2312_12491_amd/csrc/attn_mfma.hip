// bf16 MFMA flash attention (placeholder until the kernel lands: nothing is routed here).
#include "common.h"
bool attention_mfma_supported(const AttnParams&) { return false; }
void launch_attention_mfma(const AttnParams&, hipStream_t) {}
