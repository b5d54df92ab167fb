// bf16 partial attention (placeholder: routes through the fp32-arithmetic kernel).
#include "attention_common.h"

namespace dy {
void launch_attention_bf16(const AttnArgs &a, hipStream_t s) { launch_attention_f32(BF16, a, s); }
}  // namespace dy
