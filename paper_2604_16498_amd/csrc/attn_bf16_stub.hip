// Interim bf16 attention routing: the vector-ALU kernel serves decode until the
// split-KV kernel takes over.
#include "common.hpp"
namespace forge {
forge_status launch_attn_decode_bf16(const AttnArgs& a, hipStream_t s) { return launch_attn_simple_bf16(a, s); }
size_t attn_decode_workspace_bytes(int, int, int, int, int) { return 0; }
}  // namespace forge
