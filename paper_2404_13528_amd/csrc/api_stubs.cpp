// Entry points not implemented yet: they report SM_ERR_UNSUPPORTED.
#include "common.h"
using namespace sm;
extern "C" {
size_t sm_attn_block_workspace_bytes(const sm_attn_cfg*, int) { return 0; }
int sm_attn_block(const sm_attn_cfg*, const void* const*, const void*, const void*, void*, void*, size_t, int, void*) { return fail(SM_ERR_UNSUPPORTED, "sm_attn_block: not implemented"); }
}
