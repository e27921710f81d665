// Entry points not implemented yet: they report SM_ERR_UNSUPPORTED.
#include "common.h"
using namespace sm;
extern "C" {
size_t sm_attn_block_workspace_bytes(const sm_attn_cfg*, int) { return 0; }
int sm_attn_block(const sm_attn_cfg*, const void* const*, const void*, const void*, void*, void*, size_t, int, void*) { return fail(SM_ERR_UNSUPPORTED, "sm_attn_block: not implemented"); }
size_t sm_run_chain_workspace_bytes(const sm_chain_desc*, int) { return 0; }
int sm_run_chain(const sm_chain_desc*, const void* const*, int, const void*, void*, void*, void*, size_t, int, void*) { return fail(SM_ERR_UNSUPPORTED, "sm_run_chain: not implemented"); }
}
