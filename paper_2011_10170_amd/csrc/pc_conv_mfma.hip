// Matrix-core (MFMA) variant of the three passes for bf16 layers. Placeholder until the kernels land.
#include "pc_internal.h"

bool pc_mfma_supports(int F, int C) { (void)F; (void)C; return false; }
pc_status pc_launch_pack_tiles(pc_ctx *ctx, pc_packed *pk, const float *W)
{
    (void)pk; (void)W;
    return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA variant not built");
}
pc_status pc_mfma_fwd(pc_ctx *ctx, const pc_conv_desc *, const pc_packed *, const void *, void *)
{ return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA variant not built"); }
pc_status pc_mfma_bwd_data(pc_ctx *ctx, const pc_conv_desc *, const pc_packed *, const void *, void *)
{ return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA variant not built"); }
pc_status pc_mfma_bwd_weight(pc_ctx *ctx, const pc_conv_desc *, const pc_packed *, const void *, const void *, float *)
{ return pc_fail(ctx, PC_ERR_UNSUPPORTED, "MFMA variant not built"); }
