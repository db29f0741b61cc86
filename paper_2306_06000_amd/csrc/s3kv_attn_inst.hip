// Instantiations of the multi-head attention kernels for ONE head dimension (S3_INST_D, given on the
// compiler's command line); the library links one object per supported head dimension.
#include <hip/hip_runtime.h>

#include "s3kv_attn.h"

#ifndef S3_INST_D
#error "compile with -DS3_INST_D=<head dimension>"
#endif

#define S3_CAT2(a, b) a##b
#define S3_CAT(a, b) S3_CAT2(a, b)

// Kernel of shape `variant` for element type dt (S3_F16 / S3_BF16): the fused step kernel or the
// attention-only kernel; null for an unknown shape or type.
attn_fn S3_CAT(s3i_pick_mha_d, S3_INST_D)(int dt, int variant, bool fused) {
    if (dt == S3_F16) return pick_variant<S3_F16, S3_INST_D>(variant, fused);
    if (dt == S3_BF16) return pick_variant<S3_BF16, S3_INST_D>(variant, fused);
    return nullptr;
}

attn_fn S3_CAT(s3i_pick_merge_d, S3_INST_D)() { return (attn_fn)attn_merge_kernel<S3_INST_D>; }

#if S3_INST_D == 64
struct VariantShape {
    int ts, hs, u, nt, pf, ring, dyn, xs;
};
static const VariantShape kVariants[] = {
#define X(i, ts, hs, u, nt, pf, r, dyn, xs) {ts, hs, u, nt, pf, r, dyn, xs},
    S3_VARIANTS(X)
#undef X
};
int s3i_num_variants() { return (int)(sizeof(kVariants) / sizeof(kVariants[0])); }
int s3i_default_variant() { return S3_DEFAULT_VARIANT; }
int s3i_default_variant_large() { return S3_DEFAULT_VARIANT_LARGE; }  // batches of more than 128 sequences
// Threads of a workgroup of shape `variant` (the fused kernel adds its epilogue wave).
int s3i_variant_threads(int variant, bool fused) {
    if (variant < 0 || variant >= s3i_num_variants()) return 0;
    return (kVariants[variant].ts * kVariants[variant].hs + (fused ? 1 : 0)) * 64;
}
// Bytes of LDS rings a workgroup of the fused kernel of shape `variant` needs behind the batch view.
int s3i_variant_ring_bytes(int variant) {
    if (variant < 0 || variant >= s3i_num_variants()) return 0;
    return kVariants[variant].ring * 2048 * kVariants[variant].ts * kVariants[variant].hs;
}
int s3i_variant_dynamic(int variant) { return variant >= 0 && variant < s3i_num_variants() ? kVariants[variant].dyn : 0; }
// Whether the fused kernel of shape `variant` carries its row stream across items.
int s3i_variant_stream(int variant) { return variant >= 0 && variant < s3i_num_variants() ? kVariants[variant].xs : 0; }
#endif
