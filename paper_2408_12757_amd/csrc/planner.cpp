// Auto-search (paper Sec. 4.1): kernel profiles and the pipeline search.
#include "nf_internal.h"

struct NfProfile {
  int dummy;
};

void nf_profile_free(nf_ctx* ctx) {
  delete ctx->profile;
  ctx->profile = nullptr;
}

extern "C" int nf_profile(nf_ctx* ctx, const nf_model_desc* model, int max_tokens, int granule,
                          const char* cache_path) {
  (void)ctx; (void)model; (void)max_tokens; (void)granule; (void)cache_path;
  return NF_EINVAL;
}

extern "C" int nf_plan_nanobatches(nf_ctx* ctx, const nf_model_desc* model, const nf_batch* batch, int max_nano,
                                   int granule, nf_plan** out) {
  if (!ctx || !batch || !out) return NF_EINVAL;
  (void)granule;
  if (max_nano == 1 || batch->n_tokens == 0) {
    const int32_t bounds[2] = {0, batch->n_tokens};
    return nf_plan_manual(ctx, model, batch, 1, bounds, 0, 0, 0, 0, out);
  }
  return NF_EINVAL;
}
