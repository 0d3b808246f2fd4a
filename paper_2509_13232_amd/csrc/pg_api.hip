// C entry points of the clipped policy-gradient loss: argument checks and the
// choice between the fused (hidden, W) form and the logits-in form.
#include "pg_common.hpp"

namespace spo {
int fused_fwd_workspace(const spo_pg_desc *d, size_t *bytes);
int fused_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats, void *ws,
              size_t ws_bytes, hipStream_t s);
int fused_bwd_workspace(const spo_pg_desc *d, int64_t chunk_tokens, size_t *bytes);
int fused_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss, void *d_hidden,
              int d_hidden_dtype, void *d_W, int d_W_dtype, int accumulate_dW, int64_t chunk_tokens, void *ws,
              size_t ws_bytes, hipStream_t s);
int fused_fwd_bwd_workspace(const spo_pg_desc *d, int64_t chunk_tokens, size_t *bytes);
int fused_fwd_bwd(const spo_pg_desc *d, float grad_loss, float *loss, float *logp, float *lse, float *stats,
                  void *d_hidden, int d_hidden_dtype, void *d_W, int d_W_dtype, int accumulate_dW,
                  int64_t chunk_tokens, void *ws, size_t ws_bytes, hipStream_t s);
int logits_fwd_workspace(const spo_pg_desc *d, size_t *bytes);
int logits_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats, void *ws,
               size_t ws_bytes, hipStream_t s);
int logits_bwd_workspace(const spo_pg_desc *d, size_t *bytes);
int logits_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss, void *d_logits,
               void *ws, size_t ws_bytes, hipStream_t s);
}  // namespace spo

using namespace spo;

static bool dtype_ok(int t) { return t == SPO_FP32 || t == SPO_BF16; }

extern "C" const char *spo_status_string(int status) {
    switch (status) {
        case SPO_OK: return "ok";
        case SPO_EINVAL: return "invalid argument";
        case SPO_ENULL: return "required pointer is NULL";
        case SPO_ERANGE: return "size beyond what the kernels support";
        case SPO_EWORKSPACE: return "workspace missing or too small";
        case SPO_EUNSUPPORTED: return "combination not supported by this build";
        case SPO_EHIP: return "HIP runtime error at launch";
        default: return "unknown status";
    }
}

extern "C" size_t spo_pg_loss_fwd_workspace_bytes(const spo_pg_desc *d) {
    if (validate_pg_desc(d) != SPO_OK) return 0;
    size_t b = 0;
    if (d->logits) logits_fwd_workspace(d, &b); else fused_fwd_workspace(d, &b);
    return b;
}

extern "C" int spo_pg_loss_fwd(const spo_pg_desc *d, float *loss, float *logp, float *lse, float *stats,
                               void *ws, size_t ws_bytes, spo_stream_t stream) {
    const int rc = validate_pg_desc(d);
    if (rc) return rc;
    if (!loss || (d->T > 0 && (!logp || !lse))) return SPO_ENULL;
    if (!ws) return SPO_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return SPO_EINVAL;
    return d->logits ? logits_fwd(d, loss, logp, lse, stats, ws, ws_bytes, as_stream(stream))
                     : fused_fwd(d, loss, logp, lse, stats, ws, ws_bytes, as_stream(stream));
}

extern "C" size_t spo_pg_loss_bwd_workspace_bytes(const spo_pg_desc *d, int64_t chunk_tokens) {
    if (validate_pg_desc(d) != SPO_OK || chunk_tokens < 0) return 0;
    size_t b = 0;
    if (d->logits) logits_bwd_workspace(d, &b); else fused_bwd_workspace(d, chunk_tokens, &b);
    return b;
}

extern "C" int spo_pg_loss_bwd(const spo_pg_desc *d, const float *logp, const float *lse, float grad_loss,
                               void *d_hidden, int d_hidden_dtype, void *d_W, int d_W_dtype, int accumulate_dW,
                               void *d_logits, int64_t chunk_tokens, void *ws, size_t ws_bytes,
                               spo_stream_t stream) {
    const int rc = validate_pg_desc(d);
    if (rc) return rc;
    if (d->T > 0 && (!logp || !lse)) return SPO_ENULL;
    if (chunk_tokens < 0) return SPO_EINVAL;
    if (!ws) return SPO_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return SPO_EINVAL;
    if (d->logits) return logits_bwd(d, logp, lse, grad_loss, d_logits, ws, ws_bytes, as_stream(stream));
    if ((d_hidden && !dtype_ok(d_hidden_dtype)) || (d_W && !dtype_ok(d_W_dtype))) return SPO_EINVAL;
    if ((d_hidden && reinterpret_cast<uintptr_t>(d_hidden) % 16) || (d_W && reinterpret_cast<uintptr_t>(d_W) % 16))
        return SPO_EINVAL;
    return fused_bwd(d, logp, lse, grad_loss, d_hidden, d_hidden_dtype, d_W, d_W_dtype, accumulate_dW, chunk_tokens,
                     ws, ws_bytes, as_stream(stream));
}

extern "C" size_t spo_pg_loss_fwd_bwd_workspace_bytes(const spo_pg_desc *d, int64_t chunk_tokens) {
    if (validate_pg_desc(d) != SPO_OK || chunk_tokens < 0 || d->logits) return 0;
    size_t b = 0;
    fused_fwd_bwd_workspace(d, chunk_tokens, &b);
    return b;
}

extern "C" int spo_pg_loss_fwd_bwd(const spo_pg_desc *d, float grad_loss, float *loss, float *logp, float *lse,
                                   float *stats, void *d_hidden, int d_hidden_dtype, void *d_W, int d_W_dtype,
                                   int accumulate_dW, int64_t chunk_tokens, void *ws, size_t ws_bytes,
                                   spo_stream_t stream) {
    const int rc = validate_pg_desc(d);
    if (rc) return rc;
    if (d->logits) return SPO_EUNSUPPORTED;  // with the logits given there is nothing to save: call fwd, then bwd
    if (!loss || (d->T > 0 && (!logp || !lse))) return SPO_ENULL;
    if (chunk_tokens < 0) return SPO_EINVAL;
    if (!ws) return SPO_EWORKSPACE;
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0) return SPO_EINVAL;
    if ((d_hidden && !dtype_ok(d_hidden_dtype)) || (d_W && !dtype_ok(d_W_dtype))) return SPO_EINVAL;
    if ((d_hidden && reinterpret_cast<uintptr_t>(d_hidden) % 16) || (d_W && reinterpret_cast<uintptr_t>(d_W) % 16))
        return SPO_EINVAL;
    return fused_fwd_bwd(d, grad_loss, loss, logp, lse, stats, d_hidden, d_hidden_dtype, d_W, d_W_dtype, accumulate_dW,
                         chunk_tokens, ws, ws_bytes, as_stream(stream));
}
