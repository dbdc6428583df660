// Inverted-residual block: ternary pointwise expand -> int8 depthwise 3x3 -> ternary
// pointwise project (+ saturating skip), paper Section 2 and Figure 4.  This version chains
// the three kernels on the caller's stream through two intermediates in the workspace.
#include "prom.h"

namespace {
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }
}

extern "C" size_t prom_block_workspace_size(int n, int h, int w, int cin, int chid, int cout, int stride)
{
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return 0;
    const size_t ho = (size_t)(h - 1) / stride + 1, wo = (size_t)(w - 1) / stride + 1;
    return round256((size_t)n * h * w * chid) + round256((size_t)n * ho * wo * chid);
}

extern "C" int prom_block(const int8_t *x, int n, int h, int w, int cin, int chid, int cout, int stride,
                          const void *w_expand_packed, const prom_requant_t *rq_expand,
                          const int8_t *w_dw, const prom_requant_t *rq_dw,
                          const void *w_project_packed, const prom_requant_t *rq_project,
                          int add_residual, void *workspace, size_t workspace_bytes, int8_t *y,
                          void *stream)
{
    if (!x || !y || !w_expand_packed || !w_dw || !w_project_packed || !rq_expand || !rq_dw || !rq_project)
        return PROM_EINVAL;
    if (n <= 0 || h <= 0 || w <= 0 || cin <= 0 || chid <= 0 || cout <= 0 || (stride != 1 && stride != 2))
        return PROM_EINVAL;
    if (add_residual && !(stride == 1 && cin == cout)) return PROM_EINVAL;
    const size_t need = prom_block_workspace_size(n, h, w, cin, chid, cout, stride);
    if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255) != 0) return PROM_EWORKSPACE;
    const int ho = (h - 1) / stride + 1, wo = (w - 1) / stride + 1;
    int8_t *t1 = static_cast<int8_t *>(workspace);
    int8_t *t2 = t1 + round256((size_t)n * h * w * chid);
    {
        const uintptr_t ya = (uintptr_t)y, wa = (uintptr_t)workspace;
        const size_t yb = (size_t)n * ho * wo * cout;
        if (ya < wa + need && wa < ya + yb) return PROM_EALIAS;
    }
    // Validate every stage before enqueueing anything: argument errors of the later stages
    // are all covered by the checks above plus the windows checked here.
    const prom_requant_t *rqs[3] = {rq_expand, rq_dw, rq_project};
    for (const prom_requant_t *rq : rqs) {
        if (!rq->bias || !rq->mult || !rq->shift) return PROM_EINVAL;
        if (rq->act_min < -128 || rq->act_max > 127 || rq->act_min > rq->act_max) return PROM_EINVAL;
    }
    if (cin > 4096 || chid > 4096) return PROM_EUNSUPPORTED;
    int rc = prom_pw_conv(x, n, h, w, cin, w_expand_packed, chid, rq_expand, nullptr, t1, stream);
    if (rc != PROM_OK) return rc;
    rc = prom_dw_conv(t1, n, h, w, chid, w_dw, stride, rq_dw, t2, stream);
    if (rc != PROM_OK) return rc;
    return prom_pw_conv(t2, n, ho, wo, chid, w_project_packed, cout, rq_project,
                        add_residual ? x : nullptr, y, stream);
}
