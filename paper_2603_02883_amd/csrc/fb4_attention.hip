// C ABI of the FB4 quantizer library, the attention-guided entry points (Sec. 3.3, 3.4, App. F): scores on the
// matrix cores, the per-tile choice, SeDA's main anchors and correlated tokens.  Declarations and contracts are in
// include/fb4.h.
#include "fb4_common.hpp"
#include "fb4_salient.hpp"

using namespace fb4;

extern "C" {

int fb4_attention_scores(const void* q, const void* k, int64_t groups, int64_t tokens, int64_t dim, int mode,
                         float* scores, void* stream)
{
    if (groups < 0 || tokens < 0 || dim < 0 || (mode != 0 && mode != 1)) return FB4_ERR_INVALID_ARG;
    if (groups == 0 || tokens == 0) return FB4_OK;
    if (!q || !k || !scores || dim == 0) return FB4_ERR_INVALID_ARG;
    if ((dim % 8) || dim > 256 || !aligned(q, 16) || !aligned(k, 16) || !aligned(scores, 4)) return FB4_ERR_UNSUPPORTED;
    const bool small = tokens <= (int64_t)kScoreShortGroup;
    const int64_t per_wg = small ? 128 : 256;   // queries per workgroup of the two kernel shapes
    const int64_t bpg = (tokens + per_wg - 1) / per_wg;
    if (tokens * dim > 0x7FFFFFFFll || groups * bpg > 0x7FFFFFFFll) return FB4_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const dim3 grid((unsigned)(groups * bpg));
    if (dim == kDmaDim && !small && tokens % 128 == 0) {
        // rows of exactly 128 channels, key halves made of whole 64-key blocks: the kernel that loads straight to LDS
        if (mode) hipLaunchKernelGGL(attention_scores_dma_kernel<true>, grid, dim3(kScoreThreads), 0, s, static_cast<const uint16_t*>(q),
                                     static_cast<const uint16_t*>(k), (uint32_t)tokens, (uint32_t)bpg, scores);
        else hipLaunchKernelGGL(attention_scores_dma_kernel<false>, grid, dim3(kScoreThreads), 0, s, static_cast<const uint16_t*>(q),
                                static_cast<const uint16_t*>(k), (uint32_t)tokens, (uint32_t)bpg, scores);
        return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
    }
#define FB4_SCORE_ARGS static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), (uint32_t)tokens, (uint32_t)dim, (uint32_t)bpg, scores
#define FB4_SCORE_LAUNCH(d, relu, qb, keys) hipLaunchKernelGGL((attention_scores_kernel<d, relu, qb, keys>), grid, dim3(kScoreThreads), 0, s, FB4_SCORE_ARGS)
#define FB4_SCORE_CASE(d)                                   \
    case d:                                                 \
        if (small) {                                        \
            if (mode) FB4_SCORE_LAUNCH(d, true, 1, 32);     \
            else FB4_SCORE_LAUNCH(d, false, 1, 32);         \
        } else {                                            \
            if (mode) FB4_SCORE_LAUNCH(d, true, 2, 64);     \
            else FB4_SCORE_LAUNCH(d, false, 2, 64);         \
        }                                                   \
        break;
    switch ((int)((dim + 31) / 32)) {
        FB4_SCORE_CASE(1) FB4_SCORE_CASE(2) FB4_SCORE_CASE(3) FB4_SCORE_CASE(4)
        FB4_SCORE_CASE(5) FB4_SCORE_CASE(6) FB4_SCORE_CASE(7) FB4_SCORE_CASE(8)
        default: return FB4_ERR_UNSUPPORTED;
    }
#undef FB4_SCORE_CASE
#undef FB4_SCORE_LAUNCH
#undef FB4_SCORE_ARGS
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_select_salient_tokens(const float* scores, int64_t frames, int heads, int grid_h, int grid_w, int tile_h,
                              int tile_w, int32_t* rows_out, void* stream)
{
    if (frames < 0 || heads < 1 || grid_h < 1 || grid_w < 1 || tile_h < 1 || tile_w < 1) return FB4_ERR_INVALID_ARG;
    if (frames == 0) return FB4_OK;
    if (!scores || !rows_out) return FB4_ERR_INVALID_ARG;
    const int64_t tokens = (int64_t)grid_h * grid_w;
    if (tokens > (int64_t)kSelectMaxTokens || frames * tokens > 0x7FFFFFFFll || !aligned(scores, 4) || !aligned(rows_out, 4))
        return FB4_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(select_salient_kernel, dim3((unsigned)frames), dim3(kSelectThreads), 0, static_cast<hipStream_t>(stream),
                       scores, (uint32_t)heads, (uint32_t)grid_h, (uint32_t)grid_w, (uint32_t)tile_h, (uint32_t)tile_w, rows_out);
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_seda_assign(const void* q, const void* k, int joint, int64_t frames, int heads, int grid_h, int grid_w,
                    int64_t dim, const int32_t* anchors, int64_t n_anchors, int tile_h, int tile_w, int window,
                    int window_t, float threshold, int32_t* token_group, int32_t* anchor_group, float* window_scores,
                    void* stream)
{
    if (frames < 0 || heads < 1 || grid_h < 1 || grid_w < 1 || dim < 1 || n_anchors < 0 || window < 1 || window_t < 1 ||
        tile_h < 1 || tile_w < 1 || (joint != 0 && joint != 1))
        return FB4_ERR_INVALID_ARG;
    if (!(threshold == threshold)) return FB4_ERR_INVALID_ARG;
    if (!joint && window_t != 1) return FB4_ERR_INVALID_ARG;   // factorized attention has no scores across frames
    if (frames == 0) return FB4_OK;
    if (!token_group || !anchor_group || (n_anchors > 0 && (!q || !k || !anchors))) return FB4_ERR_INVALID_ARG;
    const int64_t tokens = (int64_t)grid_h * grid_w;
    if ((dim % 8) || window > 8 || window_t > 64 || !aligned(q, 16) || !aligned(k, 16) || !aligned(anchors, 4) ||
        !aligned(token_group, 4) || !aligned(anchor_group, 4) || (window_scores && !aligned(window_scores, 4)))
        return FB4_ERR_UNSUPPORTED;
    if (frames * tokens > 0x7FFFFFFFll || n_anchors > 0x7FFFFFFFll || tokens * dim > 0x7FFFFFFFll) return FB4_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint32_t n = (uint32_t)(frames * tokens);
    hipLaunchKernelGGL(seda_fill_kernel, dim3((n + 255) / 256), dim3(256), 0, s, token_group, anchor_group, n);
    if (n_anchors > 0) {
        AssignParams p = {};
        p.frames = (uint32_t)frames; p.heads = (uint32_t)heads; p.grid_h = (uint32_t)grid_h; p.grid_w = (uint32_t)grid_w;
        p.dim = (uint32_t)dim; p.tile_h = (uint32_t)tile_h; p.tile_w = (uint32_t)tile_w;
        p.window = (uint32_t)window; p.window_t = (uint32_t)window_t;
        p.stride_f = joint ? (uint64_t)tokens : (uint64_t)heads * tokens;
        p.stride_h = joint ? (uint64_t)frames * tokens : (uint64_t)tokens;
        p.threshold = threshold;
        hipLaunchKernelGGL(seda_mark_kernel, dim3((unsigned)n_anchors, (unsigned)window_t), dim3(kAssignThreads), 0, s,
                           static_cast<const uint16_t*>(q), static_cast<const uint16_t*>(k), anchors, p, token_group,
                           window_scores);
        hipLaunchKernelGGL(seda_anchor_kernel, dim3((unsigned)((n_anchors + 255) / 256)), dim3(256), 0, s, anchors,
                           (uint32_t)n_anchors, (uint32_t)frames, (uint32_t)grid_h, (uint32_t)grid_w, (uint32_t)tile_h,
                           (uint32_t)tile_w, token_group, anchor_group);
    }
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_seda_main_anchor(const float* temporal_scores, const void* qt, const void* kt, int64_t frames, int heads,
                         int grid_h, int grid_w, int64_t dim, const int32_t* candidates, int n_per_frame, int tile_h,
                         int tile_w, float prune_threshold, int32_t* main_anchor, int32_t* kept, float* prune_scores,
                         void* stream)
{
    if (frames < 0 || heads < 1 || grid_h < 1 || grid_w < 1 || dim < 1 || n_per_frame < 0 || tile_h < 1 || tile_w < 1)
        return FB4_ERR_INVALID_ARG;
    if (!(prune_threshold == prune_threshold)) return FB4_ERR_INVALID_ARG;
    if (!main_anchor) return FB4_ERR_INVALID_ARG;
    const int64_t tokens = (int64_t)grid_h * grid_w;
    const int64_t tiles = (int64_t)((grid_h + tile_h - 1) / tile_h) * ((grid_w + tile_w - 1) / tile_w);
    const int64_t n_cand = frames * n_per_frame;
    if (n_cand > 0 && (!temporal_scores || !qt || !kt || !candidates || !kept)) return FB4_ERR_INVALID_ARG;
    if ((dim % 8) || frames > (int64_t)kMainMaxFrames || !aligned(qt, 16) || !aligned(kt, 16) || !aligned(temporal_scores, 4) ||
        !aligned(candidates, 4) || !aligned(main_anchor, 4) || !aligned(kept, 4) || (prune_scores && !aligned(prune_scores, 4)))
        return FB4_ERR_UNSUPPORTED;
    if (frames * tokens > 0x7FFFFFFFll || n_cand > 0x7FFFFFFFll || frames * dim > 0x7FFFFFFFll) return FB4_ERR_UNSUPPORTED;
    hipStream_t s = static_cast<hipStream_t>(stream);
    hipLaunchKernelGGL(seda_main_anchor_kernel, dim3((unsigned)tiles), dim3(kMainThreads), 0, s, temporal_scores,
                       static_cast<const uint16_t*>(qt), static_cast<const uint16_t*>(kt), (uint32_t)frames, (uint32_t)heads,
                       (uint32_t)grid_h, (uint32_t)grid_w, (uint32_t)dim, candidates, (uint32_t)n_per_frame, (uint32_t)tile_h,
                       (uint32_t)tile_w, prune_threshold, main_anchor, kept, prune_scores);
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_seda_main_anchor_3d(const float* scores, int64_t frames, int heads, int grid_h, int grid_w, int tile_h,
                            int tile_w, int32_t* anchors, void* stream)
{
    if (frames < 1 || heads < 1 || grid_h < 1 || grid_w < 1 || tile_h < 1 || tile_w < 1) return FB4_ERR_INVALID_ARG;
    if (!scores || !anchors) return FB4_ERR_INVALID_ARG;
    const int64_t tokens = (int64_t)grid_h * grid_w;
    const int64_t tiles = (int64_t)((grid_h + tile_h - 1) / tile_h) * ((grid_w + tile_w - 1) / tile_w);
    if (frames * tokens > 0x7FFFFFFFll || !aligned(scores, 4) || !aligned(anchors, 4)) return FB4_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(seda_main_anchor_3d_kernel, dim3((unsigned)tiles), dim3(kMainThreads), 0,
                       static_cast<hipStream_t>(stream), scores, (uint32_t)frames, (uint32_t)heads, (uint32_t)grid_h,
                       (uint32_t)grid_w, (uint32_t)tile_h, (uint32_t)tile_w, anchors);
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

int fb4_probe_mfma_rate(int64_t workgroups, int64_t iterations, int random_operands, float* out, double* flop, void* stream)
{
    if (workgroups < 1 || workgroups > 65536 || iterations < 0 || iterations > 0x7FFFFFFFll || !out) return FB4_ERR_INVALID_ARG;
    if (!aligned(out, 4)) return FB4_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(probe_mfma_rate_kernel, dim3((unsigned)workgroups), dim3(256), 0, static_cast<hipStream_t>(stream), out,
                       (uint32_t)iterations, (uint32_t)(random_operands != 0));
    // four wavefronts x 8 x 4 MFMAs of 32 x 32 x 16 per iteration, two operations per multiply-add
    if (flop) *flop = (double)workgroups * 4.0 * (double)iterations * 32.0 * (2.0 * 32 * 32 * 16);
    return hipGetLastError() == hipSuccess ? FB4_OK : FB4_ERR_HIP;
}

}  // extern "C"
