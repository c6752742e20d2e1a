// Host-side plan and validation of the KD step (see kd_host.h); the kernels and their sequencing are in kd.hip.
#include "kd_host.h"

KdPlan kd_plan(const ms_kd_config *kd, int n, void *ws) {
    Arena a(ws);
    KdPlan p;
    p.keep = kd->token_block > 0;
    p.tb = p.keep && kd->token_block < n ? kd->token_block : n;
    const size_t nc = (size_t)p.tb * kd->chunk;
    const size_t nchunks = p.keep ? (size_t)ms_cdiv(kd->vocab, kd->chunk) : 1;
    p.zt = a.take<float>(nchunks * nc * 4);
    p.zs = a.take<float>(nc * 4);
    p.stats = a.take<float>((size_t)n * kKdStat * 4);
    p.dz = a.take<void>(nc * ms_dtype_size(kd->dtype));
    p.dhs = a.take<float>((size_t)n * kd->h_student * 4);
    p.bytes = a.off;
    return p;
}

ms_status validate_kd(const ms_kd_config *kd, int n_tokens) {
    if (!kd) return ms_fail(MS_ERR_INVALID_ARG, "kd: null config");
    if (n_tokens < 0) return ms_fail(MS_ERR_INVALID_ARG, "kd: negative token count");
    if (kd->dtype != MS_BF16 && kd->dtype != MS_F32) return ms_fail(MS_ERR_INVALID_ARG, "kd: bad dtype");
    if (kd->vocab <= 0 || kd->h_teacher <= 0 || kd->h_student <= 0 || kd->chunk <= 0)
        return ms_fail(MS_ERR_SHAPE, "kd: vocab, hidden sizes and chunk must be positive");
    if (!(kd->temperature > 0.f)) return ms_fail(MS_ERR_INVALID_ARG, "kd: temperature must be positive");
    if (kd->token_block < 0 || kd->token_block % 8) return ms_fail(MS_ERR_INVALID_ARG, "kd: token_block must be 0 or a positive multiple of 8");
    if (kd->vocab % 8 || kd->chunk % 8 || kd->h_teacher % 8 || kd->h_student % 8)
        return ms_fail(MS_ERR_UNSUPPORTED, "kd: vocab, chunk and hidden sizes must be multiples of 8");
    if (!kd->w_teacher_dev || !kd->w_student_dev) return ms_fail(MS_ERR_INVALID_ARG, "kd: null lm_head pointer");
    return MS_OK;
}

extern "C" size_t ms_kd_workspace_bytes(const ms_kd_config *kd, int32_t max_tokens) {
    if (!kd || max_tokens < 0 || kd->chunk <= 0 || kd->h_student <= 0 || kd->vocab <= 0 || kd->token_block < 0) return 0;
    return kd_plan(kd, max_tokens, nullptr).bytes;
}
