// Stand-ins for the kernel launchers (kernels_*.hip) in host-only builds of the runtime: the sanitizer tests link
// api.cpp, host_build.cpp and sampler.cpp without any device code; a host-only context never reaches a launcher.
#include "../../paper_2408_08490_amd/csrc/common.h"

namespace hgnn {
hgnn_status launch_merge(hipStream_t s, int dtype, int T, const void *const *store, const int32_t *feat_dim,
                         const int64_t *const *ids, const int64_t *n_rows, const int64_t *elem_off, void *out, int mode,
                         const int32_t *const *pos, const void *interleaved) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_spmm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            int max_dim, const void *x, void *z, void *zlo, int row_begin, int row_end, const TransposeJobs *tj) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_aggregate_literal(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *feature_cat,
                                     void *z, void *zlo) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_spmm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, int max_dim, uint32_t want_types, const void *dz, void *dx, float *partial) { return HGNN_EUNSUPPORTED; }
bool launch_spmm_fwd_uniform(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *z, void *zlo,
                             int row_begin, int row_end) { return false; }
bool launch_spmm_bwd_uniform(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                             int F, uint32_t want, const void *dz, void *dx, float *partial) { return false; }
hgnn_status launch_transpose_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt,
                                     const PtrTab &pt, const WtTab &wt, int H, void *wt_buf) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_gemm_fwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const WtTab &wt, const SegTab &tiles, const uint32_t *live_mask, int H,
                            int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h,
                            int only_seg, float *acc32, int tile_mn) { return HGNN_EUNSUPPORTED; }
bool launch_gemm2_fwd(hipStream_t s, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, const uint32_t *live_mask,
                      int H, int relu, const void *x, const void *z, const void *zlo, const void *wt_buf, void *h, hgnn_status *st) { return false; }
hgnn_status launch_attn_proj(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &w_type_as_root, const SegTab &tiles, int H,
                             const void *x, void *z, bool z_f32) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_agg(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const void *const *a_src, const void *const *a_dst, int H, int heads, const void *z, void *mout,
                            float *mx, float *ls) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_sem(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, const void *mbuf,
                            const void *w_sem, const void *b_sem, const void *q_sem, void *tbuf, float *wsum) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_beta(hipStream_t s, const TypeTab &tt, const RelTab &rt, const float *wsum, float *beta, const float *dbeta,
                             float *coef, int mode) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_fuse(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, int H,
                             int relu, const void *mbuf, const float *beta, void *h) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_zero(hipStream_t s, float *const *ptrs, const int64_t *counts, int n) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_dbeta(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg,
                              const void *gp, const void *mbuf, float *dbeta) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_du(hipStream_t s, int dtype, const LayerDev &L, const RelTab &rt, const void *tbuf, const void *q_sem,
                           const float *coef, void *du, float *dq, float *dbs) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_dm(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, int H, int ldg, const void *du,
                           const void *w_sem, const void *gp, const float *beta, void *dm) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_dws(hipStream_t s, int dtype, int64_t rows, int H, const void *mbuf, const void *du, float *dws) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_attn_agg_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt, const void *const *a_src,
                                const void *const *a_dst, float *const *da_src, float *const *da_dst, int H, int heads, const void *z,
                                const void *mbuf, const void *dm, const float *mx, const float *ls, float *alpha, float *dsb,
                                float *dsum, void *dz, float *partial) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_bias_act(hipStream_t s, int dtype, const TypeTab &tt, const PtrTab &pt, int H, int relu,
                            int type, const float *acc32, void *h) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_gemm_da(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const PtrTab &pt, const SegTab &tiles, int ldg, bool fast, const void *gp, void *dz) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_gemm_bwd(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                            const PtrTab &pt, const DwTab &da_tiles, const GradPtrTab &gt, const DwTab &dw_tiles,
                            int split_rows, int H, int ldg, bool fast, const void *x, const void *z, const void *gp, void *dz,
                            const float *bpart, int rpb) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_gemm_dw(hipStream_t s, int dtype, const LayerDev &L, const TypeTab &tt, const RelTab &rt,
                           const GradPtrTab &gt, const DwTab &tiles, int split_rows, int H, int ldg, bool fast,
                           const void *x, const void *z, const void *gp) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_adam_dense(hipStream_t s, int dtype, int n, void *const *param, float *const *master,
                              const float *const *grad, float *const *m, float *const *v, const int64_t *numel,
                              float lr, float b1, float b2, float eps, double c1, double c2) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_adam_rows(hipStream_t s, int dtype, void *store, float *master, float *m, float *v, int F,
                             const int64_t *ids, int64_t n_rows, const void *grad, float lr, float b1, float b2,
                             float eps, double c1, double c2) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_relu_bias_bwd(hipStream_t s, int dtype, const TypeTab &tt, int H, int ldo, int relu,
                                 const void *grad_h, const void *h, void *gp, const GradPtrTab &gt) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_pad_weights(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt,
                               const WtTab &wo, int H, int Hp, void *out) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_zero_grads(hipStream_t s, const TypeTab &tt, const RelTab &rt, const GradPtrTab &gt, int H) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_bwd_prep(hipStream_t s, int dtype, const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wo,
                            const GradPtrTab &gt, int H, int ldo, int relu, bool do_rows, bool do_zero, const void *grad_h,
                            const void *h, void *gp, float *bpart, size_t bpart_rows, void *wpad, int *rows_per_block) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_bias_reduce(hipStream_t s, const TypeTab &tt, const GradPtrTab &gt, int H, int rpb, const float *bpart) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_fill_zero(hipStream_t s, void *p, size_t bytes) { return HGNN_EUNSUPPORTED; }
bool launch_spmm_fwd_uniform(hipStream_t s, int dtype, const LayerDev &L, int F, const void *x, void *z, void *zlo,
                             int row_begin, int row_end, const uint64_t *gaddr, const TransposeJobs *tj) { return false; }
hgnn_status launch_gather_addresses(hipStream_t s, const LayerDev &L, const GatherSrc &gs, int row_bytes, uint64_t *gaddr) { return HGNN_EUNSUPPORTED; }
void make_transpose_jobs(const TypeTab &tt, const RelTab &rt, const PtrTab &pt, const WtTab &wt, int H, void *wt_buf,
                         TransposeJobs &tj) { tj.n = 0; tj.blocks = 0; }
hgnn_status launch_transpose_jobs(hipStream_t s, int dtype, const TransposeJobs &tj) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_convert(hipStream_t s, bool widen, const void *const *src, void *const *dst, const int64_t *n, int count) { return HGNN_EUNSUPPORTED; }
hgnn_status launch_xent(hipStream_t s, int dtype, const void *logits, const int64_t *labels, int64_t rows,
                        int classes, float *loss, void *grad) { return HGNN_EUNSUPPORTED; }
hgnn_status static_scratch_init(int) { return HGNN_EUNSUPPORTED; }
void *static_scratch_ptr(int) { return nullptr; }
}  // namespace hgnn
