// extern "C" boundary of the library: argument checks and dispatch only.
// Every step of the path runs in the kernels of the other translation units.

#include <stdlib.h>

#include "qadc_scan_common.h"
#include "qadc_profile.h"

namespace qadc {

char *err_buf()
{
    static thread_local char buf[512] = "";
    return buf;
}

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(err_buf(), 512, fmt, ap);
    va_end(ap);
    return code;
}

namespace {
thread_local Knobs g_knobs = {-1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1, -1};
int env_knob(const char *name)
{
    const char *s = getenv(name);
    if (!s || !*s) return -1;
    const int v = atoi(s);
    return v < 0 ? 0 : v;
}
}  // namespace

const Knobs &knobs() { return g_knobs; }

void knobs_refresh()
{
    Knobs &k = g_knobs;
    k.scan_nt = env_knob("QADC_SCAN_NT");
    k.scan_wgs = env_knob("QADC_SCAN_WGS");
    k.seed_min_tiles = env_knob("QADC_SEED_MIN_TILES");
    k.seed_wgs = env_knob("QADC_SEED_WGS");
    k.tiled = env_knob("QADC_TILED");
    k.tiled_seed = env_knob("QADC_TILED_SEED");
    k.scan_f32_wgs = env_knob("QADC_SCAN_F32_WGS");
    k.tiled_mfma = env_knob("QADC_TILED_MFMA");
    k.mfma_min_q = env_knob("QADC_MFMA_MIN_Q");
    k.mfma_min_q2 = env_knob("QADC_MFMA_MIN_Q2");
    k.mfma_min_q4 = env_knob("QADC_MFMA_MIN_Q4");
    k.mfma_waves = env_knob("QADC_MFMA_WAVES");
    k.ivf_wgs = env_knob("QADC_IVF_WGS");
    k.ivf_seed = env_knob("QADC_IVF_SEED");
    k.ivf_units = env_knob("QADC_IVF_UNITS");
    k.ivf_seed_parts = env_knob("QADC_IVF_SEED_PARTS");
    k.ivf_shared = env_knob("QADC_IVF_SHARED");
    k.ivf_shared_wgs = env_knob("QADC_IVF_SHARED_WGS");
    k.ivf_shared_min_pairs = env_knob("QADC_IVF_SHARED_MIN_PAIRS");
    k.ivf_seed_probes = env_knob("QADC_IVF_SEED_PROBES");
    k.ivf_wide_q = env_knob("QADC_IVF_WIDE_Q");
}

int build_luts(const float *, int, int, int, const float *, const float *, int, float *, hipStream_t);
int quantize_luts(int, const float *, int, int, int, const uint8_t *, int64_t, const float *, int, int,
                  int, uint8_t *, float *, float *, float *, hipStream_t);
int scan_topk_u8(int, const uint8_t *, int64_t, int, const uint8_t *, int, int, int, uint32_t *,
                 uint8_t *, void *, size_t, hipStream_t);
size_t scan_topk_u8_workspace(int, int64_t, int, int, int);
int search_u8(const float *, int, int, const float *, int, const uint8_t *, int64_t, int, int, int, int,
              uint32_t *, uint8_t *, uint8_t *, void *, size_t, hipStream_t);
size_t search_workspace(int64_t, int, int, int);
int scan_topk_f32(int, const uint8_t *, int64_t, int, const float *, int, int, uint32_t *, float *,
                  void *, size_t, hipStream_t);
size_t scan_topk_f32_workspace(int, int64_t, int, int, int);
int pq_encode(const float *, int, int, int, const float *, int64_t, uint8_t *, hipStream_t);
int rotate(const float *, int, const float *, int64_t, float *, hipStream_t);
size_t packed_bytes(int64_t, int, int);
int relayout(bool, const uint8_t *, int64_t, int, int, uint8_t *, hipStream_t);
int ivf_assign(const float *, int, int, const float *, int64_t, int32_t *, hipStream_t);
size_t ivf_group_workspace(int64_t, int);
int ivf_group(const int32_t *, int64_t, int, int64_t *, uint32_t *, void *, size_t, hipStream_t);
int ivf_encode(const float *, int, const float *, int, int, const float *, int64_t, const int32_t *,
               const uint32_t *, int64_t, uint8_t *, hipStream_t);
int multi_index_assign(const float *, int, int, const float *, int64_t, int32_t *, hipStream_t);
int multi_index_cells(const float *, int, int, float *, hipStream_t);
size_t multi_index_workspace(int, int, int);
int multi_index_probes(const float *, int, int, const float *, int, int, int32_t *, void *, size_t, hipStream_t);
size_t multi_index_group_workspace(int64_t, int);
int multi_index_group(const int32_t *, int64_t, int, int64_t, uint32_t *, int64_t *, uint32_t *, int64_t *, void *,
                      size_t, hipStream_t);
int multi_index_encode(const float *, int, const float *, int, int, const float *, int64_t, const int32_t *,
                       const uint32_t *, int64_t, uint8_t *, hipStream_t);
int multi_index_slots(const uint32_t *, int64_t, const int32_t *, int64_t, int32_t *, hipStream_t);
int workspace_init(void *, size_t, hipStream_t);
int pq_train(const float *, int64_t, int, int, int, const int64_t *, int, float *, void *, size_t,
             hipStream_t);
int ivf_search(const qadc_ivf_index *, const float *, int, int, int, int, int, int, const int32_t *,
               uint32_t *, uint8_t *, int32_t *, uint8_t *, void *, size_t, hipStream_t);
size_t ivf_workspace_bytes(const qadc_ivf_index *, int, int, int);

}  // namespace qadc

extern "C" {

int qadc_build_luts(const float *codebooks, int d, int m, int ksub, const float *queries,
                    const float *base, int nq, float *luts, void *stream)
{
    return qadc::build_luts(codebooks, d, m, ksub, queries, base, nq, luts, (hipStream_t)stream);
}

int qadc_quantize_luts(const float *luts, int nq, int ngroup, int m, const uint8_t *init_codes,
                       int64_t n_init, const float *qmax_in, int R, int nbins, int qmin_mode,
                       uint8_t *qluts, float *bias, float *delta, float *qmax_out, void *stream)
{
    return qadc::quantize_luts(16, luts, nq, ngroup, m, init_codes, n_init, qmax_in, R, nbins,
                               qmin_mode, qluts, bias, delta, qmax_out, (hipStream_t)stream);
}

int qadc_quantize_luts_8bit(const float *luts, int nq, int ngroup, int m, const uint8_t *init_codes,
                            int64_t n_init, const float *qmax_in, int R, int nbins, int qmin_mode,
                            uint8_t *qluts, float *bias, float *delta, float *qmax_out, void *stream)
{
    return qadc::quantize_luts(256, luts, nq, ngroup, m, init_codes, n_init, qmax_in, R, nbins,
                               qmin_mode, qluts, bias, delta, qmax_out, (hipStream_t)stream);
}

int qadc_quantize_luts_6bit(const float *luts, int nq, int ngroup, int m, const uint8_t *init_codes,
                            int64_t n_init, const float *qmax_in, int R, int nbins, int qmin_mode,
                            uint8_t *qluts, float *bias, float *delta, float *qmax_out, void *stream)
{
    return qadc::quantize_luts(64, luts, nq, ngroup, m, init_codes, n_init, qmax_in, R, nbins,
                               qmin_mode, qluts, bias, delta, qmax_out, (hipStream_t)stream);
}

int qadc_scan_topk(int variant, const void *codes, int64_t n, int m, const void *luts, int nq,
                   int R, int nbins, uint32_t *out_idx, void *out_dist, void *workspace,
                   size_t workspace_bytes, void *stream)
{
    qadc::knobs_refresh();
    if (!luts || !out_idx || !out_dist || (!codes && n > 0))
        return qadc::fail(QADC_EINVAL, "qadc_scan_topk: null pointer");
    if (nq == 0) return QADC_OK;
    switch (variant) {
    case QADC_U8_4BIT:
    case QADC_U8_8BIT:
    case QADC_U8_6BIT:
        return qadc::scan_topk_u8(variant, (const uint8_t *)codes, n, m, (const uint8_t *)luts, nq, R, nbins,
                                  out_idx, (uint8_t *)out_dist, workspace, workspace_bytes,
                                  (hipStream_t)stream);
    case QADC_F32_4BIT:
    case QADC_F32_8BIT:
        return qadc::scan_topk_f32(variant, (const uint8_t *)codes, n, m, (const float *)luts, nq, R,
                                   out_idx, (float *)out_dist, workspace, workspace_bytes,
                                   (hipStream_t)stream);
    default:
        return qadc::fail(QADC_EINVAL, "qadc_scan_topk: unknown variant %d", variant);
    }
}

int qadc_search(const float *codebooks, int d, int m, const float *queries, int nq,
                const uint8_t *codes, int64_t n, int R, int init, int nbins, int qmin_mode,
                uint32_t *out_idx, uint8_t *out_dist, uint8_t *qluts_out, void *workspace,
                size_t workspace_bytes, void *stream)
{
    qadc::knobs_refresh();
    return qadc::search_u8(codebooks, d, m, queries, nq, codes, n, R, init, nbins, qmin_mode, out_idx,
                           out_dist, qluts_out, workspace, workspace_bytes, (hipStream_t)stream);
}

int qadc_ivf_search(const qadc_ivf_index *ix, const float *queries, int nq, int nprobe, int R,
                    int init, int nbins, int qmin_mode, const int32_t *probes_in,
                    uint32_t *out_ids, uint8_t *out_dist, int32_t *dbg_probes, uint8_t *dbg_qluts,
                    void *workspace, size_t workspace_bytes, void *stream)
{
    qadc::knobs_refresh();
    return qadc::ivf_search(ix, queries, nq, nprobe, R, init, nbins, qmin_mode, probes_in, out_ids,
                            out_dist, dbg_probes, dbg_qluts, workspace, workspace_bytes,
                            (hipStream_t)stream);
}

size_t qadc_ivf_workspace_bytes(const qadc_ivf_index *ix, int nq, int nprobe, int R)
{
    qadc::knobs_refresh();
    return qadc::ivf_workspace_bytes(ix, nq, nprobe, R);
}

int qadc_pq_encode(const float *codebooks, int d, int m, int ksub, const float *x, int64_t n,
                   uint8_t *codes, void *stream)
{
    return qadc::pq_encode(codebooks, d, m, ksub, x, n, codes, (hipStream_t)stream);
}

int qadc_rotate(const float *rot, int d, const float *x, int64_t n, float *y, void *stream)
{
    return qadc::rotate(rot, d, x, n, y, (hipStream_t)stream);
}

size_t qadc_packed_bytes(int64_t n, int m, int layout) { return qadc::packed_bytes(n, m, layout); }

int qadc_pack_codes(const uint8_t *std_codes, int64_t n, int m, int layout, uint8_t *packed, void *stream)
{
    return qadc::relayout(true, std_codes, n, m, layout, packed, (hipStream_t)stream);
}

int qadc_unpack_codes(const uint8_t *packed, int64_t n, int m, int layout, uint8_t *std_codes, void *stream)
{
    return qadc::relayout(false, packed, n, m, layout, std_codes, (hipStream_t)stream);
}

int qadc_ivf_assign(const float *coarse, int K, int d, const float *x, int64_t n, int32_t *cells,
                    void *stream)
{
    return qadc::ivf_assign(coarse, K, d, x, n, cells, (hipStream_t)stream);
}

size_t qadc_ivf_group_workspace_bytes(int64_t n, int K) { return qadc::ivf_group_workspace(n, K); }

int qadc_ivf_group(const int32_t *cells, int64_t n, int K, int64_t *list_off, uint32_t *ids,
                   void *workspace, size_t workspace_bytes, void *stream)
{
    return qadc::ivf_group(cells, n, K, list_off, ids, workspace, workspace_bytes, (hipStream_t)stream);
}

int qadc_ivf_encode(const float *coarse, int K, const float *codebooks, int d, int m, const float *x,
                    int64_t n, const int32_t *cells, const uint32_t *ids, int64_t n_list,
                    uint8_t *codes, void *stream)
{
    return qadc::ivf_encode(coarse, K, codebooks, d, m, x, n, cells, ids, n_list, codes,
                            (hipStream_t)stream);
}

int qadc_multi_index_cells(const float *halves, int K, int d, float *coarse, void *stream)
{
    return qadc::multi_index_cells(halves, K, d, coarse, (hipStream_t)stream);
}

int qadc_multi_index_assign(const float *halves, int K, int d, const float *x, int64_t n, int32_t *cells,
                            void *stream)
{
    return qadc::multi_index_assign(halves, K, d, x, n, cells, (hipStream_t)stream);
}

size_t qadc_multi_index_workspace_bytes(int K, int nq, int nprobe)
{
    return qadc::multi_index_workspace(K, nq, nprobe);
}

int qadc_multi_index_probes(const float *halves, int K, int d, const float *queries, int nq, int nprobe,
                            int32_t *probes, void *workspace, size_t workspace_bytes, void *stream)
{
    return qadc::multi_index_probes(halves, K, d, queries, nq, nprobe, probes, workspace, workspace_bytes,
                                    (hipStream_t)stream);
}

size_t qadc_multi_index_group_workspace_bytes(int64_t n, int K) { return qadc::multi_index_group_workspace(n, K); }

int qadc_multi_index_group(const int32_t *cells, int64_t n, int K, int64_t max_lists, uint32_t *cell_ids,
                           int64_t *list_off, uint32_t *ids, int64_t *n_lists, void *workspace,
                           size_t workspace_bytes, void *stream)
{
    return qadc::multi_index_group(cells, n, K, max_lists, cell_ids, list_off, ids, n_lists, workspace,
                                   workspace_bytes, (hipStream_t)stream);
}

int qadc_multi_index_encode(const float *halves, int K, const float *codebooks, int d, int m, const float *x,
                            int64_t n, const int32_t *cells, const uint32_t *ids, int64_t n_list,
                            uint8_t *codes, void *stream)
{
    return qadc::multi_index_encode(halves, K, codebooks, d, m, x, n, cells, ids, n_list, codes,
                                    (hipStream_t)stream);
}

int qadc_multi_index_slots(const uint32_t *cell_ids, int64_t n_lists, const int32_t *cells, int64_t count,
                           int32_t *slots, void *stream)
{
    return qadc::multi_index_slots(cell_ids, n_lists, cells, count, slots, (hipStream_t)stream);
}

int qadc_profile_enable(int on) { return qadc::profile_enable(on); }

int qadc_profile_only(int which) { return qadc::profile_only(which); }

int qadc_profile_read(int which, double *total_ms, int64_t *launches)
{
    return qadc::profile_read(which, total_ms, launches);
}

int qadc_pq_train(const float *train, int64_t n, int d, int m, int ksub, const int64_t *init_rows,
                  int iters, float *codebooks, void *workspace, size_t workspace_bytes, void *stream)
{
    return qadc::pq_train(train, n, d, m, ksub, init_rows, iters, codebooks, workspace, workspace_bytes,
                          (hipStream_t)stream);
}

size_t qadc_workspace_bytes(int call, int64_t n, int m, int nq, int R)
{
    qadc::knobs_refresh();
    switch (call) {
    case QADC_WS_SCAN_TOPK: return qadc::scan_topk_u8_workspace(QADC_U8_4BIT, n, m, nq, R);
    case QADC_WS_SCAN_U8_8BIT: return qadc::scan_topk_u8_workspace(QADC_U8_8BIT, n, m, nq, R);
    case QADC_WS_SCAN_U8_6BIT: return qadc::scan_topk_u8_workspace(QADC_U8_6BIT, n, m, nq, R);
    case QADC_WS_SCAN_F32_4BIT: return qadc::scan_topk_f32_workspace(QADC_F32_4BIT, n, m, nq, R);
    case QADC_WS_SCAN_F32_8BIT: return qadc::scan_topk_f32_workspace(QADC_F32_8BIT, n, m, nq, R);
    case QADC_WS_SEARCH: return qadc::search_workspace(n, m, nq, R);
    default: return 0;
    }
}

int qadc_workspace_init(void *workspace, size_t bytes, void *stream)
{
    return qadc::workspace_init(workspace, bytes, (hipStream_t)stream);
}

const char *qadc_last_error(void) { return qadc::err_buf(); }

const char *qadc_version(void) { return "qadc-gfx950 0.1"; }

}  // extern "C"
