// C ABI of libsepattn: argument validation and dispatch.  Every entry point checks its arguments
// on the host before anything is enqueued, so a kernel never sees a shape its indexing does not
// cover.
#include "common.h"

#include <new>
#include <vector>

using namespace sepattn;

// A measurement handle: owned by the caller, attached to the calling thread for the launches it is to
// record (see sepattn.h).  The library itself keeps only the thread's pointer to the attached handle.
struct sepattn_profile {
    int kernel = -1;
    int used = 0;
    bool open = false;  // a start event was recorded and its stop is pending
    std::vector<hipEvent_t> start, stop;
};

namespace sepattn {
namespace {
thread_local sepattn_profile *t_attached = nullptr;
}  // namespace

void profile_mark(int kernel, hipStream_t st, bool stop) {
    sepattn_profile *h = t_attached;
    if (!h || kernel != h->kernel) return;
    if (!stop) {
        if (h->used >= (int)h->start.size()) return;
        h->open = hipEventRecord(h->start[h->used], st) == hipSuccess;
    } else if (h->open) {
        (void)hipEventRecord(h->stop[h->used], st);
        h->open = false;
        ++h->used;
    }
}
}  // namespace sepattn

namespace {

bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

int check_attn(const sepattn_params *p) {
    if (!p) return SEPATTN_ERR_NULL;
    if (p->B <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->L <= 0) return SEPATTN_ERR_SHAPE;
    if (p->Hq % p->Hkv != 0) return SEPATTN_ERR_SHAPE;
    if (p->d != 64 && p->d != 128) return SEPATTN_ERR_DTYPE;
    if (p->dtype != SEPATTN_BF16 && p->dtype != SEPATTN_FP32) return SEPATTN_ERR_DTYPE;
    if (p->a < 0 || p->n < 1) return SEPATTN_ERR_PARAM;
    if (!(p->scale == p->scale) || p->scale <= 0.f) return SEPATTN_ERR_PARAM;
    if (p->cap < 1) return SEPATTN_ERR_CAPACITY;
    // index arithmetic inside the kernels uses 32-bit positions and 64-bit offsets
    if ((long)p->B * p->Hq * p->L > (1L << 40)) return SEPATTN_ERR_SHAPE;
    if ((long)p->B * p->Hq > 65535L) return SEPATTN_ERR_SHAPE;  // second grid dimension
    // rows inside one head are addressed as (uniform base of the head) + 32-bit byte offset
    if ((long)p->L * p->d * 4 > 0xFFFFFFFFL) return SEPATTN_ERR_SHAPE;
    return SEPATTN_OK;
}

const HeadWin kNoHeadWin = {};  // an ordinary call: every head uses p.n

// head-wise windows: p.n becomes the largest window, hw.delta how much shorter each head's is
int head_windows(const sepattn_params *p, const int32_t *n_per_head, sepattn_params &q, HeadWin &hw) {
    if (!p) return SEPATTN_ERR_NULL;
    if (!n_per_head) return SEPATTN_ERR_NULL;
    if (p->Hq <= 0 || p->Hq > kMaxHeadwise || p->L <= 0) return SEPATTN_ERR_SHAPE;
    q = *p;
    q.n = 1;
    for (int h = 0; h < p->Hq; ++h) {
        if (n_per_head[h] < 1) return SEPATTN_ERR_PARAM;
        const int nh = n_per_head[h] < p->L ? n_per_head[h] : p->L;  // a window beyond L changes nothing
        q.n = nh > q.n ? nh : q.n;
    }
    hw = HeadWin{};
    for (int h = 0; h < p->Hq; ++h) hw.delta[h] = q.n - (n_per_head[h] < p->L ? n_per_head[h] : p->L);
    return SEPATTN_OK;
}

// a and n beyond L change nothing in the mask; clamping keeps position arithmetic in range
sepattn_params normalised(const sepattn_params *p) {
    sepattn_params q = *p;
    if (q.n > q.L) q.n = q.L;
    if (q.a > q.L) q.a = q.L;
    return q;
}

}  // namespace

namespace sepattn {
int check_kv_params(const sepkv_params *p) {
    if (!p) return SEPATTN_ERR_NULL;
    if (p->S <= 0 || p->Hq <= 0 || p->Hkv <= 0 || p->c <= 0) return SEPATTN_ERR_SHAPE;
    if (p->Hq % p->Hkv != 0) return SEPATTN_ERR_SHAPE;
    if (p->d != 64 && p->d != 128) return SEPATTN_ERR_DTYPE;
    if (p->dtype != SEPATTN_BF16 && p->dtype != SEPATTN_FP32) return SEPATTN_ERR_DTYPE;
    if (p->a < 0 || p->s < 0 || p->w < 1) return SEPATTN_ERR_PARAM;
    if ((long)p->a + p->s + p->w >= (long)p->c) return SEPATTN_ERR_PARAM;
    if (!(p->scale == p->scale) || p->scale <= 0.f) return SEPATTN_ERR_PARAM;
    if ((long)p->S * p->Hq > 65535L) return SEPATTN_ERR_SHAPE;  // second grid dimension
    // a slot's rows are addressed as (uniform base of the head) + 32-bit byte offset
    if ((long)p->c * p->d * 4 > 0xFFFFFFFFL) return SEPATTN_ERR_SHAPE;
    return SEPATTN_OK;
}
}  // namespace sepattn

namespace {
int check_kv(const sepkv_params *p) { return sepattn::check_kv_params(p); }
}  // namespace

namespace sepattn {
int compute_units() {
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev] = n;
    }
    return cached[dev];
}
}  // namespace sepattn

extern "C" {

const char *sepattn_status_string(int status) {
    switch (status) {
        case SEPATTN_OK: return "ok";
        case SEPATTN_ERR_NULL: return "a required pointer is NULL";
        case SEPATTN_ERR_SHAPE: return "invalid or inconsistent shape";
        case SEPATTN_ERR_PARAM: return "hyper-parameter out of range or misaligned buffer";
        case SEPATTN_ERR_DTYPE: return "unsupported dtype or head dimension";
        case SEPATTN_ERR_WORKSPACE: return "workspace missing or too small";
        case SEPATTN_ERR_CAPACITY: return "index list capacity too small";
        case SEPATTN_ERR_HIP: return "HIP runtime error at kernel launch";
        default: return "unknown status";
    }
}

const char *sepattn_kernel_name(int kernel) {
    static const char *names[SEPATTN_K_COUNT] = {"mark_kernel", "compact_count_kernel", "compact_write_kernel",
                                                 "fwd_bf16_kernel", "dq_kernel", "dkv_kernel",
                                                 "dkv_combine_kernel", "decode_split_kernel",
                                                 "decode_merge_kernel", "evict_sizes_kernel",
                                                 "evict_move_kernel", "cache_fill_kernel", "rope_table_kernel",
                                                 "cache_append_kernel", "mark_interval_kernel", "doc_bounds_kernel",
                                                 "mark_compact_kernel"};
    return (kernel >= 0 && kernel < SEPATTN_K_COUNT) ? names[kernel] : "unknown";
}

int sepattn_profile_create(int kernel, int max_records, sepattn_profile **out) {
    if (!out) return SEPATTN_ERR_NULL;
    *out = nullptr;
    if (kernel < 0 || kernel >= SEPATTN_K_COUNT || max_records < 1 || max_records > (1 << 20))
        return SEPATTN_ERR_PARAM;
    sepattn_profile *h = new (std::nothrow) sepattn_profile;
    if (!h) return SEPATTN_ERR_HIP;
    h->kernel = kernel;
    h->start.assign(max_records, nullptr);
    h->stop.assign(max_records, nullptr);
    for (int i = 0; i < max_records; ++i) {
        if (hipEventCreate(&h->start[i]) != hipSuccess || hipEventCreate(&h->stop[i]) != hipSuccess) {
            (void)hipGetLastError();
            sepattn_profile_destroy(h);
            return SEPATTN_ERR_HIP;
        }
    }
    *out = h;
    return SEPATTN_OK;
}

void sepattn_profile_destroy(sepattn_profile *h) {
    if (!h) return;
    if (t_attached == h) t_attached = nullptr;
    for (size_t i = 0; i < h->start.size(); ++i) {
        if (h->start[i]) (void)hipEventDestroy(h->start[i]);
        if (h->stop[i]) (void)hipEventDestroy(h->stop[i]);
    }
    delete h;
}

int sepattn_profile_attach(sepattn_profile *h) {
    if (!h) return SEPATTN_ERR_NULL;
    if (t_attached) return SEPATTN_ERR_PARAM;  // one handle per thread at a time
    t_attached = h;
    return SEPATTN_OK;
}

int sepattn_profile_detach(sepattn_profile *h) {
    if (!h) return SEPATTN_ERR_NULL;
    if (t_attached != h) return SEPATTN_ERR_PARAM;
    t_attached = nullptr;
    return SEPATTN_OK;
}

int sepattn_profile_read(sepattn_profile *h, float *ms, int max_records, int *n_records) {
    if (!h || !ms || !n_records) return SEPATTN_ERR_NULL;
    int rc = SEPATTN_OK;
    const int n = h->used < max_records ? h->used : max_records;
    for (int i = 0; i < n; ++i) {
        if (hipEventSynchronize(h->stop[i]) != hipSuccess ||
            hipEventElapsedTime(&ms[i], h->start[i], h->stop[i]) != hipSuccess)
            rc = SEPATTN_ERR_HIP;
    }
    *n_records = n;
    return rc;
}

int sepattn_mark_separators(const int32_t *token_ids, int B, int L, const int32_t *sep_ids,
                            int n_sep, uint8_t *is_sep, void *stream) {
    if (!token_ids || !sep_ids || !is_sep) return SEPATTN_ERR_NULL;
    if (B <= 0 || L <= 0) return SEPATTN_ERR_SHAPE;
    if (n_sep < 1 || n_sep > SEPATTN_MAX_SEP_IDS) return SEPATTN_ERR_PARAM;
    if (!aligned(token_ids, 16) || !aligned(is_sep, 4)) return SEPATTN_ERR_PARAM;
    SepIdSet set;
    set.n = n_sep;
    for (int k = 0; k < SEPATTN_MAX_SEP_IDS; ++k) set.ids[k] = k < n_sep ? sep_ids[k] : sep_ids[0];
    discard_stale_hip_error();
    return launch_mark(token_ids, (long)B * L, set, is_sep, static_cast<hipStream_t>(stream));
}

int sepattn_mark_interval(int B, int L, int delta, int phase, uint8_t *is_sep, void *stream) {
    if (!is_sep) return SEPATTN_ERR_NULL;
    if (B <= 0 || L <= 0) return SEPATTN_ERR_SHAPE;
    if (delta < 1 || phase < 0 || phase >= delta) return SEPATTN_ERR_PARAM;
    if (!aligned(is_sep, 4)) return SEPATTN_ERR_PARAM;
    discard_stale_hip_error();
    return launch_mark_interval(B, L, delta, phase, is_sep, static_cast<hipStream_t>(stream));
}

size_t sepattn_compact_workspace_bytes(int B, int L) {
    if (B <= 0 || L <= 0) return 0;
    size_t n_chunks = ((size_t)L + kCompactChunk - 1) / kCompactChunk;
    return align_up((size_t)B * n_chunks * sizeof(int32_t), 256);
}

int sepattn_compact_indices(const uint8_t *is_sep, int B, int L, int32_t *sep_idx, int cap,
                            int32_t *sep_count, int32_t *sep_prefix, void *workspace,
                            size_t workspace_bytes, void *stream) {
    if (!is_sep || !sep_idx || !sep_count) return SEPATTN_ERR_NULL;
    if (B <= 0 || L <= 0 || B > 65535) return SEPATTN_ERR_SHAPE;
    if (cap < 1) return SEPATTN_ERR_CAPACITY;
    if (!workspace || workspace_bytes < sepattn_compact_workspace_bytes(B, L) || !aligned(workspace, 4))
        return SEPATTN_ERR_WORKSPACE;
    discard_stale_hip_error();
    return launch_compact(is_sep, B, L, sep_idx, cap, sep_count, sep_prefix,
                          static_cast<int32_t *>(workspace), static_cast<hipStream_t>(stream));
}

int sepattn_mark_compact(const int32_t *token_ids, int B, int L, const int32_t *sep_ids, int n_sep,
                         uint8_t *is_sep, int32_t *sep_idx, int cap, int32_t *sep_count,
                         int32_t *sep_prefix, void *workspace, size_t workspace_bytes, void *stream) {
    if (!token_ids || !sep_ids || !is_sep || !sep_idx || !sep_count) return SEPATTN_ERR_NULL;
    if (B <= 0 || L <= 0 || B > 65535) return SEPATTN_ERR_SHAPE;
    if (n_sep < 1 || n_sep > SEPATTN_MAX_SEP_IDS) return SEPATTN_ERR_PARAM;
    if (cap < 1) return SEPATTN_ERR_CAPACITY;
    if (!aligned(token_ids, 16) || !aligned(is_sep, 4)) return SEPATTN_ERR_PARAM;
    if (!workspace || workspace_bytes < sepattn_compact_workspace_bytes(B, L) || !aligned(workspace, 4))
        return SEPATTN_ERR_WORKSPACE;
    SepIdSet set;
    set.n = n_sep;
    for (int k = 0; k < SEPATTN_MAX_SEP_IDS; ++k) set.ids[k] = k < n_sep ? sep_ids[k] : sep_ids[0];
    discard_stale_hip_error();
    return launch_mark_compact(token_ids, B, L, set, is_sep, sep_idx, cap, sep_count, sep_prefix,
                               static_cast<int32_t *>(workspace), static_cast<hipStream_t>(stream));
}

size_t sepattn_forward_workspace_bytes(const sepattn_params *p) {
    if (check_attn(p) != SEPATTN_OK) return 0;
    return p->dtype == SEPATTN_BF16 ? forward_bf16_workspace(normalised(p)) : 0;
}

int sepattn_forward(const sepattn_params *p, const void *Q, const void *K, const void *V,
                    const int32_t *sep_idx, const int32_t *sep_count, const int32_t *sep_prefix,
                    void *O, float *LSE, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_attn(p);
    if (rc != SEPATTN_OK) return rc;
    if (!Q || !K || !V || !sep_idx || !sep_count || !sep_prefix || !O || !LSE) return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16)) return SEPATTN_ERR_PARAM;
    size_t need = sepattn_forward_workspace_bytes(p);
    if (need > 0 && (!ws || ws_bytes < need || !aligned(ws, 256))) return SEPATTN_ERR_WORKSPACE;
    sepattn_params q = normalised(p);
    hipStream_t st = static_cast<hipStream_t>(stream);
    discard_stale_hip_error();
    if (q.dtype == SEPATTN_FP32)
        return launch_forward_fp32(q, kNoHeadWin, (const float *)Q, (const float *)K, (const float *)V, sep_idx,
                                   sep_prefix, nullptr, (float *)O, LSE, st);
    return launch_forward_bf16(q, kNoHeadWin, Q, K, V, sep_idx, sep_prefix, nullptr, nullptr, O, LSE, ws, st);
}

int sepattn_doc_bounds(const int32_t *cu_seqlens, int n_docs, int L, int a, int32_t *doc_start, int32_t *doc_end,
                       uint8_t *is_sep, void *stream) {
    if (!cu_seqlens || !doc_start || !doc_end) return SEPATTN_ERR_NULL;
    if (n_docs < 1 || L < 1 || n_docs > L) return SEPATTN_ERR_SHAPE;
    if (a < 0) return SEPATTN_ERR_PARAM;
    discard_stale_hip_error();
    return launch_doc_bounds(cu_seqlens, n_docs, L, a, doc_start, doc_end, is_sep, static_cast<hipStream_t>(stream));
}

int sepattn_forward_packed(const sepattn_params *p, const int32_t *doc_start, const int32_t *doc_end,
                           const void *Q, const void *K, const void *V, const int32_t *sep_idx,
                           const int32_t *sep_count, const int32_t *sep_prefix, void *O, float *LSE, void *ws,
                           size_t ws_bytes, void *stream) {
    int rc = check_attn(p);
    if (rc != SEPATTN_OK) return rc;
    if (p->a != 0) return SEPATTN_ERR_PARAM;  // the documents' initial tokens are in the marker bitmap
    if (!doc_start || !doc_end || !Q || !K || !V || !sep_idx || !sep_count || !sep_prefix || !O || !LSE)
        return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16)) return SEPATTN_ERR_PARAM;
    size_t need = sepattn_forward_workspace_bytes(p);
    if (need > 0 && (!ws || ws_bytes < need || !aligned(ws, 256))) return SEPATTN_ERR_WORKSPACE;
    discard_stale_hip_error();
    if (p->dtype == SEPATTN_FP32)
        return launch_forward_fp32(normalised(p), kNoHeadWin, (const float *)Q, (const float *)K, (const float *)V, sep_idx,
                                   sep_prefix, doc_start, (float *)O, LSE, static_cast<hipStream_t>(stream));
    return launch_forward_bf16(normalised(p), kNoHeadWin, Q, K, V, sep_idx, sep_prefix, doc_start, doc_end, O, LSE, ws,
                               static_cast<hipStream_t>(stream));
}

size_t sepattn_backward_workspace_bytes(const sepattn_params *p) {
    if (check_attn(p) != SEPATTN_OK) return 0;
    if (p->dtype == SEPATTN_FP32) return align_up((size_t)p->B * p->Hq * p->L * sizeof(float), 256);
    return backward_bf16_workspace(normalised(p));
}

int sepattn_backward(const sepattn_params *p, const void *Q, const void *K, const void *V,
                     const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                     const int32_t *sep_count, const int32_t *sep_prefix, void *dQ, void *dK,
                     void *dV, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_attn(p);
    if (rc != SEPATTN_OK) return rc;
    if (!Q || !K || !V || !O || !LSE || !dO || !sep_idx || !sep_count || !sep_prefix || !dQ || !dK || !dV)
        return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(dO, 16) ||
        !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16))
        return SEPATTN_ERR_PARAM;
    size_t need = sepattn_backward_workspace_bytes(p);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return SEPATTN_ERR_WORKSPACE;
    sepattn_params q = normalised(p);
    hipStream_t st = static_cast<hipStream_t>(stream);
    discard_stale_hip_error();
    if (q.dtype == SEPATTN_FP32)
        return launch_backward_fp32(q, kNoHeadWin, (const float *)Q, (const float *)K, (const float *)V,
                                    (const float *)O, LSE, (const float *)dO, sep_idx, sep_prefix, nullptr, nullptr,
                                    (float *)dQ, (float *)dK, (float *)dV, (float *)ws, st);
    return launch_backward_bf16(q, kNoHeadWin, Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix, nullptr, nullptr, dQ, dK, dV,
                                ws, st);
}

int sepattn_forward_headwise(const sepattn_params *p, const int32_t *n_per_head, const void *Q, const void *K,
                             const void *V, const int32_t *sep_idx, const int32_t *sep_count,
                             const int32_t *sep_prefix, void *O, float *LSE, void *ws, size_t ws_bytes, void *stream) {
    sepattn_params pm;
    HeadWin hw;
    int rc = head_windows(p, n_per_head, pm, hw);
    if (rc != SEPATTN_OK) return rc;
    rc = check_attn(&pm);
    if (rc != SEPATTN_OK) return rc;
    if (!Q || !K || !V || !sep_idx || !sep_count || !sep_prefix || !O || !LSE) return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16)) return SEPATTN_ERR_PARAM;
    size_t need = sepattn_forward_workspace_bytes(&pm);
    if (need > 0 && (!ws || ws_bytes < need || !aligned(ws, 256))) return SEPATTN_ERR_WORKSPACE;
    sepattn_params q = normalised(&pm);
    hipStream_t st = static_cast<hipStream_t>(stream);
    discard_stale_hip_error();
    if (q.dtype == SEPATTN_FP32)
        return launch_forward_fp32(q, hw, (const float *)Q, (const float *)K, (const float *)V, sep_idx, sep_prefix,
                                   nullptr, (float *)O, LSE, st);
    return launch_forward_bf16(q, hw, Q, K, V, sep_idx, sep_prefix, nullptr, nullptr, O, LSE, ws, st);
}

size_t sepattn_backward_headwise_workspace_bytes(const sepattn_params *p, const int32_t *n_per_head) {
    sepattn_params pm;
    HeadWin hw;
    if (head_windows(p, n_per_head, pm, hw) != SEPATTN_OK) return 0;
    return sepattn_backward_workspace_bytes(&pm);
}

int sepattn_backward_headwise(const sepattn_params *p, const int32_t *n_per_head, const void *Q, const void *K,
                              const void *V, const void *O, const float *LSE, const void *dO, const int32_t *sep_idx,
                              const int32_t *sep_count, const int32_t *sep_prefix, void *dQ, void *dK, void *dV,
                              void *ws, size_t ws_bytes, void *stream) {
    sepattn_params pm;
    HeadWin hw;
    int rc = head_windows(p, n_per_head, pm, hw);
    if (rc != SEPATTN_OK) return rc;
    rc = check_attn(&pm);
    if (rc != SEPATTN_OK) return rc;
    if (!Q || !K || !V || !O || !LSE || !dO || !sep_idx || !sep_count || !sep_prefix || !dQ || !dK || !dV)
        return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(dO, 16) ||
        !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16))
        return SEPATTN_ERR_PARAM;
    size_t need = sepattn_backward_workspace_bytes(&pm);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return SEPATTN_ERR_WORKSPACE;
    sepattn_params q = normalised(&pm);
    hipStream_t st = static_cast<hipStream_t>(stream);
    discard_stale_hip_error();
    if (q.dtype == SEPATTN_FP32)
        return launch_backward_fp32(q, hw, (const float *)Q, (const float *)K, (const float *)V, (const float *)O, LSE,
                                    (const float *)dO, sep_idx, sep_prefix, nullptr, nullptr, (float *)dQ, (float *)dK,
                                    (float *)dV, (float *)ws, st);
    return launch_backward_bf16(q, hw, Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix, nullptr, nullptr, dQ, dK, dV,
                                ws, st);
}

int sepattn_backward_packed(const sepattn_params *p, const int32_t *doc_start, const int32_t *doc_end,
                            const void *Q, const void *K, const void *V, const void *O, const float *LSE,
                            const void *dO, const int32_t *sep_idx, const int32_t *sep_count,
                            const int32_t *sep_prefix, void *dQ, void *dK, void *dV, void *ws, size_t ws_bytes,
                            void *stream) {
    int rc = check_attn(p);
    if (rc != SEPATTN_OK) return rc;
    if (p->a != 0) return SEPATTN_ERR_PARAM;  // the documents' initial tokens are in the marker bitmap
    if (!doc_start || !doc_end || !Q || !K || !V || !O || !LSE || !dO || !sep_idx || !sep_count || !sep_prefix ||
        !dQ || !dK || !dV)
        return SEPATTN_ERR_NULL;
    if (!aligned(Q, 16) || !aligned(K, 16) || !aligned(V, 16) || !aligned(O, 16) || !aligned(dO, 16) ||
        !aligned(dQ, 16) || !aligned(dK, 16) || !aligned(dV, 16))
        return SEPATTN_ERR_PARAM;
    size_t need = sepattn_backward_workspace_bytes(p);
    if (!ws || ws_bytes < need || !aligned(ws, 256)) return SEPATTN_ERR_WORKSPACE;
    discard_stale_hip_error();
    if (p->dtype == SEPATTN_FP32)
        return launch_backward_fp32(normalised(p), kNoHeadWin, (const float *)Q, (const float *)K, (const float *)V,
                                    (const float *)O, LSE, (const float *)dO, sep_idx, sep_prefix, doc_start, doc_end,
                                    (float *)dQ, (float *)dK, (float *)dV, (float *)ws,
                                    static_cast<hipStream_t>(stream));
    return launch_backward_bf16(normalised(p), kNoHeadWin, Q, K, V, O, LSE, dO, sep_idx, sep_count, sep_prefix, doc_start,
                                doc_end, dQ, dK, dV, ws, static_cast<hipStream_t>(stream));
}

size_t sepattn_decode_workspace_bytes(const sepkv_params *p) {
    if (check_kv(p) != SEPATTN_OK) return 0;
    return decode_workspace(*p);
}

int sepattn_decode(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                   const int32_t *sizes, void *out, float *lse, void *ws, size_t ws_bytes,
                   void *stream) {
    int rc = check_kv(p);
    if (rc != SEPATTN_OK) return rc;
    if (!q || !Kc || !Vc || !sizes || !out) return SEPATTN_ERR_NULL;
    if (!aligned(q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(out, 16)) return SEPATTN_ERR_PARAM;
    if (!ws || ws_bytes < decode_workspace(*p) || !aligned(ws, 256)) return SEPATTN_ERR_WORKSPACE;
    discard_stale_hip_error();
    return launch_decode(*p, q, Kc, Vc, sizes, nullptr, 0, out, lse, ws, static_cast<hipStream_t>(stream));
}

int sepkv_rope_table(int n_pos, int d, double base, float *table, void *stream) {
    if (!table) return SEPATTN_ERR_NULL;
    if (n_pos < 1 || n_pos > (1 << 28)) return SEPATTN_ERR_SHAPE;
    if (d != 64 && d != 128) return SEPATTN_ERR_DTYPE;
    if (!(base > 1.0) || base > 1e30) return SEPATTN_ERR_PARAM;
    if (!aligned(table, 16)) return SEPATTN_ERR_PARAM;
    discard_stale_hip_error();
    return launch_rope_table(n_pos, d, base, table, static_cast<hipStream_t>(stream));
}

int sepattn_decode_rope(const sepkv_params *p, const void *q, const void *Kc, const void *Vc,
                        const int32_t *sizes, const float *rope_table, int n_pos, void *out, float *lse,
                        void *ws, size_t ws_bytes, void *stream) {
    int rc = check_kv(p);
    if (rc != SEPATTN_OK) return rc;
    if (!q || !Kc || !Vc || !sizes || !out || !rope_table) return SEPATTN_ERR_NULL;
    if (n_pos < p->c) return SEPATTN_ERR_SHAPE;  // a row for every position a full cache can hold
    if (!aligned(q, 16) || !aligned(Kc, 16) || !aligned(Vc, 16) || !aligned(out, 16) || !aligned(rope_table, 16))
        return SEPATTN_ERR_PARAM;
    if (!ws || ws_bytes < decode_workspace(*p) || !aligned(ws, 256)) return SEPATTN_ERR_WORKSPACE;
    discard_stale_hip_error();
    return launch_decode(*p, q, Kc, Vc, sizes, rope_table, n_pos, out, lse, ws, static_cast<hipStream_t>(stream));
}

int sepkv_append(const sepkv_params *p, const void *k_new, const void *v_new, const uint8_t *is_sep_new,
                 void *Kc, void *Vc, uint8_t *win_is_sep, int32_t *sizes, void *stream) {
    int rc = check_kv(p);
    if (rc != SEPATTN_OK) return rc;
    if (!k_new || !v_new || !is_sep_new || !Kc || !Vc || !win_is_sep || !sizes) return SEPATTN_ERR_NULL;
    if (!aligned(k_new, 16) || !aligned(v_new, 16) || !aligned(Kc, 16) || !aligned(Vc, 16)) return SEPATTN_ERR_PARAM;
    discard_stale_hip_error();
    return launch_cache_append(*p, k_new, v_new, is_sep_new, Kc, Vc, win_is_sep, sizes,
                               static_cast<hipStream_t>(stream));
}

size_t sepkv_evict_workspace_bytes(const sepkv_params *p) {
    if (check_kv(p) != SEPATTN_OK) return 0;
    return evict_workspace(*p);
}

int sepkv_evict_window(const sepkv_params *p, void *Kc, void *Vc, const uint8_t *win_is_sep,
                       int32_t *sizes, void *ws, size_t ws_bytes, void *stream) {
    int rc = check_kv(p);
    if (rc != SEPATTN_OK) return rc;
    if (!Kc || !Vc || !win_is_sep || !sizes) return SEPATTN_ERR_NULL;
    if (!aligned(Kc, 16) || !aligned(Vc, 16)) return SEPATTN_ERR_PARAM;
    (void)ws_bytes;  // the step needs no scratch memory; ws may be NULL
    discard_stale_hip_error();
    return launch_evict(*p, Kc, Vc, win_is_sep, sizes, ws, static_cast<hipStream_t>(stream));
}

int sepkv_fill_from_prefill(const sepkv_params *p, int L, int nw, const void *K, const void *V,
                            const uint8_t *is_sep, const int32_t *sep_idx, int cap, const int32_t *sep_prefix,
                            void *Kc, void *Vc, uint8_t *win_is_sep, int32_t *sizes, void *stream) {
    int rc = check_kv(p);
    if (rc != SEPATTN_OK) return rc;
    if (!K || !V || !is_sep || !sep_idx || !sep_prefix || !Kc || !Vc || !win_is_sep || !sizes) return SEPATTN_ERR_NULL;
    if (L <= 0 || (long)p->S * p->Hkv * L > (1L << 40)) return SEPATTN_ERR_SHAPE;
    if (cap < 1) return SEPATTN_ERR_CAPACITY;
    const int n_init = p->a < L ? p->a : L;
    if (nw < 0 || nw > p->c - p->a - p->s || nw > L - n_init) return SEPATTN_ERR_PARAM;
    if (!aligned(K, 16) || !aligned(V, 16) || !aligned(Kc, 16) || !aligned(Vc, 16)) return SEPATTN_ERR_PARAM;
    discard_stale_hip_error();
    return launch_cache_fill(*p, L, nw, K, V, is_sep, sep_idx, cap, sep_prefix, Kc, Vc, win_is_sep, sizes,
                             static_cast<hipStream_t>(stream));
}

}  // extern "C"
