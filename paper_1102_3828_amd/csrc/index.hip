// Index lifetime, codebooks, offline stage (train / add / finalize) and import / export.
#include "ivfr_internal.h"

#include <algorithm>
#include <numeric>
#include <string.h>

// launchers defined in encode.hip
int ivfr_launch_list_ranks(const int32_t* list, int64_t n, int c, unsigned long long* list_fill, uint32_t* cnt,
                           int T, uint32_t* rank, hipStream_t st);
int ivfr_launch_scatter(const StagedChunk& ch, int m, int mr, const uint32_t* list_start, uint8_t* codes,
                        uint8_t* rec, int rec_stride, hipStream_t st);
int ivfr_launch_pack_records(const ivfr_index* ix, uint64_t slot0, int64_t n, const int32_t* ids_st,
                             const uint8_t* rcodes_st, hipStream_t st);
int ivfr_launch_unpack_records(const ivfr_index* ix, uint64_t slot0, int64_t n, int32_t* ids_st, uint8_t* rcodes_st,
                               hipStream_t st);
int ivfr_launch_iota(int32_t* ids, int64_t n, int64_t base, hipStream_t st);
int ivfr_launch_km_accum_rows(const float* X, int64_t n, int d, const int32_t* assign, unsigned long long* sums,
                              unsigned long long* counts, hipStream_t st);
int ivfr_launch_km_accum_pq(const float* R, int64_t n, int d, int parts, const uint8_t* codes,
                            unsigned long long* sums, unsigned long long* counts, hipStream_t st);
int ivfr_launch_km_update(float* cent, int64_t total, int width, const unsigned long long* sums,
                          const unsigned long long* counts, hipStream_t st);
int ivfr_launch_gather_rows(const float* X, int d, int col0, int width, const int64_t* idx, int count, float* out,
                            hipStream_t st);

static thread_local char g_err[512] = "";

void ivfr_set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

extern "C" const char* ivfr_last_error(void) { return g_err; }

#define ADD_SUB 1048576   // vectors encoded per internal batch

static int use_device(const ivfr_index* ix) {
    IVFR_HIP(hipSetDevice(ix->p.device));
    return IVFR_OK;
}

template <class T>
static int dev_alloc(T** p, size_t count) {
    *p = nullptr;
    if (count == 0) count = 1;
    hipError_t e = hipMalloc(reinterpret_cast<void**>(p), count * sizeof(T));
    if (e != hipSuccess) {
        (void)hipGetLastError();
        *p = nullptr;
        ivfr_set_error("device allocation of %zu bytes failed: %s", count * sizeof(T), hipGetErrorString(e));
        return IVFR_ERR_OOM;
    }
    return IVFR_OK;
}

template <class T>
static void dev_free(T*& p) {
    if (p) (void)hipFree(p);
    p = nullptr;
}

extern "C" int ivfr_create(const ivfr_params* params, ivfr_index** out) {
    IVFR_REQUIRE(params && out, "ivfr_create: null argument");
    const ivfr_params& p = *params;
    IVFR_REQUIRE(p.d > 0 && p.d % 8 == 0, "d = %d must be a positive multiple of 8", p.d);
    IVFR_REQUIRE(p.c >= 1, "c = %d must be >= 1", p.c);
    IVFR_REQUIRE(p.m == 4 || p.m == 8 || p.m == 16 || p.m == 32 || p.m == 64, "m = %d must be 4, 8, 16, 32 or 64", p.m);
    IVFR_REQUIRE(p.d % p.m == 0, "d = %d is not a multiple of m = %d", p.d, p.m);
    IVFR_REQUIRE(p.d / p.m <= 32, "d/m = %d exceeds 32", p.d / p.m);
    IVFR_REQUIRE(p.m_refine >= 0 && p.m_refine % 4 == 0, "m_refine = %d must be a non-negative multiple of 4", p.m_refine);
    if (p.m_refine) {
        IVFR_REQUIRE(p.d % p.m_refine == 0, "d = %d is not a multiple of m_refine = %d", p.d, p.m_refine);
        IVFR_REQUIRE(p.d / p.m_refine <= 32, "d/m_refine = %d exceeds 32", p.d / p.m_refine);
        int ds = p.d / p.m_refine;
        IVFR_REQUIRE((ds & (ds - 1)) == 0, "d/m_refine = %d must be a power of two", ds);
    }
    {
        int ds = p.d / p.m;
        IVFR_REQUIRE((ds & (ds - 1)) == 0, "d/m = %d must be a power of two", ds);
    }
    int ndev = 0;
    IVFR_HIP(hipGetDeviceCount(&ndev));
    IVFR_REQUIRE(p.device >= 0 && p.device < ndev, "device %d out of range (%d devices)", p.device, ndev);
    ivfr_index* ix = new (std::nothrow) ivfr_index();
    if (!ix) { ivfr_set_error("host allocation failed"); return IVFR_ERR_OOM; }
    ix->p = p;
    ix->dsub = p.d / p.m;
    ix->dsub_r = p.m_refine ? p.d / p.m_refine : 0;
    int r = use_device(ix);
    if (r == IVFR_OK) {
        hipDeviceProp_t prop;
        if (hipGetDeviceProperties(&prop, p.device) == hipSuccess) ix->n_cu = prop.multiProcessorCount;
        // function attributes are per device: set with this index's device current, every time
        r = ivfr_select_init();
        if (r == IVFR_OK) r = ivfr_scan_init();
        if (r == IVFR_OK) r = ivfr_rerank_init();
    }
    if (r == IVFR_OK) {
        hipError_t e = hipHostMalloc(reinterpret_cast<void**>(&ix->h_slots), IVFR_STATUS_SLOTS * sizeof(DevStatus),
                                     hipHostMallocDefault);
        if (e == hipSuccess) e = hipHostMalloc(reinterpret_cast<void**>(&ix->h_redo), (16 + IVFR_REDO_CHUNK) * sizeof(uint32_t), hipHostMallocDefault);
        if (e != hipSuccess) { ivfr_set_error("pinned host allocation failed"); r = IVFR_ERR_OOM; }
        else memset(ix->h_slots, 0, IVFR_STATUS_SLOTS * sizeof(DevStatus));
    }
    if (r == IVFR_OK) r = ivfr_static_scratch_address(p.device, &ix->static_ws);
    for (int i = 0; i < 4 && r == IVFR_OK; ++i) {
        if (hipStreamCreateWithFlags(&ix->side[i], hipStreamNonBlocking) != hipSuccess) {
            ivfr_set_error("stream creation failed");
            r = IVFR_ERR_HIP;
        }
    }
    for (int sl = 0; sl < IVFR_STATUS_SLOTS && r == IVFR_OK; ++sl) {
        bool ok = hipEventCreateWithFlags(&ix->ev_fork[sl], hipEventDisableTiming) == hipSuccess;
        for (int i = 0; i < 4 && ok; ++i)
            ok = hipEventCreateWithFlags(&ix->ev_join[sl][i], hipEventDisableTiming) == hipSuccess;
        for (int i = 0; i < 2 && ok; ++i)
            ok = hipEventCreateWithFlags(&ix->ev_group[sl][i], hipEventDisableTiming) == hipSuccess;
        if (!ok) { ivfr_set_error("event creation failed"); r = IVFR_ERR_HIP; }
    }
    if (r != IVFR_OK) { ivfr_destroy(ix); return r; }
    *out = ix;
    return IVFR_OK;
}

static void free_staged(ivfr_index* ix) {
    for (auto& ch : ix->staged) {
        dev_free(ch.list); dev_free(ch.rank); dev_free(ch.ids); dev_free(ch.codes); dev_free(ch.rcodes);
    }
    ix->staged.clear();
}

extern "C" int ivfr_destroy(ivfr_index* ix) {
    if (!ix) return IVFR_OK;
    (void)hipSetDevice(ix->p.device);
    (void)hipDeviceSynchronize();
    free_staged(ix);
    dev_free(ix->coarse); dev_free(ix->coarse_norm); dev_free(ix->pq); dev_free(ix->pq_norm); dev_free(ix->pq_maxnorm); dev_free(ix->rq);
    dev_free(ix->list_term);
    dev_free(ix->list_fill); dev_free(ix->list_start); dev_free(ix->list_len);
    dev_free(ix->codes); dev_free(ix->rec);
    ix->search_ws.release(); ix->cand_ws.release(); ix->encode_ws.release(); ix->dense_ws.release();
    if (ix->h_slots) (void)hipHostFree(ix->h_slots);
    if (ix->h_redo) (void)hipHostFree(ix->h_redo);
    for (int i = 0; i < 4; ++i)
        if (ix->side[i]) (void)hipStreamDestroy(ix->side[i]);
    for (int sl = 0; sl < IVFR_STATUS_SLOTS; ++sl) {
        if (ix->ev_fork[sl]) (void)hipEventDestroy(ix->ev_fork[sl]);
        for (int i = 0; i < 4; ++i)
            if (ix->ev_join[sl][i]) (void)hipEventDestroy(ix->ev_join[sl][i]);
        for (int i = 0; i < 2; ++i)
            if (ix->ev_group[sl][i]) (void)hipEventDestroy(ix->ev_group[sl][i]);
    }
    for (hipEvent_t e : ix->prof_events) (void)hipEventDestroy(e);
    ix->prof_events.clear();
    delete ix;
    return IVFR_OK;
}

static int alloc_books(ivfr_index* ix) {
    const ivfr_params& p = ix->p;
    if (ix->coarse) return IVFR_OK;
    IVFR_TRY(dev_alloc(&ix->coarse, (size_t)p.c * p.d));
    IVFR_TRY(dev_alloc(&ix->coarse_norm, (size_t)p.c));
    IVFR_TRY(dev_alloc(&ix->pq, (size_t)p.m * IVFR_KS * ix->dsub));
    IVFR_TRY(dev_alloc(&ix->pq_norm, (size_t)p.m * IVFR_KS));
    IVFR_TRY(dev_alloc(&ix->pq_maxnorm, (size_t)p.m));
    if (p.m_refine) IVFR_TRY(dev_alloc(&ix->rq, (size_t)p.m_refine * IVFR_KS * ix->dsub_r));
    return IVFR_OK;
}

static int refresh_norms(ivfr_index* ix, hipStream_t st) {
    IVFR_TRY(ivfr_launch_row_norms(ix->coarse, ix->p.c, ix->p.d, ix->coarse_norm, st));
    IVFR_TRY(ivfr_launch_row_norms(ix->pq, (int64_t)ix->p.m * IVFR_KS, ix->dsub, ix->pq_norm, st));
    IVFR_TRY(ivfr_launch_group_max_norm(ix->pq_norm, ix->p.m, IVFR_KS, ix->pq_maxnorm, st));
    return IVFR_OK;
}

extern "C" int ivfr_set_codebooks(ivfr_index* ix, const float* coarse, const float* pq, const float* rq) {
    IVFR_REQUIRE(ix && coarse && pq, "ivfr_set_codebooks: null argument");
    IVFR_REQUIRE(ix->p.m_refine == 0 || rq, "ivfr_set_codebooks: rq is required when m_refine > 0");
    if (ix->n_added > 0 || ix->finalized) { ivfr_set_error("codebooks cannot change after vectors were added"); return IVFR_ERR_STATE; }
    IVFR_TRY(use_device(ix));
    IVFR_TRY(alloc_books(ix));
    const ivfr_params& p = ix->p;
    IVFR_HIP(hipMemcpy(ix->coarse, coarse, (size_t)p.c * p.d * sizeof(float), hipMemcpyHostToDevice));
    IVFR_HIP(hipMemcpy(ix->pq, pq, (size_t)p.m * IVFR_KS * ix->dsub * sizeof(float), hipMemcpyHostToDevice));
    if (p.m_refine)
        IVFR_HIP(hipMemcpy(ix->rq, rq, (size_t)p.m_refine * IVFR_KS * ix->dsub_r * sizeof(float), hipMemcpyHostToDevice));
    IVFR_TRY(refresh_norms(ix, nullptr));
    IVFR_HIP(hipDeviceSynchronize());
    dev_free(ix->list_term);   // belongs to the previous codebooks
    ix->has_books = true;
    return IVFR_OK;
}

extern "C" int ivfr_get_codebooks(const ivfr_index* ix, float* coarse, float* pq, float* rq) {
    IVFR_REQUIRE(ix && coarse && pq, "ivfr_get_codebooks: null argument");
    if (!ix->has_books) { ivfr_set_error("no codebooks yet"); return IVFR_ERR_STATE; }
    IVFR_TRY(use_device(ix));
    const ivfr_params& p = ix->p;
    IVFR_HIP(hipMemcpy(coarse, ix->coarse, (size_t)p.c * p.d * sizeof(float), hipMemcpyDeviceToHost));
    IVFR_HIP(hipMemcpy(pq, ix->pq, (size_t)p.m * IVFR_KS * ix->dsub * sizeof(float), hipMemcpyDeviceToHost));
    if (p.m_refine && rq)
        IVFR_HIP(hipMemcpy(rq, ix->rq, (size_t)p.m_refine * IVFR_KS * ix->dsub_r * sizeof(float), hipMemcpyDeviceToHost));
    return IVFR_OK;
}

static bool is_device_ptr(const void* p) {
    hipPointerAttribute_t attr;
    hipError_t e = hipPointerGetAttributes(&attr, p);
    if (e != hipSuccess) { (void)hipGetLastError(); return false; }
    return attr.type == hipMemoryTypeDevice;
}

// uint8 rows [a, a+n) of src (host or device) -> fp32 device buffer X; `stage` holds the bytes when src is on the host
static int load_rows_f32(const uint8_t* src, bool on_device, int64_t a, int64_t n, int d, uint8_t* stage, float* X,
                         hipStream_t st) {
    const uint8_t* dsrc = src + a * d;
    if (!on_device) {
        IVFR_HIP(hipMemcpyAsync(stage, src + a * d, (size_t)n * d, hipMemcpyHostToDevice, st));
        dsrc = stage;
    }
    return ivfr_launch_u8_to_f32(dsrc, n * d, X, st);
}

// ---- training -----------------------------------------------------------------------------
static inline uint64_t mix64(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// `count` distinct row indices in [0, n), chosen by the `count` smallest hashes of (seed, salt, row)
static void draw_rows(uint64_t seed, uint64_t salt, int64_t n, int count, std::vector<int64_t>& out) {
    std::vector<std::pair<uint64_t, int64_t>> h((size_t)n);
    const uint64_t key = mix64(seed * 0x9E3779B97F4A7C15ull + salt);
    for (int64_t i = 0; i < n; ++i) h[(size_t)i] = {mix64(key + (uint64_t)(i + 1) * 0x9E3779B97F4A7C15ull), i};
    std::nth_element(h.begin(), h.begin() + (count - 1), h.end());
    out.resize((size_t)count);
    for (int i = 0; i < count; ++i) out[(size_t)i] = h[(size_t)i].second;
    std::sort(out.begin(), out.end());
}

// Lloyd iterations for the `parts` sub-quantizers of a product quantizer on the rows of R [n, d]
static int train_pq(ivfr_index* ix, float* R, int64_t n, int parts, float* book, uint64_t seed, uint64_t salt0,
                    int iters, uint8_t* codes_tmp, unsigned long long* sums, unsigned long long* counts,
                    int64_t* d_idx, hipStream_t st) {
    const int d = ix->p.d, dsub = d / parts;
    std::vector<int64_t> rows;
    for (int j = 0; j < parts; ++j) {
        draw_rows(seed, salt0 + (uint64_t)j, n, IVFR_KS, rows);
        IVFR_HIP(hipMemcpyAsync(d_idx, rows.data(), IVFR_KS * sizeof(int64_t), hipMemcpyHostToDevice, st));
        IVFR_TRY(ivfr_launch_gather_rows(R, d, j * dsub, dsub, d_idx, IVFR_KS, book + (int64_t)j * IVFR_KS * dsub, st));
        IVFR_HIP(hipStreamSynchronize(st));   // rows is reused
    }
    const int64_t total = (int64_t)parts * IVFR_KS * dsub;
    for (int it = 0; it < iters; ++it) {
        IVFR_TRY(ivfr_launch_pq_encode(R, n, d, book, parts, codes_tmp, false, st));
        IVFR_HIP(hipMemsetAsync(sums, 0, (size_t)total * sizeof(unsigned long long), st));
        IVFR_HIP(hipMemsetAsync(counts, 0, (size_t)parts * IVFR_KS * sizeof(unsigned long long), st));
        IVFR_TRY(ivfr_launch_km_accum_pq(R, n, d, parts, codes_tmp, sums, counts, st));
        IVFR_TRY(ivfr_launch_km_update(book, total, dsub, sums, counts, st));
    }
    return IVFR_OK;
}

extern "C" int ivfr_train(ivfr_index* ix, const uint8_t* train, int64_t n, int32_t iters, uint64_t seed) {
    IVFR_REQUIRE(ix && train, "ivfr_train: null argument");
    IVFR_REQUIRE(iters >= 0, "iters = %d must be >= 0", iters);
    IVFR_REQUIRE(n >= ix->p.c && n >= IVFR_KS, "training set of %lld rows is smaller than max(c, 256)", (long long)n);
    if (ix->n_added > 0 || ix->finalized) { ivfr_set_error("codebooks cannot change after vectors were added"); return IVFR_ERR_STATE; }
    IVFR_TRY(use_device(ix));
    IVFR_TRY(alloc_books(ix));
    const ivfr_params& p = ix->p;
    const int d = p.d, c = p.c;
    hipStream_t st = nullptr;
    const bool on_dev = is_device_ptr(train);

    float* T = nullptr;
    uint8_t* stage = nullptr;
    int32_t* assign = nullptr;
    uint8_t* codes_tmp = nullptr;
    unsigned long long *sums = nullptr, *counts = nullptr;
    int64_t* d_idx = nullptr;
    const int max_parts = std::max(p.m, p.m_refine);
    const size_t sum_elems = std::max((size_t)c * d, (size_t)IVFR_KS * d);
    const size_t cnt_elems = std::max((size_t)c, (size_t)max_parts * IVFR_KS);
    int r = IVFR_OK;
    auto cleanup = [&]() {
        dev_free(T); dev_free(stage); dev_free(assign); dev_free(codes_tmp); dev_free(sums); dev_free(counts);
        dev_free(d_idx);
    };
#define TR(expr) do { r = (expr); if (r != IVFR_OK) { cleanup(); return r; } } while (0)
#define TRH(expr) do { hipError_t e_ = (expr); if (e_ != hipSuccess) { ivfr_set_error("%s failed: %s", #expr, hipGetErrorString(e_)); cleanup(); return IVFR_ERR_HIP; } } while (0)
    TR(dev_alloc(&T, (size_t)n * d));
    if (!on_dev) TR(dev_alloc(&stage, (size_t)n * d));
    TR(dev_alloc(&assign, (size_t)n));
    TR(dev_alloc(&codes_tmp, (size_t)n * max_parts));
    TR(dev_alloc(&sums, sum_elems));
    TR(dev_alloc(&counts, cnt_elems));
    TR(dev_alloc(&d_idx, (size_t)std::max(c, IVFR_KS)));
    TR(load_rows_f32(train, on_dev, 0, n, d, stage, T, st));

    // coarse quantizer: initial centroids = c distinct training rows
    {
        std::vector<int64_t> rows;
        draw_rows(seed, 1, n, c, rows);
        TRH(hipMemcpyAsync(d_idx, rows.data(), (size_t)c * sizeof(int64_t), hipMemcpyHostToDevice, st));
        TR(ivfr_launch_gather_rows(T, d, 0, d, d_idx, c, ix->coarse, st));
        TRH(hipStreamSynchronize(st));
    }
    for (int it = 0; it < iters; ++it) {
        TR(ivfr_launch_row_norms(ix->coarse, c, d, ix->coarse_norm, st));
        TR(ivfr_launch_assign(T, n, ix->coarse, ix->coarse_norm, c, d, assign, st));
        TRH(hipMemsetAsync(sums, 0, (size_t)c * d * sizeof(unsigned long long), st));
        TRH(hipMemsetAsync(counts, 0, (size_t)c * sizeof(unsigned long long), st));
        TR(ivfr_launch_km_accum_rows(T, n, d, assign, sums, counts, st));
        TR(ivfr_launch_km_update(ix->coarse, (int64_t)c * d, d, sums, counts, st));
    }
    // residuals to the coarse centroid, then q_c on them, then q_r on what q_c leaves
    TR(ivfr_launch_row_norms(ix->coarse, c, d, ix->coarse_norm, st));
    TR(ivfr_launch_assign(T, n, ix->coarse, ix->coarse_norm, c, d, assign, st));
    TR(ivfr_launch_residual(T, n, d, ix->coarse, assign, st));
    TR(train_pq(ix, T, n, p.m, ix->pq, seed, 100, iters, codes_tmp, sums, counts, d_idx, st));
    if (p.m_refine) {
        TR(ivfr_launch_pq_encode(T, n, d, ix->pq, p.m, nullptr, true, st));
        TR(train_pq(ix, T, n, p.m_refine, ix->rq, seed, 200, iters, codes_tmp, sums, counts, d_idx, st));
    }
    TR(refresh_norms(ix, st));
    TRH(hipStreamSynchronize(st));
    dev_free(ix->list_term);   // belongs to the previous codebooks
#undef TR
#undef TRH
    cleanup();
    ix->has_books = true;
    return IVFR_OK;
}

// ---- add / finalize ---------------------------------------------------------------------------
extern "C" int64_t ivfr_ntotal(const ivfr_index* ix) {
    if (!ix) { ivfr_set_error("ivfr_ntotal: null index"); return IVFR_ERR_INVALID_ARG; }
    return ix->finalized ? ix->N : ix->n_added;
}

extern "C" int ivfr_add(ivfr_index* ix, const uint8_t* x, int64_t n, int64_t id_base) {
    IVFR_REQUIRE(ix && (x || n == 0), "ivfr_add: null argument");
    IVFR_REQUIRE(n >= 0, "n = %lld must be >= 0", (long long)n);
    if (!ix->has_books) { ivfr_set_error("ivfr_add before codebooks were trained or set"); return IVFR_ERR_STATE; }
    if (ix->finalized) { ivfr_set_error("ivfr_add after ivfr_finalize"); return IVFR_ERR_STATE; }
    IVFR_REQUIRE(id_base >= 0 && id_base + n <= 2147483647LL, "ids %lld..%lld do not fit int32", (long long)id_base,
                 (long long)(id_base + n));
    IVFR_REQUIRE(ix->next_id == INT64_MIN || id_base >= ix->next_id, "id ranges must increase: id_base %lld < %lld",
                 (long long)id_base, (long long)ix->next_id);
    IVFR_REQUIRE(ix->n_added + n <= 4000000000LL, "index is limited to 4e9 entries");
    if (n == 0) return IVFR_OK;
    IVFR_TRY(use_device(ix));
    const ivfr_params& p = ix->p;
    const int d = p.d, c = p.c, m = p.m, mr = p.m_refine;
    hipStream_t st = nullptr;
    if (!ix->list_fill) {
        IVFR_TRY(dev_alloc(&ix->list_fill, (size_t)c));
        IVFR_HIP(hipMemset(ix->list_fill, 0, (size_t)c * sizeof(unsigned long long)));
    }
    const bool on_dev = is_device_ptr(x);
    const int64_t sub = std::min<int64_t>(n, ADD_SUB);
    int T = 4096;
    while ((int64_t)T * c > (1ll << 27) && T > 64) T >>= 1;
    // workspace: fp32 rows, staged bytes, rank counters
    size_t off_x = 0, off_stage = off_x + (size_t)sub * d * sizeof(float);
    size_t off_cnt = off_stage + (on_dev ? 0 : ((size_t)sub * d + 255) / 256 * 256);
    size_t total = off_cnt + (size_t)T * c * sizeof(uint32_t);
    IVFR_TRY(ix->encode_ws.reserve(total));
    char* ws = ix->encode_ws.as<char>();
    float* X = reinterpret_cast<float*>(ws + off_x);
    uint8_t* stage = reinterpret_cast<uint8_t*>(ws + off_stage);
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ws + off_cnt);

    StagedChunk ch;
    ch.n = n;
    int r = IVFR_OK;
    auto fail = [&](int code) {
        dev_free(ch.list); dev_free(ch.rank); dev_free(ch.ids); dev_free(ch.codes); dev_free(ch.rcodes);
        return code;
    };
    if ((r = dev_alloc(&ch.list, (size_t)n)) != IVFR_OK) return fail(r);
    if ((r = dev_alloc(&ch.rank, (size_t)n)) != IVFR_OK) return fail(r);
    if ((r = dev_alloc(&ch.ids, (size_t)n)) != IVFR_OK) return fail(r);
    if ((r = dev_alloc(&ch.codes, (size_t)n * m)) != IVFR_OK) return fail(r);
    if ((r = dev_alloc(&ch.rcodes, (size_t)n * mr)) != IVFR_OK) return fail(r);
#define AD(expr) do { r = (expr); if (r != IVFR_OK) { (void)hipDeviceSynchronize(); return fail(r); } } while (0)
    AD(ivfr_launch_iota(ch.ids, n, id_base, st));
    for (int64_t a = 0; a < n; a += sub) {
        const int64_t nb = std::min(sub, n - a);
        AD(load_rows_f32(x, on_dev, a, nb, d, stage, X, st));
        AD(ivfr_launch_assign(X, nb, ix->coarse, ix->coarse_norm, c, d, ch.list + a, st));
        AD(ivfr_launch_residual(X, nb, d, ix->coarse, ch.list + a, st));
        AD(ivfr_launch_pq_encode(X, nb, d, ix->pq, m, ch.codes + a * m, mr > 0, st));
        if (mr > 0) AD(ivfr_launch_pq_encode(X, nb, d, ix->rq, mr, ch.rcodes + a * mr, false, st));
        AD(ivfr_launch_list_ranks(ch.list + a, nb, c, ix->list_fill, cnt, T, ch.rank + a, st));
    }
    hipError_t e = hipStreamSynchronize(st);
    if (e != hipSuccess) { ivfr_set_error("ivfr_add: %s", hipGetErrorString(e)); return fail(IVFR_ERR_HIP); }
#undef AD
    ix->staged.push_back(ch);
    ix->n_added += n;
    ix->next_id = id_base + n;
    return IVFR_OK;
}

int ivfr_check_room(const ivfr_index* ix, size_t more) {
    if (more == 0) return IVFR_OK;
    if (ix->mem_limit > 0) {
        const size_t held = ix->index_bytes + ix->search_ws.bytes + ix->cand_ws.bytes + ix->dense_ws.bytes + ix->encode_ws.bytes;
        if (held + more > (size_t)ix->mem_limit) {
            ivfr_set_error("%zu more device bytes on top of the %zu held exceed the index's memory limit of %lld",
                           more, held, (long long)ix->mem_limit);
            return IVFR_ERR_OOM;
        }
    }
    size_t free_b = 0, total_b = 0;
    if (hipMemGetInfo(&free_b, &total_b) == hipSuccess) {
        if (more > free_b) {
            ivfr_set_error("%zu more device bytes needed, %zu free of %zu", more, free_b, total_b);
            return IVFR_ERR_OOM;
        }
    } else {
        (void)hipGetLastError();
    }
    return IVFR_OK;
}

static void free_layout(ivfr_index* ix) {
    dev_free(ix->list_start); dev_free(ix->list_len);
    dev_free(ix->codes); dev_free(ix->rec);
    ix->index_bytes = 0;
}

static int install_layout_inner(ivfr_index* ix, const std::vector<int64_t>& offsets);

// logical offsets -> padded layout on the device; a failure leaves nothing allocated, so the call can be repeated
static int install_layout(ivfr_index* ix, const std::vector<int64_t>& offsets) {
    free_layout(ix);
    const int r = install_layout_inner(ix, offsets);
    if (r != IVFR_OK) free_layout(ix);
    return r;
}

static int install_layout_inner(ivfr_index* ix, const std::vector<int64_t>& offsets) {
    const int c = ix->p.c;
    ix->h_offsets = offsets;
    ix->h_start.assign((size_t)c + 1, 0);
    std::vector<uint32_t> len((size_t)c);
    uint64_t pos = 0;
    for (int l = 0; l < c; ++l) {
        ix->h_start[(size_t)l] = (uint32_t)pos;
        uint64_t n = (uint64_t)(offsets[(size_t)l + 1] - offsets[(size_t)l]);
        len[(size_t)l] = (uint32_t)n;
        pos += (n + IVFR_LIST_ALIGN - 1) / IVFR_LIST_ALIGN * IVFR_LIST_ALIGN;
    }
    if (pos + IVFR_TAIL_PAD >= 0xFFFFFFFFull) { ivfr_set_error("index too large for 32-bit entry positions"); return IVFR_ERR_INVALID_ARG; }
    ix->h_start[(size_t)c] = (uint32_t)pos;
    ix->n_slots = pos + IVFR_TAIL_PAD;
    ix->N = offsets[(size_t)c];
    {
        // a query lands in a list with a probability proportional to its size: expected visited-list length
        double s2 = 0.0;
        for (int l = 0; l < c; ++l) s2 += (double)len[(size_t)l] * (double)len[(size_t)l];
        ix->wmean_len = ix->N > 0 ? s2 / (double)ix->N : 0.0;
    }
    IVFR_TRY(ivfr_check_room(ix, ivfr_index_bytes(ix->p, ix->n_slots)));
    ix->index_bytes = ivfr_index_bytes(ix->p, ix->n_slots);
    IVFR_TRY(dev_alloc(&ix->list_start, (size_t)c + 1));
    IVFR_TRY(dev_alloc(&ix->list_len, (size_t)c));
    IVFR_HIP(hipMemcpy(ix->list_start, ix->h_start.data(), ((size_t)c + 1) * sizeof(uint32_t), hipMemcpyHostToDevice));
    IVFR_HIP(hipMemcpy(ix->list_len, len.data(), (size_t)c * sizeof(uint32_t), hipMemcpyHostToDevice));
    ix->rec_stride = ivfr_record_stride(ix->p);
    IVFR_TRY(dev_alloc(&ix->codes, (size_t)ix->n_slots * ix->p.m));
    IVFR_TRY(dev_alloc(&ix->rec, (size_t)ix->n_slots * ix->rec_stride));
    IVFR_HIP(hipMemset(ix->codes, 0, (size_t)ix->n_slots * ix->p.m));
    IVFR_HIP(hipMemset(ix->rec, 0xff, (size_t)ix->n_slots * ix->rec_stride));   // padding slots: id -1
    return IVFR_OK;
}

extern "C" int ivfr_finalize(ivfr_index* ix) {
    IVFR_REQUIRE(ix, "ivfr_finalize: null index");
    if (ix->finalized) { ivfr_set_error("index already finalized"); return IVFR_ERR_STATE; }
    if (!ix->has_books) { ivfr_set_error("ivfr_finalize before codebooks were trained or set"); return IVFR_ERR_STATE; }
    IVFR_TRY(use_device(ix));
    const int c = ix->p.c;
    std::vector<unsigned long long> fill((size_t)c, 0ull);
    if (ix->list_fill)
        IVFR_HIP(hipMemcpy(fill.data(), ix->list_fill, (size_t)c * sizeof(unsigned long long), hipMemcpyDeviceToHost));
    std::vector<int64_t> offsets((size_t)c + 1, 0);
    for (int l = 0; l < c; ++l) offsets[(size_t)l + 1] = offsets[(size_t)l] + (int64_t)fill[(size_t)l];
    if (offsets[(size_t)c] != ix->n_added) { ivfr_set_error("internal: list fill %lld != added %lld", (long long)offsets[(size_t)c], (long long)ix->n_added); return IVFR_ERR_STATE; }
    IVFR_TRY(install_layout(ix, offsets));
    for (auto& ch : ix->staged)
        IVFR_TRY(ivfr_launch_scatter(ch, ix->p.m, ix->p.m_refine, ix->list_start, ix->codes, ix->rec, ix->rec_stride, nullptr));
    IVFR_HIP(hipDeviceSynchronize());
    free_staged(ix);
    ix->encode_ws.release();
    ix->finalized = true;
    return IVFR_OK;
}

extern "C" int ivfr_export(const ivfr_index* ix, int64_t* list_offsets, int32_t* ids, uint8_t* codes, uint8_t* rcodes) {
    IVFR_REQUIRE(ix && list_offsets && ids && codes, "ivfr_export: null argument");
    IVFR_REQUIRE(ix->p.m_refine == 0 || rcodes, "ivfr_export: rcodes is required when m_refine > 0");
    if (!ix->finalized) { ivfr_set_error("ivfr_export before ivfr_finalize"); return IVFR_ERR_STATE; }
    IVFR_TRY(use_device(ix));
    const int c = ix->p.c, m = ix->p.m, mr = ix->p.m_refine;
    memcpy(list_offsets, ix->h_offsets.data(), ((size_t)c + 1) * sizeof(int64_t));
    // ids and refinement codes are unpacked from the per-entry records into dense per-slot staging arrays, a run of
    // whole lists at a time; every list is then one contiguous copy per array
    ivfr_index* mix = const_cast<ivfr_index*>(ix);
    const uint64_t chunk_slots = 1ull << 24;
    int l = 0;
    while (l < c) {
        const uint64_t s0 = ix->h_start[(size_t)l];
        int l1 = l + 1;
        while (l1 < c && (uint64_t)ix->h_start[(size_t)l1 + 1] - s0 <= chunk_slots) ++l1;
        const uint64_t ns = (uint64_t)ix->h_start[(size_t)l1] - s0;   // slots of lists l .. l1-1 (at least one list)
        if (ns > 0) {
            IVFR_TRY(ivfr_check_room(ix, ns * (4 + (size_t)mr) > ix->encode_ws.bytes ? ns * (4 + (size_t)mr) + 512 : 0));
            IVFR_TRY(mix->encode_ws.reserve(ns * (4 + (size_t)mr) + 512));
            int32_t* ids_st = mix->encode_ws.as<int32_t>();
            uint8_t* rc_st = mix->encode_ws.as<uint8_t>() + ((ns * 4 + 255) / 256 * 256);
            IVFR_TRY(ivfr_launch_unpack_records(ix, s0, (int64_t)ns, ids_st, rc_st, nullptr));
            IVFR_HIP(hipDeviceSynchronize());
            for (int j = l; j < l1; ++j) {
                const int64_t a = ix->h_offsets[(size_t)j], n = ix->h_offsets[(size_t)j + 1] - a;
                if (n == 0) continue;
                const uint64_t s = ix->h_start[(size_t)j], rel = s - s0;
                IVFR_HIP(hipMemcpy(ids + a, ids_st + rel, (size_t)n * sizeof(int32_t), hipMemcpyDeviceToHost));
                IVFR_HIP(hipMemcpy(codes + a * m, ix->codes + s * m, (size_t)n * m, hipMemcpyDeviceToHost));
                if (mr) IVFR_HIP(hipMemcpy(rcodes + a * mr, rc_st + rel * mr, (size_t)n * mr, hipMemcpyDeviceToHost));
            }
        }
        l = l1;
    }
    mix->encode_ws.release();
    return IVFR_OK;
}

extern "C" int ivfr_import(ivfr_index* ix, int64_t N, const int64_t* list_offsets, const int32_t* ids,
                           const uint8_t* codes, const uint8_t* rcodes) {
    IVFR_REQUIRE(ix && list_offsets && (N == 0 || (ids && codes)), "ivfr_import: null argument");
    IVFR_REQUIRE(ix->p.m_refine == 0 || N == 0 || rcodes, "ivfr_import: rcodes is required when m_refine > 0");
    if (!ix->has_books) { ivfr_set_error("ivfr_import before codebooks were set"); return IVFR_ERR_STATE; }
    if (ix->finalized || ix->n_added > 0) { ivfr_set_error("ivfr_import into a non-empty index"); return IVFR_ERR_STATE; }
    const int c = ix->p.c, m = ix->p.m, mr = ix->p.m_refine;
    IVFR_REQUIRE(N >= 0 && N <= 2147483647LL, "N = %lld out of range", (long long)N);
    IVFR_REQUIRE(list_offsets[0] == 0 && list_offsets[c] == N, "list_offsets must run from 0 to N");
    for (int l = 0; l < c; ++l)
        IVFR_REQUIRE(list_offsets[l + 1] >= list_offsets[l], "list_offsets must be non-decreasing (list %d)", l);
    for (int64_t i = 0; i < N; ++i)
        IVFR_REQUIRE(ids[i] >= 0, "ids must be >= 0 (entry %lld has id %d)", (long long)i, (int)ids[i]);
    IVFR_TRY(use_device(ix));
    std::vector<int64_t> offsets(list_offsets, list_offsets + c + 1);
    IVFR_TRY(install_layout(ix, offsets));
    // codes go straight to the scan's dense stream; ids and refinement codes through dense per-slot staging arrays,
    // a run of whole lists at a time, from which the per-entry records are packed on the device
    const uint64_t chunk_slots = 1ull << 24;
    int l = 0;
    while (l < c) {
        const uint64_t s0 = ix->h_start[(size_t)l];
        int l1 = l + 1;
        while (l1 < c && (uint64_t)ix->h_start[(size_t)l1 + 1] - s0 <= chunk_slots) ++l1;
        const uint64_t ns = (uint64_t)ix->h_start[(size_t)l1] - s0;
        if (ns > 0) {
            IVFR_TRY(ivfr_check_room(ix, ns * (4 + (size_t)mr) > ix->encode_ws.bytes ? ns * (4 + (size_t)mr) + 512 : 0));
            IVFR_TRY(ix->encode_ws.reserve(ns * (4 + (size_t)mr) + 512));
            int32_t* ids_st = ix->encode_ws.as<int32_t>();
            uint8_t* rc_st = ix->encode_ws.as<uint8_t>() + ((ns * 4 + 255) / 256 * 256);
            for (int j = l; j < l1; ++j) {
                const int64_t a = offsets[(size_t)j], n = offsets[(size_t)j + 1] - a;
                if (n == 0) continue;
                const uint64_t s = ix->h_start[(size_t)j], rel = s - s0;
                IVFR_HIP(hipMemcpy(ids_st + rel, ids + a, (size_t)n * sizeof(int32_t), hipMemcpyHostToDevice));
                IVFR_HIP(hipMemcpy(ix->codes + s * m, codes + a * m, (size_t)n * m, hipMemcpyHostToDevice));
                if (mr) IVFR_HIP(hipMemcpy(rc_st + rel * mr, rcodes + a * mr, (size_t)n * mr, hipMemcpyHostToDevice));
            }
            IVFR_TRY(ivfr_launch_pack_records(ix, s0, (int64_t)ns, ids_st, rc_st, nullptr));
            IVFR_HIP(hipDeviceSynchronize());
        }
        l = l1;
    }
    ix->encode_ws.release();
    IVFR_HIP(hipDeviceSynchronize());
    ix->n_added = N;
    ix->finalized = true;
    return IVFR_OK;
}

extern "C" int ivfr_set_tuning(ivfr_index* ix, int32_t full_mult, int32_t cap_mult, int32_t min_cap, int32_t batch,
                               int32_t scan_groups) {
    IVFR_REQUIRE(ix, "ivfr_set_tuning: null index");
    IVFR_REQUIRE(full_mult >= 0 && cap_mult >= 0 && min_cap >= 0 && batch >= 0 && scan_groups >= 0,
                 "tuning values must be >= 0");
    IVFR_REQUIRE(batch <= 65535, "batch = %d exceeds 65535", batch);
    if (full_mult) ix->full_mult = full_mult;
    if (cap_mult) ix->cap_mult = cap_mult;
    if (min_cap) ix->min_cap = min_cap;
    if (batch) ix->batch = batch;
    ix->scan_groups = scan_groups;
    return IVFR_OK;
}

int ivfr_ensure_list_terms(ivfr_index* ix, hipStream_t st) {
    if (ix->list_term) return IVFR_OK;
    const size_t count = (size_t)ix->p.c * ix->p.m * IVFR_KS;
    IVFR_TRY(ivfr_check_room(ix, count * sizeof(float)));
    IVFR_TRY(dev_alloc(&ix->list_term, count));
    ix->index_bytes += count * sizeof(float);
    const int r = ivfr_launch_list_terms(ix, ix->list_term, st);
    if (r != IVFR_OK) { dev_free(ix->list_term); ix->index_bytes -= count * sizeof(float); }
    return r;
}

extern "C" int ivfr_set_table_mode(ivfr_index* ix, int32_t mode) {
    IVFR_REQUIRE(ix, "ivfr_set_table_mode: null index");
    IVFR_REQUIRE(mode == 0 || mode == 1, "table mode %d must be 0 (one table per pair) or 1 (split tables)", mode);
    ix->split_tables = mode;
    return IVFR_OK;
}

extern "C" int ivfr_set_memory_limit(ivfr_index* ix, int64_t bytes) {
    IVFR_REQUIRE(ix, "ivfr_set_memory_limit: null index");
    IVFR_REQUIRE(bytes >= 0, "memory limit %lld must be >= 0", (long long)bytes);
    ix->mem_limit = bytes;
    return IVFR_OK;
}

extern "C" int ivfr_workspace_info(const ivfr_index* ix, int64_t* index_bytes, int64_t* workspace_bytes,
                                   int64_t* pool_bytes, int64_t* batch_reruns) {
    IVFR_REQUIRE(ix, "ivfr_workspace_info: null index");
    if (index_bytes) *index_bytes = (int64_t)ix->index_bytes;
    if (workspace_bytes) *workspace_bytes = (int64_t)(ix->search_ws.bytes + ix->dense_ws.bytes);
    if (pool_bytes) *pool_bytes = (int64_t)ix->cand_ws.bytes;
    if (batch_reruns) *batch_reruns = ix->st_reruns;
    return IVFR_OK;
}

extern "C" int ivfr_set_profiling(ivfr_index* ix, int32_t enable) {
    IVFR_REQUIRE(ix, "ivfr_set_profiling: null index");
    IVFR_REQUIRE(enable >= 0 && enable <= 2, "profiling level %d must be 0, 1 or 2", enable);
    ix->profiling = enable;
    return IVFR_OK;
}

extern "C" int ivfr_stage_times(const ivfr_index* ix, double* ms, int32_t* scan_launches) {
    IVFR_REQUIRE(ix && ms, "ivfr_stage_times: null argument");
    for (int i = 0; i < IVFR_N_STAGES; ++i) ms[i] = ix->prof_ms[i];
    if (scan_launches) *scan_launches = ix->prof_scan_launches;
    return IVFR_OK;
}

extern "C" int ivfr_search_stats(const ivfr_index* ix, int64_t* codes_scanned, int64_t* pairs, int64_t* dense_fallbacks,
                                 int64_t* codes_streamed, int64_t* codes_scanned_shared,
                                 int64_t* codes_scanned_shared2, int64_t* codes_scanned_shared8,
                                 int64_t* bound_retries, int64_t* codes_scanned_shared64) {
    IVFR_REQUIRE(ix, "ivfr_search_stats: null index");
    if (codes_scanned) *codes_scanned = ix->st_codes;
    if (pairs) *pairs = ix->st_pairs;
    if (dense_fallbacks) *dense_fallbacks = ix->st_dense;
    if (codes_streamed) *codes_streamed = ix->st_streamed;
    if (codes_scanned_shared) *codes_scanned_shared = ix->st_shared_codes;
    if (codes_scanned_shared2) *codes_scanned_shared2 = ix->st_shared2_codes;
    if (codes_scanned_shared8) *codes_scanned_shared8 = ix->st_shared8_codes;
    if (bound_retries) *bound_retries = ix->st_retries;
    if (codes_scanned_shared64) *codes_scanned_shared64 = ix->st_shared64_codes;
    return IVFR_OK;
}

extern "C" int ivfr_set_list_sharing(ivfr_index* ix, int32_t mode) {
    IVFR_REQUIRE(ix, "ivfr_set_list_sharing: null index");
    IVFR_REQUIRE(mode >= -1 && mode <= 3, "list sharing mode %d must be -1 (automatic), 0, 1, 2 or 3", mode);
    ix->share_lists = mode;
    return IVFR_OK;
}
