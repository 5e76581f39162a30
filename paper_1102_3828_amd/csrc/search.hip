// Query stage (section 3.2 steps 1-3 on the inverted file of section 3.3): host orchestration.
//
// Per internal batch of queries:
//   coarse distances (MFMA) -> w nearest lists -> plan of (query, list) pairs, grouped by list into
//   units of queries that share a pass -> look-up tables (MFMA) -> sample of the visited entries
//   (the same leading fraction of every visited list) -> per-query bound tau on the k'-th smallest
//   estimate -> scan of every visited entry keeping estimates <= tau (four launches side by side:
//   units of eight, four, two queries and single pairs; in sharing mode 3 a fifth for units of 64 on
//   the matrix cores) -> exact k' smallest of the survivors -> re-rank -> k smallest.
//
// Everything of a batch is enqueued without a host round trip.  What the host used to ask for in
// the middle of a batch is decided on the device instead: the kernels read their unit counts and
// work totals from device memory and pick the number of workgroups that take part from them (the
// host launches from an estimate kept from the previous call), the candidate pool is checked by
// the plan kernel (a pool that is too small voids the batch: it does no list work and is run again
// after the pool has grown), and queries with a component that is not finite only raise a flag.
// The status words of every batch go to a pinned host slot with one asynchronous copy; the host
// waits for the stream once, after the last batch, and reads them.
//
// tau is a statistical bound (the r-th smallest sampled estimate, r chosen five standard
// deviations above the expected number of true k'-best entries in the sample), so the scan
// verifies it by counting: a query whose survivors overflow its candidate buffer is rescanned
// with a tightened key bound, one that kept fewer than k' is redone through a buffer that holds
// every visited entry.  Results are therefore exact whatever the sample says; the bound only
// decides how much is written.  These redo passes are the one place where the host waits more
// than once: at most eight rescans and one unfiltered pass per failing query.
#include "ivfr_internal.h"

#include <algorithm>
#include <chrono>
#include <mutex>
#include <string.h>

int ivfr_launch_select_records(const SelectArgs& a, int out_base, const unsigned long long* sq, uint32_t* out_pos,
                               float* out_est, int32_t* out_n, int32_t* overflow, int32_t* overflow_total,
                               hipStream_t st);
int ivfr_launch_select_sorted(const SelectArgs& a, const int32_t* counts_i32, int out_base, int32_t* out_lo,
                              float* out_hi, hipStream_t st);
int ivfr_launch_rerank(const ivfr_index* ix, const float* queries, int q_base, int nq, int kprime,
                       const uint32_t* short_pos, const int32_t* short_n, uint64_t* keys, float* refined_out,
                       int32_t* ids_out, hipStream_t st);

// Workspace of ivfr_search_static, for callers that cannot allocate.  Every device holds its own copy of the
// array, at its own address, until the process ends.  In host code the array's name is only a handle: the
// address of a device's copy is asked from the runtime once, with that device current, and that address is
// what host code passes to kernels and copies from then on.
static __device__ __align__(256) unsigned char ivfr_static_scratch[IVFR_STATIC_SCRATCH_BYTES];

#define IVFR_MAX_DEVICES 64
static char* g_static_addr[IVFR_MAX_DEVICES];
static std::mutex g_static_mutex;

int ivfr_static_scratch_address(int device, char** out) {
    *out = nullptr;
    if (device < 0 || device >= IVFR_MAX_DEVICES) {
        ivfr_set_error("device %d: the static workspace covers device ordinals below %d", device, IVFR_MAX_DEVICES);
        return IVFR_ERR_INVALID_ARG;
    }
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_addr[device]) {
        IVFR_HIP(hipSetDevice(device));
        void* p = nullptr;
        IVFR_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(ivfr_static_scratch)));
        g_static_addr[device] = static_cast<char*>(p);
    }
    *out = g_static_addr[device];
    return IVFR_OK;
}

// Start of a batch: clear the counters (one contiguous block), mark every unit slot empty, tau = +inf.
__global__ __launch_bounds__(256) void batch_reset_kernel(uint32_t* zero, size_t zero_words, uint32_t* ones,
                                                          size_t ones_words, float* tau, int nb) {
    const size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (size_t i = i0; i < zero_words; i += stride) zero[i] = 0u;
    for (size_t i = i0; i < ones_words; i += stride) ones[i] = 0xFFFFFFFFu;
    for (size_t i = i0; i < (size_t)nb; i += stride) tau[i] = INFINITY;
}

// Set-up of the unfiltered redo of one query: counter 0, bound +inf.
__global__ void dense_reset_kernel(uint32_t* cnt, float* tau) {
    if (threadIdx.x == 0) { *cnt = 0u; *tau = INFINITY; }
}

__global__ void clear_u32_kernel(uint32_t* p) {
    if (threadIdx.x == 0) *p = 0u;
}

struct Carver {
    size_t off = 0;
    template <class T> size_t take(size_t count) {
        size_t a = (off + 255) / 256 * 256;
        off = a + count * sizeof(T);
        return a;
    }
};

// Smallest Poisson mean of true k'-best entries wanted inside the sample: the sample stride (one entry in
// `stride` is sampled) never exceeds k' / mu; the plan narrows it when a larger sample pays off.
#define IVFR_SAMPLE_MU 2
// Upper limit of a query's sample (entries); beyond it the stride widens and the bound loosens.
#define IVFR_MAX_SAMPLE 131072u
// Queries whose bound is expected to pass more than this share of their estimates stay out of the
// half-precision units (the fp32 re-evaluation of what passes would dominate).  Measured: at 10^9 vectors a
// query set passing 0.04 % runs twice as fast as in the fp32 units of four; the paper's k' = 20000 (0.5-0.8 %)
// runs 11 % faster with 0.01 than with 0.002; at 10^8 vectors and k' = 10000 (about 1 %, half of the queries
// on either side) 0.01 is 4 % faster than 0.002 and 0.02 is 2 % slower.
#define IVFR_HALF_UNIT_FRAC 0.01f

// Byte offsets of one batch's arrays inside the search workspace.
struct SearchLayout {
    size_t xnorm, ckeys, probe, probed, pstart, len, pre, lens, pres, items, soff, nsample, qblk, sq, su, fully, exonly,
        capq, coff, lut, pbase, tau, tauid, spos, sest, sn, over, rkeys, sref, sids, lscale, gpre, gcur, gu8, gu2, glop, gblk8,
        gblk4, gblk2, gblklo, gu64, gblk64, status, cnt, gnp;
    size_t n_items_max, n_u8, n_u4, zero_words, bytes;
};

static SearchLayout layout_search(const ivfr_params& p, int B, int w, int kprime, bool split) {
    SearchLayout L;
    const size_t P = (size_t)B * w, c = (size_t)p.c;
    Carver cv;
    L.xnorm = cv.take<float>(B);
    L.ckeys = cv.take<uint64_t>((size_t)B * c);
    L.probe = cv.take<int32_t>(P);
    L.probed = cv.take<float>(P);
    L.pstart = cv.take<uint32_t>(P);
    L.len = cv.take<uint32_t>(P);
    L.pre = cv.take<uint32_t>(P + 1);
    L.lens = cv.take<uint32_t>(P);
    L.pres = cv.take<uint32_t>(P + 1);
    // chunks of the sample: at most one partial chunk per pair plus the full ones of IVFR_MAX_SAMPLE + w entries
    L.n_items_max = P + (size_t)B * ((IVFR_MAX_SAMPLE + (size_t)w) / IVFR_SAMPLE_CHUNK + 1);
    L.items = cv.take<uint32_t>(L.n_items_max);
    L.soff = cv.take<uint32_t>(P);
    L.nsample = cv.take<uint32_t>(B);
    L.qblk = cv.take<uint32_t>(2 * (size_t)B);
    L.sq = cv.take<unsigned long long>(B);
    L.su = cv.take<unsigned long long>(B);
    L.fully = cv.take<uint8_t>(B);
    L.exonly = cv.take<uint8_t>(B);
    L.capq = cv.take<uint32_t>(B);
    L.coff = cv.take<unsigned long long>(B);
    // look-up tables: one per (query, list) pair, or with split tables one term table per query and m scalars per pair
    L.lut = cv.take<float>((split ? (size_t)B : P) * p.m * IVFR_KS);
    L.pbase = cv.take<float>(split ? P * p.m : 1);
    L.tau = cv.take<float>(B);
    L.tauid = cv.take<uint32_t>(B);
    L.spos = cv.take<uint32_t>((size_t)B * kprime);
    L.sest = cv.take<float>((size_t)B * kprime);
    L.sn = cv.take<int32_t>(B);
    L.over = cv.take<int32_t>(B);
    L.rkeys = cv.take<uint64_t>((size_t)B * kprime);
    L.sref = cv.take<float>((size_t)B * kprime);
    L.sids = cv.take<int32_t>((size_t)B * kprime);
    L.lscale = cv.take<float>(P);
    L.gpre = cv.take<uint32_t>(5 * c);
    L.gcur = cv.take<uint32_t>(2 * c);
    // units of eight: at most P/8 + c (one more per list for a remainder of 5..7); units of four likewise
    L.n_u8 = (P / 8 + c + 1) * 8;
    L.n_u4 = (P / 4 + c + 1) * 4;
    L.gu8 = cv.take<uint32_t>(L.n_u8 + L.n_u4);
    L.gu2 = cv.take<uint32_t>(2 * c + 4);
    L.glop = cv.take<uint32_t>(c + 4);
    L.gblk8 = cv.take<uint32_t>(P / 8 + c + 2);
    L.gblk4 = cv.take<uint32_t>(P / 4 + c + 2);
    L.gblk2 = cv.take<uint32_t>(c + 2);
    L.gblklo = cv.take<uint32_t>(c + 2);
    L.gu64 = cv.take<uint32_t>((P / 64 + 1) * 64);   // units of 64 are always full
    L.gblk64 = cv.take<uint32_t>(P / 64 + 2);
    // cleared by one kernel at the start of every batch: status words, candidate counters, pairs per list
    L.status = cv.take<DevStatus>(1);
    L.cnt = cv.take<uint32_t>(B);
    L.gnp = cv.take<uint32_t>(2 * c);
    L.zero_words = (cv.off - L.status + 3) / 4;
    L.bytes = (cv.off + 511) / 256 * 256;
    return L;
}

// Queries per internal batch: the tuning value, lowered so that the per-batch tables (w m KB per query) stay
// below 8 GiB, the coarse keys (8 c bytes) and the short-list arrays (24 k' bytes) below 4 GiB each; a call that
// needs several batches gets equal ones (the more queries share a batch, the more they share list reads).
static int64_t batch_size(const ivfr_index* ix, int64_t nq, int w, int kprime) {
    const ivfr_params& p = ix->p;
    int64_t B = std::min<int64_t>(nq, ix->batch);
    const int64_t budget = 4ll << 30;
    if (!ix->split_tables) B = std::min<int64_t>(B, std::max<int64_t>(1, 2 * budget / ((int64_t)w * p.m * IVFR_KS * 4)));
    B = std::min<int64_t>(B, std::max<int64_t>(1, budget / ((int64_t)kprime * 24)));
    B = std::min<int64_t>(B, std::max<int64_t>(1, budget / ((int64_t)p.c * 8)));
    return std::max<int64_t>(B, 1);
}

// Candidate-pool records a batch of nb queries is expected to want when every query visits `per_query` entries.
static unsigned long long pool_estimate(const ivfr_index* ix, int nb, int w, int kprime, double per_query) {
    const uint32_t min_cap = (uint32_t)std::max<int64_t>((int64_t)ix->cap_mult * kprime, ix->min_cap);
    const uint32_t full_limit = (uint32_t)std::min<int64_t>((int64_t)ix->full_mult * kprime, 1ll << 30);
    const uint32_t stride_k = (uint32_t)std::max(1, kprime / IVFR_SAMPLE_MU);
    const unsigned long long total = (unsigned long long)std::max(per_query, 1.0);
    const unsigned long long total_u = ivfr_sample_threshold(total, kprime);
    const QueryPlan qp = ivfr_plan_query(total, total_u, full_limit, stride_k, IVFR_MAX_SAMPLE, kprime);
    const unsigned long long sampled = qp.fully ? 0ull : total_u / qp.stride + (unsigned long long)w;
    bool eo;
    const unsigned long long cap = ivfr_plan_capacity(total, total_u, sampled, qp, min_cap, kprime, IVFR_HALF_UNIT_FRAC, &eo);
    return (unsigned long long)nb * ((cap + 31ull) & ~31ull);
}

extern "C" int ivfr_memory_required(const ivfr_params* params, int64_t N, int64_t nq, int32_t w, int32_t kprime,
                                    int64_t available_bytes, int64_t* index_bytes, int64_t* search_bytes) {
    IVFR_REQUIRE(params, "ivfr_memory_required: null params");
    const ivfr_params& p = *params;
    IVFR_REQUIRE(p.d > 0 && p.c >= 1 && p.m >= 1 && p.m_refine >= 0, "ivfr_memory_required: bad parameters");
    IVFR_REQUIRE(N >= 0 && nq >= 0 && (nq == 0 || (w >= 1 && w <= p.c && kprime >= 1)),
                 "ivfr_memory_required: bad sizes");
    const uint64_t n_slots = (uint64_t)N + (uint64_t)p.c * (IVFR_LIST_ALIGN - 1) + IVFR_TAIL_PAD;
    int64_t ib = (int64_t)ivfr_index_bytes(p, n_slots);
    ib += (int64_t)p.c * (p.d + 1) * 4 + (int64_t)(p.m + p.m_refine) * IVFR_KS * 4 + (int64_t)p.m * IVFR_KS * 4;
    int64_t sb = 0;
    if (nq > 0) {
        ivfr_index tmp;
        tmp.p = p;
        const int64_t B0 = batch_size(&tmp, nq, w, kprime);
        const int64_t nb = (nq + B0 - 1) / B0;
        const int B = (int)((nq + nb - 1) / nb);
        sb = (int64_t)layout_search(p, B, w, kprime, false).bytes;
        const double per_query = (double)w * ((double)N / (double)p.c);
        sb += (int64_t)(pool_estimate(&tmp, B, w, kprime, per_query) * sizeof(uint2));
    }
    if (index_bytes) *index_bytes = ib;
    if (search_bytes) *search_bytes = sb;
    if (available_bytes > 0 && ib + sb > available_bytes) {
        ivfr_set_error("index (%lld bytes) and search workspace (%lld bytes) exceed the %lld bytes available",
                       (long long)ib, (long long)sb, (long long)available_bytes);
        return IVFR_ERR_OOM;
    }
    return IVFR_OK;
}

namespace {
struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    int kind = 0;   // IVFR_STAGE_*
};
}

// fixed_ws != nullptr: workspace and candidate pool are carved from that buffer and nothing is allocated.
static int run_search(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                      int32_t* ids_out, float* dist_out, int32_t* probe_out, float* probe_dist_out,
                      int32_t* short_ids_out, float* short_est_out, float* short_ref_out, int32_t* short_count_out,
                      void* stream, char* fixed_ws, size_t fixed_bytes) {
    IVFR_REQUIRE(ix && (nq == 0 || (queries && ids_out && dist_out)), "ivfr_search: null argument");
    if (!ix->finalized) { ivfr_set_error("ivfr_search before ivfr_finalize / ivfr_import"); return IVFR_ERR_STATE; }
    const ivfr_params& p = ix->p;
    IVFR_REQUIRE(nq >= 0, "nq = %lld must be >= 0", (long long)nq);
    IVFR_REQUIRE(w >= 1 && w <= p.c, "w = %d must be in [1, c = %d]", w, p.c);
    IVFR_REQUIRE(kprime >= 1, "kprime = %d must be >= 1", kprime);
    IVFR_REQUIRE(k >= 1 && k <= kprime, "k = %d must be in [1, kprime = %d]", k, kprime);
    IVFR_REQUIRE(k <= 16384 && w <= 16384, "k and w are limited to 16384");
    IVFR_REQUIRE((int64_t)kprime * ix->cap_mult < (1ll << 31), "kprime * cap_mult too large");
    IVFR_HIP(hipSetDevice(p.device));
    hipStream_t st = reinterpret_cast<hipStream_t>(stream);
    ix->st_codes = ix->st_pairs = ix->st_dense = ix->st_streamed = ix->st_shared_codes = ix->st_shared2_codes = ix->st_shared8_codes = ix->st_retries = ix->st_shared64_codes = 0;
    for (int i = 0; i < IVFR_N_STAGES; ++i) ix->prof_ms[i] = 0;
    ix->prof_scan_launches = 0;
    ix->st_reruns = 0;
    if (nq == 0) return IVFR_OK;
    const bool fixed = fixed_ws != nullptr;

    const int d = p.d, c = p.c, m = p.m;
    // expected entries visited per query: lists are hit in proportion to their size
    const double visit_est = std::min((double)w * std::max(ix->wmean_len, 1.0), (double)std::max<int64_t>(ix->N, 1));
    int64_t B64 = batch_size(ix, nq, w, kprime);
    auto even_batches = [&](int64_t b) {
        const int64_t n_batches = (nq + b - 1) / b;
        return (nq + n_batches - 1) / n_batches;
    };
    B64 = even_batches(B64);
    const bool split = ix->split_tables != 0;
    if (split) {
        if (fixed_ws && !ix->list_term) {
            ivfr_set_error("split tables: the per-list table is built by the first ivfr_search call in this mode; "
                           "the fixed-workspace entry point cannot allocate it");
            return IVFR_ERR_STATE;
        }
        IVFR_TRY(ivfr_ensure_list_terms(ix, reinterpret_cast<hipStream_t>(stream)));
    }
    SearchLayout L = layout_search(p, (int)B64, w, kprime, split);
    unsigned long long pool_cap = 0;
    if (fixed) {
        // the largest batch whose arrays and expected candidate pool (with a quarter in reserve) fit the buffer
        for (;;) {
            const unsigned long long want = pool_estimate(ix, (int)B64, w, kprime, visit_est);
            const size_t need = L.bytes + (size_t)(want + want / 4 + 64) * sizeof(uint2);
            if (need <= fixed_bytes) break;
            if (B64 == 1) {
                ivfr_set_error("the fixed workspace of %zu bytes is too small for one query with w = %d, k' = %d (needs %zu); "
                               "use ivfr_search", fixed_bytes, w, kprime, need);
                return IVFR_ERR_OOM;
            }
            B64 = even_batches((B64 + 1) / 2);
            L = layout_search(p, (int)B64, w, kprime, split);
        }
        pool_cap = (fixed_bytes - L.bytes) / sizeof(uint2) - 64;
    }
    const int B = (int)B64;
    // Queries visiting no more than full_limit entries keep them all; the others get a candidate
    // buffer for the larger of their sample and min_cap survivors (sized per query by the plan).
    const uint32_t min_cap = (uint32_t)std::max<int64_t>((int64_t)ix->cap_mult * kprime, ix->min_cap);
    const uint32_t full_limit = (uint32_t)std::min<int64_t>((int64_t)ix->full_mult * kprime, 1ll << 30);
    const uint32_t stride_k = (uint32_t)std::max(1, kprime / IVFR_SAMPLE_MU);

    char* ws = nullptr;
    uint2* cand = nullptr;
    if (fixed) {
        ws = fixed_ws;
        cand = reinterpret_cast<uint2*>(fixed_ws + L.bytes);
    } else {
        const unsigned long long want = pool_estimate(ix, B, w, kprime, visit_est);
        const size_t pool_bytes = std::max((size_t)(want + want / 4 + 64) * sizeof(uint2), ix->cand_ws.bytes);
        IVFR_TRY(ivfr_check_room(ix, (L.bytes > ix->search_ws.bytes ? L.bytes : 0) +
                                         (pool_bytes > ix->cand_ws.bytes ? pool_bytes : 0)));
        IVFR_TRY(ix->search_ws.reserve(L.bytes));
        IVFR_TRY(ix->cand_ws.reserve(pool_bytes));
        ws = ix->search_ws.as<char>();
        cand = ix->cand_ws.as<uint2>();
        pool_cap = ix->cand_ws.bytes / sizeof(uint2) - 64;
    }

    float* xnorm = reinterpret_cast<float*>(ws + L.xnorm);
    uint64_t* ckeys = reinterpret_cast<uint64_t*>(ws + L.ckeys);
    int32_t* probe = reinterpret_cast<int32_t*>(ws + L.probe);
    float* probed = reinterpret_cast<float*>(ws + L.probed);
    DevStatus* dstat = reinterpret_cast<DevStatus*>(ws + L.status);
    PlanBuffers pb;
    pb.pair_start = reinterpret_cast<uint32_t*>(ws + L.pstart);
    pb.len = reinterpret_cast<uint32_t*>(ws + L.len);
    pb.blkpre = reinterpret_cast<uint32_t*>(ws + L.pre);
    pb.len_s = reinterpret_cast<uint32_t*>(ws + L.lens);
    pb.blkpre_s = reinterpret_cast<uint32_t*>(ws + L.pres);
    pb.items_s = reinterpret_cast<uint32_t*>(ws + L.items);
    pb.soff = reinterpret_cast<uint32_t*>(ws + L.soff);
    pb.nsample = reinterpret_cast<uint32_t*>(ws + L.nsample);
    pb.qblk = reinterpret_cast<uint32_t*>(ws + L.qblk);
    pb.qblk_s = pb.qblk + B;
    pb.sq = reinterpret_cast<unsigned long long*>(ws + L.sq);
    pb.su = reinterpret_cast<unsigned long long*>(ws + L.su);
    pb.fully = reinterpret_cast<uint8_t*>(ws + L.fully);
    pb.exact_only = reinterpret_cast<uint8_t*>(ws + L.exonly);
    pb.totals = dstat->totals;
    pb.status = dstat;
    pb.pool_cap = pool_cap;
    pb.capq = reinterpret_cast<uint32_t*>(ws + L.capq);
    pb.coff = reinterpret_cast<unsigned long long*>(ws + L.coff);
    float* lut = reinterpret_cast<float*>(ws + L.lut);
    float* pbase = reinterpret_cast<float*>(ws + L.pbase);
    TableSrc tsrc;
    tsrc.lut = lut;
    tsrc.w = w;
    tsrc.m = m;
    tsrc.table_words = m * IVFR_KS;
    if (split) {
        tsrc.list_term = ix->list_term;
        tsrc.pbase = pbase;
        tsrc.probe = probe;
    }
    CandLayout lay;
    lay.off = pb.coff;
    lay.capq = pb.capq;
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ws + L.cnt);
    pb.cnt = cnt;
    // Queries that keep everything get their records placed by position.  Where no such query is to be expected
    // (queries visit far more entries than the limit for keeping everything) the scans run without that path; a
    // query that keeps everything all the same then appends through its counter.
    pb.place = visit_est <= 64.0 * (double)full_limit ? 1 : 0;
    DirectPlace direct;
    if (pb.place) {
        direct.fully = pb.fully;
        direct.off = pb.soff;
    }
    float* tau = reinterpret_cast<float*>(ws + L.tau);
    uint32_t* tau_id = reinterpret_cast<uint32_t*>(ws + L.tauid);
    uint32_t* spos = reinterpret_cast<uint32_t*>(ws + L.spos);
    float* sest = reinterpret_cast<float*>(ws + L.sest);
    int32_t* sn = reinterpret_cast<int32_t*>(ws + L.sn);
    int32_t* over = reinterpret_cast<int32_t*>(ws + L.over);
    int32_t* overtot = &dstat->over_total;
    uint64_t* rkeys = reinterpret_cast<uint64_t*>(ws + L.rkeys);
    float* sref = reinterpret_cast<float*>(ws + L.sref);
    int32_t* sids = reinterpret_cast<int32_t*>(ws + L.sids);
    float* lut_scale = reinterpret_cast<float*>(ws + L.lscale);
    GroupBuffers gb;
    gb.list_np = reinterpret_cast<uint32_t*>(ws + L.gnp);
    gb.gpre = reinterpret_cast<uint32_t*>(ws + L.gpre);
    gb.cur = reinterpret_cast<uint32_t*>(ws + L.gcur);
    gb.counts = dstat->counts;
    gb.unit8_pairs = reinterpret_cast<uint32_t*>(ws + L.gu8);
    gb.unit4_pairs = gb.unit8_pairs + L.n_u8;
    gb.unit_bytes = (L.n_u8 + L.n_u4) * sizeof(uint32_t);
    gb.unit2_pairs = reinterpret_cast<uint32_t*>(ws + L.gu2);
    gb.lo_pairs = reinterpret_cast<uint32_t*>(ws + L.glop);
    gb.blk8 = reinterpret_cast<uint32_t*>(ws + L.gblk8);
    gb.blk4 = reinterpret_cast<uint32_t*>(ws + L.gblk4);
    gb.blk2 = reinterpret_cast<uint32_t*>(ws + L.gblk2);
    gb.blklo = reinterpret_cast<uint32_t*>(ws + L.gblklo);
    gb.unit64_pairs = reinterpret_cast<uint32_t*>(ws + L.gu64);
    gb.blk64 = reinterpret_cast<uint32_t*>(ws + L.gblk64);
    gb.work = dstat->work;
    const float half_frac = IVFR_HALF_UNIT_FRAC;
    // Grouping the pairs by list and running four scans side by side costs about 0.15 ms per batch, which the
    // shared scans only win back when the batch streams some 10^8 codes or more (measured: even at 3.8e8 codes per
    // 1000 queries, ahead by a third at 1.3e9).  Left to itself the call shares lists from 3e8 expected codes.
    int share_mode = ix->share_lists;
    if (share_mode < 0) share_mode = (double)std::min<int64_t>(nq, B) * visit_est >= 3.0e8 ? 2 : 0;
    const bool share = share_mode >= 1 && ivfr_shared_scan_supported(ix);
    const bool share8 = share && share_mode >= 2 && ivfr_shared8h_supported(ix);
    // the matrix-core filter's error margin is derived for materialised tables: with split tables mode 3 acts as mode 2
    const bool share64 = share8 && share_mode >= 3 && ivfr_mfma_scan_supported(ix) && !split;

    // Launch shapes.  Every workgroup of a scan takes an equal share of the launch's 512-entry blocks; about 128
    // blocks per group of 256 threads (256 for the 512-thread scan of eight, 64 for the narrower kernels) balances
    // the tail against the per-group set-up.  The kernels apply that rule to the true block count on the device;
    // the host only has to launch enough workgroups, which it estimates from the share of the work each launch
    // had in the previous call (a quarter in reserve; too few only costs balance, never correctness).
    const uint32_t g_lo = (uint32_t)ix->n_cu * 8u;
    auto shape_for = [&](double est_blocks, uint32_t bpg, const uint32_t* n_dev, int n_host) -> ScanShape {
        ScanShape sh;
        sh.n_dev = n_dev;
        sh.n_host = n_host;
        sh.g_min = g_lo;
        if (ix->scan_groups > 0) {
            sh.groups = ix->scan_groups;
            sh.bpg = 0;
            return sh;
        }
        double g = 1.25 * est_blocks / (double)bpg + 8.0;
        g = g < (double)g_lo ? (double)g_lo : (g > 32768.0 ? 32768.0 : g);
        sh.groups = ((int)g + 7) & ~7;   // a multiple of the eight XCDs
        sh.bpg = bpg;
        return sh;
    };

    std::vector<EventPair> events;
    size_t ev_used = 0;   // events of the index's pool taken by this call
    auto mark_on = [&](int kind, bool begin, hipStream_t s) -> int {
        const bool is_scan = kind == IVFR_STAGE_SCAN || kind == IVFR_STAGE_SCAN_SHARED ||
                             kind == IVFR_STAGE_SCAN_SHARED2 || kind == IVFR_STAGE_SCAN_SHARED8 ||
                             kind == IVFR_STAGE_SCAN_SHARED64;
        if (fixed || ix->profiling == 0 || (ix->profiling == 1 && !is_scan)) return IVFR_OK;
        if (begin) {
            while (ix->prof_events.size() < ev_used + 2) {
                hipEvent_t e = nullptr;
                IVFR_HIP(hipEventCreate(&e));
                ix->prof_events.push_back(e);
            }
            EventPair ep;
            ep.kind = kind;
            ep.a = ix->prof_events[ev_used];
            ep.b = ix->prof_events[ev_used + 1];
            ev_used += 2;
            IVFR_HIP(hipEventRecord(ep.a, s));
            events.push_back(ep);
        } else {   // closes the most recent pair of this kind (stages on different streams interleave)
            for (size_t i = events.size(); i-- > 0;)
                if (events[i].kind == kind) { IVFR_HIP(hipEventRecord(events[i].b, s)); break; }
        }
        return IVFR_OK;
    };
    auto mark = [&](int kind, bool begin) -> int { return mark_on(kind, begin, st); };

    // Re-rank, final top-k and the optional trace outputs of the batch that starts at query q0.
    auto finish = [&](int64_t q0, int nb) -> int {
        const float* X = queries + q0 * d;
        const int Pb = nb * w;
        IVFR_TRY(mark(IVFR_STAGE_RERANK, true));
        IVFR_TRY(ivfr_launch_rerank(ix, X, 0, nb, kprime, spos, sn, rkeys, sref, sids, st));
        IVFR_TRY(mark(IVFR_STAGE_RERANK, false));
        IVFR_TRY(mark(IVFR_STAGE_FINAL, true));
        {
            SelectArgs a;
            a.nseg = nb; a.K = k; a.keys = rkeys; a.seg_stride = kprime;
            IVFR_TRY(ivfr_launch_select_sorted(a, sn, 0, ids_out + q0 * k, dist_out + q0 * k, st));
        }
        IVFR_TRY(mark(IVFR_STAGE_FINAL, false));
        if (probe_out) IVFR_HIP(hipMemcpyAsync(probe_out + q0 * w, probe, (size_t)Pb * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        if (probe_dist_out) IVFR_HIP(hipMemcpyAsync(probe_dist_out + q0 * w, probed, (size_t)Pb * sizeof(float), hipMemcpyDeviceToDevice, st));
        const size_t sk = (size_t)nb * kprime;
        if (short_ids_out) IVFR_HIP(hipMemcpyAsync(short_ids_out + q0 * kprime, sids, sk * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        if (short_ref_out) IVFR_HIP(hipMemcpyAsync(short_ref_out + q0 * kprime, sref, sk * sizeof(float), hipMemcpyDeviceToDevice, st));
        if (short_est_out) IVFR_HIP(hipMemcpyAsync(short_est_out + q0 * kprime, sest, sk * sizeof(float), hipMemcpyDeviceToDevice, st));
        if (short_count_out) IVFR_HIP(hipMemcpyAsync(short_count_out + q0, sn, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
        return IVFR_OK;
    };

    // Everything of one batch, enqueued on st (and, for the smaller scan launches, on the side streams); its status
    // words end up in pinned slot `slot`.
    auto enqueue_batch = [&](int64_t q0, int nb, int slot) -> int {
        const int Pb = nb * w;
        const float* X = queries + q0 * d;
        hipLaunchKernelGGL(batch_reset_kernel, dim3(64), dim3(256), 0, st, reinterpret_cast<uint32_t*>(ws + L.status),
                           L.zero_words, gb.unit8_pairs, share ? gb.unit_bytes / 4 : (size_t)0, tau, nb);
        // visited lists: the w nearest coarse centroids
        IVFR_TRY(mark(IVFR_STAGE_COARSE, true));
        IVFR_TRY(ivfr_launch_row_norms(X, nb, d, xnorm, st, &dstat->bad_query));
        IVFR_TRY(ivfr_launch_dist_keys(X, xnorm, nb, ix->coarse, ix->coarse_norm, c, d, ckeys, st));
        IVFR_TRY(mark(IVFR_STAGE_COARSE, false));
        IVFR_TRY(mark(IVFR_STAGE_PROBE, true));
        {
            SelectArgs a;
            a.nseg = nb; a.K = w; a.keys = ckeys; a.seg_stride = c; a.fixed_count = c;
            IVFR_TRY(ivfr_launch_select_sorted(a, nullptr, 0, probe, probed, st));
        }
        IVFR_TRY(ivfr_launch_plan(ix, probe, nb, w, full_limit, stride_k, min_cap, IVFR_MAX_SAMPLE, kprime, half_frac, pb, st));
        if (share) {
            // The grouping of the pairs by list (four small kernels, mostly latency) is needed by the shared scans
            // only: it runs on a side stream beside the table kernel, the sample and the bound.
            IVFR_HIP(hipEventRecord(ix->ev_group[slot][0], st));
            IVFR_HIP(hipStreamWaitEvent(ix->side[0], ix->ev_group[slot][0], 0));
            IVFR_TRY(ivfr_launch_group_plan(probe, Pb, w, c, pb.exact_only, share8, share64, pb.len, gb, ix->side[0]));
            IVFR_HIP(hipEventRecord(ix->ev_group[slot][1], ix->side[0]));
        }
        IVFR_TRY(mark(IVFR_STAGE_PROBE, false));
        IVFR_TRY(mark(IVFR_STAGE_LUT, true));
        if (split) IVFR_TRY(ivfr_launch_query_terms(ix, X, probe, nb, w, lut, pbase, lut_scale, st));
        else IVFR_TRY(ivfr_launch_lut(ix, X, probe, nb, w, lut, lut_scale, st));
        IVFR_TRY(mark(IVFR_STAGE_LUT, false));
        // uniform sample of the visited entries -> bound tau on the k'-th smallest estimate (a query without a
        // sample keeps tau = +inf)
        IVFR_TRY(mark(IVFR_STAGE_SAMPLE, true));
        {
            // chunks the sample can have at most; a batch whose queries are expected to keep everything (no sample)
            // gets a small grid, whose wavefronts would still walk over whatever chunks there are
            const bool expect_sample = 1.5 * visit_est > (double)full_limit;
            const size_t max_items = expect_sample
                ? (size_t)Pb + (size_t)nb * ((IVFR_MAX_SAMPLE + (size_t)w) / IVFR_SAMPLE_CHUNK + 1) : (size_t)ix->n_cu * 4;
            IVFR_TRY(ivfr_launch_sample_scan(ix, tsrc, pb.pair_start, pb.len_s, pb.blkpre_s, pb.items_s,
                                             &dstat->n_sample_chunks, max_items, pb.soff, w, cand, lay, st));
            // the sample of query q is nsample[q] bare estimates at the start of its buffer
            SelectArgs a;
            a.nseg = nb; a.K = kprime; a.recs = cand; a.ids = reinterpret_cast<const int32_t*>(ix->rec); a.id_stride = (uint32_t)(ix->rec_stride / 4); a.counts = pb.nsample; a.lay = lay;
            IVFR_TRY(ivfr_launch_select_tau(a, pb.su, kprime, 0, pb.fully, tau, nullptr, st, true, !expect_sample));
        }
        IVFR_TRY(mark(IVFR_STAGE_SAMPLE, false));
        // scan of every visited entry, keeping estimates <= tau
        const double est_codes = (double)nb * visit_est;
        if (share) {
            // lists visited by several queries: eight, four or two queries per pass over the list; the rest pair
            // by pair.  The launches are independent (they append to the same buffers through atomics), so the
            // small ones go to side streams and fill the large one's tail.
            const double* r = ix->work_ratio;
            const ScanShape s8 = shape_for(r[0] * est_codes / 8.0 / IVFR_BLOCK + Pb / 8.0, 256, &dstat->counts[0], 0);
            const ScanShape s4 = shape_for(r[1] * est_codes / 4.0 / IVFR_BLOCK + Pb / 4.0, 128, &dstat->counts[1], 0);
            const ScanShape s2 = shape_for(r[2] * est_codes / 2.0 / IVFR_BLOCK + c, 64, &dstat->counts[2], 0);
            const ScanShape s1 = shape_for(r[3] * est_codes / IVFR_BLOCK + c, 64, &dstat->counts[3], 0);
            ScanShape s64;
            s64.n_dev = &dstat->counts[4];
            // one workgroup of eight wavefronts per compute unit at most; at least four blocks per wavefront
            s64.groups = ix->scan_groups > 0 ? std::min(ix->n_cu, (std::max(ix->scan_groups, 8) + 7) & ~7) : (ix->n_cu & ~7);
            s64.bpg = ix->scan_groups > 0 ? 0u : 32u;
            s64.g_min = 8;
            const int n_side = share64 ? 4 : 3;
            IVFR_HIP(hipStreamWaitEvent(st, ix->ev_group[slot][1], 0));   // the units are in place
            IVFR_HIP(hipEventRecord(ix->ev_fork[slot], st));
            for (int i = 0; i < n_side; ++i) IVFR_HIP(hipStreamWaitEvent(ix->side[i], ix->ev_fork[slot], 0));
            if (share64) {
                IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED64, true, ix->side[3]));
                IVFR_TRY(ivfr_launch_scan_mfma64(ix, X, probe, tsrc, lut_scale, pb.pair_start, pb.len, gb.blk64,
                                                 gb.unit64_pairs, s64, w, tau, cand, cnt, lay, ix->side[3]));
                IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED64, false, ix->side[3]));
            }
            if (share8) {
                IVFR_TRY(mark(IVFR_STAGE_SCAN_SHARED8, true));
                IVFR_TRY(ivfr_launch_scan_shared8h(ix, tsrc, lut_scale, pb.pair_start, pb.len, gb.blk8, gb.unit8_pairs, s8,
                                                   w, tau, cand, cnt, lay, st));
                IVFR_TRY(mark(IVFR_STAGE_SCAN_SHARED8, false));
            }
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED, true, ix->side[0]));
            IVFR_TRY(ivfr_launch_scan_shared(ix, 4, tsrc, pb.pair_start, pb.len, gb.blk4, gb.unit4_pairs, s4, w,
                                             tau, cand, cnt, lay, ix->side[0], share8 ? lut_scale : nullptr,
                                             share8 ? pb.exact_only : nullptr, direct));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED, false, ix->side[0]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED2, true, ix->side[1]));
            IVFR_TRY(ivfr_launch_scan_shared(ix, 2, tsrc, pb.pair_start, pb.len, gb.blk2, gb.unit2_pairs, s2, w,
                                             tau, cand, cnt, lay, ix->side[1], nullptr, nullptr, direct));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED2, false, ix->side[1]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN, true, ix->side[2]));
            IVFR_TRY(ivfr_launch_scan(ix, tsrc, pb.pair_start, pb.len, gb.blklo, gb.lo_pairs, s1, w, tau, cand, cnt,
                                      lay, ix->side[2], nullptr, direct));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN, false, ix->side[2]));
            for (int i = 0; i < n_side; ++i) {
                IVFR_HIP(hipEventRecord(ix->ev_join[slot][i], ix->side[i]));
                IVFR_HIP(hipStreamWaitEvent(st, ix->ev_join[slot][i], 0));
            }
        } else {
            const ScanShape s1 = shape_for(est_codes / IVFR_BLOCK + Pb, 64, nullptr, Pb);
            IVFR_TRY(mark(IVFR_STAGE_SCAN, true));
            IVFR_TRY(ivfr_launch_scan(ix, tsrc, pb.pair_start, pb.len, pb.blkpre, nullptr, s1, w, tau, cand, cnt, lay, st,
                                      nullptr, direct));
            IVFR_TRY(mark(IVFR_STAGE_SCAN, false));
        }
        IVFR_TRY(mark(IVFR_STAGE_SHORTLIST, true));
        {
            SelectArgs a;
            a.nseg = nb; a.K = kprime; a.recs = cand; a.ids = reinterpret_cast<const int32_t*>(ix->rec); a.id_stride = (uint32_t)(ix->rec_stride / 4); a.counts = cnt; a.lay = lay;
            IVFR_TRY(ivfr_launch_select_records(a, 0, pb.sq, spos, sest, sn, over, overtot, st));
        }
        IVFR_TRY(mark(IVFR_STAGE_SHORTLIST, false));
        // Re-rank and final top-k are enqueued before the filter's check is known; if a query failed the check it
        // is redone after the wait and they run again.
        IVFR_TRY(finish(q0, nb));
        IVFR_HIP(hipMemcpyAsync(&ix->h_slots[slot], dstat, sizeof(DevStatus), hipMemcpyDeviceToHost, st));
        return IVFR_OK;
    };

    // Queries of the batch at q0 (whose arrays are the ones in the workspace) that failed the filter's check, redone
    // one at a time.  The launches take slices of the batch's arrays: the query's w pairs, their block prefix, its
    // counter, bound and buffer.
    auto redo_failed = [&](int64_t q0, int nb) -> int {
        // pinned read-back area: [0] count, [1] capacity, [2] still over, [4..5] entries visited, [16..] a run of flags
        uint32_t* h = ix->h_redo;
        const int32_t* h_flags = reinterpret_cast<const int32_t*>(h + 16);
        for (int q = 0; q < nb; ++q) {
            if (q % IVFR_REDO_CHUNK == 0) {   // the failed-check flags of the next run of queries
                const int n_run = std::min(IVFR_REDO_CHUNK, nb - q);
                IVFR_HIP(hipMemcpyAsync(h + 16, over + q, (size_t)n_run * sizeof(int32_t), hipMemcpyDeviceToHost, st));
                IVFR_HIP(hipStreamSynchronize(st));
            }
            if (!h_flags[q % IVFR_REDO_CHUNK]) continue;
            IVFR_HIP(hipMemcpyAsync(h + 4, pb.sq + q, sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
            IVFR_HIP(hipStreamSynchronize(st));
            unsigned long long sq_q = 0;
            memcpy(&sq_q, h + 4, sizeof(sq_q));
            ScanShape sq_shape;
            sq_shape.n_host = w;
            sq_shape.g_min = g_lo;
            if (ix->scan_groups > 0) {
                sq_shape.groups = ix->scan_groups;
            } else {
                double g = (double)sq_q / (double)IVFR_BLOCK / 64.0;
                g = g < (double)g_lo ? (double)g_lo : (g > 32768.0 ? 32768.0 : g);
                sq_shape.groups = ((int)g + 7) & ~7;
            }
            const TableSrc q_lut = tsrc.slice((int64_t)q * w);
            const uint32_t* q_start = pb.pair_start + (size_t)q * w;
            const uint32_t* q_len = pb.len + (size_t)q * w;
            const uint32_t* q_pre = pb.blkpre + (size_t)q * w;   // w + 1 values of the batch-wide block prefix
            // Too many survivors: the k'-th smallest key (estimate, id) of the records that were kept (a subset
            // of the visited entries with at least k' members) is a valid and tighter bound; rescan this query
            // with it.  The id in the bound lets it cut through any number of equal estimates.
            IVFR_HIP(hipMemcpyAsync(&h[0], cnt + q, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
            IVFR_HIP(hipMemcpyAsync(&h[1], pb.capq + q, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
            IVFR_HIP(hipStreamSynchronize(st));
            uint32_t h_cnt = h[0];
            const uint32_t h_cap = h[1];
            CandLayout qlay;
            qlay.off = pb.coff + q;
            qlay.capq = pb.capq + q;
            bool settled = false;
            for (int tries = 0; tries < 8 && h_cnt > h_cap && h_cap >= (uint32_t)kprime; ++tries) {
                ix->st_retries += 1;
                SelectArgs a;
                a.nseg = 1; a.K = kprime; a.recs = cand; a.ids = reinterpret_cast<const int32_t*>(ix->rec); a.id_stride = (uint32_t)(ix->rec_stride / 4); a.counts = cnt + q; a.lay = qlay;
                IVFR_TRY(ivfr_launch_select_tau(a, pb.sq + q, kprime, kprime, nullptr, tau + q, tau_id + q, st));
                hipLaunchKernelGGL(clear_u32_kernel, dim3(1), dim3(64), 0, st, cnt + q);
                IVFR_TRY(ivfr_launch_scan(ix, q_lut, q_start, q_len, q_pre, nullptr, sq_shape, w, tau + q, cand, cnt + q,
                                          qlay, st, tau_id + q));
                IVFR_TRY(ivfr_launch_select_records(a, q, pb.sq + q, spos, sest, sn, over, nullptr, st));
                const uint32_t before = h_cnt;
                IVFR_HIP(hipMemcpyAsync(&h[0], cnt + q, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
                IVFR_HIP(hipMemcpyAsync(&h[2], over + q, sizeof(int32_t), hipMemcpyDeviceToHost, st));
                IVFR_HIP(hipStreamSynchronize(st));
                h_cnt = h[0];
                if (!h[2]) { settled = true; break; }
                if (h_cnt >= before) break;   // no progress
            }
            if (settled) continue;
            // last resort: a buffer for every visited entry, no filter
            ix->st_dense += 1;
            const uint64_t sqv = sq_q;
            IVFR_REQUIRE(sqv < 0xFFFFFFF0ull, "a query visits more than 2^32 entries");
            const size_t bytes = (size_t)(sqv + 64) * sizeof(uint2) + 1024;
            if (fixed && bytes > ix->dense_ws.bytes) {
                ivfr_set_error("query %lld needs an unfiltered pass over %llu entries, which the fixed workspace cannot hold; "
                               "use ivfr_search", (long long)(q0 + q), (unsigned long long)sqv);
                return IVFR_ERR_OOM;
            }
            if (bytes > ix->dense_ws.bytes) {
                IVFR_TRY(ivfr_check_room(ix, bytes));
                IVFR_HIP(hipStreamSynchronize(st));   // the previous query's pass may still read the buffer
                IVFR_TRY(ix->dense_ws.reserve(bytes));
            }
            uint32_t* dcnt = ix->dense_ws.as<uint32_t>();
            float* dtau = reinterpret_cast<float*>(ix->dense_ws.as<char>() + 256);
            uint2* dcand = reinterpret_cast<uint2*>(ix->dense_ws.as<char>() + 1024);
            hipLaunchKernelGGL(dense_reset_kernel, dim3(1), dim3(64), 0, st, dcnt, dtau);
            // pair r of this launch is pair q*w + r of the batch; with w pairs and divisor w the
            // kernel's query index is 0, so tau / counter / buffer are the dense ones
            CandLayout dlay;
            dlay.stride = 0;
            dlay.ucap = (uint32_t)(sqv + 1);
            IVFR_TRY(ivfr_launch_scan(ix, q_lut, q_start, q_len, q_pre, nullptr, sq_shape, w, dtau, dcand, dcnt, dlay, st));
            SelectArgs a;
            a.nseg = 1; a.K = kprime; a.recs = dcand; a.ids = reinterpret_cast<const int32_t*>(ix->rec); a.id_stride = (uint32_t)(ix->rec_stride / 4); a.counts = dcnt; a.lay = dlay;
            IVFR_TRY(ivfr_launch_select_records(a, q, nullptr, spos, sest, sn, nullptr, nullptr, st));
        }
        IVFR_TRY(finish(q0, nb));
        IVFR_HIP(hipStreamSynchronize(st));
        return IVFR_OK;
    };

    // Status of a finished batch: statistics, and whatever has to be run again.  in_ws: the workspace still holds
    // this batch's arrays (it was the last one enqueued).
    double ratio_acc[5] = {0, 0, 0, 0, 0};
    double ratio_den = 0;
    auto settle_batch = [&](int64_t q0, int nb, int slot, bool in_ws) -> int {
        DevStatus* s = &ix->h_slots[slot];
        if (s->bad_query != 0) {
            ivfr_set_error("query %lld has a component that is not finite (or a squared norm beyond fp32)",
                           (long long)(q0 + s->bad_query - 1));
            return IVFR_ERR_INVALID_ARG;
        }
        if (s->pool_short) {
            if (fixed) {
                ivfr_set_error("the fixed workspace of %zu bytes holds %llu candidate records, this batch wants %llu; "
                               "use ivfr_search", fixed_bytes, pool_cap, s->totals[1]);
                return IVFR_ERR_OOM;
            }
            const size_t pool_bytes = (size_t)(s->totals[1] + s->totals[1] / 8 + 64) * sizeof(uint2);
            IVFR_TRY(ivfr_check_room(ix, pool_bytes));
            IVFR_TRY(ix->cand_ws.reserve(pool_bytes));   // the stream is idle: nothing reads the old pool
            cand = ix->cand_ws.as<uint2>();
            pool_cap = ix->cand_ws.bytes / sizeof(uint2) - 64;
            pb.pool_cap = pool_cap;
            ix->st_reruns += 1;
            IVFR_TRY(enqueue_batch(q0, nb, slot));
            IVFR_HIP(hipStreamSynchronize(st));
            in_ws = true;
            if (s->pool_short) { ivfr_set_error("internal: candidate pool still too small after growing"); return IVFR_ERR_STATE; }
        }
        if (s->over_total > 0) {
            if (!in_ws) {   // a later batch has reused the workspace: bring this one back
                ix->st_reruns += 1;
                IVFR_TRY(enqueue_batch(q0, nb, slot));
                IVFR_HIP(hipStreamSynchronize(st));
            }
            IVFR_TRY(redo_failed(q0, nb));
        }
        ix->st_codes += (int64_t)s->totals[0];
        ix->st_pairs += (int64_t)nb * w;
        if (share) {
            ix->st_streamed += (int64_t)s->work[0];
            ix->st_shared8_codes += (int64_t)s->work[1];
            ix->st_shared_codes += (int64_t)s->work[2];
            ix->st_shared2_codes += (int64_t)s->work[3];
            ix->st_shared64_codes += (int64_t)s->work[5];
            for (int i = 0; i < 5; ++i) ratio_acc[i] += (double)s->work[1 + i];
            ratio_den += (double)nb * visit_est;
        } else {
            ix->st_streamed += (int64_t)s->totals[0];
        }
        return IVFR_OK;
    };

    // Batches are enqueued back to back, up to IVFR_STATUS_SLOTS between two host waits.
    typedef std::chrono::steady_clock Clock;
    auto ms_since = [](Clock::time_point t0) { return std::chrono::duration<double, std::milli>(Clock::now() - t0).count(); };
    for (int64_t g0 = 0; g0 < nq; g0 += (int64_t)B * IVFR_STATUS_SLOTS) {
        int n_in_flight = 0;
        Clock::time_point t0 = Clock::now();
        for (int64_t q0 = g0; q0 < nq && n_in_flight < IVFR_STATUS_SLOTS; q0 += B, ++n_in_flight)
            IVFR_TRY(enqueue_batch(q0, (int)std::min<int64_t>(B, nq - q0), n_in_flight));
        ix->prof_ms[IVFR_STAGE_HOST_ENQUEUE] += ms_since(t0);
        t0 = Clock::now();
        IVFR_HIP(hipStreamSynchronize(st));
        ix->prof_ms[IVFR_STAGE_HOST_WAIT] += ms_since(t0);
        bool ws_valid = true;   // the workspace holds the last batch enqueued until a batch is run again
        for (int i = 0; i < n_in_flight; ++i) {
            const int64_t q0 = g0 + (int64_t)i * B;
            const int nb = (int)std::min<int64_t>(B, nq - q0);
            const bool in_ws = ws_valid && i == n_in_flight - 1;
            const bool rerun = ix->h_slots[i].pool_short || (ix->h_slots[i].over_total > 0 && !in_ws);
            IVFR_TRY(settle_batch(q0, nb, i, in_ws));
            if (rerun) ws_valid = false;
        }
    }
    if (share && ratio_den > 0) {
        ix->work_ratio[0] = ratio_acc[0] / ratio_den;   // units of eight
        ix->work_ratio[1] = ratio_acc[1] / ratio_den;   // units of four
        ix->work_ratio[2] = ratio_acc[2] / ratio_den;   // units of two
        ix->work_ratio[3] = ratio_acc[3] / ratio_den;   // single pairs
        ix->work_ratio[4] = ratio_acc[4] / ratio_den;   // units of 64
    }
    for (auto& ep : events) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ep.a, ep.b) == hipSuccess) {
            ix->prof_ms[ep.kind] += ms;
            if (ep.kind == IVFR_STAGE_SCAN || ep.kind == IVFR_STAGE_SCAN_SHARED || ep.kind == IVFR_STAGE_SCAN_SHARED2 ||
                ep.kind == IVFR_STAGE_SCAN_SHARED8 || ep.kind == IVFR_STAGE_SCAN_SHARED64)
                ix->prof_scan_launches += 1;
        }
    }
    return IVFR_OK;
}

extern "C" int ivfr_search_trace(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime,
                                 int32_t k, int32_t* ids_out, float* dist_out, int32_t* probe_out,
                                 float* probe_dist_out, int32_t* short_ids_out, float* short_est_out,
                                 float* short_ref_out, int32_t* short_count_out, void* stream) {
    return run_search(ix, queries, nq, w, kprime, k, ids_out, dist_out, probe_out, probe_dist_out, short_ids_out,
                      short_est_out, short_ref_out, short_count_out, stream, nullptr, 0);
}

extern "C" int ivfr_search(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                           int32_t* ids_out, float* dist_out, void* stream) {
    return run_search(ix, queries, nq, w, kprime, k, ids_out, dist_out, nullptr, nullptr, nullptr, nullptr, nullptr,
                      nullptr, stream, nullptr, 0);
}

extern "C" int ivfr_search_static(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime,
                                  int32_t k, int32_t* ids_out, float* dist_out, void* stream) {
    IVFR_REQUIRE(ix, "ivfr_search_static: null index");
    if (!ix->static_ws) { ivfr_set_error("ivfr_search_static: the static workspace is not available on this device"); return IVFR_ERR_STATE; }
    return run_search(ix, queries, nq, w, kprime, k, ids_out, dist_out, nullptr, nullptr, nullptr, nullptr, nullptr,
                      nullptr, stream, ix->static_ws, (size_t)IVFR_STATIC_SCRATCH_BYTES);
}
