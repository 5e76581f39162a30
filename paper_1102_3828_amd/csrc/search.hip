// Query stage (section 3.2 steps 1-3 on the inverted file of section 3.3): host orchestration.
//
// Per internal batch of queries:
//   coarse distances (MFMA) -> w nearest lists -> plan of (query, list) pairs, grouped by list into
//   units of queries that share a pass -> look-up tables (MFMA) -> sample of the visited entries
//   (the same leading fraction of every visited list) -> per-query bound tau on the k'-th smallest
//   estimate -> scan of every visited entry keeping estimates <= tau (four launches side by side:
//   units of eight, four, two queries and single pairs; in sharing mode 3 a fifth for units of 64 on
//   the matrix cores) -> exact k' smallest of the survivors -> re-rank -> k smallest.
// Queries with a component that is not finite are refused after the tables are built (their norms
// are checked on the device; the flag comes back with the plan's sizes).
// The host waits twice per batch: for the plan's sizes (candidate pool, launch shapes) and at the end.
// tau is a statistical bound (the r-th smallest sampled estimate, r chosen five standard
// deviations above the expected number of true k'-best entries in the sample), so the scan
// verifies it by counting: a query whose survivors overflow its candidate buffer is rescanned
// with a tightened key bound, one that kept fewer than k' is redone through a buffer that holds
// every visited entry.  Results are therefore exact whatever the sample says; the bound only
// decides how much is written.
#include "ivfr_internal.h"

#include <algorithm>
#include <string.h>

int ivfr_launch_select_records(const SelectArgs& a, int out_base, const unsigned long long* sq, uint32_t* out_pos,
                               float* out_est, int32_t* out_n, int32_t* overflow, int32_t* overflow_total,
                               hipStream_t st);
int ivfr_launch_select_sorted(const SelectArgs& a, const int32_t* counts_i32, int out_base, int32_t* out_lo,
                              float* out_hi, hipStream_t st);
int ivfr_launch_rerank(const ivfr_index* ix, const float* queries, int q_base, int nq, int kprime,
                       const uint32_t* short_pos, const int32_t* short_n, uint64_t* keys, float* refined_out,
                       int32_t* ids_out, hipStream_t st);

// Start of a batch: clear the counters (one contiguous block), mark every unit slot empty, tau = +inf.
__global__ __launch_bounds__(256) void batch_reset_kernel(uint32_t* zero, size_t zero_words, uint32_t* ones,
                                                          size_t ones_words, float* tau, int nb) {
    const size_t i0 = (size_t)blockIdx.x * 256 + threadIdx.x, stride = (size_t)gridDim.x * 256;
    for (size_t i = i0; i < zero_words; i += stride) zero[i] = 0u;
    for (size_t i = i0; i < ones_words; i += stride) ones[i] = 0xFFFFFFFFu;
    for (size_t i = i0; i < (size_t)nb; i += stride) tau[i] = INFINITY;
}

__global__ void fill_f32_kernel(float* p, int64_t n, float v) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

struct Carver {
    size_t off = 0;
    template <class T> size_t take(size_t count) {
        size_t a = (off + 255) / 256 * 256;
        off = a + count * sizeof(T);
        return a;
    }
};

namespace {
struct EventPair {
    hipEvent_t a = nullptr, b = nullptr;
    int kind = 0;   // IVFR_STAGE_*
};
}

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

extern "C" int ivfr_search_trace(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime,
                                 int32_t k, int32_t* ids_out, float* dist_out, int32_t* probe_out,
                                 float* probe_dist_out, int32_t* short_ids_out, float* short_est_out,
                                 float* short_ref_out, int32_t* short_count_out, void* stream) {
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
    if (nq == 0) return IVFR_OK;

    const int d = p.d, c = p.c, m = p.m;
    // queries per internal batch: the tuning value, lowered so that the per-batch tables (w m KB per query) stay
    // below 8 GiB, the coarse keys (8 c bytes) and the short-list arrays (24 k' bytes) below 4 GiB each; a call that
    // needs several batches gets equal ones (the more queries share a batch, the more they share list reads)
    int64_t B64 = std::min<int64_t>(nq, ix->batch);
    {
        const int64_t budget = 4ll << 30;
        B64 = std::min<int64_t>(B64, std::max<int64_t>(1, 2 * budget / ((int64_t)w * p.m * IVFR_KS * 4)));
        B64 = std::min<int64_t>(B64, std::max<int64_t>(1, budget / ((int64_t)kprime * 24)));
        B64 = std::min<int64_t>(B64, std::max<int64_t>(1, budget / ((int64_t)p.c * 8)));
    }
    {
        const int64_t n_batches = (nq + B64 - 1) / B64;
        B64 = (nq + n_batches - 1) / n_batches;
    }
    const int B = (int)B64;
    const int P = B * w;
    // Queries visiting no more than full_limit entries keep them all; the others get a candidate
    // buffer for the larger of their sample and min_cap survivors (sized per query by the plan).
    const uint32_t min_cap = (uint32_t)std::max<int64_t>((int64_t)ix->cap_mult * kprime, ix->min_cap);
    const uint32_t full_limit = (uint32_t)std::min<int64_t>((int64_t)ix->full_mult * kprime, 1ll << 30);
    const uint32_t stride_k = (uint32_t)std::max(1, kprime / IVFR_SAMPLE_MU);
    // Workgroups per scan launch: every group takes an equal share of the launch's 512-entry blocks.  About
    // 128 blocks per group of 256 threads (256 for the 512-thread scan of eight, 64 for the narrower kernels)
    // balances the tail against the per-group set-up.
    auto pick_groups = [&](double entries, int blocks_per_group) -> int {
        if (ix->scan_groups > 0) return ix->scan_groups;
        double g = entries / (double)IVFR_BLOCK / blocks_per_group;
        const double lo = ix->n_cu * 8.0, hi = 32768.0;
        return ((int)(g < lo ? lo : (g > hi ? hi : g)) + 7) & ~7;   // a multiple of the eight XCDs
    };
    const int groups = ix->scan_groups > 0 ? ix->scan_groups : ix->n_cu * 8;   // launches whose work is not known yet

    // carve the workspace
    Carver cv;
    const size_t o_xnorm = cv.take<float>(B);
    const size_t o_ckeys = cv.take<uint64_t>((size_t)B * c);
    const size_t o_probe = cv.take<int32_t>(P);
    const size_t o_probed = cv.take<float>(P);
    const size_t o_pstart = cv.take<uint32_t>(P);
    const size_t o_len = cv.take<uint32_t>(P);
    const size_t o_pre = cv.take<uint32_t>((size_t)P + 1);
    const size_t o_lens = cv.take<uint32_t>(P);
    const size_t o_pres = cv.take<uint32_t>((size_t)P + 1);
    // chunks of the sample: at most one partial chunk per pair plus the full ones of IVFR_MAX_SAMPLE + w entries
    const size_t n_items_max = (size_t)P + (size_t)B * ((IVFR_MAX_SAMPLE + (size_t)w) / IVFR_SAMPLE_CHUNK + 1);
    const size_t o_items = cv.take<uint32_t>(n_items_max);
    const size_t o_soff = cv.take<uint32_t>(P);
    const size_t o_nsample = cv.take<uint32_t>(B);
    const size_t o_qblk = cv.take<uint32_t>(2 * (size_t)B);
    const size_t o_sq = cv.take<unsigned long long>(B);
    const size_t o_fully = cv.take<uint8_t>(B);
    const size_t o_exonly = cv.take<uint8_t>(B);
    const size_t o_capq = cv.take<uint32_t>(B);
    const size_t o_coff = cv.take<unsigned long long>(B);
    const size_t o_lut = cv.take<float>((size_t)P * m * IVFR_KS);
    const size_t o_tau = cv.take<float>(B);
    const size_t o_tauid = cv.take<uint32_t>(B);
    const size_t o_spos = cv.take<uint32_t>((size_t)B * kprime);
    const size_t o_sest = cv.take<float>((size_t)B * kprime);
    const size_t o_sn = cv.take<int32_t>(B);
    const size_t o_over = cv.take<int32_t>(B);
    const size_t o_rkeys = cv.take<uint64_t>((size_t)B * kprime);
    const size_t o_sref = cv.take<float>((size_t)B * kprime);
    const size_t o_sids = cv.take<int32_t>((size_t)B * kprime);
    const size_t o_dpre = cv.take<uint32_t>((size_t)w + 1);
    const size_t o_lscale = cv.take<float>(P);
    const size_t o_gpre = cv.take<uint32_t>(5 * (size_t)c);
    const size_t o_gcur = cv.take<uint32_t>(2 * (size_t)c);
    const size_t o_gcounts = cv.take<uint32_t>(8);
    // units of eight: at most P/8 + c (one more per list for a remainder of 5..7); units of four likewise
    const size_t n_u8 = ((size_t)P / 8 + c + 1) * 8, n_u4 = ((size_t)P / 4 + c + 1) * 4;
    const size_t o_gu8 = cv.take<uint32_t>(n_u8 + n_u4);
    const size_t o_gu2 = cv.take<uint32_t>(2 * (size_t)c + 4);
    const size_t o_glop = cv.take<uint32_t>((size_t)c + 4);
    const size_t o_gblk8 = cv.take<uint32_t>((size_t)P / 8 + c + 2);
    const size_t o_gblk4 = cv.take<uint32_t>((size_t)P / 4 + c + 2);
    const size_t o_gblk2 = cv.take<uint32_t>((size_t)c + 2);
    const size_t o_gblklo = cv.take<uint32_t>((size_t)c + 2);
    const size_t o_gu64 = cv.take<uint32_t>(((size_t)P / 64 + 1) * 64);   // units of 64 are always full
    const size_t o_gblk64 = cv.take<uint32_t>((size_t)P / 64 + 2);
    // cleared by one kernel at the start of every batch: plan totals, unit work totals, failed-filter count,
    // candidate counters, pairs per list
    const size_t o_totals = cv.take<unsigned long long>(2);
    const size_t o_gwork = cv.take<unsigned long long>(8);
    const size_t o_overtot = cv.take<int32_t>(4);
    const size_t o_cnt = cv.take<uint32_t>(B);
    const size_t o_gnp = cv.take<uint32_t>(2 * (size_t)c);
    const size_t zero_words = (cv.off - o_totals + 3) / 4;
    IVFR_TRY(ix->search_ws.reserve(cv.off + 256));
    char* ws = ix->search_ws.as<char>();
    float* xnorm = reinterpret_cast<float*>(ws + o_xnorm);
    uint64_t* ckeys = reinterpret_cast<uint64_t*>(ws + o_ckeys);
    int32_t* probe = reinterpret_cast<int32_t*>(ws + o_probe);
    float* probed = reinterpret_cast<float*>(ws + o_probed);
    PlanBuffers pb;
    pb.pair_start = reinterpret_cast<uint32_t*>(ws + o_pstart);
    pb.len = reinterpret_cast<uint32_t*>(ws + o_len);
    pb.blkpre = reinterpret_cast<uint32_t*>(ws + o_pre);
    pb.len_s = reinterpret_cast<uint32_t*>(ws + o_lens);
    pb.blkpre_s = reinterpret_cast<uint32_t*>(ws + o_pres);
    pb.items_s = reinterpret_cast<uint32_t*>(ws + o_items);
    pb.soff = reinterpret_cast<uint32_t*>(ws + o_soff);
    pb.nsample = reinterpret_cast<uint32_t*>(ws + o_nsample);
    pb.qblk = reinterpret_cast<uint32_t*>(ws + o_qblk);
    pb.qblk_s = pb.qblk + B;
    pb.sq = reinterpret_cast<unsigned long long*>(ws + o_sq);
    pb.fully = reinterpret_cast<uint8_t*>(ws + o_fully);
    pb.exact_only = reinterpret_cast<uint8_t*>(ws + o_exonly);
    pb.totals = reinterpret_cast<unsigned long long*>(ws + o_totals);
    pb.capq = reinterpret_cast<uint32_t*>(ws + o_capq);
    pb.coff = reinterpret_cast<unsigned long long*>(ws + o_coff);
    float* lut = reinterpret_cast<float*>(ws + o_lut);
    CandLayout lay;
    lay.off = pb.coff;
    lay.capq = pb.capq;
    uint32_t* cnt = reinterpret_cast<uint32_t*>(ws + o_cnt);
    float* tau = reinterpret_cast<float*>(ws + o_tau);
    uint32_t* tau_id = reinterpret_cast<uint32_t*>(ws + o_tauid);
    uint32_t* spos = reinterpret_cast<uint32_t*>(ws + o_spos);
    float* sest = reinterpret_cast<float*>(ws + o_sest);
    int32_t* sn = reinterpret_cast<int32_t*>(ws + o_sn);
    int32_t* over = reinterpret_cast<int32_t*>(ws + o_over);
    int32_t* overtot = reinterpret_cast<int32_t*>(ws + o_overtot);
    uint64_t* rkeys = reinterpret_cast<uint64_t*>(ws + o_rkeys);
    float* sref = reinterpret_cast<float*>(ws + o_sref);
    int32_t* sids = reinterpret_cast<int32_t*>(ws + o_sids);
    uint32_t* dpre = reinterpret_cast<uint32_t*>(ws + o_dpre);
    float* lut_scale = reinterpret_cast<float*>(ws + o_lscale);
    GroupBuffers gb;
    gb.list_np = reinterpret_cast<uint32_t*>(ws + o_gnp);
    gb.gpre = reinterpret_cast<uint32_t*>(ws + o_gpre);
    gb.cur = reinterpret_cast<uint32_t*>(ws + o_gcur);
    gb.counts = reinterpret_cast<uint32_t*>(ws + o_gcounts);
    gb.unit8_pairs = reinterpret_cast<uint32_t*>(ws + o_gu8);
    gb.unit4_pairs = gb.unit8_pairs + n_u8;
    gb.unit_bytes = (n_u8 + n_u4) * sizeof(uint32_t);
    gb.unit2_pairs = reinterpret_cast<uint32_t*>(ws + o_gu2);
    gb.lo_pairs = reinterpret_cast<uint32_t*>(ws + o_glop);
    gb.blk8 = reinterpret_cast<uint32_t*>(ws + o_gblk8);
    gb.blk4 = reinterpret_cast<uint32_t*>(ws + o_gblk4);
    gb.blk2 = reinterpret_cast<uint32_t*>(ws + o_gblk2);
    gb.blklo = reinterpret_cast<uint32_t*>(ws + o_gblklo);
    gb.unit64_pairs = reinterpret_cast<uint32_t*>(ws + o_gu64);
    gb.blk64 = reinterpret_cast<uint32_t*>(ws + o_gblk64);
    gb.work = reinterpret_cast<unsigned long long*>(ws + o_gwork);
    const float half_frac = IVFR_HALF_UNIT_FRAC;
    const bool share = ix->share_lists >= 1 && ivfr_shared_scan_supported(ix);
    const bool share8 = share && ix->share_lists >= 2 && ivfr_shared8h_supported(ix);
    const bool share64 = share8 && ix->share_lists >= 3 && ivfr_mfma_scan_supported(ix);

    std::vector<EventPair> events;
    size_t ev_used = 0;   // events of the index's pool taken by this call
    auto mark_on = [&](int kind, bool begin, hipStream_t s) -> int {
        const bool is_scan = kind == IVFR_STAGE_SCAN || kind == IVFR_STAGE_SCAN_SHARED ||
                             kind == IVFR_STAGE_SCAN_SHARED2 || kind == IVFR_STAGE_SCAN_SHARED8 ||
                             kind == IVFR_STAGE_SCAN_SHARED64;
        if (ix->profiling == 0 || (ix->profiling == 1 && !is_scan)) return IVFR_OK;
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
        } else {
            IVFR_HIP(hipEventRecord(events.back().b, s));
        }
        return IVFR_OK;
    };
    auto mark = [&](int kind, bool begin) -> int { return mark_on(kind, begin, st); };

    for (int64_t q0 = 0; q0 < nq; q0 += B) {
        const int nb = (int)std::min<int64_t>(B, nq - q0);
        const int Pb = nb * w;
        const float* X = queries + q0 * d;
        hipLaunchKernelGGL(batch_reset_kernel, dim3(64), dim3(256), 0, st, reinterpret_cast<uint32_t*>(ws + o_totals),
                           zero_words, gb.unit8_pairs, share ? gb.unit_bytes / 4 : (size_t)0, tau, nb);
        // visited lists: the w nearest coarse centroids
        IVFR_TRY(mark(IVFR_STAGE_COARSE, true));
        IVFR_TRY(ivfr_launch_row_norms(X, nb, d, xnorm, st, reinterpret_cast<uint32_t*>(overtot + 1)));
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
            IVFR_TRY(ivfr_launch_group_plan(probe, Pb, w, c, pb.exact_only, share8, share64, pb.len, gb, st));
            IVFR_HIP(hipMemcpyAsync(ix->h_status + 8, gb.counts, 5 * sizeof(uint32_t), hipMemcpyDeviceToHost, st));
            IVFR_HIP(hipMemcpyAsync(ix->h_status + 14, gb.work, 6 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
        }
        // the candidate pool is sized by the plan: one small read-back
        IVFR_HIP(hipMemcpyAsync(ix->h_status + 2, pb.totals, 2 * sizeof(unsigned long long), hipMemcpyDeviceToHost, st));
        IVFR_HIP(hipMemcpyAsync(ix->h_status + 6, overtot + 1, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        IVFR_HIP(hipMemcpyAsync(ix->h_status + 28, pb.blkpre_s + Pb, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
        IVFR_TRY(mark(IVFR_STAGE_PROBE, false));
        IVFR_TRY(mark(IVFR_STAGE_LUT, true));
        IVFR_TRY(ivfr_launch_lut(ix, X, probe, nb, w, lut, lut_scale, st));
        IVFR_TRY(mark(IVFR_STAGE_LUT, false));
        IVFR_HIP(hipStreamSynchronize(st));
        if (ix->h_status[6] != 0) {   // nothing after the tables has been enqueued for this batch
            ivfr_set_error("query %lld has a component that is not finite (or a squared norm beyond fp32)",
                           (long long)(q0 + ix->h_status[6] - 1));
            return IVFR_ERR_INVALID_ARG;
        }
        unsigned long long tot2[2];
        memcpy(tot2, ix->h_status + 2, sizeof(tot2));
        const uint32_t n_sample_chunks = (uint32_t)ix->h_status[28];
        ix->st_codes += (int64_t)tot2[0];
        ix->st_pairs += Pb;
        int n_unit8 = 0, n_unit4 = 0, n_unit2 = 0, n_lo = 0, n_unit64 = 0;
        int g8 = groups, g4 = groups, g2 = groups, g1 = pick_groups((double)tot2[0], 64), g64 = 8;
        if (share) {
            unsigned long long gw[6];
            memcpy(gw, ix->h_status + 14, sizeof(gw));
            n_unit8 = ix->h_status[8];
            n_unit4 = ix->h_status[9];
            n_unit2 = ix->h_status[10];
            n_lo = ix->h_status[11];
            n_unit64 = ix->h_status[12];
            // one workgroup of eight wavefronts per compute unit at most; at least four blocks per wavefront
            {
                const double blocks64 = (double)gw[5] / 64.0 / (double)IVFR_BLOCK;
                int g = (int)(blocks64 / 32.0) + 1;
                if (ix->scan_groups > 0) g = ix->scan_groups;
                g64 = std::min(ix->n_cu, (std::max(g, 8) + 7) & ~7);
            }
            ix->st_shared64_codes += (int64_t)gw[5];
            g8 = pick_groups((double)gw[1] / 8.0, 256);
            g4 = pick_groups((double)gw[2] / 4.0, 128);
            g2 = pick_groups((double)gw[3] / 2.0, 64);
            g1 = pick_groups((double)gw[4], 64);
            ix->st_streamed += (int64_t)gw[0];
            ix->st_shared8_codes += (int64_t)gw[1];
            ix->st_shared_codes += (int64_t)gw[2];
            ix->st_shared2_codes += (int64_t)gw[3];
        } else {
            ix->st_streamed += (int64_t)tot2[0];
        }
        IVFR_TRY(ix->cand_ws.reserve((size_t)(tot2[1] + 64) * sizeof(uint2)));
        uint2* cand = ix->cand_ws.as<uint2>();
        // uniform sample of the visited entries -> bound tau on the k'-th smallest estimate
        IVFR_TRY(mark(IVFR_STAGE_SAMPLE, true));
        IVFR_TRY(ivfr_launch_sample_scan(ix, lut, pb.pair_start, pb.len_s, pb.blkpre_s, pb.items_s, n_sample_chunks,
                                         pb.soff, w, cand, lay, st));
        if (n_sample_chunks > 0) {   // else every query of the batch keeps everything: tau stays +inf
            // the sample of query q is nsample[q] bare estimates at the start of its buffer
            SelectArgs a;
            a.nseg = nb; a.K = kprime; a.recs = cand; a.ids = ix->ids; a.counts = pb.nsample; a.lay = lay;
            IVFR_TRY(ivfr_launch_select_tau(a, pb.sq, kprime, 0, pb.fully, tau, nullptr, st, true));
        }
        IVFR_TRY(mark(IVFR_STAGE_SAMPLE, false));
        // scan of every visited entry, keeping estimates <= tau
        if (share) {
            // lists visited by several queries: eight, four or two queries per pass over the list; the rest pair
            // by pair.  The four launches are independent (they append to the same buffers through atomics), so
            // the three small ones go to side streams and fill the large one's tail.
            const int n_side = n_unit64 > 0 ? 4 : 3;
            IVFR_HIP(hipEventRecord(ix->ev_fork, st));
            for (int i = 0; i < n_side; ++i) IVFR_HIP(hipStreamWaitEvent(ix->side[i], ix->ev_fork, 0));
            if (n_unit64 > 0) {
                IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED64, true, ix->side[3]));
                IVFR_TRY(ivfr_launch_scan_mfma64(ix, X, probe, lut, lut_scale, pb.pair_start, pb.len, gb.blk64,
                                                 gb.unit64_pairs, n_unit64, w, tau, cand, cnt, lay, g64, ix->side[3]));
                IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED64, false, ix->side[3]));
            }
            IVFR_TRY(mark(IVFR_STAGE_SCAN_SHARED8, true));
            IVFR_TRY(ivfr_launch_scan_shared8h(ix, lut, lut_scale, pb.pair_start, pb.len, gb.blk8, gb.unit8_pairs, n_unit8,
                                               w, tau, cand, cnt, lay, g8, st));
            IVFR_TRY(mark(IVFR_STAGE_SCAN_SHARED8, false));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED, true, ix->side[0]));
            IVFR_TRY(ivfr_launch_scan_shared(ix, 4, lut, pb.pair_start, pb.len, gb.blk4, gb.unit4_pairs, n_unit4, w,
                                             tau, cand, cnt, lay, g4, ix->side[0], share8 ? lut_scale : nullptr,
                                             share8 ? pb.exact_only : nullptr));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED, false, ix->side[0]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED2, true, ix->side[1]));
            IVFR_TRY(ivfr_launch_scan_shared(ix, 2, lut, pb.pair_start, pb.len, gb.blk2, gb.unit2_pairs, n_unit2, w,
                                             tau, cand, cnt, lay, g2, ix->side[1]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN_SHARED2, false, ix->side[1]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN, true, ix->side[2]));
            IVFR_TRY(ivfr_launch_scan(ix, lut, pb.pair_start, pb.len, gb.blklo, gb.lo_pairs, n_lo, w, tau, cand, cnt,
                                      lay, g1, ix->side[2]));
            IVFR_TRY(mark_on(IVFR_STAGE_SCAN, false, ix->side[2]));
            for (int i = 0; i < n_side; ++i) {
                IVFR_HIP(hipEventRecord(ix->ev_join[i], ix->side[i]));
                IVFR_HIP(hipStreamWaitEvent(st, ix->ev_join[i], 0));
            }
        } else {
            IVFR_TRY(mark(IVFR_STAGE_SCAN, true));
            IVFR_TRY(ivfr_launch_scan(ix, lut, pb.pair_start, pb.len, pb.blkpre, nullptr, Pb, w, tau, cand, cnt, lay,
                                      g1, st));
            IVFR_TRY(mark(IVFR_STAGE_SCAN, false));
        }
        IVFR_TRY(mark(IVFR_STAGE_SHORTLIST, true));
        {
            SelectArgs a;
            a.nseg = nb; a.K = kprime; a.recs = cand; a.ids = ix->ids; a.counts = cnt; a.lay = lay;
            IVFR_TRY(ivfr_launch_select_records(a, 0, pb.sq, spos, sest, sn, over, overtot, st));
        }
        IVFR_TRY(mark(IVFR_STAGE_SHORTLIST, false));
        // Re-rank, final top-k and the optional trace outputs.  Enqueued before the filter's check is read
        // back (one host round trip less); if a query failed the check it is redone below and this runs again.
        auto finish = [&]() -> int {
            // re-rank and final top-k
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
            // optional trace outputs
            if (probe_out) IVFR_HIP(hipMemcpyAsync(probe_out + q0 * w, probe, (size_t)Pb * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            if (probe_dist_out) IVFR_HIP(hipMemcpyAsync(probe_dist_out + q0 * w, probed, (size_t)Pb * sizeof(float), hipMemcpyDeviceToDevice, st));
            const size_t sk = (size_t)nb * kprime;
            if (short_ids_out) IVFR_HIP(hipMemcpyAsync(short_ids_out + q0 * kprime, sids, sk * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            if (short_ref_out) IVFR_HIP(hipMemcpyAsync(short_ref_out + q0 * kprime, sref, sk * sizeof(float), hipMemcpyDeviceToDevice, st));
            if (short_est_out) IVFR_HIP(hipMemcpyAsync(short_est_out + q0 * kprime, sest, sk * sizeof(float), hipMemcpyDeviceToDevice, st));
            if (short_count_out) IVFR_HIP(hipMemcpyAsync(short_count_out + q0, sn, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToDevice, st));
            return IVFR_OK;
        };
        // status read-back: failed-filter count
        IVFR_HIP(hipMemcpyAsync(ix->h_status, overtot, sizeof(int32_t), hipMemcpyDeviceToHost, st));
        IVFR_TRY(finish());
        IVFR_HIP(hipStreamSynchronize(st));
        const int n_over = ix->h_status[0];
        if (n_over > 0) {
            // queries whose filter failed its check are redone one at a time
            std::vector<int32_t> h_over((size_t)nb);
            std::vector<unsigned long long> h_sq((size_t)nb);
            IVFR_HIP(hipMemcpy(h_over.data(), over, (size_t)nb * sizeof(int32_t), hipMemcpyDeviceToHost));
            IVFR_HIP(hipMemcpy(h_sq.data(), pb.sq, (size_t)nb * sizeof(unsigned long long), hipMemcpyDeviceToHost));
            for (int q = 0; q < nb; ++q) {
                if (!h_over[(size_t)q]) continue;
                // the query's w pairs; block prefix computed on the host
                std::vector<uint32_t> h_len((size_t)w), h_pre((size_t)w + 1, 0u);
                IVFR_HIP(hipMemcpy(h_len.data(), pb.len + (size_t)q * w, (size_t)w * sizeof(uint32_t), hipMemcpyDeviceToHost));
                for (int r = 0; r < w; ++r)
                    h_pre[(size_t)r + 1] = h_pre[(size_t)r] + (h_len[(size_t)r] + IVFR_BLOCK - 1) / IVFR_BLOCK;
                IVFR_HIP(hipMemcpy(dpre, h_pre.data(), ((size_t)w + 1) * sizeof(uint32_t), hipMemcpyHostToDevice));
                const int gq = pick_groups((double)h_sq[(size_t)q], 64);
                // Too many survivors: the k'-th smallest key (estimate, id) of the records that were kept (a subset
                // of the visited entries with at least k' members) is a valid and tighter bound; rescan this query
                // with it.  The id in the bound lets it cut through any number of equal estimates.
                uint32_t h_cnt = 0, h_cap = 0;
                IVFR_HIP(hipMemcpy(&h_cnt, cnt + q, sizeof(uint32_t), hipMemcpyDeviceToHost));
                IVFR_HIP(hipMemcpy(&h_cap, pb.capq + q, sizeof(uint32_t), hipMemcpyDeviceToHost));
                CandLayout qlay;
                qlay.off = pb.coff + q;
                qlay.capq = pb.capq + q;
                bool settled = false;
                for (int tries = 0; tries < 8 && h_cnt > h_cap && h_cap >= (uint32_t)kprime; ++tries) {
                    ix->st_retries += 1;
                    SelectArgs a;
                    a.nseg = 1; a.K = kprime; a.recs = cand; a.ids = ix->ids; a.counts = cnt + q; a.lay = qlay;
                    IVFR_TRY(ivfr_launch_select_tau(a, pb.sq + q, kprime, kprime, nullptr, tau + q, tau_id + q, st));
                    IVFR_HIP(hipMemsetAsync(cnt + q, 0, sizeof(uint32_t), st));
                    IVFR_TRY(ivfr_launch_scan(ix, lut + (size_t)q * w * m * IVFR_KS, pb.pair_start + (size_t)q * w,
                                              pb.len + (size_t)q * w, dpre, nullptr, w, w, tau + q, cand, cnt + q, qlay,
                                              gq, st, tau_id + q));
                    IVFR_TRY(ivfr_launch_select_records(a, q, pb.sq + q, spos, sest, sn, over, nullptr, st));
                    const uint32_t before = h_cnt;
                    int32_t still = 0;
                    IVFR_HIP(hipMemcpyAsync(&h_cnt, cnt + q, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
                    IVFR_HIP(hipMemcpyAsync(&still, over + q, sizeof(int32_t), hipMemcpyDeviceToHost, st));
                    IVFR_HIP(hipStreamSynchronize(st));
                    if (!still) { settled = true; break; }
                    if (h_cnt >= before) break;   // no progress
                }
                if (settled) continue;
                // last resort: a buffer for every visited entry, no filter
                ix->st_dense += 1;
                const uint64_t sqv = h_sq[(size_t)q];
                IVFR_REQUIRE(sqv < 0xFFFFFFF0ull, "a query visits more than 2^32 entries");
                const size_t bytes = (size_t)(sqv + 64) * sizeof(uint2) + 1024;
                IVFR_TRY(ix->dense_ws.reserve(bytes));
                uint32_t* dcnt = ix->dense_ws.as<uint32_t>();
                float* dtau = reinterpret_cast<float*>(ix->dense_ws.as<char>() + 256);
                uint2* dcand = reinterpret_cast<uint2*>(ix->dense_ws.as<char>() + 1024);
                IVFR_HIP(hipMemsetAsync(dcnt, 0, sizeof(uint32_t), st));
                hipLaunchKernelGGL(fill_f32_kernel, dim3(1), dim3(64), 0, st, dtau, (int64_t)1, INFINITY);
                // pair r of this launch is pair q*w + r of the batch; with w pairs and divisor w the
                // kernel's query index is 0, so tau / counter / buffer are the dense ones
                CandLayout dlay;
                dlay.stride = 0;
                dlay.ucap = (uint32_t)(sqv + 1);
                IVFR_TRY(ivfr_launch_scan(ix, lut + (size_t)q * w * m * IVFR_KS, pb.pair_start + (size_t)q * w,
                                          pb.len + (size_t)q * w, dpre, nullptr, w, w, dtau, dcand, dcnt, dlay, gq, st));
                SelectArgs a;
                a.nseg = 1; a.K = kprime; a.recs = dcand; a.ids = ix->ids; a.counts = dcnt; a.lay = dlay;
                IVFR_TRY(ivfr_launch_select_records(a, q, nullptr, spos, sest, sn, nullptr, nullptr, st));
            }
            IVFR_TRY(finish());
            IVFR_HIP(hipStreamSynchronize(st));
        }
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

extern "C" int ivfr_search(ivfr_index* ix, const float* queries, int64_t nq, int32_t w, int32_t kprime, int32_t k,
                           int32_t* ids_out, float* dist_out, void* stream) {
    return ivfr_search_trace(ix, queries, nq, w, kprime, k, ids_out, dist_out, nullptr, nullptr, nullptr, nullptr,
                             nullptr, nullptr, stream);
}
