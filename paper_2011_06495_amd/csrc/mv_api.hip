// Host side of the C ABI declared in include/mv.h: argument checks, scratch
// layout, and the launch sequence of one vote step (Algorithm 1 of the paper,
// error compensation .. error update).  Every step of the method runs in the
// kernels of mv_kernels.hpp; nothing is computed on the host.
#include "../../include/mv.h"
#include "mv_kernels.hpp"

#include <hip/hip_runtime.h>
#include <new>
#include <stdint.h>
#include <string.h>
#include <math.h>

namespace {

enum KernelId {
    KID_STREAM = 0,
    KID_ROW_SELECT,
    KID_ROW_VOTES,
    KID_MASK_COUNT,
    KID_GATHER,
    // add-drop voting only
    KID_AD_COLLECT,
    KID_AD_SELECT,
    KID_AD_APPLY,
    KID_AD_COMPACT_COUNT,
    KID_AD_COMPACT_EMIT,
    // rows' select with many workgroups (large K only)
    KID_SEL_HIST,
    KID_SEL_SPLIT,
    KID_SEL_RANK,
    // random selection only
    KID_RS_KEYS,
    KID_RS_HIST,
    KID_RS_SPLIT,
    KID_RS_RANK,
    KID_COUNT
};
const char* const kKernelNames[KID_COUNT] = {
    "mv_stream_collect",   "mv_row_select",      "mv_row_votes",
    "mv_mask_count",     "mv_gather_update",    "mv_ad_collect",      "mv_ad_select",
    "mv_ad_apply",       "mv_ad_compact_count", "mv_ad_compact_emit",
    "mv_sel_hist",       "mv_sel_split",       "mv_sel_rank",
    "mv_rs_keys",        "mv_rs_hist",         "mv_rs_split",         "mv_rs_rank"};

constexpr size_t kAlign = 256;
constexpr int kEventRing = 64;   // steps whose kernel durations stay readable
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Everything that follows from (N, d, K) alone.
struct Plan {
    uint32_t N, K;
    int64_t  d;
    uint32_t nseg;              // segments of 1024 coordinates per row
    uint32_t stride;            // every stride-th 32-coordinate chunk is sampled
    uint32_t n_sampled_chunks;  // per row
    uint64_t n_sampled;         // sampled coordinates per row
    uint32_t m_target;          // sampled coordinates that must lie at or above the threshold bin
    uint32_t cap;               // candidate list capacity per row
    uint32_t n_vote_blocks;     // workgroups of the mask kernels: blocks of 16384 vote_q coordinates
    uint32_t vote_q;            // quads of 16 vote bytes per thread of the mask kernels (1, 2, 3, 4, 6 or 8)
    uint32_t rs_blocks;         // workgroups of mv_rs_keys: blocks of kVoteBlock coordinates
    uint32_t list_blocks;       // workgroups per row that walk a candidate list, one thread per entry
    uint32_t vote_blocks;       // workgroups per row of mv_row_votes
    uint32_t emit_blocks;       // workgroups per row that write the sorted vote list
    uint32_t scan_parts;        // workgroups per row that scan the segment tallies (4096 segments each)
    uint32_t select_parts;      // workgroups per row of mv_row_select when they also cast the votes
    uint32_t n_spec;            // list entries per thread that mv_row_select fetches ahead of the row's count
    bool     long_lists;        // the expected lists need the instance of mv_row_select that keeps more entries
    uint32_t scan_blocks;       // workgroups per row that scan the segment tallies
    // add-drop voting (only with MV_FLAG_ADD_DROP)
    bool     add_drop;
    uint32_t nwords, nwords_pad;  // 32-bit words of a row's vote bitmap, and padded to a multiple of 4
    uint32_t cap_d;               // capacity of a row's list of removal candidates
    uint32_t bit_blocks;          // workgroups of kBitBlockWords bitmap words per row
    // rows' select with many workgroups: when about 2K candidates are far more than one workgroup keeps in registers
    bool     multi_select;
    size_t   off_selhist, off_selcount2, off_selbinwant, off_sellist2;
    // random selection
    uint32_t rs_cap;              // most coordinates that can hold a vote: min(N K, d)
    size_t   off_rshist, off_rscount, off_rsbits, off_rsblk, off_rslist, off_rslist2;
    // scratch offsets (bytes)
    uint32_t sample_wgs;        // workgroups per row that sample it (the head of the streaming kernel's grid)
    size_t off_sampledone, off_readsdone, off_taupub, off_poison, off_stepno, off_candcount;
    size_t off_hist, off_tau, off_rowcnt, off_slow, off_kth, off_tiecut, off_lvlsets, off_seg, off_segsel,
        off_segpre,
        off_blktotal, off_alist, off_dlist, off_adcount, off_adthr, off_adbits, off_adblk, off_cand, off_votes, off_blockcnt, off_subcnt, off_votethr, off_emitfail,
        off_lookback;
    uint32_t n_zero_words;      // words from off_lvlsets on that a step's first kernel zeroes
    size_t total_bytes;
};

bool config_valid(const mv_config* c)
{
    if (!c) return false;
    if (c->struct_size != sizeof(mv_config)) return false;
    if (c->n_workers < 1 || c->n_workers > 255) return false;
    if (c->d < 1 || c->d > 0x7FFFFFFFll) return false;
    if (c->k < 1 || c->k > c->d) return false;
    if (c->grad_dtype != MV_F32 && c->grad_dtype != MV_BF16) return false;
    if (c->reduce != MV_REDUCE_MEAN && c->reduce != MV_REDUCE_SUM) return false;
    if ((c->flags & ~MV_FLAG_ADD_DROP) != 0) return false;
    if (c->device < 0) return false;
    return true;
}

Plan make_plan(const mv_config* c)
{
    Plan p;
    memset(&p, 0, sizeof p);
    p.N = (uint32_t)c->n_workers;
    p.K = (uint32_t)c->k;
    p.d = c->d;
    p.nseg = (uint32_t)((p.d + mvk::kSeg - 1) / mvk::kSeg);

    // Sample about d/128 coordinates of each row, but at least ~32K when the row has them.
    const uint64_t nchunks = (uint64_t)(p.d + mvk::kChunk - 1) / mvk::kChunk;
    uint64_t want = (uint64_t)p.d / 128;
    if (want < 32768) want = 32768;
    uint64_t stride = nchunks / ((want + mvk::kChunk - 1) / mvk::kChunk);
    if (stride < 1) stride = 1;
    if (stride > 128) stride = 128;
    p.stride = (uint32_t)stride;
    p.n_sampled_chunks = (uint32_t)((nchunks + stride - 1) / stride);
    // all sampled chunks are full except possibly the row's last chunk
    p.n_sampled = (uint64_t)p.n_sampled_chunks * mvk::kChunk;
    {
        // kSampleQuads quads per thread and round; at most 16 sampling workgroups of 512 threads per row
        const uint64_t nquads = (uint64_t)p.n_sampled_chunks * (mvk::kChunk / 4);
        const uint64_t per_wg = (uint64_t)mvk::kSampleQuads * mvk::kStreamThreads;
        uint64_t bx = (nquads + per_wg - 1) / per_wg;
        if (bx > 16) bx = 16;
        if (bx < 1) bx = 1;
        p.sample_wgs = (uint32_t)bx;
    }
    if (((nchunks - 1) % stride) == 0) p.n_sampled -= (uint64_t)(nchunks * mvk::kChunk - (uint64_t)p.d);

    // A row with exactly K coordinates above the threshold shows K * frac of them in the
    // sample on average.  Ask for m sampled ones with m - 7 sqrt(m) = K * frac, never fewer
    // than 128: falling short of K is then a 7-sigma event of the sample count, and the
    // candidates exceed K by about 7 sqrt(m) / frac (a factor 2 at K = d/1000, 1.3 at d/100).
    const double frac = (double)p.n_sampled / (double)p.d;
    const double root_m = 3.5 + sqrt(12.25 + (double)p.K * frac);
    double m = ceil(root_m * root_m);
    if (m < 128.0) m = 128.0;
    m += 1.0;
    p.m_target = (m >= 4294967295.0) ? 0xFFFFFFFFu : (uint32_t)m;

    uint64_t cap = 16ull * p.K;
    if (cap < 65536) cap = 65536;
    if (cap > (uint64_t)p.d) cap = (uint64_t)p.d;
    p.cap = (uint32_t)cap;

    p.rs_blocks = (uint32_t)((p.d + mvk::kVoteBlock - 1) / mvk::kVoteBlock);
    {
        // the mask kernels: as few vote bytes per thread as keep the grid, with one more workgroup per row for
        // the segment scans, at two workgroups per compute unit: all resident at once, which the exchange of
        // counts between the blocks likes (measured: a limit of 500 beats 250 by 3 us on C4 and 13 us on C5;
        // 750 and more lose again on d = 11 M)
        static const uint32_t kQs[] = {1, 2, 3, 4, 6, 8};
        uint32_t q = 8;
        for (uint32_t cand_q : kQs)
            if ((uint64_t)p.d <= (uint64_t)(500 - (p.N < 128 ? p.N : 128)) * mvk::kMaskThreads * 16 * cand_q) {
                q = cand_q;
                break;
            }
        p.vote_q = q;
        const uint64_t per = (uint64_t)mvk::kMaskThreads * 16 * q;
        p.n_vote_blocks = (uint32_t)(((uint64_t)p.d + per - 1) / per);
    }
    // about 2K candidates per row are expected: one thread per candidate with some room, the kernels
    // stride over whatever is there
    {
        uint64_t eb = (3ull * p.K + mvk::kVoteThreads - 1) / mvk::kVoteThreads;
        const uint64_t eb_cap = ((uint64_t)p.cap + mvk::kVoteThreads - 1) / mvk::kVoteThreads;
        if (eb > eb_cap) eb = eb_cap;
        if (eb > 256) eb = 256;      // more workgroups than this only crowd the atomics (measured at K = 111,740)
        if (eb < 1) eb = 1;
        p.list_blocks = (uint32_t)eb;
    }
    p.scan_blocks = (p.nseg + 1023) / 1024;
    p.scan_parts = (p.nseg + 4095) / 4096;
    {
        // about 2K candidates are expected; fetch 3K per row ahead (never beyond the list's storage),
        // and give every workgroup of a row about four list entries per thread to cast votes for
        const uint64_t expect = (uint64_t)((double)p.m_target / frac * 1.25) + 1;   // candidates per row, with room
        uint64_t slots = (expect + mvk::kRowThreads - 1) / mvk::kRowThreads;        // list entries per thread
        const uint64_t in_cap = ((uint64_t)p.cap + mvk::kRowThreads - 1) / mvk::kRowThreads;
        if (slots > in_cap) slots = in_cap;
        if (slots < 1) slots = 1;
        p.long_lists = slots > (uint64_t)mvk::kKeepShort;
        p.n_spec = (uint32_t)(slots < (uint64_t)mvk::kSpec ? slots : (uint64_t)mvk::kSpec);
        uint64_t parts = (slots + 3) / 4;
        if (parts > 16) parts = 16;
        if (parts * p.N > 240) parts = 240 / p.N;      // all at once: with its registers a workgroup has a unit to itself
        if (parts < 1) parts = 1;
        p.select_parts = (uint32_t)parts;
        // beyond what one workgroup keeps in registers the lists go through the many-workgroup select
        p.multi_select = slots > (uint64_t)mvk::kKeepLong;
        // four list entries per thread in mv_row_votes, eight when writing the sorted lists
        uint64_t vb = (slots + 3) / 4, eb2 = (slots + 3) / 4;
        if (vb > 256) vb = 256;
        if (eb2 * p.N > 256) eb2 = 256 / p.N;
        if (eb2 < 1) eb2 = 1;
        p.vote_blocks = (uint32_t)vb;
        p.emit_blocks = (uint32_t)eb2;
    }

    size_t off = 0;
    p.off_hist = off;     off += align_up((size_t)p.N * mvk::kHistBins * 4);
    p.off_tau = off;      off += align_up((size_t)p.N * 4);
    p.off_sampledone = off; off += align_up((size_t)p.N * mvk::kCounterStride * 4);
    p.off_readsdone = off; off += align_up((size_t)p.N * mvk::kCounterStride * 4);
    p.off_taupub = off;   off += align_up((size_t)p.N * (mvk::kCounterStride / 2) * 8);
    p.off_poison = off;   off += align_up((size_t)p.N * 4);
    p.off_stepno = off;   off += align_up(4);
    p.off_candcount = off; off += align_up((size_t)p.N * 4);
    p.off_rowcnt = off;   off += 2 * align_up((size_t)p.N * mvk::kCounterStride * 4);   // one set per step parity
    p.off_slow = off;     off += align_up((size_t)p.N * 4);
    p.off_kth = off;      off += align_up((size_t)p.N * 4);
    p.off_tiecut = off;   off += align_up((size_t)p.N * 4);
    // the vote-level counters and, behind them, what mv_mask_count's blocks publish to each other (a flag word
    // and two 64-bit words per block): one stretch of words that every step's first kernel leaves at zero
    p.off_lvlsets = off;  off += (size_t)mvk::kLvlSets * 256 * 4;
    p.off_emitfail = off; off += 8;
    p.off_lookback = off; off += align_up((size_t)p.n_vote_blocks * 16);
    p.n_zero_words = (uint32_t)((off - p.off_lvlsets) / 4);
    p.off_seg = off;      off += align_up((size_t)p.N * p.nseg * 8);
    p.off_segsel = off;   off += align_up((size_t)p.N * p.nseg * 4);
    p.off_segpre = off;   off += align_up((size_t)p.N * p.nseg * 4);
    p.off_blktotal = off; off += align_up((size_t)p.N * ((p.nseg + 1023) / 1024) * 4);
    p.off_cand = off;     off += align_up((size_t)p.N * p.cap * 8);
    p.off_votes = off;    off += align_up(((size_t)p.d + 15) / 16 * 16);
    p.off_blockcnt = off; off += align_up((size_t)p.n_vote_blocks * 8);
    p.off_subcnt = off;   off += align_up((size_t)p.n_vote_blocks * (mvk::kMaskThreads / mvk::kWave) * 8);
    p.off_votethr = off;  off += align_up(2 * 4);
    p.add_drop = (c->flags & MV_FLAG_ADD_DROP) != 0;
    p.nwords = (uint32_t)((p.d + 31) / 32);
    p.nwords_pad = (p.nwords + 3) / 4 * 4;
    p.cap_d = p.K;
    p.bit_blocks = (p.nwords_pad + mvk::kBitBlockWords - 1) / mvk::kBitBlockWords;
    if (p.add_drop) {
        p.off_alist = off;   off += align_up((size_t)p.N * p.cap * 8);
        p.off_dlist = off;   off += align_up((size_t)p.N * p.cap_d * 8);
        p.off_adcount = off; off += align_up((size_t)p.N * 2 * mvk::kCounterStride * 4);
        p.off_adthr = off;   off += align_up((size_t)p.N * 4 * 4);
        p.off_adbits = off;  off += align_up((size_t)p.N * p.nwords_pad * 4);
        p.off_adblk = off;   off += align_up((size_t)p.N * p.bit_blocks * 8);
    }
    // (measured: one workgroup per row takes 20 us at 24K candidates, 38 us at 55K, 89 us at 230K; the three
    // kernels of the many-workgroup select about 40 us)
    if (p.multi_select) {
        p.off_selhist = off;    off += align_up((size_t)p.N * mvk::kSelBins * 4);
        p.off_selcount2 = off;  off += align_up((size_t)p.N * 4);
        p.off_selbinwant = off; off += align_up((size_t)p.N * 2 * 4);
        p.off_sellist2 = off;   off += align_up((size_t)p.N * p.cap * 8);
    }
    const uint64_t voted_max = (uint64_t)p.N * p.K;
    p.rs_cap = (uint32_t)(voted_max < (uint64_t)p.d ? voted_max : (uint64_t)p.d);
    p.off_rshist = off;  off += align_up((size_t)mvk::kSelBins * 4);
    p.off_rscount = off; off += align_up(4 * 4);
    p.off_rsbits = off;  off += align_up((size_t)p.nwords_pad * 4);
    p.off_rsblk = off;   off += align_up((size_t)p.bit_blocks * 8);
    p.off_rslist = off;  off += align_up((size_t)p.rs_cap * 8);
    p.off_rslist2 = off; off += align_up((size_t)p.rs_cap * 8);
    p.total_bytes = off;
    return p;
}

}  // namespace

struct mv_ctx {
    mv_config  cfg;
    Plan       plan;
    char*      ws;          // device scratch
    bool       owns_ws;
    bool       ended;
    bool       broken;      // a step's launch sequence failed: the scratch invariants no longer hold
    int32_t    profiling;
    // event pairs around kernels, a ring over the last kEventRing steps
    hipEvent_t ev[kEventRing][KID_COUNT][2];
    bool       ev_recorded[kEventRing][KID_COUNT];
    uint64_t   steps_done;
    uint32_t   spin_limit;  // polls a streaming wavefront makes for its row's threshold before it gives up
    uint32_t   head_wgs;    // streaming workgroups at the head of the grid that wait for the sampling before loading
    hipStream_t last_stream;
};

namespace {

template <typename T>
T* ws_ptr(mv_ctx* c, size_t off) { return reinterpret_cast<T*>(c->ws + off); }

struct DeviceGuard {
    int  prev;
    bool ok;
    explicit DeviceGuard(int dev) : prev(0), ok(false)
    {
        if (hipGetDevice(&prev) != hipSuccess) return;
        if (prev != dev && hipSetDevice(dev) != hipSuccess) return;
        ok = true;
    }
    ~DeviceGuard() { if (ok) (void)hipSetDevice(prev); }
};

}  // namespace

extern "C" {

size_t mv_workspace_bytes(const mv_config* cfg)
{
    if (!config_valid(cfg)) return 0;
    return make_plan(cfg).total_bytes;
}

mv_status mv_begin(const mv_config* cfg, mv_ctx** out_ctx)
{
    if (!out_ctx) return MV_ERR_INVALID_ARG;
    *out_ctx = nullptr;
    if (!config_valid(cfg)) return MV_ERR_INVALID_ARG;
    const Plan plan = make_plan(cfg);
    if (cfg->workspace) {
        if (cfg->workspace_bytes < plan.total_bytes) return MV_ERR_INVALID_ARG;
        if ((reinterpret_cast<uintptr_t>(cfg->workspace) & (kAlign - 1)) != 0) return MV_ERR_INVALID_ARG;
    }

    mv_ctx* c = new (std::nothrow) mv_ctx;
    if (!c) return MV_ERR_ALLOC;
    memset(c, 0, sizeof *c);
    c->cfg = *cfg;
    c->plan = plan;
    c->head_wgs = 2048;         // about two rounds of resident workgroups
    c->spin_limit = 1u << 20;   // of about a microsecond each; a threshold is normally there within ten

    DeviceGuard guard(cfg->device);
    if (!guard.ok) {
        delete c;
        return MV_ERR_DEVICE;
    }
    if (cfg->workspace) {
        c->ws = static_cast<char*>(cfg->workspace);
        c->owns_ws = false;
    } else {
        void* p = nullptr;
        if (hipMalloc(&p, plan.total_bytes) != hipSuccess) {
            (void)hipGetLastError();
            delete c;
            return MV_ERR_ALLOC;
        }
        c->ws = static_cast<char*>(p);
        c->owns_ws = true;
    }
    // The histogram and the packed vote words must start at zero; the kernels
    // leave them at zero after every step.
    bool ok = hipMemset(c->ws + plan.off_hist, 0, plan.off_tau - plan.off_hist) == hipSuccess &&
              hipMemset(c->ws + plan.off_votes, 0, ((size_t)plan.d + 15) / 16 * 16) == hipSuccess &&
              hipMemset(c->ws + plan.off_tau, 0, plan.off_seg - plan.off_tau) == hipSuccess;
    if (ok && plan.add_drop)   // the scratch bitmaps start at zero and are left at zero by every step
        ok = hipMemset(c->ws + plan.off_adcount, 0, plan.off_adblk - plan.off_adcount) == hipSuccess;
    if (ok && plan.multi_select)   // histograms and counters of the many-workgroup select start at zero
        ok = hipMemset(c->ws + plan.off_selhist, 0, plan.off_selbinwant - plan.off_selhist) == hipSuccess;
    // random selection: histogram, counters and bitmap start at zero and are left at zero
    ok = ok && hipMemset(c->ws + plan.off_rshist, 0, plan.off_rsblk - plan.off_rshist) == hipSuccess;
    ok = ok && hipDeviceSynchronize() == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        if (c->owns_ws) (void)hipFree(c->ws);
        delete c;
        return MV_ERR_DEVICE;
    }
    *out_ctx = c;
    return MV_OK;
}

}  // extern "C"

namespace {

// What the two step entry points pass down.
struct StepArgs {
    const void* grads; int64_t ld_g;
    float* err;        int64_t ld_e;
    uint32_t* worker_idx;
    uint8_t*  votes;
    uint32_t* mask_idx;
    float*    agg_vals;
    // add-drop voting (k_ad == 0: plain majority voting)
    int64_t   k_ad;
    uint32_t* vote_bits; int64_t ld_bits;
    uint8_t*  msum;
    uint32_t* add_idx;
    uint32_t* drop_idx;
    uint32_t* counts;
    // random selection (null: the mask is the K most voted coordinates)
    const float* rand_exp;
};

mv_status check_common(mv_ctx* c, const StepArgs& a)
{
    if (!c) return MV_ERR_INVALID_ARG;
    if (c->ended || c->broken) return MV_ERR_STATE;
    if (!a.grads || !a.err || !a.mask_idx || !a.agg_vals) return MV_ERR_INVALID_ARG;
    if (reinterpret_cast<uintptr_t>(a.rand_exp) & 3) return MV_ERR_INVALID_ARG;
    const Plan& p = c->plan;
    const bool bf16 = c->cfg.grad_dtype == MV_BF16;
    if (a.ld_g < p.d || a.ld_e < p.d) return MV_ERR_INVALID_ARG;
    if (a.ld_g % (bf16 ? 8 : 4) != 0 || a.ld_e % 4 != 0) return MV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(a.grads) & 15) || (reinterpret_cast<uintptr_t>(a.err) & 15))
        return MV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(a.mask_idx) & 3) || (reinterpret_cast<uintptr_t>(a.agg_vals) & 3) ||
        (reinterpret_cast<uintptr_t>(a.worker_idx) & 3))
        return MV_ERR_INVALID_ARG;
    return MV_OK;
}

// Enqueues one step: the part common to both voting schemes (threshold estimate,
// streaming pass, exact per-row select), then either the plain vote count or the
// add-drop update of the standing votes, then the mask and the aggregate.
mv_status enqueue_step(mv_ctx* c, const StepArgs& a, void* stream_v)
{
    const Plan& p = c->plan;
    const bool bf16 = c->cfg.grad_dtype == MV_BF16;
    const bool add_drop = a.k_ad > 0;
    const bool random_sel = a.rand_exp != nullptr;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return MV_ERR_DEVICE;
    // an error the caller left pending is not this step's: nothing is enqueued and the context stays usable
    if (hipPeekAtLastError() != hipSuccess) return MV_ERR_DEVICE;
    hipStream_t st = static_cast<hipStream_t>(stream_v);

    uint32_t* hist = ws_ptr<uint32_t>(c, p.off_hist);
    uint32_t* tau = ws_ptr<uint32_t>(c, p.off_tau);
    // the rows' candidate counters while the streaming pass runs (two sets, used in turn; the step's
    // number on the device says which), and the counts as mv_row_select leaves them for everyone after it
    const uint32_t rowcnt_set_words = (uint32_t)(align_up((size_t)p.N * mvk::kCounterStride * 4) / 4);
    uint32_t* rowcnt_sets = ws_ptr<uint32_t>(c, p.off_rowcnt);
    uint32_t* stepno = ws_ptr<uint32_t>(c, p.off_stepno);
    uint32_t* rowcnt = ws_ptr<uint32_t>(c, p.off_candcount);
    uint32_t* slow = ws_ptr<uint32_t>(c, p.off_slow);
    uint32_t* lvlsets = ws_ptr<uint32_t>(c, p.off_lvlsets);
    uint32_t* kth = ws_ptr<uint32_t>(c, p.off_kth);
    uint32_t* tiecut = ws_ptr<uint32_t>(c, p.off_tiecut);
    uint32_t* segsel = ws_ptr<uint32_t>(c, p.off_segsel);
    uint32_t* segpre = ws_ptr<uint32_t>(c, p.off_segpre);
    uint32_t* blktotal = ws_ptr<uint32_t>(c, p.off_blktotal);
    mvk::u32x2* seg = ws_ptr<mvk::u32x2>(c, p.off_seg);
    mvk::u32x2* cand = ws_ptr<mvk::u32x2>(c, p.off_cand);
    uint32_t* votes32 = ws_ptr<uint32_t>(c, p.off_votes);
    mvk::u32x2* blockcnt = ws_ptr<mvk::u32x2>(c, p.off_blockcnt);
    mvk::u32x2* subcnt = ws_ptr<mvk::u32x2>(c, p.off_subcnt);
    uint32_t* emitfail = ws_ptr<uint32_t>(c, p.off_emitfail);
    unsigned long long* lookback = ws_ptr<unsigned long long>(c, p.off_lookback);
    uint32_t* votethr = ws_ptr<uint32_t>(c, p.off_votethr);
    mvk::u32x2* alist = p.add_drop ? ws_ptr<mvk::u32x2>(c, p.off_alist) : nullptr;
    mvk::u32x2* dlist = p.add_drop ? ws_ptr<mvk::u32x2>(c, p.off_dlist) : nullptr;
    uint32_t* adcount = p.add_drop ? ws_ptr<uint32_t>(c, p.off_adcount) : nullptr;
    uint32_t* adthr = p.add_drop ? ws_ptr<uint32_t>(c, p.off_adthr) : nullptr;
    uint32_t* adbits = p.add_drop ? ws_ptr<uint32_t>(c, p.off_adbits) : nullptr;
    mvk::u32x2* adblk = p.add_drop ? ws_ptr<mvk::u32x2>(c, p.off_adblk) : nullptr;

    const int slot = (int)(c->steps_done % kEventRing);
    for (int i = 0; i < KID_COUNT; ++i) c->ev_recorded[slot][i] = false;
    const int prof = c->profiling;
    bool ev_ok = true;
    auto wanted = [&](int kid) { return prof >= 2 || (prof == 1 && kid == KID_STREAM); };
    auto before = [&](int kid) {
        if (!wanted(kid)) return;
        for (int j = 0; j < 2; ++j)   // events are created on first use
            if (!c->ev[slot][kid][j] && hipEventCreate(&c->ev[slot][kid][j]) != hipSuccess) ev_ok = false;
        if (ev_ok && hipEventRecord(c->ev[slot][kid][0], st) != hipSuccess) ev_ok = false;
    };
    auto after = [&](int kid) {
        if (!wanted(kid) || !ev_ok) return;
        if (hipEventRecord(c->ev[slot][kid][1], st) == hipSuccess) c->ev_recorded[slot][kid] = true;
    };

    // 1. one kernel: sample histogram and threshold estimate per row (its first workgroups, which
    // also reset the per-step counters), and the streaming pass a = g + e over e, candidates out
    uint32_t* sampledone = ws_ptr<uint32_t>(c, p.off_sampledone);
    uint32_t* readsdone = ws_ptr<uint32_t>(c, p.off_readsdone);
    unsigned long long* taupub = ws_ptr<unsigned long long>(c, p.off_taupub);
    uint32_t* poison = ws_ptr<uint32_t>(c, p.off_poison);
    {
        const uint32_t wpr = (p.nseg + mvk::kSegPerBlock - 1) / mvk::kSegPerBlock;
        const dim3 grid(p.N * p.sample_wgs + p.N * wpr);
        before(KID_STREAM);
        if (bf16)
            hipLaunchKernelGGL(mvk::mv_stream_collect<uint16_t>, grid, dim3(mvk::kStreamThreads), 0, st,
                               static_cast<const uint16_t*>(a.grads), a.ld_g, a.err, a.ld_e, p.d, p.N, p.sample_wgs,
                               p.stride, p.n_sampled_chunks, p.m_target, hist, sampledone, readsdone, taupub, stepno,
                               c->spin_limit, poison, lvlsets, p.n_zero_words, adcount, cand, p.cap,
                               rowcnt_sets, rowcnt_set_words, seg, segsel, p.nseg, wpr, c->head_wgs,
                               add_drop ? (uint32_t*)nullptr : votes32, (int64_t)(((size_t)p.d + 15) / 16 * 16));
        else
            hipLaunchKernelGGL(mvk::mv_stream_collect<float>, grid, dim3(mvk::kStreamThreads), 0, st,
                               static_cast<const float*>(a.grads), a.ld_g, a.err, a.ld_e, p.d, p.N, p.sample_wgs,
                               p.stride, p.n_sampled_chunks, p.m_target, hist, sampledone, readsdone, taupub, stepno,
                               c->spin_limit, poison, lvlsets, p.n_zero_words, adcount, cand, p.cap,
                               rowcnt_sets, rowcnt_set_words, seg, segsel, p.nseg, wpr, c->head_wgs,
                               add_drop ? (uint32_t*)nullptr : votes32, (int64_t)(((size_t)p.d + 15) / 16 * 16));
        after(KID_STREAM);
    }
    // 3. exact per-row select
    // (in plain voting with short lists every workgroup of a row also casts the votes of its share of the list)
    const bool sorted = a.worker_idx != nullptr;
    const bool votes_in_select = !add_drop && !p.multi_select;
    before(KID_ROW_SELECT);
    {
        const uint32_t parts = votes_in_select ? p.select_parts : 1;
        // (with the many-workgroup select this launch only serves rows that need the exact path from memory:
        // nothing of the lists is fetched ahead)
        const uint32_t n_spec = p.multi_select ? 0u : p.n_spec;
        const dim3 grid((p.N + 7) / 8 * 8 * parts);
        if (p.long_lists)
            hipLaunchKernelGGL(mvk::mv_row_select<mvk::kKeepLong>, grid, dim3(mvk::kRowThreads), 0, st, a.err, a.ld_e,
                               p.d, p.N, p.K, cand, p.cap, rowcnt_sets, rowcnt_set_words, stepno, taupub, poison, rowcnt,
                               tau, kth, tiecut,
                               a.worker_idx, votes32,
                               sorted ? segsel : nullptr, p.nseg, lvlsets, slow, parts, n_spec, add_drop ? 1 : 0,
                               p.multi_select ? 1 : 0);
        else
            hipLaunchKernelGGL(mvk::mv_row_select<mvk::kKeepShort>, grid, dim3(mvk::kRowThreads), 0, st, a.err, a.ld_e,
                               p.d, p.N, p.K, cand, p.cap, rowcnt_sets, rowcnt_set_words, stepno, taupub, poison, rowcnt,
                               tau, kth, tiecut,
                               a.worker_idx, votes32,
                               sorted ? segsel : nullptr, p.nseg, lvlsets, slow, parts, n_spec, add_drop ? 1 : 0,
                               p.multi_select ? 1 : 0);
    }
    after(KID_ROW_SELECT);
    if (p.multi_select) {
        // long candidate lists: histogram, split at the bin of the K-th largest, exact rank
        mvk::ListSelect ls;
        ls.list = cand;  ls.cap = p.cap;  ls.count = rowcnt;  ls.count_stride = 1;
        ls.base = tau;  ls.shift = mvk::kFineShift;
        ls.want = p.K;
        ls.hist = ws_ptr<uint32_t>(c, p.off_selhist);
        ls.list2 = ws_ptr<mvk::u32x2>(c, p.off_sellist2);
        ls.count2 = ws_ptr<uint32_t>(c, p.off_selcount2);
        ls.bin_want = ws_ptr<uint32_t>(c, p.off_selbinwant);
        const dim3 grid((p.cap + mvk::kListPerBlock - 1) / mvk::kListPerBlock, p.N);
        before(KID_SEL_HIST);
        hipLaunchKernelGGL(mvk::mv_sel_hist, grid, dim3(mvk::kRowThreads), 0, st, ls);
        after(KID_SEL_HIST);
        before(KID_SEL_SPLIT);
        hipLaunchKernelGGL(mvk::mv_sel_split, grid, dim3(mvk::kRowThreads), 0, st, ls);
        after(KID_SEL_SPLIT);
        before(KID_SEL_RANK);
        hipLaunchKernelGGL(mvk::mv_sel_rank, dim3(p.N), dim3(mvk::kRowThreads), 0, st, ls, kth, tiecut, slow);
        after(KID_SEL_RANK);
    }

    uint32_t* mask_votes32 = votes32;     // the packed vote bytes the mask is selected from
    if (!add_drop && p.multi_select) {
        // 4. votes of the long lists (and segment tallies when the sorted lists are wanted)
        before(KID_ROW_VOTES);
        hipLaunchKernelGGL(mvk::mv_row_votes, dim3(p.vote_blocks, p.N), dim3(mvk::kRowThreads), 0, st, cand, p.cap,
                           rowcnt, p.nseg, kth, tiecut, slow, sorted ? segsel : nullptr, votes32, lvlsets);
        after(KID_ROW_VOTES);
    } else if (add_drop) {
        // 4'. add-drop voting: candidates for addition and removal, exact K_ad-selects,
        // update of msum and of the standing votes, sorted add / drop lists
        const uint32_t k_ad = (uint32_t)a.k_ad;
        uint32_t* msum32 = reinterpret_cast<uint32_t*>(a.msum);
        before(KID_AD_COLLECT);
        hipLaunchKernelGGL(mvk::mv_ad_collect, dim3(p.list_blocks + p.bit_blocks, p.N), dim3(mvk::kVoteThreads), 0,
                           st, a.err, a.ld_e, p.d, cand, p.cap, rowcnt, kth, tiecut, slow, a.vote_bits, a.ld_bits,
                           p.nwords_pad, alist, dlist, p.cap_d, adcount, p.list_blocks);
        after(KID_AD_COLLECT);
        before(KID_AD_SELECT);
        hipLaunchKernelGGL(mvk::mv_ad_select, dim3(2, p.N), dim3(mvk::kRowThreads), 0, st, alist, p.cap, dlist,
                           p.cap_d, adcount, k_ad, tau, slow, adthr, a.counts);
        after(KID_AD_SELECT);
        before(KID_AD_APPLY);
        hipLaunchKernelGGL(mvk::mv_ad_apply, dim3(p.list_blocks, p.N), dim3(mvk::kVoteThreads), 0, st, alist, p.cap,
                           dlist, p.cap_d, adcount, adthr, adbits, p.nwords_pad, msum32);
        after(KID_AD_APPLY);
        before(KID_AD_COMPACT_COUNT);
        hipLaunchKernelGGL(mvk::mv_ad_compact_count, dim3(p.N * p.bit_blocks + p.rs_blocks), dim3(mvk::kVoteThreads),
                           0, st, adbits, p.nwords_pad, p.bit_blocks, adblk, (const uint32_t*)a.vote_bits, a.ld_bits,
                           p.N * p.bit_blocks, (const uint32_t*)msum32, p.d, lvlsets);
        after(KID_AD_COMPACT_COUNT);
        before(KID_AD_COMPACT_EMIT);
        hipLaunchKernelGGL(mvk::mv_ad_compact_emit, dim3(p.bit_blocks, p.N), dim3(mvk::kVoteThreads), 0, st,
                           adbits, p.nwords_pad, p.bit_blocks, adblk, k_ad, a.add_idx, a.drop_idx, a.vote_bits,
                           a.ld_bits);
        after(KID_AD_COMPACT_EMIT);
        mask_votes32 = msum32;
    }
    if (random_sel) {
        // 4''. random selection: keys of the voted coordinates, their histogram, split at the bin of the K-th
        // soonest, exact ranking inside that bin, ordered compaction of the winners' bitmap
        uint32_t* rshist = ws_ptr<uint32_t>(c, p.off_rshist);
        uint32_t* rscount = ws_ptr<uint32_t>(c, p.off_rscount);
        uint32_t* rsbits = ws_ptr<uint32_t>(c, p.off_rsbits);
        mvk::u32x2* rsblk = ws_ptr<mvk::u32x2>(c, p.off_rsblk);
        mvk::u32x2* rslist = ws_ptr<mvk::u32x2>(c, p.off_rslist);
        mvk::u32x2* rslist2 = ws_ptr<mvk::u32x2>(c, p.off_rslist2);
        before(KID_RS_KEYS);
        hipLaunchKernelGGL(mvk::mv_rs_keys, dim3(p.rs_blocks), dim3(mvk::kVoteThreads), 0, st, votes32, p.d,
                           a.rand_exp, rslist, p.rs_cap, rscount);
        after(KID_RS_KEYS);
        mvk::ListSelect ls;
        ls.list = rslist;  ls.cap = p.rs_cap;  ls.count = rscount;  ls.count_stride = 1;  ls.base = nullptr;
        ls.shift = 20;
        ls.want = p.K;
        ls.hist = rshist;  ls.list2 = rslist2;  ls.count2 = rscount + 1;  ls.bin_want = rscount + 2;
        const dim3 grid((p.rs_cap + mvk::kListPerBlock - 1) / mvk::kListPerBlock);
        before(KID_RS_HIST);
        hipLaunchKernelGGL(mvk::mv_rs_hist, grid, dim3(mvk::kRowThreads), 0, st, ls);
        after(KID_RS_HIST);
        before(KID_RS_SPLIT);
        hipLaunchKernelGGL(mvk::mv_rs_split, grid, dim3(mvk::kRowThreads), 0, st, ls, rsbits);
        after(KID_RS_SPLIT);
        before(KID_RS_RANK);
        hipLaunchKernelGGL(mvk::mv_rs_rank, dim3(1), dim3(mvk::kRowThreads), 0, st, ls, rscount, rsbits);
        after(KID_RS_RANK);
        before(KID_AD_COMPACT_COUNT);
        hipLaunchKernelGGL(mvk::mv_ad_compact_count, dim3(p.bit_blocks), dim3(mvk::kVoteThreads), 0, st, rsbits,
                           p.nwords_pad, p.bit_blocks, rsblk, (const uint32_t*)nullptr, (int64_t)0, p.bit_blocks,
                           (const uint32_t*)nullptr, p.d, (uint32_t*)nullptr);
        after(KID_AD_COMPACT_COUNT);
        before(KID_AD_COMPACT_EMIT);
        hipLaunchKernelGGL(mvk::mv_ad_compact_emit, dim3(p.bit_blocks, 1), dim3(mvk::kVoteThreads), 0, st, rsbits,
                           p.nwords_pad, p.bit_blocks, rsblk, p.K, a.mask_idx, (uint32_t*)nullptr,
                           (uint32_t*)nullptr, (int64_t)0);
        after(KID_AD_COMPACT_EMIT);
    }
    // 5. global mask: the vote threshold and the counts per stretch of the vote bytes (in plain voting extra
    // workgroups scan the segment tallies for the sorted vote lists); then 6. every workgroup of the last
    // kernel emits its part of the mask, gathers it, takes the mean and updates the error buffers; extra
    // workgroups write the sorted vote lists beside it.  With random selection the mask is already written.
    const bool lists = sorted && !add_drop;
    {
        const dim3 grid_c(p.n_vote_blocks + (lists ? p.N : 0));
        const dim3 block(mvk::kMaskThreads);
        uint8_t* votes_out = add_drop ? nullptr : a.votes;
        const float inv_n = 1.0f / (float)p.N;
        const uint32_t kb = mvk::kMaskThreads / p.N;
        // Up to kGatherRounds rounds of kb mask positions per gathering workgroup.  When one or two rounds keep
        // the grid, with the sorted lists' workgroups, at about one workgroup per compute unit, that is best
        // (C4: 216 workgroups); when they do not (large K, many rows), many short workgroups beat few long
        // ones: two rounds and a grid of up to a thousand measured 4 us faster at K = d/100 than four rounds.
        const uint32_t eb = p.emit_blocks;
        const uint32_t n_list = lists ? p.N * eb : 0;
        auto rounds_for = [&](uint32_t limit) {
            const uint32_t room = n_list + 64 <= limit ? limit - n_list : 64;
            uint32_t r = (uint32_t)(((uint64_t)p.K + (uint64_t)room * kb - 1) / ((uint64_t)room * kb));
            if (r > (uint32_t)mvk::kGatherRounds) r = mvk::kGatherRounds;
            return r < 1 ? 1u : r;
        };
        uint32_t rounds = rounds_for(250);
        if (rounds > 2) rounds = rounds_for(1000);
        const uint32_t n_gather = (p.K + kb * rounds - 1) / (kb * rounds);
        const dim3 grid_g(n_gather + n_list);
#define MV_LAUNCH_MASK(Q)                                                                                        \
        before(KID_MASK_COUNT);                                                                                  \
        hipLaunchKernelGGL(mvk::mv_mask_count<Q>, grid_c, block, 0, st, mask_votes32, p.d, p.N, p.K, lvlsets,     \
                           subcnt, blockcnt, votethr, votes_out, p.n_vote_blocks, p.scan_parts, p.scan_blocks,   \
                           p.nseg,                                                                               \
                           slow, segsel, segpre, blktotal, add_drop ? 1 : 0, lookback, emitfail, c->spin_limit,  \
                           random_sel ? nullptr : a.mask_idx);                                                  \
        after(KID_MASK_COUNT);                                                                                   \
        before(KID_GATHER);                                                                                      \
        hipLaunchKernelGGL(mvk::mv_gather_update<Q>, grid_g, block, 0, st, a.err, a.ld_e, p.d, p.N, p.K,          \
                           (const uint32_t*)mask_votes32, (const mvk::u32x2*)subcnt,                             \
                           (const mvk::u32x2*)blockcnt, p.n_vote_blocks,                                         \
                           (const uint32_t*)votethr, a.mask_idx, random_sel ? 1 : 0,                             \
                           (const uint32_t*)emitfail, inv_n,                                                     \
                           c->cfg.reduce == MV_REDUCE_MEAN ? 1 : 0, a.agg_vals, rounds, n_gather, eb,            \
                           cand, p.cap, rowcnt, seg, p.nseg, segpre, blktotal, p.scan_blocks, kth, tiecut, slow, \
                           a.worker_idx, stepno);                                                                \
        after(KID_GATHER);
        switch (p.vote_q) {
            case 1: { MV_LAUNCH_MASK(1) } break;
            case 2: { MV_LAUNCH_MASK(2) } break;
            case 3: { MV_LAUNCH_MASK(3) } break;
            case 4: { MV_LAUNCH_MASK(4) } break;
            case 6: { MV_LAUNCH_MASK(6) } break;
            default: { MV_LAUNCH_MASK(8) } break;
        }
#undef MV_LAUNCH_MASK
    }
    c->last_stream = st;
    c->steps_done += 1;
    if (hipGetLastError() != hipSuccess) {
        // Some kernel of the sequence was not launched: counters that every step leaves at zero, and the
        // step's number on the device, may be off.  The context refuses further steps.
        c->broken = true;
        return MV_ERR_DEVICE;
    }
    return ev_ok ? MV_OK : MV_ERR_DEVICE;
}

}  // namespace

extern "C" {

mv_status mv_vote_step(mv_ctx* c, const void* grads, int64_t ld_g, float* err, int64_t ld_e,
                       uint32_t* worker_idx, uint8_t* votes, uint32_t* mask_idx, float* agg_vals,
                       void* stream_v)
{
    StepArgs a;
    memset(&a, 0, sizeof a);
    a.grads = grads; a.ld_g = ld_g; a.err = err; a.ld_e = ld_e;
    a.worker_idx = worker_idx; a.votes = votes; a.mask_idx = mask_idx; a.agg_vals = agg_vals;
    const mv_status st = check_common(c, a);
    if (st != MV_OK) return st;
    return enqueue_step(c, a, stream_v);
}

mv_status mv_ad_vote_step(mv_ctx* c, const void* grads, int64_t ld_g, float* err, int64_t ld_e,
                          int64_t k_ad, uint32_t* vote_bits, int64_t ld_bits, uint8_t* msum,
                          uint32_t* add_idx, uint32_t* drop_idx, uint32_t* counts,
                          uint32_t* mask_idx, float* agg_vals, void* stream_v)
{
    StepArgs a;
    memset(&a, 0, sizeof a);
    a.grads = grads; a.ld_g = ld_g; a.err = err; a.ld_e = ld_e;
    a.mask_idx = mask_idx; a.agg_vals = agg_vals;
    a.k_ad = k_ad; a.vote_bits = vote_bits; a.ld_bits = ld_bits; a.msum = msum;
    a.add_idx = add_idx; a.drop_idx = drop_idx; a.counts = counts;
    const mv_status st = check_common(c, a);
    if (st != MV_OK) return st;
    if (!c->plan.add_drop) return MV_ERR_STATE;              // the context was not begun with MV_FLAG_ADD_DROP
    if (k_ad < 1 || k_ad > (int64_t)c->plan.K) return MV_ERR_INVALID_ARG;
    if (!vote_bits || !msum || !add_idx || !drop_idx || !counts) return MV_ERR_INVALID_ARG;
    if (ld_bits < (int64_t)c->plan.nwords_pad || ld_bits % 4 != 0) return MV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(vote_bits) & 15) || (reinterpret_cast<uintptr_t>(msum) & 15))
        return MV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(add_idx) & 3) || (reinterpret_cast<uintptr_t>(drop_idx) & 3) ||
        (reinterpret_cast<uintptr_t>(counts) & 3))
        return MV_ERR_INVALID_ARG;
    return enqueue_step(c, a, stream_v);
}

mv_status mv_rs_vote_step(mv_ctx* c, const void* grads, int64_t ld_g, float* err, int64_t ld_e,
                          const float* rand_exp, uint32_t* worker_idx, uint8_t* votes, uint32_t* mask_idx,
                          float* agg_vals, void* stream_v)
{
    StepArgs a;
    memset(&a, 0, sizeof a);
    a.grads = grads; a.ld_g = ld_g; a.err = err; a.ld_e = ld_e;
    a.worker_idx = worker_idx; a.votes = votes; a.mask_idx = mask_idx; a.agg_vals = agg_vals;
    a.rand_exp = rand_exp;
    if (!rand_exp) return MV_ERR_INVALID_ARG;
    const mv_status st = check_common(c, a);
    if (st != MV_OK) return st;
    return enqueue_step(c, a, stream_v);
}

mv_status mv_end(mv_ctx* c)
{
    if (!c) return MV_ERR_INVALID_ARG;
    if (c->ended) return MV_ERR_STATE;
    c->ended = true;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return MV_ERR_DEVICE;
    mv_status rc = MV_OK;
    // steps run in the order of their calls, so the last call's stream is the one that still holds work
    if (c->steps_done != 0 && hipStreamSynchronize(c->last_stream) != hipSuccess) rc = MV_ERR_DEVICE;
    for (int r = 0; r < kEventRing; ++r)
        for (int i = 0; i < KID_COUNT; ++i)
            for (int j = 0; j < 2; ++j)
                if (c->ev[r][i][j]) (void)hipEventDestroy(c->ev[r][i][j]);
    if (c->owns_ws && c->ws && hipFree(c->ws) != hipSuccess) rc = MV_ERR_DEVICE;
    c->ws = nullptr;
    return rc;
}

void mv_release(mv_ctx* c)
{
    if (!c) return;
    if (!c->ended) (void)mv_end(c);
    delete c;
}

const char* mv_status_string(mv_status s)
{
    switch (s) {
        case MV_OK: return "ok";
        case MV_ERR_INVALID_ARG: return "invalid argument";
        case MV_ERR_UNSUPPORTED: return "unsupported";
        case MV_ERR_ALLOC: return "allocation failed";
        case MV_ERR_DEVICE: return "device error";
        case MV_ERR_STATE: return "context already ended";
    }
    return "unknown status";
}

int32_t mv_kernel_count(void) { return KID_COUNT; }

const char* mv_kernel_name(int32_t i) { return (i >= 0 && i < KID_COUNT) ? kKernelNames[i] : ""; }

mv_status mv_set_profiling(mv_ctx* c, int32_t level)
{
    if (!c || level < 0 || level > 2) return MV_ERR_INVALID_ARG;
    if (c->ended) return MV_ERR_STATE;
    c->profiling = level;
    return MV_OK;
}

mv_status mv_set_spin_limit(mv_ctx* c, uint32_t polls)
{
    if (!c) return MV_ERR_INVALID_ARG;
    if (c->ended) return MV_ERR_STATE;
    c->spin_limit = polls;
    return MV_OK;
}

mv_status mv_step_kernel_ms(mv_ctx* c, int32_t steps_back, float* ms, int32_t n)
{
    if (!c || !ms || n < KID_COUNT) return MV_ERR_INVALID_ARG;
    if (c->ended) return MV_ERR_STATE;
    if (steps_back < 0 || steps_back >= kEventRing || (uint64_t)steps_back >= c->steps_done)
        return MV_ERR_INVALID_ARG;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return MV_ERR_DEVICE;
    const int slot = (int)((c->steps_done - 1 - (uint64_t)steps_back) % kEventRing);
    for (int i = 0; i < KID_COUNT; ++i) {
        ms[i] = -1.0f;
        if (!c->ev_recorded[slot][i]) continue;
        if (hipEventSynchronize(c->ev[slot][i][1]) != hipSuccess) return MV_ERR_DEVICE;
        if (hipEventElapsedTime(&ms[i], c->ev[slot][i][0], c->ev[slot][i][1]) != hipSuccess)
            return MV_ERR_DEVICE;
    }
    return MV_OK;
}

mv_status mv_last_step_row_stats(mv_ctx* c, uint32_t* cand_count, uint32_t* threshold_bits, uint32_t* slow_path)
{
    if (!c) return MV_ERR_INVALID_ARG;
    if (c->ended) return MV_ERR_STATE;
    if (c->steps_done == 0) return MV_ERR_STATE;
    DeviceGuard guard(c->cfg.device);
    if (!guard.ok) return MV_ERR_DEVICE;
    if (hipStreamSynchronize(c->last_stream) != hipSuccess) return MV_ERR_DEVICE;
    const size_t nb = (size_t)c->plan.N * 4;
    if (cand_count && hipMemcpy(cand_count, c->ws + c->plan.off_candcount, nb, hipMemcpyDeviceToHost) != hipSuccess)
        return MV_ERR_DEVICE;
    if (threshold_bits && hipMemcpy(threshold_bits, c->ws + c->plan.off_tau, nb, hipMemcpyDeviceToHost) != hipSuccess)
        return MV_ERR_DEVICE;
    if (slow_path && hipMemcpy(slow_path, c->ws + c->plan.off_slow, nb, hipMemcpyDeviceToHost) != hipSuccess)
        return MV_ERR_DEVICE;
    return MV_OK;
}

mv_status mv_probe_copy(void* dst, const void* src, size_t bytes, void* stream)
{
    if (!dst || !src || bytes == 0 || (bytes & 15) != 0) return MV_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(dst) & 15) || (reinterpret_cast<uintptr_t>(src) & 15))
        return MV_ERR_INVALID_ARG;
    const uint64_t n16 = bytes / 16;
    const uint64_t blocks = (n16 + 1023) / 1024;
    if (blocks > 0x7FFFFFFFull) return MV_ERR_INVALID_ARG;
    hipLaunchKernelGGL(mvk::mv_probe_copy_kernel, dim3((uint32_t)blocks), dim3(256), 0,
                       static_cast<hipStream_t>(stream), static_cast<const mvk::u32x4*>(src),
                       static_cast<mvk::u32x4*>(dst), n16);
    return hipGetLastError() == hipSuccess ? MV_OK : MV_ERR_DEVICE;
}

}  // extern "C"
