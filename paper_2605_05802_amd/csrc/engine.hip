// Context, KV page bookkeeping and the C boundary (sr.h) of the selective-rollout decode library.
//
// The host owns the page allocator: every live sequence advances in lock step, so the pages a
// call needs are known before anything is launched, and only the retire mask (one byte per
// group, once per gate turn) ever flows from the device to the host.
#include <limits.h>
#include <math.h>
#include <string.h>

#include <string>
#include <vector>

#include "sr_internal.h"

namespace sr {

static thread_local std::string g_hip_error;

void note_hip_error(hipError_t e, const char *what) {
    g_hip_error = std::string(hipGetErrorString(e)) + " in " + what;
}

namespace {

struct PackedMat {
    uint16_t *p = nullptr;
    int N = 0;        // valid packed rows
    int ks = 0;       // k-steps
};

struct LayerW {
    PackedMat qkv, o, gu, down;
    uint16_t *bq = nullptr, *bk = nullptr, *bv = nullptr, *norm1 = nullptr, *norm2 = nullptr;
};

constexpr int kMaxSplitK = 16;
constexpr int kScoreRows = 2048;         // rows of the LM head computed at a time when every position is scored
constexpr int kMaxAttnSplits = 16;

}  // namespace
}  // namespace sr

using namespace sr;

// Pinned host staging for small host-to-device uploads (page table, row maps): a ring of slots, each with an event
// recorded behind its copy, so that an upload never blocks the host -- the host waits only if the copy that used a
// slot four uploads ago has still not run.
struct StagingRing {
    static constexpr int kSlots = 4;
    char *base = nullptr;
    size_t slot_bytes = 0;
    hipEvent_t ev[kSlots] = {};
    bool busy[kSlots] = {};
    int next = 0, cur = 0;

    int init(size_t bytes) {
        slot_bytes = (bytes + 255) & ~(size_t)255;
        SR_HIP(hipHostMalloc((void **)&base, slot_bytes * kSlots, hipHostMallocDefault));
        for (int i = 0; i < kSlots; ++i) SR_HIP(hipEventCreateWithFlags(&ev[i], hipEventDisableTiming));
        return SR_OK;
    }
    void destroy() {
        for (int i = 0; i < kSlots; ++i)
            if (ev[i]) (void)hipEventDestroy(ev[i]);
        if (base) (void)hipHostFree(base);
        base = nullptr;
    }
    // the next slot, free to be written by the host
    int acquire(void **p) {
        cur = next;
        next = (next + 1) % kSlots;
        if (busy[cur]) {
            SR_HIP(hipEventSynchronize(ev[cur]));
            busy[cur] = false;
        }
        *p = base + (size_t)cur * slot_bytes;
        return SR_OK;
    }
    // call right behind the copy that reads the slot handed out last
    int commit(hipStream_t st) {
        SR_HIP(hipEventRecord(ev[cur], st));
        busy[cur] = true;
        return SR_OK;
    }
};

struct sr_ctx {
    sr_model_shape s{};
    sr_options o{};
    int n_groups0 = 0, G = 0, n_seq0 = 0;
    double threshold = 0;

    // weights (library-owned, packed)
    bool weights_loaded = false;
    uint16_t *embed = nullptr, *final_norm = nullptr;
    PackedMat lm;
    std::vector<LayerW> L;
    float *rope_cos = nullptr, *rope_sin = nullptr;

    // KV pool
    uint16_t *kpool = nullptr, *vpool = nullptr;
    size_t layer_stride = 0, page_elems = 0;   // elements
    int n_pages = 0, max_pages = 0;
    std::vector<int> refcnt, free_list;

    // host batch state
    int n_live_groups = 0, seq_len = 0, shared_tokens = 0, turn = 0, actions_recorded = 0;
    bool first_decode_of_turn = false, have_logits = false, gate_pending = false, pt_dirty = false;
    std::vector<int> live_orig_group;
    std::vector<std::vector<int>> pages;       // per live sequence
    StagingRing pt_ring, rows_ring, units_ring, gate_ring;   // pinned staging of the uploads below
    uint8_t *h_retire = nullptr;                // pinned [n_groups0]
    int32_t *h_rows = nullptr;                  // current slot of rows_ring: [n_seq0]

    // groups some of whose members have finished (sr_finish_sequences)
    int n_rows = 0;                            // live sequences = rows of every per-sequence array
    std::vector<int> grp_count;                // live members of every live group (rows are group-major)
    std::vector<int> row_orig;                 // original sequence id of every live row (host mirror of d_orig)
    std::vector<int> end_step;                 // by ORIGINAL sequence id: turn after which it finished, or INT_MAX
    std::vector<int> fin_index;                // by original id: row of its saved actions in d_fin_actions, or -1
    int n_finished = 0;
    bool irregular = false;                    // some live group has fewer than G live members
    int32_t *h_units = nullptr;                // current slot of units_ring [2 * n_groups0 + n_seq0]: unit_row0, unit_count, row_unit
    int32_t *d_units = nullptr;                // device copy
    int32_t *h_gate_map = nullptr;             // current slot of gate_ring [2 * n_seq0]: source of every gate slot, its end step
    int32_t *d_gate_map = nullptr;
    int32_t *d_fin_actions = nullptr;          // [n_seq0][max_turns]: action rows of finished members, in finishing order
    int32_t *d_gate_actions = nullptr;         // [n_groups0][G][max_turns]: gate input assembled from live and finished rows
    sr_signals_t *d_gate_sig = nullptr;        // [n_groups0]

    // device batch state
    int32_t *d_pt = nullptr;
    int32_t *d_actions[2] = {nullptr, nullptr};
    int32_t *d_orig[2] = {nullptr, nullptr};   // original sequence id of every live row (keys the sampler)
    float *d_logits[2] = {nullptr, nullptr};
    double *d_logprob[2] = {nullptr, nullptr};  // running teacher-forced log-likelihood of every live row
    float *d_tok_lp = nullptr;                  // per-token values of the chunk being scored [n_seq0][max_seq_len]
    float *score_logits = nullptr;              // [kScoreRows][vocab], allocated by the first scoring call
    int cur = 0;
    int32_t *d_greedy = nullptr, *d_chosen = nullptr, *d_sums = nullptr, *d_rows = nullptr;
    uint8_t *d_retire = nullptr;

    // scratch
    int R = 0, mt_total = 0;                    // row capacity (multiple of 128) and its row tiles
    int ks_h = 0, ks_q = 0, ks_f = 0;           // k-steps of hidden, q_dim, ffn
    int qkv_cols = 0;
    float *resid = nullptr, *partials = nullptr, *part_o = nullptr, *part_ml = nullptr;
    size_t partial_elems = 0, part_rows_cap = 0;
    uint4 *xn = nullptr, *attn_out = nullptr, *act = nullptr;
    uint16_t *q = nullptr;

    // single-precision debugging path (o.fp32_debug): fp32 twins of the activation buffers and of the KV pool
    bool dbg = false;
    float *xn32 = nullptr, *attn32 = nullptr, *act32 = nullptr, *q32 = nullptr;
    float *kpool32 = nullptr, *vpool32 = nullptr;

    sr_stats_t st{};
    std::vector<void *> allocs;

    // optional per-kernel event timing
    bool prof_on = false;
    struct ProfRec { int kc; hipEvent_t a, b; };
    std::vector<ProfRec> prof;
    std::vector<hipEvent_t> event_pool;

    int n_live_seq() const { return n_rows; }
};

namespace {

template <typename T>
int dev_alloc(sr_ctx *c, T **p, size_t n_elems) {
    void *v = nullptr;
    hipError_t e = hipMalloc(&v, n_elems * sizeof(T) + 256);
    if (e != hipSuccess) {
        note_hip_error(e, "hipMalloc");
        return e == hipErrorOutOfMemory ? SR_E_NOMEM : SR_E_HIP;
    }
    c->allocs.push_back(v);
    *p = (T *)v;
    return SR_OK;
}

// Run one launch, bracketed by events when profiling is on.
template <typename F>
int timed(sr_ctx *c, int kc, hipStream_t st, F &&launch) {
    if (!c->prof_on) return launch();
    hipEvent_t ev[2];
    for (int i = 0; i < 2; ++i) {
        if (!c->event_pool.empty()) {
            ev[i] = c->event_pool.back();
            c->event_pool.pop_back();
        } else {
            SR_HIP(hipEventCreate(&ev[i]));
        }
    }
    SR_HIP(hipEventRecord(ev[0], st));
    const int rc = launch();
    SR_HIP(hipEventRecord(ev[1], st));
    c->prof.push_back({kc, ev[0], ev[1]});
    return rc;
}

// Decode-time projections (M <= 128).  Matrices that are wide or deep go to the kernel with a loader
// wavefront; the number of computing wavefronts per workgroup (32 features each) is picked so that
// the matrix breaks into about 256 workgroups with as few K splits as possible: the packed gate|up
// matrix (37 888 rows at the 7B shape) gives 237 workgroups of 160 features, the down projection
// 28 blocks of 128 features x 9 splits, the LM head 320-feature workgroups over two rounds.
// Thin ones keep the 4-wavefront kernel and are split along K so that about one workgroup per CU is
// in flight -- more than that only adds partial-sum traffic.  Batches of 129 .. 1024 rows split thin matrices a
// little (pick_splits); larger ones (prefill) never split.
int decode_waves(int M, int N, int ks_total, bool swiglu) {
    if (M > 128) return 0;
    if (swiglu) return N >= 8192 || ks_total >= 256 ? 5 : 0;
    // thin and shallow (QKV, O): two computing wavefronts per workgroup give enough workgroups with three or four
    // K splits instead of seven -- the projection itself takes the same time (13.9 against 13.0 us, 11.4 against
    // 11.8 us at the 7B shape) and the kernel that adds the partial sums reads half as many
    if (N < 8192 && ks_total < 256) return 2;
    if (N < 8192) return 4;
    // wide and shallow (the LM head): 256- or 320-feature workgroups, whichever leaves fewer workgroup-rounds of work
    // on 256 CUs (152 064 rows: 594 workgroups = 3 rounds of 8 wavefronts, or 476 = 2 rounds of 10; 226 against 246 us)
    const int r8 = ceil_div(ceil_div(N, 256), 256) * 8, r10 = ceil_div(ceil_div(N, 320), 256) * 10;
    return r10 < r8 ? 10 : 8;
}

int pick_splits(int M, int N, int ks_total) {
    if (M > 1024) return 1;
    if (M > 128) {
        // a few hundred rows (decode steps of a large batch): a thin matrix gives too few 128 x 128 tiles for the
        // 256 CUs (two workgroups each), so K is split until about 320 workgroups are in flight -- measured best at
        // 512 and 304 rows for the O, down and QKV projections of the 7B shape (2-3 splits, 1.5-2.3x faster)
        const int tiles = ceil_div(M, 128) * ceil_div(N, 128);
        int s = 320 / tiles;
        const int units = ks_total / 8;
        if (s > units / 4) s = units / 4;
        if (s > 4) s = 4;
        return s < 1 ? 1 : s;
    }
    const int waves = decode_waves(M, N, ks_total, false);
    const int n_blocks = ceil_div(N, waves ? 32 * waves : 128);
    const int target = 256 / n_blocks;
    if (target <= 1) return 1;
    const int units = ks_total / 8;                 // a split covers whole groups of 8 k-steps
    const int ups = ceil_div(units, target);        // units per split at the target count ...
    int s = ceil_div(units, ups);                   // ... and the fewest splits that keep it
    if (s > kMaxSplitK) s = kMaxSplitK;
    return s < 1 ? 1 : s;
}

int alloc_packed(sr_ctx *c, PackedMat *m, int n_rows, int K, hipStream_t st) {
    m->N = n_rows;
    m->ks = round_up(ceil_div(K, 32), 16);       // the GEMMs consume k-steps in groups of 16
    // row padding covers every workgroup width of the decode kernels (256, 160 and 320 features)
    int rows = round_up(n_rows, 256);
    if (round_up(n_rows, 160) > rows) rows = round_up(n_rows, 160);
    if (round_up(n_rows, 320) > rows) rows = round_up(n_rows, 320);
    const size_t elems = (size_t)rows * m->ks * 32;
    SR_TRY(dev_alloc(c, &m->p, elems));
    SR_HIP(hipMemsetAsync(m->p, 0, elems * 2, st));
    return SR_OK;
}

int copy_vec(sr_ctx *c, uint16_t **dst, const void *src, size_t n, hipStream_t st) {
    SR_TRY(dev_alloc(c, dst, n));
    SR_HIP(hipMemcpyAsync(*dst, src, n * 2, hipMemcpyDeviceToDevice, st));
    return SR_OK;
}

int upload_page_table(sr_ctx *c, hipStream_t st) {
    if (!c->pt_dirty) return SR_OK;
    const int n = c->n_live_seq();
    if (n > 0) {
        int32_t *h_pt = nullptr;
        SR_TRY(c->pt_ring.acquire((void **)&h_pt));
        for (int r = 0; r < n; ++r) {
            int32_t *row = h_pt + (size_t)r * c->max_pages;
            const std::vector<int> &pg = c->pages[r];
            size_t i = 0;
            for (; i < pg.size(); ++i) row[i] = pg[i];
            for (; i < (size_t)c->max_pages; ++i) row[i] = 0;
        }
        SR_HIP(hipMemcpyAsync(c->d_pt, h_pt, (size_t)n * c->max_pages * 4, hipMemcpyHostToDevice, st));
        SR_TRY(c->pt_ring.commit(st));
    }
    c->pt_dirty = false;
    return SR_OK;
}

int take_page(sr_ctx *c) {
    const int p = c->free_list.back();
    c->free_list.pop_back();
    c->st.pages_in_use++;
    return p;
}

void drop_page(sr_ctx *c, int p, int *freed) {
    if (--c->refcnt[p] == 0) {
        c->free_list.push_back(p);
        c->st.pages_in_use--;
        ++*freed;
    }
}

// Make room for every live sequence to grow to new_len tokens.  For a shared chunk the new
// pages are allocated once per group and referenced by its G members.  A member about to
// append into a page that other members still reference gets its own copy first.
int grow_pages(sr_ctx *c, int new_len, bool shared, hipStream_t st) {
    const int pt = c->o.page_tokens, G = c->G;
    if (shared && c->irregular) return SR_E_STATE;      // a shared chunk needs every group complete
    const int need = ceil_div(new_len, pt);
    const int n_seq = c->n_live_seq();
    // count first, so that a failure launches nothing and changes nothing
    int want = 0;
    for (int r = 0; r < n_seq; r += shared ? G : 1) {
        const std::vector<int> &pg = c->pages[r];
        want += need - (int)pg.size();
        if (!shared && c->seq_len % pt != 0 && c->refcnt[pg[c->seq_len / pt]] > 1) want += 1;
    }
    if (want > (int)c->free_list.size()) return SR_E_NOMEM;

    for (int r = 0; r < n_seq; r += shared ? G : 1) {
        if (!shared && c->seq_len % pt != 0) {
            const int idx = c->seq_len / pt, old = c->pages[r][idx];
            if (c->refcnt[old] > 1) {
                const int np = take_page(c);
                c->refcnt[np] = 1;
                c->refcnt[old]--;
                c->pages[r][idx] = np;
                if (c->dbg)      // fp32 pages: the same copy over twice as many 16-bit units
                    SR_TRY(launch_copy_page((uint16_t *)c->kpool32, (uint16_t *)c->vpool32, c->layer_stride * 2,
                                            c->s.n_layers, c->page_elems * 2, old, np, st));
                else
                    SR_TRY(launch_copy_page(c->kpool, c->vpool, c->layer_stride, c->s.n_layers, c->page_elems, old, np, st));
                c->st.cow_page_copies++;
                c->pt_dirty = true;
            }
        }
        while ((int)c->pages[r].size() < need) {
            const int np = take_page(c);
            if (shared) {
                c->refcnt[np] = G;
                for (int m = 0; m < G; ++m) c->pages[r + m].push_back(np);
            } else {
                c->refcnt[np] = 1;
                c->pages[r].push_back(np);
            }
            c->pt_dirty = true;
        }
    }
    return upload_page_table(c, st);
}

// Row ranges of the live groups, for the kernels that walk a group's members (decode attention over the
// shared prompt) once groups have become unequal.
int upload_units(sr_ctx *c, hipStream_t st) {
    c->irregular = false;
    int row = 0;
    SR_TRY(c->units_ring.acquire((void **)&c->h_units));
    int32_t *row0 = c->h_units, *cnt = c->h_units + c->n_groups0, *ru = c->h_units + 2 * c->n_groups0;
    for (int g = 0; g < c->n_live_groups; ++g) {
        row0[g] = row;
        cnt[g] = c->grp_count[g];
        for (int m = 0; m < c->grp_count[g]; ++m) ru[row + m] = g;
        row += c->grp_count[g];
        if (c->grp_count[g] != c->G) c->irregular = true;
    }
    if (c->irregular) {
        SR_HIP(hipMemcpyAsync(c->d_units, c->h_units, (size_t)(2 * c->n_groups0 + c->n_seq0) * 4,
                              hipMemcpyHostToDevice, st));
        SR_TRY(c->units_ring.commit(st));
    }
    return SR_OK;
}

// Keep the rows listed in h_rows[0 .. n) of every per-sequence device array, in that order.
int compact_rows(sr_ctx *c, int n, hipStream_t st) {
    if (n <= 0) return SR_OK;
    SR_HIP(hipMemcpyAsync(c->d_rows, c->h_rows, (size_t)n * 4, hipMemcpyHostToDevice, st));
    SR_TRY(c->rows_ring.commit(st));
    const int nxt = c->cur ^ 1;
    SR_TRY(launch_gather_rows(c->d_actions[nxt], c->d_actions[c->cur], c->d_rows, n, (size_t)c->o.max_turns * 4, st));
    SR_TRY(launch_gather_rows(c->d_logits[nxt], c->d_logits[c->cur], c->d_rows, n, (size_t)c->s.vocab * 4, st));
    SR_TRY(launch_gather_rows(c->d_orig[nxt], c->d_orig[c->cur], c->d_rows, n, 4, st));
    SR_TRY(launch_gather_rows(c->d_logprob[nxt], c->d_logprob[c->cur], c->d_rows, n, 8, st));
    c->cur = nxt;
    return SR_OK;
}

struct Pass {
    int rows;            // rows in this pass
    int n_units, chunk;  // rows = n_units * chunk
    int pos0;            // absolute position of the chunk's first token
    int pt_row0;         // page-table row of unit 0
    int pt_row_stride;
    const int32_t *tokens;
    int tok_stride, tok_off;
    bool decode;         // use the two-phase (shared prompt / private) decode attention
    // logits
    bool want_logits;
    int logit_dup;       // output rows per unit (G for a shared chunk, else 1)
    int logit_row0;      // first output row in the logits buffer
    // teacher-forced scoring: every row's logits give the log-probability of the next token of the chunk
    bool score;
    const uint8_t *score_mask;
    int score_chunk_len, score_unit0;
};

// K splits of a projection whose partial sums go to c->partials (the same choice on the normal and on the
// single-precision debugging path)
int choose_splits(sr_ctx *c, int M, const PackedMat &W, int ld_out, int *splits, size_t *split_stride) {
    *splits = pick_splits(M, W.N, W.ks);
    *split_stride = (size_t)round_up(M, 128) * ld_out;
    if (M > 128)                                     // larger batches may split only as far as the buffer allows
        while (*splits > 1 && *split_stride * *splits > c->partial_elems) --*splits;
    if (*split_stride * *splits > c->partial_elems) return SR_E_ARG;
    return SR_OK;
}

int gemm(sr_ctx *c, const uint4 *X, const PackedMat &W, int M, GemmEpilogue epi, void *out, int ld_out,
         int *splits_out, hipStream_t st) {
    GemmArgs a{};
    a.X = X;
    a.W = (const uint4 *)W.p;
    a.M = M;
    a.N = W.N;
    a.mt_total = c->mt_total;
    a.ks_total = W.ks;
    a.out = out;
    a.ld_out = ld_out;
    a.splits = 1;
    a.wide = decode_waves(M, W.N, W.ks, epi == EPI_SWIGLU);
    a.ring = 8;
    if (epi == EPI_F32 && splits_out) {
        SR_TRY(choose_splits(c, M, W, ld_out, &a.splits, &a.split_stride));
        *splits_out = a.splits;
    }
    return launch_gemm(a, epi, st);
}

// The same projection on the single-precision debugging path: X row-major fp32 [M][K]
int gemm32(sr_ctx *c, const float *X, int K, const PackedMat &W, int M, GemmEpilogue epi, float *out, int ld_out,
           int *splits_out, hipStream_t st) {
    DbgGemmArgs a{};
    a.X = X;
    a.ldx = K;
    a.W = W.p;
    a.M = M;
    a.N = W.N;
    a.ks_total = W.ks;
    a.out = out;
    a.ld_out = ld_out;
    a.splits = 1;
    if (epi == EPI_F32 && splits_out) {
        SR_TRY(choose_splits(c, M, W, ld_out, &a.splits, &a.split_stride));
        *splits_out = a.splits;
    }
    return launch_dbg_gemm(a, epi, st);
}

int forward(sr_ctx *c, const Pass &p, hipStream_t st) {
    const sr_model_shape &s = c->s;
    const int M = p.rows, H = s.hidden;
    const int n_rep = s.n_q_heads / s.n_kv_heads;
    int n_part = 0;                  // partials of the previous projection waiting to be added to resid
    size_t part_stride = 0;
    const int32_t *pt = c->d_pt + (size_t)p.pt_row0 * c->max_pages;

    AttnArgs aa{};
    aa.q = c->q;
    aa.page_table = pt;
    aa.pt_stride = c->max_pages;
    aa.page_tokens = c->o.page_tokens;
    aa.n_q = s.n_q_heads;
    aa.n_kv = s.n_kv_heads;
    aa.d = s.head_dim;
    aa.scale = 1.0f / sqrtf((float)s.head_dim);

    // attention phases (identical for every layer)
    AttnPhase ph[2];
    int n_ph = 0;
    const int ctx = p.pos0 + p.chunk;      // context length after this pass
    size_t part_rows = 0;
    auto add_phase = [&](AttnPhase x) {
        const size_t items = (size_t)x.n_units * s.n_kv_heads * x.items_per_unit * x.n_splits;
        x.part_o = c->part_o + part_rows * s.head_dim;
        x.part_ml = c->part_ml + part_rows * 2;
        part_rows += items * 16 * x.rt;
        ph[n_ph++] = x;
    };
    if (p.decode) {
        if (c->shared_tokens > 0) {
            AttnPhase x{};
            x.n_units = c->n_live_groups;
            x.q_per_unit = c->G;
            if (c->irregular) {                     // groups of unequal size: the kernels take the row ranges from maps
                x.unit_row0 = c->d_units;
                x.unit_count = c->d_units + c->n_groups0;
                x.row_unit = c->d_units + 2 * c->n_groups0;
            }
            x.rt = n_rep > 16 ? 2 : 1;              // same row-tile count as the private phase: one launch
            x.q_per_item = (16 * x.rt) / n_rep < c->G ? (16 * x.rt) / n_rep : c->G;
            x.items_per_unit = ceil_div(c->G, x.q_per_item);
            x.pt_row_stride = c->G;
            x.t_begin = 0;
            x.t_end = c->shared_tokens;
            x.causal_pos0 = ctx - 1;
            x.causal_stride = 0;
            x.n_splits = ceil_div(c->shared_tokens, 256);
            if (x.n_splits > kMaxAttnSplits) x.n_splits = kMaxAttnSplits;
            x.split_tokens = round_up(ceil_div(c->shared_tokens, x.n_splits), 32);
            add_phase(x);
        }
        AttnPhase y{};
        y.n_units = p.n_units;
        y.q_per_unit = 1;
        y.q_per_item = 1;
        y.items_per_unit = 1;
        y.rt = n_rep > 16 ? 2 : 1;
        y.pt_row_stride = 1;
        y.t_begin = c->shared_tokens;
        y.t_end = ctx;
        y.causal_pos0 = ctx - 1;
        y.causal_stride = 0;
        const int priv = ctx - c->shared_tokens;
        // about 1024 wavefronts in the private phase (with the shared phase's, 6-8 per CU: measured 4-10 % faster
        // than 12 per CU at 128 and at 80 rows, at every context length), each at least 128 tokens long; a
        // function of the context length and the batch shape only, never of the row
        const int per_split = p.n_units * s.n_kv_heads;
        y.n_splits = (1024 + per_split / 2) / per_split;
        if (y.n_splits > ceil_div(priv, 128)) y.n_splits = ceil_div(priv, 128);
        if (y.n_splits < 1) y.n_splits = 1;
        if (y.n_splits > kMaxAttnSplits) y.n_splits = kMaxAttnSplits;
        y.split_tokens = round_up(ceil_div(priv, y.n_splits), 32);
        // a sequence's private tokens are read by one work item per kv head: streamed past the caches once the
        // stream is long enough to gain from it (measured: slower below a few hundred tokens, 8 % faster at 1900)
        y.stream_loads = priv >= 512 ? 1 : 0;
        add_phase(y);
    } else {
        AttnPhase x{};
        x.n_units = p.n_units;
        x.q_per_unit = p.chunk;
        x.rt = 2;
        x.q_per_item = 32 / n_rep < p.chunk ? 32 / n_rep : p.chunk;
        if (x.q_per_item * n_rep <= 16) x.rt = 1;
        x.items_per_unit = ceil_div(p.chunk, x.q_per_item);
        x.pt_row_stride = p.pt_row_stride;
        x.t_begin = 0;
        x.t_end = ctx;
        x.causal_pos0 = p.pos0;
        x.causal_stride = 1;
        x.n_splits = 1;
        x.split_tokens = round_up(ctx, 32);
        add_phase(x);
    }
    if (part_rows > c->part_rows_cap) return SR_E_NOMEM;
    // one partial result per query row: the attention kernel writes the merged output itself
    const bool direct = n_ph == 1 && ph[0].n_splits == 1;
    const bool dbg = c->dbg;
    const int qd = s.n_q_heads * s.head_dim;
    aa.direct_out = direct && !dbg ? (uint16_t *)c->attn_out : nullptr;
    aa.out_mt_total = c->mt_total;
    DbgAttnArgs da{};
    da.q32 = c->q32;
    da.direct_out32 = direct && dbg ? c->attn32 : nullptr;

    for (int l = 0; l < s.n_layers; ++l) {
        const LayerW &w = c->L[l];
        NormArgs na{};
        na.resid = c->resid;
        na.out = c->xn;
        na.out32 = dbg ? c->xn32 : nullptr;
        na.rows_out = M;
        na.src_dup = 1;
        na.src_stride = 1;
        na.src_off = 0;
        na.write_resid = 1;
        na.H = H;
        na.mt_total = c->mt_total;
        na.eps = s.rms_eps;
        na.gain = w.norm1;
        if (l == 0) {
            na.embed = c->embed;
            na.tokens = p.tokens;
            na.tok_chunk = p.chunk;
            na.tok_stride = p.tok_stride;
            na.tok_off = p.tok_off;
        } else {
            na.partials = c->partials;
            na.n_partials = n_part;
            na.partial_stride = part_stride;
        }
        SR_TRY(timed(c, SR_KC_NORM, st, [&] { return launch_resid_norm(na, st); }));

        int sp = 1;
        SR_TRY(timed(c, SR_KC_GEMM_QKV, st, [&] {
            return dbg ? gemm32(c, c->xn32, H, w.qkv, M, EPI_F32, c->partials, c->qkv_cols, &sp, st)
                       : gemm(c, c->xn, w.qkv, M, EPI_F32, c->partials, c->qkv_cols, &sp, st);
        }));
        QkvPostArgs qa{};
        qa.partials = c->partials;
        qa.n_partials = sp;
        qa.partial_stride = (size_t)round_up(M, 128) * c->qkv_cols;
        qa.ld = c->qkv_cols;
        qa.bq = s.qkv_bias ? w.bq : nullptr;
        qa.bk = s.qkv_bias ? w.bk : nullptr;
        qa.bv = s.qkv_bias ? w.bv : nullptr;
        qa.rope_cos = c->rope_cos;
        qa.rope_sin = c->rope_sin;
        qa.q_out = c->q;
        qa.kpool = c->kpool + (size_t)l * c->layer_stride;
        qa.vpool = c->vpool + (size_t)l * c->layer_stride;
        qa.page_table = pt;
        qa.pt_stride = c->max_pages;
        qa.pt_row_stride = p.pt_row_stride;
        qa.rows = M;
        qa.chunk = p.chunk;
        qa.pos0 = p.pos0;
        qa.n_q = s.n_q_heads;
        qa.n_kv = s.n_kv_heads;
        qa.d = s.head_dim;
        qa.page_tokens = c->o.page_tokens;
        if (dbg) {
            DbgQkvPostArgs dq{};
            dq.base = qa;
            dq.q32 = c->q32;
            dq.kpool32 = c->kpool32 + (size_t)l * c->layer_stride;
            dq.vpool32 = c->vpool32 + (size_t)l * c->layer_stride;
            SR_TRY(timed(c, SR_KC_QKV_POST, st, [&] { return launch_dbg_qkv_post(dq, st); }));
            da.base = aa;
            da.kpool32 = dq.kpool32;
            da.vpool32 = dq.vpool32;
            SR_TRY(timed(c, p.decode ? SR_KC_ATTN_DECODE : SR_KC_ATTN_PREFILL, st,
                         [&] { return launch_dbg_attention(da, ph, n_ph, st); }));
        } else {
            SR_TRY(timed(c, SR_KC_QKV_POST, st, [&] { return launch_qkv_post(qa, st); }));
            aa.kpool = qa.kpool;
            aa.vpool = qa.vpool;
            SR_TRY(timed(c, p.decode ? SR_KC_ATTN_DECODE : SR_KC_ATTN_PREFILL, st,
                         [&] { return launch_attention(aa, ph, n_ph, st); }));
        }
        if (!direct) {
            SR_TRY(timed(c, SR_KC_ATTN_MERGE, st, [&] {
                return launch_attn_merge(aa, ph, n_ph, M, c->attn_out, c->mt_total, dbg ? c->attn32 : nullptr, st);
            }));
        }

        SR_TRY(timed(c, SR_KC_GEMM_O, st, [&] {
            return dbg ? gemm32(c, c->attn32, qd, w.o, M, EPI_F32, c->partials, H, &sp, st)
                       : gemm(c, c->attn_out, w.o, M, EPI_F32, c->partials, H, &sp, st);
        }));
        na.embed = nullptr;
        na.tokens = nullptr;
        na.partials = c->partials;
        na.n_partials = sp;
        na.partial_stride = (size_t)round_up(M, 128) * H;
        na.gain = w.norm2;
        SR_TRY(timed(c, SR_KC_NORM, st, [&] { return launch_resid_norm(na, st); }));

        SR_TRY(timed(c, SR_KC_GEMM_GATE_UP, st, [&] {
            return dbg ? gemm32(c, c->xn32, H, w.gu, M, EPI_SWIGLU, c->act32, s.ffn, nullptr, st)
                       : gemm(c, c->xn, w.gu, M, EPI_SWIGLU, c->act, c->ks_f * 32, nullptr, st);
        }));
        SR_TRY(timed(c, SR_KC_GEMM_DOWN, st, [&] {
            return dbg ? gemm32(c, c->act32, s.ffn, w.down, M, EPI_F32, c->partials, H, &sp, st)
                       : gemm(c, c->act, w.down, M, EPI_F32, c->partials, H, &sp, st);
        }));
        n_part = sp;
        part_stride = (size_t)round_up(M, 128) * H;
    }

    if (p.score) {
        // final norm of every row, then the LM head kScoreRows rows at a time; each block of logits is
        // reduced to one log-probability per row before the next block overwrites it
        NormArgs na{};
        na.resid = c->resid;
        na.partials = c->partials;
        na.n_partials = n_part;
        na.partial_stride = part_stride;
        na.gain = c->final_norm;
        na.out = c->xn;
        na.out32 = dbg ? c->xn32 : nullptr;
        na.rows_out = M;
        na.src_dup = 1;
        na.src_stride = 1;
        na.src_off = 0;
        na.write_resid = 0;
        na.H = H;
        na.mt_total = c->mt_total;
        na.eps = s.rms_eps;
        SR_TRY(timed(c, SR_KC_NORM, st, [&] { return launch_resid_norm(na, st); }));
        for (int r0 = 0; r0 < M; r0 += kScoreRows) {
            const int blk = M - r0 < kScoreRows ? M - r0 : kScoreRows;
            const uint4 *x = c->xn + (size_t)(r0 / 16) * 64;      // row tile r0 / 16 of every k-step
            SR_TRY(timed(c, SR_KC_GEMM_LM_HEAD, st, [&] {
                return dbg ? gemm32(c, c->xn32 + (size_t)r0 * H, H, c->lm, blk, EPI_F32, c->score_logits, s.vocab,
                                    nullptr, st)
                           : gemm(c, x, c->lm, blk, EPI_F32, c->score_logits, s.vocab, nullptr, st);
            }));
            LogprobArgs la{};
            la.logits = c->score_logits;
            la.vocab = s.vocab;
            la.tokens = p.tokens;
            la.mask = p.score_mask;
            la.chunk_len = p.score_chunk_len;
            la.rows_per_unit = p.chunk;
            la.row0 = r0;
            la.tok0 = p.tok_off + 1;                              // a row predicts the token after it
            la.out = c->d_tok_lp + (size_t)p.score_unit0 * p.score_chunk_len;
            SR_TRY(timed(c, SR_KC_ARGMAX, st, [&] { return launch_logprob_rows(la, blk, st); }));
        }
    }

    if (p.want_logits) {
        NormArgs na{};
        na.resid = c->resid;
        na.partials = c->partials;
        na.n_partials = n_part;
        na.partial_stride = part_stride;
        na.gain = c->final_norm;
        na.out = c->xn;
        na.out32 = dbg ? c->xn32 : nullptr;
        na.rows_out = p.n_units * p.logit_dup;
        na.src_dup = p.logit_dup;
        na.src_stride = p.chunk;
        na.src_off = p.chunk - 1;
        na.write_resid = 0;
        na.H = H;
        na.mt_total = c->mt_total;
        na.eps = s.rms_eps;
        SR_TRY(timed(c, SR_KC_NORM, st, [&] { return launch_resid_norm(na, st); }));
        float *dst = c->d_logits[c->cur] + (size_t)p.logit_row0 * s.vocab;
        SR_TRY(timed(c, SR_KC_GEMM_LM_HEAD, st, [&] {
            return dbg ? gemm32(c, c->xn32, H, c->lm, na.rows_out, EPI_F32, dst, s.vocab, nullptr, st)
                       : gemm(c, c->xn, c->lm, na.rows_out, EPI_F32, dst, s.vocab, nullptr, st);
        }));
    }
    return SR_OK;
}

}  // namespace

// ------------------------------------------------------------------------------------------------
// C boundary
// ------------------------------------------------------------------------------------------------
extern "C" {

const char *sr_strerror(int status) {
    switch (status) {
        case SR_OK: return "ok";
        case SR_E_ARG: return "invalid argument";
        case SR_E_NOMEM: return "out of memory (KV page pool exhausted or allocation failed)";
        case SR_E_STATE: return "call out of order";
        case SR_E_HIP: return g_hip_error.empty() ? "HIP error" : g_hip_error.c_str();
        case SR_E_LIMIT: return "size beyond the fixed capacity of an entry point that allocates nothing";
        default: return "unknown status";
    }
}

void sr_destroy(sr_ctx *c) {
    if (!c) return;
    (void)hipDeviceSynchronize();
    for (void *p : c->allocs) (void)hipFree(p);
    c->pt_ring.destroy();
    c->rows_ring.destroy();
    c->units_ring.destroy();
    c->gate_ring.destroy();
    if (c->h_retire) (void)hipHostFree(c->h_retire);
    for (auto &r : c->prof) { (void)hipEventDestroy(r.a); (void)hipEventDestroy(r.b); }
    for (hipEvent_t e : c->event_pool) (void)hipEventDestroy(e);
    delete c;
}

static int init_impl(sr_ctx *c) {
    const sr_model_shape &s = c->s;
    const sr_options &o = c->o;
    const int d = s.head_dim;
    c->n_seq0 = c->n_groups0 * c->G;
    c->qkv_cols = (s.n_q_heads + 2 * s.n_kv_heads) * d;
    c->ks_h = round_up(s.hidden / 32, 16);       // k extents padded to groups of 16 k-steps (zeros)
    c->ks_q = round_up(s.n_q_heads * d / 32, 16);
    c->ks_f = round_up(ceil_div(s.ffn, 32), 16);
    const int max_rows = o.max_prefill_rows > 0 ? o.max_prefill_rows : 8192;
    c->R = round_up(max_rows > c->n_seq0 ? max_rows : c->n_seq0, 256);
    c->mt_total = c->R / 16;

    // RoPE tables, computed in double: angle = pos * theta^(-2i/d)
    {
        const int half = d / 2;
        std::vector<float> hc((size_t)o.max_seq_len * half), hs((size_t)o.max_seq_len * half);
        for (int i = 0; i < half; ++i) {
            const double inv_freq = pow((double)s.rope_theta, -2.0 * i / d);
            for (int pos = 0; pos < o.max_seq_len; ++pos) {
                hc[(size_t)pos * half + i] = (float)cos(pos * inv_freq);
                hs[(size_t)pos * half + i] = (float)sin(pos * inv_freq);
            }
        }
        SR_TRY(dev_alloc(c, &c->rope_cos, hc.size()));
        SR_TRY(dev_alloc(c, &c->rope_sin, hs.size()));
        SR_HIP(hipMemcpy(c->rope_cos, hc.data(), hc.size() * 4, hipMemcpyHostToDevice));
        SR_HIP(hipMemcpy(c->rope_sin, hs.data(), hs.size() * 4, hipMemcpyHostToDevice));
    }

    // KV pool: [layer][page][kv head][32-token block][32*d], K and V separately
    c->dbg = o.fp32_debug != 0;
    c->page_elems = (size_t)s.n_kv_heads * o.page_tokens * d;
    const size_t elem_bytes = c->dbg ? 4 : 2;
    const size_t page_bytes_all = c->page_elems * elem_bytes * s.n_layers * 2;
    c->n_pages = (int)(o.kv_pool_bytes / page_bytes_all);
    c->max_pages = ceil_div(o.max_seq_len, o.page_tokens);
    if (c->n_pages < 1) return SR_E_ARG;
    c->layer_stride = c->page_elems * c->n_pages;
    if (c->dbg) {
        SR_TRY(dev_alloc(c, &c->kpool32, c->layer_stride * s.n_layers));
        SR_TRY(dev_alloc(c, &c->vpool32, c->layer_stride * s.n_layers));
        SR_HIP(hipMemset(c->kpool32, 0, c->layer_stride * s.n_layers * 4));
        SR_HIP(hipMemset(c->vpool32, 0, c->layer_stride * s.n_layers * 4));
    } else {
        SR_TRY(dev_alloc(c, &c->kpool, c->layer_stride * s.n_layers));
        SR_TRY(dev_alloc(c, &c->vpool, c->layer_stride * s.n_layers));
        // masked probabilities multiply V entries that were never written: they must be finite
        SR_HIP(hipMemset(c->kpool, 0, c->layer_stride * s.n_layers * 2));
        SR_HIP(hipMemset(c->vpool, 0, c->layer_stride * s.n_layers * 2));
    }
    c->refcnt.assign(c->n_pages, 0);
    c->free_list.resize(c->n_pages);
    for (int i = 0; i < c->n_pages; ++i) c->free_list[i] = c->n_pages - 1 - i;
    c->st.pages_total = c->n_pages;

    // batch state
    c->n_live_groups = c->n_groups0;
    c->live_orig_group.resize(c->n_groups0);
    for (int g = 0; g < c->n_groups0; ++g) c->live_orig_group[g] = g;
    c->n_rows = c->n_seq0;
    c->grp_count.assign(c->n_groups0, c->G);
    c->row_orig.resize(c->n_seq0);
    for (int r = 0; r < c->n_seq0; ++r) c->row_orig[r] = r;
    c->end_step.assign(c->n_seq0, INT_MAX);
    c->fin_index.assign(c->n_seq0, -1);
    SR_TRY(c->units_ring.init((size_t)(2 * c->n_groups0 + c->n_seq0) * 4 + 16));
    SR_TRY(c->gate_ring.init((size_t)2 * c->n_seq0 * 4 + 16));
    SR_TRY(dev_alloc(c, &c->d_units, (size_t)2 * c->n_groups0 + c->n_seq0));
    SR_TRY(dev_alloc(c, &c->d_gate_map, (size_t)2 * c->n_seq0));
    SR_TRY(dev_alloc(c, &c->d_fin_actions, (size_t)c->n_seq0 * o.max_turns));
    SR_TRY(dev_alloc(c, &c->d_gate_actions, (size_t)c->n_seq0 * o.max_turns));
    SR_TRY(dev_alloc(c, &c->d_gate_sig, (size_t)c->n_groups0));
    c->pages.assign(c->n_seq0, {});
    SR_TRY(c->pt_ring.init((size_t)c->n_seq0 * c->max_pages * 4 + 16));
    SR_HIP(hipHostMalloc((void **)&c->h_retire, c->n_groups0 + 16, hipHostMallocDefault));
    SR_TRY(c->rows_ring.init((size_t)c->n_seq0 * 4 + 16));
    SR_TRY(dev_alloc(c, &c->d_pt, (size_t)c->n_seq0 * c->max_pages));
    SR_HIP(hipMemset(c->d_pt, 0, (size_t)c->n_seq0 * c->max_pages * 4));
    for (int i = 0; i < 2; ++i) {
        SR_TRY(dev_alloc(c, &c->d_actions[i], (size_t)c->n_seq0 * o.max_turns));
        SR_TRY(dev_alloc(c, &c->d_logits[i], (size_t)c->n_seq0 * s.vocab));
        SR_TRY(launch_fill_i32(c->d_actions[i], (size_t)c->n_seq0 * o.max_turns, -1, nullptr));
        SR_TRY(dev_alloc(c, &c->d_orig[i], (size_t)c->n_seq0));
        SR_TRY(dev_alloc(c, &c->d_logprob[i], (size_t)c->n_seq0));
        SR_HIP(hipMemset(c->d_logprob[i], 0, (size_t)c->n_seq0 * sizeof(double)));
    }
    {
        std::vector<int32_t> ids(c->n_seq0);
        for (int i = 0; i < c->n_seq0; ++i) ids[i] = i;
        SR_HIP(hipMemcpy(c->d_orig[0], ids.data(), ids.size() * 4, hipMemcpyHostToDevice));
    }
    SR_TRY(dev_alloc(c, &c->d_greedy, (size_t)c->n_seq0));
    SR_TRY(dev_alloc(c, &c->d_chosen, (size_t)c->n_seq0));
    SR_TRY(dev_alloc(c, &c->d_sums, (size_t)c->n_groups0));
    SR_TRY(dev_alloc(c, &c->d_rows, (size_t)c->n_seq0));
    SR_TRY(dev_alloc(c, &c->d_retire, (size_t)c->n_groups0));

    // scratch
    const size_t R = c->R;
    const int n_max = c->qkv_cols > s.hidden ? c->qkv_cols : s.hidden;
    const size_t dec_rows = round_up(c->n_seq0, 128);
    c->partial_elems = R * n_max;
    if (dec_rows * n_max * kMaxSplitK > c->partial_elems) c->partial_elems = dec_rows * n_max * kMaxSplitK;
    c->part_rows_cap = 2 * R * s.n_q_heads + (size_t)c->n_seq0 * s.n_kv_heads * 32 * (2 * kMaxAttnSplits + 1);
    SR_TRY(dev_alloc(c, &c->resid, R * s.hidden));
    SR_TRY(dev_alloc(c, &c->partials, c->partial_elems));
    SR_TRY(dev_alloc(c, &c->xn, R * (size_t)(c->ks_h * 32) / 8));
    SR_TRY(dev_alloc(c, &c->attn_out, R * (size_t)(c->ks_q * 32) / 8));
    SR_TRY(dev_alloc(c, &c->act, R * (size_t)(c->ks_f * 32) / 8));
    // padded k-steps are never written afterwards and must read as zero
    SR_HIP(hipMemset(c->xn, 0, R * (size_t)(c->ks_h * 32) * 2));
    SR_HIP(hipMemset(c->attn_out, 0, R * (size_t)(c->ks_q * 32) * 2));
    SR_HIP(hipMemset(c->act, 0, R * (size_t)(c->ks_f * 32) * 2));
    SR_TRY(dev_alloc(c, &c->q, R * (size_t)s.n_q_heads * d));
    if (c->dbg) {
        SR_TRY(dev_alloc(c, &c->xn32, R * (size_t)s.hidden));
        SR_TRY(dev_alloc(c, &c->attn32, R * (size_t)s.n_q_heads * d));
        SR_TRY(dev_alloc(c, &c->act32, R * (size_t)s.ffn));
        SR_TRY(dev_alloc(c, &c->q32, R * (size_t)s.n_q_heads * d));
    }
    SR_TRY(dev_alloc(c, &c->part_o, c->part_rows_cap * d));
    SR_TRY(dev_alloc(c, &c->part_ml, c->part_rows_cap * 2));
    SR_HIP(hipDeviceSynchronize());
    return SR_OK;
}

int sr_init(sr_ctx **out, const sr_model_shape *shape, int n_groups, int G, double threshold,
            const sr_options *opt) {
    if (!out || !shape || !opt) return SR_E_ARG;
    *out = nullptr;
    const sr_model_shape &s = *shape;
    if (n_groups < 1 || G < 2 || G > 16 || !(threshold >= 0.0) || threshold > 1.0) return SR_E_ARG;
    if (s.n_layers < 1 || s.hidden < 32 || s.hidden % 32 || s.hidden > 8192 || s.vocab < 16 || s.vocab % 16 ||
        s.ffn < 16 || s.ffn % 16 || (s.head_dim != 64 && s.head_dim != 128) || s.n_kv_heads < 1 ||
        s.n_q_heads % s.n_kv_heads || s.n_q_heads / s.n_kv_heads > 16 || !(s.rms_eps > 0.f) || !(s.rope_theta > 0.f))
        return SR_E_ARG;
    if ((opt->page_tokens != 32 && opt->page_tokens != 64 && opt->page_tokens != 128) || opt->max_seq_len < 1 ||
        opt->max_turns < 1 || opt->max_turns > 32 || opt->action_mod < 0 || opt->max_prefill_rows < 0 ||
        !(opt->temperature >= 0.f) || !(opt->tau_H >= 0.f) || opt->tau_H > 4.f ||
        (opt->fp32_debug != 0 && opt->fp32_debug != 1) || (s.tied_lm_head != 0 && s.tied_lm_head != 1))
        return SR_E_ARG;
    sr_ctx *c = new sr_ctx();
    c->s = s;
    c->o = *opt;
    c->n_groups0 = n_groups;
    c->G = G;
    c->threshold = threshold;
    const int rc = init_impl(c);
    if (rc != SR_OK) {
        sr_destroy(c);
        return rc;
    }
    *out = c;
    return SR_OK;
}

int sr_load_weights(sr_ctx *c, const sr_weights *w, void *stream) {
    if (!c || !w || !w->embed || !w->final_norm || !w->layers) return SR_E_ARG;
    if (!c->s.tied_lm_head && !w->lm_head) return SR_E_ARG;
    if (c->weights_loaded) return SR_E_STATE;
    hipStream_t st = (hipStream_t)stream;
    const sr_model_shape &s = c->s;
    const int H = s.hidden, qd = s.n_q_heads * s.head_dim, kd = s.n_kv_heads * s.head_dim;
    for (int l = 0; l < s.n_layers; ++l) {
        const sr_layer_weights &x = w->layers[l];
        if (!x.wq || !x.wk || !x.wv || !x.wo || !x.wg || !x.wu || !x.wd || !x.norm1 || !x.norm2) return SR_E_ARG;
        if (s.qkv_bias && (!x.bq || !x.bk || !x.bv)) return SR_E_ARG;
    }
    SR_TRY(copy_vec(c, &c->embed, w->embed, (size_t)s.vocab * H, st));
    SR_TRY(copy_vec(c, &c->final_norm, w->final_norm, H, st));
    SR_TRY(alloc_packed(c, &c->lm, s.vocab, H, st));
    // tied: the LM head is the embedding matrix, packed like any other projection
    SR_TRY(launch_pack_rows((const uint16_t *)(s.tied_lm_head ? w->embed : w->lm_head), s.vocab, H, c->lm.p, c->lm.ks,
                            0, 0, 0, st));
    c->L.resize(s.n_layers);
    for (int l = 0; l < s.n_layers; ++l) {
        const sr_layer_weights &x = w->layers[l];
        LayerW &y = c->L[l];
        SR_TRY(alloc_packed(c, &y.qkv, c->qkv_cols, H, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wq, qd, H, y.qkv.p, y.qkv.ks, 0, 0, 0, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wk, kd, H, y.qkv.p, y.qkv.ks, qd, 0, 0, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wv, kd, H, y.qkv.p, y.qkv.ks, qd + kd, 0, 0, st));
        SR_TRY(alloc_packed(c, &y.o, H, qd, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wo, H, qd, y.o.p, y.o.ks, 0, 0, 0, st));
        SR_TRY(alloc_packed(c, &y.gu, 2 * s.ffn, H, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wg, s.ffn, H, y.gu.p, y.gu.ks, 0, 1, 0, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wu, s.ffn, H, y.gu.p, y.gu.ks, 0, 1, 1, st));
        SR_TRY(alloc_packed(c, &y.down, H, s.ffn, st));
        SR_TRY(launch_pack_rows((const uint16_t *)x.wd, H, s.ffn, y.down.p, y.down.ks, 0, 0, 0, st));
        if (s.qkv_bias) {
            SR_TRY(copy_vec(c, &y.bq, x.bq, qd, st));
            SR_TRY(copy_vec(c, &y.bk, x.bk, kd, st));
            SR_TRY(copy_vec(c, &y.bv, x.bv, kd, st));
        }
        SR_TRY(copy_vec(c, &y.norm1, x.norm1, H, st));
        SR_TRY(copy_vec(c, &y.norm2, x.norm2, H, st));
    }
    SR_HIP(hipStreamSynchronize(st));
    c->weights_loaded = true;
    return SR_OK;
}

int sr_prefill_chunk(sr_ctx *c, const int32_t *tokens, int chunk_len, int shared_per_group, void *stream) {
    if (!c || !tokens || chunk_len <= 0) return SR_E_ARG;
    if (!c->weights_loaded) return SR_E_STATE;
    if (shared_per_group && c->seq_len != 0) return SR_E_STATE;
    if (c->n_live_groups == 0) return SR_OK;
    if (c->seq_len + chunk_len > c->o.max_seq_len) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const bool shared = shared_per_group != 0;
    const int new_len = c->seq_len + chunk_len;
    SR_TRY(grow_pages(c, new_len, shared, st));

    const int n_units = shared ? c->n_live_groups : c->n_live_seq();
    const int dup = shared ? c->G : 1;
    for (int c0 = 0; c0 < chunk_len; c0 += c->R) {
        const int cl = chunk_len - c0 < c->R ? chunk_len - c0 : c->R;
        const int upp = c->R / cl;                 // units per pass
        for (int u0 = 0; u0 < n_units; u0 += upp) {
            const int nu = n_units - u0 < upp ? n_units - u0 : upp;
            Pass p{};
            p.rows = nu * cl;
            p.n_units = nu;
            p.chunk = cl;
            p.pos0 = c->seq_len + c0;
            p.pt_row0 = u0 * dup;
            p.pt_row_stride = dup;
            p.tokens = tokens + (size_t)u0 * chunk_len;
            p.tok_stride = chunk_len;
            p.tok_off = c0;
            p.decode = false;
            p.want_logits = (c0 + cl == chunk_len);
            p.logit_dup = dup;
            p.logit_row0 = u0 * dup;
            SR_TRY(forward(c, p, st));
        }
    }
    c->seq_len = new_len;
    if (shared) {
        c->shared_tokens = (new_len / c->o.page_tokens) * c->o.page_tokens;
        c->st.prefill_tokens += (int64_t)c->n_live_groups * chunk_len;
    } else {
        c->turn++;
        c->first_decode_of_turn = true;
        c->st.prefill_tokens += (int64_t)c->n_live_seq() * chunk_len;
    }
    c->have_logits = true;
    return SR_OK;
}

int sr_score_chunk(sr_ctx *c, const int32_t *tokens, const uint8_t *action_mask, int chunk_len,
                   float *out_token_logprob, void *stream) {
    if (!c || !tokens || chunk_len <= 0) return SR_E_ARG;
    if (!c->weights_loaded || !c->have_logits || c->seq_len == 0) return SR_E_STATE;
    if (c->n_live_groups == 0) return SR_OK;
    if (c->seq_len + chunk_len > c->o.max_seq_len) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const sr_model_shape &s = c->s;
    const int n = c->n_live_seq();
    if (!c->score_logits) SR_TRY(dev_alloc(c, &c->score_logits, (size_t)kScoreRows * s.vocab));
    if (!c->d_tok_lp) SR_TRY(dev_alloc(c, &c->d_tok_lp, (size_t)c->n_seq0 * c->o.max_seq_len));
    const int new_len = c->seq_len + chunk_len;
    SR_TRY(grow_pages(c, new_len, false, st));

    // the chunk's first token is predicted by the logits of the position before the chunk
    {
        LogprobArgs la{};
        la.logits = c->d_logits[c->cur];
        la.vocab = s.vocab;
        la.tokens = tokens;
        la.mask = action_mask;
        la.chunk_len = chunk_len;
        la.row0 = 0;
        la.rows_per_unit = 1;
        la.tok0 = 0;
        la.out = c->d_tok_lp;
        SR_TRY(launch_logprob_rows(la, n, st));
    }
    for (int c0 = 0; c0 < chunk_len; c0 += c->R) {
        const int cl = chunk_len - c0 < c->R ? chunk_len - c0 : c->R;
        const int upp = c->R / cl;                 // units per pass
        for (int u0 = 0; u0 < n; u0 += upp) {
            const int nu = n - u0 < upp ? n - u0 : upp;
            Pass p{};
            p.rows = nu * cl;
            p.n_units = nu;
            p.chunk = cl;
            p.pos0 = c->seq_len + c0;
            p.pt_row0 = u0;
            p.pt_row_stride = 1;
            p.tokens = tokens + (size_t)u0 * chunk_len;
            p.tok_stride = chunk_len;
            p.tok_off = c0;
            p.decode = false;
            p.want_logits = (c0 + cl == chunk_len);
            p.logit_dup = 1;
            p.logit_row0 = u0;
            p.score = true;
            p.score_mask = action_mask ? action_mask + (size_t)u0 * chunk_len : nullptr;
            p.score_chunk_len = chunk_len;
            p.score_unit0 = u0;
            SR_TRY(forward(c, p, st));
        }
    }
    SR_TRY(launch_accumulate_logprob(c->d_tok_lp, n, chunk_len, c->d_logprob[c->cur], st));
    if (out_token_logprob)
        SR_HIP(hipMemcpyAsync(out_token_logprob, c->d_tok_lp, (size_t)n * chunk_len * sizeof(float),
                              hipMemcpyDeviceToDevice, st));
    c->seq_len = new_len;
    c->st.prefill_tokens += (int64_t)n * chunk_len;
    c->have_logits = true;
    return SR_OK;
}

int sr_get_logprob(sr_ctx *c, double *dst, void *stream) {
    if (!c || !dst) return SR_E_ARG;
    const int n = c->n_live_seq();
    if (n == 0) return SR_OK;
    SR_HIP(hipMemcpyAsync(dst, c->d_logprob[c->cur], (size_t)n * sizeof(double), hipMemcpyDeviceToDevice,
                          (hipStream_t)stream));
    return SR_OK;
}

int sr_decode_step(sr_ctx *c, const int32_t *forced, int32_t *out_tokens, void *stream) {
    if (!c) return SR_E_ARG;
    if (!c->weights_loaded || !c->have_logits) return SR_E_STATE;
    if (c->n_live_groups == 0) return SR_OK;
    if (c->seq_len + 1 > c->o.max_seq_len) return SR_E_ARG;
    hipStream_t st = (hipStream_t)stream;
    const int n = c->n_live_seq();
    SR_TRY(grow_pages(c, c->seq_len + 1, false, st));

    const bool record = c->first_decode_of_turn && c->o.action_mod > 0 && c->turn >= 1 && c->turn <= c->o.max_turns;
    SR_TRY(timed(c, SR_KC_ARGMAX, st, [&] {
        return launch_argmax(c->d_logits[c->cur], n, c->s.vocab, forced, c->d_greedy, c->d_chosen,
                             record ? c->d_actions[c->cur] : nullptr, c->o.max_turns, c->turn - 1,
                             c->o.action_mod > 0 ? c->o.action_mod : 1,
                             c->o.temperature > 0.f ? 1.0f / c->o.temperature : 0.f, c->o.sample_seed,
                             c->d_orig[c->cur], c->seq_len, st);
    }));
    if (out_tokens) SR_HIP(hipMemcpyAsync(out_tokens, c->d_greedy, (size_t)n * 4, hipMemcpyDeviceToDevice, st));
    if (c->first_decode_of_turn && c->turn >= 1) {
        if (record) c->actions_recorded = c->turn;
        c->first_decode_of_turn = false;
    }

    Pass p{};
    p.rows = n;
    p.n_units = n;
    p.chunk = 1;
    p.pos0 = c->seq_len;
    p.pt_row0 = 0;
    p.pt_row_stride = 1;
    p.tokens = c->d_chosen;
    p.tok_stride = 1;
    p.tok_off = 0;
    p.decode = true;
    p.want_logits = true;
    p.logit_dup = 1;
    p.logit_row0 = 0;
    SR_TRY(forward(c, p, st));
    c->seq_len += 1;
    c->st.decoded_tokens += n;
    return SR_OK;
}

int sr_gate(sr_ctx *c, int turn, int32_t *out_sums, uint8_t *out_retire, void *stream) {
    if (!c || turn < 1 || turn > c->o.max_turns) return SR_E_ARG;
    if (c->actions_recorded < turn) return SR_E_STATE;
    hipStream_t st = (hipStream_t)stream;
    const int ng = c->n_live_groups, G = c->G, T = c->o.max_turns;
    if (c->n_finished == 0) {
        // every member of every live group holds exactly `turn` actions: the equal-length form of Eq. 2
        GateLens lens{};
        lens.n = 1;
        lens.len[0] = turn;
        lens.bound[0] = (int)gate_bound(c->threshold, G, turn);
        SR_TRY(launch_gate(c->d_actions[c->cur], ng, G, T, lens, c->d_sums, c->d_retire, st));
    } else if (ng > 0) {
        // some members finished early: gather each group's G action rows (live rows and saved rows of
        // finished members, in member order) and evaluate d_K with per-pair longer-length normalisation,
        // and the termination-fraction clause when tau_H is set
        SR_TRY(c->gate_ring.acquire((void **)&c->h_gate_map));
        int32_t *src = c->h_gate_map, *end = c->h_gate_map + c->n_seq0;
        int row = 0;
        for (int g = 0; g < ng; ++g) {
            const int og = c->live_orig_group[g];
            for (int m = 0; m < G; ++m) {
                const int orig = og * G + m;
                if (c->end_step[orig] == INT_MAX) {
                    src[g * G + m] = row++;
                    end[g * G + m] = INT_MAX;
                } else {
                    src[g * G + m] = -1 - c->fin_index[orig];
                    end[g * G + m] = c->end_step[orig];
                }
            }
        }
        SR_HIP(hipMemcpyAsync(c->d_gate_map, c->h_gate_map, (size_t)2 * c->n_seq0 * 4, hipMemcpyHostToDevice, st));
        SR_TRY(c->gate_ring.commit(st));
        SR_TRY(launch_assemble_gate(c->d_gate_map, c->d_actions[c->cur], c->d_fin_actions, ng * G, T,
                                    c->d_gate_actions, st));
        const int len1 = turn;
        const double tau = c->o.tau_H > 0.f ? (double)c->o.tau_H : 2.0;
        SR_TRY(sr_signals_batch(c->d_gate_actions, nullptr, c->d_gate_map + c->n_seq0, ng, G, T, &len1, 1,
                                c->threshold, tau, c->d_gate_sig, st));
        SR_TRY(launch_extract_gate(c->d_gate_sig, ng, c->o.tau_H > 0.f ? 1 : 0, c->d_sums, c->d_retire, st));
    }
    if (ng > 0 && out_sums) SR_HIP(hipMemcpyAsync(out_sums, c->d_sums, (size_t)ng * 4, hipMemcpyDeviceToDevice, st));
    if (ng > 0 && out_retire) SR_HIP(hipMemcpyAsync(out_retire, c->d_retire, ng, hipMemcpyDeviceToDevice, st));
    c->gate_pending = true;
    return SR_OK;
}

// Drop the live rows for which drop[row] is set (their pages go back to the pool), keep the others in order,
// and drop the groups left without a live member.
static int remove_rows(sr_ctx *c, const std::vector<char> &drop, int *freed, hipStream_t st) {
    const int ng = c->n_live_groups, n = c->n_rows;
    int kept_rows = 0, kept_groups = 0, row = 0;
    SR_TRY(c->rows_ring.acquire((void **)&c->h_rows));
    for (int g = 0; g < ng; ++g) {
        int alive = 0;
        for (int m = 0; m < c->grp_count[g]; ++m, ++row) {
            if (drop[row]) {
                for (int pg : c->pages[row]) drop_page(c, pg, freed);
                c->pages[row].clear();
                continue;
            }
            if (kept_rows != row) {
                c->pages[kept_rows] = std::move(c->pages[row]);
                c->pages[row].clear();
                c->row_orig[kept_rows] = c->row_orig[row];
            }
            c->h_rows[kept_rows++] = row;
            ++alive;
        }
        if (alive > 0) {
            c->live_orig_group[kept_groups] = c->live_orig_group[g];
            c->grp_count[kept_groups++] = alive;
        }
    }
    if (kept_rows != n) {
        c->live_orig_group.resize(kept_groups);
        c->grp_count.resize(kept_groups);
        c->row_orig.resize(kept_rows);
        SR_TRY(compact_rows(c, kept_rows, st));
        c->n_live_groups = kept_groups;
        c->n_rows = kept_rows;
        SR_TRY(upload_units(c, st));
        c->pt_dirty = true;
        SR_TRY(upload_page_table(c, st));
    }
    return SR_OK;
}

int sr_retire_and_compact(sr_ctx *c, int *host_n_live_groups, void *stream) {
    if (!c) return SR_E_ARG;
    if (!c->gate_pending) return SR_E_STATE;
    hipStream_t st = (hipStream_t)stream;
    c->gate_pending = false;
    const int ng = c->n_live_groups;
    if (ng == 0) {
        if (host_n_live_groups) *host_n_live_groups = 0;
        return SR_OK;
    }
    SR_HIP(hipMemcpyAsync(c->h_retire, c->d_retire, ng, hipMemcpyDeviceToHost, st));
    SR_HIP(hipStreamSynchronize(st));

    std::vector<char> drop(c->n_rows, 0);
    int row = 0, freed = 0;
    for (int g = 0; g < ng; ++g) {
        if (c->h_retire[g]) c->st.groups_retired++;
        for (int m = 0; m < c->grp_count[g]; ++m, ++row) drop[row] = c->h_retire[g] ? 1 : 0;
    }
    SR_TRY(remove_rows(c, drop, &freed, st));
    c->st.pages_freed += freed;
    if (host_n_live_groups) *host_n_live_groups = c->n_live_groups;
    return SR_OK;
}

int sr_finish_sequences(sr_ctx *c, const uint8_t *host_done, int *host_n_live_seq, void *stream) {
    if (!c || !host_done) return SR_E_ARG;
    if (c->turn < 1 || c->first_decode_of_turn) return SR_E_STATE;    // between a turn's decode and the next prefill
    // the mask of a gate that has not been applied yet is indexed by the groups live at that gate; dropping a
    // whole group now would shift it onto the wrong groups
    if (c->gate_pending) return SR_E_STATE;
    hipStream_t st = (hipStream_t)stream;
    const int n = c->n_rows;
    std::vector<char> drop(n, 0);
    std::vector<int> done_rows;
    for (int r = 0; r < n; ++r)
        if (host_done[r]) {
            drop[r] = 1;
            done_rows.push_back(r);
        }
    const int n_done = (int)done_rows.size();
    if (n_done > 0) {
        // keep the finished members' action rows: the gate of a later turn still compares their prefixes
        SR_TRY(c->rows_ring.acquire((void **)&c->h_rows));
        for (int i = 0; i < n_done; ++i) c->h_rows[i] = done_rows[i];
        SR_HIP(hipMemcpyAsync(c->d_rows, c->h_rows, (size_t)n_done * 4, hipMemcpyHostToDevice, st));
        SR_TRY(c->rows_ring.commit(st));
        SR_TRY(launch_gather_rows(c->d_fin_actions + (size_t)c->n_finished * c->o.max_turns, c->d_actions[c->cur],
                                  c->d_rows, n_done, (size_t)c->o.max_turns * 4, st));
        for (int i = 0; i < n_done; ++i) {
            const int orig = c->row_orig[done_rows[i]];
            c->end_step[orig] = c->turn;
            c->fin_index[orig] = c->n_finished++;
        }
        const int groups_before = c->n_live_groups;
        int freed = 0;
        SR_TRY(remove_rows(c, drop, &freed, st));
        c->st.seqs_finished += n_done;
        c->st.groups_finished += groups_before - c->n_live_groups;
    }
    if (host_n_live_seq) *host_n_live_seq = c->n_rows;
    return SR_OK;
}

int sr_set_actions(sr_ctx *c, int turn, const int32_t *ids, void *stream) {
    if (!c || !ids || turn < 1 || turn > c->o.max_turns) return SR_E_ARG;
    const int n = c->n_live_seq();
    if (n == 0) return SR_OK;
    SR_HIP(hipMemcpy2DAsync(c->d_actions[c->cur] + (turn - 1), (size_t)c->o.max_turns * 4, ids, 4, 4, n,
                            hipMemcpyDeviceToDevice, (hipStream_t)stream));
    if (turn > c->actions_recorded) c->actions_recorded = turn;
    return SR_OK;
}

int sr_get_actions(sr_ctx *c, int32_t *dst, void *stream) {
    if (!c || !dst) return SR_E_ARG;
    const int n = c->n_live_seq();
    if (n == 0) return SR_OK;
    SR_HIP(hipMemcpyAsync(dst, c->d_actions[c->cur], (size_t)n * c->o.max_turns * 4, hipMemcpyDeviceToDevice,
                          (hipStream_t)stream));
    return SR_OK;
}

int sr_get_logits(sr_ctx *c, float *dst, void *stream) {
    if (!c || !dst) return SR_E_ARG;
    if (!c->have_logits) return SR_E_STATE;
    const int n = c->n_live_seq();
    if (n == 0) return SR_OK;
    SR_HIP(hipMemcpyAsync(dst, c->d_logits[c->cur], (size_t)n * c->s.vocab * 4, hipMemcpyDeviceToDevice,
                          (hipStream_t)stream));
    return SR_OK;
}

int sr_get_live_map(sr_ctx *c, int32_t *host_orig_seq_ids) {
    if (!c || !host_orig_seq_ids) return SR_E_ARG;
    for (int r = 0; r < c->n_rows; ++r) host_orig_seq_ids[r] = c->row_orig[r];
    return SR_OK;
}

int sr_profile(sr_ctx *c, int enable) {
    if (!c) return SR_E_ARG;
    c->prof_on = enable != 0;
    return SR_OK;
}

int sr_profile_read(sr_ctx *c, sr_kernel_time *out, void *stream) {
    if (!c || !out) return SR_E_ARG;
    SR_HIP(hipStreamSynchronize((hipStream_t)stream));
    for (int i = 0; i < SR_KC_COUNT; ++i) out[i] = sr_kernel_time{0, 0.0};
    for (auto &r : c->prof) {
        float ms = 0.f;
        SR_HIP(hipEventElapsedTime(&ms, r.a, r.b));
        out[r.kc].launches++;
        out[r.kc].total_ms += ms;
        c->event_pool.push_back(r.a);
        c->event_pool.push_back(r.b);
    }
    c->prof.clear();
    return SR_OK;
}

int sr_stats(sr_ctx *c, sr_stats_t *out) {
    if (!c || !out) return SR_E_ARG;
    c->st.n_live_groups = c->n_live_groups;
    c->st.n_live_seq = c->n_live_seq();
    c->st.seq_len = c->seq_len;
    c->st.turn = c->turn;
    *out = c->st;
    return SR_OK;
}

}  // extern "C"
