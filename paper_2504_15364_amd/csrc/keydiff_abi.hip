// Host side of the C ABI declared in include/keydiff.h: argument validation,
// the Eq. 5 state machine (len, positions) and the per-step kernel sequence.
#include "../../include/keydiff.h"

#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "kd_kernels.h"

namespace {

thread_local char g_err[512] = "";

int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof g_err, fmt, ap);
    va_end(ap);
    return code;
}

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Layout {
    size_t k_bytes, meta_bytes, scratch_bytes;
    size_t off_pos, off_ksum, off_status, off_oflags;                                 // in meta
    size_t off_part_o, off_part_ml, off_scores, off_dstmap, off_lists, off_ksum_part, off_q_rot, off_k_rot, off_argmax;  // in scratch
    int cap, max_part_rows;
    int target_wgs;   // bound used to size the partial buffers: twice the compute units of the chip
};

// Compute units of the current device (one 8-wave attention workgroup runs per unit); 256, the
// MI355X's count, where no device can be asked (sizing calls on a host without a GPU).
int compute_units()
{
    static int cached[64] = {};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) {
        (void)hipGetLastError();
        return 256;
    }
    if (cached[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n < 1) {
            (void)hipGetLastError();
            n = 256;
        }
        cached[dev] = n;
    }
    return cached[dev];
}

// Scratch of keydiff_prefill_block_static: one array per GPU the library runs on, held until the process ends.
// On the host the array's name only stands for the symbol; the memory is reached through the device
// address hipGetSymbolAddress returns, looked up once per device (static_scratch_of).
constexpr int kMaxDevices = 64;

}  // namespace

// (No `used` attribute: the compiler gives the variable a symbol the runtime can look up because
// host code below names it; emitted before that use is seen it stays local to the code object, and
// hipGetSymbolAddress then aborts the process instead of returning an error.)
static __device__ __align__(256) unsigned char scratch[KEYDIFF_STATIC_SCRATCH_BYTES];

namespace {

unsigned char *g_static_scratch[kMaxDevices] = {};   // device address of `scratch` on each GPU, once known

// device address of the static scratch array on `device`, which must be the current device
int static_scratch_of(int device, unsigned char **out)
{
    if (device < 0 || device >= kMaxDevices) return fail(KEYDIFF_ESHAPE, "device index %d out of range", device);
    if (!g_static_scratch[device]) {
        void *ptr = nullptr;
        const hipError_t e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return fail(KEYDIFF_EHIP, "hipGetSymbolAddress(static scratch): %s", hipGetErrorString(e));
        g_static_scratch[device] = static_cast<unsigned char *>(ptr);
    }
    *out = g_static_scratch[device];
    return KEYDIFF_OK;
}

int check_config(const keydiff_config_t *c)
{
    if (!c) return fail(KEYDIFF_EINVAL, "config is null");
    if (c->batch < 1 || c->n_q_heads < 1 || c->n_kv_heads < 1 || c->budget_N < 1 || c->block_B < 1)
        return fail(KEYDIFF_ESHAPE, "batch, head counts, budget_N and block_B must be positive");
    if (c->n_q_heads % c->n_kv_heads) return fail(KEYDIFF_ESHAPE, "n_q_heads must be a multiple of n_kv_heads");
    if (c->head_dim != 64 && c->head_dim != 128) return fail(KEYDIFF_ESHAPE, "head_dim must be 64 or 128");
    if ((long)c->budget_N + c->block_B > kd::MAX_CAP)
        return fail(KEYDIFF_ESHAPE, "budget_N + block_B must not exceed %d", kd::MAX_CAP);
    if ((long)c->batch * c->n_kv_heads > 65535) return fail(KEYDIFF_ESHAPE, "batch * n_kv_heads must not exceed 65535");
    if (c->anchor_mode != KEYDIFF_ANCHOR_MEAN_KEY && c->anchor_mode != KEYDIFF_ANCHOR_MEAN_UNIT_KEY)
        return fail(KEYDIFF_EINVAL, "anchor_mode must be a KEYDIFF_ANCHOR_* value");
    if (c->layout != KEYDIFF_LAYOUT_ORDERED && c->layout != KEYDIFF_LAYOUT_FILL)
        return fail(KEYDIFF_EINVAL, "layout must be a KEYDIFF_LAYOUT_* value");
    if (c->window_W < 0 || c->window_W >= c->budget_N)
        return fail(KEYDIFF_ESHAPE, "window_W must lie in [0, budget_N)");
    return KEYDIFF_OK;
}

Layout make_layout(const keydiff_config_t *c)
{
    Layout L{};
    const size_t BH = (size_t)c->batch * c->n_kv_heads;
    const int G = c->n_q_heads / c->n_kv_heads;
    const int D = c->head_dim;
    L.cap = (c->budget_N + c->block_B + 3) & ~3;   // rows per head, a multiple of four (16-byte loads of scores and positions)
    L.k_bytes = align256(BH * L.cap * D * 2);
    size_t off = 0;
    L.off_pos = off;     off += align256(BH * L.cap * 4);
    L.off_ksum = off;    off += align256(2 * BH * D * 8);  // double buffer: see StepParams::ksum_next
    L.off_status = off;  off += 256;
    L.off_oflags = off;  off += align256(BH * ((L.cap + kd::ORD_ROWS - 1) / kd::ORD_ROWS) * 4);  // ordered compaction
    L.meta_bytes = off;
    // split-KV partial rows: splits * BH * (G * Bt rounded up to 32) never exceeds this (see plan_attention)
    const int kTargetWorkgroups = 2 * compute_units();
    L.target_wgs = kTargetWorkgroups;
    const int max_mtiles = (G * c->block_B + 127) / 128;
    const size_t by_tiles = (kTargetWorkgroups + BH * max_mtiles + BH) * 256;
    const size_t Mpad_max = (size_t)((G * c->block_B + 31) / 32 * 32);                               // blocks of 32 rows
    const size_t by_rows = (kTargetWorkgroups + 2 * BH) * Mpad_max * (G * c->block_B <= 32 ? 2 : 1);  // two partials per workgroup
    L.max_part_rows = (int)(by_tiles < by_rows ? by_tiles : by_rows);
    const size_t chunks = (L.cap + kd::CHUNK_ROWS - 1) / kd::CHUNK_ROWS;
    off = 0;
    L.off_part_o = off;     off += align256((size_t)L.max_part_rows * D * 2);
    L.off_part_ml = off;    off += align256((size_t)L.max_part_rows * 8);
    L.off_scores = off;     off += align256(BH * L.cap * 4);
    L.off_dstmap = off;     off += align256(BH * L.cap * 4);
    L.off_lists = off;      off += align256(BH * 4 * (size_t)c->block_B * 4);
    L.off_ksum_part = off;  off += align256(BH * chunks * D * 8);
    L.off_q_rot = off;      off += align256((size_t)c->batch * c->n_q_heads * c->block_B * D * 2);   // rotated block (rope entry points)
    L.off_k_rot = off;      off += align256(BH * c->block_B * D * 2);
    L.off_argmax = off;     off += align256((size_t)(kTargetWorkgroups + BH) * 16);   // one arg-max record per step_main workgroup
    L.scratch_bytes = off;
    return L;
}

struct ProfEvent {
    int kind;
    hipEvent_t a, b;
};

}  // namespace

struct keydiff_cache {
    keydiff_config_t cfg;
    Layout L;
    uint16_t *k, *v;
    unsigned char *meta, *scratch;
    int device;           // the device that was current when the handle was created
    int len;
    double eps;
    float scale_log2e;
    bool contiguous;      // every block so far started where the previous one ended
    int64_t next_pos;
    int32_t epoch;        // launches of the ordered compaction so far (its flags compare against it)
    int kpar;             // which half of the key-sum double buffer holds the current sum
    bool pending;         // a deferred eviction (selection + compaction) has not been enqueued yet
    kd::StepParams pend;  // ... the parameters of the step it belongs to
    hipStream_t pend_stream;
    // ORDERED layout, eviction deferred through keydiff_prefill_block_layers: the selection has run (it
    // rode in another layer's attention launch) and the row shift by its destination map has not yet; it
    // rides in a later attention launch, or is enqueued alone by the first call that touches this cache
    bool shift_pending;
    kd::StepParams shift_p;
    hipStream_t shift_stream;
    int32_t plan[4];      // of the last block step: key ranges, row tiles per head, key tiles, carried a passenger
    bool profiling;
    std::vector<ProfEvent> events;
    std::vector<hipEvent_t> pool;
};

namespace {

struct ProfScope {
    keydiff_cache *c;
    hipStream_t s;
    ProfEvent ev;
    bool on;
    ProfScope(keydiff_cache *c_, int kind, hipStream_t s_) : c(c_), s(s_), on(c_->profiling)
    {
        if (!on) return;
        ev.kind = kind;
        for (hipEvent_t *e : {&ev.a, &ev.b}) {
            if (!c->pool.empty()) {
                *e = c->pool.back();
                c->pool.pop_back();
            } else if (hipEventCreate(e) != hipSuccess) {
                on = false;
                return;
            }
        }
        (void)hipEventRecord(ev.a, s);
    }
    ~ProfScope()
    {
        if (!on) return;
        (void)hipEventRecord(ev.b, s);
        c->events.push_back(ev);
    }
};

int hip_fail(hipError_t e, const char *what)
{
    return fail(KEYDIFF_EHIP, "%s: %s", what, hipGetErrorString(e));
}

#define KD_LAUNCH(expr, what)                                  \
    do {                                                       \
        hipError_t e__ = (expr);                               \
        if (e__ != hipSuccess) return hip_fail(e__, what);     \
    } while (0)

// Pointers and sizes every kernel of a step shares; the attention plan is filled in by plan_attention.
// `scratch`: the buffer the step's temporaries live in (the handle's own, or the static array)
kd::StepParams base_params(const keydiff_cache *c, int n, unsigned char *scratch)
{
    kd::StepParams p{};
    const keydiff_config_t &cf = c->cfg;
    p.k = c->k;
    p.v = c->v;
    p.pos = reinterpret_cast<int32_t *>(c->meta + c->L.off_pos);
    {
        double *both = reinterpret_cast<double *>(c->meta + c->L.off_ksum);
        const size_t half = (size_t)cf.batch * cf.n_kv_heads * cf.head_dim;
        p.ksum = both + (size_t)c->kpar * half;
        p.ksum_next = both + (size_t)(c->kpar ^ 1) * half;
    }
    p.status = reinterpret_cast<int32_t *>(c->meta + c->L.off_status);
    p.part_o = reinterpret_cast<_Float16 *>(scratch + c->L.off_part_o);
    p.part_ml = reinterpret_cast<float2 *>(scratch + c->L.off_part_ml);
    p.scores = reinterpret_cast<float *>(scratch + c->L.off_scores);
    p.dstmap = reinterpret_cast<int32_t *>(scratch + c->L.off_dstmap);
    p.lists = reinterpret_cast<int32_t *>(scratch + c->L.off_lists);
    p.batch = cf.batch;
    p.hq = cf.n_q_heads;
    p.hkv = cf.n_kv_heads;
    p.G = cf.n_q_heads / cf.n_kv_heads;
    p.D = cf.head_dim;
    p.n = n;
    p.N = cf.budget_N;
    p.B = cf.block_B;
    p.cap = c->L.cap;
    p.splits = 1;
    p.psplits = 1;
    p.edge_cost = 1;
    p.score_chunks = (n + kd::SCORE_ROWS - 1) / kd::SCORE_ROWS;
    if (p.score_chunks < 1) p.score_chunks = 1;
    p.lists_in_lds = kd::lists_fit_lds(n, cf.budget_N) ? 1 : 0;
    p.anchor_mode = cf.anchor_mode;
    p.layout = cf.layout;
    p.window_W = cf.window_W;
    p.scale_log2e = c->scale_log2e;
    p.eps = c->eps;
    return p;
}

#ifdef KD_TIMELINE
// Profiling build: the caller lends a device buffer for the in-kernel wall-clock stamps; launch i of
// step_main writes the records of its workgroups into slot i % slots (kTimelineWgs records of 32 words).
constexpr int kTimelineWgs = 512;
unsigned long long *g_tl_buf = nullptr;
long g_tl_slots = 0, g_tl_count = 0;
unsigned long long *timeline_slot(long wgs)   // wgs: workgroups of the launch that store a record
{
    if (!g_tl_buf || g_tl_slots < 1 || wgs > kTimelineWgs) return nullptr;   // a slot holds kTimelineWgs records
    return g_tl_buf + (size_t)(g_tl_count++ % g_tl_slots) * kTimelineWgs * 32;
}
#endif

// M tiling (GQA-packed rows per KV head) and the number of key splits that fills the chip
// `reserved`: compute units to leave to the workgroups of a carried selection
void plan_attention(const keydiff_cache *c, kd::StepParams &p, int reserved = 0)
{
    const int BH = p.batch * p.hkv;
    const int Mtot = p.G * p.Bt;
    // Workgroups of eight waves x 32 query rows, one per compute unit.  Where the rows of a head do
    // not fill the last workgroup its idle waves help (copy tiles, score rows); measured against
    // 4-wave workgroups at 64 and 128 rows per head: 29.6 vs 44.3 and 31.4 vs 47.2 us per step.  With at
    // most one wave's worth of rows (decode) two waves share the key tiles of the range between them.
    const bool alt = Mtot <= 32;
    p.NW = 8;
    const int TM = 32 * p.NW;
    p.mtiles = (Mtot + TM - 1) / TM;
    p.ntiles = (p.n + kd::TILE_KEYS - 1) / kd::TILE_KEYS;
    const int target = c->L.target_wgs / 2;   // the compute units of the chip
    // 8-wave workgroups run one per compute unit: rounding the split count up would push the last
    // workgroups into a second pass over the chip that doubles the kernel's duration
    int splits = target / (BH * p.mtiles);
    // one workgroup of 8 waves fills a compute unit: with passengers on board the attention takes
    // what is left of the chip in a single pass
    if (reserved > 0 && splits * BH * p.mtiles + reserved > target)
        splits = (target - reserved) / (BH * p.mtiles);
    if (splits > p.ntiles) splits = p.ntiles;
    if (splits < 1) splits = 1;
    // partial rows must fit the scratch sized at init
    const int Mpad = (Mtot + 31) / 32 * 32;   // partials are stored in blocks of 32 rows
    const int per = alt ? 2 : 1;              // partials a workgroup leaves per row
    while (splits > 1 && (long)per * splits * BH * Mpad > c->L.max_part_rows) --splits;
    p.splits = splits;
    p.psplits = per * splits;
    // a tile with rows of the block counts as two plain ones when the tiles are dealt out (it takes
    // about 1.4 times as long, and an equal share would make its split the last to end); every split
    // must still span at least one tile, which a span of 2 * edge_cost cost units guarantees
    const int tplain = p.len / kd::TILE_KEYS < p.ntiles ? p.len / kd::TILE_KEYS : p.ntiles;
    p.edge_cost = (tplain + 2 * (p.ntiles - tplain)) / splits >= 4 ? 2 : 1;
    const size_t merge_threads = (size_t)BH * (Mpad / 32) * (p.D / 8) * 64;
    p.merge_wgs = p.psplits > 1 ? (int)((merge_threads + kd::POST_THREADS - 1) / kd::POST_THREADS) : 0;
}

// Whether an attention launch shaped like `p` (of cache c) should take along the row shift `sp` describes,
// next to `seats_sel` workgroups of a carried selection: returns the workgroups per head to give the
// shift (0: do not), and leaves in p the plan of the attention that goes with the answer.
// The shift gets about 7/32 of the compute units (56 of 256: measured alone, 56 workgroups of this
// shape move the 66 MB of the 8192-row Llama-3.1-8B cache in 25 us, 40 in 33 us, i.e. ~48 GB/s each);
// the attention gives up key ranges for it and runs longer (12 us + 2.2 us per 64-key tile of its
// longest workgroup, from the in-kernel stamps).  Taking the shift along pays when that costs less
// than the ~12 us the shift adds to the merge launch otherwise.
int plan_with_shift(const keydiff_cache *c, kd::StepParams &p, const kd::StepParams &sp, int seats_sel)
{
    const int target = c->L.target_wgs / 2;
    plan_attention(c, p, seats_sel);
    const double att_alone = 12.0 + 2.2 * ((p.ntiles + p.splits - 1) / p.splits);
    const int heads = sp.batch * sp.hkv;
    const int nchunks = (sp.n + kd::ORD_ROWS - 1) / kd::ORD_ROWS;
    int parts = (target * 7 / 32) / heads;   // (measured at the headline shape: 5/32 42.3, 6/32 39.2, 7/32 38.6, 8/32 39.8 us per step)
    if (parts > nchunks) parts = nchunks;
    if (parts < 1 || !kd::can_host_shift(p, sp)) return 0;
    kd::StepParams ph = p;
    plan_attention(c, ph, seats_sel + parts * heads);
    if (!kd::can_host_shift(ph, sp) || ph.batch * ph.hkv * ph.mtiles * ph.splits + seats_sel + parts * heads > target) return 0;
    const double att_host = 12.0 + 2.2 * ((ph.ntiles + ph.splits - 1) / ph.splits);
    const double bytes = 2.0 * 2.0 * heads * (double)sp.n * sp.D * 2.0;   // K and V, read and written
    const double shift_us = 4.0 + bytes / (parts * heads * 48e3);
    if ((att_host > shift_us ? att_host : shift_us) >= att_alone + 12.0) return 0;
    p = ph;
    return parts;
}

bool misaligned(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) != 0; }

// ORDERED layout: the stable row shift that follows a selection, by the destination map it wrote
int compact_ordered(keydiff_cache *c, const kd::StepParams &p, hipStream_t s)
{
    ProfScope ps(c, KEYDIFF_K_COMPACT, s);
    c->epoch = c->epoch == 0x7fffffff ? 1 : c->epoch + 1;
    KD_LAUNCH(kd::launch_compact_ordered(p, reinterpret_cast<int32_t *>(c->meta + c->L.off_oflags), c->epoch, s),
              "ordered compaction kernel");
    return KEYDIFF_OK;
}

// the pending selection and compaction of `c` as a launch of its own
int finish_pending(keydiff_cache *c, hipStream_t s)
{
    if (c->shift_pending) {   // (never together with a pending selection: a new step of the cache comes through here first)
        c->shift_pending = false;
        if (int rc = compact_ordered(c, c->shift_p, c->shift_stream)) return rc;
    }
    if (!c->pending) return KEYDIFF_OK;
    kd::StepParams p = c->pend;
    p.merge_wgs = 0;
#ifdef KD_TIMELINE
    p.timeline = nullptr;   // only launches of step_main are recorded
#endif
    {
        ProfScope ps(c, KEYDIFF_K_SELECT, s);
        KD_LAUNCH(kd::launch_step_post(p, s), "step_post kernel (deferred selection)");
    }
    c->pending = false;
    if (c->cfg.layout == KEYDIFF_LAYOUT_ORDERED) return compact_ordered(c, p, s);
    return KEYDIFF_OK;
}

// `work`: the buffer for the step's temporaries -- the handle's scratch buffer, or the static array.
// Every check and every planning decision comes before the first launch, so an argument, shape or
// state error leaves nothing enqueued.
// The caller's rotary tables: float [rows][head_dim / 2] each; both null = q and k_new arrive rotated.
struct Rope {
    const float *cos_t, *sin_t;
    int64_t rows;
};

int block_step(keydiff_cache *c, const void *q, const void *k_new, const void *v_new, int32_t Bt, int64_t pos0,
               void *out, float *scores_out, bool defer, keydiff_cache *carry, unsigned char *work, hipStream_t s,
               const Rope *rope = nullptr, keydiff_cache *shifted = nullptr, bool later_launches_take_shifts = false)
{
    // shifted: another ORDERED cache whose pending row shift this step's attention launch may take along;
    // later_launches_take_shifts: the caller goes on to steps that will be offered this step's carry as
    // `shifted`, so its shift may stay pending instead of running inside this step's merge launch
    if (!c || !q || !k_new || !v_new || !out) return fail(KEYDIFF_EINVAL, "null pointer");
    if (misaligned(q) || misaligned(k_new) || misaligned(v_new) || misaligned(out))
        return fail(KEYDIFF_EINVAL, "tensors must be 16-byte aligned");
    if (Bt < 1 || Bt > c->cfg.block_B) return fail(KEYDIFF_ESHAPE, "Bt must lie in [1, block_B], got %d", Bt);
    if (pos0 < 0 || pos0 + Bt > 0x7fffffffLL) return fail(KEYDIFF_ESHAPE, "positions must fit in int32");
    if (carry == c) return fail(KEYDIFF_EINVAL, "a cache cannot carry its own eviction");
    if (rope) {
        if (!rope->cos_t || !rope->sin_t) return fail(KEYDIFF_EINVAL, "null rotary table");
        if (misaligned(rope->cos_t) || misaligned(rope->sin_t)) return fail(KEYDIFF_EINVAL, "rotary tables must be 16-byte aligned");
        if (pos0 + Bt > rope->rows) return fail(KEYDIFF_ESHAPE, "the rotary tables hold %lld positions; the block ends at %lld",
                                                (long long)rope->rows, (long long)(pos0 + Bt));
    }
    const keydiff_config_t &cf = c->cfg;
    const int len = c->len, n = len + Bt, N = cf.budget_N;
    const bool contiguous = c->contiguous && (c->next_pos < 0 || c->next_pos == pos0);
    if (cf.window_W > 0 && n > N && !contiguous)
        return fail(KEYDIFF_ESTATE, "the sliding window needs consecutive token positions across calls");

    const bool evict = n > N;
    kd::StepParams p = base_params(c, n, work);
    p.q = static_cast<const uint16_t *>(q);
    p.k_new = static_cast<const uint16_t *>(k_new);
    p.v_new = static_cast<const uint16_t *>(v_new);
    p.out = static_cast<uint16_t *>(out);
    p.scores_out = scores_out;
    p.Bt = Bt;
    p.len = len;
    p.pos0 = (int32_t)pos0;
    p.do_evict = evict;
    p.do_score = evict || scores_out != nullptr;
    if (cf.window_W > 0) p.window_pos_min = (int32_t)(pos0 + Bt - cf.window_W);

    // a passenger rides only if the attention still fits the chip in one pass beside it
    bool riding = false;
    const bool sel_offered = carry && carry->pending && carry->pend_stream == s;
    const int seats = sel_offered ? carry->cfg.batch * carry->cfg.n_kv_heads : 0;
    // ... first the row shift of `shifted` (with the selection, if one is offered and fits as well)
    int shift_parts = 0;
    if (shifted && shifted != c && shifted != carry && shifted->shift_pending && shifted->shift_stream == s) {
        shift_parts = plan_with_shift(c, p, shifted->shift_p, seats);
        if (shift_parts > 0 && sel_offered) {
            if (kd::can_carry(p, carry->pend)) riding = true;
            else shift_parts = 0;   // (the selection is the passenger that must not be left behind)
        }
    }
    if (shift_parts == 0 && sel_offered) {
        plan_attention(c, p, seats);
        riding = kd::can_carry(p, carry->pend) &&
                 p.batch * p.hkv * p.mtiles * p.splits + seats <= c->L.target_wgs / 2;
    }
    if (shift_parts == 0 && !riding) plan_attention(c, p);
    const int shift_wgs = shift_parts > 0 ? shift_parts * shifted->shift_p.batch * shifted->shift_p.hkv : 0;
    // Generation phase: the attention launch's scoring waves (the kernels with helper waves) leave the
    // arg-max of the scores per workgroup, and the selection reads the row to evict off those records.
    if (evict && n - N == 1 && cf.window_W == 0 && cf.layout == KEYDIFF_LAYOUT_FILL &&
        p.mtiles * 32 * p.NW - p.G * p.Bt >= 32 && (size_t)p.batch * p.hkv * p.splits <= (size_t)c->L.target_wgs + p.batch * p.hkv)
        p.argmax_rec = reinterpret_cast<unsigned long long *>(work + c->L.off_argmax);

    // ---- launches from here on
    if (rope) {
        // Fig. 1 step (1), as far as it lies inside this boundary: rotate the block's queries and keys
        uint16_t *q_rot = reinterpret_cast<uint16_t *>(work + c->L.off_q_rot);
        uint16_t *k_rot = reinterpret_cast<uint16_t *>(work + c->L.off_k_rot);
        ProfScope ps(c, KEYDIFF_K_AUX, s);
        KD_LAUNCH(kd::launch_rope(p.q, p.k_new, q_rot, k_rot, rope->cos_t, rope->sin_t, cf.batch * cf.n_q_heads * Bt,
                                  cf.batch * cf.n_kv_heads * Bt, Bt, cf.head_dim, (int32_t)pos0, s),
                  "rotary embedding kernel");
        p.q = q_rot;
        p.k_new = k_rot;
    }
    if (int rc = finish_pending(c, s)) return rc;   // this step reads the compacted cache
    if (carry && carry->pending && !riding)
        if (int rc = finish_pending(carry, carry->pend_stream)) return rc;
#ifdef KD_TIMELINE
    p.timeline = timeline_slot((long)p.batch * p.hkv * p.mtiles * p.splits + (riding ? carry->pend.batch * carry->pend.hkv : 0) + shift_wgs);
#endif
    {
        ProfScope ps(c, KEYDIFF_K_MAIN, s);
        if (shift_parts > 0) {
            kd::ShiftRide ride;
            ride.p = shifted->shift_p;
            ride.flags = reinterpret_cast<int32_t *>(shifted->meta + shifted->L.off_oflags);
            ride.nchunks = (ride.p.n + kd::ORD_ROWS - 1) / kd::ORD_ROWS;
            ride.parts = shift_parts;
            ride.nshift = shift_wgs;
            shifted->epoch = shifted->epoch == 0x7fffffff ? 1 : shifted->epoch + 1;
            ride.epoch = shifted->epoch;
            KD_LAUNCH(kd::launch_step_main_ride(p, riding ? &carry->pend : nullptr, ride, s),
                      "step_main kernel (with carried selection and row shift)");
            shifted->shift_pending = false;
            if (riding) carry->pending = false;
        } else if (riding) {
            KD_LAUNCH(kd::launch_step_main_carry(p, carry->pend, s), "step_main kernel (with carried selection)");
            carry->pending = false;
        } else {
            KD_LAUNCH(kd::launch_step_main(p, s), "step_main kernel");
        }
    }
    const bool deferred = defer && evict;
    // a selection that rode in this step's attention launch wrote its destination map: the rows of an
    // ORDERED carrier's cache are shifted after that launch -- inside this step's merge launch where
    // there is one (the shift is bound by memory traffic, the merge leaves the memory system idle)
    bool shift_owed = riding && carry->cfg.layout == KEYDIFF_LAYOUT_ORDERED;
    // ... or, when the caller goes on to launches that can take it along, inside one of those
    if (shift_owed && later_launches_take_shifts) {
        kd::StepParams probe = p;
        if (plan_with_shift(c, probe, carry->pend, seats) > 0) {   // (a later launch is taken to look like this one)
            carry->shift_pending = true;
            carry->shift_p = carry->pend;
            carry->shift_stream = s;
            shift_owed = false;
        }
    }
    if (deferred) {
        if (p.merge_wgs > 0) {
            kd::StepParams pm = p;
            pm.do_evict = 0;   // the merge half of step_post only
            ProfScope ps(c, KEYDIFF_K_POST, s);
            if (shift_owed && carry->pend.D == p.D) {
                carry->epoch = carry->epoch == 0x7fffffff ? 1 : carry->epoch + 1;
                KD_LAUNCH(kd::launch_merge_shift(pm, carry->pend, reinterpret_cast<int32_t *>(carry->meta + carry->L.off_oflags),
                                                 carry->epoch, s),
                          "merge + ordered compaction kernel");
                shift_owed = false;
            } else {
                KD_LAUNCH(kd::launch_step_post(pm, s), "step_post kernel (merge)");
            }
        }
        c->pending = true;
        c->pend = p;
        c->pend_stream = s;
    } else if (evict || p.merge_wgs > 0) {
#ifdef KD_TIMELINE
        p.timeline = timeline_slot((long)(evict ? p.batch * p.hkv : 0) + p.merge_wgs);   // step_post records into the next slot
#endif
        ProfScope ps(c, KEYDIFF_K_POST, s);
        KD_LAUNCH(kd::launch_step_post(p, s), "step_post kernel");
    }
    if (evict && !deferred && cf.layout == KEYDIFF_LAYOUT_ORDERED)
        if (int rc = compact_ordered(c, p, s)) return rc;
    if (shift_owed)   // ... else in a launch of its own
        if (int rc = compact_ordered(carry, carry->pend, s)) return rc;
    if (c->profiling) ProfScope ps(c, KEYDIFF_K_EVENT_PAIR, s);
    c->plan[0] = p.psplits;
    c->plan[1] = p.mtiles;
    c->plan[2] = p.ntiles;
    c->plan[3] = (riding ? 1 : 0) | (shift_parts > 0 ? 2 : 0);
    c->kpar ^= 1;   // step_main wrote the new key sum into the other half
    c->len = evict ? N : n;
    c->contiguous = contiguous;
    c->next_pos = pos0 + Bt;
    return KEYDIFF_OK;
}

}  // namespace

extern "C" {

int keydiff_version(void) { return KEYDIFF_VERSION; }

const char *keydiff_last_error(void) { return g_err; }

int keydiff_workspace_bytes(const keydiff_config_t *cfg, size_t *k_bytes, size_t *v_bytes, size_t *meta_bytes,
                            size_t *scratch_bytes)
{
    if (int rc = check_config(cfg)) return rc;
    if (!k_bytes || !v_bytes || !meta_bytes || !scratch_bytes) return fail(KEYDIFF_EINVAL, "null output pointer");
    const Layout L = make_layout(cfg);
    *k_bytes = L.k_bytes;
    *v_bytes = L.k_bytes;
    *meta_bytes = L.meta_bytes;
    *scratch_bytes = L.scratch_bytes;
    return KEYDIFF_OK;
}

int keydiff_init_cache(const keydiff_config_t *cfg, void *k_cache, void *v_cache, void *meta, void *scratch,
                       void *stream, keydiff_cache_t **out)
{
    if (int rc = check_config(cfg)) return rc;
    if (!k_cache || !v_cache || !meta || !scratch || !out) return fail(KEYDIFF_EINVAL, "null pointer");
    for (const void *p : {k_cache, v_cache, meta, scratch})
        if (reinterpret_cast<uintptr_t>(p) & 255) return fail(KEYDIFF_EINVAL, "buffers must be 256-byte aligned");
    keydiff_cache *c = new (std::nothrow) keydiff_cache();
    if (!c) return fail(KEYDIFF_EINVAL, "out of host memory");
    c->cfg = *cfg;
    c->L = make_layout(cfg);
    c->k = static_cast<uint16_t *>(k_cache);
    c->v = static_cast<uint16_t *>(v_cache);
    c->meta = static_cast<unsigned char *>(meta);
    c->scratch = static_cast<unsigned char *>(scratch);
    c->device = -1;
    if (hipGetDevice(&c->device) != hipSuccess) {
        delete c;
        return fail(KEYDIFF_EHIP, "no current device");
    }
    {   // once per device, with that device current: where this GPU holds the static scratch array.
        // A failed lookup only disables keydiff_prefill_block_static, which then reports it.
        unsigned char *unused = nullptr;
        (void)static_scratch_of(c->device, &unused);
    }
    c->len = 0;  // C_0 is empty
    c->eps = cfg->eps > 0.f ? (double)cfg->eps : 1e-8;
    const double scale = cfg->softmax_scale > 0.f ? (double)cfg->softmax_scale : 1.0 / std::sqrt((double)cfg->head_dim);
    c->scale_log2e = (float)(scale * 1.4426950408889634);
    c->contiguous = true;
    c->next_pos = -1;
    c->profiling = false;
    c->kpar = 0;
    c->epoch = 0;
    c->pending = false;
    c->shift_pending = false;
    c->pend_stream = nullptr;
    for (int32_t &x : c->plan) x = 0;
    static hipError_t configured = kd::configure_kernels();  // once per process
    hipError_t e = configured;
    if (e == hipSuccess)
        e = kd::launch_zero_words(reinterpret_cast<int32_t *>(meta), c->L.meta_bytes / 4,
                                  static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
        delete c;
        return hip_fail(e, "kernel setup / clearing metadata");
    }
    *out = c;
    return KEYDIFF_OK;
}

void keydiff_destroy_cache(keydiff_cache_t *c)
{
    if (!c) return;
    (void)finish_pending(c, c->pend_stream);   // the caller's buffers end up compacted
    for (auto &ev : c->events) {
        (void)hipEventDestroy(ev.a);
        (void)hipEventDestroy(ev.b);
    }
    for (auto &e : c->pool) (void)hipEventDestroy(e);
    delete c;
}

int keydiff_cache_len(const keydiff_cache_t *c, int32_t *len)
{
    if (!c || !len) return fail(KEYDIFF_EINVAL, "null pointer");
    *len = c->len;
    return KEYDIFF_OK;
}

int keydiff_cache_plan(const keydiff_cache_t *c, int32_t plan_out[4])
{
    if (!c || !plan_out) return fail(KEYDIFF_EINVAL, "null pointer");
    for (int i = 0; i < 4; ++i) plan_out[i] = c->plan[i];
    return KEYDIFF_OK;
}

int keydiff_prefill_block(keydiff_cache_t *c, const void *q, const void *k_new, const void *v_new, int32_t Bt,
                          int64_t pos0, void *out, float *scores_out, void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    return block_step(c, q, k_new, v_new, Bt, pos0, out, scores_out, false, nullptr, c->scratch,
                      static_cast<hipStream_t>(stream));
}

int keydiff_prefill_block_rope(keydiff_cache_t *c, const void *q, const void *k_new, const void *v_new, int32_t Bt,
                               int64_t pos0, const float *cos_table, const float *sin_table, int64_t table_rows, void *out,
                               float *scores_out, void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    const Rope rope{cos_table, sin_table, table_rows};
    return block_step(c, q, k_new, v_new, Bt, pos0, out, scores_out, false, nullptr, c->scratch,
                      static_cast<hipStream_t>(stream), &rope);
}

int keydiff_prefill_block_static(keydiff_cache_t *c, const void *q, const void *k_new, const void *v_new, int32_t Bt,
                                 int64_t pos0, void *out, float *scores_out, void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    if (c->L.scratch_bytes > (size_t)KEYDIFF_STATIC_SCRATCH_BYTES)
        return fail(KEYDIFF_ESHAPE, "this configuration needs %zu bytes of scratch; the static array holds %zu",
                    c->L.scratch_bytes, (size_t)KEYDIFF_STATIC_SCRATCH_BYTES);
    // the address was looked up when the handle was created, with its device current
    unsigned char *work = c->device >= 0 && c->device < kMaxDevices ? g_static_scratch[c->device] : nullptr;
    if (!work) return fail(KEYDIFF_ESTATE, "the static scratch array of device %d was not found at init", c->device);
    return block_step(c, q, k_new, v_new, Bt, pos0, out, scores_out, false, nullptr, work,
                      static_cast<hipStream_t>(stream));
}

int keydiff_prefill_block_deferred(keydiff_cache_t *c, const void *q, const void *k_new, const void *v_new, int32_t Bt,
                                   int64_t pos0, void *out, keydiff_cache_t *carry, void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    return block_step(c, q, k_new, v_new, Bt, pos0, out, nullptr, true, carry, c->scratch,
                      static_cast<hipStream_t>(stream));
}

static int block_layers(keydiff_cache_t *const *caches, int32_t n_layers, const void *const *q, const void *const *k_new,
                        const void *const *v_new, int32_t Bt, int64_t pos0, void *const *out, void *stream, const Rope *rope)
{
    if (!caches || !q || !k_new || !v_new || !out) return fail(KEYDIFF_EINVAL, "null pointer");
    if (n_layers < 1) return fail(KEYDIFF_ESHAPE, "n_layers must be positive, got %d", n_layers);
    for (int l = 0; l < n_layers; ++l) {
        if (!caches[l] || !q[l] || !k_new[l] || !v_new[l] || !out[l])
            return fail(KEYDIFF_EINVAL, "null pointer for layer %d", l);
        for (int m = 0; m < l; ++m)
            if (caches[m] == caches[l]) return fail(KEYDIFF_EINVAL, "layers %d and %d share a cache", m, l);
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    for (int l = 0; l < n_layers; ++l) {
        // layer 0 takes along what the last layer left pending at the previous block
        keydiff_cache *carry = n_layers > 1 ? caches[(l + n_layers - 1) % n_layers] : nullptr;
        // ... and, ORDERED layout, the row shift of the layer before that one, whose selection rode in the
        // launch of the layer between them
        keydiff_cache *shifted = n_layers > 2 ? caches[(l + n_layers - 2) % n_layers] : nullptr;
        if (int rc = block_step(caches[l], q[l], k_new[l], v_new[l], Bt, pos0, out[l], nullptr, true, carry,
                                caches[l]->scratch, s, rope, shifted, n_layers > 2))
            return rc;
    }
    return KEYDIFF_OK;
}

int keydiff_prefill_block_layers(keydiff_cache_t *const *caches, int32_t n_layers, const void *const *q,
                                 const void *const *k_new, const void *const *v_new, int32_t Bt, int64_t pos0,
                                 void *const *out, void *stream)
{
    return block_layers(caches, n_layers, q, k_new, v_new, Bt, pos0, out, stream, nullptr);
}

int keydiff_prefill_block_layers_rope(keydiff_cache_t *const *caches, int32_t n_layers, const void *const *q,
                                      const void *const *k_new, const void *const *v_new, int32_t Bt, int64_t pos0,
                                      const float *cos_table, const float *sin_table, int64_t table_rows,
                                      void *const *out, void *stream)
{
    const Rope rope{cos_table, sin_table, table_rows};
    return block_layers(caches, n_layers, q, k_new, v_new, Bt, pos0, out, stream, &rope);
}

int keydiff_finish(keydiff_cache_t *c, void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    return finish_pending(c, static_cast<hipStream_t>(stream));
}

int keydiff_decode_step(keydiff_cache_t *c, const void *q, const void *k_new, const void *v_new, int64_t pos,
                        void *out, void *stream)
{
    return keydiff_prefill_block(c, q, k_new, v_new, 1, pos, out, nullptr, stream);
}

int keydiff_scores(const keydiff_cache_t *cc, float *scores_out, void *stream)
{
    if (!cc) return fail(KEYDIFF_EINVAL, "null pointer");
    if (cc->len == 0) return fail(KEYDIFF_ESTATE, "the cache is empty");
    if (!scores_out) return fail(KEYDIFF_EINVAL, "null pointer");
    keydiff_cache *c = const_cast<keydiff_cache *>(cc);  // scratch, profiling events, a pending eviction
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int rc = finish_pending(c, s)) return rc;
    kd::StepParams p = base_params(c, c->len, c->scratch);
    p.scores_out = scores_out;
    p.do_score = 1;
    p.do_evict = 0;
    p.merge_wgs = 0;
    ProfScope ps(c, KEYDIFF_K_SCORE, s);
    KD_LAUNCH(kd::launch_step_score(p, s), "step_score kernel");
    return KEYDIFF_OK;
}

int keydiff_cache_positions(const keydiff_cache_t *c, int32_t *pos_out, void *stream)
{
    if (!c || !pos_out) return fail(KEYDIFF_EINVAL, "null pointer");
    if (int rc = finish_pending(const_cast<keydiff_cache *>(c), static_cast<hipStream_t>(stream))) return rc;
    KD_LAUNCH(kd::launch_load_pos(reinterpret_cast<const int32_t *>(c->meta + c->L.off_pos), pos_out,
                                  c->cfg.batch * c->cfg.n_kv_heads, c->L.cap, c->len, 0,
                                  static_cast<hipStream_t>(stream)),
              "position copy");
    return KEYDIFF_OK;
}

int keydiff_cache_load(keydiff_cache_t *c, const void *k, const void *v, const int32_t *pos, int32_t len,
                       void *stream)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    if (len < 0 || len > c->cfg.budget_N) return fail(KEYDIFF_ESHAPE, "len must lie in [0, budget_N]");
    if (len > 0 && (!k || !v || !pos)) return fail(KEYDIFF_EINVAL, "null pointer");
    if (len > 0 && (misaligned(k) || misaligned(v))) return fail(KEYDIFF_EINVAL, "tensors must be 16-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int rc = finish_pending(c, s)) return rc;
    const int BH = c->cfg.batch * c->cfg.n_kv_heads, D = c->cfg.head_dim;
    KD_LAUNCH(kd::launch_load_rows(static_cast<const uint16_t *>(k), c->k, BH, c->L.cap, D, len, s), "cache load");
    KD_LAUNCH(kd::launch_load_rows(static_cast<const uint16_t *>(v), c->v, BH, c->L.cap, D, len, s), "cache load");
    KD_LAUNCH(kd::launch_load_pos(pos, reinterpret_cast<int32_t *>(c->meta + c->L.off_pos), BH, c->L.cap, len, 1, s),
              "cache load");
    {
        kd::StepParams p = base_params(c, len, c->scratch);
        ProfScope ps(c, KEYDIFF_K_AUX, s);
        KD_LAUNCH(kd::launch_ksum_rebuild(p, reinterpret_cast<double *>(c->scratch + c->L.off_ksum_part), s),
                  "key sum rebuild");
    }
    c->len = len;
    c->contiguous = false;  // the loaded positions are the caller's
    c->next_pos = -1;
    return KEYDIFF_OK;
}

int keydiff_cache_status(const keydiff_cache_t *c, int32_t *status_out, void *stream)
{
    if (!c || !status_out) return fail(KEYDIFF_EINVAL, "null pointer");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (int rc = finish_pending(const_cast<keydiff_cache *>(c), s)) return rc;
    hipError_t e = hipMemcpyAsync(status_out, c->meta + c->L.off_status, 4, hipMemcpyDeviceToHost, s);
    if (e != hipSuccess) return hip_fail(e, "status copy");
    e = hipStreamSynchronize(s);
    if (e != hipSuccess) return hip_fail(e, "stream synchronize");
    return KEYDIFF_OK;
}

int keydiff_profile_enable(keydiff_cache_t *c, int32_t enable)
{
    if (!c) return fail(KEYDIFF_EINVAL, "null pointer");
    c->profiling = enable != 0;
    return KEYDIFF_OK;
}

int keydiff_profile_read(keydiff_cache_t *c, float *ms_out, int32_t *launches_out)
{
    if (!c || !ms_out || !launches_out) return fail(KEYDIFF_EINVAL, "null pointer");
    for (int i = 0; i < KEYDIFF_NKERNELS; ++i) {
        ms_out[i] = 0.f;
        launches_out[i] = 0;
    }
    for (auto &ev : c->events) {
        hipError_t e = hipEventSynchronize(ev.b);
        if (e != hipSuccess) return hip_fail(e, "event synchronize");
        float ms = 0.f;
        e = hipEventElapsedTime(&ms, ev.a, ev.b);
        if (e != hipSuccess) return hip_fail(e, "event elapsed time");
        ms_out[ev.kind] += ms;
        launches_out[ev.kind] += 1;
        c->pool.push_back(ev.a);
        c->pool.push_back(ev.b);
    }
    c->events.clear();
    return KEYDIFF_OK;
}

#ifdef KD_TIMELINE
// Profiling build only (not part of include/keydiff.h): buf is device memory of `bytes` bytes, zeroed by
// the caller; returns the number of launch slots it holds.  Pass NULL to stop recording.
KEYDIFF_API long keydiff_timeline_buffer(void *buf, size_t bytes)
{
    g_tl_buf = static_cast<unsigned long long *>(buf);
    g_tl_slots = buf ? (long)(bytes / ((size_t)kTimelineWgs * 32 * 8)) : 0;
    g_tl_count = 0;
    return g_tl_slots;
}
KEYDIFF_API long keydiff_timeline_launches(void) { return g_tl_count; }
#endif

}  // extern "C"
