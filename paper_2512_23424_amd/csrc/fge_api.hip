// Host side of the C ABI declared in include/fge.h: argument validation (before anything is
// launched), tile selection, workspace layout and the kernel launches on the caller's stream.
#include <hip/hip_runtime.h>

#include <atomic>
#include <chrono>

#include <cmath>
#include <vector>

#include "fge_launch.h"
#include "fge_rowops.h"
#include "fge_tile_table.h"

using namespace fge;

// Scratch of the entry point for callers that cannot allocate (fused_gemm_epilogue_static): one
// array per GPU, part of the code object, held until the process ends.  In host code the name
// below is only a handle; the device address is asked from the runtime once per device.
static __device__ __align__(256) unsigned char scratch[FGE_STATIC_SCRATCH_BYTES];

namespace {

thread_local int g_last_hip = 0;
// Rows of W that exist when that is fewer than the problem's N (set around the inner call of the
// repacked path, see run_repacked; 0: N)
thread_local int g_w_rows = 0;

// Launch counter: its value marks "arrived" in the cooperative form, so marks left in a
// workspace by earlier launches (or by whatever the memory held before) never match.
std::atomic<unsigned> g_generation{
    (unsigned)std::chrono::steady_clock::now().time_since_epoch().count() * 2654435761u};

// Compute units of the current device, asked once (MI355X: 8 XCDs x 32 = 256, which is also the
// answer where no device can be asked - the planning functions are callable without one).
int num_cu() {
    static const int n = [] {
        int dev = 0, cus = 0;
        if (hipGetDevice(&dev) != hipSuccess) return 256;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return 256;
        return cus;
    }();
    return n;
}
constexpr unsigned WAIT_POLLS = 1u << 20;   // polls after which a tile stops waiting for its row block
constexpr int MAX_ROWOP_N = 8192;    // a row must fit the register-resident row kernels
constexpr int MAX_SPLIT = 8192;      // column strips per row the second pass will merge (wider rows: element-granular kernels)

inline size_t esize(int dt) { return dt == FGE_F32 ? 4 : dt == FGE_F8E4M3 ? 1 : 2; }
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

// Shape after folding a dense batch into the row count.
struct Problem {
    int M, N, K, batch;
    int64_t ldx, ldw, ldo, bsx, bso;
};

struct Plan {
    Problem pr;
    int tile;
    int tiles_m, tiles_n;
    int strips;                  // statistics slots per row: column tiles x waves across a tile
    bool split;                  // rows split over several column tiles and a row op is requested
    bool coop;                   // ... and the tiles finish their rows themselves (one kernel)
    int coop_grid;               // workgroups of the cooperative launch
    bool needs_finish;           // ... or a second pass does
    size_t ws_stats;             // bytes of per-strip statistics (fused)
    size_t ws_marks;             // bytes of arrival marks + fault word (cooperative form)
    size_t ws_buf;               // bytes of one out-shaped intermediate (unfused)
    int n_bufs;                  // intermediates the unfused path needs
    bool generic;                // the element-granular kernels run this problem
    size_t ws_generic;           // fused, generic: bytes of the fp32 rows x N intermediate
};

// Tile asked for through the flags (FGE_FLAG_TILE), -1 for the automatic choice.
inline int forced_tile(const fge_params *p) { return ((p->flags & FGE_FLAG_TILE_MASK) >> 8) - 1; }

// A forced tile must be one that has kernels for the operand type; the narrow-K kernel also
// keeps its shape limits.
bool forced_tile_ok(const fge_params *p) {
    const int t = forced_tile(p);
    if (t < 0) return true;
    const bool f32 = p->in_dtype == FGE_F32;
    switch (t) {
    case TILE_64x64: case TILE_64x512: return true;
    case TILE_128x128: return !f32 || !(p->flags & FGE_FLAG_IEEE_FP32);   // fp32: split product only
    case TILE_256x256: return !f32;
    case TILE_64x128: return f32;
    case TILE_128x256: case TILE_256x128: return !f32;
    case TILE_128x128_W8: return f32 && !(p->flags & FGE_FLAG_IEEE_FP32);
    case TILE_128x128_S3: return !f32;
    case TILE_PANEL:
        return f32 && !(p->flags & FGE_FLAG_IEEE_FP32) && p->K <= 64 && p->N <= 512 &&
               (p->batch == 1 || (p->batch_stride_x == (int64_t)p->M * p->ldx && p->batch_stride_o == (int64_t)p->M * p->ldo));
    default: return false;
    }
}

// Checks everything that does not depend on the path (fused / stage) being run.
int check_common(const fge_params *p, int act, int norm, bool need_in) {
    if (p == nullptr) return FGE_ERR_NULL;
    if (act < FGE_ACT_NONE || act > FGE_ACT_CLAMP) return FGE_ERR_BAD_ENUM;
    if (norm < FGE_NORM_NONE || norm > FGE_NORM_LOGSUMEXP) return FGE_ERR_BAD_ENUM;
    if (p->flags & ~(FGE_FLAG_TWO_PASS | FGE_FLAG_IEEE_FP32 | FGE_FLAG_NO_SPLIT_K | FGE_FLAG_TILE_MASK | FGE_FLAG_TEST_EXPIRE_WAIT | FGE_FLAG_NO_TABLE))
        return FGE_ERR_BAD_ENUM;
    if (!forced_tile_ok(p)) return FGE_ERR_UNSUPPORTED;
    if (p->in_dtype < FGE_F32 || p->in_dtype > FGE_F8E4M3 || p->out_dtype < FGE_F32 || p->out_dtype > FGE_F8E4M3)
        return FGE_ERR_BAD_ENUM;
    if (p->out_dtype == FGE_F8E4M3) return FGE_ERR_UNSUPPORTED;     // an operand type only
    // out is fp32 or the 16-bit type that goes with the operands (bf16 with fp32 / bf16 / fp8, fp16 with fp16)
    if (need_in && p->out_dtype != FGE_F32 && p->out_dtype != (p->in_dtype == FGE_F16 ? FGE_F16 : FGE_BF16))
        return FGE_ERR_UNSUPPORTED;
    if (p->M <= 0 || p->N <= 0 || p->K <= 0 || p->batch <= 0) return FGE_ERR_BAD_SHAPE;
    if (p->ldo < p->N) return FGE_ERR_BAD_SHAPE;
    if (need_in && (p->ldx < p->K || p->ldw < p->K)) return FGE_ERR_BAD_SHAPE;
    if (p->batch > 1) {
        if (p->batch_stride_o < (int64_t)(p->M - 1) * p->ldo + p->N) return FGE_ERR_BAD_SHAPE;
        if (need_in && p->batch_stride_x < (int64_t)(p->M - 1) * p->ldx + p->K) return FGE_ERR_BAD_SHAPE;
    }
    if (!aligned16(p->gamma) || !aligned16(p->beta) || !aligned16(p->aux_out) || !aligned16(p->workspace))
        return FGE_ERR_ALIGN;
    if ((int64_t)p->M * p->batch > (int64_t)INT32_MAX / 2) return FGE_ERR_UNSUPPORTED;
    return FGE_OK;
}

// Whether the vectorised kernels take this problem: every extent and stride they move in
// 16-byte units must be a multiple of 16 bytes (base pointers are checked separately), and a
// row operation on its own (need_in false: the unfused K3, fge_row_op) needs the row to fit a
// wave's registers - the fused tile kernels split rows of any width over column tiles.
// Everything else goes to the element-granular kernels.
// An operand (row stride ld, stride bs between problems, both in elements) as the tile kernels
// can stage it where it lies: K, ld and bs whole 16-byte units, and rows less than 8 MiB apart
// (a row is addressed by a 32-bit byte offset from the first row of its tile, at most 256 rows).
bool operand_ok(const fge_params *p, int64_t ld, int64_t bs) {
    const int64_t is = (int64_t)esize(p->in_dtype);
    constexpr int64_t SPAN = ((int64_t)1 << 31) / 256;
    return (p->K * is) % 16 == 0 && (ld * is) % 16 == 0 && (bs * is) % 16 == 0 && ld * is < SPAN;
}

bool vectorisable(const fge_params *p, int norm, bool need_in) {
    const size_t os = esize(p->out_dtype);
    if ((p->N * os) % 16 || (p->ldo * os) % 16) return false;
    if (p->batch > 1 && (p->batch_stride_o * os) % 16) return false;
    if (need_in && (!operand_ok(p, p->ldx, p->batch > 1 ? p->batch_stride_x : 0) || !operand_ok(p, p->ldw, 0))) return false;
    if (norm != FGE_NORM_NONE && !need_in && p->N > MAX_ROWOP_N) return false;
    return true;
}

constexpr int PANEL_MIN_ROWS = 4096;   // below this the persistent kernel cannot fill the chip

// Tile choice (checked against an exhaustive search over the configurations on a sweep of
// shapes).  The rule is the same everywhere: the largest tile of the operand type's list that
// still gives every CU a workgroup and is not much wider than the row; whether the rows end up
// split over column tiles matters little, since split rows cost one small exchange.
// 16- and 8-bit operands first ask the table that the configuration search wrote
// (fge_tile_table.h: the fastest verified configuration at each point of a sweep over shapes): the
// entry nearest to the problem - in 256-row and 256-column tiles and in K, on a log2 scale, with
// the same operand class and the same answer to "does a row op follow" - decides when it lies
// within a factor of about 1.5 of the problem in total; elsewhere, and where the rule below is
// asked for by the caller, the rule decides.
// Rounds of the chip a tiling of rows x cols outputs takes: workgroups over the workgroups the
// chip holds at once (two per CU for tiles of up to 128x128, else one).
int64_t tile_rounds(int t, int64_t rows, int64_t cols, int batch) {
    const TileInfo &ti = tile_info(t);
    const int64_t count = ((rows + ti.bm - 1) / ti.bm) * ((cols + ti.bn - 1) / ti.bn) * batch;
    const int64_t capacity = (int64_t)num_cu() * (ti.bm * ti.bn <= 128 * 128 ? 2 : 1);
    return (count + capacity - 1) / capacity;
}

// The nearest table entry of the problem's class whose tile configuration takes as many rounds
// of the chip on this problem as it took at the entry's own shape: a find made where a tiling
// just filled the chip says nothing about a slightly larger problem that spills into a second
// round.
const TileTableEntry *table_entry(const Problem &pr, int in_dtype, int norm) {
    if (in_dtype == FGE_F32) return nullptr;
    const int cls = in_dtype == FGE_F8E4M3 ? 1 : 0, rowop = norm != FGE_NORM_NONE;
    // the answer for the shapes a caller keeps coming back with is remembered (per thread)
    struct Memo { int cls, rowop, M, N, K, batch; const TileTableEntry *hit; bool valid; };
    thread_local Memo memo[16] = {};
    Memo &slot = memo[((unsigned)pr.M * 2654435761u ^ (unsigned)pr.N * 40503u ^ (unsigned)pr.K * 9176u ^ (unsigned)(cls * 2 + rowop)) >> 28];
    if (slot.valid && slot.cls == cls && slot.rowop == rowop && slot.M == pr.M && slot.N == pr.N && slot.K == pr.K &&
        slot.batch == pr.batch)
        return slot.hit;
    // log2 of every entry's coordinates, once
    struct Lg { float mt, nt, k; };
    static const std::vector<Lg> lg = [] {
        std::vector<Lg> v;
        for (const TileTableEntry &e : TILE_TABLE)
            v.push_back(Lg{std::log2((float)(e.mt ? e.mt : 1)), std::log2((float)(e.nt ? e.nt : 1)), std::log2((float)(e.K ? e.K : 1))});
        return v;
    }();
    const float mt = std::log2((float)((pr.M + 255) / 256) * pr.batch), nt = std::log2((float)((pr.N + 255) / 256)),
                k = std::log2((float)pr.K);
    float best = 0.6f;
    const TileTableEntry *hit = nullptr;
    size_t i = 0;
    for (const TileTableEntry &e : TILE_TABLE) {
        const Lg &l = lg[i++];
        if (e.cls != cls || e.rowop != rowop || e.tile >= TILE_COUNT) continue;
        const float d = std::fabs(mt - l.mt) + std::fabs(nt - l.nt) + std::fabs(k - l.k);
        if (d >= best) continue;
        if (tile_rounds(e.tile, pr.M, pr.N, pr.batch) != tile_rounds(e.tile, (int64_t)e.mt * 256, (int64_t)e.nt * 256, 1)) continue;
        best = d;
        hit = &e;
    }
    slot = Memo{cls, rowop, pr.M, pr.N, pr.K, pr.batch, hit, true};
    return hit;
}

int rule_tile(const Problem &pr, int in_dtype, bool ieee_fp32);

// use_table false: the rule alone (FGE_FLAG_NO_TABLE - what the search compares its finds with).
int pick_tile(const Problem &pr, int in_dtype, int norm, bool ieee_fp32, bool use_table = true) {
    const int rule = rule_tile(pr, in_dtype, ieee_fp32);
    if (!use_table) return rule;
    // few 64x64 tiles and a long K: the K slices (k_split) build on that tile - the table was swept
    // with K left whole and has no say here
    const int64_t t64 = (int64_t)((pr.M + 63) / 64) * ((pr.N + 63) / 64) * pr.batch;
    if (rule == TILE_64x64 && t64 <= num_cu() && pr.K >= 2048) return rule;
    if (const TileTableEntry *e = table_entry(pr, in_dtype, norm)) {
        const int t = e->tile;
        if (t < TILE_COUNT && t != TILE_PANEL && t != TILE_64x128 && t != TILE_GATED &&
            tile_info(t).bn <= (pr.N > 32 ? 2 * pr.N : 64))
            return t;
    }
    return rule;
}

int rule_tile(const Problem &pr, int in_dtype, bool ieee_fp32) {
    auto count = [&](int t) {
        const TileInfo &ti = tile_info(t);
        return (int64_t)((pr.M + ti.bm - 1) / ti.bm) * ((pr.N + ti.bn - 1) / ti.bn) * pr.batch;
    };
    auto fits = [&](int t) { return tile_info(t).bn <= (pr.N > 32 ? 2 * pr.N : 64); };
    if (in_dtype == FGE_F32) {
        // narrow K, a row of 257..512 columns (all eight waves of the kernel busy), many rows:
        // bound by the output stream; the kernel for it exists with the split product only
        if (!ieee_fp32 && pr.K <= 64 && pr.N > 256 && pr.N <= 512 && pr.batch == 1 && pr.M >= PANEL_MIN_ROWS)
            return TILE_PANEL;
        // 128x128 tiles (split product only): a third less operand traffic from the L2s than 64x128
        // tiles - fp32 operands make the staging, not the MFMAs, the bound of these kernels.  With
        // more of them than CUs: four waves each, two workgroups per CU.  With one per CU at most:
        // eight waves each (the four-wave form leaves each SIMD a single wave there and nothing to
        // run under its stalls; 4096 x 1024 x 1024: 41.1 -> 36.8 us), and that already from 5/8 of
        // the CUs on (2560 x 1024 x 1024, 160 tiles: 31.9 us against 37.3 us on 64x64 tiles; at 128
        // tiles the small tiles still win, 29.2 against 31.4 us)
        if (!ieee_fp32 && fits(TILE_128x128)) {
            if (count(TILE_128x128) > num_cu()) return TILE_128x128;
            if (count(TILE_128x128) * 8 >= num_cu() * 5) return TILE_128x128_W8;
        }
        // fp32 instruction, very large problems: the wide tile halves the operand traffic per flop
        if (ieee_fp32 && fits(TILE_64x512) && pr.K >= 1024 && count(TILE_64x512) >= 2 * num_cu()) return TILE_64x512;
        // otherwise 64x128 tiles, two or three of which share a CU so that one's epilogue hides
        // behind another's MFMAs
        // (given at least two per CU; with fewer, 64x64 tiles fill the chip better)
        return fits(TILE_64x128) && count(TILE_64x128) >= 2 * num_cu() ? TILE_64x128 : TILE_64x64;
    }
    // 16- and 8-bit operands: 256x256 tiles once every CU has one - and already from half the CUs
    // on when the 128x128 tiles (two workgroups per CU) would need a second round: measured 1.2-1.4
    // times faster there (160 and 192 tiles at K = 512 and 4096), 0.8-0.9 times at 128 tiles
    if (fits(TILE_256x256) && (count(TILE_256x256) >= num_cu() ||
                               (2 * count(TILE_256x256) > num_cu() && count(TILE_128x128) > 2 * num_cu())))
        return TILE_256x256;
    // 128x128 tiles from 5/8 of the CUs on: one round of them (three stage buffers, see tile_args)
    // then beats the 64x64 tiles' several (640 x 4096 x 4096: 48.5 against 58.3 us; at 512 rows,
    // 128 tiles, the 64x64 tiles still win with 38 us)
    if (fits(TILE_128x128) && count(TILE_128x128) * 8 >= num_cu() * 5) return TILE_128x128;
    return TILE_64x64;
}

// two_pass: finish split rows with the second kernel even where the cooperative form exists
// (asked for by flag, or the stream is being captured into a graph).
Plan make_plan(const fge_params *p, int norm, bool two_pass = false, int force_tile = -1) {
    Plan pl{};
    Problem &pr = pl.pr;
    pr = Problem{p->M, p->N, p->K, p->batch, p->ldx, p->ldw, p->ldo,
                 p->batch > 1 ? p->batch_stride_x : 0, p->batch > 1 ? p->batch_stride_o : 0};
    if (pr.batch > 1 && pr.bsx == (int64_t)pr.M * pr.ldx && pr.bso == (int64_t)pr.M * pr.ldo) {
        pr.M *= pr.batch;            // dense batch: one tall problem (W, b, gamma, beta are shared)
        pr.batch = 1;
        pr.bsx = pr.bso = 0;
    }
    pl.tile = force_tile >= 0        ? force_tile
              : forced_tile(p) >= 0 ? forced_tile(p)
                                    : pick_tile(pr, p->in_dtype, norm, (p->flags & FGE_FLAG_IEEE_FP32) != 0,
                                                !(p->flags & FGE_FLAG_NO_TABLE));
    // 16- and 8-bit 128x128 tiles, no more of them than CUs (however the tile was chosen): the form
    // on eight waves with three stage buffers - no second workgroup shares a CU, so a second K-tile
    // copy in flight and a second wave per SIMD hide the latencies instead (640 x 4096 x 4096: 43.2
    // -> 40.3 us, 1024 x 1024 x 4096: 21.4 -> 19.5 us against the four-wave form with three buffers)
    if (pl.tile == TILE_128x128 && p->in_dtype != FGE_F32 &&
        (int64_t)((pr.M + 127) / 128) * ((pr.N + 127) / 128) * pr.batch <= num_cu())
        pl.tile = TILE_128x128_S3;
    const TileInfo &ti = tile_info(pl.tile);
    pl.tiles_m = (pr.M + ti.bm - 1) / ti.bm;
    pl.tiles_n = (pr.N + ti.bn - 1) / ti.bn;
    pl.split = norm != FGE_NORM_NONE && pl.tiles_n > 1;
    // cooperative form: the column tiles of a row block must all be in flight at once, so the
    // grid is a whole number of row blocks that fits the chip
    const int capacity = num_cu() * ti.coop_per_cu;
    // ... and not too many of them: every tile merges the pairs of all tiles of its rows, which
    // grows with their number (125 column tiles, 2048 x 4096 x 32000: 626 us against 544 us for the
    // second pass; equal at 64); logsumexp leaves `out` final in the first pass, so its second
    // pass only writes aux and wins from 32 column tiles on
    const int coop_max_tiles = norm == FGE_NORM_LOGSUMEXP ? 16 : 64;
    // (the table may also say that the second pass is the faster way to finish this problem's rows:
    // a persistent grid that does not divide the row blocks evenly idles part of the chip in its
    // last round)
    bool table_two_pass = false;
    if (force_tile < 0 && forced_tile(p) < 0 && !(p->flags & FGE_FLAG_NO_TABLE))
        if (const TileTableEntry *e = table_entry(pr, p->in_dtype, norm)) table_two_pass = e->tile == pl.tile && e->two_pass;
    pl.coop = pl.split && !two_pass && !table_two_pass && !(p->flags & FGE_FLAG_TWO_PASS) && tile_has_coop(pl.tile, p->in_dtype) &&
              capacity >= pl.tiles_n && pl.tiles_n <= coop_max_tiles;
    if (pl.coop) {
        const int64_t total = (int64_t)pl.tiles_m * pl.tiles_n * pr.batch;
        const int64_t g = (int64_t)(capacity / pl.tiles_n) * pl.tiles_n;
        pl.coop_grid = (int)(total < g ? total : g);
    }
    pl.needs_finish = pl.split && !pl.coop;
    // pairs per row: one per wave strip for the second pass, one per tile in the cooperative form
    pl.strips = pl.coop ? pl.tiles_n : pl.tiles_n * ti.waves_n;
    pl.ws_stats = pl.split ? round256((size_t)pr.M * pr.batch * pl.strips * sizeof(float2)) : 0;
    pl.ws_marks = pl.coop ? round256((size_t)pl.tiles_m * pr.batch * pl.tiles_n * sizeof(unsigned)) + 256 : 0;
    const size_t extent = (size_t)(pr.batch - 1) * pr.bso + (size_t)(pr.M - 1) * pr.ldo + pr.N;
    pl.ws_buf = round256(extent * esize(p->out_dtype));
    // K2 writes straight into `out` when the row op leaves the activated values in place
    pl.n_bufs = (norm == FGE_NORM_NONE || norm == FGE_NORM_LOGSUMEXP) ? 1 : 2;
    pl.generic = !vectorisable(p, norm, true) || (pl.split && pl.tiles_n * ti.waves_n > MAX_SPLIT);
    if (pl.generic) {                // no tiles, no statistics: GEMM + activation to fp32, then the row op
        pl.split = pl.coop = pl.needs_finish = false;
        pl.ws_stats = pl.ws_marks = 0;
        pl.ws_generic = norm == FGE_NORM_NONE ? 0 : round256((size_t)p->M * p->batch * p->N * sizeof(float));
    }
    return pl;
}

// K-split (one-call fused entry point only): a problem with so few tiles that most CUs would
// idle while each workgroup walks a long K alone is cut into S slices of K.  One launch of the
// tile kernel computes the S partial products (slice z of X and W starts z*K/S elements into
// every row; fp32, into the workspace), a second kernel adds the slices in slice order and
// applies scale, bias and activation, and a row operation runs over that fp32 result (a third
// kernel, one wave per row: a wave that also added the slices of its row would walk them one
// memory round trip after the other - measured 37 us for that against 8 us for the two kernels).
// Chosen when it pays (measured: 16 x 8192 x 4096, 16-bit operands, 46 us as one launch, 21 us
// in 8 slices): 64x64 tiles (the choice for small problems; with 256 tiles of 128x128 the slices
// gained nothing), no more of them than CUs, K >= 2048 (split product) / 4096 / 8192 (more than
// half the CUs busy as it is), slices of at least 512 that are whole
// staged K tiles, at most two workgroups per CU and 32 MB of partial sums.
struct KSplit {
    int slices;                  // 1: none
    size_t ws_part, ws_mid;      // bytes of the partial products / of the fp32 rows a row op reads
    size_t bytes() const { return ws_part + ws_mid; }
};

KSplit k_split(const fge_params *p, int norm, const Plan &pl) {
    KSplit ks{1, 0, 0};
    if (pl.generic || pl.tile != TILE_64x64 || pl.pr.batch != 1 || (p->flags & FGE_FLAG_NO_SPLIT_K)) return ks;
    if (norm != FGE_NORM_NONE && pl.pr.N > MAX_ROWOP_N) return ks;      // its row kernel holds a row in registers
    const int64_t tiles = (int64_t)pl.tiles_m * pl.tiles_n;
    // the 64x64 kernel of the 16- and 8-bit operands and of the fp32 instruction keeps three K tiles
    // in flight and walks K faster than the split-product kernel: slices pay later there
    const bool deep = !(p->in_dtype == FGE_F32 && !(p->flags & FGE_FLAG_IEEE_FP32));
    const int k_min = !deep ? 2048 : tiles * 2 > num_cu() ? 8192 : 4096;
    if (tiles > num_cu() || pl.pr.K < k_min) return ks;
    const size_t one = round256((size_t)pl.pr.M * pl.pr.N * sizeof(float));
    int S = 1;
    for (int c = 2; c <= 16; c *= 2)
        if (tiles * c <= 2 * num_cu() && pl.pr.K % (c * 128) == 0 && pl.pr.K / c >= 512 && one * c <= ((size_t)32 << 20)) S = c;
    if (S == 1) return ks;
    ks.slices = S;
    ks.ws_part = one * S;
    ks.ws_mid = norm == FGE_NORM_NONE ? 0 : one;
    return ks;
}

struct Repack {
    bool use;
    bool odd_out;                // the result is not storable in 16-byte units either
    bool copy_x, copy_w;         // which operands are copied (one that the tile kernels can stage where it lies is not)
    int Kp, Np;                  // padded contraction length / padded width of the fp32 rows
    int64_t rows, w_rows;        // rows of the padded X / W
    size_t off_w, off_b, off_mid, off_inner, bytes;      // workspace layout; the padded X sits at 0
    fge_params inner;            // the padded problem (workspace still to be filled in)
};

Repack plan_repack(const fge_params *p, int norm);

// Workspace of the fused path: enough for either form of split rows, since a launch on a
// stream under graph capture takes the two-pass form whatever the flags say - and for the
// K-split where the one-call entry point would take it.
size_t fused_workspace(const fge_params *p, int norm) {
    const Plan p1 = make_plan(p, norm, false), p2 = make_plan(p, norm, true);
    if (p1.generic) {                // room for the repacked operands where the problem is worth repacking
        const Repack rp = plan_repack(p, norm);
        return rp.use && rp.bytes > p1.ws_generic ? rp.bytes : p1.ws_generic;
    }
    const size_t a = p1.ws_stats + p1.ws_marks, b = p2.ws_stats + p2.ws_marks, c = k_split(p, norm, p1).bytes();
    return a > b ? (a > c ? a : c) : (b > c ? b : c);
}

// What the tile kernels need of it (the K-split is optional: without the room it is not taken).
size_t split_rows_workspace(const fge_params *p, int norm) {
    const Plan p1 = make_plan(p, norm, false), p2 = make_plan(p, norm, true);
    const size_t a = p1.ws_stats + p1.ws_marks, b = p2.ws_stats + p2.ws_marks;
    return a > b ? a : b;
}

// The gated tile kernel takes 16-bit and 8-bit operands in shapes the vectorised kernels take.
bool gated_fast(const fge_params *p, int norm) { return p->in_dtype != FGE_F32 && vectorisable(p, norm, true); }

size_t gated_workspace(const fge_params *p, int norm) {
    const Plan p1 = make_plan(p, norm, false, TILE_GATED), p2 = make_plan(p, norm, true, TILE_GATED);
    const size_t a = p1.ws_stats + p1.ws_marks, b = p2.ws_stats + p2.ws_marks;
    return a > b ? a : b;
}

GenArgs gen_args(const fge_params *p) {
    GenArgs g{};
    g.gamma = p->gamma; g.beta = p->beta; g.aux = p->aux_out;
    g.M = p->M; g.N = p->N; g.K = p->K; g.batch = p->batch;
    g.ldx = p->ldx; g.ldw = p->ldw; g.bsx = p->batch > 1 ? p->batch_stride_x : 0;
    g.ldd = p->ldo; g.bsd = p->batch > 1 ? p->batch_stride_o : 0;
    g.alpha = p->alpha; g.post = p->post_scale; g.lo = p->clamp_lo < p->clamp_hi ? p->clamp_lo : p->clamp_hi;
    g.hi = p->clamp_hi; g.eps = p->eps;
    return g;
}

// min(max(y, lo), hi) with lo > hi is hi for every y: the same as clamping to [hi, hi], which
// lets the kernels use a median-of-three for the clamp.
inline float clamp_low(const fge_params *p) { return p->clamp_lo < p->clamp_hi ? p->clamp_lo : p->clamp_hi; }

// A replayed graph launches with the arguments recorded at capture time, generation number
// included, so the arrival marks of one replay would satisfy the next: the cooperative form is
// not used on a stream that is being captured.
bool capturing(hipStream_t s) {
    hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
    return hipStreamIsCapturing(s, &st) == hipSuccess && st != hipStreamCaptureStatusNone;
}

int hip_status(hipError_t e) {
    if (e == hipSuccess) return FGE_OK;
    g_last_hip = (int)e;
    return FGE_ERR_HIP;
}

// Device address of `scratch` on the current device: every GPU holds its own copy of the array at
// its own address, so the address is kept per device (asked on the first call there).
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

int static_scratch(void **ptr) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_status(e);
    if (dev < 0 || dev >= MAX_DEVICES) return FGE_ERR_UNSUPPORTED;
    void *sp = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (sp == nullptr) {
        e = hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_status(e);
        if (sp == nullptr) return hip_status(hipErrorInvalidSymbol);
        g_scratch_ptr[dev].store(sp, std::memory_order_release);
    }
    *ptr = sp;
    return FGE_OK;
}

TileArgs tile_args(const void *X, const void *W, const float *b, int act, int norm,
                   const fge_params *p, const Plan &pl, void *out) {
    TileArgs a{};
    a.X = X; a.W = W; a.b = b; a.gamma = p->gamma; a.beta = p->beta;
    a.out = out; a.aux = p->aux_out; a.ws = reinterpret_cast<float2 *>(p->workspace);
    a.M = pl.pr.M; a.N = pl.pr.N; a.K = pl.pr.K;
    a.w_rows = g_w_rows > 0 && g_w_rows < pl.pr.N ? g_w_rows : pl.pr.N;
    a.ldx = pl.pr.ldx; a.ldw = pl.pr.ldw; a.ldo = pl.pr.ldo; a.bsx = pl.pr.bsx; a.bso = pl.pr.bso;
    a.alpha = p->alpha; a.post = p->post_scale; a.lo = clamp_low(p); a.hi = p->clamp_hi; a.eps = p->eps;
    a.act = act; a.norm = norm;
    a.tiles_m = pl.tiles_m; a.tiles_n = pl.tiles_n; a.batch = pl.pr.batch;
    a.group_m = pl.tiles_m < 8 ? pl.tiles_m : 8;
    // an output of half the last-level cache or more is stored with the streaming hint: little of
    // it would still be cached for a consumer, and on its way out it displaces the operand panels
    // the tiles share (batched K = 512 workload, 128 MiB of output: 3.7 % faster; the headline
    // workload's 64 MiB: no difference either way)
    a.stream_out = (size_t)pl.pr.M * pl.pr.batch * pl.pr.N * esize(p->out_dtype) >= ((size_t)128 << 20);
    a.coop = 0;
    if (pl.coop && norm != FGE_NORM_NONE) {
        char *base = static_cast<char *>(p->workspace) + pl.ws_stats;
        a.coop = 1;
        a.gen = g_generation.fetch_add(1) + 1;
        a.arrive = reinterpret_cast<unsigned *>(base);
        a.fault = reinterpret_cast<int *>(base + pl.ws_marks - 256);
        // staggered start of the row blocks (see the kernel): measured 1 to 7 % on problems whose
        // tiles are short (K = 256 ... 2048; 7 % on the batched K = 512 workload) and that take at
        // least three rounds of the grid; nothing either way at K = 4096, where a round's stores are a
        // small part of its time - and a plain loss on a single round, which the stagger only
        // lengthens (the 4096 x 1024 x 1024 fp32 workload: 42 -> 51 us)
        const int64_t row_blocks = (int64_t)pl.tiles_m * pl.pr.batch, per_round = pl.coop_grid / pl.tiles_n;
        a.stagger = pl.pr.K <= 2048 && row_blocks >= 3 * per_round ? 4 : 0;
        a.stagger_mask = 7;
        const bool expire = (p->flags & FGE_FLAG_TEST_EXPIRE_WAIT) != 0;
        a.spin_limit = expire ? 1u : WAIT_POLLS;
        a.withhold = expire ? 1 : 0;
    }
    return a;
}

int launch_tiles(const TileArgs &a, const fge_params *p, const Plan &pl, hipStream_t s) {
    if (pl.tile == TILE_PANEL) {
        const dim3 pgrid((unsigned)(pl.tiles_m < num_cu() ? pl.tiles_m : num_cu()));
        return hip_status(launch_panel_f32(p->out_dtype, pgrid, s, a));
    }
    const dim3 grid(a.coop ? (unsigned)pl.coop_grid : (unsigned)(pl.tiles_m * pl.tiles_n), 1,
                    a.coop ? 1u : (unsigned)pl.pr.batch);
    if (pl.tile == TILE_128x256 || pl.tile == TILE_256x128)
        return hip_status(p->in_dtype == FGE_BF16  ? launch_half_bf16(pl.tile, p->out_dtype, grid, s, a)
                          : p->in_dtype == FGE_F16 ? launch_half_f16(pl.tile, p->out_dtype, grid, s, a)
                                                   : launch_half_f8(pl.tile, p->out_dtype, grid, s, a));
    const hipError_t e = p->in_dtype == FGE_BF16       ? launch_tile_bf16(pl.tile, p->out_dtype, grid, s, a)
                         : p->in_dtype == FGE_F16      ? launch_tile_f16(pl.tile, p->out_dtype, grid, s, a)
                         : p->in_dtype == FGE_F8E4M3   ? launch_tile_f8(pl.tile, p->out_dtype, grid, s, a)
                         : (p->flags & FGE_FLAG_IEEE_FP32) ? launch_tile_f32(pl.tile, p->out_dtype, grid, s, a)
                                                           : launch_tile_f32s(pl.tile, p->out_dtype, grid, s, a);
    return hip_status(e);
}

RowArgs row_args(const void *in, void *out, int act, int norm, const fge_params *p, const Plan &pl) {
    RowArgs r{};
    r.in = in; r.out = out; r.gamma = p->gamma; r.beta = p->beta; r.aux = p->aux_out;
    r.ws = reinterpret_cast<const float2 *>(p->workspace);
    r.M = pl.pr.M; r.N = pl.pr.N; r.batch = pl.pr.batch; r.ldo = pl.pr.ldo; r.bso = pl.pr.bso;
    r.lo = clamp_low(p); r.hi = p->clamp_hi; r.eps = p->eps; r.act = act; r.norm = norm;
    r.tiles_n = pl.strips; r.bn = tile_info(pl.tile).bn / tile_info(pl.tile).waves_n;
    return r;
}

// SLICES: T = float, the row is formed from the partial products of a K-split (see RowArgs)
template <typename T, typename OutT = T, bool SLICES = false> int launch_rownorm(const RowArgs &r, hipStream_t s) {
    const int cpr = r.N / Store<T>::CW;
    const int ch = (cpr + 63) / 64;
    const int64_t rows = (int64_t)r.batch * r.M;
    const dim3 grid((unsigned)((rows + 3) / 4)), block(256);
    if (ch <= 1)       hipLaunchKernelGGL((rownorm_kernel<T, 1, OutT, SLICES>), grid, block, 0, s, r);
    else if (ch <= 2)  hipLaunchKernelGGL((rownorm_kernel<T, 2, OutT, SLICES>), grid, block, 0, s, r);
    else if (ch <= 4)  hipLaunchKernelGGL((rownorm_kernel<T, 4, OutT, SLICES>), grid, block, 0, s, r);
    else if (ch <= 8)  hipLaunchKernelGGL((rownorm_kernel<T, 8, OutT, SLICES>), grid, block, 0, s, r);
    else if (ch <= 16) hipLaunchKernelGGL((rownorm_kernel<T, 16, OutT, SLICES>), grid, block, 0, s, r);
    else if (ch <= 32) hipLaunchKernelGGL((rownorm_kernel<T, 32, OutT, SLICES>), grid, block, 0, s, r);
    else return FGE_ERR_UNSUPPORTED;
    return hip_status(hipGetLastError());
}

// S partial products of X.W^T over S slices of K (S = 1: the whole product), fp32, dense M x N
// slices `slice` elements apart at `part`: the slices are the problems of one strided-batch launch.
int launch_partials(const void *X, const void *W, const fge_params *p, const Plan &pl, int S, int64_t slice,
                    void *part, hipStream_t s) {
    const int Kc = pl.pr.K / S;
    fge_params q = *p;
    q.M = pl.pr.M; q.batch = S; q.K = Kc; q.ldx = pl.pr.ldx; q.batch_stride_x = Kc;
    q.out_dtype = FGE_F32; q.ldo = pl.pr.N; q.batch_stride_o = slice;
    q.alpha = q.post_scale = 1.0f;
    q.flags = p->flags & FGE_FLAG_IEEE_FP32;
    const Plan pq = make_plan(&q, FGE_NORM_NONE, false, pl.tile);
    if (pq.generic || pq.pr.batch != S) return FGE_ERR_UNSUPPORTED;    // (the callers admit no such shape)
    TileArgs a = tile_args(X, W, nullptr, FGE_ACT_NONE, FGE_NORM_NONE, &q, pq, part);
    a.bsw = Kc;                                // slice z of W starts z*Kc into every row, like X's
    return launch_tiles(a, &q, pq, s);
}

// Sum of the slices with scale / bias / activation (and the gate, when a second product's
// slices are given), then the row op.  `mid`: fp32 rows the row op reads (unused without one).
int finish_partials(const void *part, const void *part2, const float *b, const float *b2, int act, int norm,
                    const fge_params *p, const Plan &pl, int S, int64_t slice, void *mid, void *out, hipStream_t s) {
    GenArgs g = gen_args(p);
    g.X = part; g.W = part2; g.K = S; g.bsx = slice; g.M = pl.pr.M; g.batch = 1; g.b = b; g.b2 = b2; g.act = act;
    if (norm == FGE_NORM_NONE) {
        g.dst = out; g.ldd = pl.pr.ldo;
        return hip_status(launch_splitk_sum(p->out_dtype, s, g));
    }
    // rows of up to 8192 columns (N is a multiple of 4 here): one kernel adds the slices of a row
    // and runs the row op on it, one workgroup per row (16 x 4096 x 4096, 8 slices, RMSNorm: the sum
    // kernel plus the wave-per-row kernel took 4.3 + 8.4 us of the call's 21)
    if (pl.pr.N <= 8192 && pl.pr.N % 4 == 0) {
        SplitRowArgs q{};
        q.P = static_cast<const float *>(part); q.P2 = static_cast<const float *>(part2);
        q.b = b; q.b2 = b2; q.gamma = p->gamma; q.beta = p->beta; q.out = out; q.aux = p->aux_out;
        q.M = pl.pr.M; q.N = pl.pr.N; q.S = S; q.slice = slice; q.ldo = pl.pr.ldo; q.bso = pl.pr.bso;
        q.scale = p->post_scale * p->alpha; q.post = p->post_scale; q.lo = clamp_low(p); q.hi = p->clamp_hi; q.eps = p->eps;
        q.act = act; q.norm = norm;
        const int64_t rows = (int64_t)pl.pr.M * pl.pr.batch;
        return hip_status(p->out_dtype == FGE_BF16  ? launch_splitk_rows_t<bf16_t>(q, rows, s)
                          : p->out_dtype == FGE_F16 ? launch_splitk_rows_t<f16_t>(q, rows, s)
                                                    : launch_splitk_rows_t<float>(q, rows, s));
    }
    g.dst = mid; g.ldd = pl.pr.N;              // act(post*(alpha*sum + b)) [* gate] in fp32, dense rows
    const int rc = hip_status(launch_splitk_sum(FGE_F32, s, g));
    if (rc) return rc;
    // the row operation on the row in a wave's registers (vectorisable() keeps N <= 8192), read
    // as one fp32 "slice" that needs no further scale, bias or activation
    RowArgs r = row_args(mid, out, FGE_ACT_NONE, norm, p, pl);
    r.b = nullptr; r.scale = 1.0f; r.post = 0.0f; r.slices = 1; r.slice_stride = 0;
    return p->out_dtype == FGE_BF16  ? launch_rownorm<float, bf16_t, true>(r, s)
           : p->out_dtype == FGE_F16 ? launch_rownorm<float, f16_t, true>(r, s)
                                     : launch_rownorm<float, float, true>(r, s);
}

// The K-split of k_split(): partial products, their sum with scale / bias / activation, row op.
int run_k_split(const void *X, const void *W, const float *b, int act, int norm, const fge_params *p,
                const Plan &pl, const KSplit &ks, void *out, hipStream_t s) {
    const int S = ks.slices;
    char *part = static_cast<char *>(p->workspace);
    const int64_t slice = (int64_t)(ks.ws_part / S / sizeof(float));     // elements between slices
    const int rc = launch_partials(X, W, p, pl, S, slice, part, s);
    if (rc) return rc;
    return finish_partials(part, nullptr, b, nullptr, act, norm, p, pl, S, slice, part + ks.ws_part, out, s);
}

int run_fused(const void *X, const void *W, const float *b, int act, int norm, const fge_params *p, void *out,
              hipStream_t s);

// Operands or results whose extents or strides are not whole 16-byte units (K = 4095, a row
// stride of 4099 elements ...) cannot be staged or stored by the vectorised kernels as they
// lie.  Where the problem is large enough to pay for one more read and write of its operands,
// fused_gemm_epilogue repacks them instead of leaving the product to the element-granular
// kernel: X and W are copied into dense workspace buffers with K padded by zeros to a whole
// chunk (the extra terms of every sum are exact zeros), and the padded problem runs on the
// tile kernels.  When the result's own extents or strides are odd as well, the tile kernel
// applies the activation and writes fp32 rows of padded width into the workspace (a copied W
// gets zero rows, b zero entries for the padding columns), and a row kernel that stores
// element by element and never looks at the padding columns turns them into `out`
// (launch_generic_row: one workgroup per row, since these rows start on 16-byte boundaries).
// The stage entry points and the unfused sequence keep the element-granular product.
constexpr double REPACK_MIN_FLOP = 3.0e7;   // below this the element-granular product is as fast as four launches

Repack plan_repack(const fge_params *p, int norm) {
    Repack r{};
    if (vectorisable(p, norm, true)) return r;
    const size_t is = esize(p->in_dtype), os = esize(p->out_dtype);
    const int64_t rows = (int64_t)p->M * p->batch;
    if (2.0 * (double)rows * p->N * p->K < REPACK_MIN_FLOP || rows > INT32_MAX / 2) return r;
    const int cw = (int)(16 / is);
    r.Kp = (p->K + cw - 1) / cw * cw;
    r.odd_out = (p->N * os) % 16 || (p->ldo * os) % 16 || (p->batch > 1 && (p->batch_stride_o * os) % 16);
    r.Np = r.odd_out ? (p->N + 3) / 4 * 4 : p->N;
    r.rows = rows;
    r.w_rows = r.Np;
    // an operand that can be staged where it lies is not copied (odd N with an even K - a
    // vocabulary of 50257 entries - then costs no copy at all: the padding columns of the fp32
    // rows are fed from W's last row, see TileArgs::w_rows, and never looked at afterwards)
    const int64_t bsx = p->batch > 1 ? p->batch_stride_x : 0;
    r.copy_x = !operand_ok(p, p->ldx, bsx) || (r.odd_out && p->batch > 1 && bsx != (int64_t)p->M * p->ldx);
    r.copy_w = !operand_ok(p, p->ldw, 0);
    r.inner = *p;
    r.inner.K = r.Kp;
    if (r.copy_x) { r.inner.ldx = r.Kp; r.inner.batch_stride_x = (int64_t)p->M * r.Kp; }
    if (r.copy_w) r.inner.ldw = r.Kp;
    r.inner.workspace = nullptr;
    r.inner.workspace_bytes = 0;
    if (r.odd_out) {             // one tall problem into dense fp32 rows of padded width
        r.inner.M = (int32_t)rows;
        r.inner.batch = 1;
        r.inner.N = r.Np;
        r.inner.ldo = r.Np;
        r.inner.batch_stride_x = r.inner.batch_stride_o = 0;
        r.inner.out_dtype = FGE_F32;
        r.inner.gamma = r.inner.beta = nullptr;
        r.inner.aux_out = nullptr;
    }
    if (!vectorisable(&r.inner, r.odd_out ? FGE_NORM_NONE : norm, true)) return r;     // (cannot happen)
    const size_t xp = r.copy_x ? round256((size_t)rows * r.Kp * is) : 0, wp = r.copy_w ? round256((size_t)r.w_rows * r.Kp * is) : 0;
    r.off_w = xp;
    r.off_b = r.off_w + wp;
    r.off_mid = r.off_b + (r.odd_out ? round256((size_t)r.Np * sizeof(float)) : 0);
    r.off_inner = r.off_mid + (r.odd_out ? round256((size_t)rows * r.Np * sizeof(float)) : 0);
    r.bytes = r.off_inner + fused_workspace(&r.inner, r.odd_out ? FGE_NORM_NONE : norm);
    r.use = true;
    return r;
}

int run_repacked(const void *X, const void *W, const float *b, int act, int norm, const fge_params *p,
                 const Repack &rp, void *out, hipStream_t s) {
    char *ws = static_cast<char *>(p->workspace);
    int rc;
    const void *Xi = X, *Wi = W;
    if (rp.copy_x) {
        const PadArgs ax{X, ws, p->M, p->batch, p->K, rp.Kp, p->ldx, p->batch > 1 ? p->batch_stride_x : 0, rp.rows};
        if ((rc = hip_status(launch_pad_rows(p->in_dtype, s, ax)))) return rc;
        Xi = ws;
    }
    if (rp.copy_w) {
        const PadArgs aw{W, ws + rp.off_w, p->N, 1, p->K, rp.Kp, p->ldw, 0, rp.w_rows};
        if ((rc = hip_status(launch_pad_rows(p->in_dtype, s, aw)))) return rc;
        Wi = ws + rp.off_w;
    }
    fge_params q = rp.inner;
    q.workspace = ws + rp.off_inner;
    q.workspace_bytes = p->workspace_bytes - rp.off_inner;
    if (!rp.odd_out) return run_fused(Xi, Wi, b, act, norm, &q, out, s);
    const float *bp = nullptr;
    if (b != nullptr) {
        float *dst = reinterpret_cast<float *>(ws + rp.off_b);
        if ((rc = hip_status(launch_pad_vec(b, dst, p->N, rp.Np, s)))) return rc;
        bp = dst;
    }
    void *mid = ws + rp.off_mid;
    {
        // W as it lies has N rows, the padded problem Np columns: the tile kernels stop at row N - 1
        struct Scope { Scope(int n) { g_w_rows = n; } ~Scope() { g_w_rows = 0; } } scope(rp.copy_w ? 0 : p->N);
        if ((rc = run_fused(Xi, Wi, bp, act, FGE_NORM_NONE, &q, mid, s))) return rc;
    }
    GenArgs g = gen_args(p);
    g.X = mid; g.ldx = rp.Np; g.bsx = (int64_t)p->M * rp.Np; g.dst = out; g.norm = norm;
    return hip_status(launch_generic_row(FGE_F32, p->out_dtype, s, g));
}

// one_call: fused_gemm_epilogue, which runs the second pass, if any, from the plan returned here.
// It may finish split rows inside the tile kernel (cooperative form; if the device cannot hold
// that grid the launcher refuses it before anything runs and the two-pass form is taken) and cut
// K into slices where that pays and the workspace has the room.  The stage entry points
// (fge_fused_tiles, then fge_fused_finish) are two passes by definition: they always plan the
// two-pass form, whatever the stream or the device, so both stages and fge_fused_needs_finish
// agree without knowing about each other.
int do_fused_tiles(const void *X, const void *W, const float *b, int act, int norm,
                   const fge_params *p, void *out, hipStream_t s, Plan *plan_out, bool one_call = false) {
    int rc = check_common(p, act, norm, true);
    if (rc) return rc;
    if (!X || !W || !out) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W) || !aligned16(out) || !aligned16(b)) return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    const Plan pl = make_plan(p, norm, !one_call || capturing(s));
    if (plan_out) *plan_out = pl;
    if (pl.generic) {
        if (one_call) {
            const Repack rp = plan_repack(p, norm);
            if (rp.use && p->workspace && p->workspace_bytes >= rp.bytes) return run_repacked(X, W, b, act, norm, p, rp, out, s);
        }
        // GEMM + activation straight into out, or into an fp32 rows x N intermediate that the row
        // kernel then reads (several passes) and turns into out
        GenArgs g = gen_args(p);
        g.X = X; g.W = W; g.b = b; g.act = act; g.norm = norm;
        if (norm == FGE_NORM_NONE) {
            g.dst = out;
            return hip_status(launch_generic_gemm(p->in_dtype, p->out_dtype, s, g));
        }
        if (!p->workspace || p->workspace_bytes < pl.ws_generic) return FGE_ERR_WORKSPACE;
        g.dst = p->workspace; g.ldd = p->N; g.bsd = (int64_t)p->M * p->N;
        if ((rc = hip_status(launch_generic_gemm(p->in_dtype, FGE_F32, s, g)))) return rc;
        GenArgs r = gen_args(p);
        r.X = p->workspace; r.ldx = p->N; r.bsx = (int64_t)p->M * p->N; r.dst = out; r.norm = norm;
        return hip_status(launch_generic_row(FGE_F32, p->out_dtype, s, r));
    }
    if (one_call) {
        const KSplit ks = k_split(p, norm, pl);
        if (ks.slices > 1 && p->workspace && p->workspace_bytes >= ks.bytes()) {
            if (plan_out) plan_out->needs_finish = false;
            return run_k_split(X, W, b, act, norm, p, pl, ks, out, s);
        }
    }
    if (pl.split) {
        if (pl.strips > MAX_SPLIT) return FGE_ERR_UNSUPPORTED;
        if (!p->workspace || p->workspace_bytes < split_rows_workspace(p, norm)) return FGE_ERR_WORKSPACE;
    }
    rc = launch_tiles(tile_args(X, W, b, act, norm, p, pl, out), p, pl, s);
    if (rc == FGE_ERR_HIP && one_call && pl.coop && fge_last_hip_error() == (int)hipErrorCooperativeLaunchTooLarge) {
        const Plan p2 = make_plan(p, norm, true);
        if (plan_out) *plan_out = p2;
        rc = launch_tiles(tile_args(X, W, b, act, norm, p, p2, out), p, p2, s);
    }
    return rc;
}

int launch_finish(const Plan &pl, int act, int norm, const fge_params *p, void *out, hipStream_t s);

int do_fused_finish(int act, int norm, const fge_params *p, void *out, hipStream_t s) {
    int rc = check_common(p, act, norm, true);
    if (rc) return rc;
    if (!out) return FGE_ERR_NULL;
    if (!aligned16(out)) return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    const Plan pl = make_plan(p, norm, true);
    if (!pl.needs_finish) return FGE_OK;
    if (pl.strips > MAX_SPLIT) return FGE_ERR_UNSUPPORTED;
    if (!p->workspace || p->workspace_bytes < split_rows_workspace(p, norm)) return FGE_ERR_WORKSPACE;
    return launch_finish(pl, act, norm, p, out, s);
}

int launch_finish(const Plan &pl, int act, int norm, const fge_params *p, void *out, hipStream_t s) {
    const RowArgs r = row_args(out, out, act, norm, p, pl);
    const int64_t rows = (int64_t)r.batch * r.M;
    const dim3 block(256);
    if (r.N > MAX_ROWOP_N && rows <= INT32_MAX) {        // a wide row is shared by the four waves of a workgroup
        const dim3 grid((unsigned)rows);
        if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((finish_kernel<bf16_t, 4>), grid, block, 0, s, r);
        else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((finish_kernel<f16_t, 4>), grid, block, 0, s, r);
        else                              hipLaunchKernelGGL((finish_kernel<float, 4>), grid, block, 0, s, r);
        return hip_status(hipGetLastError());
    }
    const dim3 grid((unsigned)((rows + 3) / 4));
    if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((finish_kernel<bf16_t, 1>), grid, block, 0, s, r);
    else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((finish_kernel<f16_t, 1>), grid, block, 0, s, r);
    else                              hipLaunchKernelGGL((finish_kernel<float, 1>), grid, block, 0, s, r);
    return hip_status(hipGetLastError());
}

int run_fused(const void *X, const void *W, const float *b, int act, int norm, const fge_params *p, void *out,
              hipStream_t s) {
    Plan pl{};
    const int rc = do_fused_tiles(X, W, b, act, norm, p, out, s, &pl, true);
    if (rc || !pl.needs_finish) return rc;
    return launch_finish(pl, act, norm, p, out, s);    // with the plan the tiles ran under
}

int do_gemm_bias(const void *X, const void *W, const float *b, const fge_params *p, void *Y, hipStream_t s) {
    int rc = check_common(p, FGE_ACT_NONE, FGE_NORM_NONE, true);
    if (rc) return rc;
    if (!X || !W || !Y) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W) || !aligned16(Y) || !aligned16(b)) return FGE_ERR_ALIGN;
    const Plan pl = make_plan(p, FGE_NORM_NONE);
    if (pl.generic) {
        GenArgs g = gen_args(p);
        g.X = X; g.W = W; g.b = b; g.act = FGE_ACT_NONE; g.dst = Y;
        return hip_status(launch_generic_gemm(p->in_dtype, p->out_dtype, s, g));
    }
    return launch_tiles(tile_args(X, W, b, FGE_ACT_NONE, FGE_NORM_NONE, p, pl, Y), p, pl, s);
}

// A = act(Y), or act(Y) * U when U is given (the gate of the gated sequence)
int do_act(const void *Y, int act, const fge_params *p, void *A, hipStream_t s, const void *U = nullptr) {
    int rc = check_common(p, act, FGE_NORM_NONE, false);
    if (rc) return rc;
    if (!Y || !A) return FGE_ERR_NULL;
    if (!aligned16(Y) || !aligned16(A) || !aligned16(U)) return FGE_ERR_ALIGN;
    if (!vectorisable(p, FGE_NORM_NONE, false)) {
        GenArgs g = gen_args(p);
        g.X = Y; g.W = U; g.dst = A; g.act = act;
        return hip_status(launch_generic_act(p->out_dtype, s, g));
    }
    const Plan pl = make_plan(p, FGE_NORM_NONE);
    RowArgs r = row_args(Y, A, act, FGE_NORM_NONE, p, pl);
    r.in2 = U;
    const int cw = p->out_dtype == FGE_F32 ? 4 : 8;
    const int64_t chunks = (int64_t)r.batch * r.M * (r.N / cw);
    int64_t blocks = (chunks + 255) / 256;
    if (blocks > num_cu() * 32) blocks = num_cu() * 32;      // grid-stride beyond that
    const dim3 grid((unsigned)blocks), block(256);
    if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((act_kernel<bf16_t>), grid, block, 0, s, r);
    else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((act_kernel<f16_t>), grid, block, 0, s, r);
    else                              hipLaunchKernelGGL((act_kernel<float>), grid, block, 0, s, r);
    return hip_status(hipGetLastError());
}

int do_rownorm(const void *A, int norm, const fge_params *p, void *out, hipStream_t s) {
    int rc = check_common(p, FGE_ACT_NONE, norm, false);
    if (rc) return rc;
    if (!A || !out) return FGE_ERR_NULL;
    if (!aligned16(A) || !aligned16(out)) return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    if (!vectorisable(p, norm, false)) {
        if (vectorisable(p, FGE_NORM_NONE, false) && (int64_t)p->M * p->batch <= INT32_MAX) {
            // only the row's width stands in the way: one workgroup per row, passes over memory
            const Plan pl = make_plan(p, norm);
            const RowArgs r = row_args(A, out, FGE_ACT_NONE, norm, p, pl);
            const dim3 grid((unsigned)((int64_t)r.batch * r.M)), block(256);
            const size_t row_bytes = (size_t)r.N * esize(p->out_dtype);
            if (row_bytes <= ((size_t)64 << 10) - 256) {     // the row fits LDS twice per CU: read memory once
                if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((rownorm_wide_kernel<bf16_t, true>), grid, block, row_bytes, s, r);
                else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((rownorm_wide_kernel<f16_t, true>), grid, block, row_bytes, s, r);
                else                              hipLaunchKernelGGL((rownorm_wide_kernel<float, true>), grid, block, row_bytes, s, r);
            } else {
                if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((rownorm_wide_kernel<bf16_t, false>), grid, block, 0, s, r);
                else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((rownorm_wide_kernel<f16_t, false>), grid, block, 0, s, r);
                else                              hipLaunchKernelGGL((rownorm_wide_kernel<float, false>), grid, block, 0, s, r);
            }
            return hip_status(hipGetLastError());
        }
        GenArgs g = gen_args(p);
        g.X = A; g.ldx = p->ldo; g.bsx = g.bsd; g.dst = out; g.norm = norm;
        return hip_status(launch_generic_row(p->out_dtype, p->out_dtype, s, g));
    }
    const Plan pl = make_plan(p, norm);
    const RowArgs r = row_args(A, out, FGE_ACT_NONE, norm, p, pl);
    if (norm == FGE_NORM_NONE) {
        if (A == out) return FGE_OK;
        return do_act(A, FGE_ACT_NONE, p, out, s);       // plain copy
    }
    {
        // Rows of 8 KB and more: one workgroup per row with the row parked in LDS (the kernel of the
        // rows too wide for registers) instead of one wave per row with the row in its registers -
        // measured on 65536 rows: bf16 x 4096 columns +5 to +10 %, bf16 x 8192 +8 to +20 %, fp32 x 8192
        // (128 registers of row per lane in the wave kernel) up to +60 %, fp32 x 4096 within +-4 %;
        // below 8 KB the wave kernel wins (fp32 x 512: 5.9 against 3.9 TB/s).  With few rows the
        // workgroup form also puts four times as many waves on the chip.
        const int64_t rows = (int64_t)r.batch * r.M;
        const size_t row_bytes = (size_t)r.N * esize(p->out_dtype);
        if (row_bytes >= ((size_t)8 << 10) && row_bytes <= ((size_t)64 << 10) - 256 && rows <= INT32_MAX) {
            const dim3 grid((unsigned)rows), block(256);
            if (p->out_dtype == FGE_BF16)     hipLaunchKernelGGL((rownorm_wide_kernel<bf16_t, true>), grid, block, row_bytes, s, r);
            else if (p->out_dtype == FGE_F16) hipLaunchKernelGGL((rownorm_wide_kernel<f16_t, true>), grid, block, row_bytes, s, r);
            else                              hipLaunchKernelGGL((rownorm_wide_kernel<float, true>), grid, block, row_bytes, s, r);
            return hip_status(hipGetLastError());
        }
    }
    return p->out_dtype == FGE_BF16  ? launch_rownorm<bf16_t>(r, s)
           : p->out_dtype == FGE_F16 ? launch_rownorm<f16_t>(r, s)
                                     : launch_rownorm<float>(r, s);
}

}  // namespace

extern "C" {

int fge_fused_tiles(const void *X, const void *W, const float *b, int act, int norm,
                    const fge_params *p, void *out, void *stream) {
    return do_fused_tiles(X, W, b, act, norm, p, out, (hipStream_t)stream, nullptr);
}

int fge_fused_finish(int act, int norm, const fge_params *p, void *out, void *stream) {
    return do_fused_finish(act, norm, p, out, (hipStream_t)stream);
}

int fge_fused_needs_finish(int act, int norm, const fge_params *p) {
    const int rc = check_common(p, act, norm, true);
    if (rc) return -rc;
    return make_plan(p, norm, true).needs_finish ? 1 : 0;
}

int fge_fused_k_slices(int act, int norm, const fge_params *p) {
    const int rc = check_common(p, act, norm, true);
    if (rc) return -rc;
    return k_split(p, norm, make_plan(p, norm)).slices;
}

int fused_gemm_epilogue(const void *X, const void *W, const float *b, int act, int norm,
                        const fge_params *p, void *out, void *stream) {
    return run_fused(X, W, b, act, norm, p, out, (hipStream_t)stream);
}

int fge_static_scratch_init(void) {
    void *sp = nullptr;
    return static_scratch(&sp);
}

size_t fge_static_scratch_bytes(void) { return FGE_STATIC_SCRATCH_BYTES; }

int fused_gemm_epilogue_static(const void *X, const void *W, const float *b, int act, int norm,
                               const fge_params *p, void *out, void *stream) {
    // everything that can be refused is refused before the device is touched
    int rc = check_common(p, act, norm, true);
    if (rc) return rc;
    if (!X || !W || !out) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W) || !aligned16(out) || !aligned16(b)) return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    const Plan pl = make_plan(p, norm);
    const size_t need = pl.generic ? pl.ws_generic : split_rows_workspace(p, norm);
    if (need > FGE_STATIC_SCRATCH_BYTES) return FGE_ERR_WORKSPACE;
    fge_params q = *p;
    q.workspace = nullptr;
    q.workspace_bytes = 0;
    // (the K slices are optional: taken when their partial products fit the array as well)
    if (need > 0 || k_split(p, norm, pl).slices > 1) {
        void *sp = nullptr;
        if ((rc = static_scratch(&sp))) return rc;
        q.workspace = sp;
        q.workspace_bytes = FGE_STATIC_SCRATCH_BYTES;
    }
    return fused_gemm_epilogue(X, W, b, act, norm, &q, out, stream);
}

int fge_gemm_bias(const void *X, const void *W, const float *b, const fge_params *p, void *Y, void *stream) {
    return do_gemm_bias(X, W, b, p, Y, (hipStream_t)stream);
}

int fge_activation(const void *Y, int act, const fge_params *p, void *A, void *stream) {
    return do_act(Y, act, p, A, (hipStream_t)stream);
}

int fge_row_op(const void *A, int norm, const fge_params *p, void *out, void *stream) {
    return do_rownorm(A, norm, p, out, (hipStream_t)stream);
}

int unfused_gemm_epilogue(const void *X, const void *W, const float *b, int act, int norm,
                          const fge_params *p, void *out, void *stream) {
    int rc = check_common(p, act, norm, true);
    if (rc) return rc;
    if (!X || !W || !out) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W) || !aligned16(out) || !aligned16(b)) return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    const Plan pl = make_plan(p, norm);
    if (!p->workspace || p->workspace_bytes < pl.ws_buf * pl.n_bufs) return FGE_ERR_WORKSPACE;
    void *Y = p->workspace;
    void *A = pl.n_bufs == 2 ? static_cast<void *>(static_cast<char *>(p->workspace) + pl.ws_buf) : out;
    hipStream_t s = (hipStream_t)stream;
    if ((rc = do_gemm_bias(X, W, b, p, Y, s))) return rc;
    if ((rc = do_act(Y, act, p, A, s))) return rc;
    return do_rownorm(A, norm, p, out, s);
}

// ---- gated form: out = rowop(act(post*(alpha*X.W1^T + b1)) * (post*(alpha*X.W2^T + b2)))

int unfused_gated_gemm_epilogue(const void *X, const void *W1, const void *W2, const float *b1, const float *b2,
                                int act, int norm, const fge_params *p_in, void *out, void *stream) {
    int rc = check_common(p_in, act, norm, true);
    if (rc) return rc;
    // fp32 operands: the gate multiplies two products, and with it their errors - two split-bf16
    // products would leave the 1e-4 the fp32 path is held to, so both use the fp32 instruction
    fge_params q = *p_in;
    if (q.in_dtype == FGE_F32) q.flags |= FGE_FLAG_IEEE_FP32;
    const fge_params *p = &q;
    if (!X || !W1 || !W2 || !out) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W1) || !aligned16(W2) || !aligned16(out) || !aligned16(b1) || !aligned16(b2))
        return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    const Plan pl = make_plan(p, norm);
    if (!p->workspace || p->workspace_bytes < 2 * pl.ws_buf) return FGE_ERR_WORKSPACE;
    void *G = p->workspace;
    void *U = static_cast<char *>(p->workspace) + pl.ws_buf;
    void *A = pl.n_bufs == 2 ? G : out;             // the gate works in place where a row op follows
    hipStream_t s = (hipStream_t)stream;
    if ((rc = do_gemm_bias(X, W1, b1, p, G, s))) return rc;
    if ((rc = do_gemm_bias(X, W2, b2, p, U, s))) return rc;
    if ((rc = do_act(G, act, p, A, s, U))) return rc;
    return do_rownorm(A, norm, p, out, s);
}

// Gated form of a small problem with a long K: the gated tile kernel has 256-row tiles only, and
// with a handful of them most of the chip idles (16 x 4096 x 4096: 84 us, against 52 us for the
// unfused sequence).  Such a problem runs like a K-split instead: both products as fp32 partial
// products (one slice if K is not worth cutting), one kernel that adds the slices and applies
// scale, bias, activation and the gate in fp32, then the row op.
struct GatedSmall {
    bool use;
    Plan pl;                     // plan of one plain product of this shape
    KSplit ks;                   // slices of each product; ws_part bytes per product
    size_t bytes() const { return 2 * ks.ws_part + ks.ws_mid; }
};

GatedSmall gated_small(const fge_params *p, int norm) {
    GatedSmall g{false, make_plan(p, norm), {1, 0, 0}};
    const Plan &pl = g.pl;
    if (!gated_fast(p, norm) || pl.generic || pl.pr.batch != 1 || pl.tile == TILE_PANEL || pl.pr.K < 1024) return g;
    if (norm != FGE_NORM_NONE && pl.pr.N > MAX_ROWOP_N) return g;
    const TileInfo &gt = tile_info(TILE_GATED);
    const int64_t gated_tiles = (int64_t)((pl.pr.M + gt.bm - 1) / gt.bm) * ((pl.pr.N + gt.bn - 1) / gt.bn);
    // from about 96 of its tiles on the gated kernel is the faster one, and so it is when one plain
    // product alone has more 64x64 tiles than two per CU (256 x 4096 x 11008: 86 against 117 us)
    if (gated_tiles * 8 > num_cu() * 3 || pl.tile != TILE_64x64 || (int64_t)pl.tiles_m * pl.tiles_n > 2 * num_cu()) return g;
    g.ks = k_split(p, norm, pl);
    if (g.ks.slices == 1) {
        const size_t one = round256((size_t)pl.pr.M * pl.pr.N * sizeof(float));
        g.ks.ws_part = one;
        g.ks.ws_mid = norm == FGE_NORM_NONE ? 0 : one;
    }
    g.use = true;
    return g;
}

int fused_gated_gemm_epilogue(const void *X, const void *W1, const void *W2, const float *b1, const float *b2,
                              int act, int norm, const fge_params *p, void *out, void *stream) {
    int rc = check_common(p, act, norm, true);
    if (rc) return rc;
    if (!gated_fast(p, norm))                       // everything the gated tile kernel does not take
        return unfused_gated_gemm_epilogue(X, W1, W2, b1, b2, act, norm, p, out, stream);
    if (!X || !W1 || !W2 || !out) return FGE_ERR_NULL;
    if (!aligned16(X) || !aligned16(W1) || !aligned16(W2) || !aligned16(out) || !aligned16(b1) || !aligned16(b2))
        return FGE_ERR_ALIGN;
    if (norm == FGE_NORM_LOGSUMEXP && !p->aux_out) return FGE_ERR_NULL;
    hipStream_t s = (hipStream_t)stream;
    const GatedSmall gs = gated_small(p, norm);
    if (gs.use && p->workspace && p->workspace_bytes >= gs.bytes()) {
        const int S = gs.ks.slices;
        char *part = static_cast<char *>(p->workspace);
        const int64_t slice = (int64_t)(gs.ks.ws_part / S / sizeof(float));
        if ((rc = launch_partials(X, W1, p, gs.pl, S, slice, part, s))) return rc;
        if ((rc = launch_partials(X, W2, p, gs.pl, S, slice, part + gs.ks.ws_part, s))) return rc;
        return finish_partials(part, part + gs.ks.ws_part, b1, b2, act, norm, p, gs.pl, S, slice,
                               part + 2 * gs.ks.ws_part, out, s);
    }
    Plan pl = make_plan(p, norm, capturing(s), TILE_GATED);
    if (pl.split) {
        if (pl.strips > MAX_SPLIT) return FGE_ERR_UNSUPPORTED;
        if (!p->workspace || p->workspace_bytes < gated_workspace(p, norm)) return FGE_ERR_WORKSPACE;
    }
    for (int attempt = 0;; ++attempt) {
        TileArgs a = tile_args(X, W1, b1, act, norm, p, pl, out);
        a.W2 = W2; a.b2 = b2;
        const dim3 grid(a.coop ? (unsigned)pl.coop_grid : (unsigned)(pl.tiles_m * pl.tiles_n), 1,
                        a.coop ? 1u : (unsigned)pl.pr.batch);
        rc = hip_status(p->in_dtype == FGE_BF16  ? launch_gated_bf16(p->out_dtype, grid, s, a)
                        : p->in_dtype == FGE_F16 ? launch_gated_f16(p->out_dtype, grid, s, a)
                                                 : launch_gated_f8(p->out_dtype, grid, s, a));
        // a cooperative grid the device cannot hold is refused before anything runs: two-pass form
        if (attempt == 0 && rc == FGE_ERR_HIP && pl.coop && g_last_hip == (int)hipErrorCooperativeLaunchTooLarge) {
            pl = make_plan(p, norm, true, TILE_GATED);
            continue;
        }
        break;
    }
    if (rc || !pl.needs_finish) return rc;
    return launch_finish(pl, act, norm, p, out, s);
}

size_t fge_gated_workspace_bytes(int fused, int act, int norm, const fge_params *p) {
    if (check_common(p, act, norm, true)) return (size_t)-1;
    if (!fused || !gated_fast(p, norm)) return 2 * make_plan(p, norm).ws_buf;
    const size_t a = gated_workspace(p, norm);
    const GatedSmall gs = gated_small(p, norm);
    return gs.use && gs.bytes() > a ? gs.bytes() : a;
}

const char *fge_gated_tile_name(int act, int norm, const fge_params *p) {
    if (check_common(p, act, norm, true)) return nullptr;
    if (!gated_fast(p, norm)) return "unfused_sequence";
    return gated_small(p, norm).use ? "partial_products_then_gate" : tile_info(TILE_GATED).name;
}

size_t fge_fault_word_offset(int act, int norm, const fge_params *p) {
    if (check_common(p, act, norm, true)) return (size_t)-1;
    const Plan pl = make_plan(p, norm);
    return pl.coop ? pl.ws_stats + pl.ws_marks - 256 : (size_t)-1;
}

size_t fge_workspace_bytes(int fused, int act, int norm, const fge_params *p) {
    if (check_common(p, act, norm, true)) return (size_t)-1;
    const Plan pl = make_plan(p, norm);
    return fused ? fused_workspace(p, norm) : pl.ws_buf * pl.n_bufs;
}

const char *fge_status_string(int status) {
    switch (status) {
    case FGE_OK:              return "ok";
    case FGE_ERR_NULL:        return "a required pointer is NULL";
    case FGE_ERR_BAD_ENUM:    return "activation, row-op, dtype or flag code out of range";
    case FGE_ERR_BAD_SHAPE:   return "non-positive extent or stride smaller than the extent";
    case FGE_ERR_UNSUPPORTED: return "valid request outside the supported set";
    case FGE_ERR_ALIGN:       return "base pointer not 16-byte aligned";
    case FGE_ERR_WORKSPACE:   return "workspace missing or too small (static form: problem beyond the library's scratch array)";
    case FGE_ERR_HIP:         return "HIP launch failed";
    default:                  return "unknown status";
    }
}

int fge_last_hip_error(void) { return g_last_hip; }

const char *fge_tile_name(int fused, int act, int norm, const fge_params *p) {
    if (check_common(p, act, norm, true)) return nullptr;
    const Plan pl = make_plan(p, fused ? norm : FGE_NORM_NONE);
    if (pl.generic) return fused && plan_repack(p, norm).use ? "repacked_operands" : "generic32x32_scalar";
    const TileInfo &ti = tile_info(pl.tile);
    return p->in_dtype == FGE_F32 && !(p->flags & FGE_FLAG_IEEE_FP32) ? ti.name_split : ti.name;
}

}  // extern "C"
