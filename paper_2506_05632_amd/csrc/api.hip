// C ABI of libllc_hip.so: argument checks, launch planning, kernel launches.
#include <cmath>
#include <cstring>

#include "common.hpp"

namespace llc {
namespace {

constexpr int kMaxChunks = 4096;
constexpr long long kMaxBlocks = 0xFFFFFFFFLL / kBlock;  // workgroups of one launch
constexpr int kPlannedChunkFloor = 16;  // the workspace always covers this many chunks
constexpr long long kTargetBlocks = 1024;  // four resident workgroups on each of 256 CUs
constexpr long long kMinTilesPerChunk = 8; // a chunk pays its own warm-up: keep it worth it

inline size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

struct Plan {
  int kt, n_kgroups, n_chunks, groups_per_chunk;
};

// Drafts per workgroup pass.  With one shared proposal the per-index work is amortised over the
// drafts of a pass, so wider is better; with per-draft rows each draft brings its own loads and
// thresholds and four keep the kernel within 128 VGPRs.
int auto_ktile(long long K, bool shared) {
  if (K >= 5 && shared) return 8;
  return K >= 3 ? 4 : 2;
}

// Split the G four-element groups of a row into chunks of a multiple of kBlock groups.
void plan_chunks(long long G, int want, int *n_chunks, int *groups_per_chunk) {
  const long long tiles = (G + kBlock - 1) / kBlock;  // 256-group tiles in a row
  long long nc = want < 1 ? 1 : want;
  if (nc > tiles) nc = tiles;
  if (nc > kMaxChunks) nc = kMaxChunks;
  const long long tiles_per_chunk = (tiles + nc - 1) / nc;
  *groups_per_chunk = (int)(tiles_per_chunk * kBlock);
  *n_chunks = (int)((tiles + tiles_per_chunk - 1) / tiles_per_chunk);
}

int auto_chunks(long long B, long long n_kgroups, long long G) {
  const long long rows = B * n_kgroups;
  if (rows >= kTargetBlocks || rows <= 0) return 1;
  long long c = (kTargetBlocks + rows - 1) / rows;
  const long long tiles = (G + kBlock - 1) / kBlock;
  const long long most = tiles / kMinTilesPerChunk;
  if (c > most) c = most;
  if (c < 1) c = 1;
  return (int)(c > kMaxChunks ? kMaxChunks : c);
}

struct Layout {
  size_t keyX, idxX, keyY, idxY, kY, secX, secY, lse, lse_part, shared_tau, total;
};

Layout layout_for(long long B, long long K, long long n_kgroups, long long n_chunks) {
  Layout l;
  size_t off = 0;
  l.keyX = off; off += align256((size_t)(B * K * n_chunks) * sizeof(double));
  l.idxX = off; off += align256((size_t)(B * K * n_chunks) * sizeof(int32_t));
  l.keyY = off; off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(double));
  l.idxY = off; off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(int32_t));
  l.kY = off;   off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(int32_t));
  l.secX = off; off += align256((size_t)(B * K * n_chunks) * sizeof(double));
  l.secY = off; off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(double));
  l.lse = off;  off += align256((size_t)(B * (K + 1)) * sizeof(double));
  l.lse_part = off; off += align256((size_t)(B * (K + 1) * n_chunks) * sizeof(double));
  l.shared_tau = off; off += align256((size_t)(B * (K + 1)) * sizeof(int32_t));
  l.total = off;
  return l;
}

bool shape_ok(long long B, long long K, long long V) {
  return B >= 0 && K >= 1 && K <= 65535 && V >= 1 && V < 2147483644LL &&
         B <= (1LL << 40);
}

bool good_temp(float t) { return std::isfinite(t) && t > 0.0f; }

RowMap plain_rows(long long draft_stride_b, long long target_stride_b) {
  RowMap m;
  m.inner_count = 1;
  m.draft_outer = draft_stride_b; m.draft_inner = 0;
  m.target_outer = target_stride_b; m.target_inner = 0;
  m.row_outer = 1; m.row_inner = 0;
  return m;
}

// llc_verify keeps, beyond the scan's partials, ln(key) [B][K] fp64 and the index [B][K], and for
// the strong form the loop's state: per sequence K viability bytes, a running flag and the next
// position's row offset; the running bests that the scans of positions 1..L share; the
// normalisers of every row and of the rows that price the position at hand.
struct VerifyExtra {
  size_t cand_key, cand_sec, cand, viable, running, next_off, tau_all, lse, lse_sel, total;
};
VerifyExtra verify_extra(long long S, long long B, long long K) {  // B = S (L + 1)
  VerifyExtra e;
  size_t off = 0;
  e.cand_key = off; off += align256((size_t)(B * K) * sizeof(double));
  e.cand_sec = off; off += align256((size_t)(B * K) * sizeof(double));
  e.cand = off; off += align256((size_t)(B * K) * sizeof(int32_t));
  e.viable = off; off += align256((size_t)(S * K));
  e.running = off; off += align256((size_t)S * sizeof(int32_t));
  e.next_off = off; off += align256((size_t)S * sizeof(long long));
  e.tau_all = off; off += align256((size_t)((B - S) * (K + 1)) * sizeof(int32_t));  // running bests of positions 1..L
  e.lse = off; off += align256((size_t)(B * (K + 1)) * sizeof(double));      // the one-shot scan's normalisers
  e.lse_sel = off; off += align256((size_t)(S * (K + 1)) * sizeof(double));  // those of the rows that price a position
  e.total = off;
  return e;
}

// One scan over B rows: what llc_couple and llc_verify have in common.
struct ScanJob {
  long long B, K, V;
  int dtype, kind;
  const void *draft, *target;
  RowMap map;
  long long draft_stride_k;
  float temp_target, temp_draft_all;
  const float *temp_draft;
  uint64_t seed, row_offset;
  bool no_pool;      // draft-side reductions only
  bool need_lse;     // also compute the row normalisers (log kinds)
  bool no_draft = false;    // pool only
  bool same_race = false;   // every draft uses draft 0's race times
  bool min_first = false;   // the race times of an index are drawn through their minimum
  bool force_perk = false;  // every draft has its own row even if draft_stride_k == 0
  const uint8_t *bins = nullptr;  // binned candidates: mask of the draft rows (see ScanParams)
  long long bins_stride_b = 0;
  const int32_t *bin_of = nullptr;
  const long long *draft_row_off = nullptr;  // per-row extra offset of the draft row (see ScanParams)
  long long draft_row_off_unit = 0;  // every entry of draft_row_off is a multiple of this many elements
  size_t lse_in_extra = (size_t)-1;  // keep the normalisers at this offset of the caller's region
  size_t extra_at = (size_t)-1;      // where the caller's region starts (default: right behind the partials)
  int32_t *tau_ready = nullptr;      // the rows' shared running bests, already reset, if not in the workspace
  const FinalizeParams *fin = nullptr;  // if given, the scan may take the finalize step itself (plain
                                     // scans only); `in`, n_chunks and n_kgroups are filled in here
  int flags, v_chunks, k_tile;
  llc_stats *stats;
  void *workspace;
  size_t workspace_bytes, extra_bytes;  // extra_bytes: caller's own region behind the partials
  void *stream, *ev_begin, *ev_end;
};

// What the host decides about one scan before anything is launched.
struct ScanPlan {
  Plan pl;
  Layout lay;
  bool shared, vec;
  long long blocks;
};

// Checks the options and plans the launch; touches neither the workspace nor the device.
int plan_scan(const ScanJob &j, ScanPlan *out) {
  if (j.dtype != LLC_F32 && j.dtype != LLC_BF16) return LLC_E_DTYPE;
  if (j.kind != LLC_LOGITS && j.kind != LLC_PROBS && j.kind != LLC_LOGW) return LLC_E_DTYPE;
  if (j.flags & ~LLC_FLAG_EXACT_SCAN) return LLC_E_OPTION;  // (the entry points strip their own flags)
  if (j.min_first && (j.bins != nullptr || j.no_draft || j.same_race)) return LLC_E_OPTION;
  if (j.v_chunks < 0 || j.v_chunks > kMaxChunks) return LLC_E_OPTION;
  if (j.k_tile != 0 && j.k_tile != 1 && j.k_tile != 2 && j.k_tile != 4 && j.k_tile != 8)
    return LLC_E_OPTION;
  const bool logits = j.kind == LLC_LOGITS;
  if (logits) {
    if (!good_temp(j.temp_target)) return LLC_E_TEMP;
    if (j.temp_draft == nullptr && !good_temp(j.temp_draft_all)) return LLC_E_TEMP;
  }
  const size_t esize = j.dtype == LLC_F32 ? 4 : 2;
  if (((uintptr_t)j.draft % esize) != 0 || ((uintptr_t)j.target % esize) != 0) return LLC_E_ALIGN;

  const float *temp_draft = logits ? j.temp_draft : nullptr;
  const bool shared = j.draft_stride_k == 0 && temp_draft == nullptr && !j.force_perk;

  Plan &pl = out->pl;
  pl.kt = j.k_tile != 0 ? (j.k_tile == 1 ? 2 : j.k_tile) : auto_ktile(j.K, shared);
  pl.n_kgroups = (int)((j.K + pl.kt - 1) / pl.kt);
  const long long G = (j.V + 3) / 4;
  plan_chunks(G, j.v_chunks != 0 ? j.v_chunks : auto_chunks(j.B, pl.n_kgroups, G), &pl.n_chunks,
              &pl.groups_per_chunk);
  out->blocks = j.B * pl.n_kgroups * pl.n_chunks;
  // (a launch takes fewer than 2^32 threads in all)
  if (out->blocks > kMaxBlocks) return LLC_E_SHAPE;
  out->lay = layout_for(j.B, j.K, pl.n_kgroups, pl.n_chunks);
  out->shared = shared;

  // vector loads need every row to start on a 4-element boundary of a 16-byte (fp32) or
  // 8-byte (bf16) aligned base (per-row offsets of the draft rows included)
  const size_t vbytes = 4 * esize;
  const RowMap &m = j.map;
  out->vec = ((uintptr_t)j.draft % vbytes) == 0 && ((uintptr_t)j.target % vbytes) == 0 &&
             (m.draft_outer % 4) == 0 && (m.draft_inner % 4) == 0 && (j.draft_stride_k % 4) == 0 &&
             (m.target_outer % 4) == 0 && (m.target_inner % 4) == 0 &&
             (j.draft_row_off == nullptr || (j.draft_row_off_unit % 4) == 0);
  return LLC_OK;
}

// Where the caller's own region starts, and what the whole call needs.
size_t extra_offset(const ScanJob &j, const ScanPlan &sp) {
  return j.extra_at == (size_t)-1 ? sp.lay.total : j.extra_at;
}
bool workspace_ok(const ScanJob &j, const ScanPlan &sp) {
  const size_t at = extra_offset(j, sp);
  return j.workspace != nullptr && ((uintptr_t)j.workspace & 255) == 0 && at >= sp.lay.total &&
         j.workspace_bytes >= at + j.extra_bytes;
}

// Carves the workspace and enqueues the normaliser pass (if asked) and the scan kernel of a
// planned job whose workspace has been checked.  *extra (if given) receives the caller's region.
int launch_scan_job(const ScanJob &j, const ScanPlan &plan, Partials *partials, char **extra,
                    bool *finished = nullptr) {
  const Plan &pl = plan.pl;
  const Layout &lay = plan.lay;
  const bool shared = plan.shared, vec = plan.vec;
  const long long blocks = plan.blocks;
  const bool logits = j.kind == LLC_LOGITS;
  const float *temp_draft = logits ? j.temp_draft : nullptr;
  char *ws = (char *)j.workspace;
  const size_t extra_off = extra_offset(j, plan);
  if (extra != nullptr) *extra = ws + extra_off;

  hipStream_t st = (hipStream_t)j.stream;
  Partials part;
  part.keyX = (double *)(ws + lay.keyX);
  part.idxX = (int32_t *)(ws + lay.idxX);
  part.keyY = (double *)(ws + lay.keyY);
  part.idxY = (int32_t *)(ws + lay.idxY);
  part.kY = (int32_t *)(ws + lay.kY);
  part.secX = (double *)(ws + lay.secX);
  part.secY = (double *)(ws + lay.secY);
  part.lse = (double *)(ws + (j.lse_in_extra == (size_t)-1 ? lay.lse : extra_off + j.lse_in_extra));

  // Row normalisers: the scan forms them on its way (no second pass over the inputs): the draft
  // rows' always, the target row's too when one proposal serves all drafts (the workgroup then
  // reads two rows in all); the binned passes, and the target row beside per-draft rows, use the
  // normaliser kernel.
  const bool masked = j.bins != nullptr || j.no_draft || j.same_race;
  const bool fused_lse = j.need_lse && j.kind != LLC_PROBS && !masked;
  part.lse_part = fused_lse ? (double *)(ws + lay.lse_part) : nullptr;
  part.lse_part_target = (fused_lse && shared && !j.no_pool) ? 1 : 0;
  if (j.need_lse && j.kind != LLC_PROBS && (!fused_lse || (!j.no_pool && !part.lse_part_target))) {
    LseParams lp;
    lp.draft = j.draft; lp.target = j.target;
    lp.map = j.map; lp.draft_stride_k = j.draft_stride_k;
    lp.B = j.B; lp.K = (int)j.K; lp.V = (int)j.V; lp.dtype = j.dtype;
    lp.temp_target = logits ? j.temp_target : 1.0f;
    lp.temp_draft_all = logits ? j.temp_draft_all : 1.0f;
    lp.temp_draft = temp_draft;
    lp.is_logits = logits ? 1 : 0;
    lp.per_k = shared ? 0 : 1;
    lp.with_target = j.no_pool ? 0 : 1;
    lp.with_drafts = fused_lse ? 0 : 1;
    lp.vector_loads = vec ? 1 : 0;
    lp.bins = j.bins; lp.bins_stride_b = j.bins_stride_b; lp.bin_of = j.bin_of;
    lp.draft_row_off = j.draft_row_off;
    lp.lse = part.lse;
    if (launch_lse(st, lp) != hipSuccess) return LLC_E_LAUNCH;
  }

  // Where every row is one workgroup, a plain scan (no bins, no normalisers to merge) takes the
  // finalize step itself: one launch less.  (For rows spread over several workgroups the same was
  // tried with a ticket per row, the last workgroup finishing the row: publishing the partial
  // results needs either device-scope fences, which write back and invalidate an XCD's whole L2
  // and doubled the scan's time, or write-through stores and reads, whose latency at the end of
  // the launch cost more than the finalize launch they saved.)
  const bool finish = j.fin != nullptr && !masked && !fused_lse && pl.n_chunks * pl.n_kgroups == 1;
  if (finished != nullptr) *finished = finish;

  // a row spread over several workgroups shares its running bests through the workspace
  int32_t *shared_tau = nullptr;
  if (pl.n_chunks * pl.n_kgroups > 1) {
    if (j.tau_ready != nullptr) {
      shared_tau = j.tau_ready;
    } else {
      shared_tau = (int32_t *)(ws + lay.shared_tau);
      if (launch_fill(st, shared_tau, j.B * (j.K + 1), 0x7F800000) != hipSuccess) return LLC_E_LAUNCH;
    }
  }

  ScanParams sp;
  sp.shared_tau = shared_tau;
  sp.lse_part = part.lse_part;
  sp.bins = j.bins; sp.bins_stride_b = j.bins_stride_b; sp.bin_of = j.bin_of;
  sp.draft_row_off = j.draft_row_off;
  sp.draft = j.draft; sp.target = j.target;
  sp.map = j.map; sp.draft_stride_k = j.draft_stride_k;
  sp.B = j.B; sp.K = (int)j.K; sp.V = (int)j.V;
  sp.n_chunks = pl.n_chunks; sp.groups_per_chunk = pl.groups_per_chunk; sp.n_kgroups = pl.n_kgroups;
  sp.seed_lo = (unsigned)j.seed; sp.seed_hi = (unsigned)(j.seed >> 32);
  sp.row_offset = j.row_offset;
  sp.temp_target = logits ? j.temp_target : 1.0f;
  sp.temp_draft_all = logits ? j.temp_draft_all : 1.0f;
  sp.temp_draft = temp_draft;
  sp.vector_loads = vec ? 1 : 0;
  sp.force_exact = (j.flags & LLC_FLAG_EXACT_SCAN) ? 1 : 0;
  sp.no_pool = j.no_pool ? 1 : 0;
  sp.no_draft = j.no_draft ? 1 : 0;
  sp.same_race = j.same_race ? 1 : 0;
  sp.out = part;
  sp.stats = j.stats;
  if (finish) {
    sp.fin = *j.fin;
    sp.fin.in = part;
    sp.fin.n_chunks = pl.n_chunks;
    sp.fin.n_kgroups = pl.n_kgroups;
  } else {
    std::memset(&sp.fin, 0, sizeof(sp.fin));
  }

  const bool probs = j.kind == LLC_PROBS;
  if (j.ev_begin != nullptr && hipEventRecord((hipEvent_t)j.ev_begin, st) != hipSuccess)
    return LLC_E_LAUNCH;
  hipError_t e;
  if (j.min_first) {
    if (j.dtype == LLC_F32)
      e = shared ? launch_scan_f32_shared_minf(pl.kt, probs, finish, (unsigned)blocks, st, sp)
                 : launch_scan_f32_perk_minf(pl.kt, probs, finish, (unsigned)blocks, st, sp);
    else
      e = shared ? launch_scan_bf16_shared_minf(pl.kt, probs, finish, (unsigned)blocks, st, sp)
                 : launch_scan_bf16_perk_minf(pl.kt, probs, finish, (unsigned)blocks, st, sp);
  } else if (j.dtype == LLC_F32) {
    e = shared ? launch_scan_f32_shared(pl.kt, probs, finish, (unsigned)blocks, st, sp)
               : launch_scan_f32_perk(pl.kt, probs, finish, (unsigned)blocks, st, sp);
  } else {
    e = shared ? launch_scan_bf16_shared(pl.kt, probs, finish, (unsigned)blocks, st, sp)
               : launch_scan_bf16_perk(pl.kt, probs, finish, (unsigned)blocks, st, sp);
  }
  if (e != hipSuccess) return LLC_E_LAUNCH;
  if (j.ev_end != nullptr && hipEventRecord((hipEvent_t)j.ev_end, st) != hipSuccess)
    return LLC_E_LAUNCH;
  *partials = part;
  return LLC_OK;
}

// Plan, check the workspace, launch.  With the dry-run flag nothing is launched (*dry is set).
int run_scan(const ScanJob &j, bool dry_run, Plan *plan, Partials *partials, char **extra,
             bool *finished = nullptr) {
  ScanPlan sp;
  const int rc = plan_scan(j, &sp);
  if (rc != LLC_OK) return rc;
  if (!workspace_ok(j, sp)) return LLC_E_WORKSPACE;
  *plan = sp.pl;
  if (dry_run) return LLC_OK;
  return launch_scan_job(j, sp, partials, extra, finished);
}

}  // namespace

// llc_couple on a given workspace (the caller's, or the library's own static one).
int couple_on(const llc_couple_args *a, void *workspace, size_t workspace_bytes) {
  if (a == nullptr) return LLC_E_NULL;
  if (!shape_ok(a->B, a->K, a->V)) return LLC_E_SHAPE;
  if (a->B == 0) return LLC_OK;  // nothing to read or write: pointers may be NULL
  // the drafters' step of Algorithm 2: the draft side alone (no target is read, no Y, no accept test)
  const bool draft_only = (a->flags & LLC_FLAG_DRAFT_ONLY) != 0;
  if (a->draft == nullptr || a->X == nullptr) return LLC_E_NULL;
  if (!draft_only && (a->target == nullptr || a->Y == nullptr || a->accept == nullptr)) return LLC_E_NULL;
  if (a->draft_stride_b < 0 || a->draft_stride_k < 0 || (!draft_only && a->target_stride_b < 0)) return LLC_E_SHAPE;
  const bool dry = (a->flags & LLC_FLAG_DRY_RUN) != 0;

  ScanJob j;
  j.B = a->B; j.K = a->K; j.V = a->V; j.dtype = a->dtype; j.kind = a->kind;
  j.draft = a->draft;
  j.target = draft_only ? a->draft : a->target;  // (without a pool the target is never read)
  j.map = plain_rows(a->draft_stride_b, draft_only ? a->draft_stride_b : a->target_stride_b);
  j.draft_stride_k = a->draft_stride_k;
  j.temp_target = draft_only ? 1.0f : a->temp_target;
  j.temp_draft_all = a->temp_draft_all; j.temp_draft = a->temp_draft;
  j.seed = a->seed; j.row_offset = a->row_offset;
  j.no_pool = draft_only;
  j.need_lse = a->keyX != nullptr || (!draft_only && a->keyY != nullptr);
  j.min_first = (a->flags & LLC_FLAG_MIN_FIRST) != 0;
  j.flags = a->flags & ~(LLC_FLAG_DRY_RUN | LLC_FLAG_MIN_FIRST | LLC_FLAG_DRAFT_ONLY);
  j.v_chunks = a->v_chunks; j.k_tile = a->k_tile;
  j.stats = a->stats; j.workspace = workspace; j.workspace_bytes = workspace_bytes;
  j.stream = a->stream; j.ev_begin = a->ev_scan_begin; j.ev_end = a->ev_scan_end;
  j.extra_bytes = 0;

  FinalizeParams fp;
  fp.cand = nullptr; fp.side = nullptr; fp.source = nullptr; fp.W = nullptr; fp.A_hat = nullptr; fp.sq_err = nullptr;
  fp.cand_stride_b = 0; fp.side_stride_b = 0; fp.var_e = 0.0; fp.var_z = 0.0;
  fp.B = a->B; fp.K = (int)a->K; fp.n_chunks = 0; fp.n_kgroups = 0;
  fp.log_kind = a->kind != LLC_PROBS ? 1 : 0;
  std::memset(&fp.in, 0, sizeof(fp.in));
  fp.X = a->X; fp.Y = a->Y; fp.match_k = a->match_k; fp.accept = a->accept;
  fp.keyX = a->keyX; fp.keyY = a->keyY; fp.log_keyX = nullptr; fp.log_secX = nullptr;
  fp.y_given = 0; fp.bins = nullptr; fp.bins_stride_b = 0; fp.message = nullptr;
  fp.count_draft = 1; fp.count_pool = 1; fp.count_near = 1;
  if (draft_only) {  // (Y == nullptr is what tells the finalize step that there is no pool)
    fp.Y = nullptr; fp.accept = nullptr; fp.match_k = nullptr; fp.keyY = nullptr; fp.count_pool = 0;
  }
  fp.stats = a->stats;
  j.fin = &fp;  // (where it can, the scan finishes the rows itself and no finalize launch follows)

  Plan pl;
  Partials part;
  bool finished = false;
  const int rc = run_scan(j, dry, &pl, &part, nullptr, &finished);
  if (rc != LLC_OK || dry || finished) return rc;
  fp.n_chunks = pl.n_chunks; fp.n_kgroups = pl.n_kgroups;
  fp.in = part;
  if (launch_finalize((hipStream_t)a->stream, fp) != hipSuccess) return LLC_E_LAUNCH;
  return LLC_OK;
}

}  // namespace llc

using namespace llc;

extern "C" {

int llc_version(void) { return LLC_VERSION; }

const char *llc_status_string(int code) {
  switch (code) {
    case LLC_OK: return "ok";
    case LLC_E_NULL: return "a required pointer is NULL";
    case LLC_E_SHAPE: return "bad shape or strides";
    case LLC_E_TEMP: return "temperature must be finite and > 0";
    case LLC_E_DTYPE: return "unsupported dtype or kind";
    case LLC_E_ALIGN: return "input pointer not aligned to its element size";
    case LLC_E_WORKSPACE: return "workspace missing, misaligned or too small";
    case LLC_E_LAUNCH: return "kernel launch failed";
    case LLC_E_OPTION: return "v_chunks, k_tile, flags or list sizes out of range";
    case LLC_E_SCRATCH: return "the call needs more than the library's static scratch (LLC_STATIC_SCRATCH_BYTES)";
    default: return "unknown status";
  }
}

size_t llc_couple_workspace_size(int64_t B, int64_t K, int64_t V) {
  if (!shape_ok(B, K, V)) return 0;
  // worst case over k_tile (one draft per group) and over v_chunks up to the planned floor
  const long long G = (V + 3) / 4;
  int nc, gpc;
  int want = auto_chunks(B, 1, G);
  if (want < kPlannedChunkFloor) want = kPlannedChunkFloor;
  plan_chunks(G, want, &nc, &gpc);
  return layout_for(B, K, K, nc).total + 256;
}

int llc_couple(const llc_couple_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  return couple_on(a, a->workspace, a->workspace_bytes);
}

int llc_compress_select(const llc_compress_select_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  if (!shape_ok(a->B, a->L, a->N)) return LLC_E_SHAPE;
  if (a->B == 0) return LLC_OK;
  if (a->logw_enc == nullptr || a->logw_dec == nullptr || a->bins == nullptr || a->X == nullptr ||
      a->Y == nullptr || a->accept == nullptr)
    return LLC_E_NULL;
  if (a->enc_stride_b < 0 || a->dec_stride_b < 0 || a->dec_stride_l < 0 || a->bins_stride_b < 0)
    return LLC_E_SHAPE;
  // the decoders' outputs (optional): candidates, side information and the two variances
  const bool decode = a->W != nullptr || a->A_hat != nullptr || a->sq_err != nullptr;
  if (decode) {
    const bool estimate = a->A_hat != nullptr || a->sq_err != nullptr;
    if (a->cand == nullptr || (estimate && a->side == nullptr)) return LLC_E_NULL;
    if (a->sq_err != nullptr && a->source == nullptr) return LLC_E_NULL;
    if (a->cand_stride_b < 0 || a->side_stride_b < 0) return LLC_E_SHAPE;
    if (estimate && (!good_temp(a->var_w_given_a) || !good_temp(a->var_t_given_a))) return LLC_E_OPTION;
  }
  hipStream_t st = (hipStream_t)a->stream;
  const bool dry = (a->flags & LLC_FLAG_DRY_RUN) != 0;
  // the baseline of Section 5.3: one set of race times for the encoder and every decoder
  const bool same_race = (a->flags & LLC_FLAG_SHARED_RACE) != 0;

  // pass 1, the encoder: Y = the pool argmin under lambda_q over the L sets of race times (the
  // shared-proposal scan without a draft side; its X comes out as -1 and pass 2 overwrites it)
  ScanJob j;
  j.B = a->B; j.K = same_race ? 1 : a->L; j.V = a->N; j.dtype = LLC_F32; j.kind = LLC_LOGW;
  j.draft = a->logw_enc; j.target = a->logw_enc;
  j.map = plain_rows(a->enc_stride_b, a->enc_stride_b);
  j.draft_stride_k = 0;
  j.temp_target = 1.0f; j.temp_draft_all = 1.0f; j.temp_draft = nullptr;
  j.seed = a->seed; j.row_offset = a->row_offset;
  j.no_pool = false;
  j.no_draft = true;
  j.need_lse = a->keyY != nullptr;
  j.flags = a->flags & ~(LLC_FLAG_DRY_RUN | LLC_FLAG_SHARED_RACE); j.v_chunks = a->v_chunks; j.k_tile = a->k_tile;
  j.stats = a->stats; j.workspace = a->workspace; j.workspace_bytes = a->workspace_bytes;
  j.stream = a->stream; j.ev_begin = nullptr; j.ev_end = nullptr;
  j.extra_bytes = 0;
  Plan pl;
  Partials part;
  int rc = run_scan(j, dry, &pl, &part, nullptr);
  if (rc != LLC_OK) return rc;
  if (dry) {  // the decoders' pass is planned as well, nothing is launched
    j.K = a->L; j.same_race = same_race;
    j.draft = a->logw_dec; j.map = plain_rows(a->dec_stride_b, a->enc_stride_b);
    j.draft_stride_k = a->dec_stride_l; j.no_pool = true; j.no_draft = false;
    j.bins = a->bins; j.bins_stride_b = a->bins_stride_b; j.bin_of = a->Y;
    return run_scan(j, true, &pl, &part, nullptr);
  }
  FinalizeParams fp;
  fp.cand = nullptr; fp.side = nullptr; fp.source = nullptr; fp.W = nullptr; fp.A_hat = nullptr; fp.sq_err = nullptr;
  fp.cand_stride_b = 0; fp.side_stride_b = 0; fp.var_e = 0.0; fp.var_z = 0.0;
  // (with one shared set of race times the pool runs over that set alone: K = 1 in this pass)
  fp.B = a->B; fp.K = (int)j.K; fp.n_chunks = pl.n_chunks; fp.n_kgroups = pl.n_kgroups;
  fp.log_kind = 1;
  fp.in = part;
  fp.X = a->X; fp.Y = a->Y; fp.match_k = nullptr; fp.accept = a->accept;
  fp.keyX = nullptr; fp.keyY = a->keyY; fp.log_keyX = nullptr; fp.log_secX = nullptr;
  fp.y_given = 0; fp.bins = nullptr; fp.bins_stride_b = 0; fp.message = nullptr;
  fp.count_draft = 0; fp.count_pool = 1; fp.count_near = 1;  // pass 1's draft side is not part of the result
  fp.stats = a->stats;
  if (launch_finalize(st, fp) != hipSuccess) return LLC_E_LAUNCH;

  // pass 2, the decoders: X^(l) = argmin under lambda_p^(l) over the candidates of Y's bin
  j.K = a->L; j.same_race = same_race;
  j.draft = a->logw_dec; j.target = a->logw_enc;
  j.map = plain_rows(a->dec_stride_b, a->enc_stride_b);
  j.draft_stride_k = a->dec_stride_l;
  j.no_pool = true;
  j.no_draft = false;
  j.need_lse = a->keyX != nullptr;
  j.bins = a->bins; j.bins_stride_b = a->bins_stride_b; j.bin_of = a->Y;
  j.ev_begin = a->ev_scan_begin; j.ev_end = a->ev_scan_end;
  rc = run_scan(j, false, &pl, &part, nullptr);
  if (rc != LLC_OK) return rc;
  fp.K = (int)a->L; fp.n_chunks = pl.n_chunks; fp.n_kgroups = pl.n_kgroups;
  fp.in = part;
  if (decode) {
    fp.cand = a->cand; fp.cand_stride_b = a->cand_stride_b;
    fp.side = a->side; fp.side_stride_b = a->side_stride_b;
    fp.source = a->source;
    fp.var_e = (double)a->var_w_given_a; fp.var_z = (double)a->var_t_given_a;
    fp.W = a->W; fp.A_hat = a->A_hat; fp.sq_err = a->sq_err;
  }
  fp.X = a->X; fp.Y = a->Y; fp.match_k = a->match_l; fp.accept = a->accept;
  fp.keyX = a->keyX; fp.keyY = nullptr;
  fp.y_given = 1; fp.bins = a->bins; fp.bins_stride_b = a->bins_stride_b; fp.message = a->message;
  fp.count_draft = 1; fp.count_pool = 0; fp.count_near = 1;
  fp.stats = a->stats;
  if (launch_finalize(st, fp) != hipSuccess) return LLC_E_LAUNCH;
  return LLC_OK;
}

int llc_couple_topm(const llc_couple_topm_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  if (a->B < 0 || a->B > 0x7FFFFFFFLL || a->K < 1 || a->K > 1024 || a->Md < 1 || a->Md > 65536 ||
      a->Mt < 1 || a->Mt > 65536)
    return LLC_E_SHAPE;
  if (a->B == 0) return LLC_OK;
  if (a->draft_ids == nullptr || a->draft_val == nullptr || a->target_ids == nullptr ||
      a->target_val == nullptr || a->X == nullptr || a->Y == nullptr || a->accept == nullptr)
    return LLC_E_NULL;
  if (a->draft_stride_b < 0 || a->draft_stride_k < 0 || a->target_stride_b < 0) return LLC_E_SHAPE;
  if (a->dtype != LLC_F32 && a->dtype != LLC_BF16) return LLC_E_DTYPE;
  if (a->kind != LLC_LOGITS && a->kind != LLC_PROBS && a->kind != LLC_LOGW) return LLC_E_DTYPE;
  if (a->kind == LLC_LOGITS) {
    if (!good_temp(a->temp_target)) return LLC_E_TEMP;
    if (a->temp_draft == nullptr && !good_temp(a->temp_draft_all)) return LLC_E_TEMP;
  }
  const size_t esize = a->dtype == LLC_F32 ? 4 : 2;
  if (((uintptr_t)a->draft_val % esize) != 0 || ((uintptr_t)a->target_val % esize) != 0 ||
      ((uintptr_t)a->draft_ids % 4) != 0 || ((uintptr_t)a->target_ids % 4) != 0)
    return LLC_E_ALIGN;
  TopmParams p;
  p.B = a->B; p.K = (int)a->K; p.Md = (int)a->Md; p.Mt = (int)a->Mt;
  p.dtype = a->dtype; p.kind = a->kind;
  p.draft_ids = a->draft_ids; p.draft_val = a->draft_val;
  p.draft_stride_b = a->draft_stride_b; p.draft_stride_k = a->draft_stride_k;
  p.target_ids = a->target_ids; p.target_val = a->target_val; p.target_stride_b = a->target_stride_b;
  p.temp_target = a->temp_target; p.temp_draft_all = a->temp_draft_all;
  p.temp_draft = a->kind == LLC_LOGITS ? a->temp_draft : nullptr;
  p.seed_lo = (unsigned)a->seed; p.seed_hi = (unsigned)(a->seed >> 32);
  p.row_offset = a->row_offset;
  p.X = a->X; p.Y = a->Y; p.match_k = a->match_k; p.accept = a->accept;
  p.keyX = a->keyX; p.keyY = a->keyY; p.stats = a->stats;
  hipStream_t st = (hipStream_t)a->stream;
  if (a->ev_begin != nullptr && hipEventRecord((hipEvent_t)a->ev_begin, st) != hipSuccess) return LLC_E_LAUNCH;
  if (launch_topm(st, p) != hipSuccess) return LLC_E_LAUNCH;
  if (a->ev_end != nullptr && hipEventRecord((hipEvent_t)a->ev_end, st) != hipSuccess) return LLC_E_LAUNCH;
  return LLC_OK;
}

// (one workgroup sorts a whole row, and its loops count entries in 32 bits with room to spare)
constexpr long long kLmlMaxV = 1LL << 28;

size_t llc_lml_workspace_size(int64_t B, int64_t V) {
  if (!shape_ok(B, 1, V) || V > kLmlMaxV) return 0;
  // per slot two buffers of sort keys (4 bytes) and two of mass pairs (8 bytes); a slot serves one
  // row per launch, and no more rows than kLmlSlots can be in work at once
  const long long slots = B < kLmlSlots ? B : kLmlSlots;
  return align256((size_t)slots * 24 * (size_t)V) + 256;
}

int llc_lml_bound(const llc_lml_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  if (!shape_ok(a->B, 1, a->V) || a->B > 0x7FFFFFFFLL || a->V > kLmlMaxV) return LLC_E_SHAPE;
  if (a->n_k < 1 || a->n_k > LLC_LML_MAX_K) return LLC_E_OPTION;
  for (int n = 0; n < a->n_k; ++n)
    if (a->k[n] < 1) return LLC_E_OPTION;
  if (a->B == 0) return LLC_OK;
  if (a->draft == nullptr || a->target == nullptr || a->bound == nullptr) return LLC_E_NULL;
  if (a->draft_stride_b < 0 || a->target_stride_b < 0) return LLC_E_SHAPE;
  if (a->dtype != LLC_F32 && a->dtype != LLC_BF16) return LLC_E_DTYPE;
  if (a->kind != LLC_LOGITS && a->kind != LLC_PROBS && a->kind != LLC_LOGW) return LLC_E_DTYPE;
  const bool logits = a->kind == LLC_LOGITS;
  if (logits && (!good_temp(a->temp_target) || !good_temp(a->temp_draft))) return LLC_E_TEMP;
  const size_t esize = a->dtype == LLC_F32 ? 4 : 2;
  if (((uintptr_t)a->draft % esize) != 0 || ((uintptr_t)a->target % esize) != 0) return LLC_E_ALIGN;
  // any workspace that holds at least one row will do (rows / slots launches follow each other);
  // the size llc_lml_workspace_size gives fills the GPU with each launch
  if (a->workspace == nullptr || ((uintptr_t)a->workspace & 255) != 0 ||
      a->workspace_bytes < (size_t)24 * (size_t)a->V)
    return LLC_E_WORKSPACE;
  LmlParams p;
  p.B = a->B; p.V = (int)a->V; p.dtype = a->dtype; p.probs = a->kind == LLC_PROBS ? 1 : 0;
  p.draft = a->draft; p.target = a->target;
  p.draft_stride_b = a->draft_stride_b; p.target_stride_b = a->target_stride_b;
  p.temp_draft = logits ? a->temp_draft : 1.0f;
  p.temp_target = logits ? a->temp_target : 1.0f;
  p.n_k = a->n_k;
  for (int n = 0; n < LLC_LML_MAX_K; ++n) p.k[n] = n < a->n_k ? a->k[n] : 1;
  p.bound = a->bound; p.relaxed = a->relaxed; p.tv = a->tv;
  p.work = (char *)a->workspace;
  {
    // a larger workspace than llc_lml_workspace_size asks for means fewer, larger launches
    const size_t slots = a->workspace_bytes / ((size_t)24 * (size_t)a->V);
    p.slots = (int)(slots < (size_t)a->B ? slots : (size_t)a->B);
  }
  hipStream_t st = (hipStream_t)a->stream;
  if (a->ev_begin != nullptr && hipEventRecord((hipEvent_t)a->ev_begin, st) != hipSuccess) return LLC_E_LAUNCH;
  if (launch_lml(st, p) != hipSuccess) return LLC_E_LAUNCH;
  if (a->ev_end != nullptr && hipEventRecord((hipEvent_t)a->ev_end, st) != hipSuccess) return LLC_E_LAUNCH;
  return LLC_OK;
}

size_t llc_verify_workspace_size(int64_t S, int64_t L, int64_t K, int64_t V) {
  if (S < 0 || L < 0 || L > (1 << 20) || K > 64) return 0;
  const long long B = S * (L + 1);
  // the one-shot scan over all S(L+1) rows, or (strong form) a later position's scan over S rows,
  // whichever needs more room in front of the verifier's own region
  const size_t all = llc_couple_workspace_size(B, K, V);
  const size_t one = llc_couple_workspace_size(S, K, V);
  if (all == 0 || one == 0) return 0;
  return (all > one ? all : one) + verify_extra(S, B, K).total;
}

int llc_verify(const llc_verify_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  if (a->S < 0 || a->L < 0 || a->L > (1 << 20) || a->K > 64) return LLC_E_SHAPE;
  const long long B = a->S * (a->L + 1);
  if (!shape_ok(B, a->K, a->V)) return LLC_E_SHAPE;
  if (a->S == 0) return LLC_OK;
  if (a->target == nullptr || a->Y == nullptr || a->n_out == nullptr) return LLC_E_NULL;
  if (a->L > 0 && a->tokens == nullptr) return LLC_E_NULL;
  if (a->kind != LLC_LOGITS && a->kind != LLC_LOGW) return LLC_E_DTYPE;
  if (a->stride_s < 0 || a->stride_j < 0 || a->stride_k < 0 || a->tok_stride_s < 0 ||
      a->tok_stride_j < 0 || a->row_stride_s < 0 || a->row_stride_j < 0)
    return LLC_E_SHAPE;

  ScanJob j;
  j.B = B; j.K = a->K; j.V = a->V; j.dtype = a->dtype; j.kind = a->kind;
  // the draft side of the scan is the reduction Algorithm 2 needs per (position, draft):
  // argmin_i S_i^(j,k) / q_i^(j,k); there is no pool over a common row
  j.draft = a->target; j.target = a->target;
  j.map.inner_count = a->L + 1;
  j.map.draft_outer = a->stride_s; j.map.draft_inner = a->stride_j;
  j.map.target_outer = a->stride_s; j.map.target_inner = a->stride_j;
  j.map.row_outer = a->row_stride_s; j.map.row_inner = a->row_stride_j;
  j.draft_stride_k = a->stride_k;
  j.temp_target = a->temp_target; j.temp_draft_all = a->temp_target; j.temp_draft = nullptr;
  j.seed = a->seed; j.row_offset = a->row_offset;
  j.no_pool = true;
  j.need_lse = true;  // keys of different rows are compared: they must be normalised
  j.force_perk = true;
  if (a->flags & ~(LLC_FLAG_EXACT_SCAN | LLC_FLAG_STRONG | LLC_FLAG_DRY_RUN | LLC_FLAG_MIN_FIRST)) return LLC_E_OPTION;
  j.min_first = (a->flags & LLC_FLAG_MIN_FIRST) != 0;
  const bool strong = (a->flags & LLC_FLAG_STRONG) != 0;
  const bool dry = (a->flags & LLC_FLAG_DRY_RUN) != 0;
  j.flags = a->flags & LLC_FLAG_EXACT_SCAN; j.v_chunks = a->v_chunks; j.k_tile = a->k_tile;
  j.stats = a->stats; j.workspace = a->workspace; j.workspace_bytes = a->workspace_bytes;
  j.stream = a->stream; j.ev_begin = a->ev_scan_begin; j.ev_end = a->ev_scan_end;
  const VerifyExtra ex = verify_extra(a->S, B, a->K);
  j.extra_bytes = ex.total;
  if (strong) j.lse_in_extra = ex.lse;  // the loop over positions reuses the workspace in front of it

  // Everything is planned before anything is launched, so that a refusal comes up front.  The
  // strong form's later positions are scans over the S sequences in the shared-proposal layout
  // (one row prices all K drafts' race times); they reuse the room in front of the verifier's own
  // region, which therefore starts behind the larger of the two layouts.
  ScanPlan plan_all;
  int rc = plan_scan(j, &plan_all);
  if (rc != LLC_OK) return rc;
  ScanJob q = j;  // one later position (the fields that differ between positions are set in the loop)
  ScanPlan plan_one;
  const size_t esize = a->dtype == LLC_F32 ? 4 : 2;
  if (strong && a->L > 0) {
    q.B = a->S;
    q.map = plain_rows(a->stride_s, a->stride_s);
    q.map.row_outer = a->row_stride_s;
    q.draft_stride_k = 0;
    q.force_perk = false;
    q.draft_row_off_unit = a->stride_k;   // the offsets are (first viable draft) * stride_k
    q.need_lse = false;                   // the rows' normalisers are known from the one-shot scan
    q.lse_in_extra = (size_t)-1;
    q.stats = nullptr; q.ev_begin = nullptr; q.ev_end = nullptr;
    q.extra_bytes = 0;
    q.draft = (const char *)a->target + (size_t)a->stride_j * esize;  // position 1 stands for all
    q.target = q.draft;
    // (positions differ by a multiple of stride_j: the alignment that position 1 shows must hold
    // for all of them, so the vector path also needs stride_j to be a multiple of 4)
    rc = plan_scan(q, &plan_one);
    if (rc != LLC_OK) return rc;
    if ((a->stride_j % 4) != 0) plan_one.vec = false;
    if (plan_one.lay.total > plan_all.lay.total) j.extra_at = plan_one.lay.total;
  }
  if (!workspace_ok(j, plan_all)) return LLC_E_WORKSPACE;
  if (dry) return LLC_OK;

  Plan pl = plan_all.pl;
  Partials part;
  char *extra = nullptr;
  rc = launch_scan_job(j, plan_all, &part, &extra);
  if (rc != LLC_OK) return rc;
  double *cand_key = (double *)(extra + ex.cand_key);
  double *cand_sec = (double *)(extra + ex.cand_sec);
  int32_t *cand = a->Yk != nullptr ? a->Yk : (int32_t *)(extra + ex.cand);

  hipStream_t st = (hipStream_t)a->stream;
  FinalizeParams fp;
  fp.cand = nullptr; fp.side = nullptr; fp.source = nullptr; fp.W = nullptr; fp.A_hat = nullptr; fp.sq_err = nullptr;
  fp.cand_stride_b = 0; fp.side_stride_b = 0; fp.var_e = 0.0; fp.var_z = 0.0;
  fp.B = B; fp.K = (int)a->K; fp.n_chunks = pl.n_chunks; fp.n_kgroups = pl.n_kgroups;
  fp.log_kind = 1;
  fp.in = part;
  fp.X = cand; fp.Y = nullptr; fp.match_k = nullptr; fp.accept = nullptr;
  fp.keyX = a->keyYk; fp.keyY = nullptr; fp.log_keyX = cand_key; fp.log_secX = cand_sec;
  fp.y_given = 0; fp.bins = nullptr; fp.bins_stride_b = 0; fp.message = nullptr;
  fp.count_draft = 1; fp.count_pool = 0; fp.count_near = 0;  // (near-ties: those of the loop's pools, counted there)
  fp.stats = a->stats;
  if (launch_finalize(st, fp) != hipSuccess) return LLC_E_LAUNCH;

  if (strong) {
    // Appendix B: position by position, because which drafts are dropped (and whose row prices
    // them) is only known once the position before is settled.  The dropped drafts of a position
    // all take the first viable draft's row: one scan in the shared-proposal layout per position
    // over the S sequences, skipped by the kernels for sequences that have nothing to price, and
    // one step kernel, which also merges that scan's chunks: two launches per position.
    StrongStepParams ss;
    ss.S = a->S; ss.L = (int)a->L; ss.K = (int)a->K;
    ss.cand = cand; ss.cand_key = cand_key; ss.cand_sec = cand_sec;
    ss.part_key = nullptr; ss.part_idx = nullptr; ss.part_sec = nullptr; ss.n_chunks = 0;
    ss.stats = a->stats;
    ss.tau_all = (int32_t *)(extra + ex.tau_all);
    ss.tokens = a->tokens; ss.tok_stride_s = a->tok_stride_s; ss.tok_stride_j = a->tok_stride_j;
    ss.stride_k = a->stride_k;
    ss.viable = (uint8_t *)(extra + ex.viable); ss.running = (int32_t *)(extra + ex.running);
    ss.next_off = (long long *)(extra + ex.next_off);
    ss.lse = (const double *)(extra + ex.lse); ss.lse_sel = (double *)(extra + ex.lse_sel);
    ss.Y = a->Y; ss.n_out = a->n_out; ss.active = a->active; ss.keyY = a->keyY;
    // the first scan's partials are spent: the later positions' scans take the room in front of
    // the verifier's region (checked above to hold either layout)
    q.workspace_bytes = (size_t)(extra - (char *)a->workspace);
    q.draft_row_off = ss.next_off;
    for (long long pos = 0; pos <= a->L; ++pos) {
      if (pos > 0) {
        q.draft = (const char *)a->target + (size_t)(pos * a->stride_j) * esize;
        q.target = q.draft;
        q.row_offset = a->row_offset + (uint64_t)(pos * a->row_stride_j);
        q.tau_ready = ss.tau_all + (pos - 1) * a->S * (a->K + 1);
        Partials part2;
        const int rc2 = launch_scan_job(q, plan_one, &part2, nullptr);
        if (rc2 != LLC_OK) return rc2;
        ss.part_key = part2.keyX; ss.part_idx = part2.idxX; ss.part_sec = part2.secX;
        ss.n_chunks = plan_one.pl.n_chunks;
      }
      ss.j = (int)pos;
      if (launch_strong_step(st, ss) != hipSuccess) return LLC_E_LAUNCH;
    }
    return LLC_OK;
  }

  VerifyParams vp;
  vp.S = a->S; vp.L = (int)a->L; vp.K = (int)a->K;
  vp.cand = cand; vp.cand_key = cand_key; vp.cand_sec = cand_sec;
  vp.stats = a->stats;
  vp.tokens = a->tokens; vp.tok_stride_s = a->tok_stride_s; vp.tok_stride_j = a->tok_stride_j;
  vp.Y = a->Y; vp.n_out = a->n_out; vp.active = a->active; vp.keyY = a->keyY;
  if (launch_verify(st, vp) != hipSuccess) return LLC_E_LAUNCH;
  return LLC_OK;
}

int llc_couple_is(const llc_couple_is_args *a) {
  if (a == nullptr) return LLC_E_NULL;
  llc_couple_args c;
  std::memset(&c, 0, sizeof(c));
  c.B = a->B; c.K = a->L; c.V = a->N;
  c.dtype = LLC_F32; c.kind = LLC_LOGW;
  c.draft = a->logw_dec; c.draft_stride_b = a->dec_stride_b; c.draft_stride_k = a->dec_stride_l;
  c.target = a->logw_enc; c.target_stride_b = a->enc_stride_b;
  c.temp_target = 1.0f; c.temp_draft_all = 1.0f; c.temp_draft = nullptr;
  c.seed = a->seed; c.row_offset = a->row_offset;
  c.X = a->X; c.Y = a->Y; c.accept = a->accept; c.match_k = a->match_l;
  c.keyX = a->keyX; c.keyY = a->keyY; c.stats = a->stats;
  c.workspace = a->workspace; c.workspace_bytes = a->workspace_bytes; c.stream = a->stream;
  c.flags = a->flags; c.v_chunks = a->v_chunks; c.k_tile = a->k_tile;
  c.ev_scan_begin = a->ev_scan_begin; c.ev_scan_end = a->ev_scan_end;
  return llc_couple(&c);
}

}  // extern "C"
