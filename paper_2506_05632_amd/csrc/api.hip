// C ABI of libllc_hip.so: argument checks, launch planning, kernel launches.
#include <cmath>
#include <cstring>

#include "common.hpp"

namespace llc {
namespace {

constexpr int kMaxChunks = 4096;
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
  if (K >= 8 && shared) return 8;
  return K >= 3 ? 4 : K == 2 ? 2 : 1;
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
  size_t keyX, idxX, keyY, idxY, kY, lse, total;
};

Layout layout_for(long long B, long long K, long long n_kgroups, long long n_chunks) {
  Layout l;
  size_t off = 0;
  l.keyX = off; off += align256((size_t)(B * K * n_chunks) * sizeof(double));
  l.idxX = off; off += align256((size_t)(B * K * n_chunks) * sizeof(int32_t));
  l.keyY = off; off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(double));
  l.idxY = off; off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(int32_t));
  l.kY = off;   off += align256((size_t)(B * n_kgroups * n_chunks) * sizeof(int32_t));
  l.lse = off;  off += align256((size_t)(B * (K + 1)) * sizeof(double));
  l.total = off;
  return l;
}

bool shape_ok(long long B, long long K, long long V) {
  return B >= 0 && K >= 1 && K <= 65535 && V >= 1 && V < 2147483644LL &&
         B <= (1LL << 40);
}

bool good_temp(float t) { return std::isfinite(t) && t > 0.0f; }

}  // namespace
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
    case LLC_E_OPTION: return "v_chunks, k_tile or flags out of range";
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
  if (!shape_ok(a->B, a->K, a->V)) return LLC_E_SHAPE;
  if (a->B == 0) return LLC_OK;  // nothing to read or write: pointers may be NULL
  if (a->draft == nullptr || a->target == nullptr || a->X == nullptr || a->Y == nullptr ||
      a->accept == nullptr)
    return LLC_E_NULL;
  if (a->dtype != LLC_F32 && a->dtype != LLC_BF16) return LLC_E_DTYPE;
  if (a->kind != LLC_LOGITS && a->kind != LLC_PROBS && a->kind != LLC_LOGW) return LLC_E_DTYPE;
  if (a->draft_stride_b < 0 || a->draft_stride_k < 0 || a->target_stride_b < 0) return LLC_E_SHAPE;
  if (a->flags & ~LLC_FLAG_EXACT_SCAN) return LLC_E_OPTION;
  if (a->v_chunks < 0 || a->v_chunks > kMaxChunks) return LLC_E_OPTION;
  if (a->k_tile != 0 && a->k_tile != 1 && a->k_tile != 2 && a->k_tile != 4 && a->k_tile != 8)
    return LLC_E_OPTION;
  if (a->kind == LLC_LOGITS) {
    if (!good_temp(a->temp_target)) return LLC_E_TEMP;
    if (a->temp_draft == nullptr && !good_temp(a->temp_draft_all)) return LLC_E_TEMP;
  }
  const size_t esize = a->dtype == LLC_F32 ? 4 : 2;
  if (((uintptr_t)a->draft % esize) != 0 || ((uintptr_t)a->target % esize) != 0) return LLC_E_ALIGN;

  const bool logits = a->kind == LLC_LOGITS;
  const float *temp_draft = logits ? a->temp_draft : nullptr;
  const bool shared = a->draft_stride_k == 0 && temp_draft == nullptr;

  Plan pl;
  pl.kt = a->k_tile != 0 ? a->k_tile : auto_ktile(a->K, shared);
  pl.n_kgroups = (int)((a->K + pl.kt - 1) / pl.kt);
  const long long G = (a->V + 3) / 4;
  plan_chunks(G, a->v_chunks != 0 ? a->v_chunks : auto_chunks(a->B, pl.n_kgroups, G), &pl.n_chunks,
              &pl.groups_per_chunk);
  const long long blocks = a->B * pl.n_kgroups * pl.n_chunks;
  if (blocks > 0x7FFFFFFFLL) return LLC_E_SHAPE;

  const Layout lay = layout_for(a->B, a->K, pl.n_kgroups, pl.n_chunks);
  if (a->workspace == nullptr || ((uintptr_t)a->workspace & 255) != 0 ||
      a->workspace_bytes < lay.total)
    return LLC_E_WORKSPACE;
  char *ws = (char *)a->workspace;

  // vector loads need every row to start on a 4-element boundary of a 16-byte (fp32) or
  // 8-byte (bf16) aligned base
  const size_t vbytes = 4 * esize;
  const bool vec = ((uintptr_t)a->draft % vbytes) == 0 && ((uintptr_t)a->target % vbytes) == 0 &&
                   (a->draft_stride_b % 4) == 0 && (a->draft_stride_k % 4) == 0 &&
                   (a->target_stride_b % 4) == 0;

  hipStream_t st = (hipStream_t)a->stream;
  const bool want_keys = a->keyX != nullptr || a->keyY != nullptr;
  const bool log_kind = a->kind != LLC_PROBS;

  Partials part;
  part.keyX = (double *)(ws + lay.keyX);
  part.idxX = (int32_t *)(ws + lay.idxX);
  part.keyY = (double *)(ws + lay.keyY);
  part.idxY = (int32_t *)(ws + lay.idxY);
  part.kY = (int32_t *)(ws + lay.kY);
  part.lse = (double *)(ws + lay.lse);

  if (want_keys && log_kind) {
    LseParams lp;
    lp.draft = a->draft; lp.target = a->target;
    lp.draft_stride_b = a->draft_stride_b; lp.draft_stride_k = a->draft_stride_k;
    lp.target_stride_b = a->target_stride_b;
    lp.B = a->B; lp.K = (int)a->K; lp.V = (int)a->V; lp.dtype = a->dtype;
    lp.temp_target = logits ? a->temp_target : 1.0f;
    lp.temp_draft_all = logits ? a->temp_draft_all : 1.0f;
    lp.temp_draft = temp_draft;
    lp.is_logits = logits ? 1 : 0;
    lp.lse = part.lse;
    if (launch_lse(st, lp) != hipSuccess) return LLC_E_LAUNCH;
  }

  ScanParams sp;
  sp.draft = a->draft; sp.target = a->target;
  sp.draft_stride_b = a->draft_stride_b; sp.draft_stride_k = a->draft_stride_k;
  sp.target_stride_b = a->target_stride_b;
  sp.B = a->B; sp.K = (int)a->K; sp.V = (int)a->V;
  sp.n_chunks = pl.n_chunks; sp.groups_per_chunk = pl.groups_per_chunk; sp.n_kgroups = pl.n_kgroups;
  sp.seed_lo = (unsigned)a->seed; sp.seed_hi = (unsigned)(a->seed >> 32);
  sp.row_offset = a->row_offset;
  sp.temp_target = logits ? a->temp_target : 1.0f;
  sp.temp_draft_all = logits ? a->temp_draft_all : 1.0f;
  sp.temp_draft = temp_draft;
  sp.vector_loads = vec ? 1 : 0;
  sp.force_exact = (a->flags & LLC_FLAG_EXACT_SCAN) ? 1 : 0;
  sp.out = part;
  sp.stats = a->stats;

  const bool probs = a->kind == LLC_PROBS;
  if (a->ev_scan_begin != nullptr && hipEventRecord((hipEvent_t)a->ev_scan_begin, st) != hipSuccess)
    return LLC_E_LAUNCH;
  hipError_t e;
  if (a->dtype == LLC_F32)
    e = shared ? launch_scan_f32_shared(pl.kt, probs, (unsigned)blocks, st, sp)
               : launch_scan_f32_perk(pl.kt, probs, (unsigned)blocks, st, sp);
  else
    e = shared ? launch_scan_bf16_shared(pl.kt, probs, (unsigned)blocks, st, sp)
               : launch_scan_bf16_perk(pl.kt, probs, (unsigned)blocks, st, sp);
  if (e != hipSuccess) return LLC_E_LAUNCH;
  if (a->ev_scan_end != nullptr && hipEventRecord((hipEvent_t)a->ev_scan_end, st) != hipSuccess)
    return LLC_E_LAUNCH;

  FinalizeParams fp;
  fp.B = a->B; fp.K = (int)a->K; fp.n_chunks = pl.n_chunks; fp.n_kgroups = pl.n_kgroups;
  fp.log_kind = log_kind ? 1 : 0;
  fp.in = part;
  fp.X = a->X; fp.Y = a->Y; fp.match_k = a->match_k; fp.accept = a->accept;
  fp.keyX = a->keyX; fp.keyY = a->keyY;
  fp.stats = a->stats;
  if (launch_finalize(st, fp) != hipSuccess) return LLC_E_LAUNCH;
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
