// Host side of the Orth-Dion C ABI: argument checks, shape classes, workspace planning and
// the kernel sequence of one step.  No device memory is allocated here; everything lives
// in the caller's workspace.
#include "../../include/orthdion.h"

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "od_kernels.h"
#include "od_internal.h"

namespace {

using od::ClassDims;
using od::MatPtrs;
using od::WsArr;
using od::HalfArr;

constexpr size_t kAlign = 256;
// Two groups by default between these numbers of matrix elements.  A set below is a chain of
// short launches, where the fork and join of the second stream cost more than the overlap
// returns.  A set above comes in launch batches of many matrices, whose kernels fill the chip
// by themselves: side by side they mostly compete (measured on 96 matrices of rank 512: 2 to 4 %
// less time per step, and no kernel's time stamps mean anything any more), whereas a few matrices
// of large rank gain 13 %: there the Cholesky chains and the one-matrix launches leave room.
constexpr double kGroupMinElements = 64.0 * 1024 * 1024;
constexpr double kGroupMaxElements = 512.0 * 1024 * 1024;

size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }

// A batch: up to kMaxBatchHost matrices of identical shape and leading dimensions.
struct Batch {
  ClassDims d;
  std::vector<int> members;          // indices into the caller's arrays
  // per-matrix float arrays (offset of matrix 0 in bytes, stride in elements)
  size_t off_pa, off_pb, off_ra, off_rb, off_part, off_gram, off_tp1, off_tp2, off_tq1, off_tq2, off_w,
      off_tmp, off_colsq;
  size_t off_ph, off_pht, off_rh, off_qh, off_qht;   // pre-scaled fp16 copies of the factors (uint16 arrays)
  int64_t st_p, st_r, st_part, st_rr, st_colsq;
  int splits_proj, splits_back, splits_gram_p, splits_gram_q, slabs;
  int slot_base;                     // first row of this batch in the scal / info tables
  int rank_class;
};

// All batches of one rank r.  The r x r work of the orthogonalisations (Cholesky factor and
// inverse) does not depend on m and n, so it is launched once per rank class over all of its
// matrices: the class owns the r x r arrays, every batch a contiguous range of slices.
struct RankClass {
  int r, count, slot_base;
  int group;                         // which of the two groups a large set of one rank is dealt into
  int64_t st_rr;
  std::vector<int> batches;
  size_t off_gram, off_tp1, off_tp2, off_tq1, off_tq2, off_w, off_tmp;
};

int pick_splits(int64_t tiles, int nb, int64_t k, int kt_min) {
  int64_t want = (512 + tiles * nb - 1) / (tiles * nb);
  int64_t cap = k / kt_min;
  if (cap < 1) cap = 1;
  if (want > cap) want = cap;
  if (want > 32) want = 32;
  if (want < 1) want = 1;
  return (int)want;
}

// Splits for a kernel whose workgroups run in rounds of `slots` (256 CUs times the workgroups
// that fit one CU).  A workgroup's time is proportional to 1 / splits, so rounds / splits
// measures the launch; the fewest splits (least partial-sum traffic) within 15 % of the best
// are taken.
int pick_splits_by_rounds(int64_t tiles, int nb, int64_t k, int kt_min, int64_t slots) {
  int64_t cap = k / kt_min;
  if (cap < 1) cap = 1;
  if (cap > 32) cap = 32;
  auto cost = [&](int s) { return (double)((tiles * nb * s + slots - 1) / slots) / (double)s; };
  double best = cost(1);
  for (int s = 2; s <= (int)cap; ++s) best = cost(s) < best ? cost(s) : best;
  for (int s = 1; s <= (int)cap; ++s)
    if (cost(s) <= 1.15 * best) return s;
  return 1;
}

}  // namespace

struct orthdion_ctx {
  std::vector<orthdion_matdesc> mats;
  orthdion_config cfg;
  std::vector<Batch> batches;
  std::vector<RankClass> classes;
  std::vector<int> batch_of, slot_of;     // per matrix
  size_t off_scal, off_info, off_diag, off_dacc, off_dpart, ws_bytes;
  void* last_ws;
  bool diag_on = false, diag_valid = false;
  // optional phase timing with HIP events (host resources only)
  bool prof_on = false;
  unsigned prof_mask = 0;
  int prof_max_steps = 0, prof_steps = 0;
  std::vector<hipEvent_t> prof_events;    // [step][batch][phase][begin/end]
  std::vector<char> prof_recorded;        // [step][batch][phase]: an interval was recorded
  // a second stream for the guard of the second CholeskyQR pass (ranks above 256): its launch
  // chain returns at once for every well-conditioned matrix, and beside the main stream those
  // empty launches cost nothing (host resources; made at the first step that is not being captured)
  hipStream_t side = nullptr;
  hipEvent_t ev_fork = nullptr, ev_join = nullptr;
  bool side_tried = false;
  // Two groups: the batches are dealt to two sets of about equal work, each with rank classes
  // of its own, and the two sets run side by side on the caller's stream and on `group_stream`
  // (see orthdion_step_impl).
  bool two_groups = false;
  hipStream_t group_stream = nullptr;
  hipEvent_t ev_group_fork = nullptr, ev_group_join = nullptr;
};

static bool ensure_side_stream(orthdion_ctx* h, hipStream_t st) {
  if (h->side) return true;
  if (h->side_tried) return false;
  hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
  if (hipStreamIsCapturing(st, &cs) != hipSuccess) { (void)hipGetLastError(); return false; }
  if (cs != hipStreamCaptureStatusNone) return false;        // nothing is created under capture; a later call may
  h->side_tried = true;
  if (hipStreamCreateWithFlags(&h->side, hipStreamNonBlocking) != hipSuccess) { h->side = nullptr; (void)hipGetLastError(); return false; }
  bool ok = hipStreamCreateWithFlags(&h->group_stream, hipStreamNonBlocking) == hipSuccess;
  if (!ok) h->group_stream = nullptr;
  hipEvent_t* const events[4] = {&h->ev_fork, &h->ev_join, &h->ev_group_fork, &h->ev_group_join};
  for (hipEvent_t* e : events) ok = ok && hipEventCreateWithFlags(e, hipEventDisableTiming) == hipSuccess;
  if (!ok) {
    for (hipEvent_t* e : events) {
      if (*e) (void)hipEventDestroy(*e);
      *e = nullptr;
    }
    if (h->group_stream) (void)hipStreamDestroy(h->group_stream);
    (void)hipStreamDestroy(h->side);
    h->side = nullptr; h->group_stream = nullptr;
    (void)hipGetLastError();
    return false;
  }
  return true;
}

static hipEvent_t* prof_slot(orthdion_ctx* h, int batch, int phase, int end) {
  if (!h->prof_on || h->prof_steps >= h->prof_max_steps || !(h->prof_mask & (1u << phase))) return nullptr;
  size_t nb = h->batches.size();
  size_t idx = (((size_t)h->prof_steps * nb + (size_t)batch) * ORTHDION_NPHASE + (size_t)phase) * 2 + (size_t)end;
  if (end) h->prof_recorded[idx / 2] = 1;
  return &h->prof_events[idx];
}

static od::Prec resolve_prec(const orthdion_config& c) {
  if (c.precision == ORTHDION_PREC_FAST) return od::PREC_F16;
  if (c.precision == ORTHDION_PREC_EXACT) return od::PREC_BF3;
  return (c.x_dtype == ORTHDION_BF16 && c.g_dtype == ORTHDION_BF16) ? od::PREC_F16 : od::PREC_BF3;
}

static int check_config(const orthdion_config* c) {
  if (c->x_dtype != ORTHDION_F32 && c->x_dtype != ORTHDION_BF16) return ORTHDION_E_INVALID_ARG;
  if (c->g_dtype != ORTHDION_F32 && c->g_dtype != ORTHDION_BF16) return ORTHDION_E_INVALID_ARG;
  if (c->variant != ORTHDION_QR && c->variant != ORTHDION_COLNORM) return ORTHDION_E_INVALID_ARG;
  if (c->ef != ORTHDION_EF_DION && c->ef != ORTHDION_EF_PAPER && c->ef != ORTHDION_EF_POLYAK) return ORTHDION_E_INVALID_ARG;
  if (c->precision != ORTHDION_PREC_AUTO && c->precision != ORTHDION_PREC_FAST && c->precision != ORTHDION_PREC_EXACT)
    return ORTHDION_E_INVALID_ARG;
  if (!std::isfinite(c->mu) || c->mu < 0.f || c->mu > 1.f) return ORTHDION_E_INVALID_ARG;
  if (!std::isfinite(c->lr)) return ORTHDION_E_INVALID_ARG;
  if (c->groups < 0 || c->groups > 2) return ORTHDION_E_INVALID_ARG;
  return ORTHDION_OK;
}

static int check_shape(const orthdion_matdesc& m) {
  if (m.m < 8 || m.n < 8 || m.r < 8) return ORTHDION_E_BAD_SHAPE;
  if (m.m % 8 || m.n % 8 || m.r % 8) return ORTHDION_E_BAD_SHAPE;
  if (m.m >= (1 << 24) || m.n >= (1 << 24)) return ORTHDION_E_BAD_SHAPE;
  if (m.r > m.m || m.r > m.n) return ORTHDION_E_BAD_SHAPE;
  if (m.ldx < m.n || m.ldg < m.n || m.ldm < m.n) return ORTHDION_E_BAD_SHAPE;
  if (m.ldx % 8 || m.ldg % 8 || m.ldm % 8) return ORTHDION_E_BAD_SHAPE;
  return ORTHDION_OK;
}

// Nothing may throw across the C boundary: the entry points that allocate host memory run their
// bodies through this.
template <class F>
static int no_throw(F&& body) {
  try {
    return body();
  } catch (const std::bad_alloc&) {
    return ORTHDION_E_NO_MEMORY;
  } catch (...) {
    return ORTHDION_E_INVALID_ARG;
  }
}

static int create_impl(orthdion_handle* out, const orthdion_matdesc* mats, int32_t nmat, const orthdion_config* cfg);

extern "C" int orthdion_create(orthdion_handle* out, const orthdion_matdesc* mats, int32_t nmat,
                               const orthdion_config* cfg) {
  if (!out) return ORTHDION_E_NULL_PTR;
  *out = nullptr;
  orthdion_handle h = nullptr;
  const int rc = no_throw([&] { return create_impl(&h, mats, nmat, cfg); });
  if (rc != ORTHDION_OK) {
    delete h;
    return rc;
  }
  *out = h;
  return ORTHDION_OK;
}

static int create_impl(orthdion_handle* out, const orthdion_matdesc* mats, int32_t nmat, const orthdion_config* cfg) {
  if (!mats || !cfg) return ORTHDION_E_NULL_PTR;
  if (nmat < 1 || nmat > (1 << 20)) return ORTHDION_E_INVALID_ARG;
  int rc = check_config(cfg);
  if (rc != ORTHDION_OK) return rc;
  for (int i = 0; i < nmat; ++i)
    if ((rc = check_shape(mats[i])) != ORTHDION_OK) return rc;

  orthdion_ctx* h = new (std::nothrow) orthdion_ctx();
  if (!h) return ORTHDION_E_NO_MEMORY;
  *out = h;                        // the caller frees it if anything below fails or throws
  h->mats.assign(mats, mats + nmat);
  h->cfg = *cfg;
  h->last_ws = nullptr;
  h->batch_of.assign(nmat, -1);
  h->slot_of.assign(nmat, -1);

  // shape classes, in order of first appearance, cut into batches
  auto same_shape = [](const ClassDims& d, const orthdion_matdesc& a) {
    return d.m == a.m && d.n == a.n && d.r == a.r && d.ldx == a.ldx && d.ldg == a.ldg && d.ldm == a.ldm;
  };
  double total_elems = 0.0;
  for (int i = 0; i < nmat; ++i) total_elems += (double)mats[i].m * (double)mats[i].n;
  int groups = cfg->groups;
  if (groups == 0) groups = (nmat >= 2 && total_elems >= kGroupMinElements && total_elems < kGroupMaxElements) ? 2 : 1;
  for (int i = 0; i < nmat; ++i) {
    const orthdion_matdesc& a = mats[i];
    int found = -1;
    for (size_t b = 0; b < h->batches.size(); ++b) {
      if (same_shape(h->batches[b].d, a) && (int)h->batches[b].members.size() < od::kMaxBatchHost) found = (int)b;
    }
    if (found < 0) {
      Batch nb = {};
      nb.d.m = (int)a.m; nb.d.n = (int)a.n; nb.d.r = a.r;
      nb.d.ldx = a.ldx; nb.d.ldg = a.ldg; nb.d.ldm = a.ldm;
      nb.d.x_bf16 = cfg->x_dtype == ORTHDION_BF16;
      nb.d.g_bf16 = cfg->g_dtype == ORTHDION_BF16;
      h->batches.push_back(nb);
      found = (int)h->batches.size() - 1;
    }
    h->batch_of[i] = found;
    h->slot_of[i] = (int)h->batches[found].members.size();
    h->batches[found].members.push_back(i);
  }

  // workspace plan
  size_t off = 0;
  h->off_scal = off; off = align_up(off + (size_t)nmat * od::kScalPerMat * sizeof(float));
  h->off_info = off; off = align_up(off + (size_t)nmat * od::kInfoPerMat * sizeof(int));
  h->off_diag = off; off = align_up(off + (size_t)nmat * od::kDiagPerMat * sizeof(float));
  h->off_dacc = off; off = align_up(off + (size_t)nmat * od::kDaccPerMat * sizeof(double));
  h->off_dpart = off; off = align_up(off + (size_t)nmat * od::kDiagBlocks * 4 * sizeof(double));
  // Groups: the heaviest batch first, each to the group with less work so far (m n per matrix
  // measures a batch's step).  A set with a single batch stays one group.
  std::vector<int> group_of(h->batches.size(), 0);
  for (Batch& b : h->batches) b.d.nb = (int)b.members.size();
  if (groups == 2 && h->batches.size() >= 2) {
    std::vector<int> order(h->batches.size());
    for (size_t k = 0; k < order.size(); ++k) order[k] = (int)k;
    auto weight = [&](int k) { const ClassDims& d = h->batches[k].d; return (double)d.m * d.n * d.nb; };
    std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return weight(x) > weight(y); });
    double load[2] = {0.0, 0.0};
    for (int k : order) {
      const int g = load[1] < load[0] ? 1 : 0;
      group_of[k] = g;
      load[g] += weight(k);
    }
    h->two_groups = true;
  }
  // rank classes in order of first appearance (one per rank and group); table rows (slots) run
  // class by class
  for (size_t bi = 0; bi < h->batches.size(); ++bi) {
    Batch& b = h->batches[bi];
    int found = -1;
    for (size_t c = 0; c < h->classes.size(); ++c)
      if (h->classes[c].r == b.d.r && h->classes[c].group == group_of[bi]) found = (int)c;
    if (found < 0) {
      RankClass rc = {};
      rc.r = b.d.r;
      rc.group = group_of[bi];
      rc.st_rr = ((int64_t)b.d.r * b.d.r + 63) / 64 * 64;
      h->classes.push_back(rc);
      found = (int)h->classes.size() - 1;
    }
    b.rank_class = found;
    h->classes[found].batches.push_back((int)bi);
    h->classes[found].count += b.d.nb;
  }
  int slot_base = 0;
  for (RankClass& c : h->classes) {
    c.slot_base = slot_base;
    for (int bi : c.batches) {
      h->batches[bi].slot_base = slot_base;
      slot_base += h->batches[bi].d.nb;
    }
    auto take_rr = [&]() { size_t o = off; off = align_up(off + (size_t)c.st_rr * c.count * sizeof(float)); return o; };
    c.off_gram = take_rr(); c.off_tp1 = take_rr(); c.off_tp2 = take_rr(); c.off_tq1 = take_rr(); c.off_tq2 = take_rr();
    c.off_w = take_rr(); c.off_tmp = take_rr();
  }
  for (Batch& b : h->batches) {
    ClassDims& d = b.d;
    const RankClass& rcl = h->classes[b.rank_class];
    const int64_t m = d.m, n = d.n, r = d.r;
    const int nt = r <= 64 ? 64 : (r <= 128 ? 128 : 256);
    const int64_t tiles_r = (r + nt - 1) / nt;
    // the projection's fast-precision kernel for r > 128 works on 64-row panels: as many
    // workgroups from half the splits, hence half the partial sums to write and add up
    const int proj_rows = (resolve_prec(*cfg) == od::PREC_F16 && od::proj_uses_flat_tiles((int)m, (int)r, d.nb)) ? 64 : 128;
    b.splits_proj = pick_splits(((m + proj_rows - 1) / proj_rows) * tiles_r, d.nb, n, 128);
    b.splits_back = pick_splits(((n + 127) / 128) * tiles_r, d.nb, m, 128);
    if (resolve_prec(*cfg) == od::PREC_F16 && od::stream_kernel_eligible(d)) {
      // one 8-wave workgroup per CU and 128 x 256 / 512 tiles
      const int64_t tiles_c = (r + od::stream_tile_cols((int)r) - 1) / od::stream_tile_cols((int)r);
      b.splits_proj = pick_splits_by_rounds(((m + 127) / 128) * tiles_c, d.nb, n, 256, 256);
      b.splits_back = pick_splits_by_rounds(((n + 127) / 128) * tiles_c, d.nb, m, 256, 256);
    }
    // Gram tiles on and above the diagonal (the ones that are computed)
    const int64_t gt1 = (r + 127) / 128;
    const int64_t gt = gt1 * (gt1 + 1) / 2;
    if (r <= 32) {
      // one 32 x 32 tile, one thread per row: 256-row slabs (k_small_gram, k_small_first_pass)
      b.splits_gram_p = pick_splits(1, d.nb, m, 256);
      b.splits_gram_q = pick_splits(1, d.nb, n, 256);
    } else {
      // two workgroups of the Gram kernel fit one CU
      b.splits_gram_p = pick_splits_by_rounds(gt, d.nb, m, 256, 512);
      b.splits_gram_q = pick_splits_by_rounds(gt, d.nb, n, 256, 512);
    }
    if (b.splits_gram_p > 32) b.splits_gram_p = 32;
    if (b.splits_gram_q > 32) b.splits_gram_q = 32;
    b.slabs = (int)((n + 31) / 32);           // row slabs of the column-norm kernels: many, so the grid fills the chip
    if (b.slabs > 256) b.slabs = 256;
    int64_t part = (int64_t)b.splits_proj * m * r;
    if ((int64_t)b.splits_back * n * r > part) part = (int64_t)b.splits_back * n * r;
    if ((int64_t)b.splits_gram_p * r * r > part) part = (int64_t)b.splits_gram_p * r * r;
    if ((int64_t)b.splits_gram_q * r * r > part) part = (int64_t)b.splits_gram_q * r * r;
    // r <= 32: the Gram partials of both CholeskyQR passes live side by side
    if (r <= 32) {
      const int64_t sg = b.splits_gram_p > b.splits_gram_q ? b.splits_gram_p : b.splits_gram_q;
      if (2 * sg * r * r > part) part = 2 * sg * r * r;
    }
    if ((int64_t)b.slabs * r > part) part = (int64_t)b.slabs * r;
    // strides rounded so that every matrix slice stays 256-byte aligned
    auto rnd = [](int64_t e) { return (e + 63) / 64 * 64; };
    b.st_p = rnd(m * r); b.st_r = rnd(n * r); b.st_part = rnd(part); b.st_rr = rnd(r * r); b.st_colsq = rnd(r);
    auto take = [&](int64_t stride) { size_t o = off; off = align_up(off + (size_t)stride * d.nb * sizeof(float)); return o; };
    b.off_pa = take(b.st_p); b.off_pb = take(b.st_p);
    b.off_ra = take(b.st_r); b.off_rb = take(b.st_r);
    b.off_part = take(b.st_part);
    // this batch's slices of the class-owned r x r arrays
    const size_t in_class = (size_t)(b.slot_base - rcl.slot_base) * (size_t)rcl.st_rr * sizeof(float);
    b.off_gram = rcl.off_gram + in_class;
    b.off_tp1 = rcl.off_tp1 + in_class; b.off_tp2 = rcl.off_tp2 + in_class;
    b.off_tq1 = rcl.off_tq1 + in_class; b.off_tq2 = rcl.off_tq2 + in_class;
    b.off_w = rcl.off_w + in_class; b.off_tmp = rcl.off_tmp + in_class;
    b.off_colsq = take(b.st_colsq);
    auto take_h = [&](int64_t stride) { size_t o = off; off = align_up(off + (size_t)stride * d.nb * sizeof(uint16_t)); return o; };
    b.off_ph = take_h(b.st_p); b.off_pht = take_h(b.st_p);
    b.off_rh = take_h(b.st_r); b.off_qh = take_h(b.st_r); b.off_qht = take_h(b.st_r);
  }
  h->ws_bytes = off;
  return ORTHDION_OK;
}

extern "C" size_t orthdion_workspace_bytes(orthdion_handle h) { return h ? h->ws_bytes : 0; }

extern "C" int32_t orthdion_get_groups(orthdion_handle h) { return h ? (h->two_groups ? 2 : 1) : 0; }

extern "C" int orthdion_set_lr(orthdion_handle h, float lr) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (!std::isfinite(lr)) return ORTHDION_E_INVALID_ARG;
  h->cfg.lr = lr;
  return ORTHDION_OK;
}

extern "C" int orthdion_set_mu(orthdion_handle h, float mu) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (!std::isfinite(mu) || mu < 0.f || mu > 1.f) return ORTHDION_E_INVALID_ARG;
  h->cfg.mu = mu;
  return ORTHDION_OK;
}

extern "C" int orthdion_set_variant(orthdion_handle h, orthdion_variant v) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (v != ORTHDION_QR && v != ORTHDION_COLNORM) return ORTHDION_E_INVALID_ARG;
  h->cfg.variant = v;
  return ORTHDION_OK;
}

#define OD_TRY(expr)                                  \
  do {                                                \
    if ((expr) != hipSuccess) return ORTHDION_E_HIP;  \
  } while (0)

// orth() of `a0` (rows x r) by CholeskyQR2 comes in pieces, so that the two r x r stages in the
// middle (which do not depend on rows) can be launched once for every matrix of a rank:
//   orth_gram : Gram matrix of a0, reduced into this batch's slices of the class array
//   class_cholinv over the rank class : T1, W1
//   orth_second_pass, class_guard, orth_result : see below.
static int orth_gram(const Batch& b, char* ws, int rows, size_t off_a0, int64_t st_a, int splits, bool fast, int side,
                     const float* scal, hipStream_t st) {
  // fast precision has the sampled scale of B at hand: two-term fp16 operands (half the
  // matrix-core work of the three-way bf16 split at 22 instead of 24 bits)
  const int mode = fast ? od::kGramH2 : od::kGramBF3;
  WsArr a0{reinterpret_cast<float*>(ws + off_a0), st_a};
  WsArr part{reinterpret_cast<float*>(ws + b.off_part), b.st_part};
  WsArr gram{reinterpret_cast<float*>(ws + b.off_gram), b.st_rr};
  // one 32 x 32 tile: partial sums in plain fp32, left in the first half of `part` for the
  // kernel that factors them (its own partials go to the second half)
  if (b.d.r <= 32) {
    OD_TRY(od::launch_small_gram(b.d.nb, rows, b.d.r, a0, part, splits, st));
    return ORTHDION_OK;
  }
  // a single split is the Gram matrix itself: written straight into the class array
  if (splits == 1) {
    OD_TRY(od::launch_gram(b.d.nb, rows, b.d.r, a0, gram, 1, mode, st, &b.d, scal, side));
    return ORTHDION_OK;
  }
  OD_TRY(od::launch_gram(b.d.nb, rows, b.d.r, a0, part, splits, mode, st, &b.d, scal, side));
  // ordered reduction of the split partial sums on many workgroups: the factorisation runs on
  // one workgroup per matrix and should not spend its time summing
  OD_TRY(od::launch_reduce(b.d.nb, part, splits, (int64_t)b.d.r * b.d.r, gram, st));
  return ORTHDION_OK;
}

// Ranks of one 32 x 32 tile take the first pass in a single launch (factorisation included), so
// the class-wide Cholesky step is skipped for them.
static bool first_pass_in_one_launch(int r) { return r <= 32; }

// The rest of orth() after the first factorisation, in three pieces so that the guard in
// the middle can be launched once for every matrix of a rank:
//   orth_second_pass : a1 = a0 W1, Gram of a1, k_corr (T2 = I + Phi(E), Phi^T or W2, max|E|);
//                      r > 256: the summed Gram matrix of a flagged matrix goes to the class array
//   class_guard      : r > 256 only: Cholesky factor and inverse of I + E for every matrix of the
//                      class whose max|E| is above kFirstOrderDeviation (T2 and W2 are overwritten)
//   orth_result      : the correction a1 - a1 Phi(E) (fast precision) or a1 W2, for a flagged
//                      matrix the full product a1 W2 -> a0 | callers' Q (+ fp16 copies);
//                      r <= 256: the guard runs here, per batch (one launch: k_chol256 sums the
//                      partials itself).
// A matrix is flagged when its first pass left a deviation too large for the first-order form
// (an ill-conditioned B Q or R).  Every launch of the guard returns at once for the others.
static bool guard_is_class_wide(int r) { return r > 256; }

static int orth_second_pass(const Batch& b, char* ws, int rows, size_t off_a0, size_t off_a1, int64_t st_a, int splits,
                            size_t off_t1, size_t off_t2, int info_slot, float* scal, int* info, int exact, hipStream_t st) {
  const int nb = b.d.nb, r = b.d.r;
  WsArr a0{reinterpret_cast<float*>(ws + off_a0), st_a}, a1{reinterpret_cast<float*>(ws + off_a1), st_a};
  WsArr part{reinterpret_cast<float*>(ws + b.off_part), b.st_part};
  WsArr w{reinterpret_cast<float*>(ws + b.off_w), b.st_rr};
  WsArr t1{reinterpret_cast<float*>(ws + off_t1), b.st_rr}, t2{reinterpret_cast<float*>(ws + off_t2), b.st_rr};
  const HalfArr none{nullptr, 0};
  if (first_pass_in_one_launch(r)) {
    const WsArr part1 = part;                                   // Gram partials of a0 (orth_gram)
    part.base += (int64_t)splits * r * r;                       // Gram partials of a1, read by the second pass
    OD_TRY(od::launch_small_first_pass(nb, rows, r, a0, part1, splits, t1, w, a1, part, splits, info, info_slot, st));
  } else {
    OD_TRY(od::launch_apply(nb, rows, r, a0, w, a1, nullptr, none, none, exact, st));
    OD_TRY(od::launch_gram(nb, rows, r, a1, part, splits, exact ? od::kGramBF3 : od::kGramH2, st, nullptr, nullptr, 2));
  }
  // fast precision: Phi^T as fp16 operand words lives in the r x r scratch the factorisation no
  // longer needs; exact precision: W2 = I - Phi(E)
  const HalfArr phit{exact ? nullptr : reinterpret_cast<uint16_t*>(ws + b.off_tmp), 2 * b.st_rr};
  OD_TRY(od::launch_corr(nb, r, part, splits, t1, t2, w, phit, scal, 2 + info_slot, info, info_slot, st));
  if (guard_is_class_wide(r)) {
    const od::Pred big{scal, 2 + info_slot, od::kFirstOrderDeviation, 1};
    WsArr gram{reinterpret_cast<float*>(ws + b.off_gram), b.st_rr};
    OD_TRY(od::launch_reduce(nb, part, splits, (int64_t)r * r, gram, st, big));
  }
  return ORTHDION_OK;
}

// `which`: 0 = everything; 1 = only the first-order correction of the well-conditioned matrices,
// 2 = only the full product of the flagged ones (the two halves of a step that runs the guard on
// a second stream; fast precision and a class-wide guard only).
static int orth_result(const Batch& b, char* ws, int rows, size_t off_a0, size_t off_a1, int64_t st_a, int splits,
                       size_t off_t2, int info_slot, const MatPtrs* q_out, HalfArr hn, HalfArr ht, float* scal, int* info,
                       int exact, hipStream_t st, int which = 0) {
  const int nb = b.d.nb, r = b.d.r;
  WsArr a0{reinterpret_cast<float*>(ws + off_a0), st_a}, a1{reinterpret_cast<float*>(ws + off_a1), st_a};
  WsArr w{reinterpret_cast<float*>(ws + b.off_w), b.st_rr}, tmp{reinterpret_cast<float*>(ws + b.off_tmp), b.st_rr};
  WsArr t2{reinterpret_cast<float*>(ws + off_t2), b.st_rr};
  const od::Pred big{scal, 2 + info_slot, od::kFirstOrderDeviation, 1}, small{scal, 2 + info_slot, od::kFirstOrderDeviation, 0};
  if (!guard_is_class_wide(r)) {
    WsArr part{reinterpret_cast<float*>(ws + b.off_part), b.st_part};
    if (first_pass_in_one_launch(r)) part.base += (int64_t)splits * r * r;
    OD_TRY(od::launch_cholinv(nb, r, part, t2, w, tmp, info, info_slot, st, big, splits, (int64_t)r * r));
  }
  if (exact) {
    OD_TRY(od::launch_apply(nb, rows, r, a1, w, a0, q_out, hn, ht, exact, st));
  } else {
    const HalfArr phit{reinterpret_cast<uint16_t*>(ws + b.off_tmp), 2 * b.st_rr};
    if (which != 2) OD_TRY(od::launch_apply_correction(nb, rows, r, a1, phit, a0, q_out, hn, ht, st, small));
    if (which != 1) OD_TRY(od::launch_apply(nb, rows, r, a1, w, a0, q_out, hn, ht, exact, st, big));
  }
  return ORTHDION_OK;
}

// Cholesky factor and inverse for every matrix of a rank class; `off_t1` names the class array
// that receives the factors (left or right side).
static int class_cholinv(const RankClass& c, char* ws, size_t off_t1, int info_slot, int* info_all, hipStream_t st) {
  if (first_pass_in_one_launch(c.r)) return ORTHDION_OK;
  WsArr gram{reinterpret_cast<float*>(ws + c.off_gram), c.st_rr};
  WsArr w{reinterpret_cast<float*>(ws + c.off_w), c.st_rr}, tmp{reinterpret_cast<float*>(ws + c.off_tmp), c.st_rr};
  WsArr t1{reinterpret_cast<float*>(ws + off_t1), c.st_rr};
  OD_TRY(od::launch_cholinv(c.count, c.r, gram, t1, w, tmp, info_all + (size_t)c.slot_base * od::kInfoPerMat, info_slot, st));
  return ORTHDION_OK;
}

// The guard of the second pass for every matrix of a rank class above 256 (see orth_second_pass).
static int class_guard(const RankClass& c, char* ws, size_t off_t2, int info_slot, float* scal_all, int* info_all, hipStream_t st) {
  if (!guard_is_class_wide(c.r)) return ORTHDION_OK;
  WsArr gram{reinterpret_cast<float*>(ws + c.off_gram), c.st_rr};
  WsArr w{reinterpret_cast<float*>(ws + c.off_w), c.st_rr}, tmp{reinterpret_cast<float*>(ws + c.off_tmp), c.st_rr};
  WsArr t2{reinterpret_cast<float*>(ws + off_t2), c.st_rr};
  const od::Pred big{scal_all + (size_t)c.slot_base * od::kScalPerMat, 2 + info_slot, od::kFirstOrderDeviation, 1};
  OD_TRY(od::launch_cholinv(c.count, c.r, gram, t2, w, tmp, info_all + (size_t)c.slot_base * od::kInfoPerMat, info_slot, st, big));
  return ORTHDION_OK;
}

extern "C" int orthdion_step(orthdion_handle h, void* const* X, const void* const* G, float* const* M,
                             float* const* Q, void* workspace, size_t workspace_bytes, void* stream) {
  return orthdion_step_impl(h, X, G, M, Q, workspace, workspace_bytes, stream, 1);
}

extern "C" int orthdion_step_impl(orthdion_handle h, void* const* X, const void* const* G, float* const* M, float* const* Q,
                                  void* workspace, size_t workspace_bytes, void* stream, int allow_second_stream) {
  if (!h || !X || !G || !M || !Q || !workspace) return ORTHDION_E_NULL_PTR;
  if (workspace_bytes < h->ws_bytes) return ORTHDION_E_WORKSPACE_TOO_SMALL;
  if (reinterpret_cast<uintptr_t>(workspace) % kAlign) return ORTHDION_E_MISALIGNED;
  const int nmat = (int)h->mats.size();
  for (int i = 0; i < nmat; ++i) {
    if (!X[i] || !G[i] || !M[i] || !Q[i]) return ORTHDION_E_NULL_PTR;
    if (reinterpret_cast<uintptr_t>(X[i]) % 16 || reinterpret_cast<uintptr_t>(G[i]) % 16 ||
        reinterpret_cast<uintptr_t>(M[i]) % 16 || reinterpret_cast<uintptr_t>(Q[i]) % 16)
      return ORTHDION_E_MISALIGNED;
  }
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  // Launch errors are read back with hipGetLastError; drop whatever an earlier, unrelated
  // HIP call of this thread left there (e.g. a not-ready event query of the caller).
  (void)hipGetLastError();
  const od::Prec prec = resolve_prec(h->cfg);
  const int exact = prec == od::PREC_BF3 ? 1 : 0;
  float a_coef, b_coef;
  if (h->cfg.ef == ORTHDION_EF_DION) { a_coef = 1.f; b_coef = 1.f - h->cfg.mu; }
  else if (h->cfg.ef == ORTHDION_EF_PAPER) { a_coef = h->cfg.mu; b_coef = h->cfg.mu; }
  else { a_coef = h->cfg.mu; b_coef = 0.f; }

  int* info_all = reinterpret_cast<int*>(ws + h->off_info);
  float* scal_all = reinterpret_cast<float*>(ws + h->off_scal);
  if (prec != od::PREC_F16) {     // in fast precision the first kernel of every batch clears its own words
    // the scale words and, right behind them in the workspace, the info words: one fill (0.f and
    // 0 are the same bits)
    static_assert(sizeof(float) == sizeof(int), "one fill clears both tables");
    const int64_t words = (int64_t)((h->off_info - h->off_scal) / sizeof(int)) + (int64_t)nmat * od::kInfoPerMat;
    OD_TRY(od::launch_fill_int(reinterpret_cast<int*>(scal_all), words, 0, st));
  }
  h->last_ws = workspace;
  const bool diag = h->diag_on;
  h->diag_valid = diag;
  float* diag_all = reinterpret_cast<float*>(ws + h->off_diag);
  double* dacc_all = reinterpret_cast<double*>(ws + h->off_dacc);
  double* dpart_all = reinterpret_cast<double*>(ws + h->off_dpart);

#define OD_PHASE_BEGIN(ph)                                                   \
  do {                                                                       \
    if (hipEvent_t* e_ = prof_slot(h, bi, ph, 0)) OD_TRY(hipEventRecord(*e_, st)); \
  } while (0)
#define OD_PHASE_END(ph)                                                     \
  do {                                                                       \
    if (hipEvent_t* e_ = prof_slot(h, bi, ph, 1)) OD_TRY(hipEventRecord(*e_, st)); \
  } while (0)

  // phases that are one kernel: the kernel's own start / stop time stamps
#define OD_PHASE_KERNEL(ph)                                                  \
  do {                                                                       \
    hipEvent_t* e0_ = prof_slot(h, bi, ph, 0);                               \
    hipEvent_t* e1_ = prof_slot(h, bi, ph, 1);                               \
    if (e0_ && e1_) od::time_next_launch(*e0_, *e1_);                        \
  } while (0)

  // what every piece of a batch's work needs
  struct BatchView {
    MatPtrs ptrs;
    float* scal; int* info;
    WsArr pa, ra, part, colsq;
    HalfArr ph, pht, rh, qh, qht;
    double *dacc, *dpart;
  };
  const bool fast = prec == od::PREC_F16;
  const HalfArr none{nullptr, 0};
  auto view_of = [&](const Batch& b, BatchView& v) {
    std::memset(&v.ptrs, 0, sizeof(v.ptrs));
    for (int s = 0; s < b.d.nb; ++s) {
      int i = b.members[s];
      v.ptrs.X[s] = X[i]; v.ptrs.G[s] = G[i]; v.ptrs.M[s] = M[i]; v.ptrs.Q[s] = Q[i];
    }
    v.scal = scal_all + (size_t)b.slot_base * od::kScalPerMat;
    v.info = info_all + (size_t)b.slot_base * od::kInfoPerMat;
    v.pa = WsArr{reinterpret_cast<float*>(ws + b.off_pa), b.st_p};
    v.ra = WsArr{reinterpret_cast<float*>(ws + b.off_ra), b.st_r};
    v.part = WsArr{reinterpret_cast<float*>(ws + b.off_part), b.st_part};
    v.colsq = WsArr{reinterpret_cast<float*>(ws + b.off_colsq), b.st_colsq};
    v.ph = HalfArr{reinterpret_cast<uint16_t*>(ws + b.off_ph), b.st_p};
    v.pht = HalfArr{reinterpret_cast<uint16_t*>(ws + b.off_pht), b.st_p};
    v.rh = HalfArr{reinterpret_cast<uint16_t*>(ws + b.off_rh), b.st_r};
    v.qh = HalfArr{reinterpret_cast<uint16_t*>(ws + b.off_qh), b.st_r};
    v.qht = HalfArr{reinterpret_cast<uint16_t*>(ws + b.off_qht), b.st_r};
    v.dacc = dacc_all + (size_t)b.slot_base * od::kDaccPerMat;
    v.dpart = dpart_all + (size_t)b.slot_base * od::kDiagBlocks * 4;
  };

  // Alg. 1 lines 1-2, first part: P_raw = (M + G) Q and its Gram matrix
  auto left_head = [&](int bi) -> int {
    const Batch& b = h->batches[bi];
    const ClassDims& d = b.d;
    BatchView v;
    view_of(b, v);
    if (diag) OD_TRY(od::launch_diag_norms(d, v.ptrs, v.dpart, st));
    OD_PHASE_BEGIN(ORTHDION_PHASE_STATS);
    if (fast) OD_TRY(od::launch_stats(d, v.ptrs, v.scal, v.info, v.qht, st));
    OD_PHASE_END(ORTHDION_PHASE_STATS);
    OD_PHASE_KERNEL(ORTHDION_PHASE_PROJ);
    // a single split is the result itself: written straight to its place, nothing to add up
    const bool proj_direct = b.splits_proj == 1;
    OD_TRY(od::launch_proj(d, v.ptrs, prec, v.scal, proj_direct ? v.pa : v.part, b.splits_proj, v.qht, st));
    OD_PHASE_BEGIN(ORTHDION_PHASE_PROJ_REDUCE);
    if (!proj_direct) OD_TRY(od::launch_reduce(d.nb, v.part, b.splits_proj, (int64_t)d.m * d.r, v.pa, st));
    OD_PHASE_END(ORTHDION_PHASE_PROJ_REDUCE);
    OD_PHASE_BEGIN(ORTHDION_PHASE_GRAM_LEFT);
    int rc = orth_gram(b, ws, d.m, b.off_pa, b.st_p, b.splits_gram_p, fast, 0, v.scal, st);
    if (rc != ORTHDION_OK) return rc;
    OD_PHASE_END(ORTHDION_PHASE_GRAM_LEFT);
    return ORTHDION_OK;
  };

  // rest of line 2 (P = orth(P_raw)): second pass up to its deviation
  auto left_second = [&](int bi) -> int {
    const Batch& b = h->batches[bi];
    BatchView v;
    view_of(b, v);
    OD_PHASE_BEGIN(ORTHDION_PHASE_ORTH_LEFT);
    int rc = orth_second_pass(b, ws, b.d.m, b.off_pa, b.off_pb, b.st_p, b.splits_gram_p, b.off_tp1, b.off_tp2, 0, v.scal, v.info,
                              exact, st);
    if (rc != ORTHDION_OK) return rc;
    OD_PHASE_END(ORTHDION_PHASE_ORTH_LEFT);
    return ORTHDION_OK;
  };
  // P itself, line 3 (R = (M + G)^T P), and the head of line 4
  // `mode` (also for `tail`): 0 = the whole piece on `st`; with the guard on the second stream the
  // piece is enqueued in three parts: 1 = the result of the well-conditioned matrices on `st`,
  // 2 = the result of the flagged ones on the second stream, 3 = everything after the result
  auto middle = [&](int bi, int mode) -> int {
    const Batch& b = h->batches[bi];
    const ClassDims& d = b.d;
    BatchView v;
    view_of(b, v);
    int rc;
    if (mode == 2) {
      return orth_result(b, ws, d.m, b.off_pa, b.off_pb, b.st_p, b.splits_gram_p, b.off_tp2, 0, nullptr,
                         fast ? v.ph : none, fast ? v.pht : none, v.scal, v.info, exact, h->side, 2);
    }
    if (mode != 3) {
      OD_PHASE_BEGIN(ORTHDION_PHASE_FINISH_LEFT);
      rc = orth_result(b, ws, d.m, b.off_pa, b.off_pb, b.st_p, b.splits_gram_p, b.off_tp2, 0, nullptr,
                       fast ? v.ph : none, fast ? v.pht : none, v.scal, v.info, exact, st, mode);
      if (rc != ORTHDION_OK) return rc;
      OD_PHASE_END(ORTHDION_PHASE_FINISH_LEFT);
      if (mode == 1) return ORTHDION_OK;
    }
    OD_PHASE_KERNEL(ORTHDION_PHASE_BACK);
    // as for the projection: a single split goes straight to its place; fast precision still
    // needs the fp16 copy of R, made from there
    const bool back_direct = b.splits_back == 1;
    const bool copy_in_kernel = od::back_writes_fp16_copy(d, prec, b.splits_back);
    OD_TRY(od::launch_back(d, v.ptrs, prec, v.scal, v.pa, back_direct ? v.ra : v.part, b.splits_back, v.pht, st, v.rh, v.info));
    OD_PHASE_BEGIN(ORTHDION_PHASE_BACK_REDUCE);
    if (fast && !copy_in_kernel) OD_TRY(od::launch_reduce_r(d, back_direct ? v.ra : v.part, b.splits_back, v.ra, v.rh, v.scal, v.info, st));
    else if (!back_direct) OD_TRY(od::launch_reduce(d.nb, v.part, b.splits_back, (int64_t)d.n * d.r, v.ra, st));
    OD_PHASE_END(ORTHDION_PHASE_BACK_REDUCE);
    if (diag) OD_TRY(od::launch_diag_cols(d.nb, d.n, d.r, v.ra, v.part, b.slabs, v.dacc, st));
    if (h->cfg.variant == ORTHDION_QR) {
      OD_PHASE_BEGIN(ORTHDION_PHASE_GRAM_RIGHT);
      rc = orth_gram(b, ws, d.n, b.off_ra, b.st_r, b.splits_gram_q, fast, 1, v.scal, st);
      if (rc != ORTHDION_OK) return rc;
      OD_PHASE_END(ORTHDION_PHASE_GRAM_RIGHT);
    }
    return ORTHDION_OK;
  };

  // rest of line 4 for the QR variant: second pass of Q = orth(R) up to its deviation
  auto right_second = [&](int bi) -> int {
    const Batch& b = h->batches[bi];
    BatchView v;
    view_of(b, v);
    OD_PHASE_BEGIN(ORTHDION_PHASE_ORTH_RIGHT);
    int rc = orth_second_pass(b, ws, b.d.n, b.off_ra, b.off_rb, b.st_r, b.splits_gram_q, b.off_tq1, b.off_tq2, 1, v.scal, v.info,
                              exact, st);
    if (rc != ORTHDION_OK) return rc;
    OD_PHASE_END(ORTHDION_PHASE_ORTH_RIGHT);
    return ORTHDION_OK;
  };

  // rest of line 4: Q = orth(R) or ColNorm(R), written to the callers' Q (Q_prev is no longer
  // needed); lines 5-7: parameter update and error feedback in one pass
  auto tail = [&](int bi, int mode) -> int {
    const Batch& b = h->batches[bi];
    const ClassDims& d = b.d;
    BatchView v;
    view_of(b, v);
    if (mode == 2) {
      return orth_result(b, ws, d.n, b.off_ra, b.off_rb, b.st_r, b.splits_gram_q, b.off_tq2, 1, &v.ptrs,
                         fast ? v.qh : none, none, v.scal, v.info, exact, h->side, 2);
    }
    if (mode != 3) {
      OD_PHASE_BEGIN(ORTHDION_PHASE_FINISH_RIGHT);
      if (h->cfg.variant == ORTHDION_QR) {
        int rc = orth_result(b, ws, d.n, b.off_ra, b.off_rb, b.st_r, b.splits_gram_q, b.off_tq2, 1, &v.ptrs,
                             fast ? v.qh : none, none, v.scal, v.info, exact, st, mode);
        if (rc != ORTHDION_OK) return rc;
      } else {
        OD_TRY(od::launch_colnorm(d.nb, d.n, d.r, v.ra, v.ptrs, v.part, b.slabs, v.colsq, v.scal, v.info,
                                  fast ? v.qh : none, st));
      }
      OD_PHASE_END(ORTHDION_PHASE_FINISH_RIGHT);
      if (mode == 1) return ORTHDION_OK;
    }
    if (diag) {
      // nu = sigma_1(Q_new): Gram matrix of the new right factor, then power iteration
      WsArr rb{reinterpret_cast<float*>(ws + b.off_rb), b.st_r};
      WsArr gram{reinterpret_cast<float*>(ws + b.off_gram), b.st_rr}, tmp{reinterpret_cast<float*>(ws + b.off_tmp), b.st_rr};
      WsArr tq1{reinterpret_cast<float*>(ws + b.off_tq1), b.st_rr}, tq2{reinterpret_cast<float*>(ws + b.off_tq2), b.st_rr};
      if (h->cfg.variant == ORTHDION_QR) OD_TRY(od::launch_diag_trace(d.nb, d.r, tq1, tq2, v.dacc, st));
      OD_TRY(od::launch_gather_q(d.nb, d.n, d.r, v.ptrs, rb, st));
      OD_TRY(od::launch_gram(d.nb, d.n, d.r, rb, v.part, b.splits_gram_q, od::kGramBF3, st));
      OD_TRY(od::launch_reduce(d.nb, v.part, b.splits_gram_q, (int64_t)d.r * d.r, gram, st));
      OD_TRY(od::launch_power(d.nb, d.r, gram, tmp, 128, v.dacc, st));
      OD_TRY(od::launch_diag_final(d.nb, v.dpart, v.dacc, h->cfg.variant == ORTHDION_COLNORM ? 1 : 0,
                                   diag_all + (size_t)b.slot_base * od::kDiagPerMat, st));
    }
    OD_PHASE_KERNEL(ORTHDION_PHASE_EFX);
    if (fast) OD_TRY(od::launch_efx_h(d, v.ptrs, v.scal, v.info, v.ph, v.rh, v.qh, a_coef, b_coef, h->cfg.lr, st));
    else OD_TRY(od::launch_efx(d, v.ptrs, prec, v.scal, v.info, v.pa, v.ra, a_coef, b_coef, h->cfg.lr, st));
    return ORTHDION_OK;
  };

  // Rank class by rank class; inside a class the batches run piece by piece, so that each of
  // the two Cholesky steps is one launch sequence over all matrices of the class.  Its time is
  // booked on the first batch of the class.
  const hipStream_t caller_st = st;
  // pieces of a class between its two Cholesky steps
  auto class_head = [&](const RankClass& c) -> int {
    int rc;
    for (int b2 : c.batches)
      if ((rc = left_head(b2)) != ORTHDION_OK) return rc;
    return ORTHDION_OK;
  };
  auto class_chol = [&](const RankClass& c, int side, hipStream_t on) -> int {
    const int bi = c.batches[0];
    st = on;
    OD_PHASE_BEGIN(side == 0 ? ORTHDION_PHASE_CHOL_LEFT : ORTHDION_PHASE_CHOL_RIGHT);
    int rc = class_cholinv(c, ws, side == 0 ? c.off_tp1 : c.off_tq1, side, info_all, on);
    if (rc != ORTHDION_OK) return rc;
    OD_PHASE_END(side == 0 ? ORTHDION_PHASE_CHOL_LEFT : ORTHDION_PHASE_CHOL_RIGHT);
    st = caller_st;
    return ORTHDION_OK;
  };
  // Ranks above 256 in fast precision: the guard (a launch chain over the class that returns at
  // once for every well-conditioned matrix, then the full product of the flagged ones) runs on
  // the second stream beside the first-order result of the others; the streams join before
  // anything reads a factor.  (With two groups side by side the guard stays on its group's
  // stream: the other group fills the chip meanwhile.)
  auto class_middle = [&](const RankClass& c, bool fork_guard) -> int {
    int rc;
    const int bi = c.batches[0];
    for (int b2 : c.batches)
      if ((rc = left_second(b2)) != ORTHDION_OK) return rc;
    const bool forked = fork_guard && allow_second_stream && fast && guard_is_class_wide(c.r) && ensure_side_stream(h, st);
    if (forked) {
      OD_TRY(hipEventRecord(h->ev_fork, st));
      OD_TRY(hipStreamWaitEvent(h->side, h->ev_fork, 0));
      if ((rc = class_guard(c, ws, c.off_tp2, 0, scal_all, info_all, h->side)) != ORTHDION_OK) return rc;
      for (int b2 : c.batches)
        if ((rc = middle(b2, 2)) != ORTHDION_OK) return rc;
      OD_TRY(hipEventRecord(h->ev_join, h->side));
      for (int b2 : c.batches)
        if ((rc = middle(b2, 1)) != ORTHDION_OK) return rc;
      OD_TRY(hipStreamWaitEvent(st, h->ev_join, 0));
      for (int b2 : c.batches)
        if ((rc = middle(b2, 3)) != ORTHDION_OK) return rc;
    } else {
      OD_PHASE_BEGIN(ORTHDION_PHASE_GUARD_LEFT);
      if ((rc = class_guard(c, ws, c.off_tp2, 0, scal_all, info_all, st)) != ORTHDION_OK) return rc;
      OD_PHASE_END(ORTHDION_PHASE_GUARD_LEFT);
      for (int b2 : c.batches)
        if ((rc = middle(b2, 0)) != ORTHDION_OK) return rc;
    }
    return ORTHDION_OK;
  };
  auto class_tail = [&](const RankClass& c, bool fork_guard) -> int {
    int rc;
    const int bi = c.batches[0];
    bool forked_right = false;
    if (h->cfg.variant == ORTHDION_QR) {
      for (int b2 : c.batches)
        if ((rc = right_second(b2)) != ORTHDION_OK) return rc;
      forked_right = fork_guard && allow_second_stream && fast && guard_is_class_wide(c.r) && ensure_side_stream(h, st);
      if (forked_right) {
        OD_TRY(hipEventRecord(h->ev_fork, st));
        OD_TRY(hipStreamWaitEvent(h->side, h->ev_fork, 0));
        if ((rc = class_guard(c, ws, c.off_tq2, 1, scal_all, info_all, h->side)) != ORTHDION_OK) return rc;
        for (int b2 : c.batches)
          if ((rc = tail(b2, 2)) != ORTHDION_OK) return rc;
        OD_TRY(hipEventRecord(h->ev_join, h->side));
        for (int b2 : c.batches)
          if ((rc = tail(b2, 1)) != ORTHDION_OK) return rc;
        OD_TRY(hipStreamWaitEvent(st, h->ev_join, 0));
      } else {
        OD_PHASE_BEGIN(ORTHDION_PHASE_GUARD_RIGHT);
        if ((rc = class_guard(c, ws, c.off_tq2, 1, scal_all, info_all, st)) != ORTHDION_OK) return rc;
        OD_PHASE_END(ORTHDION_PHASE_GUARD_RIGHT);
      }
    }
    for (int b2 : c.batches)
      if ((rc = tail(b2, forked_right ? 3 : 0)) != ORTHDION_OK) return rc;
    return ORTHDION_OK;
  };

  // Two groups: the classes of group 1 go to the handle's group stream, which starts after
  // everything enqueued on the caller's stream so far and is joined before the call returns, so
  // the caller sees a single stream.  The groups share no matrix and no workspace slice;
  // whatever one group cannot fill the chip with (its Cholesky chains, the small reductions and
  // corrections, the last round of every launch) the other group's kernels run beside.
  const bool side_by_side = h->two_groups && allow_second_stream && ensure_side_stream(h, caller_st);
  if (side_by_side) {
    OD_TRY(hipEventRecord(h->ev_group_fork, caller_st));
    OD_TRY(hipStreamWaitEvent(h->group_stream, h->ev_group_fork, 0));
  }
  const bool right_chol = h->cfg.variant == ORTHDION_QR;
  for (const RankClass& c : h->classes) {
    int rc;
    const hipStream_t on = (side_by_side && c.group == 1) ? h->group_stream : caller_st;
    st = on;
    if ((rc = class_head(c)) != ORTHDION_OK) return rc;
    if ((rc = class_chol(c, 0, on)) != ORTHDION_OK) return rc;
    st = on;
    if ((rc = class_middle(c, !side_by_side)) != ORTHDION_OK) return rc;
    if (right_chol && (rc = class_chol(c, 1, on)) != ORTHDION_OK) return rc;
    st = on;
    if ((rc = class_tail(c, !side_by_side)) != ORTHDION_OK) return rc;
  }
  st = caller_st;
  if (side_by_side) {
    OD_TRY(hipEventRecord(h->ev_group_join, h->group_stream));
    OD_TRY(hipStreamWaitEvent(caller_st, h->ev_group_join, 0));
  }
  if (h->prof_on && h->prof_steps < h->prof_max_steps) h->prof_steps++;
  return ORTHDION_OK;
}

extern "C" int orthdion_profile_begin(orthdion_handle h, uint32_t phase_mask, int32_t max_steps) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (max_steps < 1 || max_steps > 100000 || h->prof_on) return ORTHDION_E_INVALID_ARG;
  size_t count = (size_t)max_steps * h->batches.size() * ORTHDION_NPHASE * 2;
  const int rc_alloc = no_throw([&] {
    h->prof_events.assign(count, nullptr);
    h->prof_recorded.assign(count / 2, 0);
    return (int)ORTHDION_OK;
  });
  if (rc_alloc != ORTHDION_OK) return rc_alloc;
  for (int s = 0; s < max_steps; ++s)
    for (size_t b = 0; b < h->batches.size(); ++b)
      for (int ph = 0; ph < ORTHDION_NPHASE; ++ph)
        if (phase_mask & (1u << ph))
          for (int e = 0; e < 2; ++e) {
            size_t idx = (((size_t)s * h->batches.size() + b) * ORTHDION_NPHASE + (size_t)ph) * 2 + (size_t)e;
            if (hipEventCreate(&h->prof_events[idx]) != hipSuccess) return ORTHDION_E_HIP;
          }
  h->prof_mask = phase_mask;
  h->prof_max_steps = max_steps;
  h->prof_steps = 0;
  h->prof_on = true;
  return ORTHDION_OK;
}

extern "C" int orthdion_profile_end(orthdion_handle h, float* ms_per_phase, int32_t* count_per_phase) {
  if (!h || !ms_per_phase || !count_per_phase) return ORTHDION_E_NULL_PTR;
  if (!h->prof_on) return ORTHDION_E_INVALID_ARG;
  int rc = ORTHDION_OK;
  for (int ph = 0; ph < ORTHDION_NPHASE; ++ph) { ms_per_phase[ph] = 0.f; count_per_phase[ph] = 0; }
  const size_t nb = h->batches.size();
  for (int s = 0; s < h->prof_steps; ++s)
    for (size_t b = 0; b < nb; ++b)
      for (int ph = 0; ph < ORTHDION_NPHASE; ++ph) {
        if (!(h->prof_mask & (1u << ph))) continue;
        size_t idx = (((size_t)s * nb + b) * ORTHDION_NPHASE + (size_t)ph) * 2;
        if (!h->prof_recorded[idx / 2]) continue;      // e.g. the Cholesky of a class: first batch only
        float ms = 0.f;
        if (hipEventSynchronize(h->prof_events[idx + 1]) != hipSuccess ||
            hipEventElapsedTime(&ms, h->prof_events[idx], h->prof_events[idx + 1]) != hipSuccess) {
          rc = ORTHDION_E_HIP;
          continue;
        }
        ms_per_phase[ph] += ms;
        count_per_phase[ph] += 1;
      }
  for (hipEvent_t e : h->prof_events)
    if (e) (void)hipEventDestroy(e);
  h->prof_events.clear();
  h->prof_on = false;
  return rc;
}

extern "C" int orthdion_get_info(orthdion_handle h, int32_t* info_host, void* stream) {
  if (!h || !info_host) return ORTHDION_E_NULL_PTR;
  if (!h->last_ws) return ORTHDION_E_NO_STEP;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int nmat = (int)h->mats.size();
  std::vector<int> raw;
  const int rc_alloc = no_throw([&] { raw.resize((size_t)nmat * od::kInfoPerMat); return (int)ORTHDION_OK; });
  if (rc_alloc != ORTHDION_OK) return rc_alloc;
  const char* ws = reinterpret_cast<const char*>(h->last_ws);
  OD_TRY(hipMemcpyAsync(raw.data(), ws + h->off_info, raw.size() * sizeof(int), hipMemcpyDeviceToHost, st));
  OD_TRY(hipStreamSynchronize(st));
  for (int i = 0; i < nmat; ++i) {
    const Batch& b = h->batches[h->batch_of[i]];
    const int* w = raw.data() + (size_t)(b.slot_base + h->slot_of[i]) * od::kInfoPerMat;
    int v = 0;
    if (w[0] != 0) v = w[0];
    else if (w[1] != 0) v = -w[1];
    else if (w[2] != 0) v = -w[2];
    info_host[i] = v;
  }
  return ORTHDION_OK;
}

extern "C" int orthdion_get_warnings(orthdion_handle h, uint32_t* warn_host, void* stream) {
  if (!h || !warn_host) return ORTHDION_E_NULL_PTR;
  if (!h->last_ws) return ORTHDION_E_NO_STEP;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int nmat = (int)h->mats.size();
  std::vector<int> raw;
  const int rc_alloc = no_throw([&] { raw.resize((size_t)nmat * od::kInfoPerMat); return (int)ORTHDION_OK; });
  if (rc_alloc != ORTHDION_OK) return rc_alloc;
  const char* ws = reinterpret_cast<const char*>(h->last_ws);
  OD_TRY(hipMemcpyAsync(raw.data(), ws + h->off_info, raw.size() * sizeof(int), hipMemcpyDeviceToHost, st));
  OD_TRY(hipStreamSynchronize(st));
  for (int i = 0; i < nmat; ++i) {
    const Batch& b = h->batches[h->batch_of[i]];
    warn_host[i] = (uint32_t)raw[(size_t)(b.slot_base + h->slot_of[i]) * od::kInfoPerMat + od::kWarnSlot];
  }
  return ORTHDION_OK;
}

extern "C" int orthdion_set_diagnostics(orthdion_handle h, int32_t enable) {
  if (!h) return ORTHDION_E_NULL_PTR;
  for (const Batch& b : h->batches)
    if (enable && b.d.r > 2048) return ORTHDION_E_BAD_SHAPE;     // power iteration keeps a vector of r floats in LDS
  h->diag_on = enable != 0;
  return ORTHDION_OK;
}

extern "C" int orthdion_get_diagnostics(orthdion_handle h, float* out_host, void* stream) {
  if (!h || !out_host) return ORTHDION_E_NULL_PTR;
  if (!h->last_ws || !h->diag_valid) return ORTHDION_E_NO_STEP;
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  const int nmat = (int)h->mats.size();
  std::vector<float> raw;
  const int rc_alloc = no_throw([&] { raw.resize((size_t)nmat * od::kDiagPerMat); return (int)ORTHDION_OK; });
  if (rc_alloc != ORTHDION_OK) return rc_alloc;
  const char* ws = reinterpret_cast<const char*>(h->last_ws);
  OD_TRY(hipMemcpyAsync(raw.data(), ws + h->off_diag, raw.size() * sizeof(float), hipMemcpyDeviceToHost, st));
  OD_TRY(hipStreamSynchronize(st));
  for (int i = 0; i < nmat; ++i) {
    const Batch& b = h->batches[h->batch_of[i]];
    const float* w = raw.data() + (size_t)(b.slot_base + h->slot_of[i]) * od::kDiagPerMat;
    for (int k = 0; k < od::kDiagPerMat; ++k) out_host[(size_t)i * ORTHDION_NDIAG + k] = w[k];
  }
  return ORTHDION_OK;
}

extern "C" int orthdion_rank_policy(float e_t, float ema_prev, int32_t r_min, int32_t r_max, float alpha, float gamma,
                                    float* ema_out, int32_t* r_next) {
  if (!ema_out || !r_next) return ORTHDION_E_NULL_PTR;
  if (r_min < 8 || r_max < r_min || r_min % 8 || r_max % 8) return ORTHDION_E_INVALID_ARG;
  if (!std::isfinite(e_t) || !std::isfinite(ema_prev) || e_t < 0.f || ema_prev < 0.f) return ORTHDION_E_INVALID_ARG;
  if (!(alpha >= 0.f && alpha <= 1.f) || !(gamma > 0.f) || !std::isfinite(gamma)) return ORTHDION_E_INVALID_ARG;
  // Alg. 2 in double precision: EMA, buffer multiplier, ceiling, clip, multiple of 8
  const double ema = (double)alpha * (double)e_t + (1.0 - (double)alpha) * (double)ema_prev;
  double target = std::ceil((double)gamma * ema);
  if (target < (double)r_min) target = (double)r_min;
  if (target > (double)r_max) target = (double)r_max;
  int32_t nxt = ((int32_t)target + 7) / 8 * 8;
  if (nxt < r_min) nxt = r_min;
  if (nxt > r_max) nxt = r_max;
  *ema_out = (float)ema;
  *r_next = nxt;
  return ORTHDION_OK;
}

extern "C" int orthdion_resize_q(const float* q_old, int64_t n, int32_t r_old, float* q_new, int32_t r_new,
                                 const float* pad, void* stream) {
  if (!q_old || !q_new) return ORTHDION_E_NULL_PTR;
  if (n < 8 || n % 8 || n >= (1 << 24) || r_old < 8 || r_new < 8 || r_old % 8 || r_new % 8 || r_old > n || r_new > n)
    return ORTHDION_E_BAD_SHAPE;
  if (r_new > r_old && !pad) return ORTHDION_E_NULL_PTR;
  if (reinterpret_cast<uintptr_t>(q_old) % 16 || reinterpret_cast<uintptr_t>(q_new) % 16 ||
      reinterpret_cast<uintptr_t>(pad) % 16)
    return ORTHDION_E_MISALIGNED;
  (void)hipGetLastError();
  OD_TRY(od::launch_resize_q(q_old, n, r_old, q_new, r_new, pad, reinterpret_cast<hipStream_t>(stream)));
  return ORTHDION_OK;
}

extern "C" int orthdion_workspace_layout(orthdion_handle h, int32_t index, size_t* off_p, size_t* off_r,
                                         size_t* off_tp1, size_t* off_tp2, size_t* off_tq1, size_t* off_tq2) {
  if (!h) return ORTHDION_E_NULL_PTR;
  if (index < 0 || index >= (int)h->mats.size()) return ORTHDION_E_INVALID_ARG;
  const Batch& b = h->batches[h->batch_of[index]];
  const size_t s = (size_t)h->slot_of[index];
  if (off_p) *off_p = b.off_pa + s * b.st_p * sizeof(float);
  if (off_r) *off_r = b.off_ra + s * b.st_r * sizeof(float);
  if (off_tp1) *off_tp1 = b.off_tp1 + s * b.st_rr * sizeof(float);
  if (off_tp2) *off_tp2 = b.off_tp2 + s * b.st_rr * sizeof(float);
  if (off_tq1) *off_tq1 = b.off_tq1 + s * b.st_rr * sizeof(float);
  if (off_tq2) *off_tq2 = b.off_tq2 + s * b.st_rr * sizeof(float);
  return ORTHDION_OK;
}

extern "C" const char* orthdion_strerror(int status) {
  switch (status) {
    case ORTHDION_OK: return "ok";
    case ORTHDION_E_INVALID_ARG: return "invalid argument";
    case ORTHDION_E_NULL_PTR: return "null pointer";
    case ORTHDION_E_BAD_SHAPE: return "unsupported shape: m, n, r, ld must be multiples of 8 with 8 <= r <= min(m, n) and ld >= n";
    case ORTHDION_E_WORKSPACE_TOO_SMALL: return "workspace too small";
    case ORTHDION_E_MISALIGNED: return "device pointer not sufficiently aligned";
    case ORTHDION_E_HIP: return "HIP call failed";
    case ORTHDION_E_NO_STEP: return "no step has been enqueued on this handle";
    case ORTHDION_E_NO_MEMORY: return "out of host memory";
    default: return "unknown status";
  }
}

extern "C" int orthdion_destroy(orthdion_handle h) {
  if (!h) return ORTHDION_E_NULL_PTR;
  for (hipEvent_t e : h->prof_events)
    if (e) (void)hipEventDestroy(e);
  if (h->ev_fork) (void)hipEventDestroy(h->ev_fork);
  if (h->ev_join) (void)hipEventDestroy(h->ev_join);
  if (h->ev_group_fork) (void)hipEventDestroy(h->ev_group_fork);
  if (h->ev_group_join) (void)hipEventDestroy(h->ev_group_join);
  if (h->side) (void)hipStreamDestroy(h->side);
  if (h->group_stream) (void)hipStreamDestroy(h->group_stream);
  delete h;
  return ORTHDION_OK;
}
