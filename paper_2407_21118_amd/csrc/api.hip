// Host side of the C ABI declared in include/palu.h: argument validation,
// launch geometry, workspace carving.  No device memory is allocated here.

#include "encode_quant.hip"
#include "rope_fold.hip"
#include "score.hip"
#include "score16.hip"
#include "score8.hip"
#include "combine.hip"
#include "pv.hip"
#include "qk.hip"
#include "probe.hip"

#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>

using namespace palu;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v, size_t a = kAlign) { return (v + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Tuning knobs (palu_set_option); 0 = automatic.
std::atomic<int> g_opt_score_waves{0};        // 4 or 8 wavefronts per score workgroup (ranks <= 256)
std::atomic<int> g_opt_score_mixed{1};        // 1: one score launch for a layer of several rank classes where the whole-head kernel takes them all
std::atomic<int> g_opt_score_chunks{0};       // sequence chunks per (sequence, head block) of the score kernel
std::atomic<int> g_opt_value_split{0};        // tokens per split of the value kernel
std::atomic<int> g_opt_score_fp8{0};          // 1: keys rebuilt from E4M3-rounded latents and weights (score8_kernel)
std::atomic<int> g_opt_shared_key_fp16{0};    // 1: the faster, fp16-rounded shared-key score form for 2 .. 16 queries per key/value head
std::atomic<int> g_opt_encode_tile{0};        // token rows per workgroup of the prompt-sized projection

int device_cu_count() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int v = cached[dev].load(std::memory_order_relaxed);
  if (v > 0) return v;
  if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) v = 256;
  cached[dev].store(v, std::memory_order_relaxed);
  return v;
}

// bits per code of a quantized latent dtype, 0 for fp16 / bf16 latents
inline int latent_bits(int dtype) { return dtype == PALU_I4 ? 4 : (dtype == PALU_I3 ? 3 : (dtype == PALU_I2 ? 2 : 0)); }

// ---- descriptor validation -------------------------------------------------
// nq: queries per sequence of the call; the kernels then see q_per_kv * nq heads per key/value head
int check_desc(const palu_layer_desc* d, Meta* m, int nq = 1) {
  if (!d || !d->group_head_off || !d->k_rank_off || !d->v_rank_off) return PALU_ERR_INVALID_ARG;
  if (d->n_heads <= 0 || d->n_groups <= 0 || d->d_head <= 0) return PALU_ERR_INVALID_ARG;
  if (d->act_dtype != PALU_F16 && d->act_dtype != PALU_BF16) return PALU_ERR_INVALID_ARG;
  for (int side = 0; side < 2; ++side) {
    const int ld = side ? d->v_latent_dtype : d->k_latent_dtype;
    if (ld != d->act_dtype && latent_bits(ld) == 0) return PALU_ERR_INVALID_ARG;
  }
  if (d->group_head_off[0] != 0 || d->k_rank_off[0] != 0 || d->v_rank_off[0] != 0) return PALU_ERR_INVALID_ARG;
  for (int j = 0; j < d->n_groups; ++j) {
    if (d->group_head_off[j + 1] <= d->group_head_off[j]) return PALU_ERR_INVALID_ARG;
    for (const int32_t* off : {d->k_rank_off, d->v_rank_off}) {
      const int r = off[j + 1] - off[j];
      if (r <= 0 || r % PALU_RANK_MULTIPLE != 0) return PALU_ERR_INVALID_ARG;
    }
  }
  if (d->group_head_off[d->n_groups] != d->n_heads) return PALU_ERR_INVALID_ARG;
  if (d->q_per_kv < 0) return PALU_ERR_INVALID_ARG;
  if (nq < 1 || nq > PALU_MAX_HEADS) return PALU_ERR_INVALID_ARG;
  const int qpk = (d->q_per_kv > 0 ? d->q_per_kv : 1) * nq;
  const bool any_i4 = latent_bits(d->k_latent_dtype) != 0 || latent_bits(d->v_latent_dtype) != 0;
  if (any_i4) {
    if (d->quant_block <= 0) return PALU_ERR_INVALID_ARG;
    for (int side = 0; side < 2; ++side) {
      if (latent_bits(side ? d->v_latent_dtype : d->k_latent_dtype) == 0) continue;
      const int32_t* off = side ? d->v_rank_off : d->k_rank_off;
      for (int j = 0; j <= d->n_groups; ++j)
        if (off[j] % d->quant_block != 0) return PALU_ERR_INVALID_ARG;
    }
  }
  // limits of this build
  if (d->d_head != PALU_D_HEAD) return PALU_ERR_UNSUPPORTED;
  if (d->n_heads > PALU_MAX_HEADS / qpk || d->n_groups > PALU_MAX_GROUPS) return PALU_ERR_UNSUPPORTED;
  if (any_i4 && (d->quant_block != 128 || d->act_dtype != PALU_F16)) return PALU_ERR_UNSUPPORTED;
  for (int j = 0; j < d->n_groups; ++j) {
    if (d->k_rank_off[j + 1] - d->k_rank_off[j] > PALU_MAX_RANK) return PALU_ERR_UNSUPPORTED;
    if (d->v_rank_off[j + 1] - d->v_rank_off[j] > PALU_MAX_RANK) return PALU_ERR_UNSUPPORTED;
  }
  if (m) {
    std::memset(m, 0, sizeof(*m));
    // from here on a head is a query head: qpk of them per key/value head of the descriptor
    m->n_heads = d->n_heads * qpk;
    m->n_groups = d->n_groups;
    m->qpk = qpk;
    m->nq = nq;
    int bk = 0, bv = 0;
    for (int j = 0; j <= d->n_groups; ++j) {
      m->head_off[j] = d->group_head_off[j] * qpk;
      m->k_off[j] = d->k_rank_off[j];
      m->v_off[j] = d->v_rank_off[j];
      m->bk_off[j] = bk;
      m->bv_off[j] = bv;
      if (j < d->n_groups) {
        const int s = (d->group_head_off[j + 1] - d->group_head_off[j]) * qpk;
        bk += (d->k_rank_off[j + 1] - d->k_rank_off[j]) * s * PALU_D_HEAD;
        bv += (d->v_rank_off[j + 1] - d->v_rank_off[j]) * s * PALU_D_HEAD;
        for (int h = d->group_head_off[j] * qpk; h < d->group_head_off[j + 1] * qpk; ++h) m->group_of_head[h] = (uint8_t)j;
      }
    }
  }
  return PALU_OK;
}

// ---- score-path work units ----------------------------------------------------
// The weight-stationary score kernel is compiled once per (rank, groups per
// workgroup): rank = 32*(c+1), c = 0..15.  Up to rank 256 a wavefront owns a whole
// head and a workgroup takes 4 heads; they may come from 1, 2 or 4 adjacent groups
// of equal rank as long as the staged row stays within 512 columns.  Above rank
// 256 a wavefront owns half a head and a workgroup takes 2 heads of one group.
constexpr int kNumRankCls = 16;
constexpr int kSlicedCls = kNumRankCls * 3;       // class of the 256-row slices of ranks above 512
constexpr int kNumScoreCls = kNumRankCls * 3 + 1; // (rank class, log2 of groups per workgroup), and the slices
constexpr int kScoreMaxWidth = 512;               // latent columns one workgroup stages per token

int rank_class(int r) { return (r >= 32 && r <= 512 && r % 32 == 0) ? r / 32 - 1 : -1; }
constexpr int kSliceRank = 256;                   // ranks above 512 are contracted in slices of this many rows
bool rank_class_half(int rc) { return rc >= 8; }

constexpr int kMaxPlanUnits = 1024;
struct ScorePlan {
  int n_cls;                           // kernel classes in use
  int cls_id[kNumScoreCls];            // rank class * 3 + log2(groups per workgroup) of each class in use
  int total_units;
  ScoreUnit units[kMaxPlanUnits];      // all units; unit_cls[i] indexes cls_id
  uint8_t unit_cls[kMaxPlanUnits];
  int slices[PALU_MAX_HEADS];          // rank slices of each head (1 unless its rank exceeds 512)
  bool half_heads[PALU_MAX_HEADS];     // head is always split over two wavefronts (rank 288..512)
  int max_slices;
};

// widen: let a unit of small groups span 2 or 4 adjacent groups of equal rank and size
int plan_score(const Meta& m, ScorePlan* p, bool widen = true, bool split16 = false) {
  p->n_cls = 0;
  p->total_units = 0;
  p->max_slices = 1;
  std::memset(p->half_heads, 0, sizeof(p->half_heads));
  int slot_of[kNumScoreCls];
  for (int& v : slot_of) v = -1;
  auto add_unit = [&](int id, const ScoreUnit& u) -> int {
    if (slot_of[id] < 0) {
      slot_of[id] = p->n_cls;
      p->cls_id[p->n_cls++] = id;
    }
    if (p->total_units >= kMaxPlanUnits) return PALU_ERR_UNSUPPORTED;
    p->units[p->total_units] = u;
    p->unit_cls[p->total_units] = (uint8_t)slot_of[id];
    ++p->total_units;
    return (int)PALU_OK;
  };
  int h = 0;
  while (h < m.n_heads) {
    const int j0 = m.group_of_head[h];
    const int r = m.k_off[j0 + 1] - m.k_off[j0];
    const int s = m.head_off[j0 + 1] - m.head_off[j0];
    ScoreUnit u;
    u.h0 = h;
    u.s = s;
    u.head_off0 = m.head_off[j0];
    u.head_stride = r * PALU_D_HEAD;
    if (r > 512) {
      // a rank too large for the register-resident weights: contract it in slices of
      // 256 rows; every slice is a unit of its own and writes its own score planes
      if (r % kSliceRank != 0) return PALU_ERR_UNSUPPORTED;
      const int nh = std::min(4, m.head_off[j0 + 1] - h);
      const int n_sl = r / kSliceRank;
      for (int sl = 0; sl < n_sl; ++sl) {
        u.nh = nh;
        u.k_off0 = m.k_off[j0] + sl * kSliceRank;
        u.bk_off0 = m.bk_off[j0] + (h - m.head_off[j0]) * u.head_stride + sl * kSliceRank * PALU_D_HEAD;
        u.head_off0 = h;                 // heads of the unit are counted from h0 inside one group
        u.part0 = 2 * sl;
        const int st = add_unit(kSlicedCls, u);
        if (st != PALU_OK) return st;
      }
      for (int x = 0; x < nh; ++x) p->slices[h + x] = n_sl;
      p->max_slices = std::max(p->max_slices, n_sl);
      h += nh;
      continue;
    }
    const int rc = rank_class(r);
    if (rc < 0) return PALU_ERR_UNSUPPORTED;
    if (rank_class_half(rc)) p->max_slices = std::max(p->max_slices, 2);      // planes for either form below
    if (rank_class_half(rc) && split16) {
      // rank 288 .. 512 on the whole-head kernel: two slices of 128 .. 256 rows (multiples of 32), each a unit
      // of its own rank class that writes one score plane
      const int nh = std::min(4, m.head_off[j0 + 1] - h);
      const int r0 = (r + 63) / 64 * 32;
      for (int sl = 0; sl < 2; ++sl) {
        u.nh = nh;
        u.k_off0 = m.k_off[j0] + sl * r0;
        u.bk_off0 = m.bk_off[j0] + (h - m.head_off[j0]) * u.head_stride + sl * r0 * PALU_D_HEAD;
        u.head_off0 = h;                 // heads of the unit are counted from h0 inside one group
        u.part0 = sl;
        const int st = add_unit(rank_class(sl ? r - r0 : r0) * 3, u);
        if (st != PALU_OK) return st;
      }
      for (int x = 0; x < nh; ++x) {
        p->slices[h + x] = 2;
        p->half_heads[h + x] = false;
      }
      h += nh;
      continue;
    }
    int nh, lg = 0;
    if (rank_class_half(rc)) {
      nh = std::min(2, m.head_off[j0 + 1] - h);
    } else {
      nh = std::min(4, m.head_off[j0 + 1] - h);
      if (widen && h == m.head_off[j0] && s <= 2) {
        // a small group: widen the unit over 2 or 4 whole adjacent groups of the same rank and size
        for (int g : {4, 2}) {
          if (g * s > 4 || g * r > kScoreMaxWidth || j0 + g > m.n_groups) continue;
          bool same = true;
          for (int x = 1; x < g; ++x)
            same = same && (m.k_off[j0 + x + 1] - m.k_off[j0 + x] == r) &&
                   (m.head_off[j0 + x + 1] - m.head_off[j0 + x] == s);
          if (same) { nh = g * s; lg = g == 4 ? 2 : 1; break; }
        }
      }
    }
    u.nh = nh;
    u.k_off0 = m.k_off[j0];
    u.bk_off0 = m.bk_off[j0];
    u.part0 = 0;
    const int st = add_unit(rc * 3 + lg, u);
    if (st != PALU_OK) return st;
    for (int x = 0; x < nh; ++x) {
      p->slices[h + x] = 1;
      p->half_heads[h + x] = rank_class_half(rc);
    }
    h += nh;
  }
  return PALU_OK;
}

// ---- value-path work units -----------------------------------------------------
// Units of the matrix-core value kernel: at most 256 latent columns and 16 heads each.
// Small adjacent groups are merged (up to 4 heads, 256 columns) so that a
// wavefront's 64 lanes all stream; wide latents are cut into column slices.
enum { kNumPvCls = 4 };            // class = 2 * (0: <=4 heads, 1: <=16) + (units of up to 256 columns)
struct PvPlan {
  int total_units;
  PvUnit units[kMaxPlanUnits];
  uint8_t unit_cls[kMaxPlanUnits];
};

int plan_pv(const Meta& m, PvPlan* p) {
  p->total_units = 0;
  auto add = [&](int h0, int nh, int c0, int ncols, int write_ml) -> int {
    if (p->total_units >= kMaxPlanUnits) return PALU_ERR_UNSUPPORTED;
    const int hs = nh <= 4 ? 0 : 1;
    PvUnit& x = p->units[p->total_units];
    x.h0 = (uint16_t)h0; x.c0 = c0; x.ncols = (uint16_t)ncols; x.nh = (uint8_t)nh; x.write_ml = (uint8_t)write_ml;
    p->unit_cls[p->total_units++] = (uint8_t)(2 * hs + (ncols > 128 ? 1 : 0));
    return PALU_OK;
  };
  int st;
  for (int j = 0; j < m.n_groups;) {
    const int s = m.head_off[j + 1] - m.head_off[j];
    const int rv = m.v_off[j + 1] - m.v_off[j];
    if (s <= 4 && rv <= 256) {
      int heads = s, cols = rv, j1 = j + 1;
      while (j1 < m.n_groups && heads + (m.head_off[j1 + 1] - m.head_off[j1]) <= 4 &&
             cols + (m.v_off[j1 + 1] - m.v_off[j1]) <= 256) {
        heads += m.head_off[j1 + 1] - m.head_off[j1];
        cols += m.v_off[j1 + 1] - m.v_off[j1];
        ++j1;
      }
      if ((st = add(m.head_off[j], heads, m.v_off[j], cols, 1)) != PALU_OK) return st;
      j = j1;
      continue;
    }
    // Larger groups: blocks of 16 heads x 256 columns.  A wavefront then has 16 KiB of latents per set in flight (with
    // 32 heads the accumulators leave room for 128 columns only, half of that, and the kernel is bound by
    // latency).  The head blocks of the same columns are neighbours in the list: they run as wavefronts of one
    // workgroup at the same time, so the second read of a latent row comes from the cache.
    const int hb = s <= 4 ? 4 : 16;
    const int cw = 256;
    for (int cs = 0; cs < rv; cs += cw)
      for (int u0 = 0; u0 < s; u0 += hb)
        if ((st = add(m.head_off[j] + u0, std::min(hb, s - u0), m.v_off[j] + cs, std::min(cw, rv - cs), cs == 0)) != PALU_OK)
          return st;
    ++j;
  }
  // One launch per head-count class: if any of its units is wider than 128 columns, the
  // narrower ones run in the two-block kernel as well (their second block idles).
  for (int hs = 0; hs < 2; ++hs) {
    bool wide = false;
    for (int i = 0; i < p->total_units; ++i) wide |= p->unit_cls[i] == 2 * hs + 1;
    if (wide)
      for (int i = 0; i < p->total_units; ++i)
        if (p->unit_cls[i] == 2 * hs) p->unit_cls[i] = (uint8_t)(2 * hs + 1);
  }
  return PALU_OK;
}

// Units of the no-RoPE score kernel: the value kernel's merging rule for small
// groups; a larger group is one unit with all its columns (32 heads at a time).
struct QkPlan {
  int total_units;
  QkUnit units[kMaxPlanUnits];
  long long qt_elems, qs_elems;    // per sequence
  size_t max_lds[2];               // staged folded-query bytes of the largest unit, per head-tile class
};

// quantized: the key latents are codes (their kernels contract the hi part of the folded query only)
int plan_qk(const Meta& m, bool quantized, QkPlan* p) {
  p->total_units = 0;
  p->qt_elems = p->qs_elems = 0;
  p->max_lds[0] = p->max_lds[1] = 0;
  auto add = [&](int h0, int nh, int c0, int ncols) -> int {
    if (p->total_units >= kMaxPlanUnits) return PALU_ERR_UNSUPPORTED;
    QkUnit& x = p->units[p->total_units++];
    x.c0 = c0; x.h0 = (uint16_t)h0; x.ncols = (uint16_t)ncols; x.nh = (uint8_t)nh;
    x.wpad = (uint16_t)(ceil_div(ncols, 256) * 256);
    x.q_off = (int32_t)p->qt_elems;
    x.qs_off = (int32_t)p->qs_elems;
    p->qt_elems += 2LL * nh * x.wpad;                  // hi and lo parts
    p->qs_elems += (long long)nh * (x.wpad >> 7);
    const size_t staged = (size_t)nh * (x.wpad + 8) * 2;
    x.use_lo = (uint8_t)((!quantized && 2 * staged <= 159 * 1024) ? 1 : 0);   // both parts staged in LDS while they fit
    size_t& lds = p->max_lds[nh > 16 ? 1 : 0];
    // quantized: the block sums of the folded query are staged behind its rows
    lds = std::max(lds, staged * (x.use_lo ? 2 : 1) + (quantized ? (size_t)nh * (x.wpad >> 7) * 4 : 0));
    return PALU_OK;
  };
  int st;
  for (int j = 0; j < m.n_groups;) {
    const int s = m.head_off[j + 1] - m.head_off[j];
    const int r = m.k_off[j + 1] - m.k_off[j];
    if (s <= 4 && r <= 256) {
      int heads = s, cols = r, j1 = j + 1;
      while (j1 < m.n_groups && heads + (m.head_off[j1 + 1] - m.head_off[j1]) <= 4 &&
             cols + (m.k_off[j1 + 1] - m.k_off[j1]) <= 256) {
        heads += m.head_off[j1 + 1] - m.head_off[j1];
        cols += m.k_off[j1 + 1] - m.k_off[j1];
        ++j1;
      }
      if ((st = add(m.head_off[j], heads, m.k_off[j], cols)) != PALU_OK) return st;
      j = j1;
      continue;
    }
    for (int u0 = 0; u0 < s; u0 += 32)
      if ((st = add(m.head_off[j] + u0, std::min(32, s - u0), m.k_off[j], r)) != PALU_OK) return st;
    ++j;
  }
  return PALU_OK;
}

// Wavefronts per compute unit the value kernel's splits aim at.
inline int value_waves_per_cu(const palu_layer_desc* d) { return latent_bits(d->v_latent_dtype) ? 8 : 4; }

// Tokens per value split and number of splits for a given attended length: a
// split is one wavefront's share; aim at four wavefronts per compute unit,
// splits of 64 to 512 tokens (more where the merge kernel's split limit asks for it).  Units of more than 4 heads
// write larger partial results per split (heads x columns floats against tokens x columns latents read), which the
// merge kernel reads again: their splits may be four times as long, where that still fills the chip.
constexpr int kPvSplitMin = 64, kPvSplitMax = 512;
void split_geometry(int total_units, int batch, int seq_len, int waves_per_cu, int max_unit_heads, int* split_tokens, int* n_split) {
  const long long items = std::max(1, total_units * batch);
  long long st = ceil_div((int)std::min<long long>(items * seq_len / ((long long)waves_per_cu * device_cu_count()) + 1, 1 << 30), 32) * 32LL;
  st = std::min<long long>(std::max<long long>(st, kPvSplitMin), max_unit_heads > 4 ? 4 * kPvSplitMax : kPvSplitMax);
  if (g_opt_value_split > 0) st = g_opt_value_split;
  st = std::max<long long>(st, ceil_div(ceil_div(seq_len, kMaxSplits), 32) * 32LL);
  *split_tokens = (int)st;
  *n_split = ceil_div(seq_len, (int)st);
}
// Upper bound of the number of splits of any attended length up to max_seq.
int split_bound(int total_units, int batch, int max_seq, int waves_per_cu) {
  int cap = std::max(ceil_div(waves_per_cu * device_cu_count(), std::max(1, total_units * batch)), ceil_div(max_seq, kPvSplitMax));
  if (g_opt_value_split > 0) cap = std::max(cap, ceil_div(max_seq, (int)g_opt_value_split));
  return std::min(cap, kMaxSplits) + 2;
}

struct Workspace {
  size_t mfold, scores, o_part, ml_part, rope_rows, qsum, qfrag, w8, w_scale, total;
  int lpad, o_stride;
  long long mfold_bstride, part_stride;
};

// per_sequence_fold: the region behind `mfold` holds something per sequence (the folded queries of the non-RoPE
// form); with RoPE it holds B_k in operand order, once.
int carve(const Meta& m, int batch, int max_seq, int n_split_cap, int n_parts, bool per_sequence_fold, Workspace* w) {
  w->lpad = ceil_div(max_seq, 32) * 32;
  w->mfold_bstride = m.bk_off[m.n_groups];
  w->o_stride = m.bv_off[m.n_groups] / PALU_D_HEAD;
  w->part_stride = (long long)batch * m.n_heads * w->lpad;
  size_t off = 0;
  w->mfold = off;   off = align_up(off + (size_t)(per_sequence_fold ? batch : 1) * w->mfold_bstride * 2);
  w->scores = off;  off = align_up(off + (size_t)n_parts * w->part_stride * 4);
  w->o_part = off;  off = align_up(off + (size_t)batch * n_split_cap * w->o_stride * 4);
  w->ml_part = off; off = align_up(off + (size_t)batch * n_split_cap * m.n_heads * 2 * 4);
  w->rope_rows = off; off = align_up(off + (size_t)(w->lpad / 32) * kRopeTileBytes);   // angle tiles gathered by k_pos
  w->qsum = off; off = align_up(off + (size_t)batch * m.n_heads * (PALU_MAX_RANK / 128 + 2) * 4);   // int4 block sums of the folded queries (no-RoPE path)
  // several queries per key/value head: rotated queries as contraction operands, 2 feature halves x 4 KiB per key/value head
  w->qfrag = off; off = align_up(off + (m.qpk > 1 ? (size_t)batch * (m.n_heads / m.qpk) * 2 * 4096 : 0));
  // 8-bit key reconstruction (option score_fp8): B_k as E4M3 bytes in operand order, and its column scales
  w->w8 = off; off = align_up(off + (g_opt_score_fp8 ? (size_t)w->mfold_bstride : 0));
  w->w_scale = off; off = align_up(off + (g_opt_score_fp8 ? (size_t)m.n_heads * PALU_D_HEAD * 4 : 0));
  w->total = off;
  return PALU_OK;
}

// Dynamic LDS next to a kernel's static arrays (at most kStaticLdsMax bytes of them): past 64 KiB in total the
// kernel's limit has to be raised.
constexpr size_t kStaticLdsMax = 16 * 1024;
template <typename K>
int allow_dynamic_lds(K kernel, size_t dynamic_bytes) {
  if (dynamic_bytes + kStaticLdsMax <= 64 * 1024) return PALU_OK;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)dynamic_bytes) == hipSuccess ? PALU_OK : PALU_ERR_HIP;
}

template <typename K>
int allow_lds(K kernel, size_t bytes) {
  if (bytes <= 64 * 1024) return PALU_OK;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                             (int)bytes) == hipSuccess ? PALU_OK : PALU_ERR_HIP;
}

using ScoreFn = void (*)(ScoreArgs);
// waves8: four heads as 8 half-head wavefronts (two per SIMD) instead of 4 whole-head ones.
template <typename T, bool I4, int NKS>
ScoreFn score_fn_g(int lg, bool waves8) {
  if constexpr (NKS > 16) {
    return score_kernel<T, NKS, 2, 1, 4, I4>;
  } else {
    if (waves8) {
      if constexpr (NKS <= 8) { if (lg == 2) return score_kernel<T, NKS, 2, 4, 8, I4>; }
      if (lg == 1) return score_kernel<T, NKS, 2, 2, 8, I4>;
      return score_kernel<T, NKS, 2, 1, 8, I4>;
    }
    if constexpr (NKS <= 8) { if (lg == 2) return score_kernel<T, NKS, 4, 4, 4, I4>; }
    if (lg == 1) return score_kernel<T, NKS, 4, 2, 4, I4>;
    return score_kernel<T, NKS, 4, 1, 4, I4>;
  }
}
template <typename T, bool I4>
ScoreFn score_fn_t(int rc, int lg, bool w8) {
  switch (rc) {
    case 0: return score_fn_g<T, I4, 2>(lg, w8);
    case 1: return score_fn_g<T, I4, 4>(lg, w8);
    case 2: return score_fn_g<T, I4, 6>(lg, w8);
    case 3: return score_fn_g<T, I4, 8>(lg, w8);
    case 4: return score_fn_g<T, I4, 10>(lg, w8);
    case 5: return score_fn_g<T, I4, 12>(lg, w8);
    case 6: return score_fn_g<T, I4, 14>(lg, w8);
    case 7: return score_fn_g<T, I4, 16>(lg, w8);
    case 8: return score_fn_g<T, I4, 18>(lg, w8);
    case 9: return score_fn_g<T, I4, 20>(lg, w8);
    case 10: return score_fn_g<T, I4, 22>(lg, w8);
    case 11: return score_fn_g<T, I4, 24>(lg, w8);
    case 12: return score_fn_g<T, I4, 26>(lg, w8);
    case 13: return score_fn_g<T, I4, 28>(lg, w8);
    case 14: return score_fn_g<T, I4, 30>(lg, w8);
    default: return score_fn_g<T, I4, 32>(lg, w8);
  }
}
ScoreFn score_fn(int act, bool i4, int cls_id, bool w8) {
  const int rc = cls_id / 3, lg = cls_id % 3;
  if (i4) return score_fn_t<F16, true>(rc, lg, w8);
  return act == PALU_F16 ? score_fn_t<F16, false>(rc, lg, w8) : score_fn_t<BF16, false>(rc, lg, w8);
}

// unquantized latents, ranks 64 .. 256, one query per head: one whole head per wavefront (score16.hip)
template <typename T, int NK>
ScoreFn score16_fn_g(int lg) {
  if constexpr (NK <= 2) { if (lg == 2) return score16_kernel<T, NK, 4>; }
  if constexpr (NK <= 4) { if (lg >= 1) return score16_kernel<T, NK, 2>; }
  return score16_kernel<T, NK, 1>;
}
template <int NK>
ScoreFn score8_fn_g(int lg) {
  if constexpr (NK <= 2) { if (lg == 2) return score8_kernel<NK, 4>; }
  if constexpr (NK <= 4) { if (lg >= 1) return score8_kernel<NK, 2>; }
  return score8_kernel<NK, 1>;
}
ScoreFn score8_fn(int rc, int lg) {
  switch (rc) {
    case 1: return score8_fn_g<2>(lg);
    case 2: return score8_fn_g<3>(lg);
    case 3: return score8_fn_g<4>(lg);
    case 4: return score8_fn_g<5>(lg);
    case 5: return score8_fn_g<6>(lg);
    case 6: return score8_fn_g<7>(lg);
    default: return score8_fn_g<8>(lg);
  }
}
template <typename T>
ScoreFn score16_fn_t(int rc, int lg) {
  switch (rc) {
    case 1: return score16_fn_g<T, 2>(lg);
    case 2: return score16_fn_g<T, 3>(lg);
    case 3: return score16_fn_g<T, 4>(lg);
    case 4: return score16_fn_g<T, 5>(lg);
    case 5: return score16_fn_g<T, 6>(lg);
    case 6: return score16_fn_g<T, 7>(lg);
    default: return score16_fn_g<T, 8>(lg);
  }
}
inline bool rank_class_16(int rc) { return rc >= 1 && rc <= 7; }
// ... and several queries per key/value head: the key rebuilt once per key/value head and pass of up to 8 query
// rows (ranks 192 .. 256) or 4 (ranks 64 .. 160); the kernel is compiled for 2, 4 and 8 rows
inline bool shared16_ok(int rc) { return rc >= 1 && rc <= 7; }
inline int shared16_rows_per_pass(int rc) { return rc >= 5 ? 8 : 4; }
template <typename T, int NK>
ScoreFn score16q_fn_n(int nq) {
  if (nq <= 2) return score16_kernel<T, NK, 1, 2>;
  if (nq <= 4) return score16_kernel<T, NK, 1, 4>;
  if constexpr (NK >= 6) { if (nq <= 8) return score16_kernel<T, NK, 1, 8>; }
  return nullptr;
}
// 4-bit key latents (ranks 128 and 256: whole quantization blocks) with several queries per key/value head
ScoreFn score16q4_fn(int rc, int nq) {
  if (rc == 3) return nq <= 2 ? score16_kernel<F16, 4, 1, 2, 4> : (nq <= 4 ? score16_kernel<F16, 4, 1, 4, 4> : nullptr);
  if (rc == 7) return nq <= 2 ? score16_kernel<F16, 8, 1, 2, 4> : (nq <= 4 ? score16_kernel<F16, 8, 1, 4, 4> : score16_kernel<F16, 8, 1, 8, 4>);
  return nullptr;
}
constexpr int score16q4_lds_bytes(int width) { return 3 * score_tile_bytes(width) + 3 * kRopeTileBytes; }
template <typename T>
ScoreFn score16q_fn_t(int rc, int nq) {
  switch (rc) {
    case 1: return score16q_fn_n<T, 2>(nq);
    case 2: return score16q_fn_n<T, 3>(nq);
    case 3: return score16q_fn_n<T, 4>(nq);
    case 4: return score16q_fn_n<T, 5>(nq);
    case 5: return score16q_fn_n<T, 6>(nq);
    case 6: return score16q_fn_n<T, 7>(nq);
    case 7: return score16q_fn_n<T, 8>(nq);
    default: return nullptr;
  }
}

// 3- and 2-bit key latents: one group per workgroup, 8 wavefronts up to rank 256, 4 half-head wavefronts above
template <int NKS>
ScoreFn score_fn_lowbit_n() {
  if constexpr (NKS > 16) return score_kernel<F16, NKS, 2, 1, 4, true, 0, true>;
  else return score_kernel<F16, NKS, 2, 1, 8, true, 0, true>;
}
ScoreFn score_fn_lowbit(int rc) {
  switch (rc) {
    case 0: return score_fn_lowbit_n<2>();
    case 1: return score_fn_lowbit_n<4>();
    case 2: return score_fn_lowbit_n<6>();
    case 3: return score_fn_lowbit_n<8>();
    case 4: return score_fn_lowbit_n<10>();
    case 5: return score_fn_lowbit_n<12>();
    case 6: return score_fn_lowbit_n<14>();
    case 7: return score_fn_lowbit_n<16>();
    case 8: return score_fn_lowbit_n<18>();
    case 9: return score_fn_lowbit_n<20>();
    case 10: return score_fn_lowbit_n<22>();
    case 11: return score_fn_lowbit_n<24>();
    case 12: return score_fn_lowbit_n<26>();
    case 13: return score_fn_lowbit_n<28>();
    case 14: return score_fn_lowbit_n<30>();
    default: return score_fn_lowbit_n<32>();
  }
}

// shared-key form (several queries per key/value head): fp16 latents, ranks up to 256, 8 wavefronts, up to 16 queries
// QP = 1: at most 4 queries per key/value head, QP = 2: at most 16
template <int QP>
ScoreFn score_fn_shared(int rc) {
  switch (rc) {
    case 0: return score_kernel<F16, 2, 2, 1, 8, false, QP>;
    case 1: return score_kernel<F16, 4, 2, 1, 8, false, QP>;
    case 2: return score_kernel<F16, 6, 2, 1, 8, false, QP>;
    case 3: return score_kernel<F16, 8, 2, 1, 8, false, QP>;
    case 4: return score_kernel<F16, 10, 2, 1, 8, false, QP>;
    case 5: return score_kernel<F16, 12, 2, 1, 8, false, QP>;
    case 6: return score_kernel<F16, 14, 2, 1, 8, false, QP>;
    default: return score_kernel<F16, 16, 2, 1, 8, false, QP>;
  }
}

// The same layer with one (virtual) query head per key/value head: the units of the shared-key score form.
Meta kv_head_meta(const Meta& m) {
  Meta k;
  std::memset(&k, 0, sizeof(k));
  k.n_heads = m.n_heads / m.qpk;
  k.n_groups = m.n_groups;
  k.qpk = 1;
  k.nq = 1;
  for (int j = 0; j <= m.n_groups; ++j) {
    k.head_off[j] = m.head_off[j] / m.qpk;
    k.k_off[j] = m.k_off[j];
    k.v_off[j] = m.v_off[j];
    k.bk_off[j] = m.bk_off[j] / m.qpk;
    k.bv_off[j] = m.bv_off[j] / m.qpk;
    if (j < m.n_groups)
      for (int h = k.head_off[j]; h < m.head_off[j + 1] / m.qpk; ++h) k.group_of_head[h] = (uint8_t)j;
  }
  return k;
}

using PvFn = void (*)(PvArgs);
template <typename T, int QB, bool TWO>
PvFn pv_fn_t(int cls) {
  switch (cls) {
    case 0: return pv_kernel<T, 2, 1, QB, TWO>;
    case 1: return pv_kernel<T, 2, 2, QB, TWO>;
    case 2: return pv_kernel<T, 8, 1, QB, TWO>;
    default: return pv_kernel<T, 8, 2, QB, TWO>;
  }
}
template <bool TWO>
PvFn pv_fn_p(int act, int bits, int cls) {
  if (bits == 4) return pv_fn_t<F16, 4, TWO>(cls);
  if (bits == 3) return pv_fn_t<F16, 3, TWO>(cls);
  if (bits == 2) return pv_fn_t<F16, 2, TWO>(cls);
  return act == PALU_F16 ? pv_fn_t<F16, 0, TWO>(cls) : pv_fn_t<BF16, 0, TWO>(cls);
}
// bits: 4, 3 or 2 for quantized value latents, else 0; two_planes: some head's scores lie in two planes
PvFn pv_fn(int act, int bits, int cls, bool two_planes) {
  return two_planes ? pv_fn_p<true>(act, bits, cls) : pv_fn_p<false>(act, bits, cls);
}

// First launch of a fused decode step: the split-K partial products of the new token's down-projection
// (the long HBM stream) and the fold of the rotated query into B_k do not depend on each other.  The grid
// is the projection's; its first fold_blocks workgroups also fold one (k-step, head, sequence) item each,
// after their weight loads have gone out; items beyond the projection's grid get workgroups of their own.
struct StepHeadArgs {
  EncodeArgs enc;
  EncodeTArgs enc_t;                     // TR instantiations: the projection from transposed weights, grid (enc_blocks)
  FoldArgs fold;
  int fold_blocks, fold_gx;              // weight layout grid (k-steps, heads), linearised
  int enc_blocks, enc_gx, enc_gy;        // projection grid (column blocks, k splits, sides), linearised
  // shared-key form of the score kernel: its rotated-query operands are further items, after the fold's
  const uint16_t* sk_q;                  // the call's q, NULL when the step has no such items
  const int32_t* sk_q_pos;
  uint16_t* sk_qfrag;
  int sk_blocks, sk_n_kv, sk_qpk, sk_nq, sk_n_heads, sk_small;
};

template <typename T, int kEncTok, bool TR>
__global__ __launch_bounds__(256) void step_head_kernel(StepHeadArgs a) {
  const int id = blockIdx.x;
  auto fold_item = [&]() __attribute__((always_inline)) {
    if (id < a.fold_blocks) {
      fold_body(a.fold, id % a.fold_gx, id / a.fold_gx);
    } else if (id < a.fold_blocks + a.sk_blocks) {
      if constexpr (__is_same(T, F16)) {             // the shared-key form exists for fp16 latents only
        struct View {                                // QfragArgs' members, read in place from this kernel's arguments
          const uint16_t* q;
          const int32_t* q_pos;
          uint16_t* qfrag;
          const float (&rev_hi)[kHalf];
          const float (&rev_lo)[kHalf];
          int n_kv, qpk, nq, n_heads, small;
        };
        const View qa{a.sk_q, a.sk_q_pos, a.sk_qfrag, a.fold.rev_hi, a.fold.rev_lo,
                      a.sk_n_kv, a.sk_qpk, a.sk_nq, a.sk_n_heads, a.sk_small};
        const int item = id - a.fold_blocks;
        qfrag_body<T>(qa, item % a.sk_n_kv, item / a.sk_n_kv);
      }
    }
  };
  if (id < a.enc_blocks) {
    if constexpr (TR) {
      encode_t_body<T, kEncTok>(a.enc_t, id, fold_item);
    } else {
      const int bx = id % a.enc_gx, rest = id / a.enc_gx;
      encode_partial_body<T, kEncTok>(a.enc, bx, rest % a.enc_gy, rest / a.enc_gy, fold_item);
    }
  } else {
    fold_item();
  }
}

// The same for non-RoPE attention: the items are those of qfold_kernel (query folded into the latent space).
struct StepHeadNoRopeArgs {
  EncodeArgs enc;
  EncodeTArgs enc_t;
  QfoldArgs qfold;
  int q_blocks, q_gx, q_gy;              // qfold grid (column blocks, heads, batch / 4), linearised
  int enc_blocks, enc_gx, enc_gy;
};

template <typename T, int kEncTok, bool TR>
__global__ __launch_bounds__(256) void step_head_norope_kernel(StepHeadNoRopeArgs a) {
  const int id = blockIdx.x;
  auto item = [&]() __attribute__((always_inline)) {
    if (id < a.q_blocks) {
      const int bx = id % a.q_gx, rest = id / a.q_gx;
      qfold_body<T>(a.qfold, bx, rest % a.q_gy, rest / a.q_gy);
    }
  };
  if (id < a.enc_blocks) {
    if constexpr (TR) {
      encode_t_body<T, kEncTok>(a.enc_t, id, item);
    } else {
      const int bx = id % a.enc_gx, rest = id / a.enc_gx;
      encode_partial_body<T, kEncTok>(a.enc, bx, rest % a.enc_gy, rest / a.enc_gy, item);
    }
  } else {
    item();
  }
}

using StepHeadNoRopeFn = void (*)(StepHeadNoRopeArgs);
StepHeadNoRopeFn step_head_norope_fn(int act, int tok_cls, bool tr) {
#define PALU_SH(K, T, TR) {K<T, 1, TR>, K<T, 2, TR>, K<T, 4, TR>, K<T, 8, TR>}
  static const StepHeadNoRopeFn f16[2][4] = {PALU_SH(step_head_norope_kernel, F16, false), PALU_SH(step_head_norope_kernel, F16, true)};
  static const StepHeadNoRopeFn bf16[2][4] = {PALU_SH(step_head_norope_kernel, BF16, false), PALU_SH(step_head_norope_kernel, BF16, true)};
  return act == PALU_F16 ? f16[tr][tok_cls] : bf16[tr][tok_cls];
}

using StepHeadFn = void (*)(StepHeadArgs);
StepHeadFn step_head_fn(int act, int tok_cls, bool tr) {
  static const StepHeadFn f16[2][4] = {PALU_SH(step_head_kernel, F16, false), PALU_SH(step_head_kernel, F16, true)};
  static const StepHeadFn bf16[2][4] = {PALU_SH(step_head_kernel, BF16, false), PALU_SH(step_head_kernel, BF16, true)};
#undef PALU_SH
  return act == PALU_F16 ? f16[tr][tok_cls] : bf16[tr][tok_cls];
}
inline int launch_ok() { return hipGetLastError() == hipSuccess ? PALU_OK : PALU_ERR_HIP; }

}  // namespace

extern "C" {

const char* palu_status_string(int status) {
  switch (status) {
    case PALU_OK: return "ok";
    case PALU_ERR_INVALID_ARG: return "invalid argument";
    case PALU_ERR_UNSUPPORTED: return "unsupported configuration";
    case PALU_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
    case PALU_ERR_HIP: return "HIP runtime error";
    default: return "unknown status";
  }
}

int palu_version(void) { return 100; }

int palu_probe_mfma(int32_t iters, float* sink, void* stream, double* out_flops) {
  if (iters <= 0 || !sink) return PALU_ERR_INVALID_ARG;
  const int cus = device_cu_count();
  hipLaunchKernelGGL(probe_mfma_kernel, dim3((unsigned)(cus * 2)), dim3(256), 0, static_cast<hipStream_t>(stream), sink, iters);
  if (out_flops) *out_flops = (double)cus * 2 * 4 /* wavefronts */ * iters * 4.0 * (2.0 * 32 * 32 * 16);
  return launch_ok();
}

int palu_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink || bytes < 16 || (reinterpret_cast<uintptr_t>(src) & 15)) return PALU_ERR_INVALID_ARG;
  hipLaunchKernelGGL(probe_read_kernel, dim3((unsigned)(device_cu_count() * 8)), dim3(256), 0, static_cast<hipStream_t>(stream),
                     static_cast<const uint4v*>(src), bytes / 16, sink);
  return launch_ok();
}

int palu_set_option(const char* name, int value) {
  if (!name || value < 0) return PALU_ERR_INVALID_ARG;
  if (!std::strcmp(name, "score_waves")) {
    if (value != 0 && value != 4 && value != 8) return PALU_ERR_INVALID_ARG;
    g_opt_score_waves = value;
  } else if (!std::strcmp(name, "score_mixed")) {
    if (value > 16) return PALU_ERR_INVALID_ARG;
    g_opt_score_mixed = value;
  } else if (!std::strcmp(name, "score_chunks")) {
    g_opt_score_chunks = value;
  } else if (!std::strcmp(name, "value_split_tokens")) {
    if (value != 0 && (value % 32 != 0 || value > 4096)) return PALU_ERR_INVALID_ARG;
    g_opt_value_split = value;
  } else if (!std::strcmp(name, "score_fp8")) {
    if (value > 1) return PALU_ERR_INVALID_ARG;
    g_opt_score_fp8 = value;
  } else if (!std::strcmp(name, "shared_key_fp16")) {
    if (value > 1) return PALU_ERR_INVALID_ARG;
    g_opt_shared_key_fp16 = value;
  } else if (!std::strcmp(name, "encode_tile_rows")) {
    if (value != 0 && value != 32 && value != 64 && value != 128 && value != 256) return PALU_ERR_INVALID_ARG;
    g_opt_encode_tile = value;
  } else {
    return PALU_ERR_INVALID_ARG;
  }
  return PALU_OK;
}

int palu_rope_table_bytes(int32_t d_head, int32_t n_pos, size_t* out_bytes) {
  if (!out_bytes || n_pos <= 0 || d_head <= 0) return PALU_ERR_INVALID_ARG;
  if (d_head != PALU_D_HEAD) return PALU_ERR_UNSUPPORTED;
  *out_bytes = rope_tiles(n_pos) * kRopeTableStride;
  return PALU_OK;
}

int palu_rope_table_init(float rope_theta, int32_t d_head, int32_t n_pos, void* table, void* stream) {
  if (!table || n_pos <= 0 || d_head <= 0) return PALU_ERR_INVALID_ARG;
  if (d_head != PALU_D_HEAD) return PALU_ERR_UNSUPPORTED;
  if ((reinterpret_cast<uintptr_t>(table) & 15) != 0) return PALU_ERR_INVALID_ARG;
  const long long n_pad = (long long)rope_tiles(n_pos) * kRopeTilePos;
  if (n_pad > (1LL << 30)) return PALU_ERR_UNSUPPORTED;
  const long long items = n_pad * kHalf;
  hipLaunchKernelGGL(rope_table_kernel, dim3((unsigned)((items + 255) / 256)), dim3(256), 0,
                     static_cast<hipStream_t>(stream), static_cast<unsigned char*>(table), (int)n_pad, rope_theta);
  return launch_ok();
}

// ------------------------------------------------------------------ encode
namespace {
constexpr int kEncodeGemmTokens = 64;    // from this many tokens on the projection runs as a tiled GEMM (no workspace)
}

int palu_encode_workspace_bytes(const palu_layer_desc* desc, int which, int32_t n_tok, size_t* out_bytes) {
  Meta m;
  const int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  if (!out_bytes || n_tok <= 0 || which < 0 || which > 2) return PALU_ERR_INVALID_ARG;
  const int d = m.n_heads * PALU_D_HEAD;
  size_t total = 0;
  for (int side = 0; side < 2; ++side) {
    if (which != 2 && which != side) continue;
    const int R = side ? m.v_off[m.n_groups] : m.k_off[m.n_groups];
    total += align_up((size_t)(d / kEncRows) * std::min(n_tok, kEncodeGemmTokens - 1) * R * 4);
  }
  *out_bytes = std::max<size_t>(total, 256);
  return PALU_OK;
}

namespace {
// A validated down-projection call, ready to launch.
struct EncodePlan {
  EncodeArgs a;
  bool gemm;              // many tokens: tiled GEMM, no workspace
  int n_sides, max_R;
  int tok_cls;            // split-K and transposed forms: 8, 4, 2 or 1 tokens per pass (index 3 .. 0)
  bool transposed;        // weights given as At [R, d]: one launch, no partial sums (t, t_lds, t_blocks)
  EncodeTArgs t;
  size_t t_lds;
  unsigned t_blocks;
};

int plan_encode(const palu_layer_desc* desc, bool do_k, bool do_v, const void* x, int32_t n_tok,
                const void* Ak, const void* Av, void* hk, int64_t hk_stride, void* hv, int64_t hv_stride,
                const int32_t* dst_row, void* workspace, size_t workspace_bytes, EncodePlan* p) {
  Meta m;
  const int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  if (!x || n_tok <= 0) return PALU_ERR_INVALID_ARG;
  if (n_tok < kEncodeGemmTokens && (!workspace || (reinterpret_cast<uintptr_t>(workspace) & 15))) return PALU_ERR_INVALID_ARG;
  const int d = m.n_heads * PALU_D_HEAD;
  p->gemm = n_tok >= kEncodeGemmTokens;
  if (reinterpret_cast<uintptr_t>(x) & 15) return PALU_ERR_INVALID_ARG;
  p->transposed = false;
  EncodeArgs& a = p->a;
  std::memset(&a, 0, sizeof(a));
  a.x = static_cast<const uint16_t*>(x);
  a.dst_row = dst_row;
  a.n_tok = n_tok;
  a.d = d;
  a.k_splits = p->gemm ? 0 : d / kEncRows;
  size_t off = 0;
  p->n_sides = 0;
  p->max_R = 0;
  for (int side = 0; side < 2; ++side) {
    if (!(side ? do_v : do_k)) continue;
    const void* A = side ? Av : Ak;
    void* lat = side ? hv : hk;
    const int64_t stride = side ? hv_stride : hk_stride;
    const int R = side ? m.v_off[m.n_groups] : m.k_off[m.n_groups];
    if (!A || !lat || stride < R || (stride & 1)) return PALU_ERR_INVALID_ARG;
    if ((reinterpret_cast<uintptr_t>(A) & 15) || (reinterpret_cast<uintptr_t>(lat) & 3)) return PALU_ERR_INVALID_ARG;
    EncodeSide& sd = a.side[p->n_sides++];
    sd.A = static_cast<const uint16_t*>(A);
    sd.partial = reinterpret_cast<float*>(static_cast<unsigned char*>(workspace) + off);
    sd.latent = static_cast<uint16_t*>(lat);
    sd.row_stride = stride;
    sd.R = R;
    off += align_up((size_t)a.k_splits * n_tok * R * 4);
    p->max_R = std::max(p->max_R, R);
  }
  if (workspace_bytes < off) return PALU_ERR_WORKSPACE_TOO_SMALL;
  p->tok_cls = n_tok >= 5 ? 3 : (n_tok >= 3 ? 2 : (n_tok == 2 ? 1 : 0));
  return PALU_OK;
}

// The same for transposed weights (Akt [R_k, d], Avt [R_v, d]), both sides, fewer than kEncodeGemmTokens tokens.
int plan_encode_t(const palu_layer_desc* desc, const void* x, int32_t n_tok, const void* Akt, const void* Avt,
                  void* hk, int64_t hk_stride, void* hv, int64_t hv_stride, const int32_t* dst_row, EncodePlan* p) {
  Meta m;
  const int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  if (!x || !Akt || !Avt || !hk || !hv || n_tok <= 0) return PALU_ERR_INVALID_ARG;
  if (n_tok >= kEncodeGemmTokens) return PALU_ERR_UNSUPPORTED;
  if (latent_bits(desc->k_latent_dtype) || latent_bits(desc->v_latent_dtype)) return PALU_ERR_UNSUPPORTED;
  const int d = m.n_heads * PALU_D_HEAD;
  const int Rk = m.k_off[m.n_groups], Rv = m.v_off[m.n_groups];
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(Akt) & 15) || (reinterpret_cast<uintptr_t>(Avt) & 15) ||
      (reinterpret_cast<uintptr_t>(hk) & 1) || (reinterpret_cast<uintptr_t>(hv) & 1) || hk_stride < Rk || hv_stride < Rv)
    return PALU_ERR_INVALID_ARG;
  std::memset(&p->a, 0, sizeof(p->a));
  p->gemm = false;
  p->transposed = true;
  p->n_sides = 2;
  p->max_R = std::max(Rk, Rv);
  EncodeTArgs& a = p->t;
  a.x = static_cast<const uint16_t*>(x);
  a.dst_row = dst_row;
  a.At[0] = static_cast<const uint16_t*>(Akt);
  a.At[1] = static_cast<const uint16_t*>(Avt);
  a.latent[0] = static_cast<uint16_t*>(hk);
  a.latent[1] = static_cast<uint16_t*>(hv);
  a.row_stride[0] = hk_stride;
  a.row_stride[1] = hv_stride;
  a.R[0] = Rk;
  a.R[1] = Rv;
  a.n_tok = n_tok;
  a.d = d;
  // tokens per pass over the weights: as many as n_tok asks for, up to 8, while their activations fit 64 KiB of LDS
  int tok = 1, cls = 0;
  while (tok < 8 && tok < n_tok && (size_t)(2 * tok) * d * 2 <= 64 * 1024) tok <<= 1, ++cls;
  if ((size_t)tok * d * 2 > 64 * 1024) return PALU_ERR_UNSUPPORTED;
  p->tok_cls = cls;
  p->t_lds = tok <= 2 ? 0 : (size_t)tok * d * 2;      // one or two tokens per pass stay in registers
  a.wg_side1 = ceil_div(Rk, 4 * kTCols);
  p->t_blocks = (unsigned)(a.wg_side1 + ceil_div(Rv, 4 * kTCols));
  return PALU_OK;
}

// grid of the projection's first (transposed weights: only) launch: (column blocks, k splits, sides)
void encode_partial_grid(const EncodePlan& p, unsigned g[3]) {
  if (p.transposed) {
    g[0] = p.t_blocks;
    g[1] = g[2] = 1;
    return;
  }
  g[0] = (unsigned)ceil_div(p.max_R, kEncCols);
  g[1] = (unsigned)p.a.k_splits;
  g[2] = (unsigned)p.n_sides;
}

// second launch of the split-K form: sum the partials, round, scatter the rows
int launch_encode_finish(int act, const EncodePlan& p, hipStream_t s) {
  if (p.transposed) return PALU_OK;         // nothing left to sum
  const dim3 g2((unsigned)ceil_div(p.max_R, 64), (unsigned)p.a.n_tok, (unsigned)p.n_sides);
  if (act == PALU_F16) hipLaunchKernelGGL(encode_finish_kernel<F16>, g2, dim3(256), 0, s, p.a);
  else hipLaunchKernelGGL(encode_finish_kernel<BF16>, g2, dim3(256), 0, s, p.a);
  return launch_ok();
}

int launch_encode_gemm(int act, const EncodeArgs& a, int max_R, int n_sides, bool quant, hipStream_t s) {
  return launch_encode_gemm_tiles(act, a, max_R, n_sides, quant, (int)g_opt_encode_tile, device_cu_count(), s);
}

int launch_encode(int act, const EncodePlan& p, hipStream_t s) {
  const EncodeArgs& a = p.a;
  if (p.gemm) return launch_encode_gemm(act, a, p.max_R, p.n_sides, false, s);
  if (p.transposed) {
    using EncTFn = void (*)(EncodeTArgs);
    static const EncTFn t_f16[4] = {encode_t_kernel<F16, 1>, encode_t_kernel<F16, 2>, encode_t_kernel<F16, 4>, encode_t_kernel<F16, 8>};
    static const EncTFn t_bf16[4] = {encode_t_kernel<BF16, 1>, encode_t_kernel<BF16, 2>, encode_t_kernel<BF16, 4>, encode_t_kernel<BF16, 8>};
    hipLaunchKernelGGL(act == PALU_F16 ? t_f16[p.tok_cls] : t_bf16[p.tok_cls], dim3(p.t_blocks), dim3(256), p.t_lds, s, p.t);
    return launch_ok();
  }
  using EncFn = void (*)(EncodeArgs);
  static const EncFn partial_f16[4] = {encode_partial_kernel<F16, 1>, encode_partial_kernel<F16, 2>,
                                       encode_partial_kernel<F16, 4>, encode_partial_kernel<F16, 8>};
  static const EncFn partial_bf16[4] = {encode_partial_kernel<BF16, 1>, encode_partial_kernel<BF16, 2>,
                                        encode_partial_kernel<BF16, 4>, encode_partial_kernel<BF16, 8>};
  unsigned g1[3];
  encode_partial_grid(p, g1);
  hipLaunchKernelGGL(act == PALU_F16 ? partial_f16[p.tok_cls] : partial_bf16[p.tok_cls], dim3(g1[0], g1[1], g1[2]), dim3(256), 0, s, a);
  if (launch_ok() != PALU_OK) return PALU_ERR_HIP;
  return launch_encode_finish(act, p, s);
}

int encode_impl(const palu_layer_desc* desc, bool do_k, bool do_v, const void* x, int32_t n_tok,
                const void* Ak, const void* Av, void* hk, int64_t hk_stride, void* hv, int64_t hv_stride,
                const int32_t* dst_row, void* workspace, size_t workspace_bytes, void* stream) {
  EncodePlan p;
  const int st = plan_encode(desc, do_k, do_v, x, n_tok, Ak, Av, hk, hk_stride, hv, hv_stride, dst_row, workspace,
                             workspace_bytes, &p);
  if (st != PALU_OK) return st;
  return launch_encode(desc->act_dtype, p, static_cast<hipStream_t>(stream));
}

}  // namespace

int palu_encode(const palu_layer_desc* desc, int which, const void* x, int32_t n_tok, const void* A,
                void* latent, int64_t row_stride_elems, const int32_t* dst_row,
                void* workspace, size_t workspace_bytes, void* stream) {
  if (which != 0 && which != 1) return PALU_ERR_INVALID_ARG;
  return encode_impl(desc, which == 0, which == 1, x, n_tok, A, A, latent, row_stride_elems, latent,
                     row_stride_elems, dst_row, workspace, workspace_bytes, stream);
}

int palu_encode_kv(const palu_layer_desc* desc, const void* x, int32_t n_tok, const void* Ak, const void* Av,
                   void* hk, int64_t hk_row_stride_elems, void* hv, int64_t hv_row_stride_elems,
                   const int32_t* dst_row, void* workspace, size_t workspace_bytes, void* stream) {
  return encode_impl(desc, true, true, x, n_tok, Ak, Av, hk, hk_row_stride_elems, hv, hv_row_stride_elems,
                     dst_row, workspace, workspace_bytes, stream);
}

int palu_encode_kv_t(const palu_layer_desc* desc, const void* x, int32_t n_tok, const void* Akt, const void* Avt,
                     void* hk, int64_t hk_row_stride_elems, void* hv, int64_t hv_row_stride_elems,
                     const int32_t* dst_row, void* stream) {
  if (!desc) return PALU_ERR_INVALID_ARG;
  static thread_local EncodePlan p;
  const int st = plan_encode_t(desc, x, n_tok, Akt, Avt, hk, hk_row_stride_elems, hv, hv_row_stride_elems, dst_row, &p);
  if (st != PALU_OK) return st;
  return launch_encode(desc->act_dtype, p, static_cast<hipStream_t>(stream));
}

int palu_encode_quant(const palu_layer_desc* desc, int which, const void* x, int32_t n_tok, const void* A,
                      uint8_t* codes, void* scale, void* zero, const int32_t* dst_row, void* stream) {
  Meta m;
  const int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  if (!x || !A || !codes || !scale || !zero || n_tok <= 0 || (which != 0 && which != 1)) return PALU_ERR_INVALID_ARG;
  if (desc->quant_block <= 0) return PALU_ERR_INVALID_ARG;
  if (desc->quant_block != 128) return PALU_ERR_UNSUPPORTED;
  const int R = which ? m.v_off[m.n_groups] : m.k_off[m.n_groups];
  if (R % 128 != 0) return PALU_ERR_INVALID_ARG;
  const int side_bits = latent_bits(which ? desc->v_latent_dtype : desc->k_latent_dtype);
  if (side_bits != 0 && side_bits != 4) return PALU_ERR_UNSUPPORTED;      // the fused write-out packs 4-bit codes only
  if ((reinterpret_cast<uintptr_t>(x) & 15) || (reinterpret_cast<uintptr_t>(A) & 15) ||
      (reinterpret_cast<uintptr_t>(codes) & 15) || (reinterpret_cast<uintptr_t>(scale) & 1) ||
      (reinterpret_cast<uintptr_t>(zero) & 1))
    return PALU_ERR_INVALID_ARG;
  EncodeArgs a;
  std::memset(&a, 0, sizeof(a));
  a.x = static_cast<const uint16_t*>(x);
  a.dst_row = dst_row;
  a.n_tok = n_tok;
  a.d = m.n_heads * PALU_D_HEAD;
  a.side[0].A = static_cast<const uint16_t*>(A);
  a.side[0].R = R;
  a.side[0].codes = codes;
  a.side[0].scale = static_cast<uint16_t*>(scale);
  a.side[0].zero = static_cast<uint16_t*>(zero);
  return launch_encode_gemm(desc->act_dtype, a, R, 1, true, static_cast<hipStream_t>(stream));
}

// ------------------------------------------------------------------ quantize
int palu_quant_latent(const palu_layer_desc* desc, int which, const void* latent, int64_t row_stride_elems,
                      int32_t n_tok, uint8_t* codes, void* scale, void* zero, const int32_t* dst_row,
                      void* stream) {
  Meta m;
  const int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  if (!latent || !codes || !scale || !zero || n_tok <= 0 || (which != 0 && which != 1)) return PALU_ERR_INVALID_ARG;
  if (desc->quant_block <= 0) return PALU_ERR_INVALID_ARG;
  if (desc->quant_block != 128) return PALU_ERR_UNSUPPORTED;
  const int R = which ? m.v_off[m.n_groups] : m.k_off[m.n_groups];
  if (R % desc->quant_block != 0) return PALU_ERR_INVALID_ARG;
  if (row_stride_elems < R || (row_stride_elems & 1) || (reinterpret_cast<uintptr_t>(latent) & 3))
    return PALU_ERR_INVALID_ARG;
  QuantArgs a;
  a.latent = static_cast<const uint16_t*>(latent);
  a.codes = codes;
  a.scale = static_cast<uint16_t*>(scale);
  a.zero = static_cast<uint16_t*>(zero);
  a.dst_row = dst_row;
  a.row_stride = row_stride_elems;
  a.n_tok = n_tok;
  a.R = R;
  a.n_blocks = R / 128;
  a.bits = latent_bits(which ? desc->v_latent_dtype : desc->k_latent_dtype);
  if (a.bits == 0) a.bits = 4;
  const long long items = (long long)n_tok * a.n_blocks;
  const dim3 g((unsigned)((items + 3) / 4));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (desc->act_dtype == PALU_F16) hipLaunchKernelGGL(quant_kernel<F16>, g, dim3(256), 0, s, a);
  else hipLaunchKernelGGL(quant_kernel<BF16>, g, dim3(256), 0, s, a);
  return launch_ok();
}

// ------------------------------------------------------------------ decode
static int decode_workspace_bytes(const palu_layer_desc* desc, int32_t batch, int32_t n_q, int32_t max_seq, size_t* out_bytes) {
  Meta m;
  int st = check_desc(desc, &m, n_q);
  if (st != PALU_OK) return st;
  if (!out_bytes || batch <= 0 || max_seq <= 0) return PALU_ERR_INVALID_ARG;
  ScorePlan sp;
  PvPlan pp;
  const int kb = latent_bits(desc->k_latent_dtype);
  if ((st = plan_score(m, &sp, !(kb == 2 || kb == 3))) != PALU_OK) return st;
  if ((st = plan_pv(m, &pp)) != PALU_OK) return st;
  Workspace w;
  carve(m, batch, max_seq, split_bound(pp.total_units, batch, max_seq, value_waves_per_cu(desc)), 2 * sp.max_slices,
        !(desc->rope_theta > 0.f), &w);
  *out_bytes = w.total;
  return PALU_OK;
}

int palu_attn_decode_workspace_bytes(const palu_layer_desc* desc, int32_t batch, int32_t max_seq, size_t* out_bytes) {
  return decode_workspace_bytes(desc, batch, 1, max_seq, out_bytes);
}

int palu_attn_decode_multi_workspace_bytes(const palu_layer_desc* desc, int32_t batch, int32_t n_q, int32_t max_seq,
                                           size_t* out_bytes) {
  return decode_workspace_bytes(desc, batch, n_q, max_seq, out_bytes);
}

// out: attention output after B_v; out_latent: output left in the value latent space (then Bv is not read).
// n_q queries per sequence (q_pos has batch * n_q entries); q_len: rows attended per query, or NULL (all of the sequence's).
static int decode_impl(const palu_layer_desc* desc, int32_t batch, int32_t n_q, const int32_t* q_len,
                       int32_t seq_len, int32_t max_seq,
                       const void* q, const int32_t* q_pos,
                       const void* hk, const void* hk_scale, const void* hk_zero,
                       const void* hv, const void* hv_scale, const void* hv_zero,
                       const int32_t* k_pos, const int32_t* seq_lens,
                       const void* Bk, const void* Bv,
                       const void* rope_table, int32_t rope_table_len,
                       float* out, float* out_latent, void* workspace, size_t workspace_bytes, void* stream,
                       void* const* stage_events, const EncodePlan* enc = nullptr) {
  // enc: the step's down-projection of the new token (validated by the caller), launched from here:
  // ahead of everything else, or, where the step folds the query into B_k, in one grid with that fold
  Meta m;
  int st = check_desc(desc, &m, n_q);
  if (st != PALU_OK) return st;
  if (n_q > 1 && out_latent) return PALU_ERR_UNSUPPORTED;
  if (batch <= 0 || seq_len <= 0 || max_seq < seq_len) return PALU_ERR_INVALID_ARG;
  if (batch > 65535) return PALU_ERR_UNSUPPORTED;      // the batch index is a grid dimension
  if (!q || !q_pos || !hk || !hv || !Bk || !rope_table || !workspace) return PALU_ERR_INVALID_ARG;
  if (out_latent ? (out != nullptr) : (!out || !Bv)) return PALU_ERR_INVALID_ARG;
  const int k_bits = latent_bits(desc->k_latent_dtype), v_bits = latent_bits(desc->v_latent_dtype);
  const bool k_i4 = k_bits != 0, v_i4 = v_bits != 0;          // quantized sides (4, 3 or 2 bits)
  if (k_i4 && (!hk_scale || !hk_zero)) return PALU_ERR_INVALID_ARG;
  if (v_i4 && (!hv_scale || !hv_zero)) return PALU_ERR_INVALID_ARG;
  if (rope_table_len <= 0 || (!k_pos && rope_table_len < seq_len)) return PALU_ERR_INVALID_ARG;
  for (const void* p : {hk, hv, Bk, Bv, rope_table, (const void*)workspace, (const void*)out_latent})
    if (reinterpret_cast<uintptr_t>(p) & 15) return PALU_ERR_INVALID_ARG;
  const int Rk = m.k_off[m.n_groups], Rv = m.v_off[m.n_groups];
  if ((Rk % 8) || (Rv % 8)) return PALU_ERR_INVALID_ARG;

  ScorePlan sp;
  PvPlan pp;
  const bool k_lowbit = k_bits == 2 || k_bits == 3;        // their score kernels take one group per workgroup
  // unquantized latents, one query per wavefront's head: every head of rank 64 and more runs on the whole-head kernel
  // (ranks above 256 in slices); the shared-key form, which leaves it, only takes layers without such ranks
  // (not with option score_fp8, whose weights are laid out per whole head)
  const bool split16 = !k_i4 && g_opt_score_waves == 0 && g_opt_score_fp8 == 0;
  if ((st = plan_score(m, &sp, !k_lowbit, split16)) != PALU_OK) return st;
  if ((st = plan_pv(m, &pp)) != PALU_OK) return st;
  const int quant_block = desc->quant_block > 0 ? desc->quant_block : 128;
  int split_tokens, n_split;
  int max_unit_heads = 0;
  for (int i = 0; i < pp.total_units; ++i) max_unit_heads = std::max(max_unit_heads, (int)pp.units[i].nh);
  split_geometry(pp.total_units, batch, seq_len, value_waves_per_cu(desc), max_unit_heads, &split_tokens, &n_split);
  if (n_split > kMaxSplits) return PALU_ERR_UNSUPPORTED;
  // the value and no-RoPE kernels address a split of the cache with 32-bit byte offsets
  if ((long long)split_tokens * std::max(Rk, Rv) * 2 >= (1LL << 32)) return PALU_ERR_UNSUPPORTED;
  const int n_split_cap = split_bound(pp.total_units, batch, max_seq, value_waves_per_cu(desc));
  Workspace w;
  const bool no_rope = !(desc->rope_theta > 0.f);
  carve(m, batch, max_seq, n_split_cap, 2 * sp.max_slices, no_rope, &w);
  if (n_split > n_split_cap) return PALU_ERR_INVALID_ARG;
  if (workspace_bytes < w.total) return PALU_ERR_WORKSPACE_TOO_SMALL;

  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const int act = desc->act_dtype;
  const bool waves8 = g_opt_score_waves != 4 || k_lowbit;
  auto mark = [&](int i) -> int {
    if (!stage_events) return PALU_OK;
    return hipEventRecord(static_cast<hipEvent_t>(stage_events[i]), s) == hipSuccess ? PALU_OK : PALU_ERR_HIP;
  };
  if (stage_events)
    for (int i = 0; i <= PALU_DECODE_STAGES; ++i)
      if (!stage_events[i]) return PALU_ERR_INVALID_ARG;

  bool enc_pending = enc != nullptr;
  bool used16 = false, used4 = false;
  if (enc_pending && enc->gemm) {
    if ((st = launch_encode(act, *enc, s)) != PALU_OK) return st;
    enc_pending = false;
  }
  if (no_rope) {
    // 1'. fold the query into the latent space (Eq. 5); 2'. scores straight from the latents
    QkPlan qp;
    if ((st = plan_qk(m, k_i4, &qp)) != PALU_OK) return st;
    if (qp.qt_elems > w.mfold_bstride) return PALU_ERR_UNSUPPORTED;     // the folded queries reuse the folded-weight region
    QfoldArgs f;
    f.q = static_cast<const uint16_t*>(q);
    f.Bk = static_cast<const uint16_t*>(Bk);
    f.qt = reinterpret_cast<uint16_t*>(ws + w.mfold);
    f.qsum = reinterpret_cast<float*>(ws + w.qsum);
    f.qt_bstride = w.mfold_bstride;
    f.qs_bstride = (long long)m.n_heads * (PALU_MAX_RANK / 128 + 2);
    if (qp.qs_elems > f.qs_bstride) return PALU_ERR_UNSUPPORTED;
    f.meta = m;
    QkArgs a;
    a.hk = hk;
    a.hk_scale = static_cast<const uint16_t*>(hk_scale);
    a.hk_zero = static_cast<const uint16_t*>(hk_zero);
    a.qt = f.qt;
    a.qsum = f.qsum;
    a.seq_lens = seq_lens;
    a.scores = reinterpret_cast<float*>(ws + w.scores);
    a.qt_bstride = f.qt_bstride;
    a.qs_bstride = f.qs_bstride;
    a.row_elems = Rk;
    a.max_seq = max_seq;
    a.seq_len = seq_len;
    a.lpad = w.lpad;
    a.batch = batch;
    a.n_heads = m.n_heads;
    a.n_blocks_q = Rk / quant_block;
    a.scale = 1.4426950408889634f / std::sqrt((float)PALU_D_HEAD);
    {   // tokens per wavefront: four wavefronts per compute unit, 64 to 512 tokens
      const long long items = std::max(1, qp.total_units * batch);
      const long long waves_per_cu = k_i4 ? 8 : 4;
      long long stq = ceil_div((int)std::min<long long>(items * seq_len / (waves_per_cu * device_cu_count()) + 1, 1 << 30), 32) * 32LL;
      stq = std::min<long long>(std::max<long long>(stq, kPvSplitMin), kPvSplitMax);
      a.split_tokens = (int)stq;
      a.n_split = ceil_div(seq_len, (int)stq);
    }
    if ((st = mark(0)) != PALU_OK) return st;
    f.batch = batch;
    for (int i0 = 0; i0 < qp.total_units; i0 += kMaxQkUnits) {     // launches of up to 64 units; heads of other units idle
      f.units.n_units = std::min(kMaxQkUnits, qp.total_units - i0);
      int wmax = 0, h_lo = m.n_heads, h_hi = 0;
      std::memset(f.unit_of_head, 0, sizeof(f.unit_of_head));
      for (int i = 0; i < f.units.n_units; ++i) {
        const QkUnit& x = f.units.u[i] = qp.units[i0 + i];
        wmax = std::max(wmax, (int)x.wpad);
        for (int h = x.h0; h < x.h0 + x.nh; ++h) f.unit_of_head[h] = (uint8_t)i;
        h_lo = std::min(h_lo, (int)x.h0);
        h_hi = std::max(h_hi, x.h0 + x.nh);
      }
      f.head0 = h_lo;
      const dim3 g((unsigned)(wmax / 128), (unsigned)(h_hi - h_lo), (unsigned)ceil_div(batch, 4));
      unsigned gq[3] = {0, 0, 0};
      if (enc_pending) encode_partial_grid(*enc, gq);
      if (enc_pending && (long long)g.x * g.y * g.z > (long long)gq[0] * gq[1] * gq[2]) {     // more items than workgroups to ride in
        if ((st = launch_encode(act, *enc, s)) != PALU_OK) return st;
        enc_pending = false;
      }
      if (enc_pending) {
        // the new token's partial products with the query fold in their shadow, then the projection's second launch
        static thread_local StepHeadNoRopeArgs hn;
        hn.enc = enc->a;
        hn.enc_t = enc->t;
        hn.qfold = f;
        hn.q_gx = (int)g.x;
        hn.q_gy = (int)g.y;
        hn.q_blocks = (int)(g.x * g.y * g.z);
        unsigned ge[3];
        encode_partial_grid(*enc, ge);
        hn.enc_gx = (int)ge[0];
        hn.enc_gy = (int)ge[1];
        hn.enc_blocks = (int)(ge[0] * ge[1] * ge[2]);
        const StepHeadNoRopeFn hfn = step_head_norope_fn(act, enc->tok_cls, enc->transposed);
        const size_t hlds = enc->transposed ? enc->t_lds : 0;
        if ((st = allow_dynamic_lds(hfn, hlds)) != PALU_OK) return st;
        hipLaunchKernelGGL(hfn, dim3((unsigned)std::max(hn.q_blocks, hn.enc_blocks)), dim3(256), hlds, s, hn);
        if ((st = launch_ok()) != PALU_OK) return st;
        if ((st = launch_encode_finish(act, *enc, s)) != PALU_OK) return st;
        enc_pending = false;
      } else {
        if (act == PALU_F16) hipLaunchKernelGGL(qfold_kernel<F16>, g, dim3(256), 0, s, f);
        else hipLaunchKernelGGL(qfold_kernel<BF16>, g, dim3(256), 0, s, f);
        if ((st = launch_ok()) != PALU_OK) return st;
      }
    }
    if ((st = mark(1)) != PALU_OK) return st;
    for (int cls = 0; cls < 2; ++cls) {              // 0: up to 16 heads per unit, 1: up to 32
      using QkFn = void (*)(QkArgs);
      QkFn fn = k_bits == 4 ? (cls ? qk_kernel<F16, 2, 4> : qk_kernel<F16, 1, 4>)
              : k_bits == 3 ? (cls ? qk_kernel<F16, 2, 3> : qk_kernel<F16, 1, 3>)
              : k_bits == 2 ? (cls ? qk_kernel<F16, 2, 2> : qk_kernel<F16, 1, 2>)
              : act == PALU_F16 ? (cls ? qk_kernel<F16, 2, 0> : qk_kernel<F16, 1, 0>)
                                : (cls ? qk_kernel<BF16, 2, 0> : qk_kernel<BF16, 1, 0>);
      const size_t lds1 = align_up(qp.max_lds[cls], 16);     // one unit's staged folded queries
      if (lds1 == 0) continue;
      auto flush = [&]() -> int {
        if (a.units.n_units == 0) return PALU_OK;
        // quantized latents: as many units per workgroup (4, 2 or 1) as the launch has and as fit 64 KiB of LDS, two
        // workgroups to a compute unit (the units then share the cache lines of their tokens' scales and zero-points;
        // unquantized latents have nothing to share and measured faster with one unit's staging per workgroup)
        int upw = k_bits == 0 ? 1 : (a.units.n_units >= 4 ? 4 : (a.units.n_units >= 2 ? 2 : 1));
        while (upw > 1 && lds1 * upw > 64 * 1024) upw >>= 1;
        a.units_per_wg = upw;
        a.lds_unit_stride = (int)lds1;
        const size_t lds = lds1 * upw;
        int rc = allow_lds(fn, lds);
        if (rc != PALU_OK) return rc;
        const dim3 grid((unsigned)ceil_div(a.units.n_units, upw), (unsigned)ceil_div(a.n_split, 4 / upw), (unsigned)batch);
        hipLaunchKernelGGL(fn, grid, dim3(256), lds, s, a);
        a.units.n_units = 0;
        return launch_ok();
      };
      a.units.n_units = 0;
      for (int i = 0; i < qp.total_units; ++i) {
        if ((qp.units[i].nh > 16 ? 1 : 0) != cls) continue;
        a.units.u[a.units.n_units++] = qp.units[i];
        if (a.units.n_units == kMaxQkUnits && (st = flush()) != PALU_OK) return st;
      }
      if ((st = flush()) != PALU_OK) return st;
    }
  } else {
    // 2 .. 16 queries per key/value head (grouped-query heads times queries per sequence) with fp16
    // latents and ranks up to 256: the score kernel rebuilds each key once for the queries that
    // share it (shared-key form).  Otherwise every query head rebuilds its key/value head's keys (one-query form).
    bool shared_key = g_opt_shared_key_fp16 != 0 && m.qpk >= 2 && m.qpk <= 16 && act == PALU_F16 && !k_i4 && waves8;
    for (int j = 0; j < m.n_groups && shared_key; ++j) shared_key = m.k_off[j + 1] - m.k_off[j] <= 256;
    // unquantized latents, one query per head: heads of rank 64 .. 256 run one whole head per wavefront
    // (option score_waves = 4 or 8 forces the half-head / ping-pong schedules of score_kernel)
    const bool use16 = !shared_key && !k_i4 && g_opt_score_waves == 0;
    // ... and with 2, 4 or 8 queries per key/value head and ranks 128 .. 256 one whole key/value head per wavefront:
    // the key is rebuilt and rotated once in float32 for the queries that share it (exact shared-key form)
    bool shared16 = use16 && m.qpk > 1 && g_opt_score_fp8 == 0;
    int sk_pass_rows = 8;
    for (int j = 0; j < m.n_groups && shared16; ++j) {
      const int r = m.k_off[j + 1] - m.k_off[j];
      // ranks 288 .. 512 run as two slices of 128 .. 256 rows (plan_score), each a unit of its own rank class
      const int r0 = (r > 256 && r <= 512 && split16) ? (r + 63) / 64 * 32 : r;
      for (int rs : {r0, r - r0}) {
        if (rs == 0) continue;
        const int rcj = rank_class(rs);
        shared16 = shared16 && shared16_ok(rcj);
        if (shared16) sk_pass_rows = std::min(sk_pass_rows, shared16_rows_per_pass(rcj));
      }
    }
    // the same with 4-bit keys (blocks of 128 channels, ranks 128 and 256): their tiles are dequantized once per pass
    // for the queries that share them
    bool shared4 = !shared_key && k_bits == 4 && quant_block == 128 && m.qpk > 1 && g_opt_score_waves == 0;
    for (int j = 0; j < m.n_groups && shared4; ++j) {
      const int r = m.k_off[j + 1] - m.k_off[j];
      shared4 = r == 128 || r == 256;
      if (shared4) sk_pass_rows = std::min(sk_pass_rows, r == 256 ? 8 : 4);
    }
    used4 = shared4;
    const bool kv_units = shared_key || shared16 || shared4;   // the score units are key/value heads
    const Meta mk = kv_units ? kv_head_meta(m) : m;
    used16 = use16;
    // option score_fp8: those heads rebuild their keys from E4M3-rounded latents and weights (fp16 layers)
    const bool use8 = use16 && g_opt_score_fp8 != 0 && act == PALU_F16;
    if (use16) {
      // the 256-row slices of ranks above 512 run there too and write one score plane each (the planned two are
      // those of the half-head wavefronts)
      for (int i = 0; i < sp.total_units; ++i)
        if (sp.cls_id[sp.unit_cls[i]] == kSlicedCls) sp.units[i].part0 /= 2;
    }
    static thread_local ScorePlan spk;                 // units over key/value heads (shared-key form only)
    if (kv_units && (st = plan_score(mk, &spk, false, shared16 && split16)) != PALU_OK) return st;
    const ScorePlan& plan = kv_units ? spk : sp;

    // 1. B_k in the score kernel's operand order (shared-key form: and the rotated queries beside it)
    static thread_local FoldArgs fa;
    {
      fa.Bk = static_cast<const uint16_t*>(Bk);
      fa.mfold = reinterpret_cast<uint16_t*>(ws + w.mfold);
      for (int f = 0; f < kHalf; ++f) {
        const double rev = desc->rope_theta > 0.f
            ? std::pow((double)desc->rope_theta, -2.0 * f / (double)PALU_D_HEAD) / 6.283185307179586476925 : 0.0;
        fa.rev_hi[f] = (float)rev;
        fa.rev_lo[f] = (float)(rev - (double)fa.rev_hi[f]);
      }
      fa.meta = mk;
      fa.layout16 = use16 ? (split16 ? 2 : 1) : (shared4 ? 1 : 0);
      int max_r = 0;
      for (int j = 0; j < m.n_groups; ++j) max_r = std::max(max_r, m.k_off[j + 1] - m.k_off[j]);
      const dim3 g((unsigned)(max_r / 16), (unsigned)mk.n_heads, 1u);
      if ((st = mark(0)) != PALU_OK) return st;
      // Fused only while every item finds a projection workgroup to ride in (the 7B shape: 512 items,
      // 512 workgroups); with more items than that they would dominate the launch.
      unsigned ge0[3] = {0, 0, 0};
      if (enc_pending) encode_partial_grid(*enc, ge0);
      const long long fold_items = (long long)g.x * g.y * g.z + (shared_key ? (long long)mk.n_heads * batch : 0);
      const bool fused_head = enc_pending && fold_items <= (long long)ge0[0] * ge0[1] * ge0[2];
      if (enc_pending && !fused_head) {
        if ((st = launch_encode(act, *enc, s)) != PALU_OK) return st;
        enc_pending = false;
      }
      if (fused_head) {
        // the new token's partial products and the fold in one grid, then the projection's second launch
        static thread_local StepHeadArgs h;
        h.enc = enc->a;
        h.enc_t = enc->t;
        h.fold = fa;
        h.fold_gx = (int)g.x;
        h.fold_blocks = (int)(g.x * g.y);
        unsigned ge[3];
        encode_partial_grid(*enc, ge);
        h.enc_gx = (int)ge[0];
        h.enc_gy = (int)ge[1];
        h.enc_blocks = (int)(ge[0] * ge[1] * ge[2]);
        h.sk_q = nullptr;
        h.sk_blocks = 0;
        if (shared_key) {                  // the rotated-query operands of the shared-key form ride along too
          h.sk_q = static_cast<const uint16_t*>(q);
          h.sk_q_pos = q_pos;
          h.sk_qfrag = reinterpret_cast<uint16_t*>(ws + w.qfrag);
          h.sk_n_kv = mk.n_heads;
          h.sk_qpk = m.qpk;
          h.sk_nq = m.nq;
          h.sk_n_heads = m.n_heads;
          h.sk_small = m.qpk <= 4 ? 1 : 0;
          h.sk_blocks = mk.n_heads * batch;
        }
        const StepHeadFn hfn = step_head_fn(act, enc->tok_cls, enc->transposed);
        const size_t hlds = enc->transposed ? enc->t_lds : 0;
        if ((st = allow_dynamic_lds(hfn, hlds)) != PALU_OK) return st;
        hipLaunchKernelGGL(hfn, dim3((unsigned)std::max(h.fold_blocks + h.sk_blocks, h.enc_blocks)), dim3(256), hlds, s, h);
        if ((st = launch_ok()) != PALU_OK) return st;
        if ((st = launch_encode_finish(act, *enc, s)) != PALU_OK) return st;
        enc_pending = false;
      } else {
        hipLaunchKernelGGL(fold_kernel, g, dim3(256), 0, s, fa);
        if ((st = launch_ok()) != PALU_OK) return st;
      }
      if (shared_key && !fused_head) {
        QfragArgs qa;
        qa.q = static_cast<const uint16_t*>(q);
        qa.q_pos = q_pos;
        qa.qfrag = reinterpret_cast<uint16_t*>(ws + w.qfrag);
        qa.theta = desc->rope_theta;
        std::memcpy(qa.rev_hi, fa.rev_hi, sizeof(qa.rev_hi));
        std::memcpy(qa.rev_lo, fa.rev_lo, sizeof(qa.rev_lo));
        qa.n_kv = mk.n_heads;
        qa.qpk = m.qpk;
        qa.nq = m.nq;
        qa.n_heads = m.n_heads;
        qa.small = m.qpk <= 4 ? 1 : 0;
        hipLaunchKernelGGL(qfrag_kernel<F16>, dim3((unsigned)mk.n_heads, (unsigned)batch), dim3(256), 0, s, qa);
        if ((st = launch_ok()) != PALU_OK) return st;
      }
    }

    if (use8) {
      Fold8Args f8;
      f8.Bk = static_cast<const uint16_t*>(Bk);
      f8.w8 = ws + w.w8;
      f8.scale = reinterpret_cast<float*>(ws + w.w_scale);
      f8.meta = m;
      hipLaunchKernelGGL(fold8_kernel<F16>, dim3((unsigned)m.n_heads, 4u), dim3(256), 0, s, f8);
      if ((st = launch_ok()) != PALU_OK) return st;
    }

    // 2. scores
    {
      static thread_local ScoreArgs a;
      a.hk = hk;
      a.hk_scale = static_cast<const uint16_t*>(hk_scale);
      a.hk_zero = static_cast<const uint16_t*>(hk_zero);
      a.mfold = reinterpret_cast<const uint16_t*>(ws + w.mfold);
      a.w_scale = reinterpret_cast<const float*>(ws + w.w_scale);
      // the table's tiles: float32 part first, the shared-key form's float16 rows behind it
      a.rope_rows = static_cast<const unsigned char*>(rope_table) + (shared_key ? kRopeTileBytes : 0);
      a.rope_tile_stride = kRopeTableStride;
      a.q = static_cast<const uint16_t*>(q);
      a.q_pos = q_pos;
      a.m_qpk = m.qpk;
      a.m_nq = m.nq;
      std::memcpy(a.rev_hi, fa.rev_hi, sizeof(a.rev_hi));
      std::memcpy(a.rev_lo, fa.rev_lo, sizeof(a.rev_lo));
      a.seq_lens = seq_lens;
      a.scores = reinterpret_cast<float*>(ws + w.scores);
      a.mfold_bstride = 0;                                       // the weights do not depend on the sequence
      a.row_elems = Rk;
      a.max_seq = max_seq;
      a.seq_len = seq_len;
      a.lpad = w.lpad;
      a.batch = batch;
      a.n_heads = m.n_heads;
      a.quant_block = desc->quant_block > 0 ? desc->quant_block : 128;
      a.n_blocks_q = Rk / a.quant_block;
      a.bits = k_bits;
      a.scale = 1.4426950408889634f / std::sqrt((float)PALU_D_HEAD);
      a.qfrag = reinterpret_cast<const uint16_t*>(ws + w.qfrag);
      a.qpk = m.qpk;
      a.n_kv = mk.n_heads;
      if ((st = mark(1)) != PALU_OK) return st;
      if (k_pos) {
        // angles in cached-token order, so that the score kernel needs no position loads
        RopeGatherArgs g;
        g.table = rope_table;
        g.k_pos = k_pos;
        g.rows = ws + w.rope_rows;
        g.n = ceil_div(seq_len, 32) * 32;
        g.k_pos_len = max_seq;
        g.table_len = rope_table_len;
        if (shared_key) hipLaunchKernelGGL(rope_gather_kernel, dim3((unsigned)ceil_div(g.n * 16, 256)), dim3(256), 0, s, g);
        else hipLaunchKernelGGL(rope_gather_tiles_kernel, dim3((unsigned)ceil_div(g.n * 64, 256)), dim3(256), 0, s, g);
        if ((st = launch_ok()) != PALU_OK) return st;
        a.rope_rows = g.rows;
        a.rope_tile_stride = shared_key ? kRopeRowsBytes : kRopeTileBytes;
      }
      const int tiles = ceil_div(seq_len, kTile);
      // Sequence chunks per (sequence, unit): every launch (one per rank class) should fill
      // the chip by itself, since launches on one stream run one after the other.
      auto set_chunks = [&](int launch_units) {
        int n_chunks = std::max(1, std::min(tiles, (int)std::lround((double)device_cu_count() / (launch_units * batch))));
        if (g_opt_score_chunks > 0) n_chunks = std::min(tiles, (int)g_opt_score_chunks);
        // the kernel addresses a chunk of the cache with 32-bit byte offsets, and rows of it with 24-bit numbers
        // (and its angle tiles with 32-bit byte offsets)
        const long long chunk_limit_tiles = std::max(1LL, std::min<long long>({(1LL << 31) / ((long long)Rk * 2 * kTile), (1LL << 24) / kTile,
                                                                                 (1LL << 31) / kRopeTableStride}));
        n_chunks = std::max(n_chunks, (int)ceil_div(tiles, (int)std::min<long long>(chunk_limit_tiles, tiles)));
        const int chunk_tiles = ceil_div(tiles, n_chunks);
        a.chunk_tokens = chunk_tiles * kTile;
        a.n_chunks = ceil_div(tiles, chunk_tiles);
      };
      // Groups of different ranks, every class on the whole-head kernel with one group per workgroup: ONE launch
      // where one round of workgroups covers the layer.  Launches on one stream run one after the other and every
      // workgroup start costs several microseconds (the head's weights go to registers, the tile ring fills), so
      // a launch per class pays that once per class; here every workgroup has a compute unit to itself, starts
      // once, and the chunk lengths per class are chosen so that all of them end at about the same time.
      bool mixed = use16 && !shared16 && !shared4 && !use8 && g_opt_score_mixed != 0 && g_opt_score_chunks == 0 &&
                   plan.n_cls > 1 && plan.n_cls <= kMaxMixClasses && plan.total_units <= kMaxScoreUnits;
      for (int cls = 0; cls < plan.n_cls && mixed; ++cls) {
        const int id = plan.cls_id[cls];
        if (id == kSlicedCls || id % 3 != 0 || !rank_class_16(id / 3)) mixed = false;
      }
      int order[kMaxMixClasses], n_units_cls[kMaxMixClasses] = {}, one_round[kMaxMixClasses];
      bool use_one_round = false;
      double mix_per_wg = 0.0;
      long long mix_chunk_limit_tiles = 1;
      // measured (uniform layers of each rank, 2048- and 1024-token chunks with every compute unit busy): microseconds per
      // 1000 tokens of one workgroup by rank / 32
      static const double kCost[9] = {0, 0, 30, 34, 38, 43, 47, 53, 56};
      auto weight = [](int nk) { return kCost[nk]; };
      if (mixed) {
        constexpr double kStartUs = 7.5;                         // measured: a launch's start plus a workgroup's own (weights into registers, tile ring filled, last tile drained)
        for (int cls = 0; cls < plan.n_cls; ++cls) order[cls] = cls;
        std::sort(order, order + plan.n_cls, [&](int x, int y) { return plan.cls_id[x] > plan.cls_id[y]; });
        for (int i = 0; i < plan.total_units; ++i) ++n_units_cls[plan.unit_cls[i]];
        double work = 0.0;                                       // weighted tokens of the whole launch
        for (int cls = 0; cls < plan.n_cls; ++cls) work += weight(plan.cls_id[cls] / 3 + 1) * n_units_cls[cls] * (double)batch * seq_len;
        const int cus = device_cu_count();
        mix_per_wg = work / ((g_opt_score_mixed > 1 ? (double)g_opt_score_mixed : 3.0) * cus);
        const long long chunk_limit_tiles = mix_chunk_limit_tiles = std::max(1LL, std::min<long long>({(1LL << 31) / ((long long)Rk * 2 * kTile), (1LL << 24) / kTile,
                                                                                 (1LL << 31) / kRopeTableStride}));
        // One round where it fits: every workgroup has a compute unit to itself and starts once.  Chunks go, one at
        // a time, to the class whose workgroups would run longest, while the launch still fits the chip.
        if (g_opt_score_mixed == 1) {
          long long total = 0;
          for (int cls = 0; cls < plan.n_cls; ++cls) {
            one_round[cls] = (int)ceil_div(tiles, (int)std::min<long long>(tiles, chunk_limit_tiles));
            total += (long long)one_round[cls] * n_units_cls[cls] * batch;
          }
          auto wg_us = [&](int cls) { return kStartUs + ceil_div(tiles, one_round[cls]) * kTile * weight(plan.cls_id[cls] / 3 + 1) * 1e-3; };
          while (total <= cus) {
            int worst = 0;
            for (int cls = 1; cls < plan.n_cls; ++cls) if (wg_us(cls) > wg_us(worst)) worst = cls;
            const long long more = (long long)n_units_cls[worst] * batch;
            if (one_round[worst] >= tiles || total + more > cus) break;
            ++one_round[worst];
            total += more;
          }
          double t1 = 0.0;
          for (int cls = 0; cls < plan.n_cls; ++cls) t1 = std::max(t1, wg_us(cls));
          const double t3 = 1.1 * (work * 1e-3 / cus + 3.0 * kStartUs);                     // three rounds of workgroups, some imbalance
          use_one_round = total <= cus && t1 < t3;
          if (!use_one_round) mixed = false;      // several rounds of mixed workgroups measured no faster than a launch per class
        }
      }
      if (mixed) {
        a.units.n_units = 0;
        a.mix.n_cls = plan.n_cls;
        long long first = 0;
        size_t lds = 0;
        for (int x = 0; x < plan.n_cls; ++x) {
          const int cls = order[x], nk = plan.cls_id[cls] / 3 + 1;
          int chunk_tiles = (int)std::min<long long>(std::max<long long>(1, std::llround(mix_per_wg / weight(nk) / kTile)), std::min<long long>(tiles, mix_chunk_limit_tiles));
          const int n_chunks = use_one_round ? one_round[cls] : ceil_div(tiles, chunk_tiles);
          chunk_tiles = ceil_div(tiles, n_chunks);               // chunks of equal length
          a.mix.first[x] = (int)first;
          a.mix.n_chunks[x] = ceil_div(tiles, chunk_tiles);
          a.mix.chunk_tokens[x] = chunk_tiles * kTile;
          a.mix.unit0[x] = a.units.n_units;
          a.mix.n_units[x] = n_units_cls[cls];
          a.mix.nk[x] = nk;
          for (int i = 0; i < plan.total_units; ++i)
            if (plan.unit_cls[i] == cls) a.units.u[a.units.n_units++] = plan.units[i];
          first += (long long)a.mix.n_chunks[x] * n_units_cls[cls] * batch;
          lds = std::max(lds, (size_t)score16_lds_bytes(32 * nk));
        }
        if (first >= (1LL << 31)) return PALU_ERR_UNSUPPORTED;
        ScoreFn fn = act == PALU_F16 ? score16_mixed_kernel<F16> : score16_mixed_kernel<BF16>;
        if ((st = allow_lds(fn, lds)) != PALU_OK) return st;
        a.mfold = reinterpret_cast<const uint16_t*>(ws + w.mfold);
        hipLaunchKernelGGL(fn, dim3((unsigned)first), dim3(256), lds, s, a);
        if ((st = launch_ok()) != PALU_OK) return st;
      }
      for (int cls = 0; cls < plan.n_cls && !mixed; ++cls) {
        const int id = plan.cls_id[cls];
        const bool sliced = id == kSlicedCls;
        const int rc = sliced ? rank_class(kSliceRank) : id / 3, lg = sliced ? 0 : id % 3;
        const int width = (32 * (rc + 1)) << lg;
        const bool dma = !k_i4;
        const bool pingpong = (waves8 && !rank_class_half(rc)) || shared_key;
        size_t lds = (size_t)score_lds_bytes(width, dma, !shared_key, pingpong);
        const bool k16 = use16 && rank_class_16(rc);
        ScoreFn fn = shared_key ? (m.qpk <= 4 ? score_fn_shared<1>(rc) : score_fn_shared<2>(rc))
                   : shared16 ? nullptr            // chosen per pass below
                   : k16 ? (act == PALU_F16 ? score16_fn_t<F16>(rc, lg) : score16_fn_t<BF16>(rc, lg))
                   : (k_lowbit ? score_fn_lowbit(rc) : score_fn(act, k_i4, rc * 3 + lg, waves8));
        if (k16) lds = (size_t)score16_lds_bytes(width);
        if (shared16 || shared4) {
          if (shared4) lds = (size_t)score16q4_lds_bytes(width);
          // exact shared-key form: passes of up to sk_pass_rows query rows of every key/value head, each pass one
          // launch per flush of units (the key tile is rebuilt once per pass)
          for (int row0 = 0; row0 < m.qpk; row0 += sk_pass_rows) {
            const int rows = std::min(sk_pass_rows, m.qpk - row0);
            fn = shared4 ? score16q4_fn(rc, rows)
                         : (act == PALU_F16 ? score16q_fn_t<F16>(rc, rows) : score16q_fn_t<BF16>(rc, rows));
            if (!fn) return PALU_ERR_UNSUPPORTED;
            if ((st = allow_lds(fn, lds)) != PALU_OK) return st;
            a.sk_row0 = row0;
            a.sk_rows = rows;
            a.mfold = reinterpret_cast<const uint16_t*>(ws + w.mfold);
            a.units.n_units = 0;
            auto flush_q = [&]() -> int {
              if (a.units.n_units == 0) return PALU_OK;
              set_chunks(a.units.n_units);
              const dim3 grid((unsigned)a.n_chunks, (unsigned)a.units.n_units, (unsigned)batch);
              hipLaunchKernelGGL(fn, grid, dim3(256), lds, s, a);
              a.units.n_units = 0;
              return launch_ok();
            };
            for (int i = 0; i < plan.total_units; ++i) {
              if (plan.unit_cls[i] != cls) continue;
              a.units.u[a.units.n_units++] = plan.units[i];
              if (a.units.n_units == kMaxScoreUnits && (st = flush_q()) != PALU_OK) return st;
            }
            if ((st = flush_q()) != PALU_OK) return st;
          }
          continue;
        }
        if (!fn) return PALU_ERR_UNSUPPORTED;
        const bool k8 = k16 && use8 && !sliced;
        if (k8) {
          fn = score8_fn(rc, lg);
          lds = (size_t)score8_lds_bytes(width);
          a.mfold = reinterpret_cast<const uint16_t*>(ws + w.w8);
        } else {
          a.mfold = reinterpret_cast<const uint16_t*>(ws + w.mfold);
        }
        if ((st = allow_lds(fn, lds)) != PALU_OK) return st;
        const unsigned threads = (waves8 && !rank_class_half(rc) && !k16) ? 512 : 256;
        auto flush = [&]() -> int {
          if (a.units.n_units == 0) return PALU_OK;
          set_chunks(a.units.n_units);
          const dim3 grid((unsigned)a.n_chunks, (unsigned)a.units.n_units, (unsigned)batch);
          hipLaunchKernelGGL(fn, grid, dim3(threads), lds, s, a);
          a.units.n_units = 0;
          return launch_ok();
        };
        a.units.n_units = 0;
        for (int i = 0; i < plan.total_units; ++i) {
          if (plan.unit_cls[i] != cls) continue;
          a.units.u[a.units.n_units++] = plan.units[i];
          if (a.units.n_units == kMaxScoreUnits && (st = flush()) != PALU_OK) return st;
        }
        if ((st = flush()) != PALU_OK) return st;
      }
    }
  }

  // 3. softmax partials and P.H_v per split
  uint8_t n_parts[PALU_MAX_HEADS];
  std::memset(n_parts, 0, sizeof(n_parts));
  int max_parts = 0;
  for (int h = 0; h < m.n_heads; ++h) {      // half-head wavefronts write two planes per rank slice
    const int rk = m.k_off[m.group_of_head[h] + 1] - m.k_off[m.group_of_head[h]];
    // one wavefront per head: one plane (per rank slice)
    const bool whole = used4 || (used16 && (split16 ? rk >= 64 : (rank_class_16(rank_class(rk)) || rk > 512)));
    n_parts[h] = no_rope ? (uint8_t)1 : (uint8_t)(((waves8 || sp.half_heads[h]) && !whole) ? 2 * sp.slices[h] : sp.slices[h]);
    max_parts = std::max(max_parts, (int)n_parts[h]);
  }
  if ((st = mark(2)) != PALU_OK) return st;
  {
    if (max_parts > 2) {                     // ranks contracted in slices: fold those heads' planes into plane 0
      PlaneSumArgs ps;
      ps.scores = reinterpret_cast<float*>(ws + w.scores);
      ps.part_stride = w.part_stride;
      ps.lpad = w.lpad;
      ps.seq_len = seq_len;
      ps.n_heads = m.n_heads;
      std::memcpy(ps.n_parts, n_parts, sizeof(n_parts));
      hipLaunchKernelGGL(plane_sum_kernel, dim3((unsigned)ceil_div(seq_len, 256), (unsigned)m.n_heads, (unsigned)batch),
                         dim3(256), 0, s, ps);
      if ((st = launch_ok()) != PALU_OK) return st;
    }
    PvArgs a;
    a.hv = hv;
    a.hv_scale = static_cast<const uint16_t*>(hv_scale);
    a.hv_zero = static_cast<const uint16_t*>(hv_zero);
    a.scores = reinterpret_cast<const float*>(ws + w.scores);
    a.seq_lens = seq_lens;
    a.q_len = q_len;
    a.o_part = reinterpret_cast<float*>(ws + w.o_part);
    a.ml_part = reinterpret_cast<float*>(ws + w.ml_part);
    a.row_elems = Rv;
    a.max_seq = max_seq;
    a.part_stride = w.part_stride;
    a.seq_len = seq_len;
    a.lpad = w.lpad;
    a.batch = batch;
    a.split_tokens = split_tokens;
    a.n_split = n_split;
    a.o_stride = w.o_stride;
    a.n_blocks_q = Rv / quant_block;
    bool two_planes = false;
    for (int h = 0; h < PALU_MAX_HEADS; ++h) {
      a.n_parts[h] = (uint8_t)(n_parts[h] > 2 ? 1 : n_parts[h]);
      two_planes |= a.n_parts[h] == 2;
    }
    a.meta = m;
    for (int cls = 0; cls < kNumPvCls; ++cls) {
      auto flush = [&]() -> int {
        if (a.units.n_units == 0) return PALU_OK;
        a.units_per_wg = a.units.n_units >= 4 ? 4 : (a.units.n_units >= 2 ? 2 : 1);
        const dim3 grid((unsigned)ceil_div(a.units.n_units, a.units_per_wg), (unsigned)ceil_div(n_split, 4 / a.units_per_wg),
                        (unsigned)batch);
        hipLaunchKernelGGL(pv_fn(act, v_bits, cls, two_planes), grid, dim3(256), 0, s, a);
        a.units.n_units = 0;
        return launch_ok();
      };
      a.units.n_units = 0;
      for (int i = 0; i < pp.total_units; ++i) {
        if (pp.unit_cls[i] != cls) continue;
        a.units.u[a.units.n_units++] = pp.units[i];
        if (a.units.n_units == kMaxPvUnits && (st = flush()) != PALU_OK) return st;
      }
      if ((st = flush()) != PALU_OK) return st;
    }
  }

  // 4. merge splits, normalise, apply B_v
  {
    CombineArgs a;
    a.o_part = reinterpret_cast<const float*>(ws + w.o_part);
    a.ml_part = reinterpret_cast<const float*>(ws + w.ml_part);
    a.Bv = static_cast<const uint16_t*>(Bv);
    a.seq_lens = seq_lens;
    a.out = out;
    a.out_latent = out_latent;
    a.n_split = n_split;
    a.split_tokens = split_tokens;
    a.seq_len = seq_len;
    a.o_stride = w.o_stride;
    a.meta = m;
    const dim3 g((unsigned)m.n_heads * 4, (unsigned)batch);
    if ((st = mark(3)) != PALU_OK) return st;
    if (act == PALU_F16) hipLaunchKernelGGL(combine_kernel<F16>, g, dim3(256), 0, s, a);
    else hipLaunchKernelGGL(combine_kernel<BF16>, g, dim3(256), 0, s, a);
    if ((st = launch_ok()) != PALU_OK) return st;
    if ((st = mark(4)) != PALU_OK) return st;
  }
  return PALU_OK;
}

int palu_attn_decode(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                     const void* q, const int32_t* q_pos,
                     const void* hk, const void* hk_scale, const void* hk_zero,
                     const void* hv, const void* hv_scale, const void* hv_zero,
                     const int32_t* k_pos, const int32_t* seq_lens,
                     const void* Bk, const void* Bv,
                     const void* rope_table, int32_t rope_table_len,
                     float* out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, hk_scale, hk_zero, hv, hv_scale, hv_zero, k_pos,
                     seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, workspace, workspace_bytes, stream, nullptr);
}

// ---- the decode step for callers that cannot allocate ---------------------------
// Its scratch is a file-scope device array: every GPU the library runs on holds its own
// copy at its own address, looked up once per device; host code only ever uses that
// address, never the array's name.
namespace {
static __device__ __align__(256) unsigned char scratch[PALU_NOALLOC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// address of `scratch` on the current device, or NULL
void* scratch_of_current_device() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p) return p;
  if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
    (void)hipGetLastError();
    return nullptr;
  }
  g_scratch_ptr[dev].store(p, std::memory_order_release);     // racing first calls look up the same address
  return p;
}
}  // namespace

int palu_attn_decode_noalloc(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                             const void* q, const int32_t* q_pos,
                             const void* hk, const void* hk_scale, const void* hk_zero,
                             const void* hv, const void* hv_scale, const void* hv_zero,
                             const int32_t* k_pos, const int32_t* seq_lens,
                             const void* Bk, const void* Bv,
                             const void* rope_table, int32_t rope_table_len,
                             float* out, void* stream) {
  size_t need = 0;
  const int st = decode_workspace_bytes(desc, batch, 1, max_seq, &need);
  if (st != PALU_OK) return st;
  if (need > (size_t)PALU_NOALLOC_SCRATCH_BYTES) return PALU_ERR_WORKSPACE_TOO_SMALL;
  void* ws = scratch_of_current_device();
  if (!ws) return PALU_ERR_HIP;
  // every region of the scratch is written by the step before it is read: nothing has to start at zero
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, hk_scale, hk_zero, hv, hv_scale, hv_zero, k_pos,
                     seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, ws, PALU_NOALLOC_SCRATCH_BYTES, stream,
                     nullptr);
}

int palu_attn_decode_staged(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                            const void* q, const int32_t* q_pos,
                            const void* hk, const void* hk_scale, const void* hk_zero,
                            const void* hv, const void* hv_scale, const void* hv_zero,
                            const int32_t* k_pos, const int32_t* seq_lens,
                            const void* Bk, const void* Bv,
                            const void* rope_table, int32_t rope_table_len,
                            float* out, void* workspace, size_t workspace_bytes, void* stream,
                            void* const* stage_events) {
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, hk_scale, hk_zero, hv, hv_scale, hv_zero, k_pos,
                     seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, workspace, workspace_bytes, stream,
                     stage_events);
}

int palu_attn_decode_latent(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                            const void* q, const int32_t* q_pos,
                            const void* hk, const void* hk_scale, const void* hk_zero,
                            const void* hv, const void* hv_scale, const void* hv_zero,
                            const int32_t* k_pos, const int32_t* seq_lens,
                            const void* Bk,
                            const void* rope_table, int32_t rope_table_len,
                            float* out_latent, void* workspace, size_t workspace_bytes, void* stream) {
  if (!out_latent) return PALU_ERR_INVALID_ARG;
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, hk_scale, hk_zero, hv, hv_scale, hv_zero, k_pos,
                     seq_lens, Bk, nullptr, rope_table, rope_table_len, nullptr, out_latent, workspace, workspace_bytes,
                     stream, nullptr);
}

int palu_attn_decode_multi(const palu_layer_desc* desc, int32_t batch, int32_t n_q, int32_t seq_len, int32_t max_seq,
                           const void* q, const int32_t* q_pos, const int32_t* q_len,
                           const void* hk, const void* hk_scale, const void* hk_zero,
                           const void* hv, const void* hv_scale, const void* hv_zero,
                           const int32_t* k_pos, const int32_t* seq_lens,
                           const void* Bk, const void* Bv,
                           const void* rope_table, int32_t rope_table_len,
                           float* out, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_impl(desc, batch, n_q, q_len, seq_len, max_seq, q, q_pos, hk, hk_scale, hk_zero, hv, hv_scale, hv_zero,
                     k_pos, seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, workspace, workspace_bytes, stream,
                     nullptr);
}

int palu_decode_step(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                     const void* x, const void* Ak, const void* Av, const int32_t* dst_row,
                     void* encode_workspace, size_t encode_workspace_bytes,
                     const void* q, const int32_t* q_pos, void* hk, void* hv,
                     const int32_t* k_pos, const int32_t* seq_lens,
                     const void* Bk, const void* Bv,
                     const void* rope_table, int32_t rope_table_len,
                     float* out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!desc) return PALU_ERR_INVALID_ARG;
  if (latent_bits(desc->k_latent_dtype) || latent_bits(desc->v_latent_dtype)) return PALU_ERR_UNSUPPORTED;
  if (batch <= 0) return PALU_ERR_INVALID_ARG;
  Meta m;
  int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  EncodePlan p;
  const int Rk = m.k_off[m.n_groups], Rv = m.v_off[m.n_groups];
  if ((st = plan_encode(desc, true, true, x, batch, Ak, Av, hk, Rk, hv, Rv, dst_row, encode_workspace,
                        encode_workspace_bytes, &p)) != PALU_OK)
    return st;
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, nullptr, nullptr, hv, nullptr, nullptr, k_pos,
                     seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, workspace, workspace_bytes, stream, nullptr,
                     &p);
}

int palu_decode_step_t(const palu_layer_desc* desc, int32_t batch, int32_t seq_len, int32_t max_seq,
                       const void* x, const void* Akt, const void* Avt, const int32_t* dst_row,
                       const void* q, const int32_t* q_pos, void* hk, void* hv,
                       const int32_t* k_pos, const int32_t* seq_lens,
                       const void* Bk, const void* Bv,
                       const void* rope_table, int32_t rope_table_len,
                       float* out, void* workspace, size_t workspace_bytes, void* stream) {
  if (!desc) return PALU_ERR_INVALID_ARG;
  if (batch <= 0) return PALU_ERR_INVALID_ARG;
  Meta m;
  int st = check_desc(desc, &m);
  if (st != PALU_OK) return st;
  static thread_local EncodePlan p;
  const int Rk = m.k_off[m.n_groups], Rv = m.v_off[m.n_groups];
  if ((st = plan_encode_t(desc, x, batch, Akt, Avt, hk, Rk, hv, Rv, dst_row, &p)) != PALU_OK) return st;
  return decode_impl(desc, batch, 1, nullptr, seq_len, max_seq, q, q_pos, hk, nullptr, nullptr, hv, nullptr, nullptr, k_pos,
                     seq_lens, Bk, Bv, rope_table, rope_table_len, out, nullptr, workspace, workspace_bytes, stream, nullptr,
                     &p);
}

}  // extern "C"
