// Host-side planning of the multi-table EmbeddingBag forward for MI355X (gfx950): the choice of
// kernel, prefetch depth, grid and block order (the decisions the paper's profiling recipe makes
// per workload, Sec. 7), the process-wide tuning keys, and the C-ABI entry points that need no
// GPU (emb_bag_plan_forward*, emb_bag_set_tuning / emb_bag_get_tuning, emb_bag_status_string,
// emb_bag_version).  Plain C++: no HIP call, no device pointer is read.

#include "emb_bag_plan.h"

#include <string.h>

namespace embbag {
namespace host {

Tuning g_tuning;

// The tuning table (emb_bag_set_tuning_table): what a sweep found best per shape.  An entry covers
// rows of at most max_row_bytes bytes and calls whose average bag length is at most max_avg_len;
// the first entry that covers a call supplies the keys that emb_bag_set_tuning has left automatic.
constexpr int kMaxTableEntries = 64;
emb_bag_tuning_entry g_table[kMaxTableEntries];
int g_table_entries = 0;

Tuning effective_tuning(const Tuning& base, uint32_t row_bytes, double avg_len) {
  Tuning tu = base;
  for (int i = 0; i < g_table_entries; ++i) {
    const emb_bag_tuning_entry& e = g_table[i];
    if ((int64_t)row_bytes > (int64_t)e.max_row_bytes || avg_len > (double)e.max_avg_len) continue;
    if (tu.depth == 0 && e.depth != 0) tu.depth = e.depth;
    if (tu.bags_per_wave == 0 && e.bags_per_wave != 0) tu.bags_per_wave = e.bags_per_wave;
    if (tu.stream == -1 && e.stream != -1) tu.stream = e.stream;
    if (tu.bags_per_group == 0 && e.bags_per_group != 0) tu.bags_per_group = e.bags_per_group;
    break;
  }
  return tu;
}

// When the short-bag kernel is chosen (measured on MI355X over row widths 128 B .. 1 KiB and
// pooling 1 .. 80): the wave kernel fetches G = 64/LPR rows of a bag per load instruction and
// needs about three such instructions per bag to hide its per-bag chain, so the stream kernel
// wins below an average of 3 * G lookups per bag (7x at 128-byte rows and one lookup per bag,
// nothing above the threshold).  A group then takes about kStreamGroupLookups lookups' worth of
// consecutive bags, fewer when the launch would drop below kStreamMinWaves wavefronts.
constexpr double kStreamBelowRowLoads = 3.0;
constexpr double kStreamGroupLookups = 4.0;
constexpr int64_t kStreamMaxAutoBags = 4;
constexpr int64_t kStreamMinWaves = 1024;

// The kernels are built one lanes-per-row class per translation unit (emb_bag_wave.hip and
// emb_bag_stream.hip, compiled once per class); here the classes are put back together.
KernelFn pick_kernel(int lpr, int elem, int depth, int op, bool buf, int variant = kVariantPlain) {
  switch (lpr) {
    case 0: return pick_wave_kernel_lpr0(elem, depth, op, buf, variant);
    case 4: return pick_wave_kernel_lpr4(elem, depth, op, buf, variant);
    case 8: return pick_wave_kernel_lpr8(elem, depth, op, buf, variant);
    case 16: return pick_wave_kernel_lpr16(elem, depth, op, buf, variant);
    case 32: return pick_wave_kernel_lpr32(elem, depth, op, buf, variant);
    case 64: return pick_wave_kernel_lpr64(elem, depth, op, buf, variant);
    default: return nullptr;
  }
}

KernelFn pick_stream_kernel(int lpr, int elem, int depth, int op, bool mixed, bool buf) {
  switch (lpr) {
    case 4: return pick_stream_kernel_lpr4(elem, depth, op, mixed, buf);
    case 8: return pick_stream_kernel_lpr8(elem, depth, op, mixed, buf);
    case 16: return pick_stream_kernel_lpr16(elem, depth, op, mixed, buf);
    case 32: return pick_stream_kernel_lpr32(elem, depth, op, mixed, buf);
    case 64: return pick_stream_kernel_lpr64(elem, depth, op, mixed, buf);
    default: return nullptr;
  }
}

FusedFn pick_fused_kernel(int elem, int depth, bool weighted) {
  switch (elem) {
    case EMB_F32: return pick_fused_kernel_elem0(depth, weighted);
    case EMB_F16: return pick_fused_kernel_elem1(depth, weighted);
    case EMB_BF16: return pick_fused_kernel_elem2(depth, weighted);
    case EMB_U8ROW: return pick_fused_kernel_elem3(depth, weighted);
    case EMB_FP8ROW: return pick_fused_kernel_elem4(depth, weighted);
    default: return nullptr;
  }
}

FusedFn pick_fused_uniform_kernel(int lpr, int elem, int depth, bool weighted) {
  switch (lpr) {
    case 4: return pick_fused_uniform_kernel_lpr4(elem, depth, weighted);
    case 8: return pick_fused_uniform_kernel_lpr8(elem, depth, weighted);
    case 16: return pick_fused_uniform_kernel_lpr16(elem, depth, weighted);
    case 32: return pick_fused_uniform_kernel_lpr32(elem, depth, weighted);
    case 64: return pick_fused_uniform_kernel_lpr64(elem, depth, weighted);
    default: return nullptr;
  }
}

bool is_quant(int table_dtype) { return table_dtype == EMB_U8ROW || table_dtype == EMB_FP8ROW; }

int check_desc(const emb_bag_desc* d, uint32_t* row_bytes_out) {
  if (!d) return EMB_ERR_NULL_PTR;
  if (d->table_dtype < EMB_F32 || d->table_dtype > EMB_FP8ROW) return EMB_ERR_BAD_DTYPE;
  if (d->mode != EMB_SUM && d->mode != EMB_MEAN && d->mode != EMB_MAX) return EMB_ERR_BAD_MODE;
  if (d->num_tables < 1 || d->dim < 1) return EMB_ERR_BAD_DIM;
  int64_t row_bytes = (int64_t)d->dim * (d->table_dtype == EMB_F32 ? 4 : 2);
  if (is_quant(d->table_dtype)) {
    row_bytes = (int64_t)d->dim + 8;  // one-byte codes, then fp32 scale and fp32 bias
    if (row_bytes > kSlabBytes) return EMB_ERR_BAD_DIM;
  }
  if (row_bytes % 16 != 0 || row_bytes > 65536) return EMB_ERR_BAD_DIM;
  if (d->batch < 0 || d->num_lookups < 0 || d->max_table_rows < 0) return EMB_ERR_BAD_SIZE;
  *row_bytes_out = (uint32_t)row_bytes;
  return EMB_OK;
}

// Lay out the grid of a launch over n tables (p.wpt wavefronts each): natural order, or the
// XCD-affine order described at KParams.  `ids` names the tables (nullptr: tables 0 .. n-1 in
// their own order); `row_units` (16-byte segments per row, indexed like ids) is given only when
// the tables of the launch differ in width, and then n <= kMaxOrdered unless natural_order.
void plan_grid(int64_t n, const uint16_t* ids, const uint16_t* row_units, bool natural_order,
               Launch* L) {
  KParams& p = L->p;
  L->tables = n;
  p.num_work = (uint32_t)(n * (int64_t)p.wpt);
  p.xcd_bpp = p.xcd_wpp = p.xcd_pshift = p.xcd_units = p.listed = 0;
  uint32_t blocks = (uint32_t)(((uint64_t)p.num_work + kWavesPerBlock - 1) / kWavesPerBlock);
  const Tuning& base = L->tuning;
  const bool remap = base.xcd_remap == 1 || (base.xcd_remap == -1 && blocks >= 4096);
  bool ordered = false;
  if (remap && blocks >= 64 && !natural_order) {
    // pieces per table: the smallest power of two that makes n * pieces a multiple of 8, so
    // that every XCD gets the same number of pieces and neighbouring XCDs share a table
    uint32_t pshift = 0;
    while (((uint64_t)n << pshift) % 8 != 0) ++pshift;
    if (base.xcd_pieces > 0) {  // forced: XCDs may then differ by one piece
      pshift = 0;
      while ((1 << pshift) < base.xcd_pieces) ++pshift;
    }
    const uint64_t wpp = ((uint64_t)p.wpt + (1u << pshift) - 1) >> pshift;
    const uint64_t bpp = (wpp + kWavesPerBlock - 1) / kWavesPerBlock;
    const uint64_t units = (uint64_t)n << pshift;
    const uint64_t grid = ((units + 7) / 8) * 8 * bpp;
    // Tables of different widths: position q of the order runs on the XCD set q % sets.  Deal
    // the tables out widest first, each to the set with the least work so far, so that every
    // XCD ends up with about the same number of bytes.
    const uint32_t sets = 8u >> (pshift < 3 ? pshift : 3);
    const bool ok = grid <= kMaxBlocks;  // else: natural order, checked by the caller
    ordered = ok && row_units && sets > 1 && n % sets == 0;
    if (ordered) {
      uint32_t head[66];  // counting sort by width, widest first
      for (int i = 0; i < 66; ++i) head[i] = 0;
      for (int64_t t = 0; t < n; ++t) ++head[64 - row_units[t] + 1];
      for (int i = 1; i < 66; ++i) head[i] += head[i - 1];
      uint16_t by_width[kMaxOrdered];
      for (int64_t t = 0; t < n; ++t) by_width[head[64 - row_units[t]]++] = (uint16_t)t;
      uint64_t load[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      uint32_t taken[8] = {0, 0, 0, 0, 0, 0, 0, 0};
      const uint32_t per_set = (uint32_t)(n / sets);  // exact: n * pieces is a multiple of 8
      for (int64_t k = 0; k < n; ++k) {
        const uint16_t t = by_width[k];
        uint32_t best = sets;
        for (uint32_t c = 0; c < sets; ++c)
          if (taken[c] < per_set && (best == sets || load[c] < load[best])) best = c;
        L->order.t[best + sets * taken[best]] = ids ? ids[t] : t;
        ++taken[best];
        load[best] += row_units[t];
      }
      p.listed = 1;
    }
    if (ok) {
      p.xcd_bpp = (uint32_t)bpp;
      p.xcd_wpp = (uint32_t)wpp;
      p.xcd_pshift = pshift;
      p.xcd_units = (uint32_t)units;
      blocks = (uint32_t)grid;
    }
  }
  if (ids && !ordered) {  // a subset of the tables, in the order given
    for (int64_t t = 0; t < n; ++t) L->order.t[t] = ids[t];
    p.listed = 1;
  }
  L->blocks = blocks;
}

// Consecutive bags per lane group of the stream kernel for an average bag length.
int64_t stream_bags_per_group(const Tuning& tu, double avg_len, int lpr, int64_t tables,
                              int64_t B) {
  const int groups = kWaveSize / lpr;
  int64_t m = tu.bags_per_group;
  if (m == 0) {
    m = (int64_t)(kStreamGroupLookups / (avg_len < 1.0 ? 1.0 : avg_len) + 0.5);
    if (m > kStreamMaxAutoBags) m = kStreamMaxAutoBags;
    while (m > 1 && tables * ((B + groups * m - 1) / (groups * m)) < kStreamMinWaves) m /= 2;
  }
  if (m > lpr - 1) m = lpr - 1;
  return m < 1 ? 1 : m;
}

// Consecutive bags per wavefront of the wave kernel.  A bag costs its wavefront a fixed chain
// of memory round trips (bounds, row ids, first rows, store) besides its row loads; with several
// bags per wavefront the bounds come with one load and the next bag's row ids are requested
// while the current bag's rows are gathered.  Automatic: enough bags to give a wavefront about
// kWaveLoadsTarget load instructions (rows_per_load rows each), at most kWaveMaxAutoBags, and
// fewer when the launch would drop below kWaveMinWaves wavefronts.
constexpr double kWaveLoadsTarget = 16.0;
constexpr int64_t kWaveMaxAutoBags = 4;
constexpr int64_t kWaveMinWaves = 32768;
constexpr int64_t kWaveMaxBags = 32;
int64_t wave_bags_per_wave(const Tuning& tu, double avg_len, int rows_per_load, int64_t tables,
                           int64_t B, int64_t slabs) {
  if (slabs > 1) return 1;
  int64_t m = tu.bags_per_wave;
  if (m == 0) {
    const double loads = (avg_len < 1.0 ? 1.0 : avg_len) / rows_per_load;
    m = (int64_t)(kWaveLoadsTarget / loads + 0.5);
    if (m > kWaveMaxAutoBags) m = kWaveMaxAutoBags;
    while (m > 1 && tables * ((B + m - 1) / m) < kWaveMinWaves) --m;
  }
  if (m > kWaveMaxBags) m = kWaveMaxBags;
  return m < 1 ? 1 : m;
}

// Descriptor checks of emb_bag_forward that need no pointer: shape, mode, weights, out_ld.
int precheck_uniform(const emb_bag_desc* desc, bool weighted, uint32_t* row_bytes,
                     int64_t* out_ld) {
  const int rc = check_desc(desc, row_bytes);
  if (rc != EMB_OK) return rc;
  const int64_t T = desc->num_tables, D = desc->dim;
  if (weighted && desc->mode != EMB_SUM) return EMB_ERR_UNSUPPORTED;
  *out_ld = desc->out_ld ? desc->out_ld : T * D;
  if (*out_ld < T * D || *out_ld % 4 != 0) return EMB_ERR_BAD_DIM;
  return EMB_OK;
}

// Append launches over the tables `ids` (all T tables in their own order if ids is empty) that
// share everything in `proto` except the grid; a launch that needs a table list takes at most
// kMaxOrdered tables.  `units` (16-byte segments per row, indexed like ids) may be empty.
void add_launches(const Launch& proto, int64_t T, const std::vector<uint16_t>& ids,
                  const std::vector<uint16_t>& units, std::vector<Launch>* launches) {
  if (ids.empty()) {
    launches->push_back(proto);
    plan_grid(T, nullptr, nullptr, false, &launches->back());
    return;
  }
  for (size_t first = 0; first < ids.size(); first += kMaxOrdered) {
    const size_t left = ids.size() - first;
    const int64_t n = (int64_t)(left < (size_t)kMaxOrdered ? left : (size_t)kMaxOrdered);
    bool differ = false;
    for (int64_t i = 1; i < n && !units.empty() && !differ; ++i)
      differ = units[first + (size_t)i] != units[first];
    launches->push_back(proto);
    plan_grid(n, ids.data() + first, differ ? units.data() + first : nullptr, false,
              &launches->back());
  }
}

// Turn `proto` (a wave-kernel launch of a uniform call) into a stream-kernel launch over
// `tables` tables of average bag length avg_len; false if the stream kernel cannot take it.
bool make_stream(const Tuning& tu, Launch* L, const emb_bag_desc* desc, int op, int depth,
                 double avg_len, int64_t tables, int64_t out_ld) {
  const int lpr = L->lpr, groups = kWaveSize / lpr;
  const int64_t B = desc->batch;
  const int64_t m = stream_bags_per_group(tu, avg_len, lpr, tables, B);
  // the wavefront's output rows are addressed through one buffer with 32-bit offsets
  if ((uint64_t)groups * (uint64_t)m * (uint64_t)out_ld * 4u > kBufMaxBytes) return false;
  KernelFn fn = pick_stream_kernel(lpr, desc->table_dtype, depth, op, false, L->buf);
  if (!fn) return false;
  L->fn = fn;
  L->kernel = EMB_KERNEL_STREAM;
  L->hot = false;  // the short-bag kernel reads every row of a table with the table's policy
  L->lds_bytes = 0;  // ... into registers
  L->depth = depth <= 4 || lpr < 8 ? 4 : 8;  // the depths that kernel is built with
  L->p.bags_per_group = (uint32_t)m;
  L->p.bags_per_wave = 1;
  L->p.wpt = (uint32_t)((B + groups * m - 1) / (groups * m));
  return true;
}

// One tuning key, checked (the values emb_bag_set_tuning documents).
int set_key(Tuning* tu, const char* key, int64_t value) {
  if (!strcmp(key, "depth")) {
    if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 16)
      return EMB_ERR_BAD_TUNING;
    tu->depth = value;
  } else if (!strcmp(key, "addressing")) {
    if (value < 0 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->addressing = value;
  } else if (!strcmp(key, "blocks_per_cu")) {
    if (value < 0 || value > 8) return EMB_ERR_BAD_TUNING;
    tu->blocks_per_cu = value;
  } else if (!strcmp(key, "xcd_remap")) {
    if (value < -1 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->xcd_remap = value;
  } else if (!strcmp(key, "use_hints")) {
    if (value < 0 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->use_hints = value;
  } else if (!strcmp(key, "stream")) {
    if (value < -1 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->stream = value;
  } else if (!strcmp(key, "bags_per_group")) {
    if (value < 0 || value > 63) return EMB_ERR_BAD_TUNING;
    tu->bags_per_group = value;
  } else if (!strcmp(key, "per_table_launch")) {
    if (value < 0 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->per_table_launch = value;
  } else if (!strcmp(key, "fuse")) {
    if (value < 0 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->fuse = value;
  } else if (!strcmp(key, "xcd_pieces")) {
    if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8)
      return EMB_ERR_BAD_TUNING;
    tu->xcd_pieces = value;
  } else if (!strcmp(key, "bags_per_wave")) {
    if (value < 0 || value > kWaveMaxBags) return EMB_ERR_BAD_TUNING;
    tu->bags_per_wave = value;
  } else if (!strcmp(key, "hot_split")) {
    if (value < 0 || value > 2) return EMB_ERR_BAD_TUNING;
    tu->hot_split = value;
  } else if (!strcmp(key, "station")) {
    if (value < 0 || value > 1) return EMB_ERR_BAD_TUNING;
    tu->station = value;
  } else {
    return EMB_ERR_BAD_TUNING;
  }
  return EMB_OK;
}

// The tuning a call is planned from: the descriptor's own, checked, or the process-wide keys.
int base_tuning(const emb_bag_tuning* t, Tuning* out) {
  if (!t) {
    *out = g_tuning;
    return EMB_OK;
  }
  *out = Tuning();
  const struct { const char* key; int32_t value; } fields[] = {
      {"depth", t->depth}, {"addressing", t->addressing}, {"blocks_per_cu", t->blocks_per_cu},
      {"xcd_remap", t->xcd_remap}, {"use_hints", t->use_hints}, {"stream", t->stream},
      {"bags_per_group", t->bags_per_group}, {"xcd_pieces", t->xcd_pieces},
      {"per_table_launch", t->per_table_launch}, {"fuse", t->fuse},
      {"bags_per_wave", t->bags_per_wave}, {"hot_split", t->hot_split}, {"station", t->station}};
  for (const auto& f : fields) {
    const int rc = set_key(out, f.key, f.value);
    if (rc != EMB_OK) return rc;
  }
  return EMB_OK;
}

// The host-side decisions of emb_bag_forward for a checked descriptor with batch > 0: one launch,
// or two when desc->table_avg_len separates tables with short bags from the others.
int plan_uniform(const emb_bag_desc* desc, bool weighted, uint32_t row_bytes, int64_t out_ld,
                 std::vector<Launch>* launches) {
  const int64_t T = desc->num_tables, B = desc->batch, D = desc->dim;
  const int64_t slabs = (row_bytes + kSlabBytes - 1) / kSlabBytes;
  const int64_t num_work = T * B * slabs;
  if (B > 0x7FFFFFFF || num_work > 0x7FFFFFFF) return EMB_ERR_BAD_SIZE;

  // lanes per row: the smallest power of two that covers min(row, 1 KiB) in 16-byte segments
  int lpr = 4;
  const uint32_t span = row_bytes < (uint32_t)kSlabBytes ? row_bytes : (uint32_t)kSlabBytes;
  while ((uint32_t)lpr * 16u < span) lpr *= 2;

  Tuning base;  // the descriptor's tuning, or the process-wide keys
  const int trc = base_tuning(desc->tuning, &base);
  if (trc != EMB_OK) return trc;
  bool buf = desc->max_table_rows > 0 &&
             (uint64_t)desc->max_table_rows * row_bytes <= kBufMaxBytes;
  if (base.addressing == 1) buf = false;

  // ... with the keys left automatic filled in from the tuning table
  const Tuning tu = effective_tuning(base, row_bytes,
                                     (double)desc->num_lookups / ((double)T * (double)B));
  int depth = (int)tu.depth;
  if (depth == 0) depth = (desc->table_dtype == EMB_F32 && row_bytes >= 512) ? 8 : 4;

  Launch wave;  // the one-wavefront-per-bag launch; the stream launch is derived from it
  wave.tuning = base;
  KParams& p = wave.p;
  p.num_lookups = desc->num_lookups;
  p.out_ld = out_ld;
  p.max_rows = desc->max_table_rows;
  p.B = (uint32_t)B;
  p.wpt = (uint32_t)(B * slabs);
  p.slabs = (uint32_t)slabs;
  p.row_bytes = row_bytes;
  p.D = (uint32_t)D;
  p.mean = desc->mode == EMB_MEAN ? 1u : 0u;
  p.has_hints = (desc->table_hints != nullptr && base.use_hints != 0) ? 1u : 0u;
  p.bags_per_group = 0;
  const int groups = kWaveSize / lpr;
  const double avg_len = (double)desc->num_lookups / ((double)T * (double)B);
  p.bags_per_wave = (uint32_t)wave_bags_per_wave(tu, avg_len, groups, T, B, slabs);
  if (slabs == 1) p.wpt = (uint32_t)((B + p.bags_per_wave - 1) / p.bags_per_wave);
  wave.kernel = EMB_KERNEL_WAVE;
  wave.lpr = lpr;
  wave.depth = depth;
  wave.buf = buf;
  const int op = desc->mode == EMB_MAX ? kOpMax : (weighted ? kOpWeighted : kOpSum);
  wave.op = op;
  if (op == kOpMax) wave.depth = depth <= 4 ? 4 : 8;
  // tables with a hot head: the kernel that reads hot and other rows with different cache
  // policies, where it is built (buffer addressing, depth 4 or 8); otherwise the head is ignored
  wave.hot = desc->hot_rows != nullptr && base.hot_split != 0 && buf &&
             pick_kernel(lpr, desc->table_dtype, depth, op, buf, (int)base.hot_split) != nullptr;
  int variant = wave.hot ? (int)base.hot_split : kVariantPlain;
  // the LDS station, where it is built (buffer addressing, sum pooling, depth 4 or 8, no hot /
  // cold split); otherwise the key is ignored
  if (base.station == 1 && !wave.hot &&
      pick_kernel(lpr, desc->table_dtype, depth, op, buf, kVariantLds) != nullptr) {
    variant = kVariantLds;
    wave.lds_bytes = (uint32_t)(kWavesPerBlock * depth * kWaveSize * 16);
  }
  wave.fn = pick_kernel(lpr, desc->table_dtype, depth, op, buf, variant);
  if (!wave.fn) return EMB_ERR_BAD_TUNING;

  // Short bags: a lane group streams several consecutive bags (emb_bag_stream.hip).  Without
  // per-table lengths the host knows the call's average bag length, NL / (T * B), and nothing
  // else; with them each table is judged by its own.
  const double threshold = kStreamBelowRowLoads * groups;
  const bool can_stream = tu.stream != 0 && slabs == 1;
  const std::vector<uint16_t> none;
  if (base.per_table_launch == 1 && T <= 65535) {
    // the paper's launch structure, for comparison: the tables one after the other
    Launch stream = wave;
    const bool s = can_stream && (tu.stream == 1 || avg_len < threshold) &&
                   make_stream(tu, &stream, desc, op, depth, avg_len, 1, out_ld);
    for (int64_t t = 0; t < T; ++t)
      add_launches(s ? stream : wave, T, std::vector<uint16_t>(1, (uint16_t)t), none, launches);
    return EMB_OK;
  }
  if (can_stream && tu.stream == -1 && desc->table_avg_len && T <= 65535) {
    std::vector<uint16_t> short_ids, long_ids;
    double short_sum = 0.0, long_sum = 0.0;
    for (int64_t t = 0; t < T; ++t) {
      if ((double)desc->table_avg_len[t] < threshold) {
        short_ids.push_back((uint16_t)t);
        short_sum += (double)desc->table_avg_len[t];
      } else {
        long_ids.push_back((uint16_t)t);
        long_sum += (double)desc->table_avg_len[t];
      }
    }
    Launch stream = wave;
    if (!short_ids.empty() && !long_ids.empty() &&
        make_stream(tu, &stream, desc, op, depth, short_sum / (double)short_ids.size(),
                    (int64_t)short_ids.size(), out_ld)) {
      // the wave part's bags per wavefront follow its own tables
      p.bags_per_wave = (uint32_t)wave_bags_per_wave(tu, long_sum / (double)long_ids.size(), groups,
                                                     (int64_t)long_ids.size(), B, slabs);
      p.wpt = (uint32_t)((B + p.bags_per_wave - 1) / p.bags_per_wave);
      add_launches(wave, T, long_ids, none, launches);  // listed in the order a fused launch
      add_launches(stream, T, short_ids, none, launches);  // runs them: long bags first
      return EMB_OK;
    }
    // all tables on one side: one launch without a list
    if (long_ids.empty() && make_stream(tu, &stream, desc, op, depth, avg_len, T, out_ld))
      add_launches(stream, T, none, none, launches);
    else
      add_launches(wave, T, none, none, launches);
    return EMB_OK;
  }
  Launch stream = wave;
  if (can_stream && (tu.stream == 1 || avg_len < threshold) &&
      make_stream(tu, &stream, desc, op, depth, avg_len, T, out_ld))
    add_launches(stream, T, none, none, launches);
  else
    add_launches(wave, T, none, none, launches);
  return EMB_OK;
}

// Descriptor checks of emb_bag_forward_mixed that need no device pointer; also the widest row
// and the total width.
int precheck_mixed(const emb_bag_mixed_desc* desc, bool weighted, uint32_t* max_row_bytes,
                   int64_t* out_ld) {
  if (!desc) return EMB_ERR_NULL_PTR;
  if (desc->table_dtype < EMB_F32 || desc->table_dtype > EMB_FP8ROW) return EMB_ERR_BAD_DTYPE;
  if (desc->mode != EMB_SUM && desc->mode != EMB_MEAN && desc->mode != EMB_MAX)
    return EMB_ERR_BAD_MODE;
  if (desc->num_tables < 1 || !desc->dims) return desc->dims ? EMB_ERR_BAD_DIM : EMB_ERR_NULL_PTR;
  if (desc->batch < 0 || desc->num_lookups < 0 || desc->max_table_bytes < 0)
    return EMB_ERR_BAD_SIZE;
  int64_t total_dim = 0;
  *max_row_bytes = 0;
  for (int64_t t = 0; t < desc->num_tables; ++t) {
    const int64_t d = desc->dims[t];
    if (d < 1) return EMB_ERR_BAD_DIM;
    const int64_t rb = is_quant(desc->table_dtype) ? d + 8
                                                     : d * (desc->table_dtype == EMB_F32 ? 4 : 2);
    if (rb % 16 != 0 || rb > kSlabBytes) return EMB_ERR_BAD_DIM;
    if (rb > *max_row_bytes) *max_row_bytes = (uint32_t)rb;
    total_dim += d;
  }
  if (weighted && desc->mode != EMB_SUM) return EMB_ERR_UNSUPPORTED;
  *out_ld = desc->out_ld ? desc->out_ld : total_dim;
  if (*out_ld < total_dim || *out_ld % 4 != 0) return EMB_ERR_BAD_DIM;
  return EMB_OK;
}

// The host-side decisions of emb_bag_forward_mixed for a checked descriptor with batch > 0: one
// launch of the wave kernel over all tables, or - with short bags - one launch of the stream
// kernel per lanes-per-row class whose tables it suits, and one of the wave kernel for the rest.
// A launch that needs a table list takes at most kMaxOrdered tables.
int plan_mixed(const emb_bag_mixed_desc* desc, bool weighted, uint32_t max_row_bytes,
               int64_t out_ld, std::vector<Launch>* launches) {
  const int64_t T = desc->num_tables, B = desc->batch;
  if (B > 0x7FFFFFFF || T * B > 0x7FFFFFFF) return EMB_ERR_BAD_SIZE;
  const int elem_bytes = desc->table_dtype == EMB_F32 ? 4 : 2;
  Tuning tu0;  // the descriptor's tuning, or the process-wide keys
  const int trc = base_tuning(desc->tuning, &tu0);
  if (trc != EMB_OK) return trc;
  bool buf = desc->max_table_bytes > 0 && (uint64_t)desc->max_table_bytes <= kBufMaxBytes;
  if (tu0.addressing == 1) buf = false;
  const Tuning tu = effective_tuning(tu0, max_row_bytes,
                                     (double)desc->num_lookups / ((double)T * (double)B));
  int depth = (int)tu.depth;
  if (depth == 0) depth = (desc->table_dtype == EMB_F32 && max_row_bytes >= 512) ? 8 : 4;
  const int op = desc->mode == EMB_MAX ? kOpMax : (weighted ? kOpWeighted : kOpSum);

  Launch base;
  base.tuning = tu0;
  KParams& p = base.p;
  p.num_lookups = desc->num_lookups;
  p.out_ld = out_ld;
  p.max_rows = 0;
  p.B = (uint32_t)B;
  p.bags_per_group = 0;
  p.slabs = 1;
  p.row_bytes = max_row_bytes;
  p.D = 0;
  p.mean = desc->mode == EMB_MEAN ? 1u : 0u;
  p.has_hints = (desc->table_hints != nullptr && tu0.use_hints != 0) ? 1u : 0u;
  base.kernel = EMB_KERNEL_WAVE;
  base.lpr = 0;
  base.depth = depth <= 4 ? 4 : 8;  // the depths the mixed-width kernels are built with
  base.buf = buf;
  base.op = op;
  base.fn = pick_kernel(0, desc->table_dtype, depth, op, buf);
  if (!base.fn) return EMB_ERR_BAD_TUNING;

  // which lanes-per-row classes (4, 8, 16, 32, 64) go to the stream kernel
  const double avg_len = (double)desc->num_lookups / ((double)T * (double)B);
  {
    int wide_lpr = 4;  // bags per wavefront: judged by the widest row (the fewest rows per load)
    while ((uint32_t)wide_lpr * 16u < max_row_bytes) wide_lpr *= 2;
    p.bags_per_wave = (uint32_t)wave_bags_per_wave(tu, avg_len, kWaveSize / wide_lpr, T, B, 1);
    p.wpt = (uint32_t)((B + p.bags_per_wave - 1) / p.bags_per_wave);
  }
  // (judged by the call's average bag length, or table by table with desc->table_avg_len)
  const bool can_stream = tu.stream != 0;
  const bool per_table = tu.stream == -1 && desc->table_avg_len != nullptr;
  bool fits[7] = {false, false, false, false, false, false, false};  // by log2(lanes per row)
  for (int lg = 2; lg <= 6 && can_stream; ++lg) {
    // the wavefront's output rows are addressed through one buffer with 32-bit offsets: checked
    // for the largest group size the class can get
    const int groups = kWaveSize >> lg;
    int64_t m = tu.bags_per_group ? tu.bags_per_group : kStreamMaxAutoBags;
    if (m > (1 << lg) - 1) m = (1 << lg) - 1;
    fits[lg] = (uint64_t)groups * (uint64_t)m * (uint64_t)out_ld * 4u <= kBufMaxBytes;
  }
  std::vector<uint16_t> units((size_t)T);
  std::vector<uint8_t> cls((size_t)T);   // log2(lanes per row)
  std::vector<uint8_t> streamed((size_t)T);
  bool widths_differ = false, any_stream = false;
  for (int64_t t = 0; t < T; ++t) {
    const int64_t d = desc->dims[t];
    const int64_t rb = is_quant(desc->table_dtype) ? d + 8 : d * elem_bytes;
    units[(size_t)t] = (uint16_t)(rb / 16);
    int lg = 2;
    while ((16 << lg) < rb) ++lg;
    cls[(size_t)t] = (uint8_t)lg;
    if (d != desc->dims[0]) widths_differ = true;
    const double len_t = per_table ? (double)desc->table_avg_len[t] : avg_len;
    streamed[(size_t)t] = fits[lg] && (tu.stream == 1 ||
                                       len_t < kStreamBelowRowLoads * (kWaveSize >> lg));
    if (streamed[(size_t)t]) any_stream = true;
  }

  if (!any_stream) {  // one launch of the wave kernel over all tables
    launches->push_back(base);
    // more tables than the list holds: such a launch keeps the natural block order
    const bool too_many = widths_differ && T > kMaxOrdered;
    plan_grid(T, nullptr, widths_differ && !too_many ? units.data() : nullptr, too_many,
              &launches->back());
    return EMB_OK;
  }

  // one group of tables per streamed class, one for everything else
  if (T > 65535) return EMB_ERR_BAD_SIZE;  // table numbers above 65535 cannot be listed
  for (int lg = 1; lg <= 6; ++lg) {  // lg == 1 stands for "the wave kernel's tables"
    std::vector<uint16_t> ids, u;
    double len_sum = 0.0;
    for (int64_t t = 0; t < T; ++t) {
      if (lg == 1 ? !streamed[(size_t)t] : (streamed[(size_t)t] && cls[(size_t)t] == lg)) {
        ids.push_back((uint16_t)t);
        u.push_back(units[(size_t)t]);
        len_sum += per_table ? (double)desc->table_avg_len[t] : avg_len;
      }
    }
    if (ids.empty()) continue;
    Launch L = base;
    if (lg >= 2) {
      const int lpr = 1 << lg;
      const int groups = kWaveSize / lpr;
      const int64_t m = stream_bags_per_group(tu, len_sum / (double)ids.size(), lpr,
                                              (int64_t)ids.size(), B);
      L.fn = pick_stream_kernel(lpr, desc->table_dtype, depth, op, true, buf);
      if (!L.fn) return EMB_ERR_BAD_TUNING;
      L.kernel = EMB_KERNEL_STREAM;
      L.lpr = lpr;
      L.depth = depth <= 4 || lpr < 8 ? 4 : 8;
      L.p.row_bytes = (uint32_t)lpr * 16u;
      L.p.bags_per_group = (uint32_t)m;
      L.p.bags_per_wave = 1;
      L.p.wpt = (uint32_t)((B + groups * m - 1) / (groups * m));
    }
    add_launches(L, T, ids, u, launches);
  }
  return EMB_OK;
}

// Fuse `segs` (the launches planned for one call) if there are several, each body occurs at most
// once, their table lists fit one list, and the grid fits one dispatch.  `mixed`: the call is for
// tables of different widths (segment 0 the wave body, 1 .. 5 the stream body by lanes per row);
// otherwise one width (segment 0 the wave body, 1 the stream body, both with lanes per row lpr).
bool plan_fused(const std::vector<Launch>& segs, bool mixed, int table_dtype, bool weighted,
                FusedLaunch* F) {
  if (segs.size() < 2 || segs.size() > (size_t)kFusedSegments || segs[0].tuning.fuse == 0)
    return false;
  if (segs[0].op == kOpMax) return false;  // the fused kernels are built for sums
  const Launch* by_slot[kFusedSegments] = {nullptr, nullptr, nullptr, nullptr, nullptr, nullptr};
  int64_t tables = 0;
  int depth = 0, lpr = 0;
  for (const Launch& L : segs) {
    int slot = 0;
    if (!L.buf) return false;  // the fused kernels address rows through buffer resources
    if (L.kernel == EMB_KERNEL_WAVE) {
      if ((L.lpr == 0) != mixed) return false;
      depth = L.depth;
    } else if (mixed) {
      while ((2 << slot) < L.lpr) ++slot;  // 4 -> 1, 8 -> 2, ... 64 -> 5
    } else {
      slot = 1;
    }
    if (slot >= kFusedSegments || by_slot[slot] || !L.p.listed) return false;
    if (!mixed && lpr != 0 && L.lpr != lpr) return false;
    lpr = L.lpr;
    by_slot[slot] = &L;
    tables += L.tables;
  }
  if (tables > kMaxOrdered) return false;
  // one depth for the launch, the wave body's (4 or 8); a stream body takes the depth its own
  // launch would: 4 if that is 4 or it has 4 lanes per row, else 8
  if (depth == 0)
    for (const Launch& L : segs)
      if (L.depth > depth) depth = L.depth;
  if (depth != 4 && depth != 8) return false;
  for (const Launch& L : segs)
    if (L.kernel == EMB_KERNEL_STREAM && L.depth != ((depth == 4 || L.lpr < 8) ? 4 : 8))
      return false;
  F->fn = mixed ? pick_fused_kernel(table_dtype, depth, weighted)
                : pick_fused_uniform_kernel(lpr, table_dtype, depth, weighted);
  if (!F->fn) return false;
  uint64_t end = 0;
  uint32_t base = 0;
  for (int k = 0; k < kFusedSegments; ++k) {
    F->f.order_base[k] = base;
    if (const Launch* L = by_slot[k]) {
      F->f.seg[k] = L->p;
      for (int64_t t = 0; t < L->tables; ++t) F->order.t[base + t] = L->order.t[t];
      base += (uint32_t)L->tables;
      end += ((uint64_t)L->blocks + 7u) & ~7ull;  // padding workgroups find no work
    } else {
      F->f.seg[k] = KParams{};
    }
    if (end > kMaxBlocks) return false;
    F->f.end_block[k] = (uint32_t)end;
  }
  F->blocks = (uint32_t)end;
  F->blocks_per_cu = segs[0].tuning.blocks_per_cu;
  return true;
}

// What emb_bag_plan_forward* report about a planned launch.
void report(const Launch& L, int32_t num_launches, emb_bag_plan* plan, uint16_t* table_order) {
  plan->kernel = L.kernel;
  plan->lanes_per_row = L.lpr;
  plan->depth = L.depth;
  plan->buffer_addressing = L.buf ? 1 : 0;
  plan->bags_per_group = (int32_t)L.p.bags_per_group;
  plan->xcd_pieces = L.p.xcd_bpp ? (int32_t)(1u << L.p.xcd_pshift) : 0;
  plan->listed = (int32_t)L.p.listed;
  plan->num_launches = num_launches;
  plan->grid_blocks = L.blocks;
  plan->wavefronts = L.p.num_work;
  plan->waves_per_table = L.p.wpt;
  plan->waves_per_piece = L.p.xcd_wpp;
  plan->blocks_per_piece = L.p.xcd_bpp;
  plan->tables = L.tables;
  plan->bags_per_wave = L.kernel == EMB_KERNEL_WAVE ? (int32_t)L.p.bags_per_wave : 0;
  plan->hot_split = L.hot ? 1 : 0;
  plan->station = L.lds_bytes ? 1 : 0;
  if (table_order)
    for (int64_t t = 0; t < L.tables && t < kMaxOrdered; ++t)
      table_order[t] = L.p.listed ? L.order.t[t] : (uint16_t)t;
}

// EMB_ERR_BAD_SIZE if a launch of the plan is larger than a dispatch can be.
int check_grids(const std::vector<Launch>& launches) {
  for (const Launch& L : launches)
    if (L.blocks > kMaxBlocks) return EMB_ERR_BAD_SIZE;
  return EMB_OK;
}

}  // namespace host
}  // namespace embbag

using namespace embbag;
using namespace embbag::host;

extern "C" {

int emb_bag_plan_forward(const emb_bag_desc* desc, int has_weights, int32_t which,
                         emb_bag_plan* plan, uint16_t* table_order) {
  if (!plan) return EMB_ERR_NULL_PTR;
  memset(plan, 0, sizeof *plan);
  uint32_t row_bytes = 0;
  int64_t out_ld = 0;
  int rc = precheck_uniform(desc, has_weights != 0, &row_bytes, &out_ld);
  if (rc != EMB_OK) return rc;
  if (desc->batch == 0) return EMB_OK;
  std::vector<Launch> launches;
  rc = plan_uniform(desc, has_weights != 0, row_bytes, out_ld, &launches);
  if (rc == EMB_OK) rc = check_grids(launches);
  if (rc != EMB_OK) return rc;
  if (which < 0 || (size_t)which >= launches.size()) return EMB_ERR_BAD_SIZE;
  report(launches[(size_t)which], (int32_t)launches.size(), plan, table_order);
  FusedLaunch fused;
  if (plan_fused(launches, false, desc->table_dtype, has_weights != 0, &fused)) {
    plan->fused = 1;
    plan->fused_grid_blocks = fused.blocks;
    plan->hot_split = 0;  // the fused kernel has no hot / cold split
    plan->station = 0;    // ... and keeps its rows in registers
  }
  return EMB_OK;
}

int emb_bag_plan_forward_mixed(const emb_bag_mixed_desc* desc, int has_weights, int32_t which,
                               emb_bag_plan* plan, uint16_t* table_order) {
  if (!plan) return EMB_ERR_NULL_PTR;
  memset(plan, 0, sizeof *plan);
  uint32_t max_row_bytes = 0;
  int64_t out_ld = 0;
  int rc = precheck_mixed(desc, has_weights != 0, &max_row_bytes, &out_ld);
  if (rc != EMB_OK) return rc;
  if (desc->batch == 0) return EMB_OK;
  std::vector<Launch> launches;
  rc = plan_mixed(desc, has_weights != 0, max_row_bytes, out_ld, &launches);
  if (rc == EMB_OK) rc = check_grids(launches);
  if (rc != EMB_OK) return rc;
  if (which < 0 || (size_t)which >= launches.size()) return EMB_ERR_BAD_SIZE;
  report(launches[(size_t)which], (int32_t)launches.size(), plan, table_order);
  FusedLaunch fused;
  if (plan_fused(launches, true, desc->table_dtype, has_weights != 0, &fused)) {
    plan->fused = 1;
    plan->fused_grid_blocks = fused.blocks;
  }
  return EMB_OK;
}

int emb_bag_set_tuning(const char* key, int64_t value) {
  if (!key) return EMB_ERR_NULL_PTR;
  return set_key(&g_tuning, key, value);
}

int emb_bag_tuning_defaults(emb_bag_tuning* t) {
  if (!t) return EMB_ERR_NULL_PTR;
  const Tuning d;
  memset(t, 0, sizeof *t);
  t->depth = (int32_t)d.depth;
  t->addressing = (int32_t)d.addressing;
  t->blocks_per_cu = (int32_t)d.blocks_per_cu;
  t->xcd_remap = (int32_t)d.xcd_remap;
  t->use_hints = (int32_t)d.use_hints;
  t->stream = (int32_t)d.stream;
  t->bags_per_group = (int32_t)d.bags_per_group;
  t->xcd_pieces = (int32_t)d.xcd_pieces;
  t->per_table_launch = (int32_t)d.per_table_launch;
  t->fuse = (int32_t)d.fuse;
  t->bags_per_wave = (int32_t)d.bags_per_wave;
  t->hot_split = (int32_t)d.hot_split;
  t->station = (int32_t)d.station;
  return EMB_OK;
}

int emb_bag_set_tuning_table(const emb_bag_tuning_entry* entries, int32_t n) {
  if (n < 0 || n > kMaxTableEntries) return EMB_ERR_BAD_SIZE;
  if (n > 0 && !entries) return EMB_ERR_NULL_PTR;
  for (int32_t i = 0; i < n; ++i) {
    const emb_bag_tuning_entry& e = entries[i];
    const bool depth_ok = e.depth == 0 || e.depth == 1 || e.depth == 2 || e.depth == 4 ||
                          e.depth == 8 || e.depth == 16;
    if (e.max_row_bytes < 16 || !(e.max_avg_len >= 0.0f) || !depth_ok || e.bags_per_wave < 0 ||
        e.bags_per_wave > kWaveMaxBags || e.stream < -1 || e.stream > 1 || e.bags_per_group < 0 ||
        e.bags_per_group > 63)
      return EMB_ERR_BAD_TUNING;
  }
  for (int32_t i = 0; i < n; ++i) g_table[i] = entries[i];
  g_table_entries = n;
  return EMB_OK;
}

int emb_bag_get_tuning(const char* key, int64_t* value) {
  if (!key || !value) return EMB_ERR_NULL_PTR;
  if (!strcmp(key, "depth")) *value = g_tuning.depth;
  else if (!strcmp(key, "addressing")) *value = g_tuning.addressing;
  else if (!strcmp(key, "blocks_per_cu")) *value = g_tuning.blocks_per_cu;
  else if (!strcmp(key, "xcd_remap")) *value = g_tuning.xcd_remap;
  else if (!strcmp(key, "use_hints")) *value = g_tuning.use_hints;
  else if (!strcmp(key, "stream")) *value = g_tuning.stream;
  else if (!strcmp(key, "bags_per_group")) *value = g_tuning.bags_per_group;
  else if (!strcmp(key, "xcd_pieces")) *value = g_tuning.xcd_pieces;
  else if (!strcmp(key, "per_table_launch")) *value = g_tuning.per_table_launch;
  else if (!strcmp(key, "fuse")) *value = g_tuning.fuse;
  else if (!strcmp(key, "bags_per_wave")) *value = g_tuning.bags_per_wave;
  else if (!strcmp(key, "hot_split")) *value = g_tuning.hot_split;
  else if (!strcmp(key, "station")) *value = g_tuning.station;
  else return EMB_ERR_BAD_TUNING;
  return EMB_OK;
}

const char* emb_bag_status_string(int status) {
  switch (status) {
    case EMB_OK: return "ok";
    case EMB_ERR_NULL_PTR: return "a required pointer is NULL";
    case EMB_ERR_BAD_DIM: return "bad dim / row size / out_ld";
    case EMB_ERR_BAD_DTYPE: return "unknown table dtype";
    case EMB_ERR_BAD_MODE: return "unknown pooling mode";
    case EMB_ERR_UNSUPPORTED: return "per-sample weights are only supported with sum pooling";
    case EMB_ERR_LAUNCH: return "kernel launch failed";
    case EMB_ERR_BAD_SIZE: return "size negative or beyond the supported range";
    case EMB_ERR_ALIGNMENT: return "tables and out must be 16-byte aligned";
    case EMB_ERR_BAD_TUNING: return "unknown tuning key or value out of range";
    default: return "unknown status";
  }
}

int emb_bag_version(void) { return 600; }
}  // extern "C"
