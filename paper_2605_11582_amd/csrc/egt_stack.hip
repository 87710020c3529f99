// Several matrices of different shapes and storage forms in one launch.
//
// Sec. 3.3 starts from one kernel per linear layer, and Sec. 3.2 makes the decoder stack a
// layer-adaptive mix of storage forms.  A GEMV of a few megabytes is over in a few
// microseconds, about half of which is the fixed cost of a launch; this entry point pays
// that cost once for a whole table of products.  The grid is two-dimensional: blockIdx.y
// names the matrix, blockIdx.x the workgroup inside it (workgroups past a matrix's own
// count leave at once).  A workgroup reads the descriptor of its matrix - pointers, storage
// form, geometry - from a table in device memory that the caller owns, and then runs the
// very body the single-matrix kernels run (2:4, 1:4 or dense INT4), so every product has
// the bits of the separate call whenever the block shape is the same, and is otherwise
// within the accumulation-order difference of two equally valid block shapes.
//
// All workgroups of a launch have the same number of waves; it is chosen on the host so
// that every matrix's tiles per row ("phases") divide it.
#include "egt_n1_body.h"
#include "egt_stream_body.h"
#include "egt_tune.h"

#include <cstring>
#include <vector>

namespace egt {

// One matrix of a multi-matrix launch, as it lies in the caller's device table.
struct StackEntry {
  const uint32_t *row_ptr;
  const uint8_t *values;
  const uint8_t *idx;
  const uint8_t *qparams;
  const __half *x;
  __half *y;
  int32_t form, nblocks, tpi, reserved;
  union {
    M1Geom s24;
    M1N1Geom s14;
    DenseGeom dense;
  } g;
};
static_assert(sizeof(StackEntry) <= EGT_STACK_ENTRY_BYTES, "descriptor larger than the published entry size");

// FORMS: the storage forms present in the table (bit 0: 2:4, bit 1: 1:4, bit 2: dense); a
// launch carries only the bodies it needs, so that the registers of the widest body (1:4)
// do not limit the occupancy of a table without it.
template <int XP, int FORMS>
__global__ __launch_bounds__(1024) void k_gemv_stack(const uint8_t *__restrict__ table) {
  const StackEntry *e = (const StackEntry *)(table + (size_t)blockIdx.y * EGT_STACK_ENTRY_BYTES);
  if ((int)blockIdx.x >= e->nblocks) return;
  const int form = e->form, tpi = e->tpi;
  if ((FORMS & 1) && form == FORM_S24) {
    const M1Geom g = e->g.s24;
    if (tpi == 4) k_sparse_m1_body<EGT_VAL_INT4, 4, XP, 1, false, 1>(e->row_ptr, e->values, e->idx, e->qparams, e->x, e->y, g);
    else k_sparse_m1_body<EGT_VAL_INT4, 2, XP, 1, false, 1>(e->row_ptr, e->values, e->idx, e->qparams, e->x, e->y, g);
  } else if ((FORMS & 2) && form == FORM_S14) {
    const M1N1Geom g = e->g.s14;
    if (tpi == 4) k_sparse_m1_n1_body<EGT_VAL_INT4, 4, XP, 1, 0>(e->row_ptr, e->values, e->idx, e->qparams, e->x, e->y, g);
    else k_sparse_m1_n1_body<EGT_VAL_INT4, 2, XP, 1, 0>(e->row_ptr, e->values, e->idx, e->qparams, e->x, e->y, g);
  } else if ((FORMS & 4) && form == FORM_DENSE) {
    const DenseGeom g = e->g.dense;
    if (tpi == 8) k_int4_m1_body<8, XP, false>(e->values, e->qparams, e->x, e->y, g);
    else k_int4_m1_body<4, XP, false>(e->values, e->qparams, e->x, e->y, g);
  }
}

static_assert(sizeof(StreamItem) == 16, "item layout");
static_assert(sizeof(StreamMatrix) <= EGT_STACK_ENTRY_BYTES, "descriptor larger than the published entry size");
// Tiles in flight per wave.  Two 12-wave workgroups fit a compute unit only at 80 registers a
// lane or fewer (6 waves per SIMD); deeper rings (3 and 4) took 86 - 92 and left one workgroup
// resident: 590 us for the 7B stack against 520 with these.
#ifndef EGT_STREAM_DEPTH_S
#define EGT_STREAM_DEPTH_S 2
#endif
#ifndef EGT_STREAM_DEPTH_D
#define EGT_STREAM_DEPTH_D 3
#endif
constexpr int STREAM_DEPTH_S = EGT_STREAM_DEPTH_S;    // 2:4 (28 B per lane and tile)
constexpr int STREAM_DEPTH_D = EGT_STREAM_DEPTH_D;    // dense INT4 (20 B per lane and tile)
constexpr int DEVICE_CUS = 256;                       // compute units of an MI355X
// bytes of the per-workgroup first-item array of a table for `nblocks` resident workgroups
__host__ __device__ constexpr size_t stream_first_bytes(int nblocks) { return ((size_t)(nblocks + 1) * 4 + 15) & ~(size_t)15; }

// Resident workgroups walking the work items of a table (see egt_stream_body.h).  The table:
// `count` matrix descriptors, the first item of every workgroup (gridDim.x + 1 words, padded
// to 16 bytes), the items.
// (the second launch bound: waves per SIMD the register allocation has to leave room for - two
//  workgroups of 12 waves; with 8 pieces of x per thread, rows wider than 12288 columns, that
//  would spill, and one workgroup stays resident)
#ifndef EGT_STREAM_WAVES_PER_SIMD
#define EGT_STREAM_WAVES_PER_SIMD 6
#endif
// (1:4 tables, FORMS == 2: workgroups of 8 waves at up to 128 registers, two resident)
template <int XP, int FORMS>
__global__ __launch_bounds__(768, FORMS == 2 ? 4 : XP <= 4 ? EGT_STREAM_WAVES_PER_SIMD : 3) void k_gemv_stream(const uint8_t *__restrict__ table, int count, int part_offset,
                                                     int nthreads, int nblocks) {
  // (block and grid size come in as arguments: read through the dispatch packet they would
  //  be loaded again for every item)
  const uint8_t *first = table + (size_t)count * EGT_STACK_ENTRY_BYTES;
  const uint8_t *items = first + stream_first_bytes(nblocks);
  stream_body<XP, FORMS, STREAM_DEPTH_S, STREAM_DEPTH_D>(table, (const uint32_t *)first, (const StreamItem *)items,
                                                         EGT_STACK_ENTRY_BYTES, part_offset, nthreads);
}

bool sparse_m1_supported(const egt_2bitcsr &w);
bool sparse_m1_n1_supported(const egt_2bitcsr &w);
bool int4_m1_supported(int cols, int group);

namespace {

inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

struct ItemShape {
  int form, phases;
  egt_2bitcsr w;          // sparse items
  int rows, cols, group;  // dense items
};

// Storage form of an item, or an error.  The tuned bodies this launch shares with the
// single-matrix kernels take INT4 values with one {scale, zero} pair per chunk.
egt_status classify(const egt_gemv_item &it, ItemShape &s) {
  const int item_rows = it.sparse ? it.sparse->rows : it.rows;
  if (item_rows != 0 && (!it.x || !it.y)) return EGT_ERR_NULL;     // an empty matrix computes nothing
  if (!aligned16(it.x)) return EGT_ERR_BUFFER;
  if (it.sparse) {
    const egt_2bitcsr &w = *it.sparse;
    if (w.rows < 0 || w.cols <= 0 || w.cols % 32 != 0 || w.val_kind != EGT_VAL_INT4 || w.group_size <= 0 ||
        w.cols % w.group_size != 0)
      return (w.val_kind == EGT_VAL_FP16 || w.val_kind == EGT_VAL_INT4_PAIRED) ? EGT_ERR_UNSUPPORTED : EGT_ERR_SHAPE;
    if ((uint64_t)w.rows * (uint64_t)w.n_keep * (uint64_t)(w.cols / 4) >= (1ull << 32)) return EGT_ERR_SHAPE;
    if (w.rows > 0 && (!w.row_ptr || !w.values || !w.idx || !w.qparams)) return EGT_ERR_NULL;
    if (!aligned16(w.row_ptr) || !aligned16(w.values) || !aligned16(w.idx) || !aligned16(w.qparams)) return EGT_ERR_BUFFER;
    s.w = w;
    if (w.n_keep == 2 && sparse_m1_supported(w) && w.group_size >= 64) s.form = FORM_S24;
    else if (w.n_keep == 1 && sparse_m1_n1_supported(w) && w.group_size >= 128) s.form = FORM_S14;
    else return (w.n_keep < 0 || w.n_keep > 4) ? EGT_ERR_SHAPE : EGT_ERR_UNSUPPORTED;
    return EGT_OK;
  }
  if (it.rows < 0 || it.cols <= 0 || it.group <= 0 || it.group % 4 != 0 || it.cols % it.group != 0) return EGT_ERR_SHAPE;
  if (it.rows > 0 && (!it.q || !it.qparams)) return EGT_ERR_NULL;
  if (!aligned16(it.q) || !aligned16(it.qparams)) return EGT_ERR_BUFFER;
  if (!int4_m1_supported(it.cols, it.group) || it.group < 128) return EGT_ERR_UNSUPPORTED;
  s.form = FORM_DENSE;
  s.rows = it.rows; s.cols = it.cols; s.group = it.group;
  return EGT_OK;
}

}  // namespace
}  // namespace egt

namespace egt {
namespace {

// Resident-workgroup form: every matrix 2:4 (one tile per 4096 columns) or dense INT4 (one
// tile per 2048 columns) with whole tiles per wave, and enough bytes to keep the device busy
// for many times the life of a workgroup.  Fills entries, items and plan; false if the
// table does not qualify.
bool plan_stream(const egt_gemv_item *items, const std::vector<ItemShape> &shapes, const std::vector<StackEntry> &block_entries,
                 int count, int nwaves, bool whatever_the_size, std::vector<StreamMatrix> &mats, std::vector<uint32_t> &first,
                 std::vector<StreamItem> &work, egt_stack_part &plan) {
  std::vector<uint64_t> row_bytes_of;
  std::vector<int> rpt_of;
  int force = -1, bpc = 0, item_kb = 4096;
  tune_pair("EGT_STREAM_TUNE", force, bpc);             // developer build: 1 = whatever the size; workgroups per compute unit
  { int unused = 0; tune_pair("EGT_STREAM_ITEM", item_kb, unused); }
  if (force == 0 || nwaves == 0) return false;
  item_kb = item_kb < 16 ? 16 : item_kb > 4096 ? 4096 : item_kb;
  uint64_t total = 0;
  int forms = 0;
  size_t x_bytes = 0, part_floats = 0;
  int xp = 0;
  mats.assign((size_t)count, StreamMatrix{});
  work.clear();
  for (int k = 0; k < count; ++k) {
    const StackEntry &e = block_entries[k];
    StreamMatrix &m = mats[k];
    uint64_t row_bytes;
    int lds_pieces, pad_shift, rpt = 1;                 // rpt: rows of a tile (1:4 with short rows: 2 or 4)
    m.mr_shift = -1;
    if (e.form == FORM_S24) {
      const M1Geom &g = e.g.s24;
      if (g.mr_shift >= 0) return false;
      const egt_2bitcsr &w = shapes[k].w;
      m.row_ptr = w.row_ptr; m.values = (const uint8_t *)w.values; m.idx = (const uint8_t *)w.idx; m.qparams = (const uint8_t *)w.qparams;
      m.rows = g.rows; m.nchunks = g.nchunks; m.phases = g.phases; m.gshift = g.gshift; m.groups_per_row = g.groups_per_row;
      const uint64_t slots = (uint64_t)w.rows * 2u * (uint64_t)(w.cols / 4);
      m.val_bytes = (uint32_t)(slots / 2); m.idx_bytes = (uint32_t)(slots / 4);
      m.qp_bytes = (uint32_t)(4ull * (uint64_t)w.rows * (uint64_t)g.groups_per_row);
      row_bytes = (uint64_t)w.cols / 4 + w.cols / 8 + 4ull * g.groups_per_row;
      lds_pieces = g.phases * 512; pad_shift = 5;
    } else if (e.form == FORM_DENSE) {
      const DenseGeom &g = e.g.dense;
      if (g.mr_shift >= 0) return false;
      m.values = items[k].q; m.qparams = (const uint8_t *)items[k].qparams;
      m.rows = g.rows; m.nchunks = g.nchunks; m.phases = g.phases; m.gshift = g.gs; m.groups_per_row = g.groups_per_row;
      m.val_bytes = (uint32_t)((uint64_t)shapes[k].rows * (uint64_t)(shapes[k].cols / 2));
      m.qp_bytes = (uint32_t)(4ull * (uint64_t)shapes[k].rows * (uint64_t)g.groups_per_row);
      row_bytes = (uint64_t)shapes[k].cols / 2 + 4ull * g.groups_per_row;
      lds_pieces = g.phases * 256; pad_shift = 4;
    } else if (e.form == FORM_S14) {
      const M1N1Geom &g = e.g.s14;
      const egt_2bitcsr &w = shapes[k].w;
      m.row_ptr = w.row_ptr; m.values = (const uint8_t *)w.values; m.idx = (const uint8_t *)w.idx; m.qparams = (const uint8_t *)w.qparams;
      m.rows = g.rows; m.nchunks = g.nchunks; m.phases = g.phases; m.gshift = g.gshift; m.groups_per_row = g.groups_per_row;
      const uint64_t slots = (uint64_t)w.rows * (uint64_t)(w.cols / 4);
      m.val_bytes = (uint32_t)(slots / 2); m.idx_bytes = (uint32_t)(slots / 4);
      m.qp_bytes = (uint32_t)(4ull * (uint64_t)w.rows * (uint64_t)g.groups_per_row);
      row_bytes = (uint64_t)w.cols / 8 + w.cols / 16 + 4ull * g.groups_per_row;
      lds_pieces = g.mr_shift >= 0 ? g.nchunks * 16 : g.phases * 1024; pad_shift = 6;
      rpt = g.mr_shift >= 0 ? 64 >> g.mr_shift : 1;
      m.mr_shift = g.mr_shift;
    } else {
      return false;
    }
    m.form = e.form;
    m.x = (const __half *)items[k].x; m.y = (__half *)items[k].y;
    forms |= 1 << e.form;
    // rows of an item at most: what the partial sums of an item may take in LDS (24 KB), a
    // whole number of rows per wave
    const int wpp = nwaves / m.phases;
    int cap = (24 * 1024) / (16 * m.phases) * rpt;
    if (cap > STREAM_MAX_ITEM_ROWS) cap = STREAM_MAX_ITEM_ROWS;
    const uint64_t by_bytes = ((uint64_t)item_kb * 1024 + row_bytes - 1) / row_bytes;
    if ((uint64_t)cap > by_bytes) cap = (int)by_bytes;
    cap -= cap % (wpp * rpt);
    if (cap < wpp * rpt) return false;
    m.item_rows = cap;
    rpt_of.push_back(rpt);
    row_bytes_of.push_back(row_bytes);
    total += (uint64_t)m.rows * row_bytes;
    const size_t xb = 16 * (size_t)lds_pieces + 16 * (size_t)((lds_pieces + (1 << pad_shift) - 1) >> pad_shift);
    x_bytes = xb > x_bytes ? xb : x_bytes;
    const size_t pf = 4 * (size_t)m.phases * (size_t)(m.item_rows / rpt);
    part_floats = pf > part_floats ? pf : part_floats;
    const int need = (lds_pieces + 64 * nwaves - 1) / (64 * nwaves);
    xp = need > xp ? need : xp;
  }
  // smaller tables: one-shot workgroups are as fast or faster (20 MB: 6.9 against 7.4 us; 37 MB: 9.8 against 9.5;
  // 48 MB: 13.1 against 11.4; a decoder layer of 83 MB: 23.6 against 17.7)
  if (force != 1 && !whatever_the_size && total < (32ull << 20)) return false;
  if (xp > 8 || total == 0) return false;
  const size_t lds = x_bytes + sizeof(float) * part_floats;
  if (lds > 64 * 1024) return false;
  // spans of equal byte count, one per workgroup, in table order: workgroup b streams the
  // bytes [b, b + 1) * total / blocks of the concatenated matrices (cut at row boundaries)
  // Two to eight workgroups per compute unit, two of them resident at a time: spans of about
  // 1.4 MB (x is staged once per item, so a span should hold many rows; shorter spans finish
  // more evenly: the 3 GB stack takes 546 us with 512 spans, 530 with 1024, 520 with 2048).
  // below 72 MB one span per compute unit
  // (1:4: two at least - its workgroups have 8 waves, and one per compute unit would leave half the waves out)
  if (bpc < 1) { bpc = (int)((total + (179ull << 20)) / (358ull << 20)); bpc = (total < (72ull << 20) && forms != 2) ? 1 : bpc < 2 ? 2 : bpc; }
  bpc = bpc < 1 ? 1 : bpc > 8 ? 8 : bpc;
  int blocks = DEVICE_CUS * bpc;
  first.assign(1, 0u);
  uint64_t done = 0;                                   // bytes of the rows handed out so far
  for (int k = 0; k < count; ++k) {
    const StreamMatrix &m = mats[k];
    const uint64_t rb = row_bytes_of[k];
    int r = 0;
    while (r < m.rows) {
      const int b = (int)first.size() - 1;             // workgroup being filled
      const uint64_t budget_end = (total * (uint64_t)(b + 1) + (uint64_t)blocks - 1) / (uint64_t)blocks;
      uint64_t room_rows = budget_end > done ? (budget_end - done + rb - 1) / rb : 0;
      if (room_rows == 0 && b + 1 < blocks) { first.push_back((uint32_t)work.size()); continue; }
      int n = m.rows - r;
      if ((uint64_t)n > room_rows && b + 1 < blocks) n = (int)room_rows;
      if (n > m.item_rows) n = m.item_rows;
      if (n % rpt_of[k]) n += rpt_of[k] - n % rpt_of[k];                     // an item starts on a tile (item_rows is a multiple)
      if (n > m.rows - r) n = m.rows - r;
      work.push_back(StreamItem{(uint32_t)k, (uint32_t)r, (uint32_t)n, 0u});
      r += n;
      done += (uint64_t)n * rb;
    }
  }
  while ((int)first.size() < blocks + 1) first.push_back((uint32_t)work.size());
  first.back() = (uint32_t)work.size();
  if (work.empty() || work.size() > 0x7FFFFFFFull) return false;
  plan.mode = 1;
  plan.grid_x = blocks;
  plan.block_threads = 64 * nwaves;
  plan.lds_bytes = (int32_t)lds;
  plan.x_pieces = xp <= 2 ? 2 : xp <= 4 ? 4 : 8;
  plan.forms = forms;
  plan.nitems = (int32_t)work.size();
  plan.part_offset = (int32_t)x_bytes;
  plan.table_bytes = (uint64_t)count * EGT_STACK_ENTRY_BYTES + stream_first_bytes(blocks) + sizeof(StreamItem) * (uint64_t)work.size();
  return true;
}

}  // namespace
}  // namespace egt

namespace egt {
namespace {

// Plans one part: `count` classified items that share a kernel.
egt_status plan_part(const egt_gemv_item *items, int count, int form, void *table, size_t table_bytes, egt_stack_part *plan) {
  std::vector<ItemShape> shapes((size_t)count);
  std::vector<StackEntry> entries((size_t)count);
  // pass 1: storage form and tiles per row ("phases") of every item
  for (int k = 0; k < count; ++k) {
    const egt_status st = classify(items[k], shapes[k]);
    if (st != EGT_OK) return st;
    StackEntry &e = entries[k];
    std::memset(&e, 0, sizeof(e));
    e.form = shapes[k].form;
    if (e.form == FORM_S24) { m1_geometry(shapes[k].w, e.g.s24); shapes[k].phases = e.g.s24.phases; }
    else if (e.form == FORM_S14) { int ni; n1_geometry(shapes[k].w, false, e.g.s14, ni); shapes[k].phases = e.g.s14.phases; }
    else { bool pre; dense_geometry(shapes[k].rows, shapes[k].cols, shapes[k].group, e.g.dense, pre); shapes[k].phases = e.g.dense.phases; }
  }
  // waves per workgroup: the smallest of 4, 6, 8, 12, 16 that every item's phases divide
  // (6 for the 7B shapes: 1, 2, 3 and 6 tiles per row)
  int nwaves = 0, want = 0, tpi_mode = 3;
  tune_pair("EGT_STACK_TUNE", want, tpi_mode);           // developer build: at least that many waves; tiles per wave
  for (int cand : {4, 6, 8, 12, 16}) {
    bool ok = cand >= want;
    for (int k = 0; k < count && ok; ++k) ok = cand % shapes[k].phases == 0;
    if (ok) { nwaves = cand; break; }
  }
  if (nwaves == 0) return EGT_ERR_UNSUPPORTED;

  egt_stack_part out;
  std::memset(&out, 0, sizeof(out));
  out.count = count;
  std::vector<StreamMatrix> mats;
  std::vector<StreamItem> work;
  std::vector<uint32_t> first;
  // streaming workgroups: the largest of 12, 8, 6, 4 waves that every item's phases divide (two
  // workgroups resident per compute unit; a big workgroup stages x once for many rows)
  // (1:4 matrices: 8 waves at most, so that two workgroups fit the registers of their body)
  int swaves = 0, swant = 12, sunused = 0;
  tune_pair("EGT_STREAM_WAVES", swant, sunused);
  if (shapes[0].form == FORM_S14 && swant > 8) swant = 8;
  for (int cand : {12, 8, 6, 4}) {
    bool ok = cand <= swant;
    for (int k = 0; k < count && ok; ++k) ok = cand % shapes[k].phases == 0;
    if (ok) { swaves = cand; break; }
  }
  const bool stream = form != EGT_STACK_GRID &&
                      plan_stream(items, shapes, entries, count, swaves, form == EGT_STACK_RESIDENT, mats, first, work, out);
  if (form == EGT_STACK_RESIDENT && !stream) return EGT_ERR_UNSUPPORTED;
  if (stream) nwaves = swaves;
  if (!stream) {
    // one grid of one-shot workgroups per matrix: block shape of every item at that many
    // waves.  Rows of three tiles take four tiles per wave here (two in the single-matrix
    // launch) and dense rows eight (four): a workgroup is short-lived, so it should carry as
    // many bytes as its registers allow.
    int grid_x = 0, xp = 0, forms = 0;
    size_t lds = 0;
    for (int k = 0; k < count; ++k) {
      StackEntry &e = entries[k];
      const egt_gemv_item &it = items[k];
      LaunchShape ls;
      bool ok;
      if (e.form == FORM_S24) {
        ok = m1_block_shape(e.g.s24, false, nwaves / shapes[k].phases, (shapes[k].phases == 3 && !(tpi_mode & 1)) ? 2 : 4, 1, 8, ls);
      } else if (e.form == FORM_S14) {
        ok = n1_block_shape(e.g.s14, false, 0, nwaves / shapes[k].phases, shapes[k].phases == 1 ? 2 : 4, 8, ls);
      } else {
        ok = dense_block_shape(e.g.dense, nwaves / shapes[k].phases, (tpi_mode & 2) ? 8 : 4, 8, ls);
      }
      if (!ok || ls.lds > 64 * 1024) return EGT_ERR_UNSUPPORTED;
      const int rows = e.form == FORM_DENSE ? shapes[k].rows : shapes[k].w.rows;
      e.nblocks = rows == 0 ? 0 : ls.nblocks;
      e.tpi = ls.tpi;
      if (e.form == FORM_DENSE) {
        e.values = it.q; e.qparams = (const uint8_t *)it.qparams;
      } else {
        e.row_ptr = shapes[k].w.row_ptr; e.values = (const uint8_t *)shapes[k].w.values;
        e.idx = (const uint8_t *)shapes[k].w.idx; e.qparams = (const uint8_t *)shapes[k].w.qparams;
      }
      e.x = (const __half *)it.x; e.y = (__half *)it.y;
      forms |= 1 << e.form;
      grid_x = e.nblocks > grid_x ? e.nblocks : grid_x;
      xp = ls.xp > xp ? ls.xp : xp;
      lds = ls.lds > lds ? ls.lds : lds;
    }
    out.mode = 0;
    out.grid_x = grid_x;
    out.block_threads = 64 * nwaves;
    out.lds_bytes = (int32_t)lds;
    out.x_pieces = xp <= 2 ? 2 : xp <= 4 ? 4 : 8;
    out.forms = forms;
    out.nitems = 0;
    out.part_offset = 0;
    out.table_bytes = (uint64_t)count * EGT_STACK_ENTRY_BYTES;
  }
  if (table) {
    if ((uint64_t)table_bytes < out.table_bytes) return EGT_ERR_SHAPE;
    uint8_t *dst = (uint8_t *)table;
    std::memset(dst, 0, (size_t)out.table_bytes);
    for (int k = 0; k < count; ++k) {
      if (stream) std::memcpy(dst + (size_t)k * EGT_STACK_ENTRY_BYTES, &mats[k], sizeof(StreamMatrix));
      else std::memcpy(dst + (size_t)k * EGT_STACK_ENTRY_BYTES, &entries[k], sizeof(StackEntry));
    }
    if (stream) {
      uint8_t *f = dst + (size_t)count * EGT_STACK_ENTRY_BYTES;
      std::memcpy(f, first.data(), sizeof(uint32_t) * first.size());
      std::memcpy(f + stream_first_bytes(out.grid_x), work.data(), sizeof(StreamItem) * work.size());
    }
  }
  *plan = out;
  return EGT_OK;
}

}  // namespace
}  // namespace egt

extern "C" {

egt_status egt_gemv_stack_plan(const egt_gemv_item *items, int count, int form, void *table, size_t table_bytes,
                               egt_stack_plan *plan) {
  using namespace egt;
  if (!items || !plan) return EGT_ERR_NULL;
  if (count < 1 || count > 65535 || form < EGT_STACK_AUTO || form > EGT_STACK_RESIDENT) return EGT_ERR_SHAPE;
  // the 1:4 matrices of a table that holds others too run as a launch of their own
  std::vector<egt_gemv_item> group[EGT_STACK_MAX_PARTS];
  for (int k = 0; k < count; ++k) {
    ItemShape shape;
    const egt_status st = classify(items[k], shape);
    if (st != EGT_OK) return st;
    group[shape.form == FORM_S14 ? 1 : 0].push_back(items[k]);
  }
  if (group[0].empty()) group[0].swap(group[1]);
  egt_stack_plan out;
  std::memset(&out, 0, sizeof(out));
  out.count = count;
  // size query of every part first: nothing is written when a part is in error
  for (int p = 0; p < EGT_STACK_MAX_PARTS && !group[p].empty(); ++p) {
    const egt_status st = plan_part(group[p].data(), (int)group[p].size(), form, nullptr, 0, &out.part[p]);
    if (st != EGT_OK) return st;
    out.table_bytes += (out.part[p].table_bytes + 15) & ~(uint64_t)15;
    out.nparts = p + 1;
  }
  if (table) {
    if ((uint64_t)table_bytes < out.table_bytes) return EGT_ERR_SHAPE;
    uint64_t at = 0;
    for (int p = 0; p < out.nparts; ++p) {
      const egt_status st = plan_part(group[p].data(), (int)group[p].size(), form, (uint8_t *)table + at,
                                      (size_t)out.part[p].table_bytes, &out.part[p]);
      if (st != EGT_OK) return st;
      at += (out.part[p].table_bytes + 15) & ~(uint64_t)15;
    }
  }
  *plan = out;
  return EGT_OK;
}

static egt_status run_part(const uint8_t *t, const egt_stack_part *plan, hipStream_t st);

egt_status egt_gemv_stack_run(const void *table_dev, const egt_stack_plan *plan, void *stream) {
  using namespace egt;
  if (!table_dev || !plan) return EGT_ERR_NULL;
  if (!aligned16(table_dev)) return EGT_ERR_BUFFER;
  if (plan->nparts < 1 || plan->nparts > EGT_STACK_MAX_PARTS) return EGT_ERR_SHAPE;
  uint64_t at = 0;
  int total = 0;
  for (int p = 0; p < plan->nparts; ++p) {           // every part is checked before the first is launched
    const egt_stack_part &q = plan->part[p];
    if (q.count < 1 || q.count > 65535 || q.grid_x < 0 || q.block_threads < 64 || q.block_threads > 1024 ||
        q.block_threads % 64 != 0 || q.lds_bytes < 0 || q.lds_bytes > 64 * 1024 ||
        (q.x_pieces != 2 && q.x_pieces != 4 && q.x_pieces != 8) || q.mode < 0 || q.mode > 1 ||
        (q.forms != 1 && q.forms != 2 && q.forms != 4 && q.forms != 5))   // 2:4 and dense together, 1:4 alone
      return EGT_ERR_SHAPE;
    if (q.mode == 0 && q.table_bytes != (uint64_t)q.count * EGT_STACK_ENTRY_BYTES) return EGT_ERR_SHAPE;
    if (q.mode == 1 && (q.nitems < 1 || q.grid_x < 1 || q.grid_x > 8 * DEVICE_CUS || q.block_threads > (q.forms == 2 ? 512 : 768) ||
                        q.part_offset < 0 || q.part_offset > q.lds_bytes ||
                        q.table_bytes != (uint64_t)q.count * EGT_STACK_ENTRY_BYTES + stream_first_bytes(q.grid_x) +
                                             16ull * (uint64_t)q.nitems))
      return EGT_ERR_SHAPE;
    at += (q.table_bytes + 15) & ~(uint64_t)15;
    total += q.count;
  }
  if (at != plan->table_bytes || total != plan->count) return EGT_ERR_SHAPE;
  at = 0;
  for (int p = 0; p < plan->nparts; ++p) {
    const egt_status st = run_part((const uint8_t *)table_dev + at, &plan->part[p], (hipStream_t)stream);
    if (st != EGT_OK) return st;
    at += (plan->part[p].table_bytes + 15) & ~(uint64_t)15;
  }
  return EGT_OK;
}

static egt_status run_part(const uint8_t *t, const egt_stack_part *plan, hipStream_t st) {
  using namespace egt;
  if (plan->grid_x == 0) return EGT_OK;               // every matrix is empty
  const size_t lds = (size_t)plan->lds_bytes;
  const dim3 block(plan->block_threads);
  hipError_t e;
  if (plan->mode == 1) {
    const dim3 grid(plan->grid_x);
#define EGT_STREAM_GO(XP)                                                                                    \
  (plan->forms == 1 ? launch(k_gemv_stream<XP, 1>, grid, block, lds, st, t, plan->count, plan->part_offset, plan->block_threads, plan->grid_x) \
   : plan->forms == 2 ? launch(k_gemv_stream<XP, 2>, grid, block, lds, st, t, plan->count, plan->part_offset, plan->block_threads, plan->grid_x) \
   : plan->forms == 4 ? launch(k_gemv_stream<XP, 4>, grid, block, lds, st, t, plan->count, plan->part_offset, plan->block_threads, plan->grid_x) \
                      : launch(k_gemv_stream<XP, 5>, grid, block, lds, st, t, plan->count, plan->part_offset, plan->block_threads, plan->grid_x))
    switch (plan->x_pieces) {
      case 2: e = EGT_STREAM_GO(2); break;
      case 4: e = EGT_STREAM_GO(4); break;
      default: e = EGT_STREAM_GO(8); break;
    }
#undef EGT_STREAM_GO
  } else {
    // (a part holds 2:4 and dense matrices, or 1:4 matrices)
    const dim3 grid(plan->grid_x, plan->count);
#define EGT_STACK_GO(XP)                                                                         \
  (plan->forms == 1 ? launch(k_gemv_stack<XP, 1>, grid, block, lds, st, t)                        \
   : plan->forms == 2 ? launch(k_gemv_stack<XP, 2>, grid, block, lds, st, t)                      \
   : plan->forms == 4 ? launch(k_gemv_stack<XP, 4>, grid, block, lds, st, t)                      \
                      : launch(k_gemv_stack<XP, 5>, grid, block, lds, st, t))
    switch (plan->x_pieces) {
      case 2: e = EGT_STACK_GO(2); break;
      case 4: e = EGT_STACK_GO(4); break;
      default: e = EGT_STACK_GO(8); break;
    }
#undef EGT_STACK_GO
  }
  if (e == hipSuccess) return EGT_OK;
  note_hip_error(e);
  return EGT_ERR_HIP;
}

}  // extern "C"
