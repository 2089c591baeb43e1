// Host side of the chunk-alignment table (paper section 3.5): packs -> chunks -> segments,
// the canonical serialisation, and the device image with the tile work lists.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cstring>
#include <new>

#include "mux_internal.h"

namespace mux {

static thread_local std::string g_err;

mux_status fail(mux_status s, const std::string& msg) {
  g_err = msg;
  return s;
}
void clear_error() { g_err.clear(); }

}  // namespace mux

using namespace mux;

extern "C" const char* mux_last_error(void) { return g_err.c_str(); }
extern "C" const char* mux_version(void) { return "muxlora-gfx950 0.1"; }

extern "C" mux_status mux_choose_chunk_size(const int32_t* lens, int32_t n, int32_t floor_, int32_t* out) {
  if (!out || n < 0 || (n > 0 && !lens) || floor_ < 1) return fail(MUX_ERR_INVALID_ARG, "mux_choose_chunk_size: bad argument");
  uint32_t all = 0;  // OR of the lengths: its lowest set bit is the greatest common power-of-two divisor
  for (int32_t i = 0; i < n; ++i)
    if (lens[i] > 0) all |= (uint32_t)lens[i];
  int32_t p = all ? (int32_t)(all & (~all + 1u)) : floor_;
  *out = p < floor_ ? floor_ : p;
  return MUX_OK;
}

namespace {
struct Pack { int32_t task, row_begin, valid, chunk_begin, chunk_count, seg_begin; };
struct Seg { int32_t task, pack, chunk, row_begin, n_rows, index_in_pack; };
struct Seq { int32_t task, pack, first_row, len; };
struct Chunk { int32_t valid = 0, seg_begin = 0, seg_count = 0, first_task = -1; };
}  // namespace

extern "C" mux_status mux_segtab_build(const mux_task_desc* tasks, int32_t n_tasks, int32_t chunk,
                                       int32_t max_pack_len, uint32_t flags, mux_segtab** out) {
  if (!out) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: out is null");
  *out = nullptr;
  if (n_tasks < 0 || n_tasks > MUX_MAX_TASKS || (n_tasks > 0 && !tasks))
    return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: bad task array");
  if (chunk < 1 || (chunk & (chunk - 1)) != 0) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: chunk must be a power of two");
  if (max_pack_len < 0) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: max_pack_len < 0");
  if (flags & ~MUX_SEGTAB_DENSE) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: unknown flag");
  int64_t total = 0;
  for (int32_t t = 0; t < n_tasks; ++t) {
    const mux_task_desc& d = tasks[t];
    if (d.kind != MUX_ADAPTER_NONE && d.kind != MUX_ADAPTER_LORA && d.kind != MUX_ADAPTER_IA3_OUT && d.kind != MUX_ADAPTER_TUNING &&
        d.kind != MUX_ADAPTER_DIFF)
      return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: unknown adapter kind");
    if ((d.kind == MUX_ADAPTER_LORA || d.kind == MUX_ADAPTER_TUNING) && (d.rank < 1 || d.rank > MUX_MAX_RANK))
      return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: adapter rank outside 1..MUX_MAX_RANK");
    if (d.n_seqs < 0 || (d.n_seqs > 0 && !d.seq_lens)) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: bad seq_lens");
    for (int32_t s = 0; s < d.n_seqs; ++s) {
      if (d.seq_lens[s] < 1) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_build: sequence length < 1");
      total += d.seq_lens[s];
    }
  }
  // padding adds < chunk rows per pack and there is at most one pack per sequence
  if (total + (int64_t)chunk * (total + 1) > (int64_t)1 << 40 || total > ((int64_t)1 << 30))
    return fail(MUX_ERR_SHAPE, "mux_segtab_build: too many tokens");

  mux_segtab* st = new (std::nothrow) mux_segtab();
  if (!st) return fail(MUX_ERR_HOST_NOMEM, "mux_segtab_build: out of host memory");
  try {
    const bool dense = (flags & MUX_SEGTAB_DENSE) != 0;
    const int64_t c = chunk;
    std::vector<Pack> packs;
    std::vector<Seg> segs;
    std::vector<Seq> seqs;
    std::vector<int32_t> timg;  // per-task words of the canonical image
    st->tasks.resize(n_tasks);
    int64_t cur = 0;            // next free row
    int32_t zrows = 0, drows = 0;
    for (int32_t t = 0; t < n_tasks; ++t) {
      const mux_task_desc& d = tasks[t];
      const int64_t task_row_begin = cur;
      const int32_t pack_begin = (int32_t)packs.size(), seq_begin = (int32_t)seqs.size();
      const int32_t seg_begin_task = (int32_t)segs.size();
      int64_t valid = 0;
      int32_t s = 0;
      while (s < d.n_seqs) {
        // step 1: one pack = a maximal in-order run of sequences within max_pack_len
        int64_t len = d.seq_lens[s];
        int32_t e = s + 1;
        while (e < d.n_seqs && (max_pack_len == 0 || len + d.seq_lens[e] <= max_pack_len)) len += d.seq_lens[e++];
        const int32_t p = (int32_t)packs.size();
        const int64_t rb = cur;
        int64_t r = rb;
        for (int32_t q = s; q < e; ++q) {
          seqs.push_back({t, p, (int32_t)r, d.seq_lens[q]});
          r += d.seq_lens[q];
        }
        // step 2: the pack's rows cut along the chunk grid
        Pack pk{t, (int32_t)rb, (int32_t)len, (int32_t)(rb / c), 0, (int32_t)segs.size()};
        int32_t piece = 0;
        for (int64_t a = rb; a < rb + len;) {
          const int64_t chunk_end = (a / c + 1) * c;
          const int64_t b = chunk_end < rb + len ? chunk_end : rb + len;
          segs.push_back({t, p, (int32_t)(a / c), (int32_t)a, (int32_t)(b - a), piece++});
          a = b;
        }
        pk.chunk_count = piece;
        packs.push_back(pk);
        valid += len;
        cur = dense ? rb + len : (rb + len + c - 1) / c * c;
        s = e;
      }
      const int32_t n_seg_task = (int32_t)segs.size() - seg_begin_task;
      const int32_t chunk_begin = n_seg_task ? segs[seg_begin_task].chunk : (int32_t)(task_row_begin / c);
      const int32_t chunk_count = n_seg_task ? segs.back().chunk - chunk_begin + 1 : 0;
      const int32_t words[8] = {(int32_t)task_row_begin, (int32_t)(cur - task_row_begin), (int32_t)valid, chunk_begin,
                                chunk_count, pack_begin, (int32_t)packs.size() - pack_begin, seq_begin};
      timg.insert(timg.end(), words, words + 8);
      HostTask& ht = st->tasks[t];
      ht.kind = d.kind;
      const bool ranked = d.kind == MUX_ADAPTER_LORA || d.kind == MUX_ADAPTER_TUNING;
      ht.rank = ranked ? d.rank : 0;
      ht.scale = ranked ? d.scale : 1.0f;
      ht.row_begin = (int32_t)task_row_begin;
      ht.row_count = (int32_t)(cur - task_row_begin);
      ht.valid = (int32_t)valid;
      ht.zrow0 = -1;
      // x W is kept for the backward pass of the kinds that need it: its rows are numbered task by task
      if (d.kind == MUX_ADAPTER_IA3_OUT || d.kind == MUX_ADAPTER_TUNING) { ht.zrow0 = zrows; zrows += ht.row_count; }
      // the rows of the Diff-Pruning tasks are copied in transposed blocks of 64 rows: numbered task by task, a block
      // never holds rows of two tasks
      if (d.kind == MUX_ADAPTER_DIFF) { ht.zrow0 = drows; drows += (ht.row_count + 63) / 64 * 64; }
      if (d.kind == MUX_ADAPTER_IA3_OUT) st->n_ia3++;
      if (d.kind == MUX_ADAPTER_TUNING) st->n_tuning++;
      if (d.kind == MUX_ADAPTER_DIFF) st->n_diff++;
      if (d.kind == MUX_ADAPTER_LORA) st->n_lora++;
      if (ranked && d.rank > st->r_max) st->r_max = d.rank;
    }
    const int64_t T = (cur + c - 1) / c * c;
    if (T > ((int64_t)1 << 30)) { delete st; return fail(MUX_ERR_SHAPE, "mux_segtab_build: too many rows"); }
    st->n_tasks = n_tasks;
    st->chunk = chunk;
    st->log2c = __builtin_ctz((unsigned)chunk);
    st->n_chunks = (int32_t)(T / c);
    st->T = (int32_t)T;
    st->valid_total = (int32_t)total;
    st->max_pack_len = max_pack_len;
    st->flags = flags;
    st->z_rows = zrows;
    st->d_rows = drows;

    std::vector<Chunk> chunks(st->n_chunks);
    for (size_t k = 0; k < segs.size(); ++k) {
      Chunk& ch = chunks[segs[k].chunk];
      if (ch.seg_count == 0) { ch.seg_begin = (int32_t)k; ch.first_task = segs[k].task; }
      ch.seg_count++;
      ch.valid += segs[k].n_rows;
    }
    for (size_t k = 1; k < chunks.size(); ++k)   // a chunk without segments cannot occur, but keep seg_begin monotone
      if (chunks[k].seg_count == 0) chunks[k].seg_begin = chunks[k - 1].seg_begin + chunks[k - 1].seg_count;

    // ---- canonical image
    std::vector<int32_t>& img = st->image;
    const int32_t hdr[16] = {0x5458554D, 1, (int32_t)flags, n_tasks, chunk, max_pack_len, st->n_chunks, st->T,
                             st->valid_total, (int32_t)packs.size(), (int32_t)segs.size(), (int32_t)seqs.size(), 0, 0, 0, 0};
    img.insert(img.end(), hdr, hdr + 16);
    img.insert(img.end(), timg.begin(), timg.end());
    for (const Pack& p : packs) { const int32_t w[6] = {p.task, p.row_begin, p.valid, p.chunk_begin, p.chunk_count, p.seg_begin}; img.insert(img.end(), w, w + 6); }
    for (const Chunk& ch : chunks) { const int32_t w[4] = {ch.valid, ch.seg_begin, ch.seg_count, ch.first_task}; img.insert(img.end(), w, w + 4); }
    for (const Seg& s : segs) { const int32_t w[6] = {s.task, s.pack, s.chunk, s.row_begin, s.n_rows, s.index_in_pack}; img.insert(img.end(), w, w + 6); }
    for (const Seq& s : seqs) { const int32_t w[4] = {s.task, s.pack, s.first_row, s.len}; img.insert(img.end(), w, w + 4); }

    // ---- row -> task
    st->row_task.assign(st->T, -1);
    for (const Seg& s : segs)
      for (int32_t i = 0; i < s.n_rows; ++i) st->row_task[s.row_begin + i] = s.task;

    // ---- tile work lists: every row of the batch is covered exactly once, an item never mixes tasks
    std::vector<int32_t> valid_prefix(st->T + 1, 0);
    for (int32_t i = 0; i < st->T; ++i) valid_prefix[i + 1] = valid_prefix[i] + (st->row_task[i] >= 0 ? 1 : 0);
    for (int ts = 0; ts < kNumTileSizes; ++ts) {
      const int32_t R = kTileRows[ts];
      std::vector<Item>& items = st->items[ts];
      st->task_item_begin[ts].assign(n_tasks, 0);
      st->task_item_count[ts].assign(n_tasks, 0);
      int32_t covered = 0;
      auto emit = [&](int32_t task, int32_t r0, int32_t r1) {
        for (int32_t a = r0; a < r1; a += R) {
          const int32_t b = a + R < r1 ? a + R : r1;
          items.push_back({task, a, b - a, valid_prefix[b] - valid_prefix[a]});
        }
      };
      for (int32_t t = 0; t < n_tasks; ++t) {
        const HostTask& ht = st->tasks[t];
        if (ht.row_begin > covered) emit(-1, covered, ht.row_begin);
        st->task_item_begin[ts][t] = (int32_t)items.size();
        emit(t, ht.row_begin, ht.row_begin + ht.row_count);
        st->task_item_count[ts][t] = (int32_t)items.size() - st->task_item_begin[ts][t];
        if (ht.row_begin + ht.row_count > covered) covered = ht.row_begin + ht.row_count;
      }
      if (covered < st->T) emit(-1, covered, st->T);
    }

    // ---- device image
    std::vector<int32_t>& dv = st->dev_image;
    dv.assign(DH_HDR_WORDS, 0);
    dv[DH_MAGIC] = (int32_t)kDevMagic;
    dv[DH_T] = st->T; dv[DH_CHUNK] = chunk; dv[DH_LOG2C] = st->log2c; dv[DH_NTASKS] = n_tasks; dv[DH_NCHUNKS] = st->n_chunks;
    dv[DH_ZROWS] = zrows; dv[DH_RMAX] = st->r_max;
    dv[DH_OFF_TASKS] = (int32_t)dv.size();
    for (int32_t t = 0; t < n_tasks; ++t) {
      const HostTask& ht = st->tasks[t];
      int32_t sb; std::memcpy(&sb, &ht.scale, 4);
      const int32_t w[DT_WORDS] = {ht.row_begin, ht.row_count, ht.valid, ht.kind, ht.rank, sb, ht.zrow0, 0};
      dv.insert(dv.end(), w, w + DT_WORDS);
    }
    dv[DH_OFF_CHUNK_VALID] = (int32_t)dv.size();
    for (const Chunk& ch : chunks) dv.push_back(ch.valid);
    for (int ts = 0; ts < kNumTileSizes; ++ts) {
      dv[DH_NITEMS0 + 3 * ts + 0] = (int32_t)st->items[ts].size();
      dv[DH_NITEMS0 + 3 * ts + 1] = (int32_t)dv.size();
      for (const Item& it : st->items[ts]) { const int32_t w[DI_WORDS] = {it.task, it.row0, it.nrows, it.nvalid}; dv.insert(dv.end(), w, w + DI_WORDS); }
      dv[DH_NITEMS0 + 3 * ts + 2] = (int32_t)dv.size();
      for (int32_t t = 0; t < n_tasks; ++t) { dv.push_back(st->task_item_begin[ts][t]); dv.push_back(st->task_item_count[ts][t]); }
    }
    // one bit per row (1 = real token), 32 rows per word, one spare word so that two-word windows never run out
    dv[DH_OFF_ROWBITS] = (int32_t)dv.size();
    {
      const size_t words = (size_t)(st->T + 31) / 32 + 1;
      const size_t base = dv.size();
      dv.resize(base + words, 0);
      for (int32_t i = 0; i < st->T; ++i)
        if (st->row_task[i] >= 0) dv[base + (i >> 5)] |= (int32_t)(1u << (i & 31));
    }
    // validity bits of the rows of every 64-row item, two words an item (bit r of the pair = row row0 + r is a real token)
    {
      dv[DH_OFF_ITEM_BITS] = (int32_t)dv.size();
      for (const Item& it : st->items[0]) {
        uint32_t w[2] = {0u, 0u};
        for (int32_t r = 0; r < it.nrows; ++r)
          if (st->row_task[it.row0 + r] >= 0) w[r >> 5] |= 1u << (r & 31);
        dv.push_back((int32_t)w[0]);
        dv.push_back((int32_t)w[1]);
      }
    }
    // Dispatch: the packed position of a task's token = the number of the task's tokens on the rows before it
    {
      dv[DH_OFF_ITEM_TOK0] = (int32_t)dv.size();
      std::vector<int32_t> seen(n_tasks, 0);
      for (const Item& it : st->items[0]) {
        dv.push_back(it.task >= 0 ? seen[it.task] : 0);
        if (it.task >= 0) seen[it.task] += it.nvalid;
      }
    }
    // attention work lists: every sequence cut into blocks of 128 tokens.  A block of queries walks the keys of its
    // sequence up to its own end, a block of keys the queries from its own start on.  Both lists keep the blocks of
    // a sequence together (they share its keys and values in the L2), longest sequence first and inside a sequence
    // the longest walk first, so that the last items of a launch are the short ones.
    {
      struct Blk { int32_t first_row, len, b0; };
      std::vector<Seq> order(seqs.begin(), seqs.end());
      std::stable_sort(order.begin(), order.end(), [](const Seq& a, const Seq& b) { return a.len > b.len; });
      std::vector<Blk> fwd, bwd;
      for (const Seq& sq : order) {
        const int32_t nb = (sq.len + kAttnBlockRows - 1) / kAttnBlockRows;
        for (int32_t b = nb - 1; b >= 0; --b) fwd.push_back({sq.first_row, sq.len, b * kAttnBlockRows});
        for (int32_t b = 0; b < nb; ++b) bwd.push_back({sq.first_row, sq.len, b * kAttnBlockRows});
      }
      st->n_attn_blocks = (int32_t)fwd.size();
      dv[DH_ATT_NBLK] = st->n_attn_blocks;
      dv[DH_ATT_OFF_FWD] = (int32_t)dv.size();
      for (const Blk& b : fwd) { const int32_t w[DA_WORDS] = {b.first_row, b.len, b.b0, 0}; dv.insert(dv.end(), w, w + DA_WORDS); }
      dv[DH_ATT_OFF_BWD] = (int32_t)dv.size();
      for (const Blk& b : bwd) { const int32_t w[DA_WORDS] = {b.first_row, b.len, b.b0, 0}; dv.insert(dv.end(), w, w + DA_WORDS); }
    }
    while (dv.size() % 64) dv.push_back(0);
    dv[DH_WORDS] = (int32_t)dv.size();
  } catch (const std::bad_alloc&) {
    delete st;
    return fail(MUX_ERR_HOST_NOMEM, "mux_segtab_build: out of host memory");
  }
  *out = st;
  return MUX_OK;
}

extern "C" void mux_segtab_free(mux_segtab* st) { delete st; }
extern "C" int32_t mux_segtab_rows(const mux_segtab* st) { return st ? st->T : -1; }
extern "C" int32_t mux_segtab_n_chunks(const mux_segtab* st) { return st ? st->n_chunks : -1; }
extern "C" int32_t mux_segtab_n_tasks(const mux_segtab* st) { return st ? st->n_tasks : -1; }
extern "C" int32_t mux_segtab_valid_tokens(const mux_segtab* st) { return st ? st->valid_total : -1; }

extern "C" size_t mux_segtab_serialized_bytes(const mux_segtab* st) { return st ? st->image.size() * 4 : 0; }

extern "C" mux_status mux_segtab_serialize(const mux_segtab* st, void* dst, size_t cap) {
  if (!st || !dst) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_serialize: null argument");
  if (cap < st->image.size() * 4) return fail(MUX_ERR_WORKSPACE, "mux_segtab_serialize: destination too small");
  std::memcpy(dst, st->image.data(), st->image.size() * 4);
  return MUX_OK;
}

extern "C" mux_status mux_segtab_row_task(const mux_segtab* st, int32_t* dst, size_t cap_entries) {
  if (!st || (!dst && st->T > 0)) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_row_task: null argument");
  if (cap_entries < (size_t)st->T) return fail(MUX_ERR_WORKSPACE, "mux_segtab_row_task: destination too small");
  if (st->T) std::memcpy(dst, st->row_task.data(), (size_t)st->T * 4);
  return MUX_OK;
}

extern "C" size_t mux_segtab_device_bytes(const mux_segtab* st) { return st ? st->dev_image.size() * 4 : 0; }

extern "C" mux_status mux_segtab_upload(const mux_segtab* st, void* dev_dst, size_t cap, void* hip_stream) {
  if (!st || !dev_dst) return fail(MUX_ERR_INVALID_ARG, "mux_segtab_upload: null argument");
  const size_t bytes = st->dev_image.size() * 4;
  if (cap < bytes) return fail(MUX_ERR_WORKSPACE, "mux_segtab_upload: destination too small");
  hipError_t e = hipMemcpyAsync(dev_dst, st->dev_image.data(), bytes, hipMemcpyHostToDevice, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(MUX_ERR_DEVICE, std::string("mux_segtab_upload: ") + hipGetErrorString(e));
  return MUX_OK;
}
