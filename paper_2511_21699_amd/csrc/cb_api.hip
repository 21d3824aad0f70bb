// Host side of libcacheback_verify.so: argument checks, workspace layout, launch planning and the
// extern "C" entry points declared in cacheback.h.  No arithmetic of the method happens here.
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <algorithm>
#include <mutex>
#include <new>

#include "cb_logits.h"

using namespace cb;

namespace {

thread_local char g_init_err[256] = "";

// Scratch memory of cb_tree_attention_noalloc: a fixed array in the library's own device image
// (every GPU the library runs on holds one copy until the process ends).  In host code the array's
// name is only a handle: its address on a device comes from hipGetSymbolAddress, once per device.
constexpr size_t kStaticScratchBytes = 32u << 20;
__device__ __align__(256) unsigned char g_static_scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_static_scratch_ptr[kMaxDevices];  // per device, filled on first use (under g_static_mutex)
std::mutex g_static_mutex;

constexpr size_t kAlign = 256;
size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
  size_t anc, parent, tokens, amax_partial, amax_out, path, len_ctx, res_len, res_tok, new_len, status,
      tickets, coop_tickets, amax_tickets, amax_lines, dbg, partial, total;
  int amax_chunks;
  int max_total_nodes;
  int max_splits;
  int scalar_splits;  // split count the scalar kernel's fp32 partials have room for
  int ticket_count;
};

int effective_max_splits(const cb_config& c) { return c.max_splits > 0 ? c.max_splits : 64; }

bool config_ok(const cb_config* c, char* err, size_t n) {
  auto fail = [&](const char* m) {
    if (err && n) snprintf(err, n, "config: %s", m);
    return false;
  };
  if (!c) return fail("null");
  if (c->num_q_heads < 1 || c->num_kv_heads < 1 || c->num_q_heads % c->num_kv_heads != 0)
    return fail("num_q_heads must be a positive multiple of num_kv_heads");
  if (c->num_q_heads > 1024) return fail("num_q_heads > 1024");
  if (c->head_dim != 64 && c->head_dim != 128) return fail("head_dim must be 64 or 128");
  if ((c->qkv_dtype != CB_F32 && c->qkv_dtype != CB_BF16) || (c->logits_dtype != CB_F32 && c->logits_dtype != CB_BF16))
    return fail("dtype must be CB_F32 or CB_BF16");
  if (c->max_batch < 1 || c->max_batch > CB_MAX_BATCH) return fail("max_batch out of range");
  if (c->max_nodes < 1 || c->max_nodes > CB_MAX_NODES) return fail("max_nodes out of range");
  if (c->max_depth < 0 || c->max_depth >= CB_MAX_NODES) return fail("max_depth out of range");
  if (c->vocab_size < 1) return fail("vocab_size < 1");
  if (c->block_size < 0 || c->block_size > 65536) return fail("block_size out of range");
  if (c->max_splits < 0 || c->max_splits > 4096) return fail("max_splits out of range");
  return true;
}

WsLayout ws_layout(const cb_config& c) {
  WsLayout L{};
  const size_t mt = (size_t)c.max_batch * c.max_nodes;
  const size_t stride = (size_t)c.max_depth + 1;
  L.max_total_nodes = (int)mt;
  L.max_splits = effective_max_splits(c);
  L.amax_chunks = (int)(((int64_t)c.vocab_size + kArgmaxChunk - 1) / kArgmaxChunk);
  const int g = c.num_q_heads / c.num_kv_heads;
  L.ticket_count = 4 * c.max_batch * c.num_kv_heads * ((c.max_nodes * g + kRowTile - 1) / kRowTile);  // two 64-bit words per tile
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  L.anc = take(mt * kAncWords * 4);
  L.parent = take(mt * 4 * 2);  // staged tree of the host-array form: parents, then tokens right behind them
  L.tokens = L.parent;         // (placed per call)
  L.amax_partial = take(mt * L.amax_chunks * sizeof(ArgmaxPartial));
  L.amax_out = take(mt * 4);
  L.path = take(c.max_batch * stride * 4);
  L.len_ctx = take(c.max_batch * 4);
  L.res_len = take(c.max_batch * (1 + stride) * 4);  // results of the host-array form: lengths, then tokens right behind them
  L.res_tok = L.res_len;                              // (placed per call)
  L.new_len = take(c.max_batch * 4);
  L.status = take(4);
  L.tickets = take((size_t)L.ticket_count * 4);
  L.coop_tickets = take((size_t)kCoopTiles * kCoopTicketStride);
  L.amax_tickets = take(CB_MAX_BATCH * 4);
  // argmax partials of the one-launch verification, one 128-byte line each (it takes sequences of at most 64 nodes)
  L.amax_lines = take((size_t)c.max_batch * std::min(c.max_nodes, 64) * L.amax_chunks * 128);
  L.dbg = take(1024 * 8 * 8);
  // The scalar kernel's fp32 partials are 8 times the size of the MFMA kernel's.  A configuration
  // the MFMA kernel takes (bf16, head_dim 128) runs the scalar one only on request (option
  // "attn_impl" = 1, a test aid): it gets room for 8 splits there, not for max_splits.
  const bool mfma_cfg = c.qkv_dtype == CB_BF16 && c.head_dim == 128;
  L.scalar_splits = mfma_cfg ? std::min(L.max_splits, 8) : L.max_splits;
  const size_t scalar_bytes = mt * c.num_q_heads * (size_t)L.scalar_splits * partial_stride(c.head_dim) * 4;
  const size_t mfma_bytes = mfma_cfg ? attn_mfma_partial_bytes(mt, c.num_q_heads, c.num_kv_heads, c.max_batch, L.max_splits) : 0;
  L.partial = take(std::max(scalar_bytes, mfma_bytes));
  L.total = o;
  return L;
}

struct Plan {
  int impl;    // 1 scalar, 2 MFMA
  int nsplit;  // partial slots per row
  int chunk;   // keys per split
  int max_nodes, max_len;
};

}  // namespace

struct cb_ctx {
  cb_config cfg;
  WsLayout lay;
  char* ws;
  // pinned host mirror
  int32_t* h_parent;
  int32_t* h_tokens;
  int32_t* h_len;
  int32_t* h_tok;
  int32_t* h_path;
  int32_t* h_argmax;
  int32_t* h_misc;  // [0] status, [1..] new_len
  int32_t* h_done;  // [max_batch] arrival flags of the host form's results (the call's sequence number)
  int32_t call_seq = 0;        // sequence number of the last host-form call (never 0 once used)
  int32_t* want_done = nullptr;  // set by cb_verify_tree for the launch it is about to make
  hipStream_t unsynced = nullptr;  // stream that may still run the tail of a host-form call that has returned
  bool have_unsynced = false;
  int32_t* d_hblock = nullptr;  // the pinned block's address on the device
  void* h_block;
  // state of the last verify
  bool have_verify;
  int32_t launch_info[6];
  bool host_knows_len;
  int batch;
  int total_nodes;
  SeqMeta meta;
  int32_t last_len[CB_MAX_BATCH];
  hipStream_t last_stream;
  // options
  int64_t opt_splits, opt_impl, opt_time, opt_stages, opt_timeline, opt_external, opt_fork, opt_fuse, opt_coop, opt_spin, opt_full_sync;
  hipEvent_t ev0, ev1, ev_fork, ev_join;
  hipStream_t aux;  // second stream (default priority) for the logits scan beside the attention
  bool ev_valid;
  const Plan* fixed_plan = nullptr;  // (cb_tree_attention_noalloc: the plan its scratch layout was cut for)
  bool counters_dirty = false;  // a launch failed: the tickets may be left non-zero
  char err[256];

  template <typename T>
  T* dev(size_t off) const { return reinterpret_cast<T*>(ws + off); }
};

namespace {

int set_err(cb_ctx* ctx, int code, const char* fmt, ...) {
  char* dst = ctx ? ctx->err : g_init_err;
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(dst, 256, fmt, ap);
  va_end(ap);
  return code;
}

#define CB_HIP(ctx, call)                                                                         \
  do {                                                                                            \
    hipError_t e__ = (call);                                                                      \
    if (e__ != hipSuccess) return set_err(ctx, CB_EHIP, "%s: %s", #call, hipGetErrorString(e__)); \
  } while (0)
// the same for the launches of run_pipeline: a failure there may leave tickets behind
#define CB_LAUNCH(ctx, call)                                                                      \
  do {                                                                                            \
    hipError_t e__ = (call);                                                                      \
    if (e__ != hipSuccess) {                                                                      \
      (ctx)->counters_dirty = true;                                                               \
      return set_err(ctx, CB_EHIP, "%s: %s", #call, hipGetErrorString(e__));                     \
    }                                                                                             \
  } while (0)

bool make_kv_addr(const cb_config& c, const cb_kv_layer& l, KvAddr* a) {
  const int64_t D = c.head_dim, H = c.num_kv_heads;
  a->k = l.k;
  a->v = l.v;
  a->block_table = l.block_table;
  a->max_blocks = l.max_blocks_per_seq;
  a->block_size = c.block_size;
  a->num_blocks = c.block_size > 0 ? l.capacity_or_num_blocks : 0;
  const int64_t tokens_per_unit = c.block_size > 0 ? c.block_size : l.capacity_or_num_blocks;
  a->seq_stride = tokens_per_unit * H * D;
  if (l.layout == CB_LAYOUT_TOKEN_MAJOR) {
    a->token_stride = H * D;
    a->head_stride = D;
  } else if (l.layout == CB_LAYOUT_HEAD_MAJOR) {
    a->token_stride = D;
    a->head_stride = tokens_per_unit * D;
  } else {
    return false;
  }
  return true;
}

// Pure host arithmetic: no device call, no context state beyond the three numbers passed in.
Plan plan_attention(const cb_config& c, int max_splits, int scalar_splits, int opt_impl, int opt_splits, int batch,
                    const int32_t* kv_len, const int32_t* node_offsets) {
  Plan p{};
  int64_t rows = 0;
  for (int b = 0; b < batch; b++) {
    const int n = node_offsets[b + 1] - node_offsets[b];
    p.max_nodes = std::max(p.max_nodes, n);
    p.max_len = std::max(p.max_len, kv_len[b] + n);
    rows += (int64_t)n * c.num_q_heads;
  }
  const bool mfma_ok = c.qkv_dtype == CB_BF16 && c.head_dim == 128;
  p.impl = (opt_impl == 1 || !mfma_ok) ? 1 : 2;
  if (p.impl == 1) max_splits = scalar_splits;
  int nsplit;
  if (opt_splits > 0) {
    nsplit = (int)std::min<int64_t>(opt_splits, max_splits);
  } else if (p.impl == 1) {
    // one workgroup per (row, split): aim for a few workgroups per compute unit, but never split
    // below 1024 keys -- a second (merge) launch costs more than a short row does
    const int64_t want = 2048;
    nsplit = (int)std::max<int64_t>(1, std::min<int64_t>((want + rows - 1) / rows, p.max_len / 1024));
  } else {
    // one workgroup per (row tile of 64, 128 or 256 rows, kv head, split)
    const int g = c.num_q_heads / c.num_kv_heads;
    const int mrows = p.max_nodes * g;
    const int rows_per_wg = attn_mfma_tile_rows(mrows);
    // Every variant runs 8 waves and a 128 KiB ring: one workgroup per compute unit, so the grid
    // should come out just under a whole number of rounds of 256 workgroups.  Take the fewest
    // splits that fill >= 85% of the machine in whole rounds (fewer splits = fewer partials).
    // efficiency of ns splits: keys swept / (256 units x whole rounds x keys of a full split)
    auto workgroups = [&](int ns) {
      const int chunk = ((p.max_len + ns - 1) / ns + 31) / 32 * 32;
      int64_t t = 0;
      for (int b = 0; b < batch; b++) {
        const int n = node_offsets[b + 1] - node_offsets[b];
        t += (int64_t)((n * g + rows_per_wg - 1) / rows_per_wg) * c.num_kv_heads * ((kv_len[b] + n + chunk - 1) / chunk);
      }
      return t;
    };
    auto efficiency = [&](int ns) {
      const int chunk = ((p.max_len + ns - 1) / ns + 31) / 32 * 32;
      int64_t t = 0, keys = 0;
      for (int b = 0; b < batch; b++) {
        const int n = node_offsets[b + 1] - node_offsets[b];
        const int64_t tl = (int64_t)((n * g + rows_per_wg - 1) / rows_per_wg) * c.num_kv_heads;
        t += tl * ((kv_len[b] + n + chunk - 1) / chunk);
        keys += tl * (kv_len[b] + n);
      }
      const int64_t rounds = (t + 255) / 256;
      return (double)keys / ((double)rounds * 256.0 * chunk);
    };
    const int cap = (int)std::max<int64_t>(1, std::min<int64_t>(max_splits, (p.max_len + 127) / 128));
    const int tiles_max = (mrows + rows_per_wg - 1) / rows_per_wg;
    if (batch > 1 && (c.num_kv_heads * tiles_max) % 8 == 0) {
      // Several sequences, launched longest first within every XCD (see the kernel's workgroup
      // numbering).  Such a list schedule ends no later than max(longest job, work / units + a job
      // of the shortest sequence), so: estimate that for every split count, in units of one 64-key
      // stage, with what a workgroup costs beside its stages (start-up and tail: about six stages;
      // a workgroup of the grid that finds no keys: one), and what a tile's merge costs its last
      // workgroup, and take the cheapest count -- the fewest splits that still spread the longest
      // sequence wide enough.
      double best_cost = 0.0;
      nsplit = 1;
      for (int ns = 1; ns <= cap; ns++) {
        const int chunk = ((p.max_len + ns - 1) / ns + 31) / 32 * 32;
        const int grid_x = (p.max_len + chunk - 1) / chunk;
        const double merge = grid_x > 1 ? 0.7 * grid_x * (rows_per_wg / 128.0) : 0.0;
        double work = 0.0, longest = 0.0, shortest = 1e30;
        int64_t jobs = 0;
        for (int b = 0; b < batch; b++) {
          const int n = node_offsets[b + 1] - node_offsets[b];
          const int len = kv_len[b] + n;
          const int64_t tl = (int64_t)((n * g + rows_per_wg - 1) / rows_per_wg) * c.num_kv_heads;
          const int full = len / chunk, rest = len - full * chunk;
          const double job_full = 6.0 + (chunk + 63) / 64, job_rest = rest > 0 ? 6.0 + (rest + 63) / 64 : 0.0;
          const int real = full + (rest > 0 ? 1 : 0);
          work += tl * (full * job_full + job_rest + (real > 1 ? merge : 0.0)) +
                  ((int64_t)c.num_kv_heads * tiles_max * grid_x - tl * real) * 1.0;
          jobs += tl * real;
          longest = std::max(longest, (full > 0 ? job_full : job_rest) + (real > 1 ? merge : 0.0));
          shortest = std::min(shortest, full > 0 ? job_full : job_rest);
        }
        const double cost = jobs <= 256 ? longest : std::max(longest, work / 256.0 + shortest);
        if (ns == 1 || cost < best_cost - 1e-9) { best_cost = cost; nsplit = ns; }
      }
    } else {
    nsplit = cap;
    double best = -1.0;
    for (int ns = 1; ns <= cap; ns++) {
      const double eff = efficiency(ns);
      if (eff >= 0.85) { nsplit = ns; best = eff; break; }
      if (eff > best) { best = eff; nsplit = ns; }
    }
    // A grid of one round merges cooperatively (no workgroup pulls a whole tile's partials), so
    // there more splits cost next to nothing: take the best-filling count among the one-round ones.
    if (best >= 0.85 && workgroups(nsplit) <= 256) {
      for (int ns = nsplit + 1; ns <= cap && ns <= 64 && workgroups(ns) <= 256; ns++) {
        const double eff = efficiency(ns);
        if (eff > best + 1e-9) { best = eff; nsplit = ns; }
      }
    }
    }
  }
  nsplit = std::max(1, std::min(nsplit, max_splits));
  int chunk = (p.max_len + nsplit - 1) / nsplit;
  chunk = (chunk + 31) / 32 * 32;
  p.chunk = std::max(chunk, 32);
  p.nsplit = (p.max_len + p.chunk - 1) / p.chunk;
  return p;
}

int check_common(cb_ctx* ctx, int32_t batch, const void* q, const cb_kv_layer* kv, const int32_t* kv_len,
                 const int32_t* node_offsets, const void* logits, void* attn_out) {
  if (!ctx) return set_err(nullptr, CB_EINVAL, "null context");
  if (!q || !kv || !kv_len || !node_offsets || !logits || !attn_out)
    return set_err(ctx, CB_EINVAL, "null argument");
  if (batch < 1 || batch > ctx->cfg.max_batch) return set_err(ctx, CB_EINVAL, "batch %d outside [1, %d]", batch, ctx->cfg.max_batch);
  if (((uintptr_t)q | (uintptr_t)kv->k | (uintptr_t)kv->v | (uintptr_t)logits | (uintptr_t)attn_out) & 15)
    return set_err(ctx, CB_EINVAL, "device pointers must be 16-byte aligned");
  return CB_OK;
}

// Enqueues the whole verification on `st`; the tree is already on the device.
int run_pipeline(cb_ctx* ctx, hipStream_t st, int batch, const void* q, const cb_kv_layer* kv,
                 const int32_t* kv_len, const int32_t* node_offsets, const int32_t* d_parent,
                 const int32_t* d_tokens, const void* logits, void* attn_out, int32_t* d_len, int32_t* d_tok,
                 int64_t stage_mask = 15) {
  const cb_config& c = ctx->cfg;
  SeqMeta meta{};
  for (int b = 0; b < batch; b++) meta.kv_len[b] = kv_len[b];
  for (int b = 0; b <= batch; b++) meta.node_off[b] = node_offsets[b];
  for (int b = 0; b < batch; b++) meta.by_length[b] = b;
  std::stable_sort(meta.by_length, meta.by_length + batch, [&](int32_t x, int32_t y) {
    return (int64_t)kv_len[x] + node_offsets[x + 1] - node_offsets[x] > (int64_t)kv_len[y] + node_offsets[y + 1] - node_offsets[y];
  });
  const int total = node_offsets[batch];
  if (ctx->have_unsynced && ctx->unsynced != st) {
    // the last host-form call returned when its results arrived; what is left of its launch still uses
    // the workspace, and only work on that same stream is ordered behind it
    CB_HIP(ctx, hipStreamSynchronize(ctx->unsynced));
    ctx->have_unsynced = false;
  }
  if (ctx->counters_dirty) {  // (after a failed launch: the kernels rely on tickets that are zero between launches)
    const hipError_t e1 = launch_zero_words(st, ctx->dev<unsigned long long>(ctx->lay.tickets), ctx->lay.ticket_count / 2, 1, 1);
    const hipError_t e2 = launch_zero_words(st, ctx->dev<unsigned long long>(ctx->lay.coop_tickets), kCoopTiles, kCoopTicketStride / 8, 2);
    const hipError_t e3 = launch_zero_words(st, ctx->dev<unsigned long long>(ctx->lay.amax_tickets), CB_MAX_BATCH / 2, 1, 1);
    if (e1 != hipSuccess || e2 != hipSuccess || e3 != hipSuccess) return set_err(ctx, CB_EHIP, "clearing the tickets after a failed launch failed");
    ctx->counters_dirty = false;
  }
  const Plan plan = ctx->fixed_plan ? *ctx->fixed_plan
                                    : plan_attention(c, ctx->lay.max_splits, ctx->lay.scalar_splits, ctx->opt_impl, ctx->opt_splits, batch, kv_len, node_offsets);

  AttnParams ap{};
  ap.q = q;
  ap.out = attn_out;
  if (!make_kv_addr(c, *kv, &ap.kv)) return set_err(ctx, CB_EINVAL, "unknown cache layout %d", kv->layout);
  ap.anc = ctx->dev<uint32_t>(ctx->lay.anc);
  ap.parent = d_parent;
  ap.partial = ctx->dev<float>(ctx->lay.partial);
  ap.tickets = ctx->dev<uint32_t>(ctx->lay.tickets);
  ap.coop_tickets = ctx->dev<uint32_t>(ctx->lay.coop_tickets);
  ap.Hq = c.num_q_heads;
  ap.Hkv = c.num_kv_heads;
  ap.D = c.head_dim;
  ap.chunk = plan.chunk;
  ap.nsplit = plan.nsplit;
  ap.batch = batch;
  ap.scale = c.softmax_scale > 0.f ? c.softmax_scale : 1.0f / sqrtf((float)c.head_dim);
  ap.status = ctx->dev<int32_t>(ctx->lay.status);
  ap.dbg_ts = ctx->dev<unsigned long long>(ctx->lay.dbg);
  ap.timeline = ctx->opt_timeline ? 1 : 0;
  ap.force_external_merge = ctx->opt_external ? 1 : 0;
  ap.max_depth = c.max_depth;
  ap.coop_merge = ctx->opt_coop ? 0 : -1;
  ap.spin_limit = (int32_t)ctx->opt_spin;

  // bit 0 ancestor sets, 1 attention, 2 argmax, 3 acceptance; the option is a measurement aid, the
  // mask is what the entry point asks for (cb_tree_attention_device: the first two)
  const int64_t stages = ctx->opt_stages & stage_mask;
  const bool use_mfma = plan.impl == 2 && attn_mfma_supports(ap);
  // The logits scan does not depend on the attention, and the MFMA attention builds the ancestor sets
  // it needs itself, so with option "parallel_scan" the scan runs beside it on the context's second
  // stream (fork/join with events; stream capture turns them into parallel graph branches).  Measured
  // on the 7B shape the cross-stream edges cost more than the 5 us scan they hide, so it is off by
  // default.  The scalar attention reads the sets from the workspace: there the scan goes first and
  // carries the blocks that build them.
  AcceptArgs acc{};
  acc.parent = d_parent;
  acc.tokens = d_tokens;
  acc.status = ctx->dev<int32_t>(ctx->lay.status);
  acc.partial = ctx->dev<ArgmaxPartial>(ctx->lay.amax_partial);
  acc.slot_stride = 1;
  acc.nchunks = ctx->lay.amax_chunks;
  acc.max_depth = c.max_depth;
  acc.argmax_out = ctx->dev<int32_t>(ctx->lay.amax_out);
  acc.path = ctx->dev<int32_t>(ctx->lay.path);
  acc.len_ctx = ctx->dev<int32_t>(ctx->lay.len_ctx);
  acc.len_user = d_len;
  acc.tok_user = d_tok;
  acc.done_flag = ctx->want_done;
  acc.done_value = ctx->call_seq;
  ctx->want_done = nullptr;
  // Small calls with the MFMA attention are one launch: the attention workgroups also scan the
  // logits and run the acceptance (option "fuse_logits", on by default; see attn_mfma_can_fuse).
  // Otherwise the scan, the attention and the acceptance are launches of their own.
  const bool fused = use_mfma && ctx->opt_fuse != 0 && (stages & 2) && (stages & 4) && (stages & 8) &&
                     attn_mfma_can_fuse(ap, plan.max_nodes, (int64_t)total * ctx->lay.amax_chunks, c.logits_dtype);
  const bool fork = !fused && ctx->opt_fork != 0 && use_mfma && (stages & 2) && (stages & 4);
  hipStream_t scan_stream = st;
  int merge_kind = plan.nsplit > 1 ? 3 : 0, kernels = 0;  // (the scalar attention always merges with a kernel of its own)
  if (fork) {
    CB_HIP(ctx, hipEventRecord(ctx->ev_fork, st));
    CB_HIP(ctx, hipStreamWaitEvent(ctx->aux, ctx->ev_fork, 0));
    scan_stream = ctx->aux;
  }
  if (fused) {
  } else if (stages & 4) {
    const bool carry = !use_mfma && (stages & 1);
    CB_LAUNCH(ctx, launch_argmax(scan_stream, logits, c.logits_dtype, total, c.vocab_size,
                              ctx->dev<ArgmaxPartial>(ctx->lay.amax_partial), ctx->lay.amax_chunks, batch, meta,
                              carry ? d_parent : nullptr, c.max_depth, carry ? ctx->dev<uint32_t>(ctx->lay.anc) : nullptr,
                              carry ? ctx->dev<int32_t>(ctx->lay.status) : nullptr));
    kernels++;
  } else if (!use_mfma && (stages & 1)) {
    CB_LAUNCH(ctx, launch_tree_prepare(st, batch, meta, d_parent, c.max_depth, ctx->dev<uint32_t>(ctx->lay.anc),
                                    ctx->dev<int32_t>(ctx->lay.status)));
    kernels++;
  }
  if (fork) CB_HIP(ctx, hipEventRecord(ctx->ev_join, ctx->aux));
  const bool timing = ctx->opt_time != 0;
  if (timing) CB_HIP(ctx, hipEventRecord(ctx->ev0, st));
  if (!(stages & 2)) {
  } else if (use_mfma) {
    LogitsWork lw{};
    lw.logits = static_cast<const uint16_t*>(logits);
    lw.V = c.vocab_size;
    lw.rows = total;
    lw.batch = batch;
    lw.tickets = ctx->dev<uint32_t>(ctx->lay.amax_tickets);
    lw.accept = acc;
    lw.accept.partial = ctx->dev<ArgmaxPartial>(ctx->lay.amax_lines);
    lw.accept.slot_stride = 16;
    lw.partial_out = ctx->dev<ArgmaxPartial>(ctx->lay.amax_lines);
    CB_LAUNCH(ctx, launch_attn_mfma(st, ap, meta, plan.max_nodes, total, fused ? &lw : nullptr, &merge_kind));  // merges its own splits
    kernels += merge_kind == 3 ? 2 : 1;
  } else {
    CB_LAUNCH(ctx, launch_attn_simt(st, ap, meta, c.qkv_dtype, plan.max_nodes));
    if (plan.nsplit > 1) CB_LAUNCH(ctx, launch_merge(st, ap, meta, c.qkv_dtype, total));
    kernels += plan.nsplit > 1 ? 2 : 1;
  }
  if (timing) {
    CB_HIP(ctx, hipEventRecord(ctx->ev1, st));
    ctx->ev_valid = true;
  }
  if (fork) CB_HIP(ctx, hipStreamWaitEvent(st, ctx->ev_join, 0));
  if ((stages & 8) && !fused) {
    CB_LAUNCH(ctx, launch_accept(st, batch, meta, acc));
    kernels++;
  }
  if (!(stage_mask & 8)) return CB_OK;  // attention alone leaves the state of the last verification as it is
  ctx->launch_info[0] = use_mfma ? 2 : 1;
  ctx->launch_info[1] = plan.nsplit;
  ctx->launch_info[2] = plan.chunk;
  ctx->launch_info[3] = fused ? 1 : 0;
  ctx->launch_info[4] = merge_kind;
  ctx->launch_info[5] = kernels;
  ctx->meta = meta;
  ctx->batch = batch;
  ctx->total_nodes = total;
  ctx->last_stream = st;
  ctx->have_verify = true;
  ctx->host_knows_len = false;
  return CB_OK;
}

// Shapes are host data in the device-resident forms too: everything except the tree's contents is checked.
int check_device_shapes(cb_ctx* ctx, int32_t batch, const cb_kv_layer* kv, const int32_t* kv_len, const int32_t* node_offsets) {
  const cb_config& c = ctx->cfg;
  if (!kv->k || !kv->v || kv->capacity_or_num_blocks < 1) return set_err(ctx, CB_EINVAL, "bad cache descriptor");
  if (c.block_size > 0 && (!kv->block_table || kv->max_blocks_per_seq < 1)) return set_err(ctx, CB_EINVAL, "paged cache without a block table");
  if (node_offsets[0] != 0) return set_err(ctx, CB_EINVAL, "node_offsets[0] must be 0");
  for (int b = 0; b < batch; b++) {
    const int64_t n = (int64_t)node_offsets[b + 1] - node_offsets[b];
    if (n < 1) return set_err(ctx, CB_EINVAL, "sequence %d has no root node", b);
    if (n > c.max_nodes) return set_err(ctx, CB_ECAP, "sequence %d has %lld nodes, max_nodes is %d", b, (long long)n, c.max_nodes);
    if (kv_len[b] < 0) return set_err(ctx, CB_EINVAL, "negative kv_len[%d]", b);
    const int64_t room = c.block_size > 0 ? (int64_t)kv->max_blocks_per_seq * c.block_size : kv->capacity_or_num_blocks;
    if (kv_len[b] + n > room || kv_len[b] + n > (1ll << 30)) return set_err(ctx, CB_ECAP, "sequence %d does not fit the cache", b);
  }
  return CB_OK;
}

}  // namespace

extern "C" {

int cb_workspace_bytes(const cb_config* cfg, size_t* bytes) {
  if (!bytes) return set_err(nullptr, CB_EINVAL, "null bytes");
  if (!config_ok(cfg, g_init_err, sizeof g_init_err)) return CB_EINVAL;
  *bytes = ws_layout(*cfg).total;
  return CB_OK;
}

int cb_plan_attention(const cb_config* cfg, int32_t batch, const int32_t* kv_len, const int32_t* node_offsets,
                      int32_t forced_splits, int32_t plan[5]) {
  if (!config_ok(cfg, nullptr, 0) || !kv_len || !node_offsets || !plan) return CB_EINVAL;
  if (batch < 1 || batch > cfg->max_batch || node_offsets[0] != 0) return CB_EINVAL;
  for (int b = 0; b < batch; b++) {
    const int64_t n = (int64_t)node_offsets[b + 1] - node_offsets[b];
    if (n < 1 || n > cfg->max_nodes || kv_len[b] < 0 || (int64_t)kv_len[b] + n > (1ll << 30)) return CB_EINVAL;
  }
  const WsLayout lay = ws_layout(*cfg);
  const Plan p = plan_attention(*cfg, lay.max_splits, lay.scalar_splits, 0, forced_splits, batch, kv_len, node_offsets);
  const int g = cfg->num_q_heads / cfg->num_kv_heads;
  const int tile = p.impl == 2 ? attn_mfma_tile_rows(p.max_nodes * g) : 1;
  int64_t wgs = 0;
  for (int b = 0; b < batch; b++) {
    const int n = node_offsets[b + 1] - node_offsets[b];
    const int64_t units = p.impl == 2 ? (int64_t)((n * g + tile - 1) / tile) * cfg->num_kv_heads : (int64_t)n * cfg->num_q_heads;
    wgs += units * ((kv_len[b] + n + p.chunk - 1) / p.chunk);
  }
  plan[0] = p.impl;
  plan[1] = p.nsplit;
  plan[2] = p.chunk;
  plan[3] = tile;
  plan[4] = (int32_t)std::min<int64_t>(wgs, INT32_MAX);
  return CB_OK;
}

int cb_check_verify_args(const cb_config* cfg, int32_t batch, const cb_kv_layer* kv, const int32_t* kv_len,
                         const int32_t* node_offsets, const int32_t* tree_parent, char* err, size_t err_len) {
  auto fail = [&](int code, const char* fmt, ...) __attribute__((format(printf, 3, 4))) {
    if (err && err_len) {
      va_list ap;
      va_start(ap, fmt);
      vsnprintf(err, err_len, fmt, ap);
      va_end(ap);
    }
    return code;
  };
  if (!config_ok(cfg, err, err_len)) return CB_EINVAL;
  if (!kv || !kv_len || !node_offsets || !tree_parent) return fail(CB_EINVAL, "null argument");
  if (batch < 1 || batch > cfg->max_batch) return fail(CB_EINVAL, "batch %d outside [1, %d]", batch, cfg->max_batch);
  if (!kv->k || !kv->v) return fail(CB_EINVAL, "null cache pointer");
  if (kv->layout != CB_LAYOUT_TOKEN_MAJOR && kv->layout != CB_LAYOUT_HEAD_MAJOR)
    return fail(CB_EINVAL, "unknown cache layout %d", kv->layout);
  if (kv->capacity_or_num_blocks < 1) return fail(CB_EINVAL, "empty cache");
  if (cfg->block_size > 0 && (!kv->block_table || kv->max_blocks_per_seq < 1))
    return fail(CB_EINVAL, "paged cache without a block table");
  if (cfg->block_size == 0 && kv->block_table) return fail(CB_EINVAL, "block table given for a contiguous cache");
  if (node_offsets[0] != 0) return fail(CB_EINVAL, "node_offsets[0] must be 0");
  for (int b = 0; b < batch; b++) {
    const int64_t n = (int64_t)node_offsets[b + 1] - node_offsets[b];
    if (n < 1) return fail(CB_EINVAL, "sequence %d has no root node", b);
    if (n > cfg->max_nodes) return fail(CB_ECAP, "sequence %d has %lld nodes, max_nodes is %d", b, (long long)n, cfg->max_nodes);
    if (kv_len[b] < 0) return fail(CB_EINVAL, "negative kv_len[%d]", b);
    const int64_t need = (int64_t)kv_len[b] + n;
    const int64_t room = cfg->block_size > 0 ? (int64_t)kv->max_blocks_per_seq * cfg->block_size : kv->capacity_or_num_blocks;
    if (need > room || need > (1ll << 30))
      return fail(CB_ECAP, "sequence %d needs %lld cache slots, %lld available", b, (long long)need, (long long)room);
    const int32_t* par = tree_parent + node_offsets[b];
    if (par[0] != -1) return fail(CB_ETREE, "sequence %d: root parent is %d, not -1", b, par[0]);
    int depth[CB_MAX_NODES];
    depth[0] = 0;
    for (int i = 1; i < n; i++) {
      if (par[i] < 0 || par[i] >= i) return fail(CB_ETREE, "sequence %d: parent[%d] = %d not in [0, %d)", b, i, par[i], i);
      depth[i] = depth[par[i]] + 1;
      if (depth[i] > cfg->max_depth) return fail(CB_ETREE, "sequence %d: node %d at depth %d > max_depth %d", b, i, depth[i], cfg->max_depth);
    }
  }
  return CB_OK;
}

int cb_init(const cb_config* cfg, void* workspace, size_t workspace_bytes, cb_ctx** out) {
  g_init_err[0] = 0;
  if (!out) return set_err(nullptr, CB_EINVAL, "null out");
  *out = nullptr;
  if (!config_ok(cfg, g_init_err, sizeof g_init_err)) return CB_EINVAL;
  const WsLayout lay = ws_layout(*cfg);
  if (!workspace || ((uintptr_t)workspace & (kAlign - 1))) return set_err(nullptr, CB_EINVAL, "workspace null or not 256-byte aligned");
  if (workspace_bytes < lay.total) return set_err(nullptr, CB_ECAP, "workspace of %zu bytes, %zu needed", workspace_bytes, lay.total);
  int ndev = 0;
  if (hipGetDeviceCount(&ndev) != hipSuccess || ndev < 1) return set_err(nullptr, CB_EHIP, "no HIP device");
  cb_ctx* ctx = new (std::nothrow) cb_ctx();
  if (!ctx) return set_err(nullptr, CB_EHIP, "out of host memory");
  ctx->cfg = *cfg;
  ctx->lay = lay;
  ctx->ws = static_cast<char*>(workspace);
  ctx->opt_stages = 15;
  ctx->opt_fuse = 1;
  ctx->opt_coop = 1;
  ctx->opt_spin = 256;
  const size_t mt = lay.max_total_nodes, stride = (size_t)cfg->max_depth + 1;
  // (two tree areas: a host-form call may return while its kernels still run, and the next call
  // must not overwrite the tree they read)
  const size_t ints = mt * 5 + cfg->max_batch * (1 + 2 * stride) + 1 + 2 * (size_t)cfg->max_batch;
  hipError_t e = hipHostMalloc(&ctx->h_block, ints * 4, hipHostMallocDefault);
  if (e != hipSuccess) {
    delete ctx;
    return set_err(nullptr, CB_EHIP, "hipHostMalloc: %s", hipGetErrorString(e));
  }
  void* dptr = nullptr;
  e = hipHostGetDevicePointer(&dptr, ctx->h_block, 0);
  if (e != hipSuccess) {
    (void)hipHostFree(ctx->h_block);
    delete ctx;
    return set_err(nullptr, CB_EHIP, "hipHostGetDevicePointer: %s", hipGetErrorString(e));
  }
  ctx->d_hblock = static_cast<int32_t*>(dptr);
  int32_t* h = static_cast<int32_t*>(ctx->h_block);
  ctx->h_parent = h; h += mt;
  ctx->h_tokens = h; h += mt;
  h += 2 * mt;                       // (the second tree area, see cb_verify_tree)
  ctx->h_argmax = h; h += mt;
  ctx->h_len = h; h += cfg->max_batch;
  ctx->h_tok = h; h += cfg->max_batch * stride;
  ctx->h_path = h; h += cfg->max_batch * stride;
  ctx->h_misc = h; h += 1 + cfg->max_batch;
  ctx->h_done = h;
  memset(ctx->h_done, 0, (size_t)cfg->max_batch * 4);
  e = hipEventCreate(&ctx->ev0);
  if (e == hipSuccess) e = hipEventCreate(&ctx->ev1);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_fork, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&ctx->ev_join, hipEventDisableTiming);
  if (e == hipSuccess) e = hipStreamCreateWithFlags(&ctx->aux, hipStreamNonBlocking);
  if (e == hipSuccess) e = hipMemset(ctx->ws + lay.status, 0, 4);
  if (e == hipSuccess) e = hipMemset(ctx->ws + lay.tickets, 0, (size_t)lay.ticket_count * 4);
  if (e == hipSuccess) e = hipMemset(ctx->ws + lay.coop_tickets, 0, (size_t)kCoopTiles * kCoopTicketStride);
  if (e == hipSuccess) e = hipMemset(ctx->ws + lay.amax_tickets, 0, CB_MAX_BATCH * 4);
  if (e == hipSuccess) e = hipDeviceSynchronize();
  if (e != hipSuccess) {
    (void)hipHostFree(ctx->h_block);
    delete ctx;
    return set_err(nullptr, CB_EHIP, "context set-up: %s", hipGetErrorString(e));
  }
  *out = ctx;
  return CB_OK;
}

int cb_verify_tree_device(cb_ctx* ctx, void* hip_stream, int32_t batch, const void* q, const cb_kv_layer* kv,
                          const int32_t* kv_len, const int32_t* node_offsets, const int32_t* d_tree_parent,
                          const int32_t* d_draft_tokens, const void* logits, void* attn_out,
                          int32_t* d_accepted_len, int32_t* d_accepted_tokens) {
  int rc = check_common(ctx, batch, q, kv, kv_len, node_offsets, logits, attn_out);
  if (rc) return rc;
  ctx->err[0] = 0;
  if (!d_tree_parent || !d_draft_tokens || !d_accepted_len || !d_accepted_tokens)
    return set_err(ctx, CB_EINVAL, "null argument");
  rc = check_device_shapes(ctx, batch, kv, kv_len, node_offsets);
  if (rc) return rc;
  return run_pipeline(ctx, static_cast<hipStream_t>(hip_stream), batch, q, kv, kv_len, node_offsets, d_tree_parent,
                      d_draft_tokens, logits, attn_out, d_accepted_len, d_accepted_tokens);
}

int cb_tree_attention_device(cb_ctx* ctx, void* hip_stream, int32_t batch, const void* q, const cb_kv_layer* kv,
                             const int32_t* kv_len, const int32_t* node_offsets, const int32_t* d_tree_parent,
                             void* attn_out) {
  if (!ctx) return set_err(nullptr, CB_EINVAL, "null context");
  ctx->err[0] = 0;
  if (!q || !kv || !kv_len || !node_offsets || !d_tree_parent || !attn_out) return set_err(ctx, CB_EINVAL, "null argument");
  if (batch < 1 || batch > ctx->cfg.max_batch) return set_err(ctx, CB_EINVAL, "batch %d outside [1, %d]", batch, ctx->cfg.max_batch);
  if (((uintptr_t)q | (uintptr_t)kv->k | (uintptr_t)kv->v | (uintptr_t)attn_out) & 15)
    return set_err(ctx, CB_EINVAL, "device pointers must be 16-byte aligned");
  const int rc = check_device_shapes(ctx, batch, kv, kv_len, node_offsets);
  if (rc) return rc;
  return run_pipeline(ctx, static_cast<hipStream_t>(hip_stream), batch, q, kv, kv_len, node_offsets, d_tree_parent,
                      nullptr, nullptr, attn_out, nullptr, nullptr, 3);
}

int cb_tree_attention_noalloc(const cb_config* cfg, void* hip_stream, int32_t batch, const void* q, const cb_kv_layer* kv,
                              const int32_t* kv_len, const int32_t* node_offsets, const int32_t* d_tree_parent,
                              void* attn_out) {
  g_init_err[0] = 0;
  if (!config_ok(cfg, g_init_err, sizeof g_init_err)) return CB_EINVAL;
  if (!q || !kv || !kv_len || !node_offsets || !d_tree_parent || !attn_out) return set_err(nullptr, CB_EINVAL, "null argument");
  if (batch < 1 || batch > cfg->max_batch) return set_err(nullptr, CB_EINVAL, "batch %d outside [1, %d]", batch, cfg->max_batch);
  if (((uintptr_t)q | (uintptr_t)kv->k | (uintptr_t)kv->v | (uintptr_t)attn_out) & 15)
    return set_err(nullptr, CB_EINVAL, "device pointers must be 16-byte aligned");
  // A context on the stack, never handed out: configuration, options at their defaults, and a
  // workspace layout cut from the static array for exactly this call's shapes.
  cb_ctx tmp{};
  tmp.cfg = *cfg;
  tmp.opt_stages = 15;
  tmp.opt_coop = 1;
  tmp.opt_spin = 256;
  int rc = check_device_shapes(&tmp, batch, kv, kv_len, node_offsets);
  if (rc) {
    memcpy(g_init_err, tmp.err, sizeof g_init_err);
    return rc;
  }
  const int total = node_offsets[batch];
  const WsLayout full = ws_layout(*cfg);
  const Plan plan = plan_attention(*cfg, full.max_splits, full.scalar_splits, 0, 0, batch, kv_len, node_offsets);
  const int g = cfg->num_q_heads / cfg->num_kv_heads;
  const int tile_count = batch * cfg->num_kv_heads * ((plan.max_nodes * g + kRowTile - 1) / kRowTile);
  WsLayout L{};
  L.max_total_nodes = total;
  L.max_splits = plan.nsplit;
  L.scalar_splits = plan.nsplit;
  L.amax_chunks = full.amax_chunks;
  L.ticket_count = 4 * tile_count;
  size_t o = 0;
  auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
  L.status = take(4);
  L.tickets = take((size_t)L.ticket_count * 4);
  L.coop_tickets = take((size_t)kCoopTiles * kCoopTicketStride);
  L.anc = take((size_t)total * kAncWords * 4);
  L.dbg = L.anc;                    // (never written: the timing aid is off)
  L.partial = take(plan.nsplit <= 1 ? 0
                   : plan.impl == 2 ? attn_mfma_partial_bytes(total, cfg->num_q_heads, cfg->num_kv_heads, batch, plan.nsplit)
                                    : (size_t)total * cfg->num_q_heads * plan.nsplit * partial_stride(cfg->head_dim) * 4);
  L.total = o;
  if (L.total > kStaticScratchBytes)
    return set_err(nullptr, CB_ECAP, "this call needs %zu bytes of scratch memory, the library's fixed buffer has %zu", L.total, kStaticScratchBytes);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess || dev < 0 || dev >= kMaxDevices) return set_err(nullptr, CB_EHIP, "hipGetDevice: %s", hipGetErrorString(e));
  void* base = nullptr;
  {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_scratch_ptr[dev]) {
      void* ptr = nullptr;
      e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(g_static_scratch));
      if (e != hipSuccess || !ptr) return set_err(nullptr, CB_EHIP, "hipGetSymbolAddress: %s", hipGetErrorString(e));
      g_static_scratch_ptr[dev] = ptr;
    }
    base = g_static_scratch_ptr[dev];
  }
  tmp.lay = L;
  tmp.fixed_plan = &plan;
  tmp.ws = static_cast<char*>(base);
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  // The array is shared by every call on this GPU and keeps the last call's contents: the words that
  // must start at zero are cleared here, by a kernel (a caller may be capturing the stream).
  e = launch_zero_words(st, tmp.dev<unsigned long long>(L.status), 1, 1, 1);
  if (e == hipSuccess) e = launch_zero_words(st, tmp.dev<unsigned long long>(L.tickets), L.ticket_count / 2, 1, 1);
  if (e == hipSuccess) e = launch_zero_words(st, tmp.dev<unsigned long long>(L.coop_tickets), std::min(tile_count, kCoopTiles), kCoopTicketStride / 8, 2);
  if (e != hipSuccess) return set_err(nullptr, CB_EHIP, "clearing the scratch counters: %s", hipGetErrorString(e));
  rc = run_pipeline(&tmp, st, batch, q, kv, kv_len, node_offsets, d_tree_parent, nullptr, nullptr, attn_out, nullptr, nullptr, 3);
  if (rc) memcpy(g_init_err, tmp.err, sizeof g_init_err);
  return rc;
}

int cb_verify_tree(cb_ctx* ctx, void* hip_stream, int32_t batch, const void* q, const cb_kv_layer* kv,
                   const int32_t* kv_len, const int32_t* node_offsets, const int32_t* tree_parent,
                   const int32_t* draft_tokens, const void* logits, void* attn_out, int32_t* accepted_len,
                   int32_t* accepted_tokens) {
  int rc = check_common(ctx, batch, q, kv, kv_len, node_offsets, logits, attn_out);
  if (rc) return rc;
  ctx->err[0] = 0;
  if (!tree_parent || !draft_tokens || !accepted_len || !accepted_tokens) return set_err(ctx, CB_EINVAL, "null argument");
  rc = cb_check_verify_args(&ctx->cfg, batch, kv, kv_len, node_offsets, tree_parent, ctx->err, sizeof ctx->err);
  if (rc) return rc;
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int total = node_offsets[batch];
  const size_t stride = (size_t)ctx->cfg.max_depth + 1;
  // No copies: the kernels read the tree from, and write the results to, the context's pinned host
  // block through its device address (a few hundred bytes each way; two staged copies cost more
  // than the kernels' reads across the bus).  Parents and tokens back to back, lengths and tokens
  // back to back.  Calls alternate between two tree areas: this call may return before its launch
  // has ended (below), and the launch of the call before it has ended by the time this one's
  // results arrive, because both run on one stream (run_pipeline synchronises when the stream changes).
  const bool early = ctx->opt_full_sync == 0 && (ctx->opt_stages & 8) != 0;
  ctx->call_seq = ctx->call_seq == INT32_MAX ? 1 : ctx->call_seq + 1;
  int32_t* h_tree = ctx->h_parent + (size_t)(ctx->call_seq & 1) * 2 * ctx->lay.max_total_nodes;
  memcpy(h_tree, tree_parent, (size_t)total * 4);
  memcpy(h_tree + total, draft_tokens, (size_t)total * 4);
  int32_t* d_parent = ctx->d_hblock + (h_tree - static_cast<int32_t*>(ctx->h_block));
  int32_t* d_tokens = d_parent + total;
  int32_t* h_res = ctx->h_len;
  int32_t* d_len = ctx->d_hblock + (h_res - static_cast<int32_t*>(ctx->h_block));
  int32_t* d_tok = d_len + batch;
  if (early) ctx->want_done = ctx->d_hblock + (ctx->h_done - static_cast<int32_t*>(ctx->h_block));
  rc = run_pipeline(ctx, st, batch, q, kv, kv_len, node_offsets, d_parent, d_tokens, logits, attn_out, d_len, d_tok);
  ctx->want_done = nullptr;
  if (rc) return rc;
  if (early) {
    // The acceptance stores a sequence's results, makes them visible at system scope and then stores
    // the call's number into the sequence's flag word; the host returns as soon as every flag shows
    // it, without waiting for the rest of the launch (the attention's split merge) and for the
    // stream's completion signal.  The stream's state is looked at now and then, so that a failed
    // launch ends the wait.
    const int32_t want = ctx->call_seq;
    bool seen = false;
    for (uint32_t polls = 1; !seen; polls++) {
      seen = true;
      for (int b = 0; b < batch; b++)
        if (__atomic_load_n(ctx->h_done + b, __ATOMIC_ACQUIRE) != want) { seen = false; break; }
      if (seen) break;
      if ((polls & 2047) == 0) {
        const hipError_t q_rc = hipStreamQuery(st);
        if (q_rc == hipSuccess) {  // everything has run: the flags are there now or never
          seen = true;
          for (int b = 0; b < batch; b++)
            if (__atomic_load_n(ctx->h_done + b, __ATOMIC_ACQUIRE) != want) seen = false;
          if (!seen) return set_err(ctx, CB_EHIP, "the verification ran but its results did not arrive");
        } else if (q_rc != hipErrorNotReady) {
          return set_err(ctx, CB_EHIP, "%s: %s", "hipStreamQuery", hipGetErrorString(q_rc));
        }
      }
      __builtin_ia32_pause();
    }
    ctx->unsynced = st;
    ctx->have_unsynced = true;
  } else {
    CB_HIP(ctx, hipStreamSynchronize(st));
  }
  memcpy(accepted_len, h_res, (size_t)batch * 4);
  memcpy(accepted_tokens, h_res + batch, (size_t)batch * stride * 4);
  memcpy(ctx->last_len, h_res, (size_t)batch * 4);
  ctx->host_knows_len = true;
  return CB_OK;
}

int cb_compact_kv(cb_ctx* ctx, void* hip_stream, int32_t num_layers, const cb_kv_layer* layers, int32_t* new_kv_len) {
  if (!ctx) return set_err(nullptr, CB_EINVAL, "null context");
  ctx->err[0] = 0;
  if (!ctx->have_verify) return set_err(ctx, CB_ESTATE, "cb_compact_kv needs a preceding successful verify call");
  if (!layers || num_layers < 1 || num_layers > CB_MAX_LAYERS) return set_err(ctx, CB_EINVAL, "num_layers outside [1, %d]", CB_MAX_LAYERS);
  const cb_config& c = ctx->cfg;
  KvAddr addrs[CB_MAX_LAYERS];
  for (int l = 0; l < num_layers; l++) {
    const cb_kv_layer& y = layers[l];
    if (!y.k || !y.v || (((uintptr_t)y.k | (uintptr_t)y.v) & 15)) return set_err(ctx, CB_EINVAL, "layer %d: null or misaligned cache pointer", l);
    if (y.capacity_or_num_blocks != layers[0].capacity_or_num_blocks || y.block_table != layers[0].block_table ||
        y.max_blocks_per_seq != layers[0].max_blocks_per_seq || y.layout != layers[0].layout)
      return set_err(ctx, CB_EINVAL, "layer %d does not share the geometry of layer 0", l);
    if (!make_kv_addr(c, y, &addrs[l])) return set_err(ctx, CB_EINVAL, "unknown cache layout %d", y.layout);
  }
  if (c.block_size > 0 && (!layers[0].block_table || layers[0].max_blocks_per_seq < 1)) return set_err(ctx, CB_EINVAL, "paged cache without a block table");
  for (int b = 0; b < ctx->batch; b++) {
    const int64_t n = ctx->meta.node_off[b + 1] - ctx->meta.node_off[b];
    const int64_t room = c.block_size > 0 ? (int64_t)layers[0].max_blocks_per_seq * c.block_size : layers[0].capacity_or_num_blocks;
    if (ctx->meta.kv_len[b] + n > room) return set_err(ctx, CB_ECAP, "sequence %d does not fit these caches", b);
  }
  hipStream_t st = static_cast<hipStream_t>(hip_stream);
  const int eb = c.qkv_dtype == CB_F32 ? 4 : 2;
  CB_HIP(ctx, launch_compact(st, ctx->batch, ctx->meta, addrs, num_layers, c.num_kv_heads, c.head_dim, eb, c.max_depth,
                             ctx->dev<int32_t>(ctx->lay.path), ctx->dev<int32_t>(ctx->lay.len_ctx),
                             ctx->dev<int32_t>(ctx->lay.new_len)));
  if (new_kv_len) {
    if (ctx->host_knows_len) {
      for (int b = 0; b < ctx->batch; b++) new_kv_len[b] = ctx->meta.kv_len[b] + ctx->last_len[b] + 1;
    } else {
      CB_HIP(ctx, hipMemcpyAsync(ctx->h_misc + 1, ctx->dev<int32_t>(ctx->lay.new_len), (size_t)ctx->batch * 4, hipMemcpyDeviceToHost, st));
      CB_HIP(ctx, hipStreamSynchronize(st));
      memcpy(new_kv_len, ctx->h_misc + 1, (size_t)ctx->batch * 4);
    }
  }
  return CB_OK;
}

int cb_get_path(cb_ctx* ctx, int32_t* path) {
  if (!ctx || !path) return set_err(ctx, CB_EINVAL, "null argument");
  if (!ctx->have_verify) return set_err(ctx, CB_ESTATE, "no verify call yet");
  const size_t n = (size_t)ctx->batch * (ctx->cfg.max_depth + 1);
  CB_HIP(ctx, hipMemcpyAsync(ctx->h_path, ctx->dev<int32_t>(ctx->lay.path), n * 4, hipMemcpyDeviceToHost, ctx->last_stream));
  CB_HIP(ctx, hipStreamSynchronize(ctx->last_stream));
  memcpy(path, ctx->h_path, n * 4);
  return CB_OK;
}

int cb_get_argmax(cb_ctx* ctx, int32_t* argmax) {
  if (!ctx || !argmax) return set_err(ctx, CB_EINVAL, "null argument");
  if (!ctx->have_verify) return set_err(ctx, CB_ESTATE, "no verify call yet");
  const size_t n = (size_t)ctx->total_nodes;
  CB_HIP(ctx, hipMemcpyAsync(ctx->h_argmax, ctx->dev<int32_t>(ctx->lay.amax_out), n * 4, hipMemcpyDeviceToHost, ctx->last_stream));
  CB_HIP(ctx, hipStreamSynchronize(ctx->last_stream));
  memcpy(argmax, ctx->h_argmax, n * 4);
  return CB_OK;
}

int cb_device_status(cb_ctx* ctx, int32_t* status) {
  if (!ctx || !status) return set_err(ctx, CB_EINVAL, "null argument");
  hipStream_t st = ctx->have_verify ? ctx->last_stream : nullptr;
  CB_HIP(ctx, hipMemcpyAsync(ctx->h_misc, ctx->dev<int32_t>(ctx->lay.status), 4, hipMemcpyDeviceToHost, st));
  CB_HIP(ctx, hipStreamSynchronize(st));
  *status = ctx->h_misc[0];
  CB_HIP(ctx, hipMemsetAsync(ctx->dev<int32_t>(ctx->lay.status), 0, 4, st));  // reading clears the sticky word
  CB_HIP(ctx, hipStreamSynchronize(st));
  return CB_OK;
}

int cb_set_option(cb_ctx* ctx, const char* name, int64_t value) {
  if (!ctx || !name) return set_err(ctx, CB_EINVAL, "null argument");
  if (!strcmp(name, "splits")) ctx->opt_splits = value;
  else if (!strcmp(name, "attn_impl")) ctx->opt_impl = value;
  else if (!strcmp(name, "time_attention")) ctx->opt_time = value;
  else if (!strcmp(name, "stages")) ctx->opt_stages = value & 15;
  else if (!strcmp(name, "timeline")) ctx->opt_timeline = value;
  else if (!strcmp(name, "full_sync")) ctx->opt_full_sync = value;
  else if (!strcmp(name, "external_merge")) ctx->opt_external = value;
  else if (!strcmp(name, "parallel_scan")) ctx->opt_fork = value;
  else if (!strcmp(name, "fuse_logits")) ctx->opt_fuse = value;
  else if (!strcmp(name, "coop_merge")) ctx->opt_coop = value;
  else if (!strcmp(name, "merge_spin_limit")) ctx->opt_spin = value < 0 ? 0 : (value > 4096 ? 4096 : value);
  else return set_err(ctx, CB_EINVAL, "unknown option '%s'", name);
  return CB_OK;
}

int cb_last_launch_info(cb_ctx* ctx, int32_t info[6]) {
  if (!ctx || !info) return set_err(ctx, CB_EINVAL, "null argument");
  if (!ctx->have_verify) return set_err(ctx, CB_ESTATE, "no verify call yet");
  for (int i = 0; i < 6; i++) info[i] = ctx->launch_info[i];
  return CB_OK;
}

int cb_last_attention_ms(cb_ctx* ctx, float* ms) {
  if (!ctx || !ms) return set_err(ctx, CB_EINVAL, "null argument");
  if (!ctx->ev_valid) return set_err(ctx, CB_ESTATE, "option time_attention was not set for the last verify");
  CB_HIP(ctx, hipEventSynchronize(ctx->ev1));
  CB_HIP(ctx, hipEventElapsedTime(ms, ctx->ev0, ctx->ev1));
  return CB_OK;
}

int cb_debug_timestamps(cb_ctx* ctx, uint64_t* out, int32_t workgroups) {
  if (!ctx || !out || workgroups < 1 || workgroups > 1024) return set_err(ctx, CB_EINVAL, "bad argument");
  hipStream_t st = ctx->have_verify ? ctx->last_stream : nullptr;
  CB_HIP(ctx, hipStreamSynchronize(st));
  CB_HIP(ctx, hipMemcpy(out, ctx->ws + ctx->lay.dbg, (size_t)workgroups * 64, hipMemcpyDeviceToHost));
  return CB_OK;
}

const char* cb_last_error(const cb_ctx* ctx) { return ctx ? ctx->err : g_init_err; }

void cb_destroy(cb_ctx* ctx) {
  if (!ctx) return;
  if (ctx->have_unsynced) (void)hipStreamSynchronize(ctx->unsynced);  // its launch may still write the pinned block
  (void)hipEventDestroy(ctx->ev0);
  (void)hipEventDestroy(ctx->ev1);
  (void)hipEventDestroy(ctx->ev_fork);
  (void)hipEventDestroy(ctx->ev_join);
  (void)hipStreamDestroy(ctx->aux);
  (void)hipHostFree(ctx->h_block);
  delete ctx;
}

}  // extern "C"
