// C-ABI entry points of libdbsa (declared in include/dbsa.h): argument checks, the
// device mirror of a layout's lists, and kernel launches.  No arithmetic of the
// method lives here.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <vector>

#include "kernels.hpp"
#include "layout.hpp"

// Partial-state buffer of dbsa_decode_attn_static: one copy per GPU, held until the process ends.
// In host code this name is only a handle for hipGetSymbolAddress; the device address it yields
// (one per device) is what kernels and copies receive.
constexpr size_t kStaticScratchBytes = DBSA_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device, looked up once per device.
hipError_t static_scratch(void** out) {
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  if (device < 0 || device >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[device]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[device] = ptr;
  }
  *out = g_scratch_ptr[device];
  return hipSuccess;
}

// Device blocks (with a pinned staging twin) are recycled between layouts: allocation
// calls, not the copied bytes, dominate the cost of a layout build.  Nothing here waits for
// the GPU: a destroyed layout's block goes back to the pool together with one event per stream
// that read its lists (recorded at the destroy call), and is handed out again only once all of
// them have completed, so a layout can be built, used and destroyed while earlier work is
// still running.
struct ListBlock {
  void* dev;
  void* pinned;
  size_t capacity;
  int device;
  std::vector<hipEvent_t> busy;  // all complete => nothing reads dev or pinned any more
};
std::mutex g_pool_mutex;
std::vector<ListBlock> g_pool_blocks;
// blocks kept per process: at the cap a build waits for the oldest busy block that fits instead of
// allocating, and idle blocks beyond it are freed, oldest first
constexpr size_t kMaxPoolBlocks = 16;

bool block_idle(ListBlock& blk) {
  for (hipEvent_t ev : blk.busy)
    if (hipEventQuery(ev) != hipSuccess) {
      (void)hipGetLastError();  // "not ready" is an answer, not an error to leave behind for the caller
      return false;
    }
  for (hipEvent_t ev : blk.busy) (void)hipEventDestroy(ev);
  blk.busy.clear();
  return true;
}

// Frees idle blocks, oldest first, until at most `keep` are pooled (g_pool_mutex held).  Blocks
// still read by running work stay; they go at a later call.
void trim_pool_locked(size_t keep) {
  for (size_t i = 0; i < g_pool_blocks.size() && g_pool_blocks.size() > keep;) {
    if (!block_idle(g_pool_blocks[i])) {
      ++i;
      continue;
    }
    (void)hipFree(g_pool_blocks[i].dev);
    (void)hipHostFree(g_pool_blocks[i].pinned);
    g_pool_blocks.erase(g_pool_blocks.begin() + static_cast<std::ptrdiff_t>(i));
  }
}

hipError_t acquire_block(size_t bytes, ListBlock* out) {
  int device = 0;
  hipError_t e = hipGetDevice(&device);
  if (e != hipSuccess) return e;
  {
    std::lock_guard<std::mutex> lock(g_pool_mutex);
    auto take = [&](size_t i) {
      *out = g_pool_blocks[i];
      g_pool_blocks.erase(g_pool_blocks.begin() + static_cast<std::ptrdiff_t>(i));
    };
    size_t fits = g_pool_blocks.size();
    for (size_t i = 0; i < g_pool_blocks.size(); ++i)
      if (g_pool_blocks[i].device == device && g_pool_blocks[i].capacity >= bytes) {
        if (block_idle(g_pool_blocks[i])) {
          take(i);
          return hipSuccess;
        }
        if (fits == g_pool_blocks.size()) fits = i;  // the one destroyed first
      }
    if (g_pool_blocks.size() >= kMaxPoolBlocks && fits < g_pool_blocks.size()) {
      for (hipEvent_t ev : g_pool_blocks[fits].busy) {
        e = hipEventSynchronize(ev);
        if (e != hipSuccess) return e;
      }
      (void)block_idle(g_pool_blocks[fits]);
      take(fits);
      return hipSuccess;
    }
    // no pooled block is large enough: make room for the new one among those that are too small
    if (g_pool_blocks.size() >= kMaxPoolBlocks) trim_pool_locked(kMaxPoolBlocks - 1);
  }
  ListBlock blk{nullptr, nullptr, (bytes + bytes / 2 + 65535) / 65536 * 65536, device, {}};
  e = hipMalloc(&blk.dev, blk.capacity);
  if (e != hipSuccess) return e;
  e = hipHostMalloc(&blk.pinned, blk.capacity, hipHostMallocDefault);
  if (e != hipSuccess) {
    (void)hipFree(blk.dev);
    return e;
  }
  *out = blk;
  return hipSuccess;
}

void release_block(const ListBlock& blk) {
  std::lock_guard<std::mutex> lock(g_pool_mutex);
  g_pool_blocks.push_back(blk);
  trim_pool_locked(kMaxPoolBlocks);
}

// Copy every list into ONE device block with a single asynchronous copy from pinned memory.
hipError_t upload_lists(dbsa_layout* L, hipStream_t stream) {
  auto pad = [](size_t n) { return (n + 255) / 256 * 256; };
  const size_t b_tab = L->qtile_tab.size() * sizeof(int32_t), b_ptr = L->list_ptr.size() * sizeof(int64_t),
               b_ent = L->list_ent.size() * sizeof(int32_t), b_ord = L->order.size() * sizeof(int32_t),
               b_dec = L->dec_ent.size() * sizeof(int32_t), b_spl = L->split_ptr.size() * sizeof(int64_t),
               b_gsp = L->gm_slot_ptr.size() * sizeof(int64_t),
               b_lsh = L->list_shift.size() * sizeof(int32_t), b_gir = L->gm_item_run.size() * sizeof(int32_t),
               b_grp = L->gm_ref_pad.size() * sizeof(int32_t), b_grw = L->gm_rows.size() * sizeof(int32_t),
               b_gse = L->gm_seg_ent.size() * sizeof(int32_t), b_gqr = L->gm_qrefs.size() * sizeof(int32_t),
               b_srec = L->qtile_tab.size() * sizeof(int32_t), b_sptr = (kMaxSchedClasses + 1) * sizeof(int32_t),
               b_mrec = L->mx_rec.size() * sizeof(int32_t), b_dsh = L->dec_shift.size() * sizeof(int32_t),
               b_gqs = L->gm_qshift.size() * sizeof(int32_t), b_mqr = L->mx_qrefs.size() * sizeof(int32_t),
               b_mqs = L->mx_qshift.size() * sizeof(int32_t), b_msp = L->mx_slot_ptr.size() * sizeof(int64_t);
  const size_t o_tab = 0, o_ptr = o_tab + pad(b_tab), o_ent = o_ptr + pad(b_ptr), o_ord = o_ent + pad(b_ent),
               o_dec = o_ord + pad(b_ord), o_spl = o_dec + pad(b_dec), o_gsp = o_spl + pad(b_spl),
               o_lsh = o_gsp + pad(b_gsp), o_gir = o_lsh + pad(b_lsh), o_grp = o_gir + pad(b_gir),
               o_grw = o_grp + pad(b_grp), o_gse = o_grw + pad(b_grw), o_gqr = o_gse + pad(b_gse),
               o_dsh = o_gqr + pad(b_gqr), o_gqs = o_dsh + pad(b_dsh), o_mqr = o_gqs + pad(b_gqs), o_mqs = o_mqr + pad(b_mqr), o_msp = o_mqs + pad(b_mqs),
               o_srec = o_msp + pad(b_msp), o_sptr = o_srec + pad(b_srec), o_mrec = o_sptr + pad(b_sptr),
               o_mptr = o_mrec + pad(b_mrec), lists_end = o_srec, total = o_mptr + pad(b_sptr) + 256;
  ListBlock blk{};
  hipError_t e = acquire_block(total, &blk);
  if (e != hipSuccess) return e;
  unsigned char* h = static_cast<unsigned char*>(blk.pinned);
  auto put = [&](size_t off, const void* src, size_t bytes) {
    if (bytes) std::memcpy(h + off, src, bytes);
  };
  put(o_tab, L->qtile_tab.data(), b_tab);
  put(o_ptr, L->list_ptr.data(), b_ptr);
  put(o_ent, L->list_ent.data(), b_ent);
  put(o_ord, L->order.data(), b_ord);
  put(o_dec, L->dec_ent.data(), b_dec);
  put(o_spl, L->split_ptr.data(), b_spl);
  put(o_gsp, L->gm_slot_ptr.data(), b_gsp);
  put(o_lsh, L->list_shift.data(), b_lsh);
  put(o_gir, L->gm_item_run.data(), b_gir);
  put(o_grp, L->gm_ref_pad.data(), b_grp);
  put(o_grw, L->gm_rows.data(), b_grw);
  put(o_gse, L->gm_seg_ent.data(), b_gse);
  put(o_gqr, L->gm_qrefs.data(), b_gqr);
  put(o_dsh, L->dec_shift.data(), b_dsh);
  put(o_gqs, L->gm_qshift.data(), b_gqs);
  put(o_mqr, L->mx_qrefs.data(), b_mqr);
  put(o_mqs, L->mx_qshift.data(), b_mqs);
  put(o_msp, L->mx_slot_ptr.data(), b_msp);
  // the staging twin stays with the block, so nothing has to wait for the copy here; calls on
  // other streams are ordered behind it through the event
  hipEvent_t uploaded = nullptr;
  e = hipEventCreateWithFlags(&uploaded, hipEventDisableTiming);
  if (e == hipSuccess) {
    // (the room behind lists_end is filled by the first calls that use a schedule)
    e = hipMemcpyAsync(blk.dev, blk.pinned, lists_end, hipMemcpyHostToDevice, stream);
    if (e == hipSuccess) e = hipEventRecord(uploaded, stream);
    if (e != hipSuccess) {
      (void)hipStreamSynchronize(stream);  // the copy may have been queued: the block must not be reused under it
      (void)hipEventDestroy(uploaded);
    }
  }
  if (e != hipSuccess) {
    release_block(blk);
    return e;
  }
  L->dev.upload_stream = stream;
  L->dev.uploaded = uploaded;
  unsigned char* b = static_cast<unsigned char*>(blk.dev);
  L->dev.base = blk.dev;
  L->dev.staging = blk.pinned;
  L->dev.capacity = blk.capacity;
  L->dev.device = blk.device;
  L->dev.qtile_tab = reinterpret_cast<int32_t*>(b + o_tab);
  L->dev.list_ptr = reinterpret_cast<int64_t*>(b + o_ptr);
  L->dev.list_ent = reinterpret_cast<int32_t*>(b + o_ent);
  L->dev.order = reinterpret_cast<int32_t*>(b + o_ord);
  L->dev.dec_ent = reinterpret_cast<int32_t*>(b + o_dec);
  L->dev.split_ptr = reinterpret_cast<int64_t*>(b + o_spl);
  L->dev.gm_slot_ptr = reinterpret_cast<int64_t*>(b + o_gsp);
  L->dev.list_shift = reinterpret_cast<int32_t*>(b + o_lsh);
  L->dev.gm_item_run = reinterpret_cast<int32_t*>(b + o_gir);
  L->dev.gm_ref_pad = reinterpret_cast<int32_t*>(b + o_grp);
  L->dev.gm_rows = reinterpret_cast<int32_t*>(b + o_grw);
  L->dev.gm_seg_ent = reinterpret_cast<int32_t*>(b + o_gse);
  L->dev.gm_qrefs = reinterpret_cast<int32_t*>(b + o_gqr);
  L->dev.dec_shift = reinterpret_cast<int32_t*>(b + o_dsh);
  L->dev.gm_qshift = reinterpret_cast<int32_t*>(b + o_gqs);
  L->dev.mx_qrefs = reinterpret_cast<int32_t*>(b + o_mqr);
  L->dev.mx_qshift = reinterpret_cast<int32_t*>(b + o_mqs);
  L->dev.mx_slot_ptr = reinterpret_cast<int64_t*>(b + o_msp);
  L->dev.sched_rec = reinterpret_cast<int32_t*>(b + o_srec);
  L->dev.sched_ptr = reinterpret_cast<int32_t*>(b + o_sptr);
  L->dev.mx_sched_rec = reinterpret_cast<int32_t*>(b + o_mrec);
  L->dev.mx_sched_ptr = reinterpret_cast<int32_t*>(b + o_mptr);
  return hipSuccess;
}

// Hand the block back without waiting: one event per stream that read the lists, recorded now.
void free_device_lists(dbsa_layout* L) {
  dbsa_device_lists& d = L->dev;
  if (d.base) {
    int current = d.device;
    (void)hipGetDevice(&current);
    if (current != d.device) (void)hipSetDevice(d.device);
    ListBlock blk{d.base, d.staging, d.capacity, d.device, {}};
    std::vector<void*> streams;
    {
      std::lock_guard<std::mutex> lock(L->use_mutex);
      streams = L->used_streams;
    }
    if (std::find(streams.begin(), streams.end(), d.upload_stream) == streams.end()) streams.push_back(d.upload_stream);
    bool recorded = true;
    for (void* s : streams) {
      hipEvent_t ev = nullptr;
      if (hipEventCreateWithFlags(&ev, hipEventDisableTiming) != hipSuccess) {
        recorded = false;
        break;
      }
      blk.busy.push_back(ev);
      if (hipEventRecord(ev, static_cast<hipStream_t>(s)) != hipSuccess) {
        recorded = false;
        break;
      }
    }
    if (!recorded) {  // e.g. a stream that no longer exists: fall back to waiting for everything
      (void)hipGetLastError();
      (void)hipDeviceSynchronize();
      for (hipEvent_t ev : blk.busy) (void)hipEventDestroy(ev);
      blk.busy.clear();
    }
    if (d.uploaded) (void)hipEventDestroy(static_cast<hipEvent_t>(d.uploaded));
    if (d.sched_uploaded) (void)hipEventDestroy(static_cast<hipEvent_t>(d.sched_uploaded));
    if (d.mx_uploaded) (void)hipEventDestroy(static_cast<hipEvent_t>(d.mx_uploaded));
    release_block(blk);
    if (current != d.device) (void)hipSetDevice(current);
  }
  d = dbsa_device_lists{};
}

// First call of a layout on a stream other than the one its lists were copied on: order the
// stream behind the copy.  Every stream is remembered for the destroy call.
hipError_t order_behind_upload(const dbsa_layout* L, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(L->use_mutex);
  void* s = stream;
  if (std::find(L->used_streams.begin(), L->used_streams.end(), s) != L->used_streams.end()) return hipSuccess;
  if (s != L->dev.upload_stream) {
    const hipError_t e = hipStreamWaitEvent(stream, static_cast<hipEvent_t>(L->dev.uploaded), 0);
    if (e != hipSuccess) return e;
  }
  L->used_streams.push_back(s);
  return hipSuccess;
}

// compute units of the current device (what a persistent launch and the decode chunking are sized for)
int device_compute_units() {
  static std::mutex m;
  static int cus[kMaxDevices] = {};
  int device = 0;
  if (hipGetDevice(&device) != hipSuccess || device < 0 || device >= kMaxDevices) return 256;
  std::lock_guard<std::mutex> lock(m);
  if (!cus[device]) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, device) != hipSuccess || n <= 0) n = 256;
    cus[device] = n;
  }
  return cus[device];
}

// One persistent-launch schedule of a layout: its host copy, its room in the device block, the
// event behind its copy.
struct ScheduleSlot {
  int32_t* classes;
  std::vector<int32_t>* ptr;
  std::vector<int32_t>* rec;
  bool* on_device;
  int32_t* dev_rec;
  int32_t* dev_ptr;
  void** uploaded;
  void** upload_stream;
};

// The schedule in `slot` for n_classes workers per head block, on the device and ordered before
// `stream`'s next work; `balance` fills it on first use.  A slot keeps ONE schedule: false if it
// already holds one for another number of workers, or if the schedule would have to be copied
// while the stream is being captured into a graph (the caller then takes its other launch form).
template <typename Balance>
bool ensure_slot(const dbsa_layout* L, const ScheduleSlot& slot, int32_t n_classes, hipStream_t stream, Balance&& balance) {
  if (n_classes < 1 || n_classes > kMaxSchedClasses || !slot.dev_rec) return false;
  std::lock_guard<std::mutex> lock(L->sched_mutex);
  if (*slot.classes != 0 && *slot.classes != n_classes) return false;
  if (!*slot.on_device) {
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone) {
      (void)hipGetLastError();
      return false;
    }
    if (*slot.classes == 0) {
      balance(n_classes, slot.ptr, slot.rec);
      *slot.classes = n_classes;
    }
    // through the pinned twin of the device block, at the same offsets
    unsigned char* dev = static_cast<unsigned char*>(L->dev.base);
    unsigned char* pin = static_cast<unsigned char*>(L->dev.staging);
    const size_t o_rec = reinterpret_cast<unsigned char*>(slot.dev_rec) - dev;
    const size_t o_ptr = reinterpret_cast<unsigned char*>(slot.dev_ptr) - dev;
    const size_t b_ptr = slot.ptr->size() * sizeof(int32_t);
    std::memcpy(pin + o_rec, slot.rec->data(), slot.rec->size() * sizeof(int32_t));
    std::memcpy(pin + o_ptr, slot.ptr->data(), b_ptr);
    hipEvent_t done = nullptr;
    if (hipEventCreateWithFlags(&done, hipEventDisableTiming) != hipSuccess) return false;
    if (hipMemcpyAsync(dev + o_rec, pin + o_rec, o_ptr + b_ptr - o_rec, hipMemcpyHostToDevice, stream) != hipSuccess ||
        hipEventRecord(done, stream) != hipSuccess) {
      (void)hipStreamSynchronize(stream);
      (void)hipEventDestroy(done);
      return false;
    }
    *slot.uploaded = done;
    *slot.upload_stream = stream;
    *slot.on_device = true;
  } else if (stream != *slot.upload_stream) {
    if (hipStreamWaitEvent(stream, static_cast<hipEvent_t>(*slot.uploaded), 0) != hipSuccess) return false;
  }
  return true;
}

// the schedule of the prefill-shaped launches over the layout's Q tiles
bool ensure_schedule(const dbsa_layout* L, int32_t n_classes, hipStream_t stream) {
  const ScheduleSlot slot{&L->sched_classes, &L->sched_ptr, &L->sched_rec, &L->sched_on_device, L->dev.sched_rec,
                          L->dev.sched_ptr, &L->dev.sched_uploaded, &L->dev.sched_stream};
  return ensure_slot(L, slot, n_classes, stream, [&](int32_t n, std::vector<int32_t>* ptr, std::vector<int32_t>* rec) {
    dbsa_balance_schedule(L, n, ptr, rec);
  });
}

// the schedule of a decode step that runs its pool items as a contraction (dbsa_layout::mx_rec)
// (planned: the layout cut its runs for exactly these workers, mx_plan_ptr deals them)
bool ensure_matrix_schedule(const dbsa_layout* L, int32_t n_classes, bool planned, hipStream_t stream) {
  if (L->mx_rec.empty()) return false;
  const ScheduleSlot slot{&L->mx_classes, &L->mx_sched_ptr, &L->mx_sched_rec, &L->mx_on_device, L->dev.mx_sched_rec,
                          L->dev.mx_sched_ptr, &L->dev.mx_uploaded, &L->dev.mx_stream};
  return ensure_slot(L, slot, n_classes, stream, [&](int32_t n, std::vector<int32_t>* ptr, std::vector<int32_t>* rec) {
    if (planned) {
      *ptr = L->mx_plan_ptr;
      *rec = L->mx_rec;
    } else {
      dbsa_balance_records(L->mx_rec, n, ptr, rec);
    }
  });
}

bool tensor_ok(const dbsa_tensor& t, int dtype) {
  const int64_t align_elems = dtype == DBSA_BF16 ? 8 : 4;
  return t.ptr != nullptr && (reinterpret_cast<uintptr_t>(t.ptr) % 16 == 0) && t.stride_tok > 0 &&
         t.stride_head > 0 && t.stride_tok % align_elems == 0 && t.stride_head % align_elems == 0;
}

TensorView view(const dbsa_tensor& t) { return TensorView{t.ptr, t.stride_tok, t.stride_head}; }

int check_shapes(int32_t dtype, int32_t hq, int32_t hkv, int32_t d, float scale) {
  if (dtype != DBSA_BF16 && dtype != DBSA_F32) return DBSA_ERR_UNSUPPORTED;
  if (hq <= 0 || hkv <= 0 || !(scale > 0.f) || !std::isfinite(scale)) return DBSA_ERR_INVALID_ARG;
  if (hq % hkv != 0) return DBSA_ERR_UNSUPPORTED;
  if (d != 64 && d != 128) return DBSA_ERR_UNSUPPORTED;
  return DBSA_OK;
}

// Largest number of query heads one workgroup can take so that heads * (block_m/32)
// wavefronts <= 8 and the heads share one KV head.
int pick_heads_per_block(int r, int block_m) {
  const int subs = block_m / 32;
  int best = 1;
  for (int h = 1; h <= r; ++h)
    if (r % h == 0 && h * subs <= 8) {
      const int nw = h * subs;
      if (nw == 1 || nw == 2 || nw == 4 || nw == 8) best = h;
    }
  return best;
}

// split query prefill: most runs per list, fewest tiles per run
constexpr int64_t kMaxQuerySplit = 4;
constexpr int64_t kMinRun = 16;
// The kernel that re-positions (attn_prefill.hip) starts a row's running maximum from the first
// tile of its run, so that tile must hold a key the row sees.  Only the tiles on a Q tile's own
// diagonal hide keys from some of its rows, they are the last block_m / 64 entries of a list and
// every row sees the first of them: a run of more entries than that never starts behind it.
static_assert(kMinRun > 256 / 64, "a run of a split list must reach back beyond the diagonal tiles of a Q tile");
// workgroups the device the layout was built for holds at two per compute unit
int64_t workgroup_slots(const dbsa_layout* L) { return 2 * static_cast<int64_t>(L->compute_units); }

// bytes of partial states one decode step writes: the larger of its two schedules
size_t decode_workspace_need(const dbsa_layout* L, int32_t n_q_heads, int32_t head_dim) {
  const size_t slots = std::max<size_t>(static_cast<size_t>(L->n_queries) * L->n_split,
                                        std::max<size_t>(L->gm_slot_ptr.empty() ? 0 : static_cast<size_t>(L->gm_slot_ptr.back()),
                                                   L->mx_slot_ptr.empty() ? 0 : static_cast<size_t>(L->mx_slot_ptr.back())));
  return slots * n_q_heads * (head_dim + kPartialPad) * sizeof(float);
}

bool mfma_tile_sizes_ok(const dbsa_layout* L) {
  const int bm = L->block_m;
  return L->block_n == 64 && (bm == 32 || bm == 64 || bm == 128 || bm == 256);
}

// Every step reads the same selected keys, more of them than the last-level cache holds, so a
// step that walks them in the order of the step before finds none of them cached.  Successive
// decode calls on one layout therefore alternate the direction in which each run of keys is
// walked (the query prefill walks forward): what the previous call read last is read first.
// Called once a call has passed every check, so that a rejected call leaves the order of
// summation of the next one as it was.
int32_t next_walk_direction(const dbsa_layout* L) { return L->last_walk_reversed.fetch_xor(1) ^ 1; }

// A re-positioning decode row of query u looks up id shift + self_len[u] - 1.  self_len lives on
// the device; what the host knows is that a query's cache holds at most stride_query / stride_tok
// tokens before it would run into the next query's, so the table must cover the largest shift of
// the layout plus that many positions.
bool decode_ids_in_table(const dbsa_layout* L, int64_t stride_query, int64_t stride_tok, int32_t rope_n_pos) {
  const int64_t t_max = std::max<int64_t>(1, stride_query / std::max<int64_t>(stride_tok, 1));
  return L->max_decode_shift + t_max - 1 < rope_n_pos;
}

// launch rows of the group-major decode for r query heads per KV head (32 % r == 0)
void fill_decode_rows(AttnParams& p, const dbsa_layout* L, int r) {
  int k = 0;
  while ((32 >> k) > 32 / r) ++k;  // a wave takes 32 / r queries
  p.gm_rows = L->dev.gm_rows + L->gm_rows_off[k];
  p.gm_n_rows = L->gm_rows_off[k + 1] - L->gm_rows_off[k];
  p.gm_pool_rows = L->gm_pool_rows[k];
}

// waves per decode workgroup for r query heads per KV head (32 % r == 0), see decode_common
int pick_decode_waves(const dbsa_layout* L, int r) {
  int k = 0;
  while ((32 >> k) > 32 / r) ++k;
  const float walks = L->gm_walks_per_key[k];
  if (r % 4 == 0 && walks >= 2.3f) return 4;
  if (r % 2 == 0 && walks >= 1.5f) return 2;
  return 1;
}

void fill_lists(AttnParams& p, const dbsa_layout* L) {
  p.qtile_tab = L->dev.qtile_tab;
  p.list_ptr = L->dev.list_ptr;
  p.list_ent = L->dev.list_ent;
  p.order = L->dev.order;
  p.dec_ent = L->dev.dec_ent;
  p.split_ptr = L->dev.split_ptr;
  p.gm_slot_ptr = L->dev.gm_slot_ptr;
  p.list_shift = L->dev.list_shift;
  p.dec_shift = L->dev.dec_shift;
  p.gm_item_run = L->dev.gm_item_run;
  p.gm_ref_pad = L->dev.gm_ref_pad;
  p.n_gm_items = static_cast<int32_t>(L->gm_items.size() / 4);
  p.gm_max_queries = L->gm_max_queries;
  p.n_pool_blocks = (p.n_gm_items + 7) / 8;
  p.n_qtiles = static_cast<int32_t>(L->n_qtiles());
  p.n_split = L->n_split;
  p.n_queries = L->n_queries;
  p.block_m = L->block_m;
  p.block_n = L->block_n;
}

int prefill_common(const dbsa_layout* L, bool want_query_stage, dbsa_tensor q, dbsa_tensor k_self, dbsa_tensor v_self,
                   dbsa_tensor k_pool, dbsa_tensor v_pool, dbsa_tensor o, float* lse, int32_t dtype, int32_t hq,
                   int32_t hkv, int32_t d, float scale, void* stream, const float* rope_table = nullptr,
                   int32_t rope_n_pos = 0, void* workspace = nullptr, size_t workspace_bytes = 0) {
  if (!L || !L->on_device || L->query_stage != want_query_stage) return DBSA_ERR_INVALID_ARG;
  if (int rc = check_shapes(dtype, hq, hkv, d, scale)) return rc;
  if (!tensor_ok(q, dtype) || !tensor_ok(k_pool, dtype) || !tensor_ok(v_pool, dtype) || !tensor_ok(o, dtype))
    return DBSA_ERR_INVALID_ARG;
  if (want_query_stage && (!tensor_ok(k_self, dtype) || !tensor_ok(v_self, dtype))) return DBSA_ERR_INVALID_ARG;
  AttnParams p{};
  fill_lists(p, L);
  p.q = view(q);
  p.o = view(o);
  p.k_pool = view(k_pool);
  p.v_pool = view(v_pool);
  p.k_self = want_query_stage ? view(k_self) : view(k_pool);
  p.v_self = want_query_stage ? view(v_self) : view(v_pool);
  p.query_stage = want_query_stage ? 1 : 0;
  p.lse = lse;
  p.lse_stride = want_query_stage ? L->n_query_tokens : L->n_tokens;
  p.n_q_heads = hq;
  p.n_kv_heads = hkv;
  p.scale = scale;
  p.scale_log2e = scale * 1.4426950408889634f;
  p.rope_table = rope_table;
  p.rope_n_pos = rope_n_pos;
  L->last_walk_reversed.store(0);  // prefill-shaped calls walk their lists front to back
  hipError_t e = order_behind_upload(L, static_cast<hipStream_t>(stream));
  if (e != hipSuccess) return DBSA_ERR_HIP;
  if (dtype == DBSA_BF16) {
    // the pipelined kernel addresses a tile's rows with 32-bit byte offsets
    const int64_t max_stride = std::max(std::max(p.k_pool.stride_tok, p.v_pool.stride_tok),
                                        std::max(p.k_self.stride_tok, p.v_self.stride_tok));
    // of the matrix kernels only the pipelined one re-positions: other shapes take the plain kernel then
    if (rope_table && !(d == 128 && max_stride < (int64_t{1} << 24))) {
      e = launch_prefill_plain(p, d, /*bf16_storage=*/true, static_cast<hipStream_t>(stream));
      return e == hipSuccess ? DBSA_OK : DBSA_ERR_HIP;
    }
    if (!mfma_tile_sizes_ok(L)) return DBSA_ERR_UNSUPPORTED;
    p.heads_per_block = pick_heads_per_block(hq / hkv, L->block_m);
    // A query prefill with fewer workgroups than the chip holds (two per compute unit) cuts every
    // list into runs of at least kMinRun tiles, up to kMaxQuerySplit of them, if the caller gave the workspace.
    p.n_rows = L->n_query_tokens;
    p.q_split = 1;
    if (want_query_stage && d == 128 && workspace && reinterpret_cast<uintptr_t>(workspace) % 16 == 0) {
      const int64_t wgs = L->n_qtiles() * (hq / p.heads_per_block);
      // eight-wave workgroups (112 KiB of LDS) sit alone on a compute unit, smaller ones in pairs
      const int64_t slots = workgroup_slots(L) / (p.heads_per_block * (L->block_m / 32) == 8 ? 2 : 1);
      int64_t split = wgs > 0 ? std::min<int64_t>(kMaxQuerySplit, (slots + wgs - 1) / wgs) : 1;
      split = std::min(split, L->shortest_list / kMinRun);
      const size_t need = static_cast<size_t>(L->n_query_tokens) * hq * static_cast<size_t>(std::max<int64_t>(split, 1)) *
                          (d + kPartialPad) * sizeof(float);
      if (wgs < slots && split > 1 && workspace_bytes >= need) {
        p.q_split = static_cast<int32_t>(split);
        p.partial = static_cast<float*>(workspace);
      }
    }
    // Launches with several Q tiles per workgroup place run persistently: as many workgroups as the
    // chip holds (one of four waves or two of two per compute unit), each walking a balanced share
    // of the Q tiles of its head block.
    const int row_blocks = p.heads_per_block * (L->block_m / 32);
    if (d == 128 && max_stride < (int64_t{1} << 24) && p.q_split == 1 && (row_blocks == 4 || row_blocks == 8)) {
      const int64_t head_blocks = hq / p.heads_per_block;
      const int64_t places = static_cast<int64_t>(L->compute_units) * (row_blocks == 8 ? 1 : 2);
      const int64_t classes = places / head_blocks;
      if (classes >= 1 && L->n_qtiles() >= 2 * classes && ensure_schedule(L, static_cast<int32_t>(classes), static_cast<hipStream_t>(stream))) {
        p.sched_rec = L->dev.sched_rec;
        p.sched_ptr = L->dev.sched_ptr;
        p.sched_classes = static_cast<int32_t>(classes);
        p.n_head_blocks = static_cast<int32_t>(head_blocks);
      }
    }
    e = (d == 128 && max_stride < (int64_t{1} << 24))
            ? launch_prefill_pipelined(p, static_cast<hipStream_t>(stream))
            : launch_prefill_mfma(p, d, static_cast<hipStream_t>(stream));
  } else {
    e = launch_prefill_plain(p, d, /*bf16_storage=*/false, static_cast<hipStream_t>(stream));
  }
  return e == hipSuccess ? DBSA_OK : DBSA_ERR_HIP;
}

int decode_common(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                  const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool, dbsa_tensor v_pool,
                  dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                  float softmax_scale, void* workspace, size_t workspace_bytes, void* stream,
                  const float* rope_table, int32_t rope_n_pos, size_t need_bytes = 0);

}  // namespace

extern "C" {

const char* dbsa_strerror(int code) {
  switch (code) {
    case DBSA_OK: return "ok";
    case DBSA_ERR_INVALID_ARG: return "invalid argument";
    case DBSA_ERR_BAD_BOUNDS: return "offsets are not strictly increasing or not anchored as documented";
    case DBSA_ERR_BAD_SELECTION: return "selected group out of range or listed twice";
    case DBSA_ERR_UNSUPPORTED: return "unsupported head_dim, head ratio, dtype or tile size";
    case DBSA_ERR_WORKSPACE: return "workspace missing or too small";
    case DBSA_ERR_HIP: return "HIP runtime error";
    default: return "unknown dbsa error code";
  }
}

namespace {
int build_layout(const dbsa_pool_desc* pool, const dbsa_select_desc* sel, int32_t first_group, int32_t block_m,
                 int32_t block_n, int32_t flags, void* stream, dbsa_layout** out) {
  if (!out || (flags & ~DBSA_LAYOUT_HOST_ONLY)) return DBSA_ERR_INVALID_ARG;
  dbsa_layout* L = new (std::nothrow) dbsa_layout();
  if (!L) return DBSA_ERR_INVALID_ARG;
  int rc = DBSA_OK;
  // the decode chunking and the split / persistent prefill launches are sized for the current device
  if (!(flags & DBSA_LAYOUT_HOST_ONLY)) L->compute_units = device_compute_units();
  try {
    rc = dbsa_build_host_lists(pool, sel, first_group, block_m, block_n, L);
  } catch (...) {
    rc = DBSA_ERR_INVALID_ARG;
  }
  if (rc != DBSA_OK) {
    delete L;
    return rc;
  }
  if (!(flags & DBSA_LAYOUT_HOST_ONLY)) {
    const hipError_t e = upload_lists(L, static_cast<hipStream_t>(stream));
    if (e != hipSuccess) {
      delete L;
      return DBSA_ERR_HIP;
    }
    L->on_device = true;
  }
  *out = L;
  return DBSA_OK;
}
}  // namespace

int dbsa_layout_build(const dbsa_pool_desc* pool, const dbsa_select_desc* sel, int32_t block_m, int32_t block_n,
                      int32_t flags, void* stream, dbsa_layout** out) {
  return build_layout(pool, sel, -1, block_m, block_n, flags, stream, out);
}

int dbsa_layout_build_append(const dbsa_pool_desc* pool, int32_t first_group, int32_t block_m, int32_t block_n,
                             int32_t flags, void* stream, dbsa_layout** out) {
  if (first_group < 0) return DBSA_ERR_INVALID_ARG;
  return build_layout(pool, nullptr, first_group, block_m, block_n, flags, stream, out);
}

int dbsa_layout_export(const dbsa_layout* L, const int32_t** qtile_tab, int64_t* n_qtiles, const int64_t** list_ptr,
                       const int32_t** list_ent, int64_t* n_ent) {
  if (!L) return DBSA_ERR_INVALID_ARG;
  if (qtile_tab) *qtile_tab = L->qtile_tab.data();
  if (n_qtiles) *n_qtiles = L->n_qtiles();
  if (list_ptr) *list_ptr = L->list_ptr.data();
  if (list_ent) *list_ent = L->list_ent.data();
  if (n_ent) *n_ent = L->n_ent();
  return DBSA_OK;
}

int dbsa_layout_export_positions(const dbsa_layout* L, const int32_t** list_shift, const int32_t** qref_shift,
                                 const int32_t** cache_len) {
  if (!L || !L->query_stage) return DBSA_ERR_INVALID_ARG;
  if (list_shift) *list_shift = L->list_shift.data();
  if (qref_shift) *qref_shift = L->gm_qshift.data();
  if (cache_len) *cache_len = L->cache_len.data();
  return DBSA_OK;
}

int dbsa_layout_export_decode(const dbsa_layout* L, const int64_t** dec_ptr, const int32_t** dec_ent,
                              int64_t* n_dec_ent, const int64_t** split_ptr, int32_t* n_split) {
  if (!L || !L->query_stage) return DBSA_ERR_INVALID_ARG;
  if (dec_ptr) *dec_ptr = L->dec_ptr.data();
  if (dec_ent) *dec_ent = L->dec_ent.data();
  if (n_dec_ent) *n_dec_ent = static_cast<int64_t>(L->dec_ent.size() / 2);
  if (split_ptr) *split_ptr = L->split_ptr.data();
  if (n_split) *n_split = L->n_split;
  return DBSA_OK;
}

int dbsa_layout_export_decode_groups(const dbsa_layout* L, const int64_t** seg_ptr, const int32_t** seg_ent,
                                     int64_t* n_seg_ent, const int32_t** items, int64_t* n_items,
                                     const int32_t** qrefs, int64_t* n_qrefs, const int64_t** slot_ptr,
                                     int32_t* chunk_tiles) {
  if (!L || !L->query_stage) return DBSA_ERR_INVALID_ARG;
  if (seg_ptr) *seg_ptr = L->gm_seg_ptr.data();
  if (seg_ent) *seg_ent = L->gm_seg_ent.data();
  if (n_seg_ent) *n_seg_ent = static_cast<int64_t>(L->gm_seg_ent.size() / 2);
  if (items) *items = L->gm_items.data();
  if (n_items) *n_items = static_cast<int64_t>(L->gm_items.size() / 4);
  if (qrefs) *qrefs = L->gm_qrefs.data();
  if (n_qrefs) *n_qrefs = static_cast<int64_t>(L->gm_qrefs.size() / 2);
  if (slot_ptr) *slot_ptr = L->gm_slot_ptr.data();
  if (chunk_tiles) *chunk_tiles = L->gm_chunk_tiles;
  return DBSA_OK;
}

int dbsa_layout_export_order(const dbsa_layout* L, const int32_t** order, int64_t* n_order) {
  if (!L) return DBSA_ERR_INVALID_ARG;
  if (order) *order = L->order.data();
  if (n_order) *n_order = static_cast<int64_t>(L->order.size());
  return DBSA_OK;
}

int dbsa_layout_export_schedule(const dbsa_layout* L, int32_t n_classes, const int32_t** class_ptr,
                                const int32_t** records) {
  if (!L || n_classes < 1 || n_classes > kMaxSchedClasses) return DBSA_ERR_INVALID_ARG;
  std::lock_guard<std::mutex> lock(L->sched_mutex);
  if (L->sched_classes != 0 && L->sched_classes != n_classes) return DBSA_ERR_INVALID_ARG;
  if (L->sched_classes == 0) {
    try {
      dbsa_balance_schedule(L, n_classes, &L->sched_ptr, &L->sched_rec);
    } catch (...) {
      return DBSA_ERR_INVALID_ARG;
    }
    L->sched_classes = n_classes;
  }
  if (class_ptr) *class_ptr = L->sched_ptr.data();
  if (records) *records = L->sched_rec.data();
  return DBSA_OK;
}

int dbsa_layout_export_matrix_plan(const dbsa_layout* L, const int32_t** plan_ptr, int32_t* n_workers,
                                   int32_t* nominal_workers, const int32_t** qrefs, int64_t* n_qrefs,
                                   const int64_t** slot_ptr) {
  if (!L || !L->query_stage) return DBSA_ERR_INVALID_ARG;
  if (plan_ptr) *plan_ptr = L->mx_plan_ptr.data();
  if (n_workers) *n_workers = L->mx_plan_ptr.empty() ? 0 : static_cast<int32_t>(L->mx_plan_ptr.size()) - 1;
  if (nominal_workers) *nominal_workers = L->mx_plan_workers;
  if (qrefs) *qrefs = L->mx_qrefs.data();
  if (n_qrefs) *n_qrefs = static_cast<int64_t>(L->mx_qrefs.size() / 2);
  if (slot_ptr) *slot_ptr = L->mx_slot_ptr.data();
  return DBSA_OK;
}

int dbsa_layout_export_matrix_records(const dbsa_layout* L, const int32_t** records, int64_t* n_records, float* row_fill) {
  if (!L || !L->query_stage) return DBSA_ERR_INVALID_ARG;
  if (records) *records = L->mx_rec.data();
  if (n_records) *n_records = static_cast<int64_t>(L->mx_rec.size() / 4);
  if (row_fill) *row_fill = L->mx_row_fill;
  return DBSA_OK;
}

int32_t dbsa_pooled_list_blocks(void) {
  std::lock_guard<std::mutex> lock(g_pool_mutex);
  return static_cast<int32_t>(g_pool_blocks.size());
}

void dbsa_layout_destroy(dbsa_layout* L) {
  if (!L) return;
  if (L->on_device) free_device_lists(L);
  delete L;
}

size_t dbsa_workspace_bytes(const dbsa_layout* L, int32_t n_q_heads, int32_t head_dim) {
  if (!L || !L->query_stage || n_q_heads <= 0 || head_dim <= 0) return 0;
  size_t slots = std::max<size_t>(static_cast<size_t>(L->n_queries) * L->n_split,
                                  std::max<size_t>(L->gm_slot_ptr.empty() ? 0 : static_cast<size_t>(L->gm_slot_ptr.back()),
                                                   L->mx_slot_ptr.empty() ? 0 : static_cast<size_t>(L->mx_slot_ptr.back())));
  // a split query prefill keeps up to kMaxQuerySplit partial states per row; it is only used when
  // the launch has fewer workgroups than the chip holds, which bounds the number of Q tiles
  if (L->n_qtiles() < workgroup_slots(L)) slots = std::max<size_t>(slots, static_cast<size_t>(L->n_query_tokens) * kMaxQuerySplit);
  return slots * n_q_heads * (head_dim + kPartialPad) * sizeof(float);
}

int dbsa_preencode_attn(const dbsa_layout* layout, dbsa_tensor q, dbsa_tensor k, dbsa_tensor v, dbsa_tensor o,
                        float* lse, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                        float softmax_scale, void* /*workspace*/, size_t /*workspace_bytes*/, void* stream) {
  return prefill_common(layout, false, q, k, v, k, v, o, lse, dtype, n_q_heads, n_kv_heads, head_dim, softmax_scale,
                        stream);
}

int dbsa_query_attn(const dbsa_layout* layout, dbsa_tensor q_self, dbsa_tensor k_self, dbsa_tensor v_self,
                    dbsa_tensor k_pool, dbsa_tensor v_pool, dbsa_tensor o, float* lse, int32_t dtype,
                    int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale, void* workspace,
                    size_t workspace_bytes, void* stream) {
  return prefill_common(layout, true, q_self, k_self, v_self, k_pool, v_pool, o, lse, dtype, n_q_heads, n_kv_heads,
                        head_dim, softmax_scale, stream, nullptr, 0, workspace, workspace_bytes);
}

int dbsa_decode_attn(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                     const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool, dbsa_tensor v_pool,
                     dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                     float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
  return decode_common(L, q_step, k_selfcache, v_selfcache, self_len, stride_query, k_pool, v_pool, o, dtype,
                       n_q_heads, n_kv_heads, head_dim, softmax_scale, workspace, workspace_bytes, stream, nullptr, 0);
}

int dbsa_decode_attn_static(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                            dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool,
                            dbsa_tensor v_pool, dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads,
                            int32_t head_dim, float softmax_scale, void* stream) {
  if (!L || !L->query_stage || n_q_heads <= 0 || head_dim <= 0) return DBSA_ERR_INVALID_ARG;
  // the partial states of this step must fit the fixed buffer
  const size_t need = decode_workspace_need(L, n_q_heads, head_dim);
  if (need > kStaticScratchBytes) return DBSA_ERR_WORKSPACE;
  void* ptr = nullptr;
  if (static_scratch(&ptr) != hipSuccess) return DBSA_ERR_HIP;
  return decode_common(L, q_step, k_selfcache, v_selfcache, self_len, stride_query, k_pool, v_pool, o, dtype,
                       n_q_heads, n_kv_heads, head_dim, softmax_scale, ptr, kStaticScratchBytes, stream, nullptr, 0,
                       std::max<size_t>(need, 1));
}

namespace {
int decode_kv8_common(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                      const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool8, dbsa_tensor v_pool8,
                      const float* k_scale, const float* v_scale, dbsa_tensor o, const float* rope_table,
                      int32_t rope_n_pos, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                      float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (!L || !L->on_device || !L->query_stage || !self_len || !k_scale || !v_scale) return DBSA_ERR_INVALID_ARG;
  if (int rc = check_shapes(DBSA_BF16, n_q_heads, n_kv_heads, head_dim, softmax_scale)) return rc;
  if (!tensor_ok(q_step, DBSA_BF16) || !tensor_ok(k_selfcache, DBSA_BF16) || !tensor_ok(v_selfcache, DBSA_BF16) ||
      !tensor_ok(o, DBSA_BF16))
    return DBSA_ERR_INVALID_ARG;
  for (const dbsa_tensor* t : {&k_pool8, &v_pool8})
    if (!t->ptr || reinterpret_cast<uintptr_t>(t->ptr) % 16 != 0 || t->stride_tok <= 0 || t->stride_head <= 0 ||
        t->stride_tok % 16 != 0 || t->stride_head % 16 != 0)
      return DBSA_ERR_INVALID_ARG;
  if (stride_query <= 0 || stride_query % 8 != 0) return DBSA_ERR_INVALID_ARG;
  const int r = n_q_heads / n_kv_heads;
  const int64_t max_stride = std::max(std::max(k_pool8.stride_tok, v_pool8.stride_tok),
                                      std::max(k_selfcache.stride_tok, v_selfcache.stride_tok));
  if (head_dim != 128 || L->block_n != 64 || r > 32 || 32 % r != 0 || max_stride >= (int64_t{1} << 24))
    return DBSA_ERR_UNSUPPORTED;
  const size_t need = dbsa_workspace_bytes(L, n_q_heads, head_dim);
  if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
    return DBSA_ERR_WORKSPACE;
  if (rope_table && !decode_ids_in_table(L, stride_query, k_selfcache.stride_tok, rope_n_pos)) return DBSA_ERR_INVALID_ARG;
  AttnParams p{};
  fill_lists(p, L);
  p.q = view(q_step);
  p.o = view(o);
  p.k_pool = view(k_pool8);
  p.v_pool = view(v_pool8);
  p.k_self = view(k_selfcache);
  p.v_self = view(v_selfcache);
  p.stride_query = stride_query;
  p.self_len = self_len;
  p.n_q_heads = n_q_heads;
  p.n_kv_heads = n_kv_heads;
  p.scale = softmax_scale;
  p.scale_log2e = softmax_scale * 1.4426950408889634f;
  p.k_scale8 = k_scale;
  p.v_scale8 = v_scale;
  p.rope_table = rope_table;
  p.rope_n_pos = rope_n_pos;
  p.partial = static_cast<float*>(workspace);
  p.decode_waves = pick_decode_waves(L, r);
  fill_decode_rows(p, L, r / p.decode_waves);
  if (order_behind_upload(L, static_cast<hipStream_t>(stream)) != hipSuccess) return DBSA_ERR_HIP;
  p.decode_reverse = next_walk_direction(L);  // nothing rejects the call from here on
  return launch_decode_group_kv8(p, static_cast<hipStream_t>(stream)) == hipSuccess ? DBSA_OK : DBSA_ERR_HIP;
}
}  // namespace

int dbsa_decode_attn_kv8(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                         const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool8, dbsa_tensor v_pool8,
                         const float* k_scale, const float* v_scale, dbsa_tensor o, int32_t n_q_heads,
                         int32_t n_kv_heads, int32_t head_dim, float softmax_scale, void* workspace,
                         size_t workspace_bytes, void* stream) {
  return decode_kv8_common(L, q_step, k_selfcache, v_selfcache, self_len, stride_query, k_pool8, v_pool8, k_scale,
                           v_scale, o, nullptr, 0, n_q_heads, n_kv_heads, head_dim, softmax_scale, workspace,
                           workspace_bytes, stream);
}

int dbsa_decode_attn_kv8_rope(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache,
                              dbsa_tensor v_selfcache, const int32_t* self_len, int64_t stride_query,
                              dbsa_tensor k_pool8, dbsa_tensor v_pool8, const float* k_scale, const float* v_scale,
                              dbsa_tensor o, const float* rope_table, int32_t rope_n_pos, int32_t n_q_heads,
                              int32_t n_kv_heads, int32_t head_dim, float softmax_scale, void* workspace,
                              size_t workspace_bytes, void* stream) {
  if (!rope_table || rope_n_pos < 1) return DBSA_ERR_INVALID_ARG;
  return decode_kv8_common(L, q_step, k_selfcache, v_selfcache, self_len, stride_query, k_pool8, v_pool8, k_scale,
                           v_scale, o, rope_table, rope_n_pos, n_q_heads, n_kv_heads, head_dim, softmax_scale,
                           workspace, workspace_bytes, stream);
}

int dbsa_rope_table(const double* inv_freq, int32_t head_dim, int32_t n_pos, float* table, void* stream) {
  if (!inv_freq || !table || n_pos < 1 || head_dim < 2 || head_dim > 128 || head_dim % 2 != 0)
    return DBSA_ERR_INVALID_ARG;
  return launch_rope_table(inv_freq, head_dim, n_pos, table, static_cast<hipStream_t>(stream)) == hipSuccess
             ? DBSA_OK
             : DBSA_ERR_HIP;
}

int dbsa_rope_apply(dbsa_tensor x, dbsa_tensor out, int32_t n_tokens, int32_t n_heads, int32_t head_dim, int32_t dtype,
                    const int32_t* positions, int32_t first_id, const float* table, int32_t n_pos, void* stream) {
  if (dtype != DBSA_BF16 && dtype != DBSA_F32) return DBSA_ERR_UNSUPPORTED;
  if (head_dim % 16 != 0 || head_dim < 16 || head_dim > 128) return DBSA_ERR_UNSUPPORTED;
  if (!x.ptr || !out.ptr || !table || n_tokens < 0 || n_heads < 1 || n_pos < 1 || x.stride_tok <= 0 ||
      x.stride_head <= 0 || out.stride_tok <= 0 || out.stride_head <= 0)
    return DBSA_ERR_INVALID_ARG;
  // ids the host can see must lie inside the table (ids read from `positions` are clamped by the kernel)
  if (!positions && (first_id < 0 || static_cast<int64_t>(first_id) + n_tokens > n_pos)) return DBSA_ERR_INVALID_ARG;
  return launch_rope_apply(view(x), view(out), n_tokens, n_heads, head_dim, dtype == DBSA_BF16, positions, first_id,
                           table, n_pos, static_cast<hipStream_t>(stream)) == hipSuccess
             ? DBSA_OK
             : DBSA_ERR_HIP;
}

int dbsa_query_attn_rope(const dbsa_layout* layout, dbsa_tensor q_self, dbsa_tensor k_self, dbsa_tensor v_self,
                         dbsa_tensor k_pool, dbsa_tensor v_pool, dbsa_tensor o, float* lse, const float* rope_table,
                         int32_t rope_n_pos, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                         float softmax_scale, void* workspace, size_t workspace_bytes, void* stream) {
  if (!rope_table || rope_n_pos < 1 || !layout || !layout->query_stage) return DBSA_ERR_INVALID_ARG;
  // the largest id any row will look up must be inside the table
  if (layout->max_rotation_id >= rope_n_pos) return DBSA_ERR_INVALID_ARG;
  return prefill_common(layout, true, q_self, k_self, v_self, k_pool, v_pool, o, lse, dtype, n_q_heads, n_kv_heads,
                        head_dim, softmax_scale, stream, rope_table, rope_n_pos, workspace, workspace_bytes);
}

int dbsa_decode_attn_rope(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                          const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool, dbsa_tensor v_pool,
                          dbsa_tensor o, const float* rope_table, int32_t rope_n_pos, int32_t dtype,
                          int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, float softmax_scale,
                          void* workspace, size_t workspace_bytes, void* stream) {
  if (!rope_table || rope_n_pos < 1) return DBSA_ERR_INVALID_ARG;
  return decode_common(L, q_step, k_selfcache, v_selfcache, self_len, stride_query, k_pool, v_pool, o, dtype,
                       n_q_heads, n_kv_heads, head_dim, softmax_scale, workspace, workspace_bytes, stream, rope_table,
                       rope_n_pos);
}

}  // extern "C"

namespace {
int decode_common(const dbsa_layout* L, dbsa_tensor q_step, dbsa_tensor k_selfcache, dbsa_tensor v_selfcache,
                  const int32_t* self_len, int64_t stride_query, dbsa_tensor k_pool, dbsa_tensor v_pool,
                  dbsa_tensor o, int32_t dtype, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim,
                  float softmax_scale, void* workspace, size_t workspace_bytes, void* stream,
                  const float* rope_table, int32_t rope_n_pos, size_t need_bytes) {
  if (!L || !L->on_device || !L->query_stage || !self_len) return DBSA_ERR_INVALID_ARG;
  if (int rc = check_shapes(dtype, n_q_heads, n_kv_heads, head_dim, softmax_scale)) return rc;
  if (!tensor_ok(q_step, dtype) || !tensor_ok(k_selfcache, dtype) || !tensor_ok(v_selfcache, dtype) ||
      !tensor_ok(k_pool, dtype) || !tensor_ok(v_pool, dtype) || !tensor_ok(o, dtype))
    return DBSA_ERR_INVALID_ARG;
  const int64_t align_elems = dtype == DBSA_BF16 ? 8 : 4;
  if (stride_query <= 0 || stride_query % align_elems != 0) return DBSA_ERR_INVALID_ARG;
  AttnParams p{};
  fill_lists(p, L);
  p.q = view(q_step);
  p.o = view(o);
  p.k_pool = view(k_pool);
  p.v_pool = view(v_pool);
  p.k_self = view(k_selfcache);
  p.v_self = view(v_selfcache);
  p.stride_query = stride_query;
  p.self_len = self_len;
  p.n_q_heads = n_q_heads;
  p.n_kv_heads = n_kv_heads;
  p.scale = softmax_scale;
  p.scale_log2e = softmax_scale * 1.4426950408889634f;
  p.rope_table = rope_table;
  p.rope_n_pos = rope_n_pos;
  hipStream_t s = static_cast<hipStream_t>(stream);
  // every reason to reject the call comes first
  const int r = n_q_heads / n_kv_heads;
  const int64_t max_stride = std::max(std::max(p.k_pool.stride_tok, p.v_pool.stride_tok),
                                      std::max(p.k_self.stride_tok, p.v_self.stride_tok));
  const bool group_major = dtype == DBSA_BF16 && head_dim == 128 && 32 % r == 0 && max_stride < (int64_t{1} << 24);
  if (dtype == DBSA_BF16) {
    if (L->block_n != 64 || r > 32) return DBSA_ERR_UNSUPPORTED;
    // need_bytes: what the caller has checked the step to write (the fixed-buffer entry point)
    const size_t need = need_bytes ? need_bytes : dbsa_workspace_bytes(L, n_q_heads, head_dim);
    if (!workspace || workspace_bytes < need || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)
      return DBSA_ERR_WORKSPACE;
    p.partial = static_cast<float*>(workspace);
  }
  if (rope_table && !decode_ids_in_table(L, stride_query, k_selfcache.stride_tok, rope_n_pos)) return DBSA_ERR_INVALID_ARG;
  hipError_t e = order_behind_upload(L, s);
  if (e != hipSuccess) return DBSA_ERR_HIP;
  p.decode_reverse = next_walk_direction(L);
  if (dtype == DBSA_BF16) {
    if (group_major) {
      // every KV run is walked once for all the queries that selected it
      // Items that serve several batches of 32 / r queries: the batches of one item run as waves
      // of ONE workgroup that share its tiles in LDS, once a key is walked often enough for that
      // to outweigh the barrier per half tile (measured over 16-256 queries at 10-100 % retrieval: 2
      // waves pay from ~1.5 walks per key on, 4 from ~2.3).
      p.decode_waves = pick_decode_waves(L, r);
      // With query heads in fours per KV head and groups that serve many queries, the pool items run
      // as a contraction: 64 queries per wave, four heads of a KV head as the four waves of a
      // workgroup, one workgroup per compute unit walking a balanced share of the records
      // (kernels.hpp: launch_decode_matrix_items).  Worth it once enough of the 64 rows carry a query.
      if (r % 4 == 0 && L->mx_row_fill >= kMatrixRowFill) {
        // one workgroup per compute unit, or per record where there are fewer
        const int32_t head_blocks = n_q_heads / 4;
        const bool planned = !L->mx_plan_ptr.empty() && L->compute_units / head_blocks == L->mx_plan_workers;
        const int32_t classes =
            planned ? static_cast<int32_t>(L->mx_plan_ptr.size()) - 1
                    : static_cast<int32_t>(std::min<int64_t>(L->compute_units / head_blocks,
                                                             static_cast<int64_t>(L->mx_rec.size() / 4)));
        if (classes >= 1 && ensure_matrix_schedule(L, classes, planned, s)) {
          p.decode_matrix = 1;
          p.decode_waves = 1;
          p.mx_sched_rec = L->dev.mx_sched_rec;
          p.mx_sched_ptr = L->dev.mx_sched_ptr;
          p.mx_ent = L->dev.gm_seg_ent;
          p.mx_classes = classes;
          // a layout with a plan has references and slots of its own for these records: the own-cache items
          // and the merge then go by its slot table too
          const bool own = !L->mx_plan_ptr.empty();
          p.gather_refs = own ? L->dev.mx_qrefs : L->dev.gm_qrefs;
          p.gather_shift = own ? L->dev.mx_qshift : L->dev.gm_qshift;
          if (own) p.gm_slot_ptr = L->dev.mx_slot_ptr;
        }
      }
      fill_decode_rows(p, L, r / p.decode_waves);
      e = launch_decode_group(p, s);
    } else if (rope_table) {
      // of the matrix kernels only the group-major one re-positions
      e = launch_decode_plain(p, head_dim, /*bf16_storage=*/true, s);
    } else {
      e = launch_decode_mfma(p, head_dim, s);
      if (e == hipSuccess) e = launch_decode_merge(p, head_dim, /*out_bf16=*/true, s);
    }
  } else {
    e = launch_decode_plain(p, head_dim, /*bf16_storage=*/false, s);
  }
  return e == hipSuccess ? DBSA_OK : DBSA_ERR_HIP;
}
}  // namespace
