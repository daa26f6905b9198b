// C ABI of the PIPE library: argument checks, expansion object life cycle, tile schedule,
// workspace and the launch sequences of the forward calls.  All arithmetic of the method
// runs in the kernels of the other files; the host only validates, sizes and schedules.
#include <algorithm>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <map>
#include <mutex>
#include <new>
#include <string>
#include <utility>

#include "pipe_internal.h"

// ------------------------------------------------------------------ errors
static thread_local std::string g_last_hip_error;

void pipe_note_hip_error(hipError_t e, const char* what) {
  g_last_hip_error = std::string(hipGetErrorString(e)) + " in " + what;
}

extern "C" const char* pipe_last_device_error(void) { return g_last_hip_error.c_str(); }

extern "C" const char* pipe_strerror(int code) {
  switch (code) {
    case PIPE_OK: return "ok";
    case PIPE_EINVAL: return "invalid argument (NULL pointer or bits/K/gamma/group out of range)";
    case PIPE_ESHAPE: return "invalid shape (out % group != 0, group % 16 != 0, size <= 0 or too large)";
    case PIPE_ENOMEM: return "out of memory";
    case PIPE_EDEVICE: return "HIP call failed";
    case PIPE_ESPLIT: return "ensemble split must be positive and sum to K";
    case PIPE_ELIMIT: return "input larger than the fixed scratch of pipe_forward_noalloc (tokens <= 8192, padded tokens x padded in_features <= 8 MiB)";
    case PIPE_ENOTREADY: return "the call would have to allocate or synchronize while its stream is being captured: run pipe_prepare first";
    default: return "unknown error";
  }
}

// ------------------------------------------------------------------ workspace
// One set of scratch blocks per (device, stream).  An entry point opens a CallScope on its
// stream; pipe_ws_get then serves that stream's set.  Blocks only grow, and a block that was
// handed out is never freed (a graph captured earlier may still hold its address): it is
// retired until the process ends.  Growth at least doubles a block, so retired blocks sum to
// less than the live one.
struct WsSet {
  PipeWorkspace slot[WS_SLOTS];
  bool amax_h_dirty = false;   // the members' max|h| slots hold a value no kernel will clear
  bool range_h_dirty = false;  // the same for the members' range slots of the asymmetric chain
};
static std::mutex g_ws_mu;
static std::map<std::pair<int, hipStream_t>, WsSet*> g_ws_sets;
static std::vector<void*> g_ws_retired;
static thread_local WsSet* t_ws = nullptr;
static thread_local bool t_capturing = false;
static thread_local bool t_dry = false;
static thread_local bool t_no_alloc = false;   // inside the entry point that allocates nothing
static thread_local int t_ws_err = PIPE_ENOMEM;

bool pipe_dry_run() { return t_dry; }
bool pipe_capturing() { return t_capturing || t_no_alloc; }
int pipe_ws_error() { return t_ws_err; }

static WsSet* ws_set_of(hipStream_t st) {
  int dev = 0;
  (void)hipGetDevice(&dev);
  std::lock_guard<std::mutex> lk(g_ws_mu);
  WsSet*& w = g_ws_sets[std::make_pair(dev, st)];
  if (w == nullptr) w = new WsSet();
  return w;
}

namespace {
struct CallScope {
  WsSet* prev_ws;
  bool prev_cap;
  explicit CallScope(void* stream) : prev_ws(t_ws), prev_cap(t_capturing) {
    hipStream_t st = (hipStream_t)stream;
    t_ws = ws_set_of(st);
    hipStreamCaptureStatus cs = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(st, &cs) != hipSuccess) {
      (void)hipGetLastError();   // e.g. the legacy null stream while another stream captures
      cs = hipStreamCaptureStatusNone;
    }
    t_capturing = cs != hipStreamCaptureStatusNone;
  }
  ~CallScope() { t_ws = prev_ws; t_capturing = prev_cap; }
};
struct DryScope {
  bool prev;
  DryScope() : prev(t_dry) { t_dry = true; }
  ~DryScope() { t_dry = prev; }
};
}  // namespace

void* pipe_ws_get(int slot, size_t bytes) {
  if (t_ws == nullptr) t_ws = ws_set_of(nullptr);   // calls outside a scope (diagnostics): the null stream's set
  PipeWorkspace& w = t_ws->slot[slot];
  if (bytes == 0) bytes = 256;
  if (w.bytes >= bytes) return w.ptr;
  if (t_capturing) {
    t_ws_err = PIPE_ENOTREADY;
    return nullptr;
  }
  const size_t want = (size_t)round_up64((int64_t)std::max(bytes, 2 * w.bytes), 1 << 20);
  void* fresh = nullptr;
  hipError_t e = hipMalloc(&fresh, want);
  if (e != hipSuccess) {
    pipe_note_hip_error(e, "hipMalloc(workspace)");
    t_ws_err = PIPE_ENOMEM;
    return nullptr;
  }
  if (w.ptr) {
    std::lock_guard<std::mutex> lk(g_ws_mu);
    g_ws_retired.push_back(w.ptr);
  }
  w.ptr = fresh;
  w.bytes = want;
  return w.ptr;
}

static int g_kernel_choice = 0;
float g_act_qmax_host = 127.f;
extern "C" int pipe_set_kernel(int which) {
  if (which < 0 || which > 2) return PIPE_EINVAL;
  g_kernel_choice = which;
  return PIPE_OK;
}

extern "C" int pipe_set_token_tile(int tokens) {
  if (tokens != 0 && tokens != 16 && tokens != 32 && tokens != 64) return PIPE_EINVAL;
  g_tiled_mtb = tokens / 16;
  return PIPE_OK;
}

extern "C" int pipe_set_activation_bits(int bits) {
  if (bits < 2 || bits > 8) return PIPE_EINVAL;
  g_act_qmax_host = (float)((1 << (bits - 1)) - 1);
  return set_act_qmax(g_act_qmax_host);
}

int g_decode_fusion = 1;

extern "C" int pipe_set_decode_fusion(int on) {
  if (on != 0 && on != 1) return PIPE_EINVAL;
  g_decode_fusion = on;
  return PIPE_OK;
}

extern "C" int pipe_set_decode_resident(int on) {
  if (on < 0 || on > 2) return PIPE_EINVAL;
  g_decode_resident = on;
  return PIPE_OK;
}

extern "C" int pipe_resident_trace(unsigned long long* trace_dev) {
  g_resident_trace = trace_dev;
  return PIPE_OK;
}

extern "C" int pipe_set_resident_spin_limit(int polls) {
  if (polls < 0) return PIPE_EINVAL;
  g_resident_spin_limit = polls == 0 ? (1 << 19) : polls;
  return PIPE_OK;
}

extern "C" int pipe_set_stream_split(int workgroups_per_bin) {
  if (workgroups_per_bin < 0 || workgroups_per_bin > PIPE_MAX_SPLIT) return PIPE_EINVAL;
  g_stream_ksplit = workgroups_per_bin;
  return PIPE_OK;
}

// ------------------------------------------------------------------ helpers
static long long n_keep_of64(float gamma, long long n) {
  const double v = (double)gamma * (double)n * (1.0 - 1e-6);
  long long k = (long long)std::ceil(v);
  if (k < 1) k = 1;
  if (k > n) k = n;
  return k;
}
static int n_keep_of(float gamma, int n_groups) { return (int)n_keep_of64(gamma, n_groups); }

static int parse_split(int K, const int* split, int M, int* lo, int* hi, int* M_out) {
  if (split == nullptr) {
    lo[0] = 0;
    hi[0] = K - 1;
    *M_out = 1;
    return PIPE_OK;
  }
  if (M < 1 || M > K) return PIPE_ESPLIT;
  int pos = 0;
  for (int m = 0; m < M; ++m) {
    if (split[m] < 1) return PIPE_ESPLIT;
    lo[m] = pos;
    pos += split[m];
    hi[m] = pos - 1;
    if (pos > K) return PIPE_ESPLIT;
  }
  if (pos != K) return PIPE_ESPLIT;
  *M_out = M;
  return PIPE_OK;
}

static void free_expansion(pipe_expansion* e) {
  if (!e) return;
  for (auto& o : e->orders) {
    if (o.gids_dev) (void)hipFree(o.gids_dev);
    if (o.scales_dev) (void)hipFree(o.scales_dev);
    if (o.packed_dev) (void)hipFree(o.packed_dev);
    if (o.pos_dev) (void)hipFree(o.pos_dev);
  }
  for (auto& t : e->tables) {
    if (t.rb_out_dev) (void)hipFree(t.rb_out_dev);
    if (t.src_dev) (void)hipFree(t.src_dev);
    if (t.cnt_dev) (void)hipFree(t.cnt_dev);
  }
  for (auto& rt : e->res_tables) {
    if (rt.subs_dev) (void)hipFree(rt.subs_dev);
    if (rt.epi_dev) (void)hipFree(rt.epi_dev);
  }
  if (e->conv_zero_dev) (void)hipFree(e->conv_zero_dev);
  if (e->dw_codes_dev) (void)hipFree(e->dw_codes_dev);
  if (e->dw_scales_dev) (void)hipFree(e->dw_scales_dev);
  if (e->bins_dev) (void)hipFree(e->bins_dev);
  if (e->codes_dev) (void)hipFree(e->codes_dev);
  if (e->scales_all_dev) (void)hipFree(e->scales_all_dev);
  if (e->split_sum_dev) (void)hipFree(e->split_sum_dev);
  if (e->split_cnt_dev) (void)hipFree(e->split_cnt_dev);
  if (e->asym_wsum_dev) (void)hipFree(e->asym_wsum_dev);
  if (e->asym_C_dev) (void)hipFree(e->asym_C_dev);
  if (e->asym_bias_dev) (void)hipFree(e->asym_bias_dev);
  if (e->asym_P_dev) (void)hipFree(e->asym_P_dev);
  delete e;
}

// Sort row blocks by the set of orders that hold them (most orders first) and pack them into the
// bins of the weight-streaming kernel; a stored row block's bin and place fix its position.
static int build_schedule(pipe_expansion* e, hipStream_t st) {
  const int K = e->K, n_rb = e->n_rb, rbpg = e->rbpg;
  std::vector<std::vector<int32_t>> slot_of(K, std::vector<int32_t>(e->n_groups, -1));
  for (int k = 0; k < K; ++k)
    for (int s = 0; s < (int)e->orders[k].gids.size(); ++s) slot_of[k][e->orders[k].gids[s]] = s;
  struct Item { uint32_t mask; int pop; int rb; };
  std::vector<Item> items(n_rb);
  for (int rb = 0; rb < n_rb; ++rb) {
    const int g = rb / rbpg;
    uint32_t mask = 0;
    for (int k = 0; k < K; ++k)
      if (slot_of[k][g] >= 0) mask |= 1u << k;
    items[rb] = Item{mask, __builtin_popcount(mask), rb};
  }
  std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) {
    if (a.pop != b.pop) return a.pop > b.pop;
    if (a.mask != b.mask) return a.mask < b.mask;
    return a.rb < b.rb;
  });
  // Bins of the weight-streaming kernel: output row blocks, most orders first, packed best-fit
  // into bins of `cap` stored row blocks (the bin with the least room that still takes the block).
  const int cap = std::min(STREAM_BIN_CAP, (std::max(4, K) + 3) / 4 * 4);   // 4, 8, 12 or 16: the kernel streams 4 items at a time
  struct BinRbs { std::vector<int> rbs; int n_items = 0; };
  std::vector<BinRbs> packed;
  std::vector<std::vector<int>> with_room(cap + 1);   // open bins by the room they have left (most recent last)
  for (int i = 0; i < n_rb; ++i) {
    const int pop = items[i].pop;
    int which = -1;
    for (int r = pop; r <= cap && which < 0; ++r)
      if (!with_room[r].empty()) { which = with_room[r].back(); with_room[r].pop_back(); }
    if (which < 0) {
      packed.push_back(BinRbs{});
      which = (int)packed.size() - 1;
    }
    packed[which].rbs.push_back(items[i].rb);
    packed[which].n_items += pop;
    if (cap - packed[which].n_items > 0) with_room[cap - packed[which].n_items].push_back(which);
  }
  // Positions in the schedule-ordered buffers.  Bins of 4: fullest bins first and the stored row blocks
  // packed without gaps, so a bin's first position and item count follow from its index and the number of
  // bins with 4, 3 and 2 items (bin_thr): the kernel still addresses its codes from its block index alone,
  // and the items a bin does not have are read from one all-zero position behind the last (zero_pos), which
  // stays in cache, instead of from zeros of the bin's own in memory.  Wider bins (more than 4 orders):
  // position = bin * cap + index, unused positions are zeros.
  if (cap == 4)
    std::stable_sort(packed.begin(), packed.end(), [](const BinRbs& a, const BinRbs& b) { return a.n_items > b.n_items; });
  std::vector<StreamBin> bins(packed.size());
  for (int k = 0; k < K; ++k) e->orders[k].pos.assign((size_t)e->orders[k].n_kept * rbpg, -1);
  e->bin_thr[0] = e->bin_thr[1] = e->bin_thr[2] = 0;
  int next_pos = 0;
  for (size_t bi = 0; bi < packed.size(); ++bi) {
    StreamBin& bn = bins[bi];
    std::memset(&bn, 0, sizeof(bn));
    const int first = cap == 4 ? next_pos : (int)bi * cap;
    for (int rb : packed[bi].rbs) {
      const int g = rb / rbpg, b = rb % rbpg;
      const int slot = bn.n_out++;
      bn.out_rb[slot] = rb;
      for (int k = 0; k < K; ++k) {
        if (slot_of[k][g] < 0) continue;
        const int it = bn.n_items++;
        bn.k[it] = k;
        bn.slot[it] = slot;
        e->orders[k].pos[(size_t)slot_of[k][g] * rbpg + b] = first + it;
      }
    }
    next_pos = first + (cap == 4 ? bn.n_items : cap);
    if (cap == 4)
      for (int n = 4; n >= 2; --n)
        if (bn.n_items >= n) e->bin_thr[4 - n] = (int)bi + 1;   // bins 0 .. bin_thr[4-n]-1 hold at least n items
  }
  e->n_bins = (int)bins.size();
  e->bin_cap = cap;
  e->n_pos = next_pos;
  e->zero_pos = next_pos;
  PIPE_HIP(hipMalloc(&e->bins_dev, bins.size() * sizeof(StreamBin)));
  PIPE_HIP(hipMemcpy(e->bins_dev, bins.data(), bins.size() * sizeof(StreamBin), hipMemcpyHostToDevice));

  // where each output row block's stored orders sit: what the tiled kernel's schedules are built from
  e->pos_of.assign((size_t)K * n_rb, -1);
  for (int rb = 0; rb < n_rb; ++rb) {
    const int g = rb / rbpg, b = rb % rbpg;
    for (int k = 0; k < K; ++k)
      if (slot_of[k][g] >= 0) e->pos_of[(size_t)k * n_rb + rb] = e->orders[k].pos[(size_t)slot_of[k][g] * rbpg + b];
  }

  // Move the stored row blocks to their positions and drop the per-order buffers.
  const int64_t rb_bytes = (int64_t)(e->in_pad / (512 / e->bits)) * 1024;
  const size_t n_pos = (size_t)e->n_pos + 1;   // and the all-zero position
  PIPE_HIP(hipMalloc(&e->codes_dev, n_pos * (size_t)rb_bytes));
  PIPE_HIP(hipMalloc(&e->scales_all_dev, n_pos * 16 * sizeof(float)));
  PIPE_HIP(hipMemsetAsync(e->codes_dev, 0, n_pos * (size_t)rb_bytes, st));
  PIPE_HIP(hipMemsetAsync(e->scales_all_dev, 0, n_pos * 16 * sizeof(float), st));
  PIPE_HIP(hipMalloc(&e->split_sum_dev, (size_t)e->n_bins * cap * PIPE_MAX_SPLIT * 256 * sizeof(int32_t)));
  PIPE_HIP(hipMalloc(&e->split_cnt_dev, (size_t)e->n_bins * sizeof(uint32_t)));
  PIPE_HIP(hipMemsetAsync(e->split_cnt_dev, 0, (size_t)e->n_bins * sizeof(uint32_t), st));
  for (int k = 0; k < K; ++k) {
    PipeOrder& o = e->orders[k];
    PIPE_HIP(hipMalloc(&o.pos_dev, o.pos.size() * sizeof(int32_t)));
    PIPE_HIP(hipMemcpyAsync(o.pos_dev, o.pos.data(), o.pos.size() * sizeof(int32_t), hipMemcpyHostToDevice, st));
    int rc = launch_gather_row_blocks(o.packed_dev, o.scales_dev, o.pos_dev, (int)o.pos.size(), rb_bytes, e->codes_dev,
                                      e->scales_all_dev, st);
    if (rc) return rc;
  }
  PIPE_HIP(hipStreamSynchronize(st));
  for (int k = 0; k < K; ++k) {
    PipeOrder& o = e->orders[k];
    (void)hipFree(o.packed_dev); o.packed_dev = nullptr;
    (void)hipFree(o.scales_dev); o.scales_dev = nullptr;
  }
  return PIPE_OK;
}

struct RoundingHook {
  pipe_rounding_fn fn = nullptr;
  void* user = nullptr;
  float* rows = nullptr;     // caller's scratch, DEVICE
  float* scales = nullptr;
  int8_t* codes = nullptr;
};

static int expand_impl(pipe_expansion* e, const float* W_dev, hipStream_t st, float** resid_out,
                       double** energy_out, const RoundingHook& hook) {
  const int out = e->out, in = e->in, K = e->K, group = e->group;
  const int n_groups = e->n_groups;
  const int keep = e->unstructured ? n_groups : n_keep_of(e->gamma, n_groups);
  const long long n_entries = (long long)out * in, keep_entries = n_keep_of64(e->gamma, n_entries);
  float* E = nullptr;
  PIPE_HIP(hipMalloc(&E, (size_t)out * in * sizeof(float)));
  *resid_out = E;
  PIPE_HIP(hipMemcpyAsync(E, W_dev, (size_t)out * in * sizeof(float), hipMemcpyDeviceToDevice, st));
  double* energy = nullptr;
  // scratch: row energies, group scores and flags of the group selection; or the histogram of the entry selection
  PIPE_HIP(hipMalloc(&energy, std::max(((size_t)out + n_groups) * sizeof(double) + (size_t)n_groups * sizeof(int32_t),
                                       (size_t)2049 * sizeof(uint32_t))));
  *energy_out = energy;
  const int ksup = 512 / e->bits;
  e->orders.resize(K);
  std::vector<int32_t> iota(n_groups);
  for (int g = 0; g < n_groups; ++g) iota[g] = g;
  for (int k = 0; k < K; ++k) {
    PipeOrder& o = e->orders[k];
    const bool dense = (k == 0) || keep == n_groups;
    o.n_kept = dense ? n_groups : keep;
    const size_t rows = (size_t)o.n_kept * group;
    o.packed_bytes = (rows / 16) * (size_t)(e->in_pad / ksup) * 1024;
    PIPE_HIP(hipMalloc(&o.gids_dev, (size_t)o.n_kept * sizeof(int32_t)));
    PIPE_HIP(hipMalloc(&o.scales_dev, rows * sizeof(float)));
    PIPE_HIP(hipMalloc(&o.packed_dev, o.packed_bytes));
    if (dense) {
      PIPE_HIP(hipMemcpyAsync(o.gids_dev, iota.data(), (size_t)n_groups * sizeof(int32_t), hipMemcpyHostToDevice, st));
    } else {
      int rc = launch_row_energy(E, out, in, energy, st);
      if (rc) return rc;
      rc = launch_group_select(energy, n_groups, group, keep, o.gids_dev, st);
      if (rc) return rc;
    }
    int rc = PIPE_OK;
    uint32_t thr_key = PIPE_NO_MASK_KEY;
    long long tie_cut = PIPE_NO_MASK_CUT;
    if (e->unstructured && k > 0 && keep_entries < n_entries) {
      rc = select_entry_threshold(E, n_entries, keep_entries, reinterpret_cast<uint32_t*>(energy), &thr_key, &tie_cut, st);
      if (rc) return rc;
    }
    if (hook.fn) {
      // another rounding operator: hand it the rows of this order and their scales, take its codes
      rc = launch_gather_rows(E, in, e->qbits, group, o.gids_dev, o.n_kept, hook.rows, hook.scales, st);
      if (rc) return rc;
      if (hook.fn(hook.user, k + 1, (int)rows, in, (1 << (e->qbits - 1)) - 1, (void*)st) != 0) return PIPE_EINVAL;
    }
    rc = launch_quantize_rows(E, out, in, e->in_pad, e->bits, e->qbits, group, o.gids_dev, o.n_kept, o.scales_dev,
                              o.packed_dev, hook.fn ? hook.codes : nullptr, thr_key, tie_cut, st);
    if (rc) return rc;
    e->stream_bytes += (int64_t)o.packed_bytes + (int64_t)rows * 4 + (int64_t)o.n_kept * 4;
  }
  PIPE_HIP(hipStreamSynchronize(st));
  for (int k = 0; k < K; ++k) {
    PipeOrder& o = e->orders[k];
    o.gids.resize(o.n_kept);
    PIPE_HIP(hipMemcpy(o.gids.data(), o.gids_dev, (size_t)o.n_kept * sizeof(int32_t), hipMemcpyDeviceToHost));
  }
  return build_schedule(e, st);
}

extern "C" int pipe_fold_batchnorm(const float* W_dev, const float* bias_dev, const float* gamma_dev,
                                   const float* beta_dev, const float* mean_dev, const float* var_dev, float eps,
                                   int out, int in, float* W_out_dev, float* bias_out_dev, void* stream) {
  if (!W_dev || !gamma_dev || !beta_dev || !mean_dev || !var_dev || !W_out_dev || !(eps >= 0.f)) return PIPE_EINVAL;
  if (out < 1 || in < 1) return PIPE_ESHAPE;
  return launch_fold_batchnorm(W_dev, bias_dev, gamma_dev, beta_dev, mean_dev, var_dev, eps, out, in, W_out_dev,
                               bias_out_dev, (hipStream_t)stream);
}

static int expand_checked(const float* W_dev, int out, int in, int bits, int K, float gamma, int group,
                          const RoundingHook& hook, bool unstructured, void* stream, pipe_expansion** exp_out) {
  if (W_dev == nullptr || exp_out == nullptr) return PIPE_EINVAL;
  if (bits < 2 || bits > 8) return PIPE_EINVAL;
  if (K < 1 || K > PIPE_MAX_K) return PIPE_EINVAL;
  if (!(gamma > 0.f) || !(gamma <= 1.f)) return PIPE_EINVAL;
  if (out <= 0 || in <= 0 || group <= 0) return PIPE_ESHAPE;
  if (out % group != 0 || group % 16 != 0) return PIPE_ESHAPE;
  // int32 accumulator of offset-binary codes: 127 * 15 * in_pad and 127 * 127 * in must fit
  if ((int64_t)in > (int64_t)130000) return PIPE_ESHAPE;
  pipe_expansion* e = new (std::nothrow) pipe_expansion();
  if (!e) return PIPE_ENOMEM;
  e->out = out; e->in = in; e->qbits = bits; e->bits = bits == 2 ? 2 : (bits <= 4 ? 4 : 8); e->K = K; e->group = group; e->gamma = gamma; e->unstructured = unstructured;
  e->n_groups = out / group;
  e->rbpg = group / 16;
  e->n_rb = out / 16;
  e->in_pad = (int)round_up64(in, IN_PAD);
  e->nks = e->in_pad / 64;
  if (hipGetDevice(&e->device) != hipSuccess) { delete e; return PIPE_EDEVICE; }
  float* resid = nullptr;
  double* energy = nullptr;
  int rc = expand_impl(e, W_dev, (hipStream_t)stream, &resid, &energy, hook);
  if (rc != PIPE_OK) (void)hipDeviceSynchronize();
  if (resid) (void)hipFree(resid);
  if (energy) (void)hipFree(energy);
  if (rc != PIPE_OK) {
    if (rc == PIPE_EDEVICE && g_last_hip_error.find("out of memory") != std::string::npos) rc = PIPE_ENOMEM;
    free_expansion(e);
    return rc;
  }
  *exp_out = e;
  return PIPE_OK;
}

extern "C" int pipe_expand(const float* W_dev, int out, int in, int bits, int K, float gamma,
                           int group, void* stream, pipe_expansion** exp_out) {
  return expand_checked(W_dev, out, in, bits, K, gamma, group, RoundingHook{}, false, stream, exp_out);
}

extern "C" int pipe_expand_unstructured(const float* W_dev, int out, int in, int bits, int K, float gamma,
                                        int group, void* stream, pipe_expansion** exp_out) {
  return expand_checked(W_dev, out, in, bits, K, gamma, group, RoundingHook{}, true, stream, exp_out);
}

extern "C" int pipe_expand_with_operator(const float* W_dev, int out, int in, int bits, int K, float gamma, int group,
                                         pipe_rounding_fn fn, void* user, float* rows_dev, float* scales_dev,
                                         int8_t* codes_dev, void* stream, pipe_expansion** exp_out) {
  if (!fn || !rows_dev || !scales_dev || !codes_dev) return PIPE_EINVAL;
  RoundingHook hook;
  hook.fn = fn; hook.user = user; hook.rows = rows_dev; hook.scales = scales_dev; hook.codes = codes_dev;
  return expand_checked(W_dev, out, in, bits, K, gamma, group, hook, false, stream, exp_out);
}

extern "C" int pipe_expand_conv2d(const float* W_dev, int out, int C, int kh, int kw, int bits, int K, float gamma,
                                  int group, void* stream, pipe_expansion** exp_out) {
  if (W_dev == nullptr || exp_out == nullptr) return PIPE_EINVAL;
  if (out <= 0 || C <= 0 || kh <= 0 || kw <= 0 || C % 64 != 0 || (int64_t)C * kh * kw > 130000) return PIPE_ESHAPE;
  hipStream_t st = (hipStream_t)stream;
  const int in = C * kh * kw;
  float* Wp = nullptr;
  PIPE_HIP(hipMalloc(&Wp, (size_t)out * in * sizeof(float)));
  int rc = launch_permute_conv_weight(W_dev, out, C, kh * kw, Wp, st);
  pipe_expansion* e = nullptr;
  if (rc == PIPE_OK) rc = expand_checked(Wp, out, in, bits, K, gamma, group, RoundingHook{}, false, stream, &e);   // synchronizes
  (void)hipFree(Wp);
  if (rc != PIPE_OK) return rc;
  e->conv_C = C; e->conv_kh = kh; e->conv_kw = kw;
  if (hipMalloc(&e->conv_zero_dev, 256) != hipSuccess || hipMemset(e->conv_zero_dev, 0, 256) != hipSuccess) {
    free_expansion(e);
    return PIPE_ENOMEM;
  }
  *exp_out = e;
  return PIPE_OK;
}

extern "C" int pipe_expansion_free(pipe_expansion* e) {
  if (!e) return PIPE_OK;
  (void)hipDeviceSynchronize();
  free_expansion(e);
  return PIPE_OK;
}

extern "C" int pipe_expansion_info(const pipe_expansion* e, int* out, int* in, int* bits, int* K,
                                   int* group, float* gamma, int64_t* packed_bytes) {
  if (!e) return PIPE_EINVAL;
  if (out) *out = e->out;
  if (in) *in = e->in;
  if (bits) *bits = e->qbits;
  if (K) *K = e->K;
  if (group) *group = e->group;
  if (gamma) *gamma = e->gamma;
  if (packed_bytes) *packed_bytes = e->stream_bytes;
  return PIPE_OK;
}

extern "C" int pipe_expansion_order(const pipe_expansion* e, int k, int* n_groups_kept,
                                    int32_t* group_ids, float* scales, int8_t* codes_unpacked) {
  if (!e || k < 1 || k > e->K) return PIPE_EINVAL;
  const PipeOrder& o = e->orders[k - 1];
  if (n_groups_kept) *n_groups_kept = o.n_kept;
  if (group_ids) std::memcpy(group_ids, o.gids.data(), (size_t)o.n_kept * sizeof(int32_t));
  const size_t rows = (size_t)o.n_kept * e->group;
  PIPE_HIP(hipDeviceSynchronize());
  if (scales && rows) {
    // row scales sit at the row blocks' schedule positions
    const size_t n_pos = (size_t)e->n_pos;
    std::vector<float> all(n_pos * 16);
    PIPE_HIP(hipMemcpy(all.data(), e->scales_all_dev, all.size() * sizeof(float), hipMemcpyDeviceToHost));
    for (size_t c = 0; c < o.pos.size(); ++c) std::memcpy(scales + c * 16, &all[(size_t)o.pos[c] * 16], 16 * sizeof(float));
  }
  if (codes_unpacked && rows) {
    int8_t* tmp = nullptr;
    PIPE_HIP(hipMalloc(&tmp, rows * (size_t)e->in));
    int rc = launch_unpack_codes(e->codes_dev, o.pos_dev, e->bits, (int)rows, e->in, e->in_pad, tmp, nullptr);
    if (rc == PIPE_OK) {
      hipError_t he = hipMemcpy(codes_unpacked, tmp, rows * (size_t)e->in, hipMemcpyDeviceToHost);
      if (he != hipSuccess) { pipe_note_hip_error(he, "hipMemcpy(codes)"); rc = PIPE_EDEVICE; }
    }
    (void)hipFree(tmp);
    if (rc) return rc;
    if (e->conv_C > 0) {
      // stored tap-major: hand the rows back flattened [C, kh, kw], as the weight was given
      const int taps = e->conv_kh * e->conv_kw, C = e->conv_C;
      std::vector<int8_t> row((size_t)e->in);
      for (size_t r = 0; r < rows; ++r) {
        int8_t* dst = codes_unpacked + r * (size_t)e->in;
        std::memcpy(row.data(), dst, (size_t)e->in);
        for (int tap = 0; tap < taps; ++tap)
          for (int c = 0; c < C; ++c) dst[(size_t)c * taps + tap] = row[(size_t)tap * C + c];
      }
    }
  }
  return PIPE_OK;
}

// ------------------------------------------------------------------ tile schedules
const PassTables* pipe_get_tables(const pipe_expansion* ce, const GemmArgs& a, int kind, int* rc_out) {
  pipe_expansion* e = const_cast<pipe_expansion*>(ce);
  const int K = e->K, n_rb = e->n_rb;
  int M = a.M;
  int member_of[PIPE_MAX_K] = {0};
  unsigned long long nib = 0;
  if (kind == 2) {
    M = 1;
  } else {
    for (int m = 0; m < a.M; ++m)
      for (int k = a.member_lo[m]; k <= a.member_hi[m]; ++k) { member_of[k] = m; nib |= (unsigned long long)m << (4 * k); }
  }
  for (const PassTables& t : e->tables)
    if (t.kind == kind && t.M == M && t.member_nib == nib) return &t;
  *rc_out = PIPE_OK;
  if (kind == 1 && n_rb % 2 != 0) { *rc_out = PIPE_ESHAPE; return nullptr; }
  if (pipe_capturing()) { *rc_out = PIPE_ENOTREADY; return nullptr; }   // building allocates and copies synchronously

  // per row block and member: the positions of its stored orders, ascending
  std::vector<std::vector<int32_t>> list((size_t)n_rb * M);
  for (int rb = 0; rb < n_rb; ++rb)
    for (int k = 0; k < K; ++k) {
      const int32_t pos = e->pos_of[(size_t)k * n_rb + rb];
      if (kind == 2) list[rb].push_back(pos);
      else if (pos >= 0) list[(size_t)rb * M + member_of[k]].push_back(pos);
    }
  auto cnt = [&](int rb, int m) { return (int)list[(size_t)rb * M + m].size(); };
  // units that must share a tile: row blocks, or (gate, up) pairs
  const int n_units = kind == 1 ? n_rb / 2 : n_rb, per_tile = kind == 1 ? 8 : 16;
  auto ucnt = [&](int u, int m) { return kind == 1 ? std::max(cnt(u, m), cnt(u + n_units, m)) : cnt(u, m); };
  std::vector<int> units(n_units);
  for (int u = 0; u < n_units; ++u) units[u] = u;
  std::stable_sort(units.begin(), units.end(), [&](int x, int y) {
    for (int m = 0; m < M; ++m)
      if (ucnt(x, m) != ucnt(y, m)) return ucnt(x, m) > ucnt(y, m);
    if (kind == 1) {
      int tx = 0, ty = 0;
      for (int m = 0; m < M; ++m) { tx += cnt(x, m) + cnt(x + n_units, m); ty += cnt(y, m) + cnt(y + n_units, m); }
      if (tx != ty) return tx > ty;
    }
    return x < y;
  });
  PassTables t;
  t.member_nib = nib; t.M = M; t.kind = kind;
  t.n_ct = ceil_div(n_units, per_tile);
  t.n_sorted = (int)round_up64((int64_t)t.n_ct * 16, 64);
  // passes per (tile, member); heaviest tiles first
  std::vector<int> tile_of(t.n_ct);
  std::vector<std::vector<int>> passes(t.n_ct, std::vector<int>(M, 0));
  std::vector<int> total(t.n_ct, 0);
  for (int i = 0; i < n_units; ++i)
    for (int m = 0; m < M; ++m) passes[i / per_tile][m] = std::max(passes[i / per_tile][m], ucnt(units[i], m));
  for (int c = 0; c < t.n_ct; ++c) {
    tile_of[c] = c;
    for (int m = 0; m < M; ++m) { total[c] += passes[c][m]; t.p_max = std::max(t.p_max, passes[c][m]); }
  }
  std::stable_sort(tile_of.begin(), tile_of.end(), [&](int x, int y) { return total[x] > total[y]; });
  if (t.p_max > 255 || M > 16) { *rc_out = PIPE_EINVAL; return nullptr; }
  t.p_max = std::max(t.p_max, 1);
  std::vector<int32_t> rb_out((size_t)t.n_sorted, -1);
  std::vector<int32_t> src((size_t)M * t.p_max * t.n_sorted, -1);
  std::vector<uint8_t> cnts((size_t)t.n_ct * 16, 0);
  for (int c = 0; c < t.n_ct; ++c) {
    const int from = tile_of[c];
    for (int m = 0; m < M; ++m) cnts[(size_t)c * 16 + m] = (uint8_t)passes[from][m];
    for (int q = 0; q < per_tile && from * per_tile + q < n_units; ++q) {
      const int u = units[from * per_tile + q];
      const int rbs[2] = {u, u + n_units}, poss[2] = {c * 16 + q, c * 16 + 8 + q};
      for (int hh = 0; hh < (kind == 1 ? 2 : 1); ++hh) {
        rb_out[poss[hh]] = u;   // a pair stores to the gate block's channels
        for (int m = 0; m < M; ++m) {
          const std::vector<int32_t>& l = list[(size_t)rbs[hh] * M + m];
          for (size_t j = 0; j < l.size(); ++j) src[((size_t)m * t.p_max + j) * t.n_sorted + poss[hh]] = l[j];
        }
      }
    }
  }
  auto fail = [&](hipError_t he, const char* what) {
    pipe_note_hip_error(he, what);
    if (t.rb_out_dev) (void)hipFree(t.rb_out_dev);
    if (t.src_dev) (void)hipFree(t.src_dev);
    if (t.cnt_dev) (void)hipFree(t.cnt_dev);
    *rc_out = PIPE_EDEVICE;
    return (const PassTables*)nullptr;
  };
  hipError_t he;
  if ((he = hipMalloc(&t.rb_out_dev, rb_out.size() * 4)) != hipSuccess) return fail(he, "hipMalloc(rb_out)");
  if ((he = hipMalloc(&t.src_dev, src.size() * 4)) != hipSuccess) return fail(he, "hipMalloc(src)");
  if ((he = hipMalloc(&t.cnt_dev, cnts.size())) != hipSuccess) return fail(he, "hipMalloc(cnt)");
  if ((he = hipMemcpy(t.rb_out_dev, rb_out.data(), rb_out.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(he, "hipMemcpy(rb_out)");
  if ((he = hipMemcpy(t.src_dev, src.data(), src.size() * 4, hipMemcpyHostToDevice)) != hipSuccess) return fail(he, "hipMemcpy(src)");
  if ((he = hipMemcpy(t.cnt_dev, cnts.data(), cnts.size(), hipMemcpyHostToDevice)) != hipSuccess) return fail(he, "hipMemcpy(cnt)");
  e->tables.push_back(t);
  return &e->tables.back();
}

// ------------------------------------------------------------------ forward
static bool use_stream_kernel(const pipe_expansion* e, int T, bool acc_out = false) {
  if (g_kernel_choice == 1) return false;
  if (e->K > 4 && acc_out) return false;   // bins of more than 4 items have no integer export
  return T <= PIPE_STREAM_MAX_T;
}

struct ActBuffers {
  uint8_t* qx;
  int32_t* rowsum;
  uint32_t* amax;        // max|x| bit pattern: zero on entry, cleared again by the contraction kernel
  float* scale;          // [PIPE_MAX_K] scales
  int T_pad;
};

static int get_act_buffers(int T, int in_pad, bool small, ActBuffers* b) {
  b->T_pad = (int)round_up64(T, small ? 16 : TOK_TILE);
  b->qx = (uint8_t*)pipe_ws_get(WS_QX, (size_t)b->T_pad * in_pad);
  b->rowsum = (int32_t*)pipe_ws_get(WS_ROWSUM, (size_t)b->T_pad * 4);
  const bool fresh = t_ws == nullptr || t_ws->slot[WS_SCAL].ptr == nullptr;
  uint8_t* sc = (uint8_t*)pipe_ws_get(WS_SCAL, 4096);
  if (!b->qx || !b->rowsum || !sc) return pipe_ws_error();
  if (fresh) PIPE_HIP(hipMemset(sc, 0, 4096));   // never under capture: a fresh block is refused there
  b->amax = (uint32_t*)sc;
  b->scale = (float*)(sc + 1024);
  return PIPE_OK;
}

// The tile schedule the tiled kernel will need, fetched before anything is launched (so a failure
// leaves no reduction slot raised).
static int ensure_tables(const pipe_expansion* e, int M, const int* lo, const int* hi, int kind) {
  GemmArgs a{};
  a.e = e;
  a.M = M;
  for (int m = 0; m < M; ++m) { a.member_lo[m] = lo[m]; a.member_hi[m] = hi[m]; }
  int rc = PIPE_OK;
  return pipe_get_tables(e, a, kind, &rc) != nullptr ? PIPE_OK : rc;
}

// An error after the max|x| reduction was launched: the slot is raised and the contraction kernel
// that would clear it will not run.  Clears it so that the next dynamic scale starts from zero.
static int fail_after_reduction(int rc, const ActBuffers& b, hipStream_t st) {
  (void)launch_zero_u32(b.amax, 1, st);
  return rc;
}

// ------------------------------------------------------------------ kernel timing
static bool g_timing_on = false;
static std::vector<hipEvent_t> g_events;   // pairs: start, stop
static size_t g_events_used = 0;
constexpr size_t MAX_TIMED = 4096;

extern "C" int pipe_timing_enable(int on) {
  g_timing_on = on != 0;
  return PIPE_OK;
}

extern "C" int pipe_timing_read(double* total_ms, int* launches) {
  double tot = 0.0;
  for (size_t i = 0; i + 1 < g_events_used; i += 2) {
    PIPE_HIP(hipEventSynchronize(g_events[i + 1]));
    float ms = 0.f;
    PIPE_HIP(hipEventElapsedTime(&ms, g_events[i], g_events[i + 1]));
    tot += ms;
  }
  if (total_ms) *total_ms = tot;
  if (launches) *launches = (int)(g_events_used / 2);
  g_events_used = 0;
  return PIPE_OK;
}

// Activation quantization of a [T, in] input into the buffers of `b`; small batches take the
// single-launch path.
// A single token: the streaming kernel quantizes it itself, one launch instead of two
// (the kernel reads x while other workgroups already write results, so an output buffer that
// overlaps x -- legal on the two-launch path, whose quantizer has consumed x by then -- keeps that path)
static bool fuse_decode_quant(const pipe_expansion* e, int T, const float* x_dev, bool small,
                              const float* out_dev, size_t out_floats) {
  const uintptr_t x0 = reinterpret_cast<uintptr_t>(x_dev), x1 = x0 + (size_t)T * e->in * sizeof(float);
  const uintptr_t o0 = reinterpret_cast<uintptr_t>(out_dev), o1 = o0 + out_floats * sizeof(float);
  const bool apart = x1 <= o0 || o1 <= x0;
  return small && g_decode_fusion && T <= PIPE_FUSED_QUANT_MAX_T && e->in_pad <= PIPE_FUSED_QUANT_MAX_IN &&
         e->in % 4 == 0 && (x0 & 15) == 0 && e->bin_cap == 4 && apart;
}

static int quantize_input(const float* x_dev, int T, int in, int in_pad, float s_x, const ActBuffers& b, bool small,
                          int8_t* qx_rowmajor, float* scale_out, hipStream_t st) {
  if (small && T <= PIPE_QUANT1_MAX_T)
    return launch_quantize_small(x_dev, 0, 1, T, in, in_pad, s_x, nullptr, b.qx, 0, b.rowsum, qx_rowmajor, scale_out, st);
  // The reduction slot is zero on entry (workspace allocation, then every contraction kernel
  // clears it again); the reduction kernel also clears the code sums, so a dynamic scale costs
  // two launches and no memset.
  const bool dynamic = !(s_x > 0.f);
  if (dynamic) {
    int rc = launch_absmax(x_dev, (int64_t)T * in, b.amax, b.rowsum, b.T_pad, st);
    if (rc) return rc;
  }
  return launch_quantize_act(x_dev, T, in, in_pad, b.T_pad, s_x, b.amax, b.qx, b.rowsum, dynamic, qx_rowmajor, scale_out, st);
}

// While timing is on: the pair of events the next contraction launch records its begin and end into.
static int timing_events(hipEvent_t* ev0, hipEvent_t* ev1, bool* timed) {
  *timed = g_timing_on && g_events_used / 2 < MAX_TIMED;
  if (!*timed) return PIPE_OK;
  while (g_events.size() < g_events_used + 2) {
    hipEvent_t ev;
    PIPE_HIP(hipEventCreate(&ev));
    g_events.push_back(ev);
  }
  *ev0 = g_events[g_events_used];
  *ev1 = g_events[g_events_used + 1];
  return PIPE_OK;
}

static int run_gemm(const GemmArgs& a0, bool small, hipStream_t st) {
  if (pipe_dry_run()) return PIPE_OK;
  GemmArgs a = a0;
  bool timed = false;
  int rc = timing_events(&a.ev_start, &a.ev_stop, &timed);
  if (rc) return rc;
  rc = small ? launch_gemm_stream(a, st) : launch_gemm_tiled(a, st);
  if (timed && rc == PIPE_OK) g_events_used += 2;
  return rc;
}

static void fill_members(GemmArgs& a, int M, const int* lo, const int* hi) {
  a.M = M;
  for (int m = 0; m < PIPE_MAX_K; ++m) { a.member_lo[m] = 0; a.member_hi[m] = -1; }
  for (int m = 0; m < M; ++m) { a.member_lo[m] = lo[m]; a.member_hi[m] = hi[m]; }
}

extern "C" int pipe_forward(const pipe_expansion* e, const float* x_dev, int T, float s_x,
                            const int* split, int M, const float* bias_dev, int reduce_members,
                            float* y_dev, void* stream) {
  if (!e || T < 0) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  const bool small = use_stream_kernel(e, T);
  ActBuffers b;
  rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  if (!small && (rc = ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  const bool fused = fuse_decode_quant(e, T, x_dev, small, y_dev, (size_t)(reduce_members ? 1 : Mm) * T * e->out);
  if (!fused) {
    rc = quantize_input(x_dev, T, e->in, e->in_pad, s_x, b, small, nullptr, b.scale, st);
    if (rc) return rc;
  }
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.qx_mstride = 0; a.rowsum = b.rowsum; a.rowsum_mstride = 0;
  a.s_x = b.scale; a.sx_mstride = 0; a.bias = bias_dev; a.reduce = reduce_members ? 1 : 0; a.act = 0;
  a.y = y_dev; a.acc_out = nullptr; a.amax_out = nullptr; a.zero_after = b.amax;
  if (fused) { a.x_f32 = x_dev; a.s_static = s_x; }
  fill_members(a, Mm, lo, hi);
  rc = run_gemm(a, small, st);
  return rc == PIPE_OK ? rc : fail_after_reduction(rc, b, st);
}

extern "C" int pipe_prepare(const pipe_expansion* e, const int* split, int M, int T_max, void* stream) {
  if (!e || T_max < 1) return PIPE_EINVAL;
  DryScope dry;
  // the addresses are never dereferenced: nothing is launched in a dry run.  Two passes: the
  // largest batch sizes the scratch, and whichever kernel serves it gets its schedule; batches
  // up to T_max may also take the tiled kernel's path, whose schedule the second pass builds.
  const float* fake_x = reinterpret_cast<const float*>(uintptr_t(256));
  float* fake_y = reinterpret_cast<float*>(uintptr_t(512));
  int rc = pipe_forward(e, fake_x, T_max, 1.f, split, M, nullptr, 1, fake_y, stream);
  if (rc == PIPE_OK && T_max > PIPE_STREAM_MAX_T + 1)
    rc = pipe_forward(e, fake_x, PIPE_STREAM_MAX_T + 1, 1.f, split, M, nullptr, 1, fake_y, stream);
  return rc;
}

extern "C" int pipe_forward_acc(const pipe_expansion* e, const float* x_dev, int T, float s_x,
                                int32_t* acc_dev, int8_t* qx_dev, float* s_x_out_dev, void* stream) {
  if (!e || T < 0) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  if (T == 0) return PIPE_OK;
  if (!x_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  const bool small = use_stream_kernel(e, T, acc_dev != nullptr);
  ActBuffers b;
  int rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  int lo = 0, hi = e->K - 1;
  if (acc_dev && !small && (rc = ensure_tables(e, 1, &lo, &hi, 2)) != PIPE_OK) return rc;
  rc = quantize_input(x_dev, T, e->in, e->in_pad, s_x, b, small, qx_dev, b.scale, st);
  if (rc) return rc;
  if (s_x_out_dev) PIPE_HIP(hipMemcpyAsync(s_x_out_dev, b.scale, sizeof(float), hipMemcpyDeviceToDevice, st));
  if (!acc_dev) return launch_zero_u32(b.amax, 1, st);   // no contraction kernel follows to clear it
  PIPE_HIP(hipMemsetAsync(acc_dev, 0, (size_t)e->K * T * e->out * sizeof(int32_t), st));
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.rowsum = b.rowsum;
  a.s_x = b.scale; a.reduce = 1; a.acc_out = acc_dev; a.zero_after = b.amax;
  fill_members(a, 1, &lo, &hi);
  rc = run_gemm(a, small, st);
  return rc == PIPE_OK ? rc : fail_after_reduction(rc, b, st);
}

// ------------------------------------------------------------------ the entry point that allocates nothing
// pipe_forward for callers that cannot allocate: its scratch -- max|x| slot and scale, token code
// sums, Q(x) in the fragment layout -- is a fixed array in device memory, one copy per GPU, shared
// by every call on that GPU and keeping the last call's contents.
constexpr size_t NOALLOC_SCAL_BYTES = 4096;                 // max|x| slot at 0, scale at 1024
constexpr int NOALLOC_MAX_TOKENS = 8192;
constexpr size_t NOALLOC_ROWSUM_BYTES = (size_t)NOALLOC_MAX_TOKENS * 4;
constexpr size_t NOALLOC_QX_BYTES = (size_t)8 << 20;        // padded tokens x padded in_features
static __device__ __align__(256) unsigned char scratch[NOALLOC_SCAL_BYTES + NOALLOC_ROWSUM_BYTES + NOALLOC_QX_BYTES];
constexpr int NOALLOC_MAX_DEVICES = 64;
static unsigned char* g_scratch_ptr[NOALLOC_MAX_DEVICES] = {};   // device address of `scratch` on each GPU
static std::mutex g_scratch_mu;

// The array's address on the current device (each GPU holds its own copy at its own address),
// looked up once per device.
static int noalloc_scratch(unsigned char** out) {
  int dev = 0;
  PIPE_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= NOALLOC_MAX_DEVICES) return PIPE_EDEVICE;
  std::lock_guard<std::mutex> lk(g_scratch_mu);
  if (g_scratch_ptr[dev] == nullptr) {
    unsigned char* ptr = nullptr;
    PIPE_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
    if (ptr == nullptr) return PIPE_EDEVICE;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return PIPE_OK;
}

extern "C" int pipe_forward_noalloc(const pipe_expansion* e, const float* x_dev, int T, float s_x, const int* split,
                                    int M, const float* bias_dev, int reduce_members, float* y_dev, void* stream) {
  if (!e || T < 0) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  const bool small = use_stream_kernel(e, T);
  ActBuffers b;
  b.T_pad = (int)round_up64(T, small ? 16 : TOK_TILE);
  if (b.T_pad > NOALLOC_MAX_TOKENS || (size_t)b.T_pad * e->in_pad > NOALLOC_QX_BYTES) return PIPE_ELIMIT;
  unsigned char* base = nullptr;
  if ((rc = noalloc_scratch(&base)) != PIPE_OK) return rc;
  b.amax = reinterpret_cast<uint32_t*>(base);
  b.scale = reinterpret_cast<float*>(base + 1024);
  b.rowsum = reinterpret_cast<int32_t*>(base + NOALLOC_SCAL_BYTES);
  b.qx = base + NOALLOC_SCAL_BYTES + NOALLOC_ROWSUM_BYTES;
  struct Guard {   // schedules are looked up, never built, inside this call
    Guard() { t_no_alloc = true; }
    ~Guard() { t_no_alloc = false; }
  } guard;
  if (!small && (rc = ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  const bool fused = fuse_decode_quant(e, T, x_dev, small, y_dev, (size_t)(reduce_members ? 1 : Mm) * T * e->out);
  if (!fused) {
    // The array keeps what the last call left: the max|x| slot has to start at zero (a call that
    // failed after its reduction, or that overlapped another one, may have left it raised).
    const bool uses_slot = !(s_x > 0.f) && !(small && T <= PIPE_QUANT1_MAX_T);
    if (uses_slot && (rc = launch_zero_u32(b.amax, 1, st)) != PIPE_OK) return rc;
    rc = quantize_input(x_dev, T, e->in, e->in_pad, s_x, b, small, nullptr, b.scale, st);
    if (rc) return rc;
  }
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.rowsum = b.rowsum; a.s_x = b.scale;
  a.bias = bias_dev; a.reduce = reduce_members ? 1 : 0; a.y = y_dev; a.zero_after = b.amax;
  if (fused) { a.x_f32 = x_dev; a.s_static = s_x; }
  fill_members(a, Mm, lo, hi);
  rc = small ? launch_gemm_stream(a, st) : launch_gemm_tiled(a, st);   // no timing events: creating one allocates
  return rc == PIPE_OK ? rc : fail_after_reduction(rc, b, st);
}

// ------------------------------------------------------------------ asymmetric activation codes
// Sums of the stored codes per order and output channel, and C[o] = sum_k s_k[o] * wsum_k[o] (fp32,
// ascending k), built once per expansion (synchronizes; allocates).
static int asym_prepare(const pipe_expansion* ce, hipStream_t st) {
  pipe_expansion* e = const_cast<pipe_expansion*>(ce);
  if (e->asym_C_dev) return PIPE_OK;
  if (pipe_capturing()) return PIPE_ENOTREADY;   // allocates and synchronizes: run the call once outside capture
  const size_t out = (size_t)e->out;
  int32_t* wsum = nullptr;
  float* C = nullptr;
  float* be = nullptr;
  float* P = nullptr;
  PIPE_HIP(hipMalloc(&wsum, (size_t)e->K * out * sizeof(int32_t)));
  hipError_t he = hipMemsetAsync(wsum, 0, (size_t)e->K * out * sizeof(int32_t), st);
  int rc = he == hipSuccess ? PIPE_OK : PIPE_EDEVICE;
  int8_t* tmp = nullptr;
  size_t max_rows = 0;
  for (auto& o : e->orders) max_rows = std::max(max_rows, (size_t)o.n_kept * e->group);
  if (rc == PIPE_OK && hipMalloc(&tmp, max_rows * (size_t)e->in) != hipSuccess) rc = PIPE_ENOMEM;
  for (int k = 0; k < e->K && rc == PIPE_OK; ++k) {
    const PipeOrder& o = e->orders[k];
    const int rows = o.n_kept * e->group;
    rc = launch_unpack_codes(e->codes_dev, o.pos_dev, e->bits, rows, e->in, e->in_pad, tmp, st);
    if (rc == PIPE_OK) rc = launch_row_code_sums(tmp, rows, e->in, e->group, o.gids_dev, wsum + (size_t)k * out, st);
  }
  std::vector<int32_t> hw((size_t)e->K * out);
  std::vector<float> all((size_t)e->n_pos * 16), hC(out, 0.f), hP((size_t)e->K * out, 0.f);
  if (rc == PIPE_OK && (hipStreamSynchronize(st) != hipSuccess ||
                        hipMemcpy(hw.data(), wsum, hw.size() * sizeof(int32_t), hipMemcpyDeviceToHost) != hipSuccess ||
                        hipMemcpy(all.data(), e->scales_all_dev, all.size() * sizeof(float), hipMemcpyDeviceToHost) != hipSuccess))
    rc = PIPE_EDEVICE;
  if (tmp) (void)hipFree(tmp);
  if (rc == PIPE_OK) {
    for (int k = 0; k < e->K; ++k) {
      const PipeOrder& o = e->orders[k];
      for (int slot = 0; slot < o.n_kept; ++slot)
        for (int j = 0; j < e->group; ++j) {
          const int r = slot * e->group + j;
          const size_t ch = (size_t)o.gids[slot] * e->group + j;
          const float pk = all[(size_t)o.pos[r >> 4] * 16 + (r & 15)] * (float)hw[(size_t)k * out + ch];
          hP[(size_t)k * out + ch] = pk;
          hC[ch] += pk;
        }
    }
    if (hipMalloc(&C, out * sizeof(float)) != hipSuccess || hipMalloc(&be, out * sizeof(float)) != hipSuccess ||
        hipMalloc(&P, hP.size() * sizeof(float)) != hipSuccess ||
        hipMemcpy(C, hC.data(), out * sizeof(float), hipMemcpyHostToDevice) != hipSuccess ||
        hipMemcpy(P, hP.data(), hP.size() * sizeof(float), hipMemcpyHostToDevice) != hipSuccess)
      rc = PIPE_EDEVICE;
  }
  if (rc != PIPE_OK) {
    if (wsum) (void)hipFree(wsum);
    if (C) (void)hipFree(C);
    if (be) (void)hipFree(be);
    if (P) (void)hipFree(P);
    return rc;
  }
  e->asym_wsum_dev = wsum; e->asym_C_dev = C; e->asym_bias_dev = be; e->asym_P_dev = P;
  return PIPE_OK;
}

// quantizes x with asymmetric codes into the activation buffers; dz (= 2^(a-1) - z) and the scale stay on the device
static int asym_quantize(const pipe_expansion* e, const float* x_dev, int T, const ActBuffers& b, uint8_t* qx_u8,
                         uint32_t** slots_out, int32_t** dz_out, hipStream_t st) {
  const int act_bits = (int)std::lround(std::log2((double)g_act_qmax_host + 1.0)) + 1;
  // |Q(x) - z| <= 2^a - 1: the exact accumulator must fit 32 bits
  if ((int64_t)((1 << act_bits) - 1) * ((1 << (e->qbits - 1)) - 1) * e->in >= ((int64_t)1 << 31)) return PIPE_ESHAPE;
  uint32_t* slots = b.amax + 64;              // two range slots, zero between calls
  int32_t* dz = reinterpret_cast<int32_t*>(b.amax + 66);
  int rc = launch_minmax(x_dev, (int64_t)T * e->in, slots, st);
  if (rc) return rc;
  rc = launch_quantize_asym(x_dev, T, e->in, e->in_pad, b.T_pad, slots, slots + 1, act_bits, b.qx, b.rowsum, qx_u8, b.scale, dz, st);
  *slots_out = slots; *dz_out = dz;
  return rc;
}

extern "C" int pipe_forward_asymmetric(const pipe_expansion* e, const float* x_dev, int T, const int* split, int M,
                                       const float* bias_dev, float* y_dev, void* stream) {
  if (!e || T < 0) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  rc = asym_prepare(e, st);
  if (rc) return rc;
  const bool small = use_stream_kernel(e, T);
  ActBuffers b;
  rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  if (!small && (rc = ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  uint32_t* slots = nullptr;
  int32_t* dz = nullptr;
  rc = asym_quantize(e, x_dev, T, b, nullptr, &slots, &dz, st);
  if (rc) return rc;
  rc = launch_asym_bias(bias_dev, e->asym_C_dev, b.scale, dz, e->asym_bias_dev, e->out, slots, st);
  if (rc) return rc;
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.qx_mstride = 0; a.rowsum = b.rowsum; a.rowsum_mstride = 0;
  a.s_x = b.scale; a.sx_mstride = 0; a.bias = e->asym_bias_dev; a.reduce = 1; a.act = 0;
  a.y = y_dev; a.acc_out = nullptr; a.amax_out = nullptr; a.zero_after = b.amax;
  fill_members(a, Mm, lo, hi);
  return run_gemm(a, small, st);
}

extern "C" int pipe_forward_conv2d_asymmetric(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W,
                                              int kh, int kw, int stride, int pad, int nhwc, const int* split, int M,
                                              const float* bias_dev, float* y_dev, void* stream) {
  if (!e) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return PIPE_ESHAPE;
  if ((int64_t)C * kh * kw != e->in) return PIPE_ESHAPE;
  const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
  if (H + 2 * pad < kh || W + 2 * pad < kw) return PIPE_ESHAPE;
  const int64_t T64 = (int64_t)N * Ho * Wo;
  if (T64 > (int64_t)1 << 30) return PIPE_ESHAPE;
  const int T = (int)T64;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  const int act_bits = (int)std::lround(std::log2((double)g_act_qmax_host + 1.0)) + 1;
  if ((int64_t)((1 << act_bits) - 1) * ((1 << (e->qbits - 1)) - 1) * e->in >= ((int64_t)1 << 31)) return PIPE_ESHAPE;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  rc = asym_prepare(e, st);
  if (rc) return rc;
  const bool small = use_stream_kernel(e, T);
  ActBuffers b;
  rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  if (!small && (rc = ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  int8_t* q8 = (int8_t*)pipe_ws_get(WS_Q8X, (size_t)N * C * H * W);   // the input's codes, in its own layout
  if (!q8) return pipe_ws_error();
  uint32_t* slots = b.amax + 64;
  int32_t* dz = reinterpret_cast<int32_t*>(b.amax + 66);
  rc = launch_minmax(x_dev, (int64_t)N * C * H * W, slots, st);
  if (rc) return rc;
  rc = launch_quantize_im2col_asym(x_dev, N, C, H, W, kh, kw, stride, pad, nhwc, Ho, Wo, e->in_pad, b.T_pad, slots, slots + 1,
                                   act_bits, q8, b.qx, b.rowsum, b.scale, dz, st);
  if (rc) return rc;
  rc = launch_asym_bias(bias_dev, e->asym_C_dev, b.scale, dz, e->asym_bias_dev, e->out, slots, st);
  if (rc) return rc;
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.rowsum = b.rowsum;
  a.s_x = b.scale; a.bias = e->asym_bias_dev; a.reduce = 1; a.y = y_dev; a.zero_after = b.amax;
  fill_members(a, Mm, lo, hi);
  return run_gemm(a, small, st);
}

extern "C" int pipe_forward_acc_asymmetric(const pipe_expansion* e, const float* x_dev, int T, int32_t* acc_dev,
                                           uint8_t* qx_dev, float* s_x_out_dev, int32_t* z_out_dev, void* stream) {
  if (!e || T < 0) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  if (T == 0) return PIPE_OK;
  if (!x_dev || !acc_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  int rc = asym_prepare(e, st);
  if (rc) return rc;
  const bool small = use_stream_kernel(e, T, true);
  ActBuffers b;
  rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  int klo = 0, khi = e->K - 1;
  if (!small && (rc = ensure_tables(e, 1, &klo, &khi, 2)) != PIPE_OK) return rc;
  uint32_t* slots = nullptr;
  int32_t* dz = nullptr;
  rc = asym_quantize(e, x_dev, T, b, qx_dev, &slots, &dz, st);
  if (rc) return rc;
  rc = launch_asym_bias(nullptr, e->asym_C_dev, b.scale, dz, e->asym_bias_dev, e->out, slots, st);   // clears the range slots
  if (rc) return rc;
  PIPE_HIP(hipMemsetAsync(acc_dev, 0, (size_t)e->K * T * e->out * sizeof(int32_t), st));
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.rowsum = b.rowsum;
  a.s_x = b.scale; a.reduce = 1; a.acc_out = acc_dev; a.zero_after = b.amax;
  fill_members(a, 1, &klo, &khi);
  rc = run_gemm(a, small, st);
  if (rc) return rc;
  rc = launch_asym_acc_fix(acc_dev, e->asym_wsum_dev, dz, e->K, T, e->out, st);
  if (rc) return rc;
  if (s_x_out_dev) PIPE_HIP(hipMemcpyAsync(s_x_out_dev, b.scale, sizeof(float), hipMemcpyDeviceToDevice, st));
  if (z_out_dev) {
    // z = 2^(a-1) - dz; an all-zero input has z = 0 and dz = 0
    const int act_bits = (int)std::lround(std::log2((double)g_act_qmax_host + 1.0)) + 1;
    int32_t hdz = 0;
    float hs = 0.f;
    PIPE_HIP(hipMemcpyAsync(&hdz, dz, sizeof(int32_t), hipMemcpyDeviceToHost, st));
    PIPE_HIP(hipMemcpyAsync(&hs, b.scale, sizeof(float), hipMemcpyDeviceToHost, st));
    PIPE_HIP(hipStreamSynchronize(st));
    const int32_t z = hs > 0.f ? (1 << (act_bits - 1)) - hdz : 0;
    PIPE_HIP(hipMemcpyAsync(z_out_dev, &z, sizeof(int32_t), hipMemcpyHostToDevice, st));
    PIPE_HIP(hipStreamSynchronize(st));
  }
  return PIPE_OK;
}

// The convolution layer; with acc_dev set, the integer export (accumulators per order, the input's codes in the
// input's own layout, the scale) instead of the fp32 output.
static int conv2d_impl(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W, int kh, int kw, int stride,
                       int pad, int nhwc, float s_x, const int* split, int M, const float* bias_dev, int reduce_members,
                       float* y_dev, int32_t* acc_dev, int8_t* qx_dev, float* s_x_out_dev, void* stream) {
  if (!e) return PIPE_EINVAL;
  if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return PIPE_ESHAPE;
  if ((int64_t)C * kh * kw != e->in) return PIPE_ESHAPE;
  const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
  if (H + 2 * pad < kh || W + 2 * pad < kw) return PIPE_ESHAPE;
  const int64_t T64 = (int64_t)N * Ho * Wo;
  if (T64 > (int64_t)1 << 30) return PIPE_ESHAPE;
  const int T = (int)T64;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  const bool export_acc = acc_dev != nullptr;
  if (!x_dev || (!y_dev && !export_acc)) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  const size_t n_in = (size_t)N * C * H * W;
  if (e->conv_C > 0) {
    // ---- implicit GEMM (an expansion stored tap-major by pipe_expand_conv2d): no patch matrix.  The input
    // is quantized once into channels-last codes with per-pixel channel sums; the tiled kernel's activation
    // stage gathers each tap's 64-channel chunks from them.  Launches: max|x| (also clears the sums),
    // quantizer, contraction.
    if (C != e->conv_C || kh != e->conv_kh || kw != e->conv_kw) return PIPE_ESHAPE;
    if (n_in >= ((size_t)1 << 31)) return PIPE_ESHAPE;   // 32-bit element offsets in the kernel
    ActBuffers b;
    rc = get_act_buffers(16, IN_PAD, true, &b);   // only the scale and max slots are used
    if (rc) return rc;
    int8_t* q8 = (int8_t*)pipe_ws_get(WS_Q8X, n_in);
    int32_t* csum = (int32_t*)pipe_ws_get(WS_CSUM, (size_t)N * H * W * sizeof(int32_t));
    if (!q8 || !csum) return pipe_ws_error();
    int klo = 0, khi = e->K - 1;
    if ((rc = export_acc ? ensure_tables(e, 1, &klo, &khi, 2) : ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
    if (!(s_x > 0.f)) rc = launch_absmax(x_dev, (int64_t)n_in, b.amax, csum, N * H * W, st);
    else rc = launch_zero_u32(reinterpret_cast<uint32_t*>(csum), N * H * W, st);
    if (rc) return rc;
    rc = launch_quantize_nhwc_sums(x_dev, N, C, H * W, nhwc, s_x, b.amax, q8, csum, b.scale, st);
    if (rc) return fail_after_reduction(rc, b, st);
    GemmArgs a{};
    a.e = e; a.T = T; a.T_pad = (int)round_up64(T, TOK_TILE); a.s_x = b.scale; a.zero_after = b.amax;
    a.conv_q8 = q8; a.conv_csum = csum; a.conv_zero = e->conv_zero_dev;
    a.conv_C = C; a.conv_H = H; a.conv_W = W; a.conv_kh = kh; a.conv_kw = kw; a.conv_stride = stride; a.conv_pad = pad;
    a.conv_Ho = Ho; a.conv_Wo = Wo;
    if (export_acc) {
      if (!pipe_dry_run()) {
        if (qx_dev) {
          // the codes in the input's own layout
          if (nhwc) PIPE_HIP(hipMemcpyAsync(qx_dev, q8, n_in, hipMemcpyDeviceToDevice, st));
          else if ((rc = launch_quantize_elem(x_dev, (int64_t)n_in, s_x, b.amax, qx_dev, nullptr, st)) != PIPE_OK) return fail_after_reduction(rc, b, st);
        }
        if (s_x_out_dev) PIPE_HIP(hipMemcpyAsync(s_x_out_dev, b.scale, sizeof(float), hipMemcpyDeviceToDevice, st));
        PIPE_HIP(hipMemsetAsync(acc_dev, 0, (size_t)e->K * T * e->out * sizeof(int32_t), st));
      }
      a.reduce = 1; a.acc_out = acc_dev;
      fill_members(a, 1, &klo, &khi);
    } else {
      a.bias = bias_dev; a.reduce = reduce_members ? 1 : 0; a.y = y_dev;
      fill_members(a, Mm, lo, hi);
    }
    rc = run_gemm(a, false, st);
    return rc == PIPE_OK ? rc : fail_after_reduction(rc, b, st);
  }
  const bool small = use_stream_kernel(e, T, export_acc);
  ActBuffers b;
  rc = get_act_buffers(T, e->in_pad, small, &b);
  if (rc) return rc;
  int8_t* q8 = (int8_t*)pipe_ws_get(WS_Q8X, n_in);   // the input's codes, in its own layout
  if (!q8) return pipe_ws_error();
  {
    int klo = 0, khi = e->K - 1;
    if (!small && (rc = export_acc ? ensure_tables(e, 1, &klo, &khi, 2) : ensure_tables(e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  }
  if (!(s_x > 0.f)) {
    rc = launch_absmax(x_dev, (int64_t)n_in, b.amax, nullptr, 0, st);
    if (rc) return rc;
  }
  rc = launch_quantize_im2col(x_dev, N, C, H, W, kh, kw, stride, pad, nhwc, Ho, Wo, e->in_pad, b.T_pad, s_x,
                              b.amax, q8, b.qx, b.rowsum, b.scale, st);
  if (rc) return rc;
  GemmArgs a{};
  a.e = e; a.T = T; a.T_pad = b.T_pad; a.qx = b.qx; a.rowsum = b.rowsum;
  a.s_x = b.scale; a.zero_after = b.amax;
  if (export_acc) {
    if (pipe_dry_run()) return PIPE_OK;
    if (qx_dev) PIPE_HIP(hipMemcpyAsync(qx_dev, q8, n_in, hipMemcpyDeviceToDevice, st));
    if (s_x_out_dev) PIPE_HIP(hipMemcpyAsync(s_x_out_dev, b.scale, sizeof(float), hipMemcpyDeviceToDevice, st));
    PIPE_HIP(hipMemsetAsync(acc_dev, 0, (size_t)e->K * T * e->out * sizeof(int32_t), st));
    a.reduce = 1; a.acc_out = acc_dev;
    int klo = 0, khi = e->K - 1;
    fill_members(a, 1, &klo, &khi);
  } else {
    a.bias = bias_dev; a.reduce = reduce_members ? 1 : 0; a.y = y_dev;
    fill_members(a, Mm, lo, hi);
  }
  rc = run_gemm(a, small, st);
  return rc == PIPE_OK ? rc : fail_after_reduction(rc, b, st);
}

extern "C" int pipe_forward_conv2d(const pipe_expansion* e, const float* x_dev, int N, int C, int H,
                                   int W, int kh, int kw, int stride, int pad, int nhwc, float s_x,
                                   const int* split, int M, const float* bias_dev,
                                   int reduce_members, float* y_dev, void* stream) {
  return conv2d_impl(e, x_dev, N, C, H, W, kh, kw, stride, pad, nhwc, s_x, split, M, bias_dev, reduce_members, y_dev,
                     nullptr, nullptr, nullptr, stream);
}

extern "C" int pipe_forward_conv2d_acc(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W, int kh,
                                       int kw, int stride, int pad, int nhwc, float s_x, int32_t* acc_dev,
                                       int8_t* qx_dev, float* s_x_out_dev, void* stream) {
  if (!acc_dev) return PIPE_EINVAL;
  return conv2d_impl(e, x_dev, N, C, H, W, kh, kw, stride, pad, nhwc, s_x, nullptr, 0, nullptr, 1, nullptr, acc_dev,
                     qx_dev, s_x_out_dev, stream);
}

extern "C" int pipe_forward_depthwise2d(const pipe_expansion* e, const float* x_dev, int N, int C, int H, int W,
                                        int kh, int kw, int stride, int pad, int nhwc, float s_x, const int* split,
                                        int M, const float* bias_dev, int reduce_members, float* y_dev, void* stream) {
  if (!e) return PIPE_EINVAL;
  if (e->conv_C > 0) return PIPE_EINVAL;   // stored tap-major: only the convolution entry points read it
  if (N < 0 || C <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0 || pad < 0) return PIPE_ESHAPE;
  if (C != e->out || kh * kw != e->in || kh * kw > 49) return PIPE_ESHAPE;
  if (H + 2 * pad < kh || W + 2 * pad < kw) return PIPE_ESHAPE;
  const int Ho = (H + 2 * pad - kh) / stride + 1, Wo = (W + 2 * pad - kw) / stride + 1;
  if ((int64_t)N * Ho * Wo * C > (int64_t)1 << 40) return PIPE_ESHAPE;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(e->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (N == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  rc = pipe_depthwise_prepare(const_cast<pipe_expansion*>(e), st);
  if (rc) return rc;
  ActBuffers b;
  rc = get_act_buffers(16, IN_PAD, true, &b);   // only the scale and max slots are used
  if (rc) return rc;
  const int64_t n = (int64_t)N * C * H * W;
  int8_t* q8 = (int8_t*)pipe_ws_get(WS_Q8X, (size_t)n);
  if (!q8) return pipe_ws_error();
  if (!(s_x > 0.f)) {
    rc = launch_absmax(x_dev, n, b.amax, nullptr, 0, st);
    if (rc) return rc;
  }
  // the codes of the input, channels last whatever the input's layout
  if (nhwc) rc = launch_quantize_elem(x_dev, n, s_x, b.amax, q8, b.scale, st);
  else rc = launch_quantize_to_nhwc(x_dev, N, C, H * W, s_x, b.amax, g_act_qmax_host, q8, b.scale, st);
  if (rc) return rc;
  rc = launch_depthwise(e, q8, b.scale, N, C, H, W, kh, kw, stride, pad, Ho, Wo, Mm, lo, hi, bias_dev,
                        reduce_members ? 1 : 0, y_dev, st);
  if (rc) return rc;
  return launch_zero_u32(b.amax, 1, st);   // no contraction kernel follows to clear the max slot
}

// ------------------------------------------------------------------ resident decode launch
// Scratch of the resident kernel in the stream's workspace: flag words, tagged maxima, the epoch the
// last launch ended with and the status word (all zero when allocated; the kernels keep them
// consistent afterwards), and one code buffer per layer.
constexpr size_t RES_FLAGS_BYTES = 4096, RES_TAG_BYTES = 1024 * 2 * 8, RES_CTRL_BYTES = RES_FLAGS_BYTES + RES_TAG_BYTES + 256;

struct ResidentLayerSpec {
  const pipe_expansion* e;
  const float* bias;
  float* out;
  const float* res;
  long long res_mstride;
  int res_members, res_pre_act, res_device, act, gated;
  const float* s_in;   // HOST: given scales of the members' tensors entering the layer, or nullptr (layers after the first)
};

// given_scales: every tensor's scale is given, so the launch exchanges no maxima
static bool resident_eligible(const pipe_expansion* const* es, int L, int T, int M, const float* x_dev, bool given_scales = false) {
  if (!g_decode_resident || g_kernel_choice == 1) return false;
  // automatic: where it measured faster (short chains of few tokens only when no maxima are exchanged)
  if (g_decode_resident == 1 && L < 3 && T <= 8 && !given_scales) return false;   // (gated MLP, 8 tokens: 60.0 against 65.2 us; 16 tokens: 68.4 against 66.5)
  if (T < 1 || T > 16 || M > PIPE_RES_MAX_M || L > PIPE_RES_MAX_LAYERS) return false;
  if (es[0]->in % 4 != 0 || (reinterpret_cast<uintptr_t>(x_dev) & 15) != 0) return false;
  for (int l = 0; l < L; ++l)
    if (es[l]->bin_cap != 4 || es[l]->K > 4 || es[l]->bits != es[0]->bits) return false;
  return true;
}

static int run_resident(const ResidentLayerSpec* ls, int L, const float* x_dev, int T, float s_x, int M, const int* lo,
                        const int* hi, hipStream_t st) {
  ResidentArgs a;
  std::memset(&a, 0, sizeof(a));
  a.L = L; a.T = T; a.M = M; a.G = pipe_resident_workgroups();
  for (int m = 0; m < M; ++m) { a.member_lo[m] = lo[m]; a.member_hi[m] = hi[m]; }
  a.x = x_dev; a.s_static = s_x;
  const bool fresh = t_ws == nullptr || t_ws->slot[WS_RES].ptr == nullptr;
  uint8_t* ctrl = (uint8_t*)pipe_ws_get(WS_RES, RES_CTRL_BYTES);
  if (!ctrl) return pipe_ws_error();
  if (fresh) PIPE_HIP(hipMemset(ctrl, 0, RES_CTRL_BYTES));   // never under capture: a fresh block is refused there
  a.flags = reinterpret_cast<uint32_t*>(ctrl);
  a.amax_tag = reinterpret_cast<unsigned long long*>(ctrl + RES_FLAGS_BYTES);
  a.gen = reinterpret_cast<uint32_t*>(ctrl + RES_FLAGS_BYTES + RES_TAG_BYTES);
  a.status = a.gen + 16;
  size_t q_bytes = 0;
  std::vector<size_t> q_off(L);
  for (int l = 0; l < L; ++l) {
    q_off[l] = q_bytes;
    q_bytes += (size_t)round_up64((int64_t)(l == 0 ? 1 : M) * 16 * ls[l].e->in_pad, 256);
  }
  uint8_t* qbuf = (uint8_t*)pipe_ws_get(WS_RES_Q, q_bytes);
  if (!qbuf) return pipe_ws_error();
  for (int l = 0; l < L; ++l) {
    ResidentLayerArgs& la = a.layers[l];
    la.e = ls[l].e;
    int rc = pipe_resident_tables(ls[l].e, ls[l].gated ? 1 : 0, a.G, &la.tables);
    if (rc) return rc;
    la.bias = ls[l].bias; la.out = ls[l].out; la.res = ls[l].res; la.res_mstride = ls[l].res_mstride;
    la.res_members = ls[l].res_members; la.res_pre_act = ls[l].res_pre_act; la.res_device = ls[l].res_device;
    la.act = ls[l].act; la.gated = ls[l].gated;
    la.s_in[0] = la.s_in[1] = 0.f;
    if (l > 0 && ls[l].s_in != nullptr)
      for (int m = 0; m < M && m < PIPE_RES_MAX_M; ++m) la.s_in[m] = ls[l].s_in[m];
    la.qin = qbuf + q_off[l];
  }
  // the busiest workgroup's unit descriptors have to fit the kernel's LDS copy; else the caller
  // takes the per-layer launches
  int desc_ints = 0;
  for (int l = 0; l < L; ++l) desc_ints += ceil_div(a.layers[l].tables.n_units, a.G) * (a.layers[l].tables.nsub * 16 + 32);
  if (desc_ints > PIPE_RES_DESC_INTS) return 1;
  bool timed = false;
  if (!pipe_dry_run()) {
    int rc = timing_events(&a.ev_start, &a.ev_stop, &timed);
    if (rc) return rc;
  }
  const int rc = launch_resident_chain(a, st);
  if (timed && rc == PIPE_OK) g_events_used += 2;
  return rc;
}

extern "C" int pipe_resident_status(void* stream, int* status_out) {
  if (!status_out) return PIPE_EINVAL;
  CallScope scope(stream);
  *status_out = 0;
  if (t_ws->slot[WS_RES].ptr == nullptr) return PIPE_OK;
  uint32_t* status = reinterpret_cast<uint32_t*>((uint8_t*)t_ws->slot[WS_RES].ptr + RES_FLAGS_BYTES + RES_TAG_BYTES) + 16;
  PIPE_HIP(hipStreamSynchronize((hipStream_t)stream));
  uint32_t v = 0;
  PIPE_HIP(hipMemcpy(&v, status, sizeof(v), hipMemcpyDeviceToHost));
  if (v != 0) PIPE_HIP(hipMemset(status, 0, sizeof(v)));
  *status_out = (int)v;
  return PIPE_OK;
}

// s_h_host: nullptr, or the given scales of the members' hidden activations (HOST, one per member)
static int mlp_forward_impl(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                            const float* x_dev, int T, float s_x, const float* s_h_host, const int* split, int M,
                            const float* bias1_dev, const float* bias2_dev, float* h_dev,
                            float* y_dev, void* stream) {
  if (!l1 || !l2 || T < 0) return PIPE_EINVAL;
  if (l1->conv_C > 0 || l2->conv_C > 0) return PIPE_EINVAL;
  if (act != PIPE_ACT_GELU && act != PIPE_ACT_SILU_GATED) return PIPE_EINVAL;
  if (l1->K != l2->K) return PIPE_ESPLIT;
  const int H = l2->in;
  if (l1->out != (act == PIPE_ACT_SILU_GATED ? 2 * H : H)) return PIPE_ESHAPE;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(l1->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (s_h_host != nullptr)
    for (int m = 0; m < Mm; ++m)
      if (!(s_h_host[m] > 0.f)) return PIPE_EINVAL;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  const bool small = use_stream_kernel(l1, T);   // both layers have the same K
  ActBuffers b;
  rc = get_act_buffers(T, l1->in_pad, small, &b);
  if (rc) return rc;
  // hidden buffers
  const int T_pad = b.T_pad;
  float* h = h_dev ? h_dev : (float*)pipe_ws_get(WS_H, (size_t)Mm * T * H * sizeof(float));
  uint8_t* qh = (uint8_t*)pipe_ws_get(WS_QH, (size_t)Mm * T_pad * l2->in_pad);
  int32_t* rowsum_h = (int32_t*)pipe_ws_get(WS_ROWSUM_H, (size_t)Mm * T_pad * 4);
  if (!h || !qh || !rowsum_h) return pipe_ws_error();
  uint32_t* amax_h = b.amax + 16;
  float* scale_h = b.scale + 16;
  {
    // decode-sized batches: both layers in one resident launch
    const pipe_expansion* es[2] = {l1, l2};
    const bool gated = act == PIPE_ACT_SILU_GATED;
    if (small && resident_eligible(es, 2, T, Mm, x_dev, s_h_host != nullptr && s_x > 0.f) && (!gated || l1->n_rb % 2 == 0)) {
      ResidentLayerSpec ls[2] = {};
      ls[0].e = l1; ls[0].bias = bias1_dev; ls[0].out = h; ls[0].act = gated ? PIPE_ACT_NONE : PIPE_ACT_GELU; ls[0].gated = gated ? 1 : 0;
      ls[0].res_pre_act = 1;
      ls[1].e = l2; ls[1].bias = bias2_dev; ls[1].out = y_dev; ls[1].act = PIPE_ACT_NONE; ls[1].res_pre_act = 1;
      ls[1].s_in = s_h_host;
      rc = run_resident(ls, 2, x_dev, T, s_x, Mm, lo, hi, st);
      if (rc != 1) return rc;   // 1: does not fit the resident kernel, per-layer launches below
    }
  }
  // the tiled kernel pairs gate and up blocks in one workgroup and writes h directly; otherwise
  // the gated layer's raw outputs pass through a buffer and an element-wise launch
  const bool paired = act == PIPE_ACT_SILU_GATED && !small && l1->n_rb % 2 == 0;
  float* y1 = nullptr;
  if (act == PIPE_ACT_SILU_GATED && !paired) {
    y1 = (float*)pipe_ws_get(WS_Y1, (size_t)Mm * T * l1->out * sizeof(float));
    if (!y1) return pipe_ws_error();
  }
  if (!small) {
    if ((rc = ensure_tables(l1, Mm, lo, hi, paired ? 1 : 0)) != PIPE_OK) return rc;
    if ((rc = ensure_tables(l2, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  }
  if (pipe_dry_run()) return PIPE_OK;

  const bool fused = fuse_decode_quant(l1, T, x_dev, small, h, (size_t)Mm * T * H);
  if (!fused) {
    rc = quantize_input(x_dev, T, l1->in, l1->in_pad, s_x, b, small, nullptr, b.scale, st);
    if (rc) return rc;
  }
  // The members' max|h| slots are zero on entry: cleared when the workspace is allocated and,
  // after each use, by the layer-2 kernel that follows their last reader.  A call that failed
  // between the two leaves them dirty; then they are cleared by a launch of their own.
  if (t_ws->amax_h_dirty) {
    rc = launch_zero_u32(amax_h, 2 * PIPE_MAX_K, st);
    if (rc) return rc;
  }
  t_ws->amax_h_dirty = true;

  // layer 1: every member reads the same Q(x); outputs stay separate
  GemmArgs a{};
  a.e = l1; a.T = T; a.T_pad = T_pad; a.qx = b.qx; a.rowsum = b.rowsum; a.s_x = b.scale;
  a.bias = bias1_dev; a.reduce = 0; a.zero_after = b.amax;
  a.zero_big = reinterpret_cast<uint32_t*>(rowsum_h); a.zero_big_n = Mm * T_pad;   // the code sums of Q(h) start at zero
  if (fused) { a.x_f32 = x_dev; a.s_static = s_x; }
  fill_members(a, Mm, lo, hi);
  if (act == PIPE_ACT_GELU) {
    a.act = PIPE_ACT_GELU; a.y = h; a.amax_out = amax_h;
    rc = run_gemm(a, small, st);
    if (rc) return fail_after_reduction(rc, b, st);
  } else if (paired) {
    a.act = PIPE_ACT_SILU_GATED; a.y = h; a.amax_out = amax_h;
    rc = run_gemm(a, small, st);
    if (rc) return rc;
  } else {
    a.act = 0; a.y = y1; a.amax_out = nullptr;
    rc = run_gemm(a, small, st);
    if (rc) return rc;
    rc = launch_mlp_act(y1, Mm, T, H, act, h, amax_h, nullptr, st);
    if (rc) return rc;
  }
  // each member quantizes its own hidden activation with its own scale
  const bool one_launch = small && T <= PIPE_QUANT1_MAX_T;
  if (s_h_host != nullptr) {
    // given scales: one launch per member (the maxima taken above are not read; layer 2 clears them)
    for (int m = 0; m < Mm; ++m) {
      if (one_launch)
        rc = launch_quantize_small(h + (size_t)m * T * H, 0, 1, T, H, l2->in_pad, s_h_host[m], nullptr, qh + (size_t)m * T_pad * l2->in_pad, 0,
                                   rowsum_h + (size_t)m * T_pad, nullptr, scale_h + m, st);
      else
        rc = launch_quantize_act(h + (size_t)m * T * H, T, H, l2->in_pad, T_pad, s_h_host[m], nullptr, qh + (size_t)m * T_pad * l2->in_pad,
                                 rowsum_h + (size_t)m * T_pad, true, nullptr, scale_h + m, st);
      if (rc) return rc;
    }
  } else if (one_launch) {
    rc = launch_quantize_small(h, (int64_t)T * H, Mm, T, H, l2->in_pad, 0.f, amax_h, qh, (int64_t)T_pad * l2->in_pad,
                               rowsum_h, nullptr, scale_h, st);
    if (rc) return rc;
  }
  if (s_h_host == nullptr && !one_launch) {
    // the gated path's separate activation pass ran after layer 1: its code sums were cleared there too
    rc = launch_quantize_members(h, (int64_t)T * H, Mm, T, H, l2->in_pad, T_pad, amax_h, qh, (int64_t)T_pad * l2->in_pad,
                                 rowsum_h, true, scale_h, st);
    if (rc) return rc;
  }
  // layer 2: member m contracts its own input with its own orders; summed in the epilogue
  GemmArgs a2{};
  a2.e = l2; a2.T = T; a2.T_pad = T_pad; a2.qx = qh; a2.qx_mstride = (int64_t)T_pad * l2->in_pad;
  a2.rowsum = rowsum_h; a2.rowsum_mstride = T_pad; a2.s_x = scale_h; a2.sx_mstride = 1;
  a2.bias = bias2_dev; a2.reduce = 1; a2.act = 0; a2.y = y_dev;
  a2.zero_after = amax_h; a2.zero_n = Mm;
  fill_members(a2, Mm, lo, hi);
  rc = run_gemm(a2, small, st);
  if (rc == PIPE_OK) t_ws->amax_h_dirty = false;
  return rc;
}

// pipe_mlp_forward with asymmetric activation codes (Sec. 4.3) in front of both layers: the input over its own
// range, every member's hidden activation over that tensor's range (taken where it is produced) with its own
// zero point; the token-free terms of the zero points join the bias vectors.
extern "C" int pipe_mlp_forward_asymmetric(const pipe_expansion* l1, const pipe_expansion* l2, int act, const float* x_dev, int T,
                                           const int* split, int M, const float* bias1_dev, const float* bias2_dev,
                                           float* h_dev, float* y_dev, void* stream) {
  if (!l1 || !l2 || T < 0) return PIPE_EINVAL;
  if (l1->conv_C > 0 || l2->conv_C > 0) return PIPE_EINVAL;
  if (act != PIPE_ACT_GELU && act != PIPE_ACT_SILU_GATED) return PIPE_EINVAL;
  if (l1->K != l2->K) return PIPE_ESPLIT;
  const int H = l2->in;
  if (l1->out != (act == PIPE_ACT_SILU_GATED ? 2 * H : H)) return PIPE_ESHAPE;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(l1->K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (T == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  const int act_bits = (int)std::lround(std::log2((double)g_act_qmax_host + 1.0)) + 1;
  for (const pipe_expansion* e : {l1, l2})   // |Q - z| <= 2^a - 1: the exact accumulator must fit 32 bits
    if ((int64_t)((1 << act_bits) - 1) * ((1 << (e->qbits - 1)) - 1) * e->in >= ((int64_t)1 << 31)) return PIPE_ESHAPE;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  if ((rc = asym_prepare(l1, st)) != PIPE_OK || (rc = asym_prepare(l2, st)) != PIPE_OK) return rc;
  const bool small = use_stream_kernel(l1, T);
  ActBuffers b;
  rc = get_act_buffers(T, l1->in_pad, small, &b);
  if (rc) return rc;
  const int T_pad = b.T_pad;
  float* h = h_dev ? h_dev : (float*)pipe_ws_get(WS_H, (size_t)Mm * T * H * sizeof(float));
  uint8_t* qh = (uint8_t*)pipe_ws_get(WS_QH, (size_t)Mm * T_pad * l2->in_pad);
  int32_t* rowsum_h = (int32_t*)pipe_ws_get(WS_ROWSUM_H, (size_t)Mm * T_pad * 4);
  float* bias_m = (float*)pipe_ws_get(WS_ABIAS, (size_t)Mm * std::max(l1->out, l2->out) * sizeof(float));
  if (!h || !qh || !rowsum_h || !bias_m) return pipe_ws_error();
  const bool paired = act == PIPE_ACT_SILU_GATED && !small && l1->n_rb % 2 == 0;
  float* y1 = nullptr;
  if (act == PIPE_ACT_SILU_GATED && !paired) {
    y1 = (float*)pipe_ws_get(WS_Y1, (size_t)Mm * T * l1->out * sizeof(float));
    if (!y1) return pipe_ws_error();
  }
  if (!small) {
    if ((rc = ensure_tables(l1, Mm, lo, hi, paired ? 1 : 0)) != PIPE_OK) return rc;
    if ((rc = ensure_tables(l2, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  }
  if (pipe_dry_run()) return PIPE_OK;
  // slots as in pipe_chain_forward_asymmetric: the input's range and offset, the members' ranges (positive parts
  // [0, 16), negative parts [16, 32)), offsets and scales
  uint32_t* slots_x = b.amax + 64;
  int32_t* dz_x = reinterpret_cast<int32_t*>(b.amax + 66);
  uint32_t* rng = b.amax + 128;
  int32_t* dz_h = reinterpret_cast<int32_t*>(b.amax + 128 + 4 * PIPE_MAX_K);
  float* scale_h = b.scale + 16;
  if (t_ws->range_h_dirty) {
    rc = launch_zero_u32(rng, 4 * PIPE_MAX_K, st);
    if (rc) return rc;
  }
  t_ws->range_h_dirty = true;

  rc = launch_minmax(x_dev, (int64_t)T * l1->in, slots_x, st);
  if (rc) return rc;
  rc = launch_quantize_asym(x_dev, T, l1->in, l1->in_pad, T_pad, slots_x, slots_x + 1, act_bits, b.qx, b.rowsum, nullptr, b.scale, dz_x, st);
  if (rc == PIPE_OK)
    rc = launch_asym_bias_members(bias1_dev, l1->asym_P_dev, b.scale, 0, dz_x, 0, Mm, lo, hi, 0, bias_m, l1->out, slots_x, 2, st);
  if (rc) {
    (void)launch_zero_u32(slots_x, 2, st);
    return rc;
  }
  // layer 1: every member reads the same codes; its own offset vector; outputs stay separate
  GemmArgs a{};
  a.e = l1; a.T = T; a.T_pad = T_pad; a.qx = b.qx; a.rowsum = b.rowsum; a.s_x = b.scale;
  a.bias = bias_m; a.bias_mstride = l1->out; a.reduce = 0; a.zero_after = nullptr; a.zero_n = 0;
  fill_members(a, Mm, lo, hi);
  if (act == PIPE_ACT_GELU || paired) {
    a.act = act; a.y = h; a.amax_out = rng; a.amax_neg = rng + PIPE_MAX_K;
    rc = run_gemm(a, small, st);
    if (rc) return rc;
  } else {
    a.act = 0; a.y = y1;
    rc = run_gemm(a, small, st);
    if (rc) return rc;
    rc = launch_mlp_act(y1, Mm, T, H, act, h, rng, rng + PIPE_MAX_K, st);
    if (rc) return rc;
  }
  for (int m = 0; m < Mm; ++m) {
    rc = launch_quantize_asym(h + (size_t)m * T * H, T, H, l2->in_pad, T_pad, rng + m, rng + PIPE_MAX_K + m, act_bits,
                              qh + (size_t)m * T_pad * l2->in_pad, rowsum_h + (size_t)m * T_pad, nullptr, scale_h + m, dz_h + m, st);
    if (rc) return rc;
  }
  rc = launch_asym_bias_members(bias2_dev, l2->asym_P_dev, scale_h, 1, dz_h, 1, Mm, lo, hi, 1, bias_m, l2->out, nullptr, 0, st);
  if (rc) return rc;
  GemmArgs a2{};
  a2.e = l2; a2.T = T; a2.T_pad = T_pad; a2.qx = qh; a2.qx_mstride = (int64_t)T_pad * l2->in_pad;
  a2.rowsum = rowsum_h; a2.rowsum_mstride = T_pad; a2.s_x = scale_h; a2.sx_mstride = 1;
  a2.bias = bias_m; a2.reduce = 1; a2.act = 0; a2.y = y_dev;
  a2.zero_after = rng; a2.zero_n = 2 * PIPE_MAX_K;
  fill_members(a2, Mm, lo, hi);
  rc = run_gemm(a2, small, st);
  if (rc == PIPE_OK) t_ws->range_h_dirty = false;
  return rc;
}

extern "C" int pipe_mlp_forward(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                                const float* x_dev, int T, float s_x, const int* split, int M,
                                const float* bias1_dev, const float* bias2_dev, float* h_dev,
                                float* y_dev, void* stream) {
  return mlp_forward_impl(l1, l2, act, x_dev, T, s_x, nullptr, split, M, bias1_dev, bias2_dev, h_dev, y_dev, stream);
}

extern "C" int pipe_mlp_forward_given_scales(const pipe_expansion* l1, const pipe_expansion* l2, int act,
                                             const float* x_dev, int T, float s_x, const float* s_h_host, const int* split,
                                             int M, const float* bias1_dev, const float* bias2_dev, float* h_dev,
                                             float* y_dev, void* stream) {
  if (!(s_x > 0.f) || s_h_host == nullptr) return PIPE_EINVAL;
  return mlp_forward_impl(l1, l2, act, x_dev, T, s_x, s_h_host, split, M, bias1_dev, bias2_dev, h_dev, y_dev, stream);
}

extern "C" int pipe_prepare_mlp(const pipe_expansion* l1, const pipe_expansion* l2, int act, const int* split, int M,
                                int T_max, void* stream) {
  if (!l1 || !l2 || T_max < 1) return PIPE_EINVAL;
  DryScope dry;
  const float* fake_x = reinterpret_cast<const float*>(uintptr_t(256));
  float* fake_y = reinterpret_cast<float*>(uintptr_t(512));
  int rc = pipe_mlp_forward(l1, l2, act, fake_x, T_max, 1.f, split, M, nullptr, nullptr, nullptr, fake_y, stream);
  if (rc == PIPE_OK && T_max > PIPE_STREAM_MAX_T + 1)
    rc = pipe_mlp_forward(l1, l2, act, fake_x, PIPE_STREAM_MAX_T + 1, 1.f, split, M, nullptr, nullptr, nullptr, fake_y, stream);
  return rc;
}

// ------------------------------------------------------------------ member chains
// Tokens form an N x H x W grid (channels-last tensors); a fully-connected layer keeps the grid,
// a convolution layer maps it to its output grid.
// Tensors leaving layers 0..L-2 of a chain, [M, T_l, out_l] each.  Tensor l lives until its last
// reader: layer l+1, or a later layer whose skip reads it.  Those the caller did not give a buffer
// for share a pool of equal slabs.
static int chain_tensors(const pipe_chain_layer* layers, int L, int Mm, const std::vector<int64_t>& Tin,
                         float* const* acts_dev, std::vector<float*>* act_out) {
  std::vector<float*>& act = *act_out;
  act.assign(L > 1 ? L - 1 : 0, nullptr);
  std::vector<int> last(L, 0), slab(L, -1);
  size_t slab_floats = 0;
  for (int l = 0; l + 1 < L; ++l) {
    last[l] = l + 1;
    for (int j = l + 1; j < L; ++j)
      if (layers[j].skip_from == l + 1) last[l] = j;
    if (!(acts_dev && acts_dev[l])) slab_floats = std::max(slab_floats, (size_t)Mm * Tin[l + 1] * layers[l].e->out);
  }
  slab_floats = (slab_floats + 63) & ~(size_t)63;
  std::vector<int> busy_until;   // per slab: the last layer that reads its tensor
  for (int l = 0; l + 1 < L; ++l) {
    if (acts_dev && acts_dev[l]) continue;
    int sl = -1;
    for (size_t i = 0; i < busy_until.size(); ++i)
      if (busy_until[i] < l) { sl = (int)i; break; }   // its last reader ran before layer l writes
    if (sl < 0) { sl = (int)busy_until.size(); busy_until.push_back(0); }
    busy_until[sl] = last[l];
    slab[l] = sl;
  }
  float* pool = nullptr;
  if (!busy_until.empty()) {
    pool = (float*)pipe_ws_get(WS_CHAIN, busy_until.size() * slab_floats * sizeof(float));
    if (!pool) return pipe_ws_error();
  }
  for (int l = 0; l + 1 < L; ++l) act[l] = (acts_dev && acts_dev[l]) ? acts_dev[l] : pool + (size_t)slab[l] * slab_floats;
  return PIPE_OK;
}

static int chain_forward_grid(const pipe_chain_layer* layers, int L, const float* x_dev, int N, int H0, int W0,
                              float s_x, const int* split, int M, float* const* acts_dev, float* y_dev, void* stream) {
  if (!layers || L < 1 || N < 0 || H0 < 1 || W0 < 1) return PIPE_EINVAL;
  std::vector<int> Hin(L + 1), Win(L + 1), Cin(L);
  std::vector<int64_t> Tin(L + 1);
  Hin[0] = H0; Win[0] = W0; Tin[0] = (int64_t)N * H0 * W0;
  for (int l = 0; l < L; ++l) {
    const pipe_chain_layer& ly = layers[l];
    if (!ly.e || ly.e->conv_C > 0) return PIPE_EINVAL;
    if (ly.act != PIPE_ACT_NONE && ly.act != PIPE_ACT_RELU && ly.act != PIPE_ACT_GELU) return PIPE_EINVAL;
    if (ly.skip_from < -1 || ly.skip_from > l) return PIPE_EINVAL;
    if (ly.e->K != layers[0].e->K) return PIPE_ESPLIT;
    if (ly.kh < 0 || ly.kw < 0 || (ly.kh == 0) != (ly.kw == 0)) return PIPE_EINVAL;
    if (l > 0 && ly.s_in != nullptr)
      for (int m = 0; m < (split ? M : 1); ++m)
        if (!(ly.s_in[m] > 0.f)) return PIPE_EINVAL;   // given scales are positive
    if (ly.kh == 0) {
      Cin[l] = ly.e->in; Hin[l + 1] = Hin[l]; Win[l + 1] = Win[l];
    } else {
      if (ly.stride < 1 || ly.pad < 0 || ly.e->in % (ly.kh * ly.kw) != 0) return PIPE_ESHAPE;
      if (Hin[l] + 2 * ly.pad < ly.kh || Win[l] + 2 * ly.pad < ly.kw) return PIPE_ESHAPE;
      Cin[l] = ly.e->in / (ly.kh * ly.kw);
      Hin[l + 1] = (Hin[l] + 2 * ly.pad - ly.kh) / ly.stride + 1;
      Win[l + 1] = (Win[l] + 2 * ly.pad - ly.kw) / ly.stride + 1;
    }
    Tin[l + 1] = (int64_t)N * Hin[l + 1] * Win[l + 1];
    if (Tin[l + 1] > (int64_t)1 << 30) return PIPE_ESHAPE;
    if (l > 0 && Cin[l] != layers[l - 1].e->out) return PIPE_ESHAPE;
    // the tensor that entered layer j is [Tin_j, Cin_j]; a skip adds it to this layer's output
    if (ly.skip_from >= 0 && (Cin[ly.skip_from] != ly.e->out || Tin[ly.skip_from] != Tin[l + 1])) return PIPE_ESHAPE;
  }
  if (layers[L - 1].act != PIPE_ACT_NONE) return PIPE_EINVAL;
  const int K = layers[0].e->K;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (N == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  // per layer: the contraction's token count is the layer's output grid
  std::vector<char> small(L);
  std::vector<int> Tpad(L);
  int T_pad_max = 0;
  size_t qh_bytes = 0, q8_bytes = 0;
  for (int l = 0; l < L; ++l) {
    small[l] = use_stream_kernel(layers[l].e, (int)Tin[l + 1]);
    Tpad[l] = (int)round_up64(Tin[l + 1], small[l] ? 16 : TOK_TILE);
    T_pad_max = std::max(T_pad_max, Tpad[l]);
    if (l > 0) qh_bytes = std::max(qh_bytes, (size_t)Mm * Tpad[l] * layers[l].e->in_pad);
    if (layers[l].kh > 0) q8_bytes = std::max(q8_bytes, (size_t)Tin[l] * Cin[l]);
  }
  ActBuffers b;
  rc = get_act_buffers((int)Tin[1], layers[0].e->in_pad, small[0], &b);
  if (rc) return rc;

  std::vector<float*> act;
  rc = chain_tensors(layers, L, Mm, Tin, acts_dev, &act);
  if (rc) return rc;
  uint8_t* qh = nullptr;
  int32_t* rowsum_h = nullptr;
  int8_t* q8 = nullptr;
  if (L > 1) {
    qh = (uint8_t*)pipe_ws_get(WS_QH, qh_bytes);
    rowsum_h = (int32_t*)pipe_ws_get(WS_ROWSUM_H, (size_t)2 * Mm * T_pad_max * 4);
    if (!qh || !rowsum_h) return pipe_ws_error();
  }
  if (q8_bytes) {
    q8 = (int8_t*)pipe_ws_get(WS_Q8X, q8_bytes);
    if (!q8) return pipe_ws_error();
  }
  // code sums of the members' quantized inputs, two buffers used in turn: the quantizer of layer l
  // adds into buffer l & 1, which the contraction of layer l-1 cleared (it reads the other one)
  int32_t* rs_buf[2] = {rowsum_h, rowsum_h ? rowsum_h + (size_t)Mm * T_pad_max : nullptr};
  // max|tensor| per member, two sets used in turn: layer l writes set l & 1 in its epilogue, the
  // quantizer of layer l+1 reads it, and the contraction of layer l+1 clears it again
  uint32_t* amax_set[2] = {b.amax + 16, b.amax + 16 + PIPE_MAX_K};
  float* scale_h = b.scale + 16;
  {
    // decode-sized batches of fully-connected layers: the whole chain in one resident launch
    std::vector<const pipe_expansion*> es(L);
    bool fc = H0 == 1 && W0 == 1;
    bool given = s_x > 0.f;
    for (int l = 0; l < L; ++l) { es[l] = layers[l].e; fc = fc && layers[l].kh == 0 && small[l]; given = given && (l == 0 || layers[l].s_in != nullptr); }
    if (fc && resident_eligible(es.data(), L, (int)Tin[0], Mm, x_dev, given)) {
      const int T = (int)Tin[0];
      std::vector<ResidentLayerSpec> ls(L);
      for (int l = 0; l < L; ++l) {
        const pipe_chain_layer& ly = layers[l];
        ls[l] = ResidentLayerSpec{};
        ls[l].e = ly.e; ls[l].bias = ly.bias_dev; ls[l].out = l == L - 1 ? y_dev : act[l]; ls[l].act = ly.act;
        ls[l].res_pre_act = ly.skip_pre_act ? 1 : 0;
        ls[l].s_in = ly.s_in;
        if (ly.skip_from == 0) {
          ls[l].res = x_dev; ls[l].res_mstride = 0; ls[l].res_members = 1; ls[l].res_device = 0;
        } else if (ly.skip_from > 0) {
          ls[l].res = act[ly.skip_from - 1]; ls[l].res_mstride = (long long)T * ly.e->out; ls[l].res_members = Mm; ls[l].res_device = 1;
        }
      }
      rc = run_resident(ls.data(), L, x_dev, T, s_x, Mm, lo, hi, st);
      if (rc != 1) return rc;   // 1: does not fit the resident kernel, per-layer launches below
    }
  }
  for (int l = 0; l < L; ++l)
    if (!small[l] && (rc = ensure_tables(layers[l].e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  if (pipe_dry_run()) return PIPE_OK;
  if (t_ws->amax_h_dirty) {
    rc = launch_zero_u32(amax_set[0], 2 * PIPE_MAX_K, st);
    if (rc) return rc;
  }
  t_ws->amax_h_dirty = true;

  for (int l = 0; l < L; ++l) {
    const pipe_chain_layer& ly = layers[l];
    const pipe_expansion* e = ly.e;
    const bool last_layer = l == L - 1, conv = ly.kh > 0;
    const int T = (int)Tin[l + 1], T_pad = Tpad[l];
    GemmArgs a{};
    a.e = e; a.T = T; a.T_pad = T_pad;
    if (l == 0) {
      // every member reads the same Q(x)
      if (conv) {
        if (!(s_x > 0.f)) {
          rc = launch_absmax(x_dev, Tin[0] * Cin[0], b.amax, nullptr, 0, st);
          if (rc) return rc;
        }
        rc = launch_quantize_im2col(x_dev, N, Cin[0], Hin[0], Win[0], ly.kh, ly.kw, ly.stride, ly.pad, 1, Hin[1], Win[1],
                                    e->in_pad, T_pad, s_x, b.amax, q8, b.qx, b.rowsum, b.scale, st);
      } else {
        rc = quantize_input(x_dev, T, e->in, e->in_pad, s_x, b, small[0], nullptr, b.scale, st);
      }
      if (rc) return rc;
      a.qx = b.qx; a.rowsum = b.rowsum; a.s_x = b.scale; a.zero_after = b.amax;
    } else {
      // each member quantizes its own tensor with its own scale
      const float* src = act[l - 1];
      const int in = e->in;
      uint32_t* amax_in = amax_set[(l - 1) & 1];
      int32_t* rs_in = rs_buf[l & 1];
      const int64_t q_ms = (int64_t)T_pad * e->in_pad;
      const float* s_given = ly.s_in;   // given scales: no maximum was taken (the producing layer was told so)
      if (conv) {
        for (int m = 0; m < Mm; ++m) {
          rc = launch_quantize_im2col(src + (size_t)m * Tin[l] * Cin[l], N, Cin[l], Hin[l], Win[l], ly.kh, ly.kw, ly.stride,
                                      ly.pad, 1, Hin[l + 1], Win[l + 1], e->in_pad, T_pad, s_given ? s_given[m] : 0.f, amax_in + m, q8,
                                      qh + (size_t)m * q_ms, rs_in + (size_t)m * T_pad_max, scale_h + m, st);
          if (rc) return rc;
        }
      } else if (s_given != nullptr) {
        // one launch per member, each with its own given scale
        for (int m = 0; m < Mm; ++m) {
          if (small[l] && T <= PIPE_QUANT1_MAX_T && T_pad == T_pad_max)
            rc = launch_quantize_small(src + (size_t)m * T * in, 0, 1, T, in, e->in_pad, s_given[m], nullptr, qh + (size_t)m * q_ms, 0,
                                       rs_in + (size_t)m * T_pad_max, nullptr, scale_h + m, st);
          else
            rc = launch_quantize_act(src + (size_t)m * T * in, T, in, e->in_pad, T_pad, s_given[m], nullptr, qh + (size_t)m * q_ms,
                                     rs_in + (size_t)m * T_pad_max, true, nullptr, scale_h + m, st);
          if (rc) return rc;
        }
      } else if (small[l] && T <= PIPE_QUANT1_MAX_T && T_pad == T_pad_max) {
        rc = launch_quantize_small(src, (int64_t)T * in, Mm, T, in, e->in_pad, 0.f, amax_in, qh, q_ms, rs_in, nullptr, scale_h, st);
        if (rc) return rc;
      } else if (T_pad == T_pad_max) {
        rc = launch_quantize_members(src, (int64_t)T * in, Mm, T, in, e->in_pad, T_pad, amax_in, qh, q_ms, rs_in, true, scale_h, st);
        if (rc) return rc;
      } else {
        for (int m = 0; m < Mm; ++m) {
          rc = launch_quantize_act(src + (size_t)m * T * in, T, in, e->in_pad, T_pad, 0.f, amax_in + m, qh + (size_t)m * q_ms,
                                   rs_in + (size_t)m * T_pad_max, true, nullptr, scale_h + m, st);
          if (rc) return rc;
        }
      }
      a.qx = qh; a.qx_mstride = q_ms;
      a.rowsum = rs_in; a.rowsum_mstride = T_pad_max;
      a.s_x = scale_h; a.sx_mstride = 1;
      a.zero_after = amax_in; a.zero_n = Mm;
    }
    if (!last_layer && rs_buf[0]) { a.zero_big = reinterpret_cast<uint32_t*>(rs_buf[(l + 1) & 1]); a.zero_big_n = Mm * T_pad_max; }
    a.bias = ly.bias_dev;
    a.act = ly.act;
    if (ly.skip_from == 0) {
      a.res = x_dev; a.res_mstride = 0; a.res_members = 1;
    } else if (ly.skip_from > 0) {
      a.res = act[ly.skip_from - 1]; a.res_mstride = (int64_t)T * e->out; a.res_members = Mm;
    }
    a.res_pre_act = ly.skip_pre_act ? 1 : 0;
    if (last_layer) {
      a.reduce = 1; a.y = y_dev;
    } else {
      a.reduce = 0; a.y = act[l];
      a.amax_out = layers[l + 1].s_in != nullptr ? nullptr : amax_set[l & 1];   // nobody asks for the maximum of a tensor whose scale is given
    }
    fill_members(a, Mm, lo, hi);
    rc = run_gemm(a, small[l], st);
    if (rc) return rc;
  }
  // the last layer cleared the set it read; the other set was cleared one layer earlier
  t_ws->amax_h_dirty = false;
  return PIPE_OK;
}

extern "C" int pipe_chain_forward(const pipe_chain_layer* layers, int L, const float* x_dev, int T, float s_x,
                                  const int* split, int M, float* const* acts_dev, float* y_dev, void* stream) {
  if (!layers || L < 1 || T < 0) return PIPE_EINVAL;
  for (int l = 0; l < L; ++l)
    if (layers[l].kh != 0 || layers[l].kw != 0) return PIPE_EINVAL;   // convolution layers need the grid: pipe_chain_forward_conv
  return chain_forward_grid(layers, L, x_dev, T, 1, 1, s_x, split, M, acts_dev, y_dev, stream);
}

extern "C" int pipe_chain_forward_conv(const pipe_chain_layer* layers, int L, const float* x_dev, int N, int H, int W,
                                       float s_x, const int* split, int M, float* const* acts_dev, float* y_dev,
                                       void* stream) {
  return chain_forward_grid(layers, L, x_dev, N, H, W, s_x, split, M, acts_dev, y_dev, stream);
}

// Member chains with asymmetric activation codes (Sec. 4.3): the same driver as above for fully-connected
// layers, with the affine quantizer in front of every layer.  A hidden tensor's range comes from the
// epilogue that produced it (positive and negative part apart), every member quantizes its own tensor with
// its own scale and zero point, and the token-free term of the zero point joins the member's bias vector.
// Member chains under asymmetric activation codes, on a grid of tokens (fully-connected chains: T x 1 x 1).
// A convolution layer quantizes every element of its input once (per member, with the member's scale and zero
// point) and gathers the patches from those codes; a tap outside the image holds the code of the real value 0.
static int chain_forward_asym_grid(const pipe_chain_layer* layers, int L, const float* x_dev, int N, int H0, int W0,
                                   const int* split, int M, float* const* acts_dev, float* y_dev, void* stream) {
  if (!layers || L < 1 || N < 0 || H0 < 1 || W0 < 1) return PIPE_EINVAL;
  std::vector<int> Hin(L + 1), Win(L + 1), Cin(L);
  std::vector<int64_t> Tin(L + 1);
  Hin[0] = H0; Win[0] = W0; Tin[0] = (int64_t)N * H0 * W0;
  int out_max = 0;
  for (int l = 0; l < L; ++l) {
    const pipe_chain_layer& ly = layers[l];
    if (!ly.e || ly.e->conv_C > 0) return PIPE_EINVAL;
    if (ly.act != PIPE_ACT_NONE && ly.act != PIPE_ACT_RELU && ly.act != PIPE_ACT_GELU) return PIPE_EINVAL;
    if (ly.skip_from < -1 || ly.skip_from > l) return PIPE_EINVAL;
    if (ly.e->K != layers[0].e->K) return PIPE_ESPLIT;
    if (ly.kh < 0 || ly.kw < 0 || (ly.kh == 0) != (ly.kw == 0)) return PIPE_EINVAL;
    if (ly.kh == 0) {
      Cin[l] = ly.e->in; Hin[l + 1] = Hin[l]; Win[l + 1] = Win[l];
    } else {
      if (ly.stride < 1 || ly.pad < 0 || ly.e->in % (ly.kh * ly.kw) != 0) return PIPE_ESHAPE;
      if (Hin[l] + 2 * ly.pad < ly.kh || Win[l] + 2 * ly.pad < ly.kw) return PIPE_ESHAPE;
      Cin[l] = ly.e->in / (ly.kh * ly.kw);
      Hin[l + 1] = (Hin[l] + 2 * ly.pad - ly.kh) / ly.stride + 1;
      Win[l + 1] = (Win[l] + 2 * ly.pad - ly.kw) / ly.stride + 1;
    }
    Tin[l + 1] = (int64_t)N * Hin[l + 1] * Win[l + 1];
    if (Tin[l + 1] > (int64_t)1 << 30) return PIPE_ESHAPE;
    if (l > 0 && Cin[l] != layers[l - 1].e->out) return PIPE_ESHAPE;
    if (ly.skip_from >= 0 && (Cin[ly.skip_from] != ly.e->out || Tin[ly.skip_from] != Tin[l + 1])) return PIPE_ESHAPE;
    out_max = std::max(out_max, ly.e->out);
  }
  if (layers[L - 1].act != PIPE_ACT_NONE) return PIPE_EINVAL;
  const int K = layers[0].e->K;
  int lo[PIPE_MAX_K], hi[PIPE_MAX_K], Mm = 1;
  int rc = parse_split(K, split, M, lo, hi, &Mm);
  if (rc) return rc;
  if (N == 0) return PIPE_OK;
  if (!x_dev || !y_dev) return PIPE_EINVAL;
  const int act_bits = (int)std::lround(std::log2((double)g_act_qmax_host + 1.0)) + 1;
  for (int l = 0; l < L; ++l)   // |Q - z| <= 2^a - 1: the exact accumulator must fit 32 bits
    if ((int64_t)((1 << act_bits) - 1) * ((1 << (layers[l].e->qbits - 1)) - 1) * layers[l].e->in >= ((int64_t)1 << 31)) return PIPE_ESHAPE;
  hipStream_t st = (hipStream_t)stream;
  CallScope scope(stream);
  for (int l = 0; l < L; ++l)
    if ((rc = asym_prepare(layers[l].e, st)) != PIPE_OK) return rc;
  // per layer: the contraction's token count is the layer's output grid; the members' code sums keep one stride
  std::vector<char> small(L);
  std::vector<int> Tpad(L);
  int T_pad_max = 0;
  size_t qh_bytes = 0, q8_bytes = 0;
  for (int l = 0; l < L; ++l) {
    small[l] = use_stream_kernel(layers[l].e, (int)Tin[l + 1]);
    Tpad[l] = (int)round_up64(Tin[l + 1], small[l] ? 16 : TOK_TILE);
    T_pad_max = std::max(T_pad_max, Tpad[l]);
    if (l > 0) qh_bytes = std::max(qh_bytes, (size_t)Mm * Tpad[l] * layers[l].e->in_pad);
    if (layers[l].kh > 0) q8_bytes = std::max(q8_bytes, (size_t)Tin[l] * Cin[l]);
  }
  ActBuffers b;
  rc = get_act_buffers(Tpad[0], layers[0].e->in_pad, false, &b);   // Tpad[0] is a multiple of what its kernel needs
  if (rc) return rc;
  std::vector<float*> act;
  rc = chain_tensors(layers, L, Mm, Tin, acts_dev, &act);
  if (rc) return rc;
  uint8_t* qh = nullptr;
  int32_t* rowsum_h = nullptr;
  int8_t* q8 = nullptr;
  if (L > 1) {
    qh = (uint8_t*)pipe_ws_get(WS_QH, qh_bytes);
    rowsum_h = (int32_t*)pipe_ws_get(WS_ROWSUM_H, (size_t)Mm * T_pad_max * 4);
    if (!qh || !rowsum_h) return pipe_ws_error();
  }
  if (q8_bytes) {
    q8 = (int8_t*)pipe_ws_get(WS_Q8X, q8_bytes);
    if (!q8) return pipe_ws_error();
  }
  float* bias_m = (float*)pipe_ws_get(WS_ABIAS, (size_t)Mm * out_max * sizeof(float));
  if (!bias_m) return pipe_ws_error();
  for (int l = 0; l < L; ++l)
    if (!small[l] && (rc = ensure_tables(layers[l].e, Mm, lo, hi, 0)) != PIPE_OK) return rc;
  if (pipe_dry_run()) return PIPE_OK;
  // the input's range slots and zero-point offset, then per member and set the hidden tensors' ranges
  // (positive parts [0, 16), negative parts [16, 32) of a set; layer l's epilogue raises set l & 1, the
  // quantizers of layer l+1 read it and layer l+1's contraction clears it), offsets and scales
  uint32_t* slots_x = b.amax + 64;
  int32_t* dz_x = reinterpret_cast<int32_t*>(b.amax + 66);
  uint32_t* rng[2] = {b.amax + 128, b.amax + 128 + 2 * PIPE_MAX_K};
  int32_t* dz_h = reinterpret_cast<int32_t*>(b.amax + 128 + 4 * PIPE_MAX_K);
  float* scale_h = b.scale + 16;
  if (t_ws->range_h_dirty) {
    rc = launch_zero_u32(rng[0], 4 * PIPE_MAX_K, st);
    if (rc) return rc;
  }
  t_ws->range_h_dirty = true;

  for (int l = 0; l < L; ++l) {
    const pipe_chain_layer& ly = layers[l];
    const pipe_expansion* e = ly.e;
    const bool last_layer = l == L - 1, conv = ly.kh > 0;
    const int T = (int)Tin[l + 1], T_pad = Tpad[l];
    GemmArgs a{};
    a.e = e; a.T = T; a.T_pad = T_pad;
    if (l == 0) {
      rc = launch_minmax(x_dev, Tin[0] * Cin[0], slots_x, st);
      if (rc) return rc;
      if (conv)
        rc = launch_quantize_im2col_asym(x_dev, N, Cin[0], Hin[0], Win[0], ly.kh, ly.kw, ly.stride, ly.pad, 1, Hin[1], Win[1], e->in_pad,
                                         T_pad, slots_x, slots_x + 1, act_bits, q8, b.qx, b.rowsum, b.scale, dz_x, st);
      else
        rc = launch_quantize_asym(x_dev, T, e->in, e->in_pad, T_pad, slots_x, slots_x + 1, act_bits, b.qx, b.rowsum, nullptr,
                                  b.scale, dz_x, st);
      if (rc == PIPE_OK)
        rc = launch_asym_bias_members(ly.bias_dev, e->asym_P_dev, b.scale, 0, dz_x, 0, Mm, lo, hi, last_layer ? 1 : 0, bias_m,
                                      e->out, slots_x, 2, st);
      if (rc) {
        (void)launch_zero_u32(slots_x, 2, st);   // the raised range slots: the kernel that clears them did not run
        return rc;
      }
      a.qx = b.qx; a.rowsum = b.rowsum; a.s_x = b.scale;
      a.zero_after = nullptr; a.zero_n = 0;
    } else {
      const float* src = act[l - 1];
      const uint32_t* r_in = rng[(l - 1) & 1];
      const int64_t q_ms = (int64_t)T_pad * e->in_pad;
      for (int m = 0; m < Mm; ++m) {
        const float* src_m = src + (size_t)m * Tin[l] * Cin[l];
        if (conv)
          rc = launch_quantize_im2col_asym(src_m, N, Cin[l], Hin[l], Win[l], ly.kh, ly.kw, ly.stride, ly.pad, 1, Hin[l + 1], Win[l + 1],
                                           e->in_pad, T_pad, r_in + m, r_in + PIPE_MAX_K + m, act_bits, q8, qh + (size_t)m * q_ms,
                                           rowsum_h + (size_t)m * T_pad_max, scale_h + m, dz_h + m, st);
        else
          rc = launch_quantize_asym(src_m, T, e->in, e->in_pad, T_pad, r_in + m, r_in + PIPE_MAX_K + m, act_bits,
                                    qh + (size_t)m * q_ms, rowsum_h + (size_t)m * T_pad_max, nullptr, scale_h + m, dz_h + m, st);
        if (rc) return rc;
      }
      rc = launch_asym_bias_members(ly.bias_dev, e->asym_P_dev, scale_h, 1, dz_h, 1, Mm, lo, hi, last_layer ? 1 : 0, bias_m, e->out,
                                    nullptr, 0, st);
      if (rc) return rc;
      a.qx = qh; a.qx_mstride = q_ms;
      a.rowsum = rowsum_h; a.rowsum_mstride = T_pad_max;
      a.s_x = scale_h; a.sx_mstride = 1;
      a.zero_after = rng[(l - 1) & 1]; a.zero_n = 2 * PIPE_MAX_K;
    }
    a.bias = bias_m;
    a.bias_mstride = last_layer ? 0 : e->out;
    a.act = ly.act;
    if (ly.skip_from == 0) {
      a.res = x_dev; a.res_mstride = 0; a.res_members = 1;
    } else if (ly.skip_from > 0) {
      a.res = act[ly.skip_from - 1]; a.res_mstride = (int64_t)T * e->out; a.res_members = Mm;
    }
    a.res_pre_act = ly.skip_pre_act ? 1 : 0;
    if (last_layer) {
      a.reduce = 1; a.y = y_dev;
    } else {
      a.reduce = 0; a.y = act[l]; a.amax_out = rng[l & 1]; a.amax_neg = rng[l & 1] + PIPE_MAX_K;
    }
    fill_members(a, Mm, lo, hi);
    rc = run_gemm(a, small[l], st);
    if (rc) return rc;
  }
  t_ws->range_h_dirty = false;
  return PIPE_OK;
}

extern "C" int pipe_chain_forward_asymmetric(const pipe_chain_layer* layers, int L, const float* x_dev, int T,
                                             const int* split, int M, float* const* acts_dev, float* y_dev, void* stream) {
  if (!layers || L < 1 || T < 0) return PIPE_EINVAL;
  for (int l = 0; l < L; ++l)
    if (layers[l].kh != 0 || layers[l].kw != 0) return PIPE_EINVAL;
  return chain_forward_asym_grid(layers, L, x_dev, T, 1, 1, split, M, acts_dev, y_dev, stream);
}

extern "C" int pipe_chain_forward_conv_asymmetric(const pipe_chain_layer* layers, int L, const float* x_dev, int N, int H, int W,
                                                  const int* split, int M, float* const* acts_dev, float* y_dev, void* stream) {
  return chain_forward_asym_grid(layers, L, x_dev, N, H, W, split, M, acts_dev, y_dev, stream);
}

extern "C" int pipe_prepare_chain(const pipe_chain_layer* layers, int L, int N, int H, int W, const int* split, int M,
                                  void* stream) {
  if (N < 1) return PIPE_EINVAL;
  DryScope dry;
  const float* fake_x = reinterpret_cast<const float*>(uintptr_t(256));
  float* fake_y = reinterpret_cast<float*>(uintptr_t(512));
  return chain_forward_grid(layers, L, fake_x, N, H, W, 1.f, split, M, nullptr, fake_y, stream);
}
