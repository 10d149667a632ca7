// Context of one model instance: parameters, fixed-region layout, plan and program.
#pragma once
#include <hip/hip_runtime.h>

#include <memory>
#include <string>
#include <vector>

#include "host_optim.h"
#include "karma.h"
#include "planner.h"

namespace karma {

enum RecordKind {
  REC_LINEAR_RELU = 1, REC_EMBED = 2, REC_BLOCK = 3, REC_CNN_STEM = 4, REC_CNN_BLOCK = 5, REC_ATTN = 6, REC_FFN = 7,
  REC_WRN_STEM = 8, REC_WRN_BLOCK = 9,
  REC_LOSS_MSE = 10, REC_LOSS_LMHEAD = 11, REC_LOSS_CNN_HEAD = 12, REC_LOSS_WRN_HEAD = 13,
  REC_UNET_DOWN = 14, REC_UNET_UP = 15, REC_LOSS_UNET_HEAD = 16
};

struct Param {
  uint64_t n = 0;
  bool dev_bf16 = false;    // device copy of the weight: bf16 (else fp32)
  bool grad_bf16 = false;   // device gradient: bf16 (else fp32)
  uint64_t w_off = 0, g_off = 0;   // byte offsets in the fixed region (resident weights)
  uint64_t w_rel = 0, g_rel = 0;   // byte offsets in the record's streamed weight / gradient buffer
  // updated on the device: fp32 master weights and optimiser state live in the fixed region at these offsets
  bool dev_opt = false;
  uint64_t dmaster_off = 0, dm_off = 0, dv_off = 0;
  std::vector<float> master, m, v; // host fp32 master copy and optimiser state
  void* stage_g = nullptr;         // pinned: gradient as it arrives from the device
  void* stage_w = nullptr;         // pinned: new weight in device format
  std::vector<hipEvent_t> chunk_ev; // gradient chunk k has landed on the host
  uint64_t w_bytes() const { return n * (dev_bf16 ? 2 : 4); }
  uint64_t g_bytes() const { return n * (grad_bf16 ? 2 : 4); }
};

// Large tensors cross the link and the optimiser in chunks so that gradient D2H, host update
// and weight H2D of one tensor overlap (this matters for the record that finishes last).
constexpr uint64_t PARAM_CHUNK = 4ull << 20;   // elements
// Records whose gradients are at most this many bytes (a convolutional block: a dozen tensors, most of them
// batch-norm vectors) cross the link whole; larger ones tensor by tensor in chunks, so that copy and update overlap.
constexpr uint64_t WHOLE_RECORD_BYTES = 4ull << 20;

struct Record {
  int kind = 0;
  std::vector<Param> p;
  uint64_t out_bytes = 0, sav_bytes = 0, ws_bytes = 0;   // from shapes
  // Streamed weights (Sec. III-G: a swapped block carries its weights): the device copy
  // lives in pinned host memory, one contiguous buffer per record, and visits the arena
  // only around the record's ops; the gradients take the opposite way after its backward.
  bool streamed = false;
  uint64_t w_total = 0, g_total = 0;     // bytes of the two buffers (parameters 256-B aligned)
  char* stage_w_all = nullptr;           // pinned; Param::stage_w point into it
  char* stage_g_all = nullptr;           // pinned; Param::stage_g point into it
  uint64_t shared_bytes = 0;             // leading part of both buffers: tensors whose gradient has the weight's type
  // Resident weights: the record's weights lie contiguously in the fixed region ([w_base, w_base + w_span)), its
  // gradients behind them ([g_base, g_base + g_span)), and the pinned buffers mirror the two spans, so that a
  // record of many small tensors crosses the link with one copy each way (whole_copies) instead of one per tensor
  uint64_t w_base = 0, w_span = 0, g_base = 0, g_span = 0;
  bool whole_copies = false;
  hipEvent_t grads_ev = nullptr;         // whole_copies: the record's gradients have landed on the host
  bool shared_staging = false;           // that part of the gradients lands in stage_w_all; stage_g_all holds the rest
};

// One op of the executable schedule; offsets are relative to the activation region,
// -1 = none, -2 = the step input in the fixed region.
struct ProgOp {
  char kind;
  uint32_t layer;
  int64_t x = -1, s = -1, out = -1, dy = -1, dx = -1, ws = -1;
  int64_t w = -1, g = -1;         // streamed weights / their gradients (F, R, B, W, G ops)
  std::vector<uint32_t> waits;
  bool record = false;
  int stream = 0;                 // 0 compute, 1 h2d, 2 d2h
  int64_t host_x = -1, host_s = -1;   // offsets in the pinned swap pool
  uint64_t x_bytes = 0, s_bytes = 0;  // bytes moved by a swap op
  // Connections between non-consecutive records (Sec. III-F.3)
  std::vector<int64_t> rx;            // F, R, B of a reader: the inputs of other records it reads again, ascending
  std::vector<int64_t> rdx;           // B of a reader: where it leaves its gradient for each of them ...
  std::vector<uint8_t> rdx_first;     // ... writing it (1: the first reader to run) or adding to it (0)
  int64_t hold = -1;                  // B of a record whose input was read again: the readers' gradient, added to dx
  uint64_t hold_elems = 0;            // elements of that tensor
};

struct Ctx {
  karma_model_desc desc{};
  karma_config cfg{};
  char* arena = nullptr;
  uint64_t arena_bytes = 0;
  hipStream_t st[3] = {nullptr, nullptr, nullptr};   // compute, h2d, d2h
  std::vector<Record> rec;       // plannable records followed by the loss record
  std::vector<karma_skip> skips; // connections between non-consecutive records (the model's; empty for most)
  uint32_t L = 0;                // number of plannable records
  uint64_t fixed_bytes = 0;
  uint64_t in_off = 0, lab_off = 0, loss_off = 0, misc_off = 0;   // fixed-region offsets
  uint64_t in_bytes = 0, lab_bytes = 0, misc_bytes = 0;
  void* stage_in = nullptr;      // pinned staging of inputs, labels, loss
  void* stage_lab = nullptr;
  float* stage_loss = nullptr;
  void* stage_misc = nullptr;

  std::vector<karma_layer_cost> cost;
  karma_loss_cost loss_cost{};
  karma_link link{};
  bool have_times = false;

  bool planned = false;
  bool inputs_resident = false;           // the fixed region and the staging buffers hold a caller's batch
  uint64_t budget = 0;
  std::vector<uint8_t> actions;
  std::vector<uint8_t> keepw;             // per record: streamed weights stay from F_i to B_i
  std::vector<karma_op> ops;
  std::vector<ProgOp> prog;
  karma_plan_summary summary{};
  std::vector<hipEvent_t> ev, ev_begin;   // per op: end event, begin event (profiling)
  std::vector<float> op_ms;               // per-op durations of the last profiled step
  std::vector<float> op_start_ms;         // and when each began on its stream, from the first op's begin
  char* swap_pool = nullptr;              // pinned host memory for swapped tensors
  uint64_t swap_pool_bytes = 0;

  // per-launch timing of the GEMM kernel (KARMA_STEP_KERNEL_TIMES)
  bool ktime = false;
  uint64_t ktime_steps = 0;               // steps run with kernel timing so far (rotates which launches are sampled)
  std::vector<hipEvent_t> kev;            // event pool, two per launch
  size_t kev_used = 0;
  std::vector<double> kflops;             // flops of launch j (events 2j, 2j+1)
  uint64_t gemm_launches = 0;
  double gemm_ms = 0, gemm_flops = 0;     // totals of the last step run with the flag

  uint32_t n_segments = 0;                // GPT: distinct token ids of the current step
  std::unique_ptr<HostPool> pool;
  uint64_t step_no = 0;
  bool applying = false;                  // the step being issued applies the optimiser
  // Host updates a step left for later (Sec. III-G, stage 5 overlapped with the next iteration): per record
  // the step number its update belongs to, 0 = none.  The gradients are already in pinned host memory.
  std::vector<uint64_t> pending_update;
  std::vector<int64_t> update_ns;   // per record: duration of its last host update (0 = none yet)
  hipEvent_t weights_uploaded = nullptr;  // recorded on the H2D stream after a late update's weight copies
  hipEvent_t program_h2d_done = nullptr;  // recorded on the H2D stream behind the last copy of a step's program
  karma_step_stats stats{};
  std::string err;

  char* fixed_ptr(uint64_t off) const { return arena + off; }
  char* act_ptr(int64_t off) const { return off < 0 ? nullptr : arena + fixed_bytes + off; }
  void* w_ptr(uint32_t r, uint32_t t) const { return arena + rec[r].p[t].w_off; }
  void* g_ptr(uint32_t r, uint32_t t) const { return arena + rec[r].p[t].g_off; }
  // weights / gradients of a record's tensor as an op sees them: inside the op's streamed
  // buffers when the record is streamed, in the fixed region otherwise
  void* w_ptr(uint32_t r, uint32_t t, const void* w_base) const {
    return rec[r].streamed ? (char*)w_base + rec[r].p[t].w_rel : arena + rec[r].p[t].w_off;
  }
  void* g_ptr(uint32_t r, uint32_t t, void* g_base) const {
    return rec[r].streamed ? (char*)g_base + rec[r].p[t].g_rel : arena + rec[r].p[t].g_off;
  }
};

#define KARMA_HIP(ctx, call)                                                                  \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess) {                                                                   \
      (ctx)->err = std::string(#call) + ": " + hipGetErrorString(e_);                         \
      return KARMA_E_HIP;                                                                     \
    }                                                                                         \
  } while (0)

// Pointers handed to a layer op.
struct LayerIO {
  const void* x = nullptr;   // layer input
  void* out = nullptr;       // layer output (may be null in a recompute whose output is not needed)
  void* sav = nullptr;       // internals
  void* ws = nullptr;        // workspace
  const void* dy = nullptr;  // gradient w.r.t. the output
  void* dx = nullptr;        // gradient w.r.t. the input (null for record 0)
  const void* w = nullptr;   // streamed weights of the record (null when resident)
  void* g = nullptr;         // buffer for the gradients of streamed weights (backward only)
  // inputs of other records that this one reads again (Sec. III-F.3), ascending by record; backward: where the
  // gradient with respect to each goes, and whether this op writes it or adds to what is there
  static constexpr int MAX_SKIPS = 4;
  int n_skips = 0;
  const void* skip_x[MAX_SKIPS] = {nullptr, nullptr, nullptr, nullptr};
  void* skip_dx[MAX_SKIPS] = {nullptr, nullptr, nullptr, nullptr};
  bool skip_dx_first[MAX_SKIPS] = {false, false, false, false};
};

// Model-specific pieces (layers_mlp.cpp, layers_gpt.cpp)
int model_build_records(Ctx& c);                         // fills rec[], sizes, in/lab/misc bytes
int model_prepare_step(Ctx& c, const void* in, const void* lab);   // inputs and labels into the staging buffers
int model_prepare_late(Ctx& c);   // host work only backward needs (runs while the GPU is busy with forward); fills stage_misc
int layer_forward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int layer_backward(Ctx& c, uint32_t i, const LayerIO& io, hipStream_t s);
int loss_op(Ctx& c, const LayerIO& io, hipStream_t s);   // x -> loss (fixed region) and dx; accumulates its own parameter gradients

// records, fixed-region layout and byte fields of the cost records from the description alone (executor.cpp)
int derive_layout(Ctx& c);

}  // namespace karma
