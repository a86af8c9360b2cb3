// Structures and constants shared by the host API and the gfx950 kernels.
#pragma once
#include <stdint.h>

namespace triaccel {

// Work decomposition: every tensor is cut into chunks of kChunk elements; a chunk is what one
// 256-thread workgroup (4 wavefronts of 64) streams per iteration: 4 rows of 256 lanes x 4
// consecutive elements, i.e. four coalesced 128-bit loads per lane and array.
constexpr int kThreads = 256;
constexpr int kVec = 4;
constexpr int kRows = 4;
constexpr int kRowElems = kThreads * kVec;   // 1024
constexpr int kChunk = kRowElems * kRows;    // 4096
constexpr int kWave = 64;
constexpr int kFinishThreads = 1024;          // workgroup of the per-tensor threshold-resolution kernel
// Sets below this many chunks (67 M parameters) are bound by the number of dependent launches, not
// by memory bandwidth: for them the step makes fewer, longer launches.
constexpr uint32_t kLaunchBoundChunks = 16384;

// Radix-select parameters: magnitudes are 31-bit keys (sign bit cleared).
constexpr int kHistBins = 2048;
constexpr int kHistBits = 11;
constexpr uint32_t kFullShift = 20;          // 2048 bins of 2^20 keys cover all 2^31 keys
constexpr uint32_t kFirstShift = 13;         // first window without a prediction: 2048 bins of 2^13 keys = the two
                                             // octaves below the largest key
constexpr uint32_t kMinPredShift = 6;        // finest predicted window: 2048 bins of 64 keys
constexpr uint32_t kUnknownPredErr = 1u << 16;  // assumed prediction error (keys) before any is measured
constexpr uint32_t kCandCap = 262144;        // keys a tensor may list in total (entries)
constexpr uint32_t kListAllMax = 8192;       // tensors up to this size list every non-zero key (no prediction)
constexpr int kFinishRegs = 8;               // listed keys per thread the finish kernel can hold in registers
constexpr uint32_t kCandLists = 64;          // sub-lists per tensor (plus one overflow list)
constexpr uint32_t kCandCounterStride = 32;  // words between list counters: one 128-byte line each

enum SelMode : uint32_t {
  kSelHist = 0,   // a histogram over the window is (being) accumulated; the scan decides what next
  kSelCand = 1,   // theta lies in [rng_lo, rng_hi): few enough keys there to list them
  kSelExact = 2,  // theta is known exactly
};

struct Hyper {
  float beta_var, beta_curv, tau_low, tau_high, tau_curv, alpha;
  uint32_t sparsity_ppm;
  float momentum, weight_decay;
  int32_t ctrl_interval;
  float scale_backoff, scale_growth;
  int32_t growth_interval;
  int32_t lambda_source;  // 0: largest kept |h_i|; 1: latched power-iteration value
  int32_t elementwise;    // 1: step size scaled per element by the masked |h_i|
  uint32_t topk_abs;      // > 0: entries kept per layer (instead of the fraction sparsity_ppm)
};

// Per-step scalars handed to the kernels.
struct StepScalars {
  float lr;
  float loss_scale;
  float inv_scale;   // 1.0f / loss_scale, one fp32 division on the host
  uint32_t pad_;
  uint64_t step_id;  // 1-based count of triaccel_step calls; the epoch of the skip / overflow flags
};

// How a kernel receives them: by value (ordinary launch), or from device memory when `dev` is set
// (a replayed graph, whose kernel arguments are frozen at capture).
struct StepArg {
  StepScalars value;
  const StepScalars* dev;
};

// Device table, one entry per tensor; re-uploaded when a pointer changes.
struct TensorDesc {
  void* param;
  const void* grad;
  const float* z;
  const float* hz;
  float* curv;
  float* mom;
  uint32_t* mask;
  int64_t numel;
  uint32_t first_chunk;  // index of the tensor's first chunk in the global chunk list
  uint32_t n_chunks;
  int32_t grad_dtype;
  int32_t has_probe;
  uint64_t cand_offset;  // first entry of the tensor's candidate lists in the pool
  uint32_t cand_cap;     // min(numel, kCandCap): capacity of the overflow list
  uint32_t sub_cap;      // capacity of each of the kCandLists sub-lists: ceil(cand_cap / kCandLists)
  uint32_t list_all;     // numel <= kListAllMax: every non-zero key is listed, no prediction
  uint32_t pad_;
};

// Per-layer device state.  The leading part mirrors triaccel_layer_info.
struct LayerDev {
  uint64_t found_epoch;    // step_id at which a non-finite gradient element was last seen
  // reported
  float mean, var, v, theta;
  uint32_t nnz;
  float lambda, lambda_ctrl, eta;
  int32_t code, prev_code;
  uint32_t found_inf, curv_nonfinite;
  uint32_t sel_passes;     // passes over h beyond the EMA pass that the last probed step needed
  uint32_t sel_listed;     // keys the EMA kernel listed at the last probed step
  uint32_t sel_outcome;    // how the band check of the last probed step ended (see select_begin)
  float lambda_power;      // max_j |Rayleigh quotient| latched by the power iteration (Sec. 3.2)
  // bookkeeping
  uint32_t applied_steps;  // steps that were not skipped
  uint32_t probes_seen;
  // threshold selection
  uint32_t theta_key;      // |theta| bit pattern (scratch while a step selects, then the result)
  uint32_t theta_key_last; // theta of the previous probed step
  uint32_t theta_key_last2;// theta of the probed step before that
  uint32_t n_theta;        // how many thresholds are known (0, 1, 2 = two or more)
  float var_hold;          // running mean squared error (keys^2) of predicting "same as last step"
  float var_ext;           // same for the damped extrapolation (pred_ext_key)
  uint32_t pred_ext_key;   // threshold the damped extrapolation expects at the next probed step (0 = none)
  uint32_t band_lo, band_hi;  // keys in [band_lo, band_hi) are listed by the EMA kernel
  uint32_t use_band;       // the EMA kernel writes the provisional mask and lists the band
  uint32_t mask_done;      // the mask needs no separate pass this step
  uint32_t window_missed;  // the predicted window did not contain theta this step
  uint32_t mode;           // SelMode
  uint32_t win_lo, win_shift, win_bins;  // histogram window (fallback passes): bin = (key - win_lo) >> win_shift
  uint32_t win_hi;         // keys in [win_lo, win_hi) are counted; win_hi <= win_lo + (win_bins << win_shift)
  uint32_t predicted;      // the window was centred on the previous theta
  uint32_t passes;         // scans done in this step (0 = the first histogram has not been scanned yet)
  uint32_t k_rem;          // rank still to resolve inside [rng_lo, rng_hi) (1 = largest)
  uint32_t above;          // non-zero keys known to lie above the window / range
  uint32_t rng_lo, rng_hi; // candidate range (kSelCand)
  uint32_t sel_count;      // keys equal to theta (kSelExact) or inside the range (kSelCand)
  uint32_t nonzero;        // number of non-zero keys
  uint32_t dens_count, dens_width;  // key density near theta: dens_count keys per dens_width keys
  uint32_t count_above;    // the next histogram pass must count the keys above its window
  uint32_t hist_arrived;   // chunks whose keys are in the histogram of the pass under way (cleared by the scan)
  // accumulators filled by atomics during a step and cleared by the kernel that consumes them
  uint32_t acc_above, acc_maxkey, acc_nonfinite;
};

// Small global record (device), copied to pinned host memory at the end of a step.
struct GlobalDev {
  uint64_t skip_epoch;     // == step_id when the step must be skipped
  int32_t good_steps;      // consecutive applied steps since the last loss-scale change
  uint32_t trans_count[2]; // number of tensors whose storage size changes (double-buffered by step parity)
  uint32_t hist_pending[2];// tensors still in histogram mode this step (same double buffering)
  uint32_t mask_pending[2];// tensors whose mask the EMA kernel did not settle this step
  // result record
  int32_t res_skipped;
  float res_next_scale;
  uint32_t pad_;
  uint64_t res_step_id;
};

struct ChunkRef {
  uint32_t tensor;
  uint32_t index;  // chunk number inside the tensor
};

struct Candidate {
  uint32_t idx;
  uint32_t key;
};

struct EmaPartial {
  uint32_t above;      // keys at or above the band
  uint32_t zeros;      // zero keys
  uint32_t maxkey;     // largest key
  uint32_t nonfinite;  // a probe sample of the chunk was non-finite
};

struct StatPartial {
  double mean;
  double m2;
};

}  // namespace triaccel
