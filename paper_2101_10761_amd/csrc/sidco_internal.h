// Internal declarations shared by the kernels and the C-ABI layer of the SIDCo library.
#ifndef SIDCO_INTERNAL_H
#define SIDCO_INTERNAL_H

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sidco.h"

namespace sidco {

constexpr int kBlock = 512;                       // threads per block: 8 wave64
constexpr int kWavesPerBlock = kBlock / 64;
constexpr int kTile = 256;                        // elements per wave step: 64 lanes x float4
constexpr int kMaxBlocks = 512;                   // 2 blocks per CU on 256 CUs
constexpr int kMaxWaves = kMaxBlocks * kWavesPerBlock;
// A non-final stage whose source is still the dense vector writes survivor lists only if the expected
// fraction of the vector that goes into them is at most this; otherwise it only counts and sums, and
// the next stage scans the dense vector again (4 B/element read, against 16 B per list entry written
// + read, writes being the dearer half).
constexpr double kMaterializeBelow = 0.16;
// Default position of a dense stage's candidate threshold between this stage's target ratio and the
// next one's, on the log scale: log(1/ratio_w) = L_m + kSpeculation * L_{m+1}.  At 0.5 the candidate
// lists serve the next stage as long as the mean excess over eta_m is at least about half of what the
// fitted law predicts (a Gaussian tail under an exponential fit still passes).
constexpr double kSpeculation = 0.5;
// A call that repeats the previous call's shape on the device (same d, law and ratios: the next
// training iteration) starts from where the previous call's next threshold really fell on that scale,
// minus this margin, and never above kHintMax: gradients change slowly from one iteration to the
// next, so the candidate lists shrink to a little more than the next stage's exceedances.
constexpr float kHintMargin = 0.1f;
constexpr float kHintMax = 0.95f;
static_assert(kMaxBlocks <= kBlock, "one thread per producer block in the prologue reductions");

constexpr int kDistExp = SIDCO_DIST_EXP;
constexpr int kDistGamma = SIDCO_DIST_GAMMA_GPD;
constexpr int kDistGpd = SIDCO_DIST_GPD;

constexpr uint32_t kStNonfinite = SIDCO_ST_NONFINITE;
constexpr uint32_t kStVarZero = SIDCO_ST_VAR_ZERO;
constexpr uint32_t kStGammaS = SIDCO_ST_GAMMA_S;
constexpr uint32_t kStGammaClamp = SIDCO_ST_GAMMA_CLAMP;
constexpr uint32_t kStStopped = SIDCO_ST_STOPPED;
constexpr uint32_t kStOverflow = SIDCO_ST_OVERFLOW;
constexpr uint32_t kStFallback = SIDCO_ST_FALLBACK;

// A fitted law as the kernels use it (see Fit in the kernel source), with the location it sits on.
struct FitRecord {
    int gpd;
    float loc;
    double s, c, a, b;
};

// Device-resident state of one call.  Stage m's kernel reads the entries stage m-1 wrote and
// writes its own, so no entry is read and written inside one kernel.
struct DevState {
    sidco_diag diag;
    uint32_t status_after[SIDCO_MAX_STAGES + 1];  // status bits accumulated up to and including stage m
    uint32_t frozen_after[SIDCO_MAX_STAGES + 1];  // 1 once an empty exceedance set stopped the refinement
    float list_eta[SIDCO_MAX_STAGES + 1];         // the lists written by stage m's kernel hold every entry above this
    FitRecord cand_fit[SIDCO_MAX_STAGES + 1];     // stage m wrote candidate lists: its fitted law and location
    // Survives from call to call (k_fit does not clear it): where stage m+1's threshold fell between
    // stage m's target ratio and its own, on the log scale of stage m's fitted law; NaN if unknown.
    float theta_seen[SIDCO_MAX_STAGES + 1];
    // Adapt_Stages bookkeeping (Algorithm 1): pairs reported by the calls since the controller last
    // looked, not counting the call in flight; k_fit folds the previous call's count in (or starts over)
    unsigned long long khat_sum;
    long long prev_cap;                           // output capacity of the previous call (clips its count)
    unsigned long long selected_ctr;              // pairs selected by the last stage (cleared by k_fit)
    uint32_t overflow;                            // 1 if selected_ctr exceeded the output capacity
    uint32_t bad_index;                           // sidco_scatter_add met an index outside [0, d) since the last check
    // who made the last call with this state (id of a stage controller, 0 otherwise), and whether a call
    // of someone else fell into the current window of the controller's count
    unsigned long long owner;
    uint32_t disturbed;
};

// Kernel arguments (passed by value).
// element type of the gradient buffer (the accumulated vector and the residual are always fp32)
constexpr int kGradF32 = 0, kGradF16 = 1, kGradBf16 = 2;

struct Params {
    const void* grad;       // d elements of type `gt`
    int gt;                 // kGrad*
    float* residual;        // NULL: memoryless
    float* acc_w;           // where k_fit stores acc: residual; for a 16-bit gradient without residual a
                            // workspace buffer; NULL when acc is the fp32 gradient itself
    const float* acc;       // dense working vector read by stage 1's compaction: acc_w, else grad
    int64_t d;
    uint32_t ntiles;        // ceil(d / kTile)
    uint32_t nfull;         // d / kTile: tiles below this index are complete
    uint32_t nwaves;        // waves that own tiles
    uint32_t nblocks;       // grid size of the kernels that read the dense vector or write partial sums
    int vec_ok;             // all dense buffers aligned for 4-element accesses (16 bytes; 8 for a 16-bit gradient)
    int reverse;            // a dense stage kernel walks every wave's tiles from the last to the first
    int acc_reset;          // k_fit: start the controller's count of reported pairs over instead of adding to it
    unsigned long long owner;  // id of the stage controller that makes the call, 0 otherwise
    int dist;
    int M;
    int stage;              // 1-based stage a k_compact launch works for
    double L[SIDCO_MAX_STAGES];  // log(1/delta_m)
    float theta;            // > 0: the lists of this kernel are candidate lists (see stage_prologue); else 0
    float theta_min;        // lowest theta a hint may lead to: below it the lists would exceed kMaterializeBelow
    int use_hint;           // the previous call on the device had this call's shape: theta_seen applies
    int prev_cand;          // the producer of this kernel's source lists wrote candidate lists
    DevState* st;
    const double* part_in;  // [4][kMaxBlocks] partial sums written by the previous kernel
    double* part_out;
    const uint32_t* cnt_in; // [kMaxWaves] survivor-list lengths written by the previous kernel
    uint32_t* cnt_out;
    const uint32_t* blk_in; // [kMaxBlocks] per-block sums of cnt
    uint32_t* blk_out;
    const int2* seg_in;     // survivor lists (index, value bits); wave w's list starts at tile_begin(w)*kTile
    int2* seg_out;
    int32_t* out_idx;
    float* out_val;
    int32_t* out_count;
    float* out_eta;
    int64_t out_cap;
    uint32_t* status_out;   // NULL, or a device word that receives the call's status bits as well
};

// ---- exact Top-k comparator (sidco_topk.hip) ----
constexpr int kTopkBins = 2048;  // digit 0 = magnitude bits 30..20; digits 1 and 2 have 1024 bins

struct TopkState {
    uint32_t prefix[3];            // bin of the k-th largest key in digit 0, 1, 2
    uint32_t k_rem[3];             // rank of that key inside the bin (k_rem[2] = ties still needed)
    uint32_t kth_key;              // the k-th largest magnitude as its bit pattern
    uint32_t k_eff;                // k when the device decides it (TopkParams::k_from_state)
    unsigned long long gt_ctr;     // output places reserved for entries above the k-th key
    unsigned long long eq_ctr;     // entries equal to the k-th key seen so far
};

struct TopkParams {
    const void* grad;       // d elements of type `gt`
    int gt;                 // kGrad*
    float* residual;        // NULL: memoryless
    float* acc_w;           // where the first kernel stores acc: residual; a workspace buffer for a 16-bit gradient
                            // without residual; NULL when acc is the fp32 gradient itself
    const float* acc;       // acc_w, else grad
    int64_t d;
    int64_t k;
    int k_from_state;       // the last kernel takes k from st->k_eff (may be 0) instead of `k`
    uint32_t ntiles, nfull, nwaves, nblocks;
    int vec_ok;
    uint32_t* hist;         // [3][kTopkBins]
    TopkState* st;
    uint32_t* cnt;          // [kMaxWaves] list lengths
    int2* seg;              // per-wave lists
    int32_t* out_idx;
    float* out_val;
    int32_t* out_count;
    float* out_kth;
};

void launch_topk_zero(const TopkParams& p, hipStream_t s);
void launch_topk_hist(const TopkParams& p, hipStream_t s);
void launch_topk_compact(const TopkParams& p, hipStream_t s);
void launch_topk_refine(const TopkParams& p, uint32_t grid, hipStream_t s);
void launch_topk_final(const TopkParams& p, uint32_t grid, hipStream_t s);

// ---- DGC comparator: threshold from a radix select on a random subset, first pass over the vector,
// second radix select on the first pass's entries ----
struct DgcState {
    TopkState sample;               // select of the k_s-th largest magnitude of the subset
    TopkState lists;                // select among the entries of the first pass
    unsigned long long first_pass;  // entries above the subset's threshold
    float eta;                      // that threshold
    float kth;                      // smallest magnitude that stayed
};

struct DgcParams {
    const void* grad; // d elements of type `gt`
    int gt;           // kGrad*
    float* residual;  // NULL: memoryless
    int64_t d;
    int64_t k;        // target number of entries
    uint32_t ntiles, nfull, nwaves, nblocks;
    int vec_ok;
    uint64_t seed;
    uint32_t n_s, k_s;  // subset size, rank of the threshold in it
    uint32_t* keys;     // [n_s] magnitude keys of the subset
    uint32_t* hist_s;   // [3][kTopkBins] digit histograms of the subset
    uint32_t* hist_l;   // [3][kTopkBins] digit histograms of the first pass's entries
    DgcState* st;
    uint32_t* cnt;      // [kMaxWaves] list lengths
    int2* seg;          // per-wave lists
    float* out_eta;
};

void launch_dgc_zero(const DgcParams& p, hipStream_t s);
void launch_dgc_sample(const DgcParams& p, hipStream_t s);
void launch_dgc_digit(const DgcParams& p, int digit, hipStream_t s);
void launch_dgc_dense(const DgcParams& p, hipStream_t s);
void launch_dgc_lists(const DgcParams& p, uint32_t grid, hipStream_t s);

// A block's place in its vector's grid (the whole launch for a single call, a slice of it in a batch).
struct Blk {
    uint32_t id;  // block index within the vector's grid
    uint32_t n;   // size of that grid
};

// ---- batched calls: several vectors (the tensors of one flat buffer) in one launch sequence ----
constexpr int kMaxBatch = kMaxBlocks;  // every vector owns at least one block of the 512-block launches

// One vector of a batch, relative to the call's base pointers (so that the table on the device depends on
// the layout alone and survives a change of buffers).
struct TensorDesc {
    int64_t offset;         // first element in grad / residual
    int64_t d;
    int64_t out_offset;     // first pair in out_idx / out_val
    int64_t out_cap;
    uint64_t seg_off;       // first slot of the vector in the survivor-list buffers
    uint32_t first_block;   // the vector's blocks in the dense grids: [first_block, first_block + nblocks)
    uint32_t nblocks;
    uint32_t first_final;   // ... and in the last stage's grid
    uint32_t nfinal;
    uint32_t index;         // position in out_counts / out_etas
    uint32_t reserved;
};

struct BatchTable {
    DevState st[kMaxBatch];
    TensorDesc desc[kMaxBatch];
    uint16_t map[kMaxBlocks];   // block of a dense grid -> vector
    uint16_t fmap[kMaxBlocks];  // block of the last stage's grid -> vector
};

// Kernel arguments of a batched launch (by value): what all vectors share.
struct BatchArgs {
    BatchTable* tb;
    const void* grad;       // base pointers of the call; the gradient's elements are of type `gt`
    int gt;                 // kGrad*
    float* residual;
    float* acc_own;         // workspace copy of acc for a 16-bit gradient without residual, else NULL
    int32_t* out_idx;
    float* out_val;
    int32_t* out_counts;
    float* out_etas;
    double* part[2];
    uint32_t* cnt[2];
    uint32_t* blk[2];
    int2* seg[2];
    int in, out;            // which half of the double buffers the kernel reads / writes
    int dist, M, stage, reverse;
    double L[SIDCO_MAX_STAGES];
    float theta, theta_min;
    int use_hint, prev_cand;
};

void launch_fit_batched(const BatchArgs& a, bool ec, uint32_t blocks, uint32_t flat_gx, double* scratch, hipStream_t s);
void launch_compact_batched(const BatchArgs& a, bool stats, bool write, bool prefetch, uint32_t blocks, hipStream_t s);
void launch_lists_batched(const BatchArgs& a, uint32_t blocks, hipStream_t s);
void launch_final_lists_batched(const BatchArgs& a, uint32_t final_blocks, hipStream_t s);
void launch_gather_batched(const BatchArgs& a, uint32_t blocks, hipStream_t s);

void launch_clear_u32(uint32_t* p, hipStream_t s);
void launch_scatter_add(float* dense, int64_t d, const int32_t* idx, const float* val, const int32_t* count,
                        int64_t capacity, float scale, uint32_t* bad, hipStream_t s);
// batches of 4 tiles that a dense stage's waves load before their threshold is known and then stay ahead of
// the batch they process (long vectors only; see compact_dense)
constexpr int kCompactPrefetch = 1;
// k_fit's shape for large vectors (see k_fit_flat): one float4 per thread, 256-thread blocks; from the
// length at which the faster sweep pays for the extra kernel that folds its partial sums
constexpr int kFlatBlock = 256;
constexpr int64_t kFlatMinD = 12000000;
inline bool fit_uses_flat(int64_t d, bool vec_ok) { return vec_ok && d >= kFlatMinD; }
inline uint32_t fit_flat_blocks(int64_t d) { return (uint32_t)((d / 4 + kFlatBlock - 1) / kFlatBlock); }
void launch_fit(const Params& p, double* scratch, hipStream_t s);
void launch_compact(const Params& p, bool stats, bool write, hipStream_t s);
void launch_lists(const Params& p, uint32_t grid_blocks, hipStream_t s);
void launch_final_lists(const Params& p, uint32_t grid_blocks, hipStream_t s);
void launch_gather(const Params& p, hipStream_t s);

}  // namespace sidco
#endif
