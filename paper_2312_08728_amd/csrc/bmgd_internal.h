// Internal interfaces between the host-side context code and the HIP kernels of libbmgd.
// Nothing here is part of the public ABI (see include/bmgd.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

struct bmgd_reader;
// Reader (reader.hip): hand out the next buffer if it is in host memory (*x = NULL if not; block = wait for it);
// *end = 1 once the data set has been delivered completely.  Status code as the public calls.
int reader_take(bmgd_reader* r, bool block, const void** x, const void** y, int64_t* rows, int* end);

namespace bmgd {

// Message that bmgd_last_error(NULL) returns on the calling thread (calls that have no context to hold one).
void set_create_error(const char* msg);

constexpr int kPermRounds = 8;
constexpr int kMaxPassesPerLaunch = 4;     // partitions kept on the device at a time
constexpr int kThetaCopies = 8;            // copies of the theta broadcast (sliced reduction)

// Round keys of the partition generator for up to kMaxPassesPerLaunch passes.
struct PermKeys {
    uint32_t key[kMaxPassesPerLaunch][kPermRounds];
};

// Host: derive the eight round keys of PERM(seed, b, t, .).
void perm_round_keys(uint64_t seed, uint32_t b, uint32_t t, uint32_t out[kPermRounds]);
// Host: half block width h of the Feistel network for a buffer of `rows` rows.
int perm_half_width(int64_t rows);

// Device: out[pass][j] = PERM(...)[j] for j < rows, pass < npass (row stride = rows).
// subset != NULL: out[pass][j] = subset[PERM(...)[j]] (a partition of the rows subset[0 .. rows) of a buffer of `limit`
// rows); an entry outside [0, limit) is replaced by 0 and *bad is set to 1.
hipError_t launch_perm(int32_t* out, int64_t rows, int npass, const PermKeys& keys, hipStream_t stream,
                       const int32_t* subset = nullptr, int64_t limit = 0, unsigned* bad = nullptr);

// Device: zero `bytes` bytes at dst (both multiples of 16) with a kernel, in stream order.
hipError_t launch_fill_zero(void* dst, size_t bytes, hipStream_t stream);

// Device: running mean of snapshots of theta (n floats), in stream order: avg <- theta if `first`, else
// avg <- avg + (theta - avg) * inv.
hipError_t launch_running_mean(float* avg, const float* theta, size_t n, float inv, bool first, hipStream_t stream);

// ---------------------------------------------------------------------------------------------------
// Update rules fed with the mini-batch gradient (Section 4.3: buffered NAG and Adam).

enum { kOptSgd = 0, kOptMomentum = 1, kOptNag = 2, kOptAdam = 3 };

struct OptArgs {
    int kind;
    float mu, b1, b2, eps;
    float* m;           // first state array (v of momentum / NAG, m of Adam), laid out like theta
    float* s;           // second state array (Adam)
    int k_base;         // updates made before this launch (Adam's bias corrections use k_base + step + 1)
};

#ifdef __HIPCC__
// Bias corrections 1 / (1 - beta^k) of Adam for update number k >= 1.
__device__ __forceinline__ void opt_corrections(const OptArgs& o, int k, float& c1, float& c2)
{
    c1 = 1.f / (1.f - powf(o.b1, (float)k));
    c2 = 1.f / (1.f - powf(o.b2, (float)k));
}

// One coordinate of one update: new theta from the mean gradient g; m and s are that coordinate's state.
__device__ __forceinline__ float opt_update(const OptArgs& o, float th, float g, float alpha, float& m, float& s, float c1,
                                            float c2)
{
    if (o.kind == kOptAdam) {
        m = o.b1 * m + (1.f - o.b1) * g;
        s = o.b2 * s + (1.f - o.b2) * g * g;
        return th - alpha * (m * c1) / (sqrtf(s * c2) + o.eps);
    }
    m = o.mu * m - alpha * g;
    return o.kind == kOptNag ? th + o.mu * m - alpha * g : th + m;
}
#endif

// ---------------------------------------------------------------------------------------------------
// GLM (least squares / logistic) chain.

enum { kReduceRedundant = 0, kReduceSliced = 1 };

struct GlmLaunchShape {
    int V;              // floats per vector load (1, 2, 4)
    int CPL;            // vector chunks of a row held per lane
    int PF;             // rows in flight per row slot
    int pipe;           // how row loads are scheduled against the theta chain (kPipe* in glm_kernels.hip)
    int L;              // lanes cooperating on one row (power of two <= 64)
    int block;          // threads per workgroup
    int G;              // workgroups
    int reduce_mode;    // kReduce*
    size_t lds_bytes;
    int max_G;          // co-resident workgroups the device can hold for this kernel
    int with_optimizer; // set by the caller after glm_plan: the kernel variant with an update rule other than the plain step
    int split;          // 1: the persistent chain runs the kernel for rows of more than 1024 floats (glm_split_kernel.hip):
                        // G is a multiple of 8, split_ch = float4 chunks of a row per lane (1: p <= 2048, 2: p <= 4096)
    int split_ch;
    int narrow;         // 1: the persistent chain runs the kernel for rows of up to 1024 floats whose share of a step fits a
                        // workgroup's registers (glm_narrow_kernel.hip): G is a multiple of 8, narrow_pf rows per row slot
    int narrow_pf;
    int64_t n;          // mini-batch size and row length the shape was planned for
    int p;
    int chain_block;    // threads per workgroup of the persistent chain's kernel
};

struct GlmArgs {
    const float* X;         // [rows][p]
    const float* y;         // [rows]
    const int32_t* perm;    // [npass][perm_stride]: partition of pass t at perm + t * perm_stride
    float* theta;           // [p]
    float* partial;         // [2][G][p] per-workgroup gradient sums (step-per-launch mode)
    unsigned long long* ll_part;   // [2][G][p] the same sums as flagged words {tag : float}, by step parity
    unsigned long long* ll_theta;  // [2][kThetaCopies][p] updated theta as flagged words (sliced reduction)
    unsigned* sync;         // [1] abort flag ([0] unused)
    unsigned tag_base;      // tag of step s is tag_base + (s - s_begin) + 1
    int s_begin, s_end;     // steps of this launch: s in [s_begin, s_end), s = pass * M + batch, all < 2^23
    int rows, p, n, npass;
    int perm_stride;        // rows, or 0 when every pass reuses one partition
    int model;
    int L, logL;
    int reduce_mode;
    float alpha;
    long long timeout_ticks;
    int single_step;        // >= 0: process only that step and stop after writing partial sums
    OptArgs opt;            // kind == kOptSgd: plain steps, no state.  Redundant reduction: every workgroup keeps a
                            // private copy of the state at m + blockIdx.x * pp (all copies stay identical)
    const float* lr_tab;    // optional learning rate per step: step s uses lr_tab[min(lr_base + s, lr_len - 1)]
    int lr_base, lr_len;
};

// Pick V/CPL/PF/L/block/G/reduce mode for a shape; returns false if p is outside the supported range.
bool glm_plan(int64_t p, int64_t n, int requested_G, int num_cus, GlmLaunchShape* out, char* why, size_t why_len);
// Query co-residency and set attributes; fills shape->max_G and clamps shape->G.
hipError_t glm_prepare(GlmLaunchShape* shape);
// One launch of the persistent chain kernel covering steps [s_begin, s_end) of the buffer.
hipError_t glm_launch_chain(const GlmLaunchShape& shape, const GlmArgs& args, hipStream_t stream);
// Step-per-launch variant: partial sums for step `args.single_step`, then reduce + update.
hipError_t glm_launch_step(const GlmLaunchShape& shape, const GlmArgs& args, int nb, hipStream_t stream);

// Persistent chain for rows of more than 1024 floats on G = 8, 16, ... workgroups (glm_split_kernel.hip): shared memory
// and threads per workgroup, co-resident capacity, one launch covering steps [s_begin, s_end).
size_t glm_split_lds_bytes(int ch);
int glm_split_block();
hipError_t glm_split_prepare(int ch, bool opt, int* max_groups);
hipError_t glm_split_launch(int ch, bool opt, int G, const GlmArgs& args, hipStream_t stream);

// Persistent chain for rows of up to 1024 floats (p even) on G = 8, 16, ... workgroups when a step's rows fit the
// registers of the grid (glm_narrow_kernel.hip).  glm_narrow_rows_in_flight: rows per row slot that a step of n rows
// needs on G workgroups, 0 if that is more than the kernel holds.
int glm_narrow_block();
int glm_narrow_rows_in_flight(int v, int cpl, int L, int G, int64_t n);
hipError_t glm_narrow_prepare(const GlmLaunchShape& shape, int p, int* max_groups);
hipError_t glm_narrow_launch(const GlmLaunchShape& shape, const GlmArgs& args, hipStream_t stream);

// Evaluation: partial[b] = sum of the per-sample losses of the rows workgroup b takes (b < nblocks <= kEvalBlocks).
constexpr int kEvalBlocks = 1024;
hipError_t glm_launch_loss(const float* X, const float* y, const float* theta, int rows, int p, int model, double* partial,
                           int nblocks, hipStream_t stream);

// ---------------------------------------------------------------------------------------------------
// Least squares in the form of eq. (3.1): per-mini-batch moment matrices, then a one-workgroup chain.

constexpr int kGramMaxP = 128;
// The automatic choice: least squares, p <= kGramMaxP and mini-batches of at least 2 p rows.
bool gram_eligible(int model, int64_t p, int64_t n);
// Bytes of moment matrices per mini-batch (Sxx_m and Sxy_m in the order the chain's threads read them).
size_t gram_bytes_per_batch(int64_t p);
// Threads of the one workgroup that runs the chain.
int gram_chain_threads(int64_t p);
// Moment matrices of all mini-batches of `npass` passes (partitions at perm + pass * perm_stride) into `gram`.
// `start` and `stop` (each may be NULL) are completed by the kernel's own dispatch, here and below.
hipError_t gram_launch_moments(const float* X, const float* y, const int32_t* perm, float* gram, int rows, int p, int n, int npass,
                               int perm_stride, hipStream_t stream, hipEvent_t start, hipEvent_t stop, bool dense = false);
// dense = true: each mini-batch's [Sxx_m | -Sxy_m] as a dense row-major matrix of order gram_dense_order(p) (p + 1 rounded
// up to 16; what lies beyond row p - 1 or column p is never written and must be zero), for gram_launch_products
int gram_dense_order(int64_t p);
size_t gram_dense_bytes_per_batch(int64_t p);
// The npass * ceil(rows / n) updates of theta from those matrices, in one workgroup.
// lr_tab (may be NULL): learning rate of step s is lr_tab[min(lr_base + s, lr_len - 1)] instead of alpha.
hipError_t gram_launch_chain(const float* gram, float* theta, int rows, int p, int n, int npass, int perm_stride, float alpha,
                             const float* lr_tab, int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream,
                             hipEvent_t start, hipEvent_t stop);
// The same chain over nsteps sets of matrices given directly (step s uses set s % period)
hipError_t gram_launch_chain_steps(const float* gram, float* theta, int p, int nsteps, int period, float alpha, const float* lr_tab,
                                   int lr_base, int lr_len, const OptArgs& opt, hipStream_t stream, hipEvent_t start,
                                   hipEvent_t stop);
// BMGD_CHAIN_PRODUCT (gram_products.hip): the npass * M steps of a launch as affine maps, multiplied together pairwise
// in log2 rounds and applied to theta once.  `gram`: the dense matrices of gram_launch_moments(..., dense = true).
// `scratch`: gram_products_scratch_floats(p, npass * M) floats.  Plain steps only.
size_t gram_products_scratch_floats(int64_t p, int64_t max_steps);
// once per device with that device current, before the first launch below (raises the kernels' shared-memory limit)
hipError_t gram_products_prepare();
hipError_t gram_launch_products(const float* gram, float* theta, float* scratch, float* product_out, int rows, int p, int n, int npass,
                                int perm_stride, float alpha, const float* lr_tab, int lr_base, int lr_len, hipStream_t stream,
                                hipEvent_t start, hipEvent_t stop, bool pairs_then_chain = false);
// product_out (optional): where the product of the launch's steps is left, gram_dense_order(p)^2 floats; gram_launch_apply
// applies such a product to theta again (fixed partitions, constant rate: the product of a buffer is the same every time).
// pairs_then_chain: one round only - neighbouring steps multiplied in pairs, written as [I - A | d] in the chain's layout -
// and the chain of eq. (3.1) then runs over half as many steps (with rate 1: theta - (I - A) theta + d = A theta + d)
hipError_t gram_launch_apply(const float* product, float* theta, int p, hipStream_t stream, hipEvent_t start, hipEvent_t stop);
// One round only: the launch's steps multiplied in neighbouring pairs, each product P written as [I - P | last column of P]
// in the layout of the chain's moment matrices ((npass * M + 1) / 2 sets), so that gram_launch_chain_steps with rate 1 applies them
hipError_t gram_launch_pairs(const float* gram, float* pairs_out, int rows, int p, int n, int npass, int perm_stride, float alpha,
                             const float* lr_tab, int lr_base, int lr_len, hipStream_t stream, hipEvent_t start, hipEvent_t stop);

// ---------------------------------------------------------------------------------------------------
// Softmax regression (bf16 predictors, fp32 master weights) on the matrix cores.

struct SoftmaxDims {
    int c_pad;          // classes padded to the tile width (padding classes get probability 0)
    int n_pad;          // mini-batch rows padded to the K tile of the gradient contraction
    int m_pad;          // mini-batch rows padded to the tile height of the logits
    int p_pad;          // features padded to the tile height of the gradient
    int splits;         // split-K factor of the logits contraction
    int k_per_split;
};

// What changes from pass to pass without changing the sequence of launches: read by the update kernels from device
// memory, written in stream order before each pass.
struct SoftmaxState {
    float alpha;        // learning rate when no per-update table is set
    int lr_pos;         // updates enqueued since the table was set, before this pass
    int opt_k;          // updates made before this pass (Adam's bias corrections)
};

struct SoftmaxStep {
    const void* X;          // slot, bf16 [rows][p]
    const int32_t* y;       // class ids [rows]
    const int32_t* idx;     // the mini-batch: nb entries of the partition
    const void* XT;         // bf16 [p][n_pad]: this mini-batch transposed
    float* W;               // fp32 master [p][c_pad]
    OptArgs opt;            // state arrays laid out like W (k_base unused: the count comes from `state`)
    const SoftmaxState* state;
    int u;                  // number of this update within its pass
    const float* lr_tab;    // optional learning rate per update (device), lr_len entries
    int lr_len;
    void* WbT;              // bf16 copy, transposed [c_pad][p_pad]
    float* U;               // logits scratch [splits][m_pad][c_pad]
    void* Rt;               // residual scratch, bf16 [c_pad][n_pad]
    int nb, p, C;
};

SoftmaxDims softmax_dims(int64_t p, int64_t n, int64_t C);
hipError_t softmax_prepare(const SoftmaxDims& d);
// XT[m][c][j] = X[perm[m n + j]][c] for every mini-batch m of one pass.
hipError_t softmax_permute_transpose(const void* X, const int32_t* perm, void* XT, int rows, int p, int n,
                                     const SoftmaxDims& d, hipStream_t stream);
// One mini-batch update: logits, residual, gradient + update (three launches in stream order).
hipError_t softmax_step(const SoftmaxStep& s, const SoftmaxDims& d, hipStream_t stream);
// *state <- (alpha, lr_pos, opt_k), in stream order.
hipError_t softmax_set_state(SoftmaxState* state, float alpha, int lr_pos, int opt_k, hipStream_t stream);
// Evaluation: cross-entropy summed over `nb` rows X[row0 .. row0 + nb) (contiguous, nb <= the batch size the context
// was created with) at the bf16 copy of W: partial[b] for b < ceil(nb / 8) workgroups.
hipError_t softmax_launch_loss(const void* X, const int32_t* y, int nb, int p, int C, const void* WbT, float* U,
                               const SoftmaxDims& d, double* partial, hipStream_t stream);
// WbT <- bf16(W) transposed, whole matrix.
hipError_t softmax_refresh_shadow(const float* W, void* WbT, int p, const SoftmaxDims& d, hipStream_t stream);

}  // namespace bmgd
