// Internal interface between the host planner (pack_api.cpp) and the gfx950 kernels
// (pack_kernels.hip).  Nothing here is part of the public ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace packk {

// Every matrix product of the step is one instance of  OUT[r, q] = sum_k A(r, k) * B(q, k),
// r in [0,R), q in [0,Q), k in [0,Kd), with the two operands fetched by a mode-specific
// address rule.  MODE selects the rules and the epilogue.
enum GemmMode : int {
    LIN_FWD = 0,   // Z[m,n]   = sum_k H[m,k] W[n,k]                 (+bias, relu)
    LIN_DX = 1,    // dH[m,k'] = sum_n dZ[m,n] W[n,k']               (mask, accumulate)
    LIN_DW = 2,    // dW[o,i]  = sum_b dZ[b,o] H[b,i]
    CONV_FWD = 3,  // Z[(b,i,j),o] = sum_(tap,c) In[b,s*i+u-1,s*j+v-1,c] W[o,tap,c]   (+bias, residual, relu)
    CONV_DX = 4,   // dIn[(b,y,x),c] = sum_(tap,o) dZ[b,(y+1-u)/s,(x+1-v)/s,o] W[o,tap,c]  (mask, accumulate)
    CONV_DW = 5    // dW[o,(tap,c)] = sum_(b,i,j) dZ[(b,i,j),o] In[b,s*i+u-1,s*j+v-1,c]   (split over the sum)
};

#ifndef PACK_LR_N
#define PACK_LR_N 256
#endif
struct LrTable { float lr[PACK_LR_N]; };

enum GemmFlags : int {
    F_RELU = 1,        // forward: max(v, 0)
    F_OUT_F32 = 2,     // forward: store float regardless of the pack dtype (logits)
    F_ACCUM = 4,       // dX: add to what the output buffer already holds
    F_MASK = 8,        // dX: zero where aux <= 0 (aux = the stored activation of the output tensor)
    F_RES_ID = 16,     // forward: add aux[row, col] before the ReLU (identity shortcut)
    F_RES_DOWN = 32,   // forward: add aux[b, 2i, 2j, col] for col < resC (subsampling shortcut)
    F_VEC_A = 64,      // operand A may be fetched as aligned 16-byte vectors
    F_VEC_B = 128,     // operand B likewise
    F_A_INPUT = 256,   // operand A is the input batch handed to this step (+ x_off)
    F_B_INPUT = 512,   // operand B is the shared input batch
    F_AUX_INPUT = 1024,// the shortcut source is the shared input batch
    F_ROWMAP = 2048,   // stride-2 input gradient, one parity class of input pixels: output row r is
                       // pixel (b, 2*yc + 1 - cls_py, 2*xc + 1 - cls_px) and the reduction runs over the
                       // taps of that class only (u = 1 or u in {0, 2}, likewise v)
    F_UPDATE = 4096,   // weight gradient, not split: apply W <- W - lr[member] * dW (and b likewise) in the
                       // epilogue instead of storing the gradient for a separate update launch
    F_KEEP_G = 8192,   // with F_UPDATE: store the gradient as well
    F_SC_ID = 16384,   // dX of the first layer of a residual block: add the gradient that arrives through the
                       // identity shortcut, sc[row, col] (same shape as the output), before the mask
    F_SC_DOWN = 32768, // likewise for the subsampling shortcut: pixel (2i, 2j) receives sc[b, i, j, col]
    F_WS = 65536,      // split weight gradient: C and dbias hold BYTE OFFSETS into the step's workspace (the
                       // buffer of partial sums the launch receives as an argument), not addresses
    F_GENERAL_TAIL = 131072   // forward / input gradient: every tile takes the general form of the tail (set by a test
                              // that compares it with the form whole tiles of the plain cases take)
};

// activation kinds (paper Table 3); the value is also what GemmProb::act / mask_act hold
enum ActKind { ACT_NONE = 0, ACT_RELU = 1, ACT_LEAKY = 2, ACT_SIGMOID = 3, ACT_TANH = 4 };

// element and vector types shared by the kernels and the host-side walks of their address rules
typedef unsigned short bf16_t;   // bfloat16 = upper half of an IEEE binary32
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
typedef __attribute__((ext_vector_type(4))) int i32x4_t;
// raw buffer descriptors of the aligned kernels: the window a descriptor covers, and the byte offset that
// stands for "this element does not exist" (at or beyond the window: the load returns zeros, no memory access)
constexpr unsigned BUF_RECORDS = 0x80000000u;
constexpr unsigned BUF_POISON = 0x80000000u;

struct GemmProb {
    const void* A;
    const void* B;
    void* C;
    const float* bias;
    const void* aux;
    const void* zeros;                     // 256 bytes of zeros: what a missing operand element reads
    float* dbias;                          // weight-gradient modes: where the bias gradient goes
                                           // (split ks writes dbias[ks * R + row]); null = skip
    int R, Q, Kd;
    int lda, ldb, ldc;
    int H, W, Cin, Ho, Wo, Cout, stride;   // geometry of the forward convolution (conv modes)
    int resH, resW, resC;                  // geometry of the shortcut source (F_RES_DOWN)
    int cls_py, cls_px, cls_h, cls_w;      // F_ROWMAP: parity class and its extent in pixels
    int row_w, row_hw;                     // conv problems whose rows are pixels: row r = (image, r % row_hw / row_w, r % row_w)
    int lg_row_w, lg_row_hw;               // their base-2 logarithms when both are powers of two, else -1
    int act;                               // forward modes: activation applied after bias and shortcut (ActKind)
    int mask_act;                          // input-gradient modes with F_MASK: activation that produced `aux`
    int flags;
    int ksplit;                            // reduction indices per split (>= Kd when not split)
    long long split_stride;                // elements between the partial outputs of two splits
    long long x_off;                       // bytes added to the step's input pointer (packs whose members read their own batch)
    float* upd_w;                          // F_UPDATE: master weights, same layout as C
    void* upd_shadow;                      // F_UPDATE: bf16 operand copy of the weights (null for fp32 packs)
    float* upd_b;                          // F_UPDATE: master bias [R]
    int member;                            // F_UPDATE: index into the step's learning-rate table
    const void* sc;                        // F_SC_ID / F_SC_DOWN: gradient wrt the block output [n, scH, scW, scC]
    int scH, scW, scC;
};

struct TileRef {      // one workgroup's job; prob < 0 marks a filler slot
    int prob;
    int tm, tn, ks;
};

struct ReduceProb {   // out[e] = sum_{s < S} in[s * stride + e], fixed order
    const float* in;      // a BYTE OFFSET into the step's workspace, not an address
    float* out;
    long long stride;
    int n, S;
    float* upd_w;         // not null: apply w[e] <- w[e] - lr[member] * sum instead of (keep_g: as well as) storing it
    void* upd_shadow;     // bf16 copy of w to refresh, or null
    int member, keep_g;
};

struct CeProb {       // softmax cross-entropy of one member
    const float* logits;   // [rows, ld]
    void* dlogits;         // [rows, ldd] pack dtype
    int* pred;             // [rows]
    float* loss;           // scalar
    int rows, C, ld, ldd;
    int label_off;         // first label of the member in the step's label vector
};

struct HeadProb {     // classifier head of one member in one kernel: logits, softmax cross-entropy, dlogits, input gradient
    const void* h;         // [rows, Kd] pack dtype: the activations the last linear layer reads
    const void* W;         // [C, Kd] pack dtype (operand copy of the weights)
    const float* bias;     // [C]
    float* logits;         // [rows, C]
    void* dlogits;         // [rows, ldd] pack dtype
    void* dh;              // [rows, Kd] pack dtype: gradient wrt h, or null when nothing upstream needs it
    int* pred;             // [rows]
    float* loss;           // scalar
    float* partial;        // [nblk] per-block loss sums
    int rows, C, Kd, ldd, label_off, mask_act, nblk;
};
constexpr int HEAD_ROWS = 4;       // rows one block of the head kernel handles
constexpr int HEAD_MAX_C = 16;     // classes the head kernel keeps in registers

struct GapProb {      // global average pool: in [n, hw, c] -> out [n, c]
    const void* in;
    void* out;
    const void* dz_out;    // backward: gradient wrt out
    void* dz_in;           // backward: gradient wrt in
    int n, hw, c;
    int mask;              // backward: ActKind that produced `in` (its derivative multiplies the gradient)
    int accum;
};

struct ShortcutProb { // backward of the residual shortcut into the source tensor's gradient
    const void* dz_out;    // [n, Ho, Wo, Co]
    const void* src;       // stored activation of the source [n, H, W, C] (mask)
    void* dz_src;
    int n, H, W, C, Ho, Wo, Co;
    int down;              // 0 identity, 1 subsample
    int mask;              // ActKind that produced `src`
    int accum;
};

struct Im2colProb {   // shared-input loader: x [B,H,W,C] -> xcol [B*Ho*Wo, Kp], k = tap*C + c, zero beyond 9*C
    void* out;
    int B, H, W, C, Ho, Wo, stride, Kp;
};

struct TransposeProb {   // convolution weights [Cout][9][Cin] -> [Cin][9][Cout], both of the pack's operand type
    const void* src;
    void* dst;
    int Cin, Cout, tiles_ci, tiles_co;   // 64 x 64 tiles per tap
};



// launch wrappers; all enqueue on `st` and return the launch status -----------------------------
// tile_cfg indexes GEMM_TILE_M / GEMM_TILE_N
// lr: the step's learning rates (used by weight-gradient launches whose problems carry F_UPDATE)
// ws: the step's workspace (partial sums of split weight gradients; problems with F_WS address it by offset)
hipError_t launch_gemm(int mode, bool bf16, int tile_cfg, const GemmProb* probs_dev, const TileRef* tiles_dev,
                       int n_tiles, const void* x_dev, char* ws, const LrTable& lr, hipStream_t st);
// halo form of the convolution weight gradient (pack_conv_dw.hip): every problem of the launch has the
// given stride and passes conv_dw_halo_ok
hipError_t launch_conv_dw_halo(bool bf16, int tile_cfg, const GemmProb* probs_dev, const TileRef* tiles_dev, int n_tiles,
                               const void* x_dev, char* ws, const LrTable& lr, hipStream_t st);
// the halo configuration (GEMM_CFG_HALO*) problem p can take, or -1
int conv_dw_halo_cfg(bool bf16, const GemmProb& p);
// the halo configuration (GEMM_CFG_ROWS*) a stride-1 convolution forward (mode CONV_FWD) or input-gradient (CONV_DX)
// problem can take, or -1
int conv_rows_halo_cfg(bool bf16, int mode, const GemmProb& p);
hipError_t launch_reduce(const ReduceProb* probs_dev, const int2* map_dev, int n_blocks, const char* ws, const LrTable& lr, hipStream_t st);
// The library's own scratch array (file-scope device memory, STATIC_SCRATCH_BYTES long, one copy per GPU):
// its address on the current device.  For the entry point that may not allocate.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)128 << 20;
hipError_t static_scratch(char** ptr);
hipError_t launch_ce(bool bf16, const CeProb* probs_dev, int K, const int32_t* labels, int* err_flag, hipStream_t st);
// max_c: the largest class count among the launch's members (<= HEAD_MAX_C)
hipError_t launch_head(bool bf16, int max_c, const HeadProb* probs_dev, const int2* map_dev, int n_blocks, const int32_t* labels,
                       int* err_flag, hipStream_t st);
hipError_t launch_head_loss(const HeadProb* probs_dev, int n_members, hipStream_t st);
hipError_t launch_gap(bool bf16, bool backward, const GapProb* probs_dev, const int2* map_dev, int n_blocks, hipStream_t st);
hipError_t launch_shortcut_bwd(bool bf16, const ShortcutProb* probs_dev, const int2* map_dev, int n_blocks, hipStream_t st);
hipError_t launch_sgd(float* master, const float* grad, void* shadow_bf16, long long n,
                      const long long* seg_end_dev, int K, const LrTable& lr, hipStream_t st);
// per-member optimiser description (device memory, one entry per member) and per-step table (by value)
struct OptStatic { int kind; float mu, beta1, beta2, eps; };
struct OptTable { float lr[256]; float c1[256]; float c2[256]; };   // c1, c2: Adam's 1/(1-beta1^t), 1/(1-beta2^t)
hipError_t launch_opt(float* master, const float* grad, void* shadow_bf16, float* m, float* v, long long n,
                      const long long* seg_end_dev, const OptStatic* params_dev, int K, const OptTable& tab, hipStream_t st);
hipError_t launch_im2col(bool bf16, const Im2colProb& p, const void* x_dev, hipStream_t st);
hipError_t launch_wtranspose(bool bf16, const TransposeProb* probs_dev, const int2* map_dev, int n_blocks, hipStream_t st);
hipError_t launch_cast_bf16(const float* src, void* dst_bf16, long long n, hipStream_t st);
hipError_t launch_fill_zero(void* dst, long long bytes, hipStream_t st);
// x_out[r] = data[idx[r]], labels_out[r] = labels_all[idx[r]] for r < rows; rows of row_bytes bytes (a multiple of 2)
hipError_t launch_ceiling_copy(const void* src, void* dst, long long bytes, hipStream_t st);
hipError_t launch_ceiling_mfma(bool bf16, float* out, int blocks, int iters, double* flops, hipStream_t st);
hipError_t launch_gather_rows(const void* data, const int32_t* labels_all, const long long* idx, long long n_samples,
                              int rows, long long row_bytes, void* x_out, int32_t* labels_out, int* err_flag, hipStream_t st);

// tile geometry the planner needs
// configurations 0..2: aligned problems (16-byte operand loads); 3: the scalar gather for any shape
// 4: the lean 128 x 128 form of the weight-gradient kernels (short reductions)
// 6, 7: the halo form of the convolution weight gradient (stride 1, stride 2): a tile is 64 output channels
// x 64 input channels x all nine taps, i.e. 64 x 576 of the [Cout][9 * Cin] gradient
// 8: the same with 32 input channels per tile (layers whose input channels are a multiple of 32 only; stride 1)
constexpr int GEMM_TILE_M[11] = {128, 128, 64, 64, 128, 128, 64, 64, 64, 256, 256};
constexpr int GEMM_TILE_N[11] = {128, 64, 64, 64, 128, 64, 576, 576, 288, 64, 32};
constexpr int GEMM_CFG_SCALAR = 3;
constexpr int GEMM_CFG_LEAN = 4;     // weight gradients, 128 x 128, short reductions
constexpr int GEMM_CFG_LEAN64 = 5;   // forward / input gradients, 128 x 64, short reductions
constexpr int GEMM_CFG_HALO_S1 = 6;  // convolution weight gradients, halo form, stride 1
constexpr int GEMM_CFG_HALO_S2 = 7;  // likewise, stride 2
constexpr int GEMM_CFG_HALO32_S1 = 8;   // 64 x 32 channel pairs per tile, stride 1
inline bool is_halo_cfg(int cfg) { return cfg >= GEMM_CFG_HALO_S1 && cfg <= GEMM_CFG_HALO32_S1; }
constexpr int GEMM_CFG_ROWS64 = 9;   // stride-1 convolution forward / input gradient, halo form, 256 pixels x 64 columns
constexpr int GEMM_CFG_ROWS32 = 10;  // likewise, 256 pixels x 32 columns
inline bool is_rows_cfg(int cfg) { return cfg == GEMM_CFG_ROWS64 || cfg == GEMM_CFG_ROWS32; }
constexpr int ELEMWISE_PER_BLOCK = 2048;   // elements one block of the elementwise kernels covers
constexpr int SGD_PER_BLOCK = 2048;        // parameters one block of the update kernel covers (measured best of 1024..8192)

}  // namespace packk
