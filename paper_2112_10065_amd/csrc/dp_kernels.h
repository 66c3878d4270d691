// Internal interface between the C-ABI layer (dp_api.hip) and the kernel files.
// Host-side launch functions take plain structs; no validation happens here.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned short bf16_t;  // raw bfloat16 bits

enum : unsigned {
    KF_BIAS = 1u,     // add bias in the epilogue
    KF_RELU = 2u,     // max(.,0) in the epilogue
    KF_OUT_F32 = 4u,  // final output stored as fp32 instead of bf16
    KF_DB = 16u,      // backward-filter: also sum the bias gradient (kernels that cannot leave db_done unset)
    KF_MASK_IN = 8u,  // backward-data: dx *= [x > 0], x = the layer's saved input (output of the preceding ReLU)
    KF_NT_A = 32u,    // forward / backward-data: every weight is read by one block only (a single pixel tile): non-temporal loads, the stream leaves the caches alone
    KF_NT_OUT = 64u,  // backward-filter: a large gradient written once: non-temporal stores
    KF_FUSED_REDUCE = 256u,  // forward / backward-data with a reduction split: the block that finishes a tile last adds the splits' partial sums itself
};

enum { PASS_FWD = 0, PASS_DGRAD = 1, PASS_WGRAD = 2 };

// Geometry of one conv layer plus its implicit-GEMM view for one pass.
//   fwd   : A rows = c_out,  B rows = output pixels (n,p,q), reduction = (r,s,c)
//   dgrad : A rows = c_in,   B rows = input pixels  (n,h,w), reduction = (r,s,k)
//   wgrad : A rows = c_out,  B rows = filter taps   (r,s,c), reduction = output pixels
// "A" / "B" are the matrix-core operands; D[i][j] has i over A rows, j over B rows.
struct ConvGeom {
    int N, H, W, C, K, R, S, sh, sw, ph, pw, Ho, Wo;
};

struct GemmPlan {
    int variant;          // tile variant index (see tile table in conv_mfma.hip)
    int TA, TB, BK;       // tile extents
    int tilesA, tilesB;   // tile counts
    int steps_total;      // reduction steps of BK
    int steps_per_split;  // steps handled by one split
    int splits;           // grid.y
    bool vecA, vecB;      // 16-byte loads allowed for operand A / B
    bool fast;            // fast-path kernel (conv_fast.hip) instead of the generic one
    bool dma;             // pipelined direct-to-LDS kernel (conv_dma.hip)
    bool halo = false;    // input-patch kernel (conv_halo.hip); implies dma
    int blocks = 0;       // persistent kernels: blocks per row tile (0: one per CU)
    bool phase = false;   // strided backward-data walks the input pixels stride phase by stride phase (conv_dma.hip)
    bool wstrip = false;  // filter gradient with the x strip shared by the taps of a filter row (conv_wstrip.hip); implies dma
    bool db_wave = false; // input-patch filter gradient: one more wave per block can sum the bias gradient (at most 15 taps)
    bool fused_reduce = false;   // pipelined forward / backward-data with splits > 1: no second kernel, the last block of a tile reduces (conv_dma.hip)
};

struct ConvArgs {
    ConvGeom g;
    GemmPlan plan;
    int pass;
    unsigned flags;
    const bf16_t *x;      // fwd: x       dgrad: saved input for KF_MASK_IN, else -        wgrad: x
    const bf16_t *w;      // fwd: w       dgrad: w        wgrad: -
    const bf16_t *dy;     // fwd: -       dgrad: dy       wgrad: dy
    const bf16_t *ymask;  // saved post-ReLU output or nullptr (dgrad, wgrad)
    const float *bias;    // fwd
    void *out;            // fwd: y, dgrad: dx (bf16 or fp32), wgrad: dw (fp32)
    float *partial;       // [splits][rowsB][rowsA] (fwd/dgrad) or [splits][rowsA][rowsB] (wgrad)
    float *db_out = nullptr;      // KF_DB: bias gradient [rowsA]
    float *db_partial = nullptr;  // KF_DB: [splits][rowsA] scratch for split plans
    int db_rows = 0;              // > 0: db_partial holds this many rows of column sums from an earlier pointwise pass; the
                                  // split-reduce kernel adds them up into db_out (the main kernel does not touch them)
};

// dp_api.hip: timing hook of dp_trace_begin / dp_trace_end.  The launch function of every kernel family calls this right
// after it has enqueued the main kernel of a pass (before any split-reduce or column-sum kernel that follows).
void dp_trace_main_kernel_done(hipStream_t st);

// conv_wstrip.hip
hipError_t wstrip_init();
bool wstrip_plan(const ConvGeom &g, int force_splits, GemmPlan *pl);
hipError_t wstrip_launch(const ConvArgs &a, hipStream_t st);

// conv_mfma.hip
hipError_t mfma_init();                                      // raises dynamic LDS limits
void mfma_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *plan);
size_t mfma_partial_bytes(const ConvGeom &g, int pass, const GemmPlan &plan);
hipError_t mfma_launch(const ConvArgs &a, hipStream_t st);
void mfma_kernel_name(int pass, const GemmPlan &plan, char *name, size_t name_bytes);
// sums a.partial into a.out; with_db: also a.db_partial [splits][rowsA] into a.db_out (backward-filter)
hipError_t launch_split_reduce(const ConvArgs &a, int rowsA, int rowsB, hipStream_t st, bool with_db = false);

// conv_fast.hip : fast path for channel counts that are multiples of the reduction step
hipError_t fast_init();
bool fast_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *plan);
hipError_t fast_launch(const ConvArgs &a, hipStream_t st);
void fast_kernel_name(int pass, const GemmPlan &plan, char *name, size_t name_bytes);

// true if this backward-filter plan's kernel sums the bias gradient itself when KF_DB is set
bool plan_sums_bias_gradient(const GemmPlan &plan);

// conv_dma.hip : multi-stage direct-to-LDS pipeline (forward, c_in % 64 == 0)
hipError_t dma_init();
bool dma_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *plan);
hipError_t dma_launch(const ConvArgs &a, hipStream_t st);
void dma_kernel_name(int pass, const GemmPlan &plan, char *name, size_t name_bytes);

// conv_halo.hip : input patch with halo resident in LDS (stride 1, 64 reduction channels per tap)
hipError_t halo_init();
bool halo_plan(const ConvGeom &g, int pass, int force_variant, int force_splits, GemmPlan *plan);
hipError_t halo_launch(const ConvArgs &a, hipStream_t st);
bool dma_plan_is_strip(const GemmPlan &plan);   // the pixel-strip forward / backward-data kernels (no fused split reduction)
bool dma_fused_reduce_fits(int rowsA, int rowsB, int splits);
bool dma_plan_fuses_reduce(const GemmPlan &plan);   // the splits are summed by the main kernel: no reduction kernel follows
void halo_kernel_name(int pass, const GemmPlan &plan, bool masked, char *name, size_t name_bytes);   // masked: backward-data with the fused input-ReLU mask

// conv_fp32.hip : plain fp32 FMA kernels (reference-precision path)
hipError_t f32_conv_fwd(const ConvGeom &g, unsigned flags, const float *x, const float *w,
                        const float *bias, float *y, hipStream_t st);
hipError_t f32_conv_dgrad(const ConvGeom &g, const float *dy, const float *ymask, const float *w, const float *xin,
                          float *dx, hipStream_t st);   // xin (may be NULL): dx *= [xin > 0]
hipError_t f32_conv_wgrad(const ConvGeom &g, const float *x, const float *dy, const float *ymask,
                          float *dw, hipStream_t st);

// pointwise.hip : ReLU-gradient / bias-gradient
size_t rbg_workspace_bytes(long long rows, int k);
hipError_t rbg_launch(long long rows, int k, bool bf16, const void *dy, const void *ymask,
                      void *g_out, float *dbias, float *ws, hipStream_t st);
// the first kernel only: column sums of `*row_blocks` row ranges in ws [row_blocks][k]; with one row block the sums
// go straight to dbias and nothing is left to add
hipError_t rbg_launch_partial(long long rows, int k, bool bf16, const void *dy, const void *ymask,
                              void *g_out, float *dbias, float *ws, hipStream_t st, int *row_blocks);
// sums ws [row_blocks][k] into dbias in row-block order
hipError_t rbg_launch_final(int k, int row_blocks, const float *ws, float *dbias, hipStream_t st);

// planner.hip : picks the cheapest fast-path variant and split for a pass (host-side cost model)
bool auto_plan(const ConvGeom &g, int pass, int force_splits, GemmPlan *plan, int restr = 0);
// the cheapest plans by the model, best first (input of the measured choice); returns the count
// restr: kernels the call may not use (bit 0: input-patch kernels, bit 1: the stationary-weight kernel)
int auto_plan_list(const ConvGeom &g, int pass, int force_splits, GemmPlan *out, int max_out, int restr = 0);

// small_c.hip : explicit im2col for layers with very few input channels (c_in % 8 != 0, R*S*C <= 256)
int small_c_kpad(const ConvGeom &g);   // padded reduction length, 0 if the layer does not qualify
hipError_t small_c_im2col(const ConvGeom &g, int kpad, const bf16_t *x, bf16_t *xcol, hipStream_t st);
hipError_t small_c_pad_weights(const ConvGeom &g, int kpad, const bf16_t *w, bf16_t *wpad, hipStream_t st);
hipError_t small_c_unpad_dw(const ConvGeom &g, int kpad, const float *dwpad, float *dw, hipStream_t st);
// direct kernels without the im2col matrix (R*S*C <= 32, c_out % 8 == 0)
// dense_stream.hip: 1x1 layers over a few pixel rows (dense layers at small batch), one launch per pass that streams the weights
bool dense_fwd_stream_shape(const ConvGeom &g);
hipError_t dense_fwd_stream(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y, hipStream_t st);
bool dense_wgrad_stream_shape(const ConvGeom &g);
const char *dense_fwd_stream_name(const ConvGeom &g);     // kernel names as a profiler prints them
const char *dense_wgrad_stream_name(const ConvGeom &g);
hipError_t dense_wgrad_stream(const ConvGeom &g, const bf16_t *x, const bf16_t *dy, float *dw, float *db, hipStream_t st);
bool dense_dgrad_stream_shape(const ConvGeom &g);
hipError_t dense_dgrad_stream(const ConvGeom &g, unsigned flags, const bf16_t *dy, const bf16_t *w, const bf16_t *xin, void *dx, hipStream_t st);
bool small_c_direct(const ConvGeom &g);
hipError_t small_c_fwd_direct(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y,
                              hipStream_t st);
// strided stems (7x7 stride 2 on RGB): forward straight from the input patch, no im2col matrix
bool small_c_stem(const ConvGeom &g);
hipError_t small_c_fwd_stem(const ConvGeom &g, unsigned flags, const bf16_t *x, const bf16_t *w, const float *bias, bf16_t *y, hipStream_t st);
int small_c_wgrad_blocks(const ConvGeom &g, bool masked);   // pixel-range blocks, each writes one fp32 partial (masked: a saved output is applied to dy)
const char *small_c_wgrad_kernel(const ConvGeom &g, bool masked, bool with_db);   // name of the kernel that runs, as a profiler prints it
const char *small_c_fwd_kernel(const ConvGeom &g);
size_t small_c_wgrad_partial_bytes(const ConvGeom &g);
// ymask (saved output, may be NULL) masks dy on the fly; db (may be NULL) receives the bias gradient of the masked dy
hipError_t small_c_wgrad_direct(const ConvGeom &g, const bf16_t *x, const bf16_t *dy, const bf16_t *ymask, float *partial, float *dw,
                                float *db, hipStream_t st);
