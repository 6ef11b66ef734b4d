// Host-side declarations shared by the translation units of libhot: argument
// checks, workspace layouts and the launchers each .hip file defines.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "hot.h"

namespace hot {

inline int64_t round_up(int64_t a, int64_t b) { return (a + b - 1) / b * b; }
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

// Position of every natural-order row of an n-block in the kept list (-1 = dropped).
struct KeepMap {
  int8_t pos[64];
};

// How the token rows of a tensor are cut into blocks of n for the token-direction
// transform: one contiguous run (S = 0), or samples of S tokens each tiled separately, the
// last block of a sample padded with zero tokens (bps blocks per sample).
struct RowTiling {
  int64_t nblk;   // blocks in the whole tensor
  int64_t S;
  int bps;
};

// Validated, resolved form of hot_config.
struct Config {
  int n, r, gx_bits, gw_bits, rounding;
  int64_t sample_tokens;   // 0 = the whole token axis is one run
  float lqs_threshold;
  int keep[64];   // r natural-order indices, in output order
  KeepMap map;    // inverse of keep
  bool lowpass_default;
  bool replayable;   // launch tags derived from the workspace epoch (HIP graph replays)
  const unsigned long long* epoch;   // device address of that epoch for the current call, or null
};

hot_status resolve_config(const hot_config* cfg, Config* out);
// Blocks of the token axis of an L-token tensor (nblk = 0 when L does not fit the tiling).
RowTiling row_tiling(const Config& c, int64_t L);

// K-contiguous operand rows are padded with zero codes to a multiple of 128 bytes.
constexpr int64_t kPitchAlign = 128;
constexpr int64_t kHeaderBytes = 256;
// Every workspace starts with 256 bytes of scalars (scales, results), two arrays
// of per-workgroup partial maxima and the flags of a split-K GEMM's partial sums.
constexpr int64_t kPartialBytes = 2048 * 4;
// Offset of the 64-bit epoch among the scalars (used by replayable calls only).
constexpr int64_t kEpochOffset = 128;
constexpr int kMaxSplitSlots = 1024;
constexpr int64_t kGemmFlagsOffset = kHeaderBytes + 2 * kPartialBytes;
constexpr int64_t kWsPrefix = kGemmFlagsOffset + kMaxSplitSlots * 8;
static_assert(kWsPrefix == HOT_WS_PREFIX_BYTES, "hot.h documents the prefix size");
// |code products| summed over K must fit int32 (INT4 operands are fed to the
// matrix cores as 16 x code, so their bound carries a factor 256).
constexpr int64_t kMaxK8 = 133144;   // 127^2 * K < 2^31
constexpr int64_t kMaxK4 = 171196;   // 256 * 7^2 * K < 2^31

// Tile shape and K split of one GEMM launch.
struct GemmPlan {
  int bm, bn, bkb;
  int split;              // workgroups (K slices) per output tile
  int64_t tiles;
  size_t partial_bytes;   // split > 1: tiles * (split - 1) * bm * bn int32
};
// `scratch`: a region of gemm_scratch_bytes() and the workspace's flag slots are available,
// so K may be split.
GemmPlan plan_gemm(int64_t M, int64_t N, int64_t k_bytes, int bits, bool scratch);
// Upper bound of partial_bytes over every plan of this shape (whatever mode is forced).
size_t gemm_scratch_bytes(int64_t M, int64_t N, int64_t k_bytes, int bits);
// Measurement / test overrides: 0 = cost model, 1 = one workgroup per tile, s >= 2 = s K
// slices wherever a split applies; bound of the wait for another workgroup's image (0:
// never wait).
void set_gemm_mode(int mode);
void set_gemm_wait_us(int us);

struct GxLayout {
  int64_t pitch;                      // bytes per operand row (K = O codes)
  size_t scalars, sg, qg, qw, partial, total;  // byte offsets into ws
};
struct GwLayout {
  int64_t Lr, pitch;                  // reduced token count, bytes per operand row
  size_t scalars, qg, partial, total;
};
// hot_linear_backward: the g_x layout first (so its operand view applies unchanged),
// then the per-token abs-max partials and the g_w operands.
struct FusedLayout {
  GxLayout gx;
  GwLayout gw;                        // pitch only; offsets below
  size_t s_gh, rowpart, qgh, partial, total;
};
struct SelLayout {
  size_t scalars, rowmax, partial, total;
};
struct WeightLayout {
  int64_t pitch;
  size_t codes, total;
};
struct ActLayout {
  int64_t Lr, pitch;
  size_t codes, total;
};

GxLayout gx_layout(const Config& c, int64_t L, int64_t O, int64_t I);
GwLayout gw_layout(const Config& c, int64_t L, int64_t O, int64_t I);
SelLayout sel_layout(const Config& c, int64_t L, int64_t O);
FusedLayout fused_layout(const Config& c, int64_t L, int64_t O, int64_t I);
ActLayout act_layout(const Config& c, int64_t L, int64_t I);
WeightLayout weight_layout(const Config& c, int64_t O, int64_t I);


// Kernel roles for the optional stage timer (names in profile.hip).
enum Stage {
  kStUnused = 0, kStActAbsmax, kStActQuant, kStWAbsmax, kStWQuant, kStGyRowQuant, kStGyRowAbsmax,
  kStGyRowQuant2, kStGxGemm, kStGyTAbsmax, kStGyTQuant, kStGwGemm, kStWGyRow, kStGyFusedAbsmax,
  kStGyFusedQuant
};
void stage_begin(int stage, hipStream_t s);
void stage_end(int stage, hipStream_t s);

// ---- launchers (each returns hipGetLastError() of its launches) -------------

// Abs-max passes leave up to kMaxPartials per-workgroup maxima; consumers reduce them.
constexpr int kMaxPartials = 2048;
// The single-pass kernels exchange maxima through the same array: two 64-bit words per
// workgroup (each carries half of the launch tag and the value).
constexpr int kMaxExchange = kMaxPartials / 4;

// Row-direction block WHT + quantise of t [rows x cols] (cols % n == 0).
//   mode 0: per-token: codes + scales[rows].
//   mode 1: abs-max of the rotated tensor: partials[0..*npartials) written.
//   mode 2: quantise with the tensor-wide abs-max = max(partials); scales[0] written.
//   mode 3: abs-max per row into scales[rows] and tensor-wide into partials.
// codes: rows x pitch bytes, `bits` = 4 (two codes per byte, even index in the
// low nibble) or 8; bytes from cols*bits/8 up to pitch are zero-filled.
// *npartials is written by modes 1/3 (host value) and read by mode 2.
hipError_t launch_row_quant(const float* t, int64_t rows, int64_t cols, int n, int bits,
                            int rounding, int mode, uint8_t* codes, int64_t pitch, float* scales,
                            float* partials, int* npartials, hipStream_t s);

// Column-direction block WHT (blocks of n rows of x [. x C], cut as `rows` says), keep r
// rows per block, one scale for the tensor; output transposed: row c of `codes`
// holds the kept values of column c, reduced row index contiguous.  Runs the single-pass
// kernel when the tensor fits it (timed as stage_quant), else the abs-max pass and the
// quantise pass; `partials` is kMaxPartials floats of scratch either way;
// *scale is written, pad bytes up to `pitch` are zero-filled.  `identity` says the
// kept list is 0..n-1 (required for bits == 4).
hipError_t launch_col_quant(const float* x, const RowTiling& rows, int64_t C, const Config& cfg, int r,
                            const KeepMap& map, bool identity, int bits, uint8_t* codes,
                            int64_t pitch, float* scale, float* partials, hipStream_t s,
                            int stage_absmax, int stage_quant);

// Both views of g_y [L x O] from shared reads (block sizes 16 and 32): token rows
// rotated along O -> qg [L x pitch_g] with scales sg ([L] per token, [1] per tensor),
// and the HLA view along L -> qgh [O x pitch_h] with scale s_gh.  part_hla / part_row:
// kMaxPartials floats each; rowpart: gy_fused_tiles_x(O) * L floats (per token only).
bool gy_fused_supported(const Config& c);
int64_t gy_fused_tiles_x(int64_t O);
hipError_t launch_gy_fused(const float* g_y, int64_t L, int64_t O, const Config& cfg, bool per_token,
                           uint8_t* qg, int64_t pitch_g, float* sg, uint8_t* qgh, int64_t pitch_h,
                           float* s_gh, float* part_hla, float* part_row, float* rowpart,
                           hipStream_t s, int stage_absmax, int stage_quant);

// bfloat16 form of the same transposed low-rank operand (g_w path with gw_bits = 16):
// out row c holds the kept values of column c as bfloat16; *scale is set to 1.
hipError_t launch_col_bf16(const float* x, const RowTiling& rows, int64_t C, const Config& cfg, uint8_t* out,
                           int64_t pitch, float* scale, hipStream_t s, int stage);

// Bounded wait of the single-pass column kernel (microseconds; < 0: always two passes), and
// the launch tags of its abs-max exchange (never repeated while stale slots may survive).
void set_exchange_wait_us(int us);
int exchange_wait_us();
uint64_t next_exchange_tag();

// Both operands of the g_x GEMM from one launch, where that exists (INT4, per-token g_y
// scales, weights small enough for the single-pass column kernel, O between 257 and 4096):
// Q(H.w) as [I x pitch] code rows with *s_w, and the rotated, per-token quantised g_y as
// [L x pitch] code rows with s_g[L].  `slots`: kMaxPartials floats of scratch.  *done says
// whether the launch was made; when not, nothing was written.
hipError_t launch_w_and_rows(const float* w, int64_t O, int64_t I, const Config& cfg, uint8_t* qw,
                             int64_t pitch, float* s_w, float* slots, const float* g_y, int64_t L,
                             uint8_t* qg, float* s_g, hipStream_t s, int stage, bool* done);

// C[M x N] = A[M x K] . B[N x K]^T on K-contiguous code rows (pitch bytes each,
// k_bytes = K * bits / 8 rounded up to the pitch alignment).
//   out_i32 != NULL: raw int32 accumulators, row-major [M x N].
//   out_f32 != NULL: out = acc * row_scale[m * row_stride] * (*col_scale) / n.
// plan.split > 1 needs `partial` (plan.partial_bytes) and `flags` (kMaxSplitSlots slots
// that only such launches ever write).  `epoch`: device address of the workspace epoch when
// the launch tag is to be derived from it (replayable calls), else null.
hipError_t launch_igemm(const uint8_t* A, const uint8_t* B, int64_t M, int64_t N, int64_t k_bytes,
                        int64_t pitch, int bits, const GemmPlan& plan, int32_t* partial,
                        unsigned long long* flags, int32_t* out_i32, float* out_f32,
                        const float* row_scale, int row_stride, const float* col_scale, int n,
                        hipStream_t s, int gemm_stage = -1, const unsigned long long* epoch = nullptr);

// Unpack K-contiguous codes [rows x pitch] into one int8 per code.
//   transpose = 0: out[row * K + k];  transpose = 1: out[k * rows + row].
hipError_t launch_unpack(const uint8_t* codes, int64_t rows, int64_t K, int64_t pitch, int bits,
                         int transpose, int8_t* out, hipStream_t s);

// Squared quantisation error of the rotated t [rows x cols] with per-token and
// per-tensor scales (rowmax[rows] and partials from launch_row_quant mode 3):
// result[0] = sum per-token, result[1] = sum per-tensor (double, fixed order).
hipError_t launch_quant_error(const float* t, int64_t rows, int64_t cols, int n, int bits,
                              int rounding, const float* rowmax, const float* partials,
                              int npartials, double* partial, double* result, hipStream_t s);

}  // namespace hot
