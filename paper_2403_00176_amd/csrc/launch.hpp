// Launch table entries: one per executed group, produced at bind from concrete shapes, strides
// and arena offsets; consumed by sod2_run.  Pointers are kept as (space, index, byte offset)
// references because the arena, weight, input and output addresses arrive with each run.
#pragma once
#include <cstdint>
#include <cstring>

namespace sod2 {

enum Space { SP_NONE = 0, SP_ARENA, SP_WEIGHT, SP_INPUT, SP_OUTPUT };
struct Ref {
  int space = SP_NONE;
  int index = 0;           // position among the weights / inputs / outputs
  int64_t byte_off = 0;    // arena offset, plus any view offset
};

enum KernelKind { K_GEMM = 0, K_CONV, K_LAYERNORM, K_SOFTMAX, K_ELTWISE, K_POOL, K_REDUCE, K_OTHER, K_GATHER, K_APPEND,
                  K_ARGMAX, K_ATTENTION, K_NONZERO, K_SCATTER, K_RESIZE, K_CONCAT, K_RANGE, K_FILL, K_ONEHOT, K_TOPK, K_GROUPNORM, K_MAXUNPOOL, K_NMS };
enum Act { ACT_NONE = 0, ACT_RELU, ACT_GELU, ACT_SIGMOID };
enum GemmVariant { V_REGULAR = 0, V_FAT = 1, V_SKINNY = 2, V_SIMPLE = 3, V_SMALL = 4, V_XFAT = 5, V_GEMV = 6, V_DL0 = 10 };   // (a contraction with a LayerNorm prologue has one kernel per shape class: ln_gamma set)
// tiles of the direct-to-LDS contraction (variant = V_DL0 + tile): BM x BN x BK, ring stages
enum DlTile { DL_128x128x64_S3_W4 = 0, DL_128x128x64_S2_W4, DL_128x128x32_S3_W4, DL_128x128x64_S2_W8, DL_256x128x64_S2_W8,
              DL_256x128x32_S3_W8, DL_64x128x64_S3_W4, DL_64x64x64_S4_W4, DL_128x64x64_S3_W4, DL_128x128x64_S3_W8,
              DL_256x256x32_S3_W8, DL_64x64x64_S4_L8, DL_64x64x64_S4_L16, DL_128x128x64_S2_L16, DL_64x128x64_S3_L8, DL_256x256x64_S2_W8, DL_256x128x64_S3_W8,
              DL_64x64x64_S4_G2, DL_64x64x64_S3_G2, DL_64x64x64_S2_G4, DL_128x128x64_S2_G2, DL_64x64x64_S2_G2, DL_128x128x64_S2_W8G2, DL_128x128x64_S2_W8T, DL_128x128x64_S3_W8T, DL_TILES };   // _Gn: n wave groups split k inside the workgroup

// C[b0,b1,m,n] = act2( act1( scale * sum_k A[b0,b1,m,k] * B[b0,b1,k,n] + bias[n] ) + R[b0,b1,m,n] )
struct GemmArgs {
  const void* A; const void* B; void* C; const void* bias; const void* res;
  int M, N, K, nb0, nb1;
  long long a_sm, a_sk, a_sb0, a_sb1;
  long long b_sk, b_sn, b_sb0, b_sb1;
  long long c_sm, c_sn, c_sb0, c_sb1;
  long long r_sm, r_sn, r_sb0, r_sb1;
  float scale;
  int act1, act2;
  int a_vec, b_mode;       // a_vec: 16-byte loads along k allowed; b_mode 0 k-contiguous vec, 1 n-contiguous vec, 2 scalar
  int c_vec;               // c_sn == 1 and rows 4-byte aligned
  int splits;              // > 1: split-K, fp32 partials in ws, summed in z order by a second kernel
  int group_m;             // tile rows per panel of the tile walk (L2 locality)
  void* ws;                // split-K workspace: splits x batch x M x N floats
  const int* step;         // replay (skinny kernel only): C advances by *step * c_step elements
  long long c_step;
  const void* ln_gamma;    // LayerNorm prologue over the rows of A (all of K), or null
  const void* ln_beta;
  float ln_eps;
  // A LayerNorm over the result's rows as a second result (fold == 1), read back by the contraction that consumes it
  // (fold == 2).  The second result is xg = bf16(x * gamma) (x the rounded first result, rows of N elements) and, behind
  // its M x N elements, per run of 32 columns and row ([N / 32][M]) the pair (sum of x, sum of squared distances from the mean of those 32).
  // The consumer multiplies xg by its weights and finishes the normalisation in its epilogue:
  // out = scale * rstd * (acc - mean * fold_s[n]) + fold_c[n], with fold_s[n] = sum_k gamma[k] W[n][k] and
  // fold_c[n] = scale * sum_k beta[k] W[n][k] + bias[n], both fp32, derived from the weights once.
  int fold;                // 0 plain, 1 emits the second result, 2 reads one
  void* fold_y;            // fold 1: xg, then the statistics
  const void* fold_gamma;  // fold 1: gamma of the LayerNorm (N elements, the first result's type)
  const void* fold_s;      // fold 2
  const void* fold_c;
};

// Optional workspace behind the planned arena (fp32 partial tiles of split-K contractions)
constexpr long long WS_PARTIAL_BYTES = 16 << 20;
constexpr long long WS_BYTES = WS_PARTIAL_BYTES;

// NHWC implicit GEMM: M = N*OH*OW, Ncol = O, K = KH*KW*C
struct ConvArgs {
  const void* x; const void* w; void* y; const void* bias; const void* res;
  int NB, H, W, C, O, KH, KW, stride, pad, OH, OW;
  int act1, act2;
  int vec;                 // C % 8 == 0 (16-byte loads along channels)
  int splits;              // > 1: split-K over (kh, kw, c) as in GemmArgs, partials in ws
  void* ws;
};

struct RowArgs {            // LayerNorm / Softmax over the last dim
  const void* x; void* y; const void* gamma; const void* beta;
  long long rows; int cols; long long x_stride, y_stride;
  float eps;
  int causal, lq;          // softmax: row index within its [lq, cols] matrix = row % lq
};

struct ReduceArgs {         // y[b, c] = mean_r x[b, r, c]
  const void* x; void* y;
  int batch; long long R; int C;
};

struct PoolArgs {
  const void* x; void* y;
  int NB, H, W, C, OH, OW, k, stride, pad;
  int avg;                 // 0: maximum of the window; 1: mean over the window positions inside the input
};

// out[idx] = chain of up to 8 elementwise operators over the output index space; operands are
// broadcast through zero strides (the single fused loop nest of Fig. 4)
enum EltOp { E_ADD = 0, E_MUL, E_RELU, E_GELU, E_SIGMOID, E_CAST, E_ROUND, E_CAST_BF16 };   // E_CAST_BF16: round to bf16 (a Cast inside a chain)
struct EltArgs {
  const void* in[5];
  void* out;
  long long stride[5][6];
  long long dims[6];
  long long total;
  int in_bf16[5];
  int rank, n_ops, n_in;
  int op[8], src[8];       // src: operand slot of a binary operator, 5 = immediate, -1 = unary
  float imm[8];
};

// y[r, :] = table[idx[r], :] (+ add[r, :]); an index outside the table is clamped into it
struct GatherArgs {
  const void* table; const void* idx; const void* add; void* y;
  long long rows, table_rows, add_stride;
  int cols, idx_i32;
  const int* step;         // replay: idx advances by *step * idx_step bytes
  long long idx_step;
};

// cache[past + r, :] = x[r, :] for r < rows (the in-place CacheAppend of a session tensor)
struct AppendArgs {
  const void* x; void* cache;
  long long rows, past, x_stride;
  int cols;
  const int* step;         // replay: past grows by *step * past_step rows
  long long past_step;
};

// y[r] = index of the largest x[r, :], the lowest index among equals
struct ArgmaxArgs {
  const void* x; void* y;
  long long rows, x_stride;
  int cols, out_i32;
  const int* step;         // replay: x and y advance by *step * x_step / y_step bytes
  long long x_step, y_step;
};

// O[b0,b1,q,:] = softmax_k(scale * Q[b0,b1,q,:] . K[b0,b1,k,:] (+ causal mask)) V[b0,b1,k,:], head size 64,
// last dim dense; strides in elements
struct AttnArgs {
  const void* q; const void* k; const void* v; void* o;
  int Lq, Lk, nb0, nb1, causal;
  float scale;
  long long q_sb0, q_sb1, q_sm;
  long long k_sb0, k_sb1, k_sn;
  long long v_sb0, v_sb1, v_sn;
  long long o_sb0, o_sb1, o_sm;
  const int* step;         // replay: Lk grows by *step * lk_step keys
  int lk_step;
  // cache append inside the few-query kernel: the last n_new of the Lk keys are new; their rows are read
  // from new_k / new_v ([n_new, heads * 64], row strides in elements) and written to rows Lk - n_new .. of k / v
  const void* new_k; const void* new_v;
  int n_new;
  long long new_k_sn, new_v_sn;
};

// NonZero (Table 2's EDO class): out[r, j] = r-th coordinate of the j-th non-zero element of x in
// row-major order, rows of `count` entries; the count goes to *count (8 bytes behind the indices'
// upper-bound storage).  One workgroup; x has n elements and rank <= 4.
struct NonzeroArgs {
  const void* x; long long* out; long long* count;
  long long n;
  int rank, x_kind;          // x_kind: 0 f32, 1 bf16, 2 i64, 3 i32
  long long dims[4];
};

// Non-maximum suppression (Table 2's EDO class): boxes visited by decreasing score (equal scores by increasing
// index), kept unless an already kept box overlaps them by more than `iou`; out[j] = index of the j-th kept box,
// *count = how many (8 bytes behind the upper-bound storage of n indices).  One workgroup, n <= NMS_MAX_BOXES.
constexpr int NMS_MAX_BOXES = 4096;
struct NmsArgs {
  const float* scores; const float* boxes; long long* out; long long* count;
  int n, max_out;
  float iou;
  char* ws;                  // the workspace (WS_BYTES) or null: with it, many boxes go through three kernels
};

// out = x with the rows idx[j] replaced by y[j] (j < n; the last j wins on duplicates); rows of
// `cols` elements, everything dense
struct ScatterArgs {
  const void* x; const void* idx; const void* y; void* out;
  long long rows, n, cols;
  int idx_i32;
};

// Nearest-neighbour Resize of a dense tensor [d0, d1, d2, c] -> [o0, o1, o2, c] (the last dim is kept):
// out[i0, i1, i2, :] = x[floor(i0 * d0 / o0), floor(i1 * d1 / o1), floor(i2 * d2 / o2), :]
struct ResizeArgs {
  const void* x; void* y;
  long long in[3], out[3];
  long long row_units;       // copy units (16 bytes or one element) per innermost vector
};

// Concat of up to 4 dense tensors along one axis, seen as rows (the dims before the axis) of runs (the axis and the
// dims behind it): out[r, :] = x0[r, :] | x1[r, :] | ...
struct ConcatArgs {
  const void* x[4]; void* y;
  long long rows;
  long long units[4];        // copy units per row of each input (0 beyond n_in)
  int n_in;
};

// y[i] = start + i * delta for i < n (int64 or int32 result)
struct RangeArgs {
  void* y;
  long long start, delta, n;
  int out_i32;
};

// y[i] = value everywhere (cols == 0), or an identity pattern: 1 where column == row + diag, else 0
struct FillArgs {
  void* y;
  long long n, cols, diag;
  float value;
  int dtype;               // SOD2_F32 / SOD2_BF16 / SOD2_I64 / SOD2_I32
};

// y[i, d] = (index[i] == d, negative indices counted from depth) ? on : off
struct OneHotArgs {
  const void* idx;
  void* y;
  long long n, depth;
  float on, off;
  int idx_i32, out_bf16;
};

// per row of n entries: the k largest, largest first (of equal entries the lower position first), and
// their positions
struct TopKArgs {
  const void* x;
  void *values, *indices;
  long long rows, n, k;
  int x_bf16, idx_i32;
};

// MaxUnpool: y (n_out elements) = 0 except y[idx[i]] = x[i] for the n_in elements of x
struct UnpoolArgs {
  const void* x; const void* idx; void* y;
  long long n_in, n_out;
};

// GroupNormalization, channels last: x[n, s, c] with s positions and C = groups * cpg channels, dense;
// y = (x - mean(n, g)) / sqrt(var(n, g) + eps) * gamma[c] + beta[c], statistics over the s * cpg elements of a group
struct GroupNormArgs {
  const void* x; void* y; const void* gamma; const void* beta;
  long long n, s;
  int groups, cpg;
  float eps;
};

struct Launch {
  int group = -1;
  int kernel = K_OTHER;
  int variant = 0;
  int in_dtype = 0, out_dtype = 0;
  Ref r[10];               // operand references, meaning depends on the kernel
  union {
    GemmArgs gemm;
    ConvArgs conv;
    RowArgs row;
    ReduceArgs red;
    PoolArgs pool;
    EltArgs elt;
    GatherArgs gather;
    AppendArgs append;
    ArgmaxArgs argmax;
    AttnArgs attn;
    NonzeroArgs nz;
    ScatterArgs scatter;
    ResizeArgs resize;
    ConcatArgs concat;
    RangeArgs range;
    FillArgs fill;
    OneHotArgs onehot;
    TopKArgs topk;
    GroupNormArgs gn;
    UnpoolArgs unpool;
    NmsArgs nms;
  } u;
  int unit_bytes = 0;      // resize / concat: bytes of one copy unit
  bool is_layernorm = false;
  double flops = 0, bytes = 0;
  long long d_past = 0;    // replay: rows the CacheAppend position / keys the attention length gain per step
  int d_lk = 0;
  bool empty = false;      // the group's result has no elements: nothing is launched
  // a contraction whose group holds a LayerNorm of its result (r[7] the LayerNorm's result, r[8] gamma, r[9] beta):
  // post_ln: the LayerNorm's row kernel runs right behind the contraction, or, with fold_pair (both contractions of the
  // pair run kernels that can), the contraction emits the second result itself.  fold_read: the contraction whose first
  // operand is such a second result; const_off: where its derived constants start in the plan's constants buffer.
  bool post_ln = false, fold_pair = false, fold_read = false;
  long long const_off = -1;
  RowArgs post;
  Launch() { std::memset(&u, 0, sizeof u); }
};

}  // namespace sod2
