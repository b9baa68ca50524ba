// Internal interface between the host state machine (easyspec.cpp) and the gfx950 kernels
// (gemv.hip, attention.hip, util.hip, accept.hip).  Plain structs and launch functions; no device code in this header.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace es {

constexpr int kMaxCols = 16;  // token columns of one forward pass (= one MFMA N tile)
constexpr int kMaxChunks = 64;  // split-KV chunks per (column, head)

// Which (sequence, position, token) each column of a forward pass stands for.
struct Cols {
  int32_t n;
  int32_t seq[kMaxCols];
  int32_t pos[kMaxCols];        // slot the column writes; the highest slot it attends to
  int32_t rope_pos[kMaxCols];   // its rotary position (= pos except for the nodes of a token tree)
  // Visibility of slots 0..pos: every slot below vis_base, and slot vis_base + i iff bit i of
  // vis_mask (pos < vis_base + 64).  Causal columns: vis_base = pos + 1.
  int32_t vis_base[kMaxCols];
  unsigned long long vis_mask[kMaxCols];
  int32_t tok_idx[kMaxCols];    // index into the caller's token array
  int32_t logit_row[kMaxCols];  // row of logits_out to write, or -1
  int32_t out_idx[kMaxCols];    // index of tokens_out to write, or -1
};

struct Shape {
  int32_t dtype;  // 0 fp32, 1 bf16
  int32_t L, d, Hq, Hkv, hd, F, V;
  int32_t HQ;     // Hq*hd
  int32_t RQKV;   // (Hq + 2 Hkv) * hd
  int32_t B, max_ctx;
  float eps;
  int32_t has_bias;
  int32_t R_ffn;  // rows per weight tile of the gate and up matrices (tile_rows(F))
  int32_t R_qkv;  // rotation pairs per tile of the QKV matrices (qkv_tile_rows); every other matrix: tiles of 16 rows
};

// Device buffers of a context.  "T" = storage dtype.  Activation arrays in T hold two parts
// [hi | lo] per slot when T is bf16 (the value is hi + lo), one part when T is fp32.  Packed matrices are arrays of 1 KB tiles
// (16 rows x 16 bytes per lane-group, see device_common.hpp) ordered [layer][row tile][k tile].
struct Buffers {
  // weights
  void *wqkv, *wo, *wg, *wu, *wd, *wlm;  // packed tiles
  void *embed;                           // plain [V][d] T
  float *bqkv;                           // [L][RQKV] or null
  float *g_attn, *g_mlp, *g_final;       // [L][d], [L][d], [d]
  float2 *rope;                          // [max_ctx][hd/2] (cos, sin)
  // cache
  void *kc, *vc;  // [L][B][Hkv][max_ctx][hd] T
  // workspaces (per forward pass).  fp32 arrays are [.][kMaxCols][width].  Arrays in T are operands of
  // the next weight contraction: per part either plain rows [column][width] (passes of one or two
  // columns) or 1 KB tiles of KT consecutive k holding [k-group][column][EPL elements], the order of
  // a wave's B fragments (see xoff() in device_common.hpp); a slot of XA / AO is PARTS * 16 * width elements.
  float *H;     // [16][d]      residual stream
  float *ssp;   // [16][d/16]   per-row-tile partial sums of squares of the vector to be normed next
  float *ssp_set;  // [MAX_SET][16][d/16]  the same per layer of a set (full-layer mode: one MLP input per layer)
  void *XA;     // [MAX_SET] x (16 x d) T   H * g_attn(layer) for the layers of the coming set (or g_final)
  void *XM;     // [MAX_SET] x (16 x d) T   H' * g_mlp(layer); one slot outside full-layer mode
  float *Q;     // [MAX_SET][16][HQ]    rotated queries
  void *AO;     // [MAX_SET] x (16 x HQ) T  attention output (rounded to T)
  float *A;     // [MAX_SET][16][d]     Attnoutput_i
  void *ACT;    // [MAX_SET] x (16 x F) T   SiLU(gate)*up; one slot outside full-layer mode
  float *PO;    // [MAX_SET*16*Hq][kMaxChunks][hd]  split-KV partial outputs
  float *PM, *PL;  // [MAX_SET*16*Hq][kMaxChunks]   partial max / sum
  float *amax_val; // [16][n_head_blocks]
  int32_t *amax_idx;
};

// Per-launch timing (easyspec_profile_*): while a timer is installed for the calling thread, every kernel
// launch of the forward pass binds the next start / stop event pair to its own dispatch, so that the pair's
// elapsed time is the kernel's begin-to-end time as a kernel trace reports it (no stream markers between).
struct LaunchTimer {
  hipEvent_t* ev;   // start / stop pairs
  int8_t* op;       // kernel class of the launch that took pair i (EASYSPEC_OP_*), one entry per pair
  size_t cap, used;
  int cur_op;       // class of the launches made right now
};
extern thread_local LaunchTimer* g_launch_timer;

// How one launch of a weight-streaming kernel class (EASYSPEC_OP_QKV, _OPROJ, _GATEUP, _DOWN, _HEAD) cuts its
// packed matrices: decided in one place (stream_plan) for the launch wrappers and for stream_walk.
struct StreamPlan {
  int op;
  int n_mat;        // packed matrices a unit reads side by side: QKV 2 (first and second rotary halves), gate/up 2, else 1
  int split_array;  // 1: the n_mat matrices are separate arrays of the same tiling (gate, up); 0: one array, one after the other
  int units;        // units per layer: row tiles, or tiles of rotation pairs
  int TP;           // units per workgroup
  int R;            // rows per tile
  int K, nkt;       // contraction length, k-tiles
  int nw;           // waves per workgroup
  int NB;           // activation fragments per k-tile
  int n_layers;     // layers the grid spans
  int grid;
  size_t mat_pieces;    // 16-byte pieces of one packed matrix of one layer
  size_t layer_pieces;  // pieces from one layer to the next inside an array
};
StreamPlan stream_plan(const Shape& s, int op, int ncols, int n_layers, bool full_layer);
// What a host walk of the launch found: the highest piece index against the pieces the launch's layers
// hold, the highest activation element against an operand slot, k-tiles never read, read twice (apart
// from the deliberate re-reads of a missing last unit), and fragment pieces no lane takes.
struct StreamWalk {
  long long w_max, w_pieces, w_out_of_range;
  long long x_max, x_slot_elems, x_out_of_range;
  long long tiles, missed_tiles, repeated_tiles, reread_tiles, uncovered_pieces;
};
int stream_walk(const Shape& s, const StreamPlan& p, int ncols, StreamWalk* r);

// Launch wrappers (all asynchronous on `st`).
// Packed matrices: row tiles of R <= 16 rows (see repack_kernel).
int tile_rows(int rows);
int qkv_tile_rows(int n_pairs);
size_t packed_bytes(int dtype, int rows, int K, int R);
// half = 0: packed row r is source row r; half > 0: source row (r / half) * 2 * half + r % half + row_add
void launch_repack(int dtype, const void* src, void* dst, int rows, int K, int R, int half, int row_add, hipStream_t st);
void launch_embed(const Shape& s, const Buffers& b, const Cols& c, const int32_t* tokens, int layer0, int n_set,
                  hipStream_t st);
// The weight kernels take an optional second pass (b2, c2: its workspaces and columns, c2->n == c.n): one launch then
// serves both passes, every wave using each weight fragment it loads for both passes' columns
// (twin_passes_fit(): whether the launch shapes of passes of n_cols columns allow it).
bool twin_passes_fit(const Shape& s, int n_cols);
void launch_qkv(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st,
                const Buffers* b2 = nullptr, const Cols* c2 = nullptr);
// How an attention launch over n_set layers cuts the contexts of these columns into split-KV chunks.
struct AttnCut {
  bool mfma;     // the matrix-core kernel takes the launch (groups of columns of one sequence)
  int n_chunks;  // chunks of the longest column = grid extent; 1: every context in one piece, no merge launch
  int chunk;     // matrix-core kernel: slots per chunk (fixed length)
  int nb_ref;    // vector kernel: batches of the longest column; shorter columns get proportionally fewer chunks
};
AttnCut attn_cut(const Shape& s, const Cols& c, int n_set);
AttnCut attn_cut_vector(const Shape& s, const Cols& c, int n_set);  // the cut the vector kernel would get
// Host evaluation of the kernels' own index arithmetic for a vector-kernel cut: the chunk count of a
// column of n_slots slots and the slots [w0, w1) that wave `wave` of chunk `chunk` works through
// (empty beyond the column's chunks); attn_waves: waves per workgroup of the launch.
int attn_waves(const AttnCut& cut);
void attn_ranges(const Shape& s, const AttnCut& cut, int n_slots, int chunk, int wave, int* nch, int* w0, int* w1);
void launch_attn(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const AttnCut& cut, hipStream_t st);
// O projection of the set's layers; the first layer's result goes straight into the residual.
void launch_oproj(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st,
                  const Buffers* b2 = nullptr, const Cols* c2 = nullptr);
// Gate/up of n_layers consecutive layers, layer i on operand slot i of XM with partial sums slot i
// of ssp ([n_layers][16][d/16]) into operand slot i of ACT.  n_layers = 1 outside full-layer mode.
void launch_gateup(const Shape& s, const Buffers& b, const Cols& c, int layer, int n_layers, const float* ssp, hipStream_t st,
                   const Buffers* b2 = nullptr, const Cols* c2 = nullptr, const float* ssp2 = nullptr);
// Full-layer-parallel mode (App. B ablation), per set: the O projections (every layer parks its
// Attnoutput and writes its own MLP's input into XM / ssp_set) and the down projections (summed
// over the set's layers and added to the residual together with the Attnoutputs).
void launch_oproj_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, hipStream_t st);
void launch_down_full(const Shape& s, const Buffers& b, const Cols& c, int layer0, int n_set, const float* gain, int n_gain,
                      void* xout, hipStream_t st);
// Down projection + residual.  a_next: Attnoutput of the next layer of the same set to add, or
// -1.  The normed-input vectors for what comes next are written with gains
// gain[0..n_gain) (stride d) into xout (stride 16*d elements of T).
void launch_down(const Shape& s, const Buffers& b, const Cols& c, int layer, int a_next, const float* gain,
                 int n_gain, void* xout, hipStream_t st, const Buffers* b2 = nullptr, const Cols* c2 = nullptr,
                 void* xout2 = nullptr);
void launch_head(const Shape& s, const Buffers& b, const Cols& c, float* logits_out, int32_t* tokens_out,
                 hipStream_t st, const Buffers* b2 = nullptr, const Cols* c2 = nullptr);
void launch_accept(const int32_t* draft, const int32_t* target, int batch, int gamma, int32_t* accept_len,
                   int32_t* bonus, hipStream_t st);
// Acceptance by speculative sampling; ws: sample_accept_workspace_bytes() of scratch.
size_t sample_accept_workspace_bytes(int batch, int gamma, int V);
void launch_sample_accept(const int32_t* draft, const float* draft_logits, const float* target_logits, const float* r,
                          const float* u, int batch, int gamma, int V, double T, double* ws, int32_t* accept_len,
                          int32_t* bonus, hipStream_t st);
// The library's own workspace for launch_sample_accept (a static device array, one copy per GPU): its
// address on the current device (resolved at the first call there) and its size.  Allocates nothing.
hipError_t sample_accept_static_workspace(double** out);
size_t sample_accept_static_capacity_bytes();
// Reads `bytes` (multiple of 16) of buf once; sink: stream_read_sink_floats() floats.
void launch_stream_read(const void* buf, size_t bytes, float* sink, hipStream_t st);
int stream_read_sink_floats();
void launch_kv_copy(const Shape& s, const Buffers& b, int seq, void* k_user, void* v_user, int n_slots,
                    int to_cache, hipStream_t st);

}  // namespace es
