// Internal declarations shared by the host plan builder, the C ABI glue and
// the kernel launchers.  Not part of the public interface.
#pragma once

#include <cstddef>
#include <cstdint>
#include <string>
#include <vector>

#include "pivot_fc.h"

namespace pivot {

void set_error(const char* fmt, ...);

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int    elem_size(int wdtype) { return wdtype == PIVOT_F32 ? 4 : 2; }
// Zero bytes kept after the tile values on the device: kernels issue clamped,
// unconditional loads of up to one group of tiles (at most 64x64 fp32).
constexpr size_t kValsPadBytes = 16 * 1024;
constexpr int kSortSrcBits = 19;               // packed gather entry: source index below, staged position above
constexpr int kSortSrcNone = (1 << kSortSrcBits) - 1;

// Which MFMA shape a row-major fp16 tile feeds: 0 = 16x16x32, 1 = 32x32x16, -1 = none.
inline int mfma_kind(int wdtype, int bh, int bw) {
    if (wdtype != PIVOT_F16) return -1;
    if (bw % 32 == 0 && bh % 16 == 0) return 0;
    if (bh % 32 == 0 && bw % 16 == 0) return 1;
    return -1;
}

// Host-side canonical arrays of one layer (what pivot_plan_view exposes).
struct HostPlan {
    pivot_fc_desc d{};
    int nbr = 0, nbc = 0, M_pad = 0, K_pad = 0, T = 0, chunk_tiles = 0, nchunks = 0, wg_waves = 4, row_slices = 1;
    int max_parts = 1;                 // largest number of pieces of one block row
    int uniform_ct = 0, uniform_parts = 0;  // set when every block row keeps the same number of tiles and every
                                       // chunk is full: chunk i = tiles [i*ct, (i+1)*ct) of block row i / parts
    std::vector<int32_t> row_ptr, col_idx, invprow, invpcol, prow_pad, pcol_pad;
    std::vector<int32_t> xidx;         // T*bw: xidx[t*bw+c] = pcol_pad[col_idx[t]*bw+c]
    // Gather lists of the LDS-fed matrix-core kernel, one per work item (chunk), at [tile_begin*bw, tile_end*bw):
    // the chunk's staged elements e = t*bw+c ordered by ascending source index, each packed as
    // source | e << kSortSrcBits (padding columns last, source field all ones).  Neighbouring lanes then
    // gather from neighbouring addresses (several elements per cache line instead of one) and scatter into
    // LDS.  xsort: source = index into a natural-order x; xsort_blk: into an x in block order.  Empty when
    // the plan cannot take that kernel or the fields do not fit.
    std::vector<int32_t> xsort, xsort_blk;
    bool sorted_ok = false;
    int lds_tiles() const { return sorted_ok ? chunk_tiles : 0; }   // what fc_path takes
    int xrow_len() const { return K_pad; }                          // likewise: the longest row of x a run can bring
    std::vector<int32_t> chunks;       // nchunks x 4
    std::vector<int32_t> part_base;    // nbr + 1
    std::vector<float>   bias_p;
    std::vector<uint8_t> vals;         // T*bh*bw elements of wdtype
};

// Device copies (one allocation, sub-arrays 256-byte aligned).
struct DevPlan {
    char*   base = nullptr;
    size_t  bytes = 0;
    void*    vals = nullptr;
    int32_t* col_idx = nullptr;
    int32_t* chunks = nullptr;
    int32_t* part_base = nullptr;
    float*   bias_p = nullptr;
    int32_t* prow_pad = nullptr;
    int32_t* pcol_pad = nullptr;
    int32_t* invprow = nullptr;
    int32_t* invpcol = nullptr;
    int32_t* xidx = nullptr;      // gather index for natural-order x
    int32_t* xidx_blk = nullptr;  // same for x already in block order: col_idx[t]*bw+c
    int32_t* xsort = nullptr;     // packed, source-ordered gather lists (see HostPlan), natural-order x
    int32_t* xsort_blk = nullptr; // same for x in block order
    int32_t* rowid_pad = nullptr; // [M_pad] r for r < M, -1 in padding: stores that stay in block order
    int32_t* row_ptr = nullptr;   // [nbr+1] (persistent recurrent kernel: work split and piece lookup)
};

// Builds every host array.  Returns PIVOT_OK or an error code (error text set).
int build_host_plan(const pivot_fc_desc& d, const void* W, int w_space, const uint8_t* tile_mask,
                    const int32_t* prow, const int32_t* pcol, const float* bias, HostPlan& hp);

// Cuts the schedule for a given chunk size (also used when the library picks it).
void build_schedule(HostPlan& hp, int chunk_tiles);

// True if the device kernels can run this plan.
bool device_supported(const pivot_fc_desc& d, std::string* why);
// Largest chunk (in tiles) whose staged input fits in LDS at the largest batch tile of the vector kernel.
int  max_chunk_tiles(const pivot_fc_desc& d);
// The library's own choice of row slices, chunk size and wavefronts per work
// item; values given in the descriptor (non-zero) are kept.
void choose_schedule(HostPlan& hp);
// Fills xsort / xsort_blk from the schedule (after choose_schedule / build_schedule).
void build_sorted_gather(HostPlan& hp);

// ---- what a kernel launch sees -------------------------------------------
struct FcLaunch {
    // plan
    const void*    vals;
    const int32_t* col_idx;
    const int32_t* chunks;      // eight ints per chunk: (block_row, tile_begin, tile_end, slot, first slot of the row, pieces, 0, 0)
    const int32_t* part_base;
    const float*   bias_p;
    const int32_t* xidx;        // [T*bw]: index into x of column c of tile t (-1 = padding): through pcol for
                                // natural-order x, the block-space column itself for x already in block order
    const int32_t* xsort;       // the same gather as packed source-ordered lists (LDS-fed matrix-core kernel), or NULL
    const int32_t* scatter;     // [M_pad] block-space row -> index into y (-1 = padding row, not stored)
    int M_pad, K_pad, bh, bw, wdtype, layout, T, act, nchunks, nbr, chunk_tiles, wg_waves, row_slices;
    int lds_tiles;              // chunk_tiles if the plan carries the packed gather lists, else 0
    int xrow_len;               // HostPlan::xrow_len()
    int uniform_ct, uniform_parts;  // > 0: regular schedule, the kernels compute the chunk descriptor
    int x_block_order;          // 1: x is [batch][K_pad] in block order (what the matrix-core kernel needs)
    int K;                      // row length of a natural-order x
    int x_resident;             // 0: never copy the whole of x into LDS; 1: the launcher decides; 2: whenever possible
    // data
    const void* x; int64_t ldx;
    void*       y; int64_t ldy;
    int out_f16;                // 1: y is fp16 (chain intermediates of F16 plans), 0: fp32
    int batch;
    float*    partials;
    uint32_t* tickets;
    void*     stream;
};

// Batch rows one launch of the layer kernel covers (grid.y repeats it).
enum { kPathVector = 0, kPathMfmaLds = 1, kPathMfmaGather = 2, kPathMfmaXrow = 3 };
// What decides the path besides the batch.  `lds_tiles`: HostPlan::lds_tiles() (0 rules the LDS-fed matrix-core
// kernel out); `chunk_tiles`, `xrow_len`: the plan's chunk size and HostPlan::xrow_len() (0 rules out the
// matrix-core kernel that gathers its fragments from a copy of x in LDS).
struct FcShape { int layout, wdtype, bh, bw, lds_tiles, chunk_tiles, xrow_len, mean_tiles; };   // mean_tiles: kept tiles per work item, rounded up
inline int mean_tiles_of(int T, int nchunks) { return nchunks > 0 ? (T + nchunks - 1) / nchunks : 0; }
inline FcShape fc_shape(const HostPlan& h) { return FcShape{h.d.layout, h.d.wdtype, h.d.bh, h.d.bw, h.lds_tiles(), h.chunk_tiles, h.xrow_len(), mean_tiles_of(h.T, h.nchunks)}; }
int    fc_path(const FcShape& s, int batch);
int    fc_batch_tile(const FcShape& s, int batch);
bool   fc_uses_matrix_cores(const FcShape& s, int batch);   // the form that needs x in block order
int    fc_row_slices(const FcShape& s, int batch, int want);
// Workspace of one layer application: [arrival counters][partials of split rows][x in block order (matrix path)]
size_t fc_ticket_bytes(const HostPlan& hp);                   // the same for every batch (0 without split block rows)
size_t fc_partial_bytes(const HostPlan& hp, int batch);
size_t fc_workspace_bytes(const HostPlan& hp, int batch);     // counters + partials
size_t fc_gather_bytes(const HostPlan& hp, int batch);        // block-order copy of a natural-order x
// describe != NULL: nothing is launched, *describe receives the name of the kernel instantiation the call would run
int    launch_fc(const FcLaunch& L, std::string* describe = nullptr);
int    launch_gather_x(const void* x, int64_t ldx, const int32_t* pcol_pad, void* xg, int K_pad, int batch,
                       int wdtype, void* stream);
int    launch_fill_zero(void* dev, size_t bytes, void* stream);
// Zeroes columns [K, K_pad) of every row of a [batch][K_pad] buffer of `es`-byte elements.
int    launch_zero_pad_cols(void* buf, int K, int K_pad, int batch, int es, void* stream);
int    launch_null(void* stream);
int    launch_stream_read(const void* buf, size_t bytes, float* out, void* stream);
int    launch_exchange_probe(void* scratch, int rounds, void* stream);
int    launch_dense(const void* W, int wdtype, int M, int K, const void* x, int64_t ldx,
                    const float* bias, void* y, int64_t ldy, int batch, int act, void* stream);

int    launch_csr(const int32_t* row_ptr, const int32_t* col, const void* val, int wdtype, int M, int64_t nnz,
                  const void* x, const float* bias, float* y, int act, void* stream);

struct LstmCellLaunch {
    const float* z;             // [batch][4H] gate pre-activations in natural order (bias included)
    const int32_t* invpcol;     // natural input column -> block-space column
    float* h; float* c;         // [batch][H]
    void* xg_next;              // [batch][K_pad] of wdtype: next step's block-order input, or NULL
    float* z_dbg;               // optional [batch][4H] natural order
    int H, M_pad, K_pad, batch, wdtype;
    void* stream;
};
int launch_lstm_cell(const LstmCellLaunch& L);
// Places x_t (natural columns H..H+I-1) of every step into its block-order input buffer.
int launch_lstm_place_inputs(const void* xs, void* xg_all, const int32_t* invpcol, int H, int I,
                             int K_pad, int steps, int batch, int wdtype, void* stream);
// Places h (fp32, natural) into one block-order input buffer.
int launch_lstm_place_state(const float* h, void* xg, const int32_t* invpcol, int H, int K_pad,
                            int batch, int wdtype, void* stream);

// The whole recurrent loop in one launch (weights resident in registers, grid barriers between the phases).
struct LstmPersistLaunch {
    const HostPlan* hp;
    const void* vals; const int32_t* col_idx; const int32_t* row_ptr; const int32_t* invprow; const int32_t* invpcol;
    const int32_t* pcol_pad; const float* bias_p;
    const void* xs;                    // [steps][batch][I]
    void* xg; size_t xg_step_elems;    // block-order inputs of all steps (written here)
    void* partials;                    // lstm_persist_partial_bytes, zeroed
    uint32_t* ctl;                     // kLstmCtlBytes, zeroed: progress word per workgroup, status word at [256]
    float* h; float* c; float* z_dbg;
    int H, I, batch, steps, device;
    void* stream;
};
bool   lstm_persist_supported(const HostPlan& hp, int H, int batch, int device, int* grid_out, int* L_out);
size_t lstm_persist_partial_bytes(const HostPlan& hp, int batch);
size_t lstm_persist_used_partial_bytes(const HostPlan& hp, int batch, int steps);
constexpr size_t kLstmCtlBytes = 2048;
int    launch_lstm_persist(const LstmPersistLaunch& P);

// A chain of layers in one launch (BRC plans of one weight type with whole block rows per work item, batch 1).
struct ChainPersistLayer {
    const HostPlan* hp;
    const void* vals; const int32_t* chunks; const int32_t* xidx; const float* bias_p; const int32_t* dst;
    const void* in; void* out;
};
struct ChainPersistLaunch {
    std::vector<ChainPersistLayer> layers;
    uint32_t* ctl;                     // chain_persist_ctl_bytes, zeroed once when the chain plan is made
    int grid, bw, wdtype; size_t smem;
    size_t smem_copy;                  // > 0: LDS size with the first layer's x copied into LDS whole (used if x is 16-byte aligned)
    void* stream;
};
bool   chain_persist_supported(const std::vector<const HostPlan*>& layers, int device, int* grid_out, size_t* smem_out,
                               size_t* smem_copy_out, std::string* why);
size_t chain_persist_ctl_bytes();
int    chain_persist_status_offset();  // byte offset of the status word inside the control block
int    launch_chain_persist(const ChainPersistLaunch& C);

}  // namespace pivot

namespace pivot {
// One layer application on a natural-order x, its scratch given as three separate regions: arrival counters
// (fc_ticket_bytes, zero between runs), partial sums (fc_partial_bytes) and the block-order copy of x
// (fc_gather_bytes); a region of size 0 may be NULL.  Checks its arguments like pivot_fc_run.
int run_layer(const pivot_fc_plan_t* plan, const void* x_dev, int64_t ldx, void* y_dev, int64_t ldy, int batch,
              void* tickets, void* partials, void* xg, void* stream);
}

struct pivot_fc_plan {
    pivot::HostPlan host;
    pivot::DevPlan  dev;
    int device = -1;
};

struct pivot_mlp_plan {
    std::vector<pivot_fc_plan_t*> layers;
    int flags = 0;
    std::vector<std::vector<int32_t>> q, dst;
    std::vector<const int32_t*> q_ptrs, dst_ptrs;
    std::vector<int32_t> identity;
    // device: dst arrays (one allocation)
    char* dev_base = nullptr;
    std::vector<int32_t*> dst_dev;
    int device = -1;
    // one-launch form: control words and one buffer of (value, tag) pairs per boundary, in dev_base
    bool persist_ok = false;
    int persist_grid = 0;
    size_t persist_smem = 0, persist_smem_copy = 0;
    uint32_t* persist_ctl = nullptr;
    std::vector<unsigned long long*> persist_pairs;
};
