// Internal declarations shared by the library's translation units (not part of the C ABI).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "hcspmm.h"

namespace hcspmm {

constexpr int kH = 16;                 // rows per window (Section IV-A: the minimum hybrid unit)
// launch guard of the hybrid routing: a path with fewer non-zeros than kGuardNnz and less than
// 1/kGuardShare of the matrix gives its windows to the other path
constexpr int64_t kGuardNnz = 1 << 18;
constexpr int64_t kGuardShare = 8;

// ---- preprocessing -----------------------------------------------------------------------------
constexpr int kUniqueSmallCap = 4096;  // windows with at most this many non-zeros are condensed by an LDS sort
constexpr int kCountMidCap = 16384;    // windows up to this many non-zeros are counted with an LDS hash set (128 KB)
constexpr int kBitmapWords = 32768;    // LDS bitmap (1 Mi columns per pass) used to condense larger windows
constexpr int kEcolLdsCap = 4096;      // distinct-column lists up to this length are searched from LDS

// ---- matrix path -------------------------------------------------------------------------------
constexpr int kMfmaSmallMaxCols = 256; // windows with more condensed columns go to a workgroup-per-window kernel
constexpr int kMfmaMidMaxCols = 1024;  // ... with the small LDS chunk up to here, the large chunk beyond
constexpr int kKcSmall = 128;          // condensed columns staged per wave and chunk (wave-per-window kernel)
constexpr int kKcMid = 256;            // condensed columns staged per workgroup and chunk, medium windows
constexpr int kKcBig = 1024;           // condensed columns staged per workgroup and chunk, wide windows
constexpr int kSliceCols = 4096;       // condensed columns per workgroup; wider windows are cut into slices

// ---- scalar path -------------------------------------------------------------------------------
constexpr int kRowsPerGroup = 8;       // most consecutive rows one lane group may walk (short rows); also the narrowest group
constexpr int kMidRow = 128;           // rows with more non-zeros than this get a whole wave
constexpr int kFusedMidRow = 256;      // with the update stage fused in, rows up to this length stay in the workgroup's tile
constexpr int kLongRow = 1024;         // rows with more non-zeros than this are cut into workgroup-sized segments
constexpr int kSegLen = 2048;          // non-zeros per segment of a long row

struct Segment { int32_t row, k_begin, k_end, slot; };    // slot < 0: writes Y directly
struct MultiRow { int32_t row, first_slot, n_slots, pad; };
// everything the wave-per-window matrix kernel needs to start on a window, in one 32-byte read
// one workgroup's share of a matrix-path window: condensed columns [kc_begin, kc_end); slot < 0: writes Y
struct WgSlice { int32_t w, kc_begin, kc_end, slot; };
struct WinDesc { int32_t w, s, e, nc; int64_t wp; int64_t pad; };
// a run of up to kRunWindows consecutive entries of the matrix path's window list whose column lists were merged
struct RunDesc { int64_t up; int32_t first, nw, nu, n_slices, slot0, pad; };   // union at ucols[up .. up + nu)
// one workgroup's share of a run: union positions [u_begin, u_end) of the list at ucols[up ..], q-th of the run's
// n_slices slices; nw windows; partial tiles (n_slices > 1) at slot0 + wave * n_slices + q
struct RunSlice { int64_t up; int32_t run, u_begin, u_end, q, nw, n_slices, slot0, pad[3]; };
// the window a wave of a slice's workgroup owns (waves beyond the run's last window repeat its first)
struct RunWin { int64_t wp; int32_t w, nc, k_last, pad; };
constexpr int kRunWindows = 4;

void set_error(const char* fmt, ...);

// Experiment knobs (HCSPMM_TUNE_* environment variables; not part of the ABI), read ONCE per process on first use.
// A value of -1 means "not set": the built-in choice applies.
struct Tune {
    int mid_row, long_row, slice_cols, serial, xcd_chunk, rpg, tiles_per_wave, no_rows16, runs, run_slice, side_nnz, bands;
};
const Tune& tune();

#define HC_HIP(call)                                                                               \
    do {                                                                                           \
        hipError_t e_ = (call);                                                                    \
        if (e_ != hipSuccess) {                                                                    \
            ::hcspmm::set_error("%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
            return HCSPMM_EHIP;                                                                    \
        }                                                                                          \
    } while (0)

// Exclusive prefix sum of n int32 values into n+1 int64 values (out[n] = total).  `scratch` holds
// at least scan_scratch_elems(n) int64.  Enqueued on `stream`.
size_t scan_scratch_elems(int64_t n);
hipError_t exclusive_scan_i32_i64(const int32_t* in, int64_t n, int64_t* out, int64_t* scratch, hipStream_t stream);
// up to kScanMaxArrays arrays of one length in one pass: out[a] (n + 1 entries; may be null when only the total is
// wanted) and totals_dev[a] (device, may be null) for every array a; scratch holds scan_multi_scratch_elems(n) values
constexpr int kScanMaxArrays = 8;
struct ScanMulti { const int32_t* in[kScanMaxArrays]; int64_t* out[kScanMaxArrays]; int k; };
size_t scan_multi_scratch_elems(int64_t n);
hipError_t exclusive_scan_multi(const ScanMulti& m, int64_t n, int64_t* totals_dev, int64_t* scratch, hipStream_t stream);

// ---- preprocessing launchers (prepare_kernels.hip) ---------------------------------------------
hipError_t launch_validate(int32_t n_rows, int32_t n_cols, int64_t nnz, const int32_t* rowptr, const int32_t* colind,
                           int32_t* err_flag, hipStream_t s);
hipError_t launch_window_nnz(int32_t W, int32_t n_rows, const int32_t* rowptr, int32_t* nnzw, int32_t* big_list,
                             int32_t* big_count, hipStream_t s);
// sorted distinct-column lists (route: null = every window, else only windows with route != 0)
hipError_t launch_unique_small(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind,
                               int32_t* tmp_cols, int32_t* ncols, const uint8_t* route, hipStream_t s);
hipError_t launch_unique_big(int32_t n_big, const int32_t* big_list, int32_t n_rows, int32_t n_cols,
                             const int32_t* rowptr, const int32_t* colind, int32_t* tmp_cols, int32_t* ncols,
                             const uint8_t* route, hipStream_t s);
// distinct-column counts only (LDS hash sets); windows above kCountMidCap non-zeros go to launch_unique_big
hipError_t launch_window_classes(int32_t W, int32_t n_rows, const int32_t* rowptr, int32_t* nnzw, int32_t* mid_list,
                                 int32_t* huge_list, int32_t* counts, hipStream_t s);
hipError_t launch_count_small(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind, int32_t* ncols,
                              hipStream_t s);
// incremental preparation: the touched windows by size class (+ range check of their columns), counts over a list
hipError_t launch_touched_classes(int32_t n_touched, const int32_t* touched, int32_t n_rows, int32_t n_cols,
                                  const int32_t* rowptr, const int32_t* colind, int32_t* t_small, int32_t* t_mid,
                                  int32_t* t_huge, int32_t* counts, int32_t* err, hipStream_t s);
hipError_t launch_count_small_list(int32_t n_list, const int32_t* list, int32_t n_rows, const int32_t* rowptr,
                                   const int32_t* colind, int32_t* ncols, hipStream_t s);
hipError_t launch_validate_rowptr(int32_t n_rows, int64_t nnz, const int32_t* rowptr, int32_t* err_flag, hipStream_t s);
// incremental preparation: which matrix-path windows keep the previous plan's condensed structure, and its copy
hipError_t launch_carry_mask(int32_t W, const uint8_t* old_route, const uint8_t* route, int32_t n_touched,
                             const int32_t* touched, uint8_t* carried, uint8_t* todo, hipStream_t s);
hipError_t launch_carry_copy(int32_t W, int32_t n_rows, const uint8_t* carried, const int64_t* old_wptr, const int64_t* wptr,
                             const int32_t* old_wcols, int32_t* wcols, const int64_t* old_start, const int32_t* rowptr,
                             const int32_t* old_erc, int32_t* erc, hipStream_t s);
hipError_t launch_count_mid(int32_t n_mid, const int32_t* mid_list, int32_t n_rows, const int32_t* rowptr,
                            const int32_t* colind, int32_t* ncols, hipStream_t s);
hipError_t launch_ecol(int32_t W, int32_t n_rows, const int32_t* rowptr, const int32_t* colind,
                       const int32_t* tmp_cols, const int32_t* ncols, const int64_t* wptr, int32_t* wcols,
                       int32_t* erc, int32_t* unsorted_flag, const uint8_t* route, int want,
                       int32_t skip_above /* leave windows with more non-zeros alone */, hipStream_t s);
// sorted list and condensed positions of the listed matrix-path windows by bitmap ranks (no search)
hipError_t launch_condense_rank(int32_t n_list, const int32_t* list, int32_t n_rows, const int32_t* rowptr,
                                const int32_t* colind, const uint8_t* route, const int64_t* wptr, int32_t* wcols,
                                int32_t* erc, int32_t* unsorted_flag, hipStream_t s);
constexpr int64_t kRankMaxCols = (int64_t)8 << 19;   // beyond this many columns a window's bitmap passes cost more than searching
hipError_t launch_select(int32_t W, const int32_t* ncols, const int32_t* nnzw, int64_t c0, int64_t c1, int64_t c2,
                         int32_t mode, uint8_t* route, int32_t* f_mfma, int32_t* f_csr, int32_t* f_small,
                         int32_t* f_mid, int32_t* f_big, int32_t* nnz_if_mfma, hipStream_t s);
hipError_t launch_masked_copy(int32_t n, const int32_t* flags, const int32_t* src, int32_t* dst, hipStream_t s);
hipError_t launch_compact_ids(int32_t n, const int32_t* flags, const int64_t* pos, int32_t* out, hipStream_t s);
hipError_t launch_row_class(int32_t n_rows, const int32_t* rowptr, const uint8_t* route, int32_t mid_row,
                            int32_t long_row, int32_t* f_short,
                            int32_t* f_mid, int32_t* n_seg, int32_t* f_multi, int32_t* n_slot, int32_t* len_long,
                            hipStream_t s);
hipError_t launch_build_desc(int32_t n_list, const int32_t* win_list, int32_t n_rows, const int32_t* rowptr,
                             const int32_t* ncols, const int64_t* wptr, WinDesc* desc, hipStream_t s);
hipError_t launch_slice_count(int32_t n_list, const int32_t* win_list, const int32_t* ncols, int32_t slice_cols,
                              int32_t* n_slices, int32_t* f_multi, int32_t* n_slots, hipStream_t s);
hipError_t launch_slice_fill(int32_t n_list, const int32_t* win_list, const int32_t* ncols, int32_t slice_cols,
                             const int64_t* slice_pos, const int64_t* multi_pos, const int64_t* slot_pos,
                             WgSlice* slices, MultiRow* multi, hipStream_t s);
hipError_t launch_build_segments(int32_t n_rows, const int32_t* rowptr, const int32_t* n_seg, const int64_t* seg_pos,
                                 const int64_t* multi_pos, const int64_t* slot_pos, Segment* segs, MultiRow* multi,
                                 hipStream_t s);

// ---- compute launchers -------------------------------------------------------------------------
struct SpmmArgs {
    int32_t n_rows;
    const int32_t* rowptr;
    const int32_t* colind;
    const float* vals;
    const void* X;
    int64_t ldx;
    int32_t d;
    int32_t x_dtype;
    float* Y;             // element type y_dtype (fp32 unless the caller asked for a 16-bit output); ldy in elements
    int64_t ldy;
    int32_t relu;
    int32_t y_dtype;
};

// Update stage of the aggregate-then-update layer: Y = act(Z W) for aggregated rows Z (Section V-A).
struct UpdateArgs {
    const float* W;       // d_in x d_out, fp32
    int64_t ldw;
    int32_t d_out;
    float* Y;             // n_rows x d_out
    int64_t ldy;
    int32_t relu;
    int32_t keep_z;       // also store every aggregated row to the workspace (a.Y), not only the rows finished later
    const float* mask;    // optional, n_rows x d_out (pitch ldm): results are stored as 0 where mask <= 0
    int64_t ldm;
    int32_t y_dtype;      // element type of Y
};

#if defined(__HIPCC__)
// fp32 -> 16-bit storage, one rounding to nearest even (the only rounding a 16-bit output adds to the fp32 result);
// two values per call, packed low | high << 16.  The conversions are the hardware's (gfx950 converts to bf16 natively).
typedef float out_f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 out_bf16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 out_f16x2 __attribute__((ext_vector_type(2)));
__device__ inline uint32_t out16_pack(float lo, float hi, int y_dtype)
{
    const out_f32x2 v = {lo, hi};
    if (y_dtype == HCSPMM_BF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, out_bf16x2));
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, out_f16x2));
}

// Stores VEC consecutive results at element offset `off` of an output matrix of element type y_dtype, after the
// optional max(0, .).  The address is aligned for VEC fp32 elements when y_dtype is fp32 and for min(VEC, 4) 16-bit
// elements otherwise (no 16-bit store is wider than 8 bytes).
template <int VEC> __device__ inline void out_store(float* __restrict__ Y, int y_dtype, int64_t off, const float (&x)[VEC], int relu)
{
    float y[VEC];
#pragma unroll
    for (int i = 0; i < VEC; ++i) y[i] = relu ? fmaxf(x[i], 0.f) : x[i];
    if (y_dtype == HCSPMM_F32) {
        float* __restrict__ p = Y + off;
        if constexpr (VEC == 8) {
            *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
            *reinterpret_cast<float4*>(p + 4) = make_float4(y[4], y[5], y[6], y[7]);
        } else if constexpr (VEC == 4) {
            *reinterpret_cast<float4*>(p) = make_float4(y[0], y[1], y[2], y[3]);
        } else if constexpr (VEC == 2) {
            *reinterpret_cast<float2*>(p) = make_float2(y[0], y[1]);
        } else {
            *p = y[0];
        }
    } else {
        unsigned short* __restrict__ p = reinterpret_cast<unsigned short*>(Y) + off;
        if constexpr (VEC >= 4) {
#pragma unroll
            for (int i = 0; i < VEC; i += 4)
                *reinterpret_cast<uint2*>(p + i) = make_uint2(out16_pack(y[i], y[i + 1], y_dtype), out16_pack(y[i + 2], y[i + 3], y_dtype));
        } else if constexpr (VEC == 2) {
            *reinterpret_cast<uint32_t*>(p) = out16_pack(y[0], y[1], y_dtype);
        } else {
            *p = (unsigned short)out16_pack(y[0], 0.f, y_dtype);
        }
    }
}
#endif

// With `upd` the kernels that can keep a 16-row result tile on chip multiply it by W and write
// upd->Y (short rows of the scalar path, wave-per-window tiles of the matrix path); every other
// row goes to a.Y, which then is the aggregation workspace Z, and launch_update_rest finishes it.
bool update_fusable(const SpmmArgs& a);
bool mfma_update_fusable(const SpmmArgs& a);
hipError_t launch_csr(const SpmmArgs& a, int32_t n_segs, const Segment* segs, float* partial, int32_t n_mid,
                      const int32_t* mid_rows, int32_t n_items, const int32_t* row_list, const uint8_t* route,
                      int32_t mid_row, hipStream_t s, const UpdateArgs* upd = nullptr);
hipError_t launch_update_rest(const SpmmArgs& a, int32_t n_rest, const int32_t* rest_rows, const UpdateArgs& upd,
                              hipStream_t s);
// dense product through the 16-row update kernel (narrow W), see spmm_csr_kernels.hip
bool gemm_rows16_usable(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx);
hipError_t launch_gemm_rows16(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                              float* T, int64_t ldt, int relu, hipStream_t s, int32_t t_dtype = HCSPMM_F32);
hipError_t launch_rest_flag(int32_t n_rows, const int32_t* rowptr, const uint8_t* route, const int32_t* ncols,
                            int32_t mid_row, int32_t* flag, hipStream_t s);
hipError_t launch_reduce_partials(const SpmmArgs& a, int32_t n_multi, const MultiRow* multi, const float* partial,
                                  hipStream_t s);
hipError_t launch_mfma_small(const SpmmArgs& a, int32_t n_list, const WinDesc* desc, const int32_t* wcols,
                             const int32_t* erc, hipStream_t s, const UpdateArgs* upd = nullptr);
hipError_t launch_mfma_wg(const SpmmArgs& a, int32_t n_list, const WgSlice* slices, const int32_t* ncols,
                          const int64_t* wptr, const int32_t* wcols, const int32_t* erc, int rows_sorted,
                          const int32_t* slice_rows, float* tile_partial, bool wide, hipStream_t s);
hipError_t launch_slice_rows(int32_t n_slices, const WgSlice* slices, int32_t n_rows, const int32_t* rowptr,
                             const int32_t* erc, int32_t* slice_rows, hipStream_t s);
// bare gather of X rows by an index stream (measurement aid)
int64_t probe_gather_blocks(int64_t n, int32_t d);
hipError_t launch_probe_gather(const int32_t* index, int64_t n, const float* X, int64_t ldx, int32_t d, int32_t n_rows_x,
                               float* out, hipStream_t s);
bool mfma_shape_supported(const SpmmArgs& a);
bool mfma_run_shape_supported(const SpmmArgs& a);
hipError_t launch_mfma_run(const SpmmArgs& a, int32_t n_slices, const RunSlice* slices, const RunWin* wins,
                           const int32_t* ucols, const int32_t* wslot, const int32_t* erc, float* tile_partial, hipStream_t s);
hipError_t launch_run_wins(int32_t n_slices, const RunSlice* slices, const RunDesc* runs, const int32_t* win_list,
                           const int32_t* ncols, const int64_t* wptr, int32_t n_rows, const int32_t* rowptr, RunWin* wins,
                           hipStream_t s);
// union column list of every run and the position of each window column in it (prepare)
hipError_t launch_run_union(int32_t n_runs, const int32_t* win_list, int32_t n_list, const int32_t* ncols,
                            const int64_t* wptr, const int32_t* wcols, int32_t* ucols, int32_t* wslot, RunDesc* runs,
                            hipStream_t s);
constexpr int kRunMinSlice = 2048;     // union columns per workgroup slice of a run, at least
constexpr int kRunTargetSlices = 4096; // ... and about this many slices over all runs of a large matrix
hipError_t launch_reduce_tiles(const SpmmArgs& a, int32_t n_multi, const MultiRow* multi, const float* tile_partial,
                               hipStream_t s);
hipError_t launch_gemm_f32(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                           float* T, int64_t ldt, int relu, hipStream_t s);
// backward pass (Eq. 3): dW = X^T S over row spans, activation mask, transpose of W
int32_t gemm_tn_spans(int64_t n_rows, int32_t d_in, int32_t d);
hipError_t launch_gemm_tn(int64_t n_rows, const float* X, int64_t ldx, int32_t d_in, const float* S, int64_t lds_,
                          int32_t d, float* dW, int64_t lddw, float* partial, hipStream_t s);
hipError_t launch_relu_mask(int64_t n, int32_t d, const float* G, int64_t ldg, const float* Yf, int64_t ldy, float* Gm,
                            int64_t ldo, hipStream_t s);
hipError_t launch_transpose(int32_t rows, int32_t cols, const float* W, int64_t ldw, float* Wt, hipStream_t s);
// same product with the output stored as t_dtype (fp32, or bf16 / fp16 rounded from the fp32 accumulators)
hipError_t launch_gemm_f32_out(int64_t m, int32_t k, int32_t n, const float* X, int64_t ldx, const float* W, int64_t ldw,
                               void* T, int64_t ldt, int32_t t_dtype, int relu, hipStream_t s);

}  // namespace hcspmm

struct BlockCache;
struct hcspmm_plan {
    int32_t H, n_rows, n_cols, W;
    int64_t nnz;
    int device;
    hcspmm_options opt;
    int64_t coef[3];
    // borrowed
    const int32_t* rowptr;
    const int32_t* colind;
    const float* vals;
    // owned, canonical
    int32_t* ncols;
    int32_t* nnzw;
    uint8_t* route;
    int64_t* wptr;
    int32_t* wcols;
    int32_t* erc;            // per non-zero: (ecol << 4) | row-in-window
    int32_t* mfma_windows;
    int32_t* csr_windows;
    int64_t total_ncols;
    int32_t n_mfma, n_csr;
    int64_t nnz_mfma;
    // owned, launch tables
    int32_t* mfma_small;
    hcspmm::WinDesc* mfma_small_desc;
    int32_t* mfma_mid;
    int32_t* mfma_big;
    int32_t n_mfma_small, n_mfma_mid, n_mfma_big;
    hcspmm::WgSlice* mid_slices;     // one per medium window
    hcspmm::WgSlice* big_slices;     // wide windows cut into kSliceCols-column slices
    int32_t n_big_slices;
    int32_t* big_slice_rows;         // per slice and window row: first non-zero inside the slice (sorted rows only)
    hcspmm::MultiRow* tile_multi;    // windows with several slices (row = window id)
    int32_t n_tile_multi;
    int64_t n_tile_slots;
    float* tile_partial;             // lazily sized: n_tile_slots x 16 x d
    int64_t tile_partial_elems;
    // runs of matrix-path windows with merged column lists (the kernel that shares gathered rows through LDS)
    int32_t* ucols;                  // per run: ascending union of its windows' column lists, at RunDesc::up
    int32_t* wslot;                  // per window column (indexed like wcols): its position in the run's union
    hcspmm::RunDesc* runs;
    hcspmm::RunSlice* run_slices;
    hcspmm::RunWin* run_wins;        // kRunWindows records per slice
    hcspmm::MultiRow* run_multi;     // windows of runs cut into several slices (row = window id)
    int32_t n_runs, n_run_slices, n_run_multi;
    int64_t n_run_tile_slots;
    int64_t run_union_cols;          // sum of the runs' union sizes
    int32_t runs_ok;                 // the run tables exist (sorted rows, column count within the bitmap-rank range)
    int32_t rows_sorted;         // 1 when every row's column indices are non-decreasing
    int32_t slice_cols;          // condensed columns per workgroup slice of a wide window (default kSliceCols)
    int32_t mid_row, long_row;   // tier thresholds this plan was built with (defaults kMidRow, kLongRow)
    int32_t fused_mid_row;       // short-tier limit of the fused aggregate-then-update launch (>= mid_row)
    int32_t* short_rows;     // rows of route-0 windows with at most mid_row non-zeros (NULL: walk every row)
    int32_t n_short;
    int32_t* mid_rows;       // rows of route-0 windows with mid_row < non-zeros <= long_row
    int32_t n_mid;
    hcspmm::Segment* segs;
    int32_t n_segs;
    hcspmm::MultiRow* multi;
    int32_t n_multi;
    int64_t n_slots;
    int32_t n_long_rows;
    int32_t condensed_complete;     // 0: wcols / erc are filled for matrix-path windows only (the rest on export)
    int32_t erc_own, wcols_own;     // erc / wcols were allocated on their own (on export), not from the plan's chunks
    void* chunks[64];               // device allocations that hold the plan-owned arrays (several arrays per chunk)
    size_t chunk_bytes[64];
    int32_t n_chunks;
    struct BlockCache* cache;       // device blocks kept between hcspmm_plan_update calls (null until the first one)
    int32_t features_complete;    // ncols / wptr / total_ncols are filled (a scalar-only plan computes them on first request)
    int32_t n_rest;                 // rows finished through the workspace by the fused update
    int32_t* rest_rows;
    int64_t nnz_long;
    // lazily sized partial-sum buffer for long rows cut into several segments
    float* partial;
    int64_t partial_elems;
    int64_t device_bytes;
    // side streams / events used to run the matrix and scalar paths concurrently
    int32_t side_ok;
    hipStream_t side[2];
    hipEvent_t ev_fork, ev_join[2];
};
