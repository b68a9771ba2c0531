// bf16 expert FFN (paper Eq. 2) per vExpert bucket, forward and backward, as grouped GEMMs on
// the CDNA4 matrix cores (fp32 accumulation).
//
// All kernels share one 256x256 workgroup tile, one workgroup per compute unit: eight wavefronts with
// 128x64 accumulator blocks (32 tiles of v_mfma_f32_16x16x32_bf16) in the direct-to-LDS kernels that
// serve contractions of whole 128-wide rounds, four wavefronts with 128x128 blocks (16 tiles of
// v_mfma_f32_32x32x16_bf16) in the register-staged kernel that serves the rest.
//
//  * rows GEMMs: C[rows of bucket v, :] = In[rows of v, :] . W_owner(v)    (fwd GEMM1/GEMM2,
//    bwd dH and dXp).  The row dimension is cut per bucket: a device-side lookup maps the flat
//    row-tile index to (vExpert, tile inside it), so highly skewed bucket sizes need no host
//    synchronisation.  Rows of a ragged last tile are clamped on load and dropped on store.
//  * weight-gradient GEMMs: dW_e = sum over the vExperts v of e of L_v^T . R_v -- the contraction
//    runs over the tokens of every bucket of e in ascending vExpert id inside one accumulator,
//    which is the single-GPU image of the paper's replica gradient synchronisation.  Output tiles
//    are issued hottest expert first so the long contractions start early; when one expert's
//    contraction is much longer than the chip-wide average per compute unit it is cut into
//    segments that accumulate into fp32 partial tiles, summed in a fixed order by a second kernel
//    (the result does not depend on scheduling).
//
// Two operand pipelines:
//  * direct-to-LDS (rows_gemm_persist_bf16, wgrad_gemm_persist_bf16, wgrad_gemm_dma_bf16; used whenever K is a
//    multiple of 128, i.e. for every benchmark shape): global_load_lds_dwordx4 copies 32-wide K tiles
//    straight into one of four LDS stages (no register staging, no LDS store instructions); an
//    operand whose contraction index is strided in memory is copied as stored and transposed on
//    the way out of LDS by ds_read_tr16_b64.  The loads of the tile three steps ahead are
//    spread between the MFMAs of the current one, and one LDS-only barrier per K tile orders
//    stage reuse.  What bounds the K loop is the energy of bringing the operands into LDS (the stripped loop
//    without its direct loads runs 27-41 % faster on random operands, 9-18 % on constant ones: csrc/probe).
//  * register-staged (rows_gemm_bf16; any K that is a multiple of 8): 64-wide K
//    tiles through registers into two LDS stages, strided operands transposed 8x8 in registers.
//
// LDS tiles are XOR-swizzled at 16-byte chunk granularity so that fragment reads and tile
// writes are free of bank conflicts (measured: SQ_LDS_BANK_CONFLICT = 0).
// The MFMA is issued as (weights-fragment, activations-fragment) so that a lane ends up with 4
// consecutive output columns of one output row; the epilogue passes the accumulators through a
// wave-private LDS patch so that global stores fill whole 128-byte lines.
// GELU and its derivative act on bf16-rounded arguments, so both are read from a table indexed
// by the argument's bits (constant data in the code object, computed from the fp64 formulas when the
// library is built; outside the table's range GELU equals ReLU to below bf16 resolution).
//
// The direct-to-LDS kernels are persistent: 256 workgroups, one per compute unit, each walking its share
// of the output tiles and issuing the next tile's first operand loads while the current tile's K loop
// drains (ffn_bf16_persist.h, wgrad_gemm_persist_bf16; weight gradients whose output is not a whole
// number of 256 x 256 tiles keep one workgroup per tile, wgrad_gemm_dma_bf16).
//
// Layout of the sources: ffn_bf16_tile.h (tile mapping, fragments, activation tables, epilogues, the
// register-staged kernel), ffn_bf16_dma.h (direct-to-LDS pipeline, one rows tile on it),
// ffn_bf16_persist.h (persistent rows kernels and their row-tile table), ffn_bf16_wgrad.h
// (weight-gradient plan and kernels); this file holds the host side.
#include <algorithm>

#include "common.h"
#include "ffn_bf16_tile.h"
#include "ffn_bf16_dma.h"
#include "ffn_bf16_persist.h"
#include "ffn_bf16_wgrad.h"

namespace flexmoe {

// =============================================================================================
// host side
// =============================================================================================
// Weight gradient: how many 32-token K tiles one workgroup contracts before the expert's sum is
// cut into a further segment: a compute unit's even share of all (output tile, K tile) pairs
// (shorter segments measured slower: more fp32 partial tiles), so that the hottest expert's contraction is no longer one serial K loop.  0 = no cutting:
// when a segment would hold more than a quarter of all tokens (many output tiles per expert: the
// grid is busy anyway, and the fp32 partial tiles would be large).
constexpr int kComputeUnits = 256;
static int wgrad_seg_tiles(int A, int d, int f) {
  const long long out_tiles = (long long)((d + BM - 1) / BM) * ((f + BN - 1) / BN);
  const long long k_tiles = A / DK;
  long long seg = k_tiles * out_tiles / kComputeUnits;
  if (seg < 32) seg = 32;
  return 4 * seg <= k_tiles ? (int)seg : 0;
}
// Upper bounds over all load distributions: extra segments (beyond one per expert), and partial
// tile sets (segments of experts that have more than one).
static int wgrad_extra_segments(int A, int V, int seg_tiles) { return seg_tiles ? (A / DK + V) / seg_tiles : 0; }
static int wgrad_partial_slots(int A, int V, int seg_tiles) { return seg_tiles ? 2 * ((A / DK + V) / seg_tiles) + 1 : 0; }

static int wgrad_seg_rows_max(int A, int d, int f, int E, int V) { return E + wgrad_extra_segments(A, V, wgrad_seg_tiles(A, d, f)); }

static int max_row_tiles(int A, int V) { return A / BM + V; }

// Partial tiles of the split last round (see lookup_row_tile): none for grids that can never fill a
// round of workgroups or whose contraction is short (the fp32 round trip would cost more than the idle
// compute units).
constexpr int kSplitMinK = 1024;
static size_t rows_split_bytes(int A, int V, int K, int NC) {
  if (K % 128 || K < kSplitMinK) return 0;
  if ((long long)max_row_tiles(A, V) * ((NC + BN - 1) / BN) <= kSplitUnits) return 0;
  return (size_t)kSplitMaxSlots * BM * BN * sizeof(float);
}

// Job table + fp32 partial tiles of one segmented weight-gradient product (0 when not segmented).
static size_t wgrad_tail_bytes(int A, int d, int f, int V) {
  const int seg_tiles = wgrad_seg_tiles(A, d, f);
  if (!seg_tiles) return 0;
  return align_up((size_t)wgrad_partial_slots(A, V, seg_tiles) * d * f * sizeof(float), 256);
}

size_t ffn_ws_bytes(int A, int d, int f, int E, int V, int dtype) {
  const size_t s = dtype == FLEXMOE_BF16 ? 2 : 4;
  size_t need = align_up((size_t)A * f * s, 256) * 2;      // dHpre (or H in forward) + H
  if (dtype == FLEXMOE_BF16) {
    need += 2 * wgrad_tail_bytes(A, d, f, V);      // one region per weight gradient
    need += rows_split_bytes(A, V, f, d);          // GEMM2 / dXp: partial tiles of the split last round
    need += align_up(wgrad_plan_bytes(wgrad_seg_rows_max(A, d, f, E, V), E, V), 256);   // work list of the weight gradients
    need += align_up(rows_tab_bytes(max_row_tiles(A, V)), 256);                         // row tiles of the bucket list
  }
  return need;
}
static i32x4* rows_tab_ws(const FfnArgs& a, void* ws) {
  return (i32x4*)((char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256) + 2 * wgrad_tail_bytes(a.A, a.d, a.f, a.V) +
                  rows_split_bytes(a.A, a.V, a.f, a.d) +
                  align_up(wgrad_plan_bytes(wgrad_seg_rows_max(a.A, a.d, a.f, a.E, a.V), a.E, a.V), 256));
}
// The row-tile table the persistent rows kernels of one call read.
static void launch_rows_plan(const FfnArgs& a, void* ws, hipStream_t s) {
  const int blocks = std::max(1, std::min(64, (max_row_tiles(a.A, a.V) + kGemmThreads - 1) / kGemmThreads));
  hipLaunchKernelGGL(rows_plan_kernel, dim3(blocks), dim3(kGemmThreads), 0, s, a.voff, a.owner, a.V, rows_tab_ws(a, ws));
}
static void* wgrad_plan_ws(const FfnArgs& a, void* ws) {
  return (char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256) + 2 * wgrad_tail_bytes(a.A, a.d, a.f, a.V) +
         rows_split_bytes(a.A, a.V, a.f, a.d);
}
static void* rows_split_ws(const FfnArgs& a, void* ws) {
  return (char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256) + 2 * wgrad_tail_bytes(a.A, a.d, a.f, a.V);
}

static RowsDmaArgs rows_dma_args(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                                 const void* hpre_in, void* out0, void* out1, const int32_t* gsrc, int gk) {
  return RowsDmaArgs{(const bf16_t*)in, (const bf16_t*)w, (const bf16_t*)bias, a.voff, a.owner, a.V, K, NC,
                     max_row_tiles(a.A, a.V), (NC + BN - 1) / BN, (const bf16_t*)hpre_in, (bf16_t*)out0,
                     (bf16_t*)out1, gsrc, gk, nullptr, 0u, nullptr};
}

template <bool WT, int EPI, int ACT>
static hipError_t launch_rows_t(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                                const void* hpre_in, void* out0, void* out1, hipStream_t s, const int32_t* gsrc, int gk,
                                void* split_ws, const int32_t* scatter_rows, const i32x4* row_tab) {
  const int col_tiles = (NC + BN - 1) / BN;
  const int row_tiles = max_row_tiles(a.A, a.V);
  const unsigned grid = patched_grid(row_tiles, col_tiles);
  if (K % 128 == 0) {
    // K is a whole number of pipeline rounds: direct-to-LDS path, one persistent workgroup per compute unit
    RowsDmaArgs p = rows_dma_args(a, in, w, bias, K, NC, hpre_in, out0, out1, gsrc, gk);
    p.scatter_rows = scatter_rows;
    const unsigned persist = std::min(grid, (unsigned)kComputeUnits);
    if (EPI == EPI_PLAIN && split_ws && rows_split_bytes(a.A, a.V, K, NC)) {
      // the last, partly filled round of tiles is cut along K, then the partial tiles are summed
      p.split_partial = (float*)split_ws;
      p.normal_grid = grid;
      hipLaunchKernelGGL((rows_gemm_persist_bf16<WT, EPI, ACT, false>), dim3(persist), dim3(kDmaThreads), 0, s, p, row_tab);
      hipLaunchKernelGGL(rows_split_reduce_kernel, dim3(kSplitSlices, kSplitUnits / 2), dim3(kGemmThreads), 0, s, p);      // up to 128 tail tiles (two segments each)
      return hipGetLastError();
    }
    if constexpr (!WT && EPI == EPI_FWD1) {
      if (gsrc) {
        hipLaunchKernelGGL((rows_gemm_persist_bf16<WT, EPI, ACT, true>), dim3(persist), dim3(kDmaThreads), 0, s, p, row_tab);
        return hipGetLastError();
      }
    }
    hipLaunchKernelGGL((rows_gemm_persist_bf16<WT, EPI, ACT, false>), dim3(persist), dim3(kDmaThreads), 0, s, p, row_tab);
    return hipGetLastError();
  }
  if (gsrc || scatter_rows) return hipErrorInvalidValue;   // gathered / scattered rows only on the direct-to-LDS path (host check upstream)
  hipLaunchKernelGGL((rows_gemm_bf16<WT, EPI, ACT>), dim3(grid), dim3(kGemmThreads), 0, s, (const bf16_t*)in,
                     (const bf16_t*)w, (const bf16_t*)bias, a.voff, a.owner, a.V, K, NC, row_tiles, col_tiles,
                     (const bf16_t*)hpre_in, (bf16_t*)out0, (bf16_t*)out1);
  return hipGetLastError();
}

template <bool WT, int EPI>
static hipError_t launch_rows(const FfnArgs& a, const void* in, const void* w, const void* bias, int K, int NC,
                              const void* hpre_in, void* out0, void* out1, void* ws, hipStream_t s,
                              const int32_t* gsrc = nullptr, int gk = 1, void* split_ws = nullptr,
                              const int32_t* scatter_rows = nullptr) {
  const i32x4* tab = rows_tab_ws(a, ws);
  if (EPI == EPI_PLAIN)
    return launch_rows_t<WT, EPI, FLEXMOE_RELU>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, split_ws,
                                                scatter_rows, tab);
  switch (a.act) {
    case FLEXMOE_RELU:
      return launch_rows_t<WT, EPI, FLEXMOE_RELU>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr, tab);
    case FLEXMOE_GELU_ERF:
      return launch_rows_t<WT, EPI, FLEXMOE_GELU_ERF>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr, tab);
    default:
      return launch_rows_t<WT, EPI, FLEXMOE_GELU_TANH>(a, in, w, bias, K, NC, hpre_in, out0, out1, s, gsrc, gk, nullptr, nullptr, tab);
  }
}

// One weight-gradient product's arguments and grid; `ws_tail` holds its job table and fp32 partial
// tiles when the contraction is cut into segments (wgrad_tail_bytes each).
// product: 0 = dW2 (M = f, NC = d), 1 = dW1 (M = d, NC = f): which of the plan's two work lists it reads.
static WgradDmaArgs wgrad_dma_args(const FfnArgs& a, const void* L, const void* R, int M, int NC, void* dw,
                                   void* ws_tail, void* ws, unsigned* grid, int product) {
  const int m_tiles = (M + BM - 1) / BM, n_tiles = (NC + BN - 1) / BN;
  const int seg_tiles = wgrad_seg_tiles(a.A, a.d, a.f);
  float* partial = seg_tiles ? (float*)ws_tail : nullptr;
  const int seg_rows_max = wgrad_seg_rows_max(a.A, a.d, a.f, a.E, a.V);
  *grid = patched_grid(seg_rows_max * m_tiles, n_tiles);
  return WgradDmaArgs{(const bf16_t*)L, (const bf16_t*)R, a.voff, a.owner, a.E, a.V, M, NC, m_tiles, n_tiles,
                      seg_tiles, seg_rows_max, partial, wgrad_plan_at(wgrad_plan_ws(a, ws), seg_rows_max, a.E, a.V, product),
                      (bf16_t*)dw};
}

// The work list both weight-gradient products of a backward call read and (with tokens) the row-tile table
// of its rows products: one small launch.
static void launch_bwd_plan(const FfnArgs& a, void* ws, hipStream_t s) {
  const int seg_rows_max = wgrad_seg_rows_max(a.A, a.d, a.f, a.E, a.V);
  const int row_blocks = a.A > 0 ? std::max(1, std::min(64, (max_row_tiles(a.A, a.V) + kGemmThreads - 1) / kGemmThreads)) : 0;
  const int f_tiles = (a.f + BM - 1) / BM, d_tiles = (a.d + BM - 1) / BM;
  const bool whole = a.f % BM == 0 && a.d % BN == 0;
  hipLaunchKernelGGL(ffn_bwd_plan_kernel, dim3(1 + row_blocks), dim3(kGemmThreads), 0, s, a.voff, a.owner, a.E, a.V,
                     wgrad_seg_tiles(a.A, a.d, a.f), seg_rows_max,
                     wgrad_plan_at(wgrad_plan_ws(a, ws), seg_rows_max, a.E, a.V, 0),
                     // (only the persistent kernels skip the holes that balancing leaves in a list)
                     whole ? wgrad_balance_geometry(f_tiles, d_tiles) : WgradBalance{1, 1},
                     whole ? wgrad_balance_geometry(d_tiles, f_tiles) : WgradBalance{1, 1}, rows_tab_ws(a, ws));
}

static void launch_wgrad_reduce(const FfnArgs& a, const WgradDmaArgs& g, hipStream_t s) {
  if (!g.seg_tiles) return;
  const int blocks = (int)std::min<size_t>(((size_t)g.M * g.NC / 4 + kGemmThreads - 1) / kGemmThreads, 2048);
  hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(blocks, a.E), dim3(kGemmThreads), 0, s, (const int4*)g.plan.table, g.M, g.NC,
                     (const float*)g.partial, g.dw);
}

static hipError_t launch_wgrad(const FfnArgs& a, const void* L, const void* R, int M, int NC, void* dw, void* ws_tail,
                               void* ws, hipStream_t s, int product) {
  unsigned grid;
  const WgradDmaArgs g = wgrad_dma_args(a, L, R, M, NC, dw, ws_tail, ws, &grid, product);
  if (M % BM == 0 && NC % BN == 0)      // whole output tiles: one persistent workgroup per compute unit
    hipLaunchKernelGGL(wgrad_gemm_persist_bf16, dim3(std::min(grid, (unsigned)kComputeUnits)), dim3(kDmaThreads), 0, s, g);
  else
    hipLaunchKernelGGL(wgrad_gemm_dma_bf16, dim3(grid), dim3(kDmaThreads), 0, s, g);
  launch_wgrad_reduce(a, g, s);
  return hipGetLastError();
}

// h_keep (all forward variants): where act(Hpre) goes -- the caller's buffer, kept for the backward pass -- or
// null: the workspace.
hipError_t launch_ffn_fwd_bf16(const FfnArgs& a, const void* xp, const void* w1, const void* b1, const void* w2,
                               const void* b2, void* hpre, void* h_keep, void* yp, void* ws, hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  launch_rows_plan(a, ws, s);
  void* h = h_keep ? h_keep : ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, xp, w1, b1, a.d, a.f, nullptr, hpre, h, ws, s);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, yp, nullptr, ws, s, nullptr, 1, rows_split_ws(a, ws));
}

// Forward with the expert-wise layout transformation folded into GEMM1's row loads: bucket row p
// is row src[p] / k of x.  d must be a multiple of 128 (direct-to-LDS path).
hipError_t launch_ffn_fwd_gather_bf16(const FfnArgs& a, const void* x, const int32_t* src, int k, const void* w1,
                                      const void* b1, const void* w2, const void* b2, void* hpre, void* h_keep, void* yp,
                                      void* ws, hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  launch_rows_plan(a, ws, s);
  void* h = h_keep ? h_keep : ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, x, w1, b1, a.d, a.f, nullptr, hpre, h, ws, s, src, k);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, yp, nullptr, ws, s, nullptr, 1, rows_split_ws(a, ws));
}

// The expert path of a top-1 layer without Xp and Yp: rows gathered through src on load (as above)
// and the second product's rows stored straight to y[src[p], :] -- with one expert per token the gate
// weight is exactly 1, so this is flexmoe_combine folded into the epilogue.  d and f multiples of 128.
hipError_t launch_ffn_fwd_top1_bf16(const FfnArgs& a, const void* x, const int32_t* src, const void* w1, const void* b1,
                                    const void* w2, const void* b2, void* hpre, void* h_keep, void* y, void* ws,
                                    hipStream_t s) {
  if (a.A == 0) return hipSuccess;
  launch_rows_plan(a, ws, s);
  void* h = h_keep ? h_keep : ws;
  hipError_t err = launch_rows<false, EPI_FWD1>(a, x, w1, b1, a.d, a.f, nullptr, hpre, h, ws, s, src, 1);
  if (err != hipSuccess) return err;
  return launch_rows<false, EPI_PLAIN>(a, h, w2, b2, a.f, a.d, nullptr, y, nullptr, ws, s, nullptr, 1, rows_split_ws(a, ws), src);
}

// scatter_src (top-1 layers, needs f % 128 == 0): bucket row p of dXp is stored as row scatter_src[p] of
// `dxp`, which is then dX [N, d] itself -- the backward reverse routing folded into the epilogue.
// h_kept: act(Hpre) as the forward pass left it in the caller's buffer, or null: it is computed again from
// hpre by the dH kernel (into the workspace), which then stores two [A, f] tensors instead of one.
hipError_t launch_ffn_bwd_bf16(const FfnArgs& a, const void* dyp, const void* xp, const void* hpre, const void* h_kept,
                               const void* w1, const void* w2, void* dxp, void* dw1, void* dw2, void* ws, hipStream_t s,
                               const int32_t* scatter_src) {
  bf16_t* dhpre = (bf16_t*)ws;
  bf16_t* h_ws = (bf16_t*)((char*)ws + align_up((size_t)a.A * a.f * sizeof(bf16_t), 256));
  const bf16_t* h = h_kept ? (const bf16_t*)h_kept : h_ws;
  hipError_t err;
  launch_bwd_plan(a, ws, s);
  if (a.A > 0) {
    // dH = dYp . W2^T fused with act'(Hpre); W2_e is [f, d], contraction index d contiguous
    err = h_kept ? launch_rows<true, EPI_DHQ>(a, dyp, w2, nullptr, a.d, a.f, hpre, dhpre, nullptr, ws, s)
                 : launch_rows<true, EPI_DH>(a, dyp, w2, nullptr, a.d, a.f, hpre, dhpre, h_ws, ws, s);
    if (err != hipSuccess) return err;
  }
  // dW2 = H^T . dYp, dW1 = Xp^T . dHpre: each with its own partial tiles.  (One launch for dXp, dW2 and dW1, which
  // filled the partly empty last rounds of the three grids, was measured against three persistent launches: the
  // latter are 2 % faster on the GPT-medium-like backward pass and 4.5 % on the Swin-like one.)
  void* ws_tail2 = (char*)ws + 2 * align_up((size_t)a.A * a.f * sizeof(bf16_t), 256);
  void* ws_tail1 = (char*)ws_tail2 + wgrad_tail_bytes(a.A, a.d, a.f, a.V);
  if (a.A > 0) {
    // dXp = dHpre . W1^T; W1_e is [d, f], contraction index f contiguous
    err = launch_rows<true, EPI_PLAIN>(a, dhpre, w1, nullptr, a.f, a.d, nullptr, dxp, nullptr, ws, s, nullptr, 1,
                                       rows_split_ws(a, ws), scatter_src);
    if (err != hipSuccess) return err;
  }
  err = launch_wgrad(a, h, dyp, a.f, a.d, dw2, ws_tail2, ws, s, 0);
  if (err != hipSuccess) return err;
  return launch_wgrad(a, xp, dhpre, a.d, a.f, dw1, ws_tail1, ws, s, 1);
}

}  // namespace flexmoe

#ifdef FLEXMOE_TILE_PHASES
// Profiling build only: copies the per-workgroup phase counters of the persistent GEMM kernels (5 x 256 x 4 uint64,
// see TilePhases) to host memory.
extern "C" int flexmoe_debug_tile_phases(unsigned long long* host_out) {
  return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(flexmoe::g_tile_phases), sizeof(flexmoe::g_tile_phases));
}
#endif
