// Which kernel a batched (5..64 rows) weight-streaming GEMM takes - host code only.
//
// Two kernels exist (dk_gemm.hip.h, dk_gemm_shared.hip.h).  The choice between them, and the number
// of K slices of the second, comes from an estimate of each candidate's duration, not from a table
// of shapes.  The estimate is a latency/occupancy model of a weight stream:
//
//   * a wave keeps a fixed number of bytes in flight, so a block streams at (waves x rate per wave)
//     until the compute units that are busy together reach the device's rate;
//   * the busiest compute unit works through ceil(blocks / compute units) blocks; blocks that are
//     resident together share its rate, blocks beyond that wait for a slot (one more block start);
//   * every 128-column step costs matrix-core and LDS time per 16-row batch tile that the stream does
//     not hide;
//   * a launch has a fixed cost, and K slices pay for the hand-over and the in-order sum of the
//     partial tiles.
//
// The constants were fitted (least squares on log time) to HBM-cold sweeps of both kernels over the
// layer matrices of the 0.6B, 3B, 8B and 30B-A3B shapes at 16..64 rows, 1..8 slices (about 400
// timings; the fit reproduces them to 13 % rms for the shared kernel, 16 % for the other).  What
// matters is the ranking: on those sweeps the estimate's choice is the measured best, or within 5 %
// of it, except where two candidates are within the sweeps' own scatter.
#pragma once
#include <algorithm>
#include <cmath>

namespace dkplan {

enum { EPI_STORE = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };   // same values as dk::GEPI_*

struct GemmPlan { int w, slices; };   // w == 0: skinny_gemm_kernel; else shared_gemm_kernel, w waves per block

// Variant of skinny_gemm_kernel: MT 16-row batch tiles per block, KS waves that split K, RT row tiles per
// wave, `groups` groups of 16 batch rows across blockIdx.y (then MT == 1).
struct SkinnyVariant { int mt, ks, rt, groups; };

// A wave that handles several row tiles per K-step reuses the activation operand it has loaded; it pays
// while enough blocks remain to fill the chip: four tiles per wave from 16 blocks per compute unit on,
// two from 1.25.  Residual projections with at most one block per compute unit take two-wave blocks
// (less to add up across waves).  A small matrix at 32..64 rows whose row tiles x groups of 16 rows
// still make at most two blocks per compute unit runs the 16-row kernel over all groups at once.
inline SkinnyVariant skinny_variant(int epi, int N, int Bp, bool q4, int cus)
{
    const int tiles = (N + 15) / 16, mt = Bp / 16;
    const bool one_matrix = epi != EPI_SWIGLU;
    const int groups = (mt >= 2 && tiles * mt <= 2 * cus) ? mt : 1;
    switch (groups > 1 ? 1 : mt) {
        case 1:
            if (one_matrix) {
                if (tiles >= 16 * cus) return {1, 8, 4, groups};
                if (tiles >= cus + cus / 4) return {1, 8, 2, groups};
                if (tiles <= cus && epi == EPI_RESID && !q4) return {1, 2, 1, groups};
            }
            return {1, 8, 1, groups};
        case 2:
            if (one_matrix && tiles >= 4 * cus) return {2, 8, 2, 1};
            return {2, 8, 1, 1};
        case 3: return {3, 4, 1, 1};
        default: return {4, 4, 1, 1};
    }
}

// ---- estimates, in microseconds (bf16 weights) ---------------------------------------------------
constexpr double kStepBytes = 4096.0;        // one 16-row x 128-column weight tile
// shared_gemm_kernel
constexpr double kShLaunch = 5.78;           // launch, first loads, epilogue
constexpr double kShBlockStart = 0.58;       // per block that starts on a busy compute unit
constexpr double kShWaveRate = 16.4e3;       // bytes per us a wave streams (two steps in flight)
constexpr double kShDeviceRate = 7.04e6;     // bytes per us all compute units together
constexpr double kShTileStep = 0.22;         // us per step, 16-row batch tile and matrix (not hidden)
constexpr double kShSliceTile = 0.18;        // us per slice, batch tile and matrix for the hand-over
// skinny_gemm_kernel
constexpr double kSkLaunch = 2.06;
constexpr double kSkWaveRate = 89.1e3;       // a lone wave is not the limit: the compute unit is
constexpr double kSkCuRate = 37.6e3;         // bytes per us the waves of one compute unit stream together
constexpr double kSkDeviceRate = 6.41e6;
constexpr double kSkActShare = 0.47;         // a wave's own activation fetch (8 KB per batch tile and step), as stream bytes
constexpr double kSkTileStep = 0.036;
constexpr double kSkReduce = 0.176;          // us per wave, batch tile, row tile and matrix summed through LDS
constexpr double kSkWavesPerCu = 32.0;       // resident waves per compute unit

inline double shared_gemm_us(int N, int K, int n_mat, int mt, int w, int slices, int cus)
{
    const int tiles = (N + 15) / 16, row_blocks = (tiles + w - 1) / w, blocks = row_blocks * slices;
    const int steps = (K / 128 + slices - 1) / slices;
    const int occ = w <= 4 ? 2 : 1;                             // blocks resident per compute unit
    const int active = std::min(cus, blocks);
    const int per_cu = (blocks + cus - 1) / cus;                // blocks of the busiest compute unit
    const int resident = std::min(occ, per_cu);
    const double rate = std::min(kShWaveRate * w * resident, kShDeviceRate / active);
    double t = kShLaunch + kShBlockStart * ((per_cu + occ - 1) / occ) +
               (double)steps * per_cu * (w * n_mat * kStepBytes / rate + kShTileStep * mt * n_mat / resident);
    if (slices > 1) t += kShSliceTile * slices * mt * n_mat;
    return t;
}

inline double skinny_gemm_us(int N, int K, int n_mat, const SkinnyVariant &v, int cus)
{
    const int tiles = (N + 15) / 16;
    const double blocks = (double)((tiles + v.rt - 1) / v.rt) * v.groups;
    const double slots = cus * std::max(1.0, kSkWavesPerCu / v.ks);
    const double rounds = std::max(1.0, blocks / slots);
    const int steps = ((K + 127) / 128 + v.ks - 1) / v.ks;
    const double conc = std::min(blocks, slots), active = std::min((double)cus, conc), per_cu = conc / active;
    const double wave_step = v.rt * n_mat * kStepBytes + kSkActShare * v.mt * 2.0 * kStepBytes;
    const double rate = std::min(std::min(kSkWaveRate, kSkCuRate / (per_cu * v.ks)), kSkDeviceRate / (active * per_cu * v.ks));
    return kSkLaunch + rounds * steps * (wave_step / rate + kSkTileStep * v.mt * v.rt * n_mat) +
           kSkReduce * v.ks * v.mt * v.rt * n_mat;
}

// K slices of shared_gemm_kernel for blocks of w waves: as many as still give one round of blocks on the
// compute units (a second, partly filled round costs more than the slices save), at least four K-steps per
// slice, at most 8; a matrix whose row blocks alone fill more than half the chip takes four.
inline int shared_gemm_slices(int N, int K, int w, int cus)
{
    const int row_blocks = ((N + 15) / 16 + w - 1) / w;
    if (row_blocks > cus / 2) return std::max(1, std::min(4, K / 512));
    return std::max(1, std::min(std::min(cus / row_blocks, 8), K / 512));
}

// 4-bit weights: thresholds from a sweep of the 4-bit kernels over the same shapes (their streams are a
// quarter as long and their steps carry the dequantisation, which this model's constants do not cover):
// the lm_head at every batch size; q | k | v from 32 rows on; the gate/up pair and the down projection of
// the 3B / 8B shapes; never the output projection.
inline GemmPlan gemm_plan_q4(int epi, int N, int K, int mt)
{
    const long long elems = (long long)N * K;
    if (epi == EPI_STORE) {
        if ((N + 15) / 16 >= 4096) return {8, 1};
        if (mt >= 2 && elems >= (8ll << 20)) return {8, 4};
    } else if (epi == EPI_SWIGLU) {
        if (elems >= (40ll << 20)) return {8, 2};
        if (elems >= (20ll << 20)) return {8, 4};
    } else {
        if (elems >= (mt >= 2 ? (20ll << 20) : (40ll << 20))) return {4, 8};
    }
    return {0, 1};
}

// The plan: the candidate with the smallest estimate.  Candidates are the skinny kernel (its variant by
// skinny_variant) and the shared kernel in the block widths that are instantiated for the epilogue - 8
// waves for plain stores and the gate/up pair (4 as well at 16 rows), 4 waves for residual projections -
// with shared_gemm_slices() slices (one slice when the row blocks alone make several rounds: the lm_head).
// est_us (optional) receives the estimate of the winner.
inline GemmPlan gemm_plan(int epi, int N, int K, int Bp, bool q4, int cus, double *est_us = nullptr)
{
    const int mt = Bp / 16;
    if (est_us) *est_us = 0.0;
    if (K % 128) return {0, 1};
    if (q4) return gemm_plan_q4(epi, N, K, mt);
    const int n_mat = epi == EPI_SWIGLU ? 2 : 1;
    GemmPlan best{0, 1};
    double best_us = skinny_gemm_us(N, K, n_mat, skinny_variant(epi, N, Bp, false, cus), cus);
    auto consider = [&](int w) {
        const int row_blocks = ((N + 15) / 16 + w - 1) / w;
        const int s = row_blocks >= 2 * cus ? 1 : shared_gemm_slices(N, K, w, cus);
        const double us = shared_gemm_us(N, K, n_mat, mt, w, s, cus);
        if (us < best_us) { best_us = us; best = {w, s}; }
    };
    if (epi == EPI_RESID) consider(4);
    else {
        consider(8);
        if (epi == EPI_SWIGLU && mt == 1) consider(4);
    }
    if (est_us) *est_us = best_us;
    return best;
}

}  // namespace dkplan
