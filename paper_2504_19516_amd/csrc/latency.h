// Internal interface of the performance estimator (host only).
#pragma once
#include <cstdint>
#include <string>
#include <vector>

#include "sts.h"

namespace sts {

constexpr int64_t INF_NS = (int64_t)1 << 60;
constexpr int64_t PPM = 1000000;

struct Grid {                          // samples on a rectilinear grid, values row-major (first axis outermost)
  std::vector<std::vector<int64_t>> axes;
  std::vector<int64_t> values;
  int64_t min_value() const;
};

struct Profile {
  int64_t n_cu = 256, granule = 32, c_peak = 2500000, d_peak = 8000, n_d = 64;
  int64_t tile_m = 256, tile_n = 256, tile_q = 128, wgs_per_cu = 1, use_waveq = 1;
  int64_t tail_cut = 0;                // > 0: GEMMs cut a partly filled last wave along K into at most this many pieces
  // Measured on the part by the offline profiler and read by the engine's tile choice (not by the estimator):
  // GFLOP/s per busy CU of the 128x128, the 256x256 and the 128x256 GEMM tiles, MB/s per CU for partial tiles written and
  // read back. The 128x256 tile runs one per CU, so its start-up and epilogue are not hidden behind another workgroup:
  // its time is gemm_fixed_128x256 ns plus the flops at gemm_rate_128x256.
  int64_t gemm_rate_128 = 3500, gemm_rate_256 = 4800, gemm_rate_128x256 = 5000, gemm_fixed_128x256 = 25000, partial_bw_cu = 20000;
  // MB/s of a plain read-only stream: per CU of a 32-CU partition, and of the whole GPU (the decode GEMM planner's rates)
  int64_t stream_bw_cu = 59000, stream_bw_gpu = 6400000;
  Grid bw;                             // D_{p,sl}; empty = use D_peak min(1, N_p/N_d)
  Grid prefill_corun;                  // slowdown (ppm, over the decode CUs beside it) of a prefill slice that shares HBM with a
                                       // running decode step; empty = none. Section 3.2.3 measures this side of the contention as
                                       // small and drops it; on this part it reaches 1.1x-1.4x and is kept as a measured table
  Grid alpha_prefill{{{256}, {2048}}, {PPM}};
  Grid alpha_decode{{{256}, {64}, {65536}}, {PPM}};
};

int64_t floor_div(__int128 a, __int128 b);
void wave_quant(int64_t g, int64_t n, int64_t b, int64_t* w, int64_t* tail);
int64_t interp(const Grid& g, const int64_t* x);
int64_t alpha_at(const Grid& g, const int64_t* x);
int64_t srm_ns(int64_t flop, int64_t mem, int64_t n_p, const Profile& hw, int64_t d_override);
int64_t prefill_roofline_ns(const sts_model_desc& s, const Profile& hw, const int32_t* sl, const int32_t* p, int n,
                            int pm, int layer_begin, int n_layers_step);
int64_t decode_roofline_ns(const sts_model_desc& s, const Profile& hw, const int32_t* cl, int n, int dm, int64_t co_tokens);
int64_t predict_prefill_ns(const sts_model_desc& s, const Profile& hw, const int32_t* sl, const int32_t* p, int n,
                           int pm, int layer_begin, int n_layers_step, int co_decode_cus = 0);
int64_t prefill_corun_ppm(const Profile& hw, int co_decode_cus);
int64_t predict_decode_ns(const sts_model_desc& s, const Profile& hw, const int32_t* cl, int n, int dm, int64_t co_tokens);
bool parse_profile(const std::string& text, Profile* hw);
std::string dump_profile(const Profile& hw);

}  // namespace sts

const sts::Profile* sts_profile_get(const sts_profile* p);
