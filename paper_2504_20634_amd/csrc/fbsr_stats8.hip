// fbsr_stats8.hip -- kernels behind fbsr_bias_stats_format8: the per-bin statistics of fbsr_bias_stats (the
// measurement behind Figs. 1 and 2: mean of the rounded samples and bias in target ulps, Sec. III) for a target
// format given by its descriptor -- any (K, P, B; M) of Sec. II, Eq. (1) with K <= 8 -- and every rounding mode of
// fbsr_round_format8.  Per bin {count, sum y, sum e, sum e^2} in fp64, y the Eq. (1) value of the rounded code and
// e = (y - x) / ulp_t(x), ulp_t(x) = 2^(e~ - P + 1) with e~ of Eq. (2).
//
// The geometry, the fixed reduction order and the workspace records are those of fbsr_stats.hip (a workgroup per
// chunk of 16384 elements, a wave per span of 4096, rows of 256 with four consecutive floats per lane; lane sums ->
// a fixed tree over the wave when a bin ends -> the four waves in order -> one record per chunk for a bin that
// continues next door, added up by the same finalizing kernel).  What differs is the element: round8 with the
// descriptor's constants as kernel arguments, the code's value from a 256-entry table in LDS, and the error in fp64
// for every element -- except on "plain" rows, which are most rows of ordinary data: when a wave's row lies in one
// bin and holds only values with |x| <= M that are zero or at least 2^(1 - B - P) (no NaN, nothing above M, no bits
// lost below the code space), the code-space word is exact and is formed without selects: the normal map of
// max(|x|, 2^(1 - B)) plus the truncated subnormal map of min(|x|, 2^(1 - B)) minus the word both give at the split.
// The error is then the integer (r & ~mask) - r0 in units of 2^-24 ulp, in magnitude space (its sign flipped for a
// negative x by an exclusive or with the sign mask and one correction sum); a lane adds at most 64 of them before
// its wave closes the span, so 32 bits hold their sum and 64 bits the sum of their squares exactly.
#include "fbsr_launch.h"
#include "fbsr_stats_common.h"

namespace fbsr {

// 1 / ulp_t(x) = 2^(P - 1 - e~), e~ = max(floor(log2 |x|), 1 - B) (Eq. (2)), from the fp32 exponent field (a field of 0
// is below every format's clamp: B <= 96); 1 for a non-finite x.  min_field = (1 - B + 127) << 23,
// top = (1023 + P - 1 + 127) << 20.
__device__ __forceinline__ double inv_ulp8(uint32_t bits, uint32_t min_field, uint32_t top) {
  const uint32_t ef = bits & 0x7F800000u;
  const uint32_t hi = top - ((ef > min_field ? ef : min_field) >> 3);
  return ef == 0x7F800000u ? 1.0 : __hiloint2double((int)hi, 0);
}

struct Stats8Args {
  Fmt8 f;
  Mode8 m;
  uint32_t min_field, top;   // of inv_ulp8
  // the plain rows' integer path (see stats8_spans): the pattern of 2^(1 - B - P), below which a target-subnormal value
  // loses bits to the truncation; -(rebias << shift_p) - 2^(23 + P); 2^(23 + P), the code-space word of 2^(1 - B)
  uint32_t u_exact, map_add;
  float split;
  uint32_t plain_ok;         // 0: the format or the mode rules the integer path out (P = 1, more than 16 random bits)
  uint32_t row_sum_exact;    // 1: M is below 2^22 steps of the subnormal grid, which every finite value is a multiple of
};

// The code of one element: any pattern, any bit count the entry point accepts.
__device__ __forceinline__ uint32_t round8_any(uint32_t bits, uint32_t n, const Fmt8& f, const Mode8& m) {
  if (m.nbits > (uint32_t)kMaxTileNbits) return round8_wide(bits, n, f, m);
  return m.ties ? round8<true, true>(bits, n, f, m) : round8<false, true>(bits, n, f, m);
}

// W: the slot width (0: the mode draws no bits; 32: more than 16 bits, a lane's four elements of a row are one block).
template <int W>
__global__ __launch_bounds__(kThreads) void stats8_spans(const float* __restrict__ x, uint8_t* __restrict__ out, uint64_t npairs,
                                                         Stats8Args a, Table8 values, uint64_t seed, uint64_t blk0, uint64_t i0,
                                                         uint64_t group, uint64_t first_bin, uint64_t chunk_base,
                                                         double* __restrict__ records, double* __restrict__ stats) {
  constexpr int WW = W == 0 ? 1 : W;
  constexpr bool DRAWS = W != 0, MANY = W == 32;
  constexpr int ROWS = kStatsSpanElems / 256;                      // rows of a span
  constexpr int ROWS_PER_ROUND = MANY || !DRAWS ? ROWS : (64 * 128 / WW / 256 < ROWS ? 64 * 128 / WW / 256 : ROWS);
  __shared__ uint4 strips[kWavesPerBlock][64];
  __shared__ float value_of[256];
  __shared__ double part[kWavesPerBlock][kStatsMaxBinsPerChunk][kStatsRecordDoubles];
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const uint64_t chunk = chunk_base + blockIdx.x;
  const uint64_t i_end = i0 + npairs * kStatsPairElems;
  const uint64_t chunk_lo = i0 + chunk * kStatsChunkElems;        // < i_end: the grid has one workgroup per started chunk
  const uint64_t chunk_hi = chunk_lo + kStatsChunkElems < i_end ? chunk_lo + kStatsChunkElems : i_end;
  const uint64_t bin_first = chunk_lo / group;
  const int nbins_here = (int)((chunk_hi - 1) / group - bin_first) + 1;   // <= kStatsMaxBinsPerChunk: group >= kStatsMinGroup

  value_of[threadIdx.x] = values.v[threadIdx.x];
  for (int t = lane; t < nbins_here * (int)kStatsRecordDoubles; t += 64) (&part[wave][0][0])[t] = 0.0;
  __syncthreads();

  const uint64_t span_lo = chunk_lo + (uint64_t)wave * kStatsSpanElems;
  const uint64_t pair0 = chunk * (kStatsChunkElems / kStatsPairElems) + (uint64_t)(wave * kStatsSpanPairs);
  const int my_pairs = pair0 >= npairs ? 0 : (npairs - pair0 < (uint64_t)kStatsSpanPairs ? (int)(npairs - pair0) : kStatsSpanPairs);
  const int my_rows = my_pairs * kRows;
  const uint64_t span_blk = blk0 + (chunk * (kStatsChunkElems / 128) + (uint64_t)wave * (kStatsSpanElems / 128)) * (uint64_t)WW;
  uint4* strip = strips[wave];

  double sy = 0.0, se = 0.0, see = 0.0;
  int32_t se_i = 0, neg_i = 0;   // plain rows: sum of e_int ^ s and of s, s = -1 for a negative x and 0 otherwise
  long long see_i = 0;
  int slot = my_rows > 0 ? (int)(span_lo / group - bin_first) : 0;
  uint64_t next_bin = my_rows > 0 ? group - span_lo % group : 0;   // span-relative index at which the next bin starts

  auto close_bin = [&]() {
    constexpr double kUnit = 1.0 / (double)(1 << 24);
    const double t0 = wave_total(sy), t1 = wave_total(se + (double)(se_i - neg_i) * kUnit);
    const double t2 = wave_total(see + (double)see_i * (kUnit * kUnit));
    if (lane == 0) {
      part[wave][slot][0] = t0; part[wave][slot][1] = t1; part[wave][slot][2] = t2;
    }
    slot += 1;
    sy = se = see = 0.0;
    se_i = neg_i = 0;
    see_i = 0;
  };

  const float* xs = x + (span_lo - i0);
  if (my_rows > 0) {
    // one row of the span: its random integers, then the plain or the general way
    auto do_row = [&](int r, const f32x4& v) {
      uint32_t n[4] = {0, 0, 0, 0};
      if constexpr (MANY) {
        uint32_t o[4];
        philox_block(span_blk + (uint64_t)(r * 64 + lane), seed, 0, o);
#pragma unroll
        for (int j = 0; j < 4; ++j) n[j] = __builtin_amdgcn_ubfe(o[j], 0u, a.m.nbits);
      } else if constexpr (DRAWS) {
        if (r % ROWS_PER_ROUND == 0) {   // the blocks of the next ROWS_PER_ROUND rows, one per lane
          __builtin_amdgcn_wave_barrier();   // the wave's own LDS traffic keeps program order; this keeps the compiler to it
          const int b = r / ROWS_PER_ROUND * 64 + lane;
          if (b < kStatsSpanElems / 128 * WW) {
            uint32_t o[4];
            philox_block(span_blk + (uint64_t)b, seed, 0, o);
            strip[lane] = make_uint4(o[0], o[1], o[2], o[3]);
          }
          __builtin_amdgcn_wave_barrier();
        }
        const uint64_t rb = read_row_bits<WW>(strip, (r % ROWS_PER_ROUND) * 256 + 4 * lane);
#pragma unroll
        for (int j = 0; j < 4; ++j) n[j] = slot_bits<WW>(rb, j, a.m.nbits);
      }
      const uint32_t b[4] = {__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)};
      const int lo_e = r * 256, hi_e = lo_e + 256;   // the row's elements in the span
      if (a.plain_ok != 0u && next_bin >= (uint64_t)hi_e) {
        const uint32_t u0 = b[0] & 0x7FFFFFFFu, u1 = b[1] & 0x7FFFFFFFu, u2 = b[2] & 0x7FFFFFFFu, u3 = b[3] & 0x7FFFFFFFu;
        const uint32_t top = max(max(u0, u1), max(u2, u3));
        const uint32_t low = min(min(u0 - 1u, u1 - 1u), min(u2 - 1u, u3 - 1u));   // a zero wraps to the largest value
        if (!__any(top > a.f.u_max || low < a.u_exact - 1u)) {
          uint32_t mag[4], r0[4], add[4];
          float y[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t u = b[j] & 0x7FFFFFFFu;
            const uint32_t normal_part = (max(u, a.f.u_sub) << a.f.shift_p) + a.map_add;
            const uint32_t sub_part = (uint32_t)fminf(__uint_as_float(u) * a.f.sub_scale, a.split);
            r0[j] = normal_part + sub_part;
            add[j] = (n[j] << a.m.shift) + a.m.fixed;
          }
          if (a.m.ties) {   // one branch for the row (the empty statement keeps it a branch: the other modes skip the work)
            asm volatile("");
#pragma unroll
            for (int j = 0; j < 4; ++j) add[j] += ((r0[j] >> a.m.shift) & 1u) ^ a.m.tie_xor;
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const uint32_t sum = r0[j] + add[j];
            mag[j] = sum >> 24;
            const int32_t e_int = (int32_t)((sum & 0xFF000000u) - r0[j]);
            const int32_t sgn = (int32_t)b[j] >> 31;
            se_i += e_int ^ sgn;
            neg_i += sgn;
            see_i += (long long)e_int * (long long)e_int;
            y[j] = __uint_as_float(__float_as_uint(value_of[mag[j]]) | (b[j] & 0x80000000u));
          }
          if (a.row_sum_exact != 0u) {   // four values of at most 22 bits on one grid: their fp32 sum is exact
            asm volatile("");
            sy += (double)((y[0] + y[1]) + (y[2] + y[3]));
          } else {
            sy += (double)y[0];
            sy += (double)y[1];
            sy += (double)y[2];
            sy += (double)y[3];
          }
          if (out != nullptr) {
            reinterpret_cast<uint32_t*>(out)[(span_lo - i0) / 4 + (uint64_t)(r * 64 + lane)] =
                with_signs4(pack4_bytes(mag[0], mag[1], mag[2], mag[3]), top_bytes4(b), a.f);   // |x| <= M: no code above max_code
          }
          return;
        }
      }
      uint32_t c[4];
      double y[4], e[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c[j] = round8_any(b[j], n[j], a.f, a.m);
        y[j] = (double)value_of[c[j]];
        e[j] = (y[j] - (double)__uint_as_float(b[j])) * inv_ulp8(b[j], a.min_field, a.top);
      }
      if (out != nullptr) {
        reinterpret_cast<uint32_t*>(out)[(span_lo - i0) / 4 + (uint64_t)(r * 64 + lane)] = pack4_bytes(c[0], c[1], c[2], c[3]);
      }
      // the bins of this row's elements [lo_e, lo_e + 256) of the span
      auto add_some = [&](int first, int last) {   // the row's elements whose index in the row lies in [first, last)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int at = 4 * lane + j;
          const bool in = at >= first && at < last;
          sy += in ? y[j] : 0.0;
          se += in ? e[j] : 0.0;
          see = in ? fma(e[j], e[j], see) : see;
        }
      };
      int from = 0;
      while (next_bin < (uint64_t)hi_e) {   // uniform over the wave
        const int cut = (int)next_bin - lo_e;
        add_some(from, cut);
        close_bin();
        from = cut;
        next_bin += group;
      }
      add_some(from, 256);
    };
    // two rows per trip, the next two loaded before these are worked on (past the end every lane reads the span's
    // first 16 bytes and drops them: a load that may or may not have been issued would make the compiler wait for
    // all of them)
    f32x4 ahead[kRows];
#pragma unroll
    for (int k = 0; k < kRows; ++k) ahead[k] = load_stream4(xs + (k * 256 + 4 * lane));
#pragma unroll 1
    for (int r = 0; r < my_rows; r += kRows) {
      f32x4 v[kRows];
#pragma unroll
      for (int k = 0; k < kRows; ++k) v[k] = ahead[k];
      const bool more = r + kRows < my_rows;
#pragma unroll
      for (int k = 0; k < kRows; ++k) ahead[k] = load_stream4(xs + (more ? (r + kRows + k) * 256 + 4 * lane : 0));
#pragma unroll
      for (int k = 0; k < kRows; ++k) do_row(r + k, v[k]);
    }
    close_bin();
  }
  __syncthreads();
  const int t = threadIdx.x;
  if (t < nbins_here * (int)kStatsRecordDoubles) {
    const int s = t / (int)kStatsRecordDoubles, k = t % (int)kStatsRecordDoubles;
    double v = part[0][s][k];
#pragma unroll
    for (int wv = 1; wv < kWavesPerBlock; ++wv) v += part[wv][s][k];
    if (s == 0) {
      records[chunk * (2 * kStatsRecordDoubles) + k] = v;
    } else if (s == nbins_here - 1) {
      records[chunk * (2 * kStatsRecordDoubles) + kStatsRecordDoubles + k] = v;
    } else {
      double* st = stats + (bin_first + (uint64_t)s - first_bin) * 4;   // a bin that lies inside this chunk: no other writer
      st[1 + k] += v;
      if (k == 0) st[0] += (double)group;
    }
  }
}

// One thread per bin, serial over the bin's elements inside [a0, a0 + n): any alignment, any group size; used for
// ragged heads and tails and for bins shorter than kStatsMinGroup.
__global__ __launch_bounds__(kThreads) void stats8_bins(const float* __restrict__ x, uint8_t* __restrict__ out, uint64_t n,
                                                        Stats8Args a, Table8 values, int W, int log2_per_block, uint64_t seed,
                                                        uint64_t a0, uint64_t group, uint64_t bin_lo, uint64_t nb,
                                                        uint64_t first_bin, double* __restrict__ stats) {
  __shared__ float value_of[256];
  value_of[threadIdx.x] = values.v[threadIdx.x];
  __syncthreads();
  const uint64_t k = (uint64_t)blockIdx.x * kThreads + threadIdx.x;
  if (k >= nb) return;
  const uint64_t bin = bin_lo + k;
  const uint64_t lo = bin * group > a0 ? bin * group : a0;
  const uint64_t be = bin_end(bin, group);
  const uint64_t hi = be < a0 + n ? be : a0 + n;
  if (lo >= hi) return;
  double sy = 0.0, se = 0.0, see = 0.0;
  for (uint64_t i = lo; i < hi; ++i) {
    const uint32_t bits = __float_as_uint(x[i - a0]);
    const uint32_t rnd = W != 0 ? element_bits(i, log2_per_block, W, a.m.nbits, seed, 0) : 0u;
    const uint32_t c = round8_any(bits, rnd, a.f, a.m);
    if (out != nullptr) out[i - a0] = (uint8_t)c;
    const double y = (double)value_of[c];
    const double e = (y - (double)__uint_as_float(bits)) * inv_ulp8(bits, a.min_field, a.top);
    sy += y;
    se += e;
    see = fma(e, e, see);
  }
  double* s = stats + (bin - first_bin) * 4;
  s[0] += (double)(hi - lo);
  s[1] += sy;
  s[2] += se;
  s[3] += see;
}

namespace {

template <int W>
hipError_t launch_spans8(const float* x, uint8_t* out, uint64_t npairs, const Stats8Args& a, const Table8& t, uint64_t seed,
                         uint64_t blk0, uint64_t i0, uint64_t group, uint64_t first_bin, double* records, double* stats,
                         hipStream_t stream) {
  const uint64_t per_chunk = kStatsChunkElems / kStatsPairElems;
  const uint64_t chunks = (npairs + per_chunk - 1) / per_chunk;
  for (uint64_t c0 = 0; c0 < chunks; c0 += kMaxTilesPerLaunch) {
    const uint64_t cnt = chunks - c0 < kMaxTilesPerLaunch ? chunks - c0 : kMaxTilesPerLaunch;
    hipLaunchKernelGGL((stats8_spans<W>), dim3((unsigned)cnt), dim3(kThreads), 0, stream, x, out, npairs, a, t, seed, blk0, i0,
                       group, first_bin, c0, records, stats);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

hipError_t launch_bins8(const float* x, uint8_t* out, uint64_t n, const Stats8Args& a, const Table8& t, int W, uint64_t seed,
                        uint64_t a0, uint64_t group, uint64_t first_bin, double* stats, hipStream_t stream) {
  if (n == 0) return hipSuccess;
  const uint64_t bin_lo = a0 / group, bin_hi = (a0 + n - 1) / group;
  const uint64_t nb = bin_hi - bin_lo + 1;
  for (uint64_t at = 0; at < nb; at += kMaxElemsPerLaunch) {
    const uint64_t m = nb - at < kMaxElemsPerLaunch ? nb - at : kMaxElemsPerLaunch;
    const uint64_t blocks = (m + kThreads - 1) / kThreads;
    hipLaunchKernelGGL(stats8_bins, dim3((unsigned)blocks), dim3(kThreads), 0, stream, x, out, n, a, t, W, W ? log2_of(128 / W) : 0,
                       seed, a0, group, bin_lo + at, m, first_bin, stats);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  return hipSuccess;
}

}  // namespace

hipError_t launch_stats_format8(const float* x, uint8_t* out, uint64_t n, const Fmt8& f, const Mode8& m, const Table8& t,
                                int P, int B, uint64_t seed, uint64_t offset, uint64_t group, uint64_t first_bin,
                                double* stats, double* workspace, hipStream_t stream) {
  Stats8Args a;
  a.f = f;
  a.m = m;
  a.min_field = (uint32_t)(1 - B + 127) << 23;
  a.top = (uint32_t)(1023 + P - 1 + 127) << 20;
  a.u_exact = (uint32_t)(1 - B - P + 127) << 23;
  a.map_add = 0u - (f.rebias << f.shift_p) - ((uint32_t)1 << (23 + P));
  a.split = (float)((uint32_t)1 << (23 + P));
  a.plain_ok = f.unit_lsb == 0u && m.nbits <= (uint32_t)kMaxTileNbits && 1 - B - P + 127 >= 1 ? 1u : 0u;
  a.row_sum_exact = (int)(f.max_code >> (P - 1)) + P - 1 <= 22 ? 1u : 0u;   // M < 2^(e_max + P - 1) grid steps
  const int W = m.nbits ? slot_width((int)m.nbits) : 0;
  const Split s = split_range(n, offset, W ? W : 8, W == 0, reinterpret_cast<uintptr_t>(x), 4, 16, reinterpret_cast<uintptr_t>(out),
                              1, 4, 0, 0, 1, kStatsPairElems);
  const uint64_t head = group < kStatsMinGroup ? 0 : s.head;
  const uint64_t npairs = group < kStatsMinGroup ? 0 : s.ntiles;
  hipError_t e = launch_bins8(x, out, head, a, t, W, seed, offset, group, first_bin, stats, stream);
  if (e != hipSuccess) return e;
  if (npairs) {
    const uint64_t i0 = offset + head;
    const uint64_t blk0 = W ? i0 / (uint64_t)(128 / W) : 0;
    uint8_t* o = out ? out + head : nullptr;
    switch (W) {
      case 0: e = launch_spans8<0>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      case 1: e = launch_spans8<1>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      case 2: e = launch_spans8<2>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      case 4: e = launch_spans8<4>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      case 8: e = launch_spans8<8>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      case 16: e = launch_spans8<16>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
      default: e = launch_spans8<32>(x + head, o, npairs, a, t, seed, blk0, i0, group, first_bin, workspace, stats, stream); break;
    }
    if (e != hipSuccess) return e;
    e = launch_stats_finalize(workspace, i0, i0 + npairs * kStatsPairElems, group, first_bin, stats, stream);
    if (e != hipSuccess) return e;
  }
  const uint64_t done = head + npairs * kStatsPairElems;
  return launch_bins8(x + done, out ? out + done : nullptr, n - done, a, t, W, seed, offset + done, group, first_bin, stats, stream);
}

}  // namespace fbsr
