// Forward-form implicit-GEMM convolution on fp32 MFMA (v_mfma_f32_16x16x4_f32), gfx950.
//
// One workgroup (4 wavefronts of 64) produces a 32-wide x (8*RP)-tall tile of pre-pool
// outputs of one image for NT*16 output channels.  Pixels sit on the MFMA M axis, output
// channels on N, the (channel, tap) contraction on K:
//   * an M-tile is 16 pixels = 4 pooling windows x 4 window positions, arranged so that the
//     4 accumulator registers of a lane are exactly the 2x2 window of one pooled pixel:
//     max-pooling, its arg-max, bias and activation need no cross-lane traffic;
//   * the 4 M-tiles a lane owns in a row pair are 4 neighbouring pooled columns, so the
//     pooled result leaves as one 16-byte store per lane;
//   * the input halo tile and the filter slice of the current channel chunk live in LDS;
//     the A operand is gathered from the halo tile with a per-step tap offset, the B
//     operand is a contiguous 64-float row of the filter slice.
// The source can be a plain tensor (forward layer, CRBM reconstruction) or the virtual
// tensor dz = unpool(dy) * act'(y) (backward-data layer), which is formed while staging and
// never reaches HBM.  With w_flip the filters are read rotated by 180 degrees and with the
// channel roles swapped, which turns the paper's "full convolution" (Section II-A) into this
// same valid-convolution engine run on an input padded by R-1-pad.
#include "dll_internal.h"

#include <type_traits>

namespace dllk {

typedef float floatx4 __attribute__((ext_vector_type(4)));

namespace {

constexpr int kThreads = 256;
constexpr int kTileW = 32;

struct EngineGeom {
  int CC, nchunks;   // channels per chunk, number of chunks
  int rows, cols;    // staged halo tile extent
  int RS, PS;        // LDS row / plane stride (floats)
  int KC, KS;        // padded taps per chunk (multiple of 4), MFMA steps per chunk
  int tiles_x, tiles_y;
  int kgroups;       // groups of NT*16 output channels (gridDim.y)
  int jw_log;        // generic kernel: log2 of the filter columns staged per N-tile (16, or fewer when Kout is small)
  unsigned src_bytes; // 3x3 instance: bytes of the source tensor (below 2 GiB)
  int pack3;          // 3x3 instance, three input channels: the 27 taps run as 7 MFMA steps, not 9
};

struct EngineParams {
  ConvEngineArgs a;
  EngineGeom g;
};

__device__ __forceinline__ float act_apply(int act, float z) {
  if (act == ACT_SIGMOID) return 1.0f / (1.0f + expf(-z));
  if (act == ACT_RELU) return z > 0.0f ? z : 0.0f;
  return z;
}

__device__ __forceinline__ float act_deriv(int act, float out) {
  if (act == ACT_SIGMOID) return out * (1.0f - out);
  if (act == ACT_RELU) return out > 0.0f ? 1.0f : 0.0f;
  return 1.0f;
}

// Probabilistic max pooling over one 2x2 block (Section II, the CRBM's pooling form): the four
// units (inputs z[v] + bias) and the state "all off" form one multinomial with weights exp(input)
// and 1; the largest exponent is subtracted before exponentiating.
__device__ __forceinline__ floatx4 pmp_block(const floatx4 z, float bias) {
  const float i0 = z[0] + bias, i1 = z[1] + bias, i2 = z[2] + bias, i3 = z[3] + bias;
  const float m = fmaxf(fmaxf(fmaxf(i0, i1), fmaxf(i2, i3)), 0.0f);
  const float e0 = expf(i0 - m), e1 = expf(i1 - m), e2 = expf(i2 - m), e3 = expf(i3 - m);
  const float inv = 1.0f / (expf(-m) + ((e0 + e1) + (e2 + e3)));
  return floatx4{e0 * inv, e1 * inv, e2 * inv, e3 * inv};
}

// dy times act'(y) for a pooled element: from the layer output, or from the index byte's flag.
__device__ __forceinline__ float pooled_dz(int act, float g, float out, unsigned char f) {
  if (act == ACT_RELU_FLAGGED) return (f & kIdxInactive) ? 0.0f : g;
  return act != ACT_IDENTITY ? g * act_deriv(act, out) : g;
}
__host__ __device__ __forceinline__ bool reads_output(int act) { return act == ACT_SIGMOID || act == ACT_RELU; }

// The lane's bias values, one per N-tile (output channel ko0 + 16nt + i16).  Read once per
// workgroup, ahead of the tile loop: a load inside the epilogue would be waited for on the spot,
// together with every prefetch load issued before it.
template <int NT>
__device__ __forceinline__ void lane_bias(const ConvEngineArgs &a, int ko0, int i16, float (&bias)[NT]) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int ko = ko0 + nt * 16 + i16;
    bias[nt] = (a.bias && ko < a.Kout) ? a.bias[ko] : 0.0f;
  }
}

// Epilogue shared by the engine kernels.  Lane owns output channel ko0+16nt+i16, window column
// 4*kq+mt of the tile, window row wave*RP+rp; acc[..][v] is window position v = 2a+b.
template <int NT, int RP, int ACT, int POOL>
__device__ __forceinline__ void engine_epilogue_as(const ConvEngineArgs &a, floatx4 (&acc)[RP][4][NT], const float (&bias)[NT],
                                                int n, int ko0, int oy0, int ox0, int wave, int i16, int kq) {
#pragma unroll
  for (int nt = 0; nt < NT; ++nt) {
    const int ko = ko0 + nt * 16 + i16;
    if (ko >= a.Kout) continue;
    const float bv = bias[nt];
#pragma unroll
    for (int rp = 0; rp < RP; ++rp) {
      const int py = (oy0 >> 1) + wave * RP + rp;   // window row (pre-pool rows 2py, 2py+1)
      const int px0 = (ox0 >> 1) + 4 * kq;          // first of the lane's 4 window columns
      if (2 * py >= a.Hout) continue;
      if (POOL == 2) {
        const int Hp = a.Hout >> 1, Wp = a.Wout >> 1;
        float yv[4];
        unsigned char iv[4];
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          const floatx4 z = acc[rp][mt][nt];
          float m = z[0];
          int arg = 0;
          if (z[1] > m) { m = z[1]; arg = 1; }
          if (z[2] > m) { m = z[2]; arg = 2; }
          if (z[3] > m) { m = z[3]; arg = 3; }
          yv[mt] = act_apply(ACT, m + bv);   // bias and a monotone activation commute with max
          iv[mt] = (unsigned char)(arg | ((ACT == ACT_RELU && !(yv[mt] > 0.0f)) ? kIdxInactive : 0));
        }
        const int o = ((n * a.Kout + ko) * Hp + py) * Wp + px0;
        if (px0 + 3 < Wp && (Wp & 3) == 0) {
          *reinterpret_cast<float4 *>(a.out + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
          if (a.out_idx) *reinterpret_cast<uchar4 *>(a.out_idx + o) = make_uchar4(iv[0], iv[1], iv[2], iv[3]);
        } else {
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
            if (px0 + mt < Wp) {
              a.out[o + mt] = yv[mt];
              if (a.out_idx) a.out_idx[o + mt] = iv[mt];
            }
        }
      } else {
        // the lane's four windows: unit outputs pr[mt][2a+b] and, for the sampling epilogues, their states
        floatx4 pr[4], sm[4] = {};
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) {
          if (ACT == ACT_PMP) {
            pr[mt] = pmp_block(acc[rp][mt][nt], bv);
          } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) pr[mt][v] = act_apply(ACT, acc[rp][mt][nt][v] + bv);
          }
        }
        if (ACT == ACT_PMP) {
          // one uniform number per block picks among "unit v on" (v = 0..3) and "all off"; the
          // pooling unit's probability is the sum of its block
          const int Hp = a.Hout >> 1, Wp = a.Wout >> 1;
          const int ob = ((n * a.Kout + ko) * Hp + py) * Wp + px0;
          float ub[4];   // the blocks' uniform numbers, loaded together from clamped addresses
          if (a.sample) {
#pragma unroll
            for (int mt = 0; mt < 4; ++mt) ub[mt] = a.uniform[ob - px0 + min(px0 + mt, Wp - 1)];   // stays inside the row
          }
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
            if (px0 + mt >= Wp) continue;
            if (a.out_pool) a.out_pool[ob + mt] = (pr[mt][0] + pr[mt][1]) + (pr[mt][2] + pr[mt][3]);
            if (a.sample) {
              const float u = ub[mt];
              float lo = 0.0f;
              bool taken = false;
#pragma unroll
              for (int v = 0; v < 4; ++v) {
                const float hi = lo + pr[mt][v];
                const bool on = !taken && lo <= u && u < hi;
                sm[mt][v] = on ? 1.0f : 0.0f;
                taken = taken || on;
                lo = hi;
              }
            }
          }
        }
#pragma unroll
        for (int wa2 = 0; wa2 < 2; ++wa2) {
          const int oy = 2 * py + wa2;
          if (oy >= a.Hout) continue;
          const int ox = 2 * px0;
          const int o = ((n * a.Kout + ko) * a.Hout + oy) * a.Wout + ox;
          float yv[8], sv[8];
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) {
            yv[2 * mt] = pr[mt][2 * wa2];
            yv[2 * mt + 1] = pr[mt][2 * wa2 + 1];
            if (ACT == ACT_PMP) { sv[2 * mt] = sm[mt][2 * wa2]; sv[2 * mt + 1] = sm[mt][2 * wa2 + 1]; }
          }
          if (ox + 7 < a.Wout && (a.Wout & 3) == 0) {
            *reinterpret_cast<float4 *>(a.out + o) = make_float4(yv[0], yv[1], yv[2], yv[3]);
            *reinterpret_cast<float4 *>(a.out + o + 4) = make_float4(yv[4], yv[5], yv[6], yv[7]);
            if (a.sample) {
              if (ACT != ACT_PMP) {
                const float4 u0 = *reinterpret_cast<const float4 *>(a.uniform + o);
                const float4 u1 = *reinterpret_cast<const float4 *>(a.uniform + o + 4);
                sv[0] = u0.x < yv[0] ? 1.f : 0.f; sv[1] = u0.y < yv[1] ? 1.f : 0.f;
                sv[2] = u0.z < yv[2] ? 1.f : 0.f; sv[3] = u0.w < yv[3] ? 1.f : 0.f;
                sv[4] = u1.x < yv[4] ? 1.f : 0.f; sv[5] = u1.y < yv[5] ? 1.f : 0.f;
                sv[6] = u1.z < yv[6] ? 1.f : 0.f; sv[7] = u1.w < yv[7] ? 1.f : 0.f;
              }
              *reinterpret_cast<float4 *>(a.sample + o) = make_float4(sv[0], sv[1], sv[2], sv[3]);
              *reinterpret_cast<float4 *>(a.sample + o + 4) = make_float4(sv[4], sv[5], sv[6], sv[7]);
            }
          } else {
            // ragged row end: the uniform numbers first, all of them and from clamped addresses (a
            // load behind the per-lane range check would be waited for on its own, eight in a row)
            float uv[8];
            if (a.sample && ACT != ACT_PMP) {
#pragma unroll
              for (int e = 0; e < 8; ++e) uv[e] = a.uniform[o - ox + min(ox + e, a.Wout - 1)];   // stays inside the row
            }
#pragma unroll
            for (int e = 0; e < 8; ++e)
              if (ox + e < a.Wout) {
                a.out[o + e] = yv[e];
                if (a.sample) a.sample[o + e] = ACT == ACT_PMP ? sv[e] : (uv[e] < yv[e] ? 1.f : 0.f);
              }
          }
        }
      }
    }
  }
}

// The activation and the pooling mode are fixed for a launch: dispatch once, so that the
// per-element code carries no branches on them.
template <int NT, int RP>
__device__ __forceinline__ void engine_epilogue(const ConvEngineArgs &a, floatx4 (&acc)[RP][4][NT], const float (&bias)[NT],
                                                int n, int ko0, int oy0, int ox0, int wave, int i16, int kq) {
#define DLL_EPI(ACT_, POOL_) engine_epilogue_as<NT, RP, ACT_, POOL_>(a, acc, bias, n, ko0, oy0, ox0, wave, i16, kq)
  if (a.pool == 2) {
    if (a.act == ACT_RELU) DLL_EPI(ACT_RELU, 2);
    else if (a.act == ACT_SIGMOID) DLL_EPI(ACT_SIGMOID, 2);
    else DLL_EPI(ACT_IDENTITY, 2);
  } else {
    if (a.act == ACT_RELU) DLL_EPI(ACT_RELU, 1);
    else if (a.act == ACT_SIGMOID) DLL_EPI(ACT_SIGMOID, 1);
    else if (a.act == ACT_PMP) DLL_EPI(ACT_PMP, 1);
    else DLL_EPI(ACT_IDENTITY, 1);
  }
#undef DLL_EPI
}

template <int NT, int RP>
__global__ __launch_bounds__(kThreads) void conv_engine_kernel(const EngineParams p) {
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const EngineGeom &g = p.g;
  float *xs = lds;                                  // [CC][PS]
  float *wl = xs + g.CC * g.PS;                     // [NT][KC][16]
  int *koff = reinterpret_cast<int *>(wl + NT * g.KC * 16);  // [KC]
  int2 *wtab = reinterpret_cast<int2 *>(koff + g.KC);        // [KC]: offset of tap kk inside a filter slice (-1: padding), channel

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int bid = blockIdx.x;
  const int tx = bid % g.tiles_x;
  const int ty = (bid / g.tiles_x) % g.tiles_y;
  const int n = bid / (g.tiles_x * g.tiles_y);
  const int ko0 = blockIdx.y * (NT * 16);
  constexpr int TH = 8 * RP;
  const int oy0 = ty * TH, ox0 = tx * kTileW;       // pre-pool output origin of the tile
  const int RSf = a.R * a.S;

  // tap offsets inside the halo tile: kk = (r*S + s)*CC + cl  ->  cl*PS + r*RS + s, and inside the
  // filter tensor relative to the chunk's first channel (rotated and transposed filters: w_flip)
  for (int kk = tid; kk < g.KC; kk += kThreads) {
    const int cl = kk % g.CC, rs = kk / g.CC;
    const int r = rs / a.S, s = rs - r * a.S;
    koff[kk] = rs < RSf ? cl * g.PS + r * g.RS + s : 0;
    const int wo = a.w_flip ? cl * a.Kout * RSf + (a.R - 1 - r) * a.S + (a.S - 1 - s) : cl * RSf + r * a.S + s;
    wtab[kk] = make_int2(rs < RSf ? wo : -1, cl);
  }
  // Only the first 2^jw_log columns of a filter slice can be non-zero (Kout is small); the others
  // are cleared once here and never written again.
  const int jw = 1 << g.jw_log;
  if (jw < 16)
    for (int e = tid; e < NT * g.KC * 16; e += kThreads) wl[e] = 0.0f;

  floatx4 acc[RP][4][NT];
#pragma unroll
  for (int rp = 0; rp < RP; ++rp)
#pragma unroll
    for (int mt = 0; mt < 4; ++mt)
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) acc[rp][mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};

  // lane's pixel inside an M-tile: window gq, position (wa, wb)
  const int gq = i16 >> 2, wa = (i16 >> 1) & 1, wb = i16 & 1;
  const int a_base = (wave * 2 * RP + wa) * g.RS + 8 * gq + wb;

  for (int chunk = 0; chunk < g.nchunks; ++chunk) {
    const int c0 = chunk * g.CC;
    __syncthreads();  // previous chunk's readers are done
    // Both staging loops work in batches of kStage elements per thread: all addresses first, then all
    // loads, unconditionally and from clamped addresses (element 0 stands in for anything that is
    // padding or out of range), then the selects and the LDS stores.  A load behind a per-lane
    // branch would be waited for before the next one is issued.
    constexpr int kStage = 4;
    // ---- filter slice: wl[nt][kk][j] = wgt(ko0 + 16nt + j, c0 + cl, r, s) for the columns j < jw
    const int f_total = NT * g.KC * jw;
    const int w_base = a.w_flip ? c0 * a.Kout * RSf : c0 * RSf;   // + ko * RSf (flipped) or ko * Cin * RSf
    const int w_ko = a.w_flip ? RSf : a.Cin * RSf;
    for (int e0 = tid; e0 < f_total; e0 += kStage * kThreads) {
      float v[kStage];
      bool ok[kStage];
      int dst[kStage];
#pragma unroll
      for (int u = 0; u < kStage; ++u) {
        const int e = min(e0 + u * kThreads, f_total - 1);
        const int j = e & (jw - 1);
        int kk = e >> g.jw_log, nt = 0;
        while (kk >= g.KC) { kk -= g.KC; ++nt; }   // at most NT - 1 rounds
        const int2 t = wtab[kk];
        const int ko = ko0 + nt * 16 + j;
        ok[u] = t.x >= 0 && ko < a.Kout && c0 + t.y < a.Cin;
        dst[u] = (nt * g.KC + kk) * 16 + j;
        v[u] = a.w[ok[u] ? w_base + ko * w_ko + t.x : 0];
      }
#pragma unroll
      for (int u = 0; u < kStage; ++u)
        if (e0 + u * kThreads < f_total) wl[dst[u]] = ok[u] ? v[u] : 0.0f;
    }
    // ---- halo tile of the source, zero outside the image (padding) and past Cin
    {
      const int total = g.CC * g.rows * g.cols;
      int col = tid % g.cols;
      int q = tid / g.cols;
      int row = q % g.rows, cl = q / g.rows;
      const int dcol = kThreads % g.cols, dq = kThreads / g.cols;
      const int Hp = a.Hin >> 1, Wp = a.Win >> 1;   // pooled dz sources only
      const bool pooled = a.src_dz && a.src_pool == 2;
      const bool need_y = a.src_dz && reads_output(a.src_act);
      for (int e0 = tid; e0 < total; e0 += kStage * kThreads) {
        float gv[kStage], yv[kStage];
        unsigned char fv[kStage];
        bool ok[kStage];
        int dst[kStage], want[kStage];
#pragma unroll
        for (int u = 0; u < kStage; ++u) {
          const int gi = oy0 - a.pad_h + row, gj = ox0 - a.pad_w + col, ci = c0 + cl;
          ok[u] = e0 + u * kThreads < total && ci < a.Cin && gi >= 0 && gi < a.Hin && gj >= 0 && gj < a.Win;
          dst[u] = cl * g.PS + row * g.RS + col;
          want[u] = ((gi & 1) << 1) | (gj & 1);
          int o = pooled ? ((n * a.Cin + ci) * Hp + (gi >> 1)) * Wp + (gj >> 1) : ((n * a.Cin + ci) * a.Hin + gi) * a.Win + gj;
          o = ok[u] ? o : 0;
          gv[u] = a.src[o];
          yv[u] = need_y ? a.src_y[o] : 0.0f;
          fv[u] = pooled ? a.src_idx[o] : (unsigned char)0;
          col += dcol;
          row += dq;
          if (col >= g.cols) { col -= g.cols; ++row; }
          while (row >= g.rows) { row -= g.rows; ++cl; }
        }
#pragma unroll
        for (int u = 0; u < kStage; ++u) {
          if (e0 + u * kThreads >= total) continue;
          float v = gv[u];
          if (a.src_dz) {
            // dz at a pre-pool position: dy routed to the recorded arg-max, times act'(y)
            if (pooled && (fv[u] & kIdxPosMask) != (unsigned char)want[u]) v = 0.0f;
            if (a.src_act == ACT_RELU_FLAGGED) v = (fv[u] & kIdxInactive) ? 0.0f : v;
            else if (a.src_act == ACT_SIGMOID) v *= yv[u] * (1.0f - yv[u]);
            else if (a.src_act == ACT_RELU) v = yv[u] > 0.0f ? v : 0.0f;
          }
          xs[dst[u]] = ok[u] ? v : 0.0f;
        }
      }
    }
    __syncthreads();
    // ---- MFMA over the chunk's taps, software-pipelined over two register sets: while step t is
    // multiplied, the operand fragments of step t+1 are on their way from LDS and the tap offset of
    // step t+2 is being read (offset -> fragment -> MFMA is a chain of two LDS latencies that a
    // plain loop would pay at every step).  Steps past the end re-read the last step and are not
    // multiplied.
    {
      float afA[RP * 4], bfA[NT], afB[RP * 4], bfB[NT];
      auto load_step = [&](int t, int o, float (&af)[RP * 4], float (&bf)[NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bf[nt] = wl[(nt * g.KC + 4 * t + kq) * 16 + i16];
#pragma unroll
        for (int rp = 0; rp < RP; ++rp)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) af[rp * 4 + mt] = xs[a_base + rp * 2 * g.RS + o + 2 * mt];
      };
      auto mfma_step = [&](const float (&af)[RP * 4], const float (&bf)[NT]) __attribute__((always_inline)) {
#pragma unroll
        for (int rp = 0; rp < RP; ++rp)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
              acc[rp][mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[rp * 4 + mt], bf[nt], acc[rp][mt][nt], 0, 0, 0);
      };
      const int last = g.KS - 1;
      int o1 = koff[4 * min(1, last) + kq];
      load_step(0, koff[kq], afA, bfA);
      for (int t = 0; t < g.KS; t += 2) {
        const int o2 = koff[4 * min(t + 2, last) + kq];
        load_step(min(t + 1, last), o1, afB, bfB);
        __builtin_amdgcn_sched_barrier(0);
        mfma_step(afA, bfA);
        __builtin_amdgcn_sched_barrier(0);
        const int o3 = koff[4 * min(t + 3, last) + kq];
        load_step(min(t + 2, last), o2, afA, bfA);
        __builtin_amdgcn_sched_barrier(0);
        if (t + 1 < g.KS) mfma_step(afB, bfB);
        __builtin_amdgcn_sched_barrier(0);
        o1 = o3;
      }
    }
  }
  float bias_v[NT];
  lane_bias<NT>(a, ko0, i16, bias_v);
  engine_epilogue<NT, RP>(a, acc, bias_v, n, ko0, oy0, ox0, wave, i16, kq);
}

inline int round_up_mod(int v, int m, int r) {  // smallest value >= v congruent to r mod m
  int x = v - (v % m) + r;
  if (x < v) x += m;
  return x;
}

bool plan_engine(const ConvEngineArgs &a, int NT, int RP, EngineGeom *g, size_t *lds_bytes) {
  const int TH = 8 * RP;
  g->rows = TH + a.R - 1;
  g->cols = kTileW + a.S - 1;
  g->RS = round_up_mod(g->cols, 8, 2);
  g->PS = round_up_mod(g->RS * g->rows, 8, 4);
  int CC = a.Cin < 16 ? a.Cin : 16;
  for (;;) {
    g->CC = CC;
    g->KC = (CC * a.R * a.S + 3) / 4 * 4;
    g->KS = g->KC / 4;
    *lds_bytes = sizeof(float) * ((size_t)CC * g->PS + (size_t)NT * g->KC * 16 + 3 * (size_t)g->KC);
    if (*lds_bytes <= 64 * 1024 || CC == 1) break;
    CC = (CC + 1) / 2;
  }
  if (*lds_bytes > 64 * 1024) return false;
  g->nchunks = (a.Cin + g->CC - 1) / g->CC;
  g->tiles_x = (a.Wout + kTileW - 1) / kTileW;
  g->tiles_y = (a.Hout + TH - 1) / TH;
  g->kgroups = (a.Kout + NT * 16 - 1) / (NT * 16);
  g->jw_log = 4;
  if (NT == 1 && a.Kout < 16)
    while (g->jw_log > 0 && (1 << (g->jw_log - 1)) >= a.Kout) --g->jw_log;
  return true;
}

template <int NT, int RP>
hipError_t launch_t(const ConvEngineArgs &a, hipStream_t stream) {
  EngineParams p;
  p.a = a;
  size_t lds = 0;
  if (!plan_engine(a, NT, RP, &p.g, &lds)) return hipErrorInvalidValue;
  const long blocks = (long)a.N * p.g.tiles_x * p.g.tiles_y;
  if (blocks <= 0 || blocks > 0x7fffffffL) return hipErrorInvalidValue;
  dim3 grid((unsigned)blocks, (unsigned)p.g.kgroups, 1);
  hipLaunchKernelGGL((conv_engine_kernel<NT, RP>), grid, dim3(kThreads), lds, stream, p);
  return hipGetLastError();
}


// ---------------------------------------------------------------------------------------
// 3x3, pad 1, 16-channel chunks: the instance every deeper layer of the paper's CNNs uses
// (Sections V and VI: 3x3 convolutions), forward and backward-data alike (pad' = 3-1-1 = 1).
// Same tiling as the generic kernel, with everything the MFMA loop needs known at compile
// time: reduction order (tap major, channel minor) makes a step's four k-indices four
// neighbouring channels, so the lane-dependent part of every LDS address is one base
// register and all tap / M-tile / chunk displacements are instruction immediates.  Staging
// uses 16-byte global loads; in backward-data mode it reads dy, y and the arg-max bytes at
// pooled resolution and expands each element to its 2x2 window while storing to LDS.
// LDS strides RS = 36 (4 mod 8), PS = 2 mod 8: conflict-free operand reads, 8-byte aligned
// vector stores (tile column 0 sits at LDS column 1 so that the aligned interior starts at 2).
// ---------------------------------------------------------------------------------------
constexpr int round_up_mod_c(int v, int m, int r) { return (v - (v % m) + r) < v ? (v - (v % m) + r + m) : (v - (v % m) + r); }

// waves per SIMD the register budget is held to: LDS lets 3 (16 filters) or 2 (32 filters)
// workgroups of the 16-channel instance share a CU, 4 of the 8- and 4-channel ones
constexpr int conv3x3_occupancy(int NT, int WAVES, int CC) { return (CC <= 8 ? 4 : (NT == 1 ? 3 : 2)) * WAVES / 4; }

// SRC: 0 plain tensor, 1 dz without pooling, 2 dz through 2x2 pooling.  CC: channels per chunk:
// 16 (32 filters per workgroup), 8 (16 filters: the smaller tile lets a fourth workgroup share the
// CU), or 4 for shallow inputs such as RGB images (surplus channels are staged as zeros).
// EPI fixes the epilogue at compile time where the launcher knows it: 1 = bias + ReLU + 2x2 pool
// (the forward pass of the networks this path is for), 2 = plain store (backward-data), 0 = decided
// at run time (any activation, pooling or sampling).  The fixed forms keep the other epilogues'
// code out of the kernel.
template <int NT, int WAVES, int SRC, int CC, bool PACK3 = false, int EPI = 0>
__global__ __launch_bounds__(WAVES * 64, conv3x3_occupancy(NT, WAVES, CC)) void conv3x3c16_kernel(const EngineParams p) {
  static_assert(!PACK3 || (CC == 4 && SRC == 0), "the packed three-channel path is a forward path of the 4-channel instance");
  constexpr int NTHR = WAVES * 64, RP = 8 / WAVES;   // 16-row tile: every wave owns RP row pairs
  constexpr int TH = 16, ROWS = TH + 2, C4 = CC / 4;
  constexpr int RS = 36, PS = round_up_mod_c(RS * ROWS, 8, 2);
  constexpr int KC = CC * 9;
  extern __shared__ float lds[];
  const ConvEngineArgs &a = p.a;
  const EngineGeom &g = p.g;
  float *xs = lds;               // [CC][PS]
  float *wl = xs + CC * PS;      // [chunk][NT][9*CC][16]

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int i16 = lane & 15, kq = lane >> 4;
  const int ko0 = blockIdx.y * (NT * 16);
  const int tiles = a.N * g.tiles_x * g.tiles_y;
  const int work = tiles * g.nchunks;          // (tile, chunk) pairs, chunk fastest
  const int Hp = a.Hin >> 1, Wp = a.Win >> 1;  // SRC == 2 only

  // ---- filter slices of every chunk, once per workgroup: wl[chunk][nt][rs*CC + cl][j];
  // three-channel inputs: wl[nt][k][j] with k = (c*3 + r)*3 + s, the filter's own order, and a zero row 27
  if (PACK3) {
    for (int e = tid; e < NT * 28 * 16; e += NTHR) {
      const int j = e & 15, q = e >> 4;
      const int k = q % 28, nt = q / 28;
      const int ko = ko0 + nt * 16 + j;
      wl[e] = (k < 27 && ko < a.Kout) ? a.w[ko * 27 + k] : 0.0f;
    }
  } else
  for (int e = tid; e < g.nchunks * NT * KC * 16; e += NTHR) {
    const int j = e & 15, q = e >> 4;
    const int kk = q % KC, q2 = q / KC;
    const int nt = q2 % NT, chunk = q2 / NT;
    const int cl = kk % CC, rs = kk / CC;
    const int r = rs / 3, s = rs - 3 * r;
    const int ko = ko0 + nt * 16 + j, ci = chunk * CC + cl;
    float v = 0.0f;
    if (ko < a.Kout && ci < a.Cin)
      v = a.w_flip ? a.w[((ci * a.Kout + ko) * 3 + (2 - r)) * 3 + (2 - s)] : a.w[((ko * a.Cin + ci) * 3 + r) * 3 + s];
    wl[e] = v;
  }

  // ---- staging: global -> registers -> LDS halo tile xs[cl][18 rows][36]: tile column t lives at
  // LDS column t + 2, the left halo at column 1, the right one at column 34.
  // Slots are dealt so that a thread's slot in round `it` differs from round 0 only by whole
  // channels: its global offset and LDS address are fixed for the whole kernel, the per-round part
  // is uniform (scalar offset of the buffer load, immediate of the LDS store).  Loads are
  // range-checked buffer loads: a slot outside the image, beyond the last channel or beyond the
  // slot count gets an offset past the end of the buffer and reads zeros, which is exactly the
  // padding value; no branch, no select.
  constexpr unsigned kOob = 0x80000000u;          // byte offset beyond any buffer (tensors are < 2 GiB)
  const __amdgpu_buffer_rsrc_t rs_src = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src), 0, (int)g.src_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_y = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.src_y ? a.src_y : a.src), 0, (int)g.src_bytes, 0x00020000);
  const __amdgpu_buffer_rsrc_t rs_idx = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.src_idx ? a.src_idx : reinterpret_cast<const unsigned char *>(a.src)), 0, (int)(g.src_bytes >> 2), 0x00020000);
  auto ld4 = [&](const __amdgpu_buffer_rsrc_t &r, unsigned voff, unsigned soff) __attribute__((always_inline)) {
    const floatx4 v = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(r, (int)voff, (int)soff, 0));
    return make_float4(v[0], v[1], v[2], v[3]);
  };
  auto ld1 = [&](const __amdgpu_buffer_rsrc_t &r, unsigned voff, unsigned soff) __attribute__((always_inline)) {
    return __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r, (int)voff, (int)soff, 0));
  };
  const bool need_y = SRC == 2 ? reads_output(a.src_act) : (SRC == 1 && a.src_act != ACT_IDENTITY);
  // source plane geometry in elements (SRC == 2: the pooled planes)
  const int SH = SRC == 2 ? Hp : a.Hin, SW = SRC == 2 ? Wp : a.Win;
  const unsigned plane = (unsigned)SH * SW;

  // slot classes (TR = tile rows of the source: 16 plain rows or 8 pooled rows; G4 = 16-byte groups per row)
  constexpr int TR = SRC == 2 ? TH / 2 : TH, G4 = SRC == 2 ? 4 : 8;
  constexpr int M_PER_C = TR * G4;                      // main slots per channel
  constexpr int M_CPR = NTHR / M_PER_C;                 // channels per round
  constexpr int NM = (CC + M_CPR - 1) / M_CPR;          // main rounds
  constexpr int S_PER_C = TR * 2;                       // side (halo column) slots per channel
  constexpr int S_CPR = NTHR / S_PER_C;
  constexpr int NS = (CC + S_CPR - 1) / S_CPR;          // side rounds
  static_assert(NTHR % M_PER_C == 0 && CC * 2 * G4 <= NTHR && CC * 4 <= NTHR, "slot classes");
  // main: rows 0..TR-1 of the tile, 16-byte groups
  const int m_j = tid % G4, m_r = (tid / G4) % TR, m_c = tid / M_PER_C;
  // top/bottom halo rows, 16-byte groups: one round, threads below CC * 2 * G4
  const int t_j = tid % G4, t_b = (tid / G4) & 1, t_c = tid / (2 * G4);
  // side columns of rows 0..TR-1, single elements
  const int s_side = tid & 1, s_r = (tid >> 1) % TR, s_c = tid / S_PER_C;
  // corners, single elements: threads below CC * 4
  const int c_side = tid & 1, c_b = (tid >> 1) & 1, c_c = tid >> 2;
  // element offsets relative to (channel c0, row sy0, column sx0) of the tile, sy0/sx0 = tile origin in the source plane
  const int m_off = m_c * (int)plane + m_r * SW + 4 * m_j;
  const int t_off = t_c * (int)plane + (t_b ? TR : -1) * SW + 4 * t_j;
  const int s_off = s_c * (int)plane + s_r * SW + (s_side ? (SRC == 2 ? 16 : kTileW) : -1);
  const int c_off = c_c * (int)plane + (c_b ? TR : -1) * SW + (c_side ? (SRC == 2 ? 16 : kTileW) : -1);

  constexpr bool M_EXACT = NM * M_CPR == CC, S_EXACT = NS * S_CPR == CC;
  float4 vm[NM], ym[NM], vt, yt;
  float vs[NS], ys[NS], vc, yc;
  int im[NM], it_;                    // SRC == 2: four index bytes per group
  unsigned char is_[NS], ic;
  // registers of the optional operands start defined; they stay so when the loads are skipped
  yt = make_float4(0.f, 0.f, 0.f, 0.f); yc = 0.0f; it_ = 0; ic = 0;
#pragma unroll
  for (int it = 0; it < NM; ++it) { ym[it] = yt; im[it] = 0; }
#pragma unroll
  for (int it = 0; it < NS; ++it) { ys[it] = 0.0f; is_[it] = 0; }

  // global -> registers for work item q
  auto load_regs = [&](int q) {
    const int tile = q / g.nchunks, chunk = q - tile * g.nchunks;
    const int tx = tile % g.tiles_x;
    const int ty = (tile / g.tiles_x) % g.tiles_y;
    const int n = tile / (g.tiles_x * g.tiles_y);
    const int oy0 = ty * TH, ox0 = tx * kTileW, c0 = chunk * CC;
    const int sy0 = SRC == 2 ? oy0 >> 1 : oy0, sx0 = SRC == 2 ? ox0 >> 1 : ox0;
    const int cleft = a.Cin - c0;                                        // valid channels from c0 on
    const unsigned base = ((unsigned)(n * a.Cin + c0) * SH) * SW;      // element offset of (n, c0, 0, 0)
    const int pos = sy0 * SW + sx0;                                      // tile origin inside the plane
    // main
    {
      const bool ok = sy0 + m_r < SH && sx0 + 4 * m_j < SW;
      const unsigned e = (unsigned)(pos + m_off);
#pragma unroll
      for (int it = 0; it < NM; ++it) {
        // 8- and 16-channel chunks are always whole (the launcher checks that Cin is a multiple of the chunk)
        const bool okc = (CC >= 8 && M_EXACT) ? ok : ok && it * M_CPR + m_c < (cleft < CC ? cleft : CC);
        const unsigned so = base + (unsigned)it * M_CPR * plane;
        vm[it] = ld4(rs_src, okc ? 4u * e : kOob, 4u * so);
        if (need_y) ym[it] = ld4(rs_y, okc ? 4u * e : kOob, 4u * so);
        if (SRC == 2) im[it] = __builtin_amdgcn_raw_buffer_load_b32(rs_idx, (int)(okc ? e : kOob), (int)so, 0);
      }
    }
    // top / bottom halo rows
    {
      const int row = sy0 + (t_b ? TR : -1);
      const bool ok = tid < CC * 2 * G4 && (unsigned)row < (unsigned)SH && sx0 + 4 * t_j < SW && t_c < cleft;
      const unsigned e = (unsigned)(pos + t_off);
      vt = ld4(rs_src, ok ? 4u * e : kOob, 4u * base);
      if (need_y) yt = ld4(rs_y, ok ? 4u * e : kOob, 4u * base);
      if (SRC == 2) it_ = __builtin_amdgcn_raw_buffer_load_b32(rs_idx, (int)(ok ? e : kOob), (int)base, 0);
    }
    // side columns
    {
      const int col = sx0 + (s_side ? (SRC == 2 ? 16 : kTileW) : -1);
      const bool ok = sy0 + s_r < SH && (unsigned)col < (unsigned)SW;
      const unsigned e = (unsigned)(pos + s_off);
#pragma unroll
      for (int it = 0; it < NS; ++it) {
        const bool okc = (CC >= 8 && S_EXACT) ? ok : ok && it * S_CPR + s_c < (cleft < CC ? cleft : CC);
        const unsigned so = base + (unsigned)it * S_CPR * plane;
        vs[it] = ld1(rs_src, okc ? 4u * e : kOob, 4u * so);
        if (need_y) ys[it] = ld1(rs_y, okc ? 4u * e : kOob, 4u * so);
        if (SRC == 2) is_[it] = __builtin_amdgcn_raw_buffer_load_b8(rs_idx, (int)(okc ? e : kOob), (int)so, 0);
      }
    }
    // corners
    {
      const int row = sy0 + (c_b ? TR : -1), col = sx0 + (c_side ? (SRC == 2 ? 16 : kTileW) : -1);
      const bool ok = tid < CC * 4 && (unsigned)row < (unsigned)SH && (unsigned)col < (unsigned)SW && c_c < cleft;
      const unsigned e = (unsigned)(pos + c_off);
      vc = ld1(rs_src, ok ? 4u * e : kOob, 4u * base);
      if (need_y) yc = ld1(rs_y, ok ? 4u * e : kOob, 4u * base);
      if (SRC == 2) ic = __builtin_amdgcn_raw_buffer_load_b8(rs_idx, (int)(ok ? e : kOob), (int)base, 0);
    }
  };

  // registers -> LDS.  Plain sources: one 16-byte group is two 8-byte stores.  Pooled sources: a
  // pooled element (row pr, column pc) expands to LDS rows 2pr+1, 2pr+2 and columns 2pc+2, 2pc+3
  // (pr, pc relative to the tile; the halo row/column keep only the half that lies inside).
  float *const m_dst = SRC == 2 ? xs + m_c * PS + (2 * m_r + 1) * RS + 2 + 8 * m_j : xs + m_c * PS + (m_r + 1) * RS + 2 + 4 * m_j;
  float *const t_dst = SRC == 2 ? xs + t_c * PS + (t_b ? 17 : 0) * RS + 2 + 8 * t_j : xs + t_c * PS + (t_b ? 17 : 0) * RS + 2 + 4 * t_j;
  float *const s_dst = SRC == 2 ? xs + s_c * PS + (2 * s_r + 1) * RS + (s_side ? kTileW + 2 : 0) : xs + s_c * PS + (s_r + 1) * RS + (s_side ? kTileW + 2 : 1);
  float *const c_dst = SRC == 2 ? xs + c_c * PS + (c_b ? 17 : 0) * RS + (c_side ? kTileW + 2 : 0) : xs + c_c * PS + (c_b ? 17 : 0) * RS + (c_side ? kTileW + 2 : 1);
  auto put4 = [&](float *d, float4 v) __attribute__((always_inline)) {
    reinterpret_cast<float2 *>(d)[0] = make_float2(v.x, v.y);
    reinterpret_cast<float2 *>(d)[1] = make_float2(v.z, v.w);
  };
  // one window row (wa2 = 0 top, 1 bottom) of four pooled elements -> 8 floats
  auto put_pooled4 = [&](float *d, const float (&gg)[4], const unsigned char (&pos)[4], int wa2) __attribute__((always_inline)) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<float2 *>(d + 2 * q) = make_float2(pos[q] == 2 * wa2 ? gg[q] : 0.0f, pos[q] == 2 * wa2 + 1 ? gg[q] : 0.0f);
  };
  auto pooled_group = [&](auto actc, float4 v, float4 y, int idx4, float (&gg)[4], unsigned char (&pos)[4]) __attribute__((always_inline)) {
    constexpr int SA = decltype(actc)::value;
    const float gv[4] = {v.x, v.y, v.z, v.w}, ov[4] = {y.x, y.y, y.z, y.w};
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const unsigned char f = (unsigned char)((unsigned)idx4 >> (8 * q));
      gg[q] = pooled_dz(SA, gv[q], ov[q], f);
      pos[q] = f & kIdxPosMask;   // slots outside the image hold dy = 0
    }
  };
  auto store_regs_as = [&](auto actc) __attribute__((always_inline)) {
    constexpr int SA = decltype(actc)::value;
    constexpr bool need_y = SRC == 2 ? (SA == ACT_SIGMOID || SA == ACT_RELU) : (SRC == 1 && SA != ACT_IDENTITY);
    if (SRC != 2) {
#pragma unroll
      for (int it = 0; it < NM; ++it) {
        if (!M_EXACT && it * M_CPR + m_c >= CC) continue;   // slot beyond the chunk's channels
        float4 v = vm[it];
        if (need_y) {
          v.x *= act_deriv(SA, ym[it].x); v.y *= act_deriv(SA, ym[it].y);
          v.z *= act_deriv(SA, ym[it].z); v.w *= act_deriv(SA, ym[it].w);
        }
        put4(m_dst + it * M_CPR * PS, v);
      }
      if (tid < CC * 2 * G4) {
        float4 v = vt;
        if (need_y) {
          v.x *= act_deriv(SA, yt.x); v.y *= act_deriv(SA, yt.y);
          v.z *= act_deriv(SA, yt.z); v.w *= act_deriv(SA, yt.w);
        }
        put4(t_dst, v);
      }
#pragma unroll
      for (int it = 0; it < NS; ++it) {
        if (!S_EXACT && it * S_CPR + s_c >= CC) continue;
        s_dst[it * S_CPR * PS] = need_y ? vs[it] * act_deriv(SA, ys[it]) : vs[it];
      }
      if (tid < CC * 4) *c_dst = need_y ? vc * act_deriv(SA, yc) : vc;
    } else {
      float gg[4];
      unsigned char pos[4];
#pragma unroll
      for (int it = 0; it < NM; ++it) {
        if (!M_EXACT && it * M_CPR + m_c >= CC) continue;
        pooled_group(actc, vm[it], ym[it], im[it], gg, pos);
        put_pooled4(m_dst + it * M_CPR * PS, gg, pos, 0);
        put_pooled4(m_dst + it * M_CPR * PS + RS, gg, pos, 1);
      }
      if (tid < CC * 2 * G4) {
        // pooled row above the tile: only its bottom window row (LDS row 0); below: only its top one (row 17)
        pooled_group(actc, vt, yt, it_, gg, pos);
        put_pooled4(t_dst, gg, pos, t_b ? 0 : 1);
      }
#pragma unroll
      for (int it = 0; it < NS; ++it) {
        if (!S_EXACT && it * S_CPR + s_c >= CC) continue;
        // left neighbour window: LDS columns 0 (unused slot) and 1; right one: 34 and 35 (unused slot)
        const float g1 = pooled_dz(SA, vs[it], ys[it], is_[it]);
        const unsigned char hp = is_[it] & kIdxPosMask;
        float *d = s_dst + it * S_CPR * PS;
        *reinterpret_cast<float2 *>(d) = make_float2(hp == 0 ? g1 : 0.0f, hp == 1 ? g1 : 0.0f);
        *reinterpret_cast<float2 *>(d + RS) = make_float2(hp == 2 ? g1 : 0.0f, hp == 3 ? g1 : 0.0f);
      }
      if (tid < CC * 4) {
        const float g1 = pooled_dz(SA, vc, yc, ic);
        const unsigned char hp = ic & kIdxPosMask;
        const int wa2 = c_b ? 0 : 1;
        *reinterpret_cast<float2 *>(c_dst) = make_float2(hp == 2 * wa2 ? g1 : 0.0f, hp == 2 * wa2 + 1 ? g1 : 0.0f);
      }
    }
  };
  // the source activation is fixed for a launch: dispatch once, no per-element branches on it
  auto store_regs = [&]() __attribute__((always_inline)) {
    if (SRC == 0 || a.src_act == ACT_IDENTITY) store_regs_as(std::integral_constant<int, ACT_IDENTITY>{});
    else if (a.src_act == ACT_RELU) store_regs_as(std::integral_constant<int, ACT_RELU>{});
    else if (a.src_act == ACT_SIGMOID) store_regs_as(std::integral_constant<int, ACT_SIGMOID>{});
    else store_regs_as(std::integral_constant<int, ACT_RELU_FLAGGED>{});
  };

  floatx4 acc[RP][4][NT];
  float bias_v[NT];
  lane_bias<NT>(a, ko0, i16, bias_v);
  const int gq = i16 >> 2, wa = (i16 >> 1) & 1, wb = i16 & 1;
  const float *a_ptr = xs + kq * PS + (wave * 2 * RP + wa) * RS + 8 * gq + wb + 1;
  const float *b_ptr = wl + kq * 16 + i16;
  const float *a3[7];   // three-channel inputs: lane's tile pointer of MFMA step t (k = 4t + kq)
#pragma unroll
  for (int t = 0; t < (PACK3 ? 7 : 0); ++t) {
    const int k = 4 * t + kq, c = k / 9, tap = k - 9 * c;
    a3[t] = a_ptr - kq * PS + (k < 27 ? c * PS + (tap / 3) * RS + tap % 3 : 0);
  }

  // persistent loop over (tile, chunk) pairs; the next pair's global loads fly during the MFMA loop
  // Tile order is XCD-aware: workgroup ids are dealt round-robin to the 8 XCDs, each with its
  // own L2, so every XCD gets one contiguous eighth of the tiles and its workgroups stride
  // through it together: tiles in flight on an XCD are neighbours, and the halo columns and
  // cache-line halves they share meet in that XCD's L2.
  const int G = gridDim.x, nx = (G % 8 == 0) ? 8 : 1;
  const int xcd = blockIdx.x % nx, slot = blockIdx.x / nx, slots = G / nx;
  const int per_xcd = (tiles + nx - 1) / nx;
  const int tile_lim = min(tiles, (xcd + 1) * per_xcd);
  int cur_tile = xcd * per_xcd + slot;
  int q = cur_tile * g.nchunks;
  const auto next_q = [&](int qq) {   // next (tile, chunk) pair of this workgroup, or `work` when done
    const int t = qq / g.nchunks, c = qq - t * g.nchunks;
    if (c + 1 < g.nchunks) return qq + 1;
    return t + slots < tile_lim ? (t + slots) * g.nchunks : work;
  };
  if (cur_tile >= tile_lim) q = work;
  const int work_end = work;
  if (q < work_end) load_regs(q);
  while (q < work_end) {
    const int tile = q / g.nchunks, chunk = q - tile * g.nchunks;
    if (chunk == 0) {
#pragma unroll
      for (int rp = 0; rp < RP; ++rp)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt) acc[rp][mt][nt] = floatx4{0.f, 0.f, 0.f, 0.f};
    }
    __syncthreads();   // previous MFMA loop no longer reads the tile (first pass: filters are staged)
    store_regs();
    __syncthreads();
    const int qn = next_q(q);
    if (qn < work_end) load_regs(qn);
    // ---- MFMA: 9 taps x 4 channel groups; inside a tap every address is base + immediate.
    // Operand fragments are double-buffered in registers: the LDS reads of step t+1 are issued
    // before the MFMAs of step t, and scheduling barriers keep that order.
    const float *a_tap = a_ptr;
    const float *b_tap = b_ptr + chunk * (NT * KC * 16);
    float af[2][RP * 4], bf[2][NT];
    auto load_frags = [&](auto bufc, const float *at, const float *bt, int c4) {
      constexpr int B_ = decltype(bufc)::value;
#pragma unroll
      for (int nt = 0; nt < NT; ++nt) bf[B_][nt] = bt[(nt * KC + 4 * c4) * 16];
#pragma unroll
      for (int rp = 0; rp < RP; ++rp)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt) af[B_][rp * 4 + mt] = at[c4 * 4 * PS + rp * 2 * RS + 2 * mt];
    };
    auto mfma_frags = [&](auto bufc) {
      constexpr int B_ = decltype(bufc)::value;
#pragma unroll
      for (int rp = 0; rp < RP; ++rp)
#pragma unroll
        for (int mt = 0; mt < 4; ++mt)
#pragma unroll
          for (int nt = 0; nt < NT; ++nt)
            acc[rp][mt][nt] = __builtin_amdgcn_mfma_f32_16x16x4f32(af[B_][rp * 4 + mt], bf[B_][nt], acc[rp][mt][nt], 0, 0, 0);
    };
    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    if (!PACK3) load_frags(I0{}, a_tap, b_tap, 0);
    if constexpr (C4 == 4) {
#pragma unroll 1
      for (int rs = 0; rs < 9; ++rs) {
        const float *a_next = a_tap + ((rs % 3 == 2) ? RS - 2 : 1);   // next tap: s+1, or first column of the next filter row
        const float *b_next = b_tap + CC * 16;                          // CC channels x 16 output channels per tap
        load_frags(I1{}, a_tap, b_tap, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I0{});
        __builtin_amdgcn_sched_barrier(0);
        load_frags(I0{}, a_tap, b_tap, 2);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I1{});
        __builtin_amdgcn_sched_barrier(0);
        load_frags(I1{}, a_tap, b_tap, 3);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I0{});
        __builtin_amdgcn_sched_barrier(0);
        if (rs < 8) load_frags(I0{}, a_next, b_next, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I1{});
        __builtin_amdgcn_sched_barrier(0);
        a_tap = a_next;
        b_tap = b_next;
      }
    } else if constexpr (C4 == 2) {
      // 8-channel chunks: two steps per tap, the same two-set rotation
#pragma unroll 1
      for (int rs = 0; rs < 9; ++rs) {
        const float *a_next = a_tap + ((rs % 3 == 2) ? RS - 2 : 1);
        const float *b_next = b_tap + CC * 16;
        load_frags(I1{}, a_tap, b_tap, 1);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I0{});
        __builtin_amdgcn_sched_barrier(0);
        if (rs < 8) load_frags(I0{}, a_next, b_next, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(I1{});
        __builtin_amdgcn_sched_barrier(0);
        a_tap = a_next;
        b_tap = b_next;
      }
    } else if constexpr (PACK3) {
      // three input channels: k = 4t + kq runs over (channel, tap) in the filter's order; the lane's
      // seven tile offsets were worked out once (a3), the filter rows are 64 floats apart
      auto load3 = [&](auto bufc, auto tc) {
        constexpr int B_ = decltype(bufc)::value, t = decltype(tc)::value;
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bf[B_][nt] = b_ptr[(nt * 28 + 4 * t) * 16];
#pragma unroll
        for (int rp = 0; rp < RP; ++rp)
#pragma unroll
          for (int mt = 0; mt < 4; ++mt) af[B_][rp * 4 + mt] = a3[t][rp * 2 * RS + 2 * mt];
      };
      auto step3 = [&](auto tc) {
        constexpr int t = decltype(tc)::value;
        if constexpr (t < 6) load3(std::integral_constant<int, (t + 1) & 1>{}, std::integral_constant<int, t + 1>{});
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(std::integral_constant<int, t & 1>{});
        __builtin_amdgcn_sched_barrier(0);
      };
      load3(I0{}, I0{});
      step3(std::integral_constant<int, 0>{}); step3(std::integral_constant<int, 1>{});
      step3(std::integral_constant<int, 2>{}); step3(std::integral_constant<int, 3>{});
      step3(std::integral_constant<int, 4>{}); step3(std::integral_constant<int, 5>{});
      step3(std::integral_constant<int, 6>{});
    } else {
      // one step per tap: nine steps, fully unrolled, tap offsets are immediates
      auto tap_step = [&](auto rsc) {
        constexpr int rs = decltype(rsc)::value;
        if constexpr (rs < 8)
          load_frags(std::integral_constant<int, (rs + 1) & 1>{}, a_tap + ((rs + 1) / 3) * RS + (rs + 1) % 3,
                     b_tap + (rs + 1) * CC * 16, 0);
        __builtin_amdgcn_sched_barrier(0);
        mfma_frags(std::integral_constant<int, rs & 1>{});
        __builtin_amdgcn_sched_barrier(0);
      };
      tap_step(std::integral_constant<int, 0>{}); tap_step(std::integral_constant<int, 1>{});
      tap_step(std::integral_constant<int, 2>{}); tap_step(std::integral_constant<int, 3>{});
      tap_step(std::integral_constant<int, 4>{}); tap_step(std::integral_constant<int, 5>{});
      tap_step(std::integral_constant<int, 6>{}); tap_step(std::integral_constant<int, 7>{});
      tap_step(std::integral_constant<int, 8>{});
    }
    if (chunk + 1 == g.nchunks) {
      const int tx = tile % g.tiles_x;
      const int ty = (tile / g.tiles_x) % g.tiles_y;
      const int n = tile / (g.tiles_x * g.tiles_y);
      if constexpr (EPI == 1) engine_epilogue_as<NT, RP, ACT_RELU, 2>(a, acc, bias_v, n, ko0, ty * TH, tx * kTileW, wave, i16, kq);
      else if constexpr (EPI == 2) engine_epilogue_as<NT, RP, ACT_IDENTITY, 1>(a, acc, bias_v, n, ko0, ty * TH, tx * kTileW, wave, i16, kq);
      else engine_epilogue<NT, RP>(a, acc, bias_v, n, ko0, ty * TH, tx * kTileW, wave, i16, kq);
    }
    q = qn;
  }
}

constexpr size_t conv3x3c16_lds_bytes(int NT, int CC, int nchunks) {
  return sizeof(float) * ((size_t)CC * round_up_mod_c(36 * 18, 8, 2) + (size_t)nchunks * NT * 9 * CC * 16);
}

inline bool aligned16(const void *q) { return (reinterpret_cast<uintptr_t>(q) & 15u) == 0; }

// Which instance of the specialised kernel takes a layer: NT (16-filter groups per workgroup), wavefronts
// and channels per chunk; NT == 0: none applies.
struct Conv3x3Pick { int NT = 0, WAVES = 0, CC = 0; };

// The specialised kernel applies to 3x3 filters with one row/column of padding, channel
// counts that are multiples of 16 (of 8 for layers of at most 16 filters) or at most 12, rows that are
// whole 16-byte groups and aligned tensors, as long as the filter slices of ALL channel chunks,
// which a workgroup keeps in LDS for its whole life, fit the CU's LDS next to the halo tile
// (deeper layers take the generic kernel, which stages one chunk's slice at a time).
Conv3x3Pick conv3x3c16_pick(const ConvEngineArgs &a) {
  Conv3x3Pick none, pick;
  if (a.R != 3 || a.S != 3 || a.pad_h != 1 || a.pad_w != 1) return none;
  // whole 16-channel chunks, whole 8-channel chunks for layers of at most 16 filters, or up to three 4-channel chunks
  if (a.Cin % 16 != 0 && !(a.Cin % 8 == 0 && a.Kout <= 16) && a.Cin > 12) return none;
  if (a.Hout != a.Hin || a.Wout != a.Win) return none;
  if (!aligned16(a.src)) return none;
  // the kernel addresses the source through 32-bit byte offsets that must stay below 2 GiB
  if ((long)a.N * a.Cin * a.Hin * a.Win * 4 >= (1L << 31)) return none;
  if (a.src_dz) {
    // the dz instances store plainly: anything else on top of a backward-form pass takes the generic kernel
    if (a.act != ACT_IDENTITY || a.pool != 1) return none;
    if (reads_output(a.src_act) && !aligned16(a.src_y)) return none;
    if (a.src_pool == 2) {
      if (a.Win % 8 != 0 || (reinterpret_cast<uintptr_t>(a.src_idx) & 3u) != 0) return none;
    }
  }
  if (a.Win % 4 != 0) return none;
  // 16 output channels: 4 waves x 2 row pairs; 32: 8 waves x 1 row pair (more waves hide the
  // longer per-step operand traffic better than more accumulators do)
  if (a.Cin % 8 == 0 && a.Kout <= 16) pick = Conv3x3Pick{1, 4, 8};   // 8-channel chunks: four workgroups fit a CU's LDS instead of three
  else if (a.Cin % 16 != 0) pick = a.Kout <= 16 ? Conv3x3Pick{1, 4, 4} : Conv3x3Pick{2, 4, 4};
  else pick = Conv3x3Pick{2, 8, 16};   // wider layers run as groups of 32 output channels
  const int nchunks = (a.Cin + pick.CC - 1) / pick.CC;
  if (conv3x3c16_lds_bytes(pick.NT, pick.CC, nchunks) > chip().lds_bytes) return none;
  return pick;
}

template <int NT, int WAVES, int CC>
hipError_t launch_3x3(const ConvEngineArgs &a, hipStream_t stream) {
  EngineParams p;
  p.a = a;
  constexpr int TH = 16;
  p.g = EngineGeom{};
  p.g.CC = CC;
  p.g.nchunks = (a.Cin + CC - 1) / CC;
  p.g.tiles_x = (a.Wout + kTileW - 1) / kTileW;
  p.g.tiles_y = (a.Hout + TH - 1) / TH;
  p.g.kgroups = (a.Kout + NT * 16 - 1) / (NT * 16);
  p.g.pack3 = (CC == 4 && a.Cin == 3 && !a.src_dz && !a.w_flip) ? 1 : 0;
  {
    const long src_elems = (a.src_dz && a.src_pool == 2) ? (long)a.N * a.Cin * (a.Hin / 2) * (a.Win / 2) : (long)a.N * a.Cin * a.Hin * a.Win;
    p.g.src_bytes = (unsigned)(src_elems * 4);
  }
  const long tiles = (long)a.N * p.g.tiles_x * p.g.tiles_y;
  if (tiles <= 0 || tiles * p.g.nchunks > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t lds = conv3x3c16_lds_bytes(NT, CC, p.g.nchunks);
  if (lds > chip().lds_bytes) return hipErrorInvalidValue;   // conv3x3c16_pick lets no such layer through
  // persistent workgroups: as many as fit on the chip at once (LDS-limited), each walks tiles
  long resident = (long)(chip().lds_bytes / lds);
  constexpr long by_regs = conv3x3_occupancy(NT, WAVES, CC) / (WAVES / 4);
  if (resident > by_regs) resident = by_regs;
  long blocks = (long)chip().cus * resident / p.g.kgroups;
  if (blocks < 1) blocks = 1;
  // Every CU gets its full set of resident workgroups even when the tiles do not divide evenly:
  // the workgroups of one CU share its MFMA pipes, so what has to balance is the tile count per
  // CU (workgroups b, b+256, b+512, ... land on the same CU), not per workgroup.
  if (blocks > tiles) blocks = tiles;
  if (blocks >= 8) blocks = (blocks + 7) / 8 * 8;   // whole rows of XCDs (see the tile order in the kernel)
  dim3 grid((unsigned)blocks, (unsigned)p.g.kgroups, 1);
  auto launch = [&](auto kern) -> hipError_t {
    const hipError_t e = allow_large_lds(reinterpret_cast<const void *>(kern), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, grid, dim3(WAVES * 64), lds, stream, p);
    return hipGetLastError();
  };
  if (!a.src_dz) {
    const bool relu_pool = a.act == ACT_RELU && a.pool == 2;
    if constexpr (CC == 4) {
      if (p.g.pack3) return relu_pool ? launch(conv3x3c16_kernel<NT, WAVES, 0, CC, true, 1>) : launch(conv3x3c16_kernel<NT, WAVES, 0, CC, true, 0>);
    }
    return relu_pool ? launch(conv3x3c16_kernel<NT, WAVES, 0, CC, false, 1>) : launch(conv3x3c16_kernel<NT, WAVES, 0, CC, false, 0>);
  }
  // dz sources: the launcher only comes here with a plain-store epilogue (conv3x3c16_applies)
  if (a.src_pool == 2) return launch(conv3x3c16_kernel<NT, WAVES, 2, CC, false, 2>);
  return launch(conv3x3c16_kernel<NT, WAVES, 1, CC, false, 2>);
}

}  // namespace

hipError_t launch_conv_engine(const ConvEngineArgs &a, hipStream_t stream) {
  // 16 output channels per N-tile.  The generic kernel uses the 8-row tile for shallow maps
  // (<= 8 pre-pool rows) and whenever 16-row tiles would leave CUs without a workgroup.
  const int nt = a.Kout <= 16 ? 1 : (a.Kout <= 32 ? 2 : 3);
  const long tiles16 = (long)a.N * ((a.Wout + kTileW - 1) / kTileW) * ((a.Hout + 15) / 16) * ((a.Kout + nt * 16 - 1) / (nt * 16));
  const bool small = a.Hout <= 8 || tiles16 < 512;
  // very few output channels: the banded-filter kernel wins when its share of real products,
  // S of every 4*ceil((16+S-1)/4) window columns, clearly beats Kout of 16 channel columns
  if (a.Kout <= 3 && a.Kout * (4 * ((16 + a.S - 1 + 3) / 4)) * 3 < 16 * a.S * 2 && conv_fewout_applies(a))
    return launch_conv_fewout(a, stream);
  if (conv_fwd_fewch_applies(a)) return launch_conv_fwd_fewch(a, stream);
  if (conv_wino_stream_applies(a) || conv_wino_stream_bwd_applies(a)) return launch_conv_wino_stream(a, stream);
  if (conv_wino_applies(a)) return launch_conv_wino(a, stream);
  if (a.Hout > 8) {
    const Conv3x3Pick pick = conv3x3c16_pick(a);
    if (pick.NT == 1 && pick.CC == 8) return launch_3x3<1, 4, 8>(a, stream);
    if (pick.NT == 1 && pick.CC == 4) return launch_3x3<1, 4, 4>(a, stream);
    if (pick.NT == 2 && pick.CC == 4) return launch_3x3<2, 4, 4>(a, stream);
    if (pick.NT == 2 && pick.CC == 16) return launch_3x3<2, 8, 16>(a, stream);
  }
  if (small) {
    if (nt == 1) return launch_t<1, 1>(a, stream);
    if (nt == 2) return launch_t<2, 1>(a, stream);
    return launch_t<3, 1>(a, stream);
  }
  if (nt == 1) return launch_t<1, 2>(a, stream);
  if (nt == 2) return launch_t<2, 2>(a, stream);
  return launch_t<3, 2>(a, stream);
}

}  // namespace dllk
